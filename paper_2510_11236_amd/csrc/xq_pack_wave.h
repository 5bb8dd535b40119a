// Wave-level quantize + bit-pack of token groups: device functions shared by the pack kernel
// (xq_pack.hip) and by the prompt-attention kernel that packs the K/V tiles it already holds
// (xq_prefill.hip).  Arithmetic contract: include/xq.h.
#pragma once
#include "xq_internal.h"

namespace {

__device__ __forceinline__ float half_bits_to_float(uint32_t h) {
    return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}
__device__ __forceinline__ uint32_t float_to_half_bits(float f) {
    return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);  // round to nearest even
}

// Keeps an fp32 intermediate as a value of its own: without it the compiler may merge a
// multiply or add with the following conversion to fp16 (v_fma_mixlo_f16), which rounds once
// instead of twice and changes the stored half in rare near-tie cases.
__device__ __forceinline__ float rounded(float x) {
    asm volatile("" : "+v"(x));
    return x;
}

// Eq. 1 and Eq. 12 for one group: returns s, writes packed (s^ | z^ << 16).
__device__ __forceinline__ float group_params(float mn, float mx, int n, float c1, float c2, uint32_t *meta) {
    float s = (mx == mn) ? 0.0f : rounded(__fdiv_rn(rounded(__fsub_rn(mx, mn)), (float)n));
    float zc = rounded(__fadd_rn(mn, rounded(__fmul_rn(c1, s))));
    float sc = rounded(__fmul_rn(c2, s));
    *meta = float_to_half_bits(sc) | (float_to_half_bits(zc) << 16);
    return s;
}

// ------------------------------------------------------------------------------------------
// One wave quantizes the keys or the values of one token group (head_dim 128) or of two
// neighbouring ones (head_dim 64: one group per half of the wave): lane = channel pair of its
// group, the g token rows stay in registers.  Everything that crosses lanes stays inside 32 lanes
// or fewer, so the two halves never mix; slice, dst_tok (and the row registers) are per lane.
//
// Codes without a division per element.  The contract is c = rint(RN((x - mn) / s)) with ties
// to even.  RN(d / s) is monotone in d, so c = [d >= D1] + [d >= D2] + [d >= D3] where Dk is
// the smallest fp32 d whose rounded quotient reaches 0.5+, 1.5, 2.5+ (the "+" levels are the
// next fp32 above, because an exact 0.5 / 2.5 rounds down to the even code).  RN(d / s)
// reaches a level tau exactly when d / s lies above the midpoint m between tau and the fp32
// below it, i.e. d > m * s.  m has 25 significant bits and s at most 24, so m * s is exact in
// fp64 and is never itself an fp32 number (its odd part has >= 25 bits): no tie can occur at
// the cut, and Dk = the first fp32 above m * s.  Three fp64 multiplies per group replace g
// IEEE divisions, and the stored codes stay bit-identical to the division form.
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

struct GroupQ {
    float nmn;         // -min
    float D1, D2, D3;  // code thresholds on d = x - min
};

__device__ __forceinline__ float first_float_above(double c) {  // c > 0, not an fp32 value
    float f = (float)c;
    if ((double)f < c) f = __uint_as_float(__float_as_uint(f) + 1u);
    return f;
}

template <int B>
__device__ __forceinline__ GroupQ group_quant(float mn, float mx, float c1, float c2, uint32_t *meta) {
    constexpr int n = (1 << B) - 1;
    mn += 0.0f;  // a zero minimum or maximum is stored as +0
    mx += 0.0f;
    const float s = group_params(mn, mx, n, c1, c2, meta);
    GroupQ q;
    q.nmn = -mn;
    if (s == 0.0f) {
        q.D1 = q.D2 = q.D3 = INFINITY;
    } else {
        const double sd = (double)s;
        q.D1 = first_float_above(sd * 0x1.000001p-1);  // midpoint of 0.5 and the next fp32
        if (B == 2) {
            q.D2 = first_float_above(sd * 0x1.7fffffp0);  // midpoint below 1.5
            q.D3 = first_float_above(sd * 0x1.400001p1);  // midpoint of 2.5 and the next fp32
        } else {
            q.D2 = q.D3 = INFINITY;
        }
    }
    return q;
}

// p = (running min, running -max) as an fp16 pair; folds in the low / high half of x.
__device__ __forceinline__ uint32_t minmax_lo(uint32_t p, uint32_t x) {
    asm("v_pk_min_f16 %0, %0, %1 op_sel:[0,0] op_sel_hi:[1,0] neg_hi:[0,1]" : "+v"(p) : "v"(x));
    return p;
}
__device__ __forceinline__ uint32_t minmax_hi(uint32_t p, uint32_t x) {
    asm("v_pk_min_f16 %0, %0, %1 op_sel:[0,1] op_sel_hi:[1,1] neg_hi:[0,1]" : "+v"(p) : "v"(x));
    return p;
}
__device__ __forceinline__ uint32_t pk_min(uint32_t a, uint32_t b) {  // no NaNs here: one instruction
    uint32_t r;
    asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float pair_min(uint32_t p) { return half_bits_to_float(p & 0xffffu); }
__device__ __forceinline__ float pair_max(uint32_t p) { return -half_bits_to_float(p >> 16); }

// d = RN(x + nmn) for the low / high fp16 half of x: the fp32 subtraction of the contract.
__device__ __forceinline__ float sub_lo(uint32_t x, float nmn) {
    float d;
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel_hi:[1,0,0]" : "=v"(d) : "v"(x), "v"(nmn));
    return d;
}
__device__ __forceinline__ float sub_hi(uint32_t x, float nmn) {
    float d;
    asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(x), "v"(nmn));
    return d;
}

// w = (w << B) | code(d), the code counted from compares, carried in through VCC.
template <int B>
__device__ __forceinline__ uint32_t push_code(uint32_t w, float d, const GroupQ &q) {
    if (B == 2) {
        float t;
        asm("v_cmp_ge_f32 vcc, %2, %4\n\t"
            "v_cndmask_b32 %1, %3, %5, vcc\n\t"
            "v_addc_co_u32 %0, vcc, %0, %0, vcc\n\t"
            "v_cmp_ge_f32 vcc, %2, %1\n\t"
            "v_addc_co_u32 %0, vcc, %0, %0, vcc"
            : "+v"(w), "=&v"(t)
            : "v"(d), "v"(q.D1), "v"(q.D2), "v"(q.D3)
            : "vcc");
    } else {
        asm("v_cmp_ge_f32 vcc, %1, %2\n\t"
            "v_addc_co_u32 %0, vcc, %0, %0, vcc"
            : "+v"(w)
            : "v"(d), "v"(q.D1)
            : "vcc");
    }
    return w;
}

// Merged code of a sharing pair (Appendix E): e_m = lut[(e_0, e_1)] from the two layers' own
// codes of one element, d0 / d1 = x - min in each layer's own group.
template <int B>
__device__ __forceinline__ uint32_t merged_code(float d0, const GroupQ &q0, float d1, const GroupQ &q1, uint32_t lut) {
    const uint32_t e = push_code<B>(push_code<B>(0u, d0, q0), d1, q1);  // (e_0 << B) | e_1
    return (lut >> (B * e)) & ((1u << B) - 1u);
}

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_from(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, false);
}

// One step of a transpose between lanes and bit fields: lanes H apart exchange the fields they hold
// for each other.  w holds fields in blocks of S bits; a lane whose index has bit H clear keeps its
// even blocks and receives the partner's even blocks into its odd ones, a lane with the bit set the
// other way round.  p = the partner's w.
template <int S>
__device__ __forceinline__ uint32_t exchange_blocks(uint32_t w, uint32_t p, bool upper) {
    constexpr uint32_t EVEN = S == 16 ? 0x0000ffffu : S == 8 ? 0x00ff00ffu : S == 4 ? 0x0f0f0f0fu : 0x33333333u;
    const uint32_t keep = upper ? ~EVEN : EVEN;
    const uint32_t moved = __builtin_amdgcn_alignbit(p, p, upper ? S : 32 - S);   // rotate right: down by S, or up by S
    return (w & keep) | (moved & ~keep);
}

// LW lanes each hold a word of LW fields of 32 / LW bits, field k of lane l being element (l, k);
// afterwards field l of lane k is that element: lane k holds what the LW lanes had at position k.
// Partners by DPP: lane ^ 8 = rotate the 16-lane row by 8; lane ^ 4 = shift the row up by 4 for the
// lanes of banks 0 and 2, down by 4 for banks 1 and 3; lane ^ 2 and lane ^ 1 = quad permutations.
template <int LW>
__device__ __forceinline__ uint32_t transpose_lanes_fields(uint32_t w, int lsel) {
    constexpr int E = 32 / LW;
    if constexpr (LW == 16) w = exchange_blocks<8 * E>(w, dpp_from<0x128>(w), (lsel & 8) != 0);
    {
        uint32_t p = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)w, 0x104, 0xf, 0x5, false);   // lane + 4
        p = (uint32_t)__builtin_amdgcn_update_dpp((int)p, (int)w, 0x114, 0xf, 0xa, false);          // lane - 4
        w = exchange_blocks<4 * E>(w, p, (lsel & 4) != 0);
    }
    w = exchange_blocks<2 * E>(w, dpp_from<0x4E>(w), (lsel & 2) != 0);
    return exchange_blocks<E>(w, dpp_from<0xB1>(w), (lsel & 1) != 0);
}

// MG: the stored codes are merged with the next layer's own codes, whose rows are rows2; that
// layer's metadata (descriptor d2) is written here as well, so that its rows are read once.
template <int G, int B, bool MG, int D = 128>
__device__ __forceinline__ void pack_keys_wave(const XqPackArgs &a, const XqLayerDesc &d, const uint32_t (&rows)[G],
                                               const uint32_t (&rows2)[MG ? G : 1], int lane, int64_t slice, int dst_tok,
                                               const XqLayerDesc *d2 = nullptr) {
    lane %= D / 2;  // channel pair inside the lane's group
    // ---- per-channel min / max down the g tokens (two channels per lane)
    uint32_t pa = 0x7c007c00u, pb = 0x7c007c00u;  // (+inf, +inf)
#pragma unroll
    for (int t = 0; t < G; ++t) {
        pa = minmax_lo(pa, rows[t]);
        pb = minmax_hi(pb, rows[t]);
    }
    const float c1 = B == 2 ? a.c1_2 : a.c1_1, c2 = B == 2 ? a.c2_2 : a.c2_1;
    uint32_t ma, mb;
    const GroupQ qa = group_quant<B>(pair_min(pa), pair_max(pa), c1, c2, &ma);
    const GroupQ qb = group_quant<B>(pair_min(pb), pair_max(pb), c1, c2, &mb);
    uint32_t *mp = (uint32_t *)(a.arena + d.k_meta + slice * a.st.k_meta) + (int64_t)(dst_tok / G) * D + 2 * lane;
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    u32x2 mab;
    mab.x = ma;
    mab.y = mb;
    __builtin_nontemporal_store(mab, (u32x2 *)mp);  // streamed out once: keep it out of the way of the reads
    if (!d.k_store) return;
    GroupQ q2a = qa, q2b = qb;  // the next layer's own groups
    if constexpr (MG) {
        uint32_t pa2 = 0x7c007c00u, pb2 = 0x7c007c00u;
#pragma unroll
        for (int t = 0; t < G; ++t) {
            pa2 = minmax_lo(pa2, rows2[t]);
            pb2 = minmax_hi(pb2, rows2[t]);
        }
        uint32_t m2a, m2b;
        q2a = group_quant<B>(pair_min(pa2), pair_max(pa2), c1, c2, &m2a);
        q2b = group_quant<B>(pair_min(pb2), pair_max(pb2), c1, c2, &m2b);
        u32x2 m2;
        m2.x = m2a;
        m2.y = m2b;
        uint32_t *mp2 = (uint32_t *)(a.arena + d2->k_meta + slice * a.st.k_meta) + (int64_t)(dst_tok / G) * D + 2 * lane;
        __builtin_nontemporal_store(m2, (u32x2 *)mp2);
    }
    const uint32_t lut = B == 2 ? a.lut2 : a.lut1;
    // ---- codes: a word holds 32/B channels of one token = LW lanes x (2 channels x B bits)
    constexpr int LW = 16 / B;             // lanes per word
    constexpr int W = D * B / 32;          // words per token row
    constexpr int CW = W < 4 ? W : 4;      // words of a row that lie together (a 16-byte chunk when the row has them)
    uint32_t *cp = (uint32_t *)(a.arena + d.k_codes + slice * (B == 2 ? a.st.k_codes2 : a.st.k_codes1));
    const int wsel = lane / LW, lsel = lane % LW;
    // Each lane first fills a word with its own two channels of LW tokens (the compare chains shift
    // the codes in, highest token first, at no extra cost), then the LW lanes of a word transpose
    // lanes against fields: lane lsel ends up with the two-channel fields of all LW lanes for token
    // t0 + lsel, in lane (= channel) order -- the stored word.
#pragma unroll
    for (int t0 = 0; t0 < G; t0 += LW) {
        uint32_t w = 0;
#pragma unroll
        for (int k = LW - 1; k >= 0; --k) {
            if constexpr (MG) {
                w = (w << B) | merged_code<B>(sub_hi(rows[t0 + k], qb.nmn), qb, sub_hi(rows2[t0 + k], q2b.nmn), q2b, lut);
                w = (w << B) | merged_code<B>(sub_lo(rows[t0 + k], qa.nmn), qa, sub_lo(rows2[t0 + k], q2a.nmn), q2a, lut);
            } else {
                w = push_code<B>(w, sub_hi(rows[t0 + k], qb.nmn), qb);
                w = push_code<B>(w, sub_lo(rows[t0 + k], qa.nmn), qa);
            }
        }
        const uint32_t keep = transpose_lanes_fields<LW>(w, lsel);
        // lane (wsel, lsel) holds word wsel of token t0 + lsel
        const int tok = dst_tok + t0 + lsel;
        __builtin_nontemporal_store(keep, &cp[(int64_t)(tok / 32) * 32 * W + (wsel / CW) * 32 * CW + (tok % 32) * CW + wsel % CW]);
    }
}

// (min, -max) of token `first + i` over the LPG lanes of lane i's channel group, from the lanes' own
// (min, -max) of their two channels for tokens first .. first + LPG - 1.  Instead of a full
// exchange per token (LPG log2 LPG shuffles), the lanes halve the set of tokens they are responsible
// for at every step and hand the other half to their partner: LPG - 1 exchanges in all, all but the
// 32-lane step by DPP.  Partners: lane ^ 16, mirror inside 16, mirror inside 8, lane ^ 2, lane ^ 1;
// a lane keeps the tokens whose index has its own bit at that step, so it ends with token i.
template <int G, int LPG>
__device__ __forceinline__ uint32_t token_minmax(const uint32_t (&rows)[G], int first, int i) {
    uint32_t q[16];
    if constexpr (LPG == 32) {
        const bool up = (i & 16) != 0;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            const uint32_t lo = minmax_hi(minmax_lo(0x7c007c00u, rows[first + k]), rows[first + k]);
            const uint32_t hi = minmax_hi(minmax_lo(0x7c007c00u, rows[first + 16 + k]), rows[first + 16 + k]);
            q[k] = pk_min(up ? hi : lo, (uint32_t)__shfl_xor((int)(up ? lo : hi), 16, 64));
        }
    } else {
#pragma unroll
        for (int k = 0; k < 16; ++k) q[k] = minmax_hi(minmax_lo(0x7c007c00u, rows[first + k]), rows[first + k]);
    }
    const bool b3 = (i & 8) != 0, b2 = (i & 4) != 0, b1 = (i & 2) != 0, b0 = (i & 1) != 0;
    uint32_t y[8], z[4], w[2];
#pragma unroll
    for (int k = 0; k < 8; ++k) y[k] = pk_min(b3 ? q[8 + k] : q[k], dpp_from<0x140>(b3 ? q[k] : q[8 + k]));
#pragma unroll
    for (int k = 0; k < 4; ++k) z[k] = pk_min(b2 ? y[4 + k] : y[k], dpp_from<0x141>(b2 ? y[k] : y[4 + k]));
#pragma unroll
    for (int k = 0; k < 2; ++k) w[k] = pk_min(b1 ? z[2 + k] : z[k], dpp_from<0x4E>(b1 ? z[k] : z[2 + k]));
    return pk_min(b0 ? w[1] : w[0], dpp_from<0xB1>(b0 ? w[0] : w[1]));
}

template <int G, int B, bool MG, int D = 128>
__device__ __forceinline__ void pack_values_wave(const XqPackArgs &a, const XqLayerDesc &d, const uint32_t (&rows)[G],
                                                 const uint32_t (&rows2)[MG ? G : 1], int lane, int64_t slice, int dst_tok,
                                                 float4 *s_par, float4 *s_par2, const XqLayerDesc *d2 = nullptr) {
    constexpr int NJ = D / G, LPG = G / 2;  // lanes per channel group
    if constexpr (D == 64) {                // the half wave's own group parameters
        s_par += (lane / 32) * G * NJ;
        s_par2 += MG ? (lane / 32) * G * NJ : 0;
        lane %= 32;
    }
    const int j = lane / LPG, i = lane % LPG;
    const float c1 = B == 2 ? a.c1_2 : a.c1_1, c2 = B == 2 ? a.c2_2 : a.c2_1;
    uint32_t *mp = (uint32_t *)(a.arena + d.v_meta + slice * a.st.v_meta) + (int64_t)dst_tok * NJ;
    // ---- per-token min / max along the g channels of a group: lane i of the group ends up with
    // token (chunk * LPG + i), so each lane owns one group's parameters
#pragma unroll
    for (int c = 0; c < G / LPG; ++c) {
        const uint32_t mine = token_minmax<G, LPG>(rows, c * LPG, i);
        uint32_t meta;
        const GroupQ q = group_quant<B>(pair_min(mine), pair_max(mine), c1, c2, &meta);
        const int t = c * LPG + i;
        __builtin_nontemporal_store(meta, &mp[t * NJ + j]);
        s_par[t * NJ + j] = make_float4(q.nmn, q.D1, q.D2, q.D3);
        if constexpr (MG) {  // the next layer's own group of the same token, and its metadata
            const uint32_t mine2 = token_minmax<G, LPG>(rows2, c * LPG, i);
            uint32_t meta2;
            const GroupQ q2 = group_quant<B>(pair_min(mine2), pair_max(mine2), c1, c2, &meta2);
            uint32_t *mp2 = (uint32_t *)(a.arena + d2->v_meta + slice * a.st.v_meta) + (int64_t)dst_tok * NJ;
            __builtin_nontemporal_store(meta2, &mp2[t * NJ + j]);
            s_par2[t * NJ + j] = make_float4(q2.nmn, q2.D1, q2.D2, q2.D3);
        }
    }
    if (!d.v_store) return;
    const uint32_t lut = B == 2 ? a.lut2 : a.lut1;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // the code of element (token t, low / high channel of the lane), pushed into w
    auto push = [&](uint32_t w, int t, bool hi) {
        const float4 f = s_par[t * NJ + j];
        GroupQ q;
        q.nmn = f.x;
        q.D1 = f.y;
        q.D2 = f.z;
        q.D3 = f.w;
        const float dd = hi ? sub_hi(rows[t], q.nmn) : sub_lo(rows[t], q.nmn);
        if constexpr (MG) {
            const float4 f2 = s_par2[t * NJ + j];
            GroupQ q2;
            q2.nmn = f2.x;
            q2.D1 = f2.y;
            q2.D2 = f2.z;
            q2.D3 = f2.w;
            return (w << B) | merged_code<B>(dd, q, hi ? sub_hi(rows2[t], q2.nmn) : sub_lo(rows2[t], q2.nmn), q2, lut);
        } else {
            return push_code<B>(w, dd, q);
        }
    };
    // ---- codes.  head_dim 128: this lane's two channels over TPW tokens fill one word, highest
    // token first.  head_dim 64: a slot of the layout is one channel, so each of the lane's two
    // channels fills words of its own with 32 / B tokens each; the two slots are neighbours, the
    // lane still stores 2 B words per 32-token block in one piece.
    constexpr int TPW = (D == 128 ? 16 : 32) / B;   // tokens per word
    constexpr int WS = 2 * B;                       // words per lane and 32-token block
    uint32_t *cp = (uint32_t *)(a.arena + d.v_codes + slice * (B == 2 ? a.st.v_codes2 : a.st.v_codes1));
#pragma unroll
    for (int blk = 0; blk < G / 32; ++blk) {
        uint32_t words[WS];
#pragma unroll
        for (int m = 0; m < WS; ++m) {
            uint32_t w = 0;
#pragma unroll
            for (int k = TPW - 1; k >= 0; --k) {
                if constexpr (D == 128) {
                    const int t = blk * 32 + m * TPW + k;
                    w = push(w, t, true);
                    w = push(w, t, false);
                } else {
                    const int t = blk * 32 + (m % B) * TPW + k;   // words 0 .. B - 1: low channel, then the high one
                    w = push(w, t, m >= B);
                }
            }
            words[m] = w;
        }
        uint32_t *wp = cp + (int64_t)(dst_tok / 32 + blk) * (D / 2) * WS + lane * WS;
        typedef uint32_t u32xw __attribute__((ext_vector_type(WS)));
        u32xw wv;
#pragma unroll
        for (int m = 0; m < WS; ++m) wv[m] = words[m];
        __builtin_nontemporal_store(wv, (u32xw *)wp);
    }
}

}  // namespace
