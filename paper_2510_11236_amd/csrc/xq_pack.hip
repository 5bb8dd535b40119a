// Quantize + bit-pack kernels (prefill pack, ring flush, ring write, debug unpack).
//
// One workgroup quantizes one token group of g tokens of one (layer, sequence, kv head):
// the g x D fp16 tile is staged in LDS once and serves both directions of grouping --
// keys reduce min/max down the token axis per channel, values along the channel axis per
// token (Sec. 4.1: per-channel keys, per-token values).  Scale, zero-point, codes and the
// calibrated metadata follow Eq. 1-2 and Eq. 12 with one correctly rounded fp32 operation
// per step (no fused multiply-add), which is what makes the packed words reproducible.
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

// Eq. 2: nearest level, ties to even, clamped to [0, n].
__device__ __forceinline__ uint32_t code_of(float x, float mn, float s, int n) {
    if (s == 0.0f) return 0u;
    float r = rintf(rounded(__fdiv_rn(rounded(__fsub_rn(x, mn)), s)));
    r = fminf(fmaxf(r, 0.0f), (float)n);
    return (uint32_t)r;
}

template <int D, int G>
__global__ __launch_bounds__(256) void xq_pack_kernel(XqPackArgs a) {
    constexpr int LDW = D / 2 + 1;  // LDS row stride in 32-bit words (one pad word)
    constexpr int NJ = D / G;       // value groups per token
    constexpr int CPL = D / 64;     // value channels per slot
    __shared__ uint32_t tile[G * LDW];
    __shared__ float s_mn[D];  // keys: per channel; values: per (token, channel group) -- G*NJ == D
    __shared__ float s_sc[D];
    // second layer of a pair whose stored codes are merged (Appendix E); unused otherwise
    __shared__ uint32_t tile2[G * LDW];
    __shared__ float s_mn2[D];
    __shared__ float s_sc2[D];

    const int tid = threadIdx.x;
    const int grp = blockIdx.x;
    const int bh = a.bh0 + blockIdx.y;
    const int lz = blockIdx.z;
    const int layer = a.layer0 + lz;
    const XqLayerDesc d = a.layers[layer];
    const int bi = blockIdx.y / a.n_kv_heads, hh = blockIdx.y % a.n_kv_heads;  // source indices are local to the call
    int src_tok0 = a.src_tok0, dst_tok0 = a.dst_tok0;
    if (a.ragged) {  // per-sequence ring flush: only sequences whose ring is full take part
        const int T = a.seq_T[bh / a.n_kv_heads];
        const int Tq = xq_quantized_len(T, G, a.R);
        if (T - Tq != a.R) return;
        src_tok0 = Tq % a.R;
        dst_tok0 = Tq;
    }
    // destination inside the slice that holds the group (the sequence's own, or a page's)
    int dst_tok;
    const int64_t slice = xq_locate(a.pg, bh / a.n_kv_heads, bh % a.n_kv_heads, a.n_kv_heads, dst_tok0 + grp * G, &dst_tok);

    auto half_at = [&](int t, int c) -> float {
        uint32_t w = tile[t * LDW + (c >> 1)];
        return half_bits_to_float((c & 1) ? (w >> 16) : (w & 0xffffu));
    };
    auto half2_at = [&](int t, int c) -> float {
        uint32_t w = tile2[t * LDW + (c >> 1)];
        return half_bits_to_float((c & 1) ? (w >> 16) : (w & 0xffffu));
    };

#pragma unroll 1
    for (int pass = 0; pass < 2; ++pass) {
        const bool is_v = pass == 1;
        const int B = is_v ? d.bv : d.bk;
        const int n = (1 << B) - 1;
        const float c1 = B == 2 ? a.c1_2 : a.c1_1;
        const float c2 = B == 2 ? a.c2_2 : a.c2_1;
        const bool store = is_v ? d.v_store : d.k_store;
        const bool mg = a.merge && (is_v ? d.v_merge : d.k_merge);  // uniform over the workgroup
        const uint32_t lut = B == 2 ? a.lut2 : a.lut1;
        // ---- stage the tile
        const uint16_t *src;
        int64_t s_tok;
        if (a.from_ring) {
            src = (const uint16_t *)(a.arena + (is_v ? d.v_res : d.k_res) + (int64_t)bh * a.st.res) +
                  (int64_t)(src_tok0 + grp * G) * D;
            s_tok = D;
        } else {
            src = (is_v ? a.v_src : a.k_src) + lz * a.s_layer + bi * a.s_batch + hh * a.s_head +
                  (int64_t)(src_tok0 + grp * G) * a.s_tok;
            s_tok = a.s_tok;
        }
        for (int idx = tid; idx < G * (D / 8); idx += 256) {
            int t = idx / (D / 8), v = idx % (D / 8);
            uint4 val = *(const uint4 *)(src + t * s_tok + v * 8);
            uint32_t *row = &tile[t * LDW + v * 4];
            row[0] = val.x;
            row[1] = val.y;
            row[2] = val.z;
            row[3] = val.w;
        }
        if (mg) {  // the same tile of the next layer
            const uint16_t *src2;
            if (a.from_ring) {
                const XqLayerDesc d2 = a.layers[layer + 1];
                src2 = (const uint16_t *)(a.arena + (is_v ? d2.v_res : d2.k_res) + (int64_t)bh * a.st.res) +
                       (int64_t)(src_tok0 + grp * G) * D;
            } else {
                src2 = src + a.s_layer;
            }
            for (int idx = tid; idx < G * (D / 8); idx += 256) {
                int t = idx / (D / 8), v = idx % (D / 8);
                uint4 val = *(const uint4 *)(src2 + t * s_tok + v * 8);
                uint32_t *row = &tile2[t * LDW + v * 4];
                row[0] = val.x;
                row[1] = val.y;
                row[2] = val.z;
                row[3] = val.w;
            }
        }
        __syncthreads();
        // ---- group statistics and metadata
        if (tid < D) {
            float mn, mx;
            if (!is_v) {  // channel tid, over the g tokens
                mn = mx = half_at(0, tid);
                for (int t = 1; t < G; ++t) {
                    float x = half_at(t, tid);
                    mn = fminf(mn, x);
                    mx = fmaxf(mx, x);
                }
            } else {  // token tid / NJ, channel group tid % NJ
                int t = tid / NJ, j = tid % NJ;
                mn = mx = half_at(t, j * G);
                for (int c = 1; c < G; ++c) {
                    float x = half_at(t, j * G + c);
                    mn = fminf(mn, x);
                    mx = fmaxf(mx, x);
                }
            }
            mn += 0.0f;  // a zero minimum or maximum is stored as +0
            mx += 0.0f;
            uint32_t meta;
            float s = group_params(mn, mx, n, c1, c2, &meta);
            s_mn[tid] = mn;
            s_sc[tid] = s;
            uint32_t *mp;
            if (!is_v)
                mp = (uint32_t *)(a.arena + d.k_meta + slice * a.st.k_meta) + (int64_t)(dst_tok / G) * D + tid;
            else
                mp = (uint32_t *)(a.arena + d.v_meta + slice * a.st.v_meta) + (int64_t)dst_tok * NJ + tid;
            *mp = meta;
            if (mg) {  // the next layer's own scale for its own codes (its metadata is written by its workgroup)
                float mn2, mx2;
                if (!is_v) {
                    mn2 = mx2 = half2_at(0, tid);
                    for (int t = 1; t < G; ++t) {
                        float x = half2_at(t, tid);
                        mn2 = fminf(mn2, x);
                        mx2 = fmaxf(mx2, x);
                    }
                } else {
                    int t = tid / NJ, j = tid % NJ;
                    mn2 = mx2 = half2_at(t, j * G);
                    for (int c = 1; c < G; ++c) {
                        float x = half2_at(t, j * G + c);
                        mn2 = fminf(mn2, x);
                        mx2 = fmaxf(mx2, x);
                    }
                }
                mn2 += 0.0f;
                mx2 += 0.0f;
                uint32_t unused;
                s_sc2[tid] = group_params(mn2, mx2, n, c1, c2, &unused);
                s_mn2[tid] = mn2;
            }
        }
        __syncthreads();
        // ---- codes (skipped by a layer that takes its codes from the layer below)
        if (store) {
            const int per = 32 / B;  // codes per word
            if (!is_v) {
                const int W = D / per, CW = W < 4 ? W : 4;
                const int64_t cs = B == 2 ? a.st.k_codes2 : a.st.k_codes1;
                uint32_t *cp = (uint32_t *)(a.arena + d.k_codes + slice * cs);
                for (int idx = tid; idx < G * W; idx += 256) {
                    int sb = idx / (32 * W), ib = idx % (32 * W);
                    int chunk = ib / (32 * CW), tau = (ib / CW) % 32, wc = ib % CW;
                    int wi = chunk * CW + wc, t = sb * 32 + tau;
                    uint32_t word = 0;
                    for (int e = 0; e < per; ++e) {
                        int c = wi * per + e;
                        uint32_t code = code_of(half_at(t, c), s_mn[c], s_sc[c], n);
                        if (mg) code = (lut >> (B * ((n + 1) * code + code_of(half2_at(t, c), s_mn2[c], s_sc2[c], n)))) & n;
                        word |= code << (B * e);
                    }
                    cp[(int64_t)(dst_tok / 32 + sb) * 32 * W + ib] = word;
                }
            } else {
                const int WS = CPL * B;
                const int64_t cs = B == 2 ? a.st.v_codes2 : a.st.v_codes1;
                uint32_t *cp = (uint32_t *)(a.arena + d.v_codes + slice * cs);
                for (int idx = tid; idx < (G / 32) * 64 * WS; idx += 256) {
                    int sb = idx / (64 * WS), ib = idx % (64 * WS);
                    int slot = ib / WS, m = ib % WS;
                    uint32_t word = 0;
                    for (int e2 = 0; e2 < per; ++e2) {
                        int e = m * per + e2;
                        int t = sb * 32 + e / CPL, c = slot * CPL + e % CPL;
                        int gi = t * NJ + c / G;
                        uint32_t code = code_of(half_at(t, c), s_mn[gi], s_sc[gi], n);
                        if (mg) code = (lut >> (B * ((n + 1) * code + code_of(half2_at(t, c), s_mn2[gi], s_sc2[gi], n)))) & n;
                        word |= code << (B * e2);
                    }
                    cp[(int64_t)(dst_tok / 32 + sb) * 64 * WS + ib] = word;
                }
            }
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------
// Wave-per-tile pack kernel for D = 128 (the production shape).  One wave quantizes the keys
// or the values of one token group: lane = channel pair, the g token rows stay in registers.
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
__device__ __forceinline__ uint32_t dpp_or(uint32_t x) {
    return x | (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, false);
}

// MG: the stored codes are merged with the next layer's own codes, whose rows are rows2.
template <int G, int B, bool MG>
__device__ __forceinline__ void pack_keys_wave(const XqPackArgs &a, const XqLayerDesc &d, const uint32_t (&rows)[G],
                                               const uint32_t (&rows2)[MG ? G : 1], int lane, int64_t slice, int dst_tok) {
    constexpr int D = 128;
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
    GroupQ q2a = qa, q2b = qb;  // the next layer's own groups (its metadata is written by its own wave)
    if constexpr (MG) {
        uint32_t pa2 = 0x7c007c00u, pb2 = 0x7c007c00u;
#pragma unroll
        for (int t = 0; t < G; ++t) {
            pa2 = minmax_lo(pa2, rows2[t]);
            pb2 = minmax_hi(pb2, rows2[t]);
        }
        uint32_t unused;
        q2a = group_quant<B>(pair_min(pa2), pair_max(pa2), c1, c2, &unused);
        q2b = group_quant<B>(pair_min(pb2), pair_max(pb2), c1, c2, &unused);
    }
    const uint32_t lut = B == 2 ? a.lut2 : a.lut1;
    // ---- codes: a word holds 32/B channels of one token = LW lanes x (2 channels x B bits)
    constexpr int LW = 16 / B;             // lanes per word
    constexpr int W = D * B / 32;          // words per token row
    constexpr int CW = 4;
    uint32_t *cp = (uint32_t *)(a.arena + d.k_codes + slice * (B == 2 ? a.st.k_codes2 : a.st.k_codes1));
    const int wsel = lane / LW, lsel = lane % LW;
    // batches of LW rows: the OR trees of a batch run side by side, so that no instruction
    // waits on the DPP read-after-write hazard of its own row
#pragma unroll
    for (int t0 = 0; t0 < G; t0 += LW) {
        uint32_t x[LW];
#pragma unroll
        for (int k = 0; k < LW; ++k) {
            uint32_t nib;
            if constexpr (MG) {
                nib = merged_code<B>(sub_hi(rows[t0 + k], qb.nmn), qb, sub_hi(rows2[t0 + k], q2b.nmn), q2b, lut) << B;
                nib |= merged_code<B>(sub_lo(rows[t0 + k], qa.nmn), qa, sub_lo(rows2[t0 + k], q2a.nmn), q2a, lut);
            } else {
                nib = push_code<B>(0u, sub_hi(rows[t0 + k], qb.nmn), qb);
                nib = push_code<B>(nib, sub_lo(rows[t0 + k], qa.nmn), qa);
            }
            x[k] = nib << (2 * B * lsel);
        }
#pragma unroll
        for (int k = 0; k < LW; ++k) x[k] = dpp_or<0xB1>(x[k]);    // lanes ^ 1
#pragma unroll
        for (int k = 0; k < LW; ++k) x[k] = dpp_or<0x4E>(x[k]);    // lanes ^ 2
#pragma unroll
        for (int k = 0; k < LW; ++k) x[k] = dpp_or<0x141>(x[k]);   // mirror inside each 8 lanes
        if (LW == 16) {
#pragma unroll
            for (int k = 0; k < LW; ++k) x[k] = dpp_or<0x140>(x[k]);  // mirror inside the 16-lane row
        }
        uint32_t keep = x[0];
#pragma unroll
        for (int k = 1; k < LW; ++k) keep = (lsel == k) ? x[k] : keep;
        // lane (wsel, lsel) holds word wsel of token t0 + lsel
        const int tok = dst_tok + t0 + lsel;
        __builtin_nontemporal_store(keep, &cp[(int64_t)(tok / 32) * 32 * W + (wsel / CW) * 32 * CW + (tok % 32) * CW + wsel % CW]);
    }
}

template <int G, int B, bool MG>
__device__ __forceinline__ void pack_values_wave(const XqPackArgs &a, const XqLayerDesc &d, const uint32_t (&rows)[G],
                                                 const uint32_t (&rows2)[MG ? G : 1], int lane, int64_t slice, int dst_tok,
                                                 float4 *s_par, float4 *s_par2) {
    constexpr int D = 128, NJ = D / G, LPG = G / 2;  // lanes per channel group
    const int j = lane / LPG, i = lane % LPG;
    const float c1 = B == 2 ? a.c1_2 : a.c1_1, c2 = B == 2 ? a.c2_2 : a.c2_1;
    uint32_t *mp = (uint32_t *)(a.arena + d.v_meta + slice * a.st.v_meta) + (int64_t)dst_tok * NJ;
    // ---- per-token min / max along the g channels of a group: reduce over the LPG lanes, then
    // lane i of the group keeps token (chunk * LPG + i), so each lane owns one group's parameters
#pragma unroll
    for (int c = 0; c < G / LPG; ++c) {
        uint32_t mine = 0;
#pragma unroll
        for (int k = 0; k < LPG; ++k) {
            const int t = c * LPG + k;
            uint32_t p = minmax_hi(minmax_lo(0x7c007c00u, rows[t]), rows[t]);
#pragma unroll
            for (int o = 1; o < LPG; o <<= 1) p = pk_min(p, (uint32_t)__shfl_xor((int)p, o, 64));
            mine = (i == k) ? p : mine;
        }
        uint32_t meta;
        const GroupQ q = group_quant<B>(pair_min(mine), pair_max(mine), c1, c2, &meta);
        const int t = c * LPG + i;
        __builtin_nontemporal_store(meta, &mp[t * NJ + j]);
        s_par[t * NJ + j] = make_float4(q.nmn, q.D1, q.D2, q.D3);
        if constexpr (MG) {  // the next layer's own group of the same token
            uint32_t mine2 = 0;
#pragma unroll
            for (int k = 0; k < LPG; ++k) {
                const int t2 = c * LPG + k;
                uint32_t p = minmax_hi(minmax_lo(0x7c007c00u, rows2[t2]), rows2[t2]);
#pragma unroll
                for (int o = 1; o < LPG; o <<= 1) p = pk_min(p, (uint32_t)__shfl_xor((int)p, o, 64));
                mine2 = (i == k) ? p : mine2;
            }
            uint32_t unused;
            const GroupQ q2 = group_quant<B>(pair_min(mine2), pair_max(mine2), c1, c2, &unused);
            s_par2[t * NJ + j] = make_float4(q2.nmn, q2.D1, q2.D2, q2.D3);
        }
    }
    if (!d.v_store) return;
    const uint32_t lut = B == 2 ? a.lut2 : a.lut1;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // ---- codes: this lane's two channels over TPW tokens fill one word, highest token first
    constexpr int TPW = 16 / B;   // tokens per word
    constexpr int WS = 2 * B;     // words per 32-token block
    uint32_t *cp = (uint32_t *)(a.arena + d.v_codes + slice * (B == 2 ? a.st.v_codes2 : a.st.v_codes1));
#pragma unroll
    for (int blk = 0; blk < G / 32; ++blk) {
        uint32_t words[WS];
#pragma unroll
        for (int m = 0; m < WS; ++m) {
            uint32_t w = 0;
#pragma unroll
            for (int k = TPW - 1; k >= 0; --k) {
                const int t = blk * 32 + m * TPW + k;
                const float4 f = s_par[t * NJ + j];
                GroupQ q;
                q.nmn = f.x;
                q.D1 = f.y;
                q.D2 = f.z;
                q.D3 = f.w;
                if constexpr (MG) {
                    const float4 f2 = s_par2[t * NJ + j];
                    GroupQ q2;
                    q2.nmn = f2.x;
                    q2.D1 = f2.y;
                    q2.D2 = f2.z;
                    q2.D3 = f2.w;
                    w = (w << B) | merged_code<B>(sub_hi(rows[t], q.nmn), q, sub_hi(rows2[t], q2.nmn), q2, lut);
                    w = (w << B) | merged_code<B>(sub_lo(rows[t], q.nmn), q, sub_lo(rows2[t], q2.nmn), q2, lut);
                } else {
                    w = push_code<B>(w, sub_hi(rows[t], q.nmn), q);
                    w = push_code<B>(w, sub_lo(rows[t], q.nmn), q);
                }
            }
            words[m] = w;
        }
        uint32_t *wp = cp + (int64_t)(dst_tok / 32 + blk) * 64 * WS + lane * WS;
        typedef uint32_t u32xw __attribute__((ext_vector_type(WS)));
        u32xw wv;
#pragma unroll
        for (int m = 0; m < WS; ++m) wv[m] = words[m];
        __builtin_nontemporal_store(wv, (u32xw *)wp);
    }
}

// One wave per item, XQ_PACK_WAVES waves per workgroup along grid.x; items 0 .. n_groups - 1 are
// the key groups, n_groups .. 2 n_groups - 1 the value groups (kept apart because workgroups are
// dealt round-robin to the 8 XCDs and the two kinds cost differently); grid.y = sequence * kv head,
// grid.z = layer.
// MG: built for caches whose sharing pairs store merged codes (Appendix E); a wave of the
// pair's first layer then also reads the second layer's rows.
#define XQ_PACK_WAVES 4   // waves (= token groups) per workgroup
template <int G, bool MG = false>
__global__ __launch_bounds__(64 * XQ_PACK_WAVES) void xq_pack_wave_kernel(XqPackArgs a) {
    constexpr int D = 128;
    __shared__ float4 s_par_all[XQ_PACK_WAVES][G * (D / G)];
    __shared__ float4 s_par2_all[XQ_PACK_WAVES][MG ? G * (D / G) : 1];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    float4 *s_par = s_par_all[wave], *s_par2 = s_par2_all[wave];
    const int item = blockIdx.x * XQ_PACK_WAVES + wave;
    if (item >= 2 * a.n_groups) return;
    const bool is_v = item >= a.n_groups;
    const int grp = is_v ? item - a.n_groups : item;
    const int bh = a.bh0 + blockIdx.y, lz = blockIdx.z;
    const XqLayerDesc d = a.layers[a.layer0 + lz];
    const int bi = blockIdx.y / a.n_kv_heads, hh = blockIdx.y % a.n_kv_heads;  // source indices are local to the call
    int src_tok0 = a.src_tok0, dst_tok0 = a.dst_tok0;
    if (a.ragged) {  // per-sequence ring flush: only sequences whose ring is full take part
        const int T = a.seq_T[bh / a.n_kv_heads];
        const int Tq = xq_quantized_len(T, G, a.R);
        if (T - Tq != a.R) return;
        src_tok0 = Tq % a.R;
        dst_tok0 = Tq;
    }
    // destination inside the slice that holds the group (the sequence's own, or a page's)
    int dst_tok;
    const int64_t slice = xq_locate(a.pg, bh / a.n_kv_heads, bh % a.n_kv_heads, a.n_kv_heads, dst_tok0 + grp * G, &dst_tok);
    const uint16_t *src;
    int64_t s_tok;
    if (a.from_ring) {
        src = (const uint16_t *)(a.arena + (is_v ? d.v_res : d.k_res) + (int64_t)bh * a.st.res) +
              (int64_t)(src_tok0 + grp * G) * D;
        s_tok = D;
    } else {
        src = (is_v ? a.v_src : a.k_src) + lz * a.s_layer + bi * a.s_batch + hh * a.s_head +
              (int64_t)(src_tok0 + grp * G) * a.s_tok;
        s_tok = a.s_tok;
    }
    uint32_t rows[G];
#pragma unroll
    for (int t = 0; t < G; ++t) rows[t] = __builtin_nontemporal_load((const uint32_t *)(src + t * s_tok + 2 * lane));
    const uint32_t none[1] = {0};
    if constexpr (MG) {
        if (is_v ? d.v_merge : d.k_merge) {  // uniform over the wave
            const uint16_t *src2;
            if (a.from_ring) {
                const XqLayerDesc d2 = a.layers[a.layer0 + lz + 1];
                src2 = (const uint16_t *)(a.arena + (is_v ? d2.v_res : d2.k_res) + (int64_t)bh * a.st.res) +
                       (int64_t)(src_tok0 + grp * G) * D;
            } else {
                src2 = src + a.s_layer;
            }
            uint32_t rows2[G];
#pragma unroll
            for (int t = 0; t < G; ++t) rows2[t] = __builtin_nontemporal_load((const uint32_t *)(src2 + t * s_tok + 2 * lane));
            if (!is_v) {
                if (d.bk == 2) pack_keys_wave<G, 2, true>(a, d, rows, rows2, lane, slice, dst_tok);
                else pack_keys_wave<G, 1, true>(a, d, rows, rows2, lane, slice, dst_tok);
            } else {
                if (d.bv == 2) pack_values_wave<G, 2, true>(a, d, rows, rows2, lane, slice, dst_tok, s_par, s_par2);
                else pack_values_wave<G, 1, true>(a, d, rows, rows2, lane, slice, dst_tok, s_par, s_par2);
            }
            return;
        }
    }
    if (!is_v) {
        if (d.bk == 2) pack_keys_wave<G, 2, false>(a, d, rows, none, lane, slice, dst_tok);
        else pack_keys_wave<G, 1, false>(a, d, rows, none, lane, slice, dst_tok);
    } else {
        if (d.bv == 2) pack_values_wave<G, 2, false>(a, d, rows, none, lane, slice, dst_tok, s_par, s_par2);
        else pack_values_wave<G, 1, false>(a, d, rows, none, lane, slice, dst_tok, s_par, s_par2);
    }
}

// Copies n_tok tokens into the fp16 rings (token index t -> slot t mod R), keys and values.
__global__ __launch_bounds__(256) void xq_ring_write_kernel(XqRingArgs a) {
    const int bh = a.bh0 + blockIdx.y, lz = blockIdx.z;
    const XqLayerDesc d = a.layers[a.layer0 + lz];
    const int bi = blockIdx.y / a.n_kv_heads, hh = blockIdx.y % a.n_kv_heads;  // source indices are local to the call
    const int dst_tok0 = a.ragged ? a.seq_T[bh / a.n_kv_heads] : a.dst_tok0;
    const int vec = a.D / 8;
    const int total = a.n_tok * vec;
    for (int idx = blockIdx.x * 256 + threadIdx.x; idx < total; idx += gridDim.x * 256) {
        int t = idx / vec, v = idx % vec;
        int64_t so = lz * a.s_layer + bi * a.s_batch + hh * a.s_head + (int64_t)(a.src_tok0 + t) * a.s_tok + v * 8;
        int slot = (dst_tok0 + t) % a.R;
        int64_t doff = (int64_t)bh * a.st.res + ((int64_t)slot * a.D + v * 8) * 2;
        *(uint4 *)(a.arena + d.k_res + doff) = *(const uint4 *)(a.k_src + so);
        *(uint4 *)(a.arena + d.v_res + doff) = *(const uint4 *)(a.v_src + so);
    }
}

// One byte per stored code, [bh][Tq][D], read back through the layout definition.
__global__ __launch_bounds__(256) void xq_unpack_kernel(XqUnpackArgs a) {
    const int64_t total = (int64_t)a.n_bh * a.Tq * a.D;
    const int B = a.B, per = 32 / B, D = a.D;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        int dd = (int)(idx % D);
        int bh = (int)(idx / ((int64_t)D * a.Tq));
        int t;  // token inside the slice that holds it
        const int64_t slice = xq_locate(a.pg, bh / a.n_kv_heads, bh % a.n_kv_heads, a.n_kv_heads, (int)((idx / D) % a.Tq), &t);
        const uint32_t *cp = (const uint32_t *)(a.codes + slice * a.stride);
        uint32_t word;
        int bit;
        if (!a.is_v) {
            int W = D / per, CW = W < 4 ? W : 4;
            int wi = dd / per;
            word = cp[(int64_t)(t / 32) * 32 * W + (wi / CW) * 32 * CW + (t % 32) * CW + wi % CW];
            bit = B * (dd % per);
        } else {
            int CPL = D / 64, WS = CPL * B;
            int e = (t % 32) * CPL + dd % CPL;
            word = cp[(int64_t)(t / 32) * 64 * WS + (dd / CPL) * WS + (e * B) / 32];
            bit = (e * B) % 32;
        }
        a.out[idx] = (uint8_t)((word >> bit) & ((1u << B) - 1u));
    }
}

__global__ void xq_zero_counts_kernel(unsigned long long *c) { c[threadIdx.x] = 0ull; }

// Page-table entries travel in the kernel arguments, so that a table update is an ordinary
// launch in the caller's stream (ordered with the kernels that read the table).
__global__ void xq_page_update_kernel(XqPageUpdateArgs a) {
    for (int i = threadIdx.x; i < a.n; i += blockDim.x) a.table[a.index[i]] = a.page[i];
}

// Histogram of |code_a - code_b| over the packed words of two layers (same layout on both
// sides, so corresponding fields are corresponding elements).  grid.y = (sequence, kv head).
__global__ __launch_bounds__(256) void xq_delta_histogram_kernel(XqDeltaArgs a) {
    __shared__ unsigned long long s_cnt[4];
    if (threadIdx.x < 4) s_cnt[threadIdx.x] = 0ull;
    __syncthreads();
    const int bh = blockIdx.y;
    const int Tq = a.ragged ? a.seq_Tq[bh / a.n_kv_heads] : a.Tq;
    const int64_t n_words = (int64_t)Tq * a.words_per_token;
    const int block_words = 32 * a.words_per_token;  // words of one 32-token block, keys or values
    unsigned int cnt[4] = {0, 0, 0, 0};
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n_words; i += (int64_t)gridDim.x * 256) {
        int tin;
        const int64_t slice = xq_locate(a.pg, bh / a.n_kv_heads, bh % a.n_kv_heads, a.n_kv_heads,
                                        (int)(i / block_words) * 32, &tin);
        const int64_t w = slice * (a.stride / 4) + (int64_t)(tin / 32) * block_words + i % block_words;
        const uint32_t x = ((const uint32_t *)a.codes_a)[w], y = ((const uint32_t *)a.codes_b)[w];
        if (a.B == 1) {
            const int d1 = __builtin_popcount(x ^ y);
            cnt[1] += d1;
            cnt[0] += 32 - d1;
        } else {
#pragma unroll
            for (int f = 0; f < 16; ++f) {
                const int d = (int)((x >> (2 * f)) & 3u) - (int)((y >> (2 * f)) & 3u);
                cnt[d < 0 ? -d : d] += 1;
            }
        }
    }
    for (int k = 0; k < 4; ++k)
        if (cnt[k]) atomicAdd(&s_cnt[k], (unsigned long long)cnt[k]);
    __syncthreads();
    if (threadIdx.x < 4 && s_cnt[threadIdx.x]) atomicAdd(&a.counts[threadIdx.x], s_cnt[threadIdx.x]);
}

}  // namespace

hipError_t xq_launch_delta_histogram(const XqDeltaArgs &a, hipStream_t s) {
    xq_zero_counts_kernel<<<dim3(1), dim3(4), 0, s>>>(a.counts);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    xq_delta_histogram_kernel<<<dim3(64, a.n_bh), dim3(256), 0, s>>>(a);
    return hipGetLastError();
}

hipError_t xq_launch_page_update(const XqPageUpdateArgs &a, hipStream_t s) {
    if (a.n <= 0) return hipSuccess;
    xq_page_update_kernel<<<dim3(1), dim3(256), 0, s>>>(a);
    return hipGetLastError();
}

hipError_t xq_launch_pack(const XqPackArgs &a, int D, int g, int n_layers, hipStream_t s) {
    if (a.n_groups <= 0) return hipSuccess;
    dim3 grid(a.n_groups, a.batch * a.n_kv_heads, n_layers), block(256);
    dim3 wgrid((2 * a.n_groups + XQ_PACK_WAVES - 1) / XQ_PACK_WAVES, a.batch * a.n_kv_heads, n_layers), wblock(64 * XQ_PACK_WAVES);
    if (D == 128 && g == 32 && !a.merge) xq_pack_wave_kernel<32><<<wgrid, wblock, 0, s>>>(a);
    else if (D == 128 && g == 64 && !a.merge) xq_pack_wave_kernel<64><<<wgrid, wblock, 0, s>>>(a);
    else if (D == 128 && g == 32) xq_pack_wave_kernel<32, true><<<wgrid, wblock, 0, s>>>(a);
    else if (D == 128 && g == 64) xq_pack_wave_kernel<64, true><<<wgrid, wblock, 0, s>>>(a);
    else if (D == 64 && g == 32) xq_pack_kernel<64, 32><<<grid, block, 0, s>>>(a);
    else if (D == 64 && g == 64) xq_pack_kernel<64, 64><<<grid, block, 0, s>>>(a);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

hipError_t xq_launch_ring_write(const XqRingArgs &a, int n_layers, hipStream_t s) {
    if (a.n_tok <= 0) return hipSuccess;
    int work = a.n_tok * (a.D / 8);
    dim3 grid((work + 255) / 256, a.batch * a.n_kv_heads, n_layers), block(256);
    xq_ring_write_kernel<<<grid, block, 0, s>>>(a);
    return hipGetLastError();
}

hipError_t xq_launch_unpack(const XqUnpackArgs &a, hipStream_t s) {
    int64_t total = (int64_t)a.n_bh * a.Tq * a.D;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65535) blocks = 65535;
    xq_unpack_kernel<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(a);
    return hipGetLastError();
}
