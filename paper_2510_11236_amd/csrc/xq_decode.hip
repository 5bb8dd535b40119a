// Split-K decode attention over the packed cache, gfx950.
//
// Dequantization X^ = X_Q * s^ + z^ (Sec. 3.2 / 3.3.3) never materialises: scale and
// zero-point are folded into the operand that is uniform over a group,
//   keys    score_t = sum_d (q_d s^_{G,d}) c_{t,d} + sum_d q_d z^_{G,d}      (per token group G)
//   values  o_d     = sum_t (p_t s^_{t,j}) c_{t,d} + sum_t p_t z^_{t,j}      (j = channel group of d)
// so the inner loops touch each code once: one AND isolates a pair of codes in the two
// halves of a register, where each half is read as an fp16 subnormal c * 2^(shift-24)
// (the power of two is undone exactly in the uniform operand), and one FMA per code
// (keys: fp32 weight x fp16 code, v_fma_mix) or one dot2 per pair (values: fp16 weights)
// accumulates in fp32.  That is the vector-ALU family; with head_dim 128 the default family hands
// the same masked codes, four at a time, to the 4x4x4 fp16 matrix instruction instead (MM below).
//
// Work split: one workgroup per (packed-token split, sequence, kv head, layer or layer pair),
// plus one per (sequence, kv head, layer) for the fp16 ring, in a 1-D grid.  A workgroup has
// 4 waves; each wave walks tiles of 128 tokens.  In a tile, a 16-lane row owns one 32-token block:
//   key phase    lane = 2 tokens x all channels; the weights q*s^ come from LDS
//   value phase  lane = D/64 channels x all 128 tokens; the weights p*s^ come from LDS
// Every "virtual head" v = (layer in pair) * NREP + (query head in GQA group) has its own
// weights and accumulators and shares the unpacked codes.
#include <type_traits>

#include "xq_internal.h"

#if !defined(XQ_D) || !defined(XQ_G) || !defined(XQ_BK) || !defined(XQ_BV)
#error "compile with -DXQ_D= -DXQ_G= -DXQ_BK= -DXQ_BV= (one translation unit per configuration)"
#endif

namespace {

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));
typedef int int8_v __attribute__((ext_vector_type(8)));
typedef short short2_t __attribute__((ext_vector_type(2)));
typedef float float2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float hbits(uint32_t h) { return (float)__builtin_bit_cast(_Float16, (uint16_t)h); }

__device__ __forceinline__ void wave_lds_fence() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// acc + w * (fp16 in the low / high half of c), fp32 result: one v_fma_mix_f32 each.  Written
// as instructions because the compiler, when several heads share one code register, converts
// the halves to fp32 first and keeps them live, which costs an extra conversion per code and
// hundreds of registers.
__device__ __forceinline__ float fma_mix_lo(float w, uint32_t c, float acc) {
    asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel_hi:[0,1,0]" : "+v"(acc) : "v"(w), "v"(c));
    return acc;
}
__device__ __forceinline__ float fma_mix_hi(float w, uint32_t c, float acc) {
    asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[0,1,0] op_sel_hi:[0,1,0]" : "+v"(acc) : "v"(w), "v"(c));
    return acc;
}

// The 4x4x4 matrix instruction as a four-row dot-product unit: 16 blocks of 4 lanes; in a block,
// lane j supplies column j of B (4 halves) and receives column j of the 4x4 result (one row per
// register); the A rows (4 halves each) come from lane i of block ABID of the lane's group of
// 2^CB blocks, so one register pair holds 2^CB different A matrices.
template <int CB>
__device__ __forceinline__ float4_t mfma_rows(half4_t a, half4_t b, float4_t c, int abid) {
    switch (abid) {
        case 0: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, CB, 0, 0);
        case 1: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, CB, 1, 0);
        case 2: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, CB, 2, 0);
        case 3: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, CB, 3, 0);
    }
    if constexpr (CB == 3) {
        switch (abid) {
            case 4: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, CB, 4, 0);
            case 5: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, CB, 5, 0);
            case 6: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, CB, 6, 0);
            case 7: return __builtin_amdgcn_mfma_f32_4x4x4f16(a, b, c, CB, 7, 0);
        }
    }
    return c;
}
__device__ __forceinline__ half4_t codes4(uint32_t lo, uint32_t hi) {
    uint2_t u = {lo, hi};
    return __builtin_bit_cast(half4_t, u);
}
// KX key path: v_mfma_f32_16x16x128_f8f6f4 with the weights as A (fp8 e4m3, rows) and the codes
// as B (fp4 e2m1, columns = 16 tokens).  A 2-bit code in the low bits of a nibble IS the fp4
// number c/2 (patterns 0000, 0001, 0010, 0011 = 0, 0.5, 1, 1.5), so one AND isolates eight codes.
// Operand layout of the instruction (found by one-hot probes on the device): lane l supplies row
// (A) / column (B) l % 16; with q = l / 16, B's nibble e holds k = 32 q + e, and A's byte e holds
// k = 16 q + e (e < 16) or 64 + 16 q + e - 16 (e >= 16); C: lane l, register x = row 4 (l / 16) + x
// of column l % 16.
__device__ __forceinline__ float4_t mfma_fp8_fp4(int8_v a, int8_v b, float4_t c) {
    return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0 /* A: fp8 e4m3 */, 4 /* B: fp4 */, 0, 0, 0, 0);
}
// fp8(x / scale), fp8(y / scale) into the low or high half of a dword (scale a power of two; no
// saturation: |x / scale| must stay below 464), and back: fp8 * scale.
template <bool HI>
__device__ __forceinline__ uint32_t cvt_fp8x2(uint32_t old, float x, float y, float scale) {
    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(__builtin_bit_cast(short2_t, old), x, y, scale, HI));
}
template <bool HI>
__device__ __forceinline__ float2_t fp8x2_back(uint32_t v, float scale) {
    return __builtin_amdgcn_cvt_scalef32_pk_f32_fp8((int)v, scale, HI);
}

template <int W>
__device__ __forceinline__ uint32_t group_umax(uint32_t v) {  // max over aligned groups of W lanes
#pragma unroll
    for (int o = W / 2; o >= 1; o >>= 1) v = max(v, (uint32_t)__shfl_xor((int)v, o, 64));
    return v;
}

// Reductions over the 16 lanes of a DPP row without the LDS crossbar: lane ^ 1, lane ^ 2 inside the
// quad, then the mirrored half row (the other quad of the 8) and the mirrored row (the other half).
__device__ __forceinline__ float row16_sum(float v) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xf, 0xf, true));   // quad_perm [1,0,3,2]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xf, 0xf, true));   // quad_perm [2,3,0,1]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xf, 0xf, true));  // row_half_mirror
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xf, 0xf, true));  // row_mirror
    return v;
}
__device__ __forceinline__ uint32_t row16_umax(uint32_t v) {
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xf, 0xf, true));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xf, 0xf, true));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xf, 0xf, true));
    v = max(v, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xf, 0xf, true));
    return v;
}

template <int W>
__device__ __forceinline__ float group_sum(float v) {  // sum over aligned groups of W lanes
#pragma unroll
    for (int o = W / 2; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Global loads.  NT = streaming (non-temporal): for bytes that one workgroup uses once per step,
// which is everything except codes that a second layer's workgroups read again from L2.
template <int N, bool NT = true>
struct VecLoad;
template <bool NT>
struct VecLoad<1, NT> {
    static __device__ __forceinline__ void ld(const uint32_t *p, uint32_t *o) { o[0] = NT ? __builtin_nontemporal_load(p) : *p; }
};
template <bool NT>
struct VecLoad<2, NT> {
    typedef uint32_t V __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ void ld(const uint32_t *p, uint32_t *o) {
        V v = NT ? __builtin_nontemporal_load((const V *)p) : *(const V *)p;
        o[0] = v.x;
        o[1] = v.y;
    }
};
template <bool NT>
struct VecLoad<4, NT> {
    typedef uint32_t V __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ void ld(const uint32_t *p, uint32_t *o) {
        V v = NT ? __builtin_nontemporal_load((const V *)p) : *(const V *)p;
        o[0] = v.x;
        o[1] = v.y;
        o[2] = v.z;
        o[3] = v.w;
    }
};
template <bool NT>
struct VecLoad<8, NT> {
    static __device__ __forceinline__ void ld(const uint32_t *p, uint32_t *o) {
        VecLoad<4, NT>::ld(p, o);
        VecLoad<4, NT>::ld(p + 4, o + 4);
    }
};

// 2^x for x <= 0 (softmax weights): the bare v_exp_f32.  Results below the fp32 normal range
// come out as 0, which is what a weight of 2^-126 may be.
__device__ __forceinline__ float exp2_le0(float x) { return __builtin_amdgcn_exp2f(x); }

// NLAY = 2: the two layers of a sharing pair (one key and one value code tensor, read by the
// first layer's descriptor) are served by one workgroup.
//
// MM = true (D = 128): the multiply-adds go through the 4x4x4 fp16 matrix instruction, used as a
// four-row dot-product unit whose rows are (virtual head, half of the weight) pairs.  The lane
// still owns its tokens (keys) or channels (values): the codes it isolated are its column of B,
// four at a time, and the weights are the rows of A, which every block of the lane's token group
// (keys) or channel group (values) takes from one block of a register pair by broadcast.  Key
// weights are split into an fp16 high and low part (two rows) after a per-group power-of-two
// scaling, which keeps ~22 bits of them for any input; value weights are the same fp16 numbers
// as in the plain path.
// (Held to 128 registers, 4 waves per SIMD, where that costs no spill: the one- and two-head matrix
// kernels and the four-head one at g = 64 unless keys and values are both 2-bit; +2 to 5 %.  The
// others spill when squeezed and keep their 3 or 2 waves.)
template <int D, int G, int BK, int BV, int NREP, int NLAY, bool REUSE = false, bool MM = false, bool KX = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(
    MM && !KX && (NREP * NLAY <= 2 || (NREP == 4 && NLAY == 1 && G == 64 && BK + BV < 4)) ? 4 : 1, 8)))
void xq_decode_kernel(XqDecodeArgs a) {
    static_assert(!KX || (MM && BK == 2 && D == 128 && NREP * NLAY >= 4),
                  "the fp8 x fp4 key path: matrix family, 2-bit keys, head_dim 128, at least four virtual heads");
    constexpr int NV = NREP * NLAY;       // virtual heads
    constexpr int CPL = D / 64;           // value channels per lane
    constexpr int NJ = D / G;             // value groups per token
    constexpr int NGT = XQ_TILE_TOKENS / G;  // key groups per tile
    constexpr int LPG = 64 / NGT;         // lanes preparing one key group
    constexpr int CPP = D / LPG;          // channels per lane in the key-weight prep
    constexpr int WK = D * BK / 32;       // words per key row
    constexpr int CWK = WK < 4 ? WK : 4;  // words per chunk
    constexpr int NCH = WK / CWK;
    constexpr int PERK = 32 / BK;         // key codes per word
    constexpr int HALFK = PERK / 2;       // ... per 16-bit half
    constexpr int BYTEK = 8 / BK;         // ... per byte
    constexpr int WS = CPL * BV;          // value words per slot per block
    constexpr int PERV = 32 / BV;
    constexpr int TPW = PERV / CPL;       // tokens per value word
    constexpr uint32_t MASKK = ((1u << BK) - 1u) * 0x00010001u;
    constexpr uint32_t MASKV = ((1u << BV) - 1u) * 0x00010001u;
    static_assert(CPP >= 2 && CPP <= 8, "prep width");
    constexpr int CPB = BYTEK / 4;        // chunks of 4 code positions per byte (keys)
    // matrix path: blocks of 4 lanes per token group = per value channel group (D = tile = 128)
    constexpr int NB = 16 / NGT;
    constexpr int CBSZ = NB == 8 ? 3 : 2;
    constexpr int NKS = (2 * NV + 3) / 4;  // sets of 4 key rows (head, weight half)
    constexpr int NVS = (NV + 3) / 4;      // sets of 4 value rows (head)
    constexpr int AREG = 32 / NB;          // register pairs that hold the 32 A matrices of a row set
    constexpr int NPL = CPP / 4;           // key A matrices one lane prepares
    constexpr int QPW = TPW / 4;           // token quads per value word
    static_assert(!MM || (D == 128 && (NB == 8 || NB == 4)), "matrix path shape");

    // per wave: key weights q * s^ (pre-scaled) and value weights p * s^ (pre-scaled, pair order);
    // the cross-wave combine at the end reuses the key-weight space
    // (rows padded so that the 4 rows of a wave, which read different groups, hit different banks)
    typedef float KwT[NV][NGT][D + 4];
    typedef _Float16 KaT[NKS][NGT][32][4][4];  // matrix path: [row set][group][A matrix][row][k]
    // fp8 x fp4 key path: [group][row = 4 * virtual head + term][128 bytes in the instruction's A order],
    // rows padded to 144 bytes so that the 16 rows a quarter wave reads start in different banks
    constexpr int KXROW = 36;
    typedef uint32_t KxT[NGT][4 * NV][KXROW];
    // (value-weight rows: padded by 8 halves against bank conflicts of the vector path's 16-byte
    // reads; the matrix path reads 8 bytes per lane from a few broadcast addresses and goes without,
    // which is what lets three workgroups of the four-head g = 32 kernel share a CU's LDS)
    typedef _Float16 VwT[NV][4][NJ][32 + (MM ? 0 : 8)];
    typedef float PartT[NV][D + 2];
    constexpr int KW_BYTES = 4 * (int)(KX ? sizeof(KxT) : MM ? sizeof(KaT) : sizeof(KwT)), PART_BYTES = 4 * (int)sizeof(PartT);
    constexpr int KP_BYTES = KW_BYTES > PART_BYTES ? KW_BYTES : PART_BYTES;
    // with several heads the scaled queries live in LDS rather than in 8 registers per head
    constexpr bool Q_LDS = NV >= 2 || MM;
    typedef float QT[NV][D];
    __shared__ __attribute__((aligned(16))) char s_raw[KP_BYTES + 4 * sizeof(VwT) + (Q_LDS ? sizeof(QT) : 0)];
    KwT *s_kw = (KwT *)s_raw;
    KaT *s_ka = (KaT *)s_raw;
    KxT *s_kx = (KxT *)s_raw;
    VwT *s_vw = (VwT *)(s_raw + KP_BYTES);
    PartT *s_part = (PartT *)s_raw;
    QT &s_q = *(QT *)(s_raw + KP_BYTES + 4 * sizeof(VwT));

    // the wave index as a scalar: everything derived from the tile number then lives in SGPRs
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    // 1-D grid, XCD-aware: workgroups go round-robin over the 8 XCDs by linear id, so the
    // (equal-sized) packed-token workgroups come first and the small ring workgroups last;
    // interleaving the two kinds would hand some XCDs only ring work.
    const int nbh = a.batch * a.n_kv_heads;
    const int n_main = a.n_splits * nbh * (int)a.n_launch_z;
    int split, bh, lz;
    if (REUSE && a.pair_order && (int)blockIdx.x < n_main) {
        // The G layers of a sharing group (G = a.pair_order; a pair when 2) read the same code
        // words: their workgroups for one (split, sequence, kv head) get ids 8 apart -- the same
        // XCD, dispatched at almost the same time -- so that the later readers find the words in
        // that XCD's L2.  Ids come in chunks of 8 G: eight items of the group's first layer, then
        // the same eight of its second, ...
        const int G_ = a.pair_order, n_items = n_main / G_, full = (n_items / 8) * 8, id = blockIdx.x;
        int item, member;
        if (id < G_ * full) {
            member = (id % (8 * G_)) / 8;
            item = (id / (8 * G_)) * 8 + id % 8;
        } else {
            const int rem = n_items - full, id2 = id - G_ * full;
            member = id2 / rem;
            item = full + id2 % rem;
        }
        split = item % a.n_splits;
        const int rest = item / a.n_splits;
        bh = rest % nbh;
        lz = G_ * (rest / nbh) + member;
    } else if ((int)blockIdx.x < n_main) {
        split = blockIdx.x % a.n_splits;
        const int rest = blockIdx.x / a.n_splits;
        bh = rest % nbh;
        lz = rest / nbh;
    } else {
        const int rid = blockIdx.x - n_main;
        split = a.n_splits;
        bh = rid % nbh;
        lz = rid / nbh;
    }
    const int layer = a.layer0 + lz * NLAY;
    const int bi = bh / a.n_kv_heads, hkv = bh % a.n_kv_heads;
    const int row = lane >> 4, r16 = lane & 15;
    // tokens this sequence holds (per sequence when the batch is ragged)
    const int seqT = a.ragged ? a.seq_T[bi] : a.T;
    const int seqTq = a.ragged ? xq_quantized_len(seqT, a.group, a.R) : a.Tq;
    const int n_blocks = seqTq / 32;

    XqLayerDesc dsc[NLAY];
#pragma unroll
    for (int y = 0; y < NLAY; ++y) dsc[y] = a.layers[layer + y];

    auto qptr = [&](int v) -> const uint16_t * {  // query of virtual head v
        int y = v / NREP, n = v % NREP;
        return a.q + (((int64_t)(lz * NLAY + y) * a.batch + bi) * a.n_q_heads + hkv * a.rep + a.q_head0 + n) * D;
    };

    float m_run[NV], l_run[NV];
    float accv[NV][CPL];
    float zacc[NV][NJ];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        m_run[v] = -INFINITY;
        l_run[v] = 0.f;
#pragma unroll
        for (int c = 0; c < CPL; ++c) accv[v][c] = 0.f;
#pragma unroll
        for (int j = 0; j < NJ; ++j) zacc[v][j] = 0.f;
    }

    if (split < a.n_splits) {
        // ------------------------------------------------------------ packed tokens
        const int gi = lane / LPG, li = lane % LPG;  // key-weight prep role
        // matrix path: value accumulators [row set][channel] x 4 heads; the A matrices this lane
        // prepares (first channel, 2^-bit of their two code positions); per head the exponent e of
        // the largest |q| (the query table holds q 2^(14 - e)) and 2^(e - 14)
        float4_t accm[MM ? NVS : 1][CPL];
        int kch[MM ? NPL : 1];
        float kpw[MM ? NPL : 1][2];
        int eq[MM ? NV : 1];
        float qsc[MM ? NV : 1];
        // fp8 x fp4 key path, preparation role: an 8-channel span of the lane's group; when a group has
        // 32 lanes, the two lanes of a span split the query heads of each layer between them
        constexpr int HP = LPG / 16;                       // lanes per span
        constexpr int NPH = NREP >= HP ? NREP / HP : 1;    // query heads of a layer that one lane prepares
        constexpr int QE = KX ? 8 : 14;                    // the query table holds q 2^(QE - e): weights below 2^QE
        const int span = li % 16, hp = li / 16;
        if constexpr (MM) {
#pragma unroll
            for (int x = 0; x < NVS; ++x)
#pragma unroll
                for (int c = 0; c < CPL; ++c) accm[x][c] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int e = 0; e < (KX ? 0 : NPL); ++e) {
                const int n = li * NPL + e, ci = n / 2, p0 = 2 * (n % 2), p4 = (ci % CPB) * 4;
                kch[e] = (ci / (2 * CPB)) * PERK + ((ci / CPB) % 2) * BYTEK + p4 + p0;
                kpw[e][0] = __builtin_ldexpf(1.0f, -BK * (p4 + p0));
                kpw[e][1] = __builtin_ldexpf(1.0f, -BK * (p4 + p0 + 1));
            }
        }
        float qz[Q_LDS ? 1 : NV][CPP];  // q * sm_scale * log2(e) for the channels this lane prepares
        float pw[CPP];      // the code of channel c arrives as c * 2^((BK*c) mod 8 - 24); undo it in the weight
#pragma unroll
        for (int k = 0; k < CPP; ++k) pw[k] = __builtin_ldexpf(1.0f, 24 - ((BK * (li * CPP + k)) & 7));
        // with few heads a second, pre-shifted copy of q saves a multiply per weight
        constexpr bool QK_COPY = NV == 1;
        float qk[QK_COPY ? NV : 1][CPP];
        // Every workgroup starts at a different tile of its range (and wraps around): slices lie
        // at large power-of-two strides, so workgroups marching in step from tile 0 would all
        // hit the same memory channels at once.  Softmax accumulation does not care about order.
        const int tile0 = split * a.tiles_per_split;
        const int n_tiles = max(min(tile0 + a.tiles_per_split, (n_blocks + 3) / 4) - tile0, 0);  // 0: a shorter sequence
        // (the layers of a group that run side by side start at the same tile: they read the same codes)
        const int lrot = (REUSE && a.pair_order) ? lz / a.pair_order : lz;
        const int rot = n_tiles > 0 ? (int)((bh * 37u + lrot * 11u) % (unsigned)n_tiles) : 0;
        // Register-resident inputs of a tile: this lane's two key rows (tokens r16 and r16 + 16 of
        // its block), the value codes of the tile for its channels, the value metadata of its two
        // tokens, and (matrix path) the key metadata of the A matrices it prepares, in their k order.
        // The plain path loads them inside the tile's own iteration.  The matrix path spends less
        // time per tile and keeps a tile's worth of loads in flight instead: each set is reloaded
        // for the wave's next tile as soon as the current tile has consumed it.
        // (fp8 x fp4 key path: kc[m] = the two words of token 16 m + lane % 16 that hold channels
        // 32 (lane / 16) .. + 31; kmeta = scale | zero of the 8 channels of the lane's span)
        uint32_t kc[KX ? 8 : 2][KX ? 2 : WK];
        uint32_t vc[4][WS];
        uint32_t vm[NLAY][2][NJ];
        uint32_t kmeta[MM ? NLAY : 1][KX ? 2 : (MM ? NPL : 1)][4];
        struct TileAt {
            int tile, tin;   // tile number; index of its first token inside the slice
            int64_t slice;   // where its 128 tokens are stored: the sequence's own slice, or a page's
        };
        auto tile_at = [&](int pos) {  // pos: position inside the split, rotation applied
            TileAt t;
            t.tile = tile0 + pos;
            t.slice = xq_locate(a.pg, bi, hkv, a.n_kv_heads, t.tile * XQ_TILE_TOKENS, &t.tin);
            return t;
        };
        auto load_kmeta = [&](const TileAt &t) {
            if constexpr (KX) {
                // (a key group past the sequence's last one reads the tile's last valid group -- see load_kcodes)
                const int gic = min(gi, (min(seqTq - t.tile * XQ_TILE_TOKENS, XQ_TILE_TOKENS) + G - 1) / G - 1);
#pragma unroll
                for (int y = 0; y < NLAY; ++y) {
                    const uint32_t *mp = (const uint32_t *)(a.arena + dsc[y].k_meta + t.slice * a.st.k_meta) +
                                         (int64_t)(t.tin / G + gic) * D + 8 * span;
                    VecLoad<8>::ld(mp, &kmeta[y][0][0]);
                }
            } else if constexpr (MM) {
                const bool g_ok = (t.tile * NGT + gi) * G < seqTq;
#pragma unroll
                for (int y = 0; y < NLAY; ++y)
#pragma unroll
                    for (int e = 0; e < NPL; ++e) {
                        const uint32_t *mp = (const uint32_t *)(a.arena + dsc[y].k_meta + t.slice * a.st.k_meta) +
                                             (int64_t)(t.tin / G + gi) * D + kch[e];
                        uint32_t t0[2] = {0, 0}, t1[2] = {0, 0};
                        if (g_ok) {
                            VecLoad<2>::ld(mp, t0);
                            VecLoad<2>::ld(mp + HALFK, t1);
                        }
                        kmeta[y][e][0] = t0[0];
                        kmeta[y][e][2] = t0[1];
                        kmeta[y][e][1] = t1[0];
                        kmeta[y][e][3] = t1[1];
                    }
            }
        };
        // In the kernels with the fp8 x fp4 key phase, blocks of a tile past the sequence's last one are
        // read from the tile's last valid block instead of being skipped: their scores are masked and
        // their softmax weights are zero, and a load that is always issued keeps the count of loads in
        // flight the same on every path, which is what lets the waits in the loop name a count (a load
        // that may be skipped forces the next wait to be a wait for all).  The other kernels skip and zero.
        auto load_kcodes = [&](const TileAt &t) {
            if constexpr (KX) {
                // column block m of the tile = tokens 16 m .. 16 m + 15; this lane: token r16 of it,
                // row words 2 (lane / 16), + 1 = half of 16-byte chunk (lane / 32) of the row
                const uint32_t *cp = (const uint32_t *)(a.arena + dsc[0].k_codes + t.slice * a.st.k_codes2) +
                                     (int64_t)(t.tin / 32) * 32 * WK + (row / 2) * 32 * CWK + r16 * CWK + 2 * (row % 2);
                const int last = min(n_blocks - t.tile * 4, 4) - 1;  // >= 0: the tile holds at least one block
#pragma unroll
                for (int m = 0; m < 8; ++m) VecLoad<2, !REUSE>::ld(cp + min(m / 2, last) * 32 * WK + (m % 2) * 16 * CWK, kc[m]);
            } else {
                const bool row_ok = t.tile * 4 + row < n_blocks;
                const uint32_t *cp = (const uint32_t *)(a.arena + dsc[0].k_codes +
                                                        t.slice * (BK == 2 ? a.st.k_codes2 : a.st.k_codes1)) +
                                     (int64_t)(t.tin / 32 + row) * 32 * WK;
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int ch = 0; ch < NCH; ++ch) {
                        if (row_ok) VecLoad<CWK, !REUSE>::ld(cp + ch * 32 * CWK + (r16 + 16 * s) * CWK, &kc[s][ch * CWK]);
                        else {
#pragma unroll
                            for (int w = 0; w < CWK; ++w) kc[s][ch * CWK + w] = 0;
                        }
                    }
            }
        };
        auto load_values = [&](const TileAt &t) {
            const int last = min(n_blocks - t.tile * 4, 4) - 1;
            const bool row_ok = KX || row <= last;
            const int rowc = KX ? min(row, last) : row;
            const uint32_t *cp = (const uint32_t *)(a.arena + dsc[0].v_codes +
                                                    t.slice * (BV == 2 ? a.st.v_codes2 : a.st.v_codes1));
#pragma unroll
            for (int kb = 0; kb < 4; ++kb) {
                if constexpr (KX) {
                    VecLoad<WS, !REUSE>::ld(cp + (int64_t)(t.tin / 32 + min(kb, last)) * 64 * WS + lane * WS, vc[kb]);
                } else {
                    if (kb <= last) VecLoad<WS, !REUSE>::ld(cp + (int64_t)(t.tin / 32 + kb) * 64 * WS + lane * WS, vc[kb]);
                    else {
#pragma unroll
                        for (int w = 0; w < WS; ++w) vc[kb][w] = 0;
                    }
                }
            }
#pragma unroll
            for (int y = 0; y < NLAY; ++y)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const uint32_t *mp = (const uint32_t *)(a.arena + dsc[y].v_meta + t.slice * a.st.v_meta) +
                                         ((int64_t)(t.tin / 32 + rowc) * 32 + r16 + 16 * s) * NJ;
                    if (row_ok) VecLoad<NJ>::ld(mp, vm[y][s]);
                    else {
#pragma unroll
                        for (int j = 0; j < NJ; ++j) vm[y][s][j] = 0;
                    }
                }
        };
        // (two heads at g = 32: the 16 registers of key metadata are loaded at the top of their own
        // tile instead, which lets the kernel fit 128 registers, 4 waves per SIMD: +2.5 %)
        constexpr bool PIPE_KMETA = !(NV == 2 && G == 32);
        int pos = n_tiles > 0 ? (wave + rot) % n_tiles : 0;  // advances by 4 and wraps; the wave's tiles are it = wave, wave + 4, ...
        if constexpr (MM) {
            if (wave < n_tiles) {
                const TileAt t = tile_at(pos);
                if constexpr (PIPE_KMETA) load_kmeta(t);
                load_kcodes(t);
                load_values(t);
            }
        }
        // ---- the queries (after the first tile's loads are under way: one memory latency, not two,
        // before the first tile can start -- a one-layer call is little more than that latency)
        if constexpr (MM) {
            // scaled queries in the order the A matrices take their channels: matrix n, element k
            for (int idx = tid; idx < NV * D; idx += 256) {
                const int v = idx / D, pos = idx % D, n = pos / 4, k = pos % 4;
                const int ci = n / 2, p = 2 * (n % 2) + k / 2;
                const int ch = KX ? pos  // (the fp8 x fp4 path reads its channels in natural order)
                                  : (ci / (2 * CPB)) * PERK + ((ci / CPB) % 2) * BYTEK + (ci % CPB) * 4 + p + (k % 2) * HALFK;
                s_q[v][pos] = hbits(qptr(v)[ch]) * a.scale_log2e;
            }
            __syncthreads();
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const float mx = wave_max(fmaxf(fabsf(s_q[v][lane]), fabsf(s_q[v][lane + 64])));
                int e = (int)((__float_as_uint(mx) >> 23) & 0xffu) - 126;  // 2^e > |q| of every channel
                e = __builtin_amdgcn_readfirstlane(min(max(e, -40), 60));
                eq[v] = e;
                qsc[v] = __uint_as_float((uint32_t)(127 - QE + e) << 23);  // 2^(e - QE)
            }
            // the table keeps q 2^(14 - e): weights come out in fp16 range without a multiply per
            // channel, and the zero-point sum is scaled back once per head
            __syncthreads();
            for (int idx = tid; idx < NV * D; idx += 256) {
                const int v = idx / D;
                float f = 1.0f;
#pragma unroll
                for (int u = 0; u < NV; ++u) f = (u == v) ? __uint_as_float((uint32_t)(127 + QE - eq[u]) << 23) : f;
                s_q[v][idx % D] *= f;
            }
            __syncthreads();
        } else if constexpr (Q_LDS) {
            for (int idx = tid; idx < NV * D; idx += 256) s_q[idx / D][idx % D] = hbits(qptr(idx / D)[idx % D]) * a.scale_log2e;
            __syncthreads();
        } else {
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const uint16_t *qp = qptr(v);
#pragma unroll
                for (int k = 0; k < CPP; ++k) {
                    qz[v][k] = hbits(qp[li * CPP + k]) * a.scale_log2e;
                    if constexpr (QK_COPY) qk[v][k] = qz[v][k] * pw[k];
                }
            }
        }
        // One tile of the wave.  more: the wave has a further tile, whose register sets are reloaded
        // inside this one.  The translation units that build the kernels with the fp8 x fp4 key phase
        // (XQ_KX_TU) make that a compile-time flag and run the wave's last tile in a second copy of the
        // body without those loads, so that in the steady-state copy every load is issued on every path
        // (see load_kcodes); the other kernels keep the plain loop.
#ifdef XQ_KX_TU
        auto one_tile = [&](auto more_flag) __attribute__((always_inline)) {
            constexpr bool more = decltype(more_flag)::value;
#else
        for (int it = wave; it < n_tiles; it += 4) {
            const bool more = it + 4 < n_tiles;
#endif
            const TileAt cur = tile_at(pos);
            pos = pos + 4 >= n_tiles ? pos + 4 - n_tiles : pos + 4;  // (a further tile means n_tiles > 4: one subtraction wraps)
            const TileAt nxt = (MM && more) ? tile_at(pos) : cur;
            const int tile = cur.tile, tin = cur.tin;
            const int64_t slice = cur.slice;
            const bool row_ok = tile * 4 + row < n_blocks;
            // ---- key weights for the tile's groups -> LDS
            float zs[NV];
            float fac[MM ? NV : 1];  // matrix path: score = (sum of the head's two rows) * fac + zs
            if constexpr (KX) {
                if constexpr (!PIPE_KMETA) load_kmeta(cur);
                // where this lane's span goes in a row of the A table: 16-channel span s16 sits in the
                // quarter s16 % 4 of the row's lanes, first or second 16 bytes by s16 / 4; its even
                // channels fill two dwords (by half of the span), its odd channels the two after them
                const int off_e = (span / 2 % 4) * 8 + (span / 8) * 4 + span % 2;  // dword of the even channels; odd: + 2
#pragma unroll
                for (int y = 0; y < NLAY; ++y) {
                    uint32_t hm = 0;
#pragma unroll
                    for (int k = 0; k < 8; ++k) hm = max(hm, kmeta[y][k / 4][k % 4] & 0x7fffu);
                    hm = row16_umax(hm);
                    if constexpr (LPG == 32) hm = max(hm, (uint32_t)__shfl_xor((int)hm, 16, 64));
                    const int es = max((int)(hm >> 10), 1) - 14;  // 2^es > every scale of the group
#pragma unroll
                    for (int x = 0; x < NPH; ++x) {
                        const int n = NREP >= HP ? hp + HP * x : 0, v = y * NREP + n;  // (runtime when HP = 2)
                        const float4 qa = *(const float4 *)&s_q[v][8 * span], qb = *(const float4 *)&s_q[v][8 * span + 4];
                        const float qv[8] = {qa.x, qa.y, qa.z, qa.w, qb.x, qb.y, qb.z, qb.w};
                        float w[8], zp = 0.f;
#pragma unroll
                        for (int k = 0; k < 8; ++k) {
                            const uint32_t mt = kmeta[y][k / 4][k % 4];
                            w[k] = qv[k] * hbits(mt & 0xffffu);  // q 2^(QE - eq) * scale: |w| < 2^(QE + es)
                            zp = fmaf(qv[k], hbits(mt >> 16), zp);
                        }
                        // w 2^-es = t0 + t1 / 16 + t2 / 256 + t3 / 4096 (+ at most 2^-16 |w|), every t an fp8
                        // number below 2^8: four rows of A.  The conversions divide by their scale operand,
                        // the residuals are exact in fp32.
                        uint32_t *dst = &s_kx[wave][gi][4 * v][off_e];
                        uint32_t ev = 0, od = 0;  // (both halves are overwritten below)
#pragma unroll
                        for (int tau = 0; tau < 4; ++tau) {
                            const float sc = __uint_as_float((uint32_t)(127 + es - 4 * tau) << 23);  // 2^es 16^-tau
                            ev = cvt_fp8x2<false>(ev, w[0], w[2], sc);
                            od = cvt_fp8x2<false>(od, w[1], w[3], sc);
                            ev = cvt_fp8x2<true>(ev, w[4], w[6], sc);
                            od = cvt_fp8x2<true>(od, w[5], w[7], sc);
                            if (NREP >= HP || hp == 0) {
                                dst[tau * KXROW] = ev;
                                dst[tau * KXROW + 2] = od;
                            }
                            if (tau < 3) {
                                const float2_t e0 = fp8x2_back<false>(ev, sc), e1 = fp8x2_back<true>(ev, sc);
                                const float2_t o0 = fp8x2_back<false>(od, sc), o1 = fp8x2_back<true>(od, sc);
                                w[0] -= e0[0]; w[2] -= e0[1]; w[4] -= e1[0]; w[6] -= e1[1];
                                w[1] -= o0[0]; w[3] -= o0[1]; w[5] -= o1[0]; w[7] -= o1[1];
                            }
                        }
                        // zero-point sum of the head over the 16 spans; the heads the other lane of the
                        // span prepared come from it
                        float qs = qsc[0];
#pragma unroll
                        for (int u = 1; u < NV; ++u) qs = (u == v) ? qsc[u] : qs;
                        const float zmine = row16_sum(zp) * qs;
                        if constexpr (HP == 2 && NREP >= 2) {
                            const float zother = __shfl_xor(zmine, 16, 64);
                            zs[y * NREP + 2 * x] = hp == 0 ? zmine : zother;
                            zs[y * NREP + 2 * x + 1] = hp == 0 ? zother : zmine;
                        } else {
                            zs[y * NREP + x] = zmine;
                        }
                    }
                    // the instruction sums (weight 2^(QE - es - eq)) (code / 2): score = sum * 2^(es + eq - QE + 1)
#pragma unroll
                    for (int n = 0; n < NREP; ++n)
                        fac[y * NREP + n] = __uint_as_float((uint32_t)(127 + 1 - QE + es + eq[y * NREP + n]) << 23);
                }
                if constexpr (PIPE_KMETA) {
                    if (more) load_kmeta(nxt);
                }
            } else if constexpr (MM) {
                if constexpr (!PIPE_KMETA) load_kmeta(cur);
#pragma unroll
                for (int y = 0; y < NLAY; ++y) {
                    uint32_t hm = 0;
#pragma unroll
                    for (int e = 0; e < NPL; ++e)
#pragma unroll
                        for (int k = 0; k < 4; ++k) hm = max(hm, kmeta[y][e][k] & 0x7fffu);
                    hm = group_umax<LPG>(hm);
                    const int es = max((int)(hm >> 10), 1) - 14;  // 2^es > every scale of the group
                    const float sinv = __uint_as_float((uint32_t)(127 - es) << 23);
                    float sh[NPL][4], zh[NPL][4];
#pragma unroll
                    for (int e = 0; e < NPL; ++e)
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            sh[e][k] = hbits(kmeta[y][e][k] & 0xffffu) * (kpw[e][k / 2] * sinv);
                            zh[e][k] = hbits(kmeta[y][e][k] >> 16);
                        }
#pragma unroll
                    for (int n = 0; n < NREP; ++n) {
                        const int v = y * NREP + n;
                        float zp = 0.f;
#pragma unroll
                        for (int e = 0; e < NPL; ++e) {
                            const float4 q4 = *(const float4 *)&s_q[v][(li * NPL + e) * 4];
                            const float qv[4] = {q4.x, q4.y, q4.z, q4.w};
                            half4_t hi, lo;
#pragma unroll
                            for (int k = 0; k < 4; ++k) {
                                const float w = qv[k] * sh[e][k];  // |w| < 2^14
                                zp = fmaf(qv[k], zh[e][k], zp);
                                hi[k] = (_Float16)w;
                                lo[k] = (_Float16)__builtin_fmaf(qv[k], sh[e][k], -(float)hi[k]);  // exact product - hi
                            }
                            *(half4_t *)&s_ka[wave][(2 * v) / 4][gi][li * NPL + e][(2 * v) % 4][0] = hi;
                            *(half4_t *)&s_ka[wave][(2 * v) / 4][gi][li * NPL + e][(2 * v) % 4 + 1][0] = lo;
                        }
                        zs[v] = group_sum<LPG>(zp) * qsc[v];
                        // codes arrive as c 2^(bit-24): sum = true sum * 2^(-es - eq - 10)
                        fac[v] = __uint_as_float((uint32_t)(127 + 10 + es + eq[v]) << 23);
                    }
                }
                if constexpr (PIPE_KMETA) {
                    if (more) load_kmeta(nxt);
                }
            } else {
                const int Gidx = tile * NGT + gi;
                const bool g_ok = Gidx * G < seqTq;
                uint32_t meta[NLAY][CPP];
#pragma unroll
                for (int y = 0; y < NLAY; ++y) {
                    const uint32_t *mp = (const uint32_t *)(a.arena + dsc[y].k_meta + slice * a.st.k_meta) +
                                         (int64_t)(tin / G + gi) * D + li * CPP;
                    if (g_ok) VecLoad<CPP>::ld(mp, meta[y]);
                    else {
#pragma unroll
                        for (int k = 0; k < CPP; ++k) meta[y][k] = 0;
                    }
                }
#pragma unroll
                for (int y = 0; y < NLAY; ++y) {
                    float sh[CPP], zh[CPP];
#pragma unroll
                    for (int k = 0; k < CPP; ++k) {
                        sh[k] = hbits(meta[y][k] & 0xffffu);
                        if constexpr (!QK_COPY) sh[k] *= pw[k];
                        zh[k] = hbits(meta[y][k] >> 16);
                    }
#pragma unroll
                    for (int n = 0; n < NREP; ++n) {
                        const int v = y * NREP + n;
                        float zp = 0.f;
                        float wv[CPP], qv[CPP];
                        if constexpr (Q_LDS) {
#pragma unroll
                            for (int k = 0; k < CPP; ++k) qv[k] = s_q[v][li * CPP + k];
                        }
#pragma unroll
                        for (int k = 0; k < CPP; ++k) {
                            if constexpr (!Q_LDS) qv[k] = qz[v][k];
                            if constexpr (QK_COPY) wv[k] = qk[v][k] * sh[k];
                            else wv[k] = qv[k] * sh[k];
                            zp = fmaf(qv[k], zh[k], zp);
                        }
#pragma unroll
                        for (int k4 = 0; k4 < CPP; k4 += 4) {
                            if constexpr (CPP >= 4)
                                *(float4 *)&s_kw[wave][v][gi][li * CPP + k4] = make_float4(wv[k4], wv[k4 + 1], wv[k4 + 2], wv[k4 + 3]);
                            else
                                *(float2 *)&s_kw[wave][v][gi][li * CPP] = make_float2(wv[0], wv[1]);
                        }
                        zs[v] = group_sum<LPG>(zp);
                    }
                }
            }
            // ---- plain path: this tile's key rows now; its value inputs now with one head, and
            // after the key phase with several, which keeps 32+ registers free during the key loop
            // (one more wave per SIMD) at the cost of latency that the other waves cover
            constexpr bool V_LOAD_EARLY = NV == 1;
            if constexpr (!MM) load_kcodes(cur);
            if constexpr (!MM && V_LOAD_EARLY) load_values(cur);
            wave_lds_fence();
            // ---- q . K^ over the packed codes
            float tsum[2][NV];  // code part of the scores of this lane's two tokens
            const int kg = (row * 32) / G;  // key group of this row inside the tile
            if constexpr (KX) {
                // One instruction per 16 tokens (column block m) and 4 virtual heads: rows 4 h .. 4 h + 3
                // are the four fp8 terms of head h, so lane (token r16, quarter row) receives the four
                // partial scores of head `row` and folds them.  A changes with the key group.
                constexpr int NSET = (NV + 3) / 4, MPG = G / 16;  // row sets; column blocks per key group
                float xs[NSET][8];
                float4_t pc = {0.f, 0.f, 0.f, 0.f};
                int px = 0, pm = 0;
#pragma unroll
                for (int gq = 0; gq < NGT; ++gq) {
                    int8_v ka[NSET];
#pragma unroll
                    for (int x = 0; x < NSET; ++x) {
                        const int rr = min(16 * x + r16, 4 * NV - 1);  // rows past the last head repeat it; nobody reads them
                        const uint4 lo = *(const uint4 *)&s_kx[wave][gq][rr][row * 8], hi = *(const uint4 *)&s_kx[wave][gq][rr][row * 8 + 4];
                        ka[x] = int8_v{(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
                    }
#pragma unroll
                    for (int mm = 0; mm < MPG; ++mm) {
                        const int m = gq * MPG + mm;
                        constexpr uint32_t NIB = 0x33333333u;
                        const int8_v kb = {(int)(kc[m][0] & NIB), (int)((kc[m][0] >> 2) & NIB), (int)(kc[m][1] & NIB),
                                           (int)((kc[m][1] >> 2) & NIB), 0, 0, 0, 0};
#pragma unroll
                        for (int x = 0; x < NSET; ++x) {
                            // (the result is folded one step later, behind the next instruction's issue)
                            const float4_t c = mfma_fp8_fp4(ka[x], kb, float4_t{0.f, 0.f, 0.f, 0.f});
                            if (m > 0 || x > 0) xs[px][pm] = fmaf(fmaf(fmaf(pc[3], 0.0625f, pc[2]), 0.0625f, pc[1]), 0.0625f, pc[0]);
                            pc = c;
                            px = x;
                            pm = m;
                        }
                    }
                }
                xs[px][pm] = fmaf(fmaf(fmaf(pc[3], 0.0625f, pc[2]), 0.0625f, pc[1]), 0.0625f, pc[0]);
                // xs[x][m] = score of (token 16 m + r16, head 4 x + row); wanted: lane (r16, row) holds tokens
                // 32 row + 16 s + r16 for every head: a 4 x 4 transpose over the lanes 16 apart, through the
                // wave's A table space (all its readers are done), rows [token r16][head][column block]
                // padded to 36 floats per head set.
                float *tp = (float *)&s_kx[wave][0][0][0];
                wave_lds_fence();
#pragma unroll
                for (int x = 0; x < NSET; ++x) {
                    float *dst = tp + ((x * 16 + r16) * 36 + row * 8);
                    *(float4 *)dst = make_float4(xs[x][0], xs[x][1], xs[x][2], xs[x][3]);
                    *(float4 *)(dst + 4) = make_float4(xs[x][4], xs[x][5], xs[x][6], xs[x][7]);
                }
                wave_lds_fence();
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const float2 t2 = *(const float2 *)(tp + (((v / 4) * 16 + r16) * 36 + (v % 4) * 8 + 2 * row));
                    tsum[0][v] = t2.x * fac[v];
                    tsum[1][v] = t2.y * fac[v];
                }
            } else if constexpr (MM) {
                // the lanes of a token group are the lanes that prepared it (kg == gi); A matrix n
                // sits in block n % NB of register pair n / NB
                constexpr int NCHUNK = WK * 2 * CPB;
                const int bx = (lane % (4 * NB)) >> 2, ri = lane & 3;
                half4_t ka[NKS][AREG];
#pragma unroll
                for (int x = 0; x < NKS; ++x)
#pragma unroll
                    for (int r = 0; r < AREG; ++r) {
                        const int rr = min(4 * x + ri, 2 * NV - 1) - 4 * x;  // rows past the last head repeat it; nobody reads them
                        ka[x][r] = *(const half4_t *)&s_ka[wave][x][kg][r * NB + bx][rr][0];
                    }
                float4_t ak[NKS][2];
#pragma unroll
                for (int x = 0; x < NKS; ++x) ak[x][0] = ak[x][1] = float4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ci = 0; ci < NCHUNK; ++ci) {
                    const int wi = ci / (2 * CPB), src = (ci / CPB) % 2, p4 = (ci % CPB) * 4;
                    uint32_t c2[2][4];
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
                        const uint32_t x = src ? (kc[s2][wi] >> 8) : kc[s2][wi];
#pragma unroll
                        for (int p = 0; p < 4; ++p) c2[s2][p] = x & (MASKK << (BK * (p4 + p)));
                    }
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int n = 2 * ci + h;
#pragma unroll
                        for (int x = 0; x < NKS; ++x)
#pragma unroll
                            for (int s2 = 0; s2 < 2; ++s2)
                                ak[x][s2] = mfma_rows<CBSZ>(ka[x][n / NB], codes4(c2[s2][2 * h], c2[s2][2 * h + 1]),
                                                            ak[x][s2], n % NB);
                    }
                }
#pragma unroll
                for (int v = 0; v < NV; ++v)
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2)
                        tsum[s2][v] = (ak[(2 * v) / 4][s2][(2 * v) % 4] + ak[(2 * v) / 4][s2][(2 * v) % 4 + 1]) * fac[v];
            } else {
                // Chains per score: low-half and high-half channels, and with several heads also even
                // and odd positions.  A head step then never reuses an accumulator within 8
                // instructions; at 4 the compiler pads every reuse with a wait state.
                constexpr int NCHAIN = NV > 1 ? 2 : 1;
                float sc[2][NV][NCHAIN], sch[2][NV][NCHAIN];
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int v = 0; v < NV; ++v)
#pragma unroll
                        for (int e = 0; e < NCHAIN; ++e) sc[s][v][e] = sch[s][v][e] = 0.f;
                constexpr int NCHUNK = WK * 2 * CPB;
                constexpr int NSTEP = NCHUNK * NV;
                constexpr int PF = NSTEP > 2 ? 2 : 1;
                float4 wl[PF + 1], wh[PF + 1];
                auto chunk_base = [](int ci) {  // first low-half channel of chunk ci
                    return (ci / (2 * CPB)) * PERK + ((ci / CPB) % 2) * BYTEK + (ci % CPB) * 4;
                };
                auto issue = [&](int st) {
                    const int base = chunk_base(st / NV);
                    wl[st % (PF + 1)] = *(const float4 *)&s_kw[wave][st % NV][kg][base];
                    wh[st % (PF + 1)] = *(const float4 *)&s_kw[wave][st % NV][kg][base + HALFK];
                };
#pragma unroll
                for (int st = 0; st < PF; ++st) issue(st);
#pragma unroll
                for (int ci = 0; ci < NCHUNK; ++ci) {
                    const int wi = ci / (2 * CPB), src = (ci / CPB) % 2, p4 = (ci % CPB) * 4;
                    uint32_t c2[2][4];
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
                        const uint32_t x = src ? (kc[s2][wi] >> 8) : kc[s2][wi];
#pragma unroll
                        for (int p = 0; p < 4; ++p) c2[s2][p] = x & (MASKK << (BK * (p4 + p)));
                    }
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        const int st = ci * NV + v;
                        if (st + PF < NSTEP) issue(st + PF);
                        const float4 lo = wl[st % (PF + 1)], hi = wh[st % (PF + 1)];
                        const float wlo[4] = {lo.x, lo.y, lo.z, lo.w}, whi[4] = {hi.x, hi.y, hi.z, hi.w};
#pragma unroll
                        for (int p = 0; p < 4; ++p)
#pragma unroll
                            for (int s2 = 0; s2 < 2; ++s2) {
                                float &al = sc[s2][v][p % NCHAIN], &ah = sch[s2][v][p % NCHAIN];
                                al = fma_mix_lo(wlo[p], c2[s2][p], al);
                                ah = fma_mix_hi(whi[p], c2[s2][p], ah);
                            }
                        if constexpr (NV > 1) __builtin_amdgcn_sched_barrier(0);
                    }
                }
#pragma unroll
                for (int v = 0; v < NV; ++v)
#pragma unroll
                    for (int s2 = 0; s2 < 2; ++s2) {
                        float t = sc[s2][v][0] + sch[s2][v][0];
                        if constexpr (NCHAIN == 2) t += sc[s2][v][1] + sch[s2][v][1];
                        tsum[s2][v] = t;
                    }
            }
            if constexpr (MM) {
                if (more) load_kcodes(nxt);
            } else if constexpr (!V_LOAD_EARLY) {
                load_values(cur);
            }
            // ---- online softmax bookkeeping (log2 domain), value weights -> LDS
            // The value weights p * s^ travel as fp16.  A token whose largest value scale is
            // >= 2^9 raises the softmax reference by the excess exponent, which keeps every
            // weight below 2^15 for any fp16 input; for ordinary scales this adds nothing.
            float eadd[NLAY][2];
#pragma unroll
            for (int y = 0; y < NLAY; ++y)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    uint32_t hmax = 0;
#pragma unroll
                    for (int j = 0; j < NJ; ++j) hmax = max(hmax, vm[y][s][j] & 0x7fffu);
                    eadd[y][s] = (float)max((int)(hmax >> 10) - 23, 0);
                }
            float pr[2][NV];
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const float t0 = tsum[0][v], t1 = tsum[1][v];
                float u0 = row_ok ? t0 + zs[v] : -INFINITY;
                float u1 = row_ok ? t1 + zs[v] : -INFINITY;
                // The running maximum only has to bound the scores: it moves when some token of the
                // tile exceeds it (one compare and a wave-uniform branch, rarely taken after the
                // first tiles), and only then is the tile's maximum reduced over the wave.
                const float tl = fmaxf(u0 + eadd[v / NREP][0], u1 + eadd[v / NREP][1]);
                if (__any(tl > m_run[v])) {
                    const float m_new = fmaxf(m_run[v], wave_max(tl));
                    float alpha = exp2_le0(m_run[v] - m_new);  // m_run = -inf gives 0
                    l_run[v] *= alpha;
#pragma unroll
                    for (int c = 0; c < CPL; ++c) {
                        if constexpr (MM) accm[v / 4][c][v % 4] *= alpha;
                        else accv[v][c] *= alpha;
                    }
#pragma unroll
                    for (int j = 0; j < NJ; ++j) zacc[v][j] *= alpha;
                    m_run[v] = m_new;
                }
                pr[0][v] = exp2_le0(u0 - m_run[v]);
                pr[1][v] = exp2_le0(u1 - m_run[v]);
                l_run[v] += pr[0][v] + pr[1][v];
            }
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const int tau = r16 + 16 * s;          // token inside the block
                const int tw = tau % TPW;              // ... inside its value word
                const int pos = (tau / TPW) * TPW + 2 * (tw % (TPW / 2)) + tw / (TPW / 2);  // pair order
                const float tsc = __builtin_ldexpf(1.0f, 6 - ((BV * CPL * tw) & 7));
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const float pt = pr[s][v] * tsc;
#pragma unroll
                    for (int j = 0; j < NJ; ++j) {
                        uint32_t m = vm[v / NREP][s][j];
                        s_vw[wave][v][row][j][pos] = (_Float16)(pt * hbits(m & 0xffffu));
                        zacc[v][j] = fmaf(pr[s][v], hbits(m >> 16), zacc[v][j]);
                    }
                }
            }
            wave_lds_fence();
            // ---- P . V^ over the packed codes
            const int jl = (lane * CPL) / G;  // channel group of this lane's channels
            if constexpr (MM) {
                // A matrix of token quad qd (4 tokens in pair order, one row per head) sits in block
                // qd % NB of register pair qd / NB; the blocks of a channel group share it
                const int bx = (lane % (4 * NB)) >> 2, ri = lane & 3;
                half4_t va[NVS][AREG];
#pragma unroll
                for (int x = 0; x < NVS; ++x)
#pragma unroll
                    for (int r = 0; r < AREG; ++r) {
                        const int qd = r * NB + bx, kb = qd / 8, q8 = qd % 8;
                        const int v = min(4 * x + ri, NV - 1);  // rows past the last head repeat it; nobody reads them
                        va[x][r] = *(const half4_t *)&s_vw[wave][v][kb][jl][(q8 / QPW) * TPW + 4 * (q8 % QPW)];
                    }
                // step st = (token quad qd, channel c); the codes of a step are isolated one step ahead
                // of the instruction that reads them (a freshly written operand would stall it)
                auto vcodes = [&](int st) {
                    const int qd = st / CPL, c = st % CPL, kb = qd / 8, m = (qd % 8) / QPW, qq = qd % QPW;
                    const int bit0 = BV * ((2 * qq) * CPL + c), bit1 = BV * ((2 * qq + 1) * CPL + c);
                    const uint32_t x0 = (bit0 >= 8) ? (vc[kb][m] >> 8) : vc[kb][m];
                    const uint32_t x1 = (bit1 >= 8) ? (vc[kb][m] >> 8) : vc[kb][m];
                    return codes4(x0 & (MASKV << (bit0 & 7)), x1 & (MASKV << (bit1 & 7)));
                };
                half4_t bn = vcodes(0);
#pragma unroll
                for (int st = 0; st < 32 * CPL; ++st) {
                    const int qd = st / CPL, c = st % CPL;
                    const half4_t b = bn;
                    if (st + 1 < 32 * CPL) bn = vcodes(st + 1);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int x = 0; x < NVS; ++x) accm[x][c] = mfma_rows<CBSZ>(va[x][qd / NB], b, accm[x][c], qd % NB);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (more) load_values(nxt);
            } else {
                constexpr int VCH = (TPW / 2) / 4;        // chunks of 4 token pairs per word
                constexpr int NCHUNK = 4 * WS * VCH;
                constexpr int NSTEP = NCHUNK * NV;
                constexpr int PF = NSTEP > 2 ? 2 : 1;
                uint4 wq[PF + 1];
                auto issue = [&](int st) {
                    const int ci = st / NV;
                    const int kb = ci / (WS * VCH), m = (ci / VCH) % WS, i0 = (ci % VCH) * 4;
                    wq[st % (PF + 1)] = *(const uint4 *)&s_vw[wave][st % NV][kb][jl][m * TPW + 2 * i0];
                };
#pragma unroll
                for (int st = 0; st < PF; ++st) issue(st);
#pragma unroll
                for (int ci = 0; ci < NCHUNK; ++ci) {
                    const int kb = ci / (WS * VCH), m = (ci / VCH) % WS, i0 = (ci % VCH) * 4;
                    half2_t c2[4][CPL];
#pragma unroll
                    for (int i = 0; i < 4; ++i)
#pragma unroll
                            for (int c = 0; c < CPL; ++c) {
                                const int bit = BV * ((i0 + i) * CPL + c);   // position inside a half, < 16
                                const uint32_t x = (bit >= 8) ? (vc[kb][m] >> 8) : vc[kb][m];
                                c2[i][c] = __builtin_bit_cast(half2_t, x & (MASKV << (bit & 7)));
                            }
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        const int st = ci * NV + v;
                        if (st + PF < NSTEP) issue(st + PF);
                        const uint4 t = wq[st % (PF + 1)];
                        const half2_t w2[4] = {__builtin_bit_cast(half2_t, t.x), __builtin_bit_cast(half2_t, t.y),
                                               __builtin_bit_cast(half2_t, t.z), __builtin_bit_cast(half2_t, t.w)};
#pragma unroll
                        for (int i = 0; i < 4; ++i)
#pragma unroll
                            for (int c = 0; c < CPL; ++c)
                                accv[v][c] = __builtin_amdgcn_fdot2(w2[i], c2[i][c], accv[v][c], false);
                        if constexpr (NV > 1) __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
            wave_lds_fence();
#ifdef XQ_KX_TU
        };
        {
            int it = wave;
            for (; it + 4 < n_tiles; it += 4) one_tile(std::true_type{});
            if (it < n_tiles) one_tile(std::false_type{});
        }
#else
        }
#endif
        // ---- wave totals
        const int jl = (lane * CPL) / G;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            l_run[v] = group_sum<64>(l_run[v]);
            float zj[NJ];
#pragma unroll
            for (int j = 0; j < NJ; ++j) zj[j] = group_sum<64>(zacc[v][j]);
            float zsel = zj[0];
#pragma unroll
            for (int j = 1; j < NJ; ++j) zsel = (jl == j) ? zj[j] : zsel;
#pragma unroll
            for (int c = 0; c < CPL; ++c) {
                if constexpr (MM) accv[v][c] = accm[v / 4][c][v % 4];
                accv[v][c] = accv[v][c] * __builtin_ldexpf(1.0f, 18 - BV * c) + zsel;
            }
        }
        __syncthreads();  // every wave is done with the key weights before their space is reused
#pragma unroll
        for (int v = 0; v < NV; ++v) {
#pragma unroll
            for (int c = 0; c < CPL; ++c) s_part[wave][v][lane * CPL + c] = accv[v][c];
            if (lane == 0) {
                s_part[wave][v][D] = m_run[v];
                s_part[wave][v][D + 1] = l_run[v];
            }
        }
    } else {
        // ------------------------------------------------------------ fp16 ring (newest tokens)
        // A 16-lane row takes one token per iteration (lane = D/16 channels), so a workgroup
        // walks 16 ring tokens at a time; each row keeps its own softmax state.
        constexpr int CR = D / 16;
        float qf[NV][CR], acr[NV][CR];
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int c = 0; c < CR; ++c) {
                qf[v][c] = hbits(qptr(v)[r16 * CR + c]) * a.scale_log2e;
                acr[v][c] = 0.f;
            }
        const int r = seqT - seqTq;
        // The rows of the row's next two tokens are in flight while the current one is worked on: with one
        // workgroup per ring the walk is a chain of memory latencies otherwise (in a call for one layer
        // of a short cache the ring workgroup is the last to finish), and two tokens per row keep
        // about as many bytes in flight per CU as the packed-token workgroups do.
        uint32_t kn[2][NLAY][CR / 2], vn[2][NLAY][CR / 2];
        auto ring_load = [&](int i, auto buf) {
            constexpr int b = decltype(buf)::value;
            const int slot = (seqTq + min(i, r - 1)) % a.R;   // (past the end: the last token again, not used)
#pragma unroll
            for (int y = 0; y < NLAY; ++y) {
                VecLoad<CR / 2>::ld((const uint32_t *)(a.arena + dsc[y].k_res + (int64_t)bh * a.st.res) + (slot * D + r16 * CR) / 2, kn[b][y]);
                VecLoad<CR / 2>::ld((const uint32_t *)(a.arena + dsc[y].v_res + (int64_t)bh * a.st.res) + (slot * D + r16 * CR) / 2, vn[b][y]);
            }
        };
        // one ring token from buffer b; its buffer is refilled with token i + 32 as soon as it is copied out
        auto ring_token = [&](int i, auto buf) {
            constexpr int b = decltype(buf)::value;
#pragma unroll
            for (int y = 0; y < NLAY; ++y) {
                uint32_t kw[CR / 2], vw[CR / 2];
#pragma unroll
                for (int c = 0; c < CR / 2; ++c) {
                    kw[c] = kn[b][y][c];
                    vw[c] = vn[b][y][c];
                }
                if (y == NLAY - 1) ring_load(i + 32, buf);
                float kf[CR], vf[CR];
#pragma unroll
                for (int c = 0; c < CR; ++c) {
                    kf[c] = hbits((c & 1) ? (kw[c / 2] >> 16) : (kw[c / 2] & 0xffffu));
                    vf[c] = hbits((c & 1) ? (vw[c / 2] >> 16) : (vw[c / 2] & 0xffffu));
                }
#pragma unroll
                for (int n = 0; n < NREP; ++n) {
                    const int v = y * NREP + n;
                    float part = 0.f;
#pragma unroll
                    for (int c = 0; c < CR; ++c) part = fmaf(qf[v][c], kf[c], part);
                    const float u = group_sum<16>(part);
                    const float m_new = fmaxf(m_run[v], u);
                    const float alpha = exp2_le0(m_run[v] - m_new);
                    const float p = exp2_le0(u - m_new);
                    l_run[v] = l_run[v] * alpha + p;
#pragma unroll
                    for (int c = 0; c < CR; ++c) acr[v][c] = fmaf(p, vf[c], acr[v][c] * alpha);
                    m_run[v] = m_new;
                }
            }
        };
        const int i_first = wave * 4 + row;
        if (r > 0) {
            ring_load(i_first, std::integral_constant<int, 0>{});
            ring_load(i_first + 16, std::integral_constant<int, 1>{});
        }
        for (int i = i_first; i < r; i += 32) {
            ring_token(i, std::integral_constant<int, 0>{});
            if (i + 16 < r) ring_token(i + 16, std::integral_constant<int, 1>{});
        }
        // merge the 4 rows of the wave
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            float M = fmaxf(m_run[v], __shfl_xor(m_run[v], 16, 64));
            M = fmaxf(M, __shfl_xor(M, 32, 64));
            const float f = (m_run[v] == -INFINITY) ? 0.f : exp2f(m_run[v] - M);
            float l = l_run[v] * f;
            l += __shfl_xor(l, 16, 64);
            l += __shfl_xor(l, 32, 64);
#pragma unroll
            for (int c = 0; c < CR; ++c) {
                float x = acr[v][c] * f;
                x += __shfl_xor(x, 16, 64);
                x += __shfl_xor(x, 32, 64);
                acr[v][c] = x;
            }
            m_run[v] = M;
            l_run[v] = l;
        }
        __syncthreads();
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            if (row == 0) {
#pragma unroll
                for (int c = 0; c < CR; ++c) s_part[wave][v][r16 * CR + c] = acr[v][c];
            }
            if (lane == 0) {
                s_part[wave][v][D] = m_run[v];
                s_part[wave][v][D + 1] = l_run[v];
            }
        }
    }

    // ---------------------------------------------------------------- combine the 4 waves
    __syncthreads();
    for (int idx = tid; idx < NV * (D + 2); idx += 256) {
        const int v = idx / (D + 2), e = idx % (D + 2);
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) M = fmaxf(M, s_part[w][v][D]);
        float val;
        if (e == D) {
            val = M;
        } else {
            val = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                float mw = s_part[w][v][D];
                float f = (mw == -INFINITY) ? 0.f : exp2f(mw - M);
                val += f * s_part[w][v][e];
            }
        }
        const int y = v / NREP, n = v % NREP;
        float *wp = a.ws + ((((int64_t)(lz * NLAY + y) * a.batch + bi) * a.n_q_heads + hkv * a.rep + a.q_head0 + n) *
                                (a.n_splits + 1) + split) * (D + 2);
        // (device-scope store: written through the L2 of this XCD, for a reader on another)
        if (a.arrivals) __hip_atomic_store(wp + e, val, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else wp[e] = val;
    }
    if (a.arrivals == nullptr) return;  // a merge launch follows
    // ---------------------------------------------------------------- the last workgroup to arrive merges
    // The n_splits + 1 workgroups of this (layer or pair, sequence, kv head) count themselves in
    // once their partials have been written; whoever finds the count complete reads all of them
    // back and writes the outputs, in the merge kernel's order and arithmetic.  Nobody waits: the
    // others simply leave.  The counter is back at zero for the next launch.
    // Ordering without cache-wide write-backs or invalidations (a device-scope fence costs an L2
    // sweep per workgroup here and halves the kernel's speed): the partials are device-scope
    // (write-through) stores; every thread waits until the memory system has acknowledged its own
    // (the wait is spelled out: a workgroup barrier by itself does not wait for stores, whose
    // visibility inside a workgroup needs no acknowledgement); after the barrier thread 0 counts the
    // workgroup in with a device-scope atomic; the last arrival's loads are device-scope loads issued
    // after its own atomic has returned.
    __shared__ uint32_t s_last;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    uint32_t *arrive = a.arrivals + (int64_t)lz * nbh + bh;
    if (tid == 0) s_last = __hip_atomic_fetch_add(arrive, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (uint32_t)a.n_splits;
    __syncthreads();
    if (!s_last) return;
    static_assert(sizeof(s_raw) >= sizeof(float) * XQ_MERGE_LDS_FLOATS(NV), "merge scratch");
    xq_merge_block<D, NV, true>(
        [&](int v) -> int64_t {
            const int y = v / NREP, n = v % NREP;
            return ((int64_t)(lz * NLAY + y) * a.batch + bi) * a.n_q_heads + hkv * a.rep + a.q_head0 + n;
        },
        a.ws, a.out, a.n_splits + 1, (float *)s_raw, tid);
    if (tid == 0) __hip_atomic_store(arrive, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // (written through, like the counts)
}

template <int NREP>
hipError_t launch_cfg(const XqDecodeArgs &a, int n_layers, int pair_fused, hipStream_t s) {
    constexpr int D = XQ_D, G = XQ_G, BK = XQ_BK, BV = XQ_BV;
    dim3 block(256);
    XqDecodeArgs b = a;
    b.n_launch_z = pair_fused ? n_layers / 2 : n_layers;
    dim3 grid((unsigned)((a.n_splits + 1) * a.batch * a.n_kv_heads * b.n_launch_z));
#ifdef XQ_KX_TU
    // the kernels with the fp8 x fp4 key phase: at least four (query head, layer) pairs per kv head
    if constexpr (D == 128 && BK == 2 && NREP >= 2) {
        if (pair_fused) {
            if constexpr (2 * NREP * (XQ_TILE_TOKENS / G) <= 16) {
                xq_decode_kernel<D, G, BK, BV, NREP, 2, false, true, true><<<grid, block, 0, s>>>(b);
                return hipGetLastError();
            }
        } else if constexpr (NREP >= 4) {
            if (a.reuse_codes) xq_decode_kernel<D, G, BK, BV, NREP, 1, true, true, true><<<grid, block, 0, s>>>(b);
            else xq_decode_kernel<D, G, BK, BV, NREP, 1, false, true, true><<<grid, block, 0, s>>>(b);
            return hipGetLastError();
        }
    }
    return hipErrorInvalidValue;
#else
    constexpr bool HAS_MM = D == 128;  // the matrix path is built for head_dim 128
    if (a.matrix && !HAS_MM) return hipErrorInvalidValue;
    if (pair_fused) {
        // 2 * NREP virtual heads must fit the LDS weight tables
        if constexpr (2 * NREP * (XQ_TILE_TOKENS / G) <= 16 && (D == 128 || NREP == 1)) {
            if constexpr (HAS_MM) {
                if (a.matrix) xq_decode_kernel<D, G, BK, BV, NREP, 2, false, true><<<grid, block, 0, s>>>(b);
                else xq_decode_kernel<D, G, BK, BV, NREP, 2><<<grid, block, 0, s>>>(b);
            } else {
                xq_decode_kernel<D, G, BK, BV, NREP, 2><<<grid, block, 0, s>>>(b);
            }
        } else {
            return hipErrorInvalidValue;
        }
    } else if (a.matrix) {
        if constexpr (HAS_MM) {
            if (a.reuse_codes) xq_decode_kernel<D, G, BK, BV, NREP, 1, true, true><<<grid, block, 0, s>>>(b);
            else xq_decode_kernel<D, G, BK, BV, NREP, 1, false, true><<<grid, block, 0, s>>>(b);
        }
    } else {
        if (a.reuse_codes) xq_decode_kernel<D, G, BK, BV, NREP, 1, true><<<grid, block, 0, s>>>(b);
        else xq_decode_kernel<D, G, BK, BV, NREP, 1><<<grid, block, 0, s>>>(b);
    }
    return hipGetLastError();
#endif
}

}  // namespace

#ifdef XQ_KX_TU
#define XQ_CAT2(a, b, c, d) xq_launch_decode_kx_##a##_##b##_##c##d
#else
#define XQ_CAT2(a, b, c, d) xq_launch_decode_##a##_##b##_##c##d
#endif
#define XQ_CAT(a, b, c, d) XQ_CAT2(a, b, c, d)

// One translation unit per (head_dim, group, key bits, value bits); n_rep = query heads per kv head.
hipError_t XQ_CAT(XQ_D, XQ_G, XQ_BK, XQ_BV)(const XqDecodeArgs &a, int n_rep, int n_layers, int pair_fused,
                                            hipStream_t s) {
    switch (n_rep) {
        case 1: return launch_cfg<1>(a, n_layers, pair_fused, s);
#if XQ_D == 128
        case 2: return launch_cfg<2>(a, n_layers, pair_fused, s);
        case 4: return launch_cfg<4>(a, n_layers, pair_fused, s);
#endif
        default: return hipErrorInvalidValue;
    }
}
