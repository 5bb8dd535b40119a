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

    const int tid = threadIdx.x;
    const int grp = blockIdx.x;
    const int bh = blockIdx.y;
    const int lz = blockIdx.z;
    const int layer = a.layer0 + lz;
    const XqLayerDesc d = a.layers[layer];
    const int bi = bh / a.n_kv_heads, hh = bh % a.n_kv_heads;
    const int dst_tok = a.dst_tok0 + grp * G;

    auto half_at = [&](int t, int c) -> float {
        uint32_t w = tile[t * LDW + (c >> 1)];
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
        // ---- stage the tile
        const uint16_t *src;
        int64_t s_tok;
        if (a.from_ring) {
            src = (const uint16_t *)(a.arena + (is_v ? d.v_res : d.k_res) + (int64_t)bh * a.st.res) +
                  (int64_t)(a.src_tok0 + grp * G) * D;
            s_tok = D;
        } else {
            src = (is_v ? a.v_src : a.k_src) + lz * a.s_layer + bi * a.s_batch + hh * a.s_head +
                  (int64_t)(a.src_tok0 + grp * G) * a.s_tok;
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
            uint32_t meta;
            float s = group_params(mn, mx, n, c1, c2, &meta);
            s_mn[tid] = mn;
            s_sc[tid] = s;
            uint32_t *mp;
            if (!is_v)
                mp = (uint32_t *)(a.arena + d.k_meta + (int64_t)bh * a.st.k_meta) + (int64_t)(dst_tok / G) * D + tid;
            else
                mp = (uint32_t *)(a.arena + d.v_meta + (int64_t)bh * a.st.v_meta) + (int64_t)dst_tok * NJ + tid;
            *mp = meta;
        }
        __syncthreads();
        // ---- codes (skipped by a layer that takes its codes from the layer below)
        if (store) {
            const int per = 32 / B;  // codes per word
            if (!is_v) {
                const int W = D / per, CW = W < 4 ? W : 4;
                const int64_t cs = B == 2 ? a.st.k_codes2 : a.st.k_codes1;
                uint32_t *cp = (uint32_t *)(a.arena + d.k_codes + (int64_t)bh * cs);
                for (int idx = tid; idx < G * W; idx += 256) {
                    int sb = idx / (32 * W), ib = idx % (32 * W);
                    int chunk = ib / (32 * CW), tau = (ib / CW) % 32, wc = ib % CW;
                    int wi = chunk * CW + wc, t = sb * 32 + tau;
                    uint32_t word = 0;
                    for (int e = 0; e < per; ++e) {
                        int c = wi * per + e;
                        word |= code_of(half_at(t, c), s_mn[c], s_sc[c], n) << (B * e);
                    }
                    cp[(int64_t)(dst_tok / 32 + sb) * 32 * W + ib] = word;
                }
            } else {
                const int WS = CPL * B;
                const int64_t cs = B == 2 ? a.st.v_codes2 : a.st.v_codes1;
                uint32_t *cp = (uint32_t *)(a.arena + d.v_codes + (int64_t)bh * cs);
                for (int idx = tid; idx < (G / 32) * 64 * WS; idx += 256) {
                    int sb = idx / (64 * WS), ib = idx % (64 * WS);
                    int slot = ib / WS, m = ib % WS;
                    uint32_t word = 0;
                    for (int e2 = 0; e2 < per; ++e2) {
                        int e = m * per + e2;
                        int t = sb * 32 + e / CPL, c = slot * CPL + e % CPL;
                        int gi = t * NJ + c / G;
                        word |= code_of(half_at(t, c), s_mn[gi], s_sc[gi], n) << (B * e2);
                    }
                    cp[(int64_t)(dst_tok / 32 + sb) * 64 * WS + ib] = word;
                }
            }
        }
        __syncthreads();
    }
}

// Copies n_tok tokens into the fp16 rings (token index t -> slot t mod R), keys and values.
__global__ __launch_bounds__(256) void xq_ring_write_kernel(XqRingArgs a) {
    const int bh = blockIdx.y, lz = blockIdx.z;
    const XqLayerDesc d = a.layers[a.layer0 + lz];
    const int bi = bh / a.n_kv_heads, hh = bh % a.n_kv_heads;
    const int vec = a.D / 8;
    const int total = a.n_tok * vec;
    for (int idx = blockIdx.x * 256 + threadIdx.x; idx < total; idx += gridDim.x * 256) {
        int t = idx / vec, v = idx % vec;
        int64_t so = lz * a.s_layer + bi * a.s_batch + hh * a.s_head + (int64_t)(a.src_tok0 + t) * a.s_tok + v * 8;
        int slot = (a.dst_tok0 + t) % a.R;
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
        int t = (int)((idx / D) % a.Tq);
        int bh = (int)(idx / ((int64_t)D * a.Tq));
        const uint32_t *cp = (const uint32_t *)(a.codes + (int64_t)bh * a.stride);
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

}  // namespace

hipError_t xq_launch_pack(const XqPackArgs &a, int D, int g, int n_layers, hipStream_t s) {
    if (a.n_groups <= 0) return hipSuccess;
    dim3 grid(a.n_groups, a.batch * a.n_kv_heads, n_layers), block(256);
    if (D == 128 && g == 32) xq_pack_kernel<128, 32><<<grid, block, 0, s>>>(a);
    else if (D == 128 && g == 64) xq_pack_kernel<128, 64><<<grid, block, 0, s>>>(a);
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
