// Quantize + bit-pack kernels (prefill pack, ring flush, ring write, debug unpack).
//
// One workgroup quantizes one token group of g tokens of one (layer, sequence, kv head):
// the g x D fp16 tile is staged in LDS once and serves both directions of grouping --
// keys reduce min/max down the token axis per channel, values along the channel axis per
// token (Sec. 4.1: per-channel keys, per-token values).  Scale, zero-point, codes and the
// calibrated metadata follow Eq. 1-2 and Eq. 12 with one correctly rounded fp32 operation
// per step (no fused multiply-add), which is what makes the packed words reproducible.
#include "xq_internal.h"
#include "xq_pack_wave.h"

namespace {

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
