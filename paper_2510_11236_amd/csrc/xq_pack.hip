// Quantize + bit-pack kernel (prefill pack and ring flush), ring write, debug unpack, page-table
// update and the code-difference histogram.
//
// The pack keeps a token group's g rows in the registers of one wave (xq_pack_wave.h): keys reduce
// min/max down the token axis per channel, values along the channel axis per token (Sec. 4.1:
// per-channel keys, per-token values).  Scale, zero-point, codes and the calibrated metadata
// follow Eq. 1-2 and Eq. 12 with one correctly rounded fp32 operation per step (no fused
// multiply-add), which is what makes the packed words reproducible.
#include "xq_internal.h"
#include "xq_pack_wave.h"

namespace {

// One wave per item, XQ_PACK_WAVES waves per workgroup along grid.x.  An item is one token group
// (head_dim 128) or two neighbouring ones, one per half of the wave (head_dim 64; an odd last group
// is done by both halves, which then store the same bytes twice).  The first half of the items are
// the key groups, the second half the value groups (kept apart because workgroups are dealt
// round-robin to the 8 XCDs and the two kinds cost differently); grid.y = sequence * kv head,
// grid.z = layer.
// MG: built for caches whose sharing pairs store merged codes (Appendix E); a wave of the
// pair's first layer then also reads the second layer's rows and writes that layer's metadata,
// and the second layer's own wave has nothing left to do.
#define XQ_PACK_WAVES 4   // waves per workgroup
template <int G, bool MG = false, int D = 128>
__global__ __launch_bounds__(64 * XQ_PACK_WAVES) void xq_pack_wave_kernel(XqPackArgs a) {
    constexpr int GPW = 128 / D;   // token groups per wave
    __shared__ float4 s_par_all[XQ_PACK_WAVES][128];   // value-group parameters: G * (D / G) per group, GPW groups
    __shared__ float4 s_par2_all[XQ_PACK_WAVES][MG ? 128 : 1];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
    float4 *s_par = s_par_all[wave], *s_par2 = s_par2_all[wave];
    const int item = blockIdx.x * XQ_PACK_WAVES + wave;
    const int n_items = (a.n_groups + GPW - 1) / GPW;   // per kind
    if (item >= 2 * n_items) return;
    const bool is_v = item >= n_items;
    // this lane's group and its channel pair inside it
    const int grp = min(((is_v ? item - n_items : item)) * GPW + lane / (D / 2), a.n_groups - 1), cl = lane % (D / 2);
    const int bh = a.bh0 + blockIdx.y, lz = blockIdx.z;
    const XqLayerDesc d = a.layers[a.layer0 + lz];
    if constexpr (MG) {
        // second layer of a pair that stores merged codes: the first layer's wave does its part
        // (a call covers whole pairs, so that layer is layer lz - 1 of this launch)
        if (lz > 0 && (is_v ? a.layers[a.layer0 + lz - 1].v_merge : a.layers[a.layer0 + lz - 1].k_merge)) return;
    }
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
    for (int t = 0; t < G; ++t) rows[t] = __builtin_nontemporal_load((const uint32_t *)(src + t * s_tok + 2 * cl));
    const uint32_t none[1] = {0};
    if constexpr (MG) {
        if (is_v ? d.v_merge : d.k_merge) {  // uniform over the wave
            const XqLayerDesc d2 = a.layers[a.layer0 + lz + 1];
            const uint16_t *src2;
            if (a.from_ring) {
                src2 = (const uint16_t *)(a.arena + (is_v ? d2.v_res : d2.k_res) + (int64_t)bh * a.st.res) +
                       (int64_t)(src_tok0 + grp * G) * D;
            } else {
                src2 = src + a.s_layer;
            }
            uint32_t rows2[G];
#pragma unroll
            for (int t = 0; t < G; ++t) rows2[t] = __builtin_nontemporal_load((const uint32_t *)(src2 + t * s_tok + 2 * cl));
            if (!is_v) {
                if (d.bk == 2) pack_keys_wave<G, 2, true, D>(a, d, rows, rows2, lane, slice, dst_tok, &d2);
                else pack_keys_wave<G, 1, true, D>(a, d, rows, rows2, lane, slice, dst_tok, &d2);
            } else {
                if (d.bv == 2) pack_values_wave<G, 2, true, D>(a, d, rows, rows2, lane, slice, dst_tok, s_par, s_par2, &d2);
                else pack_values_wave<G, 1, true, D>(a, d, rows, rows2, lane, slice, dst_tok, s_par, s_par2, &d2);
            }
            return;
        }
    }
    if (!is_v) {
        if (d.bk == 2) pack_keys_wave<G, 2, false, D>(a, d, rows, none, lane, slice, dst_tok);
        else pack_keys_wave<G, 1, false, D>(a, d, rows, none, lane, slice, dst_tok);
    } else {
        if (d.bv == 2) pack_values_wave<G, 2, false, D>(a, d, rows, none, lane, slice, dst_tok, s_par, s_par2);
        else pack_values_wave<G, 1, false, D>(a, d, rows, none, lane, slice, dst_tok, s_par, s_par2);
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
    const int items = 2 * ((a.n_groups + 128 / D - 1) / (128 / D));   // key items, then value items
    dim3 grid((items + XQ_PACK_WAVES - 1) / XQ_PACK_WAVES, a.batch * a.n_kv_heads, n_layers), block(64 * XQ_PACK_WAVES);
    if (D == 128 && g == 32 && !a.merge) xq_pack_wave_kernel<32><<<grid, block, 0, s>>>(a);
    else if (D == 128 && g == 64 && !a.merge) xq_pack_wave_kernel<64><<<grid, block, 0, s>>>(a);
    else if (D == 128 && g == 32) xq_pack_wave_kernel<32, true><<<grid, block, 0, s>>>(a);
    else if (D == 128 && g == 64) xq_pack_wave_kernel<64, true><<<grid, block, 0, s>>>(a);
    else if (D == 64 && g == 32 && !a.merge) xq_pack_wave_kernel<32, false, 64><<<grid, block, 0, s>>>(a);
    else if (D == 64 && g == 64 && !a.merge) xq_pack_wave_kernel<64, false, 64><<<grid, block, 0, s>>>(a);
    else if (D == 64 && g == 32) xq_pack_wave_kernel<32, true, 64><<<grid, block, 0, s>>>(a);
    else if (D == 64 && g == 64) xq_pack_wave_kernel<64, true, 64><<<grid, block, 0, s>>>(a);
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
