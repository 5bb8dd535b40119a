// Internal declarations shared by the host layer and the kernels of libxq.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "xq.h"

#define XQ_MAX_LAYERS 256
#define XQ_MAX_SPLITS 64     // packed-token splits per (layer, sequence, kv head)
#define XQ_TILE_TOKENS 128   // tokens one wave handles per iteration of the decode loop
#define XQ_MAX_RAGGED 256    // largest batch whose sequences may have different lengths
#define XQ_MAX_REP 16        // query heads per kv head
#define XQ_PAGE_UPDATES 240  // page-table entries one update launch carries in its arguments

// Where a layer's regions live inside the arena (byte offsets) and what it holds.
// k_codes / v_codes point at the codes the layer READS: its own, or those of the
// layer below when it shares (Sec. 3.3.4: the dominant layer is the first of the pair).
struct XqLayerDesc {
    int64_t k_codes, v_codes;
    int64_t k_meta, v_meta;
    int64_t k_res, v_res;
    int32_t bk, bv;            // bit width of keys / values
    int32_t k_store, v_store;  // 1 if this layer writes codes
    int32_t k_merge, v_merge;  // 1 if its stored codes are merged with those of the next layer
};

// Per slice strides in bytes; identical for every layer.  A slice is one (sequence, kv head)
// with room for max_tokens, or, in a paged cache, one (page, kv head) with room for a page.
struct XqStrides {
    int64_t k_codes2, k_codes1;  // key codes at 2 / 1 bit
    int64_t v_codes2, v_codes1;
    int64_t k_meta, v_meta, res;
};

// Where the packed tokens of a sequence live.  Contiguous cache: table == nullptr, sequence i
// owns slice row i.  Paged cache: token t of sequence i is token t mod P of page
// table[i * max_pages + t / P], P = 1 << shift tokens (a multiple of the 128-token decode tile).
// The fp16 rings are never paged.
struct XqPaging {
    const int32_t *table;
    int32_t shift, max_pages;
};
// Slice index (row of a [slice][bytes] region) that holds packed token tok of (sequence, kv head);
// *tok_in = index of the token inside the slice.
__host__ __device__ static inline int64_t xq_locate(const XqPaging &p, int seq, int hkv, int n_kv_heads, int tok,
                                                    int *tok_in) {
    if (!p.table) {
        *tok_in = tok;
        return (int64_t)seq * n_kv_heads + hkv;
    }
    *tok_in = tok & ((1 << p.shift) - 1);
    return (int64_t)p.table[(int64_t)seq * p.max_pages + (tok >> p.shift)] * n_kv_heads + hkv;
}

struct xq_cache {
    xq_config cfg;
    char *arena;
    size_t arena_bytes;
    XqLayerDesc layers[XQ_MAX_LAYERS];
    XqLayerDesc *dev_layers;  // copy at the start of the arena
    uint32_t *arrivals;       // arena: one arrival counter per (layer, sequence, kv head) for the decode launches, zero between launches
    XqStrides strides;
    std::vector<int32_t> len;  // tokens held, [layer][sequence]
    // paged cache: host mirror of the page table ([sequence][max_pages], -1 = none), pages in
    // use per sequence, free pages (a stack), device table inside the arena
    XqPaging paging;           // table == nullptr for a contiguous cache
    std::vector<int32_t> page_table, pages_used, free_pages;
    std::vector<int32_t> want;  // packed tokens each sequence is about to hold (sized once, at create: no allocation per call)
    int32_t tiles_per_split_override;  // 0 = automatic
};

__host__ __device__ static inline int xq_quantized_len(int T, int g, int R) {
    int over = T - R;
    return over <= 0 ? 0 : g * ((over + g - 1) / g);
}

// ---- kernel launchers (defined in the .hip files); all return a hipError_t ----
struct XqPackArgs {
    char *arena;
    const XqLayerDesc *layers;  // device
    XqStrides st;
    int32_t layer0;
    int32_t batch, n_kv_heads;
    int32_t R;
    // source: external tensor (from_ring = 0) or the layer's own fp16 ring (from_ring = 1)
    const uint16_t *k_src, *v_src;
    int64_t s_layer, s_batch, s_head, s_tok;  // element strides of the external tensor
    int32_t from_ring;
    int32_t src_tok0;   // first source token (external) or first ring slot (ring)
    int32_t dst_tok0;   // first destination token (multiple of g)
    int32_t n_groups;   // token groups of g to quantize
    float c1_1, c2_1;   // eta1 * 1, 1 - 2 eta1     (1-bit)
    float c1_2, c2_2;   // eta2 * 3, 1 - 2 eta2     (2-bit)
    int32_t merge;      // any layer merges codes: take the general kernel
    uint32_t lut1, lut2;  // merged code for every (e_0, e_1), 1-bit / 2-bit
    int32_t bh0;        // first (sequence, kv head) slice served; grid.y counts from it
    // ring flush of a batch with per-sequence lengths: sequence i holds seq_T[i] tokens and is
    // flushed (its oldest g ring tokens) only if its ring is full; src/dst offsets follow from it
    int32_t ragged;
    XqPaging pg;
    int32_t seq_T[XQ_MAX_RAGGED];
};
hipError_t xq_launch_pack(const XqPackArgs &a, int D, int g, int n_layers, hipStream_t s);

// Causal attention of a prompt (head_dim 128) with the pack of its K/V in the same kernel: pk describes
// the K/V source and the pack exactly as for xq_launch_pack (from_ring = 0, all sequences).
struct XqPrefillArgs {
    XqPackArgs pk;
    const uint16_t *q;   // [n_layers][b][h_q][T][128] fp16
    float *out;          // same shape, fp32
    int32_t T, Tq;       // prompt length; tokens of it that are packed
    int32_t batch, n_q_heads;
    int32_t n_layers;    // layers of the launch; set by the launcher
    float scale_log2e;   // sm_scale * log2(e)
};
hipError_t xq_launch_prefill(const XqPrefillArgs &a, int g, int n_layers, int pack, hipStream_t s);

struct XqRingArgs {
    char *arena;
    const XqLayerDesc *layers;
    XqStrides st;
    int32_t layer0, batch, n_kv_heads, R, D;
    const uint16_t *k_src, *v_src;
    int64_t s_layer, s_batch, s_head, s_tok;
    int32_t src_tok0;  // first source token
    int32_t dst_tok0;  // absolute index of the first token written (slot = index mod R)
    int32_t n_tok;
    int32_t bh0;       // first (sequence, kv head) slice served
    int32_t ragged;    // per-sequence destination index seq_T[i] instead of dst_tok0
    int32_t seq_T[XQ_MAX_RAGGED];
};
hipError_t xq_launch_ring_write(const XqRingArgs &a, int n_layers, hipStream_t s);

struct XqDecodeArgs {
    const char *arena;
    const XqLayerDesc *layers;
    XqStrides st;
    int32_t layer0;
    int32_t batch, n_q_heads, n_kv_heads;
    int32_t R, T, Tq;
    int32_t n_splits, tiles_per_split;
    const uint16_t *q;  // [n_layers][b][h_q][D]
    float *out;         // [n_layers][b][h_q][D]
    float *ws;          // partials: [n_layers][b][h_q][n_splits + 1][D + 2]
    float scale_log2e;  // sm_scale * log2(e)
    int32_t n_launch_z;  // layers (or layer pairs) in this launch; set by the launcher
    int32_t ragged;      // per-sequence lengths seq_T[i] instead of T (Tq follows from the split rule)
    int32_t group;       // g, for the split rule
    int32_t rep, q_head0;  // query heads per kv head; first of them that this launch serves (it serves n_rep)
    int32_t reuse_codes;  // some layer of the launch reads another layer's codes (keep them in L2)
    int32_t pair_order;   // ... and the launch is a whole number of sharing groups of this many layers (0: not): deal their workgroups out side by side
    int32_t matrix;       // 0: multiply-adds on the vector ALU; 1: on the 4x4x4 fp16 matrix instruction (head_dim 128);
                          // 2: as 1 with the key phase on the 16x16x128 fp8 x fp4 instruction (2-bit keys)
    uint32_t *arrivals;   // not null: one counter per (layer or pair of the launch, sequence, kv head), zero between
                          // launches; the workgroup that arrives last merges the partials itself (no merge launch)
    XqPaging pg;
    int32_t seq_T[XQ_MAX_RAGGED];
};
#ifdef __HIPCC__
// Log-sum-exp merge of the split partials, by one workgroup of 256 threads for NH query heads:
// partial i of a head holds the unnormalised output o_i[D], its running maximum m_i (log2 domain)
// and denominator l_i (D + 2 floats; a head's n_parts partials are contiguous in ws);
//   out = sum_i o_i 2^(m_i - M) / sum_i l_i 2^(m_i - M),   M = max_i m_i.
// Built for latency, since in a one-layer call the merge is as long as the attention itself: the
// maxima and denominators of all partials are fetched in one round of loads, the factors
// 2^(m_i - M) are worked out once per partial in LDS, and every thread fetches its channel of
// eight partials (of every head) at a time before it adds them up.  The partials of an output are divided among
// 256 / D thread groups whose sums are added in group order.  The order of every sum is fixed by
// n_parts alone, so the result depends neither on which workgroup finished first
// nor on who merges (the merge kernel or the last decode workgroup to arrive).
// COHERENT: the partials were written by other workgroups of the same launch; they are read with
// device-scope loads, which are served from beyond the reader's (per-XCD, mutually incoherent) L2.
// head_of(v) = index of head v's partial table and output row.  lds: XQ_MERGE_LDS_FLOATS(NH) floats
// that no thread still reads for anything else.  Every thread of the workgroup must call.
#define XQ_MERGE_LDS_FLOATS(NH) (3 * (NH) * (XQ_MAX_SPLITS + 1) + 2 * (NH) * 256)
template <int D, int NH, bool COHERENT, typename HeadFn>
__device__ __forceinline__ void xq_merge_block(HeadFn head_of, const float *ws, float *out, int n_parts, float *lds, int tid) {
    constexpr int NP = XQ_MAX_SPLITS + 1;
    constexpr int NG = 256 / D;   // thread groups that divide the partials of an output among themselves
    float *s_m = lds, *s_l = lds + NH * NP, *s_f = lds + 2 * NH * NP, *s_num = lds + 3 * NH * NP, *s_den = s_num + NH * 256;
    auto ld = [](const float *x) -> float {
        if constexpr (COHERENT) return __hip_atomic_load(x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else return *x;
    };
    // this thread: thread group tid / D, channel tid % D of every head; its group's partials [lo, hi)
    const int per = (n_parts + NG - 1) / NG, pg = tid / D, ch = tid % D;
    const int lo = pg * per, hi = min(n_parts, lo + per);
    const float *p[NH];
#pragma unroll
    for (int v = 0; v < NH; ++v) p[v] = ws + head_of(v) * n_parts * (D + 2) + ch;
    // the first eight partials of the group travel together with the maxima and denominators: one
    // round trip to memory instead of two in the common case of at most 8 * 256 / D partials
    float x[NH][8];
#pragma unroll
    for (int v = 0; v < NH; ++v)
#pragma unroll
        for (int k = 0; k < 8; ++k) x[v][k] = (lo + k < hi) ? ld(p[v] + (lo + k) * (D + 2)) : 0.f;
    for (int idx = tid; idx < NH * n_parts; idx += 256) {
        const int v = idx / n_parts, i = idx - v * n_parts;
        const float *q = ws + (head_of(v) * n_parts + i) * (D + 2);
        s_m[v * NP + i] = ld(q + D);
        s_l[v * NP + i] = ld(q + D + 1);
    }
    __syncthreads();
    for (int idx = tid; idx < NH * n_parts; idx += 256) {
        const int v = idx / n_parts, i = idx - v * n_parts;
        float M = -INFINITY;
        for (int j = 0; j < n_parts; ++j) M = fmaxf(M, s_m[v * NP + j]);
        const float mi = s_m[v * NP + i];
        s_f[v * NP + i] = (mi == -INFINITY) ? 0.f : exp2f(mi - M);
    }
    __syncthreads();
    float num[NH], den[NH];
#pragma unroll
    for (int v = 0; v < NH; ++v) num[v] = den[v] = 0.f;
    for (int i0 = lo; i0 < hi; i0 += 8) {
        if (i0 > lo) {
#pragma unroll
            for (int v = 0; v < NH; ++v)
#pragma unroll
                for (int k = 0; k < 8; ++k) x[v][k] = (i0 + k < hi) ? ld(p[v] + (i0 + k) * (D + 2)) : 0.f;
        }
#pragma unroll
        for (int v = 0; v < NH; ++v)
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (i0 + k < hi) {
                    const float f = s_f[v * NP + i0 + k];
                    num[v] = fmaf(f, x[v][k], num[v]);
                    den[v] = fmaf(f, s_l[v * NP + i0 + k], den[v]);
                }
    }
#pragma unroll
    for (int v = 0; v < NH; ++v) {
        s_num[v * 256 + tid] = num[v];
        s_den[v * 256 + tid] = den[v];
    }
    __syncthreads();
    for (int r = tid; r < NH * D; r += 256) {
        const int v = r / D, c = r % D;
        float n_ = 0.f, d_ = 0.f;
#pragma unroll
        for (int g = 0; g < NG; ++g) {
            n_ += s_num[v * 256 + g * D + c];
            d_ += s_den[v * 256 + g * D + c];
        }
        out[head_of(v) * D + c] = n_ / d_;
    }
}
#endif

// bk, bv: bit widths of every layer in the range; pair_fused: layers come in sharing pairs;
// n_rep in {1, 2, 4}: query heads q_head0 .. q_head0 + n_rep - 1 of every kv head.
// Writes the split partials; xq_launch_merge turns them into the outputs (with a.arrivals set the
// decode launch does that itself and no merge launch follows).
hipError_t xq_launch_decode(const XqDecodeArgs &a, int D, int g, int bk, int bv, int n_rep,
                            int n_layers, int pair_fused, hipStream_t s);
hipError_t xq_launch_merge(const XqDecodeArgs &a, int D, int n_layers, hipStream_t s);

bool xq_decode_can_fuse(int D, int g, int n_rep);
bool xq_decode_has_kx(int D, int g, int bk, int n_rep, int pair_fused);

struct XqUnpackArgs {
    const char *codes;  // region of the layer that stores them
    int64_t stride;     // per slice, bytes
    int32_t n_bh, n_kv_heads, Tq, D, B, is_v;
    XqPaging pg;
    uint8_t *out;
};
hipError_t xq_launch_unpack(const XqUnpackArgs &a, hipStream_t s);

struct XqDeltaArgs {
    const char *codes_a, *codes_b;  // code regions of the two layers
    int64_t stride;                 // per slice, bytes
    XqPaging pg;
    int32_t n_kv_heads, n_bh, B;
    int32_t words_per_token;        // D * B / 32
    int32_t ragged, Tq;             // packed tokens, or per sequence from seq_Tq
    int32_t seq_Tq[XQ_MAX_RAGGED];
    unsigned long long *counts;     // 4 values
};
hipError_t xq_launch_delta_histogram(const XqDeltaArgs &a, hipStream_t s);

// Writes n (index, page) pairs into the device page table (paged caches).
struct XqPageUpdateArgs {
    int32_t *table;
    int32_t n;
    int32_t index[XQ_PAGE_UPDATES], page[XQ_PAGE_UPDATES];
};
hipError_t xq_launch_page_update(const XqPageUpdateArgs &a, hipStream_t s);
