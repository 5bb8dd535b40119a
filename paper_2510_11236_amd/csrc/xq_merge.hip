// Merge of the split-K partials and the dispatch onto the per-configuration decode kernels.
#include "xq_internal.h"

namespace {

// The merge as a launch of its own: one workgroup per query head.
template <int D>
__global__ __launch_bounds__(256) void xq_merge_kernel(const float *ws, float *out, int n_parts) {
    __shared__ float s_merge[XQ_MERGE_LDS_FLOATS(1)];
    const int64_t head = blockIdx.x;
    xq_merge_block<D, 1, false>([&](int) { return head; }, ws, out, n_parts, s_merge, threadIdx.x);
}

}  // namespace

#define XQ_DECL(D, G, K, V) \
    hipError_t xq_launch_decode_##D##_##G##_##K##V(const XqDecodeArgs &, int, int, int, hipStream_t);
#define XQ_DECL_BITS(D, G) XQ_DECL(D, G, 1, 1) XQ_DECL(D, G, 1, 2) XQ_DECL(D, G, 2, 1) XQ_DECL(D, G, 2, 2)
XQ_DECL_BITS(128, 32)
XQ_DECL_BITS(128, 64)
XQ_DECL_BITS(64, 32)
XQ_DECL_BITS(64, 64)
// the kernels with the fp8 x fp4 key phase (head_dim 128, 2-bit keys)
#define XQ_DECL_KX(G, V) hipError_t xq_launch_decode_kx_128_##G##_2##V(const XqDecodeArgs &, int, int, int, hipStream_t);
XQ_DECL_KX(32, 1) XQ_DECL_KX(32, 2) XQ_DECL_KX(64, 1) XQ_DECL_KX(64, 2)

hipError_t xq_launch_decode(const XqDecodeArgs &a, int D, int g, int bk, int bv, int n_rep, int n_layers,
                            int pair_fused, hipStream_t s) {
    hipError_t e = hipErrorInvalidValue;
    if (a.matrix == 2 && xq_decode_has_kx(D, g, bk, n_rep, pair_fused)) {
        if (g == 32 && bv == 1) return xq_launch_decode_kx_128_32_21(a, n_rep, n_layers, pair_fused, s);
        if (g == 32 && bv == 2) return xq_launch_decode_kx_128_32_22(a, n_rep, n_layers, pair_fused, s);
        if (g == 64 && bv == 1) return xq_launch_decode_kx_128_64_21(a, n_rep, n_layers, pair_fused, s);
        if (g == 64 && bv == 2) return xq_launch_decode_kx_128_64_22(a, n_rep, n_layers, pair_fused, s);
    }
#define XQ_CASE(DD, GG, K, V) \
    if (D == DD && g == GG && bk == K && bv == V) e = xq_launch_decode_##DD##_##GG##_##K##V(a, n_rep, n_layers, pair_fused, s);
#define XQ_CASE_BITS(DD, GG) XQ_CASE(DD, GG, 1, 1) XQ_CASE(DD, GG, 1, 2) XQ_CASE(DD, GG, 2, 1) XQ_CASE(DD, GG, 2, 2)
    XQ_CASE_BITS(128, 32)
    XQ_CASE_BITS(128, 64)
    XQ_CASE_BITS(64, 32)
    XQ_CASE_BITS(64, 64)
    return e;
}

hipError_t xq_launch_merge(const XqDecodeArgs &a, int D, int n_layers, hipStream_t s) {
    const int64_t heads = (int64_t)n_layers * a.batch * a.n_q_heads;
    if (D == 128) xq_merge_kernel<128><<<dim3((unsigned)heads), dim3(256), 0, s>>>(a.ws, a.out, a.n_splits + 1);
    else xq_merge_kernel<64><<<dim3((unsigned)heads), dim3(256), 0, s>>>(a.ws, a.out, a.n_splits + 1);
    return hipGetLastError();
}

// Whether a kernel with the fp8 x fp4 key phase is built for this shape: head_dim 128, 2-bit keys, and
// at least four (query head, layer of a fused pair) combinations sharing the codes of a kv head.
bool xq_decode_has_kx(int D, int g, int bk, int n_rep, int pair_fused) {
    if (D != 128 || bk != 2) return false;
    if (pair_fused) return n_rep >= 2 && xq_decode_can_fuse(D, g, n_rep);
    return n_rep >= 4;
}

// Whether xq_launch_decode can serve a sharing pair with one workgroup for this shape.
bool xq_decode_can_fuse(int D, int g, int n_rep) {
    return 2 * n_rep * (XQ_TILE_TOKENS / g) <= 16 && (D == 128 || n_rep == 1);
}
