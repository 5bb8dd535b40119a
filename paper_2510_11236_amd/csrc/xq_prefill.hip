// Causal attention of a prompt with the quantize + pack of its K/V in the same kernel (head_dim 128).
//
// The prompt's K/V are needed twice when a request arrives: by the prompt's own attention (ordinary
// causal attention on the fp16 K/V the model has just computed) and by the quantize + pack that
// builds the cache (Appendix Alg. 1, first loop).  Run one after the other, the pack reads K and V
// from HBM a second time.  Here the workgroup that owns the diagonal block of a kv head's attention
// -- the one whose last two tiles are the tokens [128 qb, 128 qb + 128) -- first brings those two
// tiles into LDS and hands them, wave by wave, to the same wave-level pack code the pack kernel uses
// (xq_pack_wave.h), so the stored bytes are bit-identical to xq_quantize_pack; its attention loop
// then finds the tiles in L2.  The pack runs before the attention state exists, not after the
// diagonal tile's products: its 32 or 64 row registers per lane would otherwise add to the 160
// registers the attention holds and cost the kernel its third wave per SIMD.
//
// Attention: one workgroup = 128 queries of one query head; wave w owns queries 32 w .. 32 w + 31.
// Key/value tiles of 64 tokens go through LDS: K row-major, V transposed.  Both products run on
// v_mfma_f32_32x32x16_f16 with the LDS tile as A and the wave's registers as B:
//   S^T = K Q^T   (rows = tokens, columns = the wave's queries; B = the lane's query row, loaded once)
//   O^T = V^T P^T (rows = channels, columns = queries; B = P^T straight from S^T's result registers:
//                  a lane of the 32x32 result holds, for its column, rows 8 i + 4 (lane / 32) + j; eight
//                  consecutive result registers are the eight k values of the lane in the next product,
//                  whose A operand is read from LDS for the same tokens in the same order -- which token
//                  sits in which k slot does not matter as long as both operands agree)
// so the query is the lane's column in both results and the online-softmax state (running maximum,
// denominator, rescale factor) is one scalar per lane.  Scores are kept in the log2 domain.
#include <type_traits>

#include "xq_internal.h"
#include "xq_pack_wave.h"

namespace {

typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PF_BM = 128;     // queries per workgroup
constexpr int PF_BN = 64;      // tokens per key/value tile
constexpr int PF_KROW = 136;   // halves per K (and row-major V) row in LDS: 128 + 8 of padding (rows stay 16-byte aligned)
constexpr int PF_VROW = 68;    // halves per row of the transposed V tile: 64 tokens + 4

template <int G>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3)))  // at most 168 registers: three workgroups per CU
void xq_prefill_kernel(XqPrefillArgs a) {
    constexpr int D = 128;
    __shared__ __attribute__((aligned(16))) _Float16 s_k[PF_BN * PF_KROW];
    __shared__ __attribute__((aligned(16))) _Float16 s_vt[D * PF_VROW];
    static_assert(D * PF_VROW >= PF_BN * PF_KROW, "the row-major V tile of the pack reuses the transposed tile's space");
    __shared__ float4 s_par[PF_BN / G][G * (D / G)];   // value-group parameters of the pack
    const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
    // Workgroups are dealt round-robin to the 8 XCDs by linear id, and each XCD has its own L2: all
    // workgroups of a kv head (its query blocks, longest first, and the query heads that share it,
    // side by side) get ids that are equal mod 8, so that one L2 sees a head's K/V tiles and the
    // workgroups of a head that run together walk them together.  (With query blocks along the grid's
    // fastest dimension every XCD fetched every head's tiles: 157 GB of HBM traffic at the 32k shape.)
    const int n_qb = (a.T + PF_BM - 1) / PF_BM;
    const int rep = a.n_q_heads / a.pk.n_kv_heads, n_kvh = a.n_layers * a.batch * a.pk.n_kv_heads;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3, per_kv = n_qb * rep;
    const int kvidx = (slot / per_kv) * 8 + xcd;
    if (kvidx >= n_kvh) return;   // (the grid is padded to a multiple of 8 kv heads)
    const int qb = n_qb - 1 - (slot % per_kv) / rep;   // longest blocks first
    const int hkv = kvidx % a.pk.n_kv_heads, bi = (kvidx / a.pk.n_kv_heads) % a.batch, lz = kvidx / (a.pk.n_kv_heads * a.batch);
    const int hq = hkv * rep + (slot % per_kv) % rep;
    const uint16_t *kg = a.pk.k_src + lz * a.pk.s_layer + bi * a.pk.s_batch + hkv * a.pk.s_head;
    const uint16_t *vg = a.pk.v_src + lz * a.pk.s_layer + bi * a.pk.s_batch + hkv * a.pk.s_head;
    const XqLayerDesc dsc = a.pk.layers[a.pk.layer0 + lz];
    // ---- quantize + pack of the block's own 128 tokens (the diagonal tiles of its attention): done by
    // the workgroup of the kv head's first query head, before the attention state takes its registers;
    // the attention loop below finds these tiles in L2
    // (a.Tq = 0 when the caller wants the attention alone: the same kernel, so that the two can be compared)
    {
        if (hq % rep == 0) {
            _Float16 *s_v = s_vt;   // the pack wants V row-major: same space as the transposed tile of the loop
            for (int t0 = qb * PF_BM; t0 < min(qb * PF_BM + PF_BM, a.Tq); t0 += PF_BN) {   // (uniform over the workgroup)
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const int idx = p * 256 + tid, n = idx >> 4, c8 = (idx & 15) * 8;
                    uint4 kv = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
                    if (t0 + n < a.T) {
                        kv = *(const uint4 *)(kg + (int64_t)(t0 + n) * a.pk.s_tok + c8);
                        vv = *(const uint4 *)(vg + (int64_t)(t0 + n) * a.pk.s_tok + c8);
                    }
                    *(uint2 *)&s_k[n * PF_KROW + c8] = make_uint2(kv.x, kv.y);
                    *(uint2 *)&s_k[n * PF_KROW + c8 + 4] = make_uint2(kv.z, kv.w);
                    *(uint2 *)&s_v[n * PF_KROW + c8] = make_uint2(vv.x, vv.y);
                    *(uint2 *)&s_v[n * PF_KROW + c8 + 4] = make_uint2(vv.z, vv.w);
                }
                __syncthreads();
                // items: key groups first, then value groups; one wave per item and round
                constexpr int NG = PF_BN / G;
                for (int item = wave; item < 2 * NG; item += 4) {
                    const bool is_v = item >= NG;
                    const int grp = is_v ? item - NG : item, gt0 = t0 + grp * G;
                    if (gt0 >= a.Tq) continue;   // (whole groups: T_q is a multiple of g)
                    const _Float16 *src = (is_v ? s_v : s_k) + (grp * G) * PF_KROW + 2 * lane;
                    uint32_t rows[G];
#pragma unroll
                    for (int t = 0; t < G; ++t) rows[t] = *(const uint32_t *)(src + t * PF_KROW);
                    int dst_tok;
                    const int64_t slice = xq_locate(a.pk.pg, a.pk.bh0 / a.pk.n_kv_heads + bi, hkv, a.pk.n_kv_heads, gt0, &dst_tok);
                    const uint32_t none[1] = {0};
                    if (!is_v) {
                        if (dsc.bk == 2) pack_keys_wave<G, 2, false>(a.pk, dsc, rows, none, lane, slice, dst_tok);
                        else pack_keys_wave<G, 1, false>(a.pk, dsc, rows, none, lane, slice, dst_tok);
                    } else {
                        if (dsc.bv == 2) pack_values_wave<G, 2, false>(a.pk, dsc, rows, none, lane, slice, dst_tok, s_par[grp], s_par[grp]);
                        else pack_values_wave<G, 1, false>(a.pk, dsc, rows, none, lane, slice, dst_tok, s_par[grp], s_par[grp]);
                    }
                }
                __syncthreads();
            }
        }
    }
    const int col = lane & 31, g2 = lane >> 5;
    const int tq = qb * PF_BM + wave * 32 + col;          // this lane's query
    // B operand of S^T = K Q^T: the lane's query row, k-step ks holds channels 16 ks + 8 g2 .. + 7
    f16x8 qreg[8];
    {
        const int tqc = min(tq, a.T - 1);
        const uint16_t *qp = a.q + ((((int64_t)lz * a.batch + bi) * a.n_q_heads + hq) * a.T + tqc) * D;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qreg[ks] = *(const f16x8 *)(qp + 16 * ks + 8 * g2);
    }
    f32x16 oacc[4];   // O^T: block c = channels 32 c .. 32 c + 31 (rows), this lane's query (column)
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[c][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const int n_kt = min((qb * PF_BM + PF_BM - 1) / PF_BN + 1, (a.T + PF_BN - 1) / PF_BN);
    // one key/value tile; masked: some (token, query) pair of the workgroup lies above the diagonal
    auto one_tile = [&](int kt, auto masked_flag) __attribute__((always_inline)) {
        constexpr bool masked = decltype(masked_flag)::value;
        const int t0 = kt * PF_BN;
        __syncthreads();   // the previous tile's readers are done
        // ---- K tile -> LDS row-major (16 bytes per thread and pass); rows past T are zero
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int idx = p * 256 + tid, n = idx >> 4, c8 = (idx & 15) * 8;
            uint4 kv = make_uint4(0, 0, 0, 0);
            if (t0 + n < a.T) kv = *(const uint4 *)(kg + (int64_t)(t0 + n) * a.pk.s_tok + c8);
            *(uint2 *)&s_k[n * PF_KROW + c8] = make_uint2(kv.x, kv.y);
            *(uint2 *)&s_k[n * PF_KROW + c8 + 4] = make_uint2(kv.z, kv.w);
        }
        // ---- V tile -> LDS transposed: lane = token, wave = 32 channels (two-byte scatter, rows contiguous per channel)
        {
            const int n = lane;
            uint4 vv[4];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                vv[p] = make_uint4(0, 0, 0, 0);
                if (t0 + n < a.T) vv[p] = *(const uint4 *)(vg + (int64_t)(t0 + n) * a.pk.s_tok + 32 * wave + 8 * p);
            }
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                const uint32_t w4[4] = {vv[p].x, vv[p].y, vv[p].z, vv[p].w};
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint16_t h = (uint16_t)(e & 1 ? w4[e / 2] >> 16 : w4[e / 2] & 0xffffu);
                    *(uint16_t *)&s_vt[(32 * wave + 8 * p + e) * PF_VROW + n] = h;
                }
            }
        }
        __syncthreads();
        // ---- S^T = K Q^T for the tile's two blocks of 32 tokens
        f32x16 sacc[2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[rb][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const f16x8 ka = *(const f16x8 *)&s_k[(32 * rb + col) * PF_KROW + 16 * ks + 8 * g2];
                sacc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ka, qreg[ks], sacc[rb], 0, 0, 0);
            }
        }
        // ---- causal mask, online softmax (log2 domain; the scale is applied inside the exponent's
        // multiply-add); result register 4 i + j = token 8 i + 4 g2 + j of the block
        float mx = -INFINITY;
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if constexpr (masked) {
                    const int tn = t0 + 32 * rb + 8 * (r >> 2) + 4 * g2 + (r & 3);
                    sacc[rb][r] = tn > tq ? -INFINITY : sacc[rb][r];
                }
                mx = fmaxf(mx, sacc[rb][r]);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx * a.scale_log2e);   // (the scale is positive) finite from the first tile on: token 0 is visible to every query
        const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
        float psum = 0.f;
        // P^T as the B operand of the second product: its k-step (rb, i) takes the lane's result
        // registers 8 i .. 8 i + 7 of block rb, i.e. tokens 32 rb + 16 i + 4 g2 + {0..3} and + 8 + {0..3}
        f16x8 pb[2][2];
#pragma unroll
        for (int rb = 0; rb < 2; ++rb)
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(sacc[rb][8 * i + j], a.scale_log2e, -m_new));
                    psum += p;
                    pb[rb][i][j] = (_Float16)p;
                }
        psum += __shfl_xor(psum, 32, 64);
        l_run = l_run * alpha + psum;
        m_run = m_new;
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {   // (wave-uniform: the running maximum of most queries stops moving early)
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[c][r] *= alpha;
        }
        // ---- O^T += V^T P^T: the A operand takes the same tokens, in the same order, from the transposed tile
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int rb = 0; rb < 2; ++rb)
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const _Float16 *vp = &s_vt[(32 * c + col) * PF_VROW + 32 * rb + 16 * i + 4 * g2];
                    const f16x4 lo = *(const f16x4 *)vp, hi = *(const f16x4 *)(vp + 8);
                    const f16x8 va = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    oacc[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(va, pb[rb][i], oacc[c], 0, 0, 0);
                }
    };
    // tiles wholly below the diagonal of every query of the workgroup need no mask
    const int n_plain = min(n_kt, (qb * PF_BM + 1) / PF_BN);
    for (int kt = 0; kt < n_plain; ++kt) one_tile(kt, std::false_type{});
    for (int kt = n_plain; kt < n_kt; ++kt) one_tile(kt, std::true_type{});
    // ---- normalise and store: register 4 i + j of block c = channel 32 c + 8 i + 4 g2 + j of this lane's query
    if (tq < a.T) {
        const float inv = 1.0f / l_run;
        float *op = a.out + ((((int64_t)lz * a.batch + bi) * a.n_q_heads + hq) * a.T + tq) * D;
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                *(float4 *)(op + 32 * c + 8 * i + 4 * g2) =
                    make_float4(oacc[c][4 * i] * inv, oacc[c][4 * i + 1] * inv, oacc[c][4 * i + 2] * inv, oacc[c][4 * i + 3] * inv);
    }
}

}  // namespace

hipError_t xq_launch_prefill(const XqPrefillArgs &a, int g, int n_layers, int pack, hipStream_t s) {
    const int n_qb = (a.T + PF_BM - 1) / PF_BM;
    const int rep = a.n_q_heads / a.pk.n_kv_heads, n_kvh = n_layers * a.batch * a.pk.n_kv_heads;
    XqPrefillArgs b = a;
    b.n_layers = n_layers;
    dim3 grid((unsigned)(8 * ((n_kvh + 7) / 8) * n_qb * rep)), block(256);
    (void)pack;   // the attention alone is the same kernel with a.Tq = 0
    if (g == 32) xq_prefill_kernel<32><<<grid, block, 0, s>>>(b);
    else if (g == 64) xq_prefill_kernel<64><<<grid, block, 0, s>>>(b);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}
