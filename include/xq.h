/*
 * xq.h -- C ABI of the MI355X (gfx950) quantized-KV decode library.
 *
 * The library implements the data-parallel hot path of XQuant (arXiv 2510.11236):
 *   - quantize + bit-pack the K/V cache at 1 or 2 bits with asymmetric min/max
 *     group quantization (Sec. 3.1, Eq. 1-2), the data-free calibration of the
 *     stored zero-point and scale (Sec. 3.2, Eq. 12) and cross-layer sharing of
 *     the integer codes between the two layers of a pair, each layer keeping its
 *     own scale and zero-point (Sec. 3.3.3, accelerated form Sec. 3.3.4);
 *   - keys grouped per channel (g consecutive tokens of one channel), values per
 *     token (g consecutive channels of one token), the newest tokens kept in fp16
 *     (Sec. 4.1 "Baselines and Implementations": group size 32, residual 128);
 *   - decode attention that dequantizes X^ = X_Q * s^ + z^ (Sec. 3.2, 3.3.3) in
 *     registers inside q.K^T -> softmax -> .V.
 *
 * Conventions
 *   - Every "device" pointer is HIP device memory owned by the caller.  The
 *     library never allocates or frees device memory.  "host" pointers are
 *     ordinary process memory.
 *   - hip_stream is a hipStream_t passed as void* (NULL = the default stream).
 *     Kernels are enqueued on it and the call returns without waiting.  Length
 *     bookkeeping in the host handle advances at call time, so calls on one
 *     handle must be issued in program order from one thread at a time.
 *     Apart from xq_cache_create (one synchronous copy of the layer table into the arena and a
 *     clear of the arrival counters that the decode launches keep there)
 *     the calls only launch kernels: no allocation, no memset, no synchronisation.  A call may
 *     therefore be recorded by HIP stream capture; a replay repeats the recorded lengths.
 *   - fp16 = IEEE binary16.  Inputs must be finite.
 *   - Sequences of a batch may hold different numbers of tokens (prefill them one by one
 *     with xq_quantize_pack_seq; every append adds one token to each).  Ragged lengths need
 *     batch <= 256 (XQ_ERR_UNSUPPORTED beyond); a uniform batch has no such limit.
 *   - Return value: 0 (XQ_OK) or a negative XQ_ERR_* code; nothing is enqueued
 *     when an error is returned, except XQ_ERR_HIP (launch failure).
 *
 * Split rule (one policy for keys and values).  With T tokens in a layer's
 * cache, T_q = g * ceil(max(T - R, 0) / g) tokens are held as packed codes and
 * the newest r = T - T_q tokens (R - g < r <= R once T >= R) stay in an fp16
 * ring of R slots, token t in slot t mod R.  An append that finds r == R first
 * moves the oldest g ring tokens into packed form.
 *
 * Arithmetic contract (what makes the stored bytes unique).  Per group, in
 * fp32, one correctly rounded operation per step, no fused multiply-add:
 *   mn, mx = min, max of the g fp16 values;  n = 2^B - 1
 *   s  = (mx - mn) / n            (s = 0 when mx == mn)
 *   c  = clamp(rint((x - mn) / s), 0, n), ties to even; c = 0 when s == 0
 *   z^ = mn + (eta_B * n) * s ,  s^ = (1 - 2 eta_B) * s        (Eq. 12)
 * with eta_B * n and 1 - 2 eta_B formed in fp32 on the host.  s^ and z^ are
 * stored as fp16 (round to nearest even).  A layer that takes its codes from
 * the layer below computes and stores only s^ and z^ of its own data.
 *
 * Packed layout (part of the contract; all regions are per layer, then
 * [batch][kv head], 256-byte aligned, capacity max_tokens):
 *   K codes  tokens in blocks of 32.  A token's code row has W = D*B/32 words;
 *            channel d is in row word d / (32/B) at bit B * (d mod (32/B)).
 *            A block stores rows in chunks of CW = min(4, W) words:
 *            word address in block = chunk*32*CW + (t mod 32)*CW + (word mod CW),
 *            chunk = word / CW.  Block b starts at word b*32*W.
 *   V codes  tokens in blocks of 32.  Channel d belongs to slot d / CPL,
 *            CPL = D/64.  Per block a slot holds the 32*CPL codes ordered
 *            e = (t mod 32)*CPL + (d mod CPL), B bits each, LSB first, in
 *            WS = CPL*B words: word (e*B)/32, bit (e*B) mod 32.  A block is
 *            [slot 0..63][WS words]; block b starts at word b*64*WS.
 *   K meta   [token group t/g][channel d] of 4 bytes: low half s^, high half z^.
 *   V meta   [token t][channel group d/g] of 4 bytes, same halves.
 *   residual [slot t mod R][D] fp16, for K and for V.
 * Only layers that store codes have code regions.
 * In a paged cache the regions are [page][kv head] instead of [batch][kv head], a region's
 * per-slice size is that of one page, token t of a sequence is token t mod page_tokens of the
 * sequence's page number t / page_tokens, and the layouts above apply inside a page.
 */
#ifndef XQ_H
#define XQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define XQ_OK 0
#define XQ_ERR_INVALID_ARG (-1)  /* null pointer, bad shape, eta outside [0, 0.5), bad layer range */
#define XQ_ERR_UNSUPPORTED (-2)  /* head_dim / group / GQA ratio the kernels are not built for */
#define XQ_ERR_CAPACITY    (-3)  /* more than max_tokens, arena or workspace too small */
#define XQ_ERR_STATE       (-4)  /* pack on a non-empty layer, decode or unpack on an empty one */
#define XQ_ERR_HIP         (-5)  /* a HIP call or kernel launch failed */

/* Method parameters (Appendix Alg. 1 inputs kq, vq, km, vm, eta[2]; Sec. 4.1 group
 * size and residual length) and tensor shape. */
typedef struct xq_config {
    int32_t n_layers;    /* L >= 1 */
    int32_t batch;       /* b >= 1 */
    int32_t n_q_heads;   /* multiple of n_kv_heads; ratio at most 16 */
    int32_t n_kv_heads;
    int32_t head_dim;    /* D: 64 or 128 */
    int32_t group;       /* g: 32 or 64, g <= D */
    int32_t residual;    /* R: multiple of g, g <= R <= 1024 */
    int32_t max_tokens;  /* capacity per sequence */
    int32_t kq, vq;      /* layers [0, kq) hold 2-bit key codes, the others 1-bit; vq likewise for values */
    int32_t km, vm;      /* layers >= km (vm) share codes: layer l reads the codes of layer G*(l/G) + k
                          * (for the default G = 2, k = 0: the odd layer reads those of the layer below);
                          * layers below km (vm), and a trailing group without its layer k, keep their own */
    float eta1, eta2;    /* calibration parameter for 1-bit / 2-bit groups, in [0, 0.5) */
    /* Cross-layer compression variants of the ablations (Sec. 4.3 "Group Size", "Cross-Layer
     * Compression Method", Appendix E).  All zero = the accelerated pair sharing used in every
     * main experiment (G = 2, first layer dominant, gamma_0 = 1). */
    int32_t share_group;     /* G: 0 (= 2), 2, 3 or 4 consecutive layers share one code tensor */
    int32_t share_dominant;  /* k in [0, G): the layer of each group whose codes are stored */
    int32_t merge_mode;      /* XQ_MERGE_*: how the stored codes of a pair are formed (G = 2, k = 0 only) */
    float gamma0;            /* weight of the first layer's codes for XQ_MERGE_ROUND, in [0, 1] */
    /* Paged cache (both zero = every sequence owns room for max_tokens).  The packed tokens of a
     * sequence live in pages of page_tokens tokens taken from a pool of n_pages that all
     * sequences share; a page spans every layer and kv head.  max_tokens stays the limit per
     * sequence.  The fp16 rings are per sequence and not paged. */
    int32_t page_tokens;     /* 0, or a power of two >= 128 */
    int32_t n_pages;         /* pool size when page_tokens != 0 */
} xq_config;

/* merge_mode: stored codes e_m of a sharing pair from the two layers' own codes e_0, e_1 */
#define XQ_MERGE_NONE  0   /* e_m = e_0 (Sec. 3.3.4) */
#define XQ_MERGE_ROUND 1   /* e_m = floor(gamma0 e_0 + (1 - gamma0) e_1 + 1/2)  (Appendix E) */
#define XQ_MERGE_FLOOR 2   /* e_m = floor((e_0 + e_1) / 2) */
#define XQ_MERGE_CEIL  3   /* e_m = ceil((e_0 + e_1) / 2) */

typedef struct xq_cache xq_cache; /* opaque host handle */

/* Sizes the caller must provide.  arena_bytes: device memory for the whole cache.
 * workspace_bytes: device scratch for one xq_decode_attention call over all layers
 * at max_tokens.  Host pointers.  XQ_ERR_INVALID_ARG / XQ_ERR_UNSUPPORTED on a bad config
 * (including a shared pair whose two layers would have different bit widths). */
int xq_cache_bytes(const xq_config *cfg, size_t *arena_bytes, size_t *workspace_bytes);

/* Creates the host handle over a caller-owned device arena (256-byte aligned, at least
 * arena_bytes).  The arena needs no initialisation.  *out is freed with xq_cache_destroy;
 * the arena stays the caller's. */
int xq_cache_create(const xq_config *cfg, void *dev_arena, size_t arena_bytes, xq_cache **out);
void xq_cache_destroy(xq_cache *cache);

/* Sets every length to 0 (host bookkeeping only); xq_cache_reset_seq does so for one
 * sequence in every layer, e.g. to reuse a batch slot for a new request. */
int xq_cache_reset(xq_cache *cache);
int xq_cache_reset_seq(xq_cache *cache, int32_t seq);

/* Tokens held by a layer for one sequence: total T and packed T_q (host pointers, either may
 * be NULL).  xq_cache_len reports sequence 0. */
int xq_cache_len_seq(const xq_cache *cache, int32_t layer, int32_t seq, int32_t *T, int32_t *T_q);
int xq_cache_len(const xq_cache *cache, int32_t layer, int32_t *T, int32_t *T_q);

/* Prefill: quantize and pack T tokens of layers [layer0, layer0 + n_layers)
 * (Appendix Alg. 1, first loop: Quantize, or PseudoQuantize for a layer that shares).
 * k_f16, v_f16: device fp16, element (l, i, h, t, d) at
 *   base + l*strides[0] + i*strides[1] + h*strides[2] + t*strides[3] + d   (in elements),
 * l relative to layer0.  The layers must be empty (XQ_ERR_STATE otherwise); T <= max_tokens.
 * Writes codes (code-storing layers), metadata and the fp16 ring; sets the lengths to T.
 * With a merge_mode other than XQ_MERGE_NONE the range must contain both layers of every
 * sharing pair it touches (the stored codes need both), else XQ_ERR_INVALID_ARG; the same
 * holds for xq_append_token. */
int xq_quantize_pack(xq_cache *cache, int32_t layer0, int32_t n_layers, const void *k_f16,
                     const void *v_f16, const int64_t strides[4], int32_t T, void *hip_stream);

/* The same for sequences [seq0, seq0 + n_seq) only, all with T tokens: k_f16, v_f16 hold those
 * sequences, element (l, i, h, t, d) with i relative to seq0.  The other sequences are untouched. */
int xq_quantize_pack_seq(xq_cache *cache, int32_t layer0, int32_t n_layers, int32_t seq0, int32_t n_seq,
                         const void *k_f16, const void *v_f16, const int64_t strides[4], int32_t T,
                         void *hip_stream);

/* Prefill with the pack inside the prompt's own attention kernel (head_dim 128): computes the
 * causal attention of the T prompt tokens of layers [layer0, layer0 + n_layers),
 *   out[l, i, hq, t] = softmax_{j <= t}(sm_scale q[l, i, hq, t] . k[l, i, hkv, j]) v[l, i, hkv, j],
 * hkv = hq / (n_q_heads / n_kv_heads), on the fp16 K/V (the paper's procedure reads the quantized
 * cache from the first decode step on; the prompt's attention is the model's ordinary one), and
 * quantizes and packs those K/V exactly as xq_quantize_pack does (same stored bytes, same state
 * afterwards): the workgroup whose queries are the tokens of a 128-token block packs that block,
 * so that K and V come from HBM once instead of twice.
 * q_f16: device fp16 [n_layers][batch][n_q_heads][T][128], contiguous; out_f32: device fp32, same
 * shape; k_f16, v_f16, strides, T: as for xq_quantize_pack (all sequences, empty layers).
 * sm_scale must be positive and finite.
 * flags: 0, or XQ_PREFILL_NO_PACK for the attention alone (the cache is not touched).
 * XQ_ERR_UNSUPPORTED for head_dim 64 and, when packing, for caches with merged pair codes. */
#define XQ_PREFILL_NO_PACK 1
int xq_prefill_attention_pack(xq_cache *cache, int32_t layer0, int32_t n_layers, const void *q_f16, const void *k_f16,
                              const void *v_f16, const int64_t strides[4], void *out_f32, float sm_scale, int32_t T,
                              int32_t flags, void *hip_stream);

/* Decode-time append of one token per sequence to layers [layer0, layer0 + n_layers).
 * k_new_f16, v_new_f16: device fp16 [n_layers][batch][n_kv_heads][D], contiguous.
 * A sequence whose ring is full first has its oldest g tokens quantized and packed (same
 * arithmetic as xq_quantize_pack, so prefill(T) + n appends == prefill(T + n) bit for bit).
 * XQ_ERR_CAPACITY when a layer already holds max_tokens. */
int xq_append_token(xq_cache *cache, int32_t layer0, int32_t n_layers, const void *k_new_f16,
                    const void *v_new_f16, void *hip_stream);

/* Decode attention for layers [layer0, layer0 + n_layers): one query per (layer, sequence,
 * query head) against every token the layer holds (Appendix Alg. 1, second loop: codes of
 * the layer that stores them, scale and zero-point of the layer itself; then
 * softmax(sm_scale * q K^T) V).  Query head hq reads kv head hq / (n_q_heads / n_kv_heads).
 * q_f16: device fp16 [n_layers][batch][n_q_heads][D]; out_f32: device fp32, same shape.
 * dev_workspace: device scratch, at least the size xq_cache_bytes reported (less is accepted
 * when it suffices for the current lengths).  flags: 0, or XQ_DECODE_PAIR_FUSED to let one
 * workgroup serve both layers of a pair that shares key and value codes, so that the common
 * codes are fetched and unpacked once (the result is the same up to fp32 summation order; pairs
 * that share only one of the two, or not at all, run one layer per workgroup as without it).  All layers in the range must hold
 * the same, non-zero number of tokens per sequence (sequences may differ from one another), and a
 * layer outside the range whose codes a layer of the range reads must hold at least as many packed
 * tokens (XQ_ERR_STATE otherwise: e.g. the second layer of a pair decoded before the first was
 * packed, or, with share_dominant > 0, a layer decoded at a ring-flush step before the group's
 * storing layer was appended). */
#define XQ_DECODE_PAIR_FUSED 1
/* With head_dim 128 the multiply-adds run on the 4x4x4 fp16 matrix instruction (rows = query
 * heads of the kv head and layers of the pair, times the two fp16 halves of a key weight);
 * XQ_DECODE_VECTOR_ALU selects the kernels that do them on the vector ALU instead (always
 * used for head_dim 64).  Both meet the same error bound. */
#define XQ_DECODE_VECTOR_ALU 2
/* Matrix family only: 2-bit key codes are by default multiplied on the 16x16x128 fp8 x fp4 matrix
 * instruction (a 2-bit code in a nibble is the fp4 number code / 2, so one AND isolates eight codes;
 * the key weights travel as four fp8 terms, 16 significant bits).  XQ_DECODE_MATRIX_F16 keeps the
 * keys on the 4x4x4 fp16 instruction like the values (1-bit keys always are).  Same error bound. */
#define XQ_DECODE_MATRIX_F16 4
/* Who merges the split partials (per-split running maximum, denominator and output).  Either a
 * merge launch that follows the decode launch, or the decode launch itself: the workgroups of a
 * (layer, sequence, kv head) count themselves in on a counter in the cache's arena and the last to
 * arrive merges.  Both sum in the same fixed order: same results bit for bit.  By default the library
 * chooses (the decode launch merges when its workgroups run in about one round, as in a call for one
 * layer, where a second launch's fixed cost shows; a call over many layers gets the merge launch).
 * XQ_DECODE_MERGE_LAUNCH forces the merge launch, XQ_DECODE_MERGE_IN_LAUNCH the other (both:
 * XQ_ERR_INVALID_ARG).  Because of the counters, two decode calls on one cache that may merge in the
 * decode launch must not overlap in time on the GPU (calls on one stream never do); calls with
 * XQ_DECODE_MERGE_LAUNCH touch no counter and may overlap when their workspaces differ.  The counters
 * are zero whenever no decode launch is running; after an XQ_ERR_HIP from a decode call that is no
 * longer certain: create the cache anew (xq_cache_create clears them). */
#define XQ_DECODE_MERGE_LAUNCH 8
#define XQ_DECODE_MERGE_IN_LAUNCH 16
int xq_decode_attention(const xq_cache *cache, int32_t layer0, int32_t n_layers, const void *q_f16,
                        void *out_f32, float sm_scale, void *dev_workspace, size_t workspace_bytes,
                        int32_t flags, void *hip_stream);

/* For callers that cannot allocate device memory or may not pass a workspace (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): the same call as
 * xq_decode_attention, same kernels and same results, with the split partials kept in a device
 * array of XQ_STATIC_SCRATCH_BYTES that is part of the library's code object instead of a caller
 * workspace.  Each GPU the library runs on holds its own copy of that array until the process
 * ends.  The call allocates and frees nothing and clears nothing (every partial a merge reads was
 * written by the same call).  XQ_ERR_CAPACITY when the call's partials,
 *   sum over its launches of layers * batch * n_q_heads * (splits + 1) * (head_dim + 2) * 4 bytes
 * (splits <= 64, chosen by the library from the lengths), exceed XQ_STATIC_SCRATCH_BYTES: call it
 * on fewer layers at a time, or use xq_decode_attention.  All calls on one GPU share the array:
 * two calls that overlap in time on one GPU (different streams, different threads or different
 * caches) race; calls on one stream are safe.  The array's address on a device is looked up once,
 * in xq_cache_create on that device or else in the first call there. */
#define XQ_STATIC_SCRATCH_BYTES (64u << 20)
int xq_decode_attention_static(const xq_cache *cache, int32_t layer0, int32_t n_layers, const void *q_f16,
                               void *out_f32, float sm_scale, int32_t flags, void *hip_stream);

/* Test/debug: expands a layer's stored codes to one byte per element,
 * dev_codes_u8: device [batch][n_kv_heads][T_q][D].  XQ_ERR_STATE if the layer stores none or
 * its sequences differ in length. */
int xq_unpack_codes(const xq_cache *cache, int32_t layer, int32_t is_v, uint8_t *dev_codes_u8,
                    void *hip_stream);

/* Diagnostic of Sec. 3.3.2 (the analysis that motivates sharing): histogram of the absolute
 * differences |c_l - c_{l+1}| between the stored codes of two adjacent layers at the same
 * positions, over all packed tokens of all sequences.  Both layers must store their own codes
 * with one bit width and hold equal lengths (XQ_ERR_STATE otherwise).  dev_counts_u64: device,
 * 4 values (differences 0..3; 1-bit codes use the first two); overwritten. */
int xq_code_delta_histogram(const xq_cache *cache, int32_t layer, int32_t is_v, uint64_t *dev_counts_u64,
                            void *hip_stream);

/* Byte offsets of a layer's regions inside the arena (host pointer to 6 values:
 * k_codes, v_codes, k_meta, v_meta, k_residual, v_residual; a code offset is -1 for a layer
 * that stores none) and, in sizes[6], the bytes of each region per (batch, kv head) -- per
 * (page, kv head) for the four packed regions of a paged cache. */
int xq_cache_layout(const xq_cache *cache, int32_t layer, int64_t offsets[6], int64_t sizes[6]);

/* Paged caches: the pages sequence seq holds, in token order (host pointers; at most cap values
 * are written to pages, *n receives the count) and the number of free pages in the pool.
 * Pages are taken when a prefill or a ring flush needs them (XQ_ERR_CAPACITY when the pool is
 * empty; nothing is enqueued then) and go back to the pool with xq_cache_reset /
 * xq_cache_reset_seq.  XQ_ERR_STATE on a cache that is not paged. */
int xq_cache_pages(const xq_cache *cache, int32_t seq, int32_t *pages, int32_t cap, int32_t *n);
int xq_cache_free_pages(const xq_cache *cache, int32_t *n_free);

/* Test/tuning hook: forces the number of 128-token tiles per packed-token split used by
 * xq_decode_attention (0 restores the automatic plan).  Results must not depend on it beyond
 * fp32 summation order. */
void xq_debug_set_tiles_per_split(xq_cache *cache, int32_t tiles_per_split);

/* Test hook (host only, no GPU needed): the table the pack kernels use for merged pair codes
 * (Appendix E), for bits = 1 or 2: the merged code of (e_0, e_1) sits at bit position
 * bits * ((2^bits) * e_0 + e_1).  0 for a bad config or bit width. */
uint32_t xq_debug_merge_table(const xq_config *cfg, int32_t bits);

/* Equivalent bit-width (Appendix C): stored code bits per element averaged over layers and
 * over keys and values.  include_metadata = 0: the paper's figure (codes only).
 * include_metadata = 1: adds the fp16 scale/zero and the fp16 ring at T tokens per sequence. */
double xq_equivalent_bits(const xq_config *cfg, int32_t include_metadata, int32_t T);

const char *xq_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* XQ_H */
