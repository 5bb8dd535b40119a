// Host layer of libxq: configuration checks, arena carving, length bookkeeping and
// the dispatch of the C-ABI entry points declared in include/xq.h onto the kernels.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>

#include "xq_internal.h"

// Split partials of xq_decode_attention_static: one array per GPU, held from the load of the
// library's code on that GPU until the process ends.  In host code the name is only a handle for
// hipGetSymbolAddress; kernels get the address that call returned.
static __device__ __align__(256) unsigned char scratch[XQ_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices];  // address of `scratch` on each device, once resolved there

// Address of the current device's copy of `scratch` (resolved once per device, with that device
// current).  The first resolution on a device may load the library's code there, so it is done
// from xq_cache_create as well, outside any stream capture.
int static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return XQ_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return XQ_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return XQ_OK;
}

inline int64_t align256(int64_t x) { return (x + 255) & ~int64_t(255); }

inline int bits_of(const xq_config &c, int l, bool is_v) { return l < (is_v ? c.vq : c.kq) ? 2 : 1; }
inline int group_size(const xq_config &c) { return c.share_group ? c.share_group : 2; }
// The layer whose codes layer l reads.  Appendix Alg. 1 (with the dequantization loop's
// conditions) for pairs: below the sharing start, or as the dominant layer of its group, a layer
// reads its own; otherwise those of layer k of its group of G consecutive layers (Sec. 4.3
// "Group Size": G in {2,3,4}, selection index k).  A trailing group that lacks layer k keeps
// per-layer codes.
inline int code_layer(const xq_config &c, int l, bool is_v) {
    if (l < (is_v ? c.vm : c.km)) return l;
    const int G = group_size(c);
    const int cl = G * (l / G) + c.share_dominant;
    return cl < c.n_layers ? cl : l;
}
inline bool stores_codes(const xq_config &c, int l, bool is_v) { return code_layer(c, l, is_v) == l; }
// Stored codes of layer l are merged with those of layer l + 1 (Appendix E; pairs only).
inline bool merges_next(const xq_config &c, int l, bool is_v) {
    return c.merge_mode != XQ_MERGE_NONE && l + 1 < c.n_layers && stores_codes(c, l, is_v) &&
           code_layer(c, l + 1, is_v) == l;
}

// e_m for every (e_0, e_1): entry 4*e_0 + e_1 at bits [2i, 2i+1] (2-bit codes), entry 2*e_0 + e_1
// at bit i (1-bit codes).
// Weighted average with rounding, built from the interval table of Appendix E rather than from the
// average itself: with delta = e_0 - e_1 > 0 the merged code is e_1 + c, where c counts the
// interval bounds (2k - 1) / (2 delta), k = 1 .. delta, that gamma_0 has passed ((1/2); (1/4, 3/4);
// (1/6, 1/2, 5/6)); for delta < 0 the two layers swap roles, with gamma_1 = 1 - gamma_0.  The paper
// leaves gamma_0 exactly on a bound open; here such a value belongs to the interval above it.
// Floor / ceil: the two ways of rounding the plain mean at gamma_0 = 1/2.
uint32_t merge_lut(const xq_config &c, int B) {
    const int n = (1 << B) - 1;
    const double g0 = (double)c.gamma0, g1 = 1.0 - g0;
    auto passed = [](double g, int delta) {  // bounds of the delta row of the table that g has reached
        int cnt = 0;
        for (int k = 1; k <= delta; ++k)
            if (g * (2 * delta) >= (double)(2 * k - 1)) ++cnt;
        return cnt;
    };
    uint32_t lut = 0;
    for (int e0 = 0; e0 <= n; ++e0)
        for (int e1 = 0; e1 <= n; ++e1) {
            int em = e0;
            if (c.merge_mode == XQ_MERGE_ROUND) em = e0 >= e1 ? e1 + passed(g0, e0 - e1) : e0 + passed(g1, e1 - e0);
            else if (c.merge_mode == XQ_MERGE_FLOOR) em = (e0 + e1) >> 1;
            else if (c.merge_mode == XQ_MERGE_CEIL) em = (e0 + e1 + 1) >> 1;
            lut |= (uint32_t)em << (B * ((n + 1) * e0 + e1));
        }
    return lut;
}

int check_config(const xq_config *c) {
    if (!c) return XQ_ERR_INVALID_ARG;
    if (c->n_layers < 1 || c->n_layers > XQ_MAX_LAYERS || c->batch < 1 || c->n_kv_heads < 1 ||
        c->n_q_heads < 1 || c->max_tokens < 1)
        return XQ_ERR_INVALID_ARG;
    if (c->n_q_heads % c->n_kv_heads) return XQ_ERR_INVALID_ARG;
    if ((int64_t)c->batch * c->n_kv_heads > 65535) return XQ_ERR_UNSUPPORTED;  // one grid dimension of the pack kernels
    if (c->kq < 0 || c->vq < 0 || c->km < 0 || c->vm < 0) return XQ_ERR_INVALID_ARG;
    if (!(c->eta1 >= 0.0f && c->eta1 < 0.5f) || !(c->eta2 >= 0.0f && c->eta2 < 0.5f)) return XQ_ERR_INVALID_ARG;
    if (c->head_dim != 64 && c->head_dim != 128) return XQ_ERR_UNSUPPORTED;
    if (c->group != 32 && c->group != 64) return XQ_ERR_UNSUPPORTED;
    if (c->group > c->head_dim) return XQ_ERR_UNSUPPORTED;
    if (c->residual < c->group || c->residual % c->group || c->residual > 1024) return XQ_ERR_INVALID_ARG;
    int rep = c->n_q_heads / c->n_kv_heads;
    if (rep > XQ_MAX_REP) return XQ_ERR_UNSUPPORTED;
    const int G = group_size(*c);
    if (G < 2 || G > 4) return XQ_ERR_INVALID_ARG;
    if (c->share_dominant < 0 || c->share_dominant >= G) return XQ_ERR_INVALID_ARG;
    if (c->merge_mode < XQ_MERGE_NONE || c->merge_mode > XQ_MERGE_CEIL) return XQ_ERR_INVALID_ARG;
    if (c->merge_mode != XQ_MERGE_NONE && (G != 2 || c->share_dominant != 0)) return XQ_ERR_INVALID_ARG;
    if (c->merge_mode == XQ_MERGE_ROUND && !(c->gamma0 >= 0.0f && c->gamma0 <= 1.0f)) return XQ_ERR_INVALID_ARG;
    if (c->page_tokens != 0) {
        if (c->page_tokens < XQ_TILE_TOKENS || (c->page_tokens & (c->page_tokens - 1)) || c->n_pages < 1)
            return XQ_ERR_INVALID_ARG;
        if ((int64_t)c->n_pages * c->n_kv_heads > INT32_MAX) return XQ_ERR_UNSUPPORTED;
    } else if (c->n_pages != 0) {
        return XQ_ERR_INVALID_ARG;
    }
    // the layers that share one code tensor must have one bit width
    for (int l = 0; l < c->n_layers; ++l) {
        if (bits_of(*c, l, false) != bits_of(*c, code_layer(*c, l, false), false)) return XQ_ERR_INVALID_ARG;
        if (bits_of(*c, l, true) != bits_of(*c, code_layer(*c, l, true), true)) return XQ_ERR_INVALID_ARG;
    }
    return XQ_OK;
}

struct Carve {
    XqStrides st;
    int64_t total;
    int64_t page_table;  // byte offset of the device page table (paged caches)
    int64_t arrivals;    // byte offset and size of the decode launches' arrival counters
    int64_t arrivals_bytes;
    int32_t max_pages;   // its width: pages a sequence can hold
};

// Lays the regions out; fills descs when not null.
Carve carve(const xq_config &c, XqLayerDesc *descs) {
    Carve r;
    const int64_t D = c.head_dim, g = c.group, R = c.residual;
    const int64_t maxTq = xq_quantized_len(c.max_tokens, c.group, c.residual);
    const int64_t nbh = (int64_t)c.batch * c.n_kv_heads;  // ring slices
    const bool paged = c.page_tokens != 0;
    const int64_t cap = paged ? c.page_tokens : maxTq;     // tokens per packed slice
    const int64_t nsl = paged ? (int64_t)c.n_pages * c.n_kv_heads : nbh;  // packed slices
    r.st.k_codes2 = cap * D * 2 / 8;
    r.st.k_codes1 = cap * D * 1 / 8;
    r.st.v_codes2 = r.st.k_codes2;
    r.st.v_codes1 = r.st.k_codes1;
    r.st.k_meta = (cap / g) * D * 4;
    r.st.v_meta = cap * (D / g) * 4;
    r.st.res = R * D * 2;
    int64_t off = align256((int64_t)sizeof(XqLayerDesc) * c.n_layers);
    r.max_pages = paged ? (int32_t)((maxTq + c.page_tokens - 1) / c.page_tokens) : 0;
    r.page_table = off;
    if (paged) off = align256(off + (int64_t)c.batch * (r.max_pages > 0 ? r.max_pages : 1) * 4);
    r.arrivals = off;
    r.arrivals_bytes = (int64_t)c.n_layers * nbh * 4;
    off = align256(off + r.arrivals_bytes);
    for (int l = 0; l < c.n_layers; ++l) {
        XqLayerDesc d;
        d.bk = bits_of(c, l, false);
        d.bv = bits_of(c, l, true);
        d.k_store = stores_codes(c, l, false);
        d.v_store = stores_codes(c, l, true);
        d.k_merge = merges_next(c, l, false);
        d.v_merge = merges_next(c, l, true);
        d.k_codes = d.v_codes = 0;  // a sharing layer's are filled in below
        if (d.k_store) {
            d.k_codes = off;
            off = align256(off + nsl * (d.bk == 2 ? r.st.k_codes2 : r.st.k_codes1));
        }
        if (d.v_store) {
            d.v_codes = off;
            off = align256(off + nsl * (d.bv == 2 ? r.st.v_codes2 : r.st.v_codes1));
        }
        d.k_meta = off;
        off = align256(off + nsl * r.st.k_meta);
        d.v_meta = off;
        off = align256(off + nsl * r.st.v_meta);
        d.k_res = off;
        off = align256(off + nbh * r.st.res);
        d.v_res = off;
        off = align256(off + nbh * r.st.res);
        if (descs) descs[l] = d;
    }
    if (descs)
        for (int l = 0; l < c.n_layers; ++l) {
            if (!descs[l].k_store) descs[l].k_codes = descs[code_layer(c, l, false)].k_codes;
            if (!descs[l].v_store) descs[l].v_codes = descs[code_layer(c, l, true)].v_codes;
        }
    r.total = off;
    return r;
}

int max_splits_for(int Tq) {
    int tiles = (Tq + XQ_TILE_TOKENS - 1) / XQ_TILE_TOKENS;
    return tiles > XQ_MAX_SPLITS ? XQ_MAX_SPLITS : tiles;
}

size_t workspace_floats(const xq_config &c, int n_layers, int n_splits) {
    return (size_t)n_layers * c.batch * c.n_q_heads * (size_t)(n_splits + 1) * (c.head_dim + 2);
}

// Split plan: whole tiles of 128 tokens per split, equal-sized splits.  work_items = the
// (layer or fused pair, sequence, kv head) slices the call's launches cover; each becomes n
// workgroups of t tiles.  A workgroup pays a fixed cost (launch, prologue, cross-wave combine,
// partial write and its share of the merge: about 8 tiles' worth) and the chip holds about 1024
// workgroups at once (256 CUs x 4).  Workgroups are dealt out as slots free up, so a launch takes
// about
//   (t + 8) * (rounds + 0.2),   rounds = items * n / 1024, at least 1,
// tile times: the work spread over the slots (a launch that does not fill them still takes one
// workgroup's time; a small number of rounds is rounded up towards a whole number, because equal
// workgroups finish together) plus a fifth of a workgroup of ragged tail.  The constants are fitted to
// sweeps of n on the 4k, 16k, 32k and 256k configurations, all layers per call and one layer per
// call.  The plan minimises that over n, with at most XQ_MAX_SPLITS splits.
// Workgroups of the decode kernel that one CU holds at a time: set by the registers of the
// kernel variant (n_rep query heads per kv head in the pass; a fused pair doubles the heads).
int decode_wgs_per_cu(int matrix, int n_rep, bool fused, int g, int bk, int bv) {
    const int nv = n_rep * (fused ? 2 : 1);
    if (matrix == 2 && xq_decode_has_kx(128, g, bk, n_rep, fused)) return 2;
    if (matrix) {
        if (nv <= 2 || (n_rep == 4 && !fused && g == 64 && bk + bv < 4)) return 4;
        return nv <= 4 ? 3 : 2;
    }
    return nv <= 2 ? 4 : (nv <= 4 ? 3 : 2);
}

void plan_splits(const xq_cache *cache, int Tq, int64_t work_items, int slots, int *n_splits, int *tiles_per_split) {
    int tiles = (Tq + XQ_TILE_TOKENS - 1) / XQ_TILE_TOKENS;
    if (tiles == 0) {
        *n_splits = 0;
        *tiles_per_split = 4;
        return;
    }
    int tps;
    if (cache->tiles_per_split_override > 0) {
        tps = cache->tiles_per_split_override;
    } else {
        // splits of at least 16 tiles (four per wave); shorter ones, down to one tile per wave,
        // only while the launch would otherwise stay below 256 workgroups
        int min_t = 16;
        while (min_t > 4 && work_items * ((tiles + min_t - 1) / min_t) < 256) min_t /= 2;
        int most = (tiles + min_t - 1) / min_t;
        if (most > XQ_MAX_SPLITS) most = XQ_MAX_SPLITS;
        double best_cost = -1.0;
        tps = tiles;
        for (int n = 1; n <= most; ++n) {
            const int t = (tiles + n - 1) / n;
            const double fill = (double)work_items * ((tiles + t - 1) / t) / slots;
            // few rounds come in whole numbers (equal workgroups finish together); many rounds even out
            const double whole = ceil(fill), blend = fill < 8.0 ? 1.0 - fill / 8.0 : 0.0;
            const double rounds = fill <= 1.0 ? 1.0 : fill + (whole - fill) * blend;
            const double cost = (t + 8) * (rounds + 0.2);
            if (best_cost < 0 || cost < best_cost) {
                best_cost = cost;
                tps = t;
            }
        }
    }
    int min_tps = (tiles + XQ_MAX_SPLITS - 1) / XQ_MAX_SPLITS;
    if (tps < min_tps) tps = min_tps;
    *tiles_per_split = tps;
    *n_splits = (tiles + tps - 1) / tps;
}

bool range_ok(const xq_cache *c, int layer0, int n) {
    return c && layer0 >= 0 && n >= 1 && layer0 + n <= c->cfg.n_layers;
}

}  // namespace

extern "C" {

const char *xq_strerror(int code) {
    switch (code) {
        case XQ_OK: return "ok";
        case XQ_ERR_INVALID_ARG: return "invalid argument";
        case XQ_ERR_UNSUPPORTED: return "unsupported head_dim / group / head ratio";
        case XQ_ERR_CAPACITY: return "capacity exceeded (max_tokens, arena or workspace)";
        case XQ_ERR_STATE: return "call not valid in the cache's current state";
        case XQ_ERR_HIP: return "HIP call or kernel launch failed";
        default: return "unknown error code";
    }
}

int xq_cache_bytes(const xq_config *cfg, size_t *arena_bytes, size_t *workspace_bytes) {
    int rc = check_config(cfg);
    if (rc) return rc;
    Carve cv = carve(*cfg, nullptr);
    if (arena_bytes) *arena_bytes = (size_t)cv.total;
    if (workspace_bytes) {
        int maxTq = xq_quantized_len(cfg->max_tokens, cfg->group, cfg->residual);
        *workspace_bytes = workspace_floats(*cfg, cfg->n_layers, max_splits_for(maxTq)) * sizeof(float);
    }
    return XQ_OK;
}

int xq_cache_create(const xq_config *cfg, void *dev_arena, size_t arena_bytes, xq_cache **out) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!dev_arena || !out || ((uintptr_t)dev_arena & 255)) return XQ_ERR_INVALID_ARG;
    xq_cache *c = new (std::nothrow) xq_cache();
    if (!c) return XQ_ERR_INVALID_ARG;
    c->cfg = *cfg;
    c->len.assign((size_t)cfg->n_layers * cfg->batch, 0);
    Carve cv = carve(*cfg, c->layers);
    if ((size_t)cv.total > arena_bytes) {
        delete c;
        return XQ_ERR_CAPACITY;
    }
    c->strides = cv.st;
    c->arena = (char *)dev_arena;
    c->arena_bytes = arena_bytes;
    c->dev_layers = (XqLayerDesc *)dev_arena;
    c->paging.table = nullptr;
    c->paging.shift = 0;
    c->paging.max_pages = cv.max_pages;
    if (cfg->page_tokens != 0) {
        c->paging.table = (const int32_t *)(c->arena + cv.page_table);
        while ((1 << c->paging.shift) < cfg->page_tokens) ++c->paging.shift;
        c->page_table.assign((size_t)cfg->batch * cv.max_pages, -1);
        c->pages_used.assign(cfg->batch, 0);
        c->want.assign(cfg->batch, 0);
        for (int p = cfg->n_pages - 1; p >= 0; --p) c->free_pages.push_back(p);  // page 0 is handed out first
    }
    c->arrivals = (uint32_t *)(c->arena + cv.arrivals);
    if (hipMemcpy(c->dev_layers, c->layers, sizeof(XqLayerDesc) * cfg->n_layers, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemset(c->arrivals, 0, (size_t)cv.arrivals_bytes) != hipSuccess) {
        delete c;
        return XQ_ERR_HIP;
    }
    void *unused = nullptr;
    (void)static_scratch(&unused);  // resolve this device's scratch array now; a failure is reported by the call that needs it
    *out = c;
    return XQ_OK;
}

void xq_cache_destroy(xq_cache *cache) { delete cache; }

// lengths of layer l, one per sequence
static inline int32_t *len_row(xq_cache *c, int l) { return c->len.data() + (size_t)l * c->cfg.batch; }
static inline const int32_t *len_row(const xq_cache *c, int l) { return c->len.data() + (size_t)l * c->cfg.batch; }
static bool row_uniform(const xq_cache *c, int l) {
    const int32_t *r = len_row(c, l);
    for (int i = 1; i < c->cfg.batch; ++i)
        if (r[i] != r[0]) return false;
    return true;
}
static bool rows_equal(const xq_cache *c, int l0, int l1) {
    return memcmp(len_row(c, l0), len_row(c, l1), sizeof(int32_t) * c->cfg.batch) == 0;
}

// ---- paged caches: pages are handed out in the order sequences need them
static void release_pages(xq_cache *c, int seq) {
    int32_t *row = c->page_table.data() + (size_t)seq * c->paging.max_pages;
    for (int k = c->pages_used[seq] - 1; k >= 0; --k) {
        c->free_pages.push_back(row[k]);
        row[k] = -1;
    }
    c->pages_used[seq] = 0;
}
static int pages_for(const xq_cache *c, int Tq) { return (Tq + c->cfg.page_tokens - 1) >> c->paging.shift; }
// Pages that sequences seq0 .. seq0 + n_seq - 1 still lack for new_Tq[i] packed tokens each.
static int64_t pages_missing(const xq_cache *c, int seq0, int n_seq, const int32_t *new_Tq) {
    int64_t need = 0;
    for (int i = 0; i < n_seq; ++i) need += std::max(0, pages_for(c, new_Tq[i]) - c->pages_used[seq0 + i]);
    return need;
}
// Takes the missing pages (the caller has checked that the pool holds them) and enqueues the
// device table updates on the stream, ahead of the kernels that will use them.
static int take_pages(xq_cache *c, int seq0, int n_seq, const int32_t *new_Tq, hipStream_t s) {
    XqPageUpdateArgs u;
    u.table = const_cast<int32_t *>(c->paging.table);
    u.n = 0;
    for (int i = 0; i < n_seq; ++i) {
        const int seq = seq0 + i, want = pages_for(c, new_Tq[i]);
        int32_t *row = c->page_table.data() + (size_t)seq * c->paging.max_pages;
        while (c->pages_used[seq] < want) {
            const int slot = c->pages_used[seq]++;
            row[slot] = c->free_pages.back();
            c->free_pages.pop_back();
            u.index[u.n] = seq * c->paging.max_pages + slot;
            u.page[u.n] = row[slot];
            if (++u.n == XQ_PAGE_UPDATES) {
                if (xq_launch_page_update(u, s) != hipSuccess) return XQ_ERR_HIP;
                u.n = 0;
            }
        }
    }
    return xq_launch_page_update(u, s) == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

int xq_cache_pages(const xq_cache *cache, int32_t seq, int32_t *pages, int32_t cap, int32_t *n) {
    if (!cache || seq < 0 || seq >= cache->cfg.batch || cap < 0 || (cap > 0 && !pages)) return XQ_ERR_INVALID_ARG;
    if (!cache->paging.table) return XQ_ERR_STATE;
    const int used = cache->pages_used[seq];
    for (int k = 0; k < used && k < cap; ++k) pages[k] = cache->page_table[(size_t)seq * cache->paging.max_pages + k];
    if (n) *n = used;
    return XQ_OK;
}

int xq_cache_free_pages(const xq_cache *cache, int32_t *n_free) {
    if (!cache || !n_free) return XQ_ERR_INVALID_ARG;
    if (!cache->paging.table) return XQ_ERR_STATE;
    *n_free = (int32_t)cache->free_pages.size();
    return XQ_OK;
}

int xq_cache_reset(xq_cache *cache) {
    if (!cache) return XQ_ERR_INVALID_ARG;
    std::fill(cache->len.begin(), cache->len.end(), 0);
    for (int i = 0; i < cache->cfg.batch && cache->paging.table; ++i) release_pages(cache, i);
    return XQ_OK;
}

int xq_cache_reset_seq(xq_cache *cache, int32_t seq) {
    if (!cache || seq < 0 || seq >= cache->cfg.batch) return XQ_ERR_INVALID_ARG;
    for (int l = 0; l < cache->cfg.n_layers; ++l) len_row(cache, l)[seq] = 0;
    if (cache->paging.table) release_pages(cache, seq);
    return XQ_OK;
}

int xq_cache_len_seq(const xq_cache *cache, int32_t layer, int32_t seq, int32_t *T, int32_t *T_q) {
    if (!range_ok(cache, layer, 1) || seq < 0 || seq >= cache->cfg.batch) return XQ_ERR_INVALID_ARG;
    const int t = len_row(cache, layer)[seq];
    if (T) *T = t;
    if (T_q) *T_q = xq_quantized_len(t, cache->cfg.group, cache->cfg.residual);
    return XQ_OK;
}

int xq_cache_len(const xq_cache *cache, int32_t layer, int32_t *T, int32_t *T_q) {
    return xq_cache_len_seq(cache, layer, 0, T, T_q);
}

int xq_cache_layout(const xq_cache *cache, int32_t layer, int64_t offsets[6], int64_t sizes[6]) {
    if (!range_ok(cache, layer, 1) || !offsets || !sizes) return XQ_ERR_INVALID_ARG;
    const XqLayerDesc &d = cache->layers[layer];
    const XqStrides &s = cache->strides;
    offsets[0] = d.k_store ? d.k_codes : -1;
    offsets[1] = d.v_store ? d.v_codes : -1;
    offsets[2] = d.k_meta;
    offsets[3] = d.v_meta;
    offsets[4] = d.k_res;
    offsets[5] = d.v_res;
    sizes[0] = d.bk == 2 ? s.k_codes2 : s.k_codes1;
    sizes[1] = d.bv == 2 ? s.v_codes2 : s.v_codes1;
    sizes[2] = s.k_meta;
    sizes[3] = s.v_meta;
    sizes[4] = s.res;
    sizes[5] = s.res;
    return XQ_OK;
}

void xq_debug_set_tiles_per_split(xq_cache *cache, int32_t tiles_per_split) {
    if (cache) cache->tiles_per_split_override = tiles_per_split;
}

uint32_t xq_debug_merge_table(const xq_config *cfg, int32_t bits) {
    if (check_config(cfg) != XQ_OK || (bits != 1 && bits != 2)) return 0;
    return merge_lut(*cfg, bits);
}

// With merging, the stored codes of a pair need both layers in one call.
static bool merge_range_ok(const xq_config &c, int layer0, int n_layers) {
    if (c.merge_mode == XQ_MERGE_NONE) return true;
    for (int l = layer0; l < layer0 + n_layers; ++l)
        for (int v = 0; v < 2; ++v) {
            if (merges_next(c, l, v) && l + 1 >= layer0 + n_layers) return false;
            if (l == layer0 && l > 0 && merges_next(c, l - 1, v)) return false;
        }
    return true;
}

static void fill_pack_consts(const xq_config &c, XqPackArgs &a) {
    a.merge = c.merge_mode != XQ_MERGE_NONE;
    a.lut1 = merge_lut(c, 1);
    a.lut2 = merge_lut(c, 2);
    // eta_B * (2^B - 1) and 1 - 2 eta_B, each one fp32 operation (Eq. 12)
    volatile float e1 = c.eta1, e2 = c.eta2;
    volatile float t1 = 2.0f * e1, t2 = 2.0f * e2;
    a.c1_1 = e1 * 1.0f;
    a.c2_1 = 1.0f - t1;
    a.c1_2 = e2 * 3.0f;
    a.c2_2 = 1.0f - t2;
}

int xq_quantize_pack_seq(xq_cache *cache, int32_t layer0, int32_t n_layers, int32_t seq0, int32_t n_seq,
                         const void *k_f16, const void *v_f16, const int64_t strides[4], int32_t T,
                         void *hip_stream) {
    if (!range_ok(cache, layer0, n_layers) || !k_f16 || !v_f16 || !strides || T < 1) return XQ_ERR_INVALID_ARG;
    const xq_config &c = cache->cfg;
    if (seq0 < 0 || n_seq < 1 || seq0 + n_seq > c.batch) return XQ_ERR_INVALID_ARG;
    if (T > c.max_tokens) return XQ_ERR_CAPACITY;
    for (int i = 0; i < 4; ++i)
        if (strides[i] < 0 || strides[i] % 8) return XQ_ERR_INVALID_ARG;
    if (strides[3] < c.head_dim || ((uintptr_t)k_f16 & 15) || ((uintptr_t)v_f16 & 15)) return XQ_ERR_INVALID_ARG;
    if (!merge_range_ok(c, layer0, n_layers)) return XQ_ERR_INVALID_ARG;
    for (int l = layer0; l < layer0 + n_layers; ++l)
        for (int i = seq0; i < seq0 + n_seq; ++i)
            if (len_row(cache, l)[i] != 0) return XQ_ERR_STATE;
    hipStream_t s = (hipStream_t)hip_stream;
    const int Tq = xq_quantized_len(T, c.group, c.residual);
    if (cache->paging.table && Tq > 0) {
        int32_t *want = cache->want.data();
        for (int i = 0; i < n_seq; ++i) want[i] = Tq;
        if (pages_missing(cache, seq0, n_seq, want) > (int64_t)cache->free_pages.size()) return XQ_ERR_CAPACITY;
        int rc = take_pages(cache, seq0, n_seq, want, s);
        if (rc) return rc;
    }
    if (Tq > 0) {
        XqPackArgs a;
        memset(&a, 0, sizeof(a));
        a.arena = cache->arena;
        a.layers = cache->dev_layers;
        a.st = cache->strides;
        a.layer0 = layer0;
        a.batch = n_seq;
        a.bh0 = seq0 * c.n_kv_heads;
        a.n_kv_heads = c.n_kv_heads;
        a.R = c.residual;
        a.k_src = (const uint16_t *)k_f16;
        a.v_src = (const uint16_t *)v_f16;
        a.s_layer = strides[0];
        a.s_batch = strides[1];
        a.s_head = strides[2];
        a.s_tok = strides[3];
        a.from_ring = 0;
        a.src_tok0 = 0;
        a.dst_tok0 = 0;
        a.pg = cache->paging;
        a.n_groups = Tq / c.group;
        fill_pack_consts(c, a);
        if (xq_launch_pack(a, c.head_dim, c.group, n_layers, s) != hipSuccess) return XQ_ERR_HIP;
    }
    XqRingArgs r;
    memset(&r, 0, sizeof(r));
    r.arena = cache->arena;
    r.layers = cache->dev_layers;
    r.st = cache->strides;
    r.layer0 = layer0;
    r.batch = n_seq;
    r.bh0 = seq0 * c.n_kv_heads;
    r.n_kv_heads = c.n_kv_heads;
    r.R = c.residual;
    r.D = c.head_dim;
    r.k_src = (const uint16_t *)k_f16;
    r.v_src = (const uint16_t *)v_f16;
    r.s_layer = strides[0];
    r.s_batch = strides[1];
    r.s_head = strides[2];
    r.s_tok = strides[3];
    r.src_tok0 = Tq;
    r.dst_tok0 = Tq;
    r.n_tok = T - Tq;
    if (xq_launch_ring_write(r, n_layers, s) != hipSuccess) return XQ_ERR_HIP;
    for (int l = layer0; l < layer0 + n_layers; ++l)
        for (int i = seq0; i < seq0 + n_seq; ++i) len_row(cache, l)[i] = T;
    return XQ_OK;
}

int xq_prefill_attention_pack(xq_cache *cache, int32_t layer0, int32_t n_layers, const void *q_f16, const void *k_f16,
                              const void *v_f16, const int64_t strides[4], void *out_f32, float sm_scale, int32_t T,
                              int32_t flags, void *hip_stream) {
    if (!range_ok(cache, layer0, n_layers) || !q_f16 || !k_f16 || !v_f16 || !out_f32 || !strides || T < 1)
        return XQ_ERR_INVALID_ARG;
    if (flags & ~XQ_PREFILL_NO_PACK) return XQ_ERR_INVALID_ARG;
    if (!(sm_scale > 0.0f) || !(sm_scale < INFINITY)) return XQ_ERR_INVALID_ARG;  // the kernel takes the running maximum before scaling
    const xq_config &c = cache->cfg;
    if (c.head_dim != 128) return XQ_ERR_UNSUPPORTED;
    const bool pack = !(flags & XQ_PREFILL_NO_PACK);
    if (pack && c.merge_mode != XQ_MERGE_NONE) return XQ_ERR_UNSUPPORTED;  // merged codes need two layers' tiles at once
    if (pack && T > c.max_tokens) return XQ_ERR_CAPACITY;
    if ((int64_t)c.batch * c.n_q_heads > 65535) return XQ_ERR_UNSUPPORTED;
    for (int i = 0; i < 4; ++i)
        if (strides[i] < 0 || strides[i] % 8) return XQ_ERR_INVALID_ARG;
    if (strides[3] < c.head_dim || ((uintptr_t)k_f16 & 15) || ((uintptr_t)v_f16 & 15) || ((uintptr_t)q_f16 & 15) ||
        ((uintptr_t)out_f32 & 15))
        return XQ_ERR_INVALID_ARG;
    if (pack)
        for (int l = layer0; l < layer0 + n_layers; ++l)
            for (int i = 0; i < c.batch; ++i)
                if (len_row(cache, l)[i] != 0) return XQ_ERR_STATE;
    hipStream_t s = (hipStream_t)hip_stream;
    const int Tq = pack ? xq_quantized_len(T, c.group, c.residual) : 0;
    if (pack && cache->paging.table && Tq > 0) {
        int32_t *want = cache->want.data();
        for (int i = 0; i < c.batch; ++i) want[i] = Tq;
        if (pages_missing(cache, 0, c.batch, want) > (int64_t)cache->free_pages.size()) return XQ_ERR_CAPACITY;
        int rc = take_pages(cache, 0, c.batch, want, s);
        if (rc) return rc;
    }
    XqPrefillArgs a;
    memset(&a, 0, sizeof(a));
    a.pk.arena = cache->arena;
    a.pk.layers = cache->dev_layers;
    a.pk.st = cache->strides;
    a.pk.layer0 = layer0;
    a.pk.batch = c.batch;
    a.pk.n_kv_heads = c.n_kv_heads;
    a.pk.R = c.residual;
    a.pk.k_src = (const uint16_t *)k_f16;
    a.pk.v_src = (const uint16_t *)v_f16;
    a.pk.s_layer = strides[0];
    a.pk.s_batch = strides[1];
    a.pk.s_head = strides[2];
    a.pk.s_tok = strides[3];
    a.pk.pg = cache->paging;
    a.pk.n_groups = Tq / c.group;
    fill_pack_consts(c, a.pk);
    a.q = (const uint16_t *)q_f16;
    a.out = (float *)out_f32;
    a.T = T;
    a.Tq = Tq;
    a.batch = c.batch;
    a.n_q_heads = c.n_q_heads;
    a.scale_log2e = sm_scale * 1.4426950408889634f;
    if (xq_launch_prefill(a, c.group, n_layers, pack ? 1 : 0, s) != hipSuccess) return XQ_ERR_HIP;
    if (!pack) return XQ_OK;
    XqRingArgs r;
    memset(&r, 0, sizeof(r));
    r.arena = cache->arena;
    r.layers = cache->dev_layers;
    r.st = cache->strides;
    r.layer0 = layer0;
    r.batch = c.batch;
    r.n_kv_heads = c.n_kv_heads;
    r.R = c.residual;
    r.D = c.head_dim;
    r.k_src = (const uint16_t *)k_f16;
    r.v_src = (const uint16_t *)v_f16;
    r.s_layer = strides[0];
    r.s_batch = strides[1];
    r.s_head = strides[2];
    r.s_tok = strides[3];
    r.src_tok0 = Tq;
    r.dst_tok0 = Tq;
    r.n_tok = T - Tq;
    if (xq_launch_ring_write(r, n_layers, s) != hipSuccess) return XQ_ERR_HIP;
    for (int l = layer0; l < layer0 + n_layers; ++l)
        for (int i = 0; i < c.batch; ++i) len_row(cache, l)[i] = T;
    return XQ_OK;
}

int xq_quantize_pack(xq_cache *cache, int32_t layer0, int32_t n_layers, const void *k_f16,
                     const void *v_f16, const int64_t strides[4], int32_t T, void *hip_stream) {
    if (!cache) return XQ_ERR_INVALID_ARG;
    return xq_quantize_pack_seq(cache, layer0, n_layers, 0, cache->cfg.batch, k_f16, v_f16, strides, T, hip_stream);
}

int xq_append_token(xq_cache *cache, int32_t layer0, int32_t n_layers, const void *k_new_f16,
                    const void *v_new_f16, void *hip_stream) {
    if (!range_ok(cache, layer0, n_layers) || !k_new_f16 || !v_new_f16) return XQ_ERR_INVALID_ARG;
    if (((uintptr_t)k_new_f16 & 15) || ((uintptr_t)v_new_f16 & 15)) return XQ_ERR_INVALID_ARG;
    const xq_config &c = cache->cfg;
    if (!merge_range_ok(c, layer0, n_layers)) return XQ_ERR_INVALID_ARG;
    for (int l = layer0; l < layer0 + n_layers; ++l) {
        for (int i = 0; i < c.batch; ++i)
            if (len_row(cache, l)[i] >= c.max_tokens) return XQ_ERR_CAPACITY;
        if (!row_uniform(cache, l) && c.batch > XQ_MAX_RAGGED) return XQ_ERR_UNSUPPORTED;
    }
    if (c.merge_mode != XQ_MERGE_NONE)  // a pair is flushed by one launch, so its layers move together
        for (int l = layer0; l + 1 < layer0 + n_layers; ++l)
            if ((merges_next(c, l, false) || merges_next(c, l, true)) && !rows_equal(cache, l, l + 1))
                return XQ_ERR_STATE;
    hipStream_t s = (hipStream_t)hip_stream;
    if (cache->paging.table) {  // pages for the groups that this call's ring flushes will write
        int32_t *want = cache->want.data();
        for (int i = 0; i < c.batch; ++i) want[i] = 0;
        for (int l = layer0; l < layer0 + n_layers; ++l)
            for (int i = 0; i < c.batch; ++i) {
                const int t = len_row(cache, l)[i], tq = xq_quantized_len(t, c.group, c.residual);
                want[i] = std::max(want[i], t - tq == c.residual ? tq + c.group : tq);
            }
        if (pages_missing(cache, 0, c.batch, want) > (int64_t)cache->free_pages.size()) return XQ_ERR_CAPACITY;
        int rc = take_pages(cache, 0, c.batch, want, s);
        if (rc) return rc;
    }
    const int64_t D = c.head_dim;
    const int64_t per_layer = (int64_t)c.batch * c.n_kv_heads * D;
    // runs of consecutive layers with the same lengths share their launches
    int l = layer0;
    while (l < layer0 + n_layers) {
        int e = l + 1;
        while (e < layer0 + n_layers && rows_equal(cache, e, l)) ++e;
        const int32_t *row = len_row(cache, l);
        const bool ragged = !row_uniform(cache, l);
        bool any_flush = false;  // a full ring: its oldest g tokens become a packed group
        for (int i = 0; i < c.batch; ++i)
            any_flush |= row[i] - xq_quantized_len(row[i], c.group, c.residual) == c.residual;
        if (any_flush) {
            const int Tq = xq_quantized_len(row[0], c.group, c.residual);
            XqPackArgs a;
            memset(&a, 0, sizeof(a));
            a.arena = cache->arena;
            a.layers = cache->dev_layers;
            a.st = cache->strides;
            a.layer0 = l;
            a.batch = c.batch;
            a.n_kv_heads = c.n_kv_heads;
            a.R = c.residual;
            a.from_ring = 1;
            a.src_tok0 = Tq % c.residual;
            a.dst_tok0 = Tq;
            a.n_groups = 1;
            a.pg = cache->paging;
            a.ragged = ragged;
            if (ragged) memcpy(a.seq_T, row, sizeof(int32_t) * c.batch);
            fill_pack_consts(c, a);
            if (xq_launch_pack(a, c.head_dim, c.group, e - l, s) != hipSuccess) return XQ_ERR_HIP;
        }
        XqRingArgs r;
        memset(&r, 0, sizeof(r));
        r.arena = cache->arena;
        r.layers = cache->dev_layers;
        r.st = cache->strides;
        r.layer0 = l;
        r.batch = c.batch;
        r.n_kv_heads = c.n_kv_heads;
        r.R = c.residual;
        r.D = c.head_dim;
        r.k_src = (const uint16_t *)k_new_f16 + (int64_t)(l - layer0) * per_layer;
        r.v_src = (const uint16_t *)v_new_f16 + (int64_t)(l - layer0) * per_layer;
        r.s_layer = per_layer;
        r.s_batch = (int64_t)c.n_kv_heads * D;
        r.s_head = D;
        r.s_tok = D;
        r.src_tok0 = 0;
        r.dst_tok0 = row[0];
        r.n_tok = 1;
        r.ragged = ragged;
        if (ragged) memcpy(r.seq_T, row, sizeof(int32_t) * c.batch);
        if (xq_launch_ring_write(r, e - l, s) != hipSuccess) return XQ_ERR_HIP;
        for (int k = l; k < e; ++k)
            for (int i = 0; i < c.batch; ++i) len_row(cache, k)[i] += 1;
        l = e;
    }
    return XQ_OK;
}

// Plans and enqueues the decode launches of a call; the split partials go to dev_workspace.
static int decode_impl(const xq_cache *cache, int32_t layer0, int32_t n_layers, const void *q_f16,
                       void *out_f32, float sm_scale, void *dev_workspace, size_t workspace_bytes,
                       int32_t flags, void *hip_stream) {
    if (!range_ok(cache, layer0, n_layers) || !q_f16 || !out_f32 || !dev_workspace) return XQ_ERR_INVALID_ARG;
    if (flags & ~(XQ_DECODE_PAIR_FUSED | XQ_DECODE_VECTOR_ALU | XQ_DECODE_MATRIX_F16 | XQ_DECODE_MERGE_LAUNCH |
                  XQ_DECODE_MERGE_IN_LAUNCH))
        return XQ_ERR_INVALID_ARG;
    if ((flags & XQ_DECODE_MERGE_LAUNCH) && (flags & XQ_DECODE_MERGE_IN_LAUNCH)) return XQ_ERR_INVALID_ARG;
    if (((uintptr_t)q_f16 & 3) || ((uintptr_t)out_f32 & 3) || ((uintptr_t)dev_workspace & 15)) return XQ_ERR_INVALID_ARG;
    const xq_config &c = cache->cfg;
    const int32_t *row = len_row(cache, layer0);
    int T = 0;  // the longest sequence plans the splits
    for (int i = 0; i < c.batch; ++i) {
        if (row[i] < 1) return XQ_ERR_STATE;
        if (row[i] > T) T = row[i];
    }
    for (int l = layer0; l < layer0 + n_layers; ++l) {
        if (!rows_equal(cache, l, layer0)) return XQ_ERR_STATE;
        // the layer whose codes l reads may lie outside the range: it must already hold every
        // packed group that l's metadata describes
        for (int v = 0; v < 2; ++v) {
            const int cl = code_layer(c, l, v != 0);
            if (cl == l) continue;
            for (int i = 0; i < c.batch; ++i)
                if (xq_quantized_len(len_row(cache, cl)[i], c.group, c.residual) <
                    xq_quantized_len(row[i], c.group, c.residual))
                    return XQ_ERR_STATE;
        }
    }
    const bool ragged = !row_uniform(cache, layer0);
    if (ragged && c.batch > XQ_MAX_RAGGED) return XQ_ERR_UNSUPPORTED;
    const int Tq = xq_quantized_len(T, c.group, c.residual);
    hipStream_t s = (hipStream_t)hip_stream;
    const int rep = c.n_q_heads / c.n_kv_heads;
    // The kernels serve 1, 2 or 4 query heads of a kv head at a time (1 when D = 64): other
    // ratios take several passes over the kv head's cache, largest part first.
    int parts[XQ_MAX_REP], n_parts = 0;
    for (int left = rep; left > 0; left -= parts[n_parts++])
        parts[n_parts] = (c.head_dim == 64) ? 1 : (left >= 4 ? 4 : (left >= 2 ? 2 : 1));
    bool fusable = true;  // a pair shares a workgroup only if every part fits the kernel's weight tables
    for (int i = 0; i < n_parts; ++i) fusable = fusable && xq_decode_can_fuse(c.head_dim, c.group, parts[i]);
    // whether one workgroup serves the pair (a, a+1): only when the second layer reads both the
    // key and the value codes of the first (with one of the two shared, holding two code sets
    // in registers costs more than the shared unpacking saves: measured 12 % slower)
    auto fuse_mode = [&](int a) -> int {
        if (!(flags & XQ_DECODE_PAIR_FUSED) || !fusable) return 0;
        if (group_size(c) != 2 || c.share_dominant != 0) return 0;
        if (a % 2 != 0 || a + 1 >= layer0 + n_layers) return 0;
        if (cache->layers[a + 1].bk != cache->layers[a].bk || cache->layers[a + 1].bv != cache->layers[a].bv) return 0;
        return (!cache->layers[a + 1].k_store && !cache->layers[a + 1].v_store) ? 1 : 0;
    };
    // runs of layers with one (bk, bv) and one fusion mode share a launch
    struct Run {
        int l, e, fused;
        int n_splits, tps;  // each run is a launch of its own and gets its own split plan
        bool brief;         // (about) one round of workgroups: a launch whose tail a merge launch would lengthen
        int64_t ws_off;     // where its partials start in the workspace, in floats
    };
    Run runs[XQ_MAX_LAYERS];
    int n_runs = 0;
    for (int l = layer0; l < layer0 + n_layers;) {
        const XqLayerDesc &d0 = cache->layers[l];
        const int fused = fuse_mode(l);
        int e = l;
        while (e < layer0 + n_layers) {
            const XqLayerDesc &d = cache->layers[e];
            if (d.bk != d0.bk || d.bv != d0.bv) break;
            if (fused) {
                if (fuse_mode(e) != fused) break;
                e += 2;
            } else {
                if (fuse_mode(e)) break;
                e += 1;
            }
        }
        runs[n_runs++] = Run{l, e, fused, 0, 0, false, 0};
        l = e;
    }
    const bool matrix = c.head_dim == 128 && !(flags & XQ_DECODE_VECTOR_ALU);
    int64_t ws_floats = 0;
    for (int ri = 0; ri < n_runs; ++ri) {
        Run &r = runs[ri];
        // (layer or pair, sequence, kv head) slices = workgroups per split; workgroup slots of the
        // chip for the least resident kernel variant among the run's passes
        const int64_t work_items = (int64_t)(r.fused ? (r.e - r.l) / 2 : r.e - r.l) * c.batch * c.n_kv_heads;
        int wgs_per_cu = 4;
        for (int i = 0; i < n_parts; ++i)
            wgs_per_cu = std::min(wgs_per_cu, decode_wgs_per_cu(!matrix ? 0 : (flags & XQ_DECODE_MATRIX_F16) ? 1 : 2, parts[i],
                                                                r.fused != 0, c.group, cache->layers[r.l].bk,
                                                                cache->layers[r.l].bv));
        plan_splits(cache, Tq, work_items, 256 * wgs_per_cu, &r.n_splits, &r.tps);
        r.brief = work_items * (r.n_splits + 1) <= 256 * wgs_per_cu * 5 / 4;
        r.ws_off = ws_floats;
        ws_floats += (int64_t)workspace_floats(c, r.e - r.l, r.n_splits);
    }
    if ((size_t)ws_floats * sizeof(float) > workspace_bytes) return XQ_ERR_CAPACITY;
    const int64_t per_layer_q = (int64_t)c.batch * c.n_q_heads * c.head_dim;
    for (int ri = 0; ri < n_runs; ++ri) {
        const int l = runs[ri].l, e = runs[ri].e, fused = runs[ri].fused;
        const int n_splits = runs[ri].n_splits, tps = runs[ri].tps;
        const XqLayerDesc &d0 = cache->layers[l];
        XqDecodeArgs a;
        memset(&a, 0, sizeof(a));
        a.arena = cache->arena;
        a.layers = cache->dev_layers;
        a.st = cache->strides;
        a.layer0 = l;
        a.batch = c.batch;
        a.n_q_heads = c.n_q_heads;
        a.n_kv_heads = c.n_kv_heads;
        a.R = c.residual;
        a.group = c.group;
        a.T = T;
        a.Tq = Tq;
        a.ragged = ragged;
        if (ragged) memcpy(a.seq_T, row, sizeof(int32_t) * c.batch);
        a.n_splits = n_splits;
        a.tiles_per_split = tps;
        a.q = (const uint16_t *)q_f16 + (int64_t)(l - layer0) * per_layer_q;
        a.out = (float *)out_f32 + (int64_t)(l - layer0) * per_layer_q;
        a.ws = (float *)dev_workspace + runs[ri].ws_off;
        a.scale_log2e = sm_scale * 1.4426950408889634f;
        a.pg = cache->paging;
        // 2-bit keys take the fp8 x fp4 key phase unless the caller keeps everything on the fp16 instruction
        a.matrix = !matrix ? 0 : (d0.bk == 2 && !(flags & XQ_DECODE_MATRIX_F16)) ? 2 : 1;
        if (!fused)
            for (int x = l; x < e; ++x) {
                a.reuse_codes |= !cache->layers[x].k_store || !cache->layers[x].v_store;
            }
        // the run is a whole number of sharing groups (pairs by default), some of which share codes
        a.pair_order = (a.reuse_codes && l % group_size(c) == 0 && (e - l) % group_size(c) == 0) ? group_size(c) : 0;
        a.rep = rep;
        // Who merges the split partials: the last workgroup to arrive, or a launch of its own.  Measured,
        // the first wins where a second launch's fixed cost shows -- calls for one layer: 12.7 against
        // 13.5 us on a 4k cache, 75.5 against 76.5 us on the 32k one -- and loses where the decode launch
        // runs many rounds of workgroups anyway (32 layers of the 4k cache in one call: 82 against 77 us).
        const bool in_launch = (flags & XQ_DECODE_MERGE_IN_LAUNCH) || (!(flags & XQ_DECODE_MERGE_LAUNCH) && runs[ri].brief);
        a.arrivals = in_launch ? cache->arrivals : nullptr;
        for (int i = 0; i < n_parts; ++i) {
            if (xq_launch_decode(a, c.head_dim, c.group, d0.bk, d0.bv, parts[i], e - l, fused, s) != hipSuccess)
                return XQ_ERR_HIP;
            a.q_head0 += parts[i];
        }
        if (!a.arrivals && xq_launch_merge(a, c.head_dim, e - l, s) != hipSuccess) return XQ_ERR_HIP;
    }
    return XQ_OK;
}

int xq_decode_attention(const xq_cache *cache, int32_t layer0, int32_t n_layers, const void *q_f16,
                        void *out_f32, float sm_scale, void *dev_workspace, size_t workspace_bytes,
                        int32_t flags, void *hip_stream) {
    return decode_impl(cache, layer0, n_layers, q_f16, out_f32, sm_scale, dev_workspace, workspace_bytes, flags,
                       hip_stream);
}

int xq_decode_attention_static(const xq_cache *cache, int32_t layer0, int32_t n_layers, const void *q_f16,
                               void *out_f32, float sm_scale, int32_t flags, void *hip_stream) {
    if (!cache) return XQ_ERR_INVALID_ARG;
    void *ws = nullptr;
    int rc = static_scratch(&ws);
    if (rc) return rc;
    // decode_impl answers XQ_ERR_CAPACITY when the call's partials exceed XQ_STATIC_SCRATCH_BYTES
    return decode_impl(cache, layer0, n_layers, q_f16, out_f32, sm_scale, ws, XQ_STATIC_SCRATCH_BYTES, flags,
                       hip_stream);
}

int xq_unpack_codes(const xq_cache *cache, int32_t layer, int32_t is_v, uint8_t *dev_codes_u8, void *hip_stream) {
    if (!range_ok(cache, layer, 1) || !dev_codes_u8) return XQ_ERR_INVALID_ARG;
    const xq_config &c = cache->cfg;
    const XqLayerDesc &d = cache->layers[layer];
    if (!(is_v ? d.v_store : d.k_store)) return XQ_ERR_STATE;
    if (!row_uniform(cache, layer)) return XQ_ERR_STATE;  // the dense output needs one length
    const int Tq = xq_quantized_len(len_row(cache, layer)[0], c.group, c.residual);
    if (Tq == 0) return XQ_ERR_STATE;
    XqUnpackArgs a;
    a.B = is_v ? d.bv : d.bk;
    a.codes = cache->arena + (is_v ? d.v_codes : d.k_codes);
    a.stride = is_v ? (a.B == 2 ? cache->strides.v_codes2 : cache->strides.v_codes1)
                    : (a.B == 2 ? cache->strides.k_codes2 : cache->strides.k_codes1);
    a.n_bh = c.batch * c.n_kv_heads;
    a.n_kv_heads = c.n_kv_heads;
    a.pg = cache->paging;
    a.Tq = Tq;
    a.D = c.head_dim;
    a.is_v = is_v ? 1 : 0;
    a.out = dev_codes_u8;
    return xq_launch_unpack(a, (hipStream_t)hip_stream) == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

int xq_code_delta_histogram(const xq_cache *cache, int32_t layer, int32_t is_v, uint64_t *dev_counts_u64,
                            void *hip_stream) {
    if (!range_ok(cache, layer, 2) || !dev_counts_u64 || ((uintptr_t)dev_counts_u64 & 7)) return XQ_ERR_INVALID_ARG;
    const xq_config &c = cache->cfg;
    const XqLayerDesc &d0 = cache->layers[layer], &d1 = cache->layers[layer + 1];
    if (!(is_v ? d0.v_store && d1.v_store : d0.k_store && d1.k_store)) return XQ_ERR_STATE;
    const int B = is_v ? d0.bv : d0.bk;
    if (B != (is_v ? d1.bv : d1.bk) || !rows_equal(cache, layer, layer + 1)) return XQ_ERR_STATE;
    const bool ragged = !row_uniform(cache, layer);
    if (ragged && c.batch > XQ_MAX_RAGGED) return XQ_ERR_UNSUPPORTED;
    XqDeltaArgs a;
    memset(&a, 0, sizeof(a));
    a.codes_a = cache->arena + (is_v ? d0.v_codes : d0.k_codes);
    a.codes_b = cache->arena + (is_v ? d1.v_codes : d1.k_codes);
    a.stride = is_v ? (B == 2 ? cache->strides.v_codes2 : cache->strides.v_codes1)
                    : (B == 2 ? cache->strides.k_codes2 : cache->strides.k_codes1);
    a.n_kv_heads = c.n_kv_heads;
    a.pg = cache->paging;
    a.n_bh = c.batch * c.n_kv_heads;
    a.B = B;
    a.words_per_token = c.head_dim * B / 32;
    a.ragged = ragged;
    a.Tq = xq_quantized_len(len_row(cache, layer)[0], c.group, c.residual);
    if (ragged)
        for (int i = 0; i < c.batch; ++i) a.seq_Tq[i] = xq_quantized_len(len_row(cache, layer)[i], c.group, c.residual);
    a.counts = (unsigned long long *)dev_counts_u64;
    return xq_launch_delta_histogram(a, (hipStream_t)hip_stream) == hipSuccess ? XQ_OK : XQ_ERR_HIP;
}

double xq_equivalent_bits(const xq_config *cfg, int32_t include_metadata, int32_t T) {
    if (check_config(cfg)) return -1.0;
    const xq_config &c = *cfg;
    double code_bits = 0.0;  // per element position, summed over layers and K/V
    for (int l = 0; l < c.n_layers; ++l) {
        if (stores_codes(c, l, false)) code_bits += bits_of(c, l, false);
        if (stores_codes(c, l, true)) code_bits += bits_of(c, l, true);
    }
    if (!include_metadata) return code_bits / (2.0 * c.n_layers);
    if (T < 1) return -1.0;
    const double Tq = xq_quantized_len(T, c.group, c.residual), r = T - Tq;
    // per channel of one (sequence, kv head): packed tokens carry codes + 32 bits of fp16
    // scale/zero per group of g elements in every layer; ring tokens are 16-bit
    double bits = Tq * code_bits + Tq * (32.0 / c.group) * 2.0 * c.n_layers + r * 16.0 * 2.0 * c.n_layers;
    return bits / (2.0 * c.n_layers * T);
}

}  // extern "C"
