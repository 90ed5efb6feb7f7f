// Cache descriptor: config validation, HBM layout, host-side token counters, error text, and the
// export kernel that copies a layer's index table out for tests.
//
// HBM layout of a cache (all regions 256-byte aligned), chosen so that everything one
// (layer, sequence, head) unit reads in a decode step is one contiguous run:
//   per layer l:
//     spatial units  [B][Hs_l] : K plane (S+W rows) then V plane (S+W rows)
//     semantic units [B][Hm_l] : K plane (M+C rows) then V plane (M+C rows)
//     score          [B][Hm_l][M+C] float   running sum of attention probabilities (Algorithm 1)
//     pos            [B][Hm_l][M+C] int32   absolute token position held by each slot
// Spatial slots: 0..S-1 hold positions 0..S-1 (the initial sink tokens of Sec. 3.3); slot
// S + ((p-S) mod W) holds position p >= S, so the ring always contains the W newest tokens.
// Semantic slots: 0..M-1 heavy hitters (the first m in use); M..M+C-1 the row buffer of
// Algorithm 2, used as a ring so that the R protected newest tokens never have to move.
// W and M may differ per layer (the layout is per layer anyway) and per head: with budgets per head every
// unit of a layer keeps the size of the layer's largest W_h / M_h, and head h uses a ring of W_h slots, or
// the first M_h heavy slots, of its unit; the row buffer starts at slot max M_h for every semantic head.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <cmath>
#include <new>

#include "ssd_device.h"

namespace ssd {

static thread_local char g_err[512] = {0};

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(hipError_t e, const char *what) {
    snprintf(g_err, sizeof(g_err), "%s: %s", what, hipGetErrorString(e));
    return SSD_ERR_HIP;
}

void clear_error() { g_err[0] = 0; }

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static int esize_of(int dtype) { return dtype == SSD_F32 ? 4 : dtype == SSD_BF16 ? 2 : 0; }

static int validate(const ssd_config *c, const uint8_t *head_type, const int32_t *window, const int32_t *budget) {
    if (!c || !head_type) return fail(SSD_ERR_INVALID_ARG, "config or head_type is NULL");
    if (c->n_layers < 1 || c->n_layers > 1024) return fail(SSD_ERR_INVALID_ARG, "n_layers=%d outside 1..1024", c->n_layers);
    if (c->n_seqs < 1 || c->n_seqs > 65535) return fail(SSD_ERR_INVALID_ARG, "n_seqs=%d outside 1..65535", c->n_seqs);
    if (c->n_heads < 1 || c->n_heads > 128) return fail(SSD_ERR_INVALID_ARG, "n_heads=%d outside 1..128", c->n_heads);
    if (c->head_dim != 64 && c->head_dim != 128) return fail(SSD_ERR_INVALID_ARG, "head_dim=%d, supported: 64, 128", c->head_dim);
    if (esize_of(c->dtype) == 0) return fail(SSD_ERR_INVALID_ARG, "dtype=%d is neither SSD_F32 nor SSD_BF16", c->dtype);
    if (c->window < 1) return fail(SSD_ERR_INVALID_ARG, "window W=%d must be >= 1", c->window);
    if (c->n_init_sink < 0) return fail(SSD_ERR_INVALID_ARG, "n_init_sink S=%d must be >= 0", c->n_init_sink);
    if (c->budget < 1) return fail(SSD_ERR_INVALID_ARG, "budget M=%d must be >= 1", c->budget);
    if (c->recent < 0) return fail(SSD_ERR_INVALID_ARG, "recent R=%d must be >= 0", c->recent);
    if (c->stage_cap <= c->recent) return fail(SSD_ERR_INVALID_ARG, "stage_cap C=%d must exceed recent R=%d", c->stage_cap, c->recent);
    if ((int64_t)c->budget + c->stage_cap > 4096) return fail(SSD_ERR_INVALID_ARG, "M + C = %lld exceeds 4096", (long long)c->budget + c->stage_cap);
    if (c->spatial_row_buffer != 0 && c->spatial_row_buffer != 1) return fail(SSD_ERR_INVALID_ARG, "spatial_row_buffer must be 0 or 1");
    if ((int64_t)c->n_init_sink + c->window + (c->spatial_row_buffer ? c->stage_cap : 0) > 65536)
        return fail(SSD_ERR_INVALID_ARG, "a spatial head would need more than 65536 slots");
    if (!(c->softmax_scale >= 0.f) || !std::isfinite(c->softmax_scale)) return fail(SSD_ERR_INVALID_ARG, "softmax_scale must be finite and >= 0");
    for (int i = 0; i < 4; ++i)
        if (c->reserved[i] != 0) return fail(SSD_ERR_INVALID_ARG, "reserved[%d] must be 0", i);
    const size_t n = (size_t)c->n_layers * c->n_heads;
    for (size_t i = 0; i < n; ++i)
        if (head_type[i] > 1) return fail(SSD_ERR_INVALID_ARG, "head_type[%zu]=%d is neither SSD_SPATIAL nor SSD_SEMANTIC", i, head_type[i]);
    for (int l = 0; l < c->n_layers; ++l) {
        if (window) {
            if (window[l] < 1) return fail(SSD_ERR_INVALID_ARG, "window[%d]=%d must be >= 1", l, window[l]);
            if ((int64_t)c->n_init_sink + window[l] + (c->spatial_row_buffer ? c->stage_cap : 0) > 65536)
                return fail(SSD_ERR_INVALID_ARG, "window[%d]=%d: a spatial head would need more than 65536 slots", l, window[l]);
        }
        if (budget) {
            if (budget[l] < 1) return fail(SSD_ERR_INVALID_ARG, "budget[%d]=%d must be >= 1", l, budget[l]);
            if ((int64_t)budget[l] + c->stage_cap > 4096) return fail(SSD_ERR_INVALID_ARG, "budget[%d] + C = %lld exceeds 4096", l, (long long)budget[l] + c->stage_cap);
        }
    }
    return SSD_OK;
}

// Budgets per head: checks them and reduces them to the per-layer maxima that size the units.
static int validate_heads(const ssd_config *c, const uint8_t *head_type, const int32_t *head_budget,
                          std::vector<int32_t> *Wl, std::vector<int32_t> *Ml) {
    if (!c || !head_type) return fail(SSD_ERR_INVALID_ARG, "config or head_type is NULL");
    if (!head_budget) return fail(SSD_ERR_INVALID_ARG, "head_budget is NULL");
    if (c->n_layers < 1 || c->n_layers > 1024 || c->n_heads < 1 || c->n_heads > HMAX)
        return fail(SSD_ERR_INVALID_ARG, "n_layers=%d or n_heads=%d out of range", c->n_layers, c->n_heads);
    Wl->assign(c->n_layers, c->window);
    Ml->assign(c->n_layers, c->budget);
    for (int l = 0; l < c->n_layers; ++l) {
        int wmax = 0, mmax = 0;
        for (int h = 0; h < c->n_heads; ++h) {
            const size_t i = (size_t)l * c->n_heads + h;
            const int32_t v = head_budget[i];
            if (head_type[i] == SSD_SEMANTIC) {
                if (v < 1 || (int64_t)v + c->stage_cap > 4096)
                    return fail(SSD_ERR_INVALID_ARG, "head_budget[%d,%d]=%d: a semantic head's M must be >= 1 with M + C <= 4096", l, h, v);
                mmax = v > mmax ? v : mmax;
            } else {
                if (v < 1 || v > 65535)
                    return fail(SSD_ERR_INVALID_ARG, "head_budget[%d,%d]=%d: a spatial head's W must be in 1..65535", l, h, v);
                wmax = v > wmax ? v : wmax;
            }
        }
        if (wmax > 0) (*Wl)[l] = wmax;
        if (mmax > 0) (*Ml)[l] = mmax;
    }
    return SSD_OK;
}

// Fills ldesc (if non-null) and returns the total byte size.
static size_t plan_layout(const ssd_config *c, const uint8_t *head_type, const int32_t *window, const int32_t *budget,
                          std::vector<LayerDesc> *ldesc) {
    const int L = c->n_layers, H = c->n_heads;
    const size_t row = (size_t)c->head_dim * esize_of(c->dtype);
    size_t off = 0;
    if (ldesc) ldesc->resize(L);
    for (int l = 0; l < L; ++l) {
        const int W = window ? window[l] : c->window, M = budget ? budget[l] : c->budget;
        const size_t unit_sp = 2 * (size_t)(c->n_init_sink + W + (c->spatial_row_buffer ? c->stage_cap : 0)) * row;
        const size_t unit_se = 2 * (size_t)(M + c->stage_cap) * row;
        const size_t slots = (size_t)M + c->stage_cap;
        LayerDesc m;
        m.sem_mask[0] = m.sem_mask[1] = 0;
        m.n_sp = m.n_se = 0;
        for (int h = 0; h < H; ++h) {
            if (head_type[(size_t)l * H + h] == SSD_SEMANTIC) {
                m.sem_mask[h >> 6] |= 1ull << (h & 63);
                m.n_se++;
            } else {
                m.n_sp++;
            }
        }
        m.off_sp = off;
        off = align_up(off + (size_t)c->n_seqs * m.n_sp * unit_sp, 256);
        m.off_se = off;
        off = align_up(off + (size_t)c->n_seqs * m.n_se * unit_se, 256);
        m.off_score = off;
        off = align_up(off + (size_t)c->n_seqs * m.n_se * slots * sizeof(float), 256);
        m.off_pos = off;
        off = align_up(off + (size_t)c->n_seqs * m.n_se * slots * sizeof(int32_t), 256);
        if (ldesc) (*ldesc)[l] = m;
    }
    return off > 0 ? off : 256;
}

int check_layers(const ssd_cache *c, int lb, int le) {
    if (!c) return fail(SSD_ERR_INVALID_ARG, "cache is NULL");
    if (lb < 0 || le > c->cfg.n_layers || lb >= le)
        return fail(SSD_ERR_LAYER_RANGE, "layer range [%d, %d) is not inside [0, %d)", lb, le, c->cfg.n_layers);
    return SSD_OK;
}

int ensure_events(ssd_cache *c) {
    if (c->have_events) return SSD_OK;
    hipError_t e = hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming);
    if (e != hipSuccess) return hip_fail(e, "event creation");
    for (int i = 1; i < SSD_MAX_SPLIT; ++i) {
        e = hipEventCreateWithFlags(&c->ev_join[i], hipEventDisableTiming);
        if (e != hipSuccess) {
            (void)hipEventDestroy(c->ev_fork);
            for (int j = 1; j < i; ++j) (void)hipEventDestroy(c->ev_join[j]);
            return hip_fail(e, "event creation");
        }
    }
    c->have_events = true;
    return SSD_OK;
}

Geom make_geom(const ssd_cache *c, int l) {
    Geom g;
    g.base = c->dev;
    g.B = c->cfg.n_seqs;
    g.H = c->cfg.n_heads;
    g.S = c->cfg.n_init_sink;
    g.W = c->Wl[l];
    g.M = c->Ml[l];
    g.C = c->cfg.stage_cap;
    g.RW = g.W + (c->cfg.spatial_row_buffer ? g.C : 0);
    g.row_bytes = c->cfg.head_dim * c->esize;
    g.unit_sp_bytes = 2u * (uint32_t)(g.S + g.RW) * (uint32_t)g.row_bytes;
    g.unit_se_bytes = 2u * (uint32_t)(g.M + g.C) * (uint32_t)g.row_bytes;
    return g;
}

void fill_launch_meta(const ssd_cache *c, int lb, int le, LaunchMeta *out) {
    for (int l = lb; l < le; ++l) out->layer[l - lb] = c->ldesc[l];
    for (int i = le - lb; i < LMAX; ++i) out->layer[i] = c->ldesc[lb];   // never indexed; keeps the bytes defined
}

bool has_buffer(const ssd_cache *c, int l) { return c->ldesc[l].n_se > 0 || c->cfg.spatial_row_buffer != 0; }

void apply_compress_counters(ssd_cache *c, int l) {
    LayerState &x = c->st[l];
    const ssd_config &cf = c->cfg;
    if (cf.spatial_row_buffer) x.nc = x.n;             // spatial heads: the window is re-cut to the W newest tokens
    const int old = x.c - cf.recent;                   // buffered tokens that leave the row buffer
    if (!has_buffer(c, l) || old <= 0) return;
    if (c->ldesc[l].n_se > 0) {
        const int tot = x.m + old;
        x.m = tot < c->Ml[l] ? tot : c->Ml[l];
    }
    x.base = (x.base + old) % cf.stage_cap;
    x.c = cf.recent;
}

void fill_head_table(const ssd_cache *c, int l, HeadTable *out) {
    const int H = c->cfg.n_heads;
    for (int h = 0; h < HMAX; ++h) out->v[h] = per_head(c) && h < H ? c->head_budget[(size_t)l * H + h] : 0;
}

int spatial_slot(const ssd_cache *c, int l, int p) {
    return ring_slot(c->cfg.n_init_sink, c->Wl[l] + (c->cfg.spatial_row_buffer ? c->cfg.stage_cap : 0), p);
}

Segs spatial_segs(const ssd_cache *c, int l, const LayerState &st) {
    return ring_segs(c->cfg.n_init_sink, c->Wl[l], c->cfg.stage_cap, c->cfg.spatial_row_buffer != 0, st.n, st.nc);
}

Segs semantic_segs(const ssd_cache *c, int l, const LayerState &st) {
    Segs s = {{0, 0, 0}, {0, 0, 0}, 0};
    const int M = c->Ml[l], C = c->cfg.stage_cap;
    s.start[0] = 0;
    s.len[0] = st.m;
    const int first = st.base + st.c <= C ? st.c : C - st.base;   // run up to the end of the ring
    s.start[1] = M + st.base;
    s.len[1] = first;
    s.start[2] = M;
    s.len[2] = st.c - first;                                      // wrapped part
    s.total = s.len[0] + s.len[1] + s.len[2];
    return s;
}

Segs spatial_segs_fused(const ssd_cache *c, int l, const LayerState &before, const LayerState &, int new_slot) {
    return ring_segs_fused(c->cfg.n_init_sink, c->Wl[l], c->cfg.stage_cap, c->cfg.spatial_row_buffer != 0, before.n, before.nc, new_slot);
}

static bool same_geom(const ssd_cache *c, int a, int b) { return c->Wl[a] == c->Wl[b] && c->Ml[a] == c->Ml[b]; }

int same_state_run(const ssd_cache *c, int lb, int le) {
    int l = lb + 1;
    if (heads_differ(c, lb)) return l;
    // layers with and without semantic heads never share a launch: only the former have a row buffer
    const bool buf = has_buffer(c, lb), has_se = c->ldesc[lb].n_se > 0;
    while (l < le && l - lb < LMAX && c->st[l] == c->st[lb] && same_geom(c, l, lb) && has_buffer(c, l) == buf &&
           (c->ldesc[l].n_se > 0) == has_se && !heads_differ(c, l))
        ++l;
    return l;
}

int same_geom_run(const ssd_cache *c, int lb, int le) {
    int l = lb + 1;
    if (heads_differ(c, lb)) return l;
    while (l < le && l - lb < LMAX && same_geom(c, l, lb) && !heads_differ(c, l)) ++l;
    return l;
}

// ---- export ---------------------------------------------------------------

__global__ void export_kernel(Geom g, LayerDesc ld, LayerState st, Segs se, int ref, int slots, HeadTable ht, int heads,
                              int32_t *pos_out, int32_t *count_out, float *score_out) {
    const int unit = blockIdx.x;   // b*H + h
    const int b = unit / g.H, h = unit % g.H;
    const UnitRef u = unit_ref(g, ld, b, h);
    const size_t o = (size_t)unit * (size_t)slots;
    int count;
    if (u.sem) {
        if (heads) {                                  // this head's share of the heavy slots
            const int m_h = st.m < ht.v[h] ? st.m : ht.v[h];
            se.total -= se.len[0] - m_h;
            se.len[0] = m_h;
        }
        count = se.total;
        for (int s = threadIdx.x; s < slots; s += blockDim.x) {
            bool valid = false;
            for (int k = 0; k < 3; ++k) valid = valid || (s >= se.start[k] && s < se.start[k] + se.len[k]);
            if (pos_out) pos_out[o + s] = valid ? u.pos[s] : -1;
            if (score_out) score_out[o + s] = valid ? u.score[s] : 0.f;
        }
    } else {
        // retained: sinks and positions [lo, n), the window being cut at `ref` tokens
        const int W = heads ? ht.v[h] : g.W;
        const int RW = W + (g.RW - g.W);
        const int lo = ref - W > g.S ? ref - W : g.S;
        const int n_sink = st.n < g.S ? st.n : g.S;
        const int n_win = st.n > lo ? st.n - lo : 0;
        count = n_sink + n_win;
        for (int s = threadIdx.x; s < slots; s += blockDim.x) {
            int p = -1;
            if (s < g.S) {
                p = s < st.n ? s : -1;
            } else if (s < g.S + RW && n_win > 0) {
                // newest position whose ring slot is s
                const int j = s - g.S;
                const int last = st.n - 1;
                const int kl = (last - g.S) % RW;
                const int cand = last - ((kl - j + RW) % RW);
                p = cand >= lo ? cand : -1;
            }
            if (pos_out) pos_out[o + s] = p;
            if (score_out) score_out[o + s] = 0.f;
        }
    }
    if (count_out && threadIdx.x == 0) count_out[unit] = count;
}

}  // namespace ssd

using namespace ssd;

extern "C" {

size_t ssd_cache_bytes(const ssd_config *cfg, const uint8_t *head_type) { return ssd_cache_bytes_layered(cfg, head_type, nullptr, nullptr); }

int ssd_cache_init(const ssd_config *cfg, const uint8_t *head_type, void *dev_mem, size_t bytes, ssd_cache **out) {
    return ssd_cache_init_layered(cfg, head_type, nullptr, nullptr, dev_mem, bytes, out);
}

size_t ssd_cache_bytes_layered(const ssd_config *cfg, const uint8_t *head_type, const int32_t *window, const int32_t *budget) {
    clear_error();
    if (validate(cfg, head_type, window, budget) != SSD_OK) return 0;
    return plan_layout(cfg, head_type, window, budget, nullptr);
}

size_t ssd_cache_bytes_heads(const ssd_config *cfg, const uint8_t *head_type, const int32_t *head_budget) {
    clear_error();
    std::vector<int32_t> Wl, Ml;
    if (validate_heads(cfg, head_type, head_budget, &Wl, &Ml) != SSD_OK) return 0;
    return ssd_cache_bytes_layered(cfg, head_type, Wl.data(), Ml.data());
}

int ssd_cache_init_heads(const ssd_config *cfg, const uint8_t *head_type, const int32_t *head_budget, void *dev_mem, size_t bytes,
                         ssd_cache **out) {
    clear_error();
    if (!out) return fail(SSD_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    std::vector<int32_t> Wl, Ml;
    int rc = validate_heads(cfg, head_type, head_budget, &Wl, &Ml);
    if (rc != SSD_OK) return rc;
    rc = ssd_cache_init_layered(cfg, head_type, Wl.data(), Ml.data(), dev_mem, bytes, out);
    if (rc != SSD_OK) return rc;
    const size_t n = (size_t)cfg->n_layers * cfg->n_heads;
    (*out)->head_budget.resize(n);
    for (size_t i = 0; i < n; ++i) (*out)->head_budget[i] = (uint16_t)head_budget[i];
    (*out)->heads_differ.assign(cfg->n_layers, 0);
    for (int l = 0; l < cfg->n_layers; ++l)
        for (int h = 0; h < cfg->n_heads; ++h) {
            const size_t i = (size_t)l * cfg->n_heads + h;
            if (head_budget[i] != (head_type[i] == SSD_SEMANTIC ? Ml[l] : Wl[l])) (*out)->heads_differ[l] = 1;
        }
    return SSD_OK;
}

int ssd_cache_init_layered(const ssd_config *cfg, const uint8_t *head_type, const int32_t *window, const int32_t *budget,
                           void *dev_mem, size_t bytes, ssd_cache **out) {
    clear_error();
    if (!out) return fail(SSD_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    int rc = validate(cfg, head_type, window, budget);
    if (rc != SSD_OK) return rc;
    if (!dev_mem) return fail(SSD_ERR_INVALID_ARG, "dev_mem is NULL");
    if (!aligned(dev_mem, 256)) return fail(SSD_ERR_INVALID_ARG, "dev_mem is not 256-byte aligned");
    ssd_cache *c = new (std::nothrow) ssd_cache();
    if (!c) return fail(SSD_ERR_INVALID_ARG, "out of host memory");
    c->cfg = *cfg;
    c->esize = esize_of(cfg->dtype);
    c->scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
    c->head_type.assign(head_type, head_type + (size_t)cfg->n_layers * cfg->n_heads);
    c->Wl.assign(cfg->n_layers, cfg->window);
    c->Ml.assign(cfg->n_layers, cfg->budget);
    if (window) c->Wl.assign(window, window + cfg->n_layers);
    if (budget) c->Ml.assign(budget, budget + cfg->n_layers);
    const size_t need = plan_layout(cfg, head_type, window, budget, &c->ldesc);
    if (bytes < need) {
        delete c;
        return fail(SSD_ERR_INVALID_ARG, "dev_mem holds %zu bytes, the cache needs %zu", bytes, need);
    }
    c->dev = static_cast<char *>(dev_mem);
    c->bytes = bytes;
    c->launch_enabled = true;
    c->shape = LaunchShape{0, 0, 0};
    c->last_shape = LaunchShape{0, 0, 0};
    c->have_events = false;
    c->st.assign(cfg->n_layers, LayerState{0, 0, 0, 0, 0});
    *out = c;
    return SSD_OK;
}

void ssd_cache_free(ssd_cache *cache) {
    if (cache && cache->have_events) {
        (void)hipEventDestroy(cache->ev_fork);
        for (int i = 1; i < SSD_MAX_SPLIT; ++i) (void)hipEventDestroy(cache->ev_join[i]);
    }
    delete cache;
}

int ssd_cache_reset(ssd_cache *cache) {
    clear_error();
    if (!cache) return fail(SSD_ERR_INVALID_ARG, "cache is NULL");
    cache->st.assign(cache->cfg.n_layers, LayerState{0, 0, 0, 0, 0});
    return SSD_OK;
}

int ssd_cache_layer_state(const ssd_cache *cache, int layer, int32_t out4[4]) {
    clear_error();
    int rc = check_layers(cache, layer, layer + 1);
    if (rc != SSD_OK) return rc;
    if (!out4) return fail(SSD_ERR_INVALID_ARG, "out4 is NULL");
    const LayerState &s = cache->st[layer];
    out4[0] = s.n; out4[1] = s.m; out4[2] = s.c; out4[3] = s.base;
    return SSD_OK;
}

int ssd_cache_layer_window(const ssd_cache *cache, int layer, int32_t *n_at_last_compress) {
    clear_error();
    int rc = check_layers(cache, layer, layer + 1);
    if (rc != SSD_OK) return rc;
    if (!n_at_last_compress) return fail(SSD_ERR_INVALID_ARG, "output pointer is NULL");
    *n_at_last_compress = cache->st[layer].nc;
    return SSD_OK;
}

int ssd_cache_set_launch(ssd_cache *cache, int enable) {
    clear_error();
    if (!cache) return fail(SSD_ERR_INVALID_ARG, "cache is NULL");
    cache->launch_enabled = enable != 0;
    return SSD_OK;
}

int ssd_cache_layer_budget(const ssd_cache *cache, int layer, int32_t *window, int32_t *budget) {
    clear_error();
    int rc = check_layers(cache, layer, layer + 1);
    if (rc != SSD_OK) return rc;
    if (window) *window = cache->Wl[layer];
    if (budget) *budget = cache->Ml[layer];
    return SSD_OK;
}

int ssd_cache_head_budget(const ssd_cache *cache, int layer, int head, int32_t *value) {
    clear_error();
    int rc = check_layers(cache, layer, layer + 1);
    if (rc != SSD_OK) return rc;
    if (head < 0 || head >= cache->cfg.n_heads) return fail(SSD_ERR_INVALID_ARG, "head=%d outside 0..%d", head, cache->cfg.n_heads - 1);
    if (!value) return fail(SSD_ERR_INVALID_ARG, "output pointer is NULL");
    const size_t i = (size_t)layer * cache->cfg.n_heads + head;
    if (per_head(cache)) *value = cache->head_budget[i];
    else *value = cache->head_type[i] == SSD_SEMANTIC ? cache->Ml[layer] : cache->Wl[layer];
    return SSD_OK;
}

int ssd_cache_head_runs(const ssd_cache *cache, int layer, int head, int32_t start[3], int32_t len[3]) {
    clear_error();
    int rc = check_layers(cache, layer, layer + 1);
    if (rc != SSD_OK) return rc;
    if (head < 0 || head >= cache->cfg.n_heads) return fail(SSD_ERR_INVALID_ARG, "head=%d outside 0..%d", head, cache->cfg.n_heads - 1);
    if (!start || !len) return fail(SSD_ERR_INVALID_ARG, "output pointer is NULL");
    const ssd_config &cf = cache->cfg;
    const LayerState &st = cache->st[layer];
    const size_t i = (size_t)layer * cf.n_heads + head;
    Segs s;
    if (cache->head_type[i] == SSD_SEMANTIC) {
        s = semantic_segs(cache, layer, st);
        if (per_head(cache)) s.len[0] = st.m < cache->head_budget[i] ? st.m : cache->head_budget[i];
    } else {
        const int W = per_head(cache) ? cache->head_budget[i] : cache->Wl[layer];
        s = ring_segs(cf.n_init_sink, W, cf.stage_cap, cf.spatial_row_buffer != 0, st.n, st.nc);
    }
    for (int k = 0; k < 3; ++k) { start[k] = s.start[k]; len[k] = s.len[k]; }
    return SSD_OK;
}

int ssd_cache_spatial_slot(const ssd_cache *cache, int layer, int head, int position, int32_t *slot) {
    clear_error();
    int rc = check_layers(cache, layer, layer + 1);
    if (rc != SSD_OK) return rc;
    const ssd_config &cf = cache->cfg;
    if (head < 0 || head >= cf.n_heads) return fail(SSD_ERR_INVALID_ARG, "head=%d outside 0..%d", head, cf.n_heads - 1);
    const size_t i = (size_t)layer * cf.n_heads + head;
    if (cache->head_type[i] != SSD_SPATIAL) return fail(SSD_ERR_INVALID_ARG, "head %d of layer %d is not a spatial head", head, layer);
    if (position < 0 || !slot) return fail(SSD_ERR_INVALID_ARG, "bad position or output pointer");
    const int W = per_head(cache) ? cache->head_budget[i] : cache->Wl[layer];
    *slot = ring_slot(cf.n_init_sink, W + (cf.spatial_row_buffer ? cf.stage_cap : 0), position);
    return SSD_OK;
}

int ssd_cache_export_slots(const ssd_cache *cache) {
    if (!cache) return 0;
    int slots = 0;
    for (int l = 0; l < cache->cfg.n_layers; ++l) {
        const int a = cache->cfg.n_init_sink + cache->Wl[l] + (cache->cfg.spatial_row_buffer ? cache->cfg.stage_cap : 0);
        const int b = cache->Ml[l] + cache->cfg.stage_cap;
        slots = a > slots ? a : slots;
        slots = b > slots ? b : slots;
    }
    return slots;
}

int ssd_cache_export(ssd_cache *cache, int layer, int32_t *pos, int32_t *count, float *score, void *stream) {
    clear_error();
    int rc = check_layers(cache, layer, layer + 1);
    if (rc != SSD_OK) return rc;
    if (!aligned(pos, 4) || !aligned(count, 4) || !aligned(score, 4)) return fail(SSD_ERR_INVALID_ARG, "misaligned output");
    if (!cache->launch_enabled) return SSD_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const LayerState st = cache->st[layer];
    const Segs se = semantic_segs(cache, layer, st);
    const int units = cache->cfg.n_seqs * cache->cfg.n_heads;
    const int ref = cache->cfg.spatial_row_buffer ? st.nc : st.n;      // Algorithm 1: the window always ends at n
    HeadTable ht;
    fill_head_table(cache, layer, &ht);
    hipLaunchKernelGGL(export_kernel, dim3(units), dim3(64), 0, s, make_geom(cache, layer), cache->ldesc[layer], st, se, ref,
                       ssd_cache_export_slots(cache), ht, heads_differ(cache, layer) ? 1 : 0, pos, count, score);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "export launch");
    return SSD_OK;
}

const char *ssd_last_error(void) { return g_err; }

int ssd_version(void) { return 200; }

}  // extern "C"
