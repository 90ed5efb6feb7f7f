// Internal declarations shared by the translation units of libssd_hip.so.
// Nothing here is part of the public ABI (that is include/ssd.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "ssd.h"
#include "ssd_hooks.h"

namespace ssd {

// ---- layout description handed to kernels by value (kernel arguments) -------
//
// Everything a wave needs to find its unit arrives in the kernel-argument segment, so address
// computation is scalar arithmetic and the first K/V loads of a wave depend on no earlier load.

static constexpr int LMAX = 32;   // layers one launch can cover

struct LayerDesc {
    uint64_t off_sp;        // byte offset of the spatial heads' K/V units of this layer
    uint64_t off_se;        // byte offset of the semantic heads' K/V units
    uint64_t off_score;     // float [B, Hm_l, M+C]
    uint64_t off_pos;       // int32 [B, Hm_l, M+C]
    uint64_t sem_mask[2];   // bit h set = head h of this layer is a semantic head (H <= 128)
    int32_t n_sp;           // Hs_l
    int32_t n_se;           // Hm_l
};

struct LaunchMeta {
    LayerDesc layer[LMAX];
};

// Geometry common to all layers of one launch (layers with different W or M go to different launches).
struct Geom {
    char *base;               // device memory of the cache
    int32_t B, H, S, W, M, C;
    int32_t RW;               // ring slots of a spatial head: W, or W + C when spatial heads use the row buffer
    int32_t row_bytes;        // d * element size
    uint32_t unit_sp_bytes;   // 2 * (S+RW) * row_bytes : K plane then V plane
    uint32_t unit_se_bytes;   // 2 * (M+C) * row_bytes
};

// Token counters of one layer (host side; equal for all sequences of the batch).
struct LayerState {
    int32_t n;      // tokens appended so far
    int32_t m;      // heavy slots in use: slots [0, m)
    int32_t c;      // row-buffer slots in use
    int32_t base;   // ring index (0..C-1) of the oldest row-buffer slot
    int32_t nc;     // tokens held at the last compression (start of the spatial row buffer, Algorithm 2)
    bool operator==(const LayerState &o) const { return n == o.n && m == o.m && c == o.c && base == o.base && nc == o.nc; }
};

// Up to three runs of consecutive valid slots of a unit, in slot space.
struct Segs {
    int32_t start[3];
    int32_t len[3];
    int32_t total;
};

// Budgets per head (caches made by ssd_cache_init_heads): entry h is head h's own window W_h if it is a
// spatial head, its own heavy-hitter budget M_h if it is a semantic head.  Units keep the layer-wide size
// (the largest W_h / M_h of the layer, which is what Geom holds); a head uses only its own share of the slots.
// One layer per launch, so one table per launch, passed with the kernel arguments.
static constexpr int HMAX = 128;  // heads per layer
struct HeadTable {
    uint16_t v[HMAX];
};

// ---- slot arithmetic of a spatial unit, the same on the host and in kernels ----
// S sink slots, then a ring of RW slots (RW = W, or W + C when spatial heads use the row buffer).
__host__ __device__ inline int ring_slot(int S, int RW, int p) { return p < S ? p : S + (p - S) % RW; }

// Valid slots of a spatial unit that holds n tokens, the last compression having happened at nc tokens.
__host__ __device__ inline Segs ring_segs(int S, int W, int C, bool row_buffer, int n, int nc) {
    Segs s = {{0, 0, 0}, {0, 0, 0}, 0};
    if (!row_buffer) {
        // Algorithm 1: the ring fills front to back, so the valid slots are always a prefix
        const int cap = S + W;
        s.len[0] = n < cap ? n : cap;
        s.total = s.len[0];
        return s;
    }
    // Algorithm 2: sinks, then positions [max(S, nc - W), n) in a ring of W + C slots
    const int RW = W + C;
    s.len[0] = n < S ? n : S;
    const int lo = nc - W > S ? nc - W : S;
    const int count = n > lo ? n - lo : 0;
    const int start = S + (lo - S) % RW;
    const int first = count < S + RW - start ? count : S + RW - start;
    s.start[1] = start; s.len[1] = first;
    s.start[2] = S;     s.len[2] = count - first;
    s.total = s.len[0] + s.len[1] + s.len[2];
    return s;
}

// Rows a fused append + attention streams from a spatial unit that held n tokens before the append: everything
// retained after it except the new token itself (which the kernel holds in registers), whose slot is new_slot.
__host__ __device__ inline Segs ring_segs_fused(int S, int W, int C, bool row_buffer, int n, int nc, int new_slot) {
    if (row_buffer) return ring_segs(S, W, C, true, n, nc);     // the new token's slot is never a retained one
    // Algorithm 1: the new token overwrites the oldest ring slot; stream the prefix around it
    Segs s = ring_segs(S, W, C, false, n + 1, nc);
    const int end = s.len[0];
    if (new_slot < 0 || new_slot >= end) return s;
    s.start[0] = 0;            s.len[0] = new_slot;
    s.start[1] = new_slot + 1; s.len[1] = end - new_slot - 1;
    s.total = end - 1;
    return s;
}

// Override of the attention / step launch shape, kept per cache (0 = the library's choice by launch size).
struct LaunchShape {
    int ch;        // wave-wide loads of K (and of V) per chunk: 1, 2, 4
    int wpb;       // units per workgroup: 1, 2, 4; 12 / 14: one unit per workgroup shared by 2 / 4 waves
    int new_rows;  // fused step: 1 = store the new token's rows at the start of the row stream, 2 = after it
};

}  // namespace ssd

struct ssd_cache {
    ssd_config cfg;
    float scale;
    int esize;
    std::vector<uint8_t> head_type;           // [L*H]
    std::vector<ssd::LayerDesc> ldesc;        // [L]
    std::vector<int32_t> Wl, Ml;              // [L] window and budget of each layer (cfg.window / cfg.budget unless given per layer);
                                              //     with budgets per head: the largest of the layer, which sizes its units
    std::vector<uint16_t> head_budget;        // [L*H] W_h of a spatial head, M_h of a semantic head; empty unless given per head
    std::vector<uint8_t> heads_differ;        // [L] 1 where the heads of one type do not all share one budget (empty unless given per head)
    std::vector<ssd::LayerState> st;          // [L]
    char *dev;
    size_t bytes;
    bool launch_enabled;
    ssd::LaunchShape shape;                   // test / sweep override of the attention launch shape (all 0: chosen by launch size)
    ssd::LaunchShape last_shape;              // shape the newest attention / step launch took (read back by a test hook)
    hipEvent_t ev_fork, ev_join[SSD_MAX_SPLIT];   // ssd_decode_step_split: made on first use, timing disabled
    bool have_events;
};

namespace ssd {

// error reporting (thread local text behind ssd_last_error)
int fail(int code, const char *fmt, ...);
int hip_fail(hipError_t e, const char *what);
void clear_error();

// host helpers implemented in ssd_cache.hip
int check_layers(const ssd_cache *c, int lb, int le);
int ensure_events(ssd_cache *c);                                               // events of ssd_decode_step_split
Geom make_geom(const ssd_cache *c, int l);                                     // geometry of layer l
void fill_launch_meta(const ssd_cache *c, int lb, int le, LaunchMeta *out);   // le - lb <= LMAX
Segs spatial_segs(const ssd_cache *c, int l, const LayerState &st);
Segs semantic_segs(const ssd_cache *c, int l, const LayerState &st);
// Rows a fused append + attention streams from a spatial unit: everything retained after the append except
// the new token itself (which the kernel holds in registers); new_slot is where that token goes.
Segs spatial_segs_fused(const ssd_cache *c, int l, const LayerState &before, const LayerState &after, int new_slot);
// slot of position p in a spatial unit of layer l
int spatial_slot(const ssd_cache *c, int l, int p);
// host bookkeeping of one in-place compression of layer l (the kernels' effect on the counters)
void apply_compress_counters(ssd_cache *c, int l);
// does layer l keep a row buffer (semantic heads, or spatial heads under Algorithm 2)
bool has_buffer(const ssd_cache *c, int l);
// budgets given per head?
static inline bool per_head(const ssd_cache *c) { return !c->head_budget.empty(); }
// ... and do they differ inside layer l?  (then a launch covers that one layer and carries its HeadTable; a layer
// whose heads agree is an ordinary layer with that window and budget)
static inline bool heads_differ(const ssd_cache *c, int l) { return per_head(c) && c->heads_differ[l] != 0; }
void fill_head_table(const ssd_cache *c, int l, HeadTable *out);
// end of the run of layers starting at lb that share layer lb's state, window and budget, at most LMAX long
// (one layer when budgets are per head)
int same_state_run(const ssd_cache *c, int lb, int le);
// the same without the state: layers that share layer lb's window and budget
int same_geom_run(const ssd_cache *c, int lb, int le);

// implemented in ssd_compress.hip
int launch_compress_inplace(const ssd_cache *cache, int lb, int le, const LayerState &st, int seq_off, int n_seq, hipStream_t s);

static inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace ssd
