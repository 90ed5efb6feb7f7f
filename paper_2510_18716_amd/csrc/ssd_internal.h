// Internal declarations shared by the translation units of libssd_hip.so.
// Nothing here is part of the public ABI (that is include/ssd.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "ssd.h"

namespace ssd {

// ---- device-resident layout tables (uploaded once per cache) ---------------

struct LayerMeta {
    uint64_t off_sp;     // byte offset of the spatial heads' K/V units of this layer
    uint64_t off_se;     // byte offset of the semantic heads' K/V units
    uint64_t off_score;  // float [B, Hm_l, M+C]
    uint64_t off_pos;    // int32 [B, Hm_l, M+C]
    int32_t n_sp;        // Hs_l
    int32_t n_se;        // Hm_l
};

// head_info[l*H + h]: bit 31 = head is semantic, bits 0..30 = index among the heads of its type in layer l
static constexpr uint32_t HEAD_SEM_BIT = 0x80000000u;

// Geometry handed to every kernel by value.
struct Geom {
    char *base;               // device memory of the cache
    const LayerMeta *lmeta;   // [L]
    const uint32_t *hinfo;    // [L*H]
    int32_t B, H, S, W, M, C;
    int32_t row_bytes;        // d * element size
    uint32_t unit_sp_bytes;   // 2 * (S+W) * row_bytes : K plane then V plane
    uint32_t unit_se_bytes;   // 2 * (M+C) * row_bytes
};

// Token counters of one layer (host side; equal for all sequences of the batch).
struct LayerState {
    int32_t n;      // tokens appended so far
    int32_t m;      // heavy slots in use: slots [0, m)
    int32_t c;      // row-buffer slots in use
    int32_t base;   // ring index (0..C-1) of the oldest row-buffer slot
    bool operator==(const LayerState &o) const { return n == o.n && m == o.m && c == o.c && base == o.base; }
};

// Up to three runs of consecutive valid slots of a unit, in slot space.
struct Segs {
    int32_t start[3];
    int32_t len[3];
    int32_t total;
};

}  // namespace ssd

struct ssd_cache {
    ssd_config cfg;
    float scale;
    int esize;
    std::vector<uint8_t> head_type;           // [L*H]
    std::vector<ssd::LayerMeta> lmeta;        // host copy of the device tables
    std::vector<uint32_t> hinfo;
    std::vector<ssd::LayerState> st;          // [L]
    char *dev;
    size_t bytes;
    size_t meta_bytes;                        // size of the table region at the start of dev
    bool meta_uploaded;
    bool launch_enabled;
    int n_sp_total, n_se_total;               // heads of each type over all layers
};

namespace ssd {

// error reporting (thread local text behind ssd_last_error)
int fail(int code, const char *fmt, ...);
int hip_fail(hipError_t e, const char *what);
void clear_error();

// host helpers implemented in ssd_cache.hip
int check_layers(const ssd_cache *c, int lb, int le);
int ensure_meta(ssd_cache *c, hipStream_t s);       // uploads the tables on first use
Geom make_geom(const ssd_cache *c);
Segs spatial_segs(const ssd_cache *c, const LayerState &st);
Segs semantic_segs(const ssd_cache *c, const LayerState &st);
// first layer index > lb (and <= le) whose state differs from layer lb's
int same_state_run(const ssd_cache *c, int lb, int le);

static inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

}  // namespace ssd
