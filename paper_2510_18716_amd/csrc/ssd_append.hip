// ssd_append_token: write the new token's K and V rows into every head's cache
// (Algorithm 1 "Append"; Algorithm 2 "Append k_t, v_t to row buffer").
//
// Pure data movement: one lane moves one 16-byte fragment, so a row is a run of adjacent lanes
// on both the read side (k_new/v_new, [L',B,H,d]) and the write side (the unit's slot).
#include "ssd_device.h"

namespace ssd {

struct AppendArgs {
    Geom g;
    LaunchMeta lm;
    const char *k_new;
    const char *v_new;
    int layer_off;       // index of that layer inside k_new / v_new
    int n_units;         // layers * B * H
    int lpr;             // 16-byte fragments per row
    int slot_sp;         // destination slot of spatial heads
    int slot_se;         // destination slot of semantic heads
    int pos;             // absolute position of the token
    int heads;           // budgets per head: a spatial head's slot follows from its own window
    HeadTable ht;
};

__global__ __launch_bounds__(256) void append_kernel(AppendArgs a) {
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int frag_per_unit = 2 * a.lpr;
    const long long unit_ll = t / frag_per_unit;
    if (unit_ll >= a.n_units) return;
    const int unit = (int)unit_ll;
    const int f = (int)(t % frag_per_unit);
    const int kv = f / a.lpr;          // 0 = K, 1 = V
    const int sub = f % a.lpr;
    const int BH = a.g.B * a.g.H;
    const int lrel = unit / BH;
    const int rem = unit % BH;
    const int b = rem / a.g.H, h = rem % a.g.H;
    const UnitRef u = unit_ref(a.g, a.lm.layer[lrel], b, h);
    const size_t src_row = ((size_t)(a.layer_off + lrel) * BH + rem) * (size_t)a.g.row_bytes;
    const char *src = (kv ? a.v_new : a.k_new) + src_row + (size_t)sub * 16u;
    int slot = u.sem ? a.slot_se : a.slot_sp;
    if (a.heads && !u.sem) slot = ring_slot(a.g.S, a.ht.v[h] + (a.g.RW - a.g.W), a.pos);
    char *dst = (kv ? u.V : u.K) + (size_t)slot * (size_t)a.g.row_bytes + (size_t)sub * 16u;
    *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src);
    if (u.sem && f == 0) {
        u.pos[slot] = a.pos;
        u.score[slot] = 0.f;
    }
}

}  // namespace ssd

using namespace ssd;

extern "C" int ssd_append_token(ssd_cache *cache, int layer_begin, int layer_end, const void *k_new,
                                const void *v_new, void *stream) {
    clear_error();
    int rc = check_layers(cache, layer_begin, layer_end);
    if (rc != SSD_OK) return rc;
    if (!k_new || !v_new) return fail(SSD_ERR_INVALID_ARG, "k_new or v_new is NULL");
    if (!aligned(k_new, 16) || !aligned(v_new, 16)) return fail(SSD_ERR_INVALID_ARG, "k_new / v_new must be 16-byte aligned");
    const ssd_config &cf = cache->cfg;
    // a full row buffer in any layer refuses the whole call (nothing is appended anywhere)
    for (int l = layer_begin; l < layer_end; ++l)
        if (has_buffer(cache, l) && cache->st[l].c >= cf.stage_cap)
            return fail(SSD_ERR_STAGE_OVERFLOW, "row buffer overflow: layer %d already buffers %d tokens (C=%d); call ssd_compress_kv",
                        l, cache->st[l].c, cf.stage_cap);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int BH = cf.n_seqs * cf.n_heads;
    for (int lb = layer_begin; lb < layer_end;) {
        const int le = same_state_run(cache, lb, layer_end);
        const LayerState st = cache->st[lb];
        if (cache->launch_enabled) {
            AppendArgs a;
            a.g = make_geom(cache, lb);
            a.k_new = static_cast<const char *>(k_new);
            a.v_new = static_cast<const char *>(v_new);
            fill_launch_meta(cache, lb, le, &a.lm);
            a.layer_off = lb - layer_begin;
            a.n_units = (le - lb) * BH;
            a.lpr = a.g.row_bytes / 16;
            a.pos = st.n;
            a.slot_sp = spatial_slot(cache, lb, st.n);
            a.slot_se = cache->Ml[lb] + (st.base + st.c) % cf.stage_cap;
            a.heads = heads_differ(cache, lb) ? 1 : 0;
            fill_head_table(cache, lb, &a.ht);
            const long long threads = (long long)a.n_units * 2 * a.lpr;
            const unsigned blocks = (unsigned)((threads + 255) / 256);
            hipLaunchKernelGGL(append_kernel, dim3(blocks), dim3(256), 0, s, a);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return hip_fail(e, "append launch");
        }
        for (int l = lb; l < le; ++l) {
            cache->st[l].n += 1;
            if (has_buffer(cache, l)) cache->st[l].c += 1;       // a layer of Algorithm-1 spatial heads only has no row buffer
        }
        lb = le;
    }
    return SSD_OK;
}
