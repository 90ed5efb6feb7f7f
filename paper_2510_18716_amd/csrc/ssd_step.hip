// ssd_decode_attn and ssd_decode_step: single-token attention over the compressed cache, the
// running-score update of semantic heads (Algorithm 1: "AttentionScores",
// "AggregateAttentionScores"), and -- in the fused entry point -- the append before it and the
// compression after it, all by the one workgroup that owns the (layer, sequence, head) unit.
//
// One wave64 per unit, a few units per workgroup.  A unit is small (S+W or m+c rows, ~33 KB at
// W = M = 64, d = 128, bf16) and contiguous in HBM, so the kernel is a pure stream: every byte is
// read once, straight into registers (nothing is reused, so there is nothing for LDS staging to
// serve), and a launch exposes thousands of independent units to cover HBM latency.  Spatial and
// semantic units share one launch; they differ only in where their valid rows are.  Because one
// wave owns a unit from the append to the selection, no step needs a workgroup barrier or an atomic.
//
// Roofline: HBM.  Algorithmic bytes per unit and step = rows * 2 * d * e (K and V) + 2 * d * e
// (q in, out) + 8 * rows for a semantic unit's score read-modify-write.
#include "ssd_select.h"

namespace ssd {

// Field order matters: a wave reads its arguments with scalar loads, and every 64-byte line of the
// argument block it touches for the first time is a trip to memory that the whole (in-phase) launch waits
// for.  Everything a unit needs sits in the first lines; the per-layer table, of which a wave reads one
// entry, comes last.
struct StepArgs {
    const char *q;
    char *out;
    const char *k_new;   // fused append only
    const char *v_new;
    float qscale;        // softmax scale * log2(e)
    int layer_off;       // index of the launch's first layer inside q / out / k_new / v_new
    int new_slot_sp;     // fused append: destination slots and position of the new token
    int new_slot_se;
    int new_pos;
    int accumulate;
    int do_compress;     // run the selection after the attention (semantic units)
    int m, c, base, R;   // row-buffer state the selection works on (c counts a fused new token)
    int lpr;
    int zcap;            // floats of LDS per wave for the logits of a semantic unit
    int wave_lds;        // bytes of LDS per wave (logits + selection scratch)
    int probe;           // SSD_PROBE builds only
    int sem_first;       // semantic units have more rows than spatial ones: dispatch them first
    Segs sp, se;         // rows streamed from the cache (fused append: without the new token's slot)
    Geom g;
    LaunchMeta lm;
};

// One wave per unit, WPB units (consecutive heads of one sequence and layer) per workgroup;
// grid = (ceil(H / WPB), B, layers of the launch).  Nothing below needs a workgroup barrier.
#ifdef SSD_PROBE      // probe / 100 == 1: the kernel with its stores left out (what the write path costs)
#define SSD_ST16(ptr, val) do { if (a.probe / 100 != 1) *reinterpret_cast<uint4 *>(ptr) = (val); } while (0)
#define SSD_ST4(ptr, val) do { if (a.probe / 100 != 1) *(ptr) = (val); } while (0)
#else
#define SSD_ST16(ptr, val) (*reinterpret_cast<uint4 *>(ptr) = (val))
#define SSD_ST4(ptr, val) (*(ptr) = (val))
#endif

template <typename T, int D, int CH, int WPB, bool FUSED, bool PF = true>
__global__ __launch_bounds__(WPB * 64) void step_kernel(StepArgs a) {
    constexpr int VEC = Elem<T>::VEC;
    constexpr int LPR = D / VEC;
    extern __shared__ __align__(16) unsigned char lds_raw[];

    // The arguments the tail of a unit needs are fetched now, with everything else, and pinned in scalar
    // registers: fetched lazily they would add a memory round trip to the end of every wave.
    int t_m = a.m, t_c = a.c, t_base = a.base, t_R = a.R, t_lpr = a.lpr, t_new_pos = a.new_pos,
        t_new_slot_se = a.new_slot_se, t_do_compress = a.do_compress, t_accumulate = a.accumulate,
        t_M = a.g.M, t_C = a.g.C, t_row_bytes = a.g.row_bytes;
    asm volatile("" : "+s"(t_m), "+s"(t_c), "+s"(t_base), "+s"(t_R), "+s"(t_lpr), "+s"(t_new_pos), "+s"(t_new_slot_se),
                      "+s"(t_do_compress), "+s"(t_accumulate), "+s"(t_M), "+s"(t_C), "+s"(t_row_bytes));
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: everything per-unit stays uniform
    const int lane = threadIdx.x & 63;
    const int sub = lane % LPR;
    // grid = (ceil(max heads of a type / WPB), B, 2 * layers): z selects the layer and the head type, the type
    // with more rows first, so that within a layer the long units are dispatched before the short ones and
    // all waves of a workgroup have units of one length
    const int lrel = blockIdx.z >> 1;
    const bool sem_unit = ((blockIdx.z & 1) == 0) == (a.sem_first != 0);
    const int local = blockIdx.x * WPB + w;               // index among the heads of this type in this layer
    const LayerDesc &ld = a.lm.layer[lrel];
    if (local >= (sem_unit ? ld.n_se : ld.n_sp)) return;
    const uint64_t m0 = sem_unit ? ld.sem_mask[0] : ~ld.sem_mask[0];
    const uint64_t m1 = sem_unit ? ld.sem_mask[1] : ~ld.sem_mask[1];
    const int h = kth_set_bit(m0, m1, local);             // spatial heads: bits above H are never reached (local < n_sp)
    const int rem = blockIdx.y * a.g.H + h;
    const UnitRef u = unit_ref_local(a.g, ld, blockIdx.y, sem_unit, local);
    const Segs sg = u.sem ? a.se : a.sp;       // by value: the runs stay in scalar registers to the end
    const size_t qoff = ((size_t)(a.layer_off + lrel) * (size_t)(a.g.B * a.g.H) + rem) * (size_t)a.g.row_bytes + (size_t)sub * 16u;
    unsigned char *region = lds_raw + (size_t)w * a.wave_lds;
    float *zbuf = reinterpret_cast<float *>(region);                    // [zcap]
    unsigned char *sel = region + (size_t)a.zcap * 4;                   // selection scratch

    const typename Elem<T>::Q q = Elem<T>::load_q(*reinterpret_cast<const uint4 *>(a.q + qoff));
    Softmax<VEC> sm;
    sm.init();
    const bool want_z = u.sem && t_accumulate;

    // No memory round trip may be left exposed after the last row, so everything the tail of this wave
    // needs is requested around the start of the K/V stream.  The new token's fragments (fused append) are
    // fetched by every lane group alike (the same 16 lines, no extra traffic): only group 0 uses them, but a
    // load under a per-lane condition costs a branch and a wait.
    const bool compress = t_do_compress != 0;
    const bool tail = u.sem && (t_accumulate || compress || FUSED);
    uint4 new_k = make_uint4(0, 0, 0, 0), new_v = make_uint4(0, 0, 0, 0);
    if (FUSED) {
        new_k = *reinterpret_cast<const uint4 *>(a.k_new + qoff);
        new_v = *reinterpret_cast<const uint4 *>(a.v_new + qoff);
    }
    float pre_score[2] = {0.f, 0.f};
    int pre_pos[2] = {0, 0};

    // Runs once, right after the stream's first loads have been issued, so that nothing here delays them:
    //  - fused append: the new token's rows go to their slot now and drain during the stream instead of in
    //    the tail of the unit;
    //  - the running scores and positions of the first 128 rows (one or two per lane) are requested now and
    //    have long arrived when the tail needs them.  The loads are unconditional (rows past the end are
    //    clamped to a valid slot and ignored later): a load under a per-lane condition makes the compiler
    //    wait for it on the spot.
    auto after_first_issue = [&]() {
        if (FUSED && lane < LPR) {
            const int slot = u.sem ? a.new_slot_se : a.new_slot_sp;
            const size_t off = (size_t)slot * (size_t)a.g.row_bytes + (size_t)sub * 16u;
            SSD_ST16(u.K + off, new_k);
            SSD_ST16(u.V + off, new_v);
        }
        if (tail) {
            const int last = sg.total > 0 ? sg.total - 1 : 0;    // no rows yet: slot of row 0, inside the unit
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int r = lane + 64 * k;
                const int slot = seg_slot(sg, r < last ? r : last);
                pre_score[k] = u.score[slot];
                pre_pos[k] = u.pos[slot];
            }
        }
    };
#ifdef SSD_PROBE
    if (a.probe % 100 == 2 || a.probe % 100 == 3 || a.probe % 100 >= 10) { sm.l = 1.f; after_first_issue(); } else
#endif
    if (want_z)
        stream_rows<T, D, CH, true, false, PF>(u.K, u.V, a.g.row_bytes, sg, 0, sg.total, 0, 1, q, a.qscale, sm, zbuf, 0, 0, a.probe, after_first_issue);
    else
        stream_rows<T, D, CH, false, false, PF>(u.K, u.V, a.g.row_bytes, sg, 0, sg.total, 0, 1, q, a.qscale, sm, nullptr, 0, 0, a.probe, after_first_issue);
    if (FUSED) {
        // The new token, from the registers it was loaded into, is folded into lane group 0's softmax as
        // one more row (index sg.total).
        const float z = group_sum<LPR>(Elem<T>::dot(q, new_k)) * a.qscale;
        if (lane < LPR) {
            const float m_new = fmaxf(sm.m, z);
            const float alpha = fast_exp2(sm.m - m_new);
            const float p = fast_exp2(z - m_new);
            float vf[VEC];
            Elem<T>::unpack(new_v, vf);
            sm.l = sm.l * alpha + p;
#pragma unroll
            for (int e = 0; e < VEC; ++e) sm.acc[e] = fmaf(p, vf[e], sm.acc[e] * alpha);
            sm.m = m_new;
            if (want_z && lane == 0) zbuf[sg.total] = z;
        }
    }
    merge_groups<VEC, LPR, false>(sm);
    const float m_all = sm.m;
    const float inv_l = sm.l > 0.f ? 1.0f / sm.l : 0.f;
#ifdef SSD_PROBE
    if (a.probe % 10 == 3) return;
#endif
    if (lane < LPR) {
        float o[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = sm.acc[e] * inv_l;
        SSD_ST16(a.out + qoff, Elem<T>::pack(o));
    }

    if (!tail) return;
#ifdef SSD_PROBE
    if (a.probe % 10 == 4) return;
#endif
    lds_sync();                                           // the logits written by the group leaders
    const int M = t_M, C = t_C;
    const int n_old = t_c - t_R;                          // buffered tokens that become candidates
    const int n_cand = t_m + n_old;
    const int n_evict = n_cand - M;                       // <= 0: everything is kept
    // At most one eviction among at most 128 candidates (always the case when compressing after every
    // token) is settled in registers; anything else ranks all candidates through LDS.
    const bool general = compress && (n_evict >= 2 || n_cand > 128);
    unsigned long long *keys = reinterpret_cast<unsigned long long *>(sel);
    unsigned long long my_key[2] = {~0ull, ~0ull};        // keys of rows lane and lane + 64, if candidates
    const int total = sg.total + (FUSED ? 1 : 0);
    // One row's share: add the probability to its running score, note position and key.
    auto score_row = [&](int r, float s_old, int pos_old) -> unsigned long long {
        const bool is_new = FUSED && r == sg.total;
        const int slot = is_new ? t_new_slot_se : seg_slot(sg, r);
        const float p = t_accumulate ? fast_exp2(zbuf[r] - m_all) * inv_l : 0.f;
        const float s = (is_new ? 0.f : s_old) + p;
        if (t_accumulate || is_new) SSD_ST4(&u.score[slot], s);
        if (is_new) SSD_ST4(&u.pos[slot], t_new_pos);
        unsigned long long key = ~0ull;
        if (compress && r < n_cand) {
            key = make_key(s, is_new ? t_new_pos : pos_old);
            if (general) keys[r] = key;
        }
        return key;
    };
    // rows 0..127 use the scores and positions fetched before the stream: no load, and therefore no wait
    // on this wave's own stores, in the common case
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int r = lane + 64 * k;
        if (r < total) my_key[k] = score_row(r, pre_score[k], pre_pos[k]);
    }
    for (int r = lane + 128; r < total; r += 64) {       // long row buffers only
        const bool is_new = FUSED && r == sg.total;
        const int slot = is_new ? t_new_slot_se : seg_slot(sg, r);
        score_row(r, is_new ? 0.f : u.score[slot], (is_new || !compress) ? 0 : u.pos[slot]);
    }
    if (!compress) return;
#ifdef SSD_PROBE
    if (a.probe % 10 == 5) return;
#endif
    if (general) {
        lds_sync();
        select_and_move<64, true>(a.g, u, sel, n_cand, t_m, n_old, t_base, t_lpr, lane);
        return;
    }
    // The promoted buffered tokens and the slots they go to follow from the index of the single evicted
    // candidate (the one with the smallest key), if any.
    int e_idx = -1;
    if (n_evict == 1) {
        const unsigned long long min_key = wave_min_u64(my_key[0] < my_key[1] ? my_key[0] : my_key[1]);
        const unsigned long long hit0 = __ballot(my_key[0] == min_key);
        const unsigned long long hit1 = __ballot(my_key[1] == min_key);
        e_idx = hit0 ? __builtin_ctzll(hit0) : 64 + __builtin_ctzll(hit1);
    }
#ifdef SSD_PROBE
    if (a.probe % 10 == 6) return;
#endif
    const bool ev_heavy = e_idx >= 0 && e_idx < t_m;
    const bool ev_staged = e_idx >= t_m;
    const int n_move = n_old - (ev_staged ? 1 : 0);
    if (n_move <= 0) return;
    wave_global_sync();                                   // rows / scores stored earlier by other lanes of this wave
    const int frag_per_tok = 2 * t_lpr;
    // k-th promoted candidate (oldest first) and k-th free heavy slot
    auto src_idx = [&](int k) { return t_m + k + ((ev_staged && k >= e_idx - t_m) ? 1 : 0); };
    auto dst_slot = [&](int k) { return ev_heavy ? (k == 0 ? e_idx : t_m + k - 1) : t_m + k; };
    for (int t = lane; t < n_move * frag_per_tok; t += 64) {
        const int k = t / frag_per_tok;
        const int f = t % frag_per_tok;
        const int kv = f / t_lpr, fs = f % t_lpr;
        char *plane = kv ? u.V : u.K;
        const int from = M + (t_base + (src_idx(k) - t_m)) % C;
        const uint4 v = *reinterpret_cast<const uint4 *>(plane + (size_t)from * t_row_bytes + (size_t)fs * 16u);
        *reinterpret_cast<uint4 *>(plane + (size_t)dst_slot(k) * t_row_bytes + (size_t)fs * 16u) = v;
    }
    // position and score travel with the token: its key sits in the registers of lane (index mod 64)
    for (int k0 = 0; k0 < n_move; k0 += 64) {             // wave-uniform trip count: the shuffles need every lane
        const int k = k0 + lane;
        const int src = k < n_move ? src_idx(k) : 0;
        const unsigned long long c0 = __shfl(my_key[0], src & 63);
        const unsigned long long c1 = __shfl(my_key[1], src & 63);
        const unsigned long long key = src < 64 ? c0 : c1;
        if (k < n_move) {
            u.pos[dst_slot(k)] = key_pos(key);
            u.score[dst_slot(k)] = key_score(key);
        }
    }
}

struct Tuning {
    int ch;      // wave-wide loads of K (and of V) per chunk; two chunks are in flight per wave (0 = by launch size)
    int wpb;     // units (waves) per workgroup (0 = by launch size)
};

static int g_probe = 0;
static constexpr Tuning DEFAULT_TUNE = {0, 0};
static Tuning g_tune = DEFAULT_TUNE;

// Largest candidate count the fused entry point ranks with a single wave; beyond it the stand-alone
// compression kernel (a whole workgroup per head) runs after the attention.
static constexpr int FUSED_SELECT_MAX = 1024;

template <typename T, int D, int CH, int WPB, bool PF = true>
static void launch_one(const StepArgs &a, dim3 blocks, size_t lds, bool fused, hipStream_t s) {
    if (fused) hipLaunchKernelGGL((step_kernel<T, D, CH, WPB, true, PF>), blocks, dim3(WPB * 64), lds, s, a);
    else hipLaunchKernelGGL((step_kernel<T, D, CH, WPB, false, PF>), blocks, dim3(WPB * 64), lds, s, a);
}

template <typename T, int D>
static hipError_t launch_step(StepArgs &a, int H, int max_type_heads, int B, int layers, bool fused, int M, hipStream_t s) {
    const int n_old = a.c - a.R, n_cand = a.m + n_old;
    // Launch shape by the number of units (measured on the 7B- and 1B-shaped workloads).  Up to half of
    // what the chip holds at once (256 CUs x 16 waves): the launch is latency-bound, so spread the waves
    // over as many CUs as possible (one unit per workgroup) and give each a deep load queue.  Around one
    // resident round: shallow queues finish sooner.  Many rounds: waves come and go, deeper per-wave
    // queues keep HBM busier.
    const long long units = (long long)H * B * layers;
    int ch = g_tune.ch ? g_tune.ch : (units <= 2048 || units > 16384 ? 4 : 2);
    int wpb = g_tune.wpb ? g_tune.wpb : (units <= 2048 ? 1 : 4);
    a.wave_lds = (int)(((size_t)a.zcap * 4 + (a.do_compress ? select_lds_bytes(M, n_cand, n_old) + 16 : 0) + 15) / 16 * 16);
    while (wpb > 1 && (size_t)wpb * a.wave_lds > 60000) wpb >>= 1;
    size_t lds = (size_t)wpb * a.wave_lds;
#ifdef SSD_PROBE
    if ((size_t)(g_probe / 1000) * 1024 > lds) lds = (size_t)(g_probe / 1000) * 1024;   // occupancy experiments: pad the workgroup's LDS
#endif
    const dim3 blocks((unsigned)((max_type_heads + wpb - 1) / wpb), (unsigned)B, (unsigned)(2 * layers));
#define SSD_CASE(CH_, WPB_) if (ch == CH_ && wpb == WPB_) { launch_one<T, D, CH_, WPB_>(a, blocks, lds, fused, s); return hipGetLastError(); }
    if constexpr (sizeof(T) == 2 && D == 128) {       // the shape the sweeps are run on has every variant
        SSD_CASE(1, 1) SSD_CASE(2, 1) SSD_CASE(4, 1)
        SSD_CASE(1, 2) SSD_CASE(2, 2) SSD_CASE(4, 2)
        SSD_CASE(1, 4) SSD_CASE(2, 4) SSD_CASE(4, 4)
#ifdef SSD_PROBE
#define SSD_CASE_NPF(CODE_, CH_, WPB_) if (ch == CODE_ && wpb == WPB_) { launch_one<T, D, CH_, WPB_, false>(a, blocks, lds, fused, s); return hipGetLastError(); }
        SSD_CASE_NPF(14, 4, 4) SSD_CASE_NPF(18, 8, 4) SSD_CASE_NPF(14, 4, 8) SSD_CASE_NPF(18, 8, 8) SSD_CASE_NPF(18, 8, 2) SSD_CASE(4, 8) SSD_CASE(2, 8)
#undef SSD_CASE_NPF
#endif
    } else {
        if (ch == 1) ch = 2;
        SSD_CASE(2, 1) SSD_CASE(4, 1) SSD_CASE(2, 2) SSD_CASE(4, 2) SSD_CASE(2, 4) SSD_CASE(4, 4)
    }
#undef SSD_CASE
    return hipErrorInvalidValue;
}

// Shared by ssd_decode_attn (k_new == NULL, compress == 0) and ssd_decode_step.
static int run_step(ssd_cache *cache, int layer_begin, int layer_end, const void *q, const void *k_new, const void *v_new,
                    void *out, int accumulate, int compress, void *stream, const char *what) {
    const ssd_config &cf = cache->cfg;
    const bool fused = k_new != nullptr;
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int lb = layer_begin; lb < layer_end;) {
        const int le = same_state_run(cache, lb, layer_end);
        const LayerState before = cache->st[lb];
        const bool has_se = cache->ldesc[lb].n_se > 0;     // uniform over the run, like the row-buffer flag
        const bool has_buf = has_buffer(cache, lb);
        LayerState at = before;                      // state the attention sees
        if (fused) { at.n += 1; if (has_buf) at.c += 1; }
        const int n_old = at.c - cf.recent;
        const bool do_compress = compress && has_se && n_old > 0;
        const bool in_kernel = do_compress && at.m + n_old <= FUSED_SELECT_MAX;
        if (cache->launch_enabled) {
            StepArgs a;
            a.g = make_geom(cache, lb);
            fill_launch_meta(cache, lb, le, &a.lm);
            a.q = static_cast<const char *>(q);
            a.out = static_cast<char *>(out);
            a.k_new = static_cast<const char *>(k_new);
            a.v_new = static_cast<const char *>(v_new);
            a.layer_off = lb - layer_begin;
            a.new_pos = before.n;
            a.new_slot_sp = spatial_slot(cache, lb, before.n);
            a.new_slot_se = cache->Ml[lb] + (before.base + before.c) % cf.stage_cap;
            if (fused) {
                a.sp = spatial_segs_fused(cache, lb, before, at, a.new_slot_sp);
                a.se = semantic_segs(cache, lb, before);
            } else {
                a.sp = spatial_segs(cache, lb, at);
                a.se = semantic_segs(cache, lb, at);
            }
            a.qscale = cache->scale * LOG2E;
            a.accumulate = accumulate ? 1 : 0;
            a.zcap = ((a.se.total + 1 + 63) / 64) * 64;
            a.do_compress = in_kernel ? 1 : 0;
            a.m = at.m; a.c = at.c; a.base = at.base; a.R = cf.recent;
            a.lpr = a.g.row_bytes / 16;
            a.probe = g_probe;
            int mth = 1;
            for (int l = lb; l < le; ++l) {
                mth = cache->ldesc[l].n_sp > mth ? cache->ldesc[l].n_sp : mth;
                mth = cache->ldesc[l].n_se > mth ? cache->ldesc[l].n_se : mth;
            }
            a.sem_first = a.se.total + (fused ? 1 : 0) >= a.sp.total + (fused ? 1 : 0) ? 1 : 0;
            hipError_t e;
            if (cf.dtype == SSD_BF16)
                e = cf.head_dim == 128 ? launch_step<bf16_t, 128>(a, cf.n_heads, mth, cf.n_seqs, le - lb, fused, cache->Ml[lb], s)
                                       : launch_step<bf16_t, 64>(a, cf.n_heads, mth, cf.n_seqs, le - lb, fused, cache->Ml[lb], s);
            else
                e = cf.head_dim == 128 ? launch_step<float, 128>(a, cf.n_heads, mth, cf.n_seqs, le - lb, fused, cache->Ml[lb], s)
                                       : launch_step<float, 64>(a, cf.n_heads, mth, cf.n_seqs, le - lb, fused, cache->Ml[lb], s);
            if (e != hipSuccess) return hip_fail(e, what);
            if (do_compress && !in_kernel) {
                const int rc = launch_compress_inplace(cache, lb, le, at, s);
                if (rc != SSD_OK) return rc;
            }
        }
        for (int l = lb; l < le; ++l) {
            LayerState &x = cache->st[l];
            if (fused) { x.n += 1; if (has_buf) x.c += 1; }
            if (compress) apply_compress_counters(cache, l);
        }
        lb = le;
    }
    return SSD_OK;
}

}  // namespace ssd

using namespace ssd;

// Launch-shape knobs for benchmarking sweeps (not part of the documented ABI): wave-wide loads per
// chunk (1, 2, 4; 0 = chosen from the launch size) and units per workgroup (1, 2, 4); (0, 0) restores
// the default.
extern "C" int ssd_tune_attend(int ch, int wpb, int probe) {
    g_probe = probe;
    if (ch == 0 && wpb == 0) { g_tune = DEFAULT_TUNE; return SSD_OK; }
#ifndef SSD_PROBE
    if ((ch != 0 && ch != 1 && ch != 2 && ch != 4) || (wpb != 0 && wpb != 1 && wpb != 2 && wpb != 4)) return SSD_ERR_INVALID_ARG;
#endif
    g_tune.ch = ch; g_tune.wpb = wpb;
    return SSD_OK;
}

extern "C" int ssd_decode_attn(ssd_cache *cache, int layer_begin, int layer_end, const void *q, void *out,
                               int accumulate_scores, void *stream) {
    clear_error();
    int rc = check_layers(cache, layer_begin, layer_end);
    if (rc != SSD_OK) return rc;
    if (!q || !out) return fail(SSD_ERR_INVALID_ARG, "q or out is NULL");
    if (!aligned(q, 16) || !aligned(out, 16)) return fail(SSD_ERR_INVALID_ARG, "q / out must be 16-byte aligned");
    for (int l = layer_begin; l < layer_end; ++l)
        if (cache->st[l].n < 1) return fail(SSD_ERR_ORDER, "layer %d holds no token: call ssd_append_token first", l);
    return run_step(cache, layer_begin, layer_end, q, nullptr, nullptr, out, accumulate_scores, 0, stream, "attention launch");
}

extern "C" int ssd_decode_step(ssd_cache *cache, int layer_begin, int layer_end, const void *q, const void *k_new,
                               const void *v_new, void *out, int accumulate_scores, int compress, void *stream) {
    clear_error();
    int rc = check_layers(cache, layer_begin, layer_end);
    if (rc != SSD_OK) return rc;
    if (!q || !out || !k_new || !v_new) return fail(SSD_ERR_INVALID_ARG, "q, k_new, v_new or out is NULL");
    if (!aligned(q, 16) || !aligned(out, 16) || !aligned(k_new, 16) || !aligned(v_new, 16))
        return fail(SSD_ERR_INVALID_ARG, "q / k_new / v_new / out must be 16-byte aligned");
    for (int l = layer_begin; l < layer_end; ++l)
        if (has_buffer(cache, l) && cache->st[l].c >= cache->cfg.stage_cap)
            return fail(SSD_ERR_STAGE_OVERFLOW, "row buffer overflow: layer %d already buffers %d tokens (C=%d); call ssd_compress_kv",
                        l, cache->st[l].c, cache->cfg.stage_cap);
    return run_step(cache, layer_begin, layer_end, q, k_new, v_new, out, accumulate_scores, compress, stream, "decode step launch");
}
