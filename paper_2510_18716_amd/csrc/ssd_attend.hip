// ssd_decode_attn: single-token attention over the compressed cache, plus the running-score
// update of semantic heads (Algorithm 1: "AttentionScores", "AggregateAttentionScores").
//
// One wave64 per (layer, sequence, head) unit.  A unit is small (S+W or m+c rows, ~33 KB at
// W = M = 64, d = 128, bf16) and contiguous in HBM, so the kernel is a pure stream: every byte
// is read exactly once, straight into registers (no reuse exists that LDS staging could serve),
// and the launch exposes tens of thousands of independent units to cover HBM latency.
// Spatial and semantic units share one launch; they differ only in where their valid rows are.
//
// Roofline: HBM.  Algorithmic bytes per unit and step = rows * 2 * d * e (K and V) + 2 * d * e
// (q in, out) + 8 * rows for a semantic unit's score read-modify-write.
#include "ssd_device.h"

namespace ssd {

struct AttendArgs {
    Geom g;
    const char *q;
    char *out;
    int layer_begin;
    int layer_off;
    int n_units;
    Segs sp, se;
    float qscale;        // softmax scale * log2(e)
    int accumulate;
    int zcap;            // floats of LDS per wave for the logits of a semantic unit
};

template <typename T, int D, int CH, int WPB>
__global__ __launch_bounds__(WPB * 64) void attend_kernel(AttendArgs a) {
    constexpr int VEC = Elem<T>::VEC;
    constexpr int LPR = D / VEC;
    extern __shared__ float zbuf_all[];
    const int wave = threadIdx.x >> 6;
    const int lane = threadIdx.x & 63;
    const int sub = lane % LPR;
    float *zbuf = zbuf_all + (size_t)wave * a.zcap;
    const int BH = a.g.B * a.g.H;

    for (int unit = blockIdx.x * WPB + wave; unit < a.n_units; unit += gridDim.x * WPB) {
        const int lrel = unit / BH;
        const int rem = unit % BH;
        const int b = rem / a.g.H, h = rem % a.g.H;
        const UnitRef u = unit_ref(a.g, a.layer_begin + lrel, b, h);
        const Segs &sg = u.sem ? a.se : a.sp;
        const size_t qoff = ((size_t)(a.layer_off + lrel) * BH + rem) * (size_t)a.g.row_bytes + (size_t)sub * 16u;

        float q[VEC];
        {
            const uint4 qr = *reinterpret_cast<const uint4 *>(a.q + qoff);
            Elem<T>::unpack(qr, q);
#pragma unroll
            for (int e = 0; e < VEC; ++e) q[e] *= a.qscale;
        }
        Softmax<VEC> sm;
        sm.init();
        const bool want_scores = u.sem && a.accumulate;
        if (want_scores)
            stream_rows<T, D, CH, true, false>(u.K, u.V, a.g.row_bytes, sg, 0, sg.total, q, sm, zbuf, 0, 0);
        else
            stream_rows<T, D, CH, false, false>(u.K, u.V, a.g.row_bytes, sg, 0, sg.total, q, sm, nullptr, 0, 0);
        merge_groups<VEC, LPR, false>(sm);
        const float inv_l = sm.l > 0.f ? 1.0f / sm.l : 0.f;
        if (lane < LPR) {
            float o[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) o[e] = sm.acc[e] * inv_l;
            *reinterpret_cast<uint4 *>(a.out + qoff) = Elem<T>::pack(o);
        }
        if (want_scores) {
            // the logits were written by other lanes of this same wave: order the LDS traffic
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            for (int r = lane; r < sg.total; r += 64) {
                const int slot = seg_slot(sg, r);
                const float p = fast_exp2(zbuf[r] - sm.m) * inv_l;
                u.score[slot] += p;
            }
            // keep the next unit's logits from overtaking these reads
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
        }
    }
}

struct Tuning {
    int ch;      // rows-per-lane-group in flight per loop trip (CH)
    int wpb;     // waves per workgroup
    int upw;     // target units per wave (grid = units / (wpb * upw))
};

static Tuning g_tune = {4, 4, 1};

template <typename T, int D>
static hipError_t launch_attend(const AttendArgs &a, hipStream_t s) {
    const int wpb = g_tune.wpb;
    const int upw = g_tune.upw < 1 ? 1 : g_tune.upw;
    long long waves = ((long long)a.n_units + upw - 1) / upw;
    unsigned blocks = (unsigned)((waves + wpb - 1) / wpb);
    if (blocks < 1) blocks = 1;
    const size_t lds = (size_t)wpb * a.zcap * sizeof(float);
#define SSD_LAUNCH(CH_, WPB_) hipLaunchKernelGGL((attend_kernel<T, D, CH_, WPB_>), dim3(blocks), dim3(WPB_ * 64), lds, s, a)
    if (wpb == 1) {
        if (g_tune.ch == 2) SSD_LAUNCH(2, 1); else if (g_tune.ch == 8) SSD_LAUNCH(8, 1); else SSD_LAUNCH(4, 1);
    } else if (wpb == 2) {
        if (g_tune.ch == 2) SSD_LAUNCH(2, 2); else if (g_tune.ch == 8) SSD_LAUNCH(8, 2); else SSD_LAUNCH(4, 2);
    } else {
        if (g_tune.ch == 2) SSD_LAUNCH(2, 4); else if (g_tune.ch == 8) SSD_LAUNCH(8, 4); else SSD_LAUNCH(4, 4);
    }
#undef SSD_LAUNCH
    return hipGetLastError();
}

}  // namespace ssd

using namespace ssd;

// Launch-shape knobs for benchmarking sweeps (not part of the documented ABI): rows in flight
// per lane group (2, 4, 8), waves per workgroup (1, 2, 4), units per wave (>= 1).
extern "C" int ssd_tune_attend(int ch, int wpb, int upw) {
    if ((ch != 2 && ch != 4 && ch != 8) || (wpb != 1 && wpb != 2 && wpb != 4) || upw < 1) return SSD_ERR_INVALID_ARG;
    g_tune.ch = ch; g_tune.wpb = wpb; g_tune.upw = upw;
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
    if (!cache->launch_enabled) return SSD_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    rc = ensure_meta(cache, s);
    if (rc != SSD_OK) return rc;
    const ssd_config &cf = cache->cfg;
    const int BH = cf.n_seqs * cf.n_heads;
    for (int lb = layer_begin; lb < layer_end;) {
        const int le = same_state_run(cache, lb, layer_end);
        const LayerState st = cache->st[lb];
        AttendArgs a;
        a.g = make_geom(cache);
        a.q = static_cast<const char *>(q);
        a.out = static_cast<char *>(out);
        a.layer_begin = lb;
        a.layer_off = lb - layer_begin;
        a.n_units = (le - lb) * BH;
        a.sp = spatial_segs(cache, st);
        a.se = semantic_segs(cache, st);
        a.qscale = cache->scale * LOG2E;
        a.accumulate = accumulate_scores ? 1 : 0;
        a.zcap = accumulate_scores ? ((a.se.total + 63) / 64) * 64 : 0;
        hipError_t e;
        if (cf.dtype == SSD_BF16)
            e = cf.head_dim == 128 ? launch_attend<bf16_t, 128>(a, s) : launch_attend<bf16_t, 64>(a, s);
        else
            e = cf.head_dim == 128 ? launch_attend<float, 128>(a, s) : launch_attend<float, 64>(a, s);
        if (e != hipSuccess) return hip_fail(e, "attention launch");
        lb = le;
    }
    return SSD_OK;
}
