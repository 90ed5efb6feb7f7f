// ssd_dense_decode_attn: single-token attention over a full, uncompressed cache -- the "Full Cache"
// baseline of Sec. 4.1 -- which also emits, per (sequence, head), the two attention masses the
// sparsity metric of Sec. 3.3 is built from (mass on all visual rows, mass on visual rows older
// than the recency window).
//
// Same streaming loop as the compressed kernel, over rows 0..n-1 of a [B, H, n_cap, d] cache.
// With only B*H units per layer and n up to a few thousand rows, the rows of a unit are split
// over several waves (split-K); each wave leaves an unnormalised partial (max, sum, masses,
// output) in a caller-provided workspace and a second small kernel merges them.
// Roofline: HBM; algorithmic bytes per unit = n * 2 * d * e.
#include <mutex>
#include <type_traits>

#include "ssd_device.h"

namespace ssd {

struct DenseArgs {
    const char *q;
    const char *K;
    const char *V;
    char *out;
    float *ws;          // [units, splits, 4 + D] when splits > 1
    float *far;
    float *tot;
    int n_units;
    int n_cap;
    int n;
    int row_bytes;
    int splits;
    int rows_per_split;
    int mass_stride;
    int vis_start;
    int far_last;       // last row index that counts as "far": n - 1 - w
    float qscale;
};

// passed to the kernels by value: plain data, 7 pointers and 10 four-byte fields, no padding
static_assert(sizeof(DenseArgs) == 96 && alignof(DenseArgs) == 8 && std::is_trivially_copyable<DenseArgs>::value,
              "DenseArgs is copied into the kernel-argument segment as it is");

template <typename T, int D, int CH, int WPB>
__global__ __launch_bounds__(WPB * 64) void dense_kernel(DenseArgs a) {
    constexpr int VEC = Elem<T>::VEC;
    constexpr int LPR = D / VEC;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    const int sub = lane % LPR;
    const long long item = (long long)blockIdx.x * WPB + wave;       // unit * splits + split
    if (item >= (long long)a.n_units * a.splits) return;
    const int unit = (int)(item / a.splits);
    const int split = (int)(item % a.splits);
    const size_t qoff = (size_t)unit * a.row_bytes + (size_t)sub * 16u;
    const typename Elem<T>::Q q = Elem<T>::load_q(*reinterpret_cast<const uint4 *>(a.q + qoff));
    const char *Kb = a.K + (size_t)unit * (size_t)a.n_cap * (size_t)a.row_bytes;
    const char *Vb = a.V + (size_t)unit * (size_t)a.n_cap * (size_t)a.row_bytes;
    Segs sg = {{0, 0, 0}, {a.n, 0, 0}, a.n};
    const int r_begin = split * a.rows_per_split;
    int r_end = r_begin + a.rows_per_split;
    if (r_end > a.n) r_end = a.n;
    Softmax<VEC> sm;
    sm.init();
    if (r_begin < r_end)
        stream_rows<T, D, CH, false, true, NoHook, false>(Kb, Vb, a.row_bytes, sg, r_begin, r_end, 0, 1, q, a.qscale, sm, nullptr, a.vis_start, a.far_last);
    merge_groups<VEC, LPR, true>(sm);
    if (a.splits == 1) {
        const float inv_l = sm.l > 0.f ? 1.0f / sm.l : 0.f;
        if (lane < LPR) {
            float o[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) o[e] = sm.acc[e] * inv_l;
            *reinterpret_cast<uint4 *>(a.out + qoff) = Elem<T>::pack(o);
        }
        if (lane == 0 && a.far) {
            a.far[(size_t)unit * a.mass_stride] = sm.far * inv_l;
            a.tot[(size_t)unit * a.mass_stride] = sm.tot * inv_l;
        }
    } else {
        float *w = a.ws + (size_t)item * (4 + D);
        if (lane == 0) { w[0] = sm.m; w[1] = sm.l; w[2] = sm.far; w[3] = sm.tot; }
        if (lane < LPR) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) w[4 + sub * VEC + e] = sm.acc[e];
        }
    }
}

// merge the split partials of one unit: one thread per output element
template <typename T, int D>
__global__ __launch_bounds__(D) void dense_merge_kernel(DenseArgs a) {
    const int unit = blockIdx.x;
    const int e = threadIdx.x;
    const float *w = a.ws + (size_t)unit * a.splits * (4 + D);
    float m = NEG_BIG;
    for (int s = 0; s < a.splits; ++s) m = fmaxf(m, w[(size_t)s * (4 + D)]);
    float l = 0.f, far = 0.f, tot = 0.f, acc = 0.f;
    for (int s = 0; s < a.splits; ++s) {
        const float *ws = w + (size_t)s * (4 + D);
        const float f = fast_exp2(ws[0] - m);
        l += ws[1] * f; far += ws[2] * f; tot += ws[3] * f;
        acc += ws[4 + e] * f;
    }
    const float inv_l = l > 0.f ? 1.0f / l : 0.f;
    const float o = acc * inv_l;
    if (sizeof(T) == 4) reinterpret_cast<float *>(a.out)[(size_t)unit * D + e] = o;
    else reinterpret_cast<uint16_t *>(a.out)[(size_t)unit * D + e] = (uint16_t)f32_to_bf16_bits(o);
    if (e == 0 && a.far) {
        a.far[(size_t)unit * a.mass_stride] = far * inv_l;
        a.tot[(size_t)unit * a.mass_stride] = tot * inv_l;
    }
}

static int pick_splits(int units, int n) {
    // aim for >= 8192 waves (8 per SIMD on 256 CUs) but keep at least 128 rows per wave
    int s = (8192 + units - 1) / units;
    const int max_s = n / 128 > 1 ? n / 128 : 1;
    if (s > max_s) s = max_s;
    if (s > 64) s = 64;
    return s < 1 ? 1 : s;
}

template <typename T, int D>
static hipError_t launch_dense(const DenseArgs &a, hipStream_t s) {
    constexpr int WPB = 4;
    const long long items = (long long)a.n_units * a.splits;
    const unsigned blocks = (unsigned)((items + WPB - 1) / WPB);
    hipLaunchKernelGGL((dense_kernel<T, D, 4, WPB>), dim3(blocks), dim3(WPB * 64), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.splits > 1) {
        hipLaunchKernelGGL((dense_merge_kernel<T, D>), dim3((unsigned)a.n_units), dim3(D), 0, s, a);
        e = hipGetLastError();
    }
    return e;
}

// ---- scratch of ssd_dense_decode_attn_static ---------------------------------------------------------------
//
// The partial results of the row splits, for callers that may not allocate: a fixed array in the code object
// instead of a caller's workspace.  Every GPU the library runs on holds its own copy until the process ends.
// The array's name is a host-side stand-in and never goes to a kernel: the device address is looked up once per
// device and kept.
static constexpr size_t SCRATCH_BYTES = SSD_DENSE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

static constexpr int MAX_DEVICES = 64;
static void *g_scratch_ptr[MAX_DEVICES];     // device address of `scratch` on device i, 0 until first used there
static std::mutex g_scratch_mutex;

// Address of the current device's copy of `scratch`.
static int scratch_address(void **out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
    if (dev < 0 || dev >= MAX_DEVICES) return fail(SSD_ERR_INVALID_ARG, "device index %d outside 0..%d", dev, MAX_DEVICES - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e, "hipGetSymbolAddress of the static scratch");
        if (!ptr) return fail(SSD_ERR_HIP, "hipGetSymbolAddress returned no address for the static scratch");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SSD_OK;
}

}  // namespace ssd

using namespace ssd;

// splits == 0: chosen from the shape.  static_scratch: the partials go to this device's fixed scratch array
// instead of `workspace`.
static int dense_run(const void *q, const void *K, const void *V, void *out, int B, int H, int d, int dtype, int n_cap, int n,
                     float softmax_scale, float *far, float *tot, int mass_stride, int vis_start, int w, int splits,
                     void *workspace, size_t workspace_bytes, void *stream, bool static_scratch = false) {
    clear_error();
    if (!q || !K || !V || !out) return fail(SSD_ERR_INVALID_ARG, "q, K, V or out is NULL");
    if (!aligned(q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(out, 16)) return fail(SSD_ERR_INVALID_ARG, "q, K, V, out must be 16-byte aligned");
    if (B < 1 || H < 1 || (long long)B * H > 0x3fffffffLL) return fail(SSD_ERR_INVALID_ARG, "bad B or H");
    if (d != 64 && d != 128) return fail(SSD_ERR_INVALID_ARG, "head_dim=%d, supported: 64, 128", d);
    if (dtype != SSD_F32 && dtype != SSD_BF16) return fail(SSD_ERR_INVALID_ARG, "bad dtype");
    if (n < 1 || n > n_cap) return fail(SSD_ERR_INVALID_ARG, "n=%d must be in 1..n_cap=%d", n, n_cap);
    if ((far == nullptr) != (tot == nullptr)) return fail(SSD_ERR_INVALID_ARG, "far and tot must both be given or both be NULL");
    if (far && (mass_stride < 1 || vis_start < 0 || w < 0)) return fail(SSD_ERR_INVALID_ARG, "bad mass_stride, vis_start or w");
    if (!(softmax_scale >= 0.f)) return fail(SSD_ERR_INVALID_ARG, "softmax_scale must be >= 0");
    if (splits < 0 || splits > 64) return fail(SSD_ERR_INVALID_ARG, "splits=%d outside 0..64", splits);
    DenseArgs a;
    a.q = static_cast<const char *>(q);
    a.K = static_cast<const char *>(K);
    a.V = static_cast<const char *>(V);
    a.out = static_cast<char *>(out);
    a.far = far;
    a.tot = tot;
    a.n_units = B * H;
    a.n_cap = n_cap;
    a.n = n;
    a.row_bytes = d * (dtype == SSD_F32 ? 4 : 2);
    a.splits = splits > 0 ? splits : pick_splits(a.n_units, n);
    a.rows_per_split = (n + a.splits - 1) / a.splits;
    a.mass_stride = mass_stride;
    a.vis_start = far ? vis_start : 0;
    a.far_last = n - 1 - w;
    a.qscale = (softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)d)) * LOG2E;
    a.ws = static_cast<float *>(workspace);
    if (a.splits > 1) {
        const size_t need = (size_t)a.n_units * a.splits * (4 + d) * sizeof(float);
        if (static_scratch) {
            if (need > SCRATCH_BYTES)
                return fail(SSD_ERR_INVALID_ARG, "%d units in %d row splits need %zu bytes of partial results, the static scratch holds %zu: "
                            "use ssd_dense_decode_attn with a workspace", a.n_units, a.splits, need, SCRATCH_BYTES);
            void *ptr = nullptr;
            const int rc = scratch_address(&ptr);
            if (rc != SSD_OK) return rc;
            a.ws = static_cast<float *>(ptr);
        } else if (!workspace || workspace_bytes < need || !aligned(workspace, 256)) {
            return fail(SSD_ERR_INVALID_ARG, "workspace of %zu bytes (256-byte aligned) needed, got %zu", need, workspace_bytes);
        }
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    if (dtype == SSD_BF16) e = d == 128 ? launch_dense<bf16_t, 128>(a, s) : launch_dense<bf16_t, 64>(a, s);
    else e = d == 128 ? launch_dense<float, 128>(a, s) : launch_dense<float, 64>(a, s);
    if (e != hipSuccess) return hip_fail(e, "dense attention launch");
    return SSD_OK;
}

extern "C" size_t ssd_dense_workspace_bytes(int B, int H, int d, int n) {
    if (B < 1 || H < 1 || d < 1 || n < 1) return 0;
    // room for the largest split count the library ever picks
    return (size_t)B * H * 64 * (size_t)(4 + d) * sizeof(float);
}

extern "C" int ssd_dense_decode_attn(const void *q, const void *K, const void *V, void *out, int B, int H, int d, int dtype,
                                     int n_cap, int n, float softmax_scale, float *far, float *tot, int mass_stride,
                                     int vis_start, int w, void *workspace, size_t workspace_bytes, void *stream) {
    return dense_run(q, K, V, out, B, H, d, dtype, n_cap, n, softmax_scale, far, tot, mass_stride, vis_start, w, 0,
                     workspace, workspace_bytes, stream);
}

extern "C" int ssd_dense_decode_attn_splits(const void *q, const void *K, const void *V, void *out, int B, int H, int d, int dtype,
                                            int n_cap, int n, float softmax_scale, float *far, float *tot, int mass_stride,
                                            int vis_start, int w, int splits, void *workspace, size_t workspace_bytes,
                                            void *stream) {
    return dense_run(q, K, V, out, B, H, d, dtype, n_cap, n, softmax_scale, far, tot, mass_stride, vis_start, w, splits,
                     workspace, workspace_bytes, stream);
}

extern "C" int ssd_dense_decode_attn_static(const void *q, const void *K, const void *V, void *out, int B, int H, int d, int dtype,
                                            int n_cap, int n, float softmax_scale, float *far, float *tot, int mass_stride,
                                            int vis_start, int w, void *stream) {
    return dense_run(q, K, V, out, B, H, d, dtype, n_cap, n, softmax_scale, far, tot, mass_stride, vis_start, w, 0,
                     nullptr, 0, stream, true);
}
