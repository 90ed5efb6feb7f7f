// ssd_classify_heads: the sparsity metric s_{l,h} of Sec. 3.3 ("Spatial Sparsity Analysis") and
// the threshold rule of Eq. (3).
//
// One workgroup per (layer, head).  Each thread sums the ratios far/tot of a fixed, strided subset
// of the P*T terms; the 256 partial sums are then added by a fixed binary tree in LDS, so the
// result does not depend on scheduling and is bit-reproducible.  Input is read once, coalesced
// along t.  Small (2 x 35 MB at the 7B shape) and offline: not on the per-token path.
#include "ssd_device.h"

namespace ssd {

__global__ __launch_bounds__(256) void classify_kernel(const float *__restrict__ far, const float *__restrict__ tot,
                                                       int P, int H, int T, float tau, float *s_out, uint8_t *type_out) {
    __shared__ float part[256];
    const int l = blockIdx.x / H, h = blockIdx.x % H;
    const int tid = threadIdx.x;
    float acc = 0.f;
    for (int p = 0; p < P; ++p) {
        const size_t base = (((size_t)l * P + p) * H + h) * (size_t)T;
        for (int t = tid; t < T; t += 256) {
            const float den = tot[base + t];
            const float num = far[base + t];
            acc += den > 0.f ? num / den : 0.f;
        }
    }
    part[tid] = acc;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if (tid < w) part[tid] += part[tid + w];
        __syncthreads();
    }
    if (tid == 0) {
        const float s = part[0] / ((float)P * (float)T);
        if (s_out) s_out[blockIdx.x] = s;
        if (type_out) type_out[blockIdx.x] = s > tau ? SSD_SEMANTIC : SSD_SPATIAL;
    }
}

}  // namespace ssd

using namespace ssd;

extern "C" int ssd_classify_heads(const float *far, const float *tot, int L, int P, int H, int T, float tau,
                                  float *s_out, uint8_t *type_out, void *stream) {
    clear_error();
    if (!far || !tot) return fail(SSD_ERR_INVALID_ARG, "far or tot is NULL");
    if (!s_out && !type_out) return fail(SSD_ERR_INVALID_ARG, "s_out and type_out are both NULL");
    if (L < 1 || P < 1 || H < 1 || T < 1) return fail(SSD_ERR_INVALID_ARG, "L, P, H, T must be >= 1");
    if ((long long)L * H > 0x7fffffffLL) return fail(SSD_ERR_INVALID_ARG, "L*H too large");
    if (!aligned(far, 4) || !aligned(tot, 4) || !aligned(s_out, 4)) return fail(SSD_ERR_INVALID_ARG, "misaligned pointer");
    if (!(tau == tau)) return fail(SSD_ERR_INVALID_ARG, "tau is NaN");
    hipLaunchKernelGGL(classify_kernel, dim3((unsigned)(L * H)), dim3(256), 0, static_cast<hipStream_t>(stream), far, tot, P,
                       H, T, tau, s_out, type_out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "classification launch");
    return SSD_OK;
}
