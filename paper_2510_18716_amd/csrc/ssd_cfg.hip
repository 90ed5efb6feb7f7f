// ssd_cfg_mix: classifier-free guidance of the two next-token distributions of each prompt (Sec. 3.1,
// Eq. 1):  out[i, v] = p[2i, v] + gamma * (p[2i, v] - p[2i+1, v]),  sequence 2i being the pass conditioned
// on the prompt and 2i+1 the unconditional one.  It is what follows the decode attention of the last layer
// on the way to the next token: after it, one token is sampled per prompt and fed to both sequences.
//
// Elementwise and read-once, so the bound is HBM: 2 * V * e bytes in and 4 * V bytes out per prompt.  Each
// lane takes 16-byte fragments of the two rows (coalesced) and writes fp32; rows whose length is not a
// multiple of the fragment go through the scalar tail loop.
#include <cmath>

#include "ssd_device.h"

namespace ssd {

struct CfgArgs {
    const char *p;
    float *out;
    long long frags_per_row;   // whole 16-byte fragments per row
    int V;
    int n_prompts;
    float gamma;
};

static __device__ __forceinline__ float widen(float x) { return x; }
static __device__ __forceinline__ float widen(bf16_t x) { return __uint_as_float((uint32_t)x.bits << 16); }

template <typename T>
__global__ __launch_bounds__(256) void cfg_mix_kernel(CfgArgs a) {
    constexpr int VEC = Elem<T>::VEC;
    const long long n_frag = a.frags_per_row * a.n_prompts;
    const size_t row_bytes = (size_t)a.V * sizeof(T);
    const bool vec_ok = row_bytes % 16 == 0;                  // otherwise odd rows are not 16-byte aligned
    const long long stride = (long long)gridDim.x * blockDim.x;
    const long long tid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (vec_ok) {
        for (long long f = tid; f < n_frag; f += stride) {
            const long long i = f / a.frags_per_row, j = f % a.frags_per_row;
            const char *c = a.p + (size_t)(2 * i) * row_bytes + (size_t)j * 16u;
            float cf[VEC], uf[VEC];
            Elem<T>::unpack(*reinterpret_cast<const uint4 *>(c), cf);
            Elem<T>::unpack(*reinterpret_cast<const uint4 *>(c + row_bytes), uf);
            float *o = a.out + (size_t)i * a.V + (size_t)j * VEC;
#pragma unroll
            for (int e = 0; e < VEC; e += 4) {
                float4 r;
                r.x = fmaf(a.gamma, cf[e] - uf[e], cf[e]);
                r.y = fmaf(a.gamma, cf[e + 1] - uf[e + 1], cf[e + 1]);
                r.z = fmaf(a.gamma, cf[e + 2] - uf[e + 2], cf[e + 2]);
                r.w = fmaf(a.gamma, cf[e + 3] - uf[e + 3], cf[e + 3]);
                *reinterpret_cast<float4 *>(o + e) = r;
            }
        }
        return;
    }
    // rows of a length that breaks the alignment: one element per lane
    const long long n_el = (long long)a.V * a.n_prompts;
    const T *p = reinterpret_cast<const T *>(a.p);
    for (long long x = tid; x < n_el; x += stride) {
        const long long i = x / a.V, v = x % a.V;
        const float c = widen(p[(size_t)(2 * i) * a.V + v]);
        const float u = widen(p[(size_t)(2 * i + 1) * a.V + v]);
        a.out[x] = fmaf(a.gamma, c - u, c);
    }
}

}  // namespace ssd

using namespace ssd;

extern "C" int ssd_cfg_mix(const void *p, int n_seqs, int V, int dtype, float gamma, float *out, void *stream) {
    clear_error();
    if (!p || !out) return fail(SSD_ERR_INVALID_ARG, "p or out is NULL");
    if (!aligned(p, 16) || !aligned(out, 16)) return fail(SSD_ERR_INVALID_ARG, "p and out must be 16-byte aligned");
    if (n_seqs < 2 || n_seqs % 2 != 0) return fail(SSD_ERR_INVALID_ARG, "n_seqs=%d must be even and >= 2 (conditional / unconditional pairs)", n_seqs);
    if (V < 1) return fail(SSD_ERR_INVALID_ARG, "V=%d must be >= 1", V);
    if (dtype != SSD_F32 && dtype != SSD_BF16) return fail(SSD_ERR_INVALID_ARG, "bad dtype");
    if (!std::isfinite(gamma)) return fail(SSD_ERR_INVALID_ARG, "gamma must be finite");
    CfgArgs a;
    a.p = static_cast<const char *>(p);
    a.out = out;
    a.V = V;
    a.n_prompts = n_seqs / 2;
    a.gamma = gamma;
    const int esize = dtype == SSD_F32 ? 4 : 2;
    a.frags_per_row = ((long long)V * esize) / 16;
    const bool vec_ok = ((long long)V * esize) % 16 == 0;
    const long long work = vec_ok ? a.frags_per_row * a.n_prompts : (long long)V * a.n_prompts;
    long long blocks = (work + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;                  // grid-stride beyond 32 workgroups per CU
    if (blocks < 1) blocks = 1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == SSD_BF16) hipLaunchKernelGGL((cfg_mix_kernel<bf16_t>), dim3((unsigned)blocks), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((cfg_mix_kernel<float>), dim3((unsigned)blocks), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "guidance mix launch");
    return SSD_OK;
}
