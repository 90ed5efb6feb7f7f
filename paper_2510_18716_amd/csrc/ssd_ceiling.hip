// ssd_bench_stream: a measurement aid, not part of the method.  It moves what a launch of the decode path moves,
// with none of its arithmetic: n_units independent units of unit_bytes each (a K plane and a V plane), one
// wavefront per unit, four units per workgroup, every byte read once with the same 16-byte fragments -- and,
// optionally, a few 256-byte rows stored per unit, which is the least a decode step must write (the new token's
// K and V rows).  Timing it at a launch shape gives the level the memory system allows a kernel of that shape,
// with and without the writes.
#include "ssd_device.h"

namespace ssd {

template <int ROWS_OUT>
__global__ __launch_bounds__(256) void bench_stream_kernel(uint4 *__restrict__ p, int unit_u4, long long n_units,
                                                          uint4 *__restrict__ sink, int slot) {
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long long unit = (long long)blockIdx.x * 4 + w;
    if (unit >= n_units) return;
    const int lane = threadIdx.x & 63;
    uint4 *b = p + (size_t)unit * unit_u4;
    const int half = unit_u4 / 2;
    uint32_t acc = 0;
    for (int i = lane; i < half; i += 256) {            // four wave-wide loads of each plane in flight
        uint4 a[4], c[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            int j = i + k * 64;
            j = j < half ? j : half - 1;
            a[k] = load_once(reinterpret_cast<const char *>(b + j));              // the load the decode kernels stream with
            c[k] = load_once(reinterpret_cast<const char *>(b + half + j));
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) acc += a[k].x ^ c[k].y ^ a[k].z ^ c[k].w;
    }
    const uint4 row = make_uint4(acc, acc, acc, acc);
    if (ROWS_OUT >= 2 && lane < 16) {                   // one 256-byte row into each plane of the unit
        b[slot * 16 + lane] = row;
        b[half + slot * 16 + lane] = row;
    }
    if (ROWS_OUT == 0 && acc == 0x12345678u && lane == 0) sink[0] = row;   // keeps the loads alive
}

// Plain copy, 16 bytes per lane, grid-stride: a kernel whose HBM reads and writes are known exactly, against
// which the profiler's byte counters are scaled.
__global__ __launch_bounds__(256) void bench_copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, long long n_u4) {
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n_u4; i += (long long)gridDim.x * 256) dst[i] = src[i];
}

}  // namespace ssd

using namespace ssd;

extern "C" int ssd_bench_copy(void *dst, const void *src, size_t bytes, void *stream) {
    clear_error();
    if (!dst || !src || !aligned(dst, 16) || !aligned(src, 16)) return fail(SSD_ERR_INVALID_ARG, "dst and src must be given, 16-byte aligned");
    if (bytes < 16 || bytes % 16 != 0) return fail(SSD_ERR_INVALID_ARG, "bytes must be a positive multiple of 16");
    const long long n_u4 = (long long)(bytes / 16);
    const long long want = (n_u4 + 255) / 256;
    const unsigned blocks = (unsigned)(want < 65536 ? want : 65536);
    hipLaunchKernelGGL(bench_copy_kernel, dim3(blocks), dim3(256), 0, static_cast<hipStream_t>(stream), static_cast<uint4 *>(dst),
                       static_cast<const uint4 *>(src), n_u4);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "copy benchmark launch");
    return SSD_OK;
}

extern "C" int ssd_bench_stream(void *buf, size_t unit_bytes, long long n_units, int rows_written, void *sink, void *stream) {
    clear_error();
    if (!buf || !sink || !aligned(buf, 16) || !aligned(sink, 16)) return fail(SSD_ERR_INVALID_ARG, "buf and sink must be given, 16-byte aligned");
    if (unit_bytes < 1024 || unit_bytes % 512 != 0 || unit_bytes > (1u << 30)) return fail(SSD_ERR_INVALID_ARG, "unit_bytes must be a multiple of 512, at least 1024");
    if (n_units < 1 || n_units > (1ll << 31)) return fail(SSD_ERR_INVALID_ARG, "bad n_units");
    if (rows_written != 0 && rows_written != 2) return fail(SSD_ERR_INVALID_ARG, "rows_written is 0 or 2");
    const unsigned blocks = (unsigned)((n_units + 3) / 4);
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint4 *p = static_cast<uint4 *>(buf);
    const int unit_u4 = (int)(unit_bytes / 16);
    if (rows_written == 2) hipLaunchKernelGGL((bench_stream_kernel<2>), dim3(blocks), dim3(256), 0, s, p, unit_u4, n_units, static_cast<uint4 *>(sink), 0);
    else hipLaunchKernelGGL((bench_stream_kernel<0>), dim3(blocks), dim3(256), 0, s, p, unit_u4, n_units, static_cast<uint4 *>(sink), 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "stream benchmark launch");
    return SSD_OK;
}
