// ssd_prefill_scores: accumulated attention scores of a prompt that is processed at once
// (Algorithm 2: the scores of semantic heads are accumulated whenever attention weights exist, and a
// prefill is followed by a compression at once).  For every (layer, sequence, head) unit
//     a_i      = softmax over keys 0..i of scale * q_i . k_j        (causal)
//     score[j] = sum_{i >= j} a_i(j)
// which is what ssd_compress_kv's dense-source mode takes as score_src.
//
// This is the one step of the path that is a dense contraction (an n x n x d product per unit), so
// it runs on the matrix cores: 32 x 32 output tiles of Q K^T with v_mfma_f32_32x32x16_bf16 (bf16
// inputs, 8 k-values per lane and step) or v_mfma_f32_32x32x2_f32 (fp32 inputs).  Both operands
// are read straight from their row-major [n, d] layout: lane l supplies row (l mod 32) and the
// k-slice selected by (l div 32), the same slice for Q and K, so no transpose or LDS staging is
// needed.  A tile's 32 x 32 results sit 16 per lane: column = l mod 32, row = 8*(v/4) + 4*(l/32) + v%4.
//
// One workgroup per unit, of as many waves as the prompt has blocks of 32 queries (at most four); wave
// w owns query blocks w, w + waves, ...  Prompts of up to 128 tokens (one block per wave) hold their
// key fragments and logits in registers and touch memory once; longer ones make, per query block, two
// sweeps over the key blocks up to the diagonal: the first keeps a running max and sum per lane and
// result register and merges them over the 32 lanes of a row once at its end, the second recomputes
// the tile, normalises and adds the tile's column sums into a wave-private LDS array; the waves'
// arrays are added in a fixed order at the end (bit-reproducible, no atomics).
// Bound: HBM for the short prompts this is meant for (Q and K of a unit are read once from HBM,
// re-reads of K tiles hit in L2); at n = 64, d = 128 a unit does 1 MFLOP on 32 KB.
#include <cmath>

#include "ssd_device.h"

namespace ssd {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

template <typename T> struct Mma;

template <> struct Mma<bf16_t> {
    static constexpr int KSTEP = 16;                 // k-values one MFMA consumes
    typedef uint4 Frag;                              // 8 bf16 per lane
    static __device__ __forceinline__ Frag load(const char *row, int ks, int half) {
        return *reinterpret_cast<const uint4 *>(row + (size_t)(ks * KSTEP + 8 * half) * 2);
    }
    static __device__ __forceinline__ f32x16_t mma(const Frag &a, const Frag &b, const f32x16_t &c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};

template <> struct Mma<float> {
    static constexpr int KSTEP = 2;
    typedef float Frag;                              // 1 float per lane
    static __device__ __forceinline__ Frag load(const char *row, int ks, int half) {
        return *reinterpret_cast<const float *>(row + (size_t)(ks * KSTEP + half) * 4);
    }
    static __device__ __forceinline__ f32x16_t mma(const Frag &a, const Frag &b, const f32x16_t &c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
};

// max / sum over the 32 lanes that share (lane div 32): DPP inside a 16-lane row, one swap across rows
static __device__ __forceinline__ float half_max(float v) {
    v = fmaxf(v, dpp_f<0xB1>(v));
    v = fmaxf(v, dpp_f<0x4E>(v));
    v = fmaxf(v, dpp_f<0x141>(v));
    v = fmaxf(v, dpp_f<0x140>(v));
    float a, b;
    rows_pair(v, a, b);
    return fmaxf(a, b);
}
static __device__ __forceinline__ float half_sum(float v) {
    v += dpp_f<0xB1>(v);
    v += dpp_f<0x4E>(v);
    v += dpp_f<0x141>(v);
    v += dpp_f<0x140>(v);
    float a, b;
    rows_pair(v, a, b);
    return a + b;
}

struct PrefillArgs {
    const char *Q;
    const char *K;
    float *score_out;
    int n;
    int row_bytes;
    float qscale;        // softmax scale * log2(e)
};

// Fragments of one block of 32 rows (queries or keys): row = first + (lane mod 32), clamped to the last row.
template <typename T, int D>
static __device__ __forceinline__ void load_block(const char *base, int first, int n, int row_bytes, int l32, int half,
                                                  typename Mma<T>::Frag (&f)[D / Mma<T>::KSTEP]) {
    int row = first + l32;
    if (row > n - 1) row = n - 1;                          // rows past the end repeat the last one; masked later
#pragma unroll
    for (int ks = 0; ks < D / Mma<T>::KSTEP; ++ks) f[ks] = Mma<T>::load(base + (size_t)row * row_bytes, ks, half);
}

// One 32 x 32 tile of scaled logits, masked where key > query (causal) or either lies beyond n.
template <typename T, int D>
static __device__ __forceinline__ void logits_tile(const typename Mma<T>::Frag (&qa)[D / Mma<T>::KSTEP],
                                                   const typename Mma<T>::Frag (&kf)[D / Mma<T>::KSTEP], int qb, int kb, int n,
                                                   int l32, int half, float qscale, float (&z)[16]) {
    f32x16_t c = {0.f};
#pragma unroll
    for (int ks = 0; ks < D / Mma<T>::KSTEP; ++ks) c = Mma<T>::mma(qa[ks], kf[ks], c);
    const int key = kb * 32 + l32;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int row = qb * 32 + (v >> 2) * 8 + half * 4 + (v & 3);
        z[v] = (key < n && key <= row && row < n) ? c[v] * qscale : NEG_BIG;
    }
}

// Row maxima and sums held per lane -> per query row (over the 32 lanes that share it); l becomes 1 / sum.
static __device__ __forceinline__ void merge_rows(float (&m)[16], float (&l)[16]) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const float m_row = half_max(m[v]);
        const float l_row = half_sum(l[v] * fast_exp2(m[v] - m_row));
        m[v] = m_row;
        l[v] = l_row > 0.f ? 1.0f / l_row : 0.f;
    }
}

// Sum over the tile's 32 queries of the normalised probabilities of key (lane mod 32); valid in lanes 0..31.
static __device__ __forceinline__ float column_sum(const float (&z)[16], const float (&m)[16], const float (&inv_l)[16]) {
    float cs = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) cs += z[v] > NEG_BIG * 0.5f ? fast_exp2(z[v] - m[v]) * inv_l[v] : 0.f;
    float lo, hi;
    halves_pair(cs, lo, hi);                               // the other 16 rows of the tile live in the other half
    return lo + hi;
}

static __device__ __forceinline__ void write_scores(const PrefillArgs &a, const float *colsum, int waves) {
    __syncthreads();
    float *out = a.score_out + (size_t)blockIdx.x * (size_t)a.n;
    for (int j = threadIdx.x; j < a.n; j += blockDim.x) {
        float t = colsum[j];
        for (int x = 1; x < waves; ++x) t += colsum[x * a.n + j];
        out[j] = t;
    }
}

// Any prompt length: wave w owns query blocks w, w + waves, ...; key tiles are fetched in both sweeps.
template <typename T, int D>
__global__ __launch_bounds__(256) void prefill_scores_kernel(PrefillArgs a) {
    typedef typename Mma<T>::Frag Frag;
    constexpr int NK = D / Mma<T>::KSTEP;
    extern __shared__ float colsum[];                      // [waves][n]
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int waves = blockDim.x >> 6;
    const int lane = threadIdx.x & 63;
    const int half = lane >> 5;
    const int l32 = lane & 31;
    const int n = a.n;
    const size_t unit_off = (size_t)blockIdx.x * (size_t)n * (size_t)a.row_bytes;
    const char *Qu = a.Q + unit_off;
    const char *Ku = a.K + unit_off;
    float *mine = colsum + (size_t)w * n;
    for (int j = lane; j < n; j += 64) mine[j] = 0.f;      // only this wave touches `mine` until the final sum

    const int n_blocks = (n + 31) / 32;
    for (int qb = w; qb < n_blocks; qb += waves) {
        Frag qa[NK], kf[NK];
        load_block<T, D>(Qu, qb * 32, n, a.row_bytes, l32, half, qa);
        float m[16], l[16], z[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) { m[v] = NEG_BIG; l[v] = 0.f; }
        for (int kb = 0; kb <= qb; ++kb) {                 // sweep 1: per-lane running max and sum
            load_block<T, D>(Ku, kb * 32, n, a.row_bytes, l32, half, kf);
            logits_tile<T, D>(qa, kf, qb, kb, n, l32, half, a.qscale, z);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float m_new = fmaxf(m[v], z[v]);
                const float p = z[v] > NEG_BIG * 0.5f ? fast_exp2(z[v] - m_new) : 0.f;
                l[v] = l[v] * fast_exp2(m[v] - m_new) + p;
                m[v] = m_new;
            }
        }
        merge_rows(m, l);
        for (int kb = 0; kb <= qb; ++kb) {                 // sweep 2: normalised column sums
            load_block<T, D>(Ku, kb * 32, n, a.row_bytes, l32, half, kf);
            logits_tile<T, D>(qa, kf, qb, kb, n, l32, half, a.qscale, z);
            const float cs = column_sum(z, m, l);
            const int key = kb * 32 + l32;
            if (half == 0 && key < n) mine[key] += cs;
        }
    }
    write_scores(a, colsum, waves);
}

// Prompts of at most KT blocks of 32 tokens: one wave per query block, launched with exactly that many
// waves.  Wave w needs key tiles 0..w; all their fragments are requested before the first product, and
// the logits stay in registers between the two sweeps, so a wave waits for memory once.
template <typename T, int D, int KT>
__global__ __launch_bounds__(64 * KT) void prefill_scores_short_kernel(PrefillArgs a) {
    typedef typename Mma<T>::Frag Frag;
    constexpr int NK = D / Mma<T>::KSTEP;
    extern __shared__ float colsum[];                      // [waves][n]
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // = this wave's query block
    const int waves = blockDim.x >> 6;
    const int lane = threadIdx.x & 63;
    const int half = lane >> 5;
    const int l32 = lane & 31;
    const int n = a.n;
    const size_t unit_off = (size_t)blockIdx.x * (size_t)n * (size_t)a.row_bytes;
    const char *Qu = a.Q + unit_off;
    const char *Ku = a.K + unit_off;
    float *mine = colsum + (size_t)w * n;

    Frag qa[NK], kf[KT][NK];
    load_block<T, D>(Qu, w * 32, n, a.row_bytes, l32, half, qa);
#pragma unroll
    for (int kb = 0; kb < KT; ++kb)
        if (kb <= w) load_block<T, D>(Ku, kb * 32, n, a.row_bytes, l32, half, kf[kb]);
    for (int j = lane; j < n; j += 64) mine[j] = 0.f;

    float z[KT][16], m[16], l[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) { m[v] = NEG_BIG; l[v] = 0.f; }
#pragma unroll
    for (int kb = 0; kb < KT; ++kb) {
        if (kb <= w) {
            logits_tile<T, D>(qa, kf[kb], w, kb, n, l32, half, a.qscale, z[kb]);
#pragma unroll
            for (int v = 0; v < 16; ++v) m[v] = fmaxf(m[v], z[kb][v]);
        }
    }
#pragma unroll
    for (int kb = 0; kb < KT; ++kb) {
        if (kb <= w) {
#pragma unroll
            for (int v = 0; v < 16; ++v) l[v] += z[kb][v] > NEG_BIG * 0.5f ? fast_exp2(z[kb][v] - m[v]) : 0.f;
        }
    }
    merge_rows(m, l);
#pragma unroll
    for (int kb = 0; kb < KT; ++kb) {
        if (kb <= w) {
            const float cs = column_sum(z[kb], m, l);
            const int key = kb * 32 + l32;
            if (half == 0 && key < n) mine[key] = cs;
        }
    }
    write_scores(a, colsum, waves);
}

}  // namespace ssd

using namespace ssd;

extern "C" int ssd_prefill_scores(const void *Q, const void *K, int n_units, int n_src, int d, int dtype, float softmax_scale,
                                  float *score_out, void *stream) {
    clear_error();
    if (!Q || !K || !score_out) return fail(SSD_ERR_INVALID_ARG, "Q, K or score_out is NULL");
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(score_out, 4)) return fail(SSD_ERR_INVALID_ARG, "Q / K must be 16-byte aligned");
    if (n_units < 1) return fail(SSD_ERR_INVALID_ARG, "n_units=%d must be >= 1", n_units);
    if (n_src < 1 || n_src > 4096) return fail(SSD_ERR_INVALID_ARG, "n_src=%d outside 1..4096", n_src);
    if (d != 64 && d != 128) return fail(SSD_ERR_INVALID_ARG, "head_dim=%d, supported: 64, 128", d);
    if (dtype != SSD_F32 && dtype != SSD_BF16) return fail(SSD_ERR_INVALID_ARG, "bad dtype");
    if (!(softmax_scale >= 0.f) || !std::isfinite(softmax_scale)) return fail(SSD_ERR_INVALID_ARG, "softmax_scale must be finite and >= 0");
    PrefillArgs a;
    a.Q = static_cast<const char *>(Q);
    a.K = static_cast<const char *>(K);
    a.score_out = score_out;
    a.n = n_src;
    a.row_bytes = d * (dtype == SSD_F32 ? 4 : 2);
    a.qscale = (softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)d)) * LOG2E;
    const int n_blocks = (n_src + 31) / 32;
    const int waves = n_blocks < 4 ? n_blocks : 4;
    const size_t lds = (size_t)waves * (size_t)n_src * sizeof(float);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)n_units), block(64u * waves);
#define SSD_PREFILL(T_, D_)                                                                                          \
    do {                                                                                                             \
        if (n_blocks <= 2) hipLaunchKernelGGL((prefill_scores_short_kernel<T_, D_, 2>), grid, block, lds, s, a);     \
        else if (n_blocks <= 4) hipLaunchKernelGGL((prefill_scores_short_kernel<T_, D_, 4>), grid, block, lds, s, a); \
        else hipLaunchKernelGGL((prefill_scores_kernel<T_, D_>), grid, block, lds, s, a);                            \
    } while (0)
    if (dtype == SSD_BF16) {
        if (d == 128) SSD_PREFILL(bf16_t, 128); else SSD_PREFILL(bf16_t, 64);
    } else {
        if (d == 128) SSD_PREFILL(float, 128); else SSD_PREFILL(float, 64);
    }
#undef SSD_PREFILL
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "prefill score launch");
    return SSD_OK;
}
