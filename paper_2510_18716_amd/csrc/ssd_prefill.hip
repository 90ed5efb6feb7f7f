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
// One workgroup per unit at a time, of as many waves as the prompt has blocks of 32 queries (at most four);
// wave w owns query blocks w, w + waves, ...
// Prompts of up to 128 tokens (one block per wave; the case the decode path's prompts fall in): the workgroup
// fetches the unit's Q and K once, fully coalesced, and hands the matrix cores their fragments through LDS; the
// tiles are taken as K Q^T so that a query's softmax statistics stay inside a lane pair and only the column
// sums cross lanes; the logits stay in registers; workgroups are persistent and request the next unit's rows
// while working on the current one.  This form is bound by HBM: at n = 64, d = 128 a unit does 1 MFLOP on 32 KB,
// and what used to hold it back was the softmax bookkeeping on the vector ALUs (about 1100 instructions per
// wave with the queries along the registers, about 400 now), not the matrix cores or the memory.
// Longer prompts make, per query block, two sweeps over the key blocks up to the diagonal, operands read
// straight from memory in fragment layout: the first keeps a running max and sum per lane and result register
// and merges them over the 32 lanes of a row once at its end, the second recomputes the tile, normalises and
// adds the tile's column sums into a wave-private LDS array.  In both forms the waves' arrays are added in a
// fixed order at the end (bit-reproducible, no atomics).
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
    int n_units;
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
        l[v] = l_row > 0.f ? __builtin_amdgcn_rcpf(l_row) : 0.f;
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

static __device__ __forceinline__ void write_scores(const PrefillArgs &a, const float *colsum, int waves, int unit) {
    __syncthreads();
    float *out = a.score_out + (size_t)unit * (size_t)a.n;
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
    write_scores(a, colsum, waves, (int)blockIdx.x);
}

// Fragment of an operand block that was staged in LDS (rows of `stride` bytes): what Mma<T>::load takes from memory.
template <typename T> static __device__ __forceinline__ typename Mma<T>::Frag lds_frag(const unsigned char *row, int ks, int half);
template <> __device__ __forceinline__ uint4 lds_frag<bf16_t>(const unsigned char *row, int ks, int half) {
    return *reinterpret_cast<const uint4 *>(row + (ks * Mma<bf16_t>::KSTEP + 8 * half) * 2);
}
template <> __device__ __forceinline__ float lds_frag<float>(const unsigned char *row, int ks, int half) {
    return *reinterpret_cast<const float *>(row + (ks * Mma<float>::KSTEP + half) * 4);
}

// ---- tiles with the keys along the registers (short prompts) --------------------------------------------------
//
// The product is taken as K Q^T: a tile's 32 x 32 results then sit with the query along the lanes (column =
// lane mod 32) and the key along the registers (row = 8*(v/4) + 4*(lane/32) + v%4).  Every lane pair (l, l + 32)
// owns one query, so the softmax statistics of a row are sums and maxima over a lane's own registers plus one
// exchange between the halves -- no reduction over lanes -- and what is left to add up over lanes is the column
// sums, which only one lane per key has to end up with.

// One tile of scaled logits, masked where key > query (causal) or either lies beyond n.  `plain`: the tile lies
// below the diagonal and inside the prompt, nothing to mask.
template <typename T, int D>
static __device__ __forceinline__ void logits_tile_keys_in_regs(const typename Mma<T>::Frag (&kf)[D / Mma<T>::KSTEP],
                                                                const typename Mma<T>::Frag (&qa)[D / Mma<T>::KSTEP], int qb, int kb,
                                                                int n, int l32, int half, float qscale, bool plain, float (&z)[16]) {
    f32x16_t c = {0.f};
#pragma unroll
    for (int ks = 0; ks < D / Mma<T>::KSTEP; ++ks) c = Mma<T>::mma(kf[ks], qa[ks], c);
    if (plain) {                                           // wave-uniform
#pragma unroll
        for (int v = 0; v < 16; ++v) z[v] = c[v] * qscale;
        return;
    }
    const int query = qb * 32 + l32;
    const int key0 = kb * 32 + half * 4;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int key = key0 + (v >> 2) * 8 + (v & 3);
        z[v] = (key <= query && query < n) ? c[v] * qscale : NEG_BIG;      // key <= query < n implies key < n
    }
}

// Column sums of one tile: x[v] of lane l is the probability of key (v, l / 32) for query l mod 32; the sum over
// the 32 queries ends up in the 16 lanes of each half that have bit 1 of the lane index clear, lane l holding
// key row  8*(u/4) + 4*(l/32) + u%4  with  u = 8*bit4(l) + 4*bit3(l) + 2*bit2(l) + bit0(l).
// Five exchange steps (the two 16-lane rows of a half, then lanes 8 apart, mirrored within 8, neighbours,
// lanes 2 apart), each of the first four halving the values a lane still carries: 38 operations for the 512 sums.
static __device__ __forceinline__ float column_sums_over_lanes(const float (&x)[16], int lane) {
    float y[8], wv[4], r[2];
#pragma unroll
    for (int v = 0; v < 8; ++v) {                          // row 0 of the half keeps keys 0..7, row 1 keys 8..15
        const uint2v_t sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(x[v]), __float_as_uint(x[v + 8]), false, false);
        y[v] = __uint_as_float(sw.x) + __uint_as_float(sw.y);
    }
    const bool b3 = (lane & 8) != 0, b2 = (lane & 4) != 0, b0 = (lane & 1) != 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) wv[u] = (b3 ? y[u + 4] : y[u]) + dpp_f<0x128>(b3 ? y[u] : y[u + 4]);        // row_ror:8
#pragma unroll
    for (int u = 0; u < 2; ++u) r[u] = (b2 ? wv[u + 2] : wv[u]) + dpp_f<0x141>(b2 ? wv[u] : wv[u + 2]);     // row_half_mirror
    const float q = (b0 ? r[1] : r[0]) + dpp_f<0xB1>(b0 ? r[0] : r[1]);                                     // quad_perm [1,0,3,2]
    return q + dpp_f<0x4E>(q);                                                                              // quad_perm [2,3,0,1]
}
static __device__ __forceinline__ int column_sum_key_row(int lane) {       // the key row (0..31) the lane's sum belongs to
    const int u = ((lane >> 4) & 1) * 8 + ((lane >> 3) & 1) * 4 + ((lane >> 2) & 1) * 2 + (lane & 1);
    return (u >> 2) * 8 + (lane >> 5) * 4 + (u & 3);
}

// Prompts of at most KT blocks of 32 tokens: one wave per query block, launched with exactly that many waves.
// The unit's Q and K (two contiguous runs of n rows) are brought in by the whole workgroup with fully coalesced
// loads -- every wave-wide load is 1 KB of consecutive bytes, every byte is requested once per workgroup, all
// requests of a thread are in flight together -- and pass through LDS, from which each wave takes the fragments
// the matrix cores want (lane = row of the block, register = k-slice).  One staging area serves both operands:
// Q goes through it first (every wave leaves with its own query block in registers), then K, which stays for the
// tiles; K's requests are in flight all the while.  Rows are padded by 16 bytes in LDS: with that, the 16 lanes
// of one pass of a 16-byte LDS access hit the 64 banks exactly once, on the way in (16 lanes = 16 consecutive
// fragments of one row) and on the way out (16 lanes = 16 consecutive rows).
// The logits stay in registers between the two sweeps.
// A workgroup takes units blockIdx.x, blockIdx.x + gridDim.x, ... (the grid is sized to what the chip holds at
// once): the next unit's rows are requested as soon as this unit's have left the registers for LDS, so the
// memory pipe stays busy while the matrix cores and the softmax arithmetic work on the current unit.
template <typename T, int D, int KT>
__global__ __launch_bounds__(64 * KT) void prefill_scores_short_kernel(PrefillArgs a) {
    typedef typename Mma<T>::Frag Frag;
    constexpr int NK = D / Mma<T>::KSTEP;
    constexpr int ROW = D * (int)sizeof(T);                // bytes of a row in memory
    constexpr int STRIDE = ROW + 16;                       // ... and in LDS
    constexpr int FPR = ROW / 16;                          // 16-byte fragments per row
    constexpr int NF = FPR / 2;                            // fragments of one operand per thread: 32 rows per wave of 64 threads
    extern __shared__ __align__(16) unsigned char lds_raw[];
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // = this wave's query block
    const int waves = blockDim.x >> 6;
    const int lane = threadIdx.x & 63;
    const int half = lane >> 5;
    const int l32 = lane & 31;
    const int n = a.n;
    const int n_pad = waves * 32;
    unsigned char *stage = lds_raw;                        // [n_pad][STRIDE]: Q, then K
    float *colsum = reinterpret_cast<float *>(lds_raw + (size_t)n_pad * STRIDE);     // [waves][n]
    float *mine = colsum + (size_t)w * n;

    // thread t owns fragments t, t + threads, ... of either operand (NF of them: n_pad * FPR in all)
    const int n_frag = n * FPR;
    const int step = (int)blockDim.x;
    u32x4_nt_t qv[NF], kv[NF];
    auto request = [&](int unit) {                         // clamped, unconditional: every request is out before the first wait
        const size_t unit_off = (size_t)unit * (size_t)n * (size_t)ROW;
        const char *Qu = a.Q + unit_off;
        const char *Ku = a.K + unit_off;
#pragma unroll
        for (int i = 0; i < NF; ++i) {
            int f = (int)threadIdx.x + i * step;
            f = f < n_frag ? f : n_frag - 1;
            qv[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt_t *>(Qu + (size_t)f * 16));
        }
#pragma unroll
        for (int i = 0; i < NF; ++i) {
            int f = (int)threadIdx.x + i * step;
            f = f < n_frag ? f : n_frag - 1;
            kv[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt_t *>(Ku + (size_t)f * 16));
        }
    };
    const u32x4_nt_t zero = {0u, 0u, 0u, 0u};
    auto to_lds = [&](const u32x4_nt_t (&v)[NF]) {
#pragma unroll
        for (int i = 0; i < NF; ++i) {
            const int f = (int)threadIdx.x + i * step;
            if (f < n_pad * FPR)                           // rows past the prompt's end: zeros (masked later anyway)
                *reinterpret_cast<u32x4_nt_t *>(stage + (f / FPR) * STRIDE + (f % FPR) * 16) = f < n_frag ? v[i] : zero;
        }
    };
    // a wave only ever writes the columns of its own key blocks; the others stay zero for every unit
    for (int j = lane; j < n; j += 64) mine[j] = 0.f;

    int unit = (int)blockIdx.x;                            // < n_units (the grid is never larger)
    request(unit);
    for (;;) {
        to_lds(qv);
        __syncthreads();
        Frag qa[NK], kf[NK];
        {
            const unsigned char *qrow = stage + (size_t)(w * 32 + l32) * STRIDE;
#pragma unroll
            for (int ks = 0; ks < NK; ++ks) qa[ks] = lds_frag<T>(qrow, ks, half);
        }
        __syncthreads();                                   // everybody has its query block: the area is free for K
        to_lds(kv);
        __syncthreads();
        const int next = unit + (int)gridDim.x;
        if (next < a.n_units) request(next);               // wave-uniform

        // logits of this query block against key blocks 0..w, kept in registers; running maximum per lane
        float z[KT][16];
        float m_lane = NEG_BIG;
        const bool whole = n == n_pad;                     // the prompt fills its last block: nothing lies beyond n
#pragma unroll
        for (int kb = 0; kb < KT; ++kb) {
            if (kb <= w) {
                const unsigned char *krow = stage + (size_t)(kb * 32 + l32) * STRIDE;
#pragma unroll
                for (int ks = 0; ks < NK; ++ks) kf[ks] = lds_frag<T>(krow, ks, half);
                logits_tile_keys_in_regs<T, D>(kf, qa, w, kb, n, l32, half, a.qscale, whole && kb < w, z[kb]);
#pragma unroll
                for (int v = 0; v < 16; ++v) m_lane = fmaxf(m_lane, z[kb][v]);
            }
        }
        // the query of lanes l and l + 32: maximum and sum over both halves' keys
        float h0, h1;
        halves_pair(m_lane, h0, h1);
        const float m_row = fmaxf(h0, h1);
        float l_lane = 0.f;
#pragma unroll
        for (int kb = 0; kb < KT; ++kb) {
            if (kb <= w) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {             // a masked logit gives exp2(-3e38 - m) = 0; a query beyond n is zeroed below
                    z[kb][v] = fast_exp2(z[kb][v] - m_row);
                    l_lane += z[kb][v];
                }
            }
        }
        halves_pair(l_lane, h0, h1);
        const float inv_l = (w * 32 + l32 < n) ? __builtin_amdgcn_rcpf(h0 + h1) : 0.f;
        const int key_row = column_sum_key_row(lane);
#pragma unroll
        for (int kb = 0; kb < KT; ++kb) {
            if (kb <= w) {
#pragma unroll
                for (int v = 0; v < 16; ++v) z[kb][v] *= inv_l;
                const float cs = column_sums_over_lanes(z[kb], lane);
                const int key = kb * 32 + key_row;
                if ((lane & 2) == 0 && key < n) mine[key] = cs;
            }
        }
        write_scores(a, colsum, waves, unit);              // starts with a barrier: every wave is done with the staged K
        if (next >= a.n_units) break;
        unit = next;
        // the next round's column sums are written only after three more barriers: write_scores' reads are long over
    }
}

// Grid of a kernel whose workgroups walk the units with a stride of the grid size: as many workgroups as are
// resident at once (workgroups per compute unit x compute units of the current device), trimmed so that every
// workgroup gets the same number of units, give or take one at the very end.  0 on failure.
static dim3 resident_grid(int n_units, int per_cu) {
    int dev = 0, cus = 0;
    if (per_cu < 1 || hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return dim3(0);
    const long long resident = (long long)per_cu * cus;
    const long long rounds = (n_units + resident - 1) / resident;
    return dim3((unsigned)((n_units + rounds - 1) / rounds));
}

// LDS of the short kernel: the staging area of one operand and the waves' column sums.
static size_t short_lds_bytes(int waves, int n, int row_bytes) {
    return (size_t)(waves * 32) * (size_t)(row_bytes + 16) + (size_t)waves * (size_t)n * sizeof(float);
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
    a.n_units = n_units;
    a.n = n_src;
    a.row_bytes = d * (dtype == SSD_F32 ? 4 : 2);
    a.qscale = (softmax_scale > 0.f ? softmax_scale : 1.0f / sqrtf((float)d)) * LOG2E;
    const int n_blocks = (n_src + 31) / 32;
    const int waves = n_blocks < 4 ? n_blocks : 4;
    const size_t lds_long = (size_t)waves * (size_t)n_src * sizeof(float);
    const size_t lds_short = short_lds_bytes(waves, n_src, a.row_bytes);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)n_units), block(64u * waves);
    hipError_t attr = hipSuccess;
    // more than 64 KB of dynamic LDS has to be asked for (the longest short prompts in fp32: 70 KB of the CU's 160 KB)
#define SSD_PREFILL_SHORT(T_, D_, KT_)                                                                                          \
    do {                                                                                                                        \
        const void *fn = reinterpret_cast<const void *>(&prefill_scores_short_kernel<T_, D_, KT_>);                             \
        if (lds_short > 65536) attr = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_short);      \
        int per_cu = 0;                                                                                                         \
        if (attr == hipSuccess) attr = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, (int)block.x, lds_short);      \
        if (attr == hipSuccess) {                                                                                               \
            const dim3 g = resident_grid(n_units, per_cu);                                                                      \
            if (g.x == 0) attr = hipErrorInvalidValue;                                                                          \
            else hipLaunchKernelGGL((prefill_scores_short_kernel<T_, D_, KT_>), g, block, lds_short, s, a);                     \
        }                                                                                                                       \
    } while (0)
#define SSD_PREFILL(T_, D_)                                                                                          \
    do {                                                                                                             \
        if (n_blocks <= 2) SSD_PREFILL_SHORT(T_, D_, 2);                                                             \
        else if (n_blocks <= 4) SSD_PREFILL_SHORT(T_, D_, 4);                                                        \
        else hipLaunchKernelGGL((prefill_scores_kernel<T_, D_>), grid, block, lds_long, s, a);                       \
    } while (0)
    if (dtype == SSD_BF16) {
        if (d == 128) SSD_PREFILL(bf16_t, 128); else SSD_PREFILL(bf16_t, 64);
    } else {
        if (d == 128) SSD_PREFILL(float, 128); else SSD_PREFILL(float, 64);
    }
#undef SSD_PREFILL
#undef SSD_PREFILL_SHORT
    if (attr != hipSuccess) return hip_fail(attr, "prefill score kernel attribute");
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "prefill score launch");
    return SSD_OK;
}
