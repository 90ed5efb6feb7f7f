// Top-M selection and slot-stable consolidation of one semantic head, executed by one workgroup
// (Algorithm 1 "IndicesOfTopM" / "SelectAndAppend"; Algorithm 2 "Compress semantic cache").
//
// Selection is exact integer work: a candidate's (score, position) pair becomes one 64-bit key
//   key = score_bits << 32 | (0xFFFFFFFF - position)
// Scores are sums of probabilities, hence non-negative floats, whose IEEE bit patterns order like
// the numbers; the inverted position makes the lower position win a tie.  Keys are distinct, so
// rank(i) = #{j : key_j > key_i} is a total order and "rank < M" is the kept set -- the same set
// any correct sort would give, bit for bit.  The candidates of one head live in LDS and every
// thread counts ranks for its own candidates; the inner loop reads one LDS word per step as a
// broadcast, so there are no bank conflicts.
//
// Consolidation is slot-stable: a heavy token that survives stays where it is; buffered tokens
// that are promoted fill the slots of evicted (or never used) heavy slots, so the rows moved per
// compression are only the newly promoted ones.  The row buffer is a ring, so the R protected
// newest tokens stay put as well.
#pragma once

#include "ssd_device.h"

namespace ssd {

static __device__ __forceinline__ unsigned long long make_key(float score, int pos) {
    return ((unsigned long long)__float_as_uint(score) << 32) | (unsigned long long)(0xFFFFFFFFu - (uint32_t)pos);
}
static __device__ __forceinline__ float key_score(unsigned long long k) { return __uint_as_float((uint32_t)(k >> 32)); }
static __device__ __forceinline__ int key_pos(unsigned long long k) { return (int)(0xFFFFFFFFu - (uint32_t)(k & 0xFFFFFFFFull)); }

// Make LDS writes of this wave's lanes visible to its other lanes (a unit handled by one wave needs no
// workgroup barrier).  LDS only: it does not wait for this wave's outstanding global stores, which would
// put a full memory round trip into the tail of every unit.
static __device__ __forceinline__ void lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Order this wave's earlier global stores before its later global loads and stores (rows, scores and
// positions that one lane wrote and another lane of the same wave is about to read or overwrite).
static __device__ __forceinline__ void wave_global_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

template <bool WAVE> static __device__ __forceinline__ void unit_sync() {
    if (WAVE) lds_sync();
    else __syncthreads();
}

// Exclusive prefix count of `flag` over the lanes of one wave, plus the wave total.
static __device__ __forceinline__ int wave_prefix(bool flag, int &total) {
    const unsigned long long mask = __ballot(flag);
    const int lane = threadIdx.x & 63;
    total = __popcll(mask);
    return __popcll(mask & ((1ull << lane) - 1ull));
}

// LDS bytes select_and_move needs for n_cand candidates of which n_old come from the row buffer.
static __host__ __device__ inline size_t select_lds_bytes(int M, int n_cand, int n_old) {
    size_t b = 8 * (size_t)n_cand + 64 + 4 * (size_t)M + 4 * (size_t)n_old + 8 + (size_t)M + (size_t)n_old;
    return (b + 15) / 16 * 16;
}

// Candidates i = 0..n_cand-1: i < m is heavy slot i; i >= m is the (i-m)-th oldest buffered token,
// living in slot M + (base + i - m) mod C.  On entry keys[0..n_cand) are in LDS (at `lds`, 8-byte
// aligned) and a barrier of the cooperating threads has made them visible.  On exit the kept candidates occupy
// heavy slots [0, min(M, n_cand)) with their rows, positions and scores.
//
// M is the head's budget (at most g.M, the layer-wide size of the heavy region that the row buffer follows).
//
// THREADS threads with ids tid = 0..THREADS-1 cooperate: a whole workgroup (WAVE = false, synchronised
// with __syncthreads) or a single wave (WAVE = true, THREADS = 64, tid = lane).
template <int THREADS, bool WAVE>
static __device__ __forceinline__ void select_and_move(const Geom &g, const UnitRef &u, unsigned char *lds, int n_cand,
                                                      int m, int n_old, int base, int lpr, int tid, int M) {
    const int C = g.C;
    unsigned long long *keys = reinterpret_cast<unsigned long long *>(lds);   // [n_cand]
    unsigned long long *wave_least = keys + n_cand;                            // [8]     one minimum per wave of a workgroup
    int *dest = reinterpret_cast<int *>(wave_least + 8);                       // [M]     free heavy slots, ascending
    int *src = dest + M;                                                       // [n_old] promoted candidates (indices)
    int *counts = src + n_old;                                                 // [2]
    unsigned char *flag = reinterpret_cast<unsigned char *>(counts + 2);       // [M + n_old]

    // rank by counting; bit k of keepbits = candidate tid + k*THREADS is kept
    unsigned long long keepbits = 0;
    static_assert((4096 + THREADS - 1) / THREADS <= 64, "one 64-bit mask per thread");
    const int n_evict = n_cand - M;
    const int per = (n_cand + THREADS - 1) / THREADS;                // candidates per thread
    if (n_cand <= M) {
        keepbits = ~0ull;
    } else if ((long long)n_evict * (per + (WAVE ? 20 : 60)) < (long long)per * n_cand) {
        // Few evictions among many candidates (compression after every token: one): take the smallest keys out one
        // by one -- a pass over this thread's keys and a minimum over all threads each -- instead of ranking every
        // candidate against every other.  Keys are distinct, so each minimum has one owner, and the kept set is the same.
        keepbits = ~0ull;
        for (int e = 0; e < n_evict; ++e) {
            unsigned long long least = ~0ull;
            int at = -1;
            for (int k = 0; k * THREADS + tid < n_cand; ++k) {
                const unsigned long long key = keys[k * THREADS + tid];
                if (((keepbits >> k) & 1ull) && key < least) { least = key; at = k; }
            }
            unsigned long long lowest = wave_min_u64(least);            // every lane takes part, with or without a candidate
            if (!WAVE && THREADS > 64) {                                // a workgroup: the waves' minima meet in LDS
                static_assert(THREADS <= 512, "room for eight waves' minima");
                if ((tid & 63) == 0) wave_least[tid >> 6] = lowest;
                __syncthreads();
#pragma unroll
                for (int wv = 0; wv < THREADS / 64; ++wv) lowest = min_u64(lowest, wave_least[wv]);
                __syncthreads();                                        // before the next round writes the minima again
            }
            if (at >= 0 && least == lowest) keepbits &= ~(1ull << at);
        }
    } else {
        for (int k = 0; k * THREADS + tid < n_cand; ++k) {
            const unsigned long long mine = keys[k * THREADS + tid];
            int rank = 0;
            for (int j = 0; j < n_cand; ++j) rank += keys[j] > mine ? 1 : 0;
            if (rank < M) keepbits |= 1ull << k;
        }
    }
    // flag[s], s < M: heavy slot s is free after compression (evicted or never used)
    // flag[M + j]   : buffered candidate j is promoted
    for (int k = 0; k * THREADS + tid < n_cand; ++k) {
        const int i = k * THREADS + tid;
        const bool keep = (keepbits >> k) & 1ull;
        if (i < m) flag[i] = keep ? 0 : 1;
        else flag[M + (i - m)] = keep ? 1 : 0;
    }
    for (int s = m + tid; s < M; s += THREADS) flag[s] = 1;
    unit_sync<WAVE>();
    if (tid < 64) {       // wave 0 compacts both lists
        int nfree = 0;
        for (int s0 = 0; s0 < M; s0 += 64) {
            const int s = s0 + tid;
            const bool f = s < M && flag[s] != 0;
            int tot;
            const int pre = wave_prefix(f, tot);
            if (f) dest[nfree + pre] = s;
            nfree += tot;
        }
        int nmove = 0;
        for (int j0 = 0; j0 < n_old; j0 += 64) {
            const int j = j0 + tid;
            const bool f = j < n_old && flag[M + j] != 0;
            int tot;
            const int pre = wave_prefix(f, tot);
            if (f) src[nmove + pre] = m + j;
            nmove += tot;
        }
        if (tid == 0) { counts[0] = nfree; counts[1] = nmove; }
    }
    unit_sync<WAVE>();
    const int nmove = counts[1];              // <= counts[0] by construction
    if (WAVE) wave_global_sync();             // rows / scores stored earlier by other lanes of this wave
    // move the promoted tokens: 2*lpr 16-byte fragments per token (K row, V row) ...
    const int frag_per_tok = 2 * lpr;
    for (int t = tid; t < nmove * frag_per_tok; t += THREADS) {
        const int k = t / frag_per_tok;
        const int f = t % frag_per_tok;
        const int kv = f / lpr, sub = f % lpr;
        char *plane = kv ? u.V : u.K;
        const int from = g.M + (base + (src[k] - m)) % C;
        const uint4 v = *reinterpret_cast<const uint4 *>(plane + (size_t)from * g.row_bytes + (size_t)sub * 16u);
        *reinterpret_cast<uint4 *>(plane + (size_t)dest[k] * g.row_bytes + (size_t)sub * 16u) = v;
    }
    // ... and their position and score, which the keys still hold
    for (int k = tid; k < nmove; k += THREADS) {
        const unsigned long long key = keys[src[k]];
        u.pos[dest[k]] = key_pos(key);
        u.score[dest[k]] = key_score(key);
    }
}

}  // namespace ssd
