// Device-side building blocks: 16-byte row-fragment loads, bf16 <-> fp32, reductions inside a
// wave64, and the streaming softmax-attention loop that both the compressed-cache kernel and the
// full-cache baseline kernel instantiate.
//
// Work decomposition (gfx950, wave64): a K or V row of d elements is d*e bytes; each lane owns one
// 16-byte fragment of a row, so a row occupies LPR = d*e/16 adjacent lanes (16 for bf16 d=128) and
// one wave-wide load instruction brings in RPW = 64/LPR whole rows, 1 KB, fully coalesced.  The
// q.k dot product is reduced over the LPR lanes of a row with DPP moves (never through memory);
// each group of LPR lanes runs its own online softmax over the rows it sees and the RPW groups
// are merged once at the end.  The arithmetic is ~1 flop per byte streamed: there is no dense
// contraction here and therefore no MFMA.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ssd_internal.h"

namespace ssd {

static constexpr float NEG_BIG = -3.0e38f;   // "minus infinity" that stays finite under subtraction
static constexpr float LOG2E = 1.4426950408889634f;

struct bf16_t { uint16_t bits; };   // tag type: storage is a raw bfloat16

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

// Elem<T>: how a 16-byte fragment of T is turned into arithmetic.
//   Q       : register form of this lane's query fragment
//   dot     : fp32 dot product of the query fragment with a raw K fragment
//   unpack  : raw fragment -> VEC floats (for the p * V accumulation)
template <typename T> struct Elem;

template <> struct Elem<float> {
    static constexpr int VEC = 4;
    struct Q { float f[4]; };
    static __device__ __forceinline__ void unpack(const uint4 &r, float (&f)[4]) {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
    static __device__ __forceinline__ uint4 pack(const float (&f)[4]) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
    static __device__ __forceinline__ Q load_q(const uint4 &r) {
        Q q;
        unpack(r, q.f);
        return q;
    }
    static __device__ __forceinline__ float dot(const Q &q, const uint4 &k) {
        float d = q.f[0] * __uint_as_float(k.x);
        d = fmaf(q.f[1], __uint_as_float(k.y), d);
        d = fmaf(q.f[2], __uint_as_float(k.z), d);
        d = fmaf(q.f[3], __uint_as_float(k.w), d);
        return d;
    }
};

// round-to-nearest-even fp32 -> bf16 (NaN stays NaN)
static __device__ __forceinline__ uint32_t f32_to_bf16_bits(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

template <> struct Elem<bf16_t> {
    static constexpr int VEC = 8;
    struct Q { uint4 r; };      // the query stays packed: v_dot2_f32_bf16 multiplies bf16 pairs exactly into fp32
    static __device__ __forceinline__ void unpack(const uint4 &r, float (&f)[8]) {
        f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
        f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
        f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
        f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
    }
    static __device__ __forceinline__ uint4 pack(const float (&f)[8]) {
        return make_uint4(f32_to_bf16_bits(f[0]) | (f32_to_bf16_bits(f[1]) << 16),
                          f32_to_bf16_bits(f[2]) | (f32_to_bf16_bits(f[3]) << 16),
                          f32_to_bf16_bits(f[4]) | (f32_to_bf16_bits(f[5]) << 16),
                          f32_to_bf16_bits(f[6]) | (f32_to_bf16_bits(f[7]) << 16));
    }
    static __device__ __forceinline__ Q load_q(const uint4 &r) { return Q{r}; }
    static __device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float c) {
        return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
    }
    static __device__ __forceinline__ float dot(const Q &q, const uint4 &k) {
        float d = dot2(q.r.x, k.x, 0.f);
        d = dot2(q.r.y, k.y, d);
        d = dot2(q.r.z, k.z, d);
        d = dot2(q.r.w, k.w, d);
        return d;
    }
};

// ---- streaming loads -------------------------------------------------------
//
// A 16-byte fragment of cache data that this launch reads exactly once.  The load carries the non-temporal
// hint, so the line is first in line for replacement in L2 instead of pushing out what is worth keeping there:
// the lines this launch has written (new rows, outputs, scores).  With ordinary loads the read stream -- 35
// times the size of all L2s per layer of the 7B shape -- evicts those dirty lines one by one and their
// write-backs trickle into the reads all through the launch; measured on that shape, the hint alone takes the
// fused step from 0.762 to 0.718 ms (two streams) and from 0.827 to 0.787 ms (one stream).
typedef uint32_t u32x4_nt_t __attribute__((ext_vector_type(4)));
static __device__ __forceinline__ uint4 load_once(const char *p) {
    const u32x4_nt_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_nt_t *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// ---- reductions over the lanes of a wave64 ---------------------------------

template <int CTRL> static __device__ __forceinline__ float dpp_f(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, false));
}

// Sum over an aligned group of G adjacent lanes (G = 8, 16 or 32); every lane of the group gets the sum.
template <int G> static __device__ __forceinline__ float group_sum(float v) {
    v += dpp_f<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_f<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_f<0x141>(v);   // row_half_mirror: 8 lanes done
    if (G >= 16) v += dpp_f<0x140>(v);   // row_mirror: 16 lanes done
    if (G >= 32) v += __shfl_xor(v, 16);
    return v;
}

// Exchange with the lane 16 (resp. 32) positions away, as two VALU swaps instead of LDS-crossbar
// permutes: v_permlane16_swap trades the odd 16-lane rows of its first operand with the even rows of
// its second, v_permlane32_swap the upper half of the first with the lower half of the second.  Fed the
// same value twice, the two results hold, in every lane, the value of its own row (half) and of the
// partner row (half).
typedef unsigned uint2v_t __attribute__((ext_vector_type(2)));
static __device__ __forceinline__ void rows_pair(float v, float &a, float &b) {
    const uint2v_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    a = __uint_as_float(r.x); b = __uint_as_float(r.y);
}
static __device__ __forceinline__ void halves_pair(float v, float &a, float &b) {
    const uint2v_t r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    a = __uint_as_float(r.x); b = __uint_as_float(r.y);
}

// Combine the values held by the 64/G groups of a wave (lanes equal inside a group on entry).
template <int G> static __device__ __forceinline__ float across_groups_sum(float v) {
    float a, b;
    if (G <= 8) v += dpp_f<0x128>(v);                  // row_ror:8 = the lane 8 away inside a 16-lane row
    if (G <= 16) { rows_pair(v, a, b); v = a + b; }
    halves_pair(v, a, b);
    return a + b;
}
template <int G> static __device__ __forceinline__ float across_groups_max(float v) {
    float a, b;
    if (G <= 8) v = fmaxf(v, dpp_f<0x128>(v));
    if (G <= 16) { rows_pair(v, a, b); v = fmaxf(a, b); }
    halves_pair(v, a, b);
    return fmaxf(a, b);
}

// Minimum of a 64-bit key over the 64 lanes of a wave; every lane gets it.
template <int CTRL> static __device__ __forceinline__ unsigned long long dpp_u64(unsigned long long v) {
    const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)v, CTRL, 0xF, 0xF, false);
    const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)(v >> 32), CTRL, 0xF, 0xF, false);
    return ((unsigned long long)hi << 32) | lo;
}
static __device__ __forceinline__ unsigned long long min_u64(unsigned long long a, unsigned long long b) { return a < b ? a : b; }
static __device__ __forceinline__ unsigned long long wave_min_u64(unsigned long long v) {
    v = min_u64(v, dpp_u64<0xB1>(v));      // quad_perm [1,0,3,2]
    v = min_u64(v, dpp_u64<0x4E>(v));      // quad_perm [2,3,0,1]
    v = min_u64(v, dpp_u64<0x141>(v));     // row_half_mirror
    v = min_u64(v, dpp_u64<0x140>(v));     // row_mirror: 16 lanes done
    {
        const uint2v_t lo = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
        const uint2v_t hi = __builtin_amdgcn_permlane16_swap((unsigned)(v >> 32), (unsigned)(v >> 32), false, false);
        v = min_u64(((unsigned long long)hi.x << 32) | lo.x, ((unsigned long long)hi.y << 32) | lo.y);
    }
    {
        const uint2v_t lo = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
        const uint2v_t hi = __builtin_amdgcn_permlane32_swap((unsigned)(v >> 32), (unsigned)(v >> 32), false, false);
        v = min_u64(((unsigned long long)hi.x << 32) | lo.x, ((unsigned long long)hi.y << 32) | lo.y);
    }
    return v;
}

static __device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// slot of the r-th valid row of a unit (branch-free: two compares and selects)
static __device__ __forceinline__ int seg_slot(const Segs &s, int r) {
    const int e0 = s.len[0], e1 = s.len[0] + s.len[1];
    const int a0 = s.start[0], a1 = s.start[1] - e0, a2 = s.start[2] - e1;
    return r + (r < e0 ? a0 : (r < e1 ? a1 : a2));
}

// ---- the streaming loop ----------------------------------------------------
//
// State of one lane group's online softmax (log2 domain: logits are pre-multiplied by log2 e).
template <int VEC> struct Softmax {
    float m, l, acc[VEC];
    float far, tot;     // only used by the full-cache kernel's mass outputs
    __device__ __forceinline__ void init() {
        m = NEG_BIG; l = 0.f; far = 0.f; tot = 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) acc[i] = 0.f;
    }
};

// Stream valid rows of one unit.  Rows are taken RPW at a time ("iterations", one wave-wide 1 KB
// load of K and one of V); this wave handles iterations first_iter, first_iter + iter_stride, ...
// counted from row_begin, so the waves that share a unit read adjacent 1 KB pieces at the same
// time.  CH iterations form a chunk; the loads of the next chunk are issued before the arithmetic
// of the current one (two register buffers), so a wave always has requests in flight.
//   Kb, Vb    : first K / V row of the unit (slot 0); wave-uniform
//   sg        : valid-slot runs; row index r means the r-th valid row
//   q, qscale : this lane's query fragment and softmax scale * log2(e)
//   zbuf      : LDS, receives the scaled logit of every row (index r) when ZBUF
//   MASS      : also accumulate the probability mass of rows >= vis_start (tot) and of rows in
//               [vis_start, far_last] (far)
// first_iter and iter_stride must be wave-uniform (scalar) values.
// after_first_issue() runs once, right after the loads of the first chunk have been issued: work that
// needs data requested before the stream (and so returned before it) can go there without delaying it.
struct NoHook { __device__ __forceinline__ void operator()() const {} };

// PAD: every chunk issues its full 2 * CH loads and consumes them all (see `load` and `compute`); this is what
// launches of few rounds want.  Without it loads and arithmetic past the end are skipped, which is slightly
// better when many rounds of waves hide each other's waits anyway (the full-cache kernel).
template <typename T, int D, int CH, bool ZBUF, bool MASS, typename Hook = NoHook, bool PAD = true>
static __device__ __forceinline__ void stream_rows(const char *__restrict__ Kb, const char *__restrict__ Vb,
                                                  int row_bytes, const Segs &sg, int row_begin, int row_end,
                                                  int first_iter, int iter_stride,
                                                  const typename Elem<T>::Q &q, float qscale,
                                                  Softmax<Elem<T>::VEC> &sm, float *zbuf, int vis_start, int far_last,
                                                  Hook after_first_issue = Hook()) {
    constexpr int VEC = Elem<T>::VEC;
    constexpr int LPR = D / VEC;
    constexpr int RPW = 64 / LPR;
    const int lane = threadIdx.x & 63;
    const int grp = lane / LPR;
    const uint32_t lane_off = (uint32_t)(lane % LPR) * 16u;
    const int n_iter = (row_end - row_begin + RPW - 1) / RPW;
    const int chunk_iters = CH * iter_stride;

    // Issue the loads of the chunk that starts at iteration it0.  Always exactly 2 * CH loads, whatever
    // it0: rows past the end are clamped to the last row (a cache line some lane has just fetched, so no
    // extra HBM traffic).  A fixed number of requests per chunk is what lets the compiler wait for "all but
    // the newest chunk" instead of "everything": with loads under a condition it has to assume the fewest.
    auto load = [&](int it0, uint4 (&kr)[CH], uint4 (&vr)[CH]) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            if (!PAD && it0 + i * iter_stride >= n_iter) continue;   // wave-uniform
            int r = row_begin + (it0 + i * iter_stride) * RPW + grp;
            r = r < row_end ? r : row_end - 1;
            uint32_t off = (uint32_t)seg_slot(sg, r) * (uint32_t)row_bytes + lane_off;
            kr[i] = load_once(Kb + off);
            vr[i] = load_once(Vb + off);
        }
    };
    auto compute = [&](int it0, const uint4 (&kr)[CH], const uint4 (&vr)[CH]) {
        float z[CH];
        float mx = NEG_BIG;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int it = it0 + i * iter_stride;
            const int r = row_begin + it * RPW + grp;
            const bool ok = it < n_iter && r < row_end;
            const float dot = group_sum<LPR>(Elem<T>::dot(q, kr[i]));
            z[i] = ok ? dot * qscale : NEG_BIG;
            mx = fmaxf(mx, z[i]);
        }
        const float m_new = fmaxf(sm.m, mx);
        const float alpha = fast_exp2(sm.m - m_new);
        sm.l *= alpha;
        if (MASS) { sm.far *= alpha; sm.tot *= alpha; }
#pragma unroll
        for (int e = 0; e < VEC; ++e) sm.acc[e] *= alpha;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            // rows past the end were clamped to the unit's last row on loading: finite data, weight 0.  They are
            // masked rather than skipped, so that every loaded fragment is consumed on every path and no load
            // stays pending across the loop's back edge (which would cost a full wait at the loop head).
            const int it = it0 + i * iter_stride;
            if (!PAD && it >= n_iter) continue;                      // wave-uniform
            const int r = row_begin + it * RPW + grp;
            const bool ok = it < n_iter && r < row_end;
            const float p = ok ? fast_exp2(z[i] - m_new) : 0.f;
            sm.l += p;
            float vf[VEC];
            Elem<T>::unpack(vr[i], vf);
#pragma unroll
            for (int e = 0; e < VEC; ++e) sm.acc[e] = fmaf(p, vf[e], sm.acc[e]);
            if (ZBUF) { if (ok && lane_off == 0) zbuf[r] = z[i]; }
            if (MASS) {
                sm.tot += (r >= vis_start) ? p : 0.f;
                sm.far += (r >= vis_start && r <= far_last) ? p : 0.f;
            }
        }
        sm.m = m_new;
    };

    int it = first_iter;
    if (it >= n_iter) { after_first_issue(); return; }
    uint4 ka[CH], va[CH], kb[CH], vb[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) { ka[i] = va[i] = kb[i] = vb[i] = make_uint4(0, 0, 0, 0); }
    load(it, ka, va);
    after_first_issue();
    for (;;) {                                     // PAD: the chunk after the last one is requested too (clamped) and dropped
        if (PAD || it + chunk_iters < n_iter) load(it + chunk_iters, kb, vb);
        compute(it, ka, va);
        it += chunk_iters;
        if (it >= n_iter) break;
        if (PAD || it + chunk_iters < n_iter) load(it + chunk_iters, ka, va);
        compute(it, kb, vb);
        it += chunk_iters;
        if (it >= n_iter) break;
    }
}

// Merge the RPW lane groups of a wave: afterwards every lane holds the wave-wide max m, the
// wave-wide l (and far/tot) and the full sum of its own output fragment.
template <int VEC, int LPR, bool MASS> static __device__ __forceinline__ void merge_groups(Softmax<VEC> &sm) {
    const float m_all = across_groups_max<LPR>(sm.m);
    const float f = fast_exp2(sm.m - m_all);
    sm.m = m_all;
    sm.l = across_groups_sum<LPR>(sm.l * f);
    if (MASS) {
        sm.far = across_groups_sum<LPR>(sm.far * f);
        sm.tot = across_groups_sum<LPR>(sm.tot * f);
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) sm.acc[e] = across_groups_sum<LPR>(sm.acc[e] * f);
}

// Addresses of one (layer, sequence, head) unit of the compressed cache.
struct UnitRef {
    bool sem;
    char *K;          // slot 0 of the K plane
    char *V;          // slot 0 of the V plane
    float *score;     // semantic only: [M+C]
    int32_t *pos;     // semantic only: [M+C]
};

// Index of the k-th set bit (k = 0 for the lowest) of the 128-bit mask (m1:m0); k must be below the
// number of set bits.  Scalar arithmetic: a popcount-guided binary search.
static __device__ __forceinline__ int kth_set_bit(uint64_t m0, uint64_t m1, int k) {
    int r = 0;
    uint64_t m = m0;
    const int c0 = __popcll(m0);
    if (k >= c0) { k -= c0; r = 64; m = m1; }
    uint32_t lo = (uint32_t)m;
    const int c = __popc(lo);
    if (k >= c) { k -= c; r += 32; lo = (uint32_t)(m >> 32); }
#pragma unroll
    for (int wd = 16; wd >= 1; wd >>= 1) {
        const int cc = __popc(lo & ((1u << wd) - 1u));
        if (k >= cc) { k -= cc; r += wd; lo >>= wd; }
    }
    return r;
}

// Addresses of the unit that is the `local`-th head of its type (sem) in its layer, sequence b.
static __device__ __forceinline__ UnitRef unit_ref_local(const Geom &g, const LayerDesc &ld, int b, bool sem, int local) {
    UnitRef u;
    u.sem = sem;
    if (sem) {
        const size_t idx = (size_t)b * (size_t)ld.n_se + (size_t)local;
        u.K = g.base + ld.off_se + idx * (size_t)g.unit_se_bytes;
        u.V = u.K + (size_t)(g.M + g.C) * (size_t)g.row_bytes;
        u.score = reinterpret_cast<float *>(g.base + ld.off_score) + idx * (size_t)(g.M + g.C);
        u.pos = reinterpret_cast<int32_t *>(g.base + ld.off_pos) + idx * (size_t)(g.M + g.C);
    } else {
        const size_t idx = (size_t)b * (size_t)ld.n_sp + (size_t)local;
        u.K = g.base + ld.off_sp + idx * (size_t)g.unit_sp_bytes;
        u.V = u.K + (size_t)(g.S + g.RW) * (size_t)g.row_bytes;
        u.score = nullptr;
        u.pos = nullptr;
    }
    return u;
}

// ld: the layer's entry of the launch's LaunchMeta (kernel-argument memory, scalar loads)
static __device__ __forceinline__ UnitRef unit_ref(const Geom &g, const LayerDesc &ld, int b, int h) {
    UnitRef u;
    const uint64_t m0 = ld.sem_mask[0], m1 = ld.sem_mask[1];
    const uint64_t word = h < 64 ? m0 : m1;
    const uint64_t below = (1ull << (h & 63)) - 1ull;
    u.sem = ((word >> (h & 63)) & 1ull) != 0;
    // semantic heads with a lower index than h
    const int sem_below = h < 64 ? __popcll(m0 & below) : __popcll(m0) + __popcll(m1 & below);
    if (u.sem) {
        const size_t idx = (size_t)b * (size_t)ld.n_se + (size_t)sem_below;
        u.K = g.base + ld.off_se + idx * (size_t)g.unit_se_bytes;
        u.V = u.K + (size_t)(g.M + g.C) * (size_t)g.row_bytes;
        u.score = reinterpret_cast<float *>(g.base + ld.off_score) + idx * (size_t)(g.M + g.C);
        u.pos = reinterpret_cast<int32_t *>(g.base + ld.off_pos) + idx * (size_t)(g.M + g.C);
    } else {
        const size_t idx = (size_t)b * (size_t)ld.n_sp + (size_t)(h - sem_below);
        u.K = g.base + ld.off_sp + idx * (size_t)g.unit_sp_bytes;
        u.V = u.K + (size_t)(g.S + g.RW) * (size_t)g.row_bytes;
        u.score = nullptr;
        u.pos = nullptr;
    }
    return u;
}

}  // namespace ssd
