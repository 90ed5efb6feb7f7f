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

template <typename T> struct Elem;

template <> struct Elem<float> {
    static constexpr int VEC = 4;
    static __device__ __forceinline__ void unpack(const uint4 &r, float (&f)[4]) {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
    static __device__ __forceinline__ uint4 pack(const float (&f)[4]) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
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
};

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

// Combine the values held by the 64/G groups of a wave (lanes equal inside a group on entry).
template <int G> static __device__ __forceinline__ float across_groups_sum(float v) {
#pragma unroll
    for (int off = G; off < 64; off <<= 1) v += __shfl_xor(v, off);
    return v;
}
template <int G> static __device__ __forceinline__ float across_groups_max(float v) {
#pragma unroll
    for (int off = G; off < 64; off <<= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}

static __device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// slot of the r-th valid row of a unit
static __device__ __forceinline__ int seg_slot(const Segs &s, int r) {
    if (r < s.len[0]) return s.start[0] + r;
    r -= s.len[0];
    if (r < s.len[1]) return s.start[1] + r;
    return s.start[2] + (r - s.len[1]);
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

// Stream the valid rows [row_begin, row_end) of one unit.
//   Kb, Vb    : first K / V row of the unit (slot 0)
//   sg        : valid-slot runs; row index r means the r-th valid row
//   q         : this lane's VEC query elements, already multiplied by scale * log2(e)
//   zbuf      : wave-private LDS, receives the logit of every row (index r) when ZBUF
//   MASS      : also accumulate the probability mass of rows >= vis_start (tot) and of rows in
//               [vis_start, far_last] (far)
template <typename T, int D, int CH, bool ZBUF, bool MASS>
static __device__ __forceinline__ void stream_rows(const char *__restrict__ Kb, const char *__restrict__ Vb,
                                                  int row_bytes, const Segs &sg, int row_begin, int row_end,
                                                  const float (&q)[Elem<T>::VEC], Softmax<Elem<T>::VEC> &sm,
                                                  float *zbuf, int vis_start, int far_last) {
    constexpr int VEC = Elem<T>::VEC;
    constexpr int LPR = D / VEC;
    constexpr int RPW = 64 / LPR;
    const int lane = threadIdx.x & 63;
    const int grp = lane / LPR;
    const int sub = lane % LPR;

    for (int r0 = row_begin; r0 < row_end; r0 += RPW * CH) {
        uint4 kr[CH], vr[CH];
        bool ok[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int r = r0 + i * RPW + grp;
            ok[i] = r < row_end;
            const int slot = seg_slot(sg, ok[i] ? r : row_begin);
            const size_t off = (size_t)slot * (size_t)row_bytes + (size_t)sub * 16u;
            if (ok[i]) {
                kr[i] = *reinterpret_cast<const uint4 *>(Kb + off);
                vr[i] = *reinterpret_cast<const uint4 *>(Vb + off);
            } else {
                kr[i] = make_uint4(0, 0, 0, 0);
                vr[i] = make_uint4(0, 0, 0, 0);
            }
        }
        float z[CH];
        float mx = NEG_BIG;
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            float kf[VEC];
            Elem<T>::unpack(kr[i], kf);
            float dot = 0.f;
#pragma unroll
            for (int e = 0; e < VEC; ++e) dot = fmaf(q[e], kf[e], dot);
            dot = group_sum<LPR>(dot);
            z[i] = ok[i] ? dot : NEG_BIG;
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
            const int r = r0 + i * RPW + grp;
            const float p = ok[i] ? fast_exp2(z[i] - m_new) : 0.f;
            sm.l += p;
            float vf[VEC];
            Elem<T>::unpack(vr[i], vf);
#pragma unroll
            for (int e = 0; e < VEC; ++e) sm.acc[e] = fmaf(p, vf[e], sm.acc[e]);
            if (ZBUF) { if (ok[i] && sub == 0) zbuf[r] = z[i]; }
            if (MASS) {
                sm.tot += (r >= vis_start) ? p : 0.f;
                sm.far += (r >= vis_start && r <= far_last) ? p : 0.f;
            }
        }
        sm.m = m_new;
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

static __device__ __forceinline__ UnitRef unit_ref(const Geom &g, int layer, int b, int h) {
    UnitRef u;
    const uint32_t info = g.hinfo[layer * g.H + h];
    const LayerMeta lm = g.lmeta[layer];
    const uint32_t hl = info & ~HEAD_SEM_BIT;
    u.sem = (info & HEAD_SEM_BIT) != 0;
    if (u.sem) {
        const size_t idx = (size_t)b * (size_t)lm.n_se + hl;
        u.K = g.base + lm.off_se + idx * (size_t)g.unit_se_bytes;
        u.V = u.K + (size_t)(g.M + g.C) * (size_t)g.row_bytes;
        u.score = reinterpret_cast<float *>(g.base + lm.off_score) + idx * (size_t)(g.M + g.C);
        u.pos = reinterpret_cast<int32_t *>(g.base + lm.off_pos) + idx * (size_t)(g.M + g.C);
    } else {
        const size_t idx = (size_t)b * (size_t)lm.n_sp + hl;
        u.K = g.base + lm.off_sp + idx * (size_t)g.unit_sp_bytes;
        u.V = u.K + (size_t)(g.S + g.W) * (size_t)g.row_bytes;
        u.score = nullptr;
        u.pos = nullptr;
    }
    return u;
}

}  // namespace ssd
