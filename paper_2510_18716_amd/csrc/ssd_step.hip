// ssd_decode_attn and ssd_decode_step: single-token attention over the compressed cache, the
// running-score update of semantic heads (Algorithm 1: "AttentionScores",
// "AggregateAttentionScores"), and -- in the fused entry point -- the append before it and the
// compression after it, all by the one workgroup that owns the (layer, sequence, head) unit.
//
// One wave64 per unit, a few units per workgroup.  A unit is small (S+W or m+c rows, ~33 KB at
// W = M = 64, d = 128, bf16) and contiguous in HBM, so the kernel is a pure stream: every byte is
// read once, straight into registers (nothing is reused, so there is nothing for LDS staging to
// serve), and a launch exposes thousands of independent units to cover HBM latency.  Spatial and
// semantic units share one launch; they differ only in where their valid rows are.  Because one
// wave owns a unit from the append to the selection, no step needs a workgroup barrier or an atomic.
//
// Roofline: HBM.  Algorithmic bytes per unit and step = rows * 2 * d * e (K and V) + 2 * d * e
// (q in, out) + 8 * rows for a semantic unit's score read-modify-write.
//
// Optional variants of the same kernel: HEADS (every head its own window or budget, taken from a table in the
// arguments; heads dispatched longest first), ROPE (the fused step rotates q and the new k by the token's
// position on the way in) and SHARE (several waves share a unit: for launches of few units).  The plain
// kernel pays for none of them.
#include <algorithm>

#include "ssd_select.h"

namespace ssd {

// What a wave needs from the argument block: these fields and its one entry of the per-layer table.
struct StepHot {
    const char *q;
    char *out;
    const char *k_new;   // fused append only
    const char *v_new;
    float qscale;        // softmax scale * log2(e)
    int layer_off;       // index of the launch's first layer inside q / out / k_new / v_new
    int new_slot_sp;     // fused append: destination slots and position of the new token
    int new_slot_se;
    int new_pos;
    int accumulate;
    int do_compress;     // run the selection after the attention (semantic units)
    int m, c, base, R;   // row-buffer state the selection works on (c counts a fused new token)
    int lpr;
    int zcap;            // floats of LDS per wave for the logits of a semantic unit
    int wave_lds;        // bytes of LDS per wave (logits + selection scratch)
    int sem_first;       // semantic units have more rows than spatial ones: dispatch them first
    int seq_off;         // first sequence of this launch (a launch may cover a part of the batch only)
    int late_new_store;  // fused append: store the new token's rows after the stream instead of at its start
    int n_att, nc;       // budgets per head: tokens the attention sees, tokens held at the last compression,
    int row_buffer;      //   and whether spatial heads use the row buffer (a spatial unit derives its own rows)
    int rope_layout;     // rotary embedding of q and k_new on the way in: 0 none, SSD_ROPE_HALF, SSD_ROPE_INTERLEAVED
    const float *rope_cos;   // [d/2] cosines and sines of the new token's position
    const float *rope_sin;
    Segs sp, se;         // rows streamed from the cache (fused append: without the new token's slot)
    Geom g;
};

// Budgets per head (one-layer launches only): the layer's heads ranked by the rows they stream, longest
// first, and each one's budget, by rank.  Workgroups are dispatched in rank order, so the units that take
// longest start first and the short ones fill in behind them.
struct HeadOrder {
    uint8_t head[HMAX];      // head index of rank i
    uint16_t budget[HMAX];   // its W_h (spatial head) or M_h (semantic head)
};

// Workgroups per block of ranks.  Measured on the 7B shape with budgets of 32..96 rows: dispatching strictly by
// rank (1) and by sequence first (all 8 workgroups of a sequence together) differ by 7 %; 1, 2 and 4 are within 1 %.
static constexpr int RANK_GROUPS = 2;

struct StepArgs {
    StepHot h;
    LaunchMeta lm;
    HeadOrder ho;
};

// A wave reads its arguments with scalar loads from the kernel-argument segment.  Left to itself the
// compiler fetches each field where it is first used, which here gave seven dependent groups of loads, each
// a round trip through the scalar cache -- and to memory for the first waves of every CU, which in a launch
// that is one resident round means for everybody -- before the first K/V row was requested.  So the kernel
// reads the segment itself: four 64-byte loads for the fixed part and four smaller ones for its entry of
// the per-layer table (whose address depends on the block index only), all issued back to back and waited
// for once.  The empty asm names all eight results, so none of the loads can sink to a later use.
typedef uint32_t u32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
#define SSD_KERNARG __attribute__((address_space(4)))

static __device__ __forceinline__ void fetch_args(int lrel, StepHot &a, LayerDesc &ld) {
    static_assert(sizeof(StepHot) <= 256, "the fixed part is read as four 64-byte pieces");
    static_assert(sizeof(LayerDesc) == 56, "one table entry is read as three 16-byte pieces and one of 8 bytes");
    static_assert(sizeof(StepArgs) >= 256 && sizeof(StepArgs) == sizeof(StepHot) + sizeof(LaunchMeta) + sizeof(HeadOrder), "layout of the argument block");
    const SSD_KERNARG char *kp = (const SSD_KERNARG char *)__builtin_amdgcn_kernarg_segment_ptr();
    struct { u32x16_t w[4]; } fixed;
    struct { u32x4_t w[3]; u32x2_t t; } entry;
#pragma unroll
    for (int i = 0; i < 4; ++i) fixed.w[i] = *reinterpret_cast<const SSD_KERNARG u32x16_t *>(kp + 64 * i);
    const SSD_KERNARG char *ep = kp + sizeof(StepHot) + (size_t)lrel * sizeof(LayerDesc);
#pragma unroll
    for (int i = 0; i < 3; ++i) entry.w[i] = *reinterpret_cast<const SSD_KERNARG u32x4_t *>(ep + 16 * i);
    entry.t = *reinterpret_cast<const SSD_KERNARG u32x2_t *>(ep + 48);
    asm volatile("" : "+s"(fixed.w[0]), "+s"(fixed.w[1]), "+s"(fixed.w[2]), "+s"(fixed.w[3]), "+s"(entry.w[0]), "+s"(entry.w[1]),
                      "+s"(entry.w[2]), "+s"(entry.t));
    // field by field out of the loaded words (constant indices only, so everything stays in registers)
#define SSD_W(off) (fixed.w[(off) / 64][((off) % 64) / 4])
#define SSD_I(f) a.f = (int32_t)SSD_W(offsetof(StepHot, f))
#define SSD_U(f) a.f = SSD_W(offsetof(StepHot, f))
    // (through a global-address-space pointer: rebuilt from bare integers a pointer would be generic, and every
    // access through it a flat instruction, which counts against both memory counters)
#define SSD_P(f, T_) a.f = (T_)(__attribute__((address_space(1))) char *)((uint64_t)SSD_W(offsetof(StepHot, f)) | ((uint64_t)SSD_W(offsetof(StepHot, f) + 4) << 32))
    SSD_P(q, const char *); SSD_P(out, char *); SSD_P(k_new, const char *); SSD_P(v_new, const char *);
    a.qscale = __uint_as_float(SSD_W(offsetof(StepHot, qscale)));
    SSD_I(layer_off); SSD_I(new_slot_sp); SSD_I(new_slot_se); SSD_I(new_pos); SSD_I(accumulate); SSD_I(do_compress);
    SSD_I(m); SSD_I(c); SSD_I(base); SSD_I(R); SSD_I(lpr); SSD_I(zcap); SSD_I(wave_lds); SSD_I(sem_first); SSD_I(seq_off);
    SSD_I(late_new_store); SSD_I(n_att); SSD_I(nc); SSD_I(row_buffer); SSD_I(rope_layout);
    SSD_P(rope_cos, const float *); SSD_P(rope_sin, const float *);
    SSD_I(sp.start[0]); SSD_I(sp.start[1]); SSD_I(sp.start[2]); SSD_I(sp.len[0]); SSD_I(sp.len[1]); SSD_I(sp.len[2]); SSD_I(sp.total);
    SSD_I(se.start[0]); SSD_I(se.start[1]); SSD_I(se.start[2]); SSD_I(se.len[0]); SSD_I(se.len[1]); SSD_I(se.len[2]); SSD_I(se.total);
    SSD_P(g.base, char *); SSD_I(g.B); SSD_I(g.H); SSD_I(g.S); SSD_I(g.W); SSD_I(g.M); SSD_I(g.C); SSD_I(g.RW); SSD_I(g.row_bytes);
    SSD_U(g.unit_sp_bytes); SSD_U(g.unit_se_bytes);
#undef SSD_W
#define SSD_W(off) ((off) < 48 ? entry.w[((off) % 48) / 16][((off) % 16) / 4] : entry.t[((off) % 16) / 4])
#define SSD_Q(f) ld.f = (uint64_t)SSD_W(offsetof(LayerDesc, f)) | ((uint64_t)SSD_W(offsetof(LayerDesc, f) + 4) << 32)
    SSD_Q(off_sp); SSD_Q(off_se); SSD_Q(off_score); SSD_Q(off_pos); SSD_Q(sem_mask[0]); SSD_Q(sem_mask[1]);
    ld.n_sp = (int32_t)SSD_W(offsetof(LayerDesc, n_sp));
    ld.n_se = (int32_t)SSD_W(offsetof(LayerDesc, n_se));
#undef SSD_W
#undef SSD_I
#undef SSD_U
#undef SSD_P
#undef SSD_Q
}

// Entry `rank` of the launch's HeadOrder (two independent scalar loads from the kernel-argument segment).
static __device__ __forceinline__ void fetch_head_order(int rank, int &head, int &budget) {
    const SSD_KERNARG char *kp = (const SSD_KERNARG char *)__builtin_amdgcn_kernarg_segment_ptr() + sizeof(StepHot) + sizeof(LaunchMeta);
    const uint32_t wh = *reinterpret_cast<const SSD_KERNARG uint32_t *>(kp + offsetof(HeadOrder, head) + (size_t)(rank >> 2) * 4);
    const uint32_t wb = *reinterpret_cast<const SSD_KERNARG uint32_t *>(kp + offsetof(HeadOrder, budget) + (size_t)(rank >> 1) * 4);
    head = (int)((wh >> ((rank & 3) * 8)) & 0xffu);
    budget = (int)((wb >> ((rank & 1) * 16)) & 0xffffu);
}
#undef SSD_KERNARG

// Rotary position embedding (Su et al., RoFormer) of this lane's 16-byte fragment of a d-element row: pairs of
// elements are rotated by the position's angles, element a of pair i to a*cos_i - b*sin_i and element b to
// b*cos_i + a*sin_i.  SSD_ROPE_HALF pairs element i with i + d/2 (the "rotate half" form of the LLaMA family;
// the partner element sits in the lane LPR/2 away), SSD_ROPE_INTERLEAVED pairs 2i with 2i+1 (both in this
// fragment).  fp32, as one product and one fused multiply-add per element, rounded to T once.
template <typename T, int D>
static __device__ __forceinline__ uint4 rope_fragment(const uint4 &raw, const float *cs, const float *sn, int layout, int sub) {
    constexpr int VEC = Elem<T>::VEC;
    constexpr int LPR = D / VEC;
    float x[VEC], r[VEC];
    Elem<T>::unpack(raw, x);
    if (layout == SSD_ROPE_HALF) {
        uint4 praw;
        praw.x = __shfl_xor(raw.x, LPR / 2); praw.y = __shfl_xor(raw.y, LPR / 2);
        praw.z = __shfl_xor(raw.z, LPR / 2); praw.w = __shfl_xor(raw.w, LPR / 2);
        float y[VEC];
        Elem<T>::unpack(praw, y);
        const int i0 = (sub * VEC) % (D / 2);
        const bool first = sub < LPR / 2;              // this fragment holds the a elements of its pairs
#pragma unroll
        for (int e4 = 0; e4 < VEC; e4 += 4) {
            const float4 c = *reinterpret_cast<const float4 *>(cs + i0 + e4);
            const float4 s = *reinterpret_cast<const float4 *>(sn + i0 + e4);
            const float cc[4] = {c.x, c.y, c.z, c.w}, ss[4] = {s.x, s.y, s.z, s.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float t = y[e4 + e] * ss[e];
                r[e4 + e] = fmaf(x[e4 + e], cc[e], first ? -t : t);
            }
        }
    } else {
        const int i0 = sub * (VEC / 2);
#pragma unroll
        for (int j2 = 0; j2 < VEC / 2; j2 += 2) {
            const float2 c = *reinterpret_cast<const float2 *>(cs + i0 + j2);
            const float2 s = *reinterpret_cast<const float2 *>(sn + i0 + j2);
            const float cc[2] = {c.x, c.y}, ss[2] = {s.x, s.y};
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float xa = x[2 * (j2 + j)], xb = x[2 * (j2 + j) + 1];
                const float ta = xb * ss[j], tb = xa * ss[j];
                r[2 * (j2 + j)] = fmaf(xa, cc[j], -ta);
                r[2 * (j2 + j) + 1] = fmaf(xb, cc[j], tb);
            }
        }
    }
    return Elem<T>::pack(r);
}

// One wave per unit, WPB units (consecutive heads of one sequence and layer) per workgroup;
// grid = (ceil(H / WPB), B, layers of the launch).  Nothing below needs a workgroup barrier.
// HEADS: budgets per head.  The launch covers one layer; a unit takes its head's W_h or M_h from the table
// in the arguments and derives its own rows and slots from it (the host's are those of the largest head).
// ROPE: q and the new token's k are rotated by the position's angles on the way in (the rotated k is what the
// cache receives), so that no separate launch has to touch them between the projections and this kernel.
// SHARE > 1 (with WPB = 1): SHARE waves share one unit, taking every SHARE-th wave-load of its rows, and meet
// once in LDS; wave 0 carries on alone.  For launches of few units, which would leave most of the chip's wave
// slots empty.  The partial sums of the waves are combined in another order than one wave adds them: outputs
// and scores of the two forms agree to rounding, not to the bit.
template <typename T, int D, int CH, int WPB, bool FUSED, bool HEADS = false, bool ROPE = false, int SHARE = 1>
__global__ __launch_bounds__(WPB * SHARE * 64) void step_kernel(StepArgs) {      // read through fetch_args
    constexpr int VEC = Elem<T>::VEC;
    constexpr int LPR = D / VEC;
    extern __shared__ __align__(16) unsigned char lds_raw[];
    StepHot a;
    LayerDesc ld;
    fetch_args(HEADS ? 0 : blockIdx.z >> 1, a, ld);

    int t_m = a.m;
    const int t_c = a.c, t_base = a.base, t_R = a.R, t_lpr = a.lpr, t_new_pos = a.new_pos,
              t_new_slot_se = a.new_slot_se, t_do_compress = a.do_compress, t_accumulate = a.accumulate,
              t_M = a.g.M, t_C = a.g.C, t_row_bytes = a.g.row_bytes;
    static_assert(SHARE == 1 || WPB == 1, "a shared unit has its workgroup to itself");
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: everything per-unit stays uniform
    const int w = SHARE > 1 ? 0 : wave;                   // unit of this workgroup the wave works on
    const int part = SHARE > 1 ? wave : 0;                // its share of that unit's rows
    const int lane = threadIdx.x & 63;
    const int sub = lane % LPR;
    // grid = (ceil(max heads of a type / WPB), B, 2 * layers): z selects the layer and the head type, the type
    // with more rows first, so that within a layer the long units are dispatched before the short ones and
    // all waves of a workgroup have units of one length
    const int lrel = HEADS ? 0 : blockIdx.z >> 1;
    bool sem_unit;
    int local, h, seq, hb = 0;
    if constexpr (HEADS) {
        // grid = (RANK_GROUPS, B, ceil(H / (WPB * RANK_GROUPS))): z walks the heads in rank order (longest first,
        // whatever their type), RANK_GROUPS workgroups' worth at a time; inside such a block of ranks the
        // sequences are the slow index, as in the uniform launch
        const int rank = (blockIdx.z * RANK_GROUPS + blockIdx.x) * WPB + w;
        if (rank >= a.g.H) return;
        fetch_head_order(rank, h, hb);
        seq = a.seq_off + blockIdx.y;
        const uint64_t word = h < 64 ? ld.sem_mask[0] : ld.sem_mask[1];
        const uint64_t below = (1ull << (h & 63)) - 1ull;
        sem_unit = ((word >> (h & 63)) & 1ull) != 0;
        const int sem_below = h < 64 ? __popcll(ld.sem_mask[0] & below) : __popcll(ld.sem_mask[0]) + __popcll(ld.sem_mask[1] & below);
        local = sem_unit ? sem_below : h - sem_below;
    } else {
        sem_unit = ((blockIdx.z & 1) == 0) == (a.sem_first != 0);
        local = blockIdx.x * WPB + w;                     // index among the heads of this type in this layer
        if (local >= (sem_unit ? ld.n_se : ld.n_sp)) return;
        const uint64_t m0 = sem_unit ? ld.sem_mask[0] : ~ld.sem_mask[0];
        const uint64_t m1 = sem_unit ? ld.sem_mask[1] : ~ld.sem_mask[1];
        h = kth_set_bit(m0, m1, local);                   // spatial heads: bits above H are never reached (local < n_sp)
        seq = a.seq_off + blockIdx.y;
    }
    const int rem = seq * a.g.H + h;
    const UnitRef u = unit_ref_local(a.g, ld, seq, sem_unit, local);
    // field by field, constant indices: a choice between two structs, or an index the compiler has not
    // unrolled yet, would pin the argument copy in (scratch) memory
    Segs sg;
    sg.start[0] = u.sem ? a.se.start[0] : a.sp.start[0];
    sg.start[1] = u.sem ? a.se.start[1] : a.sp.start[1];
    sg.start[2] = u.sem ? a.se.start[2] : a.sp.start[2];
    sg.len[0] = u.sem ? a.se.len[0] : a.sp.len[0];
    sg.len[1] = u.sem ? a.se.len[1] : a.sp.len[1];
    sg.len[2] = u.sem ? a.se.len[2] : a.sp.len[2];
    sg.total = u.sem ? a.se.total : a.sp.total;
    int t_Mh = t_M;                                       // the head's own budget (t_M stays the start of the row buffer)
    if constexpr (HEADS) {
        if (u.sem) {
            t_Mh = hb;
            t_m = t_m < hb ? t_m : hb;                    // heavy slots this head has in use
            sg.total -= sg.len[0] - t_m;
            sg.len[0] = t_m;
        } else {
            const int RW = hb + (a.g.RW - a.g.W);
            a.new_slot_sp = ring_slot(a.g.S, RW, a.new_pos);
            sg = FUSED ? ring_segs_fused(a.g.S, hb, a.g.C, a.row_buffer != 0, a.n_att - 1, a.nc, a.new_slot_sp)
                       : ring_segs(a.g.S, hb, a.g.C, a.row_buffer != 0, a.n_att, a.nc);
        }
    }
    const size_t qoff = ((size_t)(a.layer_off + lrel) * (size_t)(a.g.B * a.g.H) + rem) * (size_t)a.g.row_bytes + (size_t)sub * 16u;
    unsigned char *region = lds_raw + (size_t)w * a.wave_lds;
    float *zbuf = reinterpret_cast<float *>(region);                    // [zcap]
    unsigned char *sel = region + (size_t)a.zcap * 4;                   // selection scratch

    const uint4 raw_q = *reinterpret_cast<const uint4 *>(a.q + qoff);
    typename Elem<T>::Q q = Elem<T>::load_q(raw_q);       // ROPE: replaced by the rotated query behind the first loads
    Softmax<VEC> sm;
    sm.init();
    const bool want_z = u.sem && t_accumulate;

    // No memory round trip may be left exposed after the last row, so everything the tail of this wave
    // needs is requested around the start of the K/V stream.  The new token's fragments (fused append) are
    // fetched by every lane group alike (the same 16 lines, no extra traffic): only group 0 uses them, but a
    // load under a per-lane condition costs a branch and a wait.
    const bool compress = t_do_compress != 0;
    const bool tail = u.sem && (t_accumulate || compress || FUSED);
    uint4 new_k = make_uint4(0, 0, 0, 0), new_v = make_uint4(0, 0, 0, 0);
    if (FUSED) {
        new_k = *reinterpret_cast<const uint4 *>(a.k_new + qoff);
        new_v = *reinterpret_cast<const uint4 *>(a.v_new + qoff);
    }
    float pre_score[2] = {0.f, 0.f};
    int pre_pos[2] = {0, 0};

    // Runs once, right after the stream's first loads have been issued, so that nothing here delays them: the
    // running scores and positions of the first 128 rows (one or two per lane) are requested now and have
    // long arrived when the tail needs them.  The loads are unconditional (rows past the end are clamped to a
    // valid slot and ignored later): a load under a per-lane condition makes the compiler wait for it on the
    // spot.
    auto store_new = [&]() {
        if (FUSED && lane < LPR && part == 0) {
            const int slot = u.sem ? a.new_slot_se : a.new_slot_sp;
            const size_t off = (size_t)slot * (size_t)a.g.row_bytes + (size_t)sub * 16u;
            *reinterpret_cast<uint4 *>(u.K + off) = new_k;
            *reinterpret_cast<uint4 *>(u.V + off) = new_v;
        }
    };
    auto after_first_issue = [&]() {
        if constexpr (ROPE) {
            // here, not before the stream: the rotation waits for q, k_new and the angles, and the first K/V
            // rows are better requested before that wait than after it
            q = Elem<T>::load_q(rope_fragment<T, D>(raw_q, a.rope_cos, a.rope_sin, a.rope_layout, sub));
            new_k = rope_fragment<T, D>(new_k, a.rope_cos, a.rope_sin, a.rope_layout, sub);
        }
        if (!a.late_new_store) store_new();
        if (tail && part == 0) {
            const int last = sg.total > 0 ? sg.total - 1 : 0;    // no rows yet: slot of row 0, inside the unit
#pragma unroll
            for (int k = 0; k < 2; ++k) {
                const int r = lane + 64 * k;
                const int slot = seg_slot(sg, r < last ? r : last);
                pre_score[k] = u.score[slot];
                pre_pos[k] = u.pos[slot];
            }
        }
    };
    if (want_z)
        stream_rows<T, D, CH, true, false>(u.K, u.V, a.g.row_bytes, sg, 0, sg.total, part, SHARE, q, a.qscale, sm, zbuf, 0, 0, after_first_issue);
    else
        stream_rows<T, D, CH, false, false>(u.K, u.V, a.g.row_bytes, sg, 0, sg.total, part, SHARE, q, a.qscale, sm, nullptr, 0, 0, after_first_issue);
    if (FUSED && part == 0) {
        // The new token, from the registers it was loaded into, is folded into lane group 0's softmax as
        // one more row (index sg.total).
        const float z = group_sum<LPR>(Elem<T>::dot(q, new_k)) * a.qscale;
        if (lane < LPR) {
            const float m_new = fmaxf(sm.m, z);
            const float alpha = fast_exp2(sm.m - m_new);
            const float p = fast_exp2(z - m_new);
            float vf[VEC];
            Elem<T>::unpack(new_v, vf);
            sm.l = sm.l * alpha + p;
#pragma unroll
            for (int e = 0; e < VEC; ++e) sm.acc[e] = fmaf(p, vf[e], sm.acc[e] * alpha);
            sm.m = m_new;
            if (want_z && lane == 0) zbuf[sg.total] = z;
        }
    }
    merge_groups<VEC, LPR, false>(sm);
    if constexpr (SHARE > 1) {
        // the waves of the unit leave their partial (max, sum, output) in LDS; wave 0 combines them and goes on alone
        float *mg = reinterpret_cast<float *>(lds_raw + a.wave_lds);       // [SHARE][2 + D]
        float *mine = mg + part * (2 + D);
        if (lane == 0) { mine[0] = sm.m; mine[1] = sm.l; }
        if (lane < LPR) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) mine[2 + sub * VEC + e] = sm.acc[e];
        }
        __syncthreads();                                  // also publishes every wave's logits in zbuf
        if (part != 0) return;
        float m_u = NEG_BIG;
#pragma unroll
        for (int p = 0; p < SHARE; ++p) m_u = fmaxf(m_u, mg[p * (2 + D)]);
        float l_u = 0.f, acc_u[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc_u[e] = 0.f;
#pragma unroll
        for (int p = 0; p < SHARE; ++p) {
            const float f = fast_exp2(mg[p * (2 + D)] - m_u);
            l_u = fmaf(mg[p * (2 + D) + 1], f, l_u);
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc_u[e] = fmaf(mg[p * (2 + D) + 2 + sub * VEC + e], f, acc_u[e]);
        }
        sm.m = m_u; sm.l = l_u;
#pragma unroll
        for (int e = 0; e < VEC; ++e) sm.acc[e] = acc_u[e];
    }
    const float m_all = sm.m;
    const float inv_l = sm.l > 0.f ? 1.0f / sm.l : 0.f;
    if (lane < LPR) {
        float o[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = sm.acc[e] * inv_l;
        *reinterpret_cast<uint4 *>(a.out + qoff) = Elem<T>::pack(o);
    }
    // Fused append, the new token's rows.  Stores and loads share one in-order counter per wave, and a store is
    // acknowledged much later than a load returns: issued at the start of the stream, these two stores keep
    // the counter up and the stream's "all but the newest chunk" waits wait for more loads than they mean to.
    // In a launch of one resident round that costs 1.1 us, so there the rows are stored here, after the
    // stream; where other waves or another stream's kernel fill such gaps anyway, storing them early is
    // better (the stores drain during the stream and the wave ends sooner).  The host chooses.
    if (a.late_new_store) store_new();

    if (!tail) return;
    lds_sync();                                           // the logits written by the group leaders
    const int M = t_M, C = t_C;
    const int n_old = t_c - t_R;                          // buffered tokens that become candidates
    const int n_cand = t_m + n_old;
    const int n_evict = n_cand - t_Mh;                    // <= 0: everything is kept
    // At most one eviction among at most 128 candidates (always the case when compressing after every
    // token) is settled in registers; anything else ranks all candidates through LDS.
    const bool general = compress && (n_evict >= 2 || n_cand > 128);
    unsigned long long *keys = reinterpret_cast<unsigned long long *>(sel);
    unsigned long long my_key[2] = {~0ull, ~0ull};        // keys of rows lane and lane + 64, if candidates
    const int total = sg.total + (FUSED ? 1 : 0);
    // One row's share: add the probability to its running score, note position and key.
    auto score_row = [&](int r, float s_old, int pos_old) -> unsigned long long {
        const bool is_new = FUSED && r == sg.total;
        const int slot = is_new ? t_new_slot_se : seg_slot(sg, r);
        const float p = t_accumulate ? fast_exp2(zbuf[r] - m_all) * inv_l : 0.f;
        const float s = (is_new ? 0.f : s_old) + p;
        if (t_accumulate || is_new) u.score[slot] = s;
        if (is_new) u.pos[slot] = t_new_pos;
        unsigned long long key = ~0ull;
        if (compress && r < n_cand) {
            key = make_key(s, is_new ? t_new_pos : pos_old);
            if (general) keys[r] = key;
        }
        return key;
    };
    // rows 0..127 use the scores and positions fetched before the stream: no load, and therefore no wait
    // on this wave's own stores, in the common case
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        const int r = lane + 64 * k;
        if (r < total) my_key[k] = score_row(r, pre_score[k], pre_pos[k]);
    }
    // Rows from 128 on (long budgets and row buffers only), four per lane at a time: the four loads of a batch are
    // issued together and the stores follow them.  One row at a time, every load had to wait for the store before it
    // (the compiler cannot tell the slots apart), a memory round trip per 64 rows at the end of the unit's longest wave.
    for (int r0 = lane + 128; r0 - lane < total; r0 += 4 * 64) {
        float s_old[4];
        int p_old[4];
        const int last = total - 1;
#pragma unroll
        for (int j = 0; j < 4; ++j) {                     // unconditional loads: rows past the end read the last row's slot
            const int r = r0 + 64 * j < last ? r0 + 64 * j : last;
            const int slot = (FUSED && r == sg.total) ? t_new_slot_se : seg_slot(sg, r);
            s_old[j] = u.score[slot];
            p_old[j] = u.pos[slot];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = r0 + 64 * j;
            if (r < total) score_row(r, s_old[j], p_old[j]);
        }
    }
    if (!compress) return;
    if (general) {
        lds_sync();
        select_and_move<64, true>(a.g, u, sel, n_cand, t_m, n_old, t_base, t_lpr, lane, t_Mh);
        return;
    }
    // The promoted buffered tokens and the slots they go to follow from the index of the single evicted
    // candidate (the one with the smallest key), if any.
    int e_idx = -1;
    if (n_evict == 1) {
        const unsigned long long min_key = wave_min_u64(my_key[0] < my_key[1] ? my_key[0] : my_key[1]);
        const unsigned long long hit0 = __ballot(my_key[0] == min_key);
        const unsigned long long hit1 = __ballot(my_key[1] == min_key);
        e_idx = hit0 ? __builtin_ctzll(hit0) : 64 + __builtin_ctzll(hit1);
    }
    const bool ev_heavy = e_idx >= 0 && e_idx < t_m;
    const bool ev_staged = e_idx >= t_m;
    const int n_move = n_old - (ev_staged ? 1 : 0);
    if (n_move <= 0) return;
    const int frag_per_tok = 2 * t_lpr;
    // k-th promoted candidate (oldest first) and k-th free heavy slot
    auto src_idx = [&](int k) { return t_m + k + ((ev_staged && k >= e_idx - t_m) ? 1 : 0); };
    auto dst_slot = [&](int k) { return ev_heavy ? (k == 0 ? e_idx : t_m + k - 1) : t_m + k; };
    wave_global_sync();                                   // rows stored earlier by other lanes of this wave
    for (int t = lane; t < n_move * frag_per_tok; t += 64) {
        const int k = t / frag_per_tok;
        const int f = t % frag_per_tok;
        const int kv = f / t_lpr, fs = f % t_lpr;
        char *plane = kv ? u.V : u.K;
        const int from = M + (t_base + (src_idx(k) - t_m)) % C;
        const uint4 v = *reinterpret_cast<const uint4 *>(plane + (size_t)from * t_row_bytes + (size_t)fs * 16u);
        *reinterpret_cast<uint4 *>(plane + (size_t)dst_slot(k) * t_row_bytes + (size_t)fs * 16u) = v;
    }
    // position and score travel with the token: its key sits in the registers of lane (index mod 64)
    for (int k0 = 0; k0 < n_move; k0 += 64) {             // wave-uniform trip count: the shuffles need every lane
        const int k = k0 + lane;
        const int src = k < n_move ? src_idx(k) : 0;
        const unsigned long long c0 = __shfl(my_key[0], src & 63);
        const unsigned long long c1 = __shfl(my_key[1], src & 63);
        const unsigned long long key = src < 64 ? c0 : c1;
        if (k < n_move) {
            u.pos[dst_slot(k)] = key_pos(key);
            u.score[dst_slot(k)] = key_score(key);
        }
    }
}

// Largest candidate count the fused entry point ranks with a single wave; beyond it the stand-alone
// compression kernel (a whole workgroup per head) runs after the attention.
static constexpr int FUSED_SELECT_MAX = 1024;

// Rank the heads of layer l by the rows this launch streams from their units, longest first (ties: lower head index).
static void fill_head_order(const ssd_cache *c, int l, const LayerState &before, const LayerState &at, bool fused, HeadOrder *out) {
    const ssd_config &cf = c->cfg;
    const int H = cf.n_heads;
    int rows[HMAX], idx[HMAX];
    for (int h = 0; h < H; ++h) {
        const int v = c->head_budget[(size_t)l * H + h];
        idx[h] = h;
        if (c->head_type[(size_t)l * H + h] == SSD_SEMANTIC) {
            rows[h] = (at.m < v ? at.m : v) + at.c;
        } else {
            const bool rb = cf.spatial_row_buffer != 0;
            rows[h] = fused ? ring_segs_fused(cf.n_init_sink, v, cf.stage_cap, rb, before.n, before.nc, -1).total
                            : ring_segs(cf.n_init_sink, v, cf.stage_cap, rb, at.n, at.nc).total;
        }
    }
    std::stable_sort(idx, idx + H, [&](int x, int y) { return rows[x] > rows[y]; });
    for (int i = 0; i < HMAX; ++i) {
        out->head[i] = (uint8_t)(i < H ? idx[i] : 0);
        out->budget[i] = i < H ? c->head_budget[(size_t)l * H + idx[i]] : 0;
    }
}

template <typename T, int D, int CH, int SHARE>
static void launch_shared(const StepArgs &full, dim3 blocks, size_t lds, bool fused, bool heads, hipStream_t s) {
    const bool rope = full.h.rope_layout != 0;
    if (heads || rope) {                                  // four wave-loads per chunk only; the rotary step is always fused (the host sees to both)
        if constexpr (CH == 4) {
            if (rope && heads) hipLaunchKernelGGL((step_kernel<T, D, CH, 1, true, true, true, SHARE>), blocks, dim3(SHARE * 64), lds, s, full);
            else if (rope) hipLaunchKernelGGL((step_kernel<T, D, CH, 1, true, false, true, SHARE>), blocks, dim3(SHARE * 64), lds, s, full);
            else if (fused) hipLaunchKernelGGL((step_kernel<T, D, CH, 1, true, true, false, SHARE>), blocks, dim3(SHARE * 64), lds, s, full);
            else hipLaunchKernelGGL((step_kernel<T, D, CH, 1, false, true, false, SHARE>), blocks, dim3(SHARE * 64), lds, s, full);
        }
        return;
    }
    if (fused) hipLaunchKernelGGL((step_kernel<T, D, CH, 1, true, false, false, SHARE>), blocks, dim3(SHARE * 64), lds, s, full);
    else hipLaunchKernelGGL((step_kernel<T, D, CH, 1, false, false, false, SHARE>), blocks, dim3(SHARE * 64), lds, s, full);
}

template <typename T, int D, int CH, int WPB>
static void launch_one(const StepArgs &full, dim3 blocks, size_t lds, bool fused, bool heads, hipStream_t s) {
    const bool rope = full.h.rope_layout != 0;            // fused launches only (checked by the entry point)
    if (heads || rope) {
        // budgets per head, rotary embedding: one variant (four wave-loads per chunk) per workgroup size
        if constexpr (CH == 4) {
            if (rope && heads) hipLaunchKernelGGL((step_kernel<T, D, CH, WPB, true, true, true>), blocks, dim3(WPB * 64), lds, s, full);
            else if (rope) hipLaunchKernelGGL((step_kernel<T, D, CH, WPB, true, false, true>), blocks, dim3(WPB * 64), lds, s, full);
            else if (fused) hipLaunchKernelGGL((step_kernel<T, D, CH, WPB, true, true>), blocks, dim3(WPB * 64), lds, s, full);
            else hipLaunchKernelGGL((step_kernel<T, D, CH, WPB, false, true>), blocks, dim3(WPB * 64), lds, s, full);
        }
        return;
    }
    if (fused) hipLaunchKernelGGL((step_kernel<T, D, CH, WPB, true>), blocks, dim3(WPB * 64), lds, s, full);
    else hipLaunchKernelGGL((step_kernel<T, D, CH, WPB, false>), blocks, dim3(WPB * 64), lds, s, full);
}

// One launch over sequences [a.seq_off, a.seq_off + B) of the layers in `full`.  concurrent: the launch is one part of
// a split call, so another part's launch runs beside it on another stream.
template <typename T, int D>
static hipError_t launch_step(StepArgs &full, const LaunchShape &shape, LaunchShape *used, int H, int max_sp_heads, int max_se_heads, int B,
                              int layers, bool fused, bool heads, bool concurrent, int M, hipStream_t s) {
    StepHot &a = full.h;
    const int max_type_heads = max_sp_heads > max_se_heads ? max_sp_heads : max_se_heads;
    const int n_old = a.c - a.R, n_cand = a.m + n_old;
    // Launch shape by the number of units (measured on the 7B- and 1B-shaped workloads at 16 to 256 prompts).
    // Up to half of what the chip holds at once (256 CUs x 16 waves) the launch is latency-bound: the waves
    // are spread over as many CUs as possible (one unit per workgroup).  Four wave-loads of K and of V per
    // chunk (two chunks in flight) are best at every size.  Between half a round and four rounds the new
    // token's rows are stored after the stream (see the kernel).
    const long long units = (long long)H * B * layers;
    a.late_new_store = shape.new_rows == 1 ? 0 : shape.new_rows == 2 ? 1 : (units > 2048 && units <= 16384 ? 1 : 0);
    int ch = shape.ch && !heads && !a.rope_layout ? shape.ch : 4;
    int wpb = shape.wpb ? shape.wpb : (units <= 2048 ? 1 : 4);
    // Several waves per unit (codes 12 and 14: two and four) where one wave per unit leaves wave slots empty:
    //  * few and long units (the high-resolution shape, 2048 units of 129 to 385 rows): four, 41.0 -> 38.1 us;
    //  * parts of a split call, two launches in flight: two waves for parts of 1025 to 2048 units (7B shape,
    //    128 sequences on two streams: 0.705 -> 0.687 ms per step), four for parts of 513 to 1024 units (64
    //    sequences: 0.415 -> 0.385 ms).  Alone on the chip such launches are faster with one wave per unit
    //    (64 sequences on one stream: 0.443 ms against 0.452 and 0.466), and smaller parts gain nothing.
    const int longest = a.se.total > a.sp.total ? a.se.total : a.sp.total;
    if (!shape.wpb && units <= 2048) {
        if (longest >= 96 && !heads) wpb = 14;            // (budgets per head: `longest` is the largest head's, most units are shorter)
        else if (concurrent && units > 1024) wpb = 12;
        else if (concurrent && units > 512) wpb = 14;
    }
    //  * a few long units beside many short ones -- the head mix the paper's threshold gives (Sec. 3.3, Table 6: a
    //    handful of semantic heads with a large budget, most heads spatial with a short window): with one wave per
    //    unit the launch lasts as long as its longest units while the waves of the short ones are long gone.  Where
    //    one head type streams at least twice the rows of the other and has at most a quarter of the heads, every
    //    unit gets two waves -- four if the long type is the semantic one with at least 96 rows and the launch is
    //    small (up to 2048 units, or up to 4096 with at least 192 rows).  7B shape, 30 spatial heads with W = 32
    //    beside 2 semantic ones, one stream, ms per step: M = 64 0.678 -> 0.482, M = 128 0.856 -> 0.588, M = 320
    //    1.523 -> 0.742; 512 sequences, M = 128: 2.999 -> 1.792.  (On two streams the parts of those shapes had two
    //    waves per unit already; four bring 0.555 -> 0.514 at M = 128 and 0.781 -> 0.706 at M = 320.)
    const bool long_sem = a.sem_first != 0;
    const int rows_long = long_sem ? a.se.total : a.sp.total, rows_short = long_sem ? a.sp.total : a.se.total;
    const int heads_long = long_sem ? max_se_heads : max_sp_heads;
    if (!shape.wpb && !heads && max_sp_heads > 0 && max_se_heads > 0 && rows_short > 0 && rows_long >= 2 * rows_short &&
        4 * heads_long <= H)
        wpb = long_sem && rows_long >= 96 && (units <= 2048 || (units <= 4096 && rows_long >= 192)) ? 14 : 12;
    if (wpb > 10 && ch == 1) ch = 2;                      // the shared-unit launch exists with two and four loads per chunk
    a.wave_lds = (int)(((size_t)a.zcap * 4 + (a.do_compress ? select_lds_bytes(M, n_cand, n_old) + 16 : 0) + 15) / 16 * 16);
    while (wpb > 1 && wpb < 10 && (size_t)wpb * a.wave_lds > 60000) wpb >>= 1;
    const size_t lds = (size_t)wpb * a.wave_lds;
    *used = LaunchShape{ch, wpb, a.late_new_store ? 2 : 1};
    const dim3 blocks = heads ? dim3((unsigned)RANK_GROUPS, (unsigned)B, (unsigned)(((H + wpb - 1) / wpb + RANK_GROUPS - 1) / RANK_GROUPS))   // rank order, see the kernel
                              : dim3((unsigned)((max_type_heads + wpb - 1) / wpb), (unsigned)B, (unsigned)(2 * layers));
    // wpb codes 12 and 14: one unit per workgroup, shared by 2 or 4 waves
#define SSD_SHARED(CH_, SHARE_) if (ch == CH_ && wpb == 10 + SHARE_) { launch_shared<T, D, CH_, SHARE_>(full, heads ? dim3((unsigned)RANK_GROUPS, (unsigned)B, (unsigned)((H + RANK_GROUPS - 1) / RANK_GROUPS)) : dim3((unsigned)max_type_heads, (unsigned)B, (unsigned)(2 * layers)), (size_t)a.wave_lds + SHARE_ * (2 + D) * sizeof(float), fused, heads, s); return hipGetLastError(); }
    SSD_SHARED(2, 2) SSD_SHARED(4, 2) SSD_SHARED(2, 4) SSD_SHARED(4, 4)
#undef SSD_SHARED
#define SSD_CASE(CH_, WPB_) if (ch == CH_ && wpb == WPB_) { launch_one<T, D, CH_, WPB_>(full, blocks, lds, fused, heads, s); return hipGetLastError(); }
    if constexpr (sizeof(T) == 2 && D == 128) {       // the shape the sweeps are run on has every variant
        SSD_CASE(1, 1) SSD_CASE(2, 1) SSD_CASE(4, 1)
        SSD_CASE(1, 2) SSD_CASE(2, 2) SSD_CASE(4, 2)
        SSD_CASE(1, 4) SSD_CASE(2, 4) SSD_CASE(4, 4)
    } else {
        if (ch == 1) ch = 2;
        SSD_CASE(2, 1) SSD_CASE(4, 1) SSD_CASE(2, 2) SSD_CASE(4, 2) SSD_CASE(2, 4) SSD_CASE(4, 4)
    }
#undef SSD_CASE
    return hipErrorInvalidValue;
}

struct Rope {
    const float *cos, *sin;
    int layout;
};

// How a split call cuts the batch: consecutive parts of `seqs` sequences (an even number: the two sequences of a
// prompt under classifier-free guidance stay together; the last part takes what is left), part i going to stream
// i mod n_streams.  At least one part per stream; more when a part's launch would exceed about one resident
// round of waves (4096 units over the layers of the call): launches of that size keep their dirty lines in L2
// until they end and write them back in one burst, larger ones spill them into the read stream all along
// (large batch, 512 sequences on two streams: 2.996 ms per step with 2 parts, 2.804 with 4, 2.796 with 8).  Small
// launches pay their fixed cost instead (7B shape, 128 sequences: 0.720 / 0.860 / 1.188 ms with 2 / 4 / 8 parts),
// so never more than four parts per stream.
struct SplitPlan {
    int seqs;      // sequences per part
    int parts;
};
static constexpr int SPLIT_UNITS_PER_LAUNCH = 4096;
static SplitPlan split_plan(int B, int H, int layers, int n_streams) {
    auto even = [](int x) { return (x + 1) / 2 * 2; };
    int seqs = even((B + n_streams - 1) / n_streams);                      // one part per stream
    const long long per_seq = (long long)H * layers;
    int fit = (int)(SPLIT_UNITS_PER_LAUNCH / per_seq) / 2 * 2;             // sequences whose units fill one resident round
    if (fit < 2) fit = 2;
    if (n_streams > 1 && fit < seqs) seqs = fit;
    const int floor_seqs = even((B + 4 * n_streams - 1) / (4 * n_streams));  // at most four parts per stream
    if (seqs < floor_seqs) seqs = floor_seqs;
    SplitPlan p;
    p.seqs = seqs;
    p.parts = (B + seqs - 1) / seqs;
    return p;
}

// Shared by ssd_decode_attn (k_new == NULL, compress == 0), ssd_decode_step, ssd_decode_step_rope and
// ssd_decode_step_split.  streams[0..n_streams): part i of the batch is enqueued on streams[i mod n_streams].
static int run_step(ssd_cache *cache, int layer_begin, int layer_end, const void *q, const void *k_new, const void *v_new,
                    void *out, int accumulate, int compress, void *const *streams, int n_streams, const char *what,
                    Rope rope = {nullptr, nullptr, 0}) {
    const ssd_config &cf = cache->cfg;
    const bool fused = k_new != nullptr;
    // one plan per call, from the layers the call covers (its launches may cover fewer: runs of layers in one state)
    const int span = layer_end - layer_begin;
    const SplitPlan plan = split_plan(cf.n_seqs, cf.n_heads, span < LMAX ? span : LMAX, n_streams);
    const int Bp = plan.seqs;
    for (int lb = layer_begin; lb < layer_end;) {
        const int le = same_state_run(cache, lb, layer_end);
        const LayerState before = cache->st[lb];
        const bool has_se = cache->ldesc[lb].n_se > 0;     // uniform over the run, like the row-buffer flag
        const bool has_buf = has_buffer(cache, lb);
        LayerState at = before;                      // state the attention sees
        if (fused) { at.n += 1; if (has_buf) at.c += 1; }
        const int n_old = at.c - cf.recent;
        const bool do_compress = compress && has_se && n_old > 0;
        const bool in_kernel = do_compress && at.m + n_old <= FUSED_SELECT_MAX;
        if (cache->launch_enabled) {
            StepArgs full;
            StepHot &a = full.h;
            a.g = make_geom(cache, lb);
            fill_launch_meta(cache, lb, le, &full.lm);
            a.q = static_cast<const char *>(q);
            a.out = static_cast<char *>(out);
            a.k_new = static_cast<const char *>(k_new);
            a.v_new = static_cast<const char *>(v_new);
            a.layer_off = lb - layer_begin;
            a.new_pos = before.n;
            a.new_slot_sp = spatial_slot(cache, lb, before.n);
            a.new_slot_se = cache->Ml[lb] + (before.base + before.c) % cf.stage_cap;
            if (fused) {
                a.sp = spatial_segs_fused(cache, lb, before, at, a.new_slot_sp);
                a.se = semantic_segs(cache, lb, before);
            } else {
                a.sp = spatial_segs(cache, lb, at);
                a.se = semantic_segs(cache, lb, at);
            }
            a.qscale = cache->scale * LOG2E;
            a.accumulate = accumulate ? 1 : 0;
            a.zcap = ((a.se.total + 1 + 63) / 64) * 64;
            a.do_compress = in_kernel ? 1 : 0;
            a.m = at.m; a.c = at.c; a.base = at.base; a.R = cf.recent;
            a.lpr = a.g.row_bytes / 16;
            a.n_att = at.n; a.nc = before.nc; a.row_buffer = cf.spatial_row_buffer;
            a.rope_layout = rope.layout; a.rope_cos = rope.cos; a.rope_sin = rope.sin;
            if (heads_differ(cache, lb)) fill_head_order(cache, lb, before, at, fused, &full.ho);
            else full.ho = HeadOrder{};                  // never read then; keeps the argument bytes defined
            int mx_sp = 0, mx_se = 0;                       // most heads of a type in a layer of the launch
            for (int l = lb; l < le; ++l) {
                mx_sp = cache->ldesc[l].n_sp > mx_sp ? cache->ldesc[l].n_sp : mx_sp;
                mx_se = cache->ldesc[l].n_se > mx_se ? cache->ldesc[l].n_se : mx_se;
            }
            a.sem_first = a.se.total + (fused ? 1 : 0) >= a.sp.total + (fused ? 1 : 0) ? 1 : 0;
            for (int part = 0; part < plan.parts; ++part) {
                hipStream_t s = static_cast<hipStream_t>(streams[part % n_streams]);
                a.seq_off = part * Bp;
                const int Bn = cf.n_seqs - a.seq_off < Bp ? cf.n_seqs - a.seq_off : Bp;
                const bool hd = heads_differ(cache, lb);
                hipError_t e;
                if (cf.dtype == SSD_BF16)
                    e = cf.head_dim == 128 ? launch_step<bf16_t, 128>(full, cache->shape, &cache->last_shape, cf.n_heads, mx_sp, mx_se, Bn, le - lb, fused, hd, plan.parts > 1 && n_streams > 1, cache->Ml[lb], s)
                                           : launch_step<bf16_t, 64>(full, cache->shape, &cache->last_shape, cf.n_heads, mx_sp, mx_se, Bn, le - lb, fused, hd, plan.parts > 1 && n_streams > 1, cache->Ml[lb], s);
                else
                    e = cf.head_dim == 128 ? launch_step<float, 128>(full, cache->shape, &cache->last_shape, cf.n_heads, mx_sp, mx_se, Bn, le - lb, fused, hd, plan.parts > 1 && n_streams > 1, cache->Ml[lb], s)
                                           : launch_step<float, 64>(full, cache->shape, &cache->last_shape, cf.n_heads, mx_sp, mx_se, Bn, le - lb, fused, hd, plan.parts > 1 && n_streams > 1, cache->Ml[lb], s);
                if (e != hipSuccess) return hip_fail(e, what);
                if (do_compress && !in_kernel) {
                    const int rc = launch_compress_inplace(cache, lb, le, at, a.seq_off, Bn, s);
                    if (rc != SSD_OK) return rc;
                }
            }
        }
        for (int l = lb; l < le; ++l) {
            LayerState &x = cache->st[l];
            if (fused) { x.n += 1; if (has_buf) x.c += 1; }
            if (compress) apply_compress_counters(cache, l);
        }
        lb = le;
    }
    return SSD_OK;
}

// Argument and overflow checks common to the fused entry points.
static int check_step_args(ssd_cache *cache, int layer_begin, int layer_end, const void *q, const void *k_new, const void *v_new,
                           const void *out) {
    int rc = check_layers(cache, layer_begin, layer_end);
    if (rc != SSD_OK) return rc;
    if (!q || !out || !k_new || !v_new) return fail(SSD_ERR_INVALID_ARG, "q, k_new, v_new or out is NULL");
    if (!aligned(q, 16) || !aligned(out, 16) || !aligned(k_new, 16) || !aligned(v_new, 16))
        return fail(SSD_ERR_INVALID_ARG, "q / k_new / v_new / out must be 16-byte aligned");
    for (int l = layer_begin; l < layer_end; ++l)
        if (has_buffer(cache, l) && cache->st[l].c >= cache->cfg.stage_cap)
            return fail(SSD_ERR_STAGE_OVERFLOW, "row buffer overflow: layer %d already buffers %d tokens (C=%d); call ssd_compress_kv",
                        l, cache->st[l].c, cache->cfg.stage_cap);
    return SSD_OK;
}

}  // namespace ssd

using namespace ssd;

extern "C" int ssd_cache_set_launch_shape(ssd_cache *cache, int ch, int wpb, int new_rows) {
    clear_error();
    if (!cache) return fail(SSD_ERR_INVALID_ARG, "cache is NULL");
    if ((ch != 0 && ch != 1 && ch != 2 && ch != 4) || (wpb != 0 && wpb != 1 && wpb != 2 && wpb != 4 && wpb != 12 && wpb != 14) ||
        new_rows < 0 || new_rows > 2)
        return fail(SSD_ERR_INVALID_ARG, "launch shape (%d, %d, %d) is not one the library has", ch, wpb, new_rows);
    cache->shape = LaunchShape{ch, wpb, new_rows};
    return SSD_OK;
}

extern "C" int ssd_cache_last_launch_shape(const ssd_cache *cache, int32_t out3[3]) {
    clear_error();
    if (!cache || !out3) return fail(SSD_ERR_INVALID_ARG, "cache or out3 is NULL");
    out3[0] = cache->last_shape.ch; out3[1] = cache->last_shape.wpb; out3[2] = cache->last_shape.new_rows;
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
    return run_step(cache, layer_begin, layer_end, q, nullptr, nullptr, out, accumulate_scores, 0, &stream, 1, "attention launch");
}

extern "C" int ssd_decode_step(ssd_cache *cache, int layer_begin, int layer_end, const void *q, const void *k_new,
                               const void *v_new, void *out, int accumulate_scores, int compress, void *stream) {
    clear_error();
    const int rc = check_step_args(cache, layer_begin, layer_end, q, k_new, v_new, out);
    if (rc != SSD_OK) return rc;
    return run_step(cache, layer_begin, layer_end, q, k_new, v_new, out, accumulate_scores, compress, &stream, 1, "decode step launch");
}

// Common body of the split entry points: stream list and sync checks, fork, the launches, join.
static int run_split(ssd_cache *cache, int layer_begin, int layer_end, const void *q, const void *k_new, const void *v_new, void *out,
                     int accumulate_scores, int compress, void *const *streams, int n_streams, int sync, const char *what, Rope rope) {
    if (!streams || n_streams < 1 || n_streams > SSD_MAX_SPLIT)
        return fail(SSD_ERR_INVALID_ARG, "streams is NULL or n_streams=%d outside 1..%d", n_streams, SSD_MAX_SPLIT);
    if (sync & ~(SSD_SPLIT_FORK | SSD_SPLIT_JOIN)) return fail(SSD_ERR_INVALID_ARG, "sync=%d has unknown bits", sync);
    for (int i = 0; i < n_streams; ++i)
        for (int j = 0; j < i; ++j)
            if (streams[i] == streams[j]) return fail(SSD_ERR_INVALID_ARG, "streams[%d] and streams[%d] are the same stream", j, i);
    const bool live = cache->launch_enabled && n_streams > 1;
    if (live && sync) {
        const int rc = ensure_events(cache);
        if (rc != SSD_OK) return rc;
    }
    if (live && (sync & SSD_SPLIT_FORK)) {
        // the other streams take up the work where streams[0] stands now
        hipError_t e = hipEventRecord(cache->ev_fork, static_cast<hipStream_t>(streams[0]));
        for (int i = 1; i < n_streams && e == hipSuccess; ++i) e = hipStreamWaitEvent(static_cast<hipStream_t>(streams[i]), cache->ev_fork, 0);
        if (e != hipSuccess) return hip_fail(e, "fork of the split step");
    }
    const int rc = run_step(cache, layer_begin, layer_end, q, k_new, v_new, out, accumulate_scores, compress, streams, n_streams, what, rope);
    if (rc != SSD_OK) return rc;
    if (live && (sync & SSD_SPLIT_JOIN)) {
        // streams[0] goes on only when every part is done
        for (int i = 1; i < n_streams; ++i) {
            hipError_t e = hipEventRecord(cache->ev_join[i], static_cast<hipStream_t>(streams[i]));
            if (e == hipSuccess) e = hipStreamWaitEvent(static_cast<hipStream_t>(streams[0]), cache->ev_join[i], 0);
            if (e != hipSuccess) return hip_fail(e, "join of the split step");
        }
    }
    return SSD_OK;
}

static int check_rope_args(const float *cos_p, const float *sin_p, int rope_layout) {
    if (rope_layout != SSD_ROPE_HALF && rope_layout != SSD_ROPE_INTERLEAVED)
        return fail(SSD_ERR_INVALID_ARG, "rope_layout=%d is neither SSD_ROPE_HALF nor SSD_ROPE_INTERLEAVED", rope_layout);
    if (!cos_p || !sin_p || !aligned(cos_p, 16) || !aligned(sin_p, 16))
        return fail(SSD_ERR_INVALID_ARG, "cos / sin must be given and 16-byte aligned");
    return SSD_OK;
}

extern "C" int ssd_decode_step_split(ssd_cache *cache, int layer_begin, int layer_end, const void *q, const void *k_new,
                                     const void *v_new, void *out, int accumulate_scores, int compress,
                                     void *const *streams, int n_streams, int sync) {
    clear_error();
    const int rc = check_step_args(cache, layer_begin, layer_end, q, k_new, v_new, out);
    if (rc != SSD_OK) return rc;
    return run_split(cache, layer_begin, layer_end, q, k_new, v_new, out, accumulate_scores, compress, streams, n_streams, sync,
                     "split decode step launch", Rope{nullptr, nullptr, 0});
}

extern "C" int ssd_decode_step_split_rope(ssd_cache *cache, int layer_begin, int layer_end, const void *q, const void *k_new,
                                          const void *v_new, void *out, int accumulate_scores, int compress, const float *cos_p,
                                          const float *sin_p, int rope_layout, void *const *streams, int n_streams, int sync) {
    clear_error();
    int rc = check_step_args(cache, layer_begin, layer_end, q, k_new, v_new, out);
    if (rc != SSD_OK) return rc;
    rc = check_rope_args(cos_p, sin_p, rope_layout);
    if (rc != SSD_OK) return rc;
    return run_split(cache, layer_begin, layer_end, q, k_new, v_new, out, accumulate_scores, compress, streams, n_streams, sync,
                     "split decode step launch (rotary)", Rope{cos_p, sin_p, rope_layout});
}

extern "C" int ssd_decode_step_split_plan(const ssd_cache *cache, int layers_per_call, int n_streams, int32_t *part_seqs,
                                          int32_t *n_parts) {
    clear_error();
    if (!cache) return fail(SSD_ERR_INVALID_ARG, "cache is NULL");
    if (layers_per_call < 1 || layers_per_call > cache->cfg.n_layers)
        return fail(SSD_ERR_INVALID_ARG, "layers_per_call=%d outside 1..%d", layers_per_call, cache->cfg.n_layers);
    if (n_streams < 1 || n_streams > SSD_MAX_SPLIT) return fail(SSD_ERR_INVALID_ARG, "n_streams=%d outside 1..%d", n_streams, SSD_MAX_SPLIT);
    const SplitPlan p = split_plan(cache->cfg.n_seqs, cache->cfg.n_heads, layers_per_call < LMAX ? layers_per_call : LMAX, n_streams);
    if (part_seqs) *part_seqs = p.seqs;
    if (n_parts) *n_parts = p.parts;
    return SSD_OK;
}

extern "C" int ssd_decode_step_rope(ssd_cache *cache, int layer_begin, int layer_end, const void *q, const void *k_new,
                                    const void *v_new, void *out, int accumulate_scores, int compress, const float *cos_p,
                                    const float *sin_p, int rope_layout, void *stream) {
    clear_error();
    int rc = check_step_args(cache, layer_begin, layer_end, q, k_new, v_new, out);
    if (rc != SSD_OK) return rc;
    rc = check_rope_args(cos_p, sin_p, rope_layout);
    if (rc != SSD_OK) return rc;
    return run_step(cache, layer_begin, layer_end, q, k_new, v_new, out, accumulate_scores, compress, &stream, 1,
                    "decode step launch (rotary)", Rope{cos_p, sin_p, rope_layout});
}
