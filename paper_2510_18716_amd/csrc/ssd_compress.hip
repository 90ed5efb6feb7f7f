// ssd_compress_kv: top-M selection by accumulated score and the gather into the compact cache
// (Algorithm 1 "IndicesOfTopM" / "SelectAndAppend"; Algorithm 2 "Compress semantic cache
// (heavy-hitter) ... Reset row buffer" and its prefill branch).  The selection itself is in
// ssd_select.h; this file holds the stand-alone in-place kernel and the dense-source kernel.
#include "ssd_select.h"

namespace ssd {

struct CompressArgs {
    Geom g;
    LaunchMeta lm;
    int m;             // heavy slots in use
    int c;             // buffered tokens
    int base;          // ring index of the oldest buffered token
    int R;
    int lpr;           // 16-byte fragments per row
    int heads;         // budgets per head
    int seq_off;       // the launch covers sequences [seq_off, seq_off + n_seq)
    int n_seq;
    HeadTable ht;
};

// One workgroup per (layer, sequence, head); spatial heads return at once.
template <int THREADS>
__global__ __launch_bounds__(THREADS) void compress_inplace_kernel(CompressArgs a) {
    extern __shared__ __align__(16) unsigned char lds[];
    const int BH = a.n_seq * a.g.H;
    const int unit = blockIdx.x;
    const int lrel = unit / BH;
    const int rem = unit % BH;
    const UnitRef u = unit_ref(a.g, a.lm.layer[lrel], a.seq_off + rem / a.g.H, rem % a.g.H);
    if (!u.sem) return;                       // uniform for the whole workgroup
    const int Mh = a.heads ? a.ht.v[rem % a.g.H] : a.g.M;     // this head's budget
    const int m = a.m < Mh ? a.m : Mh;        // heavy slots this head has in use
    const int n_old = a.c - a.R;              // buffered tokens that become candidates (> 0, checked on the host)
    const int n_cand = m + n_old;
    unsigned long long *keys = reinterpret_cast<unsigned long long *>(lds);
    for (int i = threadIdx.x; i < n_cand; i += THREADS) {
        const int slot = i < m ? i : a.g.M + (a.base + (i - m)) % a.g.C;
        keys[i] = make_key(u.score[slot], u.pos[slot]);
    }
    __syncthreads();
    select_and_move<THREADS, false>(a.g, u, lds, n_cand, m, n_old, a.base, a.lpr, threadIdx.x, Mh);
}

// ---- dense-source mode -------------------------------------------------------

struct DenseSrcArgs {
    Geom g;
    LaunchMeta lm;
    const char *K_src;      // [L', B, H, n_src, d]
    const char *V_src;
    const float *score_src; // [L', B, H, n_src] or NULL
    int layer_off;
    int n_src;
    int R;
    int lpr;
    int heads;              // budgets per head
    HeadTable ht;
};

template <int THREADS>
__global__ __launch_bounds__(THREADS) void compress_dense_kernel(DenseSrcArgs a) {
    extern __shared__ unsigned long long smem_u64[];
    const int BH = a.g.B * a.g.H;
    const int unit = blockIdx.x;
    const int lrel = unit / BH;
    const int rem = unit % BH;
    const UnitRef u = unit_ref(a.g, a.lm.layer[lrel], rem / a.g.H, rem % a.g.H);
    const size_t src_unit = (size_t)(a.layer_off + lrel) * BH + rem;
    const char *Ks = a.K_src + src_unit * (size_t)a.n_src * a.g.row_bytes;
    const char *Vs = a.V_src + src_unit * (size_t)a.n_src * a.g.row_bytes;
    const int tid = threadIdx.x;
    const int frag_per_tok = 2 * a.lpr;

    if (!u.sem) {
        // positions {0..S-1} and the last W: destination slot as in ssd_append_token
        const int S = a.g.S, W = a.heads ? a.ht.v[rem % a.g.H] : a.g.W, RW = W + (a.g.RW - a.g.W);
        const int n_sink = a.n_src < S ? a.n_src : S;
        const int w_begin = a.n_src - W > S ? a.n_src - W : S;
        const int n_win = a.n_src > w_begin ? a.n_src - w_begin : 0;
        const int n_rows = n_sink + n_win;
        for (int t = tid; t < n_rows * frag_per_tok; t += THREADS) {
            const int k = t / frag_per_tok;
            const int f = t % frag_per_tok;
            const int kv = f / a.lpr, sub = f % a.lpr;
            const int p = k < n_sink ? k : w_begin + (k - n_sink);
            const int slot = p < S ? p : S + (p - S) % RW;
            const uint4 v = *reinterpret_cast<const uint4 *>((kv ? Vs : Ks) + (size_t)p * a.g.row_bytes + (size_t)sub * 16u);
            *reinterpret_cast<uint4 *>((kv ? u.V : u.K) + (size_t)slot * a.g.row_bytes + (size_t)sub * 16u) = v;
        }
        return;
    }

    const int M = a.heads ? a.ht.v[rem % a.g.H] : a.g.M;  // this head's budget; the row buffer starts at slot g.M
    const int n_rec = a.n_src < a.R ? a.n_src : a.R;      // newest tokens that go to the row buffer
    const int n_cand = a.n_src - n_rec;
    const float *sc = a.score_src ? a.score_src + src_unit * (size_t)a.n_src : nullptr;
    unsigned long long *keys = smem_u64;                               // [n_cand]
    int *kept = reinterpret_cast<int *>(keys + (n_cand > 0 ? n_cand : 0));   // [M] kept positions, ascending
    unsigned char *flag = reinterpret_cast<unsigned char *>(kept + M);       // [n_cand]
    __shared__ int s_nkeep;

    for (int i = tid; i < n_cand; i += THREADS) keys[i] = make_key(sc ? sc[i] : 0.f, i);
    __syncthreads();
    for (int i = tid; i < n_cand; i += THREADS) {
        bool keep = true;
        if (n_cand > M) {
            const unsigned long long mine = keys[i];
            int rank = 0;
            for (int j = 0; j < n_cand; ++j) rank += keys[j] > mine ? 1 : 0;
            keep = rank < M;
        }
        flag[i] = keep ? 1 : 0;
    }
    __syncthreads();
    if (tid < 64) {
        int nkeep = 0;
        for (int i0 = 0; i0 < n_cand; i0 += 64) {
            const int i = i0 + tid;
            const bool f = i < n_cand && flag[i] != 0;
            int tot;
            const int pre = wave_prefix(f, tot);
            if (f) kept[nkeep + pre] = i;
            nkeep += tot;
        }
        if (tid == 0) s_nkeep = nkeep;
    }
    __syncthreads();
    const int nkeep = s_nkeep;                // = min(M, n_cand)
    // heavy slots 0..nkeep-1 in ascending position; row buffer (ring index 0..) gets the newest n_rec
    const int n_rows = nkeep + n_rec;
    for (int t = tid; t < n_rows * frag_per_tok; t += THREADS) {
        const int k = t / frag_per_tok;
        const int f = t % frag_per_tok;
        const int kv = f / a.lpr, sub = f % a.lpr;
        const int p = k < nkeep ? kept[k] : n_cand + (k - nkeep);
        const int slot = k < nkeep ? k : a.g.M + (k - nkeep);
        const uint4 v = *reinterpret_cast<const uint4 *>((kv ? Vs : Ks) + (size_t)p * a.g.row_bytes + (size_t)sub * 16u);
        *reinterpret_cast<uint4 *>((kv ? u.V : u.K) + (size_t)slot * a.g.row_bytes + (size_t)sub * 16u) = v;
    }
    for (int k = tid; k < n_rows; k += THREADS) {
        const int p = k < nkeep ? kept[k] : n_cand + (k - nkeep);
        const int slot = k < nkeep ? k : a.g.M + (k - nkeep);
        u.pos[slot] = p;
        u.score[slot] = sc ? sc[p] : 0.f;
    }
}

// In-place compression of sequences [seq_off, seq_off + n_seq) of layers [lb, le), which all hold the state `st`
// (st.c - R > 0).
int launch_compress_inplace(const ssd_cache *cache, int lb, int le, const LayerState &st, int seq_off, int n_seq, hipStream_t s) {
    const ssd_config &cf = cache->cfg;
    const int n_old = st.c - cf.recent;
    CompressArgs a;
    a.g = make_geom(cache, lb);
    fill_launch_meta(cache, lb, le, &a.lm);
    a.m = st.m;
    a.c = st.c;
    a.base = st.base;
    a.R = cf.recent;
    a.lpr = cf.head_dim * cache->esize / 16;
    a.heads = heads_differ(cache, lb) ? 1 : 0;
    a.seq_off = seq_off;
    a.n_seq = n_seq;
    fill_head_table(cache, lb, &a.ht);
    const int n_cand = st.m + n_old;
    const unsigned units = (unsigned)((le - lb) * n_seq * cf.n_heads);
    const size_t lds = select_lds_bytes(cache->Ml[lb], n_cand, n_old);
    if (n_cand <= 192)
        hipLaunchKernelGGL((compress_inplace_kernel<64>), dim3(units), dim3(64), lds, s, a);
    else
        hipLaunchKernelGGL((compress_inplace_kernel<256>), dim3(units), dim3(256), lds, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return hip_fail(e, "compression launch");
    return SSD_OK;
}

}  // namespace ssd

using namespace ssd;

extern "C" int ssd_compress_kv(ssd_cache *cache, int layer_begin, int layer_end, const void *K_src,
                               const void *V_src, const float *score_src, int n_src, void *stream) {
    clear_error();
    int rc = check_layers(cache, layer_begin, layer_end);
    if (rc != SSD_OK) return rc;
    const ssd_config &cf = cache->cfg;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int BH = cf.n_seqs * cf.n_heads;
    const int lpr = cf.head_dim * cache->esize / 16;

    if (K_src || V_src) {
        if (!K_src || !V_src) return fail(SSD_ERR_INVALID_ARG, "K_src and V_src must both be given");
        if (n_src < 1 || n_src > 4096) return fail(SSD_ERR_INVALID_ARG, "n_src=%d outside 1..4096", n_src);
        if (!aligned(K_src, 16) || !aligned(V_src, 16) || !aligned(score_src, 4))
            return fail(SSD_ERR_INVALID_ARG, "K_src / V_src must be 16-byte aligned, score_src 4-byte aligned");
        const int n_rec = n_src < cf.recent ? n_src : cf.recent;
        const int n_cand = n_src - n_rec;
        if (cache->launch_enabled) {
            for (int lb = layer_begin, le; lb < layer_end; lb = le) {
                le = same_geom_run(cache, lb, layer_end);
                DenseSrcArgs a;
                a.g = make_geom(cache, lb);
                fill_launch_meta(cache, lb, le, &a.lm);
                a.K_src = static_cast<const char *>(K_src);
                a.V_src = static_cast<const char *>(V_src);
                a.score_src = score_src;
                a.layer_off = lb - layer_begin;
                a.n_src = n_src;
                a.R = cf.recent;
                a.lpr = lpr;
                a.heads = heads_differ(cache, lb) ? 1 : 0;
                fill_head_table(cache, lb, &a.ht);
                const size_t lds = sizeof(unsigned long long) * (size_t)n_cand + sizeof(int) * (size_t)cache->Ml[lb] + (size_t)n_cand + 16;
                hipLaunchKernelGGL((compress_dense_kernel<256>), dim3((unsigned)((le - lb) * BH)), dim3(256), lds, s, a);
                hipError_t e = hipGetLastError();
                if (e != hipSuccess) return hip_fail(e, "dense-source compression launch");
            }
        }
        for (int l = layer_begin; l < layer_end; ++l) {
            LayerState &st = cache->st[l];
            st.n = n_src;
            st.m = cache->ldesc[l].n_se > 0 ? (n_cand < cache->Ml[l] ? n_cand : cache->Ml[l]) : 0;
            st.c = has_buffer(cache, l) ? n_rec : 0;
            st.base = 0;
            st.nc = n_src;
        }
        return SSD_OK;
    }

    if (score_src) return fail(SSD_ERR_INVALID_ARG, "score_src without K_src / V_src");
    for (int lb = layer_begin; lb < layer_end;) {
        const int le = same_state_run(cache, lb, layer_end);
        const LayerState st = cache->st[lb];
        const int n_old = st.c - cf.recent;
        // kernels run only where semantic heads have candidates; the counters (and the spatial window of
        // Algorithm 2) move in every layer of the range
        if (n_old > 0 && cache->ldesc[lb].n_se > 0 && cache->launch_enabled) {
            rc = launch_compress_inplace(cache, lb, le, st, 0, cf.n_seqs, s);
            if (rc != SSD_OK) return rc;
        }
        for (int l = lb; l < le; ++l) apply_compress_counters(cache, l);
        lb = le;
    }
    return SSD_OK;
}
