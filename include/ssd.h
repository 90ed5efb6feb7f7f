/*
 * ssd.h -- C ABI of the MI355X (gfx950) library for the decode-time hot path
 * of SSD, spatial-semantic head-decoupled KV-cache compression
 * (arxiv 2510.18716).
 *
 * What the library does: batched single-token decode attention over a
 * per-head heterogeneous compressed KV cache.  Each attention head of each
 * layer is either a spatial-locality head, which keeps S initial "sink"
 * tokens and a ring of the W most recent tokens, or a semantic-sink head,
 * which keeps up to M heavy-hitter tokens chosen by accumulated attention
 * probability plus a row buffer of up to C recently appended tokens of which
 * the newest R are never evicted (Sec. 3.3, Algorithm 1; row buffer:
 * Appendix B, Algorithm 2).
 *
 * Conventions that hold for every entry point
 *   - "dev" pointers are device (HBM) addresses owned by the caller; "host"
 *     pointers are ordinary host memory.  The library allocates no device
 *     memory and frees none; it keeps nothing on the device besides the
 *     caller's cache memory (layout tables travel as kernel arguments).  Tensors are dense, row-major, innermost
 *     dimension last, 16-byte aligned.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls only enqueue work on it and never wait for the device.
 *   - Return value: 0 (SSD_OK) or a negative ssd_status.  Argument, range,
 *     ordering and overflow errors are found from host-side counters before
 *     anything is enqueued and leave the cache unchanged.  The text of the
 *     last error of the calling thread is available from ssd_last_error().
 *   - All sequences of a cache advance together (same prompt length, same
 *     number of generated tokens; Sec. 3.1: every image has the same N), so
 *     token counts are kept per layer on the host, not per sequence.
 *   - Sequences b = 2i and b = 2i+1 are the conditional / unconditional pair
 *     of prompt i under classifier-free guidance (Sec. 3.1, Eq. 1).  The
 *     library treats them as independent sequences.
 *   - Token positions are absolute, 0-based, prompt tokens first and visual
 *     tokens after them in raster order (Sec. 3.1).
 *
 * Call order per generated token and layer:
 *     ssd_append_token -> ssd_decode_attn -> (ssd_compress_kv when due)
 * or the same three fused into one launch: ssd_decode_step -- or, with the
 * batch dealt to several streams so that the launches overlap,
 * ssd_decode_step_split.
 * Compressing after every token is Algorithm 1; compressing every 24 tokens
 * (one grid row) is Algorithm 2.  The row buffer holds C tokens, so at most
 * C - R tokens can be appended between two compressions.
 */
#ifndef SSD_H
#define SSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ssd_dtype { SSD_F32 = 0, SSD_BF16 = 1 } ssd_dtype;

/* Head types of Eq. (3). */
typedef enum ssd_head_type { SSD_SPATIAL = 0, SSD_SEMANTIC = 1 } ssd_head_type;

typedef enum ssd_status {
    SSD_OK = 0,
    SSD_ERR_INVALID_ARG = -1,    /* null / misaligned pointer, bad config value, bad size       */
    SSD_ERR_LAYER_RANGE = -2,    /* [layer_begin, layer_end) not inside [0, n_layers)           */
    SSD_ERR_STAGE_OVERFLOW = -3, /* append with a full row buffer ("Row buffer overflow", Alg. 2) */
    SSD_ERR_ORDER = -4,          /* attention or export on a layer that holds no token yet      */
    SSD_ERR_HIP = -5             /* the HIP runtime refused a copy or a launch                  */
} ssd_status;

/*
 * Shape and policy parameters (Algorithm 1 "Parameter" line; Sec. 3.3).
 * One config describes one cache: all layers share S, R, C, and also W and M
 * unless ssd_cache_init_layered gives those per layer or ssd_cache_init_heads
 * per head.
 */
typedef struct ssd_config {
    int32_t n_layers;      /* L                                                            */
    int32_t n_seqs;        /* B = 2 x prompts                                              */
    int32_t n_heads;       /* H <= 128, one query row per KV head (plain multi-head attention) */
    int32_t head_dim;      /* d: 64 or 128                                                 */
    int32_t dtype;         /* ssd_dtype of q, k, v, the cache rows and the output          */
    int32_t window;        /* W >= 1: ring slots of a spatial head, counts the new token   */
    int32_t n_init_sink;   /* S >= 0: first S positions a spatial head always keeps        */
    int32_t budget;        /* M >= 1: heavy-hitter slots of a semantic head                */
    int32_t recent;        /* R >= 0: newest tokens a semantic head never evicts           */
    int32_t stage_cap;     /* C > R: row-buffer slots of a semantic head; M + C <= 4096    */
    float   softmax_scale; /* 0 selects 1/sqrt(d)                                          */
    int32_t spatial_row_buffer; /* 0: a spatial head keeps exactly its S sinks and the W newest tokens
                                   (Algorithm 1).  1: Algorithm 2 -- it attends to the sinks, the W
                                   newest tokens as of the last compression, and every token appended
                                   since (the row buffer), so its window grows from W to W + C - R between
                                   compressions; ssd_compress_kv re-cuts the window.  Requires S+W+C <= 65536 */
    int32_t reserved[4];   /* must be 0                                                    */
} ssd_config;

/* Host-side descriptor of a cache: layout, per-layer head lists, token counters. */
typedef struct ssd_cache ssd_cache;

/*
 * Bytes of device memory a cache needs for `cfg` and the head-type table
 * `head_type` (host, [L*H], values of ssd_head_type; the table Algorithm 1
 * takes as given).  Returns 0 if the config or the table is invalid.
 */
size_t ssd_cache_bytes(const ssd_config *cfg, const uint8_t *head_type);

/*
 * Create the descriptor of a cache that lives in dev_mem[0..bytes).
 * dev_mem: device, 256-byte aligned, at least ssd_cache_bytes() long, owned
 * by the caller and must outlive the descriptor; its contents need not be
 * initialised.  Touches no device memory.  The cache starts empty.
 */
int ssd_cache_init(const ssd_config *cfg, const uint8_t *head_type, void *dev_mem,
                   size_t bytes, ssd_cache **out);

/*
 * The same two calls with a window and a budget per layer (layer-wise budget
 * allocation: Sec. 3.3 finds the share of long-range attention to fall from
 * the lower to the upper layers, and Sec. 5 "Integration with Other
 * Compression Techniques" names layer-wise allocation as a combination).
 *   window, budget : host int32 [L], or NULL for cfg->window / cfg->budget in
 *                    every layer; each entry obeys the limits of the config
 *                    field it replaces.  The arrays are copied.
 * Layers of different W or M have units of different size and go to separate
 * launches; everything else (call order, counters, errors) is unchanged.
 */
size_t ssd_cache_bytes_layered(const ssd_config *cfg, const uint8_t *head_type,
                               const int32_t *window, const int32_t *budget);
int ssd_cache_init_layered(const ssd_config *cfg, const uint8_t *head_type,
                           const int32_t *window, const int32_t *budget, void *dev_mem,
                           size_t bytes, ssd_cache **out);
/* Window and budget of one layer (either output may be NULL); with budgets per head, the layer's largest. */
int ssd_cache_layer_budget(const ssd_cache *cache, int layer, int32_t *window, int32_t *budget);

/*
 * The same two calls with a budget per head (head-wise adaptive allocation,
 * which Sec. 5 "Integration with Other Compression Techniques" names beside
 * the layer-wise one).
 *   head_budget : host int32 [L*H]; entry [l*H + h] is the window W_h of head h
 *                 of layer l if head_type says it is a spatial head (1..65535),
 *                 its heavy-hitter budget M_h if it is a semantic head (>= 1,
 *                 M_h + C <= 4096).  cfg->window / cfg->budget are ignored
 *                 except in a layer that has no head of that type.  Copied.
 * Layout: every unit of a layer keeps one size, that of the layer's largest
 * W_h (spatial) or M_h (semantic); head h uses a ring of W_h slots, or the
 * first M_h heavy slots, of its unit, and the row buffer of every semantic
 * head of the layer starts at slot max_h M_h.  So memory is that of the
 * largest head, while the rows a step reads are each head's own.  A layer
 * whose heads differ takes a launch of its own in every call (a layer whose
 * heads of each type agree is handled like one of ssd_cache_init_layered).
 * Everything else is unchanged; the host
 * counter m of ssd_cache_layer_state is the layer's largest (a head has
 * min(m, M_h) heavy slots in use).
 */
size_t ssd_cache_bytes_heads(const ssd_config *cfg, const uint8_t *head_type, const int32_t *head_budget);
int ssd_cache_init_heads(const ssd_config *cfg, const uint8_t *head_type, const int32_t *head_budget,
                         void *dev_mem, size_t bytes, ssd_cache **out);
/* W_h (spatial head) or M_h (semantic head) of one head, whichever init call made the cache. */
int ssd_cache_head_budget(const ssd_cache *cache, int layer, int head, int32_t *value);

/* Free the descriptor (not dev_mem).  NULL is allowed. */
void ssd_cache_free(ssd_cache *cache);

/* Forget every token: all host counters back to zero.  Enqueues nothing. */
int ssd_cache_reset(ssd_cache *cache);

/*
 * Host counters of one layer: out4 = { n tokens appended, m heavy slots in
 * use, c row-buffer slots in use, ring index of the oldest row-buffer slot }.
 */
int ssd_cache_layer_state(const ssd_cache *cache, int layer, int32_t out4[4]);

/* Token count of the layer at its last compression (the start of a spatial head's row buffer). */
int ssd_cache_layer_window(const ssd_cache *cache, int layer, int32_t *n_at_last_compress);

/*
 * Head classification by attention sparsity (Sec. 3.3, "Spatial Sparsity
 * Analysis", and Eq. 3).
 *   far, tot : dev float [L, P, H, T].  For profiled sequence p and visual
 *              step t (1-based), with a the attention distribution of that
 *              step's query over all rows and visual rows indexed
 *              i = 0..t-1 (i = t-1 is the query's own row):
 *              tot = sum_{i=0}^{t-1} a(i), far = sum_{i=0}^{t-1-w} a(i).
 *              ssd_dense_decode_attn produces them.
 *   s_out    : dev float [L, H]  = mean over (p, t) of far/tot (0 where tot = 0)
 *   type_out : dev uint8 [L, H]  = SSD_SEMANTIC if s > tau else SSD_SPATIAL
 */
int ssd_classify_heads(const float *far, const float *tot, int L, int P, int H, int T,
                       float tau, float *s_out, uint8_t *type_out, void *stream);

/*
 * Append one new token to layers [layer_begin, layer_end) (the "Append" of
 * Algorithm 1, the row-buffer append of Algorithm 2).
 *   k_new, v_new : dev [layer_end - layer_begin, B, H, d] of the cache dtype.
 * Spatial head: the row overwrites the oldest ring slot (positions < S go to
 * the sink slots).  Semantic head: the row enters the row buffer with
 * accumulated score 0.  Fails with SSD_ERR_STAGE_OVERFLOW, appending to no
 * layer, if any layer of the range already holds C buffered tokens.
 */
int ssd_append_token(ssd_cache *cache, int layer_begin, int layer_end,
                     const void *k_new, const void *v_new, void *stream);

/*
 * Single-token attention of every (sequence, head) of the layers over its
 * retained rows: out = softmax(scale * q K^T) V (Algorithm 1,
 * "AttentionScores"; the retained rows include the token just appended).
 *   q   : dev [layer_end - layer_begin, B, H, d], cache dtype
 *   out : dev, same shape and dtype
 * accumulate_scores != 0: every semantic head also adds this step's
 * post-softmax probabilities to the running scores of its retained tokens
 * (Algorithm 1, "AggregateAttentionScores", fp32).
 * SSD_ERR_ORDER if a layer of the range holds no token.
 */
int ssd_decode_attn(ssd_cache *cache, int layer_begin, int layer_end,
                    const void *q, void *out, int accumulate_scores, void *stream);

/*
 * Compression (Algorithm 1 "IndicesOfTopM" + "SelectAndAppend"; Algorithm 2
 * "Compress ... Reset row buffer").
 *
 * In-place mode (K_src == NULL): for every semantic head of the layers,
 * candidates = heavy tokens + buffered tokens except the R newest; the M
 * candidates with the highest accumulated score stay (ties: lower position
 * first; all stay if there are at most M), the rest are dropped with their
 * scores; the R newest tokens remain in the row buffer.  Spatial heads need
 * no data movement: under Algorithm 1 their ring evicts by itself, under
 * Algorithm 2 (spatial_row_buffer) the call re-cuts their window to the W
 * newest tokens.  A layer with at most R buffered tokens keeps its semantic
 * heads as they are.
 *
 * Dense-source mode (K_src != NULL): rebuild the layers from a full cache
 * segment (the prefill branch of Algorithm 2).
 *   K_src, V_src : dev [layer_end - layer_begin, B, H, n_src, d], cache dtype
 *   score_src    : dev float [layer_end - layer_begin, B, H, n_src] accumulated
 *                  scores of those tokens, or NULL for all zero.  Every value
 *                  must be finite and >= 0 (sums of probabilities are): the
 *                  selection orders scores by their bit patterns, which is the
 *                  numerical order for such values only; the library does not
 *                  check this
 *   n_src        : 1 .. 4096 tokens
 * Spatial heads take positions {0..S-1} and the last W; semantic heads take
 * the top-M of positions 0..n_src-R-1 and put the R newest into the row
 * buffer.  Afterwards the layers hold n_src tokens.
 */
int ssd_compress_kv(ssd_cache *cache, int layer_begin, int layer_end,
                    const void *K_src, const void *V_src, const float *score_src,
                    int n_src, void *stream);

/*
 * Accumulated attention scores of a prompt processed in one piece (Algorithm 2:
 * scores are accumulated whenever attention weights exist, and a prefill is
 * compressed at once; Sec. 3.3 for what is accumulated).  For every unit
 * u = (layer, sequence, head) and prompt token j
 *     score_out[u, j] = sum over i >= j of softmax_{j' <= i}(scale * q_i . k_j')[j]
 * i.e. the column sums of the causal attention matrix -- the value the decode
 * path would have accumulated had the prompt been fed token by token.  The
 * result is the score_src argument of ssd_compress_kv's dense-source mode.
 *   Q, K      : dev [n_units, n_src, d] of `dtype` (the K_src layout with the
 *               leading three dimensions flattened)
 *   n_units   : >= 1;  n_src : 1 .. 4096 (as ssd_compress_kv);  d : 64 or 128
 *   dtype     : ssd_dtype;  softmax_scale : 0 selects 1/sqrt(d)
 *   score_out : dev float [n_units, n_src], overwritten
 * The products run on the matrix cores with fp32 accumulation; the sum over i
 * is taken in a fixed order (bit-reproducible).
 */
int ssd_prefill_scores(const void *Q, const void *K, int n_units, int n_src, int d,
                       int dtype, float softmax_scale, float *score_out, void *stream);

/*
 * Classifier-free guidance of the two next-token distributions of each prompt
 * (Sec. 3.1, Eq. 1):
 *     out[i, v] = p[2i, v] + gamma * (p[2i, v] - p[2i+1, v])
 * where sequence 2i is the pass conditioned on the prompt and 2i+1 the
 * unconditional one (the pairing of the conventions above).  The paper writes
 * the rule on the distributions; the arithmetic is the same whatever the rows
 * hold (probabilities or logits), and the result is not renormalised.
 *   p      : dev [n_seqs, V] of `dtype`, n_seqs even
 *   out    : dev float [n_seqs / 2, V], 16-byte aligned, overwritten
 *   gamma  : guidance strength (the paper takes gamma > 1; any finite value is accepted)
 */
int ssd_cfg_mix(const void *p, int n_seqs, int V, int dtype, float gamma, float *out, void *stream);

/*
 * One whole decode step of the layers in a single launch per layer group:
 * ssd_append_token, then ssd_decode_attn, then (compress != 0) the in-place
 * mode of ssd_compress_kv, with their results: the same kept sets, outputs
 * and scores equal to the rounding of the fp32 sums (the new token enters the
 * softmax from registers as the last term of its sum, not at its slot).  Each (sequence, head)
 * is handled by one wavefront from append to selection, so the three steps
 * of Algorithm 1 cost one pass over the head's rows.
 *   q, k_new, v_new, out : dev [layer_end - layer_begin, B, H, d], cache dtype
 * Errors as for the three separate calls (overflow is checked first and
 * leaves every layer unchanged).
 */
int ssd_decode_step(ssd_cache *cache, int layer_begin, int layer_end, const void *q,
                    const void *k_new, const void *v_new, void *out,
                    int accumulate_scores, int compress, void *stream);

/*
 * The same step with the batch dealt to several streams, so that the launches
 * of different parts of the batch overlap: while one part's launch ramps up
 * or drains, another part's is streaming.  Sequences are independent of each
 * other (Sec. 3.1: each prompt is decoded on its own; the two sequences of a
 * prompt meet only in Eq. 1, after the last layer), so a caller that runs its
 * model on parts of the batch in turn (micro-batches) keeps every part's
 * layers in order on that part's stream and never has to make the parts meet
 * between layers.  The kernels are those of ssd_decode_step; results are the
 * same up to rounding.  How many wavefronts share a (sequence, head) unit --
 * and with it the order in which the unit's rows enter its softmax sums -- is
 * chosen from the size of a launch, and a part's launch is smaller than the
 * whole batch's (and has another launch running beside it).  Where both calls
 * give a unit the same number of wavefronts the results are equal bit for bit
 * (in ssd_hooks.h, ssd_cache_last_launch_shape reports what a launch took and
 * ssd_cache_set_launch_shape pins it; batches of at most 512 (sequence, head,
 * layer) units per call always qualify); otherwise outputs and scores differ
 * by the rounding of fp32 sums, and the kept sets are the same unless two
 * candidates' scores are that close.
 *   streams   : host array of n_streams distinct hipStream_t, all of the
 *               default priority; n_streams in 1..SSD_MAX_SPLIT
 *   The batch is cut into n_parts consecutive parts of P sequences (P even: a prompt's two sequences stay
 *   together; the last part takes what is left), part i = sequences [i * P, min(B, (i + 1) * P)).  Part i's work
 *   is enqueued on streams[i mod n_streams] only, and the rows of q, k_new, v_new it reads and of out it writes
 *   are ordered with respect to that stream only.  The library picks P: one part per stream, or more (at most
 *   four per stream) when a part would otherwise exceed about 4096 (sequence, head, layer) units per launch --
 *   launches of about one resident round of wavefronts write their dirty lines back in one burst at their end,
 *   larger ones spill them into the read stream.  ssd_decode_step_split_plan returns P and n_parts for a call
 *   that covers layers_per_call layers (they depend on the cache's shape, that number and n_streams only).
 *   sync      : SSD_SPLIT_FORK  -- before anything is enqueued, streams[1..]
 *               are made to wait for what streams[0] holds so far;
 *               SSD_SPLIT_JOIN  -- afterwards streams[0] is made to wait for
 *               what the other streams hold.  A caller with one stream of its
 *               own forks at a token's first layer and joins at its last.
 *               Both use events the cache keeps (made on first use, timing
 *               disabled); nothing waits on the host, nothing is allocated on
 *               the device.
 * The host counters advance once per call (all parts move together), so a
 * cache must not be used through this call and through the one-stream calls
 * in between a fork and its join.  Errors as ssd_decode_step, plus
 * SSD_ERR_INVALID_ARG for a bad stream list or sync value.
 */
enum { SSD_MAX_SPLIT = 4 };
enum { SSD_SPLIT_FORK = 1, SSD_SPLIT_JOIN = 2 };
int ssd_decode_step_split(ssd_cache *cache, int layer_begin, int layer_end, const void *q,
                          const void *k_new, const void *v_new, void *out,
                          int accumulate_scores, int compress,
                          void *const *streams, int n_streams, int sync);
int ssd_decode_step_split_plan(const ssd_cache *cache, int layers_per_call, int n_streams,
                               int32_t *part_seqs, int32_t *n_parts);   /* either output may be NULL */

/*
 * The same step with rotary position embedding (Su et al., "RoFormer") applied
 * to q and k_new on the way in, so that the rows the projections produce need
 * no launch of their own before this one.  The paper does not describe the
 * model's position encoding; this is the standard form used by the LLaMA
 * family of language models that Janus-Pro builds on.
 *   cos, sin    : dev float [d/2], 16-byte aligned: cos and sin of the new
 *                 token's angles theta_i * position, i = 0..d/2-1 (one row of
 *                 the caller's tables; the same for every layer, sequence and
 *                 head of the call)
 *   rope_layout : SSD_ROPE_HALF pairs element i with element i + d/2 ("rotate
 *                 half"); SSD_ROPE_INTERLEAVED pairs element 2i with 2i+1.
 * A pair (a, b) becomes (a*cos_i - b*sin_i, b*cos_i + a*sin_i), computed in
 * fp32 and rounded once to the cache dtype; the rotated k is what the cache
 * stores, v_new is untouched.  The result equals ssd_decode_step on rows
 * rotated and rounded beforehand.  Errors as ssd_decode_step, plus
 * SSD_ERR_INVALID_ARG for a bad layout or missing / misaligned cos, sin.
 */
enum { SSD_ROPE_HALF = 1, SSD_ROPE_INTERLEAVED = 2 };
int ssd_decode_step_rope(ssd_cache *cache, int layer_begin, int layer_end, const void *q,
                         const void *k_new, const void *v_new, void *out, int accumulate_scores,
                         int compress, const float *cos, const float *sin, int rope_layout,
                         void *stream);
/* ssd_decode_step_rope with the batch dealt to several streams: the stream arguments of ssd_decode_step_split. */
int ssd_decode_step_split_rope(ssd_cache *cache, int layer_begin, int layer_end, const void *q,
                               const void *k_new, const void *v_new, void *out, int accumulate_scores,
                               int compress, const float *cos, const float *sin, int rope_layout,
                               void *const *streams, int n_streams, int sync);

/* ---- exports for tests and benchmarks (not steps of the method) ------------ */

/*
 * Test / benchmark export of one layer's index table.
 *   pos   : dev int32 [B, H, slots]  absolute position held by each slot, -1 if unused
 *   score : dev float [B, H, slots]  accumulated score of the slot (0 for spatial heads)
 *   count : dev int32 [B, H]         retained tokens of the head
 * slots = ssd_cache_export_slots(cache) = max(S + W, M + C) over all layers.  Any of the three may be NULL.
 */
int ssd_cache_export_slots(const ssd_cache *cache);
int ssd_cache_export(ssd_cache *cache, int layer, int32_t *pos, int32_t *count,
                     float *score, void *stream);

/*
 * Full-cache decode attention, the baseline the paper compares against
 * (Sec. 4.1 "Full Cache"), which also produces the (far, tot) masses that
 * ssd_classify_heads consumes.
 *   q, out : dev [B, H, d]
 *   K, V   : dev [B, H, n_cap, d]; rows 0..n-1 are attended
 *   far, tot : dev float, element of unit (b, h) at index (b*H + h) * mass_stride;
 *              both NULL to skip.  Visual rows start at vis_start; w is the
 *              recency window of the metric (the paper uses 32).
 *   workspace : dev scratch of at least ssd_dense_workspace_bytes(B, H, d, n) bytes,
 *               256-byte aligned (partial results of the split over rows)
 */
size_t ssd_dense_workspace_bytes(int B, int H, int d, int n);
int ssd_dense_decode_attn(const void *q, const void *K, const void *V, void *out,
                          int B, int H, int d, int dtype, int n_cap, int n,
                          float softmax_scale, float *far, float *tot, int mass_stride,
                          int vis_start, int w, void *workspace, size_t workspace_bytes,
                          void *stream);

/*
 * ssd_dense_decode_attn for callers that cannot allocate device memory or hand over a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without the workspace,
 * same kernels, same results bit for bit; the partial results of the row splits go to a fixed scratch array of
 * SSD_DENSE_STATIC_SCRATCH_BYTES that is part of the library's code object (every GPU the library runs on holds
 * its own copy until the process ends).  The call allocates nothing and frees nothing.
 *   - The device of `stream` must be the calling thread's current device (the scratch is looked up per device,
 *     once, at the first call on that device).
 *   - A shape whose partial results (B * H * splits * (4 + d) floats, splits as ssd_dense_decode_attn picks them)
 *     exceed the scratch is refused with SSD_ERR_INVALID_ARG before anything is enqueued; B * H >= 8192 needs no
 *     scratch at all.
 *   - All calls on one GPU share that GPU's scratch and leave their partial results in it: two calls that may
 *     run at the same time on one GPU (different streams, different threads) race and must not be made; calls
 *     on one stream are ordered and safe.  Nothing in it has to start at zero.
 */
#define SSD_DENSE_STATIC_SCRATCH_BYTES (8u << 20)
int ssd_dense_decode_attn_static(const void *q, const void *K, const void *V, void *out,
                                 int B, int H, int d, int dtype, int n_cap, int n,
                                 float softmax_scale, float *far, float *tot, int mass_stride,
                                 int vis_start, int w, void *stream);

/* Text of the calling thread's most recent error ("" if none). Never NULL. */
const char *ssd_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int ssd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SSD_H */
