/*
 * hca.h: C ABI of libhca.so, the decode-time heterogeneous attention path of
 * HCAttention (arXiv 2507.19823) for one AMD MI355X (gfx950).
 *
 * The path evaluates the paper's Eq. 2,
 *     y~ = F_evict(softmax(q . Q(K)^T / sqrt(d))) . F_evict(V),
 * in four steps: compress keys (Q), score the query against the whole compressed
 * key cache (Sec. 3.2 "GPU part", Eq. 3), select the highest-scoring tokens
 * (the sorted prefix of Sec. 3.2 / Eq. 4, here with k given), and form the
 * softmax-weighted sum over the selected values only (Eq. 5), the values living
 * in pinned host memory (Sec. 3.2 "CPU part": value offloading) or in an HBM
 * slice.  A fifth call keeps the cache bounded by accumulated-score eviction.
 *
 * Conventions
 *  - Every call returns an int32_t status: HCA_OK or a negative HCA_ERR_*.
 *    Arguments are validated on the host before any device work; a call that
 *    returns an error has launched nothing.  No exception crosses the boundary.
 *  - "device" pointers are HBM addresses valid on the current HIP device;
 *    "host" pointers are ordinary host memory read during the call;
 *    "pinned" pointers are host memory allocated with hipHostMalloc (or a
 *    pinned torch tensor) and are dereferenced by GPU kernels.
 *  - The caller owns every buffer.  The library allocates no device memory;
 *    scratch space comes from the `workspace` argument, at least
 *    hca_workspace_bytes() bytes, 256-byte aligned, private to the call while
 *    it is in flight (two calls that may overlap need two workspaces).
 *  - Calls are asynchronous: they enqueue work on `stream` (a hipStream_t
 *    passed as void*, NULL = the default stream) and return.  They never
 *    synchronise the device.
 *  - Shapes: query head hq belongs to KV head hq / (n_q_heads / n_kv_heads).
 *    A "row" is one (sequence, KV head) pair, r = b * n_kv_heads + h.
 *  - n_resident is a host array [batch]: tokens currently in the cache of each
 *    sequence (equal for all KV heads of a sequence).
 *  - Supported shapes: head_dim 128; (bits, group) = (4, 32) or (2, 64);
 *    n_q_heads / n_kv_heads in {1, 2, 4}.  Anything else: HCA_ERR_UNSUPPORTED.
 *  - Inputs must be finite (no NaN / Inf); the result is unspecified otherwise.
 *  - State the library keeps between calls (everything else is the caller's):
 *    the process-wide launch knobs of hca_tune (read by the per-call entry
 *    points; a step driver copies them once at creation); a per-thread ring of HIP events used inside
 *    hca_sparse_attend; the worker threads of hca_host_weighted_sum, started by
 *    its first call with n_threads > 1, asleep between calls and never joined
 *    before the process ends; the 16 MiB device array of hca_topk_noalloc; and
 *    whatever an hca_pipeline object holds until hca_pipeline_destroy (events,
 *    its own worker threads and pinned exchange buffers when host_chunks > 0).
 */
#ifndef HCA_H_
#define HCA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HCA_OK 0
#define HCA_ERR_BAD_ARG (-1)     /* null pointer, negative size, inconsistent shape */
#define HCA_ERR_UNSUPPORTED (-2) /* shape outside the supported set */
#define HCA_ERR_CAPACITY (-3)    /* append past capacity, k or M out of range */
#define HCA_ERR_HIP (-4)         /* a HIP call failed; see hca_last_hip_error() */

typedef struct {
  int32_t batch;      /* sequences */
  int32_t n_q_heads;  /* query heads per sequence */
  int32_t n_kv_heads; /* KV heads per sequence */
  int32_t head_dim;   /* d of Eq. 1; 128 */
  int32_t bits;       /* bits per key code */
  int32_t group;      /* channels sharing one scale / zero */
  int64_t capacity;   /* max resident tokens per (sequence, KV head) */
} hca_shape;

/* Library version string (static storage). */
const char* hca_version(void);

/* Overrides a launch-shape knob for the per-call entry points (process-wide state, meant for tuning and
 * profiling sessions, not needed for correct results; a step driver takes its knobs from its own
 * hca_pipeline_desc instead and only starts from these).  Names: "gather_wgs", "gather_unroll", "score_bpw", "score_depth", "select_wg" (threads per workgroup of the
 * selection over the candidate lists of hca_score_topk: 1024 - pairs staged in 128 KiB of LDS, needs a whole compute
 * unit - or 256 - four waves, pairs staged in 96 KiB of LDS when k <= 4096 and read from L2 otherwise, fits into
 * the room one finished scan workgroup leaves, slower where measured; 0: 1024; the launch for rows that needed a
 * second scan always takes the 256 form when two layers are selected by one launch),
 * "host_isa" (2: the hybrid value side's host threads use their AVX2 form even where the CPU has AVX-512; 0: the
 * widest form), "host_spin_us" (how long the worker threads of hca_host_weighted_sum poll for the next
 * call before they sleep; default 100, 0 = sleep at once).
 * Returns HCA_ERR_BAD_ARG for an unknown name. */
int32_t hca_tune(const char* name, int32_t value);

/* hipError_t of the most recent failing HIP call made by this thread (0 if none). */
int32_t hca_last_hip_error(void);

/* Bytes of the compressed key cache for `shape` (codes + scales + zeros of all
 * rows, in the library's private tiled layout); 0 if the shape is unsupported.
 * Sec. 3.3 "Compression ratio": the code part is head_dim*bits/8 bytes per token
 * per KV head, i.e. 1/4 (4-bit) or 1/8 (2-bit) of the fp16 keys. */
size_t hca_kcache_bytes(const hca_shape* shape);

/* Workspace bytes sufficient for any call with top-k <= k_max and eviction
 * keep-count <= m_max on this shape. */
size_t hca_workspace_bytes(const hca_shape* shape, int64_t k_max, int64_t m_max);

/* Step 1, Q(K) of Eq. 2: quantise T new tokens per row and append them at slots
 * n_resident[b] .. n_resident[b]+T-1.
 *   k_new_f16   device, fp16 [batch, n_kv_heads, T, head_dim], contiguous
 *   kcache      device, hca_kcache_bytes() bytes, updated in place
 * Per (token, group): zero = min, scale = fp16((max-min)/(2^bits-1)) (1.0 if that
 * is 0), code = clamp(rint((x-zero)*(1/scale)), 0, 2^bits-1).
 * Slot bookkeeping for the new tokens is fused in when acc_opt / pos_opt are given:
 *   acc_opt     device, fp32 [batch, n_kv_heads, capacity] or NULL: acc[slot] = 0
 *   pos_opt     device, int32 [batch, n_kv_heads, capacity] or NULL:
 *               pos[slot of new token t] = value_row0[b] + t
 *   value_row0  host, int64 [batch]: value-store row of each sequence's first new token
 *               (required iff pos_opt is given)
 * The caller adds T to n_resident afterwards.
 * Errors: HCA_ERR_CAPACITY if n_resident[b]+T > capacity. */
int32_t hca_quantize_keys(const hca_shape* shape, void* kcache, const void* k_new_f16,
                          int64_t T, const int64_t* n_resident, float* acc_opt, int32_t* pos_opt,
                          const int64_t* value_row0, void* stream);

/* Step 2, z~ = q . Q(K)^T of Eq. 2 / Eq. 3 for every resident token, keys
 * dequantised on the fly.  The query is first mapped to 15-bit fixed point per
 * head (qfx = rint(q * 2^s), |qfx| < 2^14) so that each group's dot product is an
 * exact integer; then z~ = 2^-s * sum_g fma(scale_g, D_g, zero_g * Q_g).
 *   q_f16   device, fp16 [batch, n_q_heads, head_dim]
 *   sel     device, fp32 [batch, n_kv_heads, capacity]; sel[r][j] = max over the
 *           query heads of row r of z~[hq][j], written for j < n_resident
 *   z_opt   device, fp32 [batch, n_q_heads, capacity] or NULL: every z~ */
int32_t hca_score_qkeys(const hca_shape* shape, const void* kcache, const void* q_f16,
                        const int64_t* n_resident, float* sel, float* z_opt,
                        void* workspace, void* stream);

/* Step 3a, the sorted prefix Pi_k of Sec. 3.2 with k fixed: per row the
 * k' = min(k, n_resident) slots with the largest sel, ties broken towards the
 * lower slot, reported in ascending slot order.
 *   idx    device, int32 [batch, n_kv_heads, k]; entries past k' are left untouched
 *   count  device, int32 [batch, n_kv_heads] = k'
 * Errors: HCA_ERR_CAPACITY if k < 1 or k > capacity. */
int32_t hca_topk(const hca_shape* shape, const float* sel, const int64_t* n_resident,
                 int32_t k, int32_t* idx, int32_t* count, void* workspace, void* stream);

/* hca_topk for callers that cannot allocate or pass device scratch memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same result as hca_topk, bit for bit; the scratch memory of
 * its kernels is a 16 MiB array inside the library's device image (one copy per GPU, held until the process
 * ends) instead of a workspace.  The call allocates nothing and frees nothing.
 * Limit: rows * (32 KiB + 8 B * (roundup(n_max, 1024) + 2 * max(4096, roundup(ceil(n_max / 1024), 1024)))) must
 * not exceed 16 MiB, n_max being the largest n_resident and rows = batch * n_kv_heads - e.g. 8 rows of 131 136
 * slots, 32 rows of 32 Ki; beyond it: HCA_ERR_CAPACITY (nothing launched).  capacity may be larger than n_max.
 * All calls on one GPU share that GPU's array: calls that may overlap there (different streams, different
 * threads) race; calls on one stream are ordered and safe.  Other arguments and errors as hca_topk. */
int32_t hca_topk_noalloc(const hca_shape* shape, const float* sel, const int64_t* n_resident, int32_t k,
                         int32_t* idx, int32_t* count, void* stream);

/* Steps 2 and 3a in one call (Eq. 2, then the sorted prefix Pi_k of Sec. 3.2): idx and count exactly as
 * hca_score_qkeys followed by hca_topk would leave them, without the score of every slot ever reaching
 * memory.  A strided sample of each row (8192 to 65536 slots) is scored first and gives a threshold that at least k
 * slots of the row pass with overwhelming probability; the scan then keeps only the (score, slot) pairs
 * at or above it, and the selection runs on those few thousand pairs.  A row whose sample misled (fewer
 * than k pairs) is scanned a second time inside the same call - with a lower threshold that a count taken
 * during the first scan proves sufficient, else with none -, so the result never depends on the sample;
 * only the time does.
 *   workspace  device, hca_workspace_bytes(shape, k, 1) bytes
 * Errors: HCA_ERR_CAPACITY if k < 1, k > capacity, or a row holds more than 8 Mi resident slots. */
int32_t hca_score_topk(const hca_shape* shape, const void* kcache, const void* q_f16, const int64_t* n_resident,
                       int32_t k, int32_t* idx, int32_t* count, void* workspace, void* stream);

/* What the last hca_score_topk on `workspace` did (same shape and n_resident; to be called before the workspace
 * is used for anything else): per row the number of (score, slot) pairs that passed the threshold of the scan
 * that produced the result - all resident slots if that was the second scan - and whether the row needed that
 * second scan.  A monitor for the sampling step with which the top-k of Sec. 3.2 is found here, not part of the
 * method.
 *   candidates, rescanned  device, int32 [batch, n_kv_heads] each */
int32_t hca_score_topk_report(const hca_shape* shape, const int64_t* n_resident, void* workspace,
                              int32_t* candidates, int32_t* rescanned, void* stream);

/* The same monitor kept running over many calls: every fused selection on `workspace` (hca_score_topk, or a layer
 * of hca_pipeline_step that was given it as ws_select) adds to four figures per row - selections counted, the
 * fewest and the most pairs a first scan let through, selections that needed the second scan.  This call copies
 * them to `out` (if not null) and then, if reset != 0, starts them afresh (count 0, fewest 2^31 - 1, most 0,
 * second scans 0).  A workspace's figures mean nothing before its first reset.  Not part of the method either.
 *   out  device, int32 [batch, n_kv_heads, 4], or null */
int32_t hca_score_topk_monitor(const hca_shape* shape, void* workspace, int32_t* out, int32_t reset, void* stream);

/* Step 3b, Eq. 5 with the softmax taken over the selected set: for each query
 * head, l_i = z~[idx_i] * sm_scale (z~ recomputed from the codes),
 * a = softmax(l), y = sum_i a_i * V[pos[idx_i]].
 *   idx, count  device, as written by hca_topk (k = row stride of idx)
 *   pos         device, int32 [batch, n_kv_heads, capacity]: value row of each slot
 *   v_host      pinned, fp16 [batch, n_kv_heads, host_stride, head_dim]; serves value
 *               rows < n_host_rows (may be NULL if n_host_rows == 0)
 *   v_hbm       device, fp16 [batch, n_kv_heads, hbm_stride, head_dim]; serves value
 *               row v >= n_host_rows at index v - n_host_rows (may be NULL if unused)
 *   y           device, fp32 [batch, n_q_heads, head_dim]
 *   acc_opt     device, fp32 [batch, n_kv_heads, capacity] or NULL:
 *               acc[idx_i] += sum over the row's query heads of max(a_i, 1e-30)
 *   gather_stream  the value rows are first gathered into the workspace on this
 *               stream (ordered after `stream`'s work enqueued so far); `stream`
 *               then waits for the gather.  May equal `stream`. */
int32_t hca_sparse_attend(const hca_shape* shape, const void* kcache, const void* q_f16,
                          const int32_t* idx, const int32_t* count, int32_t k,
                          const int32_t* pos,
                          const void* v_host, int64_t host_stride, int64_t n_host_rows,
                          const void* v_hbm, int64_t hbm_stride,
                          float sm_scale, float* y, float* acc_opt,
                          void* workspace, void* gather_stream, void* stream);

/* The two halves of hca_sparse_attend, for callers that overlap the host-link gather of one
 * layer with the key scan of the next (Sec. 3.2: the value side runs off the GPU's critical
 * path).  hca_gather_values copies the selected value rows into `workspace` on `stream`;
 * hca_attend_gathered, called later with the same idx / count / k / workspace and ordered
 * after the gather by the caller (event or same stream), computes y and updates acc_opt.
 * Arguments as in hca_sparse_attend. */
int32_t hca_gather_values(const hca_shape* shape, const int32_t* idx, const int32_t* count, int32_t k,
                          const int32_t* pos, const void* v_host, int64_t host_stride, int64_t n_host_rows,
                          const void* v_hbm, int64_t hbm_stride, void* workspace, void* stream);
int32_t hca_attend_gathered(const hca_shape* shape, const void* kcache, const void* q_f16, const int32_t* idx,
                            const int32_t* count, int32_t k, float sm_scale, float* y, float* acc_opt,
                            void* workspace, void* stream);

/* Step 4, accumulated-score eviction.  Rows with n_resident > M keep their newest
 * n_protect slots and, of the others, the M - n_protect with the highest acc (ties
 * towards the lower slot); the kept slots move, in ascending old-slot order, to
 * slots 0..M-1 of kcache, acc and pos.  The caller then sets
 * n_resident[b] = min(n_resident[b], M).
 * Two modes:
 *   in place (kcache_dst == acc_dst == pos_dst == NULL): the compacted rows are staged
 *     in the workspace and copied back; rows of sequences with n_resident <= M are
 *     left untouched;
 *   out of place (all three given, distinct from the sources): the compacted rows are
 *     written straight into a second cache / acc / pos of the same shape, rows with
 *     n_resident <= M are carried over unchanged, and the caller swaps the buffers
 *     afterwards.  This halves the bytes moved; one spare buffer serves any number of
 *     layers, the source of one eviction being the spare of the next.
 *   kept_opt  device, int32 [batch, n_kv_heads, M] or NULL: old slot of each new slot
 *             (written only for rows that were compacted)
 * Errors: HCA_ERR_CAPACITY if M < 1, M > capacity or n_protect > M. */
int32_t hca_evict(const hca_shape* shape, void* kcache, float* acc, int32_t* pos,
                  const int64_t* n_resident, int64_t M, int64_t n_protect,
                  int32_t* kept_opt, void* workspace, void* kcache_dst, float* acc_dst,
                  int32_t* pos_dst, void* stream);

/* ---- Step driver -------------------------------------------------------------------------
 * One decode step over all layers of a model, enqueued as a four-stage pipeline across layers:
 * (append + key scan) | top-k | host-link gather | (attend + eviction), one stream per stage,
 * the stages of a layer chained by events, different layers overlapping (Sec. 3.2: the value
 * side runs beside the GPU's scoring, not after it).  It issues exactly the kernels of the
 * per-step calls above; it exists because enqueueing ~15 launches per layer from a scripting
 * language costs more than the kernels take.  Legal only when the queries of all layers exist
 * before the step (benchmarks with synthetic queries; speculative / batched serving). */
typedef struct {
  void* kcache; float* acc; int32_t* pos;   /* device; swapped with the spare set when the layer is evicted */
  const void* k_new;                        /* device, fp16 [batch, n_kv_heads, 1, head_dim]: this step's key */
  const void* q;                            /* device, fp16 [batch, n_q_heads, head_dim] */
  const void* v_host;                       /* pinned value store (rows < n_host_rows) or NULL */
  const void* v_hbm;                        /* device value slice (rows >= n_host_rows) or NULL */
  float* y;                                 /* device, fp32 [batch, n_q_heads, head_dim] */
  /* codebook form only (hca_pipeline_desc.vq_groups > 0): kcache is then the layer's index cache
     (hca_vq_pcache_bytes) */
  const float* vq_centroids;                /* device, the layer's codebook, fp32 [n_kv_heads, g, c, dbar] */
  float* vq_lut;                            /* device, hca_vq_lut_bytes: the layer's table, written by the scan
                                               stage and read by its attend */
} hca_layer;

#define HCA_PIPELINE_MAX_SEL 64
#define HCA_PIPELINE_MAX_PIPE 8
typedef struct {
  /* hipStream_t of the four stages.  Distinct streams let the stages of different layers overlap (the throughput
     form).  The same stream may be given for several stages, which then run one after another; with one stream
     for all four a step is the plain sequence of its kernels with no event hop between them - the form with the
     lowest latency for a single layer. */
  void *stream_scan, *stream_topk, *stream_gather, *stream_attend;
  float* sel[HCA_PIPELINE_MAX_SEL]; /* device, fp32 [batch, n_kv_heads, capacity] each; the first n_sel are used */
  int32_t n_sel;                 /* 3 .. HCA_PIPELINE_MAX_SEL score buffers.  With one per layer the key scan of a
                                    layer never waits for the top-k of an earlier layer to release its buffer */
  int32_t* idx[HCA_PIPELINE_MAX_PIPE];    /* device, int32 [batch, n_kv_heads, k] each; the first n_pipe are used */
  int32_t* count[HCA_PIPELINE_MAX_PIPE];  /* device, int32 [batch, n_kv_heads] each */
  void* ws_attend[HCA_PIPELINE_MAX_PIPE]; /* device, hca_workspace_bytes(shape, k, 1) each */
  void* ws_topk;                 /* device, hca_workspace_bytes(shape, k, 1); owned by the driver from
                                    hca_pipeline_create on (it keeps a histogram there between steps) */
  void* ws_evict;                /* device, hca_workspace_bytes(shape, k, M); NULL if eviction is never asked for */
  void* spare_kcache; float* spare_acc; int32_t* spare_pos;   /* spare set for out-of-place eviction (all three), or all
                                    NULL: layers are then compacted in place, which moves only the slots at and after
                                    the first dropped one */
  /* optional profiling of the key scan: device, uint64 [timing_slots][n_layers][scan_stamp_pairs][2];
     every wave of a timed scan launch stores its start and end wall-clock tick there (zero-filled by the
     caller; entries left 0 belong to waves that had nothing to do).  NULL: off. */
  void* scan_stamps; int64_t scan_stamp_pairs;
  int32_t timing_layer_stride;   /* HIP-event brackets only around the scan of layers l % stride == 0 (0, 1: all);
                                    each bracket costs two more packets on the scan stream */
  /* The paper's own form of the step (Sec. 3.1, 3.2).  vq_groups > 0: the key side is the codebook form -
     hca_vq_assign, hca_vq_score, hca_vq_attend_gathered, hca_vq_evict (in place: the spare_* fields must be
     NULL) instead of their uniform-code counterparts, with the codebook shape given here and each layer's
     centroids and table in its hca_layer; the workspaces above are then sized with hca_vq_workspace_bytes.
     topp_tau > 0: the selection is Eq. 4 (hca_topp with this tau and the
     step's k as the cut-off) instead of top-k.  The two are independent. */
  int32_t vq_groups, vq_codewords;
  double topp_tau;
  /* fused_select != 0: scan and top-k as in hca_score_topk (uniform codes and top-k only): the scan stage
     estimates the threshold and leaves the candidate lists, the top-k stage selects from them.  No score
     buffer is written: sel[] is ignored, and the first n_sel entries of ws_select are the per-slot
     workspaces instead (device, hca_workspace_bytes(shape, k, 1) each). */
  int32_t fused_select;
  void* ws_select[HCA_PIPELINE_MAX_SEL];
  /* optional profiling of the value gather, like scan_stamps: device, uint64 [timing_slots][n_layers][1024][2],
     zero-filled by the caller; every workgroup of a timed gather launch (at most 1024) stores its start and end
     wall-clock tick.  NULL: off. */
  void* gather_stamps;
  /* Hybrid value side (Sec. 3.2 "CPU part", Eq. 5 for a share of the selection; uniform codes only).
     host_chunks > 0: of every row's selected tokens (ascending slot order, chunks of 256) the first host_chunks
     chunks are not gathered over the host link; the GPU sends, per token, its value-row number and one fp32
     weight per query head (relative to the chunk's maximum) to pinned memory, host threads of the driver form
     the chunk's partial sums from the value store where it lives, and the GPU merges them with the partial sums
     of the gathered chunks under the one softmax normaliser.  Selection, accumulated scores and eviction are
     unaffected; y differs from the all-gather form by fp32 summation order only.  Tokens of those chunks whose
     value row is not in the host store (rows >= n_host_rows) are summed on the GPU.
     host_threads: worker threads (1 .. 64; they poll while steps are in flight and sleep when idle; 0 starts
     none - then every merge times out, for tests of that path).  host_spin_limit: polls of the host's flag
     before a merge gives up and records a timeout (0: about a second); see hca_pipeline_host_status.
     The driver owns the pinned exchange buffers (28 bytes per selected token of the host share - four fp32 weights, a
     row number, and 2 KiB of partial sums per chunk of 256 -, one set per
     idx / count / ws_attend set) and the threads from hca_pipeline_create to hca_pipeline_destroy. */
  int32_t host_chunks, host_threads, host_spin_limit;
  /* Launch-shape knobs of this pipeline's kernels (0: the library's default; ranges as in hca_tune). */
  int32_t gather_wgs, gather_unroll, score_bpw, score_depth, select_wg;
  /* Sets of idx / count / ws_attend in use: 0 or 4 .. HCA_PIPELINE_MAX_PIPE.  A set is held by a layer from its
     top-k to the end of its attend; with the hybrid value side that span holds the host threads' turn too, and
     more than four layers have to be in flight to keep every stage busy. */
  int32_t n_pipe;
  /* fused_select only, n_sel >= 6 or one workspace per layer.
     dual_scan == 1: two scan streams.  Even layers run append + scan + selection on stream_scan, odd layers on
     stream_topk; the scans of the two overlap, so the key stream from HBM does not pause between launches.
     dual_scan == 2: paired launches.  Layers l and l + 1 (l even) are scanned by one launch on stream_scan, their
     selections follow on stream_topk: half as many pauses between scan launches, one launch tail per two
     layers.  hca_pipeline_scan_ms then reports the shared launch under the even layer and -1 for the odd one. */
  int32_t dual_scan;
  /* Optional: one result buffer per layer for the selection instead of the idx / count of the n_pipe sets.
     layer_idx != NULL: layer l's selected slots go to layer_idx + l * layer_idx_stride (int32 [batch, n_kv_heads, k],
     layer_idx_stride >= batch * n_kv_heads * k elements) and its counts to layer_count + l * batch * n_kv_heads;
     idx[] / count[] are ignored.  The selection of a layer then waits for nothing but its own scan - a set of
     ws_attend (and of the host share's exchange buffers) is claimed only by the gather stage - so selections run
     in step with the scans, well ahead of the value side, and the stages behind them are fed as soon as a set
     comes free instead of once per scan launch. */
  int32_t* layer_idx;
  int32_t* layer_count;
  int64_t layer_idx_stride;
} hca_pipeline_desc;

typedef struct hca_pipeline hca_pipeline;

/* Creates the driver (host object + HIP events; no device memory).  timing_slots > 0 reserves
 * that many sets of timing events around the key-scan launches.  NULL on bad arguments. */
hca_pipeline* hca_pipeline_create(const hca_shape* shape, int32_t n_layers, const hca_pipeline_desc* desc,
                                  int32_t timing_slots);
void hca_pipeline_destroy(hca_pipeline* p);

/* Enqueues one decode step.  Every argument, length and capacity of every layer is checked before the first
 * enqueue: an HCA_ERR_BAD_ARG / HCA_ERR_CAPACITY return has launched nothing and has changed neither n_resident
 * nor layers.  HCA_ERR_HIP (a HIP call failed while enqueueing) can come from the middle of a step: part of it
 * is then enqueued and n_resident / layers updated for the layers reached; the caller synchronises the device
 * and abandons the pipeline.
 * layers: host array [n_layers], updated when buffers swap on eviction.
 * n_resident: host, int64 [n_layers][batch], updated (+1 for the appended token, then min(., evict_M)).
 * value_row0: value-store row of the appended token (all sequences).  evict_M: host, int64 [n_layers]
 * or NULL; layer l with evict_M[l] != 0 and n_resident > evict_M[l] is evicted to evict_M[l] after its
 * attend (callers stagger the layers over the steps of an eviction period so that no step carries all
 * of them).  timing_slot < 0: no timing. */
int32_t hca_pipeline_step(hca_pipeline* p, hca_layer* layers, int64_t* n_resident, int64_t value_row0, int32_t k,
                          int64_t host_stride, int64_t n_host_rows, int64_t hbm_stride, float sm_scale,
                          const int64_t* evict_M, int64_t n_protect, int32_t timing_slot);

/* Hybrid value side: *wait_timeouts != 0 if a merge ever gave up waiting for the host threads (its y is then
 * wrong), *bad_rows = value-row numbers outside the host store that the host threads were handed (skipped).
 * Both stay 0 in a correct run.  *mean_job_us: mean time the host threads took per layer, from the GPU's signal
 * to the last chunk's partial sum; *mean_chunk_us: mean time per chunk of 256 tokens.  Any pointer may be NULL. */
int32_t hca_pipeline_host_status(hca_pipeline* p, uint32_t* wait_timeouts, uint32_t* bad_rows, double* mean_job_us,
                                 double* mean_chunk_us);

/* Host code, blocks until done: reads one byte of every 4 KiB page of [ptr, ptr + bytes) with n_threads threads
 * (1 .. 64).  For a pinned value store that the hybrid value side's host threads (or hca_host_weighted_sum) will
 * read: the first CPU access to a page of a pinned allocation is a page fault of several microseconds, which
 * would otherwise be paid inside the first decode steps, once per selected row. */
int32_t hca_host_prefault(const void* ptr, size_t bytes, int32_t n_threads);

/* Test / debug, host code: the work of one host thread of the hybrid value side on one chunk of 256 selected
 * tokens: py[h][c] = sum_i p[h][i] * V[vrow[i]][c] over the entries with vrow[i] >= 0, for h < gqa (rows of the
 * other heads are zero).
 *   p      host, fp32 [4][256]         vrow  host, int32 [256]
 *   v_rows host, fp16 [n_rows][128]    py    host, fp32 [4][128]
 * Returns the number of entries with vrow >= n_rows (skipped), or HCA_ERR_BAD_ARG. */
int32_t hca_debug_host_chunk_sum(int32_t gqa, const float* p, const int32_t* vrow, const void* v_rows, int64_t n_rows,
                                 float* py);

/* (start, end) pairs a key-scan launch over n_tokens resident tokens may write into scan_stamps. */
int64_t hca_scan_stamp_pairs(const hca_shape* shape, int64_t n_tokens);
/* Rate of the wall clock behind scan_stamps in kHz (0 if unknown). */
int32_t hca_wall_clock_khz(void);

/* After the device has finished the step recorded in `timing_slot`: duration of each layer's
 * key-scan launch in milliseconds, ms[n_layers] (host). */
int32_t hca_pipeline_scan_ms(hca_pipeline* p, int32_t timing_slot, float* ms);

/* Test / debug: export the cache in canonical row-major form.
 *   codes  device, uint8 [batch, n_kv_heads, capacity, head_dim*bits/8]; channel c in bits
 *          [(c*bits)%8, +bits) of byte c*bits/8
 *   scale_f16, zero_f16  device, fp16 [batch, n_kv_heads, capacity, head_dim/group]
 * Only slots < n_resident are written. */
int32_t hca_export_kcache(const hca_shape* shape, const void* kcache, const int64_t* n_resident,
                          uint8_t* codes, void* scale_f16, void* zero_f16, void* stream);

/* ---- The paper's selection rule ---------------------------------------------------------------
 * Sec. 3.2, Eq. 4: with the slots of a row sorted by score in descending order (ties towards the lower
 * slot, as in hca_topk), keep the shortest prefix whose cumulative attention weight reaches tau.  The
 * weights are a~_j = softmax_j(sel_j * sm_scale) over the row's resident slots, sel being the per-KV-head
 * selection score of hca_score_qkeys / hca_vq_score.  So that the integer k* does not depend on the order
 * of a floating-point sum, each weight is an integer: l = sel * sm_scale; u = l - max l; t = u * log2(e)
 * (all fp32); 0 below t = -64; fl = floor(t), f = t - fl; p = 2^f by the degree-6 Taylor polynomial in f ln 2
 * (Horner, fused multiply-adds); w = (uint64)(p * 2^31) >> -fl.  Z = sum w; Theta = max(1, floor(Z * floor(tau *
 * 2^64) / 2^64)) (Theta = Z for tau >= 1); k* = least k with w_(1) + ... + w_(k) >= Theta.
 *   k_max     the prefix is cut at k_max slots (capacity of idx); 1 <= k_max <= capacity
 *   idx       device, int32 [batch, n_kv_heads, k_max]: selected slots in ascending order
 *   count     device, int32 [batch, n_kv_heads]: min(k*, k_max); 0 for a sequence without resident slots
 *   mass_opt  device, uint64 [batch, n_kv_heads, 2] or NULL: (Theta, Z) of each row
 *   workspace device, hca_workspace_bytes(shape, k_max, 1)
 * The result feeds hca_gather_values / hca_attend_gathered like the result of hca_topk (k = k_max).
 * Errors: HCA_ERR_BAD_ARG unless tau > 0 and sm_scale > 0; HCA_ERR_CAPACITY for k_max out of range. */
int32_t hca_topp(const hca_shape* shape, const float* sel, const int64_t* n_resident, float sm_scale, double tau,
                 int32_t k_max, int32_t* idx, int32_t* count, uint64_t* mass_opt, void* workspace, void* stream);

/* The paper's own weights (Sec. 3.2, Eq. 5): a~ = softmax(z~ / sqrt(d)) is taken over ALL resident tokens
 * and the weights of the selected ones are used as they are, not renormalised over the selected set.
 * hca_score_qkeys_lse is hca_score_qkeys with a second output, the log of that softmax's denominator,
 *   lse  device, fp32 [batch, n_q_heads]: log sum_{j < n_resident} exp(z~[hq][j] * sm_scale); -inf for a
 *        sequence without resident tokens
 *   workspace  device, hca_workspace_bytes(shape, 1, 1)
 * and hca_attend_gathered_global is hca_attend_gathered with the weights exp(l_i - lse[hq]): y is shorter than
 * the renormalised one by the factor (weight mass of the selected tokens), acc_opt accumulates the same weights. */
int32_t hca_score_qkeys_lse(const hca_shape* shape, const void* kcache, const void* q_f16,
                            const int64_t* n_resident, float sm_scale, float* sel, float* lse, void* workspace,
                            void* stream);
int32_t hca_attend_gathered_global(const hca_shape* shape, const void* kcache, const void* q_f16, const int32_t* idx,
                                   const int32_t* count, int32_t k, float sm_scale, const float* lse, float* y,
                                   float* acc_opt, void* workspace, void* stream);

/* ---- The paper's CPU-GPU split of the value side ----------------------------------------------
 * Sec. 3.2 "CPU part", Eq. 5, and Sec. 3.3 "Communication overhead": the values never leave host memory;
 * per selected token only its value-row number and one 2-byte weight per query head cross the link, and the
 * host forms the weighted sum.  (The graded path does the opposite: value rows come to the GPU,
 * hca_gather_values.)
 * hca_attend_weights: softmax weights of the selected tokens, as hca_attend_gathered computes them
 * (renormalised over the selected set, or the paper's exp(l - lse) when lse_opt is given), rounded to fp16.
 *   w_f16    device or pinned host, fp16 [batch, n_q_heads, k]: weight of selected token i for each query
 *            head; 0 past count
 *   vrow     device or pinned host, int32 [batch, n_kv_heads, k]: pos[idx[i]], the token's row in the value
 *            store; -1 past count
 *   acc_opt  as in hca_sparse_attend (the unrounded weights are accumulated)
 *   workspace device, hca_workspace_bytes(shape, k, 1)
 * hca_host_weighted_sum: host code, blocks until done: y[hq] = sum_i w[hq][i] * V[vrow[i]] in fp32.
 *   vrow, count, w_f16  host-readable copies of the outputs above (count: int32 [batch, n_kv_heads])
 *   v_host   host, fp16 [batch, n_kv_heads, host_stride, head_dim]
 *   y        host, fp32 [batch, n_q_heads, head_dim]
 *   n_threads  host threads to use (1 .. 64), the calling thread among them.  The others are worker
 *            threads the library starts on first use and keeps until the process ends (they sleep
 *            between calls, after polling for "host_spin_us" microseconds, see hca_tune); calls from
 *            several threads at once are served one after another.
 * Errors: HCA_ERR_CAPACITY if a value row lies outside host_stride. */
int32_t hca_attend_weights(const hca_shape* shape, const void* kcache, const void* q_f16, const int32_t* idx,
                           const int32_t* count, int32_t k, const int32_t* pos, float sm_scale, const float* lse_opt,
                           void* w_f16, int32_t* vrow, float* acc_opt, void* workspace, void* stream);
int32_t hca_host_weighted_sum(const hca_shape* shape, const int32_t* vrow, const int32_t* count, int32_t k,
                              const void* w_f16, const void* v_host, int64_t host_stride, float* y,
                              int32_t n_threads);

/* ---- Codebook form of the key path ---------------------------------------------------------
 * The paper's own compressor: grouped vector quantisation (Sec. 3.1) and table-lookup scores
 * (Sec. 3.2, Eq. 3).  The head dimension is cut into g groups of dbar = head_dim / g channels, a
 * token is stored as one centroid index per group (the matrix P), a query is first turned into the
 * table T = qbar . C (one entry per group and centroid) and the score of a token is the sum over
 * the groups of the table entries its indices select.  Top-k (hca_topk), the value gather
 * (hca_gather_values) and eviction decisions are those of the uniform-code path and are called
 * with the same hca_shape; its bits / group fields are not used by the hca_vq_* calls.
 *
 * Supported: head_dim 128, g in {32, 64}, 1 <= c <= 8192, in two storage forms chosen by the codebook's
 * shape.  Narrow (c <= 256 and g * c * n_q_heads/n_kv_heads <= 32768): indices are bytes and the whole
 * table of a KV head (<= 128 KiB) sits in the LDS of the compute unit that scans it.  Wide (anything
 * else, up to the paper's own c = 8192 of Fig. 4 / Table 4a): 16-bit indices, the table (up to 4 MiB per
 * KV head) passes through LDS a slice of groups at a time, once per tile of 16 Ki tokens.
 *
 * Arithmetic (the same on the oracle's side, so that indices, tables and scores match bit for bit):
 *   distance  d = 0; channels of the group ascending: e = x - c; d = fmaf(e, e, d); nearest = smallest d,
 *             ties to the lowest index
 *   table     t = 0; channels ascending: t = fmaf(q, c, t)
 *   score     the sum of Eq. 3 is exact: per query head s = 23 - floor(log2(max |T|)) (0 if T is all zero),
 *             Tfx = (int) rintf(ldexpf(T, s)), z = ldexpf((float) sum_i Tfx[i, P_i], -s); selection score =
 *             max over the KV head's query heads.  A table with a NaN or an infinity is an input error
 *             (not detected).
 * Layouts: centroids fp32 [n_kv_heads, g, c, dbar] (row (b, h) uses the codebook of KV head h);
 * pcache, narrow: uint8 [batch, n_kv_heads, capacity, g], the g index bytes of a slot in a slot-dependent
 * order: byte p of slot j holds the index of group 16 * (p / 16) + (p + j) % 16 (hca_vq_export_pcache undoes
 * it); wide: uint16 [batch, n_kv_heads, ceil(capacity / 16384), g, 16384] - tiles of 16 Ki slots, inside a
 * tile the indices of one group side by side (the scan takes the groups a few at a time);
 * lut: fp32 T [batch, n_kv_heads, c, g, n_q_heads/n_kv_heads] (wide form: [batch, n_kv_heads, g, c, ...]),
 * then fp32 [batch, n_kv_heads, g, 4], the
 * largest |T| per group and query head, then int32 [batch, n_kv_heads, 4], the exponents s of the row's
 * query heads. */
typedef struct {
  int32_t groups;             /* g */
  int32_t codewords;          /* c */
  const float* centroids;     /* device */
} hca_vq_codebook;

size_t hca_vq_pcache_bytes(const hca_shape* shape, const hca_vq_codebook* cb);
size_t hca_vq_lut_bytes(const hca_shape* shape, const hca_vq_codebook* cb);
/* Size of the `workspace` argument of the hca_vq_* calls (and of hca_topk, hca_topp, hca_gather_values used with
 * them): hca_workspace_bytes of the same shape with bits = 4, group = 32, whatever those fields hold. */
size_t hca_vq_workspace_bytes(const hca_shape* shape, const hca_vq_codebook* cb, int64_t k_max, int64_t m_max);

/* Offline codebook training on the host (Sec. 3.1): Lloyd's k-means per group over the sub-vectors
 * of a validation set.  Host pointers only, no device work, blocks until done.
 * The paper trains with mini-batch k-means (Sec. 4.1, implementation details); this is the full-batch
 * form - every round assigns all n_val sub-vectors and then moves every centroid to the mean of its
 * members - with the seeds handed in by the caller, so that a second implementation reproduces the
 * codebook bit for bit.  Any codebook of the same shape, however trained, can be given to the other
 * hca_vq_* calls.
 *   kval_f16   host, fp16 [n_val, head_dim]
 *   init       host, int32: shared == 0: [g, c] validation tokens whose sub-vectors seed group i's
 *              centroids; shared != 0: [c] entries of the pool of all g * n_val sub-vectors (entry
 *              t * g + i is sub-vector i of token t), one codebook trained on the pool and copied to
 *              every group
 *   iters      assignment + mean-update rounds; a centroid without members keeps its place
 *   centroids  host out, fp32 [g, c, dbar]
 *   inertia_opt host out, double [iters + 1] or NULL: k-means objective at each round's assignment and
 *              after the last update
 * Errors: HCA_ERR_BAD_ARG on bad sizes or seeds out of range. */
int32_t hca_vq_train(const void* kval_f16, int64_t n_val, int32_t head_dim, int32_t groups, int32_t codewords,
                     const int32_t* init, int32_t iters, int32_t shared, float* centroids, double* inertia_opt);

/* Appends T tokens per row: nearest-centroid index of every group (Sec. 3.2, the matrix P).
 * k_new_f16, n_resident, acc_opt, pos_opt, value_row0: as in hca_quantize_keys.
 * Errors: HCA_ERR_CAPACITY if n_resident + T exceeds the capacity. */
int32_t hca_vq_assign(const hca_shape* shape, const hca_vq_codebook* cb, void* pcache, const void* k_new_f16,
                      int64_t T, const int64_t* n_resident, float* acc_opt, int32_t* pos_opt,
                      const int64_t* value_row0, void* stream);

/* Test / debug: the index rows in canonical order.
 *   indices  device, [batch, n_kv_heads, capacity, g], uint8 for the narrow form and uint16 for the wide one:
 *            indices[.., j, i] = index of group i of slot j, slots >= n_resident untouched */
int32_t hca_vq_export_pcache(const hca_shape* shape, const hca_vq_codebook* cb, const void* pcache,
                             const int64_t* n_resident, void* indices, void* stream);

/* Builds the table of every query head into `lut` (device, hca_vq_lut_bytes; kept for
 * hca_vq_attend_gathered), then scores every resident token (Eq. 3).
 *   sel    device, fp32 [batch, n_kv_heads, capacity]: max over the KV head's query heads; slots
 *          >= n_resident are left untouched
 *   z_opt  device, fp32 [batch, n_q_heads, capacity] or NULL */
int32_t hca_vq_score(const hca_shape* shape, const hca_vq_codebook* cb, const void* pcache, const void* q_f16,
                     const int64_t* n_resident, float* lut, float* sel, float* z_opt, void* stream);

/* As hca_attend_gathered, with the logits of the selected tokens read from `lut` (Eq. 3) instead of
 * recomputed from uniform codes: softmax over the selected set, weighted sum of the value rows that
 * hca_gather_values left in `workspace`, optional accumulated-score update. */
int32_t hca_vq_attend_gathered(const hca_shape* shape, const hca_vq_codebook* cb, const void* pcache,
                               const float* lut, const int32_t* idx, const int32_t* count, int32_t k,
                               float sm_scale, float* y, float* acc_opt, void* workspace, void* stream);

/* hca_evict for a codebook cache: the same keep-set (newest n_protect slots, then the M - n_protect
 * highest accumulated scores, ties to the lower slot) and the same stable compaction, applied to the
 * index rows of pcache together with acc and pos.  In place (all three *_dst NULL) or into a second
 * buffer set (all three given, distinct from the sources; rows with n_resident <= M are carried over
 * unchanged).  workspace: hca_vq_workspace_bytes(shape, cb, k, M).  Afterwards n_resident = min(n_resident, M).
 * Errors: HCA_ERR_CAPACITY if M < 1, M > capacity or n_protect > M. */
int32_t hca_vq_evict(const hca_shape* shape, const hca_vq_codebook* cb, void* pcache, float* acc, int32_t* pos,
                     const int64_t* n_resident, int64_t M, int64_t n_protect, int32_t* kept_opt, void* workspace,
                     void* pcache_dst, float* acc_dst, int32_t* pos_dst, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HCA_H_ */
