/*
 * difa.h -- C ABI of the head-wise MMDiT joint-attention library for AMD MI355X (gfx950).
 *
 * The operator is the fused multi-strategy attention of DiTFastAttnV2, Sec. 3.3: in one
 * call every head of a layer independently runs
 *   - full attention                                   (DIFA_HEAD_FULL),
 *   - arrow attention with its own window, Sec. 3.1    (DIFA_HEAD_ARROW): the language-to-
 *     anything and visual-to-language quadrants are kept whole and the visual-to-visual
 *     quadrant keeps the band |i - j| <= w of the flattened image sequence, or
 *   - output caching, Sec. 3.2                         (DIFA_HEAD_CACHE): attention is skipped
 *     and the head's output of the previous denoising step is reused
 *     (the cache-fill statement that ends Alg. 1).
 *
 * Conventions: N = n_text + n_img tokens, text tokens first ([0, n_text)), image tokens
 * after them in flattened row-major order.  Tensors are dense [batch, heads, N, head_dim]
 * (DIFA_LAYOUT_BHND) or [batch, N, heads, head_dim] (DIFA_LAYOUT_BNHD), head_dim contiguous.
 *
 * Plain C99: no C++ types, no HIP headers needed by callers.  No entry point throws or
 * aborts; every failure is a return code and launches nothing.
 */
#ifndef DIFA_H
#define DIFA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct difa_plan difa_plan_t; /* opaque */

typedef enum {
    DIFA_OK = 0,
    DIFA_ERR_INVALID_ARG = 1, /* NULL pointer, bad mode/window/size, missing cache        */
    DIFA_ERR_UNSUPPORTED = 2, /* head_dim, dtype, layout or device the library cannot run */
    DIFA_ERR_ALLOC = 3,       /* host or device allocation failed                         */
    DIFA_ERR_HIP = 4          /* a HIP runtime call failed; text in difa_last_error()     */
} difa_status_t;

enum { DIFA_HEAD_FULL = 0, DIFA_HEAD_ARROW = 1, DIFA_HEAD_CACHE = 2,
       DIFA_HEAD_ARROW_RESIDUAL = 3 /* only with difa_joint_attention_residual, see there */ };
enum { DIFA_DTYPE_BF16 = 0, DIFA_DTYPE_F32 = 1 }; /* F32 = slow all-fp32 debug path */
enum { DIFA_LAYOUT_BHND = 0, DIFA_LAYOUT_BNHD = 1 };
/* Plan flags.  DIFA_FLAG_BLOCK_BAND selects the block-granular band of the paper's own kernel
 * (Sec. 3.3, Fig. 4: a block that mixes kept and discarded pairs is computed as a dense block, so
 * that only the sequence tail needs masking): an ARROW head then attends to every pair of a (query
 * tile, key tile) block of difa_tile_shape() rows x keys that holds at least one pair of the exact
 * arrow pattern.  Without the flag the band is exact, pair by pair.
 * DIFA_FLAG_IMAGE_FIRST: the joint sequence is [n_img image tokens, n_text text tokens] instead of
 * [text, image] (the paper says "concatenated" without naming an order, Sec. 2.1 / 3.1; public
 * MMDiT pipelines use both).  The operator is the same: text queries see every key, image queries
 * see the text keys and the image keys within the band. */
enum { DIFA_FLAG_BLOCK_BAND = 1u, DIFA_FLAG_IMAGE_FIRST = 2u };

/* Static description of a layer's attention call; fixed for the life of a plan object. */
typedef struct {
    int32_t batch;         /* B >= 1; the per-head plan is shared by all batch entries      */
    int32_t heads;         /* H >= 1                                                       */
    int32_t head_dim;      /* 64 or 128                                                    */
    int32_t dtype;         /* DIFA_DTYPE_*: element type of q, k, v, out and cache         */
    int32_t layout;        /* DIFA_LAYOUT_*                                                */
    int32_t max_tokens;    /* upper bound on n_text + n_img of any later call (>= 1)       */
    float   softmax_scale; /* 0 selects 1/sqrt(head_dim)                                   */
    int32_t device;        /* HIP device ordinal                                           */
    uint32_t flags;        /* DIFA_FLAG_* bits; unknown bits are rejected                   */
} difa_plan_desc_t;

/*
 * Create the per-layer plan object (Sec. 3.3: the operator is driven by a per-head plan;
 * Sec. 3.4.2: the plan is indexed by timestep, layer and head -- one object serves one layer
 * shape and is fed that layer's per-step head plan on every call).
 *   desc      HOST pointer, read during the call only.
 *   plan_out  HOST pointer; receives the object.  The object owns small device and pinned
 *             host buffers (compiled work lists), sized from desc->max_tokens.
 * Errors: INVALID_ARG (NULL, sizes < 1, unknown flag bits), UNSUPPORTED (head_dim not 64/128,
 * unknown dtype/layout, device is not gfx950), ALLOC, HIP.  On error *plan_out is NULL.
 */
difa_status_t difa_plan_create(const difa_plan_desc_t* desc, difa_plan_t** plan_out);

/*
 * One fused head-wise joint-attention call (Sec. 3.3; in Alg. 1, the head-wise attention call
 * under the chosen plan together with the cache fill that follows it).
 *   q, k, v    DEVICE, read-only, shape/layout/dtype of the plan, N = n_text + n_img.
 *   out        DEVICE, same shape; every row of every head is written.  Must not alias q/k/v.
 *   cache      DEVICE, same shape: the layer's output of the previous denoising step.  Read
 *              only for CACHE heads, whose rows are copied bit for bit.  May be NULL iff no
 *              head is CACHE.  cache == out is allowed (CACHE heads are then left untouched).
 *   head_plan  HOST, int32[heads], DIFA_HEAD_* per head.
 *   n_text, n_img  token counts (>= 0, sum in [1, max_tokens]).
 *   window     HOST, int32[heads], half-width w >= 0 of each ARROW head (an image query i
 *              sees image keys j with |i - j| <= w); ignored for other heads; may be NULL iff
 *              no head is ARROW.  w >= n_img - 1 makes the head identical to FULL.
 *   stream     hipStream_t passed as void*; NULL is the default stream.
 * The call enqueues one kernel launch on `stream` (two on the fp32 debug path when a head is cached)
 * and returns without waiting for it; host arrays may be freed on return.  Device tensors stay owned
 * by the caller and must stay valid until the stream has run the work.  Calls on one plan object
 * must not be issued from two threads at once; calls that name different streams are kept in the
 * order they were made (the later stream waits for an event on the earlier one), because they share
 * the object's buffers.  A call with a (head plan, windows, n_text, n_img) combination the object has
 * not seen lately compiles its work list on the host and uploads it from one of 16 pinned buffers
 * used in turn; the host waits only if the upload issued from that buffer 16 such calls earlier has
 * not been carried out yet (the queue is that deep).
 * Errors: INVALID_ARG; UNSUPPORTED when, for bf16, one head's K/V rows span 2 GiB or more in the
 * plan's layout (32-bit byte offsets inside a head); ALLOC (host memory); HIP.  On error no kernel has
 * been launched and `out` is untouched (an upload into the object's own buffers may have been queued).
 */
difa_status_t difa_joint_attention(difa_plan_t* plan, const void* q, const void* k, const void* v,
                                   void* out, const void* cache, const int32_t* head_plan,
                                   int32_t n_text, int32_t n_img, const int32_t* window,
                                   void* stream);

/*
 * The same operator for callers that cannot allocate device memory or let a library do so on their
 * behalf while they run: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Arguments, result, asynchrony and errors are those of difa_joint_attention.  The only
 * difference: the partial results of work records that the schedule cuts into pieces are kept in a
 * device array that is part of the library's code object (68 157 440 bytes per GPU, there from the
 * moment the library is loaded until the process ends) instead of the plan object's own buffer.  The
 * call makes no hipMalloc / hipFree and calls no allocating library routine.
 * Limit: a call whose schedule needs more than the array holds -- pieces * 256 rows * (head_dim + 2)
 * floats; 512 pieces at head_dim 128, which covers every schedule for a GPU of up to 256 compute
 * units -- fails with DIFA_ERR_UNSUPPORTED and a message naming both sizes.
 * Every call of this entry point on one GPU uses the same array, whatever the plan object or stream:
 * two such calls that overlap in time on one GPU race and produce wrong rows; the caller orders them
 * (one stream, or events).  Calls of difa_joint_attention are not affected by it.
 */
difa_status_t difa_joint_attention_static(difa_plan_t* plan, const void* q, const void* k, const void* v,
                                          void* out, const void* cache, const int32_t* head_plan,
                                          int32_t n_text, int32_t n_img, const int32_t* window,
                                          void* stream);

/*
 * Arrow attention with residual sharing, the optional method the paper keeps from its predecessor (Sec. 2.4;
 * evaluated in Sec. 4.6.1 and Table 4; the technique itself is defined in the predecessor's paper, so the
 * reading is this library's): at a refresh step a head runs full attention and arrow attention and keeps the
 * difference of the two outputs,
 *     r = O_full - O_arrow                  (difa_residual_store; rounded once, to the element type);
 * at the following steps it runs arrow attention only and adds the kept difference before the result is
 * rounded,
 *     O = ArrowAttention(Q, K, V; w) + r    (a head in mode DIFA_HEAD_ARROW_RESIDUAL).
 *
 * difa_joint_attention_residual is difa_joint_attention with one more tensor:
 *   residual   DEVICE, shape/layout/dtype of `out`, read-only, read only for DIFA_HEAD_ARROW_RESIDUAL heads
 *              (their window comes from `window` as for ARROW heads).  May be NULL iff no head has that mode.
 *              Must not alias `out`.
 * Everything else -- arguments, asynchrony, errors -- as difa_joint_attention, which itself rejects the
 * mode with INVALID_ARG.
 *
 * difa_residual_store writes residual[e] = o_full[e] - o_arrow[e] for every element of the plan's tensor
 * shape with n_tokens tokens (all heads; a caller that shares the residual of some heads only ignores the
 * rest).  The three tensors are DEVICE, 16-byte aligned, of the plan's dtype; `residual` may alias neither
 * input.  Asynchronous on `stream`.  Returns DIFA_OK, INVALID_ARG or HIP.
 */
difa_status_t difa_joint_attention_residual(difa_plan_t* plan, const void* q, const void* k, const void* v,
                                            void* out, const void* cache, const void* residual,
                                            const int32_t* head_plan, int32_t n_text, int32_t n_img,
                                            const int32_t* window, void* stream);
difa_status_t difa_residual_store(difa_plan_t* plan, const void* o_full, const void* o_arrow, void* residual,
                                  int32_t n_tokens, void* stream);

/* Release the object and its buffers (waits for the device to finish work that uses them).
 * NULL is a no-op that returns DIFA_OK.  (This call and the two below manage the object and report
 * errors; they correspond to no passage of the paper.) */
difa_status_t difa_plan_destroy(difa_plan_t* plan);

/* Static text for a status code. */
const char* difa_status_string(difa_status_t status);

/* Text of the last failure on this plan (owned by the plan, valid until its next call);
 * with plan == NULL, the text of the last failed difa_plan_create in this thread. */
const char* difa_last_error(const difa_plan_t* plan);

/* ------------------------------------------------------------------ host-side work list
 * Sec. 4.5 names the per-thread-block determination of the arrow pattern as the overhead
 * that shows at high sparsity.  Here that determination is done once on the host: the head
 * plan is compiled into one record per (batch entry, computed head, query tile) that lists
 * the key tiles the tile must visit, so that masked tiles are never loaded and in-tile masks
 * are applied only where a band edge, the text/image boundary or the sequence end crosses a
 * tile.  Exposed so that it can be checked without a GPU.
 *
 * Key tiles are named by their position in an order that starts with the tiles holding text keys:
 * position u is key tile (u + rot) % n_kv_tiles, n_kv_tiles = ceil(N / bn), where rot = 0 when the
 * text comes first and rot = n_img / bn with DIFA_FLAG_IMAGE_FIRST (when both kinds of token are
 * present).  The ranges below are ranges of positions.
 */
typedef struct {
    int32_t bh;        /* batch * heads + head                                            */
    int32_t q_tile;    /* query rows [q_tile*bm, min(N, (q_tile+1)*bm)); < 0: padding     */
    int32_t kv0_end;   /* first key-tile range  [0, kv0_end)          (text keys, or all) */
    int32_t nm0_end;   /*   tiles [0, nm0_end) of it need no in-tile mask                 */
    int32_t kv1_begin; /* second key-tile range [kv1_begin, kv1_end)  (band), >= kv0_end  */
    int32_t kv1_end;
    int32_t nm1_begin; /*   tiles [nm1_begin, nm1_end) of it need no in-tile mask         */
    int32_t nm1_end;
    int32_t window;    /* half-width for an ARROW head, -1 for a FULL head                */
    int32_t n_tiles;   /* number of key tiles visited (the record's cost)                 */
    int32_t flags;     /* DIFA_ITEM_ADD_RESIDUAL: the head's kept difference is added     */
} difa_work_item_t;
enum { DIFA_ITEM_ADD_RESIDUAL = 1 };

/* Tile shape (query rows bm, keys bn) the kernels use for a head_dim/dtype; 0 on success. */
int32_t difa_tile_shape(int32_t head_dim, int32_t dtype, int32_t* bm, int32_t* bn);

/*
 * Compile a head plan into work items (HOST only, no GPU needed).
 *   n_xcd           1: records ordered most-key-tiles-first.  > 1: the list is laid out for a GPU
 *                   whose workgroup p runs on accelerator die p % n_xcd (each with its own L2):
 *                   n_xcd interleaved queues of equal total cost, heads kept together on a die,
 *                   short queues padded with records whose q_tile is -1.
 *   flags           DIFA_FLAG_BLOCK_BAND: ARROW records visit the same key tiles but carry window -1 and
 *                   need the in-tile mask on the sequence tail only.  DIFA_FLAG_IMAGE_FIRST: see above.
 *   items/capacity  HOST array to fill (may be NULL with capacity 0 to only count).
 *   n_items_out     number of records, padding included (written also when capacity is short).
 *   copy_heads/n_copy_out  optional: int32[heads] receiving the indices of CACHE heads.
 * Returns DIFA_OK, INVALID_ARG (bad mode/window/sizes) or ALLOC (capacity too small; nothing
 * useful in items).
 */
difa_status_t difa_worklist_build(int32_t batch, int32_t heads, const int32_t* head_plan,
                                  const int32_t* window, int32_t n_text, int32_t n_img,
                                  int32_t bm, int32_t bn, int32_t n_xcd, uint32_t flags, difa_work_item_t* items,
                                  int32_t capacity, int32_t* n_items_out, int32_t* copy_heads,
                                  int32_t* n_copy_out);

/* ------------------------------------------------------------------ host-side schedule
 * The attention kernel is persistent: it is launched with one workgroup per compute unit, and each
 * workgroup walks its own list of segments.  A segment is a work record restricted to a range of the
 * positions of its visiting order (position p = the p-th key tile the record visits: the tiles of
 * the first range, then those of the second).  Most segments are whole records; to give every
 * compute unit the same amount of work, some records are cut into several segments that different
 * workgroups execute, each leaving an unnormalised partial result (fp32 O, row reference, row sum)
 * in a scratch slot; the workgroup that finishes its piece last folds the other pieces' slots into
 * its own result and writes the record's rows.
 */
typedef struct {
    int32_t bh, q_tile;          /* as in the record                                                  */
    int32_t kv0_end, nm0_end, kv1_begin, kv1_end, nm1_begin, nm1_end, window;
    int32_t pos_begin, pos_end;  /* positions [pos_begin, pos_end) of the record's visiting order      */
    int32_t part_slot;           /* -1: the segment is the whole record and writes `out`; otherwise
                                    the scratch slot that receives the partial result                 */
    int32_t merge_idx;           /* index of the record's difa_merge_item_t, -1 for a whole record     */
    int32_t n_parts;             /* number of pieces the record was cut into (1 for a whole record)    */
    int32_t first_slot;          /* scratch slot of the record's first piece (its pieces use consecutive
                                    slots), -1 for a whole record                                      */
    int32_t flags;               /* DIFA_ITEM_* bits of the record; the record is 64 bytes              */
} difa_segment_t;

typedef struct {
    int32_t bh, q_tile;          /* the record whose rows are merged                                   */
    int32_t first_slot, n_parts; /* its partial results sit in slots first_slot .. first_slot+n_parts-1 */
} difa_merge_item_t;

/*
 * Distribute records over n_wg workgroups (HOST only, no GPU needed).
 *   items/n_items   records as difa_worklist_build(..., n_xcd = 1, ...) returns them (any order; records
 *                   with q_tile < 0 are ignored).
 *   n_wg, n_xcd     number of workgroups and of accelerator dies; workgroup p runs on die p % n_xcd.
 *                   n_wg must be a multiple of n_xcd.  Heads are kept on one die (two where a cut between
 *                   dies falls inside a head) so that a head's K and V stay in that die's L2.
 *   segs/seg_capacity      receives the segments, grouped by workgroup; wg_begin[n_wg + 1] receives each
 *                          workgroup's first index into segs (wg_begin[n_wg] = number of segments).
 *   merges/merge_capacity  receives one entry per record that was cut.
 *   n_slots_out     number of scratch slots used (at most 2 * n_wg).
 * Returns DIFA_OK, INVALID_ARG, or ALLOC when a capacity is too small.
 */
difa_status_t difa_schedule_build(const difa_work_item_t* items, int32_t n_items, int32_t n_wg, int32_t n_xcd,
                                  difa_segment_t* segs, int32_t seg_capacity, int32_t* wg_begin,
                                  int32_t* n_segs_out, difa_merge_item_t* merges, int32_t merge_capacity,
                                  int32_t* n_merges_out, int32_t* n_slots_out);

/* ------------------------------------------------------------------ calibration helper
 * The influence of a method on each head, as the plan search measures it (Sec. 3.4.1, Eq. 1; Alg. 1:
 * Influence[h, m] = RSE(O[h], O'[h])):
 *     rse_out[h] = sum (y_m - y_o)^2 / sum (y_o - mean(y_o))^2,
 * every sum over all elements head h owns: batch entries, tokens, features.  (The printed Eq. 1 has
 * the mean of y_o in the numerator as well; the numerator is read as the error against y_o, which
 * is what makes a perfect method score 0.)
 *   y_m, y_o   device, 16-byte aligned, laid out like `out` of difa_joint_attention for the plan's batch,
 *              heads, head_dim, dtype and layout, with n_tokens (<= max_tokens) tokens: the output of the
 *              method under test and the original output.  Read-only.
 *   rse_out    device, heads fp32 values, written by this call.  If y_o is constant over a head the
 *              value is +inf (or NaN when the error is zero too).
 * Asynchronous on `stream`; allocates nothing (the plan object owns a scratch for partial sums, so
 * calls on one object from different streams are ordered by an event).  fp32 arithmetic inside one
 * 16-byte vector, fp64 across vectors: the result is within 1e-5 relative of exact arithmetic.
 * Returns DIFA_OK, INVALID_ARG or HIP.
 */
difa_status_t difa_head_rse(difa_plan_t* plan, const void* y_m, const void* y_o, int32_t n_tokens,
                            float* rse_out, void* stream);

/* Head-wise plan selection for one layer (Sec. 3.4.2, Eq. 2), host only, exact:
 *     minimise   sum_h ( latency_full + sum_m X[h,m] * (latency[m] - latency_full) )
 *     subject to sum_h sum_m X[h,m] * influence[h,m] <= delta,
 *                X[h,m] = 1 only if influence[h,m] <= (c / heads) * delta,
 *                sum_m X[h,m] <= 1,  X binary.
 * (The printed objective lists the method latencies only; a head without a method is priced at
 * latency_full here, without which the minimum would be "choose nothing".)
 *   influence   host, heads x n_methods, row-major, >= 0: the values difa_head_rse produced per method.
 *               +inf is accepted (such a method is never chosen for that head); NaN is rejected.
 *   latency     host, n_methods finite values >= 0; latency_full finite, >= 0: cost of one head under
 *               each method.
 *   choice_out  host, heads entries: the method index chosen for each head, -1 = full attention.
 *   total_latency_out, total_influence_out  host, may be NULL.
 * Among several optimal assignments one is returned.  Returns DIFA_OK, INVALID_ARG (NULL pointers,
 * negative or NaN values, infinite latencies), ALLOC, or UNSUPPORTED when the search frontier outgrows 2^20 entries.
 */
difa_status_t difa_plan_solve(const double* influence, const double* latency, double latency_full,
                              int32_t heads, int32_t n_methods, double delta, double c,
                              int32_t* choice_out, double* total_latency_out, double* total_influence_out);

/* ------------------------------------------------------------------ measurement hooks
 * With timing enabled the library brackets its kernel launches with HIP events on the caller's
 * stream; difa_plan_timing_read waits for the last bracket and returns the accumulated kernel
 * milliseconds and launch count since the last reset.  attn_ms: the call's layer kernel (on the bf16 path it
 * holds the cached-head copy as well; a bf16 layer with every head cached is one launch of the copy kernel,
 * counted here); copy_ms: the separate copy kernel of the fp32 debug path.
 */
difa_status_t difa_plan_timing_enable(difa_plan_t* plan, int32_t enable);
difa_status_t difa_plan_timing_read(difa_plan_t* plan, double* attn_ms, double* copy_ms,
                                    int64_t* launches, int32_t reset);
/* The same for difa_head_rse: accumulated milliseconds of its two kernels and the number of calls. */
difa_status_t difa_plan_timing_read_head_rse(difa_plan_t* plan, double* rse_ms, int64_t* launches, int32_t reset);
/*
 * What the plan object has learnt about the accelerator dies.  Under load the dies of one GPU settle at
 * clocks a few percent apart; the bf16 kernel reports how long each workgroup ran, the object averages the
 * dies' relative speeds from the reports of finished launches, and a layer's schedule exists in two versions:
 * dies alike, or work in proportion to the speeds.  The version made first runs until three launches of it
 * have been timed, then the other one, then the faster of the two stays (so a memoised schedule is made
 * again at most twice in its life).  No call waits for a report: a call uses what has arrived by then.
 *   speeds     HOST array of `capacity` doubles: receives the relative speeds (mean 1), one per die.
 *   n_dies     number of dies the scheduler distinguishes (1: the mechanism is off).
 *   samples    launches whose reports went into the running average (a new plan object starts from what
 *              earlier ones on the same device have learnt, counted as three); below three every die counts
 *              as 1.0.
 *   retunes    memoised schedules made again so far.
 * Returns INVALID_ARG for a NULL plan or too small a capacity.  Lifecycle/diagnostic call: it matches no
 * passage of the paper.
 */
difa_status_t difa_plan_die_speeds(difa_plan_t* plan, double* speeds, int32_t capacity, int32_t* n_dies,
                                   int32_t* samples, int32_t* retunes);

/* What the runtime reports for a device: number of compute units, peak engine and memory clocks (kHz), L2
 * size of one accelerator die (bytes), architecture name.  Any output pointer may be NULL.  For a
 * benchmark's report; not part of the operator.  Returns DIFA_OK, INVALID_ARG (no such device) or HIP. */
difa_status_t difa_device_info(int32_t device, int32_t* compute_units, int32_t* clock_khz,
                               int32_t* memory_clock_khz, int32_t* l2_bytes, char* arch, int32_t arch_len);

/* The rate at which the current device sustains dense bf16 MFMA (v_mfma_f32_32x32x16_bf16, the
 * instruction both contractions of the operator use) on the caller's operand data: a kernel of
 * nothing but independent MFMAs on every compute unit, timed with HIP events on `stream`.  The
 * published peak assumes the full clock; for how long a GPU holds it depends on the operand bits
 * (it is power-limited on N(0,1) data), so a benchmark can report this beside the operator's rate.
 * Not part of the operator.
 *   data            device pointer, 16-byte aligned, n_elems bf16 values (>= 8) the operands are taken from.
 *   waves_per_simd  1 or 2 wavefronts per SIMD.
 *   rounds          64 MFMAs per wavefront each, in [1, 2^22]; 50 000 rounds take about 50 ms.
 *   scratch4        device pointer to 4 writable bytes (never written in practice).
 *   tflops_out, ms_out (ms_out may be NULL)  host.
 * Synchronises the stream.  Returns DIFA_OK, INVALID_ARG or HIP.
 */
difa_status_t difa_probe_mfma_rate(const void* data, int64_t n_elems, int32_t waves_per_simd, int32_t rounds,
                                   void* scratch4, void* stream, double* tflops_out, double* ms_out);

#ifdef __cplusplus
}
#endif
#endif /* DIFA_H */
