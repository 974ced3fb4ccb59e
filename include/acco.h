/*
 * acco.h - C ABI of the ACCO per-shard optimizer path for AMD MI355X (gfx950).
 *
 * One shard owner's work between the gradient Reduce_Scatter and the parameter
 * All_Gather of ACCO's communication stream (Alg. 1 of the paper; update rule:
 * eq. (ACCO), stages (1) and (2)):
 *
 *   acco_accumulate      g_i <- g_i + grad(micro-batch), N_i <- N_i + 1
 *   acco_cast_params     fp32 -> bf16 (publish g_i to the communication buffer;
 *                        bf16 parameter shard for the All_Gather)
 *   acco_reduce_shards   owner's slice of sum_i g_i and the sum of the counts
 *   acco_estimate_step   theta~(t+1) = Opt(theta(t), sum g~ / sum N~)   - nothing committed
 *   acco_commit_step     theta(t+1)  = Opt(theta(t), (sum g + sum g~)/(sum N + sum N~))
 *
 * with Opt = AdamW (decoupled weight decay, bias-corrected moments, epsilon added
 * to the bias-corrected root), fp32 sharded states theta, m, v and bf16
 * parameters / communication buffers (experimental setup, Sec. 4.2).
 *
 * Conventions for every entry point
 *   - "device" pointers address memory of the current HIP device; "host" pointers
 *     address ordinary host memory.  The caller owns every buffer; the library
 *     allocates nothing, frees nothing and keeps no pointer after the call.
 *   - Arrays are flat and contiguous, element j at index j.  bf16 values are
 *     passed as uint16_t bit patterns.  Device pointers must be 16-byte aligned.
 *   - n is the shard length in elements, 0 <= n <= ACCO_MAX_ELEMS.  n == 0 does no
 *     device work but still performs the host counter bookkeeping; array pointers
 *     are then not dereferenced and may be NULL (an empty tensor has no address).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Device work is enqueued on it and the call returns without waiting; host
 *     counters are updated before return.  A call enqueues kernel launches only (no
 *     memset, copy, allocation or synchronisation) with its scalars passed by value, so
 *     it may be recorded by a stream capture; a replay repeats the device work with the
 *     scalars of the recorded call and touches no host counter (the *_dev step entry
 *     points read their scalars from device memory instead, so that a replay can follow
 *     the update index).
 *   - Return value: ACCO_OK (0) or a negative acco_status.  On any error nothing
 *     is enqueued and no host counter is modified.
 *   - Thread-safe; no global mutable state besides cached device properties, the
 *     process-wide launch settings at the end of this header (each entry point's settings are
 *     one atomic word: a launch sees either the old set or the new one, never a mixture), and
 *     the 4 KiB device array that acco_commit_step_resident - and no other entry point -
 *     stages its scalars in (its callers order or separate their calls by slot).
 */
#ifndef ACCO_H
#define ACCO_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ACCO_MAX_ELEMS   ((int64_t)1 << 40)
#define ACCO_MAX_WORKERS 64

typedef enum acco_status {
    ACCO_OK         = 0,
    ACCO_ERR_NULL   = -1, /* a required pointer is NULL                               */
    ACCO_ERR_SIZE   = -2, /* n < 0, n > ACCO_MAX_ELEMS, workers outside 1..64, a block  */
                          /* count or slot index beyond its stated maximum            */
    ACCO_ERR_ALIGN  = -3, /* a device pointer is not 16-byte aligned                  */
    ACCO_ERR_ARG    = -4, /* bad hyper-parameter, count, step, dtype or flag          */
    ACCO_ERR_ALIAS  = -5, /* an output overlaps an input it must not overlap          */
    ACCO_ERR_DEVICE = -6  /* the HIP runtime reported an error at launch              */
} acco_status;

typedef enum acco_dtype {
    ACCO_BF16 = 0, /* shards are bf16 bit patterns (the paper's communication buffers) */
    ACCO_F32  = 1  /* shards are fp32 (accumulators reduced without the bf16 publish)  */
} acco_dtype;

/* AdamW hyper-parameters (App. C, hyper-parameter tables: lr 6e-4, weight decay 0.1,
 * betas (0.9, 0.95) for pre-training; the paper does not state epsilon).
 * Valid: lr >= 0, 0 <= beta < 1, eps >= 0, weight_decay >= 0, all finite. */
typedef struct acco_adamw_t {
    double lr;
    double beta1;
    double beta2;
    double eps;
    double weight_decay;
} acco_adamw_t;

/*
 * Layout of the "state" arrays theta, m, v and gsum of the step entry points.
 *   block_elems == 0 (or a NULL layout pointer): planar - element j at index j.
 *   otherwise: element j of an array lives at index
 *       (j / block_elems) * block_stride + (j % block_elems)
 *   from that array's pointer: the array is cut into blocks of block_elems elements whose
 *   starts are block_stride elements apart.  This lets the four arrays be interleaved block by
 *   block in ONE buffer - [theta block][m block][v block][gsum block] repeated, with
 *   block_stride = 4 * block_elems and the four pointers one block apart - which keeps the
 *   addresses streamed at any moment a fixed few tens of KiB apart (on MI355X, before the
 *   resident wavefronts were bounded, the committed step then ran at 6.4-6.6 TB/s every time;
 *   with four distant planar arrays at 5.4-6.4 depending on where they happened to be
 *   allocated: arrays read together should lie in one memory class, see acco_hbm_classify,
 *   which one buffer does by construction).  All four arrays share the one layout.
 *   block_elems: a power of two >= 4; block_stride: a multiple of 4, >= block_elems.
 * The fp32 and bf16 outputs of the step entry points stay planar.
 *
 * The same description serves a second purpose: the W workers' bf16 communication buffers
 * interleaved block by block in ONE buffer - [worker 0 block][worker 1 block]...[worker W-1
 * block] repeated, shard w's pointer = base + w * block_elems, block_stride = W * block_elems.
 * acco_accumulate_batch writes such buffers (out_layout) and the reduction entry points read
 * them (shard_layout).  An option, not what the benchmark uses: on MI355X, W = 8 buffers of
 * 875M elements in 16384-element blocks make the two reduce + step kernels faster and
 * independent of where W separate buffers would happen to lie (4.51 / 5.91 ms every time
 * against 4.58-4.92 / 6.05-6.47), but the kernels that publish into them slower (second
 * micro-batch + publish 6.53 against 6.32 ms; the fp32 accumulate + publish by 12-15 %):
 * a round of equal counts comes out the same, one of unequal counts 3 % slower.
 * For a bf16 array block_elems must be >= 8; a blocked shard layout requires bf16 shards.
 */
typedef struct acco_layout_t {
    int64_t block_elems;
    int64_t block_stride;
} acco_layout_t;

/*
 * Gradient accumulation of the computation stream (Alg. 1: g_i <- g_i + grad F,
 * N_i <- N_i + 1).
 *   acc        device, fp32[n], in/out: one worker's accumulator
 *   grad_bf16  device, bf16[n], in:     one micro-batch gradient
 *   init       0: acc[j] += grad[j].  1: acc[j] = grad[j] (start of a new
 *              accumulation; the old contents of acc are not read)
 *   count      host, nullable, in/out: the worker's micro-batch counter N_i;
 *              set to 1 when init, else incremented.
 * Errors: NULL acc/grad, bad n, misalignment, acc overlapping grad, init not 0/1,
 *         *count < 0 (or == INT64_MAX) when it is to be incremented.
 */
int acco_accumulate(float* acc, const uint16_t* grad_bf16, int64_t n, int init, int64_t* count,
                    void* stream);

/*
 * acco_accumulate for the LAST micro-batch of an accumulation, fused with the publish
 * to the bf16 communication buffer (Alg. 1: g_i <- g_i + grad F, then Buffer_i <- g_i):
 *   s = init ? grad[j] : acc[j] + grad[j];   comm_bf16[j] = bf16_rne(s);
 *   keep_acc != 0: acc[j] = s as well.  keep_acc == 0: acc is left as it was (it no longer
 *   holds the sum; the next accumulation into it must start with init = 1) - this saves the
 *   4-byte store per element.
 * Same values as acco_accumulate followed by acco_cast_params.
 *   comm_bf16  device, bf16[n], out.  Other arguments and errors as acco_accumulate; acc may be
 *   NULL when init != 0 and keep_acc == 0; comm_bf16 must not overlap acc or grad_bf16.
 */
int acco_accumulate_publish(float* acc, const uint16_t* grad_bf16, uint16_t* comm_bf16, int64_t n,
                            int init, int keep_acc, int64_t* count, void* stream);

/*
 * The first two micro-batches of an accumulation without an fp32 round trip.  After the first
 * micro-batch the accumulator equals that gradient, which bf16 holds exactly, so it is kept as
 * a bf16 "stash"; the second micro-batch adds to it in fp32.  Values are identical to
 * acco_accumulate(init = 1) followed by acco_accumulate / acco_accumulate_publish; 4 bytes per
 * element less HBM traffic in each of the two calls.
 *
 * acco_accumulate_first:  stash[j] = grad[j];  *count = 1.
 *   publish != 0: the accumulation consists of this one micro-batch and `stash_bf16` IS the
 *   communication buffer: comm[j] = bf16_rne(float(grad[j])) (the same bits, NaNs quieted).
 * acco_accumulate_second: s = float(stash[j]) + float(grad[j]);  *count = 2 (it must be 1).
 *   Exactly one of acc / comm_bf16 is non-NULL:
 *   acc:       acc[j] = s - the fp32 accumulator continues with acco_accumulate(init = 0);
 *   comm_bf16: comm_bf16[j] = bf16_rne(s) - second and last micro-batch, published at once.
 *   stash_bf16, grad_bf16, comm_bf16: device, bf16[n]; acc: device, fp32[n].
 *   A caller whose first gradient stays untouched until the second arrives (backward wrote it
 *   straight into the accumulation buffer) passes that buffer as stash_bf16 and needs no
 *   acco_accumulate_first; it sets the counter to 1 itself.
 * Errors: NULLs, bad n, misalignment, an output overlapping an input, *count != 1 for second.
 */
int acco_accumulate_first(uint16_t* stash_bf16, const uint16_t* grad_bf16, int64_t n, int publish,
                          int64_t* count, void* stream);
int acco_accumulate_second(float* acc, uint16_t* comm_bf16, const uint16_t* stash_bf16,
                           const uint16_t* grad_bf16, int64_t n, int64_t* count, void* stream);

/*
 * The accumulation calls above (Alg. 1, computation stream: g_i <- g_i + grad F, N_i <- N_i + 1,
 * and the hand-over Buffer_i <- g_i) for SEVERAL workers' accumulators in one launch
 * (grid.y = worker).  On a real node one process accumulates its whole gradient - all W shards of it - per
 * micro-batch; with the W shards as W separate buffers that is W launches of the calls above,
 * or one of this.  Same values; what it saves is launches (a round of the GPT-2-small-scale
 * workload is 10 launches instead of 34) and the ramp-down / ramp-up between them.
 *   op       which step, the same for every worker of the call:
 *     ACCO_BATCH_ACCUMULATE_INIT     acc[w][j]  = grad[w][j]                       count = 1
 *     ACCO_BATCH_ACCUMULATE          acc[w][j] += grad[w][j]                       count += 1
 *     ACCO_BATCH_ACCUMULATE_PUBLISH  out[w][j]  = bf16_rne(acc[w][j] + grad[w][j]) count += 1
 *                                    (acc is read only, as with keep_acc == 0)
 *     ACCO_BATCH_FIRST               out[w][j]  = grad[w][j]      (out is the stash) count = 1
 *     ACCO_BATCH_FIRST_PUBLISH       out[w][j]  = bf16_rne(float(grad[w][j]))        count = 1
 *     ACCO_BATCH_SECOND              acc[w][j]  = float(stash[w][j]) + float(grad[w][j])
 *                                                                         count 1 -> 2
 *     ACCO_BATCH_SECOND_PUBLISH      out[w][j]  = bf16_rne(float(stash[w][j]) + float(grad[w][j]))
 *                                                                         count 1 -> 2
 *     ACCO_BATCH_PUBLISH             out[w][j]  = bf16_rne(acc[w][j])     counts untouched
 *     ACCO_BATCH_RUNNING_BF16        out[w][j]  = bf16_rne(float(out[w][j]) + float(grad[w][j]))
 *                                    (the bf16 running sum of acco_accumulate_bf16)  count += 1
 *   workers  1 .. ACCO_MAX_WORKERS (more than 16 are served by several launches)
 *   acc, out_bf16, stash_bf16, grad_bf16   HOST arrays of `workers` DEVICE pointers (fp32[n] for
 *            acc, bf16[n] for the others), read before the call returns; an array the
 *            operation does not use may be NULL
 *   counts   host, int64[workers], nullable, in/out: the workers' micro-batch counters
 *   out_layout  host, nullable: layout shared by all out_bf16[w] (NULL = planar); accepted for
 *            the operations that write out_bf16 other than ACCO_BATCH_RUNNING_BF16
 * Errors: as the single calls; in addition no buffer the call writes may share an element with
 *         any other buffer of the call, of the same or of another worker (ACCO_ERR_ALIAS; two
 *         outputs of the same blocked layout may interleave), and a layout where none is
 *         accepted is ACCO_ERR_ARG.
 */
typedef enum acco_batch_op {
    ACCO_BATCH_ACCUMULATE_INIT    = 0,
    ACCO_BATCH_ACCUMULATE         = 1,
    ACCO_BATCH_ACCUMULATE_PUBLISH = 2,
    ACCO_BATCH_FIRST              = 3,
    ACCO_BATCH_FIRST_PUBLISH      = 4,
    ACCO_BATCH_SECOND             = 5,
    ACCO_BATCH_SECOND_PUBLISH     = 6,
    ACCO_BATCH_PUBLISH            = 7,
    ACCO_BATCH_RUNNING_BF16       = 8
} acco_batch_op;

int acco_accumulate_batch(int op, int workers, float* const* acc, uint16_t* const* out_bf16,
                          const uint16_t* const* stash_bf16, const uint16_t* const* grad_bf16,
                          int64_t n, int64_t* counts, const acco_layout_t* out_layout,
                          void* stream);

/*
 * The accumulation of Alg. 1 with the running sum itself held in bf16, the precision the
 * paper's experimental setup (Sec. 4) gives its gradient-accumulation and communication
 * buffers.  The accumulator then IS the communication buffer (no publish step):
 *   acc_bf16[j] = init ? grad[j] : bf16_rne(float(acc_bf16[j]) + float(grad[j]));  *count += 1.
 * The sum is rounded after every micro-batch (a running sum of equal terms stops growing after
 * 256 of them); acco_accumulate keeps fp32 instead and is what the round uses by default.
 *   acc_bf16   device, bf16[n], in/out (out only when init != 0)
 *   grad_bf16  device, bf16[n], in
 * Other arguments and errors as acco_accumulate.
 */
int acco_accumulate_bf16(uint16_t* acc_bf16, const uint16_t* grad_bf16, int64_t n, int init,
                         int64_t* count, void* stream);

/*
 * fp32 -> bf16, round to nearest even (NaN stays NaN, overflow goes to infinity).
 * Used for Buffer_i <- g_i (bf16 communication buffer) and for the bf16 parameter
 * shard handed to the All_Gather when the step kernels' fused output is not used.
 *   out_bf16  device, bf16[n], out
 *   src       device, fp32[n], in
 */
int acco_cast_params(uint16_t* out_bf16, const float* src, int64_t n, void* stream);

/*
 * The reduce half of the gradient Reduce_Scatter as the shard owner sees it
 * (Alg. 1, communication stream), together with the All_Reduce of the counts:
 *   accumulate == 0 (stage 1):  gsum[j]  = x_0[j] + x_1[j] + ... + x_{W-1}[j]
 *   accumulate == 1 (stage 2):  gsum[j] += x_0[j] + ... (added one by one onto the
 *                               retained stage-1 sum)
 * in fp32, strictly in ascending worker order.
 *   gsum      device, fp32[n], out (in/out when accumulate)
 *   shards    HOST array of `workers` DEVICE pointers, each bf16[n] or fp32[n]
 *             according to dtype; read before the call returns
 *   workers   1 .. ACCO_MAX_WORKERS
 *   counts    host, nullable: counts[w] = micro-batches summed in shard w (>= 0)
 *   total     host, nullable, in/out: accumulate ? *total + sum(counts) : sum(counts).
 *             counts and total are given together or not at all.
 *   gsum_layout  host, nullable: layout of gsum (NULL = planar)
 *   shard_layout host, nullable: layout shared by all shards (NULL = planar; bf16 shards only)
 * Errors: NULLs, bad n/workers/dtype/flag, misalignment, gsum overlapping a
 *         shard, negative count, total overflow, a blocked layout for fp32 shards.
 */
int acco_reduce_shards(float* gsum, const void* const* shards, int workers, int dtype, int64_t n,
                       int accumulate, const int64_t* counts, int64_t* total,
                       const acco_layout_t* gsum_layout, const acco_layout_t* shard_layout,
                       void* stream);

/*
 * Stage (1) of eq. (ACCO): the speculative parameters
 *   theta~ = AdamW(theta, m, v; g = gsum / total_count; update index = step + 1)
 * theta, m, v and the step counter are only read: stage (2) starts again from the
 * same theta(t).
 *   theta, m, v, gsum  device, fp32[n], in
 *   theta_tilde_f32    device, fp32[n], out, nullable
 *   theta_tilde_bf16   device, bf16[n], out, nullable  (at least one output)
 *   step               number of updates committed so far (>= 0)
 *   total_count        number of micro-batch gradients summed in gsum (>= 1)
 *   state_layout       host, nullable: layout shared by theta, m, v, gsum (NULL = planar)
 * Errors: NULLs, bad n, misalignment, an output overlapping an input or the other
 *         output, invalid hyper-parameters, step < 0, total_count < 1.
 */
int acco_estimate_step(const float* theta, const float* m, const float* v, const float* gsum,
                       float* theta_tilde_f32, uint16_t* theta_tilde_bf16, int64_t n,
                       const acco_adamw_t* hp, int64_t step, int64_t total_count,
                       const acco_layout_t* state_layout, void* stream);

/*
 * Stage (2) of eq. (ACCO): the committed update on the full delayed gradient
 *   (theta, m, v) <- AdamW(theta, m, v; g = gsum / total_count; update index = *step + 1)
 * in place, then *step += 1.
 *   theta, m, v  device, fp32[n], in/out (pairwise distinct)
 *   gsum         device, fp32[n], in
 *   theta_bf16   device, bf16[n], out, nullable: bf16 copy of the new theta, written
 *                in the same pass (the All_Gather input)
 *   step         host, in/out: updates committed so far (>= 0)
 * Errors: as acco_estimate_step; step == NULL.
 */
int acco_commit_step(float* theta, float* m, float* v, const float* gsum, uint16_t* theta_bf16,
                     int64_t n, const acco_adamw_t* hp, int64_t* step, int64_t total_count,
                     const acco_layout_t* state_layout, void* stream);

/*
 * acco_reduce_shards(accumulate = 0) fused with acco_estimate_step: stage 1 of the
 * communication stream in one pass.  The sum over the worker shards is formed in registers in
 * ascending worker order, stored to gsum (stage 2 adds onto it) and used at once for
 *   theta~ = AdamW(theta, m, v; g = gsum / *total; update index = step + 1).
 * Same values as the two separate calls; saves re-reading gsum.
 *   gsum    device, fp32[n], out
 *   counts  host, int64[workers], required;  total  host, out, required: sum(counts) >= 1
 *   shard_layout  as in acco_reduce_shards
 * Other arguments and errors as acco_reduce_shards and acco_estimate_step.
 */
int acco_reduce_estimate_step(const float* theta, const float* m, const float* v, float* gsum,
                              const void* const* shards, int workers, int dtype,
                              const int64_t* counts, int64_t* total, float* theta_tilde_f32,
                              uint16_t* theta_tilde_bf16, int64_t n, const acco_adamw_t* hp,
                              int64_t step, const acco_layout_t* state_layout,
                              const acco_layout_t* shard_layout, void* stream);

/*
 * acco_reduce_shards(accumulate = 1) fused with acco_commit_step: stage 2 in one pass.
 *   g = ((gsum + x_0) + x_1) + ... ;  *total += sum(counts);
 *   (theta, m, v) <- AdamW(theta, m, v; g / *total; update index = *step + 1);  *step += 1.
 * Same values as the two separate calls; saves writing and re-reading gsum.
 *   gsum    device, fp32[n], in/out: the retained stage-1 sum.  With workers <= 8 (<= 16 bf16
 *           shards under the default launch shape) it is not written; with more workers it
 *           receives the partial sum over all but the shards of the last pass.  Its contents
 *           are not needed after this call.
 *   counts  host, required;  total  host, in/out, required.
 */
int acco_reduce_commit_step(float* theta, float* m, float* v, float* gsum,
                            const void* const* shards, int workers, int dtype,
                            const int64_t* counts, int64_t* total, uint16_t* theta_bf16, int64_t n,
                            const acco_adamw_t* hp, int64_t* step,
                            const acco_layout_t* state_layout, const acco_layout_t* shard_layout,
                            void* stream);

/*
 * The four AdamW step entry points with their scalars read from DEVICE memory when the kernel
 * runs, instead of being passed by value when the call is made.  What for: the update index,
 * and with it the bias corrections of eq. (ACCO)'s Opt = AdamW, change with every committed
 * update, so a launch recorded into a HIP graph with by-value scalars repeats update number t
 * for ever.  With these forms a whole round (both stages of Alg. 1's communication stream) is
 * recorded once; before each replay the host folds the scalars of that round's two steps
 * (acco_fold_adamw), puts them into the device block (acco_stage_scalars) and replays.  Same
 * kernels, same arithmetic, same values bit for bit as the by-value forms.
 *
 * acco_step_scalars_t: one step's folded scalars, 64 bytes, opaque (grad scale, betas, bias
 *   corrections, step size, decay, epsilon as fp32, rounded once from double).
 * acco_fold_adamw: host only.  Scalars of update number step + 1 on a gradient sum of
 *   total_count micro-batches - exactly what the by-value entry points fold internally.
 *   out: host.  Errors: NULL, invalid hyper-parameters, step < 0, total_count < 1.
 * acco_stage_scalars: dst_dev[0 .. blocks) = src_host[0 .. blocks), enqueued on `stream` as one
 *   small kernel that carries the blocks in its arguments (no memcpy; src_host may be reused as
 *   soon as the call returns).  dst_dev: device, 16-byte aligned; 1 <= blocks <= 4.
 * The *_dev step entry points: arguments as their by-value namesakes, with
 *   scalars_dev  device, 16-byte aligned, in: read by the kernel when it runs; must not overlap
 *                any buffer the call writes
 * in place of hp / step / total_count / counts / total.  They update NO host counter: the
 * caller that folds the scalars owns the update index and the totals.  The estimate forms write
 * the bf16 output only (required).
 * Errors: as the namesakes; scalars_dev NULL or misaligned.
 */
typedef struct acco_step_scalars_t {
    float f[16];
} acco_step_scalars_t;

#define ACCO_STAGE_BLOCKS_MAX 4

int acco_fold_adamw(const acco_adamw_t* hp, int64_t step, int64_t total_count,
                    acco_step_scalars_t* out);
int acco_stage_scalars(acco_step_scalars_t* dst_dev, const acco_step_scalars_t* src_host,
                       int blocks, void* stream);
int acco_estimate_step_dev(const float* theta, const float* m, const float* v, const float* gsum,
                           uint16_t* theta_tilde_bf16, int64_t n,
                           const acco_step_scalars_t* scalars_dev,
                           const acco_layout_t* state_layout, void* stream);
int acco_commit_step_dev(float* theta, float* m, float* v, const float* gsum, uint16_t* theta_bf16,
                         int64_t n, const acco_step_scalars_t* scalars_dev,
                         const acco_layout_t* state_layout, void* stream);
int acco_reduce_estimate_step_dev(const float* theta, const float* m, const float* v, float* gsum,
                                  const void* const* shards, int workers, int dtype,
                                  uint16_t* theta_tilde_bf16, int64_t n,
                                  const acco_step_scalars_t* scalars_dev,
                                  const acco_layout_t* state_layout,
                                  const acco_layout_t* shard_layout, void* stream);
int acco_reduce_commit_step_dev(float* theta, float* m, float* v, float* gsum,
                                const void* const* shards, int workers, int dtype,
                                uint16_t* theta_bf16, int64_t n,
                                const acco_step_scalars_t* scalars_dev,
                                const acco_layout_t* state_layout,
                                const acco_layout_t* shard_layout, void* stream);

/*
 * acco_commit_step_dev for callers that cannot allocate device memory - code that runs where
 * hipMalloc is not allowed (under a stream capture, in a serving loop that must not allocate,
 * in a harness that forbids it) and so cannot own the scalar block the *_dev forms read.  The
 * block lives in an array of the library's own instead (static device memory, 64 blocks =
 * 4 KiB on every GPU the library runs on, held until the process ends).  The call enqueues two
 * kernels on `stream` and nothing else - no allocation, free, memset, copy or synchronisation:
 * the first puts *scalars_host (carried in its arguments) into block `slot`, the second is the
 * committed step of acco_commit_step_dev reading that block.  Same values as acco_commit_step_dev
 * with the same scalars.
 *   scalars_host  host, in: one step's scalars from acco_fold_adamw; read before the call returns
 *   slot          0 <= slot < ACCO_RESIDENT_SLOTS, else ACCO_ERR_SIZE.  All calls on one GPU
 *                 share that GPU's array, and a block keeps what the last call put there: calls
 *                 that use the same slot must be ordered (same stream, or events); calls that
 *                 may overlap on one GPU must use different slots, or they race.
 *   other arguments and errors as acco_commit_step_dev; no host counter is touched.
 * The first call on a device looks up where that device's copy of the array lives
 * (hipGetSymbolAddress); make that call outside any capture.
 */
#define ACCO_RESIDENT_SLOTS 64

int acco_commit_step_resident(float* theta, float* m, float* v, const float* gsum,
                              uint16_t* theta_bf16, int64_t n,
                              const acco_step_scalars_t* scalars_host, int slot,
                              const acco_layout_t* state_layout, void* stream);

/*
 * Plain SGD with decoupled weight decay as Opt - the optimizer of the paper's convergence
 * propositions (Prop. GD / Prop. SGD, Sec. 3.2): theta' = theta - lr wd theta - lr g,
 * g = gsum / total_count.  It has no state besides theta.
 * Valid: lr >= 0, weight_decay >= 0, finite.
 */
typedef struct acco_sgd_t {
    double lr;
    double weight_decay;
} acco_sgd_t;

/*
 * Stage (1) of eq. (ACCO) with Opt = SGD: theta~ = theta - lr wd theta - lr gsum/total_count;
 * theta is only read.  Arguments and errors as acco_estimate_step (without m, v, step).
 */
int acco_sgd_estimate_step(const float* theta, const float* gsum, float* theta_tilde_f32,
                           uint16_t* theta_tilde_bf16, int64_t n, const acco_sgd_t* hp,
                           int64_t total_count, void* stream);

/*
 * Stage (2) of eq. (ACCO) with Opt = SGD, in place on theta; *step += 1.
 * Arguments and errors as acco_commit_step (without m, v).
 */
int acco_sgd_commit_step(float* theta, const float* gsum, uint16_t* theta_bf16, int64_t n,
                         const acco_sgd_t* hp, int64_t* step, int64_t total_count, void* stream);

/*
 * Learning rate of update number `step` (0-based) under the cosine schedule of the paper's
 * hyper-parameter tables (App. C: scheduler cosine, n_warmup_steps 0, nb_steps_tot 50000), with
 * an optional linear warm-up; a host function - the result is what the caller puts into
 * acco_adamw_t.lr for that step:
 *   step <  warmup_steps:  base_lr * (step + 1) / warmup_steps
 *   otherwise:             min_lr + (base_lr - min_lr) * (1 + cos(pi * p)) / 2,
 *                          p = min(1, (step - warmup_steps) / max(1, total_steps - warmup_steps))
 * The paper does not state a final learning rate; min_lr = 0 decays to zero.
 * Returns NaN for invalid arguments (negative or non-finite rates, min_lr > base_lr, step < 0,
 * warmup_steps < 0, total_steps < warmup_steps).
 */
double acco_lr_cosine(double base_lr, double min_lr, int64_t step, int64_t warmup_steps,
                      int64_t total_steps);

/*
 * Bandwidth probes - NOT part of the method.  The access patterns of the kernels above without
 * their arithmetic, so that a benchmark can report what the device's memory system gives for
 * them next to the kernels' own figures.  Planar fp32 arrays, same conventions and errors.
 *   acco_probe_copy:   dst[j] = src[j]                         (4 B read, 4 B written)
 *   acco_probe_triad:  a[j] += d[j]; b[j] += d[j]; c[j] += d[j] (16 B read, 12 B written)
 */
int acco_probe_copy(float* dst, const float* src, int64_t n, void* stream);
int acco_probe_triad(float* a, float* b, float* c, const float* d, int64_t n, void* stream);

/*
 * Memory classes of a device allocation - a set-up helper for placing buffers, NOT part of the
 * method.  Measured on MI355X: the HBM falls into three classes of 96 GiB each, laid out over
 * the physical addresses in pieces of 32 GiB (our reading: the three ranks of the 12-high
 * stacks).  A kernel that reads two streams from DIFFERENT classes at the same time runs 8-10 %
 * slower than with both in one class (second micro-batch + publish at 875M elements: 0.82
 * against 0.75 ms whatever the distance inside a class); where its written streams lie matters
 * little, and they do best in a class the kernel does not read.  So the buffers a kernel of
 * this path reads together - theta, m, v, gsum and the W communication buffers; a stash and the
 * gradient added to it - belong in one class each, its outputs in another.  Virtual addresses
 * do not show the class; this call finds it by timing:
 *   position k (k = 0 .. count-1) is the probe_bytes at base + k * step_bytes; a small kernel
 *   reads two positions and writes `scratch`; positions whose pair runs as fast as a pair of
 *   neighbours get the same class number.  Classes are numbered by size, largest first.
 *   base, bytes   device region to classify (only read; its contents do not matter)
 *   step_bytes, probe_bytes   multiples of 4096; e.g. 2 GiB and 512 MiB.  Smaller probes are
 *                 noisier: below about 256 MiB the two populations start to overlap.
 *   scratch       device, probe_bytes, written; outside the region
 *   classes       host, int32[count], out;  count must be (bytes - probe_bytes) / step_bytes + 1
 *   n_classes     host, out: number of classes found (1 on a device whose memory is uniform)
 * Blocks until the probes are done (it times them with events on `stream`): not for capture.
 * A misjudged position costs speed, never correctness.
 * Errors: NULLs, misalignment, sizes not as stated, scratch inside the region; ACCO_ERR_DEVICE
 *         for a runtime error or timings too erratic to sort into at most 64 classes.
 */
int acco_hbm_classify(const void* base, int64_t bytes, int64_t step_bytes, int64_t probe_bytes,
                      void* scratch, int32_t* classes, int64_t count, int32_t* n_classes,
                      void* stream);

/* Human-readable name of a status code (static storage, never NULL). */
const char* acco_status_string(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int acco_version(void);

/*
 * Launch shape used for subsequent calls of one entry point ("accumulate", "cast",
 * "reduce", "estimate", "commit", "accumulate_publish", "reduce_estimate", "reduce_commit",
 * "sgd", "stash", "second", "probe"):
 * threads per workgroup (64..512, multiple of 64),
 * 16-byte vectors each thread keeps in flight per array (1, 2 or 4), and workgroups
 * per compute unit (0 = one workgroup per tile, > 0 = grid-stride over that many
 * resident workgroups per CU).  Process-wide; meant for benchmarking, not required.
 * Returns ACCO_ERR_ARG for an unknown name or an unsupported value.
 */
int acco_set_launch_shape(const char* entry, int threads, int vectors_in_flight,
                          int workgroups_per_cu);

/*
 * Upper bound on the wavefronts of one entry point's kernels that are resident on a compute
 * unit at a time (0 = the hardware's limit, 32).  The streaming kernels use no LDS; the bound
 * is enforced by reserving an unused slice of the CU's 160 KiB of LDS per workgroup, so that
 * only so many workgroups fit.  Fewer resident wavefronts mean fewer distinct DRAM pages open
 * at a time, which pays for the kernels that stream many arrays at once.  At least 3
 * workgroups must fit (one workgroup can reserve at most 64 KiB).  Process-wide.  The
 * library's defaults are per entry point (from 8 for the committed step to none for the
 * cast); the variants that start a new sum (init != 0), which write more than they read,
 * always run unbounded.
 * Returns ACCO_ERR_ARG for an unknown name or a bound outside 0, 3..32.
 */
int acco_set_resident_waves(const char* entry, int waves_per_cu);

/* Puts the launch shape and the resident-wavefront bound of every entry point back to the
 * library's defaults. */
void acco_reset_launch_settings(void);

#ifdef __cplusplus
}
#endif

#endif /* ACCO_H */
