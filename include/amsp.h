/*
 * amsp.h: C ABI of the per-GPU model-state step of a ZeRO-style data-parallel rank.
 *
 * One rank owns a contiguous flat shard of the model states: bf16 parameters P, bf16
 * gradients G and the fp32 optimizer states OS (master copy, first and second Adam
 * moments): 2 + 2 + 12 bytes per parameter (Section II-C, "ZeRO"; Section IV-D).  Between
 * "the partial gradients have arrived" and "the updated bf16 shard is ready to ship" the
 * rank does, on its Phi/s elements (Section IV-C.2):
 *
 *   1. reduce      sum the k partial bf16 gradient buffers in fp32: the arithmetic half of
 *                  the ReduceScatter / AllReduce-then-select of Sections II-C and IV-C;
 *   2. sqnorm      squared L2 norm of the reduced gradient, for global-norm clipping
 *                  (not in the paper; the usual rule  scale = min(1, c/(||g|| + clip_eps)));
 *   3. AdamW       update fp32 master/m/v in place (Adam under mixed precision, Section II-C);
 *   4. cast        round the updated master to bf16: the payload the AllGather / Broadcast of
 *                  Section IV-C.2 ships.
 *
 * amsp_adamw_step_shard fuses 1 + 3 + 4 in one streaming pass (2k + 26 bytes per element).
 *
 * Conventions, for every function below
 *   - Returns an int status: AMSP_OK (0) or a negative AMSP_E* code.  Never throws or aborts,
 *     never allocates, frees or copies device memory and never waits for the device (the two
 *     host-only helpers amsp_partition_tensors and amsp_plan_sharding use a little host memory
 *     of their own).  Arguments are checked before anything is enqueued: on every error but
 *     AMSP_EDEVICE nothing has been enqueued and outputs are untouched.  AMSP_EDEVICE (a launch
 *     the runtime refused) may come after earlier launches of the same call went out (calls that
 *     take several launches: buckets, segment lists, the norm's finishing pass), so the outputs
 *     are then undefined.
 *   - The library keeps no state between calls and reads no environment variables; launch shapes
 *     are compile-time constants.  (amsp_grad_sqnorm_static alone writes to a buffer of the
 *     library's own; see there.)
 *   - "device" pointers are HIP device memory valid on the current device; "host" pointers
 *     are ordinary host memory read during the call only.  The caller owns every buffer.
 *   - Every data pointer addresses the FIRST element of the range to process (the caller
 *     applies its shard or bucket offset); element i of every buffer is the same model-state
 *     element.  Buffers must not overlap, except that master/m/v are updated in place.
 *   - Pointers need only natural alignment (2 B bf16, 4 B fp32, 8 B double).  When all
 *     streams of a call reach the alignment of their vector access (8 or 16 bytes) at the
 *     same element index, as they do when every buffer is offset by the same number of
 *     elements from a 16-byte boundary, the kernels use vector accesses; otherwise a slower
 *     element-wise path gives the same results.  Fastest is every buffer at the same element
 *     offset from a 1 KiB boundary (as separately allocated buffers are): the leading elements
 *     up to the first such boundary (at most 255) are then done one by one and every wave's
 *     accesses are aligned to their own size.
 *   - Where the buffers lie matters for speed, not for results.  Large device allocations start on
 *     2 MiB boundaries, which puts element i of every stream at the same offset modulo 8 KiB; on
 *     MI355X a wave's accesses to the 2k + 7 streams then wait on each other in the memory system
 *     and the fused step runs 4-6 % slower for k = 8 and 16.  Shifting the streams' bases against
 *     each other by an odd multiple of 4 KiB (stream j at allocation base + j * 4 KiB: still aligned
 *     to 1 KiB) avoids it; multiples of 8 KiB do not.  The kernels cannot do this for the caller.
 *   - bf16 values are passed as uint16_t bit patterns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is
 *     enqueued and the call returns without waiting; amsp_shard_range alone is synchronous.
 *   - `bucket_elems` (Section IV-C.2: gradients are synchronised in buckets of size U; here
 *     counted in elements): 0 processes [0,n) in one launch; U > 0 processes the buckets
 *     [bU, min((b+1)U, n)) in order, each bucket a range of its own with its own ragged head
 *     and tail; buckets of one call may share a launch.
 *   - n is not limited by the launch size: a range (or a bucket) of more than 2^33 elements is cut
 *     on the host into consecutive launches of at most 2^25 workgroups (2^33 elements) each.
 *   - n == 0 is valid: AMSP_OK, nothing launched (amsp_grad_sqnorm still writes 0 when
 *     accumulate == 0).
 *   - The reduction order over j = 0..k-1 is fixed and fp32, identical in every entry point,
 *     so the gradient seen by the norm, the separate reduce and the fused step is bitwise
 *     the same.  All results are deterministic run to run.
 */
#ifndef AMSP_H
#define AMSP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    AMSP_OK = 0,
    AMSP_EINVAL = -1,     /* bad k / shard factor / rank / hyper-parameter */
    AMSP_ENULL = -2,      /* a required pointer is NULL */
    AMSP_EALIGN = -3,     /* a pointer is not aligned to its element size */
    AMSP_EWORKSPACE = -4, /* workspace smaller than the entry point's requirement */
    AMSP_EDEVICE = -5,    /* a HIP call failed */
    AMSP_ENOPLAN = -6,    /* amsp_plan_sharding: no sharding fits the memory limit and the table */
    AMSP_ESIZE = -7       /* amsp_grad_sqnorm_static: n above AMSP_STATIC_MAX_ELEMS */
};

#define AMSP_MAX_K 32u

/* Static description of a status code; never NULL. */
const char *amsp_status_string(int status);

/* Bytes of device workspace amsp_grad_sqnorm needs (a fixed, small number). */
size_t amsp_workspace_bytes(void);

/*
 * Rank `rank`'s range [*begin, *end) of a flat buffer of `total_elems` elements split evenly
 * over `shard_factor` ranks (Section IV-B: sharding factor s, 1 = Full-Replica; Section IV-C.2:
 * each GPU updates Phi/s_os parameters, split evenly).  The first total_elems % shard_factor
 * ranks get one element more; ranges are contiguous, disjoint and cover [0, total_elems).
 * Host only, pure.  begin/end: host, written on success.
 * Errors: AMSP_EINVAL if shard_factor == 0 or rank >= shard_factor; AMSP_ENULL.
 */
int amsp_shard_range(uint64_t total_elems, uint32_t shard_factor, uint32_t rank,
                     uint64_t *begin, uint64_t *end);

/*
 * Step 1 alone: grad_out[i] (=|+=) sum_{j<k} partials[j][i], in fp32, j ascending: the arithmetic
 * half of the ReduceScatter / AllReduce-then-select of Sections II-C and IV-C.
 *   partials    host array of k device pointers, each bf16[n]
 *   k           1..AMSP_MAX_K
 *   grad_out    device fp32[n]
 *   accumulate  0: overwrite; 1: add the sum to what grad_out holds (gradient accumulation
 *               over micro-batches, Section IV-C.3)
 * Errors: AMSP_EINVAL (k == 0, k > AMSP_MAX_K), AMSP_ENULL, AMSP_EALIGN, AMSP_EDEVICE.
 */
int amsp_reduce_grad_shard(const uint16_t *const *partials, uint32_t k, uint64_t n,
                           uint64_t bucket_elems, float *grad_out, int accumulate, void *stream);

/*
 * Steps 1 and 2 in one pass, for callers that keep the fp32 gradient anyway (gradient accumulation
 * over micro-batches, Section IV-C.3): as amsp_reduce_grad_shard, and
 * *d_sqnorm (=|+=) sum_i grad_out[i]^2 of the values just written (after `accumulate`), in fp64 in a
 * fixed order, the buckets added in bucket order.  The update then reads 4 bytes per element of
 * gradient (amsp_adamw_step_shard with k = 0) instead of re-reading the 2k of the partials.
 *   d_sqnorm           device double, required
 *   sqnorm_accumulate  0: overwrite; 1: add to the value already there
 *   workspace          device, >= amsp_reduce_workspace_bytes(n, bucket_elems) (about n/256 doubles:
 *                      the block sums of every bucket side by side, added once after the last
 *                      bucket), 8-byte aligned; no initialisation needed, clobbered
 * Errors: as amsp_reduce_grad_shard, and AMSP_EWORKSPACE.
 */
size_t amsp_reduce_workspace_bytes(uint64_t n, uint64_t bucket_elems);
int amsp_reduce_grad_sqnorm_shard(const uint16_t *const *partials, uint32_t k, uint64_t n,
                                  uint64_t bucket_elems, float *grad_out, int accumulate,
                                  double *d_sqnorm, int sqnorm_accumulate,
                                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * Step 2: *d_sqnorm (=|+=) sum_i g[i]^2 with g the reduced gradient, accumulated in fp64 in a
 * fixed order.  The cross-rank sum of these scalars (one 8-byte all-reduce) is the caller's.
 *   k >= 1      g is recomputed from `partials` exactly as in step 1 (grad_f32 ignored)
 *   k == 0      g is read from grad_f32, device fp32[n] (partials ignored)
 *   d_sqnorm    device double, written when the enqueued work completes
 *   accumulate  0: overwrite; 1: add to the value already there
 *   The order of the additions is fixed by (n, bucket_elems, the pointers' alignment, the number of
 *   compute units): the same call gives the same bits every time.
 *   workspace   device, >= amsp_workspace_bytes(), 8-byte aligned; contents need no
 *               initialisation and are clobbered; calls sharing a workspace must be ordered
 *               on one stream
 */
int amsp_grad_sqnorm(const uint16_t *const *partials, uint32_t k, const float *grad_f32,
                     uint64_t n, uint64_t bucket_elems, double *d_sqnorm, int accumulate,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * amsp_grad_sqnorm for callers that cannot allocate or bring device memory of their own for it: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * meaning, kernels and bits as amsp_grad_sqnorm, without the workspace: the block sums go to a buffer
 * inside the library, a file-scope device array of 526,336 bytes (65,792 doubles) of which every GPU
 * the library runs on holds one copy until the process ends.  The call allocates and frees nothing.
 *   - n above AMSP_STATIC_MAX_ELEMS (2^34 elements) is refused with AMSP_ESIZE and a line on stderr
 *     before anything is enqueued; longer ranges go through amsp_grad_sqnorm.
 *   - Every call on a GPU shares that GPU's buffer: calls that overlap in time on one GPU (different
 *     streams, different threads) race on it and give undefined sums; order them on one stream.
 *     The buffer needs no clearing between calls (every sum is written before it is read); it keeps
 *     the previous call's contents.
 *   - The buffer's device address is looked up on the first call on each device (with that device
 *     current); make that first call outside any stream capture.
 * Errors: as amsp_grad_sqnorm, AMSP_ESIZE, and AMSP_EDEVICE if the address lookup fails.
 */
#define AMSP_STATIC_MAX_ELEMS (1ull << 34)
int amsp_grad_sqnorm_static(const uint16_t *const *partials, uint32_t k, const float *grad_f32,
                            uint64_t n, uint64_t bucket_elems, double *d_sqnorm, int accumulate,
                            void *stream);

/*
 * Hyper-parameters of one AdamW step.  With g' = scale * g:
 *   m <- beta1 m + (1 - beta1) g'
 *   v <- beta2 v + (1 - beta2) g'^2
 *   p <- p - lr ( (m / (1 - beta1^step)) / (sqrt(v / (1 - beta2^step)) + eps) + weight_decay p )
 * scale:
 *   d_total_sqnorm != NULL: read on the device when the kernel runs,
 *       scale = max_norm > 0 ? min(1, max_norm / (sqrt(*d_total_sqnorm) + clip_eps)) : 1
 *       (no host synchronisation between the norm pass and the update), times grad_scale;
 *   d_total_sqnorm == NULL: scale = grad_scale (max_norm and clip_eps unused).
 * grad_scale is where a caller folds 1/(number of micro-batches or ranks) or a loss scale.
 * The arithmetic is fp32, every operation correctly rounded once, in this order (fma = fused
 * multiply-add; 1 - beta and 1/(1 - beta^step) are formed in double on the host and rounded to fp32):
 *   gs = scale * g
 *   m  = fma(beta1, m, (1 - beta1) * gs)
 *   v  = fma(beta2, v, ((1 - beta2) * gs) * gs)
 *   u  = (m * (1/(1 - beta1^step))) / (sqrt(v * (1/(1 - beta2^step))) + eps)
 *   p  = fma(-lr, fma(weight_decay, p, u), p)
 * so results are reproducible bit for bit from the inputs on any implementation of these operations.
 */
typedef struct amsp_adamw_hparams {
    float lr;
    float beta1;
    float beta2;
    float eps;
    float weight_decay;
    uint32_t step;                /* t >= 1: index of the update being applied */
    float max_norm;               /* <= 0: no clipping */
    float clip_eps;               /* conventionally 1e-6 */
    const double *d_total_sqnorm; /* device, may be NULL */
    float grad_scale;             /* 1.0f for none */
} amsp_adamw_hparams;

/*
 * Steps 1 + 3 + 4 fused: one pass that reduces the partials, updates master/m/v in place and
 * writes the bf16 parameters.
 *   k >= 1          gradient = fp32 sum of `partials` (as step 1); grad_f32 ignored
 *   k == 0          gradient read from grad_f32, device fp32[n]
 *   master, exp_avg, exp_avg_sq   device fp32[n], read and written in place
 *   param_bf16_out  device bf16[n], or NULL to skip step 4
 *   hp              host, read during the call
 * Errors: AMSP_EINVAL for k > AMSP_MAX_K, step == 0, non-finite lr/beta/eps/weight_decay/
 * clip_eps/grad_scale, beta outside [0,1), eps < 0; AMSP_ENULL; AMSP_EALIGN; AMSP_EDEVICE.
 *
 * Which composition of a whole step (norm known before the update) moves fewer bytes:
 *   amsp_grad_sqnorm (2k) + this call with k >= 1 (2k + 26)                   4k + 26 bytes/element, no extra buffer
 *   amsp_reduce_grad_sqnorm_shard (2k + 4) + this call with k == 0 (30)       2k + 34 bytes/element, fp32 gradient buffer
 * The second is cheaper from k = 5 on (measured on MI355X, k = 8: 6.4 ms against 7.3 ms for 842 M elements;
 * k = 16: 8.5 against 11.2 ms) and is the natural form when gradients are accumulated over micro-batches;
 * the first needs no gradient buffer and wins for k <= 4.  Results are the same bits either way.
 */
int amsp_adamw_step_shard(const uint16_t *const *partials, uint32_t k, const float *grad_f32,
                          uint64_t n, uint64_t bucket_elems,
                          float *master, float *exp_avg, float *exp_avg_sq,
                          uint16_t *param_bf16_out, const amsp_adamw_hparams *hp, void *stream);

/*
 * Step 4 alone: param_bf16_out[i] = bf16(master[i]), round to nearest even on the bit pattern;
 * NaN -> quiet NaN with the sign kept (0x7FC0 | sign), +-Inf kept, finite overflow -> +-Inf,
 * subnormals rounded, not flushed.  master: device fp32[n]; param_bf16_out: device bf16[n].
 */
int amsp_cast_param_shard(const float *master, uint16_t *param_bf16_out, uint64_t n, void *stream);

/* ------------------------------------------------------------------------------------------------
 * Inter-tensor shards (Section IV-C.2, second scheme; the one the paper adopts): every parameter
 * tensor goes, whole, with its optimizer states, to one rank, by a greedy rule that balances the
 * ranks' memory; after the gradient AllReduce a rank "selects" the gradients of its own tensors
 * from the flat buffer and drops the rest (Sections IV-C.2 and IV-C.3).  A rank's shard is then a
 * list of segments of the flat whole-model buffer, and its optimizer states are stored compactly,
 * segment after segment.
 */
typedef struct amsp_segment {
    uint64_t flat_offset;  /* first element in the flat whole-model buffers (gradients, bf16 params) */
    uint64_t local_offset; /* first element in the rank's compact master / exp_avg / exp_avg_sq */
    uint64_t length;       /* elements */
} amsp_segment;

/*
 * Greedy assignment of num_tensors tensors (tensor_elems[i] elements each, in model order) to
 * shard_factor ranks: tensors are visited in order and each goes to the rank that holds the fewest
 * elements so far, the lowest such rank on a tie (the paper names only "a greedy algorithm to
 * balance GPU memory usage"; this is the reading taken).  Host only, pure.
 * owner: host out [num_tensors].  Errors: AMSP_EINVAL (shard_factor == 0), AMSP_ENULL.
 */
int amsp_partition_tensors(const uint64_t *tensor_elems, uint32_t num_tensors, uint32_t shard_factor,
                           uint32_t *owner);

/*
 * The segments of `rank` under `owner`: its tensors in model order, flat neighbours merged, local
 * offsets back to back.  segments: host out [capacity] or NULL to only count.  *num_segments and
 * *local_elems (the rank's shard size) are always written; AMSP_EINVAL if capacity is too small.
 */
int amsp_owned_segments(const uint64_t *tensor_elems, const uint32_t *owner, uint32_t num_tensors,
                        uint32_t rank, amsp_segment *segments, uint32_t capacity,
                        uint32_t *num_segments, uint64_t *local_elems);

/*
 * Step 1 over a segment list ("select" into the rank's compact gradient buffer): for every owned
 * segment, grad_f32_local[local_offset + i] (=|+=) sum_j partials_flat[j][flat_offset + i], as
 * amsp_reduce_grad_shard does for a flat range.  With accumulate = 1 over the micro-batches of a step
 * (Section IV-C.3) the buffer ends up holding the step's gradient of the rank's tensors; its squared
 * norm is then amsp_grad_sqnorm(k = 0) over the compact buffer, and the update the k = 0 form of
 * amsp_adamw_step_segments.
 */
int amsp_reduce_grad_segments(const uint16_t *const *partials_flat, uint32_t k, uint64_t flat_elems,
                              const amsp_segment *segments, uint32_t num_segments,
                              uint64_t local_elems, float *grad_f32_local, int accumulate, void *stream);

/*
 * Steps 2 and 1+3+4 over a segment list: as amsp_grad_sqnorm / amsp_adamw_step_shard ("select":
 * only owned elements are read; "drop": nothing else is touched).  Long segments get a launch of
 * their own; segments shorter than 2^20 elements share launches, 32 to a launch, and so do the
 * segments of the norm pass: a shard of thousands of small tensors is not bound by launches.
 *   partials_flat    host array of k device pointers, each bf16[flat_elems] (flat whole-model
 *                    gradient buffers: one all-reduced buffer, k = 1, or k partial ones)
 *   k, grad_f32_local  k >= 1: the gradient is summed from partials_flat (grad_f32_local ignored).
 *                    k == 0 (amsp_adamw_step_segments only): it is read from grad_f32_local, device
 *                    fp32[local_elems], laid out like the optimizer states (partials_flat ignored)
 *   segments         host array [num_segments]; each must lie inside [0, flat_elems) and
 *                    [0, local_elems), else AMSP_EINVAL and nothing is enqueued
 *   master_local ... device fp32[local_elems], updated in place
 *   param_bf16_flat  device bf16[flat_elems] or NULL: the updated parameters land at their flat
 *                    positions, ready for the per-tensor Broadcast of Section IV-C.2
 *   d_amax           device float[num_segments] or NULL.  Not NULL: d_amax[i] = max |p'| over segment i
 *                    of the parameters just written (as amsp_fp8_payload_segments computes it, taken
 *                    inside the update so that the FP8 payload needs no pass of its own for it);
 *                    entries of empty segments are 0
 *   amax_workspace   device, >= amsp_amax_workspace_bytes(num_segments), 4-byte aligned, used only
 *                    when d_amax != NULL (else may be NULL); no initialisation needed, clobbered
 * The squared norm is accumulated in segment order (accumulate = 0 overwrites first).
 */
int amsp_grad_sqnorm_segments(const uint16_t *const *partials_flat, uint32_t k, uint64_t flat_elems,
                              const amsp_segment *segments, uint32_t num_segments,
                              double *d_sqnorm, int accumulate,
                              void *workspace, size_t workspace_bytes, void *stream);
int amsp_adamw_step_segments(const uint16_t *const *partials_flat, uint32_t k,
                             const float *grad_f32_local, uint64_t flat_elems,
                             const amsp_segment *segments, uint32_t num_segments, uint64_t local_elems,
                             float *master_local, float *exp_avg_local, float *exp_avg_sq_local,
                             uint16_t *param_bf16_flat, float *d_amax, void *amax_workspace,
                             size_t amax_workspace_bytes, const amsp_adamw_hparams *hp, void *stream);
size_t amsp_amax_workspace_bytes(uint32_t num_segments);

/* ------------------------------------------------------------------------------------------------
 * FP8 payload with per-tensor scaling factors: Section IV-C.2 adopts inter-tensor shards because
 * each FP8 tensor travels with its own scale.  The paper fixes no format; this library ships OCP E4M3
 * (bias 7, 3 mantissa bits, subnormals, no infinities, largest finite 448, NaN = S.1111.111), rounds
 * to nearest even, saturates beyond +-448, and scales each tensor by 448 / max|p| (1 when that
 * maximum is 0 or not finite), the maximum, the scale and the product all in fp32.
 */

/* Step 4 as FP8: param_fp8_out[i] = e4m3(master[i] * *d_scale).  master: device fp32[n];
 * d_scale: device float; param_fp8_out: device uint8[n] (codes). */
int amsp_cast_param_fp8_shard(const float *master, uint64_t n, const float *d_scale,
                              uint8_t *param_fp8_out, void *stream);

/*
 * Per segment of a rank's compact master: d_amax[i] = max |master| over the segment (exact and
 * order-free: an integer maximum of the bit patterns; a NaN in the segment yields a NaN),
 * d_scale[i] = 448 / d_amax[i], and the segment's E4M3 codes written at its flat position.
 *   master_local    device fp32[local_elems]
 *   param_fp8_flat  device uint8[flat_elems]; only owned segments are written
 *   d_amax, d_scale device float[num_segments], written (the scales are what a receiver needs to
 *                   decode: value = code / scale)
 *   amax_ready      0: the maxima are computed here (one more read of the master).  1: d_amax already
 *                   holds them, as amsp_adamw_step_segments left them for this segment list
 * The maxima of 32 segments share a launch, and so do their codes, whatever the segments' lengths.
 * Codes are stored 16 bytes at a time when some element of the segment has its fp32 value on a
 * 16-byte boundary and its code on a 4-byte boundary (then that holds every 4 elements; offsets that
 * are multiples of 4 elements into 16-byte-aligned buffers give it), else byte by byte.
 * Errors as amsp_adamw_step_segments.
 */
int amsp_fp8_payload_segments(const float *master_local, uint64_t local_elems,
                              const amsp_segment *segments, uint32_t num_segments,
                              uint64_t flat_elems, uint8_t *param_fp8_flat,
                              float *d_amax, int amax_ready, float *d_scale, void *stream);

/* ------------------------------------------------------------------------------------------------
 * Sharding planner (Section V-B).  Chooses the device meshes s_p, s_g, s_os = (GPUs per node) x
 * (nodes) over which parameters, gradients and optimizer states are sharded: the feasible tuple of
 * least per-step communication time
 *     T_comm = T_p + T_g + T_os^0 + T_os^1                                   (Section IV-C)
 *     T_p    = M L sum_i ( 2 t(AG, 2 Phi_i, s_p) + t(RS, 2 Phi_i, s_p) )
 *     T_os^0 = 2 Phi / (U s_p) * t(AR, U, s_dp / s_p)
 *     T_os^1 = s_os / s_p * t(BC, 2 Phi / s_os, s_os / s_p)
 *     T_g    = (M - 1) 2 Phi / (U s_p) * t(AR, U, s_g / s_p)
 * with t(o, v, mesh) = v / w(o, v, mesh) from a profiled bandwidth table (Section IV-A; linear in v
 * between profiled sizes, end values outside; a one-GPU mesh costs 0), subject to
 *     2 Phi/s_p + 2 Phi/s_g + 12 Phi/s_os + activations + temporaries <= GPU memory   (Eq. 2, IV-D)
 *     1 <= s_p <= s_g <= s_os <= s_dp in each mesh dimension                          (Eq. 3, 4)
 *     every factor divides s_dp in its dimension                                      (Eq. 5, 6)
 *     a component spans nodes only once it spans the whole node                       (Eq. 7)
 *     s_g in {s_p, s_os}                                                              (Section IV-C.3)
 * and s_dp = gpus_per_node x nodes.  Where the paper is silent: a mesh missing from the table makes a
 * tuple unusable; ties go to the tuple that is first in lexicographic order of
 * (s_p^0, s_p^1, s_g^0, s_g^1, s_os^0, s_os^1).  Host only, pure; every pointer is host memory.
 */
enum { AMSP_OP_ALLGATHER = 0, AMSP_OP_REDUCESCATTER = 1, AMSP_OP_ALLREDUCE = 2, AMSP_OP_BROADCAST = 3 };

typedef struct amsp_bw_sample {   /* one profiled point: effective bandwidth of `op` on mesh p0 x p1 */
    uint32_t op, p0, p1;
    double bytes;                 /* message size v */
    double bytes_per_s;           /* w(op, v, p0 x p1) */
} amsp_bw_sample;

typedef struct amsp_plan_problem {
    double phi;                   /* parameters of the model */
    uint32_t layers;              /* L */
    uint32_t modules_per_layer;   /* K */
    const double *module_params;  /* Phi_i, host array [modules_per_layer] */
    uint32_t micro_batches;       /* M >= 1 */
    double bucket_bytes;          /* U > 0 */
    uint32_t gpus_per_node;       /* R = s_dp^0 */
    uint32_t nodes;               /* N = s_dp^1 */
    double gpu_memory_bytes, activation_bytes, tmp_bytes;
} amsp_plan_problem;

typedef struct amsp_plan {
    uint32_t sp0, sp1, sg0, sg1, sos0, sos1;
    double t_p, t_g, t_os0, t_os1, t_comm; /* seconds */
    double d_modelstate;                   /* bytes per GPU */
} amsp_plan;

/* best: host out.  feasible_count: host out or NULL, the number of tuples that passed every constraint
 * and could be priced.  Errors: AMSP_ENULL, AMSP_EINVAL (zero R, N, M, Phi or U), AMSP_ENOPLAN. */
int amsp_plan_sharding(const amsp_plan_problem *problem, const amsp_bw_sample *table, uint32_t rows,
                       amsp_plan *best, uint32_t *feasible_count);

#ifdef __cplusplus
}
#endif
#endif /* AMSP_H */
