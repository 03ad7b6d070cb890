/*
 * adam_mini.h -- C ABI of the MI355X (gfx950) Adam-mini optimizer-step library.
 *
 * What the library computes is one step of the paper's Algorithm 1 ("Adam-mini,
 * general form", Section 2.3; repeated as Algorithm 2 in Appendix B) over a list
 * of tensors.  For every block b of the parameter partition, with g the block's
 * gradient, n_b its element count, t the 1-based step and
 * bc1 = 1 - beta1^t, bc2 = 1 - beta2^t:
 *
 *     param_i <- param_i - lr * lambda_k * param_i            (decoupled decay)
 *     m_i     <- (1 - beta1) * g_i + beta1 * m_i
 *     v_b     <- (1 - beta2) * (sum_i g_i^2) / n_b + beta2 * v_b   (ONE scalar per block)
 *     param_i <- param_i - (lr / bc1) * m_i / (sqrt(v_b / bc2) + eps)
 *
 * The partition (listing "Partition for Transformers", Appendix B: embedding
 * and output layers by token, query/key by head, value / attention projection /
 * MLP by output neuron, everything else as one block) always cuts a row-major
 * tensor whose partition dimension is outermost into equal, contiguous runs of
 * elements, so a tensor's partition is described by one number, block_numel.
 * block_numel == 1 makes the step vanilla AdamW with a dense v (Section 2.3:
 * Adam-mini replaces g*g of Adam by its block mean); block_numel == numel is the
 * "Partition for non-Transformers" of Appendix B.
 *
 * Conventions
 *   - Every pointer named *_dev / documented "device" is a HIP device pointer on
 *     the layout's device; everything else is host memory.
 *   - All functions return ADAM_MINI_OK (0) or a negative adam_mini_status code.
 *     Nothing is thrown across the boundary.  Argument validation happens before
 *     any kernel launch: on a validation error no device memory was touched.
 *   - The library owns only the layout handle (host tables, device work tables,
 *     partial-sum scratch).  The caller owns params, grads, exp_avg and v.
 */
#ifndef ADAM_MINI_H_
#define ADAM_MINI_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum adam_mini_status {
  ADAM_MINI_OK = 0,
  ADAM_MINI_INVALID_ARG = -1,   /* null pointer, zero size, block_numel does not divide numel,
                                   a reserved flag bit or an unknown ADAM_MINI_REDUCE_* value, step == 0,
                                   beta outside [0,1), eps < 0, non-finite hyper-parameter, unknown dtype,
                                   bad tensor index, a size beyond a documented limit */
  ADAM_MINI_MISALIGNED = -2,    /* a device base pointer is not 16-byte aligned */
  ADAM_MINI_OUT_OF_MEMORY = -3, /* host or device allocation failed */
  ADAM_MINI_HIP_ERROR = -4,     /* a HIP runtime call failed (see adam_mini_last_hip_error) */
  ADAM_MINI_NO_DEVICE = -5,     /* the layout was built with device < 0 (host-only layout) */
  ADAM_MINI_TOO_LARGE = -6      /* adam_mini_step_static: the layout's work tables and scratch exceed
                                   ADAM_MINI_STATIC_SCRATCH_BYTES */
} adam_mini_status;

/* Gradient element type.  Params, exp_avg (m) and v are always fp32. */
enum { ADAM_MINI_GRAD_F32 = 0, ADAM_MINI_GRAD_BF16 = 1 };

/* Which kernel family serves a tensor (reported by adam_mini_export_layout). */
enum {
  ADAM_MINI_PATH_ELEMENTWISE = 0, /* block_numel == 1: AdamW-equivalent, dense v */
  ADAM_MINI_PATH_ROW = 1,         /* whole block held in registers of <= one workgroup; single pass */
  ADAM_MINI_PATH_LARGE = 2,       /* block spans several workgroups: partial sums, finalize, update */
  ADAM_MINI_PATH_ROW_LDS = 3,     /* whole block staged in one workgroup's LDS; single pass */
  ADAM_MINI_PATH_STRIDED = 4,     /* blocks are columns of the stored matrix: column partial sums, finalize, update */
  ADAM_MINI_PATH_FUSED = 5        /* small tensor list: every tensor in one launch of a generic single-pass kernel */
};

/* adam_mini_tensor_desc.flags */
enum {
  /* The tensor is stored as a row-major [block_numel, numel/block_numel] matrix and block j is its
   * COLUMN j (elements r*n_blocks + j): the layout of a weight whose codebase keeps W as its
   * transpose, for which the paper's Appendix D says the blocks must be re-ordered.  Results equal
   * those of the contiguous form on the transposed data. */
  ADAM_MINI_FLAG_STRIDED = 1u,

  /* Bits 4-6: the block statistic r of g .* g that feeds the second moment,
   *     v_b <- beta2 v_b + (1 - beta2) r(g_b .* g_b).
   * MEAN (0, the default) is the method itself (Algorithm 1, Section 2.3).  The others are the
   * candidates of the appendix's "Ablation Studies on the Design of Adam-mini", which names them
   * (2-norm, 1-norm, max, min of Adam's elementwise g .* g) without a formula; they are read as
   * Algorithm 1 with only the word "mean" replaced:
   *     NORM1  sum_i g_i^2        NORM2  sqrt(sum_i g_i^4)        MAX  max_i g_i^2        MIN  min_i g_i^2
   * A NaN in the block's gradient makes every statistic NaN.  With block_numel = 1 all five are
   * g^2 (AdamW).  Sums are fp32 like the mean's; g^4 leaves the normal fp32 range below |g| ~ 3e-10. */
  ADAM_MINI_REDUCE_MEAN = 0u << 4,
  ADAM_MINI_REDUCE_NORM1 = 1u << 4,
  ADAM_MINI_REDUCE_NORM2 = 2u << 4,
  ADAM_MINI_REDUCE_MAX = 3u << 4,
  ADAM_MINI_REDUCE_MIN = 4u << 4,
  ADAM_MINI_REDUCE_MASK = 7u << 4
};

/*
 * One tensor of the multi-tensor list.  The tensor is contiguous, row-major, with
 * the partition dimension outermost; its blocks are elements
 * [j*block_numel, (j+1)*block_numel), j = 0 .. numel/block_numel - 1
 * (with ADAM_MINI_FLAG_STRIDED the partition dimension is innermost instead, see the flag).
 *   rows of an [out,in] weight (value / attn.proj / mlp; embed / output by token): block_numel = in
 *   heads of a [heads*head_dim, in] query / key weight:                            block_numel = head_dim*in
 *   any other tensor (norm gains, biases):                                          block_numel = numel
 *   AdamW-equivalent:                                                               block_numel = 1
 */
typedef struct adam_mini_tensor_desc {
  uint64_t numel;       /* > 0 */
  uint64_t block_numel; /* > 0 and divides numel */
  float wd_scale;       /* lambda_k = weight_decay * wd_scale (1 for decayed tensors, 0 for none); finite, >= 0 */
  uint32_t flags;       /* ADAM_MINI_FLAG_STRIDED and / or one ADAM_MINI_REDUCE_*; other bits are reserved and must be 0 */
} adam_mini_tensor_desc;

/* Hyper-parameters of one step (the inputs of Algorithm 1 and its step counter t). */
typedef struct adam_mini_hparams {
  float lr;           /* eta_t, finite */
  float beta1;        /* in [0,1) */
  float beta2;        /* in [0,1) */
  float eps;          /* >= 0 */
  float weight_decay; /* lambda, finite */
  uint64_t step;      /* t >= 1 (t = 0 would divide by 1 - beta^0 = 0) */
} adam_mini_hparams;

typedef struct adam_mini_layout adam_mini_layout; /* opaque */

/*
 * Build the block layout of a tensor list ("Partition for Transformers", Appendix B, realised as descriptors).
 * Host-only work: validates the descriptors, assigns v indices (the v scalars of
 * all tensors are stored back to back in tensor order: tensor k owns
 * v[v_offset[k] .. v_offset[k+1]), v_offset = exclusive prefix sum of
 * numel/block_numel), picks a kernel family per tensor and builds the work tables.
 * No HIP call is made here; device tables and scratch are created by the first
 * adam_mini_step / adam_mini_write_block_ids on `device`.
 *   descs      host array [n_tensors], copied
 *   grad_dtype ADAM_MINI_GRAD_F32 or ADAM_MINI_GRAD_BF16, same for all tensors
 *   device     HIP device ordinal, or -1 for a host-only layout (export works, step does not)
 *   out        receives the handle; free with adam_mini_destroy_layout
 */
int adam_mini_init_layout(const adam_mini_tensor_desc* descs, uint32_t n_tensors,
                          int grad_dtype, int device, adam_mini_layout** out);

/* Number of fp32 scalars the caller must provide in v (sum over tensors of
 * numel/block_numel).  0 if layout is null. */
uint64_t adam_mini_num_blocks(const adam_mini_layout* layout);

/* Number of tensors of the layout (0 if null). */
uint32_t adam_mini_num_tensors(const adam_mini_layout* layout);

/*
 * Copy out the integer layout.  v_offset: host array [n_tensors + 1] (may be null);
 * path_kind: host array [n_tensors] of ADAM_MINI_PATH_* (may be null).
 */
int adam_mini_export_layout(const adam_mini_layout* layout, uint64_t* v_offset,
                            uint32_t* path_kind);

/* Host lookup: index into v used by element `elem` of tensor `tensor`, written to
 * *out.  Same answer the device tables give (adam_mini_write_block_ids). */
int adam_mini_block_id(const adam_mini_layout* layout, uint32_t tensor, uint64_t elem,
                       uint64_t* out);

/*
 * Device check of the layout: for tensor `tensor`, every element's v index is
 * written by walking the same device work tables, with the same work-item to
 * element mapping, that adam_mini_step uses.  ids_dev: device array of numel
 * uint64.  Asynchronous on hip_stream (a hipStream_t passed as void*; null = the
 * default stream).  Used to compare the block-index layout bit for bit with an
 * independent implementation.
 */
int adam_mini_write_block_ids(adam_mini_layout* layout, uint32_t tensor,
                              uint64_t* ids_dev, void* hip_stream);

/*
 * One optimizer step over all tensors (the body of Algorithm 1's loop, for every block).
 *   params   host array [n_tensors] of device pointers, fp32, updated in place
 *   grads    host array [n_tensors] of device pointers, fp32 or bf16 per the layout; read only
 *   exp_avg  host array [n_tensors] of device pointers, fp32 first moment m, updated in place
 *   v_dev    device array of adam_mini_num_blocks() fp32, updated in place
 *   hp       host pointer, read during the call
 *   hip_stream  hipStream_t as void* (null = default stream); all work is enqueued there
 * m and v must be zero before the first step (t = 1).  Every device pointer must be
 * 16-byte aligned.  Tensors must not overlap each other.  The call is asynchronous:
 * it never waits for the device, and after the first call on a layout (which creates
 * the device work tables and scratch and uploads the tables with a blocking copy) it
 * never allocates or copies.  When the three pointer lists differ from the previous
 * call's, the new pointers travel to the device tables as arguments of a few small
 * kernels enqueued on hip_stream ahead of the step's own: a caller whose gradient
 * buffers move every step pays a few microseconds of device time, no host stall.
 * Results are bitwise reproducible: no atomics on floating-point data, fixed
 * summation order.  Every call enqueues kernels only (no memset, no copy) once the
 * device state exists, so it may be captured into a HIP graph; the captured step
 * replays with the hyper-parameters and pointers it was captured with.
 * Calls on one layout must be ordered (one stream, or streams the caller orders):
 * concurrent calls race on the layout's tables and scratch; use one layout per
 * stream.  Non-finite gradients are not skipped: they propagate into the block's
 * v and parameters (and no other block's).
 */
int adam_mini_step(adam_mini_layout* layout, void* const* params,
                   const void* const* grads, void* const* exp_avg, float* v_dev,
                   const adam_mini_hparams* hp, void* hip_stream);

/*
 * The same step with the hyper-parameters in DEVICE memory, for training loops that run under a HIP
 * graph: adam_mini_step bakes lr, the betas and above all the step counter t into its kernel
 * arguments, so a captured step replays as the SAME step; here a one-thread kernel enqueued ahead of
 * the step's own reads *hp_dev, forms the step's scalars from it (in double, as the host does) and the
 * step kernels read those from device memory.
 *   hp_dev   device pointer (8-byte aligned) to one adam_mini_hparams; read -- and with
 *            ADAM_MINI_STEP_ADVANCE written -- when the work runs on the stream, not during the call
 *   flags    0, or ADAM_MINI_STEP_ADVANCE: hp_dev->step is incremented first and the new value is
 *            this step's t (start it at 0).  A graph that captured such a call therefore performs
 *            steps t+1, t+2, ... on successive replays; change lr by writing hp_dev->lr between replays.
 * The values in *hp_dev cannot be validated by the host: the caller keeps them in the ranges
 * adam_mini_step accepts (t >= 1 when used, betas in [0,1), eps >= 0, finite lr and weight_decay).
 * Everything else (pointers, alignment, ordering, first-call behaviour) is as for adam_mini_step.
 */
enum { ADAM_MINI_STEP_ADVANCE = 1u };
int adam_mini_step_device_hparams(adam_mini_layout* layout, void* const* params,
                                  const void* const* grads, void* const* exp_avg, float* v_dev,
                                  adam_mini_hparams* hp_dev, uint32_t flags, void* hip_stream);

/*
 * The same step for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same results bit for bit, same validation as adam_mini_step; but the work tables,
 * the partial sums and the step scales live in one fixed array of
 * ADAM_MINI_STATIC_SCRATCH_BYTES inside the library's code object (every GPU the
 * library runs on holds its own copy until the process ends), and the tables reach it
 * as arguments of small kernels on hip_stream.  The call makes no hipMalloc, no
 * hipFree, no copy and no other allocating call, on its first use or later (the host
 * staging of the tables is sized by adam_mini_init_layout).
 * A layout needs  n_tensors * 116 + (partial sums + step scales) * 4 + 256  bytes, each part
 * rounded up to 256 (partial sums: one per 4096-element chunk of every block that
 * spans several workgroups, or one per column and tile of rows for column blocks);
 * the five benchmark shapes need 0.1 to 2.1 MB.  ADAM_MINI_TOO_LARGE if it does not
 * fit; nothing was launched then.
 * All layouts stepped this way on one GPU share that GPU's array, which keeps the last
 * call's contents: the tables are rewritten whenever the previous call on the GPU was
 * another layout's or had other pointers, and every partial sum a step reads is
 * written earlier in the same step, so nothing needs clearing.  Calls that overlap in
 * time on one GPU (two streams, two threads) race on the array: order them.
 * adam_mini_step on the same layout keeps working beside it (it uses the layout's own
 * allocations).
 */
#define ADAM_MINI_STATIC_SCRATCH_BYTES (16u << 20)
int adam_mini_step_static(adam_mini_layout* layout, void* const* params,
                          const void* const* grads, void* const* exp_avg, float* v_dev,
                          const adam_mini_hparams* hp, void* hip_stream);

/*
 * Launch structure and timing.  A step is a short sequence of launches ("buckets"):
 * all tensors served by the same kernel variant share one launch (three for the
 * multi-workgroup path: partial sums, finalize, update).
 */
typedef struct adam_mini_bucket_info {
  int32_t family;          /* ADAM_MINI_PATH_* */
  int32_t vec;             /* elements per unit (4 or 8), 1 = scalar fallback */
  int32_t lanes;           /* threads cooperating on one work item */
  int32_t upt;             /* units per thread */
  uint32_t n_tensors;      /* tensors served by this bucket */
  uint32_t n_kernels;      /* kernel launches per step (1, or 3 for ADAM_MINI_PATH_LARGE) */
  uint64_t n_items;        /* work items per launch */
  uint64_t numel;          /* parameters updated per launch */
  uint64_t n_blocks;       /* v scalars updated per launch */
  uint64_t timed_launches; /* steps whose launch of this bucket was timed since the last read */
  double total_ms;         /* sum of those durations (HIP events on the step's stream) */
  char kernel[96];         /* name of the (main) kernel, as a profiler prints it */
} adam_mini_bucket_info;

/* Number of buckets of the layout (0 if null). */
uint32_t adam_mini_num_buckets(const adam_mini_layout* layout);

/*
 * Turn per-bucket timing on (max_steps > 0: HIP events are created now, and the next
 * max_steps calls of adam_mini_step record one event pair around each bucket on the
 * step's stream) or off (max_steps == 0: events destroyed).  Needs a device layout.
 */
int adam_mini_profile_enable(adam_mini_layout* layout, uint32_t max_steps);

/*
 * Fill out[0 .. min(capacity, num_buckets)) .  If timing is on, first waits for the
 * recorded events, adds their elapsed times into total_ms / timed_launches and rearms
 * the event pool.  Works on a host-only layout too (timing fields are then zero).
 */
int adam_mini_profile_read(adam_mini_layout* layout, adam_mini_bucket_info* out, uint32_t capacity);

/*
 * Process-wide performance knobs, read by later adam_mini_init_layout calls (an
 * existing layout keeps the values it was built with).  They choose which kernel
 * variant serves a block size and how launches are shaped; they never change what
 * is computed beyond the order of the fp32 partial sums.  Keys (value >= 0):
 *   "bf16_vec"           4 or 8: elements per lane and access with bf16 gradients (4: 64-bit gradient
 *                        loads beside lane-contiguous 128-bit m / p; 8: 128-bit gradient loads)
 *   "subwave_max_units"  blocks of at most this many units may use 16-thread teams
 *   "wave_max_units"     ... at most this many units: one 64-thread wavefront per block
 *   "team_max_lanes"     largest number of threads that may share one block (256, 512 or 1024)
 *   "max_upt"            preferred bound on units per thread; the smallest team within it is used
 *   "row_max_units"      blocks above this leave the single-pass register kernel
 *   "lds_max_bytes"      > 0: such blocks whose gradient fits in this much LDS use the LDS-staged kernel
 *   "cu_count"           compute units assumed when deciding whether the LDS-staged kernel (one workgroup per
 *                        block) pays: a list with more staged blocks than this whose last round of workgroups
 *                        would be mostly empty (under 80 % filled on average with bf16 gradients, 55 % with
 *                        fp32) uses the multi-workgroup path for them instead; default 256, 0 = always stage
 *   "large_chunk_upt"    units per thread of a chunk in the multi-workgroup path (1, 2, 4, 8, 16)
 *   "large_slice_mb"     > 0: the multi-workgroup bucket is cut at block boundaries into slices of at most this
 *                        many MB of gradient, each running its three kernels back to back (a measurement knob:
 *                        every extra launch costs about 4 us and the second gradient read is not served on
 *                        chip, so the default 0, one slice, is fastest)
 *   "large_wide_chunks"  a multi-workgroup bucket with a block of at least this many chunks (whole-tensor blocks)
 *                        sums each block's chunk partials with one 1024-thread workgroup instead of one
 *                        wavefront; default 512, 0 = never
 *   "large_keep_g"       1: the multi-workgroup kernels read the gradient with ordinary cached loads instead of
 *                        streaming ones (a measurement knob; no effect seen)
 *   "ew_upt"             units per thread of a tile in the AdamW-equivalent kernel (1, 2, 4, 8)
 *   "grid_cap"           > 0: cap on workgroups per launch (grid-stride loop beyond it)
 *   "row_inflight_kb"    row kernel: resident workgroups per compute unit are capped so that the loads
 *                        they keep in flight stay near this many KB (HBM efficiency drops when the chip
 *                        is oversubscribed); 0 = no cap
 *   "row_wg_per_cu"      > 0: fixed cap on resident row-kernel workgroups per compute unit instead
 *   "row_blocked"        1: each wavefront of a row team owns a contiguous span of the block
 *   "stream_wg_per_cu"   the same cap for the large-block update kernel
 *   "ew_wg_per_cu"       the same cap for the AdamW-equivalent kernel
 *   "strided_wg_per_cu"  the same cap for the column-block (ADAM_MINI_FLAG_STRIDED) update kernel
 *   "fuse_max_params"    > 0: a tensor list of at most this many elements, all of whose blocks fit one
 *                        1024-lane team of the generic kernel, is stepped in ONE launch (a step of a small
 *                        model is bound by the number of launches); 0 = always one launch per kernel variant
 *   "fuse_target_items"  the one-launch kernel groups blocks so that the list makes about this many work items
 *                        (default 224, fewer than the chip has compute units, so that every workgroup is
 *                        resident at once)
 *   "strided_rows"       column-block kernels: rows of the stored matrix per work item (multiple of 4, >= 4)
 *   "xcd_count"          number of XCDs workgroups are dealt to round-robin (power of two; 8 on an
 *                        unpartitioned device, the default)
 *   "xcd_chunk"          row kernels: a power of two C > 0 makes each of the XCDs (dies with an L2 of
 *                        their own, fed workgroups round-robin) walk runs of C consecutive workgroup
 *                        passes instead of every 8th one; 0 keeps the hardware order
 *   "xcd_chunk_stream"   the same for the AdamW-equivalent and large-block kernels
 *   "xcd_chunk_strided"  the same for the column-block kernels
 *   "reset"              restore the defaults (value ignored)
 * Returns ADAM_MINI_INVALID_ARG for an unknown key or a negative value.
 */
int adam_mini_set_option(const char* key, int64_t value);

/* Frees host and device resources of the layout (null is a no-op).  The caller
 * must make sure no step using the layout is still running. */
void adam_mini_destroy_layout(adam_mini_layout* layout);

/* Static description of a status code (never null). */
const char* adam_mini_strerror(int status);

/* Text of the last HIP error seen by this thread inside the library ("" if none). */
const char* adam_mini_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* ADAM_MINI_H_ */
