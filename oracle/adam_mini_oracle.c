/*
 * Adam-mini step oracle: test infrastructure, NOT part of the product.
 *
 * A plain, slow CPU statement of what one optimizer step computes, used only
 * by the tests, the smoke check and the CPU-baseline leg of the benchmark.
 * It shares no code with the HIP library and the HIP library never calls it.
 *
 * Arithmetic: everything in IEEE double.  State (param, m, v) is held in
 * double between steps; gradients arrive as fp32 or bf16 bit patterns and are
 * widened exactly.  Hyper-parameters arrive as doubles (the caller widens the
 * same fp32 values the GPU library receives).
 *
 * What is computed is Algorithm 1 ("Adam-mini, general form", Section 2.3; the
 * same update again in PyTorch style as Algorithm 2, Appendix B).  With g the
 * block's gradient, n its size and t >= 1 the step, this file evaluates it as
 *     stat   = (1/n) * sum_i g_i^2                  the block's mean squared gradient
 *     v      = (1 - beta2) * stat + beta2 * v       ONE second moment per block
 *     v_hat  = v / (1 - beta2^t)
 *   and then for every element i of the block
 *     param_i = param_i - lr * lambda * param_i     decoupled weight decay
 *     m_i     = (1 - beta1) * g_i + beta1 * m_i
 *     m_hat   = m_i / (1 - beta1^t)
 *     param_i = param_i - lr * m_hat / (sqrt(v_hat) + eps)
 * The statistic comes first only because everything after it needs it; each
 * element still sees decay, first moment and step in Algorithm 1's order.
 * The blocks of one tensor are the consecutive, equally sized, contiguous runs
 * of `block_numel` elements of the row-major tensor: that is what "partition
 * by tokens / heads / output neurons" (listing "Partition for Transformers",
 * Appendix B) yields when the
 * partition dimension is the outermost one.  When a codebase stores the weight
 * transposed (Appendix D notes that re-ordering is then needed) the same blocks
 * are the COLUMNS of the stored matrix: the `strided` form below.  block_numel == 1 is vanilla AdamW
 * (Section 2.3: the method is Adam with g .* g replaced by its block mean); block_numel
 * == numel is the non-Transformer partition (Algorithm "Partition for
 * non-Transformers", Appendix B).
 *
 * The ablation on the design of Adam-mini (appendix section "Ablation Studies on
 * the Design of Adam-mini") swaps the mean for other statistics taken from Adam's
 * elementwise g .* g: its 2-norm, 1-norm, max and min.  The paper gives no
 * formula for them; the reading taken here keeps Algorithm 1 as it stands and
 * replaces only the word "mean" in its v line:
 *     v = (1 - beta2) * r(g .* g) + beta2 * v,   r in {mean, 1-norm, 2-norm, max, min}
 * with the vector norms of the n-vector g .* g written out.  `reducer` selects r;
 * AMO_REDUCE_MEAN is the method itself.
 *
 * Pins (tests/test_oracle_pins.py): AdamW special case against a library
 * routine, constant-gradient closed form, EMA identity, hand-worked rational
 * example, brute force against a dictionary-of-slices transcription of the
 * partition, symmetries, layout invariants.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#define AMO_GRAD_F32 0
#define AMO_GRAD_BF16 1
#define AMO_GRAD_F64 2

#define AMO_REDUCE_MEAN 0  /* sum_i g_i^2 / n : Algorithm 1 */
#define AMO_REDUCE_NORM1 1 /* sum_i |g_i^2| */
#define AMO_REDUCE_NORM2 2 /* sqrt(sum_i (g_i^2)^2) */
#define AMO_REDUCE_MAX 3   /* largest g_i^2 */
#define AMO_REDUCE_MIN 4   /* smallest g_i^2 */

/* Exact widening of one gradient element to double. */
static double amo_grad_at(const void *g, int dtype, uint64_t i) {
  if (dtype == AMO_GRAD_F32) {
    return (double)((const float *)g)[i];
  } else if (dtype == AMO_GRAD_BF16) {
    /* bf16 is the upper half of an fp32 word */
    uint32_t bits = ((uint32_t)((const uint16_t *)g)[i]) << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
  }
  return ((const double *)g)[i];
}

/*
 * One step of Algorithm 1 on ONE block of n elements.
 *   p, m : the block's first element; element i of the block is p[i * stride]
 *          (stride 1: a contiguous run; stride > 1: a column of a row-major matrix)
 *   v    : the block's scalar, in place
 *   g, dtype, g_first : gradient buffer, its element type, index of the block's
 *                       first element inside it (element i is g_first + i * stride)
 *   t >= 1 : step counter used by the bias corrections
 *   reducer : AMO_REDUCE_*, the statistic of g .* g that feeds v
 */
void amo_step_block(double *p, double *m, double *v, const void *g, int dtype,
                    uint64_t g_first, uint64_t n, uint64_t stride, double lr,
                    double beta1, double beta2, double eps, double lambda,
                    uint64_t t, int reducer) {
  double bias1 = 1.0 - pow(beta1, (double)t);
  double bias2 = 1.0 - pow(beta2, (double)t);

  /* the block statistic of Algorithm 1: the mean over the block of the squared gradient entries */
  double sum_sq = 0.0;
  for (uint64_t i = 0; i < n; ++i) {
    double gi = amo_grad_at(g, dtype, g_first + i * stride);
    sum_sq += gi * gi;
  }
  double mean_sq = sum_sq / (double)n;
  double stat = mean_sq;
  if (reducer != AMO_REDUCE_MEAN) {
    /* the ablation's other statistics of the vector s = g .* g, s_i = g_i^2 */
    double norm1 = 0.0, sum_s2 = 0.0, largest = 0.0, smallest = 0.0;
    int any_nan = 0;
    for (uint64_t i = 0; i < n; ++i) {
      double gi = amo_grad_at(g, dtype, g_first + i * stride);
      double si = gi * gi;
      norm1 += fabs(si);
      sum_s2 += si * si;
      if (si != si) any_nan = 1;
      if (i == 0 || si > largest) largest = si;
      if (i == 0 || si < smallest) smallest = si;
    }
    if (reducer == AMO_REDUCE_NORM1) stat = norm1;
    if (reducer == AMO_REDUCE_NORM2) stat = sqrt(sum_s2);
    if (reducer == AMO_REDUCE_MAX) stat = largest;
    if (reducer == AMO_REDUCE_MIN) stat = smallest;
    /* a comparison never selects a NaN; like the sums, max and min hand it on */
    if (any_nan) stat = NAN;
  }
  /* the block's single second moment: running average of the statistic, then its bias correction */
  *v = (1.0 - beta2) * stat + beta2 * (*v);
  double v_hat = *v / bias2;

  /* every element of the block: decoupled decay, first moment, bias-corrected step.  All
   * elements divide by the same sqrt(v_hat) + eps: eps is added outside the root. */
  for (uint64_t i = 0; i < n; ++i) {
    p[i * stride] = p[i * stride] - lr * lambda * p[i * stride];
    double gi = amo_grad_at(g, dtype, g_first + i * stride);
    m[i * stride] = (1.0 - beta1) * gi + beta1 * m[i * stride];
    double m_hat = m[i * stride] / bias1;
    p[i * stride] = p[i * stride] - lr * m_hat / (sqrt(v_hat) + eps);
  }
}

/*
 * One step on one tensor of `numel` elements cut into numel/block_numel blocks.
 * strided == 0: block b is the contiguous run [b*block_numel, (b+1)*block_numel).
 * strided != 0: the tensor is a row-major [block_numel, n_blocks] matrix and
 *               block b is its COLUMN b (elements r*n_blocks + b): the layout a
 *               weight takes when a codebase stores W as its transpose, the case
 *               for which the paper's appendix says re-ordering is needed
 *               (Appendix D, last paragraph on Hessian plots).
 * v points at this tensor's first scalar (one per block).  Blocks never
 * interact, so they are handed to the host threads as they come.
 * Returns 0, or -1 when the descriptor is not a valid uniform partition.
 */
int amo_step_tensor(double *p, double *m, double *v, const void *g, int dtype,
                    uint64_t numel, uint64_t block_numel, int strided, double lr,
                    double beta1, double beta2, double eps, double lambda,
                    uint64_t t, int reducer) {
  if (numel == 0 || block_numel == 0 || numel % block_numel != 0 || t == 0)
    return -1;
  if (reducer < AMO_REDUCE_MEAN || reducer > AMO_REDUCE_MIN) return -1;
  int64_t n_blocks = (int64_t)(numel / block_numel);
#pragma omp parallel for schedule(static)
  for (int64_t b = 0; b < n_blocks; ++b) {
    uint64_t first = strided ? (uint64_t)b : (uint64_t)b * block_numel;
    uint64_t stride = strided ? (uint64_t)n_blocks : 1;
    amo_step_block(p + first, m + first, v + b, g, dtype, first, block_numel,
                   stride, lr, beta1, beta2, eps, lambda, t, reducer);
  }
  return 0;
}

/*
 * Index of the second-moment scalar that element `elem` of tensor `tensor`
 * uses, when the v scalars of all tensors are stored back to back in tensor
 * order.  Written as a running count of blocks, independent of any table.
 * strided may be NULL (all tensors contiguous).
 * Returns UINT64_MAX on a bad argument.
 */
uint64_t amo_block_id(const uint64_t *numel, const uint64_t *block_numel,
                      const int32_t *strided, uint32_t n_tensors,
                      uint32_t tensor, uint64_t elem) {
  if (tensor >= n_tensors || elem >= numel[tensor]) return UINT64_MAX;
  uint64_t blocks_before = 0;
  for (uint32_t k = 0; k < tensor; ++k)
    blocks_before += numel[k] / block_numel[k];
  if (strided && strided[tensor])
    return blocks_before + elem % (numel[tensor] / block_numel[tensor]);
  return blocks_before + elem / block_numel[tensor];
}

/* amo_block_id for every element of one tensor: out[e], e = 0 .. numel[tensor]-1. */
int amo_block_ids_tensor(const uint64_t *numel, const uint64_t *block_numel,
                         const int32_t *strided, uint32_t n_tensors,
                         uint32_t tensor, uint64_t *out) {
  if (tensor >= n_tensors) return -1;
  for (uint64_t e = 0; e < numel[tensor]; ++e)
    out[e] = amo_block_id(numel, block_numel, strided, n_tensors, tensor, e);
  return 0;
}

/* Total number of v scalars of a tensor list. */
uint64_t amo_num_blocks(const uint64_t *numel, const uint64_t *block_numel,
                        uint32_t n_tensors) {
  uint64_t total = 0;
  for (uint32_t k = 0; k < n_tensors; ++k) total += numel[k] / block_numel[k];
  return total;
}

/* Threads the tensor loop will use (for the CPU-baseline report). */
int amo_num_threads(void) {
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  return omp_get_max_threads();
#else
  return 1;
#endif
}
