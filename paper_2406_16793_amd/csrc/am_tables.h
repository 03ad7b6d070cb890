// Work tables shared by the host layout builder and the gfx950 kernels.
//
// A step is a handful of launches; each launch ("bucket") serves every tensor that
// was assigned the same kernel variant.  A bucket's work items are numbered
// 0 .. n_items-1 across all its tensors; AmSeg records where one tensor's items
// start, so a workgroup finds its tensor with a binary search over item_first.
#ifndef AM_TABLES_H_
#define AM_TABLES_H_

#include <stdint.h>

// Kernel families.
enum AmFamily : int {
  AM_FAM_ELEMENTWISE = 0,  // block_numel == 1; item = tile of units of one tensor
  AM_FAM_ROW = 1,          // item = one block, held in the registers of a team of LANES threads
  AM_FAM_LARGE = 2,        // item = one chunk of a block; partial sums + finalize + update
  AM_FAM_ROW_LDS = 3,      // item = one block, gradient staged in the workgroup's LDS
  AM_FAM_STRIDED = 4,      // blocks are columns: item = (row chunk, group of 256 or 512 column units)
  AM_FAM_FUSED = 5         // small layouts: every tensor in one launch; item = a workgroup's worth of blocks or units
};

// One tensor inside one bucket.  Device pointers are filled in at step time.
struct AmSeg {
  float* p;               // params (fp32)
  const void* g;          // grads (fp32 or bf16)
  float* m;               // first moment (fp32)
  uint64_t v_first;       // index of the tensor's first scalar in v
  uint64_t block_numel;   // elements per block (ELEMENTWISE: numel of the tensor)
  uint64_t units_per_block;  // block_numel / VEC (ELEMENTWISE: ceil(numel / VEC))
  uint32_t item_first;    // number of work items of the bucket before this tensor
  uint32_t lblock_first;  // LARGE: number of large blocks of the bucket before this tensor
  uint32_t chunks_per_block; // LARGE: work items per block; STRIDED: column groups per row chunk; otherwise 1
  uint32_t tensor;        // index in the caller's tensor list
  float wd_scale;         // lambda_k = weight_decay * wd_scale
  uint32_t reducer;       // block statistic of g .* g that feeds v: 0 mean (the method), 1 1-norm, 2 2-norm, 3 max, 4 min
  uint64_t aux;           // STRIDED: index of the tensor's first partial sum in the scratch
  uint64_t row_len;       // STRIDED: elements per stored row (= number of blocks C)
  uint64_t n_blocks;      // number of blocks of the tensor
  uint32_t team_lanes;    // FUSED: lanes of the team that holds one block (16, 64, 256, 1024); 0: one-element blocks
  uint32_t blocks_per_item;  // FUSED: whole blocks per work item (<= 1024 / team_lanes)
};
// STRIDED reuses the fields as: block_numel = rows R of the stored [R, C] matrix (elements per block),
// units_per_block = units per ROW (C / VEC), chunks_per_block = column groups per row chunk,
// lblock_first = number of columns of the bucket before this tensor (index into the scale scratch).

// A bucket's device tables.  The two key arrays repeat item_first / lblock_first of every
// segment densely, so the binary search of a workgroup stays inside a few cache lines.
struct AmTable {
  const AmSeg* segs;
  const uint32_t* item_keys;    // [n_segs] ascending
  const uint32_t* lblock_keys;  // [n_segs] ascending (LARGE only; otherwise zeros)
  uint32_t n_segs;
  uint32_t xcd_code;            // low byte: log2 of the run of work-item groups one XCD walks (>= 32: identity
                                // order); next byte: log2 of the number of XCDs
};

// Tile of the STRIDED family, shared by the layout builder and the kernels: a workgroup of
// kStridedThreads lanes owns kStridedThreads * aux units of a row (aux = AmVariant::aux, 1 or 2) over
// AmVariant::upt consecutive rows.
constexpr int kStridedThreads = 256;
// The STRIDED update pass has work items of its own: tiles of kStridedThreads * kStridedUpdateUpt consecutive
// units of the tensor (AmBucket::item2_first / n_items2, the bucket's second key array on the device).
constexpr int kStridedUpdateUpt = 4;

// Workgroup of the FUSED family, shared by the layout builder and the kernel: 1024 threads; a block is
// held by a team of 16, 64, 256 or 1024 of them at up to kFusedUpt units per lane (AmSeg::team_lanes; 0 for a
// tensor of one-element blocks), AmSeg::blocks_per_item whole blocks to a work item.
constexpr int kFusedThreads = 1024;
constexpr int kFusedUpt = 4;

// Per-step scalars, computed on the host in double and rounded once to fp32.
struct AmScalars {
  float beta1;      // beta1
  float omb1;       // 1 - beta1
  float beta2;      // beta2
  float omb2;       // 1 - beta2
  float eps;        // eps
  float bc2;        // 1 - beta2^t
  float step_size;  // lr / (1 - beta1^t)
  float lr_wd;      // lr * weight_decay
};

// How the per-step scalars reach a kernel: by value (computed on the host for this call), or -- dev not
// null -- read from device memory, where a small kernel put them from hyper-parameters that live on the
// device (a step that a HIP graph can replay with an advancing step counter).
struct AmScalarsArg {
  AmScalars val;
  const AmScalars* dev;
};

// Variant of a kernel family: how a block (or tile) is spread over threads.
struct AmVariant {
  int family;  // AmFamily
  int vec;     // elements per unit: 1 (scalar fallback), 4 (fp32 grads) or 8 (bf16 grads)
  int lanes;   // threads cooperating on one item
  int upt;     // units per thread (compile-time unroll); STRIDED: rows per work item (a launch argument)
  int aux;     // STRIDED: units of a row per lane (1 or 2); otherwise 0
};

#endif  // AM_TABLES_H_
