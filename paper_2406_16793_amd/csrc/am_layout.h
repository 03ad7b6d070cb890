// Host-side layout builder: descriptors -> v offsets, kernel variant per tensor,
// launch buckets and their work tables.  Pure C++ (no HIP), so it can be exercised
// on a machine without a GPU.
#ifndef AM_LAYOUT_H_
#define AM_LAYOUT_H_

#include <stdint.h>

#include <vector>

#include "../../include/adam_mini.h"
#include "am_tables.h"

struct AmTensorInfo {
  uint64_t numel;
  uint64_t block_numel;
  float wd_scale;
  uint64_t v_first;   // exclusive prefix sum of numel / block_numel
  uint64_t n_blocks;
  bool strided;       // blocks are the columns of the stored [block_numel, n_blocks] matrix
  int bucket;         // index into AmHostLayout::buckets
  int seg;            // index into that bucket's segs
};

// One contiguous run of a LARGE bucket's work items and blocks: a launch triple of its own.
struct AmSlice {
  uint32_t item_first, n_items, lblock_first, n_lblocks;
};

struct AmBucket {
  AmVariant var;
  std::vector<AmSeg> segs;  // pointers left null here; filled at step time
  uint64_t n_items = 0;     // total work items (ROW: blocks, LARGE: chunks, ELEMENTWISE: tiles)
  std::vector<uint32_t> item2_first;  // STRIDED: per segment, work items of the UPDATE pass before this tensor
  uint64_t n_items2 = 0;    // STRIDED: work items of the update pass (linear tiles)
  uint64_t n_lblocks = 0;   // LARGE: total blocks, STRIDED: total columns (length of the scale scratch)
  uint64_t n_partials = 0;  // STRIDED: floats of partial sums the bucket needs
  uint64_t table_offset = 0;  // index of segs[0] in the concatenated device table
  uint64_t lds_bytes = 0;     // ROW_LDS: bytes of LDS that hold the largest block's gradient
  uint64_t max_chunks = 0;    // LARGE: chunks of the bucket's largest block
  std::vector<AmSlice> slices;  // LARGE: the bucket as one slice, or cut by large_slice_mb (see am_layout.cpp)
  bool alt_reducer = false;   // some tensor's block statistic is not a plain sum of squares (2-norm, max, min)
};

// Knobs of the variant choice (process-wide defaults; copied into a layout when it is built).
struct AmTuning {
  int64_t bf16_vec = 4;             // elements per unit with bf16 gradients: 4 (64-bit g loads, lane-contiguous
                                    //   128-bit m / p) or 8 (128-bit g loads, m / p as two adjacent 128-bit words)
  int64_t subwave_max_units = 64;   // blocks of <= this many units may use 16-thread teams
  int64_t wave_max_units = 256;     // blocks of <= this many units may use one 64-thread wavefront each
  int64_t team_max_lanes = 1024;    // largest team (threads per block) the row kernel may use
  int64_t max_upt = 2;              // preferred upper bound on units per thread: the smallest team that
                                    //   stays within it is chosen; exceeded only when no team fits otherwise
  int64_t row_max_units = 1 << 30;  // blocks above this never use the single-pass register kernel
  int64_t lds_max_bytes = 150 * 1024;       // > 0: blocks that do not fit the register kernel and whose gradient fits
                                    //      in this many bytes of LDS use the LDS-staged single-pass kernel
  int64_t cu_count = 256;           // compute units the LDS-staged kernel's workgroups (one per block, one or two per
                                    //   unit) are dealt to: a list whose staged blocks fill their last round of
                                    //   workgroups badly sends them to the multi-workgroup kernels instead
                                    //   (am_staging_pays in am_layout.cpp); 0 = never mind the balance
  int64_t large_chunk_upt = 4;      // LARGE: units per thread of a 256-thread chunk (1, 2, 4, 8 or 16)
  int64_t ew_upt = 4;               // ELEMENTWISE: units per thread of a 256-thread tile (1, 2, 4 or 8)
  int64_t large_slice_mb = 0;       // LARGE: > 0 cuts the bucket into slices of at most this many MB of gradient,
                                    //   each running partial sums, finalize and update back to back; 0 = one slice
  int64_t large_wide_chunks = 512;  // LARGE: a bucket with a block of at least this many chunks sums each block's
                                    //   chunk partials with a 1024-thread workgroup instead of one wavefront; 0 = never
  int64_t large_keep_g = 0;         // LARGE: 1 = the gradient is read with ordinary cached loads in both passes
  int64_t grid_cap = 0;             // > 0: at most this many workgroups per launch (grid-stride beyond)
  int64_t row_inflight_kb = 80;     // row kernel: resident workgroups per compute unit are capped so that the
                                    //   loads they keep in flight stay near this many KB (0 = no cap)
  int64_t row_wg_per_cu = 0;        // > 0: fixed cap on resident row-kernel workgroups per compute unit (overrides row_inflight_kb)
  int64_t row_blocked = 0;          // 1: each wavefront of a row team owns a contiguous span of the block
  int64_t strided_wg_per_cu = 2;    // > 0: cap on resident workgroups per compute unit of the column-block update kernel
  int64_t stream_wg_per_cu = 2;     // > 0: same for the large-block update kernel
  int64_t ew_wg_per_cu = 2;         // > 0: same for the AdamW-equivalent (one-element-block) kernel
  int64_t fuse_max_params = 16 << 20;  // > 0: a tensor list of at most this many elements whose blocks all fit one
                                    //   team of the generic kernel is stepped in ONE launch (small models are
                                    //   bound by the number of launches); 0 = never
  int64_t fuse_target_items = 224;  // the one-launch kernel: blocks are grouped so that the list makes about this many
                                    //   work items (fewer than the chip has compute units: one round of workgroups)
  int64_t strided_rows = 128;       // column-block kernels: rows of the stored matrix per work item (multiple of 4)
  int64_t xcd_count = 8;            // XCDs the hardware deals workgroups to round-robin (power of two; 8 when the
                                    //   device is one partition)
  int64_t xcd_chunk = 64;           // row kernels: consecutive workgroup passes one XCD walks (power of two; 0 = the
                                    //   hardware's round-robin order, item by item)
  int64_t xcd_chunk_stream = 16;    // same for the elementwise and large-block kernels
  int64_t xcd_chunk_strided = 16;   // same for the column-block kernels
};

struct AmHostLayout {
  int grad_dtype = 0;
  AmTuning tuning;
  std::vector<AmTensorInfo> tensors;
  std::vector<AmBucket> buckets;
  uint64_t num_blocks = 0;    // length of v
  uint64_t n_partials = 0;    // max over LARGE buckets of n_items   (scratch floats)
  uint64_t n_lblocks = 0;     // max over LARGE buckets of n_lblocks (scratch floats)
  uint64_t n_segs = 0;        // total segments over all buckets
};

// Returns ADAM_MINI_OK or ADAM_MINI_INVALID_ARG.
int am_build_layout(const adam_mini_tensor_desc* descs, uint32_t n_tensors, int grad_dtype,
                    const AmTuning& tuning, AmHostLayout* out);

// Does the whole list qualify for the one-launch generic kernel (AM_FAM_FUSED)?
bool am_list_is_fusable(int grad_dtype, const adam_mini_tensor_desc* descs, uint32_t n_tensors,
                        const AmTuning& tuning);

// Kernel variant that serves a tensor.
AmVariant am_choose_variant(int grad_dtype, uint64_t numel, uint64_t block_numel, uint64_t v_first,
                            const AmTuning& tuning);

// Units a team of the row kernel variant (lanes, upt) can hold.
inline uint64_t am_row_capacity(const AmVariant& v) { return (uint64_t)v.lanes * (uint64_t)v.upt; }

// Work items per workgroup-sized chunk / tile for the LARGE and ELEMENTWISE families.
inline uint64_t am_tile_units(const AmVariant& v) { return (uint64_t)v.lanes * (uint64_t)v.upt; }

int am_path_kind(const AmVariant& v);

#endif  // AM_LAYOUT_H_
