// Host-side layout builder (see am_layout.h).  The partition itself is the paper's
// listing "Partition for Transformers" (Appendix B) already reduced by the
// caller to one block_numel per tensor; here the v scalars are numbered and each
// tensor is routed to the kernel variant that fits its block size.
#include "am_layout.h"

#include <cmath>

namespace {

// Row-kernel instantiations that exist (must match AM_ROW_VARIANTS in adam_mini.hip).
const int kLanes[] = {16, 64, 256, 512, 1024};
const int kUpt16[] = {1, 2, 4};
const int kUpt64[] = {1, 2, 4, 8, 16};
const int kUpt256[] = {1, 2, 3, 4, 6, 8, 12, 16};
const int kUpt512[] = {1, 2, 3, 4, 6, 8};
const int kUpt1024[] = {1, 2, 3, 4, 6};

// Register budget: a unit costs 3*vec data registers (g, m, p); 1024-thread workgroups
// get 128 registers per lane, smaller ones 256.
bool fits_registers(int vec, int lanes, int upt) {
  const int budget = lanes >= 1024 ? 128 : 256;
  return upt * vec * 3 + 34 <= budget;
}

// Smallest instantiated upt >= need for a team of `lanes`, or 0.
int round_up_upt(int lanes, uint64_t need, int vec) {
  const int* tab = nullptr;
  size_t n = 0;
  switch (lanes) {
    case 16: tab = kUpt16; n = sizeof kUpt16 / sizeof(int); break;
    case 64: tab = kUpt64; n = sizeof kUpt64 / sizeof(int); break;
    case 256: tab = kUpt256; n = sizeof kUpt256 / sizeof(int); break;
    case 512: tab = kUpt512; n = sizeof kUpt512 / sizeof(int); break;
    case 1024: tab = kUpt1024; n = sizeof kUpt1024 / sizeof(int); break;
    default: return 0;
  }
  for (size_t i = 0; i < n; ++i)
    if ((uint64_t)tab[i] >= need) return fits_registers(vec, lanes, tab[i]) ? tab[i] : 0;
  return 0;
}

bool lanes_allowed(int lanes, uint64_t units, const AmTuning& t) {
  if (lanes == 16) return units <= (uint64_t)t.subwave_max_units;
  if (lanes == 64) return units <= (uint64_t)t.wave_max_units;
  return lanes <= t.team_max_lanes || lanes == 256;
}

bool same_variant(const AmVariant& a, const AmVariant& b) {
  return a.family == b.family && a.vec == b.vec && a.lanes == b.lanes && a.upt == b.upt && a.aux == b.aux;
}

}  // namespace

// The LARGE bucket as one slice, or -- large_slice_mb > 0 -- cut at block boundaries into slices whose
// gradients are at most that many MB each: partial sums, finalize and update of a slice then run back to
// back (a measurement knob: would the update's second read of a slice's gradient be served on chip?).
static std::vector<AmSlice> large_slices(const AmBucket& bk, size_t grad_bytes, const AmTuning& t) {
  std::vector<AmSlice> out;
  if (t.large_slice_mb <= 0) {
    out.push_back(AmSlice{0u, (uint32_t)bk.n_items, 0u, (uint32_t)bk.n_lblocks});
    return out;
  }
  const uint64_t limit = (uint64_t)t.large_slice_mb << 20;
  AmSlice cur{0u, 0u, 0u, 0u};
  uint64_t bytes = 0;
  for (const AmSeg& s : bk.segs) {
    const uint64_t block_bytes = s.block_numel * grad_bytes;
    const uint64_t n_blocks = s.n_blocks;
    for (uint64_t b = 0; b < n_blocks; ++b) {
      if (cur.n_lblocks > 0 && bytes + block_bytes > limit) {
        out.push_back(cur);
        cur = AmSlice{cur.item_first + cur.n_items, 0u, cur.lblock_first + cur.n_lblocks, 0u};
        bytes = 0;
      }
      cur.n_items += s.chunks_per_block;
      cur.n_lblocks += 1;
      bytes += block_bytes;
    }
  }
  if (cur.n_lblocks > 0) out.push_back(cur);
  return out;
}

int am_path_kind(const AmVariant& v) {
  switch (v.family) {
    case AM_FAM_ELEMENTWISE: return ADAM_MINI_PATH_ELEMENTWISE;
    case AM_FAM_ROW: return ADAM_MINI_PATH_ROW;
    case AM_FAM_ROW_LDS: return ADAM_MINI_PATH_ROW_LDS;
    case AM_FAM_STRIDED: return ADAM_MINI_PATH_STRIDED;
    case AM_FAM_FUSED: return ADAM_MINI_PATH_FUSED;
    default: return ADAM_MINI_PATH_LARGE;
  }
}

AmVariant am_choose_variant(int grad_dtype, uint64_t numel, uint64_t block_numel, uint64_t v_first,
                            const AmTuning& t) {
  const int native = grad_dtype == ADAM_MINI_GRAD_BF16 ? (t.bf16_vec == 8 ? 8 : 4) : 4;
  AmVariant var{};
  if (block_numel == 1) {
    // AdamW-equivalent: dense v.  128-bit access needs whole units and a 16-byte aligned v slice.
    var.family = AM_FAM_ELEMENTWISE;
    var.vec = (numel % (uint64_t)native == 0 && v_first % 4 == 0) ? native : 1;
    var.lanes = 256;
    var.upt = (t.ew_upt == 1 || t.ew_upt == 2 || t.ew_upt == 8) ? (int)t.ew_upt : 4;
    return var;
  }
  // Every block starts on a 16-byte boundary iff block_numel is a whole number of units
  // (8-byte gradient words of a 4-element bf16 unit are then aligned as well).
  var.vec = (block_numel % (uint64_t)native == 0) ? native : 1;
  const uint64_t units = block_numel / (uint64_t)var.vec;
  if (units <= (uint64_t)t.row_max_units) {
    // first choice: the smallest team whose units per thread stay within max_upt
    // second choice: the largest allowed team (fewest units per thread) that can hold the block
    for (int pass = 0; pass < 2; ++pass) {
      for (int i = 0; i < 5; ++i) {
        const int lanes = pass == 0 ? kLanes[i] : kLanes[4 - i];
        if (!lanes_allowed(lanes, units, t)) continue;
        const uint64_t need = (units + (uint64_t)lanes - 1) / (uint64_t)lanes;
        if (pass == 0 && need > (uint64_t)t.max_upt) continue;
        const int upt = round_up_upt(lanes, need, var.vec);
        if (upt == 0) continue;
        if (pass == 0 && upt > t.max_upt) continue;
        var.family = AM_FAM_ROW;
        var.lanes = lanes;
        var.upt = upt;
        return var;
      }
    }
  }
  const uint64_t g_bytes = block_numel * (grad_dtype == ADAM_MINI_GRAD_BF16 ? 2u : 4u);
  if (t.lds_max_bytes > 0 && g_bytes <= (uint64_t)t.lds_max_bytes && var.vec > 1) {
    var.family = AM_FAM_ROW_LDS;
    var.lanes = 1024;
    var.upt = 1;
    return var;
  }
  var.family = AM_FAM_LARGE;
  var.lanes = 256;
  var.upt = (t.large_chunk_upt == 1 || t.large_chunk_upt == 2 || t.large_chunk_upt == 8 || t.large_chunk_upt == 16)
                ? (int)t.large_chunk_upt : 4;
  if (var.vec * var.upt > 64) var.upt = 64 / var.vec;  // the partial-sum kernel holds a chunk's gradient in registers
  return var;
}

// The LDS-staged kernel runs ONE workgroup per block and a compute unit holds one or two of them, so its
// launch proceeds in rounds of cu_count workgroups.  With n staged blocks in the list, the last round is
// n - (rounds - 1) * cu_count workgroups wide and the others wait for it: at 288 blocks of 96 KB (the
// query/key heads of a 12-layer, 12-head model with bf16 gradients) the staged kernel takes 22 % longer
// than partial sums / finalize / update, which spread every block over several workgroups, at 256 or
// 512 blocks it is equal or faster.  Staging saves the second read of the gradient: 4 of 24 bytes per
// element with fp32 gradients, 2 of 20 with bf16, so fp32 lists tolerate a worse balance (measured:
// still 2 to 8 % ahead at 288 and 384 blocks).  Lists with fewer staged blocks than compute units
// run in one round and are left alone.
bool am_staging_pays(int grad_dtype, uint64_t n_staged_blocks, const AmTuning& t) {
  if (t.cu_count <= 0 || n_staged_blocks <= (uint64_t)t.cu_count) return true;
  const uint64_t cu = (uint64_t)t.cu_count;
  const uint64_t rounds = (n_staged_blocks + cu - 1) / cu;
  const double balance = (double)n_staged_blocks / (double)(rounds * cu);
  return balance >= (grad_dtype == ADAM_MINI_GRAD_BF16 ? 0.8 : 0.55);
}

// A small list goes through the one-launch generic kernel when every tensor fits it -- contiguous blocks of
// whole 4-element units that one 1024-lane team can hold, or one-element blocks in whole units with a
// 16-byte aligned v slice -- and when that saves launches, i.e. the tuned kernels would need more than one.
// (Descriptors are validated by the caller's loop; invalid ones just answer no.)
bool am_list_is_fusable(int grad_dtype, const adam_mini_tensor_desc* descs, uint32_t n_tensors, const AmTuning& t) {
  if (t.fuse_max_params <= 0) return false;
  uint64_t total = 0, v_next = 0;
  AmVariant first{};
  bool several = false;
  for (uint32_t k = 0; k < n_tensors; ++k) {
    const adam_mini_tensor_desc& d = descs[k];
    if (d.numel == 0 || d.block_numel == 0 || d.numel % d.block_numel != 0) return false;
    total += d.numel;
    if (total > (uint64_t)t.fuse_max_params) return false;
    const uint64_t n_blocks = d.numel / d.block_numel;
    if ((d.flags & ADAM_MINI_FLAG_STRIDED) != 0 && n_blocks > 1 && d.block_numel > 1) return false;
    if (d.block_numel == 1) {
      if (d.numel % 4 != 0 || v_next % 4 != 0) return false;
    } else if (d.block_numel % 4 != 0 || d.block_numel / 4 > (uint64_t)kFusedThreads * kFusedUpt) {
      return false;
    }
    const AmVariant var = am_choose_variant(grad_dtype, d.numel, d.block_numel, v_next, t);
    if (k == 0) first = var;
    else if (!same_variant(first, var)) several = true;
    v_next += n_blocks;
  }
  return several;
}

int am_build_layout(const adam_mini_tensor_desc* descs, uint32_t n_tensors, int grad_dtype,
                    const AmTuning& tuning, AmHostLayout* out) {
  if (!descs || !out || n_tensors == 0) return ADAM_MINI_INVALID_ARG;
  if (grad_dtype != ADAM_MINI_GRAD_F32 && grad_dtype != ADAM_MINI_GRAD_BF16) return ADAM_MINI_INVALID_ARG;
  out->grad_dtype = grad_dtype;
  out->tuning = tuning;
  out->tensors.clear();
  out->buckets.clear();
  const bool fused = am_list_is_fusable(grad_dtype, descs, n_tensors, tuning);
  // variant choice per tensor, with LDS staging switched off for the whole list where it would not pay
  AmTuning choice = tuning;
  if (!fused && tuning.lds_max_bytes > 0) {
    uint64_t n_staged = 0, v_at = 0;
    for (uint32_t k = 0; k < n_tensors; ++k) {
      const adam_mini_tensor_desc& d = descs[k];
      if (d.numel == 0 || d.block_numel == 0 || d.numel % d.block_numel != 0) return ADAM_MINI_INVALID_ARG;
      const uint64_t n_blocks = d.numel / d.block_numel;
      const bool strided = (d.flags & ADAM_MINI_FLAG_STRIDED) != 0 && n_blocks > 1 && d.block_numel > 1;
      if (!strided && am_choose_variant(grad_dtype, d.numel, d.block_numel, v_at, tuning).family == AM_FAM_ROW_LDS)
        n_staged += n_blocks;
      v_at += n_blocks;
    }
    if (!am_staging_pays(grad_dtype, n_staged, tuning)) choice.lds_max_bytes = 0;
  }
  uint64_t fused_item_bytes = 0;
  if (fused) {
    uint64_t total = 0;
    for (uint32_t k = 0; k < n_tensors; ++k) total += descs[k].numel;
    const uint64_t target_items = tuning.fuse_target_items > 0 ? (uint64_t)tuning.fuse_target_items : 1;
    fused_item_bytes = total * (16 + (grad_dtype == ADAM_MINI_GRAD_BF16 ? 2u : 4u)) / target_items;
    if (fused_item_bytes < 32 * 1024) fused_item_bytes = 32 * 1024;
  }
  uint64_t v_next = 0;
  for (uint32_t k = 0; k < n_tensors; ++k) {
    const adam_mini_tensor_desc& d = descs[k];
    if (d.numel == 0 || d.block_numel == 0 || d.numel % d.block_numel != 0) return ADAM_MINI_INVALID_ARG;
    if ((d.flags & ~(uint32_t)(ADAM_MINI_FLAG_STRIDED | ADAM_MINI_REDUCE_MASK)) != 0) return ADAM_MINI_INVALID_ARG;
    if ((d.flags & ADAM_MINI_REDUCE_MASK) > ADAM_MINI_REDUCE_MIN) return ADAM_MINI_INVALID_ARG;
    if (!std::isfinite(d.wd_scale) || d.wd_scale < 0.0f) return ADAM_MINI_INVALID_ARG;
    if (d.numel >= (1ull << 48)) return ADAM_MINI_INVALID_ARG;  // keeps every product below in 64 bits
    AmTensorInfo ti{};
    ti.numel = d.numel;
    ti.block_numel = d.block_numel;
    ti.wd_scale = d.wd_scale;
    ti.n_blocks = d.numel / d.block_numel;
    ti.v_first = v_next;
    v_next += ti.n_blocks;

    // Column blocks of a [block_numel, n_blocks] matrix.  With one column the block is the whole
    // (contiguous) tensor and with one row every element is its own block: both are plain layouts.
    ti.strided = (d.flags & ADAM_MINI_FLAG_STRIDED) != 0 && ti.n_blocks > 1 && d.block_numel > 1;
    AmVariant var{};
    if (fused) {
      var.family = AM_FAM_FUSED;
      var.vec = 4;
      var.lanes = kFusedThreads;
      var.upt = kFusedUpt;
    } else if (ti.strided) {
      const int native = grad_dtype == ADAM_MINI_GRAD_BF16 ? (tuning.bf16_vec == 8 ? 8 : 4) : 4;
      var.family = AM_FAM_STRIDED;
      // a row must be a whole number of units (the per-column step scales are read one float at a time,
      // so the tensor's v slice needs no alignment of its own)
      var.vec = (ti.n_blocks % (uint64_t)native == 0) ? native : 1;
      var.lanes = 256;
      var.upt = (int)tuning.strided_rows;
      // bf16 gradients in 4-element units: two units per lane where every row holds whole pairs, so that the
      // read-only partial pass can take a lane's 8 gradients in one 128-bit load
      var.aux = (grad_dtype == ADAM_MINI_GRAD_BF16 && var.vec == 4 && ti.n_blocks % 8 == 0) ? 2 : 1;
    } else {
      var = am_choose_variant(grad_dtype, d.numel, d.block_numel, ti.v_first, choice);
    }
    int b = -1;
    for (size_t i = 0; i < out->buckets.size(); ++i)
      if (same_variant(out->buckets[i].var, var)) b = (int)i;
    if (b < 0) {
      AmBucket nb;
      nb.var = var;
      out->buckets.push_back(nb);
      b = (int)out->buckets.size() - 1;
    }
    AmBucket& bk = out->buckets[b];

    AmSeg s{};
    s.p = nullptr;
    s.g = nullptr;
    s.m = nullptr;
    s.v_first = ti.v_first;
    s.item_first = (uint32_t)bk.n_items;
    s.block_numel = d.block_numel;
    s.chunks_per_block = 1;
    s.n_blocks = ti.n_blocks;
    s.lblock_first = (uint32_t)bk.n_lblocks;
    s.tensor = k;
    s.wd_scale = d.wd_scale;
    s.reducer = (d.flags & ADAM_MINI_REDUCE_MASK) >> 4;  // same numbering as the kernels' AM_RED_*
    if ((d.flags & ADAM_MINI_REDUCE_MASK) > ADAM_MINI_REDUCE_NORM1) bk.alt_reducer = true;
    uint64_t items = 0;
    if (var.family == AM_FAM_FUSED) {
      if (d.block_numel == 1) {
        s.block_numel = d.numel;
        s.units_per_block = d.numel / 4;
        s.team_lanes = 0;
        items = (s.units_per_block + am_tile_units(var) - 1) / am_tile_units(var);
      } else {
        s.units_per_block = d.block_numel / 4;
        uint32_t team = 16;
        while ((uint64_t)team * kFusedUpt < s.units_per_block) team *= 4;   // 16, 64, 256, 1024
        // blocks per item: enough bytes per workgroup that the whole list makes about fuse_target_items items
        const uint64_t block_bytes = d.block_numel * (16 + (grad_dtype == ADAM_MINI_GRAD_BF16 ? 2u : 4u));
        uint64_t per_item = (fused_item_bytes + block_bytes - 1) / block_bytes;
        const uint64_t cap = (uint64_t)kFusedThreads / team;
        if (per_item > cap) per_item = cap;
        if (per_item < 1) per_item = 1;
        s.team_lanes = team;
        s.blocks_per_item = (uint32_t)per_item;
        items = (ti.n_blocks + per_item - 1) / per_item;
      }
    } else if (var.family == AM_FAM_ELEMENTWISE) {
      s.block_numel = d.numel;
      s.units_per_block = (d.numel + (uint64_t)var.vec - 1) / (uint64_t)var.vec;
      items = (s.units_per_block + am_tile_units(var) - 1) / am_tile_units(var);
    } else if (var.family == AM_FAM_STRIDED) {
      const uint64_t rows = d.block_numel, cols = ti.n_blocks;
      s.row_len = cols;
      s.units_per_block = cols / (uint64_t)var.vec;                        // units per stored row
      const uint64_t group_units = (uint64_t)kStridedThreads * (uint64_t)var.aux;
      const uint64_t groups = (s.units_per_block + group_units - 1) / group_units;          // column groups
      const uint64_t row_chunks = (rows + (uint64_t)var.upt - 1) / (uint64_t)var.upt;       // tiles along the rows
      if (groups >= (1ull << 31) || cols >= (1ull << 31)) return ADAM_MINI_INVALID_ARG;
      s.chunks_per_block = (uint32_t)groups;
      s.aux = bk.n_partials;                                               // partial sums: [row_chunks][cols]
      bk.n_partials += row_chunks * cols;
      bk.n_lblocks += cols;                                                // one step scale per column
      items = row_chunks * groups;
      // the update pass walks the tensor linearly in tiles of its own
      const uint64_t tile = (uint64_t)kStridedThreads * kStridedUpdateUpt;
      bk.item2_first.push_back((uint32_t)bk.n_items2);
      bk.n_items2 += (rows * s.units_per_block + tile - 1) / tile;
      if (bk.n_items2 >= (1ull << 31)) return ADAM_MINI_INVALID_ARG;
    } else if (var.family == AM_FAM_ROW || var.family == AM_FAM_ROW_LDS) {
      s.units_per_block = d.block_numel / (uint64_t)var.vec;
      items = ti.n_blocks;
    } else {
      s.units_per_block = d.block_numel / (uint64_t)var.vec;
      const uint64_t cpb = (s.units_per_block + am_tile_units(var) - 1) / am_tile_units(var);
      if (cpb >= (1ull << 31)) return ADAM_MINI_INVALID_ARG;
      s.chunks_per_block = (uint32_t)cpb;
      if (cpb > bk.max_chunks) bk.max_chunks = cpb;
      items = ti.n_blocks * cpb;
      bk.n_lblocks += ti.n_blocks;
    }
    if (var.family == AM_FAM_ROW_LDS) {
      const uint64_t bytes = d.block_numel * (grad_dtype == ADAM_MINI_GRAD_BF16 ? 2u : 4u);
      if (bytes > bk.lds_bytes) bk.lds_bytes = bytes;
    }
    bk.n_items += items;
    // a launch indexes work items with 32 bits
    if (bk.n_items >= (1ull << 31) || bk.n_lblocks >= (1ull << 31)) return ADAM_MINI_INVALID_ARG;
    ti.bucket = b;
    ti.seg = (int)bk.segs.size();
    bk.segs.push_back(s);
    out->tensors.push_back(ti);
  }
  out->num_blocks = v_next;
  out->n_partials = 0;
  out->n_lblocks = 0;
  out->n_segs = 0;
  for (AmBucket& bk : out->buckets) {
    bk.table_offset = out->n_segs;
    out->n_segs += bk.segs.size();
    if (bk.var.family == AM_FAM_LARGE) {
      bk.slices = large_slices(bk, grad_dtype == ADAM_MINI_GRAD_BF16 ? 2 : 4, tuning);
      if (bk.n_items > out->n_partials) out->n_partials = bk.n_items;
      if (bk.n_lblocks > out->n_lblocks) out->n_lblocks = bk.n_lblocks;
    } else if (bk.var.family == AM_FAM_STRIDED) {
      if (bk.n_partials > out->n_partials) out->n_partials = bk.n_partials;
      if (bk.n_lblocks > out->n_lblocks) out->n_lblocks = bk.n_lblocks;
    }
  }
  return ADAM_MINI_OK;
}
