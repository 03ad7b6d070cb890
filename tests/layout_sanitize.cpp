// Host-only checker of the layout builder (csrc/am_layout.cpp), meant to be compiled with
// -fsanitize=address,undefined and run on the CPU by tests/test_layout_sanitized.py.
//
// It builds many layouts -- seeded random tensor lists under random tuning values, the crafted
// lists of the host ABI tests, the size limits, the flag combinations -- and checks, with arithmetic
// of its own, that the work tables cover every element of every tensor exactly once:
//   v offsets are the running count of blocks; every tensor sits in exactly one segment of one
//   bucket; a bucket's item numbering is the prefix sum of its segments' item counts; the unit /
//   chunk / tile counts of a segment tile its blocks with no gap and no overlap; scratch offsets of
//   column-block tensors do not overlap and fit the bucket's total.
// Any out-of-bounds access, overflow or other undefined behaviour inside the builder aborts the run
// through the sanitizers.  Exit status 0 = all checks passed.
#include <cinttypes>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../paper_2406_16793_amd/csrc/am_layout.h"

namespace {

int g_failures = 0;
#define CHECK(cond, ...)                                      \
  do {                                                        \
    if (!(cond)) {                                            \
      ++g_failures;                                           \
      std::fprintf(stderr, "%s:%d: CHECK(%s) failed: ", __FILE__, __LINE__, #cond); \
      std::fprintf(stderr, __VA_ARGS__);                      \
      std::fprintf(stderr, "\n");                             \
    }                                                         \
  } while (0)

struct Rng {  // xorshift64*: the checker's own generator, nothing of the library's
  uint64_t s;
  explicit Rng(uint64_t seed) : s(seed * 0x9E3779B97F4A7C15ull + 1) {}
  uint64_t next() {
    s ^= s >> 12;
    s ^= s << 25;
    s ^= s >> 27;
    return s * 0x2545F4914F6CDD1Dull;
  }
  uint64_t in(uint64_t lo, uint64_t hi) { return lo + next() % (hi - lo + 1); }  // inclusive
  template <typename T, size_t N>
  T pick(const T (&a)[N]) { return a[next() % N]; }
};

uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }

// Every structural property of one built layout.
void check_layout(const std::vector<adam_mini_tensor_desc>& descs, int grad_dtype, const AmTuning& tuning,
                  const AmHostLayout& L, const char* what) {
  CHECK(L.tensors.size() == descs.size(), "%s: tensor count", what);
  if (L.tensors.size() != descs.size()) return;
  uint64_t v_next = 0;
  std::vector<int> seen(descs.size(), 0);
  for (size_t k = 0; k < descs.size(); ++k) {
    const AmTensorInfo& ti = L.tensors[k];
    CHECK(ti.v_first == v_next, "%s: v offset of tensor %zu", what, k);
    CHECK(ti.n_blocks == descs[k].numel / descs[k].block_numel, "%s: block count of tensor %zu", what, k);
    v_next += descs[k].numel / descs[k].block_numel;
    CHECK(ti.bucket >= 0 && (size_t)ti.bucket < L.buckets.size(), "%s: bucket index", what);
    if (ti.bucket < 0 || (size_t)ti.bucket >= L.buckets.size()) return;
    const AmBucket& bk = L.buckets[ti.bucket];
    CHECK(ti.seg >= 0 && (size_t)ti.seg < bk.segs.size(), "%s: segment index", what);
    if (ti.seg < 0 || (size_t)ti.seg >= bk.segs.size()) return;
    CHECK(bk.segs[ti.seg].tensor == k, "%s: segment of tensor %zu names tensor %u", what, k, bk.segs[ti.seg].tensor);
  }
  CHECK(L.num_blocks == v_next, "%s: num_blocks", what);

  uint64_t n_segs = 0;
  for (const AmBucket& bk : L.buckets) {
    const AmVariant& var = bk.var;
    CHECK(bk.table_offset == n_segs, "%s: table offset", what);
    n_segs += bk.segs.size();
    CHECK(!bk.segs.empty(), "%s: empty bucket", what);
    CHECK(var.vec == 1 || var.vec == 4 || (var.vec == 8 && grad_dtype == ADAM_MINI_GRAD_BF16), "%s: vec %d", what, var.vec);
    uint64_t items = 0, items2 = 0, lblocks = 0, partials = 0;
    for (const AmSeg& s : bk.segs) {
      CHECK(s.tensor < descs.size(), "%s: tensor index in segment", what);
      if (s.tensor >= descs.size()) return;
      const adam_mini_tensor_desc& d = descs[s.tensor];
      const AmTensorInfo& ti = L.tensors[s.tensor];
      seen[s.tensor]++;
      CHECK(s.item_first == items, "%s: item_first of tensor %u is %u, want %" PRIu64, what, s.tensor, s.item_first, items);
      CHECK(s.v_first == ti.v_first, "%s: v_first of segment", what);
      CHECK(s.wd_scale == d.wd_scale, "%s: wd_scale", what);
      CHECK(s.reducer == ((d.flags & ADAM_MINI_REDUCE_MASK) >> 4), "%s: reducer", what);
      CHECK(s.n_blocks == ti.n_blocks, "%s: block count of segment", what);
      const uint64_t vec = (uint64_t)var.vec;
      uint64_t seg_items = 0;
      switch (var.family) {
        case AM_FAM_ELEMENTWISE: {
          CHECK(d.block_numel == 1 || (ti.n_blocks > 0 && d.block_numel == 1) || (d.flags & ADAM_MINI_FLAG_STRIDED),
                "%s: elementwise family for block_numel %" PRIu64, what, d.block_numel);
          CHECK(s.block_numel == d.numel, "%s: elementwise segment length", what);
          CHECK(s.units_per_block == ceil_div(d.numel, vec), "%s: elementwise units", what);
          if (vec > 1) CHECK(d.numel % vec == 0 && ti.v_first % 4 == 0, "%s: wide elementwise units need whole units and an aligned v slice", what);
          const uint64_t tile = (uint64_t)var.lanes * (uint64_t)var.upt;
          seg_items = ceil_div(s.units_per_block, tile);
          CHECK(var.lanes == 256 && (var.upt == 1 || var.upt == 2 || var.upt == 4 || var.upt == 8), "%s: elementwise tile", what);
          break;
        }
        case AM_FAM_ROW:
        case AM_FAM_ROW_LDS: {
          CHECK(!ti.strided, "%s: row family for a column-block tensor", what);
          CHECK(s.block_numel == d.block_numel, "%s: row block size", what);
          CHECK(d.block_numel % vec == 0 && s.units_per_block * vec == d.block_numel, "%s: row units", what);
          seg_items = ti.n_blocks;
          if (var.family == AM_FAM_ROW) {
            CHECK(s.units_per_block <= (uint64_t)var.lanes * (uint64_t)var.upt, "%s: block of %" PRIu64 " units in a %dx%d team",
                  what, s.units_per_block, var.lanes, var.upt);
            CHECK(var.upt * var.vec * 3 + 34 <= (var.lanes >= 1024 ? 128 : 256), "%s: register budget of %dx%d vec %d", what,
                  var.lanes, var.upt, var.vec);
            if (var.lanes == 16) CHECK(s.units_per_block <= (uint64_t)tuning.subwave_max_units, "%s: 16-lane team above its limit", what);
            if (var.lanes == 64) CHECK(s.units_per_block <= (uint64_t)tuning.wave_max_units, "%s: wavefront team above its limit", what);
            CHECK(s.units_per_block <= (uint64_t)tuning.row_max_units, "%s: register kernel above row_max_units", what);
          } else {
            const uint64_t bytes = d.block_numel * (grad_dtype == ADAM_MINI_GRAD_BF16 ? 2u : 4u);
            CHECK(vec > 1 && bytes <= (uint64_t)tuning.lds_max_bytes && bytes <= bk.lds_bytes, "%s: staged block of %" PRIu64 " bytes", what, bytes);
          }
          break;
        }
        case AM_FAM_LARGE: {
          CHECK(!ti.strided, "%s: large family for a column-block tensor", what);
          CHECK(d.block_numel % vec == 0 && s.units_per_block * vec == d.block_numel, "%s: large units", what);
          const uint64_t tile = (uint64_t)var.lanes * (uint64_t)var.upt;
          CHECK(var.lanes == 256 && var.vec * var.upt <= 64, "%s: large chunk shape", what);
          CHECK((uint64_t)s.chunks_per_block * tile >= s.units_per_block, "%s: chunks leave a gap", what);
          CHECK((uint64_t)(s.chunks_per_block - 1) * tile < s.units_per_block, "%s: an empty chunk", what);
          CHECK(s.lblock_first == lblocks, "%s: lblock_first", what);
          seg_items = ti.n_blocks * s.chunks_per_block;
          lblocks += ti.n_blocks;
          break;
        }
        case AM_FAM_STRIDED: {
          CHECK(ti.strided && (d.flags & ADAM_MINI_FLAG_STRIDED), "%s: column family for a contiguous tensor", what);
          const uint64_t rows = d.block_numel, cols = ti.n_blocks;
          CHECK(s.block_numel == rows && s.row_len == cols, "%s: stored matrix shape", what);
          CHECK(cols % vec == 0 && s.units_per_block * vec == cols, "%s: units per row", what);
          CHECK(var.upt == (int)tuning.strided_rows && var.upt >= 4, "%s: tile height", what);
          CHECK(var.aux == 1 || (var.aux == 2 && grad_dtype == ADAM_MINI_GRAD_BF16 && var.vec == 4 && s.units_per_block % 2 == 0),
                "%s: units per lane %d", what, var.aux);
          const uint64_t group_units = 256ull * (uint64_t)var.aux;
          CHECK(s.chunks_per_block == ceil_div(s.units_per_block, group_units), "%s: column groups", what);
          const uint64_t row_chunks = ceil_div(rows, (uint64_t)var.upt);
          CHECK(s.aux == partials, "%s: partial-sum offset", what);
          CHECK(s.lblock_first == lblocks, "%s: scale offset", what);
          partials += row_chunks * cols;
          lblocks += cols;
          seg_items = row_chunks * s.chunks_per_block;
          // second numbering: linear tiles of the update pass
          const size_t si = (size_t)(&s - bk.segs.data());
          CHECK(bk.item2_first.size() == bk.segs.size(), "%s: second numbering has %zu entries", what, bk.item2_first.size());
          if (si < bk.item2_first.size()) CHECK(bk.item2_first[si] == items2, "%s: item2_first", what);
          items2 += ceil_div(rows * s.units_per_block, (uint64_t)kStridedThreads * kStridedUpdateUpt);
          break;
        }
        case AM_FAM_FUSED: {
          CHECK(!ti.strided && var.vec == 4 && var.lanes == kFusedThreads && var.upt == kFusedUpt, "%s: fused variant", what);
          CHECK(L.buckets.size() == 1, "%s: a fused list has one bucket", what);
          if (d.block_numel == 1) {
            CHECK(d.numel % 4 == 0 && ti.v_first % 4 == 0, "%s: fused one-element blocks need whole units and an aligned v slice", what);
            CHECK(s.team_lanes == 0 && s.block_numel == d.numel && s.units_per_block * 4 == d.numel, "%s: fused tile tensor", what);
            seg_items = ceil_div(s.units_per_block, (uint64_t)kFusedThreads * kFusedUpt);
          } else {
            const uint64_t team = s.team_lanes, per_item = s.blocks_per_item;
            CHECK(team == 16 || team == 64 || team == 256 || team == 1024, "%s: fused team of %" PRIu64, what, team);
            CHECK(per_item >= 1 && per_item * team <= (uint64_t)kFusedThreads, "%s: %" PRIu64 " blocks per fused item", what, per_item);
            CHECK(d.block_numel % 4 == 0 && s.units_per_block * 4 == d.block_numel && s.block_numel == d.block_numel, "%s: fused units", what);
            CHECK(s.units_per_block <= team * kFusedUpt, "%s: fused block of %" PRIu64 " units in a team of %" PRIu64, what, s.units_per_block, team);
            CHECK(team == 16 || s.units_per_block > (team / 4) * kFusedUpt, "%s: fused team larger than needed", what);
            seg_items = per_item ? ceil_div(ti.n_blocks, per_item) : 0;
          }
          break;
        }
        default:
          CHECK(false, "%s: unknown family %d", what, var.family);
      }
      items += seg_items;
    }
    CHECK(bk.n_items == items, "%s: bucket items %" PRIu64 " want %" PRIu64, what, bk.n_items, items);
    CHECK(bk.n_items < (1ull << 31), "%s: item count beyond 31 bits", what);
    if (var.family == AM_FAM_LARGE) {
      CHECK(bk.n_lblocks == lblocks, "%s: large blocks", what);
      CHECK(L.n_partials >= bk.n_items && L.n_lblocks >= bk.n_lblocks, "%s: scratch of a large bucket", what);
      // the slices tile the bucket's items and blocks in order, and respect the byte limit unless one block exceeds it
      uint64_t it = 0, lb = 0;
      for (const AmSlice& sl : bk.slices) {
        CHECK(sl.item_first == it && sl.lblock_first == lb && sl.n_items > 0 && sl.n_lblocks > 0, "%s: slice order", what);
        it += sl.n_items;
        lb += sl.n_lblocks;
      }
      CHECK(it == bk.n_items && lb == bk.n_lblocks, "%s: slices cover %" PRIu64 " of %" PRIu64 " items", what, it, bk.n_items);
      if (tuning.large_slice_mb <= 0) CHECK(bk.slices.size() == 1, "%s: unsliced bucket in %zu slices", what, bk.slices.size());
    }
    if (var.family == AM_FAM_STRIDED) {
      CHECK(bk.n_lblocks == lblocks && bk.n_partials == partials, "%s: column scratch", what);
      CHECK(bk.n_items2 == items2 && bk.n_items2 < (1ull << 31), "%s: update-pass items", what);
      CHECK(L.n_partials >= bk.n_partials && L.n_lblocks >= bk.n_lblocks, "%s: scratch of a column bucket", what);
    }
  }
  CHECK(L.n_segs == n_segs && n_segs == descs.size(), "%s: segment total", what);
  if (!L.buckets.empty() && L.buckets[0].var.family == AM_FAM_FUSED) {
    uint64_t total = 0;
    for (const adam_mini_tensor_desc& d : descs) total += d.numel;
    CHECK(tuning.fuse_max_params > 0 && total <= (uint64_t)tuning.fuse_max_params, "%s: fused list of %" PRIu64 " elements", what, total);
  }
  for (size_t k = 0; k < descs.size(); ++k) CHECK(seen[k] == 1, "%s: tensor %zu in %d segments", what, k, seen[k]);
}

int build(const std::vector<adam_mini_tensor_desc>& descs, int grad_dtype, const AmTuning& tuning, const char* what,
          bool check = true) {
  AmHostLayout L;
  const int rc = am_build_layout(descs.data(), (uint32_t)descs.size(), grad_dtype, tuning, &L);
  if (rc == ADAM_MINI_OK && check) check_layout(descs, grad_dtype, tuning, L, what);
  return rc;
}

adam_mini_tensor_desc desc(uint64_t n_blocks, uint64_t block_numel, float wd = 1.0f, uint32_t flags = 0) {
  adam_mini_tensor_desc d;
  d.numel = n_blocks * block_numel;
  d.block_numel = block_numel;
  d.wd_scale = wd;
  d.flags = flags;
  return d;
}

AmTuning random_tuning(Rng& r) {
  AmTuning t;
  const int64_t vecs[] = {4, 8}, lanes[] = {256, 512, 1024}, upts[] = {1, 2, 3, 4, 6, 8, 12, 16};
  const int64_t chunk_upt[] = {1, 2, 4, 8, 16}, ew_upt[] = {1, 2, 4, 8}, rows[] = {4, 16, 20, 64, 256, 4096};
  t.bf16_vec = r.pick(vecs);
  t.subwave_max_units = (int64_t)r.in(0, 80);
  t.wave_max_units = (int64_t)r.in(0, 1200);
  t.team_max_lanes = r.pick(lanes);
  t.max_upt = r.pick(upts);
  t.row_max_units = r.in(0, 3) == 0 ? (int64_t)r.in(1, 8000) : (1 << 30);
  t.lds_max_bytes = r.in(0, 2) == 0 ? 0 : (int64_t)r.in(1024, 159 * 1024);
  t.large_chunk_upt = r.pick(chunk_upt);
  t.ew_upt = r.pick(ew_upt);
  t.strided_rows = r.pick(rows);
  t.fuse_max_params = r.in(0, 3) == 0 ? 0 : (int64_t)r.in(1, 40000000);
  t.fuse_target_items = (int64_t)r.in(1, 2000);
  t.large_slice_mb = r.in(0, 2) == 0 ? (int64_t)r.in(1, 4) : 0;
  return t;
}

void random_layouts() {
  Rng r(2024);
  const uint64_t shapes[] = {256, 768, 1024, 4096, 5120, 11008, 13824, 14336};
  for (int trial = 0; trial < 400; ++trial) {
    std::vector<adam_mini_tensor_desc> descs;
    const int n = (int)r.in(1, 14);
    for (int i = 0; i < n; ++i) {
      uint64_t bn, nb;
      switch (r.in(0, 4)) {
        case 0: bn = 1; nb = r.in(1, 5000); break;
        case 1: bn = r.in(2, 70); nb = r.in(1, 200); break;
        case 2: bn = r.pick(shapes); nb = r.in(1, 40); break;
        case 3: bn = r.in(20000, 300000); nb = r.in(1, 4); break;
        default: bn = r.in(1, 40000); nb = r.in(1, 6); break;
      }
      uint32_t flags = r.in(0, 9) < 3 ? ADAM_MINI_FLAG_STRIDED : 0;
      flags |= (uint32_t)r.in(0, 4) << 4;
      descs.push_back(desc(nb, bn, r.in(0, 1) ? 1.0f : 0.0f, flags));
    }
    const AmTuning t = trial % 4 == 0 ? AmTuning() : random_tuning(r);
    char what[64];
    std::snprintf(what, sizeof what, "random layout %d", trial);
    const int rc = build(descs, trial % 2 ? ADAM_MINI_GRAD_BF16 : ADAM_MINI_GRAD_F32, t, what);
    CHECK(rc == ADAM_MINI_OK, "%s: rc %d", what, rc);
  }
}

// Small lists of whole 4-element units: the ones the one-launch generic kernel may serve.
void small_regular_layouts() {
  Rng r(99);
  const uint64_t blocks[] = {4, 8, 64, 256, 260, 1024, 1028, 4096, 4100, 11008, 16384, 16388};
  int fused = 0;
  for (int trial = 0; trial < 300; ++trial) {
    std::vector<adam_mini_tensor_desc> descs;
    const int n = (int)r.in(1, 10);
    for (int i = 0; i < n; ++i) {
      if (r.in(0, 5) == 0) descs.push_back(desc(4 * r.in(1, 3000), 1));
      else descs.push_back(desc(r.in(1, 300), r.pick(blocks), 1.0f, (uint32_t)r.in(0, 4) << 4));
    }
    const AmTuning t = trial % 3 == 0 ? AmTuning() : random_tuning(r);
    AmHostLayout L;
    char what[64];
    std::snprintf(what, sizeof what, "small list %d", trial);
    const int g = trial % 2 ? ADAM_MINI_GRAD_BF16 : ADAM_MINI_GRAD_F32;
    const int rc = am_build_layout(descs.data(), (uint32_t)descs.size(), g, t, &L);
    CHECK(rc == ADAM_MINI_OK, "%s: rc %d", what, rc);
    if (rc != ADAM_MINI_OK) continue;
    check_layout(descs, g, t, L, what);
    if (L.buckets[0].var.family == AM_FAM_FUSED) ++fused;
  }
  CHECK(fused > 30, "only %d of 300 small lists took the one-launch kernel", fused);
}

void crafted_layouts() {
  // the list of the host ABI test, and a list of every family with column blocks and statistics
  std::vector<adam_mini_tensor_desc> mixed = {desc(3, 4), desc(1, 7, 0.0f), desc(30, 1), desc(2, 2), desc(3, 4096),
                                              desc(2, 49152), desc(1000, 1, 0.5f), desc(2, 11008), desc(1, 3, 0.0f)};
  std::vector<adam_mini_tensor_desc> cols = {desc(4, 3), desc(5, 7, 1.0f, ADAM_MINI_FLAG_STRIDED),
                                             desc(64, 48, 1.0f, ADAM_MINI_FLAG_STRIDED | ADAM_MINI_REDUCE_MAX), desc(30, 1),
                                             desc(1, 9, 0.0f, ADAM_MINI_FLAG_STRIDED), desc(8, 1, 1.0f, ADAM_MINI_FLAG_STRIDED),
                                             desc(32000, 4096, 1.0f, ADAM_MINI_FLAG_STRIDED), desc(1001, 17, 1.0f, ADAM_MINI_FLAG_STRIDED)};
  for (int g : {ADAM_MINI_GRAD_F32, ADAM_MINI_GRAD_BF16}) {
    CHECK(build(mixed, g, AmTuning(), "mixed list") == ADAM_MINI_OK, "mixed list rejected");
    CHECK(build(cols, g, AmTuning(), "column list") == ADAM_MINI_OK, "column list rejected");
  }
  // the five benchmark shapes' block sizes, thousands of tensors
  std::vector<adam_mini_tensor_desc> many;
  Rng r(7);
  for (int i = 0; i < 3000; ++i) many.push_back(desc(r.in(1, 9), r.in(1, 1100), 1.0f, 0));
  CHECK(build(many, ADAM_MINI_GRAD_BF16, AmTuning(), "3000 tensors") == ADAM_MINI_OK, "3000 tensors rejected");
}

void limits_and_flags() {
  const AmTuning t;
  AmHostLayout L;
  CHECK(am_build_layout(nullptr, 1, 0, t, &L) == ADAM_MINI_INVALID_ARG, "null descriptors accepted");
  std::vector<adam_mini_tensor_desc> one = {desc(4, 4)};
  CHECK(am_build_layout(one.data(), 0, 0, t, &L) == ADAM_MINI_INVALID_ARG, "zero tensors accepted");
  CHECK(am_build_layout(one.data(), 1, 7, t, &L) == ADAM_MINI_INVALID_ARG, "unknown gradient type accepted");
  CHECK(am_build_layout(one.data(), 1, 0, t, nullptr) == ADAM_MINI_INVALID_ARG, "null output accepted");
  auto rejected = [&](adam_mini_tensor_desc d, const char* why) {
    std::vector<adam_mini_tensor_desc> v = {desc(3, 5), d};
    CHECK(build(v, ADAM_MINI_GRAD_BF16, t, why) == ADAM_MINI_INVALID_ARG, "%s accepted", why);
  };
  adam_mini_tensor_desc d = desc(4, 4);
  d.numel = 0; rejected(d, "numel 0");
  d = desc(4, 4); d.block_numel = 0; rejected(d, "block_numel 0");
  d = desc(4, 4); d.block_numel = 5; rejected(d, "block_numel not dividing numel");
  d = desc(4, 4); d.block_numel = 32; rejected(d, "block larger than the tensor");
  d = desc(4, 4); d.flags = 2; rejected(d, "reserved flag bit 1");
  d = desc(4, 4); d.flags = 1u << 7; rejected(d, "reserved flag bit 7");
  d = desc(4, 4); d.flags = 5u << 4; rejected(d, "statistic code 5");
  d = desc(4, 4); d.wd_scale = -1.0f; rejected(d, "negative wd_scale");
  d = desc(4, 4); d.wd_scale = 0.0f / 0.0f; rejected(d, "NaN wd_scale");
  // sizes at the 2^31 work-item and 2^48 element limits (no memory is touched: host tables only)
  rejected(desc(1ull << 31, 4), "2^31 row blocks in one bucket");
  rejected(desc(1ull << 44, 1), "2^31 elementwise tiles");
  rejected(desc(1, 1ull << 48), "2^48 elements");
  rejected(desc(1ull << 33, 4096, 1.0f, ADAM_MINI_FLAG_STRIDED), "2^33 columns");
  for (int g : {ADAM_MINI_GRAD_F32, ADAM_MINI_GRAD_BF16}) {
    std::vector<adam_mini_tensor_desc> big = {desc((1ull << 31) - 1, 4), desc(1, (1ull << 48) - 4096),
                                              desc(1ull << 30, 1), desc((1ull << 30) + 8, 8192, 1.0f, ADAM_MINI_FLAG_STRIDED),
                                              desc(1u << 20, 1ull << 20), desc(3, (1ull << 40) + 4)};
    for (size_t i = 0; i < big.size(); ++i) {
      std::vector<adam_mini_tensor_desc> v = {desc(7, 64), big[i], desc(3, 256)};
      char what[64];
      std::snprintf(what, sizeof what, "large case %zu", i);
      const int rc = build(v, g, t, what);
      CHECK(rc == ADAM_MINI_OK || rc == ADAM_MINI_INVALID_ARG, "%s: rc %d", what, rc);
    }
    // two buckets' worth of items just below the limit each, then one more tensor tips a bucket over
    std::vector<adam_mini_tensor_desc> two = {desc((1ull << 30), 4), desc((1ull << 30) - 1, 4)};
    CHECK(build(two, g, t, "2^31 - 1 items") == ADAM_MINI_OK, "2^31 - 1 items rejected");
    two.push_back(desc(1, 4));
    CHECK(build(two, g, t, "2^31 items") == ADAM_MINI_INVALID_ARG, "2^31 items accepted");
  }
}

}  // namespace

int main() {
  random_layouts();
  small_regular_layouts();
  crafted_layouts();
  limits_and_flags();
  if (g_failures) {
    std::fprintf(stderr, "%d check(s) failed\n", g_failures);
    return 1;
  }
  std::printf("layout checks passed\n");
  return 0;
}
