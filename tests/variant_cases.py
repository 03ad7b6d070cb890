"""The option sets under which the GPU variant tests (test_gpu_variants.py) step the mixed tensor
list, and that list itself.  Kept in a module of its own so that a CPU test can check, on host-only
layouts, that these option sets between them reach every kernel instantiation the dispatcher of
csrc/adam_mini.hip can launch."""
from __future__ import annotations

# (n_blocks, block_numel[, wd_scale])
ROWS = [(5, 8), (70, 64), (33, 128), (9, 256), (5, 264), (6, 768), (4, 1024), (3, 2048), (5, 3072), (6, 4096),
        (3, 5120), (2, 8192), (3, 11008), (2, 14336), (1, 16384), (2, 20480), (1, 24576), (1, 4096, 0.0)]
ODD = [(4, 2), (5, 3), (6, 7), (3, 25), (3, 63), (3, 101), (2, 201), (2, 257), (2, 501), (2, 601), (2, 1001),
       (1, 1501), (1, 2001), (1, 3001), (1, 4001), (2, 4099), (1, 5001), (1, 6001), (1, 9001)]
STAGED = [(3, 24580), (2, 32768), (1, 38400)]                    # gradient fits in LDS, block not in registers
LARGE = [(2, 16392 * 4), (3, 49152 * 2), (1, 524288), (2, 20001 * 5), (1, 40000 * 8)]
ADAMW_ALIGNED = [(4096 * 8, 1)]                                  # first in the list: its v slice starts at 0
ADAMW = [(1000, 1), (4096 * 5, 1), (7, 1), (1025 * 8, 1), (3, 1, 0.0)]
COLUMNS = [(1024, 64), (1000, 33), (1001, 17), (260, 3), (2048, 130), (8, 8)]   # (columns, rows) of a stored [rows, columns]


def specs():
    from paper_2406_16793_amd.partition import TensorSpec
    out = []
    for i, b in enumerate(ADAMW_ALIGNED + ROWS + ODD + STAGED + LARGE + ADAMW):
        out.append(TensorSpec("t%d" % i, (b[0], b[1]), b[1], b[2] if len(b) > 2 else 1.0))
    for i, b in enumerate(COLUMNS):
        out.append(TensorSpec("c%d" % i, (b[1], b[0]), b[1], 1.0, True))
    return out


# A small list of whole 4-element units whose blocks each fit one 1024-lane team: the kind the one-launch
# generic kernel serves (teams of 64, 256 and 1024 lanes, one-element blocks with an aligned v slice first).
FUSED_LIST = [(4096 * 3, 1), (300, 64), (1030, 256), (70, 260), (33, 768), (40, 1024), (9, 1028), (5, 4096),
              (3, 4100), (3, 11008), (5, 16384), (2, 16380), (1, 4096, 0.0), (67, 8), (8 * 513, 1)]


def fused_specs(reducers=("mean",)):
    from paper_2406_16793_amd.partition import TensorSpec
    return [TensorSpec("f%d" % i, (b[0], b[1]), b[1], b[2] if len(b) > 2 else 1.0, False, reducers[i % len(reducers)])
            for i, b in enumerate(FUSED_LIST)]


def _o(**kw):
    return dict(kw)


# (id, options, gradient types)
BOTH = ("f32", "bf16")
CASES = [
    # the grid-stride loop of every kernel: several work-item groups per workgroup
    ("grid_cap=1", _o(grid_cap=1), BOTH),
    ("grid_cap=7", _o(grid_cap=7), BOTH),
    ("grid_cap=64", _o(grid_cap=64), BOTH),
    ("grid_cap=3-wide-teams", _o(grid_cap=3, team_max_lanes=512, max_upt=16, row_blocked=1), BOTH),
    ("grid_cap=16-vec8", _o(grid_cap=16, bf16_vec=8, large_chunk_upt=8, ew_upt=8), ("bf16",)),
    ("grid_cap=5-upt1", _o(grid_cap=5, max_upt=1), BOTH),
    # 8-element units with bf16 gradients, in every family and team shape
    ("bf16_vec=8", _o(bf16_vec=8), ("bf16",)),
    ("bf16_vec=8-upt1", _o(bf16_vec=8, max_upt=1, large_chunk_upt=1, ew_upt=1), ("bf16",)),
    ("bf16_vec=8-upt2", _o(bf16_vec=8, max_upt=2, large_chunk_upt=2, ew_upt=2), ("bf16",)),
    ("bf16_vec=8-upt16-256", _o(bf16_vec=8, max_upt=16, team_max_lanes=256, wave_max_units=1024), ("bf16",)),
    ("bf16_vec=8-512", _o(bf16_vec=8, team_max_lanes=512, row_blocked=1), ("bf16",)),
    ("bf16_vec=8-no-small-teams", _o(bf16_vec=8, subwave_max_units=0, wave_max_units=0), ("bf16",)),
    # blocked unit map
    ("row_blocked", _o(row_blocked=1), BOTH),
    ("row_blocked-256-upt16", _o(row_blocked=1, max_upt=16, team_max_lanes=256), BOTH),
    # chunk / tile sizes of the streaming families
    ("large_chunk_upt=1", _o(large_chunk_upt=1), BOTH),
    ("large_chunk_upt=2", _o(large_chunk_upt=2), BOTH),
    ("large_chunk_upt=8", _o(large_chunk_upt=8), BOTH),
    ("large_chunk_upt=16", _o(large_chunk_upt=16), BOTH),
    ("large_slice_mb=1", _o(large_slice_mb=1), BOTH),               # the multi-workgroup bucket in several slices
    ("large_slice_mb=2-keep", _o(large_slice_mb=2, large_keep_g=1, grid_cap=3, large_chunk_upt=2), BOTH),
    ("large_keep_g", _o(large_keep_g=1), ("bf16",)),
    ("large_wide_chunks=1", _o(large_wide_chunks=1), BOTH),         # a workgroup per block sums the chunk partials
    ("large_wide_chunks=1-small-chunks", _o(large_wide_chunks=1, large_chunk_upt=1, grid_cap=2), BOTH),
    ("large_wide_chunks=0", _o(large_wide_chunks=0), ("f32",)),
    ("ew_upt=1", _o(ew_upt=1), BOTH),
    ("ew_upt=2", _o(ew_upt=2), BOTH),
    ("ew_upt=8", _o(ew_upt=8), BOTH),
    # team shapes of the register kernel
    ("team_max_lanes=256", _o(team_max_lanes=256), BOTH),
    ("team_max_lanes=512", _o(team_max_lanes=512), BOTH),
    ("max_upt=1", _o(max_upt=1), BOTH),
    ("max_upt=4", _o(max_upt=4), BOTH),
    ("max_upt=3", _o(max_upt=3), BOTH),
    ("max_upt=16", _o(max_upt=16), BOTH),
    ("max_upt=16-wide-waves", _o(max_upt=16, wave_max_units=1024), BOTH),
    ("max_upt=8-wide-waves-512", _o(max_upt=8, wave_max_units=512, team_max_lanes=512), BOTH),
    ("max_upt=6", _o(max_upt=6), BOTH),
    ("max_upt=12-256", _o(max_upt=12, team_max_lanes=256), BOTH),
    # thresholds between the families
    ("subwave_max_units=0", _o(subwave_max_units=0), BOTH),
    ("subwave_max_units=16", _o(subwave_max_units=16), BOTH),
    ("wave_max_units=0", _o(wave_max_units=0), BOTH),
    ("no-small-teams", _o(subwave_max_units=0, wave_max_units=0), BOTH),
    ("row_max_units=64", _o(row_max_units=64), BOTH),
    ("row_max_units=1024-no-lds", _o(row_max_units=1024, lds_max_bytes=0), BOTH),
    ("lds_max_bytes=0", _o(lds_max_bytes=0), BOTH),
    ("lds_max_bytes=100K", _o(lds_max_bytes=100 * 1024), BOTH),
    ("cu_count=4", _o(cu_count=4), BOTH),          # 6 staged blocks on "4 compute units": badly balanced, not staged
    ("cu_count=3", _o(cu_count=3), BOTH),          # two full rounds: staged
    ("cu_count=0", _o(cu_count=0), ("bf16",)),     # balance never considered
    # occupancy caps (dynamic LDS the kernels never touch) and XCD run lengths: launch shape only
    ("row_wg_per_cu=1", _o(row_wg_per_cu=1), ("bf16",)),
    ("row_wg_per_cu=3", _o(row_wg_per_cu=3), ("f32",)),
    ("row_inflight_kb=0", _o(row_inflight_kb=0), ("bf16",)),
    ("row_inflight_kb=16", _o(row_inflight_kb=16), ("f32",)),
    ("ew_wg_per_cu=0", _o(ew_wg_per_cu=0), ("bf16",)),
    ("ew_wg_per_cu=1", _o(ew_wg_per_cu=1), ("f32",)),
    ("stream_wg_per_cu=0", _o(stream_wg_per_cu=0), ("bf16",)),
    ("stream_wg_per_cu=1", _o(stream_wg_per_cu=1), ("f32",)),
    ("stream_wg_per_cu=8", _o(stream_wg_per_cu=8), ("bf16",)),
    ("strided_wg_per_cu=0", _o(strided_wg_per_cu=0), ("bf16",)),
    ("strided_wg_per_cu=1", _o(strided_wg_per_cu=1), ("f32",)),
    ("strided_rows=4", _o(strided_rows=4), BOTH),
    ("strided_rows=16", _o(strided_rows=16), ("bf16",)),
    ("strided_rows=20", _o(strided_rows=20), BOTH),
    ("strided_rows=256", _o(strided_rows=256), ("f32",)),
    ("strided_rows=4096-vec8", _o(strided_rows=4096, bf16_vec=8), ("bf16",)),
    ("xcd_count=1", _o(xcd_count=1, xcd_chunk=2, xcd_chunk_stream=2, xcd_chunk_strided=2), ("bf16",)),
    ("xcd_count=2", _o(xcd_count=2, xcd_chunk=2, xcd_chunk_stream=4, xcd_chunk_strided=1), ("f32",)),
    ("xcd_count=4", _o(xcd_count=4, xcd_chunk=4, xcd_chunk_stream=2, xcd_chunk_strided=2), ("bf16",)),
    ("xcd_count=16", _o(xcd_count=16, xcd_chunk=1, xcd_chunk_stream=1, xcd_chunk_strided=1), ("f32",)),
    ("xcd_chunks=1", _o(xcd_chunk=1, xcd_chunk_stream=1, xcd_chunk_strided=1), ("bf16",)),
    ("xcd_chunks=0", _o(xcd_chunk=0, xcd_chunk_stream=0, xcd_chunk_strided=0), ("f32",)),
]


# (id, options, gradient types, block statistics) for the small list above
FUSED_CASES = [
    ("fused", _o(), BOTH, ("mean",)),
    ("fused-grid_cap=1", _o(grid_cap=1), BOTH, ("mean",)),
    ("fused-grid_cap=5", _o(grid_cap=5), BOTH, ("mean", "max", "norm2", "min", "norm1")),
    ("fused-statistics", _o(), BOTH, ("max", "norm2", "mean", "min", "norm1")),
    ("fused-one-block-per-item", _o(fuse_target_items=100000), BOTH, ("mean", "max")),
    ("fused-full-items", _o(fuse_target_items=1), BOTH, ("norm2", "mean")),
    ("fused-16-items-grid_cap=2", _o(fuse_target_items=16, grid_cap=2), ("bf16",), ("mean", "min")),
    ("fused-off", _o(fuse_max_params=0), BOTH, ("mean",)),
    ("fused-limit-below-the-list", _o(fuse_max_params=100000), ("bf16",), ("mean",)),
]


def instantiations(buckets, grad_dtype):
    """Kernel instantiations a list of adam_mini_bucket_info dicts launches: (family, grad, vec, lanes, upt)."""
    return {(b["family"], grad_dtype, b["vec"], b["lanes"], b["upt"]) for b in buckets}
