"""Host logic of the C ABI, exercised without a GPU: the library loads, exports
every declared symbol, validates arguments before touching a device, and numbers
the v scalars exactly like the oracle's independent block-index function."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2406_16793_amd import binding as B
from paper_2406_16793_amd import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = []
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if not fn.endswith(".h"):
            continue
        text = open(os.path.join(inc, fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names += re.findall(r"\b(adam_mini_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol():
    lib = B.load()
    declared = _declared_functions()
    assert len(declared) >= 10
    for name in declared:
        assert hasattr(lib, name), "libadam_mini.so does not export %s" % name
    assert sorted(B.EXPORTS) == declared


def test_strerror():
    for code in (0, -1, -2, -3, -4, -5, -99):
        assert isinstance(B.adam_mini_strerror(code), str) and B.adam_mini_strerror(code)


def _init_rc(descs, dtype=B.GRAD_F32, device=-1):
    try:
        h = B.adam_mini_init_layout(descs, dtype, device)
    except B.AdamMiniError as e:
        return e.status
    B.adam_mini_destroy_layout(h)
    return 0


def test_init_layout_validation():
    assert _init_rc([(16, 4, 1.0)]) == 0
    assert _init_rc([]) == B.INVALID_ARG
    assert _init_rc([(0, 1, 1.0)]) == B.INVALID_ARG                 # numel = 0
    assert _init_rc([(16, 0, 1.0)]) == B.INVALID_ARG                # block_numel = 0
    assert _init_rc([(16, 5, 1.0)]) == B.INVALID_ARG                # does not divide
    assert _init_rc([(16, 32, 1.0)]) == B.INVALID_ARG               # block larger than tensor
    assert _init_rc([(16, 4, 1.0, 2)]) == B.INVALID_ARG             # reserved flag bits
    assert _init_rc([(16, 4, 1.0, B.FLAG_STRIDED)]) == 0
    assert _init_rc([(16, 4, float("nan"))]) == B.INVALID_ARG
    assert _init_rc([(16, 4, -1.0)]) == B.INVALID_ARG
    assert _init_rc([(16, 4, 1.0)], dtype=7) == B.INVALID_ARG
    assert _init_rc([(16, 4, 1.0)], device=-2) == B.INVALID_ARG
    lib = B.load()
    assert lib.adam_mini_init_layout(None, 1, 0, -1, ctypes.byref(ctypes.c_void_p())) == B.INVALID_ARG
    assert lib.adam_mini_init_layout((B.TensorDesc * 1)(), 1, 0, -1, None) == B.INVALID_ARG
    assert B.adam_mini_num_blocks(None) == 0 and B.adam_mini_num_tensors(None) == 0
    B.adam_mini_destroy_layout(None)                                 # no-op


def _step_rc(h, n, hp, p=0x1000, g=0x2000, m=0x3000, v=0x4000):
    lib = B.load()
    P, G, M = B.pointer_array([p] * n), B.pointer_array([g] * n), B.pointer_array([m] * n)
    return lib.adam_mini_step(h, P, G, M, ctypes.c_void_p(v), ctypes.byref(hp), None)


def test_step_validation_happens_before_any_device_use():
    h = B.adam_mini_init_layout([(16, 4, 1.0), (8, 8, 0.0)], B.GRAD_F32, -1)
    good = dict(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1)
    hp = lambda **kw: B.HParams(**{**good, **kw})
    # a valid call on a host-only layout gets as far as the device check and no further
    assert _step_rc(h, 2, hp()) == B.NO_DEVICE
    assert _step_rc(h, 2, hp(step=0)) == B.INVALID_ARG
    assert _step_rc(h, 2, hp(beta1=1.0)) == B.INVALID_ARG
    assert _step_rc(h, 2, hp(beta1=-0.1)) == B.INVALID_ARG
    assert _step_rc(h, 2, hp(beta2=1.5)) == B.INVALID_ARG
    assert _step_rc(h, 2, hp(beta2=float("nan"))) == B.INVALID_ARG
    assert _step_rc(h, 2, hp(eps=-1e-8)) == B.INVALID_ARG
    assert _step_rc(h, 2, hp(lr=float("inf"))) == B.INVALID_ARG
    assert _step_rc(h, 2, hp(weight_decay=float("nan"))) == B.INVALID_ARG
    assert _step_rc(h, 2, hp(), p=0) == B.INVALID_ARG               # null entry in a pointer list
    assert _step_rc(h, 2, hp(), p=0x1004) == B.MISALIGNED
    assert _step_rc(h, 2, hp(), g=0x2008) == B.MISALIGNED
    assert _step_rc(h, 2, hp(), v=0x4004) == B.MISALIGNED
    lib = B.load()
    assert lib.adam_mini_step(h, None, None, None, None, None, None) == B.INVALID_ARG
    assert lib.adam_mini_write_block_ids(h, 0, ctypes.c_void_p(0x1000), None) == B.NO_DEVICE
    assert lib.adam_mini_write_block_ids(h, 5, ctypes.c_void_p(0x1000), None) == B.INVALID_ARG
    out = ctypes.c_uint64()
    assert lib.adam_mini_block_id(h, 0, 16, ctypes.byref(out)) == B.INVALID_ARG
    assert lib.adam_mini_block_id(h, 2, 0, ctypes.byref(out)) == B.INVALID_ARG
    B.adam_mini_destroy_layout(h)


def test_set_option_validation():
    with pytest.raises(B.AdamMiniError):
        B.adam_mini_set_option("no_such_key", 1)
    with pytest.raises(B.AdamMiniError):
        B.adam_mini_set_option("row_max_units", -1)
    B.adam_mini_set_option("row_max_units", 1024)
    h = B.adam_mini_init_layout([(4096 * 8, 4096 * 2, 1.0)], B.GRAD_F32, -1)
    assert B.adam_mini_export_layout(h)[1] == [B.PATH_ROW_LDS]      # 32 KB of gradient: staged in LDS
    B.adam_mini_destroy_layout(h)
    B.adam_mini_set_option("lds_max_bytes", 0)
    h = B.adam_mini_init_layout([(4096 * 8, 4096 * 2, 1.0)], B.GRAD_F32, -1)
    assert B.adam_mini_export_layout(h)[1] == [B.PATH_LARGE]
    B.adam_mini_destroy_layout(h)
    with pytest.raises(B.AdamMiniError):
        B.adam_mini_set_option("lds_max_bytes", 200 * 1024)          # more than a compute unit has
    for key in ("xcd_chunk", "xcd_chunk_stream", "xcd_chunk_strided"):
        with pytest.raises(B.AdamMiniError):
            B.adam_mini_set_option(key, 48)                          # not a power of two
        B.adam_mini_set_option(key, 0)
        B.adam_mini_set_option(key, 128)
    B.adam_mini_set_option("reset", 0)
    h = B.adam_mini_init_layout([(4096 * 8, 4096 * 2, 1.0)], B.GRAD_F32, -1)
    assert B.adam_mini_export_layout(h)[1] == [B.PATH_ROW]
    B.adam_mini_destroy_layout(h)


MIXED = [(12, 4, 1.0), (7, 7, 0.0), (30, 1, 1.0), (4, 2, 1.0), (4096 * 3, 4096, 1.0),
         (49152 * 2, 49152, 1.0), (1000, 1, 0.5), (11008 * 2, 11008, 1.0), (3, 3, 0.0)]


@pytest.mark.parametrize("dtype", [B.GRAD_F32, B.GRAD_BF16])
def test_layout_matches_oracle_block_index(oracle, dtype):
    """Bit-exact: v offsets and per-element v indices against the oracle's own function."""
    numel = [d[0] for d in MIXED]
    bnum = [d[1] for d in MIXED]
    h = B.adam_mini_init_layout(MIXED, dtype, -1)
    assert B.adam_mini_num_blocks(h) == oracle.num_blocks(numel, bnum)
    voff, kind = B.adam_mini_export_layout(h)
    for k in range(len(MIXED)):
        assert voff[k] == oracle.block_id(numel, bnum, k, 0)
        want = oracle.block_ids_tensor(numel, bnum, k)
        rng = np.random.default_rng(k)
        probe = set([0, numel[k] - 1]) | set(int(x) for x in rng.integers(0, numel[k], 64))
        for e in probe:
            assert B.adam_mini_block_id(h, k, e) == int(want[e])
    assert kind[2] == B.PATH_ELEMENTWISE and kind[6] == B.PATH_ELEMENTWISE
    # 49152-element blocks: 192 KB of fp32 gradient needs the multi-workgroup path, 96 KB of bf16 fits in LDS
    assert kind[4] == B.PATH_ROW and kind[5] == (B.PATH_LARGE if dtype == B.GRAD_F32 else B.PATH_ROW_LDS)
    B.adam_mini_destroy_layout(h)


@pytest.mark.parametrize("name", ["tiny", "gpt2_small", "llama2_7b", "llama3_8b", "llama2_13b"])
def test_layout_of_benchmark_configs(oracle, name):
    wl = workloads.get(name)
    numel = [s.numel for s in wl.specs]
    bnum = [s.block_numel for s in wl.specs]
    h = B.adam_mini_init_layout([(s.numel, s.block_numel, s.wd_scale) for s in wl.specs],
                                B.GRAD_BF16 if wl.grad_dtype == "bf16" else B.GRAD_F32, -1)
    assert B.adam_mini_num_blocks(h) == wl.n_blocks == oracle.num_blocks(numel, bnum)
    voff, kind = B.adam_mini_export_layout(h)
    assert voff[-1] == wl.n_blocks
    for k in (0, 1, len(numel) // 2, len(numel) - 1):
        assert voff[k] == oracle.block_id(numel, bnum, k, 0)
        e = numel[k] - 1
        assert B.adam_mini_block_id(h, k, e) == oracle.block_id(numel, bnum, k, e)
    if name == "tiny":
        # a small list that the tuned kernels would serve in three launches: one launch of the generic kernel
        assert set(kind) == {B.PATH_FUSED}
        assert len(B.adam_mini_profile_read(h)) == 1
        B.adam_mini_destroy_layout(h)
        return
    for s, kd in zip(wl.specs, kind):
        if "query" in s.name or "key" in s.name:
            assert kd in (B.PATH_LARGE, B.PATH_ROW_LDS) or s.block_numel <= 16384 * 2
        else:
            assert kd == B.PATH_ROW or "wpe" in s.name
    B.adam_mini_destroy_layout(h)


@pytest.mark.parametrize("dtype", [B.GRAD_F32, B.GRAD_BF16])
def test_strided_layout_matches_oracle_block_index(oracle, dtype):
    """Column blocks (ADAM_MINI_FLAG_STRIDED): v numbering against the oracle, bit for bit."""
    descs = [(12, 4, 1.0, 0), (35, 5, 1.0, 1), (64 * 48, 64, 1.0, 1), (30, 1, 1.0, 0), (9, 9, 0.0, 1), (8, 1, 1.0, 1)]
    numel = [d[0] for d in descs]
    bnum = [d[1] for d in descs]
    strided = [bool(d[3]) for d in descs]
    h = B.adam_mini_init_layout(descs, dtype, -1)
    assert B.adam_mini_num_blocks(h) == oracle.num_blocks(numel, bnum)
    voff, kind = B.adam_mini_export_layout(h)
    for k in range(len(descs)):
        want = oracle.block_ids_tensor(numel, bnum, k, strided)
        for e in range(numel[k]):
            assert B.adam_mini_block_id(h, k, e) == int(want[e]), (k, e)
    assert kind[1] == B.PATH_STRIDED and kind[2] == B.PATH_STRIDED
    assert kind[4] == B.PATH_ROW             # one column: the block is the whole contiguous tensor
    assert kind[5] == B.PATH_ELEMENTWISE     # one row: every element its own block
    B.adam_mini_destroy_layout(h)


def test_random_layouts_against_oracle(oracle):
    """Seeded random tensor lists (contiguous, column-block and AdamW-mode tensors of many sizes):
    v numbering bit-exact against the oracle, and every block size lands on a kernel family
    that can hold it."""
    rng = np.random.default_rng(2024)
    for trial in range(40):
        descs = []
        for _ in range(int(rng.integers(1, 12))):
            kind = rng.integers(0, 5)
            if kind == 0:
                bn, nb = 1, int(rng.integers(1, 5000))
            elif kind == 1:
                bn, nb = int(rng.integers(2, 70)), int(rng.integers(1, 200))
            elif kind == 2:
                bn, nb = int(rng.choice([256, 768, 1024, 4096, 5120, 11008, 13824, 14336])), int(rng.integers(1, 40))
            elif kind == 3:
                bn, nb = int(rng.integers(20000, 300000)), int(rng.integers(1, 4))
            else:
                bn, nb = int(rng.integers(1, 40000)), int(rng.integers(1, 6))
            flags = B.FLAG_STRIDED if rng.random() < 0.3 else 0
            descs.append((bn * nb, bn, float(rng.choice([0.0, 1.0])), flags))
        dtype = B.GRAD_BF16 if trial % 2 else B.GRAD_F32
        numel = [d[0] for d in descs]
        bnum = [d[1] for d in descs]
        strided = [bool(d[3]) for d in descs]
        h = B.adam_mini_init_layout(descs, dtype, -1)
        assert B.adam_mini_num_blocks(h) == oracle.num_blocks(numel, bnum)
        voff, kind = B.adam_mini_export_layout(h)
        for k, d in enumerate(descs):
            assert voff[k] == oracle.block_id(numel, bnum, k, 0, strided)
            for e in set([0, d[0] - 1] + [int(x) for x in rng.integers(0, d[0], 16)]):
                assert B.adam_mini_block_id(h, k, e) == oracle.block_id(numel, bnum, k, e, strided)
            nb = d[0] // d[1]
            if d[1] == 1 or (strided[k] and d[1] == 1):
                assert kind[k] == B.PATH_ELEMENTWISE
            elif strided[k] and nb > 1:
                assert kind[k] == B.PATH_STRIDED
            elif d[1] % 4 != 0:
                # scalar-unit fallback: a team holds at most 6144 one-element units
                assert kind[k] == (B.PATH_ROW if d[1] <= 6144 else B.PATH_LARGE)
            elif d[1] <= 24576:
                assert kind[k] == B.PATH_ROW
            else:
                g_bytes = d[1] * (2 if dtype == B.GRAD_BF16 else 4)
                native = 4
                if g_bytes <= 150 * 1024 and d[1] % native == 0:
                    assert kind[k] == B.PATH_ROW_LDS
                else:
                    assert kind[k] == B.PATH_LARGE
        infos = B.adam_mini_profile_read(h)
        assert sum(b["n_tensors"] for b in infos) == len(descs)
        assert sum(b["numel"] for b in infos) == sum(numel)
        assert sum(b["n_blocks"] for b in infos) == B.adam_mini_num_blocks(h)
        B.adam_mini_destroy_layout(h)


def test_reducer_flags_are_validated():
    """Bits 4-6 of the descriptor flags select the block statistic; codes above MIN and other bits are rejected."""
    for name, flag in B.REDUCE_FLAGS.items():
        h = B.adam_mini_init_layout([(4096 * 4, 4096, 1.0, flag), (64, 8, 1.0, flag | B.FLAG_STRIDED)], B.GRAD_BF16, -1)
        assert B.adam_mini_num_blocks(h) == 4 + 8, name
        B.adam_mini_destroy_layout(h)
    for bad in (5 << 4, 7 << 4, 1 << 7, 1 << 1, 1 << 3):
        with pytest.raises(B.AdamMiniError):
            B.adam_mini_init_layout([(4096, 4096, 1.0, bad)], B.GRAD_F32, -1)


def test_static_step_refuses_layouts_beyond_its_scratch_without_touching_a_device():
    """adam_mini_step_static checks the layout's need against ADAM_MINI_STATIC_SCRATCH_BYTES on the host."""
    # column blocks of a [4096, 2^21] matrix: 64 tiles of rows x 2^21 columns of partial sums = 512 MB
    h = B.adam_mini_init_layout([(4096 * (1 << 21), 4096, 1.0, B.FLAG_STRIDED)], B.GRAD_BF16, 0)
    lib = B.load()
    P = B.pointer_array([0x1000])
    hp = B.HParams(1e-3, 0.9, 0.95, 1e-8, 0.1, 1)
    assert lib.adam_mini_step_static(h, P, P, P, ctypes.c_void_p(0x1000), ctypes.byref(hp), None) == B.TOO_LARGE
    assert lib.adam_mini_step_static(h, P, P, P, ctypes.c_void_p(0x1004), ctypes.byref(hp), None) == B.MISALIGNED
    assert lib.adam_mini_step_static(h, None, P, P, ctypes.c_void_p(0x1000), ctypes.byref(hp), None) == B.INVALID_ARG
    B.adam_mini_destroy_layout(h)
    h = B.adam_mini_init_layout([(16, 4, 1.0)], B.GRAD_F32, -1)
    assert lib.adam_mini_step_static(h, P, P, P, ctypes.c_void_p(0x1000), ctypes.byref(hp), None) == B.NO_DEVICE
    B.adam_mini_destroy_layout(h)
    assert "scratch" in B.adam_mini_strerror(B.TOO_LARGE)


def test_small_lists_take_one_launch_only_when_that_saves_launches():
    """The generic one-launch kernel serves a list only if it is small, every block fits one team of it,
    and the tuned kernels would need more than one launch."""
    def kinds(descs, dtype=B.GRAD_F32):
        h = B.adam_mini_init_layout(descs, dtype, -1)
        out = B.adam_mini_export_layout(h)[1]
        n = len(B.adam_mini_profile_read(h))
        B.adam_mini_destroy_layout(h)
        return out, n
    rows, heads, gains, adamw = (1024 * 256, 256, 1.0), (4 * 16384, 16384, 1.0), (256, 256, 0.0), (4096, 1, 1.0)
    assert kinds([rows, heads, gains]) == ([B.PATH_FUSED] * 3, 1)
    assert kinds([adamw, rows, heads]) == ([B.PATH_FUSED] * 3, 1)               # one-element blocks, aligned v slice
    assert kinds([rows, rows]) == ([B.PATH_ROW] * 2, 1)                          # already one launch
    assert kinds([rows, (8 * 16388, 16388, 1.0)])[0][0] == B.PATH_ROW            # a block beyond one team
    assert kinds([rows, (30, 3, 1.0)])[0][0] == B.PATH_ROW                       # not whole 4-element units
    assert kinds([rows, (64 * 48, 64, 1.0, B.FLAG_STRIDED)])[0][0] == B.PATH_ROW  # column blocks
    assert kinds([gains, (3, 1, 1.0), adamw])[0][0] == B.PATH_ROW                # one-element blocks, v slice not aligned
    assert kinds([(1 << 24, 4096, 1.0), heads])[0][0] == B.PATH_ROW              # more than fuse_max_params elements
    B.adam_mini_set_option("fuse_max_params", 0)
    try:
        assert kinds([rows, heads, gains])[1] == 2      # 16-lane teams for the rows and the gains, a 1024-lane team for the heads
    finally:
        B.adam_mini_set_option("reset", 0)


def test_lds_staging_is_dropped_where_its_last_round_of_workgroups_would_be_mostly_empty():
    """One workgroup per staged block: 288 blocks on 256 compute units leave the second round 12 % full."""
    def kinds(descs, dtype):
        h = B.adam_mini_init_layout(descs, dtype, -1)
        out = B.adam_mini_export_layout(h)[1]
        B.adam_mini_destroy_layout(h)
        return out
    head = 64 * 768                                   # 96 KB of bf16 gradient: beyond the registers, within the LDS
    qk = lambda n: [(12 * head, head, 1.0)] * (n // 12)
    rows = (4096 * 768, 768, 1.0)
    assert kinds(qk(288) + [rows], B.GRAD_BF16) == [B.PATH_LARGE] * 24 + [B.PATH_ROW]
    assert kinds(qk(240) + [rows], B.GRAD_BF16) == [B.PATH_ROW_LDS] * 20 + [B.PATH_ROW]      # a single round
    assert kinds(qk(504), B.GRAD_BF16) == [B.PATH_ROW_LDS] * 42                              # 504 / 512
    assert kinds(qk(384), B.GRAD_BF16) == [B.PATH_LARGE] * 32                                # 384 / 512
    assert kinds(qk(2340), B.GRAD_BF16) == [B.PATH_ROW_LDS] * 195                            # 2340 / 2560
    small = 64 * 512                                  # 128 KB of fp32 gradient
    assert kinds([(12 * small, small, 1.0)] * 24, B.GRAD_F32) == [B.PATH_ROW_LDS] * 24       # 288 / 512 is enough with fp32
    assert kinds([(small, small, 1.0)] * 260, B.GRAD_F32) == [B.PATH_LARGE] * 260            # 260 / 512 is not
    B.adam_mini_set_option("cu_count", 0)
    try:
        assert kinds(qk(288), B.GRAD_BF16) == [B.PATH_ROW_LDS] * 24
        B.adam_mini_set_option("cu_count", 96)
        assert kinds(qk(288), B.GRAD_BF16) == [B.PATH_ROW_LDS] * 24                          # three full rounds
    finally:
        B.adam_mini_set_option("reset", 0)


def test_device_hparams_step_validates_on_the_host_what_it_can():
    h = B.adam_mini_init_layout([(16, 4, 1.0)], B.GRAD_F32, -1)
    lib = B.load()
    P = B.pointer_array([0x1000])
    call = lambda p, v, hp, flags: lib.adam_mini_step_device_hparams(h, p, P, P, ctypes.c_void_p(v), ctypes.c_void_p(hp),
                                                                     flags, None)
    assert call(P, 0x1000, 0x2000, 0) == B.NO_DEVICE          # everything checkable passed
    assert call(P, 0x1000, 0, 0) == B.INVALID_ARG             # null hyper-parameter pointer
    assert call(P, 0x1000, 0x2004, 0) == B.MISALIGNED
    assert call(P, 0x1000, 0x2000, 2) == B.INVALID_ARG        # unknown flag
    assert call(P, 0x1004, 0x2000, 0) == B.MISALIGNED
    assert call(None, 0x1000, 0x2000, 1) == B.INVALID_ARG
    B.adam_mini_destroy_layout(h)
    assert ctypes.sizeof(B.HParams) == 32


def test_header_is_plain_c_and_a_c_client_links(tmp_path):
    """include/adam_mini.h is the boundary: it must compile as C99 and as C++11 on its own, and a C program
    that uses nothing else must link against the library and run its host-only calls."""
    import shutil
    import subprocess
    gcc, gxx = shutil.which("gcc"), shutil.which("g++")
    if gcc is None or gxx is None:
        pytest.skip("no gcc / g++")
    header = os.path.join(ROOT, "include", "adam_mini.h")
    for cc, std, lang in ((gcc, "-std=c99", "c"), (gxx, "-std=c++11", "c++")):
        res = subprocess.run([cc, std, "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", lang, header],
                             stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert res.returncode == 0, res.stdout
    src = tmp_path / "client.c"
    src.write_text(r'''
#include <stdio.h>
#include "adam_mini.h"
int main(void) {
  adam_mini_tensor_desc d[2] = {{4096u * 8u, 4096u, 1.0f, 0u}, {256u, 256u, 0.0f, 0u}};
  adam_mini_layout* L = 0;
  uint64_t off[3], id = 0;
  uint32_t kind[2];
  if (adam_mini_init_layout(d, 2, ADAM_MINI_GRAD_BF16, -1, &L) != ADAM_MINI_OK) return 1;
  if (adam_mini_num_blocks(L) != 9 || adam_mini_num_tensors(L) != 2) return 2;
  if (adam_mini_export_layout(L, off, kind) != ADAM_MINI_OK || off[1] != 8 || off[2] != 9) return 3;
  if (adam_mini_block_id(L, 0, 4096u * 3u + 5u, &id) != ADAM_MINI_OK || id != 3) return 4;
  if (adam_mini_init_layout(d, 0, ADAM_MINI_GRAD_BF16, -1, &L) != ADAM_MINI_INVALID_ARG) return 5;
  printf("%s\n", adam_mini_strerror(ADAM_MINI_MISALIGNED));
  return 0;
}
''')
    exe = str(tmp_path / "client")
    libdir = os.path.dirname(B.LIB_PATH)
    res = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-I", os.path.join(ROOT, "include"), str(src), "-o", exe,
                          "-L", libdir, "-ladam_mini", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    run = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    assert run.returncode == 0, (run.returncode, run.stdout)
    assert "16-byte aligned" in run.stdout
