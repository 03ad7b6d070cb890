"""CPU check that the GPU variant tests leave no shipped kernel instantiation unexercised: the
option sets of variant_cases.CASES (plus the defaults), applied to host-only layouts of the test's
tensor list, must between them select every (family, gradient type, unit width, team, unroll)
combination that the dispatcher in csrc/adam_mini.hip can launch."""
import os
import re

import variant_cases as V
from paper_2406_16793_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAM_EW, FAM_ROW, FAM_LARGE, FAM_ROW_LDS, FAM_STRIDED, FAM_FUSED = 0, 1, 2, 3, 4, 5


def _variant_list(src, name):
    body = re.search(r"#define %s\(X\)(.*?)\n(?!\s*X)" % name, src, re.S).group(1)
    return [(int(a), int(b)) for a, b in re.findall(r"X\((\d+),\s*(\d+)\)", body)]


def _launchable():
    """Instantiations the dispatcher holds, from its variant lists and the two compile-time filters
    (the register budget of the row kernel, the chunk size limit of the multi-workgroup kernels)."""
    src = open(os.path.join(ROOT, "paper_2406_16793_amd", "csrc", "adam_mini.hip")).read()
    assert "upt * vec * 3 + 34 <= (lanes >= 1024 ? 128 : 256)" in src      # am_row_ok, mirrored below
    assert "if constexpr (VEC * U <= 64)" in src                           # launch_large, mirrored below
    rows, large, ew = (_variant_list(src, n) for n in ("AM_ROW_VARIANTS", "AM_LARGE_VARIANTS", "AM_EW_VARIANTS"))
    out = set()
    for grad, vecs in (("f32", (1, 4)), ("bf16", (1, 4, 8))):
        for vec in vecs:
            out |= {(FAM_ROW, grad, vec, l, u) for l, u in rows if u * vec * 3 + 34 <= (128 if l >= 1024 else 256)}
            out |= {(FAM_LARGE, grad, vec, l, u) for l, u in large if vec * u <= 64}
            out |= {(FAM_EW, grad, vec, l, u) for l, u in ew}
            if vec > 1:
                out.add((FAM_ROW_LDS, grad, vec, 1024, 1))
            if vec == 4:
                out.add((FAM_FUSED, grad, vec, 1024, 4))
            out.add((FAM_STRIDED, grad, vec, 256, 1))
            if grad == "bf16" and vec == 4:
                out.add((FAM_STRIDED, grad, vec, 256, 2))          # two units of a row per lane
    return out


def test_variant_cases_reach_every_kernel_instantiation():
    def descs_of(specs):
        return [(s.numel, s.block_numel, s.wd_scale, B.FLAG_STRIDED if s.strided else 0) for s in specs]
    mixed, small = descs_of(V.specs()), descs_of(V.fused_specs())
    reached = set()
    try:
        for cid, opts, grads, descs in ([("default", {}, V.BOTH, mixed)] + [c + (mixed,) for c in V.CASES]
                                        + [c[:3] + (small,) for c in V.FUSED_CASES]):
            for grad in grads:
                B.adam_mini_set_option("reset", 0)
                for k, v in opts.items():
                    B.adam_mini_set_option(k, v)
                h = B.adam_mini_init_layout(descs, B.GRAD_BF16 if grad == "bf16" else B.GRAD_F32, -1)
                for b in B.adam_mini_profile_read(h):
                    upt = b["upt"]
                    if b["family"] == FAM_STRIDED:      # upt holds the tile height (a launch argument); the template
                        upt = int(b["kernel"].rstrip(">").split(",")[-1])   # argument is the units per lane

                    reached.add((b["family"], grad, b["vec"], b["lanes"], upt))
                B.adam_mini_destroy_layout(h)
    finally:
        B.adam_mini_set_option("reset", 0)
    launchable = _launchable()
    assert not (reached - launchable), "layout builder chose variants the dispatcher lacks: %r" % sorted(reached - launchable)
    assert not (launchable - reached), "no variant case exercises: %r" % sorted(launchable - reached)


def test_every_option_key_is_exercised():
    """Every key adam_mini_set_option accepts appears in a variant case or in another GPU test."""
    src = open(os.path.join(ROOT, "paper_2406_16793_amd", "csrc", "adam_mini.hip")).read()
    body = src[src.index("int adam_mini_set_option"):src.index("int adam_mini_init_layout")]
    keys = set(re.findall(r'k == "([a-z0-9_]+)"', body)) - {"reset"}
    used = set()
    for case in V.CASES + V.FUSED_CASES:
        used |= set(case[1])
    other_tests = "".join(open(os.path.join(ROOT, "tests", f)).read() for f in os.listdir(os.path.join(ROOT, "tests"))
                          if f.startswith("test_gpu") or f.startswith("test_zz"))
    missing = {k for k in keys - used if ('"%s"' % k) not in other_tests}
    assert not missing, "option keys without a GPU parity test: %r" % sorted(missing)
