"""Pins for the CPU oracle: each check compares the oracle with something that is
NOT the oracle -- a library routine, a closed form, an identity, a hand-worked
example or a brute-force transcription of the paper's partition listing.

Every function takes an ``oracle.OracleLib`` and raises AssertionError when the
pin does not hold, so the same checks can be run against deliberately broken
copies of the oracle (tests/test_oracle_mutants.py) to show that they bite.
"""
from __future__ import annotations

import math
import os
from fractions import Fraction

import numpy as np

import oracle as orc

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _close(a, b, rtol, atol=0.0, what=""):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    err = np.abs(a - b)
    tol = atol + rtol * np.abs(b)
    if not np.all(err <= tol) or not np.all(np.isfinite(a) == np.isfinite(b)):
        i = int(np.argmax(err - tol))
        raise AssertionError("%s: got %r want %r (idx %d, max err %g)"
                             % (what, a.flat[i], b.flat[i], i, float(err.max())))


# ---------------------------------------------------------------------------
# P0: hand-worked example (tests/golden/hand_worked_block.txt), exact fractions
# ---------------------------------------------------------------------------
def pin_hand_worked(lib):
    rows = []
    with open(os.path.join(GOLDEN, "hand_worked_block.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            rows.append((int(tok[0]), [float(Fraction(x)) for x in tok[1:]]))
    hp = orc.Hyper(lr=0.5, beta1=0.5, beta2=0.5, eps=0.0, weight_decay=0.5)
    grads = {1: [2.0, -2.0, 2.0], 2: [1.0, -4.0, 7.0]}
    p = np.ones(3)
    m = np.zeros(3)
    v = np.zeros(1)
    for t, want in rows:
        lib.step_tensor(p, m, v, np.array(grads[t], dtype=np.float64), 3, hp, t)
        _close(p, want[0:3], 1e-15, 1e-16, "hand-worked param t=%d" % t)
        _close(m, want[3:6], 1e-15, 1e-16, "hand-worked m t=%d" % t)
        _close(v, want[6:7], 1e-15, 1e-16, "hand-worked v t=%d" % t)


# ---------------------------------------------------------------------------
# P1: block size 1 is AdamW (Section 2.3: Adam-mini replaces g*g by its block
# mean; with one element per block the mean is g*g itself).  Compared with
# PyTorch's own CPU AdamW in float64, a library routine.
# ---------------------------------------------------------------------------
def pin_adamw_reduction(lib):
    import torch
    rng = np.random.default_rng(11)
    n = 37
    hp = orc.Hyper(lr=3e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    p0 = rng.normal(0, 0.5, n)
    p = p0.copy()
    m = np.zeros(n)
    v = np.zeros(n)
    tp = torch.nn.Parameter(torch.tensor(p0, dtype=torch.float64))
    opt = torch.optim.AdamW([tp], lr=hp.lr, betas=(hp.beta1, hp.beta2), eps=hp.eps,
                            weight_decay=hp.weight_decay, amsgrad=False, foreach=False)
    for t in range(1, 8):
        g = rng.normal(0, 10.0 ** rng.uniform(-4, 0), n)
        lib.step_tensor(p, m, v, g, 1, hp, t)
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        st = opt.state[tp]
        _close(p, tp.detach().numpy(), 1e-12, 1e-15, "AdamW param t=%d" % t)
        _close(m, st["exp_avg"].numpy(), 1e-12, 1e-18, "AdamW m t=%d" % t)
        _close(v, st["exp_avg_sq"].numpy(), 1e-12, 1e-24, "AdamW v t=%d" % t)


# ---------------------------------------------------------------------------
# P2: constant gradient over steps.  From Algorithm 1: m_t = (1-b1^t) g, so
# m_hat = g; v_t = (1-b2^t) mean(g^2), so v_hat = mean(g^2).  Hence with
# a = 1 - lr*lambda and u = g / (rms(g) + eps):
#     param_t = a^t param_0 - lr * u * (1 - a^t)/(1 - a)
# ---------------------------------------------------------------------------
def pin_constant_gradient(lib):
    rng = np.random.default_rng(5)
    for lam in (0.1, 0.0):
        hp = orc.Hyper(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=lam)
        nb, bs = 4, 6
        g = rng.normal(0, 1e-2, nb * bs)
        p0 = rng.normal(0, 1.0, nb * bs)
        p, m, v = p0.copy(), np.zeros(nb * bs), np.zeros(nb)
        msq = (g.reshape(nb, bs) ** 2).mean(axis=1)
        u = g / np.repeat(np.sqrt(msq) + hp.eps, bs)
        a = 1.0 - hp.lr * lam
        for t in range(1, 13):
            lib.step_tensor(p, m, v, g.copy(), bs, hp, t)
            geo = t if lam == 0.0 else (1 - a ** t) / (1 - a)
            _close(p, a ** t * p0 - hp.lr * u * geo, 1e-11, 1e-14, "closed-form param t=%d lam=%g" % (t, lam))
            _close(m, (1 - hp.beta1 ** t) * g, 1e-12, 0, "closed-form m t=%d" % t)
            _close(v, (1 - hp.beta2 ** t) * msq, 1e-12, 0, "closed-form v t=%d" % t)


# ---------------------------------------------------------------------------
# P3: v_b(t) is the EMA of the block mean of g^2, equivalently the block mean of
# Adam's elementwise v (the 5-parameter example of Section 2.3, partition
# (1,2,3),(4,5): u_mini = lr / sqrt(mean of Adam's v over the block)).
# ---------------------------------------------------------------------------
def pin_ema_and_five_param_example(lib):
    rng = np.random.default_rng(3)
    hp = orc.Hyper(lr=1e-3, beta1=0.9, beta2=0.95, eps=0.0, weight_decay=0.0)
    T = 6
    G = rng.normal(0, 1.0, (T, 5))
    # Adam's elementwise v and m on the same gradients: oracle with block size 1
    pa, ma, va = np.zeros(5), np.zeros(5), np.zeros(5)
    # Adam-mini on partition (1,2,3): one tensor of 3 / block 3; (4,5): one of 2 / block 2
    p3, m3, v3 = np.zeros(3), np.zeros(3), np.zeros(1)
    p2, m2, v2 = np.zeros(2), np.zeros(2), np.zeros(1)
    ema3 = ema2 = 0.0
    for t in range(1, T + 1):
        g = G[t - 1]
        lib.step_tensor(pa, ma, va, g.copy(), 1, hp, t)
        before3, before2 = p3.copy(), p2.copy()
        lib.step_tensor(p3, m3, v3, g[:3].copy(), 3, hp, t)
        lib.step_tensor(p2, m2, v2, g[3:].copy(), 2, hp, t)
        ema3 = (1 - hp.beta2) * np.mean(g[:3] ** 2) + hp.beta2 * ema3
        ema2 = (1 - hp.beta2) * np.mean(g[3:] ** 2) + hp.beta2 * ema2
        _close(v3, [ema3], 1e-13, 0, "EMA of block mean (block of 3) t=%d" % t)
        _close(v2, [ema2], 1e-13, 0, "EMA of block mean (block of 2) t=%d" % t)
        _close(v3, [va[:3].mean()], 1e-13, 0, "v_b = mean of Adam's v, block (1,2,3) t=%d" % t)
        _close(v2, [va[3:].mean()], 1e-13, 0, "v_b = mean of Adam's v, block (4,5) t=%d" % t)
        # w <- w - u * m_hat with u = lr / sqrt(mean of Adam's v_hat)  (eps = 0, lambda = 0)
        bc1, bc2 = 1 - hp.beta1 ** t, 1 - hp.beta2 ** t
        u3 = hp.lr / math.sqrt(va[:3].mean() / bc2)
        u2 = hp.lr / math.sqrt(va[3:].mean() / bc2)
        _close(p3, before3 - u3 * ma[:3] / bc1, 1e-12, 1e-18, "u_mini update (1,2,3) t=%d" % t)
        _close(p2, before2 - u2 * ma[3:] / bc1, 1e-12, 1e-18, "u_mini update (4,5) t=%d" % t)
        _close(m3, ma[:3], 1e-14, 0, "m is Adam's m")
    # explicit EMA sum  v(t) = (1-b2) sum_k b2^(t-k) mean(g_k^2)
    s = sum((1 - hp.beta2) * hp.beta2 ** (T - k) * np.mean(G[k - 1, :3] ** 2) for k in range(1, T + 1))
    _close(v3, [s], 1e-13, 0, "explicit EMA sum")


# ---------------------------------------------------------------------------
# P4: brute force.  The listing "Partition for Transformers" (Appendix B)
# transcribed as a dictionary name+i -> slice param[i], and Algorithm 2 run on
# each dictionary entry with Python floats.  The oracle is driven through the
# (numel, block_numel) description of the same partition.
# ---------------------------------------------------------------------------
def _partition_by_name(named, n_heads):
    """named: list of (name, 2-D or 1-D float array).  Returns dict key -> (name, slice)."""
    blocks = {}
    for name, arr in named:
        if "embed" in name or "output" in name:
            for i in range(arr.shape[0]):                      # by tokens
                blocks[name + str(i)] = (name, np.s_[i])
        elif "query" in name or "key" in name:
            hd = arr.shape[0] // n_heads                       # by heads
            for i in range(n_heads):
                blocks[name + str(i)] = (name, np.s_[i * hd:(i + 1) * hd])
        elif "value" in name or "attn.proj" in name or "mlp" in name:
            for i in range(arr.shape[0]):                      # by output neurons
                blocks[name + str(i)] = (name, np.s_[i])
        else:
            blocks[name] = (name, np.s_[...])
    return blocks


def _descriptor_block_numel(name, shape, n_heads):
    numel = int(np.prod(shape))
    if "embed" in name or "output" in name:
        return numel // shape[0]
    if "query" in name or "key" in name:
        return numel // n_heads
    if "value" in name or "attn.proj" in name or "mlp" in name:
        return numel // shape[0]
    return numel


def pin_bruteforce_partition(lib):
    rng = np.random.default_rng(17)
    n_heads = 2
    shapes = [("embed.weight", (5, 4)), ("layer0.query.weight", (4, 4)), ("layer0.key.weight", (4, 4)),
              ("layer0.value.weight", (4, 4)), ("layer0.attn.proj.weight", (4, 4)),
              ("layer0.mlp.up.weight", (6, 4)), ("layer0.mlp.down.weight", (4, 6)),
              ("layer0.norm.weight", (4,)), ("output.weight", (5, 4))]
    hp = orc.Hyper(lr=2e-2, beta1=0.8, beta2=0.9, eps=1e-6, weight_decay=0.05)
    P = {n: rng.normal(0, 1, s) for n, s in shapes}
    M = {n: np.zeros(s) for n, s in shapes}
    V = {}                                                 # per dictionary key
    blocks = _partition_by_name([(n, P[n]) for n, _ in shapes], n_heads)
    numel = [int(np.prod(s)) for _, s in shapes]
    bnum = [_descriptor_block_numel(n, s, n_heads) for n, s in shapes]
    st = orc.OracleState(numel, bnum, None, [P[n] for n, _ in shapes], lib=lib)
    T = 3
    for t in range(1, T + 1):
        G = {n: rng.normal(0, 0.3, s) for n, s in shapes}
        # --- brute force, Python floats, one dictionary entry at a time
        for key, (name, sl) in blocks.items():
            g = np.atleast_1d(G[name][sl]).ravel().tolist()
            pv = np.atleast_1d(P[name][sl]).ravel().tolist()
            mv = np.atleast_1d(M[name][sl]).ravel().tolist()
            v = V.get(key, 0.0)
            pv = [x - hp.lr * hp.weight_decay * x for x in pv]
            mv = [(1 - hp.beta1) * gi + hp.beta1 * mi for gi, mi in zip(g, mv)]
            mhat = [mi / (1 - hp.beta1 ** t) for mi in mv]
            v = (1 - hp.beta2) * (sum(gi * gi for gi in g) / len(g)) + hp.beta2 * v
            vhat = v / (1 - hp.beta2 ** t)
            pv = [x - hp.lr * mh / (math.sqrt(vhat) + hp.eps) for x, mh in zip(pv, mhat)]
            V[key] = v
            shape = np.shape(P[name][sl])
            P[name][sl] = np.array(pv).reshape(shape)
            M[name][sl] = np.array(mv).reshape(shape)
        # --- oracle through descriptors
        st.step([G[n].ravel() for n, _ in shapes], hp)
        for k, (n, s) in enumerate(shapes):
            _close(st.p[k], P[n].ravel(), 1e-12, 1e-15, "brute-force param %s t=%d" % (n, t))
            _close(st.m[k], M[n].ravel(), 1e-12, 1e-15, "brute-force m %s t=%d" % (n, t))
    # v scalars in dictionary insertion order == tensor order, block order
    want_v = [V[key] for key in blocks]
    _close(st.v_flat(), want_v, 1e-12, 0, "brute-force v order")
    # the block-index function agrees with the dictionary: the j-th inserted key of a tensor
    keys = list(blocks)
    for k, (n, s) in enumerate(shapes):
        flat_ids = np.empty(numel[k], dtype=np.int64)
        marker = np.full(s, -1, dtype=np.int64)
        for idx, key in enumerate(keys):
            name, sl = blocks[key]
            if name == n:
                marker[sl] = idx
        flat_ids[:] = marker.ravel()
        for e in range(numel[k]):
            got = lib.block_id(numel, bnum, k, e)
            if got != flat_ids[e]:
                raise AssertionError("block_id(%s,%d)=%d want %d" % (n, e, got, flat_ids[e]))


# ---------------------------------------------------------------------------
# P5: symmetries that follow from Algorithm 1.
# ---------------------------------------------------------------------------
def pin_symmetries(lib):
    rng = np.random.default_rng(23)
    nb, bs = 3, 8
    n = nb * bs
    p0 = rng.normal(0, 1, n)
    Gs = [rng.normal(0, 0.1, n) for _ in range(4)]

    def run(p0, Gs, hp, bs):
        p, m, v = p0.copy(), np.zeros(p0.size), np.zeros(p0.size // bs)
        for t, g in enumerate(Gs, 1):
            lib.step_tensor(p, m, v, g.copy(), bs, hp, t)
        return p, m, v

    hp = orc.Hyper(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    p, m, v = run(p0, Gs, hp, bs)
    # (a) permutation inside each block permutes p and m and leaves v (up to summation order)
    perm = np.concatenate([b * bs + rng.permutation(bs) for b in range(nb)])
    pp, mp, vp = run(p0[perm], [g[perm] for g in Gs], hp, bs)
    _close(pp, p[perm], 1e-12, 1e-15, "permutation param")
    _close(mp, m[perm], 1e-13, 0, "permutation m")
    _close(vp, v, 1e-13, 0, "permutation v")
    # (b) blocks never interact: changing g in block 1 leaves blocks 0 and 2 bit-identical
    Gs2 = [g.copy() for g in Gs]
    for g in Gs2:
        g[bs:2 * bs] *= 3.0
    p2, m2, v2 = run(p0, Gs2, hp, bs)
    for sl in (np.s_[0:bs], np.s_[2 * bs:3 * bs]):
        if not (np.array_equal(p2[sl], p[sl]) and np.array_equal(m2[sl], m[sl])):
            raise AssertionError("blocks interact")
    if not (v2[0] == v[0] and v2[2] == v[2]) or v2[1] == v[1]:
        raise AssertionError("v of an untouched block changed, or touched block did not")
    # (c) eps = 0: scaling g by alpha scales m by alpha, v by alpha^2, leaves param
    hp0 = orc.Hyper(lr=1e-2, beta1=0.9, beta2=0.95, eps=0.0, weight_decay=0.1)
    pa, ma, va = run(p0, Gs, hp0, bs)
    pb, mb, vb = run(p0, [7.0 * g for g in Gs], hp0, bs)
    _close(pb, pa, 1e-12, 1e-15, "scale invariance param")
    _close(mb, 7.0 * ma, 1e-13, 0, "scale m")
    _close(vb, 49.0 * va, 1e-13, 0, "scale v")
    # (d) an all-zero block at t = 1: m = v = 0 and the update is 0/(0+eps) = 0; only decay acts
    g0 = Gs[0].copy()
    g0[:bs] = 0.0
    pz, mz, vz = run(p0, [g0], hp, bs)
    _close(pz[:bs], p0[:bs] * (1 - hp.lr * hp.weight_decay), 1e-15, 0, "zero block decay only")
    if vz[0] != 0.0 or np.any(mz[:bs] != 0.0):
        raise AssertionError("zero block must keep m = v = 0")
    # (e) a NaN gradient poisons its own block only
    gn = Gs[0].copy()
    gn[bs + 2] = np.nan
    pn, mn, vn = run(p0, [gn], hp, bs)
    if not (np.all(np.isnan(pn[bs:2 * bs])) and np.isnan(vn[1])):
        raise AssertionError("NaN must poison the whole block")
    if np.any(np.isnan(pn[:bs])) or np.any(np.isnan(pn[2 * bs:])) or np.isnan(vn[0]) or np.isnan(vn[2]):
        raise AssertionError("NaN leaked into another block")
    # (f) weight decay acts on the parameter, not on the gradient: with g = 0 forever
    #     param_t = (1 - lr*lambda)^t param_0 exactly as a product
    pz2, _, _ = run(p0, [np.zeros(n)] * 3, hp, bs)
    _close(pz2, p0 * (1 - hp.lr * hp.weight_decay) ** 3, 1e-14, 0, "pure decay")
    # (g) wd_scale multiplies lambda
    p_h, m_h, v_h = p0.copy(), np.zeros(n), np.zeros(nb)
    lib.step_tensor(p_h, m_h, v_h, Gs[0].copy(), bs, hp, 1, wd_scale=0.0)
    hp_nowd = orc.Hyper(hp.lr, hp.beta1, hp.beta2, hp.eps, 0.0)
    p_i, m_i, v_i = p0.copy(), np.zeros(n), np.zeros(nb)
    lib.step_tensor(p_i, m_i, v_i, Gs[0].copy(), bs, hp_nowd, 1)
    if not np.array_equal(p_h, p_i):
        raise AssertionError("wd_scale = 0 must equal weight_decay = 0")


# ---------------------------------------------------------------------------
# P6: bias correction, separately from P2: after ONE step from zero state with
# eps = 0 and lambda = 0 the update is exactly lr * g / rms_block(g) whatever
# the betas are (m_hat = g and v_hat = mean g^2 at t = 1).
# ---------------------------------------------------------------------------
def pin_first_step(lib):
    rng = np.random.default_rng(29)
    for b1, b2 in ((0.9, 0.95), (0.5, 0.999), (0.0, 0.0)):
        hp = orc.Hyper(lr=0.1, beta1=b1, beta2=b2, eps=0.0, weight_decay=0.0)
        g = rng.normal(0, 1, 12)
        p, m, v = np.zeros(12), np.zeros(12), np.zeros(3)
        lib.step_tensor(p, m, v, g.copy(), 4, hp, 1)
        rms = np.repeat(np.sqrt((g.reshape(3, 4) ** 2).mean(axis=1)), 4)
        _close(p, -0.1 * g / rms, 1e-13, 0, "first step (b1=%g,b2=%g)" % (b1, b2))


# ---------------------------------------------------------------------------
# P7: gradient element types widen exactly: fp32 and bf16 bit patterns give the
# same result as the same values passed as float64.
# ---------------------------------------------------------------------------
def pin_grad_dtypes(lib):
    rng = np.random.default_rng(31)
    hp = orc.Hyper(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    g32 = rng.normal(0, 1e-3, 16).astype(np.float32)
    bits = (g32.view(np.uint32) >> 16).astype(np.uint16)          # truncate to bf16 bits
    gbf = (bits.astype(np.uint32) << 16).view(np.float32)
    for garr, g64 in ((g32, g32.astype(np.float64)), (bits, gbf.astype(np.float64))):
        pa, ma, va = np.ones(16), np.zeros(16), np.zeros(2)
        pb, mb, vb = np.ones(16), np.zeros(16), np.zeros(2)
        lib.step_tensor(pa, ma, va, garr, 8, hp, 1)
        lib.step_tensor(pb, mb, vb, g64, 8, hp, 1)
        if not (np.array_equal(pa, pb) and np.array_equal(ma, mb) and np.array_equal(va, vb)):
            raise AssertionError("gradient widening is not exact for %s" % garr.dtype)


# ---------------------------------------------------------------------------
# P8: layout invariants of the block-index function.
# ---------------------------------------------------------------------------
def pin_layout_invariants(lib):
    numel = [12, 7, 30, 4]
    bnum = [4, 7, 1, 2]
    total = lib.num_blocks(numel, bnum)
    if total != 3 + 1 + 30 + 2:
        raise AssertionError("num_blocks")
    seen = {}
    last = -1
    for k in range(len(numel)):
        for e in range(numel[k]):
            b = lib.block_id(numel, bnum, k, e)
            if b < last:
                raise AssertionError("block ids must be non-decreasing")
            last = b
            seen[b] = seen.get(b, 0) + 1
            owner = seen.setdefault(("t", b), k)
            if owner != k:
                raise AssertionError("a block spans two tensors")
    if sorted(x for x in seen if not isinstance(x, tuple)) != list(range(total)):
        raise AssertionError("block ids must be 0..num_blocks-1 without gaps")
    for k in range(len(numel)):
        first = lib.block_id(numel, bnum, k, 0)
        for j in range(numel[k] // bnum[k]):
            if seen[first + j] != bnum[k]:
                raise AssertionError("block %d has %d elements, want %d" % (first + j, seen[first + j], bnum[k]))


# ---------------------------------------------------------------------------
# P9: strided (column) blocks.  A weight stored as its transpose has the same blocks, now as
# the columns of the stored matrix (Appendix D: "some extra re-ordering is needed").  The
# strided form must give, bit for bit, the transpose of what the contiguous form gives on
# the re-ordered data, and must agree with a brute-force loop over param[:, j].
# ---------------------------------------------------------------------------
def pin_strided_blocks(lib):
    rng = np.random.default_rng(41)
    B, n = 7, 5                                   # 7 blocks of 5 elements
    hp = orc.Hyper(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    W0 = rng.normal(0, 1, (B, n))                 # logical layout: block = row
    pc, mc, vc = W0.ravel().copy(), np.zeros(B * n), np.zeros(B)
    ps, ms, vs = W0.T.ravel().copy(), np.zeros(B * n), np.zeros(B)     # stored transposed: [n, B]
    P = W0.T.copy()
    M = np.zeros((n, B))
    V = [0.0] * B
    for t in range(1, 4):
        G = rng.normal(0, 0.1, (B, n))
        lib.step_tensor(pc, mc, vc, G.ravel().copy(), n, hp, t)
        lib.step_tensor(ps, ms, vs, G.T.ravel().copy(), n, hp, t, strided=True)
        if not (np.array_equal(ps.reshape(n, B).T.ravel(), pc) and np.array_equal(ms.reshape(n, B).T.ravel(), mc)
                and np.array_equal(vs, vc)):
            raise AssertionError("strided result is not the transpose of the contiguous result (t=%d)" % t)
        GT = G.T
        for j in range(B):                        # brute force over param[:, j], Python floats
            g = GT[:, j].tolist()
            pv = [x - hp.lr * hp.weight_decay * x for x in P[:, j].tolist()]
            mv = [(1 - hp.beta1) * gi + hp.beta1 * mi for gi, mi in zip(g, M[:, j].tolist())]
            V[j] = (1 - hp.beta2) * (sum(gi * gi for gi in g) / n) + hp.beta2 * V[j]
            vhat = V[j] / (1 - hp.beta2 ** t)
            pv = [x - hp.lr * (mi / (1 - hp.beta1 ** t)) / (math.sqrt(vhat) + hp.eps) for x, mi in zip(pv, mv)]
            P[:, j] = pv
            M[:, j] = mv
        _close(ps, P.ravel(), 1e-12, 1e-15, "strided brute-force param t=%d" % t)
        _close(ms, M.ravel(), 1e-12, 1e-15, "strided brute-force m t=%d" % t)
        _close(vs, V, 1e-12, 0, "strided brute-force v t=%d" % t)
    # block ids: element (r, j) of the stored [n, B] matrix belongs to block j
    numel, bnum, strided = [6, B * n, 4], [3, n, 1], [False, True, False]
    want = 2 + np.tile(np.arange(B), n)
    for e in range(B * n):
        if lib.block_id(numel, bnum, 1, e, strided) != int(want[e]):
            raise AssertionError("strided block_id(%d)" % e)
    if lib.block_id(numel, bnum, 2, 0, strided) != 2 + B:
        raise AssertionError("blocks after a strided tensor")
    if not np.array_equal(lib.block_ids_tensor(numel, bnum, 1, strided), want.astype(np.uint64)):
        raise AssertionError("strided block_ids_tensor")


# ---------------------------------------------------------------------------
# P10: the ablation's other block statistics ("Ablation Studies on the Design of Adam-mini":
# 2-norm, 1-norm, max, min in place of the mean).  Reading: Algorithm 1 with r(g .* g) in its v
# line.  Pinned by numpy's norm / max / min routines on the vector g*g, the EMA written as an
# explicit sum, the constant-gradient closed form with rms replaced by sqrt(r), the chain
# min <= mean <= max <= 2-norm <= 1-norm, hand values, the one-element block (every statistic is
# the element itself, i.e. AdamW), the scaling law, NaN hand-over and the strided form.
# ---------------------------------------------------------------------------
def _statistic(name, s):
    if name == "mean":
        return float(np.mean(s))
    if name == "norm1":
        return float(np.linalg.norm(s, 1))
    if name == "norm2":
        return float(np.linalg.norm(s, 2))
    return float(np.max(s)) if name == "max" else float(np.min(s))


def pin_alternative_reducers(lib):
    rng = np.random.default_rng(77)
    names = ["mean", "norm1", "norm2", "max", "min"]
    nb, bs, T = 5, 7, 4
    hp = orc.Hyper(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1)
    grads = [rng.normal(0, 1e-2, nb * bs) * np.repeat(rng.uniform(0.1, 10, nb), bs) for _ in range(T)]
    p0 = rng.normal(0, 1.0, nb * bs)
    vs = {}
    for name in names:
        p, m, v = p0.copy(), np.zeros(nb * bs), np.zeros(nb)
        P, M = p0.copy(), np.zeros(nb * bs)
        for t in range(1, T + 1):
            lib.step_tensor(p, m, v, grads[t - 1].copy(), bs, hp, t, reducer=name)
            # v_b(t) = (1 - b2) sum_k b2^(t-k) r(g_k * g_k), statistics from numpy
            want_v = np.array([sum((1 - hp.beta2) * hp.beta2 ** (t - k) * _statistic(name, grads[k - 1][b * bs:(b + 1) * bs] ** 2)
                                   for k in range(1, t + 1)) for b in range(nb)])
            _close(v, want_v, 1e-12, 0, "%s: EMA of the numpy statistic, t=%d" % (name, t))
            # the rest of Algorithm 1 around that v, vectorised
            P = P - hp.lr * hp.weight_decay * P
            M = (1 - hp.beta1) * grads[t - 1] + hp.beta1 * M
            P = P - hp.lr * (M / (1 - hp.beta1 ** t)) / np.repeat(np.sqrt(want_v / (1 - hp.beta2 ** t)) + hp.eps, bs)
            _close(p, P, 1e-11, 1e-14, "%s: param t=%d" % (name, t))
            _close(m, M, 1e-12, 0, "%s: m t=%d" % (name, t))
        vs[name] = v.copy()
    if not (np.all(vs["min"] <= vs["mean"]) and np.all(vs["mean"] <= vs["max"]) and np.all(vs["max"] <= vs["norm2"])
            and np.all(vs["norm2"] <= vs["norm1"]) and np.all(vs["min"] < vs["norm1"])):
        raise AssertionError("min <= mean <= max <= 2-norm <= 1-norm violated")
    # hand values: g = (1, -2, 2, 0), g*g = (1, 4, 4, 0); beta2 = 1/2, one step: v = r / 2
    hp2 = orc.Hyper(lr=0.5, beta1=0.5, beta2=0.5, eps=0.0, weight_decay=0.0)
    hand = {"mean": 9 / 8, "norm1": 9 / 2, "norm2": math.sqrt(33) / 2, "max": 2.0, "min": 0.0}
    for name in names:
        p, m, v = np.ones(4), np.zeros(4), np.zeros(1)
        lib.step_tensor(p, m, v, np.array([1.0, -2.0, 2.0, 0.0]), 4, hp2, 1, reducer=name)
        _close(v, [hand[name]], 1e-15, 0, "%s: hand value" % name)
        if name != "min":     # v_hat = r, m_hat = g: param = 1 - g / (2 sqrt(r))
            _close(p, 1 - np.array([1.0, -2.0, 2.0, 0.0]) / (2 * math.sqrt(2 * hand[name])), 1e-15, 0, "%s: hand param" % name)
    # |g| = c over the block: mean = max = min = c^2, 1-norm = n c^2, 2-norm = sqrt(n) c^2
    c, n = 0.25, 9
    g = c * np.where(rng.random(n) < 0.5, -1.0, 1.0)
    for name, want in (("mean", c * c), ("max", c * c), ("min", c * c), ("norm1", n * c * c), ("norm2", 3 * c * c)):
        p, m, v = np.zeros(n), np.zeros(n), np.zeros(1)
        lib.step_tensor(p, m, v, g.copy(), n, hp, 1, reducer=name)
        _close(v, [(1 - hp.beta2) * want], 1e-15, 0, "%s: equal magnitudes" % name)
    # constant gradient: v_hat = r(g*g) at every step, so param follows the closed form with sqrt(r) for the rms
    g = rng.normal(0, 1e-2, nb * bs)
    for name in names:
        p, m, v = p0.copy(), np.zeros(nb * bs), np.zeros(nb)
        r = np.array([_statistic(name, g[b * bs:(b + 1) * bs] ** 2) for b in range(nb)])
        u = g / np.repeat(np.sqrt(r) + hp.eps, bs)
        a = 1.0 - hp.lr * hp.weight_decay
        for t in range(1, 9):
            lib.step_tensor(p, m, v, g.copy(), bs, hp, t, reducer=name)
        _close(p, a ** 8 * p0 - hp.lr * u * (1 - a ** 8) / (1 - a), 1e-11, 1e-14, "%s: closed-form param" % name)
        _close(v, (1 - hp.beta2 ** 8) * r, 1e-12, 0, "%s: closed-form v" % name)
    # one-element blocks: every statistic of a 1-vector is the element, so all five are AdamW
    ref = None
    for name in names:
        p, m, v = p0.copy(), np.zeros(nb * bs), np.zeros(nb * bs)
        for t in range(1, 4):
            lib.step_tensor(p, m, v, grads[t - 1].copy(), 1, hp, t, reducer=name)
        if ref is None:
            ref = (p.copy(), v.copy())
        _close(p, ref[0], 1e-14, 0, "%s: one-element blocks param" % name)
        _close(v, ref[1], 1e-14, 0, "%s: one-element blocks v" % name)
    # scaling g by alpha scales every statistic by alpha^2
    for name in names:
        v1, v2 = np.zeros(nb), np.zeros(nb)
        lib.step_tensor(p0.copy(), np.zeros(nb * bs), v1, grads[0].copy(), bs, hp, 1, reducer=name)
        lib.step_tensor(p0.copy(), np.zeros(nb * bs), v2, 4.0 * grads[0], bs, hp, 1, reducer=name)
        _close(v2, 16.0 * v1, 1e-14, 0, "%s: scaling" % name)
    # a NaN gradient poisons its own block under every statistic, and only that block
    gn = grads[0].copy()
    gn[2 * bs + 3] = np.nan
    for name in names:
        p, m, v = p0.copy(), np.zeros(nb * bs), np.zeros(nb)
        lib.step_tensor(p, m, v, gn.copy(), bs, hp, 1, reducer=name)
        if not (np.isnan(v[2]) and np.isfinite(np.delete(v, 2)).all() and np.isnan(p[2 * bs:3 * bs]).all()
                and np.isfinite(np.delete(p, np.arange(2 * bs, 3 * bs))).all()):
            raise AssertionError("%s: NaN hand-over" % name)
    # strided form: bit for bit the transpose of the contiguous form
    B, n = 6, 5
    W0, G = rng.normal(0, 1, (B, n)), rng.normal(0, 0.1, (B, n))
    for name in names:
        pc, mc, vc = W0.ravel().copy(), np.zeros(B * n), np.zeros(B)
        ps, ms, vs_ = W0.T.ravel().copy(), np.zeros(B * n), np.zeros(B)
        lib.step_tensor(pc, mc, vc, G.ravel().copy(), n, hp, 1, reducer=name)
        lib.step_tensor(ps, ms, vs_, G.T.ravel().copy(), n, hp, 1, reducer=name, strided=True)
        if not (np.array_equal(ps.reshape(n, B).T.ravel(), pc) and np.array_equal(vs_, vc)):
            raise AssertionError("%s: strided form differs from the transposed contiguous form" % name)


ALL_PINS = [pin_hand_worked, pin_adamw_reduction, pin_constant_gradient,
            pin_ema_and_five_param_example, pin_bruteforce_partition, pin_symmetries,
            pin_first_step, pin_grad_dtypes, pin_layout_invariants, pin_strided_blocks,
            pin_alternative_reducers]
