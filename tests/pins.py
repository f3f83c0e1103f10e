"""Checks that pin the CPU oracle to facts that do not come from the oracle itself.

The paper prints no numeric example of an optimizer step (its only worked
example, Fig. 3, is about tagging AllGather chunks), so absolute values are
pinned by closed forms, by exact rational arithmetic on tiny inputs, by the
IEEE definition of the formats, and by library routines for the special cases
that reduce to them (torch.optim.AdamW, torch.nn.utils.clip_grad_norm_,
torch's bfloat16 conversion).

Each function raises AssertionError on a violation.  test_oracle_pins.py runs
them against the oracle; test_oracle_mutants.py runs them against copies of the
oracle with one planted mistake each and expects a failure.
"""
from __future__ import annotations

import math
from fractions import Fraction

import numpy as np
import torch

import oracle
from oracle import HParams

F32 = np.float32


def _rng(seed):
    return np.random.default_rng(seed)


def _bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 patterns through torch's conversion (a library routine)."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16).copy()


# --------------------------------------------------------------------------- widen
def pin_widen_bf16_exhaustive():
    h = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.widen_bf16(h)
    # (a) library routine
    lib = torch.from_numpy(h.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(got.view(np.uint32), lib.view(np.uint32))
    # (b) the format's definition: sign, 8-bit exponent, 7-bit fraction
    for bits in list(range(0, 65536, 97)) + [0x0001, 0x007F, 0x0080, 0x7F7F, 0x8000, 0x8001, 0xFF7F, 0x3F80]:
        s, e, f = bits >> 15, (bits >> 7) & 0xFF, bits & 0x7F
        if e == 0xFF:
            continue
        val = math.ldexp(f / 128.0, -126) if e == 0 else math.ldexp(1.0 + f / 128.0, e - 127)
        val = -val if s else val
        assert float(got[bits]) == val and math.copysign(1.0, float(got[bits])) == (-1.0 if s else 1.0), bits
    assert np.isinf(got[0x7F80]) and np.isinf(got[0xFF80]) and np.isnan(got[0x7FC0])


# --------------------------------------------------------------------------- fold
def pin_fold_identity_and_equal_workers():
    g = (_rng(1).standard_normal(1000) * 1e-3).astype(F32)
    r = oracle.fold([g], mean=True)
    assert np.array_equal(r.view(np.uint32), g.view(np.uint32))          # W=1 is the identity
    r = oracle.fold([g], mean=False)
    assert np.array_equal(r.view(np.uint32), g.view(np.uint32))
    hb = _bf16_bits(g)
    assert np.array_equal(oracle.fold([hb]), oracle.widen_bf16(hb))
    # all workers equal, W = 2^k: with 8-bit significands every partial sum k*g is exact in float
    g = oracle.widen_bf16(hb)
    for W in (2, 4, 8, 16, 32):
        assert np.array_equal(oracle.fold([g] * W), g), W
        assert np.array_equal(oracle.fold([hb] * W), oracle.widen_bf16(hb)), W
        assert np.array_equal(oracle.fold([g] * W, mean=False), g * F32(W)), W


def pin_fold_order_and_precision():
    # left-to-right in float: (2^24 + 1) + 1 = 2^24 (ties to even twice); any other order gives 2^24 + 2
    a, one = np.array([2.0 ** 24], F32), np.array([1.0], F32)
    assert oracle.fold([a, one, one], mean=False)[0] == 2.0 ** 24
    assert oracle.fold([one, one, a], mean=False)[0] == 2.0 ** 24 + 2
    # bfloat16 inputs are added in float, never in bfloat16: 256 + 1 = 257 (not representable in bf16)
    h256, h1 = _bf16_bits(np.array([256.0], F32)), _bf16_bits(np.array([1.0], F32))
    assert oracle.fold([h256, h1], mean=False)[0] == 257.0
    assert oracle.fold([h256, h1], mean=True)[0] == 128.5
    # mean with W not a power of two is one multiply by float(1/W)
    x = np.array([1.0, 5.0, 7.0], F32)
    r = oracle.fold([x, x, x], mean=True)
    expect = (x + x + x) * F32(1.0 / 3.0)
    assert np.array_equal(r, expect)
    # worker 0 is included (a fold that starts at worker 1 loses it)
    assert oracle.fold([np.array([5.0], F32), np.array([1.0], F32)], mean=False)[0] == 6.0


def pin_fold_bruteforce_rational():
    rng = _rng(2)
    for W in (1, 3, 4, 7, 8):
        n = 257
        gs = [(rng.standard_normal(n) * 1e-3).astype(F32) for _ in range(W)]
        hs = [_bf16_bits(g) for g in gs]
        for views, vals in ((gs, gs), (hs, [oracle.widen_bf16(h) for h in hs])):
            r32 = oracle.fold(views, mean=True)
            r64 = oracle.fold(views, mean=True, precision="f64")
            s32 = oracle.fold(views, mean=False)
            for i in range(n):
                exact = sum(Fraction(float(v[i])) for v in vals)
                mag = sum(abs(Fraction(float(v[i]))) for v in vals)
                assert abs(Fraction(float(s32[i])) - exact) <= mag * W * Fraction(1, 2 ** 24)
                assert abs(Fraction(float(r32[i])) - exact / W) <= (mag / W) * (W + 1) * Fraction(1, 2 ** 24)
                assert abs(Fraction(float(r64[i])) - exact / W) <= (mag / W) * Fraction(1, 2 ** 50) + Fraction(1, 2 ** 1070)


# --------------------------------------------------------------------------- AdamW closed forms
def _hp(**kw):
    d = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, max_grad_norm=0.0)
    d.update(kw)
    return HParams(**d)


def pin_adamw_first_step_closed_form():
    """m=v=0, t=1, no decay: the bias-corrected moments are g and g^2, so dp = -lr*g/(|g|+eps)."""
    hp = _hp()
    lr, eps = hp.f32("lr"), hp.f32("eps")
    g = np.concatenate([(_rng(3).standard_normal(500) * s) for s in (1e-6, 1e-3, 1.0, 30.0)] + [np.array([0.0, 1e-8, -1e-8, 3e-9])])
    g32 = g.astype(F32)
    p0 = (_rng(4).standard_normal(g.size) * 0.02).astype(F32)
    # double variant
    p, m, v = p0.astype(np.float64), np.zeros(g.size), np.zeros(g.size)
    oracle.adamw_f64(p, m, v, g32.astype(np.float64), False, hp, 1)
    gd = g32.astype(np.float64)
    want = -lr * gd / (np.abs(gd) + eps)
    dp = p - p0.astype(np.float64)
    assert np.allclose(dp, want, rtol=1e-11, atol=1e-18)
    assert np.allclose(m, (1 - hp.f32("beta1")) * gd, rtol=1e-14, atol=0)
    assert np.allclose(v, (1 - hp.f32("beta2")) * gd * gd, rtol=1e-14, atol=0)
    # float variant (starting from p=0 so that dp is not rounded against p)
    p, m, v = np.zeros(g.size, F32), np.zeros(g.size, F32), np.zeros(g.size, F32)
    oracle.adamw_f32(p, m, v, g32, False, hp, 1)
    assert np.allclose(p.astype(np.float64), want, rtol=2e-6, atol=1e-30)
    nz = gd != 0
    assert np.all(np.sign(p[nz]) == -np.sign(g32[nz])) and np.all(np.abs(p) < lr * (1 + 1e-6))
    assert np.all(p[~nz] == 0)


def pin_zero_grad_geometric_decay():
    hp = _hp()
    rng = _rng(5)
    n, T = 300, 25
    m0 = (rng.standard_normal(n) * 1e-3).astype(F32)
    v0 = (rng.random(n) * 1e-6).astype(F32)
    z = np.zeros(n, F32)
    p, m, v = np.zeros(n, F32), m0.copy(), v0.copy()
    mm, vv = m0.copy(), v0.copy()
    pd, md, vd = np.zeros(n), m0.astype(np.float64), v0.astype(np.float64)
    for t in range(1, T + 1):
        oracle.adamw_f32(p, m, v, z, False, hp, t)
        oracle.adamw_f64(pd, md, vd, z.astype(np.float64), False, hp, t)
        mm = F32(0.9) * mm            # beta*x + (1-beta)*0 is one rounded multiply
        vv = F32(0.999) * vv
        assert np.array_equal(m, mm) and np.array_equal(v, vv), t
    b1, b2 = hp.f32("beta1"), hp.f32("beta2")
    assert np.allclose(md, m0.astype(np.float64) * b1 ** T, rtol=1e-13, atol=0)
    assert np.allclose(vd, v0.astype(np.float64) * b2 ** T, rtol=1e-13, atol=0)
    assert np.allclose(m, md, rtol=T * 1.2e-7, atol=0) and np.allclose(v, vd, rtol=T * 1.2e-7, atol=0)


def pin_constant_grad_closed_form():
    """Constant g: m_t = g(1-b1^t), v_t = g^2(1-b2^t), so every step moves p by -lr*g/(|g|+eps)."""
    hp = _hp()
    lr, eps, b1, b2 = (hp.f32(k) for k in ("lr", "eps", "beta1", "beta2"))
    g32 = np.array([1e-3, -2.5e-4, 0.7, -3.0, 1e-7], F32)
    gd = g32.astype(np.float64)
    T = 12
    pd, md, vd = np.zeros(5), np.zeros(5), np.zeros(5)
    p, m, v = np.zeros(5, F32), np.zeros(5, F32), np.zeros(5, F32)
    for t in range(1, T + 1):
        oracle.adamw_f64(pd, md, vd, gd, False, hp, t)
        oracle.adamw_f32(p, m, v, g32, False, hp, t)
        assert np.allclose(md, gd * (1 - b1 ** t), rtol=1e-12, atol=0)
        assert np.allclose(vd, gd * gd * (1 - b2 ** t), rtol=1e-12, atol=0)
        assert np.allclose(pd, -t * lr * gd / (np.abs(gd) + eps), rtol=1e-10, atol=0)
        assert np.allclose(m, md, rtol=1e-5, atol=0) and np.allclose(v, vd, rtol=1e-5, atol=0)
        assert np.allclose(p, pd, rtol=1e-5, atol=0)


def pin_weight_decay():
    hp = _hp(weight_decay=0.01)
    n, T = 200, 15
    p0 = (_rng(6).standard_normal(n) * 0.02).astype(F32)
    z = np.zeros(n, F32)
    p, m, v = p0.copy(), z.copy(), z.copy()
    q, mq, vq = p0.copy(), z.copy(), z.copy()
    pd, md, vd = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    decay = F32(1.0 - float(F32(1e-3)) * float(F32(0.01)))
    want = p0.copy()
    for t in range(1, T + 1):
        oracle.adamw_f32(p, m, v, z, True, hp, t)
        oracle.adamw_f32(q, mq, vq, z, False, hp, t)      # masked tensor
        oracle.adamw_f64(pd, md, vd, z.astype(np.float64), True, hp, t)
        want = want * decay
        assert np.array_equal(p, want), t
        assert np.array_equal(q.view(np.uint32), p0.view(np.uint32)), t
    assert np.allclose(pd, p0.astype(np.float64) * (1 - hp.f32("lr") * hp.f32("weight_decay")) ** T, rtol=1e-13)
    # decay is decoupled: it acts on p BEFORE the Adam step and does not enter m or v
    g = np.full(4, 1e-3, F32)
    p1, m1, v1 = np.ones(4, F32), np.zeros(4, F32), np.zeros(4, F32)
    oracle.adamw_f32(p1, m1, v1, g, True, hp, 1)
    assert np.allclose(m1, 1e-4, rtol=1e-6) and np.allclose(v1, 1e-9, rtol=1e-5)
    want1 = 1.0 * (1 - 1e-5) - 1e-3 * 1e-3 / (1e-3 + 1e-8)
    assert np.allclose(p1, want1, rtol=2e-7)


# --------------------------------------------------------------------------- clip
def pin_clip():
    # one-hot: the norm is |g|
    r = np.zeros(1000, F32)
    r[123] = -4.0
    c = oracle.clip_coef([r], 1.0)
    assert c == F32(1.0 / (4.0 + 1e-6))
    # 3-4-5 split over two buckets: the norm is global, not per bucket
    c = oracle.clip_coef([np.array([3.0], F32), np.array([0.0, 4.0], F32)], 1.0, precision="f64")
    assert abs(c - 1.0 / (5.0 + 1e-6)) < 1e-15
    # small norm: coefficient is exactly one, including the 1e-6 guard
    assert oracle.clip_coef([np.array([0.5], F32)], 1.0) == F32(1.0)
    assert oracle.clip_coef([np.array([1.0 - 1e-6 - 1e-7], F32)], 1.0, precision="f64") == 1.0
    c = oracle.clip_coef([np.array([1e-6], F32)], 1e-6, precision="f64")      # guard term matters here
    assert abs(c - float(F32(1e-6)) / (float(F32(1e-6)) + 1e-6)) < 1e-12
    # after clipping the norm is at most max_norm; scaling a clipped gradient by 2^k leaves c*r (nearly) unchanged
    g = (_rng(7).standard_normal(5000)).astype(F32)
    for mx in (0.5, 1.0):
        c = oracle.clip_coef([g], mx, precision="f64")
        assert np.linalg.norm(g.astype(np.float64) * c) <= mx
        c8 = oracle.clip_coef([g * F32(8)], mx, precision="f64")
        assert abs(c8 * 8 / c - 1) < 1e-6
    # library routine: torch's clip_grad_norm_ (same definition, evaluated in float)
    tp = torch.nn.Parameter(torch.zeros(5000))
    tp.grad = torch.from_numpy(g.copy())
    torch.nn.utils.clip_grad_norm_([tp], 1.0)
    assert np.allclose(tp.grad.numpy(), g * oracle.clip_coef([g], 1.0), rtol=1e-5, atol=0)
    # weighted accumulation (tiled inputs) equals the plain one
    tile = g[:10]
    cnt = np.array([3, 3, 3, 3, 2, 2, 2, 2, 2, 2], np.uint64)
    full = np.concatenate([tile, tile, tile[:4]])
    a = oracle.SumSq().add(full).value
    b = oracle.SumSq().add(tile, cnt).value
    assert abs(a - b) <= 1e-15 * a


def pin_clip_is_noop_below_threshold():
    hp0, hp1 = _hp(weight_decay=0.01), _hp(weight_decay=0.01, max_grad_norm=1.0)
    n = 64
    g = (_rng(8).standard_normal(n) * 1e-3).astype(F32)
    p0 = (_rng(9).standard_normal(n) * 0.02).astype(F32)
    c = oracle.clip_coef([g], 1.0)
    assert c == F32(1.0)
    a = [p0.copy(), np.zeros(n, F32), np.zeros(n, F32)]
    b = [p0.copy(), np.zeros(n, F32), np.zeros(n, F32)]
    oracle.adamw_f32(*a, g, True, hp0, 1)
    oracle.adamw_f32(*b, g, True, hp1, 1, c=c)
    for x, y in zip(a, b):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    # and a coefficient below one scales the gradient before both moments
    a = [np.zeros(n, F32), np.zeros(n, F32), np.zeros(n, F32)]
    b = [np.zeros(n, F32), np.zeros(n, F32), np.zeros(n, F32)]
    oracle.adamw_f32(*a, g * F32(0.25), False, hp0, 1)
    oracle.adamw_f32(*b, g, False, hp1, 1, c=F32(0.25))
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


# --------------------------------------------------------------------------- library special cases
def _torch_run(layout, hp, p0_by_tensor, grads_by_step_tensor, dtype):
    params = [torch.nn.Parameter(torch.tensor(x, dtype=dtype)) for x in p0_by_tensor]
    wd_on = [p for p, (n, wd) in zip(params, layout) if wd]
    wd_off = [p for p, (n, wd) in zip(params, layout) if not wd]
    groups = []
    if wd_on:
        groups.append({"params": wd_on, "weight_decay": hp.f32("weight_decay")})
    if wd_off:
        groups.append({"params": wd_off, "weight_decay": 0.0})
    opt = torch.optim.AdamW(groups, lr=hp.f32("lr"), betas=(hp.f32("beta1"), hp.f32("beta2")),
                            eps=hp.f32("eps"), foreach=False)
    for grads in grads_by_step_tensor:
        for p, g in zip(params, grads):
            p.grad = torch.tensor(g, dtype=dtype)
        if hp.max_grad_norm > 0:
            torch.nn.utils.clip_grad_norm_(params, float(F32(hp.max_grad_norm)))
        opt.step()
    st = [opt.state[p] for p in params]
    return ([p.detach().numpy() for p in params], [s["exp_avg"].numpy() for s in st],
            [s["exp_avg_sq"].numpy() for s in st])


def pin_whole_step_vs_torch(clip=True, W=3, steps=6, grad_kind="bf16"):
    """Whole driver (layout, fold, clip, masked AdamW over several buckets) against
    torch.optim.AdamW + clip_grad_norm_ in double on the exact mean gradient."""
    tensors = [(37, True), (5, False), (64, True), (200, True), (3, False), (129, True)]
    hp = _hp(weight_decay=0.01, max_grad_norm=(0.01 if clip else 0.0))
    lay = oracle.build_layout(tensors, 2 if grad_kind == "bf16" else 4, 300)
    assert len(lay.buckets) >= 3
    rng = _rng(10)
    p0_t = [(rng.standard_normal(n) * 0.02).astype(F32) for n, _ in tensors]
    # per-step, per-worker, per-tensor gradients
    graw = [[[(rng.standard_normal(n) * 1e-3).astype(F32) for n, _ in tensors] for _ in range(W)] for _ in range(steps)]
    if grad_kind == "bf16":
        gbits = [[[_bf16_bits(g) for g in wk] for wk in st] for st in graw]
        gval = [[[oracle.widen_bf16(h).astype(np.float64) for h in wk] for wk in st] for st in gbits]
        views_src = gbits
    else:
        gval = [[[g.astype(np.float64) for g in wk] for wk in st] for st in graw]
        views_src = graw

    def pack(per_tensor, dtype):
        out = []
        for b in lay.buckets:
            out.append(np.concatenate([np.asarray(per_tensor[s.tensor], dtype=dtype) for s in b.segments]))
        return out

    results = {}
    for prec in ("f64", "f32"):
        orc = oracle.OracleShadow(lay, hp, pack(p0_t, F32), precision=prec)
        for st in range(steps):
            grads = {}
            for bi, b in enumerate(lay.buckets):
                grads[bi] = [np.concatenate([views_src[st][w][s.tensor] for s in b.segments]) for w in range(W)]
            orc.step(grads)
        results[prec] = orc
    mean_grads = [[sum(gval[st][w][t] for w in range(W)) / W for t in range(len(tensors))] for st in range(steps)]
    tp, tm, tv = _torch_run(tensors, hp, p0_t, mean_grads, torch.float64)
    o64 = results["f64"]
    for bi, b in enumerate(lay.buckets):
        for s in b.segments:
            sl = slice(s.offset, s.offset + s.numel)
            assert np.allclose(o64.p[bi][sl], tp[s.tensor], rtol=1e-11, atol=1e-16), ("p", s.tensor)
            assert np.allclose(o64.m[bi][sl], tm[s.tensor], rtol=1e-11, atol=1e-18), ("m", s.tensor)
            assert np.allclose(o64.v[bi][sl], tv[s.tensor], rtol=1e-11, atol=1e-24), ("v", s.tensor)
    # the float variant stays within a forward rounding bound of the double one
    o32 = results["f32"]
    for bi in range(len(lay.buckets)):
        assert np.allclose(o32.p[bi], o64.p[bi], rtol=0, atol=steps * 4e-9 + 2e-9), "p32"
        scale_m = np.abs(o64.m[bi]).max()
        assert np.abs(o32.m[bi] - o64.m[bi]).max() <= 20 * steps * 2 ** -24 * scale_m
        assert np.allclose(o32.v[bi], o64.v[bi], rtol=20 * steps * 2 ** -24, atol=0)
    if clip:
        assert o64.last_coef < 1.0
        assert abs(float(o32.last_coef) / o64.last_coef - 1) < 1e-6


def pin_f32_vs_torch_f32():
    """Float variant against torch's float AdamW on one tensor (a few ulp: same formulas, other rounding order)."""
    hp = _hp(weight_decay=0.01)
    n, T = 4096, 10
    rng = _rng(11)
    p0 = (rng.standard_normal(n) * 0.02).astype(F32)
    gs = [(rng.standard_normal(n) * 1e-3).astype(F32) for _ in range(T)]
    p, m, v = p0.copy(), np.zeros(n, F32), np.zeros(n, F32)
    for t, g in enumerate(gs, 1):
        oracle.adamw_f32(p, m, v, g, True, hp, t)
    tp, tm, tv = _torch_run([(n, True)], hp, [p0], [[g] for g in gs], torch.float32)
    assert np.allclose(p, tp[0], rtol=0, atol=T * 1e-8)
    assert np.abs(m - tm[0]).max() <= 8 * T * 2 ** -24 * np.abs(tm[0]).max()
    assert np.allclose(v, tv[0], rtol=8 * T * 2 ** -24, atol=0)


# --------------------------------------------------------------------------- layout
def pin_layout():
    # hand-worked: sizes in elements of 1 byte, cap 50, walking from the last tensor:
    #   5 -> bucket 0; 100 (> cap) -> bucket 1 alone; 30 -> bucket 2; 20 -> bucket 2 (50 <= 50); 10 -> bucket 3
    lay = oracle.build_layout([(10, True), (20, False), (30, True), (100, True), (5, False)], 1, 50)
    assert lay.bucket_of_tensor == [3, 2, 2, 1, 0]
    assert [b.numel for b in lay.buckets] == [5, 100, 50, 10]
    assert [(s.tensor, s.offset) for s in lay.buckets[2].segments] == [(2, 0), (1, 30)]
    assert [s.weight_decay for s in lay.buckets[2].segments] == [True, False]
    # the cap is in gradient BYTES: with 2-byte gradients only 25 elements fit
    lay2 = oracle.build_layout([(10, True), (20, False), (30, True), (100, True), (5, False)], 2, 50)
    assert lay2.bucket_of_tensor == [4, 3, 2, 1, 0]
    # an oversize tensor closes the open bucket: the 20 after it does not join the 5 before it
    lay3 = oracle.build_layout([(20, True), (100, True), (5, True)], 1, 50)
    assert lay3.bucket_of_tensor == [2, 1, 0]
    # properties on a random list
    rng = _rng(12)
    tensors = [(int(n), bool(w)) for n, w in zip(rng.integers(1, 5000, 300), rng.integers(0, 2, 300))]
    cap = 8000
    lay = oracle.build_layout(tensors, 2, cap)
    seen = [0] * len(tensors)
    prev_first = len(tensors)
    for bi, b in enumerate(lay.buckets):
        off = 0
        ids = [s.tensor for s in b.segments]
        assert ids == sorted(ids, reverse=True) and ids == list(range(ids[0], ids[-1] - 1, -1))
        assert ids[0] == prev_first - 1
        prev_first = ids[-1]
        for s in b.segments:
            assert s.offset == off and s.numel == tensors[s.tensor][0] and s.weight_decay == tensors[s.tensor][1]
            off += s.numel
            seen[s.tensor] += 1
            assert lay.bucket_of_tensor[s.tensor] == bi
        assert off == b.numel
        assert b.numel * 2 <= cap or len(b.segments) == 1
        if bi + 1 < len(lay.buckets) and len(b.segments) >= 1 and b.numel * 2 <= cap:
            nxt = tensors[lay.buckets[bi + 1].segments[0].tensor][0]
            assert (b.numel + nxt) * 2 > cap      # greedy: the next tensor did not fit
    assert seen == [1] * len(tensors) and prev_first == 0
    assert lay.num_params == sum(n for n, _ in tensors)
    # explicit assignment
    lay = oracle.build_layout([(4, True)] * 4, 4, 0, bucket_of_tensor=[0, 1, 2, 3])
    assert [b.numel for b in lay.buckets] == [4, 4, 4, 4]


def pin_step_scalars():
    hp = _hp(weight_decay=0.01)
    for t in (1, 2, 10, 1000, 100000):
        s = oracle.step_scalars(hp, t)
        b1, b2, lr, wd = (Fraction(hp.f32(k)) for k in ("beta1", "beta2", "lr", "weight_decay"))
        want = [1 - lr * wd, 1 - b1, 1 - b2, lr / (1 - b1 ** t)]
        for got, w in zip(s[:4], want):
            assert abs(Fraction(float(got)) - w) <= abs(w) * Fraction(1, 2 ** 23), t
        isq = Fraction(float(s[4]))
        assert abs(isq * isq * (1 - b2 ** t) - 1) <= Fraction(1, 2 ** 21), t


# --------------------------------------------------------------------------- Adam (L2 in the gradient) and SGD
def pin_adam_coupled_decay():
    # without decay Adam and AdamW are the same arithmetic, bit for bit
    hp0 = _hp(weight_decay=0.0)
    n, T = 500, 5
    rng = _rng(21)
    p0 = (rng.standard_normal(n) * 0.02).astype(F32)
    gs = [(rng.standard_normal(n) * 1e-3).astype(F32) for _ in range(T)]
    a = [p0.copy(), np.zeros(n, F32), np.zeros(n, F32)]
    b = [p0.copy(), np.zeros(n, F32), np.zeros(n, F32)]
    for t, g in enumerate(gs, 1):
        oracle.adamw_f32(*a, g, True, hp0, t)
        oracle.adam_f32(*b, g, True, hp0, t)
    for x, y in zip(a, b):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32))
    # with decay the penalty enters the gradient: zero gradient, first step: g' = wd*p, dp = -lr*g'/(|g'|+eps)
    hp = _hp(weight_decay=0.1)
    lr, eps, wd = hp.f32("lr"), hp.f32("eps"), hp.f32("weight_decay")
    pd, md, vd = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    oracle.adam_f64(pd, md, vd, np.zeros(n), True, hp, 1)
    gp = wd * p0.astype(np.float64)
    assert np.allclose(pd - p0, -lr * gp / (np.abs(gp) + eps), rtol=1e-10, atol=1e-18)
    assert np.allclose(md, (1 - hp.f32("beta1")) * gp, rtol=1e-13) and np.allclose(vd, (1 - hp.f32("beta2")) * gp * gp, rtol=1e-13)
    # masked tensor: no penalty, zero gradient leaves everything unchanged
    q = [p0.copy(), np.zeros(n, F32), np.zeros(n, F32)]
    oracle.adam_f32(*q, np.zeros(n, F32), False, hp, 1)
    assert np.array_equal(q[0], p0) and not q[1].any() and not q[2].any()
    # float order: g' = g + wd*p (one multiply, one add)
    g = gs[0]
    q = [p0.copy(), np.zeros(n, F32), np.zeros(n, F32)]
    oracle.adam_f32(*q, g, True, hp, 1)
    g2 = g + F32(wd) * p0
    assert np.array_equal(q[1], F32(1.0 - hp.f32("beta1")) * g2)
    # library: torch.optim.Adam with weight_decay, double
    tp = torch.nn.Parameter(torch.tensor(p0, dtype=torch.float64))
    opt = torch.optim.Adam([tp], lr=lr, betas=(hp.f32("beta1"), hp.f32("beta2")), eps=eps, weight_decay=wd, foreach=False)
    pd, md, vd = p0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t, g in enumerate(gs, 1):
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        oracle.adam_f64(pd, md, vd, g.astype(np.float64), True, hp, t)
    assert np.allclose(pd, tp.detach().numpy(), rtol=1e-11, atol=1e-16)
    assert np.allclose(md, opt.state[tp]["exp_avg"].numpy(), rtol=1e-11, atol=1e-18)
    assert np.allclose(vd, opt.state[tp]["exp_avg_sq"].numpy(), rtol=1e-11, atol=1e-24)
    # float variant near the double one
    q = [p0.copy(), np.zeros(n, F32), np.zeros(n, F32)]
    for t, g in enumerate(gs, 1):
        oracle.adam_f32(*q, g, True, hp, t)
    assert np.allclose(q[0], pd, rtol=0, atol=T * 4e-9 + 2e-9)


def pin_sgd_momentum():
    hp = HParams(lr=0.1, beta1=0.9, weight_decay=0.0, optimizer="sgd")
    lr, mu = hp.f32("lr"), hp.f32("beta1")
    g32 = np.array([1e-3, -2.5e-4, 0.7, -3.0], F32)
    gd = g32.astype(np.float64)
    T = 9
    pd, bd = np.zeros(4), np.zeros(4)
    p, b = np.zeros(4, F32), np.zeros(4, F32)
    total = np.zeros(4)
    for t in range(1, T + 1):
        oracle.sgd_f64(pd, bd, gd, False, hp)
        oracle.sgd_f32(p, b, g32, False, hp)
        want_b = gd * (1 - mu ** t) / (1 - mu)            # geometric series: b_t = g (1 + mu + ... + mu^(t-1))
        total += want_b
        assert np.allclose(bd, want_b, rtol=1e-12) and np.allclose(pd, -lr * total, rtol=1e-12)
        assert np.allclose(b, bd, rtol=1e-5) and np.allclose(p, pd, rtol=1e-5)
    # first step: the buffer is the gradient itself
    p, b = np.ones(4, F32), np.zeros(4, F32)
    oracle.sgd_f32(p, b, g32, False, hp)
    assert np.array_equal(b, g32) and np.array_equal(p, np.ones(4, F32) - F32(0.1) * g32)
    # zero gradient: the buffer decays geometrically and keeps moving p
    b0 = g32.copy()
    p, b = np.zeros(4, F32), b0.copy()
    z = np.zeros(4, F32)
    bb, pp = b0.copy(), np.zeros(4, F32)
    for t in range(6):
        oracle.sgd_f32(p, b, z, False, hp)
        bb = F32(0.9) * bb
        pp = pp - F32(0.1) * bb
        assert np.array_equal(b, bb) and np.array_equal(p, pp)
    # no momentum: plain gradient descent
    hp_plain = HParams(lr=0.1, beta1=0.0, weight_decay=0.0, optimizer="sgd")
    p, b = np.ones(4, F32), np.zeros(4, F32)
    for t in range(3):
        oracle.sgd_f32(p, b, g32, False, hp_plain)
    want = np.ones(4, F32)
    for t in range(3):
        want = want - F32(0.1) * g32
    assert np.array_equal(p, want)
    # L2 penalty and its mask; clipping scales the gradient before the penalty is added
    hp_wd = HParams(lr=0.1, beta1=0.9, weight_decay=0.5, optimizer="sgd")
    p, b = np.full(4, 2.0, F32), np.zeros(4, F32)
    oracle.sgd_f32(p, b, z, True, hp_wd)
    assert np.array_equal(b, np.full(4, 1.0, F32)) and np.array_equal(p, np.full(4, 2.0, F32) - F32(0.1) * F32(1.0))
    p, b = np.full(4, 2.0, F32), np.zeros(4, F32)
    oracle.sgd_f32(p, b, z, False, hp_wd)
    assert np.array_equal(p, np.full(4, 2.0, F32)) and not b.any()
    p, b = np.full(4, 2.0, F32), np.zeros(4, F32)
    oracle.sgd_f32(p, b, np.full(4, 4.0, F32), True, hp_wd, c=F32(0.25))
    assert np.array_equal(b, np.full(4, 2.0, F32))            # 4*0.25 + 0.5*2
    # library: torch.optim.SGD, double
    rng = _rng(22)
    n, T = 300, 6
    p0 = (rng.standard_normal(n) * 0.02).astype(F32)
    gs = [(rng.standard_normal(n) * 1e-3).astype(F32) for _ in range(T)]
    hp_t = HParams(lr=0.05, beta1=0.9, weight_decay=0.01, optimizer="sgd")
    tp = torch.nn.Parameter(torch.tensor(p0, dtype=torch.float64))
    opt = torch.optim.SGD([tp], lr=hp_t.f32("lr"), momentum=hp_t.f32("beta1"), weight_decay=hp_t.f32("weight_decay"), foreach=False)
    pd, bd = p0.astype(np.float64), np.zeros(n)
    p, b = p0.copy(), np.zeros(n, F32)
    for g in gs:
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        oracle.sgd_f64(pd, bd, g.astype(np.float64), True, hp_t)
        oracle.sgd_f32(p, b, g, True, hp_t)
    assert np.allclose(pd, tp.detach().numpy(), rtol=1e-13, atol=1e-18)
    assert np.allclose(bd, opt.state[tp]["momentum_buffer"].numpy(), rtol=1e-13, atol=1e-20)
    assert np.allclose(p, pd, rtol=0, atol=T * 4e-9) and np.abs(b - bd).max() <= 8 * T * 2 ** -24 * np.abs(bd).max()


def pin_driver_dispatches_optimizers():
    """OracleShadow routes every tensor through the optimizer named in the hyper-parameters."""
    tensors = [(40, True), (9, False), (70, True)]
    lay = oracle.build_layout(tensors, 4, 200)
    rng = _rng(23)
    p0 = [(rng.standard_normal(b.numel) * 0.02).astype(F32) for b in lay.buckets]
    g = {bi: [(rng.standard_normal(b.numel) * 1e-3).astype(F32) for _ in range(2)] for bi, b in enumerate(lay.buckets)}
    for name in ("adamw", "adam", "sgd"):
        hp = HParams(lr=1e-2, weight_decay=0.1, optimizer=name, max_grad_norm=1e-3)
        orc = oracle.OracleShadow(lay, hp, p0)
        orc.step(g)
        c = orc.last_coef
        for bi, b in enumerate(lay.buckets):
            r = oracle.fold(g[bi])
            for sgm in b.segments:
                sl = slice(sgm.offset, sgm.offset + sgm.numel)
                q = [p0[bi][sl].copy(), np.zeros(sgm.numel, F32), np.zeros(sgm.numel, F32)]
                if name == "sgd":
                    oracle.sgd_f32(q[0], q[1], r[sl].copy(), sgm.weight_decay, hp, c)
                else:
                    getattr(oracle, name + "_f32")(*q, r[sl].copy(), sgm.weight_decay, hp, 1, c)
                assert np.array_equal(orc.p[bi][sl], q[0]) and np.array_equal(orc.m[bi][sl], q[1])
    a = oracle.OracleShadow(lay, HParams(lr=1e-2, weight_decay=0.1, optimizer="adamw"), p0)
    b = oracle.OracleShadow(lay, HParams(lr=1e-2, weight_decay=0.1, optimizer="adam"), p0)
    a.step(g); b.step(g)
    assert not np.array_equal(a.p[0], b.p[0])         # decoupled and coupled decay differ


ALL_PINS = [
    pin_widen_bf16_exhaustive,
    pin_fold_identity_and_equal_workers,
    pin_fold_order_and_precision,
    pin_fold_bruteforce_rational,
    pin_adamw_first_step_closed_form,
    pin_zero_grad_geometric_decay,
    pin_constant_grad_closed_form,
    pin_weight_decay,
    pin_clip,
    pin_clip_is_noop_below_threshold,
    pin_whole_step_vs_torch,
    pin_f32_vs_torch_f32,
    pin_layout,
    pin_step_scalars,
    pin_adam_coupled_decay,
    pin_sgd_momentum,
    pin_driver_dispatches_optimizers,
]
