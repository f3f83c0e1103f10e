"""Host-side checks of libshadow.so that need no GPU: exports, layout, argument validation."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_2507_13522_amd as sh
from paper_2507_13522_amd import binding
import synth
from harness import assert_layouts_agree, lib_layout, oracle_layout

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_every_declared_symbol():
    import glob
    headers = sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))
    assert [os.path.basename(h) for h in headers] == ["shadow.h", "shadow_measure.h"]
    hdr = "".join(open(h).read() for h in headers)
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(shadow_[a-z_0-9]+)\s*\(", hdr))
    assert len(declared) >= 30
    L = sh.lib()
    for name in sorted(declared):
        assert hasattr(L, name), f"{name} declared in shadow.h but not exported"
    assert declared == set(binding.EXPORTS)


def test_strerror():
    assert sh.shadow_strerror(0) == "ok"
    for code in range(-7, 0):
        assert sh.shadow_strerror(code) not in ("ok", "unknown status")
    assert sh.shadow_strerror(-99) == "unknown status"


@pytest.mark.parametrize("name", list(synth.WORKLOADS))
def test_layout_matches_oracle_on_workloads(name):
    wl = synth.get_workload(name)
    ol, ll = oracle_layout(wl), lib_layout(wl)
    assert_layouts_agree(ol, ll)
    if name == "tiny":
        assert ll.num_buckets == 4
    if name == "llama7b":
        # 50 MiB of bf16 = 26,214,400 elements: embeddings, w1/w2/w3 exceed it and sit alone
        sizes = [ll.bucket(b)[1] for b in range(ll.num_buckets)]
        assert sizes.count(131_072_000) == 2 and sizes.count(45_088_768) == 96
        assert max(s for s in sizes if s not in (131_072_000, 45_088_768)) <= 26_214_400


def test_layout_matches_oracle_on_random_lists():
    rng = np.random.default_rng(3)
    for trial in range(30):
        T = int(rng.integers(1, 60))
        tensors = [(int(rng.integers(1, 3000)), bool(rng.integers(0, 2))) for _ in range(T)]
        gb = int(rng.choice([2, 4]))
        cap = int(rng.integers(100, 6000))
        assert_layouts_agree(oracle.build_layout(tensors, gb, cap), sh.Layout(tensors, gb, cap))
    tensors = [(7, True), (9, False), (11, True), (13, True)]
    fixed = [1, 0, 1, 2]
    assert_layouts_agree(oracle.build_layout(tensors, 4, 0, fixed), sh.Layout(tensors, 4, 0, fixed))


def test_layout_rejects_bad_arguments():
    with pytest.raises(sh.ShadowError):
        sh.Layout([], 2, 100)
    with pytest.raises(sh.ShadowError):
        sh.Layout([(0, True)], 2, 100)
    with pytest.raises(sh.ShadowError):
        sh.Layout([(5, True)], 3, 100)
    with pytest.raises(sh.ShadowError):
        sh.Layout([(5, True)], 2, 0)
    with pytest.raises(sh.ShadowError):
        sh.Layout([(5, True), (6, True)], 2, 0, [0, 2])      # ids not dense
    with pytest.raises(sh.ShadowError):
        sh.Layout([(5, True), (6, True)], 2, 0, [0, 0xFFFFFFFF])   # id + 1 would wrap to zero buckets
    with pytest.raises(sh.ShadowError):
        sh.Layout([(5, True), (6, True)], 2, 0, [1, 1])      # bucket 0 unused
    with pytest.raises(sh.ShadowError):
        sh.Layout([((1 << 48) + 1, True)], 2, 1 << 20)           # beyond the largest supported tensor
    with pytest.raises(sh.ShadowError):
        sh.Layout([(1 << 47, True), (1 << 47, True), (8, True)], 2, 1 << 20)   # total beyond 2^48 elements
    big = sh.Layout([(1 << 40, True), (3, False)], 2, 1 << 20)   # sizes far beyond 32 bits are planned exactly
    assert big.num_params == (1 << 40) + 3 and big.num_buckets == 2 and big.bucket(1) == (64, 1 << 40, 1)
    lay = sh.Layout([(5, True)], 2, 100)
    with pytest.raises(sh.ShadowError) as e:
        lay.bucket(1)
    assert e.value.status == binding.EBUCKET


def test_init_validates_before_touching_the_gpu():
    lay = sh.Layout([(100, True)], 2, 1000)
    good = dict(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, max_grad_norm=0.0, num_workers=2,
                grad_dtype=sh.GRAD_BF16, reduce_op=sh.REDUCE_MEAN, num_streams=1)
    bad = [dict(beta1=1.0), dict(beta2=-0.1), dict(eps=0.0), dict(lr=-1.0), dict(num_workers=0), dict(num_workers=65),
           dict(grad_dtype=7), dict(grad_dtype=sh.GRAD_F32), dict(reduce_op=3), dict(num_streams=0), dict(num_streams=17),
           dict(weight_decay=-1.0), dict(launch=sh.LaunchShape(fold_block=96)), dict(launch=sh.LaunchShape(sweep_block=2048)),
           dict(launch=sh.LaunchShape(sweep_waves_per_cu=33)), dict(launch=sh.LaunchShape(fused_waves_per_cu=40)), dict(launch=sh.LaunchShape(max_launch_threads=(1 << 31) + 1))]
    for kw in bad:
        hp = sh.HParams(**{**good, **kw})
        with pytest.raises(sh.ShadowError) as e:
            sh.Shadow(lay, hp, 256, 512, 768, None)
        assert e.value.status == binding.EINVAL, kw
    hp = sh.HParams(**good)
    for ptrs in [(0, 512, 768), (256, 512 + 4, 768), (256, 256, 768)]:
        with pytest.raises(sh.ShadowError) as e:
            sh.Shadow(lay, hp, *ptrs, None)
        assert e.value.status == binding.EINVAL
    with pytest.raises(sh.ShadowError):       # scratch given although clipping is off
        sh.Shadow(lay, hp, 256, 512, 768, 1024)


def test_null_handles_are_rejected():
    L = sh.lib()
    assert L.shadow_sync(None) == binding.EINVAL
    assert L.shadow_apply_bucket(None, 0, None, 1, None) == binding.EINVAL
    assert L.shadow_ingest_bucket(None, 0, None, 1, None) == binding.EINVAL
    assert L.shadow_record_consumed(None, 0, None) == binding.EINVAL
    assert L.shadow_snapshot(None, None, None, None, None, None) == binding.EINVAL
    assert L.shadow_snapshot_attach(None, None, None, None) == binding.EINVAL
    assert L.shadow_snapshot_arm(None, None, None, None) == binding.EINVAL
    assert L.shadow_snapshot_record(None, None) == binding.EINVAL
    assert L.shadow_snapshot_wait(None, None) == binding.EINVAL
    assert L.shadow_num_buckets(None, None) == binding.EINVAL
    assert L.shadow_bucket_info(None, 0, None, None) == binding.EINVAL
    assert L.shadow_destroy(None) == binding.OK
    assert L.shadow_profile_kinds(None, 1) == binding.EINVAL
    assert L.shadow_copy_probe(None, None, 16, None, 0) == binding.EINVAL
    assert L.shadow_stream_probe(None, 1, None, 1, None, 16, None, 0, 0) == binding.EINVAL
    assert sh.shadow_stream_probe([], [], 16) == binding.EINVAL                     # no stream at all
    assert sh.shadow_stream_probe([256], [512], 24) == binding.EINVAL               # not a multiple of 16
    assert sh.shadow_stream_probe([256], [512, 768, 1024], 16) == binding.EINVAL    # a mix the kernel is not built for
    assert sh.shadow_stream_probe([256], [520], 16) == binding.EINVAL               # misaligned source
    assert sh.shadow_stream_probe([], [512], 16) == binding.EINVAL                  # reads alone need the sink
    assert sh.shadow_stream_probe([256], [512], 16, block=96) == binding.EINVAL
    assert sh.shadow_stream_probe([256], [512], 0) == binding.OK                    # nothing to do


def test_placement_advice():
    wl = synth.get_workload("llama7b")
    lay = lib_layout(wl)
    assert lay.arena_stride() == 32 << 30                       # 25.1 GiB arena -> 32 GiB
    W = wl.num_workers
    total = lay.staging_bytes(W)
    prev_end = 0
    for b in range(lay.num_buckets):
        n = lay.bucket(b)[1]
        for w in range(W):
            off = lay.staging_view(W, b, w)
            assert off >= prev_end
            if n * 2 >= (2 << 20):
                assert off % (2 << 20) == w * 4096             # views of one bucket are skewed by a page each
            else:
                assert off % 256 == 0
            prev_end = off + n * 2
    assert prev_end <= total <= 1.03 * lay.num_params * 2 * W    # bucket-major, little padding
    small = sh.Layout([(100, True), (7, False)], 4, 64)
    assert small.arena_stride() == 2 << 20 and small.num_buckets == 2
    assert small.staging_view(3, 0, 0) == 0 and small.staging_view(3, 0, 1) == 256 and small.staging_view(3, 1, 0) == 2 << 20
    with pytest.raises(sh.ShadowError):
        small.staging_view(3, 0, 3)
    with pytest.raises(sh.ShadowError):
        small.staging_view(3, 2, 0)


def test_device_plan():
    """Scratch arena, param and m end the first 96 GiB region, v starts the second, staging follows; nothing overlaps."""
    G = 1 << 30
    for name, scratch in (("llama7b", True), ("gpt1p3b", True), ("gpt2s", False), ("llama7b_w1", False)):
        wl = synth.get_workload(name)
        lay = lib_layout(wl)
        W = wl.num_workers
        plan = lay.device_plan(scratch, lay.staging_bytes(W))
        assert plan is not None and plan.block_bytes == 256 * G
        assert (plan.snap_param_offset, plan.snap_m_offset, plan.snap_v_offset) == (0, 0, 0)
        arena = lay.arena_numel * 4
        parts = [(plan.param_offset, arena), (plan.m_offset, arena), (plan.v_offset, arena), (plan.staging_offset, lay.staging_bytes(W))]
        if scratch:
            parts.append((plan.scratch_offset, arena))
            assert plan.scratch_offset + arena <= plan.param_offset          # first region, below param
        else:
            assert plan.scratch_offset == 0
        assert plan.param_offset + arena <= plan.m_offset and plan.m_offset + arena <= 96 * G
        assert plan.v_offset >= 96 * G and plan.staging_offset >= plan.v_offset + arena
        parts.sort()
        for (o1, n1), (o2, _) in zip(parts, parts[1:]):
            assert o1 % G == 0 and o1 + n1 <= o2
        assert parts[-1][0] + parts[-1][1] <= plan.block_bytes
    # without a staging buffer the offset is 0; a replica too large for the scheme gets no plan
    wl = synth.get_workload("llama7b")
    lay = lib_layout(wl)
    assert lay.device_plan(True, 0).staging_offset == 0
    assert lay.device_plan(True, lay.staging_bytes(32)) is None                # 32 resident views of 7B: 400 GiB
    ring = lay.device_plan(True, 100 << 30)                                   # a 100 GiB ring instead
    assert ring is not None and ring.staging_offset + (100 << 30) <= ring.block_bytes
    # a snapshot staging set (a second param, m, v) follows v; the views' buffer comes last
    snap = lay.device_plan(True, 48 << 30, True)
    assert snap is not None
    arena = lay.arena_numel * 4
    assert snap.snap_param_offset >= snap.v_offset + arena and snap.snap_m_offset >= snap.snap_param_offset + arena
    assert snap.snap_v_offset >= snap.snap_m_offset + arena and snap.staging_offset >= snap.snap_v_offset + arena
    assert snap.staging_offset + (48 << 30) <= snap.block_bytes
    assert lay.device_plan(True, lay.staging_bytes(8), True) is None          # all views resident AND a second state: too much
    huge = sh.Layout([(13_000_000_000, True)], 4, 1 << 40)
    assert huge.device_plan(False, 0) is None                          # two arenas exceed one region
    L = binding.lib()
    assert L.shadow_layout_device_plan(None, 0, 0, 0, None) == binding.EINVAL

