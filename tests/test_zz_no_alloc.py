"""lshmoe_compress_static (the entry point that allocates nothing: its scratch is an array inside the library's
device image) against lshmoe_compress with a caller-owned workspace: every output bit for bit, on two calls in a
row, the second on a smaller input, so that whatever the first call left in the shared scratch is in the way."""
import numpy as np
import pytest
import torch

import paper_2411_08446_amd as lsh
from workloads import synth

pytestmark = pytest.mark.gpu


def _both(cfg):
    """Run lshmoe_compress and lshmoe_compress_static on the same inputs; return the two output sets."""
    w = synth.generate(cfg)
    dt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    if cfg.dtype == "f32":
        x = torch.from_numpy(np.ascontiguousarray(w.tokens)).cuda()
        rot = torch.from_numpy(np.ascontiguousarray(w.rot)).cuda()
    else:
        x = torch.from_numpy(np.ascontiguousarray(w.tokens).view(np.int16)).cuda().view(torch.bfloat16)
        rot = torch.from_numpy(np.ascontiguousarray(w.rot).view(np.int16)).cuda().view(torch.bfloat16)
    expert = torch.from_numpy(w.expert).cuda()
    bucket = torch.empty(cfg.T, dtype=torch.int64, device="cuda")
    lsh.lshmoe_hash(x, rot, bucket)
    outs = []
    for static in (False, True):
        o = lsh.CompressOutputs.allocate(cfg.T, cfg.d, cfg.k, cfg.E, cfg.L, cfg.r, dt)
        for t in (o.seg_offsets, o.seg_expert, o.expert_offsets, o.perm, o.seg_of, o.num_segments):
            t.fill_(-7)
        o.centroids.view(torch.int16 if cfg.dtype == "bf16" else torch.int32).fill_(0x7FC0 if cfg.dtype == "bf16" else 0x7FC00000)
        o.workspace.fill_(0xA5)
        if static:
            before = torch.cuda.memory_allocated()
            lsh.lshmoe_compress_static(x, expert, bucket, cfg.E, cfg.L, cfg.r, o)
            assert torch.cuda.memory_allocated() == before
            torch.cuda.synchronize()
            assert bool((o.workspace == 0xA5).all()), "the static entry point must not touch the caller's workspace"
        else:
            lsh.lshmoe_compress(x, expert, bucket, cfg.E, cfg.L, cfg.r, o)
        torch.cuda.synchronize()
        outs.append(o)
    return outs


def _assert_same(a, b, cfg):
    S = int(a.num_segments.item())
    assert S == int(b.num_segments.item()) and 0 < S <= cfg.N
    assert torch.equal(a.seg_offsets[:S + 1], b.seg_offsets[:S + 1])
    assert torch.equal(a.seg_expert[:S], b.seg_expert[:S])
    assert torch.equal(a.expert_offsets, b.expert_offsets)
    assert torch.equal(a.perm, b.perm)
    assert torch.equal(a.seg_of, b.seg_of)
    bits = torch.int16 if cfg.dtype == "bf16" else torch.int32
    assert torch.equal(a.centroids[:S].view(bits), b.centroids[:S].view(bits))      # same kernels: bit for bit
    assert torch.equal(a.centroids[S:].view(bits), b.centroids[S:].view(bits))      # rows beyond S untouched by both
    return S


def test_static_scratch_matches_workspace_twice_second_smaller():
    # first call: long clusters (window sums and their counters live in the scratch) at the GPT shape;
    # second call: a smaller input of another shape and dtype, which finds the first call's leftovers
    big = synth.config("gpt", T=16384, centers=8, sigma=0.001, gate="content")
    S1 = _assert_same(*_both(big), big)
    small = synth.config("tiny", T=1500)
    S2 = _assert_same(*_both(small), small)
    again = synth.config("swin", T=6000, centers=4, sigma=0.001, gate="content")
    S3 = _assert_same(*_both(again), again)
    print("static scratch: S = %d, %d, %d" % (S1, S2, S3))


def test_static_scratch_rejects_sizes_beyond_its_limit():
    cfg = synth.config("t5")
    T = 4 * cfg.T                                     # four times the largest paper shape: needs ~47 MB of scratch
    assert lsh.lshmoe_workspace_bytes(T, cfg.d, cfg.k, cfg.E, cfg.L, cfg.r, lsh.LSHMOE_BF16) > (16 << 20)
    lib = lsh.load_library()
    p = 0x1000
    rc = lib.lshmoe_compress_static(p, p, p, T, cfg.d, cfg.k, cfg.E, cfg.L, cfg.r, lsh.LSHMOE_BF16, p, p, p, p, p, p, p, None)
    assert rc == lsh.LSHMOE_ERR_WORKSPACE
    assert b"scratch" in lib.lshmoe_last_error()
