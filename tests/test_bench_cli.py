"""Host-side behaviour of bench.py that needs no GPU: refusing more than one GPU, failing loudly without a GPU,
and the workload generator's determinism (the module both the oracle's tests and the HIP path's tests share)."""
import os
import subprocess
import sys

import numpy as np

from workloads import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _run(*args, env=None):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          env={**os.environ, **(env or {})}, timeout=300)


def test_more_than_one_gpu_is_refused_with_a_message():
    res = _run("--gpus", "2")
    assert res.returncode != 0
    assert "single-GPU" in (res.stderr + res.stdout)
    res = _run("--gpus", "1", env={"WORLD_SIZE": "4"})
    assert res.returncode != 0 and "single-GPU" in (res.stderr + res.stdout)


def test_no_gpu_is_an_error_not_a_cpu_fallback():
    import torch
    if torch.cuda.is_available():
        return  # covered by the GPU tests on a GPU machine
    res = _run("--steps", "1", "--warmup", "0")
    assert res.returncode != 0
    assert "no GPU" in (res.stderr + res.stdout)
    assert not any(line.startswith("{") for line in res.stdout.splitlines()), "no benchmark line without a GPU"


def test_workloads_are_seeded_and_shaped_as_named():
    for name, (T, d, k, E, L, r) in {"tiny": (2048, 256, 1, 4, 2, 16), "swin": (25088, 512, 1, 32, 2, 32),
                                     "roberta": (16384, 768, 1, 16, 2, 32), "gpt": (32768, 1024, 2, 32, 3, 32),
                                     "t5": (65536, 1024, 2, 64, 4, 64)}.items():
        cfg = synth.config(name)
        assert (cfg.T, cfg.d, cfg.k, cfg.E, cfg.L, cfg.r) == (T, d, k, E, L, r)
    cfg = synth.config("gpt", T=512, centers=16)
    a, b = synth.generate(cfg), synth.generate(cfg)
    assert np.array_equal(a.tokens, b.tokens) and np.array_equal(a.expert, b.expert) and np.array_equal(a.rot, b.rot)
    c = synth.generate(cfg, seed=a.seed + 1)
    assert not np.array_equal(a.tokens, c.tokens)
    assert a.expert.shape == (512, 2) and a.expert.min() >= 0 and a.expert.max() < cfg.E
    assert np.all(a.expert[:, 0] != a.expert[:, 1]), "the k experts of a token are distinct"
    assert a.tokens.dtype == np.uint16 and a.tokens.shape == (512, cfg.d)
