"""Randomised parity cases: shapes, dtypes, cluster structures and key widths drawn from fixed seeds, every case
within the documented limits.  They complement the hand-picked cases of test_gpu_parity.py: a dispatch mistake
(a shape sent to a kernel instance that cannot hold it) shows up here without anyone having thought of the shape."""
import numpy as np
import pytest
import torch

from workloads import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import gpu_harness
    gpu_harness.lsh.load_library()
    return gpu_harness


def _scale_fn(c):
    return (c * 0.5 + 1.0).to(c.dtype)


def _draw_path_case(seed):
    """(T, d, k, E, L, r, dtype, centers, sigma) within the limits of the library, or None to redraw."""
    rng = np.random.default_rng(seed)
    dtype = ["f32", "bf16"][rng.integers(0, 2)]
    item = 4 if dtype == "f32" else 2
    d = int(rng.choice([8, 16, 24, 40, 64, 72, 128, 136, 256, 264, 512, 520, 768, 1024, 1032, 2048]))
    if dtype == "f32":
        d = max(4, d // 2)
    r = int(rng.choice([2, 3, 4, 5, 8, 12, 16, 20, 24, 32, 40, 48, 64, 72, 88, 100, 128, 160, 256]))
    bits_per = int(np.ceil(np.log2(2 * r)))
    E = int(rng.choice([1, 2, 3, 4, 7, 8, 16, 31, 32, 64, 100, 256, 300]))
    ebits = int(np.ceil(np.log2(E))) if E > 1 else 0
    Lmax = min(10, 63 // bits_per, (64 - ebits) // bits_per)
    while Lmax >= 1 and (2 * r) ** Lmax >= 2 ** 63:
        Lmax -= 1
    if Lmax < 1:
        return None
    L = int(rng.integers(1, Lmax + 1))
    k = int(rng.integers(1, min(E, 4) + 1))
    T = int(rng.choice([1, 2, 31, 63, 64, 65, 200, 777, 2048, 4097, 5000, 8192, 8193, 12000, 24576, 30011, 66000, 70001]))
    if L * r > 1024 or T * d * item > 300e6 or T * L * r * d > 6e10:
        return None
    centers = max(1, int(T // rng.choice([1, 2, 6, 40, 400])))
    sigma = float(rng.choice([0.0, 0.02, 0.1, 0.3]))
    return T, d, k, E, L, r, dtype, centers, sigma


@pytest.mark.parametrize("seed", range(1000, 1030))
def test_random_path_case(H, seed):
    case, s = None, seed * 7919
    while case is None:
        case, s = _draw_path_case(s), s + 1
    T, d, k, E, L, r, dtype, centers, sigma = case
    print("case T=%d d=%d k=%d E=%d L=%d r=%d %s centers=%d sigma=%g" % case, flush=True)
    rng = np.random.default_rng(seed)
    ctr = rng.standard_normal((centers, d)).astype(np.float32)
    x = ctr[rng.integers(0, centers, T)] + sigma * rng.standard_normal((T, d)).astype(np.float32)
    tokens = synth.f32_to_storage(x, dtype)
    rot = synth.f32_to_storage(rng.standard_normal((L, r, d)).astype(np.float32), dtype)
    expert = np.argsort(rng.random((T, E)), axis=1)[:, :k].astype(np.int32)
    flags = int(rng.integers(0, 2)) if rng.random() < 0.3 else 0
    run = H.run_and_check(tokens, rot, expert, E, dtype, _scale_fn, flags=flags, use_seg_offsets=bool(rng.random() < 0.8))
    H.check_combine(run, tokens, rng.random((T, k)).astype(np.float32), k, dtype, flags=flags)
    H.check_backward(run, T, d, k, dtype, seed=seed, flags=flags)


@pytest.mark.parametrize("seed", range(2000, 2030))
def test_random_grouping_case(H, seed):
    # supplied bucket ids: skewed popularity (a few ids hold most tokens: clusters of thousands of members) and
    # skewed experts, keys of 2 to 64 bits, 1 to 300 000 tokens; grouping, centroids, restore and the backward pair
    rng = np.random.default_rng(seed)
    while True:
        dtype = ["f32", "bf16"][rng.integers(0, 2)]
        d = int(rng.choice([8, 16, 64, 136, 256, 520]))
        if dtype == "f32":
            d = max(4, d // 2)
        k = int(rng.choice([1, 1, 2, 3]))
        E = int(rng.choice([1, 2, 4, 8, 33, 64, 256]))
        k = min(k, E)
        L, r = [(1, 2), (1, 16), (2, 16), (3, 32), (4, 64), (6, 64), (8, 64), (9, 32)][rng.integers(0, 8)]
        bits = L * int(np.log2(2 * r))
        ebits = int(np.ceil(np.log2(E))) if E > 1 else 0
        T = int(rng.choice([1, 5, 1000, 4096, 4097, 20000, 40000, 70000, 131072, 200000, 300000]))
        if bits + ebits <= 64 and T * k * d * 4 <= 400e6:
            break
    pool_n = max(1, int(T // rng.choice([1, 3, 10, 100, 1000, 100000])))
    pool = rng.integers(0, 1 << bits, pool_n, dtype=np.uint64)
    mode = rng.integers(0, 3)
    if mode == 0:
        pick = rng.integers(0, pool_n, T)
    elif mode == 1:
        pick = np.minimum(rng.zipf(1.3, T) - 1, pool_n - 1)
    else:
        pick = np.minimum(rng.pareto(0.7, T).astype(np.int64), pool_n - 1)
    ids = pool[pick]
    emode = rng.integers(0, 3)
    if k == 1 and emode == 0:
        expert = (pick % E).astype(np.int32)[:, None]
    elif k == 1 and emode == 1:
        expert = np.minimum(rng.zipf(1.5, T) - 1, E - 1).astype(np.int32)[:, None]
    else:
        expert = np.argsort(rng.random((T, E)), axis=1)[:, :k].astype(np.int32)
    print("case T=%d d=%d k=%d E=%d key bits=%d %s pool=%d" % (T, d, k, E, bits + ebits, dtype, pool_n), flush=True)
    tokens = synth.f32_to_storage(rng.standard_normal((T, d)).astype(np.float32), dtype)
    rot = synth.f32_to_storage(rng.standard_normal((L, r, d)).astype(np.float32), dtype)
    run = H.run_and_check(tokens, rot, expert, E, dtype, _scale_fn, bucket_override=ids, skip_hash=True)
    H.check_backward(run, T, d, k, dtype, seed=seed)


@pytest.mark.parametrize("seed", range(3000, 3024))
def test_random_hash_gate_case(H, seed):
    import oracle
    rng = np.random.default_rng(seed)
    while True:
        dtype = ["f32", "bf16"][rng.integers(0, 2)]
        item = 4 if dtype == "f32" else 2
        d = int(rng.choice([1, 2, 3, 4, 8])) * (512 // item)          # rows of whole 512-byte blocks
        r = int(rng.choice([8, 16, 24, 32, 40, 64, 128, 256]))
        bits_per = int(np.ceil(np.log2(2 * r)))
        L = int(rng.integers(1, min(10, 62 // bits_per) + 1))
        E = int(rng.choice([1, 2, 3, 4, 8, 16, 30, 32, 64, 100, 128]))
        T = int(rng.choice([1, 63, 777, 4097, 8192, 8193, 20000, 24576, 24577, 40001, 65536, 65537, 70001]))
        if L * r <= 768 and T * d * item <= 400e6 and T * (L * r + E) * d <= 4e10:
            break
    print("case T=%d d=%d L=%d r=%d E=%d %s" % (T, d, L, r, E, dtype), flush=True)
    tokens = synth.f32_to_storage(rng.standard_normal((T, d)).astype(np.float32), dtype)
    rot = synth.f32_to_storage(rng.standard_normal((L, r, d)).astype(np.float32), dtype)
    gate = synth.f32_to_storage(rng.standard_normal((E, d)).astype(np.float32), dtype)
    xt, rt, gt = H.to_device(tokens, dtype), H.to_device(rot, dtype), H.to_device(gate, dtype)
    bt = torch.full((T + 4,), -1, dtype=torch.int64, device="cuda")
    lt = torch.full((T + 2, E), float("nan"), dtype=torch.float32, device="cuda")
    H.lsh.lshmoe_hash_gate(xt, rt, gt, bt[:T], lt[:T])
    torch.cuda.synchronize()
    assert np.all(bt[T:].cpu().numpy() == -1) and torch.isnan(lt[T:]).all(), "nothing is written past T"
    bucket = bt[:T].cpu().numpy().view(np.uint64)
    H.check_hash(bucket, tokens, rot, dtype)
    plain = torch.empty(T, dtype=torch.int64, device="cuda")
    H.lsh.lshmoe_hash(xt, rt, plain)
    torch.cuda.synchronize()
    assert np.array_equal(plain.cpu().numpy().view(np.uint64), bucket)
    ref = oracle.gate_logits_ref(tokens, gate, dtype)
    got = lt[:T].cpu().numpy().astype(np.float64)
    xa, wa = np.abs(oracle.widen(tokens, dtype)), np.abs(oracle.widen(gate, dtype))
    bound = (d / 16 + 8) * 2.0 ** -24 * (xa @ wa.T)     # binary32 accumulation, 16 products per MFMA
    assert np.max(np.abs(got - ref) - bound) <= 0.0
