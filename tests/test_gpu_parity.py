"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element, on the same seeded inputs.  Integer outputs bit-exact (hash ids
modulo near ties, which are counted); centroids and restored rows within
1e-5 (fp32) / 2e-2 (bf16) row-scaled."""
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


def _standin(cfg, seed):
    return lambda c: synth.expert_standin(c, cfg, seed)


def _rand_inputs(seed, T, d, k, E, L, r, dtype, centers=None, sigma=0.1):
    rng = np.random.default_rng(seed)
    if centers:
        ctr = rng.standard_normal((centers, d)).astype(np.float32)
        x = ctr[rng.integers(0, centers, T)] + sigma * rng.standard_normal((T, d)).astype(np.float32)
    else:
        x = rng.standard_normal((T, d)).astype(np.float32)
    tokens = synth.f32_to_storage(x, dtype)
    rot = synth.f32_to_storage(rng.standard_normal((L, r, d)).astype(np.float32), dtype)
    expert = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    return tokens, rot, expert


def _scale_fn(c):
    return (c * 0.5 + 1.0).to(c.dtype)


# ------------------------------------------------------------------ named configs
@pytest.mark.parametrize("name,T", [("tiny", None), ("swin", 3001), ("roberta", 2500), ("gpt", 2077), ("t5", 1500)])
def test_named_configs_reduced(H, name, T):
    cfg = synth.config(name) if T is None else synth.config(name, T=T, centers=max(8, synth.config(name).centers * T // synth.config(name).T))
    w = synth.generate(cfg)
    print("case", cfg.name, "T", cfg.T, flush=True)
    run = H.run_and_check(w.tokens, w.rot, w.expert, cfg.E, cfg.dtype, _standin(cfg, w.seed))
    print("  S/N %.3f  tie flips %d" % (run.S / cfg.N, run.ties), flush=True)


@pytest.mark.parametrize("name", ["swin", "roberta", "gpt", "t5"])
def test_named_configs_full_size(H, name):
    cfg = synth.config(name)
    w = synth.generate(cfg)
    print("case", cfg.name, "full size T", cfg.T, flush=True)
    run = H.run_and_check(w.tokens, w.rot, w.expert, cfg.E, cfg.dtype, _standin(cfg, w.seed))
    print("  S/N %.3f  tie flips %d" % (run.S / cfg.N, run.ties), flush=True)
    # the fused gate-weighted combine and the backward pair at the same size, on the clusters of this run
    H.check_combine(run, w.tokens, w.gate_weight, cfg.k, cfg.dtype)
    H.check_backward(run, cfg.T, cfg.d, cfg.k, cfg.dtype, seed=w.seed + 17)


def test_content_correlated_gate_long_segments(H):
    # the regime the paper measured: same-cluster tokens go to the same expert -> long clusters
    cfg = synth.config("swin", T=6000, centers=40, gate="center_mod")
    w = synth.generate(cfg)
    run = H.run_and_check(w.tokens, w.rot, w.expert, cfg.E, cfg.dtype, _standin(cfg, w.seed))
    assert run.S / cfg.N < 0.3


def test_hash_count_sweep_refines_clusters(H):
    # Section 4.3's sweep of the number of hash functions (2, 4, 6, 8, 10), hash lists being prefixes of one
    # another: every L is checked against the oracle stage by stage; a further hash function only splits
    # clusters, so S/N does not fall, and the ids of the shorter list are the longer one's with the last
    # mixed-radix digits dropped.  L = 10 with r = 32 needs two passes over the tokens (320 rows of R).
    r = 32
    cfg = synth.config("gpt", T=8192 + 5, L=10, r=r, E=8, gate="content", sigma=0.05, centers=256)
    w = synth.generate(cfg)
    rates, prev_seg, prev_b, prev_L, prev_ties = [], None, None, None, 0
    for L in (2, 4, 6, 8, 10):
        print("case hash-count sweep L", L, flush=True)
        run = H.run_and_check(w.tokens, w.rot[:L], w.expert, cfg.E, cfg.dtype, _standin(cfg, w.seed))
        seg_of = run.out.seg_of.cpu().numpy().copy()
        if prev_seg is not None and run.ties == 0 and prev_ties == 0:   # a legal near-tie flip may differ between runs
            assert np.array_equal(run.bucket // np.uint64((2 * r) ** (L - prev_L)), prev_b)
            pairs = np.unique(np.stack([seg_of, prev_seg], axis=1), axis=0)
            assert len(pairs) == run.S
        rates.append(run.S / cfg.N)
        prev_seg, prev_b, prev_L, prev_ties = seg_of, run.bucket.copy(), L, run.ties
    print("  S/N by L:", ["%.3f" % x for x in rates], flush=True)
    assert rates == sorted(rates) and rates[0] < rates[-1]


# ------------------------------------------------------------------ shapes and edge cases
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T,d,k,E,L,r", [
    (1, 8, 1, 1, 1, 2),          # smallest everything
    (37, 16, 2, 3, 1, 3),        # odd r, ragged T
    (129, 24, 1, 5, 3, 5),       # one token past a block of 128
    (1000, 40, 3, 7, 2, 12),     # r not a multiple of 8
    (513, 64, 2, 300, 4, 16),    # many experts (9 expert bits)
    (300, 32, 4, 4, 8, 64),      # k == E, 56 bucket bits
    (700, 264, 1, 2, 2, 256),    # r at the supported maximum, two passes over the tokens
    (2500, 128, 2, 8, 5, 40),    # 200 rows of R in one pass, odd tile split
    (640, 72, 1, 6, 6, 8),       # the paper's default count of hash functions
    (300, 4096, 2, 4, 2, 16),    # rows of 8 KB (bf16) / 16 KB (binary32)
])
def test_shapes(H, dtype, T, d, k, E, L, r):
    tokens, rot, expert = _rand_inputs(100 + T, T, d, k, E, L, r, dtype, centers=max(2, T // 6))
    H.run_and_check(tokens, rot, expert, E, dtype, _scale_fn)


@pytest.mark.parametrize("N", [4097, 32768, 32769, 70001, 131071, 131072, 300000, 524288, 524289])
@pytest.mark.parametrize("E,L,r", [(1, 1, 2), (2, 1, 4), (3, 2, 4), (8, 1, 32), (5, 2, 16), (64, 2, 32), (9, 4, 16),
                                   (64, 4, 64), (2, 6, 64), (100, 7, 64), (256, 8, 64)])
def test_group_routes_by_key_width_and_size(H, N, E, L, r):
    # The grouping step picks its route by the number of assignments and the width of the (expert, bucket) key:
    # one workgroup up to 4096, one global pass on the top key bits plus sorts inside the bins up to 256 tiles
    # (keys of at most 9 bits need no bin sort), radix passes beyond.  Keys from 2 bits to all 64, with bucket
    # ids drawn from a pool a third as large as N so that clusters of several members exist at every width.
    d, dtype = 8, "bf16"
    rng = np.random.default_rng(N * 31 + E)
    tokens = synth.f32_to_storage(rng.standard_normal((N, d)).astype(np.float32), dtype)
    rot = synth.f32_to_storage(rng.standard_normal((L, r, d)).astype(np.float32), dtype)
    expert = rng.integers(0, E, (N, 1)).astype(np.int32)
    bits = L * int(np.log2(2 * r))
    pool = rng.integers(0, 1 << bits, max(1, N // 3), dtype=np.uint64)
    pool[0], pool[-1] = 0, (1 << bits) - 1                          # both ends of the id range
    ids = pool[rng.integers(0, pool.size, N)]
    print("case group N", N, "E", E, "bucket bits", bits, flush=True)
    H.run_and_check(tokens, rot, expert, E, dtype, _scale_fn, bucket_override=ids, skip_hash=True)


@pytest.mark.parametrize("N,bins_used,distinct", [
    (4100, 1, 3), (6149, 1, 4000), (10240, 1, 7), (34817, 1, 20000), (65536, 1, 1), (131072, 1, 90000),
    (524288, 1, 300000), (524288, 1, 2), (70001, 3, 50000), (200003, 5, 11), (300000, 2, 150000), (40000, 7, 64)])
def test_group_bins_of_many_chunks(H, N, bins_used, distinct):
    # Bins of the one global pass that hold 2 .. 256 chunks of 2048 keys (all keys share the top key bits of a few
    # bins): the chunks are merged pairwise by the workgroups that sorted them, level by level; odd chunk counts,
    # a ragged last chunk, runs without a neighbour, many equal keys and all-distinct keys.
    d, dtype, E, L, r = 8, "bf16", 4, 4, 16                     # 2 expert bits + 20 bucket bits: top 9 bits pick the bin
    rng = np.random.default_rng(N + 7 * bins_used + distinct)
    tokens = synth.f32_to_storage(rng.standard_normal((N, d)).astype(np.float32), dtype)
    rot = synth.f32_to_storage(rng.standard_normal((L, r, d)).astype(np.float32), dtype)
    low_bits = 20 - 7                                            # key bits below the bin digit
    tops = rng.choice(4 << 7, bins_used, replace=False)          # (expert, top 7 bucket bits) of the bins used
    pool_top = tops[rng.integers(0, bins_used, distinct)]
    pool_low = rng.integers(0, 1 << low_bits, distinct, dtype=np.uint64)
    pick = rng.integers(0, distinct, N)
    top = pool_top[pick]
    expert = (top >> 7).astype(np.int32).reshape(N, 1)
    ids = ((top & 127).astype(np.uint64) << np.uint64(low_bits)) | pool_low[pick]
    print("case many chunks N", N, "bins", bins_used, "distinct keys", distinct, flush=True)
    H.run_and_check(tokens, rot, expert, E, dtype, _scale_fn, bucket_override=ids, skip_hash=True)


def test_chunk_merges_give_the_same_result_every_time(H):
    # The merges inside the bin-sort launch depend on which of two neighbouring workgroups finishes last; the result
    # must not.  One bin of 64 chunks and three bins of a dozen, forty calls on the same buffers (workspace included),
    # every output compared with the first call's (which the parity cases above compare with the oracle).
    lsh = H.lsh
    E, L, r, d, N = 4, 4, 16, 8, 131072
    rng = np.random.default_rng(99)
    for bins_used in (1, 3):
        tops = rng.choice(4 << 7, bins_used, replace=False)
        top = tops[rng.integers(0, bins_used, N)]
        expert = torch.tensor((top >> 7).astype(np.int32).reshape(N, 1), device="cuda")
        ids = torch.tensor((((top & 127).astype(np.uint64) << np.uint64(13)) |
                            rng.integers(0, 1 << 13, N, dtype=np.uint64)).astype(np.int64), device="cuda")
        x = torch.randn((N, d), device="cuda").to(torch.bfloat16)
        out = lsh.CompressOutputs.allocate(N, d, 1, E, L, r, torch.bfloat16)
        first = None
        for call in range(40):
            lsh.lshmoe_compress(x, expert, ids, E, L, r, out)
            torch.cuda.synchronize()
            S = int(out.num_segments.item())
            got = (S, out.perm.clone(), out.seg_of.clone(), out.seg_offsets[:S + 1].clone(), out.seg_expert[:S].clone(),
                   out.centroids[:S].clone())
            if first is None:
                first = got
                continue
            assert got[0] == first[0], "call %d: cluster count differs" % call
            for a, b in zip(got[1:], first[1:]):
                assert torch.equal(a, b), "call %d differs from the first call" % call


def test_large_inputs_take_the_histogram_scan_scatter_route(H):
    # more than 256 sort tiles: per-pass histogram + table scan + scatter kernels
    tokens, rot, expert = _rand_inputs(41, 280000, 8, 2, 3, 2, 4, "bf16", centers=5000)
    H.run_and_check(tokens, rot, expert, 3, "bf16", _scale_fn)
    # more than 4096 numbering tiles: scanned tile counts
    tokens, rot, expert = _rand_inputs(42, 2150000, 8, 2, 2, 3, 2, "bf16", centers=3000)
    H.run_and_check(tokens, rot, expert, 2, "bf16", _scale_fn)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_all_tokens_identical_one_cluster(H, dtype):
    T, d, E = 3000, 64, 1
    tokens, rot, _ = _rand_inputs(7, 1, d, 1, E, 2, 16, dtype)
    tokens = np.repeat(tokens, T, axis=0)
    expert = np.zeros((T, 1), np.int32)
    run = H.run_and_check(tokens, rot, expert, E, dtype, _scale_fn)
    assert run.S == 1
    if dtype == "bf16":      # binary32 sum / n rounds back to the very same bf16 value
        assert np.array_equal(run.centroids[0], tokens[0])
    else:                    # in binary32 the sum n*x itself rounds: one ulp
        assert np.all(np.abs(run.centroids[0] - tokens[0]) <= 2.0 ** -23 * np.abs(tokens[0]))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("d,k", [(64, 1), (1032, 1), (520, 2), (4096, 1)])
def test_long_clusters_are_summed_in_windows(H, dtype, d, k):
    # cluster sizes around the window length of the centroid step (128 sorted positions) and far beyond it, with
    # heads on and off the window grid; d = 1032 makes rows wider than one pass of a wave over the row; with
    # d = 4096 the four partial rows of a workgroup-shared sum no longer fit the LDS set aside for them, so
    # clusters of 33..1024 members stay with one wave
    sizes = [128, 129, 1, 127, 256, 257, 3, 1000, 2, 5000, 131, 1, 1, 384, 640, 7, 2049]
    T, E, L, r = sum(sizes), 3, 2, 16
    tokens, rot, _ = _rand_inputs(21, T, d, 1, E, L, r, dtype)
    rng = np.random.default_rng(22)
    group = np.repeat(np.arange(len(sizes)), sizes)
    where = rng.permutation(T)                       # members of a cluster are scattered over the tokens
    ids = np.empty(T, np.uint64)
    ids[where] = group.astype(np.uint64)
    if k == 1:
        expert = np.empty((T, 1), np.int32)
        expert[where, 0] = group * E // len(sizes)   # non-decreasing with the group: cluster order = group order
    else:
        expert = np.tile(np.array([[2, 0]], np.int32), (T, 1))
    run = H.run_and_check(tokens, rot, expert, E, dtype, _scale_fn, bucket_override=ids)
    assert run.S == k * len(sizes)
    n = np.diff(run.out.seg_offsets[:run.S + 1].cpu().numpy())
    assert sorted(n.tolist()) == sorted(sizes * k)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_one_huge_cluster_many_windows(H, dtype):
    # 20000 identical tokens on the multi-launch grouping route: 157 window sums are combined by the last wave
    T, d, E = 20000, 64, 2
    tokens, rot, _ = _rand_inputs(23, 1, d, 1, E, 2, 16, dtype)
    tokens = np.repeat(tokens, T, axis=0)
    expert = np.ones((T, 1), np.int32)
    run = H.run_and_check(tokens, rot, expert, E, dtype, _scale_fn)
    assert run.S == 1
    if dtype == "bf16":
        assert np.array_equal(run.centroids[0], tokens[0])
    else:
        assert np.all(np.abs(run.centroids[0] - tokens[0]) <= 2.0 ** -23 * np.abs(tokens[0]))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_every_token_its_own_cluster_reconstructs_exactly(H, dtype):
    # supplied bucket ids are all distinct: every cluster has one member, Y == E(x) bit for bit
    T, d, k, E, L, r = 1111, 48, 2, 4, 4, 64
    tokens, rot, expert = _rand_inputs(8, T, d, k, E, L, r, dtype)
    ids = np.random.default_rng(3).permutation(T).astype(np.uint64) * np.uint64(104729)
    run = H.run_and_check(tokens, rot, expert, E, dtype, _scale_fn, bucket_override=ids)
    assert run.S == T * k
    assert np.array_equal(run.y, run.expert_out[run.out.seg_of.cpu().numpy()])


def test_zero_tokens_and_exact_ties(H):
    # all-zero tokens hash to code 0 in every hash; +-tied coordinates resolve to the lowest index
    d, r, L = 16, 8, 2
    rot = np.zeros((L, r, d), np.float32)
    rot[0, np.arange(r), np.arange(r)] = 1.0
    rot[1, np.arange(r), np.arange(r) + 8] = 1.0
    x = np.zeros((6, d), np.float32)
    x[1, 2] = 3.0; x[1, 5] = -3.0            # tie between coordinates 2 (+) and 5 (-) -> 2
    x[2, 7] = -1.0; x[2, 0] = -1.0           # tie 0, 7 both negative -> 0 + r
    x[3, 8 + 4] = 2.0; x[3, 8 + 6] = 2.0     # second hash tie -> 4
    x[4, 3] = -0.0                           # negative zero counts as positive
    x[5, :] = 1.0                            # all equal
    expert = np.zeros((6, 1), np.int32)
    run = H.run_and_check(x, rot, expert, 1, "f32", _scale_fn)
    assert run.bucket.tolist() == [0, 2 * 16, 8 * 16, 4, 0, 0]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_exact_ties_on_the_fast_hash_instance(H, dtype):
    # rows of 4 x 128 bytes and r a multiple of 8 select the fast kernel instance; +m / -m ties inside one lane's
    # rows (rows 1 and 2 of a tile sit in the same lane) and across the two lane halves (rows 2 and 5)
    d = 256 if dtype == "bf16" else 128
    r, L = 8, 2
    rot = np.zeros((L, r, d), np.float32)
    rot[0, np.arange(r), np.arange(r)] = 1.0
    rot[1, np.arange(r), np.arange(r) + 8] = 1.0
    x = np.zeros((8, d), np.float32)
    x[0, 1] = -3.0; x[0, 2] = 3.0            # same lane, lowest row negative -> code 1 + r
    x[1, 1] = 3.0; x[1, 2] = -3.0            # same lane, lowest row positive -> code 1
    x[2, 2] = 3.0; x[2, 5] = -3.0            # different lane halves -> code 2
    x[3, 2] = -3.0; x[3, 5] = 3.0            # -> code 2 + r
    x[4, 8 + 6] = -1.0; x[4, 8 + 7] = 1.0; x[4, 8 + 3] = 1.0   # second hash: three-way tie -> row 3, positive
    x[5, :] = 0.0                            # zero token
    x[6, 0:8] = -2.0                         # all rows tie, all negative -> 0 + r
    x[7, 4] = -0.0                           # negative zero counts as positive
    expert = np.zeros((8, 1), np.int32)
    run = H.run_and_check(synth.f32_to_storage(x, dtype), synth.f32_to_storage(rot, dtype), expert, 1, dtype, _scale_fn)
    assert run.bucket.tolist() == [9 * 16, 1 * 16, 2 * 16, 10 * 16, 3, 0, 8 * 16, 0]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T,L,r", [(65536 + 77, 4, 64), (65536 + 77, 2, 256), (65536 + 77, 7, 32),
                                   (65536 + 77, 5, 32), (65536 + 77, 6, 32),
                                   (32768 + 77, 3, 32), (24576 + 3, 1, 16), (16384 + 5, 2, 32), (8192 + 1, 2, 64),
                                   # beyond 256 workgroups of 128 tokens: the short-ring instances, 1..4 row tiles
                                   (65536 + 77, 1, 16), (40000, 2, 64), (50000 + 1, 4, 32), (33000, 2, 32), (70000, 3, 40)])
def test_hash_streaming_instances(H, dtype, T, L, r):
    _hash_case(H, dtype, T, L, r)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T", [777, 8192 + 33, 24576 + 9])
@pytest.mark.parametrize("L,r", [(1, 32), (2, 32), (3, 32), (4, 32), (5, 32), (6, 32), (7, 32), (8, 32), (10, 16),
                                 (4, 40), (6, 24), (7, 20), (2, 88), (1, 160), (9, 32), (3, 100)])
def test_hash_every_row_tile_count(H, dtype, T, L, r):
    # 1..8 tiles of 32 rows per pass over the tokens (L * r rows, at most 256 per pass), at sizes that take the
    # small, the 64-token and the 128-token workgroups; 129..160 rows (5 tiles) must take a 6-tile instance;
    # r = 20 and r = 100 are not multiples of 8 (general epilogue), (9, 32) and (3, 100) need two passes.
    _hash_case(H, dtype, T, L, r)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T", [777, 8192 + 33, 65536 + 77])
@pytest.mark.parametrize("L,r", [(1, 32), (4, 32), (5, 32), (6, 32), (8, 32), (3, 100), (2, 256)])
def test_hash_rows_with_a_tail(H, dtype, T, L, r):
    # rows of 33 16-byte pieces: not a whole number of 128-byte chunks, so every size takes the general kernel
    # with its tail step, at every number of row tiles
    _hash_case(H, dtype, T, L, r, d=264 if dtype == "bf16" else 132)


def _hash_case(H, dtype, T, L, r, d=None):
    # Large inputs with rows of whole 128-byte chunks take the kernels that stage both operands through LDS:
    # 193..256 rows of R per pass and T >= 65536 the one that splits the rows of R between two waves and joins the
    # halves at the end (r = 256 puts ONE hash on both halves, L = 7 with r = 32 leaves the last 32 staged rows
    # unused); up to 128 rows the 128-token (T >= 24576) or 64-token workgroups.  Random tokens plus exact +-ties
    # inside a lane, across lane halves, across tiles and across the two row halves, at the start and in the
    # ragged tail.
    import oracle
    if d is None:
        d = 256 if dtype == "bf16" else 128
    rng = np.random.default_rng(41)
    x = rng.standard_normal((T, d)).astype(np.float32)
    rot = rng.standard_normal((L, r, d)).astype(np.float32) * 0.05
    cols = min(r, d)
    for l in range(L):                        # rows 0..cols-1 of every hash pick out one coordinate each
        rot[l, :cols, :] = 0.0
        rot[l, np.arange(cols), (np.arange(cols) + 8 * l) % d] = 1.0
    special = [0, 1, 2, 3, 4, 5, 31, 32, 255, 256, T - 79, T - 78, T - 2, T - 1]
    pairs = [(1, 2), (2, 5), (3, 40 % cols), (10, min(cols, 200) - 1), (0, cols - 1), (7, 8), (33 % cols, 97 % cols)]
    for j, t in enumerate(special):
        x[t, :] = 0.0
        a, b = pairs[j % len(pairs)]
        sgn = 1.0 if j % 2 else -1.0
        x[t, a % d] = sgn * 4.0               # hash 0 sees rows a and b tie at magnitude 4 with opposite signs
        x[t, b % d] = -sgn * 4.0
    x[special[5], :] = 0.0                    # and one all-zero token
    tokens, rots = synth.f32_to_storage(x, dtype), synth.f32_to_storage(rot, dtype)
    xt, rt = H.to_device(tokens, dtype), H.to_device(rots, dtype)
    bt = torch.full((T + 8,), -1, dtype=torch.int64, device="cuda")
    H.lsh.lshmoe_hash(xt, rt, bt[:T])
    torch.cuda.synchronize()
    got = bt.cpu().numpy()
    assert np.all(got[T:] == -1), "ids past T must stay untouched"
    bucket = got[:T].view(np.uint64)
    H.check_hash(bucket, tokens, rots, dtype)
    ref, _, margin, _ = oracle.hash_ref(tokens, rots, dtype)
    assert np.array_equal(bucket[special], ref[special]), "exact ties resolve to the lowest row, as in the oracle"


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_no_residual_flag_and_without_seg_offsets(H, dtype):
    tokens, rot, expert = _rand_inputs(9, 900, 32, 2, 6, 2, 8, dtype, centers=30)
    H.run_and_check(tokens, rot, expert, 6, dtype, _scale_fn, flags=H.lsh.LSHMOE_FLAG_NO_RESIDUAL)
    H.run_and_check(tokens, rot, expert, 6, dtype, _scale_fn, use_seg_offsets=False)


@pytest.mark.parametrize("name,T", [("gpt", 3000), ("t5", 2200)])
def test_fused_gate_weighted_combine_named(H, name, T):
    cfg = synth.config(name, T=T, centers=120)
    w = synth.generate(cfg)
    run = H.run_and_check(w.tokens, w.rot, w.expert, cfg.E, cfg.dtype, _standin(cfg, w.seed))
    H.check_combine(run, w.tokens, w.gate_weight, cfg.k, cfg.dtype)
    H.check_combine(run, w.tokens, w.gate_weight, cfg.k, cfg.dtype, flags=H.lsh.LSHMOE_FLAG_NO_RESIDUAL)
    H.check_combine(run, w.tokens, w.gate_weight, cfg.k, cfg.dtype, use_seg_offsets=False)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T,d,k,E", [(700, 24, 3, 5), (333, 512, 1, 4), (50, 8, 4, 4), (61, 16, 6, 7), (130, 1024, 5, 9)])
def test_fused_gate_weighted_combine_shapes(H, dtype, T, d, k, E):
    tokens, rot, expert = _rand_inputs(77 + T, T, d, k, E, 2, 8, dtype, centers=max(2, T // 8))
    gw = np.random.default_rng(T).random((T, k)).astype(np.float32) + 0.1
    run = H.run_and_check(tokens, rot, expert, E, dtype, _scale_fn)
    H.check_combine(run, tokens, gw, k, dtype)
    # weights of one reproduce the plain sum of the k restored rows
    ones = np.ones((T, k), np.float32)
    H.check_combine(run, tokens, ones, k, dtype)


# ------------------------------------------------------------------ backward
@pytest.mark.parametrize("name,T", [("tiny", None), ("gpt", 3000), ("t5", 2200), ("swin", 4000)])
def test_backward_named(H, name, T):
    cfg = synth.config(name) if T is None else synth.config(name, T=T, centers=max(8, synth.config(name).centers * T // synth.config(name).T))
    w = synth.generate(cfg)
    run = H.run_and_check(w.tokens, w.rot, w.expert, cfg.E, cfg.dtype, _standin(cfg, w.seed))
    H.check_backward(run, cfg.T, cfg.d, cfg.k, cfg.dtype, seed=31)
    H.check_backward(run, cfg.T, cfg.d, cfg.k, cfg.dtype, seed=32, flags=1)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T,d,k,E", [(700, 24, 3, 5), (333, 512, 1, 4), (50, 8, 4, 4), (1, 64, 1, 1)])
def test_backward_shapes(H, dtype, T, d, k, E):
    tokens, rot, expert = _rand_inputs(33, T, d, k, E, 2, 4, dtype, centers=6)
    run = H.run_and_check(tokens, rot, expert, E, dtype, _scale_fn)
    H.check_backward(run, T, d, k, dtype, seed=34)
    H.check_backward(run, T, d, k, dtype, seed=35, flags=1)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_long_clusters(H, dtype):
    # the segment sum of clusters longer than a window goes through the window sums too
    sizes = [128, 129, 1, 127, 256, 257, 3, 1000, 2, 5000, 131, 1, 1, 384, 640, 7, 2049]
    T, d, E = sum(sizes), 136, 3
    tokens, rot, _ = _rand_inputs(36, T, d, 1, E, 2, 16, dtype)
    ids = np.empty(T, np.uint64)
    ids[np.random.default_rng(37).permutation(T)] = np.repeat(np.arange(len(sizes)), sizes).astype(np.uint64)
    expert = np.tile(np.array([[2, 0]], np.int32), (T, 1))
    run = H.run_and_check(tokens, rot, expert, E, dtype, _scale_fn, bucket_override=ids)
    H.check_backward(run, T, d, 2, dtype, seed=38)


# ------------------------------------------------------------------ hash fused with the gate projection
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T,L,r,E", [(32768 + 9, 3, 32, 32),    # GPT shape: 96 + 32 rows, one pass, 128-token workgroups
                                     (16384 + 3, 2, 32, 16),    # RoBERTa shape: 64-token workgroups
                                     (9000, 1, 8, 5),           # E not a multiple of 4, a single tile
                                     (70000, 4, 64, 64),        # T5 shape: hash as usual, then the gate rows alone
                                     (100, 2, 16, 128),         # tiny T, widest gate
                                     (5000, 12, 8, 30),         # 96 + 30 rows
                                     (20000, 6, 16, 1),         # a single gate row: a logit can cancel to almost nothing
                                     (24576, 10, 32, 2),        # 320 hash rows (two passes), two gate rows
                                     (40000, 8, 32, 64),        # 256 + 64 rows in one pass: a gate tile per wave half, r = 32
                                     (33000, 2, 128, 40),       # ... r = 128, the second gate tile partly filled
                                     (50001, 5, 40, 7),         # ... hashes that straddle tiles and halves (generic arg-max), odd E
                                     (65536, 1, 256, 64),       # ... one hash over both halves
                                     (32768, 3, 64, 33),        # ... three of four hashes, one row in the second gate tile
                                     (40000 + 5, 2, 32, 16)])   # more than 256 workgroups: the short-ring gate instance
def test_hash_gate(H, dtype, T, L, r, E):
    import oracle
    d = 256 if dtype == "bf16" else 128
    rng = np.random.default_rng(51)
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
    H.lsh.lshmoe_hash(xt, rt, plain)                       # the fused call hashes exactly like the plain one
    torch.cuda.synchronize()
    assert np.array_equal(plain.cpu().numpy().view(np.uint64), bucket)
    ref = oracle.gate_logits_ref(tokens, gate, dtype)
    got = lt[:T].cpu().numpy().astype(np.float64)
    # binary32 accumulation of d exact-or-binary32 products, 16 per MFMA: |error| <= (d/16 + 8) 2^-24 sum_i |x_i w_i|.
    # (Scaling by the row's largest logit, as for the other outputs, is not meaningful here: with one or two gate
    # rows every logit of a token can cancel to almost nothing.)
    xa, wa = np.abs(oracle.widen(tokens, dtype)), np.abs(oracle.widen(gate, dtype))
    bound = (d / 16 + 8) * 2.0 ** -24 * (xa @ wa.T)
    worst = np.max(np.abs(got - ref) - bound)
    assert worst <= 0.0, "gate logits off by %.3g beyond the accumulation bound" % worst
    print("gate logits T=%d L=%d r=%d E=%d %s: largest |error| / bound = %.3f" %
          (T, L, r, E, dtype, float(np.max(np.abs(got - ref) / np.maximum(bound, 1e-300)))), flush=True)
    if E >= 4:
        err = oracle.row_rel_err(got, ref)
        assert err.max() <= 1e-5, "gate logits: row %d off by %.3g" % (int(err.argmax()), err.max())
        H.WORST[("gate logits", "f32")] = max(H.WORST.get(("gate logits", "f32"), 0.0), float(err.max()))


# ------------------------------------------------------------------ spherical hash (Section 4.5, "SP")
def _check_sphere(H, tokens, pivots, radius_sq, dtype, exact=False):
    """lshmoe_hash_sphere against the oracle: every bit equal, except that a bit whose squared distance is within
    1e-4 (relative) of the squared radius may differ (counted).  exact: no bit may differ."""
    import oracle
    T, B = tokens.shape[0], pivots.shape[0]
    xt, pt = H.to_device(tokens, dtype), H.to_device(pivots, dtype)
    rt = torch.from_numpy(np.ascontiguousarray(radius_sq, dtype=np.float32)).cuda()
    bt = torch.full((T + 4,), -1, dtype=torch.int64, device="cuda")
    H.lsh.lshmoe_hash_sphere(xt, pt, rt, bt[:T])
    torch.cuda.synchronize()
    assert np.all(bt[T:].cpu().numpy() == -1), "nothing is written past T"
    got = bt[:T].cpu().numpy().view(np.uint64)
    ref, bit, margin = oracle.sphere_hash_ref(tokens, pivots, radius_sq.astype(np.float32).astype(np.float64), dtype)
    assert np.all(got >> np.uint64(B) == 0), "bucket id out of range"
    gbit = ((got[:, None] >> (np.uint64(B - 1) - np.arange(B, dtype=np.uint64))[None, :]) & np.uint64(1)).astype(np.uint8)
    diff = gbit != bit
    bad = diff & (margin >= 1e-4)
    assert not bad.any(), "spherical hash bit differs away from the surface at (token, sphere) %s" % (np.argwhere(bad)[:8].tolist(),)
    if exact:
        assert not diff.any()
    return got, int(diff.sum())


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("T,d,B", [(1, 64, 1), (300, 72, 5), (4097, 256, 32), (20000, 1024, 33), (65536 + 7, 512, 63),
                                   (1000, 8, 2), (129, 2048, 17)])
def test_sphere_hash(H, dtype, T, d, B):
    rng = np.random.default_rng(900 + T + B)
    tokens = synth.f32_to_storage(rng.standard_normal((T, d)).astype(np.float32), dtype)
    pivots = synth.f32_to_storage(rng.standard_normal((B, d)).astype(np.float32), dtype)
    radius_sq = (2.0 * d + rng.standard_normal(B) * np.sqrt(8.0 * d)).astype(np.float32)    # around the mean squared distance
    got, flips = _check_sphere(H, tokens, pivots, radius_sq, dtype)
    gbits = np.unpackbits(got.view(np.uint8).reshape(T, 8), axis=1, bitorder="little")[:, :B]
    if T >= 300:
        assert 0.02 < gbits.mean() < 0.98, "balanced radii: both sides of the spheres are populated"
    print("sphere hash T=%d d=%d B=%d %s: %d borderline bits differ" % (T, d, B, dtype, flips), flush=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sphere_hash_exact_on_integers(H, dtype):
    # small integers: every product, sum and squared distance is exact in binary32, and many tokens sit exactly on a
    # sphere (which counts as inside): no bit may differ
    rng = np.random.default_rng(77)
    T, d, B = 5000, 32, 40
    tokens = synth.f32_to_storage(rng.integers(-4, 5, size=(T, d)).astype(np.float32), dtype)
    pivots = synth.f32_to_storage(rng.integers(-3, 4, size=(B, d)).astype(np.float32), dtype)
    radius_sq = rng.integers(250, 420, size=B).astype(np.float32)
    import oracle
    _, _, margin = oracle.sphere_hash_ref(tokens, pivots, radius_sq.astype(np.float64), dtype)
    assert (margin == 0.0).sum() > 100
    _check_sphere(H, tokens, pivots, radius_sq, dtype, exact=True)
    # degenerate radii: nothing inside, everything inside
    got, _ = _check_sphere(H, tokens, pivots, np.full(B, -1.0, np.float32), dtype, exact=True)
    assert not got.any()
    got, _ = _check_sphere(H, tokens, pivots, np.full(B, 1e9, np.float32), dtype, exact=True)
    assert np.all(got == np.uint64((1 << B) - 1))


def test_sphere_hash_feeds_the_rest_of_the_path(H):
    # bucket ids of the spherical hash go through compress and decompress like cross-polytope ones
    cfg = synth.config("gpt", T=6000, centers=40)
    w = synth.generate(cfg)
    B = 11
    rng = np.random.default_rng(5)
    pivots = synth.f32_to_storage(rng.standard_normal((B, cfg.d)).astype(np.float32), cfg.dtype)
    radius_sq = np.full(B, cfg.d * (2.0 + cfg.sigma ** 2), np.float32)
    got, _ = _check_sphere(H, w.tokens, pivots, radius_sq, cfg.dtype)
    L, r = (B + 1) // 2, 2                                  # (2r)^L = 4^6 >= 2^11 bounds the ids
    dummy_rot = np.zeros((L, r, cfg.d), w.rot.dtype)
    run = H.run_and_check(w.tokens, dummy_rot, w.expert, cfg.E, cfg.dtype, _standin(cfg, w.seed), bucket_override=got,
                          skip_hash=True)
    assert run.S < cfg.N                                    # the spheres do put tokens of a mixture centre together


def test_path_replays_from_a_graph(H):
    # the calls only enqueue kernels on the caller's stream (no allocation, no host synchronisation, no memset
    # nodes), so a step can be captured once and replayed: three replays on fresh inputs, with eager work and
    # synchronisations in between, each compared bit for bit with the eager result on the same inputs
    lsh = H.lsh
    cfg = synth.config("gpt", T=6000, centers=400)
    T, d, k, E, L, r, N = cfg.T, cfg.d, cfg.k, cfg.E, cfg.L, cfg.r, cfg.N
    ws = [synth.generate(cfg, seed=100 + i) for i in range(3)]
    x = torch.empty((T, d), dtype=torch.bfloat16, device="cuda")
    rot = H.to_device(ws[0].rot, cfg.dtype)
    expert = torch.empty((T, k), dtype=torch.int32, device="cuda")
    ec = torch.randn((N, d), device="cuda").to(torch.bfloat16)
    bucket = torch.empty(T, dtype=torch.int64, device="cuda")
    out = lsh.CompressOutputs.allocate(T, d, k, E, L, r, torch.bfloat16)
    y = torch.empty((T, k, d), dtype=torch.bfloat16, device="cuda")

    def step():
        lsh.lshmoe_hash(x, rot, bucket)
        lsh.lshmoe_compress(x, expert, bucket, E, L, r, out)
        lsh.lshmoe_decompress(x, out.centroids, ec, out.seg_of, out.seg_offsets, k, y, perm=out.perm,
                              num_segments=out.num_segments)

    def load(w):
        x.copy_(H.to_device(w.tokens, cfg.dtype))
        expert.copy_(torch.from_numpy(w.expert).cuda())

    load(ws[0])
    step()                                   # warm-up outside the capture (sets kernel attributes)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for w in ws:
        load(w)
        step()
        torch.cuda.synchronize()
        want = [t.clone() for t in (bucket, out.perm, out.seg_of, out.seg_offsets, out.num_segments, out.expert_offsets, y)]
        S = int(out.num_segments.item())
        want_c = out.centroids[:S].clone()
        for t in (bucket, out.perm, out.seg_of, out.seg_offsets, out.num_segments, out.expert_offsets):
            t.fill_(-3)
        y.zero_()
        out.centroids.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (bucket, out.perm, out.seg_of, out.seg_offsets, out.num_segments, out.expert_offsets, y)
        assert torch.equal(got[4], want[4])
        for g, wnt, name in zip(got, want, ("bucket", "perm", "seg_of", "seg_offsets", "S", "expert_offsets", "y")):
            if name == "seg_offsets":
                assert torch.equal(g[:S + 1], wnt[:S + 1]), name
            else:
                assert torch.equal(g, wnt), name
        assert torch.equal(out.centroids[:S], want_c)


def test_deterministic_across_runs(H):
    cfg = synth.config("gpt", T=4000, centers=300)
    w = synth.generate(cfg)
    a = H.run_and_check(w.tokens, w.rot, w.expert, cfg.E, cfg.dtype, _standin(cfg, w.seed))
    b = H.run_and_check(w.tokens, w.rot, w.expert, cfg.E, cfg.dtype, _standin(cfg, w.seed))
    assert np.array_equal(a.bucket, b.bucket) and np.array_equal(a.centroids, b.centroids) and np.array_equal(a.y, b.y)


def test_outputs_do_not_overrun(H):
    # canaries after every compress output stay untouched
    T, d, k, E, L, r = 777, 32, 2, 5, 2, 16
    tokens, rot, expert = _rand_inputs(10, T, d, k, E, L, r, "bf16", centers=50)
    lsh = H.lsh
    N = T * k
    xt, rt = H.to_device(tokens, "bf16"), H.to_device(rot, "bf16")
    et = torch.from_numpy(expert).cuda()
    bt = torch.empty(T + 8, dtype=torch.int64, device="cuda").fill_(-1)
    lsh.lshmoe_hash(xt, rt, bt[:T])
    out = lsh.CompressOutputs.allocate(T, d, k, E, L, r, xt.dtype)
    pad = 16
    big = {n: torch.full((getattr(out, n).numel() + pad,), -3, dtype=torch.int32, device="cuda")
           for n in ("seg_offsets", "seg_expert", "expert_offsets", "perm", "seg_of", "num_segments")}
    cent = torch.full((N + 2, d), 7.0, dtype=xt.dtype, device="cuda")
    sub = lsh.CompressOutputs(cent[:N], *(big[n][:getattr(out, n).numel()] for n in
                                           ("seg_offsets", "seg_expert", "expert_offsets", "perm", "seg_of",
                                            "num_segments")), out.workspace)
    lsh.lshmoe_compress(xt, et, bt[:T], E, L, r, sub)
    torch.cuda.synchronize()
    assert torch.all(bt[T:] == -1)
    for n, t in big.items():
        assert torch.all(t[-pad:] == -3), n
    assert torch.all(cent[N:] == 7.0)
    S = int(sub.num_segments.item())
    assert torch.all(cent[S:N] == 7.0)       # rows past S are left alone


def test_maximum_size_indexing(H):
    # 2^27 + 6 assignments (T = 2^26 + 3 tokens, k = 2) of 272-byte rows: the centroid step then starts more than
    # 2^26 waves and the restore step more than 2^27 rows, where a 32-bit thread index would wrap.  The oracle
    # cannot run at this size: clusters are built so that every output has a closed form (tokens 2m and 2m + 1
    # share bucket m and both go to experts 2(m mod 2) and 2(m mod 2) + 1), which torch evaluates on the device
    # with the path's own arithmetic (binary32 sum of two rows, halved, rounded once; e + (x - c) rounded once),
    # and sampled tokens, clusters and rows are compared with the oracle.
    import oracle
    dtype, tdt = "bf16", torch.bfloat16
    T, d, k, E, L, r = (1 << 26) + 3, 136, 2, 4, 6, 16
    N, M = T * k, (T + 1) // 2
    dev = "cuda"
    print("case maximum size T", T, "N", N, flush=True)
    g = torch.Generator(device=dev)
    g.manual_seed(77)
    xt = torch.empty((T, d), dtype=tdt, device=dev)
    step = 1 << 22
    for lo in range(0, T, step):
        hi = min(T, lo + step)
        xt[lo:hi] = torch.randn((hi - lo, d), generator=g, device=dev).to(tdt)
    rot_np = synth.f32_to_storage(np.random.default_rng(5).standard_normal((L, r, d)).astype(np.float32), dtype)
    rt = H.to_device(rot_np, dtype)
    tt = torch.arange(T, device=dev, dtype=torch.int64)
    m_of_t = tt // 2
    et = torch.stack([(m_of_t % 2) * 2, (m_of_t % 2) * 2 + 1], dim=1).to(torch.int32).contiguous()

    # hash at full size, checked on a sample
    bt = torch.empty(T, dtype=torch.int64, device=dev)
    H.lsh.lshmoe_hash(xt, rt, bt)
    torch.cuda.synchronize()
    rng = np.random.default_rng(9)
    samp = np.unique(np.concatenate([rng.integers(0, T, 4000), [0, 1, T - 2, T - 1, (1 << 26) - 1, 1 << 26]]))
    st = torch.from_numpy(samp).to(dev)
    H.check_hash(bt[st].cpu().numpy().view(np.uint64), H.to_storage(xt[st], dtype), rot_np, dtype)
    print("  hash sample ok", flush=True)

    out = H.lsh.CompressOutputs.allocate(T, d, k, E, L, r, tdt)
    H.lsh.lshmoe_compress(xt, et, m_of_t, E, L, r, out)
    torch.cuda.synchronize()
    S = int(out.num_segments.item())
    assert S == 2 * M
    # expected order: experts 0, 1 hold the even m (slot j = 0, 1), experts 2, 3 the odd m
    perm_parts, size_parts = [], []
    for e in range(E):
        j, par = e % 2, e // 2
        ms = torch.arange(par, M, 2, device=dev, dtype=torch.int64)
        a0, a1 = (2 * ms) * k + j, (2 * ms + 1) * k + j
        both = torch.stack([a0, a1], dim=1).reshape(-1)
        keep = torch.stack([2 * ms < T, 2 * ms + 1 < T], dim=1).reshape(-1)
        perm_parts.append(both[keep])
        size_parts.append((2 * ms + 1 < T).to(torch.int64) + 1)
    perm_ref = torch.cat(perm_parts)
    sizes = torch.cat(size_parts)
    offs_ref = torch.zeros(S + 1, dtype=torch.int64, device=dev)
    offs_ref[1:] = torch.cumsum(sizes, 0)
    assert perm_ref.numel() == N and int(offs_ref[-1]) == N
    assert torch.equal(out.perm.to(torch.int64), perm_ref)
    assert torch.equal(out.seg_offsets[:S + 1].to(torch.int64), offs_ref)
    seg_ref = torch.empty(N, dtype=torch.int64, device=dev)
    seg_ref[perm_ref] = torch.repeat_interleave(torch.arange(S, device=dev), sizes)
    assert torch.equal(out.seg_of.to(torch.int64), seg_ref)
    eoff = [0]
    for part in size_parts:
        eoff.append(eoff[-1] + part.numel())
    assert out.expert_offsets.cpu().tolist() == eoff
    assert torch.equal(out.seg_expert[:S].to(torch.int64),
                       torch.repeat_interleave(torch.arange(E, device=dev), torch.tensor([p.numel() for p in size_parts], device=dev)))
    del seg_ref, perm_parts, size_parts
    print("  grouping ok, S", S, flush=True)

    # centroids: (x0 + x1) / 2 in binary32, rounded once; one-member clusters copy their token
    first = perm_ref[offs_ref[:-1]] // k
    second = perm_ref[torch.clamp(offs_ref[:-1] + 1, max=N - 1)] // k
    two = sizes == 2
    cstep = 1 << 22
    for lo in range(0, S, cstep):
        hi = min(S, lo + cstep)
        x0, x1 = xt[first[lo:hi]].float(), xt[second[lo:hi]].float()
        ref = torch.where(two[lo:hi, None], (x0 + x1) / 2.0, x0).to(tdt)
        assert torch.equal(out.centroids[lo:hi].view(torch.int16), ref.view(torch.int16)), "centroid rows %d.." % lo
    del first, second
    print("  centroids ok", flush=True)
    cs = np.unique(np.concatenate([rng.integers(0, S, 1500), [0, 1, S - 2, S - 1, S // 2]]))
    for s in cs[:: max(1, len(cs) // 300)]:   # the oracle on a few hundred clusters, one at a time
        lo, hi = int(offs_ref[s]), int(offs_ref[s + 1])
        rows = H.to_storage(xt[perm_ref[lo:hi] // k], dtype)
        c_ref = oracle.centroid_ref(rows, np.arange(hi - lo, dtype=np.int32), np.array([0, hi - lo], np.int32), 1, dtype)
        H.assert_rows_close(H.to_storage(out.centroids[s:s + 1], dtype), c_ref, dtype, "centroid %d" % s)

    ect = torch.empty((S, d), dtype=tdt, device=dev)
    for lo in range(0, S, cstep):
        hi = min(S, lo + cstep)
        ect[lo:hi] = _scale_fn(out.centroids[lo:hi])
    y1 = torch.empty((T, k, d), dtype=tdt, device=dev)
    y2 = torch.empty((T, k, d), dtype=tdt, device=dev)
    H.lsh.lshmoe_decompress(xt, out.centroids, ect, out.seg_of, out.seg_offsets, k, y1)
    H.lsh.lshmoe_decompress(xt, out.centroids, ect, out.seg_of, out.seg_offsets, k, y2, perm=out.perm,
                            num_segments=out.num_segments)
    torch.cuda.synchronize()
    y1f, y2f = y1.view(N, d), y2.view(N, d)
    astep = 1 << 22
    for lo in range(0, N, astep):
        hi = min(N, lo + astep)
        s_a = out.seg_of[lo:hi].to(torch.int64)
        t_a = torch.arange(lo, hi, device=dev) // k
        ref = (ect[s_a].float() + (xt[t_a].float() - out.centroids[s_a].float())).to(tdt)
        assert torch.equal(y1f[lo:hi].view(torch.int16), ref.view(torch.int16)), "restored rows %d.." % lo
        assert torch.equal(y2f[lo:hi].view(torch.int16), ref.view(torch.int16)), "restored rows (cluster order) %d.." % lo
    print("  restore ok", flush=True)
    asamp = np.unique(np.concatenate([rng.integers(0, N, 3000), [0, 1, N - 2, N - 1, (1 << 27) - 1, 1 << 27]]))
    at = torch.from_numpy(asamp).to(dev)
    s_a = out.seg_of[at].to(torch.int64)
    y_ref = oracle.restore_ref(H.to_storage(xt[at // k], dtype), H.to_storage(out.centroids[s_a], dtype),
                               H.to_storage(ect[s_a], dtype), np.arange(len(asamp), dtype=np.int32), 1, dtype)
    H.assert_rows_close(H.to_storage(y1f[at], dtype), y_ref, dtype, "restore sample")
