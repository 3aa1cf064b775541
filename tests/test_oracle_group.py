"""Pins for the oracle's grouping step (Alg. 1: dispatch by expert, then split
each expert's tokens into clusters by bucket)."""
import numpy as np
import pytest

from oracle import group_ref


def _dict_grouping(expert, bucket):
    """Pure-Python grouping: dict keyed by (expert, bucket), insertion in
    assignment order; clusters listed by sorted key."""
    T, k = expert.shape
    groups = {}
    for t in range(T):
        for j in range(k):
            groups.setdefault((int(expert[t, j]), int(bucket[t])), []).append(t * k + j)
    keys = sorted(groups)
    return keys, [groups[key] for key in keys]


def _check_structure(g, expert, bucket, E):
    T, k = expert.shape
    N = T * k
    perm, off, sexp, eoff, seg_of, S = (g[n] for n in
                                        ("perm", "seg_offsets", "seg_expert", "expert_offsets", "seg_of", "S"))
    assert perm.dtype == np.int32 and off.dtype == np.int32 and seg_of.dtype == np.int32
    assert sorted(perm.tolist()) == list(range(N))
    assert off[0] == 0 and off[S] == N and np.all(np.diff(off) > 0) and off.size == S + 1
    ea = expert.reshape(-1)[perm]
    ba = np.repeat(bucket, k)[perm]
    keys = list(zip(ea.tolist(), ba.tolist()))
    assert keys == sorted(keys)
    for s in range(S):
        seg_keys = set(keys[off[s]:off[s + 1]])
        assert len(seg_keys) == 1
        assert sexp[s] == next(iter(seg_keys))[0]
        if s:
            assert keys[off[s] - 1] != keys[off[s]]
        members = perm[off[s]:off[s + 1]]
        assert np.all(np.diff(members) > 0)               # ascending assignment index
        assert np.all(seg_of[members] == s)
    assert eoff.size == E + 1 and eoff[0] == 0 and eoff[E] == S and np.all(np.diff(eoff) >= 0)
    for e in range(E):
        assert np.all(sexp[eoff[e]:eoff[e + 1]] == e)


@pytest.mark.parametrize("seed,T,k,E,nb", [(0, 50, 1, 4, 6), (1, 40, 2, 5, 3), (2, 97, 3, 7, 1000), (3, 1, 1, 1, 1),
                                           (4, 64, 2, 9, 2)])
def test_group_matches_dict_brute_force(seed, T, k, E, nb):
    rng = np.random.default_rng(seed)
    expert = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    bucket = rng.integers(0, nb, size=T).astype(np.uint64)
    g = group_ref(expert, bucket, E)
    keys, members = _dict_grouping(expert, bucket)
    assert g["S"] == len(keys)
    assert g["seg_expert"].tolist() == [key[0] for key in keys]
    assert g["seg_offsets"].tolist() == np.concatenate([[0], np.cumsum([len(m) for m in members])]).tolist()
    assert g["perm"].tolist() == [a for m in members for a in m]
    _check_structure(g, expert, bucket, E)


def test_group_matches_numpy_unique():
    rng = np.random.default_rng(9)
    T, k, E = 3000, 2, 16
    expert = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    bucket = rng.integers(0, 40, size=T).astype(np.uint64) * np.uint64(2 ** 40 + 12345)   # wide 64-bit ids
    g = group_ref(expert, bucket, E)
    # independent route: one flat integer key (python ints, no overflow) + numpy.unique
    flat = np.array([int(e) * (2 ** 64) + int(b) for e, b in
                     zip(expert.reshape(-1), np.repeat(bucket, k))], dtype=object)
    uniq, inverse, counts = np.unique(flat, return_inverse=True, return_counts=True)
    assert g["S"] == uniq.size
    assert np.array_equal(np.diff(g["seg_offsets"]), counts)
    assert np.array_equal(g["seg_of"], inverse)
    assert np.array_equal(g["perm"], np.argsort(inverse, kind="stable"))
    _check_structure(g, expert, bucket, E)


def test_bucket_ids_above_2_pow_53_are_kept_apart():
    # ids that differ only in low bits beyond double precision must not merge
    expert = np.zeros((4, 1), np.int32)
    bucket = np.array([2 ** 62 + 1, 2 ** 62, 2 ** 62 + 1, 2 ** 62 + 2], np.uint64)
    g = group_ref(expert, bucket, 1)
    assert g["S"] == 3
    assert g["perm"].tolist() == [1, 0, 2, 3]
    assert g["seg_offsets"].tolist() == [0, 1, 3, 4]


def test_special_cases():
    # one expert, one bucket -> a single cluster in assignment order
    g = group_ref(np.zeros((7, 1), np.int32), np.full(7, 5, np.uint64), 3)
    assert g["S"] == 1 and g["perm"].tolist() == list(range(7))
    assert g["expert_offsets"].tolist() == [0, 1, 1, 1]
    # all keys distinct -> S == N and perm is the sort order
    expert = np.array([[2], [0], [1], [0]], np.int32)
    bucket = np.array([3, 9, 1, 4], np.uint64)
    g = group_ref(expert, bucket, 4)
    assert g["S"] == 4 and g["perm"].tolist() == [3, 1, 2, 0]
    assert g["seg_expert"].tolist() == [0, 0, 1, 2]
    assert g["expert_offsets"].tolist() == [0, 2, 3, 4, 4]     # expert 3 receives nothing
    # clusters never span experts even when the bucket id is the same (clusters are formed inside X_i)
    expert = np.array([[0, 1], [1, 0], [0, 1]], np.int32)
    bucket = np.array([7, 7, 7], np.uint64)
    g = group_ref(expert, bucket, 2)
    assert g["S"] == 2
    assert g["perm"].tolist() == [0, 3, 4, 1, 2, 5]
    assert g["seg_of"].tolist() == [0, 1, 1, 0, 0, 1]
    # empty leading expert
    g = group_ref(np.array([[2], [2]], np.int32), np.array([1, 0], np.uint64), 3)
    assert g["expert_offsets"].tolist() == [0, 0, 0, 2]


def test_more_hash_functions_refine_the_clusters():
    """Section 4.3 (ablation on the number of hash functions): with the hash functions of a shorter list being a
    prefix of a longer one, a further hash function can split a cluster but never merge two, so the cluster count
    (and with it the compression rate S/N) does not fall; the bucket id of the shorter list is the longer one's
    id with its last mixed-radix digits dropped (hash 0 is the most significant digit)."""
    from oracle import hash_ref
    from workloads import synth
    r = 16
    cfg = synth.config("gpt", T=3000, L=10, r=r, gate="content", sigma=0.05, centers=64)
    w = synth.generate(cfg)
    N = cfg.T * cfg.k
    counts, prev_seg, prev_b, prev_L = [], None, None, None
    for L in (2, 4, 6, 8, 10):
        b = hash_ref(w.tokens, w.rot[:L], cfg.dtype)[0]
        g = group_ref(w.expert, b, cfg.E)
        counts.append(g["S"])
        if prev_seg is not None:
            assert np.array_equal(b // np.uint64((2 * r) ** (L - prev_L)), prev_b)
            pairs = np.unique(np.stack([g["seg_of"], prev_seg], axis=1), axis=0)
            assert len(pairs) == g["S"]               # every cluster lies inside exactly one cluster of the shorter list
            assert len(np.unique(pairs[:, 1])) == len(np.unique(prev_seg))
        prev_seg, prev_b, prev_L = g["seg_of"], b, L
    assert counts == sorted(counts) and counts[0] < counts[-1] <= N
