"""Placement of buffers by memory class (paper_2502_12996_amd/placement.py).

CPU: the two pure steps, on rates measured on an MI355X (two 2 GiB read streams, GB/s) and on made-up
label lists.  GPU: the arena's mechanics on a small scale (chunks mapped, classified, placed; kernels
give the same bits on placed memory as on ordinary memory; memory goes back), and one classification
at real scale.
"""
import numpy as np
import pytest

from paper_2502_12996_amd import placement as P

# chunk 0 against chunks 1..127 of a fresh process, in mapping order (hundreds of GB/s dropped: GB/s / 100)
MEASURED = """72 73 72 73 73 72 73 74 73 74 73 73 73 73 71 73 73 73 72 73 72 73 74 73 74 74 74 74 73 73 73 72 72 72 72 72 73 73
74 73 73 74 73 73 72 74 70 70 70 69 71 69 69 69 70 70 69 69 69 69 70 70 69 70 70 69 70 70 70 69 70 69 70 69 69 70 69 69 70 70 69 70
70 69 69 69 69 69 69 70 70 70 70 70 70 69 69 69 70 70 70 70 69 70 70 69 69 69 70 69 69 70 70 70 69 69 70 70 69 69 70 70 69 70 69 69 70"""
# another run, chunk 0 against the other 127, sorted: 80 chunks of other classes, 3 chunks that straddle two
# classes (7067, 7135 and, arguably, 7029), 44 of chunk 0's class
SORTED = """6879 6890 6893 6898 6898 6900 6902 6903 6907 6910 6911 6913 6913 6917 6918 6921 6922 6923 6923 6925 6929 6930
6931 6932 6932 6934 6938 6939 6939 6939 6939 6940 6940 6944 6945 6945 6948 6948 6949 6951 6952 6953 6955 6955 6958 6959 6961
6964 6964 6966 6967 6969 6969 6969 6970 6971 6971 6971 6972 6973 6973 6973 6974 6974 6974 6976 6978 6985 6985 6987 6990 6990
6991 6997 7000 7000 7002 7013 7024 7029 7067 7135 7184 7185 7195 7211 7233 7234 7241 7242 7244 7246 7247 7266 7269 7269 7270
7271 7273 7275 7278 7281 7282 7285 7295 7295 7297 7298 7303 7305 7318 7320 7323 7328 7334 7342 7347 7359 7367 7369 7372 7376
7380 7381 7388 7392 7422"""


def test_split_finds_the_class_of_the_reference_in_measured_rates():
    coarse = [float(x) * 100.0 for x in MEASURED.split()]
    rates = {k + 1: v for k, v in enumerate(coarse)}
    thr, same, other = P.split_by_rate(rates)
    assert thr is not None and 7000.0 < thr < 7200.0
    # chunks 1..46 share chunk 0's class (one 7100 among them: a chunk that straddles two classes)
    assert set(range(1, 47)) - set(same) <= {15} and all(k < 47 or k == 51 for k in same) and len(same) >= 45
    exact = [float(x) for x in SORTED.split()]
    assert len(exact) == 127
    thr, same, other = P.split_by_rate(dict(enumerate(exact)))
    assert 7067.0 < thr < 7184.0
    assert all(exact[k] >= 7135.0 for k in same) and all(exact[k] <= 7135.0 for k in other)
    assert len(same) in (45, 46) and len(same) + len(other) == 127


def test_split_reports_one_group_when_there_is_no_contrast():
    rng = np.random.default_rng(3)
    rates = {k: 7250.0 * (1.0 + 0.006 * rng.standard_normal()) for k in range(40)}
    thr, same, other = P.split_by_rate(rates)
    assert thr is None and sorted(same) == list(range(40)) and other == []
    assert P.split_by_rate({}) == (None, [], [])
    assert P.split_by_rate({3: 7000.0}) == (None, [3], [])


def test_groups_come_from_one_class_where_one_suffices():
    labels = [0] * 10 + [1] * 6 + [2] * 8 + [-1] * 2
    plan = P.plan_groups(labels, [7, 6])
    assert all(labels[c] == 2 for c in plan[0])              # best fit: the 8 of class 2, not the 10 of class 0
    assert all(labels[c] == 1 for c in plan[1])
    assert len(set(plan[0]) | set(plan[1])) == 13
    # a group larger than every class: the largest class first, then the next, mixed chunks last
    plan = P.plan_groups(labels, [19])
    got = [labels[c] for c in plan[0]]
    assert got.count(0) == 10 and got.count(2) == 8 and got.count(1) == 1 and -1 not in got
    plan = P.plan_groups(labels, [25])
    assert sorted(labels[c] for c in plan[0]).count(-1) == 1
    with pytest.raises(P.PlacementError):
        P.plan_groups(labels, [20, 7])
    assert P.plan_groups([], []) == []


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_labelling_recovers_the_classes_of_a_simulated_memory(seed):
    """139 chunks in scrambled order over three classes, some straddling two; the rate of a pair is what was
    measured: about 6.92 TB/s across classes, 7.25 within one (spread 2.5 %), noise on top."""
    rng = np.random.default_rng(seed)
    n = 139
    frac = np.zeros((n, 3))
    truth = rng.permutation(np.repeat([0, 1, 2], [46, 47, 46]))
    frac[np.arange(n), truth] = 1.0
    straddlers = rng.choice(n, size=7, replace=False)
    for k in straddlers:                                    # part of the chunk lies in the next class
        f = rng.uniform(0.25, 0.75)
        frac[k] = 0.0
        frac[k, truth[k]], frac[k, (truth[k] + 1) % 3] = f, 1.0 - f
    within = rng.uniform(-0.09, 0.09, size=(n, n))          # rates inside a class spread (distance, position)
    within = (within + within.T) / 2

    def measure(ref, rest):
        return {k: 1000.0 * (6.92 + (0.33 + within[ref, k]) * float(frac[ref] @ frac[k]) + 0.012 * rng.standard_normal())
                for k in rest}
    labels, history = P.label_chunks(n, measure)
    pure = [k for k in range(n) if k not in set(straddlers)]
    classes = sorted(set(labels[k] for k in pure) - {-1})
    assert len(classes) == 3
    # one label per true class on the pure chunks, nearly all of them labelled
    for c in range(3):
        got = [labels[k] for k in pure if truth[k] == c]
        top = max(set(got), key=got.count)
        assert top >= 0 and got.count(top) >= len(got) - 2, (c, got)
    assert len({max(set(g := [labels[k] for k in pure if truth[k] == c]), key=g.count) for c in range(3)}) == 3
    assert max(labels.count(c) for c in classes) <= P.CLASS_CHUNKS_MAX
    assert len(history) <= 12


def test_labelling_of_a_memory_without_classes():
    rng = np.random.default_rng(5)
    labels, _ = P.label_chunks(30, lambda ref, rest: {k: 7200.0 + 20.0 * rng.standard_normal() for k in rest})
    assert labels == [0] * 30
    assert P.label_chunks(1, lambda ref, rest: {}) == ([0], [{}])
    assert P.label_chunks(0, lambda ref, rest: {}) == ([], [])


@pytest.mark.gpu
def test_arena_places_buffers_that_behave_like_any_other_memory():
    import torch

    import paper_2502_12996_amd as d
    from paper_2502_12996_amd import workloads as W
    dev = "cuda:0"
    torch.cuda.empty_cache()
    free0 = torch.cuda.mem_get_info()[0]
    arena = P.Arena(chunk_bytes=256 << 20, max_chunks=10)
    assert len(arena.handles) == 10 and torch.cuda.mem_get_info()[0] <= free0 - 9 * (256 << 20)
    labels = arena.classify(reps=2)
    assert len(labels) == 10 and all(-1 <= lab < 4 for lab in labels)
    M, n = 3, 20_000_003                                     # 240 MB a buffer: groups span several chunks
    nbytes = M * n * 4
    bufs = arena.place([[("theta", nbytes), ("m1", nbytes), ("m2", nbytes), ("grad", nbytes)],
                        [("spare", 100 << 20)]])
    arena.release_rest()
    assert len(arena.placed) == 5 and sum(h is not None for h in arena.handles) == 5
    assert torch.cuda.mem_get_info()[0] >= free0 - 6 * (256 << 20)
    wl = W.Workload("case", M=M, n=n, theta_dtype="f32")
    ref = W.adamw_state(wl, n, seed=7, device=dev)
    mine = {k: bufs[k].view(torch.float32).view(M, n) for k in ref}
    for k in ref:
        assert mine[k].data_ptr() % 4096 == 0
        mine[k].copy_(ref[k])
    kw = dict(lr=wl.lr, beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, weight_decay=wl.weight_decay, step=5)
    d.inner_adamw(ref["theta"], ref["m1"], ref["m2"], ref["grad"], **kw)
    d.inner_adamw(mine["theta"], mine["m1"], mine["m2"], mine["grad"], **kw)
    torch.cuda.synchronize()
    for k in ref:
        assert torch.equal(ref[k], mine[k]), k
    bufs["spare"].fill_(7)
    assert int(bufs["spare"].sum(dtype=torch.int64)) == 7 * (100 << 20)
    del mine, bufs
    held = torch.cuda.mem_get_info()[0]
    arena.close()
    arena.close()                                            # a second close is a no-op
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= held + 5 * (256 << 20) - (64 << 20)   # the five placed chunks came back


@pytest.mark.gpu
def test_classification_at_real_scale():
    import torch
    torch.cuda.empty_cache()
    arena = P.Arena(max_chunks=72)                           # up to 144 GiB: more than one class holds
    try:
        if len(arena.handles) < 56:
            pytest.skip("not enough free device memory to span two classes")
        labels = arena.classify()
        assert len(labels) == len(arena.handles)
        classes = sorted(set(labels) - {-1})
        if len(classes) < 2:
            pytest.skip("this device shows no memory classes in the two-stream read rate")
        counts = {c: labels.count(c) for c in classes}
        assert max(counts.values()) <= P.CLASS_CHUNKS_MAX, counts
        # a reference that told two groups apart: its own class reads faster with it than the others do
        splits = [(r, P.split_by_rate(r)) for r in arena.rates]
        splits = [(r, s) for r, s in splits if s[0] is not None and len(s[1]) >= 5 and len(s[2]) >= 5]
        assert splits, "two classes were labelled, so some reference must have seen both"
        ref_rates, (thr, same, other) = splits[0]
        fast = np.mean([ref_rates[k] for k in same])
        slow = np.mean([ref_rates[k] for k in other])
        assert fast > slow * (1.0 + P.SAME_CLASS_MIN_GAIN), (fast, slow)
    finally:
        arena.close()
