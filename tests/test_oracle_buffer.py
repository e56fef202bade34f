"""Pins for the circular-buffer oracle (Section 3.2): brute force on tiny rings."""
import copy
import itertools

import numpy as np
import pytest

from oracle.buffer import BufferFull, BufferOracle, NotEnoughLive, RingOracle, bf16_bits_to_f32
import oracle


def _state(r):
    return (list(r.count), r.w, r.r)


@pytest.mark.parametrize("N,K", [(1, 1), (3, 1), (4, 2), (5, 3), (8, 3)])
def test_every_item_is_replayed_exactly_K_times_in_order(N, K):
    rng = np.random.default_rng(100 * N + K)
    ring = RingOracle(N, K)
    owner = {}                 # slot -> id of the item living there
    seen = {}                  # id -> list of counts returned
    next_id = 0
    retired = []
    for _ in range(400):
        if rng.random() < 0.5:
            n = int(rng.integers(0, N + 1))
            before = _state(ring)
            try:
                slots = ring.insert(n)
            except BufferFull:
                assert N - ring.num_live() < n
                assert _state(ring) == before          # all-or-nothing
                continue
            assert len(set(slots)) == n
            for s in slots:
                assert s not in owner                  # a live item is never overwritten
                owner[s] = next_id
                seen[next_id] = []
                next_id += 1
        else:
            B = int(rng.integers(0, N + 1))
            before = _state(ring)
            try:
                slots, counts = ring.sample(B)
            except NotEnoughLive:
                assert ring.num_live() < B
                assert _state(ring) == before
                continue
            assert len(set(slots)) == B                # distinct items within one batch
            for s, k in zip(slots, counts):
                item = owner[s]
                assert k == len(seen[item])            # count before this traversal: 0, 1, ..., K-1
                seen[item].append(k)
                if len(seen[item]) == K:
                    del owner[s]                       # discarded after K traversals
                    retired.append(item)
    assert retired, "the walk should retire some items"
    for item in retired:
        assert seen[item] == list(range(K))
    for item, ks in seen.items():
        assert len(ks) <= K


def test_full_ring_without_inserts_is_K_passes_of_the_same_minibatches():
    # the PPO analogy of Section 3.2: N minibatches, K SGD iterations over them
    N, K, B = 12, 3, 4
    ring = RingOracle(N, K)
    assert ring.insert(N) == list(range(N))
    passes = []
    for _ in range(K):
        passes.append([ring.sample(B) for _ in range(N // B)])
    for k, p in enumerate(passes):
        assert [s for s, _ in p] == [list(range(i, i + B)) for i in range(0, N, B)]
        assert all(c == [k] * B for _, c in p)
    assert ring.num_live() == 0
    with pytest.raises(NotEnoughLive):
        ring.sample(1)


def test_fifo_and_replacement_after_discard():
    ring = RingOracle(4, 2)
    assert ring.insert(3) == [0, 1, 2]
    assert ring.sample(2) == ([0, 1], [0, 0])
    assert ring.insert(1) == [3]
    with pytest.raises(BufferFull):
        ring.insert(1)
    assert ring.sample(3) == ([2, 3, 0], [0, 0, 1])     # slot 0 now traversed twice: freed
    assert ring.insert(1) == [0]                          # the freed place takes the new item
    assert ring.sample(4) == ([1, 2, 3, 0], [1, 1, 1, 0])
    assert ring.num_live() == 1


def test_bad_arguments():
    with pytest.raises(ValueError):
        RingOracle(0, 1)
    with pytest.raises(ValueError):
        RingOracle(4, 0)


@pytest.mark.parametrize("storage", ["f32", "bf16"])
@pytest.mark.parametrize("dist", ["categorical", "gaussian"])
def test_gather_is_an_index_loop(dist, storage):
    import workloads
    base = workloads.C1 if dist == "categorical" else workloads.C3
    wl = workloads.Workload(**{**base.__dict__, "T": 5, "B": 3, "A": 4, "num_slots": 6, "K": 2, "storage": storage})
    buf = BufferOracle(dist, wl.T, wl.A, wl.num_slots, wl.K, storage)
    x = workloads.make_trajectories(wl, 5, stream=9)
    slots = buf.insert_records(x["worker"], x["actions"], x["rewards"], x["dones"], target=x["target"])
    assert slots == [0, 1, 2, 3, 4]
    got_slots, counts = buf.sample(3)
    out = buf.gather(got_slots)
    for i, s in enumerate(got_slots):
        for t in range(wl.T):
            w = out["worker"][t, i]
            src = x["worker"][t, s]
            if storage == "f32":
                assert w.tobytes() == src.tobytes()
            else:
                assert np.array_equal(w, oracle.quantize_bf16(src)[0])
            assert out["dones"][t, i] == x["dones"][t, s]
