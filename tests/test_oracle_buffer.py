"""Pins for the circular-buffer oracle (Section 3.2): brute force on tiny rings."""
import copy
import itertools

import numpy as np
import pytest

from oracle.buffer import BufferFull, BufferOracle, NotEnoughLive, RingOracle, bf16_bits_to_f32, target_period
import oracle


def _state(r):
    return (list(r.count), list(r.has_target), r.w, r.r, r.t)


@pytest.mark.parametrize("N,K", [(1, 1), (3, 1), (4, 2), (5, 3), (8, 3)])
def test_every_item_is_replayed_exactly_K_times_in_order(N, K):
    rng = np.random.default_rng(100 * N + K)
    ring = RingOracle(N, K)
    owner = {}                 # slot -> id of the item living there (until its place is released)
    seen = {}                  # id -> list of counts returned
    next_id = 0
    retired = []
    pending = set()            # slots whose item was handed out for the K-th time and whose place is not yet released
    blocked_by_pending = 0
    for _ in range(600):
        u = rng.random()
        if u < 0.45:
            n = int(rng.integers(0, N + 1))
            before = _state(ring)
            occupied = len(owner)                      # live items and items awaiting release
            try:
                slots = ring.insert(n, with_target=False)
            except BufferFull:
                assert N - occupied < n
                blocked_by_pending += (N - (occupied - len(pending)) >= n)
                assert _state(ring) == before          # all-or-nothing
                continue
            assert N - occupied >= n
            assert len(set(slots)) == n
            for s in slots:
                assert s not in owner                  # neither a live item nor one whose last gradient step is pending is overwritten
                owner[s] = next_id
                seen[next_id] = []
                next_id += 1
        elif u < 0.9:
            B = int(rng.integers(0, N + 1))
            before = _state(ring)
            try:
                slots, counts = ring.sample(B)
            except NotEnoughLive:
                assert len(owner) - len(pending) < B
                assert _state(ring) == before
                continue
            if B == 0:
                assert (slots, counts) == ([], []) and _state(ring) == before      # an empty request changes nothing
                continue
            for s in pending:                          # the next iteration has begun: the previous one's discards are final
                del owner[s]
            pending.clear()
            assert len(set(slots)) == B                # distinct items within one batch
            # Algorithm 1: the items handed out for the first time (k = 0) are the ones that lack the target's output
            assert [i for i, k in enumerate(counts) if k == 0] == ring.missing_targets(slots)
            ring.mark_target([slots[i] for i in ring.missing_targets(slots)])
            assert ring.missing_targets(slots) == []
            for s, k in zip(slots, counts):
                item = owner[s]
                assert k == len(seen[item])            # count before this traversal: 0, 1, ..., K-1
                seen[item].append(k)
                if len(seen[item]) == K:
                    pending.add(s)                     # discarded after K traversals, once the gradient step is done
                    retired.append(item)
        else:
            ring.release()
            for s in pending:
                del owner[s]
            pending.clear()
        assert ring.num_live() == len(owner) - len(pending) and ring.num_empty() == N - len(owner)
    assert retired, "the walk should retire some items"
    assert N == 1 or blocked_by_pending, "the walk should meet an insert that only the pending discards keep out"
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


def test_target_update_every_N_K_steps_is_ppo_s_schedule():
    """Section 4.1.1 / 3.2: with the target updated every n = N K learner steps, a ring of N batches replayed
    K times each behaves like PPO: between two updates of the target the learner makes exactly K passes
    (epochs) over the same N minibatches, the target's output is computed once per minibatch (at k = 0), and
    the update falls on the step that exhausts the ring."""
    n_batches, K, B = 5, 3, 4
    N = n_batches * B
    assert target_period(N, B, K) == n_batches * K == 15
    assert target_period(65536, 16384, 4) == 16 and target_period(64, 32, 2) == 4
    ring = RingOracle(N, K)
    for cycle in range(3):                               # three PPO iterations
        assert ring.insert(N, with_target=False) == list(range(N))      # the workers' N fresh minibatches
        visits = {s: 0 for s in range(N)}
        target_evaluations = 0
        for step in range(1, n_batches * K + 1):
            slots, counts = ring.sample(B)
            need = ring.missing_targets(slots)
            assert need == (list(range(B)) if step <= n_batches else [])   # first epoch only
            ring.mark_target([slots[i] for i in need])
            target_evaluations += len(need)
            for s in slots:
                visits[s] += 1
            due = ring.learner_step(target_period(N, B, K))
            assert due == (step == n_batches * K)                           # on the last step of the K-th epoch
            assert (ring.num_live() == 0) == due                            # ... which is the step that empties the ring
        assert set(visits.values()) == {K} and target_evaluations == N
        assert ring.t == (cycle + 1) * n_batches * K
        assert ring.num_empty() == N - B
        with pytest.raises(BufferFull):
            ring.insert(N)                                # the last batch's places are not free before its gradient step
        ring.release()
    with pytest.raises(ValueError):
        ring.learner_step(0)


def test_fifo_and_replacement_after_discard():
    ring = RingOracle(4, 2)
    assert ring.insert(3) == [0, 1, 2]
    assert ring.sample(2) == ([0, 1], [0, 0])
    assert ring.insert(1) == [3]
    with pytest.raises(BufferFull):
        ring.insert(1)
    assert ring.sample(3) == ([2, 3, 0], [0, 0, 1])     # slot 0 now traversed twice: discarded ...
    assert ring.num_live() == 3 and ring.num_empty() == 0
    with pytest.raises(BufferFull):                       # ... but its gradient step is still to come (Algorithm 1)
        ring.insert(1)
    ring.release()
    assert ring.num_empty() == 1
    assert ring.insert(1) == [0]                          # the freed place takes the new item
    assert ring.sample(4) == ([1, 2, 3, 0], [1, 1, 1, 0])
    assert ring.num_live() == 1 and ring.num_empty() == 0
    assert ring.sample(1) == ([0], [1])                   # the next iteration begins: slots 1, 2, 3 are free now
    assert ring.num_empty() == 3 and ring.num_live() == 0
    assert ring.insert(3) == [1, 2, 3]                    # slot 0 waits for its own release


def test_items_inserted_with_their_target_output_need_none():
    ring = RingOracle(5, 2)
    a = ring.insert(2, with_target=True)
    b = ring.insert(3, with_target=False)
    slots, counts = ring.sample(5)
    assert counts == [0] * 5 and ring.missing_targets(slots) == [2, 3, 4]
    ring.mark_target([slots[3]])
    assert ring.missing_targets(slots) == [2, 4]
    assert ring.missing_targets(list(reversed(slots))) == [0, 2]       # positions in the batch as given
    # a place that is reused starts over
    ring.sample(5)
    ring.release()
    c = ring.insert(5, with_target=False)
    assert sorted(c) == sorted(a + b)
    slots, _ = ring.sample(5)
    assert ring.missing_targets(slots) == [0, 1, 2, 3, 4]


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


def test_one_byte_action_indices_are_a_storage_variant_only():
    """The records come back as they went in, as bytes; the variant exists for index actions of at most 256 values."""
    import pytest
    from oracle.buffer import BufferOracle
    rng = np.random.default_rng(0)
    T, A, n = 7, 256, 5
    worker = rng.standard_normal((T, n, A)).astype(np.float32)
    actions = rng.integers(0, A, (T, n)).astype(np.int32)
    actions[0, 0], actions[1, 1] = 255, 0
    rewards = rng.standard_normal((T, n)).astype(np.float32)
    dones = (rng.random((T, n)) < 0.2).astype(np.uint8)
    a, b = BufferOracle("categorical", T, A, 8, 2), BufferOracle("categorical", T, A, 8, 2, actions_u8=True)
    sa = a.insert_records(worker, actions, rewards, dones, target=worker)
    sb = b.insert_records(worker, actions, rewards, dones, target=worker)
    assert sa == sb
    ga, gb = a.gather(sa[::-1]), b.gather(sb[::-1])
    assert ga["actions"].dtype == np.int32 and gb["actions"].dtype == np.uint8
    np.testing.assert_array_equal(ga["actions"], gb["actions"].astype(np.int32))
    np.testing.assert_array_equal(gb["actions"], actions[:, ::-1].astype(np.uint8))
    with pytest.raises(ValueError):
        BufferOracle("categorical", T, 257, 8, 2, actions_u8=True)
    with pytest.raises(ValueError):
        BufferOracle("gaussian", T, 3, 8, 2, actions_u8=True)
