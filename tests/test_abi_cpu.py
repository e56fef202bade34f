"""The C-ABI library: it loads, exports what the header declares, and its host-side logic
(argument checks, ring bookkeeping) behaves -- none of this needs a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle.buffer import BufferFull, NotEnoughLive, RingOracle
from paper_1912_00167_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE_DEV = ctypes.c_void_p(0x7000_0000_0000)      # 256-aligned, never dereferenced by host-only calls


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_1912_00167_amd import build
        build.build()
    return B.load()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "impact.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(impact_[a-z0-9_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert B.impact_version() == "0.1"
    assert B.status_string(0) == "ok" and "full" in B.status_string(B.IMPACT_ERR_BUFFER_FULL)


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(B.impact_buffer_desc_t) == 28
    assert ctypes.sizeof(B.impact_loss_config_t) == 40
    assert ctypes.sizeof(B.impact_batch_t) == 6 * ctypes.sizeof(ctypes.c_void_p)
    assert ctypes.sizeof(B.impact_loss_out_t) == 7 * ctypes.sizeof(ctypes.c_void_p)


def _create(lib, dist=0, T=4, A=3, N=8, K=2, storage=0, ptr=FAKE_DEV, nbytes=None):
    d = B.impact_buffer_desc_t(dist, T, A, N, K, storage)
    need = lib.impact_buffer_storage_bytes(ctypes.byref(d))
    h = ctypes.c_void_p()
    rc = lib.impact_buffer_create(ctypes.byref(d), ptr, need if nbytes is None else nbytes, ctypes.byref(h))
    return rc, h, need


def test_storage_bytes_cover_all_planes(lib):
    up = lambda x, a: (x + a - 1) // a * a
    for dist, storage in ((0, 0), (0, 1), (1, 0), (1, 1)):
        for T, A, N in ((7, 5, 11), (50, 18, 64), (128, 17, 8)):
            d = B.impact_buffer_desc_t(dist, T, A, N, 2, storage)
            es = 4 if storage == 0 else 2
            W = A if dist == 0 else 2 * A
            # distribution and action planes: every slot padded to 16 bytes; rewards and flags packed;
            # each plane followed by >= 16 bytes and aligned to 256; one 256-byte block of kernel bookkeeping
            planes = [N * up(T * W * es, 16)] * 2 + [N * up(T * 4 if dist == 0 else T * A * es, 16), N * T * es, N * T]
            want = sum(up(p + 16, 256) for p in planes) + 256
            got = lib.impact_buffer_storage_bytes(ctypes.byref(d))
            assert got == want, (dist, storage, T, A, N)


def test_storage_of_a_buffer_that_caches_log_probabilities(lib):
    up = lambda x, a: (x + a - 1) // a * a
    T, A, N = 50, 18, 64
    for dist, storage in ((0, 0), (1, 1)):
        es = 4 if storage == 0 else 2
        W = A if dist == 0 else 2 * A
        act = N * up(T * 4 if dist == 0 else T * A * es, 16)
        common = [act, N * T * es, N * T, N * T * 16]           # actions, rewards, flags, two doubles per step
        for flags, extra in ((B.IMPACT_BUFFER_CACHE_LOGP, [N * up(T * W * es, 16)]),
                             (B.IMPACT_BUFFER_CACHE_LOGP | B.IMPACT_BUFFER_NO_TARGET_DIST, [])):
            d = B.impact_buffer_desc_t(dist, T, A, N, 2, storage, flags)
            want = sum(up(p + 16, 256) for p in common + extra) + 256
            assert lib.impact_buffer_storage_bytes(ctypes.byref(d)) == want, (dist, storage, flags)
    # dropping the target's distribution makes sense only when its log-probabilities are cached
    d = B.impact_buffer_desc_t(0, T, A, N, 2, 0, B.IMPACT_BUFFER_NO_TARGET_DIST)
    assert lib.impact_buffer_storage_bytes(ctypes.byref(d)) == 0
    d = B.impact_buffer_desc_t(0, T, A, N, 2, 0, 8)
    assert lib.impact_buffer_storage_bytes(ctypes.byref(d)) == 0


def test_storage_of_a_buffer_with_one_byte_action_indices(lib):
    up = lambda x, a: (x + a - 1) // a * a
    for T, A, N, storage in ((50, 18, 64, 0), (13, 256, 24, 1), (100, 6, 8, 0)):
        es = 4 if storage == 0 else 2
        planes = [N * up(T * A * es, 16)] * 2 + [N * up(T, 16), N * T * es, N * T]
        d = B.impact_buffer_desc_t(0, T, A, N, 2, storage, B.IMPACT_BUFFER_ACTIONS_U8)
        assert lib.impact_buffer_storage_bytes(ctypes.byref(d)) == sum(up(p + 16, 256) for p in planes) + 256
    # an index of one byte names at most 256 actions, and a Gaussian policy's action is no index
    for dist, A in ((0, 257), (1, 3)):
        d = B.impact_buffer_desc_t(dist, 8, A, 16, 1, 0, B.IMPACT_BUFFER_ACTIONS_U8)
        assert lib.impact_buffer_storage_bytes(ctypes.byref(d)) == 0


def test_invalid_descriptors_and_arguments(lib):
    for kw in (dict(K=0), dict(N=0), dict(T=0), dict(A=0), dict(dist=2), dict(storage=3)):
        d = dict(dist=0, T=4, A=3, N=8, K=2, storage=0)
        d.update(kw)
        desc = B.impact_buffer_desc_t(d["dist"], d["T"], d["A"], d["N"], d["K"], d["storage"])
        assert lib.impact_buffer_storage_bytes(ctypes.byref(desc)) == 0
        rc, h, _ = _create(lib, **d)
        assert rc == B.IMPACT_ERR_INVALID_ARG and not h
    rc, h, need = _create(lib, ptr=None)
    assert rc == B.IMPACT_ERR_INVALID_ARG
    rc, h, need = _create(lib, ptr=ctypes.c_void_p(0x7000_0000_0010))     # not 256-aligned
    assert rc == B.IMPACT_ERR_INVALID_ARG
    rc, h, need = _create(lib, nbytes=100)                                  # too small
    assert rc == B.IMPACT_ERR_INVALID_ARG
    rc, h, need = _create(lib)
    assert rc == B.IMPACT_OK and h
    out = (ctypes.c_int32 * 4)()
    assert lib.impact_buffer_sample(h, 2, None, out) == B.IMPACT_ERR_INVALID_ARG
    assert lib.impact_buffer_sample(h, -1, out, out) == B.IMPACT_ERR_INVALID_ARG
    assert lib.impact_buffer_reserve(h, 2, None) == B.IMPACT_ERR_INVALID_ARG
    assert lib.impact_buffer_sample(None, 1, out, out) == B.IMPACT_ERR_INVALID_ARG
    assert lib.impact_buffer_insert(h, 1, None, out, None) == B.IMPACT_ERR_INVALID_ARG
    assert lib.impact_buffer_put_target(h, 1, out, None, None) == B.IMPACT_ERR_INVALID_ARG
    bad_slots = (ctypes.c_int32 * 1)(99)
    assert lib.impact_buffer_put_target(h, 1, bad_slots, FAKE_DEV, None) == B.IMPACT_ERR_INVALID_ARG
    assert lib.impact_buffer_gather(h, 1, None, None, None) == B.IMPACT_ERR_INVALID_ARG
    assert lib.impact_buffer_sample(h, 0, None, None) == B.IMPACT_OK          # empty request: no-op
    assert lib.impact_buffer_insert(h, 0, None, None, None) == B.IMPACT_OK
    assert lib.impact_buffer_destroy(h) == B.IMPACT_OK
    assert lib.impact_buffer_destroy(None) == B.IMPACT_OK


def test_loss_argument_checks_happen_before_any_device_work(lib):
    assert lib.impact_loss_workspace_bytes(0, 0, 8, 4) == 0
    assert lib.impact_loss_workspace_bytes(2, 4, 8, 4) == 0
    ws = lib.impact_loss_workspace_bytes(0, 100, 8192, 18)
    assert ws >= (8192 // 8) * 8 * 4 and ws % 256 == 0
    p = FAKE_DEV
    batch = B.impact_batch_t(p, p, p, p, p)
    out = B.impact_loss_out_t(p, p, None, None, p)
    good = B.make_config()
    call = lambda cfg=good, T=4, Bn=8, A=3, b=batch, o=out, w=p, wb=ws, dist=0, dt=0, learner=p: \
        lib.impact_loss_fwd_bwd(dist, dt, T, Bn, A, learner, p, p, ctypes.byref(b) if b else None,
                                ctypes.byref(cfg) if cfg else None, ctypes.byref(o) if o else None, w, wb, None)
    E = B.IMPACT_ERR_INVALID_ARG
    assert call(T=0) == E and call(Bn=0) == E and call(A=0) == E          # empty inputs
    assert call(dist=5) == E and call(dt=7) == E
    assert call(cfg=None) == E and call(b=None) == E and call(o=None) == E and call(w=None) == E
    assert call(wb=8) == E                                                 # workspace too small
    assert call(learner=None) == E
    assert call(learner=ctypes.c_void_p(0x7000_0000_0004)) == E            # misaligned
    assert call(b=B.impact_batch_t(p, None, p, p, p)) == E
    assert call(o=B.impact_loss_out_t(p, None, None, None, p)) == E
    for kw in (dict(gamma=float("nan")), dict(lam=float("inf")), dict(rho_bar=-1.0), dict(c_bar=-0.5),
               dict(rho_clip=0.5), dict(rho_clip=float("nan")), dict(eps=-0.1), dict(vf_coeff=float("inf"))):
        assert call(cfg=B.make_config(**kw)) == E, kw


def _vp(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _same_target_bookkeeping(lib, h, ring, slots):
    """impact_buffer_missing_targets against the oracle, for the batch `slots`."""
    s = np.ascontiguousarray(slots, np.int32)
    pos = np.full(max(len(s), 1), -7, np.int32)
    n = ctypes.c_int32(-1)
    assert lib.impact_buffer_missing_targets(h, len(s), _vp(s), _vp(pos), ctypes.byref(n)) == B.IMPACT_OK
    want = ring.missing_targets(list(slots))
    assert n.value == len(want) and pos[: n.value].tolist() == want
    assert np.all(pos[n.value:] == -7)
    return want


def _lib_state_walk(lib, N, K, seed, steps=300):
    rng = np.random.default_rng(seed)
    rc, h, _ = _create(lib, N=N, K=K)
    assert rc == 0
    ring = RingOracle(N, K)
    t_target = int(rng.integers(1, 7))
    for _ in range(steps):
        u = rng.random()
        if u < 0.45:
            n = int(rng.integers(0, N + 2))
            out = np.full(max(n, 1), -7, np.int32)
            rc = lib.impact_buffer_reserve(h, n, _vp(out))
            try:
                want = ring.insert(n, with_target=False)
                assert rc == B.IMPACT_OK
                assert out[:n].tolist() == want
            except BufferFull:
                assert rc == B.IMPACT_ERR_BUFFER_FULL
                assert np.all(out == -7)                       # untouched
        elif u < 0.9:
            Bn = int(rng.integers(0, N + 2))
            s = np.full(max(Bn, 1), -7, np.int32)
            c = np.full(max(Bn, 1), -7, np.int32)
            rc = lib.impact_buffer_sample(h, Bn, _vp(s), _vp(c))
            try:
                ws, wc = ring.sample(Bn)
                assert rc == B.IMPACT_OK
                assert s[:Bn].tolist() == ws and c[:Bn].tolist() == wc
                # Algorithm 1: the target is evaluated on what is handed out for the first time ...
                need = _same_target_bookkeeping(lib, h, ring, ws)
                assert need == [i for i, k in enumerate(wc) if k == 0]
                got_target = np.asarray([ws[i] for i in need], np.int32)
                assert lib.impact_buffer_mark_target(h, len(got_target), _vp(got_target) if len(got_target) else None) == 0
                ring.mark_target(got_target.tolist())
                assert _same_target_bookkeeping(lib, h, ring, ws) == []
                # ... one learner step is counted, and the target update falls on every t_target-th
                t, due = ctypes.c_int64(-1), ctypes.c_int32(-1)
                assert lib.impact_buffer_learner_step(h, t_target, ctypes.byref(t), ctypes.byref(due)) == 0
                assert bool(due.value) == ring.learner_step(t_target) and t.value == ring.t
            except NotEnoughLive:
                assert rc == B.IMPACT_ERR_NOT_ENOUGH_LIVE
                assert np.all(s == -7) and np.all(c == -7)
        else:
            assert lib.impact_buffer_release_discarded(h) == B.IMPACT_OK
            ring.release()
        assert lib.impact_buffer_num_live(h) == ring.num_live()
        assert lib.impact_buffer_num_empty(h) == ring.num_empty()
    lib.impact_buffer_destroy(h)


@pytest.mark.parametrize("N,K", [(1, 1), (3, 1), (4, 2), (8, 3), (64, 2), (257, 5)])
def test_ring_bookkeeping_is_bit_exact_with_the_oracle(lib, N, K):
    for seed in range(4):
        _lib_state_walk(lib, N, K, seed)


def _walk(lib, h, ring, rng, N, steps):
    for _ in range(steps):
        n = int(rng.integers(0, N + 1))
        out = np.empty(max(n, 1), np.int32)
        u = rng.random()
        if u < 0.45:
            rc = lib.impact_buffer_reserve(h, n, _vp(out))
            try:
                assert out[:n].tolist() == ring.insert(n, with_target=False) and rc == 0
            except BufferFull:
                assert rc == B.IMPACT_ERR_BUFFER_FULL
        elif u < 0.9:
            c = np.empty(max(n, 1), np.int32)
            rc = lib.impact_buffer_sample(h, n, _vp(out), _vp(c))
            try:
                ws, wc = ring.sample(n)
                assert rc == 0 and out[:n].tolist() == ws and c[:n].tolist() == wc
                need = _same_target_bookkeeping(lib, h, ring, ws)
                if rng.random() < 0.5 and need:                      # some batches get their target output, some not yet
                    got_target = np.asarray([ws[i] for i in need[::2]], np.int32)
                    assert lib.impact_buffer_mark_target(h, len(got_target), _vp(got_target)) == 0
                    ring.mark_target(got_target.tolist())
                t = ctypes.c_int64(-1)
                assert lib.impact_buffer_learner_step(h, 3, ctypes.byref(t), None) == 0
                ring.learner_step(3)
                assert t.value == ring.t
            except NotEnoughLive:
                assert rc == B.IMPACT_ERR_NOT_ENOUGH_LIVE
        else:
            assert lib.impact_buffer_release_discarded(h) == 0
            ring.release()


@pytest.mark.parametrize("N,K", [(5, 2), (64, 3)])
def test_ring_state_survives_export_and_import(lib, N, K):
    """Stop and resume: a ring restored from an exported record continues exactly as the oracle's ring does."""
    rng = np.random.default_rng(N)
    rc, h, _ = _create(lib, N=N, K=K)
    assert rc == 0
    ring = RingOracle(N, K)
    _walk(lib, h, ring, rng, N, 120)
    nbytes = lib.impact_buffer_state_bytes(h)
    assert nbytes == 56 + 5 * N
    state = np.zeros(nbytes, np.uint8)
    vp = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    assert lib.impact_buffer_export_state(h, vp(state), nbytes - 1) == B.IMPACT_ERR_INVALID_ARG
    assert lib.impact_buffer_export_state(h, vp(state), nbytes) == 0
    lib.impact_buffer_destroy(h)
    rc, h2, _ = _create(lib, N=N, K=K)
    assert rc == 0 and lib.impact_buffer_num_live(h2) == 0
    # malformed records change nothing
    for damage in ("magic", "count", "count_low", "live", "cursor", "short", "flag", "time"):
        bad = state.copy()
        words = bad[: 56 + 4 * N].view(np.int32)      # header (14 words) and the per-slot counts
        if damage == "magic":
            words[0] ^= 1
        elif damage == "count":
            words[14] = K
        elif damage == "count_low":
            words[14] = -3
        elif damage == "flag":
            bad[56 + 4 * N] = 2
        elif damage == "time":
            words[13] = -1                       # high word of the step counter: negative
        elif damage == "live":
            words[10] += 1
        elif damage == "cursor":
            words[8] = N
        size = nbytes - 4 if damage == "short" else nbytes
        assert lib.impact_buffer_import_state(h2, vp(bad), size) == B.IMPACT_ERR_INVALID_ARG, damage
        assert lib.impact_buffer_num_live(h2) == 0
    # a record from a ring of another shape is refused
    rc, h3, _ = _create(lib, N=N + 1, K=K)
    assert lib.impact_buffer_import_state(h3, vp(state), nbytes) == B.IMPACT_ERR_INVALID_ARG
    lib.impact_buffer_destroy(h3)
    assert lib.impact_buffer_import_state(h2, vp(state), nbytes) == 0
    assert lib.impact_buffer_num_live(h2) == ring.num_live() and lib.impact_buffer_num_empty(h2) == ring.num_empty()
    _walk(lib, h2, ring, rng, N, 120)
    assert lib.impact_buffer_num_live(h2) == ring.num_live() and lib.impact_buffer_num_empty(h2) == ring.num_empty()
    lib.impact_buffer_destroy(h2)


def test_ring_at_full_workload_size_matches_oracle(lib):
    # the largest ring of the workloads: 65536 slots, K = 4, batches of 16384
    N, K, Bn = 65536, 4, 16384
    rc, h, _ = _create(lib, dist=1, T=128, A=17, N=N, K=K, storage=1)
    assert rc == 0
    ring = RingOracle(N, K)
    out = np.empty(N, np.int32)
    assert lib.impact_buffer_reserve(h, N, out.ctypes.data_as(ctypes.c_void_p)) == 0
    assert out.tolist() == ring.insert(N)
    s, c = np.empty(Bn, np.int32), np.empty(Bn, np.int32)
    for step in range(N * K // Bn):
        assert lib.impact_buffer_sample(h, Bn, s.ctypes.data_as(ctypes.c_void_p), c.ctypes.data_as(ctypes.c_void_p)) == 0
        ws, wc = ring.sample(Bn)
        assert np.array_equal(s, np.asarray(ws, np.int32)) and np.array_equal(c, np.asarray(wc, np.int32))
        if step == 11:      # three full passes done: nothing has been traversed K times yet
            assert lib.impact_buffer_num_live(h) == N
        if step == 13:      # half of the fourth pass: half of the ring discarded
            assert lib.impact_buffer_num_live(h) == N // 2
    assert lib.impact_buffer_num_live(h) == 0
    assert lib.impact_buffer_sample(h, 1, s.ctypes.data_as(ctypes.c_void_p), c.ctypes.data_as(ctypes.c_void_p)) \
        == B.IMPACT_ERR_NOT_ENOUGH_LIVE
    # the last batch's places wait for its gradient step; the three before it were freed as the next was drawn
    assert lib.impact_buffer_num_empty(h) == N - Bn == ring.num_empty()
    assert lib.impact_buffer_reserve(h, N, out.ctypes.data_as(ctypes.c_void_p)) == B.IMPACT_ERR_BUFFER_FULL
    assert lib.impact_buffer_release_discarded(h) == 0
    assert lib.impact_buffer_num_empty(h) == N
    assert lib.impact_buffer_reserve(h, N, out.ctypes.data_as(ctypes.c_void_p)) == 0
    lib.impact_buffer_destroy(h)


def test_target_period_and_ppo_schedule_through_the_library(lib):
    """Section 4.1.1's n = N K, and Section 3.2's PPO analogy on the library's own ring: K passes over the
    same N minibatches between two target updates, the target evaluated once per minibatch."""
    from oracle.buffer import target_period
    for num_slots, Bn, K in ((65536, 16384, 4), (32768, 8192, 8), (64, 32, 2), (20, 4, 3), (7, 2, 5), (3, 4, 2)):
        assert lib.impact_target_period(num_slots, Bn, K) == target_period(num_slots, Bn, K)
    assert lib.impact_target_period(0, 4, 2) == 0 and lib.impact_target_period(8, 0, 2) == 0 and lib.impact_target_period(8, 4, 0) == 0
    n_batches, K, Bn = 5, 3, 4
    N = n_batches * Bn
    period = lib.impact_target_period(N, Bn, K)
    rc, h, _ = _create(lib, N=N, K=K)
    assert rc == 0
    out, s, c = (np.empty(N, np.int32) for _ in range(3))
    for cycle in range(2):
        assert lib.impact_buffer_reserve(h, N, _vp(out)) == 0
        first_pass = []
        for step in range(1, period + 1):
            assert lib.impact_buffer_sample(h, Bn, _vp(s), _vp(c)) == 0
            if step <= n_batches:
                first_pass.append(s[:Bn].tolist())
            assert s[:Bn].tolist() == first_pass[(step - 1) % n_batches]          # the same minibatches, pass after pass
            assert c[:Bn].tolist() == [(step - 1) // n_batches] * Bn
            due = ctypes.c_int32(-1)
            assert lib.impact_buffer_learner_step(h, period, None, ctypes.byref(due)) == 0
            assert bool(due.value) == (step == period)
        assert lib.impact_buffer_num_live(h) == 0
        assert lib.impact_buffer_release_discarded(h) == 0
    assert lib.impact_buffer_learner_step(h, 0, None, None) == B.IMPACT_ERR_INVALID_ARG
    assert lib.impact_buffer_learner_step(None, 1, None, None) == B.IMPACT_ERR_INVALID_ARG
    bad = np.array([0, N], np.int32)
    n = ctypes.c_int32(0)
    assert lib.impact_buffer_missing_targets(h, 2, _vp(bad), _vp(out), ctypes.byref(n)) == B.IMPACT_ERR_INVALID_ARG
    assert lib.impact_buffer_missing_targets(h, 2, _vp(bad), _vp(out), None) == B.IMPACT_ERR_INVALID_ARG
    assert lib.impact_buffer_missing_targets(h, 0, None, None, ctypes.byref(n)) == 0 and n.value == 0
    assert lib.impact_buffer_reset_lanes(h) == 0 and lib.impact_buffer_reset_lanes(None) == B.IMPACT_ERR_INVALID_ARG
    assert lib.impact_buffer_release_discarded(None) == B.IMPACT_ERR_INVALID_ARG
    assert lib.impact_buffer_num_empty(None) == B.IMPACT_ERR_INVALID_ARG
    lib.impact_buffer_destroy(h)


def test_a_discarded_slot_is_not_reused_before_its_release(lib):
    """Algorithm 1 discards a batch after its gradient step: between the sample that hands a slot out for the
    K-th time and the release (or the next sample) no insert may take the slot."""
    rc, h, _ = _create(lib, N=4, K=1)
    assert rc == 0
    out, s, c = (np.empty(4, np.int32) for _ in range(3))
    assert lib.impact_buffer_reserve(h, 4, _vp(out)) == 0
    assert lib.impact_buffer_sample(h, 3, _vp(s), _vp(c)) == 0 and s[:3].tolist() == [0, 1, 2]
    assert lib.impact_buffer_num_live(h) == 1 and lib.impact_buffer_num_empty(h) == 0
    assert lib.impact_buffer_reserve(h, 1, _vp(out)) == B.IMPACT_ERR_BUFFER_FULL      # the loss of slots 0-2 is still to come
    assert lib.impact_buffer_release_discarded(h) == 0
    assert lib.impact_buffer_reserve(h, 2, _vp(out)) == 0 and out[:2].tolist() == [0, 1]
    # without an explicit release the next sample frees them
    assert lib.impact_buffer_sample(h, 2, _vp(s), _vp(c)) == 0 and s[:2].tolist() == [3, 0]
    assert lib.impact_buffer_num_empty(h) == 1                                        # slot 2; 3 and 0 wait
    assert lib.impact_buffer_sample(h, 1, _vp(s), _vp(c)) == 0 and s[0] == 1
    assert lib.impact_buffer_num_empty(h) == 3
    lib.impact_buffer_destroy(h)


def test_an_invalid_fused_call_leaves_the_handle_as_it_was(lib):
    """impact_loss_fwd_bwd_from_buffer checks every argument before it touches the stream or the handle."""
    rc, h, _ = _create(lib, N=8, K=2)
    assert rc == 0
    p = FAKE_DEV
    out = B.impact_loss_out_t(p, p, None, None, p)
    ws = lib.impact_loss_workspace_bytes(0, 4, 8, 3)
    bad = B.make_config(gamma=float("nan"))
    E = B.IMPACT_ERR_INVALID_ARG
    call = lambda cfg, o=out, w=p, wb=ws, slots=p: lib.impact_loss_fwd_bwd_from_buffer(
        h, 8, slots, p, p, p, ctypes.byref(cfg) if cfg else None, ctypes.byref(o) if o else None, w, wb, None)
    assert call(bad) == E and call(None) == E and call(B.make_config(), o=None) == E
    assert call(B.make_config(), w=None) == E and call(B.make_config(), wb=8) == E and call(B.make_config(), slots=None) == E
    lib.impact_buffer_destroy(h)
