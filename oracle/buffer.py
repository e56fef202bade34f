"""Oracle for the circular buffer C(N, K) (Section 3.2, Algorithm 1) -- test infrastructure.

The paper fixes: N stored items, each traversable at most K times, after which
it is discarded and its place taken by a new worker batch.  The order of
traversal, and what happens when the ring is full or short, are readings of a
text that is silent on them: ring order from a read cursor, inserts never
overwrite a live item, insert and sample are all-or-nothing.  (The bookkeeping
itself is pinned by a brute-force simulation in the tests.)

Algorithm 1's learner loop orders a step as: obtain the batch and its count k;
if k = 0 evaluate it on the target and append the result; compute the gradients;
"if k = K, discard"; "if t = 0 (mod t_target), update the target network".  So a
batch handed out for the K-th time is still needed by the gradient computation
that follows: its place becomes free for a new worker batch only after that,
here when `release` is called or at the next `sample` (which begins the next
iteration of the loop).  The same loop's bookkeeping of "does this batch still
need the target's evaluation" and of the step counter t live here as well.

Plain Python, one loop per operation; the stored records are numpy arrays in
slot-major order ``[N, T, ...]``.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

import numpy as np

from . import quantize_bf16

EMPTY, DISCARDED = -1, -2


class BufferFull(Exception):
    pass


class NotEnoughLive(Exception):
    pass


def target_period(num_slots: int, B: int, K: int) -> int:
    """Section 4.1.1: the target is updated every n = N K learner steps, N the number of batches the
    buffer holds (here num_slots trajectories in batches of B) and K the replay limit."""
    return (num_slots // B) * K


class RingOracle:
    """Integer bookkeeping only."""

    def __init__(self, num_slots: int, K: int):
        if num_slots < 1 or K < 1:
            raise ValueError("num_slots and K must be positive")
        self.N, self.K = num_slots, K
        # EMPTY, DISCARDED (traversed K times, its last gradient step possibly still to come), else times traversed so far (0..K-1)
        self.count = [EMPTY] * num_slots
        self.has_target = [False] * num_slots   # the target network's output for this item is stored
        self.w = 0                      # write cursor
        self.r = 0                      # read cursor
        self.t = 0                      # learner steps counted

    def num_live(self) -> int:
        return sum(1 for c in self.count if c >= 0)

    def num_empty(self) -> int:
        return sum(1 for c in self.count if c == EMPTY)

    def insert(self, n: int, with_target: bool = True) -> List[int]:
        if n < 0:
            raise ValueError("n < 0")
        if self.num_empty() < n:
            raise BufferFull()
        slots = []
        for _ in range(n):
            while self.count[self.w] != EMPTY:
                self.w = (self.w + 1) % self.N
            self.count[self.w] = 0
            self.has_target[self.w] = with_target
            slots.append(self.w)
            self.w = (self.w + 1) % self.N
        return slots

    def release(self) -> None:
        """Algorithm 1, "if k = K, discard": the places of the items whose K-th traversal was handed out
        become free for new worker batches."""
        for s in range(self.N):
            if self.count[s] == DISCARDED:
                self.count[s] = EMPTY

    def sample(self, B: int) -> Tuple[List[int], List[int]]:
        if B < 0:
            raise ValueError("B < 0")
        if self.num_live() < B:
            raise NotEnoughLive()
        if B == 0:
            return [], []                         # an empty request is no iteration of the loop: nothing changes
        self.release()                            # the previous iteration's gradient step is behind us
        slots, counts = [], []
        for _ in range(B):
            while self.count[self.r] < 0:
                self.r = (self.r + 1) % self.N
            s = self.r
            slots.append(s)
            counts.append(self.count[s])          # traversals before this one
            self.count[s] += 1
            if self.count[s] == self.K:
                self.count[s] = DISCARDED         # traversed K times: not handed out again
            self.r = (self.r + 1) % self.N
        return slots, counts

    def mark_target(self, slots) -> None:
        for s in slots:
            self.has_target[s] = True

    def missing_targets(self, slots) -> List[int]:
        """Algorithm 1, "if k = 0, evaluate B on target, append target output to B": the positions in
        the batch whose item has no target output stored yet."""
        return [i for i, s in enumerate(slots) if not self.has_target[s]]

    def learner_step(self, t_target: int) -> bool:
        """Count one learner step; Algorithm 1, "if t = 0 (mod t_target), update target network"."""
        if t_target < 1:
            raise ValueError("t_target < 1")
        self.t += 1
        return self.t % t_target == 0


class BufferOracle(RingOracle):
    """Ring bookkeeping plus the stored records (slot-major), for gather checks."""

    def __init__(self, dist: str, T: int, A: int, num_slots: int, K: int, storage: str = "f32",
                 actions_u8: bool = False):
        super().__init__(num_slots, K)
        if actions_u8 and (dist != "categorical" or A > 256):
            raise ValueError("one-byte action indices: categorical policies with at most 256 actions")
        self.dist, self.T, self.A, self.storage = dist, T, A, storage
        self.W = A if dist == "categorical" else 2 * A
        fdt = np.float32 if storage == "f32" else np.uint16
        N = num_slots
        self.worker = np.zeros((N, T, self.W), fdt)
        self.target = np.zeros((N, T, self.W), fdt)
        # categorical: the index of the action taken, as int32 or (a storage variant) as one byte
        idt = np.uint8 if actions_u8 else np.int32
        self.actions = np.zeros((N, T), idt) if dist == "categorical" else np.zeros((N, T, A), fdt)
        self.rewards = np.zeros((N, T), fdt)
        self.dones = np.zeros((N, T), np.uint8)

    def _store(self, x: np.ndarray) -> np.ndarray:
        x = np.asarray(x, np.float32)
        return x if self.storage == "f32" else quantize_bf16(x)[0]

    def insert_records(self, worker, actions, rewards, dones, target=None) -> List[int]:
        """Time-major fp32 inputs [T, n, ...]; returns the slots used."""
        n = worker.shape[1]
        slots = self.insert(n, with_target=target is not None)
        for i, s in enumerate(slots):
            self.worker[s] = self._store(worker[:, i])
            if self.dist == "categorical":
                self.actions[s] = actions[:, i]
            else:
                self.actions[s] = self._store(actions[:, i])
            self.rewards[s] = self._store(rewards[:, i])
            self.dones[s] = dones[:, i]
            if target is not None:
                self.target[s] = self._store(target[:, i])
        return slots

    def put_target(self, slots, target) -> None:
        for i, s in enumerate(slots):
            self.target[s] = self._store(target[:, i])
        self.mark_target(slots)

    def gather(self, slots) -> Dict[str, np.ndarray]:
        """Time-major copies, in the storage dtype (bf16 as uint16 bit patterns)."""
        B = len(slots)
        out = dict(worker=np.empty((self.T, B, self.W), self.worker.dtype),
                   target=np.empty((self.T, B, self.W), self.target.dtype),
                   actions=np.empty((self.T, B) + self.actions.shape[2:], self.actions.dtype),
                   rewards=np.empty((self.T, B), self.rewards.dtype),
                   dones=np.empty((self.T, B), np.uint8))
        for i, s in enumerate(slots):
            out["worker"][:, i] = self.worker[s]
            out["target"][:, i] = self.target[s]
            out["actions"][:, i] = self.actions[s]
            out["rewards"][:, i] = self.rewards[s]
            out["dones"][:, i] = self.dones[s]
        return out


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to fp32 values."""
    return (bits.astype(np.uint32) << 16).view(np.float32)
