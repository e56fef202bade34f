"""Do the pins notice a mistake?  Each case plants one plausible slip (a dropped term, a wrong sign or index,
swapped operands) in a copy of the oracle's C source, builds it, and runs the pin files named for it in a
child interpreter that loads the copy: at least one pin has to fail.  The oracle itself is untouched."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "oracle", "impact_oracle.c")

VTRACE = ["test_oracle_vtrace.py"]
SURR = ["test_oracle_surrogate.py"]
GRAD = ["test_oracle_gradients.py"]
POLICY = ["test_oracle_policy.py"]
CACHED = ["test_oracle_cached.py"]

# (what is planted, text in the source, replacement, pin files that must notice)
MUTATIONS = [
    ("rho truncated at c_bar", "double rho = fmin(cfg->rho_bar, w);", "double rho = fmin(cfg->c_bar, w);", VTRACE),
    ("lambda dropped from the recurrence", "acc = delta + gamma_t * cfg->lambda * c * acc;", "acc = delta + gamma_t * c * acc;", VTRACE),
    ("importance weight upside down", "return exp(logp_target - logp_worker);", "return exp(logp_worker - logp_target);", VTRACE),
    ("next value taken from the same step", "double v_next = (t == T - 1) ? bootstrap : values[t + 1];",
     "double v_next = (t == T - 1) ? bootstrap : values[t];", VTRACE),
    ("episode ends ignored in the scan", "double gamma_t = dones[t] ? 0.0 : cfg->gamma;", "double gamma_t = cfg->gamma;", VTRACE),
    ("c not truncated", "double c = fmin(cfg->c_bar, w);", "double c = w;", VTRACE),
    ("advantage without the value baseline in delta", "double delta = rho * (rewards[t] + gamma_t * v_next - values[t]);",
     "double delta = rho * (rewards[t] + gamma_t * v_next);", VTRACE + ["test_oracle_ppo.py"]),
    ("rho_clip multiplies instead of divides", "double alt = logp_worker - log(rho_clip);", "double alt = logp_worker + log(rho_clip);", SURR),
    ("min of the denominator instead of max", "if (alt > log_den) log_den = alt;", "if (alt < log_den) log_den = alt;", SURR),
    ("surrogate takes the larger branch", "return unclipped < clipped ? unclipped : clipped;", "return unclipped > clipped ? unclipped : clipped;", SURR),
    ("clip window not centred on one", "double clipped = clip(R, 1.0 - eps, 1.0 + eps) * adv;", "double clipped = clip(R, -eps, eps) * adv;", SURR),
    ("gradient gate on the wrong sign of the advantage", "if (adv > 0.0 && R > 1.0 + eps) return 0;", "if (adv < 0.0 && R > 1.0 + eps) return 0;", GRAD + SURR),
    ("value error with the wrong sign", "double dv = values[s] - vs[s];", "double dv = vs[s] + values[s];", GRAD + ["test_oracle_ppo.py"]),
    ("entropy gradient without the +H term", "double dH = -p[k] * ((zl[k] - lse_l) + H);", "double dH = -p[k] * (zl[k] - lse_l);", GRAD),
    ("KL gradient with the wrong sign", "double dKL = zt ? p[k] - pt[k] : 0.0;", "double dKL = zt ? pt[k] - p[k] : 0.0;", GRAD),
    ("softmax gradient without the indicator", "double dlogp = ((k == a) ? 1.0 : 0.0) - p[k];", "double dlogp = -p[k];", GRAD),
    ("Gaussian log-sigma gradient without the -1", "double dlogp_dls = zed * zed - 1.0;", "double dlogp_dls = zed * zed;", GRAD),
    ("Gaussian mean gradient divided by sigma once", "double dlogp_dmu = diff / (sl * sl);", "double dlogp_dmu = diff / sl;", GRAD),
    ("Gaussian KL gradient without the mean term", "dKL_dls = 1.0 - (st * st + dm * dm) / (sl * sl);", "dKL_dls = 1.0 - (st * st) / (sl * sl);", GRAD),
    ("policy gradient not divided by the batch", "double g = active ? (-adv[s] * R / M) : 0.0;", "double g = active ? (-adv[s] * R) : 0.0;", GRAD),
    ("policy gradient without the ratio", "double g = active ? (-adv[s] * R / M) : 0.0;", "double g = active ? (-adv[s] / M) : 0.0;", GRAD),
    ("entropy bonus added to the loss instead of subtracted", "loss5[0] = pg + cfg->vf_coeff * vf - cfg->ent_coeff * h + cfg->kl_coeff * kl;",
     "loss5[0] = pg + cfg->vf_coeff * vf + cfg->ent_coeff * h + cfg->kl_coeff * kl;", GRAD + SURR),
    ("KL taken from theta to target", "KL = zt ? oracle_cat_kl(zt, zl, A) : 0.0;", "KL = zt ? oracle_cat_kl(zl, zt, A) : 0.0;", GRAD),
    ("Gaussian KL with the means' term halved twice", "(st * st + dm * dm) / (2.0 * sl * sl) - 0.5;", "(st * st + 0.5 * dm * dm) / (2.0 * sl * sl) - 0.5;", POLICY),
    ("Gaussian density without the normalising constant", "lp += -0.5 * zed * zed - p[D + d] - 0.5 * LOG_2PI;", "lp += -0.5 * zed * zed - p[D + d];", POLICY),
    ("Gaussian entropy without the +1", "h += p[D + d] + 0.5 * (LOG_2PI + 1.0);", "h += p[D + d] + 0.5 * LOG_2PI;", POLICY),
    ("softmax normaliser without the shift added back", "return m + log(s);", "return log(s);", POLICY),
    ("categorical entropy with the wrong sign", "h -= exp(lp) * lp;", "h += exp(lp) * lp;", POLICY),
    ("cached pair read in the wrong order (loss)", "lp_t = cached_logp ? cached_logp[2 * s + 1] : oracle_cat_logp(zt, A, a);",
     "lp_t = cached_logp ? cached_logp[2 * s] : oracle_cat_logp(zt, A, a);", CACHED),
    ("cached pair read in the wrong order (scan)", "lpw[t] = cached_logp[2 * s];", "lpw[t] = cached_logp[2 * s + 1];", CACHED),
]


@pytest.fixture(scope="module")
def source():
    with open(SRC) as f:
        return f.read()


@pytest.mark.parametrize("mi", range(len(MUTATIONS)), ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_a_pin(source, tmp_path, mi):
    what, old, new, pins = MUTATIONS[mi]
    assert source.count(old) == 1, f"'{old}' must occur exactly once in the oracle's source"
    c_file, so_file = tmp_path / "mutant.c", tmp_path / "mutant.so"
    c_file.write_text(source.replace(old, new))
    subprocess.run(["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-w", "-o", str(so_file), str(c_file), "-lm"], check=True)
    env = dict(os.environ, ORACLE_LIB_OVERRIDE=str(so_file))
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"]
                         + [os.path.join(HERE, p) for p in pins], env=env, cwd=ROOT, capture_output=True, text=True)
    assert run.returncode == 1 and " failed" in run.stdout, f"no pin noticed: {what}\n{run.stdout[-600:]}"


def test_the_untouched_source_passes_the_same_way(source, tmp_path):
    """The harness itself: a copy without a planted mistake, loaded the same way, passes every pin file."""
    c_file, so_file = tmp_path / "copy.c", tmp_path / "copy.so"
    c_file.write_text(source)
    subprocess.run(["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-w", "-o", str(so_file), str(c_file), "-lm"], check=True)
    env = dict(os.environ, ORACLE_LIB_OVERRIDE=str(so_file))
    pins = sorted({p for m in MUTATIONS for p in m[3]})
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu"]
                         + [os.path.join(HERE, p) for p in pins], env=env, cwd=ROOT, capture_output=True, text=True)
    assert run.returncode == 0, run.stdout[-800:]


# ---- the ring's bookkeeping oracle (plain Python): the same game, in-process ----------------------

RING_SRC = os.path.join(ROOT, "oracle", "buffer.py")
# (Not in the list: taking the search for an empty slot out of insert.  Items retire in the order they were
# inserted, so the live slots form one arc of the ring and the write cursor, which follows its newest end,
# stands on an empty slot whenever there is one: on every reachable state that search finds its slot at once.)
RING_MUTATIONS = [
    ("an item lives for K + 1 traversals", "if self.count[s] == self.K:", "if self.count[s] == self.K + 1:"),
    ("a discarded item's place is free before its gradient step", "self.count[s] = DISCARDED", "self.count[s] = EMPTY"),
    ("release frees nothing", "                self.count[s] = EMPTY\n", "                pass\n"),
    ("the next sample does not release", "        self.release()                            # the previous", "        pass  # the previous"),
    ("the target period counts trajectories, not batches", "return (num_slots // B) * K", "return num_slots * K"),
    ("the target update is due one step late", "return self.t % t_target == 0", "return self.t % t_target == 1"),
    ("the step counter stands still", "        self.t += 1\n", ""),
    ("missing_targets lists the items that have one", "if not self.has_target[s]]", "if self.has_target[s]]"),
    ("a fresh item inherits its place's target flag", "            self.has_target[self.w] = with_target\n", ""),
    ("the count returned includes this traversal", "counts.append(self.count[s])", "counts.append(self.count[s] + 1)"),
    ("sample does not skip empty slots", "while self.count[self.r] < 0:", "while False:"),
    ("the read cursor stays where it is", "            self.r = (self.r + 1) % self.N\n        return slots, counts", "        return slots, counts"),
    ("an insert that fits exactly is refused", "if self.num_empty() < n:", "if self.num_empty() <= n:"),
    ("a fresh item starts at count one", "self.count[self.w] = 0", "self.count[self.w] = 1"),
]


def _ring_pins(monkeypatch, module):
    import test_oracle_buffer as pins
    for name in ("RingOracle", "BufferOracle", "BufferFull", "NotEnoughLive", "target_period"):
        monkeypatch.setattr(pins, name, getattr(module, name))
    for N, K in [(1, 1), (3, 1), (4, 2), (5, 3), (8, 3)]:
        pins.test_every_item_is_replayed_exactly_K_times_in_order(N, K)
    pins.test_full_ring_without_inserts_is_K_passes_of_the_same_minibatches()
    pins.test_fifo_and_replacement_after_discard()
    pins.test_target_update_every_N_K_steps_is_ppo_s_schedule()
    pins.test_items_inserted_with_their_target_output_need_none()
    pins.test_bad_arguments()


def _ring_module(source, name):
    import types
    module = types.ModuleType("oracle." + name)
    module.__file__ = RING_SRC
    module.__package__ = "oracle"                  # its relative import of the bf16 rounding resolves as in the original
    exec(compile(source, RING_SRC, "exec"), module.__dict__)
    return module


@pytest.mark.timeout(60)
@pytest.mark.parametrize("mi", range(len(RING_MUTATIONS)), ids=[m[0] for m in RING_MUTATIONS])
def test_a_planted_mistake_in_the_ring_fails_a_pin(monkeypatch, mi):
    what, old, new = RING_MUTATIONS[mi]
    with open(RING_SRC) as f:
        source = f.read()
    assert source.count(old) == 1, f"'{old}' must occur exactly once in the ring oracle"
    with pytest.raises((AssertionError, KeyError, IndexError, pytest.fail.Exception)):
        _ring_pins(monkeypatch, _ring_module(source.replace(old, new), "ring_mutant"))


def test_the_untouched_ring_passes_the_same_way(monkeypatch):
    with open(RING_SRC) as f:
        _ring_pins(monkeypatch, _ring_module(f.read(), "ring_copy"))
