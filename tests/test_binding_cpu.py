"""The binding refuses tensors whose element type or shape is not what the call reads or writes, before the
library sees an address (the C side gets pointers only; a kernel would run outside the allocation).  No GPU:
every call here must fail in the binding."""
import pytest
import torch

from paper_1912_00167_amd import binding


def _src(T, n, W, A, gaussian, action_dtype):
    return dict(worker=torch.zeros(T, n, W), target=torch.zeros(T, n, W),
                actions=torch.zeros((T, n, A) if gaussian else (T, n), dtype=action_dtype),
                rewards=torch.zeros(T, n), dones=torch.zeros(T, n, dtype=torch.uint8))


def test_insert_refuses_wrong_element_types_and_shapes():
    T, A, N = 6, 3, 8
    buf = binding.Buffer("gaussian", T, A, N, 2, "bf16", device="cpu")        # (a handle needs no GPU; nothing is launched)
    good = _src(T, 4, 2 * A, A, True, torch.float32)
    for key, bad in (("actions", good["actions"].to(torch.bfloat16)),     # insert takes fp32 and rounds itself
                     ("worker", good["worker"].to(torch.float64)),
                     ("dones", good["dones"].to(torch.bool)),
                     ("rewards", good["rewards"].to(torch.float16))):
        with pytest.raises(TypeError, match=key):
            binding.impact_buffer_insert(buf, dict(good, **{key: bad}))
    for key, bad in (("actions", torch.zeros(T, 4)), ("target", torch.zeros(T, 4, A)), ("rewards", torch.zeros(T, 5)),
                     ("dones", torch.zeros(T + 1, 4, dtype=torch.uint8))):
        with pytest.raises(ValueError, match=key):
            binding.impact_buffer_insert(buf, dict(good, **{key: bad}))
    with pytest.raises(ValueError, match="target"):
        binding.impact_buffer_put_target(buf, [0, 1], torch.zeros(T, 3, 2 * A))
    assert binding.impact_buffer_num_live(buf) == 0                            # none of them reached the library
    buf.close()

    cat = binding.Buffer("categorical", T, A, N, 2, "f32", device="cpu", flags=binding.IMPACT_BUFFER_ACTIONS_U8)
    with pytest.raises(TypeError, match="actions"):
        binding.impact_buffer_insert(cat, _src(T, 4, A, A, False, torch.int32))
    cat.close()
    cat = binding.Buffer("categorical", T, A, N, 2, "f32", device="cpu")
    with pytest.raises(TypeError, match="actions"):
        binding.impact_buffer_insert(cat, _src(T, 4, A, A, False, torch.int64))
    cat.close()


def test_loss_calls_refuse_wrong_element_types_and_shapes():
    T, B, A = 5, 8, 4
    cfg = binding.make_config()
    learner, values, boot = torch.zeros(T, B, A), torch.zeros(T, B), torch.zeros(B)
    batch = dict(worker=torch.zeros(T, B, A), target=torch.zeros(T, B, A), actions=torch.zeros(T, B, dtype=torch.int32),
                 rewards=torch.zeros(T, B), dones=torch.zeros(T, B, dtype=torch.uint8))
    out = binding.alloc_loss_out(T, B, A, device="cpu")
    ws = torch.zeros(1 << 16, dtype=torch.uint8)
    call = lambda **kw: binding.impact_loss_fwd_bwd("categorical", kw.get("learner", learner), kw.get("values", values),
                                                    kw.get("bootstrap", boot), kw.get("batch", batch), kw.get("cfg", cfg),
                                                    out=kw.get("out", out), workspace=ws)
    with pytest.raises(ValueError, match="values"):
        call(values=torch.zeros(B, T))
    with pytest.raises(ValueError, match="bootstrap"):
        call(bootstrap=torch.zeros(B, 1))
    with pytest.raises(TypeError, match="learner"):
        call(learner=learner.to(torch.float16))
    with pytest.raises(TypeError, match="actions"):
        call(batch=dict(batch, actions=batch["actions"].to(torch.uint8)))      # bytes need IMPACT_FLAG_ACTIONS_U8
    with pytest.raises(TypeError, match="actions"):
        call(batch=batch, cfg=binding.make_config(flags=binding.IMPACT_FLAG_ACTIONS_U8))
    with pytest.raises(TypeError, match="worker"):
        call(batch=dict(batch, worker=batch["worker"].to(torch.bfloat16)))     # one float type per batch: that of the rewards
    with pytest.raises(ValueError, match="grad_dist"):
        call(out=dict(out, grad_dist=torch.zeros(T, B, A + 1)))
    with pytest.raises(ValueError, match="vs"):
        call(out=dict(out, vs=torch.zeros(T * B)))
    # batch-major learner side: [B][T]
    bm = binding.make_config(flags=binding.IMPACT_FLAG_BATCH_MAJOR)
    with pytest.raises(ValueError, match="values"):
        binding.impact_loss_fwd_bwd("categorical", torch.zeros(B, T, A), values, boot, batch, bm,
                                    out=binding.alloc_loss_out(B, T, A, device="cpu"), workspace=ws)

    buf = binding.Buffer("categorical", T, A, 16, 2, "f32", device="cpu")
    slots = torch.zeros(B, dtype=torch.int32)
    with pytest.raises(ValueError, match="learner"):                           # another trajectory length than the buffer's
        binding.impact_loss_fwd_bwd_from_buffer(buf, slots, torch.zeros(T + 1, B, A), torch.zeros(T + 1, B), boot, cfg,
                                                out=binding.alloc_loss_out(T + 1, B, A, device="cpu"), workspace=ws)
    with pytest.raises(TypeError, match="slots"):
        binding.impact_loss_fwd_bwd_from_buffer(buf, slots.to(torch.int64), learner, values, boot, cfg, out=out, workspace=ws)
    with pytest.raises(ValueError, match="slots"):
        binding.impact_loss_fwd_bwd_from_buffer(buf, slots[:-1], learner, values, boot, cfg, out=out, workspace=ws)
    with pytest.raises(TypeError, match="actions"):
        binding.impact_buffer_gather(buf, slots, dict(batch, actions=torch.zeros(T, B, dtype=torch.uint8)))
    buf.close()
