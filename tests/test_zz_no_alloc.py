"""The entry point that allocates nothing, moe_layer_step_noalloc, against moe_layer_step: same decisions, same
traces, bit-identical outputs, on two calls in a row of which the second has the smaller input -- and the oracle's
bound on the block output, read through x_out.  Its kernels keep their intermediate results in a fixed array inside
the library instead of the context's arena; the array keeps the previous call's contents, so the second, smaller
call would show anything that was left behind and not cleared."""
import numpy as np
import pytest
import torch

import workload as W
from oracle import moe_oracle as O
from paper_2312_17238_amd import binding as B

from harness import Model, check_x_out, oracle_routing, oracle_y

pytestmark = pytest.mark.gpu


def step_both(ref: Model, sut: Model, l: int, x: torch.Tensor, tag: str):
    """One step of layer l through both entry points on twin models; returns the checked output."""
    dev = ref.stack.device
    Bn, H = x.shape
    xd = x.to(dev)
    outs, hs, trs = [], [], []
    for model, fn in ((ref, B.moe_layer_step), (sut, B.moe_layer_step_noalloc)):
        out = torch.empty_like(xd)
        h = torch.empty_like(xd)
        tr = B.StepTrace()
        nxt = model.stack.layers[l + 1] if l + 1 < model.L else None
        fn(model.stack.layers[l], nxt, xd.data_ptr(), Bn, out.data_ptr(), h.data_ptr(), tr)
        model.stack.synchronize()
        outs.append(out.cpu().numpy()); hs.append(h.cpu().numpy()); trs.append(tr)
    assert trs[0].routing() == trs[1].routing(), tag
    assert trs[0].accesses() == trs[1].accesses() and trs[0].guesses() == trs[1].guesses(), tag
    assert trs[0].weights() == trs[1].weights(), tag
    assert (hs[0].view(np.uint16) == hs[1].view(np.uint16)).all(), f"{tag}: gate input differs"
    assert (outs[0].view(np.uint16) == outs[1].view(np.uint16)).all(), f"{tag}: x_out differs"
    # and against the oracle, so that the pair cannot be wrong together
    x_np = x.numpy()
    for b, (h, idx, w, _) in enumerate(oracle_routing(sut, l, x_np)):
        assert trs[1].routing()[b] == idx
        check_x_out(outs[1][b], x_np[b], oracle_y(sut, l, h, idx, w, O.expert_ffn), f"{tag} b={b}")
    return outs[1]


@pytest.mark.parametrize("formats,K,k", [([(4, 64), (4, 64)], 2, 2), ([(3, 64), (2, 16)], 2, 4), ([(4, 64), (4, 64)], 4, 4)])
def test_noalloc_step_matches_step_on_two_calls_in_a_row(formats, K, k):
    L, H, F, E = 2, 512, 1024, 8
    ref = Model(L, H, F, E, K, formats, k, 2, 1e-5, max_batch=4, seed=101)
    sut = Model(L, H, F, E, K, formats, k, 2, 1e-5, max_batch=4, seed=101, keep_layers=[])
    # the entry point that allocates nothing runs the GEMV kernels whatever the batch; so does the reference here
    B.moe_ctx_set_option(ref.stack.ctx, "mfma_min_batch", 1000)
    xs = W.hidden_ar1(101, 6, 4, H)
    # first call: four tokens (the general kernels, several tokens per expert); second call: one token (the
    # single-token kernels) -- a smaller input over the scratch the first call left behind; then on through layer 1
    # and a few more alternations
    for t, Bn in enumerate((4, 1, 3, 1, 2, 4)):
        x = xs[t, :Bn].contiguous()
        y0 = step_both(ref, sut, 0, x, f"t={t} layer 0 batch {Bn}")
        step_both(ref, sut, 1, torch.from_numpy(y0), f"t={t} layer 1 batch {Bn}")
    a, b = ref.stack.total_stats(), sut.stack.total_stats()
    assert a == b and a["steps_device_routed"] == 0
    ref.close(); sut.close()


def test_noalloc_step_rejects_what_does_not_fit():
    H, F = 256, 512
    model = Model(1, H, F, 8, 2, None, 2, 0, 0.0, max_batch=8, seed=103, keep_layers=[])
    dev = model.stack.device
    x = torch.zeros(8, H, dtype=torch.float16, device=dev)
    out = torch.empty_like(x)
    with pytest.raises(B.MoeError) as e:
        B.moe_layer_step_noalloc(model.stack.layers[0], None, x.data_ptr(), 5, out.data_ptr(), None, None)
    assert e.value.code == B.MOE_EINVAL and "exceed" in str(e.value)
    B.moe_ctx_profile_enable(model.stack.ctx, True)
    with pytest.raises(B.MoeError) as e:
        B.moe_layer_step_noalloc(model.stack.layers[0], None, x.data_ptr(), 1, out.data_ptr(), None, None)
    assert e.value.code == B.MOE_ESTATE
    B.moe_ctx_profile_enable(model.stack.ctx, False)
    B.moe_layer_step_noalloc(model.stack.layers[0], None, x.data_ptr(), 4, out.data_ptr(), None, None)
    model.stack.synchronize()
    assert (out[:4].cpu().numpy() == 0).all()      # zero input: y = 0
    model.close()
