"""Caller-supplied gradients: a torch.nn.Module trained by the library's events (GPU only)."""
import numpy as np
import pytest

from paper_1710_06952_amd.studies import torch_model as T


def test_flat_module_views_round_trip():
    import torch
    flat = T.FlatModule(T.build_module(8, 16, 3))
    x = torch.from_numpy(flat.flatten_initial())
    assert x.numel() == flat.d == 8 * 16 + 16 + 16 + 16 + 16 * 3 + 3
    parts = flat.unflatten(x)
    for name, p in flat.module.named_parameters():
        assert torch.equal(parts[name], p.detach())
    out = torch.zeros(flat.d)
    inputs, labels = torch.randn(5, 8), torch.tensor([0, 1, 2, 1, 0])
    loss = flat.loss_and_gradient(x, inputs, labels, out)
    ref = torch.nn.functional.cross_entropy(flat.module(inputs), labels)
    ref.backward()
    want = torch.cat([p.grad.reshape(-1) for p in flat.module.parameters()])
    assert torch.allclose(loss, ref) and torch.allclose(out, want, atol=1e-7)


@pytest.mark.gpu
def test_a_torch_module_trains_under_the_library_events():
    res = T.run_study(n=6, dims=(16, 32, 4), rows=512, M=32, epochs=3, T_max=3, gamma=0.05, seed=1)
    assert res["events"] == 3 * 6 * 512 // 32 and res["rounds"] < res["events"]
    assert res["loss"][-1] < 0.5 * res["loss"][0] and res["error"][-1] < 0.6 * res["error"][0]
    assert np.isfinite(res["loss"]).all() and 0 < res["consensus_distance"] < 1.0
    assert "epoch" in T.format_table(res)
