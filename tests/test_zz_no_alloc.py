"""aura_material_scores_static (the entry point that allocates nothing) against aura_material_scores: the same kernels
on a scratch array inside the library instead of a caller's workspace, so the same bits.  Two calls in a row, the second
with a smaller input, so that what the first call left in the shared array would show if the second read any of it."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _case(rng, N, D, K, P):
    f = rng.standard_normal((N, D)); f /= np.linalg.norm(f, axis=1, keepdims=True)
    t = rng.standard_normal((K, D)); t /= np.linalg.norm(t, axis=1, keepdims=True)
    y = rng.uniform(100, 8000, (K, P))
    return f.astype(np.float32), t.astype(np.float32), y.astype(np.float32)


def test_static_scratch_call_matches_the_workspace_call_twice_in_a_row(orc):
    import paper_2511_03126_amd as aura
    from paper_2511_03126_amd import binding
    assert torch.cuda.is_available()
    dev = "cuda:0"
    rng = np.random.default_rng(2024)
    par = aura.Params(temperature=0.1)
    # the largest shape the fixed array takes (1536 channels, 128 materials: 768 KiB of the 1 MiB), then a smaller
    # one in every dimension, then the first again
    for N, D, K, P in [(5000, 1536, 128, 2), (777, 100, 5, 1), (5000, 1536, 128, 2)]:
        f, t, y = _case(rng, N, D, K, P)
        fd, td, yd = (torch.from_numpy(a).to(dev) for a in (f, t, y))
        out = {}
        for name in ("workspace", "static"):
            scores = torch.full((N, K), float("nan"), device=dev)
            prop = torch.full((N, P), float("nan"), device=dev)
            label = torch.full((N,), -7, dtype=torch.int32, device=dev)
            if name == "workspace":
                ws = torch.empty(aura.workspace_bytes(binding.CALL_MATERIAL_SCORES, D=D, K=K), dtype=torch.uint8, device=dev)
                aura.material_scores(fd, td, yd, par, scores, prop, label, ws)
            else:
                before = torch.cuda.memory_allocated()
                aura.material_scores_static(fd, td, yd, par, scores, prop, label)
                assert torch.cuda.memory_allocated() == before
            torch.cuda.synchronize()
            out[name] = (scores.cpu().numpy(), prop.cpu().numpy(), label.cpu().numpy())
        for a, b in zip(out["workspace"], out["static"]):
            assert np.array_equal(a.view(np.uint8), b.view(np.uint8))
        # and both against the oracle, to the bar of the scoring call
        ref = orc.material_scores(f.astype(np.float64), t, y, T=0.1)
        s, p, l = out["static"]
        assert np.abs(s - ref["scores"]).max() <= 1e-5
        assert (np.abs(p - ref["prop"]) / np.abs(y).max(0)).max() <= 1e-4
        assert not ((l != ref["label"]) & (ref["margin"] > 2e-4)).any()
