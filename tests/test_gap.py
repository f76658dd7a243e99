"""Measured logit gap (Appendix A's Delta) and the gap form of the temperature update:
library against oracle."""
import math

import numpy as np
import pytest
import torch

import paper_2505_18573_amd as e3
from oracle import e3_oracle as o
from paper_2505_18573_amd import workloads as wl

V_Q = 151_936


def test_update_gap_matches_oracle_on_host():
    rng = np.random.default_rng(0)
    for _ in range(300):
        tau, Ht, H0 = rng.uniform(0.3, 2.0), rng.uniform(0.05, 2.0), rng.uniform(0.05, 2.0)
        gap = float(rng.choice([0.0, -1.0, 0.5, 5.0, 14.4, 30.0]))
        t, ta, tm = int(rng.integers(0, 600)), int(rng.choice([-1, 288])), 480
        eta = float(rng.choice([0.0, 0.9, 1.0]))
        rc, want, want_t = o.temperature_update_gap(tau, Ht, H0, gap, t, ta, tm, eta)
        if rc == 0:
            got, got_t = e3.e3_temperature_update_gap(tau, Ht, H0, gap, t, ta, tm, eta)
            assert got == pytest.approx(want, rel=1e-14) and got_t == pytest.approx(want_t, rel=1e-14)
        else:
            with pytest.raises(e3.E3Error):
                e3.e3_temperature_update_gap(tau, Ht, H0, gap, t, ta, tm, eta)
    D = math.log(V_Q) + math.log(math.log(V_Q))
    assert e3.e3_temperature_update_gap(1.2, 0.3, 0.33, D)[0] == pytest.approx(
        e3.e3_temperature_update(1.2, 0.3, 0.33, V_Q)[0], rel=1e-15)


def _close(x, ref, rel=1e-4, floor=1e-6):
    return np.abs(np.asarray(x, np.float64) - ref) <= rel * np.maximum(np.abs(ref), floor)


@pytest.mark.gpu
def test_gap_parity_on_gpu():
    dev = "cuda:0"
    # two-level rows: the measured gap is Delta itself
    deltas = [3.0, 10.0, 15.0, 16.0, 17.0, 24.0]
    lg = wl.delta_model_rows(dev, deltas, V=V_Q, dtype=torch.float32)
    _, ent, gap, hs, gs, cnt = e3.e3_logprob_entropy_gap(lg, None, None, None, 0.8)
    assert np.allclose(gap.cpu().numpy(), deltas, rtol=1e-5)
    # general rows, per-row tau, mask, several shapes incl. ragged tails and fp32 / bf16
    g = torch.Generator(device=dev).manual_seed(5)
    for rows, V, dtype in ((9, 1000, torch.float32), (6, 20_003, torch.bfloat16), (12, V_Q, torch.bfloat16)):
        pitch = -(-V // 8) * 8
        x = ((torch.randn((rows, pitch), generator=g, device=dev) * 3).to(dtype))[:, :V]
        tau = (0.6 + 0.8 * torch.rand(rows, generator=g, device=dev)).float()
        mask = (torch.rand(rows, generator=g, device=dev) < 0.7).to(torch.uint8)
        tgt = torch.randint(0, V, (rows,), generator=g, device=dev).to(torch.int32)
        logp, ent, gap, hs, gs, cnt = e3.e3_logprob_entropy_gap(x, tgt, mask, tau, 1.0)
        want = o.logit_gaps(wl.host_bits(x), tau.cpu().numpy(), 1.0)
        assert _close(gap.cpu().numpy(), want).all()
        ref = o.logprob_entropy(wl.host_bits(x), tgt.cpu().numpy(), mask.cpu().numpy(), tau.cpu().numpy(), 1.0)
        assert _close(ent.cpu().numpy(), ref.entropy).all() and _close(logp.cpu().numpy(), ref.logp).all()
        keep = mask.bool()
        assert cnt.item() == int(keep.sum())
        assert gs.item() == pytest.approx(gap.double()[keep].sum().item(), rel=1e-12)
        assert hs.item() == pytest.approx(ref.entropy_sum, rel=1e-6)
    # a scheduler step driven by the measured batch-mean gap
    w = wl.training_pass(dev, rows=256)
    _, ent, gap, hs, gs, cnt = e3.e3_logprob_entropy_gap(w.logits, w.target_ids, None, None, 1.0)
    H_t, gap_t = hs.item() / cnt.item(), gs.item() / cnt.item()
    want_gap = o.logit_gaps(wl.host_bits(w.logits), None, 1.0).mean()
    assert gap_t == pytest.approx(want_gap, rel=1e-5)
    tau1, _ = e3.e3_temperature_update_gap(1.0, H_t, 1.05 * H_t, gap_t)
    assert tau1 == pytest.approx(1 + math.log(1.05) / want_gap, rel=1e-5)
    # one-column rows have no rest
    one = torch.zeros((3, 8), device=dev)[:, :1]
    _, _, gap1, _, _, _ = e3.e3_logprob_entropy_gap(one, None, None, None, 1.0)
    assert torch.isnan(gap1).all()
