"""Parity of e3_sample_restricted (top-k / top-p sampling) with the CPU oracle.

Bars: kept counts identical except on rows the oracle flags near_cut (top-p target
within 1e-9 relative of a cumulative level mass); tokens identical except on near_cut
or near_tie rows (two best race scores within 1e-5 relative); logp within 1e-4
relative (it is evaluated in fp64 and stored as fp32).
"""
import numpy as np
import pytest
import torch
from scipy import stats

import paper_2505_18573_amd as e3
from oracle import e3_oracle as o
from paper_2505_18573_amd import workloads as wl

DEV = "cuda:0"
NT = 16


def check(logits, tau_rows, tau_scalar, k, p, seed, row_base, label):
    tok, logp, kept = e3.e3_sample_restricted(logits, tau_rows, tau_scalar, k, p, seed, row_base)
    torch.cuda.synchronize()
    ref = o.sample_restricted(wl.host_bits(logits), None if tau_rows is None else tau_rows.cpu().numpy(),
                              tau_scalar, k, p, seed, row_base, nthreads=NT)
    tok, logp, kept = tok.cpu().numpy(), logp.cpu().numpy(), kept.cpu().numpy()
    V = logits.shape[1]
    assert ((tok >= 0) & (tok < V)).all()
    cut_ok = ref.near_cut == 0
    bad_kept = (kept != ref.kept) & cut_ok
    assert not bad_kept.any(), f"{label}: kept differs on rows {np.flatnonzero(bad_kept)[:8]}: " \
                               f"{kept[bad_kept][:8]} vs {ref.kept[bad_kept][:8]}"
    exempt = (ref.near_cut != 0) | (ref.near_tie != 0)
    bad_tok = (tok != ref.token) & ~exempt
    print(f"[{label}] rows={tok.size} near_cut={int(ref.near_cut.sum())} near_tie={int(ref.near_tie.sum())} "
          f"token mismatches={int((tok != ref.token).sum())} kept range {kept.min()}..{kept.max()}")
    assert not bad_tok.any(), f"{label}: tokens differ on rows {np.flatnonzero(bad_tok)[:8]}"
    same = tok == ref.token
    err = np.abs(logp[same] - ref.logp[same])
    assert (err <= 1e-4 * np.maximum(np.abs(ref.logp[same]), 1e-6)).all(), f"{label}: logp off by {err.max()}"
    return ref


@pytest.mark.gpu
@pytest.mark.parametrize("k,p", [(50, 1.0), (0, 0.9), (50, 0.95), (1, 1.0), (0, 1.0), (3, 0.5)])
def test_decode_rows_full_vocab(k, p):
    w = wl.decode_step(DEV, seed=1, prompts=8, rollouts=8)            # 64 rows x 151,936 bf16
    check(w.logits, w.tau_rows, 1.0, k, p, seed=17, row_base=1000, label=f"decode k={k} p={p}")


@pytest.mark.gpu
def test_cuts_among_negative_values_and_back():
    g = torch.Generator(device=DEV).manual_seed(31)
    lg = (torch.randn((12, 40_000), generator=g, device=DEV) * 3).to(torch.bfloat16)
    tau = (0.6 + 0.8 * torch.rand(12, generator=g, device=DEV)).float()
    # about half of the values are negative: k = 30,000 puts the count cut among them
    check(lg, tau, 1.0, 30_000, 1.0, 5, 0, "k among negatives")
    # ... and the nucleus of that set ends among the non-negative values again (third sweep)
    check(lg, tau, 1.0, 30_000, 0.5, 5, 0, "k among negatives, p back")
    # nucleus that needs negative values: a flat row at a high temperature
    check(lg, None, 50.0, 0, 0.9, 5, 0, "p among negatives")
    check(lg, None, 50.0, 30_000, 0.99, 5, 0, "k and p among negatives")
    # rows without any non-negative value
    neg = (lg.float() - 40.0).to(torch.bfloat16)
    check(neg, tau, 1.0, 40, 0.9, 6, 0, "all negative")
    check(neg, tau, 1.0, 0, 1.0, 6, 0, "all negative, no cut")


@pytest.mark.gpu
@pytest.mark.parametrize("V", [1, 5, 8, 1000, 8200 + 4, 70_001 + 7])
def test_shapes_and_tails(V):
    g = torch.Generator(device=DEV).manual_seed(V)
    pitch = -(-V // 8) * 8
    lg = (torch.randn((9, pitch), generator=g, device=DEV) * 2.5).to(torch.bfloat16)[:, :V]
    check(lg, None, 0.8, 7, 0.9, V, 3, f"V={V}")
    check(lg, None, 0.8, 0, 1.0, V, 3, f"V={V} no cut")


@pytest.mark.gpu
def test_widest_accepted_row():
    V = 1_040_384
    g = torch.Generator(device=DEV).manual_seed(44)
    lg = (torch.randn((2, V), generator=g, device=DEV) * 2.5).to(torch.bfloat16)
    check(lg, None, 0.9, 50, 0.95, 8, 1, "widest row k=50 p=0.95")
    check(lg, None, 0.9, 0, 0.9, 8, 1, "widest row p=0.9")
    same = torch.full((1, V), -1.5, device=DEV).to(torch.bfloat16)     # one level of 1,040,384 columns
    r = check(same, None, 1.0, 3, 0.5, 2, 0, "widest row, all equal")
    assert (r.kept == V).all()


@pytest.mark.gpu
def test_repeated_values_and_signed_zeros():
    # few distinct values: every level holds many columns, cuts fall inside repeated values
    g = torch.Generator(device=DEV).manual_seed(8)
    vals = torch.tensor([3.0, 2.5, 2.5, 1.0, 0.0, -0.0, -1.0, -1.0, -4.0], device=DEV)
    idx = torch.randint(0, vals.numel(), (16, 5000), generator=g, device=DEV)
    lg = vals[idx].to(torch.bfloat16)
    for k, p in [(10, 1.0), (600, 0.9), (0, 0.7), (3000, 1.0), (3000, 0.999), (0, 1.0)]:
        check(lg, None, 1.2, k, p, 3, 77, f"repeated k={k} p={p}")
    same = torch.full((4, 2048), 0.5, device=DEV).to(torch.bfloat16)
    r = check(same, None, 1.0, 5, 0.3, 1, 0, "all equal")
    assert (r.kept == 2048).all()


@pytest.mark.gpu
def test_top_k_exactly_on_a_level_boundary():
    # every row is a permutation of one multiset, so the cumulative level counts are the same
    # in all rows and k can be put exactly on a boundary, one before and one after it
    counts = [(3.0, 1), (2.5, 37), (1.0, 1200), (0.0, 700), (-0.0, 11), (-1.0, 2500), (-4.0, 551)]
    base = torch.cat([torch.full((n,), v) for v, n in counts])
    V = base.numel()
    g = torch.Generator().manual_seed(3)
    lg = torch.stack([base[torch.randperm(V, generator=g)] for _ in range(6)]).to(torch.bfloat16).to(DEV)
    cum = np.cumsum([n for _, n in counts])
    for j in (0, 1, 2, 3, 4, 5):
        for k in (int(cum[j]) - 1, int(cum[j]), int(cum[j]) + 1):
            if k < 1:
                continue
            r = check(lg, None, 0.9, k, 1.0, 5, 40, f"boundary level {j} k={k}")
            want = int(cum[np.searchsorted(cum, k)])          # first cumulative count >= k
            assert (r.kept == want).all(), (j, k, r.kept, want)


@pytest.mark.gpu
def test_frequencies_follow_the_truncated_softmax():
    vals = torch.tensor([[2.0, 1.5, 2.0, 0.5, 1.5, 1.5, -1.0, 0.5, 0.0, -0.0, 3.0, -2.0, -2.0, 1.0, 0.25, -3.0]],
                        device=DEV)
    n = 40_000
    lg = vals.to(torch.bfloat16).expand(n, 16).contiguous()
    tok, logp, kept = e3.e3_sample_restricted(lg, None, 1.1, 9, 0.97, seed=11, row_base=0)
    tok = tok.cpu().numpy()
    ref = o.sample_restricted(wl.host_bits(lg[:1]), None, 1.1, 9, 0.97, 11, 0)
    assert (kept.cpu().numpy() == ref.kept[0]).all()
    v = vals[0].double().cpu().numpy()
    order = np.sort(v)[::-1]
    keep = v >= order[ref.kept[0] - 1]
    pr = np.where(keep, np.exp((v - v.max()) / np.float32(1.1)), 0.0)
    pr /= pr.sum()
    counts = np.bincount(tok, minlength=16)
    assert counts[~keep].sum() == 0
    chi2, pval = stats.chisquare(counts[keep], pr[keep] * n)
    assert pval > 1e-3, (chi2, pval)


@pytest.mark.gpu
def test_rows_do_not_depend_on_batching():
    w = wl.decode_step(DEV, seed=3, prompts=2, rollouts=4, V=20_000)
    a = e3.e3_sample_restricted(w.logits, w.tau_rows, 1.0, 40, 0.9, seed=5, row_base=50)
    b = e3.e3_sample_restricted(w.logits[3:6], w.tau_rows[3:6].contiguous(), 1.0, 40, 0.9, seed=5, row_base=53)
    for x, y in zip(a, b):
        assert torch.equal(x[3:6], y)


def test_argument_checks_need_no_gpu():
    L = e3.lib()
    call = lambda dtype=1, k=5, p=0.9, tok=0x2000, tau=1.0: L.e3_sample_restricted(
        0x1000, dtype, 4, 64, 64, None, tau, k, p, 1, 0, tok, None, None, None)
    assert call(dtype=0) == -3            # fp32 logits: E3_ERR_DTYPE
    assert call(k=-1) == -5
    assert call(p=0.0) == -5 and call(p=float("nan")) == -5 and call(p=-0.5) == -5
    assert call(tau=0.0) == -5
    assert call(tok=None) == -1
    assert L.e3_sample_restricted(None, 1, 0, 64, 64, None, 1.0, 5, 0.9, 1, 0, None, None, None, None) == 0


def _random_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        V = int(rng.choice([rng.integers(1, 100), rng.integers(100, 9000), rng.integers(9000, 60_000)]))
        rows = int(rng.integers(1, 12))
        k = int(rng.choice([0, 1, 2, rng.integers(3, 200), rng.integers(1, V + 2), V // 2 + 1]))
        p = float(rng.choice([1.0, 0.999, 0.9, 0.5, 0.1, 1e-4]))
        out.append((i, V, rows, k, p, float(rng.choice([0.1, 1.0, 4.0, 60.0])), float(rng.choice([0.3, 3.0, 10.0])),
                    float(rng.choice([0.0, 0.0, -8.0, 8.0]))))
    return out


@pytest.mark.gpu
@pytest.mark.parametrize("i,V,rows,k,p,tau,sigma,shift", _random_cases(32, 77))
def test_seeded_random_settings(i, V, rows, k, p, tau, sigma, shift):
    g = torch.Generator(device=DEV).manual_seed(500 + i)
    pitch = -(-V // 8) * 8 + 8 * (i % 2)
    lg = (torch.randn((rows, pitch), generator=g, device=DEV) * sigma + shift).to(torch.bfloat16)[:, :V]
    tau_rows = None if i % 2 else (tau * (0.5 + torch.rand(rows, generator=g, device=DEV))).float()
    check(lg, tau_rows, tau, k, p, seed=i, row_base=i << 20, label=f"case {i}: {rows}x{V} k={k} p={p} tau={tau}")
