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
def test_levels_longer_than_a_16_bit_counter():
    # the one-sweep form counts in 16 bits; a level of 65,536 columns or more wraps its counter
    # (into its neighbour when it sits in the low half of a word, into nothing in the high half)
    # and the row must be recognised and recounted in 32 bits.  65,535 still fits.
    V = 200_000
    g = torch.Generator(device=DEV).manual_seed(45)
    even, odd = 0.5, 0.50390625                        # bf16 patterns 0x3F00 and 0x3F01: one LDS word
    base = (torch.randn((6, V), generator=g, device=DEV) * 0.05 - 2.0)
    runs = [(65_536, even, 0, odd), (65_536, odd, 0, even), (65_535, even, 65_535, odd),
            (70_000, odd, 3, even), (131_072, even, 1, odd), (65_537, odd, 65_536, even)]
    for r, (n_a, v_a, n_b, v_b) in enumerate(runs):
        perm = torch.randperm(V, generator=g, device=DEV)
        base[r, perm[:n_a]] = v_a
        base[r, perm[n_a:n_a + n_b]] = v_b
    lg = base.to(torch.bfloat16)
    for k, p in [(0, 0.9), (1000, 1.0), (0, 0.2), (100_000, 0.999), (300, 0.5)]:
        check(lg, None, 1.0, k, p, 21, 5, f"long levels k={k} p={p}")


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
    assert call(dtype=0, k=0) == -5       # fp32 rows are served for 1 <= top_k <= 256 only
    assert call(dtype=0, k=257) == -5
    assert call(dtype=7) == -3
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


# ---------------------------------------------------------------- fp32 rows and the selection path
# top_k <= 256 is served by selection (chunk maxima, a lower bound from the thread maxima, an
# exact radix select) for bf16 and fp32 rows alike; larger k and top-p alone need the bf16 histogram.
@pytest.mark.gpu
@pytest.mark.parametrize("k,p", [(50, 1.0), (50, 0.95), (1, 1.0), (256, 0.9), (3, 0.5), (200, 1e-4)])
def test_fp32_decode_rows_full_vocab(k, p):
    w = wl.decode_step(DEV, seed=2, prompts=8, rollouts=8)
    lg = w.logits.float() + 1e-3 * torch.randn(w.logits.shape, device=DEV,
                                               generator=torch.Generator(device=DEV).manual_seed(k))
    check(lg, w.tau_rows, 1.0, k, p, seed=19, row_base=1 << 35, label=f"fp32 decode k={k} p={p}")


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("V", [1, 3, 4, 5, 8, 9, 1000, 4096, 8200 + 4, 70_001 + 7, 300_000])
def test_selection_shapes_and_tails(V, dtype):
    g = torch.Generator(device=DEV).manual_seed(V + 1)
    per = 8 if dtype == torch.bfloat16 else 4
    pitch = -(-V // per) * per
    lg = (torch.randn((5, pitch), generator=g, device=DEV) * 2.5).to(dtype)[:, :V]
    for k, p in ((7, 0.9), (1, 1.0), (256, 1.0), (64, 0.3)):
        check(lg, None, 0.8, k, p, V, 3, f"select V={V} {dtype} k={k} p={p}")


@pytest.mark.gpu
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_selection_repeated_values_plateaus_and_signed_zeros(dtype):
    g = torch.Generator(device=DEV).manual_seed(9)
    vals = torch.tensor([3.0, 2.5, 2.5, 1.0, 0.0, -0.0, -1.0, -1.0, -4.0], device=DEV)
    idx = torch.randint(0, vals.numel(), (12, 5000), generator=g, device=DEV)
    lg = vals[idx].to(dtype)
    for k, p in [(1, 1.0), (10, 1.0), (200, 0.9), (256, 0.999), (256, 0.2)]:
        check(lg, None, 1.2, k, p, 3, 77, f"select repeated {dtype} k={k} p={p}")
    # zeros of both signs around the cut: +0 ranks above -0
    z = torch.zeros((6, 3000), device=DEV)
    z[:, ::3] = -0.0
    z[:, 5::7] = 0.5
    z[:, 1::11] = -0.25
    check(z.to(dtype), None, 0.9, 256, 1.0, 4, 5, f"select zeros {dtype}")
    check(z.to(dtype), None, 0.9, 255, 0.95, 4, 5, f"select zeros {dtype} p")
    # one level holds the whole row: the cut level is a plateau, its pos-th column is counted out
    same = torch.full((4, 2048), 0.5, device=DEV).to(dtype)
    r = check(same, None, 1.0, 5, 0.3, 1, 0, f"select all equal {dtype}")
    assert (r.kept == 2048).all()
    # the same inside a short candidate list: nothing above the cut level, 200 columns on it
    same_small = torch.full((4, 200), 0.5, device=DEV).to(dtype)
    r = check(same_small, None, 1.0, 5, 0.3, 1, 0, f"select all equal, short row {dtype}")
    assert (r.kept == 200).all()
    wide = torch.full((2, 40_000), -1.5, device=DEV)
    wide[:, 17] = 2.0
    r = check(wide.to(dtype), None, 1.0, 3, 1.0, 2, 0, f"select plateau under one peak {dtype}")
    assert (r.kept == 40_000).all()
    # a cut level of 150 equal columns under ten larger ones, the rest far below: a short candidate
    # list whose cut level is longer than the 64 columns that are listed apart; the level holds
    # most of the mass, so most rows draw from it
    lvl = torch.full((24, 3000), -20.0, device=DEV) - torch.rand((24, 3000), generator=g, device=DEV)
    for r in range(24):
        perm = torch.randperm(3000, generator=g, device=DEV)
        lvl[r, perm[:150]] = 0.5
        lvl[r, perm[150:160]] = 0.75 + 0.125 * torch.arange(10, device=DEV)
    for k, p in [(20, 1.0), (20, 0.999), (64, 1.0), (11, 0.9)]:
        r = check(lvl.to(dtype), None, 1.0, k, p, 12, 0, f"select long cut level {dtype} k={k} p={p}")
        assert (r.kept == 160).all()
    # rows without a non-negative value, and values down in the subnormals
    neg = (torch.randn((6, 9000), generator=g, device=DEV) * 3 - 40.0).to(dtype)
    check(neg, None, 1.0, 40, 0.9, 6, 0, f"select all negative {dtype}")
    tiny = (torch.randn((4, 3000), generator=g, device=DEV) * 1e-39).to(dtype)
    check(tiny, None, 1.0, 9, 1.0, 6, 0, f"select subnormal {dtype}")


@pytest.mark.gpu
def test_selection_on_sorted_and_blocky_rows():
    # adversarial for the lower bound: the largest values sit next to each other (one chunk holds
    # many kept columns) or are spread so that single threads hold several of them
    V = 151_936
    asc = torch.arange(V, device=DEV, dtype=torch.float32) * 1e-4
    rows = torch.stack([asc, asc.flip(0), torch.roll(asc, 12345), (asc % 7.0) + (asc > 15.0) * 3.0])
    for dtype in (torch.float32, torch.bfloat16):
        for k in (1, 17, 256):
            check(rows.to(dtype), None, 0.5, k, 0.97, 8, 9, f"select sorted {dtype} k={k}")


@pytest.mark.gpu
def test_selection_widest_row():
    V = 1_040_384
    g = torch.Generator(device=DEV).manual_seed(45)
    lg = (torch.randn((2, V), generator=g, device=DEV) * 2.5)
    check(lg, None, 0.9, 50, 0.95, 8, 1, "select widest fp32")
    check(lg.to(torch.bfloat16), None, 0.9, 256, 0.95, 8, 1, "select widest bf16")
    same = torch.full((1, V), -1.5, device=DEV)
    r = check(same, None, 1.0, 3, 0.5, 2, 0, "select widest fp32, all equal")
    assert (r.kept == V).all()


def _random_select_cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        V = int(rng.choice([rng.integers(1, 100), rng.integers(100, 9000), rng.integers(9000, 60_000)]))
        rows = int(rng.integers(1, 10))
        k = int(rng.choice([1, 2, rng.integers(3, 257), 256]))
        p = float(rng.choice([1.0, 0.999, 0.9, 0.5, 0.1, 1e-4]))
        out.append((i, V, rows, k, p, float(rng.choice([0.1, 1.0, 4.0, 60.0])), float(rng.choice([0.3, 3.0, 10.0])),
                    float(rng.choice([0.0, 0.0, -8.0, 8.0])), bool(rng.integers(0, 2))))
    return out


@pytest.mark.gpu
@pytest.mark.parametrize("i,V,rows,k,p,tau,sigma,shift,coarse", _random_select_cases(40, 78))
def test_seeded_random_fp32_settings(i, V, rows, k, p, tau, sigma, shift, coarse):
    g = torch.Generator(device=DEV).manual_seed(900 + i)
    pitch = -(-V // 4) * 4 + 4 * (i % 2)
    lg = (torch.randn((rows, pitch), generator=g, device=DEV) * sigma + shift)
    if coarse:                                     # few distinct values: levels with many columns
        lg = torch.round(lg * 4) / 4
    lg = lg[:, :V]
    tau_rows = None if i % 2 else (tau * (0.5 + torch.rand(rows, generator=g, device=DEV))).float()
    check(lg, tau_rows, tau, k, p, seed=i, row_base=i << 21, label=f"fp32 case {i}: {rows}x{V} k={k} p={p} tau={tau}")


@pytest.mark.gpu
def test_fp32_rows_need_a_small_top_k():
    lg = torch.zeros((2, 64), device=DEV)
    for k in (0, 257, 1000):
        with pytest.raises(e3.E3Error) as ei:
            e3.e3_sample_restricted(lg, None, 1.0, k, 0.9, 1, 0)
        assert ei.value.status == -5
