"""The C ABI without a GPU: exported symbols, host-side argument checks (they run
before any launch), and the host-only temperature scheduler against the oracle."""
import ctypes as C
import math
import os
import re

import numpy as np
import pytest

import paper_2505_18573_amd as e3
from oracle import e3_oracle as o

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    names = set()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(e3_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported():
    names = _declared_functions()
    assert set(names) >= {"e3_sample_entropy", "e3_logprob_entropy", "e3_grpo_advantages",
                          "e3_temperature_update", "e3_workspace_bytes", "e3_strerror"}
    L = e3.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_partition_constants_are_frozen_and_the_binding_repeats_them():
    # the partition is part of the definition of the sampled token: (8, 64, 8) is frozen
    from tests.partition import LIB_PARTITION
    assert LIB_PARTITION == (8, 64, 8)
    assert (e3.binding.E3_TILE_CHUNK, e3.binding.E3_TILE_LANES, e3.binding.E3_TILE_DEPTH) == LIB_PARTITION


def test_strerror_and_workspace():
    assert e3.e3_strerror(0) == "ok"
    for code in range(-7, 0):
        assert e3.e3_strerror(code) not in ("ok", "unknown status")
    assert e3.e3_strerror(-99) == "unknown status"
    assert e3.e3_workspace_bytes(0, 1) == 0
    # 32 bytes per run of columns, at most one run per super-tile of 4096 columns and 64 per row
    assert e3.e3_workspace_bytes(512, 151_936) == 512 * 38 * 32
    assert e3.e3_workspace_bytes(3, 1024) == 3 * 1 * 32
    assert e3.e3_workspace_bytes(1024, 2_000_000) == 1024 * 64 * 32
    assert e3.e3_workspace_bytes(1025, 151_936) == 0         # large batches need none


def _sample(logits=0x1000, dtype=1, rows=4, V=64, stride=64, tau_rows=None, tau=1.0,
            tok=0x2000, ws=None, ws_bytes=0):
    return e3.lib().e3_sample_entropy(logits, dtype, rows, V, stride, tau_rows, tau, 1, 0,
                                      tok, None, None, ws, ws_bytes, None)


def test_sample_entropy_argument_checks_precede_any_launch():
    # fake non-null addresses: every call below must be rejected on the host
    assert _sample(dtype=7) == -3
    assert _sample(rows=-1) == -2
    assert _sample(V=0) == -2
    assert _sample(stride=63) == -2
    assert _sample(logits=None) == -1
    assert _sample(logits=0x1008) == -4                      # base not 16-byte aligned
    assert _sample(V=60, stride=60, dtype=1) == -4           # 120-byte pitch
    assert _sample(V=60, stride=64, dtype=1, tau=0.0) == -5
    assert _sample(tau=float("nan")) == -5
    assert _sample(tau=-1.0) == -5
    assert _sample(tok=None) == -1
    assert _sample(V=1 << 22, stride=1 << 22) == -2          # too wide for the LDS tables
    assert _sample(rows=0, logits=None, tok=None) == 0       # empty batch is a no-op


def test_noalloc_entry_point_checks_and_row_limit():
    L = e3.lib()
    def call(logits=0x1000, dtype=1, rows=4, V=64, stride=64, tau=1.0, tok=0x2000):
        return L.e3_sample_entropy_noalloc(logits, dtype, rows, V, stride, None, tau, 1, 0, tok, None, None, None)
    assert call(dtype=9) == -3 and call(V=0) == -2 and call(logits=0x1004) == -4 and call(tau=0.0) == -5
    assert call(rows=e3.binding.E3_NOALLOC_MAX_ROWS + 1) == -6        # E3_ERR_WORKSPACE, before any launch
    assert call(rows=0, logits=None, tok=None) == 0
    text = open(os.path.join(ROOT, "include", "e3.h")).read()
    assert int(re.search(r"#define E3_NOALLOC_MAX_ROWS (\d+)", text).group(1)) == e3.binding.E3_NOALLOC_MAX_ROWS
    # what the array must hold for the largest batch it serves
    assert e3.e3_workspace_bytes(e3.binding.E3_NOALLOC_MAX_ROWS, 2_000_000) == 2 * 1024 * 1024


def test_logprob_entropy_argument_checks():
    L = e3.lib()
    def call(logits=0x1000, dtype=0, rows=4, V=64, stride=64, tgt=0x3000, tau=1.0,
             logp=0x4000, ent=0x5000):
        return L.e3_logprob_entropy(logits, dtype, rows, V, stride, tgt, None, None, tau,
                                    logp, ent, None, None, None, 0, None)
    assert call(dtype=2) == -3
    assert call(V=-5) == -2
    assert call(ent=None) == -1
    assert call(tgt=None) == -1                              # logp requested without targets
    assert call(stride=66) == -4                             # 264-byte pitch
    assert call(tau=float("inf")) == -5
    assert call(rows=0, logits=None, ent=None, logp=None, tgt=None) == 0


def test_grpo_argument_checks():
    L = e3.lib()
    assert L.e3_grpo_advantages(0x1000, 0x2000, -1, 0, 0.0, 0x3000, None) == -2
    # the combined call checks both halves before anything is launched
    def both(rows=4, V=64, ent=0x4000, groups=2, ddof=0, eps=0.0, rew=0x5000, off=0x6000, adv=0x7000):
        return L.e3_logprob_entropy_advantages(0x1000, 1, rows, V, 64, None, None, None, 1.0, None, ent,
                                               None, None, rew, off, groups, ddof, eps, adv, None, 0, None)
    assert both(ent=None) == -1 and both(groups=-1) == -2 and both(ddof=2) == -5
    assert both(eps=-1.0) == -5 and both(adv=None) == -1 and both(rew=None) == -1
    assert both(V=0) == -2
    assert both(rows=0, groups=0, rew=None, off=None, adv=None, ent=None) == 0
    assert L.e3_grpo_advantages(0x1000, 0x2000, 4, 2, 0.0, 0x3000, None) == -5
    assert L.e3_grpo_advantages(0x1000, 0x2000, 4, 0, -1.0, 0x3000, None) == -5
    assert L.e3_grpo_advantages(None, 0x2000, 4, 0, 0.0, 0x3000, None) == -1
    assert L.e3_grpo_advantages(0x1000, 0x2000, 4, 0, 0.0, None, None) == -1
    assert L.e3_grpo_advantages(None, None, 0, 0, 0.0, None, None) == 0


def test_temperature_update_matches_oracle():
    rng = np.random.default_rng(0)
    for _ in range(300):
        tau = float(rng.uniform(0.3, 2.0))
        Ht = float(rng.uniform(0.05, 2.0))
        H0 = float(rng.uniform(0.05, 2.0))
        vocab = int(rng.choice([3, 1024, 32000, 151_936]))
        t = int(rng.integers(0, 600))
        ta = int(rng.choice([-1, 0, 288, 480]))
        tm = int(rng.choice([0, 288, 480]))
        eta = float(rng.choice([0.0, 0.5, 0.9, 1.0]))
        rc, want, want_t = o.temperature_update(tau, Ht, H0, vocab, t, ta, tm, eta)
        if rc == 0:
            got, got_t = e3.e3_temperature_update(tau, Ht, H0, vocab, t, ta, tm, eta)
            assert got == pytest.approx(want, rel=1e-14)
            assert got_t == pytest.approx(want_t, rel=1e-14)
        else:
            with pytest.raises(e3.E3Error):
                e3.e3_temperature_update(tau, Ht, H0, vocab, t, ta, tm, eta)


def test_temperature_update_pins_and_errors():
    D = math.log(151_936) + math.log(math.log(151_936))
    assert e3.e3_temperature_update(1.0, 1.0, 1.1, 151_936)[0] == pytest.approx(
        1 + math.log(1.1) / D, abs=1e-15)
    assert e3.e3_temperature_update(0.8, 0.3, 0.3, 151_936) == (0.8, 0.3)     # alpha = 1
    tau, tgt = e3.e3_temperature_update(1.0, 0.3, 0.37, 151_936, t=480, t_anneal=288,
                                        t_max=480, eta=0.9)
    assert tgt == pytest.approx(0.9 * 0.37, abs=1e-15)
    assert e3.e3_temperature_update(1.0, 0.2, 0.4, 151_936, tau_min=0.5, tau_max=1.01)[0] == 1.01
    for bad in (dict(tau_t=0.0), dict(H_t=-1.0), dict(H_init=float("nan")), dict(vocab=2),
                dict(eta=1.5), dict(tau_min=-0.1), dict(tau_min=2.0, tau_max=1.0)):
        kw = dict(tau_t=1.0, H_t=0.2, H_init=0.2, vocab=151_936)
        kw.update(bad)
        with pytest.raises(e3.E3Error) as ei:
            e3.e3_temperature_update(**kw)
        assert ei.value.status == -5
    L = e3.lib()
    assert L.e3_temperature_update(1.0, 0.2, 0.2, 1000, 0, -1, 0, 1.0, 0.0, float("inf"),
                                   None, None) == -1
    out = C.c_double(123.0)
    assert L.e3_temperature_update(0.0, 0.2, 0.2, 1000, 0, -1, 0, 1.0, 0.0, float("inf"),
                                   C.addressof(out), None) == -5
    assert out.value == 123.0                                  # untouched on error


def test_widest_row_that_fits_the_lds_tables():
    # 254 super-tiles of 4096 columns: the level-1 noise table of one row fills the LDS budget
    assert _sample(V=1_040_384 + 8, stride=1_040_384 + 8) == -2          # E3_ERR_SHAPE
    assert _sample(V=1_040_384, stride=1_040_384, logits=None) == -1     # shape accepted: next check (NULL)
