"""Host-side logic of libnt that needs no GPU: exported symbols, the batch planner
(brute-force invariants), closed forms and argument validation."""
import ctypes as C
import os
import re
from fractions import Fraction
import math

import numpy as np
import pytest

import nt_synth
import paper_2109_08003_amd as nt

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    L = nt.load_library()
    header = open(os.path.join(ROOT, "include", "nt.h")).read()
    declared = set(re.findall(r"\b(nt_[a-z_0-9]+)\s*\(", header))
    assert declared == set(nt.EXPORTS)
    for name in declared:
        assert hasattr(L, name), name


def test_n_steps_and_param_count():
    for n in range(0, 250):
        assert nt.n_steps(n) == math.ceil(Fraction(12, 10) * n) + 2
    for name in ("C0", "C1", "C3", "C4", "C5"):
        cfg = nt_synth.model_config(name)
        assert nt.param_count(cfg) == nt_synth.blob_numel(cfg)
    # a decoder shaped on its own: heads only matter with relative keys, -1 removes the decoder FFN only
    for kw in (dict(dec_n_heads=1, rpr_clip=4), dict(dec_d_ffn=-1), dict(dec_d_ffn=512), dict(dec_n_heads=8, dec_d_ffn=2048)):
        cfg = nt_synth.model_config("C3", **kw)
        assert nt.param_count(cfg) == nt_synth.blob_numel(cfg), kw
    assert nt.param_count(nt_synth.model_config("C3", dec_n_heads=8, dec_d_ffn=2048)) == nt.param_count(nt_synth.model_config("C3"))
    assert nt.param_count(nt_synth.model_config("C1", tie_output=1)) == nt_synth.blob_numel(
        nt_synth.model_config("C1", tie_output=1))


def test_output_slots():
    """nt_output_slots against the step rule written out with exact fractions; empty sentences take no slot."""
    rng = np.random.default_rng(3)
    lens = rng.integers(0, 200, size=500)
    lens[:5] = 0
    offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    want = sum(math.ceil(Fraction(12, 10) * int(n)) + 2 for n in lens if n > 0)
    assert nt.binding.output_slots(offsets) == want
    assert nt.binding.output_slots(np.zeros(1, np.int64)) == 0
    with pytest.raises(nt.NtError) as e:
        nt.binding.output_slots(np.array([0, 5, 3], np.int64))
    assert e.value.code == -6


def check_plan(lengths, budget, max_rows):
    lengths = np.asarray(lengths, dtype=np.int32)
    order, starts = nt.plan_batches(lengths, budget, max_rows)
    N = len(lengths)
    assert sorted(order.tolist()) == list(range(N))                      # a permutation
    sl = lengths[order]
    assert all(sl[i] >= sl[i + 1] for i in range(N - 1))                 # descending
    for i in range(N - 1):                                               # stable: ties keep input order
        if sl[i] == sl[i + 1]:
            assert order[i] < order[i + 1]
    n_real = int((lengths > 0).sum())
    assert starts[0] == 0 and starts[-1] == n_real                       # every real sentence in exactly one batch
    assert all(starts[k] < starts[k + 1] for k in range(len(starts) - 1))
    for k in range(len(starts) - 1):
        a, b = starts[k], starts[k + 1]
        rows, longest = b - a, sl[a]
        assert rows == 1 or rows * longest <= budget
        assert max_rows == 0 or rows <= max_rows
        if b < n_real:                                                   # maximal: the next one would not fit
            assert (rows + 1) * longest > budget or (max_rows and rows + 1 > max_rows)
    inv = np.empty(N, dtype=np.int64)                                    # un-permutation restores input order
    inv[order] = np.arange(N)
    assert np.array_equal(lengths[order][inv], lengths)


def test_plan_batches_brute_force():
    rng = np.random.default_rng(0)
    for trial in range(300):
        n = int(rng.integers(0, 40))
        lengths = rng.integers(0, 12, size=n)
        check_plan(lengths, int(rng.integers(1, 40)), int(rng.choice([0, 0, 1, 3, 7])))
    check_plan([], 10, 0)
    check_plan([0, 0, 0], 10, 0)
    check_plan([50], 10, 0)          # longer than the budget: a batch of its own
    tokens, offsets = nt_synth.workload("C1")
    order, starts = nt.plan_batches(np.diff(offsets), 4096)
    check_plan(np.diff(offsets), 4096, 0)
    assert len(starts) - 1 == 27     # the paper-shaped workload packs into 27 batches at a 4,096-token budget


def test_plan_batches_rejects_bad_arguments():
    with pytest.raises(nt.NtError) as e:
        nt.plan_batches([3, 4], 0)
    assert e.value.code == -1
    with pytest.raises(nt.NtError):
        nt.plan_batches([3, -1], 8)


def test_load_rejects_bad_config_and_blob_before_touching_the_gpu():
    L = nt.load_library()
    cfg = nt_synth.model_config("C0")
    blob = np.zeros(nt_synth.blob_numel(cfg), dtype=np.float16)
    h = C.c_void_p()

    def load(c, nbytes):
        return L.nt_load_weights(C.byref(c), blob.ctypes.data_as(C.c_void_p), nbytes, None, C.byref(h))

    c = nt.make_config(cfg, 4096)
    assert load(c, blob.nbytes - 2) == -3 and b"blob" in L.nt_last_error()
    c.struct_size = 12
    assert load(c, blob.nbytes) == -1
    for key, val in (("d_model", 100), ("n_heads", 3), ("d_ffn", 100), ("max_len", 4096), ("rpr_clip", 99),
                     ("dec_n_heads", 3), ("dec_n_heads", 16), ("dec_d_ffn", 100), ("dec_d_ffn", -2)):
        c = nt.make_config(dict(cfg, **{key: val}), 4096)
        assert load(c, blob.nbytes) == -2, key
    assert load(nt.make_config(dict(cfg, ln_l1=2), 4096), blob.nbytes) == -1
    c = nt.make_config(dict(cfg, bos_id=cfg["vocab"]), 4096)
    assert load(c, blob.nbytes) == -6
    assert L.nt_load_weights(None, None, 0, None, C.byref(h)) == -1
    assert nt.param_count(dict(cfg, d_model=100)) == 0


def test_q8_weight_quantiser_of_the_library_equals_the_oracles(oracle):
    """Eq. 3, 4 on the host side of the library (what nt_load_weights applies to the output matrix) against the
    oracle's, bit for bit: codes, scale and zero point, on random rows, shifted rows, flat rows and rows whose
    zero point saturates."""
    rng = np.random.default_rng(12)
    rows = [rng.normal(0, 512 ** -0.5, 512), rng.normal(0.3, 0.05, 512), rng.normal(-2.0, 0.01, 256),
            np.full(256, 0.125), np.zeros(512), rng.standard_cauchy(512) * 0.01, rng.normal(0, 1e-4, 512)]
    rows += [rng.normal(rng.normal(0, 0.05), abs(rng.normal(0.05, 0.02)) + 1e-4, 512) for _ in range(40)]
    for w in rows:
        w = np.asarray(w, dtype=np.float64).astype(np.float16)
        q, sc, z = nt.q8_quantize_row(w)
        oq, osc, oz = oracle.q8_weight_row(w.astype(np.float32))
        assert np.array_equal(q, oq) and sc == osc and z == oz


def test_workload_recipe_statistics():
    """The synthetic stand-in has the length and token structure the benchmark describes."""
    tokens, offsets = nt_synth.workload("C1")
    lens = np.diff(offsets)
    assert lens.min() >= 1 and lens.max() <= 200 and len(lens) == 4096
    assert abs(np.log(lens).mean() - 3.1) < 0.05 and abs(np.log(lens).std() - 0.5) < 0.05
    assert tokens.min() >= 4 and tokens.max() < 32000
    counts = np.bincount(tokens, minlength=32000)[4:]
    assert counts[0] == counts.max()                       # rank 1 is the most frequent id
    # Zipf slope: log-frequency against log-rank over the head of the distribution
    r = np.arange(1, 51)
    slope = np.polyfit(np.log(r), np.log(counts[:50]), 1)[0]
    assert abs(slope + 1.1) < 0.15
    t0, o0 = nt_synth.workload("C0")
    l0 = np.diff(o0)
    assert len(l0) == 8 and l0.min() >= 5 and l0.max() <= 30 and t0.min() >= 4 and t0.max() < 4000
