"""Pins for the CPU oracle: each part is checked against something other than itself -
closed forms, library routines used as independent arithmetic, special cases with a
textbook answer, brute force, and the paper's printed parameter counts."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import nt_synth
from oracle import nt_oracle_np as onp

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def tiny(**kw):
    cfg = nt_synth.model_config("C0", d_model=32, vocab=61, n_enc=2, max_len=64)
    cfg.update(kw)
    return cfg


# ---------------------------------------------------------------- primitives
def test_half_to_float_all_patterns(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.lib().ora_half_to_float(int(b)) for b in bits], dtype=np.float32)
    ok = np.isnan(want) | (want.view(np.uint32) == got.view(np.uint32))
    assert ok.all()
    assert np.isnan(got[np.isnan(want)]).all()


def test_pe_golden_and_closed_form(oracle):
    for line in open(os.path.join(GOLD, "sinusoid.txt")):
        if line.startswith("#") or not line.strip():
            continue
        pos, dim, d, val = line.split()
        assert abs(oracle.pe(int(pos), int(d))[int(dim)] - float(val)) < 1e-15
    d = 512
    assert np.array_equal(oracle.pe(0, d), np.tile([0.0, 1.0], d // 2))
    for p in (1, 7, 241):
        row = oracle.pe(p, d)
        assert abs(row[d - 1] - math.cos(p * 10000.0 ** (-(d - 2) / d))) < 1e-12
        assert abs(row[0] - math.sin(p)) < 1e-12
        # sin^2 + cos^2 = 1 for every frequency pair
        assert np.allclose(row[0::2] ** 2 + row[1::2] ** 2, 1.0, atol=1e-12)
        assert np.allclose(row, onp.positions(p + 1, d)[p], atol=1e-12)


def test_layer_norm_invariants_and_library(oracle):
    rng = np.random.default_rng(0)
    for d in (32, 256, 512):
        x = rng.normal(3.0, 2.5, d)
        one, zero = np.ones(d, np.float32), np.zeros(d, np.float32)
        y = oracle.layer_norm(x, one, zero, 1e-5)
        assert abs(y.mean()) < 1e-12
        assert abs(y.var() - 1.0) < 1e-5          # biased variance; eps shifts it by ~eps/var
        g = rng.normal(1, 0.1, d).astype(np.float32)
        b = rng.normal(0, 0.1, d).astype(np.float32)
        want = torch.nn.functional.layer_norm(torch.from_numpy(x), (d,), torch.from_numpy(g).double(),
                                              torch.from_numpy(b).double(), 1e-5).numpy()
        assert np.allclose(oracle.layer_norm(x, g, b, 1e-5), want, atol=1e-12)


def test_l1_layer_norm_closed_forms_and_gaussian_limit(oracle):
    """L1-norm layer normalisation (Sec. 3.1): mean absolute deviation times sqrt(pi/2) in place of the
    standard deviation.  Pinned by a two-level vector (closed form), by the Gaussian limit in which it must
    agree with the vanilla normalisation (this fixes the constant), and by its invariances."""
    d = 64
    one, zero = np.ones(d, np.float32), np.zeros(d, np.float32)
    # x = m +- a: mean m, every |x - mean| = a  ->  y = +-1 / sqrt(pi/2) = +-0.79788456...
    x = 5.0 + 3.0 * np.where(np.arange(d) % 2 == 0, 1.0, -1.0)
    y = oracle.layer_norm_l1(x, one, zero, 0.0)
    assert np.allclose(y, np.where(np.arange(d) % 2 == 0, 1.0, -1.0) * 0.7978845608028654, atol=1e-14)
    # three quarters at 0, one quarter at 4: mean 1, mean |dev| = 1.5 -> y = (-1, 3) / (1.5 sqrt(pi/2))
    x = np.where(np.arange(d) % 4 == 0, 4.0, 0.0)
    y = oracle.layer_norm_l1(x, one, zero, 0.0)
    assert np.allclose(y, np.where(np.arange(d) % 4 == 0, 3.0, -1.0) / (1.5 * 1.2533141373155001), atol=1e-14)
    # eps sits in the denominator beside the deviation: all-equal input gives exactly the offset
    b = np.linspace(-1, 1, d).astype(np.float32)
    assert np.array_equal(oracle.layer_norm_l1(np.full(d, 2.5), one, b, 1e-5), b.astype(np.float64))
    x = np.array([1.0, -1.0] * (d // 2))
    assert np.allclose(oracle.layer_norm_l1(x, one, zero, 0.25), x / (1.2533141373155001 + 0.25), atol=1e-14)
    # Gaussian limit: sqrt(pi/2) E|x - mu| = sigma, so both normalisations agree up to sampling noise
    rng = np.random.default_rng(5)
    n = 400000
    x = rng.normal(-2.0, 7.0, n)
    g1, b0 = np.ones(n, np.float32), np.zeros(n, np.float32)
    ya, yb = oracle.layer_norm_l1(x, g1, b0, 0.0), oracle.layer_norm(x, g1, b0, 0.0)
    assert np.abs(ya / yb - 1.0).max() < 5e-3
    # a heavy-tailed input separates the two (so the L1 path is not the vanilla one in disguise)
    x = rng.laplace(0.0, 1.0, n)
    r = oracle.layer_norm_l1(x, g1, b0, 0.0) / oracle.layer_norm(x, g1, b0, 0.0)
    assert abs(r.mean() - np.sqrt(2.0) / np.sqrt(np.pi / 2)) < 5e-3      # Laplace: sigma = sqrt(2) b, E|x| = b
    # invariances: shift, positive scale; sign flip is odd; gain and offset are applied last
    x = rng.normal(0, 1, d)
    g = rng.normal(1, 0.1, d).astype(np.float32)
    y = oracle.layer_norm_l1(x, one, zero, 0.0)
    assert np.allclose(oracle.layer_norm_l1(x + 11.0, one, zero, 0.0), y, atol=1e-12)
    assert np.allclose(oracle.layer_norm_l1(3.5 * x, one, zero, 0.0), y, atol=1e-12)
    assert np.allclose(oracle.layer_norm_l1(-x, one, zero, 0.0), -y, atol=1e-12)
    assert np.allclose(oracle.layer_norm_l1(x, g, b, 0.0), g.astype(np.float64) * y + b, atol=1e-12)
    assert abs(y.mean()) < 1e-12 and abs(np.abs(y).mean() - 0.7978845608028654) < 1e-12


def test_softmax_sums_to_one_masked_zero_and_library(oracle):
    rng = np.random.default_rng(1)
    s = rng.normal(0, 30.0, 77)                     # large scores: must not overflow
    p = oracle.softmax(s)
    assert abs(p.sum() - 1.0) < 1e-12 and (p >= 0).all()
    assert np.allclose(p, torch.softmax(torch.from_numpy(s), 0).numpy(), atol=1e-14)
    s[[3, 10, 76]] = -np.inf
    p = oracle.softmax(s)
    assert p[3] == 0.0 and p[10] == 0.0 and p[76] == 0.0
    assert abs(p.sum() - 1.0) < 1e-12
    # numpy path: masked positions exactly zero, rows sum to one
    sc = rng.normal(0, 5, (2, 3, 9))
    mask = rng.random((2, 3, 9)) < 0.6
    mask[..., 0] = True
    pm = onp.masked_softmax(sc, mask)
    assert (pm[~mask] == 0).all() and np.allclose(pm.sum(-1), 1.0, atol=1e-12)


def test_linear_orientation(oracle):
    rng = np.random.default_rng(2)
    W = rng.normal(size=(5, 7)).astype(np.float32)
    b = rng.normal(size=7).astype(np.float32)
    x = rng.normal(size=5)
    assert np.allclose(oracle.linear(x, W, b), x @ W.astype(np.float64) + b, atol=1e-13)
    assert np.allclose(oracle.linear(x, W, None), x @ W.astype(np.float64), atol=1e-13)


@pytest.mark.parametrize("heads", [1, 4])
def test_attend_matches_sdpa(oracle, heads):
    rng = np.random.default_rng(3)
    n, d = 11, 32
    dh = d // heads
    q, K, V = rng.normal(size=d), rng.normal(size=(n, d)), rng.normal(size=(n, d))
    c, probs = oracle.attend(q, K, V, heads=heads)
    tq = torch.from_numpy(q).reshape(1, heads, 1, dh)
    tk = torch.from_numpy(K).reshape(1, n, heads, dh).transpose(1, 2)
    tv = torch.from_numpy(V).reshape(1, n, heads, dh).transpose(1, 2)
    want = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, scale=1.0)
    assert np.allclose(c, want.transpose(1, 2).reshape(d).numpy(), atol=1e-12)
    assert np.allclose(probs.sum(-1), 1.0, atol=1e-12)


def test_attend_relative_keys_brute_force(oracle):
    """score_j = q . (k_j + rk[clip(j - i)])  (relative position keys, Sec. 2.1)."""
    rng = np.random.default_rng(4)
    n, d, heads, clip = 25, 16, 2, 3
    dh = d // heads
    q, K, V = rng.normal(size=d), rng.normal(size=(n, d)), rng.normal(size=(n, d))
    rk = rng.normal(size=(2 * clip + 1, dh)).astype(np.float32)
    for qpos in (0, 4, 12, 24):
        c, probs = oracle.attend(q, K, V, heads=heads, rk=rk, clip=clip, qpos=qpos)
        want = np.zeros(d)
        for h in range(heads):
            sc = []
            for j in range(n):
                rel = max(-clip, min(clip, j - qpos))
                key = K[j, h * dh:(h + 1) * dh] + rk[rel + clip].astype(np.float64)
                sc.append(float(q[h * dh:(h + 1) * dh] @ key))
            e = np.exp(np.array(sc) - max(sc))
            p = e / e.sum()
            assert np.allclose(probs[h], p, atol=1e-12)
            want[h * dh:(h + 1) * dh] = p @ V[:, h * dh:(h + 1) * dh]
        assert np.allclose(c, want, atol=1e-12)
    # keys farther than the clip distance share one relative embedding: shifting the query
    # far to the left of every key makes the relative term constant over keys -> no effect
    c_far, _ = oracle.attend(q, K, V, heads=heads, rk=rk, clip=clip, qpos=-100)
    c_none, _ = oracle.attend(q, K, V, heads=heads)
    assert np.allclose(c_far, c_none, atol=1e-12)


# ---------------------------------------------------------------- special cases of the network
def test_len1_layer_is_affine_chain(oracle):
    """One position -> attention weight 1 -> layer = x + (LN(x) Wv + bv) Wo + bo."""
    cfg = tiny(n_enc=1)
    blob = nt_synth.make_weights(cfg, seed=5, random_affine=True)
    W = onp.Weights(cfg, blob)
    d = cfg["d_model"]
    tok = 17
    x = math.sqrt(d) * W["E"][tok] + np.tile([0.0, 1.0], d // 2)
    ln = torch.nn.functional.layer_norm
    a = ln(torch.from_numpy(x), (d,), torch.from_numpy(W["enc0.ln1.g"]), torch.from_numpy(W["enc0.ln1.b"]), 1e-5).numpy()
    x1 = x + (a @ W["enc0.self.Wv"] + W["enc0.self.bv"]) @ W["enc0.self.Wo"] + W["enc0.self.bo"]
    want = ln(torch.from_numpy(x1), (d,), torch.from_numpy(W["enc_final.g"]), torch.from_numpy(W["enc_final.b"]), 1e-5).numpy()
    m = oracle.Model(cfg, blob)
    assert np.allclose(m.encode([tok])[0], want, atol=1e-11)


def test_zero_query_gives_uniform_attention(oracle):
    """Wq = 0, bq = 0 -> all scores 0 -> context = mean of the values."""
    cfg = tiny(n_enc=1)
    blob = nt_synth.make_weights(cfg, seed=6)
    nt_synth.blob_view(cfg, blob, "enc0.self.Wq")[:] = 0
    nt_synth.blob_view(cfg, blob, "enc0.self.bq")[:] = 0
    W = onp.Weights(cfg, blob)
    d = cfg["d_model"]
    src = np.array([5, 9, 33, 60, 12, 7])
    x = math.sqrt(d) * W["E"][src] + onp.positions(len(src), d)
    a = torch.nn.functional.layer_norm(torch.from_numpy(x), (d,)).numpy()
    v = a @ W["enc0.self.Wv"] + W["enc0.self.bv"]
    x1 = x + v.mean(0, keepdims=True) @ W["enc0.self.Wo"] + W["enc0.self.bo"]
    want = torch.nn.functional.layer_norm(torch.from_numpy(x1), (d,)).numpy()
    m = oracle.Model(cfg, blob)
    assert np.allclose(m.encode(src), want, atol=1e-11)


CASES = [
    dict(),                                                          # the student: 1 head, no FFN
    dict(n_heads=4, d_ffn=48),                                       # ablation shape
    dict(n_heads=4, d_ffn=48, n_dec=2, rpr_clip=3),                  # teacher shape
    dict(n_heads=2, rpr_clip=2, tie_output=1),
    # decoder shaped on its own (Table 2: multi-head encoder with FFN, one-head decoder, narrower or no FFN)
    dict(n_heads=4, d_ffn=48, dec_n_heads=1, dec_d_ffn=24),
    dict(n_heads=4, d_ffn=48, dec_n_heads=1, dec_d_ffn=-1, rpr_clip=2),
    dict(n_heads=1, d_ffn=0, dec_n_heads=2, dec_d_ffn=16, rpr_clip=3),
    # L1-norm layer normalisation in every block
    dict(ln_l1=1),
    dict(n_heads=4, d_ffn=48, n_dec=2, ln_l1=1),
]


@pytest.mark.parametrize("kw", CASES)
def test_incremental_equals_full_recompute(oracle, kw):
    """C oracle (per sentence, cached, incremental) == numpy path (padded batch, masks, full)."""
    cfg = tiny(**kw)
    blob = nt_synth.make_weights(cfg, seed=7, random_affine=True)
    m = oracle.Model(cfg, blob)
    rng = np.random.default_rng(8)
    src = [rng.integers(4, cfg["vocab"], size=n) for n in (1, 9, 4, 13)]
    outs = [m.greedy(s)[0] for s in src]
    tgt_in = [np.concatenate([[cfg["bos_id"]], o[:-1]]) for o in outs]
    enc_np, lens = onp.encode(cfg, blob, src)
    full = onp.teacher_forced_logits(cfg, blob, src, tgt_in)
    for i, s in enumerate(src):
        assert np.allclose(m.encode(s), enc_np[i, : len(s)], atol=1e-10)
        inc = m.teacher_forced(s, tgt_in[i])
        assert np.allclose(inc, full[i], atol=1e-9)
        # greedy picks the argmax of those logits, lowest id first
        assert np.array_equal(np.argmax(inc, -1), outs[i])


def test_decoder_shape_of_its_own_is_not_the_encoder_shape(oracle):
    """A decoder given its own head count and FFN width differs from the shared-shape model (so the
    fields are read), and spelling the encoder's shape out for the decoder changes nothing."""
    cfg = tiny(n_heads=4, d_ffn=48)
    same = dict(cfg, dec_n_heads=4, dec_d_ffn=48)
    blob = nt_synth.make_weights(cfg, seed=21, random_affine=True)
    assert nt_synth.blob_numel(same) == nt_synth.blob_numel(cfg)
    src, tgt = np.array([9, 8, 7, 6, 5]), np.array([1, 11, 12])
    a = oracle.Model(cfg, blob).teacher_forced(src, tgt)
    assert np.array_equal(a, oracle.Model(same, blob).teacher_forced(src, tgt))
    one = dict(cfg, dec_n_heads=1)                     # same blob layout (no relative keys), other arithmetic
    b = oracle.Model(one, blob).teacher_forced(src, tgt)
    assert np.abs(a - b).max() > 1e-3
    # the encoder half is untouched by the decoder's fields
    assert np.array_equal(oracle.Model(cfg, blob).encode(src), oracle.Model(one, blob).encode(src))


def test_l1_model_differs_from_vanilla_and_uses_l1_everywhere(oracle):
    """The L1 model is not the vanilla model, and the final normalisation's gain and offset act linearly on
    the logits (they are applied after the division, as in the vanilla form)."""
    cfg = tiny(d_ffn=48, ln_l1=1)
    blob = nt_synth.make_weights(cfg, seed=31, random_affine=True)
    src, tgt = np.array([9, 8, 7, 6, 5]), np.array([1, 11, 12])
    base = oracle.Model(cfg, blob).teacher_forced(src, tgt)
    assert np.abs(base - oracle.Model(dict(cfg, ln_l1=0), blob).teacher_forced(src, tgt)).max() > 1e-2
    # doubling gain and offset of the final decoder normalisation doubles the logits
    b2 = blob.copy()
    nt_synth.blob_view(cfg, b2, "dec_final.g")[:] *= np.float16(2.0)
    nt_synth.blob_view(cfg, b2, "dec_final.b")[:] *= np.float16(2.0)
    assert np.allclose(oracle.Model(cfg, b2).teacher_forced(src, tgt), 2.0 * base, atol=1e-9)


def test_padding_and_batch_mates_do_not_matter(oracle):
    cfg = tiny(n_heads=2, rpr_clip=2)
    blob = nt_synth.make_weights(cfg, seed=9)
    rng = np.random.default_rng(10)
    a, b, c = (rng.integers(4, cfg["vocab"], size=n) for n in (6, 15, 3))
    tgt = [np.array([1, 8, 9, 10]), np.array([1, 5]), np.array([1, 7, 7])]
    base = onp.teacher_forced_logits(cfg, blob, [a, b, c], tgt)
    padded = onp.teacher_forced_logits(cfg, blob, [a, b, c], tgt, extra_pad=5)
    alone = onp.teacher_forced_logits(cfg, blob, [a], tgt[:1])
    assert np.allclose(base[0], padded[0], atol=1e-12) and np.allclose(base[2], padded[2], atol=1e-12)
    assert np.allclose(base[0], alone[0], atol=1e-12)


def test_argmax_without_log_softmax(oracle):
    """Greedy needs no log-softmax on the output layer (Sec. 3.3): same argmax."""
    cfg = tiny()
    blob = nt_synth.make_weights(cfg, seed=11)
    m = oracle.Model(cfg, blob)
    src = np.array([4, 5, 6, 7, 8])
    out, margin = m.greedy(src)
    logits = m.teacher_forced(src, np.concatenate([[1], out[:-1]]))
    lsm = torch.log_softmax(torch.from_numpy(logits), -1).numpy()
    assert np.array_equal(lsm.argmax(-1), out)
    top2 = np.sort(logits, -1)[:, -2:]
    assert np.allclose(margin, top2[:, 1] - top2[:, 0], atol=1e-12) and (margin >= 0).all()


def test_eos_terminated_greedy_search(oracle):
    """EOS-terminated greedy search (Sec. 3.3): pinned against (a) the fixed-length search, of which it is the
    prefix up to and including the first EOS, (b) a search written here that recomputes the whole prefix
    through the teacher-forced call at every step, (c) the cap."""
    cfg = tiny(vocab=300)
    eos = nt_synth.EOS_ID
    blob = nt_synth.make_weights(cfg, seed=13, random_affine=True, eos_gain=1.8)
    m = oracle.Model(cfg, blob)
    rng = np.random.default_rng(14)
    ended = capped = 0
    for n in (1, 2, 3, 5, 8, 9, 12, 17, 20, 24, 30, 33):
        src = rng.integers(4, cfg["vocab"], size=n)
        fixed, _ = m.greedy(src)
        got, margin = m.greedy_eos(src, eos)
        hits = np.nonzero(fixed == eos)[0]
        want = fixed[: hits[0] + 1] if len(hits) else fixed
        assert np.array_equal(got, want)
        assert 1 <= len(got) <= oracle.n_steps(n) and (got[:-1] != eos).all() and len(margin) == len(got)
        ended += got[-1] == eos
        capped += got[-1] != eos
        # step-by-step search that recomputes everything from scratch
        prefix, mine = [cfg["bos_id"]], []
        while len(mine) < oracle.n_steps(n):
            y = int(np.argmax(m.teacher_forced(src, np.array(prefix))[-1]))
            mine.append(y)
            prefix.append(y)
            if y == eos:
                break
        assert np.array_equal(got, mine)
        # a tighter cap cuts the sentence without an EOS
        if len(got) > 2:
            cut, _ = m.greedy_eos(src, eos, max_steps=len(got) - 1)
            assert np.array_equal(cut, got[:-1])
    assert ended >= 3 and capped >= 3          # the stand-in weights produce both kinds of ending
    # the translate call: fixed-length slots, lengths, padding after the end; eos outside the vocabulary is refused
    sents = [rng.integers(4, cfg["vocab"], size=n) for n in (7, 0, 15, 4)]
    off = np.concatenate([[0], np.cumsum([len(x) for x in sents])])
    out, oo, ol, _ = m.translate_eos(np.concatenate(sents), off, eos)
    assert np.array_equal(np.diff(oo), [oracle.n_steps(len(x)) if len(x) else 0 for x in sents]) and ol[1] == 0
    for i, x in enumerate(sents):
        if len(x):
            g, _ = m.greedy_eos(x, eos)
            assert ol[i] == len(g) and np.array_equal(out[oo[i]: oo[i] + ol[i]], g)
            assert (out[oo[i] + ol[i]: oo[i + 1]] == cfg["pad_id"]).all()
    with pytest.raises(ValueError):
        m.greedy_eos(sents[0], cfg["vocab"])


# ---------------------------------------------------------------- 8-bit output layer (Sec. 3.2, Eq. 3-6)
def test_q8_weight_quantiser_closed_forms_and_error_bound(oracle):
    d = 64
    # +-a alternating: mean 0, sd a -> scale 14a/255, zero = rint(127 - 127.5) = rint(-0.5) = 0 (to even),
    # codes rint(+-255/14) = +-18
    a = 0.03125
    q, sc, z = oracle.q8_weight_row(np.where(np.arange(d) % 2 == 0, a, -a))
    assert sc == np.float32(14 * a / 255) and z == 0
    assert np.array_equal(q, np.where(np.arange(d) % 2 == 0, 18, -18))
    # shifted by m = 3a: zero = rint(127 - (3a + 7a) * 255 / (14a)) = rint(127 - 182.142...) = -55,
    # codes rint((3a +- a) * 255 / (14a) - 55) = rint(72.857 - 55), rint(36.43 - 55) = 18, -19
    q, sc, z = oracle.q8_weight_row(3 * a + np.where(np.arange(d) % 2 == 0, a, -a))
    assert z == -55 and np.array_equal(q, np.where(np.arange(d) % 2 == 0, 18, -19))
    # the ends of the range: mean + 7 sd -> 127 and mean - 7 sd -> -128 (Eq. 3, 4 as read); beyond: clamped.
    # one large entry among zeros: n = 256 values, one of them b -> mean b/256, sd = b sqrt(255)/256
    n, b = 256, 1.0
    w = np.zeros(n); w[7] = b
    q, sc, z = oracle.q8_weight_row(w)
    mean, sd = b / n, b * math.sqrt(n - 1) / n
    scale = 14 * sd / 255
    assert sc == np.float32(scale) and z == round(127 - (mean + 7 * sd) / scale)
    assert q[7] == 127 and q[0] == round(0 / scale + z)          # b is 15.9 sd above the mean: clamped
    # rounding error of everything inside the range is at most half a step
    rng = np.random.default_rng(3)
    w = (rng.normal(0.01, 0.05, 512)).astype(np.float16).astype(np.float64)
    q, sc, z = oracle.q8_weight_row(w)
    inside = np.abs(w - w.mean()) < 6.9 * w.std()
    back = float(sc) * (q.astype(np.float64) - z)
    assert np.abs(back - w)[inside].max() <= 0.5 * float(sc) * (1 + 1e-6)
    assert inside.all() and -128 <= q.min() and q.max() <= 127
    # a constant column has no spread: scale 1, every code equal
    q, sc, z = oracle.q8_weight_row(np.full(d, 0.25))
    assert sc == 1.0 and len(set(q.tolist())) == 1


def test_q8_activation_quantiser_ends_codes_and_error_bound(oracle):
    rng = np.random.default_rng(4)
    h = rng.normal(0, 1, 512).astype(np.float32)
    u, sc, z = oracle.q8_activation_row(h)
    assert sc == np.float32((h.max() - h.min()) / np.float32(255))
    assert u[h.argmax()] == 255 and u[h.argmin()] == 0                      # Eq. 5, 6 as read: the ends of the range
    back = np.float64(sc) * (u.astype(np.float64) - z)
    assert np.abs(back - h).max() <= 0.5 * float(sc) * 1.001 + 1e-6
    # exact small case: h = 0, 1, ..., 255 -> scale 1, zero 0, codes = h
    u, sc, z = oracle.q8_activation_row(np.arange(256, dtype=np.float32))
    assert sc == 1.0 and z == 0 and np.array_equal(u, np.arange(256))
    # shifted and scaled: h = -10 + 0.5 k -> scale 0.5, zero = rint(255 - 117.5 / 0.5) = 20, codes k
    u, sc, z = oracle.q8_activation_row((-10 + 0.5 * np.arange(256)).astype(np.float32))
    assert sc == 0.5 and z == 20 and np.array_equal(u, np.arange(256))
    # a row entirely above zero: the zero point rint(255 - 137.5 / 0.5) = -20 is kept inside the code range (0),
    # the codes h / 0.5 = 20 + k saturate at 255
    u, sc, z = oracle.q8_activation_row((10 + 0.5 * np.arange(256)).astype(np.float32))
    assert sc == 0.5 and z == 0 and np.array_equal(u, np.minimum(20 + np.arange(256), 255))
    # likewise a weight column far to one side of zero: mean 5, sd 0.01 -> the zero point saturates at -128
    q, wsc, wz = oracle.q8_weight_row(5.0 + 0.01 * np.where(np.arange(64) % 2 == 0, 1.0, -1.0))
    assert wz == -128 and (q == 127).all()
    u, sc, z = oracle.q8_activation_row(np.full(16, 3.0, dtype=np.float32))           # no spread: scale 1
    assert sc == 1.0 and len(set(u.tolist())) == 1


def _eq56_in_double(h):
    """Eq. 5, 6 (as read) for the rows of h, every operation in double: codes [R, d], scale [R], unclamped zero [R]."""
    h = h.astype(np.float64)
    mx, mn = h.max(axis=1), h.min(axis=1)
    scale = np.where(mx > mn, (mx - mn) / 255.0, 1.0)
    zero = np.rint(255.0 - mx / scale)
    codes = np.clip(np.rint(h / scale[:, None] + zero[:, None]), 0, 255)
    return codes, scale, zero


def test_q8_activation_quantiser_in_fp32_stays_within_one_step_of_eq_5_6_in_double(oracle):
    """The oracle's activation leg is specified operation by operation in fp32 (so that integer codes can be compared
    bit for bit); this pins it to the equations themselves, evaluated in double: on 100,000 random rows and on rows
    built to sit on rounding boundaries no code differs by more than one step, the scale agrees to fp32 rounding,
    the zero points differ by at most one, and on every row that straddles zero - every LayerNorm output does - the
    zero point of Eq. 6 lies inside the code range by itself, so the clamp changes nothing."""
    rng = np.random.default_rng(2024)
    d = 64
    rows = [rng.normal(0, 1, (40000, d)),                                         # decoder-state-like rows
            rng.normal(0, 1, (20000, d)) * np.exp(rng.normal(0, 3, (20000, 1))),  # scales over many octaves
            rng.normal(rng.normal(0, 2, (20000, 1)), 1.0, (20000, d)),            # shifted: some rows one-sided
            rng.laplace(0, 1, (10000, d)) ** 3]                                   # heavy tails: few large entries
    # rows on rounding boundaries: h = s (k + 1/2 - z) for integers k lands exactly between two codes
    s = 2.0 ** rng.integers(-6, 3, (10000, 1))
    z = rng.integers(0, 256, (10000, 1))
    k = rng.integers(0, 255, (10000, d))
    tie = s * (k + 0.5 - z)
    tie[:, 0], tie[:, 1] = (s * (0 - z))[:, 0], (s * (255 - z))[:, 0]             # the ends fix scale = s, zero = z
    rows.append(tie)
    h = np.concatenate(rows).astype(np.float32)
    assert len(h) >= 100000
    want_u, want_sc, want_z = _eq56_in_double(h)
    worst, straddle_rows, one_sided_rows, differing = 0, 0, 0, 0
    for r in range(len(h)):
        u, sc, zp = oracle.q8_activation_row(h[r])
        assert abs(float(sc) - want_sc[r]) <= 1.2e-7 * want_sc[r]                 # one fp32 rounding of the quotient
        straddles = h[r].min() <= 0.0 <= h[r].max()
        if straddles:
            straddle_rows += 1
            assert 0 <= want_z[r] <= 255                                          # Eq. 6 needs no clamp here ...
            assert abs(zp - want_z[r]) <= 1                                       # ... and fp32 moves it by at most one
            diff = np.abs(u.astype(np.int64) - want_u[r].astype(np.int64))
            # a zero point that moved by one shifts every code by one more
            assert diff.max() <= 1 + abs(zp - int(want_z[r])), (r, diff.max())
            worst = max(worst, int(diff.max()))
            differing += int((diff > 0).sum())
        else:
            one_sided_rows += 1
            assert zp == int(min(max(want_z[r], 0), 255))                         # the documented reading: a code itself
    assert straddle_rows > 90000 and one_sided_rows > 1000
    assert worst >= 1 and differing < 0.02 * straddle_rows * d                     # ties do flip; almost nothing else does


def test_q8_logits_within_the_quantisation_bound_of_the_exact_product(oracle):
    """The 8-bit logits against the product they approximate, h . w_v in double, with the half-step bound of both
    quantisers (weights: 0.5 b_scale per element inside mean +- 7 sd; activations: 0.5 a_scale per element, 1.5 when
    the fp32 leg moved a code or the zero point by one)."""
    cfg = tiny(vocab=211, q8_output=1, d_model=64)
    blob = nt_synth.make_weights(cfg, seed=43, random_affine=True)
    m = oracle.Model(cfg, blob)
    W = onp.Weights(cfg, blob)["W_out"]
    rng = np.random.default_rng(44)
    h = rng.normal(0, 1, (200, cfg["d_model"])).astype(np.float32)
    logits, am = m.q8_output_layer(h)
    exact = h.astype(np.float64) @ W.T
    for r in range(len(h)):
        _, a_sc, _ = oracle.q8_activation_row(h[r])
        for v in range(0, cfg["vocab"], 7):
            _, b_sc, _ = m.q8_weights(v)
            bound = 0.5 * b_sc * np.abs(h[r]).sum() + 1.5 * a_sc * np.abs(W[v]).sum() + 0.75 * a_sc * b_sc * cfg["d_model"]
            assert abs(logits[r, v] - exact[r, v]) <= bound * 1.01
    # and the layer is useful: the 8-bit arg-max is the exact arg-max except where the exact top two are close
    top2 = np.sort(exact, axis=1)[:, -2:]
    clear = (top2[:, 1] - top2[:, 0]) > 0.1
    assert clear.sum() > 100 and np.array_equal(am[clear], exact.argmax(axis=1)[clear])


def test_q8_argmax_sensitivity_to_a_small_change_of_the_quantised_state(oracle):
    """What a tiny difference of the decoder state does to the 8-bit layer, on the benchmark's output matrix
    (32,000 x 512): this is the derivation behind the greedy tolerance of the 8-bit model.  Two pipelines that
    agree to a relative 1e-4 of the state (fp16 matrix cores with head/tail activations against fp64) put a few of
    the 512 codes on the other side of a rounding boundary; each moves every logit by a_scale |w|, so the logits
    differ by about 1e-3 and the arg-max of a step changes with a probability of a few in a thousand - always
    between two entries whose 8-bit logits are closer than 1e-2.  Over the ~32 steps of a sentence that is up to
    one sentence in ten, which is why the greedy test of the 8-bit model asks for 90 % identical sentences and
    audits every mismatch at 1e-2."""
    cfg = nt_synth.model_config("C1", q8_output=1, n_enc=1)
    blob = nt_synth.make_weights(cfg, seed=0)
    m = oracle.Model(cfg, blob)
    rng = np.random.default_rng(7)
    R = 400
    h = rng.normal(0, 1, (R, 512)).astype(np.float32)                      # LayerNorm outputs: mean 0, variance 1
    l0, a0 = m.q8_output_layer(h)
    for eps, flips_lo, flips_hi, rms_hi, rate_hi in ((1e-4, 0.5, 8.0, 4e-3, 0.012), (1e-3, 8.0, 80.0, 1.2e-2, 0.03)):
        h2 = (h.astype(np.float64) + eps * rng.normal(0, 1, h.shape)).astype(np.float32)
        l1, a1 = m.q8_output_layer(h2)
        flips = np.mean([(oracle.q8_activation_row(h[r])[0] != oracle.q8_activation_row(h2[r])[0]).sum() for r in range(R)])
        assert flips_lo <= flips <= flips_hi, (eps, flips)
        assert 1e-4 < float((l1 - l0).std()) < rms_hi, (eps, float((l1 - l0).std()))
        changed = np.nonzero(a0 != a1)[0]
        assert len(changed) <= rate_hi * R, (eps, len(changed))
        for r in changed:                                                  # only near-ties of the 8-bit logits flip
            assert abs(float(l0[r, a0[r]]) - float(l0[r, a1[r]])) < 1e-2


def test_q8_output_layer_is_the_integer_definition_and_close_to_the_exact_layer(oracle):
    cfg = tiny(vocab=97, q8_output=1)
    blob = nt_synth.make_weights(cfg, seed=41, random_affine=True)
    m, exact = oracle.Model(cfg, blob), oracle.Model(dict(cfg, q8_output=0), blob)
    d, V = cfg["d_model"], cfg["vocab"]
    W = onp.Weights(cfg, blob)["W_out"]                                       # [V, d] float64
    rng = np.random.default_rng(42)
    h = rng.normal(0, 1, (5, d)).astype(np.float32)
    logits, am = m.q8_output_layer(h)
    for r in range(5):
        u, a_sc, a_z = oracle.q8_activation_row(h[r])
        worst = 0.0
        for v in range(V):
            q, b_sc, b_z = m.q8_weights(v)
            q2, b_sc2, b_z2 = oracle.q8_weight_row(W[v])
            assert np.array_equal(q, q2) and b_sc == b_sc2 and b_z == b_z2   # the model holds Eq. 3, 4 of its own matrix
            I = sum((int(u[k]) - a_z) * (int(q[k]) - b_z) for k in range(d))   # Python integers: exact
            t = np.float32(b_sc) * np.float32(I)
            assert logits[r, v] == np.float32(np.float64(a_sc) * np.float64(t))
            # against the exact product: each factor is off by at most half a step
            bound = (0.5 * b_sc * np.abs(h[r]).sum() + 0.5 * a_sc * np.abs(W[v]).sum() + 0.25 * a_sc * b_sc * d) * 1.01
            err = abs(float(logits[r, v]) - float(h[r].astype(np.float64) @ W[v]))
            assert err <= bound
            worst = max(worst, err / bound)
        assert worst > 0.01                                                    # the bound is not vacuous
        assert am[r] == int(np.argmax(logits[r]))
    # inside the model: the decoder's logits are this layer applied to its final state; the rest is untouched
    src, tgt = np.array([9, 8, 7, 6, 5]), np.array([1, 11, 12])
    lq, le = m.teacher_forced(src, tgt), exact.teacher_forced(src, tgt)
    assert np.array_equal(m.encode(src), exact.encode(src))
    assert 1e-4 < np.abs(lq - le).max() < 0.2
    out, _ = m.greedy(src, 6)
    assert np.array_equal(out, np.argmax(m.teacher_forced(src, np.concatenate([[1], out[:-1]])), -1))


def test_tied_embedding_collapse(oracle):
    """With tied output weights, sqrt(d) embedding scale and random weights the logit of the
    previous token dominates (~ sqrt(d) |E_y|^2 / sigma_z against N(0,1) for the others), so
    greedy decoding re-emits BOS at every step: an end-to-end analytic prediction that runs
    embed -> every layer -> final LayerNorm -> projection -> argmax."""
    cfg = nt_synth.model_config("C0", tie_output=1)
    blob = nt_synth.make_weights(cfg, seed=0)
    m = oracle.Model(cfg, blob)
    tokens, offsets = nt_synth.workload("C0")
    for i in range(3):
        out, margin = m.greedy(tokens[offsets[i]:offsets[i + 1]])
        assert (out == cfg["bos_id"]).all()
        assert margin.min() > 1.0


def test_translate_matches_per_sentence_and_threads(oracle):
    cfg = tiny()
    blob = nt_synth.make_weights(cfg, seed=12)
    m = oracle.Model(cfg, blob)
    rng = np.random.default_rng(13)
    lens = [3, 0, 7, 1, 12]
    toks = rng.integers(4, cfg["vocab"], size=sum(lens)).astype(np.int32)
    offs = np.concatenate([[0], np.cumsum(lens)])
    out, oo, used = m.translate(toks, offs, n_threads=3)
    assert used == 3
    for i, n in enumerate(lens):
        seg = out[oo[i]:oo[i + 1]]
        if n == 0:
            assert seg.size == 0
        else:
            assert np.array_equal(seg, m.greedy(toks[offs[i]:offs[i + 1]])[0])


def test_invalid_inputs_rejected(oracle):
    cfg = tiny()
    blob = nt_synth.make_weights(cfg, seed=12)
    with pytest.raises(ValueError):
        oracle.Model(cfg, blob[:-1])
    m = oracle.Model(cfg, blob)
    with pytest.raises(ValueError):
        m.encode([cfg["vocab"]])
    with pytest.raises(ValueError):
        m.encode(np.full(cfg["max_len"] + 1, 5))


# ---------------------------------------------------------------- closed forms
def test_n_steps_is_ceil_1p2_len_plus_2(oracle):
    for n in range(1, 201):
        assert oracle.n_steps(n) == math.ceil(Fraction(12, 10) * n) + 2


def test_param_count_matches_layout_and_paper_tables(oracle):
    for name in ("C0", "C1", "C3", "C4", "C5"):
        cfg = nt_synth.model_config(name)
        assert oracle.param_count(cfg) == nt_synth.blob_numel(cfg)
    # the paper's models: encoder keeps the vanilla FFN, Dim-FFN is the decoder's (Table 2 caption)
    V = 32000
    for line in open(os.path.join(GOLD, "param_counts.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, ne, nd, d, fe, fd, printed = line.split()
        ne, nd, d, fe, fd, printed = int(ne), int(nd), int(d), int(fe), int(fd), float(printed)
        cfg = nt_synth.model_config("C1", n_enc=ne, n_dec=nd, d_model=d, d_ffn=fe, tie_output=1, vocab=V,
                                    n_heads=8, dec_n_heads=1 if nd == 1 else 0, dec_d_ffn=fd if fd else -1)
        n = oracle.param_count(cfg)
        # head counts do not change the count without relative position keys
        assert n == oracle.param_count(dict(cfg, dec_n_heads=0))
        # written out: embedding, per layer 4 projections (+bias), FFN (+biases), LayerNorms
        attn, ln = 4 * (d * d + d), 2 * d
        ffn = lambda F: (2 * d * F + F + d + ln) if F else 0
        assert n == V * d + ne * (ln + attn + ffn(fe)) + ln + nd * (2 * (ln + attn) + ffn(fd)) + ln
        assert abs(n / 1e6 - printed) / printed < 0.025, (name, n)
    c5 = oracle.param_count(nt_synth.model_config("C5"))
    assert abs(c5 / 1e6 - 28) / 28 < 0.025
