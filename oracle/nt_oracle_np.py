"""Second, independently written oracle path: full recomputation on a padded batch.

TEST INFRASTRUCTURE ONLY (used by tests/ to cross-check oracle/nt_oracle.c).  Where the
C oracle walks one sentence at a time and decodes incrementally with caches, this path
pads a whole batch, masks explicitly and recomputes every target position from scratch
with a causal mask.  numpy, fp64 throughout; weights are the blob's fp16 values widened.

Follows the same passages of the paper as the C oracle: student architecture (Sec. 2.2,
Table 2), vanilla-Transformer defaults (Sec. 2.1), query scaling and full-precision
softmax (Sec. 3.1 "FP16 Inference"), plain logits for greedy search (Sec. 3.3), relative
position keys with clipping (Sec. 2.1).
"""
from __future__ import annotations

import numpy as np

import nt_synth


class Weights:
    def __init__(self, cfg: dict, blob: np.ndarray):
        self.cfg = cfg
        self.off = nt_synth.blob_offsets(cfg)
        assert blob.dtype == np.float16 and blob.size == self.off["__total__"][0]
        self.blob = blob

    def __getitem__(self, name: str) -> np.ndarray:
        o, shape = self.off[name]
        return self.blob[o:o + int(np.prod(shape))].reshape(shape).astype(np.float64)


def positions(n: int, d: int) -> np.ndarray:
    """[n, d] sinusoid table: even columns sin, odd columns cos, wavelength 10000^(2k/d)."""
    p = np.arange(n, dtype=np.float64)[:, None]
    k = np.arange(0, d, 2, dtype=np.float64)[None, :]
    ang = p / np.power(10000.0, k / d)
    pe = np.zeros((n, d))
    pe[:, 0::2] = np.sin(ang)
    pe[:, 1::2] = np.cos(ang)[:, : d // 2]
    return pe


def layer_norm(x, g, b, eps, l1=False):
    mu = x.mean(-1, keepdims=True)
    if l1:   # L1-norm variant (Sec. 3.1): scaled mean absolute deviation in place of the standard deviation
        return g * (x - mu) / (np.sqrt(np.pi / 2) * np.abs(x - mu).mean(-1, keepdims=True) + eps) + b
    var = ((x - mu) ** 2).mean(-1, keepdims=True)
    return g * (x - mu) / np.sqrt(var + eps) + b


def masked_softmax(s, mask):
    """softmax over the last axis; positions where mask is False get exactly 0."""
    s = np.where(mask, s, -np.inf)
    s = s - s.max(-1, keepdims=True)
    e = np.where(mask, np.exp(s), 0.0)
    return e / e.sum(-1, keepdims=True)


def attention(W: Weights, prefix: str, xq, xkv, mask, rpr: bool, H: int):
    """xq [B,Tq,d], xkv [B,Tk,d], mask [B,Tq,Tk] bool, H heads -> (context projected [B,Tq,d], probs)."""
    cfg = W.cfg
    d = cfg["d_model"]
    dh = d // H
    B, Tq, _ = xq.shape
    Tk = xkv.shape[1]
    q = (xq @ W[f"{prefix}.Wq"] + W[f"{prefix}.bq"]) / np.sqrt(dh)
    k = xkv @ W[f"{prefix}.Wk"] + W[f"{prefix}.bk"]
    v = xkv @ W[f"{prefix}.Wv"] + W[f"{prefix}.bv"]
    q = q.reshape(B, Tq, H, dh).transpose(0, 2, 1, 3)
    k = k.reshape(B, Tk, H, dh).transpose(0, 2, 1, 3)
    v = v.reshape(B, Tk, H, dh).transpose(0, 2, 1, 3)
    s = q @ k.transpose(0, 1, 3, 2)                      # [B,H,Tq,Tk]
    c = cfg["rpr_clip"]
    if rpr and c > 0:
        rk = W[f"{prefix}.rk"]                            # [2c+1, dh]
        rel = np.clip(np.arange(Tk)[None, :] - np.arange(Tq)[:, None], -c, c) + c   # [Tq,Tk]
        qr = q @ rk.T                                     # [B,H,Tq,2c+1]
        s = s + np.take_along_axis(qr, np.broadcast_to(rel, (B, H, Tq, Tk)), axis=-1)
    p = masked_softmax(s, mask[:, None, :, :])
    ctx = (p @ v).transpose(0, 2, 1, 3).reshape(B, Tq, d)
    return ctx @ W[f"{prefix}.Wo"] + W[f"{prefix}.bo"], p


def ffn(W: Weights, ln: str, prefix: str, x):
    a = layer_norm(x, W[f"{ln}.g"], W[f"{ln}.b"], W.cfg["ln_eps"], W.cfg.get("ln_l1", 0))
    u = np.maximum(a @ W[f"{prefix}.W1"] + W[f"{prefix}.b1"], 0.0)
    return x + u @ W[f"{prefix}.W2"] + W[f"{prefix}.b2"]


def pad_batch(seqs, pad_id):
    L = max(len(s) for s in seqs)
    ids = np.full((len(seqs), L), pad_id, dtype=np.int64)
    for i, s in enumerate(seqs):
        ids[i, : len(s)] = s
    lens = np.array([len(s) for s in seqs])
    return ids, lens


def encode(cfg: dict, blob: np.ndarray, src: list, extra_pad: int = 0):
    """Padded-batch encoder.  Returns (enc [B,S,d], lens)."""
    W = Weights(cfg, blob)
    d, eps, l1 = cfg["d_model"], cfg["ln_eps"], cfg.get("ln_l1", 0)
    ids, lens = pad_batch(src, cfg["pad_id"])
    if extra_pad:
        ids = np.concatenate([ids, np.full((ids.shape[0], extra_pad), cfg["pad_id"], dtype=np.int64)], 1)
    B, S = ids.shape
    x = np.sqrt(d) * W["E"][ids] + positions(S, d)[None]
    key_ok = np.arange(S)[None, :] < lens[:, None]                         # [B,S]
    mask = np.broadcast_to(key_ok[:, None, :], (B, S, S))
    for l in range(cfg["n_enc"]):
        a = layer_norm(x, W[f"enc{l}.ln1.g"], W[f"enc{l}.ln1.b"], eps, l1)
        o, _ = attention(W, f"enc{l}.self", a, a, mask, True, cfg["n_heads"])
        x = x + o
        if cfg["d_ffn"] > 0:
            x = ffn(W, f"enc{l}.ln2", f"enc{l}.ffn", x)
    return layer_norm(x, W["enc_final.g"], W["enc_final.b"], eps, l1), lens


def teacher_forced_logits(cfg: dict, blob: np.ndarray, src: list, tgt_in: list, extra_pad: int = 0):
    """Full (non-incremental) decoder over padded tgt_in; returns list of [T_i, V] logits."""
    W = Weights(cfg, blob)
    d, eps, l1 = cfg["d_model"], cfg["ln_eps"], cfg.get("ln_l1", 0)
    enc, lens = encode(cfg, blob, src, extra_pad)
    S = enc.shape[1]
    tid, tlens = pad_batch(tgt_in, cfg["pad_id"])
    B, T = tid.shape
    z = np.sqrt(d) * W["E"][tid] + positions(T, d)[None]
    causal = np.broadcast_to(np.tril(np.ones((T, T), dtype=bool))[None], (B, T, T))
    cross = np.broadcast_to((np.arange(S)[None, :] < lens[:, None])[:, None, :], (B, T, S))
    # the decoder may have its own head count and FFN width (Table 2: 8-head encoder, 1-head decoder)
    Hd = cfg.get("dec_n_heads", 0) or cfg["n_heads"]
    Fd = {0: cfg["d_ffn"], -1: 0}.get(cfg.get("dec_d_ffn", 0), cfg.get("dec_d_ffn", 0))
    for l in range(cfg["n_dec"]):
        a = layer_norm(z, W[f"dec{l}.ln1.g"], W[f"dec{l}.ln1.b"], eps, l1)
        o, _ = attention(W, f"dec{l}.self", a, a, causal, True, Hd)
        z = z + o
        a = layer_norm(z, W[f"dec{l}.ln2.g"], W[f"dec{l}.ln2.b"], eps, l1)
        o, _ = attention(W, f"dec{l}.cross", a, enc, cross, False, Hd)
        z = z + o
        if Fd > 0:
            z = ffn(W, f"dec{l}.ln3", f"dec{l}.ffn", z)
    h = layer_norm(z, W["dec_final.g"], W["dec_final.b"], eps, l1)
    Wout = W["E"] if cfg["tie_output"] else W["W_out"]
    logits = h @ Wout.T
    return [logits[i, : tlens[i]] for i in range(B)]
