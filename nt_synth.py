"""Seeded synthetic inputs: model configurations, weight blobs and source sentences.

This module is the only code shared by the CPU oracle and the HIP library's tests.
It holds no arithmetic of the translation method: it only draws random numbers,
rounds them to fp16 and lays them out in the documented blob order.  Both
implementations parse the blob with their own code.

Weight blob format (little-endian IEEE fp16, flat, no header).  Every matrix is
stored in "math" orientation W[in][out] (y = x @ W + b), row-major:

    E                       [V, d]        token embedding, source = target
    W_out                   [V, d]        output projection, only if tie_output == 0
    per encoder layer l = 0..n_enc-1:
        ln1.g [d] ln1.b [d]
        Wq [d,d] bq [d]  Wk [d,d] bk [d]  Wv [d,d] bv [d]  Wo [d,d] bo [d]
        rk [2c+1, d_h]                    only if rpr_clip = c > 0
        ln2.g [d] ln2.b [d] W1 [d,F] b1 [F] W2 [F,d] b2 [d]      only if d_ffn = F > 0
    enc_final.g [d] enc_final.b [d]
    per decoder layer l = 0..n_dec-1:
        ln1.g ln1.b   self: Wq bq Wk bk Wv bv Wo bo   rk [2c+1, d_h] (if c > 0)
        ln2.g ln2.b   cross: Wq bq Wk bk Wv bv Wo bo
        ln3.g ln3.b W1 b1 W2 b2                                  only if F_dec > 0
    dec_final.g [d] dec_final.b [d]

The decoder may have its own head count and FFN width (the paper's submitted students: a base
encoder in front of a single-head decoder, Table 2): dec_n_heads = 0 means "as the encoder",
dec_d_ffn = 0 means "as the encoder", -1 means no decoder FFN; d_h and F above are then the
decoder's values in the decoder layers (dec_heads / dec_ffn below resolve them).

Workload recipes (the synthetic stand-ins for the WMT21 efficiency-task input,
which is not available here):
    C0  8 sentences, lengths uniform in [5,30], ids uniform in [4,V)
    C1+ lengths = clip(round(exp(N(3.1, 0.5^2))), 1, 200); ids Zipf(s=1.1) by rank
        over ids 4..V-1 (rank r=1 -> id 4), normalised over the finite support.
"""
from __future__ import annotations

import numpy as np

PAD_ID, BOS_ID, EOS_ID, UNK_ID = 0, 1, 2, 3
N_SPECIAL = 4

_BASE = dict(n_enc=6, n_dec=1, d_model=512, n_heads=1, d_ffn=0, vocab=32000,
             max_len=256, rpr_clip=0, tie_output=0, bos_id=BOS_ID, pad_id=PAD_ID,
             ln_eps=1e-5, dec_n_heads=0, dec_d_ffn=0, ln_l1=0, q8_output=0)

CONFIGS = {
    # tiny parity student
    "C0": dict(_BASE, d_model=256, vocab=4000),
    # paper-shaped student (also the C2 throughput student)
    "C1": dict(_BASE),
    "C2": dict(_BASE),
    # ablation student: multi-head attention and FFN restored everywhere
    "C3": dict(_BASE, n_heads=8, d_ffn=2048),
    # deep teacher-shaped model with relative position keys
    "C4": dict(_BASE, n_enc=30, n_dec=6, n_heads=8, d_ffn=2048, rpr_clip=8),
    # shape of the paper's fastest GPU submission (Student-3-1-512, Table 2 / Sec. 5): base encoder of 3
    # layers (8 heads, FFN 2,048), one decoder layer with a single head and an FFN of 512, shared embedding
    "C5": dict(_BASE, n_enc=3, n_heads=8, d_ffn=2048, dec_n_heads=1, dec_d_ffn=512, tie_output=1),
}


def dec_heads(cfg: dict) -> int:
    return cfg.get("dec_n_heads", 0) or cfg["n_heads"]


def dec_ffn(cfg: dict) -> int:
    f = cfg.get("dec_d_ffn", 0)
    return cfg["d_ffn"] if f == 0 else max(f, 0)


def model_config(name: str, **overrides) -> dict:
    cfg = dict(CONFIGS[name])
    cfg.update(overrides)
    return cfg


def blob_layout(cfg: dict) -> list[tuple[str, tuple[int, ...]]]:
    """Ordered (name, shape) list of every tensor in the blob."""
    d, V, F = cfg["d_model"], cfg["vocab"], cfg["d_ffn"]
    c, dh = cfg["rpr_clip"], cfg["d_model"] // cfg["n_heads"]
    Fd, dhd = dec_ffn(cfg), cfg["d_model"] // dec_heads(cfg)
    out: list[tuple[str, tuple[int, ...]]] = [("E", (V, d))]
    if not cfg["tie_output"]:
        out.append(("W_out", (V, d)))

    def attn(prefix: str, rpr: bool, dh: int = dh):
        for w in ("q", "k", "v", "o"):
            out.append((f"{prefix}.W{w}", (d, d)))
            out.append((f"{prefix}.b{w}", (d,)))
        if rpr and c > 0:
            out.append((f"{prefix}.rk", (2 * c + 1, dh)))

    def ln(prefix: str):
        out.append((f"{prefix}.g", (d,)))
        out.append((f"{prefix}.b", (d,)))

    def ffn(prefix: str, F: int = F):
        out.append((f"{prefix}.W1", (d, F)))
        out.append((f"{prefix}.b1", (F,)))
        out.append((f"{prefix}.W2", (F, d)))
        out.append((f"{prefix}.b2", (d,)))

    for l in range(cfg["n_enc"]):
        ln(f"enc{l}.ln1")
        attn(f"enc{l}.self", True)
        if F > 0:
            ln(f"enc{l}.ln2")
            ffn(f"enc{l}.ffn")
    ln("enc_final")
    for l in range(cfg["n_dec"]):
        ln(f"dec{l}.ln1")
        attn(f"dec{l}.self", True, dhd)
        ln(f"dec{l}.ln2")
        attn(f"dec{l}.cross", False, dhd)
        if Fd > 0:
            ln(f"dec{l}.ln3")
            ffn(f"dec{l}.ffn", Fd)
    ln("dec_final")
    return out


def blob_offsets(cfg: dict) -> dict[str, tuple[int, tuple[int, ...]]]:
    """name -> (offset in fp16 elements, shape)."""
    off, res = 0, {}
    for name, shape in blob_layout(cfg):
        res[name] = (off, shape)
        off += int(np.prod(shape))
    res["__total__"] = (off, ())
    return res


def blob_numel(cfg: dict) -> int:
    return blob_offsets(cfg)["__total__"][0]


def make_weights(cfg: dict, seed: int = 0, random_affine: bool = False, eos_gain: float | None = None) -> np.ndarray:
    """Draw the fp16 weight blob.

    eos_gain (models with their own output matrix only): after the draw, the EOS row of the output matrix is
    multiplied by this factor.  Logits of a random model are close to N(0, 1), so the row's logit wins a step
    with probability about P(N(0,1) > 4 / eos_gain): sentences then end at varied, data-dependent steps, which
    random weights alone never produce (EOS would win about once in `vocab` steps).

    One PCG64 stream; tensors are drawn in blob order.  Every matrix, bias and
    embedding entry is N(0, 1/d) (std d^-1/2) rounded to fp16; LayerNorm gain is 1
    and offset 0 unless random_affine, in which case gain = 1 + 0.1 N(0,1) and
    offset = 0.1 N(0,1) (drawn in the same stream, so the blob differs throughout).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    std = cfg["d_model"] ** -0.5
    parts = []
    for name, shape in blob_layout(cfg):
        leaf = name.rsplit(".", 1)[-1]
        is_ln = ".ln" in name or name.startswith("enc_final") or name.startswith("dec_final")
        if is_ln and leaf == "g":
            t = 1.0 + 0.1 * rng.standard_normal(shape) if random_affine else np.ones(shape)
        elif is_ln and leaf == "b":
            t = 0.1 * rng.standard_normal(shape) if random_affine else np.zeros(shape)
        else:
            t = std * rng.standard_normal(shape)
        parts.append(np.asarray(t, dtype=np.float64).astype(np.float16).ravel())
    blob = np.concatenate(parts)
    if eos_gain is not None:
        assert not cfg["tie_output"], "eos_gain needs a separate output matrix"
        row = blob_view(cfg, blob, "W_out")[EOS_ID]
        row[:] = (row.astype(np.float64) * eos_gain).astype(np.float16)
    return blob


def blob_view(cfg: dict, blob: np.ndarray, name: str) -> np.ndarray:
    """Writable view of one tensor inside the blob (for tests that edit weights)."""
    off, shape = blob_offsets(cfg)[name]
    return blob[off:off + int(np.prod(shape))].reshape(shape)


def draw_sentences(kind: str, n: int, vocab: int, seed: int):
    """Return (tokens int32 [sum len], offsets int64 [n+1]).

    kind "uniform": the C0 recipe; kind "lognormal_zipf": the C1..C4 recipe.
    Draw order: all lengths first, then all token ids, from one PCG64(seed) stream.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    if kind == "uniform":
        lengths = rng.integers(5, 31, size=n)
        total = int(lengths.sum())
        tokens = rng.integers(N_SPECIAL, vocab, size=total)
    elif kind == "lognormal_zipf":
        lengths = np.clip(np.rint(np.exp(rng.normal(3.1, 0.5, size=n))), 1, 200).astype(np.int64)
        total = int(lengths.sum())
        ranks = np.arange(1, vocab - N_SPECIAL + 1, dtype=np.float64)
        cdf = np.cumsum(ranks ** -1.1)
        cdf /= cdf[-1]
        r = np.searchsorted(cdf, rng.random(total), side="left")
        tokens = np.minimum(r, vocab - N_SPECIAL - 1) + N_SPECIAL
    else:
        raise ValueError(kind)
    offsets = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(lengths, out=offsets[1:])
    return tokens.astype(np.int32), offsets


WORKLOADS = {
    # name: (sentence recipe, count, input seed)
    "C0": ("uniform", 8, 0),
    "C1": ("lognormal_zipf", 4096, 1),
    "C2": ("lognormal_zipf", 200000, 2),
    "C3": ("lognormal_zipf", 16384, 3),
    "C4": ("lognormal_zipf", 2048, 4),
    "C5": ("lognormal_zipf", 200000, 5),
}


def workload(name: str, n: int | None = None):
    kind, count, seed = WORKLOADS[name]
    return draw_sentences(kind, count if n is None else n, CONFIGS[name]["vocab"], seed)
