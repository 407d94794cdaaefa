"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This module holds none of the training method's arithmetic: it only draws random
numbers (token ids, initial weights) and names the workload shapes.  Both sides
receive the arrays it returns as plain inputs, so neither owns a random generator.

The token streams stand in for the character/word corpora the paper trains on
(Section "Datasets"), which are not available: ids are i.i.d. Zipf-distributed
ranks, P(id = r-1) proportional to r**(-s), drawn by inverse transform of an fp64
CDF on seeded uniforms.
"""
from __future__ import annotations

import numpy as np

# name -> workload shape.  Field names follow the C config struct.
CONFIGS = {
    # Tiny fp32 parity case: 2 layers, K=2, SGD lr 0.1, 3 steps.
    "cfg1": dict(n_layer=2, d_model=64, n_head=2, d_head=32, d_ff=256, vocab=256,
                 seq_len=32, mem_len=0, batch=4, n_module=2, rel_pos=0, dtype=0,
                 optimizer=0, lr=0.1, zipf_s=1.1, seed=0, steps=3),
    # Headline bench case: 12 layers, K=4, Adam, bf16 + fp32 master.
    "cfg2": dict(n_layer=12, d_model=512, n_head=8, d_head=64, d_ff=2048, vocab=32768,
                 seq_len=512, mem_len=0, batch=16, n_module=4, rel_pos=0, dtype=1,
                 optimizer=1, lr=2.5e-4, zipf_s=1.1, seed=2, steps=8),
    # Transformer-XL style, odd dims.
    "cfg3": dict(n_layer=16, d_model=410, n_head=10, d_head=41, d_ff=2100, vocab=32768,
                 seq_len=150, mem_len=150, batch=32, n_module=4, rel_pos=1, dtype=1,
                 optimizer=1, lr=2.5e-4, zipf_s=1.1, seed=3, steps=8),
    # Larger plain decoder, K=8.
    "cfg4": dict(n_layer=24, d_model=1024, n_head=16, d_head=64, d_ff=4096, vocab=50257,
                 seq_len=1024, mem_len=0, batch=8, n_module=8, rel_pos=0, dtype=1,
                 optimizer=1, lr=2.5e-4, zipf_s=1.1, seed=4, steps=12),
    # Large Transformer-XL style.
    "cfg5": dict(n_layer=18, d_model=1024, n_head=16, d_head=64, d_ff=4096, vocab=65536,
                 seq_len=384, mem_len=384, batch=16, n_module=4, rel_pos=1, dtype=1,
                 optimizer=1, lr=2.5e-4, zipf_s=1.05, seed=5, steps=8),
}


def zipf_cdf(vocab: int, s: float) -> np.ndarray:
    """fp64 CDF of P(rank r) ~ r**(-s), r = 1..vocab."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-float(s))
    c = np.cumsum(w)
    c /= c[-1]
    c[-1] = 1.0
    return c


def zipf_tokens(rng: np.random.Generator, shape, vocab: int, s: float) -> np.ndarray:
    """int32 token ids in [0, vocab), Zipf(s) over ranks, id = rank - 1."""
    u = rng.random(size=shape)
    ids = np.searchsorted(zipf_cdf(vocab, s), u, side="left")
    return np.minimum(ids, vocab - 1).astype(np.int32)


def token_batches(vocab: int, batch: int, seq_len: int, steps: int, s: float, seed: int,
                  contiguous: bool):
    """Returns (tokens, targets), each int32 [steps, batch, seq_len].

    contiguous=False: every step draws a fresh [batch, seq_len+1] block; inputs are
    its first seq_len columns and targets its last seq_len columns.
    contiguous=True: `batch` independent streams of length steps*seq_len+1 are cut
    into consecutive segments, so a segment memory carries over between steps.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    if contiguous:
        stream = zipf_tokens(rng, (batch, steps * seq_len + 1), vocab, s)
        tok = np.stack([stream[:, t * seq_len:(t + 1) * seq_len] for t in range(steps)])
        tgt = np.stack([stream[:, t * seq_len + 1:(t + 1) * seq_len + 1] for t in range(steps)])
    else:
        blk = zipf_tokens(rng, (steps, batch, seq_len + 1), vocab, s)
        tok, tgt = blk[:, :, :seq_len], blk[:, :, 1:]
    return np.ascontiguousarray(tok), np.ascontiguousarray(tgt)


def markov_token_batches(vocab: int, batch: int, seq_len: int, steps: int, s: float, seed: int,
                         follow: float = 0.75):
    """(tokens, targets) int32 [steps, batch, seq_len] from a first-order Markov source:
    with probability `follow` the next id is a fixed function of the current one
    (id * 5 + 3 mod vocab), otherwise a fresh Zipf(s) draw.  A structured stand-in for
    text: its entropy rate is well below its unigram entropy, so a model that learns
    the context beats any context-free predictor.  Every step draws fresh blocks."""
    rng = np.random.Generator(np.random.PCG64(seed))
    fresh = zipf_tokens(rng, (steps, batch, seq_len + 1), vocab, s)
    keep = rng.random(size=(steps, batch, seq_len + 1)) < follow
    blk = fresh.copy()
    for i in range(1, seq_len + 1):
        succ = (blk[:, :, i - 1].astype(np.int64) * 5 + 3) % vocab
        blk[:, :, i] = np.where(keep[:, :, i], succ, fresh[:, :, i])
    return np.ascontiguousarray(blk[:, :, :seq_len]), np.ascontiguousarray(blk[:, :, 1:])


def layer_param_layout(d_model: int, n_head: int, d_head: int, d_ff: int, rel_pos: int):
    """Ordered (name, shape, kind) list of one layer's parameters in the fp32 blob.

    kind: 'w' matrix drawn N(0, std), 'b' bias (zeros), 'g' LayerNorm gain (ones).
    This is the documented parameter-blob order of the C boundary.
    """
    d, f = d_model, d_ff
    out = [("W_qkv", (d, 3 * d), "w"), ("W_o", (d, d), "w")]
    if rel_pos:
        out += [("W_r", (d, d), "w"), ("u", (n_head, d_head), "w"), ("v", (n_head, d_head), "w")]
    out += [("ln1_g", (d,), "g"), ("ln1_b", (d,), "b"),
            ("W_1", (d, f), "w"), ("b_1", (f,), "b"),
            ("W_2", (f, d), "w"), ("b_2", (d,), "b"),
            ("ln2_g", (d,), "g"), ("ln2_b", (d,), "b")]
    return out


def layer_param_count(d_model, n_head, d_head, d_ff, rel_pos) -> int:
    return int(sum(int(np.prod(s)) for _, s, _ in
                   layer_param_layout(d_model, n_head, d_head, d_ff, rel_pos)))


def default_layers_per_module(n_layer: int, n_module: int):
    """Contiguous split; the remainder goes to interior modules first (modules 1 and K
    also carry the embedding / softmax work)."""
    base, rem = divmod(n_layer, n_module)
    sizes = [base] * n_module
    order = list(range(1, n_module - 1)) + [0, n_module - 1]
    for i in range(rem):
        sizes[order[i % n_module]] += 1
    return sizes


def init_params(cfg: dict, seed: int = 0, std: float = 0.02, perturb: float = 0.0):
    """fp32 parameter blobs: [V, module 1, ..., module K].

    Matrices (incl. V, u, v) ~ N(0, std^2); biases 0; LayerNorm gain 1, bias 0.
    perturb>0 adds N(0, perturb^2) noise to biases and gains as well, which makes
    parity tests sensitive to every parameter.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    lay = layer_param_layout(cfg["d_model"], cfg["n_head"], cfg["d_head"], cfg["d_ff"],
                             cfg["rel_pos"])
    lpm = cfg.get("layers_per_module") or default_layers_per_module(cfg["n_layer"],
                                                                    cfg["n_module"])
    blobs = [(rng.standard_normal((cfg["vocab"], cfg["d_model"])) * std).astype(np.float32).ravel()]
    for nl in lpm:
        parts = []
        for _ in range(nl):
            for _, shape, kind in lay:
                n = int(np.prod(shape))
                if kind == "w":
                    a = rng.standard_normal(n) * std
                elif kind == "g":
                    a = np.ones(n) + (rng.standard_normal(n) * perturb if perturb else 0.0)
                else:
                    a = np.zeros(n) + (rng.standard_normal(n) * perturb if perturb else 0.0)
                parts.append(a.astype(np.float32))
        blobs.append(np.concatenate(parts) if parts else np.zeros(0, np.float32))
    return blobs
