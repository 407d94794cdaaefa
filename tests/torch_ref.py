"""An independent autograd model built from torch library routines (CPU, fp64).

Used only to pin the numpy oracle: same reading of the layer, but written with
F.layer_norm / F.gelu / softmax / F.cross_entropy / F.embedding and autograd instead
of hand-derived backward formulas, and with the Transformer-XL position term built
from an explicit per-pair table R[i, j] = sinusoid(p_i - p_j) instead of a gather.
"""
import math

import torch
import torch.nn.functional as F


def sinusoid_t(pos, d):
    m = torch.arange(d // 2, dtype=torch.float64)
    ang = pos.to(torch.float64)[..., None] * torch.pow(torch.tensor(10000.0, dtype=torch.float64), -2.0 * m / d)
    return torch.cat([torch.sin(ang), torch.cos(ang)], dim=-1)


def layer_forward(cfg, p, h, mem=None, m1=None, m2=None):
    """One block on h [B,T,d] (mem: constant [B,Mv,d] or None; m1, m2: constant dropout masks,
    already scaled, on the attention-projection and feed-forward outputs)."""
    B, T, _ = h.shape
    d, H, dh = cfg.d_model, cfg.n_head, cfg.d_head
    Mv = 0 if mem is None else mem.shape[1]
    cat = h if Mv == 0 else torch.cat([mem, h], dim=1)
    S = Mv + T
    q = (h @ p["W_qkv"][:, :d]).view(B, T, H, dh).permute(0, 2, 1, 3)
    k = (cat @ p["W_qkv"][:, d:2 * d]).view(B, S, H, dh).permute(0, 2, 1, 3)
    v = (cat @ p["W_qkv"][:, 2 * d:]).view(B, S, H, dh).permute(0, 2, 1, 3)
    pi = torch.arange(T)[:, None] + Mv
    pj = torch.arange(S)[None, :]
    if cfg.rel_pos:
        rel = (pi - pj).clamp(min=0)                       # [T,S]
        Rij = sinusoid_t(rel, d)                           # [T,S,d] explicit per-pair table
        rij = (Rij @ p["W_r"]).view(T, S, H, dh)
        s = torch.einsum("bhic,bhjc->bhij", q + p["u"][None, :, None, :], k) \
            + torch.einsum("bhic,ijhc->bhij", q + p["v"][None, :, None, :], rij)
    else:
        s = q @ k.transpose(-1, -2)
    s = s / math.sqrt(dh)
    s = s.masked_fill((pj > pi)[None, None], float("-inf"))
    a = (torch.softmax(s, dim=-1) @ v).permute(0, 2, 1, 3).reshape(B, T, d)
    o = a @ p["W_o"]
    if m1 is not None:
        o = o * m1
    y = F.layer_norm(h + o, (d,), p["ln1_g"], p["ln1_b"], 1e-5)
    f = F.gelu(y @ p["W_1"] + p["b_1"]) @ p["W_2"] + p["b_2"]
    if m2 is not None:
        f = f * m2
    return F.layer_norm(y + f, (d,), p["ln2_g"], p["ln2_b"], 1e-5)


def embed(cfg, Vi, tokens):
    h = cfg.emb_scale * F.embedding(tokens, Vi)
    if not cfg.rel_pos:
        h = h + sinusoid_t(torch.arange(tokens.shape[1]), cfg.d_model)[None]
    return h


def forward(cfg, layers, Vi, Vo, tokens, targets, mems=None, masks=None):
    """layers: list of dicts of torch fp64 tensors (requires_grad leaves).  masks: optional dict
    of constant dropout masks, keys "emb" and (layer, site)."""
    B, T = tokens.shape
    h = embed(cfg, Vi, tokens)
    if masks is not None:
        h = h * masks["emb"]
    inputs = []
    for l, p in enumerate(layers):
        inputs.append(h)
        h = layer_forward(cfg, p, h, None if mems is None else mems[l],
                          None if masks is None else masks[(l, 1)], None if masks is None else masks[(l, 2)])
    logits = h @ Vo.t()
    loss = F.cross_entropy(logits.view(B * T, -1), targets.reshape(-1).long(), reduction="mean")
    return loss, inputs
