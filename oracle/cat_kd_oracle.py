"""fp64 CPU oracle for the full PARD-2 token loss  s_{n,k} * (beta * CE + KD)  (Eq.12).

TEST INFRASTRUCTURE ONLY, like cat_oracle.py beside it (whose weight, mask and
prefix-length routines it reuses): it shares no code with the HIP library and must
never be imported by it.

Eq.12 adds a distillation term L^KD to the weighted cross-entropy of Eq.11 without
defining it.  The reading taken here (parity unpinned by the paper):

  teacher   p_t = softmax(Ht[t] . Wt^T): the target model's next-token distribution under
            teacher forcing, i.e. the very distribution whose entry at the ground-truth
            token is the confidence c of Eq.9.  Ht[T, dt], Wt[V, dt] are the target model's
            final hidden states (gathered token-major by the caller) and LM head.
  KD        forward KL at temperature 1:  KD_t = sum_v p_t[v] (log p_t[v] - log q_t[v]),
            q_t the draft's distribution; no gradient flows into the teacher.
  loss      (1/N) sum_t w_t (beta * (-log q_t(y_t)) + KD_t), w the stop-gradient CAT
            weight (Eq.10) with the same masks and normaliser as the CE-only loss.
  c         conf_in if given, else the teacher head's own p_t(y_t) (Eq.9 as printed).
  gradient  dZ[t,v] = g_t (beta (q_t[v] - 1[v = y_t]) + q_t[v] - p_t[v]),  g_t = gout w_t / N.

Everything is float64 from the stored inputs; numpy `@` is the contraction step; rows
go in slabs only to bound memory.
"""
from __future__ import annotations

import numpy as np

from . import cat_oracle as O


def kd_stats(H, W64, Ht, Wt64, y, ignore_index=-100, slab=128, rows=None):
    """Per-row statistics of both heads for token rows `rows` (default all).

    Returns float64 `lse`, `lse_t` (draft / teacher log-sum-exp), `logq`, `logp_t` (draft /
    teacher log-prob of the target; 0 on ignored rows), `kd` (KL(p_t || q_t), by its
    definition), `m`, `gap` and int64 `argmax` of the draft head.
    """
    H = np.asarray(H)
    Ht = np.asarray(Ht)
    T = H.shape[0]
    rsel = np.arange(T) if rows is None else np.asarray(rows, dtype=np.int64)
    V = W64.shape[0]
    y = np.asarray(y).astype(np.int64)
    n = len(rsel)
    out = {k: np.zeros(n) for k in ("lse", "lse_t", "logq", "logp_t", "kd", "m", "gap")}
    out["argmax"] = np.zeros(n, dtype=np.int64)
    for i0 in range(0, n, slab):
        r = rsel[i0:i0 + slab]
        ar = np.arange(len(r))
        Zd = np.asarray(H[r], dtype=np.float64) @ W64.T
        Zt = np.asarray(Ht[r], dtype=np.float64) @ Wt64.T
        a = np.argmax(Zd, axis=1)
        md = Zd[ar, a]
        lse_d = md + np.log(np.sum(np.exp(Zd - md[:, None]), axis=1))
        mt = Zt.max(axis=1)
        lse_t = mt + np.log(np.sum(np.exp(Zt - mt[:, None]), axis=1))
        logQ = Zd - lse_d[:, None]
        logP = Zt - lse_t[:, None]
        P = np.exp(logP)
        sl = slice(i0, i0 + len(r))
        out["kd"][sl] = np.sum(P * (logP - logQ), axis=1)
        out["lse"][sl], out["lse_t"][sl], out["m"][sl], out["argmax"][sl] = lse_d, lse_t, md, a
        yy = y[r]
        ok = yy != ignore_index
        if np.any(ok & ((yy < 0) | (yy >= V))):
            raise ValueError("target id out of range")
        out["logq"][sl][ok] = logQ[ar[ok], yy[ok]]
        out["logp_t"][sl][ok] = logP[ar[ok], yy[ok]]
        if V > 1:
            Zd[ar, a] = -np.inf
            out["gap"][sl] = md - Zd.max(axis=1)
        else:
            out["gap"][sl] = np.inf
    return out


def cat_kd_forward(H, W, Ht, Wt, y, B, K, conf_in=None, valid_len=None, mode=O.W_CAT, gamma=1.0,
                   beta=0.1, reduction=O.RED_MEAN_VALID, ignore_index=-100, slab=128, stats=None):
    """Forward of the weighted (beta CE + KD) loss.  Returns a dict like cat_forward's plus
    `kd`, `lse_t`, `logp_t`."""
    T = B * K
    y = np.asarray(y).astype(np.int64).reshape(T)
    if stats is None:
        stats = kd_stats(H, np.asarray(W, dtype=np.float64), Ht, np.asarray(Wt, dtype=np.float64), y,
                         ignore_index, slab)
    st = stats
    valid = O.valid_mask(y, B, K, valid_len, ignore_index)
    has_target = y != ignore_index
    if conf_in is not None:
        conf = np.asarray(conf_in, dtype=np.float64).reshape(T)
    else:
        conf = np.where(has_target, np.exp(st["logp_t"]), 1.0)        # Eq.9: the teacher's p(y)
    s, exp_len = O.cat_weights(conf, B, K, valid_len, mode, gamma)
    w = np.where(valid, s, 0.0)
    n_valid = int(valid.sum())
    n_norm = float(n_valid) if reduction == O.RED_MEAN_VALID else 1.0
    tok = beta * (-st["logq"]) + st["kd"]
    if reduction == O.RED_MEAN_VALID and n_valid == 0:
        loss = 0.0
    else:
        loss = float(np.sum(w * np.where(valid, tok, 0.0))) / n_norm
    hit = has_target & (st["argmax"] == y)
    return {
        "loss": loss, "lse": st["lse"], "lse_t": st["lse_t"], "logq": st["logq"], "logp_t": st["logp_t"],
        "kd": st["kd"], "conf": conf, "s": s, "w": w, "argmax": st["argmax"], "gap": st["gap"],
        "hit": hit, "accept_len": O.accepted_prefix(hit, B, K, valid_len), "exp_len": exp_len,
        "n_valid": n_valid, "n_norm": n_norm,
    }


def kd_row_scale(w, n_valid, reduction=O.RED_MEAN_VALID, gout=1.0):
    """g_t = gout * w_t / N (beta sits inside the bracket of Eq.12, not here)."""
    return O.row_scale(w, 1.0, n_valid, reduction, gout)


def cat_kd_backward(H, W, Ht, Wt, y, lse, lse_t, g, beta, ignore_index=-100, slab=128, rows=None,
                    vrows=None):
    """dH = dZ @ W, dW = dZ^T @ H of the draft head with
    dZ[t,v] = g_t (beta (q_t[v] - 1[v = y_t]) + q_t[v] - p_t[v]).
    `rows` / `vrows` select token rows of dH / vocabulary rows of dW as in cat_backward."""
    H64 = np.asarray(H, dtype=np.float64)
    W64 = np.asarray(W, dtype=np.float64)
    Ht64 = np.asarray(Ht, dtype=np.float64)
    Wt64 = np.asarray(Wt, dtype=np.float64)
    T, d = H64.shape
    V = W64.shape[0]
    y = np.asarray(y).astype(np.int64).reshape(T)
    lse = np.asarray(lse, dtype=np.float64)
    lse_t = np.asarray(lse_t, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    want_dH = rows is not None or vrows is None
    want_dW = vrows is not None or rows is None
    out = {}

    def dz(r, vsel):
        Wd = W64 if vsel is None else W64[vsel]
        Wtt = Wt64 if vsel is None else Wt64[vsel]
        Q = np.exp(H64[r] @ Wd.T - lse[r][:, None])
        P = np.exp(Ht64[r] @ Wtt.T - lse_t[r][:, None])
        hot = np.zeros_like(Q)
        yy = y[r]
        has = yy != ignore_index
        if vsel is None:
            col = np.where(has, yy, -1)
        else:
            pos = np.full(V, -1, dtype=np.int64)
            pos[vsel] = np.arange(len(vsel))
            col = np.where(has, pos[np.where(has, yy, 0)], -1)
        sel = col >= 0
        hot[np.arange(len(r))[sel], col[sel]] = 1.0
        return g[r][:, None] * (beta * (Q - hot) + (Q - P))

    if want_dH:
        rsel = np.arange(T) if rows is None else np.asarray(rows, dtype=np.int64)
        dH = np.zeros((len(rsel), d))
        for i0 in range(0, len(rsel), slab):
            r = rsel[i0:i0 + slab]
            dH[i0:i0 + slab] = dz(r, None) @ W64
        out["dH"] = dH
    if want_dW:
        vsel = None if vrows is None else np.asarray(vrows, dtype=np.int64)
        dW = np.zeros((V if vsel is None else len(vsel), d))
        for r0 in range(0, T, slab):
            r = np.arange(r0, min(T, r0 + slab))
            dW += dz(r, vsel).T @ H64[r]
        out["dW"] = dW
    return out


def cat_kd_loss_and_grads(H, W, Ht, Wt, y, B, K, conf_in=None, valid_len=None, mode=O.W_CAT, gamma=1.0,
                          beta=0.1, reduction=O.RED_MEAN_VALID, ignore_index=-100, gout=1.0):
    """Forward + full backward (small problems)."""
    f = cat_kd_forward(H, W, Ht, Wt, y, B, K, conf_in, valid_len, mode, gamma, beta, reduction, ignore_index)
    g = kd_row_scale(f["w"], f["n_valid"], reduction, gout)
    f.update(cat_kd_backward(H, W, Ht, Wt, y, f["lse"], f["lse_t"], g, beta, ignore_index))
    f["g"] = g
    return f
