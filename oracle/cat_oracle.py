"""fp64 CPU oracle for the Confidence-Adaptive Token (CAT) weighted loss of PARD-2.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
library is checked against.  It shares no code with the HIP path and must never
be imported by it; only tests, the smoke check and the benchmark's CPU-baseline
leg may call it.

Everything is evaluated in float64 from the stored (already rounded) inputs:

  * head logits  z[t,v] = sum_i H[t,i] W[v,i]                (the head of Eq.4/5)
  * log-softmax  log q_t(v) = z[t,v] - logsumexp_v z[t,v]     (Eq.5, the log P term)
  * confidence   c_t: the teacher's probability of the ground-truth token (Eq.9);
                 passed in as `conf_in`, or, in the self-teacher instance where
                 the head given plays the teacher's role too, c_t = q_t(y_t)
  * CAT weight   s[b,0] = 1, s[b,k] = s[b,k-1] * c[b,k-1]     (Eq.10)
  * loss         (beta / N) * sum_t w_t * (-log q_t(y_t))     (Eq.11; beta of Eq.12)
  * gradients    with the weight held constant (stop-gradient, text before Eq.11)
  * diagnostics  greedy argmax, accepted-prefix length (longest run of leading
                 hits, Sec.2.1 last paragraph), estimated acceptance length
                 sum_k s_k c_k (Eq.8 with the estimates of Eq.9/10)

A library matmul (numpy float64 `@`) serves as the contraction step.  Rows are
handled in slabs purely to bound memory: every row is independent of the others
in the forward pass, and the backward sums over rows are plain accumulations.

Readings of the paper where it is silent (also listed in the design notes):
  normaliser  MEAN_VALID divides by the number of valid (block, slot) tokens, which
              equals Eq.11's 1/K averaged over anchors when all blocks are full;
              SUM does not divide (Eq.12 as printed).
  ignored     a slot whose target is `ignore_index`, or that lies at k >= valid_len[b],
              carries no loss or gradient; the product of Eq.10 runs through an
              ignored slot with its conf_in (external) or with c := 1 (self-teacher).
  ties        argmax is the lowest index attaining the maximum.
Parity unpinned by the paper: normaliser, beta placement, self-teacher mode and the
ignored-slot rule follow the readings above.
"""
from __future__ import annotations

import numpy as np

W_CAT, W_DECAY, W_UNIFORM = 0, 1, 2
RED_MEAN_VALID, RED_SUM = 0, 1


# --------------------------------------------------------------------------
# step 1-2: head logits and per-row softmax statistics
# --------------------------------------------------------------------------
def head_logits(H, W, rows=None):
    """z[rows, :] = H[rows] @ W^T in float64."""
    H = np.asarray(H, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    Hr = H if rows is None else H[rows]
    return Hr @ W.T


def head_stats(H, W, y, ignore_index=-100, slab=256, W64=None):
    """Per-row statistics of the head's softmax.

    Returns dict with float64 `m` (row max), `lse`, `logq` (log-prob of the target,
    0 on ignored rows), `gap` (top-1 minus top-2 logit) and int64 `argmax`.
    """
    H = np.asarray(H)
    T = H.shape[0]
    W64 = np.asarray(W, dtype=np.float64) if W64 is None else W64
    V = W64.shape[0]
    y = np.asarray(y).astype(np.int64)
    m = np.empty(T)
    lse = np.empty(T)
    logq = np.zeros(T)
    gap = np.empty(T)
    amax = np.empty(T, dtype=np.int64)
    for r0 in range(0, T, slab):
        r1 = min(T, r0 + slab)
        Z = np.asarray(H[r0:r1], dtype=np.float64) @ W64.T
        a = np.argmax(Z, axis=1)                 # first index attaining the max
        rows = np.arange(r1 - r0)
        mm = Z[rows, a]
        amax[r0:r1] = a
        m[r0:r1] = mm
        lse[r0:r1] = mm + np.log(np.sum(np.exp(Z - mm[:, None]), axis=1))
        yy = y[r0:r1]
        ok = yy != ignore_index
        if np.any(ok & ((yy < 0) | (yy >= V))):
            raise ValueError("target id out of range")
        logq[r0:r1][ok] = Z[rows[ok], yy[ok]] - lse[r0:r1][ok]
        if V > 1:
            Z[rows, a] = -np.inf
            gap[r0:r1] = mm - Z.max(axis=1)
        else:
            gap[r0:r1] = np.inf
    return {"m": m, "lse": lse, "logq": logq, "gap": gap, "argmax": amax}


def target_logq(H, W64, y, lse, ignore_index=-100):
    """log q_t(y_t) = z[t, y_t] - lse_t from already known lse (0 on ignored rows).

    Lets a caller that holds the y-independent statistics (lse, argmax) of a head
    attach targets afterwards; z[t, y_t] is the plain dot product of the definition.
    """
    H64 = np.asarray(H, dtype=np.float64)
    y = np.asarray(y).astype(np.int64)
    out = np.zeros(len(y))
    has = y != ignore_index
    if np.any(has & ((y < 0) | (y >= W64.shape[0]))):
        raise ValueError("target id out of range")
    out[has] = np.sum(H64[has] * W64[y[has]], axis=1) - np.asarray(lse)[has]
    return out


# --------------------------------------------------------------------------
# step 3-4: confidences and CAT weights
# --------------------------------------------------------------------------
def cat_weights(conf, B, K, valid_len=None, mode=W_CAT, gamma=1.0):
    """Unmasked importance s[B*K] and estimated acceptance length exp_len[B].

    CAT:     s[b,0] = 1, s[b,k] = s[b,k-1] * conf[b,k-1]   (Eq.10), left-to-right.
    DECAY:   s[b,k] = gamma**k   (fixed position decay of the ablation, Table 3).
    UNIFORM: s = 1               (Eq.5).
    exp_len[b] = sum_{k < K_b} s[b,k] * conf[b,k]          (Eq.8 with Eq.9/10).
    """
    conf = np.asarray(conf, dtype=np.float64).reshape(B, K)
    vl = np.full(B, K, dtype=np.int64) if valid_len is None else np.asarray(valid_len, dtype=np.int64)
    s = np.empty((B, K))
    exp_len = np.zeros(B)
    for b in range(B):
        run = 1.0
        for k in range(K):
            if mode == W_CAT:
                s[b, k] = run
                run = run * conf[b, k]
            elif mode == W_DECAY:
                s[b, k] = float(gamma) ** k
            elif mode == W_UNIFORM:
                s[b, k] = 1.0
            else:
                raise ValueError("unknown weight mode")
            if k < vl[b]:
                exp_len[b] += s[b, k] * conf[b, k]
    return s.reshape(B * K), exp_len


def cat_weights_seq(c_seq, anchor_pos, seq_end, K):
    """Anchor-dependent weights of Sec.3.3 from per-position teacher confidences.

    For block b anchored at position n = anchor_pos[b] of a sequence ending (exclusively) at
    seq_end[b]:  conf[b,k] = c_seq[n + k] and  s[b,k] = prod_{j<k} c_seq[n + j]  (Eq.10 with the
    anchor made explicit), for the slots that exist, n + k < seq_end[b] (Eq.12 sums, for offset k,
    the anchors n <= N - k only).  Non-existing slots get conf = 1 and are excluded by valid_len.
    Returns (conf[B*K], valid_len[B], s[B*K], exp_len[B]).
    """
    c_seq = np.asarray(c_seq, dtype=np.float64)
    anchor_pos = np.asarray(anchor_pos, dtype=np.int64)
    seq_end = np.asarray(seq_end, dtype=np.int64)
    B = len(anchor_pos)
    conf = np.ones((B, K))
    s = np.ones((B, K))
    vl = np.zeros(B, dtype=np.int64)
    exp_len = np.zeros(B)
    for b in range(B):
        n = anchor_pos[b]
        end = min(seq_end[b], len(c_seq))
        vl[b] = 0 if n < 0 else max(0, min(K, end - n))
        for k in range(K):
            if k < vl[b]:
                conf[b, k] = c_seq[n + k]
            s[b, k] = np.prod(conf[b, :k])          # the definition: product over j < k
            if k < vl[b]:
                exp_len[b] += s[b, k] * conf[b, k]
    return conf.reshape(B * K), vl, s.reshape(B * K), exp_len


def valid_mask(y, B, K, valid_len=None, ignore_index=-100):
    """Boolean [T]: slot lies below its block's valid length and has a real target."""
    y = np.asarray(y).reshape(B, K)
    vl = np.full(B, K, dtype=np.int64) if valid_len is None else np.asarray(valid_len, dtype=np.int64)
    slot = np.arange(K)[None, :]
    return ((slot < vl[:, None]) & (y != ignore_index)).reshape(B * K)


def accepted_prefix(hit, B, K, valid_len=None):
    """accept_len[b]: number of leading slots k < K_b whose greedy prediction hits the target."""
    hit = np.asarray(hit, dtype=bool).reshape(B, K)
    vl = np.full(B, K, dtype=np.int64) if valid_len is None else np.asarray(valid_len, dtype=np.int64)
    out = np.zeros(B, dtype=np.int64)
    for b in range(B):
        n = 0
        while n < vl[b] and hit[b, n]:
            n += 1
        out[b] = n
    return out


# --------------------------------------------------------------------------
# steps 1-5 and 7: forward
# --------------------------------------------------------------------------
def cat_forward(H, W, y, B, K, conf_in=None, valid_len=None, mode=W_CAT, gamma=1.0,
                beta=1.0, reduction=RED_MEAN_VALID, ignore_index=-100, slab=256, W64=None,
                stats=None):
    """CAT-weighted loss forward.  Returns a dict of float64/int64 arrays and scalars."""
    T = B * K
    y = np.asarray(y).astype(np.int64).reshape(T)
    st = head_stats(H, W, y, ignore_index, slab, W64) if stats is None else stats
    valid = valid_mask(y, B, K, valid_len, ignore_index)
    has_target = y != ignore_index
    if conf_in is not None:
        conf = np.asarray(conf_in, dtype=np.float64).reshape(T)
    else:
        conf = np.where(has_target, np.exp(st["logq"]), 1.0)
    s, exp_len = cat_weights(conf, B, K, valid_len, mode, gamma)
    w = np.where(valid, s, 0.0)
    n_valid = int(valid.sum())
    n_norm = float(n_valid) if reduction == RED_MEAN_VALID else 1.0
    if reduction == RED_MEAN_VALID and n_valid == 0:
        loss = 0.0
    else:
        loss = (beta / n_norm) * float(np.sum(w * (-st["logq"])))
    hit = has_target & (st["argmax"] == y)
    return {
        "loss": loss, "lse": st["lse"], "logq": st["logq"], "conf": conf, "s": s, "w": w,
        "argmax": st["argmax"], "gap": st["gap"], "m": st["m"], "hit": hit,
        "accept_len": accepted_prefix(hit, B, K, valid_len), "exp_len": exp_len,
        "n_valid": n_valid, "n_norm": n_norm,
    }


# --------------------------------------------------------------------------
# step 6: backward with the weight held constant
# --------------------------------------------------------------------------
def row_scale(w, beta, n_valid, reduction=RED_MEAN_VALID, gout=1.0):
    """g_t = gout * beta * w_t / N  (all zero when a MEAN_VALID batch has no valid token)."""
    w = np.asarray(w, dtype=np.float64)
    if reduction == RED_MEAN_VALID:
        if n_valid == 0:
            return np.zeros_like(w)
        return gout * beta * w / float(n_valid)
    return gout * beta * w


def cat_backward(H, W, y, lse, g, ignore_index=-100, slab=256, rows=None, vrows=None, W64=None):
    """dH = dZ @ W and dW = dZ^T @ H with dZ[t,v] = g_t * (q_t[v] - 1[v == y_t]).

    `rows`:  if given, dH is returned only for these token rows ([len(rows), d]).
    `vrows`: if given, dW is returned only for these vocabulary rows ([len(vrows), d]).
    Passing one of them skips the other output unless both are given.
    """
    H64 = np.asarray(H, dtype=np.float64)
    W64 = np.asarray(W, dtype=np.float64) if W64 is None else W64
    T, d = H64.shape
    V = W64.shape[0]
    y = np.asarray(y).astype(np.int64).reshape(T)
    lse = np.asarray(lse, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    want_dH = rows is not None or vrows is None
    want_dW = vrows is not None or rows is None
    out = {}
    if want_dH:
        rsel = np.arange(T) if rows is None else np.asarray(rows, dtype=np.int64)
        dH = np.zeros((len(rsel), d))
        for i0 in range(0, len(rsel), slab):
            r = rsel[i0:i0 + slab]
            Q = np.exp(H64[r] @ W64.T - lse[r][:, None])          # q_t[v]
            hot = np.zeros_like(Q)
            has = y[r] != ignore_index
            hot[np.arange(len(r))[has], y[r][has]] = 1.0
            dZ = g[r][:, None] * (Q - hot)
            dH[i0:i0 + slab] = dZ @ W64
        out["dH"] = dH
    if want_dW:
        vsel = np.arange(V) if vrows is None else np.asarray(vrows, dtype=np.int64)
        Wv = W64[vsel]
        dW = np.zeros((len(vsel), d))
        # column position of every target id inside vsel (-1 if absent)
        pos = np.full(V, -1, dtype=np.int64)
        pos[vsel] = np.arange(len(vsel))
        for r0 in range(0, T, slab):
            r1 = min(T, r0 + slab)
            Q = np.exp(H64[r0:r1] @ Wv.T - lse[r0:r1][:, None])
            hot = np.zeros_like(Q)
            yy = y[r0:r1]
            has = yy != ignore_index
            col = np.where(has, pos[np.where(has, yy, 0)], -1)
            sel = col >= 0
            hot[np.arange(r1 - r0)[sel], col[sel]] = 1.0
            dZ = g[r0:r1][:, None] * (Q - hot)
            dW += dZ.T @ H64[r0:r1]
        out["dW"] = dW
    return out


def cat_loss_and_grads(H, W, y, B, K, conf_in=None, valid_len=None, mode=W_CAT, gamma=1.0,
                       beta=1.0, reduction=RED_MEAN_VALID, ignore_index=-100, gout=1.0, slab=256):
    """Forward + full backward (small problems)."""
    W64 = np.asarray(W, dtype=np.float64)
    f = cat_forward(H, W, y, B, K, conf_in, valid_len, mode, gamma, beta, reduction,
                    ignore_index, slab, W64)
    g = row_scale(f["w"], beta, f["n_valid"], reduction, gout)
    b = cat_backward(H, W, y, f["lse"], g, ignore_index, slab, W64=W64)
    f.update(b)
    f["g"] = g
    return f
