"""CPU oracle for the PISA forward pass -- TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what piecewise sparse attention
computes, written from the paper's Methodology section.  Only the tests, the
smoke check and the CPU-baseline leg of the benchmark may import this module;
the product path (the HIP library and its Python binding) never does, and the
two share no code.

Everything here works on ONE head: 2-D arrays `Q, K, V` of shape `[L, d]`
(any float dtype; widened to fp64 on entry).  Notation follows the paper:
block size `B`, `N = ceil(L / B)` blocks, block `j` holds rows
`[jB, min((j+1)B, L))` and has `B_j` rows, `S_i` is the set of key/value blocks
query block `i` attends exactly, `U_i` its complement, `s` the softmax scale.

What is computed (citations are to the paper):

* `block_stats`  -- "Prepare" step of the forward-pass algorithm (Alg. 1)
  with the definitions of the block centroid and of `H_j` from the
  "Formulation" / "Global First-Order Correction" paragraphs.
* `select`       -- block-wise top-k of pooled scores (Alg. 1, "Select" step; the score
  is the covariance-aware score equation; its `log(M_j + eps)` term, which the
  paper switches on for image models only, enters as an optional column bias
  built from `block_heterogeneity`).
* `attention_rows` -- the output definition: `o_t = N_t / D_t` with the exact
  term, the block-wise zeroth-order term and one of the first-order variants
  (block-wise first-order equations; hybrid equations with the global `H`).
* `alg1_forward` -- the same result obtained the way Alg. 1 states it (online
  softmax over tiles, column mask, `diag(l_tail) (Q_i H) / L`).

Readings taken where the paper is silent or inconsistent (each is pinned by a
test in tests/test_oracle_pins.py):

* scale: every formula is used with `q <- s * q`; in particular the
  first-order term is `alpha * (s q_t) H_j` (Taylor expansion of
  `exp(s q k^T)` about the centroid).
* the "global H" of Alg. 1 is the un-normalised sum `H_sum = sum_j H_j` over
  ALL blocks; the algorithm's `l_tail / L * (Q_i H)` then equals the hybrid
  equation's `(sum_U alpha) * q_t * Hbar`, `Hbar = H_sum / N`, provided the
  centroid logits carry `+ ln B` and the centroid "values" are block means.
* ragged last block: means and sums run over its `B_j` valid rows, `B -> B_j`
  in the denominator, and the first-order weight is the token-weighted
  `T / L`, `T = sum_U B_j alpha_j` (identical to the equations when `B | L`).
* selection uses the block-mean query; ties go to the lower block index; the
  index list is returned ascending.
* sparsity r -> k = N - floor(r N + 1e-9) exact blocks.

Parity status: the paper prints no worked numerical example and its code is
not available, so agreement with the authors' own kernel is unpinned; the
definition itself is pinned by closed forms, invariants, convergence orders
and the r = 0 / textbook-softmax special case.
"""
from __future__ import annotations

import math
from typing import Optional, Sequence

import numpy as np

MODES = ("dense", "sparse", "pisa0", "pisa1", "hybrid", "hybrid_eq")


def num_blocks(L: int, B: int) -> int:
    return -(-L // B)


def topk_count(N: int, r: float) -> int:
    """Number of exactly-attended blocks at sparsity r (Implementation Details:
    sparsity = share of blocks handled by the approximation)."""
    return min(N, max(0, N - int(math.floor(r * N + 1e-9))))


def block_sizes(L: int, B: int) -> np.ndarray:
    N = num_blocks(L, B)
    sizes = np.full(N, B, dtype=np.int64)
    sizes[-1] = L - (N - 1) * B
    return sizes


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


# ----------------------------------------------------------------------------
# Prepare: block statistics  (Alg. 1, "Prepare" step)
# ----------------------------------------------------------------------------
def block_stats(Q, K, V, B: int, per_block_H: bool = False):
    """Return dict(qbar[N,d], kbar[N,d], vsum[N,d], hsum[d,d], (Hj[N,d,d])).

    kbar_j = mean of block j's keys           (Formulation paragraph)
    vsum_j = sum  of block j's values         (zeroth-order term)
    H_j    = sum_n (k_{j,n} - kbar_j)^T v_{j,n}   (Global First-Order Correction)
    hsum   = sum over all N blocks of H_j
    """
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    L, d = K.shape
    N = num_blocks(L, B)
    qbar = np.empty((N, d))
    kbar = np.empty((N, d))
    vsum = np.empty((N, d))
    hsum = np.zeros((d, d))
    Hj = np.empty((N, d, d)) if per_block_H else None
    for j in range(N):
        lo, hi = j * B, min((j + 1) * B, L)
        qbar[j] = Q[lo:hi].sum(axis=0) / (hi - lo)
        kbar[j] = K[lo:hi].sum(axis=0) / (hi - lo)
        vsum[j] = V[lo:hi].sum(axis=0)
        Hblk = (K[lo:hi] - kbar[j]).T @ V[lo:hi]
        hsum += Hblk
        if per_block_H:
            Hj[j] = Hblk
    out = dict(qbar=qbar, kbar=kbar, vsum=vsum, hsum=hsum)
    if per_block_H:
        out["Hj"] = Hj
    return out


# ----------------------------------------------------------------------------
# Select: pooled block scores and top-k  (Alg. 1, "Select" step)
# ----------------------------------------------------------------------------
def pooled_logits(qbar, kbar, scale: float) -> np.ndarray:
    return scale * (_f64(qbar) @ _f64(kbar).T)


def block_heterogeneity(Hj, hsum, kind: str = "spectral") -> np.ndarray:
    """M_j = || H_j - Hbar ||, Hbar = hsum / N  (Covariance-Aware Block Selection).
    kind: "spectral" (operator 2-norm, the norm the error analysis uses) or "frobenius"."""
    Hj = _f64(Hj)
    N = Hj.shape[0]
    Dm = Hj - _f64(hsum)[None] / N
    if kind == "spectral":
        return np.array([np.linalg.norm(Dm[j], 2) for j in range(N)])
    if kind == "frobenius":
        return np.sqrt((Dm * Dm).sum(axis=(1, 2)))
    raise ValueError(kind)


def select(qbar, kbar, scale: float, k: int, col_bias=None):
    """Top-k key blocks per query block.

    Returns (idx[N, k] int32 ascending, gap[N]) where gap is the logit
    difference between the k-th and (k+1)-th best block (inf when k is 0 or N).
    Softmax over a row is monotone, so ranking uses the logits directly.
    col_bias[j] (optional) is added to every logit of key block j: with
    col_bias = log(M_j + eps) this is the covariance-aware score.
    """
    z = pooled_logits(qbar, kbar, scale)
    if col_bias is not None:
        z = z + _f64(col_bias)[None, :]
    Nq, N = z.shape
    order = np.argsort(-z, axis=1, kind="stable")       # ties -> lower index first
    idx = np.sort(order[:, :k], axis=1).astype(np.int32)
    if 0 < k < N:
        zs = np.take_along_axis(z, order, axis=1)
        gap = zs[:, k - 1] - zs[:, k]
    else:
        gap = np.full(Nq, np.inf)
    return idx, gap


# ----------------------------------------------------------------------------
# Output definition, equation form
# ----------------------------------------------------------------------------
def attention_rows(Q, K, V, B: int, i: int, S_i: Optional[Sequence[int]], scale: float,
                   mode: str = "hybrid", stats: Optional[dict] = None):
    """Output rows of query block i.  Returns (O[B_i, d], lse[B_i]).

    mode:
      dense     softmax(s Q K^T) V                       (Preliminaries, first equation)
      sparse    keep S_i, drop the rest                  (masked form, second equation)
      pisa0     exact on S_i + block-wise zeroth order on U_i
      pisa1     ... + block-wise first-order term with each block's own H_j
      hybrid    ... + global first-order term, token-weighted: (T / L) (s q_t) H_sum
      hybrid_eq ... + global first-order term as the hybrid equations print it:
                (sum_U alpha) (s q_t) Hbar, Hbar = H_sum / N
    lse = log of the denominator D_t (with the max folded back in).
    """
    assert mode in MODES
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    L, d = K.shape
    N = num_blocks(L, B)
    sizes = block_sizes(L, B)
    Qi = Q[i * B:min((i + 1) * B, L)]
    sq = scale * Qi
    if mode == "dense":
        x = sq @ K.T
        mu = x.max(axis=1, keepdims=True)
        p = np.exp(x - mu)
        D = p.sum(axis=1, keepdims=True)
        return (p @ V) / D, (mu + np.log(D))[:, 0]

    S = np.zeros(N, dtype=bool)
    S[np.asarray(S_i, dtype=np.int64)] = True
    U = ~S
    tok_sel = np.repeat(S, sizes)                      # per-token membership of S_i
    if stats is None:
        stats = block_stats(Q, K, V, B, per_block_H=(mode == "pisa1"))
    kbar, vsum = stats["kbar"], stats["vsum"]

    x = sq @ K[tok_sel].T                              # exact logits   [B_i, |S| tokens]
    a = sq @ kbar[U].T                                 # centroid logits [B_i, |U|]
    Bu = sizes[U].astype(np.float64)
    use_tail = mode != "sparse"
    cands = [x.max(axis=1)] if x.shape[1] else []
    if use_tail and a.shape[1]:
        cands.append((a + np.log(Bu)).max(axis=1))
    mu = np.max(np.stack(cands, axis=0), axis=0)[:, None]
    p = np.exp(x - mu)
    D = p.sum(axis=1, keepdims=True)
    Num = p @ V[tok_sel]
    if use_tail:
        alpha = np.exp(a - mu)                         # alpha_{t,j}, shifted by the row max
        T = (alpha * Bu).sum(axis=1, keepdims=True)    # tail mass: sum_U B_j alpha_j
        D = D + T
        Num = Num + alpha @ vsum[U]                    # zeroth order: alpha_j * (sum_n v_{j,n})
        if mode == "pisa1":
            Hu = stats["Hj"][U]                        # [|U|, d, d]
            Num = Num + np.einsum("tu,tc,ucd->td", alpha, sq, Hu)
        elif mode == "hybrid":
            Num = Num + (T / L) * (sq @ stats["hsum"])
        elif mode == "hybrid_eq":
            Num = Num + alpha.sum(axis=1, keepdims=True) * (sq @ (stats["hsum"] / N))
    return Num / D, (mu + np.log(D))[:, 0]


def attention_head(Q, K, V, B: int, idx: Optional[np.ndarray], scale: float,
                   mode: str = "hybrid", blocks: Optional[Sequence[int]] = None,
                   stats: Optional[dict] = None):
    """All (or the listed) query blocks of one head.  Returns (O, lse) for those rows,
    concatenated in the order of `blocks`."""
    Q = _f64(Q)
    L = Q.shape[0]
    N = num_blocks(L, B)
    blocks = range(N) if blocks is None else blocks
    if stats is None and mode not in ("dense", "sparse"):
        stats = block_stats(Q, K, V, B, per_block_H=(mode == "pisa1"))
    outs, lses = [], []
    for i in blocks:
        S_i = None if mode == "dense" else idx[i]
        o, l = attention_rows(Q, K, V, B, i, S_i, scale, mode, stats)
        outs.append(o)
        lses.append(l)
    return np.concatenate(outs, axis=0), np.concatenate(lses, axis=0)


# ----------------------------------------------------------------------------
# The same result the way the forward-pass algorithm states it  (Alg. 1, the loop over query blocks (its three phases))
# ----------------------------------------------------------------------------
def alg1_forward(Q, K, V, B: int, C: int, idx: np.ndarray, scale: float,
                 stats: Optional[dict] = None, blocks: Optional[Sequence[int]] = None):
    """Online-softmax tile loop: Phase 1 over the selected blocks, Phase 2 over
    groups of C centroids with the selected columns masked, Phase 3 adding
    diag(l_tail) (Q_i H) / L, then the division by l.  The safe-softmax steps the
    listing leaves out are written in; centroid logits carry + ln B_j and the
    centroid values are block means (see module header)."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    L, d = K.shape
    N = num_blocks(L, B)
    sizes = block_sizes(L, B).astype(np.float64)
    if stats is None:
        stats = block_stats(Q, K, V, B)
    kbar, hsum = stats["kbar"], stats["hsum"]
    vbar = stats["vsum"] / sizes[:, None]
    blocks = range(N) if blocks is None else blocks
    outs = []
    for i in blocks:
        Qi = scale * Q[i * B:min((i + 1) * B, L)]
        rows = Qi.shape[0]
        O = np.zeros((rows, d))
        ell = np.zeros(rows)
        ell_tail = np.zeros(rows)
        m = np.full(rows, -np.inf)

        def absorb(S_tile, V_tile, tail):
            nonlocal O, ell, ell_tail, m
            m_new = np.maximum(m, S_tile.max(axis=1))
            live = np.isfinite(m_new)
            m_safe = np.where(live, m_new, 0.0)
            corr = np.where(live, np.exp(m - m_safe), 1.0)
            P = np.exp(S_tile - m_safe[:, None])
            O = O * corr[:, None] + P @ V_tile
            ell = ell * corr + P.sum(axis=1)
            ell_tail = ell_tail * corr + (P.sum(axis=1) if tail else 0.0)
            m = m_new

        for j in idx[i]:                                        # Phase 1
            lo, hi = j * B, min((j + 1) * B, L)
            absorb(Qi @ K[lo:hi].T, V[lo:hi], tail=False)
        chosen = np.zeros(N, dtype=bool)
        chosen[idx[i]] = True
        for g in range(0, N, C):                                # Phase 2
            cols = slice(g, min(g + C, N))
            S_tile = Qi @ kbar[cols].T + np.log(sizes[cols])[None, :]
            S_tile[:, chosen[cols]] = -np.inf                   # column masking
            absorb(S_tile, vbar[cols], tail=True)
        R = ell_tail[:, None] * (Qi @ hsum) / L                 # Phase 3
        outs.append((O + R) / ell[:, None])
    return np.concatenate(outs, axis=0)


def pisa_forward(Q, K, V, B: int, r: float, scale: Optional[float] = None,
                 mode: str = "hybrid"):
    """Whole head, end to end: stats -> select -> attention.  Returns (O, idx, lse)."""
    Q, K, V = _f64(Q), _f64(K), _f64(V)
    L, d = Q.shape
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    N = num_blocks(L, B)
    st = block_stats(Q, K, V, B, per_block_H=(mode == "pisa1"))
    idx, _ = select(st["qbar"], st["kbar"], scale, topk_count(N, r))
    O, lse = attention_head(Q, K, V, B, idx, scale, mode, stats=st)
    return O, idx, lse
