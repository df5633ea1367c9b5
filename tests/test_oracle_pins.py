"""Pins for the CPU oracle: closed forms, invariants, convergence orders and
special cases that the paper and the mathematics fix.  No GPU, no HIP code.

Each test names the passage of the paper it rests on.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import pisa_oracle as po

RNG = np.random.default_rng(1234)
HERE = os.path.dirname(os.path.abspath(__file__))


def rand_qkv(L, d, rng=RNG, spread=1.0):
    return (rng.standard_normal((L, d)), spread * rng.standard_normal((L, d)),
            rng.standard_normal((L, d)))


def random_idx(N, k, rng=RNG):
    return np.stack([np.sort(rng.choice(N, size=k, replace=False)) for _ in range(N)]).astype(np.int32) \
        if k > 0 else np.zeros((N, 0), dtype=np.int32)


# --- P1: r = 0 is dense attention; dense is the textbook softmax --------------------
@pytest.mark.parametrize("L,B", [(96, 16), (100, 16), (64, 64)])
def test_all_blocks_exact_equals_dense(L, B):
    """With U_i empty every term of N_t and D_t is the exact one (Formulation)."""
    d = 8
    Q, K, V = rand_qkv(L, d)
    s = 1 / math.sqrt(d)
    N = po.num_blocks(L, B)
    idx = np.tile(np.arange(N, dtype=np.int32), (N, 1))
    Od, lsed = po.attention_head(Q, K, V, B, None, s, "dense")
    for mode in ("sparse", "pisa0", "pisa1", "hybrid"):
        O, lse = po.attention_head(Q, K, V, B, idx, s, mode)
        assert np.abs(O - Od).max() < 1e-12
        assert np.abs(lse - lsed).max() < 1e-12
    assert np.abs(po.alg1_forward(Q, K, V, B, 3, idx, s) - Od).max() < 1e-12


def test_dense_is_library_softmax_attention():
    """Preliminaries, first equation, against torch's fp64 CPU attention routine."""
    L, d = 77, 16
    Q, K, V = rand_qkv(L, d)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None])[0].numpy()
    O, lse = po.attention_head(Q, K, V, 16, None, 1 / math.sqrt(d), "dense")
    assert np.abs(O - ref).max() < 1e-12
    ref_lse = torch.logsumexp(torch.from_numpy(Q @ K.T) / math.sqrt(d), dim=1).numpy()
    assert np.abs(lse - ref_lse).max() < 1e-12


# --- P2: coincident keys make the expansion exact ------------------------------------
@pytest.mark.parametrize("L,B,k", [(96, 16, 0), (96, 16, 2), (90, 16, 1), (90, 16, 0)])
def test_coincident_keys_exact_for_any_selection(L, B, k):
    """If every key of a block equals its centroid, alpha_{t,j} is the exact
    exponential for each of the block's B_j keys and H_j = 0, so all variants
    equal dense attention whatever S_i is (Formulation equations)."""
    d = 8
    N = po.num_blocks(L, B)
    Q, _, V = rand_qkv(L, d)
    cent = RNG.standard_normal((N, d))
    K = np.repeat(cent, B, axis=0)[:L]
    s = 0.4
    idx = random_idx(N, k)
    Od, lsed = po.attention_head(Q, K, V, B, None, s, "dense")
    for mode in ("pisa0", "pisa1", "hybrid"):
        O, lse = po.attention_head(Q, K, V, B, idx, s, mode)
        assert np.abs(O - Od).max() < 1e-12, mode
        assert np.abs(lse - lsed).max() < 1e-12, mode
    assert np.abs(po.alg1_forward(Q, K, V, B, 4, idx, s) - Od).max() < 1e-12


# --- P3: convergence order pins the first-order term and its scale -------------------
def _errors_vs_delta(mode, k, s, deltas, L=128, B=16, d=6, seed=7):
    rng = np.random.default_rng(seed)
    N = L // B
    Q = rng.standard_normal((L, d))
    V = rng.standard_normal((L, d))
    cent = rng.standard_normal((N, d))
    xi = rng.standard_normal((L, d))
    idx = random_idx(N, k, rng)
    errs = []
    for dl in deltas:
        K = np.repeat(cent, B, axis=0) + dl * xi
        Od, _ = po.attention_head(Q, K, V, B, None, s, "dense")
        O, _ = po.attention_head(Q, K, V, B, idx, s, mode)
        errs.append(np.abs(O - Od).max())
    return np.array(errs)


@pytest.mark.parametrize("k", [0, 2])
@pytest.mark.parametrize("s", [0.35, 1.0])
def test_taylor_orders(k, s):
    """Keys c_j + delta*xi: dropping the first-order term leaves an O(delta) error in
    the numerator, keeping it leaves O(delta^2) (first-order Taylor expansion about
    the centroid; the denominator's first-order term vanishes).  A wrong sign,
    a transposed H_j or a missing / doubled scale turns slope 2 into slope 1."""
    deltas = 2.0 ** -np.arange(3, 9)
    e0 = _errors_vs_delta("pisa0", k, s, deltas)
    e1 = _errors_vs_delta("pisa1", k, s, deltas)
    slope0 = np.polyfit(np.log(deltas), np.log(e0), 1)[0]
    slope1 = np.polyfit(np.log(deltas), np.log(e1), 1)[0]
    assert abs(slope0 - 1.0) < 0.1, slope0
    assert abs(slope1 - 2.0) < 0.1, slope1
    assert np.all(e1 < e0)


# --- P4: equal H_j in every block => hybrid equals block-wise first order ------------
@pytest.mark.parametrize("k", [0, 3])
def test_hybrid_equals_blockwise_when_blocks_share_H(k):
    """Theorem 1 with M = 0: if all H_j coincide, replacing sum_U alpha_j H_j by
    (sum_U alpha_j) Hbar changes nothing.  Pins H_sum, the averaging over ALL N
    blocks and the tail weight."""
    L, B, d = 128, 16, 5
    N = L // B
    rng = np.random.default_rng(3)
    Q = rng.standard_normal((L, d))
    cent = rng.standard_normal((N, d))
    dev = 0.3 * rng.standard_normal((B, d))
    w = rng.standard_normal((B, d))
    K = np.repeat(cent, B, axis=0) + np.tile(dev, (N, 1))
    V = np.tile(w, (N, 1))
    idx = random_idx(N, k, rng)
    s = 0.5
    O1, _ = po.attention_head(Q, K, V, B, idx, s, "pisa1")
    for mode in ("hybrid", "hybrid_eq"):
        Oh, _ = po.attention_head(Q, K, V, B, idx, s, mode)
        assert np.abs(Oh - O1).max() < 1e-12
    # and the term is not vacuous here
    O0, _ = po.attention_head(Q, K, V, B, idx, s, "pisa0")
    assert np.abs(O0 - O1).max() > 1e-4


# --- P5: Theorem 1, first inequality ---------------------------------------------------
def test_theorem_bound_on_global_replacement():
    """|| o~_t - o_t ||_2 <= ||s q_t|| * max_U ||H_j - Hbar|| * sum_U alpha / D_t
    (Error Analysis, first inequality; Frobenius norm upper-bounds the spectral one)."""
    L, B, d = 192, 16, 6
    N = L // B
    rng = np.random.default_rng(5)
    Q, K, V = rand_qkv(L, d, rng, spread=0.7)
    s = 0.5
    idx = random_idx(N, 3, rng)
    st = po.block_stats(Q, K, V, B, per_block_H=True)
    Hbar = st["hsum"] / N
    for i in range(N):
        O1, lse = po.attention_rows(Q, K, V, B, i, idx[i], s, "pisa1", st)
        Oh, lse_h = po.attention_rows(Q, K, V, B, i, idx[i], s, "hybrid_eq", st)
        assert np.allclose(lse, lse_h)
        U = np.setdiff1d(np.arange(N), idx[i])
        M2 = max(np.linalg.norm(st["Hj"][j] - Hbar, 2) for j in U)
        Qi = s * Q[i * B:(i + 1) * B]
        a = Qi @ st["kbar"][U].T
        tail_over_D = np.exp(a - lse[:, None]).sum(axis=1)
        bound = np.linalg.norm(Qi, axis=1) * M2 * tail_over_D
        err = np.linalg.norm(Oh - O1, axis=1)
        assert np.all(err <= bound * (1 + 1e-9) + 1e-15)
        assert err.max() > 1e-6            # the bound is not vacuous


# --- P6: Jensen: the PISA denominator never exceeds the dense one ---------------------
@pytest.mark.parametrize("L,B", [(128, 16), (120, 16)])
def test_denominator_below_dense(L, B):
    """B_j exp(q kbar_j) <= sum_n exp(q k_{j,n}) block by block (Jensen step of the
    error analysis), so lse_PISA <= lse_dense for every row."""
    d = 8
    Q, K, V = rand_qkv(L, d)
    N = po.num_blocks(L, B)
    idx = random_idx(N, 2)
    s = 0.6
    _, lsed = po.attention_head(Q, K, V, B, None, s, "dense")
    _, lse = po.attention_head(Q, K, V, B, idx, s, "hybrid")
    assert np.all(lse <= lsed + 1e-12)
    assert np.any(lse < lsed - 1e-6)


# --- P7: constant values are reproduced exactly ---------------------------------------
@pytest.mark.parametrize("L,B,k", [(96, 16, 2), (90, 16, 0), (90, 16, 6)])
def test_constant_values_reproduced(L, B, k):
    """sum_n (k_{j,n} - kbar_j) = 0 (remark after the block-wise equations): with all
    value rows equal to c every H_j vanishes and N_t = c * D_t in every variant."""
    d = 7
    Q, K, _ = rand_qkv(L, d)
    c = RNG.standard_normal(d)
    V = np.tile(c, (L, 1))
    N = po.num_blocks(L, B)
    idx = random_idx(N, k) if k else np.zeros((N, 0), dtype=np.int32)
    modes = ("pisa0", "pisa1", "hybrid") + (("sparse",) if k else ())
    for mode in modes:
        O, _ = po.attention_head(Q, K, V, B, idx, 0.5, mode)
        assert np.abs(O - c).max() < 1e-11, mode
    assert np.abs(po.alg1_forward(Q, K, V, B, 4, idx, 0.5) - c).max() < 1e-11


# --- P8: order inside a key/value block does not matter -------------------------------
def test_permutation_within_kv_blocks():
    L, B, d = 96, 16, 6
    Q, K, V = rand_qkv(L, d)
    perm = np.concatenate([j * B + RNG.permutation(B) for j in range(L // B)])
    O, idx, lse = po.pisa_forward(Q, K, V, B, 0.67)
    O2, idx2, lse2 = po.pisa_forward(Q, K[perm], V[perm], B, 0.67)
    assert np.array_equal(idx, idx2)
    assert np.abs(O - O2).max() < 1e-12


# --- P9: selection against brute force; the sparsity -> k relation ---------------------
@pytest.mark.parametrize("N,k", [(5, 0), (7, 3), (16, 4), (32, 31), (32, 32)])
def test_select_against_full_sort(N, k):
    d = 6
    qbar = RNG.standard_normal((N, d))
    kbar = RNG.standard_normal((N, d))
    kbar[3] = kbar[1]                      # an exact tie: lower index must win
    idx, gap = po.select(qbar, kbar, 0.5, k)
    assert idx.shape == (N, k) and idx.dtype == np.int32
    for i in range(N):
        z = [0.5 * float(np.dot(qbar[i], kbar[j])) for j in range(N)]
        ranked = sorted(range(N), key=lambda j: (-z[j], j))
        assert list(idx[i]) == sorted(ranked[:k])
        if 0 < k < N:
            assert gap[i] == pytest.approx(z[ranked[k - 1]] - z[ranked[k]], abs=1e-12)
            assert gap[i] >= 0
        else:
            assert np.isinf(gap[i])


def test_tie_goes_to_lower_index():
    qbar = np.ones((1, 2))
    kbar = np.array([[1.0, 0.0], [0.5, 0.5], [0.0, 1.0], [2.0, 2.0]])   # logits 1,1,1,4
    idx, gap = po.select(qbar, kbar, 1.0, 2)
    assert list(idx[0]) == [0, 3] and gap[0] == 0.0


def test_sparsity_to_block_count_fixture():
    """The sparsity/density pairs the paper states (Kernel Efficiency Evaluation)."""
    with open(os.path.join(HERE, "golden", "sparsity_density.txt")) as f:
        rows = [l.split() for l in f if l.strip() and not l.startswith("#")]
    for n, r, k in rows:
        assert po.topk_count(int(n), float(r)) == int(k)
    # block counts at the benchmark shapes (block 64): tiny, FLUX, Wan, Hunyuan
    assert [po.topk_count(po.num_blocks(L, 64), r) for L, r in
            ((1024, .75), (4608, .85), (75600, .85), (119056, .90))] == [4, 11, 178, 187]
    assert po.topk_count(po.num_blocks(75600, 128), .85) == 89


# --- P10: the algorithm listing and the equations give one result ----------------------
@pytest.mark.parametrize("C", [1, 3, 8, 64])
def test_alg1_equals_equations_when_block_divides_length(C):
    """ln B on the centroid logits, block-mean values and l_tail/L * H_sum reproduce
    (sum_U alpha) q Hbar of the hybrid equations; the group size C is result-neutral."""
    L, B, d = 128, 16, 6
    Q, K, V = rand_qkv(L, d)
    N = L // B
    idx = random_idx(N, 3)
    s = 0.45
    Oeq, _ = po.attention_head(Q, K, V, B, idx, s, "hybrid_eq")
    Oh, _ = po.attention_head(Q, K, V, B, idx, s, "hybrid")
    Oa = po.alg1_forward(Q, K, V, B, C, idx, s)
    assert np.abs(Oa - Oeq).max() < 1e-12
    assert np.abs(Oh - Oeq).max() < 1e-12


@pytest.mark.parametrize("k", [0, 2, 8])
def test_alg1_equals_token_weighted_form_on_ragged_length(k):
    L, B, d = 120, 16, 6                  # last block has 8 rows
    Q, K, V = rand_qkv(L, d)
    N = po.num_blocks(L, B)
    idx = random_idx(N, k)
    Oh, _ = po.attention_head(Q, K, V, B, idx, 0.45, "hybrid")
    Oa = po.alg1_forward(Q, K, V, B, 5, idx, 0.45)
    assert Oh.shape == (L, d)
    assert np.abs(Oa - Oh).max() < 1e-12


# --- P11: a common shift of all keys changes nothing -----------------------------------
@pytest.mark.parametrize("mag", [1.0, 300.0])
def test_key_shift_invariance(mag):
    """q (k + c)^T = q k^T + const per row: the softmax, the pooled ranking and the
    centred H_j are unchanged, also where an unshifted exp would overflow."""
    L, B, d = 96, 16, 6
    Q, K, V = rand_qkv(L, d)
    c = mag * RNG.standard_normal(d)
    O, idx, _ = po.pisa_forward(Q, K, V, B, 0.67)
    O2, idx2, _ = po.pisa_forward(Q, K + c, V, B, 0.67)
    assert np.array_equal(idx, idx2)
    assert np.all(np.isfinite(O2))
    assert np.abs(O - O2).max() < 1e-9 * max(1.0, mag)


# --- P12 and closed forms for the statistics -------------------------------------------
@pytest.mark.parametrize("L,B", [(96, 16), (90, 16)])
def test_hsum_identity(L, B):
    """sum_j H_j = K^T V - Kbar^T Vhat (expanding the definition of H_j)."""
    d = 5
    Q, K, V = rand_qkv(L, d)
    st = po.block_stats(Q, K, V, B, per_block_H=True)
    sizes = po.block_sizes(L, B)
    assert np.abs(st["hsum"] - (K.T @ V - st["kbar"].T @ st["vsum"])).max() < 1e-11
    assert np.abs(st["Hj"].sum(axis=0) - st["hsum"]).max() < 1e-12
    assert st["qbar"].shape == (len(sizes), d)
    # ragged tail: mean over the valid rows only
    lo = (len(sizes) - 1) * B
    assert np.allclose(st["kbar"][-1], K[lo:].mean(axis=0))
    assert np.allclose(st["qbar"][-1], Q[lo:].mean(axis=0))
    assert np.allclose(st["vsum"][-1], V[lo:].sum(axis=0))


def test_stats_closed_form_ramp():
    """k_{j,n} = n e_a, v_{j,n} = n e_b (n = 0..B-1): kbar = (B-1)/2 e_a,
    vsum = B(B-1)/2 e_b and H_j = B(B^2-1)/12 e_a e_b^T -- orientation included."""
    B, N, d, a, b = 8, 3, 4, 1, 2
    n = np.tile(np.arange(B, dtype=float), N)
    K = np.zeros((B * N, d)); K[:, a] = n
    V = np.zeros((B * N, d)); V[:, b] = n
    st = po.block_stats(K, K, V, B, per_block_H=True)
    Hexp = np.zeros((d, d)); Hexp[a, b] = B * (B * B - 1) / 12
    assert np.allclose(st["kbar"][:, a], (B - 1) / 2)
    assert np.allclose(st["vsum"][:, b], B * (B - 1) / 2)
    for j in range(N):
        assert np.allclose(st["Hj"][j], Hexp)
    assert np.allclose(st["hsum"], N * Hexp)


# --- a literal loop over the equations on a tiny case ----------------------------------
def test_hybrid_against_scalar_loops():
    """Hybrid equations written out with scalar loops (exact term, B*alpha in D_t,
    alpha*Vhat_j, q Hbar sum_U alpha) on L=12, B=4."""
    L, B, d, s = 12, 4, 3, 0.7
    N = L // B
    rng = np.random.default_rng(11)
    Q, K, V = rand_qkv(L, d, rng)
    S = {0: [1], 1: [0], 2: [2]}
    idx = np.array([S[i] for i in range(N)], dtype=np.int32)
    kb = [[sum(K[j * B + n][c] for n in range(B)) / B for c in range(d)] for j in range(N)]
    H = [[[sum((K[j * B + n][a] - kb[j][a]) * V[j * B + n][b] for n in range(B))
           for b in range(d)] for a in range(d)] for j in range(N)]
    Hbar = [[sum(H[j][a][b] for j in range(N)) / N for b in range(d)] for a in range(d)]
    O = np.zeros((L, d))
    for t in range(L):
        i = t // B
        D = 0.0
        Nt = [0.0] * d
        tail = 0.0
        for j in range(N):
            if j in S[i]:
                for n in range(B):
                    e = math.exp(s * sum(Q[t][c] * K[j * B + n][c] for c in range(d)))
                    D += e
                    for c in range(d):
                        Nt[c] += e * V[j * B + n][c]
            else:
                al = math.exp(s * sum(Q[t][c] * kb[j][c] for c in range(d)))
                D += B * al
                tail += al
                for c in range(d):
                    Nt[c] += al * sum(V[j * B + n][c] for n in range(B))
        for c in range(d):
            Nt[c] += tail * sum(s * Q[t][a] * Hbar[a][c] for a in range(d))
        O[t] = [x / D for x in Nt]
    Oh, _ = po.attention_head(Q, K, V, B, idx, s, "hybrid")
    assert np.abs(Oh - O).max() < 1e-13


def test_error_shrinks_with_key_spread_and_beats_sparse():
    """The approximation error falls as the keys of a block tighten around their
    centroid, and covering U_i beats dropping it (the paper's central claim,
    Ablation Study: zeroth-order below sparse, hybrid below zeroth-order)."""
    L, B, d, s = 256, 16, 8, 0.35
    N = L // B
    rng = np.random.default_rng(2)
    Q = rng.standard_normal((L, d))
    V = rng.standard_normal((L, d))
    cent = rng.standard_normal((N, d))
    xi = rng.standard_normal((L, d))
    prev = None
    for spread in (0.4, 0.2, 0.1):
        K = np.repeat(cent, B, axis=0) + spread * xi
        st = po.block_stats(Q, K, V, B)
        idx, _ = po.select(st["qbar"], st["kbar"], s, 4)
        Od, _ = po.attention_head(Q, K, V, B, None, s, "dense")
        err = {m: np.abs(po.attention_head(Q, K, V, B, idx, s, m)[0] - Od).sum() / np.abs(Od).sum()
               for m in ("sparse", "pisa0", "pisa1")}
        assert err["pisa1"] < err["pisa0"] < err["sparse"]
        if prev is not None:
            assert err["pisa0"] < prev["pisa0"] and err["pisa1"] < prev["pisa1"]
        prev = err


# --- covariance-aware selection -----------------------------------------------------------
def test_covariance_aware_score_is_alpha_times_M():
    """Adding log(M_j + eps) to the pooled logit ranks blocks by exp(z_ij) (M_j + eps)
    (Covariance-Aware Block Selection and its appendix derivation: routing factor
    exp(q kbar_j) M_j / Mbar, the constant Mbar drops out of the softmax)."""
    L, B, d = 160, 16, 5
    N = L // B
    rng = np.random.default_rng(21)
    Q, K, V = rand_qkv(L, d, rng)
    st = po.block_stats(Q, K, V, B, per_block_H=True)
    eps = 1e-6
    for kind in ("spectral", "frobenius"):
        M = po.block_heterogeneity(st["Hj"], st["hsum"], kind)
        assert M.shape == (N,) and np.all(M > 0)
        idx, _ = po.select(st["qbar"], st["kbar"], 0.5, 3, col_bias=np.log(M + eps))
        z = po.pooled_logits(st["qbar"], st["kbar"], 0.5)
        for i in range(N):
            w = np.exp(z[i]) * (M + eps)
            assert sorted(np.argsort(-w, kind="stable")[:3].tolist()) == idx[i].tolist()
    # spectral <= Frobenius <= sqrt(rank) * spectral
    Ms = po.block_heterogeneity(st["Hj"], st["hsum"], "spectral")
    Mf = po.block_heterogeneity(st["Hj"], st["hsum"], "frobenius")
    assert np.all(Ms <= Mf * (1 + 1e-12)) and np.all(Mf <= math.sqrt(d) * Ms * (1 + 1e-12))


def test_covariance_bias_is_neutral_when_blocks_are_alike():
    """Equal M_j for all blocks shifts every logit alike, so the selection is unchanged;
    a block whose H_j stands out is pulled into S_i."""
    L, B, d = 256, 16, 4
    N = L // B
    rng = np.random.default_rng(22)
    Q = rng.standard_normal((L, d))
    cent = rng.standard_normal((N, d))
    dev = 0.3 * rng.standard_normal((B, d))
    w = rng.standard_normal((B, d))
    K = np.repeat(cent, B, axis=0) + np.tile(dev, (N, 1))
    V = np.tile(w, (N, 1))
    V[5 * B:6 * B] *= 30.0                      # block 5: a much larger H_5
    st = po.block_stats(Q, K, V, B, per_block_H=True)
    M = po.block_heterogeneity(st["Hj"], st["hsum"], "spectral")
    others = np.delete(M, 5)
    assert np.allclose(others, others[0], rtol=1e-9) and M[5] > 5 * others[0]
    plain, _ = po.select(st["qbar"], st["kbar"], 0.5, 2)
    biased, _ = po.select(st["qbar"], st["kbar"], 0.5, 2, col_bias=np.log(M + 1e-6))
    assert np.all((biased == 5).any(axis=1))     # every query block now keeps block 5 exact
    flat, _ = po.select(st["qbar"], st["kbar"], 0.5, 2, col_bias=np.full(N, math.log(others[0])))
    assert np.array_equal(flat, plain)


# --- keep-or-drop at k < N is the masked softmax of the Preliminaries ----------------
@pytest.mark.parametrize("L,B,k", [(96, 16, 2), (90, 16, 3), (90, 16, 1)])
def test_sparse_mode_is_block_masked_library_attention(L, B, k):
    """Preliminaries, second equation: keep-or-drop attention is dense attention with a
    mask of 0 on the selected blocks' tokens and -inf elsewhere.  Checked against torch's
    fp64 CPU attention routine fed that additive mask (ragged last block included)."""
    d = 8
    Q, K, V = rand_qkv(L, d)
    s = 1 / math.sqrt(d)
    N = po.num_blocks(L, B)
    idx = random_idx(N, k)
    blk_q = np.arange(L) // B
    blk_k = np.arange(L) // B
    keep = np.zeros((L, L), dtype=bool)
    for i in range(N):
        keep[np.ix_(blk_q == i, np.isin(blk_k, idx[i]))] = True
    mask = np.where(keep, 0.0, -np.inf)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None], torch.from_numpy(K)[None], torch.from_numpy(V)[None],
        attn_mask=torch.from_numpy(mask)[None], scale=s)[0].numpy()
    O, lse = po.attention_head(Q, K, V, B, idx, s, "sparse")
    assert np.abs(O - ref).max() < 1e-12
    ref_lse = torch.logsumexp(torch.from_numpy(s * (Q @ K.T) + mask), dim=1).numpy()
    assert np.abs(lse - ref_lse).max() < 1e-12
    # and it is NOT the dense result (the mask matters at k < N)
    Od, _ = po.attention_head(Q, K, V, B, None, s, "dense")
    assert np.abs(O - Od).max() > 1e-3


# --- rank-one blocks give the heterogeneity in closed form ----------------------------
@pytest.mark.parametrize("L,B", [(96, 16), (90, 16)])
def test_heterogeneity_closed_form_rank_one(L, B):
    """Covariance-Aware Block Selection: M_j = ||H_j - Hbar||.  Keys k_{j,n} = c_j + u_n a and
    values v_{j,n} = g_j u_n b / sum_n u_n^2 + w (sum_n u_n = 0 inside every block) give
    H_j = g_j a^T b exactly, so Hbar = mean(g) a^T b and
    M_j = |g_j - mean(g)| ||a|| ||b|| in the spectral and in the Frobenius norm alike."""
    d = 5
    rng = np.random.default_rng(31)
    N = po.num_blocks(L, B)
    sizes = po.block_sizes(L, B)
    a, b, w = rng.standard_normal(d), rng.standard_normal(d), rng.standard_normal(d)
    g = rng.standard_normal(N) * 3.0
    cent = rng.standard_normal((N, d))
    K = np.empty((L, d))
    V = np.empty((L, d))
    for j in range(N):
        u = rng.standard_normal(sizes[j])
        u -= u.mean()
        lo = j * B
        K[lo:lo + sizes[j]] = cent[j] + np.outer(u, a)
        V[lo:lo + sizes[j]] = g[j] * np.outer(u, b) / (u @ u) + w
    Q = rng.standard_normal((L, d))
    st = po.block_stats(Q, K, V, B, per_block_H=True)
    for j in range(N):
        assert np.abs(st["Hj"][j] - g[j] * np.outer(a, b)).max() < 1e-12
    want = np.abs(g - g.mean()) * np.linalg.norm(a) * np.linalg.norm(b)
    for kind in ("spectral", "frobenius"):
        M = po.block_heterogeneity(st["Hj"], st["hsum"], kind)
        assert np.abs(M - want).max() < 1e-11 * max(1.0, want.max())
