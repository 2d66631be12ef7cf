"""Pins for the CPU oracle (no GPU needed).

Each test fixes the oracle to something other than itself: a hand-evaluated
example, a closed form, a brute-force evaluation of the unrolled sum, or an
identity that the paper's operators imply.  Citations name the passage of the
DiG paper that fixes the expected value.
"""
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
ROW_FWD, ROW_REV, COL_FWD, COL_REV = 0, 1, 2, 3


def _rand(rng, *shape):
    return rng.standard_normal(shape)


def _gates(rng, *shape, scale=0.3):
    # log alpha <= 0
    return -np.abs(rng.standard_normal(shape)) * scale


@pytest.fixture(params=["c", "numpy"])
def fwd(request, oracle):
    return oracle.gla_fwd if request.param == "c" else oracle.gla_fwd_numpy


# --------------------------------------------------------------------------
# hand-evaluated and closed-form values
# --------------------------------------------------------------------------
def test_two_token_hand_example(fwd):
    """Sec. 3.1, Eq. (attn_gla) rows 1-3 evaluated by hand (tests/golden/two_token_example.txt)."""
    vals = {}
    with open(os.path.join(GOLDEN, "two_token_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, *nums = line.split()
            vals[name] = np.array([float(x) for x in nums])
    q = np.array([[1.0, 2.0], [-1.0, 4.0]]).reshape(1, 1, 2, 2)
    k = np.array([[3.0, -1.0], [2.0, 5.0]]).reshape(1, 1, 2, 2)
    v = np.array([[1.0, 0.0, 2.0], [0.0, 1.0, -1.0]]).reshape(1, 1, 2, 3)
    la = np.log(np.array([[0.5, 0.25], [0.5, 0.25]])).reshape(1, 1, 2, 2)
    out, S = fwd(q, k, v, la, 1, 2, ROW_FWD)
    np.testing.assert_allclose(out[0, 0, 0], vals["o1"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(out[0, 0, 1], vals["o2"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(S[0, 0, 0], vals["S2_row0"], rtol=0, atol=1e-13)
    np.testing.assert_allclose(S[0, 0, 1], vals["S2_row1"], rtol=0, atol=1e-13)


def test_scalar_half_gate_closed_form(fwd):
    """dk=dv=1, q=k=v=1, alpha=1/2: o_t = 2 - 2^(1-t) (tests/golden/scalar_half_gate.txt)."""
    tab = np.loadtxt(os.path.join(GOLDEN, "scalar_half_gate.txt"))
    T = tab.shape[0]
    one = np.ones((1, 1, T, 1))
    la = np.full((1, 1, T, 1), np.log(0.5))
    out, S = fwd(one, one, one, la, 1, T, ROW_FWD)
    np.testing.assert_allclose(out[0, 0, :, 0], tab[:, 1], rtol=0, atol=1e-14)
    assert abs(S[0, 0, 0, 0] - tab[-1, 1]) < 1e-14


def test_single_token(fwd):
    """T = 1: o = (q.k) v and S_1 = k^T v (Eq. (attn_gla) rows 2-3 with S_0 = 0)."""
    rng = np.random.default_rng(1)
    q, k, v = _rand(rng, 2, 3, 1, 5), _rand(rng, 2, 3, 1, 5), _rand(rng, 2, 3, 1, 7)
    la = _gates(rng, 2, 3, 1, 5)
    out, S = fwd(q, k, v, la, 1, 1, ROW_FWD)
    qk = np.sum(q * k, axis=-1, keepdims=True)
    np.testing.assert_allclose(out, qk * v, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(S, k[:, :, 0, :, None] * v[:, :, 0, None, :], rtol=1e-13, atol=1e-13)


def test_no_decay_is_causal_linear_attention(fwd):
    """alpha = 1 reduces the recurrence to Eq. (attn_simple): o_t = sum_{i<=t} (q_t.k_i) v_i."""
    rng = np.random.default_rng(2)
    B, H, T, dk, dv = 2, 2, 12, 4, 6
    q, k, v = _rand(rng, B, H, T, dk), _rand(rng, B, H, T, dk), _rand(rng, B, H, T, dv)
    la = np.zeros((B, H, T, dk))
    out, S = fwd(q, k, v, la, 3, 4, ROW_FWD)
    ref = np.zeros_like(out)
    for b in range(B):
        for h in range(H):
            for t in range(T):
                for i in range(t + 1):
                    ref[b, h, t] += np.dot(q[b, h, t], k[b, h, i]) * v[b, h, i]
    np.testing.assert_allclose(out, ref, rtol=1e-12, atol=1e-12)
    Sref = np.einsum("bhtc,bhtj->bhcj", k, v)
    np.testing.assert_allclose(S, Sref, rtol=1e-12, atol=1e-12)


def test_unrolled_sum_brute_force(fwd):
    """Unrolling Eq. (attn_gla): o_t = sum_{i<=t} sum_c q_tc k_ic prod_{m=i+1..t} alpha_mc v_i.

    Pins the gate's index (alpha_t decays what came before token t, not token t
    itself), its axis (key channel) and the read-after-update order.
    """
    rng = np.random.default_rng(3)
    T, dk, dv = 7, 3, 2
    q, k, v = _rand(rng, 1, 1, T, dk), _rand(rng, 1, 1, T, dk), _rand(rng, 1, 1, T, dv)
    alpha = rng.uniform(0.2, 0.95, size=(1, 1, T, dk))
    out, S = fwd(q, k, v, np.log(alpha), 1, T, ROW_FWD)
    ref = np.zeros((T, dv))
    for t in range(T):
        for i in range(t + 1):
            for c in range(dk):
                w = 1.0
                for m in range(i + 1, t + 1):
                    w *= alpha[0, 0, m, c]
                ref[t] += q[0, 0, t, c] * k[0, 0, i, c] * w * v[0, 0, i]
    np.testing.assert_allclose(out[0, 0], ref, rtol=1e-12, atol=1e-12)
    Sref = np.zeros((dk, dv))
    for i in range(T):
        for c in range(dk):
            w = np.prod(alpha[0, 0, i + 1:, c])
            Sref[c] += k[0, 0, i, c] * w * v[0, 0, i]
    np.testing.assert_allclose(S[0, 0], Sref, rtol=1e-12, atol=1e-12)


def test_closed_gate_forgets_everything(fwd):
    """alpha -> 0: the state is wiped before each token, so o_t = (q_t.k_t) v_t."""
    rng = np.random.default_rng(4)
    T, dk, dv = 9, 4, 3
    q, k, v = _rand(rng, 1, 2, T, dk), _rand(rng, 1, 2, T, dk), _rand(rng, 1, 2, T, dv)
    la = np.full((1, 2, T, dk), -800.0)
    out, _ = fwd(q, k, v, la, 3, 3, ROW_FWD)
    np.testing.assert_allclose(out, np.sum(q * k, -1, keepdims=True) * v, rtol=1e-13, atol=1e-13)


def test_first_gate_is_irrelevant(fwd):
    """alpha at the first scan step multiplies S_0 = 0."""
    rng = np.random.default_rng(5)
    T, dk, dv = 6, 3, 4
    q, k, v = _rand(rng, 1, 1, T, dk), _rand(rng, 1, 1, T, dk), _rand(rng, 1, 1, T, dv)
    la = _gates(rng, 1, 1, T, dk)
    la2 = la.copy()
    la2[0, 0, 0] = -5.0
    a, _ = fwd(q, k, v, la, 2, 3, ROW_FWD)
    b, _ = fwd(q, k, v, la2, 2, 3, ROW_FWD)
    np.testing.assert_array_equal(a, b)


# --------------------------------------------------------------------------
# scan orders (Sec. 3.3 / Algorithm 1; flip, transpose, flatten of Algorithms 2-4)
# --------------------------------------------------------------------------
def test_scan_index_matches_reshape_definition(oracle):
    for gh, gw in [(1, 1), (1, 5), (5, 1), (3, 4), (4, 3), (4, 4)]:
        for d in range(4):
            pi = oracle.scan_order(d, gh, gw)
            got = [oracle.scan_index(d, s, gh, gw) for s in range(gh * gw)]
            assert got == list(pi)
            assert sorted(got) == list(range(gh * gw))


def test_scan_order_small_grid_by_hand(oracle):
    # 2 x 3 grid, tokens numbered row-major:  0 1 2 / 3 4 5
    assert list(oracle.scan_order(ROW_FWD, 2, 3)) == [0, 1, 2, 3, 4, 5]
    assert list(oracle.scan_order(ROW_REV, 2, 3)) == [5, 4, 3, 2, 1, 0]
    assert list(oracle.scan_order(COL_FWD, 2, 3)) == [0, 3, 1, 4, 2, 5]
    assert list(oracle.scan_order(COL_REV, 2, 3)) == [5, 2, 4, 1, 3, 0]


def test_reversed_scan_is_forward_on_flipped_tokens(fwd):
    """Algorithm 2 (flip -> GLA -> flip)."""
    rng = np.random.default_rng(6)
    gh, gw, dk, dv = 3, 5, 3, 4
    T = gh * gw
    q, k, v = _rand(rng, 2, 1, T, dk), _rand(rng, 2, 1, T, dk), _rand(rng, 2, 1, T, dv)
    la = _gates(rng, 2, 1, T, dk)
    out, S = fwd(q, k, v, la, gh, gw, ROW_REV)
    f = lambda x: x[:, :, ::-1]
    o2, S2 = fwd(f(q), f(k), f(v), f(la), gh, gw, ROW_FWD)
    np.testing.assert_allclose(out, f(o2), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(S, S2, rtol=1e-13, atol=1e-13)


def _transpose_tokens(x, gh, gw):
    B, H, T, d = x.shape
    return x.reshape(B, H, gh, gw, d).transpose(0, 1, 3, 2, 4).reshape(B, H, T, d)


def test_column_scan_is_row_scan_of_transposed_grid(fwd):
    """Algorithm 3: flatten(transpose(reshape2d(z))) -> GLA -> transpose back."""
    rng = np.random.default_rng(7)
    gh, gw, dk, dv = 4, 3, 2, 3
    T = gh * gw
    q, k, v = _rand(rng, 1, 2, T, dk), _rand(rng, 1, 2, T, dk), _rand(rng, 1, 2, T, dv)
    la = _gates(rng, 1, 2, T, dk)
    tr = lambda x: _transpose_tokens(x, gh, gw)
    for d_col, d_row in ((COL_FWD, ROW_FWD), (COL_REV, ROW_REV)):
        out, S = fwd(q, k, v, la, gh, gw, d_col)
        o2, S2 = fwd(tr(q), tr(k), tr(v), tr(la), gw, gh, d_row)
        np.testing.assert_allclose(out, _transpose_tokens(o2, gw, gh), rtol=1e-13, atol=1e-13)
        np.testing.assert_allclose(S, S2, rtol=1e-13, atol=1e-13)


def test_degenerate_grids(fwd):
    """A 1 x T or T x 1 grid has a single line of tokens: column order = row order."""
    rng = np.random.default_rng(8)
    T, dk, dv = 6, 2, 2
    q, k, v = _rand(rng, 1, 1, T, dk), _rand(rng, 1, 1, T, dk), _rand(rng, 1, 1, T, dv)
    la = _gates(rng, 1, 1, T, dk)
    for gh, gw in ((1, T), (T, 1)):
        a, _ = fwd(q, k, v, la, gh, gw, ROW_FWD)
        b, _ = fwd(q, k, v, la, gh, gw, COL_FWD)
        np.testing.assert_array_equal(a, b)
        a, _ = fwd(q, k, v, la, gh, gw, ROW_REV)
        b, _ = fwd(q, k, v, la, gh, gw, COL_REV)
        np.testing.assert_array_equal(a, b)


def test_block_by_block_reorientation_cycles_four_orders(oracle):
    """Algorithm 1: alternating transpose / flip of the residual stream walks the scan
    through exactly the four orders with period four, for either parity convention."""
    N = 4
    T = N * N
    orders = {d: tuple(oracle.scan_order(d, N, N)) for d in range(4)}
    for first_is_transpose in (True, False):
        seq = np.arange(T)
        seen = []
        for l in range(8):
            seen.append(tuple(seq))
            transpose = (l % 2 == 0) == first_is_transpose
            if transpose:
                seq = seq.reshape(N, N).T.reshape(-1)
            else:
                seq = seq[::-1]
        assert set(seen[:4]) == set(orders.values())
        assert seen[4:] == seen[:4]
        assert seen[0] == orders[ROW_FWD]


def test_block_schedule_names_the_order_each_block_sees(oracle):
    """Algorithm 1 (flip after odd blocks, transpose after even ones) and Algorithm 4 (parities swapped), worked out
    by hand on a 2 x 2 grid with tokens 0 1 / 2 3: block 1 sees 0 1 2 3; Algorithm 1 then flips (3 2 1 0 = row
    reversed), transposes (3 1 2 0 = column reversed), flips (0 2 1 3 = column forward), transposes (0 1 2 3)."""
    assert [oracle.block_scan_dir(l, oracle.SCHEDULE_BLOCK_PROCESS) for l in range(1, 10)] == \
        [ROW_FWD, ROW_REV, COL_REV, COL_FWD, ROW_FWD, ROW_REV, COL_REV, COL_FWD, ROW_FWD]
    # Algorithm 4: transposes first (0 2 1 3 = column forward), flips (3 1 2 0), transposes (3 2 1 0), flips
    assert [oracle.block_scan_dir(l, oracle.SCHEDULE_BLOCK_SCAN) for l in range(1, 10)] == \
        [ROW_FWD, COL_FWD, COL_REV, ROW_REV, ROW_FWD, COL_FWD, COL_REV, ROW_REV, ROW_FWD]
    # the hand-worked sequences themselves
    assert list(oracle.scan_order(ROW_REV, 2, 2)) == [3, 2, 1, 0]
    assert list(oracle.scan_order(COL_REV, 2, 2)) == [3, 1, 2, 0]
    assert list(oracle.scan_order(COL_FWD, 2, 2)) == [0, 2, 1, 3]
    # independent of the grid the index array is drawn on
    for grid in (2, 3, 5):
        for sched in (oracle.SCHEDULE_BLOCK_PROCESS, oracle.SCHEDULE_BLOCK_SCAN):
            assert [oracle.block_scan_dir(l, sched, grid) for l in range(1, 6)] == \
                [oracle.block_scan_dir(l, sched) for l in range(1, 6)]
    with pytest.raises(ValueError):
        oracle.block_scan_dir(0)


# --------------------------------------------------------------------------
# structure: chunked evaluation, carried state, linearity
# --------------------------------------------------------------------------
def _chunked(q, k, v, la, C):
    """Chunk-parallel form (Sec. 3.5): per chunk, decay-weighted causal scores inside the
    chunk plus the carried state; written independently of the oracle, in numpy fp64."""
    T, dk = q.shape
    dv = v.shape[1]
    S = np.zeros((dk, dv))
    out = np.zeros((T, dv))
    for s0 in range(0, T, C):
        sl = slice(s0, min(T, s0 + C))
        b = np.cumsum(la[sl], axis=0)                     # inclusive log-decay inside the chunk
        qt = q[sl] * np.exp(b)
        kt = k[sl] * np.exp(-b)
        A = np.tril(qt @ kt.T)
        out[sl] = A @ v[sl] + qt @ S
        khat = k[sl] * np.exp(b[-1] - b)
        S = np.exp(b[-1])[:, None] * S + khat.T @ v[sl]
    return out, S


@pytest.mark.parametrize("C", [1, 3, 16, 64, 50])
def test_chunked_evaluation_matches_recurrence(oracle, C):
    rng = np.random.default_rng(9)
    T, dk, dv = 50, 5, 7
    q, k, v = _rand(rng, T, dk), _rand(rng, T, dk), _rand(rng, T, dv)
    la = _gates(rng, T, dk, scale=0.1)
    out, S = oracle.gla_fwd(q[None, None], k[None, None], v[None, None], la[None, None], 5, 10, ROW_FWD)
    o2, S2 = _chunked(q, k, v, la, C)
    np.testing.assert_allclose(out[0, 0], o2, rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(S[0, 0], S2, rtol=1e-10, atol=1e-10)


def test_state_carry_over(fwd):
    """Running two halves back to back with the carried state equals one run."""
    rng = np.random.default_rng(10)
    T, dk, dv = 10, 3, 4
    q, k, v = _rand(rng, 1, 2, T, dk), _rand(rng, 1, 2, T, dk), _rand(rng, 1, 2, T, dv)
    la = _gates(rng, 1, 2, T, dk)
    out, S = fwd(q, k, v, la, 1, T, ROW_FWD)
    h = 4
    o1, S1 = fwd(q[:, :, :h], k[:, :, :h], v[:, :, :h], la[:, :, :h], 1, h, ROW_FWD)
    o2, S2 = fwd(q[:, :, h:], k[:, :, h:], v[:, :, h:], la[:, :, h:], 1, T - h, ROW_FWD, initial_state=S1)
    np.testing.assert_allclose(np.concatenate([o1, o2], 2), out, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(S2, S, rtol=1e-13, atol=1e-13)


def test_linearity_and_column_independence(fwd):
    rng = np.random.default_rng(11)
    T, dk, dv = 8, 3, 5
    q, k, v = _rand(rng, 1, 1, T, dk), _rand(rng, 1, 1, T, dk), _rand(rng, 1, 1, T, dv)
    q2, v2 = _rand(rng, 1, 1, T, dk), _rand(rng, 1, 1, T, dv)
    la = _gates(rng, 1, 1, T, dk)
    f = lambda q_, v_: fwd(q_, k, v_, la, 2, 4, COL_FWD)[0]
    np.testing.assert_allclose(f(2 * q + q2, v), 2 * f(q, v) + f(q2, v), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(f(q, v - 3 * v2), f(q, v) - 3 * f(q, v2), rtol=1e-12, atol=1e-12)
    # column j of the output depends on column j of v only
    v3 = v.copy()
    v3[..., 1:] = v2[..., 1:]
    np.testing.assert_array_equal(f(q, v)[..., 0], f(q, v3)[..., 0])


def test_c_and_numpy_renderings_agree(oracle):
    rng = np.random.default_rng(12)
    B, H, gh, gw, dk, dv = 2, 3, 5, 6, 4, 6
    T = gh * gw
    q, k, v = _rand(rng, B, H, T, dk), _rand(rng, B, H, T, dk), _rand(rng, B, H, T, dv)
    la = _gates(rng, B, H, T, dk)
    for d in range(4):
        a, Sa = oracle.gla_fwd(q, k, v, la, gh, gw, d)
        b, Sb = oracle.gla_fwd_numpy(q, k, v, la, gh, gw, d)
        np.testing.assert_allclose(a, b, rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(Sa, Sb, rtol=1e-12, atol=1e-12)


def test_oracle_rejects_bad_grid(oracle):
    x = np.zeros((1, 1, 6, 2))
    with pytest.raises(ValueError):
        oracle.gla_fwd(x, x, x, x, 2, 2, ROW_FWD)


# ---------------------------------------------------------------------------
# multi-directional scanning (supplement, Algorithms 2 and 3) written out with the matrix operators the
# paper names (flip, reshape2d, transpose, flatten, +) around the row-forward scan only
# ---------------------------------------------------------------------------
def _flip(x):
    return x[:, :, ::-1]


def _transpose_tokens(x, gh, gw):
    """flatten(transpose(reshape2d(x))) for a token axis that is row-major over a gh x gw grid."""
    B, H, T, D = x.shape
    return x.reshape(B, H, gh, gw, D).transpose(0, 1, 3, 2, 4).reshape(B, H, T, D)


def test_bidirectional_and_four_directional_scanning_written_out(oracle):
    rng = np.random.default_rng(77)
    B, H, gh, gw, dk, dv = 2, 2, 3, 5, 4, 6
    T = gh * gw
    q, k, g = _rand(rng, B, H, T, dk), _rand(rng, B, H, T, dk), _gates(rng, B, H, T, dk)
    v = _rand(rng, B, H, T, dv)
    row = lambda a, b, c, d, h, w: oracle.gla_fwd(a, b, c, d, h, w, ROW_FWD)[0]
    # Algorithm 2: GLA(z) + flip(GLA(flip(z)))
    out1 = row(q, k, v, g, gh, gw)
    out2 = _flip(row(_flip(q), _flip(k), _flip(v), _flip(g), gh, gw))
    np.testing.assert_allclose(oracle.gla_fwd_multi(q, k, v, g, gh, gw, (ROW_FWD, ROW_REV)), out1 + out2,
                               rtol=1e-12, atol=1e-12)
    # Algorithm 3: the third input is the transposed grid flattened, the fourth its flip; each output is
    # brought back by the inverse operators (the transpose of a gw x gh grid, after un-flipping)
    tq, tk, tv, tg = (_transpose_tokens(a, gh, gw) for a in (q, k, v, g))
    o3 = row(tq, tk, tv, tg, gw, gh)
    out3 = _transpose_tokens(o3, gw, gh)
    o4 = row(_flip(tq), _flip(tk), _flip(tv), _flip(tg), gw, gh)
    out4 = _transpose_tokens(_flip(o4), gw, gh)
    np.testing.assert_allclose(oracle.gla_fwd_multi(q, k, v, g, gh, gw, (0, 1, 2, 3)), out1 + out2 + out3 + out4,
                               rtol=1e-12, atol=1e-12)
    # each direction contributes: dropping one changes the sum
    assert np.abs(oracle.gla_fwd_multi(q, k, v, g, gh, gw, (0, 1, 2)) - (out1 + out2 + out3 + out4)).max() > 1e-3
    with pytest.raises(ValueError):
        oracle.gla_fwd_multi(q, k, v, g, gh, gw, ())


def test_bidirectional_without_decay_is_full_attention_plus_diagonal(oracle):
    # with all gates open the forward scan sums over i <= t and the reversed one over i >= t: together every
    # pair once and the diagonal twice
    rng = np.random.default_rng(78)
    B, H, T, dk, dv = 1, 2, 9, 3, 4
    q, k, v = _rand(rng, B, H, T, dk), _rand(rng, B, H, T, dk), _rand(rng, B, H, T, dv)
    g = np.zeros((B, H, T, dk))
    a = np.einsum("bhic,bhjc->bhij", q, k)
    full = np.einsum("bhij,bhjn->bhin", a, v) + np.einsum("bhii,bhin->bhin", a, v)
    np.testing.assert_allclose(oracle.gla_fwd_multi(q, k, v, g, 3, 3, (ROW_FWD, ROW_REV)), full, rtol=1e-12, atol=1e-12)
