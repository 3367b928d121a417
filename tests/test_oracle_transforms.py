"""Pins for the offline FP64 transforms: the identities the paper states must hold (and the one
it says must fail).  Toy sizes, random weights, tolerances ~1e-10."""
import numpy as np
import pytest

from oracle import transforms as T

H, M_REP, D_HEAD, D_MODEL, L = 2, 2, 16, 64, 8


def toy_weights(seed=0):
    rng = np.random.default_rng(seed)
    Wq = rng.standard_normal((D_MODEL, M_REP * H * D_HEAD)) / 8
    Wk = rng.standard_normal((D_MODEL, H * D_HEAD)) / 8
    Wv = rng.standard_normal((D_MODEL, H * D_HEAD)) / 8
    Wo = rng.standard_normal((M_REP * H * D_HEAD, D_MODEL)) / 8
    X = rng.standard_normal((L, D_MODEL))
    return rng, X, Wq, Wk, Wv, Wo


def random_tk(rng, sigma=1.0, pairs=None, reflect=None):
    scales = np.exp(0.5 * sigma * rng.standard_normal((H, D_HEAD // 2))) * rng.choice([-1.0, 1.0], (H, D_HEAD // 2))
    angles = sigma * rng.uniform(-np.pi, np.pi, (H, D_HEAD // 2))
    return T.prerope_transform(scales, angles, M_REP, pairs, reflect)


def random_tv(rng, sigma=1.0):
    heads = [np.eye(D_HEAD) + sigma * 0.3 * rng.standard_normal((D_HEAD, D_HEAD)) for _ in range(H)]
    return T.value_transform(heads, M_REP)


def rel(a, b):
    return np.abs(a - b).max() / max(np.abs(b).max(), 1e-300)


@pytest.mark.parametrize("pairing", ["adjacent", "half_split"])
def test_theorem1_logits_unchanged(pairing):
    """<f(x_i W~_q, i), f(x_j W~_k, j)> = <f(x_i W_q, i), f(x_j W_k, j)> for every head and position pair."""
    rng, X, Wq, Wk, _, _ = toy_weights(1)
    pairs = T.adjacent_pairs(D_HEAD) if pairing == "adjacent" else T.half_split_pairs(D_HEAD)
    Tk, Tk_bar = random_tk(rng, pairs=pairs)
    Wq2, Wk2 = Wq @ Tk_bar, Wk @ Tk
    thetas = T.default_thetas(D_HEAD)
    for hq in range(M_REP * H):
        hk = hq // M_REP
        sq = slice(hq * D_HEAD, (hq + 1) * D_HEAD)
        sk = slice(hk * D_HEAD, (hk + 1) * D_HEAD)
        for i, j in [(0, 0), (3, 1), (7, 7), (2, 6), (1000, 3)]:
            xi, xj = X[i % L], X[j % L]
            a = T.qk_logit(xi, xj, Wq2[:, sq], Wk2[:, sk], i, j, thetas, pairs)
            b = T.qk_logit(xi, xj, Wq[:, sq], Wk[:, sk], i, j, thetas, pairs)
            assert abs(a - b) <= 1e-10 * max(1.0, abs(b))
    assert rel(Wk2, Wk) > 0.1          # the transform is not the identity


def test_tk_commutes_with_rope_and_bar_is_inverse_transpose():
    rng = np.random.default_rng(2)
    scales = np.exp(rng.standard_normal(D_HEAD // 2))
    angles = rng.uniform(-np.pi, np.pi, D_HEAD // 2)
    pairs = T.adjacent_pairs(D_HEAD)
    Tk, Tb = T.prerope_head_transform(scales, angles, pairs, D_HEAD)
    thetas = T.default_thetas(D_HEAD)
    for pos in (0, 1, 17, 4095):
        R = T.rope_matrix(D_HEAD, pos, thetas, pairs)
        assert rel(Tk @ R, R @ Tk) < 1e-12
    assert rel(Tb @ Tk.T, np.eye(D_HEAD)) < 1e-12
    # RoPE itself: relative-position property <f(q,i), f(k,j)> = q R_{i-j} k^T
    q, k = rng.standard_normal(D_HEAD), rng.standard_normal(D_HEAD)
    lhs = (q @ T.rope_matrix(D_HEAD, 9, thetas)) @ (k @ T.rope_matrix(D_HEAD, 4, thetas))
    rhs = q @ T.rope_matrix(D_HEAD, 5, thetas) @ k
    assert abs(lhs - rhs) < 1e-12


def test_reflection_breaks_the_identity():
    """Remark after the proof: an orthogonal block with a reflection does not commute with RoPE."""
    rng, X, Wq, Wk, _, _ = toy_weights(3)
    reflect = np.zeros((H, D_HEAD // 2), bool)
    reflect[0, 2] = True
    Tk, Tk_bar = random_tk(rng, reflect=reflect)
    thetas = T.default_thetas(D_HEAD)
    sq, sk = slice(0, D_HEAD), slice(0, D_HEAD)
    a = T.qk_logit(X[1], X[4], (Wq @ Tk_bar)[:, sq], (Wk @ Tk)[:, sk], 5, 2, thetas)
    b = T.qk_logit(X[1], X[4], Wq[:, sq], Wk[:, sk], 5, 2, thetas)
    assert abs(a - b) > 1e-4
    # ... and a scale that differs inside a pair breaks it too (one scalar per pair is required)
    Tbad = np.diag(np.r_[2.0, 3.0, np.ones(D_HEAD - 2)])
    R = T.rope_matrix(D_HEAD, 3, thetas)
    assert rel(Tbad @ R, R @ Tbad) > 1e-3


def test_value_transform_identity():
    """(A (X W_v T_v)) (T_v-bar W_o) = (A (X W_v)) W_o with the inverses repeated over the m query heads."""
    rng, X, Wq, Wk, Wv, Wo = toy_weights(4)
    Tv, Tv_bar = random_tv(rng)
    base = T.attention(X, Wq, Wk, Wv, Wo, H, M_REP, D_HEAD)
    new = T.attention(X, Wq, Wk, Wv @ Tv, Tv_bar @ Wo, H, M_REP, D_HEAD)
    assert rel(new, base) < 1e-10
    # wrong bookkeeping (inverse not repeated, heads shifted) must fail
    wrong = T.block_diag([np.linalg.inv(Tv[h * D_HEAD:(h + 1) * D_HEAD, h * D_HEAD:(h + 1) * D_HEAD])
                          for h in (0, 1, 0, 1)])
    bad = T.attention(X, Wq, Wk, Wv @ Tv, wrong @ Wo, H, M_REP, D_HEAD)
    assert rel(bad, base) > 1e-3


@pytest.mark.parametrize("sigma", [0.0, 0.1, 0.3, 1.0, 3.0])
def test_merged_attention_is_function_preserving_under_parameter_noise(sigma):
    """All merges at once; the output does not move however far the transform parameters are
    pushed (noise levels of the sensitivity study, App. L)."""
    rng, X, Wq, Wk, Wv, Wo = toy_weights(5)
    gain = np.exp(0.2 * rng.standard_normal(D_MODEL))
    Xn = X / T.rms(X) * gain
    base = T.attention(Xn, Wq, Wk, Wv, Wo, H, M_REP, D_HEAD)
    Tk, Tk_bar = random_tk(rng, sigma)
    heads = [np.eye(D_HEAD) + sigma * 0.1 * rng.standard_normal((D_HEAD, D_HEAD)) for _ in range(H)]
    Tv, Tv_bar = T.value_transform(heads, M_REP)
    Wq2, Wk2, Wv2, Wo2 = T.merge_attention(Wq, Wk, Wv, Wo, Tk, Tk_bar, Tv, Tv_bar)
    Wq2, Wk2, Wv2 = (T.fold_norm_gain(W, gain) for W in (Wq2, Wk2, Wv2))
    new = T.attention(X / T.rms(X), Wq2, Wk2, Wv2, Wo2, H, M_REP, D_HEAD)
    assert rel(new, base) < 1e-9


def test_per_token_scale_commutes_with_bias_free_linear_and_bmm():
    rng = np.random.default_rng(6)
    X = rng.standard_normal((L, D_MODEL))
    W = rng.standard_normal((D_MODEL, 24))
    S = np.exp(rng.standard_normal((L, 1)))
    assert rel((S * X) @ W, S * (X @ W)) < 1e-12
    A = rng.random((L, L))
    V = rng.standard_normal((L, 5))
    # scaling applied to the rows of the probabilities commutes with the PV product
    assert rel((S * A) @ V, S * (A @ V)) < 1e-12


def test_scale_recursion_equals_definition():
    """S_n from the recursion equals 1 / RMS(X_n), Z~_n = S_n Z_n, and a final RMSNorm removes S_N."""
    rng = np.random.default_rng(7)
    Ws = [rng.standard_normal((D_MODEL, D_MODEL)) / 4 for _ in range(6)]
    blocks = [(lambda W: (lambda h: np.tanh(h @ W) @ W.T))(W) for W in Ws]
    X1 = rng.standard_normal((L, D_MODEL)) * np.exp(2 * rng.standard_normal((L, 1)))
    Xs, Zs = T.residual_stack(X1, blocks)
    Ss, Zts = T.scaled_residual_stack(X1, blocks)
    for n in range(len(blocks)):
        assert rel(Ss[n], 1.0 / T.rms(Xs[n])) < 1e-10
        assert rel(Zts[n], Ss[n] * Zs[n]) < 1e-10
    assert rel(Zts[-1] / T.rms(Zts[-1]), Zs[-1] / T.rms(Zs[-1])) < 1e-10
    # the row scale the oracle's hot path computes is this S_1 (gain-free)
    from oracle import linear
    from fptq_workloads import f32_to_bf16_bits, bf16_bits_to_f32
    xb = f32_to_bf16_bits(X1.astype(np.float32))
    r = linear.row_scale(xb, linear.MODE_RMS, 0.0)
    want = 1.0 / T.rms(bf16_bits_to_f32(xb).astype(np.float64))[:, 0]
    assert np.abs(r - want).max() <= 1e-6 * want.max()


def test_rtn_weights_against_rationals():
    from fractions import Fraction
    import math
    rng = np.random.default_rng(8)
    W = rng.standard_normal((5, 12))
    W[2] *= 100
    w, s_w = T.rtn_weights(W)
    assert w.dtype == np.int8 and s_w.dtype == np.float32
    assert w.min() >= -8 and w.max() <= 7
    for o in range(5):
        assert s_w[o] == np.float32(np.abs(W[o]).max() / 7.0)
        assert np.abs(w[o]).max() == 7               # the channel's largest weight lands on +-7
        for k in range(12):
            p = Fraction(float(W[o, k])) / Fraction(float(s_w[o]))
            fl = math.floor(p)
            d = p - fl
            want = fl + 1 if d > Fraction(1, 2) else fl if d < Fraction(1, 2) else fl + (fl % 2)
            assert w[o, k] == max(-8, min(7, want))


def test_merged_quantized_weights_feed_the_linear_layer():
    """The offline side ends in what the hot path consumes: [N, K] int4 values + fp32 scales, and
    the dequantised merged weight stays within half a step of the merged FP weight."""
    rng, X, Wq, Wk, Wv, Wo = toy_weights(9)
    Tk, Tk_bar = random_tk(rng)
    Tv, Tv_bar = random_tv(rng)
    Wq2, Wk2, Wv2, Wo2 = T.merge_attention(Wq, Wk, Wv, Wo, Tk, Tk_bar, Tv, Tv_bar)
    Wqkv = T.to_out_in(np.concatenate([Wq2, Wk2, Wv2], axis=1))
    assert Wqkv.shape == ((M_REP + 2) * H * D_HEAD, D_MODEL)
    w, s_w = T.rtn_weights(Wqkv)
    assert np.all(np.abs(w * s_w[:, None].astype(np.float64) - Wqkv) <= s_w[:, None] / 2 * (1 + 1e-6))


def test_static_scale_rules():
    rng = np.random.default_rng(10)
    x = rng.standard_normal(4096)
    x[7] = 30.0
    s_inf = T.static_scale_absmax(x)
    assert s_inf == np.float32(30.0 / 7.0)
    s3 = T.static_scale_lp(x, 3.0)
    assert 0 < s3 < s_inf                    # the L3 grid clips the outlier
    err = lambda s: np.sum(np.abs(x - s * np.clip(np.rint(x / s), -8, 7)) ** 3)
    assert err(float(s3)) <= err(float(s_inf))


def test_residual_rotation_is_mergeable_and_commutes_with_the_norm():
    """x' = x T_r with every reader T_r^-1 W and every writer W T_r (Sec. 3.1.4): a two-block pre-norm residual
    network gives the rotated output, block by block, and a non-orthogonal T_r does not (the norm sees it)."""
    rng = np.random.default_rng(21)
    d, f, L = 24, 40, 6
    X = rng.standard_normal((L, d)) * np.exp(rng.standard_normal((L, 1)))
    Wg, Wu, Wd = (rng.standard_normal((d, f)) / 5, rng.standard_normal((d, f)) / 5, rng.standard_normal((f, d)) / 5)
    W1, W2 = rng.standard_normal((d, d)) / 4, rng.standard_normal((d, d)) / 4      # a second, purely linear block: in, out

    def net(X, W1, W2, Wg, Wu, Wd):
        Z = X + (X / T.rms(X)) @ W1 @ W2
        return Z + T.gated_mlp(Z / T.rms(Z), Wg, Wu, Wd)

    want = net(X, W1, W2, Wg, Wu, Wd)
    Tr = T.random_orthogonal(rng, d)
    (W1r, Wgr, Wur), (W2r, Wdr) = T.merge_residual_rotation([W1, Wg, Wu], [W2, Wd], Tr)
    got = net(X @ Tr, W1r, W2r, Wgr, Wur, Wdr)
    assert np.abs(got - want @ Tr).max() <= 1e-10 * np.abs(want).max()
    bad = Tr * (1.0 + 0.3 * np.arange(d))[None, :]                                 # invertible, not orthogonal
    (W1b, Wgb, Wub), (W2b, Wdb) = T.merge_residual_rotation([W1, Wg, Wu], [W2, Wd], bad)
    assert np.abs(net(X @ bad, W1b, W2b, Wgb, Wub, Wdb) - want @ bad).max() > 1e-3 * np.abs(want).max()


def test_up_down_scaler_is_function_preserving_also_with_the_hadamard():
    """T_u merged into W_u and W_d (Sec. 3.1.4, App. H) leaves the gated MLP unchanged, alone and stacked with the
    block-wise Hadamard in front of the down projection; scaling the gate branch instead would not."""
    rng = np.random.default_rng(22)
    d, f, L = 16, 96, 5                                      # f = 3 * 32: a Hadamard block of 32
    x = rng.standard_normal((L, d))
    Wg, Wu, Wd = rng.standard_normal((d, f)) / 4, rng.standard_normal((d, f)) / 4, rng.standard_normal((f, d)) / 6
    u = np.exp(rng.standard_normal(f))
    want = T.gated_mlp(x, Wg, Wu, Wd)
    Wu2, Wd2 = T.merge_up_down_scaler(Wu, Wd, u)
    assert np.abs(T.gated_mlp(x, Wg, Wu2, Wd2) - want).max() <= 1e-12 * np.abs(want).max()
    g = x @ Wg
    h = (g / (1.0 + np.exp(-g))) * (x @ Wu2)                 # what the online transform sees
    Td = T.block_hadamard_matrix(f, 32)
    assert np.abs((h @ Td) @ T.merge_hadamard_down(Wd2, 32) - want).max() <= 1e-12 * np.abs(want).max()
    Wg_bad = Wg * u[None, :]                                 # the gate goes through a nonlinearity: not mergeable there
    assert np.abs(T.gated_mlp(x, Wg_bad, Wu, Wd2) - want).max() > 1e-3 * np.abs(want).max()


def test_static_scale_lp_against_exhaustive_search_over_levels():
    """App. D range setting by brute force on tiny vectors: for every candidate scale the quantized value of an entry is,
    by definition, the nearest of the 16 levels s * {-8 .. 7}; the error is the sum of cubed distances; all in exact
    rationals, every candidate tried.  Also the closed-form case: data lying on the min-max grid keep the min-max scale."""
    from fractions import Fraction
    rng = np.random.default_rng(77)
    for trial in range(6):
        n = 160 if trial % 2 else int(rng.integers(3, 9))
        x = [Fraction(int(v), 64) for v in rng.integers(-400, 401, n)]
        if trial % 2:
            x[0] = Fraction(int(rng.integers(700, 900)), 64)            # an outlier worth clipping among 159 small values
        n_grid = 40
        s_max = max(abs(v) for v in x) / 7
        best, best_err = None, None
        for i in range(1, n_grid + 1):
            s = s_max * i / n_grid
            err = sum(min(abs(v - s * q) for q in range(-8, 8)) ** 3 for v in x)
            if best_err is None or err < best_err:
                best, best_err = s, err
        got = T.static_scale_lp(np.array([float(v) for v in x]), 3.0, n_grid)
        assert got == np.float32(float(best)), (trial, got, float(best))
        if trial % 2:
            assert best < s_max                                            # the outlier is clipped
    # points on the grid of the min-max scale, both ends used: zero error there and nowhere else among the candidates
    g = np.array([-7, -3, 0, 1, 5, 7, 2, -6], np.float64) * 0.375
    assert T.static_scale_lp(g, 3.0) == np.float32(0.375)
