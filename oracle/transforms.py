"""Offline, FP64 side of the oracle: the mergeable function-preserving transforms and the
weight quantizer that produce the INT4 weights the hot path consumes (test infrastructure only).

Convention of the paper is kept here: tokens are row vectors, y = x W with W of shape
[d_in, d_out].  `to_out_in` turns a merged weight into the [N, K] = [out, in] layout the
linear layer uses.

Passages followed:
  pre-RoPE transform  (T_k, T_k-bar)      Sec. 3.1.1, Theorem 1, Eq. (1)-(4), App. C (proof, remark)
  multi-head value transform (T_v)        Sec. 3.1.2
  per-token residual scaling S_n          Sec. 3.1.3, Eq. (5)-(7)
  RMSNorm gain folded into the next linear  Sec. 4.1 (transforms and norm scales are merged)
  online Hadamard T_d before the down projection, block-wise for non-powers of 2   Sec. 3.1.4, App. D
  residual rotation T_r and per-channel up/down scaler T_u (both fully mergeable)   Sec. 3.1.4, Sec. 3.2.1 (Eq. 8), App. H
  round-to-nearest weight quantization    Sec. 4 "RTN", App. D

Readings where the text is inconsistent:
  * Theorem 1 takes s_n per 2x2 block while Eq. (1) writes s in R^d: one scalar per
    rotation pair is used, since a scale that differs inside a pair does not commute with RoPE.
  * Theorem 1 says R_n in O(2), the remark after the proof excludes reflections: rotations
    only; `reflect` exists to build the counter-example.
  * Eq. (4) and the T_v-bar equation print only the first head repeated m times: every
    head's block is repeated m times (text of Sec. 3.1.1 / 3.1.2).
"""
import numpy as np


# ----------------------------------------------------------------------------- RoPE
def adjacent_pairs(d_head):
    """RoPE pairs (2n, 2n+1) -- the block-diagonal form used in App. C."""
    return [(2 * n, 2 * n + 1) for n in range(d_head // 2)]


def half_split_pairs(d_head):
    """The 'rotate-half' channel pairing (n, n + d/2) used by some implementations."""
    return [(n, n + d_head // 2) for n in range(d_head // 2)]


def rot2(phi):
    c, s = np.cos(phi), np.sin(phi)
    return np.array([[c, s], [-s, c]], dtype=np.float64)  # acts on row vectors: x @ R


def pair_block_matrix(blocks, pairs, d_head):
    """d x d matrix that applies 2x2 block n to channel pair pairs[n] (row-vector convention)."""
    T = np.zeros((d_head, d_head), dtype=np.float64)
    for B, (a, b) in zip(blocks, pairs):
        T[np.ix_([a, b], [a, b])] = B
    return T


def rope_matrix(d_head, pos, thetas, pairs=None):
    """R_{Theta,pos}: block n rotates pair n by pos * theta_n (App. C, RoPE background)."""
    pairs = adjacent_pairs(d_head) if pairs is None else pairs
    return pair_block_matrix([rot2(pos * th) for th in thetas], pairs, d_head)


def default_thetas(d_head, base=10000.0):
    n = np.arange(d_head // 2, dtype=np.float64)
    return base ** (-2.0 * n / d_head)


# ----------------------------------------------------------------------------- T_k
def prerope_head_transform(scales, angles, pairs, d_head, reflect=None):
    """One key head's (T, T-bar): T = diag(s) diag(R_n), T-bar = diag(1/s) diag(R_n)  (Theorem 1).

    scales, angles: one per rotation pair.  reflect: optional boolean per pair that swaps the
    rotation for a reflection (det -1) -- only for the negative test of the remark in App. C.
    """
    scales = np.asarray(scales, dtype=np.float64)
    blocks, blocks_bar = [], []
    for n, (s, phi) in enumerate(zip(scales, angles)):
        R = rot2(phi)
        if reflect is not None and reflect[n]:
            R = R @ np.array([[1.0, 0.0], [0.0, -1.0]])
        blocks.append(s * R)
        blocks_bar.append(R / s)
    return pair_block_matrix(blocks, pairs, d_head), pair_block_matrix(blocks_bar, pairs, d_head)


def block_diag(mats):
    n = sum(m.shape[0] for m in mats)
    out = np.zeros((n, n), dtype=np.float64)
    o = 0
    for m in mats:
        d = m.shape[0]
        out[o:o + d, o:o + d] = m
        o += d
    return out


def prerope_transform(scales, angles, m, pairs=None, reflect=None):
    """Eq. (1)-(4): T_k over H key heads and T_k-bar over m*H query heads.

    scales, angles: [H, d_head/2].  Query heads h*m .. h*m+m-1 read key head h.
    """
    scales, angles = np.asarray(scales, np.float64), np.asarray(angles, np.float64)
    H, N = scales.shape
    d_head = 2 * N
    pairs = adjacent_pairs(d_head) if pairs is None else pairs
    Ts, Tbars = [], []
    for h in range(H):
        T, Tb = prerope_head_transform(scales[h], angles[h], pairs, d_head,
                                       None if reflect is None else reflect[h])
        Ts.append(T)
        Tbars.extend([Tb] * m)
    return block_diag(Ts), block_diag(Tbars)


# ----------------------------------------------------------------------------- T_v
def value_transform(Tv_heads, m):
    """Sec. 3.1.2: T_v = diag(T_v^(h)), T_v-bar = diag of the inverses, each repeated m times."""
    Tv_heads = [np.asarray(T, np.float64) for T in Tv_heads]
    bars = []
    for T in Tv_heads:
        bars.extend([np.linalg.inv(T)] * m)
    return block_diag(Tv_heads), block_diag(bars)


# ----------------------------------------------------------------------------- merging
def merge_attention(Wq, Wk, Wv, Wo, Tk, Tk_bar, Tv, Tv_bar):
    """W~_q = W_q T_k-bar, W~_k = W_k T_k (Theorem 1); W~_v = W_v T_v, W~_o = T_v-bar W_o (Sec. 3.1.2)."""
    return Wq @ Tk_bar, Wk @ Tk, Wv @ Tv, Tv_bar @ Wo


def fold_norm_gain(W, gain):
    """RMSNorm(x) W with gain g equals (x / RMS(x)) (diag(g) W): the gain moves into the weight."""
    return np.asarray(gain, np.float64)[:, None] * W


def to_out_in(W):
    """[d_in, d_out] of the paper -> [N, K] = [out, in] of the linear layer."""
    return np.ascontiguousarray(W.T)


# ----------------------------------------------------------------------------- toy attention
def rms(x):
    """||x||_R = ||x||_2 / sqrt(d) along the last axis (Sec. 3.1.3, Step 1)."""
    return np.sqrt(np.mean(np.square(x), axis=-1, keepdims=True))


def attention(X, Wq, Wk, Wv, Wo, H, m, d_head, thetas=None, pairs=None, causal=True):
    """Plain grouped-query attention with RoPE on row-vector tokens X [L, d_model], FP64."""
    L = X.shape[0]
    thetas = default_thetas(d_head) if thetas is None else thetas
    q = (X @ Wq).reshape(L, m * H, d_head)
    k = (X @ Wk).reshape(L, H, d_head)
    v = (X @ Wv).reshape(L, H, d_head)
    for i in range(L):
        R = rope_matrix(d_head, i, thetas, pairs)
        q[i] = q[i] @ R
        k[i] = k[i] @ R
    out = np.zeros((L, m * H, d_head))
    for hq in range(m * H):
        hk = hq // m
        logits = q[:, hq, :] @ k[:, hk, :].T / np.sqrt(d_head)
        if causal:
            logits = np.where(np.tril(np.ones((L, L), bool)), logits, -np.inf)
        logits = logits - logits.max(axis=1, keepdims=True)
        A = np.exp(logits)
        A /= A.sum(axis=1, keepdims=True)
        out[:, hq, :] = A @ v[:, hk, :]
    return out.reshape(L, m * H * d_head) @ Wo


def qk_logit(xi, xj, Wq_head, Wk_head, i, j, thetas, pairs=None):
    """<f(x_i W_q, i), f(x_j W_k, j)> of Theorem 1 for one head."""
    d_head = Wq_head.shape[1]
    return float((xi @ Wq_head @ rope_matrix(d_head, i, thetas, pairs))
                 @ (xj @ Wk_head @ rope_matrix(d_head, j, thetas, pairs)))


# ----------------------------------------------------------------------------- S_n recursion
def residual_stack(X1, blocks):
    """Reference pre-norm residual network: X_{n+1} = Z_n = X_n + F_n(X_n / RMS(X_n)).

    Returns the lists [X_1..X_N] and [Z_1..Z_N]."""
    Xs, Zs = [], []
    X = X1
    for F in blocks:
        Z = X + F(X / rms(X))
        Xs.append(X)
        Zs.append(Z)
        X = Z
    return Xs, Zs


def scaled_residual_stack(X1, blocks):
    """The same network with the norm moved onto the residual (Sec. 3.1.3, Steps 1-2) and S_n
    from the recursion of Eq. (6)-(7): S_0 = 1, Z~_0 = X_1, S_n = S_{n-1} / RMS(Z~_{n-1}).

    Only Z~ and S are carried from block to block; X_n itself is never rebuilt.
    Returns the lists [S_1..S_N] (each [L, 1]) and [Z~_1..Z~_N]."""
    Ss, Zts = [], []
    S_prev = np.ones((X1.shape[0], 1))
    Zt_prev = X1
    for F in blocks:
        nrm = rms(Zt_prev)
        S = S_prev / nrm
        Xt = Zt_prev / nrm                 # = S_n * X_n, unit RMS
        Yt = S * F(Xt / rms(Xt))           # Eq. (5): block output rescaled by the same S_n
        Zt = Xt + Yt
        Ss.append(S)
        Zts.append(Zt)
        S_prev, Zt_prev = S, Zt
    return Ss, Zts


# ----------------------------------------------------------------------------- online Hadamard T_d
def hadamard_matrix(n):
    """H_n = kron of [[1, 1], [1, -1]] (App. D), n a power of two; unnormalised."""
    H = np.ones((1, 1))
    while H.shape[0] < n:
        H = np.kron(H, np.array([[1.0, 1.0], [1.0, -1.0]]))
    assert H.shape[0] == n
    return H


def block_hadamard_matrix(K, block):
    """T_d for a width that is not a power of two: blockdiag of H_block / sqrt(block) (App. D)."""
    assert K % block == 0
    return block_diag([hadamard_matrix(block) / np.sqrt(block)] * (K // block))


def merge_hadamard_down(Wd, block):
    """W~_d = T_d^T W_d for y = x W_d with W_d [d_ff, d_model]: (x T_d)(T_d^T W_d) = x W_d."""
    Td = block_hadamard_matrix(Wd.shape[0], block)
    return Td.T @ Wd


def largest_pow2_divisor(K):
    return K & (-K)


# ----------------------------------------------------------------------------- T_r and T_u
def merge_residual_rotation(W_in, W_out, Tr):
    """Rotating the residual stream, x' = x T_r (Sec. 3.1.4): every linear that reads the residual becomes
    T_r^-1 W and every linear that writes to it W T_r, the placement the local objective of Sec. 3.2.1 sums
    over.  An orthogonal T_r commutes with the gain-free RMS normalisation (row norms are kept), so nothing
    runs at inference time.  W_in, W_out: lists of [d_in, d_out] matrices."""
    Tr = np.asarray(Tr, np.float64)
    Tr_inv = np.linalg.inv(Tr)
    return [Tr_inv @ W for W in W_in], [W @ Tr for W in W_out]


def merge_up_down_scaler(Wu, Wd, u):
    """Per-channel scaler T_u = diag(u) between the up and the down projection (Sec. 3.1.4, App. H): the up
    projection's output channels are scaled, W_u diag(u), and the down projection undoes it, diag(1/u) W_d.
    The gate branch multiplies element-wise and is left alone, so (act(x W_g) * (x W_u diag(u))) diag(1/u) W_d
    is the original MLP."""
    u = np.asarray(u, np.float64)
    return np.asarray(Wu, np.float64) * u[None, :], np.asarray(Wd, np.float64) / u[:, None]


def random_orthogonal(rng, d):
    Q, R = np.linalg.qr(rng.standard_normal((d, d)))
    return Q * np.sign(np.diag(R))


def gated_mlp(x, Wg, Wu, Wd):
    g = x @ Wg
    return ((g / (1.0 + np.exp(-g))) * (x @ Wu)) @ Wd


# ----------------------------------------------------------------------------- weight quantizer
def rtn_weights(W_out_in):
    """Per-output-channel symmetric round-to-nearest INT4: s_w[o] = max_k |W[o,k]| / 7 (fp32),
    w = clamp(rne(W / s_w), -8, 7).  Returns (int8 [N, K], float32 [N])."""
    W = np.asarray(W_out_in, np.float64)
    s_w = (np.abs(W).max(axis=1) / 7.0).astype(np.float32)
    s_w = np.where(s_w > 0, s_w, np.float32(1.0)).astype(np.float32)
    w = np.clip(np.rint(W / s_w.astype(np.float64)[:, None]), -8, 7).astype(np.int8)
    return w, s_w


def static_scale_absmax(x_tilde):
    """Min-max (L-infinity) range setting of App. D: s_a = max|x~| / 7 on calibration data."""
    return np.float32(np.abs(np.asarray(x_tilde, np.float64)).max() / 7.0)


def static_scale_lp(x_tilde, p=3.0, n_grid=100):
    """App. D range setting: the scale minimising ||x~ - s q(x~ / s)||_p over a grid of
    shrink factors of the min-max scale (p = 3 in the paper)."""
    x = np.asarray(x_tilde, np.float64).ravel()
    s_max = np.abs(x).max() / 7.0
    best, best_err = s_max, np.inf
    for i in range(1, n_grid + 1):
        s = s_max * i / n_grid
        err = np.sum(np.abs(x - s * np.clip(np.rint(x / s), -8, 7)) ** p)
        if err < best_err:
            best, best_err = s, err
    return np.float32(best)
