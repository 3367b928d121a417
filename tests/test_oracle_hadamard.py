"""Pins for the oracle's block-wise online Hadamard transform (App. D, "Hadamard non-powers of 2")."""
import numpy as np
import pytest

from oracle import transforms as T
import fptq_workloads as synth


def test_matches_the_kronecker_definition_exactly_on_small_integers(oracle):
    """Small integer inputs: every partial sum is exact in fp32, so the butterflies must equal x H."""
    rng = np.random.default_rng(0)
    for K, B in [(8, 8), (64, 16), (768, 256), (11008 // 43 * 3, 256), (2048, 1024), (1024, 512), (4096, 2048), (4096, 4096)]:
        x = rng.integers(-8, 9, (5, K)).astype(np.float32)
        h = oracle.hadamard_rows(synth.f32_to_bf16_bits(x), B)
        Hb = T.block_hadamard_matrix(K, B) * np.sqrt(B)
        assert np.array_equal(h.astype(np.float64), x.astype(np.float64) @ Hb)


def test_matches_the_definition_within_fp32_on_random_inputs(oracle):
    rng = np.random.default_rng(1)
    K, B = 1024, 256
    xb = synth.f32_to_bf16_bits(rng.standard_normal((7, K)).astype(np.float32) * 3)
    h = oracle.hadamard_rows(xb, B).astype(np.float64)
    want = synth.bf16_bits_to_f32(xb).astype(np.float64) @ (T.block_hadamard_matrix(K, B) * np.sqrt(B))
    assert np.abs(h - want).max() <= 8 * 2.0 ** -24 * np.abs(want).max() * np.log2(B)


def test_involution_parseval_and_block_locality(oracle):
    rng = np.random.default_rng(2)
    K, B = 512, 128
    x = rng.integers(-4, 5, (3, K)).astype(np.float32)
    xb = synth.f32_to_bf16_bits(x)
    h = oracle.hadamard_rows(xb, B)
    # Parseval: ||H x||^2 = B ||x||^2 per block
    for b in range(K // B):
        blk = slice(b * B, (b + 1) * B)
        assert np.allclose((h[:, blk].astype(np.float64) ** 2).sum(1), B * (x[:, blk].astype(np.float64) ** 2).sum(1))
    # H (H x) = B x (values stay small integers times B: exact)
    hh = oracle.hadamard_rows(synth.f32_to_bf16_bits(h), B)
    assert np.array_equal(hh, B * x)
    # changing one block changes only that block of the output
    x2 = x.copy()
    x2[:, B:2 * B] += 1
    h2 = oracle.hadamard_rows(synth.f32_to_bf16_bits(x2), B)
    assert np.array_equal(h2[:, :B], h[:, :B]) and np.array_equal(h2[:, 2 * B:], h[:, 2 * B:])
    assert not np.array_equal(h2[:, B:2 * B], h[:, B:2 * B])
    # first output of a block is the plain sum, the transform of a unit vector is a +-1 row
    e = np.zeros((1, K), np.float32)
    e[0, 5] = 1
    he = oracle.hadamard_rows(synth.f32_to_bf16_bits(e), B)
    assert set(np.unique(he[0, :B]).tolist()) == {-1.0, 1.0} and not he[0, B:].any()
    assert np.array_equal(h[:, 0], x[:, :B].sum(1))


def test_bad_block_is_rejected(oracle):
    xb = np.zeros((1, 96), np.uint16)
    for B in (0, 3, 64, 24):
        with pytest.raises(ValueError):
            oracle.hadamard_rows(xb, B)
    assert oracle.hadamard_rows(xb, 32).shape == (1, 96)


def test_blockwise_hadamard_is_function_preserving_and_zero_padding_is_not():
    """(x T_d)(T_d^T W_d) = x W_d for a width that is not a power of two (43 * 16 here, as 11008 = 43 * 256);
    padding with zeros to the next power of two and dropping the extra outputs is not (App. D)."""
    rng = np.random.default_rng(3)
    d_ff, d_model, B = 43 * 16, 24, 16
    x = rng.standard_normal((6, d_ff))
    Wd = rng.standard_normal((d_ff, d_model))
    Td = T.block_hadamard_matrix(d_ff, B)
    assert np.allclose(Td @ Td.T, np.eye(d_ff))
    assert np.abs((x @ Td) @ T.merge_hadamard_down(Wd, B) - x @ Wd).max() < 1e-10
    n2 = 1024
    Hp = T.hadamard_matrix(n2) / np.sqrt(n2)
    xp = np.concatenate([x, np.zeros((6, n2 - d_ff))], axis=1) @ Hp          # transform of the padded input
    Wp = (Hp.T @ np.concatenate([Wd, np.zeros((n2 - d_ff, d_model))], axis=0))  # merged, padded weight
    assert np.abs(xp @ Wp - x @ Wd).max() < 1e-10            # keeping all n2 rows would be fine ...
    assert np.abs(xp[:, :d_ff] @ Wp[:d_ff] - x @ Wd).max() > 1e-2   # ... dropping the added rows is not
    assert T.largest_pow2_divisor(11008) == 256 and T.largest_pow2_divisor(14336) == 2048 and T.largest_pow2_divisor(28672) == 4096


def test_quantize_hadamard_uses_the_scalar_rule_on_the_transformed_row(oracle):
    rng = np.random.default_rng(4)
    K, B = 512, 256
    xb = synth.f32_to_bf16_bits(rng.standard_normal((4, K)).astype(np.float32))
    r = rng.uniform(0.5, 2, 4).astype(np.float32)
    s_a = np.float32(0.6)
    q = oracle.quantize_hadamard(xb, s_a, B, r)
    h = oracle.hadamard_rows(xb, B)
    L = oracle.lib()
    for t in range(4):
        c = L.oracle_hadamard_multiplier(float(r[t]), float(s_a), 1, B)
        assert c == float(np.float32(np.float32(r[t] * np.float32(np.float32(1.0) / s_a)) * np.float32(1.0 / 16.0)))
        for k in range(0, K, 37):
            u = np.float32(h[t, k]) * np.float32(c)
            assert q[t, k] == int(np.clip(np.rint(u), -8, 7))
    # the transform spreads an outlier: quantizing after it clips less than quantizing the raw row
    x = rng.standard_normal((1, K)).astype(np.float32)
    x[0, 3] = 60.0
    xb = synth.f32_to_bf16_bits(x)
    hq = oracle.quantize_hadamard(xb, np.float32(1.0), B)
    assert np.abs(hq).max() <= 8 and (hq != 0).mean() > 0.5


def _f32_nearest(fr):
    """Correctly rounded (nearest, ties to even) float32 of a positive normal-range rational, in exact arithmetic."""
    from fractions import Fraction
    e = 0
    while Fraction(2) ** (e + 1) <= fr:
        e += 1
    while Fraction(2) ** e > fr:
        e -= 1
    m = round(fr / Fraction(2) ** (e - 23))          # Python rounds a Fraction half to even
    return float(np.float32(float(Fraction(m) * Fraction(2) ** (e - 23))))


def _f32_inv_sqrt(B):
    """The float32 nearest to 1 / sqrt(B), found without any floating-point square root: f is the nearest float32
    iff the real value lies between the midpoints to its neighbours, i.e. lo^2 * B < 1 < hi^2 * B in rationals."""
    from fractions import Fraction
    f = np.float32(1.0)
    while Fraction(float(f)) ** 2 * B > 1:            # walk down to the binade below 1 / sqrt(B) ...
        f = np.float32(f / 2)
    lo, hi = f, np.float32(f * 2)
    while np.nextafter(lo, np.float32(2)) < hi:       # ... then bisect on float32 values, comparing exactly
        mid = np.float32((float(lo) + float(hi)) / 2)
        if Fraction(float(mid)) ** 2 * B > 1:
            hi = mid
        else:
            lo = mid
    below, above = Fraction(float(lo)), Fraction(float(hi))
    midpoint = (below + above) / 2
    pick = hi if midpoint ** 2 * B < 1 else lo
    # the bracket that makes `pick` the nearest float32
    up, dn = np.nextafter(pick, np.float32(2)), np.nextafter(pick, np.float32(0))
    assert ((Fraction(float(pick)) + Fraction(float(dn))) / 2) ** 2 * B < 1 < ((Fraction(float(pick)) + Fraction(float(up))) / 2) ** 2 * B
    return float(pick)


@pytest.mark.parametrize("B", [8, 32, 128, 256, 512, 1024, 2048, 4096])
def test_hadamard_multiplier_rounding_and_product_order(oracle, B):
    """c_t = (S_t * (1 / s_a)) * float32(1 / sqrt(B)): the normalisation is the correctly rounded float32 of the
    irrational 1 / sqrt(B) for odd powers of two (512, 2048: the Llama-3-8B block), and the two products are taken in
    that order, each rounded to float32 once.  Everything on the expected side is exact rational arithmetic."""
    from fractions import Fraction
    L = oracle.lib()
    hn = _f32_inv_sqrt(B)
    rng = np.random.default_rng(B)
    order_matters = 0
    for _ in range(200):
        r = float(np.float32(rng.uniform(0.05, 20.0)))
        s_a = float(np.float32(rng.uniform(0.01, 3.0)))
        inv = _f32_nearest(Fraction(1) / Fraction(s_a))
        c1 = _f32_nearest(Fraction(r) * Fraction(inv))
        want = _f32_nearest(Fraction(c1) * Fraction(hn))
        assert L.oracle_hadamard_multiplier(r, s_a, 1, B) == want
        other = _f32_nearest(Fraction(r) * Fraction(_f32_nearest(Fraction(inv) * Fraction(hn))))
        order_matters += other != want
        # without a row scale the first product is skipped
        assert L.oracle_hadamard_multiplier(123.0, s_a, 0, B) == _f32_nearest(Fraction(inv) * Fraction(hn))
    if B in (512, 2048, 8, 32, 128):
        assert order_matters > 0          # the pin can tell the two association orders apart
