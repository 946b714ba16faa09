"""Pins for the oracle's winner-take-all codes and band packing (Eq. 4-8, Table 5).

Each check is against something other than the oracle itself: the paper's printed example,
numpy's argmax, or an invariance the definition implies (the code depends only on the relative
order of the K selected coordinates)."""
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden", "table5_wta_example.txt")


def _read_table5():
    H, perms, K, W, codes, bands = None, [], None, None, None, None
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        key, *vals = line.split()
        if key == "H":
            H = np.array([float(v) for v in vals], dtype=np.float32)
        elif key == "K":
            K = int(vals[0])
        elif key == "W":
            W = int(vals[0])
        elif key == "permute":
            perms.append([int(v) - 1 for v in vals])     # printed 1-based
        elif key == "codes_printed":
            codes = np.array([int(v) - 1 for v in vals])  # printed 1-based
        elif key == "bands_printed":
            bands = np.array([int(v, 2) for v in vals])
        elif key == "field_bits_printed":
            field_bits = int(vals[0])
    # the table prints each code in a field of `field_bits` bits; a window of 2**field_bits
    # entries is the K whose codes need exactly that width
    return H, np.array(perms, dtype=np.int32), K, W, codes, bands, 1 << field_bits


def test_table5_rows_as_printed_pin_last_band():
    H, perms, K, W, codes, bands, K_printed_width = _read_table5()
    got = oracle.wta_codes(H[None, :], perms[:, :K])[0]
    assert got[2] == codes[2] and got[3] == codes[3]
    assert oracle.band_codes(got[None, :], W, K_printed_width)[0][1] == bands[1] == 0b0100
    assert oracle.band_codes(got[None, :], W, K)[0][1] == 0b10      # u*log2(K) = 2 bits


def test_table5_first_two_rows_exchanged_reproduces_everything():
    H, perms, K, W, codes, bands, K_printed_width = _read_table5()
    perms = perms[[1, 0, 2, 3]]
    got = oracle.wta_codes(H[None, :], perms[:, :K])[0]
    assert got.tolist() == codes.tolist() == [0, 1, 1, 0]
    b = oracle.band_codes(got[None, :], W, K_printed_width)[0]
    assert b.tolist() == bands.tolist() == [0b0001, 0b0100]
    assert oracle.band_codes(got[None, :], W, K)[0].tolist() == [0b01, 0b10]


def test_table5_packing_rule_alone():
    # printed codes (1,2) -> (00)(01) -> 0001 ; (2,1) -> 0100 : 0-based, first code most significant
    codes = np.array([[0, 1, 1, 0]], dtype=np.int32)
    assert oracle.band_codes(codes, 2, 4)[0].tolist() == [0b0001, 0b0100]   # 2-bit fields as printed
    assert oracle.band_codes(codes, 2, 2)[0].tolist() == [0b01, 0b10]       # 1-bit fields (K=2)


def test_code_is_numpy_argmax_of_gathered_window():
    rng = np.random.default_rng(1)
    X = rng.standard_normal((50, 40)).astype(np.float32)
    perms = np.stack([rng.permutation(40)[:8] for _ in range(12)]).astype(np.int32)
    got = oracle.wta_codes(X, perms)
    want = np.argmax(X[:, perms], axis=2)       # [n, P, K] -> first maximum
    assert np.array_equal(got, want)


def test_identity_window_over_all_dims_is_argmax():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((30, 16)).astype(np.float32)
    perms = np.arange(16, dtype=np.int32)[None, :]
    assert np.array_equal(oracle.wta_codes(X, perms)[:, 0], np.argmax(X, axis=1))


def test_ties_go_to_lowest_index_and_signed_zero_ties():
    X = np.array([[1.0, 1.0, 1.0, 1.0], [0.0, 2.0, 2.0, -1.0], [-0.0, 0.0, -5.0, -5.0]],
                 dtype=np.float32)
    perms = np.array([[0, 1, 2, 3], [3, 2, 1, 0]], dtype=np.int32)
    got = oracle.wta_codes(X, perms)
    assert got.tolist() == [[0, 0], [1, 1], [0, 2]]


def test_invariant_under_order_preserving_maps():
    rng = np.random.default_rng(3)
    # well separated values so that no fp32 rounding can create or break a tie
    X = (rng.permutation(64 * 20).reshape(20, 64).astype(np.float32) - 600.0) / 16.0
    perms = np.stack([rng.permutation(64)[:8] for _ in range(16)]).astype(np.int32)
    base = oracle.wta_codes(X, perms)
    for f in (lambda x: x * 4.0, lambda x: x * 0.125, lambda x: x + 3.0,
              lambda x: x ** 3, lambda x: np.exp(x / 16.0), lambda x: np.arctan(x)):
        Y = f(X.astype(np.float64)).astype(np.float32)
        assert np.array_equal(oracle.wta_codes(Y, perms), base)


def test_negation_turns_argmax_into_argmin():
    rng = np.random.default_rng(4)
    X = rng.standard_normal((40, 32)).astype(np.float32)
    perms = np.stack([rng.permutation(32)[:4] for _ in range(8)]).astype(np.int32)
    got = oracle.wta_codes(-X, perms)
    assert np.array_equal(got, np.argmin(X[:, perms], axis=2))


def test_bf16_rows_hash_on_their_stored_values():
    import workloads
    rng = np.random.default_rng(5)
    X = rng.standard_normal((64, 48)).astype(np.float32)
    bits = workloads.f32_to_bf16_bits(X)
    perms = np.stack([rng.permutation(48)[:8] for _ in range(8)]).astype(np.int32)
    Xr = workloads.bf16_bits_to_f32(bits)
    assert np.array_equal(oracle.wta_codes(bits, perms), np.argmax(Xr[:, perms], axis=2))
    # coarse values: many exact ties inside a window, all resolved to the lowest index
    coarse = workloads.f32_to_bf16_bits(np.round(X).astype(np.float32))
    vals = workloads.bf16_bits_to_f32(coarse)[:, perms]
    assert (np.sort(vals, axis=2)[:, :, -1] == np.sort(vals, axis=2)[:, :, -2]).any()
    assert np.array_equal(oracle.wta_codes(coarse, perms), np.argmax(vals, axis=2))


@pytest.mark.parametrize("K,P,W", [(8, 16, 4), (16, 48, 12), (2, 4, 2), (5, 6, 2), (64, 20, 4)])
def test_band_packing_roundtrip(K, P, W):
    rng = np.random.default_rng(6)
    codes = rng.integers(0, K, size=(100, P)).astype(np.int32)
    bits = int(np.ceil(np.log2(K)))
    u = P // W
    band = oracle.band_codes(codes, W, K)
    assert band.min() >= 0 and band.max() < (1 << (u * bits))
    for i in range(u):                      # unpack: first code is most significant
        shift = bits * (u - 1 - i)
        assert np.array_equal((band >> shift) & ((1 << bits) - 1),
                              codes.reshape(100, W, u)[:, :, i])
    # equal band code <=> equal u-tuple
    a, b = codes[:50].reshape(50, W, u), codes[50:].reshape(50, W, u)
    assert np.array_equal(band[:50] == band[50:], (a == b).all(axis=2))


def test_band_packing_rejects_bad_shapes():
    codes = np.zeros((1, 33), dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.band_codes(codes, 4, 8)          # P % W != 0
    with pytest.raises(ValueError):
        oracle.band_codes(np.zeros((1, 33), dtype=np.int32), 3, 8)   # u*bits = 33 > 30
