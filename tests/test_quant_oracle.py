"""CPU-only pins of the quantisation oracle (paper Eq. "quan" / "dequan") against things other than itself."""
import numpy as np
import pytest
import torch

from oracle import quant_oracle as qo


def test_hand_cases_with_a_tie():
    # block 1: absmax 2 -> c = 63.5 ; 63.5 * 1 = 63.5 is a tie -> even: 64 ; 63.5 * 0.5 = 31.75 -> 32
    # block 2: absmax 0.25 -> c = 508 ; 0.1 -> 50.8 -> 51 ; -0.25 -> -127 ; 0 -> 0 ; 0.001 -> 0.508 -> 1
    x = np.array([-2.0, 1.0, 0.5, 2.0, 0.1, -0.25, 0.0, 0.001], dtype=np.float32)
    codes, consts = qo.quant(x, 4, 8)
    assert consts.tolist() == [63.5, 508.0]
    assert codes.tolist() == [-127, 64, 32, 127, 51, -127, 0, 1]
    # 4 bits: c = 3.5 ; 3.5 -> tie -> 4 ; 1.75 -> 2 ;   c = 28 ; 2.8 -> 3 ; -7 ; 0 ; 0.028 -> 0
    codes4, consts4 = qo.quant(x, 4, 4)
    assert consts4.tolist() == [3.5, 28.0]
    assert qo.unpack(codes4, 8, 4).tolist() == [-7, 4, 2, 7, 3, -7, 0, 0]
    assert codes4.view(np.uint8).tolist() == [0x49, 0x72, 0x93, 0x00]      # even index in the low nibble
    # an all-zero block
    codes0, consts0 = qo.quant(np.zeros(5, dtype=np.float32), 4, 8)
    assert consts0.tolist() == [1.0, 1.0] and not codes0.any()
    # dequantisation is the division of Eq. "dequan"
    np.testing.assert_array_equal(qo.dequant(codes, consts, 8, 4, 8),
                                  np.array([-127, 64, 32, 127, 51, -127, 0, 1], dtype=np.float32)
                                  / np.repeat(consts, 4))


@pytest.mark.parametrize("bits", [8, 4])
def test_error_bound_extremes_and_ragged_tail(bits):
    rng = np.random.default_rng(3)
    qmax = 127 if bits == 8 else 7
    x = (rng.standard_normal(1000) * np.exp(rng.uniform(-3, 3, size=1000))).astype(np.float32)   # ragged: 1000 = 15 * 64 + 40
    codes, consts = qo.quant(x, 64, bits)
    q = qo.unpack(codes, x.size, bits)
    assert consts.size == 16 and np.abs(q).max() <= qmax
    back = qo.dequant(codes, consts, x.size, 64, bits)
    for b in range(16):
        blk = slice(64 * b, min(1000, 64 * b + 64))
        amax = np.abs(x[blk]).max()
        assert np.abs(q[blk]).max() == qmax                                  # the largest element maps to +-qmax
        # rounding to the nearest code: at most half a step, absmax / (2 qmax), plus float32 rounding of the products
        assert np.abs(back[blk].astype(np.float64) - x[blk]).max() <= amax / (2 * qmax) * (1 + 1e-5)


def test_blocks_are_independent():
    """An outlier only spoils the block it sits in (the reason the paper quantises block-wise)."""
    rng = np.random.default_rng(4)
    x = rng.standard_normal(256).astype(np.float32)
    y = x.copy()
    y[70] = 1000.0
    cx, kx = qo.quant(x, 64, 8)
    cy, ky = qo.quant(y, 64, 8)
    same = np.r_[0:64, 128:256]
    assert np.array_equal(cx[same], cy[same]) and kx[0] == ky[0] and np.array_equal(kx[2:], ky[2:])
    assert ky[1] == np.float32(127.0) / np.float32(1000.0) and not np.array_equal(cx[64:128], cy[64:128])
    # tensor-wise quantisation (one block) of the same data loses far more on the ordinary values
    err_block = np.abs(qo.dequant(cy, ky, 256, 64, 8) - y)[same].max()
    cz, kz = qo.quant(y, 256, 8)
    err_tensor = np.abs(qo.dequant(cz, kz, 256, 256, 8) - y)[same].max()
    assert err_tensor > 20 * err_block


def test_rounding_matches_a_library_routine():
    rng = np.random.default_rng(5)
    x = rng.standard_normal(64 * 50).astype(np.float32)
    codes, consts = qo.quant(x, 64, 8)
    xt = torch.from_numpy(x).reshape(50, 64)
    amax = xt.abs().amax(dim=1, keepdim=True)
    c = torch.tensor(127.0, dtype=torch.float32) / amax
    ref = torch.round(c * xt).to(torch.int32).ravel().numpy()              # torch.round: half to even, float32
    np.testing.assert_array_equal(codes.astype(np.int32), ref)
    np.testing.assert_array_equal(consts, c.ravel().numpy())


@pytest.mark.parametrize("bits", [8, 4])
def test_linear_layer_is_a_matrix_product_with_the_dequantised_weights(bits):
    rng = np.random.default_rng(6)
    M, K, N, block = 7, 128, 5, 32
    W = rng.standard_normal((N, K)).astype(np.float32)
    x = rng.standard_normal((M, K)).astype(np.float32)
    codes, consts = qo.quant(W, block, bits)
    Wd = qo.dequant(codes, consts, N * K, block, bits).reshape(N, K)
    y = qo.dequant_linear(x, codes, consts, N, block, bits)
    np.testing.assert_allclose(y, x.astype(np.float64) @ Wd.astype(np.float64).T, rtol=1e-13, atol=1e-13)
    # and the storage form costs what the paper says it saves: one byte (half a byte) per weight plus one float per block
    assert codes.nbytes == N * K * bits // 8 and consts.nbytes == N * K // block * 4
