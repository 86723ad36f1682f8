"""Pins of the oracle's LSTM cell step (quantised gate matrices stacked into one 4H-row matrix,
Sec. II-C for the layer shape; the cell is the textbook one) against a library routine and closed
forms, chosen so that a swapped gate, a dropped bias or a wrong activation fails one of them."""
import numpy as np
import pytest


def _inputs(H, n, q, b, seed):
    rng = np.random.default_rng(seed)
    B = (rng.integers(0, 2, size=(q, 4 * H, n), dtype=np.int8) * 2 - 1).astype(np.int8)
    alpha = rng.uniform(0.01, 0.08, size=(q, 4 * H)).astype(np.float32)
    bias = rng.uniform(-0.5, 0.5, size=4 * H).astype(np.float32)
    X = rng.standard_normal((b, n)).astype(np.float32)
    C = rng.standard_normal((b, H)).astype(np.float32)
    return B, alpha, bias, X, C


def test_against_torch_lstm_cell_on_the_dense_weights(oracle):
    """torch.nn.LSTMCell (gates i, f, g, o) in float64 on W = sum_i alpha_i B_i split into its input
    and recurrent column blocks, [x ; h] split accordingly."""
    import torch

    for (H, I, q, b) in [(5, 7, 2, 3), (16, 16, 3, 1), (9, 30, 1, 4)]:
        n = I + H
        B, alpha, bias, X, C = _inputs(H, n, q, b, 100 + H)
        W = np.einsum("im,imn->mn", alpha.astype(np.float64), B.astype(np.float64))
        cell = torch.nn.LSTMCell(I, H, bias=True, dtype=torch.float64)
        with torch.no_grad():
            cell.weight_ih.copy_(torch.from_numpy(W[:, :I]))
            cell.weight_hh.copy_(torch.from_numpy(W[:, I:]))
            cell.bias_ih.copy_(torch.from_numpy(bias.astype(np.float64)))
            cell.bias_hh.zero_()
            h_t, c_t = cell(torch.from_numpy(X[:, :I].astype(np.float64)),
                            (torch.from_numpy(X[:, I:].astype(np.float64)), torch.from_numpy(C.astype(np.float64))))
        h, c = oracle.lstm_cell(B, alpha, bias, X, C)
        np.testing.assert_allclose(h, h_t.numpy(), rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(c, c_t.numpy(), rtol=1e-12, atol=1e-14)


def test_zero_scales_give_the_closed_form(oracle):
    """alpha = 0 and bias = 0: every pre-activation is 0, sigma(0) = 1/2, tanh(0) = 0, hence
    c' = c / 2 and h' = tanh(c / 2) / 2."""
    B, alpha, bias, X, C = _inputs(6, 11, 2, 3, 7)
    h, c = oracle.lstm_cell(B, np.zeros_like(alpha), np.zeros_like(bias), X, C)
    np.testing.assert_allclose(c, C.astype(np.float64) / 2, rtol=0, atol=1e-16)
    np.testing.assert_allclose(h, np.tanh(C.astype(np.float64) / 2) / 2, rtol=1e-15, atol=0)


def test_saturated_gates_select_each_path(oracle):
    """Biases of +-40 saturate the sigmoids to 0 / 1 (to 4e-18): each gate's role shows on its own."""
    H, n, q, b = 4, 9, 2, 2
    B, alpha, bias, X, C = _inputs(H, n, q, b, 11)
    Z = oracle.gemm_dense(B, alpha, X)                                  # pre-activations without bias
    big = np.float32(40.0)
    # forget gate open, input gate shut, output gate open: c' = c, h' = tanh(c)
    bias1 = np.concatenate([-big * np.ones(H), big * np.ones(H), np.zeros(H), big * np.ones(H)]).astype(np.float32)
    h, c = oracle.lstm_cell(B, np.zeros_like(alpha), bias1, X, C)
    np.testing.assert_allclose(c, C, rtol=0, atol=1e-15)
    np.testing.assert_allclose(h, np.tanh(C.astype(np.float64)), rtol=1e-15, atol=1e-16)
    # input gate open, forget gate shut: c' = tanh(z_g) with z_g from rows [2H, 3H) plus their bias
    a2 = alpha.copy(); a2[:, :2 * H] = 0; a2[:, 3 * H:] = 0            # only the candidate rows multiply
    bias2 = np.concatenate([big * np.ones(H), -big * np.ones(H), 0.25 * np.ones(H), big * np.ones(H)]).astype(np.float32)
    Zg = oracle.gemm_dense(B, a2, X)[:, 2 * H:3 * H] + 0.25
    h, c = oracle.lstm_cell(B, a2, bias2, X, C)
    np.testing.assert_allclose(c, np.tanh(Zg), rtol=1e-14, atol=1e-15)
    np.testing.assert_allclose(h, np.tanh(np.tanh(Zg)), rtol=1e-14, atol=1e-15)
    # output gate from rows [3H, 4H): h' = sigma(z_o) tanh(c') with c' = c (as in the first case)
    a3 = alpha.copy(); a3[:, :3 * H] = 0
    bias3 = np.concatenate([-big * np.ones(H), big * np.ones(H), np.zeros(H), np.zeros(H)]).astype(np.float32)
    Zo = oracle.gemm_dense(B, a3, X)[:, 3 * H:]
    h, c = oracle.lstm_cell(B, a3, bias3, X, C)
    np.testing.assert_allclose(h, np.tanh(C.astype(np.float64)) / (1 + np.exp(-Zo)), rtol=1e-14, atol=1e-15)
    assert Z.shape == (b, 4 * H)


def test_argument_errors(oracle):
    B, alpha, bias, X, C = _inputs(3, 5, 1, 2, 3)
    with pytest.raises(oracle.OracleError):
        oracle.lstm_cell(B[:, :11], alpha[:, :11], bias[:11], X, C)      # rows not a multiple of 4
    with pytest.raises(oracle.OracleError):
        oracle.lstm_cell(B, alpha, bias, X, C[:, :2])
