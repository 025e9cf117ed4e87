"""Pins for the CPU checker's normalisation, value networks and argmin scan."""
import math

import numpy as np
import pytest
import torch

from paper_2011_14486_amd import inputs as I


def test_plog2_closed_forms(ovf):
    assert ovf.plog2([0])[0] == 0.0
    for k in range(31):
        assert ovf.plog2([1 << k])[0] == float(k)      # exact at powers of two
    assert ovf.plog2([3])[0] == 1.5 and ovf.plog2([6])[0] == 2.5 and ovf.plog2([5])[0] == 2.25
    assert ovf.plog2([2 ** 31 - 1])[0] == 31.0          # (float)(2^31-1) rounds up to 2^31
    rng = np.random.default_rng(0)
    x = np.concatenate([np.arange(1, 5000), rng.integers(1, 2 ** 31 - 1, 20000)]).astype(np.int64)
    p = ovf.plog2(x.astype(np.int32)).astype(np.float64)
    # a chord of log2 lies below the curve by at most 1 + log2(log2 e) - log2 e = 0.08607...
    err = np.log2(x.astype(np.float64)) - p
    assert err.min() > -1e-6 and err.max() <= 0.0861
    xs = np.sort(x)
    assert (np.diff(ovf.plog2(xs.astype(np.int32))) >= 0).all()  # monotone


def test_plog2_matches_integer_formula(ovf):
    """Below 2^24 the conversion to float is exact, so plog2(x) = e + (x - 2^e)/2^e with
    e = bit_length - 1: a pure-integer restatement."""
    rng = np.random.default_rng(1)
    x = np.concatenate([np.arange(1, 3000), rng.integers(1, 1 << 24, 5000)])
    want = np.array([(int(v).bit_length() - 1) + (int(v) - (1 << (int(v).bit_length() - 1))) /
                     (1 << (int(v).bit_length() - 1)) for v in x])
    got = ovf.plog2(x.astype(np.int32)).astype(np.float64)
    # one float32 rounding of the final add
    assert np.array_equal(got, want.astype(np.float32).astype(np.float64))


def test_bf16_round_matches_library_conversion(ovf):
    rng = np.random.default_rng(2)
    v = np.concatenate([rng.standard_normal(4000) * 10 ** rng.uniform(-6, 6, 4000),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, np.inf, -np.inf]]).astype(np.float32)
    want = torch.from_numpy(v).to(torch.bfloat16).to(torch.float32).numpy()
    got = ovf.bf16_round(v)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    # ties go to the even neighbour: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert ovf.bf16_round([1.00390625])[0] == 1.0 and ovf.bf16_round([1.01171875])[0] == 1.015625


def torch_mlp(dims, w, x_norm, bf16):
    """Library second opinion: torch.nn.functional.linear in float64."""
    h = torch.from_numpy(x_norm.astype(np.float64))  # [M][F]
    off = 0
    for k in range(len(dims) - 1):
        fin, fout = dims[k], dims[k + 1]
        W = torch.from_numpy(w[off:off + fin * fout].reshape(fout, fin)); off += fin * fout
        b = torch.from_numpy(w[off:off + fout]); off += fout
        if bf16:
            W = W.to(torch.bfloat16).to(torch.float32)
        h = torch.nn.functional.linear(h, W.double(), b.double())
        if k < len(dims) - 2:
            h = torch.relu(h)
            if bf16:
                h = h.float().to(torch.bfloat16).double()
    return h[:, 0].numpy()


@pytest.mark.parametrize("dims,dtype", [([64, 128, 128, 1], I.FP32), ([256, 512, 512, 1], I.BF16),
                                        ([64, 32, 1], I.BF16), ([64, 1], I.FP32)])
def test_mlp_against_library_linear(ovf, dims, dtype):
    rng = np.random.default_rng(5)
    M = 96
    x = np.floor(np.exp2(rng.random((dims[0], M)) * 20)).astype(np.int32)
    x[0, :4] = 0
    w = I.mlp_weights(dims, seed=7, bias_std=0.3)
    got = ovf.score_mlp(I.model_record(I.MLP, dims, dtype), w, x).astype(np.float64)
    xn = ovf.plog2(x).T
    if dtype == I.BF16:
        xn = torch.from_numpy(xn).to(torch.bfloat16).to(torch.float32).numpy()
    want = torch_mlp(dims, w, xn, dtype == I.BF16)
    scale = max(np.sqrt(np.mean(want ** 2)), 1e-30)
    # both sides accumulate in double and round at the same declared points; what is left
    # is the final float rounding
    tol = 2e-7 if dtype == I.FP32 else 1e-6
    assert np.max(np.abs(got - want) / np.maximum(np.abs(want), scale)) < tol


def test_mlp_special_cases(ovf):
    dims = [64, 16, 16, 1]
    n = I.mlp_param_count(dims)
    rng = np.random.default_rng(0)
    x = rng.integers(0, 1 << 20, (64, 40)).astype(np.int32)
    mod = I.model_record(I.MLP, dims, I.FP32)
    # zero weights: the value is the last bias
    w = np.zeros(n, np.float32); w[-1] = 2.5
    assert np.array_equal(ovf.score_mlp(mod, w, x), np.full(40, 2.5, np.float32))
    # a single path x_j -> hidden 3 -> hidden 5 -> out picks out plog2(x_j), and ReLU cuts a
    # negated copy to zero
    j = 11
    w = np.zeros(n, np.float32)
    W1 = w[:64 * 16].reshape(16, 64); W1[3, j] = 1.0; W1[4, j] = -1.0
    o2 = 64 * 16 + 16
    W2 = w[o2:o2 + 256].reshape(16, 16); W2[5, 3] = 1.0; W2[6, 4] = 1.0
    o3 = o2 + 256 + 16
    w[o3 + 5] = 1.0; w[o3 + 6] = 1.0
    got = ovf.score_mlp(mod, w, x)
    assert np.array_equal(got, ovf.plog2(x[j]))
    # a transposed weight matrix would be caught: W[out][in] with out != in
    dims2 = [64, 3, 1]
    w = np.zeros(I.mlp_param_count(dims2), np.float32)
    w[:192].reshape(3, 64)[2, 7] = 1.0   # hidden 2 reads input 7
    w[192 + 3 + 2] = 1.0
    assert np.array_equal(ovf.score_mlp(I.model_record(I.MLP, dims2, I.FP32), w, x), ovf.plog2(x[7]))
    # NaN weights give NaN scores (which then can never win an argmin)
    w[:] = np.nan
    assert np.isnan(ovf.score_mlp(I.model_record(I.MLP, dims2, I.FP32), w, x)).all()


def torch_lstm(F, H, w, xs, bf16):
    """Second opinion: torch.nn.LSTM (gate order i,f,g,o) in float64 for the unrounded
    model; for bf16 a step-by-step torch.nn.LSTMCell with the fed-back h rounded."""
    o = 0
    Wih = torch.from_numpy(w[o:o + 4 * H * F].reshape(4 * H, F)); o += 4 * H * F
    Whh = torch.from_numpy(w[o:o + 4 * H * H].reshape(4 * H, H)); o += 4 * H * H
    bih = torch.from_numpy(w[o:o + 4 * H]); o += 4 * H
    bhh = torch.from_numpy(w[o:o + 4 * H]); o += 4 * H
    wh = torch.from_numpy(w[o:o + H]); o += H
    bh = float(w[o])
    x = torch.from_numpy(xs.astype(np.float64))  # [B][T][F]
    B, T, _ = x.shape
    if not bf16:
        net = torch.nn.LSTM(F, H, batch_first=True).double()
        with torch.no_grad():
            net.weight_ih_l0.copy_(Wih); net.weight_hh_l0.copy_(Whh)
            net.bias_ih_l0.copy_(bih); net.bias_hh_l0.copy_(bhh)
            hs, _ = net(x)
        return (hs @ wh.double()).sum(1).numpy() + T * bh
    r = lambda t: t.float().to(torch.bfloat16).double()
    cell = torch.nn.LSTMCell(F, H).double()
    with torch.no_grad():
        cell.weight_ih.copy_(r(Wih)); cell.weight_hh.copy_(r(Whh))
        cell.bias_ih.copy_(bih); cell.bias_hh.copy_(bhh)
        h = torch.zeros(B, H, dtype=torch.float64); c = torch.zeros(B, H, dtype=torch.float64)
        v = torch.zeros(B, dtype=torch.float64)
        for t in range(T):
            h, c = cell(x[:, t], (r(h), c))
            v += h @ r(wh) + bh
    return v.numpy()


@pytest.mark.parametrize("dtype", [I.FP32, I.BF16])
def test_lstm_against_library(ovf, dtype):
    F, H, T, B = 24, 16, 9, 256
    w = I.lstm_weights(F, H, seed=3, bias_std=0.2)
    xb = I.feature_sequences(0, B, T=T, F=F, seed=9, max_log2=4.0)
    xs = (xb.astype(np.uint32) << 16).view(np.float32)
    got = ovf.score_lstm(I.model_record(I.LSTM, [F, H, 1], dtype), w, xb).astype(np.float64)
    want = torch_lstm(F, H, w, xs, dtype == I.BF16)
    scale = np.sqrt(np.mean(want ** 2))
    # the library version rounds at the same declared points (weights, x_t, fed-back h), so
    # the two agree to float rounding; a missing rounding point shows up at the 1e-3 level
    tol = 3e-7 if dtype == I.FP32 else 1e-6
    assert np.max(np.abs(got - want) / np.maximum(np.abs(want), scale)) < tol


def test_lstm_special_cases(ovf):
    F, H, T, B = 8, 4, 5, 256
    n = I.lstm_param_count(F, H)
    xb = I.feature_sequences(0, B, T=T, F=F, seed=1, max_log2=3.0)
    mod = I.model_record(I.LSTM, [F, H, 1], I.FP32)
    # zero weights: h_t = 0.5*tanh(0) = 0, so the value is T * b_head
    w = np.zeros(n, np.float32); w[-1] = 0.75
    assert np.allclose(ovf.score_lstm(mod, w, xb), T * 0.75, rtol=0, atol=1e-6)
    # T = 1: one gated step from h = c = 0: v = w . (sig(o) * tanh(sig(i) * tanh(g))) + b
    w = I.lstm_weights(F, H, seed=2, bias_std=0.5)
    x1 = xb[:, :1]
    got = ovf.score_lstm(mod, w, x1).astype(np.float64)
    xs = (x1[:, 0].astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    Wih = w[:4 * H * F].reshape(4 * H, F).astype(np.float64)
    o = 4 * H * F + 4 * H * H
    b = (w[o:o + 4 * H] + w[o + 4 * H:o + 8 * H]).astype(np.float64)
    wh = w[o + 8 * H:o + 9 * H].astype(np.float64); bh = float(w[-1])
    z = xs @ Wih.T + b
    sig = lambda t: 1 / (1 + np.exp(-t))
    hh = sig(z[:, 3 * H:]) * np.tanh(sig(z[:, :H]) * np.tanh(z[:, 2 * H:3 * H]))
    assert np.allclose(got, hh @ wh + bh, rtol=0, atol=2e-6)
    # per-timestep head summed == head of the summed hidden states plus T * b (Sec. 3.2)
    w2 = w.copy(); w2[-1] = 0.0
    xT = xb
    v_b = ovf.score_lstm(mod, w, xT).astype(np.float64)
    v_0 = ovf.score_lstm(mod, w2, xT).astype(np.float64)
    assert np.allclose(v_b - v_0, T * bh, atol=1e-5)


def test_argmin_scan(ovf):
    inf, nan = np.inf, np.nan
    bi, bv = ovf.argmin([3, 1, 2, 1, 5])
    assert (bi[0], bv[0]) == (1, 1.0)                       # first of two equal minima
    bi, bv = ovf.argmin([nan, 4, nan, 4, 7])
    assert (bi[0], bv[0]) == (1, 4.0)                       # NaN never wins
    bi, bv = ovf.argmin([nan, inf, nan])
    assert bi[0] == -1 and bv[0] == inf                     # nothing is < +inf
    bi, bv = ovf.argmin([1, 2, 3], valid=[0, 0, 0])
    assert bi[0] == -1 and bv[0] == inf
    bi, bv = ovf.argmin([1, 2, 3, 0.5], valid=[0, 1, 1, 0])
    assert (bi[0], bv[0]) == (1, 2.0)
    bi, bv = ovf.argmin([-inf, 2, -inf])
    assert bi[0] == 0 and bv[0] == -inf
    bi, bv = ovf.argmin([0.0, -0.0])
    assert bi[0] == 0                                       # -0.0 < 0.0 is false
    bi, bv = ovf.argmin([5, 4, 9, 9, 1, 1, nan, nan], group=2)
    assert bi.tolist() == [1, 2, 4, -1] and bv[:3].tolist() == [4.0, 9.0, 1.0] and bv[3] == inf
    bi, bv = ovf.argmin([5, 4, 9, 0, 7], group=3)           # ragged last group, global ids
    assert bi.tolist() == [1, 3]
    bi, bv = ovf.argmin([])
    assert bi.tolist() == [-1] and bv[0] == inf
    rng = np.random.default_rng(0)
    s = rng.integers(0, 50, 4096).astype(np.float32)
    bi, bv = ovf.argmin(s, group=256)
    for g in range(16):
        blk = s[g * 256:(g + 1) * 256]
        assert bi[g] == g * 256 + int(np.argmin(blk)) and bv[g] == blk.min()   # numpy's argmin is also first-min
