"""Pins of the LSTM sequence-to-sequence oracle: library twins (torch.nn.LSTMCell, torch.nn.LSTM
with an explicit one-hot input), closed forms with zero or bias-only weights, and the task
generator decoded back to integers."""
import numpy as np
import pytest
import torch

from oracle import seq2seq as s2s, generation as ogen
from workloads import generators as gen


def _random_theta(seed, H, scale=0.3):
    return np.random.default_rng(seed).standard_normal(s2s.param_count(H)) * scale


def test_param_count_and_layout():
    H = 128
    assert s2s.param_count(H) == 2 * (12 * 512 + 128 * 512 + 512) + 1280 + 10 == 145674
    th = np.arange(s2s.param_count(8), dtype=np.float64)
    (ex, eh, eb), (dx, dh, db), Wo, bo = s2s.unpack(th, 8)
    assert ex[0, 0] == 0 and ex[1, 0] == 32 and eh[0, 0] == 12 * 32 and eb[0] == 12 * 32 + 8 * 32
    assert dx[0, 0] == eb[-1] + 1 and Wo[0, 0] == db[-1] + 1 and bo[-1] == th[-1]
    with pytest.raises(ValueError):
        s2s.unpack(th[:-1], 8)


def test_cell_against_torch_lstmcell():
    """torch's cell uses the same gate order (i, f, g, o); its input is the explicit one-hot row."""
    H, B = 16, 9
    rng = np.random.default_rng(3)
    Wx, Wh, b = rng.standard_normal((12, 4 * H)), rng.standard_normal((H, 4 * H)) * 0.5, rng.standard_normal(4 * H)
    h, c = rng.standard_normal((B, H)) * 0.5, rng.standard_normal((B, H))
    tok = rng.integers(0, 12, B)
    cell = torch.nn.LSTMCell(12, H).double()
    with torch.no_grad():
        cell.weight_ih.copy_(torch.tensor(Wx.T))
        cell.weight_hh.copy_(torch.tensor(Wh.T))
        cell.bias_ih.copy_(torch.tensor(b))
        cell.bias_hh.zero_()
        th, tc = cell(torch.nn.functional.one_hot(torch.tensor(tok), 12).double(), (torch.tensor(h), torch.tensor(c)))
    oh, oc = s2s.lstm_cell(tok, h, c, Wx, Wh, b)
    np.testing.assert_allclose(oh, th.numpy(), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(oc, tc.numpy(), rtol=1e-12, atol=1e-14)


def test_encoder_decoder_against_torch_lstm():
    H, B = 8, 7
    theta = _random_theta(4, H, 0.5)
    query, answer = gen.addition_batch(11, 1, B, 3)
    logits, states = s2s.forward(theta[None, :], query, answer, H, return_state=True)
    (ex, eh, eb), (dx, dh, db), Wo, bo = s2s.unpack(theta, H)

    def lstm(Wx, Wh, b):
        net = torch.nn.LSTM(12, H, batch_first=True).double()
        with torch.no_grad():
            net.weight_ih_l0.copy_(torch.tensor(Wx.T))
            net.weight_hh_l0.copy_(torch.tensor(Wh.T))
            net.bias_ih_l0.copy_(torch.tensor(b))
            net.bias_hh_l0.zero_()
        return net

    one_hot = lambda t: torch.nn.functional.one_hot(torch.tensor(np.asarray(t, dtype=np.int64)), 12).double()
    with torch.no_grad():
        _, (h, c) = lstm(ex, eh, eb)(one_hot(query))
        np.testing.assert_allclose(states[0][0], h[0].numpy(), rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(states[0][1], c[0].numpy(), rtol=1e-11, atol=1e-13)
        dec_in = np.concatenate([np.full((B, 1), s2s.TOK_EQ), answer[:, :-1]], axis=1)
        out, _ = lstm(dx, dh, db)(one_hot(dec_in), (h, c))
        want = out.numpy() @ Wo + bo
    np.testing.assert_allclose(logits[0], want, rtol=1e-10, atol=1e-12)
    ce = torch.nn.functional.cross_entropy(torch.tensor(want).reshape(-1, 10), torch.tensor(answer, dtype=torch.int64).reshape(-1))
    np.testing.assert_allclose(s2s.fitness(logits, answer)[0], -ce.item(), rtol=1e-12)


def test_closed_forms():
    H, B = 4, 5
    query, answer = gen.addition_batch(12, 1, B, 3)
    P = s2s.param_count(H)
    # all weights zero: gates are 0, c stays 0, h stays 0, logits = bo = 0 -> CE = ln 10, accuracy from ties = digit 0
    z = s2s.forward(np.zeros((1, P)), query, answer, H)
    assert np.all(z == 0.0)
    np.testing.assert_allclose(s2s.fitness(z, answer), -np.log(10.0), rtol=1e-14)
    # biases only: c_t = s(bf) c_{t-1} + s(bi) tanh(bg) is a geometric series, the same for every sample
    theta = np.zeros(P)
    (ex, eh, eb), (dx, dh, db), Wo, bo = s2s.unpack(theta, H)
    bi, bf, bg, bo_gate = 0.3, -0.2, 0.7, 0.1
    for b in (eb, db):
        b[0:H], b[H:2 * H], b[2 * H:3 * H], b[3 * H:] = bi, bf, bg, bo_gate
    Wo[:, 3] = 1.0
    s = lambda x: 1.0 / (1.0 + np.exp(-x))
    steps = query.shape[1] + answer.shape[1]
    r, inc = s(bf), s(bi) * np.tanh(bg)
    z = s2s.forward(theta[None, :], query, answer, H)
    for j in range(answer.shape[1]):
        n = query.shape[1] + j + 1
        c = inc * (1.0 - r ** n) / (1.0 - r)
        np.testing.assert_allclose(z[0, :, j, 3], H * s(bo_gate) * np.tanh(c), rtol=1e-12)
        assert np.all(z[0, :, j, [0, 1, 2, 4]] == 0.0)
    assert steps == 12
    # a sample's logits do not depend on the other samples of the batch; members are independent
    th2 = np.stack([_random_theta(5, H), _random_theta(6, H)])
    full = s2s.forward(th2, query, answer, H)
    one = s2s.forward(th2[1:], query[2:3], answer[2:3], H)
    np.testing.assert_allclose(full[1, 2], one[0, 0], rtol=1e-13)
    # accuracy: logits that put the true digit on top everywhere score 1, one wrong digit loses the sample
    good = np.zeros((1, B, 4, 10))
    np.put_along_axis(good, answer[None, :, :, None], 5.0, axis=-1)
    assert s2s.accuracy(good, answer)[0] == 1.0
    good[0, 0, 2, (answer[0, 2] + 1) % 10] = 9.0
    assert s2s.accuracy(good, answer)[0] == (B - 1) / B


def test_teacher_forcing_uses_the_previous_true_digit():
    H, B = 6, 4
    theta = _random_theta(7, H, 0.8)
    query, answer = gen.addition_batch(13, 2, B, 3)
    base = s2s.forward(theta[None], query, answer, H)
    changed = answer.copy()
    changed[:, 1] = (changed[:, 1] + 3) % 10          # digit 1 is the decoder's input at position 2
    z = s2s.forward(theta[None], query, changed, H)
    assert np.array_equal(z[:, :, :2], base[:, :, :2]) and not np.allclose(z[:, :, 2], base[:, :, 2])
    changed = answer.copy()
    changed[:, -1] = (changed[:, -1] + 1) % 10        # the last digit is never an input
    assert np.array_equal(s2s.forward(theta[None], query, changed, H), base)


def test_addition_generator_decodes_to_a_correct_sum():
    for digits in (1, 3, 5):
        q, a = gen.addition_batch(14, 3, 500, digits)
        assert q.shape == (500, 2 * digits + 2) and a.shape == (500, digits + 1)
        assert q.dtype == np.int32 and (q[:, digits] == 10).all() and (q[:, -1] == 11).all()
        val = lambda d: (d * 10 ** np.arange(d.shape[1] - 1, -1, -1)).sum(1)
        x, y = val(q[:, :digits]), val(q[:, digits + 1:-1])
        assert (val(a) == x + y).all() and a.max() <= 9 and a.min() >= 0
        assert len(np.unique(x)) > min(8, 10 ** digits - 2)
    q2, _ = gen.addition_batch(14, 4, 500, 3)
    assert not np.array_equal(q, q2[:, :0]) and not np.array_equal(gen.addition_batch(14, 3, 500, 3)[0], q2)


def test_generation_runs_the_seq2seq_task():
    from oracle import pgpe
    H = 4
    P = s2s.param_count(H)
    q, a = gen.addition_batch(15, 1, 6, 2)
    st = pgpe.PGPEState.create(pgpe.PGPEConfig(P=P, pop_max=8))
    params, fit = ogen.run_generation(st, {"kind": "seq2seq", "H": H, "query": q, "answer": a}, 3, 8)
    assert fit.shape == (8,) and np.isfinite(fit).all() and st.t == 2
    np.testing.assert_allclose(fit, s2s.fitness(s2s.forward(params, q, a, H), a), rtol=1e-6)
