"""CPU ORACLE (test infrastructure, not part of the product path) -- a policy with carried
state: the LSTM sequence-to-sequence model of the paper's "Seq2Seq Learning" example.

Section 3 describes the task: the query is a string for the addition of two random integers,
padded with leading zeros to equal lengths ("012+345="), the answer is the string of the sum;
the policy is an LSTM-based sequence-to-sequence model.  Section 4 ("Exploring Novel Policy
Architectures") gives the interface: get_actions(t_states, params, p_states) with p_states
carrying, for example, the cells of an LSTM from one step to the next.  The paper prints no
architecture, so the following is this build's reading.

  Tokens: digits 0..9, '+' = 10, '=' = 11 (V = 12); the answer has digits 0..9 (n_out = 10).
  LSTM cell (the standard one; gates in the order i, f, g, o, each H wide):
      a = Wx[token] + h Wh + b            (a one-hot input selects a row of Wx)
      c' = sigmoid(a_f) c + sigmoid(a_i) tanh(a_g);     h' = sigmoid(a_o) tanh(c')
  Encoder: (h, c) = 0, one cell step per query token.  Decoder: its own cell, starts from the
  encoder's final (h, c) -- the carried policy state -- and takes one step per answer position j
  with input token '=' for j = 0 and the true answer digit j - 1 after that (teacher forcing);
  logits_j = h_j Wo + bo.
  Flat parameters: enc Wx[V][4H], enc Wh[H][4H], enc b[4H], dec Wx[V][4H], dec Wh[H][4H],
  dec b[4H], Wo[H][n_out], bo[n_out]   (column g H + u of a gate matrix is gate g of unit u).
  Fitness = -mean over samples and answer positions of the cross-entropy of the true digit.

fp64 arithmetic.  Pins: tests/test_oracle_seq2seq.py (torch.nn.LSTMCell / torch.nn.LSTM as
library twins, zero-weight and bias-only closed forms, the generator decoded back to integers).
"""
import numpy as np

V_TOKENS, N_DIGITS, TOK_PLUS, TOK_EQ = 12, 10, 10, 11


def param_count(H, V=V_TOKENS, n_out=N_DIGITS):
    return 2 * (V * 4 * H + H * 4 * H + 4 * H) + H * n_out + n_out


def unpack(theta, H, V=V_TOKENS, n_out=N_DIGITS):
    """Views (enc, dec, Wo, bo) of one flat parameter vector; enc and dec are (Wx, Wh, b)."""
    o = 0
    cells = []
    for _ in range(2):
        Wx = theta[o:o + V * 4 * H].reshape(V, 4 * H)
        o += V * 4 * H
        Wh = theta[o:o + H * 4 * H].reshape(H, 4 * H)
        o += H * 4 * H
        b = theta[o:o + 4 * H]
        o += 4 * H
        cells.append((Wx, Wh, b))
    Wo = theta[o:o + H * n_out].reshape(H, n_out)
    o += H * n_out
    bo = theta[o:o + n_out]
    o += n_out
    if o != theta.shape[0]:
        raise ValueError("parameter vector has %d entries, layout needs %d" % (theta.shape[0], o))
    return cells[0], cells[1], Wo, bo


def _sigmoid(x):
    return 1.0 / (1.0 + np.exp(-x))


def lstm_cell(tokens, h, c, Wx, Wh, b):
    """One step for a batch: tokens[B] int, h[B,H], c[B,H] -> (h', c')."""
    H = h.shape[1]
    a = Wx[tokens] + h @ Wh + b
    i, f, g, o = (a[:, k * H:(k + 1) * H] for k in range(4))
    c_new = _sigmoid(f) * c + _sigmoid(i) * np.tanh(g)
    return _sigmoid(o) * np.tanh(c_new), c_new


def forward(params, query, answer, H, V=V_TOKENS, n_out=N_DIGITS, return_state=False):
    """params[pop,P]; query[B,Lq], answer[B,La] int tokens shared by all members.
    Returns logits[pop,B,La,n_out] fp64 (and the encoder's final (h, c) per member if asked)."""
    params = np.asarray(params, dtype=np.float64)
    query = np.asarray(query, dtype=np.int64)
    answer = np.asarray(answer, dtype=np.int64)
    pop, (B, Lq), La = params.shape[0], query.shape, answer.shape[1]
    logits = np.empty((pop, B, La, n_out))
    states = []
    for m in range(pop):
        enc, dec, Wo, bo = unpack(params[m], H, V, n_out)
        h = np.zeros((B, H))
        c = np.zeros((B, H))
        for t in range(Lq):
            h, c = lstm_cell(query[:, t], h, c, *enc)
        states.append((h.copy(), c.copy()))
        for j in range(La):
            tok = np.full(B, TOK_EQ, dtype=np.int64) if j == 0 else answer[:, j - 1]
            h, c = lstm_cell(tok, h, c, *dec)
            logits[m, :, j, :] = h @ Wo + bo
    return (logits, states) if return_state else logits


def fitness(logits, answer):
    """-mean cross-entropy of the true digits: logits[pop,B,La,n_out], answer[B,La] -> [pop]."""
    z = np.asarray(logits, dtype=np.float64)
    zmax = z.max(axis=-1, keepdims=True)
    lse = zmax[..., 0] + np.log(np.exp(z - zmax).sum(axis=-1))
    picked = np.take_along_axis(z, np.asarray(answer, dtype=np.int64)[None, :, :, None], axis=-1)[..., 0]
    return -(lse - picked).mean(axis=(-2, -1))


def accuracy(logits, answer):
    """Fraction of samples whose every answer digit is the arg-max of its logits: [pop]."""
    hit = (np.asarray(logits).argmax(axis=-1) == np.asarray(answer)[None, :, :]).all(axis=-1)
    return hit.mean(axis=-1)
