"""Float64 / complex128 CPU oracle for the complex-gated LRU (test infrastructure).

Appendix B ("Complex-Gated Linear Recurrent Unit") of the Griffin/Hawk paper, written out in
plain numpy, one time step after the other, in the appendix's own order and notation. Shares
no code with the HIP library; only tests, the smoke check and the benchmark's cpu_baseline leg
may import it.

The layer (D real channels, H = D / 2 complex ones):
    x~_t  = x_t[:H] + i x_t[H:]                       first half real part, second half imaginary
    r_t   = sigmoid(W_a x_t + b_a)            in R^H  recurrence gate
    i_t   = sigmoid(W_x x_t + b_x)            in R^H  input gate
    a~    = sigmoid(Lambda) e^{i theta}               complex diagonal recurrence weight
    a~_t  = a~^{c r_t} = exp(c r_t (log sigmoid(Lambda) + i theta))
    h~_t  = a~_t h~_{t-1} + sqrt(1 - |a~_t|^2) (i_t x~_t)
    y_t   = [Re h~_t ; Im h~_t]               in R^D

Readings where the appendix is silent:
  * Gate weights. The gates have H outputs and see all D inputs. The real layer's gate
    matrices are block diagonal (Section 4.1), and the appendix does not say how that carries
    over; here block g (of nb) owns the complex channels g*hs .. (g+1)*hs-1 (hs = H / nb) and
    sees the real AND the imaginary part of exactly those channels:
        W[g] is [hs][2 hs], input k <  hs : channel g*hs + k           (real part)
                            input k >= hs : channel H + g*hs + (k-hs)  (imaginary part)
    nb = 1 is the appendix's dense H x D matrix (with its columns in the order of x_t).
  * The power a~^{c r_t} is taken on the principal branch of the parameterisation, i.e. as
    exp(c r_t log a~) with log a~ = log sigmoid(Lambda) + i theta (theta itself, not reduced).
  * States carried between calls are the stacked [Re h~ ; Im h~] in R^D, like y_t.
  * The temporal Conv1D in front (Section 2.3) is the real layer's, on all D channels.

Arrays: x, y, dy [B,T,D]; W_a, W_x [nb,hs,2hs]; b_a, b_x, Lambda, theta [H]; h0, hT [B,D].
"""
import numpy as np


def _sigmoid(z):
    return 0.5 * (1.0 + np.tanh(0.5 * z))


def _log_sigmoid(z):
    return -np.logaddexp(0.0, -z)


def _block_inputs(x, nb):
    """[B,T,D] -> [B,T,nb,2hs]: per gate block, its channels' real parts then imaginary parts."""
    B, T, D = x.shape
    H = D // 2
    hs = H // nb
    return np.concatenate([x[..., :H].reshape(B, T, nb, hs), x[..., H:].reshape(B, T, nb, hs)], axis=-1)


def cg_gates(x, W_a, W_x, b_a, b_x, Lambda, theta, c=8.0):
    """Gates and the complex decay for every step. Returns dict r, i [B,T,H] (real),
    a [B,T,H] (complex), m = sqrt(1 - |a|^2) [B,T,H] (real)."""
    x = np.asarray(x, np.float64)
    B, T, D = x.shape
    nb, hs, two_hs = W_a.shape
    H = D // 2
    assert D % 2 == 0 and nb * hs == H and two_hs == 2 * hs and W_x.shape == W_a.shape
    xin = _block_inputs(x, nb)
    p = np.einsum("gjk,btgk->btgj", np.asarray(W_a, np.float64), xin).reshape(B, T, H) + b_a
    q = np.einsum("gjk,btgk->btgj", np.asarray(W_x, np.float64), xin).reshape(B, T, H) + b_x
    r, i = _sigmoid(p), _sigmoid(q)
    log_mod = c * r * _log_sigmoid(np.asarray(Lambda, np.float64))     # log |a~_t| <= 0
    phase = c * r * np.asarray(theta, np.float64)
    a = np.exp(log_mod) * (np.cos(phase) + 1j * np.sin(phase))
    m = np.sqrt(-np.expm1(2.0 * log_mod))                               # sqrt(1 - |a~_t|^2)
    return dict(r=r, i=i, a=a, m=m, log_mod=log_mod, phase=phase)


def cg_lru(x, W_a, W_x, b_a, b_x, Lambda, theta, h0=None, c=8.0, want_gates=False):
    """The CG-LRU layer on (already convolved) x [B,T,D]. Returns y [B,T,D], hT [B,D]
    (and the gates)."""
    x = np.asarray(x, np.float64)
    B, T, D = x.shape
    H = D // 2
    g = cg_gates(x, W_a, W_x, b_a, b_x, Lambda, theta, c)
    xt = x[..., :H] + 1j * x[..., H:]
    h = np.zeros((B, H), np.complex128) if h0 is None else np.asarray(h0, np.float64)[:, :H] + 1j * np.asarray(h0, np.float64)[:, H:]
    y = np.empty((B, T, D))
    for t in range(T):
        h = g["a"][:, t] * h + g["m"][:, t] * (g["i"][:, t] * xt[:, t])
        y[:, t, :H] = h.real
        y[:, t, H:] = h.imag
    hT = np.concatenate([h.real, h.imag], axis=-1)
    return (y, hT, g) if want_gates else (y, hT)


def _conv1d(u, conv_w, conv_b, state_in):
    """Section 2.3's causal per-channel filter, lag-indexed taps [K,D]; state_in [B,K-1,D]
    chronological (oldest first) or None."""
    u = np.asarray(u, np.float64)
    B, T, D = u.shape
    K = conv_w.shape[0]
    hist = np.zeros((B, K - 1, D)) if state_in is None else np.asarray(state_in, np.float64)
    ext = np.concatenate([hist, u], axis=1)                 # ext[:, K-1+t] = u_t
    x = np.zeros((B, T, D)) if conv_b is None else np.broadcast_to(np.asarray(conv_b, np.float64), (B, T, D)).copy()
    for k in range(K):
        x += np.asarray(conv_w, np.float64)[k] * ext[:, K - 1 - k:K - 1 - k + T]
    return x, ext[:, T:T + K - 1].copy()


def cg_forward(u, W_a, W_x, b_a, b_x, Lambda, theta, conv_w=None, conv_b=None, h0=None,
               state_in=None, c=8.0):
    """Conv1D (skipped when conv_w is None) then the CG-LRU. Returns y, hT, state_out
    ([B,3,D] chronological; None without the Conv1D)."""
    if conv_w is None:
        y, hT = cg_lru(u, W_a, W_x, b_a, b_x, Lambda, theta, h0, c)
        return y, hT, None
    x, st = _conv1d(u, conv_w, conv_b, state_in)
    y, hT = cg_lru(x, W_a, W_x, b_a, b_x, Lambda, theta, h0, c)
    return y, hT, st


def cg_backward(u, W_a, W_x, b_a, b_x, Lambda, theta, dy, conv_w=None, conv_b=None, h0=None,
                state_in=None, dhT=None, c=8.0):
    """Adjoint of cg_forward for the real loss L = sum(dy * y) + sum(dhT * hT) (the appendix
    prints none; derived from its equations with the real and imaginary parts as independent
    real variables). Returns float64 grads: du, dh0, dW_a, dW_x, db_a, db_x, dLambda, dtheta
    and, with the Conv1D, dconv_w, dconv_b."""
    u = np.asarray(u, np.float64)
    dy = np.asarray(dy, np.float64)
    B, T, D = u.shape
    H = D // 2
    nb, hs, _ = W_a.shape
    W_a, W_x = np.asarray(W_a, np.float64), np.asarray(W_x, np.float64)
    Lambda, theta = np.asarray(Lambda, np.float64), np.asarray(theta, np.float64)
    if conv_w is None:
        x = u
    else:
        x, _ = _conv1d(u, conv_w, conv_b, state_in)
    y, _, g = cg_lru(x, W_a, W_x, b_a, b_x, Lambda, theta, h0, c, want_gates=True)
    xt = x[..., :H] + 1j * x[..., H:]
    hc = y[..., :H] + 1j * y[..., H:]
    h_init = np.zeros((B, H), np.complex128) if h0 is None else np.asarray(h0, np.float64)[:, :H] + 1j * np.asarray(h0, np.float64)[:, H:]
    # a complex number stands for the pair (d/dRe, d/dIm) throughout
    carry = np.zeros((B, H), np.complex128) if dhT is None else np.asarray(dhT, np.float64)[:, :H] + 1j * np.asarray(dhT, np.float64)[:, H:]
    dx = np.zeros((B, T, D))
    dp = np.zeros((B, T, H))
    dq = np.zeros((B, T, H))
    dLambda = np.zeros(H)
    dtheta = np.zeros(H)
    log_sig = _log_sigmoid(Lambda)
    for t in range(T - 1, -1, -1):
        a, m, r, i = g["a"][:, t], g["m"][:, t], g["r"][:, t], g["i"][:, t]
        delta = dy[:, t, :H] + 1j * dy[:, t, H:] + carry            # dL/dh~_t
        h_prev = hc[:, t - 1] if t > 0 else h_init
        # h~_t = a~_t h~_{t-1} + m_t i_t x~_t
        G = delta * np.conj(h_prev)                                  # (dL/dRe a~_t, dL/dIm a~_t)
        s = (delta.real * xt[:, t].real + delta.imag * xt[:, t].imag)   # dL/d(m_t i_t)
        d_m = s * i
        d_i = s * m
        d_xt = delta * (m * i)
        # a~_t = exp(log_mod + i phase): d a~/d log_mod = a~, d a~/d phase = i a~
        d_log_mod = (G.real * a.real + G.imag * a.imag)
        d_phase = (-G.real * a.imag + G.imag * a.real)
        # m_t = sqrt(1 - exp(2 log_mod)): d m/d log_mod = -|a~_t|^2 / m_t
        mod2 = np.exp(2.0 * g["log_mod"][:, t])
        d_log_mod = d_log_mod + np.where(m > 0, -d_m * mod2 / np.where(m > 0, m, 1.0), 0.0)
        # log_mod = c r log sigmoid(Lambda), phase = c r theta
        d_r = c * (d_log_mod * log_sig + d_phase * theta)
        dLambda += np.sum(d_log_mod * c * r * _sigmoid(-Lambda), axis=0)   # d log sigmoid = sigmoid(-Lambda)
        dtheta += np.sum(d_phase * c * r, axis=0)
        dp[:, t] = d_r * r * (1.0 - r)
        dq[:, t] = d_i * i * (1.0 - i)
        dx[:, t, :H] = d_xt.real
        dx[:, t, H:] = d_xt.imag
        carry = np.conj(a) * delta
    dh0 = np.concatenate([carry.real, carry.imag], axis=-1)
    # gate products: p = W_a xin + b_a, q = W_x xin + b_x per block
    xin = _block_inputs(x, nb)
    dpb, dqb = dp.reshape(B, T, nb, hs), dq.reshape(B, T, nb, hs)
    dW_a = np.einsum("btgj,btgk->gjk", dpb, xin)
    dW_x = np.einsum("btgj,btgk->gjk", dqb, xin)
    dxin = np.einsum("btgj,gjk->btgk", dpb, W_a) + np.einsum("btgj,gjk->btgk", dqb, W_x)
    dx[..., :H] += dxin[..., :hs].reshape(B, T, H)
    dx[..., H:] += dxin[..., hs:].reshape(B, T, H)
    out = dict(dh0=dh0, dW_a=dW_a, dW_x=dW_x, db_a=dp.sum(axis=(0, 1)), db_x=dq.sum(axis=(0, 1)),
               dLambda=dLambda, dtheta=dtheta)
    if conv_w is None:
        out["du"] = dx
        return out
    K = conv_w.shape[0]
    conv_w = np.asarray(conv_w, np.float64)
    hist = np.zeros((B, K - 1, D)) if state_in is None else np.asarray(state_in, np.float64)
    ext = np.concatenate([hist, u], axis=1)
    du = np.zeros((B, T, D))
    dconv_w = np.zeros((K, D))
    for k in range(K):
        du[:, :T - k] += conv_w[k] * dx[:, k:]
        dconv_w[k] = np.sum(dx * ext[:, K - 1 - k:K - 1 - k + T], axis=(0, 1))
    out["du"] = du
    out["dconv_w"] = dconv_w
    out["dconv_b"] = dx.sum(axis=(0, 1))
    return out


def cg_decode_step(u_t, W_a, W_x, b_a, b_x, Lambda, theta, h, state, conv_w=None, conv_b=None,
                   c=8.0):
    """One token per sequence; h [B,D] and state [B,3,D] (chronological; ignored without the
    Conv1D) are updated in place. Returns y_t [B,D]."""
    u_t = np.asarray(u_t, np.float64)
    if conv_w is None:
        y, hT = cg_lru(u_t[:, None, :], W_a, W_x, b_a, b_x, Lambda, theta, h, c)
    else:
        x, st = _conv1d(u_t[:, None, :], conv_w, conv_b, state)
        y, hT = cg_lru(x, W_a, W_x, b_a, b_x, Lambda, theta, h, c)
        state[...] = st
    h[...] = hT
    return y[:, 0]
