"""Plain CPU oracle of the per-worker compression step of variance-based gradient
compression (Tsuzuku, Imachi, Akiba, arXiv 1802.06058).

TEST INFRASTRUCTURE ONLY.  It is slow and obviously correct on purpose, shares no
code with the HIP path, and is imported only by the tests, the smoke check and the
benchmark's CPU-baseline leg.

What is implemented, in the paper's order and notation:

  sqgrad_*            the two per-parameter sums of Alg. 1,
                      g_i = sum_z (grad_i f_z / B) and s_i = sum_z (grad_i f_z / B)^2,
                      from the definition of a per-sample gradient (Section 4.1).
                      float64 throughout.  sqgrad_conv_nhwc*: the same for a convolution
                      given by its input and output-gradient tensors (no im2col matrix).
  accumulate_select   the body of the `foreach parameters` loop of Alg. 1 with the
                      criterion of Eq. 2 and the decay of Section 4.4; float32, one
                      rounding per operation.
  quantise_prose      Section 4.2 read literally in real arithmetic.
  quantise_bits       the integer recipe of Section 4.4 (truncate the mantissa; round
                      by adding one at the mantissa's top bit).
  pack                Encode() of Alg. 1: per weight-matrix group, floor(log2 M_k),
                      4-bit value code and 28-bit index in one 32-bit word (Section 4.2).
  unpack_add          the decode-and-sum half of CommunicateAndUpdate() (Section 4.3).
  momentum_sgd_step,  the parameter update that follows it (Sections 4.1, 4.3), with the
  adam_step,          elements nobody sent entering as zero; unpack_apply = decode + one step.
  unpack_apply
  pack_compact,       the compressed index encoding Section 4.2's last paragraph names without an algorithm
  unpack_compact      (this build's own format: gap to the previous element, one or two bytes per element).

Readings taken where the paper is silent are stated at the function that needs them.
Every function here is pinned by tests that do not go through this module's own
arithmetic (hand-computed values, the worked example of Appendix B, the identity of
Appendix A, closed forms and brute force); no part is "parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np

F32 = np.float32
U32 = np.uint32

INDEX_BITS = 28                      # Section 4.2: "the rest 28-bits" hold the index
INDEX_MASK = (1 << INDEX_BITS) - 1
MAX_GROUP = 1 << INDEX_BITS
D_MAX = 7                            # Section 4.2: three exponent bits, d in 0..7


# --------------------------------------------------------------------------------------
# (a) per-parameter sums over the mini-batch  (Alg. 1, first two lines of the loop body)
# --------------------------------------------------------------------------------------

def sqgrad_bruteforce_fc(X, D, c):
    """Materialise every per-sample gradient of a fully-connected weight and sum.

    For sample z the gradient of its loss w.r.t. W[i, j] is x_z[i] * delta_z[j]
    (Section 4.1 defines grad_i f_z as the gradient of sample z's loss).  `c` is the
    1/B of Alg. 1 (or 1 if delta already carries it).  Pure loops, float64; tiny
    inputs only.
    """
    X = np.asarray(X, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64)
    B, J = X.shape
    _, C = D.shape
    g = np.zeros((J, C))
    s = np.zeros((J, C))
    for z in range(B):
        for i in range(J):
            for j in range(C):
                grad = c * X[z, i] * D[z, j]
                g[i, j] += grad
                s[i, j] += grad * grad
    return g, s


def sqgrad_bruteforce_conv(U, D, c):
    """Same for a weight shared over P positions (a convolution seen through im2col).

    Sample z's gradient w.r.t. W[j, k] is sum_p U[z, p, j] * D[z, p, k]; the square is
    taken of that per-sample gradient, i.e. after the sum over positions
    (Section 4.1: the variance is over the samples z of the mini-batch).
    """
    U = np.asarray(U, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64)
    B, P, J = U.shape
    C = D.shape[2]
    g = np.zeros((J, C))
    s = np.zeros((J, C))
    for z in range(B):
        for j in range(J):
            for k in range(C):
                grad = 0.0
                for p in range(P):
                    grad += U[z, p, j] * D[z, p, k]
                grad *= c
                g[j, k] += grad
                s[j, k] += grad * grad
    return g, s


def sqgrad_fc(X, D, c):
    """FC layer at config sizes: the per-sample gradient is an outer product, so
    s = c^2 (X.X)^T (D.D) and g = c X^T D exactly.  Cost 2*N*B multiply-adds per
    output array, the count Section 5 gives for the statistic.  float64."""
    X = np.asarray(X, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64)
    g = (X.T @ D) * c
    s = ((X * X).T @ (D * D)) * (c * c)
    return g, s


def sqgrad_conv(U, D, c):
    """Shared-weight layer at config sizes: one per-sample gradient matrix at a time
    (G_z = U_z^T D_z), accumulated and square-accumulated.  float64."""
    U = np.asarray(U)
    D = np.asarray(D)
    B, P, J = U.shape
    C = D.shape[2]
    g = np.zeros((J, C))
    s = np.zeros((J, C))
    for z in range(B):
        G = (U[z].astype(np.float64).T @ D[z].astype(np.float64)) * c
        g += G
        s += G * G
    return g, s


def conv_out_size(n_in, k, stride, pad):
    """Output extent of a convolution along one axis (no dilation)."""
    return (n_in + 2 * pad - k) // stride + 1


def sqgrad_conv_nhwc_bruteforce(act, D, kh, kw, stride, pad, c):
    """The same sums for a 2-d convolution given as it is stored, without an im2col matrix.

    act [B, H, W, Cin] is the layer's input, D [B, Ho, Wo, Cout] the gradient of each sample's loss
    w.r.t. the layer's output.  Sample z's gradient w.r.t. the weight W[ky, kx, i, o] is
        sum_{y, x} act[z, y*stride + ky - pad, x*stride + kx - pad, i] * D[z, y, x, o]
    with positions outside the input contributing zero (zero padding).  The result is indexed
    [(ky*kw + kx)*Cin + i, o].  Pure loops, float64; tiny inputs only.
    """
    act = np.asarray(act, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64)
    B, H, W, Cin = act.shape
    _, Ho, Wo, Cout = D.shape
    sh, sw = stride
    ph, pw = pad
    assert Ho == conv_out_size(H, kh, sh, ph) and Wo == conv_out_size(W, kw, sw, pw)
    g = np.zeros((kh * kw * Cin, Cout))
    s = np.zeros((kh * kw * Cin, Cout))
    for z in range(B):
        for ky in range(kh):
            for kx in range(kw):
                for i in range(Cin):
                    for o in range(Cout):
                        grad = 0.0
                        for y in range(Ho):
                            iy = y * sh + ky - ph
                            if iy < 0 or iy >= H:
                                continue
                            for x in range(Wo):
                                ix = x * sw + kx - pw
                                if ix < 0 or ix >= W:
                                    continue
                                grad += act[z, iy, ix, i] * D[z, y, x, o]
                        grad *= c
                        g[(ky * kw + kx) * Cin + i, o] += grad
                        s[(ky * kw + kx) * Cin + i, o] += grad * grad
    return g, s


def sqgrad_conv_nhwc(act, D, kh, kw, stride, pad, c):
    """Convolution at config sizes: per sample and per filter tap (ky, kx) the gradient block
    G_z[ky, kx] = A^T D_z, A the input window that tap sees (a strided slice of the zero-padded
    input), accumulated and square-accumulated over the samples.  float64."""
    act = np.asarray(act)
    D = np.asarray(D)
    B, H, W, Cin = act.shape
    _, Ho, Wo, Cout = D.shape
    sh, sw = stride
    ph, pw = pad
    assert Ho == conv_out_size(H, kh, sh, ph) and Wo == conv_out_size(W, kw, sw, pw)
    g = np.zeros((kh * kw * Cin, Cout))
    s = np.zeros((kh * kw * Cin, Cout))
    for z in range(B):
        a = np.zeros((H + 2 * ph, W + 2 * pw, Cin))
        a[ph:ph + H, pw:pw + W] = act[z].astype(np.float64)
        d = D[z].astype(np.float64).reshape(Ho * Wo, Cout)
        for ky in range(kh):
            for kx in range(kw):
                win = a[ky:ky + sh * (Ho - 1) + 1:sh, kx:kx + sw * (Wo - 1) + 1:sw]     # [Ho, Wo, Cin]
                G = (win.reshape(Ho * Wo, Cin).T @ d) * c
                j0 = (ky * kw + kx) * Cin
                g[j0:j0 + Cin] += G
                s[j0:j0 + Cin] += G * G
    return g, s


# --------------------------------------------------------------------------------------
# (b) accumulate, test, reset or decay  (Alg. 1 loop body, Eq. 2, Section 4.4)
# --------------------------------------------------------------------------------------

def accumulate_select(g, s, r, v, alpha, zeta):
    """One step of Alg. 1 for every parameter.

    float32 state, every operation rounded once, no fused multiply-add; alpha and zeta
    are rounded to float32 first.  The comparison is strict as printed in Eq. 2 and
    Alg. 1: equality is not sent.

    Returns (r_acc, r_out, v_out, send): r_acc is the accumulated value handed to
    Encode() (before the reset), r_out / v_out the state after the step.
    """
    g = np.asarray(g, dtype=F32)
    s = np.asarray(s, dtype=F32)
    r = np.asarray(r, dtype=F32)
    v = np.asarray(v, dtype=F32)
    a32 = F32(alpha)
    z32 = F32(zeta)
    r_acc = r + g                     # r_i += sum grad/B
    v_acc = v + s                     # v_i += sum (grad/B)^2
    lhs = r_acc * r_acc               # r_i^2
    rhs = a32 * v_acc                 # alpha v_i
    send = lhs > rhs
    zero = F32(0.0)
    v_out = np.where(send, zero, z32 * v_acc).astype(F32)   # reset, else v_i *= zeta
    r_out = np.where(send, zero, r_acc).astype(F32)         # reset, else keep
    assert r_acc.dtype == F32 and v_out.dtype == F32 and lhs.dtype == F32 and rhs.dtype == F32
    return r_acc, r_out, v_out, send


# --------------------------------------------------------------------------------------
# (c) quantise and encode  (Section 4.2, Section 4.4, Appendix B)
# --------------------------------------------------------------------------------------

def floor_log2(a):
    """floor(log2 a) for a positive finite float, exactly (math.frexp, no logarithm)."""
    m, ex = math.frexp(float(a))      # a = m * 2**ex with 0.5 <= m < 1
    return ex - 1


def quantise_prose(a, E):
    """Section 4.2 literally, in exact real arithmetic (float64 holds every float32 and
    every 1.5 * 2**e exactly).

    a : positive magnitudes of the elements to send (any float array);  E : floor(log2 M_k).
    Returns (lq, keep): lq = log2 of the preprocessed magnitude g'_i, keep = (d_i <= 7)
    with d_i = E - lq, and additionally g'_i must be a normal float32 power of two
    (lq >= -126) so that the receiver can rebuild it from an exponent field.

    Readings: "round to the closer value" is the linear midpoint 1.5 * 2**e and a tie
    goes up, which is what the integer recipe of Section 4.4 does.
    """
    a = np.asarray(a, dtype=np.float64)
    _, ex = np.frexp(a)
    e = ex.astype(np.int64) - 1                       # floor(log2 a)
    lower = np.ldexp(1.0, e)
    lq = np.where(a >= 1.5 * lower, e + 1, e)         # closer of 2**floor, 2**ceil
    lq = np.where(a > math.ldexp(1.0, E), E, lq)      # larger than 2**E: truncate to it
    d = E - lq
    keep = (d <= D_MAX) & (lq >= -126)
    return lq, keep


def quantise_bits(abs_bits, exp_field):
    """The integer recipe of Section 4.4 on the float32 bit pattern with the sign cleared.

    Adding one at the mantissa's top bit carries into the exponent exactly when the
    mantissa is at least one half; dropping the mantissa then leaves the rounded
    power of two.  `exp_field` is the biased exponent field of M_k, i.e. its mantissa
    truncated.  Returns (e_field, d, keep): the biased exponent of g'_i, the 3-bit
    code, and whether the element is encoded at all (d <= 7 and a non-zero exponent
    field; a zero field cannot be decoded as a power of two).
    """
    abs_bits = np.asarray(abs_bits, dtype=np.uint64)
    rounded = (abs_bits + np.uint64(0x00400000)) >> np.uint64(23)
    e_field = np.minimum(rounded, np.uint64(exp_field)).astype(np.int64)
    d = np.int64(exp_field) - e_field
    keep = (d <= D_MAX) & (e_field >= 1)
    return e_field, d, keep


def pack(r_acc, send, groups, max_over="sent", check=True):
    """Encode() of Alg. 1 for a whole model.

    r_acc  : float32 accumulated values (before the reset), length N
    send   : boolean mask of Alg. 1's test
    groups : list of (offset, size) tiling [0, N); one group per weight matrix / tensor
             (Section 4.2), size <= 2**28.

    Per group k: M_k = largest magnitude among the elements being sent (Section 4.2
    opens "after deciding which gradient elements to send"; `max_over="all"` takes the
    other reading, the whole group).  Header = (biased exponent field of M_k, count,
    offset of the group's first word).  An empty group has header (0, 0, offset).
    Word = sign << 31 | d << 28 | index, index local to the group and 0-based, words in
    ascending index order.  Elements with d > 7 are rounded to zero: no word.

    Returns (words uint32[], headers list[(exp_field, count, word_offset)],
             encoded bool[N]  -- True where a word was written).
    """
    r_acc = np.asarray(r_acc, dtype=F32)
    send = np.asarray(send, dtype=bool)
    bits = r_acc.view(U32)
    abs_bits = bits & U32(0x7FFFFFFF)
    words = []
    headers = []
    encoded = np.zeros(r_acc.shape[0], dtype=bool)
    word_offset = 0
    for (off, size) in groups:
        assert 0 < size <= MAX_GROUP
        sl = slice(off, off + size)
        idx = np.flatnonzero(send[sl])                 # ascending local indices
        if idx.size == 0:
            headers.append((0, 0, word_offset))
            continue
        ab = abs_bits[sl][idx]
        if max_over == "sent":
            m_bits = int(ab.max())                     # monotone in |x| for finite floats
        elif max_over == "all":
            m_bits = int(abs_bits[sl].max())
        else:
            raise ValueError(max_over)
        exp_field = m_bits >> 23                       # truncate the mantissa
        e_field, d, keep = quantise_bits(ab, exp_field)
        if check and exp_field >= 1:
            # the prose of Section 4.2 must give the same answer for normal magnitudes
            a = np.abs(r_acc[sl][idx].astype(np.float64))
            normal = ab >= (1 << 23)
            lq, keep_p = quantise_prose(a[normal], exp_field - 127)
            assert np.array_equal(lq + 127, e_field[normal])
            assert np.array_equal(keep_p, keep[normal])
        sign = (bits[sl][idx] >> U32(31)).astype(np.uint64)
        w = (sign << np.uint64(31)) | (d.astype(np.uint64) << np.uint64(28)) | idx.astype(np.uint64)
        w = w[keep].astype(U32)
        encoded[off + idx[keep]] = True
        count = int(w.size)
        headers.append((exp_field if count else 0, count, word_offset))
        words.append(w)
        word_offset += count
    words = np.concatenate(words) if words else np.zeros(0, dtype=U32)
    return words, headers, encoded


# --------------------------------------------------------------------------------------
# (d) decode and sum  (Section 4.3; CommunicateAndUpdate() of Alg. 1)
# --------------------------------------------------------------------------------------

def decode_words(words, exp_field):
    """Split words into (local index, float32 value).  The value is the power of two
    whose biased exponent is exp_field - d, with the word's sign bit."""
    words = np.asarray(words, dtype=U32)
    idx = (words & U32(INDEX_MASK)).astype(np.int64)
    d = (words >> U32(28)) & U32(7)
    sign = words & U32(0x80000000)
    vbits = ((U32(exp_field) - d) << U32(23)) | sign
    return idx, vbits.astype(U32).view(F32)


def unpack_add(words, headers, groups, scale, out):
    """Add one worker's message into the dense float32 buffer `out`, in place.

    out[base_k + idx] = fl32(out[...] + fl32(scale * value)); indices inside one message
    are distinct, and several messages are applied by calling this once per message in
    worker order, which fixes the order of the float32 additions (Section 4.3 sums the
    workers' contributions; `scale` = 1/p gives the mean it also mentions).
    """
    assert out.dtype == F32
    sc = F32(scale)
    for (off, size), (exp_field, count, word_offset) in zip(groups, headers):
        if count == 0:
            continue
        idx, val = decode_words(words[word_offset:word_offset + count], exp_field)
        assert idx.max() < size
        contrib = (sc * val).astype(F32)
        out[off + idx] = out[off + idx] + contrib
    return out


# --------------------------------------------------------------------------------------
# Hybrid algorithm (Alg. 2, Section 4.5): variance criterion combined with Strom's threshold
# --------------------------------------------------------------------------------------

def accumulate_select_hybrid(g, s, r, v, alpha, zeta, tau, abs_r="before"):
    """One step of Alg. 2 for every parameter, float32, one rounding per operation.

        r += g;  v += s
        if |r| > tau and r^2 > alpha v:   send Sign(r);  r -= Sign(r) tau;  v = max(v - 2|r|tau + tau^2, 0)
        v *= zeta                                        (always, unlike Alg. 1)

    The correction of v is Section 4.5's "modify a^2 to (a - b)^2" with b = S = +-tau the value sent and
    a the accumulated gradient, so |r| in it is the value BEFORE tau is subtracted (abs_r="before");
    Alg. 2 as printed updates r first, which would use the value after (abs_r="after").  The expression
    is evaluated left to right: ((v - (2|r|) tau) + tau*tau).

    Returns (r_out, v_out, send, sign) with sign = +1 / -1 where sent, 0 elsewhere.
    """
    g = np.asarray(g, dtype=F32)
    s = np.asarray(s, dtype=F32)
    r = np.asarray(r, dtype=F32)
    v = np.asarray(v, dtype=F32)
    a32, z32, t32 = F32(alpha), F32(zeta), F32(tau)
    r_acc = r + g
    v_acc = v + s
    send = (np.abs(r_acc) > t32) & ((r_acc * r_acc) > (a32 * v_acc))
    sgn = np.where(r_acc < 0, F32(-1), F32(1)).astype(F32)
    r_sent = (r_acc - sgn * t32).astype(F32)
    absr = np.abs(r_acc) if abs_r == "before" else np.abs(r_sent)
    if abs_r not in ("before", "after"):
        raise ValueError(abs_r)
    two_r_tau = ((F32(2) * absr) * t32).astype(F32)
    v_sent = np.maximum(((v_acc - two_r_tau) + (t32 * t32)).astype(F32), F32(0))
    r_out = np.where(send, r_sent, r_acc).astype(F32)
    v_out = (z32 * np.where(send, v_sent, v_acc)).astype(F32)
    sign = np.where(send, sgn, F32(0)).astype(F32)
    return r_out, v_out, send, sign


def pack_hybrid(sign, send, groups):
    """Encode(Sign(r)) of Alg. 2 in the word format of Section 4.2: one word per sent element with the
    sign bit and the group-local index, exponent code d = 0.  The header's exponent field is 127
    (2^0 = 1): a message is in units of tau, and the receiver decodes with scale = tau (times 1/p for
    the mean), so the decoder of the basic algorithm serves unchanged."""
    sign = np.asarray(sign, dtype=F32)
    send = np.asarray(send, dtype=bool)
    words, headers, word_offset = [], [], 0
    for (off, size) in groups:
        idx = np.flatnonzero(send[off:off + size])
        if idx.size == 0:
            headers.append((0, 0, word_offset))
            continue
        neg = (sign[off:off + size][idx] < 0).astype(np.uint64)
        words.append(((neg << np.uint64(31)) | idx.astype(np.uint64)).astype(U32))
        headers.append((127, int(idx.size), word_offset))
        word_offset += int(idx.size)
    words = np.concatenate(words) if words else np.zeros(0, dtype=U32)
    return words, headers


# --------------------------------------------------------------------------------------
# Parameter update after the exchange (Sections 4.1 and 4.3): the decoded, summed gradient
# feeds the optimizer directly; an element no worker sent enters as zero
# --------------------------------------------------------------------------------------

def momentum_sgd_step(ghat, w, m, lr, mu):
    """One Momentum SGD step on the decoded gradient `ghat` (Section 4.1: elements not sent are
    taken to be zero, i.e. ghat holds 0 there and the momentum simply decays).

    The paper names the optimizer but prints no formula.  Reading taken: the classical form
        m <- mu m - lr ghat;   w <- w + m
    in float32, one rounding per operation: t1 = mu*m, t2 = lr*ghat, m = t1 - t2, w = w + m.
    Returns (w, m).
    """
    assert ghat.dtype == F32 and w.dtype == F32 and m.dtype == F32
    lr32, mu32 = F32(lr), F32(mu)
    t1 = (mu32 * m).astype(F32)
    t2 = (lr32 * ghat).astype(F32)
    m_new = (t1 - t2).astype(F32)
    w_new = (w + m_new).astype(F32)
    return w_new, m_new


def adam_step(ghat, w, m, v, lr, beta1, beta2, eps, t):
    """One Adam step (the method Section 4.3 says is computed locally after the exchange; the
    experiments use its default hyperparameters), step count t >= 1, on the decoded gradient:
        m <- b1 m + (1 - b1) ghat;  v <- b2 v + (1 - b2) ghat^2
        w <- w - lr (m / (1 - b1^t)) / (sqrt(v / (1 - b2^t)) + eps)
    float32, one rounding per operation, in exactly this order; 1 - b1, 1 - b2, 1 - b1^t and
    1 - b2^t are formed in float64 and rounded to float32 once.  Returns (w, m, v).
    """
    assert ghat.dtype == F32 and w.dtype == F32 and m.dtype == F32 and v.dtype == F32 and t >= 1
    b1, b2 = F32(beta1), F32(beta2)
    omb1, omb2 = F32(1.0 - float(b1)), F32(1.0 - float(b2))
    bias1, bias2 = F32(1.0 - float(b1) ** t), F32(1.0 - float(b2) ** t)
    m_new = ((b1 * m).astype(F32) + (omb1 * ghat).astype(F32)).astype(F32)
    g2 = (ghat * ghat).astype(F32)
    v_new = ((b2 * v).astype(F32) + (omb2 * g2).astype(F32)).astype(F32)
    mhat = (m_new / bias1).astype(F32)
    vhat = (v_new / bias2).astype(F32)
    denom = (np.sqrt(vhat).astype(F32) + F32(eps)).astype(F32)
    step = ((F32(lr) * mhat).astype(F32) / denom).astype(F32)
    w_new = (w - step).astype(F32)
    return w_new, m_new, v_new


def unpack_apply(messages, groups, scale, n, optimizer, w, state1, state2=None, **hyper):
    """CommunicateAndUpdate() after the allgatherv (Section 4.3) with the update folded in: the
    messages [(words, headers)] are decoded and summed in worker order into a zero gradient,
    then one optimizer step is taken.  optimizer: "momentum_sgd" (hyper: lr, mu) or "adam"
    (hyper: lr, beta1, beta2, eps, t).  Returns the new (w, state1[, state2])."""
    ghat = np.zeros(n, F32)
    for words, headers in messages:
        unpack_add(words, headers, groups, scale, ghat)
    if optimizer == "momentum_sgd":
        return momentum_sgd_step(ghat, w, state1, hyper["lr"], hyper["mu"])
    if optimizer == "adam":
        return adam_step(ghat, w, state1, state2, hyper["lr"], hyper["beta1"], hyper["beta2"], hyper["eps"], hyper["t"])
    raise ValueError(optimizer)


# --------------------------------------------------------------------------------------
# Compressed index encoding (Section 4.2, closing remark: the index bits can be reduced
# further by compressing the indexes; the paper names the idea and gives no algorithm)
# --------------------------------------------------------------------------------------
# Reading taken (the format is this build's own): the words of a message are in ascending
# index order, so an element is stored as the distance from its predecessor instead of a
# 28-bit absolute index.  The parameter space of a group is cut into tiles of COMPACT_TILE
# consecutive elements (the last one of a group may be partial), and tiles into runs of
# COMPACT_RUN consecutive tiles of one group.  For every tile, in order, every element of
# the message inside it, in ascending index order, becomes
#     gap  = pos - prev - 1      pos = index inside the tile, prev = pos of the tile's previous
#                                element, -1 for its first
#     code = sign << 3 | d       the 4-bit value of Section 4.2 (top four bits of the word)
#     gap < 8 :  one byte    gap << 4 | code                       (bit 7 clear)
#     else    :  two bytes   0x80 | (gap & 7) << 4 | code,  gap >> 3     (gap <= 2047, so <= 255)
# The message is: the group headers (exp_field, count, byte offset of the group's first tile),
# tile_bytes[t] (uint16, bytes of every tile), run_offsets[r] (uint64, byte offset of every
# run's first tile) and the byte stream.  Each element takes one or two bytes where the plain
# format takes four.

COMPACT_TILE = 2048
COMPACT_RUN = 64


def compact_layout(groups):
    """[(group, first element inside the group, elements)] per tile and the index of each run's first tile."""
    tiles, run_first = [], []
    for k, (off, size) in enumerate(groups):
        for i, start in enumerate(range(0, size, COMPACT_TILE)):
            if i % COMPACT_RUN == 0:
                run_first.append(len(tiles))
            tiles.append((k, start, min(COMPACT_TILE, size - start)))
    return tiles, run_first


def pack_compact(words, headers, groups):
    """Re-encode a message (words, headers as `pack` returns them) with compressed indexes.
    Returns (stream uint8[], tile_bytes uint16[n_tiles], run_offsets uint64[n_runs],
             headers [(exp_field, count, byte offset of the group's stream)]).
    Plain loops over tiles and elements, in the order the format is defined."""
    words = np.asarray(words, dtype=U32)
    tiles, run_first = compact_layout(groups)
    stream = bytearray()
    tile_bytes = np.zeros(len(tiles), np.uint16)
    tile_offset = np.zeros(len(tiles) + 1, np.uint64)
    out_headers = []
    t = 0
    for k, ((off, size), (exp_field, count, word_offset)) in enumerate(zip(groups, headers)):
        out_headers.append((exp_field, count, len(stream)))
        w = words[word_offset:word_offset + count]
        idx = (w & U32(INDEX_MASK)).astype(np.int64)
        code = (w >> U32(28)).astype(np.int64)
        assert np.all(np.diff(idx) > 0) and (count == 0 or idx[-1] < size)
        j = 0
        for start in range(0, size, COMPACT_TILE):
            begin = len(stream)
            prev = -1
            while j < count and idx[j] < start + COMPACT_TILE:
                pos = int(idx[j]) - start
                gap = pos - prev - 1
                assert 0 <= gap < COMPACT_TILE
                if gap < 8:
                    stream.append((gap << 4) | int(code[j]))
                else:
                    stream.append(0x80 | ((gap & 7) << 4) | int(code[j]))
                    stream.append(gap >> 3)
                prev = pos
                j += 1
            tile_offset[t] = begin
            tile_bytes[t] = len(stream) - begin
            t += 1
        assert j == count
    tile_offset[t] = len(stream)
    run_offsets = np.array([tile_offset[f] for f in run_first], np.uint64)
    return np.frombuffer(bytes(stream), np.uint8).copy(), tile_bytes, run_offsets, out_headers


def unpack_compact(stream, tile_bytes, run_offsets, headers, groups):
    """Inverse of pack_compact: the message in the plain format (words uint32[], headers).  Walks the runs
    through run_offsets and the tiles through tile_bytes, as a receiver does."""
    stream = np.asarray(stream, dtype=np.uint8)
    tiles, run_first = compact_layout(groups)
    run_of_tile = {f: r for r, f in enumerate(run_first)}
    words = []
    out_headers = []
    word_offset = 0
    cursor = 0
    per_group = [0] * len(groups)
    for t, (k, start, m) in enumerate(tiles):
        if t in run_of_tile:
            cursor = int(run_offsets[run_of_tile[t]])
        end = cursor + int(tile_bytes[t])
        pos = -1
        while cursor < end:
            b = int(stream[cursor]); cursor += 1
            gap = (b >> 4) & 7
            if b & 0x80:
                gap |= int(stream[cursor]) << 3; cursor += 1
            pos += gap + 1
            assert pos < m
            words.append(((b & 15) << 28) | (start + pos))
            per_group[k] += 1
        assert cursor == end
    for k, (exp_field, count, _) in enumerate(headers):
        assert per_group[k] == count
        out_headers.append((exp_field, count, word_offset))
        word_offset += count
    return np.array(words, dtype=np.uint64).astype(U32), out_headers
