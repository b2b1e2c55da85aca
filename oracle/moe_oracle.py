"""TEST INFRASTRUCTURE -- plain CPU oracle for the Sparsely-Gated Mixture-of-Experts layer.

Only tests, the smoke check and the benchmark's `cpu_baseline` leg may import this module.
It shares no code with the HIP library and never calls it.

Every function is the paper's definition written out with numpy in binary64.  The single
exception is the *selection arithmetic* (the fp32 values of H on which top-k is decided),
which lives in gate_arith.c because the reading R1-R3 stated there needs fused
multiply-adds that numpy does not have.

Citations are to the paper's sections/equations:
  Eq.(1)   y = sum_i G(x)_i E_i(x)                                  Section 2
  Eq.(2)   G_sigma(x) = Softmax(x W_g)                              Section 2.1
  Eq.(3)   G(x) = Softmax(KeepTopK(H(x), k))                        Section 2.1
  Eq.(4)   H(x)_i = (x W_g)_i + N(0,1) Softplus((x W_noise)_i)      Section 2.1
  Eq.(5)   KeepTopK                                                 Section 2.1
  Eq.(6,7) Importance, L_importance = w CV(Importance)^2            Section 4
  Eq.(8-11) P(x,i), Load, L_load                                    Appendix A
  Eq.(12-14) hierarchical output, Importance_H, Load_H              Appendix B
  Eq.(15-20) strictly balanced gating: softmax gate, batchwise mask,
             threshold mask, L_batchwise                            Appendix F
Readings of points the paper leaves open are listed next to the code that takes them.
"""
import ctypes
import os
from dataclasses import dataclass

import numpy as np
from scipy.special import ndtr

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        path = os.path.join(_HERE, "libmoe_oracle.so")
        if not os.path.exists(path):
            from . import build as _b
            _b.build()
        lib = ctypes.CDLL(path)
        f32p = ctypes.POINTER(ctypes.c_float)
        i32p = ctypes.POINTER(ctypes.c_int32)
        lib.oracle_softplus_array.argtypes = [f32p, f32p, ctypes.c_size_t]
        lib.oracle_softplus_array.restype = None
        lib.oracle_dot_chain_f32.argtypes = [f32p, i32p, f32p, ctypes.c_int64, ctypes.c_int64,
                                             ctypes.c_int64, f32p]
        lib.oracle_dot_chain_f32.restype = None
        lib.oracle_noisy_logits_f32.argtypes = [f32p, f32p, f32p, f32p, ctypes.c_int64,
                                                ctypes.c_int64, f32p, f32p, f32p]
        lib.oracle_noisy_logits_f32.restype = None
        _LIB = lib
    return _LIB


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


# --------------------------------------------------------------------------------------
# Eq.(4): the noisy logits, in the pinned fp32 arithmetic (R1-R3 of gate_arith.c)
# --------------------------------------------------------------------------------------

def softplus_f32(z):
    z, zp = _f32(z)
    out = np.empty_like(z)
    _lib().oracle_softplus_array(zp, out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), z.size)
    return out


def dot_chain_f32(x, W, rows=None):
    """[T,n] fp32 = x[rows] . W with the sequential fused-multiply-add chain over j."""
    x, xp = _f32(x)
    W, Wp = _f32(W)
    d, n = W.shape
    assert x.shape[1] == d
    if rows is None:
        T, rp = x.shape[0], None
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        T, rp = rows.shape[0], rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    out = np.empty((T, n), dtype=np.float32)
    _lib().oracle_dot_chain_f32(xp, rp, Wp, T, d, n,
                                out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    return out


@dataclass
class Logits:
    cleanb: np.ndarray   # (x W_g)_i (+ bias_i)            [T,n]
    raw: np.ndarray      # (x W_noise)_i                   [T,n]
    sp: np.ndarray       # Softplus(raw)                   [T,n]
    H: np.ndarray        # Eq.(4)                          [T,n]
    eps: np.ndarray      # the standard-normal draws used  [T,n] (zeros when noise-free)


def noisy_logits_f32(x, W_g, W_noise, eps=None, bias=None, rows=None) -> Logits:
    """Eq.(4) in the pinned fp32 arithmetic.  eps=None gives the noise-free H = x W_g."""
    clean = dot_chain_f32(x, W_g, rows)
    raw = dot_chain_f32(x, W_noise, rows)
    T, n = clean.shape
    cleanb = np.empty_like(clean)
    sp = np.empty_like(clean)
    H = np.empty_like(clean)
    f32p = ctypes.POINTER(ctypes.c_float)
    bp = None
    if bias is not None:
        bias, bp = _f32(bias)
    ep = None
    if eps is not None:
        eps, ep = _f32(eps)
        assert eps.shape == (T, n)
    _lib().oracle_noisy_logits_f32(clean.ctypes.data_as(f32p), raw.ctypes.data_as(f32p), bp, ep,
                                   T, n, cleanb.ctypes.data_as(f32p), sp.ctypes.data_as(f32p),
                                   H.ctypes.data_as(f32p))
    return Logits(cleanb, raw, sp, H, eps if eps is not None else np.zeros_like(clean))


def noisy_logits_f64(x, W_g, W_noise, eps=None, bias=None) -> Logits:
    """Eq.(4) in plain binary64 (used for finite-difference pins and precision studies)."""
    x = np.asarray(x, np.float64)
    cleanb = x @ np.asarray(W_g, np.float64)
    if bias is not None:
        cleanb = cleanb + np.asarray(bias, np.float64)
    raw = x @ np.asarray(W_noise, np.float64)
    sp = np.logaddexp(0.0, raw)
    e = np.zeros_like(cleanb) if eps is None else np.asarray(eps, np.float64)
    H = cleanb + e * sp if eps is not None else cleanb.copy()
    return Logits(cleanb, raw, sp, H, e)


# --------------------------------------------------------------------------------------
# Eq.(5) KeepTopK and Eq.(3) softmax over the kept entries
# --------------------------------------------------------------------------------------

def keep_top_k(H, k):
    """Indices of the k largest entries of each row, in descending order of H; equal values
    are ordered by ascending index (reading: ties go to the lower index; +0 and -0 are equal).
    """
    H = np.asarray(H)
    n = H.shape[1]
    assert 1 <= k <= n
    order = np.argsort(-H, axis=1, kind="stable")
    return order[:, :k].astype(np.int32)


def topk_softmax(H, idx):
    """Eq.(3): Softmax of KeepTopK(H,k).  Entries set to -inf contribute exp(-inf) = 0, so the
    softmax runs over the k kept values only.  Returns gates [T,k] (binary64), aligned with idx."""
    Hk = np.take_along_axis(np.asarray(H, np.float64), idx.astype(np.int64), axis=1)
    z = Hk - Hk.max(axis=1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=1, keepdims=True)


def dense_gates(idx, gates, n):
    """The sparse n-vector G(x) of Eq.(3) as a dense [T,n] array (small cases only)."""
    T, k = idx.shape
    G = np.zeros((T, n), dtype=np.float64)
    G[np.arange(T)[:, None], idx] = gates
    return G


# --------------------------------------------------------------------------------------
# Experts (Appendix C: one ReLU hidden layer, no biases: 512*1024 + 1024*512 = 1M params)
# and Eq.(1)
# --------------------------------------------------------------------------------------

def expert_ffn(xrows, W1, W2):
    """E(x) = relu(x W1) W2 in binary64; W1 [d,h], W2 [h,d]."""
    z = np.asarray(xrows, np.float64) @ np.asarray(W1, np.float64)
    return np.maximum(z, 0.0) @ np.asarray(W2, np.float64)


def moe_output(x, idx, gates, weight_fn, n, token_subset=None):
    """Eq.(1): y = sum_i G(x)_i E_i(x), skipping every (x, i) with G(x)_i = 0 (Section 2).

    weight_fn(e) -> (W1 [d,h], W2 [h,d]) as arrays of the values the experts really hold
    (bf16 values widened exactly, or fp32).  token_subset: optional array of token ids; only
    those rows of y are computed (rows of the result follow token_subset)."""
    x = np.asarray(x, np.float64)
    T, d = x.shape
    if token_subset is None:
        tok = np.arange(T)
    else:
        tok = np.asarray(token_subset, dtype=np.int64)
    idx_s = idx[tok]
    g_s = np.asarray(gates, np.float64)[tok]
    y = np.zeros((tok.shape[0], d), dtype=np.float64)
    for e in np.unique(idx_s):
        r, s = np.nonzero(idx_s == e)          # tokens (within subset) with G(x)_e != 0
        W1, W2 = weight_fn(int(e))
        y[r] += g_s[r, s][:, None] * expert_ffn(x[tok[r]], W1, W2)
    return y


# --------------------------------------------------------------------------------------
# Dispatch bookkeeping by brute force (Section 3.1: each expert gets the combined batch of
# the examples routed to it)
# --------------------------------------------------------------------------------------

def routing(idx, n):
    """counts[e] = number of assignments (t,s) with idx[t,s] = e; offsets = exclusive prefix
    sum; perm = assignment ids a = t*k+s sorted by expert, ties in ascending a (stable);
    inv_perm = inverse permutation."""
    flat = np.asarray(idx).reshape(-1).astype(np.int64)
    counts = np.bincount(flat, minlength=n).astype(np.int32)
    offsets = np.zeros(n + 1, dtype=np.int32)
    offsets[1:] = np.cumsum(counts)
    perm = np.argsort(flat, kind="stable").astype(np.int32)
    inv = np.empty_like(perm)
    inv[perm] = np.arange(perm.shape[0], dtype=np.int32)
    return counts, offsets, perm, inv


# --------------------------------------------------------------------------------------
# Balancing losses: Eq.(6)-(7) and Eq.(8)-(11)
# --------------------------------------------------------------------------------------

def importance(idx, gates, n):
    """Eq.(6): Importance(X) = sum over the batch of G(x)."""
    imp = np.zeros(n, dtype=np.float64)
    np.add.at(imp, np.asarray(idx).reshape(-1), np.asarray(gates, np.float64).reshape(-1))
    return imp


def cv_squared(v):
    """Square of the coefficient of variation.  Reading: population variance (divide by n),
    no epsilon in the denominator."""
    v = np.asarray(v, np.float64)
    mu = v.mean()
    return float(((v - mu) ** 2).mean() / (mu * mu))


def kth_excluding(H, k, idx):
    """kth_excluding(H, k, i) for every i (Appendix A): the k-th highest component of H not
    counting component i.  With S the row sorted descending this is S[k] (0-based) when i is
    one of the top k and S[k-1] otherwise.  Also returns, per row, the indices of the two
    elements that supply those values (needed by the backward pass).
    Requires k < n."""
    H = np.asarray(H)
    T, n = H.shape
    assert k < n
    order = np.argsort(-H, axis=1, kind="stable")
    in_top = np.zeros((T, n), dtype=bool)
    in_top[np.arange(T)[:, None], idx] = True
    j_in = order[:, k]        # supplies the threshold for selected experts
    j_out = order[:, k - 1]   # supplies the threshold for the others
    thr = np.where(in_top, H[np.arange(T), j_in][:, None], H[np.arange(T), j_out][:, None])
    return thr, in_top, j_in, j_out


def load(lg: Logits, k, idx):
    """Eq.(9)-(10): P(x,i) = Phi((clean_i - kth_excluding(H,k,i)) / Softplus(raw_i)),
    Load(X)_i = sum_x P(x,i).  Reading for k = n: every expert is always selected, so P = 1."""
    T, n = lg.H.shape
    if k == n:
        P = np.ones((T, n), dtype=np.float64)
        return P.sum(axis=0), P
    thr, _, _, _ = kth_excluding(lg.H, k, idx)
    u = (np.asarray(lg.cleanb, np.float64) - np.asarray(thr, np.float64)) / np.asarray(lg.sp, np.float64)
    P = ndtr(u)
    return P.sum(axis=0), P


@dataclass
class FlatForward:
    idx: np.ndarray
    gates: np.ndarray
    logits: Logits
    importance: np.ndarray
    load: np.ndarray
    loss_importance: float
    loss_load: float


def gate_and_losses(lg: Logits, k, w_importance=0.1, w_load=0.1) -> FlatForward:
    """Eq.(3),(5) on the given logits, then Eq.(6),(7),(10),(11)."""
    n = lg.H.shape[1]
    idx = keep_top_k(lg.H, k)
    gates = topk_softmax(lg.H, idx)
    imp = importance(idx, gates, n)
    ld, _ = load(lg, k, idx)
    return FlatForward(idx, gates, lg, imp, ld, w_importance * cv_squared(imp), w_load * cv_squared(ld))


# --------------------------------------------------------------------------------------
# Hierarchical MoE: Eq.(12)-(14)
# --------------------------------------------------------------------------------------

@dataclass
class HierForward:
    idx: np.ndarray          # [T, k_p*k_s] global expert id i*b + j, slot-major (p-slot, s-slot)
    gates: np.ndarray        # [T, k_p*k_s] G_primary(x)_i * G_i(x)_j
    group_idx: np.ndarray    # [T, k_p]
    group_gates: np.ndarray  # [T, k_p]
    sec_idx: np.ndarray      # [T, k_p, k_s] index j within the group
    sec_gates: np.ndarray    # [T, k_p, k_s]
    importance: np.ndarray   # [a*b]  Eq.(13)
    load: np.ndarray         # [a*b]  Eq.(14)
    load_primary: np.ndarray
    group_counts: np.ndarray  # |X^(i)|
    loss_importance: float
    loss_load: float


def hier_gate_and_losses(x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, k_p, k_s,
                         w_importance=0.1, w_load=0.1) -> HierForward:
    """Primary noisy top-k gate over a groups; for every group i the secondary gate G_i is
    evaluated on X^(i) = {x : G_primary(x)_i > 0} only (Appendix B).
    Reading: the secondary noise tensor is indexed by the primary slot, eps_s[t, p, :]."""
    a, d, b = Wg_s.shape
    T = x.shape[0]
    lp = noisy_logits_f32(x, Wg_p, Wn_p, eps_p)
    gidx = keep_top_k(lp.H, k_p)
    ggate = topk_softmax(lp.H, gidx)
    load_p, _ = load(lp, k_p, gidx)

    sec_idx = np.zeros((T, k_p, k_s), dtype=np.int32)
    sec_gate = np.zeros((T, k_p, k_s), dtype=np.float64)
    load_s = np.zeros((a, b), dtype=np.float64)
    gcount = np.zeros(a, dtype=np.int64)
    for i in range(a):
        tt, pp = np.nonzero(gidx == i)           # members of X^(i) and the slot that chose i
        gcount[i] = tt.shape[0]
        if tt.shape[0] == 0:
            continue
        li = noisy_logits_f32(x, Wg_s[i], Wn_s[i], eps_s[tt, pp, :], rows=tt)
        si = keep_top_k(li.H, k_s)
        sec_idx[tt, pp, :] = si
        sec_gate[tt, pp, :] = topk_softmax(li.H, si)
        load_s[i], _ = load(li, k_s, si)

    idx = (gidx[:, :, None].astype(np.int64) * b + sec_idx).reshape(T, k_p * k_s).astype(np.int32)
    gates = (ggate[:, :, None] * sec_gate).reshape(T, k_p * k_s)
    imp = importance(idx, gates, a * b)          # Eq.(13)
    # Eq.(14); reading: an empty X^(i) gives Load_H(i, .) = 0 instead of 0/0.
    denom = np.where(gcount > 0, gcount, 1).astype(np.float64)
    load_h = (load_p[:, None] * load_s / denom[:, None]).reshape(-1)
    return HierForward(idx, gates, gidx, ggate, sec_idx, sec_gate, imp, load_h, load_p, gcount,
                       w_importance * cv_squared(imp), w_load * cv_squared(load_h))


# --------------------------------------------------------------------------------------
# Backward pass (Section 2.1, "Training the Gating Network": plain back-propagation through
# the kept gate values, the experts and both losses; Appendix D: hidden activations are
# recomputed, nothing but gate quantities is kept from the forward pass)
# --------------------------------------------------------------------------------------

def round_to_bf16(a):
    """Round fp32 values to the nearest bfloat16 (ties to even), returned as float32."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def dcv_squared(v):
    """Gradient of cv_squared with respect to v (population variance)."""
    v = np.asarray(v, np.float64)
    n = v.shape[0]
    S = v.sum()
    return 2.0 * n * v / S ** 2 - 2.0 * n * (v * v).sum() / S ** 3


@dataclass
class Grads:
    dx: np.ndarray
    dW_g: np.ndarray
    dW_noise: np.ndarray
    dbias: np.ndarray
    dW1: dict   # expert id -> [d,h]
    dW2: dict   # expert id -> [h,d]


def gate_level_backward(lg: Logits, idx, g, dgate, gL, k):
    """Backward of one noisy top-k gate (Eq.(3)-(5), (8)-(10)) on its own rows.
    dgate [R,k]: everything that arrives at the kept softmax values; gL [n]: dJ/dLoad of this
    gate's Load vector, or None when it carries no Load term.  Returns (dclean, draw) [R,n]:
    gradients with respect to the clean logits (bias included) and to the raw noise logits."""
    g = np.asarray(g, np.float64)
    dgate = np.asarray(dgate, np.float64)
    cleanb = np.asarray(lg.cleanb, np.float64)
    sp = np.asarray(lg.sp, np.float64)
    raw = np.asarray(lg.raw, np.float64)
    eps = np.asarray(lg.eps, np.float64)
    T, n = cleanb.shape

    # softmax over the kept entries, Eq.(3)
    dH = np.zeros((T, n), dtype=np.float64)
    inner = (g * dgate).sum(axis=1, keepdims=True)
    dH[np.arange(T)[:, None], idx] = g * (dgate - inner)

    dclean = np.zeros((T, n), dtype=np.float64)
    dsp = np.zeros((T, n), dtype=np.float64)
    # L_load, Eq.(8)-(11)
    if gL is not None and k < n:
        gL = np.asarray(gL, np.float64)
        thr, in_top, j_in, j_out = kth_excluding(lg.H, k, idx)
        thr = np.asarray(thr, np.float64)
        u = (cleanb - thr) / sp
        phi = np.exp(-0.5 * u * u) / np.sqrt(2.0 * np.pi)
        c = gL[None, :] * phi / sp
        dclean += c
        dsp += -c * u
        rows = np.arange(T)
        np.add.at(dH, (rows, j_in), -(c * in_top).sum(axis=1))
        np.add.at(dH, (rows, j_out), -(c * ~in_top).sum(axis=1))

    # H = cleanb + eps * sp, Eq.(4)
    dclean += dH
    dsp += dH * eps
    draw = dsp / (1.0 + np.exp(-raw))        # d softplus = sigmoid
    return dclean, draw


def experts_backward(xe_all, idx, g, weight_fn, dy, experts_for_dW=None, only=None):
    """Backward of Eq.(1) and of the experts (Appendix C) for assignments idx [T,k] with gate values
    g [T,k]: returns (dx through the experts [T,d], dgate [T,k] = <dy_t, E_e(x_t)>, dW1, dW2).
    only: evaluate just these experts (for sampled checks of dW1/dW2 at sizes where the whole loop
    is too slow; dx and dgate are then partial)."""
    xe_all = np.asarray(xe_all, np.float64)
    g = np.asarray(g, np.float64)
    dx = np.zeros_like(xe_all)
    dgate = np.zeros_like(g)
    dW1, dW2 = {}, {}
    keep = None if experts_for_dW is None else set(int(e) for e in experts_for_dW)
    for e in (np.unique(idx) if only is None else sorted(set(int(q) for q in only))):
        r, s = np.nonzero(idx == e)
        if r.size == 0:
            continue
        W1, W2 = (np.asarray(w, np.float64) for w in weight_fn(int(e)))
        xe = xe_all[r]
        z = xe @ W1
        hid = np.maximum(z, 0.0)
        out = hid @ W2
        dgate[r, s] = np.einsum("ij,ij->i", dy[r], out)
        dout = g[r, s][:, None] * dy[r]
        dh = dout @ W2.T
        dz = dh * (z > 0.0)
        dx[r] += dz @ W1.T          # a token reaches an expert at most once, so r has no repeats
        if keep is None or int(e) in keep:
            dW2[int(e)] = hid.T @ dout
            dW1[int(e)] = xe.T @ dz
    return dx, dgate, dW1, dW2


def expert_input_grad(xe, dout, W1, W2, relu_mask=None):
    """Gradient of <dout, E(xe)> with respect to the rows xe of ONE expert (Appendix C):
    ((dout W2^T) * [z > 0]) W1^T with z = xe W1.  relu_mask [rows,h] (bool) replaces the sign test
    z > 0: parity tests use it to evaluate a row on the other side's decision at hidden units whose
    pre-activation is zero to within rounding, where either decision is a correct evaluation."""
    xe, dout = np.asarray(xe, np.float64), np.asarray(dout, np.float64)
    W1, W2 = np.asarray(W1, np.float64), np.asarray(W2, np.float64)
    z = xe @ W1
    mask = (z > 0.0) if relu_mask is None else np.asarray(relu_mask, bool)
    return ((dout @ W2.T) * mask) @ W1.T


def flat_backward(x, W_g, W_noise, fwd: FlatForward, k, weight_fn, dy,
                  w_importance=0.1, w_load=0.1, experts_for_dW=None, expert_input=None) -> Grads:
    """Gradients of J = <dy, y> + L_importance + L_load for the flat layer.

    The top-k selection is piecewise constant, so no gradient flows through *which* experts
    are kept; it flows through the kept softmax values, through P(x,i) of Eq.(9) (including
    the threshold element kth_excluding picks, as differentiating Eq.(9) as printed gives) and
    through the experts.  relu'(0) is taken as 0.
    experts_for_dW: optional iterable restricting which experts' dW1/dW2 are returned.
    expert_input: optional [T,d] array the experts see instead of x.  For the bf16 workloads the
    experts' input activations are bf16(x); the sign test z > 0 of the ReLU derivative is a binary
    decision, so it has to be taken on the same rounded input on both sides of a parity test
    (a flipped unit changes dz by its full size).  The gating path always uses x itself."""
    x = np.asarray(x, np.float64)
    xe_all = x if expert_input is None else np.asarray(expert_input, np.float64)
    dy = np.asarray(dy, np.float64)
    W_g = np.asarray(W_g, np.float64)
    W_noise = np.asarray(W_noise, np.float64)
    T, d = x.shape
    n = W_g.shape[1]
    lg = fwd.logits
    idx, g = fwd.idx, np.asarray(fwd.gates, np.float64)
    cleanb = np.asarray(lg.cleanb, np.float64)
    sp = np.asarray(lg.sp, np.float64)
    raw = np.asarray(lg.raw, np.float64)
    eps = np.asarray(lg.eps, np.float64)
    H = np.asarray(lg.H, np.float64)

    dx, dgate, dW1, dW2 = experts_backward(xe_all, idx, g, weight_fn, dy, experts_for_dW)

    # L_importance, Eq.(6)-(7)
    gI = w_importance * dcv_squared(fwd.importance)
    dgate += gI[idx]

    gL = w_load * dcv_squared(fwd.load) if (k < n and w_load != 0.0) else None
    dclean, draw = gate_level_backward(lg, idx, g, dgate, gL, k)
    dW_g = x.T @ dclean
    dW_noise = x.T @ draw
    dx += dclean @ W_g.T + draw @ W_noise.T
    return Grads(dx, dW_g, dW_noise, dclean.sum(axis=0), dW1, dW2)


def flat_objective(x, W_g, W_noise, eps, bias, k, weight_fn, dy, w_importance, w_load,
                   fixed_idx=None):
    """J = <dy,y> + L_importance + L_load evaluated entirely in binary64 (for finite
    differences).  fixed_idx freezes the selection so that J is smooth in the parameters."""
    lg = noisy_logits_f64(x, W_g, W_noise, eps, bias)
    n = lg.H.shape[1]
    idx = keep_top_k(lg.H, k) if fixed_idx is None else fixed_idx
    gates = topk_softmax(lg.H, idx)
    y = moe_output(x, idx, gates, weight_fn, n)
    imp = importance(idx, gates, n)
    ld, _ = load(lg, k, idx)
    return float((np.asarray(dy, np.float64) * y).sum()
                 + w_importance * cv_squared(imp) + w_load * cv_squared(ld))


@dataclass
class HierGrads:
    dx: np.ndarray
    dWg_p: np.ndarray      # [d,a]
    dWn_p: np.ndarray
    dWg_s: np.ndarray      # [a,d,b]
    dWn_s: np.ndarray
    dW1: dict
    dW2: dict


def _hier_forward_parts(x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, k_p, k_s, logits_fn,
                        fixed_gidx=None, fixed_sidx=None):
    """The hierarchical gate with every intermediate the backward pass needs."""
    a, d, b = Wg_s.shape
    T = x.shape[0]
    lp = logits_fn(x, Wg_p, Wn_p, eps_p)
    gidx = keep_top_k(lp.H, k_p) if fixed_gidx is None else fixed_gidx
    ggate = topk_softmax(lp.H, gidx)
    load_p = load(lp, k_p, gidx)[0]
    sec_idx = np.zeros((T, k_p, k_s), dtype=np.int64)
    sec_gate = np.zeros((T, k_p, k_s), dtype=np.float64)
    load_s = np.zeros((a, b), dtype=np.float64)
    gcount = np.zeros(a, dtype=np.int64)
    members, sec_logits = {}, {}
    for i in range(a):
        tt, pp = np.nonzero(gidx == i)
        gcount[i] = tt.shape[0]
        if tt.shape[0] == 0:
            continue
        li = logits_fn(x[tt], Wg_s[i], Wn_s[i], eps_s[tt, pp, :])
        si = keep_top_k(li.H, k_s) if fixed_sidx is None else fixed_sidx[tt, pp, :]
        sec_idx[tt, pp, :] = si
        sec_gate[tt, pp, :] = topk_softmax(li.H, si)
        load_s[i] = load(li, k_s, si)[0]
        members[i], sec_logits[i] = (tt, pp), li
    idx = (gidx[:, :, None].astype(np.int64) * b + sec_idx).reshape(T, k_p * k_s)
    gates = (ggate[:, :, None] * sec_gate).reshape(T, k_p * k_s)
    imp = importance(idx, gates, a * b)
    denom = np.where(gcount > 0, gcount, 1).astype(np.float64)
    load_h = (load_p[:, None] * load_s / denom[:, None]).reshape(-1)
    return dict(lp=lp, gidx=gidx, ggate=ggate, load_p=load_p, sec_idx=sec_idx, sec_gate=sec_gate,
                load_s=load_s, gcount=gcount, denom=denom, members=members, sec_logits=sec_logits,
                idx=idx, gates=gates, imp=imp, load_h=load_h)


def hier_backward(x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, k_p, k_s, weight_fn, dy,
                  w_importance=0.1, w_load=0.1, experts_for_dW=None, expert_input=None,
                  logits_fn=None) -> HierGrads:
    """Gradients of J = <dy, y> + w_importance CV^2(Importance_H) + w_load CV^2(Load_H) for the
    hierarchical layer (Appendix B, Eq.(12)-(14)), by the chain rule through
        gate(t, i, j) = G_primary(x_t)_i * G_i(x_t)_j,
        Importance_H(i,j) = sum_t gate(t,i,j),
        Load_H(i,j) = Load_primary(i) * Load_i(X^(i))_j / |X^(i)|     (|X^(i)| is a count: constant),
    into both gating levels (each a noisy top-k gate: gate_level_backward) and the experts.
    logits_fn defaults to the pinned fp32 logits of the forward pass."""
    if logits_fn is None:
        logits_fn = noisy_logits_f32
    x64 = np.asarray(x, np.float64)
    dy = np.asarray(dy, np.float64)
    a, d, b = Wg_s.shape
    T = x64.shape[0]
    f = _hier_forward_parts(x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, k_p, k_s, logits_fn)
    xe_all = x64 if expert_input is None else np.asarray(expert_input, np.float64)
    dx_e, dgate, dW1, dW2 = experts_backward(xe_all, f["idx"], f["gates"], weight_fn, dy, experts_for_dW)
    dx = dx_e.copy()

    # Eq.(13): the composite gate values also feed Importance_H
    dgate = dgate + (w_importance * dcv_squared(f["imp"]))[f["idx"]]
    dg3 = dgate.reshape(T, k_p, k_s)
    dGp = (dg3 * f["sec_gate"]).sum(axis=2)                    # Eq.(12): product rule
    dGs = dg3 * f["ggate"][:, :, None]

    # Eq.(14)
    dLoad_p, dLoad_s = None, None
    if w_load != 0.0:
        gLh = (w_load * dcv_squared(f["load_h"])).reshape(a, b)
        dLoad_p = (gLh * f["load_s"]).sum(axis=1) / f["denom"]
        dLoad_s = gLh * f["load_p"][:, None] / f["denom"][:, None]

    Wg_p64, Wn_p64 = np.asarray(Wg_p, np.float64), np.asarray(Wn_p, np.float64)
    dclean, draw = gate_level_backward(f["lp"], f["gidx"], f["ggate"], dGp, dLoad_p, k_p)
    dWg_p, dWn_p = x64.T @ dclean, x64.T @ draw
    dx += dclean @ Wg_p64.T + draw @ Wn_p64.T

    dWg_s = np.zeros((a, d, b))
    dWn_s = np.zeros((a, d, b))
    for i, (tt, pp) in f["members"].items():
        dci, dri = gate_level_backward(f["sec_logits"][i], f["sec_idx"][tt, pp, :], f["sec_gate"][tt, pp, :],
                                       dGs[tt, pp, :], None if dLoad_s is None else dLoad_s[i], k_s)
        dWg_s[i] = x64[tt].T @ dci
        dWn_s[i] = x64[tt].T @ dri
        # a token picks a group at most once, so tt has no repeats
        dx[tt] += dci @ np.asarray(Wg_s[i], np.float64).T + dri @ np.asarray(Wn_s[i], np.float64).T
    return HierGrads(dx, dWg_p, dWn_p, dWg_s, dWn_s, dW1, dW2)


def hier_objective(x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, k_p, k_s, weight_fn, dy,
                   w_importance, w_load, fixed_gidx, fixed_sidx):
    """J of hier_backward evaluated entirely in binary64 with both selections frozen (for
    finite differences)."""
    f = _hier_forward_parts(x, Wg_p, Wn_p, eps_p, Wg_s, Wn_s, eps_s, k_p, k_s, noisy_logits_f64,
                            fixed_gidx, fixed_sidx)
    a, _, b = Wg_s.shape
    y = moe_output(x, f["idx"], f["gates"], weight_fn, a * b)
    return float((np.asarray(dy, np.float64) * y).sum()
                 + w_importance * cv_squared(f["imp"]) + w_load * cv_squared(f["load_h"]))



# --------------------------------------------------------------------------------------
# Appendix F: strictly balanced gating
# --------------------------------------------------------------------------------------

def softmax_gate_f32(x, W_g, bias=None):
    """Eq.(15): G_sigma(x) = Softmax(x W_g) over all n experts.  The logits are the fp32 values of
    reading R1 (the same ones noisy top-k gating selects on); the softmax itself is the plain
    definition in binary64 -- exponentials of (logit - row maximum), ONE accumulator summing them
    over i ascending, one division -- rounded once to fp32.  Returns (logits, G_sigma), both fp32."""
    clean = dot_chain_f32(x, W_g)
    if bias is not None:
        clean = (clean + np.asarray(bias, np.float32)[None, :]).astype(np.float32)
    l = clean.astype(np.float64)
    e = np.exp(l - l.max(axis=1, keepdims=True))
    s = np.zeros(l.shape[0])
    for i in range(l.shape[1]):          # sequential, i ascending (numpy's sum is pairwise)
        s = s + e[:, i]
    return clean, (e / s[:, None]).astype(np.float32)


def batchwise_mask(X, m):
    """Eq.(18): M_batchwise(X, m)[j, i] = 1 iff X[j, i] is among the m largest values of column i.
    Reading: equal values -> the lower token index first.  Returns (mask [T,n] bool, tokens [n,m]
    int32: the kept tokens of every expert in ascending order)."""
    X = np.asarray(X)
    T, n = X.shape
    assert 0 <= m <= T
    order = np.argsort(-X.astype(np.float64), axis=0, kind="stable")   # per column, ties: lower j first
    kept = np.sort(order[:m, :], axis=0)                               # [m, n]
    mask = np.zeros((T, n), dtype=bool)
    mask[kept, np.arange(n)[None, :]] = True
    return mask, np.ascontiguousarray(kept.T.astype(np.int32))


def balanced_gates(X, mask):
    """Eq.(16): G(x)_i = G_sigma(x)_i M_i / sum_j G_sigma(x)_j M_j.  Reading: a token that no
    expert keeps has G(x) = 0 (the quotient would be 0/0).  Returns (G [T,n] float64, denom [T])."""
    Xm = np.where(mask, np.asarray(X, np.float64), 0.0)
    denom = Xm.sum(axis=1)
    G = np.divide(Xm, denom[:, None], out=np.zeros_like(Xm), where=denom[:, None] > 0)
    return G, denom


def threshold_mask(X, thresholds):
    """Eq.(19): M_threshold(x, T)_i = 1 iff x_i > T_i."""
    return np.asarray(X, np.float64) > np.asarray(thresholds, np.float64)[None, :]


def batchwise_loss(X, mask, thresholds):
    """Eq.(20): L_batchwise = sum_j sum_i (M_threshold - M_batchwise)(X_ji - T_i)."""
    X = np.asarray(X, np.float64)
    Tv = np.asarray(thresholds, np.float64)[None, :]
    diff = threshold_mask(X, thresholds).astype(np.float64) - mask.astype(np.float64)
    return float((diff * (X - Tv)).sum())


def batchwise_loss_dthresholds(X, mask, thresholds):
    """d L_batchwise / d T_i (Eq.(20)).  Both masks are piecewise constant in T, so only the factor
    (X_ji - T_i) varies: the derivative is -sum_j (M_threshold - M_batchwise)_ji, i.e. the number of
    tokens the batchwise mask keeps for expert i minus the number above its threshold."""
    diff = threshold_mask(X, thresholds).astype(np.float64) - np.asarray(mask, np.float64)
    return -diff.sum(axis=0)


def balanced_output(x, G, weight_fn, token_subset=None):
    """Eq.(1) with the gates of Eq.(16): y_t = sum_i G(x_t)_i E_i(x_t)."""
    x64 = np.asarray(x, np.float64)
    T, n = G.shape
    toks = np.arange(T) if token_subset is None else np.asarray(token_subset)
    y = np.zeros((len(toks), x64.shape[1]))
    sub = G[toks]
    for e in range(n):
        rows = np.nonzero(sub[:, e] > 0)[0]
        if rows.size == 0:
            continue
        W1, W2 = weight_fn(e)
        y[rows] += sub[rows, e][:, None] * expert_ffn(x64[toks[rows]], W1, W2)
    return y


@dataclass
class BalancedGrads:
    dx: np.ndarray
    dW_g: np.ndarray
    dbias: np.ndarray
    dW1: dict
    dW2: dict
    dlogits: np.ndarray


def balanced_backward(x, W_g, Gs, mask, thresholds, weight_fn, dy, w_batchwise=0.0,
                      experts_for_dW=None, expert_input=None) -> BalancedGrads:
    """Gradients of J = <dy, y> + w_batchwise * L_batchwise for the layer with strictly balanced
    gating (Appendix F), with respect to x, W_g (and a bias added to the logits) and the experts.

    Both masks are piecewise constant, so the gradient reaches the gate only through the values
    G_sigma: through the quotient of Eq.(16), through the factor (G_sigma - T_i) of Eq.(20) as
    printed, and from there through the softmax of Eq.(15) over all n experts.  relu'(0) = 0.
    Gs [T,n]: the softmax values the forward pass used; mask [T,n] bool: M_batchwise.
    expert_input / experts_for_dW as in flat_backward."""
    x = np.asarray(x, np.float64)
    xe_all = x if expert_input is None else np.asarray(expert_input, np.float64)
    dy = np.asarray(dy, np.float64)
    W_g = np.asarray(W_g, np.float64)
    Gs = np.asarray(Gs, np.float64)
    mask = np.asarray(mask, bool)
    T, n = Gs.shape
    G, denom = balanced_gates(Gs, mask)
    keep = None if experts_for_dW is None else set(int(e) for e in experts_for_dW)
    dx = np.zeros_like(x)
    dG = np.zeros((T, n))
    dW1, dW2 = {}, {}
    for e in range(n):
        r = np.nonzero(mask[:, e])[0]
        if r.size == 0:
            continue
        W1, W2 = (np.asarray(w, np.float64) for w in weight_fn(e))
        xe = xe_all[r]
        z = xe @ W1
        hid = np.maximum(z, 0.0)
        out = hid @ W2
        dG[r, e] = np.einsum("ij,ij->i", dy[r], out)          # Eq.(1)
        dout = G[r, e][:, None] * dy[r]
        dz = (dout @ W2.T) * (z > 0.0)
        dx[r] += dz @ W1.T
        if keep is None or e in keep:
            dW2[e] = hid.T @ dout
            dW1[e] = xe.T @ dz
    # Eq.(16): G_i = Gs_i M_i / D, D = sum_j Gs_j M_j
    inner = (G * dG).sum(axis=1)
    live = denom > 0
    dGs = np.zeros((T, n))
    dGs[live] = np.where(mask[live], (dG[live] - inner[live, None]) / denom[live, None], 0.0)
    # Eq.(20)
    if w_batchwise != 0.0:
        dGs += w_batchwise * (threshold_mask(Gs, thresholds).astype(np.float64) - mask.astype(np.float64))
    # Eq.(15)
    dlogits = Gs * (dGs - (Gs * dGs).sum(axis=1)[:, None])
    dW_g = x.T @ dlogits
    dx += dlogits @ W_g.T
    return BalancedGrads(dx, dW_g, dlogits.sum(axis=0), dW1, dW2, dlogits)


def balanced_objective(x, W_g, bias, thresholds, m, weight_fn, dy, w_batchwise, fixed_masks=None):
    """J = <dy, y> + w_batchwise * L_batchwise of the balanced layer entirely in binary64 (for
    finite differences).  fixed_masks = (M_batchwise, M_threshold) freezes both masks so that J is
    smooth.  Returns (J, M_batchwise, M_threshold, G_sigma)."""
    x = np.asarray(x, np.float64)
    logits = x @ np.asarray(W_g, np.float64)
    if bias is not None:
        logits = logits + np.asarray(bias, np.float64)[None, :]
    ex = np.exp(logits - logits.max(axis=1, keepdims=True))
    Gs = ex / ex.sum(axis=1, keepdims=True)
    if fixed_masks is None:
        mb, _ = batchwise_mask(Gs, m)
        mt = threshold_mask(Gs, thresholds)
    else:
        mb, mt = fixed_masks
    G, _ = balanced_gates(Gs, mb)
    y = balanced_output(x, G, weight_fn)
    Lb = ((mt.astype(np.float64) - mb.astype(np.float64)) * (Gs - np.asarray(thresholds, np.float64)[None, :])).sum()
    return float((np.asarray(dy, np.float64) * y).sum() + w_batchwise * Lb), mb, mt, Gs


# --------------------------------------------------------------------------------------
# Appendix D: Adam with beta1 = 0 and a factored second-moment estimator for the expert matrices
# --------------------------------------------------------------------------------------

def factored_adam_step(W, G, v_row, v_col, lr, beta2, eps, step):
    """One update of a parameter matrix W [R, C] with gradient G (Appendix D, "Optimizer").

    No first-moment estimator (beta1 = 0: the update direction is G itself).  Instead of the
    full matrix V of second-moment estimates only its row-wise and column-wise averages are
    kept: v_row [R], v_col [C].  V obeys V <- beta2 V + (1 - beta2) G*G elementwise, and
    averaging is linear, so the two vectors obey the same recursion with the row and column
    averages of G*G.  At the step the matrix of estimators is taken as
        Vhat[r, c] = v_row[r] * v_col[c] / mean(v_row)        (mean(v_row) == mean(v_col)).
    Readings where the paper is silent: Adam's bias correction Vhat / (1 - beta2**step) with
    step counted from 1, and its epsilon outside the square root,
        W <- W - lr * G / (sqrt(Vhat / (1 - beta2**step)) + eps);
    an all-zero gradient history (mean(v_row) == 0) leaves W unchanged.
    Returns (W_new, v_row_new, v_col_new), all float64."""
    W = np.asarray(W, np.float64)
    G = np.asarray(G, np.float64)
    g2 = G * G
    v_row = beta2 * np.asarray(v_row, np.float64) + (1.0 - beta2) * g2.mean(axis=1)
    v_col = beta2 * np.asarray(v_col, np.float64) + (1.0 - beta2) * g2.mean(axis=0)
    m = v_row.mean()
    if m == 0.0:
        return W.copy(), v_row, v_col
    vhat = np.outer(v_row, v_col) / m / (1.0 - beta2 ** step)
    return W - lr * G / (np.sqrt(vhat) + eps), v_row, v_col


# --------------------------------------------------------------------------------------
# Appendix C, "Model Architecture": what the language models do with the MoE layer's output
# --------------------------------------------------------------------------------------

def layer_epilogue(y, x, keep, drop_prob):
    """out = x + dropout(sigmoid(y)): the MoE output goes through a sigmoid, each activation is
    dropped with probability drop_prob and the survivors are divided by 1 - drop_prob, then the
    layer's input is added (residual connection).  keep [T,d] bool is the dropout draw (an input:
    True = the activation survives); keep=None means no dropout (drop_prob must then be 0)."""
    y = np.asarray(y, np.float64)
    s = 1.0 / (1.0 + np.exp(-y))
    if keep is None:
        assert drop_prob == 0.0
        return np.asarray(x, np.float64) + s
    assert 0.0 <= drop_prob < 1.0
    return np.asarray(x, np.float64) + np.where(np.asarray(keep, bool), s / (1.0 - drop_prob), 0.0)
