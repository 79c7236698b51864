"""CPU oracle for the QTALE inference hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct NumPy implementation of what the GPU library
computes.  It exists to check the HIP path; nothing in the product imports it,
and it shares no code, tables or helpers with the HIP sources.

What is implemented, and the passage of the paper each part follows:

* residual decoder layer  x_{l+1} = x_l + f_l(x_l)                  (Sec. 2.1, Eq. 1)
* token-adaptive execution: executed tokens take Eq. 1, bypassed tokens keep
  x_{l+1} = x_l exactly                                            (Sec. 2.2, Eq. 3)
* routing decision: p = softmax(g_l(x_l)), execute iff p_0 >= theta, with one
  theta shared by all layers; theta = 0.5 is the arg-max rule of Eq. 2
                                                                    (Sec. 3.4, Eq. 9)
* active tokens are gathered into a dense matrix before the layer   (App. B.2)
* weight-only group quantization with groups along the input dimension,
  4 bit and 3 bit (Sec. 4.1 setup); 2 bit for the mixed 2-/4-bit stack of the
  paper's mixed-precision appendix
* two-phase grid search for the global theta (coarse 0.05, fine 0.01 on (0, 0.5]),
  with the average execution ratio as the objective                 (Sec. 3.4)

The paper gives no formula for the quantizer, the router's architecture, or the
inside of f_l; those follow the readings listed in this repository's design
notes: round-to-nearest asymmetric min/max quantizer with fp16 scale and integer
zero-point; a linear router whose single output is the execute-minus-bypass
logit z (softmax over two classes of logits (z_e, z_b) gives p_0 = sigmoid(z_e -
z_b)); f_l is a textbook pre-norm LLaMA block (RMSNorm, rotary embedding with
half-split pairing at the token's original absolute position, causal softmax
attention among the *executed* tokens of the same sequence, SwiGLU MLP).

Pins (tests/test_oracle_*.py): brute-force nearest-code search for the quantizer,
closed forms for dequantisation, full-sort check and nesting/monotonicity for
the selection, ratio 1 == dense layer, ratio 0 == identity, bypassed rows
bit-identical, agreement with an independent per-token brute-force loop
(`layer_forward_bruteforce`), torch fp64 library attention/matmul as a third
opinion, rotary relative-position property, the paper's FLOPs-per-token figure;
the theta search against an exhaustive scan of all 50 grid points and a closed-form
score distribution.
Numeric values of hidden states: parity unpinned by the paper (it prints no
activations); pinned only by the self-consistency checks above.

All floating point is fp64 except where a bit-exact contract fixes fp32/fp16
(the quantizer, and the final rounding of the router score to fp32).
"""
import math

import numpy as np

# --------------------------------------------------------------------------
# Quantizer (setup step; group-wise round-to-nearest, Sec. 4.1 "group size")
# --------------------------------------------------------------------------


def n_groups(K, group):
    return (K + group - 1) // group


def quantize_rtn(W, bits=4, group=128):
    """Quantize an fp32 matrix W [N, K] row by row in groups along K.

    Per (row, group): lo = min(0, min W), hi = max(0, max W); the fp32 scale
    (hi - lo) / (2^bits - 1) is rounded to fp16 (1.0 if that is zero or not
    finite); zero-point = clamp(rint(-lo / s)); code = clamp(rint(W / s) + zero).
    All arithmetic is IEEE fp32 with round-half-even.  A short last group uses
    only its own members.

    Returns codes uint8 [N, K], scales fp16 [N, n_groups], zeros fp16 [N, n_groups].
    """
    W = np.asarray(W, dtype=np.float32)
    N, K = W.shape
    qmax = np.float32((1 << bits) - 1)
    ng = n_groups(K, group)
    codes = np.zeros((N, K), dtype=np.uint8)
    scales = np.zeros((N, ng), dtype=np.float16)
    zeros = np.zeros((N, ng), dtype=np.float16)
    for g in range(ng):
        k0, k1 = g * group, min((g + 1) * group, K)
        Wg = W[:, k0:k1]
        lo = np.minimum(np.float32(0), Wg.min(axis=1)).astype(np.float32)
        hi = np.maximum(np.float32(0), Wg.max(axis=1)).astype(np.float32)
        s32 = ((hi - lo).astype(np.float32) / qmax).astype(np.float32)
        with np.errstate(over="ignore"):
            s16 = s32.astype(np.float16)
        bad = (s16 == 0) | ~np.isfinite(s16)
        s16[bad] = np.float16(1.0)
        sf = s16.astype(np.float32)
        z = np.clip(np.rint((-lo / sf).astype(np.float32)), 0, qmax).astype(np.float32)
        z = z + np.float32(0.0)          # the zero-point is an integer code: -0.0 (from lo == 0) is stored as +0
        q = np.rint((Wg / sf[:, None]).astype(np.float32)).astype(np.float32) + z[:, None]
        q = np.clip(q, 0, qmax)
        codes[:, k0:k1] = q.astype(np.uint8)
        scales[:, g] = s16
        zeros[:, g] = z.astype(np.float16)
    return codes, scales, zeros


def pack_codes(codes, bits=4):
    """Canonical packing of the codes of one matrix, uint32 [N, words per row].

    4 bit: ceil(K/8) words per row, nibble j of word w holds the code of k = 8*w + j
    (least-significant nibble first); rows are padded with code 0.
    2 bit: ceil(K/16) words per row, bit pair j of word w holds the code of k = 16*w + j.
    3 bit: the codes of a row form one little-endian bit stream, code k at bits [3k, 3k+3), cut into
    32-bit words (32 codes fill exactly 3 words); rows are padded with code 0 to a whole number of
    32-code blocks, i.e. 3*ceil(K/32) words per row."""
    N, K = codes.shape
    if bits == 4:
        nw = (K + 7) // 8
        padded = np.zeros((N, nw * 8), dtype=np.uint32)
        padded[:, :K] = codes
        out = np.zeros((N, nw), dtype=np.uint32)
        for j in range(8):
            out |= padded[:, j::8] << np.uint32(4 * j)
        return out
    if bits == 2:
        nw = (K + 15) // 16
        padded = np.zeros((N, nw * 16), dtype=np.uint32)
        padded[:, :K] = codes
        out = np.zeros((N, nw), dtype=np.uint32)
        for j in range(16):
            out |= padded[:, j::16] << np.uint32(2 * j)
        return out
    assert bits == 3
    nb = (K + 31) // 32
    padded = np.zeros((N, nb * 32), dtype=np.uint64)
    padded[:, :K] = codes
    out = np.zeros((N, nb * 3), dtype=np.uint32)
    for b in range(nb):
        lo = np.zeros(N, dtype=np.uint64)                       # bits 0..62 of the block's 96-bit stream
        hi = np.zeros(N, dtype=np.uint64)                       # bits 63..95
        for j in range(32):
            c = padded[:, b * 32 + j]
            if j < 21:
                lo |= c << np.uint64(3 * j)
            else:
                hi |= c << np.uint64(3 * j - 63)
        full_lo = lo | ((hi & np.uint64(1)) << np.uint64(63))   # bits 0..63
        rest = hi >> np.uint64(1)                               # bits 64..95
        out[:, 3 * b] = (full_lo & np.uint64(0xFFFFFFFF)).astype(np.uint32)
        out[:, 3 * b + 1] = (full_lo >> np.uint64(32)).astype(np.uint32)
        out[:, 3 * b + 2] = (rest & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    return out


def unpack_codes(words, K, bits=4):
    N, nw = words.shape
    if bits == 4:
        out = np.zeros((N, nw * 8), dtype=np.uint8)
        for j in range(8):
            out[:, j::8] = (words >> np.uint32(4 * j)) & np.uint32(0xF)
        return out[:, :K]
    if bits == 2:
        out = np.zeros((N, nw * 16), dtype=np.uint8)
        for j in range(16):
            out[:, j::16] = (words >> np.uint32(2 * j)) & np.uint32(0x3)
        return out[:, :K]
    assert bits == 3 and nw % 3 == 0
    out = np.zeros((N, (nw // 3) * 32), dtype=np.uint8)
    w64 = words.astype(np.uint64)
    for k in range(out.shape[1]):
        bit = 3 * k
        w, off = bit // 32, bit % 32
        v = w64[:, w] >> np.uint64(off)
        if off > 29:                                            # the code continues in the next word
            v |= w64[:, w + 1] << np.uint64(32 - off)
        out[:, k] = (v & np.uint64(7)).astype(np.uint8)
    return out[:, :K]


def dequantize(codes, scales, zeros, group):
    """W' = (code - zero) * scale in fp64, [N, K]."""
    N, K = codes.shape
    g = np.arange(K) // group
    s = scales.astype(np.float64)[:, g]
    z = zeros.astype(np.float64)[:, g]
    return (codes.astype(np.float64) - z) * s


# --------------------------------------------------------------------------
# Router and selection (Eq. 2, Eq. 9; runtime ratio control, Sec. 3.4)
# --------------------------------------------------------------------------


def router_scores(x, w, b=0.0):
    """Execute-minus-bypass logit of every token: fp64 dot product rounded once to fp32.

    x [T, H] (values of a 16-bit dtype held in fp64), w [H] fp32, b scalar."""
    z = np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float32).astype(np.float64)
    z = z + np.float64(np.float32(b))
    return z.astype(np.float32)


def router_scores_mlp(x, W1, b1, W2, b2):
    """Two-output MLP router (Sec. 2.2: the router is a lightweight MLP with two outputs; Eq. 9 applies a
    softmax to them).  The paper states neither depth, width nor activation; this reading is one hidden
    layer with ReLU:  u = relu(W1 x + b1),  (l_e, l_b) = W2 u + b2,  and since the softmax over two classes
    gives p_0 = sigmoid(l_e - l_b), the score is z = l_e - l_b.  Everything in fp64, one rounding to fp32.

    x [T, H]; W1 [R, H], b1 [R], W2 [2, R], b2 [2], all fp32 parameters."""
    x = np.asarray(x, dtype=np.float64)
    W1 = np.asarray(W1, dtype=np.float32).astype(np.float64)
    b1 = np.asarray(b1, dtype=np.float32).astype(np.float64)
    W2 = np.asarray(W2, dtype=np.float32).astype(np.float64)
    b2 = np.asarray(b2, dtype=np.float32).astype(np.float64)
    u = np.maximum(x @ W1.T + b1, 0.0)
    logits = u @ W2.T + b2
    return (logits[:, 0] - logits[:, 1]).astype(np.float32)


def execute_probability(z):
    """p_0 of Eq. 9 for the two-class softmax over (z_e, z_b) with z = z_e - z_b."""
    z = np.asarray(z, dtype=np.float64)
    return 1.0 / (1.0 + np.exp(-z))


def theta_to_logit(theta):
    """The score z_thr with p_0 >= theta  <=>  z >= z_thr (sigmoid is strictly increasing).
    theta <= 0 executes everything, theta >= 1 nothing."""
    theta = float(theta)
    if math.isnan(theta):
        raise ValueError("theta is NaN")
    if theta <= 0.0:
        return np.float32(-np.inf)
    if theta >= 1.0:
        return np.float32(np.inf)
    return np.float32(math.log(theta / (1.0 - theta)))


def executed_count(r, T):
    """k = floor(r*T + 1/2) for the fp32 ratio r, computed in fp64, clamped to [0, T]."""
    r = float(np.float32(r))
    if math.isnan(r) or r < 0.0 or r > 1.0:
        raise ValueError("ratio outside [0, 1]")
    return int(min(T, max(0, math.floor(r * T + 0.5))))


def select_ratio(z, r):
    """Ratio mode: the k highest scores execute; equal scores go to the lower token index.
    Returns ascending int32 indices."""
    z = np.asarray(z, dtype=np.float32)
    T = z.shape[0]
    k = executed_count(r, T)
    order = sorted(range(T), key=lambda t: (-float(z[t]), t))
    return np.array(sorted(order[:k]), dtype=np.int32)


def select_threshold(z, theta):
    """Threshold mode (Eq. 9): execute iff p_0 >= theta, decided in the logit domain."""
    z = np.asarray(z, dtype=np.float32)
    zthr = theta_to_logit(theta)
    return np.nonzero(z >= zthr)[0].astype(np.int32)


# --------------------------------------------------------------------------
# Decoder layer pieces
# --------------------------------------------------------------------------


def rmsnorm(x, gain, eps):
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, dtype=np.float64)


def rope(v, pos, head_dim, base):
    """Rotary embedding, half-split pairing: element i pairs with i + d/2, angle pos * base^(-2i/d).
    v [..., n_heads*head_dim] for a single token at absolute position pos."""
    v = np.asarray(v, dtype=np.float64)
    d = head_dim
    out = v.reshape(-1, d).copy()
    i = np.arange(d // 2, dtype=np.float64)
    ang = float(pos) * np.power(float(base), -2.0 * i / d)
    c, s = np.cos(ang), np.sin(ang)
    a, b = out[:, : d // 2].copy(), out[:, d // 2:].copy()
    out[:, : d // 2] = a * c - b * s
    out[:, d // 2:] = b * c + a * s
    return out.reshape(v.shape)


def silu(a):
    return a / (1.0 + np.exp(-a))


class LayerParams:
    """Dequantized fp64 weights of one layer plus gains and router."""

    def __init__(self, Wq, Wk, Wv, Wo, Wg, Wu, Wd, g1, g2, router_w, router_b=0.0, router_mlp=None):
        self.Wq, self.Wk, self.Wv, self.Wo = Wq, Wk, Wv, Wo
        self.Wg, self.Wu, self.Wd = Wg, Wu, Wd
        self.g1 = np.asarray(g1, dtype=np.float64)
        self.g2 = np.asarray(g2, dtype=np.float64)
        self.router_w = np.asarray(router_w, dtype=np.float32)
        self.router_b = float(router_b)
        self.router_mlp = router_mlp        # None (linear router) or (W1, b1, W2, b2) of the two-output MLP


class KVCache:
    """Per-layer cache of executed tokens only: k, v [B, cap, n_kv*d] fp64, kv_len [B]."""

    def __init__(self, k, v, kv_len):
        self.k = np.array(k, dtype=np.float64)
        self.v = np.array(v, dtype=np.float64)
        self.kv_len = np.array(kv_len, dtype=np.int64)


def _seq_of(t, seq_offsets):
    for b in range(len(seq_offsets) - 1):
        if seq_offsets[b] <= t < seq_offsets[b + 1]:
            return b
    raise ValueError("token outside every sequence")


def decide(x, p, mode, control):
    """Scores and ascending executed indices for one layer."""
    if getattr(p, "router_mlp", None) is not None:
        z = router_scores_mlp(x, *p.router_mlp)
    else:
        z = router_scores(x, p.router_w, p.router_b)
    if mode == "ratio":
        idx = select_ratio(z, control)
    elif mode == "threshold":
        idx = select_threshold(z, control)
    elif mode == "forced":
        idx = np.array(sorted(int(i) for i in control), dtype=np.int32)
    else:
        raise ValueError(mode)
    return z, idx


def layer_forward(x, p, cfg, seq_offsets, positions, mode, control, kv=None):
    """One token-adaptive layer in the gather -> dense -> scatter form (App. B.2).

    x [T, H] fp64 (not modified).  cfg: dict with n_heads, n_kv_heads, head_dim, rms_eps,
    rope_base.  mode/control: ("ratio", r) | ("threshold", theta) | ("forced", indices).
    kv: optional KVCache of this layer, updated in place with the executed tokens.
    Returns (x_out [T, H] fp64, idx int32 ascending, z fp32 [T])."""
    x = np.asarray(x, dtype=np.float64)
    nh, nkv, d = cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    eps, base = cfg["rms_eps"], cfg["rope_base"]
    z, idx = decide(x, p, mode, control)
    out = x.copy()
    if len(idx) == 0:
        return out, idx, z
    xc = x[idx]                                        # gather
    n1 = rmsnorm(xc, p.g1, eps)
    q = n1 @ p.Wq.T
    k = n1 @ p.Wk.T
    v = n1 @ p.Wv.T
    for i, t in enumerate(idx):
        q[i] = rope(q[i], positions[t], d, base)
        k[i] = rope(k[i], positions[t], d, base)
    attn = np.zeros((len(idx), nh * d))
    B = len(seq_offsets) - 1
    rep = nh // nkv
    for b in range(B):
        rows = [i for i, t in enumerate(idx) if seq_offsets[b] <= t < seq_offsets[b + 1]]
        if not rows:
            continue
        kb, vb = k[rows], v[rows]
        n_old = 0
        if kv is not None:
            n_old = int(kv.kv_len[b])
            kb = np.concatenate([kv.k[b, :n_old], kb], axis=0)
            vb = np.concatenate([kv.v[b, :n_old], vb], axis=0)
        for h in range(nh):
            hk = h // rep
            qh = q[rows][:, h * d:(h + 1) * d]
            kh = kb[:, hk * d:(hk + 1) * d]
            vh = vb[:, hk * d:(hk + 1) * d]
            s = qh @ kh.T / math.sqrt(d)
            for i in range(len(rows)):                 # causal among executed tokens
                s[i, n_old + i + 1:] = -np.inf
            s = s - s.max(axis=1, keepdims=True)
            w = np.exp(s)
            w = w / w.sum(axis=1, keepdims=True)
            attn[rows, h * d:(h + 1) * d] = w @ vh
        if kv is not None:
            kv.k[b, n_old:n_old + len(rows)] = k[rows]
            kv.v[b, n_old:n_old + len(rows)] = v[rows]
            kv.kv_len[b] = n_old + len(rows)
    h1 = xc + attn @ p.Wo.T
    n2 = rmsnorm(h1, p.g2, eps)
    y = h1 + (silu(n2 @ p.Wg.T) * (n2 @ p.Wu.T)) @ p.Wd.T
    out[idx] = y                                       # scatter; other rows untouched
    return out, idx, z


def dense_layer_forward(x, p, cfg, seq_offsets, positions):
    """The plain (non-adaptive) quantized decoder layer on every token (Eq. 1), written
    separately from layer_forward so that "ratio 1.0 equals the dense layer" is a real check.
    No cache.  Processes one sequence at a time with full matrices."""
    x = np.asarray(x, dtype=np.float64)
    nh, nkv, d = cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    eps, base = cfg["rms_eps"], cfg["rope_base"]
    out = np.empty_like(x)
    half = d // 2
    inv_freq = np.power(float(base), -2.0 * np.arange(half, dtype=np.float64) / d)
    for b in range(len(seq_offsets) - 1):
        a, e = int(seq_offsets[b]), int(seq_offsets[b + 1])
        if e == a:
            continue
        xs = x[a:e]
        S = e - a
        n1 = xs / np.sqrt((xs ** 2).mean(axis=1, keepdims=True) + eps) * p.g1
        ang = np.asarray(positions[a:e], dtype=np.float64)[:, None] * inv_freq[None, :]
        cos, sin = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]

        def rot(m, heads):
            m = m.reshape(S, heads, d)
            lo, hi = m[..., :half], m[..., half:]
            return np.concatenate([lo * cos - hi * sin, hi * cos + lo * sin], axis=-1)

        q = rot(n1 @ p.Wq.T, nh)
        k = rot(n1 @ p.Wk.T, nkv)
        v = (n1 @ p.Wv.T).reshape(S, nkv, d)
        mask = np.triu(np.ones((S, S), dtype=bool), 1)
        ctx = np.empty((S, nh, d))
        for h in range(nh):
            hk = h // (nh // nkv)
            sc = q[:, h] @ k[:, hk].T / math.sqrt(d)
            sc[mask] = -np.inf
            sc = np.exp(sc - sc.max(axis=1, keepdims=True))
            ctx[:, h] = (sc / sc.sum(axis=1, keepdims=True)) @ v[:, hk]
        h1 = xs + ctx.reshape(S, nh * d) @ p.Wo.T
        n2 = h1 / np.sqrt((h1 ** 2).mean(axis=1, keepdims=True) + eps) * p.g2
        gate = n2 @ p.Wg.T
        out[a:e] = h1 + ((gate / (1.0 + np.exp(-gate))) * (n2 @ p.Wu.T)) @ p.Wd.T
    return out


def layer_forward_bruteforce(x, p, cfg, seq_offsets, positions, mode, control, kv=None):
    """Independent per-token form of the same layer: for every token decide; if executed,
    compute its own norm, q/k/v, loop over the earlier executed tokens of its sequence (and
    the cache) one key at a time, then the MLP.  Pure loops; tiny inputs only.
    Does not modify kv; returns (x_out, idx, appended) where appended[b] is the list of
    (k, v) rows sequence b would append."""
    x = np.asarray(x, dtype=np.float64)
    T, H = x.shape
    nh, nkv, d = cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    eps, base = cfg["rms_eps"], cfg["rope_base"]
    # decision per token
    z = [np.float32(sum(float(x[t, h]) * float(p.router_w[h]) for h in range(H)) + float(np.float32(p.router_b)))
         for t in range(T)]
    if mode == "ratio":
        k_exec = executed_count(control, T)
        executed = []
        for t in range(T):
            # rank of t: number of tokens that beat it (higher score, or equal score and lower index)
            beat = sum(1 for u in range(T) if (z[u] > z[t]) or (z[u] == z[t] and u < t))
            if beat < k_exec:
                executed.append(t)
    elif mode == "threshold":
        zthr = theta_to_logit(control)
        executed = [t for t in range(T) if z[t] >= zthr]
    else:
        executed = sorted(int(i) for i in control)
    exec_set = set(executed)

    def token_kv(t):
        n1 = rmsnorm(x[t], p.g1, eps)
        kk = rope(p.Wk @ n1, positions[t], d, base)
        vv = p.Wv @ n1
        return kk, vv

    out = x.copy()
    B = len(seq_offsets) - 1
    appended = [[] for _ in range(B)]
    for t in range(T):
        if t not in exec_set:
            continue
        b = _seq_of(t, seq_offsets)
        n1 = rmsnorm(x[t], p.g1, eps)
        q = rope(p.Wq @ n1, positions[t], d, base)
        keys, vals = [], []
        if kv is not None:
            for j in range(int(kv.kv_len[b])):
                keys.append(kv.k[b, j])
                vals.append(kv.v[b, j])
        for u in range(int(seq_offsets[b]), t + 1):
            if u in exec_set:
                ku, vu = token_kv(u)
                keys.append(ku)
                vals.append(vu)
        appended[b].append((keys[-1], vals[-1]))
        attn = np.zeros(nh * d)
        for h in range(nh):
            hk = h // (nh // nkv)
            qh = q[h * d:(h + 1) * d]
            logits = [float(np.dot(qh, kj[hk * d:(hk + 1) * d])) / math.sqrt(d) for kj in keys]
            m = max(logits)
            e = [math.exp(l - m) for l in logits]
            tot = sum(e)
            acc = np.zeros(d)
            for ej, vj in zip(e, vals):
                acc += (ej / tot) * vj[hk * d:(hk + 1) * d]
            attn[h * d:(h + 1) * d] = acc
        h1 = x[t] + p.Wo @ attn
        n2 = rmsnorm(h1, p.g2, eps)
        g = p.Wg @ n2
        u_ = p.Wu @ n2
        out[t] = h1 + p.Wd @ (np.array([gi / (1.0 + math.exp(-gi)) for gi in g]) * u_)
    return out, np.array(executed, dtype=np.int32), appended


def stack_forward(x, layers, cfg, seq_offsets, positions, mode, control, kvs=None, round_to=None):
    """L layers in sequence with the same control for every layer (one global knob, Sec. 3.4).

    round_to: optional function applied to the hidden state after every layer (e.g. rounding
    to the 16-bit activation dtype the GPU stores between layers).  Returns
    (x_out, [idx per layer], [layer inputs])."""
    x = np.asarray(x, dtype=np.float64)
    sel, inputs = [], []
    for l, p in enumerate(layers):
        inputs.append(x.copy())
        ctl = control[l] if mode == "forced" else control
        x, idx, _ = layer_forward(x, p, cfg, seq_offsets, positions, mode, ctl,
                                  None if kvs is None else kvs[l])
        if round_to is not None:
            x = round_to(x)
        sel.append(idx)
    return x, sel, inputs


# --------------------------------------------------------------------------
# Threshold calibration (Sec. 3.4: two-phase grid search for the global theta)
# --------------------------------------------------------------------------
# The paper searches theta in (0, 0.5] on a small calibration set, first with step 0.05, then with
# step 0.01 around the best coarse point, and keeps the theta with the best task metric.  Task
# metrics need the paper's datasets; here the objective is the one its rate loss trains for: the
# average execution ratio R_avg over layers should hit a target.  theta_n = fp32(n / 100), n = 1..50.

def theta_grid(n):
    return np.float32(n / 100.0)


def two_phase_search(ratio_of_n, target):
    """ratio_of_n(n) -> R_avg at theta_n.  Coarse pass over n = 5, 10, ..., 50; fine pass over the
    not-yet-evaluated n within 4 steps of the best coarse point (clipped to 1..50); the answer is the
    evaluated n with the smallest |R_avg - target|, ties going to the larger theta.
    Returns (n, R_avg(n), {n: R_avg} of everything evaluated, in evaluation order)."""
    target = float(target)
    seen = {}

    def best():
        return min(seen, key=lambda n: (abs(seen[n] - target), -n))

    for n in range(5, 51, 5):
        seen[n] = float(ratio_of_n(n))
    c = best()
    for n in range(max(1, c - 4), min(50, c + 4) + 1):
        if n not in seen:
            seen[n] = float(ratio_of_n(n))
    b = best()
    return b, seen[b], seen


def calibrate_theta_from_scores(scores, target):
    """scores: fp32 [L, T] router scores of a calibration batch, taken as fixed.  R_avg(theta) is the
    fraction of all L*T (layer, token) pairs with p_0 >= theta (Eq. 9)."""
    z = np.asarray(scores, dtype=np.float32)
    total = z.size

    def ratio(n):
        return int(np.count_nonzero(z >= theta_to_logit(theta_grid(n)))) / total

    n, r, seen = two_phase_search(ratio, target)
    return theta_grid(n), r, seen


def calibrate_theta(x, layers, cfg, seq_offsets, positions, target, round_to=None):
    """Same search with R_avg measured by running the stack in threshold mode on the calibration batch
    x for every candidate theta (skipping changes the hidden states that later routers see)."""
    T = np.asarray(x).shape[0]

    def ratio(n):
        _, sel, _ = stack_forward(x, layers, cfg, seq_offsets, positions, "threshold", theta_grid(n), round_to=round_to)
        return sum(len(i) for i in sel) / (len(layers) * T)

    n, r, seen = two_phase_search(ratio, target)
    return theta_grid(n), r, seen


def flops_per_token(hidden, n_heads, n_kv_heads, head_dim, inter, n_layers):
    """Dense linear FLOPs (2 per multiply-add) of one token through the full stack (App. B.1 table)."""
    per_layer = (hidden * n_heads * head_dim + 2 * hidden * n_kv_heads * head_dim
                 + n_heads * head_dim * hidden + 3 * hidden * inter)
    return 2 * per_layer * n_layers


def parity_error(got, want):
    """max_i |got_i - want_i| / max(|want_i|, rms(want row)) over a [rows, H] pair."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    if want.size == 0:
        return 0.0
    rms = np.sqrt(np.mean(want * want, axis=-1, keepdims=True))
    den = np.maximum(np.abs(want), rms)
    den = np.where(den == 0, 1.0, den)
    return float(np.max(np.abs(got - want) / den))
