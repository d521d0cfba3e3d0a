"""fp64 CPU oracle for the SPES MoE-layer hot path.  TEST INFRASTRUCTURE ONLY.

This file is the yardstick the device kernels are compared against.  It is a
plain, slow, definition-by-definition numpy implementation in float64; it shares
no code with the device path and must never be imported by the product package.
Only the tests, the smoke check and the benchmark's CPU-baseline leg use it.

What it follows (paper sections; equation numbers count displayed equations in
order of appearance):

* MoE block  MoE(x) = sum_j G_j(x) E_j(x)                      -- Sec. 3.1, Eq. 2
* softmax routing over all M experts, then top-k; drop-less     -- Sec. 3.2
* SwiGLU experts  E(x) = W_d ( SiLU(W_g x) * W_u x )            -- Sec. 3.2
* gate renormalisation over the chosen k (upcycled model)       -- Sec. 4 "Implementation details"
* only assigned experts (and shared modules, i.e. the router)
  receive parameter gradients; frozen experts still carry the
  input gradient                                                -- Sec. 3.3, Eq. 3; App. A, block mask U_i
* sparse synchronisation (average / direct assignment)          -- Sec. 3.3, Eq. 4; App. A sync rules
* expert-merging warm-up (cosine similarity, top-K, task
  arithmetic, all right-hand sides pre-merge)                   -- Sec. 3.3, Eq. 5-6; App. A merge step
* router auxiliary losses: load-balancing loss and router
  z-loss, with the coefficients of the implementation details   -- Sec. 3.3 "Training Losses"; App. B
* AdamW on the assigned experts and the shared parameters only
  (the "3 x |Phi_i|" of the memory model)                       -- Sec. 3.3 "Efficiency Analysis"; App. B, Table A1
* only the trained experts travel at a synchronisation           -- Sec. 3.3 (sparse synchronisation), Eq. 4
* upcycling: replicate one dense FFN, add Gaussian noise to a
  share of the parameters                                       -- Sec. 4 "upcycling settings"

Every function takes numpy arrays of already-rounded inputs and up-converts them
to float64; nothing is blocked, fused or reordered beyond "for each expert, the
rows routed to it".  Pins for each function live in tests/test_oracle_*.py; no
function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def _f64(a):
    return None if a is None else np.asarray(a, dtype=F64)


# ----------------------------------------------------------------------------
# routing: Sec. 3.2 (softmax routing, top-k, drop-less dispatch)
# ----------------------------------------------------------------------------


def router_logits(x, w_router, router_bias=None):
    """s[t,e] = <x_t, w_router_e> (+ bias_e).  x [T,d], w_router [M,d]."""
    s = _f64(x) @ _f64(w_router).T
    if router_bias is not None:
        s = s + _f64(router_bias)[None, :]
    return s


def softmax(s):
    """Row softmax over all M experts, with the row maximum subtracted first."""
    z = s - s.max(axis=1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=1, keepdims=True)


def top_k(s, k):
    """Indices of the k largest scores per row, in descending score order; ties go to the lower index."""
    order = np.argsort(-s, axis=1, kind="stable")   # stable: equal scores keep ascending index order
    return order[:, :k].astype(np.int32)


def gates(p, idx, renorm):
    """G_j(x) for the selected experts: the softmax probability, optionally renormalised over the k chosen."""
    g = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if renorm:
        g = g / g.sum(axis=1, keepdims=True)
    return g


def routing_tables(idx, M):
    """Drop-less dispatch tables for idx [T,k].

    count[e]  = number of routed (token, slot) pairs with expert e
    offset    = exclusive prefix sum of count, length M+1
    perm[r]   = flat pair index t*k+j held by row r of the expert-contiguous order
                (rows of one expert keep ascending flat index: a stable sort)
    inv[t*k+j]= row of that pair
    """
    flat = idx.reshape(-1).astype(np.int64)
    count = np.bincount(flat, minlength=M).astype(np.int32)
    offset = np.zeros(M + 1, dtype=np.int32)
    offset[1:] = np.cumsum(count)
    perm = np.argsort(flat, kind="stable").astype(np.int32)
    inv = np.empty_like(perm)
    inv[perm] = np.arange(perm.size, dtype=np.int32)
    return count, offset, perm, inv


# ----------------------------------------------------------------------------
# one SwiGLU expert on a block of rows: Sec. 3.2
# ----------------------------------------------------------------------------


def sigmoid(a):
    return 1.0 / (1.0 + np.exp(-a))


def expert_forward(x_rows, w_gate, w_up, w_down):
    """a = W_g x, b = W_u x, h = SiLU(a)*b, yp = W_d h  for every row of x_rows [n,d].

    w_gate, w_up are [f,d]; w_down is [d,f] (all stored [out,in]).
    """
    x_rows, w_gate, w_up, w_down = _f64(x_rows), _f64(w_gate), _f64(w_up), _f64(w_down)
    a = x_rows @ w_gate.T
    b = x_rows @ w_up.T
    h = a * sigmoid(a) * b
    yp = h @ w_down.T
    return a, b, h, yp


def expert_backward(x_rows, dyp_rows, a, b, h, w_gate, w_up, w_down):
    """Gradients of one expert for upstream dyp_rows [n,d].

    Returns dx_rows [n,d], dW_g [f,d], dW_u [f,d], dW_d [d,f].
    """
    x_rows, w_gate, w_up, w_down = _f64(x_rows), _f64(w_gate), _f64(w_up), _f64(w_down)
    dh = dyp_rows @ w_down                       # yp = h W_d^T
    sg = sigmoid(a)
    da = dh * b * sg * (1.0 + a * (1.0 - sg))    # d/da [a*sigmoid(a)] = sg*(1 + a*(1-sg))
    db = dh * a * sg
    dx_rows = da @ w_gate + db @ w_up
    d_w_down = dyp_rows.T @ h
    d_w_gate = da.T @ x_rows
    d_w_up = db.T @ x_rows
    return dx_rows, d_w_gate, d_w_up, d_w_down


# ----------------------------------------------------------------------------
# the layer: Eq. 2 forward, chain rule backward with the block mask of Eq. 3
# ----------------------------------------------------------------------------


def moe_forward(x, w_router, router_bias, w_gate, w_up, w_down, k, renorm, keep=True):
    """Forward of the routed feed-forward layer.

    Returns a dict with y [T,d], logits, p, idx [T,k], gate [T,k], count, offset,
    perm, inv, and (keep=True) per-pair intermediates a,b,h [T,k,f], yp [T,k,d]
    indexed by (token, slot).
    """
    x = _f64(x)
    T, d = x.shape
    M = w_router.shape[0]
    f = w_gate.shape[1]
    s = router_logits(x, w_router, router_bias)
    p = softmax(s)
    idx = top_k(s, k)
    g = gates(p, idx, renorm)
    count, offset, perm, inv = routing_tables(idx, M)
    a = np.zeros((T, k, f)); b = np.zeros((T, k, f)); h = np.zeros((T, k, f)); yp = np.zeros((T, k, d))
    for e in range(M):
        t_e, j_e = np.nonzero(idx == e)          # the pairs routed to expert e
        if t_e.size == 0:
            continue
        a_e, b_e, h_e, yp_e = expert_forward(x[t_e], w_gate[e], w_up[e], w_down[e])
        a[t_e, j_e], b[t_e, j_e], h[t_e, j_e], yp[t_e, j_e] = a_e, b_e, h_e, yp_e
    y = np.zeros((T, d))
    for j in range(k):                            # Eq. 2: weighted sum over the selected experts
        y += g[:, j:j + 1] * yp[:, j, :]
    out = dict(y=y, logits=s, p=p, idx=idx, gate=g, count=count, offset=offset, perm=perm, inv=inv)
    if keep:
        out.update(a=a, b=b, h=h, yp=yp)
    return out


def gating_backward(p, idx, gate, dgate, renorm):
    """dL/dlogits [T,M] from dL/dgate [T,k], following the forward order:
    softmax over all M -> pick k -> (optionally) divide by the sum of the picked."""
    T, M = p.shape
    dsel = dgate
    if renorm:
        S = np.take_along_axis(p, idx.astype(np.int64), axis=1).sum(axis=1, keepdims=True)
        # gate_j = p_j / S  =>  dL/dp_j = (dgate_j - sum_i dgate_i gate_i) / S
        dsel = (dgate - (dgate * gate).sum(axis=1, keepdims=True)) / S
    dp = np.zeros((T, M))
    np.put_along_axis(dp, idx.astype(np.int64), dsel, axis=1)
    return p * (dp - (dp * p).sum(axis=1, keepdims=True))


def router_aux_losses(logits, idx):
    """The two auxiliary router losses named in Sec. 3.3 "Training Losses" (the paper names them and cites their
    sources; the formulas are the cited ones, written out).

    load-balancing:  L_lb = M * sum_e f_e * P_e,  f_e = share of the T*k routed pairs that went to expert e,
                     P_e = mean over tokens of the softmax probability of expert e;
    router z-loss:   L_z  = mean over tokens of (log sum_e exp(logit_te))^2.
    Returns (L_lb, L_z, f [M], P [M]).
    """
    s = _f64(logits)
    T, M = s.shape
    k = idx.shape[1]
    f = np.zeros(M)
    for e in range(M):
        f[e] = np.count_nonzero(idx == e) / float(T * k)
    P = softmax(s).mean(axis=0)
    m = s.max(axis=1)
    lse = m + np.log(np.exp(s - m[:, None]).sum(axis=1))
    return float(M * (f * P).sum()), float((lse ** 2).mean()), f, P


def router_aux_dlogits(logits, idx, lb_coef, z_coef, grad_scale=1.0):
    """d/dlogits of grad_scale * (lb_coef * L_lb + z_coef * L_z).  The routed shares f_e are counts and carry no
    gradient; L_lb reaches the logits through P_e only."""
    s = _f64(logits)
    T, M = s.shape
    _, _, f, _ = router_aux_losses(s, idx)
    p = softmax(s)
    m = s.max(axis=1)
    lse = m + np.log(np.exp(s - m[:, None]).sum(axis=1))
    dP = lb_coef * M * f / T                                    # dL/dp_te, the same for every token
    d_lb = p * (dP[None, :] - (p * dP[None, :]).sum(axis=1, keepdims=True))
    d_z = z_coef * (2.0 / T) * lse[:, None] * p                 # d lse / d logit = p
    return grad_scale * (d_lb + d_z)


def moe_backward(fwd, dy, x, w_router, w_gate, w_up, w_down, renorm, wgrad_experts=None, extra_dlogits=None):
    """Backward of the layer given the forward record `fwd` (keep=True) and dy [T,d].
    `extra_dlogits` [T,M], if given, is added to the gating gradient before it reaches the router
    (the auxiliary router losses enter here).

    The selected index set is treated as constant.  Input gradients flow through
    every routed expert.  Weight gradients are returned per expert in dicts
    d_w_gate/d_w_up/d_w_down keyed by expert id, for the experts in
    `wgrad_experts` (default: all, so tests can compare any mask).
    """
    x, dy = _f64(x), _f64(dy)
    T, d = x.shape
    M = w_router.shape[0]
    idx, g = fwd["idx"], fwd["gate"]
    k = idx.shape[1]
    if wgrad_experts is None:
        wgrad_experts = range(M)
    wgrad_experts = set(int(e) for e in wgrad_experts)
    dgate = np.einsum("td,tjd->tj", dy, fwd["yp"])
    dx = np.zeros((T, d))
    dwg, dwu, dwd = {}, {}, {}
    for e in range(M):
        t_e, j_e = np.nonzero(idx == e)
        if t_e.size == 0:
            if e in wgrad_experts:
                f = w_gate.shape[1]
                dwg[e], dwu[e], dwd[e] = np.zeros((f, d)), np.zeros((f, d)), np.zeros((d, f))
            continue
        dyp_e = g[t_e, j_e][:, None] * dy[t_e]
        dx_e, dwg_e, dwu_e, dwd_e = expert_backward(
            x[t_e], dyp_e, fwd["a"][t_e, j_e], fwd["b"][t_e, j_e], fwd["h"][t_e, j_e],
            w_gate[e], w_up[e], w_down[e])
        np.add.at(dx, t_e, dx_e)
        if e in wgrad_experts:
            dwg[e], dwu[e], dwd[e] = dwg_e, dwu_e, dwd_e
    dlogits = gating_backward(fwd["p"], idx, g, dgate, renorm)
    if extra_dlogits is not None:
        dlogits = dlogits + _f64(extra_dlogits)
    d_w_router = dlogits.T @ x
    dx_experts = dx.copy()
    dx = dx + dlogits @ _f64(w_router)
    return dict(dx=dx, dx_experts=dx_experts, d_w_router=d_w_router, dgate=dgate, dlogits=dlogits,
                d_w_gate=dwg, d_w_up=dwu, d_w_down=dwd)


def expert_weight_grads(e, fwd_routing, dy, x, w_gate_e, w_up_e, w_down_e):
    """dW_g, dW_u, dW_d of the single expert e from routing results only (idx, gate).

    Lets a large configuration be checked one expert at a time: it recomputes the
    expert's forward on the rows routed to it and applies expert_backward.
    """
    idx, g = fwd_routing["idx"], fwd_routing["gate"]
    t_e, j_e = np.nonzero(idx == e)
    x_e = _f64(np.asarray(x)[t_e])
    a, b, h, _ = expert_forward(x_e, w_gate_e, w_up_e, w_down_e)
    dyp = g[t_e, j_e][:, None] * _f64(np.asarray(dy)[t_e])
    _, dwg, dwu, dwd = expert_backward(x_e, dyp, a, b, h, w_gate_e, w_up_e, w_down_e)
    return dwg, dwu, dwd


def expert_gate_grads(e, fwd_routing, dy, x, w_gate_e, w_up_e, w_down_e):
    """Gate gradients dgate[t,j] = <dy_t, E_e(x_t)> of the pairs routed to the single expert e (Eq. 2: the gate
    multiplies the expert's output), from routing results only.

    Returns (t_e, j_e, values): token and slot of each such pair and its gate gradient.  Visiting every expert fills
    the whole dgate [T,k] without keeping any per-pair intermediate, which is how a large configuration gets its
    router gradient checked.
    """
    idx = fwd_routing["idx"]
    t_e, j_e = np.nonzero(idx == e)
    _, _, _, yp = expert_forward(_f64(np.asarray(x)[t_e]), w_gate_e, w_up_e, w_down_e)
    return t_e, j_e, np.einsum("nd,nd->n", _f64(np.asarray(dy)[t_e]), yp)


# ----------------------------------------------------------------------------
# synchronisation: Eq. 4 and its generalisation to several / no trainers
# ----------------------------------------------------------------------------


def sync_merge(base, stores, slot, node_weight=None):
    """Global value of every expert after synchronisation.

    base [M,E]: previous global values.  stores[i] [n_i,E]: node i's trained
    experts; slot[i,j] = row of expert j in stores[i] or -1.  Expert j becomes the
    node_weight-weighted mean of its trainers' copies (uniform weights and every
    node training it: the FedAvg mean; a single trainer: direct assignment);
    with no trainer it keeps its previous value.  Returns (dst [M,E], trainer_count [M]).
    """
    base = _f64(base)
    M = base.shape[0]
    n_nodes = len(stores)
    w = np.ones(n_nodes) if node_weight is None else _f64(node_weight)
    dst = base.copy()
    trainer_count = np.zeros(M, dtype=np.int32)
    for j in range(M):
        num = np.zeros(base.shape[1])
        den = 0.0
        for i in range(n_nodes):                  # ascending node id
            s = int(slot[i][j])
            if s < 0:
                continue
            num += w[i] * _f64(stores[i][s])
            den += w[i]
            trainer_count[j] += 1
        if trainer_count[j] > 0:
            dst[j] = num / den
    return dst, trainer_count


# ----------------------------------------------------------------------------
# expert-merging warm-up: Eq. 5 (similarity), top-K peers, Eq. 6 (task arithmetic)
# ----------------------------------------------------------------------------


def cosine_similarity(w_in):
    """A[j,k] = <w_j, w_k> / (|w_j| |w_k|) over flattened input projections w_in [M,E] (Eq. 5).

    Eq. 5 is undefined when an input projection is all zeros; the reading taken here gives such a pair the
    similarity 0 (also on the diagonal), so a zero expert is nobody's preferred peer and everything stays finite."""
    w = _f64(w_in).reshape(w_in.shape[0], -1)
    G = w @ w.T
    n = np.sqrt(np.einsum("je,je->j", w, w))
    den = np.outer(n, n)
    return np.divide(G, den, out=np.zeros_like(G), where=den > 0)


def top_K_neighbours(A, K):
    """Q_j: the K experts most similar to j, j itself excluded; ties go to the lower index."""
    M = A.shape[0]
    B = A.copy()
    B[np.arange(M), np.arange(M)] = -np.inf
    return np.argsort(-B, axis=1, kind="stable")[:, :K].astype(np.int32)


def warmup_merge(phi, nbr, alpha):
    """phi~_j = phi_j + (alpha/K) sum_{k in Q_j} (phi_k - phi_j), every phi on the right pre-merge.

    phi [M,E] is one parameter matrix of all experts; call once per matrix with the same nbr.
    """
    phi = _f64(phi)
    M, K = nbr.shape
    out = np.empty_like(phi)
    for j in range(M):
        acc = np.zeros(phi.shape[1])
        for kk in nbr[j]:
            acc += phi[int(kk)] - phi[j]
        out[j] = phi[j] + (alpha / K) * acc
    return out


# ----------------------------------------------------------------------------
# optimizer step on the trainable subset: Sec. 3.3 "Efficiency Analysis" (gradients and the two AdamW
# moments exist only for the assigned experts and the shared parameters); hyper-parameters App. B, Table A1
# ----------------------------------------------------------------------------

def adamw_step(w, m, v, g, lr, beta1, beta2, eps, weight_decay, step, grad_scale=1.0):
    """One AdamW update (decoupled weight decay) of the arrays w, m, v with gradient grad_scale * g at step
    number `step` (1-based).  Returns new (w, m, v); nothing is rounded."""
    w, m, v, g = _f64(w), _f64(m), _f64(v), _f64(g) * grad_scale
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** step)
    v_hat = v / (1.0 - beta2 ** step)
    w = w - lr * (m_hat / (np.sqrt(v_hat) + eps) + weight_decay * w)
    return w, m, v


def masked_adamw(param, trainable, master, m, v, grad, **hyper):
    """The update applied to a full expert store: expert e = trainable[s] owns slot s of the compact arrays
    master/m/v/grad [n_trainable, ...]; every other expert is left untouched.  Returns (param, master, m, v) with
    param[e] = new master[s] (the caller rounds it to the storage type)."""
    param = _f64(param).copy()
    master, m, v = _f64(master).copy(), _f64(m).copy(), _f64(v).copy()
    for s_, e in enumerate(trainable):
        master[s_], m[s_], v[s_] = adamw_step(master[s_], m[s_], v[s_], grad[s_], **hyper)
        param[e] = master[s_]
    return param, master, m, v


# ----------------------------------------------------------------------------
# what a node uploads at a synchronisation: the rows of its trained experts, contiguous (Sec. 3.3, Eq. 4)
# ----------------------------------------------------------------------------

def pack_experts(store, trainable):
    """[n_trainable, ...] copy of the rows `trainable` (ascending expert ids) of the full store."""
    return np.asarray(store)[list(trainable)].copy()


def unpack_experts(store, trainable, packed):
    """The full store with the rows `trainable` replaced by `packed`; every other row unchanged."""
    out = np.asarray(store).copy()
    for s_, e in enumerate(trainable):
        out[e] = packed[s_]
    return out


# ----------------------------------------------------------------------------
# upcycling initialiser (Sec. 4 "upcycling settings": the dense FFN is replicated and Gaussian noise of standard
# deviation 0.02 is added to 50 % of the parameters).  The random draws are defined by a counter-based generator so
# that the device can reproduce them: Philox-4x64-10 (Salmon et al., SC'11) keyed by the seed, one call per group
# of four consecutive elements of the [M, elems] output.
# ----------------------------------------------------------------------------

_PHILOX_M0, _PHILOX_M1 = 0xD2E7470EE14C6C93, 0xCA5A826395121157
_PHILOX_W0, _PHILOX_W1 = 0x9E3779B97F4A7C15, 0xBB67AE8584CAA73B
_U64 = (1 << 64) - 1


def philox4x64(counter, key, rounds=10):
    """The Philox-4x64 bijection on one 256-bit counter (four Python ints) under a 128-bit key (two ints)."""
    c0, c1, c2, c3 = [int(c) & _U64 for c in counter]
    k0, k1 = [int(k) & _U64 for k in key]
    for _ in range(rounds):
        p0, p1 = _PHILOX_M0 * c0, _PHILOX_M1 * c2
        c0, c1, c2, c3 = ((p1 >> 64) ^ c1 ^ k0) & _U64, p1 & _U64, ((p0 >> 64) ^ c3 ^ k1) & _U64, p0 & _U64
        k0, k1 = (k0 + _PHILOX_W0) & _U64, (k1 + _PHILOX_W1) & _U64
    return c0, c1, c2, c3


def upcycle_draws(group_index, seed, stream_id):
    """Random draws for the four elements of group `group_index` (= flat element index // 4 of the [M, elems]
    output): returns (select_byte[4], normal[4]).

    One generator call with counter (group_index, stream_id, 0, 0) and key (seed, 0) yields four 64-bit words
    w_0..w_3.  Element j is selected iff the low byte of w_j is below fraction * 256.  The standard normals come from
    Box-Muller: elements 2q and 2q+1 are r cos(t) and r sin(t) with r = sqrt(-2 ln u1), t = 2 pi u2,
    u1 = (top 24 bits of w_{2q} + 0.5) / 2^24 and u2 = (top 24 bits of w_{2q+1} + 0.5) / 2^24.
    """
    w = philox4x64((group_index, stream_id, 0, 0), (seed, 0))
    sel = [x & 0xFF for x in w]
    z = []
    for q in range(2):
        u1 = ((w[2 * q] >> 40) + 0.5) / 16777216.0
        u2 = ((w[2 * q + 1] >> 40) + 0.5) / 16777216.0
        r = np.sqrt(-2.0 * np.log(u1))
        z += [r * np.cos(2.0 * np.pi * u2), r * np.sin(2.0 * np.pi * u2)]
    return sel, z


def upcycle_init(dense, n_experts, fraction, sigma, seed, stream_id=0):
    """out[e] = dense + select * sigma * z with the draws above; dense is one flattened matrix [elems] (elems a
    multiple of 4).  Nothing is rounded here."""
    dense = _f64(dense).ravel()
    elems = dense.size
    thr = int(np.floor(fraction * 256.0))
    out = np.empty((n_experts, elems))
    for e in range(n_experts):
        for g in range(elems // 4):
            sel, z = upcycle_draws((e * elems) // 4 + g, seed, stream_id)
            for j in range(4):
                i = 4 * g + j
                out[e, i] = dense[i] + (sigma * z[j] if sel[j] < thr else 0.0)
    return out
