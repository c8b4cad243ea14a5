"""CPU oracle for the Symi MoE hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what one GPU's share of Symi's adaptive MoE
training step computes.  It exists to check the HIP library; the product path never
imports it (only tests, the smoke check and the bench's cpu_baseline leg may), and it
imports nothing from the HIP package.  Library primitives used as steps: numpy's
stable sort and matmul.

What each function follows
  router_forward, router_backward   Sec. 2.1: the learned gate network (a linear layer)
  route             Sec. 2.1 (top-k gating) and Sec. 3.2 step 1 (per-class token count)
  place             Appendix A.3, Algorithm 1 (Expert Placement Scheduler), Sec. 3.4
  dispatch          Sec. 3.2 step 2 (tokens of a class are spread over its replicas)
  slot_capacity, dispatch_capacity   Sec. 3.4: capacity(e_i) = slot_capacity * r_i; the
                    assignments of a class beyond its capacity are dropped
  moe_forward       Sec. 2.1: Y[t] = sum_j gate[t,j] * FFN_{idx[t,j]}(X[t]), SwiGLU FFN
  moe_backward      the derivative of that definition (Sec. 3.2 step 3 only changes
                    where the class gradient is summed, not its value)
  slot_gradients, replica_allreduce   Sec. 4.1 (Fig. 7): per-slot gradients, then
                    add into the representative slot, scale, copy back
  host_table, source_matrix, gradient_plan   App. A.4, Algorithm 2 (gradient collection plan), Sec. 4.3
  rank_group        Sec. 4.2 (groups of consecutive ranks)
  comm_cost         Sec. 3.3 (I)-(III), App. A.5: memory, data volume, communication time
  adam_step, adam_to_replicas   Sec. 3.2 steps 4-8: Adam on the static 1/N shard of
                    every class, then the weight write into next iteration's slots

Readings where the paper is silent (each is stated at its function):
  gate = softmax over all classes, top-k, optional renormalisation; ties go to the
  lower class index; a class's rows are split over its replicas in contiguous
  near-equal blocks in stable order; the gradient of a class is the plain sum over
  its rows times a caller-supplied scale; Adam has bias correction, eps outside the
  square root and decoupled weight decay; a shard is a contiguous range of the flat
  vector [W1 | W2] of a class; slot_capacity is rounded up to whole rows, the kept
  assignments of a class are its first ones in assignment order, a dropped assignment
  contributes nothing and the remaining gates are not renormalised.  These conventions
  have no external pin ("parity
  unpinned" beyond self-consistency); everything else is pinned in tests/ by brute
  force, invariants, closed forms, finite differences or library routines.
"""
import numpy as np

F64 = np.float64


# -------------------------------------------------------------------------- router
def router_forward(X, Wr, b=None):
    """logits[t,e] = <X[t], Wr[e]> + b[e]  (Sec. 2.1: the learned router), fp64."""
    z = np.asarray(X, dtype=F64) @ np.asarray(Wr, dtype=F64).T
    return z if b is None else z + np.asarray(b, dtype=F64)[None, :]


def router_backward(X, Wr, dlogits):
    """Gradients of the linear router: dWr = dlogits^T X, db = column sums, dX = dlogits Wr."""
    dl = np.asarray(dlogits, dtype=F64)
    return dl.T @ np.asarray(X, dtype=F64), dl.sum(axis=0), dl @ np.asarray(Wr, dtype=F64)


# --------------------------------------------------------------------------- route
def softmax_rows(logits):
    z = np.asarray(logits, dtype=F64)
    z = z - z.max(axis=1, keepdims=True)
    p = np.exp(z)
    return p / p.sum(axis=1, keepdims=True)


def route(logits, k, renorm=True):
    """Top-k routing (Sec. 2.1) + popularity histogram (Sec. 3.2 step 1).

    logits [T,E] (compared at the precision given: fp32 values are exact in fp64).
    Returns idx int32 [T,k] ordered by (score descending, class index ascending),
    gate fp64 [T,k], hist int64 [E] counting every (token, choice) pair.
    """
    z = np.asarray(logits, dtype=F64)
    T, E = z.shape
    order = np.argsort(-z, axis=1, kind="stable")  # stable: equal scores keep index order
    idx = order[:, :k].astype(np.int32)
    p = softmax_rows(z)
    gate = np.take_along_axis(p, idx.astype(np.int64), axis=1)
    if renorm:
        gate = gate / gate.sum(axis=1, keepdims=True)
    hist = np.bincount(idx.ravel(), minlength=E).astype(np.int64)
    return idx, gate, hist


def route_backward(logits, idx, gate, dgate, renorm=True):
    """dL/dlogits [T,E] given dL/dgate [T,k], through renormalisation and softmax."""
    z = np.asarray(logits, dtype=F64)
    p = softmax_rows(z)
    ii = idx.astype(np.int64)
    dg = np.asarray(dgate, dtype=F64)
    if renorm:
        psel = np.take_along_axis(p, ii, axis=1)
        ssum = psel.sum(axis=1, keepdims=True)
        dsel = (dg - (dg * np.asarray(gate, dtype=F64)).sum(axis=1, keepdims=True)) / ssum
    else:
        dsel = dg
    dp = np.zeros_like(p)
    np.put_along_axis(dp, ii, dsel, axis=1)
    return p * (dp - (dp * p).sum(axis=1, keepdims=True))


# --------------------------------------------------------------------------- place
def place(popularity, S_tot):
    """Algorithm 1 in exact integer arithmetic.

    goal_i = pop_i * S_tot / P is kept as a rational; diff_i = counts_i - goal_i is
    held as its numerator D_i = counts_i*P - pop_i*S_tot.  argmax / argmin take the
    first extremum.  An all-zero popularity (also: no previous iteration) is read as
    uniform.  Returns counts [E], placement [S_tot] (slot -> class, non-decreasing),
    first_slot [E+1].
    """
    pop = [int(x) for x in popularity]
    E = len(pop)
    S_tot = int(S_tot)
    if S_tot < E:
        raise ValueError("S_tot < E: every class needs one slot")
    if any(x < 0 for x in pop):
        raise ValueError("negative popularity")
    P = sum(pop)
    if P == 0:
        pop = [1] * E
        P = E
    counts = [max(1, (x * S_tot) // P) for x in pop]          # floor(maximum(goal, 1))
    D = [c * P - x * S_tot for c, x in zip(counts, pop)]       # diff * P
    while sum(counts) > S_tot:
        i = max(range(E), key=lambda j: (D[j], -j))             # first maximum
        if counts[i] > 1:
            counts[i] -= 1
        D[i] -= P
    while sum(counts) < S_tot:
        i = min(range(E), key=lambda j: (D[j], j))              # first minimum
        counts[i] += 1
        D[i] += P
    placement = []
    for e, c in enumerate(counts):
        placement += [e] * c
    first_slot = np.concatenate([[0], np.cumsum(counts)])
    return (np.array(counts, dtype=np.int32), np.array(placement, dtype=np.int32),
            first_slot.astype(np.int32))


# ------------------------------------------------------------------------ dispatch
def dispatch(idx, counts, first_slot):
    """Token -> replica permutation (Sec. 3.2 step 2).

    Assignment a = t*k + j has class idx[t,j].  Rows are the assignments in stable
    class order (class ascending, assignment id ascending inside a class).  Replica i
    of class e (slot first_slot[e]+i, r_e = counts[e] replicas, c_e rows starting at
    O_e) owns rows [O_e + floor(i*c_e/r_e), O_e + floor((i+1)*c_e/r_e)).
    Returns row_of_assign [A], assign_of_row [A], slot_offsets [S_tot+1] (int32).
    """
    cls = np.asarray(idx).ravel().astype(np.int64)
    A = cls.size
    E = len(counts)
    assign_of_row = np.argsort(cls, kind="stable").astype(np.int32)
    row_of_assign = np.empty(A, dtype=np.int32)
    row_of_assign[assign_of_row] = np.arange(A, dtype=np.int32)
    c = np.bincount(cls, minlength=E)
    O = np.concatenate([[0], np.cumsum(c)])
    S_tot = int(first_slot[E])
    slot_offsets = np.zeros(S_tot + 1, dtype=np.int32)
    for e in range(E):
        r = int(counts[e])
        for i in range(r):
            slot_offsets[int(first_slot[e]) + i] = O[e] + (i * int(c[e])) // r
    slot_offsets[S_tot] = A
    return row_of_assign, assign_of_row, slot_offsets


def slot_capacity(capacity_factor, A, S_tot):
    """Sec. 3.4: slot_capacity = capacity_factor * tokens_per_batch / (s*N) with
    tokens_per_batch = A assignments and s*N = S_tot slots, evaluated in binary64 in that
    order and rounded up to whole rows (at least one)."""
    x = np.float64(capacity_factor) * np.float64(A) / np.float64(S_tot)
    return max(1, int(np.ceil(x)))


def dispatch_capacity(idx, counts, first_slot, slot_cap):
    """dispatch under the capacity rule of Sec. 3.4: class e keeps at most
    slot_cap * counts[e] assignments, the first ones in assignment order.

    Returns row_of_assign [A] (-1 = dropped), assign_of_row [A'] (kept rows only),
    slot_offsets [S_tot+1] over the kept rows, keep [A] bool.  The survival rate of the
    iteration (Sec. 5.2) is A'/A.
    """
    cls = np.asarray(idx).ravel().astype(np.int64)
    A = cls.size
    E = len(counts)
    order = np.argsort(cls, kind="stable")           # assignments in stable class order
    c = np.bincount(cls, minlength=E)
    O = np.concatenate([[0], np.cumsum(c)])
    rank = np.empty(A, dtype=np.int64)                # position of an assignment inside its class
    rank[order] = np.arange(A) - O[cls[order]]
    cap = np.minimum(np.asarray(counts, dtype=np.int64) * int(slot_cap), A)
    keep = rank < cap[cls]
    ck = np.minimum(c, cap)                           # kept rows per class
    Ok = np.concatenate([[0], np.cumsum(ck)])
    row_of_assign = np.where(keep, Ok[cls] + rank, -1).astype(np.int32)
    assign_of_row = order[keep[order]].astype(np.int32)
    S_tot = int(first_slot[E])
    slot_offsets = np.zeros(S_tot + 1, dtype=np.int32)
    for e in range(E):
        r = int(counts[e])
        for i in range(r):
            slot_offsets[int(first_slot[e]) + i] = Ok[e] + (i * int(ck[e])) // r
    slot_offsets[S_tot] = Ok[E]
    return row_of_assign, assign_of_row, slot_offsets, keep


# ------------------------------------------------------------------------- forward
def silu(u):
    return u / (1.0 + np.exp(-u))


def sigmoid(u):
    return 1.0 / (1.0 + np.exp(-u))


def expert_ffn(x, W1_e, W2_e):
    """SwiGLU FFN of one class on rows x [n,d]: W1_e [2f,d] = gate rows | up rows, W2_e [d,f]."""
    f = W2_e.shape[1]
    u = x @ W1_e[:f].T
    v = x @ W1_e[f:].T
    h = silu(u) * v
    return h @ W2_e.T


def moe_forward(X, idx, gate, W1, W2):
    """Y[t] = sum_{j<k} gate[t,j] * FFN_{idx[t,j]}(X[t])  (j ascending), all in fp64.

    No slots, no permutation: replication changes where a token is processed, never
    what is computed.  W1 [E,2f,d], W2 [E,d,f].
    """
    X = np.asarray(X, dtype=F64)
    gate = np.asarray(gate, dtype=F64)
    T, d = X.shape
    k = idx.shape[1]
    E = W1.shape[0]
    Y = np.zeros((T, d), dtype=F64)
    for j in range(k):
        for e in range(E):
            sel = np.nonzero(idx[:, j] == e)[0]
            if sel.size == 0:
                continue
            y = expert_ffn(X[sel], np.asarray(W1[e], dtype=F64), np.asarray(W2[e], dtype=F64))
            Y[sel] += gate[sel, j][:, None] * y
    return Y


def moe_forward_pertoken(X, idx, gate, W1, W2):
    """The same definition as a pure per-token loop (small cases; pins moe_forward)."""
    X = np.asarray(X, dtype=F64)
    T, d = X.shape
    Y = np.zeros((T, d), dtype=F64)
    for t in range(T):
        for j in range(idx.shape[1]):
            e = int(idx[t, j])
            y = expert_ffn(X[t:t + 1], np.asarray(W1[e], dtype=F64), np.asarray(W2[e], dtype=F64))[0]
            Y[t] += float(gate[t, j]) * y
    return Y


# ------------------------------------------------------------------------ backward
def moe_backward(X, idx, gate, W1, W2, dY):
    """Gradients of L = sum(Y * dY) for the definition in moe_forward.

    Returns dX [T,d], dW1 [E,2f,d], dW2 [E,d,f], dgate [T,k] (fp64).  The class
    gradient is the plain sum over every assignment of the class.
    """
    X = np.asarray(X, dtype=F64)
    dY = np.asarray(dY, dtype=F64)
    gate = np.asarray(gate, dtype=F64)
    T, d = X.shape
    k = idx.shape[1]
    E = W1.shape[0]
    f = W2.shape[2]
    dX = np.zeros((T, d), dtype=F64)
    dW1 = np.zeros((E, 2 * f, d), dtype=F64)
    dW2 = np.zeros((E, d, f), dtype=F64)
    dgate = np.zeros((T, k), dtype=F64)
    for j in range(k):
        for e in range(E):
            sel = np.nonzero(idx[:, j] == e)[0]
            if sel.size == 0:
                continue
            Wg = np.asarray(W1[e, :f], dtype=F64)
            Wu = np.asarray(W1[e, f:], dtype=F64)
            Wd = np.asarray(W2[e], dtype=F64)
            x = X[sel]
            u = x @ Wg.T
            v = x @ Wu.T
            sg = sigmoid(u)
            h = u * sg * v
            y = h @ Wd.T
            dgate[sel, j] = (dY[sel] * y).sum(axis=1)
            dy = gate[sel, j][:, None] * dY[sel]
            dh = dy @ Wd
            du = dh * v * sg * (1.0 + u * (1.0 - sg))
            dv = dh * u * sg
            dW2[e] += dy.T @ h
            dW1[e, :f] += du.T @ x
            dW1[e, f:] += dv.T @ x
            dX[sel] += du @ Wg + dv @ Wu
    return dX, dW1, dW2, dgate


def slot_gradients(X, idx, gate, W1, W2, dY, row_of_assign, slot_offsets):
    """Weight gradient of every replica slot on its own: slot q holds the assignments whose
    row lies in [slot_offsets[q], slot_offsets[q+1]); its gradient is moe_backward's class
    gradient restricted to them.  Returns dW1 [S_tot,2f,d], dW2 [S_tot,d,f] (fp64)."""
    T, k = idx.shape
    S_tot = len(slot_offsets) - 1
    E, f = W1.shape[0], W2.shape[2]
    d = W2.shape[1]
    roa = np.asarray(row_of_assign).reshape(T, k)
    g1 = np.zeros((S_tot, 2 * f, d), dtype=F64)
    g2 = np.zeros((S_tot, d, f), dtype=F64)
    for q in range(S_tot):
        lo, hi = int(slot_offsets[q]), int(slot_offsets[q + 1])
        if hi == lo:
            continue
        mine = (roa >= lo) & (roa < hi)
        _, dW1, dW2, _ = moe_backward(X, idx, np.asarray(gate, dtype=F64) * mine, W1, W2, dY)
        e = int(idx[mine][0])                      # all rows of a slot belong to one class
        g1[q], g2[q] = dW1[e], dW2[e]
    return g1, g2


def replica_allreduce(g_slot, first_slot, scale=1.0):
    """Sec. 4.1 steps 1 and 3 on one rank: per class, the slots after the representative (the
    class's first slot) add their tensor to it, the sum is scaled ("normalized") and copied to
    every slot of the class.  Returns a new array."""
    out = np.array(g_slot, dtype=F64)
    for e in range(len(first_slot) - 1):
        q0, q1 = int(first_slot[e]), int(first_slot[e + 1])
        rep = out[q0].copy()
        for q in range(q0 + 1, q1):
            rep += out[q]
        rep *= scale
        for q in range(q0, q1):
            out[q] = rep
    return out


# ---------------------------------------------------------------------------- Adam
def adam_step(w, m, v, g, lr, beta1, beta2, eps, weight_decay, grad_scale, step):
    """Textbook Adam with bias correction (eps outside the root, decoupled decay)."""
    w = np.asarray(w, dtype=F64)
    m = np.asarray(m, dtype=F64)
    v = np.asarray(v, dtype=F64)
    g = grad_scale * np.asarray(g, dtype=F64)
    m2 = beta1 * m + (1.0 - beta1) * g
    v2 = beta2 * v + (1.0 - beta2) * g * g
    mhat = m2 / (1.0 - beta1 ** step)
    vhat = v2 / (1.0 - beta2 ** step)
    w2 = w - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * w)
    return w2, m2, v2


def round_to_bf16(x):
    """Round fp32 values to the nearest bf16 (ties to even); returns fp32 holding bf16 values."""
    a = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    bits = a.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    return (rounded & 0xFFFFFFFF).astype(np.uint32).view(np.float32).reshape(a.shape)


def shard_range(P_e, N, n):
    """Flat range of the class vector [W1 | W2] owned by optimizer partition n of N."""
    per = P_e // N
    return n * per, (n + 1) * per


def adam_to_replicas(dW1, dW2, master_w, m, v, placement_next, N, n, hp, bf16,
                     W1_slots, W2_slots):
    """Steps 4-8 of Sec. 3.2 for optimizer partition n.

    dW1 [E,2f,d], dW2 [E,d,f]: class gradients.  master_w, m, v [E, P_e/N]: this
    partition's fp32-valued state.  Every slot q of placement_next receives, on the
    flat range of partition n, the fresh weights of class placement_next[q] (rounded to
    bf16 from their fp32 value when bf16 is set).  W1_slots [S,2f,d] and W2_slots
    [S,d,f] are modified in place; returns the new (master_w, m, v) in fp64.
    """
    E = dW1.shape[0]
    n1 = dW1[0].size
    P_e = n1 + dW2[0].size
    lo, hi = shard_range(P_e, N, n)
    g = np.concatenate([np.asarray(dW1, dtype=F64).reshape(E, -1),
                        np.asarray(dW2, dtype=F64).reshape(E, -1)], axis=1)[:, lo:hi]
    w2, m2, v2 = adam_step(master_w, m, v, g, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"],
                           hp["weight_decay"], hp["grad_scale"], hp["step"])
    fresh = w2.astype(np.float32)
    if bf16:
        fresh = round_to_bf16(fresh)
    S = len(placement_next)
    flat1 = W1_slots.reshape(S, -1)
    flat2 = W2_slots.reshape(S, -1)
    for q in range(S):
        e = int(placement_next[q])
        a, b = lo, min(hi, n1)
        if a < b:
            flat1[q, a:b] = fresh[e, a - lo:b - lo]
        a, b = max(lo, n1), hi
        if a < b:
            flat2[q, a - n1:b - n1] = fresh[e, a - lo:b - lo]
    return w2, m2, v2


# ------------------------------------------------------- multi-rank planning (host side)
def host_table(placement, N, E):
    """hosted [E,N] bool: rank r holds at least one replica slot of class e.  Slot q lives on
    rank q // s, s = S_tot / N (Sec. 4.1: slots are numbered rank by rank)."""
    pl = np.asarray(placement, dtype=np.int64)
    s = len(pl) // N
    hosted = np.zeros((E, N), dtype=bool)
    hosted[pl, np.arange(len(pl)) // s] = True
    return hosted


def source_matrix(placement, N, E):
    """App. A.4 (Algorithm 2), Sec. 4.3, for all (class, destination) pairs at once:
    src[e, r] = the one rank that supplies class e's gradient shard to the optimizer
    partition on rank r.  A rank that hosts the class serves itself (local first); every other
    destination r is served by the hosting rank number (r mod #hosts) of the ascending list of
    hosting ranks, so the hosts share the remote destinations in turn."""
    hosted = host_table(placement, N, E)
    dest = np.arange(N)
    src = np.empty((E, N), dtype=np.int64)
    for e in range(E):
        ranks = np.flatnonzero(hosted[e])
        src[e] = np.where(hosted[e], dest, ranks[dest % len(ranks)])
    return src


def gradient_plan(placement, N, E, rank):
    """What `rank` receives and sends in one gradient collection (App. A.4): recv_src [E] =
    column `rank` of the source matrix; send = {class hosted on rank: ascending destinations
    whose partition this rank serves} (the partition index equals the destination rank)."""
    src = source_matrix(placement, N, E)
    hosted = host_table(placement, N, E)
    send = {e: np.flatnonzero(src[e] == rank).tolist() for e in range(E) if hosted[e, rank]}
    return src[:, rank].copy(), send


def rank_group(N, first_rank, last_rank):
    """Sec. 4.2: position of the group {first_rank..last_rank} among all groups of two or more
    consecutive ranks, listed by first rank and then by last rank (N(N-1)/2 of them)."""
    groups = [(a, b) for a in range(N) for b in range(a + 1, N)]
    return groups.index((first_rank, last_rank))


def comm_cost(E, N, s, G, W, O, bw_pci, bw_net, placement_counts=None):
    """Sec. 3.3.  (I) memory E*(1/r)*r*O vs E*(1/N)*N*O; (II) data moved, for Symi summed
    over the actual replica counts r_i (default: any counts summing to s*N); (III) per-rank
    time of the gradient and the weight phase; extra = (T_symi - T_static) / T_static."""
    from fractions import Fraction as Fr
    E_, N_, s_ = Fr(E), Fr(N), Fr(s)
    G_, W_, O_ = Fr(G), Fr(W), Fr(O)
    r = s_ * N_ / E_                                  # static replication degree, eq. (1)
    counts = [Fr(int(c)) for c in placement_counts] if placement_counts is not None else [r] * int(E)
    assert sum(counts) == s_ * N_                     # eq. (2)
    inf = bw_pci == float("inf")
    pci = None if inf else Fr(bw_pci)
    net = Fr(bw_net)
    out = {
        "mem_static": E_ * (1 / r) * r * O_,
        "mem_symi": E_ * (1 / N_) * N_ * O_,
        "data_grad_static": E_ * r * (G_ / r) * r,
        "data_weight_static": E_ * r * (W_ / r) * r,
        "data_grad_symi": sum(ri * (G_ / N_) * N_ for ri in counts),
        "data_weight_symi": sum(N_ * (W_ / N_) * ri for ri in counts),
    }
    for nm, X in (("grad", G_), ("weight", W_)):
        host = 0 if inf else E_ / N_ * X / pci
        out[f"t_{nm}_static"] = host + (s_ * N_ - E_) / N_ * X / net
        out[f"t_{nm}_symi"] = host + (s_ * N_ - s_) / N_ * X / net
    ts = out["t_grad_static"] + out["t_weight_static"]
    out["extra_fraction"] = (out["t_grad_symi"] + out["t_weight_symi"] - ts) / ts
    return {k: float(v) for k, v in out.items()}
