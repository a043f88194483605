"""CPU oracle for the STEM token-indexed FFN layer — TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy statement of what the layer computes, written from
the paper's definition of the STEM layer (Method, "STEM", the equation
y = W_d (SiLU(W_g x) * U[t])) and of the two layers it is compared with: the
SwiGLU FFN (Background, first equation) and the additive variant (appendix
"STEM-dagger"), forward and backward (up_forward / up_backward).
It shares no code with the HIP path and imports nothing from it.  Only
tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import it;
the product never routes through it.

The paper prints no backward pass; the gradients below are the chain rule of
the forward equation and are pinned by finite differences in the tests.  The
optimiser is AdamW with the paper's stated hyper-parameters (Experiments,
"Training details" and the hyper-parameter table: weight decay 0.1,
beta1 0.9, beta2 0.95), applied only to the rows a batch touches.

Every function takes numpy arrays; floating inputs are used as fp64.  No
intermediate is rounded, except where a function says so (bf16 shadow of the
table, the residual stream of the stacked decode chain).

Pin status: every function here is pinned by tests/test_oracle_pins.py
(one-hot matmul forms, finite differences, torch autograd, the dense-SwiGLU
invariant, torch's AdamW, closed forms, brute force).  Nothing is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


# ----------------------------------------------------------------------------
# elementary pieces
# ----------------------------------------------------------------------------
def sigmoid(z: np.ndarray) -> np.ndarray:
    """Logistic function 1 / (1 + exp(-z)), evaluated without overflow."""
    z = np.asarray(z, dtype=np.float64)
    out = np.empty_like(z)
    pos = z >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-z[pos]))
    ez = np.exp(z[~pos])
    out[~pos] = ez / (1.0 + ez)
    return out


def silu(z: np.ndarray) -> np.ndarray:
    """SiLU(z) = z * sigmoid(z), the gate nonlinearity of SwiGLU (Background)."""
    return np.asarray(z, dtype=np.float64) * sigmoid(z)


def silu_prime(z: np.ndarray) -> np.ndarray:
    """d/dz [z sigmoid(z)] = sigmoid(z) (1 + z (1 - sigmoid(z)))."""
    s = sigmoid(z)
    return s * (1.0 + np.asarray(z, dtype=np.float64) * (1.0 - s))


def gather_rows(E: np.ndarray, ids: np.ndarray) -> np.ndarray:
    """U[t] for every token: row ids[i] of the per-layer table (Method, STEM)."""
    ids = np.asarray(ids)
    E = np.asarray(E)               # any float storage type; rows are widened on copy
    V = E.shape[0]
    if ids.size and (ids.min() < 0 or ids.max() >= V):
        raise IndexError("token id outside [0, V)")
    out = np.empty((ids.shape[0], E.shape[1]), dtype=np.float64)
    for i in range(ids.shape[0]):
        out[i, :] = E[int(ids[i]), :]
    return out


# ----------------------------------------------------------------------------
# forward  (Method, STEM equation)
# ----------------------------------------------------------------------------
def ffn_forward(x, ids, W_gate, W_down, E):
    """y_i = W_down (SiLU(W_gate x_i) * E[ids_i]) for every token i.

    x [T,d], ids [T], W_gate [F,d], W_down [d,F], E [V,F].
    Returns (y [T,d], dict with g, a, u, h [T,F]).
    """
    x = np.asarray(x, dtype=np.float64)
    Wg = np.asarray(W_gate, dtype=np.float64)
    Wd = np.asarray(W_down, dtype=np.float64)
    g = x @ Wg.T                      # gate pre-activation  W_g x
    a = silu(g)                       # SiLU(W_g x)
    u = gather_rows(E, ids)           # U[t]
    h = a * u                         # elementwise product
    y = h @ Wd.T                      # W_d ( . )
    return y, {"g": g, "a": a, "u": u, "h": h}


def swiglu_forward(x, W_gate, W_up, W_down):
    """Dense SwiGLU FFN  y = W_d (SiLU(W_g x) * (W_u x))  (Background, first equation)."""
    x = np.asarray(x, dtype=np.float64)
    g = x @ np.asarray(W_gate, dtype=np.float64).T
    up = x @ np.asarray(W_up, dtype=np.float64).T
    return (silu(g) * up) @ np.asarray(W_down, dtype=np.float64).T


def stem_dagger_forward(x, ids, W_gate, W_up, W_down, E):
    """Additive variant  y = W_d (SiLU(W_g x) * (W_u x + U[t]))  (appendix, STEM-dagger)."""
    x = np.asarray(x, dtype=np.float64)
    g = x @ np.asarray(W_gate, dtype=np.float64).T
    up = x @ np.asarray(W_up, dtype=np.float64).T
    return (silu(g) * (up + gather_rows(E, ids))) @ np.asarray(W_down, dtype=np.float64).T


# ----------------------------------------------------------------------------
# cost model (System Implementation, theoretical-efficiency table and "Training efficiency")
# ----------------------------------------------------------------------------
def train_flops_per_layer(B: int, L: int, d: int, d_ff: int, stem: bool) -> int:
    """Per-layer training FLOPs in the paper's units (forward + backward, element-wise work and
    biases ignored): attention 4 L d^2 + 2 L^2 d per sequence, FFN 3 L d d_ff for the dense
    SwiGLU layer and 2 L d d_ff when the up projection is replaced by the table."""
    return B * (4 * L * d * d + 2 * L * L * d + (2 if stem else 3) * L * d * d_ff)


def train_saving_fraction(d: int, d_ff: int, L: int) -> float:
    """(F_base - F_stem) / F_base = d_ff / (4 d + 2 L + 3 d_ff)."""
    base = train_flops_per_layer(1, L, d, d_ff, stem=False)
    return (base - train_flops_per_layer(1, L, d, d_ff, stem=True)) / base


def ffn_macs_per_token(d: int, d_ff: int, stem: bool) -> int:
    """Multiply-adds of one token's FFN forward: three d x d_ff projections, two with the table
    (efficiency table, prefill / training row, per token and without the element-wise term)."""
    return (2 if stem else 3) * d * d_ff


# ----------------------------------------------------------------------------
# backward  (chain rule of the STEM equation; not printed in the paper)
# ----------------------------------------------------------------------------
def ffn_backward(dy, x, ids, W_gate, W_down, E):
    """Gradients of L = sum_i <y_i, dy_i>.

    Returns dict: dx [T,d], dW_gate [F,d], dW_down [d,F], dU [T,F] (gradient with
    respect to each token's gathered row), dG [T,F].
    """
    dy = np.asarray(dy, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    Wg = np.asarray(W_gate, dtype=np.float64)
    Wd = np.asarray(W_down, dtype=np.float64)
    _, f = ffn_forward(x, ids, Wg, Wd, E)
    dh = dy @ Wd                      # W_d^T dy
    dU = dh * f["a"]                  # d/du of a*u
    da = dh * f["u"]                  # d/da of a*u
    dG = da * silu_prime(f["g"])
    dx = dG @ Wg                      # W_g^T dg
    dW_down = dy.T @ f["h"]           # sum_i dy_i h_i^T
    dW_gate = dG.T @ x                # sum_i dg_i x_i^T
    return {"dx": dx, "dW_gate": dW_gate, "dW_down": dW_down, "dU": dU, "dG": dG}


def up_forward(x, ids, W_gate, W_up, W_down, E=None):
    """FFN with an up projection: dense SwiGLU (E is None; Background, first equation) or the
    additive variant  y = W_d (SiLU(W_g x) * (W_u x + U[t]))  (appendix).

    Returns (y [T,d], dict g, up, v = up (+ gathered rows), h [T,F]).
    """
    x = np.asarray(x, dtype=np.float64)
    g = x @ np.asarray(W_gate, dtype=np.float64).T
    up = x @ np.asarray(W_up, dtype=np.float64).T
    v = up if E is None else up + gather_rows(E, ids)
    h = silu(g) * v
    return h @ np.asarray(W_down, dtype=np.float64).T, {"g": g, "up": up, "v": v, "h": h}


def up_backward(dy, x, ids, W_gate, W_up, W_down, E=None):
    """Gradients of L = sum_i <y_i, dy_i> for up_forward (chain rule; not printed in the paper).

    Returns dict: dx [T,d], dW_gate [F,d], dW_up [F,d], dW_down [d,F], dV [T,F] (gradient with
    respect to v = W_u x + U[t]: it is both the up projection's output gradient and, in the
    additive variant, the gradient of each token's gathered row), dG [T,F].
    """
    dy = np.asarray(dy, dtype=np.float64)
    x = np.asarray(x, dtype=np.float64)
    Wg = np.asarray(W_gate, dtype=np.float64)
    Wu = np.asarray(W_up, dtype=np.float64)
    Wd = np.asarray(W_down, dtype=np.float64)
    _, f = up_forward(x, ids, Wg, Wu, Wd, E)
    dh = dy @ Wd                       # W_d^T dy
    dV = dh * silu(f["g"])             # h = SiLU(g) * v
    dG = dh * f["v"] * silu_prime(f["g"])
    dx = dG @ Wg + dV @ Wu             # x feeds both projections
    return {"dx": dx, "dW_gate": dG.T @ x, "dW_up": dV.T @ x, "dW_down": dy.T @ f["h"], "dV": dV, "dG": dG}


# ----------------------------------------------------------------------------
# embedding gradient: sort -> unique -> offsets -> per-row sums
# ----------------------------------------------------------------------------
def sort_ids(ids):
    """Positions ordered by (id ascending, position ascending).

    Returns (sorted_ids [T] int32, perm [T] int32) with sorted_ids[k] = ids[perm[k]].
    """
    ids = np.asarray(ids, dtype=np.int64)
    perm = np.argsort(ids, kind="stable")
    return ids[perm].astype(np.int32), perm.astype(np.int32)


def unique_segments(sorted_ids):
    """Distinct ids ascending and where each one's run starts in sorted_ids.

    Returns (uniq_ids [U] int32, seg_offsets [U+1] int32), seg_offsets[U] = T.
    """
    s = np.asarray(sorted_ids, dtype=np.int64)
    T = s.shape[0]
    uniq, offs = [], []
    for k in range(T):
        if k == 0 or s[k] != s[k - 1]:
            uniq.append(int(s[k]))
            offs.append(k)
    offs.append(T)
    return np.asarray(uniq, dtype=np.int32), np.asarray(offs, dtype=np.int32)


def embed_grad(ids, dU):
    """dE[v,:] = sum over tokens i with ids[i] = v of dU[i,:], for touched v only.

    Returns dict: sorted_ids, perm, uniq_ids, seg_offsets, n_uniq and dE_rows [U,F]
    (row j belongs to table row uniq_ids[j]); rows of the table that no token names
    have zero gradient and are not represented.
    """
    dU = np.asarray(dU, dtype=np.float64)
    sorted_ids, perm = sort_ids(ids)
    uniq_ids, seg_offsets = unique_segments(sorted_ids)
    U = uniq_ids.shape[0]
    dE_rows = np.zeros((U, dU.shape[1]), dtype=np.float64)
    for j in range(U):
        for k in range(int(seg_offsets[j]), int(seg_offsets[j + 1])):
            dE_rows[j, :] += dU[int(perm[k]), :]
    return {"sorted_ids": sorted_ids, "perm": perm, "uniq_ids": uniq_ids,
            "seg_offsets": seg_offsets, "n_uniq": U, "dE_rows": dE_rows}


# ----------------------------------------------------------------------------
# sparse AdamW over touched rows
# ----------------------------------------------------------------------------
def bf16_round(a):
    """Round fp64/fp32 values to the nearest bfloat16 (ties to even); returns fp64.

    Done on the fp32 bit pattern: bfloat16 is the top 16 bits of an IEEE fp32.
    Values are first rounded to fp32 (the master copy of the table is fp32).
    """
    f = np.asarray(a, dtype=np.float32)
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = (bits + np.uint64(0x7FFF) + lsb) >> np.uint64(16)
    out = (rounded << np.uint64(16)).astype(np.uint32).view(np.float32)
    nan = np.isnan(f)
    out = np.where(nan, f, out)
    return out.astype(np.float64)


def sparse_adamw(uniq_ids, dE_rows, p, m, v, lr, beta1, beta2, eps, weight_decay, step):
    """One decoupled-weight-decay Adam step on rows uniq_ids of the table only.

    For a touched row r = uniq_ids[j], element-wise with g = dE_rows[j]:
        m <- beta1 m + (1-beta1) g ;  v <- beta2 v + (1-beta2) g^2
        mhat = m / (1-beta1^step) ;   vhat = v / (1-beta2^step)
        p <- p - lr*wd*p - lr * mhat / (sqrt(vhat) + eps)
    Rows not named keep p, m, v unchanged (no decay of any kind).  `step` >= 1 is
    the global step count.  Returns new (p, m, v) as fp64 copies of shape [V,F].
    """
    p = np.array(p, dtype=np.float64, copy=True)
    m = np.array(m, dtype=np.float64, copy=True)
    v = np.array(v, dtype=np.float64, copy=True)
    g_all = np.asarray(dE_rows, dtype=np.float64)
    c1 = 1.0 - beta1 ** step
    c2 = 1.0 - beta2 ** step
    for j, r in enumerate(np.asarray(uniq_ids)):
        r = int(r)
        g = g_all[j]
        m[r] = beta1 * m[r] + (1.0 - beta1) * g
        v[r] = beta2 * v[r] + (1.0 - beta2) * g * g
        mhat = m[r] / c1
        vhat = v[r] / c2
        p[r] = p[r] - lr * weight_decay * p[r] - lr * mhat / (np.sqrt(vhat) + eps)
    return p, m, v


def sparse_adamw_rows(dE_rows, p_rows, m_rows, v_rows, lr, beta1, beta2, eps, weight_decay, step):
    """Same update as sparse_adamw, on already-gathered rows (for large tables,
    where only the touched rows are brought to the host).  Returns (p, m, v) rows."""
    U = np.asarray(dE_rows).shape[0]
    return sparse_adamw(np.arange(U), dE_rows, p_rows, m_rows, v_rows,
                        lr, beta1, beta2, eps, weight_decay, step)


# ----------------------------------------------------------------------------
# host-resident table: token de-duplication for prefetch (System Implementation)
# ----------------------------------------------------------------------------
def dedup_remap(ids):
    """Distinct ids ascending and, per token, the slot of its id in that list."""
    ids = np.asarray(ids, dtype=np.int64)
    uniq = sorted(set(int(t) for t in ids))
    slot = {t: j for j, t in enumerate(uniq)}
    remap = np.asarray([slot[int(t)] for t in ids], dtype=np.int32)
    return np.asarray(uniq, dtype=np.int32), remap


class LfuRowCache:
    """Least-frequently-used cache of table rows kept on the device in host-resident mode
    (System Implementation: the hot rows stay in GPU memory, only misses are prefetched).

    The paper names the policy (LFU) and a hit rate, not its details; the reading taken:
    * freq[id] counts every token occurrence of id seen so far;
    * a batch's distinct ids are hits (row already in a cache slot) or misses; misses are
      numbered in order of first use and their rows go to the staging area behind the cache:
      remap[i] = slot (hit) or n_slots + miss number (miss);
    * after the batch, misses are offered to the cache in order (freq descending, id ascending):
      a free slot (lowest index first) is taken; otherwise the coldest cached row that this
      batch did not use (freq ascending, id ascending) is replaced if the candidate's freq is
      strictly larger; the first candidate that fails ends the update.
    """

    def __init__(self, vocab: int, n_slots: int):
        self.n_slots = int(n_slots)
        self.freq = np.zeros(int(vocab), dtype=np.int64)
        self.id_in_slot = [-1] * self.n_slots
        self.slot_of = {}

    def step(self, ids):
        """Returns (remap [T] int32, misses [n_miss] int32 in copy order, installs list of
        (id, slot, miss number))."""
        ids = [int(t) for t in np.asarray(ids, dtype=np.int64)]
        for t in ids:
            self.freq[t] += 1
        miss_no, misses, used = {}, [], set()
        remap = np.empty(len(ids), dtype=np.int32)
        for i, t in enumerate(ids):
            used.add(t)
            if t in self.slot_of:
                remap[i] = self.slot_of[t]
            else:
                if t not in miss_no:
                    miss_no[t] = len(misses)
                    misses.append(t)
                remap[i] = self.n_slots + miss_no[t]
        free = [s for s in range(self.n_slots) if self.id_in_slot[s] < 0]
        cold = sorted((int(self.freq[t]), t) for t in self.slot_of if t not in used)
        installs = []
        for t in sorted(misses, key=lambda t: (-int(self.freq[t]), t)):
            if free:
                slot = free.pop(0)
            elif cold and int(self.freq[t]) > cold[0][0]:
                _, victim = cold.pop(0)
                slot = self.slot_of.pop(victim)
            else:
                break
            self.id_in_slot[slot] = t
            self.slot_of[t] = slot
            installs.append((t, slot, miss_no[t]))
        return remap, np.asarray(misses, dtype=np.int32), installs


# ----------------------------------------------------------------------------
# knowledge editing: replacing the rows of a source entity's tokens by a target entity's
# (Experiments / appendix, "knowledge editing" of STEM embeddings)
# ----------------------------------------------------------------------------
EDIT_REPLACE, EDIT_PAD_LEFT, EDIT_COPY, EDIT_AVERAGE = 0, 1, 2, 3


def edit_target_index(n_s: int, n_t: int, mode: int):
    """For each of the n_s source positions, the index of the target token whose row replaces
    it; -1 = the padding token's row; None for EDIT_AVERAGE (every position gets the mean).

    EDIT_REPLACE: equal lengths, one to one.  EDIT_PAD_LEFT (n_s >= n_t): the target sequence
    padded on the left to n_s tokens.  EDIT_COPY (n_s >= n_t): every target token repeated
    floor(n_s / n_t) times and the last one repeated further to cover all n_s positions.
    """
    if n_s < 1 or n_t < 1:
        raise ValueError("both entities need at least one token")
    if mode == EDIT_AVERAGE:
        return None
    if mode == EDIT_REPLACE:
        if n_s != n_t:
            raise ValueError("one-to-one replacement needs equal token counts")
        return list(range(n_s))
    if n_s < n_t:
        raise ValueError("padding and copying need a source span at least as long as the target")
    if mode == EDIT_PAD_LEFT:
        return [-1] * (n_s - n_t) + list(range(n_t))
    if mode == EDIT_COPY:
        r = n_s // n_t
        out = []
        for k in range(n_t):
            out += [k] * r
        out += [n_t - 1] * (n_s - len(out))
        return out
    raise ValueError("unknown edit mode")


def edit_rows(E, src_ids, tgt_ids, mode: int, pad_id: int = 0, round_row=None):
    """Returns (edited copy of the table, the original rows of the source tokens).  All
    replacement rows are taken from the table as it was before the edit.  The mean of
    EDIT_AVERAGE is rounded by `round_row` (e.g. bf16_round) if given."""
    E = np.asarray(E, dtype=np.float64)
    src = [int(t) for t in src_ids]
    tgt = [int(t) for t in tgt_ids]
    idx = edit_target_index(len(src), len(tgt), mode)
    if idx is None:
        mean = E[tgt].sum(axis=0) / len(tgt)
        rows = np.tile(mean if round_row is None else round_row(mean), (len(src), 1))
    else:
        rows = np.stack([E[pad_id] if k < 0 else E[tgt[k]] for k in idx])
    out = E.copy()
    backup = E[src].copy()
    for j, t in enumerate(src):
        out[t] = rows[j]
    return out, backup


# ----------------------------------------------------------------------------
# stacked decode chain (several STEM layers joined by a residual stream)
# ----------------------------------------------------------------------------
def decode_chain(x0, ids, layers, round_stream=bf16_round):
    """x_{l+1} = round(x_l + y_l), y_l = STEM layer l applied to x_l, same ids at
    every layer (the table is indexed by token id, one vector per id per layer).
    `layers` is a list of (W_gate, W_down, E).  The residual stream is rounded to
    the storage type between layers, as the harness stores it; nothing else is.
    Returns the list [x_1, ..., x_N].
    """
    x = np.asarray(x0, dtype=np.float64)
    outs = []
    for (Wg, Wd, E) in layers:
        y, _ = ffn_forward(x, ids, Wg, Wd, E)
        x = round_stream(x + y)
        outs.append(x)
    return outs
