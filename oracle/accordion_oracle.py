"""CPU oracle for the Accordion gradient-compression hot path (arxiv 2010.16248).

TEST INFRASTRUCTURE ONLY.  This file is a plain, slow, obviously-correct numpy
statement of what the path computes.  It is imported by the tests, by the smoke
check and by the benchmark's cpu_baseline leg, and by nothing else; the product
(the HIP library and its binding) shares no code with it and never calls it.

What is computed, and where the paper defines it
------------------------------------------------
* Distributed SGD with a compressor C(., l) and the mean over workers:
  Section 3, "Distributed SGD with adaptive gradient compression".
* Error feedback ("memory term"): Section 5.3 and Appendix A, "Hyperparameters":
  the part of (gradient + memory) that the compressor dropped is the next memory.
* PowerSGD: Section 5 names it (low-rank factorisation per layer, "with memory
  term" in Appendix A) and prints no listing; one warm-started subspace iteration
  per step: P = M Q, orthogonalise P, Q = M^T P, decompress P Q^T, with
  M = gradient + memory.  1-D tensors are not compressed
  (appendix "Compression Ratio Selection").
* TopK: Section 5, "choosing the K entries with largest absolute values"; per
  gradient tensor (Section 1).  Ties go to the lower flat index.
* Accumulated per-layer gradient, its norm, the critical-regime test and the two
  levels: Section 4.2 (equation and Algorithm 1), "Computational and memory
  overhead".
* Batch-size mode (Section 3 "Distributed SGD with adaptive batch size"; Section
  4.2: the same algorithm switching B_low / B_high on the gradient of the whole
  model; Section 5.1 "Hyperparameters": learning rate scaled in the same ratio;
  Appendix A "Additional Details for Batch Size experiment": the large batch is
  several backward passes accumulated before one exchange, and the batch size is
  only allowed to grow).
* Overlap of the Top-K supports of two stochastic gradients: Section 4.3
  ("Relationship between gradient compression and adaptive batch-size").
* The comparison detector (Section 5.6 "Comparison with Prior Work"): the mean to
  standard deviation ratio (MSDR) of the gradients; when it has dropped by a given
  fraction the compression is reduced.
* The optimizer that consumes the averaged decompressed gradient: SGD with
  Nesterov momentum 0.9 (Appendix A, table "Hyperparameters") applied to the
  update rule of Section 3.

Precision: operands and stored state are fp32 (the paper's implementation is
fp32 PyTorch); every contraction, norm and orthogonalisation is evaluated in fp64
on those fp32 operands and rounded to fp32 where it is stored.  The error-feedback
add, the TopK comparison and the regime decision are taken in fp32, because they
decide integers (which entries are kept, which level is used) and both sides must
decide in the same precision.

The optimizer update is taken in fp32, one rounding per multiplication and per
addition, in the order written in nesterov_update.

The MSDR rule is this build's reading of the one sentence the paper spends on the
comparison method (see msdr_should_switch): "parity unpinned" for the rule; the
statistic itself is pinned.

Pins: tests/test_oracle_*.py check every function below against brute force on
tiny inputs, library QR/SVD, closed forms, the paper's printed "Data Sent"
columns and hand-written decision sequences.  The choice of k from a percentage
(ceil) and the start-critical convention have no printed value to pin against:
"parity unpinned" for those two conventions (they are documented readings).
"""
from __future__ import annotations

import math
from typing import List, Sequence, Tuple

import numpy as np

F32 = np.float32
F64 = np.float64

POWERSGD = 0
TOPK = 1


# ---------------------------------------------------------------------------
# elementary pieces
# ---------------------------------------------------------------------------

def ef_add(g: np.ndarray, e: np.ndarray) -> np.ndarray:
    """Delta = gradient + error memory, one fp32 add per element
    (Section 5.3 "with error-feedback"; Appendix A "with memory term")."""
    return (g.astype(F32) + e.astype(F32)).astype(F32)


def k_from_fraction(n: int, num: int, den: int) -> int:
    """Kept count for "K = num/den of the entries" (Section 5): the paper does not
    say how a fractional count is rounded; reading: ceil, at least 1."""
    return max(1, -((-int(n) * int(num)) // int(den)))


def effective_rank(rank: int, rows: int, cols: int) -> int:
    """A rank above min(rows, cols) cannot be used; it is capped."""
    return max(1, min(int(rank), int(rows), int(cols)))


def gram_schmidt(p: np.ndarray) -> np.ndarray:
    """Orthonormalise the columns of P in order (modified Gram-Schmidt):
    column i has its components along the finished columns j < i removed one after
    the other, then is scaled to unit length; a column of zero length stays zero."""
    a = p.astype(F64).copy()
    r = a.shape[1]
    for i in range(r):
        for j in range(i):
            a[:, i] -= np.dot(a[:, j], a[:, i]) * a[:, j]
        nrm = math.sqrt(float(np.dot(a[:, i], a[:, i])))
        if nrm > 0.0:
            a[:, i] /= nrm
        else:
            a[:, i] = 0.0
    return a.astype(F32)


def powersgd_layer(deltas: Sequence[np.ndarray], q: np.ndarray):
    """One PowerSGD round for one layer over W workers.

    deltas: W matrices (n x m, fp32) = gradient + memory of each worker.
    q:      m x r right factor from the previous step (fp32).
    Returns (P_hat n x r, Q_bar m x r, D n x m), all fp32:
      P_w = Delta_w Q;  P_bar = mean_w P_w;  P_hat = orthonormalised P_bar;
      Q_w = Delta_w^T P_hat;  Q_bar = mean_w Q_w;  D = P_hat Q_bar^T.
    The two means are what the all-reduce produces (Section 5.1 "Implementation")
    together with the 1/N of the update rule (Section 3)."""
    w = len(deltas)
    q64 = q.astype(F64)
    p_w = [(d.astype(F64) @ q64).astype(F32) for d in deltas]
    p_bar = (sum(p.astype(F64) for p in p_w) / w).astype(F32)
    p_hat = gram_schmidt(p_bar)
    ph64 = p_hat.astype(F64)
    q_w = [(d.astype(F64).T @ ph64).astype(F32) for d in deltas]
    q_bar = (sum(x.astype(F64) for x in q_w) / w).astype(F32)
    d_out = (ph64 @ q_bar.astype(F64).T).astype(F32)
    return p_hat, q_bar, d_out


def topk_select(delta: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    """The k entries of a flat fp32 tensor with the largest absolute value
    (Section 5).  Order: |value| descending, compared on the fp32 bit pattern with
    the sign cleared (so +0 and -0 tie); equal magnitudes: lower flat index first.
    Returns (indices ascending, int32; values = the untouched entries, fp32)."""
    flat = np.ascontiguousarray(delta, dtype=F32).reshape(-1)
    key = (flat.view(np.uint32) & np.uint32(0x7FFFFFFF)).astype(np.int64)
    order = np.argsort(-key, kind="stable")      # stable: ties keep index order
    kept = np.sort(order[:k]).astype(np.int32)
    return kept, flat[kept].copy()


def topk_residual(delta: np.ndarray, kept: np.ndarray) -> np.ndarray:
    """Error memory after TopK: zero where an entry was sent, Delta elsewhere."""
    e = np.array(delta, dtype=F32).reshape(-1).copy()
    e[kept] = F32(0.0)
    return e


def payload_layout(n: int, kept: np.ndarray, values: np.ndarray):
    """What one worker sends for a layer of n entries of which `kept` (ascending indices) are
    kept.  The paper's own levels keep K = 99 % inside critical regimes (Section 5.4, TopK
    tables); a list of (index, value) pairs then costs 1.98 n floats, more than the dense
    tensor.  So: at most half kept -> ("index_value", indices, values), 2k words; more than
    half kept -> ("values_holes", indices of the dropped entries ascending, values in index
    order), n words.  The selection itself is the same in both."""
    k = int(len(kept))
    if 2 * k <= int(n):
        return "index_value", np.asarray(kept, np.int32), np.asarray(values, F32)
    mask = np.ones(int(n), dtype=bool)
    mask[kept] = False
    return "values_holes", np.flatnonzero(mask).astype(np.int32), np.asarray(values, F32)


def payload_words_packed(n: int, k: int) -> int:
    """Floats (or 4-byte indices) in payload_layout's message."""
    return 2 * int(k) if 2 * int(k) <= int(n) else int(n)


def payload_decode(n: int, layout):
    """(indices, values) of the kept entries from either layout."""
    kind, idx, values = layout
    if kind == "index_value":
        return idx, values
    mask = np.ones(int(n), dtype=bool)
    mask[idx] = False
    return np.flatnonzero(mask).astype(np.int32), values


def support_overlap(idx_a: np.ndarray, idx_b: np.ndarray) -> int:
    """Number of coordinates two kept-index sets have in common (Section 4.3: the overlap in
    coordinates of the Top-10 % entries of a pair of stochastic gradients).  The overlap
    fraction the paper plots is this count over k."""
    return int(np.intersect1d(np.asarray(idx_a), np.asarray(idx_b), assume_unique=True).size)


def sparse_mean(n: int, payloads: Sequence[Tuple[np.ndarray, np.ndarray]], n_workers: int) -> np.ndarray:
    """Dense mean of W sparse payloads (the all-gather of Section 5.1 followed by
    the 1/N sum of Section 3).  Taken in fp32, workers in order 0..W-1 starting
    from +0, then one division by W, so that the result has one definite value."""
    acc = np.zeros(n, dtype=F32)
    for idx, val in payloads:
        acc[idx] = (acc[idx] + val.astype(F32)).astype(F32)
    return (acc / F32(n_workers)).astype(F32)


def layer_norm(a: np.ndarray) -> np.float32:
    """l2 norm of one layer's accumulated gradient (Section 4.2, "Computational and
    memory overhead"), summed in fp64 and stored as fp32."""
    x = a.astype(F64).reshape(-1)
    return F32(math.sqrt(float(np.dot(x, x))))


def msdr(grads: Sequence[np.ndarray]) -> np.float32:
    """Mean to standard deviation ratio of T gradients of one layer (Section 5.6), written
    out as the definition: || mean_t g_t ||_2 over sqrt( mean_t || g_t - mean ||_2^2 ), in
    fp64 on the fp32 inputs; +inf when the gradients do not vary at all."""
    g = np.stack([np.asarray(x, dtype=F64).reshape(-1) for x in grads])
    mean = g.mean(axis=0)
    var = float(np.mean(np.sum((g - mean) ** 2, axis=1)))
    num = math.sqrt(float(np.dot(mean, mean)))
    return F32(np.inf) if var <= 0.0 else F32(num / math.sqrt(var))


def msdr_streaming(sum_vec: np.ndarray, sum_sq: float, t: int) -> np.float32:
    """The same ratio from what a detector can keep without storing the gradients: the
    element-wise sum of the T gradients (the accumulator of Section 4.2), the sum of their
    squared norms and T:  mean_t ||g_t - m||^2 = (sum_t ||g_t||^2) / T - ||m||^2."""
    a = np.asarray(sum_vec, dtype=F64).reshape(-1)
    mu2 = float(np.dot(a, a)) / (float(t) * float(t))
    var = float(sum_sq) / float(t) - mu2
    return F32(np.inf) if var <= 0.0 else F32(math.sqrt(mu2 / var))


def msdr_should_switch(ref, m, has_ref: bool, delta) -> bool:
    """Reading of Section 5.6's description of the comparison method: once the ratio has
    dropped by the fraction delta relative to its value at the last switch (or at the first
    window), the layer moves to the more accurate level, and it never moves back.  fp32."""
    if not has_ref:
        return False
    return bool(F32(m) <= F32(F32(F32(1.0) - F32(delta)) * F32(ref)))


def regime_is_critical(old, curr, has_old: bool, eta, lr_curr, lr_next) -> bool:
    """Algorithm 1 / the Section 4.2 criterion, in fp32:
    critical  <=>  | ||D_old|| - ||D_curr|| | / ||D_old|| >= eta   or   lr_next < lr_curr.
    Readings where the paper is silent: no previous norm yet, or a previous norm of
    zero (the ratio is undefined) => critical, as early training is."""
    if F32(lr_next) < F32(lr_curr):
        return True
    if not has_old:
        return True
    old = F32(old)
    curr = F32(curr)
    if old == F32(0.0):
        return True
    ratio = F32(np.abs(F32(old - curr))) / old
    return bool(F32(ratio) >= F32(eta))


def nesterov_update(w: np.ndarray, v: np.ndarray, d: np.ndarray, lr, momentum,
                    weight_decay=0.0) -> Tuple[np.ndarray, np.ndarray]:
    """One step of SGD with Nesterov momentum on the averaged decompressed gradient d
    (Appendix A, table "Hyperparameters": optimizer Nesterov, momentum 0.9; Section 3:
    w_{k+1} = w_k - gamma_k * mean_i C(g_i), here with the momentum term):

        d' = d + lambda * w          (only if lambda != 0; the paper names no weight decay)
        v  = mu * v + d'             (velocity, zero before the first step)
        w  = w - gamma * (d' + mu * v)

    Every product and every sum is rounded to fp32 on its own, in this order.
    Returns (w, v) after the step."""
    w = np.asarray(w, dtype=F32)
    v = np.asarray(v, dtype=F32)
    d = np.asarray(d, dtype=F32)
    lr, mu, lam = F32(lr), F32(momentum), F32(weight_decay)
    if lam != F32(0.0):
        d = (d + (lam * w).astype(F32)).astype(F32)
    v_new = ((mu * v).astype(F32) + d).astype(F32)
    look = (d + (mu * v_new).astype(F32)).astype(F32)
    w_new = (w - (lr * look).astype(F32)).astype(F32)
    return w_new, v_new


# ---------------------------------------------------------------------------
# the whole path as a state machine
# ---------------------------------------------------------------------------

class AccordionOracle:
    """State: error memory e[w] (W x N), accumulated gradient A (N), right factors Q
    (one m x r_max block per matrix layer), previous norms, level per layer.

    layers: sequence of (offset, rows, cols, is_matrix).
    level_crit / level_noncrit: rank (PowerSGD) or numerator of K over k_den (TopK)
    used inside / outside critical regimes.  In the paper's words the level used in
    critical regimes is l_low (low compression: higher rank, larger K)."""

    def __init__(self, method: int, layers, n_workers: int, level_crit: int,
                 level_noncrit: int, k_den: int = 100, eta: float = 0.5,
                 initial_level: int = 1, q_init: np.ndarray | None = None,
                 detector: str = "norm"):
        self.method = int(method)
        self.layers = [tuple(int(v) for v in l) for l in layers]
        self.W = int(n_workers)
        self.level_crit, self.level_noncrit = int(level_crit), int(level_noncrit)
        self.k_den = int(k_den)
        self.eta = F32(eta)
        self.N = sum(r * c for (_, r, c, _) in self.layers)
        nl = len(self.layers)
        self.e = np.zeros((self.W, self.N), dtype=F32)
        self.A = np.zeros(self.N, dtype=F32)
        self.level = np.full(nl, int(initial_level), dtype=np.int32)
        self.norm_old = np.zeros(nl, dtype=F32)
        self.norm_curr = np.zeros(nl, dtype=F32)
        self.norm_prev = np.zeros(nl, dtype=F32)   # the old norm the last decision used
        self.has_old = np.zeros(nl, dtype=np.int32)
        self.r_max = max(self.level_crit, self.level_noncrit) if method == POWERSGD else 0
        self.Q = {}
        if method == POWERSGD:
            pos = 0
            for li, (_, r, c, is_m) in enumerate(self.layers):
                if is_m:
                    blk = c * self.r_max
                    self.Q[li] = np.array(q_init[pos:pos + blk], dtype=F32).reshape(c, self.r_max).copy()
                    pos += blk
        assert detector in ("norm", "msdr")
        self.detector = detector
        self.sq = np.zeros(nl, dtype=F64)       # msdr: sum over the window of ||g_0||^2 per layer
        self.T = 0                              # msdr: steps in the window
        self.words_last = 0
        self.words_cum = 0
        # intermediates of the last step, kept for comparison
        self.P_hat = {}
        self.Q_bar = {}
        self.payload = {}       # (worker, layer) -> (idx, val)

    # -- level lookup ------------------------------------------------------
    def level_value(self, li: int) -> int:
        return self.level_crit if self.level[li] == 1 else self.level_noncrit

    def layer_rank(self, li: int) -> int:
        _, r, c, _ = self.layers[li]
        return effective_rank(self.level_value(li), r, c)

    def layer_k(self, li: int) -> int:
        _, r, c, _ = self.layers[li]
        return k_from_fraction(r * c, self.level_value(li), self.k_den)

    # -- one training step ---------------------------------------------------
    def step(self, grads: Sequence[np.ndarray]) -> np.ndarray:
        """Consume one gradient per worker, return the averaged decompressed
        gradient (N, fp32); updates e, A, Q and the payload counters."""
        assert len(grads) == self.W
        out = np.zeros(self.N, dtype=F32)
        # accumulate the raw gradient of worker 0 (the deciding node, Section 3 "Goals")
        self.A = (self.A + grads[0].astype(F32)).astype(F32)
        if self.detector == "msdr":
            for li, (off, rows, cols, _) in enumerate(self.layers):
                g0 = grads[0][off:off + rows * cols].astype(F64)
                self.sq[li] += float(np.dot(g0, g0))
            self.T += 1
        delta = [ef_add(grads[w], self.e[w]) for w in range(self.W)]
        words = 0
        self.P_hat, self.Q_bar, self.payload = {}, {}, {}
        for li, (off, rows, cols, is_m) in enumerate(self.layers):
            n = rows * cols
            sl = slice(off, off + n)
            if self.method == POWERSGD:
                if is_m:
                    r = self.layer_rank(li)
                    mats = [delta[w][sl].reshape(rows, cols) for w in range(self.W)]
                    p_hat, q_bar, d = powersgd_layer(mats, self.Q[li][:, :r])
                    self.Q[li][:, :r] = q_bar          # warm start of the next step
                    self.P_hat[li], self.Q_bar[li] = p_hat, q_bar
                    out[sl] = d.reshape(-1)
                    for w in range(self.W):
                        self.e[w, sl] = (mats[w] - d).astype(F32).reshape(-1)
                    words += r * (rows + cols)
                else:
                    # 1-D tensors are sent as they are: plain mean, no memory
                    acc = sum(grads[w][sl].astype(F64) for w in range(self.W)) / self.W
                    out[sl] = acc.astype(F32)
                    self.e[:, sl] = F32(0.0)
                    words += n
            else:
                k = self.layer_k(li)
                pays = []
                for w in range(self.W):
                    idx, val = topk_select(delta[w][sl], k)
                    self.e[w, sl] = topk_residual(delta[w][sl], idx)
                    self.payload[(w, li)] = (idx, val)
                    pays.append((idx, val))
                out[sl] = sparse_mean(n, pays, self.W)
                words += 2 * k
        self.words_last = words
        self.words_cum += words
        return out

    def step_update(self, grads: Sequence[np.ndarray], w: np.ndarray, v: np.ndarray, lr,
                    momentum, weight_decay=0.0) -> np.ndarray:
        """One training step followed by the optimizer: the averaged decompressed gradient
        of step() drives nesterov_update on every element that belongs to a layer; w and v
        (N, fp32) are changed in place.  Returns the averaged gradient."""
        d = self.step(grads)
        for off, rows, cols, _ in self.layers:
            sl = slice(off, off + rows * cols)
            w[sl], v[sl] = nesterov_update(w[sl], v[sl], d[sl], lr, momentum, weight_decay)
        return d

    # -- end of a window -----------------------------------------------------
    def detect_regime(self, lr_curr: float, lr_next: float) -> np.ndarray:
        """Norm of each layer's accumulated gradient, Algorithm 1 per layer, then
        curr -> old and the accumulator restarts.  Returns the new level vector
        (1 = critical)."""
        if self.detector == "msdr":
            return self._detect_msdr()
        for li, (off, rows, cols, _) in enumerate(self.layers):
            c = layer_norm(self.A[off:off + rows * cols])
            crit = regime_is_critical(self.norm_old[li], c, bool(self.has_old[li]),
                                      self.eta, lr_curr, lr_next)
            self.level[li] = 1 if crit else 0
            self.norm_prev[li] = self.norm_old[li]
            self.norm_curr[li] = c
            self.norm_old[li] = c
            self.has_old[li] = 1
        self.A[:] = F32(0.0)
        return self.level.copy()

    def _detect_msdr(self) -> np.ndarray:
        """Window end with the comparison detector: norm_curr holds the window's ratio,
        norm_old the reference (the ratio at the last switch, or of the first window)."""
        for li, (off, rows, cols, _) in enumerate(self.layers):
            m = msdr_streaming(self.A[off:off + rows * cols], self.sq[li], max(self.T, 1))
            self.norm_prev[li] = self.norm_old[li]
            self.norm_curr[li] = m
            if not self.has_old[li]:
                self.norm_old[li] = m
                self.has_old[li] = 1
            elif msdr_should_switch(self.norm_old[li], m, True, self.eta):
                self.level[li] = 1
                self.norm_old[li] = m
        self.A[:] = F32(0.0)
        self.sq[:] = 0.0
        self.T = 0
        return self.level.copy()

    def reset_accumulator(self) -> None:
        self.A[:] = F32(0.0)
        self.sq[:] = 0.0
        self.T = 0

    def words_per_step(self) -> int:
        """Floats one worker sends per step at the current levels."""
        total = 0
        for li, (_, rows, cols, is_m) in enumerate(self.layers):
            if self.method == POWERSGD:
                total += self.layer_rank(li) * (rows + cols) if is_m else rows * cols
            else:
                total += 2 * self.layer_k(li)
        return total


# ---------------------------------------------------------------------------
# batch-size mode
# ---------------------------------------------------------------------------

class BatchSizeOracle:
    """Accordion switching the batch size instead of the compression level.

    One call of micro_step() is one backward pass of every worker on a micro-batch of
    B_low samples.  Inside a critical regime (level 1) every micro-step is exchanged
    (batch B_low); outside (level 0) `multiplier` = floor(B_high / B_low) micro-steps
    are summed locally first and exchanged once (batch B_high), so that the workers
    communicate `multiplier` times less (Section 3).  The exchanged gradient is the
    mean over workers and accumulated micro-steps; the learning rate of that update is
    the base rate times the number of micro-steps in it (Section 5.1).

    The detector looks at the whole model (Section 4.2): A sums worker 0's raw
    micro-batch gradients over the window, one norm over all layers, Algorithm 1 once.
    monotone (Appendix A): once the large batch is reached the level never returns.

    fp32 state; sums in the order written (micro-steps in time order, workers in index
    order starting from worker 0's sum), one division by W * (micro-steps)."""

    def __init__(self, layers, n_workers: int, multiplier: int, eta: float = 0.5,
                 initial_level: int = 1, monotone: bool = True):
        self.layers = [tuple(int(v) for v in l) for l in layers]
        self.W = int(n_workers)
        self.M = int(multiplier)
        assert self.M >= 1
        self.eta = F32(eta)
        self.monotone = bool(monotone)
        self.N = max(off + r * c for (off, r, c, _) in self.layers)
        self.mask = np.zeros(self.N, dtype=bool)
        for off, r, c, _ in self.layers:
            self.mask[off:off + r * c] = True
        self.S = np.zeros((self.W, self.N), dtype=F32)
        self.A = np.zeros(self.N, dtype=F32)
        self.j = 0                       # micro-steps summed since the last exchange
        self.level = int(initial_level)
        self.norm_old = F32(0.0)
        self.norm_curr = F32(0.0)
        self.norm_prev = F32(0.0)
        self.has_old = 0
        self.words_last = 0              # floats one worker sent in the last micro-step
        self.words_cum = 0
        self.exchanges = 0
        self.n_model = int(self.mask.sum())

    def micro_step(self, grads: Sequence[np.ndarray]):
        """Returns (D, n_micro): the averaged gradient of the batch that this micro-step
        completed and the number of micro-steps in it, or (None, 0) if nothing was
        exchanged.  Elements outside every layer are zero in D."""
        assert len(grads) == self.W
        m = self.mask
        self.A[m] = (self.A[m] + grads[0][m].astype(F32)).astype(F32)
        for w in range(self.W):
            if self.j == 0:
                self.S[w, m] = grads[w][m].astype(F32)
            else:
                self.S[w, m] = (self.S[w, m] + grads[w][m].astype(F32)).astype(F32)
        self.j += 1
        target = 1 if self.level == 1 else self.M
        if self.j < target:
            self.words_last = 0
            return None, 0
        acc = self.S[0].copy()
        for w in range(1, self.W):
            acc = (acc + self.S[w]).astype(F32)
        d = (acc / F32(self.W * self.j)).astype(F32)
        d[~m] = F32(0.0)
        n_micro = self.j
        self.j = 0
        self.words_last = self.n_model           # dense all-reduce of the whole model
        self.words_cum += self.n_model
        self.exchanges += 1
        return d, n_micro

    def micro_step_update(self, grads, w: np.ndarray, v: np.ndarray, lr, momentum,
                          weight_decay=0.0) -> int:
        """micro_step followed, when a batch was completed, by the optimizer step with the
        learning rate lr * (micro-steps in the batch), the product rounded to fp32.
        Returns the number of micro-steps in the applied batch (0: no update)."""
        d, n_micro = self.micro_step(grads)
        if d is None:
            return 0
        lr_eff = F32(F32(lr) * F32(n_micro))
        m = self.mask
        w[m], v[m] = nesterov_update(w[m], v[m], d[m], lr_eff, momentum, weight_decay)
        return n_micro

    def detect_regime(self, lr_curr: float, lr_next: float) -> int:
        c = layer_norm(self.A[self.mask])
        crit = regime_is_critical(self.norm_old, c, bool(self.has_old), self.eta, lr_curr, lr_next)
        new_level = 1 if crit else 0
        if self.monotone and self.level == 0:
            new_level = 0                         # the batch size is only allowed to grow
        self.level = new_level
        self.norm_prev = self.norm_old
        self.norm_curr = c
        self.norm_old = c
        self.has_old = 1
        self.A[:] = F32(0.0)
        return self.level
