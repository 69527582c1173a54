"""CPU oracle for the classifier-layer hot path of ASTRA (arXiv 2409.20156).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition of what
the GPU library must compute.  Only the test-suite, the smoke check and the
`cpu_baseline` leg of the benchmark may import it.  It shares no code with the
HIP path and never imports it.  Everything is numpy in float64; pure Python
integers are used where 128-bit products are needed.

Functions and the passage of the paper each one follows
-------------------------------------------------------
mine_negatives      Alg. 1 "ANNS refresh" step, realised as exact search (the
                    paper's own control experiment, Sec. 5.2.1(a)): ids of the
                    k_h labels with the largest <w_l, z_i> (Sec. 2.1 score).
sample_negatives    Alg. 1 hard+random step and Sec. 3.1 Idea 2: all k_h stale
                    hard negatives plus k_r i.i.d. uniform draws from
                    [L] \\ H_i, p = 1/(L-k_h) as under Eq. 2.  Warm-up mode
                    (Alg. 1, t < tau_s): all negatives uniform on [L].
sample_negatives_mixture
                    Sec. 3.1 Idea 2 taken literally: negatives drawn from the mixture
                    (1-r) P_imp + r P_unif, P_imp proportional to the sigmoid of the
                    stale score over a shortlist wider than k_h (the importance
                    sampling the paper motivates and then replaces by "retrieve the
                    top"), r = k_r/(k_h+k_r); logq = log of the expected count.
xc_step             Eq. 2 (sampled BCE) with its analytic gradient (form given
                    in the proof of Lemma 1) and the mini-batch SGD update of
                    W from Alg. 1; loss averaged over data points (Sec. 4).
                    A soft-max variant with proposal-corrected logits is the
                    second loss kind.
train_schedule      the outer loop of Alg. 1 over the three functions above:
                    warm-up steps with uniform negatives while t < tau_s, then a
                    shortlist refresh every tau_r steps and hard+random steps.
full_bce_loss       Eq. 1, every one of the L labels, for pinning Eq. 2.
full_softmax_loss   plain soft-max cross-entropy over all L labels.

Readings of the paper taken here (each is listed in the design document):
labels are 0..L-1 and W is stored L x d; random negatives are drawn with
replacement; positives are not excluded from the draw but get weight zero
through the (1 - y_l) factor; ids outside [0, L) are padding.

Parity status: every function below is pinned by tests that do not re-use its
own formula (closed forms, brute force over all labels through a library BCE,
Monte-Carlo unbiasedness of Eq. 2 against Eq. 1, finite differences, exhaustive
enumeration of the complement map, published splitmix64 vectors).
"""
from __future__ import annotations

import numpy as np

LOSS_BCE = 0
LOSS_SOFTMAX = 1

_MASK64 = (1 << 64) - 1
_K_QUERY = 0x9E3779B97F4A7C15   # odd constant separating query streams
_K_DRAW = 0xD1B54A32D192ED03    # odd constant separating draws of one query


# --------------------------------------------------------------------------
# storage rounding
# --------------------------------------------------------------------------
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bfloat16 value (ties to even),
    returned as float64.  bfloat16 keeps 8 significant bits, so the spacing of
    representable numbers around x = m * 2**e (0.5 <= |m| < 1) is 2**(e-8)."""
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)
    e = np.maximum(e, -125)                     # below that bf16 is subnormal
    q = np.ldexp(1.0, e - 8)
    return np.rint(x / q) * q                   # rint rounds half to even


def round_to_f32(x: np.ndarray) -> np.ndarray:
    return np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)


def _round_storage(x, dtype: str):
    if dtype == "bf16":
        return round_to_bf16(x)
    if dtype == "f32":
        return round_to_f32(x)
    if dtype == "f64":
        return np.asarray(x, dtype=np.float64)
    raise ValueError(dtype)


# --------------------------------------------------------------------------
# S1  mining: exact top-k inner product
# --------------------------------------------------------------------------
def mine_negatives(Z, W, k_h: int, chunk: int = 1 << 16):
    """For every query row z_i return the ids of the k_h rows of W with the
    largest inner product, best first; equal scores are ordered by smaller id.
    Returns (ids int32 [Zq,k_h], scores float64 [Zq,k_h]).

    Definition written out: all L scores, then a full ordering.  `chunk` only
    bounds the size of the temporary score block; the block results are
    concatenated candidates that are ordered again, so nothing is approximated.
    """
    Z = np.asarray(Z, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    Zq, d = Z.shape
    L, d2 = W.shape
    assert d == d2 and 1 <= k_h <= L
    cand_s = np.empty((Zq, 0), dtype=np.float64)
    cand_i = np.empty((Zq, 0), dtype=np.int64)
    for l0 in range(0, L, chunk):
        l1 = min(L, l0 + chunk)
        S = Z @ W[l0:l1].T                                  # [Zq, l1-l0]
        ids = np.broadcast_to(np.arange(l0, l1, dtype=np.int64), S.shape)
        s_all = np.concatenate([cand_s, S], axis=1)
        i_all = np.concatenate([cand_i, ids], axis=1)
        # order each row by (score descending, id ascending)
        order = np.lexsort((i_all, -s_all), axis=1)[:, :k_h]
        cand_s = np.take_along_axis(s_all, order, axis=1)
        cand_i = np.take_along_axis(i_all, order, axis=1)
    return cand_i.astype(np.int32), cand_s


# --------------------------------------------------------------------------
# S2  sampling
# --------------------------------------------------------------------------
def _fmix64(x: int) -> int:
    """Finaliser of the splitmix64 generator (Steele, Lea, Flood 2014)."""
    x &= _MASK64
    x ^= x >> 30
    x = (x * 0xBF58476D1CE4E5B9) & _MASK64
    x ^= x >> 27
    x = (x * 0x94D049BB133111EB) & _MASK64
    x ^= x >> 31
    return x


def draw_u64(seed: int, i: int, j: int) -> int:
    """Counter-based 64-bit word for query i, draw j: a function of the three
    integers only, so any thread layout reproduces it."""
    a = _fmix64((seed & _MASK64) ^ ((_K_QUERY * (i + 1)) & _MASK64))
    return _fmix64((a + _K_DRAW * (j + 1)) & _MASK64)


def bounded(u: int, m: int) -> int:
    """Map a 64-bit word to [0, m) by the high half of the 128-bit product."""
    return (u * m) >> 64


def complement_select(hs_sorted, r: int) -> int:
    """r-th smallest (0-based) element of {0,1,2,...} \\ hs_sorted.
    hs_sorted is strictly increasing.  With c = #{m : hs[m] - m <= r} the
    answer is r + c: exactly c excluded ids lie below it."""
    c = 0
    for m, h in enumerate(hs_sorted):
        if h - m <= r:
            c += 1
    return r + c


def sample_negatives(shortlist, B: int, k_h: int, k_r: int, L: int, seed: int, rows=None):
    """Negatives and log-proposal for one mini-batch.

    shortlist: int [B, k_h] (row i = stale hard negatives of query i) or None
    for the warm-up phase.  Returns (neg int32 [B, k_h+k_r], logq float32).

    Hard mode: slots 0..k_h-1 are the shortlist row verbatim with logq = 0
    (taken with probability one, weight 1 in Eq. 2).  Slots k_h.. hold k_r
    i.i.d. uniform draws from [L] \\ H_i, where H_i is the set of distinct
    in-range ids of the row (size u_i, equal to k_h for a mined shortlist);
    logq = log(k_r / (L - u_i)), the log of the expected number of copies of a
    label among the draws, so that exp(-logq) = 1/(p k_r) of Eq. 2.
    Warm-up mode: all k_h+k_r slots uniform on [L], logq = log((k_h+k_r)/L).
    `rows` (optional) restricts the work to those query indices of the batch; the
    other rows of the outputs are left at -1 / 0 (used to spot-check large batches).
    """
    n = k_h + k_r
    neg = np.full((B, n), -1, dtype=np.int32)
    logq = np.zeros((B, n), dtype=np.float32)
    for i in (range(B) if rows is None else rows):
        if shortlist is None:
            hs = []
            n_draw, first = n, 0
        else:
            row = [int(v) for v in shortlist[i][:k_h]]
            neg[i, :k_h] = row
            logq[i, :k_h] = 0.0
            hs = sorted({v for v in row if 0 <= v < L})
            n_draw, first = k_r, k_h
        M = L - len(hs)
        assert M >= 1
        for j in range(n_draw):
            r = bounded(draw_u64(seed, i, j), M)
            neg[i, first + j] = complement_select(hs, r)
        if n_draw:
            logq[i, first:] = np.float32(np.log(np.float64(n_draw) / np.float64(M)))
    return neg, logq


# --------------------------------------------------------------------------
# S2'  sampling from the mixture proposal itself (Sec. 3.1, Idea 2)
# --------------------------------------------------------------------------
_LOG2E_Q16 = 94548                      # round(log2(e) * 2^16)
# ln(2)^k / k! * 2^30, k = 1..5: Taylor coefficients of 2^u on [0, 1]
_POW2_C = (744261118, 257941248, 59597083, 10327387, 1431680)


def sigmoid_weight(score) -> int:
    """Integer importance weight of a shortlist slot: floor-arithmetic image of
    2^32 * sigmoid(score), the quantity the paper's importance distribution is
    proportional to (Sec. 3.1, Observation 2).  Fixed point throughout, so that
    the sampler is a function of the score's bits alone:
      t = floor(clamp(score, -30, 30) * 2^16);  y = (|t| * 94548) >> 16   (|x| log2 e, Q16)
      2^-y in Q30 from a degree-5 polynomial for the fractional part and a shift;
      s = (E << 32) / (2^30 + E)   (sigmoid(-|x|) in Q32);  weight = s or 2^32 - s.
    The relative accuracy (about 1e-4) only shapes the proposal: the estimator's
    weights use the same integers, so it stays exactly unbiased.  NaN -> 0."""
    x = np.float32(score)
    if x != x:
        return 0
    x = min(max(float(x), -30.0), 30.0)
    t = int(np.floor(np.float64(x) * 65536.0))
    a = abs(t)
    y = (a * _LOG2E_Q16) >> 16
    i, f = y >> 16, y & 0xFFFF
    if f == 0:
        m, shift = 1 << 30, i
    else:
        u = 65536 - f                       # 2^-f/65536 = 2^(u/65536) / 2
        r = _POW2_C[4]
        for c in (_POW2_C[3], _POW2_C[2], _POW2_C[1], _POW2_C[0]):
            r = c + ((r * u) >> 16)
        m, shift = (1 << 30) + ((r * u) >> 16), i + 1
    e = m >> shift if shift < 62 else 0
    sn = (e << 32) // ((1 << 30) + e)
    w = (1 << 32) - sn if t >= 0 else sn
    return max(w, 1)


def sample_negatives_mixture(shortlist, scores, B: int, M: int, k_h: int, k_r: int, L: int, seed: int, rows=None):
    """n = k_h + k_r negatives per query, drawn independently from the mixture proposal of
    Sec. 3.1 Idea 2 with r = k_r / n, in stratified form: slots 0..k_h-1 are draws from the
    importance part (label of shortlist slot m with probability w_m / T, w_m =
    sigmoid_weight(stale score of the slot), T their sum, slots with an id outside [0,L) or a
    NaN score excluded); slots k_h.. are uniform draws from all of [0,L).  Every slot gets
    logq = log(expected number of copies of its label among the n draws)
         = log(k_h * W_l / T + k_r / L),  W_l = total weight of the slots holding label l,
    so that a pair weighted by exp(-logq) makes the sampled sum an unbiased estimate of the sum
    over all L labels (the uniform part reaches every label).  A row without any valid slot
    falls back to n uniform draws (logq = log(n / L)), the warm-up sampler.
    Draw j of query i uses the same 64-bit word as sample_negatives; the importance draw is
    r = floor(u*T / 2^64) located in the running sums of the weights in slot order.
    Returns (neg int32 [B, n], logq float32 [B, n])."""
    n = k_h + k_r
    neg = np.full((B, n), -1, dtype=np.int32)
    logq = np.zeros((B, n), dtype=np.float32)
    for i in (range(B) if rows is None else rows):
        ids = [int(v) for v in shortlist[i][:M]]
        w = [sigmoid_weight(scores[i][m]) if 0 <= ids[m] < L else 0 for m in range(M)]
        T = sum(w)
        per_label = {}
        for m in range(M):
            if w[m]:
                per_label[ids[m]] = per_label.get(ids[m], 0) + w[m]
        cum, run = [], 0
        for m in range(M):
            run += w[m]
            cum.append(run)
        n_imp = k_h if T > 0 else 0
        for j in range(n):
            u = draw_u64(seed, i, j)
            if j < n_imp:
                r = bounded(u, T)
                m = next(mm for mm in range(M) if cum[mm] > r)
                lab = ids[m]
            else:
                lab = bounded(u, L)
            neg[i, j] = lab
            if T > 0:
                c = np.float64(k_h) * np.float64(per_label.get(lab, 0)) / np.float64(T) + np.float64(k_r) / np.float64(L)
            else:
                c = np.float64(n) / np.float64(L)
            logq[i, j] = np.float32(np.log(c))
    return neg, logq


def pps_select(w, k: int, u: int):
    """k of the slots with weight w[m] > 0, without replacement, slot m included with probability
    proportional to its weight: pi_m = min(1, k' w_m / T') exactly.  Two steps.
    (1) Certain slots: while some remaining slot has k' w_m >= T' (k' slots still to choose, T' the
        remaining total weight), all such slots are taken at once, k' and T' shrink, and the test is
        repeated.
    (2) Systematic sampling of the rest (Madow 1949): on the axis of the running sums c_m of the
        remaining weights in slot order, scaled by k', the k' points U + j T' (j = 0..k'-1) are marked,
        U = floor(u T' / 2^64) uniform on 0..T'-1; slot m is taken if a point falls into
        [k' c_{m-1}, k' c_m).  Every such interval is shorter than T', so no slot is taken twice, exactly
        k' are taken, and of the T' equally likely offsets exactly k' w_m take slot m.
    Returns (taken slots in slot order, pi as a list of (numerator, denominator) per slot; (0, 1) for
    weightless slots).  Needs 1 <= k <= number of slots with weight."""
    M = len(w)
    state = [1 if w[m] > 0 else 0 for m in range(M)]          # 1 remaining, 2 certain
    kk, TT = k, sum(w)
    while True:
        sure = [m for m in range(M) if state[m] == 1 and kk * w[m] >= TT]
        if not sure:
            break
        for m in sure:
            state[m] = 2
        kk -= len(sure)
        TT -= sum(w[m] for m in sure)
    pi = [(1, 1) if state[m] == 2 else ((kk * w[m], TT) if state[m] == 1 else (0, 1)) for m in range(M)]
    taken = [m for m in range(M) if state[m] == 2]
    if kk > 0:
        U = bounded(u, TT)

        def points_below(x):                                 # number of j in [0, kk) with U + j TT < x
            return 0 if x <= U else min(kk, (x - U - 1) // TT + 1)
        c = 0
        for m in range(M):
            if state[m] != 1:
                continue
            if points_below(kk * (c + w[m])) - points_below(kk * c) == 1:
                taken.append(m)
            c += w[m]
    return sorted(taken), pi


def sample_negatives_pps(shortlist, scores, B: int, M: int, k_h: int, k_r: int, L: int, seed: int, rows=None):
    """Hard negatives SAMPLED from a wider stale shortlist without replacement (Sec. 3.1: the
    importance distribution proportional to the sigmoid of the stale score, Observation 2, inside the
    mixture of Idea 2).  Per query: k = min(k_h, slots with weight) shortlist slots are chosen by
    pps_select with the weights sigmoid_weight(stale score) and the query's draw 0 as random word, and
    fill slots 0..k-1 in slot order; slots k..k_h+k_r-1 are uniform draws from all of [0, L) (draw j for
    slot j, as in the other samplers).  logq of a slot = log(expected number of copies of its label)
      = log(sum of pi_m over the shortlist slots that hold the label + (k_h + k_r - k) / L),
    so pairs weighted by exp(-logq) estimate a sum over all L labels without bias (a Horvitz-Thompson
    estimate on the shortlist part).  A row without any weight: all slots uniform.
    Returns (neg int32 [B, k_h+k_r], logq float32 [B, k_h+k_r])."""
    n = k_h + k_r
    neg = np.full((B, n), -1, dtype=np.int32)
    logq = np.zeros((B, n), dtype=np.float32)
    for i in (range(B) if rows is None else rows):
        ids = [int(v) for v in shortlist[i][:M]]
        w = [sigmoid_weight(scores[i][m]) if 0 <= ids[m] < L else 0 for m in range(M)]
        nv = sum(1 for x in w if x > 0)
        k = min(k_h, nv)
        taken, pi = pps_select(w, k, draw_u64(seed, i, 0)) if k > 0 else ([], [(0, 1)] * M)
        per_label = {}
        for m in range(M):                                   # in slot order
            if pi[m][0]:
                per_label[ids[m]] = per_label.get(ids[m], np.float64(0.0)) + np.float64(pi[m][0]) / np.float64(pi[m][1])
        unif = np.float64(n - k) / np.float64(L)
        for j in range(n):
            lab = ids[taken[j]] if j < k else bounded(draw_u64(seed, i, j), L)
            neg[i, j] = lab
            logq[i, j] = np.float32(np.log(per_label.get(lab, np.float64(0.0)) + unif))
    return neg, logq


# --------------------------------------------------------------------------
# S3-S5  the sampled training step
# --------------------------------------------------------------------------
def _softplus(x):
    """log(1 + exp(x)) without overflow."""
    return np.maximum(x, 0.0) + np.log1p(np.exp(-np.abs(x)))


def _sigmoid(x):
    return np.where(x >= 0, 1.0 / (1.0 + np.exp(-np.abs(x))),
                    np.exp(-np.abs(x)) / (1.0 + np.exp(-np.abs(x))))


def _candidates(i, pos, neg, logq, L):
    """Lists (label, is_positive, weight a, logq) of query i after masking:
    out-of-range ids are padding; a negative that is one of the query's
    positives carries the factor (1 - y_l) = 0 and is dropped."""
    pset = [int(l) for l in pos[i] if 0 <= l < L]
    out = [(l, True, 1.0, 0.0) for l in pset]
    pmember = set(pset)
    for j in range(neg.shape[1]):
        l = int(neg[i, j])
        if 0 <= l < L and l not in pmember:
            lq = float(logq[i, j])
            out.append((l, False, float(np.exp(-lq)), lq))
    return out


def xc_step(Z, W, pos, neg, logq, lr: float, kind: int = LOSS_BCE,
            storage: str = "f64"):
    """One classifier-layer step.  Inputs: Z [B,d], W [L,d] (values as stored;
    not modified), pos int [B,k_p] (-1 padded), neg int [B,n], logq [B,n].

    Returns dict with
      loss     float64 scalar, mean over the B queries
      dZ       float64 [B,d], gradient of `loss` w.r.t. Z (pre-update W)
      touched  int32 ascending unique labels whose row changed
      W_rows   float64 [len(touched), d] the updated rows, rounded to `storage`
      coef     list per query of (label, dloss/dscore) for inspection

    BCE kind (Eq. 2):  loss_i = sum_pos log(1+e^{-s}) + sum_neg a (s + log(1+e^{-s}))
    with a = exp(-logq): 1 for hard, (L-k_h)/k_r = 1/(p k_r) for random.
    d/ds: positives sigma(s)-1, negatives a sigma(s).
    Soft-max kind: logits s - logq over the candidate set, loss_i = mean over
    the positives of -log softmax; d/ds = softmax - [positive]/|pos_i|.
    """
    Z = np.asarray(Z, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    B, d = Z.shape
    L = W.shape[0]
    loss = 0.0
    dZ = np.zeros((B, d))
    dW = {}                                    # label -> gradient row
    coef = []
    for i in range(B):
        cand = _candidates(i, pos, neg, logq, L)
        labels = np.array([c[0] for c in cand], dtype=np.int64)
        ispos = np.array([c[1] for c in cand], dtype=bool)
        a = np.array([c[2] for c in cand])
        lq = np.array([c[3] for c in cand])
        if len(cand) == 0:
            coef.append([])
            continue
        rows = W[labels]                       # [n_i, d]
        s = rows @ Z[i]
        if kind == LOSS_BCE:
            li = np.where(ispos, _softplus(-s), a * _softplus(s))
            g = np.where(ispos, _sigmoid(s) - 1.0, a * _sigmoid(s))
            loss_i = li.sum()
        elif kind == LOSS_SOFTMAX:
            npos = int(ispos.sum())
            if npos == 0:       # no positive: the query is skipped entirely
                coef.append([])
                continue
            t = s - lq
            m = t.max()
            lse = m + np.log(np.exp(t - m).sum())
            loss_i = -(t[ispos] - lse).sum() / npos
            g = np.exp(t - lse) - ispos / npos
        else:
            raise ValueError(kind)
        g = g / B                              # mean over the batch
        loss += loss_i / B
        dZ[i] = g @ rows
        for l, gj in zip(labels, g):
            dW.setdefault(int(l), np.zeros(d))
            dW[int(l)] += gj * Z[i]
        coef.append([(int(l), float(gj)) for l, gj in zip(labels, g)])
    touched = np.array(sorted(dW.keys()), dtype=np.int32)
    W_rows = np.empty((len(touched), d))
    for r, l in enumerate(touched):
        W_rows[r] = _round_storage(W[l] - lr * dW[int(l)], storage)
    return {"loss": loss, "dZ": dZ, "touched": touched, "W_rows": W_rows,
            "coef": coef, "dW": dW}


# --------------------------------------------------------------------------
# full-label references (tiny inputs only, O(B L d))
# --------------------------------------------------------------------------
def train_schedule(Z_pool, W, pos_pool, B: int, k_h: int, k_r: int, steps: int, tau_s: int, tau_r: int,
                   lr: float, seeds, kind: int = LOSS_BCE, storage: str = "f32", lag: int = 0):
    """Alg. 1 for the classifier alone (encoder frozen: the query pool Z_pool is fixed).

    Step t uses the mini-batch of rows (t mod nbatch)*B .. +B of the pool.  While t < tau_s the
    negatives are all uniform (warm-up).  From t = tau_s on, the shortlists of the WHOLE pool are
    rebuilt by exact search whenever (t - tau_s) is a multiple of tau_r, from W as it stands
    before step t.  With lag = 0 step t already uses them; with lag > 0 the search is taken to
    run beside the training steps (the paper's asynchronous refresh) and its result replaces the
    older shortlists only from step t + lag on, so steps t .. t+lag-1 still use the older ones
    (warm-up negatives if there are none yet).  The step takes its batch's rows of the active
    (stale) shortlist as hard negatives plus k_r uniform ones.  seeds[t] is the sampler's seed of
    step t.  W (float64 [L,d]) is updated in place, rounded to `storage` after every step as the
    stored matrix is.

    Returns a dict: loss (list, per step), neg (list, per step: the sampled ids), shortlists
    (list of (t, int32 [pool,k_h]) per refresh, t = the step whose W was searched), overlap
    (list, per refresh after the first: mean over queries of |fresh & previous| / k_h).
    """
    pool, L = Z_pool.shape[0], W.shape[0]
    nbatch = max(1, pool // B)
    out = {"loss": [], "shortlists": [], "overlap": [], "neg": []}
    shortlist = None          # active
    newest = None             # last one built (equal to the active one once its lag has passed)
    pending = []              # (activation step, shortlist)
    for t in range(steps):
        if t >= tau_s and (t - tau_s) % tau_r == 0:
            fresh, _ = mine_negatives(Z_pool, W, k_h)
            if newest is not None:
                same = [len(set(fresh[q].tolist()) & set(newest[q].tolist())) for q in range(pool)]
                out["overlap"].append(float(np.mean(same)) / k_h)
            newest = fresh
            pending.append((t + lag, fresh))
            out["shortlists"].append((t, fresh.copy()))
        while pending and pending[0][0] <= t:
            shortlist = pending.pop(0)[1]
        b = t % nbatch
        lo, hi = b * B, (b + 1) * B
        rows = shortlist[lo:hi] if shortlist is not None else None
        neg, logq = sample_negatives(rows, B, k_h, k_r, L, seeds[t])
        res = xc_step(Z_pool[lo:hi], W, pos_pool[lo:hi], neg, logq, lr, kind=kind, storage=storage)
        W[res["touched"]] = res["W_rows"]
        out["loss"].append(res["loss"])
        out["neg"].append(neg)
    return out


def full_bce_loss(Z, W, pos):
    """Eq. 1 averaged over the batch: every label is either a positive of the
    query (first sum) or a negative (second sum)."""
    Z = np.asarray(Z, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    B, L = Z.shape[0], W.shape[0]
    total = 0.0
    for i in range(B):
        y = np.zeros(L)
        for l in pos[i]:
            if 0 <= l < L:
                y[int(l)] = 1.0
        s = W @ Z[i]
        total += (y * _softplus(-s)).sum() + ((1.0 - y) * (s + _softplus(-s))).sum()
    return total / B


def full_softmax_loss(Z, W, pos):
    """Soft-max cross-entropy over all L labels, averaged over the positives
    of a query and over the batch."""
    Z = np.asarray(Z, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    B, L = Z.shape[0], W.shape[0]
    total = 0.0
    for i in range(B):
        p = [int(l) for l in pos[i] if 0 <= l < L]
        s = W @ Z[i]
        m = s.max()
        lse = m + np.log(np.exp(s - m).sum())
        total += -(s[p] - lse).sum() / len(p)
    return total / B
