"""CPU oracle for the Continual Context Distillation (CCD) compression step.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP path is checked against.  Nothing in the product path may import it; only
the tests, the smoke check and the benchmark's CPU-baseline leg do.  It shares
no code with the HIP kernels or their Python binding and imports neither.

Every floating-point step runs in fp64 on the exact values of the (fp32 or
bf16) inputs.  The only narrowing is the final score, which is cast to fp32
because the selection is defined on fp32 scores (the precision the library's
`scores` array has).

Notation follows the paper: a pot holds n cached context tokens per (layer,
KV head); |P| catalyst-prompt (CaP) query tokens attend to them; |C| = k
entries survive, T of which are reserved for the tokens with the highest
Novelty-under-Compression (NuC) score.

Steps, per unit (sequence b, layer l, KV head h), in the paper's order:

  nuc_slots     Sec. 3.3.3, first step: the T tokens with the largest novelty.
  cap_scores    Eq. 2: representative score = sum over the CaP query tokens of
                their attention probability on each context token (the Listing
                in App. B sums the CaP rows of the attention map and keeps the
                context columns only).  With grouped-query attention the G
                query heads that share the KV head are summed as well.  Two readings of
                "the attention row" are provided: the softmax over the n context tokens
                alone (the default: the benchmark's interface hands over the cache only),
                and, with K_cap, the model's own causal row, in which CaP token i also
                attends to the CaP keys 0 .. i (Eq. 2 places the CaP tokens at the end of
                the same sequence).  A sliding attention window (window > 0) hides the oldest
                cached tokens from the later CaP tokens.  cap_scores_given_lse is the same sum
                with each query's normaliser (log-sum-exp of its row) handed in by the caller.
  pool          1-D pooling of the score along the token axis (not in the
                paper; the paper's implementation follows a code base that
                clusters scores this way, and the benchmark configs ask for a
                window of 7).
  combine       App. B "Combine NuC and CaP": NuC-selected tokens are lifted
                above every CaP score so that they always survive (+inf here).
  select        Sec. 3.3.3, second step / App. B "Final Token Selection":
                top-k per head; ties go to the lower index; the kept indices
                are emitted in ascending (temporal) order.
  compact       App. B: K' = K[keep], V' = V[keep] (bit copies).
  append        Sec. 3.2: between two distillations the pot is filled - the keys, values and novelty of the next
                chunk of context go behind the cached tokens (bit copies; the novelty of a token is the same
                for every head).
  nuc_from_logits  Sec. 3.3.2, Eq. 3 / App. B "Calculate NuC Score": the novelty of a token is its cross
                entropy under the model, n_t = -log P(x_t | context), read off the logits row that
                predicts x_t.  (Which context the model saw - the compressed one of Eq. 4 - is the
                model's forward pass, outside this step; the alignment of logits rows and labels is
                the caller's: row r must be the prediction FOR label r.)
  cr_rope       Sec. 3.5 (CR-RoPE): the pot holds keys before the rotary embedding; after a
                distillation the kept entries get the rotary embedding of positions
                0 .. |C|-1 (their new places), whatever their original positions were.

Parity status of the choices the paper does not fix (pool mode, the GQA
reduction, softmax over context tokens only, +inf sentinel, per-head carried
novelty): pinned by the benchmark's wording only - "parity unpinned" against
the paper for those choices.  All arithmetic (softmax-sum, pooling, top-k,
gather) is pinned by the tests in tests/test_oracle_pins.py.

CR-RoPE: the paper names RoPE without fixing the pairing of dimensions; the
half-split pairing (dimension i with i + d/2) of the LLaMA / Mistral models it
evaluates is used - "parity unpinned" for that choice.  The rotation itself
is pinned in tests/test_oracle_rope_pins.py.  Angle tables are inputs (the
caller's rope base and scaling), as are the positions.
"""
from __future__ import annotations

import math

import numpy as np

POOL_NONE, POOL_MAX, POOL_AVG = 0, 1, 2
FLT_MIN = float(np.finfo(np.float32).tiny)


def to_f64(x: np.ndarray) -> np.ndarray:
    """Exact fp64 value of an input array: float32, or bf16 bit patterns (uint16)."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if x.dtype in (np.float32, np.float64):
        return x.astype(np.float64)
    raise TypeError(f"unsupported input dtype {x.dtype}")


def nuc_slots(novelty: np.ndarray, T: int) -> np.ndarray:
    """Sec. 3.3.3, step 1: indices of the T largest novelty scores (ascending).

    Equal novelty goes to the lower index.  Tokens whose novelty is NaN or
    -inf never take a slot, so fewer than T may be returned.
    """
    nov = np.asarray(novelty, dtype=np.float32)
    n = nov.shape[0]
    eligible = np.flatnonzero(~np.isnan(nov) & (nov > -np.inf))
    if T <= 0 or eligible.size == 0:
        return np.zeros(0, dtype=np.int64)
    vals = nov[eligible].astype(np.float64)
    order = np.lexsort((eligible, -vals))  # primary: novelty descending; then index ascending
    take = eligible[order[: min(T, eligible.size)]]
    assert take.size <= n
    return np.sort(take)


def cap_scores(Q: np.ndarray, K: np.ndarray, scale: float, K_cap: np.ndarray | None = None, P: int | None = None,
               window: int = 0) -> np.ndarray:
    """Eq. 2: u_t = sum over CaP queries of softmax_t(scale * <q, k_t>).

    Q is [G*P, d] (all query rows that attend through this KV head, row g*P + i = CaP token i
    of query head g), K is [n, d]; both already fp64.  Without K_cap the softmax runs over the
    n context tokens.  With K_cap [P, d] (the CaP tokens' own keys) it is the model's causal
    attention row of Eq. 2: CaP token i also sees the CaP keys 0 .. i, which take their share
    of the probability mass; the score still sums the context columns only.
    window > 0: sliding-window attention (the footnote on Mistral-v0.1 in Sec. 4): the cached
    tokens stand at positions 0 .. n-1 and CaP token i at position n + i; a query at position p
    sees the keys at positions p - window + 1 .. p only, so context token t is hidden from CaP
    token i when t < n + i + 1 - window.  (CaP keys j <= i are always inside the window:
    window >= P is required.  Without K_cap a CaP token whose window holds no cached token
    gives nothing to any score.)
    """
    n = K.shape[0]
    if P is None and K_cap is not None:
        P = K_cap.shape[0]
    S = scale * (Q @ K.T)                      # [G*P, n] attention logits
    if window and window > 0:
        assert P is not None and window >= P
        i = np.arange(Q.shape[0]) % P          # CaP position of each query row
        first_visible = n + i + 1 - window
        S = np.where(np.arange(n)[None, :] >= first_visible[:, None], S, -np.inf)
    if K_cap is None:
        m = S.max(axis=1, keepdims=True)
        m = np.where(np.isneginf(m), 0.0, m)   # a row whose window holds no cached token (window == P at most)
        E = np.exp(S - m)
        Z = E.sum(axis=1, keepdims=True)
        A = np.divide(E, Z, out=np.zeros_like(E), where=Z > 0)   # attention probabilities, rows sum to 1 (or are empty)
        return A.sum(axis=0)                   # sum over the CaP rows
    assert K_cap.shape[0] == P and Q.shape[0] % P == 0
    C = scale * (Q @ K_cap.T)                  # [G*P, P] logits on the CaP keys
    i = np.arange(Q.shape[0]) % P              # CaP position of each query row
    C = np.where(np.arange(P)[None, :] <= i[:, None], C, -np.inf)   # causal: key j visible iff j <= i
    m = np.maximum(S.max(axis=1, keepdims=True), C.max(axis=1, keepdims=True))
    E, Ec = np.exp(S - m), np.exp(C - m)
    Z = E.sum(axis=1, keepdims=True) + Ec.sum(axis=1, keepdims=True)
    return (E / Z).sum(axis=0)                 # context columns only


def cap_scores_given_lse(Q: np.ndarray, K: np.ndarray, scale: float, lse: np.ndarray, P: int | None = None,
                         window: int = 0) -> np.ndarray:
    """Eq. 2 with the normalisers handed in: u_t = sum over CaP queries of exp(scale * <q, k_t> - lse_q).

    lse [G*P] is the natural-log-sum-exp of each CaP query's attention row, over whatever keys the model let it
    attend to (attention kernels return it next to their output); the probabilities on the cached tokens follow from
    it without a pass over the row.  window > 0 hides cached tokens as in cap_scores (their probability is 0).
    """
    n = K.shape[0]
    S = scale * (Q @ K.T)
    A = np.exp(S - np.asarray(lse, dtype=np.float64)[:, None])
    if window and window > 0:
        assert P is not None and window >= P
        i = np.arange(Q.shape[0]) % P
        A = np.where(np.arange(n)[None, :] >= (n + i + 1 - window)[:, None], A, 0.0)
    return A.sum(axis=0)


def pool(u: np.ndarray, w: int, mode: int) -> np.ndarray:
    """Stride-1 pooling along the token axis with an odd window w, centred.

    max: the window is clipped at both ends.  avg: zero padding, divide by w.
    """
    if mode == POOL_NONE or w <= 1:
        return u.copy()
    n = u.shape[0]
    r = w // 2
    out = np.empty_like(u)
    for t in range(n):
        lo, hi = max(0, t - r), min(n, t + r + 1)
        if mode == POOL_MAX:
            out[t] = u[lo:hi].max()
        elif mode == POOL_AVG:
            out[t] = u[lo:hi].sum() / w
        else:
            raise ValueError("pool mode")
    return out


def combine(ubar: np.ndarray, nuc: np.ndarray) -> np.ndarray:
    """fp32 score: pooled CaP score, subnormals flushed to zero, +inf at NuC tokens."""
    with np.errstate(under="ignore", over="ignore"):
        s = ubar.astype(np.float32)
    s[np.abs(s) < np.float32(FLT_MIN)] = np.float32(0.0)
    s[nuc] = np.float32(np.inf)
    return s


def select(scores: np.ndarray, k: int) -> np.ndarray:
    """Top-k of fp32 scores; equal scores -> lower index; result ascending.

    NaN ranks with -inf.
    """
    s = np.asarray(scores, dtype=np.float32).astype(np.float64)
    s = np.where(np.isnan(s), -np.inf, s)
    idx = np.arange(s.shape[0])
    order = np.lexsort((idx, -s))
    return np.sort(order[:k]).astype(np.int32)


def compact(X: np.ndarray, keep: np.ndarray) -> np.ndarray:
    """Rows of X at the kept indices, in that order (a copy of the stored bits)."""
    return X[np.asarray(keep, dtype=np.int64)].copy()


def append(pot: np.ndarray, n_valid: int, chunk: np.ndarray) -> np.ndarray:
    """Sec. 3.2, filling the pot: a copy of `pot` [..., n_cap(, d)] whose token rows n_valid .. n_valid + m - 1 hold the
    m rows of `chunk` [..., m(, d)] (leading dimensions of the chunk broadcast over the pot's: one novelty value per
    token goes to every head); the other rows are untouched.  The token axis is axis 3 for K and V [B, L, Hkv, n, d]
    and the last axis for novelty."""
    out = pot.copy()
    m = chunk.shape[3] if pot.ndim == 5 else chunk.shape[-1]
    if n_valid < 0 or n_valid + m > (pot.shape[3] if pot.ndim == 5 else pot.shape[-1]):
        raise ValueError("the chunk does not fit behind the cached tokens")
    if pot.ndim == 5:
        out[:, :, :, n_valid:n_valid + m, :] = chunk
    else:
        out[..., n_valid:n_valid + m] = chunk
    return out


def nuc_from_logits(logits: np.ndarray, labels: np.ndarray) -> np.ndarray:
    """Eq. 3: per-token cross entropy, n_r = log(sum_v exp(z_rv)) - z_{r, label_r}, as fp32 [rows].

    logits [rows, V] in storage form (fp32 or bf16 bits); labels [rows] integer.  A label outside
    [0, V) marks a token without a prediction: its novelty is -inf, so it never takes a NuC slot.
    """
    z = to_f64(logits)
    labels = np.asarray(labels).astype(np.int64)
    rows, V = z.shape
    out = np.full(rows, -np.inf, dtype=np.float64)
    for r in range(rows):
        if 0 <= labels[r] < V:
            m = z[r].max()
            out[r] = m + math.log(np.exp(z[r] - m).sum()) - z[r, labels[r]]
    return out.astype(np.float32)


def rope_rotate(X: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Rotary embedding of the rows of X [n, d] (fp64) by the angles whose cos/sin are given, [n, d/2].

    Dimension i is paired with dimension i + d/2 and the pair is rotated by angle[n, i]:
        y_i       = x_i * cos - x_{i+d/2} * sin
        y_{i+d/2} = x_{i+d/2} * cos + x_i * sin
    """
    X = np.asarray(X, dtype=np.float64)
    h = X.shape[-1] // 2
    c, s = np.asarray(cos, dtype=np.float64), np.asarray(sin, dtype=np.float64)
    x1, x2 = X[..., :h], X[..., h:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def round_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp64 -> bf16 storage bits, round to nearest even, straight from the fp64 value (8 significant bits).

    Normal range only (|x| in [2^-126, 2^127]); a zero keeps its sign.  Overflow and subnormals are not needed here."""
    x = np.asarray(x, dtype=np.float64)
    m, e = np.frexp(x)                       # x = m * 2^e, 0.5 <= |m| < 1
    q = np.rint(m * 256.0)                   # 8 significant bits, ties to even
    y = np.ldexp(q, e - 8).astype(np.float32)   # exactly representable in fp32
    return (y.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def cr_rope(K_kept: np.ndarray, cos: np.ndarray, sin: np.ndarray) -> np.ndarray:
    """Sec. 3.5: rotary embedding of the kept (pre-RoPE) keys at their NEW positions 0 .. k-1.

    K_kept [k, d] in storage form (bf16 bits or fp32); cos/sin tables with at least k rows.  The result is
    rounded once to the storage type."""
    k = K_kept.shape[0]
    y = rope_rotate(to_f64(K_kept), cos[:k], sin[:k])
    if np.asarray(K_kept).dtype == np.uint16:
        return round_bf16_bits(y)
    return y.astype(np.float32)


def score_unit(Q, K, novelty, *, T, scale, pool_w, pool_mode, K_cap=None, P=None, window=0, lse=None):
    """Final fp32 scores of one unit. Q [G*P, d], K [n, d], K_cap [P, d] or None: raw inputs; novelty [n] fp32;
    lse [G*P] fp32 or None: the rows' log-sum-exps handed in (then K_cap is not used)."""
    if lse is not None:
        u = cap_scores_given_lse(to_f64(Q), to_f64(K), scale, to_f64(lse), P=P, window=window)
    else:
        u = cap_scores(to_f64(Q), to_f64(K), scale, None if K_cap is None else to_f64(K_cap), P=P, window=window)
    ubar = pool(u, pool_w, pool_mode)
    return combine(ubar, nuc_slots(novelty, T))


def default_scale(d: int) -> float:
    return 1.0 / math.sqrt(d)


def compress(Q_cat, K, V, novelty, *, k, T, pool_w=1, pool_mode=POOL_MAX, scale=None,
             n_valid=None, units=None, rope_cos=None, rope_sin=None, K_score=None, K_cap=None, window=0, lse=None):
    """One CCD compression over a whole cache.

    Q_cat [B, L, Hq, P, d]; K, V [B, L, Hkv, n_cap, d]; novelty [B, n] (shared by
    all layers and heads) or [B, L, Hkv, n_cap] (carried per head).  Returns a dict
    with scores [B, L, Hkv, n] fp32, keep_idx [B, L, Hkv, k] int32, K', V'
    [B, L, Hkv, k, d] and, for per-head novelty, novelty' [B, L, Hkv, k].
    `units` optionally restricts the work to a list of (b, l, h) triples; the
    other entries of the outputs stay zero.  With rope_cos / rope_sin [>= k, d/2] the
    dict also holds K_rot [B, L, Hkv, k, d]: the kept keys after CR-RoPE (Sec. 3.5).
    K_score (same shape as K): the keys the CaP queries attend to, when they are not the
    stored ones - with CR-RoPE the pot stores keys before the rotary embedding while the
    model attends to the embedded keys of the current positions.
    K_cap [B, L, Hkv, P, d]: the CaP tokens' own keys; with them the attention rows are the
    model's causal ones (see cap_scores).  window > 0: sliding-window attention (see cap_scores).
    lse [B, L, Hq, P] fp32: the log-sum-exp of every CaP query's attention row, handed in (see cap_scores_given_lse).
    """
    B, L, Hq, P, d = Q_cat.shape
    Hkv, n_cap = K.shape[2], K.shape[3]
    G = Hq // Hkv
    assert Hq == G * Hkv
    n = n_cap if n_valid is None else n_valid
    scale = default_scale(d) if not scale else float(scale)
    per_head = novelty.ndim == 4
    scores = np.zeros((B, L, Hkv, n), dtype=np.float32)
    keep_idx = np.zeros((B, L, Hkv, k), dtype=np.int32)
    Kc = np.zeros((B, L, Hkv, k, d), dtype=K.dtype)
    Vc = np.zeros((B, L, Hkv, k, d), dtype=V.dtype)
    novc = np.zeros((B, L, Hkv, k), dtype=np.float32) if per_head else None
    Krot = np.zeros((B, L, Hkv, k, d), dtype=K.dtype) if rope_cos is not None else None
    todo = units if units is not None else [(b, l, h) for b in range(B) for l in range(L) for h in range(Hkv)]
    for (b, l, h) in todo:
        Qu = Q_cat[b, l, h * G:(h + 1) * G].reshape(G * P, d)
        nov = novelty[b, l, h, :n] if per_head else novelty[b, :n]
        Ks = K if K_score is None else K_score
        s = score_unit(Qu, Ks[b, l, h, :n], nov, T=T, scale=scale, pool_w=pool_w, pool_mode=pool_mode,
                       K_cap=None if K_cap is None else K_cap[b, l, h], P=P, window=window,
                       lse=None if lse is None else lse[b, l, h * G:(h + 1) * G].reshape(G * P))
        keep = select(s, k)
        scores[b, l, h] = s
        keep_idx[b, l, h] = keep
        Kc[b, l, h] = compact(K[b, l, h], keep)
        Vc[b, l, h] = compact(V[b, l, h], keep)
        if per_head:
            novc[b, l, h] = compact(novelty[b, l, h], keep)
        if Krot is not None:
            Krot[b, l, h] = cr_rope(Kc[b, l, h], rope_cos, rope_sin)
    return {"scores": scores, "keep_idx": keep_idx, "K": Kc, "V": Vc, "novelty": novc, "K_rot": Krot}
