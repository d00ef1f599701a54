"""Plain CPU oracle for quality-adaptive KV-cache quantization (QAQ).

TEST INFRASTRUCTURE ONLY.  This module is the slow, obviously-correct statement
of what the GPU library has to compute.  Only the tests, the smoke check and the
CPU-baseline leg of the benchmark may import it; the product path never does,
and this module imports nothing from the product.  It shares no code, table or
constant with the HIP path.

Every function restates a passage of the paper (arXiv 2403.04643) and says
which one.  Where the paper leaves a choice open, the reading taken is written
next to the code.  All "fp32" steps use numpy float32 arithmetic (IEEE-754
binary32, round to nearest even, one rounding per operation, never fused);
attention is evaluated in float64.

Parity status of the parts (what pins each one is listed in tests/test_oracle_*):
  * attention, prompt score rows, quantizer, requantization, outlier split,
    thresholds, bit rule, window, accounting: pinned.
  * the variance approximation behind the key rule (second-order expansion of
    a ratio, Section 4.1 "Key cache quantization") is a heuristic of the paper:
    only its algebra is pinned -- "parity unpinned" beyond that.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

F32 = np.float32
F16 = np.float16
DEFAULT_BIT_SET = (2, 3, 4, 8)


# ----------------------------------------------------------------------------
# Section 2.1 (problem description): single-query attention of one head.
# ----------------------------------------------------------------------------
def attention(q: np.ndarray, K: np.ndarray, V: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """S = softmax(q K^T / sqrt(D)),  X = S V  for one head (Section 2.1).

    q: [D], K: [T, D], V: [T, D]; any real dtype, evaluated in float64.
    Returns (X [D], S [T]).
    """
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    D = q.shape[0]
    a = (K @ q) / math.sqrt(D)
    a = a - a.max()
    e = np.exp(a)
    S = e / e.sum()
    X = S @ V
    return X, S


# ----------------------------------------------------------------------------
# Section 2.1, prompt encoding: every prompt token attends to itself and to the
# tokens before it.  Section 4.2 "attention window" needs, when generation
# starts, the scores each token received in the last n steps: those are the last
# n rows of the prompt's causal score matrix.  The paper does not say which keys
# the prompt's scores are taken over; reading: the unquantized ones (the prompt
# is encoded before anything is quantized).
# ----------------------------------------------------------------------------
def prefill_score_rows(q_last: np.ndarray, K: np.ndarray) -> List[np.ndarray]:
    """Last n causal score rows of one head.  q_last: [n, D], the queries of prompt
    positions T-n .. T-1; K: [T, D].  Row i is softmax(q_i K[:T-n+i+1]^T / sqrt(D)),
    of length T-n+i+1 (a token does not attend to later ones).  float64."""
    q_last = np.asarray(q_last, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    n, D = q_last.shape
    T = K.shape[0]
    assert 1 <= n <= T
    rows = []
    for i in range(n):
        length = T - n + i + 1
        a = (K[:length] @ q_last[i]) / math.sqrt(D)
        e = np.exp(a - a.max())
        rows.append(e / e.sum())
    return rows


# ----------------------------------------------------------------------------
# Section 4.2 "Outliers": values beyond the alpha% quantile at both ends stay
# unquantized in a sparse side store.
# Reading: the population of the quantile is the token vector (the same group
# whose [min, max] the quantizer of Section 4.1 uses); alpha is the total over
# both ends, so each end keeps ceil(alpha/2 * D) values; ties go to the lower
# channel.  Bottom outliers are picked among what is left after the top ones.
# ----------------------------------------------------------------------------
def outliers_per_side(alpha: float, D: int) -> int:
    if alpha <= 0.0:
        return 0
    return int(math.ceil(alpha / 2.0 * D - 1e-12))


def outlier_split(x: np.ndarray, n_o: int) -> np.ndarray:
    """x: fp16 [N, D].  Returns bool mask [N, D], True at outlier channels.

    Exactly n_o largest and n_o smallest entries of every row are marked.
    """
    x = np.asarray(x, dtype=F16)
    N, D = x.shape
    mask = np.zeros((N, D), dtype=bool)
    if n_o == 0:
        return mask
    assert D - 2 * n_o >= 1, "a token vector must keep at least one regular value"
    xf = x.astype(np.float64)
    rows = np.arange(N)[:, None]
    # n_o largest, equal values -> lower channel first (stable sort on -x).
    top = np.argsort(-xf, axis=1, kind="stable")[:, :n_o]
    mask[rows, top] = True
    # n_o smallest among the remaining ones.
    rest = np.where(mask, np.inf, xf)
    bot = np.argsort(rest, axis=1, kind="stable")[:, :n_o]
    mask[rows, bot] = True
    return mask


def outlier_split_threshold(x: np.ndarray, lo: float, hi: float, cap: int) -> np.ndarray:
    """Variant of Section 4.2 "Outliers" read literally: an outlier is a value outside fixed
    thresholds [lo, hi] (calibrated once as the alpha/2 and 1 - alpha/2 quantiles of a
    population, see calibrate_outlier_thresholds), so a token has a variable number of them.
    A token keeps at most `cap` per end: the `cap` largest of those above hi and the `cap`
    smallest of those below lo (equal values: lower channel first).  x: fp16 [N, D];
    thresholds are compared as fp32 numbers, strictly.  Returns the bool mask [N, D]."""
    x = np.asarray(x, dtype=F16)
    N, D = x.shape
    assert D - 2 * cap >= 1 and lo <= hi
    xf = x.astype(F32)
    mask = np.zeros((N, D), dtype=bool)
    if cap == 0:
        return mask
    rows = np.arange(N)[:, None]
    top = np.argsort(-xf.astype(np.float64), axis=1, kind="stable")[:, :cap]
    mask[rows, top] = xf[rows, top] > F32(hi)
    bot = np.argsort(xf.astype(np.float64), axis=1, kind="stable")[:, :cap]
    mask[rows, bot] |= xf[rows, bot] < F32(lo)
    return mask


def calibrate_outlier_thresholds(population: np.ndarray, alpha: float) -> Tuple[np.float32, np.float32]:
    """The two thresholds that make a fraction alpha (alpha/2 per end) of a calibration
    population outliers: the lower and upper empirical quantiles, taken as order statistics
    (elements of the population, hence fp16 numbers): exactly floor(alpha/2 * N) values lie
    strictly above hi, and as many strictly below lo, unless equal values straddle the cut."""
    v = np.sort(np.asarray(population, dtype=F16).astype(F32).reshape(-1))
    k = int(math.floor(alpha / 2.0 * v.size))
    return F32(v[k]), F32(v[v.size - 1 - k])


def token_range(x: np.ndarray, omask: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """min_t and max_t over the non-outlier entries of each token (Section 4.1,
    "Determining quantization bits"; Section 4.2 benefit 2).  fp16 in, fp16 out
    (both are elements of the input, hence exact)."""
    xf = np.asarray(x, dtype=F16).astype(F32)
    mn = np.where(omask, np.inf, xf).min(axis=1)
    mx = np.where(omask, -np.inf, xf).max(axis=1)
    return mn.astype(F16), mx.astype(F16)


def range_f32(mn: np.ndarray, mx: np.ndarray) -> np.ndarray:
    """range = fl32(float(max) - float(min))."""
    return (np.asarray(mx, dtype=F16).astype(F32) - np.asarray(mn, dtype=F16).astype(F32)).astype(F32)


# ----------------------------------------------------------------------------
# Section 4.1 "Determining quantization bits": split [min_t, max_t] into 2^B
# equal segments, represent a value by its segment, reconstruct at the midpoint.
# The fp32 operation order below is the contract for bit-exact codes.
# ----------------------------------------------------------------------------
def encode(x: np.ndarray, mn: np.ndarray, mx: np.ndarray, bits: np.ndarray) -> np.ndarray:
    """x fp16 [N, D]; mn, mx fp16 [N]; bits int [N].  Returns uint8 codes [N, D].

    code = clamp(floor(fl32(fl32(x - min) * inv)), 0, 2^B - 1), inv = fl32(2^B / range);
    a token with range 0 gets code 0 everywhere.  Outlier channels are encoded
    like any other (they clamp to 0 or 2^B-1); their exact value lives in the
    side store.
    """
    xf = np.asarray(x, dtype=F16).astype(F32)
    mnf = np.asarray(mn, dtype=F16).astype(F32)[:, None]
    rng = range_f32(mn, mx)
    bits = np.asarray(bits).astype(np.int64)
    levels = np.ldexp(F32(1.0), bits).astype(F32)            # 2^B, exact
    with np.errstate(divide="ignore", invalid="ignore"):
        inv = (levels / rng).astype(F32)                      # one correctly rounded division
    diff = (xf - mnf).astype(F32)
    with np.errstate(invalid="ignore"):
        prod = (diff * inv[:, None]).astype(F32)          # 0 * inf only where range == 0
    c = np.floor(prod)
    c = np.clip(c, 0.0, (levels - F32(1.0))[:, None])
    c = np.where((rng > 0)[:, None], c, 0.0)
    return c.astype(np.uint8)


def decode(codes: np.ndarray, mn: np.ndarray, mx: np.ndarray, bits: np.ndarray) -> np.ndarray:
    """Midpoint reconstruction in fp32: fl32(fl32((c + 0.5) * scale) + min),
    scale = range * 2^-B (exact scaling).  Returns float32 [N, D]."""
    mnf = np.asarray(mn, dtype=F16).astype(F32)[:, None]
    rng = range_f32(mn, mx)
    bits = np.asarray(bits).astype(np.int64)
    scale = np.ldexp(rng, -bits).astype(F32)
    half = (codes.astype(F32) + F32(0.5)).astype(F32)          # exact
    return ((half * scale[:, None]).astype(F32) + mnf).astype(F32)


def dequantize(codes, mn, mx, bits, omask, x_outlier_src) -> np.ndarray:
    """decode(), then the outlier channels take their stored fp16 value exactly
    (Section 4.2 benefit 1).  x_outlier_src: fp16 [N, D] holding the stored
    values at the masked positions (other positions are ignored)."""
    xh = decode(codes, mn, mx, bits)
    return np.where(omask, np.asarray(x_outlier_src, dtype=F16).astype(F32), xh).astype(F32)


def pack_canonical(codes_row: np.ndarray, bits: int) -> np.ndarray:
    """Canonical packed form of one token: channel d occupies bits
    [d*B, (d+1)*B) of a little-endian bit string; D*B/8 bytes."""
    D = codes_row.shape[0]
    b = ((codes_row.astype(np.uint16)[:, None] >> np.arange(bits)) & 1).astype(np.uint8)  # [D, B], LSB first
    return np.packbits(b.reshape(-1), bitorder="little")[: (D * bits + 7) // 8]


def requantize_codes(codes: np.ndarray, old_bits: np.ndarray, new_bits: np.ndarray) -> np.ndarray:
    """Section 4.2 "Integration": going to fewer bits keeps [min, max] and drops
    the low code bits (segments of the finer grid nest in those of the coarser
    one).  Only defined for new_bits <= old_bits."""
    sh = (np.asarray(old_bits).astype(np.int64) - np.asarray(new_bits).astype(np.int64))
    assert (sh >= 0).all()
    return (codes.astype(np.uint16) >> sh[:, None].astype(np.uint16)).astype(np.uint8)


# ----------------------------------------------------------------------------
# Section 4.1: bounds on the per-token noise, turned into thresholds.
# ----------------------------------------------------------------------------
def key_variance_bound(T: int, sigma_s_max: float, qnorm2: float) -> float:
    """sigma_K^2 <= log(T^3/(T-1) * sigma_Smax^2 + 1) / sum_d Q_d^2
    (last display of "Key cache quantization").  qnorm2 is the caller's
    statistic of the squared query norm (the paper uses its upper-10% quantile);
    the reading taken here is that the query in this formula already carries the
    1/sqrt(D) of the softmax argument, i.e. qnorm2 = quantile(|q|^2) / D."""
    if T < 2:
        return math.inf
    return math.log1p(float(T) ** 3 / (T - 1.0) * sigma_s_max ** 2) / qnorm2


def score_variance_model(T: int, var_k: float, qnorm2: float) -> float:
    """The paper's model of Var[S_t] that the key bound inverts:
    (1/T^2)(1 - 1/T)(exp(qnorm2 * var_k) - 1).  (The display before it prints the
    mean/variance ratio upside down; the line used here and the final bound agree
    with each other.)"""
    return (1.0 / T ** 2) * (1.0 - 1.0 / T) * math.expm1(qnorm2 * var_k)


def key_threshold(T: int, sigma_s_max: float, qnorm2: float) -> np.float32:
    """tau_K = 2*sqrt(3)*sigma_K, computed in double, rounded once to fp32.
    B_K = ceil(log2(range / tau_K)) <= b  <=>  range <= 2^b * tau_K."""
    v = key_variance_bound(T, sigma_s_max, qnorm2)
    return F32(2.0 * math.sqrt(3.0) * math.sqrt(v)) if math.isfinite(v) else F32(np.inf)


def value_threshold(T: int, sigma_x_max: float) -> np.float32:
    """c_V = 2*sqrt(3)*sigma_Xmax/sqrt(T), double then one rounding to fp32.
    With sigma_V <= sigma_Xmax / (sqrt(T) |S_t|) ("Value cache quantization"),
    B_V <= b  <=>  range * S_t <= 2^b * c_V."""
    return F32(2.0 * math.sqrt(3.0) * sigma_x_max / math.sqrt(T))


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Finite fp32 numbers rounded to bfloat16 (8 significant bits, fp32's exponent range),
    ties to even, returned as fp32: on the bit pattern, add half a unit of the kept part
    (one less when the kept part is even) and clear the 16 dropped bits."""
    u = np.ascontiguousarray(x, dtype=F32).view(np.uint32).astype(np.uint64)
    r = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16
    return r.astype(np.uint32).view(F32).reshape(np.shape(x))


def window_predict(history: Sequence[np.ndarray], n: int, T: int) -> np.ndarray:
    """Section 3.2 / 4.2 "attention window": predicted score of a token = max of
    its last n observed scores.  history: list of score rows (oldest first), row
    r has the scores of the tokens that existed at that step (length <= T).
    Tokens seen fewer than n times use what exists; never-seen tokens get 0."""
    pred = np.zeros(T, dtype=F32)
    for row in list(history)[-n:]:
        row = np.asarray(row, dtype=F32)
        pred[: row.shape[0]] = np.maximum(pred[: row.shape[0]], row)
    return pred


def gqa_reduce(scores_q: np.ndarray, n_kv_heads: int) -> np.ndarray:
    """scores_q: [Hq, T] -> [Hkv, T], max over the query heads that share a KV
    head (the value bound has to hold for each of them; not in the paper, which
    only treats one query per KV head)."""
    Hq, T = scores_q.shape
    G = Hq // n_kv_heads
    return np.asarray(scores_q, dtype=F32).reshape(n_kv_heads, G, T).max(axis=1)


def snap_bits_from_compare(lhs: np.ndarray, thr: np.float32, bit_set: Sequence[int]) -> np.ndarray:
    """Smallest b in bit_set with lhs <= fl32(2^b * thr); the largest b if none."""
    bit_set = sorted(bit_set)
    out = np.full(lhs.shape, bit_set[-1], dtype=np.int16)
    for b in reversed(bit_set):
        lim = F32(np.ldexp(F32(thr), b))
        out = np.where(lhs <= lim, np.int16(b), out)
    return out


def select_bits_key(range_k: np.ndarray, tau_k: np.float32, bit_set=DEFAULT_BIT_SET) -> np.ndarray:
    return snap_bits_from_compare(np.asarray(range_k, dtype=F32), tau_k, bit_set).astype(np.uint8)


def select_bits_value(range_v: np.ndarray, s_pred: np.ndarray, c_v: np.float32, bit_set=DEFAULT_BIT_SET) -> np.ndarray:
    lhs = (np.asarray(range_v, dtype=F32) * np.asarray(s_pred, dtype=F32)).astype(F32)
    return snap_bits_from_compare(lhs, c_v, bit_set).astype(np.uint8)


def bits_formula_f64(range_, sigma) -> np.ndarray:
    """The printed rule itself, B = ceil(log2(range / (2 sqrt(3) sigma))), in
    double precision (used only to pin the compare form above)."""
    with np.errstate(divide="ignore"):
        return np.ceil(np.log2(np.asarray(range_, dtype=np.float64) / (2.0 * math.sqrt(3.0) * np.asarray(sigma, dtype=np.float64))))


# ----------------------------------------------------------------------------
# One (sequence, KV head) worth of quantized cache and the per-step procedure of
# Section 4.2 "Integration in text generation process".
# ----------------------------------------------------------------------------
@dataclass
class HeadCache:
    D: int
    n_o: int                               # outliers per end; with thresholds: the most a token keeps per end
    thr: Optional[Tuple[float, float]] = None   # (lo, hi): the threshold variant of the outlier rule
    bits: np.ndarray = field(default_factory=lambda: np.zeros(0, np.uint8))
    mn: np.ndarray = field(default_factory=lambda: np.zeros(0, F16))
    mx: np.ndarray = field(default_factory=lambda: np.zeros(0, F16))
    omask: Optional[np.ndarray] = None     # [T, D] bool
    oval: Optional[np.ndarray] = None      # [T, D] fp16, meaningful where omask
    codes: Optional[np.ndarray] = None     # [T, D] uint8 at width bits[t]

    def __post_init__(self):
        if self.omask is None:
            self.omask = np.zeros((0, self.D), bool)
            self.oval = np.zeros((0, self.D), F16)
            self.codes = np.zeros((0, self.D), np.uint8)

    @property
    def T(self) -> int:
        return self.bits.shape[0]

    def append(self, x: np.ndarray, bits: np.ndarray) -> None:
        x = np.asarray(x, dtype=F16).reshape(-1, self.D)
        bits = np.asarray(bits, dtype=np.uint8).reshape(-1)
        om = outlier_split(x, self.n_o) if self.thr is None else outlier_split_threshold(x, self.thr[0], self.thr[1], self.n_o)
        mn, mx = token_range(x, om)
        c = encode(x, mn, mx, bits)
        self.bits = np.concatenate([self.bits, bits])
        self.mn = np.concatenate([self.mn, mn])
        self.mx = np.concatenate([self.mx, mx])
        self.omask = np.concatenate([self.omask, om])
        self.oval = np.concatenate([self.oval, np.where(om, x, F16(0))])
        self.codes = np.concatenate([self.codes, c])

    def requantize(self, new_bits: np.ndarray, originals: Optional[np.ndarray]) -> int:
        """Lower width: shift the codes.  Higher width: re-encode from the
        caller's unquantized copy with the stored [min, max] (which, like the
        outlier set, does not depend on the width).  Without that copy the token
        keeps its width; the number of such refusals is returned."""
        new_bits = np.asarray(new_bits, dtype=np.uint8)
        assert new_bits.shape[0] == self.T
        refused = 0
        down = new_bits < self.bits
        if down.any():
            self.codes[down] = requantize_codes(self.codes[down], self.bits[down], new_bits[down])
            self.bits[down] = new_bits[down]
        up = new_bits > self.bits
        if up.any():
            if originals is None:
                refused = int(up.sum())
            else:
                xo = np.asarray(originals, dtype=F16)[up]
                self.codes[up] = encode(xo, self.mn[up], self.mx[up], new_bits[up])
                self.bits[up] = new_bits[up]
        return refused

    def dequantize(self) -> np.ndarray:
        return dequantize(self.codes, self.mn, self.mx, self.bits, self.omask, self.oval)

    def ranges(self) -> np.ndarray:
        return range_f32(self.mn, self.mx)

    def outlier_lists(self) -> Tuple[np.ndarray, np.ndarray]:
        """Side store as sorted-by-channel lists: idx uint8 [T, 2 n_o], val fp16 [T, 2 n_o].
        With thresholds a token may have fewer: the rest of its row is (255, 0)."""
        k = 2 * self.n_o
        idx = np.full((self.T, k), 255 if self.thr is not None else 0, np.uint8)
        val = np.zeros((self.T, k), F16)
        for t in range(self.T):
            ch = np.nonzero(self.omask[t])[0]
            idx[t, : len(ch)] = ch
            val[t, : len(ch)] = self.oval[t, ch]
        return idx, val

    def packed(self, t: int) -> np.ndarray:
        return pack_canonical(self.codes[t], int(self.bits[t]))


@dataclass
class Config:
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    bit_set: Tuple[int, ...] = DEFAULT_BIT_SET
    outlier_frac: float = 0.01
    n_outlier_per_side: int = -1
    window: int = 5
    sigma_s_max: float = 1e-3
    sigma_x_max: float = 1e-2
    qnorm2: Optional[np.ndarray] = None   # [n_kv_heads]
    window_fp16: bool = False             # variant: the window keeps its score rows in fp16
    window_bf16: bool = False             # variant: ... in bfloat16
    outlier_thresholds: Optional[np.ndarray] = None   # variant: fp32 [2 (K, V), n_kv_heads, 2 (lo, hi)]; then
                                                      # n_outlier_per_side (or the count alpha gives) caps a token's outliers per end

    def n_o(self) -> int:
        if self.n_outlier_per_side >= 0:
            return self.n_outlier_per_side
        return outliers_per_side(self.outlier_frac, self.head_dim)


class OracleCache:
    """The whole cache of one layer: batch x KV heads of HeadCache pairs, plus the
    score history that the attention window needs."""

    def __init__(self, cfg: Config):
        self.cfg = cfg
        B, H, D = cfg.batch, cfg.n_kv_heads, cfg.head_dim
        thr = cfg.outlier_thresholds
        pair = lambda side, h: None if thr is None else (float(thr[side][h][0]), float(thr[side][h][1]))
        self.K = [[HeadCache(D, cfg.n_o(), pair(0, h)) for h in range(H)] for _ in range(B)]
        self.V = [[HeadCache(D, cfg.n_o(), pair(1, h)) for h in range(H)] for _ in range(B)]
        self.history: List[np.ndarray] = []     # rows [B, Hkv, T_row], oldest first
        self.refused = 0

    @property
    def T(self) -> int:
        return self.K[0][0].T

    def append(self, k: np.ndarray, v: np.ndarray, k_bits=None, v_bits=None) -> None:
        """k, v: fp16 [B, Hkv, n_new, D]; bits uint8 [B, Hkv, n_new] or None (= widest)."""
        cfg = self.cfg
        n_new = k.shape[2]
        wide = max(cfg.bit_set)
        for b in range(cfg.batch):
            for h in range(cfg.n_kv_heads):
                kb = np.full(n_new, wide, np.uint8) if k_bits is None else k_bits[b, h]
                vb = np.full(n_new, wide, np.uint8) if v_bits is None else v_bits[b, h]
                self.K[b][h].append(k[b, h], kb)
                self.V[b][h].append(v[b, h], vb)

    def observe(self, scores: np.ndarray) -> None:
        """scores: fp32 [B, Hq, T] normalised attention of one decode step."""
        cfg = self.cfg
        row = np.stack([gqa_reduce(scores[b], cfg.n_kv_heads) for b in range(cfg.batch)])
        if cfg.window_fp16:
            # Section 4.2 "attention window" keeps scores, not a precision: a variant stores them
            # as fp16 (round to nearest even); the predicted score is the maximum of the
            # stored values, this step's included.
            row = row.astype(F16)
        elif cfg.window_bf16:
            row = round_to_bf16(row)
        self.history.append(row.astype(F32))
        self.history = self.history[-cfg.window:]

    def prefill(self, q_last: np.ndarray, k: np.ndarray, v: np.ndarray, score_rows=None):
        """Prompt encoding (Section 2.1) followed by the first quantization (Section 4.2):
        the last n causal score rows of the prompt (from the unquantized keys) become the
        window, every prompt token gets the width the rules give for T = prompt length,
        and is quantized at it.  q_last: fp16 [B, Hq, n, D]; k, v: fp16 [B, Hkv, T, D].
        score_rows: n arrays fp32 [B, Hq, T-n+i+1] to use instead of computing them (a
        caller that has to take the width decisions from given fp32 numbers).
        Returns (k_bits, v_bits, rows)."""
        cfg = self.cfg
        assert self.T == 0
        G = cfg.n_q_heads // cfg.n_kv_heads
        n = q_last.shape[2]
        if score_rows is None:
            per_head = [[prefill_score_rows(q_last[b, hq], k[b, hq // G]) for hq in range(cfg.n_q_heads)]
                        for b in range(cfg.batch)]
            score_rows = [np.stack([np.stack([per_head[b][hq][i] for hq in range(cfg.n_q_heads)])
                                    for b in range(cfg.batch)]).astype(F32) for i in range(n)]
        self.append(k, v)             # widest width: fixes [min, max] and the outliers
        for row in score_rows:
            self.observe(row)
        bk, bv = self.select_bits()
        self.requantize(bk, bv)       # narrowing only; equals direct quantization at that width
        return bk, bv, score_rows

    def select_bits(self) -> Tuple[np.ndarray, np.ndarray]:
        """Bits for all T cached tokens from the current window (Section 4.2:
        "calculate the quantization bits for all existing tokens")."""
        cfg = self.cfg
        B, H, T = cfg.batch, cfg.n_kv_heads, self.T
        bk = np.zeros((B, H, T), np.uint8)
        bv = np.zeros((B, H, T), np.uint8)
        c_v = value_threshold(T, cfg.sigma_x_max)
        for b in range(B):
            for h in range(H):
                tau = key_threshold(T, cfg.sigma_s_max, float(cfg.qnorm2[h]))
                pred = window_predict([r[b, h] for r in self.history], cfg.window, T)
                bk[b, h] = select_bits_key(self.K[b][h].ranges(), tau, cfg.bit_set)
                bv[b, h] = select_bits_value(self.V[b][h].ranges(), pred, c_v, cfg.bit_set)
        return bk, bv

    def requantize(self, bk, bv, k_orig=None, v_orig=None) -> None:
        cfg = self.cfg
        for b in range(cfg.batch):
            for h in range(cfg.n_kv_heads):
                self.refused += self.K[b][h].requantize(bk[b, h], None if k_orig is None else k_orig[b, h])
                self.refused += self.V[b][h].requantize(bv[b, h], None if v_orig is None else v_orig[b, h])

    def dequantize(self) -> Tuple[np.ndarray, np.ndarray]:
        cfg = self.cfg
        K = np.stack([np.stack([self.K[b][h].dequantize() for h in range(cfg.n_kv_heads)]) for b in range(cfg.batch)])
        V = np.stack([np.stack([self.V[b][h].dequantize() for h in range(cfg.n_kv_heads)]) for b in range(cfg.batch)])
        return K, V

    def decode_attention(self, q: np.ndarray, k_new=None, v_new=None) -> Tuple[np.ndarray, np.ndarray]:
        """q fp16 [B, Hq, D]; k_new, v_new fp16 [B, Hkv, D] or None.  The new
        token takes part unquantized (Section 4.2: the new token "combined with
        the quantized KV cache of previous tokens").  Returns X [B, Hq, D] and
        S [B, Hq, T(+1)] in float64."""
        cfg = self.cfg
        G = cfg.n_q_heads // cfg.n_kv_heads
        Kh, Vh = self.dequantize()
        Xs, Ss = [], []
        for b in range(cfg.batch):
            xr, sr = [], []
            for hq in range(cfg.n_q_heads):
                h = hq // G
                Kc = Kh[b, h].astype(np.float64)
                Vc = Vh[b, h].astype(np.float64)
                if k_new is not None:
                    Kc = np.concatenate([Kc, np.asarray(k_new[b, h], F16).astype(np.float64)[None]])
                    Vc = np.concatenate([Vc, np.asarray(v_new[b, h], F16).astype(np.float64)[None]])
                X, S = attention(np.asarray(q[b, hq], F16).astype(np.float64), Kc, Vc)
                xr.append(X)
                sr.append(S)
            Xs.append(np.stack(xr))
            Ss.append(np.stack(sr))
        return np.stack(Xs), np.stack(Ss)

    # -- accounting (Section 2.1: memory "calculated by the quantized bit") ----
    def code_bytes(self) -> int:
        D = self.cfg.head_dim
        n = 0
        for side in (self.K, self.V):
            for row in side:
                for hc in row:
                    n += int(hc.bits.astype(np.int64).sum()) * D // 8
        return n

    def ratio_codes(self) -> float:
        """fp16 bytes over code bytes = 32 / mean(bK + bV)."""
        cfg = self.cfg
        n_tok = cfg.batch * cfg.n_kv_heads * self.T
        return (n_tok * cfg.head_dim * 2 * 2) / self.code_bytes()

    def ratio_all(self) -> float:
        """fp16 bytes over everything stored: codes, fp16 min/max, one width tag
        per side, and (u8 channel, fp16 value) per outlier."""
        cfg = self.cfg
        n_tok = cfg.batch * cfg.n_kv_heads * self.T
        if cfg.outlier_thresholds is None:
            meta = n_tok * (8 + 2 + 2 * 2 * cfg.n_o() * 3)
        else:   # a variable number of entries per token, plus (u16 offset, u8 count) per token and side
            entries = sum(int(hc.omask.sum()) for side in (self.K, self.V) for row in side for hc in row)
            meta = n_tok * (8 + 2 + 2 * 3) + entries * 3
        return (n_tok * cfg.head_dim * 2 * 2) / (self.code_bytes() + meta)


def query_norm_statistic(queries: np.ndarray, D: int, upper: float = 0.10) -> float:
    """"Upper 10% quantile" of the squared query norm (Section 4.1), i.e. its
    0.9-quantile (linear interpolation), divided by D (see key_variance_bound)."""
    n2 = (np.asarray(queries, dtype=np.float64) ** 2).sum(axis=-1).reshape(-1)
    return float(np.quantile(n2, 1.0 - upper)) / D
