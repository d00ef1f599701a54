"""Outliers by thresholds (a variant: Section 4.2 "Outliers" read literally -- values outside
thresholds calibrated as quantiles of a population, hence a variable number per token, kept in a
variable-length side store): every step of the path against the oracle, bit for bit for the
cache, within 2e-3 for the attention."""
import numpy as np
import pytest

from oracle import qaq_oracle as O
from paper_2403_04643_amd import workloads as W
from tests.parity_util import F16, F32, attention_errors, compare_canonical, dev, make_pair

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _thresholds(K, V, alpha):
    """[2 (K, V)][Hkv][2 (lo, hi)], each KV head calibrated on its own values."""
    return np.array([[O.calibrate_outlier_thresholds(X[:, h], alpha) for h in range(X.shape[1])] for X in (K, V)], F32)


def _check_attention(oc, gc, q, kn=None, vn=None, tag=""):
    X, S = gc.decode_attention(dev(q), None if kn is None else dev(kn), None if vn is None else dev(vn), want_scores=True)
    Xo, So = oc.decode_attention(q, kn, vn)
    ex, es = attention_errors(X.cpu().numpy(), S.cpu().numpy(), Xo, So)
    assert ex.max() < TOL and es.max() < TOL, (tag, ex.max(), es.max())
    return S


@pytest.mark.parametrize("head_dim,context,cap,alpha,bit_set", [
    (128, 700, 4, 0.01, (2, 3, 4, 8)), (64, 300, 2, 0.03, (2, 3, 4, 8)), (128, 260, 1, 0.01, (1, 2, 3, 4, 8)), (64, 37, 4, 0.2, (2, 4))])
def test_append_requantize_export_dequantize(head_dim, context, cap, alpha, bit_set):
    sh = W.shape(2, batch=2, n_q_heads=3, n_kv_heads=3, head_dim=head_dim, context=context)
    print(f"threshold outliers: {sh} cap={cap} alpha={alpha}", flush=True)
    K, V = W.make_kv(2, sh)
    thr = _thresholds(K, V, alpha)
    rng = np.random.default_rng(13)
    oc, gc = make_pair(sh, 0.01, bit_set=bit_set, n_outlier_per_side=cap, outlier_thresholds=thr)
    widths = np.array(bit_set, np.uint8)
    bk, bv = rng.choice(widths, size=K.shape[:3]), rng.choice(widths, size=K.shape[:3])
    cut = context // 3
    for lo, hi in ((0, cut), (cut, context)):        # the second call lands in a partly filled tile
        oc.append(K[:, :, lo:hi], V[:, :, lo:hi], bk[:, :, lo:hi], bv[:, :, lo:hi])
        gc.quantize_append(dev(K[:, :, lo:hi]), dev(V[:, :, lo:hi]), dev(bk[:, :, lo:hi]), dev(bv[:, :, lo:hi]))
    compare_canonical(oc, gc, "append")
    counts = np.stack([np.stack([hc.omask.sum(1) for hc in row]) for row in oc.K])
    print(f"  outliers per key token: min {counts.min()} mean {counts.mean():.2f} max {counts.max()}", flush=True)
    assert counts.min() < counts.max()               # a variable number per token
    Kd, Vd = gc.dequantize()
    Ko, Vo = oc.dequantize()
    np.testing.assert_array_equal(Kd.cpu().numpy().view(np.uint16), Ko.astype(F16).view(np.uint16))
    np.testing.assert_array_equal(Vd.cpu().numpy().view(np.uint16), Vo.astype(F16).view(np.uint16))
    q = W.make_queries(2, sh)[0]
    _check_attention(oc, gc, q, tag="append")
    b2k, b2v = rng.choice(widths, size=K.shape[:3]), rng.choice(widths, size=K.shape[:3])
    oc.requantize(b2k, b2v, K, V); gc.requantize(dev(b2k), dev(b2v), dev(K), dev(V))
    compare_canonical(oc, gc, "requantized")
    _check_attention(oc, gc, q, tag="requantized")
    st = gc.stats()
    entries = sum(int(hc.omask.sum()) for side in (oc.K, oc.V) for row in side for hc in row)
    th = sh.batch * sh.n_kv_heads * context
    assert st.meta_bytes == 2 * th * (4 + 1 + 3) + 3 * entries


def test_decode_steps():
    sh = W.shape(3, batch=2, n_q_heads=4, n_kv_heads=2, head_dim=128, context=500)
    steps = 14
    K, V = W.make_kv(3, sh)
    thr = _thresholds(K, V, 0.01)
    qn = O.query_norm_statistic(W.make_queries(3, sh, n=64, seed_offset=9), sh.head_dim)
    oc, gc = make_pair(sh, qn, max_tokens=sh.context + steps, window=3, n_outlier_per_side=4,
                       outlier_thresholds=thr, sigma_s_max=2.5e-4, sigma_x_max=0.05)
    q_last = np.ascontiguousarray(W.make_queries(3, sh, n=3, seed_offset=8).transpose(1, 2, 0, 3))
    rows = gc.prefill_window(dev(q_last), dev(K)).cpu().numpy()
    bk_g, bv_g = gc.quantize_append_selected(dev(K), dev(V), want_bits=True)
    T = sh.context
    bk_o, bv_o, _ = oc.prefill(q_last, K, V, score_rows=[rows[i][..., : T - 3 + i + 1] for i in range(3)])
    np.testing.assert_array_equal(bk_g.cpu().numpy(), bk_o)
    np.testing.assert_array_equal(bv_g.cpu().numpy(), bv_o)
    compare_canonical(oc, gc, "prompt")
    Korig, Vorig = K.copy(), V.copy()
    qs = W.make_queries(3, sh, n=steps)
    for s in range(steps):
        kn, vn = W.make_new_token(3, sh, step=s)
        S = _check_attention(oc, gc, qs[s], kn, vn, tag=f"step {s}")
        Korig = np.concatenate([Korig, kn[:, :, None]], 2); Vorig = np.concatenate([Vorig, vn[:, :, None]], 2)
        with_orig = s % 3 != 1
        oc.append(kn[:, :, None], vn[:, :, None])
        oc.observe(S.cpu().numpy())
        bk_o, bv_o = oc.select_bits()
        oc.requantize(bk_o, bv_o, Korig if with_orig else None, Vorig if with_orig else None)
        bk_g, bv_g = gc.decode_update(S, dev(kn), dev(vn), dev(Korig) if with_orig else None, dev(Vorig) if with_orig else None, want_bits=True)
        np.testing.assert_array_equal(bk_g.cpu().numpy(), bk_o, err_msg=f"step {s}")
        np.testing.assert_array_equal(bv_g.cpu().numpy(), bv_o, err_msg=f"step {s}")
    compare_canonical(oc, gc, "after decode steps")
