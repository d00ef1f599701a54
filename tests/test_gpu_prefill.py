"""GPU parity of the prompt-encoding path: the last n causal score rows of a prompt computed
from the unquantized keys (qaq_prefill_window), installed as the attention window, and the
first quantization at the widths the rules give from that window
(qaq_quantize_append_selected), against the CPU oracle.  Scores within 2e-3 of the row
maximum; widths, [min,max], outliers and codes bit for bit (the oracle takes its width
decisions from the fp32 score rows the library emitted, which are themselves checked)."""
import numpy as np
import pytest

from oracle import qaq_oracle as O
from paper_2403_04643_amd import qaq, workloads as W
from tests.parity_util import F16, F32, attention_errors, compare_canonical, dev, make_pair

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _log(msg):
    print(msg, flush=True)


def _check_rows(rows_gpu, q_last, K, G, units=None):
    """rows_gpu: [n, B, Hq, T]; q_last: [B, Hq, n, D]; K: [B, Hkv, T, D]."""
    n, B, Hq, T = rows_gpu.shape
    worst = 0.0
    for b in range(B):
        for hq in range(Hq):
            if units is not None and (b, hq // G) not in units:
                continue
            ref = O.prefill_score_rows(q_last[b, hq], K[b, hq // G])
            for i in range(n):
                length = T - n + i + 1
                got = rows_gpu[i, b, hq]
                assert (got[length:] == 0).all(), "a token must not receive weight from an earlier query"
                err = np.abs(got[:length].astype(np.float64) - ref[i]).max() / ref[i].max()
                worst = max(worst, err)
                assert err < TOL, f"row {i} b={b} hq={hq}: {err:.2e}"
    np.testing.assert_allclose(rows_gpu.sum(-1, dtype=np.float64), 1.0, rtol=2e-5)
    return worst


@pytest.mark.parametrize("name,over,n,kw", [
    ("three tiles, ragged tail", dict(batch=2, n_q_heads=8, n_kv_heads=4, context=600), 5,
     dict(window=5, sigma_s_max=4e-4, sigma_x_max=6e-3)),
    ("8 query heads per KV head, 40 query rows, D=64", dict(batch=1, n_q_heads=8, n_kv_heads=1, head_dim=64, context=300), 5,
     dict(window=5, sigma_s_max=1e-3, sigma_x_max=1e-2)),
    ("one row, less than a tile", dict(batch=2, n_q_heads=4, n_kv_heads=4, context=17), 1,
     dict(window=1, sigma_s_max=2e-3, sigma_x_max=5e-2)),
    ("fewer rows than the window", dict(batch=1, n_q_heads=4, n_kv_heads=2, context=257), 2,
     dict(window=5, sigma_s_max=4e-4, sigma_x_max=1e-2)),
    ("as many rows as tokens", dict(batch=1, n_q_heads=2, n_kv_heads=2, context=3), 3,
     dict(window=4, sigma_s_max=2e-3, sigma_x_max=5e-2)),
])
def test_prefill_window_and_first_quantization(name, over, n, kw):
    sh = W.shape(3, **over)
    _log(f"prefill case: {name}: {sh} rows={n}")
    G = sh.n_q_heads // sh.n_kv_heads
    T = sh.context
    K, V = W.make_kv(3, sh)
    q_last = np.ascontiguousarray(W.make_queries(3, sh, n=n, seed_offset=4).transpose(1, 2, 0, 3))   # [B, Hq, n, D]
    qn = O.query_norm_statistic(W.make_queries(3, sh, n=64, seed_offset=9), sh.head_dim)
    steps = 2
    oc, gc = make_pair(sh, qn, max_tokens=T + steps, **kw)

    rows = gc.prefill_window(dev(q_last), dev(K)).cpu().numpy()
    worst = _check_rows(rows, q_last, K, G)
    _log(f"  worst score error {worst:.2e}")
    bk_g, bv_g = gc.quantize_append_selected(dev(K), dev(V), want_bits=True)
    assert gc.length() == T

    bk_o, bv_o, _ = oc.prefill(q_last, K, V, score_rows=[rows[i][..., : T - n + i + 1] for i in range(n)])
    np.testing.assert_array_equal(bk_g.cpu().numpy(), bk_o)
    np.testing.assert_array_equal(bv_g.cpu().numpy(), bv_o)
    compare_canonical(oc, gc, name)
    if T > 100:
        assert len(np.unique(bv_o)) > 1, "the case must exercise several value widths"

    # generation goes on from this state: the window rows must be the ones the next steps use
    Korig, Vorig = K.copy(), V.copy()
    qs = W.make_queries(3, sh, n=steps)
    for s in range(steps):
        kn, vn = W.make_new_token(3, sh, step=s)
        X, S = gc.decode_attention(dev(qs[s]), dev(kn), dev(vn), want_scores=True)
        Xo, So = oc.decode_attention(qs[s], kn, vn)
        ex, es = attention_errors(X.cpu().numpy(), S.cpu().numpy(), Xo, So)
        assert ex.max() < TOL and es.max() < TOL
        Korig = np.concatenate([Korig, kn[:, :, None]], 2); Vorig = np.concatenate([Vorig, vn[:, :, None]], 2)
        bk_g, bv_g = gc.decode_update(S, dev(kn), dev(vn), dev(Korig), dev(Vorig), want_bits=True)
        oc.append(kn[:, :, None], vn[:, :, None])
        oc.observe(S.cpu().numpy())
        bk_o, bv_o = oc.select_bits()
        oc.requantize(bk_o, bv_o, Korig, Vorig)
        np.testing.assert_array_equal(bk_g.cpu().numpy(), bk_o)
        np.testing.assert_array_equal(bv_g.cpu().numpy(), bv_o)
    compare_canonical(oc, gc, name + ", after two decode steps")


def test_prefill_equals_the_three_call_sequence():
    """Append at the selected widths in one pass gives the cache that appending at the widest
    width, selecting from the same window and requantizing gives."""
    sh = W.shape(3, batch=2, n_q_heads=8, n_kv_heads=4, context=700)
    T, n = sh.context, 4
    K, V = W.make_kv(3, sh)
    q_last = np.ascontiguousarray(W.make_queries(3, sh, n=n, seed_offset=5).transpose(1, 2, 0, 3))
    qn = O.query_norm_statistic(W.make_queries(3, sh, n=64, seed_offset=9), sh.head_dim)
    kw = dict(window=5, sigma_s_max=4e-4, sigma_x_max=6e-3)
    _, g1 = make_pair(sh, qn, **kw)
    _, g3 = make_pair(sh, qn, **kw)
    g1.prefill_window(dev(q_last), dev(K))
    bk1, bv1 = g1.quantize_append_selected(dev(K), dev(V), want_bits=True)
    g3.prefill_window(dev(q_last), dev(K))
    g3.quantize_append(dev(K), dev(V))
    bk3, bv3 = g3.select_bits(None)
    g3.requantize(bk3, bv3)
    np.testing.assert_array_equal(bk1.cpu().numpy(), bk3.cpu().numpy())
    np.testing.assert_array_equal(bv1.cpu().numpy(), bv3.cpu().numpy())
    for side in (0, 1):
        e1, e3 = g1.export_canonical(side), g3.export_canonical(side)
        for key in e1:
            np.testing.assert_array_equal(e1[key].cpu().numpy(), e3[key].cpu().numpy(), err_msg=f"side {side} {key}")


def test_prefill_argument_errors():
    sh = W.shape(3, batch=1, n_q_heads=2, n_kv_heads=2, context=64)
    K, V = W.make_kv(3, sh)
    _, gc = make_pair(sh, 0.01, window=3)
    q = np.zeros((1, 2, 4, sh.head_dim), F16)
    with pytest.raises(qaq.QaqError):
        gc.prefill_window(dev(q), dev(K))                      # more rows than the window
    gc.quantize_append(dev(K[:, :, :8]), dev(V[:, :, :8]))
    with pytest.raises(qaq.QaqError):
        gc.prefill_window(dev(q[:, :, :2]), dev(K))            # cache not empty


def test_append_selected_to_a_partly_filled_tile():
    """qaq_quantize_append_selected on a cache that already holds tokens: the new tokens get
    the widths of the rules for T = tokens after the append and the window as it stands (no
    row covers them: predicted score 0), the cached tokens are not touched."""
    sh = W.shape(3, batch=2, n_q_heads=8, n_kv_heads=4, context=300)
    T, n, extra = sh.context, 3, 7
    K, V = W.make_kv(3, sh, n_tokens=T + extra)
    q_last = np.ascontiguousarray(W.make_queries(3, sh, n=n, seed_offset=6).transpose(1, 2, 0, 3))
    qn = O.query_norm_statistic(W.make_queries(3, sh, n=64, seed_offset=9), sh.head_dim)
    kw = dict(window=5, sigma_s_max=4e-4, sigma_x_max=6e-3)
    oc, gc = make_pair(sh, qn, max_tokens=T + extra, **kw)
    Kp, Vp = np.ascontiguousarray(K[:, :, :T]), np.ascontiguousarray(V[:, :, :T])
    rows = gc.prefill_window(dev(q_last), dev(Kp)).cpu().numpy()
    gc.quantize_append_selected(dev(Kp), dev(Vp))
    oc.prefill(q_last, Kp, Vp, score_rows=[rows[i][..., : T - n + i + 1] for i in range(n)])
    compare_canonical(oc, gc, "prompt")
    Kn, Vn = np.ascontiguousarray(K[:, :, T:]), np.ascontiguousarray(V[:, :, T:])
    bk_g, bv_g = gc.quantize_append_selected(dev(Kn), dev(Vn), want_bits=True)
    # the oracle: append at the widest width, select for everybody, keep the cached tokens' widths
    old_k = np.stack([[oc.K[b][h].bits.copy() for h in range(sh.n_kv_heads)] for b in range(sh.batch)])
    old_v = np.stack([[oc.V[b][h].bits.copy() for h in range(sh.n_kv_heads)] for b in range(sh.batch)])
    oc.append(Kn, Vn)
    bk_o, bv_o = oc.select_bits()
    bk_o[:, :, :T] = old_k; bv_o[:, :, :T] = old_v
    oc.requantize(bk_o, bv_o)
    np.testing.assert_array_equal(bk_g.cpu().numpy(), bk_o[:, :, T:])
    np.testing.assert_array_equal(bv_g.cpu().numpy(), bv_o[:, :, T:])
    assert (bv_o[:, :, T:] == 2).all(), "no window row covers the new tokens: narrowest value width"
    compare_canonical(oc, gc, "after the append")


@pytest.mark.parametrize("store", ["window_fp16", "window_bf16"])
def test_window_kept_in_fp16(store):
    """The variants that keep the window's score rows in fp16 or bfloat16: prompt encoding,
    separate selection and fused decode steps all take the predicted score over the rounded rows."""
    sh = W.shape(3, batch=2, n_q_heads=8, n_kv_heads=4, context=520)
    T, n, steps = sh.context, 4, 6
    K, V = W.make_kv(3, sh)
    q_last = np.ascontiguousarray(W.make_queries(3, sh, n=n, seed_offset=8).transpose(1, 2, 0, 3))
    qn = O.query_norm_statistic(W.make_queries(3, sh, n=64, seed_offset=9), sh.head_dim)
    kw = dict(window=5, sigma_s_max=4e-4, sigma_x_max=6e-3)
    oc, gc = make_pair(sh, qn, max_tokens=T + steps, **dict(kw, **{store: True}))
    oc32, _ = make_pair(sh, qn, max_tokens=T + steps, **kw)
    rows = gc.prefill_window(dev(q_last), dev(K)).cpu().numpy()
    bk_g, bv_g = gc.quantize_append_selected(dev(K), dev(V), want_bits=True)
    given = [rows[i][..., : T - n + i + 1] for i in range(n)]
    bk_o, bv_o, _ = oc.prefill(q_last, K, V, score_rows=given)
    _, bv_32, _ = oc32.prefill(q_last, K, V, score_rows=given)
    np.testing.assert_array_equal(bk_g.cpu().numpy(), bk_o)
    np.testing.assert_array_equal(bv_g.cpu().numpy(), bv_o)
    _log(f"  value widths that differ from the fp32 window: {int((bv_o != bv_32).sum())} of {bv_o.size}")
    compare_canonical(oc, gc, "prompt")
    Korig, Vorig = K.copy(), V.copy()
    qs = W.make_queries(3, sh, n=steps)
    for s in range(steps):
        kn, vn = W.make_new_token(3, sh, step=s)
        X, S = gc.decode_attention(dev(qs[s]), dev(kn), dev(vn), want_scores=True)
        Korig = np.concatenate([Korig, kn[:, :, None]], 2); Vorig = np.concatenate([Vorig, vn[:, :, None]], 2)
        oc.append(kn[:, :, None], vn[:, :, None])
        oc.observe(S.cpu().numpy())
        bk_o, bv_o = oc.select_bits()
        oc.requantize(bk_o, bv_o, Korig, Vorig)
        if s % 2 == 0:       # the fused call
            bk_g, bv_g = gc.decode_update(S, dev(kn), dev(vn), dev(Korig), dev(Vorig), want_bits=True)
        else:                # the separate calls
            gc.quantize_append(dev(kn[:, :, None]), dev(vn[:, :, None]))
            bk_g, bv_g = gc.select_bits(S)
            gc.requantize(bk_g, bv_g, dev(Korig), dev(Vorig))
        np.testing.assert_array_equal(bk_g.cpu().numpy(), bk_o)
        np.testing.assert_array_equal(bv_g.cpu().numpy(), bv_o)
    compare_canonical(oc, gc, "after the decode steps")
