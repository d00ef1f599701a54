"""The 1-bit width (a variant: the paper's experiments use {2,3,4,8}; a wider set that
reaches down to one bit is what its highest compression ratios need): every step of the path
with 1 in the width set, against the oracle -- codes, ranges and outliers bit for bit,
attention within 2e-3."""
import numpy as np
import pytest

from oracle import qaq_oracle as O
from paper_2403_04643_amd import workloads as W
from tests.parity_util import F16, F32, attention_errors, compare_canonical, dev, make_pair

pytestmark = pytest.mark.gpu
TOL = 2e-3
SET5 = (1, 2, 3, 4, 8)


def _rand_bits(rng, shape, p=(0.3, 0.25, 0.2, 0.15, 0.1)):
    return rng.choice(np.array(SET5, np.uint8), size=shape, p=p)


def _check_attention(oc, gc, q, kn=None, vn=None, tag=""):
    X, S = gc.decode_attention(dev(q), None if kn is None else dev(kn), None if vn is None else dev(vn), want_scores=True)
    Xo, So = oc.decode_attention(q, kn, vn)
    ex, es = attention_errors(X.cpu().numpy(), S.cpu().numpy(), Xo, So)
    assert ex.max() < TOL and es.max() < TOL, (tag, ex.max(), es.max())
    return S


@pytest.mark.parametrize("head_dim,context,n_o", [(128, 700, 1), (64, 300, 2), (128, 256, 0), (64, 37, 1)])
def test_append_requantize_export_dequantize(head_dim, context, n_o):
    sh = W.shape(2, batch=2, n_q_heads=3, n_kv_heads=3, head_dim=head_dim, context=context)
    print(f"one bit: {sh} n_o={n_o}", flush=True)
    K, V = W.make_kv(2, sh)
    rng = np.random.default_rng(11)
    oc, gc = make_pair(sh, 0.01, bit_set=SET5, n_outlier_per_side=n_o)
    # first quantization at mixed widths, in two calls (the second lands in a partly filled tile)
    bk, bv = _rand_bits(rng, K.shape[:3]), _rand_bits(rng, K.shape[:3], p=(0.5, 0.2, 0.1, 0.1, 0.1))
    cut = context // 3
    for lo, hi in ((0, cut), (cut, context)):
        oc.append(K[:, :, lo:hi], V[:, :, lo:hi], bk[:, :, lo:hi], bv[:, :, lo:hi])
        gc.quantize_append(dev(K[:, :, lo:hi]), dev(V[:, :, lo:hi]), dev(bk[:, :, lo:hi]), dev(bv[:, :, lo:hi]))
    compare_canonical(oc, gc, "append")
    st = gc.stats()
    assert st.hist_k[4] == int((bk == 1).sum()) and st.hist_v[4] == int((bv == 1).sum())
    assert st.code_bytes == int(bk.astype(np.int64).sum() + bv.astype(np.int64).sum()) * head_dim // 8
    Kd, Vd = gc.dequantize()
    Ko, Vo = oc.dequantize()
    np.testing.assert_array_equal(Kd.cpu().numpy().view(np.uint16), Ko.astype(F16).view(np.uint16))
    np.testing.assert_array_equal(Vd.cpu().numpy().view(np.uint16), Vo.astype(F16).view(np.uint16))
    q = W.make_queries(2, sh)[0]
    _check_attention(oc, gc, q, tag="append")
    # mixed moves without the unquantized copy, then with it
    b2k, b2v = _rand_bits(rng, K.shape[:3]), _rand_bits(rng, K.shape[:3])
    oc.requantize(b2k, b2v); gc.requantize(dev(b2k), dev(b2v))
    compare_canonical(oc, gc, "mixed, no originals")
    assert gc.stats().refused_upgrades == oc.refused > 0
    _check_attention(oc, gc, q, tag="narrowed")
    b3k, b3v = _rand_bits(rng, K.shape[:3]), _rand_bits(rng, K.shape[:3])
    oc.requantize(b3k, b3v, K, V); gc.requantize(dev(b3k), dev(b3v), dev(K), dev(V))
    compare_canonical(oc, gc, "mixed, with originals")
    np.testing.assert_array_equal(gc.export_canonical(0)["bits"].cpu().numpy(), b3k)
    _check_attention(oc, gc, q, tag="with originals")
    # everything to one bit
    ones = np.ones(K.shape[:3], np.uint8)
    oc.requantize(ones, ones); gc.requantize(dev(ones), dev(ones))
    compare_canonical(oc, gc, "all one bit")
    _check_attention(oc, gc, q, tag="all one bit")


@pytest.mark.parametrize("G,window_kw", [(1, dict()), (4, dict(window_fp16=True)), (2, dict(window_bf16=True))])
def test_decode_steps_with_one_bit_in_the_set(G, window_kw):
    sh = W.shape(3, batch=2, n_q_heads=2 * G, n_kv_heads=2, head_dim=128, context=500)
    steps = 14          # crosses into the third tile
    K, V = W.make_kv(3, sh)
    qn = O.query_norm_statistic(W.make_queries(3, sh, n=64, seed_offset=9), sh.head_dim)
    oc, gc = make_pair(sh, qn, max_tokens=sh.context + steps, window=3, bit_set=SET5,
                       sigma_s_max=6e-4, sigma_x_max=0.12, **window_kw)
    oc.append(K, V); gc.quantize_append(dev(K), dev(V))
    Korig, Vorig = K.copy(), V.copy()
    qs = W.make_queries(3, sh, n=steps)
    seen = set()
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
        seen |= set(np.unique(bk_o)) | set(np.unique(bv_o))
        assert gc.stats().refused_upgrades == oc.refused
    assert 1 in seen and len(seen) >= 3, seen       # the hyper-parameters spread the widths, one bit included
    compare_canonical(oc, gc, "after decode steps")


@pytest.mark.parametrize("G,context", [(1, 9000), (2, 3000)])
def test_long_context_in_the_two_kernel_form(G, context):
    """Few heads and a long context: one workgroup per part and the merge kernel, with the
    fifth class present (and grouped queries in the second case)."""
    sh = W.shape(4, batch=1, n_q_heads=G, n_kv_heads=1, context=context)
    K, V = W.make_kv(4, sh)
    rng = np.random.default_rng(29)
    bk, bv = _rand_bits(rng, K.shape[:3]), _rand_bits(rng, K.shape[:3], p=(0.6, 0.2, 0.1, 0.05, 0.05))
    oc, gc = make_pair(sh, 0.01, bit_set=SET5)
    oc.append(K, V, bk, bv); gc.quantize_append(dev(K), dev(V), dev(bk), dev(bv))
    q = W.make_queries(4, sh)[0]
    kn, vn = W.make_new_token(4, sh)
    S = _check_attention(oc, gc, q, kn, vn, tag="two-kernel form")
    np.testing.assert_allclose(S.cpu().numpy().sum(-1, dtype=np.float64), 1.0, rtol=2e-5)
    compare_canonical(oc, gc, "long context")
