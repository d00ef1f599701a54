"""Sequences of different lengths in one cache (qaq_set_shortfall): every sequence must behave
exactly as if it had a cache of its own -- its own T in the thresholds of Section 4.1, its own
softmax, its own window rows (Section 4.2).  The oracle knows nothing of batches with mixed
lengths: each sequence is checked against a single-sequence oracle cache of its own."""
import dataclasses

import numpy as np
import pytest

from oracle import qaq_oracle as O
from paper_2403_04643_amd import qaq
from paper_2403_04643_amd import workloads as W
from tests.parity_util import F16, F32, attention_errors, dev, make_oracle, make_pair

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _log(msg):
    print("  " + msg, flush=True)


def _rand_bits(rng, shape, p=(0.4, 0.3, 0.2, 0.1)):
    return rng.choice(np.array([2, 3, 4, 8], np.uint8), size=shape, p=p)


def _pair_per_sequence(sh, qn, **kw):
    """(list of single-sequence oracle caches, one GPU cache for the whole batch)."""
    one = dataclasses.replace(sh, batch=1)
    ocs = [make_oracle(one, qn, **kw) for _ in range(sh.batch)]
    _, gc = make_pair(sh, qn, **kw)
    return ocs, gc


def compare_sequence(oc, gc_export, b, what):
    """Bit-exact comparison of sequence b of the GPU cache's exported view with a single-sequence
    oracle cache: widths, [min, max], outlier lists, packed codes of its own tokens."""
    cfg = oc.cfg
    D = cfg.head_dim
    for side, heads in ((0, oc.K), (1, oc.V)):
        ex = gc_export[side]
        for h in range(cfg.n_kv_heads):
            hc = heads[0][h]
            T = hc.T
            tag = f"{what} side={side} b={b} h={h}"
            np.testing.assert_array_equal(ex["bits"][b, h, :T], hc.bits, err_msg=tag + " bits")
            np.testing.assert_array_equal(ex["minmax"][b, h, :T, 0].astype(F32), hc.mn.astype(F32), err_msg=tag + " min")
            np.testing.assert_array_equal(ex["minmax"][b, h, :T, 1].astype(F32), hc.mx.astype(F32), err_msg=tag + " max")
            if cfg.n_o():
                idx, val = hc.outlier_lists()
                np.testing.assert_array_equal(ex["oidx"][b, h, :T], idx, err_msg=tag + " outlier idx")
                np.testing.assert_array_equal(ex["oval"][b, h, :T].view(np.uint16), val.view(np.uint16), err_msg=tag + " outlier val")
            want = np.zeros((T, D), np.uint8)
            for t in range(T):
                p = hc.packed(t)
                want[t, : len(p)] = p
            np.testing.assert_array_equal(ex["codes"][b, h, :T], want, err_msg=tag + " packed codes")


def export_both(gc):
    return [{k: v.cpu().numpy() for k, v in gc.export_canonical(side).items()} for side in (0, 1)]


def compare_all(ocs, gc, what):
    ex = export_both(gc)
    for b, oc in enumerate(ocs):
        compare_sequence(oc, ex, b, what)


@pytest.mark.parametrize("n_q_heads,n_kv_heads,lens", [(8, 4, [766, 300, 511]), (8, 2, [766, 300, 511]),
                                                        (8, 4, [1000, 780, 1021])])
def test_decode_steps_with_sequences_of_different_lengths(n_q_heads, n_kv_heads, lens):
    """Append prompts of different lengths (padded to the longest), then decode steps that take
    sequences across a tile border at different steps; the grouped-query attention kernel serves the
    second shape; in the third every sequence has as many tiles as a head has parts, so the
    attention call is one kernel until the longest sequence grows a fifth tile.  Attention output
    and scores, the selected widths and the cache contents of every sequence against its own
    oracle cache, at every step."""
    import torch
    B, Tmax = len(lens), max(lens)
    steps = 6
    sh = W.shape(3, batch=B, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads, context=Tmax)
    K, V = W.make_kv(3, sh)
    qn = O.query_norm_statistic(W.make_queries(3, sh, n=64, seed_offset=9), sh.head_dim)
    kw = dict(max_tokens=Tmax + steps + 300, window=3, sigma_s_max=4e-4, sigma_x_max=6e-3)
    ocs, gc = _pair_per_sequence(sh, qn, **kw)
    rng = np.random.default_rng(11)
    bk0, bv0 = _rand_bits(rng, (B, n_kv_heads, Tmax)), _rand_bits(rng, (B, n_kv_heads, Tmax))
    gc.set_shortfall([Tmax - n for n in lens])
    gc.quantize_append(dev(K), dev(V), dev(bk0), dev(bv0))
    for b, oc in enumerate(ocs):
        n = lens[b]
        oc.append(K[b:b + 1, :, :n], V[b:b + 1, :, :n], bk0[b:b + 1, :, :n], bv0[b:b + 1, :, :n])
    assert gc.length() == Tmax and gc.lengths() == lens
    compare_all(ocs, gc, "after the first append")
    _log("first append matches")

    Korig = np.zeros((B, n_kv_heads, Tmax + steps, sh.head_dim), F16)
    Vorig = np.zeros_like(Korig)
    for b, n in enumerate(lens):
        Korig[b, :, :n] = K[b, :, :n]; Vorig[b, :, :n] = V[b, :, :n]
    qs = W.make_queries(3, sh, n=steps)
    cur = list(lens)
    for s in range(steps):
        kn, vn = W.make_new_token(3, sh, step=s)
        # padding of the score array is poisoned: nothing may read it
        S = torch.full((B, n_q_heads, gc.length() + 1), float("nan"), dtype=torch.float32, device="cuda")
        X, _ = gc.decode_attention(dev(qs[s]), dev(kn), dev(vn), scores_out=S)
        Xh, Sh = X.cpu().numpy(), S.cpu().numpy()
        for b, oc in enumerate(ocs):
            Xo, So = oc.decode_attention(qs[s][b:b + 1], kn[b:b + 1], vn[b:b + 1])
            ex, es = attention_errors(Xh[b:b + 1], Sh[b:b + 1, :, : cur[b] + 1], Xo, So)
            assert ex.max() < TOL and es.max() < TOL, (s, b, ex.max(), es.max())
            assert np.isnan(Sh[b, :, cur[b] + 1:]).all(), "scores past a sequence's own tokens must be left alone"
        with_orig = s != 4
        ko, vo = (dev(Korig), dev(Vorig)) if with_orig else (None, None)     # the update adds the new tokens itself
        for b in range(B):
            Korig[b, :, cur[b]] = kn[b]; Vorig[b, :, cur[b]] = vn[b]
        bk_g, bv_g = gc.decode_update(S, dev(kn), dev(vn), ko, vo, want_bits=True)
        bk_g, bv_g = bk_g.cpu().numpy(), bv_g.cpu().numpy()
        for b, oc in enumerate(ocs):
            oc.append(kn[b:b + 1, :, None], vn[b:b + 1, :, None])
            oc.observe(Sh[b:b + 1, :, : cur[b] + 1])
            bk_o, bv_o = oc.select_bits()
            oc.requantize(bk_o, bv_o, Korig[b:b + 1, :, : cur[b] + 1] if with_orig else None,
                          Vorig[b:b + 1, :, : cur[b] + 1] if with_orig else None)
            cur[b] += 1
            np.testing.assert_array_equal(bk_g[b, :, : cur[b]], bk_o[0], err_msg=f"step {s} b={b} key widths")
            np.testing.assert_array_equal(bv_g[b, :, : cur[b]], bv_o[0], err_msg=f"step {s} b={b} value widths")
        if with_orig:      # the unquantized copies got every sequence's new token at its own position
            np.testing.assert_array_equal(ko.cpu().numpy(), Korig)
            np.testing.assert_array_equal(vo.cpu().numpy(), Vorig)
        assert gc.lengths() == cur
        compare_all(ocs, gc, f"step {s}")
        _log(f"step {s}: lengths {cur} match")
    st = gc.stats()
    assert st.refused_upgrades == sum(oc.refused for oc in ocs)
    assert sum(st.hist_k) == sum(cur) * n_kv_heads == sum(st.hist_v)
    assert st.fp16_bytes == sum(cur) * n_kv_heads * sh.head_dim * 4

    # the three-call sequence on the same cache: widths from the window as it stands
    bk3, bv3 = gc.select_bits()
    bk3, bv3 = bk3.cpu().numpy(), bv3.cpu().numpy()
    for b, oc in enumerate(ocs):
        bk_o, bv_o = oc.select_bits()
        np.testing.assert_array_equal(bk3[b, :, : cur[b]], bk_o[0])
        np.testing.assert_array_equal(bv3[b, :, : cur[b]], bv_o[0])

    # a later append adds the same number of tokens to every sequence
    n2 = 300
    K2, V2 = W.make_kv(3, sh, n_tokens=n2, seed_offset=3)
    bk2, bv2 = _rand_bits(rng, (B, n_kv_heads, n2)), _rand_bits(rng, (B, n_kv_heads, n2))
    gc.quantize_append(dev(K2), dev(V2), dev(bk2), dev(bv2))
    for b, oc in enumerate(ocs):
        oc.append(K2[b:b + 1], V2[b:b + 1], bk2[b:b + 1], bv2[b:b + 1])
        cur[b] += n2
    assert gc.lengths() == cur
    compare_all(ocs, gc, "after the second append")
    Kd, Vd = gc.dequantize()
    Kd, Vd = Kd.cpu().numpy(), Vd.cpu().numpy()
    for b, oc in enumerate(ocs):
        Ko, Vo = oc.dequantize()
        np.testing.assert_array_equal(Kd[b, :, : cur[b]].view(np.uint16), Ko[0].astype(F16).view(np.uint16))
        np.testing.assert_array_equal(Vd[b, :, : cur[b]].view(np.uint16), Vo[0].astype(F16).view(np.uint16))
    X, S = gc.decode_attention(dev(qs[0]), want_scores=True)
    Xh, Sh = X.cpu().numpy(), S.cpu().numpy()
    for b, oc in enumerate(ocs):
        Xo, So = oc.decode_attention(qs[0][b:b + 1])
        ex, es = attention_errors(Xh[b:b + 1], Sh[b:b + 1, :, : cur[b]], Xo, So)
        assert ex.max() < TOL and es.max() < TOL
    gc.close()


def test_prompt_encoding_with_sequences_of_different_lengths():
    """Section 2.1 prompt encoding + Section 4.2 window: the last n score rows of every prompt are
    those of its own last n positions, softmaxed over its own tokens, and the widths come from
    its own T."""
    lens = [600, 257, 443]
    B, Tmax, n = len(lens), max(lens), 3
    sh = W.shape(3, batch=B, n_q_heads=8, n_kv_heads=4, context=Tmax)
    K, V = W.make_kv(3, sh)
    qn = O.query_norm_statistic(W.make_queries(3, sh, n=64, seed_offset=9), sh.head_dim)
    kw = dict(max_tokens=Tmax + 8, window=n, sigma_s_max=4e-4, sigma_x_max=6e-3)
    ocs, gc = _pair_per_sequence(sh, qn, **kw)
    q_last = np.ascontiguousarray(np.moveaxis(W.make_queries(3, sh, n=n, seed_offset=2), 0, 2))   # [B, Hq, n, D]
    gc.set_shortfall([Tmax - x for x in lens])
    rows = gc.prefill_window(dev(q_last), dev(K)).cpu().numpy()            # [n, B, Hq, Tmax]
    bk_g, bv_g = gc.quantize_append_selected(dev(K), dev(V), want_bits=True)
    bk_g, bv_g = bk_g.cpu().numpy(), bv_g.cpu().numpy()
    for b, oc in enumerate(ocs):
        T = lens[b]
        # the oracle's own rows (fp64 softmax) against the library's, then the width decisions
        # from the library's fp32 rows, so that both sides decide on the same numbers
        _, _, rows_o = oc.prefill(q_last[b:b + 1], K[b:b + 1, :, :T], V[b:b + 1, :, :T])
        for i in range(n):
            L = T - n + i + 1
            err = np.abs(rows[i, b, :, :L].astype(np.float64) - rows_o[i][0]).max() / rows_o[i][0].max()
            assert err < TOL, (b, i, err)
            assert (rows[i, b, :, L:] == 0).all()
        one = dataclasses.replace(sh, batch=1)
        oc2 = make_oracle(one, qn, **kw)
        bk_o, bv_o, _ = oc2.prefill(q_last[b:b + 1], K[b:b + 1, :, :T], V[b:b + 1, :, :T],
                                    score_rows=[rows[i, b:b + 1, :, : T - n + i + 1] for i in range(n)])
        np.testing.assert_array_equal(bk_g[b, :, :T], bk_o[0], err_msg=f"b={b} key widths")
        np.testing.assert_array_equal(bv_g[b, :, :T], bv_o[0], err_msg=f"b={b} value widths")
        ocs[b] = oc2
    compare_all(ocs, gc, "after prompt encoding")
    gc.close()


def test_shortfall_argument_errors():
    sh = W.shape(3, batch=2, n_q_heads=4, n_kv_heads=4, context=64)
    K, V = W.make_kv(3, sh)
    _, gc = make_pair(sh, 1.0, max_tokens=128)
    with pytest.raises(qaq.QaqError):
        gc.set_shortfall([3, 5])                      # no sequence is the longest
    with pytest.raises(qaq.QaqError):
        gc.set_shortfall([0, -1])
    gc.set_shortfall([0, 64])
    with pytest.raises(qaq.QaqError):                 # sequence 1 would stay empty
        gc.quantize_append(dev(K), dev(V))
    assert gc.length() == 0
    gc.set_shortfall([0, 63])
    gc.quantize_append(dev(K), dev(V))
    assert gc.lengths() == [64, 1]
    with pytest.raises(qaq.QaqError):                 # only an empty cache takes new length differences
        gc.set_shortfall([0, 0])
    gc.reset()
    assert gc.lengths() == [0, 0]
    gc.quantize_append(dev(K), dev(V))
    assert gc.lengths() == [64, 64]                   # a reset cache has one length again
    gc.close()
