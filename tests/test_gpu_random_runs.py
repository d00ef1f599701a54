"""Seeded random runs of the whole path against the oracle: random shapes, hyper-parameters,
width sets, outlier counts, window lengths and precisions, prompts installed either by prompt
encoding or by a plain append, decode steps through the fused call or the separate calls,
with and without the unquantized copies, and a hyper-parameter that moves during the run.
Widths every step, the cache (widths, ranges, outliers, codes) and the counters at the end,
bit for bit; attention within 2e-3."""
import numpy as np
import pytest

from oracle import qaq_oracle as O
from paper_2403_04643_amd import workloads as W
from tests.parity_util import attention_errors, compare_canonical, dev, make_pair

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.mark.parametrize("seed", list(range(60)))
def test_random_run(seed):
    rng = np.random.default_rng(9000 + seed)
    G = int(rng.choice([1, 2, 4]))
    Hkv = int(rng.choice([1, 2, 3, 4]))
    D = int(rng.choice([64, 128]))
    T0 = int(rng.choice([1, 5, 63, 250, 255, 256, 257, 300, 511, 700, 767, 1023, 1300]))
    steps = int(rng.integers(3, 8))
    window = int(rng.integers(1, 9))
    n_o = int(rng.choice([0, 1, 1, 2, 4]))
    sets = [(2, 3, 4, 8), (2, 3, 4, 8), (2, 4, 8), (3, 8), (2, 3), (4,), (2, 8), (1, 2, 3, 4, 8), (1, 2, 3, 4, 8), (1, 3), (1, 4, 8), (1,)]
    bit_set = sets[int(rng.integers(len(sets)))]
    sh = W.shape(3, batch=int(rng.choice([1, 2, 3])), n_q_heads=Hkv * G, n_kv_heads=Hkv, head_dim=D, context=T0)
    kw = dict(max_tokens=T0 + steps, window=window, n_outlier_per_side=n_o, bit_set=bit_set,
              sigma_s_max=float(10 ** rng.uniform(-4.3, -3.2)), sigma_x_max=float(10 ** rng.uniform(-2.6, -1.2)),
              **[dict(), dict(window_fp16=True), dict(window_bf16=True)][int(rng.integers(3))])
    K, V = W.make_kv(3, sh, seed_offset=seed)
    if n_o > 0 and rng.integers(3) == 0:       # outliers by thresholds, calibrated per KV head on the prompt
        alpha = float(rng.choice([0.005, 0.02, 0.1]))
        kw["outlier_thresholds"] = np.array([[O.calibrate_outlier_thresholds(X[:, h], alpha) for h in range(Hkv)]
                                             for X in (K, V)], np.float32)
    print(f"seed {seed}: {sh} steps={steps} {kw}", flush=True)
    qn = O.query_norm_statistic(W.make_queries(3, sh, n=64, seed_offset=9), sh.head_dim)
    oc, gc = make_pair(sh, qn, **kw)
    n_rows = min(window, T0, int(rng.integers(1, 9)))
    if rng.integers(2):
        q_last = np.ascontiguousarray(W.make_queries(3, sh, n=n_rows, seed_offset=40 + seed).transpose(1, 2, 0, 3))
        rows = gc.prefill_window(dev(q_last), dev(K)).cpu().numpy()
        bk_g, bv_g = gc.quantize_append_selected(dev(K), dev(V), want_bits=True)
        bk_o, bv_o, _ = oc.prefill(q_last, K, V, score_rows=[rows[i][..., : T0 - n_rows + i + 1] for i in range(n_rows)])
        np.testing.assert_array_equal(bk_g.cpu().numpy(), bk_o)
        np.testing.assert_array_equal(bv_g.cpu().numpy(), bv_o)
    else:
        oc.append(K, V); gc.quantize_append(dev(K), dev(V))
    Korig, Vorig = K.copy(), V.copy()
    qs = W.make_queries(3, sh, n=steps, seed_offset=seed)
    served = 0
    for s in range(steps):
        if s == steps // 2:
            new_s = float(oc.cfg.sigma_s_max * 10 ** rng.uniform(-0.7, 0.7))
            new_x = float(oc.cfg.sigma_x_max * 10 ** rng.uniform(-0.7, 0.7))
            oc.cfg.sigma_s_max, oc.cfg.sigma_x_max = new_s, new_x
            gc.set_sigmas(new_s, new_x)
        kn, vn = W.make_new_token(3, sh, step=100 * seed + s)
        X, S = gc.decode_attention(dev(qs[s]), dev(kn), dev(vn), want_scores=True)
        Xo, So = oc.decode_attention(qs[s], kn, vn)
        ex, es = attention_errors(X.cpu().numpy(), S.cpu().numpy(), Xo, So)
        assert ex.max() < TOL and es.max() < TOL, f"step {s}"
        Korig = np.concatenate([Korig, kn[:, :, None]], 2); Vorig = np.concatenate([Vorig, vn[:, :, None]], 2)
        with_orig = bool(rng.integers(4))
        ko, vo = (dev(Korig), dev(Vorig)) if with_orig else (None, None)
        oc.append(kn[:, :, None], vn[:, :, None])
        oc.observe(S.cpu().numpy())
        bk_o, bv_o = oc.select_bits()
        before = oc.refused
        oc.requantize(bk_o, bv_o, Korig if with_orig else None, Vorig if with_orig else None)
        mode = int(rng.integers(3))
        if mode == 0:
            bk_g, bv_g = gc.decode_update(S, dev(kn), dev(vn), ko, vo, want_bits=True)
        elif mode == 1:
            gc.decode_update(S, dev(kn), dev(vn), ko, vo, want_bits=False)
            bk_g = bv_g = None
        else:
            gc.quantize_append(dev(kn[:, :, None]), dev(vn[:, :, None]))
            bk_g, bv_g = gc.select_bits(S)
            gc.requantize(bk_g, bv_g, ko, vo)
        if bk_g is not None:
            np.testing.assert_array_equal(bk_g.cpu().numpy(), bk_o, err_msg=f"step {s}")
            np.testing.assert_array_equal(bv_g.cpu().numpy(), bv_o, err_msg=f"step {s}")
        assert gc.stats().refused_upgrades == oc.refused, f"step {s} (refused before {before})"
    compare_canonical(oc, gc, f"seed {seed}")
    Kd, Vd = gc.dequantize()
    Ko, Vo = oc.dequantize()
    np.testing.assert_array_equal(Kd.cpu().numpy().view(np.uint16), Ko.astype(np.float16).view(np.uint16))
    np.testing.assert_array_equal(Vd.cpu().numpy().view(np.uint16), Vo.astype(np.float16).view(np.uint16))


@pytest.mark.parametrize("bit_set,with_orig", [((2, 3, 4, 8), True), ((1, 2, 3, 4, 8), True), ((1, 2, 3, 4, 8), False)])
def test_long_decode_run(bit_set, with_orig):
    """400 decode steps from a 200-token prompt (the cache grows through two tile boundaries, class
    counts cross many multiples of 16, so regions move again and again; with the unquantized
    copies widths go up and down, without them only down): widths at every step, the whole
    cache every 20 steps."""
    sh = W.shape(3, batch=1, n_q_heads=4, n_kv_heads=2, head_dim=128, context=200)
    steps = 400
    K, V = W.make_kv(3, sh, seed_offset=5)
    qn = O.query_norm_statistic(W.make_queries(3, sh, n=64, seed_offset=9), sh.head_dim)
    oc, gc = make_pair(sh, qn, max_tokens=sh.context + steps, window=3, bit_set=bit_set,
                       sigma_s_max=2.5e-4, sigma_x_max=0.05)
    oc.append(K, V); gc.quantize_append(dev(K), dev(V))
    Korig, Vorig = K.copy(), V.copy()
    qs = W.make_queries(3, sh, n=steps, seed_offset=2)
    seen = set()
    for s in range(steps):
        kn, vn = W.make_new_token(3, sh, step=s)
        X, S = gc.decode_attention(dev(qs[s]), dev(kn), dev(vn), want_scores=True)
        if s % 20 == 0:
            Xo, So = oc.decode_attention(qs[s], kn, vn)
            ex, es = attention_errors(X.cpu().numpy(), S.cpu().numpy(), Xo, So)
            assert ex.max() < TOL and es.max() < TOL, f"step {s}"
        Korig = np.concatenate([Korig, kn[:, :, None]], 2); Vorig = np.concatenate([Vorig, vn[:, :, None]], 2)
        oc.append(kn[:, :, None], vn[:, :, None])
        oc.observe(S.cpu().numpy())
        bk_o, bv_o = oc.select_bits()
        oc.requantize(bk_o, bv_o, Korig if with_orig else None, Vorig if with_orig else None)
        bk_g, bv_g = gc.decode_update(S, dev(kn), dev(vn), dev(Korig) if with_orig else None,
                                      dev(Vorig) if with_orig else None, want_bits=True)
        np.testing.assert_array_equal(bk_g.cpu().numpy(), bk_o, err_msg=f"step {s}")
        np.testing.assert_array_equal(bv_g.cpu().numpy(), bv_o, err_msg=f"step {s}")
        seen |= set(np.unique(bk_o)) | set(np.unique(bv_o))
        if s % 20 == 19:
            compare_canonical(oc, gc, f"step {s}")
            assert gc.stats().refused_upgrades == oc.refused
    assert len(seen) >= 3, seen
