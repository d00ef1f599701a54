"""GPU parity at the full sizes of the stated configurations (2^20 token-heads per layer),
in the launch configuration the benchmark times: the whole batch goes through libqaq in
one call per operation, and the CPU oracle recomputes a seeded sample of (sequence, KV head)
units one by one -- every unit is independent of the others, so a unit's oracle result is the
full-size result for that unit.  Widths, codes, [min,max] and outlier lists of the sampled
units are compared bit for bit, attention within 2e-3; properties that hold at any size
(scores sum to one, outputs inside the value range) are checked on every head."""
import numpy as np
import pytest

from oracle import qaq_oracle as O
from paper_2403_04643_amd import qaq, workloads as W
from tests.parity_util import F16, F32, attention_errors, dev

pytestmark = pytest.mark.gpu
TOL = 2e-3


def _log(msg):
    print(msg, flush=True)


def _unit_oracle(sh, qn, b, h, **kw):
    """Oracle cache holding the single unit (sequence b, KV head h) with its G query heads."""
    G = sh.n_q_heads // sh.n_kv_heads
    cfg = O.Config(1, G, 1, sh.head_dim, qnorm2=np.asarray([qn[h]], F32), **kw)
    return O.OracleCache(cfg), G


def _compare_unit(ex, side_heads, b, h, D, n_o, tag):
    hc = side_heads
    np.testing.assert_array_equal(ex["bits"][b, h], hc.bits, err_msg=tag + " bits")
    np.testing.assert_array_equal(ex["minmax"][b, h, :, 0].astype(F32), hc.mn.astype(F32), err_msg=tag + " min")
    np.testing.assert_array_equal(ex["minmax"][b, h, :, 1].astype(F32), hc.mx.astype(F32), err_msg=tag + " max")
    if n_o:
        idx, val = hc.outlier_lists()
        np.testing.assert_array_equal(ex["oidx"][b, h], idx, err_msg=tag + " outlier idx")
        np.testing.assert_array_equal(ex["oval"][b, h].view(np.uint16), val.view(np.uint16), err_msg=tag + " outlier val")
    want = np.zeros((hc.T, D), np.uint8)
    for t in range(hc.T):
        p = hc.packed(t)
        want[t, : len(p)] = p
    np.testing.assert_array_equal(ex["codes"][b, h], want, err_msg=tag + " packed codes")


def _global_properties(X, S, V, Vnew):
    S = S.cpu().numpy()
    np.testing.assert_allclose(S.sum(-1, dtype=np.float64), 1.0, rtol=2e-5)
    assert np.isfinite(S).all() and (S >= 0).all()
    X = X.cpu().numpy()
    assert np.isfinite(X).all()
    # a convex combination of reconstructed values: inside the per-channel value range,
    # widened by half a 2-bit quantization step of the widest token range
    G = X.shape[1] // V.shape[1]
    lo = np.minimum(V.min(2), Vnew).astype(F32).repeat(G, 1)
    hi = np.maximum(V.max(2), Vnew).astype(F32).repeat(G, 1)
    slack = (hi.max(-1, keepdims=True) - lo.min(-1, keepdims=True)) / 8 + 1e-3
    assert (X >= lo - slack).all() and (X <= hi + slack).all()


def _sample_units(sh, n, seed):
    rng = np.random.default_rng(seed)
    picks = {(0, 0), (sh.batch - 1, sh.n_kv_heads - 1)}
    while len(picks) < n:
        picks.add((int(rng.integers(sh.batch)), int(rng.integers(sh.n_kv_heads))))
    return sorted(picks)


@pytest.mark.parametrize("cfgno,p_k,p_v", [
    (2, (0.49, 0.50, 0.007, 0.003), (0.89, 0.10, 0.007, 0.003)),   # the benchmark's operating point, plus a few wide tokens
    (5, (0.3, 0.3, 0.3, 0.1), (0.5, 0.3, 0.15, 0.05)),              # 8 query heads per KV head
    (2, (0.45, 0.03, 0.01, 0.01, 0.5), (0.18, 0.01, 0.005, 0.005, 0.8)),   # width set with 1: the bench's point of that kind
])
def test_full_size_given_widths(cfgno, p_k, p_v):
    sh = W.shape(cfgno)
    _log(f"full size cfg={cfgno} shape={sh} width classes={len(p_k)}")
    K, V = W.make_kv(cfgno, sh)
    rng = np.random.default_rng(97 + cfgno)
    widths = np.array([2, 3, 4, 8, 1][:len(p_k)], np.uint8)
    bk = rng.choice(widths, size=K.shape[:3], p=p_k)
    bv = rng.choice(widths, size=K.shape[:3], p=p_v)
    qn = np.full(sh.n_kv_heads, 0.01, F32)
    bit_set = tuple(sorted(int(w) for w in widths))
    gc = qaq.Cache(qaq.make_config(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.context + 1, qn.tolist(), bit_set=bit_set))
    gc.quantize_append(dev(K), dev(V), dev(bk), dev(bv))
    q = W.make_queries(cfgno, sh)[0]
    kn, vn = W.make_new_token(cfgno, sh)
    X, S = gc.decode_attention(dev(q), dev(kn), dev(vn), want_scores=True)
    _global_properties(X, S, V, vn)
    Xg, Sg = X.cpu().numpy(), S.cpu().numpy()
    exK = {k: v.cpu().numpy() for k, v in gc.export_canonical(0).items()}
    exV = {k: v.cpu().numpy() for k, v in gc.export_canonical(1).items()}
    worst = 0.0
    for b, h in _sample_units(sh, 5, 11 + cfgno):
        oc, G = _unit_oracle(sh, qn, b, h, bit_set=bit_set)
        oc.append(K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1], bk[b:b + 1, h:h + 1], bv[b:b + 1, h:h + 1])
        _compare_unit(exK, oc.K[0][0], b, h, sh.head_dim, oc.cfg.n_o(), f"K b={b} h={h}")
        _compare_unit(exV, oc.V[0][0], b, h, sh.head_dim, oc.cfg.n_o(), f"V b={b} h={h}")
        Xo, So = oc.decode_attention(q[b:b + 1, h * G:(h + 1) * G], kn[b:b + 1, h:h + 1], vn[b:b + 1, h:h + 1])
        ex, es = attention_errors(Xg[b:b + 1, h * G:(h + 1) * G], Sg[b:b + 1, h * G:(h + 1) * G], Xo, So)
        _log(f"  unit b={b} h={h}: max rel err X {ex.max():.2e}, S {es.max():.2e}")
        worst = max(worst, ex.max(), es.max())
        assert ex.max() < TOL and es.max() < TOL
    _log(f"  worst sampled error {worst:.2e}")


def test_long_context_selected_widths():
    """Config 4: context 32768, widths chosen by the value rule from a Zipf(1.1) importance
    profile and by the key rule, narrowed in place from the 8-bit prefill, then attention."""
    sh = W.shape(4)
    _log(f"full size cfg=4 shape={sh}")
    K, V = W.make_kv(4, sh)
    T = sh.context
    rows = W.zipf_score_rows(sh, T)
    qcal = W.make_queries(4, sh, n=32, seed_offset=9)
    qn = np.full(sh.n_kv_heads, O.query_norm_statistic(qcal, sh.head_dim), F32)
    # hyper-parameters that spread the widths: centre the thresholds on the ranges of one unit
    probe, _ = _unit_oracle(sh, qn, 0, 0)
    probe.append(K[:1, :1], V[:1, :1])
    rk, rv = probe.K[0][0].ranges().astype(np.float64), probe.V[0][0].ranges().astype(np.float64)
    sigma_x = float(np.median(rv * rows[0, 0]) * np.sqrt(T) / (2 * np.sqrt(3)) / 2 ** 2.5)
    var_k = (np.median(rk) / 2 ** 3.0 / (2 * np.sqrt(3))) ** 2
    sigma_s = float(np.sqrt(np.expm1(var_k * float(qn[0])) * (T - 1) / T ** 3))
    kw = dict(sigma_s_max=sigma_s, sigma_x_max=sigma_x, window=5)
    gc = qaq.Cache(qaq.make_config(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, T + 1, qn.tolist(), **kw))
    gc.quantize_append(dev(K), dev(V))
    bk, bv = gc.select_bits(dev(rows))
    gc.requantize(bk, bv)
    bk, bv = bk.cpu().numpy(), bv.cpu().numpy()
    hist_v = [int((bv == w).sum()) for w in (2, 3, 4, 8)]
    hist_k = [int((bk == w).sum()) for w in (2, 3, 4, 8)]
    _log(f"  width histograms K {hist_k} V {hist_v}")
    assert min(hist_v) > 0, "value widths must spread over all of {2,3,4,8}"
    q = W.make_queries(4, sh)[0]
    kn, vn = W.make_new_token(4, sh)
    X, S = gc.decode_attention(dev(q), dev(kn), dev(vn), want_scores=True)
    _global_properties(X, S, V, vn)
    Xg, Sg = X.cpu().numpy(), S.cpu().numpy()
    exK = {k: v.cpu().numpy() for k, v in gc.export_canonical(0).items()}
    exV = {k: v.cpu().numpy() for k, v in gc.export_canonical(1).items()}
    for b, h in _sample_units(sh, 3, 15):
        oc, G = _unit_oracle(sh, qn, b, h, **kw)
        oc.append(K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1])
        oc.observe(rows[b:b + 1, h * G:(h + 1) * G])
        bko, bvo = oc.select_bits()
        np.testing.assert_array_equal(bk[b, h], bko[0, 0])
        np.testing.assert_array_equal(bv[b, h], bvo[0, 0])
        oc.requantize(bko, bvo)
        _compare_unit(exK, oc.K[0][0], b, h, sh.head_dim, oc.cfg.n_o(), f"K b={b} h={h}")
        _compare_unit(exV, oc.V[0][0], b, h, sh.head_dim, oc.cfg.n_o(), f"V b={b} h={h}")
        Xo, So = oc.decode_attention(q[b:b + 1, h * G:(h + 1) * G], kn[b:b + 1, h:h + 1], vn[b:b + 1, h:h + 1])
        ex, es = attention_errors(Xg[b:b + 1, h * G:(h + 1) * G], Sg[b:b + 1, h * G:(h + 1) * G], Xo, So)
        _log(f"  unit b={b} h={h}: max rel err X {ex.max():.2e}, S {es.max():.2e}")
        assert ex.max() < TOL and es.max() < TOL


def test_full_size_prompt_encoding():
    """Config 2 at full size: the window from the last five causal score rows of the prompt
    and the first quantization at the selected widths, in the two library calls the
    benchmark times; sampled units against the oracle."""
    sh = W.shape(2)
    _log(f"full size prompt encoding cfg=2 shape={sh}")
    T, n = sh.context, 5
    G = sh.n_q_heads // sh.n_kv_heads
    K, V = W.make_kv(2, sh)
    q_last = np.ascontiguousarray(W.make_queries(2, sh, n=n, seed_offset=3).transpose(1, 2, 0, 3))
    qcal = W.make_queries(2, sh, n=4, seed_offset=7).astype(np.float64)
    qn = np.full(sh.n_kv_heads, float(np.quantile((qcal ** 2).sum(-1).reshape(-1), 0.9)) / sh.head_dim, F32)
    kw = dict(sigma_s_max=1.8e-5, sigma_x_max=1.85e-2, window=5)     # near the benchmark's operating point A
    gc = qaq.Cache(qaq.make_config(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, T + 1, qn.tolist(), **kw))
    rows = gc.prefill_window(dev(q_last), dev(K)).cpu().numpy()
    np.testing.assert_allclose(rows.sum(-1, dtype=np.float64), 1.0, rtol=2e-5)
    for i in range(n):
        assert (rows[i][..., T - n + i + 1:] == 0).all()
    bk, bv = gc.quantize_append_selected(dev(K), dev(V), want_bits=True)
    bk, bv = bk.cpu().numpy(), bv.cpu().numpy()
    hist_k = [int((bk == w).sum()) for w in (2, 3, 4, 8)]
    hist_v = [int((bv == w).sum()) for w in (2, 3, 4, 8)]
    _log(f"  width histograms K {hist_k} V {hist_v}")
    assert sum(c > 0 for c in hist_k) > 1 and sum(c > 0 for c in hist_v) > 1
    exK = {k: v.cpu().numpy() for k, v in gc.export_canonical(0).items()}
    exV = {k: v.cpu().numpy() for k, v in gc.export_canonical(1).items()}
    for b, h in _sample_units(sh, 4, 23):
        worst = 0.0
        for g in range(G):
            hq = h * G + g
            ref = O.prefill_score_rows(q_last[b, hq], K[b, h])
            for i in range(n):
                got = rows[i, b, hq, : T - n + i + 1]
                worst = max(worst, np.abs(got.astype(np.float64) - ref[i]).max() / ref[i].max())
        _log(f"  unit b={b} h={h}: worst score error {worst:.2e}")
        assert worst < TOL
        oc, _ = _unit_oracle(sh, qn, b, h, **kw)
        unit_rows = [rows[i][b:b + 1, h * G:(h + 1) * G, : T - n + i + 1] for i in range(n)]
        bko, bvo, _ = oc.prefill(q_last[b:b + 1, h * G:(h + 1) * G], K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1], score_rows=unit_rows)
        np.testing.assert_array_equal(bk[b, h], bko[0, 0])
        np.testing.assert_array_equal(bv[b, h], bvo[0, 0])
        _compare_unit(exK, oc.K[0][0], b, h, sh.head_dim, oc.cfg.n_o(), f"K b={b} h={h}")
        _compare_unit(exV, oc.V[0][0], b, h, sh.head_dim, oc.cfg.n_o(), f"V b={b} h={h}")


@pytest.mark.parametrize("batch,parts", [(16, 2), (10, 3)])
def test_attention_with_two_and_three_parts_per_head(batch, parts):
    """Head counts at which a head's tiles are split into two resp. three parts that share a
    workgroup (512 resp. 320 query heads, five tiles each): sampled units against the oracle."""
    sh = W.shape(3, batch=batch, n_q_heads=32, n_kv_heads=32, head_dim=64, context=1100)
    _log(f"parts per head {parts}: {sh}")
    K, V = W.make_kv(3, sh)
    rng = np.random.default_rng(300 + parts)
    widths = np.array([2, 3, 4, 8], np.uint8)
    bk = rng.choice(widths, size=K.shape[:3], p=(0.4, 0.4, 0.15, 0.05))
    bv = rng.choice(widths, size=K.shape[:3], p=(0.6, 0.25, 0.1, 0.05))
    qn = np.full(sh.n_kv_heads, 0.02, F32)
    gc = qaq.Cache(qaq.make_config(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.context + 1, qn.tolist()))
    gc.quantize_append(dev(K), dev(V), dev(bk), dev(bv))
    q = W.make_queries(3, sh)[0]
    kn, vn = W.make_new_token(3, sh)
    X, S = gc.decode_attention(dev(q), dev(kn), dev(vn), want_scores=True)
    _global_properties(X, S, V, vn)
    Xg, Sg = X.cpu().numpy(), S.cpu().numpy()
    X2, _ = gc.decode_attention(dev(q), dev(kn), dev(vn))                 # without scores: no logit store in LDS
    np.testing.assert_array_equal(X2.cpu().numpy(), Xg)
    for b, h in _sample_units(sh, 4, 31 + parts):
        oc, G = _unit_oracle(sh, qn, b, h)
        oc.append(K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1], bk[b:b + 1, h:h + 1], bv[b:b + 1, h:h + 1])
        Xo, So = oc.decode_attention(q[b:b + 1, h * G:(h + 1) * G], kn[b:b + 1, h:h + 1], vn[b:b + 1, h:h + 1])
        ex, es = attention_errors(Xg[b:b + 1, h * G:(h + 1) * G], Sg[b:b + 1, h * G:(h + 1) * G], Xo, So)
        _log(f"  unit b={b} h={h}: max rel err X {ex.max():.2e}, S {es.max():.2e}")
        assert ex.max() < TOL and es.max() < TOL


def test_one_kernel_attention_with_more_tiles_than_lds_holds_logits_for():
    """256 query heads and 36 tiles each: four parts per head in one workgroup, but the head's raw
    logits (36 KB) do not fit next to the parts' working blocks, so they wait in the score buffer until
    the workgroup has merged its parts.  Sampled units against the oracle, all heads against
    the properties that hold at any size, and the output again without the scores."""
    sh = W.shape(3, batch=8, n_q_heads=32, n_kv_heads=32, head_dim=64, context=9000)
    _log(f"one kernel, logits in the score buffer: {sh}")
    K, V = W.make_kv(3, sh)
    rng = np.random.default_rng(411)
    widths = np.array([2, 3, 4, 8], np.uint8)
    bk = rng.choice(widths, size=K.shape[:3], p=(0.5, 0.4, 0.07, 0.03))
    bv = rng.choice(widths, size=K.shape[:3], p=(0.8, 0.15, 0.03, 0.02))
    qn = np.full(sh.n_kv_heads, 0.02, F32)
    gc = qaq.Cache(qaq.make_config(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.context + 1, qn.tolist()))
    gc.quantize_append(dev(K), dev(V), dev(bk), dev(bv))
    q = W.make_queries(3, sh)[0]
    kn, vn = W.make_new_token(3, sh)
    gc.profile_begin(1)
    X, S = gc.decode_attention(dev(q), dev(kn), dev(vn), want_scores=True)
    t_tile, t_merge = gc.profile_read()
    gc.profile_begin(0)
    assert t_merge == [0.0], "the call was expected to run as one kernel"
    _global_properties(X, S, V, vn)
    Xg, Sg = X.cpu().numpy(), S.cpu().numpy()
    X2, _ = gc.decode_attention(dev(q), dev(kn), dev(vn))
    np.testing.assert_array_equal(X2.cpu().numpy(), Xg)
    for b, h in _sample_units(sh, 4, 77):
        oc, G = _unit_oracle(sh, qn, b, h)
        oc.append(K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1], bk[b:b + 1, h:h + 1], bv[b:b + 1, h:h + 1])
        Xo, So = oc.decode_attention(q[b:b + 1, h * G:(h + 1) * G], kn[b:b + 1, h:h + 1], vn[b:b + 1, h:h + 1])
        ex, es = attention_errors(Xg[b:b + 1, h * G:(h + 1) * G], Sg[b:b + 1, h * G:(h + 1) * G], Xo, So)
        _log(f"  unit b={b} h={h}: max rel err X {ex.max():.2e}, S {es.max():.2e}")
        assert ex.max() < TOL and es.max() < TOL


def test_full_size_decode_update_across_a_tile_border():
    """Config 2 at full size through the call the benchmark times for the second half of a
    step: qaq_decode_update on all 256 (sequence, head) units at once, four consecutive decode
    steps from 4094 cached tokens (the third one opens a 17th tile per head), the unquantized
    copies resident so that tokens widen, without the width outputs in two of the steps (the
    form the benchmark runs: key tiles inside their threshold interval are skipped).  The
    cache starts from prompt encoding at hyper-parameters close to the benchmark's operating
    point.  Sampled units follow the oracle at every step: scores and outputs of the attention
    within 2e-3, widths, [min,max], outlier lists and packed codes bit for bit."""
    import torch
    sh = W.shape(2)
    steps, T0, n = 4, 4094, 5
    Tcap = T0 + steps
    G = sh.n_q_heads // sh.n_kv_heads
    _log(f"full size decode update cfg=2 shape={sh} prompt={T0} steps={steps}")
    K, V = W.make_kv(2, sh, n_tokens=T0)
    q_last = np.ascontiguousarray(W.make_queries(2, sh, n=n, seed_offset=3).transpose(1, 2, 0, 3))
    qcal = W.make_queries(2, sh, n=4, seed_offset=7).astype(np.float64)
    qn = np.full(sh.n_kv_heads, float(np.quantile((qcal ** 2).sum(-1).reshape(-1), 0.9)) / sh.head_dim, F32)
    kw = dict(sigma_s_max=1.8e-5, sigma_x_max=1.85e-2, window=5)
    gc = qaq.Cache(qaq.make_config(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, Tcap, qn.tolist(), **kw))
    Kd, Vd = dev(K), dev(V)
    rows = gc.prefill_window(dev(q_last), Kd).cpu().numpy()
    gc.quantize_append_selected(Kd, Vd)
    oK = torch.zeros((sh.batch, sh.n_kv_heads, Tcap, sh.head_dim), dtype=torch.float16, device="cuda")
    oV = torch.zeros_like(oK)
    oK[:, :, :T0] = Kd; oV[:, :, :T0] = Vd
    del Kd, Vd
    units = _sample_units(sh, 4, 41)
    oracles = {}
    for b, h in units:
        oc, _ = _unit_oracle(sh, qn, b, h, **kw)
        unit_rows = [rows[i][b:b + 1, h * G:(h + 1) * G, : T0 - n + i + 1] for i in range(n)]
        oc.prefill(q_last[b:b + 1, h * G:(h + 1) * G], K[b:b + 1, h:h + 1], V[b:b + 1, h:h + 1], score_rows=unit_rows)
        oracles[(b, h)] = (oc, K[b:b + 1, h:h + 1].copy(), V[b:b + 1, h:h + 1].copy())
    qs = W.make_queries(2, sh, n=steps, seed_offset=1)
    served0 = gc.stats().served_upgrades
    for s in range(steps):
        kn, vn = W.make_new_token(2, sh, step=s)
        X, S = gc.decode_attention(dev(qs[s]), dev(kn), dev(vn), want_scores=True)
        Xg, Sg = X.cpu().numpy(), S.cpu().numpy()
        want_bits = s % 2 == 0
        bk_g, bv_g = gc.decode_update(S, dev(kn), dev(vn), oK, oV, want_bits=want_bits)
        torch.cuda.synchronize()
        assert gc.length() == T0 + s + 1
        # the call wrote the new token into the copies
        np.testing.assert_array_equal(oK[:, :, T0 + s].cpu().numpy(), kn)
        np.testing.assert_array_equal(oV[:, :, T0 + s].cpu().numpy(), vn)
        exK = {k: v.cpu().numpy() for k, v in gc.export_canonical(0).items()}
        exV = {k: v.cpu().numpy() for k, v in gc.export_canonical(1).items()}
        widened = 0
        for b, h in units:
            oc, Ko, Vo = oracles[(b, h)]
            Xo, So = oc.decode_attention(qs[s][b:b + 1, h * G:(h + 1) * G], kn[b:b + 1, h:h + 1], vn[b:b + 1, h:h + 1])
            ex, es = attention_errors(Xg[b:b + 1, h * G:(h + 1) * G], Sg[b:b + 1, h * G:(h + 1) * G], Xo, So)
            assert ex.max() < TOL and es.max() < TOL, (s, b, h, ex.max(), es.max())
            Ko = np.concatenate([Ko, kn[b:b + 1, h:h + 1, None]], 2); Vo = np.concatenate([Vo, vn[b:b + 1, h:h + 1, None]], 2)
            before = oc.V[0][0].bits.copy()
            oc.append(kn[b:b + 1, h:h + 1, None], vn[b:b + 1, h:h + 1, None])
            oc.observe(Sg[b:b + 1, h * G:(h + 1) * G])
            bko, bvo = oc.select_bits()
            oc.requantize(bko, bvo, Ko, Vo)
            widened += int((bvo[0, 0, :-1] > before).sum())
            oracles[(b, h)] = (oc, Ko, Vo)
            if want_bits:
                np.testing.assert_array_equal(bk_g[b, h].cpu().numpy(), bko[0, 0])
                np.testing.assert_array_equal(bv_g[b, h].cpu().numpy(), bvo[0, 0])
            _compare_unit(exK, oc.K[0][0], b, h, sh.head_dim, oc.cfg.n_o(), f"step {s} K b={b} h={h}")
            _compare_unit(exV, oc.V[0][0], b, h, sh.head_dim, oc.cfg.n_o(), f"step {s} V b={b} h={h}")
        _log(f"  step {s}: {T0 + s + 1} cached tokens, {widened} value tokens widened in the {len(units)} sampled units")
        assert widened > 0, "the case must exercise widening from the unquantized copies"
    st = gc.stats()
    assert st.refused_upgrades == 0 and st.served_upgrades > served0
    assert sum(st.hist_k) == sum(st.hist_v) == sh.batch * sh.n_kv_heads * Tcap
