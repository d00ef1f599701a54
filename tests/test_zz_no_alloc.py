"""qaq_decode_attention_static (the entry point for callers that cannot allocate: partial
results in the library's file-scope device array) against qaq_decode_attention on the same
caches: same kernels, same order of operations, so outputs and scores must be identical bit
for bit -- on two calls in a row, the second on a smaller cache (fewer heads and tiles, so it
uses a smaller part of the array the first call left its partial results in)."""
import ctypes as C

import numpy as np
import pytest

from paper_2403_04643_amd import qaq, workloads as W
from tests.parity_util import F32, dev

pytestmark = pytest.mark.gpu


def _cache(sh, seed):
    import torch
    K, V = W.make_kv(3, sh, seed_offset=seed)
    rng = np.random.default_rng(700 + seed)
    widths = np.array([2, 3, 4, 8], np.uint8)
    bk = rng.choice(widths, size=K.shape[:3], p=(0.45, 0.4, 0.1, 0.05))
    bv = rng.choice(widths, size=K.shape[:3], p=(0.7, 0.2, 0.07, 0.03))
    qn = np.full(sh.n_kv_heads, 0.02, F32)
    gc = qaq.Cache(qaq.make_config(sh.batch, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.context + 1, qn.tolist()))
    gc.quantize_append(dev(K), dev(V), dev(bk), dev(bv))
    q = dev(W.make_queries(3, sh, seed_offset=seed)[0])
    kn, vn = W.make_new_token(3, sh, step=seed)
    torch.cuda.synchronize()
    return gc, q, dev(kn), dev(vn)


def test_static_scratch_entry_point_matches_the_arena_one():
    import torch
    print("no-alloc entry point: two calls in a row, the second smaller", flush=True)
    lib = qaq.load()
    # the most the launcher asks for at this GPU's size: four parts per compute unit, head_dim 128
    assert lib.qaq_static_scratch_limit() >= 4 * 256 * 132 * 4
    # few heads and many tiles: a head's tiles are scanned by more than four workgroups, so the
    # scan kernel leaves partial results for the merge kernel (the form that needs scratch)
    big = W.shape(3, batch=1, n_q_heads=8, n_kv_heads=4, head_dim=128, context=5000)     # 20 tiles, 20 parts per head
    small = W.shape(3, batch=1, n_q_heads=4, n_kv_heads=4, head_dim=64, context=1700)    # 7 tiles, 7 parts per head
    # grouped queries: four query heads per pass over a KV head's codes, also a form with partial results
    grouped = W.shape(3, batch=2, n_q_heads=8, n_kv_heads=2, head_dim=128, context=1300)
    shapes = (big, small, grouped)
    cases = [_cache(big, 1), _cache(small, 2), _cache(grouped, 3)]
    ref = []
    for (gc, q, kn, vn), sh in zip(cases, shapes):
        X, S = gc.decode_attention(q, kn, vn, want_scores=True)
        ref.append((X.clone(), S.clone()))
    torch.cuda.synchronize()
    for rep in range(2):
        for i, ((gc, q, kn, vn), sh) in enumerate(zip(cases, shapes)):
            out = torch.full((sh.batch, sh.n_q_heads, sh.head_dim), float("nan"), dtype=torch.float32, device="cuda")
            sc = torch.full((sh.batch, sh.n_q_heads, sh.context + 1), float("nan"), dtype=torch.float32, device="cuda")
            gc.decode_attention_static(q, kn, vn, out, sc)
            torch.cuda.synchronize()
            np.testing.assert_array_equal(out.cpu().numpy(), ref[i][0].cpu().numpy())
            np.testing.assert_array_equal(sc.cpu().numpy(), ref[i][1].cpu().numpy())
    # without the new token and without scores, fp16 output
    gc, q, kn, vn = cases[1]
    X16, _ = gc.decode_attention(q, out_fp32=False)
    out16 = torch.zeros((small.batch, small.n_q_heads, small.head_dim), dtype=torch.float16, device="cuda")
    gc.decode_attention_static(q, None, None, out16)
    np.testing.assert_array_equal(out16.cpu().numpy(), X16.cpu().numpy())
