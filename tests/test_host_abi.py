"""Host-side checks that need no GPU: the library loads, exports what the header
declares, rejects bad arguments, and its code layout is a bijection."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2403_04643_amd import qaq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    """Every function declared in include/*.h (the product interface and the measurement / test aids)."""
    inc = os.path.join(ROOT, "include")
    names = set()
    for f in sorted(os.listdir(inc)):
        if f.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, f)).read(), flags=re.S)
            names |= set(re.findall(r"\b(qaq_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = qaq.load()
    names = _declared()
    assert {"qaq_select_bits", "qaq_quantize_append", "qaq_requantize", "qaq_decode_attention",
            "qaq_dequantize"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
        assert n in qaq.SIGNATURES, f"binding lacks {n}"
    assert sorted(qaq.SIGNATURES) == names


def test_config_validation_without_gpu():
    lib = qaq.load()
    good = qaq.make_config(2, 8, 8, 128, 1000, [0.01] * 8)
    n = lib.qaq_arena_bytes(C.byref(good))
    assert n > 2 * 2 * 8 * 1024 * 128          # at least the 8-bit codes of K and V
    assert lib.qaq_outliers_per_side(C.byref(good)) == 1
    assert lib.qaq_arena_bytes(C.byref(qaq.make_config(2, 8, 8, 128, 1000, [0.01] * 8, bit_set=(1, 2, 3, 4, 8)))) == n
    for kw in (dict(head_dim=96), dict(bit_set=(2, 5)), dict(bit_set=(0, 2)), dict(bit_set=(3, 2)), dict(window=0),
               dict(n_outlier_per_side=5), dict(sigma_s_max=0.0), dict(n_q_heads=7)):
        args = dict(batch=2, n_q_heads=8, n_kv_heads=8, head_dim=128, max_tokens=1000, qnorm2=[0.01] * 8)
        args.update(kw)
        bad = qaq.make_config(**args)
        assert lib.qaq_arena_bytes(C.byref(bad)) == 0
        assert lib.qaq_last_error()
    h = C.c_void_p()
    assert lib.qaq_create(C.byref(good), None, n, C.byref(h)) == qaq.ERR_INVALID_ARG
    assert lib.qaq_create(C.byref(good), 256, n - 1, C.byref(h)) == qaq.ERR_CAPACITY
    assert lib.qaq_create(C.byref(good), 257, n, C.byref(h)) == qaq.ERR_INVALID_ARG
    assert lib.qaq_reset(None) == qaq.ERR_INVALID_ARG
    assert b"NULL" in lib.qaq_last_error()
    no_out = qaq.make_config(1, 4, 4, 64, 10, [1.0] * 4, outlier_frac=0.0)
    assert lib.qaq_outliers_per_side(C.byref(no_out)) == 0
    four = qaq.make_config(1, 4, 4, 128, 10, [1.0] * 4, outlier_frac=0.05)
    assert lib.qaq_outliers_per_side(C.byref(four)) == 4


@pytest.mark.parametrize("side", [0, 1])
@pytest.mark.parametrize("D", [64, 128])
def test_layout_is_a_bijection(side, D):
    """Every code bit of every token lands on its own bit of the tile image, inside the
    region bounds and the reserved capacity; the image has no other holes than the
    documented padding."""
    rng = np.random.default_rng(D + side)
    cap = qaq.load().qaq_debug_tile_capacity(side, D)
    cases = [(256, 0, 0, 0, 0), (0, 256, 0, 0, 0), (0, 0, 256, 0, 0), (0, 0, 0, 256, 0), (0, 0, 0, 0, 256),
             (1, 1, 1, 1, 1), (17, 9, 3, 33, 21), (1, 1, 1, 252, 1)]
    for k in range(6):
        cut = np.sort(rng.integers(0, 257, 4))
        if k < 3:
            cut[3] = 256                      # no 1-bit tokens: the layout of the paper's width set
        cases.append((cut[0], cut[1] - cut[0], cut[2] - cut[1], cut[3] - cut[2], 256 - cut[3]))
    for n3, n2, n4, n8, n1 in cases:
        counts = (int(n3), int(n2), int(n4), int(n8), int(n1))
        used = np.zeros(cap * 8, dtype=np.uint8)
        end = None
        def mark(bf, idx, width_mask_bits):
            nonlocal end
            for d in range(D):
                off, sh, end = qaq.debug_field(side, D, counts, bf, idx, d)
                assert off % 4 == 0 and sh + width_mask_bits <= 32
                lo = off * 8 + sh
                assert lo + width_mask_bits <= end * 8 <= cap * 8
                assert not used[lo:lo + width_mask_bits].any(), (counts, bf, idx, d)
                used[lo:lo + width_mask_bits] = 1
        for s in range(n3 + n2):
            mark(2, s, 2)
        for s in range(n3):
            mark(1, s, 1)
        for s in range(n4):
            mark(4, s, 4)
        for s in range(n8):
            mark(8, s, 8)
        for s in range(n1):
            mark(0, s, 1)
        total_bits = D * (3 * n3 + 2 * n2 + 4 * n4 + 8 * n8 + n1)
        assert used.sum() == total_bits
        if end is not None:
            pad = end * 8 - total_bits
            # at most one partly filled group per region: keys 15 records of D/4 + D/8 + D/2 + D/8
            # bytes, values 15/16 of a 4D- and of two 2D-byte units and 7/8 of a 4D-byte half-unit
            assert pad <= 8 * (15 * D)


# ---- code objects in the built library: the kernels on the decode path keep their working set in registers ----

def _gfx950_code_objects(path):
    """The gfx950 code objects inside the library's .hip_fatbin section (one offload bundle per source file;
    bundle layout: magic, u64 entry count, then per entry u64 offset, u64 size, u64 triple length, triple)."""
    import struct
    import subprocess
    import tempfile
    objcopy = "/opt/rocm/llvm/bin/llvm-objcopy"
    if not os.path.exists(objcopy):
        pytest.skip("llvm-objcopy not found")
    with tempfile.TemporaryDirectory() as d:
        fat = os.path.join(d, "fat.bin")
        subprocess.run([objcopy, f"--dump-section=.hip_fatbin={fat}", path, os.path.join(d, "unused")], check=True)
        blob = open(fat, "rb").read()
    magic = b"__CLANG_OFFLOAD_BUNDLE__"
    out = []
    at = blob.find(magic)
    while at >= 0:
        p = at + len(magic)
        (n,) = struct.unpack_from("<Q", blob, p)
        p += 8
        for _ in range(n):
            off, size, tl = struct.unpack_from("<QQQ", blob, p)
            triple = blob[p + 24:p + 24 + tl].decode()
            p += 24 + tl
            if "gfx950" in triple:
                out.append(blob[at + off:at + off + size])
        at = blob.find(magic, at + len(magic))
    return out


def _kernel_metadata(code_object):
    """name -> metadata map of every kernel of one code object (the msgpack document of the NT_AMDGPU_METADATA note)."""
    import struct
    import msgpack
    e = code_object
    assert e[:4] == b"\x7fELF" and e[4] == 2
    shoff, = struct.unpack_from("<Q", e, 0x28)
    shentsize, shnum = struct.unpack_from("<HH", e, 0x3A)
    kernels = {}
    for i in range(shnum):
        sh = shoff + i * shentsize
        sh_type, = struct.unpack_from("<I", e, sh + 4)
        off, size = struct.unpack_from("<QQ", e, sh + 0x18)
        if sh_type != 7:       # SHT_NOTE
            continue
        p = off
        while p + 12 <= off + size:
            namesz, descsz, ntype = struct.unpack_from("<III", e, p)
            name = e[p + 12:p + 12 + namesz]
            desc_at = p + 12 + ((namesz + 3) & ~3)
            if name.rstrip(b"\0") == b"AMDGPU" and ntype == 32:
                doc = msgpack.unpackb(e[desc_at:desc_at + descsz], raw=False, strict_map_key=False)
                for k in doc.get("amdhsa.kernels", []):
                    kernels[k[".name"]] = k
            p = desc_at + ((descsz + 3) & ~3)
    return kernels


def test_decode_path_kernels_do_not_spill():
    """A change elsewhere in a source file can push a kernel over its register budget or make the compiler call
    its helpers out of line; both show as private (scratch) memory in the kernel's metadata long before a test of
    the results notices anything.  The kernels of a decode step and of the bulk quantization at the benchmark's
    shape (head_dim 128, one outlier per end, no 1-bit width) are held to none."""
    if not os.path.exists(qaq.LIB_PATH):
        pytest.skip("library not built")
    kernels = {}
    for co in _gfx950_code_objects(qaq.LIB_PATH):
        kernels.update(_kernel_metadata(co))
    assert kernels, "no gfx950 code object found in the library"
    held = {"k_attn_tileILi128ELi2ELi4ELb0": 128, "k_attn_tileILi128ELi2ELi0ELb0": 128, "k_updateILi128": 64,
            "k_selectE": 128, "k_buildILi128ELb1ELb0": 128, "k_attn_combineILi128": 128}
    seen = set()
    for name, k in kernels.items():
        for key, max_vgpr in held.items():
            if key in name:
                seen.add(key)
                assert k[".private_segment_fixed_size"] == 0, (name, k[".private_segment_fixed_size"])
                assert k[".vgpr_count"] <= max_vgpr, (name, k[".vgpr_count"])
    assert seen == set(held), set(held) - seen
