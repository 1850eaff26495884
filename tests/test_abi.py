"""The C ABI library loads and exports every function include/usp.h declares; argument
validation that needs no GPU rejects bad calls with the documented status."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "usp.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(usp_[a-z0-9_]+)\s*\(", src)))


def _lib():
    path = os.path.join(ROOT, "paper_2602_10940_amd", "libusp.so")
    if not os.path.exists(path):
        from paper_2602_10940_amd import build
        build.build()
    return ctypes.CDLL(path)


def test_header_symbols_exported():
    lib = _lib()
    names = _declared()
    assert {"usp_ring_attn_fwd", "usp_lse_merge", "usp_fp8_quant", "usp_fp8_dequant",
            "usp_ring_attn_workspace_bytes", "usp_last_error", "usp_version"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_binding_declares_same_exports():
    from paper_2602_10940_amd import binding
    assert sorted(binding.EXPORTS) == _declared()


def test_validation_without_gpu():
    lib = _lib()
    lib.usp_last_error.restype = ctypes.c_char_p
    i64, i32, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p
    lib.usp_fp8_quant.argtypes = [i64, i64, i32, vp, vp, vp, vp]
    assert lib.usp_fp8_quant(4, 12, 1, None, None, None, None) == -1        # cols % 8
    assert b"multiple of 8" in lib.usp_last_error()
    assert lib.usp_fp8_quant(4, 16, 7, None, None, None, None) == -1        # dtype
    assert lib.usp_fp8_quant(4, 16, 1, None, None, None, None) == -1        # null pointers
    assert lib.usp_fp8_quant(0, 16, 1, None, None, None, None) == 0         # empty: nothing to do
    lib.usp_lse_merge.argtypes = [i64, i32, i32, vp, vp, vp, vp, vp, vp, vp]
    assert lib.usp_lse_merge(8, 12, 1, None, None, None, None, None, None, None) == -1
    assert lib.usp_lse_merge(0, 128, 1, None, None, None, None, None, None, None) == 0


def test_diag_library_is_separate_from_the_abi():
    """The MFMA-rate probe and the arrival-wait hook live in libusp_diag.so with a header of their own:
    include/usp.h declares neither, libusp.so exports neither."""
    lib = _lib()
    assert not hasattr(lib, "usp_diag_mfma_rate") and not hasattr(lib, "usp_probe_mfma_rate")
    assert all(not n.startswith("usp_diag") and "probe" not in n for n in _declared())
    from paper_2602_10940_amd import diag
    dl = diag.load_diag_library()
    lib.usp_last_error.restype = ctypes.c_char_p
    assert dl.usp_diag_mfma_rate(0, 10, 1, 0, None, None, None) == -1         # wgs out of range
    assert dl.usp_diag_mfma_rate(4, 10, 1, 0, None, None, None) == -1         # NULL buffers
    assert b"NULL" in lib.usp_last_error()
    src = open(os.path.join(ROOT, "paper_2602_10940_amd", "csrc", "diag", "usp_diag.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    for n in sorted(set(re.findall(r"\b(usp_diag_[a-z0-9_]+)\s*\(", src))):
        assert hasattr(dl, n), n


def test_workspace_sizes_and_descriptor_checks():
    from paper_2602_10940_amd import binding as b
    lib = b.load_library()
    lens = (ctypes.c_int32 * 4)(1152, 1152, 1152, 1152)
    d = b.AttnDesc()
    d.B, d.H, d.d, d.Sq, d.n_chunks = 1, 24, 128, 1152, 4
    d.chunk_len = ctypes.cast(lens, ctypes.POINTER(ctypes.c_int32))
    d.qo_dtype = d.kv_dtype = b.USP_BF16
    for i, s in enumerate((24 * 1152 * 128, 1152 * 128, 128)):
        d.q_stride[i] = d.o_stride[i] = s
    rows = 24 * 1152
    # bf16 d=128: per-(head, 64-key tile) records of 1 KB for masks / scales / ragged chunks, plus
    # one live-tile count per batch entry (256-byte granularity)
    recs = 24 * (1152 // 64) * 1024 + 256
    # one launch over the four chunks: records of all 4 * 18 tiles per head, should a chunk come with a mask
    ring_recs = 24 * 72 * 1024
    assert b.usp_ring_attn_workspace_bytes(d) == rows * 128 * 4 + recs + ring_recs     # fp32 carried O
    d.flags = b.USP_ATTN_STEPWISE
    assert b.usp_ring_attn_workspace_bytes(d) == rows * 128 * 4 + recs
    d.flags = b.USP_ATTN_DOUBLE_BUFFER
    assert b.usp_ring_attn_workspace_bytes(d) == rows * 128 * 4 + 4 * rows * 128 * 2 + recs
    d.flags = b.USP_ATTN_FUSED_PREFETCH | b.USP_ATTN_STEPWISE             # same two staging buffers
    assert b.usp_ring_attn_workspace_bytes(d) == rows * 128 * 4 + 4 * rows * 128 * 2 + recs
    # transfers inside one launch over the whole ring: a buffer (K | V) for each of the 3 later chunks
    # on top, and the arrival counters
    d.flags = b.USP_ATTN_FUSED_PREFETCH
    assert b.usp_ring_attn_workspace_bytes(d) == rows * 128 * 4 + 4 * rows * 128 * 2 + recs + 3 * 2 * rows * 128 * 2 + 256 + ring_recs
    for both in (b.USP_ATTN_FUSED_PREFETCH | b.USP_ATTN_DOUBLE_BUFFER,
                 b.USP_ATTN_KERNEL_WIDE | b.USP_ATTN_KERNEL_SPLIT, b.USP_ATTN_KERNEL_SPLIT | b.USP_ATTN_KERNEL_MIXED):
        d.flags = both
        with pytest.raises(b.UspError):
            b.usp_ring_attn_workspace_bytes(d)
    d.flags = b.USP_ATTN_DOUBLE_BUFFER
    d.kv_dtype = b.USP_FP8_E4M3FN
    fp8 = b.usp_ring_attn_workspace_bytes(d)
    assert fp8 == rows * 128 * 4 + 2 * (2 * rows * 128 + 2 * rows * 4) + 2 * rows * 128 * 2 + recs
    # FP8 chunks decoded inside one launch over the ring (plain call or fused prefetch): on top of the
    # per-chunk form's buffers (fp32 carried O, one decoded K | V, records), bf16 K | V of every chunk,
    # the records of all 4 * 18 tiles per head and the arrival counters
    per_chunk = rows * 128 * 4 + 2 * rows * 128 * 2 + recs
    one_launch = 4 * 2 * rows * 128 * 2 + 24 * 72 * 1024 + 256
    d.flags = 0
    assert b.usp_ring_attn_workspace_bytes(d) == per_chunk + one_launch
    d.flags = b.USP_ATTN_STEPWISE
    assert b.usp_ring_attn_workspace_bytes(d) == per_chunk
    d.flags = b.USP_ATTN_FUSED_PREFETCH
    assert b.usp_ring_attn_workspace_bytes(d) == fp8 + one_launch
    d.n_chunks = 1; d.flags = 0; d.kv_dtype = b.USP_BF16
    assert b.usp_ring_attn_workspace_bytes(d) == recs
    d.d = 64                              # bf16 d = 64 runs on the matrix-core kernels in place: nothing but the records
    for i, s in enumerate((24 * 1152 * 64, 1152 * 64, 64)):
        d.q_stride[i] = d.o_stride[i] = s
    assert b.usp_ring_attn_workspace_bytes(d) == recs
    d.qo_dtype = d.kv_dtype = b.USP_F32                                    # generic kernel: nothing
    for i, s in enumerate((24 * 1152 * 64, 1152 * 64, 64)):
        d.q_stride[i] = d.o_stride[i] = s
    assert b.usp_ring_attn_workspace_bytes(d) == 0
    d.qo_dtype = d.kv_dtype = b.USP_BF16
    d.d = 100
    with pytest.raises(b.UspError):
        b.usp_ring_attn_workspace_bytes(d)


def test_noalloc_entry_point_limits_without_gpu():
    """usp_ring_attn_fwd_noalloc refuses, before any HIP call, a descriptor that needs more workspace
    than its built-in scratch holds, and the side-stream schedule."""
    from paper_2602_10940_amd import binding as b
    lib = b.load_library()
    hdr = open(os.path.join(ROOT, "include", "usp.h")).read()
    m = re.search(r"#define\s+USP_NOALLOC_SCRATCH_BYTES\s+\((\d+)u\s*<<\s*(\d+)\)", hdr)
    assert m and (int(m.group(1)) << int(m.group(2))) == b.USP_NOALLOC_SCRATCH_BYTES
    lens = (ctypes.c_int32 * 2)(4096, 4096)
    d = b.AttnDesc()
    d.B, d.H, d.d, d.Sq, d.n_chunks = 1, 24, 128, 4096, 2
    d.chunk_len = ctypes.cast(lens, ctypes.POINTER(ctypes.c_int32))
    d.qo_dtype = b.USP_BF16
    d.kv_dtype = b.USP_FP8_E4M3FN
    for i, s in enumerate((24 * 4096 * 128, 4096 * 128, 128)):
        d.q_stride[i] = d.o_stride[i] = s
    assert b.usp_ring_attn_workspace_bytes(d) > b.USP_NOALLOC_SCRATCH_BYTES
    assert lib.usp_ring_attn_fwd_noalloc(ctypes.byref(d), None, None, None, None, None, None, None, None, None) == b.USP_ERR_WORKSPACE
    assert b"scratch" in lib.usp_last_error()
    d.kv_dtype = b.USP_BF16
    d.Sq = 256
    lens[0] = lens[1] = 64
    d.flags = b.USP_ATTN_DOUBLE_BUFFER
    assert lib.usp_ring_attn_fwd_noalloc(ctypes.byref(d), None, None, None, None, None, None, None, None, None) == b.USP_ERR_UNSUPPORTED


def test_header_is_plain_c():
    """include/usp.h is the boundary: it must compile as C99 and as C++ with nothing but the standard headers."""
    import shutil
    import subprocess
    hdr = os.path.join(ROOT, "include", "usp.h")
    for cc, std, lang in (("gcc", "-std=c99", "c"), ("g++", "-std=c++11", "c++")):
        if shutil.which(cc) is None:
            pytest.skip(cc + " not available")
        r = subprocess.run([cc, std, "-Wall", "-Werror", "-fsyntax-only", "-x", lang, hdr], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_batch_times_heads_beyond_the_launch_grid_is_refused():
    """(batch, head) pairs index a 16-bit grid dimension in some kernels: more than 65535 of them are
    refused when the call is planned, not at launch."""
    from paper_2602_10940_amd import binding as b
    lens = (ctypes.c_int32 * 1)(64)
    d = b.AttnDesc()
    d.B, d.H, d.d, d.Sq, d.n_chunks = 4, 16384, 128, 64, 1
    d.chunk_len = ctypes.cast(lens, ctypes.POINTER(ctypes.c_int32))
    d.qo_dtype = d.kv_dtype = b.USP_BF16
    for i, s in enumerate((16384 * 64 * 128, 64 * 128, 128)):
        d.q_stride[i] = d.o_stride[i] = s
    with pytest.raises(b.UspError, match="65535"):
        b.usp_ring_attn_workspace_bytes(d)
    d.H = 16383                                   # 65532 pairs: planned
    assert b.usp_ring_attn_workspace_bytes(d) > 0


def test_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    """Without the built library the binding raises; no Python or CPU path stands in for the kernels."""
    from paper_2602_10940_amd import binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", str(tmp_path / "libusp.so"))
    with pytest.raises(b.UspError, match="no fallback"):
        b.load_library()
    with pytest.raises(b.UspError):
        b.usp_version()


def test_product_code_does_not_import_the_oracle():
    """oracle/ is test infrastructure: nothing under the package (Python or HIP sources) names it."""
    import glob
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2602_10940_amd")
    files = glob.glob(os.path.join(pkg, "*.py")) + glob.glob(os.path.join(pkg, "csrc", "*.*")) + \
        glob.glob(os.path.join(pkg, "csrc", "diag", "*.*")) + \
        glob.glob(os.path.join(root, "include", "*.h"))
    assert files
    for f in files:
        text = open(f, encoding="utf-8", errors="replace").read()
        assert "import oracle" not in text and "from oracle" not in text and "usp_oracle" not in text, f
