"""Boundary checks that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad descriptors with the documented error codes."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2507_20030_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions():
    src = open(os.path.join(ROOT, "include", "iwdft.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b((?:iwdft_|compressed_)\w+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    names = header_functions()
    assert set(names) == set(B.EXPORTED)
    for n in names:
        assert hasattr(lib, n), n


def desc(**kw):
    args = dict(n_layers=2, batch=1, n_kv_heads=2, n_q_heads=4, head_dim=128, kv_dtype=B.IWDFT_BF16,
                M=64, bins=[np.arange(8), np.array([0, 3, 9, 63])])
    args.update(kw)
    return B.Descriptor(**args)


def test_query_bytes_accounts_for_padded_rows():
    d = desc()
    state, ws = B.iwdft_query_bytes(d)
    # rows are padded to 32 bins: 2 layers * 2 slices * 128 channels * 32 * 8 B per tensor
    coef = 2 * 2 * 128 * 32 * 8
    assert state >= 2 * coef and state < 2 * coef + 4096
    assert ws >= 2 * (2 * 2 * 2 * 32 * 8)
    assert state % 256 == 0 and ws % 256 == 0


@pytest.mark.parametrize("kw,code", [
    (dict(n_layers=0, bins=[]), B.IWDFT_ERR_ARG),
    (dict(n_q_heads=3), B.IWDFT_ERR_ARG),
    (dict(kv_dtype=7), B.IWDFT_ERR_ARG),
    (dict(M=0), B.IWDFT_ERR_ARG),
    (dict(M=(1 << 30) + 1), B.IWDFT_ERR_ARG),
    (dict(flags=1 << 20), B.IWDFT_ERR_ARG),
    (dict(write_every=17), B.IWDFT_ERR_ARG),
    (dict(flags=B.IWDFT_FLAG_DENSE_PREFILL | B.IWDFT_FLAG_FFT_PREFILL), B.IWDFT_ERR_ARG),
    (dict(flags=B.IWDFT_FLAG_FFT_PREFILL), B.IWDFT_ERR_UNSUPPORTED),   # M = 64: below the FFT's smallest length
    (dict(flags=B.IWDFT_FLAG_FFT_PREFILL, M=768), B.IWDFT_ERR_UNSUPPORTED),  # not a power of two
    (dict(head_dim=64), B.IWDFT_ERR_UNSUPPORTED),
    (dict(n_sink=-1), B.IWDFT_ERR_ARG),
    (dict(n_recent=-3), B.IWDFT_ERR_ARG),
    (dict(n_sink=1000, n_recent=25), B.IWDFT_ERR_UNSUPPORTED),
    # a long prime M: no O(M log M) attention, too many terms for the direct sums chosen unasked
    (dict(M=1048583, bins=[np.arange(2048), np.arange(8)]), B.IWDFT_ERR_UNSUPPORTED),
    (dict(bins=[np.arange(8), np.array([0, 3, 3, 9])]), B.IWDFT_ERR_BINS),
    (dict(bins=[np.arange(8), np.array([5, 3])]), B.IWDFT_ERR_BINS),
    (dict(bins=[np.arange(8), np.array([0, 64])]), B.IWDFT_ERR_BINS),
    (dict(bins=[np.arange(8), np.array([-1, 2])]), B.IWDFT_ERR_BINS),
    (dict(bins=[np.arange(8), np.zeros(0, np.int32)]), B.IWDFT_ERR_BINS),
    (dict(bins=[np.arange(8), np.arange(4)], bin_weights=[np.ones(8), np.array([1, np.nan, 1, 1])]),
     B.IWDFT_ERR_BINS),
])
def test_bad_descriptors_are_rejected(kw, code):
    with pytest.raises(B.IwdftError) as e:
        B.iwdft_query_bytes(desc(**kw))
    assert e.value.code == code
    assert B.iwdft_last_error()


def test_null_pointers_and_null_ctx():
    lib = B.load_library()
    assert lib.iwdft_query_bytes(None, None, None) == B.IWDFT_ERR_ARG
    s = ctypes.c_size_t()
    assert lib.iwdft_query_bytes(None, ctypes.byref(s), ctypes.byref(s)) == B.IWDFT_ERR_ARG
    assert lib.iwdft_num_tokens(None) == -1
    assert lib.iwdft_destroy(None) == B.IWDFT_OK
    assert lib.iwdft_set_num_tokens(None, 5) == B.IWDFT_ERR_ARG
    assert lib.iwdft_prefill_kind(None) == -1
    assert lib.iwdft_attn_kind(None) == -1
    assert lib.iwdft_attn_pipelined(None) == -1
    assert lib.iwdft_flush(None, None) == B.IWDFT_ERR_ARG
    assert lib.iwdft_phase_timing(None, 1) == B.IWDFT_ERR_ARG
    ms, n = (ctypes.c_double * 3)(), ctypes.c_int64()
    assert lib.iwdft_phase_times(None, ms, ctypes.byref(n)) == B.IWDFT_ERR_ARG
    d = desc()
    out = ctypes.c_void_p()
    assert lib.iwdft_create(ctypes.byref(d.c), None, 0, None, 0, ctypes.byref(out)) == B.IWDFT_ERR_ARG
    assert lib.iwdft_create(ctypes.byref(d.c), None, 0, None, 0, None) == B.IWDFT_ERR_ARG


def test_workspace_holds_the_deferred_tokens():
    bins = [np.arange(40), np.arange(40)]
    ws1 = B.iwdft_query_bytes(desc(M=1024, bins=bins))[1]
    ws8 = B.iwdft_query_bytes(desc(M=1024, bins=bins, write_every=8))[1]
    # 8 rows of 128 bf16 for K and for V per slice, and 16 floats per (slice, query head)
    assert ws8 - ws1 >= 2 * (4 * 8 * 128 * 2) + 4 * 2 * 16 * 4
    # M = 64 has no FFT attention path, so nothing is deferred and nothing is reserved
    assert B.iwdft_query_bytes(desc(write_every=8))[1] == B.iwdft_query_bytes(desc())[1]


def test_query_bytes_grows_with_exact_windows():
    s0, w0 = B.iwdft_query_bytes(desc())
    s1, w1 = B.iwdft_query_bytes(desc(n_sink=10, n_recent=50))
    # 4 slices x (10 + 50) tokens x 128 channels x 2 B (bf16), K and V
    assert s1 - s0 >= 2 * 4 * 60 * 128 * 2 and s1 - s0 < 2 * 4 * 60 * 128 * 2 + 2048
    assert w1 > w0


def test_static_scratch_symbol_is_visible_to_the_hip_runtime(tmp_path):
    """The HIP runtime finds a registered device variable by name in the code object and aborts the process
    when it is missing, so the library's file-scope scratch array must be a GLOBAL symbol of the device code."""
    import shutil
    import subprocess
    obj = os.path.join(os.path.dirname(B.LIB_PATH), "_build", "api.o")
    tools = "/opt/rocm/llvm/bin"
    if not (os.path.exists(obj) and os.path.exists(f"{tools}/clang-offload-bundler") and shutil.which("objcopy")):
        pytest.skip("object file or LLVM tools not available")
    fat, co = str(tmp_path / "fat.bin"), str(tmp_path / "dev.co")
    subprocess.run(["objcopy", "-O", "binary", "--only-section=.hip_fatbin", obj, fat], check=True)
    subprocess.run([f"{tools}/clang-offload-bundler", "--unbundle", "--type=o", f"--input={fat}",
                    "--targets=hipv4-amdgcn-amd-amdhsa--gfx950", f"--output={co}"], check=True)
    syms = subprocess.run([f"{tools}/llvm-readelf", "-s", co], check=True, capture_output=True, text=True).stdout
    rows = [ln.split() for ln in syms.splitlines() if ln.strip().endswith("scratch")]
    assert rows, "no scratch symbol in the device code object"
    assert all(r[4] == "GLOBAL" and int(r[2]) == B.IWDFT_STATIC_SCRATCH_BYTES for r in rows), rows


def test_plan_accepts_long_contexts_with_a_small_divisor_and_the_direct_sums_on_request():
    # 2^20 - 64 = 129 * 8128: 129 decimated blocks of 8128 points (chirp-z); a long prime is accepted when the caller
    # insists on the direct sums
    big = [np.arange(2048), np.arange(8)]
    assert B.iwdft_query_bytes(desc(M=(1 << 20) - 64 * 1, bins=big))[0] > 0
    assert B.iwdft_query_bytes(desc(M=1048583, bins=big, flags=B.IWDFT_FLAG_DIRECT_SYNTHESIS))[0] > 0
    assert B.iwdft_query_bytes(desc(M=10007, bins=big))[0] > 0      # 10007 * 2048 terms: the direct sums are fine
