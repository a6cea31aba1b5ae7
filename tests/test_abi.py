"""The C ABI without a GPU: the library loads, exports every declared symbol, and rejects bad
arguments on the host before anything is launched."""
import ctypes as C
import os
import re

import pytest

from paper_2603_28458_amd import hisa

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(hisa.LIB_PATH):
        from paper_2603_28458_amd.build import build
        build(verbose=False)
    return hisa.lib()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "hisa.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b((?:hisa|dsa)_[a-z0-9_]+)\s*\(", header))
    assert declared == set(hisa.EXPORTS), declared ^ set(hisa.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_status_strings_and_version(lib):
    assert hisa.status_string(0) == "ok"
    assert "m*B >= k" in hisa.status_string(4)
    assert hisa.version().count(".") == 1


def _structs(T=512, H=64, d=128, n_seq=1, s_max=1024, qd=hisa.HISA_BF16, kd=hisa.HISA_BF16, fake=0x1000):
    q = hisa._Queries(fake, fake, None, None, None, T, H, 0, qd)
    k = hisa._Keys(fake, fake, fake, n_seq, s_max, d, kd)
    return q, k


def test_host_side_validation_rejects_before_launch(lib):
    """Pointers here are fake non-null values: every call must fail in validation, never launch."""
    fake = 0x1000
    q, k = _structs()
    i32 = C.c_int32
    # infeasible budgets (Section 4.1: m*B >= k), m < 2
    assert lib.hisa_token_refine_topk(C.byref(q), C.byref(k), 128, 4, fake, 2048, fake, None, None, None, 0, None) == 4
    assert lib.hisa_block_score_topk(C.byref(q), C.byref(k), fake, 1, 128, 1, fake, None, fake, 1 << 30, None) == 4
    # null pointers
    assert lib.hisa_token_refine_topk(C.byref(q), C.byref(k), 128, 8, None, 512, fake, None, None, None, 0, None) == 1
    assert lib.hisa_pool_blocks(C.byref(k), 128, 0, 8, None, 1, None) == 1
    assert lib.dsa_flat_indexer_topk(None, C.byref(k), 64, fake, None, fake, 1 << 30, None) == 1
    # shapes: s_max not a multiple of B, unsupported H / d on the MFMA path, block range
    assert lib.hisa_pool_blocks(C.byref(k), 100, 0, 8, fake, 1, None) == 2
    assert lib.hisa_pool_blocks(C.byref(k), 128, 0, 9, fake, 1, None) == 2
    q2, k2 = _structs(H=48)
    assert lib.dsa_flat_indexer_topk(C.byref(q2), C.byref(k2), 64, fake, None, fake, 1 << 30, None) == 2
    q2, k2 = _structs(d=64)
    assert lib.dsa_flat_indexer_topk(C.byref(q2), C.byref(k2), 64, fake, None, fake, 1 << 30, None) == 2
    assert lib.hisa_token_refine_topk(C.byref(q), C.byref(k), 48, 16, fake, 512, fake, None, None, None, 0, None) == 2
    # a sequence's key array must stay below 2 GiB (32-bit byte offsets)
    q2, k2 = _structs(s_max=1 << 23)
    assert lib.dsa_flat_indexer_topk(C.byref(q2), C.byref(k2), 64, fake, None, fake, 1 << 30, None) == 2
    # dtype combinations
    q2, k2 = _structs(qd=hisa.HISA_F32, kd=hisa.HISA_BF16)
    assert lib.dsa_flat_indexer_topk(C.byref(q2), C.byref(k2), 64, fake, None, fake, 1 << 30, None) == 3
    assert lib.hisa_pool_blocks(C.byref(k), 128, 0, 8, fake, 2, None) == 3
    # workspace missing / too small
    assert lib.dsa_flat_indexer_topk(C.byref(q), C.byref(k), 64, fake, None, None, 0, None) == 5
    assert lib.dsa_flat_indexer_topk(C.byref(q), C.byref(k), 64, fake, None, fake, 100, None) == 5
    assert lib.hisa_block_score_topk(C.byref(q), C.byref(k), fake, 1, 128, 4, fake, None, None, 0, None) == 5
    qs, ks = _structs(T=8)
    assert lib.hisa_token_refine_topk(C.byref(qs), C.byref(ks), 128, 8, fake, 512, fake, None, None, None, 0, None) == 5
    # alignment
    q3 = hisa._Queries(fake + 4, fake, None, None, None, 512, 64, 0, hisa.HISA_BF16)
    assert lib.dsa_flat_indexer_topk(C.byref(q3), C.byref(k), 64, fake, None, fake, 1 << 30, None) == 6


def test_query_and_sequence_counts_beyond_the_launch_limits_are_refused(lib):
    """T <= 4194304 and n_seq <= 65535 (header, "Supported shapes"): every entry point that takes
    queries returns HISA_ERR_SHAPE on the host, before any kernel of the call is enqueued."""
    fake = 0x1000
    big = (1 << 22) + 1
    q, k = _structs(T=big, s_max=65536)
    ok_q, _ = _structs(T=1 << 22, s_max=65536)
    huge = 1 << 40
    assert lib.hisa_block_score_topk(C.byref(q), C.byref(k), fake, 1, 128, 64, fake, None, fake, huge, None) == 2
    assert lib.hisa_token_refine_topk(C.byref(q), C.byref(k), 128, 64, fake, 2048, fake, None, None, fake, huge, None) == 2
    assert lib.hisa_token_refine_topk_static(C.byref(q), C.byref(k), 128, 64, fake, 2048, fake, None, None) == 2
    assert lib.hisa_indexer_topk(C.byref(q), C.byref(k), fake, 1, 128, 64, 2048, None, fake, None, None) == 2
    assert lib.dsa_flat_indexer_topk(C.byref(q), C.byref(k), 2048, fake, None, fake, huge, None) == 2
    # the limit itself passes this check (and fails a later one here: the workspace is too small)
    assert lib.hisa_block_score_topk(C.byref(ok_q), C.byref(k), fake, 1, 128, 64, fake, None, fake, 16, None) == 5
    q2, k2 = _structs(n_seq=65536)
    assert lib.hisa_pool_blocks(C.byref(k2), 128, 0, 8, fake, 1, None) == 2
    assert lib.dsa_flat_indexer_topk(C.byref(q2), C.byref(k2), 64, fake, None, fake, 1 << 30, None) == 2


def test_static_scratch_call_validates_like_the_workspace_call(lib):
    fake = 0x1000
    q, k = _structs(T=8)
    # hisa_token_refine_topk_static(queries, keys, B, m, block_idx, k, topk_idx, topk_scores, stream)
    assert lib.hisa_token_refine_topk_static(None, C.byref(k), 128, 8, fake, 512, fake, None, None) == 1
    assert lib.hisa_token_refine_topk_static(C.byref(q), C.byref(k), 128, 8, None, 512, fake, None, None) == 1
    assert lib.hisa_token_refine_topk_static(C.byref(q), C.byref(k), 128, 4, fake, 2048, fake, None, None) == 4
    assert lib.hisa_token_refine_topk_static(C.byref(q), C.byref(k), 48, 16, fake, 512, fake, None, None) == 2
    # more candidate scores than the static array holds (200 x 65536 x 4 B > 16 MiB): refused
    q2, k2 = _structs(T=200, s_max=131072)
    assert lib.hisa_token_refine_topk_static(C.byref(q2), C.byref(k2), 128, 512, fake, 512, fake, None, None) == 5
    assert hisa.STATIC_SCRATCH_BYTES == 16 << 20
    header = open(os.path.join(ROOT, "include", "hisa.h")).read()
    assert "#define HISA_STATIC_SCRATCH_BYTES (16u << 20)" in header


def test_validation_of_the_auxiliary_entry_points(lib):
    fake = 0x1000
    q, k = _structs()
    assert lib.hisa_pool_append(C.byref(k), 128, None, 16, fake, 1, None) == 1
    assert lib.hisa_pool_append(C.byref(k), 100, fake, 16, fake, 1, None) == 2
    assert lib.hisa_pool_append(C.byref(k), 128, fake, -1, fake, 1, None) == 2
    assert lib.hisa_pool_append(C.byref(k), 128, fake, 16, fake, 2, None) == 3
    assert lib.hisa_pool_append(C.byref(k), 128, fake, 0, fake, 1, None) == 0      # nothing to do, no launch
    assert lib.hisa_block_sparse_tokens(C.byref(q), C.byref(k), 128, 8, None, fake, None) == 1
    assert lib.hisa_block_sparse_tokens(C.byref(q), C.byref(k), 96, 8, fake, fake, None) == 2
    assert lib.hisa_index_iou(None, fake, 4, 4, fake, None) == 1
    assert lib.hisa_index_iou(fake, fake, 0, 4, fake, None) == 2


def test_validation_of_the_single_launch_call_and_the_probes(lib):
    fake = 0x1000
    q, k = _structs()
    bf16 = hisa.HISA_BF16
    # hisa_indexer_topk(queries, keys, pooled, pooled_dtype, B, m, k, block_idx, topk_idx, topk_scores, stream)
    assert lib.hisa_indexer_topk(C.byref(q), C.byref(k), None, bf16, 128, 8, 512, None, fake, None, None) == 1
    assert lib.hisa_indexer_topk(C.byref(q), C.byref(k), fake, bf16, 128, 8, 512, None, None, None, None) == 1
    assert lib.hisa_indexer_topk(C.byref(q), C.byref(k), fake + 4, bf16, 128, 8, 512, None, fake, None, None) == 6
    assert lib.hisa_indexer_topk(C.byref(q), C.byref(k), fake, bf16, 128, 1, 64, None, fake, None, None) == 4    # m < 2
    assert lib.hisa_indexer_topk(C.byref(q), C.byref(k), fake, bf16, 128, 4, 2048, None, fake, None, None) == 4  # m*B < k
    assert lib.hisa_indexer_topk(C.byref(q), C.byref(k), fake, hisa.HISA_F32, 128, 8, 512, None, fake, None, None) == 3
    assert lib.hisa_indexer_topk(C.byref(q), C.byref(k), fake, bf16, 48, 16, 512, None, fake, None, None) == 2   # s_max % B
    q2, k2 = _structs(s_max=1 << 20)
    assert lib.hisa_indexer_topk(C.byref(q2), C.byref(k2), fake, bf16, 64, 128, 512, None, fake, None, None) == 2  # > 8192 blocks
    assert lib.hisa_indexer_topk(C.byref(q2), C.byref(k2), fake, bf16, 256, 128, 512, None, fake, None, None) == 2  # m*B > 16384
    q3, k3 = _structs(qd=hisa.HISA_F32, kd=hisa.HISA_F32, H=4, d=64)
    assert lib.hisa_indexer_topk(C.byref(q3), C.byref(k3), fake, hisa.HISA_F32, 128, 8, 512, None, fake, None, None) == 3
    # probes
    flop = C.c_double(0.0)
    assert lib.hisa_probe_copy(None, fake, 1024, None) == 1
    assert lib.hisa_probe_copy(fake, fake, 1000, None) == 2
    assert lib.hisa_probe_copy(fake + 8, fake, 1024, None) == 6
    assert lib.hisa_probe_mfma(None, 10, C.byref(flop), None) == 1
    assert lib.hisa_probe_mfma(fake, 0, C.byref(flop), None) == 2
    assert lib.hisa_probe_mfma_fp8(None, 10, C.byref(flop), None) == 1
    assert lib.hisa_probe_mfma_fp8(fake, 0, C.byref(flop), None) == 2
    assert lib.hisa_probe_mfma_toggling(None, 10, 0, C.byref(flop), None) == 1
    assert lib.hisa_probe_mfma_toggling(fake, 0, 1, C.byref(flop), None) == 2
    assert lib.hisa_probe_mfma_toggling(fake, 10, 2, C.byref(flop), None) == 2


def test_workspace_sizes(lib):
    q, k = _structs(T=65536, s_max=65536)
    assert lib.hisa_workspace_bytes(hisa.OP_POOL, C.byref(q), C.byref(k), 128, 64, 2048, 0) == 0
    assert lib.hisa_workspace_bytes(hisa.OP_BLOCK_SCORE_TOPK, C.byref(q), C.byref(k), 128, 64, 2048, 0) == 65536 * 512 * 4
    assert lib.hisa_workspace_bytes(hisa.OP_TOKEN_REFINE_TOPK, C.byref(q), C.byref(k), 128, 64, 2048, 0) == 0
    q2, k2 = _structs(T=32, s_max=131072, n_seq=32)
    assert lib.hisa_workspace_bytes(hisa.OP_TOKEN_REFINE_TOPK, C.byref(q2), C.byref(k2), 128, 64, 2048, 0) == 32 * 8192 * 4
    flat = lib.hisa_workspace_bytes(hisa.OP_FLAT_TOPK, C.byref(q), C.byref(k), 1, 0, 2048, 0)
    assert 8 * 65536 * 4 <= flat <= (9 << 29)


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(hisa, "_lib", None)
    monkeypatch.setattr(hisa, "LIB_PATH", "/nonexistent/libhisa.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        hisa.lib()


def test_the_header_is_valid_c_and_the_plain_c_example_links(tmp_path):
    """include/hisa.h is a C header: the example program is C11, compiled by gcc with warnings as
    errors, and links against the library and the HIP runtime (nothing is run here)."""
    import shutil
    import subprocess
    from paper_2603_28458_amd import build as B
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    if not os.path.exists(B.LIB_PATH):
        pytest.skip("library not built")
    out = str(tmp_path / "example_decode")
    res = subprocess.run(B.example_command(out), capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    assert os.path.exists(out)
