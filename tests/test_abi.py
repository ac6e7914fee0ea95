"""CPU-only checks of the boundary: the C-ABI library loads, exports every symbol the header
declares, and its host-side validation returns the documented codes without touching a GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2504_09285_amd as dsv
from paper_2504_09285_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "dsv_attn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return re.findall(r"^\s*(?:size_t|int|const char\*)\s+(\w+)\s*\(", text, flags=re.M)


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dsv.library_path()):
        from paper_2504_09285_amd import build
        build.build()
    return dsv.load_library()


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_struct_layouts_match_header():
    assert C.sizeof(binding._Pool) == 48
    assert binding.CHUNK_DTYPE.itemsize == 24
    assert binding.CHUNK_DTYPE.fields["chunk_offset"][1] == 16


def test_build_info(lib):
    assert "gfx950" in dsv.build_info()


def test_workspace_bytes_rejects_invalid_batches(lib):
    f = dsv.attn_mixed_batch_workspace_bytes
    assert f([0, 1, 3], [10, 20], 32, 8, 128) > 0
    assert f([0, 1, 3], [10, 1], 32, 8, 128) == 0         # ctx < q_len
    assert f([0, 1, 1], [10, 20], 32, 8, 128) == 0        # empty segment
    assert f([0, 1, 3], [10, 20], 32, 5, 128) == 0        # Hq % Hkv
    assert f([0, 1, 3], [10, 20], 32, 8, 96) == 0         # head_dim
    assert f([1, 2, 3], [10, 20], 32, 8, 128) == 0        # offsets must start at 0


def test_workspace_grows_with_split_work(lib):
    f = dsv.attn_mixed_batch_workspace_bytes
    small = f([0, 1], [100], 32, 8, 128)
    big = f([0, 1], [100000], 32, 8, 128)
    assert big > small > 0


def test_null_and_unsupported_arguments_return_codes_without_gpu(lib):
    pool = binding._Pool(0, 0, 0, 1, 4, 16, 8, 128)
    qo = np.array([0, 1], np.int32)
    cl = np.array([5], np.int32)
    p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    rc = lib.attn_mixed_batch(None, None, C.byref(pool), 0, None, 1, None, None, p(qo), p(cl), 1, 32,
                              0.1, 0, None, 0, None)
    assert rc == -1                                        # null pool bases
    pool = binding._Pool(4096, 4096, 0, 1, 4, 32, 8, 128)
    rc = lib.attn_mixed_batch(None, None, C.byref(pool), 0, None, 1, None, None, p(qo), p(cl), 1, 32,
                              0.1, 0, None, 0, None)
    assert rc == -2                                        # block_size != 16
    pool = binding._Pool(4096, 4096, 0, 1, 4, 16, 8, 80)
    assert lib.kv_pack_chunks(C.byref(pool), None, 1, None, None, 1, None, None) == -2
    pool = binding._Pool(4096, 4096, 0, 1, 4, 16, 8, 128)
    assert lib.kv_pack_chunks(C.byref(pool), None, 1, None, None, 1, None, None) == -1
    assert lib.kv_pack_chunks(C.byref(pool), None, 1, None, None, 0, None, None) == 0     # no-op
    assert lib.attn_mixed_batch(None, None, C.byref(pool), 0, None, 1, None, None, None, None, 0, 32,
                                0.1, 0, None, 0, None) == 0                               # no-op


def test_fp8kv_entry_points_check_scales_and_workspace_before_any_gpu_work(lib):
    pool = binding._Pool(4096, 4096, 0, 1, 4, 16, 8, 128)
    qo = np.array([0, 1], np.int32)
    cl = np.array([5], np.int32)
    p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    fake = 4096                                            # non-null, 16-byte aligned, never dereferenced
    call = lambda ks, vs, ws_bytes: lib.attn_mixed_batch_fp8kv(
        fake, fake, C.byref(pool), 0, fake, 1, fake, fake, p(qo), p(cl), 1, 32, 0.1, ks, vs, 0,
        fake * 4, ws_bytes, None)
    assert call(0.0, 1.0, 0) == -1
    assert call(1.0, float("inf"), 0) == -1
    assert call(float("nan"), 1.0, 0) == -1
    assert call(0.5, 0.5, 0) == -3                          # valid arguments, workspace too small
    assert lib.kv_append_fp8(fake, fake, C.byref(pool), 0, fake, 1, fake, fake, p(qo), p(cl), 1,
                             0.0, 1.0, None) == -1
    assert lib.kv_append_fp8(fake, fake, C.byref(pool), 0, fake, 1, fake, fake, p(qo), p(cl), 0,
                             1.0, 1.0, None) == 0           # empty batch: no-op
    f8 = dsv.attn_mixed_batch_fp8kv_workspace_bytes
    f16 = dsv.attn_mixed_batch_workspace_bytes
    assert f8([0, 1, 3], [10, 20], 32, 8, 128) == f16([0, 1, 3], [10, 20], 32, 8, 128)   # no span of 16+
    grow = f8([0, 64], [640], 32, 8, 128) - f16([0, 64], [640], 32, 8, 128)
    assert grow >= 640 * 4 * 8 * 128                        # the bf16 copy of the span's context
    assert lib.kv_pack_chunks_fp8(C.byref(pool), None, 1, None, None, 0, None, None) == 0
    assert lib.kv_pack_chunks_fp8(C.byref(pool), None, 1, None, None, 1, None, None) == -1


def test_workspace_holds_partials_when_query_tiles_are_cut(lib, monkeypatch):
    f = dsv.attn_mixed_batch_workspace_bytes
    monkeypatch.delenv("DSV_TILE_PART_TILES", raising=False)
    cut = f([0, 128], [20128], 32, 8, 128)              # 2 query tiles on 20,000 cached tokens: cut
    monkeypatch.setenv("DSV_TILE_PART_TILES", "-1")
    uncut = f([0, 128], [20128], 32, 8, 128)
    assert cut - uncut >= 128 * 2 * 32 * 128 * 4        # at least two partials per token and head
    monkeypatch.delenv("DSV_TILE_PART_TILES", raising=False)
    assert f([0, 2048], [2048], 32, 8, 128) == pytest.approx(f([0, 2048], [2048], 32, 8, 128))
    monkeypatch.setenv("DSV_TILE_PART_TILES", "-1")
    assert f([0, 2048] * 1, [2048], 32, 8, 128) > 0


def test_empty_batches_are_no_ops_on_every_attention_and_append_entry_point(lib):
    pool = binding._Pool(4096, 4096, 0, 1, 4, 16, 8, 128)
    assert lib.attn_mixed_batch(None, None, C.byref(pool), 0, None, 1, None, None, None, None, 0, 32,
                                0.1, 0, None, 0, None) == 0
    assert lib.attn_mixed_batch_fp8kv(None, None, C.byref(pool), 0, None, 1, None, None, None, None, 0, 32,
                                      0.1, 0.5, 0.5, 0, None, 0, None) == 0
    assert lib.kv_append(None, None, C.byref(pool), 0, None, 1, None, None, None, None, 0, None) == 0
    assert lib.kv_unpack_chunks_fp8(None, None, None, 0, C.byref(pool), None, 1, None) == 0
    assert dsv.attn_mixed_batch_workspace_bytes([0], [], 32, 8, 128) > 0      # lists only, no partials


def test_plan_entry_points_check_their_arguments_before_any_gpu_work(lib):
    """attn_mixed_batch_plan / *_planned: bad arguments and a plan record that does not match the
    call are refused on the host (nothing here reaches a launch, so no GPU is needed)."""
    pool = binding._Pool(4096, 4096, 0, 1, 4, 16, 8, 128)
    qo = np.array([0, 1], np.int32)
    cl = np.array([5], np.int32)
    p = lambda a: a.ctypes.data_as(C.POINTER(C.c_int32))
    fake = 4096                                            # non-null, aligned, never dereferenced
    plan = binding._Plan()
    f = lib.attn_mixed_batch_plan
    assert f(None, fake, 1, fake, fake, p(qo), p(cl), 1, 32, 8, 128, 2, fake, 1 << 30, None) == -1   # no plan record
    assert f(C.byref(plan), fake, 1, fake, fake, p(qo), p(cl), 1, 32, 8, 128, 3, fake, 1 << 30, None) == -1  # element size
    assert f(C.byref(plan), fake, 1, fake, fake, p(qo), p(cl), 1, 32, 8, 96, 2, fake, 1 << 30, None) == -2   # head_dim
    assert f(C.byref(plan), fake, 1, fake, fake, p(qo), p(cl), 1, 32, 8, 128, 2, None, 1 << 30, None) == -1  # no workspace
    assert f(C.byref(plan), fake, 1, fake, fake, p(qo), p(cl), 1, 32, 8, 128, 2, fake, 16, None) == -3       # too small
    assert f(C.byref(plan), None, 1, None, None, None, None, 0, 32, 8, 128, 2, None, 0, None) == 0           # empty batch
    need = dsv.attn_mixed_batch_workspace_bytes(qo, cl, 32, 8, 128)
    # a record that no plan call filled: the planned calls refuse it
    rc = lib.attn_mixed_batch_planned(C.byref(plan), fake, fake, C.byref(pool), 0, fake, 1, fake, fake, p(qo), p(cl),
                                      1, 32, 0.1, 0, fake, need, None)
    assert rc == -1
    rc = lib.attn_mixed_batch_fp8kv_planned(C.byref(plan), fake, fake, C.byref(pool), 0, fake, 1, fake, fake, p(qo),
                                            p(cl), 1, 32, 0.1, 0.5, 0.5, 0,
                                            fake, dsv.attn_mixed_batch_fp8kv_workspace_bytes(qo, cl, 32, 8, 128), None)
    assert rc == -1
    assert lib.attn_mixed_batch_planned(None, fake, fake, C.byref(pool), 0, fake, 1, fake, fake, p(qo), p(cl),
                                        1, 32, 0.1, 0, fake, need, None) == -1
    assert lib.attn_mixed_batch_planned(C.byref(plan), None, None, C.byref(pool), 0, None, 1, None, None, None, None,
                                        0, 32, 0.1, 0, None, 0, None) == 0                                   # empty batch


def test_loading_the_library_first_leaves_one_hip_runtime_in_the_process():
    """torch ships a HIP runtime of its own.  Whatever is imported first, the process must end up
    with a single libamdhip64 mapped: two runtimes do not know each other's allocations."""
    import subprocess
    import sys
    code = ("import paper_2504_09285_amd as dsv; dsv.load_library(); import torch; "
            "paths = {l.split()[-1] for l in open('/proc/self/maps') if 'libamdhip64' in l}; "
            "assert len(paths) == 1, paths; print('one runtime')")
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, cwd=ROOT)
    assert r.returncode == 0 and "one runtime" in r.stdout, r.stderr[-2000:]


def test_static_entry_point_refuses_oversized_and_invalid_batches_on_the_host(lib):
    """attn_mixed_batch_static checks the batch against its fixed array before any GPU call, so the
    refusal needs no GPU: too large -> DSV_E_WORKSPACE, invalid -> DSV_E_INVALID, empty -> no-op."""
    assert dsv.attn_mixed_batch_static_max_bytes() == 64 << 20
    pool = binding._Pool(0x1000, 0x2000, 0, 1, 4, 16, 8, 128)
    n = 4096
    qo = np.arange(n + 1, dtype=np.int32)
    cl = np.full(n, 4096, np.int32)
    i32p = C.POINTER(C.c_int32)

    def call(qo, cl, n, Hq=64):
        return lib.attn_mixed_batch_static(0x3000, 0x4000, C.byref(pool), 0, 0x5000, 4096, 0x6000, 0x7000,
                                           qo.ctypes.data_as(i32p), cl.ctypes.data_as(i32p), n, Hq, 0.1, 0, None)
    assert dsv.attn_mixed_batch_workspace_bytes(qo, cl, 64, 8, 128) > 64 << 20
    assert call(qo, cl, n) == -3
    assert call(qo, cl, 0) == 0
    assert call(qo, cl, n, Hq=60) == -1
    bad = cl.copy()
    bad[3] = 0
    assert call(qo, bad, n) == -1


def test_plan_info_says_how_a_batch_is_cut(lib, monkeypatch):
    """attn_mixed_batch_plan_info is host-only.  Long decode-only batches run as row streams (three
    quarters of the compute units; 256 are assumed where no device answers), small ones as items
    of a partition size; a batch with a prefill span reports its tile items; the knob forces
    streams; invalid batches are refused as by attn_mixed_batch."""
    for k in ("DSV_ROWS_STREAM", "DSV_PART_TOKENS", "DSV_MIXED_LAUNCH"):
        monkeypatch.delenv(k, raising=False)
    qo = np.arange(65, dtype=np.int32)
    cl = np.full(64, 40000, np.int32)
    big = dsv.attn_mixed_batch_plan_info(qo, cl, 32, 8, 128)
    assert big["row_streams"] > 0 and big["row_streams"] % 8 == 0 and big["part_tokens"] == 0
    assert big["rows"] == 64 and big["row_items"] == 64 + big["row_streams"] - 1 and big["tile_items"] == 0
    small = dsv.attn_mixed_batch_plan_info([0, 1, 2], [100, 200], 32, 8, 128)
    assert small["row_streams"] == 0 and small["part_tokens"] % 16 == 0 and small["rows"] == 2
    mixed = dsv.attn_mixed_batch_plan_info([0, 2048, 2049], [2048, 900], 32, 8, 128)
    assert mixed["tile_items"] >= 32 and mixed["rows"] == 1 and mixed["one_launch"] == 1 and mixed["tile_tokens"] == 64
    monkeypatch.setenv("DSV_ROWS_STREAM", "5")
    assert dsv.attn_mixed_batch_plan_info([0, 1, 2], [100, 200], 32, 8, 128)["row_streams"] == 5
    monkeypatch.setenv("DSV_ROWS_STREAM", "0")
    assert dsv.attn_mixed_batch_plan_info(qo, cl, 32, 8, 128)["row_streams"] == 0
    monkeypatch.delenv("DSV_ROWS_STREAM")
    with pytest.raises(dsv.DsvError):
        dsv.attn_mixed_batch_plan_info([0, 1], [0], 32, 8, 128)
    with pytest.raises(dsv.DsvError):
        dsv.attn_mixed_batch_plan_info([0, 1], [5], 32, 8, 96)
    assert dsv.attn_mixed_batch_plan_info([0, 1], [5], 32, 8, 128, kv_elem_bytes=1)["rows"] == 1
