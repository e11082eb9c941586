"""Host-side checks of the C-ABI library: it loads without a GPU, exports every
symbol the header declares, its pure host functions behave, and argument errors
are reported before any GPU work."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2603_08453_amd import binding as lc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(lc.LIB_PATH):
        from paper_2603_08453_amd import build
        build.build(verbose=False)
    return lc.lib()


def test_header_symbols_are_exported(L):
    hdr = open(os.path.join(ROOT, "include", "lychee.h")).read() + open(os.path.join(ROOT, "include", "lychee_bench.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(lc_[a-z_0-9]+)\s*\(", hdr))
    assert {"lc_build_index", "lc_retrieve", "lc_sparse_decode", "lc_append", "lc_decode_step", "lc_recluster",
            "lc_chunk_tokens"} <= names
    for n in sorted(names):
        assert hasattr(L, n), f"{n} declared in lychee.h but not exported"


def test_config_struct_matches_header(L):
    cfg = lc.lc_config_default()
    assert (cfg.levels, cfg.fanout, cfg.kmeans_iters) == (3, 16, 10)
    assert cfg.geometry == lc.LC_GEOMETRY_TOKEN_BALL and cfg.policy == lc.LC_POLICY_EXACT
    assert ctypes.sizeof(lc.LcConfig) == 4 * (5 + lc.LC_MAX_LEVELS + 6 + lc.LC_MAX_LEVELS)
    assert cfg.center_dtype == lc.LC_CENTER_F32
    hdr = open(os.path.join(ROOT, "include", "lychee.h")).read()
    assert f"#define LC_MAX_LEVELS {lc.LC_MAX_LEVELS}" in hdr
    assert f"#define LC_MAX_GROUP {lc.LC_MAX_GROUP}" in hdr


def test_size_queries(L):
    cfg = lc.lc_config_default(levels=4, fanout=16, max_chunks=4096, max_tokens=140000)
    n1 = lc.lc_index_bytes(cfg, 1, 8)
    n2 = lc.lc_index_bytes(cfg, 2, 8)
    assert n1 > 0 and n2 > n1 and n1 % 256 == 0
    # dominated by the float32 chunk centers: 4096 chunks x 128 x 4 B x 8 heads
    assert 4096 * 512 * 8 <= n1 <= 4096 * 512 * 8 * 1.25
    assert lc.lc_workspace_bytes(cfg, 1, 32, 8) > 0
    # bfloat16 chunk centers: half of that, the small upper levels stay float32
    half = lc.lc_config_default(levels=4, fanout=16, max_chunks=4096, max_tokens=140000, center_dtype=lc.LC_CENTER_BF16)
    nh = lc.lc_index_bytes(half, 1, 8)
    assert 4096 * 256 * 8 <= nh <= 4096 * 256 * 8 * 1.4 and nh < 0.62 * n1
    assert lc.lc_index_bytes(lc.lc_config_default(max_chunks=64, max_tokens=1024, center_dtype=2), 1, 8) == 0
    # fan-outs of their own per level: 4096 chunks -> 2048 fine clusters -> 94 coarse units
    tiers = lc.lc_config_default(levels=3, fanout=16, fanouts=[0, 2, 22], max_chunks=4096, max_tokens=140000)
    flat = lc.lc_config_default(levels=3, fanout=16, max_chunks=4096, max_tokens=140000)
    assert lc.lc_index_bytes(tiers, 1, 1) > lc.lc_index_bytes(flat, 1, 1) + 2048 * 512 - 256 * 512
    assert lc.lc_index_bytes(lc.lc_config_default(max_chunks=64, max_tokens=1024, fanouts=[0, -1]), 1, 8) == 0
    # invalid: d != 128, capacities unset, G too large, H_q not a multiple
    assert lc.lc_index_bytes(cfg, 1, 8, 64) == 0
    assert lc.lc_index_bytes(lc.lc_config_default(), 1, 8) == 0
    assert lc.lc_workspace_bytes(cfg, 1, 72, 8) == 0
    assert lc.lc_workspace_bytes(cfg, 1, 30, 8) == 0
    assert lc.lc_index_bytes(lc.lc_config_default(levels=7, max_chunks=10, max_tokens=10), 1, 1) == 0


def test_strerror(L):
    for code in (0, -1, -2, -3, -4, -5, -6):
        assert lc.lc_strerror(code) not in ("", "unknown error")
    assert lc.lc_strerror(-99) == "unknown error"


def test_argument_errors_before_any_gpu_work(L):
    cfg = lc.lc_config_default(levels=2, fanout=4, max_chunks=64, max_tokens=1024)
    out = ctypes.c_void_p()
    strides = (ctypes.c_int64 * 3)(8 * 1024 * 128, 1024 * 128, 128)
    seq = (ctypes.c_int32 * 1)(100)
    bounds = (ctypes.c_int32 * 3)(0, 40, 100)
    counts = (ctypes.c_int32 * 1)(2)
    fake = ctypes.c_void_p(0x10000)           # never dereferenced: every call below fails validation first
    call = lambda **kw: L.lc_build_index(
        ctypes.byref(out), ctypes.byref(kw.get("cfg", cfg)), kw.get("K", fake), kw.get("strides", strides), seq,
        kw.get("bounds", bounds), kw.get("counts", counts), 1, 8, kw.get("d", 128), fake, kw.get("ib", 1 << 30),
        fake, kw.get("wb", 1 << 30), None)
    assert call(K=None) == lc.LC_ERR_INVALID_ARG
    assert call(d=64) == lc.LC_ERR_BAD_SHAPE
    assert call(strides=(ctypes.c_int64 * 3)(1024 * 128, 128 * 1024, 100)) == lc.LC_ERR_BAD_SHAPE
    assert call(bounds=(ctypes.c_int32 * 3)(0, 40, 30)) == lc.LC_ERR_INVALID_ARG       # not ascending
    assert call(bounds=(ctypes.c_int32 * 3)(0, 40, 101)) == lc.LC_ERR_INVALID_ARG      # past the sequence
    assert call(counts=(ctypes.c_int32 * 1)(65)) == lc.LC_ERR_CAPACITY
    assert call(ib=1024) == lc.LC_ERR_WORKSPACE_TOO_SMALL
    assert call(wb=1024) == lc.LC_ERR_WORKSPACE_TOO_SMALL
    bad = lc.lc_config_default(levels=0, max_chunks=64, max_tokens=1024)
    assert call(cfg=bad) == lc.LC_ERR_INVALID_ARG
    assert out.value is None
    # calls on a null handle
    assert L.lc_retrieve(None, fake, 32, 10, fake, fake, None, 16, fake, 1 << 20, None) == lc.LC_ERR_INVALID_ARG
    assert L.lc_sparse_decode(None, fake, fake, fake, strides, fake, fake, 16, 32, fake, None, fake, 1 << 20,
                              None) == lc.LC_ERR_INVALID_ARG
    assert L.lc_decode_step(None, fake, fake, fake, strides, 32, 10, fake, None, None, None, 0, fake, 1 << 20,
                            None) == lc.LC_ERR_INVALID_ARG
    assert L.lc_recluster(None, fake, 1 << 20, None) == lc.LC_ERR_INVALID_ARG
    four = (ctypes.c_float * 4)()
    assert L.lc_index_drift(None, 1, four, fake, 1 << 20, None) == lc.LC_ERR_INVALID_ARG
    assert L.lc_bench_select_attend(None, fake, fake, fake, strides, 8, 16, fake, None, fake, 1 << 20, None) == lc.LC_ERR_INVALID_ARG
    assert L.lc_bench_read_sweep(None, 1 << 20, fake, 2048, None) == lc.LC_ERR_INVALID_ARG
    assert L.lc_bench_read_sweep(fake, 100, fake, 2048, None) == lc.LC_ERR_INVALID_ARG          # not a multiple of 16
    assert L.lc_bench_read_sweep(ctypes.c_void_p(0x10008), 1 << 20, fake, 2048, None) == lc.LC_ERR_INVALID_ARG
    assert L.lc_bench_read_sweep(fake, 1 << 20, fake, 100, None) == lc.LC_ERR_WORKSPACE_TOO_SMALL
    assert L.lc_append(None, fake, fake, strides, fake, fake, None, fake, 0, None) == lc.LC_ERR_INVALID_ARG
    assert L.lc_set_policy(None, 0, None, 0) == lc.LC_ERR_INVALID_ARG
    assert L.lc_index_info(None, 0, None, None, None) == lc.LC_ERR_INVALID_ARG
    # import: malformed blobs are rejected on the host
    blob = bytes(64)
    assert L.lc_index_import(ctypes.byref(out), ctypes.byref(cfg), blob, 64, fake, 1 << 30, None) == lc.LC_ERR_BAD_BLOB
    assert L.lc_index_import(ctypes.byref(out), ctypes.byref(cfg), blob, 10, fake, 1 << 30, None) == lc.LC_ERR_BAD_BLOB
    L.lc_index_destroy(None)


def test_blob_roundtrip_python_side():
    r = np.random.default_rng(0)
    d, L_, F = 128, 2, 4
    seqs = []
    for M in (5, 3):
        n1 = -(-M // F)
        bounds = np.concatenate([[0], np.cumsum(r.integers(1, 9, size=M))]).astype(np.int32)
        heads = []
        for _ in range(2):
            lv = []
            for n in (M, n1):
                lv.append(dict(center=r.standard_normal((n, d)).astype(np.float32),
                               radius=r.random(n).astype(np.float32),
                               parent=r.integers(0, n1, size=n).astype(np.int32),
                               ntok=r.integers(1, 9, size=n).astype(np.int32),
                               nchunk=np.ones(n, dtype=np.int32)))
            heads.append(lv)
        seqs.append(dict(T=int(bounds[-1]) + 2, bounds=bounds, heads=heads))
    blob = lc.pack_blob(2, 2, d, L_, F, 0, seqs)
    back = lc.unpack_blob(blob)
    assert back["B"] == 2 and back["L"] == 2
    for s, t in zip(seqs, back["seqs"]):
        assert s["T"] == t["T"] and np.array_equal(s["bounds"], t["bounds"])
        for hs, ht in zip(s["heads"], t["heads"]):
            for a, b in zip(hs, ht):
                for k in a:
                    assert np.array_equal(a[k], b[k])


def test_build_reports_and_rejects_register_spills():
    """The build parses the compiler's per-kernel resource remarks; a kernel with scratch memory
    (spilled registers) must make it fail."""
    from paper_2603_08453_amd import build as B
    remarks = """\
a.hip:5:1: remark: Function Name: _Z3fooPf [-Rpass-analysis=kernel-resource-usage]
    5 | foo(float* p) {
      | ^
a.hip:5:1: remark:     VGPRs: 26 [-Rpass-analysis=kernel-resource-usage]
a.hip:5:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
a.hip:9:1: remark: Function Name: _Z3barPf [-Rpass-analysis=kernel-resource-usage]
a.hip:9:1: remark:     VGPRs: 128 [-Rpass-analysis=kernel-resource-usage]
a.hip:9:1: remark:     ScratchSize [bytes/lane]: 56 [-Rpass-analysis=kernel-resource-usage]
"""
    k = B.kernel_resources(remarks)
    assert k == {"_Z3fooPf": {"vgprs": 26, "scratch": 0}, "_Z3barPf": {"vgprs": 128, "scratch": 56}}
