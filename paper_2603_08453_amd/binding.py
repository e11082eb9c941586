"""ctypes binding of liblychee.so: same names as the C ABI, argument marshalling only.

PyTorch provides device memory and streams; every step of the path runs inside
the library's HIP kernels.  There is no CPU fallback: if the shared library has
not been built, importing the symbols raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

LC_MAX_LEVELS = 6
LC_MAX_GROUP = 8
LC_HEAD_DIM = 128

LC_OK = 0
LC_ERR_INVALID_ARG = -1
LC_ERR_BAD_SHAPE = -2
LC_ERR_WORKSPACE_TOO_SMALL = -3
LC_ERR_CAPACITY = -4
LC_ERR_HIP = -5
LC_ERR_BAD_BLOB = -6

LC_GEOMETRY_TOKEN_BALL = 0
LC_GEOMETRY_PAPER_UNIT = 1
LC_POLICY_EXACT = 0
LC_POLICY_BEAM = 1
LC_PRUNE_AUTO = 0
LC_PRUNE_ALWAYS = 1
LC_PRUNE_NEVER = 2
LC_CENTER_F32 = 0
LC_CENTER_BF16 = 1

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("LYCHEE_LIB", os.path.join(_HERE, "liblychee.so"))


class LcConfig(ctypes.Structure):
    _fields_ = [
        ("levels", ctypes.c_int32),
        ("fanout", ctypes.c_int32),
        ("kmeans_iters", ctypes.c_int32),
        ("geometry", ctypes.c_int32),
        ("policy", ctypes.c_int32),
        ("beam", ctypes.c_int32 * LC_MAX_LEVELS),
        ("sink_tokens", ctypes.c_int32),
        ("max_chunks", ctypes.c_int32),
        ("max_tokens", ctypes.c_int32),
        ("decode_splits", ctypes.c_int32),
        ("prune", ctypes.c_int32),
        ("center_dtype", ctypes.c_int32),
        ("fanouts", ctypes.c_int32 * LC_MAX_LEVELS),
    ]


class LycheeError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = lib().lc_strerror(code).decode()
        if code == LC_ERR_HIP:
            msg += ": " + lib().lc_last_hip_error().decode()
        super().__init__(f"{where}: {msg} ({code})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it first (python -m paper_2603_08453_amd.build)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32p, u8p, f32p = ctypes.c_void_p, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_uint8), ctypes.c_void_p
    i64p = ctypes.POINTER(ctypes.c_int64)
    cfgp = ctypes.POINTER(LcConfig)
    L.lc_config_default.argtypes = [cfgp]
    L.lc_config_default.restype = None
    L.lc_strerror.argtypes = [ctypes.c_int]
    L.lc_strerror.restype = ctypes.c_char_p
    L.lc_last_hip_error.argtypes = []
    L.lc_last_hip_error.restype = ctypes.c_char_p
    L.lc_index_bytes.argtypes = [cfgp, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    L.lc_index_bytes.restype = ctypes.c_size_t
    L.lc_workspace_bytes.argtypes = [cfgp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    L.lc_workspace_bytes.restype = ctypes.c_size_t
    L.lc_build_index.argtypes = [ctypes.POINTER(vp), cfgp, vp, i64p, i32p, i32p, i32p,
                                 ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
    L.lc_build_index.restype = ctypes.c_int
    L.lc_set_policy.argtypes = [vp, ctypes.c_int, i32p, ctypes.c_int]
    L.lc_set_policy.restype = ctypes.c_int
    L.lc_set_prune.argtypes = [vp, ctypes.c_int]
    L.lc_set_prune.restype = ctypes.c_int
    L.lc_retrieve.argtypes = [vp, vp, ctypes.c_int, ctypes.c_int, vp, vp, f32p, ctypes.c_int, vp, ctypes.c_size_t, vp]
    L.lc_retrieve.restype = ctypes.c_int
    L.lc_sparse_decode.argtypes = [vp, vp, vp, vp, i64p, vp, vp, ctypes.c_int, ctypes.c_int, vp, vp,
                                   vp, ctypes.c_size_t, vp]
    L.lc_sparse_decode.restype = ctypes.c_int
    L.lc_decode_step.argtypes = [vp, vp, vp, vp, i64p, ctypes.c_int, ctypes.c_int, vp, vp, vp, vp, ctypes.c_int,
                                 vp, ctypes.c_size_t, vp]
    L.lc_decode_step.restype = ctypes.c_int
    L.lc_decode_step_static.argtypes = [vp, vp, vp, vp, i64p, ctypes.c_int, ctypes.c_int, vp, vp, vp, vp, ctypes.c_int, vp]
    L.lc_decode_step_static.restype = ctypes.c_int
    L.lc_decode_workspace_bytes.argtypes = [cfgp, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int]
    L.lc_decode_workspace_bytes.restype = ctypes.c_size_t
    L.lc_static_workspace_bytes.argtypes = []
    L.lc_static_workspace_bytes.restype = ctypes.c_size_t
    L.lc_index_drift.argtypes = [vp, ctypes.c_int, ctypes.POINTER(ctypes.c_float), vp, ctypes.c_size_t, vp]
    L.lc_index_drift.restype = ctypes.c_int
    L.lc_walk_limits.argtypes = [i32p, i32p]
    L.lc_walk_limits.restype = None
    L.lc_recluster.argtypes = [vp, vp, ctypes.c_size_t, vp]
    L.lc_recluster.restype = ctypes.c_int
    # measurement aids (lychee_bench.h)
    L.lc_bench_select_attend.argtypes = [vp, vp, vp, vp, i64p, ctypes.c_int, ctypes.c_int, vp, vp,
                                         vp, ctypes.c_size_t, vp]
    L.lc_bench_select_attend.restype = ctypes.c_int
    L.lc_bench_read_sweep.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
    L.lc_bench_read_sweep.restype = ctypes.c_int
    L.lc_append.argtypes = [vp, vp, vp, i64p, vp, vp, u8p, vp, ctypes.c_size_t, vp]
    L.lc_append.restype = ctypes.c_int
    L.lc_index_info.argtypes = [vp, ctypes.c_int, i32p, i32p, i32p]
    L.lc_index_info.restype = ctypes.c_int
    L.lc_index_export.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_size_t), vp]
    L.lc_index_export.restype = ctypes.c_int
    L.lc_index_import.argtypes = [ctypes.POINTER(vp), cfgp, vp, ctypes.c_size_t, vp, ctypes.c_size_t, vp]
    L.lc_index_import.restype = ctypes.c_int
    L.lc_index_destroy.argtypes = [vp]
    L.lc_index_destroy.restype = None
    L.lc_chunk_tokens.argtypes = [ctypes.c_char_p, i64p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                  i32p, ctypes.c_int, ctypes.POINTER(ctypes.c_int)]
    L.lc_chunk_tokens.restype = ctypes.c_int
    _lib = L
    return L


# ------------------------------------------------------------------ helpers

def _check(rc: int, where: str) -> None:
    if rc != LC_OK:
        raise LycheeError(rc, where)


def _ptr(t) -> Optional[int]:
    """Device (or host) address of a torch tensor; None passes NULL."""
    return None if t is None else int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return int(stream.cuda_stream) or None


def _strides3(t) -> "ctypes.Array":
    assert t.dim() == 4 and t.stride(3) == 1, "cache must be [B][H_kv][tokens][d] with d contiguous"
    return (ctypes.c_int64 * 3)(t.stride(0), t.stride(1), t.stride(2))


def _i32(a):
    """Host int32 array for a C `const int32_t*` argument (the numpy array owns the memory for the call)."""
    arr = np.array(a, dtype=np.int32).reshape(-1)          # a private, writable, contiguous copy
    if arr.size == 0:
        arr = np.zeros(1, dtype=np.int32)
    return (ctypes.c_int32 * arr.size).from_buffer(arr)    # keeps `arr` alive


def lc_config_default(**overrides) -> LcConfig:
    cfg = LcConfig()
    lib().lc_config_default(ctypes.byref(cfg))
    for k, v in overrides.items():
        if k in ("beam", "fanouts"):
            arr = getattr(cfg, k)
            for i in range(LC_MAX_LEVELS):
                arr[i] = int(v[i]) if i < len(v) else 0
        else:
            setattr(cfg, k, int(v))
    return cfg


def lc_strerror(code: int) -> str:
    return lib().lc_strerror(code).decode()


def lc_index_bytes(cfg: LcConfig, B: int, H_kv: int, d: int = LC_HEAD_DIM) -> int:
    return int(lib().lc_index_bytes(ctypes.byref(cfg), B, H_kv, d))


def lc_workspace_bytes(cfg: LcConfig, B: int, H_q: int, H_kv: int, d: int = LC_HEAD_DIM) -> int:
    return int(lib().lc_workspace_bytes(ctypes.byref(cfg), B, H_q, H_kv, d))


class Index:
    """Owns an lc_index handle and keeps the caller-provided index buffer alive."""

    def __init__(self, handle: int, cfg: LcConfig, index_buf, B: int, H_kv: int):
        self.handle = ctypes.c_void_p(handle)
        self.cfg = cfg
        self.index_buf = index_buf
        self.B = B
        self.H_kv = H_kv

    def info(self, b: int):
        T, M = ctypes.c_int32(), ctypes.c_int32()
        n = (ctypes.c_int32 * LC_MAX_LEVELS)()
        _check(lib().lc_index_info(self.handle, b, ctypes.byref(T), ctypes.byref(M), n), "lc_index_info")
        return int(T.value), int(M.value), [int(x) for x in n][: self.cfg.levels]

    def close(self):
        if self.handle:
            lib().lc_index_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def lc_build_index(cfg: LcConfig, K, seq_lens: Sequence[int], chunk_bounds: Sequence[Sequence[int]],
                   index_buf, ws, stream=None) -> Index:
    """K: torch bf16 [B][H_kv][tokens][d] on the GPU; chunk_bounds: per sequence, host ints."""
    B, H_kv, _, d = K.shape
    counts = [len(b) - 1 for b in chunk_bounds]
    flat = np.concatenate([np.asarray(b, dtype=np.int32).reshape(-1) for b in chunk_bounds])
    out = ctypes.c_void_p()
    rc = lib().lc_build_index(ctypes.byref(out), ctypes.byref(cfg), _ptr(K), _strides3(K), _i32(seq_lens),
                              _i32(flat), _i32(counts), B, H_kv, d, _ptr(index_buf),
                              index_buf.numel() * index_buf.element_size(), _ptr(ws),
                              ws.numel() * ws.element_size(), _stream(stream))
    _check(rc, "lc_build_index")
    return Index(out.value, cfg, index_buf, B, H_kv)


def lc_set_policy(idx: Index, policy: int, beam: Optional[Sequence[int]] = None, sink_tokens: int = 0) -> None:
    arr = None
    if beam is not None:
        arr = _i32(list(beam) + [0] * (LC_MAX_LEVELS - len(beam)))
    _check(lib().lc_set_policy(idx.handle, policy, arr, sink_tokens), "lc_set_policy")


def lc_set_prune(idx: Index, prune: int) -> None:
    _check(lib().lc_set_prune(idx.handle, prune), "lc_set_prune")


def lc_retrieve(idx: Index, q, budget: int, chunk_ids, counts, ws, scores=None, stream=None) -> None:
    """q bf16 [B][H_q][d]; chunk_ids int32 [B][H_kv][cap]; counts int32 [B][H_kv]."""
    H_q = q.shape[1]
    cap = chunk_ids.shape[2]
    rc = lib().lc_retrieve(idx.handle, _ptr(q), H_q, budget, _ptr(chunk_ids), _ptr(counts), _ptr(scores), cap,
                           _ptr(ws), ws.numel() * ws.element_size(), _stream(stream))
    _check(rc, "lc_retrieve")


def lc_sparse_decode(idx: Index, q, K, V, chunk_ids, counts, out, ws, lse=None, stream=None) -> None:
    """out float32 [B][H_q][d]; lse float32 [B][H_q] or None."""
    H_q = q.shape[1]
    cap = chunk_ids.shape[2]
    assert K.stride() == V.stride()
    rc = lib().lc_sparse_decode(idx.handle, _ptr(q), _ptr(K), _ptr(V), _strides3(K), _ptr(chunk_ids), _ptr(counts),
                                cap, H_q, _ptr(out), _ptr(lse), _ptr(ws), ws.numel() * ws.element_size(),
                                _stream(stream))
    _check(rc, "lc_sparse_decode")


def lc_index_drift(idx: Index, level: int, ws, stream=None) -> np.ndarray:
    """[B][H_kv][4] floats: sum of the level's radii at build, sum now, largest growth, nodes counted."""
    out = (ctypes.c_float * (idx.B * idx.H_kv * 4))()
    _check(lib().lc_index_drift(idx.handle, int(level), out, _ptr(ws), ws.numel() * ws.element_size(),
                                _stream(stream)), "lc_index_drift")
    return np.frombuffer(out, dtype=np.float32).reshape(idx.B, idx.H_kv, 4).copy()


def lc_walk_limits():
    """(internal nodes the exact walk holds, nodes of one level under top-k per level)."""
    a, b = ctypes.c_int32(), ctypes.c_int32()
    lib().lc_walk_limits(ctypes.byref(a), ctypes.byref(b))
    return int(a.value), int(b.value)


def lc_recluster(idx: Index, ws, stream=None) -> None:
    _check(lib().lc_recluster(idx.handle, _ptr(ws), ws.numel() * ws.element_size(), _stream(stream)), "lc_recluster")


def lc_bench_select_attend(idx: Index, q, K, V, budget: int, out, ws, lse=None, stream=None) -> None:
    """Measurement aid: the select+attend kernel of lc_decode_step alone, on the score keys that the
    previous lc_decode_step with the same query, index, budget and workspace left in `ws`."""
    assert K.shape == V.shape and K.stride() == V.stride()
    _check(lib().lc_bench_select_attend(idx.handle, _ptr(q), _ptr(K), _ptr(V), _strides3(K), int(q.shape[1]),
                                        int(budget), _ptr(out), _ptr(lse), _ptr(ws),
                                        ws.numel() * ws.element_size(), _stream(stream)), "lc_bench_select_attend")


def lc_bench_read_sweep(src, sink, stream=None) -> None:
    """Measurement aid: reads the device tensor `src` once; `sink` is an int32 device tensor of >= 2048 words."""
    _check(lib().lc_bench_read_sweep(_ptr(src), src.numel() * src.element_size(), _ptr(sink), sink.numel(),
                                     _stream(stream)), "lc_bench_read_sweep")


def lc_decode_step(idx: Index, q, K, V, budget: int, out, ws, lse=None, chunk_ids=None, counts=None,
                   stream=None) -> None:
    """q bf16 [B][H_q][d]; out f32 [B][H_q][d]; optional chunk_ids int32 [B][H_kv][cap] + counts."""
    assert K.shape == V.shape and K.stride() == V.stride()
    H_q = int(q.shape[1])
    cap = int(chunk_ids.shape[-1]) if chunk_ids is not None else 0
    _check(lib().lc_decode_step(idx.handle, _ptr(q), _ptr(K), _ptr(V), _strides3(K), H_q, int(budget), _ptr(out),
                                _ptr(lse), _ptr(chunk_ids), _ptr(counts), cap, _ptr(ws),
                                ws.numel() * ws.element_size(), _stream(stream)), "lc_decode_step")


def lc_decode_step_static(idx: Index, q, K, V, budget: int, out, lse=None, chunk_ids=None, counts=None,
                          stream=None) -> None:
    """lc_decode_step on the library's own static scratch array (no workspace argument)."""
    assert K.shape == V.shape and K.stride() == V.stride()
    H_q = int(q.shape[1])
    cap = int(chunk_ids.shape[-1]) if chunk_ids is not None else 0
    _check(lib().lc_decode_step_static(idx.handle, _ptr(q), _ptr(K), _ptr(V), _strides3(K), H_q, int(budget),
                                       _ptr(out), _ptr(lse), _ptr(chunk_ids), _ptr(counts), cap,
                                       _stream(stream)), "lc_decode_step_static")


def lc_decode_workspace_bytes(cfg: LcConfig, B: int, H_q: int, H_kv: int, d: int = LC_HEAD_DIM) -> int:
    return int(lib().lc_decode_workspace_bytes(ctypes.byref(cfg), B, H_q, H_kv, d))


def lc_static_workspace_bytes() -> int:
    return int(lib().lc_static_workspace_bytes())


def lc_append(idx: Index, K, V, k_new, v_new, close_chunk: Optional[Sequence[int]], ws, stream=None) -> None:
    """k_new, v_new bf16 [B][H_kv][d]; close_chunk: host flags per sequence (or None)."""
    cc = None
    if close_chunk is not None:
        cc = (ctypes.c_uint8 * len(close_chunk))(*[1 if c else 0 for c in close_chunk])
    assert K.stride() == V.stride()
    rc = lib().lc_append(idx.handle, _ptr(K), _ptr(V), _strides3(K), _ptr(k_new), _ptr(v_new), cc,
                         _ptr(ws), ws.numel() * ws.element_size(), _stream(stream))
    _check(rc, "lc_append")


def lc_index_export(idx: Index, stream=None) -> bytes:
    n = ctypes.c_size_t(0)
    _check(lib().lc_index_export(idx.handle, None, ctypes.byref(n), _stream(stream)), "lc_index_export(size)")
    buf = ctypes.create_string_buffer(n.value)
    _check(lib().lc_index_export(idx.handle, buf, ctypes.byref(n), _stream(stream)), "lc_index_export")
    return buf.raw[: n.value]


def lc_index_import(cfg: LcConfig, blob: bytes, index_buf, stream=None) -> Index:
    out = ctypes.c_void_p()
    rc = lib().lc_index_import(ctypes.byref(out), ctypes.byref(cfg), blob, len(blob), _ptr(index_buf),
                               index_buf.numel() * index_buf.element_size(), _stream(stream))
    _check(rc, "lc_index_import")
    hdr = np.frombuffer(blob[:64], dtype=np.int32)
    return Index(out.value, cfg, index_buf, int(hdr[2]), int(hdr[3]))


def lc_chunk_tokens(tokens: Sequence[str], min_len: int, max_len: int) -> List[int]:
    """Chunk boundaries of a token stream given as the tokens' texts (host routine)."""
    raw = [t.encode("utf-8") for t in tokens]
    n = len(raw)
    off = (ctypes.c_int64 * (n + 1))()
    acc = 0
    for i, r in enumerate(raw):
        off[i] = acc
        acc += len(r)
    off[n] = acc
    bounds = (ctypes.c_int32 * (n + 1))()
    m = ctypes.c_int(0)
    _check(lib().lc_chunk_tokens(b"".join(raw), off, n, int(min_len), int(max_len), bounds, n + 1,
                                 ctypes.byref(m)), "lc_chunk_tokens")
    return [int(bounds[i]) for i in range(m.value + 1)]


# ------------------------------------------------------------------ blob (de)serialisation
# The flat format documented in lychee.h; pure data marshalling.

_MAGIC = 0x5849434C


def pack_blob(B: int, H_kv: int, d: int, L: int, F: int, geometry: int, seqs: List[Dict],
              center_dtype: int = LC_CENTER_F32, fanouts: Optional[Sequence[int]] = None) -> bytes:
    """seqs[b] = {"T": int, "bounds": int array [M+1],
                  "heads": [ per head: [ per level: dict(center, radius, parent, ntok, nchunk) ] ]}"""
    hdr = np.zeros(16, dtype=np.int32)
    hdr[:9] = [_MAGIC, 1, B, H_kv, d, L, F, geometry, center_dtype]
    for l in range(1, LC_MAX_LEVELS):
        hdr[8 + l] = int(fanouts[l]) if fanouts is not None and l < len(fanouts) else 0
    parts = [hdr.tobytes()]
    for s in seqs:
        M = len(s["bounds"]) - 1
        levels0 = s["heads"][0]
        rec = [int(s["T"]), M] + [len(levels0[l]["radius"]) for l in range(1, L)]
        parts.append(np.asarray(rec, dtype=np.int32).tobytes())
        parts.append(np.asarray(s["bounds"], dtype=np.int32).tobytes())
    for s in seqs:
        for head in s["heads"]:
            for l in range(L):
                lv = head[l]
                parts.append(np.ascontiguousarray(lv["center"], dtype=np.float32).tobytes())
                parts.append(np.ascontiguousarray(lv["radius"], dtype=np.float32).tobytes())
                parts.append(np.ascontiguousarray(lv["parent"], dtype=np.int32).tobytes())
                parts.append(np.ascontiguousarray(lv["ntok"], dtype=np.int32).tobytes())
                parts.append(np.ascontiguousarray(lv["nchunk"], dtype=np.int32).tobytes())
    return b"".join(parts)


def unpack_blob(blob: bytes) -> Dict:
    hdr = np.frombuffer(blob, dtype=np.int32, count=16)
    assert hdr[0] == _MAGIC and hdr[1] == 1
    B, H_kv, d, L, F, geometry = (int(x) for x in hdr[2:8])
    off = 64
    seqs = []
    for _ in range(B):
        rec = np.frombuffer(blob, dtype=np.int32, count=2 + (L - 1), offset=off)
        off += rec.nbytes
        T, M = int(rec[0]), int(rec[1])
        N = [M] + [int(x) for x in rec[2:]]
        bounds = np.frombuffer(blob, dtype=np.int32, count=M + 1, offset=off).copy()
        off += bounds.nbytes
        seqs.append({"T": T, "bounds": bounds, "N": N, "heads": []})
    for s in seqs:
        for _h in range(H_kv):
            levels = []
            for l in range(L):
                n = s["N"][l]
                lv = {}
                lv["center"] = np.frombuffer(blob, dtype=np.float32, count=n * d, offset=off).reshape(n, d).copy()
                off += n * d * 4
                for name, dt in (("radius", np.float32), ("parent", np.int32), ("ntok", np.int32), ("nchunk", np.int32)):
                    lv[name] = np.frombuffer(blob, dtype=dt, count=n, offset=off).copy()
                    off += n * 4
                levels.append(lv)
            s["heads"].append(levels)
    assert off == len(blob), (off, len(blob))
    return {"B": B, "H_kv": H_kv, "d": d, "L": L, "F": F, "geometry": geometry, "center_dtype": int(hdr[8]),
            "fanouts": [0] + [int(x) for x in hdr[9:9 + LC_MAX_LEVELS - 1]], "seqs": seqs}
