"""ctypes binding of libattncache.so: argument marshalling only.

Every function mirrors one C entry point of ``include/attncache.h`` under the
same name.  Tensors are torch CUDA tensors (PyTorch supplies device memory and
streams, nothing else); this layer checks device / dtype / shape / contiguity
so that no malformed pointer can reach a kernel, then passes ``data_ptr()`` and
the current stream.  There is no CPU fallback: without the built library, or
without a GPU tensor, the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

from . import build as _build

AC_F32, AC_F16, AC_BF16 = 0, 1, 2
AC_IP, AC_L2 = 0, 1
AC_LAYOUT_DENSE, AC_LAYOUT_PACKED = 0, 1
AC_MAX_K = 64

_DTYPE_CODE = {torch.float32: AC_F32, torch.float16: AC_F16, torch.bfloat16: AC_BF16}

SYMBOLS = ["attncache_workspace_bytes", "attncache_map_entry_bytes", "attncache_pack_maps",
           "attncache_build_db", "attncache_destroy_db",
           "attncache_search", "attncache_search_static", "attncache_apply", "attention_exact", "attncache_insert",
           "attncache_cache_stats", "attncache_cache_reset",
           "attncache_project_workspace_bytes", "attncache_project", "attncache_status_string",
           "attncache_last_hip_error", "attncache_version", "attncache_set_pointer_checks"]


class AttnCacheError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().attncache_status_string(status).decode()
        hip = lib().attncache_last_hip_error() if status == -8 else 0
        super().__init__(f"{where}: status {status} ({msg})" + (f", hipError {hip}" if hip else ""))


class DbDesc(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "n_emb", "emb_dim", "emb_dtype", "metric", "n_entries", "n_layers", "n_q_heads",
        "n_kv_heads", "head_dim", "seq_len", "map_dtype", "causal", "maps_on_host", "map_layout")]


_lib = None


def lib_path() -> str:
    return _build.LIB


def lib():
    """Load libattncache.so (it must have been built: see build.py / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build the HIP library first "
                               "(python -m paper_2510_25979_amd.build)")
        L = ctypes.CDLL(path)
        i32, f32, vp, sz = ctypes.c_int32, ctypes.c_float, ctypes.c_void_p, ctypes.c_size_t
        L.attncache_workspace_bytes.restype = i32
        L.attncache_workspace_bytes.argtypes = [ctypes.POINTER(DbDesc), i32, i32, ctypes.POINTER(sz)]
        L.attncache_map_entry_bytes.restype = i32
        L.attncache_map_entry_bytes.argtypes = [ctypes.POINTER(DbDesc), ctypes.POINTER(sz)]
        L.attncache_pack_maps.restype = i32
        L.attncache_pack_maps.argtypes = [ctypes.POINTER(DbDesc), vp, i32, vp, vp]
        L.attncache_build_db.restype = i32
        L.attncache_build_db.argtypes = [ctypes.POINTER(DbDesc), vp, vp, vp, vp, sz, vp,
                                         ctypes.POINTER(vp)]
        L.attncache_destroy_db.restype = i32
        L.attncache_destroy_db.argtypes = [vp]
        L.attncache_search.restype = i32
        L.attncache_search.argtypes = [vp, vp, i32, i32, f32, vp, vp, vp, vp, sz, vp]
        L.attncache_search_static.restype = i32
        L.attncache_search_static.argtypes = [vp, vp, i32, i32, f32, vp, vp, vp, vp]
        L.attncache_apply.restype = i32
        L.attncache_apply.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp]
        L.attention_exact.restype = i32
        L.attention_exact.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, i32, i32, f32, vp]
        L.attncache_insert.restype = i32
        L.attncache_insert.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, f32, vp]
        L.attncache_cache_stats.restype = i32
        L.attncache_cache_stats.argtypes = [vp, ctypes.POINTER(ctypes.c_uint64), ctypes.POINTER(ctypes.c_uint64)]
        L.attncache_cache_reset.restype = i32
        L.attncache_cache_reset.argtypes = [vp]
        L.attncache_project_workspace_bytes.restype = sz
        L.attncache_project_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.attncache_project.restype = i32
        L.attncache_project.argtypes = [vp] * 7 + [i32] * 8 + [vp, sz, vp]
        L.attncache_status_string.restype = ctypes.c_char_p
        L.attncache_status_string.argtypes = [i32]
        L.attncache_last_hip_error.restype = i32
        L.attncache_last_hip_error.argtypes = []
        L.attncache_set_pointer_checks.restype = i32
        L.attncache_set_pointer_checks.argtypes = [i32]
        L.attncache_version.restype = i32
        L.attncache_version.argtypes = []
        _lib = L
    return _lib


def _check(status: int, where: str):
    if status != 0:
        raise AttnCacheError(status, where)


def _dev(t: torch.Tensor, name: str, dtype=None, shape=None) -> int:
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise ValueError(f"{name} must be a CUDA tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, has {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, has {tuple(t.shape)}")
    return t.data_ptr()


def _stream(stream: Optional[torch.cuda.Stream]) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


class Database:
    """Owner of an ``attncache_db`` handle; keeps the borrowed tensors alive."""

    def __init__(self, handle, desc: DbDesc, keep):
        self.handle = handle
        self.desc = desc
        self._keep = keep

    def close(self):
        if self.handle:
            _check(lib().attncache_destroy_db(self.handle), "attncache_destroy_db")
            self.handle = None
            self._keep = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def attncache_set_pointer_checks(on: bool) -> bool:
    """Per-call memory-space checks on/off; returns the previous setting."""
    return bool(lib().attncache_set_pointer_checks(int(bool(on))))


def attncache_workspace_bytes(desc: DbDesc, max_batch: int, k: int) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().attncache_workspace_bytes(ctypes.byref(desc), max_batch, k, ctypes.byref(out)),
           "attncache_workspace_bytes")
    return int(out.value)


def attncache_map_entry_bytes(desc: DbDesc) -> int:
    out = ctypes.c_size_t(0)
    _check(lib().attncache_map_entry_bytes(ctypes.byref(desc), ctypes.byref(out)),
           "attncache_map_entry_bytes")
    return int(out.value)


def packed_tile_elems(seq_len: int, causal: bool) -> int:
    """Elements of one packed [S][S] map (what attncache_map_entry_bytes reports per head)."""
    d = DbDesc(n_emb=1, emb_dim=8, emb_dtype=AC_F16, metric=AC_IP, n_entries=1, n_layers=1,
               n_q_heads=1, n_kv_heads=1, head_dim=64, seq_len=seq_len, map_dtype=AC_BF16,
               causal=int(causal), maps_on_host=0, map_layout=AC_LAYOUT_PACKED)
    return attncache_map_entry_bytes(d) // 2


def attncache_pack_maps(dense: torch.Tensor, packed: torch.Tensor, *, causal: bool = True,
                        stream: Optional[torch.cuda.Stream] = None) -> None:
    """dense [n,L,Hq,S,S] bf16 (cuda) -> packed [n,L,Hq,packed_tile_elems(S)] bf16 (cuda)."""
    if dense.dim() != 5 or dense.shape[3] != dense.shape[4]:
        raise ValueError("dense must be [n,L,Hq,S,S]")
    n, L, Hq, S, _ = dense.shape
    d = DbDesc(n_emb=1, emb_dim=8, emb_dtype=AC_F16, metric=AC_IP, n_entries=max(n, 1), n_layers=L,
               n_q_heads=Hq, n_kv_heads=Hq, head_dim=64, seq_len=S, map_dtype=AC_BF16,
               causal=int(causal), maps_on_host=0, map_layout=AC_LAYOUT_PACKED)
    dp = _dev(dense, "dense", torch.bfloat16)
    pp = _dev(packed, "packed", torch.bfloat16, (n, L, Hq, packed_tile_elems(S, causal)))
    _check(lib().attncache_pack_maps(ctypes.byref(d), dp, n, pp, _stream(stream)),
           "attncache_pack_maps")


def attncache_build_db(emb: torch.Tensor, maps: torch.Tensor, *, n_kv_heads: int, head_dim: int,
                       metric: int = AC_IP, causal: bool = True,
                       map_of: Optional[torch.Tensor] = None,
                       staging: Optional[torch.Tensor] = None,
                       side_stream: Optional[torch.cuda.Stream] = None,
                       seq_len: Optional[int] = None) -> Database:
    """emb [N,E] (cuda, f16/f32); maps (cuda, or pinned host) bf16/f32: dense [M,L,Hq,S,S], or
    packed [M,L,Hq,packed_tile_elems(S)] with ``seq_len`` given."""
    packed = maps.dim() == 4
    if packed:
        if seq_len is None or maps.shape[3] != packed_tile_elems(seq_len, causal):
            raise ValueError("packed maps must be [M,L,Hq,packed_tile_elems(seq_len)]")
    elif emb.dim() != 2 or maps.dim() != 5 or maps.shape[3] != maps.shape[4]:
        raise ValueError("emb must be [N,E] and maps [M,L,Hq,S,S]")
    else:
        if seq_len is not None and seq_len != maps.shape[3]:
            raise ValueError("seq_len disagrees with the dense maps")
        seq_len = maps.shape[3]
    on_host = not maps.is_cuda
    if on_host and not maps.is_pinned():
        raise ValueError("host-resident maps must be pinned memory")
    if not maps.is_contiguous():
        raise ValueError("maps must be contiguous")
    if emb.dtype not in (torch.float16, torch.float32) or maps.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("unsupported dtype")
    d = DbDesc(n_emb=emb.shape[0], emb_dim=emb.shape[1], emb_dtype=_DTYPE_CODE[emb.dtype],
               metric=metric, n_entries=maps.shape[0], n_layers=maps.shape[1],
               n_q_heads=maps.shape[2], n_kv_heads=n_kv_heads, head_dim=head_dim,
               seq_len=seq_len, map_dtype=_DTYPE_CODE[maps.dtype], causal=int(causal),
               maps_on_host=int(on_host),
               map_layout=AC_LAYOUT_PACKED if packed else AC_LAYOUT_DENSE)
    emb_p = _dev(emb, "emb")
    mo_p = None if map_of is None else _dev(map_of, "map_of", torch.int32, (emb.shape[0],))
    st_p, st_bytes, ss = None, 0, None
    if on_host:
        if staging is None or side_stream is None:
            raise ValueError("host-resident maps need a staging tensor and a side stream")
        st_p = _dev(staging, "staging")
        st_bytes = staging.numel() * staging.element_size()
        ss = side_stream.cuda_stream
    handle = ctypes.c_void_p()
    _check(lib().attncache_build_db(ctypes.byref(d), emb_p, mo_p, maps.data_ptr(), st_p, st_bytes,
                                    ss, ctypes.byref(handle)), "attncache_build_db")
    return Database(handle, d, (emb, maps, map_of, staging, side_stream))


def attncache_search(db: Database, q: torch.Tensor, k: int, threshold: float,
                     idx: torch.Tensor, score: torch.Tensor, hit: torch.Tensor,
                     ws: torch.Tensor, stream: Optional[torch.cuda.Stream] = None) -> None:
    d = db.desc
    B = q.shape[0]
    emb_dt = torch.float16 if d.emb_dtype == AC_F16 else torch.float32
    qp = _dev(q, "q", emb_dt, (B, d.emb_dim))
    ip = _dev(idx, "idx", torch.int32, (B, k))
    sp = _dev(score, "score", torch.float32, (B, k))
    hp = _dev(hit, "hit", torch.int32, (B,))
    wp = _dev(ws, "ws")
    _check(lib().attncache_search(db.handle, qp, B, k, float(threshold), ip, sp, hp, wp,
                                  ws.numel() * ws.element_size(), _stream(stream)),
           "attncache_search")


AC_STATIC_SCRATCH_BYTES = 4 << 20


def attncache_search_static(db: Database, q: torch.Tensor, k: int, threshold: float,
                            idx: torch.Tensor, score: torch.Tensor, hit: torch.Tensor,
                            stream: Optional[torch.cuda.Stream] = None) -> None:
    """attncache_search on the library's built-in workspace (no allocation anywhere)."""
    d = db.desc
    B = q.shape[0]
    emb_dt = torch.float16 if d.emb_dtype == AC_F16 else torch.float32
    qp = _dev(q, "q", emb_dt, (B, d.emb_dim))
    ip = _dev(idx, "idx", torch.int32, (B, k))
    sp = _dev(score, "score", torch.float32, (B, k))
    hp = _dev(hit, "hit", torch.int32, (B,))
    _check(lib().attncache_search_static(db.handle, qp, B, k, float(threshold), ip, sp, hp,
                                         _stream(stream)), "attncache_search_static")


def attncache_apply(db: Database, hit: torch.Tensor, V: torch.Tensor, O: torch.Tensor,
                    layer_begin: int = 0, layer_count: Optional[int] = None,
                    stream: Optional[torch.cuda.Stream] = None) -> None:
    d = db.desc
    Lc = d.n_layers - layer_begin if layer_count is None else layer_count
    B = V.shape[0]
    dt = torch.bfloat16 if d.map_dtype == AC_BF16 else torch.float32
    vp = _dev(V, "V", dt, (B, Lc, d.n_kv_heads, d.seq_len, d.head_dim))
    op = _dev(O, "O", dt, (B, Lc, d.n_q_heads, d.seq_len, d.head_dim))
    if d.maps_on_host:
        if hit.is_cuda or hit.dtype != torch.int32 or not hit.is_contiguous() or tuple(hit.shape) != (B,):
            raise ValueError("hit must be a contiguous host int32 tensor [B] for host-resident maps")
        hp = hit.data_ptr()
    else:
        hp = _dev(hit, "hit", torch.int32, (B,))
    _check(lib().attncache_apply(db.handle, hp, vp, op, B, layer_begin, Lc, _stream(stream)),
           "attncache_apply")


def attncache_cache_stats(db: Database):
    """(lookups, copies) of the entry cache of a host-resident database."""
    a, b = ctypes.c_uint64(), ctypes.c_uint64()
    _check(lib().attncache_cache_stats(db.handle, ctypes.byref(a), ctypes.byref(b)), "attncache_cache_stats")
    return a.value, b.value


def attncache_cache_reset(db: Database) -> None:
    _check(lib().attncache_cache_reset(db.handle), "attncache_cache_reset")


def attncache_insert(db: Database, Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, O: torch.Tensor, *,
                     slot: Optional[torch.Tensor] = None, feat: Optional[torch.Tensor] = None,
                     row_sel: Optional[torch.Tensor] = None,
                     key_len: Optional[torch.Tensor] = None, layer_begin: int = 0,
                     scale: float = 0.0, stream: Optional[torch.cuda.Stream] = None) -> None:
    """Q,O [B,Lc,Hq,S,D]; K,V [B,Lc,Hkv,S,D] bf16; slot, row_sel, key_len [B] int32; feat [B,E]."""
    d = db.desc
    if Q.dim() != 5:
        raise ValueError("Q must be [B,Lc,Hq,S,D]")
    B, Lc = Q.shape[0], Q.shape[1]
    dt = torch.bfloat16
    qp = _dev(Q, "Q", dt, (B, Lc, d.n_q_heads, d.seq_len, d.head_dim))
    kp = _dev(K, "K", dt, (B, Lc, d.n_kv_heads, d.seq_len, d.head_dim))
    vp = _dev(V, "V", dt, (B, Lc, d.n_kv_heads, d.seq_len, d.head_dim))
    op = _dev(O, "O", dt, (B, Lc, d.n_q_heads, d.seq_len, d.head_dim))
    sp = None if slot is None else _dev(slot, "slot", torch.int32, (B,))
    rp = None if row_sel is None else _dev(row_sel, "row_sel", torch.int32, (B,))
    lp = None if key_len is None else _dev(key_len, "key_len", torch.int32, (B,))
    fdt = torch.float16 if d.emb_dtype == AC_F16 else torch.float32
    fp = None if feat is None else _dev(feat, "feat", fdt, (B, d.emb_dim))
    _check(lib().attncache_insert(db.handle, fp, sp, rp, lp, qp, kp, vp, op, B, layer_begin, Lc,
                                  float(scale), _stream(stream)), "attncache_insert")


def attention_exact(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, O: torch.Tensor, *,
                    causal: bool = True, scale: float = 0.0,
                    row_sel: Optional[torch.Tensor] = None,
                    key_len: Optional[torch.Tensor] = None,
                    stream: Optional[torch.cuda.Stream] = None) -> None:
    """Q,O [B,Hq,S,D]; K,V [B,Hkv,S,D]; bf16 or f32; row_sel, key_len [B] int32."""
    if Q.dim() != 4 or K.dim() != 4:
        raise ValueError("Q must be [B,Hq,S,D] and K,V [B,Hkv,S,D]")
    B, Hq, S, D = Q.shape
    Hkv = K.shape[1]
    if Q.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("unsupported dtype")
    qp = _dev(Q, "Q")
    kp = _dev(K, "K", Q.dtype, (B, Hkv, S, D))
    vp = _dev(V, "V", Q.dtype, (B, Hkv, S, D))
    op = _dev(O, "O", Q.dtype, (B, Hq, S, D))
    rp = None if row_sel is None else _dev(row_sel, "row_sel", torch.int32, (B,))
    lp = None if key_len is None else _dev(key_len, "key_len", torch.int32, (B,))
    _check(lib().attention_exact(qp, kp, vp, op, rp, lp, B, Hq, Hkv, S, D, _DTYPE_CODE[Q.dtype],
                                 int(causal), float(scale), _stream(stream)), "attention_exact")


def attncache_project_workspace_bytes(B: int, model_dim: int, hidden_dim: int, emb_dim: int) -> int:
    return int(lib().attncache_project_workspace_bytes(B, model_dim, hidden_dim, emb_dim))


def attncache_project(h: torch.Tensor, W1: torch.Tensor, b1: Optional[torch.Tensor],
                      W2: torch.Tensor, b2: Optional[torch.Tensor], feat: torch.Tensor,
                      workspace: torch.Tensor, *, seq_len: Optional[torch.Tensor] = None,
                      normalize: bool = True, stream: Optional[torch.cuda.Stream] = None) -> None:
    """h [B,S,dm] bf16|f32; W1 [hid,dm], b1 [hid], W2 [E,hid], b2 [E] f32; feat [B,E] f16|f32."""
    if h.dim() != 3 or W1.dim() != 2 or W2.dim() != 2:
        raise ValueError("h must be [B,S,dm], W1 [hid,dm], W2 [E,hid]")
    B, S, dm = h.shape
    hid, E = W1.shape[0], W2.shape[0]
    if h.dtype not in (torch.bfloat16, torch.float32):
        raise ValueError("h must be bf16 or f32")
    if feat.dtype not in (torch.float16, torch.float32):
        raise ValueError("feat must be f16 or f32")
    f32 = torch.float32
    hp = _dev(h, "h")
    w1 = _dev(W1, "W1", f32, (hid, dm))
    w2 = _dev(W2, "W2", f32, (E, hid))
    b1p = None if b1 is None else _dev(b1, "b1", f32, (hid,))
    b2p = None if b2 is None else _dev(b2, "b2", f32, (E,))
    fp = _dev(feat, "feat", None, (B, E))
    sp = None if seq_len is None else _dev(seq_len, "seq_len", torch.int32, (B,))
    wp = _dev(workspace, "workspace")
    _check(lib().attncache_project(hp, sp, w1, b1p, w2, b2p, fp, B, S, dm, hid, E,
                                   _DTYPE_CODE[h.dtype], _DTYPE_CODE[feat.dtype], int(normalize),
                                   wp, workspace.numel() * workspace.element_size(),
                                   _stream(stream)), "attncache_project")
