"""Thin ctypes binding over the C-ABI library (include/persia_emb.h).

Argument marshalling only: every step of the path runs in the HIP kernels.  torch is used for
device memory and streams; tensors are passed to the library as raw device pointers.  There is no
CPU fallback: if the built library is missing, importing a symbol from it raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np
import torch  # imported before the library so that both use the HIP runtime torch ships

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpersia_emb.so")

EMB_OK, EMB_EINVAL, EMB_ENOMEM, EMB_EDEVICE, EMB_ESTATE = 0, -1, -2, -3, -4
_STATUS = {EMB_EINVAL: "EMB_EINVAL", EMB_ENOMEM: "EMB_ENOMEM", EMB_EDEVICE: "EMB_EDEVICE", EMB_ESTATE: "EMB_ESTATE"}


class emb_table_desc(C.Structure):
    _fields_ = [("rows", C.c_uint64), ("dim", C.c_uint32), ("dtype", C.c_int32)]


class emb_slot_desc(C.Structure):
    _fields_ = [("table", C.c_uint32), ("reserved", C.c_uint32), ("salt", C.c_uint64)]


class emb_config(C.Structure):
    _fields_ = [("num_tables", C.c_uint32), ("num_slots", C.c_uint32),
                ("tables", C.POINTER(emb_table_desc)), ("slots", C.POINTER(emb_slot_desc)),
                ("hash", C.c_int32), ("opt", C.c_int32),
                ("lr", C.c_float), ("eps", C.c_float), ("acc_init", C.c_float),
                ("init_lo", C.c_float), ("init_hi", C.c_float), ("device", C.c_int32),
                ("init_seed", C.c_uint64), ("max_ids", C.c_uint64),
                ("max_batch", C.c_uint32), ("reserved", C.c_uint32)]


class emb_batch(C.Structure):
    _fields_ = [("batch_size", C.c_uint32), ("reserved", C.c_uint32), ("num_ids", C.c_uint64),
                ("ids", C.c_void_p), ("offsets", C.c_void_p)]


class mlp_config(C.Structure):
    _fields_ = [("num_layers", C.c_uint32), ("pooled_width", C.c_uint32), ("dense_width", C.c_uint32),
                ("max_batch", C.c_uint32), ("widths", C.POINTER(C.c_uint32)), ("lr", C.c_float),
                ("loss_mean", C.c_int32), ("device", C.c_int32), ("reserved", C.c_uint32)]


class EmbError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_STATUS.get(code, code)}: {msg}")
        self.code = code


_lib = None


def load_library() -> C.CDLL:
    """Loads the in-tree library; raises if it has not been built (python -m paper_2111_05897_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python paper_2111_05897_amd/build.py`")
    L = C.CDLL(LIB_PATH)
    vp, u32, u64, i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int
    L.emb_create.argtypes = [C.POINTER(emb_config), C.POINTER(vp)]
    L.emb_destroy.argtypes = [vp]
    L.emb_create_cached.argtypes = [C.POINTER(emb_config), vp, C.POINTER(vp)]
    L.emb_cache_stats.argtypes = [vp, u32, vp]
    L.emb_cache_where.argtypes = [vp, u32, vp]
    L.emb_cache_flush.argtypes = [vp, vp]
    for name in ("emb_create_cached", "emb_cache_stats", "emb_cache_where", "emb_cache_flush"):
        getattr(L, name).restype = C.c_int
    L.emb_lookup_pool.argtypes = [vp, C.POINTER(emb_batch), vp, vp]
    L.emb_hash_rows.argtypes = [vp, C.POINTER(emb_batch), vp, vp]
    L.emb_lookup_pool_indexed.argtypes = [vp, u32, u64, u64, vp, vp, vp, vp, vp]
    L.emb_lookup_pool_indexed.restype = C.c_int
    L.emb_backward_update.argtypes = [vp, C.POINTER(emb_batch), vp, vp]
    L.emb_backward_update_static.argtypes = [vp, C.POINTER(emb_batch), vp, vp]
    L.emb_backward_update_static.restype = C.c_int
    L.emb_static_max_ids.argtypes = []
    L.emb_static_max_ids.restype = u64
    L.emb_probe_random_rows.argtypes = [vp, u64, u32, u64, u64, u32, vp, vp]
    L.emb_probe_random_rows.restype = C.c_int
    L.emb_dedup_sizes.argtypes = [vp, C.POINTER(u64), C.POINTER(u64)]
    L.emb_read_dedup.argtypes = [vp, vp, vp, vp]
    L.emb_read_rows.argtypes = [vp, u32, vp, u64, vp, vp]
    L.emb_write_rows.argtypes = [vp, u32, vp, u64, vp, vp]
    L.emb_table_ptr.argtypes = [vp, u32, C.POINTER(vp), C.POINTER(vp)]
    L.emb_set_profiling.argtypes = [vp, i32]
    L.emb_stage_count.argtypes = []
    L.emb_tile_entries.argtypes = []
    L.emb_tile_entries.restype = u32
    L.emb_stage_name.argtypes = [i32]
    L.emb_stage_name.restype = C.c_char_p
    L.emb_read_stage_ms.argtypes = [vp, vp, vp]
    L.emb_reset_stage_ms.argtypes = [vp]
    L.emb_device_bytes.argtypes = [vp]
    L.emb_device_bytes.restype = u64
    L.emb_codec_compress.argtypes = [vp, u64, u32, C.c_float, vp, vp, vp]
    L.emb_codec_decompress.argtypes = [vp, vp, u64, u32, C.c_float, vp, vp]
    L.emb_codec_compress.restype = C.c_int
    L.emb_codec_decompress.restype = C.c_int
    L.mlp_create.argtypes = [C.POINTER(mlp_config), vp, vp, C.POINTER(vp)]
    L.mlp_step.argtypes = [vp, u32, vp, vp, vp, vp, vp, vp]
    L.mlp_read_weights.argtypes = [vp, u32, vp, vp]
    L.mlp_set_update_delay.argtypes = [vp, u32]
    L.mlp_set_update_delay.restype = C.c_int
    L.mlp_destroy.argtypes = [vp]
    L.mlp_device_bytes.argtypes = [vp]
    L.mlp_device_bytes.restype = u64
    L.mlp_last_error.argtypes = [vp]
    L.mlp_last_error.restype = C.c_char_p
    L.mlp_gemm_nt.argtypes = [i32, vp, u32, vp, u32, u32, u32, u32, vp, u32, vp, vp, u32, vp]
    L.mlp_read_state.argtypes = [vp, i32, u32, vp, u64]
    for name in ("mlp_create", "mlp_step", "mlp_read_weights", "mlp_destroy", "mlp_gemm_nt", "mlp_read_state"):
        getattr(L, name).restype = C.c_int
    L.hyb_create.argtypes = [vp, vp, u32, C.POINTER(vp)]
    L.hyb_submit.argtypes = [vp, C.POINTER(emb_batch), vp, vp]
    L.hyb_drain.argtypes = [vp]
    L.hyb_sync.argtypes = [vp]
    L.hyb_wait_inputs.argtypes = [vp]
    L.hyb_counts.argtypes = [vp, C.POINTER(u64), C.POINTER(u64)]
    L.hyb_read_losses.argtypes = [vp, u64, u64, vp]
    L.hyb_destroy.argtypes = [vp]
    L.hyb_last_error.argtypes = [vp]
    L.hyb_last_error.restype = C.c_char_p
    L.emb_describe.argtypes = [vp, C.POINTER(u32), C.POINTER(u32), C.POINTER(u32), C.POINTER(u64), C.POINTER(i32)]
    L.mlp_describe.argtypes = [vp, C.POINTER(u32), C.POINTER(u32), C.POINTER(u32), C.POINTER(i32)]
    for name in ("hyb_create", "hyb_submit", "hyb_drain", "hyb_sync", "hyb_wait_inputs", "hyb_counts", "hyb_read_losses",
                 "hyb_destroy", "emb_describe", "mlp_describe"):
        getattr(L, name).restype = C.c_int
    L.emb_last_error.argtypes = [vp]
    L.emb_last_error.restype = C.c_char_p
    for name in ("emb_create", "emb_destroy", "emb_lookup_pool", "emb_hash_rows", "emb_backward_update",
                 "emb_dedup_sizes", "emb_read_dedup", "emb_read_rows", "emb_write_rows", "emb_table_ptr",
                 "emb_set_profiling", "emb_stage_count", "emb_read_stage_ms", "emb_reset_stage_ms"):
        getattr(L, name).restype = C.c_int
    _lib = L
    return L


def _stream_ptr(stream: Optional[torch.cuda.Stream]) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


class DeviceBatch:
    """A CSR batch resident on the GPU: ids uint64 [N] (held as int64 bits), offsets int32 [B*S+1]."""

    def __init__(self, batch_size: int, ids: np.ndarray, offsets: np.ndarray, device="cuda:0"):
        ids = np.ascontiguousarray(ids, dtype=np.uint64)
        offsets = np.ascontiguousarray(offsets, dtype=np.int32)
        self.batch_size = int(batch_size)
        self.num_ids = int(offsets[-1]) if len(offsets) else 0
        assert self.num_ids == len(ids)
        self.ids = torch.from_numpy(ids.view(np.int64)).to(device)
        self.offsets = torch.from_numpy(offsets).to(device)
        self.c = emb_batch(self.batch_size, 0, self.num_ids, self.ids.data_ptr() if self.num_ids else None,
                           self.offsets.data_ptr())


class EmbContext:
    """Owns one emb_ctx.  Method names mirror the C entry points."""

    def __init__(self, tables: Sequence[Tuple[int, int, int]], slots: Sequence[Tuple[int, int]], hash_kind: int,
                 opt: int, lr: float, eps: float, acc_init: float, init_seed: int, init_lo: float, init_hi: float,
                 max_batch: int, max_ids: int, device: int = 0, cache_rows: Optional[Sequence[int]] = None):
        """cache_rows (optional, one entry per table): device-memory slots of a table kept in host memory behind
        the LRU cache (emb_create_cached); 0 keeps the table resident."""
        self.L = load_library()
        self.tables = [tuple(t) for t in tables]
        self.slots = [tuple(s) for s in slots]
        self.device = device
        self._t = (emb_table_desc * len(tables))(*[emb_table_desc(r, d, dt) for r, d, dt in tables])
        self._s = (emb_slot_desc * len(slots))(*[emb_slot_desc(t, 0, salt) for t, salt in slots])
        cfg = emb_config(len(tables), len(slots), self._t, self._s, hash_kind, opt, lr, eps, acc_init, init_lo, init_hi,
                         device, init_seed, max_ids, max_batch, 0)
        h = C.c_void_p()
        if cache_rows is None:
            rc = self.L.emb_create(C.byref(cfg), C.byref(h))
        else:
            assert len(cache_rows) == len(tables)
            cr = (C.c_uint64 * len(tables))(*[int(c) for c in cache_rows])
            rc = self.L.emb_create_cached(C.byref(cfg), cr, C.byref(h))
        if rc:
            raise EmbError(rc, self.L.emb_last_error(None).decode())
        self.h = h
        self.S = len(slots)
        self.width = sum(self.tables[t][1] for t, _ in slots)

    @classmethod
    def from_config(cls, cfg, max_batch: int, max_ids: int, device: int = 0, cache_rows=None):
        """cfg: workload.EmbConfig (duck-typed)."""
        return cls([(t.rows, t.dim, t.dtype) for t in cfg.tables], [(s.table, s.salt) for s in cfg.slots],
                   cfg.hash_kind, cfg.opt, cfg.lr, cfg.eps, cfg.acc_init, cfg.init_seed, cfg.init_lo, cfg.init_hi,
                   max_batch, max_ids, device, cache_rows=cache_rows)

    def _ck(self, rc: int):
        if rc:
            raise EmbError(rc, self.L.emb_last_error(self.h).decode())

    def close(self):
        if getattr(self, "h", None):
            self.L.emb_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- hot calls (enqueue only) ----
    def emb_lookup_pool(self, batch: DeviceBatch, pooled: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
        if pooled is None:
            pooled = torch.empty((batch.batch_size, self.width), dtype=torch.float32, device=batch.offsets.device)
        assert pooled.is_contiguous() and pooled.dtype == torch.float32
        assert pooled.shape == (batch.batch_size, self.width)
        self._ck(self.L.emb_lookup_pool(self.h, C.byref(batch.c), pooled.data_ptr(), _stream_ptr(stream)))
        return pooled

    def emb_lookup_pool_indexed(self, batch_size: int, keys: torch.Tensor, seg_off: torch.Tensor, seg_bags: torch.Tensor,
                                pooled: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
        """keys: int64 bits of (table << 32) | row [U]; seg_off: int32 bits of uint32 [U+1]; seg_bags: int32 [N]."""
        if pooled is None:
            pooled = torch.empty((batch_size, self.width), dtype=torch.float32, device=seg_off.device)
        assert pooled.is_contiguous() and pooled.dtype == torch.float32 and pooled.shape == (batch_size, self.width)
        assert keys.dtype == torch.int64 and seg_off.dtype == torch.int32 and seg_bags.dtype == torch.int32
        assert keys.is_contiguous() and seg_off.is_contiguous() and seg_bags.is_contiguous()
        U, N = keys.numel(), seg_bags.numel()
        assert seg_off.numel() == U + 1
        self._ck(self.L.emb_lookup_pool_indexed(self.h, batch_size, U, N, keys.data_ptr() if U else None,
                                                seg_off.data_ptr(), seg_bags.data_ptr() if N else None,
                                                pooled.data_ptr(), _stream_ptr(stream)))
        return pooled

    def emb_hash_rows(self, batch: DeviceBatch, stream=None) -> torch.Tensor:
        rows = torch.empty(max(batch.num_ids, 1), dtype=torch.int32, device=batch.offsets.device)
        self._ck(self.L.emb_hash_rows(self.h, C.byref(batch.c), rows.data_ptr(), _stream_ptr(stream)))
        return rows[: batch.num_ids]

    def emb_backward_update(self, batch: DeviceBatch, d_pooled: torch.Tensor, stream=None) -> None:
        assert d_pooled.is_contiguous() and d_pooled.dtype == torch.float32
        assert d_pooled.shape == (batch.batch_size, self.width)
        self._ck(self.L.emb_backward_update(self.h, C.byref(batch.c), d_pooled.data_ptr(), _stream_ptr(stream)))

    def emb_backward_update_static(self, batch: DeviceBatch, d_pooled: torch.Tensor, stream=None) -> None:
        assert d_pooled.is_contiguous() and d_pooled.dtype == torch.float32
        assert d_pooled.shape == (batch.batch_size, self.width)
        self._ck(self.L.emb_backward_update_static(self.h, C.byref(batch.c), d_pooled.data_ptr(), _stream_ptr(stream)))

    # ---- inspection (synchronous) ----
    def emb_dedup_sizes(self) -> Tuple[int, int]:
        U, N = C.c_uint64(), C.c_uint64()
        self._ck(self.L.emb_dedup_sizes(self.h, C.byref(U), C.byref(N)))
        return U.value, N.value

    def emb_read_dedup(self):
        U, N = self.emb_dedup_sizes()
        keys = np.empty(U, dtype=np.uint64)
        seg_off = np.empty(U + 1, dtype=np.uint32)
        seg_bags = np.empty(N, dtype=np.uint32)
        self._ck(self.L.emb_read_dedup(self.h, keys.ctypes.data, seg_off.ctypes.data, seg_bags.ctypes.data))
        return keys, seg_off, seg_bags

    def emb_read_rows(self, table: int, rows) -> Tuple[np.ndarray, np.ndarray]:
        rows = np.ascontiguousarray(rows, dtype=np.uint64)
        w = np.empty((len(rows), self.tables[table][1]), dtype=np.float32)
        acc = np.empty(len(rows), dtype=np.float32)
        self._ck(self.L.emb_read_rows(self.h, table, rows.ctypes.data, len(rows), w.ctypes.data, acc.ctypes.data))
        return w, acc

    def emb_write_rows(self, table: int, rows, w, acc=None) -> None:
        rows = np.ascontiguousarray(rows, dtype=np.uint64)
        w = np.ascontiguousarray(w, dtype=np.float32)
        assert w.shape == (len(rows), self.tables[table][1])
        ap = None
        if acc is not None:
            acc = np.ascontiguousarray(acc, dtype=np.float32)
            ap = acc.ctypes.data
        self._ck(self.L.emb_write_rows(self.h, table, rows.ctypes.data, len(rows), w.ctypes.data, ap))

    def emb_cache_stats(self, table: int) -> dict:
        st = (C.c_uint64 * 4)()
        self._ck(self.L.emb_cache_stats(self.h, table, st))
        return {"requested": st[0], "misses": st[1], "written_back": st[2], "overflows": st[3]}

    def emb_cache_where(self, table: int) -> np.ndarray:
        out = np.empty(self.tables[table][0], dtype=np.int32)
        self._ck(self.L.emb_cache_where(self.h, table, out.ctypes.data))
        return out

    def emb_cache_flush(self, stream=None) -> None:
        self._ck(self.L.emb_cache_flush(self.h, _stream_ptr(stream)))

    def emb_table_ptr(self, table: int) -> Tuple[int, int]:
        w, a = C.c_void_p(), C.c_void_p()
        self._ck(self.L.emb_table_ptr(self.h, table, C.byref(w), C.byref(a)))
        return w.value, a.value

    def emb_set_profiling(self, enabled: bool) -> None:
        self._ck(self.L.emb_set_profiling(self.h, 1 if enabled else 0))

    def emb_reset_stage_ms(self) -> None:
        self._ck(self.L.emb_reset_stage_ms(self.h))

    def emb_read_stage_ms(self) -> dict:
        n = self.L.emb_stage_count()
        ms = (C.c_float * n)()
        cnt = (C.c_uint32 * n)()
        self._ck(self.L.emb_read_stage_ms(self.h, ms, cnt))
        return {self.L.emb_stage_name(i).decode(): (float(ms[i]), int(cnt[i])) for i in range(n)}

    def emb_device_bytes(self) -> int:
        return int(self.L.emb_device_bytes(self.h))


def emb_probe_random_rows(base_ptr: int, rows: int, row_bytes: int, n_reads: int, sink: torch.Tensor, hot_rows: int = 0,
                          hot_of_8: int = 0, stream=None) -> None:
    """Enqueues the bare random-row read probe on the array at device address base_ptr (rows * row_bytes bytes)."""
    L = load_library()
    assert sink.is_cuda and sink.numel() * sink.element_size() >= 16
    rc = L.emb_probe_random_rows(base_ptr, rows, row_bytes, n_reads, hot_rows, hot_of_8, sink.data_ptr(), _stream_ptr(stream))
    if rc:
        raise EmbError(rc, "emb_probe_random_rows: bad arguments")


def emb_codec_compress(v: torch.Tensor, block_len: int, kappa: float = 2.0 ** 15, stream=None):
    """v: fp32 device tensor, numel a multiple of block_len -> (q fp16 [n_blocks, block_len], norm fp32 [n_blocks])."""
    L = load_library()
    assert v.is_contiguous() and v.dtype == torch.float32 and v.numel() % block_len == 0
    n_blocks = v.numel() // block_len
    q = torch.empty((n_blocks, block_len), dtype=torch.float16, device=v.device)
    norm = torch.empty(max(n_blocks, 1), dtype=torch.float32, device=v.device)
    rc = L.emb_codec_compress(v.data_ptr(), n_blocks, block_len, kappa, q.data_ptr(), norm.data_ptr(), _stream_ptr(stream))
    if rc:
        raise EmbError(rc, L.emb_last_error(None).decode())
    return q, norm[:n_blocks]


def emb_codec_decompress(q: torch.Tensor, norm: torch.Tensor, kappa: float = 2.0 ** 15, stream=None) -> torch.Tensor:
    L = load_library()
    assert q.is_contiguous() and q.dtype == torch.float16 and q.dim() == 2 and norm.dtype == torch.float32
    n_blocks, block_len = q.shape
    out = torch.empty((n_blocks, block_len), dtype=torch.float32, device=q.device)
    rc = L.emb_codec_decompress(q.data_ptr(), norm.data_ptr(), n_blocks, block_len, kappa, out.data_ptr(),
                                _stream_ptr(stream))
    if rc:
        raise EmbError(rc, L.emb_last_error(None).decode())
    return out


class MlpContext:
    """Owns one mlp_ctx (the optional dense step).  weights[l]: numpy fp32 [widths[l], widths[l+1]]."""

    def __init__(self, widths, pooled_width, dense_width, max_batch, lr, weights, biases, loss_mean=True, device=0):
        self.L = load_library()
        self.widths = list(widths)
        self.pooled_width, self.dense_width = pooled_width, dense_width
        nl = len(widths) - 1
        self._w = (C.c_uint32 * len(widths))(*widths)
        ws = [np.ascontiguousarray(w, dtype=np.float32) for w in weights]
        bs = [np.ascontiguousarray(b, dtype=np.float32) for b in biases]
        assert len(ws) == nl and len(bs) == nl
        for l in range(nl):
            assert ws[l].shape == (widths[l], widths[l + 1]) and bs[l].shape == (widths[l + 1],)
        wp = (C.c_void_p * nl)(*[w.ctypes.data for w in ws])
        bp = (C.c_void_p * nl)(*[b.ctypes.data for b in bs])
        cfg = mlp_config(nl, pooled_width, dense_width, max_batch, self._w, lr, 1 if loss_mean else 0, device, 0)
        h = C.c_void_p()
        rc = self.L.mlp_create(C.byref(cfg), wp, bp, C.byref(h))
        if rc:
            raise EmbError(rc, self.L.mlp_last_error(None).decode())
        self.h = h

    def _ck(self, rc):
        if rc:
            raise EmbError(rc, self.L.mlp_last_error(self.h).decode())

    def mlp_step(self, pooled, dense, labels, d_pooled=None, stream=None):
        B = pooled.shape[0]
        assert pooled.is_contiguous() and pooled.dtype == torch.float32 and pooled.shape == (B, self.pooled_width)
        assert dense.is_contiguous() and dense.dtype == torch.float32 and dense.shape == (B, self.dense_width)
        assert labels.is_contiguous() and labels.dtype == torch.float32 and labels.shape == (B,)
        if d_pooled is None:
            d_pooled = torch.empty_like(pooled)
        loss = torch.empty(1, dtype=torch.float32, device=pooled.device)
        self._ck(self.L.mlp_step(self.h, B, pooled.data_ptr(), dense.data_ptr(), labels.data_ptr(), d_pooled.data_ptr(),
                                 loss.data_ptr(), _stream_ptr(stream)))
        return d_pooled, loss

    def mlp_set_update_delay(self, delay: int):
        self._ck(self.L.mlp_set_update_delay(self.h, int(delay)))

    def mlp_read_weights(self, layer):
        w = np.empty((self.widths[layer], self.widths[layer + 1]), dtype=np.float32)
        b = np.empty(self.widths[layer + 1], dtype=np.float32)
        self._ck(self.L.mlp_read_weights(self.h, layer, w.ctypes.data, b.ctypes.data))
        return w, b

    def mlp_read_state(self, what, layer, batch):
        """what: 'h' | 'delta' | 'dW' | 'db' | 'dz'.  bf16 states come back widened to fp32."""
        kind = {"h": 0, "delta": 1, "dW": 2, "db": 3, "dz": 4}[what]
        if kind <= 1:
            raw = np.empty((batch, self.widths[layer]), dtype=np.uint16)
        elif kind == 2:
            raw = np.empty((self.widths[layer], self.widths[layer + 1]), dtype=np.float32)
        elif kind == 3:
            raw = np.empty(self.widths[layer + 1], dtype=np.float32)
        else:
            raw = np.empty(batch, dtype=np.float32)
        self._ck(self.L.mlp_read_state(self.h, kind, layer, raw.ctypes.data, raw.nbytes))
        if kind <= 1:
            return (raw.astype(np.uint32) << 16).view(np.float32)
        return raw

    def mlp_device_bytes(self):
        return int(self.L.mlp_device_bytes(self.h))

    def close(self):
        if getattr(self, "h", None):
            self.L.mlp_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def mlp_gemm_nt(epilogue, A, Bt, bias=None, mask=None, stream=None):
    """C = A @ Bt.T for bf16 device tensors A [M, K], Bt [N, K]; see include/persia_emb.h for the epilogues."""
    L = load_library()
    assert A.dtype == torch.bfloat16 and Bt.dtype == torch.bfloat16 and A.is_contiguous() and Bt.is_contiguous()
    M, K = A.shape
    N = Bt.shape[0]
    Cm = torch.empty((M, N), dtype=torch.float32 if epilogue == 1 else torch.bfloat16, device=A.device)
    rc = L.mlp_gemm_nt(epilogue, A.data_ptr(), K, Bt.data_ptr(), K, M, N, K, Cm.data_ptr(), N,
                       bias.data_ptr() if bias is not None else None, mask.data_ptr() if mask is not None else None,
                       N, _stream_ptr(stream))
    if rc:
        raise EmbError(rc, L.mlp_last_error(None).decode())
    return Cm


class HybridLoop:
    """Owns one hyb_ctx: the step loop with staleness tau over an EmbContext and an MlpContext (both stay owned by
    the caller and must outlive the loop).  Method names mirror the C entry points."""

    def __init__(self, emb: "EmbContext", mlp: "MlpContext", tau: int):
        self.L = load_library()
        self.emb, self.mlp, self.tau = emb, mlp, int(tau)
        h = C.c_void_p()
        rc = self.L.hyb_create(emb.h, mlp.h, self.tau, C.byref(h))
        if rc:
            raise EmbError(rc, self.L.hyb_last_error(None).decode())
        self.h = h

    def _ck(self, rc):
        if rc:
            raise EmbError(rc, self.L.hyb_last_error(self.h).decode())

    def hyb_submit(self, batch: "DeviceBatch", dense, labels):
        B = batch.batch_size
        assert labels.is_contiguous() and labels.dtype == torch.float32 and labels.shape == (B,)
        assert dense is None or (dense.is_contiguous() and dense.dtype == torch.float32 and dense.shape[0] == B)
        self._ck(self.L.hyb_submit(self.h, C.byref(batch.c), dense.data_ptr() if dense is not None else None,
                                   labels.data_ptr()))

    def hyb_drain(self):
        self._ck(self.L.hyb_drain(self.h))

    def hyb_sync(self):
        self._ck(self.L.hyb_sync(self.h))

    def hyb_wait_inputs(self):
        self._ck(self.L.hyb_wait_inputs(self.h))

    def hyb_counts(self):
        a, b = C.c_uint64(), C.c_uint64()
        self._ck(self.L.hyb_counts(self.h, C.byref(a), C.byref(b)))
        return a.value, b.value

    def hyb_read_losses(self, first, count):
        out = np.empty(count, dtype=np.float32)
        self._ck(self.L.hyb_read_losses(self.h, first, count, out.ctypes.data))
        return out

    def close(self):
        if getattr(self, "h", None):
            self.L.hyb_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
