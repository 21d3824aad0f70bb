"""ctypes binding of libcacheback_verify.so (see include/cacheback.h): argument marshalling only.

Every step of the verification runs inside the library's HIP kernels; PyTorch is used here for
device memory and streams.  Loading fails loudly when the library has not been built
(``python -m paper_2511_21699_amd.build``); there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcacheback_verify.so")

CB_F32, CB_BF16 = 0, 1
CB_OK, CB_EINVAL, CB_ETREE, CB_ECAP, CB_ESTATE, CB_EHIP = range(6)
CB_LAYOUT_TOKEN_MAJOR, CB_LAYOUT_HEAD_MAJOR = 0, 1
ERROR_NAMES = {0: "CB_OK", 1: "CB_EINVAL", 2: "CB_ETREE", 3: "CB_ECAP", 4: "CB_ESTATE", 5: "CB_EHIP"}

EXPORTS = ["cb_workspace_bytes", "cb_init", "cb_check_verify_args", "cb_plan_attention", "cb_verify_tree", "cb_verify_tree_device", "cb_tree_attention_device", "cb_tree_attention_noalloc",
           "cb_compact_kv", "cb_get_path", "cb_get_argmax", "cb_device_status", "cb_set_option",
           "cb_last_launch_info", "cb_last_attention_ms", "cb_debug_timestamps", "cb_probe_stream_read", "cb_last_error",
           "cb_destroy"]


DRAFTER_EXPORTS = ["cbd_table_create", "cbd_table_destroy", "cbd_table_insert", "cbd_table_update", "cbd_table_query",
                   "cbd_table_build_frozen", "cbd_table_freeze", "cbd_table_size", "cbd_grow_tree"]


class CbConfig(C.Structure):
    _fields_ = [("num_q_heads", C.c_int32), ("num_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("qkv_dtype", C.c_int32), ("logits_dtype", C.c_int32), ("max_batch", C.c_int32),
                ("max_nodes", C.c_int32), ("max_depth", C.c_int32), ("vocab_size", C.c_int32),
                ("block_size", C.c_int32), ("max_splits", C.c_int32), ("softmax_scale", C.c_float)]


class CbKvLayer(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("capacity_or_num_blocks", C.c_int64),
                ("block_table", C.c_void_p), ("max_blocks_per_seq", C.c_int32), ("layout", C.c_int32)]


class CbError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"{ERROR_NAMES.get(code, code)}: {text}")
        self.code = code


_lib = None


def load():
    """dlopen the HIP library; raises if it is missing (no fallback of any kind)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2511_21699_amd.build` (needs hipcc)")
    L = C.CDLL(LIB_PATH)
    vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
    L.cb_workspace_bytes.argtypes = [C.POINTER(CbConfig), C.POINTER(C.c_size_t)]
    L.cb_init.argtypes = [C.POINTER(CbConfig), vp, C.c_size_t, C.POINTER(vp)]
    L.cb_check_verify_args.argtypes = [C.POINTER(CbConfig), C.c_int32, C.POINTER(CbKvLayer), i32p, i32p, i32p,
                                       C.c_char_p, C.c_size_t]
    L.cb_plan_attention.argtypes = [C.POINTER(CbConfig), C.c_int32, i32p, i32p, C.c_int32, i32p]
    L.cb_verify_tree.argtypes = [vp, vp, C.c_int32, vp, C.POINTER(CbKvLayer), i32p, i32p, i32p, i32p, vp, vp, i32p, i32p]
    L.cb_verify_tree_device.argtypes = [vp, vp, C.c_int32, vp, C.POINTER(CbKvLayer), i32p, i32p, vp, vp, vp, vp, vp, vp]
    L.cb_tree_attention_device.argtypes = [vp, vp, C.c_int32, vp, C.POINTER(CbKvLayer), i32p, i32p, vp, vp]
    L.cb_tree_attention_noalloc.argtypes = [C.POINTER(CbConfig), vp, C.c_int32, vp, C.POINTER(CbKvLayer), i32p, i32p, vp, vp]
    L.cb_compact_kv.argtypes = [vp, vp, C.c_int32, C.POINTER(CbKvLayer), i32p]
    L.cb_get_path.argtypes = [vp, i32p]
    L.cb_get_argmax.argtypes = [vp, i32p]
    L.cb_device_status.argtypes = [vp, i32p]
    L.cb_set_option.argtypes = [vp, C.c_char_p, C.c_int64]
    L.cb_last_launch_info.argtypes = [vp, i32p]
    L.cb_last_attention_ms.argtypes = [vp, C.POINTER(C.c_float)]
    L.cb_debug_timestamps.argtypes = [vp, C.POINTER(C.c_uint64), C.c_int32]
    L.cb_probe_stream_read.argtypes = [vp, vp, C.c_int64, vp]
    L.cbd_table_create.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(vp)]
    L.cbd_table_destroy.argtypes = [vp]
    L.cbd_table_destroy.restype = None
    L.cbd_table_insert.argtypes = [vp, i32p, i32p]
    L.cbd_table_update.argtypes = [vp, i32p, C.c_int64, C.c_int64]
    L.cbd_table_query.argtypes = [vp, i32p, C.c_int32, i32p, i32p]
    L.cbd_table_build_frozen.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, i32p, C.c_int64, C.POINTER(vp)]
    L.cbd_table_freeze.argtypes = [vp]
    L.cbd_table_size.argtypes = [vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
    L.cbd_grow_tree.argtypes = [C.POINTER(vp), C.c_int32, i32p, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                i32p, i32p, i32p, i32p]
    L.cb_last_error.argtypes = [vp]
    L.cb_last_error.restype = C.c_char_p
    L.cb_destroy.argtypes = [vp]
    L.cb_destroy.restype = None
    for name in EXPORTS:
        if name not in ("cb_last_error", "cb_destroy"):
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ip(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def make_config(Hq: int, Hkv: int, D: int, qkv_dtype: str, logits_dtype: str, max_batch: int, max_nodes: int,
                max_depth: int, vocab: int, block_size: int = 0, max_splits: int = 0,
                softmax_scale: float = 0.0) -> CbConfig:
    dt = {"f32": CB_F32, "bf16": CB_BF16}
    return CbConfig(Hq, Hkv, D, dt[qkv_dtype], dt[logits_dtype], max_batch, max_nodes, max_depth, vocab,
                    block_size, max_splits, softmax_scale)


def kv_layer(k, v, block_table=None, layout: int = CB_LAYOUT_TOKEN_MAJOR, paged: bool = False) -> CbKvLayer:
    """Describe one layer's cache held in torch tensors (token-major shapes as in cacheback.h)."""
    if paged:
        cap = k.shape[0]
        return CbKvLayer(k.data_ptr(), v.data_ptr(), cap, block_table.data_ptr(), block_table.shape[1], layout)
    cap = k.shape[1] if layout == CB_LAYOUT_TOKEN_MAJOR else k.shape[2]
    return CbKvLayer(k.data_ptr(), v.data_ptr(), cap, None, 0, layout)


def check_verify_args(cfg: CbConfig, batch: int, kv: CbKvLayer, kv_len, node_offsets, parent) -> Tuple[int, str]:
    """Host-only argument check (no GPU needed)."""
    L = load()
    buf = C.create_string_buffer(256)
    a, b, c = _i32(kv_len), _i32(node_offsets), _i32(parent)
    rc = L.cb_check_verify_args(C.byref(cfg), batch, C.byref(kv), _ip(a), _ip(b), _ip(c), buf, 256)
    return rc, buf.value.decode()


def plan_attention(cfg: CbConfig, kv_len, node_offsets, forced_splits: int = 0) -> dict:
    """Host-only: the attention stage's split plan for these lengths (no GPU needed)."""
    a, b = _i32(kv_len), _i32(node_offsets)
    out = (C.c_int32 * 5)()
    rc = load().cb_plan_attention(C.byref(cfg), len(a), _ip(a), _ip(b), forced_splits, out)
    if rc:
        raise CbError(rc, "cb_plan_attention rejected the shape")
    return dict(impl=out[0], nsplit=out[1], chunk=out[2], tile_rows=out[3], workgroups=out[4])


def probe_stream_read(d_src, nbytes: int, d_sink, stream=None) -> None:
    """Enqueue a bare streaming read of the first `nbytes` of the tensor d_src (cb_probe_stream_read)."""
    import torch
    st = stream if stream is not None else torch.cuda.current_stream()
    rc = load().cb_probe_stream_read(C.c_void_p(st.cuda_stream), C.c_void_p(d_src.data_ptr()), nbytes,
                                     C.c_void_p(d_sink.data_ptr()))
    if rc:
        raise CbError(rc, "cb_probe_stream_read rejected the arguments")


def tree_attention_noalloc(cfg: CbConfig, q, kv: CbKvLayer, kv_len, node_offsets, d_parent, attn_out, stream=None) -> None:
    """cb_tree_attention_noalloc on torch tensors: no context, no workspace, launches only."""
    import torch
    st = stream if stream is not None else torch.cuda.current_stream()
    kv_len, node_offsets = _i32(kv_len), _i32(node_offsets)
    L = load()
    rc = L.cb_tree_attention_noalloc(C.byref(cfg), C.c_void_p(st.cuda_stream), kv_len.shape[0], q.data_ptr(), C.byref(kv),
                                     _ip(kv_len), _ip(node_offsets), d_parent.data_ptr(), attn_out.data_ptr())
    if rc:
        raise CbError(rc, L.cb_last_error(None).decode())


def workspace_bytes(cfg: CbConfig) -> int:
    n = C.c_size_t(0)
    rc = load().cb_workspace_bytes(C.byref(cfg), C.byref(n))
    if rc:
        raise CbError(rc, load().cb_last_error(None).decode())
    return n.value


class Verifier:
    """One library context plus its torch-owned workspace."""

    def __init__(self, cfg: CbConfig, device: str = "cuda:0"):
        import torch
        self._torch = torch
        self.L = load()
        self.cfg = cfg
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        nbytes = workspace_bytes(cfg)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        ctx = C.c_void_p()
        rc = self.L.cb_init(C.byref(cfg), base, nbytes, C.byref(ctx))
        if rc:
            raise CbError(rc, self.L.cb_last_error(None).decode())
        self.ctx = ctx
        self.stride = cfg.max_depth + 1

    def close(self):
        if getattr(self, "ctx", None):
            self.L.cb_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _raise(self, rc: int):
        if rc:
            raise CbError(rc, self.L.cb_last_error(self.ctx).decode())

    def _stream(self, stream) -> Optional[int]:
        if stream is None:
            stream = self._torch.cuda.current_stream(self.device)
        return C.c_void_p(stream.cuda_stream)

    def verify_tree(self, q, kv: CbKvLayer, kv_len, node_offsets, parent, tokens, logits, attn_out=None, stream=None):
        """Host-array form; returns (attn_out, accepted_len[B], accepted_tokens[B, max_depth+1])."""
        kv_len, node_offsets, parent, tokens = _i32(kv_len), _i32(node_offsets), _i32(parent), _i32(tokens)
        batch = kv_len.shape[0]
        if attn_out is None:
            attn_out = self._torch.empty_like(q)
        acc_len = np.zeros(batch, dtype=np.int32)
        acc_tok = np.zeros((batch, self.stride), dtype=np.int32)
        rc = self.L.cb_verify_tree(self.ctx, self._stream(stream), batch, q.data_ptr(), C.byref(kv), _ip(kv_len),
                                   _ip(node_offsets), _ip(parent), _ip(tokens), logits.data_ptr(),
                                   attn_out.data_ptr(), _ip(acc_len), _ip(acc_tok))
        self._raise(rc)
        return attn_out, acc_len, acc_tok

    def verify_tree_device(self, q, kv: CbKvLayer, kv_len, node_offsets, d_parent, d_tokens, logits, attn_out,
                           d_acc_len, d_acc_tok, stream=None):
        """Device-resident form: enqueues launches only."""
        kv_len, node_offsets = _i32(kv_len), _i32(node_offsets)
        rc = self.L.cb_verify_tree_device(self.ctx, self._stream(stream), kv_len.shape[0], q.data_ptr(), C.byref(kv),
                                          _ip(kv_len), _ip(node_offsets), d_parent.data_ptr(), d_tokens.data_ptr(),
                                          logits.data_ptr(), attn_out.data_ptr(), d_acc_len.data_ptr(),
                                          d_acc_tok.data_ptr())
        self._raise(rc)

    def tree_attention_device(self, q, kv: CbKvLayer, kv_len, node_offsets, d_parent, attn_out, stream=None):
        """Tree attention alone (a model's layers below the last): enqueues launches only."""
        kv_len, node_offsets = _i32(kv_len), _i32(node_offsets)
        rc = self.L.cb_tree_attention_device(self.ctx, self._stream(stream), kv_len.shape[0], q.data_ptr(), C.byref(kv),
                                             _ip(kv_len), _ip(node_offsets), d_parent.data_ptr(), attn_out.data_ptr())
        self._raise(rc)

    def bind_model_step(self, qs, kvs, kv_len, node_offsets, d_parent, d_tokens, logits, attn_outs, d_acc_len, d_acc_tok,
                        stream=None):
        """Pre-marshalled step of a whole model: tree attention for every layer (the last one inside the
        verification call, which also scans the logits and accepts), then one compaction of all layers.
        Returns a zero-argument callable that only makes the C calls."""
        kv_len, node_offsets = _i32(kv_len), _i32(node_offsets)
        st = self._stream(stream)
        nl = len(kvs)
        arr = (CbKvLayer * nl)(*kvs)
        b = kv_len.shape[0]
        att = [(self.ctx, st, b, qs[i].data_ptr(), C.byref(arr[i]), _ip(kv_len), _ip(node_offsets), d_parent.data_ptr(),
                attn_outs[i].data_ptr()) for i in range(nl - 1)]
        last = (self.ctx, st, b, qs[-1].data_ptr(), C.byref(arr[nl - 1]), _ip(kv_len), _ip(node_offsets),
                d_parent.data_ptr(), d_tokens.data_ptr(), logits.data_ptr(), attn_outs[-1].data_ptr(),
                d_acc_len.data_ptr(), d_acc_tok.data_ptr())
        keep = (kv_len, node_offsets, arr, qs, kvs, logits, attn_outs)
        attention, verify, compact = self.L.cb_tree_attention_device, self.L.cb_verify_tree_device, self.L.cb_compact_kv

        def call(_keep=keep):
            rc = 0
            for a in att:
                rc = rc or attention(*a)
            rc = rc or verify(*last)
            rc = rc or compact(self.ctx, st, nl, arr, None)
            if rc:
                self._raise(rc)
        return call

    def bind_step(self, q, kv: CbKvLayer, kv_len, node_offsets, d_parent, d_tokens, logits, attn_out, d_acc_len,
                  d_acc_tok, layers: Sequence[CbKvLayer], stream=None):
        """Pre-marshalled cb_verify_tree_device + cb_compact_kv pair: returns a zero-argument callable that
        only makes the two C calls (for launch loops where per-call marshalling would dominate)."""
        kv_len, node_offsets = _i32(kv_len), _i32(node_offsets)
        arr = (CbKvLayer * len(layers))(*layers) if layers else None
        st = self._stream(stream)
        a = (self.ctx, st, kv_len.shape[0], q.data_ptr(), C.byref(kv), _ip(kv_len), _ip(node_offsets),
             d_parent.data_ptr(), d_tokens.data_ptr(), logits.data_ptr(), attn_out.data_ptr(), d_acc_len.data_ptr(),
             d_acc_tok.data_ptr())
        keep = (kv_len, node_offsets, arr, kv, q, logits, attn_out)
        verify, compact, nl = self.L.cb_verify_tree_device, self.L.cb_compact_kv, len(layers)

        def call(_keep=keep):
            rc = verify(*a)
            if rc == 0 and nl:
                rc = compact(self.ctx, st, nl, arr, None)
            if rc:
                self._raise(rc)
        return call

    def bind_host_step(self, q, kv: CbKvLayer, logits, attn_out, batch: int = 1, layers: Sequence[CbKvLayer] = (),
                       stream=None, parent=None, tokens=None) -> "HostStep":
        """Pre-marshalled cb_verify_tree (+ cb_compact_kv): the caller fills the returned object's host arrays in
        place and calls `verify()` / `compact()`, which only make the C calls (for decode loops, where per-call
        marshalling would cost as much as the GPU work).  `parent` / `tokens`: int32 arrays to bind as the tree
        (a TreeGrower's outputs, say) instead of arrays of the object's own."""
        return HostStep(self, q, kv, logits, attn_out, batch, layers, stream, parent, tokens)

    def compact_kv(self, layers: Sequence[CbKvLayer], batch: int, want_len: bool = True, stream=None):
        arr = (CbKvLayer * len(layers))(*layers)
        new_len = np.zeros(batch, dtype=np.int32)
        rc = self.L.cb_compact_kv(self.ctx, self._stream(stream), len(layers), arr, _ip(new_len) if want_len else None)
        self._raise(rc)
        return new_len if want_len else None

    def get_path(self, batch: int) -> np.ndarray:
        out = np.zeros((batch, self.stride), dtype=np.int32)
        self._raise(self.L.cb_get_path(self.ctx, _ip(out)))
        return out

    def get_argmax(self, total_nodes: int) -> np.ndarray:
        out = np.zeros(total_nodes, dtype=np.int32)
        self._raise(self.L.cb_get_argmax(self.ctx, _ip(out)))
        return out

    def device_status(self) -> int:
        s = C.c_int32(0)
        self._raise(self.L.cb_device_status(self.ctx, C.byref(s)))
        return s.value

    def set_option(self, name: str, value: int):
        self._raise(self.L.cb_set_option(self.ctx, name.encode(), int(value)))

    def debug_timestamps(self, workgroups: int) -> np.ndarray:
        out = np.zeros((workgroups, 8), dtype=np.uint64)
        self._raise(self.L.cb_debug_timestamps(self.ctx, out.ctypes.data_as(C.POINTER(C.c_uint64)), workgroups))
        return out

    def last_launch_info(self) -> dict:
        out = (C.c_int32 * 6)()
        self._raise(self.L.cb_last_launch_info(self.ctx, out))
        return dict(impl=out[0], nsplit=out[1], chunk=out[2], fused=bool(out[3]),
                    merge=("none", "cooperative", "last_arrival", "merge_kernel")[out[4]], kernels=out[5])

    def last_attention_ms(self) -> float:
        ms = C.c_float(0)
        self._raise(self.L.cb_last_attention_ms(self.ctx, C.byref(ms)))
        return ms.value


class HostStep:
    """One decode step through the host-array form, marshalled once.  Fill `kv_len`, `node_offsets`, `parent` and
    `tokens` in place (int32, sized for the configuration's maxima), call `verify()`, read `accepted_len` and
    `accepted_tokens`; `compact()` enqueues the compaction of the bound layers."""

    def __init__(self, ver: "Verifier", q, kv, logits, attn_out, batch, layers, stream, parent=None, tokens=None):
        cfg = ver.cfg
        self._ver = ver
        self.kv_len = np.zeros(batch, dtype=np.int32)
        self.node_offsets = np.zeros(batch + 1, dtype=np.int32)
        # (a drafter's own output arrays can be bound instead: then the tree needs no copy at all)
        self.parent = np.zeros(cfg.max_batch * cfg.max_nodes, dtype=np.int32) if parent is None else parent
        self.tokens = np.zeros(cfg.max_batch * cfg.max_nodes, dtype=np.int32) if tokens is None else tokens
        for a in (self.parent, self.tokens):
            if a.dtype != np.int32 or not a.flags.c_contiguous:
                raise ValueError("parent and tokens must be contiguous int32 arrays")
        self.accepted_len = np.zeros(batch, dtype=np.int32)
        self.accepted_tokens = np.zeros((batch, ver.stride), dtype=np.int32)
        st = ver._stream(stream)
        self._kv = kv
        self._layers = (CbKvLayer * len(layers))(*layers) if layers else None
        self._keep = (q, logits, attn_out)
        self._verify_args = (ver.ctx, st, batch, q.data_ptr(), C.byref(self._kv), _ip(self.kv_len), _ip(self.node_offsets),
                             _ip(self.parent), _ip(self.tokens), logits.data_ptr(), attn_out.data_ptr(),
                             _ip(self.accepted_len), _ip(self.accepted_tokens))
        self._compact_args = (ver.ctx, st, len(layers), self._layers, None)
        self._verify_fn, self._compact_fn = ver.L.cb_verify_tree, ver.L.cb_compact_kv

    def verify(self):
        rc = self._verify_fn(*self._verify_args)
        if rc:
            self._ver._raise(rc)

    def compact(self):
        rc = self._compact_fn(*self._compact_args)
        if rc:
            self._ver._raise(rc)


# ----------------------------------------------------------------------------- host drafter (cacheback_drafter.h)
class DraftTable:
    """One leader -> follower cache table of the native drafter."""

    def __init__(self, ll: int, fl: int, lc: int, fc: int, frozen_from=None):
        """An empty table, or (``frozen_from`` = token sample) the frozen table built from a corpus sample."""
        self.L = load()
        self.ll, self.fl, self.lc, self.fc = ll, fl, lc, fc
        h = C.c_void_p()
        if frozen_from is None:
            rc = self.L.cbd_table_create(ll, fl, lc, fc, C.byref(h))
        else:
            a = _i32(frozen_from)
            rc = self.L.cbd_table_build_frozen(ll, fl, lc, fc, _ip(a), len(a), C.byref(h))
        if rc:
            raise CbError(rc, "cbd_table_create")
        self.h = h
        self._fol = (C.c_int32 * (fc * fl))()

    def close(self):
        if self.h:
            self.L.cbd_table_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def insert(self, leader, follower):
        a, b = _i32(leader), _i32(follower)
        if len(a) != self.ll or len(b) != self.fl:
            raise ValueError("leader/follower length mismatch")
        rc = self.L.cbd_table_insert(self.h, _ip(a), _ip(b))
        if rc:
            raise CbError(rc, "cbd_table_insert")

    def update(self, tokens, start: int = 0):
        a = _i32(tokens)
        rc = self.L.cbd_table_update(self.h, _ip(a), len(a), start)
        if rc:
            raise CbError(rc, "cbd_table_update")

    def query(self, leader, refresh: bool = True):
        a = _i32(leader)
        if len(a) != self.ll:
            raise ValueError("leader length mismatch")
        n = C.c_int32(0)
        rc = self.L.cbd_table_query(self.h, _ip(a), 1 if refresh else 0, self._fol, C.byref(n))
        if rc:
            raise CbError(rc, "cbd_table_query")
        return [tuple(self._fol[i * self.fl:(i + 1) * self.fl]) for i in range(n.value)]

    def freeze(self):
        self.L.cbd_table_freeze(self.h)
        return self

    def size(self):
        a, b = C.c_int64(0), C.c_int64(0)
        self.L.cbd_table_size(self.h, C.byref(a), C.byref(b))
        return a.value, b.value


class TreeGrower:
    """cbd_grow_tree with everything marshalled once: fixed tables, budget and output buffers.  `grow`
    returns views of its own buffers (valid until the next call)."""

    def __init__(self, tables, node_budget: int, depth_cap: int, crt: int = 0):
        self._fn = load().cbd_grow_tree
        self._tables = list(tables)
        self._hs = (C.c_void_p * len(tables))(*[t.h for t in tables])
        self._args = (len(tables),)
        self._tail = (node_budget, depth_cap, crt)
        self.parent = np.empty(node_budget, dtype=np.int32)
        self.token = np.empty(node_budget, dtype=np.int32)
        self.depth = np.empty(node_budget, dtype=np.int32)
        self._out = (_ip(self.parent), _ip(self.token), _ip(self.depth))
        self._n = C.c_int32(0)
        self._nref = C.byref(self._n)
        self._ctx_arr, self._ctx_ptr = None, None

    def grow(self, context: np.ndarray, n_ctx: int):
        """`context` is an int32 array whose first n_ctx entries are the text so far."""
        if context is not self._ctx_arr:
            if context.dtype != np.int32 or not context.flags.c_contiguous:
                raise ValueError("context must be a contiguous int32 array")
            self._ctx_arr, self._ctx_ptr = context, _ip(context)
        rc = self._fn(self._hs, self._args[0], self._ctx_ptr, n_ctx, *self._tail, *self._out, self._nref)
        if rc:
            raise CbError(rc, "cbd_grow_tree")
        n = self._n.value
        return self.parent[:n], self.token[:n], self.depth[:n]


def grow_tree(context, tables, node_budget: int, depth_cap: int, crt: int = 0):
    """Native tree growth; returns int32 arrays (parent, token, depth)."""
    L = load()
    ctx = _i32(context)
    hs = (C.c_void_p * len(tables))(*[t.h for t in tables])
    par = np.empty(node_budget, dtype=np.int32)
    tok = np.empty(node_budget, dtype=np.int32)
    dep = np.empty(node_budget, dtype=np.int32)
    n = C.c_int32(0)
    rc = L.cbd_grow_tree(hs, len(tables), _ip(ctx), len(ctx), node_budget, depth_cap, crt, _ip(par), _ip(tok), _ip(dep),
                         C.byref(n))
    if rc:
        raise CbError(rc, "cbd_grow_tree")
    return par[:n.value], tok[:n.value], dep[:n.value]


# ----------------------------------------------------------------------------- numpy <-> torch marshalling
def to_device(a: np.ndarray, dtype: str, device="cuda:0"):
    """numpy (float32, or uint16 bf16 bit patterns) -> torch tensor on the GPU, bit for bit."""
    import torch
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)


def to_host(t, dtype: str) -> np.ndarray:
    """torch tensor -> numpy (float32, or uint16 bf16 bit patterns), bit for bit."""
    import torch
    if dtype == "bf16":
        return t.detach().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.detach().cpu().numpy()


def config_for_case(case, max_splits: int = 0) -> CbConfig:
    n = np.diff(case.node_offsets)
    return make_config(case.Hq, case.Hkv, case.D, case.dtype, case.dtype, case.B, int(n.max()), case.max_depth,
                       case.V, case.block_size, max_splits)


class DeviceCase:
    """A workload's tensors uploaded to the GPU, plus its cache descriptor."""

    def __init__(self, case, device="cuda:0", layout: int = CB_LAYOUT_TOKEN_MAJOR):
        import torch
        self.case = case
        self.q = to_device(case.q, case.dtype, device)
        k, v = case.k, case.v
        if layout == CB_LAYOUT_HEAD_MAJOR:
            k, v = np.ascontiguousarray(k.swapaxes(1, 2)), np.ascontiguousarray(v.swapaxes(1, 2))
        self.k = to_device(k, case.dtype, device)
        self.v = to_device(v, case.dtype, device)
        self.logits = to_device(case.logits, case.dtype, device)
        self.block_table = None
        if case.block_size > 0:
            self.block_table = torch.from_numpy(np.ascontiguousarray(case.block_table, dtype=np.int32)).to(device)
        self.layout = layout
        self.kv = kv_layer(self.k, self.v, self.block_table, layout, paged=case.block_size > 0)
