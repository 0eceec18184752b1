"""ctypes binding of libls_stage.so: same names as include/ls_stage.h, marshalling only.

`Stage` below is a convenience holder for the device buffers the C ABI asks the caller
to own (weight slab, workspace, KV cache), allocated through PyTorch; every step of the
forward pass runs inside the library's HIP kernels.  There is no CPU fallback: if the
shared library is missing, importing this module raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np
# PyTorch ships its own HIP runtime (same SONAME as ROCm's).  It must be in the process
# before libls_stage.so is opened, so that the library binds to that one runtime and its
# streams, events and device pointers mean the same thing on both sides.
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libls_stage.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        "libls_stage.so is not built: run `python -m paper_2502_09922_amd.build` "
        "(hipcc --offload-arch=gfx950); there is no fallback path"
    )
lib = C.CDLL(LIB_PATH)

LS_ABI_VERSION = 1
LS_STATIC_SCRATCH_BYTES = 16 << 20
LS_DTYPE_F32, LS_DTYPE_BF16 = 0, 1
LS_BLOCK_EMBED = -1
LS_OP_NONE, LS_OP_NORM, LS_OP_GEMM_QKV = 0, 1, 2
LS_WS_QKV, LS_WS_ATTN, LS_WS_FFN = 1, 2, 3
LS_OP_ATTENTION, LS_OP_GEMM_O, LS_OP_GEMM_GATEUP, LS_OP_GEMM_DOWN = 4, 5, 6, 7
(LS_OK, LS_ERR_INVALID_ARG, LS_ERR_BLOCK_RANGE, LS_ERR_NOT_LOADED, LS_ERR_ALREADY_LOADED,
 LS_ERR_KV_OVERFLOW, LS_ERR_OOM, LS_ERR_HIP) = (0, -1, -2, -3, -4, -5, -6, -7)


class ls_cfg(C.Structure):
    _fields_ = [
        ("abi_version", C.c_uint32), ("dtype", C.c_uint32), ("n_layers_total", C.c_uint32),
        ("hidden", C.c_uint32), ("n_q_heads", C.c_uint32), ("n_kv_heads", C.c_uint32),
        ("head_dim", C.c_uint32), ("ffn", C.c_uint32), ("vocab", C.c_uint32),
        ("rms_eps", C.c_float), ("rope_base", C.c_float),
        ("max_batch", C.c_uint32), ("max_seq", C.c_uint32), ("max_tokens", C.c_uint32),
    ]


class ls_kv(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("seq_lens", C.c_void_p)]


class ls_microbatch(C.Structure):
    _fields_ = [
        ("in_", C.c_void_p), ("cu_seqlens_dev", C.c_void_p), ("cu_seqlens_host", C.POINTER(C.c_int32)),
        ("batch", C.c_int32), ("total_tokens", C.c_int32), ("max_ctx", C.c_int32),
        ("kv", C.POINTER(ls_kv)), ("handoff", C.POINTER(C.c_void_p)), ("out", C.c_void_p),
        ("logits_out", C.c_void_p),
    ]


_P = C.c_void_p
_SIGS = {
    "ls_block_bytes": (C.c_size_t, [C.POINTER(ls_cfg), C.c_int]),
    "ls_block_tensor_count": (C.c_int, [C.POINTER(ls_cfg), C.c_int]),
    "ls_block_tensor": (C.c_int, [C.POINTER(ls_cfg), C.c_int, C.c_int, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]),
    "ls_stage_slab_bytes": (C.c_size_t, [C.POINTER(ls_cfg), C.c_int, C.c_int]),
    "ls_stage_workspace_bytes": (C.c_size_t, [C.POINTER(ls_cfg), C.c_int, C.c_int]),
    "ls_stage_kv_bytes": (C.c_size_t, [C.POINTER(ls_cfg), C.c_int, C.c_int]),
    "ls_stage_create": (C.c_int, [C.POINTER(ls_cfg), C.c_int, C.c_int, _P, C.c_size_t, _P, C.c_size_t, C.POINTER(_P)]),
    "ls_stage_destroy": (None, [_P]),
    "ls_stage_block_bytes": (C.c_size_t, [_P, C.c_int]),
    "ls_stage_block_device_ptr": (_P, [_P, C.c_int]),
    "ls_stage_load_block": (C.c_int, [_P, _P, C.c_int, _P]),
    "ls_stage_load_layers": (C.c_int, [_P, _P, C.c_int, C.c_int, _P]),
    "ls_stage_adopt_block": (C.c_int, [_P, C.c_int, _P]),
    "ls_stage_reset_blocks": (C.c_int, [_P]),
    "ls_stage_prefill": (C.c_int, [_P, _P, _P, C.POINTER(C.c_int32), C.c_int, C.c_int, C.POINTER(ls_kv), _P, _P, _P]),
    "ls_stage_decode": (C.c_int, [_P, _P, C.c_int, C.c_int, C.POINTER(ls_kv), _P, _P, _P]),
    "ls_stage_decode_static": (C.c_int, [_P, _P, C.c_int, C.c_int, C.POINTER(ls_kv), _P, _P, _P]),
    "ls_stage_check_prefill": (C.c_int, [_P, C.POINTER(C.c_int32), C.c_int, C.c_int]),
    "ls_stage_check_decode": (C.c_int, [_P, C.c_int, C.c_int]),
    "ls_stage_set_profiling": (C.c_int, [_P, C.c_int]),
    "ls_stage_layer_times": (C.c_int, [_P, C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_float), C.c_int]),
    "ls_stage_block_times": (C.c_int, [_P, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_float)]),
    "ls_stage_pass_times": (C.c_int, [_P, C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(C.c_float)]),
    "ls_stage_probe": (C.c_int, [_P, C.c_int, C.c_int, C.c_int]),
    "ls_stage_probe_times": (C.c_int, [_P, C.POINTER(C.c_float), C.c_int, C.POINTER(C.c_int)]),
    "ls_stage_probe_is_kernel_exact": (C.c_int, [_P]),
    "ls_stage_workspace_region": (C.c_int, [_P, C.c_int, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]),
    "ls_stage_info": (C.c_int, [_P, C.POINTER(ls_cfg), C.POINTER(C.c_int), C.POINTER(C.c_int)]),
    "ls_pipeline_create": (C.c_int, [C.POINTER(_P), C.c_int, C.POINTER(_P)]),
    "ls_pipeline_destroy": (None, [_P]),
    "ls_pipeline_run": (C.c_int, [_P, C.c_int, C.POINTER(ls_microbatch), C.c_int, C.POINTER(_P)]),
    "ls_plan_chunk_span": (C.c_int, [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)]),
    "ls_plan_kway_order": (C.c_int, [C.c_int, C.c_int, C.c_int, C.POINTER(C.c_int32)]),
    "ls_plan_subgroup_sizes": (C.c_int, [C.c_int, C.c_int, C.POINTER(C.c_int32)]),
    "ls_plan_pipelines": (C.c_int, [C.POINTER(C.c_int32), C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int32),
                                    C.POINTER(C.c_int32), C.c_int, C.POINTER(C.c_int)]),
    "ls_plan_multicast_steps": (C.c_int, [C.c_int, C.c_int]),
    "ls_probe_read_gbps": (C.c_double, [C.c_void_p, C.c_size_t, C.c_int, C.c_void_p, C.c_void_p]),
    "ls_probe_mfma_tflops": (C.c_double, [C.c_int, C.c_int, C.c_void_p, C.c_void_p]),
    "ls_plan_multicast_schedule": (C.c_int, [C.c_int, C.c_int, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.c_int,
                                             C.POINTER(C.c_int)]),
    "ls_last_error": (C.c_char_p, []),
}
for _name, (_res, _args) in _SIGS.items():
    _fn = getattr(lib, _name)
    _fn.restype, _fn.argtypes = _res, _args
    globals()[_name] = _fn
EXPORTED = tuple(_SIGS)


class LsError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__("ls_status %d: %s" % (status, lib.ls_last_error().decode()))


def check(status: int) -> None:
    if status != LS_OK:
        raise LsError(status)


def make_cfg(shape, max_batch: int, max_seq: int, max_tokens: int) -> ls_cfg:
    """ls_cfg from an object with the decoder's hyper-parameters as attributes."""
    return ls_cfg(
        LS_ABI_VERSION, LS_DTYPE_F32 if shape.dtype == "f32" else LS_DTYPE_BF16, shape.n_layers_total,
        shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.ffn, shape.vocab,
        shape.rms_eps, shape.rope_base, max_batch, max_seq, max_tokens,
    )


def pack_block(cfg: ls_cfg, layer: int, tensors: Sequence[np.ndarray], out: Optional[np.ndarray] = None) -> np.ndarray:
    """Lay the tensors of one block (in block order) into one contiguous uint8 buffer
    at the offsets ls_block_tensor reports.  Padding bytes are zero."""
    n = lib.ls_block_tensor_count(C.byref(cfg), layer)
    if n == 0 or n != len(tensors):
        raise ValueError("block %d holds %d tensors, got %d" % (layer, n, len(tensors)))
    total = lib.ls_block_bytes(C.byref(cfg), layer)
    buf = np.zeros(total, np.uint8) if out is None else out
    assert buf.dtype == np.uint8 and buf.size == total
    off, nb = C.c_size_t(), C.c_size_t()
    for i, t in enumerate(tensors):
        check(lib.ls_block_tensor(C.byref(cfg), layer, i, C.byref(off), C.byref(nb)))
        raw = np.ascontiguousarray(t).view(np.uint8).reshape(-1)
        if raw.size != nb.value:
            raise ValueError("tensor %d of block %d has %d bytes, format says %d" % (i, layer, raw.size, nb.value))
        buf[off.value : off.value + nb.value] = raw
    return buf


class Stage:
    """One ls_stage plus the device buffers it needs, allocated with PyTorch."""

    def __init__(self, shape, layer_lo: int, layer_hi: int, max_batch: int, max_seq: int, max_tokens: int, device="cuda:0"):
        self.torch = torch
        self.shape, self.lo, self.hi = shape, layer_lo, layer_hi
        self.cfg = make_cfg(shape, max_batch, max_seq, max_tokens)
        self.device = torch.device(device)
        self.first = shape.vocab > 0 and layer_lo == 0
        self.last = shape.vocab > 0 and layer_hi == shape.n_layers_total
        self.tdtype = torch.float32 if shape.dtype == "f32" else torch.bfloat16
        cfgp = C.byref(self.cfg)
        sb = lib.ls_stage_slab_bytes(cfgp, layer_lo, layer_hi)
        wb = lib.ls_stage_workspace_bytes(cfgp, layer_lo, layer_hi)
        kb = lib.ls_stage_kv_bytes(cfgp, layer_lo, layer_hi)
        if not (sb and wb and kb):
            raise ValueError("invalid shape or layer span")
        with torch.cuda.device(self.device):
            self.slab = torch.empty(sb, dtype=torch.uint8, device=self.device)
            self.workspace = torch.empty(wb, dtype=torch.uint8, device=self.device)
            self.k = torch.zeros(kb, dtype=torch.uint8, device=self.device)
            self.v = torch.zeros(kb, dtype=torch.uint8, device=self.device)
            self.seq_lens = torch.zeros(max_batch, dtype=torch.int32, device=self.device)
            self.kv = ls_kv(self.k.data_ptr(), self.v.data_ptr(), self.seq_lens.data_ptr())
            h = _P()
            check(lib.ls_stage_create(cfgp, layer_lo, layer_hi, self.slab.data_ptr(), sb,
                                      self.workspace.data_ptr(), wb, C.byref(h)))
        self.handle = h
        self._pinned: Dict[int, object] = {}

    def close(self):
        if getattr(self, "handle", None):
            self.torch.cuda.synchronize(self.device)
            lib.ls_stage_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def block_ids(self):
        ids = [LS_BLOCK_EMBED] if self.first else []
        ids += list(range(self.lo, self.hi))
        if self.last:
            ids.append(self.shape.n_layers_total)
        return ids

    @staticmethod
    def _stream_ptr(stream) -> int:
        return 0 if stream is None else stream.cuda_stream

    def stage_host_block(self, layer: int, packed: np.ndarray):
        """Copy a packed block into pinned host memory (kept alive by the stage)."""
        t = self.torch.empty(packed.size, dtype=self.torch.uint8, pin_memory=True)
        t.numpy()[:] = packed
        self._pinned[layer] = t
        return t

    def load_block(self, layer: int, host, stream=None):
        """host: pinned torch uint8 tensor or numpy uint8 array holding the packed block."""
        ptr = host.data_ptr() if hasattr(host, "data_ptr") else host.ctypes.data
        check(lib.ls_stage_load_block(self.handle, ptr, layer, self._stream_ptr(stream)))

    def load_layers(self, first: int, last: int, host, stream=None):
        """host: pinned uint8 tensor holding the packed blocks of layers first..last back to back."""
        check(lib.ls_stage_load_layers(self.handle, host.data_ptr(), first, last, self._stream_ptr(stream)))

    def adopt_block(self, layer: int, stream=None):
        """The packed bytes of block `layer` are already in the slab (written on `stream`)."""
        check(lib.ls_stage_adopt_block(self.handle, layer, self._stream_ptr(stream)))

    def block_view(self, layer: int):
        """uint8 view of block `layer` inside the slab."""
        ptr = lib.ls_stage_block_device_ptr(self.handle, layer)
        off = ptr - self.slab.data_ptr()
        return self.slab[off : off + lib.ls_stage_block_bytes(self.handle, layer)]

    def block_times(self, layer: int):
        a, b = C.c_float(), C.c_float()
        check(lib.ls_stage_block_times(self.handle, layer, C.byref(a), C.byref(b)))
        return a.value, b.value

    def pass_times(self):
        a, b, c = C.c_float(), C.c_float(), C.c_float()
        check(lib.ls_stage_pass_times(self.handle, C.byref(a), C.byref(b), C.byref(c)))
        return a.value, b.value, c.value

    def reset_blocks(self):
        check(lib.ls_stage_reset_blocks(self.handle))

    def prefill(self, inp, lengths: Sequence[int], stream=None, want_logits=False):
        torch = self.torch
        cu = np.zeros(len(lengths) + 1, np.int32)
        cu[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
        total, batch = int(cu[-1]), len(lengths)
        cu_dev = torch.from_numpy(cu).to(self.device)
        out = (torch.empty(batch, dtype=torch.int32, device=self.device) if self.last
               else torch.empty(total, self.shape.hidden, dtype=self.tdtype, device=self.device))
        logits = (torch.empty(batch, self.shape.vocab, dtype=torch.float32, device=self.device)
                  if (want_logits and self.last) else None)
        check(lib.ls_stage_prefill(
            self.handle, inp.data_ptr(), cu_dev.data_ptr(), cu.ctypes.data_as(C.POINTER(C.c_int32)), batch, total,
            C.byref(self.kv), out.data_ptr(), logits.data_ptr() if logits is not None else None,
            self._stream_ptr(stream)))
        self._keep = (cu_dev, inp)
        return (out, logits) if want_logits else out

    def decode(self, inp, batch: int, max_ctx: int, stream=None, want_logits=False, out=None, static=False):
        """static=True: ls_stage_decode_static (partial results in the library's static array)."""
        torch = self.torch
        fn = lib.ls_stage_decode_static if static else lib.ls_stage_decode
        if out is None:
            out = (torch.empty(batch, dtype=torch.int32, device=self.device) if self.last
                   else torch.empty(batch, self.shape.hidden, dtype=self.tdtype, device=self.device))
        logits = (torch.empty(batch, self.shape.vocab, dtype=torch.float32, device=self.device)
                  if (want_logits and self.last) else None)
        check(fn(
            self.handle, inp.data_ptr(), batch, max_ctx, C.byref(self.kv), out.data_ptr(),
            logits.data_ptr() if logits is not None else None, self._stream_ptr(stream)))
        return (out, logits) if want_logits else out

    def workspace_region(self, which: int, rows: int):
        """[rows, columns] view of an intermediate result inside the workspace (see ls_stage.h)."""
        off, nb = C.c_size_t(), C.c_size_t()
        check(lib.ls_stage_workspace_region(self.handle, which, C.byref(off), C.byref(nb)))
        esz = 4 if self.shape.dtype == "f32" else 2
        cols = nb.value // (self.cfg.max_tokens * esz)
        flat = self.workspace[off.value : off.value + rows * cols * esz].view(self.tdtype)
        return flat.view(rows, cols)

    def probe(self, op: int, layer: int = 0, phase: int = 1):
        check(lib.ls_stage_probe(self.handle, op, layer, phase))

    def probe_times(self):
        arr, n = (C.c_float * 512)(), C.c_int()
        check(lib.ls_stage_probe_times(self.handle, arr, 512, C.byref(n)))
        return list(arr[: n.value])

    def probe_is_kernel_exact(self) -> bool:
        return bool(lib.ls_stage_probe_is_kernel_exact(self.handle))

    def set_profiling(self, on: bool):
        check(lib.ls_stage_set_profiling(self.handle, int(on)))

    def layer_times(self, want_copy=True):
        n = self.hi - self.lo
        arrs = [(C.c_float * n)() for _ in range(4)]
        a = [arrs[0] if want_copy else None, arrs[1], arrs[2] if want_copy else None, arrs[3]]
        check(lib.ls_stage_layer_times(self.handle, a[0], a[1], a[2], a[3], n))
        return {
            "copy_ms": list(arrs[0]) if want_copy else None,
            "compute_ms": list(arrs[1]),
            "copy_end_ms": list(arrs[2]) if want_copy else None,
            "compute_end_ms": list(arrs[3]),
        }


class MicroBatch:
    """Device buffers of one micro-batch of a Pipeline: a KV cache per stage, hand-off
    buffers between the stages, the output; allocated with PyTorch."""

    def __init__(self, pipe: "Pipeline", max_rows: int):
        torch = pipe.torch
        st0 = pipe.stages[0]
        self.caches = []
        for st in pipe.stages:
            kb = lib.ls_stage_kv_bytes(C.byref(st.cfg), st.lo, st.hi)
            k = torch.zeros(kb, dtype=torch.uint8, device=st.device)
            v = torch.zeros(kb, dtype=torch.uint8, device=st.device)
            sl = torch.zeros(st.cfg.max_batch, dtype=torch.int32, device=st.device)
            self.caches.append((k, v, sl))
        self.kv = (ls_kv * len(pipe.stages))(*[ls_kv(k.data_ptr(), v.data_ptr(), sl.data_ptr()) for k, v, sl in self.caches])
        self.handoff_t = [torch.empty(max_rows, st0.shape.hidden, dtype=st0.tdtype, device=st0.device)
                          for _ in pipe.stages[1:]]
        self.handoff = (C.c_void_p * max(1, len(self.handoff_t)))(*[t.data_ptr() for t in self.handoff_t])
        self.max_rows = max_rows


class Pipeline:
    """ls_pipeline over Stage objects, one torch stream per stage."""

    def __init__(self, stages):
        self.torch = torch
        self.stages = list(stages)
        hs = (_P * len(self.stages))(*[s.handle for s in self.stages])
        h = _P()
        check(lib.ls_pipeline_create(hs, len(self.stages), C.byref(h)))
        self.handle = h
        self.streams = [torch.cuda.Stream(device=s.device) for s in self.stages]
        self._stream_ptrs = (_P * len(self.stages))(*[s.cuda_stream for s in self.streams])
        self._keep = []

    def close(self):
        if getattr(self, "handle", None):
            self.torch.cuda.synchronize()
            lib.ls_pipeline_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _out(self, rows, batch):
        last = self.stages[-1]
        if last.last:
            return self.torch.empty(batch, dtype=self.torch.int32, device=last.device)
        return self.torch.empty(rows, last.shape.hidden, dtype=last.tdtype, device=last.device)

    def run(self, phase: int, mbs: Sequence[MicroBatch], inputs, lengths=None, max_ctx=None, want_logits=False):
        """phase 0: lengths[m] = prompt lengths of micro-batch m; phase 1: max_ctx[m] bounds its
        cached lengths and its batch is len(inputs[m]).  Returns the outputs (and logits)."""
        torch = self.torch
        arr = (ls_microbatch * len(mbs))()
        outs, logits, keep = [], [], []
        last = self.stages[-1]
        for m, mb in enumerate(mbs):
            if phase == 0:
                cu = np.zeros(len(lengths[m]) + 1, np.int32)
                cu[1:] = np.cumsum(np.asarray(lengths[m], dtype=np.int64))
                batch, rows = len(lengths[m]), int(cu[-1])
                cu_dev = torch.from_numpy(cu).to(last.device)
                keep += [cu, cu_dev]
                arr[m].cu_seqlens_dev = cu_dev.data_ptr()
                arr[m].cu_seqlens_host = cu.ctypes.data_as(C.POINTER(C.c_int32))
                arr[m].total_tokens = rows
            else:
                batch = rows = int(inputs[m].shape[0])
                arr[m].max_ctx = int(max_ctx[m])
            if rows > mb.max_rows:
                raise ValueError("micro-batch %d has %d rows, its hand-off buffers hold %d" % (m, rows, mb.max_rows))
            out = self._out(rows, batch)
            lg = (torch.empty(batch, last.shape.vocab, dtype=torch.float32, device=last.device)
                  if (want_logits and last.last) else None)
            arr[m].in_ = inputs[m].data_ptr()
            arr[m].batch = batch
            arr[m].kv = mb.kv
            arr[m].handoff = mb.handoff
            arr[m].out = out.data_ptr()
            arr[m].logits_out = lg.data_ptr() if lg is not None else None
            outs.append(out)
            logits.append(lg)
        # inputs were produced on the current stream or, when a step feeds on the previous
        # one's tokens, on the last stage's stream: the stage streams wait for both
        cur = torch.cuda.current_stream()
        for s in self.streams:
            s.wait_stream(cur)
        self.streams[0].wait_stream(self.streams[-1])
        # buffers allocated on the current stream are used on the stage streams
        for t in outs + [l for l in logits if l is not None]:
            t.record_stream(self.streams[-1])
        for t in keep:
            if hasattr(t, "record_stream"):
                for s in self.streams:
                    t.record_stream(s)
        for t in inputs:
            t.record_stream(self.streams[0])
        check(lib.ls_pipeline_run(self.handle, phase, arr, len(mbs), self._stream_ptrs))
        self._keep = [keep, list(inputs), outs, logits]
        return (outs, logits) if want_logits else outs

    def join(self):
        """Order the current torch stream after everything the pipeline has enqueued."""
        cur = self.torch.cuda.current_stream()
        for s in self.streams:
            cur.wait_stream(s)
