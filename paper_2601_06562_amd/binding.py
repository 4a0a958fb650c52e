"""ctypes binding of libmosaic.so -- argument marshalling only.

Every step of the path runs in the HIP kernels behind the C ABI declared in
``include/mosaic.h``; the functions here have the same names and only turn torch tensors
into device pointers.  There is no CPU or PyTorch fallback: if the library is missing,
loading raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmosaic.so")

MOSAIC_OK = 0
MOSAIC_ERR_INVALID_ARG = -1
MOSAIC_ERR_UNSUPPORTED_SHAPE = -2
MOSAIC_ERR_WORKSPACE_TOO_SMALL = -3
MOSAIC_ERR_HIP = -4
ROW_TILE = 256
VOCAB_TILE = 256
K_TILE = 64
PLAN_GENERAL_KERNEL = 1   # plan.flags bit: force the general 8-wave kernel
PLAN_SAMPLING = 2         # plan.flags bit: sized for a sampling step (20 bytes per partial)
STATIC_WORKSPACE_BYTES = 4 << 20   # the fixed array behind mosaic_masked_logits_reduce_static
SYNC_BYTES = 1024                  # round counters at the end of every workspace

EXPORTS = (
    "mosaic_status_string", "mosaic_plan_workspace", "mosaic_compact_scratch_bytes", "mosaic_mask_compact",
    "mosaic_masked_logits_reduce", "mosaic_masked_logits_reduce_static", "mosaic_masked_logits_kernel_name",
    "mosaic_sample_workspace_bytes",
    "mosaic_masked_logits_sample",
    "mosaic_unmask_topn", "mosaic_shift_indices", "mosaic_mfma_probe_flops", "mosaic_mfma_probe", "mosaic_version",
    "mosaic_vmm_create", "mosaic_vmm_resize", "mosaic_vmm_ptr", "mosaic_vmm_committed_bytes",
    "mosaic_vmm_reserved_bytes", "mosaic_vmm_granularity", "mosaic_vmm_kept_contents", "mosaic_vmm_last_error",
    "mosaic_vmm_destroy",
)
GRAPH_EXPORTS = (
    "mosaic_graph_create", "mosaic_graph_destroy", "mosaic_graph_add_dim", "mosaic_graph_add_chunk_param",
    "mosaic_graph_add_tensor", "mosaic_graph_add_op", "mosaic_graph_add_alias", "mosaic_graph_add_barrier",
    "mosaic_graph_plan", "mosaic_graph_search",
)


class MosaicPlacement(ctypes.Structure):
    _fields_ = [("tensor", ctypes.c_int32), ("iteration", ctypes.c_int32), ("first_step", ctypes.c_int32),
                ("last_step", ctypes.c_int32), ("offset", ctypes.c_int64), ("bytes", ctypes.c_int64)]


class MosaicPlanSummary(ctypes.Structure):
    _fields_ = [("peak_bytes", ctypes.c_int64), ("num_blocks", ctypes.c_int64), ("num_steps", ctypes.c_int32),
                ("peak_block", ctypes.c_int32), ("peak_op", ctypes.c_int32), ("peak_chunk", ctypes.c_int32)]


class MosaicPlan(ctypes.Structure):
    _fields_ = [
        ("workspace_bytes", ctypes.c_int64),
        ("num_chunks", ctypes.c_int32),
        ("rows_per_chunk", ctypes.c_int32),
        ("vocab_splits", ctypes.c_int32),
        ("tile_panel", ctypes.c_int32),
        ("grid", ctypes.c_int32),
        ("flags", ctypes.c_int32),
    ]

    def __repr__(self):
        return ("MosaicPlan(workspace_bytes=%d, num_chunks=%d, rows_per_chunk=%d, vocab_splits=%d, tile_panel=%d, "
                "grid=%d)" % (self.workspace_bytes, self.num_chunks, self.rows_per_chunk, self.vocab_splits,
                              self.tile_panel, self.grid))


class MosaicError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_lib = None


def lib():
    """The loaded libmosaic.so.  Raises if it has not been built (run __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is missing: build it with `python -m paper_2601_06562_amd.build` "
                                    "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        p, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        L.mosaic_status_string.restype = ctypes.c_char_p
        L.mosaic_status_string.argtypes = [ctypes.c_int]
        L.mosaic_version.restype = ctypes.c_int
        L.mosaic_version.argtypes = []
        L.mosaic_plan_workspace.restype = ctypes.c_int
        L.mosaic_plan_workspace.argtypes = [i64, i64, i32, i32, i64, i32, i32, ctypes.POINTER(MosaicPlan)]
        L.mosaic_compact_scratch_bytes.restype = i64
        L.mosaic_compact_scratch_bytes.argtypes = [i64]
        L.mosaic_mask_compact.restype = ctypes.c_int
        L.mosaic_mask_compact.argtypes = [p, i64, p, p, p, i64, p]
        L.mosaic_masked_logits_reduce.restype = ctypes.c_int
        L.mosaic_masked_logits_reduce.argtypes = [p, i64, i32, i64, p, i32, p, p, i64, p, p, p,
                                                  ctypes.POINTER(MosaicPlan), p, i64, p]
        L.mosaic_masked_logits_reduce_static.restype = ctypes.c_int
        L.mosaic_masked_logits_reduce_static.argtypes = [p, i64, i32, i64, p, i32, p, p, i64, p, p, p,
                                                         ctypes.POINTER(MosaicPlan), p]
        L.mosaic_masked_logits_kernel_name.restype = ctypes.c_char_p
        L.mosaic_masked_logits_kernel_name.argtypes = [i64, i32, i64, i32, ctypes.POINTER(MosaicPlan), i32]
        L.mosaic_sample_workspace_bytes.restype = i64
        L.mosaic_sample_workspace_bytes.argtypes = [ctypes.POINTER(MosaicPlan)]
        L.mosaic_masked_logits_sample.restype = ctypes.c_int
        L.mosaic_masked_logits_sample.argtypes = [p, i64, i32, i64, p, i32, p, p, p, i64, ctypes.c_float, ctypes.c_uint64,
                                                  p, p, p, ctypes.POINTER(MosaicPlan), p, i64, p]
        L.mosaic_unmask_topn.restype = ctypes.c_int
        L.mosaic_unmask_topn.argtypes = [p, p, p, p, i64, p, i32, p, p, p, i64, p]
        L.mosaic_shift_indices.restype = ctypes.c_int
        L.mosaic_shift_indices.argtypes = [p, p, i64, p, i32, p, p]
        L.mosaic_mfma_probe_flops.restype = i64
        L.mosaic_mfma_probe_flops.argtypes = [i32, i32]
        L.mosaic_mfma_probe.restype = ctypes.c_int
        L.mosaic_mfma_probe.argtypes = [p, p, i32, i32, p]
        L.mosaic_vmm_create.restype = ctypes.c_int
        L.mosaic_vmm_create.argtypes = [ctypes.c_int, i64, ctypes.POINTER(ctypes.c_void_p)]
        L.mosaic_vmm_resize.restype = ctypes.c_int
        L.mosaic_vmm_resize.argtypes = [p, i64]
        L.mosaic_vmm_ptr.restype = p
        L.mosaic_vmm_ptr.argtypes = [p]
        for name in ("mosaic_vmm_committed_bytes", "mosaic_vmm_reserved_bytes", "mosaic_vmm_granularity"):
            getattr(L, name).restype = i64
            getattr(L, name).argtypes = [p]
        L.mosaic_vmm_kept_contents.restype = ctypes.c_int
        L.mosaic_vmm_kept_contents.argtypes = [p]
        L.mosaic_vmm_last_error.restype = ctypes.c_char_p
        L.mosaic_vmm_last_error.argtypes = [p, ctypes.POINTER(ctypes.c_int)]
        L.mosaic_vmm_destroy.restype = ctypes.c_int
        L.mosaic_vmm_destroy.argtypes = [p]
        L.mosaic_graph_create.restype = p
        L.mosaic_graph_create.argtypes = []
        L.mosaic_graph_destroy.restype = None
        L.mosaic_graph_destroy.argtypes = [p]
        L.mosaic_graph_add_dim.restype = ctypes.c_int
        L.mosaic_graph_add_dim.argtypes = [p, ctypes.c_char_p]
        L.mosaic_graph_add_chunk_param.restype = ctypes.c_int
        L.mosaic_graph_add_chunk_param.argtypes = [p, ctypes.c_char_p, ctypes.c_int]
        L.mosaic_graph_add_tensor.restype = ctypes.c_int
        L.mosaic_graph_add_tensor.argtypes = [p, ctypes.c_char_p, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int]
        L.mosaic_graph_add_op.restype = ctypes.c_int
        L.mosaic_graph_add_op.argtypes = [p, ctypes.c_char_p, p, ctypes.c_int, p, ctypes.c_int, ctypes.c_int]
        L.mosaic_graph_add_alias.restype = ctypes.c_int
        L.mosaic_graph_add_alias.argtypes = [p, ctypes.c_int, ctypes.c_int]
        L.mosaic_graph_add_barrier.restype = ctypes.c_int
        L.mosaic_graph_add_barrier.argtypes = [p, ctypes.c_int, ctypes.c_int]
        L.mosaic_graph_plan.restype = ctypes.c_int
        L.mosaic_graph_plan.argtypes = [p, p, ctypes.c_int, p, ctypes.c_int, p, i64, ctypes.POINTER(MosaicPlanSummary)]
        L.mosaic_graph_search.restype = ctypes.c_int
        L.mosaic_graph_search.argtypes = [p, p, ctypes.c_int, i64, p, ctypes.c_int, ctypes.POINTER(MosaicPlanSummary), p]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().mosaic_status_string(int(status)).decode()


def _check(status, where):
    if status != MOSAIC_OK:
        raise MosaicError(status, where)


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev_ptr(t, name, dtype=None):
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda:
        raise ValueError(f"{name} must live in device memory")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    return ctypes.c_void_p(t.data_ptr())


def _workspace_args(workspace):
    """(pointer, bytes) of a workspace given as a device tensor or as a VmmWorkspace (its mapped prefix)."""
    if workspace is None:
        return ctypes.c_void_p(0), 0
    if isinstance(workspace, VmmWorkspace):
        return ctypes.c_void_p(workspace.ptr), workspace.committed_bytes
    return _dev_ptr(workspace, "workspace"), workspace.numel() * workspace.element_size()


def mosaic_plan_workspace(T, max_rows, d, V, budget_bytes=0, num_cus=0, sampling=False) -> MosaicPlan:
    plan = MosaicPlan()
    _check(lib().mosaic_plan_workspace(T, max_rows, d, V, budget_bytes, num_cus, int(sampling), ctypes.byref(plan)),
           "mosaic_plan_workspace")
    return plan


def mosaic_compact_scratch_bytes(T) -> int:
    return int(lib().mosaic_compact_scratch_bytes(T))


def mosaic_mask_compact(mask, out_idx, out_count, scratch, stream=None):
    """mask uint8[T] -> out_idx int32[>=max(T,1)] (first M written), out_count int32[1]; all device tensors."""
    T = mask.numel()
    if T and not mask.is_contiguous():
        raise ValueError("mask must be contiguous")
    _check(lib().mosaic_mask_compact(_dev_ptr(mask, "mask", torch.uint8) if T else ctypes.c_void_p(0), T,
                                     _dev_ptr(out_idx, "out_idx", torch.int32),
                                     _dev_ptr(out_count, "out_count", torch.int32), _dev_ptr(scratch, "scratch"),
                                     scratch.numel() * scratch.element_size(), _stream_ptr(stream)),
           "mosaic_mask_compact")


def mosaic_masked_logits_reduce(hidden, w, idx, count, max_rows, out_token, out_conf, out_lse, plan, workspace,
                                stream=None):
    """hidden bf16[T,d] (row stride >= d), w bf16[V,d], idx int32, count int32[1] -> out_* (device tensors)."""
    T, d = hidden.shape
    V, d2 = w.shape
    if d != d2:
        raise ValueError("hidden and w disagree on d")
    if hidden.stride(1) != 1 or not w.is_contiguous():
        raise ValueError("hidden rows and w must be dense along d")
    ld_h = hidden.stride(0) if T > 1 else d
    _check(lib().mosaic_masked_logits_reduce(
        _dev_ptr(hidden, "hidden", torch.bfloat16), T, d, ld_h, _dev_ptr(w, "w", torch.bfloat16), V,
        _dev_ptr(idx, "idx", torch.int32), _dev_ptr(count, "count", torch.int32), max_rows,
        _dev_ptr(out_token, "out_token", torch.int32), _dev_ptr(out_conf, "out_conf", torch.float32),
        _dev_ptr(out_lse, "out_lse", torch.float32), ctypes.byref(plan), *_workspace_args(workspace),
        _stream_ptr(stream)),
        "mosaic_masked_logits_reduce")


def mosaic_masked_logits_reduce_static(hidden, w, idx, count, max_rows, out_token, out_conf, out_lse, plan, stream=None):
    """mosaic_masked_logits_reduce on the library's own fixed workspace (allocates nothing)."""
    T, d = hidden.shape
    V, d2 = w.shape
    if d != d2:
        raise ValueError("hidden and w disagree on d")
    if hidden.stride(1) != 1 or not w.is_contiguous():
        raise ValueError("hidden rows and w must be dense along d")
    ld_h = hidden.stride(0) if T > 1 else d
    _check(lib().mosaic_masked_logits_reduce_static(
        _dev_ptr(hidden, "hidden", torch.bfloat16), T, d, ld_h, _dev_ptr(w, "w", torch.bfloat16), V,
        _dev_ptr(idx, "idx", torch.int32), _dev_ptr(count, "count", torch.int32), max_rows,
        _dev_ptr(out_token, "out_token", torch.int32), _dev_ptr(out_conf, "out_conf", torch.float32),
        _dev_ptr(out_lse, "out_lse", torch.float32), ctypes.byref(plan), _stream_ptr(stream)),
        "mosaic_masked_logits_reduce_static")


def mosaic_masked_logits_kernel_name(T, d, ld_h, V, plan, sampling=False) -> str:
    """The kernel(s) the fused pass launches for these sizes and this plan (for reports)."""
    return lib().mosaic_masked_logits_kernel_name(T, d, ld_h, V, ctypes.byref(plan), int(sampling)).decode()


def mosaic_sample_workspace_bytes(plan) -> int:
    """Workspace bytes mosaic_masked_logits_sample needs for this plan at temperature > 0."""
    return int(lib().mosaic_sample_workspace_bytes(ctypes.byref(plan)))


def mosaic_masked_logits_sample(hidden, w, idx, count, max_rows, temperature, seed, out_token, out_conf, out_lse, plan,
                                workspace, stream=None, noise_idx=None):
    """As mosaic_masked_logits_reduce, with Gumbel-max sampling at `temperature` from the 64-bit `seed`;
    noise_idx (int32 device tensor or None) names the position each row predicts when idx is a shifted list."""
    T, d = hidden.shape
    V, d2 = w.shape
    if d != d2:
        raise ValueError("hidden and w disagree on d")
    if hidden.stride(1) != 1 or not w.is_contiguous():
        raise ValueError("hidden rows and w must be dense along d")
    ld_h = hidden.stride(0) if T > 1 else d
    _check(lib().mosaic_masked_logits_sample(
        _dev_ptr(hidden, "hidden", torch.bfloat16), T, d, ld_h, _dev_ptr(w, "w", torch.bfloat16), V,
        _dev_ptr(idx, "idx", torch.int32), _dev_ptr(noise_idx, "noise_idx", torch.int32),
        _dev_ptr(count, "count", torch.int32), max_rows, float(temperature), int(seed) & 0xFFFFFFFFFFFFFFFF,
        _dev_ptr(out_token, "out_token", torch.int32), _dev_ptr(out_conf, "out_conf", torch.float32),
        _dev_ptr(out_lse, "out_lse", torch.float32), ctypes.byref(plan), *_workspace_args(workspace),
        _stream_ptr(stream)),
        "mosaic_masked_logits_sample")


def mosaic_unmask_topn(conf, token, idx, count, max_rows, seq_starts, n_per_seq, tokens, mask, stream=None):
    """Per sequence, write the tokens of the n highest-confidence masked rows and clear their mask bytes."""
    _check(lib().mosaic_unmask_topn(
        _dev_ptr(conf, "conf", torch.float32), _dev_ptr(token, "token", torch.int32), _dev_ptr(idx, "idx", torch.int32),
        _dev_ptr(count, "count", torch.int32), max_rows, _dev_ptr(seq_starts, "seq_starts", torch.int32),
        n_per_seq.numel(), _dev_ptr(n_per_seq, "n_per_seq", torch.int32), _dev_ptr(tokens, "tokens", torch.int32),
        _dev_ptr(mask, "mask", torch.uint8), mask.numel(), _stream_ptr(stream)), "mosaic_unmask_topn")


def mosaic_shift_indices(idx, count, max_rows, seq_starts, out_gather, stream=None):
    """out_gather[j] = idx[j] - 1, except at the first position of a sequence (device tensors)."""
    _check(lib().mosaic_shift_indices(
        _dev_ptr(idx, "idx", torch.int32), _dev_ptr(count, "count", torch.int32), max_rows,
        _dev_ptr(seq_starts, "seq_starts", torch.int32), seq_starts.numel() - 1,
        _dev_ptr(out_gather, "out_gather", torch.int32), _stream_ptr(stream)), "mosaic_shift_indices")


def mosaic_mfma_probe(operands, sink, iters, num_wgs, stream=None) -> int:
    """Enqueue the register-only MFMA loop (a measurement aid); returns the flops of the launch."""
    if operands.numel() * operands.element_size() < 65536 or sink.numel() < 65536:
        raise ValueError("operands must hold 64 KiB, sink 65536 floats")
    _check(lib().mosaic_mfma_probe(_dev_ptr(operands, "operands", torch.bfloat16), _dev_ptr(sink, "sink", torch.float32),
                                   int(iters), int(num_wgs), _stream_ptr(stream)), "mosaic_mfma_probe")
    return int(lib().mosaic_mfma_probe_flops(int(iters), int(num_wgs)))


class VmmWorkspace:
    """A reserved virtual range whose mapped prefix follows the planned peak (mosaic_vmm_*)."""

    def __init__(self, reserve_bytes, device=0):
        h = ctypes.c_void_p()
        _check(lib().mosaic_vmm_create(int(device), int(reserve_bytes), ctypes.byref(h)), "mosaic_vmm_create")
        self._h = h

    def resize(self, nbytes):
        rc = lib().mosaic_vmm_resize(self._h, int(nbytes))
        if rc == MOSAIC_ERR_HIP:
            code = ctypes.c_int(0)
            call = lib().mosaic_vmm_last_error(self._h, ctypes.byref(code)).decode()
            raise MosaicError(rc, f"mosaic_vmm_resize [{call} -> hipError {code.value}]")
        _check(rc, "mosaic_vmm_resize")

    @property
    def ptr(self) -> int:
        return int(lib().mosaic_vmm_ptr(self._h) or 0)

    @property
    def committed_bytes(self) -> int:
        return int(lib().mosaic_vmm_committed_bytes(self._h))

    @property
    def reserved_bytes(self) -> int:
        return int(lib().mosaic_vmm_reserved_bytes(self._h))

    @property
    def granularity(self) -> int:
        return int(lib().mosaic_vmm_granularity(self._h))

    @property
    def kept_contents(self) -> int:
        """Nonzero if the last resize that changed the size kept what the range held (growth in place): 1 or 2,
        by which of its two access calls the driver accepted."""
        return int(lib().mosaic_vmm_kept_contents(self._h))

    def tensor(self, offset, count, dtype):
        """A torch view of `count` elements of `dtype` at byte `offset` of the mapped prefix (no copy, no ownership:
        it must not be used after a resize that changes the mapping)."""
        nbytes = int(count) * torch.empty((), dtype=dtype).element_size()
        if offset < 0 or offset + nbytes > self.committed_bytes:
            raise ValueError("slice lies outside the mapped prefix of the range")

        class _Raw:
            pass
        raw = _Raw()
        raw.__cuda_array_interface__ = {"shape": (max(nbytes, 1),), "typestr": "|u1",
                                        "data": (self.ptr + int(offset), False), "version": 2}
        return torch.as_tensor(raw, device="cuda")[:nbytes].view(dtype)

    def close(self):
        h, self._h = getattr(self, "_h", None), None
        if h:
            _check(lib().mosaic_vmm_destroy(h), "mosaic_vmm_destroy")

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class GraphTemplate:
    """The graph registrar behind the C ABI (mosaic_graph_*): same primitive names, marshalling only."""
    NONE = -1

    def __init__(self):
        self._g = lib().mosaic_graph_create()
        if not self._g:
            raise MemoryError("mosaic_graph_create")
        self.n_dims = 0
        self.n_chunks = 0

    def __del__(self):
        g, self._g = getattr(self, "_g", None), None
        if g:
            lib().mosaic_graph_destroy(g)

    def _id(self, rc, where):
        if rc < 0:
            raise MosaicError(rc, where)
        return rc

    def add_dim(self, name):
        rc = self._id(lib().mosaic_graph_add_dim(self._g, name.encode()), "mosaic_graph_add_dim")
        self.n_dims += 1
        return rc

    def add_chunk_param(self, name, dim):
        rc = self._id(lib().mosaic_graph_add_chunk_param(self._g, name.encode(), dim), "mosaic_graph_add_chunk_param")
        self.n_chunks += 1
        return rc

    def add_tensor(self, name, bytes_per_row, dim=-1, chunk=-1, persistent=False):
        return self._id(lib().mosaic_graph_add_tensor(self._g, name.encode(), int(bytes_per_row), dim, chunk,
                                                      int(bool(persistent))), "mosaic_graph_add_tensor")

    def add_op(self, name, inputs, outputs, chunk=-1):
        ins = (ctypes.c_int32 * max(len(inputs), 1))(*inputs)
        outs = (ctypes.c_int32 * max(len(outputs), 1))(*outputs)
        return self._id(lib().mosaic_graph_add_op(self._g, name.encode(), ins, len(inputs), outs, len(outputs), chunk),
                        "mosaic_graph_add_op")

    def add_alias(self, a, b):
        _check(lib().mosaic_graph_add_alias(self._g, a, b), "mosaic_graph_add_alias")

    def add_barrier(self, tensor, chunk):
        _check(lib().mosaic_graph_add_barrier(self._g, tensor, chunk), "mosaic_graph_add_barrier")

    def plan(self, dims, chunks, placements=True):
        """(list of placement dicts in placement order, summary dict) for one instantiation."""
        d = (ctypes.c_int64 * max(len(dims), 1))(*dims)
        k = (ctypes.c_int32 * max(len(chunks), 1))(*chunks)
        summary = MosaicPlanSummary()
        _check(lib().mosaic_graph_plan(self._g, d, len(dims), k, len(chunks), None, 0, ctypes.byref(summary)),
               "mosaic_graph_plan")
        out = []
        if placements and summary.num_blocks:
            buf = (MosaicPlacement * summary.num_blocks)()
            _check(lib().mosaic_graph_plan(self._g, d, len(dims), k, len(chunks), buf, summary.num_blocks,
                                           ctypes.byref(summary)), "mosaic_graph_plan")
            out = [dict(tensor=b.tensor, iteration=b.iteration, first_step=b.first_step, last_step=b.last_step,
                        offset=b.offset, bytes=b.bytes) for b in buf]
        return out, {f: getattr(summary, f) for f, _ in MosaicPlanSummary._fields_}

    def search(self, dims, budget_bytes):
        """(ok, chunk counts, summary dict, planning passes) of the bottleneck-driven search."""
        d = (ctypes.c_int64 * max(len(dims), 1))(*dims)
        k = (ctypes.c_int32 * max(self.n_chunks, 1))()
        summary = MosaicPlanSummary()
        evals = ctypes.c_int32(0)
        rc = lib().mosaic_graph_search(self._g, d, len(dims), int(budget_bytes), k, self.n_chunks,
                                       ctypes.byref(summary), ctypes.byref(evals))
        if rc not in (MOSAIC_OK, MOSAIC_ERR_WORKSPACE_TOO_SMALL):
            raise MosaicError(rc, "mosaic_graph_search")
        return (rc == MOSAIC_OK, list(k)[:self.n_chunks],
                {f: getattr(summary, f) for f, _ in MosaicPlanSummary._fields_}, evals.value)


class MaskOnlyLogits:
    """Caller-side buffers for one shape, reused across denoising steps: the index list, the count, the
    scan scratch, the partials workspace and the three outputs.  `step` enqueues compaction + the fused
    reduction on the current stream and returns views; it never synchronises."""

    def __init__(self, T, d, V, max_rows=None, budget_bytes=0, device="cuda", sampling=False):
        self.T, self.d, self.V = T, d, V
        self.max_rows = T if max_rows is None else max_rows
        self.plan = mosaic_plan_workspace(T, self.max_rows, d, V, budget_bytes, sampling=sampling)
        dev = torch.device(device)
        self.idx = torch.empty(max(T, 1), dtype=torch.int32, device=dev)
        self.count = torch.zeros(1, dtype=torch.int32, device=dev)
        self.scratch = torch.empty(max(mosaic_compact_scratch_bytes(T), 16), dtype=torch.uint8, device=dev)
        ws = self.plan.workspace_bytes          # sized by the selector for the decode mode, within the budget
        self.workspace = torch.empty(max(ws, 16), dtype=torch.uint8, device=dev)
        n = max(self.max_rows, 1)
        self.token = torch.empty(n, dtype=torch.int32, device=dev)
        self.conf = torch.empty(n, dtype=torch.float32, device=dev)
        self.lse = torch.empty(n, dtype=torch.float32, device=dev)

    def replan(self, max_rows, budget_bytes=0):
        """A new plan for a smaller bound on the masked rows (the host knows how many masks are left: paper section
        4.4), so that few rows are spread over more vocabulary splits and still fill the chip.  Buffers are kept; the
        partials workspace grows if the new plan needs more."""
        if not 0 <= max_rows <= self.token.numel():
            raise ValueError("max_rows must lie between 0 and the bound the buffers were made for")
        sampling = bool(self.plan.flags & PLAN_SAMPLING)
        self.max_rows = max_rows
        self.plan = mosaic_plan_workspace(self.T, max_rows, self.d, self.V, budget_bytes, sampling=sampling)
        if self.plan.workspace_bytes > self.workspace.numel():
            self.workspace = torch.empty(self.plan.workspace_bytes, dtype=torch.uint8, device=self.workspace.device)

    @property
    def workspace_bytes(self) -> int:
        """Every device byte the path holds beyond its inputs and its three outputs."""
        return (self.idx.numel() * 4 + 4 + self.scratch.numel() + self.workspace.numel())

    def step(self, hidden, w, mask, stream=None):
        mosaic_mask_compact(mask, self.idx, self.count, self.scratch, stream)
        mosaic_masked_logits_reduce(hidden, w, self.idx, self.count, self.max_rows, self.token, self.conf, self.lse,
                                    self.plan, self.workspace, stream)
        return self.idx, self.count, self.token, self.conf, self.lse

    def sample_step(self, hidden, w, mask, temperature, seed, stream=None):
        """As `step`, drawing the tokens at `temperature` (the object must have been made with sampling=True)."""
        mosaic_mask_compact(mask, self.idx, self.count, self.scratch, stream)
        mosaic_masked_logits_sample(hidden, w, self.idx, self.count, self.max_rows, temperature, seed, self.token,
                                    self.conf, self.lse, self.plan, self.workspace, stream)
        return self.idx, self.count, self.token, self.conf, self.lse
