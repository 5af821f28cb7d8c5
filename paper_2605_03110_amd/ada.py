"""ctypes binding of libada (argument marshalling only; every step runs in the HIP kernels).

PyTorch is used for device memory and streams.  The functions mirror the C ABI in
``include/ada.h`` and return DEVICE tensors without synchronising; ``fetch`` brings a
result to the host and raises on a device-reported status.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libada.so")
SRC_DIR = os.path.join(_HERE, "csrc")
SOURCES = ("ada_kernels.hip",)

ADA_F32, ADA_BF16 = 0, 1
FLAG_CROSS_EARLIER_ONLY = 1
FLAG_TWO_PASS = 2
FLAG_RESIDENT_PASS = 4
FLAG_ATTN_CAUSAL = 8
FLAG_GREEDY_COVER = 16
OK = 0

SYMBOLS = ("ada_status_string", "ada_workspace_bytes", "ada_workspace_init", "ada_select_full", "ada_cascade_step",
           "ada_cascade_layers", "ada_cascade_layers_batched", "ada_cascade_step_grouped", "ada_cascade_layers_grouped", "ada_select_full_grouped", "ada_pipeline_layers", "ada_cascade_layers_adaptive", "ada_plan_tile_shape", "ada_plan_full_units",
           "ada_set_overlap", "ada_cascade_report", "ada_profile_enable",
           "ada_profile_collect", "ada_profile_copy_probe", "ada_profile_mfma_probe", "ada_assign_nearest",
           "ada_attention_compressed", "ada_cascade_step_static")

KERNEL_CLASSES = ("norm_prep", "gram_full", "gram_rep", "gram_cross", "update", "cascade_fused", "mfma_probe", "assign", "attn")


class AdaGroups(ctypes.Structure):
    """ada_groups of include/ada.h."""
    _fields_ = [("G", ctypes.c_int), ("x_gstride", ctypes.c_int64), ("list_gstride", ctypes.c_int64),
                ("counts_gstride", ctypes.c_int64), ("ops_gstride", ctypes.c_int64)]


class AdaTauControl(ctypes.Structure):
    """ada_tau_control of include/ada.h."""
    _fields_ = [("kappa", ctypes.c_double), ("eta_target", ctypes.c_double), ("tau_min", ctypes.c_double),
                ("tau_max", ctypes.c_double)]


class AdaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__("%s: %s" % (where, status_string(status)))


# Private (scratch) memory the hot kernels may use, in bytes per lane: a private array or a spill that lands in one of
# them costs every launch microseconds (k_cascade_fused once lost 10 us per step to a 64-byte array in its last
# workgroup's code), so the build refuses it instead of letting a benchmark find out.
SCRATCH_BUDGET = {
    "k_cascade_fusedItLb1ELi2ELb1E": 64,       # bf16, aligned rows, two K-groups, direct-to-LDS: the cascade step
    "k_gram_dmaILb1E": 0,                      # one-launch full selection
    "k_gram_dmaILb0E": 0,                      # full Gram beyond T = 4096
    "k_attn_rep2ILi256E": 64,                  # attention on the representative set, d_h = 256
}


def kernel_resources(remarks: str) -> Dict[str, Dict[str, int]]:
    """{mangled kernel name: {VGPRs, AGPRs, ScratchSize, ...}} from hipcc's -Rpass-analysis=kernel-resource-usage."""
    out: Dict[str, Dict[str, int]] = {}
    cur = None
    for line in remarks.splitlines():
        if "Function Name:" in line:
            cur = line.split("Function Name:")[1].split("[")[0].strip()
            out[cur] = {}
        elif cur and "remark:" in line and ":" in line.split("remark:")[1]:
            key, _, val = line.split("remark:")[1].partition(":")
            val = val.split("[")[0].strip()
            if val.isdigit():
                out[cur][key.strip().split(" [")[0]] = int(val)
    return out


def build_library(verbose: bool = False) -> str:
    """Compile the HIP sources for gfx950 into libada.so next to this file; fails if a hot kernel needs more private
    memory than SCRATCH_BUDGET allows."""
    tmp = LIB_PATH + ".tmp.%d" % os.getpid()
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Rpass-analysis=kernel-resource-usage"]
    cmd += [os.path.join(SRC_DIR, s) for s in SOURCES] + ["-o", tmp]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose:
        print(res.stderr)
    usage = kernel_resources(res.stderr)
    for tag, budget in SCRATCH_BUDGET.items():
        hits = {k: v for k, v in usage.items() if tag in k}
        if not hits:
            os.remove(tmp)
            raise RuntimeError("no resource report for kernel *%s*: has it been renamed?" % tag)
        for k, v in hits.items():
            if v.get("ScratchSize", 0) > budget:
                os.remove(tmp)
                raise RuntimeError("%s uses %d bytes of private memory per lane (budget %d)" % (k, v["ScratchSize"], budget))
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


def library_is_stale() -> bool:
    """True if libada.so is missing or older than a source it is built from."""
    if not os.path.exists(LIB_PATH):
        return True
    built = os.path.getmtime(LIB_PATH)
    inc = os.path.join(os.path.dirname(_HERE), "include")
    deps = [os.path.join(SRC_DIR, f) for f in os.listdir(SRC_DIR)] + [os.path.join(inc, f) for f in os.listdir(inc)]
    return any(os.path.getmtime(f) > built for f in deps)


_lib = None


def lib():
    """Load libada.so; fail loudly if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libada.so is missing at %s: run __graft_entry__.build() "
                               "(or paper_2605_03110_amd.ada.build_library()) first" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, f32, u32, sz = (ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float,
                                      ctypes.c_uint, ctypes.c_size_t)
        L.ada_status_string.restype = ctypes.c_char_p
        L.ada_status_string.argtypes = [i32]
        L.ada_workspace_bytes.restype = sz
        L.ada_workspace_bytes.argtypes = [i32]
        L.ada_workspace_init.restype = i32
        L.ada_workspace_init.argtypes = [vp, sz, vp]
        L.ada_select_full.restype = i32
        L.ada_select_full.argtypes = [vp, i32, i32, i64, i32, f32, vp, vp, vp, vp, vp, sz, vp, u32]
        L.ada_cascade_step.restype = i32
        L.ada_cascade_step.argtypes = [vp, i32, i32, i64, i32, f32, vp, i32, vp, vp, vp, vp, vp, vp, vp,
                                       vp, sz, vp, u32]
        L.ada_cascade_step_static.restype = i32
        L.ada_cascade_step_static.argtypes = [vp, i32, i32, i64, i32, f32, vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, u32]
        L.ada_cascade_layers.restype = i32
        L.ada_cascade_layers.argtypes = [ctypes.POINTER(vp), i32, i32, i32, i64, i32, f32, vp, vp, vp, vp, vp,
                                         vp, sz, vp, u32]
        L.ada_cascade_layers_batched.restype = i32
        L.ada_cascade_layers_batched.argtypes = [ctypes.POINTER(vp), i32, i32, i32, i32, i64, i32, f32, vp, vp, vp, vp, vp,
                                                 vp, sz, ctypes.POINTER(vp), vp, u32]
        L.ada_cascade_step_grouped.restype = i32
        L.ada_cascade_step_grouped.argtypes = [ctypes.POINTER(AdaGroups), vp, i32, i32, i64, i32, f32, vp, i32, vp, vp, vp, vp,
                                               vp, vp, vp, sz, vp, u32]
        L.ada_pipeline_layers.restype = i32
        L.ada_pipeline_layers.argtypes = [ctypes.POINTER(vp)] * 4 + [i32, i32, i32, i32, i64, i32, f32, vp, vp, vp, vp, vp,
                                          ctypes.POINTER(vp), i64, vp, sz, vp, vp, vp, u32]
        L.ada_cascade_layers_adaptive.restype = i32
        L.ada_cascade_layers_adaptive.argtypes = [ctypes.POINTER(vp), i32, i32, i32, i64, i32, f32,
                                                  ctypes.POINTER(AdaTauControl), vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, u32]
        L.ada_plan_tile_shape.restype = i32
        L.ada_plan_tile_shape.argtypes = [i32, i32, i32, i32]
        L.ada_plan_full_units.restype = i32
        L.ada_plan_full_units.argtypes = [i32, i32, i32]
        L.ada_select_full_grouped.restype = i32
        L.ada_select_full_grouped.argtypes = [ctypes.POINTER(AdaGroups), vp, i32, i32, i64, i32, f32, vp, vp, vp, vp, sz, vp, u32]
        L.ada_cascade_layers_grouped.restype = i32
        L.ada_cascade_layers_grouped.argtypes = [ctypes.POINTER(AdaGroups), ctypes.POINTER(vp), i32, i32, i32, i64, i32, f32,
                                                 vp, vp, vp, vp, vp, vp, sz, vp, u32]
        L.ada_set_overlap.restype = i32
        L.ada_set_overlap.argtypes = [vp, vp, i32, vp, vp]
        L.ada_cascade_report.restype = i32
        L.ada_cascade_report.argtypes = [i32, i32, vp, vp, vp, vp, vp]
        L.ada_profile_enable.restype = i32
        L.ada_profile_enable.argtypes = [i32]
        L.ada_profile_collect.restype = i32
        L.ada_profile_collect.argtypes = [vp, vp]
        L.ada_profile_copy_probe.restype = i32
        L.ada_profile_copy_probe.argtypes = [vp, vp, sz, vp]
        L.ada_profile_mfma_probe.restype = i32
        L.ada_profile_mfma_probe.argtypes = [i32, i32, vp, vp]
        L.ada_attention_compressed.restype = i32
        L.ada_attention_compressed.argtypes = [vp, vp, vp, i32, i32, i32, i64, i32, vp, i32, vp, vp, vp, i64, vp,
                                               vp, sz, vp, u32]
        L.ada_assign_nearest.restype = i32
        L.ada_assign_nearest.argtypes = [vp, i32, i32, i64, i32, vp, i32, vp, vp, vp, vp, vp, sz, vp, u32]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().ada_status_string(int(status)).decode()


def workspace_bytes(T: int) -> int:
    return int(lib().ada_workspace_bytes(int(T)))


def workspace_batched(T: int, B: int, device="cuda") -> torch.Tensor:
    """B zero-filled workspaces back to back, for ada_cascade_layers_batched."""
    return torch.zeros(workspace_bytes(T) * int(B), dtype=torch.uint8, device=device)


def workspace(T: int, device="cuda") -> torch.Tensor:
    """A zero-filled workspace (the library needs it zeroed before first use and keeps it ready afterwards)."""
    return torch.zeros(workspace_bytes(T), dtype=torch.uint8, device=device)


def ada_workspace_init(ws: torch.Tensor, *, stream=None) -> None:
    rc = lib().ada_workspace_init(_ptr(ws), ws.numel(), _stream(stream))
    if rc != OK:
        raise AdaError(rc, "ada_workspace_init")


def _dtype_code(X: torch.Tensor) -> int:
    if X.dtype == torch.float32:
        return ADA_F32
    if X.dtype == torch.bfloat16:
        return ADA_BF16
    raise TypeError("X must be float32 or bfloat16, got %s" % X.dtype)


def _check_x(X: torch.Tensor):
    if not X.is_cuda:
        raise ValueError("X must live on the GPU")
    if X.dim() != 2 or (X.shape[1] > 1 and X.stride(1) != 1):
        raise ValueError("X must be a row-major T x d matrix (unit stride along d)")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def ada_select_full(X: torch.Tensor, tau: float, *, ws: Optional[torch.Tensor] = None, stream=None,
                    flags: int = 0) -> Dict[str, torch.Tensor]:
    """Full Gram-threshold selection.  Returns device tensors mask[T] u8, idx[T] i32, counts[4] i32, gamma[T] f32."""
    _check_x(X)
    T, d = X.shape
    dev = X.device
    ws = workspace(T, dev) if ws is None else ws
    out = dict(mask=torch.empty(T, dtype=torch.uint8, device=dev),
               idx=torch.empty(T, dtype=torch.int32, device=dev),
               counts=torch.empty(4, dtype=torch.int32, device=dev),
               gamma=torch.empty(T, dtype=torch.float32, device=dev))
    rc = lib().ada_select_full(_ptr(X), T, d, X.stride(0), _dtype_code(X), float(tau), _ptr(out["mask"]),
                               _ptr(out["idx"]), _ptr(out["counts"]), _ptr(out["gamma"]), _ptr(ws), ws.numel(),
                               _stream(stream), int(flags))
    if rc != OK:
        raise AdaError(rc, "ada_select_full")
    out["_keep"] = ws
    return out


def ada_cascade_step(X: torch.Tensor, tau: float, prev_idx: torch.Tensor, r: Optional[int] = None,
                     r_dev: Optional[torch.Tensor] = None, *, ws: Optional[torch.Tensor] = None, stream=None,
                     flags: int = 0) -> Dict[str, torch.Tensor]:
    """One cascade step.  prev_idx: device int32, ascending.  r defaults to prev_idx.numel() (an upper bound
    when r_dev, a device int32 holding the actual size, is given).  Returns device tensors idx[T], adds[T],
    removes[r], counts[4], gram_ops[1] (int64 storage of the uint64), gamma[T]."""
    _check_x(X)
    T, d = X.shape
    dev = X.device
    if prev_idx.dtype != torch.int32 or not prev_idx.is_cuda or not prev_idx.is_contiguous():
        raise ValueError("prev_idx must be a contiguous int32 device tensor")
    r = int(prev_idx.numel()) if r is None else int(r)
    if r > prev_idx.numel():
        raise ValueError("r exceeds the capacity of prev_idx")
    ws = workspace(T, dev) if ws is None else ws
    out = dict(idx=torch.empty(T, dtype=torch.int32, device=dev),
               adds=torch.empty(T, dtype=torch.int32, device=dev),
               removes=torch.empty(max(r, 1), dtype=torch.int32, device=dev),
               counts=torch.empty(4, dtype=torch.int32, device=dev),
               gram_ops=torch.empty(1, dtype=torch.int64, device=dev),
               gamma=torch.empty(T, dtype=torch.float32, device=dev))
    rc = lib().ada_cascade_step(_ptr(X), T, d, X.stride(0), _dtype_code(X), float(tau), _ptr(prev_idx), r,
                                _ptr(r_dev), _ptr(out["idx"]), _ptr(out["adds"]), _ptr(out["removes"]),
                                _ptr(out["counts"]), _ptr(out["gram_ops"]), _ptr(out["gamma"]), _ptr(ws),
                                ws.numel(), _stream(stream), int(flags))
    if rc != OK:
        raise AdaError(rc, "ada_cascade_step")
    out["_keep"] = (ws, prev_idx, r_dev)
    return out


STATIC_MAX_T = 4096


def ada_cascade_step_static(X: torch.Tensor, tau: float, prev_idx: torch.Tensor, out: Dict[str, torch.Tensor],
                            r: Optional[int] = None, r_dev: Optional[torch.Tensor] = None, *, stream=None,
                            flags: int = 0) -> Dict[str, torch.Tensor]:
    """ada_cascade_step on the library's own scratch array: no workspace, and nothing is allocated here either --
    the caller brings the output tensors (`out`: idx[T], adds[T], removes[>= r], counts[4], gram_ops[1] int64,
    gamma[T]), e.g. those of an earlier ada_cascade_step."""
    _check_x(X)
    T, d = X.shape
    if prev_idx.dtype != torch.int32 or not prev_idx.is_cuda or not prev_idx.is_contiguous():
        raise ValueError("prev_idx must be a contiguous int32 device tensor")
    r = int(prev_idx.numel()) if r is None else int(r)
    if r > prev_idx.numel() or out["removes"].numel() < r or out["idx"].numel() < T or out["adds"].numel() < T:
        raise ValueError("r exceeds the capacity of prev_idx, or an output tensor is too small")
    rc = lib().ada_cascade_step_static(_ptr(X), T, d, X.stride(0), _dtype_code(X), float(tau), _ptr(prev_idx), r,
                                       _ptr(r_dev), _ptr(out["idx"]), _ptr(out["adds"]), _ptr(out["removes"]),
                                       _ptr(out["counts"]), _ptr(out["gram_ops"]), _ptr(out.get("gamma")),
                                       _stream(stream), int(flags))
    if rc != OK:
        raise AdaError(rc, "ada_cascade_step_static")
    return out


def ada_assign_nearest(X: torch.Tensor, idx: torch.Tensor, r: Optional[int] = None,
                       r_dev: Optional[torch.Tensor] = None, *, ws: Optional[torch.Tensor] = None, stream=None,
                       flags: int = 0) -> Dict[str, torch.Tensor]:
    """Nearest representative of every token (Section 2.3).  idx: device int32, ascending token ids of R; r
    defaults to idx.numel() (an upper bound when r_dev is given).  Returns device tensors assign[T] (int32),
    corr[T] (float32) and info[4] = {T - r, 0, 0, status}."""
    _check_x(X)
    T, d = X.shape
    dev = X.device
    if idx.dtype != torch.int32 or not idx.is_cuda or not idx.is_contiguous():
        raise ValueError("idx must be a contiguous int32 device tensor")
    r = int(idx.numel()) if r is None else int(r)
    if r > idx.numel():
        raise ValueError("r exceeds the capacity of idx")
    ws = workspace(T, dev) if ws is None else ws
    out = dict(assign=torch.empty(T, dtype=torch.int32, device=dev),
               corr=torch.empty(T, dtype=torch.float32, device=dev),
               info=torch.empty(4, dtype=torch.int32, device=dev))
    rc = lib().ada_assign_nearest(_ptr(X), T, d, X.stride(0), _dtype_code(X), _ptr(idx), r, _ptr(r_dev),
                                  _ptr(out["assign"]), _ptr(out["corr"]), _ptr(out["info"]), _ptr(ws), ws.numel(),
                                  _stream(stream), int(flags))
    if rc != OK:
        raise AdaError(rc, "ada_assign_nearest")
    out["_keep"] = (ws, idx, r_dev)
    return out


def ada_attention_compressed(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, H: int, idx: torch.Tensor,
                             assign: torch.Tensor, r: Optional[int] = None, r_dev: Optional[torch.Tensor] = None, *,
                             ws: Optional[torch.Tensor] = None, stream=None, flags: int = 0,
                             out: Optional[torch.Tensor] = None) -> Dict[str, torch.Tensor]:
    """Attention on the representative set (eq. (1)) with every token taking its representative's output row.
    Q, K, V: device T x (H * d_h), same dtype and strides.  Returns device tensors out[T, H * d_h] (float32; the
    caller's `out`, a float32 T x (H * d_h) view with unit column stride, if one is given) and
    info[4] = {|R|, 0, 0, status}."""
    for M in (Q, K, V):
        _check_x(M)
    T, D = Q.shape
    if K.shape != Q.shape or V.shape != Q.shape or K.dtype != Q.dtype or V.dtype != Q.dtype:
        raise ValueError("Q, K, V must share shape and dtype")
    if K.stride(0) != Q.stride(0) or V.stride(0) != Q.stride(0):
        raise ValueError("Q, K, V must share their leading dimension")
    if D % int(H) != 0:
        raise ValueError("the row length must be H * d_h")
    for a, name in ((idx, "idx"), (assign, "assign")):
        if a.dtype != torch.int32 or not a.is_cuda or not a.is_contiguous():
            raise ValueError("%s must be a contiguous int32 device tensor" % name)
    if assign.numel() != T:
        raise ValueError("assign must have T entries")
    r = int(idx.numel()) if r is None else int(r)
    if r > idx.numel():
        raise ValueError("r exceeds the capacity of idx")
    dev = Q.device
    ws = workspace(T, dev) if ws is None else ws
    if out is None:
        out = torch.empty((T, D), dtype=torch.float32, device=dev)
    elif (out.dtype != torch.float32 or out.device != dev or tuple(out.shape) != (T, D) or out.stride(1) != 1
          or out.stride(0) < D):
        raise ValueError("out must be a float32 T x (H * d_h) device view with unit column stride")
    out = dict(out=out, info=torch.empty(4, dtype=torch.int32, device=dev))
    rc = lib().ada_attention_compressed(_ptr(Q), _ptr(K), _ptr(V), T, int(H), D // int(H), Q.stride(0), _dtype_code(Q),
                                        _ptr(idx), r, _ptr(r_dev), _ptr(assign), _ptr(out["out"]), out["out"].stride(0),
                                        _ptr(out["info"]),
                                        _ptr(ws), ws.numel(), _stream(stream), int(flags))
    if rc != OK:
        raise AdaError(rc, "ada_attention_compressed")
    out["_keep"] = (ws, Q, K, V, idx, assign, r_dev)
    return out


def ada_cascade_layers(Xs: Sequence[torch.Tensor], tau: float, *, want_lists: bool = True,
                       ws: Optional[torch.Tensor] = None, stream=None, flags: int = 0,
                       out: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
    """Full selection at layer 0 and cascade steps at layers 1..L-1, chained on the device.
    Returns device tensors idx[L,T], counts[L,4], gram_ops[L] and, if want_lists, adds[L,T], removes[L,T]."""
    L = len(Xs)
    if L < 1:
        raise ValueError("need at least one layer")
    for X in Xs:
        _check_x(X)
        if X.shape != Xs[0].shape or X.dtype != Xs[0].dtype or X.stride(0) != Xs[0].stride(0):
            raise ValueError("all layers must share shape, dtype and leading dimension")
    T, d = Xs[0].shape
    dev = Xs[0].device
    ws = workspace(T, dev) if ws is None else ws
    if out is None:
        out = dict(idx=torch.empty((L, T), dtype=torch.int32, device=dev),
                   counts=torch.empty((L, 4), dtype=torch.int32, device=dev),
                   gram_ops=torch.empty(L, dtype=torch.int64, device=dev))
        if want_lists:
            out["adds"] = torch.empty((L, T), dtype=torch.int32, device=dev)
            out["removes"] = torch.empty((L, T), dtype=torch.int32, device=dev)
    ptrs = (ctypes.c_void_p * L)(*[X.data_ptr() for X in Xs])
    rc = lib().ada_cascade_layers(ptrs, L, T, d, Xs[0].stride(0), _dtype_code(Xs[0]), float(tau), _ptr(out["idx"]),
                                  _ptr(out["counts"]), _ptr(out["gram_ops"]), _ptr(out.get("adds")),
                                  _ptr(out.get("removes")), _ptr(ws), ws.numel(), _stream(stream), int(flags))
    if rc != OK:
        raise AdaError(rc, "ada_cascade_layers")
    out["_keep"] = (ws, list(Xs))
    return out


def ada_cascade_layers_batched(seqs: Sequence[Sequence[torch.Tensor]], tau: float, *, want_lists: bool = False,
                               ws: Optional[torch.Tensor] = None, streams=None, stream=None, flags: int = 0,
                               out: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
    """ada_cascade_layers for B sequences (seqs[b][l]: the T x d matrix of sequence b at layer l), sequence b on
    streams[b] (torch streams; None = all on `stream`, one after the other).  Work enqueued on `stream` (default: the
    current stream) after the call waits for all chains.  ws: B workspaces back to back (workspace_batched).
    Returns device tensors idx[B,L,T], counts[B,L,4], gram_ops[B,L] and, if want_lists, adds / removes [B,L,T]."""
    B = len(seqs)
    if B < 1 or len(seqs[0]) < 1:
        raise ValueError("need at least one sequence and one layer")
    L = len(seqs[0])
    X0 = seqs[0][0]
    for s in seqs:
        if len(s) != L:
            raise ValueError("all sequences must have the same number of layers")
        for X in s:
            _check_x(X)
            if X.shape != X0.shape or X.dtype != X0.dtype or X.stride(0) != X0.stride(0) or X.device != X0.device:
                raise ValueError("all matrices must share shape, dtype, leading dimension and device")
    if streams is not None and len(streams) != B:
        raise ValueError("need one stream per sequence")
    T, d = X0.shape
    dev = X0.device
    ws = workspace_batched(T, B, dev) if ws is None else ws
    if out is None:
        out = dict(idx=torch.empty((B, L, T), dtype=torch.int32, device=dev),
                   counts=torch.empty((B, L, 4), dtype=torch.int32, device=dev),
                   gram_ops=torch.empty((B, L), dtype=torch.int64, device=dev))
        if want_lists:
            out["adds"] = torch.empty((B, L, T), dtype=torch.int32, device=dev)
            out["removes"] = torch.empty((B, L, T), dtype=torch.int32, device=dev)
    ptrs = (ctypes.c_void_p * (B * L))(*[X.data_ptr() for s in seqs for X in s])
    sarr = None if streams is None else (ctypes.c_void_p * B)(*[s.cuda_stream for s in streams])
    rc = lib().ada_cascade_layers_batched(ptrs, B, L, T, d, X0.stride(0), _dtype_code(X0), float(tau), _ptr(out["idx"]),
                                          _ptr(out["counts"]), _ptr(out["gram_ops"]), _ptr(out.get("adds")),
                                          _ptr(out.get("removes")), _ptr(ws), ws.numel(), sarr, _stream(stream),
                                          int(flags))
    if rc != OK:
        raise AdaError(rc, "ada_cascade_layers_batched")
    out["_keep"] = (ws, [list(s) for s in seqs], streams)
    return out


def heads_view(X: torch.Tensor, H: int) -> torch.Tensor:
    """The H column blocks of a T x (H d_h) matrix as a [H, T, d_h] view (no copy): the groups of the per-head cascade."""
    T, d = X.shape
    if d % H != 0:
        raise ValueError("d must be a multiple of the head count")
    return X.view(T, H, d // H).permute(1, 0, 2)


def _check_xg(Xg: torch.Tensor):
    if not Xg.is_cuda:
        raise ValueError("X must live on the GPU")
    if Xg.dim() != 3 or (Xg.shape[2] > 1 and Xg.stride(2) != 1):
        raise ValueError("X must be a [G, T, d] tensor (or view) with unit stride along d")


def ada_select_full_grouped(Xg: torch.Tensor, tau: float, *, ws: Optional[torch.Tensor] = None, stream=None,
                            flags: int = 0, out: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
    """Full selection of G problems in one allocation (Xg: [G, T, d] view).  Returns mask [G, T] u8, idx [G, T] i32,
    counts [G, 4] i32 (usable as prev_idx / r_dev of ada_cascade_step_grouped)."""
    _check_xg(Xg)
    G, T, d = Xg.shape
    dev = Xg.device
    ws = workspace_batched(T, G, dev) if ws is None else ws
    if out is None:
        out = dict(mask=torch.empty((G, T), dtype=torch.uint8, device=dev),
                   idx=torch.empty((G, T), dtype=torch.int32, device=dev),
                   counts=torch.empty((G, 4), dtype=torch.int32, device=dev))
    g = AdaGroups(G, Xg.stride(0) if G > 1 else d, T, 4, 1)
    rc = lib().ada_select_full_grouped(ctypes.byref(g), _ptr(Xg), T, d, Xg.stride(1), _dtype_code(Xg), float(tau),
                                       _ptr(out["mask"]), _ptr(out["idx"]), _ptr(out["counts"]), _ptr(ws), ws.numel(),
                                       _stream(stream), int(flags))
    if rc != OK:
        raise AdaError(rc, "ada_select_full_grouped")
    out["_keep"] = (ws, Xg)
    return out


def ada_cascade_step_grouped(Xg: torch.Tensor, tau: float, prev_idx: torch.Tensor, r: Optional[int] = None,
                             r_dev: Optional[torch.Tensor] = None, *, ws: Optional[torch.Tensor] = None, stream=None,
                             flags: int = 0) -> Dict[str, torch.Tensor]:
    """One cascade step for G problems in one allocation.  Xg: [G, T, d] view (heads_view, or stacked sequences);
    prev_idx: [G, T] int32 (row g: group g's inherited set, ascending); r bounds every group's count (default T when
    r_dev, a [G, 4] int32 tensor with the counts in column 0, is given).  Returns idx, adds, removes [G, T], counts
    [G, 4], gram_ops [G]."""
    _check_xg(Xg)
    G, T, d = Xg.shape
    dev = Xg.device
    if prev_idx.dtype != torch.int32 or not prev_idx.is_cuda or prev_idx.dim() != 2 or prev_idx.shape[0] != G \
            or prev_idx.stride(1) != 1:
        raise ValueError("prev_idx must be a [G, n] int32 device tensor with contiguous rows")
    if r_dev is not None and (r_dev.dtype != torch.int32 or r_dev.dim() != 2 or r_dev.shape != (G, 4) or not r_dev.is_contiguous()):
        raise ValueError("r_dev must be a contiguous [G, 4] int32 device tensor")
    r = int(prev_idx.shape[1]) if r is None else int(r)
    if r > prev_idx.shape[1]:
        raise ValueError("r exceeds the rows of prev_idx")
    ws = workspace_batched(T, G, dev) if ws is None else ws
    out = dict(idx=torch.empty((G, T), dtype=torch.int32, device=dev), adds=torch.empty((G, T), dtype=torch.int32, device=dev),
               removes=torch.empty((G, T), dtype=torch.int32, device=dev),
               counts=torch.empty((G, 4), dtype=torch.int32, device=dev),
               gram_ops=torch.empty(G, dtype=torch.int64, device=dev))
    if prev_idx.stride(0) != T and G > 1:
        raise ValueError("prev_idx rows must be T entries apart (the outputs are)")
    g = AdaGroups(G, Xg.stride(0) if G > 1 else d, T, 4, 1)
    rc = lib().ada_cascade_step_grouped(ctypes.byref(g), _ptr(Xg), T, d, Xg.stride(1), _dtype_code(Xg), float(tau),
                                        _ptr(prev_idx), r, _ptr(r_dev), _ptr(out["idx"]), _ptr(out["adds"]),
                                        _ptr(out["removes"]), _ptr(out["counts"]), _ptr(out["gram_ops"]), _ptr(ws),
                                        ws.numel(), _stream(stream), int(flags))
    if rc != OK:
        raise AdaError(rc, "ada_cascade_step_grouped")
    out["_keep"] = (ws, Xg, prev_idx, r_dev)
    return out


def ada_cascade_layers_grouped(Xgs: Sequence[torch.Tensor], tau: float, *, want_lists: bool = False,
                               ws: Optional[torch.Tensor] = None, stream=None, flags: int = 0,
                               out: Optional[Dict[str, torch.Tensor]] = None) -> Dict[str, torch.Tensor]:
    """The layer loop for G problems per layer (Xgs[l]: [G, T, d] view of layer l; all layers with the same strides).
    Returns idx[G,L,T], counts[G,L,4], gram_ops[G,L] and, if want_lists, adds / removes [G,L,T]."""
    L = len(Xgs)
    if L < 1:
        raise ValueError("need at least one layer")
    for Xg in Xgs:
        _check_xg(Xg)
        if Xg.shape != Xgs[0].shape or Xg.dtype != Xgs[0].dtype or Xg.stride() != Xgs[0].stride():
            raise ValueError("all layers must share shape, dtype and strides")
    G, T, d = Xgs[0].shape
    dev = Xgs[0].device
    ws = workspace_batched(T, G, dev) if ws is None else ws
    if out is None:
        out = dict(idx=torch.empty((G, L, T), dtype=torch.int32, device=dev),
                   counts=torch.empty((G, L, 4), dtype=torch.int32, device=dev),
                   gram_ops=torch.empty((G, L), dtype=torch.int64, device=dev))
        if want_lists:
            out["adds"] = torch.empty((G, L, T), dtype=torch.int32, device=dev)
            out["removes"] = torch.empty((G, L, T), dtype=torch.int32, device=dev)
    g = AdaGroups(G, Xgs[0].stride(0) if G > 1 else d, 0, 0, 0)
    ptrs = (ctypes.c_void_p * L)(*[X.data_ptr() for X in Xgs])
    rc = lib().ada_cascade_layers_grouped(ctypes.byref(g), ptrs, L, T, d, Xgs[0].stride(1), _dtype_code(Xgs[0]), float(tau),
                                          _ptr(out["idx"]), _ptr(out["counts"]), _ptr(out["gram_ops"]),
                                          _ptr(out.get("adds")), _ptr(out.get("removes")), _ptr(ws), ws.numel(),
                                          _stream(stream), int(flags))
    if rc != OK:
        raise AdaError(rc, "ada_cascade_layers_grouped")
    out["_keep"] = (ws, list(Xgs))
    return out


def ada_pipeline_layers(Xs: Sequence[torch.Tensor], Qs: Sequence[torch.Tensor], Ks: Sequence[torch.Tensor],
                        Vs: Sequence[torch.Tensor], H: int, tau: float, *, ws: Optional[torch.Tensor] = None,
                        stream_sel=None, stream_attn=None, stream=None, flags: int = 0,
                        out: Optional[Dict[str, object]] = None) -> Dict[str, object]:
    """Selection, assignment and attention on the representative set for L layers, the selection on stream_sel and
    the rest on stream_attn (torch streams; None = `stream`).  Returns idx[L,T], counts[L,4], gram_ops[L],
    assign[L,T], info[L,8] and out (a list of L float tensors T x d)."""
    L = len(Xs)
    if L < 1 or not (len(Qs) == len(Ks) == len(Vs) == L):
        raise ValueError("need the same number (>= 1) of X, Q, K and V matrices")
    X0 = Xs[0]
    for M in list(Xs) + list(Qs) + list(Ks) + list(Vs):
        _check_x(M)
        if M.shape != X0.shape or M.dtype != X0.dtype or M.stride(0) != X0.stride(0) or M.device != X0.device:
            raise ValueError("all matrices must share shape, dtype, leading dimension and device")
    T, d = X0.shape
    if d % H != 0:
        raise ValueError("d must be a multiple of the head count")
    dev = X0.device
    ws = workspace_batched(T, 2, dev) if ws is None else ws
    if out is None:
        out = dict(idx=torch.empty((L, T), dtype=torch.int32, device=dev),
                   counts=torch.empty((L, 4), dtype=torch.int32, device=dev),
                   gram_ops=torch.empty(L, dtype=torch.int64, device=dev),
                   assign=torch.empty((L, T), dtype=torch.int32, device=dev),
                   info=torch.empty((L, 8), dtype=torch.int32, device=dev),
                   out=[torch.empty((T, d), dtype=torch.float32, device=dev) for _ in range(L)])
    arr = lambda ms: (ctypes.c_void_p * L)(*[m.data_ptr() for m in ms])
    sp = lambda s_: None if s_ is None else ctypes.c_void_p(s_.cuda_stream)
    rc = lib().ada_pipeline_layers(arr(Xs), arr(Qs), arr(Ks), arr(Vs), L, T, H, d // H, X0.stride(0), _dtype_code(X0),
                                   float(tau), _ptr(out["idx"]), _ptr(out["counts"]), _ptr(out["gram_ops"]),
                                   _ptr(out["assign"]), _ptr(out["info"]), arr(out["out"]), out["out"][0].stride(0),
                                   _ptr(ws), ws.numel(), sp(stream_sel), sp(stream_attn), _stream(stream), int(flags))
    if rc != OK:
        raise AdaError(rc, "ada_pipeline_layers")
    out["_keep"] = (ws, list(Xs), list(Qs), list(Ks), list(Vs), stream_sel, stream_attn)
    return out


def ada_cascade_layers_adaptive(Xs: Sequence[torch.Tensor], tau0: float, kappa: float, eta_target: float, tau_min: float,
                                tau_max: float, *, want_lists: bool = True, ws: Optional[torch.Tensor] = None,
                                stream=None, flags: int = 0) -> Dict[str, torch.Tensor]:
    """ada_cascade_layers with the threshold adapted from the turnover between layers, on the device (Section 8.1).
    Returns the tensors of ada_cascade_layers plus tau[L] (float64) and thr[L] (float32): what each layer used."""
    L = len(Xs)
    if L < 1:
        raise ValueError("need at least one layer")
    for X in Xs:
        _check_x(X)
        if X.shape != Xs[0].shape or X.dtype != Xs[0].dtype or X.stride(0) != Xs[0].stride(0):
            raise ValueError("all layers must share shape, dtype and leading dimension")
    T, d = Xs[0].shape
    dev = Xs[0].device
    ws = workspace(T, dev) if ws is None else ws
    out = dict(idx=torch.empty((L, T), dtype=torch.int32, device=dev),
               counts=torch.empty((L, 4), dtype=torch.int32, device=dev),
               gram_ops=torch.empty(L, dtype=torch.int64, device=dev),
               tau=torch.empty(L, dtype=torch.float64, device=dev), thr=torch.empty(L, dtype=torch.float32, device=dev))
    if want_lists:
        out["adds"] = torch.empty((L, T), dtype=torch.int32, device=dev)
        out["removes"] = torch.empty((L, T), dtype=torch.int32, device=dev)
    ctl = AdaTauControl(float(kappa), float(eta_target), float(tau_min), float(tau_max))
    ptrs = (ctypes.c_void_p * L)(*[X.data_ptr() for X in Xs])
    rc = lib().ada_cascade_layers_adaptive(ptrs, L, T, d, Xs[0].stride(0), _dtype_code(Xs[0]), float(tau0), ctypes.byref(ctl),
                                           _ptr(out["idx"]), _ptr(out["counts"]), _ptr(out["gram_ops"]),
                                           _ptr(out.get("adds")), _ptr(out.get("removes")), _ptr(out["tau"]),
                                           _ptr(out["thr"]), _ptr(ws), ws.numel(), _stream(stream), int(flags))
    if rc != OK:
        raise AdaError(rc, "ada_cascade_layers_adaptive")
    out["_keep"] = (ws, list(Xs))
    return out


def ada_plan_tile_shape(r: int, T: int, d: int, workgroups: int) -> int:
    """Tile shape of a one-launch cascade step of this size (0 = 64 x 64, 1 = 64 x 128, 2 = 128 x 128; -1: bad
    arguments); host-side evaluation of the kernel's own choice."""
    return int(lib().ada_plan_tile_shape(int(r), int(T), int(d), int(workgroups)))


def ada_plan_full_units(T: int, d: int, workgroups: int) -> int:
    """How the full selection's direct-to-LDS kernel cuts the triangle into units (0, 1, 2; -1 outside its range).
    Host only."""
    return int(lib().ada_plan_full_units(int(T), int(d), int(workgroups)))


def ada_set_overlap(mask_a: torch.Tensor, mask_b: torch.Tensor, *, stream=None) -> torch.Tensor:
    """Device int32 [2] = {|A n B|, |A u B|} of two uint8 masks (eq. (3))."""
    if mask_a.dtype != torch.uint8 or mask_b.dtype != torch.uint8 or mask_a.numel() != mask_b.numel():
        raise ValueError("masks must be uint8 tensors of equal length")
    out = torch.empty(2, dtype=torch.int32, device=mask_a.device)
    rc = lib().ada_set_overlap(_ptr(mask_a), _ptr(mask_b), mask_a.numel(), _ptr(out), _stream(stream))
    if rc != OK:
        raise AdaError(rc, "ada_set_overlap")
    return out


def ada_cascade_report(counts_host: torch.Tensor, gram_ops_host: torch.Tensor, T: int) -> Dict[str, object]:
    """Host bookkeeping (Jaccard eq. (3), turnover eq. (8), Gram-op savings of Table 6) from HOST copies of
    ada_cascade_layers' counts[L,4] (int32) and gram_ops[L] (int64)."""
    counts_host = counts_host.contiguous().to(torch.int32).cpu()
    gram_ops_host = gram_ops_host.contiguous().to(torch.int64).cpu()
    L = counts_host.shape[0]
    jac = torch.zeros(L, dtype=torch.float64)
    eta = torch.zeros(L, dtype=torch.float64)
    sav = ctypes.c_double(0.0)
    rc = lib().ada_cascade_report(L, int(T), _ptr(counts_host), _ptr(gram_ops_host), _ptr(jac), _ptr(eta),
                                  ctypes.cast(ctypes.byref(sav), ctypes.c_void_p))
    if rc != OK:
        raise AdaError(rc, "ada_cascade_report")
    return dict(jaccard=jac.tolist(), turnover=eta.tolist(), savings=float(sav.value))


def ada_profile_enable(on: bool) -> None:
    lib().ada_profile_enable(int(bool(on)))


def ada_profile_collect() -> Dict[str, Dict[str, float]]:
    """Per kernel class: summed event-pair milliseconds and launch count since the last collect."""
    n = len(KERNEL_CLASSES)
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int * n)()
    rc = lib().ada_profile_collect(ctypes.cast(ms, ctypes.c_void_p), ctypes.cast(cnt, ctypes.c_void_p))
    if rc != OK:
        raise AdaError(rc, "ada_profile_collect")
    return {k: dict(ms=float(ms[i]), launches=int(cnt[i])) for i, k in enumerate(KERNEL_CLASSES)}


def ada_profile_copy_probe(dst: torch.Tensor, src: torch.Tensor, *, stream=None) -> None:
    """Plain copy kernel of known size (the yardstick for traffic counters)."""
    n = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != n:
        raise ValueError("dst and src must have the same size in bytes")
    rc = lib().ada_profile_copy_probe(_ptr(dst), _ptr(src), n, _stream(stream))
    if rc != OK:
        raise AdaError(rc, "ada_profile_copy_probe")


def fetch(res: Dict[str, torch.Tensor]) -> Dict[str, object]:
    """Synchronise and bring one ada_select_full / ada_cascade_step result to the host, trimmed to its counts."""
    counts = res["counts"].cpu().tolist()
    if counts[3] != OK:
        raise AdaError(counts[3], "device status")
    out: Dict[str, object] = dict(r=counts[0], n_adds=counts[1], n_removes=counts[2])
    out["idx"] = res["idx"][:counts[0]].cpu().numpy()
    if "mask" in res:
        out["mask"] = res["mask"].cpu().numpy()
    if "adds" in res:
        out["adds"] = res["adds"][:counts[1]].cpu().numpy()
        out["removes"] = res["removes"][:counts[2]].cpu().numpy()
        out["gram_ops"] = int(res["gram_ops"].cpu().item())
    out["gamma"] = res["gamma"].cpu().numpy()
    return out


def ada_profile_mfma_probe(workgroups: int, iters: int, *, device="cuda", stream=None) -> float:
    """Launch the matrix-instruction-only kernel; returns the flops it performs (time it via ada_profile_collect)."""
    sink = torch.zeros(int(workgroups), dtype=torch.float32, device=device)
    rc = lib().ada_profile_mfma_probe(int(workgroups), int(iters), _ptr(sink), _stream(stream))
    if rc != OK:
        raise AdaError(rc, "ada_profile_mfma_probe")
    return float(workgroups) * 4.0 * float(iters) * 16.0 * 32768.0
