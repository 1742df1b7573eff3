"""Thin ctypes binding over the C-ABI HIP library (argument marshalling only).

Function names mirror include/mgrit.h.  PyTorch is used for device memory and
streams; every computation happens inside the library's kernels.  There is no
CPU fallback: if the shared library is missing, loading fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmgrit_hip.so")

MGRIT_OK = 0
MGRIT_INVALID_ARG, MGRIT_UNSUPPORTED, MGRIT_WORKSPACE_TOO_SMALL, MGRIT_HIP_ERROR = -1, -2, -3, -4
P_NAMES = ["ln1_g", "ln1_b", "bqkv", "bo", "ln2_g", "ln2_b", "b1", "b2", "ln3_g", "ln3_b", "bq_c",
           "bkv_c", "bo_c", "Wqkv", "Wo", "W1", "W2", "Wq_c", "Wkv_c", "Wo_c"]
P_COUNT = len(P_NAMES)


class Indicator(C.Structure):
    """mgrit_indicator: the host-side inexactness controller (plain data)."""
    _fields_ = [("iters", C.c_int32), ("probe_every", C.c_int32), ("mitigation", C.c_int32),
                ("max_iters", C.c_int32), ("threshold", C.c_float), ("last_factor", C.c_float),
                ("batch", C.c_int64), ("serial", C.c_int32), ("probing", C.c_int32), ("failures", C.c_int32),
                ("reserved", C.c_int32)]


MITIGATE_SERIAL, MITIGATE_MORE_ITERATIONS = 0, 1


class BufferOpts(C.Structure):
    _fields_ = [("n_open", C.c_int32), ("n_close", C.c_int32), ("h_buffer", C.c_float)]


class ModelDesc(C.Structure):
    _fields_ = [("arch", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_ff", C.c_int32),
                ("batch", C.c_int32), ("seq", C.c_int32), ("mem_seq", C.c_int32), ("dtype", C.c_int32),
                ("ln_eps", C.c_float)]


class Opts(C.Structure):
    _fields_ = [("N", C.c_int32), ("h", C.c_float), ("cf", C.c_int32), ("levels", C.c_int32),
                ("iters", C.c_int32), ("relax", C.c_int32), ("init_guess", C.c_int32)]


class ThetaLayout(C.Structure):
    _fields_ = [("block_bytes", C.c_int64), ("offset", C.c_int64 * P_COUNT), ("rows", C.c_int32 * P_COUNT),
                ("cols", C.c_int32 * P_COUNT), ("elem_bytes", C.c_int32 * P_COUNT)]


class MgritError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().mgrit_status_string(status).decode()
        hip = lib().mgrit_last_hip_error() if status == -4 else 0
        super().__init__(f"{where}: {msg} (status {status}" + (f", hipError {hip})" if hip else ")"))


_lib = None


def lib() -> C.CDLL:
    """Load the HIP library (built by `python -m paper_2601_09026_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2601_09026_amd.build` (no CPU fallback exists)")
        L = C.CDLL(LIB_PATH)
        vp, vpp = C.c_void_p, C.POINTER(C.c_void_p)
        L.mgrit_theta_layout.argtypes = [C.POINTER(ModelDesc), C.POINTER(ThetaLayout)]
        L.mgrit_theta_layout.restype = C.c_int
        L.mgrit_workspace_bytes.argtypes = [C.POINTER(ModelDesc), C.POINTER(Opts), C.c_int]
        L.mgrit_workspace_bytes.restype = C.c_size_t
        L.mgrit_layer_step_workspace_bytes.argtypes = [C.POINTER(ModelDesc), C.c_int, C.c_int]
        L.mgrit_layer_step_workspace_bytes.restype = C.c_size_t
        L.mgrit_step_evaluations.argtypes = [C.POINTER(Opts)]
        L.mgrit_step_evaluations.restype = C.c_int64
        L.mgrit_measure_mfma_ceiling.argtypes = [C.c_void_p, C.c_size_t, C.c_int, C.POINTER(C.c_double), C.c_void_p]
        L.mgrit_measure_mfma_ceiling.restype = C.c_int
        L.mgrit_measure_copy_ceiling.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.POINTER(C.c_double), C.c_void_p]
        L.mgrit_measure_copy_ceiling.restype = C.c_int
        L.mgrit_step_depth.argtypes = [C.POINTER(Opts)]
        L.mgrit_step_depth.restype = C.c_int64
        L.mgrit_forward.argtypes = [C.POINTER(ModelDesc), C.POINTER(Opts), vp, vpp, vp, vp, vp, vp,
                                    C.c_size_t, vp]
        L.mgrit_forward.restype = C.c_int
        L.mgrit_adjoint.argtypes = [C.POINTER(ModelDesc), C.POINTER(Opts), vp, vpp, vp, vp, vp, vp, vpp, vp,
                                    vp, C.c_size_t, vp]
        L.mgrit_adjoint.restype = C.c_int
        L.mgrit_forward_linearising.argtypes = [C.POINTER(ModelDesc), C.POINTER(Opts), vp, vpp, vp, vp, vp, vp,
                                                C.c_size_t, vp, C.c_size_t, C.c_int, vp]
        L.mgrit_forward_linearising.restype = C.c_int
        L.mgrit_adjoint_linearised.argtypes = L.mgrit_adjoint.argtypes
        L.mgrit_adjoint_linearised.restype = C.c_int
        L.layer_step_batched.argtypes = [C.POINTER(ModelDesc), C.c_int, C.c_int, vpp, vpp, vpp, vpp, vpp, vp,
                                         C.c_float, vp, C.c_size_t, vp]
        L.layer_step_batched.restype = C.c_int
        L.mgrit_layer_step_static_bytes.argtypes = [C.POINTER(ModelDesc), C.c_int, C.c_int]
        L.mgrit_layer_step_static_bytes.restype = C.c_size_t
        L.layer_step_batched_static.argtypes = [C.POINTER(ModelDesc), C.c_int, C.c_int, vpp, vpp, vpp, vpp, vpp, vp,
                                                C.c_float, vp]
        L.layer_step_batched_static.restype = C.c_int
        L.mgrit_buffered_workspace_bytes.argtypes = [C.POINTER(ModelDesc), C.POINTER(Opts), C.POINTER(BufferOpts),
                                                     C.c_int]
        L.mgrit_buffered_workspace_bytes.restype = C.c_size_t
        L.mgrit_forward_buffered.argtypes = [C.POINTER(ModelDesc), C.POINTER(Opts), C.POINTER(BufferOpts), vp, vpp,
                                             vp, vp, vp, vp, C.c_size_t, vp]
        L.mgrit_forward_buffered.restype = C.c_int
        L.mgrit_adjoint_buffered.argtypes = [C.POINTER(ModelDesc), C.POINTER(Opts), C.POINTER(BufferOpts), vp, vpp,
                                             vp, vp, vp, vp, vpp, vp, vp, C.c_size_t, vp]
        L.mgrit_adjoint_buffered.restype = C.c_int
        L.mgrit_buffered_linearised_workspace_bytes.argtypes = [C.POINTER(ModelDesc), C.POINTER(Opts),
                                                                C.POINTER(BufferOpts), C.c_int]
        L.mgrit_buffered_linearised_workspace_bytes.restype = C.c_size_t
        L.mgrit_forward_buffered_linearising.argtypes = [C.POINTER(ModelDesc), C.POINTER(Opts), C.POINTER(BufferOpts),
                                                         vp, vpp, vp, vp, vp, vp, C.c_size_t, vp, C.c_size_t, C.c_int,
                                                         vp]
        L.mgrit_forward_buffered_linearising.restype = C.c_int
        L.mgrit_adjoint_buffered_linearised.argtypes = L.mgrit_adjoint_buffered.argtypes
        L.mgrit_adjoint_buffered_linearised.restype = C.c_int
        L.mgrit_stacked_workspace_bytes.argtypes = [C.POINTER(ModelDesc), C.POINTER(Opts), C.c_int, C.c_int]
        L.mgrit_stacked_workspace_bytes.restype = C.c_size_t
        L.mgrit_forward_stacked.argtypes = [C.POINTER(ModelDesc), C.POINTER(Opts), C.c_int, vp, vpp, vp, vp, vp,
                                            C.c_size_t, vp]
        L.mgrit_forward_stacked.restype = C.c_int
        L.mgrit_adjoint_stacked.argtypes = [C.POINTER(ModelDesc), C.POINTER(Opts), C.c_int, vp, vpp, vp, vp, vpp, vp,
                                            vp, C.c_size_t, vp]
        L.mgrit_adjoint_stacked.restype = C.c_int
        L.mgrit_forward_stacked_linearising.argtypes = [C.POINTER(ModelDesc), C.POINTER(Opts), C.c_int, vp, vpp, vp,
                                                        vp, vp, C.c_size_t, vp, C.c_size_t, C.c_int, vp]
        L.mgrit_forward_stacked_linearising.restype = C.c_int
        L.mgrit_adjoint_stacked_linearised.argtypes = L.mgrit_adjoint_stacked.argtypes
        L.mgrit_adjoint_stacked_linearised.restype = C.c_int
        L.mgrit_indicator_init.argtypes = [C.POINTER(Indicator), C.c_int, C.c_int, C.c_int, C.c_int, C.c_float]
        L.mgrit_indicator_init.restype = C.c_int
        L.mgrit_indicator_begin_batch.argtypes = [C.POINTER(Indicator)]
        L.mgrit_indicator_begin_batch.restype = C.c_int
        L.mgrit_indicator_end_batch.argtypes = [C.POINTER(Indicator), C.POINTER(C.c_float), C.c_int]
        L.mgrit_indicator_end_batch.restype = C.c_int
        L.mgrit_status_string.argtypes = [C.c_int]
        L.mgrit_status_string.restype = C.c_char_p
        L.mgrit_last_hip_error.argtypes = []
        L.mgrit_last_hip_error.restype = C.c_int
        L.mgrit_set_max_groups_per_launch.argtypes = [C.c_int]
        L.mgrit_set_max_groups_per_launch.restype = None
        L.mgrit_default_groups_per_launch.argtypes = [C.POINTER(ModelDesc), C.c_int]
        L.mgrit_default_groups_per_launch.restype = C.c_int
        L.mgrit_debug_pipeline_chunk.argtypes = [C.c_int]
        L.mgrit_debug_pipeline_chunk.restype = None
        L.mgrit_set_lanes.argtypes = [C.c_int]
        L.mgrit_set_lanes.restype = None
        L.mgrit_debug_force_simple_kernels.argtypes = [C.c_int, C.c_int]
        L.mgrit_debug_force_simple_kernels.restype = None
        L.mgrit_debug_gemm_tile_config.argtypes = [C.c_int]
        L.mgrit_debug_gemm_tile_config.restype = None
        L.mgrit_debug_attention_wide_blocks.argtypes = [C.c_int]
        L.mgrit_debug_attention_wide_blocks.restype = None
        L.mgrit_debug_pipeline_coarse_solve.argtypes = [C.c_int]
        L.mgrit_debug_pipeline_coarse_solve.restype = None
        L.mgrit_profile_enable.argtypes = [C.c_int]
        L.mgrit_profile_enable.restype = C.c_int
        L.mgrit_profile_reset.argtypes = []
        L.mgrit_profile_reset.restype = None
        L.mgrit_profile_read.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                         C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.mgrit_profile_read.restype = C.c_int
        _lib = L
    return _lib


# ------------------------------------------------------------------ descriptors
def model_desc(wl) -> ModelDesc:
    """ModelDesc from any object with the Workload fields."""
    return ModelDesc(wl.arch, wl.d_model, wl.n_heads, wl.d_ff, wl.batch, wl.seq, wl.mem_seq, wl.dtype,
                     wl.ln_eps)


def mgrit_opts(N, h, cf, levels, iters, relax=1, init_guess=0) -> Opts:
    return Opts(N, h, cf, levels, iters, relax, init_guess)


def mgrit_theta_layout(desc: ModelDesc) -> ThetaLayout:
    out = ThetaLayout()
    st = lib().mgrit_theta_layout(C.byref(desc), C.byref(out))
    if st != MGRIT_OK:
        raise MgritError(st, "mgrit_theta_layout")
    return out


def mgrit_workspace_bytes(desc: ModelDesc, opts: Opts, adjoint) -> int:
    """adjoint: 0/False forward, 1/True adjoint, 2 adjoint with parameter gradients."""
    return int(lib().mgrit_workspace_bytes(C.byref(desc), C.byref(opts), int(adjoint)))


def grad_layout(desc: ModelDesc) -> ThetaLayout:
    """Layout of a gradient block: the fp32 parameter block of the same model."""
    d32 = ModelDesc.from_buffer_copy(desc)
    d32.dtype = 0
    return mgrit_theta_layout(d32)


def unpack_grad(desc: ModelDesc, block: torch.Tensor) -> Dict[str, np.ndarray]:
    """Copies a gradient block (uint8 device tensor) back into named float32 arrays."""
    lay = grad_layout(desc)
    raw = block.cpu().numpy()
    out = {}
    for i, name in enumerate(P_NAMES):
        if lay.offset[i] < 0:
            continue
        n = lay.rows[i] * lay.cols[i]
        a = raw[lay.offset[i]:lay.offset[i] + 4 * n].view(np.float32)
        out[name] = a.reshape(lay.rows[i], lay.cols[i]) if lay.cols[i] > 1 else a.copy()
    return out


def mgrit_layer_step_workspace_bytes(desc: ModelDesc, adjoint: bool, n_groups: int) -> int:
    return int(lib().mgrit_layer_step_workspace_bytes(C.byref(desc), int(adjoint), n_groups))


def mgrit_step_evaluations(opts: Opts) -> int:
    return int(lib().mgrit_step_evaluations(C.byref(opts)))


def mgrit_step_depth(opts: Opts) -> int:
    return int(lib().mgrit_step_depth(C.byref(opts)))


def mgrit_indicator_init(iters: int, probe_every: int, mitigation: int = MITIGATE_SERIAL, max_iters: int = 0,
                         threshold: float = 1.0) -> Indicator:
    ind = Indicator()
    st = lib().mgrit_indicator_init(C.byref(ind), iters, probe_every, mitigation, max_iters, threshold)
    if st != MGRIT_OK:
        raise MgritError(st, "mgrit_indicator_init")
    return ind


def mgrit_indicator_begin_batch(ind: Indicator) -> int:
    return int(lib().mgrit_indicator_begin_batch(C.byref(ind)))


def mgrit_indicator_end_batch(ind: Indicator, resnorm) -> int:
    r = np.ascontiguousarray(resnorm, dtype=np.float32)
    return int(lib().mgrit_indicator_end_batch(C.byref(ind), r.ctypes.data_as(C.POINTER(C.c_float)), r.size))


def mgrit_set_max_groups_per_launch(n: int) -> None:
    lib().mgrit_set_max_groups_per_launch(int(n))


def mgrit_set_lanes(n: int) -> None:
    lib().mgrit_set_lanes(int(n))


def mgrit_set_adjoint_cache(on: bool) -> None:
    """False: no N-layer linearisation cache in the adjoint workspace (recomputed per launch chunk)."""
    lib().mgrit_set_adjoint_cache(int(bool(on)))


PROFILE_CLASSES = {0: "gemm_generic", 1: "attn_fwd", 2: "attn_bwd", 3: "ln_fwd", 4: "ln_vjp", 5: "elementwise",
                   6: "ln_fwd_single", 7: "ln_vjp_single",
                   8: "gemm_mfma_store", 9: "gemm_mfma_gelu", 10: "gemm_mfma_sublayer_sum",
                   11: "gemm_mfma_euler", 12: "gemm_mfma_dgelu", 13: "gemm_mfma_store_f32",
                   14: "gemm_mfma_gelu_prime", 15: "gemm_mfma_gelu_both"}
# the same epilogues launched over a single group (the serial coarse chain)
PROFILE_CLASSES.update({c + 8: n.replace("gemm_mfma_", "gemm_mfma_single_") for c, n in list(PROFILE_CLASSES.items())
                        if c >= 8})


def mgrit_profile_enable(max_records: int) -> None:
    st = lib().mgrit_profile_enable(int(max_records))
    if st != MGRIT_OK:
        raise MgritError(st, "mgrit_profile_enable")


def mgrit_profile_reset() -> None:
    lib().mgrit_profile_reset()


def mgrit_profile_read() -> Dict[str, dict]:
    """Totals per kernel class since the last reset (synchronise the stream first)."""
    out = {}
    for cls, name in PROFILE_CLASSES.items():
        ms, fl, by, n = C.c_double(), C.c_double(), C.c_double(), C.c_int64()
        st = lib().mgrit_profile_read(cls, C.byref(ms), C.byref(fl), C.byref(by), C.byref(n))
        if st not in (0, -3):
            raise MgritError(st, "mgrit_profile_read")
        if n.value:
            out[name] = {"ms": ms.value, "flops": fl.value, "bytes": by.value, "launches": n.value,
                         "overflow": st == -3}
    return out


def mgrit_measure_mfma_ceiling(scratch: torch.Tensor, iters: int = 20000, stream=None) -> float:
    """TFLOP/s of the register-resident MFMA loop (scratch: device tensor of at least 512 KiB)."""
    out = C.c_double()
    st = lib().mgrit_measure_mfma_ceiling(scratch.data_ptr(), scratch.numel() * scratch.element_size(), int(iters),
                                          C.byref(out), _stream_handle(stream))
    if st != MGRIT_OK:
        raise MgritError(st, "mgrit_measure_mfma_ceiling")
    return out.value


def mgrit_measure_copy_ceiling(src: torch.Tensor, dst: torch.Tensor, stream=None) -> float:
    """GB/s (read + written) of a grid-stride copy of src into dst (device tensors of equal size)."""
    out = C.c_double()
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    st = lib().mgrit_measure_copy_ceiling(src.data_ptr(), dst.data_ptr(), nbytes, C.byref(out), _stream_handle(stream))
    if st != MGRIT_OK:
        raise MgritError(st, "mgrit_measure_copy_ceiling")
    return out.value


def mgrit_measure_event_bracket(stream=None) -> float:
    """Microseconds that an event pair adds to the launch it brackets (median around an empty kernel)."""
    out = C.c_double()
    st = lib().mgrit_measure_event_bracket(C.byref(out), _stream_handle(stream))
    if st != MGRIT_OK:
        raise MgritError(st, "mgrit_measure_event_bracket")
    return out.value


# ------------------------------------------------------------------ parameter packing (byte copies only)
def pack_theta(desc: ModelDesc, params: Dict[str, np.ndarray], device="cuda") -> torch.Tensor:
    """One layer's named fp32 arrays -> packed device block (uint8 tensor) in the library's layout."""
    lay = mgrit_theta_layout(desc)
    host = torch.zeros(int(lay.block_bytes), dtype=torch.uint8)
    for i, name in enumerate(P_NAMES):
        off = int(lay.offset[i])
        if off < 0:
            continue
        a = torch.from_numpy(np.ascontiguousarray(params[name], dtype=np.float32))
        assert a.numel() == lay.rows[i] * lay.cols[i], name
        if lay.elem_bytes[i] == 2:
            raw = a.to(torch.bfloat16).view(torch.uint8).reshape(-1)
        else:
            raw = a.view(torch.uint8).reshape(-1)
        host[off:off + raw.numel()] = raw
    return host.to(device)


def _ptr(t: Optional[torch.Tensor]) -> C.c_void_p:
    return C.c_void_p(0 if t is None else t.data_ptr())


def _ptr_array(ts: Optional[Sequence[torch.Tensor]]):
    if ts is None:
        return None
    arr = (C.c_void_p * len(ts))(*[t.data_ptr() for t in ts])
    return arr


def _stream_handle(stream: Optional[torch.cuda.Stream]) -> C.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _check_state(t: torch.Tensor, shape, name: str):
    if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and tuple(t.shape) == tuple(shape)):
        raise ValueError(f"{name}: expected contiguous fp32 device tensor of shape {tuple(shape)}, "
                         f"got {t.dtype} {tuple(t.shape)} on {t.device}")


# ------------------------------------------------------------------ entry points
def mgrit_forward(desc: ModelDesc, opts: Opts, Z0: torch.Tensor, theta: List[torch.Tensor],
                  memory: Optional[torch.Tensor] = None, Z_all: Optional[torch.Tensor] = None,
                  resnorm: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                  stream: Optional[torch.cuda.Stream] = None, adjoint_workspace: Optional[torch.Tensor] = None,
                  with_gradients: bool = False):
    """Returns (Z_all [(N+1),T,d], resnorm [iters]).  Buffers are allocated here if not given.
    adjoint_workspace: call mgrit_forward_linearising instead, which also leaves the internals of its
    closing relaxation there for mgrit_adjoint(..., workspace=adjoint_workspace, linearised=True)."""
    T, d = desc.batch * desc.seq, desc.d_model
    _check_state(Z0, (T, d), "Z0")
    if len(theta) != opts.N:
        raise ValueError("theta must hold N blocks")
    if Z_all is None:
        Z_all = torch.empty((opts.N + 1, T, d), dtype=torch.float32, device=Z0.device)
    _check_state(Z_all, (opts.N + 1, T, d), "Z_all")
    if resnorm is None:
        resnorm = torch.zeros(max(opts.iters, 1), dtype=torch.float32, device=Z0.device)
    need = mgrit_workspace_bytes(desc, opts, False)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=Z0.device)
    if adjoint_workspace is not None:
        st = lib().mgrit_forward_linearising(C.byref(desc), C.byref(opts), _ptr(Z0), _ptr_array(theta), _ptr(memory),
                                             _ptr(Z_all), _ptr(resnorm), _ptr(workspace), workspace.numel(),
                                             _ptr(adjoint_workspace), adjoint_workspace.numel(),
                                             int(bool(with_gradients)), _stream_handle(stream))
        if st != MGRIT_OK:
            raise MgritError(st, "mgrit_forward_linearising")
        return Z_all, resnorm
    st = lib().mgrit_forward(C.byref(desc), C.byref(opts), _ptr(Z0), _ptr_array(theta), _ptr(memory),
                             _ptr(Z_all), _ptr(resnorm), _ptr(workspace), workspace.numel(),
                             _stream_handle(stream))
    if st != MGRIT_OK:
        raise MgritError(st, "mgrit_forward")
    return Z_all, resnorm


def mgrit_adjoint(desc: ModelDesc, opts: Opts, Z_all: torch.Tensor, theta: List[torch.Tensor],
                  lambda_N: torch.Tensor, memory: Optional[torch.Tensor] = None,
                  lambda_all: Optional[torch.Tensor] = None, resnorm: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None,
                  dtheta: Optional[List[torch.Tensor]] = None, dmemory: Optional[torch.Tensor] = None,
                  linearised: bool = False):
    """Returns (lambda_all [(N+1),T,d], resnorm [iters]).  dtheta: N uint8 device tensors of
    grad_layout(desc).block_bytes each, filled with the parameter gradients; dmemory: fp32
    [batch*mem_seq, d] device tensor filled with the gradient of the cross-attention memory.
    linearised: call mgrit_adjoint_linearised (workspace = the adjoint_workspace that mgrit_forward filled)."""
    T, d = desc.batch * desc.seq, desc.d_model
    _check_state(Z_all, (opts.N + 1, T, d), "Z_all")
    _check_state(lambda_N, (T, d), "lambda_N")
    if len(theta) != opts.N:
        raise ValueError("theta must hold N blocks")
    if lambda_all is None:
        lambda_all = torch.empty((opts.N + 1, T, d), dtype=torch.float32, device=Z_all.device)
    _check_state(lambda_all, (opts.N + 1, T, d), "lambda_all")
    if resnorm is None:
        resnorm = torch.zeros(max(opts.iters, 1), dtype=torch.float32, device=Z_all.device)
    if dtheta is not None and len(dtheta) != opts.N:
        raise ValueError("dtheta must hold N blocks")
    if dmemory is not None:
        _check_state(dmemory, (desc.batch * desc.mem_seq, d), "dmemory")
    need = mgrit_workspace_bytes(desc, opts, 2 if (dtheta is not None or dmemory is not None) else 1)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=Z_all.device)
    if linearised and workspace is None:
        raise ValueError("linearised: pass the adjoint workspace that the forward call filled")
    entry = lib().mgrit_adjoint_linearised if linearised else lib().mgrit_adjoint
    st = entry(C.byref(desc), C.byref(opts), _ptr(Z_all), _ptr_array(theta), _ptr(memory),
               _ptr(lambda_N), _ptr(lambda_all), _ptr(dmemory), _ptr_array(dtheta), _ptr(resnorm),
               _ptr(workspace), workspace.numel(), _stream_handle(stream))
    if st != MGRIT_OK:
        raise MgritError(st, "mgrit_adjoint_linearised" if linearised else "mgrit_adjoint")
    return lambda_all, resnorm


def layer_step_batched(desc: ModelDesc, adjoint: bool, inputs: List[torch.Tensor], outputs: List[torch.Tensor],
                       theta: List[torch.Tensor], hstep: float,
                       lin_state: Optional[List[torch.Tensor]] = None,
                       rhs: Optional[List[torch.Tensor]] = None, memory: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None):
    """out[g] = in[g] + hstep*F(in[g]; theta[g]) (+rhs[g]), or its adjoint at lin_state[g]."""
    G = len(inputs)
    T, d = desc.batch * desc.seq, desc.d_model
    for t in list(inputs) + list(outputs) + list(lin_state or []) + list(rhs or []):
        _check_state(t, (T, d), "state")
    need = mgrit_layer_step_workspace_bytes(desc, adjoint, G)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=inputs[0].device)
    st = lib().layer_step_batched(C.byref(desc), int(adjoint), G, _ptr_array(inputs), _ptr_array(outputs),
                                  _ptr_array(theta), _ptr_array(lin_state), _ptr_array(rhs), _ptr(memory),
                                  float(hstep), _ptr(workspace), workspace.numel(), _stream_handle(stream))
    if st != MGRIT_OK:
        raise MgritError(st, "layer_step_batched")
    return outputs


STATIC_SCRATCH_BYTES = 256 << 20     # MGRIT_STATIC_SCRATCH_BYTES of the header


def mgrit_layer_step_static_bytes(desc: ModelDesc, adjoint: bool, n_groups: int) -> int:
    return int(lib().mgrit_layer_step_static_bytes(C.byref(desc), int(adjoint), n_groups))


def layer_step_batched_static(desc: ModelDesc, adjoint: bool, inputs: List[torch.Tensor],
                              outputs: List[torch.Tensor], theta: List[torch.Tensor], hstep: float,
                              lin_state: Optional[List[torch.Tensor]] = None,
                              rhs: Optional[List[torch.Tensor]] = None, memory: Optional[torch.Tensor] = None,
                              stream: Optional[torch.cuda.Stream] = None):
    """layer_step_batched on the library's own fixed scratch array: no workspace, nothing allocated."""
    G = len(inputs)
    T, d = desc.batch * desc.seq, desc.d_model
    for t in list(inputs) + list(outputs) + list(lin_state or []) + list(rhs or []):
        _check_state(t, (T, d), "state")
    st = lib().layer_step_batched_static(C.byref(desc), int(adjoint), G, _ptr_array(inputs), _ptr_array(outputs),
                                         _ptr_array(theta), _ptr_array(lin_state), _ptr_array(rhs), _ptr(memory),
                                         float(hstep), _stream_handle(stream))
    if st != MGRIT_OK:
        raise MgritError(st, "layer_step_batched_static")
    return outputs


def mgrit_buffered_workspace_bytes(desc: ModelDesc, opts: Opts, buf: BufferOpts, adjoint) -> int:
    return int(lib().mgrit_buffered_workspace_bytes(C.byref(desc), C.byref(opts), C.byref(buf), int(adjoint)))


def mgrit_buffered_linearised_workspace_bytes(desc: ModelDesc, opts: Opts, buf: BufferOpts, with_gradients) -> int:
    return int(lib().mgrit_buffered_linearised_workspace_bytes(C.byref(desc), C.byref(opts), C.byref(buf),
                                                               int(bool(with_gradients))))


def mgrit_forward_buffered(desc: ModelDesc, opts: Opts, buf: BufferOpts, Z0: torch.Tensor,
                           theta: List[torch.Tensor], memory: Optional[torch.Tensor] = None,
                           stream: Optional[torch.cuda.Stream] = None,
                           adjoint_workspace: Optional[torch.Tensor] = None, with_gradients: bool = False):
    """Serial open / close layers around the MGRIT middle.  Returns (Z_all, resnorm).
    adjoint_workspace (mgrit_buffered_linearised_workspace_bytes): mgrit_forward_buffered_linearising."""
    T, d = desc.batch * desc.seq, desc.d_model
    n = buf.n_open + opts.N + buf.n_close
    _check_state(Z0, (T, d), "Z0")
    if len(theta) != n:
        raise ValueError("theta must hold n_open + N + n_close blocks")
    Z_all = torch.empty((n + 1, T, d), dtype=torch.float32, device=Z0.device)
    resnorm = torch.zeros(max(opts.iters, 1), dtype=torch.float32, device=Z0.device)
    ws = torch.empty(max(mgrit_buffered_workspace_bytes(desc, opts, buf, 0), 256), dtype=torch.uint8, device=Z0.device)
    if adjoint_workspace is not None:
        st = lib().mgrit_forward_buffered_linearising(C.byref(desc), C.byref(opts), C.byref(buf), _ptr(Z0),
                                                      _ptr_array(theta), _ptr(memory), _ptr(Z_all), _ptr(resnorm),
                                                      _ptr(ws), ws.numel(), _ptr(adjoint_workspace),
                                                      adjoint_workspace.numel(), int(bool(with_gradients)),
                                                      _stream_handle(stream))
        if st != MGRIT_OK:
            raise MgritError(st, "mgrit_forward_buffered_linearising")
        return Z_all, resnorm
    st = lib().mgrit_forward_buffered(C.byref(desc), C.byref(opts), C.byref(buf), _ptr(Z0), _ptr_array(theta),
                                      _ptr(memory), _ptr(Z_all), _ptr(resnorm), _ptr(ws), ws.numel(),
                                      _stream_handle(stream))
    if st != MGRIT_OK:
        raise MgritError(st, "mgrit_forward_buffered")
    return Z_all, resnorm


def mgrit_adjoint_buffered(desc: ModelDesc, opts: Opts, buf: BufferOpts, Z_all: torch.Tensor,
                           theta: List[torch.Tensor], lambda_N: torch.Tensor, memory: Optional[torch.Tensor] = None,
                           dtheta: Optional[List[torch.Tensor]] = None,
                           stream: Optional[torch.cuda.Stream] = None, workspace: Optional[torch.Tensor] = None,
                           linearised: bool = False):
    """Returns (lambda_all, resnorm) of the buffered network; dtheta as in mgrit_adjoint.
    linearised: mgrit_adjoint_buffered_linearised on the workspace the forward call filled."""
    T, d = desc.batch * desc.seq, desc.d_model
    n = buf.n_open + opts.N + buf.n_close
    _check_state(Z_all, (n + 1, T, d), "Z_all")
    _check_state(lambda_N, (T, d), "lambda_N")
    if len(theta) != n or (dtheta is not None and len(dtheta) != n):
        raise ValueError("theta / dtheta must hold n_open + N + n_close blocks")
    lambda_all = torch.empty_like(Z_all)
    resnorm = torch.zeros(max(opts.iters, 1), dtype=torch.float32, device=Z_all.device)
    if linearised and workspace is None:
        raise ValueError("linearised: pass the adjoint workspace that the forward call filled")
    need = mgrit_buffered_workspace_bytes(desc, opts, buf, 2 if dtheta is not None else 1)
    ws = workspace if workspace is not None else torch.empty(max(need, 256), dtype=torch.uint8, device=Z_all.device)
    entry = lib().mgrit_adjoint_buffered_linearised if linearised else lib().mgrit_adjoint_buffered
    st = entry(C.byref(desc), C.byref(opts), C.byref(buf), _ptr(Z_all), _ptr_array(theta),
               _ptr(memory), _ptr(lambda_N), _ptr(lambda_all), None, _ptr_array(dtheta),
               _ptr(resnorm), _ptr(ws), ws.numel(), _stream_handle(stream))
    if st != MGRIT_OK:
        raise MgritError(st, "mgrit_adjoint_buffered_linearised" if linearised else "mgrit_adjoint_buffered")
    return lambda_all, resnorm


# ---- stacked encoder-decoder grid -------------------------------------------------------------
def encoder_desc(desc: ModelDesc) -> ModelDesc:
    """The encoder half of a stacked grid described by its decoder `desc`."""
    return ModelDesc(0, desc.d_model, desc.n_heads, desc.d_ff, desc.batch, desc.mem_seq, 0, desc.dtype, desc.ln_eps)


def mgrit_stacked_workspace_bytes(desc: ModelDesc, opts: Opts, n_enc: int, adjoint: int) -> int:
    return int(lib().mgrit_stacked_workspace_bytes(C.byref(desc), C.byref(opts), int(n_enc), int(adjoint)))


def mgrit_forward_stacked(desc: ModelDesc, opts: Opts, n_enc: int, Z0: torch.Tensor, theta: List[torch.Tensor],
                          Z_all: Optional[torch.Tensor] = None, resnorm: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None,
                          adjoint_workspace: Optional[torch.Tensor] = None, with_gradients: bool = False):
    """One MGRIT grid over n_enc encoder layers followed by decoder layers; state rows = encoder
    tokens then decoder tokens.  Returns (Z_all, resnorm).  Buffers are allocated here if not given.
    adjoint_workspace: mgrit_forward_stacked_linearising (see mgrit_forward)."""
    T, d = desc.batch * (desc.mem_seq + desc.seq), desc.d_model
    _check_state(Z0, (T, d), "Z0")
    if len(theta) != opts.N:
        raise ValueError("theta must hold N blocks")
    if Z_all is None:
        Z_all = torch.empty((opts.N + 1, T, d), dtype=torch.float32, device=Z0.device)
    _check_state(Z_all, (opts.N + 1, T, d), "Z_all")
    if resnorm is None:
        resnorm = torch.zeros(max(opts.iters, 1), dtype=torch.float32, device=Z0.device)
    if workspace is None:
        workspace = torch.empty(max(mgrit_stacked_workspace_bytes(desc, opts, n_enc, 0), 256), dtype=torch.uint8,
                                device=Z0.device)
    if adjoint_workspace is not None:
        st = lib().mgrit_forward_stacked_linearising(C.byref(desc), C.byref(opts), int(n_enc), _ptr(Z0),
                                                     _ptr_array(theta), _ptr(Z_all), _ptr(resnorm), _ptr(workspace),
                                                     workspace.numel(), _ptr(adjoint_workspace),
                                                     adjoint_workspace.numel(), int(bool(with_gradients)),
                                                     _stream_handle(stream))
        if st != MGRIT_OK:
            raise MgritError(st, "mgrit_forward_stacked_linearising")
        return Z_all, resnorm
    st = lib().mgrit_forward_stacked(C.byref(desc), C.byref(opts), int(n_enc), _ptr(Z0), _ptr_array(theta),
                                     _ptr(Z_all), _ptr(resnorm), _ptr(workspace), workspace.numel(),
                                     _stream_handle(stream))
    if st != MGRIT_OK:
        raise MgritError(st, "mgrit_forward_stacked")
    return Z_all, resnorm


def mgrit_adjoint_stacked(desc: ModelDesc, opts: Opts, n_enc: int, Z_all: torch.Tensor, theta: List[torch.Tensor],
                          lambda_N: torch.Tensor, dtheta: Optional[List[torch.Tensor]] = None,
                          lambda_all: Optional[torch.Tensor] = None, resnorm: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None, stream: Optional[torch.cuda.Stream] = None,
                          linearised: bool = False):
    """Returns (lambda_all, resnorm) of the stacked grid; dtheta as in mgrit_adjoint (encoder
    layers' blocks in the encoder's fp32 layout, decoder layers' in the decoder's).
    linearised: mgrit_adjoint_stacked_linearised on the workspace the forward call filled."""
    T, d = desc.batch * (desc.mem_seq + desc.seq), desc.d_model
    _check_state(Z_all, (opts.N + 1, T, d), "Z_all")
    _check_state(lambda_N, (T, d), "lambda_N")
    if len(theta) != opts.N or (dtheta is not None and len(dtheta) != opts.N):
        raise ValueError("theta / dtheta must hold N blocks")
    if lambda_all is None:
        lambda_all = torch.empty_like(Z_all)
    _check_state(lambda_all, (opts.N + 1, T, d), "lambda_all")
    if resnorm is None:
        resnorm = torch.zeros(max(opts.iters, 1), dtype=torch.float32, device=Z_all.device)
    if workspace is None:
        need = mgrit_stacked_workspace_bytes(desc, opts, n_enc, 2 if dtheta is not None else 1)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=Z_all.device)
    entry = lib().mgrit_adjoint_stacked_linearised if linearised else lib().mgrit_adjoint_stacked
    st = entry(C.byref(desc), C.byref(opts), int(n_enc), _ptr(Z_all), _ptr_array(theta),
               _ptr(lambda_N), _ptr(lambda_all), _ptr_array(dtheta), _ptr(resnorm),
               _ptr(workspace), workspace.numel(), _stream_handle(stream))
    if st != MGRIT_OK:
        raise MgritError(st, "mgrit_adjoint_stacked_linearised" if linearised else "mgrit_adjoint_stacked")
    return lambda_all, resnorm
