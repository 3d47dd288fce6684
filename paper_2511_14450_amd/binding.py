"""ctypes binding of include/hyp_stage.h: same names, argument marshalling only.

PyTorch appears here solely as the owner of device memory and streams; every
step of the stage runs inside the HIP library.
"""
from __future__ import annotations

import ctypes as C
import pathlib
from typing import Dict, List, Optional, Sequence

import torch

_PKG = pathlib.Path(__file__).resolve().parent
_LIB: Optional[C.CDLL] = None

HYP_OK, HYP_EINVAL, HYP_ESHAPE, HYP_ECAPACITY, HYP_ESTATE, HYP_EDEVICE, HYP_ENOMEM = range(7)
STATUS_NAMES = ["HYP_OK", "HYP_EINVAL", "HYP_ESHAPE", "HYP_ECAPACITY", "HYP_ESTATE", "HYP_EDEVICE", "HYP_ENOMEM"]
HYP_F32, HYP_BF16 = 0, 1
HYP_FLAG_PLAIN_KERNELS = 1
HYP_FLAG_NO_GRAPH = 2
HYP_FLAG_PAGED_KV = 4
HYP_KV_PAGE_KEYS = 128

EXPORTS = ("stage_workspace_bytes", "stage_create", "stage_prefill", "stage_decode_step", "stage_decode_step_noalloc",
           "stage_set_page_table", "stage_export_kv", "stage_context_len", "stage_destroy", "stage_last_error",
           "stage_uses_mfma", "stage_profile", "stage_profile_read",
           "hyp_measure_mfma_ceiling", "hyp_measure_hbm_read_ceiling")
EXPORTS_PLAN = ("hypsplit_dp", "hypsched_rt", "hypsched_simulate")  # include/hyp_plan.h

KERNEL_CLASSES = ("add_norm", "gemm_qkv", "attn_prefill", "gemm_o", "gemm_gateup", "gemm_down", "gemv_qkv",
                  "dec_qkv_finish", "attn_decode", "gemv_o", "gemv_gateup", "dec_swiglu", "gemv_down")


class HypError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < 7 else status}: {message}")
        self.status = status


class StageConfig(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("ffn_dim", C.c_int32), ("rms_eps", C.c_float),
                ("rope_base", C.c_float), ("dtype", C.c_int32), ("max_batch", C.c_int32),
                ("max_seq", C.c_int32), ("max_prefill_tokens", C.c_int64), ("flags", C.c_uint32),
                ("kv_pool_pages", C.c_uint32)]


_WEIGHT_FIELDS = ("attn_norm_g", "wq", "wk", "wv", "wo", "ffn_norm_g", "w_gate", "w_up", "w_down")


class LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WEIGHT_FIELDS]


def stage_config(shape, max_batch: int, max_seq: int, max_prefill_tokens: int, flags: int = 0,
                 kv_pool_pages: int = 0) -> StageConfig:
    """StageConfig from any object with the block-shape attributes (hidden, n_q_heads,
    n_kv_heads, head_dim, ffn_dim, rms_eps, rope_base, dtype in {"f32", "bf16"})."""
    return StageConfig(hidden=shape.hidden, n_q_heads=shape.n_q_heads, n_kv_heads=shape.n_kv_heads,
                       head_dim=shape.head_dim, ffn_dim=shape.ffn_dim, rms_eps=shape.rms_eps,
                       rope_base=shape.rope_base, dtype=HYP_BF16 if shape.dtype == "bf16" else HYP_F32,
                       max_batch=max_batch, max_seq=max_seq, max_prefill_tokens=max_prefill_tokens,
                       flags=flags, kv_pool_pages=kv_pool_pages)


def library_path() -> pathlib.Path:
    return _PKG / "libhyp_stage.so"


def load_library() -> C.CDLL:
    """Load libhyp_stage.so; raises if it has not been built."""
    global _LIB
    if _LIB is not None:
        return _LIB
    path = library_path()
    if not path.exists():
        raise ImportError(f"{path} is missing: build it with `python -m paper_2511_14450_amd.build` "
                          "(there is no fallback path)")
    lib = C.CDLL(str(path))
    lib.stage_workspace_bytes.restype = C.c_size_t
    lib.stage_workspace_bytes.argtypes = [C.POINTER(StageConfig), C.c_int32, C.c_int32]
    lib.stage_create.restype = C.c_int
    lib.stage_create.argtypes = [C.POINTER(StageConfig), C.c_int32, C.c_int32, C.POINTER(LayerWeights),
                                 C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_void_p)]
    lib.stage_prefill.restype = C.c_int
    lib.stage_prefill.argtypes = [C.c_void_p, C.c_void_p, C.POINTER(C.c_int32), C.c_int32, C.c_void_p]
    lib.stage_decode_step.restype = C.c_int
    lib.stage_decode_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    lib.stage_decode_step_noalloc.restype = C.c_int
    lib.stage_decode_step_noalloc.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
    lib.stage_set_page_table.restype = C.c_int
    lib.stage_set_page_table.argtypes = [C.c_void_p, C.POINTER(C.c_int32), C.c_int32, C.c_int32]
    lib.stage_export_kv.restype = C.c_int
    lib.stage_export_kv.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.stage_context_len.restype = C.c_int
    lib.stage_context_len.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_int32)]
    lib.stage_destroy.restype = C.c_int
    lib.stage_destroy.argtypes = [C.c_void_p]
    lib.stage_last_error.restype = C.c_char_p
    lib.stage_last_error.argtypes = [C.c_void_p]
    lib.stage_profile.restype = C.c_int
    lib.stage_profile.argtypes = [C.c_void_p, C.c_uint32]
    lib.stage_profile_read.restype = C.c_int
    lib.stage_profile_read.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.hyp_measure_mfma_ceiling.restype = C.c_int
    lib.hyp_measure_mfma_ceiling.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
    lib.hyp_measure_hbm_read_ceiling.restype = C.c_int
    lib.hyp_measure_hbm_read_ceiling.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.POINTER(C.c_double)]
    lib.stage_uses_mfma.restype = C.c_int32
    lib.stage_uses_mfma.argtypes = [C.c_void_p]
    dp, ip, bp = C.POINTER(C.c_double), C.POINTER(C.c_int32), C.POINTER(C.c_uint8)
    lib.hypsplit_dp.restype = C.c_int
    lib.hypsplit_dp.argtypes = [C.c_int32, C.c_int32, dp, dp, dp, dp, C.c_double, ip, dp, ip]
    lib.hypsched_rt.restype = C.c_int
    lib.hypsched_rt.argtypes = [C.c_int32, dp, dp, bp, dp, dp, C.c_double, C.c_double, ip]
    lib.hypsched_simulate.restype = C.c_int
    lib.hypsched_simulate.argtypes = [C.c_int32, dp, C.c_int32, dp, dp, ip, dp, dp, bp, dp, ip, dp]
    _LIB = lib
    return lib


def _torch_dtype(dtype: int):
    return torch.bfloat16 if dtype == HYP_BF16 else torch.float32


def _check(status: int, handle) -> None:
    if status != HYP_OK:
        raise HypError(status, stage_last_error(handle))


def stage_last_error(handle) -> str:
    return load_library().stage_last_error(handle).decode()


def stage_workspace_bytes(cfg: StageConfig, l_start: int, l_end: int) -> int:
    return int(load_library().stage_workspace_bytes(C.byref(cfg), l_start, l_end))


class Stage:
    """Handle plus the tensors that must outlive it (workspace, stream)."""

    def __init__(self, handle, cfg: StageConfig, workspace: torch.Tensor, stream, l_start: int, l_end: int):
        self.handle, self.cfg, self.workspace, self.stream = handle, cfg, workspace, stream
        self.l_start, self.l_end = l_start, l_end

    # method spellings of the module-level calls
    def prefill(self, hidden_in, seq_lens, hidden_out=None):
        return stage_prefill(self, hidden_in, seq_lens, hidden_out)

    def decode_step(self, hidden_in, hidden_out=None):
        return stage_decode_step(self, hidden_in, hidden_out)

    def decode_step_noalloc(self, hidden_in, hidden_out):
        return stage_decode_step_noalloc(self, hidden_in, hidden_out)

    def set_page_table(self, table):
        return stage_set_page_table(self, table)

    def export_kv(self, layer, request):
        return stage_export_kv(self, layer, request)

    def context_len(self, request):
        return stage_context_len(self, request)

    def profile(self, classes):
        return stage_profile(self, classes)

    def profile_read(self, kernel_class):
        return stage_profile_read(self, kernel_class)

    def uses_mfma(self):
        return stage_uses_mfma(self)

    def destroy(self):
        stage_destroy(self)

    def __del__(self):
        try:
            if self.handle:
                stage_destroy(self)
        except Exception:
            pass


def stage_create(cfg: StageConfig, l_start: int, l_end: int, layers: Sequence[Dict[str, torch.Tensor]],
                 stream: Optional[torch.cuda.Stream] = None, workspace: Optional[torch.Tensor] = None) -> Stage:
    """layers[i][name] are device tensors of the config dtype, shapes as in hyp_layer_weights_t."""
    lib = load_library()
    need = stage_workspace_bytes(cfg, l_start, l_end)
    if need == 0:
        # let stage_create produce the precise status
        need = 256
    dt = _torch_dtype(cfg.dtype)
    n = len(layers)
    arr = (LayerWeights * max(n, 1))()
    keep = []
    for i, w in enumerate(layers):
        for name in _WEIGHT_FIELDS:
            t = w[name]
            if t is None:
                setattr(arr[i], name, None)
                continue
            if not t.is_cuda or t.dtype != dt or not t.is_contiguous():
                raise ValueError(f"layer {i} {name}: need a contiguous {dt} device tensor")
            keep.append(t)
            setattr(arr[i], name, t.data_ptr())
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device="cuda")
    stream = stream if stream is not None else torch.cuda.current_stream()
    handle = C.c_void_p()
    status = lib.stage_create(C.byref(cfg), l_start, l_end, arr, workspace.data_ptr(), workspace.numel(),
                              C.c_void_p(stream.cuda_stream), C.byref(handle))
    _check(status, None)
    del keep  # stage_create returns after the weights were copied
    return Stage(handle, cfg, workspace, stream, l_start, l_end)


def stage_prefill(stage: Stage, hidden_in: torch.Tensor, seq_lens: Sequence[int],
                  hidden_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    lens = (C.c_int32 * len(seq_lens))(*[int(v) for v in seq_lens])
    if hidden_out is None:
        hidden_out = torch.empty_like(hidden_in)
    _validate_io(stage, hidden_in, hidden_out, sum(int(v) for v in seq_lens))
    status = load_library().stage_prefill(stage.handle, hidden_in.data_ptr(), lens, len(seq_lens),
                                          hidden_out.data_ptr())
    _check(status, stage.handle)
    return hidden_out


def stage_decode_step(stage: Stage, hidden_in: torch.Tensor, hidden_out: Optional[torch.Tensor] = None) -> torch.Tensor:
    if hidden_out is None:
        hidden_out = torch.empty_like(hidden_in)
    _validate_io(stage, hidden_in, hidden_out, None)
    status = load_library().stage_decode_step(stage.handle, hidden_in.data_ptr(), hidden_out.data_ptr())
    _check(status, stage.handle)
    return hidden_out


def stage_decode_step_noalloc(stage: Stage, hidden_in: torch.Tensor, hidden_out: torch.Tensor) -> torch.Tensor:
    """stage_decode_step with the step's temporaries in the library's static device array; the
    caller supplies the output tensor, nothing is allocated."""
    _validate_io(stage, hidden_in, hidden_out, None)
    status = load_library().stage_decode_step_noalloc(stage.handle, hidden_in.data_ptr(), hidden_out.data_ptr())
    _check(status, stage.handle)
    return hidden_out


def _validate_io(stage: Stage, a: torch.Tensor, b: torch.Tensor, rows: Optional[int]) -> None:
    dt = _torch_dtype(stage.cfg.dtype)
    for t in (a, b):
        if not t.is_cuda or t.dtype != dt or not t.is_contiguous() or t.dim() != 2 or t.shape[1] != stage.cfg.hidden:
            raise ValueError(f"hidden states must be contiguous {dt} device tensors [rows, {stage.cfg.hidden}]")
    if a.shape != b.shape or (rows is not None and a.shape[0] != rows):
        raise ValueError("hidden_in / hidden_out row count does not match the request lengths")


def stage_set_page_table(stage: Stage, table: Sequence[Sequence[int]]) -> None:
    """table[r][i] = pool page of keys [128 i, 128 i + 128) of request slot r, -1 for none (rows of equal length)."""
    n, ppr = len(table), len(table[0]) if len(table) else 0
    flat = (C.c_int32 * max(n * ppr, 1))(*[int(v) for row in table for v in row])
    _check(load_library().stage_set_page_table(stage.handle, flat, n, ppr), stage.handle)


def stage_context_len(stage: Stage, request: int) -> int:
    out = C.c_int32()
    status = load_library().stage_context_len(stage.handle, request, C.byref(out))
    if status != HYP_OK:
        raise HypError(status, "no such request")
    return out.value


def stage_export_kv(stage: Stage, layer: int, request: int):
    n = stage_context_len(stage, request)
    kvd = stage.cfg.n_kv_heads * stage.cfg.head_dim
    k = torch.empty((n, kvd), dtype=_torch_dtype(stage.cfg.dtype), device="cuda")
    v = torch.empty_like(k)
    status = load_library().stage_export_kv(stage.handle, layer, request, k.data_ptr(), v.data_ptr())
    _check(status, stage.handle)
    return k, v


def stage_profile(stage: Stage, classes: Sequence[str]) -> None:
    """Start timing the named kernel classes (empty sequence: stop)."""
    mask = 0
    for c in classes:
        mask |= 1 << KERNEL_CLASSES.index(c)
    _check(load_library().stage_profile(stage.handle, mask), stage.handle)


def stage_profile_read(stage: Stage, kernel_class: str):
    """(total milliseconds, launches) of one kernel class since stage_profile()."""
    ms, n = C.c_double(), C.c_int64()
    _check(load_library().stage_profile_read(stage.handle, KERNEL_CLASSES.index(kernel_class), C.byref(ms), C.byref(n)),
           stage.handle)
    return ms.value, n.value


def hyp_measure_mfma_ceiling(gaussian: bool = True, shape_32x32x16: bool = False) -> float:
    """bf16 MFMA TFLOP/s of a register-only loop on the current device (16x16x32, or 32x32x16 on request)."""
    scratch = torch.empty(4 << 20, dtype=torch.uint8, device="cuda")
    out = C.c_double()
    st = load_library().hyp_measure_mfma_ceiling(scratch.data_ptr(), scratch.numel(), (1 if gaussian else 0) | (2 if shape_32x32x16 else 0),
                                                 C.c_void_p(torch.cuda.current_stream().cuda_stream), C.byref(out))
    if st != HYP_OK:
        raise HypError(st, "hyp_measure_mfma_ceiling failed")
    return out.value


def hyp_measure_hbm_read_ceiling(gib: int = 4) -> float:
    """GB/s of a plain streaming read of a `gib` GiB buffer on the current device."""
    buf = torch.empty(gib << 30, dtype=torch.uint8, device="cuda").fill_(1)
    out = C.c_double()
    st = load_library().hyp_measure_hbm_read_ceiling(buf.data_ptr(), buf.numel(),
                                                     C.c_void_p(torch.cuda.current_stream().cuda_stream), C.byref(out))
    if st != HYP_OK:
        raise HypError(st, "hyp_measure_hbm_read_ceiling failed")
    return out.value


def stage_uses_mfma(stage: Stage) -> bool:
    return bool(load_library().stage_uses_mfma(stage.handle))


def stage_destroy(stage: Stage) -> None:
    if stage.handle:
        stage.stream.synchronize()
        status = load_library().stage_destroy(stage.handle)
        stage.handle = None
        if status != HYP_OK:
            raise HypError(status, "stage_destroy failed")


# ---------------------------------------------------------------- include/hyp_plan.h
def _dbl(v):
    return (C.c_double * len(v))(*[float(x) for x in v])


def hypsplit_dp(f: Sequence[float], m: Sequence[float], Cj: Sequence[float], Mj: Sequence[float], eps: float):
    """(p* as a list p_1..p_{T-1}, or None if no partition fits the memory limits; tau*)."""
    N, T = len(f), len(Cj)
    if len(m) != N or len(Mj) != T:
        raise ValueError("f / m need one entry per block, C / M one per tier")
    p = (C.c_int32 * max(T - 1, 1))()
    tau, ok = C.c_double(), C.c_int32()
    st = load_library().hypsplit_dp(N, T, _dbl(f), _dbl(m), _dbl(Cj), _dbl(Mj), float(eps), p, C.byref(tau), C.byref(ok))
    if st != HYP_OK:
        raise HypError(st, "hypsplit_dp rejected its arguments")
    return ([int(p[i]) for i in range(T - 1)] if ok.value else None), tau.value


def hypsched_rt(F_new: float, m_act: float, Ck: Sequence[float], M_avail: Sequence[float], available: Sequence[bool],
                F_run_rem: Sequence[float], F_wait: Sequence[float]) -> Optional[int]:
    """Index of the node Algorithm 2 picks, or None if no node is eligible."""
    K = len(Ck)
    if not (len(M_avail) == len(available) == len(F_run_rem) == len(F_wait) == K):
        raise ValueError("one entry per node in every array")
    k = C.c_int32()
    av = (C.c_uint8 * max(K, 1))(*[1 if a else 0 for a in available])
    st = load_library().hypsched_rt(K, _dbl(Ck), _dbl(M_avail), av, _dbl(F_run_rem), _dbl(F_wait),
                                    float(F_new), float(m_act), C.byref(k))
    if st != HYP_OK:
        raise HypError(st, "hypsched_rt rejected its arguments")
    return None if k.value < 0 else int(k.value)


def hypsched_simulate(arrivals: Sequence[float], F: Sequence[float], m_act: Sequence[float],
                      Cjk: Sequence[Sequence[float]], Mjk: Sequence[Sequence[float]], transfer: Sequence[float],
                      available: Optional[Sequence[Sequence[bool]]] = None):
    """(node[task][tier], finish[task][tier]) of the FIFO queue model driven by HypSched-RT."""
    T, n = len(F), len(arrivals)
    if len(m_act) != T or len(Cjk) != T or len(Mjk) != T or len(transfer) != max(T - 1, 0):
        raise ValueError("per-tier arrays need one entry per tier, transfer one per boundary")
    per = (C.c_int32 * T)(*[len(c) for c in Cjk])
    flatC = [x for c in Cjk for x in c]
    flatM = [x for c in Mjk for x in c]
    av = None
    if available is not None:
        flat = [1 if a else 0 for c in available for a in c]
        av = (C.c_uint8 * len(flat))(*flat)
    node = (C.c_int32 * (n * T))()
    fin = (C.c_double * (n * T))()
    st = load_library().hypsched_simulate(n, _dbl(arrivals), T, _dbl(F), _dbl(m_act), per, _dbl(flatC), _dbl(flatM),
                                          av, _dbl(transfer) if T > 1 else None, node, fin)
    if st != HYP_OK:
        raise HypError(st, "hypsched_simulate rejected its arguments")
    return ([[int(node[q * T + j]) for j in range(T)] for q in range(n)],
            [[float(fin[q * T + j]) for j in range(T)] for q in range(n)])
