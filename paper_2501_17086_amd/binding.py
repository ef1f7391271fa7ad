"""ctypes binding of libhbp (include/hbp.h).  Argument marshalling only: every
step of the path runs in the library's HIP kernels.  torch is used to hold
device memory and to name the stream.

The library is opened on first use and a missing build raises: there is no
fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
from dataclasses import dataclass
from typing import Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhbp.so")

HBP_OK = 0
STATUS_NAMES = {0: "HBP_OK", 1: "HBP_E_INVALID_ARG", 2: "HBP_E_UNSUPPORTED", 3: "HBP_E_WORKSPACE",
                4: "HBP_E_NULL", 5: "HBP_E_DEVICE"}
F32, BF16 = 0, 1
MLP, RNN, GATED, LSTM, GRU, TRANSFORMER = 0, 1, 2, 3, 4, 5
KIND = {"mlp": MLP, "rnn": RNN, "gated": GATED, "lstm": LSTM, "gru": GRU, "transformer": TRANSFORMER}
ACT = {"gelu": 0, "tanh": 1, "identity": 2}
NORM = {"none": 0, "rms": 1}
POST = {"none": 0, "relu": 1, "rms": 2}
LAMBDA_ONE, LAMBDA_CHANNEL, LAMBDA_TOKEN = 0, 1, 2

EXPORTS = ("hbp_workspace_size", "hbp_check", "hbp_forward", "hbp_backward", "hbp_exact_backward",
           "hbp_scan_workspace_size", "hbp_initial_estimate", "hbp_initial_estimate_static",
           "hbp_param_grads", "hbp_train_scratch_size", "hbp_loss_mse", "hbp_optimizer_step", "hbp_train_step",
           "hbp_profile_enable", "hbp_profile_read", "hbp_status_string")
PROF_CLASSES = ("vjp1", "vjp2", "scan", "dw", "forward", "other", "attn")


class hbp_desc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("kind", C.c_int32), ("dtype", C.c_int32), ("act", C.c_int32),
                ("norm", C.c_int32), ("lambda_kind", C.c_int32), ("loss_every_state", C.c_int32),
                ("eps", C.c_float), ("L", C.c_int64), ("N", C.c_int64), ("d", C.c_int64), ("d_ff", C.c_int64),
                ("d_in", C.c_int64), ("gamma", C.c_float), ("post", C.c_int32),
                ("heads", C.c_int32), ("causal", C.c_int32), ("seq_len", C.c_int64)]


class hbp_buffers(C.Structure):
    _fields_ = [("struct_size", C.c_uint32),
                ("W1", C.c_void_p), ("W2", C.c_void_p), ("U", C.c_void_p), ("lambda_", C.c_void_p),
                ("x", C.c_void_p), ("y", C.c_void_p), ("rinv", C.c_void_p), ("z", C.c_void_p),
                ("dphi", C.c_void_p), ("xin", C.c_void_p), ("mask", C.c_void_p), ("e", C.c_void_p),
                ("g", C.c_void_p),
                ("dW1", C.c_void_p), ("dW2", C.c_void_p), ("dU", C.c_void_p),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("Wqkv", C.c_void_p), ("Wo", C.c_void_p), ("qkv", C.c_void_p), ("attn_o", C.c_void_p),
                ("lse", C.c_void_p), ("dWqkv", C.c_void_p), ("dWo", C.c_void_p)]


OPT_SGD, OPT_ADAMW = 0, 1


class hbp_optim(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("kind", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float),
                ("beta2", C.c_float), ("eps", C.c_float), ("weight_decay", C.c_float), ("clip_norm", C.c_float),
                ("step", C.c_int64)]


class hbp_optim_state(C.Structure):
    _fields_ = [("struct_size", C.c_uint32),
                ("master1", C.c_void_p), ("master2", C.c_void_p), ("masterU", C.c_void_p),
                ("m1", C.c_void_p), ("m2", C.c_void_p), ("mU", C.c_void_p),
                ("v1", C.c_void_p), ("v2", C.c_void_p), ("vU", C.c_void_p),
                ("scratch", C.c_void_p), ("scratch_bytes", C.c_size_t),
                ("masterQ", C.c_void_p), ("masterO", C.c_void_p), ("mQ", C.c_void_p), ("mO", C.c_void_p),
                ("vQ", C.c_void_p), ("vO", C.c_void_p)]


class HbpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {STATUS_NAMES.get(status, status)} ({status_string(status)})")


_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built; run `python -m paper_2501_17086_amd.build`")
        # torch ships its own HIP runtime under the same soname: load it first, so that this library binds to the
        # runtime that owns the tensors' memory and streams (two runtimes in one process do not share them)
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.hbp_workspace_size.argtypes = [C.POINTER(hbp_desc), C.POINTER(C.c_size_t)]
        L.hbp_check.argtypes = [C.POINTER(hbp_desc), C.POINTER(hbp_buffers)]
        L.hbp_forward.argtypes = [C.POINTER(hbp_desc), C.POINTER(hbp_buffers), C.c_void_p]
        L.hbp_backward.argtypes = [C.POINTER(hbp_desc), C.c_int, C.POINTER(hbp_buffers), C.c_void_p]
        L.hbp_exact_backward.argtypes = [C.POINTER(hbp_desc), C.POINTER(hbp_buffers), C.c_void_p]
        L.hbp_scan_workspace_size.argtypes = [C.POINTER(hbp_desc), C.c_int, C.POINTER(C.c_size_t)]
        L.hbp_initial_estimate.argtypes = [C.POINTER(hbp_desc), C.c_int, C.POINTER(hbp_buffers), C.c_void_p]
        L.hbp_initial_estimate_static.argtypes = [C.POINTER(hbp_desc), C.POINTER(hbp_buffers), C.c_void_p]
        L.hbp_param_grads.argtypes = [C.POINTER(hbp_desc), C.POINTER(hbp_buffers), C.c_void_p]
        L.hbp_train_scratch_size.argtypes = [C.POINTER(C.c_size_t)]
        L.hbp_loss_mse.argtypes = [C.POINTER(hbp_desc), C.POINTER(hbp_buffers), C.c_void_p, C.c_void_p, C.c_void_p,
                                   C.c_void_p, C.c_size_t, C.c_void_p]
        L.hbp_optimizer_step.argtypes = [C.POINTER(hbp_desc), C.POINTER(hbp_buffers), C.POINTER(hbp_optim),
                                         C.POINTER(hbp_optim_state), C.c_void_p]
        L.hbp_train_step.argtypes = [C.POINTER(hbp_desc), C.c_int, C.POINTER(hbp_buffers), C.c_void_p, C.c_void_p,
                                     C.POINTER(hbp_optim), C.POINTER(hbp_optim_state), C.c_void_p]
        L.hbp_profile_enable.argtypes = [C.c_int]
        L.hbp_profile_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64)]
        L.hbp_status_string.argtypes = [C.c_int]
        L.hbp_status_string.restype = C.c_char_p
        for n in EXPORTS[:-1]:
            getattr(L, n).restype = C.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().hbp_status_string(status).decode()


def make_desc(kind: str, dtype: str, act: str, norm: str, L: int, N: int, d: int, d_ff: int, d_in: int = 0,
              lambda_channel: bool = False, loss_every_state: bool = False, eps: float = 1e-6,
              gamma: float = 0.0, lambda_token: bool = False, post: str = "none", heads: int = 0,
              causal: bool = True, seq_len: int = 0) -> hbp_desc:
    return hbp_desc(C.sizeof(hbp_desc), KIND[kind], BF16 if dtype == "bf16" else F32,
                    ACT[act], NORM[norm],
                    LAMBDA_TOKEN if lambda_token else LAMBDA_CHANNEL if lambda_channel else LAMBDA_ONE,
                    1 if loss_every_state else 0, eps, L, N, d, d_ff, d_in, gamma, POST[post], heads,
                    1 if causal else 0, seq_len)


def workspace_size(desc: hbp_desc) -> int:
    n = C.c_size_t(0)
    st = lib().hbp_workspace_size(C.byref(desc), C.byref(n))
    if st != HBP_OK:
        raise HbpError(st, "hbp_workspace_size")
    return n.value


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


@dataclass
class Problem:
    """Device tensors of one stack, laid out as include/hbp.h describes."""
    desc: hbp_desc
    W1: "object"
    W2: "object"
    U: "object" = None
    lam: "object" = None
    x: "object" = None
    y: "object" = None
    rinv: "object" = None
    z: "object" = None
    dphi: "object" = None
    xin: "object" = None
    mask: "object" = None
    e: "object" = None
    g: "object" = None
    dW1: "object" = None
    dW2: "object" = None
    dU: "object" = None
    workspace: "object" = None
    Wqkv: "object" = None
    Wo: "object" = None
    qkv: "object" = None
    attn_o: "object" = None
    lse: "object" = None
    dWqkv: "object" = None
    dWo: "object" = None

    def buffers(self) -> hbp_buffers:
        ws = self.workspace
        return hbp_buffers(C.sizeof(hbp_buffers), _ptr(self.W1), _ptr(self.W2), _ptr(self.U), _ptr(self.lam),
                           _ptr(self.x), _ptr(self.y), _ptr(self.rinv), _ptr(self.z), _ptr(self.dphi),
                           _ptr(self.xin), _ptr(self.mask), _ptr(self.e), _ptr(self.g), _ptr(self.dW1), _ptr(self.dW2),
                           _ptr(self.dU), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                           _ptr(self.Wqkv), _ptr(self.Wo), _ptr(self.qkv), _ptr(self.attn_o), _ptr(self.lse),
                           _ptr(self.dWqkv), _ptr(self.dWo))


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream


def _call(name: str, st: int) -> None:
    if st != HBP_OK:
        raise HbpError(st, name)


def hbp_check(p: Problem) -> int:
    b = p.buffers()
    return lib().hbp_check(C.byref(p.desc), C.byref(b))


def hbp_forward(p: Problem, stream=None) -> None:
    b = p.buffers()
    _call("hbp_forward", lib().hbp_forward(C.byref(p.desc), C.byref(b), _stream(stream)))


def hbp_backward(p: Problem, k: int, stream=None, gamma: Optional[float] = None) -> None:
    """gamma overrides the descriptor's for this call."""
    b = p.buffers()
    desc = p.desc
    if gamma is not None:
        desc = hbp_desc.from_buffer_copy(p.desc)
        desc.gamma = float(gamma)
    _call("hbp_backward", lib().hbp_backward(C.byref(desc), int(k), C.byref(b), _stream(stream)))


SCAN_ALGORITHMS = {"auto": 0, "sequential": 1, "chunked": 2, "hillis_steele": 3, "single_pass": 4}


def scan_workspace_size(desc: hbp_desc, algorithm: str) -> int:
    n = C.c_size_t(0)
    _call("hbp_scan_workspace_size", lib().hbp_scan_workspace_size(C.byref(desc), SCAN_ALGORITHMS[algorithm], C.byref(n)))
    return n.value


def hbp_initial_estimate(p: Problem, algorithm: str = "auto", stream=None, workspace=None) -> None:
    """g := w^0 by the named form of the scan; `workspace` (a uint8 tensor of
    scan_workspace_size bytes) replaces the Problem's for this call."""
    saved = p.workspace
    if workspace is not None:
        p.workspace = workspace
    try:
        b = p.buffers()
    finally:
        p.workspace = saved
    _call("hbp_initial_estimate",
          lib().hbp_initial_estimate(C.byref(p.desc), SCAN_ALGORITHMS[algorithm], C.byref(b), _stream(stream)))


STATIC_SCRATCH_BYTES = 32 << 20


def hbp_initial_estimate_static(p: Problem, stream=None) -> None:
    """g := w^0 by the chunked scan with the library's own fixed scratch: no workspace, no allocation."""
    saved = p.workspace
    p.workspace = None
    try:
        b = p.buffers()
    finally:
        p.workspace = saved
    _call("hbp_initial_estimate_static",
          lib().hbp_initial_estimate_static(C.byref(p.desc), C.byref(b), _stream(stream)))


def hbp_exact_backward(p: Problem, stream=None) -> None:
    b = p.buffers()
    _call("hbp_exact_backward", lib().hbp_exact_backward(C.byref(p.desc), C.byref(b), _stream(stream)))


def hbp_param_grads(p: Problem, stream=None) -> None:
    b = p.buffers()
    _call("hbp_param_grads", lib().hbp_param_grads(C.byref(p.desc), C.byref(b), _stream(stream)))


def train_scratch_size() -> int:
    n = C.c_size_t(0)
    _call("hbp_train_scratch_size", lib().hbp_train_scratch_size(C.byref(n)))
    return n.value


def make_optim(kind: str, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8,
               weight_decay: float = 0.0, clip_norm: float = 0.0, step: int = 1) -> hbp_optim:
    return hbp_optim(C.sizeof(hbp_optim), OPT_ADAMW if kind == "adamw" else OPT_SGD, lr, beta1, beta2, eps,
                     weight_decay, clip_norm, step)


@dataclass
class OptimState:
    """Device tensors of the optimizer: fp32 master copies of the weights (optional), moments, reduction scratch."""
    master: tuple
    m: tuple
    v: tuple
    scratch: "object"
    loss: "object"        # device float: the last loss value

    def struct(self) -> hbp_optim_state:
        ptrs = lambda ts: [_ptr(t) for t in (tuple(ts) + (None,) * 5)[:5]]     # W1, W2, U, Wqkv, Wo
        ma, m, v = ptrs(self.master), ptrs(self.m), ptrs(self.v)
        return hbp_optim_state(C.sizeof(hbp_optim_state), *ma[:3], *m[:3], *v[:3], _ptr(self.scratch),
                               self.scratch.numel() * self.scratch.element_size(),
                               ma[3], ma[4], m[3], m[4], v[3], v[4])


def allocate_optim(p: Problem, adamw: bool, master: bool = True) -> OptimState:
    import torch
    ws = (p.W1, p.W2, p.U, p.Wqkv, p.Wo)
    f = lambda w: None if w is None else torch.zeros(w.shape, dtype=torch.float32, device=w.device)
    return OptimState(master=tuple((None if (w is None or not master) else w.float().clone()) for w in ws),
                      m=tuple(f(w) for w in ws), v=tuple((f(w) if adamw else None) for w in ws),
                      scratch=torch.zeros(train_scratch_size() // 4, dtype=torch.float32, device=p.W1.device),
                      loss=torch.zeros(1, dtype=torch.float32, device=p.W1.device))


def hbp_loss_mse(p: Problem, target, st: OptimState, stream=None) -> None:
    """Writes p.e (the loss gradient) and st.loss from p.x and `target`."""
    b = p.buffers()
    _call("hbp_loss_mse", lib().hbp_loss_mse(C.byref(p.desc), C.byref(b), target.data_ptr(), p.e.data_ptr(),
                                             st.loss.data_ptr(), st.scratch.data_ptr(),
                                             st.scratch.numel() * 4, _stream(stream)))


def hbp_optimizer_step(p: Problem, opt: hbp_optim, st: OptimState, stream=None) -> None:
    b = p.buffers()
    s = st.struct()
    _call("hbp_optimizer_step", lib().hbp_optimizer_step(C.byref(p.desc), C.byref(b), C.byref(opt), C.byref(s),
                                                         _stream(stream)))


def hbp_train_step(p: Problem, k: int, target, opt: hbp_optim, st: OptimState, stream=None) -> None:
    """forward, loss, hbp_backward(k) (k < 0: exact backpropagation), parameter gradients, optimizer update."""
    b = p.buffers()
    s = st.struct()
    _call("hbp_train_step", lib().hbp_train_step(C.byref(p.desc), int(k), C.byref(b), target.data_ptr(),
                                                 st.loss.data_ptr(), C.byref(opt), C.byref(s), _stream(stream)))


def profile_enable(on: bool) -> None:
    _call("hbp_profile_enable", lib().hbp_profile_enable(1 if on else 0))


def profile_read() -> dict:
    """{class: (milliseconds, launches)} since the previous read."""
    n = len(PROF_CLASSES)
    ms = (C.c_double * n)()
    cnt = (C.c_int64 * n)()
    _call("hbp_profile_read", lib().hbp_profile_read(ms, cnt))
    return {PROF_CLASSES[i]: (ms[i], cnt[i]) for i in range(n)}


def allocate(w, inputs, device="cuda:0", N: Optional[int] = None) -> Problem:
    """Device tensors for workload `w` (a synth.Workload) from make_inputs()'s
    arrays: uploads parameters, x[0], xin and e; allocates the saved state,
    outputs and workspace."""
    import torch
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    N = inputs["x0"].shape[0] if N is None else N
    dev = torch.device(device)

    def up(a, dtype=dt):
        return None if a is None else torch.from_numpy(a).to(dev).to(dtype).contiguous()

    lam = inputs["lam"]
    if w.kind in ("gated", "lstm", "gru"):   # the cell's own residual coefficient, written by hbp_forward: [L,N,d], storage type
        lam = np.zeros((w.L, N, w.d), np.float32)
    per_token = lam is not None and lam.ndim == 3      # [L,N,d] in the storage type; [L,d] is fp32
    desc = make_desc(w.kind, w.dtype, w.act, w.norm, w.L, N, w.d, w.d_ff, w.d_in,
                     lambda_channel=lam is not None and not per_token, lambda_token=per_token,
                     loss_every_state=w.loss_every_state, eps=w.eps, post=getattr(w, "post", "none"),
                     heads=getattr(w, "heads", 0), causal=getattr(w, "causal", True), seq_len=getattr(w, "seq_len", 0),
                     gamma=getattr(w, "gamma", 0.0))
    L, d, dff = w.L, w.d, w.d_ff
    tfm = w.kind == "transformer"
    Li = L // 2 if tfm else L        # rows of the inner state: one per MLP block
    x = torch.zeros((L + 1, N, d), dtype=dt, device=dev)
    x[0] = up(inputs["x0"])
    rms = w.norm == "rms"
    post = getattr(w, "post", "none")
    p = Problem(
        desc=desc, W1=up(inputs["W1"]), W2=up(inputs["W2"]), U=up(inputs["U"]),
        lam=up(lam, dt if per_token else torch.float32), x=x,
        y=torch.zeros((L, N, d), dtype=dt, device=dev) if rms else None,
        rinv=torch.zeros((L, N), dtype=torch.float32, device=dev) if (rms or post == "rms") else None,
        z=torch.zeros((Li, N, dff), dtype=dt, device=dev),
        dphi=torch.zeros((Li, N, dff), dtype=dt, device=dev) if w.act == "gelu" else None,
        xin=up(inputs["xin"]), e=up(inputs["e"]),
        mask=torch.zeros((L, N, d // 8), dtype=torch.uint8, device=dev) if getattr(w, "post", "none") == "relu" else None,
        g=torch.zeros((L + 1, N, d), dtype=dt, device=dev),
        dW1=torch.zeros(inputs["W1"].shape, dtype=torch.float32, device=dev),
        dW2=None if inputs["W2"] is None else torch.zeros(inputs["W2"].shape, dtype=torch.float32, device=dev),
        dU=None if inputs["U"] is None else torch.zeros(inputs["U"].shape, dtype=torch.float32, device=dev),
    )
    if tfm:
        p.Wqkv, p.Wo = up(inputs["Wqkv"]), up(inputs["Wo"])
        p.qkv = torch.zeros((Li, N, 3 * d), dtype=dt, device=dev)
        p.attn_o = torch.zeros((Li, N, d), dtype=dt, device=dev)
        p.lse = torch.zeros((Li, N * w.heads), dtype=torch.float32, device=dev)
        p.dWqkv = torch.zeros(inputs["Wqkv"].shape, dtype=torch.float32, device=dev)
        p.dWo = torch.zeros(inputs["Wo"].shape, dtype=torch.float32, device=dev)
    p.workspace = torch.zeros(workspace_size(desc), dtype=torch.uint8, device=dev)
    return p
