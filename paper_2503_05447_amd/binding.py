"""Thin Python binding of the C-ABI library declared in include/lsm.h.

Argument marshalling only: tensors are torch device tensors (PyTorch is used
for device memory and streams, nothing else), every step of the path runs in
the HIP kernels of liblsm_hip.so.  There is no fallback: if the library cannot
be loaded, importing works but every call raises.
"""
import ctypes
import os

from . import build as _build

DECAY_NONE, DECAY_HEAD, DECAY_SCALAR, DECAY_VECTOR = 0, 1, 2, 3
DTYPE_F32, DTYPE_BF16 = 0, 1
LAYOUT_BHTD, LAYOUT_BTHD = 0, 1
FLAG_SAVE_STATES, FLAG_SAVE_ALWAYS = 1, 2


class LsmError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__("%s failed: status %d (%s)" % (where, status, _status_string(status)))


class _Params(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("B", ctypes.c_int32), ("H", ctypes.c_int32),
                ("T", ctypes.c_int32), ("d_k", ctypes.c_int32), ("d_v", ctypes.c_int32),
                ("chunk_size", ctypes.c_int32), ("decay_kind", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("layout", ctypes.c_int32), ("n_seq", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("cu_seqlens", ctypes.c_void_p)]


_lib = None


def library():
    """Load liblsm_hip.so (building it only if no built library exists; a library older than its sources is
    loaded as it is, with a warning: rebuild with paper_2503_05447_amd.build.build_library())."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.LIB_PATH
    if not os.path.exists(path):
        _build.build_library()
    elif _build._stale():
        import warnings
        warnings.warn("liblsm_hip.so is older than its sources; run paper_2503_05447_amd.build.build_library()",
                      RuntimeWarning, stacklevel=2)
    lib = ctypes.CDLL(path)
    vp, sz, pp = ctypes.c_void_p, ctypes.c_size_t, ctypes.POINTER(_Params)
    lib.lsm_chunk_fwd.restype = ctypes.c_int
    lib.lsm_chunk_fwd.argtypes = [pp] + [vp] * 8 + [sz, vp]
    lib.lsm_chunk_fwd_noalloc.restype = ctypes.c_int
    lib.lsm_chunk_fwd_noalloc.argtypes = [pp] + [vp] * 8
    lib.lsm_chunk_bwd.restype = ctypes.c_int
    lib.lsm_chunk_bwd.argtypes = [pp] + [vp] * 13 + [sz, vp]
    lib.lsm_chunk_fwd_workspace_bytes.restype = sz
    lib.lsm_chunk_fwd_workspace_bytes.argtypes = [pp]
    lib.lsm_chunk_bwd_workspace_bytes.restype = sz
    lib.lsm_chunk_bwd_workspace_bytes.argtypes = [pp]
    lib.lsm_kernel_path.restype = ctypes.c_int
    lib.lsm_kernel_path.argtypes = [pp]
    lib.lsm_status_string.restype = ctypes.c_char_p
    lib.lsm_status_string.argtypes = [ctypes.c_int]
    lib.lsm_version.restype = ctypes.c_int
    lib.lsm_profile_start.restype = ctypes.c_int
    lib.lsm_profile_stop.restype = ctypes.c_int
    lib.lsm_profile_stop.argtypes = [ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_float), ctypes.c_int]
    lib.lsm_kernel_name.restype = ctypes.c_char_p
    lib.lsm_kernel_name.argtypes = [ctypes.c_int]
    lib.lsm_keeps_states.restype = ctypes.c_int
    lib.lsm_keeps_states.argtypes = [pp]
    lib.lsm_step.restype = ctypes.c_int
    lib.lsm_step.argtypes = [pp] + [vp] * 7
    lib.lsm_calib_copy.restype = ctypes.c_int
    lib.lsm_calib_copy.argtypes = [vp, vp, sz, vp]
    lib.lsm_calib_mfma.restype = ctypes.c_int
    lib.lsm_calib_mfma.argtypes = [vp, ctypes.c_int, ctypes.c_int, vp]
    lib.lsm_calib_mfma_flops.restype = ctypes.c_double
    lib.lsm_calib_mfma_flops.argtypes = [ctypes.c_int, ctypes.c_int]
    lib.lsm_bench_intra_chunk_workspace_bytes.restype = sz
    lib.lsm_delta_fwd.restype = ctypes.c_int
    lib.lsm_delta_fwd.argtypes = [pp] + [vp] * 10 + [sz, vp]
    lib.lsm_delta_fwd_workspace_bytes.restype = sz
    lib.lsm_delta_fwd_workspace_bytes.argtypes = [pp]
    lib.lsm_delta_step.restype = ctypes.c_int
    lib.lsm_delta_step.argtypes = [pp] + [vp] * 9
    lib.lsm_delta_bwd.restype = ctypes.c_int
    lib.lsm_delta_bwd.argtypes = [pp] + [vp] * 17 + [sz, vp]
    lib.lsm_delta_bwd_workspace_bytes.restype = sz
    lib.lsm_delta_bwd_workspace_bytes.argtypes = [pp]
    lib.lsm_bench_intra_chunk_workspace_bytes.argtypes = [pp]
    lib.lsm_bench_intra_chunk.restype = ctypes.c_int
    lib.lsm_bench_intra_chunk.argtypes = [pp] + [vp] * 6 + [sz, ctypes.c_int, vp]
    _lib = lib
    return lib


def _status_string(status):
    return library().lsm_status_string(int(status)).decode()


def make_params(B, H, T, d_k, d_v, chunk_size, decay_kind, dtype, layout=LAYOUT_BHTD, n_seq=0, cu_seqlens=None,
                flags=0):
    """cu_seqlens: device address (int) of n_seq + 1 int32 sequence starts, or None."""
    return _Params(ctypes.sizeof(_Params), B, H, T, d_k, d_v, chunk_size, decay_kind, dtype, layout, n_seq, flags,
                   cu_seqlens)


def lsm_chunk_fwd_workspace_bytes(params):
    return int(library().lsm_chunk_fwd_workspace_bytes(ctypes.byref(params)))


def lsm_chunk_bwd_workspace_bytes(params):
    return int(library().lsm_chunk_bwd_workspace_bytes(ctypes.byref(params)))


def kernel_path(params):
    """1 = MFMA kernels, 0 = generic fp32-arithmetic kernels, < 0 = invalid parameters."""
    return int(library().lsm_kernel_path(ctypes.byref(params)))


def keeps_states(params):
    """1 = the forward call keeps its chunk states for the backward call, 0 = the backward call recomputes them."""
    return int(library().lsm_keeps_states(ctypes.byref(params)))


def lsm_profile_start():
    """Bracket every kernel the library enqueues with HIP events until lsm_profile_stop()."""
    library().lsm_profile_start()


def lsm_profile_stop(capacity=65536):
    """Return [(kernel name, elapsed ms), ...] in launch order and switch timing off."""
    ids = (ctypes.c_int * capacity)()
    ms = (ctypes.c_float * capacity)()
    n = library().lsm_profile_stop(ids, ms, capacity)
    return [(library().lsm_kernel_name(ids[i]).decode(), float(ms[i])) for i in range(n)]


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(None)


def _check(t, shape, dtype, name):
    import torch  # noqa: F401
    if t is None:
        return
    if not t.is_cuda or not t.is_contiguous() or t.dtype != dtype or tuple(t.shape) != tuple(shape):
        raise ValueError("%s: need a contiguous device tensor %s of %s, got %s %s on %s"
                         % (name, tuple(shape), dtype, tuple(t.shape), t.dtype, t.device))


def _save_flags(save):
    """False: none; True: keep the states where the library finds it faster; "always": wherever it can."""
    if not save:
        return 0
    return FLAG_SAVE_STATES | (FLAG_SAVE_ALWAYS if save == "always" else 0)


def _setup(q, k, v, log_decay, decay_kind, chunk_size, layout=LAYOUT_BHTD, cu_seqlens=None, flags=0):
    import torch
    if q.dtype == torch.float32:
        dt = DTYPE_F32
    elif q.dtype == torch.bfloat16:
        dt = DTYPE_BF16
    else:
        raise ValueError("q must be float32 or bfloat16")
    if layout == LAYOUT_BTHD:
        B, T, H, dk = q.shape
    else:
        B, H, T, dk = q.shape
    dv = v.shape[-1]
    tshape = (lambda d_: (B, T, H, d_)) if layout == LAYOUT_BTHD else (lambda d_: (B, H, T, d_))
    _check(q, tshape(dk), q.dtype, "q")
    _check(k, tshape(dk), q.dtype, "k")
    _check(v, tshape(dv), q.dtype, "v")
    gshape = {DECAY_NONE: None, DECAY_HEAD: (H,), DECAY_SCALAR: tshape(dk)[:3], DECAY_VECTOR: tshape(dk)}[decay_kind]
    if gshape is not None:
        if log_decay is None:
            raise ValueError("log_decay required for this decay kind")
        _check(log_decay, gshape, torch.float32, "log_decay")
    elif log_decay is not None:
        raise ValueError("log_decay must be None for DECAY_NONE")
    n_seq, cu_ptr = 0, None
    if cu_seqlens is not None:
        if B != 1:
            raise ValueError("packed variable-length input needs B == 1")
        n_seq = cu_seqlens.numel() - 1
        _check(cu_seqlens, (n_seq + 1,), torch.int32, "cu_seqlens")
        cu_ptr = cu_seqlens.data_ptr()
    p = make_params(B, H, T, dk, dv, chunk_size, decay_kind, dt, layout, n_seq, cu_ptr, flags)
    return p, (n_seq or B, H, T, dk, dv), gshape


def _alloc_on(stream):
    """Context in which torch allocates for `stream` (its caching allocator ties a block to the stream that is
    current at allocation time; a temporary used on another stream could be handed out again too early)."""
    import contextlib
    import torch
    return torch.cuda.stream(stream) if stream is not None else contextlib.nullcontext()


def _stream_handle(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def lsm_chunk_workspace(q, k, v, log_decay, decay_kind, chunk_size=64, layout=LAYOUT_BHTD, cu_seqlens=None,
                        save_states=True):
    """A workspace tensor large enough for both the forward and the backward call on these inputs."""
    import torch
    p, _, _ = _setup(q, k, v, log_decay, decay_kind, chunk_size, layout, cu_seqlens,
                     _save_flags(save_states))
    need = max(lsm_chunk_fwd_workspace_bytes(p), lsm_chunk_bwd_workspace_bytes(p), 256)
    return torch.empty(need, dtype=torch.uint8, device=q.device)


def lsm_chunk_fwd(q, k, v, log_decay, decay_kind, chunk_size=64, init_state=None,
                  want_final_state=True, workspace=None, stream=None, layout=LAYOUT_BHTD, cu_seqlens=None,
                  save_states=False):
    """o, final_state = chunkwise forward of M_t = diag(a_t) M_{t-1} + k_t^T v_t, o_t = q_t M_t.

    save_states: keep the chunk states in ``workspace`` (required then, see lsm_chunk_workspace) for a
    following lsm_chunk_bwd(..., workspace=the same tensor, states_saved=<the same value>) on the same
    inputs.  True leaves the choice to the library (it recomputes where that is faster), "always" does not.

    layout: LAYOUT_BHTD ([B,H,T,d]) or LAYOUT_BTHD ([B,T,H,d]).  cu_seqlens (int32 device tensor of
    n_seq + 1 sequence starts, B == 1): packed variable-length input; states are then [n_seq,H,d_k,d_v].
    Enqueues on ``stream`` (default: torch's current stream) and returns without synchronising.
    """
    import torch
    if save_states and workspace is None:
        raise ValueError("save_states needs a caller-owned workspace that is passed on to lsm_chunk_bwd")
    p, (B, H, T, dk, dv), _ = _setup(q, k, v, log_decay, decay_kind, chunk_size, layout, cu_seqlens,
                                     _save_flags(save_states))
    _check(init_state, (B, H, dk, dv), torch.float32, "init_state")
    need = lsm_chunk_fwd_workspace_bytes(p)
    with _alloc_on(stream):   # what is allocated here is used on `stream`: allocate it there
        if workspace is None:
            workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
        o = torch.empty_like(v)
        final = torch.empty((B, H, dk, dv), dtype=torch.float32, device=q.device) if want_final_state else None
    rc = library().lsm_chunk_fwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(log_decay), _ptr(init_state),
                                 _ptr(o), _ptr(final), _ptr(workspace), workspace.numel(), _stream_handle(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_chunk_fwd")
    return o, final


def lsm_delta_step(q, k, v, state, log_alpha=None, beta=None, b=None, o=None, stream=None):
    """One recurrent step of the delta-rule rows: ``state`` [B,H,d_k,d_v] fp32 is updated in place, returns o [B,H,d_v].
    q, k [B,H,d_k], v [B,H,d_v]; log_alpha, beta, b: [B,H] float32 or None (= 1)."""
    import torch
    B, H, dk = q.shape
    dv = v.shape[-1]
    dt = DTYPE_F32 if q.dtype == torch.float32 else DTYPE_BF16
    if q.dtype not in (torch.float32, torch.bfloat16):
        raise ValueError("q must be float32 or bfloat16")
    _check(k, (B, H, dk), q.dtype, "k")
    _check(v, (B, H, dv), q.dtype, "v")
    for name, t_ in (("log_alpha", log_alpha), ("beta", beta), ("b", b)):
        _check(t_, (B, H), torch.float32, name)
    _check(state, (B, H, dk, dv), torch.float32, "state")
    if state is None:
        raise ValueError("state is required")
    if o is None:
        with _alloc_on(stream):
            o = torch.empty((B, H, dv), dtype=q.dtype, device=q.device)
    else:
        _check(o, (B, H, dv), q.dtype, "o")
    p = make_params(B, H, 1, dk, dv, 64, DECAY_NONE if log_alpha is None else DECAY_SCALAR, dt)
    rc = library().lsm_delta_step(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(beta), _ptr(b), _ptr(state),
                                  _ptr(o), _stream_handle(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_delta_step")
    return o


def lsm_delta_workspace(q, k, v, log_alpha=None, layout=LAYOUT_BHTD, cu_seqlens=None):
    """A workspace tensor that serves lsm_delta_fwd(..., save_states=True) and the lsm_delta_bwd(..., states_saved=True)
    that follows it on the same inputs."""
    import torch
    kind = DECAY_NONE if log_alpha is None else DECAY_SCALAR
    p, _, _ = _setup(q, k, v, log_alpha, kind, 64, layout, cu_seqlens, FLAG_SAVE_STATES)
    need = library().lsm_delta_bwd_workspace_bytes(ctypes.byref(p))
    if need == 0:
        raise LsmError(-3, "lsm_delta_workspace")
    return torch.empty(need, dtype=torch.uint8, device=q.device)


def lsm_delta_fwd(q, k, v, log_alpha=None, beta=None, b=None, init_state=None, want_final_state=True, workspace=None,
                  stream=None, layout=LAYOUT_BHTD, save_states=False, cu_seqlens=None):
    """o, final_state = chunkwise forward of the delta-rule rows of Table 1,
    M_t = alpha_t (I - beta_t k_t^T k_t) M_{t-1} + b_t k_t^T v_t, o_t = q_t M_t.

    DeltaNet: log_alpha None, beta = the row's a_t, b = the row's b_t.  Gated DeltaNet: log_alpha = log a_t, beta None.
    log_alpha, beta, b: float32 per token ([B,H,T], or [B,T,H] for LAYOUT_BTHD), None = the constant 1.
    bf16, d_k = d_v = 128 only.  cu_seqlens: packed variable-length input as in lsm_chunk_fwd (B == 1, states
    [n_seq,H,d_k,d_v]).  Enqueues on ``stream`` (default: torch's current stream) without synchronising.
    save_states: leave what the backward call needs of this call in ``workspace`` (required then, see
    lsm_delta_workspace) for lsm_delta_bwd(..., workspace=the same tensor, states_saved=True) on the same inputs."""
    import torch
    if save_states and workspace is None:
        raise ValueError("save_states needs a caller-owned workspace that is passed on to lsm_delta_bwd")
    kind = DECAY_NONE if log_alpha is None else DECAY_SCALAR
    p, (B, H, T, dk, dv), gshape = _setup(q, k, v, log_alpha, kind, 64, layout, cu_seqlens, FLAG_SAVE_STATES if save_states else 0)
    pshape = tuple(q.shape[:3])   # per-token scalars follow q's first three axes (B is the sequence count for packed input)
    _check(beta, pshape, torch.float32, "beta")
    _check(b, pshape, torch.float32, "b")
    _check(init_state, (B, H, dk, dv), torch.float32, "init_state")
    need = library().lsm_delta_fwd_workspace_bytes(ctypes.byref(p))
    if need == 0:
        raise LsmError(-3, "lsm_delta_fwd")
    with _alloc_on(stream):
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        o = torch.empty_like(v)
        final = torch.empty((B, H, dk, dv), dtype=torch.float32, device=q.device) if want_final_state else None
    rc = library().lsm_delta_fwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(beta), _ptr(b),
                                 _ptr(init_state), _ptr(o), _ptr(final), _ptr(workspace), workspace.numel(),
                                 _stream_handle(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_delta_fwd")
    return o, final


def lsm_delta_bwd(q, k, v, d_o, log_alpha=None, beta=None, b=None, init_state=None, d_final_state=None, workspace=None,
                  stream=None, layout=LAYOUT_BHTD, want_d_init_state=True, states_saved=False, cu_seqlens=None):
    """Gradients of L = <o, d_o> + <M_T, d_final_state> for the delta-rule rows (see lsm_delta_fwd): a dict with dq, dk,
    dv (like q, k, v), d_log_alpha, d_beta, d_b (float32 per token, None where the parameter was None) and
    d_init_state.  states_saved: ``workspace`` is the one a preceding lsm_delta_fwd(..., save_states=True) on the same
    inputs filled."""
    import torch
    if states_saved and workspace is None:
        raise ValueError("states_saved needs the workspace of the forward call")
    kind = DECAY_NONE if log_alpha is None else DECAY_SCALAR
    p, (B, H, T, dk, dv), gshape = _setup(q, k, v, log_alpha, kind, 64, layout, cu_seqlens, FLAG_SAVE_STATES if states_saved else 0)
    pshape = tuple(q.shape[:3])
    _check(beta, pshape, torch.float32, "beta")
    _check(b, pshape, torch.float32, "b")
    _check(d_o, tuple(v.shape), q.dtype, "d_o")
    _check(init_state, (B, H, dk, dv), torch.float32, "init_state")
    _check(d_final_state, (B, H, dk, dv), torch.float32, "d_final_state")
    need = library().lsm_delta_bwd_workspace_bytes(ctypes.byref(p))
    if need == 0:
        raise LsmError(-3, "lsm_delta_bwd")
    with _alloc_on(stream):
        if workspace is None:
            workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
        dq, dk_, dv_ = torch.empty_like(q), torch.empty_like(k), torch.empty_like(v)
        par = lambda x: None if x is None else torch.empty(pshape, dtype=torch.float32, device=q.device)
        dla, dbe, dbw = par(log_alpha), par(beta), par(b)
        d_m0 = torch.empty((B, H, dk, dv), dtype=torch.float32, device=q.device) if want_d_init_state else None
    rc = library().lsm_delta_bwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(log_alpha), _ptr(beta), _ptr(b),
                                 _ptr(init_state), _ptr(d_o), _ptr(d_final_state), _ptr(dq), _ptr(dk_), _ptr(dv_),
                                 _ptr(dla), _ptr(dbe), _ptr(dbw), _ptr(d_m0), _ptr(workspace), workspace.numel(),
                                 _stream_handle(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_delta_bwd")
    return dict(dq=dq, dk=dk_, dv=dv_, d_log_alpha=dla, d_beta=dbe, d_b=dbw, d_init_state=d_m0)


NOALLOC_SCRATCH_BYTES = 8 << 20


def lsm_chunk_fwd_noalloc(q, k, v, log_decay, decay_kind, o, final_state=None, chunk_size=64, init_state=None, stream=None,
                          layout=LAYOUT_BHTD, cu_seqlens=None):
    """lsm_chunk_fwd without a workspace: the library's built-in scratch is used, nothing is allocated
    (the caller passes the outputs ``o`` and, if wanted, ``final_state``).  Raises LsmError (workspace) for
    shapes whose scratch need exceeds NOALLOC_SCRATCH_BYTES."""
    import torch
    p, (B, H, T, dk, dv), _ = _setup(q, k, v, log_decay, decay_kind, chunk_size, layout, cu_seqlens, 0)
    _check(init_state, (B, H, dk, dv), torch.float32, "init_state")
    _check(final_state, (B, H, dk, dv), torch.float32, "final_state")
    _check(o, tuple(v.shape), q.dtype, "o")
    if o is None:
        raise ValueError("o is required")
    rc = library().lsm_chunk_fwd_noalloc(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(log_decay), _ptr(init_state),
                                         _ptr(o), _ptr(final_state), _stream_handle(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_chunk_fwd_noalloc")
    return o, final_state


def lsm_step(q, k, v, log_decay, decay_kind, state, o=None, stream=None):
    """One recurrent step: ``state`` [B,H,d_k,d_v] fp32 is updated in place, returns o [B,H,d_v].

    q, k [B,H,d_k], v [B,H,d_v]; log_decay None / [H] / [B,H] / [B,H,d_k] by decay kind."""
    import torch
    B, H, dk = q.shape
    dv = v.shape[-1]
    tdt = {torch.float32: 0, torch.bfloat16: 1}[q.dtype]
    p = make_params(B, H, 1, dk, dv, 64, decay_kind, tdt)
    _check(q, (B, H, dk), q.dtype, "q"); _check(k, (B, H, dk), q.dtype, "k"); _check(v, (B, H, dv), q.dtype, "v")
    gshape = {DECAY_NONE: None, DECAY_HEAD: (H,), DECAY_SCALAR: (B, H), DECAY_VECTOR: (B, H, dk)}[decay_kind]
    if gshape is None:
        if log_decay is not None:
            raise ValueError("log_decay must be None for DECAY_NONE")
    else:
        _check(log_decay, gshape, torch.float32, "log_decay")
        if log_decay is None:
            raise ValueError("log_decay is required for this decay kind")
    _check(state, (B, H, dk, dv), torch.float32, "state")
    if state is None:
        raise ValueError("state is required")
    if o is None:
        o = torch.empty((B, H, dv), dtype=q.dtype, device=q.device)
    rc = library().lsm_step(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(log_decay), _ptr(state), _ptr(o),
                            _stream_handle(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_step")
    return o


def lsm_bench_intra_chunk(q, k, v, log_decay, decay_kind, o, workspace, repeats, chunk_size=64, stream=None):
    """Benchmark aid: the intra-chunk forward kernel with its compute phase repeated ``repeats`` times.

    ``workspace``: at least lsm_bench_intra_chunk_workspace(...) bytes (None: allocated here)."""
    p, _, _ = _setup(q, k, v, log_decay, decay_kind, chunk_size)
    if workspace is None:
        workspace = lsm_bench_intra_chunk_workspace(q, k, v, log_decay, decay_kind, chunk_size)
    rc = library().lsm_bench_intra_chunk(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(log_decay), _ptr(o),
                                         _ptr(workspace), workspace.numel(), int(repeats), _stream_handle(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_bench_intra_chunk")


def lsm_calib_copy(dst, src, stream=None):
    """Benchmark aid: dst <- src with the library's plain streaming-copy kernel (uint8 tensors, equal sizes)."""
    rc = library().lsm_calib_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size(), _stream_handle(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_calib_copy")


def lsm_calib_mfma(out, workgroups, iters, stream=None):
    """Benchmark aid: a loop of nothing but bf16 MFMAs; returns the flop count of the launch."""
    rc = library().lsm_calib_mfma(_ptr(out), int(workgroups), int(iters), _stream_handle(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_calib_mfma")
    return float(library().lsm_calib_mfma_flops(int(workgroups), int(iters)))


def lsm_bench_intra_chunk_workspace(q, k, v, log_decay, decay_kind, chunk_size=64):
    import torch
    p, _, _ = _setup(q, k, v, log_decay, decay_kind, chunk_size)
    need = int(library().lsm_bench_intra_chunk_workspace_bytes(ctypes.byref(p)))
    return torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)


def lsm_chunk_bwd(q, k, v, log_decay, decay_kind, d_o, chunk_size=64, init_state=None, d_final_state=None,
                  want_d_log_decay=True, want_d_init_state=True, workspace=None, stream=None,
                  layout=LAYOUT_BHTD, cu_seqlens=None, states_saved=False):
    """dict(dq, dk, dv, dg, d_init_state): chunkwise backward of <o, d_o> + <M_T, d_final_state>.

    states_saved: ``workspace`` is the tensor that lsm_chunk_fwd(..., save_states=True) filled for the same
    inputs and nothing has written to it since; the chunk states are then read from it, not recomputed."""
    import torch
    if states_saved and workspace is None:
        raise ValueError("states_saved needs the workspace of the forward call")
    p, (B, H, T, dk, dv), gshape = _setup(q, k, v, log_decay, decay_kind, chunk_size, layout, cu_seqlens,
                                          _save_flags(states_saved))
    _check(init_state, (B, H, dk, dv), torch.float32, "init_state")
    _check(d_final_state, (B, H, dk, dv), torch.float32, "d_final_state")
    _check(d_o, tuple(v.shape), q.dtype, "d_o")
    need = lsm_chunk_bwd_workspace_bytes(p)
    with _alloc_on(stream):
        if workspace is None:
            workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
        dq = torch.empty_like(q)
        dk_ = torch.empty_like(k)
        dv_ = torch.empty_like(v)
        dg = torch.empty(gshape, dtype=torch.float32, device=q.device) if (gshape and want_d_log_decay) else None
        d_init = torch.empty((B, H, dk, dv), dtype=torch.float32, device=q.device) if want_d_init_state else None
    rc = library().lsm_chunk_bwd(ctypes.byref(p), _ptr(q), _ptr(k), _ptr(v), _ptr(log_decay), _ptr(init_state),
                                 _ptr(d_o), _ptr(d_final_state), _ptr(dq), _ptr(dk_), _ptr(dv_), _ptr(dg),
                                 _ptr(d_init), _ptr(workspace), workspace.numel(), _stream_handle(stream))
    if rc != 0:
        raise LsmError(rc, "lsm_chunk_bwd")
    return dict(dq=dq, dk=dk_, dv=dv_, dg=dg, d_init_state=d_init)
