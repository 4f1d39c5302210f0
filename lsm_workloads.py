"""Seeded synthetic inputs for the LSM hot path (shared by tests, bench, smoke).

Holds NO arithmetic of the method: only random draws, the value distributions
of the benchmark configurations, and bf16 round-to-nearest-even of the drawn
values (so that the CPU oracle and the GPU library consume identical numbers).

The five named configurations stand in for the activations of the paper's
A0.3B-2B / A1B-7B model series (Table 2: head dim 128, 8 or 16 heads, trained
at 2K tokens, efficiency runs at 2K-16K tokens); the corpus and weights are
not needed, only shapes and scales.
"""
import numpy as np

KIND_NONE, KIND_HEAD, KIND_SCALAR, KIND_VECTOR = 0, 1, 2, 3
KIND_NAMES = {0: "none", 1: "head", 2: "scalar", 3: "vector"}

BASE_SEED = 20250305


def bf16_round(x):
    """Round float32 values to the nearest bf16 (ties to even); returns float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    r = ((u + 0x7FFF + lsb) >> 16) << 16
    return r.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x):
    """uint16 bit patterns of float32 values that are already bf16-exact."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def _softplus(x):
    return np.logaddexp(0.0, x)


def g_shape(kind, B, H, T, dk):
    return {KIND_NONE: None, KIND_HEAD: (H,), KIND_SCALAR: (B, H, T), KIND_VECTOR: (B, H, T, dk)}[kind]


def make_inputs(B, H, T, dk, dv, kind, dtype="bf16", seed=0, decay="default",
                init_state=False, d_final=False, init_std=0.1):
    """Draw q, k, v, g, m0, d_o, d_mT (in this order) from one seeded stream.

    q, k, v ~ N(0,1)/sqrt(dk); d_o ~ N(0,1).  ``decay`` picks the log-decay law:
      head kind   : g_h = -2^-(5 + 8 h / H)                          (config 2)
      "default"   : scalar -softplus(N+3) ; vector logsigmoid(N)/16  (configs 3, 4)
      "strong4"   : scalar -softplus(N+4)                            (config 5)
      "weak"      : -softplus(N-4)     (inter-chunk terms dominate)
      "harsh"     : -20 * U(0,1)       (underflow stress)
      "zero"      : all zeros
    Values are float32; with dtype "bf16" q, k, v, d_o are rounded to bf16.
    """
    rng = np.random.default_rng(seed)
    scale = np.float32(1.0 / np.sqrt(dk))
    q = rng.standard_normal((B, H, T, dk), dtype=np.float32) * scale
    k = rng.standard_normal((B, H, T, dk), dtype=np.float32) * scale
    v = rng.standard_normal((B, H, T, dv), dtype=np.float32) * scale
    gs = g_shape(kind, B, H, T, dk)
    g = None
    if kind == KIND_HEAD:
        n = rng.standard_normal(gs, dtype=np.float32)
        if decay in ("default", "strong4"):
            g = -np.exp2(-(5.0 + 8.0 * np.arange(H) / H)).astype(np.float32)
        elif decay == "weak":
            g = (-_softplus(n - 4.0)).astype(np.float32)
        elif decay == "harsh":
            g = (-3.0 * np.abs(n)).astype(np.float32)
        else:
            g = np.zeros(gs, dtype=np.float32)
    elif gs is not None:
        n = rng.standard_normal(gs, dtype=np.float32)
        if decay == "default":
            g = -_softplus(n + 3.0) if kind == KIND_SCALAR else -_softplus(-n) / 16.0
        elif decay == "strong4":
            g = -_softplus(n + 4.0)
        elif decay == "weak":
            g = -_softplus(n - 4.0)
        elif decay == "harsh":
            g = -20.0 * rng.random(gs, dtype=np.float32)
        elif decay == "zero":
            g = np.zeros(gs)
        else:
            raise ValueError(decay)
        g = np.ascontiguousarray(g, dtype=np.float32)
    m0 = (rng.standard_normal((B, H, dk, dv), dtype=np.float32) * np.float32(init_std)) if init_state else None
    d_o = rng.standard_normal((B, H, T, dv), dtype=np.float32)
    d_mT = rng.standard_normal((B, H, dk, dv), dtype=np.float32) * np.float32(init_std) if d_final else None
    if dtype == "bf16":
        q, k, v, d_o = bf16_round(q), bf16_round(k), bf16_round(v), bf16_round(d_o)
    elif dtype != "f32":
        raise ValueError(dtype)
    return dict(q=q, k=k, v=v, g=g, m0=m0, d_o=d_o, d_mT=d_mT, kind=kind, dtype=dtype,
                B=B, H=H, T=T, dk=dk, dv=dv)


def make_delta_inputs(B, H, T, dk, dv, gated, dtype="bf16", seed=0, decay="default", init_state=False, d_final=False,
                      init_std=0.1, tie_b=True):
    """Inputs of the delta-rule rows (DeltaNet: gated False; Gated DeltaNet: gated True), from one seeded stream.

    q ~ N(0,1)/sqrt(dk); k drawn N(0,1) and scaled to unit length (as the delta-rule models normalise their keys);
    v ~ N(0,1); the row's write strength b_s = sigmoid(N(0,1)); DeltaNet's erase strength a_s = b_s (``tie_b``, the
    usual parametrisation) or an independent draw of the same law; Gated DeltaNet's decay log a_s by the scalar-decay
    law named by ``decay`` (see make_inputs; "harsh" = -20 U(0,1)).  Values are float32; with dtype "bf16" q, k, v, d_o are rounded to bf16
    (so a key's length is 1 up to that rounding).
    """
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((B, H, T, dk), dtype=np.float32) * np.float32(1.0 / np.sqrt(dk))
    k = rng.standard_normal((B, H, T, dk), dtype=np.float32)
    k /= np.maximum(np.sqrt((k * k).sum(-1, keepdims=True)), np.float32(1e-6))
    v = rng.standard_normal((B, H, T, dv), dtype=np.float32)
    sig = lambda n: (1.0 / (1.0 + np.exp(-n))).astype(np.float32)
    b = sig(rng.standard_normal((B, H, T), dtype=np.float32))
    n2 = rng.standard_normal((B, H, T), dtype=np.float32)
    n3 = rng.standard_normal((B, H, T), dtype=np.float32)
    beta = None if gated else (b.copy() if tie_b else sig(n2))
    log_alpha = None
    if gated:
        if decay == "harsh":    # underflow stress, as for the diagonal kinds
            log_alpha = (-20.0 * rng.random((B, H, T), dtype=np.float32)).astype(np.float32)
        else:
            shift = {"default": 3.0, "strong4": 4.0, "weak": -4.0}.get(decay)
            if shift is None:
                raise ValueError(decay)
            log_alpha = np.ascontiguousarray(-_softplus(n3 + shift), dtype=np.float32)
    m0 = (rng.standard_normal((B, H, dk, dv), dtype=np.float32) * np.float32(init_std)) if init_state else None
    d_o = rng.standard_normal((B, H, T, dv), dtype=np.float32)
    d_mT = rng.standard_normal((B, H, dk, dv), dtype=np.float32) * np.float32(init_std) if d_final else None
    if dtype == "bf16":
        q, k, v, d_o = bf16_round(q), bf16_round(k), bf16_round(v), bf16_round(d_o)
    elif dtype != "f32":
        raise ValueError(dtype)
    return dict(q=q, k=k, v=v, log_alpha=log_alpha, beta=beta, b=b, m0=m0, d_o=d_o, d_mT=d_mT, gated=gated, dtype=dtype,
                B=B, H=H, T=T, dk=dk, dv=dv)


# The five benchmark configurations (index 0..4 = configs 1..5 of the benchmark spec).
CONFIGS = [
    dict(name="config1_bla_f32", B=1, H=2, T=256, dk=64, dv=64, kind=KIND_NONE, dtype="f32",
         decay="default", init_state=False, backward=False, chunk=64),
    dict(name="config2_fixed_head", B=8, H=16, T=2048, dk=128, dv=128, kind=KIND_HEAD, dtype="bf16",
         decay="default", init_state=False, backward=True, chunk=64),
    dict(name="config3_scalar", B=4, H=16, T=8192, dk=128, dv=128, kind=KIND_SCALAR, dtype="bf16",
         decay="default", init_state=False, backward=True, chunk=64),
    dict(name="config4_vector", B=4, H=16, T=4096, dk=128, dv=256, kind=KIND_VECTOR, dtype="bf16",
         decay="default", init_state=False, backward=True, chunk=64),
    dict(name="config5_long_carried", B=1, H=32, T=65536, dk=128, dv=128, kind=KIND_SCALAR, dtype="bf16",
         decay="strong4", init_state=True, backward=True, chunk=64),
]


def make_config(index, **override):
    """Inputs of benchmark configuration ``index`` (0-based); shape keys may be overridden."""
    c = dict(CONFIGS[index])
    c.update(override)
    return make_inputs(c["B"], c["H"], c["T"], c["dk"], c["dv"], c["kind"], dtype=c["dtype"],
                       seed=BASE_SEED + index + 1, decay=c["decay"], init_state=c["init_state"]), c
