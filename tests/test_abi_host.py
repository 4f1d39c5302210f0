"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
include/lsm.h declares, and rejects bad arguments before any HIP call."""
import ctypes
import os
import re

import pytest

import paper_2503_05447_amd as pkg
from paper_2503_05447_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    """Every function that any header under include/ declares."""
    import glob
    names = set()
    for h in glob.glob(os.path.join(ROOT, "include", "*.h")):
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(lsm_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported():
    lib = pkg.library()
    names = declared_symbols()
    assert {"lsm_chunk_fwd", "lsm_chunk_bwd", "lsm_chunk_fwd_workspace_bytes", "lsm_chunk_bwd_workspace_bytes",
            "lsm_status_string", "lsm_version", "lsm_kernel_path", "lsm_bench_intra_chunk", "lsm_chunk_fwd_noalloc",
            "lsm_step", "lsm_calib_copy", "lsm_calib_mfma", "lsm_profile_start"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert lib.lsm_version() >= 1


def P(**kw):
    base = dict(B=2, H=2, T=100, d_k=64, d_v=64, chunk_size=64, decay_kind=2, dtype=1)
    base.update(kw)
    return pkg.make_params(**base)


def fwd(p, q=0x1000, k=0x2000, v=0x3000, g=0x4000, m0=None, o=0x5000, mT=None, ws=0x10000, wsb=1 << 40):
    vp = ctypes.c_void_p
    return pkg.library().lsm_chunk_fwd(ctypes.byref(p), vp(q), vp(k), vp(v), vp(g), vp(m0), vp(o), vp(mT), vp(ws), wsb, vp(None))


def bwd(p, q=0x1000, k=0x2000, v=0x3000, g=0x4000, m0=None, d_o=0x6000, dmT=None, dq=0x7000, dk=0x8000, dv=0x9000,
        dg=0xa000, dm0=None, ws=0x10000, wsb=1 << 40):
    vp = ctypes.c_void_p
    return pkg.library().lsm_chunk_bwd(ctypes.byref(p), vp(q), vp(k), vp(v), vp(g), vp(m0), vp(d_o), vp(dmT), vp(dq),
                                       vp(dk), vp(dv), vp(dg), vp(dm0), vp(ws), wsb, vp(None))


def test_error_codes_are_reached_before_any_launch():
    ERR_NULL, ERR_SHAPE, ERR_UNSUP, ERR_ALIGN, ERR_WS = -1, -2, -3, -4, -5
    assert fwd(P(), q=None) == ERR_NULL
    assert fwd(P(), o=None) == ERR_NULL
    assert fwd(P(), g=None) == ERR_NULL                       # decay required
    assert fwd(P(decay_kind=0)) == ERR_NULL                   # decay forbidden for kind none
    assert bwd(P(decay_kind=0), g=None) == ERR_NULL           # d_log_decay forbidden for kind none
    assert bwd(P(), dq=None) == ERR_NULL
    assert fwd(P(T=0)) == ERR_SHAPE
    assert fwd(P(B=-1)) == ERR_SHAPE
    assert fwd(P(B=256, H=256)) == ERR_SHAPE                  # B * H beyond the largest grid dimension (65535)
    bad = P(); bad.struct_size = 12
    assert fwd(bad) == ERR_SHAPE
    assert fwd(P(d_k=96)) == ERR_UNSUP
    assert fwd(P(d_v=512)) == ERR_UNSUP
    assert fwd(P(chunk_size=48)) == ERR_UNSUP
    assert fwd(P(decay_kind=4)) == ERR_UNSUP
    assert fwd(P(dtype=2)) == ERR_UNSUP
    assert fwd(P(), k=0x2004) == ERR_ALIGN
    assert bwd(P(), dm0=0xb008) == ERR_ALIGN
    assert fwd(P(), ws=None) == ERR_WS
    assert fwd(P(), wsb=16) == ERR_WS
    assert bwd(P(), wsb=16) == ERR_WS
    # layout and packed variable-length input
    assert fwd(P(layout=2)) == ERR_UNSUP
    assert fwd(P(n_seq=2, cu_seqlens=0x20000)) == ERR_SHAPE            # packed input needs B == 1
    assert fwd(P(B=1, n_seq=2)) == ERR_NULL                            # cu_seqlens missing
    assert fwd(P(B=1, cu_seqlens=0x20000)) == ERR_NULL                 # cu_seqlens without n_seq
    assert fwd(P(B=1, n_seq=2, cu_seqlens=0x20004)) == ERR_ALIGN
    assert fwd(P(B=1, n_seq=-1)) == ERR_SHAPE
    # recurrent step and benchmark aid: same checks, before any HIP call
    vp = ctypes.c_void_p
    lib = pkg.library()
    step = lambda p, q=0x1000, g=0x4000, st=0x5000: lib.lsm_step(ctypes.byref(p), vp(q), vp(0x2000), vp(0x3000), vp(g), vp(st),
                                                                  vp(0x6000), vp(None))
    assert step(P(T=1), q=None) == ERR_NULL
    assert step(P(T=1), st=None) == ERR_NULL
    assert step(P(T=1), g=None) == ERR_NULL
    assert step(P(T=1, decay_kind=0)) == ERR_NULL
    assert step(P(T=1, d_k=96)) == ERR_UNSUP
    assert step(P(T=1), st=0x5004) == ERR_ALIGN
    assert lib.lsm_bench_intra_chunk(ctypes.byref(P()), vp(0x1000), vp(0x2000), vp(0x3000), vp(0x4000), vp(0x5000),
                                     vp(0x10000), 1 << 40, 4, vp(None)) == ERR_UNSUP   # d = 64 is not on the MFMA path
    assert pkg.library().lsm_chunk_fwd(None, *([ctypes.c_void_p(None)] * 8), 0, ctypes.c_void_p(None)) == ERR_NULL
    # the entry point without a workspace: the same checks, and the size limit of its built-in scratch
    na = lambda p, q=0x1000, o=0x5000: lib.lsm_chunk_fwd_noalloc(ctypes.byref(p), vp(q), vp(0x2000), vp(0x3000), vp(0x4000),
                                                                   vp(None), vp(o), vp(None), vp(None))
    assert na(P(), q=None) == ERR_NULL
    assert na(P(), o=0x5004) == ERR_ALIGN
    assert na(P(d_k=96)) == ERR_UNSUP
    big = P(B=4, H=16, T=8192, d_k=128, d_v=128)
    assert pkg.lsm_chunk_fwd_workspace_bytes(big) > pkg.NOALLOC_SCRATCH_BYTES and na(big) == ERR_WS


def test_workspace_queries_and_status_strings():
    p = P()
    f, b = pkg.lsm_chunk_fwd_workspace_bytes(p), pkg.lsm_chunk_bwd_workspace_bytes(p)
    assert f > 0 and b >= f
    assert pkg.lsm_chunk_fwd_workspace_bytes(P(d_k=3)) == 0
    assert pkg.lsm_chunk_bwd_workspace_bytes(P(T=0)) == 0
    assert pkg.kernel_path(P()) in (0, 1)
    assert pkg.kernel_path(P(dtype=0)) == 0                   # fp32 inputs never take bf16 MFMA operands
    assert pkg.kernel_path(P(d_k=3)) < 0
    # workspace grows with the number of chunks
    assert pkg.lsm_chunk_fwd_workspace_bytes(P(T=6400)) > f
    assert pkg.lsm_chunk_fwd_workspace_bytes(P(B=1, n_seq=3, cu_seqlens=0x20000)) > pkg.lsm_chunk_fwd_workspace_bytes(P(B=1))
    for s in range(0, -7, -1):
        assert len(binding._status_string(s)) > 1
    assert binding._status_string(-99) == "unknown status"
    with pytest.raises(pkg.LsmError):
        raise pkg.LsmError(-3, "x")


def test_binding_rejects_host_tensors():
    import torch
    q = torch.zeros(1, 1, 8, 64)
    with pytest.raises(ValueError):
        pkg.lsm_chunk_fwd(q, q, q, None, pkg.DECAY_NONE, 64)


def test_saved_state_flags_and_workspace_sizes():
    """One buffer serves both calls when states are kept; the flag checks are host logic."""
    fwdb, bwdb = pkg.lsm_chunk_fwd_workspace_bytes, pkg.lsm_chunk_bwd_workspace_bytes
    big = dict(B=4, H=16, T=8192, d_k=128, d_v=128)
    plain, keep = P(**big), P(**big, flags=pkg.FLAG_SAVE_STATES)
    assert fwdb(keep) == bwdb(keep) == bwdb(plain) > fwdb(plain) > 0   # the backward carving starts with the forward's
    assert pkg.keeps_states(keep) == 1 and pkg.keeps_states(plain) == 0
    # scalar kinds keep one state per segment of chunks, not one per chunk: a fraction of the inputs' size
    assert fwdb(plain) < 4 * 16 * 8192 * 128 * 2 // 2
    assert pkg.keeps_states(P(**big, decay_kind=3, flags=1)) == 1
    assert fwdb(P(**big, decay_kind=3, flags=1)) > bwdb(P(**big, decay_kind=3))   # vector kind: chunk states in both orders
    # kernels that keep nothing: the one buffer is the larger of the two
    gen = dict(B=2, H=2, T=300, d_k=64, d_v=64, dtype=0)
    assert pkg.keeps_states(P(**gen, flags=1)) == 0
    assert fwdb(P(**gen, flags=3)) == bwdb(P(**gen, flags=3)) == max(fwdb(P(**gen)), bwdb(P(**gen)))
    # benchmark aid: its own workspace figure, zero where it does not apply
    aid = pkg.library().lsm_bench_intra_chunk_workspace_bytes
    assert aid(ctypes.byref(plain)) >= 4 * 16 * 128 * 128 * 128 * 2 and aid(ctypes.byref(P(**gen))) == 0
    ERR_UNSUP = -3
    assert fwd(P(flags=2)) == ERR_UNSUP          # "always" without the flag it qualifies
    assert fwd(P(flags=4)) == ERR_UNSUP
    assert bwd(P(flags=8)) == ERR_UNSUP


def test_delta_rule_entry_points_reject_bad_arguments_before_any_launch():
    ERR_NULL, ERR_UNSUP, ERR_ALIGN, ERR_WS = -1, -3, -4, -5
    vp = ctypes.c_void_p
    lib = pkg.library()

    def dfwd(p, q=0x1000, k=0x2000, v=0x3000, la=None, be=0x4000, b=0x4100, m0=None, o=0x5000, mT=None, ws=0x10000, wsb=1 << 40):
        return lib.lsm_delta_fwd(ctypes.byref(p), vp(q), vp(k), vp(v), vp(la), vp(be), vp(b), vp(m0), vp(o), vp(mT), vp(ws), wsb,
                                 vp(None))

    def dbwd(p, la=None, be=0x4000, b=0x4100, dla=None, dbe=0xb000, db=0xc000, d_o=0x6000, dq=0x7000, ws=0x10000, wsb=1 << 40):
        return lib.lsm_delta_bwd(ctypes.byref(p), vp(0x1000), vp(0x2000), vp(0x3000), vp(la), vp(be), vp(b), vp(None), vp(d_o),
                                 vp(None), vp(dq), vp(0x8000), vp(0x9000), vp(dla), vp(dbe), vp(db), vp(None), vp(ws), wsb, vp(None))

    ok = P(d_k=128, d_v=128, decay_kind=0)
    gated = P(d_k=128, d_v=128, decay_kind=2)
    need_f, need_b = lib.lsm_delta_fwd_workspace_bytes(ctypes.byref(ok)), lib.lsm_delta_bwd_workspace_bytes(ctypes.byref(ok))
    assert 0 < need_f < need_b
    keep = P(d_k=128, d_v=128, decay_kind=0, flags=pkg.FLAG_SAVE_STATES)   # one buffer serves both calls
    assert lib.lsm_delta_fwd_workspace_bytes(ctypes.byref(keep)) == lib.lsm_delta_bwd_workspace_bytes(ctypes.byref(keep)) == need_b
    # shapes the rows are not served for: the size query says 0 and the calls say unsupported
    for bad in (P(d_k=64, d_v=64, decay_kind=0), P(d_k=128, d_v=128, decay_kind=0, dtype=0), P(d_k=128, d_v=128, decay_kind=0, chunk_size=32),
                P(d_k=128, d_v=256, decay_kind=0)):
        assert lib.lsm_delta_fwd_workspace_bytes(ctypes.byref(bad)) == 0
        assert dfwd(bad) == ERR_UNSUP and dbwd(bad) == ERR_UNSUP
    assert dfwd(P(d_k=128, d_v=128, decay_kind=1), la=0x4200) == ERR_UNSUP      # per-head and vector decays: not these rows
    assert dfwd(P(d_k=128, d_v=128, decay_kind=3), la=0x4200) == ERR_UNSUP
    assert dfwd(ok, q=None) == ERR_NULL and dfwd(ok, o=None) == ERR_NULL
    assert dfwd(ok, la=0x4200) == ERR_NULL          # a decay without decay_kind scalar
    assert dfwd(gated) == ERR_NULL                  # decay_kind scalar without a decay
    assert dfwd(ok, be=0x4004) == ERR_ALIGN
    assert dfwd(ok, ws=None) == ERR_WS and dfwd(ok, wsb=need_f - 1) == ERR_WS
    # backward: a gradient exactly where a parameter was given
    assert dbwd(ok, dbe=None) == ERR_NULL and dbwd(ok, be=None) == ERR_NULL
    assert dbwd(ok, dla=0xd000) == ERR_NULL
    assert dbwd(gated, la=0x4200) == ERR_NULL       # d_log_alpha missing
    assert dbwd(ok, d_o=None) == ERR_NULL and dbwd(ok, dq=None) == ERR_NULL
    assert dbwd(ok, wsb=need_b - 1) == ERR_WS
