"""fp64 CPU oracle for the bidirectional Mamba mixer path -- TEST INFRASTRUCTURE.

Thin ctypes marshalling around oracle/bimamba_oracle.c (all arithmetic lives in
the C file).  Only tests, the smoke check and the benchmark's cpu_baseline leg
may import this package; the HIP library never does.

Arrays are numpy.  Activations and parameters are float32 arrays whose values
are exactly representable in the I/O dtype under test; results are float64.
"""
import ctypes as C
import os

import numpy as np

from .build import LIB, LIB_UBSAN
from .build import build as build_lib
from .build import build_sanitized

_lib = None


class Desc(C.Structure):
    _fields_ = [(n, C.c_int) for n in (
        "batch", "seqlen", "d_inner", "d_state", "n_heads", "n_groups", "d_conv",
        "a_kind", "d_kind", "dt_softplus", "conv_bc", "combine")]


class Params(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("conv_w", "conv_b", "A", "D", "dt_bias")]


class Inputs(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("x", "z", "dt", "B", "C")]


def lib():
    global _lib
    if _lib is None:
        path = LIB
        if os.environ.get("BIMAMBA_ORACLE_UBSAN"):     # the pins under the undefined-behaviour sanitizer (tests only)
            path = build_sanitized()[0]
        elif not os.path.exists(LIB):
            build_lib()
        _lib = C.CDLL(path)
        _lib.orc_bimamba_fwd.restype = C.c_int
        _lib.orc_bimamba_block_fwd.restype = C.c_int
        _lib.orc_one_direction.restype = C.c_int
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def _f32(a):
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def _f64(a):
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.float64))


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _desc(cfg, seqlen=None):
    return Desc(cfg["batch"], cfg["seqlen"] if seqlen is None else seqlen, cfg["d_inner"], cfg["d_state"],
                cfg["n_heads"], cfg["n_groups"], cfg["d_conv"], cfg.get("a_kind", 0), cfg.get("d_kind", 0),
                cfg.get("dt_softplus", 0), cfg.get("conv_bc", 0), cfg.get("combine", 0))


def _params(p):
    keep = {k: _f32(p.get(k)) for k in ("conv_w", "conv_b", "A", "D", "dt_bias")}
    return Params(*[_ptr(keep[k]) for k in ("conv_w", "conv_b", "A", "D", "dt_bias")]), keep


def _inputs(i):
    keep = {k: _f32(i[k]) for k in ("x", "z", "dt", "B", "C")}
    return Inputs(*[_ptr(keep[k]) for k in ("x", "z", "dt", "B", "C")]), keep


def _sel(sel):
    if sel is None:
        return None, 0, None
    s = np.ascontiguousarray(np.asarray(sel, dtype=np.int32))
    return s.ctypes.data_as(C.c_void_p), int(s.size), s


def num_threads():
    return lib().orc_num_threads()


def set_num_threads(n):
    lib().orc_set_num_threads(C.c_int(int(n)))


def bimamba_fwd(cfg, params_f, params_b, in_f, in_b=None, sel=None):
    """out[batch, L, n_sel] (combine=0) or [batch, L, 2, n_sel] (combine=1), float64."""
    d = _desc(cfg)
    pf, k1 = _params(params_f)
    pb, k2 = _params(params_b)
    i_f, k3 = _inputs(in_f)
    i_b, k4 = _inputs(in_f if in_b is None else in_b)
    sp, ns, k5 = _sel(sel)
    n_sel = ns if sel is not None else cfg["d_inner"]
    shape = (cfg["batch"], cfg["seqlen"], n_sel) if not cfg.get("combine", 0) else (cfg["batch"], cfg["seqlen"], 2, n_sel)
    out = np.zeros(shape, dtype=np.float64)
    rc = lib().orc_bimamba_fwd(C.byref(d), C.byref(pf), C.byref(pb), C.byref(i_f), C.byref(i_b),
                               sp, C.c_int(ns), _ptr(out))
    if rc != 0:
        raise ValueError("oracle: shape outside the definition")
    return out


def bimamba_block_fwd(cfg, params_f, params_b, in_f, in_b=None, h_in=None, tail_in=None, sel=None,
                      want_h=True, want_tail=True):
    """Returns (out, h_out, tail_out); h_out [batch, d_inner, d_state], tail_out [batch, d_conv-1, tail_ch], float64."""
    d = _desc(cfg)
    pf, k1 = _params(params_f)
    pb, k2 = _params(params_b)
    i_f, k3 = _inputs(in_f)
    i_b, k4 = _inputs(in_f if in_b is None else in_b)
    sp, ns, k5 = _sel(sel)
    n_sel = ns if sel is not None else cfg["d_inner"]
    Bt, L, Dn, N, K = cfg["batch"], cfg["seqlen"], cfg["d_inner"], cfg["d_state"], cfg["d_conv"]
    tail_ch = Dn + (2 * cfg["n_groups"] * N if cfg.get("conv_bc", 0) else 0)
    shape = (Bt, L, n_sel) if not cfg.get("combine", 0) else (Bt, L, 2, n_sel)
    out = np.zeros(shape, dtype=np.float64)
    hin = _f64(h_in)
    tin = _f64(tail_in)
    if hin is not None:
        assert hin.shape == (Bt, Dn, N)
    if tin is not None:
        assert tin.shape == (Bt, K - 1, tail_ch)
    h_out = np.zeros((Bt, Dn, N), dtype=np.float64) if want_h else None
    tail_out = np.zeros((Bt, K - 1, tail_ch), dtype=np.float64) if want_tail else None
    rc = lib().orc_bimamba_block_fwd(C.byref(d), C.byref(pf), C.byref(pb), C.byref(i_f), C.byref(i_b),
                                     _ptr(hin), _ptr(tin), sp, C.c_int(ns), _ptr(out), _ptr(h_out), _ptr(tail_out))
    if rc != 0:
        raise ValueError("oracle: shape outside the definition")
    return out, h_out, tail_out


def one_direction(cfg, params, inputs, direction, h_in=None, tail_in=None, want_h=True):
    """Gated single-direction output g[batch, L, d_inner] and final state (direction=+1 forward, -1 reverse)."""
    d = _desc(cfg)
    p, k1 = _params(params)
    i, k2 = _inputs(inputs)
    Bt, L, Dn, N = cfg["batch"], cfg["seqlen"], cfg["d_inner"], cfg["d_state"]
    g = np.zeros((Bt, L, Dn), dtype=np.float64)
    hin = _f64(h_in)
    tin = _f64(tail_in)
    h_out = np.zeros((Bt, Dn, N), dtype=np.float64) if want_h else None
    rc = lib().orc_one_direction(C.byref(d), C.byref(p), C.byref(i), C.c_int(direction), _ptr(hin), _ptr(tin),
                                 _ptr(g), _ptr(h_out))
    if rc != 0:
        raise ValueError("oracle: shape outside the definition")
    return g, h_out


class InputGrads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("dx", "dz", "ddt", "dB", "dC")]


class ParamGrads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("dconv_w", "dconv_b", "dA", "dD", "ddt_bias")]


def bimamba_bwd(cfg, params_f, params_b, in_f, in_b=None, dout=None, sel=None):
    """Gradients of bimamba_fwd given dout (shaped like its output).  Returns (din_f, din_b, dparams_f, dparams_b):
    din_*: dict of float64 arrays dx, dz [batch, L, n_sel], ddt [batch, L, n_heads], dB, dC [batch, L, groups, d_state];
    din_b is None when in_b is None (both directions read in_f, whose gradients then hold the sum of both).
    dparams_*: dict of float64 arrays shaped like the parameters (dconv_b / ddt_bias are returned even where the
    parameter itself was None, i.e. zero)."""
    d = _desc(cfg)
    pf, k1 = _params(params_f)
    pb, k2 = _params(params_b)
    i_f, k3 = _inputs(in_f)
    i_b, k4 = _inputs(in_f if in_b is None else in_b)
    sp, ns, k5 = _sel(sel)
    Bt, L, Dn, N, H, G, K = (cfg[k] for k in ("batch", "seqlen", "d_inner", "d_state", "n_heads", "n_groups", "d_conv"))
    n_sel = ns if sel is not None else Dn
    conv_ch = Dn + (2 * G * N if cfg.get("conv_bc", 0) else 0)
    do = _f64(dout)
    assert do.size == Bt * L * n_sel * (2 if cfg.get("combine", 0) else 1)

    def input_grads():
        g = dict(dx=np.zeros((Bt, L, n_sel)), dz=np.zeros((Bt, L, n_sel)), ddt=np.zeros((Bt, L, H)),
                 dB=np.zeros((Bt, L, G, N)), dC=np.zeros((Bt, L, G, N)))
        return g, InputGrads(*[_ptr(g[k]) for k in ("dx", "dz", "ddt", "dB", "dC")])

    def param_grads():
        g = dict(dconv_w=np.zeros((conv_ch, K)), dconv_b=np.zeros(conv_ch),
                 dA=np.zeros((H, N) if cfg.get("a_kind", 0) == 0 else (H,)),
                 dD=np.zeros(Dn if cfg.get("d_kind", 0) == 0 else H), ddt_bias=np.zeros(H))
        return g, ParamGrads(*[_ptr(g[k]) for k in ("dconv_w", "dconv_b", "dA", "dD", "ddt_bias")])

    gf, cgf = input_grads()
    gb, cgb = (gf, cgf) if in_b is None else input_grads()
    qf, cqf = param_grads()
    qb, cqb = param_grads()
    fn = lib().orc_bimamba_bwd
    fn.restype = C.c_int
    rc = fn(C.byref(d), C.byref(pf), C.byref(pb), C.byref(i_f), C.byref(i_b), sp, C.c_int(ns), _ptr(do),
            C.byref(cgf), C.byref(cgb), C.byref(cqf), C.byref(cqb))
    if rc != 0:
        raise ValueError("oracle: shape outside the definition")
    return gf, (None if in_b is None else gb), qf, qb
