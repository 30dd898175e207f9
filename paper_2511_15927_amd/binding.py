"""ctypes binding of the C ABI in include/bimamba.h: argument marshalling only.

Tensors are torch tensors on the GPU (torch owns device memory and streams); every step of the path runs in the
HIP library.  There is no fallback: if libbimamba.so has not been built, loading raises.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libbimamba.so")

F32, BF16 = 0, 1
A_PER_HEAD_STATE, A_SCALAR_PER_HEAD = 0, 1
D_PER_CHANNEL, D_PER_HEAD = 0, 1
COMBINE_ADD, COMBINE_SEPARATE = 0, 1

STATUS = {0: "BIMAMBA_OK", -1: "BIMAMBA_ERR_NULL_POINTER", -2: "BIMAMBA_ERR_BAD_SHAPE", -3: "BIMAMBA_ERR_UNSUPPORTED",
          -4: "BIMAMBA_ERR_MISALIGNED", -5: "BIMAMBA_ERR_WORKSPACE_TOO_SMALL", -6: "BIMAMBA_ERR_HIP",
          -7: "BIMAMBA_ERR_SCRATCH_EXCEEDED", -8: "BIMAMBA_ERR_ALIAS"}
STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = ("bimamba_fwd", "bimamba_block_fwd", "bimamba_block_fwd_static", "bimamba_bwd", "bimamba_workspace_bytes",
           "bimamba_bwd_workspace_bytes", "bimamba_time_chunks", "bimamba_profile_next_call", "bimamba_status_string",
           "bimamba_version")


class Desc(C.Structure):
    _fields_ = [("struct_size", C.c_uint32)] + [(n, C.c_int32) for n in (
        "batch", "seqlen", "d_inner", "d_state", "n_heads", "n_groups", "d_conv", "io_dtype", "a_kind", "d_kind",
        "dt_softplus", "conv_bc", "combine", "time_chunks", "state_split")]


class Params(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("conv_w", "conv_b", "A", "D", "dt_bias")]


class Tensor(C.Structure):
    _fields_ = [("ptr", C.c_void_p), ("stride_batch", C.c_int64), ("stride_token", C.c_int64)]


class Inputs(C.Structure):
    _fields_ = [(n, Tensor) for n in ("x", "z", "dt", "B", "C")]


class InputGrads(C.Structure):
    _fields_ = [("dx", Tensor), ("dz", Tensor), ("ddt", Tensor), ("dB", C.c_void_p), ("dC", C.c_void_p)]


class ParamGrads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("dconv_w", "dconv_b", "dA", "dD", "ddt_bias")]


class BimambaError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = lib().bimamba_status_string(status).decode()
        super().__init__("%s failed: %s (%s)" % (where, STATUS.get(status, status), msg))


_lib = None


def lib():
    """Load libbimamba.so (built by paper_2511_15927_amd/build.py); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libbimamba.so is not built: run `python -m paper_2511_15927_amd.build` "
                               "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        L.bimamba_fwd.restype = C.c_int
        L.bimamba_fwd.argtypes = [C.POINTER(Desc), C.POINTER(Params), C.POINTER(Params), C.POINTER(Inputs),
                                  C.POINTER(Inputs), C.POINTER(Tensor), C.c_void_p, C.c_size_t, C.c_void_p]
        L.bimamba_block_fwd.restype = C.c_int
        L.bimamba_block_fwd.argtypes = [C.POINTER(Desc), C.POINTER(Params), C.POINTER(Params), C.POINTER(Inputs),
                                        C.POINTER(Inputs), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.POINTER(Tensor), C.c_void_p, C.c_size_t, C.c_void_p]
        L.bimamba_block_fwd_static.restype = C.c_int
        L.bimamba_block_fwd_static.argtypes = [C.POINTER(Desc), C.POINTER(Params), C.POINTER(Params), C.POINTER(Inputs),
                                               C.POINTER(Inputs), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                               C.POINTER(Tensor), C.c_void_p]
        L.bimamba_bwd.restype = C.c_int
        L.bimamba_bwd.argtypes = [C.POINTER(Desc), C.POINTER(Params), C.POINTER(Params), C.POINTER(Inputs),
                                  C.POINTER(Inputs), C.POINTER(Tensor), C.POINTER(InputGrads), C.POINTER(InputGrads),
                                  C.POINTER(ParamGrads), C.POINTER(ParamGrads), C.c_void_p, C.c_size_t, C.c_void_p]
        L.bimamba_bwd_workspace_bytes.restype = C.c_size_t
        L.bimamba_bwd_workspace_bytes.argtypes = [C.POINTER(Desc)]
        L.bimamba_workspace_bytes.restype = C.c_size_t
        L.bimamba_workspace_bytes.argtypes = [C.POINTER(Desc), C.c_int]
        L.bimamba_time_chunks.restype = C.c_int
        L.bimamba_time_chunks.argtypes = [C.POINTER(Desc)]
        L.bimamba_status_string.restype = C.c_char_p
        L.bimamba_status_string.argtypes = [C.c_int]
        L.bimamba_version.restype = C.c_int
        L.bimamba_profile_next_call.restype = None
        L.bimamba_profile_next_call.argtypes = [C.c_void_p, C.c_void_p]
        _lib = L
    return _lib


def make_desc(cfg, seqlen=None, **override):
    """C descriptor from a config dict (keys as in synth.mixer_cfg)."""
    c = dict(cfg)
    c.update(override)
    return Desc(C.sizeof(Desc), c["batch"], c["seqlen"] if seqlen is None else seqlen, c["d_inner"], c["d_state"],
                c["n_heads"], c["n_groups"], c["d_conv"], BF16 if c["io"] == "bf16" else F32, c["a_kind"], c["d_kind"],
                c["dt_softplus"], c["conv_bc"], c["combine"], c.get("time_chunks", 0), c.get("state_split", 0))


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def make_params(p):
    """p: dict of float32 device tensors conv_w, conv_b, A, D, dt_bias (conv_b / dt_bias may be None)."""
    for k in ("conv_w", "conv_b", "A", "D", "dt_bias"):
        t = p.get(k)
        if t is not None:
            assert t.dtype == torch.float32 and t.is_contiguous(), k
    return Params(_ptr(p["conv_w"]), _ptr(p.get("conv_b")), _ptr(p["A"]), _ptr(p["D"]), _ptr(p.get("dt_bias")))


def make_tensor(t):
    """[batch, L, channels] view with unit channel stride (batch/token strides are passed through)."""
    assert t.dim() == 3 and (t.numel() == 0 or t.shape[2] == 1 or t.stride(2) == 1), "channel dimension must be contiguous"
    return Tensor(t.data_ptr(), t.stride(0), t.stride(1))


def make_inputs(i):
    """i: dict of device tensors x, z [Bt,L,Dn]; dt [Bt,L,H]; B, C [Bt,L,G,N] or [Bt,L,G*N]."""
    def three(t):
        if t.dim() == 3:
            return t
        assert t.dim() == 4 and (t.shape[2] == 1 or t.stride(2) == t.shape[3] * t.stride(3)), "B/C groups must be adjacent"
        return t.as_strided((t.shape[0], t.shape[1], t.shape[2] * t.shape[3]), (t.stride(0), t.stride(1), t.stride(3)))
    return Inputs(*[make_tensor(three(i[k])) for k in ("x", "z", "dt", "B", "C")])


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def bimamba_workspace_bytes(desc, block_variant=0):
    return int(lib().bimamba_workspace_bytes(C.byref(desc), int(block_variant)))


def bimamba_time_chunks(desc):
    return int(lib().bimamba_time_chunks(C.byref(desc)))


def bimamba_version():
    return int(lib().bimamba_version())


def bimamba_profile_next_call(ev_start, ev_stop):
    """ev_start/ev_stop: torch.cuda.Event(enable_timing=True) that have been recorded once (so the HIP event
    exists), or None to disarm."""
    h0 = None if ev_start is None else C.c_void_p(ev_start.cuda_event)
    h1 = None if ev_stop is None else C.c_void_p(ev_stop.cuda_event)
    lib().bimamba_profile_next_call(h0, h1)


def bimamba_fwd(desc, pf, pb, in_f, in_b, out, workspace, stream=None, check=True):
    """Enqueue the full-sequence path.  pf/pb: Params; in_f/in_b: Inputs (in_b None = shared); out: Tensor struct;
    workspace: uint8 device tensor or None.  Returns the status code (raises on error when check)."""
    ws_ptr = None if workspace is None else C.c_void_p(workspace.data_ptr())
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().bimamba_fwd(C.byref(desc), C.byref(pf), C.byref(pb), C.byref(in_f),
                           None if in_b is None else C.byref(in_b), C.byref(out), ws_ptr, ws_bytes, _stream_ptr(stream))
    if check and rc != 0:
        raise BimambaError(rc, "bimamba_fwd")
    return rc


def make_input_grads(g):
    """g: dict of device tensors dx, dz [Bt,L,Dn], ddt [Bt,L,H] (io dtype, unit channel stride) and dB, dC
    [Bt,L,G,N] float32 contiguous."""
    for k in ("dB", "dC"):
        assert g[k].dtype == torch.float32 and g[k].is_contiguous(), k
    return InputGrads(make_tensor(g["dx"]), make_tensor(g["dz"]), make_tensor(g["ddt"]), g["dB"].data_ptr(), g["dC"].data_ptr())


def make_param_grads(g):
    """g: dict of float32 contiguous device tensors dconv_w, dA, dD and optionally dconv_b, ddt_bias."""
    for k in ("dconv_w", "dconv_b", "dA", "dD", "ddt_bias"):
        t = g.get(k)
        if t is not None:
            assert t.dtype == torch.float32 and t.is_contiguous(), k
    return ParamGrads(_ptr(g["dconv_w"]), _ptr(g.get("dconv_b")), _ptr(g["dA"]), _ptr(g["dD"]), _ptr(g.get("ddt_bias")))


def bimamba_bwd_workspace_bytes(desc):
    return int(lib().bimamba_bwd_workspace_bytes(C.byref(desc)))


def bimamba_bwd(desc, pf, pb, in_f, in_b, dout, din_f, din_b, dpf, dpb, workspace, stream=None, check=True):
    """Enqueue the gradients of bimamba_fwd.  dout: Tensor; din_f/din_b: InputGrads (din_b None with shared
    activations); dpf/dpb: ParamGrads; workspace: uint8 device tensor of bimamba_bwd_workspace_bytes(desc)."""
    ws_ptr = None if workspace is None else C.c_void_p(workspace.data_ptr())
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().bimamba_bwd(C.byref(desc), C.byref(pf), C.byref(pb), C.byref(in_f), None if in_b is None else C.byref(in_b),
                           C.byref(dout), C.byref(din_f), None if din_b is None else C.byref(din_b), C.byref(dpf),
                           C.byref(dpb), ws_ptr, ws_bytes, _stream_ptr(stream))
    if check and rc != 0:
        raise BimambaError(rc, "bimamba_bwd")
    return rc


def bimamba_block_fwd(desc, pf, pb, in_f, in_b, h_in, tail_in, h_out, tail_out, out, workspace, stream=None, check=True):
    """Enqueue the block variant.  h_in/h_out: float32 device tensors or None; tail_in/tail_out: io-dtype device
    tensors or None."""
    ws_ptr = None if workspace is None else C.c_void_p(workspace.data_ptr())
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().bimamba_block_fwd(C.byref(desc), C.byref(pf), C.byref(pb), C.byref(in_f),
                                 None if in_b is None else C.byref(in_b), _ptr(h_in), _ptr(tail_in), _ptr(h_out),
                                 _ptr(tail_out), C.byref(out), ws_ptr, ws_bytes, _stream_ptr(stream))
    if check and rc != 0:
        raise BimambaError(rc, "bimamba_block_fwd")
    return rc


def bimamba_block_fwd_static(desc, pf, pb, in_f, in_b, h_in, tail_in, h_out, tail_out, out, stream=None, check=True):
    """bimamba_block_fwd on the library's own fixed scratch buffer: no workspace argument, nothing allocated."""
    rc = lib().bimamba_block_fwd_static(C.byref(desc), C.byref(pf), C.byref(pb), C.byref(in_f),
                                        None if in_b is None else C.byref(in_b), _ptr(h_in), _ptr(tail_in), _ptr(h_out),
                                        _ptr(tail_out), C.byref(out), _stream_ptr(stream))
    if check and rc != 0:
        raise BimambaError(rc, "bimamba_block_fwd_static")
    return rc


# ---- conveniences used by tests and the benchmark (allocation through torch, no arithmetic) ----

def io_dtype(cfg):
    return torch.bfloat16 if cfg["io"] == "bf16" else torch.float32


def to_device(tensors, cfg=None, device="cuda"):
    """Upload a dict of CPU float32 tensors; activations are cast to the config's I/O dtype (exact: values were
    rounded to it by the generator), parameters stay float32."""
    out = {}
    for k, v in tensors.items():
        if v is None:
            out[k] = None
        elif cfg is not None and k in ("x", "z", "dt", "B", "C"):
            out[k] = v.to(device=device, dtype=io_dtype(cfg)).contiguous()
        else:
            out[k] = v.to(device=device, dtype=torch.float32).contiguous()
    return out


def alloc_out(cfg, device="cuda", seqlen=None):
    L = cfg["seqlen"] if seqlen is None else seqlen
    width = cfg["d_inner"] * (2 if cfg["combine"] == COMBINE_SEPARATE else 1)
    return torch.empty(cfg["batch"], L, width, dtype=io_dtype(cfg), device=device)


def alloc_workspace(desc, block_variant=0, device="cuda"):
    n = bimamba_workspace_bytes(desc, block_variant)
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)
