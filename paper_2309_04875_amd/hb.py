"""ctypes binding of the C ABI in include/hb.h -- argument marshalling only.

Every function has the name and meaning of its C counterpart; tensors are torch int64 CUDA tensors
whose `data_ptr()` is handed through, and the stream is torch's current stream unless one is given.
There is no fallback: if libhb.so has not been built, loading raises.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIBRARY = os.path.join(HERE, "libhb.so")

HB_OK, HB_EINVAL, HB_EALIGN, HB_EHIP, HB_ENOTSUP, HB_ETOOBIG = 0, -1, -2, -3, -4, -5
HB_PARTY_STATIC_BYTES = 64 << 20
HB_DEALER_PER_GATE, HB_DEALER_SHARED_MASK = 0, 1
BASELINE_BITS_PER_ELEMENT = 29 * 64   # unpacked 64-bit ring, Sec. 2.3 accounting

EXPORTS = ("hb_drelu", "hb_relu", "hb_sign_shares", "hb_open", "hb_relu_batch", "hb_drelu_batch", "hb_eco_scan", "hb_eco_choose",
           "hb_share_f32", "hb_reveal_f32", "hb_sim_relu_f32", "hb_relu_party", "hb_relu_party_ex", "hb_party_workspace_bytes_ex", "hb_party_wire_words_ex", "hb_party_wire_offset_ex", "hb_relu_party_static", "hb_party_workspace_bytes", "hb_party_wire_words", "hb_party_wire_offset",
           "hb_drelu_ex", "hb_relu_ex", "hb_relu_batch_ex", "hb_drelu_batch_ex", "hb_plan_create", "hb_plan_run", "hb_plan_destroy",
           "hb_drelu_mp", "hb_relu_mp", "hb_opened_bits_mp",
           "hb_tensor_seed",
           "hb_opened_bits", "hb_opened_bits_ex", "hb_strerror", "hb_last_hip_error")

_lib = None


class hb_tensor(ctypes.Structure):
    """Mirror of `struct hb_tensor` in include/hb.h."""
    _fields_ = [("share0", ctypes.c_void_p), ("share1", ctypes.c_void_p), ("out0", ctypes.c_void_p),
                ("out1", ctypes.c_void_p), ("n", ctypes.c_size_t), ("k", ctypes.c_int), ("m", ctypes.c_int),
                ("seed", ctypes.c_uint64)]


class HbError(RuntimeError):
    def __init__(self, status, text):
        super().__init__("hb status %d: %s" % (status, text))
        self.status = status


def load():
    """Load libhb.so (once) and declare the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIBRARY):
        raise ImportError("%s is missing: build it with `python -m paper_2309_04875_amd.build` "
                          "(there is no CPU fallback)" % LIBRARY)
    lib = ctypes.CDLL(LIBRARY)
    vp, u64, sz, ci = ctypes.c_void_p, ctypes.c_uint64, ctypes.c_size_t, ctypes.c_int
    u64p = ctypes.POINTER(ctypes.c_uint64)
    for name in ("hb_drelu", "hb_relu", "hb_sign_shares"):
        f = getattr(lib, name)
        f.restype = ci
        f.argtypes = [vp, vp, sz, ci, ci, u64, vp, vp, u64p, vp]
    for name in ("hb_relu_batch", "hb_drelu_batch"):
        f = getattr(lib, name)
        f.restype = ci
        f.argtypes = [ctypes.POINTER(hb_tensor), sz, u64p, vp]
    for name in ("hb_drelu_ex", "hb_relu_ex"):
        f = getattr(lib, name)
        f.restype = ci
        f.argtypes = [vp, vp, sz, ci, ci, u64, ci, vp, vp, u64p, vp]
    for name in ("hb_relu_batch_ex", "hb_drelu_batch_ex"):
        f = getattr(lib, name)
        f.restype = ci
        f.argtypes = [ctypes.POINTER(hb_tensor), sz, ci, u64p, vp]
    lib.hb_plan_create.restype = ci
    lib.hb_plan_create.argtypes = [ctypes.POINTER(hb_tensor), sz, ci, ci, ctypes.POINTER(vp)]
    lib.hb_plan_run.restype = ci
    lib.hb_plan_run.argtypes = [vp, u64p, vp]
    lib.hb_plan_destroy.restype = None
    lib.hb_plan_destroy.argtypes = [vp]
    lib.hb_opened_bits_ex.restype = u64
    lib.hb_opened_bits_ex.argtypes = [ci, ci, ci, sz, ci]
    for name in ("hb_drelu_mp", "hb_relu_mp"):
        f = getattr(lib, name)
        f.restype = ci
        f.argtypes = [ctypes.POINTER(vp), ci, sz, ci, ci, u64, ctypes.POINTER(vp), u64p, vp]
    lib.hb_opened_bits_mp.restype = u64
    lib.hb_opened_bits_mp.argtypes = [ci, ci, ci, ci, sz]
    lib.hb_share_f32.restype = ci
    lib.hb_share_f32.argtypes = [vp, sz, u64, vp, vp, vp]
    lib.hb_reveal_f32.restype = ci
    lib.hb_reveal_f32.argtypes = [vp, vp, sz, vp, vp]
    lib.hb_sim_relu_f32.restype = ci
    lib.hb_sim_relu_f32.argtypes = [vp, sz, ci, ci, u64, u64, vp, vp]
    lib.hb_relu_party.restype = ci
    lib.hb_relu_party.argtypes = [vp, vp, sz, ci, ci, u64, vp, vp, vp, sz, u64p, vp]
    lib.hb_relu_party_ex.restype = ci
    lib.hb_relu_party_ex.argtypes = [vp, vp, sz, ci, ci, u64, ci, vp, vp, vp, sz, u64p, vp]
    lib.hb_party_workspace_bytes_ex.restype = sz
    lib.hb_party_workspace_bytes_ex.argtypes = [sz, ci, ci, ci]
    lib.hb_party_wire_words_ex.restype = sz
    lib.hb_party_wire_words_ex.argtypes = [sz, ci, ci, ci]
    lib.hb_party_wire_offset_ex.restype = sz
    lib.hb_party_wire_offset_ex.argtypes = [sz, ci, ci, ci, ci]
    lib.hb_relu_party_static.restype = ci
    lib.hb_relu_party_static.argtypes = [vp, vp, sz, ci, ci, u64, vp, vp, u64p, vp]
    lib.hb_party_workspace_bytes.restype = sz
    lib.hb_party_workspace_bytes.argtypes = [sz, ci, ci]
    lib.hb_party_wire_words.restype = sz
    lib.hb_party_wire_words.argtypes = [sz, ci, ci]
    lib.hb_party_wire_offset.restype = sz
    lib.hb_party_wire_offset.argtypes = [sz, ci, ci, ci]
    lib.hb_eco_scan.restype = ci
    lib.hb_eco_scan.argtypes = [vp, vp, sz, vp, vp]
    lib.hb_eco_choose.restype = ci
    lib.hb_eco_choose.argtypes = [u64p]
    lib.hb_open.restype = ci
    lib.hb_open.argtypes = [vp, vp, sz, ci, vp, vp]
    lib.hb_tensor_seed.restype = u64
    lib.hb_tensor_seed.argtypes = [u64, u64]
    lib.hb_opened_bits.restype = u64
    lib.hb_opened_bits.argtypes = [ci, ci, ci, sz]
    lib.hb_strerror.restype = ctypes.c_char_p
    lib.hb_strerror.argtypes = [ci]
    lib.hb_last_hip_error.restype = ctypes.c_char_p
    lib.hb_last_hip_error.argtypes = []
    _lib = lib
    return lib


def strerror(status):
    return load().hb_strerror(int(status)).decode()


def last_hip_error():
    return load().hb_last_hip_error().decode()


def _check(status):
    if status != HB_OK:
        text = strerror(status)
        if status == HB_EHIP:
            text += ": " + last_hip_error()
        raise HbError(status, text)


def _tensor_args(*tensors):
    import torch
    n = tensors[0].numel()
    for t in tensors:
        if not isinstance(t, torch.Tensor) or t.dtype != torch.int64 or not t.is_cuda or not t.is_contiguous():
            raise TypeError("expected contiguous int64 CUDA tensors")
        if t.numel() != n:
            raise ValueError("tensors differ in size")
    return n


def _stream_handle(stream):
    import torch
    if stream is None:
        # the raw handle of torch's current stream; several times cheaper than building a torch.cuda.Stream object
        raw_stream = getattr(torch._C, "_cuda_getCurrentRawStream", None)
        if raw_stream is not None:
            return ctypes.c_void_p(raw_stream(torch.cuda.current_device()))
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _shares_call(name, share0, share1, k, m, seed, out0, out1, stream, dealer=None):
    import torch
    if out0 is None:
        out0 = torch.empty_like(share0)
    if out1 is None:
        out1 = torch.empty_like(share1)
    n = _tensor_args(share0, share1, out0, out1)
    bits = ctypes.c_uint64(0)
    layout = () if dealer is None else (int(dealer),)
    st = getattr(load(), name)(share0.data_ptr(), share1.data_ptr(), n, int(k), int(m), int(seed) & (2**64 - 1),
                               *layout, out0.data_ptr(), out1.data_ptr(), ctypes.byref(bits), _stream_handle(stream))
    _check(st)
    return out0, out1, int(bits.value)


def hb_drelu(share0, share1, k, m, seed, out0=None, out1=None, stream=None):
    """Arithmetic shares of DReLU on the slice [k, m); returns (out0, out1, opened_bits)."""
    return _shares_call("hb_drelu", share0, share1, k, m, seed, out0, out1, stream)


def hb_relu(share0, share1, k, m, seed, out0=None, out1=None, stream=None):
    """Arithmetic shares of x * DReLU; returns (out0, out1, opened_bits)."""
    return _shares_call("hb_relu", share0, share1, k, m, seed, out0, out1, stream)


def hb_drelu_ex(share0, share1, k, m, seed, dealer, out0=None, out1=None, stream=None):
    """hb_drelu on the dealer layout `dealer` (HB_DEALER_PER_GATE or HB_DEALER_SHARED_MASK)."""
    return _shares_call("hb_drelu_ex", share0, share1, k, m, seed, out0, out1, stream, dealer)


def hb_relu_ex(share0, share1, k, m, seed, dealer, out0=None, out1=None, stream=None):
    """hb_relu on the dealer layout `dealer`."""
    return _shares_call("hb_relu_ex", share0, share1, k, m, seed, out0, out1, stream, dealer)


def hb_sign_shares(share0, share1, k, m, seed, out0=None, out1=None, stream=None):
    """XOR shares (0/1) of the sign bit after the adder circuit; returns (out0, out1, opened_bits)."""
    return _shares_call("hb_sign_shares", share0, share1, k, m, seed, out0, out1, stream)


def _mp_call(name, shares, k, m, seed, outs, stream):
    import torch
    shares = list(shares)
    if outs is None:
        outs = [torch.empty_like(s) for s in shares]
    outs = list(outs)
    if len(outs) != len(shares):
        raise ValueError("one output per party")
    n = _tensor_args(*shares, *outs) if shares else 0
    p = len(shares)
    tab_in = (ctypes.c_void_p * max(p, 1))(*[s.data_ptr() for s in shares])
    tab_out = (ctypes.c_void_p * max(p, 1))(*[o.data_ptr() for o in outs])
    bits = ctypes.c_uint64(0)
    _check(getattr(load(), name)(tab_in, p, n, int(k), int(m), int(seed) & (2**64 - 1), tab_out, ctypes.byref(bits),
                                 _stream_handle(stream)))
    return outs, int(bits.value)


def hb_drelu_mp(shares, k, m, seed, outs=None, stream=None):
    """DReLU among len(shares) parties; returns (list of output share tensors, opened bits per link)."""
    return _mp_call("hb_drelu_mp", shares, k, m, seed, outs, stream)


def hb_relu_mp(shares, k, m, seed, outs=None, stream=None):
    """Approximate ReLU among len(shares) parties; returns (list of output share tensors, opened bits per link)."""
    return _mp_call("hb_relu_mp", shares, k, m, seed, outs, stream)


def hb_opened_bits_mp(relu, parties, k, m, n):
    return int(load().hb_opened_bits_mp(int(bool(relu)), int(parties), int(k), int(m), int(n)))


def make_batch(items):
    """ctypes descriptor array for a batched call; items: (share0, share1, out0, out1, k, m, seed) with torch tensors."""
    arr = (hb_tensor * len(items))()
    for d, (s0, s1, o0, o1, k, m, seed) in zip(arr, items):
        d.n = _tensor_args(s0, s1, o0, o1)
        d.share0, d.share1, d.out0, d.out1 = s0.data_ptr(), s1.data_ptr(), o0.data_ptr(), o1.data_ptr()
        d.k, d.m, d.seed = int(k), int(m), int(seed) & (2**64 - 1)
    return arr


def _batch_call(name, batch, stream, dealer=None):
    if not isinstance(batch, ctypes.Array):
        batch = make_batch(batch)
    bits = ctypes.c_uint64(0)
    layout = () if dealer is None else (int(dealer),)
    _check(getattr(load(), name)(batch, len(batch), *layout, ctypes.byref(bits), _stream_handle(stream)))
    return int(bits.value)


def hb_relu_batch(batch, stream=None):
    """hb_relu over a set of tensors (list of (share0, share1, out0, out1, k, m, seed) or a make_batch array);
    returns the total opened bits."""
    return _batch_call("hb_relu_batch", batch, stream)


def hb_drelu_batch(batch, stream=None):
    return _batch_call("hb_drelu_batch", batch, stream)


def hb_relu_batch_ex(batch, dealer, stream=None):
    return _batch_call("hb_relu_batch_ex", batch, stream, dealer)


def hb_drelu_batch_ex(batch, dealer, stream=None):
    return _batch_call("hb_drelu_batch_ex", batch, stream, dealer)


class Plan:
    """Handle of hb_plan_create; keeps the tensors of the set alive.  run() enqueues the set's launches."""

    def __init__(self, batch, relu=True, dealer=HB_DEALER_PER_GATE):
        self._keep = batch
        arr = batch if isinstance(batch, ctypes.Array) else make_batch(batch)
        handle = ctypes.c_void_p(None)
        _check(load().hb_plan_create(arr, len(arr), int(bool(relu)), int(dealer), ctypes.byref(handle)))
        self._handle = handle
        self._bits = ctypes.c_uint64(0)
        self._run = load().hb_plan_run

    def run(self, stream=None):
        """Returns the opened bits of the set."""
        st = self._run(self._handle, ctypes.byref(self._bits), _stream_handle(stream))
        if st != HB_OK:
            _check(st)
        return self._bits.value

    def close(self):
        if self._handle is not None and self._handle.value:
            load().hb_plan_destroy(self._handle)
        self._handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def hb_plan_create(batch, relu=True, dealer=HB_DEALER_PER_GATE):
    """Validate a set once (list of (share0, share1, out0, out1, k, m, seed) or a make_batch array); returns a Plan."""
    return Plan(batch, relu, dealer)


def hb_plan_run(plan, stream=None):
    """Enqueue the plan's launches; returns the opened bits of the set."""
    return plan.run(stream)


def hb_plan_destroy(plan):
    plan.close()


def _float_arg(t):
    import torch
    if not isinstance(t, torch.Tensor) or t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
        raise TypeError("expected a contiguous float32 CUDA tensor")
    return t.numel()


def hb_share_f32(x, share_seed, share0=None, share1=None, stream=None):
    """Encode to 2^16 fixed point and share additively; returns (share0, share1)."""
    import torch
    n = _float_arg(x)
    if share0 is None:
        share0 = torch.empty(x.shape, dtype=torch.int64, device=x.device)
    if share1 is None:
        share1 = torch.empty(x.shape, dtype=torch.int64, device=x.device)
    if _tensor_args(share0, share1) != n:
        raise ValueError("tensors differ in size")
    _check(load().hb_share_f32(x.data_ptr(), n, int(share_seed) & (2**64 - 1), share0.data_ptr(), share1.data_ptr(),
                               _stream_handle(stream)))
    return share0, share1


def hb_reveal_f32(share0, share1, out=None, stream=None):
    """Open and decode to float32."""
    import torch
    n = _tensor_args(share0, share1)
    if out is None:
        out = torch.empty(share0.shape, dtype=torch.float32, device=share0.device)
    if _float_arg(out) != n:
        raise ValueError("tensors differ in size")
    _check(load().hb_reveal_f32(share0.data_ptr(), share1.data_ptr(), n, out.data_ptr(), _stream_handle(stream)))
    return out


def hb_sim_relu_f32(x, k, m, seed, share_seed, out=None, stream=None):
    """Approximate ReLU of plaintext floats through the protocol, one kernel."""
    import torch
    n = _float_arg(x)
    if out is None:
        out = torch.empty_like(x)
    if _float_arg(out) != n:
        raise ValueError("tensors differ in size")
    _check(load().hb_sim_relu_f32(x.data_ptr(), n, int(k), int(m), int(seed) & (2**64 - 1),
                                  int(share_seed) & (2**64 - 1), out.data_ptr(), _stream_handle(stream)))
    return out


def hb_party_workspace_bytes(n, k, m):
    return int(load().hb_party_workspace_bytes(int(n), int(k), int(m)))


def hb_party_wire_words(n, k, m):
    return int(load().hb_party_wire_words(int(n), int(k), int(m)))


def hb_party_wire_offset(n, k, m, party):
    return int(load().hb_party_wire_offset(int(n), int(k), int(m), int(party)))


def hb_party_workspace_bytes_ex(n, k, m, dealer):
    return int(load().hb_party_workspace_bytes_ex(int(n), int(k), int(m), int(dealer)))


def hb_party_wire_words_ex(n, k, m, dealer):
    return int(load().hb_party_wire_words_ex(int(n), int(k), int(m), int(dealer)))


def hb_party_wire_offset_ex(n, k, m, dealer, party):
    return int(load().hb_party_wire_offset_ex(int(n), int(k), int(m), int(dealer), int(party)))


def hb_relu_party_ex(share0, share1, k, m, seed, dealer, out0=None, out1=None, workspace=None, stream=None):
    """Party-faithful ReLU on a dealer layout; returns (out0, out1, wire0, wire1, wire_bytes) where wire_p is an
    int64 view of party p's wire inside the workspace (a uint8 CUDA tensor, allocated here unless one is passed)."""
    import torch
    if out0 is None:
        out0 = torch.empty_like(share0)
    if out1 is None:
        out1 = torch.empty_like(share1)
    n = _tensor_args(share0, share1, out0, out1)
    need = hb_party_workspace_bytes_ex(n, k, m, dealer)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=share0.device)
    if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous uint8 CUDA tensor")
    wire_bytes = ctypes.c_uint64(0)
    st = load().hb_relu_party_ex(share0.data_ptr(), share1.data_ptr(), n, int(k), int(m), int(seed) & (2**64 - 1),
                                 int(dealer), out0.data_ptr(), out1.data_ptr(), workspace.data_ptr(),
                                 workspace.numel(), ctypes.byref(wire_bytes), _stream_handle(stream))
    _check(st)
    words = hb_party_wire_words_ex(n, k, m, dealer)
    wires = []
    for p in (0, 1):
        off = hb_party_wire_offset_ex(n, k, m, dealer, p)
        wires.append(workspace[off:off + 8 * words].view(torch.int64))
    return out0, out1, wires[0], wires[1], int(wire_bytes.value)


def hb_relu_party(share0, share1, k, m, seed, out0=None, out1=None, workspace=None, stream=None):
    """Party-faithful ReLU on the standard dealer layout (through the C entry point hb_relu_party)."""
    import torch
    if out0 is None:
        out0 = torch.empty_like(share0)
    if out1 is None:
        out1 = torch.empty_like(share1)
    n = _tensor_args(share0, share1, out0, out1)
    need = hb_party_workspace_bytes(n, k, m)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=share0.device)
    if workspace.dtype != torch.uint8 or not workspace.is_cuda or not workspace.is_contiguous():
        raise TypeError("workspace must be a contiguous uint8 CUDA tensor")
    wire_bytes = ctypes.c_uint64(0)
    st = load().hb_relu_party(share0.data_ptr(), share1.data_ptr(), n, int(k), int(m), int(seed) & (2**64 - 1),
                              out0.data_ptr(), out1.data_ptr(), workspace.data_ptr(), workspace.numel(),
                              ctypes.byref(wire_bytes), _stream_handle(stream))
    _check(st)
    words = hb_party_wire_words(n, k, m)
    wires = []
    for p in (0, 1):
        off = hb_party_wire_offset(n, k, m, p)
        wires.append(workspace[off:off + 8 * words].view(torch.int64))
    return out0, out1, wires[0], wires[1], int(wire_bytes.value)


def hb_relu_party_static(share0, share1, k, m, seed, out0, out1, stream=None):
    """hb_relu_party on the library's static workspace; out0 / out1 are the caller's; returns the wire bytes per party."""
    n = _tensor_args(share0, share1, out0, out1)
    wire_bytes = ctypes.c_uint64(0)
    _check(load().hb_relu_party_static(share0.data_ptr(), share1.data_ptr(), n, int(k), int(m), int(seed) & (2**64 - 1),
                                       out0.data_ptr(), out1.data_ptr(), ctypes.byref(wire_bytes),
                                       _stream_handle(stream)))
    return int(wire_bytes.value)


def hb_eco_scan(share0, share1, counts=None, stream=None):
    """counts[m-1] = elements whose DReLU on [0, m) differs from the full ring; returns the 64-entry device tensor."""
    import torch
    if counts is None:
        counts = torch.empty(64, dtype=torch.int64, device=share0.device)
    n = _tensor_args(share0, share1)
    if counts.dtype != torch.int64 or counts.numel() != 64 or not counts.is_cuda or not counts.is_contiguous():
        raise TypeError("counts must be a contiguous int64 CUDA tensor of 64 entries")
    _check(load().hb_eco_scan(share0.data_ptr(), share1.data_ptr(), n, counts.data_ptr(), _stream_handle(stream)))
    return counts


def hb_eco_choose(counts):
    """Smallest m with no mismatch at any m' >= m; counts: 64 host integers (or a tensor, copied to the host)."""
    if hasattr(counts, "cpu"):
        counts = counts.cpu().tolist()
    arr = (ctypes.c_uint64 * 64)(*[int(c) & (2**64 - 1) for c in counts])
    m = load().hb_eco_choose(arr)
    _check(m if m < 0 else HB_OK)
    return m


def hb_open(share0, share1, binary=False, out=None, stream=None):
    """share0 + share1 (mod 2^64), or share0 ^ share1 when binary."""
    import torch
    if out is None:
        out = torch.empty_like(share0)
    n = _tensor_args(share0, share1, out)
    _check(load().hb_open(share0.data_ptr(), share1.data_ptr(), n, int(bool(binary)), out.data_ptr(),
                          _stream_handle(stream)))
    return out


def hb_tensor_seed(root_seed, tensor_id):
    return int(load().hb_tensor_seed(int(root_seed) & (2**64 - 1), int(tensor_id)))


def hb_opened_bits(relu, k, m, n):
    return int(load().hb_opened_bits(int(bool(relu)), int(k), int(m), int(n)))


def hb_opened_bits_ex(relu, k, m, n, dealer):
    return int(load().hb_opened_bits_ex(int(bool(relu)), int(k), int(m), int(n), int(dealer)))


def raw(name, *args):
    """Call an entry point with raw integers / pointers (tests of the error paths); returns its status."""
    return getattr(load(), name)(*args)
