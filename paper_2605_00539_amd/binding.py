"""ctypes binding of libagoq.so.  Argument marshalling only."""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libagoq.so")      # the in-tree build, the only one ever loaded
_lib = None

_I64 = ctypes.c_int64
_INT = ctypes.c_int
_P = ctypes.c_void_p
_SLOTS = 5
MAX_LAYER_SLOTS = 8


class ActSlot(ctypes.Structure):
    """agoq_act_slot: one stored tensor of a layer call (device pointers)."""
    _fields_ = [("bf16", _P), ("codes", _P), ("scales", _P), ("numel", _I64), ("bits", _INT)]


class AgoqError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("agoq status %d: %s" % (status, message))
        self.status = status


def library_path():
    return _LIB_PATH


def load_library():
    """Load libagoq.so (built by paper_2605_00539_amd/build.py).  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            "libagoq.so is not built: run `python -m paper_2605_00539_amd.build` "
            "(or __graft_entry__.build()) first; there is no fallback path")
    # torch ships its own HIP runtime; importing it first makes this library bind to the
    # same runtime, so that torch's device pointers and streams are valid here
    import torch  # noqa: F401
    L = ctypes.CDLL(_LIB_PATH)
    L.agoq_act_quant.argtypes = [_P, _I64, _INT, _INT, _P, _P, _P]
    L.agoq_act_dequant.argtypes = [_P, _P, _I64, _INT, _INT, _P, _P]
    L.agoq_act_quant_layer.argtypes = [ctypes.POINTER(ActSlot), _INT, _INT, _P]
    L.agoq_act_dequant_layer.argtypes = [ctypes.POINTER(ActSlot), _INT, _INT, _P]
    L.agoq_grad_quant.argtypes = [_P, _I64, _INT, _P, _P, _P]
    L.agoq_grad_reduce_requant.argtypes = [_P, _I64, _P, _I64, _INT, _I64, _INT, _P, _P, _P]
    L.agoq_act_dequant_rmsnorm.argtypes = [_P, _P, _I64, _I64, _INT, _INT, _P, ctypes.c_float, _P, _P, _P]
    L.agoq_act_dequant_silu_mul.argtypes = [_P, _P, _INT, _P, _P, _INT, _I64, _INT, _P, _P]
    L.agoq_rmsnorm_fwd_quant.argtypes = [_P, _I64, _I64, _P, ctypes.c_float, _INT, _INT, _P, _P, _P, _P, _P]
    L.agoq_silu_mul_fwd_quant.argtypes = [_P, _P, _I64, _INT, _INT, _INT, _P, _P, _P, _P, _P, _P]
    L.agoq_grad_accumulate.argtypes = [_P, _P, _P, _INT, _I64, _INT, _P, _P, _P]
    L.agoq_grad_dequant.argtypes = [_P, _P, _I64, _INT, _P, _P]
    L.agoq_fp4_act_dequant_rmsnorm.argtypes = [_P, _P, _I64, _I64, _INT, _P, ctypes.c_float, _P, _P, _P]
    L.agoq_fp4_act_dequant_silu_mul.argtypes = [_P, _P, _P, _P, _I64, _INT, _P, _P]
    L.agoq_fp4_rmsnorm_fwd_quant.argtypes = [_P, _I64, _I64, _P, ctypes.c_float, _INT, _P, _P, _P, _P, _P]
    L.agoq_fp4_silu_mul_fwd_quant.argtypes = [_P, _P, _I64, _INT, _P, _P, _P, _P, _P, _P]
    L.agoq_fp4_act_quant.argtypes = [_P, _I64, _INT, _P, _P, _P]
    L.agoq_fp4_act_dequant.argtypes = [_P, _P, _I64, _INT, _P, _P]
    L.agoq_fp8_grad_quant.argtypes = [_P, _I64, _INT, _P, _P, _P]
    L.agoq_fp8_grad_dequant.argtypes = [_P, _P, _I64, _INT, _P, _P]
    L.agoq_fp8_grad_reduce_requant.argtypes = [_P, _I64, _P, _I64, _INT, _I64, _INT, _P, _P, _P]
    L.agoq_fp8_grad_accumulate.argtypes = [_P, _P, _P, _INT, _I64, _INT, _P, _P, _P]
    L.agoq_probe_stream.argtypes = [_P, _INT, _P, _INT, _I64, _P]
    _U32 = ctypes.c_uint32
    L.agoq_act_quant_sr.argtypes = [_P, _I64, _INT, _INT, _U32, _P, _P, _P]
    L.agoq_grad_quant_sr.argtypes = [_P, _I64, _INT, _U32, _P, _P, _P]
    L.agoq_grad_reduce_requant_sr.argtypes = [_P, _I64, _P, _I64, _INT, _I64, _INT, _U32, _P, _P, _P]
    L.agoq_grad_accumulate_sr.argtypes = [_P, _P, _P, _INT, _I64, _INT, _U32, _P, _P, _P]
    L.agoq_codes_bytes.argtypes = [_I64, _INT]
    L.agoq_codes_bytes.restype = _I64
    L.agoq_num_groups.argtypes = [_I64, _INT]
    L.agoq_num_groups.restype = _I64
    L.agoq_dbca_stored_microbatches.argtypes = [_INT, _INT]
    L.agoq_dbca_bits.argtypes = [_INT, _INT, ctypes.POINTER(_INT)]
    L.agoq_layer_bitmap.argtypes = [_INT, ctypes.POINTER(_INT * _SLOTS)]
    L.agoq_layer_bitmap_native.argtypes = [_INT, ctypes.POINTER(_INT * _SLOTS)]
    L.agoq_layer_stored_bytes.argtypes = [_I64, _I64, _I64, _INT, ctypes.POINTER(_INT * _SLOTS), _INT]
    L.agoq_layer_stored_bytes.restype = _I64
    L.agoq_strerror.argtypes = [_INT]
    L.agoq_strerror.restype = ctypes.c_char_p
    L.agoq_version.argtypes = []
    _lib = L
    return L


def strerror(status):
    return load_library().agoq_strerror(int(status)).decode()


def version():
    return load_library().agoq_version()


def _check(status):
    if status != 0:
        raise AgoqError(status, strerror(status))


def _dev(t, dtype, name):
    import torch
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError("%s must be a tensor on the GPU" % name)
    if t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    return t


def _holds(t, count, name):
    """The kernels take plain pointers and trust the sizes they are given: a buffer too small
    for the call is refused here, where its size is still known."""
    if t.numel() < count:
        raise ValueError("%s holds %d elements, this call needs %d" % (name, t.numel(), count))


def _code_bytes(n, bits):
    return n * bits // 8 if bits in (4, 5, 6, 8) else 0


def _groups(n, group):
    return n // group if group > 0 else 0


def _stream(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


class _on_device:
    """Make the tensor's device current for the call; free when it already is."""

    def __init__(self, device):
        import torch
        self.guard = None if device.index == torch.cuda.current_device() else torch.cuda.device(device)

    def __enter__(self):
        if self.guard is not None:
            self.guard.__enter__()

    def __exit__(self, *exc):
        if self.guard is not None:
            self.guard.__exit__(*exc)


def _raw(ptr):
    return ctypes.c_void_p(ptr)


# ---- device entry points ------------------------------------------------------

def act_quant(x, group, bits, codes=None, scales=None, stream=None, sr_seed=None):
    """x: bf16 tensor on the GPU.  Returns (codes uint8 [numel*bits/8], scales float32 [numel/group]).
    sr_seed: an integer selects the stochastic-rounding variant (agoq_act_quant_sr) under that seed."""
    import torch
    L = load_library()
    x = _dev(x, torch.bfloat16, "x")
    n = x.numel()
    if codes is None:
        codes = torch.empty(max(n * bits // 8, 1), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty(max(n // max(group, 1), 1), dtype=torch.float32, device=x.device)
    _dev(codes, torch.uint8, "codes")
    _dev(scales, torch.float32, "scales")
    _holds(codes, _code_bytes(n, bits), "codes")
    _holds(scales, _groups(n, group), "scales")
    with _on_device(x.device):
        if sr_seed is None:
            _check(L.agoq_act_quant(_raw(x.data_ptr()), n, group, bits, _raw(codes.data_ptr()),
                                    _raw(scales.data_ptr()), _stream(stream)))
        else:
            _check(L.agoq_act_quant_sr(_raw(x.data_ptr()), n, group, bits, int(sr_seed) & 0xFFFFFFFF,
                                       _raw(codes.data_ptr()), _raw(scales.data_ptr()), _stream(stream)))
    return codes, scales


def act_dequant(codes, scales, numel, group, bits, out=None, stream=None):
    """Returns a flat bf16 tensor of numel elements."""
    import torch
    L = load_library()
    _dev(codes, torch.uint8, "codes")
    _dev(scales, torch.float32, "scales")
    if out is None:
        out = torch.empty(numel, dtype=torch.bfloat16, device=codes.device)
    _dev(out, torch.bfloat16, "out")
    _holds(codes, _code_bytes(numel, bits), "codes")
    _holds(scales, _groups(numel, group), "scales")
    _holds(out, numel, "out")
    with _on_device(codes.device):
        _check(L.agoq_act_dequant(_raw(codes.data_ptr()), _raw(scales.data_ptr()), numel, group,
                                  bits, _raw(out.data_ptr()), _stream(stream)))
    return out


class LayerSlots:
    """Descriptor array of a layer call (host memory, raw device pointers) together with the
    tensors those pointers belong to, which it keeps alive for as long as it lives."""

    def __init__(self, array, count, group, device, tensors):
        self.array, self.count, self.group, self.device = array, count, group, device
        self._tensors = tensors

    def __iter__(self):                     # (array, count) = slots
        return iter((self.array, self.count))


def layer_slots(xs, bits_list, codes_list, scales_list, group):
    """Descriptor array for a layer call from lists of device tensors: xs bf16, codes_list uint8,
    scales_list float32, bits_list ints.  Every buffer's size is checked against what a call
    with this `group` reads or writes.  Reusable across calls; holds references to the tensors."""
    import torch
    count = len(xs)
    if not (len(bits_list) == len(codes_list) == len(scales_list) == count):
        raise ValueError("layer call: the four lists must have one entry per tensor")
    arr = (ActSlot * max(count, 1))()
    for i, (x, b, c, s) in enumerate(zip(xs, bits_list, codes_list, scales_list)):
        _dev(x, torch.bfloat16, "bf16[%d]" % i)
        _dev(c, torch.uint8, "codes[%d]" % i)
        _dev(s, torch.float32, "scales[%d]" % i)
        if c.device != x.device or s.device != x.device or x.device != xs[0].device:
            raise ValueError("layer call: all tensors must be on one device")
        _holds(c, _code_bytes(x.numel(), int(b)), "codes[%d]" % i)
        _holds(s, _groups(x.numel(), group), "scales[%d]" % i)
        arr[i] = ActSlot(x.data_ptr(), c.data_ptr(), s.data_ptr(), x.numel(), int(b))
    device = xs[0].device if count else None
    return LayerSlots(arr, count, group, device, (list(xs), list(codes_list), list(scales_list)))


def _slots_for(slots, group):
    if not isinstance(slots, LayerSlots):
        raise TypeError("slots must come from layer_slots()")
    if slots.group != group:
        raise ValueError("slots were made for group %d, this call uses %d" % (slots.group, group))
    return slots


def act_quant_layer(xs, group, bits_list, codes_list=None, scales_list=None, slots=None, stream=None):
    """Quantize all stored tensors of a layer in one launch.  xs: list of bf16 tensors;
    bits_list: the bit map.  Returns (codes_list, scales_list).  `slots` = a descriptor array
    from layer_slots() to skip the marshalling on repeated calls."""
    import torch
    L = load_library()
    if slots is None:
        if codes_list is None:
            codes_list = [torch.empty(max(x.numel() * b // 8, 1), dtype=torch.uint8, device=x.device)
                          for x, b in zip(xs, bits_list)]
        if scales_list is None:
            scales_list = [torch.empty(max(x.numel() // max(group, 1), 1), dtype=torch.float32,
                                       device=x.device) for x in xs]
        slots = layer_slots(xs, bits_list, codes_list, scales_list, group)
    slots = _slots_for(slots, group)
    with _on_device(slots.device):
        _check(L.agoq_act_quant_layer(slots.array, slots.count, group, _stream(stream)))
    return codes_list, scales_list


def act_dequant_layer(codes_list, scales_list, numels, group, bits_list, outs=None, slots=None,
                      stream=None):
    """Dequantize all stored tensors of a layer in one launch.  Returns the list of flat bf16
    outputs."""
    import torch
    L = load_library()
    if slots is None:
        if outs is None:
            outs = [torch.empty(n, dtype=torch.bfloat16, device=c.device)
                    for n, c in zip(numels, codes_list)]
        for n, o in zip(numels, outs):
            if o.numel() != n:
                raise ValueError("layer call: output size differs from numel")
        slots = layer_slots(outs, bits_list, codes_list, scales_list, group)
    slots = _slots_for(slots, group)
    with _on_device(slots.device):
        _check(L.agoq_act_dequant_layer(slots.array, slots.count, group, _stream(stream)))
    return outs


def act_dequant_rmsnorm(codes, scales, rows, cols, group, bits, gamma, eps, out=None, r_out=None,
                        stream=None, fp4=False):
    """Stored RMSNorm input -> (y bf16 [rows, cols] = gamma * x' / r, r float32 [rows]).
    fp4=True: the codes are E2M1 (bits must be 4)."""
    import torch
    L = load_library()
    _dev(codes, torch.uint8, "codes")
    _dev(scales, torch.float32, "scales")
    _dev(gamma, torch.float32, "gamma")
    if gamma.numel() != cols:
        raise ValueError("gamma must have cols elements")
    if out is None:
        out = torch.empty((rows, cols), dtype=torch.bfloat16, device=codes.device)
    if r_out is None:
        r_out = torch.empty(rows, dtype=torch.float32, device=codes.device)
    _dev(out, torch.bfloat16, "out")
    _dev(r_out, torch.float32, "r_out")
    _holds(codes, _code_bytes(rows * cols, bits), "codes")
    _holds(scales, _groups(rows * cols, group), "scales")
    _holds(out, rows * cols, "out")
    _holds(r_out, rows, "r_out")
    with _on_device(codes.device):
        if fp4:
            if bits != 4:
                raise ValueError("E2M1 codes are 4 bits wide")
            _check(L.agoq_fp4_act_dequant_rmsnorm(
                _raw(codes.data_ptr()), _raw(scales.data_ptr()), rows, cols, group,
                _raw(gamma.data_ptr()), float(eps), _raw(out.data_ptr()), _raw(r_out.data_ptr()),
                _stream(stream)))
        else:
            _check(L.agoq_act_dequant_rmsnorm(
                _raw(codes.data_ptr()), _raw(scales.data_ptr()), rows, cols, group, bits,
                _raw(gamma.data_ptr()), float(eps), _raw(out.data_ptr()), _raw(r_out.data_ptr()),
                _stream(stream)))
    return out, r_out


def act_dequant_silu_mul(gate_codes, gate_scales, gate_bits, up_codes, up_scales, up_bits, numel,
                         group, out=None, stream=None, fp4=False):
    """Stored gate and up tensors -> z bf16 [numel] = up' * gate' * sigmoid(gate').
    fp4=True: both tensors hold E2M1 codes (both widths must be 4)."""
    import torch
    L = load_library()
    _dev(gate_codes, torch.uint8, "gate_codes")
    _dev(gate_scales, torch.float32, "gate_scales")
    _dev(up_codes, torch.uint8, "up_codes")
    _dev(up_scales, torch.float32, "up_scales")
    if out is None:
        out = torch.empty(numel, dtype=torch.bfloat16, device=gate_codes.device)
    _dev(out, torch.bfloat16, "out")
    _holds(gate_codes, _code_bytes(numel, gate_bits), "gate_codes")
    _holds(up_codes, _code_bytes(numel, up_bits), "up_codes")
    _holds(gate_scales, _groups(numel, group), "gate_scales")
    _holds(up_scales, _groups(numel, group), "up_scales")
    _holds(out, numel, "out")
    with _on_device(gate_codes.device):
        if fp4:
            if gate_bits != 4 or up_bits != 4:
                raise ValueError("E2M1 codes are 4 bits wide")
            _check(L.agoq_fp4_act_dequant_silu_mul(
                _raw(gate_codes.data_ptr()), _raw(gate_scales.data_ptr()), _raw(up_codes.data_ptr()),
                _raw(up_scales.data_ptr()), numel, group, _raw(out.data_ptr()), _stream(stream)))
        else:
            _check(L.agoq_act_dequant_silu_mul(
                _raw(gate_codes.data_ptr()), _raw(gate_scales.data_ptr()), gate_bits,
                _raw(up_codes.data_ptr()), _raw(up_scales.data_ptr()), up_bits, numel, group,
                _raw(out.data_ptr()), _stream(stream)))
    return out


def rmsnorm_fwd_quant(x, gamma, eps, group, bits, stream=None, fp4=False):
    """x bf16 [rows, cols] -> (y bf16 [rows, cols], r float32 [rows], codes uint8, scales float32).
    fp4=True: E2M1 codes (bits must be 4)."""
    import torch
    L = load_library()
    x = _dev(x, torch.bfloat16, "x")
    _dev(gamma, torch.float32, "gamma")
    if x.dim() != 2 or gamma.numel() != x.shape[1]:
        raise ValueError("x must be [rows, cols] and gamma [cols]")
    rows, cols = x.shape
    n = rows * cols
    y = torch.empty_like(x)
    r = torch.empty(rows, dtype=torch.float32, device=x.device)
    codes = torch.empty(max(n * bits // 8, 1), dtype=torch.uint8, device=x.device)
    scales = torch.empty(max(n // max(group, 1), 1), dtype=torch.float32, device=x.device)
    with _on_device(x.device):
        if fp4:
            if bits != 4:
                raise ValueError("E2M1 codes are 4 bits wide")
            _check(L.agoq_fp4_rmsnorm_fwd_quant(
                _raw(x.data_ptr()), rows, cols, _raw(gamma.data_ptr()), float(eps), group,
                _raw(y.data_ptr()), _raw(r.data_ptr()), _raw(codes.data_ptr()),
                _raw(scales.data_ptr()), _stream(stream)))
        else:
            _check(L.agoq_rmsnorm_fwd_quant(
                _raw(x.data_ptr()), rows, cols, _raw(gamma.data_ptr()), float(eps), group, bits,
                _raw(y.data_ptr()), _raw(r.data_ptr()), _raw(codes.data_ptr()),
                _raw(scales.data_ptr()), _stream(stream)))
    return y, r, codes, scales


def silu_mul_fwd_quant(gate, up, group, gate_bits, up_bits, stream=None, fp4=False):
    """gate, up bf16 -> (z bf16, gate_codes, gate_scales, up_codes, up_scales).
    fp4=True: E2M1 codes for both (both widths must be 4)."""
    import torch
    L = load_library()
    gate = _dev(gate, torch.bfloat16, "gate")
    up = _dev(up, torch.bfloat16, "up")
    n = gate.numel()
    if up.numel() != n:
        raise ValueError("gate and up must have the same number of elements")
    z = torch.empty_like(gate)
    gc = torch.empty(max(n * gate_bits // 8, 1), dtype=torch.uint8, device=gate.device)
    uc = torch.empty(max(n * up_bits // 8, 1), dtype=torch.uint8, device=gate.device)
    gs = torch.empty(max(n // max(group, 1), 1), dtype=torch.float32, device=gate.device)
    us = torch.empty(max(n // max(group, 1), 1), dtype=torch.float32, device=gate.device)
    with _on_device(gate.device):
        if fp4:
            if gate_bits != 4 or up_bits != 4:
                raise ValueError("E2M1 codes are 4 bits wide")
            _check(L.agoq_fp4_silu_mul_fwd_quant(
                _raw(gate.data_ptr()), _raw(up.data_ptr()), n, group, _raw(z.data_ptr()),
                _raw(gc.data_ptr()), _raw(gs.data_ptr()), _raw(uc.data_ptr()), _raw(us.data_ptr()),
                _stream(stream)))
        else:
            _check(L.agoq_silu_mul_fwd_quant(
                _raw(gate.data_ptr()), _raw(up.data_ptr()), n, group, gate_bits, up_bits,
                _raw(z.data_ptr()), _raw(gc.data_ptr()), _raw(gs.data_ptr()), _raw(uc.data_ptr()),
                _raw(us.data_ptr()), _stream(stream)))
    return z, gc, gs, uc, us


def grad_quant(grad, group, codes=None, scales=None, stream=None, sr_seed=None):
    """grad: fp32 tensor on the GPU.  Returns (codes int8 [numel], scales float32 [numel/group]).
    sr_seed: an integer selects the stochastic-rounding variant under that seed."""
    import torch
    L = load_library()
    grad = _dev(grad, torch.float32, "grad")
    n = grad.numel()
    if codes is None:
        codes = torch.empty(max(n, 1), dtype=torch.int8, device=grad.device)
    if scales is None:
        scales = torch.empty(max(n // max(group, 1), 1), dtype=torch.float32, device=grad.device)
    _dev(codes, torch.int8, "codes")
    _dev(scales, torch.float32, "scales")
    _holds(codes, n, "codes")
    _holds(scales, _groups(n, group), "scales")
    with _on_device(grad.device):
        if sr_seed is None:
            _check(L.agoq_grad_quant(_raw(grad.data_ptr()), n, group, _raw(codes.data_ptr()),
                                     _raw(scales.data_ptr()), _stream(stream)))
        else:
            _check(L.agoq_grad_quant_sr(_raw(grad.data_ptr()), n, group, int(sr_seed) & 0xFFFFFFFF,
                                        _raw(codes.data_ptr()), _raw(scales.data_ptr()), _stream(stream)))
    return codes, scales


def grad_reduce_requant(in_codes, in_scales, numel, group, out_codes=None, out_scales=None,
                        stream=None, sr_seed=None):
    """in_codes: int8 [K, stride_c]; in_scales: float32 [K, stride_s] (the receive buffer of the
    All-to-All, chunk k in row k).  Returns (codes int8 [numel], scales float32 [numel/group])."""
    import torch
    L = load_library()
    _dev(in_codes, torch.int8, "in_codes")
    _dev(in_scales, torch.float32, "in_scales")
    if in_codes.dim() != 2 or in_scales.dim() != 2 or in_codes.shape[0] != in_scales.shape[0]:
        raise ValueError("expected in_codes [K, stride_c] and in_scales [K, stride_s]")
    K = in_codes.shape[0]
    if out_codes is None:
        out_codes = torch.empty(max(numel, 1), dtype=torch.int8, device=in_codes.device)
    if out_scales is None:
        out_scales = torch.empty(max(numel // max(group, 1), 1), dtype=torch.float32,
                                 device=in_codes.device)
    _dev(out_codes, torch.int8, "out_codes")
    _dev(out_scales, torch.float32, "out_scales")
    _holds(out_codes, numel, "out_codes")
    _holds(out_scales, _groups(numel, group), "out_scales")
    with _on_device(in_codes.device):
        if sr_seed is None:
            _check(L.agoq_grad_reduce_requant(
                _raw(in_codes.data_ptr()), in_codes.shape[1], _raw(in_scales.data_ptr()),
                in_scales.shape[1], K, numel, group, _raw(out_codes.data_ptr()),
                _raw(out_scales.data_ptr()), _stream(stream)))
        else:
            _check(L.agoq_grad_reduce_requant_sr(
                _raw(in_codes.data_ptr()), in_codes.shape[1], _raw(in_scales.data_ptr()),
                in_scales.shape[1], K, numel, group, int(sr_seed) & 0xFFFFFFFF,
                _raw(out_codes.data_ptr()), _raw(out_scales.data_ptr()), _stream(stream)))
    return out_codes, out_scales


def grad_accumulate(main_codes, main_scales, g_new, group, out_codes=None, out_scales=None,
                    stream=None, sr_seed=None):
    """main_codes int8 [numel], main_scales float32 [numel/group], g_new float32 or bfloat16
    [numel].  With out_codes/out_scales left None the stored gradient is updated in place."""
    import torch
    L = load_library()
    _dev(main_codes, torch.int8, "main_codes")
    _dev(main_scales, torch.float32, "main_scales")
    if not isinstance(g_new, torch.Tensor) or g_new.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("g_new must be a float32 or bfloat16 tensor")
    _dev(g_new, g_new.dtype, "g_new")
    n = main_codes.numel()
    if g_new.numel() != n:
        raise ValueError("g_new must have as many elements as main_codes")
    if out_codes is None:
        out_codes = main_codes
    if out_scales is None:
        out_scales = main_scales
    _dev(out_codes, torch.int8, "out_codes")
    _dev(out_scales, torch.float32, "out_scales")
    _holds(main_scales, _groups(n, group), "main_scales")
    _holds(out_codes, n, "out_codes")
    _holds(out_scales, _groups(n, group), "out_scales")
    with _on_device(main_codes.device):
        if sr_seed is None:
            _check(L.agoq_grad_accumulate(
                _raw(main_codes.data_ptr()), _raw(main_scales.data_ptr()), _raw(g_new.data_ptr()),
                1 if g_new.dtype == torch.bfloat16 else 0, n, group, _raw(out_codes.data_ptr()),
                _raw(out_scales.data_ptr()), _stream(stream)))
        else:
            _check(L.agoq_grad_accumulate_sr(
                _raw(main_codes.data_ptr()), _raw(main_scales.data_ptr()), _raw(g_new.data_ptr()),
                1 if g_new.dtype == torch.bfloat16 else 0, n, group, int(sr_seed) & 0xFFFFFFFF,
                _raw(out_codes.data_ptr()), _raw(out_scales.data_ptr()), _stream(stream)))
    return out_codes, out_scales


def grad_dequant(codes, scales, group, out=None, stream=None):
    """int8 codes + float32 scales -> float32 tensor of the same length."""
    import torch
    L = load_library()
    _dev(codes, torch.int8, "codes")
    _dev(scales, torch.float32, "scales")
    n = codes.numel()
    if out is None:
        out = torch.empty(max(n, 1), dtype=torch.float32, device=codes.device)
    _dev(out, torch.float32, "out")
    _holds(scales, _groups(n, group), "scales")
    _holds(out, n, "out")
    with _on_device(codes.device):
        _check(L.agoq_grad_dequant(_raw(codes.data_ptr()), _raw(scales.data_ptr()), n, group,
                                   _raw(out.data_ptr()), _stream(stream)))
    return out


# ---- floating-point code books (E2M1 activations, E4M3 gradients) -----------------

def fp4_act_quant(x, group, codes=None, scales=None, stream=None):
    import torch
    L = load_library()
    x = _dev(x, torch.bfloat16, "x")
    n = x.numel()
    if codes is None:
        codes = torch.empty(max(n // 2, 1), dtype=torch.uint8, device=x.device)
    if scales is None:
        scales = torch.empty(max(n // max(group, 1), 1), dtype=torch.float32, device=x.device)
    _dev(codes, torch.uint8, "codes")
    _dev(scales, torch.float32, "scales")
    _holds(codes, n // 2, "codes")
    _holds(scales, _groups(n, group), "scales")
    with _on_device(x.device):
        _check(L.agoq_fp4_act_quant(_raw(x.data_ptr()), n, group, _raw(codes.data_ptr()),
                                    _raw(scales.data_ptr()), _stream(stream)))
    return codes, scales


def fp4_act_dequant(codes, scales, numel, group, out=None, stream=None):
    import torch
    L = load_library()
    _dev(codes, torch.uint8, "codes")
    _dev(scales, torch.float32, "scales")
    if out is None:
        out = torch.empty(numel, dtype=torch.bfloat16, device=codes.device)
    _dev(out, torch.bfloat16, "out")
    _holds(codes, numel // 2, "codes")
    _holds(scales, _groups(numel, group), "scales")
    _holds(out, numel, "out")
    with _on_device(codes.device):
        _check(L.agoq_fp4_act_dequant(_raw(codes.data_ptr()), _raw(scales.data_ptr()), numel, group,
                                      _raw(out.data_ptr()), _stream(stream)))
    return out


def fp8_grad_quant(grad, group, codes=None, scales=None, stream=None):
    import torch
    L = load_library()
    grad = _dev(grad, torch.float32, "grad")
    n = grad.numel()
    if codes is None:
        codes = torch.empty(max(n, 1), dtype=torch.uint8, device=grad.device)
    if scales is None:
        scales = torch.empty(max(n // max(group, 1), 1), dtype=torch.float32, device=grad.device)
    _dev(codes, torch.uint8, "codes")
    _dev(scales, torch.float32, "scales")
    _holds(codes, n, "codes")
    _holds(scales, _groups(n, group), "scales")
    with _on_device(grad.device):
        _check(L.agoq_fp8_grad_quant(_raw(grad.data_ptr()), n, group, _raw(codes.data_ptr()),
                                     _raw(scales.data_ptr()), _stream(stream)))
    return codes, scales


def fp8_grad_dequant(codes, scales, group, out=None, stream=None):
    import torch
    L = load_library()
    _dev(codes, torch.uint8, "codes")
    _dev(scales, torch.float32, "scales")
    n = codes.numel()
    if out is None:
        out = torch.empty(max(n, 1), dtype=torch.float32, device=codes.device)
    _dev(out, torch.float32, "out")
    _holds(scales, _groups(n, group), "scales")
    _holds(out, n, "out")
    with _on_device(codes.device):
        _check(L.agoq_fp8_grad_dequant(_raw(codes.data_ptr()), _raw(scales.data_ptr()), n, group,
                                       _raw(out.data_ptr()), _stream(stream)))
    return out


def fp8_grad_reduce_requant(in_codes, in_scales, numel, group, out_codes=None, out_scales=None,
                            stream=None):
    import torch
    L = load_library()
    _dev(in_codes, torch.uint8, "in_codes")
    _dev(in_scales, torch.float32, "in_scales")
    if in_codes.dim() != 2 or in_scales.dim() != 2 or in_codes.shape[0] != in_scales.shape[0]:
        raise ValueError("expected in_codes [K, stride_c] and in_scales [K, stride_s]")
    K = in_codes.shape[0]
    if out_codes is None:
        out_codes = torch.empty(max(numel, 1), dtype=torch.uint8, device=in_codes.device)
    if out_scales is None:
        out_scales = torch.empty(max(numel // max(group, 1), 1), dtype=torch.float32,
                                 device=in_codes.device)
    _dev(out_codes, torch.uint8, "out_codes")
    _dev(out_scales, torch.float32, "out_scales")
    _holds(out_codes, numel, "out_codes")
    _holds(out_scales, _groups(numel, group), "out_scales")
    with _on_device(in_codes.device):
        _check(L.agoq_fp8_grad_reduce_requant(
            _raw(in_codes.data_ptr()), in_codes.shape[1], _raw(in_scales.data_ptr()),
            in_scales.shape[1], K, numel, group, _raw(out_codes.data_ptr()),
            _raw(out_scales.data_ptr()), _stream(stream)))
    return out_codes, out_scales


def fp8_grad_accumulate(main_codes, main_scales, g_new, group, out_codes=None, out_scales=None,
                        stream=None):
    """E4M3 form of grad_accumulate; in place when out_codes / out_scales are left None."""
    import torch
    L = load_library()
    _dev(main_codes, torch.uint8, "main_codes")
    _dev(main_scales, torch.float32, "main_scales")
    if not isinstance(g_new, torch.Tensor) or g_new.dtype not in (torch.float32, torch.bfloat16):
        raise TypeError("g_new must be a float32 or bfloat16 tensor")
    _dev(g_new, g_new.dtype, "g_new")
    n = main_codes.numel()
    if g_new.numel() != n:
        raise ValueError("g_new must have as many elements as main_codes")
    out_codes = main_codes if out_codes is None else out_codes
    out_scales = main_scales if out_scales is None else out_scales
    _dev(out_codes, torch.uint8, "out_codes")
    _dev(out_scales, torch.float32, "out_scales")
    _holds(main_scales, _groups(n, group), "main_scales")
    _holds(out_codes, n, "out_codes")
    _holds(out_scales, _groups(n, group), "out_scales")
    with _on_device(main_codes.device):
        _check(L.agoq_fp8_grad_accumulate(
            _raw(main_codes.data_ptr()), _raw(main_scales.data_ptr()), _raw(g_new.data_ptr()),
            1 if g_new.dtype == torch.bfloat16 else 0, n, group, _raw(out_codes.data_ptr()),
            _raw(out_scales.data_ptr()), _stream(stream)))
    return out_codes, out_scales


# ---- host helpers ---------------------------------------------------------------

def codes_bytes(numel, bits):
    return load_library().agoq_codes_bytes(numel, bits)


def num_groups(numel, group):
    return load_library().agoq_num_groups(numel, group)


def dbca_stored_microbatches(n_stages, stage):
    return load_library().agoq_dbca_stored_microbatches(n_stages, stage)


def dbca_bits(n_stages, stage):
    out = _INT(0)
    _check(load_library().agoq_dbca_bits(n_stages, stage, ctypes.byref(out)))
    return out.value


def layer_bitmap(target_bits, native=False):
    """Bits for (norm1 input, out-proj input, norm2 input, gate, up).  native=True: every
    tensor at the stage's own width; else a mix of 4- and 8-bit codes."""
    arr = (_INT * _SLOTS)()
    fn = load_library().agoq_layer_bitmap_native if native else load_library().agoq_layer_bitmap
    _check(fn(target_bits, ctypes.byref(arr)))
    return list(arr)


def layer_stored_bytes(tokens, hidden, ffn, group, bits, with_scales=True):
    arr = (_INT * _SLOTS)(*bits)
    return load_library().agoq_layer_stored_bytes(tokens, hidden, ffn, group, ctypes.byref(arr),
                                                  1 if with_scales else 0)
