"""numpy-facing wrapper around oracle/libagoq_ref.so (host pointers only).

TEST INFRASTRUCTURE.  Every function takes and returns numpy arrays; bf16
data travels as uint16 bit patterns.  No arithmetic of the method happens in
this file: it marshals arguments for the C oracle.
"""
import ctypes
import os

import numpy as np

from . import build as _build

__all__ = [
    "lib", "rmsnorm_fwd", "silu_mul_fwd", "fp4_act_quant", "fp4_act_dequant", "fp8_grad_quant", "fp8_grad_dequant",
    "fp8_grad_reduce_requant", "fp8_grad_accumulate", "e2m1_encode", "e2m1_decode", "e4m3_encode", "e4m3_decode", "act_quant", "act_dequant", "act_dequant_rmsnorm", "act_dequant_silu_mul", "grad_quant", "grad_dequant",
    "grad_reduce_requant", "grad_reduce_f64", "grad_accumulate", "dbca_bits",
    "act_quant_sr", "grad_quant_sr", "grad_reduce_requant_sr", "grad_accumulate_sr", "sr_word", "sr_u",
    "dbca_stored_microbatches", "bf16_to_f32", "f32_to_bf16", "max_threads",
    "set_threads", "OracleError", "Oracle",
]

_I64 = ctypes.c_int64
_INT = ctypes.c_int
_P = ctypes.c_void_p


class OracleError(RuntimeError):
    def __init__(self, status):
        super().__init__("oracle returned status %d" % status)
        self.status = status


def _bind(path):
    L = ctypes.CDLL(path)
    L.agoq_ref_act_quant.argtypes = [_P, _I64, _INT, _INT, _P, _P]
    L.agoq_ref_act_dequant.argtypes = [_P, _P, _I64, _INT, _INT, _P]
    L.agoq_ref_grad_quant.argtypes = [_P, _I64, _INT, _P, _P]
    L.agoq_ref_grad_dequant.argtypes = [_P, _P, _I64, _INT, _P]
    L.agoq_ref_grad_reduce_requant.argtypes = [_P, _I64, _P, _I64, _INT, _I64, _INT, _P, _P]
    L.agoq_ref_grad_reduce_f64.argtypes = [_P, _I64, _P, _I64, _INT, _I64, _INT, _P, _P]
    L.agoq_ref_grad_accumulate.argtypes = [_P, _P, _P, _INT, _I64, _INT, _P, _P]
    L.agoq_ref_act_dequant_rmsnorm.argtypes = [_P, _P, _I64, _I64, _INT, _INT, _P, ctypes.c_float, _P, _P]
    L.agoq_ref_act_dequant_silu_mul.argtypes = [_P, _P, _INT, _P, _P, _INT, _I64, _INT, _P]
    L.agoq_ref_rmsnorm_fwd.argtypes = [_P, _I64, _I64, _P, ctypes.c_float, _P, _P]
    L.agoq_ref_silu_mul_fwd.argtypes = [_P, _P, _I64, _P]
    L.agoq_ref_fp4_act_quant.argtypes = [_P, _I64, _INT, _P, _P]
    L.agoq_ref_fp4_act_dequant.argtypes = [_P, _P, _I64, _INT, _P]
    L.agoq_ref_fp8_grad_quant.argtypes = [_P, _I64, _INT, _P, _P]
    L.agoq_ref_fp8_grad_dequant.argtypes = [_P, _P, _I64, _INT, _P]
    L.agoq_ref_fp8_grad_reduce_requant.argtypes = [_P, _I64, _P, _I64, _INT, _I64, _INT, _P, _P]
    L.agoq_ref_fp8_grad_accumulate.argtypes = [_P, _P, _P, _INT, _I64, _INT, _P, _P]
    _U32 = ctypes.c_uint32
    L.agoq_ref_act_quant_sr.argtypes = [_P, _I64, _INT, _INT, _U32, _P, _P]
    L.agoq_ref_grad_quant_sr.argtypes = [_P, _I64, _INT, _U32, _P, _P]
    L.agoq_ref_grad_reduce_requant_sr.argtypes = [_P, _I64, _P, _I64, _INT, _I64, _INT, _U32, _P, _P]
    L.agoq_ref_grad_accumulate_sr.argtypes = [_P, _P, _P, _INT, _I64, _INT, _U32, _P, _P]
    L.agoq_ref_sr_word.argtypes = [_U32, ctypes.c_uint64]
    L.agoq_ref_sr_word.restype = _U32
    L.agoq_ref_sr_u.argtypes = [_U32, _I64]
    L.agoq_ref_sr_u.restype = ctypes.c_float
    for name in ("e2m1", "e4m3"):
        enc = getattr(L, "agoq_ref_%s_encode" % name)
        enc.argtypes = [ctypes.c_float]
        enc.restype = ctypes.c_uint8
        dec = getattr(L, "agoq_ref_%s_decode" % name)
        dec.argtypes = [ctypes.c_uint8]
        dec.restype = ctypes.c_float
    L.agoq_ref_dbca_bits.argtypes = [_INT, _INT, ctypes.POINTER(_INT)]
    L.agoq_ref_dbca_stored_microbatches.argtypes = [_INT, _INT]
    L.agoq_ref_bf16_to_f32.argtypes = [ctypes.c_uint16]
    L.agoq_ref_bf16_to_f32.restype = ctypes.c_float
    L.agoq_ref_f32_to_bf16.argtypes = [ctypes.c_float]
    L.agoq_ref_f32_to_bf16.restype = ctypes.c_uint16
    L.agoq_ref_set_threads.argtypes = [_INT]
    L.agoq_ref_set_threads.restype = None
    return L


def _ptr(a):
    return a.ctypes.data_as(_P)


def _c(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != np.dtype(dtype):
        raise TypeError("expected %s, got %s" % (np.dtype(dtype), a.dtype))
    return a


def _check(status):
    if status != 0:
        raise OracleError(status)


def _chunks(in_codes, in_scales):
    in_codes = _c(in_codes, np.int8)
    in_scales = _c(in_scales, np.float32)
    if in_codes.ndim != 2 or in_scales.ndim != 2 or in_codes.shape[0] != in_scales.shape[0]:
        raise ValueError("expected codes [K, stride_c] and scales [K, stride_s]")
    return in_codes, in_scales


class Oracle:
    """One loaded oracle library.  The module-level functions use the default build;
    the tests also load deliberately broken builds through this class to show that
    the pins notice them."""

    OracleError = OracleError

    def __init__(self, path=None):
        if path is None:
            path = _build.build(force=False)
        if not os.path.exists(path):
            raise RuntimeError("oracle library missing: run python oracle/build.py")
        self.lib = _bind(path)

    def act_quant(self, x_bf16_bits, group, bits):
        """uint16 bf16 patterns (any shape, flattened) -> (codes uint8, scales float32)."""
        x = _c(x_bf16_bits, np.uint16).reshape(-1)
        n = x.size
        codes = np.zeros(max(n * bits // 8, 0), np.uint8)
        scales = np.zeros(max(n // max(group, 1), 0), np.float32)
        _check(self.lib.agoq_ref_act_quant(_ptr(x), n, group, bits, _ptr(codes), _ptr(scales)))
        return codes, scales

    # ---- stochastic rounding (optional variant; the paper never uses it) ----

    def sr_word(self, seed, block):
        return self.lib.agoq_ref_sr_word(int(seed) & 0xFFFFFFFF, int(block))

    def sr_u(self, seed, index):
        return self.lib.agoq_ref_sr_u(int(seed) & 0xFFFFFFFF, int(index))

    def act_quant_sr(self, x_bf16_bits, group, bits, seed):
        x = _c(x_bf16_bits, np.uint16).reshape(-1)
        n = x.size
        codes = np.zeros(max(n * bits // 8, 0), np.uint8)
        scales = np.zeros(max(n // max(group, 1), 0), np.float32)
        _check(self.lib.agoq_ref_act_quant_sr(_ptr(x), n, group, bits, int(seed) & 0xFFFFFFFF, _ptr(codes),
                                              _ptr(scales)))
        return codes, scales

    def grad_quant_sr(self, g, group, seed):
        g = _c(g, np.float32).reshape(-1)
        codes = np.zeros(g.size, np.int8)
        scales = np.zeros(g.size // max(group, 1), np.float32)
        _check(self.lib.agoq_ref_grad_quant_sr(_ptr(g), g.size, group, int(seed) & 0xFFFFFFFF, _ptr(codes),
                                               _ptr(scales)))
        return codes, scales

    def grad_reduce_requant_sr(self, in_codes, in_scales, numel, group, seed):
        in_codes, in_scales = _chunks(in_codes, in_scales)
        K = in_codes.shape[0]
        out_codes = np.zeros(numel, np.int8)
        out_scales = np.zeros(numel // max(group, 1), np.float32)
        _check(self.lib.agoq_ref_grad_reduce_requant_sr(
            _ptr(in_codes), in_codes.shape[1], _ptr(in_scales), in_scales.shape[1], K, numel, group,
            int(seed) & 0xFFFFFFFF, _ptr(out_codes), _ptr(out_scales)))
        return out_codes, out_scales

    def grad_accumulate_sr(self, main_codes, main_scales, g_new, group, seed):
        main_codes = _c(main_codes, np.int8).reshape(-1)
        main_scales = _c(main_scales, np.float32).reshape(-1)
        g_new = np.ascontiguousarray(g_new).reshape(-1)
        if g_new.dtype not in (np.dtype(np.float32), np.dtype(np.uint16)):
            raise TypeError("g_new must be float32 or uint16 (bf16 bits)")
        n = main_codes.size
        out_codes = np.zeros(n, np.int8)
        out_scales = np.zeros(n // max(group, 1), np.float32)
        _check(self.lib.agoq_ref_grad_accumulate_sr(
            _ptr(main_codes), _ptr(main_scales), _ptr(g_new), 1 if g_new.dtype == np.uint16 else 0, n, group,
            int(seed) & 0xFFFFFFFF, _ptr(out_codes), _ptr(out_scales)))
        return out_codes, out_scales

    def act_dequant(self, codes, scales, numel, group, bits):
        codes = _c(codes, np.uint8).reshape(-1)
        scales = _c(scales, np.float32).reshape(-1)
        y = np.zeros(numel, np.uint16)
        _check(self.lib.agoq_ref_act_dequant(_ptr(codes), _ptr(scales), numel, group, bits,
                                             _ptr(y)))
        return y

    def act_dequant_rmsnorm(self, codes, scales, rows, cols, group, bits, gamma, eps):
        """Returns (y bf16 bits [rows*cols], r float32 [rows])."""
        codes = _c(codes, np.uint8).reshape(-1)
        scales = _c(scales, np.float32).reshape(-1)
        gamma = _c(gamma, np.float32).reshape(-1)
        y = np.zeros(rows * cols, np.uint16)
        r = np.zeros(rows, np.float32)
        _check(self.lib.agoq_ref_act_dequant_rmsnorm(_ptr(codes), _ptr(scales), rows, cols, group,
                                                     bits, _ptr(gamma), float(eps), _ptr(y), _ptr(r)))
        return y, r

    def act_dequant_silu_mul(self, gate_codes, gate_scales, gate_bits, up_codes, up_scales, up_bits,
                             numel, group):
        gate_codes = _c(gate_codes, np.uint8).reshape(-1)
        up_codes = _c(up_codes, np.uint8).reshape(-1)
        gate_scales = _c(gate_scales, np.float32).reshape(-1)
        up_scales = _c(up_scales, np.float32).reshape(-1)
        z = np.zeros(numel, np.uint16)
        _check(self.lib.agoq_ref_act_dequant_silu_mul(
            _ptr(gate_codes), _ptr(gate_scales), gate_bits, _ptr(up_codes), _ptr(up_scales),
            up_bits, numel, group, _ptr(z)))
        return z

    def rmsnorm_fwd(self, x_bf16_bits, rows, cols, gamma, eps):
        x = _c(x_bf16_bits, np.uint16).reshape(-1)
        gamma = _c(gamma, np.float32).reshape(-1)
        y = np.zeros(rows * cols, np.uint16)
        r = np.zeros(rows, np.float32)
        _check(self.lib.agoq_ref_rmsnorm_fwd(_ptr(x), rows, cols, _ptr(gamma), float(eps), _ptr(y), _ptr(r)))
        return y, r

    def silu_mul_fwd(self, gate_bits, up_bits):
        g = _c(gate_bits, np.uint16).reshape(-1)
        u = _c(up_bits, np.uint16).reshape(-1)
        z = np.zeros(g.size, np.uint16)
        _check(self.lib.agoq_ref_silu_mul_fwd(_ptr(g), _ptr(u), g.size, _ptr(z)))
        return z

    # ---- floating-point code books (E2M1 activations, E4M3 gradients) ----

    def fp4_act_quant(self, x_bf16_bits, group):
        x = _c(x_bf16_bits, np.uint16).reshape(-1)
        codes = np.zeros(x.size // 2, np.uint8)
        scales = np.zeros(x.size // max(group, 1), np.float32)
        _check(self.lib.agoq_ref_fp4_act_quant(_ptr(x), x.size, group, _ptr(codes), _ptr(scales)))
        return codes, scales

    def fp4_act_dequant(self, codes, scales, numel, group):
        codes = _c(codes, np.uint8).reshape(-1)
        scales = _c(scales, np.float32).reshape(-1)
        y = np.zeros(numel, np.uint16)
        _check(self.lib.agoq_ref_fp4_act_dequant(_ptr(codes), _ptr(scales), numel, group, _ptr(y)))
        return y

    def fp8_grad_quant(self, g, group):
        g = _c(g, np.float32).reshape(-1)
        codes = np.zeros(g.size, np.uint8)
        scales = np.zeros(g.size // max(group, 1), np.float32)
        _check(self.lib.agoq_ref_fp8_grad_quant(_ptr(g), g.size, group, _ptr(codes), _ptr(scales)))
        return codes, scales

    def fp8_grad_dequant(self, codes, scales, group):
        codes = _c(codes, np.uint8).reshape(-1)
        scales = _c(scales, np.float32).reshape(-1)
        out = np.zeros(codes.size, np.float32)
        _check(self.lib.agoq_ref_fp8_grad_dequant(_ptr(codes), _ptr(scales), codes.size, group, _ptr(out)))
        return out

    def fp8_grad_reduce_requant(self, in_codes, in_scales, numel, group):
        in_codes = _c(in_codes, np.uint8)
        in_scales = _c(in_scales, np.float32)
        if in_codes.ndim != 2 or in_scales.ndim != 2 or in_codes.shape[0] != in_scales.shape[0]:
            raise ValueError("expected codes [K, stride_c] and scales [K, stride_s]")
        K = in_codes.shape[0]
        out_codes = np.zeros(numel, np.uint8)
        out_scales = np.zeros(numel // max(group, 1), np.float32)
        _check(self.lib.agoq_ref_fp8_grad_reduce_requant(
            _ptr(in_codes), in_codes.shape[1], _ptr(in_scales), in_scales.shape[1], K, numel,
            group, _ptr(out_codes), _ptr(out_scales)))
        return out_codes, out_scales

    def fp8_grad_accumulate(self, main_codes, main_scales, g_new, group):
        main_codes = _c(main_codes, np.uint8).reshape(-1)
        main_scales = _c(main_scales, np.float32).reshape(-1)
        g_new = np.ascontiguousarray(g_new).reshape(-1)
        if g_new.dtype not in (np.dtype(np.float32), np.dtype(np.uint16)):
            raise TypeError("g_new must be float32 or uint16 (bf16 bits)")
        n = main_codes.size
        out_codes = np.zeros(n, np.uint8)
        out_scales = np.zeros(n // max(group, 1), np.float32)
        _check(self.lib.agoq_ref_fp8_grad_accumulate(
            _ptr(main_codes), _ptr(main_scales), _ptr(g_new), 1 if g_new.dtype == np.uint16 else 0,
            n, group, _ptr(out_codes), _ptr(out_scales)))
        return out_codes, out_scales

    def e2m1_encode(self, t):
        return self.lib.agoq_ref_e2m1_encode(float(t))

    def e2m1_decode(self, c):
        return self.lib.agoq_ref_e2m1_decode(int(c))

    def e4m3_encode(self, t):
        return self.lib.agoq_ref_e4m3_encode(float(t))

    def e4m3_decode(self, c):
        return self.lib.agoq_ref_e4m3_decode(int(c))

    def grad_quant(self, g, group):
        g = _c(g, np.float32).reshape(-1)
        codes = np.zeros(g.size, np.int8)
        scales = np.zeros(g.size // max(group, 1), np.float32)
        _check(self.lib.agoq_ref_grad_quant(_ptr(g), g.size, group, _ptr(codes), _ptr(scales)))
        return codes, scales

    def grad_dequant(self, codes, scales, group):
        codes = _c(codes, np.int8).reshape(-1)
        scales = _c(scales, np.float32).reshape(-1)
        out = np.zeros(codes.size, np.float32)
        _check(self.lib.agoq_ref_grad_dequant(_ptr(codes), _ptr(scales), codes.size, group,
                                              _ptr(out)))
        return out

    def grad_reduce_requant(self, in_codes, in_scales, numel, group):
        """in_codes int8 [K, stride_c >= numel], in_scales float32 [K, stride_s >= numel/group]."""
        in_codes, in_scales = _chunks(in_codes, in_scales)
        K = in_codes.shape[0]
        out_codes = np.zeros(numel, np.int8)
        out_scales = np.zeros(numel // max(group, 1), np.float32)
        _check(self.lib.agoq_ref_grad_reduce_requant(
            _ptr(in_codes), in_codes.shape[1], _ptr(in_scales), in_scales.shape[1], K, numel,
            group, _ptr(out_codes), _ptr(out_scales)))
        return out_codes, out_scales

    def grad_reduce_f64(self, in_codes, in_scales, numel, group):
        in_codes, in_scales = _chunks(in_codes, in_scales)
        K = in_codes.shape[0]
        s = np.zeros(numel, np.float64)
        a = np.zeros(numel, np.float64)
        _check(self.lib.agoq_ref_grad_reduce_f64(
            _ptr(in_codes), in_codes.shape[1], _ptr(in_scales), in_scales.shape[1], K, numel,
            group, _ptr(s), _ptr(a)))
        return s, a

    def grad_accumulate(self, main_codes, main_scales, g_new, group):
        """g_new: float32, or uint16 holding bf16 bit patterns."""
        main_codes = _c(main_codes, np.int8).reshape(-1)
        main_scales = _c(main_scales, np.float32).reshape(-1)
        g_new = np.ascontiguousarray(g_new).reshape(-1)
        if g_new.dtype == np.float32:
            is_bf16 = 0
        elif g_new.dtype == np.uint16:
            is_bf16 = 1
        else:
            raise TypeError("g_new must be float32 or uint16 (bf16 bits)")
        n = main_codes.size
        out_codes = np.zeros(n, np.int8)
        out_scales = np.zeros(n // max(group, 1), np.float32)
        _check(self.lib.agoq_ref_grad_accumulate(
            _ptr(main_codes), _ptr(main_scales), _ptr(g_new), is_bf16, n, group,
            _ptr(out_codes), _ptr(out_scales)))
        return out_codes, out_scales

    def dbca_bits(self, n_stages, stage):
        out = _INT(0)
        _check(self.lib.agoq_ref_dbca_bits(n_stages, stage, ctypes.byref(out)))
        return out.value

    def dbca_stored_microbatches(self, n_stages, stage):
        return self.lib.agoq_ref_dbca_stored_microbatches(n_stages, stage)

    def bf16_to_f32(self, h):
        return self.lib.agoq_ref_bf16_to_f32(int(h))

    def f32_to_bf16(self, f):
        return self.lib.agoq_ref_f32_to_bf16(float(f))

    def max_threads(self):
        return self.lib.agoq_ref_max_threads()

    def set_threads(self, n):
        self.lib.agoq_ref_set_threads(int(n))


_default = Oracle()
lib = _default.lib
act_quant = _default.act_quant
act_dequant = _default.act_dequant
act_dequant_rmsnorm = _default.act_dequant_rmsnorm
rmsnorm_fwd = _default.rmsnorm_fwd
silu_mul_fwd = _default.silu_mul_fwd
act_dequant_silu_mul = _default.act_dequant_silu_mul
grad_quant = _default.grad_quant
fp4_act_quant = _default.fp4_act_quant
fp4_act_dequant = _default.fp4_act_dequant
fp8_grad_quant = _default.fp8_grad_quant
fp8_grad_dequant = _default.fp8_grad_dequant
fp8_grad_reduce_requant = _default.fp8_grad_reduce_requant
fp8_grad_accumulate = _default.fp8_grad_accumulate
e2m1_encode = _default.e2m1_encode
e2m1_decode = _default.e2m1_decode
e4m3_encode = _default.e4m3_encode
e4m3_decode = _default.e4m3_decode
grad_dequant = _default.grad_dequant
grad_reduce_requant = _default.grad_reduce_requant
grad_reduce_f64 = _default.grad_reduce_f64
grad_accumulate = _default.grad_accumulate
act_quant_sr = _default.act_quant_sr
grad_quant_sr = _default.grad_quant_sr
grad_reduce_requant_sr = _default.grad_reduce_requant_sr
grad_accumulate_sr = _default.grad_accumulate_sr
sr_word = _default.sr_word
sr_u = _default.sr_u
dbca_bits = _default.dbca_bits
dbca_stored_microbatches = _default.dbca_stored_microbatches
bf16_to_f32 = _default.bf16_to_f32
f32_to_bf16 = _default.f32_to_bf16
max_threads = _default.max_threads
set_threads = _default.set_threads
