"""ctypes binding of ``libdraco.so`` (declared in ``include/draco.h``).

Argument marshalling only: every step of the encode/decode path runs in the
library's HIP kernels and host algebra.  Device memory is passed as torch
tensors (``data_ptr()``), streams as ``torch.cuda.Stream`` objects or ``None``
for torch's current stream.  If the shared library has not been built the
import fails with instructions; there is no fallback implementation.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
LIB_PATH = os.path.join(_HERE, "libdraco.so")
SOURCES = [os.path.join(_HERE, "csrc", n) for n in (
    # slowest first: the per-s encoder units dominate the build time
    "cyc_encode_s16.hip", "cyc_encode_s15.hip", "cyc_encode_s14.hip", "cyc_encode_s13.hip", "cyc_encode_s12.hip",
    "cyc_encode_s11.hip", "cyc_encode_s10.hip", "cyc_encode_s9.hip", "cyc_encode_s8.hip", "cyc_encode_s7.hip", "cyc_encode_s6.hip", "cyc_encode_s5.hip", "cyc_encode_s4.hip", "cyc_encode_s3.hip",
    "cyc_encode_s2.hip", "cyc_encode_s1.hip", "cyc_encode_s0.hip", "rep.hip", "cyc_encode.hip", "cyc_decode.hip",
    "locate.hip", "update.hip", "api.hip", "host_math.cpp")]
HEADERS = [os.path.join(_HERE, "csrc", n) for n in (
    "kernels.hpp", "device_util.hpp", "cyc_encode_kernels.hpp", "cyc_encode_s.inc", "cyc_encode_narrow.hpp",
    "cyc_encode_narrow_s.inc", "host_math.hpp", "projection_rng.hpp")] + [
    os.path.join(_ROOT, "include", "draco.h"), os.path.join(_ROOT, "include", "draco_bench.h")]
BUILD_DIR = os.path.join(_HERE, "_build")

CODE_REPETITION, CODE_CYCLIC = 0, 1
WIRE_PACKED, WIRE_UNPACKED = 0, 1
TAU, TAU_WIDE, TAU_BF16, TAU_I8 = 32.0 / 16777216.0, 1.0 / 68719476736.0, 32.0 / 8589934592.0, 32.0 / 4294967296.0
SECOND_WORD_F32, SECOND_WORD_BF16, SECOND_WORD_I8 = 0, 1, 2
OK, NO_MAJORITY, LOCATE_FAILED = 0, 1, 2
EINVAL, EALIGN, EHIP, ENOMEM = -1, -2, -3, -4
KIND_ENCODE, KIND_VOTE, KIND_PROJECT, KIND_RECOMBINE, KIND_LOCATE = 0, 1, 2, 3, 4
MAX_NODES = 256

EXPORTS = [
    "draco_plan_create", "draco_plan_prepare", "draco_plan_destroy", "draco_message_len",
    "draco_plan_assign", "draco_plan_weights", "draco_encode", "draco_encode_node",
    "draco_decode_repetition", "draco_decode_repetition_async", "draco_decode_cyclic",
    "draco_decode_cyclic_async", "draco_decode_cyclic_hostphi", "draco_encode_wide", "draco_encode_samples",
    "draco_decode_cyclic_wide", "draco_decode_cyclic_wide_async",
    "draco_cyclic_locate", "draco_cyclic_recombination_vector", "draco_strerror",
    "draco_last_hip_error", "draco_plan_set_speculation",
    "draco_plan_set_projection_seed", "draco_projection_vector", "draco_plan_set_wire",
    "draco_cyclic_locate_tol", "draco_decode_repetition_static",
    "draco_plan_last_projection_seed", "draco_encode_oneshot", "draco_decode_repetition_oneshot",
    "draco_decode_cyclic_oneshot", "draco_cache_clear", "draco_apply_update", "draco_encode_samples_wide",
    "draco_plan_set_second_word", "draco_encode_node_wide",
]
# the measuring instruments of include/draco_bench.h
BENCH_EXPORTS = ["draco_copy_probe", "draco_plan_set_timing", "draco_plan_kernel_time", "draco_plan_kernel_times"]


def build(verbose: bool = False) -> str:
    """Compile the library for gfx950 in-tree with hipcc (cross-compiles without a GPU):
    one object per source, compiled in parallel, then one link."""
    from concurrent.futures import ThreadPoolExecutor

    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-fcomplex-arithmetic=basic",
             "-I" + os.path.join(_ROOT, "include")]
    os.makedirs(BUILD_DIR, exist_ok=True)

    def compile_one(src):
        obj = os.path.join(BUILD_DIR, os.path.basename(src) + ".o")
        res = subprocess.run([hipcc, *flags, "-c", src, "-o", obj], capture_output=True, text=True)
        return src, obj, res

    objs = []
    with ThreadPoolExecutor(max_workers=min(os.cpu_count() or 4, 8, len(SOURCES))) as ex:
        for src, obj, res in ex.map(compile_one, SOURCES):
            if verbose or res.returncode != 0:
                print(src)
                print(res.stdout)
                print(res.stderr)
            if res.returncode != 0:
                raise RuntimeError(f"hipcc failed compiling {src}")
            objs.append(obj)
    res = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH],
                         capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed linking libdraco.so")
    return LIB_PATH


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -c 'import __graft_entry__ as g; g.build()'` "
            "(there is no non-HIP fallback)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    L.draco_plan_create.argtypes = [ctypes.POINTER(vp), i32, i32, i32, i64]
    L.draco_plan_create.restype = i32
    L.draco_plan_prepare.argtypes = [vp]
    L.draco_plan_prepare.restype = i32
    L.draco_plan_destroy.argtypes = [vp]
    L.draco_plan_destroy.restype = None
    L.draco_message_len.argtypes = [vp]
    L.draco_message_len.restype = i64
    L.draco_plan_assign.argtypes = [vp, vp]
    L.draco_plan_assign.restype = i32
    L.draco_plan_weights.argtypes = [vp, vp]
    L.draco_plan_weights.restype = i32
    L.draco_encode.argtypes = [vp, vp, i64, vp, i64, vp]
    L.draco_encode.restype = i32
    L.draco_encode_node.argtypes = [vp, i32, vp, i64, vp, vp]
    L.draco_encode_node.restype = i32
    L.draco_decode_repetition.argtypes = [vp, vp, i64, vp, vp, vp]
    L.draco_decode_repetition.restype = i32
    L.draco_decode_repetition_async.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    L.draco_decode_repetition_async.restype = i32
    L.draco_decode_repetition_static.argtypes = [i32, i32, i64, vp, i64, vp, vp, vp, vp]
    L.draco_decode_repetition_static.restype = i32
    L.draco_decode_cyclic.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    L.draco_decode_cyclic.restype = i32
    L.draco_decode_cyclic_hostphi.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    L.draco_decode_cyclic_hostphi.restype = i32
    L.draco_decode_cyclic_async.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp]
    L.draco_decode_cyclic_async.restype = i32
    L.draco_encode_samples.argtypes = [vp, vp, i64, i64, vp, i64, vp]
    L.draco_encode_samples.restype = i32
    L.draco_encode_samples_wide.argtypes = [vp, vp, i64, i64, vp, vp, i64, vp]
    L.draco_encode_samples_wide.restype = i32
    L.draco_encode_node_wide.argtypes = [vp, i32, vp, i64, vp, vp, vp]
    L.draco_encode_node_wide.restype = i32
    L.draco_encode_wide.argtypes = [vp, vp, i64, vp, vp, i64, vp]
    L.draco_encode_wide.restype = i32
    L.draco_decode_cyclic_wide.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp]
    L.draco_decode_cyclic_wide.restype = i32
    L.draco_decode_cyclic_wide_async.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp]
    L.draco_decode_cyclic_wide_async.restype = i32
    L.draco_cyclic_locate.argtypes = [vp, vp, vp, vp]
    L.draco_cyclic_locate.restype = i32
    L.draco_cyclic_recombination_vector.argtypes = [vp, vp, vp]
    L.draco_cyclic_recombination_vector.restype = i32
    L.draco_strerror.argtypes = [i32]
    L.draco_strerror.restype = ctypes.c_char_p
    L.draco_last_hip_error.argtypes = []
    L.draco_last_hip_error.restype = ctypes.c_char_p
    L.draco_cyclic_locate_tol.argtypes = [vp, vp, ctypes.c_double, vp, vp]
    L.draco_cyclic_locate_tol.restype = i32
    L.draco_plan_set_wire.argtypes = [vp, i32]
    L.draco_plan_set_wire.restype = i32
    L.draco_plan_set_second_word.argtypes = [vp, i32]
    L.draco_plan_set_second_word.restype = i32
    L.draco_plan_set_projection_seed.argtypes = [vp, ctypes.c_uint64]
    L.draco_plan_set_projection_seed.restype = i32
    L.draco_projection_vector.argtypes = [vp, ctypes.c_uint64, vp]
    L.draco_projection_vector.restype = i32
    L.draco_plan_set_speculation.argtypes = [vp, i32]
    L.draco_plan_set_speculation.restype = i32
    L.draco_copy_probe.argtypes = [vp, vp, i32, i64, i64, vp]
    L.draco_copy_probe.restype = i32
    L.draco_plan_set_timing.argtypes = [vp, i32]
    L.draco_plan_set_timing.restype = i32
    L.draco_plan_kernel_time.argtypes = [vp, i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
    L.draco_plan_kernel_time.restype = i32
    L.draco_plan_kernel_times.argtypes = [vp, i32, vp, i32, ctypes.POINTER(i32)]
    L.draco_plan_kernel_times.restype = i32
    L.draco_plan_last_projection_seed.argtypes = [vp, ctypes.POINTER(ctypes.c_uint64)]
    L.draco_plan_last_projection_seed.restype = i32
    L.draco_encode_oneshot.argtypes = [vp, i32, i32, i64, vp, i64, i64, vp, i64, vp]
    L.draco_encode_oneshot.restype = i32
    L.draco_decode_repetition_oneshot.argtypes = [vp, i64, i32, i32, i64, vp, vp, vp]
    L.draco_decode_repetition_oneshot.restype = i32
    L.draco_decode_cyclic_oneshot.argtypes = [vp, i64, i32, i32, i64, vp, vp, vp]
    L.draco_decode_cyclic_oneshot.restype = i32
    L.draco_cache_clear.argtypes = []
    L.draco_cache_clear.restype = None
    L.draco_apply_update.argtypes = [vp, vp, i64, ctypes.c_float, vp]
    L.draco_apply_update.restype = i32
    _lib = L
    return L


class DracoError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        detail = lib().draco_last_hip_error().decode() if status == EHIP else ""
        super().__init__(f"draco status {status}: {lib().draco_strerror(status).decode()}"
                         + (f" [{detail}]" if detail else ""))


def _check(status: int) -> None:
    if status < 0:
        raise DracoError(status)


def _stream_ptr(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def _ptr_or_null(t):
    return None if t is None else t.data_ptr()


def mask_words(P: int) -> int:
    return (P + 63) // 64


def mask_to_bool(words: np.ndarray, P: int) -> np.ndarray:
    return np.array([(int(words[j >> 6]) >> (j & 63)) & 1 for j in range(P)], dtype=bool)


def bool_to_mask(mask, P: int) -> np.ndarray:
    words = np.zeros(mask_words(P), dtype=np.uint64)
    for j in range(P):
        if mask[j]:
            words[j >> 6] |= np.uint64(1) << np.uint64(j & 63)
    return words


class Plan:
    """One (code, P, s, d) instance of the library's plan object."""

    def __init__(self, code: int, P: int, s: int, d: int):
        self._h = ctypes.c_void_p()
        status = lib().draco_plan_create(ctypes.byref(self._h), code, P, s, d)
        if status != OK:
            self._h = None
            raise DracoError(status)
        self.code, self.P, self.s, self.d = code, P, s, d
        self._second_word = SECOND_WORD_F32

    def close(self) -> None:
        if getattr(self, "_h", None):
            lib().draco_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:       # interpreter shutdown: the module globals may be gone
            pass

    # ---- host-only ----
    @property
    def message_len(self) -> int:
        return int(lib().draco_message_len(self._h))

    def assign(self) -> np.ndarray:
        A = np.zeros((self.P, self.P), dtype=np.uint8)
        _check(lib().draco_plan_assign(self._h, A.ctypes.data))
        return A

    def weights(self) -> np.ndarray:
        W = np.zeros((self.P, self.P, 2), dtype=np.float64)
        _check(lib().draco_plan_weights(self._h, W.ctypes.data))
        return W[..., 0] + 1j * W[..., 1]

    def cyclic_locate(self, gamma: np.ndarray, tau: float | None = None):
        """(mask bool[P], t complex[P], status) from the P projections; tau: relative zero
        threshold of the syndromes (default: the one-word wire's)."""
        g = np.ascontiguousarray(np.stack([gamma.real, gamma.imag], axis=-1), dtype=np.float64)
        words = np.zeros(mask_words(self.P), dtype=np.uint64)
        t = np.zeros((self.P, 2), dtype=np.float64)
        if tau is None:
            status = lib().draco_cyclic_locate(self._h, g.ctypes.data, words.ctypes.data, t.ctypes.data)
        else:
            status = lib().draco_cyclic_locate_tol(self._h, g.ctypes.data, tau, words.ctypes.data, t.ctypes.data)
        _check(status)
        return mask_to_bool(words, self.P), t[:, 0] + 1j * t[:, 1], status

    def cyclic_recombination_vector(self, mask) -> np.ndarray:
        words = bool_to_mask(mask, self.P)
        b = np.zeros((self.P, 2), dtype=np.float64)
        status = lib().draco_cyclic_recombination_vector(self._h, words.ctypes.data, b.ctypes.data)
        if status != OK:
            raise DracoError(status)
        return b[:, 0] + 1j * b[:, 1]

    # ---- device ----
    def prepare(self) -> None:
        _check(lib().draco_plan_prepare(self._h))

    def encode(self, grads, messages, stream=None) -> None:
        _check(lib().draco_encode(self._h, grads.data_ptr(), grads.stride(0), messages.data_ptr(),
                                  messages.stride(0), _stream_ptr(stream)))

    def encode_node(self, node: int, node_grads, message, stream=None) -> None:
        _check(lib().draco_encode_node(self._h, node, node_grads.data_ptr(), node_grads.stride(0),
                                       message.data_ptr(), _stream_ptr(stream)))

    def encode_node_wide(self, node: int, node_grads, hi, lo, stream=None) -> None:
        want = {SECOND_WORD_BF16: "torch.bfloat16", SECOND_WORD_I8: "torch.int8"}.get(self._second_word, "torch.float32")
        assert str(lo.dtype) == want, (lo.dtype, want)
        _check(lib().draco_encode_node_wide(self._h, node, node_grads.data_ptr(), node_grads.stride(0), hi.data_ptr(),
                                            lo.data_ptr(), _stream_ptr(stream)))

    def decode_repetition(self, messages, out_sum, stream=None):
        """-> (mask bool[P], status); the sum is written to ``out_sum``."""
        words = np.zeros(mask_words(self.P), dtype=np.uint64)
        status = lib().draco_decode_repetition(self._h, messages.data_ptr(), messages.stride(0),
                                               out_sum.data_ptr(), words.ctypes.data, _stream_ptr(stream))
        _check(status)
        return mask_to_bool(words, self.P), status

    def decode_repetition_async(self, messages, out_sum, mask_dev, status_dev, stream=None) -> None:
        _check(lib().draco_decode_repetition_async(self._h, messages.data_ptr(), messages.stride(0),
                                                   out_sum.data_ptr(), mask_dev.data_ptr(),
                                                   status_dev.data_ptr(), _stream_ptr(stream)))

    def decode_cyclic(self, messages, f, out_sum, stream=None):
        words = np.zeros(mask_words(self.P), dtype=np.uint64)
        status = lib().draco_decode_cyclic(self._h, messages.data_ptr(), messages.stride(0), _ptr_or_null(f),
                                           out_sum.data_ptr(), words.ctypes.data, _stream_ptr(stream))
        _check(status)
        return mask_to_bool(words, self.P), status

    def decode_cyclic_hostphi(self, messages, f, out_sum, stream=None):
        words = np.zeros(mask_words(self.P), dtype=np.uint64)
        status = lib().draco_decode_cyclic_hostphi(self._h, messages.data_ptr(), messages.stride(0), _ptr_or_null(f),
                                                   out_sum.data_ptr(), words.ctypes.data, _stream_ptr(stream))
        _check(status)
        return mask_to_bool(words, self.P), status

    def decode_cyclic_async(self, messages, f, out_sum, mask_dev, status_dev, stream=None) -> None:
        _check(lib().draco_decode_cyclic_async(self._h, messages.data_ptr(), messages.stride(0), _ptr_or_null(f),
                                               out_sum.data_ptr(), mask_dev.data_ptr(), status_dev.data_ptr(),
                                               _stream_ptr(stream)))

    def encode_samples(self, samples, messages, stream=None) -> None:
        """samples: [B][ld] with B a multiple of P (B/P per-sample rows per unit gradient)."""
        _check(lib().draco_encode_samples(self._h, samples.data_ptr(), samples.shape[0], samples.stride(0),
                                          messages.data_ptr(), messages.stride(0), _stream_ptr(stream)))

    def encode_samples_wide(self, samples, hi, lo, stream=None) -> None:
        self._check_lo(hi, lo)
        _check(lib().draco_encode_samples_wide(self._h, samples.data_ptr(), samples.shape[0], samples.stride(0),
                                               hi.data_ptr(), lo.data_ptr(), hi.stride(0), _stream_ptr(stream)))

    def encode_wide(self, grads, hi, lo, stream=None) -> None:
        self._check_lo(hi, lo)
        _check(lib().draco_encode_wide(self._h, grads.data_ptr(), grads.stride(0), hi.data_ptr(), lo.data_ptr(),
                                       hi.stride(0), _stream_ptr(stream)))

    def decode_cyclic_wide(self, hi, lo, f, out_sum, stream=None):
        self._check_lo(hi, lo)
        words = np.zeros(mask_words(self.P), dtype=np.uint64)
        status = lib().draco_decode_cyclic_wide(self._h, hi.data_ptr(), lo.data_ptr(), hi.stride(0), _ptr_or_null(f),
                                                out_sum.data_ptr(), words.ctypes.data, _stream_ptr(stream))
        _check(status)
        return mask_to_bool(words, self.P), status

    def decode_cyclic_wide_async(self, hi, lo, f, out_sum, mask_dev, status_dev, stream=None) -> None:
        self._check_lo(hi, lo)
        _check(lib().draco_decode_cyclic_wide_async(self._h, hi.data_ptr(), lo.data_ptr(), hi.stride(0), _ptr_or_null(f),
                                                    out_sum.data_ptr(), mask_dev.data_ptr(), status_dev.data_ptr(),
                                                    _stream_ptr(stream)))

    def set_wire(self, wire: int) -> None:
        _check(lib().draco_plan_set_wire(self._h, wire))

    def set_second_word(self, fmt: int) -> None:
        """Two-word wire: SECOND_WORD_F32 (float32 slab), SECOND_WORD_BF16 (bfloat16 slab) or
        SECOND_WORD_I8 (int8 slab), all of the first word's shape."""
        _check(lib().draco_plan_set_second_word(self._h, fmt))
        self._second_word = fmt

    def _check_lo(self, hi, lo) -> None:
        """The second slab has the first one's row stride in elements and the plan's element type."""
        want = {SECOND_WORD_BF16: "torch.bfloat16", SECOND_WORD_I8: "torch.int8"}.get(self._second_word, "torch.float32")
        assert hi.stride(0) == lo.stride(0) and str(lo.dtype) == want, (lo.dtype, want)

    def set_projection_seed(self, seed: int) -> None:
        _check(lib().draco_plan_set_projection_seed(self._h, seed))

    def projection_vector(self, seed: int) -> np.ndarray:
        f = np.zeros(self.message_len // 2, dtype=np.float32)
        _check(lib().draco_projection_vector(self._h, seed, f.ctypes.data))
        return f

    def last_projection_seed(self) -> int:
        seed = ctypes.c_uint64()
        _check(lib().draco_plan_last_projection_seed(self._h, ctypes.byref(seed)))
        return seed.value

    def set_speculation(self, enabled: bool) -> None:
        _check(lib().draco_plan_set_speculation(self._h, 1 if enabled else 0))

    def set_timing(self, max_records: int) -> None:
        _check(lib().draco_plan_set_timing(self._h, max_records))

    def kernel_time(self, kind: int):
        """(total_ms, launches) of the timed kernels of one kind since the last query."""
        ms, n = ctypes.c_double(), ctypes.c_int()
        _check(lib().draco_plan_kernel_time(self._h, kind, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, n.value

    def kernel_times(self, kind: int, capacity: int = 4096) -> np.ndarray:
        """Durations in ms of the timed launches of one kind since the last query, in launch order."""
        out = np.zeros(capacity, dtype=np.float64)
        n = ctypes.c_int()
        _check(lib().draco_plan_kernel_times(self._h, kind, out.ctypes.data, capacity, ctypes.byref(n)))
        return out[:min(n.value, capacity)].copy()


def draco_copy_probe(src, dst, rows: int, row_len: int, ld: int, stream=None) -> None:
    _check(lib().draco_copy_probe(src.data_ptr(), dst.data_ptr(), rows, row_len, ld, _stream_ptr(stream)))


def draco_decode_repetition_static(P: int, s: int, d: int, messages, out_sum, mask_dev, status_dev, stream=None) -> None:
    """The allocation-free repetition decoder (no plan); outputs stay on the device."""
    _check(lib().draco_decode_repetition_static(P, s, d, messages.data_ptr(), messages.stride(0), out_sum.data_ptr(),
                                                mask_dev.data_ptr(), status_dev.data_ptr(), _stream_ptr(stream)))


# Names of the C entry points, module-level, same spelling as the header.
def draco_encode(plan: Plan, grads, messages, stream=None) -> None:
    plan.encode(grads, messages, stream)


def draco_encode_node(plan: Plan, node: int, node_grads, message, stream=None) -> None:
    plan.encode_node(node, node_grads, message, stream)


def draco_decode_repetition(plan: Plan, messages, out_sum, stream=None):
    return plan.decode_repetition(messages, out_sum, stream)


def draco_decode_cyclic(plan: Plan, messages, f, out_sum, stream=None):
    return plan.decode_cyclic(messages, f, out_sum, stream)


# ---------------------------------------------------------------------------
# The three calls without a plan, on torch tensors: encode(assign, grads) -> messages;
# decode(messages, P, s) -> (sum, mask).  The library keeps the plans; this side only
# allocates the outputs and marshals.
# ---------------------------------------------------------------------------
def _row_stride(n: int) -> int:
    return (n + 3) // 4 * 4


def draco_apply_update(params, out_sum, d: int, scale: float, stream=None) -> None:
    """params[:d] -= scale * out_sum[:d] on the device (the parameter server's SGD step)."""
    _check(lib().draco_apply_update(params.data_ptr(), out_sum.data_ptr(), d, scale, _stream_ptr(stream)))


def encode(assign: np.ndarray, code: int, grads, d: int | None = None):
    """assign [P][P] 0/1 (the code's allocation matrix), grads [B][>= d] fp32 on the GPU with B a
    multiple of P -> messages [P][message_len]."""
    import torch
    A = np.ascontiguousarray(assign, dtype=np.uint8)
    P = A.shape[0]
    d = grads.shape[1] if d is None else d
    mlen = d if code == CODE_REPETITION else 2 * ((d + 1) // 2)
    with torch.cuda.device(grads.device):
        out = torch.empty((P, _row_stride(mlen)), dtype=torch.float32, device=grads.device)
        st = lib().draco_encode_oneshot(A.ctypes.data, code, P, d, grads.data_ptr(), grads.shape[0], grads.stride(0),
                                        out.data_ptr(), out.stride(0), _stream_ptr(None))
    if st != OK:
        raise DracoError(st)
    return out[:, :mlen]


def decode_repetition(messages, P: int, s: int):
    """messages [P][d] -> (sum [d], mask bool[P], status)."""
    import torch
    assert messages.shape[0] == P
    d = messages.shape[1]
    words = np.zeros(mask_words(P), dtype=np.uint64)
    with torch.cuda.device(messages.device):
        out = torch.empty(_row_stride(d), dtype=torch.float32, device=messages.device)
        status = lib().draco_decode_repetition_oneshot(messages.data_ptr(), messages.stride(0), P, s, d, out.data_ptr(),
                                                       words.ctypes.data, _stream_ptr(None))
    _check(status)
    return out[:d], mask_to_bool(words, P), status


def decode_cyclic(messages, P: int, s: int, d: int):
    """messages [P][2*ceil(d/2)] -> (sum [d], mask bool[P], status); the projection vector is
    drawn inside the library, afresh for every call."""
    import torch
    assert messages.shape[0] == P
    words = np.zeros(mask_words(P), dtype=np.uint64)
    with torch.cuda.device(messages.device):
        out = torch.empty(_row_stride(d), dtype=torch.float32, device=messages.device)
        status = lib().draco_decode_cyclic_oneshot(messages.data_ptr(), messages.stride(0), P, s, d, out.data_ptr(),
                                                   words.ctypes.data, _stream_ptr(None))
    _check(status)
    return out[:d], mask_to_bool(words, P), status
