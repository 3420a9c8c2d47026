"""ctypes binding of libs3gd.so: the same entry points as include/s3gd.h.

Only argument marshalling happens here.  PyTorch supplies device memory (tensors) and
streams; every step of the path runs in the library's HIP kernels.  There is no fallback:
if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libs3gd.so")

OK, E_INVAL, E_RANGE, E_HIP, E_NOMEM, E_NAN, E_FORMAT, E_CAPACITY, E_TOOBIG = 0, -1, -2, -3, -4, -5, -6, -7, -8
STATIC_SCRATCH_BYTES = 128 << 20
PAD = 0xFFFFFFFF
N_LIMIT = (1 << 31) - 2

EXPORTS = (
    "s3gd_workspace_bytes", "s3gd_create", "s3gd_destroy", "s3gd_topk_sign_encode", "s3gd_majority_vote",
    "s3gd_apply_update", "s3gd_step", "s3gd_step_static", "s3gd_topk_sign_encode_ec", "s3gd_step_ec", "s3gd_topk_sign_encode_acc", "s3gd_step_acc",
    "s3gd_apply_update_momentum", "s3gd_step_momentum", "s3gd_vote_update", "s3gd_packed_row_words",
    "s3gd_pack_messages", "s3gd_unpack_messages", "s3gd_votes_to_message", "s3gd_randk_sign_encode", "s3gd_step_randk", "s3gd_last_async_status", "s3gd_last_encode_info", "s3gd_last_hip_error",
    "s3gd_strerror", "s3gd_last_row_state", "s3gd_calibrate_read", "s3gd_calibrate_rmw", "s3gd_encode_plan_info", "s3gd_encode_sample_unit_start", "s3gd_profile_enable", "s3gd_profile_read", "s3gd_profile_kernel_name",
)
PROFILE_KERNELS = 26

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")

_lib = ctypes.CDLL(LIB_PATH)

_vp, _u32, _u64, _f32, _int = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_float, ctypes.c_int
_lib.s3gd_workspace_bytes.restype = ctypes.c_size_t
_lib.s3gd_workspace_bytes.argtypes = [_u32, _u64, _u64]
_lib.s3gd_create.restype = _int
_lib.s3gd_create.argtypes = [ctypes.POINTER(_vp), _int, _u32, _u64, _u64]
_lib.s3gd_destroy.restype = _int
_lib.s3gd_destroy.argtypes = [_vp]
_lib.s3gd_topk_sign_encode.restype = _int
_lib.s3gd_topk_sign_encode.argtypes = [_vp, _vp, _u32, _u64, _u64, _vp, _vp, _vp]
_lib.s3gd_majority_vote.restype = _int
_lib.s3gd_majority_vote.argtypes = [_vp, _vp, _vp, _u32, _u64, _u64, _vp, _vp, _vp]
_lib.s3gd_apply_update.restype = _int
_lib.s3gd_apply_update.argtypes = [_vp, _vp, _vp, _f32, _u64, _vp]
_lib.s3gd_step.restype = _int
_lib.s3gd_step.argtypes = [_vp, _vp, _u32, _u64, _u64, _vp, _f32, _vp, _vp, _vp, _vp, _vp]
_lib.s3gd_step_static.restype = _int
_lib.s3gd_step_static.argtypes = [_int, _vp, _u32, _u64, _u64, _vp, _f32, _vp, _vp, _vp, _vp, _vp, _vp]
_lib.s3gd_topk_sign_encode_acc.restype = _int
_lib.s3gd_topk_sign_encode_acc.argtypes = [_vp, _vp, _u32, _u64, _u64, _vp, _vp, _vp]
_lib.s3gd_step_acc.restype = _int
_lib.s3gd_step_acc.argtypes = [_vp, _vp, _u32, _u64, _u64, _vp, _f32, _vp, _vp, _vp, _vp, _vp]
_lib.s3gd_topk_sign_encode_ec.restype = _int
_lib.s3gd_topk_sign_encode_ec.argtypes = [_vp, _vp, _vp, _f32, _u32, _u64, _u64, _vp, _vp, _vp]
_lib.s3gd_step_ec.restype = _int
_lib.s3gd_step_ec.argtypes = [_vp, _vp, _vp, _f32, _u32, _u64, _u64, _vp, _f32, _vp, _vp, _vp, _vp, _vp]
_lib.s3gd_apply_update_momentum.restype = _int
_lib.s3gd_apply_update_momentum.argtypes = [_vp, _vp, _vp, _vp, _f32, _f32, _u64, _vp]
_lib.s3gd_step_momentum.restype = _int
_lib.s3gd_step_momentum.argtypes = [_vp, _vp, _vp, _f32, _u32, _u64, _u64, _vp, _vp, _f32, _f32, _vp, _vp, _vp]
_lib.s3gd_vote_update.restype = _int
_lib.s3gd_vote_update.argtypes = [_vp, _vp, _vp, _u32, _u64, _u64, _vp, _f32, _vp]
_lib.s3gd_packed_row_words.restype = _u64
_lib.s3gd_packed_row_words.argtypes = [_u64, _u64]
_lib.s3gd_pack_messages.restype = _int
_lib.s3gd_pack_messages.argtypes = [_vp, _vp, _vp, _u32, _u64, _u64, _vp, _u64, _vp]
_lib.s3gd_unpack_messages.restype = _int
_lib.s3gd_unpack_messages.argtypes = [_vp, _vp, _u64, _u32, _u64, _u64, _vp, _vp, _vp]
_lib.s3gd_votes_to_message.restype = _int
_lib.s3gd_votes_to_message.argtypes = [_vp, _vp, _u64, _u64, _vp, _vp, _vp]
_lib.s3gd_randk_sign_encode.restype = _int
_lib.s3gd_randk_sign_encode.argtypes = [_vp, _vp, _u32, _u64, _u64, _u64, _u32, _vp, _vp, _vp]
_lib.s3gd_step_randk.restype = _int
_lib.s3gd_step_randk.argtypes = [_vp, _vp, _u32, _u64, _u64, _u64, _u32, _vp, _f32, _vp, _vp, _vp, _vp, _vp]
_lib.s3gd_last_async_status.restype = _int
_lib.s3gd_last_async_status.argtypes = [_vp, _vp]
_lib.s3gd_last_encode_info.restype = _int
_lib.s3gd_last_encode_info.argtypes = [_vp, _vp, ctypes.POINTER(_u32)]
_lib.s3gd_last_hip_error.restype = _int
_lib.s3gd_last_hip_error.argtypes = [_vp]
_lib.s3gd_strerror.restype = ctypes.c_char_p
_lib.s3gd_strerror.argtypes = [_int]

_lib.s3gd_last_row_state.restype = _int
_lib.s3gd_last_row_state.argtypes = [_vp, _vp, _u32, ctypes.POINTER(_u32)]
_lib.s3gd_calibrate_read.restype = _int
_lib.s3gd_calibrate_read.argtypes = [_vp, _vp, _u64, _vp]
_lib.s3gd_calibrate_rmw.restype = _int
_lib.s3gd_calibrate_rmw.argtypes = [_vp, _vp, _vp, _u64, _vp]
_lib.s3gd_encode_plan_info.restype = _int
_lib.s3gd_encode_plan_info.argtypes = [_vp, _u32, _u64, _u64, _int, ctypes.POINTER(_u64)]
_lib.s3gd_encode_sample_unit_start.restype = _u64
_lib.s3gd_encode_sample_unit_start.argtypes = [_u32, _u64]
_lib.s3gd_profile_enable.restype = _int
_lib.s3gd_profile_enable.argtypes = [_vp, _int]
_lib.s3gd_profile_read.restype = _int
_lib.s3gd_profile_read.argtypes = [_vp, _vp, ctypes.POINTER(_f32), ctypes.POINTER(_u32), _int]
_lib.s3gd_profile_kernel_name.restype = ctypes.c_char_p
_lib.s3gd_profile_kernel_name.argtypes = [_int]

raw = _lib  # for tests that call the C ABI with hand-made arguments


class S3GDError(RuntimeError):
    def __init__(self, code: int, where: str, hip: int = 0):
        self.code = code
        msg = _lib.s3gd_strerror(code).decode()
        super().__init__(f"{where}: {msg} (code {code}" + (f", hipError {hip})" if hip else ")"))


def strerror(code: int) -> str:
    return _lib.s3gd_strerror(code).decode()


def workspace_bytes(M_max: int, N_max: int, K_max: int) -> int:
    return int(_lib.s3gd_workspace_bytes(M_max, N_max, K_max))


def encode_sample_unit_start(u: int, unit_stride: int) -> int:
    return int(_lib.s3gd_encode_sample_unit_start(u, unit_stride))


def packed_row_words(N: int, K: int) -> int:
    """32-bit words (an even number) that hold the packed form of any message of at most K entries."""
    return int(_lib.s3gd_packed_row_words(N, K))


def _ptr(t: torch.Tensor | None) -> int | None:
    return None if t is None else t.data_ptr()


def _stream(stream) -> int | None:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream or None


def step_static(grads: torch.Tensor, K: int, x: torch.Tensor, lr: float, words: torch.Tensor, counts: torch.Tensor,
                tally: torch.Tensor | None = None, votes: torch.Tensor | None = None, nan_flag: torch.Tensor | None = None,
                stream=None) -> int:
    """s3gd_step on the library's static scratch array: no context, nothing allocated.  Returns the C return code."""
    M, N = grads.shape
    return int(_lib.s3gd_step_static(grads.device.index or 0, _ptr(grads), M, N, K, _ptr(x), float(lr), _ptr(words), _ptr(counts),
                                     _ptr(tally), _ptr(votes), _ptr(nan_flag), _stream(stream)))


class Context:
    """Owns the library's scratch memory for problems up to (M_max, N_max, K_max)."""

    def __init__(self, M_max: int, N_max: int, K_max: int, device: int = 0):
        self._h = _vp()
        self.device = device
        rc = _lib.s3gd_create(ctypes.byref(self._h), device, M_max, N_max, K_max)
        if rc:
            self._h = None
            raise S3GDError(rc, "s3gd_create")

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:  # _lib is None while the interpreter shuts down
            _lib.s3gd_destroy(self._h)
            self._h = None

    __del__ = close

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def _check(self, rc: int, where: str):
        if rc:
            raise S3GDError(rc, where, _lib.s3gd_last_hip_error(self._h))

    # -- the three calls of the paper's problem statement ------------------------------------
    def topk_sign_encode(self, grads: torch.Tensor, K: int, words: torch.Tensor | None = None,
                         counts: torch.Tensor | None = None, stream=None):
        """words[M,K], counts[M] (int32 storage holding uint32 values) = TopKSign of every row."""
        M, N = grads.shape
        if words is None:
            words = torch.empty((M, K), dtype=torch.int32, device=grads.device)
        if counts is None:
            counts = torch.empty((M,), dtype=torch.int32, device=grads.device)
        self._check(_lib.s3gd_topk_sign_encode(self._h, _ptr(grads), M, N, K, _ptr(words), _ptr(counts), _stream(stream)),
                    "s3gd_topk_sign_encode")
        return words, counts

    def majority_vote(self, words: torch.Tensor, counts: torch.Tensor, N: int, tally: torch.Tensor | None = None,
                      votes: torch.Tensor | None = None, stream=None):
        M, K = words.shape
        self._check(_lib.s3gd_majority_vote(self._h, _ptr(words), _ptr(counts), M, N, K, _ptr(tally), _ptr(votes),
                                            _stream(stream)), "s3gd_majority_vote")
        return tally, votes

    def apply_update(self, x: torch.Tensor, votes: torch.Tensor, lr: float, stream=None):
        self._check(_lib.s3gd_apply_update(self._h, _ptr(x), _ptr(votes), float(lr), x.numel(), _stream(stream)),
                    "s3gd_apply_update")
        return x

    def step(self, grads: torch.Tensor, K: int, x: torch.Tensor, lr: float, words: torch.Tensor, counts: torch.Tensor,
             tally: torch.Tensor | None = None, votes: torch.Tensor | None = None, stream=None):
        M, N = grads.shape
        self._check(_lib.s3gd_step(self._h, _ptr(grads), M, N, K, _ptr(x), float(lr), _ptr(words), _ptr(counts),
                                   _ptr(tally), _ptr(votes), _stream(stream)), "s3gd_step")
        return x

    # -- the same with the error-compensation memory ------------------------------------------
    def topk_sign_encode_ec(self, grads: torch.Tensor, err: torch.Tensor, eta: float, K: int,
                            words: torch.Tensor | None = None, counts: torch.Tensor | None = None, stream=None):
        """Encodes g = grads + eta * err and leaves the new memory g - TopK(g) in err."""
        M, N = grads.shape
        if words is None:
            words = torch.empty((M, K), dtype=torch.int32, device=grads.device)
        if counts is None:
            counts = torch.empty((M,), dtype=torch.int32, device=grads.device)
        self._check(_lib.s3gd_topk_sign_encode_ec(self._h, _ptr(grads), _ptr(err), float(eta), M, N, K, _ptr(words),
                                                  _ptr(counts), _stream(stream)), "s3gd_topk_sign_encode_ec")
        return words, counts

    def step_ec(self, grads: torch.Tensor, err: torch.Tensor, eta: float, K: int, x: torch.Tensor, lr: float,
                words: torch.Tensor, counts: torch.Tensor, tally: torch.Tensor | None = None,
                votes: torch.Tensor | None = None, stream=None):
        M, N = grads.shape
        self._check(_lib.s3gd_step_ec(self._h, _ptr(grads), _ptr(err), float(eta), M, N, K, _ptr(x), float(lr),
                                      _ptr(words), _ptr(counts), _ptr(tally), _ptr(votes), _stream(stream)), "s3gd_step_ec")
        return x

    def topk_sign_encode_acc(self, acc: torch.Tensor, K: int, words: torch.Tensor | None = None,
                             counts: torch.Tensor | None = None, stream=None):
        """The encode when g = g~ + e already sits in the memory buffer `acc`; on return acc is the new memory."""
        M, N = acc.shape
        if words is None:
            words = torch.empty((M, K), dtype=torch.int32, device=acc.device)
        if counts is None:
            counts = torch.empty((M,), dtype=torch.int32, device=acc.device)
        self._check(_lib.s3gd_topk_sign_encode_acc(self._h, _ptr(acc), M, N, K, _ptr(words), _ptr(counts), _stream(stream)),
                    "s3gd_topk_sign_encode_acc")
        return words, counts

    def step_acc(self, acc: torch.Tensor, K: int, x: torch.Tensor, lr: float, words: torch.Tensor, counts: torch.Tensor,
                 tally: torch.Tensor | None = None, votes: torch.Tensor | None = None, stream=None):
        M, N = acc.shape
        self._check(_lib.s3gd_step_acc(self._h, _ptr(acc), M, N, K, _ptr(x), float(lr), _ptr(words), _ptr(counts),
                                       _ptr(tally), _ptr(votes), _stream(stream)), "s3gd_step_acc")
        return x

    # -- momentum form of the update -----------------------------------------------------------
    def apply_update_momentum(self, x: torch.Tensor, v: torch.Tensor, votes: torch.Tensor, lr: float, mu: float, stream=None):
        self._check(_lib.s3gd_apply_update_momentum(self._h, _ptr(x), _ptr(v), _ptr(votes), float(lr), float(mu), x.numel(),
                                                    _stream(stream)), "s3gd_apply_update_momentum")
        return x, v

    def step_momentum(self, grads: torch.Tensor, K: int, x: torch.Tensor, v: torch.Tensor, lr: float, mu: float,
                      words: torch.Tensor, counts: torch.Tensor, err: torch.Tensor | None = None, eta: float = 1.0, stream=None):
        M, N = (grads if grads is not None else err).shape
        self._check(_lib.s3gd_step_momentum(self._h, _ptr(grads), _ptr(err), float(eta), M, N, K, _ptr(x), _ptr(v), float(lr),
                                            float(mu), _ptr(words), _ptr(counts), _stream(stream)), "s3gd_step_momentum")
        return x, v

    # -- Algorithm 2: random-K instead of top-K ------------------------------------------------
    def randk_sign_encode(self, grads: torch.Tensor, K: int, seed: int, t: int, words: torch.Tensor | None = None,
                          counts: torch.Tensor | None = None, stream=None):
        M, N = grads.shape
        if words is None:
            words = torch.empty((M, K), dtype=torch.int32, device=grads.device)
        if counts is None:
            counts = torch.empty((M,), dtype=torch.int32, device=grads.device)
        self._check(_lib.s3gd_randk_sign_encode(self._h, _ptr(grads), M, N, K, seed, t, _ptr(words), _ptr(counts),
                                                _stream(stream)), "s3gd_randk_sign_encode")
        return words, counts

    def step_randk(self, grads: torch.Tensor, K: int, seed: int, t: int, x: torch.Tensor, lr: float, words: torch.Tensor,
                   counts: torch.Tensor, tally: torch.Tensor | None = None, votes: torch.Tensor | None = None, stream=None):
        M, N = grads.shape
        self._check(_lib.s3gd_step_randk(self._h, _ptr(grads), M, N, K, seed, t, _ptr(x), float(lr), _ptr(words),
                                         _ptr(counts), _ptr(tally), _ptr(votes), _stream(stream)), "s3gd_step_randk")
        return x

    # -- messages that are already there, and the compact wire format -------------------------------
    def vote_update(self, words: torch.Tensor, counts: torch.Tensor, N: int, x: torch.Tensor, lr: float, stream=None):
        M, K = words.shape
        self._check(_lib.s3gd_vote_update(self._h, _ptr(words), _ptr(counts), M, N, K, _ptr(x), float(lr), _stream(stream)),
                    "s3gd_vote_update")
        return x

    def pack_messages(self, words: torch.Tensor, counts: torch.Tensor, N: int, packed: torch.Tensor | None = None, stream=None):
        M, K = words.shape
        if packed is None:
            packed = torch.empty((M, packed_row_words(N, K)), dtype=torch.int32, device=words.device)
        self._check(_lib.s3gd_pack_messages(self._h, _ptr(words), _ptr(counts), M, N, K, _ptr(packed), packed.shape[1],
                                            _stream(stream)), "s3gd_pack_messages")
        return packed

    def unpack_messages(self, packed: torch.Tensor, N: int, K: int, words: torch.Tensor | None = None,
                        counts: torch.Tensor | None = None, stream=None):
        M = packed.shape[0]
        if words is None:
            words = torch.empty((M, K), dtype=torch.int32, device=packed.device)
        if counts is None:
            counts = torch.empty((M,), dtype=torch.int32, device=packed.device)
        self._check(_lib.s3gd_unpack_messages(self._h, _ptr(packed), packed.shape[1], M, N, K, _ptr(words), _ptr(counts),
                                              _stream(stream)), "s3gd_unpack_messages")
        return words, counts

    def votes_to_message(self, votes: torch.Tensor, capacity: int, words: torch.Tensor | None = None,
                         count: torch.Tensor | None = None, stream=None):
        if words is None:
            words = torch.empty((capacity,), dtype=torch.int32, device=votes.device)
        if count is None:
            count = torch.empty((1,), dtype=torch.int32, device=votes.device)
        self._check(_lib.s3gd_votes_to_message(self._h, _ptr(votes), votes.numel(), capacity, _ptr(words), _ptr(count),
                                               _stream(stream)), "s3gd_votes_to_message")
        return words, count

    # -- diagnostics ---------------------------------------------------------------------------
    def last_async_status(self, stream=None) -> int:
        return int(_lib.s3gd_last_async_status(self._h, _stream(stream)))

    def last_encode_info(self, stream=None) -> tuple[int, int]:
        """(rows, rows on the general multi-pass route)."""
        return self.last_encode_details(stream)[:2]

    def last_encode_details(self, stream=None) -> tuple[int, int, int]:
        """(rows, rows on the general route, single-pass rows that needed the full radix select)."""
        return self.last_encode_routes(stream)[:3]

    def last_encode_routes(self, stream=None) -> tuple[int, int, int, int, int]:
        """The five counters of s3gd_last_encode_info: rows, general route, wide radix select, row passes with a
        known threshold, general rows that skipped the single pass."""
        out = (_u32 * 5)()
        self._check(_lib.s3gd_last_encode_info(self._h, _stream(stream), out), "s3gd_last_encode_info")
        return tuple(int(v) for v in out)

    def last_row_state(self, m: int, stream=None) -> dict[str, int]:
        out = (_u32 * 16)()
        self._check(_lib.s3gd_last_row_state(self._h, _stream(stream), m, out), "s3gd_last_row_state")
        names = ("prefix", "k_rem", "T", "q", "c_gt", "count", "mode", "L", "U", "row_emit", "n_cand", "n_brk")
        return {k: int(v) for k, v in zip(names, out)}

    def calibrate_read(self, buf: torch.Tensor, stream=None):
        """A plain read of `buf` (fp32) with the selection pass's launch shape; timed through the profile."""
        self._check(_lib.s3gd_calibrate_read(self._h, _ptr(buf), buf.numel(), _stream(stream)), "s3gd_calibrate_read")

    def calibrate_rmw(self, a: torch.Tensor, b: torch.Tensor, stream=None):
        """b <- a + b (fp32) with the launch shape of the selection pass with a memory; timed through the profile."""
        if a.numel() != b.numel():
            raise ValueError("calibrate_rmw: a and b differ in size")
        self._check(_lib.s3gd_calibrate_rmw(self._h, _ptr(a), _ptr(b), a.numel(), _stream(stream)), "s3gd_calibrate_rmw")

    def encode_plan_info(self, M: int, N: int, K: int, with_memory: bool = False) -> dict[str, int]:
        """How an encode of this shape is laid over the device (see s3gd_encode_plan_info)."""
        out = (_u64 * 12)()
        self._check(_lib.s3gd_encode_plan_info(self._h, M, N, K, int(with_memory), out), "s3gd_encode_plan_info")
        names = ("candidates", "chunks", "record_shift", "blocks_per_row", "tiles_per_wave", "slab", "cand_stride", "n_units",
                 "unit_stride", "sample_rank", "chain", "sample_unit")
        info = {k: int(v) for k, v in zip(names, out)}
        info["zero_sure"] = info["chunks"] >> 1
        info["chunks"] &= 1
        return info

    def profile_enable(self, on: bool | int = True):
        """True / 1: time every kernel; 2: only the passes over the gradients; False / 0: off."""
        self._check(_lib.s3gd_profile_enable(self._h, int(on)), "s3gd_profile_enable")

    def profile_read(self, stream=None) -> dict[str, tuple[float, int]]:
        """{kernel name: (summed milliseconds, launches)} since the last read."""
        ms = (_f32 * PROFILE_KERNELS)()
        cnt = (_u32 * PROFILE_KERNELS)()
        self._check(_lib.s3gd_profile_read(self._h, _stream(stream), ms, cnt, PROFILE_KERNELS), "s3gd_profile_read")
        return {_lib.s3gd_profile_kernel_name(i).decode(): (float(ms[i]), int(cnt[i]))
                for i in range(PROFILE_KERNELS) if cnt[i]}
