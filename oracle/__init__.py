"""CPU oracle for the SGNS training path -- TEST INFRASTRUCTURE ONLY.

ctypes front end of sgns_oracle.c.  Nothing in the product package may import
this module; only tests, the smoke check and the benchmark's cpu_baseline leg do.
"""
import ctypes as C

import numpy as np

from . import build as _build

_u64p = np.ctypeslib.ndpointer(np.uint64, flags="C_CONTIGUOUS")
_u32p = np.ctypeslib.ndpointer(np.uint32, flags="C_CONTIGUOUS")
_i32p = np.ctypeslib.ndpointer(np.int32, flags="C_CONTIGUOUS")
_u8p = np.ctypeslib.ndpointer(np.uint8, flags="C_CONTIGUOUS")


class Params(C.Structure):
    _fields_ = [("vocab", C.c_uint32), ("dim", C.c_uint32), ("window", C.c_uint32),
                ("negatives", C.c_uint32), ("window_mode", C.c_uint32), ("update_mode", C.c_uint32),
                ("total_epochs", C.c_uint32), ("epoch", C.c_uint32),
                ("tokens_per_epoch", C.c_uint64), ("first_token_global_pos", C.c_uint64),
                ("seed", C.c_uint64), ("table_size", C.c_uint64),
                ("lr0", C.c_double), ("lr_min_frac", C.c_double),
                ("negative_block", C.c_uint32), ("storage", C.c_uint32)]


class Oracle:
    """One precision of the oracle: real='float' (what the GPU is compared with) or 'double'."""

    def __init__(self, real: str = "float"):
        _build.build()
        self.real = np.float32 if real == "float" else np.float64
        L = C.CDLL(_build.lib_path(real))
        self.L = L
        rp = np.ctypeslib.ndpointer(self.real, flags="C_CONTIGUOUS")
        creal = C.c_float if real == "float" else C.c_double
        L.orc_mix64.restype = C.c_uint64
        L.orc_mix64.argtypes = [C.c_uint64]
        L.orc_draw.restype = C.c_uint64
        L.orc_draw.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32]
        L.orc_table_ends.restype = C.c_int
        L.orc_table_ends.argtypes = [_u64p, C.c_uint32, C.c_uint64, _u64p]
        L.orc_word_of_slot.restype = C.c_int32
        L.orc_word_of_slot.argtypes = [_u64p, C.c_uint32, C.c_uint64]
        L.orc_negative.restype = C.c_int32
        L.orc_negative.argtypes = [_u64p, C.c_uint32, C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32]
        L.orc_thresholds.restype = None
        L.orc_thresholds.argtypes = [_u64p, C.c_uint32, C.c_double, _u32p]
        L.orc_keep.restype = C.c_int
        L.orc_keep.argtypes = [_u32p, C.c_int32, C.c_uint64, C.c_uint32, C.c_uint64]
        L.orc_width.restype = C.c_uint32
        L.orc_width.argtypes = [C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint64]
        L.orc_lr.restype = C.c_float
        L.orc_lr.argtypes = [C.c_double, C.c_double, C.c_uint32, C.c_uint32, C.c_uint64, C.c_uint64]
        L.orc_init_weights.restype = None
        L.orc_init_weights.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, rp, rp]
        for name in ("orc_window_step", "orc_window_step_immediate", "orc_window_step_pairwise"):
            f = getattr(L, name)
            f.restype = None
            f.argtypes = [rp, rp, C.c_uint32, _i32p, C.c_uint32, _i32p, C.c_uint32, creal,
                          C.POINTER(C.c_double)]
        L.orc_train_range.restype = C.c_int
        L.orc_train_range.argtypes = [C.POINTER(Params), rp, rp, _u64p, _u32p, _i32p, _u64p,
                                      C.c_uint64, C.c_uint64, C.c_uint64,
                                      C.POINTER(C.c_double), C.POINTER(C.c_uint64),
                                      C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_round_bits.restype = C.c_uint32
        L.orc_round_bits.argtypes = [C.c_uint64, C.c_uint32, C.c_uint64, C.c_uint32, C.c_uint32]
        L.orc_to_bf16.restype = C.c_float
        L.orc_to_bf16.argtypes = [C.c_float, C.c_uint32, C.c_uint32]
        L.orc_real_size.restype = C.c_uint32
        assert L.orc_real_size() == np.dtype(self.real).itemsize

    # ---- scalar pieces -------------------------------------------------
    def mix64(self, z):
        return int(self.L.orc_mix64(z & 0xFFFFFFFFFFFFFFFF))

    def draw(self, seed, epoch, pos, j):
        return int(self.L.orc_draw(seed & 0xFFFFFFFFFFFFFFFF, epoch, pos, j))

    def table_ends(self, counts, table_size):
        counts = np.ascontiguousarray(counts, np.uint64)
        end = np.zeros(len(counts), np.uint64)
        if self.L.orc_table_ends(counts, len(counts), table_size, end) != 0:
            raise ValueError("all counts are zero")
        return end

    def word_of_slot(self, end, slot):
        return int(self.L.orc_word_of_slot(end, len(end), slot))

    def negative(self, end, table_size, seed, epoch, pos, k):
        return int(self.L.orc_negative(end, len(end), table_size, seed, epoch, pos, k))

    def thresholds(self, counts, t):
        counts = np.ascontiguousarray(counts, np.uint64)
        thr = np.zeros(len(counts), np.uint32)
        self.L.orc_thresholds(counts, len(counts), float(t), thr)
        return thr

    def keep(self, thr, w, seed, epoch, pos):
        return bool(self.L.orc_keep(thr, w, seed, epoch, pos))

    def width(self, W, mode, seed, epoch, pos):
        return int(self.L.orc_width(W, mode, seed, epoch, pos))

    def lr(self, lr0, lr_min_frac, epoch, total_epochs, tokens_per_epoch, sentence_start):
        return float(self.L.orc_lr(lr0, lr_min_frac, epoch, total_epochs, tokens_per_epoch, sentence_start))

    def init_weights(self, seed, V, d, storage=0):
        """storage != 0: the initial values rounded to the nearest bfloat16 (ties to even)."""
        syn0 = np.zeros((V, d), self.real)
        syn1 = np.zeros((V, d), self.real)
        self.L.orc_init_weights(seed, V, d, syn0, syn1)
        if storage:
            syn0[...] = self.nearest_bf16(syn0)
        return syn0, syn1

    def nearest_bf16(self, x):
        """Array version of to_bf16(x, 2, 0) (round to nearest bfloat16, ties to even; finite inputs)."""
        b = np.ascontiguousarray(x, np.float32).view(np.uint32).astype(np.uint64)
        b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
        return b.astype(np.uint32).view(np.float32).astype(self.real).reshape(np.shape(x))

    def round_bits(self, seed, epoch, pos, tag, e):
        return int(self.L.orc_round_bits(seed & 0xFFFFFFFFFFFFFFFF, epoch, pos, tag, e))

    def to_bf16(self, x, mode, bits16):
        return float(self.L.orc_to_bf16(x, mode, bits16))

    # ---- one window ----------------------------------------------------
    def window_step(self, syn0, syn1neg, ctx, out, alpha, immediate=False, pairwise=False):
        """In-place update of syn0/syn1neg by one window; returns the window's loss sum."""
        assert syn0.dtype == self.real and syn1neg.dtype == self.real
        ctx = np.ascontiguousarray(ctx, np.int32)
        out = np.ascontiguousarray(out, np.int32)
        loss = C.c_double(0.0)
        f = self.L.orc_window_step_immediate if immediate else self.L.orc_window_step
        if pairwise:
            f = self.L.orc_window_step_pairwise
        f(syn0, syn1neg, syn0.shape[1], ctx, len(ctx), out, len(out), alpha, C.byref(loss))
        return loss.value

    # ---- one epoch -----------------------------------------------------
    def train_epoch(self, syn0, syn1neg, counts, tokens, sent_off, *, window, negatives,
                    seed, epoch=0, total_epochs=1, tokens_per_epoch=None, first_token_global_pos=0,
                    table_size=1 << 24, lr0=0.025, lr_min_frac=1e-4, subsample_t=0.0,
                    window_mode=0, update_mode=0, dump=False, s_begin=0, s_end=None, s_stride=1,
                    negative_block=0, storage=0):
        """Serial SGNS over sentences [s_begin, s_end) with the given stride, in place.
        Returns dict(loss_sum, pairs[, keep, width, neg])."""
        assert syn0.dtype == self.real and syn1neg.dtype == self.real
        V, d = syn0.shape
        tokens = np.ascontiguousarray(tokens, np.int32)
        sent_off = np.ascontiguousarray(sent_off, np.uint64)
        n_sent = len(sent_off) - 1
        if s_end is None:
            s_end = n_sent
        T = len(tokens)
        P = Params(V, d, window, negatives, window_mode, update_mode, total_epochs, epoch,
                   T if tokens_per_epoch is None else tokens_per_epoch, first_token_global_pos,
                   seed, table_size, lr0, lr_min_frac, negative_block, storage)
        end = self.table_ends(counts, table_size)
        thr = self.thresholds(counts, subsample_t)
        loss = C.c_double(0.0)
        pairs = C.c_uint64(0)
        keep = width = neg = None
        kp = wp = npp = None
        if dump:
            keep = np.zeros(T, np.uint8)
            width = np.zeros(T, np.uint8)
            neg = np.full((T, max(negatives, 1)), -1, np.int32)[:, :negatives].copy()
            kp, wp, npp = keep.ctypes.data, width.ctypes.data, neg.ctypes.data
        rc = self.L.orc_train_range(C.byref(P), syn0, syn1neg, end, thr, tokens, sent_off,
                                    s_begin, s_end, s_stride, C.byref(loss), C.byref(pairs),
                                    kp, wp, npp)
        if rc != 0:
            raise ValueError("oracle: window/negatives out of range")
        res = {"loss_sum": loss.value, "pairs": pairs.value}
        if dump:
            res.update(keep=keep, width=width, neg=neg)
        return res
