"""Thin ctypes binding of libw2v.so (include/w2v.h).  Argument marshalling only: every step of the
training path runs in the library's HIP kernels.  torch is used for device buffers and streams.

The functions carry the C names (w2v_create, w2v_build_unigram_table, w2v_train_epoch,
w2v_get_embeddings, w2v_loss, ...).  There is no CPU fallback: if the library is missing the
import of this module's `lib()` raises.
"""
import ctypes as C
import os

import numpy as np

W2V_OK, W2V_EINVAL, W2V_ESTATE, W2V_ENOMEM, W2V_EHIP = 0, -1, -2, -3, -4
_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libw2v.so")
EXPORTS = ["w2v_query_ld", "w2v_query_workspace", "w2v_create", "w2v_destroy", "w2v_build_unigram_table",
           "w2v_train_epoch", "w2v_train_epoch_static", "w2v_train_epoch_host", "w2v_train_epoch_naive", "w2v_get_embeddings", "w2v_loss", "w2v_counters", "w2v_debug_draws",
           "w2v_debug_train_draws", "w2v_debug_set_update", "w2v_debug_get_plan",
           "w2v_debug_set_units", "w2v_debug_set_unit_tail", "w2v_debug_reduce", "w2v_last_error"]


class W2VConfig(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("vocab", C.c_uint32), ("dim", C.c_uint32), ("window", C.c_uint32),
                ("negatives", C.c_uint32), ("window_mode", C.c_uint32), ("total_epochs", C.c_uint32),
                ("sentences_in_flight", C.c_uint32), ("tokens_per_epoch", C.c_uint64), ("seed", C.c_uint64),
                ("lr0", C.c_double), ("lr_min_frac", C.c_double), ("subsample_t", C.c_double),
                ("syn0", C.c_void_p), ("syn1neg", C.c_void_p), ("ld", C.c_uint32), ("device", C.c_int32),
                ("stream", C.c_void_p), ("workspace", C.c_void_p), ("workspace_bytes", C.c_uint64),
                ("negative_block", C.c_uint32), ("update_mode", C.c_uint32), ("storage", C.c_uint32), ("reserved", C.c_uint32)]


class W2VError(RuntimeError):
    def __init__(self, code, text):
        super().__init__(f"w2v error {code}: {text}")
        self.code = code


_lib = None


def lib():
    """The loaded library; built beforehand by paper_2312_07743_amd/build.py."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2312_07743_amd.build` "
                               "(there is no fallback implementation)")
        L = C.CDLL(LIB_PATH)
        vp, u32, u64, i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int
        L.w2v_query_ld.argtypes = [u32, C.POINTER(u32)]
        L.w2v_query_workspace.argtypes = [C.POINTER(W2VConfig), u32, C.POINTER(u64)]
        L.w2v_create.argtypes = [C.POINTER(W2VConfig), i32, C.POINTER(vp)]
        L.w2v_destroy.argtypes = [vp]
        L.w2v_build_unigram_table.argtypes = [vp, vp, u32]
        L.w2v_train_epoch.argtypes = [vp, vp, vp, u64, u64, u32]
        L.w2v_train_epoch_static.argtypes = [vp, vp, vp, u64, u64, u32, vp, vp]
        L.w2v_train_epoch_naive.argtypes = [vp, vp, vp, u64, u64, u32]
        L.w2v_train_epoch_host.argtypes = [vp, vp, vp, u64, u64, u32, vp, u64]
        L.w2v_get_embeddings.argtypes = [vp, i32, vp, u64, i32]
        L.w2v_loss.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(u64), i32]
        L.w2v_counters.argtypes = [vp, C.POINTER(u64), C.POINTER(u64), i32]
        L.w2v_debug_draws.argtypes = [vp, vp, vp, u64, u64, u32, vp, vp, vp]
        L.w2v_debug_train_draws.argtypes = [vp, vp, vp, u64, u64, u32, vp, vp, vp]
        L.w2v_debug_set_update.argtypes = [vp, i32]
        L.w2v_debug_get_plan.argtypes = [vp, C.POINTER(u32), C.POINTER(u32), C.POINTER(u64), C.POINTER(u64), C.POINTER(u32),
                                         C.POINTER(u64)]
        L.w2v_debug_reduce.argtypes = [vp, vp, vp]
        L.w2v_debug_set_units.argtypes = [vp, i32]
        L.w2v_debug_set_unit_tail.argtypes = [vp, i32, u64]
        L.w2v_last_error.argtypes = [vp]
        L.w2v_last_error.restype = C.c_char_p
        for n in EXPORTS:
            if n != "w2v_last_error":
                getattr(L, n).restype = C.c_int
        _lib = L
    return _lib


def _ptr(x):
    """Device or host address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return x.data_ptr()


def _check(rc, ctx=None):
    if rc != W2V_OK:
        raise W2VError(rc, (lib().w2v_last_error(ctx) or b"").decode())


def w2v_last_error(ctx=None):
    return (lib().w2v_last_error(ctx) or b"").decode()


def w2v_query_ld(dim):
    out = C.c_uint32(0)
    _check(lib().w2v_query_ld(dim, C.byref(out)))
    return out.value


def w2v_query_workspace(vocab, table_size, dim=0, window=0, negatives=0, window_mode=0, update_mode=1):
    """update_mode 1 (overwrite) needs no snapshot space and no dim / window / negatives."""
    cfg = W2VConfig(struct_size=C.sizeof(W2VConfig), vocab=vocab, dim=dim, window=window, negatives=negatives,
                    window_mode=window_mode, update_mode=update_mode)
    out = C.c_uint64(0)
    _check(lib().w2v_query_workspace(C.byref(cfg), table_size, C.byref(out)))
    return out.value


def make_config(*, vocab, dim, window, negatives, tokens_per_epoch, seed, syn0, syn1neg, ld, workspace,
                workspace_bytes, device=0, stream=None, window_mode=0, total_epochs=1, sentences_in_flight=0,
                lr0=0.025, lr_min_frac=1e-4, subsample_t=0.0, negative_block=0, update_mode=0, storage=0):
    return W2VConfig(struct_size=C.sizeof(W2VConfig), vocab=vocab, dim=dim, window=window, negatives=negatives,
                     window_mode=window_mode, total_epochs=total_epochs, sentences_in_flight=sentences_in_flight,
                     tokens_per_epoch=tokens_per_epoch, seed=seed, lr0=lr0, lr_min_frac=lr_min_frac,
                     subsample_t=subsample_t, syn0=_ptr(syn0), syn1neg=_ptr(syn1neg), ld=ld, device=device,
                     stream=_ptr(stream), workspace=_ptr(workspace), workspace_bytes=workspace_bytes,
                     negative_block=negative_block, update_mode=update_mode, storage=storage, reserved=0)


def w2v_create(cfg, init_weights=1):
    ctx = C.c_void_p(None)
    _check(lib().w2v_create(C.byref(cfg), int(init_weights), C.byref(ctx)))
    return ctx


def w2v_destroy(ctx):
    _check(lib().w2v_destroy(ctx))


def w2v_build_unigram_table(ctx, counts_host, table_size):
    counts = np.ascontiguousarray(counts_host, dtype=np.uint64)
    _check(lib().w2v_build_unigram_table(ctx, counts.ctypes.data, table_size), ctx)


def w2v_train_epoch(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos=0, epoch=0):
    _check(lib().w2v_train_epoch(ctx, _ptr(tokens_dev), _ptr(sent_off_dev), n_sent, first_token_global_pos, epoch), ctx)


def w2v_train_epoch_static(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos, epoch, loss_sum_dev, pairs_dev):
    _check(lib().w2v_train_epoch_static(ctx, _ptr(tokens_dev), _ptr(sent_off_dev), n_sent, first_token_global_pos,
                                        epoch, _ptr(loss_sum_dev), _ptr(pairs_dev)), ctx)


def w2v_train_epoch_host(ctx, tokens_host, sent_off_host, n_sent, first_token_global_pos, epoch, staging_dev,
                         staging_bytes):
    _check(lib().w2v_train_epoch_host(ctx, _ptr(tokens_host), _ptr(sent_off_host), n_sent, first_token_global_pos,
                                      epoch, _ptr(staging_dev), staging_bytes), ctx)


def w2v_train_epoch_naive(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos=0, epoch=0):
    _check(lib().w2v_train_epoch_naive(ctx, _ptr(tokens_dev), _ptr(sent_off_dev), n_sent, first_token_global_pos,
                                       epoch), ctx)


def w2v_debug_set_units(ctx, unit_shift):
    _check(lib().w2v_debug_set_units(ctx, int(unit_shift)), ctx)


def w2v_debug_set_unit_tail(ctx, fine_shift, coarse_sentences):
    _check(lib().w2v_debug_set_unit_tail(ctx, int(fine_shift), int(coarse_sentences)), ctx)


def w2v_get_embeddings(ctx, which, dst, dst_floats, dst_is_device):
    _check(lib().w2v_get_embeddings(ctx, which, _ptr(dst), dst_floats, int(dst_is_device)), ctx)


def w2v_loss(ctx, reset=0):
    s, p = C.c_double(0.0), C.c_uint64(0)
    _check(lib().w2v_loss(ctx, C.byref(s), C.byref(p), int(reset)), ctx)
    return s.value, p.value


def w2v_counters(ctx, reset=0):
    k, d = C.c_uint64(0), C.c_uint64(0)
    _check(lib().w2v_counters(ctx, C.byref(k), C.byref(d), int(reset)), ctx)
    return k.value, d.value


def w2v_debug_draws(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos, epoch, keep_dev, width_dev, neg_dev):
    _check(lib().w2v_debug_draws(ctx, _ptr(tokens_dev), _ptr(sent_off_dev), n_sent, first_token_global_pos, epoch,
                                 _ptr(keep_dev), _ptr(width_dev), _ptr(neg_dev)), ctx)


def w2v_debug_train_draws(ctx, tokens_dev, sent_off_dev, n_sent, first_token_global_pos, epoch, keep_dev, width_dev,
                          neg_dev):
    _check(lib().w2v_debug_train_draws(ctx, _ptr(tokens_dev), _ptr(sent_off_dev), n_sent, first_token_global_pos,
                                       epoch, _ptr(keep_dev), _ptr(width_dev), _ptr(neg_dev)), ctx)


def w2v_debug_set_update(ctx, update):
    _check(lib().w2v_debug_set_update(ctx, int(update)), ctx)


def w2v_debug_get_plan(ctx):
    """dict(unit_shift, fine_shift, coarse_sentences, units, update, wavefronts) of the last launch"""
    us, fs, cs, n, up, wv = C.c_uint32(0), C.c_uint32(0), C.c_uint64(0), C.c_uint64(0), C.c_uint32(0), C.c_uint64(0)
    _check(lib().w2v_debug_get_plan(ctx, C.byref(us), C.byref(fs), C.byref(cs), C.byref(n), C.byref(up), C.byref(wv)), ctx)
    return dict(unit_shift=us.value, fine_shift=fs.value, coarse_sentences=cs.value, units=n.value, update=up.value,
                wavefronts=wv.value)


def w2v_debug_reduce(in_dev, out_dev, stream=None):
    _check(lib().w2v_debug_reduce(_ptr(in_dev), _ptr(out_dev), _ptr(stream)))
