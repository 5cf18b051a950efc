"""The C-ABI library: it loads, exports every symbol the header declares, and rejects bad
arguments before touching the GPU (these tests run on a machine without one)."""
import ctypes as C
import os
import re

import numpy as np
import pytest
import torch

from paper_2312_07743_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "w2v.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(w2v_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = _declared()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None


def test_struct_layout_matches_the_header():
    # compile a two-line C program against the header and compare sizeof/offsetof with the ctypes mirror
    import subprocess, tempfile
    fields = [f[0] for f in B.W2VConfig._fields_]
    prog = '#include <stdio.h>\n#include <stddef.h>\n#include "w2v.h"\nint main(void){printf("%zu", sizeof(w2v_config));' + \
        "".join(f'printf(" %zu", offsetof(w2v_config, {f}));' for f in fields) + "return 0;}"
    with tempfile.TemporaryDirectory() as d:
        src = os.path.join(d, "t.c")
        open(src, "w").write(prog)
        subprocess.check_call(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), src, "-o", os.path.join(d, "t")])
        out = subprocess.check_output([os.path.join(d, "t")]).decode().split()
    assert int(out[0]) == C.sizeof(B.W2VConfig)
    assert [int(x) for x in out[1:]] == [getattr(B.W2VConfig, f).offset for f in fields]


def test_query_ld_and_workspace():
    assert B.w2v_query_ld(128) == 128 and B.w2v_query_ld(300) == 320 and B.w2v_query_ld(1) == 32
    with pytest.raises(B.W2VError):
        B.w2v_query_ld(0)
    with pytest.raises(B.W2VError):
        B.w2v_query_ld(513)
    small, big = B.w2v_query_workspace(1000, 1 << 10), B.w2v_query_workspace(1000, 1 << 20)
    assert big - small >= 4 * ((1 << 20) - (1 << 10)) and small % 256 == 0
    with pytest.raises(B.W2VError):
        B.w2v_query_workspace(1000, 0)
    # summed lock-free updates keep a snapshot of (2W+2) ring rows for each of up to 4,096 wavefronts
    auto = B.w2v_query_workspace(1000, 1 << 10, dim=128, window=10, negatives=5, update_mode=0)
    assert auto - small == 4096 * 22 * 128 * 4
    assert B.w2v_query_workspace(1000, 1 << 10, dim=128, window=10, negatives=5, window_mode=1, update_mode=2) - small == 4096 * 12 * 128 * 4
    # no such kernel for rows of more than 256 floats or fewer than 5 negatives: no snapshot space
    assert B.w2v_query_workspace(1000, 1 << 10, dim=300, window=5, negatives=10, update_mode=0) == small
    assert B.w2v_query_workspace(1000, 1 << 10, dim=128, window=5, negatives=2, update_mode=0) == small


def _good_cfg(**over):
    kw = dict(vocab=100, dim=128, window=5, negatives=5, tokens_per_epoch=1000, seed=1, syn0=0x1000, syn1neg=0x2000,
              ld=128, workspace=0x10000, workspace_bytes=1 << 30)
    kw.update(over)
    return B.make_config(**kw)


@pytest.mark.parametrize("over", [
    dict(vocab=0), dict(vocab=(1 << 27) + 1), dict(dim=0), dict(dim=513), dict(window=0), dict(window=17),
    dict(negatives=21), dict(window_mode=2), dict(negative_block=3), dict(negative_block=128), dict(update_mode=3),
    dict(update_mode=2, dim=300, ld=320), dict(update_mode=2, negatives=3), dict(update_mode=2, window=11),
    dict(storage=2), dict(storage=1, update_mode=2), dict(storage=1, dim=512, ld=512), dict(storage=1, negatives=2),
    dict(storage=1, window=11), dict(storage=1, dim=130, ld=160),
    dict(total_epochs=0), dict(tokens_per_epoch=0), dict(lr0=0.0),
    dict(lr0=float("nan")), dict(lr_min_frac=1.5), dict(subsample_t=-1.0), dict(syn0=None), dict(syn1neg=None),
    dict(ld=127), dict(ld=64), dict(ld=130), dict(workspace=None), dict(workspace=0x10001), dict(device=-1),
    dict(dim=512, ld=512, window=11), dict(dim=321, ld=352, window=11),
])
def test_create_rejects_bad_config_without_touching_the_gpu(over):
    ctx = C.c_void_p(None)
    rc = B.lib().w2v_create(C.byref(_good_cfg(**over)), 1, C.byref(ctx))
    assert rc == B.W2V_EINVAL and not ctx.value
    assert len(B.w2v_last_error(None)) > 0


def test_create_rejects_wrong_struct_size_null_and_small_workspace():
    ctx = C.c_void_p(None)
    cfg = _good_cfg()
    cfg.struct_size -= 8
    assert B.lib().w2v_create(C.byref(cfg), 1, C.byref(ctx)) == B.W2V_EINVAL
    assert B.lib().w2v_create(None, 1, C.byref(ctx)) == B.W2V_EINVAL
    assert B.lib().w2v_create(C.byref(_good_cfg()), 1, None) == B.W2V_EINVAL
    assert B.lib().w2v_create(C.byref(_good_cfg(workspace_bytes=16)), 1, C.byref(ctx)) == B.W2V_ENOMEM


def test_null_context_is_an_error_everywhere():
    L = B.lib()
    assert L.w2v_destroy(None) == B.W2V_EINVAL
    assert L.w2v_build_unigram_table(None, None, 16) == B.W2V_EINVAL
    assert L.w2v_train_epoch(None, None, None, 1, 0, 0) == B.W2V_EINVAL
    assert L.w2v_train_epoch_naive(None, None, None, 1, 0, 0) == B.W2V_EINVAL
    assert L.w2v_train_epoch_static(None, None, None, 1, 0, 0, None, None) == B.W2V_EINVAL
    assert L.w2v_get_embeddings(None, 0, None, 0, 0) == B.W2V_EINVAL
    assert L.w2v_loss(None, None, None, 0) == B.W2V_EINVAL
    assert L.w2v_counters(None, None, None, 0) == B.W2V_EINVAL
    assert L.w2v_debug_draws(None, None, None, 1, 0, 0, None, None, None) == B.W2V_EINVAL
    assert L.w2v_debug_reduce(None, None, None) == B.W2V_EINVAL
    assert L.w2v_debug_set_units(None, 0) == B.W2V_EINVAL
    assert L.w2v_debug_train_draws(None, None, None, 1, 0, 0, None, None, None) == B.W2V_EINVAL
    assert L.w2v_debug_set_update(None, 0) == B.W2V_EINVAL
    assert L.w2v_debug_get_plan(None, None, None, None, None, None, None) == B.W2V_EINVAL
    assert L.w2v_debug_set_unit_tail(None, 0, 0) == B.W2V_EINVAL
    assert L.w2v_train_epoch_host(None, None, None, 1, 0, 0, None, 0) == B.W2V_EINVAL


@pytest.mark.skipif(torch.cuda.is_available(), reason="checks the no-GPU error path")
def test_without_a_gpu_create_fails_loudly_not_silently():
    ctx = C.c_void_p(None)
    rc = B.lib().w2v_create(C.byref(_good_cfg()), 1, C.byref(ctx))
    assert rc == B.W2V_EHIP and not ctx.value
    from paper_2312_07743_amd.trainer import Trainer
    with pytest.raises(RuntimeError):
        Trainer(vocab=10, dim=8, window=2, negatives=2, counts=np.ones(10, np.uint64), tokens_per_epoch=10, seed=1)
