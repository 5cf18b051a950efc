"""Convenience holder of the device buffers one training context needs (torch tensors for memory,
the current torch stream for ordering).  All computation is done by the C-ABI library."""
import numpy as np
import torch

from . import binding as B


_UNCACHED = []          # every uncached device allocation of the process: (pointer, owner of the interface dict)
_UNCACHED_FREE = {}     # (device index, shape) -> tensors handed back by Trainer.close(), reused by later Trainers


def _uncached_zeros(shape, dev):
    """float32 zeros in device memory that the L2 caches do not hold (hipExtMallocWithFlags, hipDeviceMallocUncached),
    as a torch tensor.  Every access then goes to the memory side, which all eight XCDs share, so a wavefront sees
    the rows another XCD has just written.  The allocation is never freed: freeing uncached memory that kernels
    have read has been followed by wrong values in later allocations on this platform.  Trainer.close() returns
    its buffers to a pool instead, and a later Trainer of the same shape takes them from there, so a process that
    builds many Trainers holds as much uncached memory as the most it used at one time."""
    import ctypes as C
    key = (dev.index or 0, tuple(int(x) for x in shape))
    if _UNCACHED_FREE.get(key):
        t = _UNCACHED_FREE[key].pop()
        t.zero_()
        return t
    hip = C.CDLL("libamdhip64.so")
    hip.hipExtMallocWithFlags.argtypes = [C.POINTER(C.c_void_p), C.c_size_t, C.c_uint]
    n = int(np.prod(shape))
    ptr = C.c_void_p()
    with torch.cuda.device(dev):
        rc = hip.hipExtMallocWithFlags(C.byref(ptr), n * 4, 0x3)
    if rc != 0 or not ptr.value:
        raise RuntimeError(f"hipExtMallocWithFlags(uncached, {n * 4} bytes) failed with error {rc}")

    class _Raw:
        __cuda_array_interface__ = {"shape": tuple(int(x) for x in shape), "typestr": "<f4",
                                    "data": (ptr.value, False), "version": 2}
    raw = _Raw()
    t = torch.as_tensor(raw, device=dev)
    assert t.data_ptr() == ptr.value
    _UNCACHED.append((ptr, raw))
    t.zero_()
    return t


class Trainer:
    def __init__(self, *, vocab, dim, window, negatives, counts, tokens_per_epoch, seed, table_size=1 << 24,
                 subsample_t=0.0, total_epochs=1, sentences_in_flight=0, window_mode=0, lr0=0.025,
                 lr_min_frac=1e-4, device=0, init_weights=True, syn0=None, syn1neg=None, negative_block=0,
                 coherent_tables=False, update_mode=0, storage=0):
        """storage: cfg.storage of the library (0 float tables, 1 bfloat16 tables with stochastic rounding).
        update_mode: cfg.update_mode of the library (0 automatic, 1 overwrite, 2 summed lock-free updates).
        coherent_tables (experiments only; the library's summed mode reaches the same end with system-scope
        accesses to ordinary memory): keep syn0 / syn1neg, or the one table named, in uncached device memory.  Such
        memory is never freed (see _uncached_zeros); close() hands it to a pool for later Trainers."""
        if not torch.cuda.is_available():
            raise RuntimeError("the SGNS trainer needs a GPU; there is no CPU implementation in this package")
        self.dev = torch.device("cuda", device)
        self.vocab, self.dim, self.window, self.negatives = vocab, dim, window, negatives
        self.ld = B.w2v_query_ld(dim)
        self.coherent_tables = coherent_tables
        self.storage = storage
        self._uncached = []
        table_dtype = torch.bfloat16 if storage else torch.float32
        assert not (storage and coherent_tables)

        def table(name):       # coherent_tables may also name one table ("syn0" / "syn1neg")
            if coherent_tables is True or coherent_tables == name:
                t = _uncached_zeros((vocab, self.ld), self.dev)
                self._uncached.append(t)
                return t
            return torch.zeros((vocab, self.ld), dtype=table_dtype, device=self.dev)
        self.syn0, self.syn1neg = table("syn0"), table("syn1neg")
        if syn0 is not None:
            self.syn0[:, :dim] = torch.as_tensor(np.asarray(syn0, np.float32)).to(self.dev).to(table_dtype)
            self.syn1neg[:, :dim] = torch.as_tensor(np.asarray(syn1neg, np.float32)).to(self.dev).to(table_dtype)
            init_weights = False
        ws_bytes = B.w2v_query_workspace(vocab, table_size, dim=dim, window=window, negatives=negatives,
                                         window_mode=window_mode, update_mode=update_mode)
        self.workspace = torch.zeros(ws_bytes, dtype=torch.uint8, device=self.dev)
        assert self.workspace.data_ptr() % 256 == 0
        self.stream = torch.cuda.current_stream(self.dev)
        self.cfg = B.make_config(vocab=vocab, dim=dim, window=window, negatives=negatives,
                                 tokens_per_epoch=tokens_per_epoch, seed=seed, syn0=self.syn0, syn1neg=self.syn1neg,
                                 ld=self.ld, workspace=self.workspace, workspace_bytes=ws_bytes, device=device,
                                 stream=self.stream.cuda_stream, window_mode=window_mode, total_epochs=total_epochs,
                                 sentences_in_flight=sentences_in_flight, lr0=lr0, lr_min_frac=lr_min_frac,
                                 subsample_t=subsample_t, negative_block=negative_block, update_mode=update_mode,
                                 storage=storage)
        torch.cuda.synchronize(self.dev)
        self.ctx = B.w2v_create(self.cfg, 1 if init_weights else 0)
        B.w2v_build_unigram_table(self.ctx, counts, table_size)
        self.tokens = self.sent_off = None
        self.n_sent = 0

    def set_corpus(self, tokens, sent_off):
        """tokens: int32 word ids; sent_off: S+1 offsets (numpy uint64, or int64 tensor of the same bytes).  numpy
        arrays are copied to the device, device tensors are used where they are."""
        if isinstance(tokens, torch.Tensor):
            assert tokens.dtype == torch.int32 and sent_off.dtype == torch.int64 and tokens.is_contiguous()
            self.tokens, self.sent_off = tokens.to(self.dev), sent_off.to(self.dev)
        else:
            self.tokens = torch.as_tensor(np.ascontiguousarray(tokens, np.int32)).to(self.dev)
            # torch has no uint64 arithmetic, but the bytes are all the library needs
            self.sent_off = torch.as_tensor(np.ascontiguousarray(sent_off, np.uint64).view(np.int64)).to(self.dev)
        self.n_tokens = int(self.tokens.numel())
        if self.n_tokens == 0:                  # only empty sentences: the library still wants a pointer
            self.tokens = torch.zeros(1, dtype=torch.int32, device=self.dev)
        self.n_sent = len(sent_off) - 1
        torch.cuda.synchronize(self.dev)

    def train_epoch(self, epoch=0, first_token_global_pos=0, naive=False):
        f = B.w2v_train_epoch_naive if naive else B.w2v_train_epoch
        f(self.ctx, self.tokens, self.sent_off, self.n_sent, first_token_global_pos, epoch)

    def train_epoch_from_host(self, tokens, sent_off, epoch=0, first_token_global_pos=0, staging_bytes=128 << 20):
        """tokens / sent_off: host arrays (numpy int32 / uint64, or pinned torch tensors of the same bytes); they
        are cut into batches that are copied into a device staging buffer while the previous batch trains."""
        if getattr(self, "staging", None) is None or self.staging.numel() != staging_bytes:
            self.staging = torch.empty(staging_bytes, dtype=torch.uint8, device=self.dev)
            assert self.staging.data_ptr() % 256 == 0
        B.w2v_train_epoch_host(self.ctx, tokens, sent_off, len(sent_off) - 1, first_token_global_pos, epoch,
                               self.staging, staging_bytes)

    def loss(self, reset=False):
        return B.w2v_loss(self.ctx, reset)

    def counters(self, reset=False):
        return B.w2v_counters(self.ctx, reset)

    def embeddings(self, which=0):
        if self.storage:                         # bfloat16 tables are widened on the device
            dev = torch.empty((self.vocab, self.dim), dtype=torch.float32, device=self.dev)
            B.w2v_get_embeddings(self.ctx, which, dev, dev.numel(), True)
            return dev.cpu().numpy()
        out = np.empty((self.vocab, self.dim), np.float32)
        B.w2v_get_embeddings(self.ctx, which, out, out.size, False)
        return out

    def draws(self, epoch=0, first_token_global_pos=0):
        T = self.n_tokens
        keep = torch.zeros(T, dtype=torch.uint8, device=self.dev)
        width = torch.zeros(T, dtype=torch.uint8, device=self.dev)
        neg = torch.zeros((T, max(self.negatives, 1)), dtype=torch.int32, device=self.dev)
        B.w2v_debug_draws(self.ctx, self.tokens, self.sent_off, self.n_sent, first_token_global_pos, epoch, keep,
                          width, neg)
        torch.cuda.synchronize(self.dev)
        return keep.cpu().numpy(), width.cpu().numpy(), neg.cpu().numpy()[:, :self.negatives]

    def train_draws(self, epoch=0, first_token_global_pos=0):
        """One training pass in which the window kernel itself writes out its integer decisions."""
        T = self.n_tokens
        keep = torch.empty(T, dtype=torch.uint8, device=self.dev)
        width = torch.empty(T, dtype=torch.uint8, device=self.dev)
        neg = torch.empty((T, max(self.negatives, 1)), dtype=torch.int32, device=self.dev)
        if self.negatives == 0:
            neg.fill_(-1)
        B.w2v_debug_train_draws(self.ctx, self.tokens, self.sent_off, self.n_sent, first_token_global_pos, epoch, keep,
                                width, neg.view(-1)[:T * self.negatives] if self.negatives else neg)
        torch.cuda.synchronize(self.dev)
        return keep.cpu().numpy(), width.cpu().numpy(), neg.view(-1)[:T * self.negatives].view(T, self.negatives).cpu().numpy()

    def close(self):
        if self.ctx is not None:
            B.w2v_destroy(self.ctx)           # waits for the stream: nothing uses the tables any more
            self.ctx = None
            for t in self._uncached:
                _UNCACHED_FREE.setdefault((self.dev.index or 0, tuple(t.shape)), []).append(t)
            self._uncached = []

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
