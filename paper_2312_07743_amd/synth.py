"""Seeded synthetic corpora with the shapes of the paper's workloads (Table 3).

This module only produces inputs (token ids, sentence offsets, word counts,
planted-cluster labels).  It holds none of the training method's arithmetic and
is the one module that both the GPU path's callers and the CPU oracle's callers
may use.  numpy only.
"""
from dataclasses import dataclass
from typing import Optional

import numpy as np


@dataclass
class Corpus:
    tokens: np.ndarray            # int32 [T] word ids, sentence after sentence
    sent_off: np.ndarray          # uint64 [S+1] offsets into tokens
    counts: np.ndarray            # uint64 [V] occurrences of each id in tokens
    labels: Optional[np.ndarray] = None   # int32 [V] planted cluster of a word, -1 = none

    @property
    def vocab(self) -> int:
        return int(len(self.counts))

    @property
    def n_tokens(self) -> int:
        return int(len(self.tokens))

    @property
    def n_sent(self) -> int:
        return int(len(self.sent_off) - 1)


def _zipf_cdf(vocab: int, s: float) -> np.ndarray:
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-float(s))
    cdf = np.cumsum(w)
    return cdf / cdf[-1]


def _uniform_offsets(n_sent: int, sent_len: int) -> np.ndarray:
    return (np.arange(n_sent + 1, dtype=np.uint64) * np.uint64(sent_len)).astype(np.uint64)


def zipf_corpus(vocab: int, s: float, n_sent: int, sent_len: int, seed: int) -> Corpus:
    """iid Zipf(s) ids; id 0 is the most frequent word (a count-sorted vocabulary).
    'Tiny' = zipf_corpus(1000, 1.0, 100, 1000, seed)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    cdf = _zipf_cdf(vocab, s)
    T = n_sent * sent_len
    tok = np.searchsorted(cdf, rng.random(T), side="right").astype(np.int32)
    np.minimum(tok, vocab - 1, out=tok)
    counts = np.bincount(tok, minlength=vocab).astype(np.uint64)
    return Corpus(tok, _uniform_offsets(n_sent, sent_len), counts)


def planted_corpus(vocab: int = 71000, s: float = 1.05, n_sent: int = 17000, sent_len: int = 1000,
                   seed: int = 1, n_clusters: int = 16, cluster_size: int = 50,
                   band_start: int = 2000, burst_p: float = 0.02, burst_len: int = 8,
                   min_count: int = 5, progress=None) -> Corpus:
    """'Mid': Zipf(s) text with planted co-occurrence clusters.

    n_clusters*cluster_size words are taken from the rank band starting at
    band_start (frequent enough to survive min_count, rare enough not to be
    subsampled away).  With probability burst_p a position starts a burst of
    burst_len consecutive tokens drawn uniformly from one cluster.  Words with
    fewer than min_count occurrences are then removed and ids re-numbered in
    rank order (the rule of Table 3's caption); sentences keep their boundaries.
    `progress`, if given, is called with a short text after each stage (large corpora take minutes).
    """
    say = progress or (lambda text: None)
    rng = np.random.Generator(np.random.PCG64(seed))
    cdf = _zipf_cdf(vocab, s)
    T = n_sent * sent_len
    tok = np.empty(T, np.int32)
    step = 1 << 25                      # the uniform draws are consumed in order, so pieces give the same ids
    for a in range(0, T, step):
        b = min(T, a + step)
        tok[a:b] = np.searchsorted(cdf, rng.random(b - a), side="right")
        say(f"corpus: {b} of {T} Zipf ids drawn")
    np.minimum(tok, vocab - 1, out=tok)
    n_planted = n_clusters * cluster_size
    assert band_start + n_planted <= vocab
    perm = rng.permutation(n_planted)
    labels_full = np.full(vocab, -1, np.int32)
    labels_full[band_start + perm] = (np.arange(n_planted) // cluster_size).astype(np.int32)
    members = [band_start + perm[c * cluster_size:(c + 1) * cluster_size] for c in range(n_clusters)]
    starts = np.flatnonzero(rng.random(T) < burst_p)
    which = rng.integers(0, n_clusters, size=len(starts))
    picks = rng.integers(0, cluster_size, size=(len(starts), burst_len))
    members = np.stack(members)                                   # [C, cluster_size]
    for j in range(burst_len):
        pos = starts + j
        ok = (pos // sent_len) == (starts // sent_len)            # stay inside the sentence
        tok[pos[ok]] = members[which[ok], picks[ok, j]]
    say("corpus: bursts planted")
    counts_full = np.bincount(tok, minlength=vocab)
    keep_word = counts_full >= min_count
    remap = np.cumsum(keep_word) - 1
    keep_tok = keep_word[tok]
    new_tok = remap[tok[keep_tok]].astype(np.int32)
    sent_id = np.repeat(np.arange(n_sent), sent_len)[keep_tok]
    lens = np.bincount(sent_id, minlength=n_sent)
    sent_off = np.zeros(n_sent + 1, np.uint64)
    sent_off[1:] = np.cumsum(lens).astype(np.uint64)
    counts = counts_full[keep_word].astype(np.uint64)
    labels = labels_full[keep_word]
    say("corpus: rare words removed, ids renumbered")
    return Corpus(new_tok, sent_off, counts, labels)


def disjoint_slice_corpus(vocab: int, n_sent: int, sent_len: int, seed: int) -> Corpus:
    """Sentence s only uses ids of its own slice [s*V/S, (s+1)*V/S): with zero negatives
    no two sentences touch the same row, so any execution order gives the same result."""
    rng = np.random.Generator(np.random.PCG64(seed))
    per = vocab // n_sent
    assert per >= 2
    base = (np.arange(n_sent) * per).repeat(sent_len)
    tok = (base + rng.integers(0, per, size=n_sent * sent_len)).astype(np.int32)
    counts = np.bincount(tok, minlength=vocab).astype(np.uint64)
    return Corpus(tok, _uniform_offsets(n_sent, sent_len), counts)


def barabasi_albert_graph(n_nodes: int, m: int, rng, progress=None):
    """Seeded Barabasi-Albert graph in CSR form (rowptr int64[n+1], neighbours int64[2E], degrees int64[n]).
    The graph is grown with the repeated-endpoint list (a node is picked with probability
    proportional to its degree by picking a uniform entry of the list of edge endpoints)."""
    say = progress or (lambda text: None)
    assert n_nodes > m >= 1
    src = np.empty((n_nodes - m) * m, np.int64)
    dst = np.empty((n_nodes - m) * m, np.int64)
    endpoints = np.empty(2 * (n_nodes - m) * m + m, np.int64)
    endpoints[:m] = np.arange(m)
    n_end = m
    e = 0
    for v in range(m, n_nodes):
        targets = set()
        while len(targets) < m:
            for t in endpoints[rng.integers(0, n_end, size=m - len(targets))]:
                targets.add(int(t))
        for t in targets:
            src[e] = v
            dst[e] = t
            endpoints[n_end] = v
            endpoints[n_end + 1] = t
            n_end += 2
            e += 1
    say("graph: grown")
    a = np.concatenate([src, dst])
    b = np.concatenate([dst, src])
    order = np.argsort(a, kind="stable")
    a, b = a[order], b[order]
    deg = np.bincount(a, minlength=n_nodes)
    rowptr = np.zeros(n_nodes + 1, np.int64)
    rowptr[1:] = np.cumsum(deg)
    return rowptr, b, deg


def barabasi_albert_walks(n_nodes: int, m: int, walks_per_node: int, walk_len: int, seed: int,
                          progress=None) -> Corpus:
    """'Graph': uniform random walks on a seeded Barabasi-Albert graph; node id = word id."""
    say = progress or (lambda text: None)
    rng = np.random.Generator(np.random.PCG64(seed))
    rowptr, b, deg = barabasi_albert_graph(n_nodes, m, rng, progress)
    n_walks = n_nodes * walks_per_node
    cur = np.tile(np.arange(n_nodes, dtype=np.int64), walks_per_node)
    walks = np.empty((n_walks, walk_len), np.int32)
    walks[:, 0] = cur
    for step in range(1, walk_len):
        r = rng.random(n_walks)
        nxt = b[rowptr[cur] + (r * deg[cur]).astype(np.int64)]
        walks[:, step] = nxt
        cur = nxt
        if step % 8 == 0:
            say(f"graph: step {step} of {walk_len} of {n_walks} walks")
    tok = walks.reshape(-1)
    counts = np.bincount(tok, minlength=n_nodes).astype(np.uint64)
    return Corpus(tok, _uniform_offsets(n_walks, walk_len), counts)
