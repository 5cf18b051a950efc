"""Synthetic corpora of the paper's largest shapes (Table 3; 800M tokens), generated in device memory with torch
so that they take seconds instead of minutes.  Like synth.py this module only produces inputs (token ids,
sentence offsets, word counts) and holds none of the training method's arithmetic."""
import numpy as np
import torch

from . import synth


def zipf_tokens(vocab: int, s: float, n_tokens: int, seed: int, device="cuda"):
    """iid Zipf(s) word ids (id 0 the most frequent) as an int32 device tensor, and their counts (numpy uint64)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    cdf = torch.as_tensor(synth._zipf_cdf(vocab, s), device=device)
    tok = torch.empty(n_tokens, dtype=torch.int32, device=device)
    counts = torch.zeros(vocab, dtype=torch.int64, device=device)
    step = 1 << 26
    for a in range(0, n_tokens, step):
        b = min(n_tokens, a + step)
        ids = torch.searchsorted(cdf, torch.rand(b - a, dtype=torch.float64, device=device, generator=gen), right=True)
        ids.clamp_(max=vocab - 1)
        tok[a:b] = ids
        counts += torch.bincount(ids, minlength=vocab)
    return tok, counts.cpu().numpy().astype(np.uint64)


def barabasi_albert_walk_tokens(n_nodes: int, m: int, walks_per_node: int, walk_len: int, seed: int, device="cuda"):
    """Uniform random walks (walks_per_node from every node) on the seeded Barabasi-Albert graph of synth.py, walked
    on the device: int32 tensor [n_walks * walk_len] (node id = word id) and the visit counts (numpy uint64)."""
    rowptr, nbr, deg = synth.barabasi_albert_graph(n_nodes, m, np.random.Generator(np.random.PCG64(seed)))
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    rowptr_d = torch.as_tensor(rowptr[:-1], device=device)
    nbr_d = torch.as_tensor(nbr, device=device)
    deg_d = torch.as_tensor(deg, device=device)
    n_walks = n_nodes * walks_per_node
    cur = torch.arange(n_nodes, dtype=torch.int64, device=device).repeat(walks_per_node)
    walks = torch.empty((n_walks, walk_len), dtype=torch.int32, device=device)
    walks[:, 0] = cur
    for step in range(1, walk_len):
        r = torch.rand(n_walks, dtype=torch.float64, device=device, generator=gen)
        pick = torch.minimum((r * deg_d[cur]).long(), deg_d[cur] - 1)
        cur = nbr_d[rowptr_d[cur] + pick]
        walks[:, step] = cur
    tok = walks.reshape(-1)
    counts = torch.bincount(tok, minlength=n_nodes)
    return tok, counts.cpu().numpy().astype(np.uint64)
