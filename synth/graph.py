"""Chung-Lu power-law graph generator producing a symmetric, simple, row-sorted CSR."""
import math

import torch


def _expected_degree_weights(num_nodes, target_nnz, gamma):
    """w_r = min(c * (r+1)^(-1/(gamma-1)), sqrt(target_nnz)), c chosen so that sum(w) = target_nnz.

    Computed on the CPU: parallel floating-point reductions on the GPU are not bit-reproducible from
    run to run, and the weights decide which edges are drawn."""
    alpha = 1.0 / (gamma - 1.0)
    base = torch.arange(1, num_nodes + 1, dtype=torch.float64).pow_(-alpha)
    cap = math.sqrt(float(target_nnz))
    lo, hi = 0.0, float(target_nnz)          # base[0] == 1, so c = target_nnz certainly overshoots
    for _ in range(48):
        mid = 0.5 * (lo + hi)
        total = torch.clamp(base * mid, max=cap).sum().item()
        if total < target_nnz:
            lo = mid
        else:
            hi = mid
    return torch.clamp(base * hi, max=cap)


def chung_lu_csr(num_nodes, mean_degree, gamma, seed, device="cpu", offsets64=False,
                 chunk=1 << 26, communities=0, p_in=0.0, return_communities=False):
    """Return (row_ptr, col_idx) of an undirected simple graph stored as a directed CSR.

    With communities = C > 0 the nodes fall into C equal groups (every group gets its share of hubs) and the second
    endpoint of an edge is drawn inside the first endpoint's group with probability p_in, anywhere otherwise: a
    degree-corrected planted partition, which gives a locality-aware partitioner something to find.  With
    return_communities the group label of every node (int64 [N]) is returned as a third value.

    Both endpoints of each of target_nnz/2 undirected edges are drawn with probability
    proportional to the expected-degree weights; node ranks are relabelled by a seeded
    permutation (hubs are not the low ids); self loops and duplicate edges are dropped,
    the edge set is symmetrised and every row is sorted ascending.  row_ptr is int64 when
    offsets64 else int32; col_idx is int32.
    """
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(int(seed))
    n = int(num_nodes)
    target_nnz = int(round(mean_degree * n))
    n_und = target_nnz // 2

    w = _expected_degree_weights(n, target_nnz, gamma)
    cdf = torch.cumsum(w, 0)
    cdf /= cdf[-1].clone()
    cdf = cdf.to(device)
    del w
    perm = torch.randperm(n, generator=gen, device=device)
    C = int(communities)
    labels = None
    group_idx, group_cdf = [], []
    if C > 0:
        # rank r belongs to group r % C; per group, the ranks and the cumulative weights for draws inside it
        labels = torch.empty(n, dtype=torch.int64, device=device)
        labels[perm] = torch.arange(n, device=device) % C
        w_dev = torch.diff(cdf, prepend=cdf.new_zeros(1))
        for c in range(C):
            idx = torch.arange(c, n, C, device=device)
            gc = torch.cumsum(w_dev[idx], 0)
            group_idx.append(idx)
            group_cdf.append(gc / gc[-1].clone())

    keys = []
    done = 0
    while done < n_und:
        m = min(chunk, n_und - done)
        a = torch.searchsorted(cdf, torch.rand(m, dtype=torch.float64, generator=gen, device=device))
        b = torch.searchsorted(cdf, torch.rand(m, dtype=torch.float64, generator=gen, device=device))
        a.clamp_(max=n - 1)
        b.clamp_(max=n - 1)
        if C > 0:
            inside = torch.rand(m, dtype=torch.float64, generator=gen, device=device) < p_in
            u = torch.rand(m, dtype=torch.float64, generator=gen, device=device)
            for c in range(C):
                sel = inside & (a % C == c)
                pick = torch.searchsorted(group_cdf[c], u[sel]).clamp_(max=group_idx[c].numel() - 1)
                b[sel] = group_idx[c][pick]
        a = perm[a]
        b = perm[b]
        keep = a != b
        a, b = a[keep], b[keep]
        lo, hi = torch.minimum(a, b), torch.maximum(a, b)
        keys.append(lo * n + hi)
        done += m
    del cdf, perm
    und = torch.unique(torch.cat(keys)) if keys else torch.empty(0, dtype=torch.int64, device=device)
    del keys
    lo, hi = und // n, und % n
    del und
    directed = torch.cat([lo * n + hi, hi * n + lo])
    del lo, hi
    directed, _ = torch.sort(directed)
    rows = directed // n
    col_idx = (directed % n).to(torch.int32)
    del directed
    deg = torch.bincount(rows, minlength=n)
    del rows
    row_ptr = torch.zeros(n + 1, dtype=torch.int64, device=device)
    torch.cumsum(deg, 0, out=row_ptr[1:])
    if not offsets64:
        assert int(row_ptr[-1]) < 2 ** 31
        row_ptr = row_ptr.to(torch.int32)
    if return_communities:
        return row_ptr, col_idx, labels
    return row_ptr, col_idx
