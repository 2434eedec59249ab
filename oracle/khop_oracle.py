"""TEST INFRASTRUCTURE: multi-hop temporal sampling as a chain of one-hop oracle calls.

Section 4.2 of the paper (multi-hop neighbourhood sampling): the one-hop step is repeated per
GNN layer, the nodes sampled in one layer being the targets of the next; a temporal random
walk is the case of fan-out 1 per layer.  Section 2.1 describes the result as a tree rooted
at the target.  The paper does not say which time the next layer's query carries; the reading
taken (the convention of the sampler the paper cites for this step) is:

  * hop h+1 has one query per sampled edge of hop h, in the order of hop h's dense result
    (query order, then slot order);
  * its target is that edge's neighbour, its window end is that edge's timestamp,
    its window start is end - delta computed in fp32 (delta = +inf: no lower bound);
  * with several graph instances, an instance's queries of hop h+1 are the dense entries of
    its queries of hop h, so the next offsets are rowptr_h[offsets_h];
  * uniform policy: query i of hop h has generator id  base + cap_1 + ... + cap_{h-1} + i  with
    cap_1 = number of first-hop queries and cap_{h+1} = cap_h * fanout_h (the most queries hop
    h+1 can have), so that ids never collide between hops whatever the data.

Everything else (window, selection, padding, compaction) is the one-hop oracle, called as is.
Pinned by tests/test_khop_oracle.py (toy example of section 2.1 as far as the text fixes it,
brute-force temporal walk, fp32 window start, id bases, two instances).
"""
from __future__ import annotations

import numpy as np

from . import Sampled, compact


def _one_hop(adjs, targets, t_start, t_end, inst_rowptr, fanout, policy, inclusive_end, seed, first_id, threads):
    """One-hop oracle over all instances: instance b serves queries inst_rowptr[b] .. inst_rowptr[b+1]-1."""
    n = len(targets)
    out = Sampled(n, fanout)
    bounds = [0, n] if inst_rowptr is None else [int(x) for x in inst_rowptr]
    for b, adj in enumerate(adjs):
        lo, hi = bounds[b], bounds[b + 1]
        ids = np.arange(first_id + lo, first_id + hi, dtype=np.int64)
        part = adj.sample(targets[lo:hi], None if t_start is None else t_start[lo:hi], t_end[lo:hi], fanout,
                          policy=policy, inclusive_end=inclusive_end, seed=seed, q_ids=ids, threads=threads)
        out.nbr[lo:hi], out.eid[lo:hi], out.ts[lo:hi], out.count[lo:hi] = part.nbr, part.eid, part.ts, part.count
    return out


def khop(adjs, targets, t_start, t_end, inst_rowptr, fanouts, delta=float("inf"), policy=0, inclusive_end=0, seed=0,
         query_id_base=0, threads=1):
    """Returns one dict per hop: padded (Sampled), rowptr, cmp_nbr, cmp_eid, cmp_ts, num_queries,
    inst_rowptr (the offsets the hop was run with, None for one instance)."""
    targets = np.ascontiguousarray(targets, dtype=np.int32)
    t_end = np.ascontiguousarray(t_end, dtype=np.float32)
    t_start = None if t_start is None else np.ascontiguousarray(t_start, dtype=np.float32)
    offs = None if inst_rowptr is None else np.ascontiguousarray(inst_rowptr, dtype=np.int64)
    hops = []
    first_id = int(query_id_base)
    cap = len(targets)
    for f in fanouts:
        padded = _one_hop(adjs, targets, t_start, t_end, offs, f, policy, inclusive_end, seed, first_id, threads)
        rowptr, cn, ce, ct = compact(padded)
        hops.append(dict(padded=padded, rowptr=rowptr, cmp_nbr=cn, cmp_eid=ce, cmp_ts=ct, num_queries=len(targets),
                         inst_rowptr=offs))
        # next layer: one query per sampled edge, in dense order
        if offs is not None:
            offs = rowptr[offs]
        targets = cn
        t_end = ct
        t_start = None if np.isinf(delta) else (ct - np.float32(delta)).astype(np.float32)
        first_id += cap
        cap *= f
    return hops
