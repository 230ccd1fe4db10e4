"""Oracle for the two ends of the bridge layer (Section 3.2.3) on one device.

TEST INFRASTRUCTURE ONLY; shares no code with the library and never imports it.

The bridge layer gathers the distributed outputs of a TaskGraph so that the next TaskGraph reads
a complete tensor: for `replicate` the parts are different batches, concatenated along the batch
dimension; for `split` they are slices of the split dimension, concatenated there.  Both are the
plain definition of concatenation.  On the way back in front of a split TaskGraph every shard
holds a partial gradient of the gathered tensor; the gradient of a replica's part is the matching
row block of their sum.  The fusion rule: a gather followed by a partition along the same
dimension with the same cuts is the identity, so both are dropped (reading: the cuts have to
coincide too, the paper names only the dimension).
"""
import numpy as np


def gather(dim, parts):
    """Concatenation of the parts along dim (0 = batch_dim of the replicate pattern, 1 = split_dim)."""
    return np.concatenate(parts, axis=dim)


def partition(x, dim, extents):
    """The inverse cut: consecutive blocks of the given extents along dim."""
    out, at = [], 0
    for e in extents:
        idx = [slice(None)] * x.ndim
        idx[dim] = slice(at, at + e)
        out.append(x[tuple(idx)])
        at += e
    assert at == x.shape[dim]
    return out


def reduce_partition(partials, rows):
    """Row blocks of the sum of the shards' partial gradients, in fp64."""
    total = np.zeros(partials[0].shape, dtype=np.float64)
    for p in partials:
        total = total + np.asarray(p, dtype=np.float64)
    return partition(total, 0, rows)


def fusable(gather_dim, src_extents, partition_dim, dst_extents):
    return gather_dim == partition_dim and list(src_extents) == list(dst_extents)
