"""Helpers shared by the tests.  Nothing here computes random values or index maps:
the merge below rebuilds a global tensor from shards by concatenation only."""
import itertools

import numpy as np


def mesh_coords(mesh_shape):
    return list(itertools.product(*[range(p) for p in mesh_shape]))


class NotGatherable(Exception):
    """The shards cannot be put back together by plain concatenation: an interleaved piece whose
    length is not a whole number of groups (interleave over an uneven split)."""


def merge_shards(shards, mesh_shape, placements):
    """Rebuilds the global array from {mesh_coord: local array} the way a sharded
    tensor is gathered: along each mesh dimension (innermost first) the ranks'
    pieces are concatenated on the placement's tensor dimension; replicas must agree;
    interleaved pieces are concatenated group by group."""
    def rec(prefix):
        m = len(prefix)
        if m == len(mesh_shape):
            return shards[tuple(prefix)]
        parts = [rec(prefix + [r]) for r in range(mesh_shape[m])]
        pl = placements[m]
        if pl[0] == "R":
            for p in parts[1:]:
                assert p.shape == parts[0].shape and np.array_equal(p, parts[0]), "replicas differ"
            return parts[0]
        if pl[0] == "S":
            return np.concatenate(parts, axis=pl[1])
        if pl[0] == "IS":
            d, groups = pl[1], pl[2]
            out = []
            for g in range(groups):
                for p in parts:
                    if p.shape[d] % groups != 0:
                        raise NotGatherable("%s over pieces of length %d" % (pl, p.shape[d]))
                    out.append(np.split(p, groups, axis=d)[g])
            return np.concatenate(out, axis=d)
        raise AssertionError(pl)
    return rec([])


def all_placements(ndim, mesh_ndim, global_shape=None, interleaves=(2, 3)):
    """Every assignment of Replicate / Shard(d) / InterleavedShard(d, k) to the mesh dims."""
    one = [("R",)] + [("S", d) for d in range(ndim)]
    one += [("IS", d, k) for d in range(ndim) for k in interleaves]
    return list(itertools.product(one, repeat=mesh_ndim))
