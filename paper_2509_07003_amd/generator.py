"""The caller-side RNG state of the sharded operators: a seed and an offset.

The library keeps no state (veScale, Section 5: all ranks share one global seed and step to the
same next global offset after every operator).  This class is that bookkeeping and nothing else:
each method issues ONE library call with the current (seed, offset) and then advances the offset
by what the operator consumed on the GLOBAL tensor (vesrng_advance_offset), which is the same
number on every rank whatever its shard.  Ranks that perform the same sequence of calls therefore
stay in lockstep without exchanging anything, and the values equal those of one device performing
that sequence on the unsharded tensors.
"""
from . import binding as _b


class Generator:
    """seed: 64-bit; offset: multiple of 4 (a whole generator block)."""

    def __init__(self, seed, offset=0):
        if offset % 4:
            raise ValueError("offset must be a multiple of 4")
        self.seed = int(seed)
        self.offset = int(offset)

    def get_state(self):
        return self.seed, self.offset

    def set_state(self, state):
        seed, offset = state
        if offset % 4:
            raise ValueError("offset must be a multiple of 4")
        self.seed, self.offset = int(seed), int(offset)

    def _advance(self, sharding):
        self.offset = _b.vesrng_advance_offset(sharding, self.offset)

    def raw_u32_(self, sharding, out, stream=None):
        _b.vesrng_raw_u32(sharding, self.seed, self.offset, out, stream)
        self._advance(sharding)
        return out

    def uniform_(self, sharding, dtype, out, low=0.0, high=1.0, stream=None):
        _b.vesrng_uniform(sharding, dtype, low, high, self.seed, self.offset, out, stream)
        self._advance(sharding)
        return out

    def normal_(self, sharding, dtype, out, mean=0.0, std=1.0, stream=None):
        _b.vesrng_normal(sharding, dtype, mean, std, self.seed, self.offset, out, stream)
        self._advance(sharding)
        return out

    def randint_(self, sharding, out, low, high, stream=None):
        _b.vesrng_randint(sharding, low, high, self.seed, self.offset, out, stream)
        self._advance(sharding)
        return out

    def dropout(self, sharding, dtype, p, x, y, mask=None, stream=None):
        """Returns the (seed, offset) the call used: the backward pass replays the keep
        decisions by calling vesrng_dropout on the gradient with exactly that state."""
        used = (self.seed, self.offset)
        _b.vesrng_dropout(sharding, dtype, p, self.seed, self.offset, x, y, mask, stream)
        self._advance(sharding)
        return used

    def dropout_add(self, sharding, dtype, p, x, residual, y, mask=None, stream=None):
        used = (self.seed, self.offset)
        _b.vesrng_dropout_add(sharding, dtype, p, self.seed, self.offset, x, residual, y, mask, stream)
        self._advance(sharding)
        return used
