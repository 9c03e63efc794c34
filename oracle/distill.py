"""Synthetic "distilled" drafters: a level whose logits are a deeper level's logits plus seeded Gaussian noise.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper's drafters are smaller trained models whose distributions are close to the target's (acceptance rates of
0.6-0.9 between neighbouring levels, Sec. 5); random-init stand-ins of different shapes agree far less.  The workload
description asks for the closeness to be produced synthetically: level i's next-token logits are the source level's
logits at the same context plus N(0, std_i^2) noise per vocabulary entry, fixed by (seed, level, position), so that a
level is still a deterministic function of its context, as the problem statement of Sec. 3.2 requires of a model.
The source may be synthetic itself (a chain: each level is the next one up plus one noise term, so neighbours are
close and distant levels less so).
Nothing here is from the paper beyond that requirement; the generator is spelled out so that the library can
reproduce it:
    block   = Philox4x32-10(key = seed, counter = (v // 4, pos, level | 2^31, 0x4E4F4953))
    (n_0, n_1) = BoxMuller(block[0], block[1]),  (n_2, n_3) = BoxMuller(block[2], block[3])   for entries 4 (v // 4) + 0..3
    BoxMuller(a, b): u1 = (a + 0.5) 2^-32, u2 = (b + 0.5) 2^-32, r = sqrt(-2 ln u1), (r cos 2 pi u2, r sin 2 pi u2)
where pos is the position of the last context token.  The drafter's own network still runs (it is what its cost
is), its logits are simply not used.
"""
import numpy as np

from . import decoder as _decoder
from . import philox

NOISE_TAG = 0x4E4F4953


def gaussian_noise(seed, level, pos, vocab):
    """The noise row of (level, pos): `vocab` standard normals in fp64."""
    nblk = (vocab + 3) // 4
    ctr = np.zeros((nblk, 4), dtype=np.uint64)
    ctr[:, 0] = np.arange(nblk)
    ctr[:, 1] = pos
    ctr[:, 2] = (level | 0x80000000)
    ctr[:, 3] = NOISE_TAG
    key = (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    w = philox.philox4x32_10(ctr, key).astype(np.float64)
    out = np.empty((nblk, 4))
    for a, b, o in ((0, 1, 0), (2, 3, 2)):
        u1 = (w[:, a] + 0.5) * 2.0 ** -32
        u2 = (w[:, b] + 0.5) * 2.0 ** -32
        r = np.sqrt(-2.0 * np.log(u1))
        out[:, o] = r * np.cos(2.0 * np.pi * u2)
        out[:, o + 1] = r * np.sin(2.0 * np.pi * u2)
    return out.reshape(-1)[:vocab]


class DistilledLevel(_decoder.Level):
    """Level `level_index` of a hierarchy: distribution rows from `source` (another Level)'s logits plus noise."""

    def __init__(self, own_decoder, own_exit, source, level_index, std, seed, temperature):
        super().__init__(own_decoder, own_exit, temperature)
        self.source, self.level_index, self.std, self.seed = source, level_index, float(std), int(seed)

    def logit_rows(self, context, n_rows):
        """The level's logits for the last n_rows prefixes of `context`: the source's (a real network's, or another
        synthetic level's, which then carries its own noise already) plus this level's noise."""
        if isinstance(self.source, DistilledLevel):
            z = self.source.logit_rows(context, n_rows)
        else:
            z = np.array(self.source.decoder.next_logits(context, n_rows, self.source.exit_layer), dtype=np.float64)
        L = len(context)
        for r in range(n_rows):
            pos = L - n_rows + r                    # position of the last token of this row's context
            z[r] += self.std * gaussian_noise(self.seed, self.level_index, pos, z.shape[1])
        return z

    def next_dists(self, context, n_rows):
        z = self.logit_rows(context, n_rows)
        self.last_logits = z
        top2 = np.partition(z, -2, axis=-1)[:, -2:]
        self.min_top2_gap = min(self.min_top2_gap, float(np.min(top2[:, 1] - top2[:, 0])))
        return _decoder.distributions(z, self.temperature)
