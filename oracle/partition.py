"""Oracle: random layer-wise split of the global ResNet into S sub-ResNets (Sec. 2.2).

TEST INFRASTRUCTURE ONLY.

What the paper fixes (Sec. 2.2, Fig. 1, Sec. 2.6 "Subnetwork Depth"):
  * indices of the partitionable blocks are randomly permuted and dealt round-robin;
  * every sub-ResNet receives the same number of blocks;
  * a block may be given to several sub-ResNets to reach a minimum depth;
  * blocks that are not partitionable (stem, strided first blocks, final layer ...)
    belong to every sub-ResNet; no block is ever left out of a round (Sec. 4).
What the paper leaves open, and the reading taken here:
  * random source: splitmix64 seeded with seed XOR (round * golden-ratio constant),
    Fisher-Yates from the top index down, j = next() mod (i+1);
  * equal sizes when S does not divide P: every sub-ResNet gets D = max(ceil(P/S),
    min(min_depth, P)) dealt blocks; sub s takes permuted positions s, s+S, s+2S, ...
    modulo P; a position whose block the sub already holds is advanced by one until free.
Pins: Fig. 1's worked example (5 blocks, S=2 -> 3+3, one shared), Table 1's byte counts
(11 / 6 / 4 dealt blocks at 2 / 4 / 8 machines), permutation/coverage/equal-size invariants,
the published splitmix64 test vector.  The sampled indices themselves are fixed only by the
reading above ("parity unpinned" against the paper: it prints no sampled partition).
"""

MASK64 = (1 << 64) - 1
GOLDEN = 0x9E3779B97F4A7C15


class SplitMix64:
    def __init__(self, state):
        self.state = state & MASK64

    def next(self):
        self.state = (self.state + GOLDEN) & MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        return z ^ (z >> 31)


def stage_first_blocks(blocks_per_stage):
    first, b = [], 0
    for nb in blocks_per_stage:
        first.append(b)
        b += nb
    return first, b


def permutation(P, seed, rnd):
    rng = SplitMix64(seed ^ ((rnd * GOLDEN) & MASK64))
    perm = list(range(P))
    for i in range(P - 1, 0, -1):
        j = rng.next() % (i + 1)
        perm[i], perm[j] = perm[j], perm[i]
    return perm


def partition(blocks_per_stage, S, min_depth, seed, rnd, partitionable=None):
    """Returns (sub_blocks: list of S ascending lists of global block indices, owner_count[B]).

    partitionable: optional list of B flags; None = every non-first block of every stage.
    """
    first, B = stage_first_blocks(blocks_per_stage)
    if partitionable is None:
        partitionable = [0 if b in first else 1 for b in range(B)]
    part = [b for b in range(B) if partitionable[b]]
    fixed = [b for b in range(B) if not partitionable[b]]
    P = len(part)
    subs = [set(fixed) for _ in range(S)]
    if P > 0:
        perm = permutation(P, seed, rnd)
        D = max(-(-P // S), min(min_depth, P))
        for s in range(S):
            dealt = set()
            for j in range(D):
                pos = (s + j * S) % P
                while perm[pos] in dealt:
                    pos = (pos + 1) % P
                dealt.add(perm[pos])
            subs[s] |= {part[i] for i in dealt}
    sub_blocks = [sorted(x) for x in subs]
    owner = [sum(1 for x in subs if b in x) for b in range(B)]
    return sub_blocks, owner
