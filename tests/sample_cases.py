"""Hand-worked seeded-sampling cases whose expected tokens follow from the written rule alone (section 6.6
as read in the design notes: cut at the first prefix sum >= top_p * total, pick the first prefix sum >
u * kept total), with the uniform u recomputed here from the published splitmix64 output function.  Equal
logits make every e_i = 1, so the prefix sums are the integers 1, 2, 3, ... and products with the chosen u
are exact in fp32: the expected token is arithmetic on integers, on both sides of each comparison."""
import numpy as np

import detsynth as ds


def uniform_bits(seed, seq, steps):
    """Top 24 bits of the counter-based hash for (seed, seq, step), step over an array."""
    steps = np.asarray(steps, dtype=np.int64)
    out = np.empty(steps.shape, dtype=np.int64)
    for i, st in enumerate(steps.reshape(-1)):
        out.reshape(-1)[i] = int(ds._hash_np(seed, (int(seq) << 32) | int(st), 1)[0]) >> 40
    return out


def find_steps(seed, seq, want, limit=1 << 21, count=6):
    """Steps in [0, limit) of sequence `seq` whose 24 uniform bits satisfy want(bits) (vectorised search)."""
    bits = (ds._hash_np(seed, int(seq) << 32, limit) >> np.uint64(40)).astype(np.int64)
    hit = np.nonzero(want(bits))[0][:count]
    assert hit.size == count, "search range too small"
    return hit.astype(np.int32), bits[hit]


def pick_boundary_case(seed=0xC0FFEE, seq=3):
    """Equal logits, top_k = 1024, top_p = 1: prefix sums 1..1024, kept total 1024, target = u * 1024.
    u a multiple of 2^-10 puts the target exactly ON prefix sum j = u * 1024: the rule's strict '>' then
    selects rank j (a '>=' would select j - 1).  u one 2^-24 step below puts it just under: rank j - 1.
    Returns (logits [R, V], steps, expected tokens, seq ids)."""
    V = 2048
    on, bits_on = find_steps(seed, seq, lambda b: (b % (1 << 14) == 0) & (b > 0))
    under, bits_un = find_steps(seed, seq, lambda b: b % (1 << 14) == (1 << 14) - 1)
    steps = np.concatenate([on, under])
    want = np.concatenate([bits_on >> 14, bits_un >> 14])   # j, and (j*2^14 - 1) >> 14 = j - 1
    logits = np.zeros((steps.size, V), dtype=np.float32)
    return logits, steps, want.astype(np.int32), np.full(steps.size, seq, dtype=np.int32)


def cut_boundary_case(seed=0xBEEF, seq=9, R=256):
    """Equal logits, top_k = 4: prefix sums 1, 2, 3, 4.
    top_p = 0.5: cut = 2 exactly ON prefix sum 2, so '>=' keeps n = 2 candidates (a '>' would keep 3):
    target = 2u, token = 0 if u < 1/2 else 1.
    top_p = 0.5 + 2^-20: cut = fp32(4 * top_p) > 2, n = 3: target = fp32(3u), token = number of prefix sums
    among (1, 2) that are <= target.  Returns [(top_p, expected tokens)], logits, steps, seq ids."""
    steps = np.arange(R, dtype=np.int32)
    bits = uniform_bits(seed, seq, steps)
    u = bits.astype(np.float32) * np.float32(2.0 ** -24)
    exp_half = (u >= np.float32(0.5)).astype(np.int32)
    t3 = u * np.float32(3.0)                                  # fp32 product, as the rule computes it
    exp_beside = (t3 >= np.float32(1.0)).astype(np.int32) + (t3 >= np.float32(2.0)).astype(np.int32)
    logits = np.zeros((R, 64), dtype=np.float32)
    p_beside = float(np.float32(0.5) + np.float32(2.0 ** -20))
    return [(0.5, exp_half), (p_beside, exp_beside)], logits, steps, np.full(R, seq, dtype=np.int32)
