"""CPU oracle of stochastic token sampling.  TEST INFRASTRUCTURE ONLY: the
product path never imports this module.

The paper keeps "token sampling" in its dynamic domain (Sec. III-A, III-C) and
names the isolation of stochastic operations as an open limitation (Sec. VI-C);
it prints no sampling algorithm.  What is written out here is the textbook
definition of temperature / top-k / top-p (nucleus) sampling, with every choice
the definition leaves open fixed as a reading:

  z_i  = float32(logit_i) * float32(1 / T)                       (fp32, one multiply)
  C    = the top_k largest z (all of them if top_k = 0 or >= V); equal values
         enter in order of increasing index
  e_i  = exp(z_i - max z),  S = sum over C
  F    = nucleus: the candidates strictly above the threshold value tau plus
         the first n_tie candidates equal to tau (increasing index), where tau is
         the largest value whose upper set {z >= tau} has mass >= top_p * S and
         n_tie = ceil((top_p * S - mass{z > tau}) / e_tau), at least 1
         (F = C if top_p = 1)
  draw = walk F in order of increasing INDEX, return the first token whose
         running sum of e exceeds u * sum_F e  (the last one if rounding leaves none)
  u    = (x0 >> 8) * 2^-24 with (x0, ..) = Philox4x32-10(counter = (draw index, 0, 0, 0),
         key = (seed low word, seed high word)); draw index = tokens produced
         since the last reset, so a reset replays the same stream.

All sums are fp64 here; the GPU kernel sums in fp32 in another order, so the
parity tests accept a token whose interval of the running sum, widened by the
rounding error of those sums, contains the target.
"""
import numpy as np

M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def philox4x32_10(counter, key):
    """Philox4x32 with 10 rounds (Salmon et al., "Parallel random numbers: as easy as 1, 2, 3").
    counter: 4 words, key: 2 words; returns 4 words."""
    c0, c1, c2, c3 = [int(x) & MASK for x in counter]
    k0, k1 = [int(x) & MASK for x in key]
    for _ in range(10):
        p0 = M0 * c0
        p1 = M1 * c2
        hi0, lo0 = p0 >> 32, p0 & MASK
        hi1, lo1 = p1 >> 32, p1 & MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & MASK, lo1, (hi0 ^ c3 ^ k1) & MASK, lo0
        k0 = (k0 + W0) & MASK
        k1 = (k1 + W1) & MASK
    return c0, c1, c2, c3


def uniform(seed, draw_index):
    """24-bit uniform in [0, 1) for the draw_index-th token since reset."""
    x0 = philox4x32_10((draw_index, 0, 0, 0), (seed & MASK, (seed >> 32) & MASK))[0]
    return (x0 >> 8) * 2.0 ** -24


def scaled_logits(logits, temperature):
    inv_t = np.float32(1.0 / float(temperature))
    return (np.asarray(logits, dtype=np.float32) * inv_t).astype(np.float32)


def candidates(z, top_k):
    """Boolean mask of the top_k largest values; equal values enter by increasing index."""
    v = z.shape[0]
    if top_k <= 0 or top_k >= v:
        return np.ones(v, dtype=bool)
    order = np.lexsort((np.arange(v), -z.astype(np.float64)))   # value descending, index ascending
    mask = np.zeros(v, dtype=bool)
    mask[order[:top_k]] = True
    return mask


def nucleus(z, e, cand, top_p):
    """Boolean mask of the nucleus inside the candidate set (see the module text)."""
    if top_p >= 1.0:
        return cand.copy()
    idx = np.flatnonzero(cand)
    s = float(e[idx].sum())
    want = float(top_p) * s
    values = np.unique(z[idx])[::-1]                 # distinct candidate values, descending
    mass_gt = 0.0
    for tau in values:
        ties = idx[z[idx] == tau]
        m_tau = float(e[ties].sum())
        if mass_gt + m_tau >= want:
            e_tau = float(e[ties[0]])
            n_tie = int(np.ceil((want - mass_gt) / e_tau))
            n_tie = min(max(n_tie, 1), ties.shape[0])
            mask = cand & (z > tau)
            mask[ties[:n_tie]] = True
            return mask
        mass_gt += m_tau
    return cand.copy()                               # rounding left the total below the target


def sample(logits, temperature, top_k, top_p, u):
    """One draw.  Returns (token, info) where info holds the pieces the parity
    tests need: z, e (fp64), candidate mask, nucleus mask, target and running sums."""
    z = scaled_logits(logits, temperature)
    cand = candidates(z, int(top_k))
    zmax = float(z[cand].max())
    e = np.where(cand, np.exp(z.astype(np.float64) - zmax), 0.0)
    keep = nucleus(z, e, cand, float(top_p))
    idx = np.flatnonzero(keep)
    csum = np.cumsum(e[idx])
    total = float(csum[-1])
    target = float(u) * total
    pos = int(np.searchsorted(csum, target, side="right"))   # first running sum > target
    if pos >= idx.shape[0]:
        pos = idx.shape[0] - 1
    info = dict(z=z, e=e, cand=cand, keep=keep, idx=idx, csum=csum, total=total, target=target)
    return int(idx[pos]), info


def sample_step(logits, temperature, top_k, top_p, seed, draw_index):
    if temperature == 0.0:
        z = np.asarray(logits, dtype=np.float32)
        return int(np.flatnonzero(z == z.max())[0]), None
    return sample(logits, temperature, top_k, top_p, uniform(seed, draw_index))
