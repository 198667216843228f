"""CPU oracle for the sampling epilogue of the parallel draft step.  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this file; it imports
nothing of the HIP path.

What it computes.  Algorithm 1's draft line obtains the draft tokens by "sampling from the parallel draft
model": token j is a draw from q(. | x_<n, [MASK]_1..j); the T = 1.0 rows of Table 1 are such runs (the T = 0
rows take the most probable token).  With a temperature T the distribution of a row with logits l is
softmax(l / T).

* tempered(logits, T): z = l / T, lse = log sum exp z, probs = exp(z - lse): the plain definition.
* The draw uses the Gumbel-max construction (Gumbel 1954; an exact sampler: argmax_i (z_i + g_i) with g_i
  independent standard Gumbel variables is distributed as softmax(z)): g_i = -log(-log(u_i)), and the
  uniform number u_i of output row r and token i comes from a counter-based generator - a fixed hash of
  (seed, r, i) - that the HIP path implements too, so both sides draw the same numbers without exchanging any.
  Equal perturbed values go to the lower id.

The generator (uniform_u32): three rounds of the 32-bit finaliser of MurmurHash3 (Appleby, public domain:
h ^= h >> 16; h *= 0x85EBCA6B; h ^= h >> 13; h *= 0xC2B2AE35; h ^= h >> 16) over the seed's low word plus
0x9E3779B9 (row + 1), then xor the seed's high word, then xor (id * 0x9E3779B1 + 0x7F4A7C15), all modulo 2^32.
u = ((h >> 9) + 0.5) * 2^-23 lies in (0, 1) and is exact in float32.

Pins (tests/test_oracle_sampling.py, CPU): tempered() against scipy's softmax / logsumexp; the finaliser
against its published inverse (it is a bijection); uniformity of u (moments, chi-square over buckets, no
correlation between neighbouring ids, rows and seeds); the Gumbel-max draw against the exact probabilities
(chi-square over many seeds) and against a plain inversion sampler's frequencies; T -> 0 reproduces the argmax
and planted mistakes (a missing minus sign, sampling the untempered row) fail the frequency test.
"""
import numpy as np

_M32 = np.uint64(0xFFFFFFFF)


def fmix32(h):
    """The 32-bit finaliser of MurmurHash3 on an array of uint64 holding 32-bit values."""
    h = np.asarray(h, dtype=np.uint64) & _M32
    h ^= h >> np.uint64(16)
    h = (h * np.uint64(0x85EBCA6B)) & _M32
    h ^= h >> np.uint64(13)
    h = (h * np.uint64(0xC2B2AE35)) & _M32
    h ^= h >> np.uint64(16)
    return h


def uniform_u32(seed, row, ids):
    """The generator's 32-bit output for (seed, row, ids); seed: 64-bit unsigned, ids: array."""
    seed = int(seed) & 0xFFFFFFFFFFFFFFFF
    lo, hi = np.uint64(seed & 0xFFFFFFFF), np.uint64(seed >> 32)
    ids = np.asarray(ids, dtype=np.uint64)
    x = fmix32((lo + np.uint64(0x9E3779B9) * np.uint64(int(row) + 1)) & _M32)
    x = fmix32(x ^ hi)
    x = fmix32(x ^ ((ids * np.uint64(0x9E3779B1) + np.uint64(0x7F4A7C15)) & _M32))
    return x


def uniform(seed, row, ids):
    """u in (0, 1), a multiple of 2^-24 (exact in float32)."""
    return ((uniform_u32(seed, row, ids) >> np.uint64(9)).astype(np.float64) + 0.5) * 2.0 ** -23


def gumbel(seed, row, ids):
    return -np.log(-np.log(uniform(seed, row, ids)))


def tempered(logits, temperature):
    """z = logits / T, log-sum-exp of z, softmax(z); row-wise on [..., V]."""
    z = np.asarray(logits, dtype=np.float64) / float(temperature)
    mx = np.max(z, axis=-1, keepdims=True)
    lse = (mx + np.log(np.sum(np.exp(z - mx), axis=-1, keepdims=True)))[..., 0]
    return z, lse, np.exp(z - lse[..., None])


def gumbel_sample(z_row, seed, row):
    """The draw for one output row: (token id, its perturbed value, margin to the runner-up)."""
    v = np.asarray(z_row, dtype=np.float64) + gumbel(seed, row, np.arange(len(z_row)))
    order = np.lexsort((np.arange(len(v)), -v))
    best = int(order[0])
    margin = float(v[best] - v[order[1]]) if len(v) > 1 else np.inf
    return best, float(v[best]), margin
