"""Seeded synthetic inputs shaped like the paper's workloads.

This module only produces input arrays.  It holds none of the selection
method's arithmetic (no key transform, no digits, no comparisons of keys) and
is the one piece of code that both the GPU tests / benchmark and the CPU oracle
tests are fed from.

Random numbers come from a counter-based generator written out here (a 64-bit
mix of ``seed`` and the element's position), so a dataset depends only on
(seed, position), never on a library's stream or on chunking.

Recipes (the paper evaluates on synthetic distributions only: uniform [0,1] in
its Sections 5.3.1-5.3.2, narrow uniform ranges and a Zipfian in Section 5.5,
and it motivates normal-like distances and peaked token distributions in
Section 4.1):

``uniform01``        i.i.d. uniform on the 24-bit grid j/2^24, exact in fp32.
``normal``           i.i.d. N(0, sigma^2) by Box-Muller in float64, rounded to fp32.
``llm_logits``       rows of N(0, 3^2) with 8 entries per row raised by +15
                     (a "peaked" token distribution), rounded to bf16.
``uniform_range``    i.i.d. uniform in [lo, hi) in float64, rounded to fp32.
``narrow``           uniform in [1, 1 + 2^-12): every key shares its leading
                     21 bits (the paper's U[128.6, 128.7] case pushed further).
``duplicates``       90 % of positions hold one value, the rest uniform [0,1).
``specials_ramp``    +-inf, +-0 and subnormals sprinkled over a descending ramp.
``zipf``             Zipf(n, s) ranks mapped to probabilities, as in Section 5.5.
"""
from __future__ import annotations

import numpy as np

_M64 = np.uint64(0xFFFFFFFFFFFFFFFF)
_CHUNK = 1 << 22


def _mix(counter: np.ndarray, seed: int, stream: int) -> np.ndarray:
    """64-bit avalanche of (seed, stream, counter); uint64 in, uint64 out."""
    with np.errstate(over="ignore"):
        z = counter.astype(np.uint64) + np.uint64((0x9E3779B97F4A7C15 * (2 * int(seed) + 1)) & 0xFFFFFFFFFFFFFFFF)
        z = z ^ np.uint64((0xD1B54A32D192ED03 * (int(stream) + 1)) & 0xFFFFFFFFFFFFFFFF)
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
        z = (z ^ (z >> np.uint64(33))) * np.uint64(0xFF51AFD7ED558CCD)
        z = z ^ (z >> np.uint64(29))
    return z


def _u01(start: int, count: int, seed: int, stream: int) -> np.ndarray:
    """float64 uniform in [0, 1) with 53 random bits, for positions start..start+count-1."""
    c = np.arange(start, start + count, dtype=np.uint64)
    return (_mix(c, seed, stream) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def _chunks(n: int):
    for s in range(0, n, _CHUNK):
        yield s, min(_CHUNK, n - s)


def uniform01(n: int, seed: int) -> np.ndarray:
    """fp32, i.i.d. uniform on {j / 2^24}."""
    out = np.empty(n, dtype=np.float32)
    for s, m in _chunks(n):
        c = np.arange(s, s + m, dtype=np.uint64)
        out[s:s + m] = (_mix(c, seed, 0) >> np.uint64(40)).astype(np.float32) * np.float32(1.0 / (1 << 24))
    return out


def uniform_range(n: int, seed: int, lo: float, hi: float) -> np.ndarray:
    """fp32, i.i.d. uniform in [lo, hi) (drawn in float64, rounded once)."""
    out = np.empty(n, dtype=np.float32)
    for s, m in _chunks(n):
        out[s:s + m] = (lo + (hi - lo) * _u01(s, m, seed, 0)).astype(np.float32)
    return out


def _normal64(start: int, count: int, seed: int) -> np.ndarray:
    u1 = _u01(start, count, seed, 1)
    u2 = _u01(start, count, seed, 2)
    r = np.sqrt(-2.0 * np.log1p(-u1))           # 1 - u1 is in (0, 1]
    return r * np.cos(2.0 * np.pi * u2)


def normal(n: int, seed: int, sigma: float = 1.0) -> np.ndarray:
    """fp32, i.i.d. N(0, sigma^2)."""
    out = np.empty(n, dtype=np.float32)
    for s, m in _chunks(n):
        out[s:s + m] = (sigma * _normal64(s, m, seed)).astype(np.float32)
    return out


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 storage words (uint16), round to nearest even; NaN stays NaN."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = ((b.astype(np.uint64) + np.uint64(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1)).astype(np.uint64))
               >> np.uint64(16)).astype(np.uint16)
    nan = (b & np.uint32(0x7FFFFFFF)) > np.uint32(0x7F800000)
    return np.where(nan, ((b >> np.uint32(16)) | np.uint32(0x40)).astype(np.uint16), rounded)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    """bfloat16 storage words -> fp32 (exact)."""
    return (np.ascontiguousarray(h, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def llm_logits(rows: int, n: int, seed: int, sigma: float = 3.0, spikes: int = 8, spike: float = 15.0) -> np.ndarray:
    """[rows, n] bfloat16 storage words: N(0, sigma^2) logits, ``spikes`` entries per row raised by ``spike``."""
    out = np.empty((rows, n), dtype=np.uint16)
    for r in range(rows):
        x = (sigma * _normal64(r * n, n, seed)).astype(np.float32)
        # distinct spike positions: walk the row's private stream until enough distinct ones are found
        pos, j = [], 0
        want = min(spikes, n)
        while len(pos) < want:
            p = int(_mix(np.array([r * 4096 + j], dtype=np.uint64), seed, 3)[0] % np.uint64(n))
            if p not in pos:
                pos.append(p)
            j += 1
        x[pos] += np.float32(spike)
        out[r] = to_bf16_bits(x)
    return out


def narrow(n: int, seed: int, dtype=np.float32) -> np.ndarray:
    """uniform in [1, 1 + 2^-12): 2048 distinct fp32 values; a single fp16 value (1.0)."""
    out = np.empty(n, dtype=dtype)
    for s, m in _chunks(n):
        j = np.floor(_u01(s, m, seed, 0) * 2048.0)          # the 2048 fp32 values of the range, equally likely
        out[s:s + m] = (1.0 + j * 2.0 ** -23).astype(np.float32).astype(dtype)
    return out


def duplicates(n: int, seed: int, dtype=np.float32, value: float = 0.999, frac: float = 0.9) -> np.ndarray:
    """each position holds ``value`` with probability ``frac``, else uniform [0, 1)."""
    out = np.empty(n, dtype=dtype)
    for s, m in _chunks(n):
        noise = _u01(s, m, seed, 0).astype(np.float32)
        dup = _u01(s, m, seed, 4) < frac
        out[s:s + m] = np.where(dup, np.float32(value), noise).astype(dtype)
    return out


def specials_ramp(n: int, seed: int, dtype=np.float32, with_nan: bool = False) -> np.ndarray:
    """Non-increasing ramp from +A to -A (A = 1e6 for fp32, 6e4 for fp16) with special values at random
    positions: about n/2^11 each of +inf and -inf, n/64 each of +0, -0 and subnormals (random sign and
    fraction), and -- only if ``with_nan`` -- about n/256 NaNs of both signs with varied payloads."""
    is16 = np.dtype(dtype) == np.float16
    amp = 6.0e4 if is16 else 1.0e6
    u = np.concatenate([_u01(s, m, seed, 0) for s, m in _chunks(n)])
    p_inf, p_zero = 2.0 ** -11, 2.0 ** -6
    p_nan = 2.0 ** -8 if with_nan else 0.0
    edges = np.cumsum([p_inf, p_inf, p_zero, p_zero, p_zero, p_nan])
    cat = np.searchsorted(edges, u, side="right")       # 0..5 special, 6 ramp
    ramp_pos = np.flatnonzero(cat == 6)
    m = ramp_pos.size
    out = np.zeros(n, dtype=dtype)
    if m:
        t = np.arange(m, dtype=np.float64) / max(m - 1, 1)
        out[ramp_pos] = (amp - 2.0 * amp * t).astype(np.float32).astype(dtype)
    out[cat == 0] = np.inf
    out[cat == 1] = -np.inf
    out[cat == 2] = 0.0
    out[cat == 3] = -0.0
    word = np.uint16 if is16 else np.uint32
    frac_bits = 10 if is16 else 23
    nbits = 16 if is16 else 32
    bits = out.view(word)
    r = np.concatenate([_mix(np.arange(s, s + mm, dtype=np.uint64), seed, 5) for s, mm in _chunks(n)])
    frac = (r & np.uint64((1 << frac_bits) - 1)).astype(word)
    frac = np.where(frac == 0, word(1), frac).astype(word)
    sign = ((r >> np.uint64(40)) & np.uint64(1)).astype(word) << word(nbits - 1)
    sub = cat == 4
    bits[sub] = (sign | frac)[sub]
    nan = cat == 5
    exp_all = word(((1 << (nbits - 1 - frac_bits)) - 1) << frac_bits)
    bits[nan] = (sign | exp_all | frac)[nan]
    return out


def zipf(n: int, seed: int, s: float = 1.1) -> np.ndarray:
    """fp32: element i gets probability mass rank^-s / H, rank = a seeded permutation-free hash rank in 1..n."""
    out = np.empty(n, dtype=np.float32)
    h = np.sum(np.arange(1, min(n, 1 << 20) + 1, dtype=np.float64) ** -s)
    for st, m in _chunks(n):
        rank = (_mix(np.arange(st, st + m, dtype=np.uint64), seed, 6) % np.uint64(n)).astype(np.float64) + 1.0
        out[st:st + m] = (rank ** -s / h).astype(np.float32)
    return out


# ---------------------------------------------------------------------------
# the five named configurations (full sizes by default; tests pass smaller ones)
# ---------------------------------------------------------------------------

def config1(n: int = 1 << 16) -> np.ndarray:
    """single query, uniform [0,1), seed 0 (k = 32, largest)."""
    return uniform01(n, seed=0)


def config2(n: int = 1 << 24) -> np.ndarray:
    """single query, standard normal (k swept, both directions)."""
    return normal(n, seed=2000)


def config3(rows: int = 1024, n: int = 131072) -> np.ndarray:
    """batched LLM-sampling shape, bfloat16 storage words."""
    return llm_logits(rows, n, seed=3000)


def config4(n: int = 1 << 28) -> np.ndarray:
    """large-k single query, uniform [-1e6, 1e6)."""
    return uniform_range(n, seed=4000, lo=-1.0e6, hi=1.0e6)


def config5(case: str, n: int = 1 << 26, dtype=np.float32) -> np.ndarray:
    """adversarial inputs: case 'a' narrow range, 'b' 90 % duplicates, 'c' specials over a ramp."""
    if case == "a":
        return narrow(n, seed=5001, dtype=dtype)
    if case == "b":
        return duplicates(n, seed=5002, dtype=dtype)
    if case == "c":
        return specials_ramp(n, seed=5003, dtype=dtype)
    raise ValueError("case must be 'a', 'b' or 'c'")
