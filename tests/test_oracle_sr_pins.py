"""Pins for the oracle's stochastic-rounding variant (CPU only).

The paper never uses stochastic rounding; the variant exists because the benchmark spec
allows one "driven by a counter-based hash the oracle reproduces".  Reading (stated in the
oracle's header): code = clamp(floor(x*inv + u)), u = B/256, B a byte of a 32-bit hash word
that four consecutive elements share; the hash is MurmurHash3's 32-bit finalizer applied to
the block counter xor a per-seed key.

What fixes it from outside the oracle: the finalizer's published test vectors, the structure
of the keyed counter hash (identities between calls), the exact arithmetic of one binary32
addition followed by floor (re-evaluated here in binary64, where that sum is exact), closed
forms (grid values stay, u = 0 gives floor, half-way values go up iff u >= 1/2), the
statistics of the variates, and unbiasedness over seeds.
"""
import numpy as np
import pytest
import torch

from exact import all_finite_bf16_bits, bf16_bits_to_f64, unpack_codes

ALL_BITS = [4, 5, 6, 8]


def bf16_bits(x):
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def variates(ref, seed, n, first=0):
    return np.array([ref.sr_u(seed, first + i) for i in range(n)], np.float64)


# ---------------------------------------------------------------------------
# the hash
# ---------------------------------------------------------------------------

def test_finalizer_matches_the_published_murmur3_vectors(ref):
    # MurmurHash3_x86_32 of the empty key is its finalizer applied to the seed: the
    # reference implementation's verification values 0 -> 0, 1 -> 0x514E28B7,
    # 0xFFFFFFFF -> 0x81F16F39.  With seed 0 the key is mix(0) = 0, so the word of block b
    # is mix(b).
    assert ref.sr_word(0, 0) == 0x00000000
    assert ref.sr_word(0, 1) == 0x514E28B7
    assert ref.sr_word(0, 0xFFFFFFFF) == 0x81F16F39


def test_keyed_counter_structure(ref):
    rng = np.random.default_rng(11)
    for _ in range(200):
        seed = int(rng.integers(0, 1 << 32))
        block = int(rng.integers(0, 1 << 32))
        # word(seed, b) = mix(b xor mix(seed)), and mix(s) is word(0, s)
        key = ref.sr_word(0, seed)
        assert ref.sr_word(seed, block) == ref.sr_word(0, block ^ key)
        # the high half of the block counter enters the key, times the golden-ratio constant
        hi = int(rng.integers(1, 1 << 20))
        assert ref.sr_word(seed, block + (hi << 32)) == ref.sr_word(seed ^ ((hi * 0x9E3779B9) & 0xFFFFFFFF), block)
    # distinct seeds give distinct streams, the same seed the same one
    a = [ref.sr_word(5, b) for b in range(64)]
    assert a == [ref.sr_word(5, b) for b in range(64)] and a != [ref.sr_word(6, b) for b in range(64)]


def test_variate_is_a_byte_of_the_block_word(ref):
    for seed in (0, 1, 12345, 0xFFFFFFFF):
        for i in list(range(40)) + [(1 << 34) + 3, (1 << 40) + 6]:
            word = ref.sr_word(seed, i >> 2)
            byte = (word >> (8 * (i & 3))) & 0xFF        # byte 0 = least significant = element 4b
            assert ref.sr_u(seed, i) == byte / 256.0
    u = variates(ref, 77, 4096)
    assert np.all((u >= 0) & (u < 1)) and np.all(u * 256 == np.floor(u * 256))


def test_variates_look_uniform_and_independent(ref):
    n = 1 << 16
    for seed in (0, 1, 0xDEADBEEF):
        b = (variates(ref, seed, n) * 256).astype(np.int64)
        counts = np.bincount(b, minlength=256)
        chi2 = ((counts - n / 256) ** 2 / (n / 256)).sum()
        assert chi2 < 255 + 6 * np.sqrt(2 * 255), chi2          # six sigma of a chi-square with 255 dof
        assert abs(b.mean() - 127.5) < 6 * 73.9 / np.sqrt(n)
        x = b - b.mean()
        for lag in (1, 2, 3, 4, 5, 128):
            r = (x[:-lag] * x[lag:]).sum() / (x * x).sum()
            assert abs(r) < 6 / np.sqrt(n), (seed, lag, r)
    # streams of different seeds are uncorrelated at equal indices
    a = variates(ref, 1, n) - 0.498
    c = variates(ref, 2, n) - 0.498
    assert abs((a * c).sum() / np.sqrt((a * a).sum() * (c * c).sum())) < 6 / np.sqrt(n)


# ---------------------------------------------------------------------------
# the rounding step, exactly
# ---------------------------------------------------------------------------

PLANTED_AMAX_BITS = [0x3F80, 0x40E0, 0x42FE, 0x4049, 0x3C4A, 0x0D80, 0x7F7F]


@pytest.mark.parametrize("bits", ALL_BITS)
@pytest.mark.parametrize("amax_bits", PLANTED_AMAX_BITS)
def test_codes_exact_all_bf16_patterns(ref, bits, amax_bits):
    G, seed = 128, 0xC0FFEE + bits
    qmax = (1 << (bits - 1)) - 1
    amax = float(bf16_bits_to_f64(np.array([amax_bits], np.uint16))[0])
    pats = all_finite_bf16_bits()
    pats = pats[np.abs(bf16_bits_to_f64(pats)) <= amax]
    per = G - 1
    n_groups = -(-pats.size // per)
    x = np.zeros((n_groups, G), np.uint16)
    x[:, 0] = amax_bits
    x[1::2, 0] |= 0x8000
    flat = np.zeros(n_groups * per, np.uint16)
    flat[:pats.size] = pats
    x[:, 1:] = flat.reshape(n_groups, per)

    codes, scales = ref.act_quant_sr(x, G, bits, seed)
    got = unpack_codes(codes, x.size, bits).reshape(n_groups, G)
    # the scales do not depend on the rounding mode
    assert np.array_equal(scales.view(np.uint32), ref.act_quant(x, G, bits)[1].view(np.uint32))

    inv = np.float32(qmax) / np.float32(amax)                     # IEEE division (pinned elsewhere)
    t = (bf16_bits_to_f64(x) * np.float64(inv)).astype(np.float32)   # exact product, one rounding
    u = variates(ref, seed, x.size).reshape(n_groups, G)
    # t + u is exact in binary64 (24-bit and 8-bit significands, exponents less than 2^29 apart,
    # or t so small that the sum rounds to u either way); one rounding to binary32, then floor
    shifted = (t.astype(np.float64) + u).astype(np.float32)
    want = np.clip(np.floor(shifted.astype(np.float64)), -qmax, qmax).astype(np.int32)
    assert np.array_equal(got, want)
    # nothing exceeds qmax (the planted extreme itself lands on +-qmax or, where amax * inv
    # rounds to just below qmax and the variate is tiny, one step inside)
    assert np.abs(got).max() == qmax and np.all(np.abs(got[:, 0]) >= qmax - 1)
    # never more than one step from the unrounded value, never below its floor
    d = got - t.astype(np.float64)
    assert np.all((d > -1.0 - 2.0 ** -16) & (d < 1.0 + 2.0 ** -16))


@pytest.mark.parametrize("bits", ALL_BITS)
def test_grid_values_are_unchanged_and_zero_variate_gives_floor(ref, bits):
    G = 128
    qmax = (1 << (bits - 1)) - 1
    rng = np.random.default_rng(bits)
    k = rng.integers(-qmax, qmax + 1, size=(64, G))
    k[:, 0] = qmax                                               # power-of-two scale 2^-3
    x = bf16_bits((k * 0.125).astype(np.float32))
    for seed in (0, 1, 99):
        codes, scales = ref.act_quant_sr(x, G, bits, seed)
        assert np.all(scales == np.float32(0.125))
        assert np.array_equal(unpack_codes(codes, x.size, bits).reshape(64, G), k)
    # half-way values k + 0.5 (qmax <= 15 keeps them in bf16's 8 bits): up iff u >= 0.5; and
    # wherever the variate is 0 the code is the floor
    if qmax <= 15:
        kk = rng.integers(-qmax, qmax, size=(64, G))
        half = (kk + 0.5) * 0.125
        half[:, 0] = qmax * 0.125
        x = bf16_bits(half.astype(np.float32))
        seed = 4242
        codes, _ = ref.act_quant_sr(x, G, bits, seed)
        got = unpack_codes(codes, x.size, bits).reshape(64, G)
        u = variates(ref, seed, x.size).reshape(64, G)
        want = kk + (u >= 0.5)
        want[:, 0] = qmax
        assert np.array_equal(got, want)
        assert (u == 0).any() and np.array_equal(got[u == 0][1:], (kk[u == 0])[1:])


def test_mean_over_seeds_is_the_unrounded_value(ref):
    # one group, power-of-two scale 1 (amax = 127): t = x exactly; 8-bit codes
    G, n_seeds = 128, 4096
    t = np.linspace(-100.0, 100.0, G).astype(np.float32)
    t = bf16_bits_to_f64(bf16_bits(t))                           # what bf16 holds
    t[0] = 127.0
    x = bf16_bits(t.astype(np.float32))
    acc = np.zeros(G)
    for seed in range(n_seeds):
        codes, scales = ref.act_quant_sr(x, G, 8, seed)
        acc += codes.view(np.int8)
    assert scales[0] == 1.0
    mean = acc / n_seeds
    frac = t - np.floor(t)
    sigma = np.sqrt(np.maximum(frac * (1 - frac), 1e-12) / n_seeds)
    # the 8-bit variate rounds the up-probability down to a multiple of 1/256
    assert np.all(mean <= t + 4 * sigma + 1e-9)
    assert np.all(mean >= t - 1 / 256 - 4 * sigma - 1e-9)
    # nearest rounding has no such property: the same test fails for it
    rn = ref.act_quant(x, G, 8)[0].view(np.int8).astype(np.float64)
    assert not np.all(np.abs(rn - t) <= 1 / 256 + 4 * sigma + 1e-9)


def test_dead_and_non_finite_groups_follow_the_same_rule(ref):
    G = 128
    x = bf16_bits(np.random.default_rng(3).standard_normal(4 * G).astype(np.float32))
    x[G:2 * G] = 0                                               # dead group
    x[2 * G + 5] = 0x7F80                                        # +Inf
    for bits in ALL_BITS:
        a = ref.act_quant_sr(x, G, bits, 7)
        b = ref.act_quant(x, G, bits)
        assert np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32))
        q = unpack_codes(a[0], x.size, bits).reshape(4, G)
        assert not q[1].any() and not q[2].any() and q[0].any() and q[3].any()


# ---------------------------------------------------------------------------
# the gradient forms: same rounding step, variate of the (output) element index
# ---------------------------------------------------------------------------

def test_gradient_store_rounds_like_the_activation_form(ref):
    G = 128
    rng = np.random.default_rng(21)
    g = (rng.standard_normal(G * 37) * 1e-3).astype(np.float32)
    g[::G] = 0.01                                                # the same abs-max in every group
    seed = 31337
    codes, scales = ref.grad_quant_sr(g, G, seed)
    inv = np.float32(127) / np.float32(0.01)
    t = (g.astype(np.float64) * np.float64(inv)).astype(np.float32)
    u = variates(ref, seed, g.size)
    want = np.clip(np.floor((t.astype(np.float64) + u).astype(np.float32).astype(np.float64)), -127, 127)
    assert np.array_equal(codes.astype(np.float64), want)
    assert np.array_equal(scales.view(np.uint32), ref.grad_quant(g, G)[1].view(np.uint32))
    assert not np.array_equal(codes, ref.grad_quant(g, G)[0])
    assert not np.array_equal(codes, ref.grad_quant_sr(g, G, seed + 1)[0])


@pytest.mark.parametrize("K", [1, 3, 8])
def test_reduce_and_accumulate_round_their_sums_stochastically(ref, K):
    # small integer codes and power-of-two scales: the fp32 sums are exact, so they can be
    # formed here and handed to the (separately pinned) gradient store
    G, n = 128, 128 * 9
    rng = np.random.default_rng(50 + K)
    stride_c, stride_s = n + 32, n // G + 3
    codes = rng.integers(-50, 51, size=(K, stride_c)).astype(np.int8)
    scales = np.full((K, stride_s), 2.0 ** -12, np.float32)
    scales[1 % K] = 2.0 ** -11
    acc = np.zeros(n, np.float64)
    for k in range(K):
        acc += codes[k, :n].astype(np.float64) * np.repeat(scales[k, :n // G], G)
    acc32 = acc.astype(np.float32)
    assert np.array_equal(acc32.astype(np.float64), acc)
    seed = 9000 + K
    want = ref.grad_quant_sr(acc32, G, seed)
    got = ref.grad_reduce_requant_sr(codes, scales, n, G, seed)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1].view(np.uint32), want[1].view(np.uint32))
    assert not np.array_equal(got[0], ref.grad_reduce_requant(codes, scales, n, G)[0])
    # accumulation: stored code * scale + new gradient (exact for these values)
    add = (rng.integers(-40, 41, size=n) * 2.0 ** -13).astype(np.float32)
    total = (codes[0, :n].astype(np.float64) * np.repeat(scales[0, :n // G], G) + add).astype(np.float32)
    want = ref.grad_quant_sr(total, G, seed)
    got = ref.grad_accumulate_sr(np.ascontiguousarray(codes[0, :n]), np.ascontiguousarray(scales[0, :n // G]),
                                 add, G, seed)
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1].view(np.uint32), want[1].view(np.uint32))
    got16 = ref.grad_accumulate_sr(np.ascontiguousarray(codes[0, :n]), np.ascontiguousarray(scales[0, :n // G]),
                                   bf16_bits(add), G, seed)
    assert np.array_equal(got16[0], want[0])                     # these addends are bf16 values


def test_results_do_not_depend_on_the_thread_count(ref):
    G = 64
    x = bf16_bits(np.random.default_rng(8).standard_normal(G * 999).astype(np.float32))
    threads = ref.max_threads()
    a = ref.act_quant_sr(x, G, 5, 3)
    ref.set_threads(1)
    b = ref.act_quant_sr(x, G, 5, 3)
    ref.set_threads(threads)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
