"""Pins for the oracle's 1-bit group quantizer (Alg. 1 step 1, Eq. 5 read as round-to-nearest, Sec. 3.3)
and the append of Sec. 3.1.  Nothing here re-uses the oracle's formula: the checks are closed forms,
invariants, special cases and the values the paper prints for the storage ratio (Eq. 8, Tab. 1, Tab. 4)."""
import os

import numpy as np
import pytest

from paper_2508_08256_amd import synth

F16, BF16 = 0, 1
G = 32


def _rand_K(rng, U, L, D, dtype, scale=1.0):
    x = rng.standard_normal((U, L, D)).astype(np.float32) * scale
    return synth.f32_to_words(x, dtype)


def _exact(words, dtype):
    return synth.words_to_f32(words, dtype).astype(np.float64)


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_two_levels_nearest_and_error_bound(oracle, dtype):
    rng = np.random.default_rng(10 + dtype)
    U, L, D = 3, 4 * G, 16
    K = _rand_K(rng, U, L, D, dtype, scale=3.0)
    Lu = np.full(U, L, np.int32)
    bits, s, z = oracle.quantize(K, Lu, G, dtype)
    Kt = oracle.dequantize(bits, s, z, Lu, G, dtype)
    Kx = _exact(K, dtype).reshape(U, L // G, G, D)
    mn = Kx.min(axis=2, keepdims=True)
    mx = Kx.max(axis=2, keepdims=True)
    zz = _exact(z, dtype)[:, :, None, :]
    ss = _exact(s, dtype)[:, :, None, :]
    Ktg = Kt.reshape(U, L // G, G, D)
    b = bits.reshape(U, L // G, G, D)
    # z is the group minimum exactly, s is the range up to one rounding to the storage dtype
    assert np.array_equal(zz, mn)
    eps = 2.0 ** -11 if dtype == F16 else 2.0 ** -8
    assert np.all(np.abs(ss - (mx - mn)) <= eps * (mx - mn) * (1 + 1e-6) + 1e-30)
    # every reconstructed value is one of the two levels, and it is the nearer one
    assert np.all((Ktg == zz) | (Ktg == zz + ss))
    assert np.all(np.abs(Kx - Ktg) <= ss / 2 + eps * np.abs(Kx) + eps * ss)
    dist0 = np.abs(Kx - mn)
    dist1 = np.abs(Kx - mx)
    slack = 2 * eps * (mx - mn)
    assert np.all(b[dist0 + slack < dist1] == 0)
    assert np.all(b[dist1 + slack < dist0] == 1)
    # the group's smallest element reproduces exactly, its largest to within the rounding of s
    assert np.all(Ktg[Kx == mn] == np.broadcast_to(mn, Kx.shape)[Kx == mn])
    top = Kx == mx
    assert np.all(np.abs(Ktg[top] - Kx[top]) <= eps * np.broadcast_to(mx - mn, Kx.shape)[top] + 1e-30)
    # and both levels are used in every non-constant group
    assert np.all(b[Kx == mn][np.broadcast_to(mx > mn, Kx.shape)[Kx == mn]] == 0)
    assert np.all(b[top] == 1)


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_constant_group_and_two_level_roundtrip(oracle, dtype):
    U, L, D = 1, 2 * G, 8
    x = np.zeros((U, L, D), np.float32)
    x[0, :G, :] = np.linspace(-3, 4, D, dtype=np.float32)[None, :]       # constant per channel
    rng = np.random.default_rng(5)
    lo = rng.integers(-20, 20, D).astype(np.float32)
    span = rng.integers(1, 30, D).astype(np.float32)
    pick = rng.integers(0, 2, (G, D)).astype(np.float32)
    pick[0] = 0
    pick[1] = 1
    x[0, G:, :] = lo[None, :] + span[None, :] * pick                      # already two-level, exact in 16 bit
    K = synth.f32_to_words(x, dtype)
    assert np.array_equal(synth.words_to_f32(K, dtype), x)
    Lu = np.full(U, L, np.int32)
    bits, s, z = oracle.quantize(K, Lu, G, dtype)
    Kt = oracle.dequantize(bits, s, z, Lu, G, dtype)
    assert np.array_equal(Kt, x.astype(np.float64))                       # exact round trip
    assert np.all(s[0, 0] == 0) and np.all(bits[0, :G] == 1)              # constant group: s = 0, all bits 1
    assert np.array_equal(bits[0, G:], pick.astype(np.uint8))


def test_signed_zero_is_canonical(oracle):
    x = np.zeros((1, G, 4), np.float32)
    x[0, :, 0] = -0.0
    x[0, ::2, 1] = -0.0
    x[0, :, 2] = np.where(np.arange(G) % 2 == 0, -0.0, 1.0)
    x[0, :, 3] = np.where(np.arange(G) % 2 == 0, -0.0, -1.0)
    K = synth.f32_to_words(x, F16)
    bits, s, z = oracle.quantize(K, np.array([G], np.int32), G, F16)
    assert z[0, 0, 0] == 0 and s[0, 0, 0] == 0
    assert z[0, 0, 1] == 0 and s[0, 0, 1] == 0
    assert z[0, 0, 2] == 0 and s[0, 0, 2] == 0x3C00
    assert z[0, 0, 3] == 0xBC00 and s[0, 0, 3] == 0x3C00


def test_midpoint_rounds_up(oracle):
    x = np.zeros((1, G, 1), np.float32)
    x[0, :, 0] = 0.0
    x[0, 1, 0] = 2.0
    x[0, 2, 0] = 1.0          # exactly halfway between the levels 0 and 2
    x[0, 3, 0] = 0.9990234375  # the binary16 value just below 1
    bits, s, z = oracle.quantize(synth.f32_to_words(x, F16), np.array([G], np.int32), G, F16)
    assert bits[0, 1, 0] == 1 and bits[0, 2, 0] == 1 and bits[0, 3, 0] == 0 and bits[0, 0, 0] == 0


def test_groups_run_along_tokens_per_channel(oracle):
    """A group is 32 consecutive tokens of ONE channel: metadata has shape [L/32][D] and channel c's
    range is taken over tokens only (transposing the grouping would mix the channel scales)."""
    rng = np.random.default_rng(12)
    U, L, D = 1, 3 * G, 8
    ch_scale = (2.0 ** np.arange(D)).astype(np.float32)
    x = rng.uniform(0, 1, (U, L, D)).astype(np.float32) * ch_scale
    K = synth.f32_to_words(x, F16)
    bits, s, z = oracle.quantize(K, np.array([L], np.int32), G, F16)
    assert s.shape == (U, L // G, D)
    sv = synth.words_to_f32(s, F16)
    kv = synth.words_to_f32(K, F16).reshape(U, L // G, G, D)
    rng_np = kv.max(axis=2) - kv.min(axis=2)
    assert np.allclose(sv, rng_np, rtol=2e-3)
    assert np.all(sv[..., -1] > 30 * sv[..., 0])


def test_partial_tail_group_uses_present_tokens_only(oracle):
    rng = np.random.default_rng(13)
    U, Lcap, D = 2, 4 * G, 16
    K = _rand_K(rng, U, Lcap, D, F16)
    Lu = np.array([2 * G + 5, 1], np.int32)
    bits, s, z = oracle.quantize(K, Lu, G, F16)
    for u in range(U):
        L = int(Lu[u])
        Kc = np.zeros((1, Lcap, D), np.uint16)
        Kc[0, :L] = K[u, :L]
        # pad the tail group by repeating its first present row: the range over present tokens is unchanged
        t0 = (L // G) * G
        Kc[0, L:t0 + G] = K[u, t0]
        b2, s2, z2 = oracle.quantize(Kc, np.array([t0 + G], np.int32), G, F16)
        ng = -(-L // G)
        assert np.array_equal(s[u, :ng], s2[0, :ng]) and np.array_equal(z[u, :ng], z2[0, :ng])
        assert np.array_equal(bits[u, :L], b2[0, :L])
        assert np.all(bits[u, L:] == 0)
        assert np.all(s[u, ng:] == 0) and np.all(z[u, ng:] == 0)


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_sign_symmetric_convention_is_equivalent(oracle, dtype):
    """Alg. 1 writes the codes as {-1, +1}.  With z' = mid-range and s' = half-range that alphabet
    reconstructs the same two levels as the stored {0, 1} codes with z = min, s = range."""
    rng = np.random.default_rng(14)
    U, L, D = 2, 2 * G, 32
    K = _rand_K(rng, U, L, D, dtype, scale=2.0)
    Lu = np.full(U, L, np.int32)
    bits, s, z = oracle.quantize(K, Lu, G, dtype)
    Kt = oracle.dequantize(bits, s, z, Lu, G, dtype).reshape(U, L // G, G, D)
    Kx = _exact(K, dtype).reshape(U, L // G, G, D)
    mn = Kx.min(axis=2, keepdims=True)
    mx = Kx.max(axis=2, keepdims=True)
    mid, half = (mx + mn) / 2, (mx - mn) / 2
    code = np.where(Kx >= mid, 1.0, -1.0)
    Kt_pm = code * half + mid
    eps = 2.0 ** -11 if dtype == F16 else 2.0 ** -8
    near_mid = np.abs(Kx - mid) <= 2 * eps * (mx - mn)
    ok = np.abs(Kt - Kt_pm) <= eps * (mx - mn) + 1e-30
    assert np.all(ok | near_mid)
    assert np.mean(near_mid) < (0.01 if dtype == F16 else 0.05)


@pytest.mark.parametrize("dtype", [F16, BF16])
def test_append_equals_bulk_quantize(oracle, dtype):
    """Invariant: the packed state after any number of appends equals quantizing the whole prefix."""
    rng = np.random.default_rng(15)
    U, Lcap, D = 2, 4 * G, 16
    Kfull = _rand_K(rng, U, Lcap, D, dtype)
    Vfull = _rand_K(rng, U, Lcap, D, dtype)
    L0 = np.array([G - 3, 2 * G], np.int32)
    K = np.zeros_like(Kfull)
    V = np.zeros_like(Vfull)
    for u in range(U):
        K[u, :L0[u]] = Kfull[u, :L0[u]]
        V[u, :L0[u]] = Vfull[u, :L0[u]]
    bits, s, z = oracle.quantize(K, L0, G, dtype)
    L = L0.copy()
    for step in range(G + 7):
        k_new = np.stack([Kfull[u, L[u]] for u in range(U)])
        v_new = np.stack([Vfull[u, L[u]] for u in range(U)])
        oracle.append(K, V, L, k_new, v_new, bits, s, z, G, dtype)
        L = (L + 1).astype(np.int32)
        Kp = np.zeros_like(Kfull)
        for u in range(U):
            Kp[u, :L[u]] = Kfull[u, :L[u]]
        b2, s2, z2 = oracle.quantize(Kp, L, G, dtype)
        assert np.array_equal(K, Kp)
        assert np.array_equal(bits, b2) and np.array_equal(s, s2) and np.array_equal(z, z2), step
    for u in range(U):
        assert np.array_equal(V[u, :L[u]], Vfull[u, :L[u]])


def _golden():
    rows = {}
    path = os.path.join(os.path.dirname(__file__), "golden", "car_values.txt")
    with open(path) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            kind, key, val, dec = line.split()
            rows[(kind, key)] = (float(val), int(dec))
    return rows


def test_storage_ratio_matches_printed_values(oracle):
    """Eq. 8: 1 bit per element + two 16-bit numbers per group over a 16-bit key cache = (1+32/g)/16;
    Tab. 4 prints 0.125 / 0.08 / 0.07 for g = 32 / 128 / 256, Tab. 1 prints 12.5 + 10.0 = 22.5 % at k = l/10."""
    gold = _golden()
    L, D = 1024, 128
    K = _rand_K(np.random.default_rng(16), 1, L, D, F16)
    for g in (32, 128, 256):
        bits, s, z = oracle.quantize(K, np.array([L], np.int32), g, F16)
        stored_bits = bits.size * 1 + (s.size + z.size) * 16
        ratio = stored_bits / (K.size * 16)
        assert ratio == (1 + 32 / g) / 16
        want, dec = gold[("tab4", f"g={g}")]
        assert abs(ratio - want) <= 0.5 * 10.0 ** -dec + 1e-12 or round(ratio, dec) == want, (g, ratio)
    sel = 100 * (1 + 32 / 32) / 16
    dec_pct = 100 * (L // 10 * D * 16) / (L * D * 16 - (L % 10) * D * 16)
    assert sel == gold[("tab1", "fier_sel_percent")][0]
    assert abs(dec_pct - gold[("tab1", "fier_dec_percent")][0]) < 0.05
    assert abs(sel + dec_pct - gold[("tab1", "fier_total_percent")][0]) < 0.05
    assert 2 / 16 == gold[("sec34", "quest_page16_ratio")][0] == (1 + 32 / 32) / 16
