"""Integer identities the GPU kernels rely on, checked on the CPU by enumeration (no GPU).

These do not test kernel code (that is what the GPU parity tests do); they establish the facts the
kernel comments state: the Newton reciprocal is exact for every divisor it can meet, the
reciprocal-multiply normalisation equals floor division, the folded form of Algorithm 2 equals
the printed one, and the 32-bit ScaleRelease equals the 64-bit definition.
"""
import numpy as np

M32 = (1 << 32) - 1
C1 = round(48 / 17 * 2 ** 30)
C2 = round(16 / 17 * 2 ** 32)


def recip_ceil(dn, L):
    """ceil(2^(2L+8) / dn) for dn in (2^(L-1), 2^L]: the kernel's algorithm on uint32 semantics."""
    dn = np.asarray(dn, dtype=object)
    d31 = (dn << (31 - L)) & M32
    x = (C1 - ((C2 * d31) >> 32)) << 1
    assert max(x) <= M32 and min(x) >= 0
    for _ in range(3):
        f = (1 << 31) - ((d31 * x) >> 32)
        assert min(f) >= 0
        x = ((x * f) >> 32) << 2
        assert max(x) <= M32
    q = x >> (23 - L)
    rem = (M32 - ((q * dn) & M32)) & M32
    rem = np.array([r - (1 << 32) if r >= (1 << 31) else r for r in rem], dtype=object)
    q = np.where(rem < 0, q - 1, np.where(rem >= dn, q + 1, q))
    return q + 1


def test_constants():
    assert (C1, C2) == (3031741621, 4042322161)


def test_newton_reciprocal_exact_for_every_divisor():
    for L in (16, 20):
        dn = np.arange((1 << (L - 1)) + 1, (1 << L) + 1, dtype=object)
        K = 2 * L + 8
        assert np.all(recip_ceil(dn, L) == -((-(1 << K)) // dn)), L


def test_reciprocal_multiply_is_floor_division():
    """floor(u * R / 2^(2L+8)) == u // d for every u < 256 d (sampled u, many d, both widths)."""
    rng = np.random.default_rng(0)
    for L in (16, 20):
        K = 2 * L + 8
        d = rng.integers((1 << (L - 1)) + 1, (1 << L) + 1, size=2000).astype(object)
        d[:2] = [(1 << (L - 1)) + 1, 1 << L]
        R = recip_ceil(d, L)
        for _ in range(20):
            u = np.array([int(rng.integers(0, 256 * int(x))) for x in d], dtype=object)
            assert np.all((u * R) >> K == u // d)
        for u in (np.zeros_like(d), 256 * d - 1, 255 * d, 255 * d - 1):
            assert np.all((u * R) >> K == u // d)


def test_biased_quotient_equals_saturated_floor_division():
    """byte(floor((O + 128 l) clamped / l)) ^ 0x80 == clamp(floor(O / l), -128, 127)."""
    rng = np.random.default_rng(1)
    for _ in range(20000):
        l = int(rng.integers(1, 1 << 19))
        o = int(rng.integers(-200 * l, 200 * l))
        u = min(max(o + 128 * l, 0), 256 * l - 1)
        t = u // l
        got = (t ^ 0x80) - 256 if (t ^ 0x80) >= 128 else (t ^ 0x80)
        assert got == max(-128, min(127, o // l))


def test_folded_shift_exp2_equals_printed_form():
    """((r >> 1) + s_inv) >> q == (r + 2 s_inv) >> (q + 1) for every r with r + 2 s_inv >= 0."""
    rng = np.random.default_rng(2)
    for _ in range(20000):
        s_inv = int(rng.integers(1024, 1 << 18))
        r = int(rng.integers(-2 * s_inv, s_inv // 8))
        q = int(rng.integers(0, 29))
        assert ((r >> 1) + s_inv) >> q == (r + 2 * s_inv) >> (q + 1)


def test_scale_release_32bit_form():
    """mul_hi(x << 2, alpha16 << 14) == floor(x * alpha16 / 2^16) for |x| < 2^26, alpha16 <= 2^16."""
    rng = np.random.default_rng(3)
    x = rng.integers(-(1 << 26) + 1, 1 << 26, size=20000).astype(object)
    a = rng.integers(0, 65537, size=20000).astype(object)
    a[:3] = [0, 65536, 1]
    assert np.all(((x << 2) * (a << 14)) >> 32 == (x * a) >> 16)
    assert max(abs(x << 2)) < (1 << 31) and max(a << 14) < (1 << 31)


def test_scale_release_on_offset_accumulators():
    """With y = x + 2^31 (uint32), mul_hi_u32(y, A) + C (mod 2^32) == floor(x alpha16 / 2^16) + 2^31,
    where A = alpha16 << 16, C = 2^31 - A/2, and for the identity alpha16 = 2^16: A = 2^32 - 1, C = 1."""
    rng = np.random.default_rng(4)
    x = rng.integers(-(1 << 26) + 1, 1 << 26, size=40000).astype(object)
    x[:6] = [0, 1, -1, (1 << 26) - 1, -(1 << 26) + 1, 12345]
    a = rng.integers(0, 65537, size=40000).astype(object)
    a[:8] = [0, 65536, 1, 65535, 32768, 32767, 65536, 65536]
    a[20000:30000] = 65536
    one = a >> 16
    A = ((a << 16) - one) & M32
    C = ((1 << 31) - (a << 15) + one) & M32
    y = (x + (1 << 31)) & M32
    got = (((y * A) >> 32) + C) & M32
    want = (((x * a) >> 16) + (1 << 31)) & M32
    assert np.all(got == want)


def test_offset_scores_give_the_table_index_in_one_saturating_subtraction():
    """max(0, s - m + x_p) == usub_sat(s + 2^31, m + 2^31 - x_p) on uint32 for scores in (-2^21, 2^21);
    a padded column stored as 0 gives index 0; the unsigned maximum orders offset scores like signed ones."""
    rng = np.random.default_rng(5)
    for _ in range(20000):
        x_p = int(rng.integers(1, 40960))
        s = int(rng.integers(-(1 << 21) + 1, 1 << 21))
        m = int(rng.integers(s, 1 << 21))
        sb, mb = (s + (1 << 31)) & M32, (m + (1 << 31)) & M32
        edge = (mb - x_p) & M32
        assert max(0, sb - edge) == max(0, s - m + x_p) <= x_p
        assert max(0, 0 - edge) == 0
        assert (sb <= mb) and ((-(1 << 21) + (1 << 31)) & M32) <= sb


def test_one_offset_per_score_block():
    """The 32-key blocks of a tile carry the offsets 2^30 + {0, 2^23, -2^23, -2^24} (bit patterns of 2.0, 4.0,
    1.0, 0.5).  Removing a block's own offset from its maximum and adding it to the table edge gives the
    index and the maximum of the common offset 2^30; a key beyond the sequence stands at 2^24 above the
    common offset: below every real score, index 0, and no subtraction wraps."""
    import struct
    off = 1 << 30
    deltas = [0, 1 << 23, -(1 << 23), -(1 << 24)]
    for d, f in zip(deltas, (2.0, 4.0, 1.0, 0.5)):
        assert struct.unpack("<I", struct.pack("<f", f))[0] == off + d
    masked = 1 << 24
    rng = np.random.default_rng(11)
    for _ in range(20000):
        x_p = int(rng.integers(1, 40960))
        scores = [int(v) for v in rng.integers(-(1 << 21) + 1, 1 << 21, size=4)]
        m = int(rng.integers(max(scores), 1 << 21))
        edge = (m + off - x_p) & M32                           # common offset
        block_max = []
        for s, d in zip(scores, deltas):
            sb = (s + off + d) & M32                           # what the product leaves in the block
            edge_kb = (edge + d) & M32
            assert max(0, sb - edge_kb) == max(0, s - m + x_p)
            mb = (masked + d) & M32                            # a key beyond the sequence
            assert 0 <= masked + d < (1 << 32) and max(0, mb - edge_kb) == 0
            assert mb < sb
            block_max.append(((max(sb, mb) - d) & M32))        # the block's maximum at the common offset
        assert max(block_max) == max(scores) + off
        assert all(((masked + d) - d) & M32 == masked for d in deltas)


def test_inline_assembly_never_has_a_vector_register_as_a_pure_output():
    """A pure output ("=v") may be placed in a result register of a matrix instruction that is still
    in flight (a result nobody reads counts as free), where the compiler adds no idle cycles for
    an assembly statement and the late result write then destroys the statement's value.  Every
    vector output in the kernel sources is tied to an input ("+v") instead."""
    import glob
    import os
    import re
    csrc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2604_25306_amd", "csrc")
    files = sorted(glob.glob(os.path.join(csrc, "*.h")) + glob.glob(os.path.join(csrc, "*.hip")) + glob.glob(os.path.join(csrc, "*.cpp")))
    assert files
    statements = 0
    for path in files:
        text = open(path).read()
        for m in re.finditer(r"\basm\b(?:\s+volatile)?\s*\(", text):
            depth, i = 1, m.end()
            while depth:
                depth += {"(": 1, ")": -1}.get(text[i], 0)
                i += 1
            stmt = text[m.end():i]
            statements += 1
            assert '"=v"' not in stmt and '"=&v"' not in stmt, "%s: %s" % (os.path.basename(path), stmt.strip()[:120])
    assert statements > 10
