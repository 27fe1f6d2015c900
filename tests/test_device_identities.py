"""Host-side models of two pieces of lane- and bit-level arithmetic the kernels rely on, checked
against their plain definitions: the code packing by a magic addition (q8_pack4 in
csrc/q8_device.h) and the transposed wave reduction (wave_reduce_t / t_index there)."""
import numpy as np

MAGIC = np.float32(12582912.0)          # 1.5 * 2^23


def _codes_by_magic(x, inv):
    """Low byte of the bits of fl(fl(x * inv) + 1.5 * 2^23), read as a signed byte."""
    v = (x.astype(np.float32) * np.float32(inv)).astype(np.float32)
    s = (v + MAGIC).astype(np.float32)
    return (s.view(np.uint32) & 0xFF).astype(np.uint8).view(np.int8)


def _codes_by_definition(x, inv):
    """Section 3's rule as the oracle writes it: round half to even, clamp to [-127, 127]."""
    v = (x.astype(np.float32) * np.float32(inv)).astype(np.float32)
    return np.clip(np.rint(v), -127, 127).astype(np.int8)


def test_magic_addition_rounds_like_rint_for_every_scale():
    rng = np.random.default_rng(0)
    for trial in range(200):
        n = 4096
        kind = trial % 4
        if kind == 0:
            x = rng.standard_normal(n)
        elif kind == 1:
            x = rng.uniform(-1, 1, n) * 10.0 ** rng.integers(-30, 30)
        elif kind == 2:
            x = np.tanh(rng.standard_normal(n) * 3)
        else:                                   # many exact ties: multiples of half a quantization step
            x = rng.integers(-254, 255, n) * 0.5 * rng.uniform(0.1, 3.0)
        x = x.astype(np.float32)
        m = np.abs(x).max()
        if m < 2.0 ** -100:
            continue
        inv = np.float32(127.0) / np.float32(m)
        a, b = _codes_by_magic(x, inv), _codes_by_definition(x, inv)
        assert (a == b).all(), (trial, x[a != b][:4], a[a != b][:4], b[a != b][:4])
        assert np.abs(b).max() == 127           # the largest magnitude always maps to +-127: the clamp never acts


def test_magic_addition_ties_go_to_even():
    # products that are exactly k + 0.5 for every k in range
    k = np.arange(-127, 127)
    x = (k + 0.5).astype(np.float32)
    got = _codes_by_magic(x, 1.0)
    want = np.rint(x).astype(np.int8)            # numpy rounds half to even
    assert (got == want).all()
    assert _codes_by_magic(np.array([-0.3, 0.3, -0.0, 0.0], np.float32), 1.0).tolist() == [0, 0, 0, 0]


# ---- transposed wave reduction: the stage partners and the lane bit that picks the kept half

PARTNER_XOR = [7, 1, 2, 8, 16, 32]
BIT = [2, 0, 1, 3, 4, 5]


def _t_index(lane, M):
    K = M.bit_length() - 1
    return sum(((lane >> BIT[s]) & 1) * (M >> (s + 1)) for s in range(K))


def _wave_reduce_t(vals, op):
    """vals[lane][i], 64 lanes x M values; returns what every lane holds in slot 0 at the end."""
    M = len(vals[0])
    K = M.bit_length() - 1
    cur = [list(v) for v in vals]
    for s in range(6):
        nxt = [list(v) for v in cur]
        for lane in range(64):
            p = lane ^ PARTNER_XOR[s]
            if s < K:
                half = M >> (s + 1)
                up = (lane >> BIT[s]) & 1
                for i in range(half):
                    keep = cur[lane][i + half] if up else cur[lane][i]
                    pup = (p >> BIT[s]) & 1
                    give_of_partner = cur[p][i] if pup else cur[p][i + half]
                    nxt[lane][i] = op(keep, give_of_partner)
            else:
                nxt[lane][0] = op(cur[lane][0], cur[p][0])
        cur = nxt
    return [c[0] for c in cur]


def test_transposed_reduction_delivers_every_total_to_its_lane():
    rng = np.random.default_rng(1)
    for M in (1, 2, 4, 8, 16, 32, 64):
        vals = rng.integers(-1000, 1000, (64, M)).tolist()
        totals = np.array(vals).sum(0)
        got = _wave_reduce_t(vals, lambda a, b: a + b)
        seen = set()
        for lane in range(64):
            idx = _t_index(lane, M)
            assert 0 <= idx < M
            assert got[lane] == totals[idx], (M, lane, idx)
            seen.add(idx)
        assert seen == set(range(M))             # every value has 64 / M holders
        maxima = np.array(vals).max(0)
        gotm = _wave_reduce_t(vals, max)
        assert all(gotm[lane] == maxima[_t_index(lane, M)] for lane in range(64))
