"""Pins for the oracle's CPO / CPS encoders, decoder and sparse convolutions.

Sources of truth used here, none of which is the oracle's own code: the worked example the
paper's text gives for Fig. 1, hand-derived small cases, the SI's closed forms for stream
sizes, round trips, structural invariants checked by a separate pure-Python walker, and brute
force against the dense definition.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from oracle import NPC, NPF
from paper_2104_08314_amd import workloads

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "fig1_worked_example.txt")


def _read_golden():
    d = {"nze": []}
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, val = line.split(":", 1)
            if key == "nze":
                d["nze"].append([int(v) for v in val.split()])
            elif key == "shape":
                d["shape"] = {k: int(v) for k, v in (kv.split("=") for kv in val.split())}
            else:
                d[key] = [int(v) for v in val.split()]
    return d


def _fig1_inputs():
    g = _read_golden()
    s = g["shape"]
    shape = (s["C"], s["H"], s["W"], s["K"], s["kh"], s["kw"], s["stride"], s["pad"])
    act = np.zeros((s["C"], s["H"], s["W"]), np.float32)
    for h, j, v in g["nze"]:
        act[0, h - s["pad"], j - s["pad"]] = v
    return g, shape, act


def test_fig1_worked_example_streams():
    g, shape, act = _fig1_inputs()
    cpo = oracle.cpo_encode(act, shape)
    cps = oracle.cps_encode(act, shape)
    assert cpo.ptr.tolist() == g["ptr"]
    assert cps.ptr.tolist() == g["ptr"]
    assert cpo.da.tolist() == [float(v) for v in g["da"]]
    assert cps.da.tolist() == [float(v) for v in g["da"]]
    assert cpo.ind.tolist() == g["in_cpo"]
    assert cps.ind.tolist() == g["in_cps"]
    # the text's own statements about ptr: ptr[8] is partition A of overlap4 with one NZE,
    # ptr[9]-ptr[8] = 4 NZEs in partition B
    assert cpo.ptr[8] == 1 and cpo.ptr[9] - cpo.ptr[8] == 4


def test_fig1_nze_10_touches_the_four_cells_the_text_names():
    g, shape, act = _fig1_inputs()
    only10 = np.zeros_like(act)
    only10[act == 10.0] = 10.0
    w = np.arange(1, 17, dtype=np.float32).reshape(1, 1, 4, 4)
    for enc in (oracle.cpo_encode, oracle.cps_encode):
        out = oracle.sparse_conv(enc(only10, shape), w)
        touched = sorted(zip(*[a.tolist() for a in np.nonzero(out[0])]))
        cells = g["touched_by_10"]
        assert touched == sorted(zip(cells[0::2], cells[1::2]))


def test_fig1_convolution_equals_dense_definition():
    _, shape, act = _fig1_inputs()
    w = (np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4) - 5.0)
    ref = oracle.conv_direct(act, w, shape)
    assert np.array_equal(oracle.sparse_conv(oracle.cpo_encode(act, shape), w), ref)
    assert np.array_equal(oracle.sparse_conv(oracle.cps_encode(act, shape), w), ref)


def test_valid_padding_nop_segment_hand_derived():
    # 3x5 map, kernel 2x3, stride 1, VALID padding: Ow = 3.  Column 0 and 4 are NOP (one
    # partition each), columns 1 and 3 overlap2, column 2 overlap3.  Derived by hand from the
    # NOP block and the overlap loop of Algorithm 1.
    act = np.array([[[1, 0, 2, 0, 3],
                     [0, 4, 0, 0, 0],
                     [5, 0, 6, 7, 0]]], np.float32)
    shape = (1, 3, 5, 1, 2, 3, 1, 0)
    cpo = oracle.cpo_encode(act, shape)
    assert cpo.ptr.tolist() == [0, 2, 3, 1, 1, 2, -1, 2, 2, -1, -1]
    assert cpo.da.tolist() == [1, 5, 3, 4, 7, 2, 6]
    assert cpo.ind.tolist() == [0, 6, 2, 4, 8, 2, 8]
    cps = oracle.cps_encode(act, shape)
    assert cps.ptr.tolist() == cpo.ptr.tolist() and cps.da.tolist() == cpo.da.tolist()
    assert cps.ind.tolist() == [0, 6, 2, 4, 8, -2, -8]
    w = np.array([[[[1, 10, 100], [1000, 10000, 100000]]]], np.float32)
    ref = oracle.conv_direct(act, w, shape)
    assert np.array_equal(oracle.sparse_conv(cpo, w), ref)
    assert np.array_equal(oracle.sparse_conv(cps, w), ref)


def test_set4_rules_hand_derived():
    # One overlap3 column (3x3 kernel, pad 1) of a 9-row map: padded rows 1..9 hold the map.
    # Column j=2 (what = 2, kw = 3): index = 2 + 3h.
    col = [1, 1, 1, 0, 0, 1, 0, 1, 1]           # map rows 0..8 -> padded rows 1..9
    act = np.zeros((1, 9, 3), np.float32)
    act[0, :, 1] = col
    act[0, :, 1] *= np.arange(1, 10)
    shape = (1, 9, 3, 1, 3, 3, 1, 1)
    cps = oracle.cps_encode(act, shape)
    # set4 of padded rows 0-3: rows 1,2,3 -> pattern 0b1110 = 14, first NZE index 2+3*1 = 5
    # rows 4-7: row 6 only  -> singleton -(2+18) = -20
    # rows 8-11 (zero extended): rows 8, 9 -> two negated indices -26, -29
    assert cps.ind.tolist() == [5, 14, -20, -26, -29]
    assert cps.da.tolist() == [1, 2, 3, 6, 8, 9]
    assert cps.ptr.tolist() == [NPF, 2, 6, -1, -1]   # overlap2 (padded columns 1, 3) empty; Ow = 3
    cpo = oracle.cpo_encode(act, shape)
    assert cpo.ind.tolist() == [5, 8, 11, 20, 26, 29]


# ---------------------------------------------------------------------------------------
# independent pure-Python walker: geometry from the definition, stream structure checks
# ---------------------------------------------------------------------------------------

def _unpack(shape):
    """(C, H, W, K, kh, kw, stride, pad) or (.., stride, pad_h, pad_w) -> nine values."""
    v = tuple(shape)
    return v if len(v) == 9 else v + (v[7],)


def _py_geometry(shape):
    C, H, W, K, kh, kw, s, ph, p = _unpack(shape)
    Ih, Iw = H + 2 * ph, W + 2 * p
    Ow = (Iw - kw) // s + 1
    cols = []
    for j in range(Iw):
        parts = [q for q in range(Ow) if q * s <= j <= q * s + kw - 1]
        cols.append(dict(j=j, m=len(parts), p0=parts[0] if parts else None,
                         real=p <= j < p + W))
    present = sorted({c["m"] - 1 for c in cols if c["m"] and c["real"]})
    return Ih, Iw, Ow, cols, present


def _py_expected_streams(act, shape, algo):
    """Straight from the prose description of the format (Sections 3.2-3.4), as Python lists."""
    C, H, W, K, kh, kw, s, ph, p = _unpack(shape)
    Ih, Iw, Ow, cols, present = _py_geometry(shape)
    pad = np.pad(act, ((0, 0), (ph, ph), (p, p)))
    top = -(-kw // s) - 1
    nop3 = s == 1 and p == 0 and kw >= 2 and Ow >= 2
    ptr, da, ind = [], [], []
    for c in range(C):
        cptr, cda, cind = [], [], []
        for t in present:
            seg = [t] + [-1] * Ow
            n = 0
            three = [0]
            for col in cols:
                if col["m"] - 1 != t or not col["real"]:
                    continue
                j = col["j"]
                what = j - col["p0"] * s
                rows = [h for h in range(Ih) if pad[c, h, j] != 0]
                cda += [float(pad[c, h, j]) for h in rows]
                if algo == 1 and t == top and t >= 1:
                    for q in range(0, Ih, 4):
                        grp = [h for h in rows if q <= h < q + 4]
                        if len(grp) >= 3:
                            cind += [what + grp[0] * kw, sum(1 << (h - q) for h in grp)]
                        else:
                            cind += [-(what + h * kw) for h in grp]
                else:
                    cind += [what + h * kw for h in rows]
                n += len(rows)
                seg[1 + col["p0"]] = n
                three.append(n)
            if nop3 and t == 0:
                cptr += three
            elif n == 0:
                cptr += [NPF]
            else:
                cptr += seg
        if not cda:
            cptr = [NPC]
        ptr += cptr
        da += cda
        ind += cind
    return ptr, da, ind


CASES = [
    (3, 7, 9, 2, 3, 3, 1, 1),
    (2, 8, 8, 2, 4, 4, 1, 1),
    (2, 9, 10, 2, 5, 5, 1, 2),
    (3, 10, 11, 2, 3, 3, 2, 1),
    (2, 11, 8, 2, 3, 2, 3, 0),
    (2, 12, 13, 2, 7, 7, 2, 3),
    (4, 6, 5, 2, 1, 3, 1, 0),
    (2, 5, 6, 2, 3, 1, 1, 0),
    (2, 6, 3, 2, 3, 3, 1, 0),     # Ow = 1: every column in one partition
    (2, 6, 4, 2, 3, 3, 1, 0),     # Ow = 2 < kw: no overlap-kw type
    (3, 13, 9, 2, 3, 5, 2, 2),
    (2, 9, 9, 2, 3, 3, 1, 2),     # more padding than overlap
    # rows and columns padded differently (.., stride, pad_h, pad_w): the 1 x n and n x 1 layers
    # of the SI's layer tables keep their map size with padding in one direction only
    (3, 9, 8, 2, 1, 7, 1, 0, 3),
    (3, 9, 8, 2, 7, 1, 1, 3, 0),
    (2, 7, 6, 2, 1, 3, 1, 0, 1),
    (2, 7, 6, 2, 3, 1, 1, 1, 0),
    (3, 7, 9, 2, 3, 3, 1, 0, 1),  # columns padded, rows not
    (3, 7, 9, 2, 3, 3, 1, 2, 0),  # rows padded, columns VALID: three-entry NOP segment
    (2, 10, 11, 2, 5, 3, 2, 1, 2),
]


@pytest.mark.parametrize("shape", CASES)
@pytest.mark.parametrize("zero_frac", [0.0, 0.5, 0.9])
def test_streams_match_prose_description(shape, zero_frac):
    act, _ = workloads.random_case(17, *shape[:8], zero_frac=zero_frac, zero_channels=1 if shape[0] > 2 else 0)
    for algo in (0, 1):
        m = oracle.encode(act, shape, algo)
        ptr, da, ind = _py_expected_streams(act, shape, algo)
        assert m.ptr.tolist() == ptr
        assert m.da.tolist() == da
        assert m.ind.tolist() == ind


@pytest.mark.parametrize("shape", CASES)
def test_round_trip_and_invariants(shape):
    C, H, W, K, kh, kw, s, ph, p = _unpack(shape)
    Ih, Iw, Ow, cols, present = _py_geometry(shape)
    covered = np.array([c["m"] > 0 for c in cols])[p:p + W]
    for seed, zero_frac in itertools.product(range(3), (0.3, 0.7)):
        act, _ = workloads.random_case(100 + seed, *shape[:8], zero_frac=zero_frac, zero_channels=1)
        # random_case leaves -0.0 where a negative draw was masked out: those are zeros
        expect = np.where((act != 0) & covered[None, None, :], act, np.float32(0.0))
        nnz = int(np.count_nonzero(expect))
        cpo, cps = oracle.cpo_encode(act, shape), oracle.cps_encode(act, shape)
        # decode(encode(x)) == x on every covered cell, bit for bit
        assert np.array_equal(oracle.decode(cpo).view(np.int32), expect.view(np.int32))
        assert np.array_equal(oracle.decode(cps).view(np.int32), expect.view(np.int32))
        # NZE count preserved: |DA| = |IN_cpo| = nnz (SI, size of DA and IN)
        assert cpo.da.size == cpo.ind.size == nnz and cps.da.size == nnz
        assert np.array_equal(cpo.da, cps.da) and np.array_equal(cpo.ptr, cps.ptr)
        assert cps.ind.size <= cpo.ind.size        # SI: CPS never needs more indices than CPO
        assert np.all(cpo.da != 0)
        assert np.all((cpo.ind >= 0) & (cpo.ind < Ih * kw))
        # all-zero channels: one NPC entry, nothing in DA / IN
        dead = [c for c in range(C) if not np.any(expect[c])]
        assert int(np.count_nonzero(cpo.ptr == NPC)) == len(dead)
        for c in dead:
            assert cpo.chan_off[0, c + 1] - cpo.chan_off[0, c] == 1
            assert cpo.ptr[cpo.chan_off[0, c]] == NPC
            assert cpo.chan_off[1, c + 1] == cpo.chan_off[1, c]
            assert cps.chan_off[2, c + 1] == cps.chan_off[2, c]
        assert cpo.chan_off[0, C] == cpo.ptr.size and cpo.chan_off[1, C] == nnz
        assert cps.chan_off[2, C] == cps.ind.size
        for c in range(C):
            assert cpo.chan_off[1, c + 1] - cpo.chan_off[1, c] == np.count_nonzero(expect[c])


def _set4_histogram(act, shape):
    """C''_k of the SI: number of set4 groups with k NZEs in the overlap-kw columns, and the
    NZE count elsewhere, computed with array operations only."""
    C, H, W, K, kh, kw, s, ph, p = _unpack(shape)
    Ih, Iw, Ow, cols, present = _py_geometry(shape)
    pad = np.pad(act, ((0, 0), (ph, ph), (p, p))) != 0
    top = -(-kw // s) - 1
    top_cols = [c["j"] for c in cols if c["real"] and c["m"] - 1 == top and top >= 1]
    other_cols = [c["j"] for c in cols if c["real"] and c["m"] > 0 and c["j"] not in top_cols]
    Ih4 = -(-Ih // 4) * 4
    grid = np.zeros((C, Ih4, Iw), bool)
    grid[:, :Ih] = pad
    per_set = grid[:, :, top_cols].reshape(C, Ih4 // 4, 4, len(top_cols)).sum(axis=2)
    hist = [int(np.count_nonzero(per_set == k)) for k in range(5)]
    return hist, int(pad[:, :, other_cols].sum())


@pytest.mark.parametrize("shape", CASES)
def test_stream_sizes_match_si_closed_forms(shape):
    C, H, W, K, kh, kw, s, ph, p = _unpack(shape)
    Ih, Iw, Ow, cols, present = _py_geometry(shape)
    act, _ = workloads.random_case(23, *shape[:8], zero_frac=0.45, zero_channels=1)
    cpo, cps = oracle.cpo_encode(act, shape), oracle.cps_encode(act, shape)
    hist, elsewhere = _set4_histogram(act, shape)
    # SI, size of IN_CPS: C'_1+2C'_2+3C'_3+4C'_4 (= NZEs outside overlap-kw) + C''_1+2C''_2+2C''_3+2C''_4
    assert cps.ind.size == elsewhere + hist[1] + 2 * hist[2] + 2 * hist[3] + 2 * hist[4]
    assert cpo.ind.size == elsewhere + hist[1] + 2 * hist[2] + 3 * hist[3] + 4 * hist[4]
    # SI, size of ptr: per channel max(1, [rho>0](NOP_size + OP_size)), an NPF shrinking a
    # (1+Ow)-entry segment to one entry
    nop3 = s == 1 and p == 0 and kw >= 2 and Ow >= 2
    full = sum(3 if (nop3 and t == 0) else 1 + Ow for t in present)
    live = sum(1 for c in range(C) if np.any(act[c][:, [cc["j"] - p for cc in cols if cc["real"] and cc["m"]]]))
    n_npf = int(np.count_nonzero(cpo.ptr == NPF))
    assert cpo.ptr.size == (C - live) + live * full - n_npf * Ow
    if s == 1 and Ow >= kw:
        # stride 1: (ceil(kw/s) - M) overlap types with M = max(1, pad), NOP of size 3 if VALID
        # (OP_size is 1+Ow when kw = 1: a single type and no NOP)
        M = max(1, p)
        if kw == 1:
            assert full == 1 + Ow
        else:
            assert full == (3 if p == 0 else 0) + max(0, kw - M) * (1 + Ow)


def test_all_zero_and_fully_dense_maps():
    shape = (3, 8, 8, 2, 3, 3, 1, 1)
    zero = np.zeros((3, 8, 8), np.float32)
    for algo in (0, 1):
        m = oracle.encode(zero, shape, algo)
        assert m.ptr.tolist() == [NPC] * 3 and m.da.size == 0 and m.ind.size == 0
    dense = np.arange(1, 3 * 64 + 1, dtype=np.float32).reshape(3, 8, 8)
    cpo, cps = oracle.cpo_encode(dense, shape), oracle.cps_encode(dense, shape)
    assert NPF not in cpo.ptr.tolist() and NPC not in cpo.ptr.tolist()
    assert cpo.ptr.size == 3 * 2 * (1 + 8)
    # padded column of 10 rows holding map rows in padded rows 1..8: set4 sizes 3, 4, 1 ->
    # 2 + 2 + 1 index entries per overlap3 column (6 such columns), 8 per overlap2 column
    assert cps.ind.size == 3 * (6 * 5 + 2 * 8)
    # -0.0 is a zero, a denormal is not
    tricky = np.zeros((1, 4, 4), np.float32)
    tricky[0, 1, 1] = -0.0
    tricky[0, 2, 2] = np.float32(1e-45)
    m = oracle.cpo_encode(tricky, (1, 4, 4, 1, 3, 3, 1, 1))
    assert m.da.size == 1 and m.da.view(np.int32)[0] == 1


def test_patterns_and_monotone_ptr_on_workload_1():
    spec = workloads.layers(1)[0]
    act, _ = workloads.make_layer(spec)
    cps = oracle.cps_encode(act, spec.shape_tuple)
    cpo = oracle.cpo_encode(act, spec.shape_tuple)
    Ow = spec.Ow
    # walk ptr: 3x3 pad 1 -> types 1 and 2 present, every live segment is 1+Ow long
    i, segs = 0, []
    for c in range(spec.C):
        if cpo.ptr[i] == NPC:
            i += 1
            continue
        for t in (1, 2):
            if cpo.ptr[i] == NPF:
                i += 1
                continue
            assert cpo.ptr[i] == t
            seg = cpo.ptr[i + 1:i + 1 + Ow]
            vals = seg[seg >= 0]
            assert np.all(np.diff(vals) >= 0) and vals.size > 0
            segs.append((c, t, int(vals[-1])))
            i += 1 + Ow
    assert i == cpo.ptr.size
    assert sum(n for _, _, n in segs) == cpo.da.size          # last cumulative entry = type count
    assert int(np.count_nonzero(cpo.ptr == NPC)) == spec.zero_channels
    # CPS: inside a run of non-negative IN entries of the overlap-kw type, odd positions are patterns
    ind = cps.ind
    pos = np.nonzero(ind >= 0)[0]
    # overlap2 entries are plain non-negative indices too: restrict to the overlap-kw parts
    for c in range(spec.C):
        lo, hi = cps.chan_off[2, c], cps.chan_off[2, c + 1]
        if hi == lo:
            continue
        # overlap2 of this channel comes first and has as many IN entries as DA entries
        pi = cps.chan_off[0, c]
        n2 = 0
        if cps.ptr[pi] != NPF:
            seg = cps.ptr[pi + 1:pi + 1 + Ow]
            n2 = int(seg[seg >= 0][-1])
        run = ind[lo + n2:hi]
        k = 0
        while k < run.size:
            if run[k] < 0:
                k += 1
            else:
                assert run[k + 1] in (7, 11, 13, 14, 15)
                k += 2
    assert pos.size > 0


def test_all_binary_4x4_maps_brute_force():
    # every one of the 2^16 binary 4x4 maps, 3x3 kernel, pad 1: Algorithm 2 and Algorithm 4 on
    # the encodings give exactly the dense definition (integer-valued fp32 arithmetic)
    shape = (1, 4, 4, 2, 3, 3, 1, 1)
    w = np.stack([np.arange(1, 10, dtype=np.float32).reshape(1, 3, 3),
                  (np.arange(9, dtype=np.float32).reshape(1, 3, 3) ** 2) - 7.0])
    bits = (np.arange(1 << 16)[:, None] >> np.arange(16)[None, :]) & 1
    maps = bits.reshape(-1, 1, 4, 4).astype(np.float32)
    # dense reference for all maps at once from the lowered matrices of single-pixel maps
    # (linearity): out(map) = sum over set pixels of out(unit map at that pixel)
    basis = np.stack([oracle.conv_direct(np.eye(16, dtype=np.float32)[i].reshape(1, 4, 4), w, shape)
                      for i in range(16)])
    ref = np.tensordot(bits.astype(np.float32), basis, axes=(1, 0))
    for i in range(0, 1 << 16):
        a = maps[i]
        cpo = oracle.cpo_encode(a, shape)
        assert cpo.da.size == int(bits[i].sum())
        assert np.array_equal(oracle.sparse_conv(cpo, w), ref[i]), i
        cps = oracle.cps_encode(a, shape)
        assert np.array_equal(oracle.sparse_conv(cps, w), ref[i]), i
        assert np.array_equal(oracle.decode(cps), a), i


def test_random_tiny_layers_brute_force():
    rng = np.random.default_rng(2024)
    done = 0
    while done < 400:
        C, K = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        H, W = int(rng.integers(1, 10)), int(rng.integers(1, 10))
        kh, kw = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        s, ph, pw = int(rng.integers(1, 4)), int(rng.integers(0, 3)), int(rng.integers(0, 3))
        # rows and columns padded alike in half of the layers, independently in the others
        if done % 2 == 0:
            pw = ph
        if H + 2 * ph < kh or W + 2 * pw < kw:
            continue
        shape = (C, H, W, K, kh, kw, s, ph) if done % 2 == 0 else (C, H, W, K, kh, kw, s, ph, pw)
        act, w = workloads.random_case(int(rng.integers(1 << 30)), *shape[:8],
                                       zero_frac=float(rng.choice([0.0, 0.3, 0.6, 0.9])),
                                       zero_channels=int(rng.integers(0, 2)), integer=True)
        ref = oracle.conv_direct(act, w, shape)
        assert np.array_equal(oracle.sparse_conv(oracle.cpo_encode(act, shape), w), ref), shape
        assert np.array_equal(oracle.sparse_conv(oracle.cps_encode(act, shape), w), ref), shape
        done += 1


@pytest.mark.parametrize("shape", [(3, 9, 8, 2, 7, 1, 1, 0), (2, 6, 11, 2, 3, 1, 1, 0), (4, 5, 5, 3, 1, 1, 1, 0),
                                   (3, 9, 8, 2, 7, 1, 1, 3, 0), (2, 6, 11, 2, 3, 1, 1, 1, 0)],
                         ids=lambda s: "x".join(map(str, s)))
def test_kw_1_streams_are_the_special_case_of_the_si(shape):
    """K_w = 1 (SI, the encoding algorithm for K_w = 1): no overlap regions, every column is its
    own sub-matrix.  Per live channel ptr is [0, running NZE count after column 0, 1, ..], IN holds
    the (padded) row of each NZE, DA the values column by column; an empty channel is one NPC
    entry.  The general encoder must produce exactly that, and CPS has nothing to pack.  The
    n x 1 layers of the SI's tables keep their map height: rows padded, columns not."""
    C, H, W = shape[:3]
    ph = shape[7]
    act, w = workloads.random_case(31, *shape[:8], zero_frac=0.6, zero_channels=1)
    ptr, da, ind = [], [], []
    for c in range(C):
        if not np.any(act[c] != 0):
            ptr.append(oracle.NPC)
            continue
        ptr.append(0)
        running = 0
        for j in range(W):
            for h in range(H):
                if act[c, h, j] != 0:
                    da.append(act[c, h, j]); ind.append(h + ph); running += 1
            ptr.append(running)
    for enc in (oracle.cpo_encode(act, shape), oracle.cps_encode(act, shape)):
        assert enc.ptr.tolist() == ptr
        assert enc.ind.tolist() == ind
        assert np.array_equal(enc.da, np.array(da, np.float32))
    # the convolution from these streams equals Eq. 1 exactly on integer-valued inputs (every product
    # and partial sum is an integer far below 2^24, so neither summation order nor precision matters)
    act_i = np.where(act != 0, np.rint(act * 8.0) + np.sign(act), 0.0).astype(np.float32)
    w_i = np.rint(w * 16.0).astype(np.float32)
    for enc in (oracle.cpo_encode(act_i, shape), oracle.cps_encode(act_i, shape)):
        assert np.array_equal(oracle.sparse_conv(enc, w_i), oracle.conv_direct(act_i, w_i, shape))


def test_every_in_entry_fits_sixteen_bits():
    """A compact map stores IN as int16.  Largest entry: the index of the last padded row and the
    last column of a partition, (Ih - 1) * kw + kw - 1 with Ih <= 256 and kw <= 11; patterns are
    below 16; CPS negates indices.  Checked on the tallest maps the library takes."""
    assert 255 * 11 + 10 < 2 ** 15
    for shape in [(2, 250, 9, 3, 3, 3, 1, 3), (1, 246, 12, 2, 11, 11, 1, 5), (2, 256, 7, 2, 5, 5, 2, 0)]:
        act, _ = workloads.random_case(5, *shape, zero_frac=0.3)
        for m in (oracle.cpo_encode(act, shape), oracle.cps_encode(act, shape)):
            assert m.ind.size and int(np.abs(m.ind).max()) < 2 ** 15
            assert np.array_equal(m.ind.astype(np.int16).astype(np.int32), m.ind)
        Ih, kw = shape[1] + 2 * shape[7], shape[5]
        assert int(oracle.cpo_encode(act, shape).ind.max()) <= (Ih - 1) * kw + kw - 1
