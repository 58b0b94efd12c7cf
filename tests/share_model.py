"""Test infrastructure: a Python model of the share schedule (the format and the way the builder fills
it) and an executor that multiplies with nothing but the schedule, in the kernel's order of steps.  The
format is checked against the oracle on the CPU, the HIP builder against the model record for record.

Format (csrc/gcoo_share.hpp): a super-group Q is 8 consecutive groups; ucols(Q) = its distinct columns,
ascending; band b = ucols[48b : 48b+48].  The entries of one (group, band) become blocks of 16 records
{value bits, row inside the group, 1024 * slot of the column inside the band, 0}: first the Q blocks (four
quads each: four entries of one column), then the S blocks (singles, handled four at a time).  Header of
(band, wave) = (quads, groups of four singles).
"""
import numpy as np

W = 8
BAND = 48
RUNCAP = 32
SINK = 48
UNUSED = (0, SINK, 0, 0)


def stretches(cols_band):
    """(start, end) of every run of equal columns, cut into stretches of at most RUNCAP."""
    out = []
    i, n = 0, len(cols_band)
    while i < n:
        j = i
        while j < n and cols_band[j] == cols_band[i]:
            j += 1
        for s in range(i, j, RUNCAP):
            out.append((s, min(s + RUNCAP, j)))
        i = j
    return out


def build(m, k, p, gIdxes, rows, cols, vals):
    """-> (per super-group: (ucols, NB), per stream q: list over bands of (nq, ns4, blocks[n, 16, 4] uint32))."""
    g = (m + p - 1) // p
    nQ = (g + W - 1) // W
    vbits = np.asarray(vals, np.float32).view(np.uint32)
    info, streams = [], []
    for Q in range(nQ):
        q0, q1 = Q * W, min(Q * W + W, g)
        e0, e1 = int(gIdxes[q0]), int(gIdxes[q1])
        ucols = np.unique(cols[e0:e1])
        NB = (len(ucols) + BAND - 1) // BAND
        info.append((ucols, NB))
        for w in range(W):
            q = q0 + w
            s, e = (int(gIdxes[q]), int(gIdxes[q + 1])) if q < g else (0, 0)
            gc = cols[s:e]
            place = np.searchsorted(ucols, gc) if e > s else np.zeros(0, np.int64)
            bands = []
            for b in range(NB):
                lo = int(np.searchsorted(place, BAND * b, "left"))
                hi = int(np.searchsorted(place, BAND * b + BAND, "left"))
                quads, singles = [], []
                for (a, z) in stretches(gc[lo:hi]):
                    full = (z - a) & ~3
                    for x in range(a, a + full, 4):
                        quads.append([lo + x + u for u in range(4)])
                    singles.extend(lo + x for x in range(a + full, z))
                nq, ns4 = len(quads), (len(singles) + 3) // 4

                def record(i):
                    return (int(vbits[s + i]), int(rows[s + i]) - q * p, 1024 * (int(place[i]) - BAND * b), 0)
                recs = []
                for quad in quads:
                    recs.extend(record(i) for i in quad)
                recs.extend([UNUSED] * (16 * ((nq + 3) // 4) - 4 * nq))
                recs.extend(record(i) for i in singles)
                recs.extend([UNUSED] * (16 * ((ns4 + 3) // 4) - len(singles)))
                blocks = np.array(recs, np.uint32).reshape(-1, 16, 4) if recs else np.zeros((0, 16, 4), np.uint32)
                bands.append((nq, ns4, blocks))
            streams.append(bands)
    return info, streams


def execute(m, k, p, N, info, streams, B):
    """C (fp64) from the schedule alone, in the kernel's order: per band first the quads (one B row per
    quad, taken from its first record), then the singles four at a time (the unused records included)."""
    g = (m + p - 1) // p
    C = np.zeros((g * p + W * SINK + SINK + 1, N))
    B64 = B.astype(np.float64)
    for q, bands in enumerate(streams):
        Q = q // W
        ucols, NB = info[Q]
        assert len(bands) == NB
        sums = np.zeros((SINK + 1, N))
        for b, (nq, ns4, blocks) in enumerate(bands):
            band_rows = ucols[BAND * b: BAND * b + BAND]
            flat = blocks.reshape(-1, 4)
            nqb = (nq + 3) // 4
            assert len(blocks) == nqb + (ns4 + 3) // 4
            for j in range(nq):
                off = int(flat[4 * j, 2])
                assert off % 1024 == 0 and off // 1024 < len(band_rows)
                brow = B64[band_rows[off // 1024]]
                for u in range(4):
                    val, row, o2, _ = flat[4 * j + u]
                    assert o2 == off and row < p
                    sums[row] += float(np.uint32(val).view(np.float32)) * brow
            base = 16 * nqb
            for j in range(4 * ns4):
                val, row, off, _ = flat[base + j]
                assert off % 1024 == 0 and off // 1024 < max(len(band_rows), 1) and row <= SINK
                if row == SINK:
                    assert val == 0
                    continue
                sums[row] += float(np.uint32(val).view(np.float32)) * B64[band_rows[off // 1024]]
        if q < g:
            C[q * p: q * p + p] = sums[:p]
    return C[:m]
