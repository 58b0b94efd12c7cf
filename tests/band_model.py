"""Test infrastructure: a Python model of the band schedule (the format and the way the builder
fills it) and an executor that multiplies with nothing but the streams, so that the format can
be checked against the oracle on the CPU and the HIP builder against the model bit for bit.

Two shapes: W = 8 waves (groups of 17..32 rows) and W = 16 (groups of at most 16 rows).

Format (per group stream, 32-bit words):
  stream(q) = pre-block, then for every band b of the super-group Q = q // W the blocks of (q, b)
  block = 12 header words + chunks; at most 256 (W = 8) or 128 (W = 16) words
    w0  n1 | n2<<8 | n4<<16 | n8<<24      chunk counts per type
    w1  bit0: last block of its band; bits 1..2: piece slots in use in the last T1 chunk (0 = all four / none);
        bits 8..15: columns of the next band (first block of a band / pre-block only)
    w2  words from this block's start to the first block of the next band (first block of a band / pre-block only)
    w3  words of this block
    w4..w11  B rows that wave w = q % W loads for the next band (slot t*W + w, t < 64/W; 0 where there is none)
  chunk types: T1 4 runs x 1 entry (8 words), T2 4 x 2 (12), T4 2 x 4 (12), T8 1 x 8 (12)
"""
import numpy as np
R = 64; HDR = 12
def waves_of(p): return 16 if p <= 16 else 8
def seg_of(W): return 68 if W == 8 else 24
def block_max_of(W): return 256 if W == 8 else 128
TYPES = (1, 2, 4, 8); JT = {1: 4, 2: 4, 4: 2, 8: 1}; SZ = {1: 8, 2: 12, 4: 12, 8: 12}

def pieces_of_run(ell):
    out = []; x = 0
    while ell - x >= 8: out.append((x, 8)); x += 8
    r = ell - x
    for t in (4, 2, 1):
        if r & t: out.append((x, t)); x += t
    return out

def build(m, k, p, gIdxes, rows, cols, vals):
    G = waves_of(p); SEG = seg_of(G)
    g = (m + p - 1) // p; nQ = (g + G - 1) // G
    streams = []; info = []
    for Q in range(nQ):
        q0, q1 = Q * G, min(Q * G + G, g)
        e0, e1 = int(gIdxes[q0]), int(gIdxes[q1])
        ucols = np.unique(cols[e0:e1]); nU = len(ucols); NB = (nU + R - 1) // R
        info.append((ucols, NB))
        for w in range(G):
            q = q0 + w
            words = []
            def loader_ids(b):   # ids for band b
                n = max(0, min(R, nU - R * b)); ids = [0] * 8
                for t in range(R // G):
                    if t * G + w < n: ids[t] = int(ucols[R * b + t * G + w])
                return n, ids
            if q < g: s, e = int(gIdxes[q]), int(gIdxes[q + 1])
            else: s = e = 0
            gc = cols[s:e]; gr = rows[s:e] - q * p; gv = vals[s:e]
            rank = np.searchsorted(ucols, gc) if e > s else np.zeros(0, np.int64)
            band_blocks = []
            for b in range(NB):
                lo = np.searchsorted(rank, R * b, 'left'); hi = np.searchsorted(rank, R * b + R, 'left')
                # segments of capped runs, walked the way the builder walks them
                RUNCAP = 32
                seglist = []
                cur = lo
                while True:
                    seg_end = cur + SEG
                    if seg_end >= hi:
                        seg_end = hi
                    else:
                        c = gc[seg_end]; rs = seg_end
                        while rs > cur and gc[rs - 1] == c: rs -= 1
                        cs = rs + (seg_end - rs) // RUNCAP * RUNCAP
                        if cs != seg_end:
                            stop = min(cs + RUNCAP, hi)
                            while seg_end < stop and gc[seg_end] == c: seg_end += 1
                    runs = []
                    i = cur
                    while i < seg_end:
                        j = i
                        while j < seg_end and j < i + RUNCAP and gc[j] == gc[i]: j += 1
                        runs.append((i, j)); i = j
                    seglist.append(runs)
                    cur = seg_end
                    if cur >= hi: break
                blocks = []
                for runs in seglist:
                    lists = {t: [] for t in TYPES}
                    for (i, j) in runs:
                        slot = int(rank[i]) - R * b
                        for (x, t) in pieces_of_run(j - i):
                            lists[t].append((slot, i + x))
                    # pieces that would leave a chunk of 4s or 2s partly filled are halved and join the
                    # end of the next smaller type's list (the two halves in order)
                    for t in (4, 2):
                        J = JT[t]; keep = len(lists[t]) // J * J
                        for (sl, st) in lists[t][keep:]:
                            lists[t // 2] += [(sl, st), (sl, st + t // 2)]
                        del lists[t][keep:]
                    body = []
                    counts = {}
                    for t in TYPES:
                        J = JT[t]; n = (len(lists[t]) + J - 1) // J; counts[t] = n
                        for c in range(n):
                            ch = lists[t][c * J:(c + 1) * J]
                            pad = J - len(ch)
                            offs = [sl * 1024 for (sl, _) in ch] + [0] * pad
                            rws = []; vls = []
                            for (sl, st) in ch:
                                rws += [int(gr[st + u]) for u in range(t)]; vls += [np.float32(gv[st + u]) for u in range(t)]
                            rws += [p] * (pad * t); vls += [np.float32(0)] * (pad * t)
                            wds = []
                            if t in (1, 2):
                                wds += [offs[0] | offs[1] << 16, offs[2] | offs[3] << 16]
                            elif t == 4:
                                wds += [offs[0] | offs[1] << 16]
                            else:
                                wds += [offs[0]]
                            rb = bytes(rws) + bytes((-len(rws)) % 4)
                            wds += list(np.frombuffer(rb, np.uint32))
                            while len(wds) % 4: wds.append(0)
                            wds += list(np.array(vls, np.float32).view(np.uint32))
                            assert len(wds) == SZ[t], (t, len(wds))
                            body += wds
                    assert all(n < 256 for n in counts.values())
                    counts["rem"] = len(lists[1]) % 4
                    blocks.append((counts, body))
                band_blocks.append(blocks)
            # assemble with headers
            def hdr(counts, last, ncn, delta, size, ids):
                w0 = counts[1] | counts[2] << 8 | counts[4] << 16 | counts[8] << 24
                return [w0, (1 if last else 0) | counts.get("rem", 0) << 1 | ncn << 8, delta, size] + ids
            sizes = [[HDR + len(body) for (_, body) in blocks] for blocks in band_blocks]
            for blocks in sizes:
                for sz in blocks: assert sz <= block_max_of(G), sz
            n0, ids0 = loader_ids(0)
            words += hdr({1: 0, 2: 0, 4: 0, 8: 0}, True, n0, HDR, HDR, ids0)
            for b, blocks in enumerate(band_blocks):
                nn, ids = loader_ids(b + 1)
                tot = sum(sizes[b])
                for i, (counts, body) in enumerate(blocks):
                    first = i == 0
                    words += hdr(counts, i == len(blocks) - 1, nn if first else 0, tot if first else 0, sizes[b][i], ids if first else [0] * 8)
                    words += body
            streams.append(np.array(words, dtype=np.uint32))
    return streams, info

def execute(m, k, p, N, streams, info, B):
    """C = A x B from the streams alone (fp64), following the kernel's steps."""
    G = waves_of(p)
    g = (m + p - 1) // p; C = np.zeros((g * p + 1, N))
    nQ = len(info)
    for Q in range(nQ):
        ucols, NB = info[Q]
        for w in range(G):
            q = Q * G + w
            st = streams[Q * G + w]; pos = 0
            acc = np.zeros((p + 1, N))
            # pre-block
            assert st[pos + 3] == HDR and (st[pos + 1] & 1)
            lds = {}     # slot -> B row id, for the band being processed
            def load(hpos):
                n = int(st[hpos + 1] >> 8) & 255; d = {}
                for t in range(R // G):
                    if t * G + w < n: d[t * G + w] = int(st[hpos + 4 + t])
                for t in range(R // G, 8): assert st[hpos + 4 + t] == 0
                return n, d
            nxt_n, mine = load(pos)
            # the other waves' rows: take from ucols (the model checks only its own ids)
            pos += int(st[pos + 2])
            for b in range(NB):
                n = nxt_n
                band_rows = {i: int(ucols[R * b + i]) for i in range(n)}
                for sl, rid in mine.items(): assert band_rows[sl] == rid
                first = True
                while True:
                    w0 = int(st[pos]); fl = int(st[pos + 1]); size = int(st[pos + 3])
                    if first:
                        nxt_n, mine = load(pos); nextpos = pos + int(st[pos + 2]); first = False
                    cnt = {1: w0 & 255, 2: w0 >> 8 & 255, 4: w0 >> 16 & 255, 8: w0 >> 24 & 255}
                    rem = fl >> 1 & 3
                    assert rem == 0 or cnt[1] > 0
                    at = pos + HDR
                    for t in TYPES:
                        J = JT[t]
                        for c in range(cnt[t]):
                            ch = st[at:at + SZ[t]]; at += SZ[t]
                            if t in (1, 2): offs = [ch[0] & 0xffff, ch[0] >> 16, ch[1] & 0xffff, ch[1] >> 16]; nr = 2
                            elif t == 4: offs = [ch[0] & 0xffff, ch[0] >> 16]; nr = 1
                            else: offs = [ch[0]]; nr = 1
                            nrw = (J * t + 3) // 4
                            rb = ch[nr:nr + nrw].tobytes()
                            vo = (nr + nrw + 3) // 4 * 4
                            vv = ch[vo:vo + J * t].view(np.float32)
                            for j in range(J):
                                assert offs[j] % 1024 == 0
                                sl = int(offs[j]) // 1024
                                unused = t == 1 and c == cnt[1] - 1 and rem and j >= rem     # a slot the kernel may skip
                                for u in range(t):
                                    r = rb[j * t + u]; a = float(vv[j * t + u])
                                    assert r <= p
                                    if unused: assert r == p and a == 0.0
                                    if r == p: assert a == 0.0 and (t > 1 or unused); continue
                                    acc[r] += a * B[band_rows[sl]].astype(np.float64)
                    assert at == pos + size
                    pos += size
                    if fl & 1: break
                assert pos == nextpos
            assert pos == len(st)
            if q < g: C[q * p:q * p + p] = acc[:p]
    return C[:m]

