"""Independent Python reading of the EC-CSR device image (layout as documented in csrc/ecspmv_format.h).

Used by the tests only: it re-derives columns from bases and 8- or 4-bit deltas with the recurrence
I_k = I_0 + sum_{i<=k} dI_i (paper Section 6.2) and undoes the value permutation of Section 6.3.2, without
calling the library's own decoder.
"""
import numpy as np

IMAGE_HEADER = 256
PH = dict(ROW0=0, NROWS=1, NSLOTS=2, NRLANES=3, NRENTRIES=4, ROWSLOT_OFF=5, RCHUNK_OFF=6, RENTRY_OFF=7,
          RD_OFF=8, RV_OFF=9, NUNITS=10, UTAB_OFF=14, BD_OFF=18, BV_OFF=22, PANEL_BYTES=26, META_BYTES=27, ROWLU_OFF=28, ZERO_OFF=29,
          ROWIDX_OFF=30)


def image_header(img: np.ndarray) -> dict:
    w = img[:64].view(np.uint32)
    q = img[40:56].view(np.uint64)
    return dict(magic=int(w[0]), version=int(w[1]), m=int(w[2]), n=int(w[3]), num_panels=int(w[4]),
                threads_per_wg=int(w[5]), panel_stride=int(w[6]), meta_stride=int(w[7]), max_slots=int(w[8]),
                lds_bytes=int(w[9]), image_bytes=int(q[0]), nnz=int(q[1]), delta_bits=int(w[14]))


def panel_rows(img: np.ndarray) -> list:
    """The output rows each panel owns, in the panel's own order, read from the row index tables."""
    ih = image_header(img)
    out = []
    for p in range(ih["num_panels"]):
        P = img[IMAGE_HEADER + p * ih["panel_stride"]: IMAGE_HEADER + (p + 1) * ih["panel_stride"]]
        hdr = P[:128].view(np.uint32)
        nrows, o = int(hdr[PH["NROWS"]]), int(hdr[PH["ROWIDX_OFF"]])
        rows = P[o:o + 4 * nrows].view(np.uint32).astype(np.int64).tolist()
        assert rows and rows[0] == int(hdr[PH["ROW0"]])
        out.append(rows)
    assert sorted(r for rows in out for r in rows) == list(range(ih["m"]))      # every row is owned exactly once
    return out


def panel_bounds(img: np.ndarray) -> list:
    """Row bounds [r_0 = 0, r_1, ..., r_P = m] of the image's panels (rows dealt to panels as they come)."""
    rows = panel_rows(img)
    out = [0]
    for r in rows:
        assert r == list(range(out[-1], out[-1] + len(r)))             # contiguous and in order
        out.append(out[-1] + len(r))
    return out


def deltas_of(raw: np.ndarray, bits: int) -> np.ndarray:
    """The indices held in `raw` bytes: one delta per byte, or two per byte with the earlier one in the low nibble, or
    (bits = 16, index compression off) one 16-bit column per two bytes."""
    if bits == 16:
        return np.ascontiguousarray(raw).view(np.uint16).astype(np.int64)
    if bits == 8:
        return raw.astype(np.int64)
    out = np.empty(2 * len(raw), dtype=np.int64)
    out[0::2] = raw & 0x0F
    out[1::2] = raw >> 4
    return out


def walk(img: np.ndarray):
    """Yields dicts describing every unit of the image.

    kind 'block': g, rows (g,), cols (64,), deltas (64,), base, values (64, g) uint16
    kind 'lane':  row, cols (16,), deltas (16,), values (16,) uint16, first_of_row (bool)"""
    ih = image_header(img)
    bits = ih["delta_bits"]
    assert bits in (4, 8, 16)
    udb, ldb, cdb = 8 * bits, 2 * bits, 128 * bits           # delta bytes per unit, lane unit, full residual chunk
    for p in range(ih["num_panels"]):
        P = img[IMAGE_HEADER + p * ih["panel_stride"]: IMAGE_HEADER + (p + 1) * ih["panel_stride"]]
        hdr = P[:128].view(np.uint32)
        nrows = int(hdr[PH["NROWS"]])
        o = int(hdr[PH["ROWIDX_OFF"]])
        rowidx = P[o:o + 4 * nrows].view(np.uint32).astype(np.int64)
        o = int(hdr[PH["ROWSLOT_OFF"]])
        rowslot = P[o:o + 2 * (nrows + 1)].view(np.uint16).astype(np.int64)

        def row_of_slot(s):
            return int(np.searchsorted(rowslot, s, side="right")) - 1

        for t in (3, 2, 1, 0):
            g = 2 << t
            nu = int(hdr[PH["NUNITS"] + t])
            ut, bd, bv = int(hdr[PH["UTAB_OFF"] + t]), int(hdr[PH["BD_OFF"] + t]), int(hdr[PH["BV_OFF"] + t])
            for u in range(nu):
                ue = P[ut + 2 * (1 + g) * u: ut + 2 * (1 + g) * (u + 1)].view(np.uint16)
                d = deltas_of(P[bd + udb * u: bd + udb * (u + 1)], bits)
                cols = d if bits == 16 else int(ue[0]) + np.cumsum(d)  # I_k = I_0 + sum of deltas; 16 bits: the columns
                raw = P[bv + 128 * g * u: bv + 128 * g * (u + 1)].view(np.uint16)
                flat = np.empty(64 * g, dtype=np.uint16)               # undo: k-th 8-half group of lane j at k*128 + 8j
                for j in range(16):
                    for k in range(g // 2):
                        flat[4 * j * g + 8 * k: 4 * j * g + 8 * k + 8] = raw[k * 128 + 8 * j: k * 128 + 8 * j + 8]
                yield dict(kind="block", panel=p, g=g, base=int(ue[0]), deltas=d, cols=cols,
                           rows=np.array([rowidx[row_of_slot(int(s))] for s in ue[1:]]),
                           slots=ue[1:].astype(np.int64), values=flat.reshape(64, g))
        nlanes = int(hdr[PH["NRLANES"]])
        rc, re_, rd, rv = (int(hdr[PH[k]]) for k in ("RCHUNK_OFF", "RENTRY_OFF", "RD_OFF", "RV_OFF"))
        prev_row = -1
        o = int(hdr[PH["ROWLU_OFF"]])
        rowlu = P[o:o + 4 * (nrows + 1)].view(np.uint32).astype(np.int64)
        assert rowlu[0] == 0 and rowlu[-1] == nlanes and np.all(np.diff(rowlu) >= 0)
        z = int(hdr[PH["ZERO_OFF"]])
        assert not P[z:z + 16].any()
        for c in range((nlanes + 63) // 64):
            ch = P[rc + 16 * c: rc + 16 * (c + 1)]
            mask = int(ch[:8].view(np.uint64)[0])
            entry0, nl = (int(v) for v in ch[8:16].view(np.uint32))
            assert nl == min(64, nlanes - 64 * c) and (mask & 1)
            excl = 0
            for l in range(nl):
                seg = bin(mask & ((2 << l) - 1)).count("1") - 1
                e = P[re_ + 8 * (entry0 + seg): re_ + 8 * (entry0 + seg + 1)]
                cc = int(e[:4].view(np.int32)[0])
                _, row_local = (int(v) for v in e[4:8].view(np.uint16))
                # chunk c sits at rd + c * rv (rv: bytes from one chunk to the next): its deltas, then its values with the
                # k-th 128-bit load of lane l at k * 1024 + 16 * l
                # (a last chunk with nl < 64 lane units is stored tightly: nl delta runs padded
                # to 16 bytes, then the k-th load of lane l at 16 * nl * k + 16 * l)
                cb = rd + rv * c
                tight = nl < 64
                vb = cb + ((ldb * nl + 15) // 16 * 16 if tight else cdb)
                vs = 16 * (nl if tight else 64)
                d = deltas_of(P[cb + ldb * l: cb + ldb * (l + 1)], bits)
                v0 = P[vb + 16 * l: vb + 16 * (l + 1)].view(np.uint16)
                v1 = P[vb + vs + 16 * l: vb + vs + 16 * (l + 1)].view(np.uint16)
                cols = d if bits == 16 else cc + excl + np.cumsum(d)
                excl += 0 if bits == 16 else int(d.sum())
                assert rowlu[row_local] <= 64 * c + l < rowlu[row_local + 1]     # a row's lane units are consecutive
                yield dict(kind="lane", panel=p, row=int(rowidx[row_local]), deltas=d, cols=cols,
                           values=np.concatenate([v0, v1]), first_of_row=(row_local != prev_row),
                           head=bool((mask >> l) & 1))
                prev_row = row_local


def triples(img: np.ndarray):
    """(rows, cols, value bits) of every stored entry (padding zeros dropped), sorted by (row, col)."""
    r, c, v = [], [], []
    for u in walk(img):
        if u["kind"] == "block":
            for k in range(u["g"]):
                r.append(np.full(64, u["rows"][k]))
                c.append(u["cols"])
                v.append(u["values"][:, k])
        else:
            r.append(np.full(16, u["row"]))
            c.append(u["cols"])
            v.append(u["values"])
    if not r:
        z = np.zeros(0, dtype=np.int64)
        return z, z, z.astype(np.uint16)
    r, c, v = np.concatenate(r), np.concatenate(c), np.concatenate(v)
    keep = (v & 0x7FFF) != 0
    r, c, v = r[keep], c[keep], v[keep]
    o = np.lexsort((c, r))
    return r[o], c[o], v[o]
