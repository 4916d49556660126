"""Independent reader of the packed blob, written from the layout description alone
(numpy indexing; shares no code with the library).  Used to check the packer."""
import struct

import numpy as np

TILE = 16


def read_header(blob: np.ndarray) -> dict:
    raw = bytes(blob[:256])
    names = ["magic", "version", "N", "K", "g1", "g2", "g2_axis", "G", "S", "n2", "n4", "U2", "U4", "B2", "B4", "T"]
    vals = struct.unpack_from("<II14i", raw, 0)
    h = dict(zip(names, vals))
    h["nnz"] = struct.unpack_from("<q", raw, 64)[0]
    offs = struct.unpack_from("<9Q", raw, 72)
    for n, v in zip(["off_units", "off_tiles", "tile_stride", "side_bytes", "codes_off", "ocap", "r0", "r1", "total"], offs):
        h[n] = v
    h["is4_bits"] = np.frombuffer(raw[144:256], dtype=np.uint8)      # bit g: K-group g is 4-bit (if G <= 896)
    return h


def unpack(blob: np.ndarray) -> dict:
    h = read_header(blob)
    assert h["version"] == 9
    N, K, g1, g2, G, S, T = h["N"], h["K"], h["g1"], h["g2"], h["G"], h["S"], h["T"]
    axis = h["g2_axis"]
    B2, B4 = h["B2"], h["B4"]
    C = B2 + B4
    PU2, PU4 = max(1, 64 // g1), max(1, 32 // g1)            # pieces (groups) per unit
    nsub = 1 if g2 >= TILE else TILE // g2                    # g2_axis 1: blocks of g2 rows per tile
    m2_bytes = 64 * (S + 1) if axis == 0 else -(-(4 * nsub * (G + 1)) // 16) * 16
    zero2 = 64 * S if axis == 0 else 4 * nsub * G
    paper = h["r0"] == 1                                     # the paper's aligned metadata packing (g1 = 16)
    assert h["r0"] in (0, 1) and (not paper or g1 == 16)
    if paper:
        T3 = -(-h["n2"] // 3)                                 # triples of 2-bit groups
        E = 16 * (S + 1) if axis == 0 else nsub * (G + 1)     # second-order entries, zero entries included
        zero_e = 16 * S if axis == 0 else nsub * G
        off_m1b = 32 * (T3 + 1)
        off_s2 = off_m1b + 16 * (h["n4"] + 1)
        off_z2 = off_s2 + -(-(2 * E) // 16) * 16
        o0 = off_z2 + -(-E // 16) * 16
        assert h["side_bytes"] == o0 + 128 + 4 * h["ocap"] and h["ocap"] % 32 == 0
    else:
        assert h["side_bytes"] == 32 * (G + 1) + m2_bytes + 128 + 4 * h["ocap"] and h["ocap"] % 32 == 0
    assert h["codes_off"] % 128 == 0 and h["codes_off"] >= h["side_bytes"] and h["tile_stride"] % 256 == 0
    assert h["tile_stride"] >= h["codes_off"] + C * 1024 and h["total"] == blob.size
    assert h["U2"] == (h["n2"] * (g1 // 64) if g1 >= 64 else -(-h["n2"] // PU2))
    assert h["U4"] == (h["n4"] * (g1 // 32) if g1 >= 32 else -(-h["n4"] // PU4))
    units = blob[h["off_units"]: h["off_units"] + 32 * PU2 * C].view(np.uint32).reshape(4 * C, PU2, 2)
    tiles = blob[h["off_tiles"]: h["off_tiles"] + T * h["tile_stride"]].reshape(T, h["tile_stride"])
    # gaps inside a tile record are zero; the outlier block index (r1 = its offset, 0 = none) follows the codes
    oidx_off, codes_end = h["r1"], h["codes_off"] + C * 1024
    want_index = 0 < h["ocap"] <= 65535
    assert (oidx_off != 0) == want_index
    assert not tiles[:, h["side_bytes"]: h["codes_off"]].any()
    if oidx_off:
        assert oidx_off % 64 == 0 and codes_end <= oidx_off < codes_end + 64
        assert h["tile_stride"] == -(-(oidx_off + 32 * (B2 + 1)) // 256) * 256
        assert not tiles[:, codes_end: oidx_off].any() and not tiles[:, oidx_off + 32 * (B2 + 1):].any()
    else:
        assert h["tile_stride"] == -(-codes_end // 256) * 256 and not tiles[:, codes_end:].any()
    cw = np.ascontiguousarray(tiles[:, h["codes_off"]: h["codes_off"] + C * 1024]).view(np.uint32).reshape(T, C, 4, 16, 4)
    codes = np.zeros((T * TILE, K), dtype=np.uint8)
    is4 = np.full(G, 255, dtype=np.uint8)
    stream_groups = []                       # K-group of each stream group, 2-bit stream first
    m2off = {}                               # K-group -> meta2 offset recorded in the unit table
    for u in range(4 * C):
        four = u >= 4 * B2
        ul = u - 4 * B2 if four else u
        PU = PU4 if four else PU2
        width, per = (4, 32) if four else (2, 64)
        cpp = per // PU                                   # columns per piece
        words = cw[:, u // 4, u % 4]                      # [T, 16 rows, 4 dwords]
        field = np.zeros((T * TILE, per), dtype=np.uint8)
        for kl in range(per):
            w = words[:, :, (kl % 8) // 2].astype(np.uint64)
            if four:
                v = (w >> (16 * (kl % 2) + 4 * (kl // 8))) & 15
            else:
                # 2-bit unit: dword = 8 nibbles; step P = kl // 8 uses nibble nn = P % 4 + 4 * (kl % 2).
                # first 32 columns: code in nibble bits 1, 2; last 32: bit 0 of the code in nibble bit 3,
                # bit 1 of the code in bit 0 of the next nibble (wrapping inside the dword)
                nn = (kl // 8) % 4 + 4 * (kl % 2)
                if kl < 32:
                    v = (w >> (4 * nn + 1)) & 3
                else:
                    v = ((w >> (4 * nn + 3)) & 1) | (((w >> ((4 * nn + 4) % 32)) & 1) << 1)
            field[:, kl] = v.astype(np.uint8).reshape(-1)
        for q in range(PU2):
            e, e1 = int(units[u, q, 0]), int(units[u, q, 1])
            if paper:
                gi = ul * PU + q                               # g1 = 16: piece q of unit ul is stream group gi of its width
                if q >= PU or gi >= (h["n4"] if four else h["n2"]):
                    # padding piece: points at the zero entries and holds zero codes
                    assert e == 0 and (e1 & 0xFFFF) == ((16 * h["n4"]) if four else 32 * T3) and (e1 >> 16) == zero_e
                    if q < PU:
                        assert not field[:, q * cpp: (q + 1) * cpp].any()
                    continue
                k0 = e // 2
                g = k0 // g1
                assert is4[g] == 255 and k0 % g1 == 0
                is4[g] = 1 if four else 0
                si = len(stream_groups)
                assert si == (h["n2"] + gi if four else gi)
                want1 = 16 * gi if four else 32 * (gi // 3) + gi % 3
                want2 = (g // g2) * 16 if axis == 0 else si * nsub
                assert (e1 & 0xFFFF) == want1 and (e1 >> 16) == want2, (u, q, hex(e1), want1, want2)
                stream_groups.append(g)
                codes[:, k0: k0 + cpp] = field[:, q * cpp: (q + 1) * cpp]
                continue
            if (e1 & 0xFFFF) == 32 * G:                    # padding piece: points at the zero entries
                assert e == 0 and (e1 >> 16) == zero2
                if q < PU:
                    assert not field[:, q * cpp: (q + 1) * cpp].any()   # padding pieces hold zero codes
                continue
            assert q < PU and ul < (h["U4"] if four else h["U2"])
            k0 = e // 2
            g = k0 // g1
            assert is4[g] in (255, 1 if four else 0)
            is4[g] = 1 if four else 0
            if k0 % g1 == 0:
                assert (e1 & 0xFFFF) == 32 * len(stream_groups)
                stream_groups.append(g)
                m2off[g] = e1 >> 16
            else:
                assert m2off[g] == e1 >> 16 and (e1 & 0xFFFF) == 32 * stream_groups.index(g)
            codes[:, k0: k0 + cpp] = field[:, q * cpp: (q + 1) * cpp]
    assert len(stream_groups) == G and sorted(stream_groups) == list(range(G))
    bits = np.unpackbits(h["is4_bits"], bitorder="little")
    assert np.array_equal(bits[:G], is4) and not bits[G:].any() if G <= 896 else not bits.any()
    if paper:
        m1a = np.ascontiguousarray(tiles[:, : 32 * (T3 + 1)]).view(np.uint16).reshape(T, T3 + 1, TILE).astype(np.uint32)
        m1b = tiles[:, off_m1b: off_m1b + 16 * (h["n4"] + 1)].reshape(T, h["n4"] + 1, TILE)
        assert not m1a[:, T3].any() and not m1b[:, h["n4"]].any()
        s_int = np.zeros((T * TILE, G), dtype=np.uint8)
        z1 = np.zeros((T * TILE, G), dtype=np.uint8)
        for si, g in enumerate(stream_groups):
            if si < h["n2"]:
                w, pos = m1a[:, si // 3, :], si % 3
                z1[:, g] = ((w >> (2 * pos)) & 3).reshape(-1)
                s_int[:, g] = ((w >> (6, 10, 13)[pos]) & (15, 7, 7)[pos]).reshape(-1)
            else:
                b8 = m1b[:, si - h["n2"], :]
                s_int[:, g] = (b8 & 15).reshape(-1)
                z1[:, g] = (b8 >> 4).reshape(-1)
        if h["n2"] % 3:                                        # unused fields of the last triple are zero
            w = m1a[:, T3 - 1, :]
            for pos in range(h["n2"] % 3, 3):
                assert not ((w >> (2 * pos)) & 3).any() and not ((w >> (6, 10, 13)[pos]) & (15, 7, 7)[pos]).any()
        s2a = np.ascontiguousarray(tiles[:, off_s2: off_s2 + 2 * E]).view(np.uint16).reshape(T, E)
        z2a = tiles[:, off_z2: off_z2 + E].reshape(T, E)
        assert not s2a[:, zero_e:].any() and not z2a[:, zero_e:].any()
        z2h = z2a.astype(np.float16).view(np.uint16)           # the byte as the fp16 integer the logical format holds
        if axis == 0:
            s2 = s2a[:, :zero_e].reshape(T, S, TILE).transpose(0, 2, 1).reshape(T * TILE, S)[:N]
            z2 = z2h[:, :zero_e].reshape(T, S, TILE).transpose(0, 2, 1).reshape(T * TILE, S)[:N]
        else:
            NB = -(-N // g2)
            s2 = np.zeros((NB, G), dtype=np.uint16)
            z2 = np.zeros((NB, G), dtype=np.uint16)
            for si, g in enumerate(stream_groups):
                for t in range(T):
                    for sub in range(nsub):
                        n0 = t * TILE + (sub * g2 if g2 < TILE else 0)
                        if n0 >= N:
                            assert s2a[t, si * nsub + sub] == 0 and z2a[t, si * nsub + sub] == 0
                            continue
                        s2[n0 // g2, g], z2[n0 // g2, g] = s2a[t, si * nsub + sub], z2h[t, si * nsub + sub]
        m2_bytes = o0 - 32 * (G + 1)                           # so that the outlier record is found below
    if not paper:
        m1 = np.ascontiguousarray(tiles[:, : 32 * (G + 1)]).view(np.uint16).reshape(T, G + 1, TILE)
        assert not m1[:, G].any()                             # the zero entry padding pieces point at
        s_int = np.zeros((T * TILE, G), dtype=np.uint8)
        z1 = np.zeros((T * TILE, G), dtype=np.uint8)
        for sg, g in enumerate(stream_groups):
            s_int[:, g] = (m1[:, sg, :] & 0xFF).reshape(-1)
            z1[:, g] = (m1[:, sg, :] >> 8).reshape(-1)
    raw2 = np.ascontiguousarray(tiles[:, 32 * (G + 1): 32 * (G + 1) + m2_bytes])
    if paper:
        pass
    elif axis == 0:
        m2 = raw2.view(np.uint32).reshape(T, S + 1, TILE)
        assert not m2[:, S].any()
        m2 = m2[:, :S]
        for g in range(G):
            assert m2off[g] == (g // g2) * 64
        s2 = (m2 & 0xFFFF).astype(np.uint16).transpose(0, 2, 1).reshape(T * TILE, S)[:N]
        z2 = (m2 >> 16).astype(np.uint16).transpose(0, 2, 1).reshape(T * TILE, S)[:N]
    else:
        m2 = raw2[:, : 4 * nsub * (G + 1)].copy().view(np.uint32).reshape(T, G + 1, nsub)
        assert not m2[:, G].any() and not raw2[:, 4 * nsub * (G + 1):].any()
        NB = -(-N // g2)
        s2 = np.zeros((NB, G), dtype=np.uint16)
        z2 = np.zeros((NB, G), dtype=np.uint16)
        for sg, g in enumerate(stream_groups):
            assert m2off[g] == sg * 4 * nsub
            for t in range(T):
                for sub in range(nsub):
                    n0 = t * TILE + (sub * g2 if g2 < TILE else 0)
                    if n0 >= N:
                        assert m2[t, sg, sub] == 0        # blocks of rows beyond N stay zero
                        continue
                    nb = n0 // g2
                    v = int(m2[t, sg, sub])
                    if g2 > TILE and (t * TILE) % g2 != 0:
                        assert (s2[nb, g], z2[nb, g]) == (v & 0xFFFF, v >> 16)   # every tile of a block holds a copy
                    s2[nb, g], z2[nb, g] = v & 0xFFFF, v >> 16
    # outliers: one record per tile = 32 words of row starts (17 used) + ocap words
    o0 = 32 * (G + 1) + m2_bytes
    recs = np.ascontiguousarray(tiles[:, o0: o0 + 128 + 4 * h["ocap"]]).view(np.uint32).reshape(T, 32 + h["ocap"])
    row_ptr = [0]
    words = []
    fullest = 0
    for t in range(T):
        start = recs[t, :17].astype(np.int64)
        assert start[0] == 0 and np.all(np.diff(start) >= 0) and not recs[t, 17:32].any()
        cnt = int(start[16])
        fullest = max(fullest, cnt)
        assert cnt <= h["ocap"] and not recs[t, 32 + cnt:].any()        # padding words are zero
        for r in range(TILE):
            if t * TILE + r < N:
                row_ptr.append(row_ptr[-1] + int(start[r + 1] - start[r]))
            else:
                assert start[r + 1] == start[r]                         # rows beyond N are empty
        words.append(recs[t, 32: 32 + cnt])
    assert h["ocap"] == -(-fullest // 32) * 32
    if oidx_off:
        # entry [c][r]: how many words of the tile come before the first word of row r that lies in 2-bit block c
        # or later = words of earlier rows + words of row r in blocks < c (brute force over the unit table)
        oidx = np.ascontiguousarray(tiles[:, oidx_off: oidx_off + 32 * (B2 + 1)]).view(np.uint16).reshape(T, B2 + 1, TILE)
        block_of_col = np.full(K, -1, dtype=np.int64)
        pad_word = (32 * T3) if paper else 32 * G        # what word 1 of a padding 2-bit piece holds in bits 0-15
        for u in range(4 * B2):
            for q in range(PU2):
                e, e1 = int(units[u, q, 0]), int(units[u, q, 1])
                if (e1 & 0xFFFF) != pad_word:
                    block_of_col[e // 2: e // 2 + 64 // PU2] = u // 4
        for t in range(T):
            start = recs[t, :17].astype(np.int64)
            cols = (recs[t, 32: 32 + int(start[16])] & 0xFFFF).astype(np.int64)
            assert np.all(block_of_col[cols] >= 0)                      # outliers only in 2-bit groups
            for r in range(TILE):
                blk = block_of_col[cols[start[r]: start[r + 1]]]
                assert np.all(np.diff(blk) >= 0)                        # K order = block order inside a row
                for c in range(B2 + 1):
                    want = start[r + 1] if c == B2 else start[r] + int(np.sum(blk < c))
                    assert oidx[t, c, r] == want, (t, c, r, oidx[t, c, r], want)
    outl = np.concatenate(words) if words else np.zeros(0, np.uint32)
    assert outl.size == h["nnz"]
    return dict(h=h, is4=is4, codes=codes[:N], s_int=s_int[:N], z1=z1[:N], s2=s2, z2=z2,
                row_ptr=np.array(row_ptr, dtype=np.int32), col=(outl & 0xFFFF).astype(np.uint16),
                val=(outl >> 16).astype(np.uint16), pad_rows_codes=codes[N:], pad_s=s_int[N:])
