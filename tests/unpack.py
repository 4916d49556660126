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
    for n, v in zip(["unit2", "unit4", "codes2", "codes4", "meta1", "meta2", "otile"], offs[:7]):
        h["off_" + n] = v
    h["ocap"], h["off_total"] = offs[7], offs[8]
    return h


def unpack(blob: np.ndarray) -> dict:
    h = read_header(blob)
    N, K, g1, g2, G, S, T = h["N"], h["K"], h["g1"], h["g2"], h["G"], h["S"], h["T"]
    unit2 = blob[h["off_unit2"]: h["off_unit2"] + 32 * h["B2"]].view(np.uint32).reshape(-1, 2)
    unit4 = blob[h["off_unit4"]: h["off_unit4"] + 32 * h["B4"]].view(np.uint32).reshape(-1, 2)
    c2 = blob[h["off_codes2"]: h["off_codes2"] + T * h["B2"] * 1024].view(np.uint32).reshape(T, h["B2"], 4, 16, 4)
    c4 = blob[h["off_codes4"]: h["off_codes4"] + T * h["B4"] * 1024].view(np.uint32).reshape(T, h["B4"], 4, 16, 4)
    codes = np.zeros((T * TILE, K), dtype=np.uint8)
    is4 = np.full(G, 255, dtype=np.uint8)
    stream_groups = []                       # K-group of each stream group, 2-bit stream first
    group_of_super = {}
    for u in range(4 * h["B2"]):
        e, e1 = int(unit2[u, 0]), int(unit2[u, 1])
        if e & 0x80000000:
            assert u >= h["U2"] and e == 0x80000000 and e1 == 0
            assert not c2[:, u // 4, u % 4].any()        # padding units are zero
            continue
        k0 = e // 2
        g = k0 // g1
        is4[g] = 0
        assert (e1 >> 16) == (g // g2) * 64
        if k0 % g1 == 0:
            assert (e1 & 0xFFFF) == 32 * len(stream_groups)
            stream_groups.append(g)
        words = c2[:, u // 4, u % 4]                      # [T, 16 rows, 4 dwords]
        for kl in range(64):
            d, sh = (kl % 8) // 2, 16 * (kl % 2) + 2 * (kl // 8)
            codes[:, k0 + kl] = ((words[:, :, d] >> sh) & 3).reshape(-1)
    for u in range(4 * h["B4"]):
        e, e1 = int(unit4[u, 0]), int(unit4[u, 1])
        if e & 0x80000000:
            assert u >= h["U4"] and e == 0x80000000 and e1 == 0
            assert not c4[:, u // 4, u % 4].any()
            continue
        k0 = e // 2
        g = k0 // g1
        is4[g] = 1
        assert (e1 >> 16) == (g // g2) * 64
        if k0 % g1 == 0:
            assert (e1 & 0xFFFF) == 32 * len(stream_groups)
            stream_groups.append(g)
        words = c4[:, u // 4, u % 4]
        for kl in range(32):
            d, sh = (kl % 8) // 2, 16 * (kl % 2) + 4 * (kl // 8)
            codes[:, k0 + kl] = ((words[:, :, d] >> sh) & 15).reshape(-1)
    assert len(stream_groups) == G and sorted(stream_groups) == list(range(G))
    m1 = blob[h["off_meta1"]: h["off_meta1"] + T * G * TILE * 2].view(np.uint16).reshape(T, G, TILE)
    s_int = np.zeros((T * TILE, G), dtype=np.uint8)
    z1 = np.zeros((T * TILE, G), dtype=np.uint8)
    for sg, g in enumerate(stream_groups):
        s_int[:, g] = (m1[:, sg, :] & 0xFF).reshape(-1)
        z1[:, g] = (m1[:, sg, :] >> 8).reshape(-1)
    m2 = blob[h["off_meta2"]: h["off_meta2"] + T * S * TILE * 4].view(np.uint32).reshape(T, S, TILE)
    s2 = (m2 & 0xFFFF).astype(np.uint16).transpose(0, 2, 1).reshape(T * TILE, S)
    z2 = (m2 >> 16).astype(np.uint16).transpose(0, 2, 1).reshape(T * TILE, S)
    # outliers: one record per tile = 32 words of row starts (17 used) + ocap words
    rec_words = 32 + h["ocap"]
    recs = blob[h["off_otile"]: h["off_otile"] + 4 * T * rec_words].view(np.uint32).reshape(T, rec_words)
    assert h["ocap"] % 32 == 0
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
    outl = np.concatenate(words) if words else np.zeros(0, np.uint32)
    assert outl.size == h["nnz"]
    return dict(h=h, is4=is4, codes=codes[:N], s_int=s_int[:N], z1=z1[:N], s2=s2[:N], z2=z2[:N],
                row_ptr=np.array(row_ptr, dtype=np.int32), col=(outl & 0xFFFF).astype(np.uint16),
                val=(outl >> 16).astype(np.uint16), pad_rows_codes=codes[N:], pad_s=s_int[N:])
