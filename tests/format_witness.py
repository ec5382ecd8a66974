"""Second, independent reading of the compressed layout, in numpy, for cross-checking the
C oracle (it is not the oracle and not part of the product).  Written from the layout
table alone: a chunk slot is HDR(128) | SM | [LO] | P0 | P1 | P2 | IDX | ESC, each section
padded to 128 bytes, little-endian.
"""
import numpy as np


def _pad(x):
    return -(-int(x) // 128) * 128


def section_offsets(n, dtype, G):
    """Byte offset of every section inside a slot and the slot capacity."""
    off = {}
    pos = 0
    off["HDR"] = pos; pos += 128
    off["SM"] = pos; pos += _pad(n)
    if dtype == 1:
        off["LO"] = pos; pos += _pad(2 * n)
    nb = -(-n // 8)
    for k in range(3):
        off[f"P{k}"] = pos; pos += _pad(nb)
    off["IDX"] = pos; pos += _pad(4 * (-(-n // G)))
    off["ESC"] = pos; pos += _pad(n)
    off["CAP"] = pos
    return off


def read_header(slot):
    h = bytes(slot[:128])
    return dict(magic=h[0:4], version=int.from_bytes(h[4:8], "little"), dtype=int.from_bytes(h[8:12], "little"),
                G=int.from_bytes(h[12:16], "little"), n=int.from_bytes(h[16:24], "little"),
                n_esc=int.from_bytes(h[24:32], "little"), chunk_bytes=int.from_bytes(h[32:40], "little"),
                dec=list(h[40:48]), rest=h[48:128])


def decode_slot(slot):
    """Vectorised decode of one slot; returns uint16 (bf16) or uint32 (fp32) words."""
    hd = read_header(slot)
    assert hd["magic"] == b"ZPCL" and hd["version"] == 1
    n, dtype, G = hd["n"], hd["dtype"], hd["G"]
    off = section_offsets(n, dtype, G)
    sm = slot[off["SM"]:off["SM"] + n].astype(np.uint32)
    nb = -(-n // 8)
    code = np.zeros(n, dtype=np.uint32)
    for k in range(3):
        bits = np.unpackbits(slot[off[f"P{k}"]:off[f"P{k}"] + nb], bitorder="little")[:n]
        code |= bits.astype(np.uint32) << k
    is_esc = code == 0
    # position of every zero-point in ESC = index of its group + its rank inside the group
    ng = -(-n // G)
    idx = slot[off["IDX"]:off["IDX"] + 4 * ng].view("<u4").astype(np.int64)
    grp = np.arange(n) // G
    csum = np.cumsum(is_esc) - is_esc             # zero-points before element i, whole chunk
    grp_first = csum[np.minimum(grp * G, n - 1)] if n else csum
    rank = csum - grp_first
    pos = idx[grp] + rank if n else rank
    esc = slot[off["ESC"]:off["ESC"] + hd["n_esc"]].astype(np.uint32)
    dec = np.array(hd["dec"], dtype=np.uint32)
    E = dec[code]
    if is_esc.any():
        E = E.copy()
        E[is_esc] = esc[pos[is_esc]]
    hi = ((sm & 0x80) << 8) | (E << 7) | (sm & 0x7F)
    if dtype == 0:
        return hi.astype(np.uint16)
    lo = slot[off["LO"]:off["LO"] + 2 * n].view("<u2").astype(np.uint32)
    return (hi << 16) | lo


def write_slot(words, dtype, G, dec, codes, esc_list):
    """Build a slot from an explicit (codes, zero-point list) assignment -- used by the brute
    force test to enumerate every stream a decoder could accept for a tiny input."""
    n = len(words)
    off = section_offsets(n, dtype, G)
    n_esc = len(esc_list)
    used = off["ESC"] + _pad(n_esc)
    slot = np.zeros(off["CAP"], dtype=np.uint8)
    hi = [(w >> 16) if dtype == 1 else w for w in words]
    for i in range(n):
        slot[off["SM"] + i] = ((hi[i] >> 8) & 0x80) | (hi[i] & 0x7F)
        if dtype == 1:
            slot[off["LO"] + 2 * i] = words[i] & 0xFF
            slot[off["LO"] + 2 * i + 1] = (words[i] >> 8) & 0xFF
        for k in range(3):
            slot[off[f"P{k}"] + i // 8] |= ((codes[i] >> k) & 1) << (i % 8)
    running = 0
    for i in range(n):
        if i % G == 0:
            slot[off["IDX"] + 4 * (i // G):off["IDX"] + 4 * (i // G) + 4] = np.frombuffer(
                int(running).to_bytes(4, "little"), dtype=np.uint8)
        running += codes[i] == 0
    for j, e in enumerate(esc_list):
        slot[off["ESC"] + j] = e
    hdr = b"ZPCL" + (1).to_bytes(4, "little") + int(dtype).to_bytes(4, "little") + int(G).to_bytes(4, "little") \
        + n.to_bytes(8, "little") + n_esc.to_bytes(8, "little") + used.to_bytes(8, "little") + bytes(dec)
    slot[:len(hdr)] = np.frombuffer(hdr, dtype=np.uint8)
    return slot, used
