"""CPU oracle for the compressed expert pool: TEST INFRASTRUCTURE, not a product path.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this
module.  It shares no code with the HIP library and never calls it.

What it follows.  The paper's compressed-GPU backend (Sec. 4.2 "Compressed GPU backend",
Sec. 5 "Expert memory backends", App. "Expert-weight compressibility") Huffman-codes only
the 8 exponent bits of every BF16 routed-expert weight and leaves sign and mantissa bits
unchanged; decoding must give back the original tensor exactly.  The paper prints no
stream format, so everything below the level "Huffman over the exponent byte, raw
sign/mantissa, lossless" is this build's container, written here from its specification:

  split      w (uint16) -> exponent symbol e = (w >> 7) & 0xFF,
             raw byte sm = ((w >> 8) & 0x80) | (w & 0x7F)   (sign in bit 7, 7 mantissa bits)
  lengths    optimal prefix code over the used symbols of one (layer, tensor-type) group,
             lengths limited to lmax (<= 12); one used symbol -> length 1; unused -> 0
  codes      canonical: symbols sorted by (length, value); first code 0;
             next = (prev + 1) << (len - prev_len); a code's first bit is its MSB
  bit order  stream bit k is bit (k & 7) of byte (k >> 3) (equivalently bit k & 31 of
             little-endian u32 word k >> 5); a code is written first bit first
  block      exactly block_bytes bytes, independently decodable:
               +0    u32  n          elements in the block, a positive multiple of 64
               +4    u32  e0         index of the block's first element in its tensor
               +8    u16  sub_bits[64]
               +136  u8   sm[n]      raw sign|mantissa bytes in element order
               +136+n     code area: 64 sub-streams back to back, then zero padding
             element m of the block (0 <= m < n) belongs to sub-stream (m >> 3) & 63;
             a sub-stream is the concatenation of its elements' codes in increasing m
  packing    greedy: n is the largest multiple of 64 (not beyond the tensor's end) with
             136 + n + 4 * ceil(code_bits(n) / 32) <= block_bytes

parity unpinned against the paper for the stream format itself (the paper prints none);
pinned by losslessness, hand-built streams, the Shannon bound and Huffman optimality
(tests/test_oracle_codec.py).
"""
from __future__ import annotations

import heapq

import numpy as np

HEADER_BYTES = 136
N_SUB = 64          # sub-streams per block
RUN = 8             # consecutive elements per sub-stream visit
GROUP = 64          # block element counts are multiples of this


# ----------------------------------------------------------------------------- split/join
def split_bf16(w: np.ndarray):
    """BF16 bit patterns -> (exponent byte, raw sign|mantissa byte).  A bit permutation:
    NaN, Inf, zeros and subnormals are not special."""
    w = np.asarray(w, dtype=np.uint16)
    e = ((w >> 7) & 0xFF).astype(np.uint8)
    sm = (((w >> 8) & 0x80) | (w & 0x7F)).astype(np.uint8)
    return e, sm


def join_bf16(e: np.ndarray, sm: np.ndarray) -> np.ndarray:
    e = np.asarray(e, dtype=np.uint16)
    sm = np.asarray(sm, dtype=np.uint16)
    return (((sm & 0x80) << 8) | (e << 7) | (sm & 0x7F)).astype(np.uint16)


def exponent_histogram(w: np.ndarray) -> np.ndarray:
    e, _ = split_bf16(np.asarray(w).reshape(-1))
    return np.bincount(e, minlength=256).astype(np.int64)


# ----------------------------------------------------------------------------- code lengths
def code_lengths(hist: np.ndarray, lmax: int = 12) -> np.ndarray:
    """Optimal length-limited prefix-code lengths (package-merge, Larmore & Hirschberg).

    Every used symbol starts as one coin per level 1..lmax (face value 2^-level, cost = its
    count).  Going from the deepest level up, the coins of a level are sorted by cost and
    paired into packages that join the next level.  The 2*(m-1) cheapest items at level 1
    are bought; a symbol's length is the number of its coins that were bought.
    """
    hist = np.asarray(hist, dtype=np.int64)
    used = [int(s) for s in np.nonzero(hist)[0]]
    lens = np.zeros(256, dtype=np.uint8)
    m = len(used)
    if m == 0:
        return lens
    if m == 1:
        lens[used[0]] = 1
        return lens
    if (1 << lmax) < m:
        raise ValueError("lmax too small for the number of used symbols")
    # an item is (cost, tie, tuple of symbols it contains)
    leaves = sorted((int(hist[s]), s, (s,)) for s in used)
    prev = []                                   # packages coming up from the level below
    for _level in range(lmax, 0, -1):
        items = sorted(leaves + prev, key=lambda t: (t[0], t[1]))
        if _level == 1:
            chosen = items[: 2 * (m - 1)]
            for _cost, _tie, syms in chosen:
                for s in syms:
                    lens[s] += 1
            break
        prev = []
        for i in range(0, len(items) - 1, 2):
            a, b = items[i], items[i + 1]
            prev.append((a[0] + b[0], min(a[1], b[1]), a[2] + b[2]))
    return lens


def huffman_cost_unlimited(hist: np.ndarray) -> int:
    """Total bits of an unrestricted optimal Huffman code = sum of all merged weights."""
    heap = [int(c) for c in hist if c > 0]
    if len(heap) == 1:
        return heap[0]
    heapq.heapify(heap)
    total = 0
    while len(heap) > 1:
        a = heapq.heappop(heap)
        b = heapq.heappop(heap)
        total += a + b
        heapq.heappush(heap, a + b)
    return total


def canonical_codes(lens: np.ndarray) -> np.ndarray:
    """codes[s] for every used symbol (value read MSB first, `lens[s]` bits wide)."""
    lens = np.asarray(lens, dtype=np.int64)
    codes = np.zeros(256, dtype=np.int64)
    order = sorted((int(lens[s]), s) for s in range(256) if lens[s] > 0)
    code = 0
    prev_len = order[0][0] if order else 0
    for i, (ln, s) in enumerate(order):
        if i > 0:
            code = (code + 1) << (ln - prev_len)
        codes[s] = code
        prev_len = ln
    return codes


def payload_bits(hist: np.ndarray, lens: np.ndarray) -> int:
    return int((np.asarray(hist, dtype=np.int64) * np.asarray(lens, dtype=np.int64)).sum())


# ----------------------------------------------------------------------------- encoder
def _fits(n: int, bits: int, block_bytes: int) -> bool:
    return HEADER_BYTES + n + 4 * ((bits + 31) // 32) <= block_bytes


def plan_blocks(elem_bits: np.ndarray, block_bytes: int) -> list:
    """Greedy packing: first-element index of every block, plus the tensor length at the end."""
    N = elem_bits.size
    assert N % GROUP == 0 and N > 0
    group_bits = elem_bits.reshape(-1, GROUP).sum(axis=1).astype(np.int64)
    cum = np.concatenate([[0], np.cumsum(group_bits)])        # bits of the first g groups
    n_groups = group_bits.size
    first = [0]
    g0 = 0
    while g0 < n_groups:
        g = g0
        # linear scan in whole groups: the condition is monotone in g
        while g < n_groups and _fits((g + 1 - g0) * GROUP, int(cum[g + 1] - cum[g0]), block_bytes):
            g += 1
        if g == g0:
            raise ValueError("block_bytes too small for one group of 64 elements")
        first.append(g * GROUP)
        g0 = g
    return first


def encode_block(w: np.ndarray, e0: int, lens: np.ndarray, codes: np.ndarray,
                 block_bytes: int) -> np.ndarray:
    """One block for elements w (n of them, starting at tensor index e0)."""
    n = w.size
    e, sm = split_bf16(w)
    ln = lens[e].astype(np.int64)
    cd = codes[e]
    assert (ln > 0).all(), "symbol without a code"
    m = np.arange(n)
    sub = (m >> 3) & (N_SUB - 1)
    sub_bits = np.bincount(sub, weights=ln, minlength=N_SUB).astype(np.int64)
    # the code area is the concatenation, over sub-streams j = 0..63, of each sub-stream's
    # codes in increasing m: sort elements by (sub-stream, m); a code's bit position is the
    # total length of everything sorted before it
    order = np.lexsort((m, sub))
    ln_sorted = ln[order]
    pos = np.empty(n, dtype=np.int64)
    pos[order] = np.cumsum(ln_sorted) - ln_sorted
    total_bits = int(sub_bits.sum())
    assert _fits(n, total_bits, block_bytes)
    area_bytes = block_bytes - HEADER_BYTES - n
    bits = np.zeros(area_bytes * 8, dtype=np.uint8)
    for l in range(int(ln.max())):
        sel = ln > l
        bits[pos[sel] + l] = (cd[sel] >> (ln[sel] - 1 - l)) & 1
    blk = np.zeros(block_bytes, dtype=np.uint8)
    blk[0:4] = np.frombuffer(np.uint32(n).tobytes(), dtype=np.uint8)
    blk[4:8] = np.frombuffer(np.uint32(e0).tobytes(), dtype=np.uint8)
    blk[8:HEADER_BYTES] = np.frombuffer(sub_bits.astype("<u2").tobytes(), dtype=np.uint8)
    blk[HEADER_BYTES:HEADER_BYTES + n] = sm
    blk[HEADER_BYTES + n:] = np.packbits(bits, bitorder="little")
    return blk


def encode_tensor(w: np.ndarray, lens: np.ndarray, block_bytes: int = 4096):
    """Flat uint16 tensor -> (blocks uint8 [nblocks][block_bytes], first_elem int64 [nblocks+1])."""
    w = np.asarray(w, dtype=np.uint16).reshape(-1)
    lens = np.asarray(lens, dtype=np.uint8)
    codes = canonical_codes(lens)
    e, _ = split_bf16(w)
    first = plan_blocks(lens[e].astype(np.int64), block_bytes)
    blocks = np.zeros((len(first) - 1, block_bytes), dtype=np.uint8)
    for k in range(len(first) - 1):
        blocks[k] = encode_block(w[first[k]:first[k + 1]], first[k], lens, codes, block_bytes)
    return blocks, np.asarray(first, dtype=np.int64)


# ----------------------------------------------------------------------------- decoders
def block_header(blk: np.ndarray):
    n = int(np.frombuffer(blk[0:4].tobytes(), dtype="<u4")[0])
    e0 = int(np.frombuffer(blk[4:8].tobytes(), dtype="<u4")[0])
    sub_bits = np.frombuffer(blk[8:HEADER_BYTES].tobytes(), dtype="<u2").astype(np.int64)
    return n, e0, sub_bits


def decode_block_bitwise(blk: np.ndarray, lens: np.ndarray):
    """Slowest, most literal decoder (pure Python): read one bit at a time and stop as soon
    as the bits read so far equal a code of that length.  No table of any kind."""
    codes = canonical_codes(lens)
    book = {(int(lens[s]), int(codes[s])): s for s in range(256) if lens[s] > 0}
    lmax = max(k[0] for k in book)
    n, e0, sub_bits = block_header(blk)
    sm = blk[HEADER_BYTES:HEADER_BYTES + n]
    area = blk[HEADER_BYTES + n:]

    def bit(k):
        return (int(area[k >> 3]) >> (k & 7)) & 1

    start = [0] * N_SUB
    for j in range(1, N_SUB):
        start[j] = start[j - 1] + int(sub_bits[j - 1])
    pos = list(start)
    out = np.zeros(n, dtype=np.uint16)
    for m in range(n):
        j = (m >> 3) & (N_SUB - 1)
        val, ln = 0, 0
        while True:
            val = (val << 1) | bit(pos[j])
            pos[j] += 1
            ln += 1
            if (ln, val) in book:
                break
            if ln >= lmax:
                raise ValueError("corrupt stream: no code matches")
        s = book[(ln, val)]
        out[m] = ((int(sm[m]) & 0x80) << 8) | (s << 7) | (int(sm[m]) & 0x7F)
    for j in range(N_SUB):
        if pos[j] - start[j] != int(sub_bits[j]):
            raise ValueError("corrupt stream: sub-stream length mismatch")
    return e0, out


def _peek_table(lens: np.ndarray, lmax: int):
    """sym/len for every lmax-bit prefix (first stream bit = most significant index bit)."""
    codes = canonical_codes(lens)
    sym = np.full(1 << lmax, -1, dtype=np.int64)
    ln = np.zeros(1 << lmax, dtype=np.int64)
    for s in range(256):
        L = int(lens[s])
        if L:
            lo = int(codes[s]) << (lmax - L)
            hi = (int(codes[s]) + 1) << (lmax - L)
            assert (sym[lo:hi] == -1).all(), "codes are not prefix free"
            sym[lo:hi] = s
            ln[lo:hi] = L
    return sym, ln


def decode_blocks(blocks: np.ndarray, lens: np.ndarray):
    """Decode many blocks at once (numpy): all sub-streams of all blocks advance one symbol
    per step.  Returns (e0 int64 [nb], n int64 [nb], list of uint16 arrays)."""
    blocks = np.asarray(blocks, dtype=np.uint8)
    if blocks.ndim == 1:
        blocks = blocks[None, :]
    nb, B = blocks.shape
    lens = np.asarray(lens, dtype=np.uint8)
    lmax = int(lens.max())
    sym_t, len_t = _peek_table(lens, lmax)
    n = blocks[:, 0:4].copy().view("<u4").reshape(nb).astype(np.int64)
    e0 = blocks[:, 4:8].copy().view("<u4").reshape(nb).astype(np.int64)
    sub_bits = blocks[:, 8:HEADER_BYTES].copy().view("<u2").reshape(nb, N_SUB).astype(np.int64)
    if ((n <= 0) | (n % GROUP != 0) | (HEADER_BYTES + n > B)).any():
        raise ValueError("corrupt block header")
    bits = np.unpackbits(blocks, axis=1, bitorder="little")
    bits = np.concatenate([bits, np.zeros((nb, lmax), dtype=np.uint8)], axis=1)
    area0 = (HEADER_BYTES + n) * 8                                     # [nb]
    start = area0[:, None] + np.cumsum(sub_bits, axis=1) - sub_bits    # [nb][64]
    pos = start.copy()
    n_max = int(n.max())
    exps = np.zeros((nb, n_max), dtype=np.uint8)
    rows = np.arange(nb)[:, None]
    lane = np.arange(N_SUB)[None, :]
    weights = (1 << np.arange(lmax - 1, -1, -1)).astype(np.int64)
    runs_max = (n_max // RUN + N_SUB - 1) // N_SUB
    for u in range(runs_max):
        for i in range(RUN):
            m = (u * N_SUB + lane) * RUN + i                            # [1][64]
            active = m < n[:, None]                                    # [nb][64]
            idx = np.zeros((nb, N_SUB), dtype=np.int64)
            for l in range(lmax):
                idx += bits[rows, pos + l].astype(np.int64) * weights[l]
            s = sym_t[idx]
            if (s[active] < 0).any():
                raise ValueError("corrupt stream: no code matches")
            r, c = np.nonzero(active)
            exps[r, m[0, c]] = s[r, c]
            pos = pos + np.where(active, len_t[idx], 0)
    if ((pos - start) != sub_bits).any():
        raise ValueError("corrupt stream: sub-stream length mismatch")
    out = []
    for b in range(nb):
        k = int(n[b])
        out.append(join_bf16(exps[b, :k], blocks[b, HEADER_BYTES:HEADER_BYTES + k]))
    return e0, n, out


def decode_tensor(blocks: np.ndarray, lens: np.ndarray, n_elems: int, chunk: int = 512):
    """All blocks of one tensor -> flat uint16 array of n_elems (placed by each block's e0)."""
    blocks = np.asarray(blocks, dtype=np.uint8)
    out = np.zeros(n_elems, dtype=np.uint16)
    covered = 0
    for b0 in range(0, blocks.shape[0], chunk):
        e0, n, parts = decode_blocks(blocks[b0:b0 + chunk], lens)
        for a, k, p in zip(e0, n, parts):
            if a + k > n_elems:
                raise ValueError("block outside its tensor")
            out[a:a + k] = p
            covered += int(k)
    if covered != n_elems:
        raise ValueError("blocks do not cover the tensor")
    return out


# ----------------------------------------------------------------------------- layer pool
def encode_layer(w13: np.ndarray, w2: np.ndarray, lmax: int = 12, block_bytes: int = 4096):
    """One layer's pool.  w13 uint16 [E][2][H][F], w2 uint16 [E][F][H].

    One code per tensor type over all routed experts of the layer.  Blob order: the down
    tensors (type 2) of experts 0..E-1, then the fused gate/up tensors (type 1): the paper
    offloads down-projection tensors first (Sec. 4.2, "down-projection tensors alone can
    approximate the target"), so a prefix of the blob is what goes to the host tier.
    Returns dict(lens13, lens2, blocks [nb][B], tensor_first_block {(d, e): (b0, b1)},
    first_elem {(d, e): array}).
    """
    E = w13.shape[0]
    lens13 = code_lengths(exponent_histogram(w13), lmax)
    lens2 = code_lengths(exponent_histogram(w2), lmax)
    chunks, index, felem = [], {}, {}
    b = 0
    for d, arr, lens in ((2, w2, lens2), (1, w13, lens13)):
        for ex in range(E):
            blk, first = encode_tensor(arr[ex].reshape(-1), lens, block_bytes)
            chunks.append(blk)
            index[(d, ex)] = (b, b + blk.shape[0])
            felem[(d, ex)] = first
            b += blk.shape[0]
    return dict(lens13=lens13, lens2=lens2, blocks=np.concatenate(chunks, axis=0),
                tensor_blocks=index, first_elem=felem)


def host_tier_blocks(n_blocks_layer: int, host_fraction: float) -> int:
    """Number of leading blocks of a layer blob kept in pinned host memory."""
    return int(np.ceil(host_fraction * n_blocks_layer - 1e-12)) if host_fraction > 0 else 0
