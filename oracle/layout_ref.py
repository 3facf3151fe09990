"""Reference statement of the packed-weight layout and of the lookup-table buffer layout.
TEST INFRASTRUCTURE ONLY -- shares no code with the HIP library.

The paper asks for one pre-permuted, bit-serial weight copy that both the decoding and the prefill
kernel read in contiguous blocks (Sec. 4.1 "Unified Layout", "Unified tiling strategy"); its own
tile picture is hardware specific.  The layout used here is documented as a pure function
``(m, k, i) -> (byte, bit)`` and this file is that function written one bit at a time:

* rows are cut into row blocks of 64, columns into K tiles of 128 weights; tile block ``(rb, kt)``
  starts at ``128 + (rb * n_ktiles + kt) * tile_bytes``;
* inside a tile block, "lane" ``l = m % 64`` owns the 128 weights ``k = 128 kt + [0,128)`` of row ``m``;
  they are cut into ``bits`` chunks of ``128 / bits`` weights; chunk ``v`` of all 64 lanes forms one
  1024-byte sub-block (16 bytes per lane), so a 64-lane wave reads it with one coalesced 16-byte
  load per lane;
* the 16 bytes of a chunk are little-endian 32-bit words; word ``ksub * bits + i`` holds bit-plane ``i``
  (bit ``i`` of the codes, Sec. 2.2 one-bit decomposition) of the 32 weights ``ksub * 32 + [0,32)`` of
  the chunk, weight ``beta`` in bit ``beta``.  Four consecutive bits are therefore one 4-bit table
  index with weight ``t`` in bit ``t`` (Sec. 4.1 "Bit repacking" example);
* after the ``bits`` sub-blocks come the lane's quantization-group parameters: for each of its
  ``128 / group`` groups the fp16 scale followed (when the format has zeros) by the fp16 zero.
* rows >= M and columns >= K are padding: zero bits, zero scale, zero zero-point.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

HEADER_BYTES = 128
ROWS = 64
KTILE = 128
MAGIC = b"TMANPK1\x00"


@dataclass(frozen=True)
class PackedLayout:
    M: int
    K: int
    bits: int
    group: int
    has_zero: bool

    @property
    def n_row_blocks(self) -> int:
        return -(-self.M // ROWS)

    @property
    def n_ktiles(self) -> int:
        return -(-self.K // KTILE)

    @property
    def meta_entry(self) -> int:
        return 4 if self.has_zero else 2

    @property
    def meta_per_lane(self) -> int:
        return (KTILE // self.group) * self.meta_entry

    @property
    def tile_bytes(self) -> int:
        return self.bits * 1024 + 64 * self.meta_per_lane

    @property
    def total_bytes(self) -> int:
        return HEADER_BYTES + self.n_row_blocks * self.n_ktiles * self.tile_bytes

    def header(self) -> np.ndarray:
        h = np.zeros(HEADER_BYTES // 4, dtype="<i4")
        h[0:2] = np.frombuffer(MAGIC, dtype="<i4")
        h[2:14] = [self.M, self.K, self.bits, self.group, int(self.has_zero), ROWS, KTILE, self.n_row_blocks,
                   self.n_ktiles, self.tile_bytes, HEADER_BYTES, 1]
        return h.view(np.uint8)

    def code_bit_position(self, m, k, i):
        """(byte offset, bit in byte) of plane ``i`` of weight (m, k); arrays broadcast."""
        chunk = KTILE // self.bits
        rb, r = m // ROWS, m % ROWS
        kt, kk = k // KTILE, k % KTILE
        v, kc = kk // chunk, kk % chunk
        ksub, beta = kc // 32, kc % 32
        lane = r
        off = (HEADER_BYTES + (rb * self.n_ktiles + kt) * self.tile_bytes + v * 1024 + lane * 16
               + (ksub * self.bits + i) * 4 + beta // 8)
        return off, beta % 8

    def meta_position(self, m, G):
        """byte offset of the fp16 scale of (row m, quantization group G); the zero follows at +2."""
        k0 = G * self.group
        rb, r = m // ROWS, m % ROWS
        kt, kk = k0 // KTILE, k0 % KTILE
        gi = kk // self.group
        lane = r
        return (HEADER_BYTES + (rb * self.n_ktiles + kt) * self.tile_bytes + self.bits * 1024
                + lane * self.meta_per_lane + gi * self.meta_entry)


def pack_reference(q: np.ndarray, scale: np.ndarray, zero, bits: int, group: int) -> np.ndarray:
    """Naive packer: places every code bit and every scale/zero one by one at its documented position."""
    q = np.asarray(q, dtype=np.uint8)
    M, K = q.shape
    L = PackedLayout(M, K, bits, group, zero is not None)
    blob = np.zeros(L.total_bytes, dtype=np.uint8)
    blob[:HEADER_BYTES] = L.header()
    m, k = np.meshgrid(np.arange(M, dtype=np.int64), np.arange(K, dtype=np.int64), indexing="ij")
    for i in range(bits):
        off, bit = L.code_bit_position(m, k, i)
        val = (((q >> i) & 1).astype(np.uint8) << bit.astype(np.uint8)).astype(np.uint8)
        np.bitwise_or.at(blob, off.ravel(), val.ravel())
    G = K // group
    mm, gg = np.meshgrid(np.arange(M, dtype=np.int64), np.arange(G, dtype=np.int64), indexing="ij")
    pos = L.meta_position(mm, gg).ravel()
    s = np.asarray(scale, dtype=np.float16).reshape(M, G).view(np.uint16).ravel()
    blob[pos] = (s & 0xFF).astype(np.uint8)
    blob[pos + 1] = (s >> 8).astype(np.uint8)
    if zero is not None:
        z = np.asarray(zero, dtype=np.float16).reshape(M, G).view(np.uint16).ravel()
        blob[pos + 2] = (z & 0xFF).astype(np.uint8)
        blob[pos + 3] = (z >> 8).astype(np.uint8)
    return blob


def unpack_reference(blob: np.ndarray, M: int, K: int, bits: int, group: int, has_zero: bool):
    """Inverse of :func:`pack_reference`, again one bit at a time."""
    L = PackedLayout(M, K, bits, group, has_zero)
    blob = np.asarray(blob, dtype=np.uint8)
    m, k = np.meshgrid(np.arange(M, dtype=np.int64), np.arange(K, dtype=np.int64), indexing="ij")
    q = np.zeros((M, K), dtype=np.uint8)
    for i in range(bits):
        off, bit = L.code_bit_position(m, k, i)
        q |= (((blob[off] >> bit.astype(np.uint8)) & 1) << i).astype(np.uint8)
    G = K // group
    mm, gg = np.meshgrid(np.arange(M, dtype=np.int64), np.arange(G, dtype=np.int64), indexing="ij")
    pos = L.meta_position(mm, gg)
    s = (blob[pos].astype(np.uint16) | (blob[pos + 1].astype(np.uint16) << 8)).view(np.float16)
    z = None
    if has_zero:
        z = (blob[pos + 2].astype(np.uint16) | (blob[pos + 3].astype(np.uint16) << 8)).view(np.float16)
    return q, s, z


def lut_layout_decode(buf: np.ndarray, N: int, K: int, group: int):
    """Read the lookup-table buffer written for ``N`` tokens back into T[n][j][p] (fp16) and
    S[n][G] (fp32).

    Documented layout: tokens are padded to NP = 1, 2, 4 or 8 and K to a multiple of 128 (n_ktiles
    tiles); fp16 entry (n, j, p) sits at element ``(j * 16 + p) * NP + n`` (table j covers
    activations 4j..4j+3, pattern bit t selects activation 4j+t); the fp32 group sums follow at
    byte ``n_ktiles * 1024 * NP``, element ``G * NP + n``."""
    NP = 1 if N == 1 else 2 if N == 2 else 4 if N <= 4 else 8
    nkt = -(-K // KTILE)
    buf = np.asarray(buf, dtype=np.uint8)
    t_bytes = nkt * 1024 * NP
    T = buf[:t_bytes].view(np.float16).reshape(nkt * 32, 16, NP)
    T = np.transpose(T, (2, 0, 1))[:N, : K // 4, :]
    n_groups_padded = nkt * (KTILE // group)
    S = buf[t_bytes:t_bytes + n_groups_padded * NP * 4].view(np.float32).reshape(n_groups_padded, NP)
    S = S.T[:N, : K // group]
    return np.ascontiguousarray(T), np.ascontiguousarray(S)
