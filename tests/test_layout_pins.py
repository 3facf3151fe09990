"""CPU pins of ``oracle/layout_ref.py`` (the reference statement of the packed-weight layout and of the
lookup-table buffer layout), against things other than itself: bytes written out by hand from the documented
layout, counting arguments (every payload bit owned by exactly one weight bit), the index definition of the
bit-serial form (Sec. 2.2) computed by the C oracle from the unpacked codes, and the paper's printed
repacking example (Sec. 4.1 "Bit repacking")."""
import os

import numpy as np
import pytest

import oracle
import synth
from oracle.layout_ref import HEADER_BYTES, KTILE, ROWS, PackedLayout, lut_layout_decode, pack_reference, unpack_reference

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

CASES = [
    # M, K, bits, group, has_zero   (the ragged cases of the GPU packing test)
    (256, 512, 4, 64, True),
    (70, 96, 4, 32, True),
    (33, 384, 2, 64, True),
    (64, 256, 2, 32, True),
    (96, 1024, 4, 128, True),
    (40, 768, 1, 64, False),
    (32, 256, 1, 128, True),
    (1, 32, 2, 32, True),
    (130, 2816, 2, 64, True),
]


def _case(seed, M, K, bits, group, hz):
    q = synth.uniform_codes(seed, M * K, bits).reshape(M, K)
    s = synth.uniform_fp16(seed + 1, M * (K // group), 0.005, 0.02).reshape(M, -1)
    z = synth.uniform_fp16(seed + 2, M * (K // group), 0.5, 9.0).reshape(M, -1) if hz else None
    return q, s, z


@pytest.mark.parametrize("M,K,bits,group,hz", CASES)
def test_round_trip(M, K, bits, group, hz):
    q, s, z = _case(500 + M + K, M, K, bits, group, hz)
    blob = pack_reference(q, s, z, bits, group)
    assert blob.dtype == np.uint8 and blob.size == PackedLayout(M, K, bits, group, hz).total_bytes
    q2, s2, z2 = unpack_reference(blob, M, K, bits, group, hz)
    assert np.array_equal(q2, q)
    assert np.array_equal(s2.view(np.uint16), s.view(np.uint16))
    if hz:
        assert np.array_equal(z2.view(np.uint16), z.view(np.uint16))
    else:
        assert z2 is None


@pytest.mark.parametrize("M,K,bits,group,hz", CASES)
def test_every_payload_bit_has_one_owner_and_padding_is_zero(M, K, bits, group, hz):
    """The position function is injective, stays inside its tile block's sub-block, never lands on a
    parameter byte, and whatever it does not reach is zero in a blob packed from all-ones input."""
    L = PackedLayout(M, K, bits, group, hz)
    m, k = np.meshgrid(np.arange(M, dtype=np.int64), np.arange(K, dtype=np.int64), indexing="ij")
    owner = np.zeros(L.total_bytes * 8, dtype=np.uint8)
    for i in range(bits):
        off, bit = L.code_bit_position(m, k, i)
        assert off.min() >= HEADER_BYTES and off.max() < L.total_bytes
        # inside a tile block, code bits live in the first bits * 1024 bytes
        assert ((off - HEADER_BYTES) % L.tile_bytes).max() < bits * 1024
        np.add.at(owner, (off * 8 + bit).ravel(), 1)
    assert owner.max() == 1 and int(owner.sum()) == M * K * bits
    G = K // group
    mm, gg = np.meshgrid(np.arange(M, dtype=np.int64), np.arange(G, dtype=np.int64), indexing="ij")
    pos = L.meta_position(mm, gg).ravel()
    assert ((pos - HEADER_BYTES) % L.tile_bytes).min() >= bits * 1024  # parameters follow the code sub-blocks
    mbytes = np.zeros(L.total_bytes, dtype=np.uint8)
    for d in range(L.meta_entry):
        np.add.at(mbytes, pos + d, 1)
    assert mbytes.max() == 1 and int(mbytes.sum()) == M * G * L.meta_entry
    # all-ones input: every owned bit is set, everything else (padding rows / columns) stays zero
    ones_q = np.full((M, K), (1 << bits) - 1, dtype=np.uint8)
    ff = np.full((M, G), 0xFFFF, dtype=np.uint16).view(np.float16)
    blob = pack_reference(ones_q, ff, ff if hz else None, bits, group)
    body_bits = np.unpackbits(blob, bitorder="little")
    expect = owner.copy()
    expect[np.repeat(mbytes, 8) == 1] = 1
    expect[: HEADER_BYTES * 8] = body_bits[: HEADER_BYTES * 8]
    assert np.array_equal(body_bits, expect)
    if M % ROWS == 0 and K % KTILE == 0:  # no padding: the payload is exactly the algorithmic bytes
        assert int(expect[HEADER_BYTES * 8:].sum()) == (L.total_bytes - HEADER_BYTES) * 8


def test_hand_written_blob_of_the_smallest_case():
    """M = 1, K = 32, 2 bits, group 32, written out from the documented layout: one tile block of
    2 * 1024 + 64 * 16 bytes (four groups of 32 per 128-column tile, 4 bytes each, per lane) after the header; the row is lane 0; its first chunk starts the
    first sub-block and holds plane 0 of weights 0..31 in word 0 and plane 1 in word 1 (weight t in bit t);
    its scale and zero open the parameter area."""
    q = np.zeros((1, 32), dtype=np.uint8)
    q[0, [0, 5, 9, 31]] = [1, 2, 3, 1]  # plane 0: bits 0, 9, 31; plane 1: bits 5, 9
    s = np.array([[1.5]], dtype=np.float16)   # 0x3E00
    z = np.array([[-2.0]], dtype=np.float16)  # 0xC000
    blob = pack_reference(q, s, z, 2, 32)
    assert blob.size == 128 + 2 * 1024 + 64 * 16
    body = blob[128:]
    expect = np.zeros_like(body)
    expect[0:4] = np.frombuffer(np.uint32((1 << 0) | (1 << 9) | (1 << 31)).tobytes(), dtype=np.uint8)
    expect[4:8] = np.frombuffer(np.uint32((1 << 5) | (1 << 9)).tobytes(), dtype=np.uint8)
    expect[2048:2052] = [0x00, 0x3E, 0x00, 0xC0]
    assert np.array_equal(body, expect)
    # header: magic, then M, K, bits, group, has_zero, rows per block, columns per tile, row blocks, K tiles,
    # tile block bytes, header bytes, layout version; the rest zero
    words = blob[:128].view("<i4")
    assert blob[:8].tobytes() == b"TMANPK1\x00"
    assert words[2:14].tolist() == [1, 32, 2, 32, 1, 64, 128, 1, 1, 3072, 128, 1]
    assert not words[14:].any()


def test_hand_written_positions_in_a_larger_blob():
    """Weight (m, k) = (70, 300), 4 bits, group 64, K = 512 (4 tiles of 4 * 1024 + 64 * 8 = 4608 bytes):
    row block 1, lane 6, tile 2, column 44 of the tile -> chunk 1 (32 weights per chunk), 32-weight block 0
    of the chunk, bit 12.  Plane i is word i of the lane's 16 bytes in sub-block 1."""
    L = PackedLayout(128, 512, 4, 64, True)
    tile0 = 128 + (1 * 4 + 2) * 4608
    for i in range(4):
        off, bit = L.code_bit_position(np.int64(70), np.int64(300), i)
        assert (int(off), int(bit)) == (tile0 + 1 * 1024 + 6 * 16 + i * 4 + 12 // 8, 12 % 8)
    # its quantization group is 300 // 64 = 4, the second half (group 0 of tile 2 is group 4): entry 0 of lane 6
    assert int(L.meta_position(np.int64(70), np.int64(4))) == tile0 + 4096 + 6 * 8
    assert int(L.meta_position(np.int64(70), np.int64(5))) == tile0 + 4096 + 6 * 8 + 4
    # 2 bits: 64 weights per chunk, two 32-weight blocks per chunk: column 44 is block 1 of chunk 0, bit 12
    L2 = PackedLayout(128, 512, 2, 64, True)
    t2 = 128 + (1 * 4 + 2) * (2048 + 512)
    off, bit = L2.code_bit_position(np.int64(70), np.int64(256 + 44), 1)
    assert (int(off), int(bit)) == (t2 + 0 * 1024 + 6 * 16 + (1 * 2 + 1) * 4 + 1, 4)


@pytest.mark.parametrize("M,K,bits,group,hz", CASES[:6])
def test_blob_nibbles_are_the_lookup_indices(oracle_lib, M, K, bits, group, hz):
    """Sec. 2.2 / Sec. 4.1: four consecutive bits of a plane word are the 4-bit pattern that plane i of the
    weights 4j .. 4j+3 presents to table j.  The C oracle computes that pattern from the unpacked codes."""
    q, s, z = _case(900 + M, M, K, bits, group, hz)
    blob = pack_reference(q, s, z, bits, group)
    idx = oracle.lut_indices(q, bits, 4)  # [i][m][j]
    L = PackedLayout(M, K, bits, group, hz)
    m, j = np.meshgrid(np.arange(M, dtype=np.int64), np.arange(K // 4, dtype=np.int64), indexing="ij")
    for i in range(bits):
        off, bit = L.code_bit_position(m, 4 * j, i)
        assert np.all(bit % 4 == 0)
        nib = (blob[off] >> bit.astype(np.uint8)) & 15
        assert np.array_equal(nib, idx[i])


def test_paper_repack_example_through_the_blob(oracle_lib):
    """Sec. 4.1 "Bit repacking": four INT4 weights whose most significant bits read 0b0011 (weights 0 and 1
    set) repack to 0b0000_0000_1000_1000.  Here: pack such weights, read the index nibble of plane 3 from the
    blob, push it through the repack table; the result must be the four codes side by side."""
    with open(os.path.join(GOLDEN, "repack_example.txt")) as f:
        plane, index, expect = [l.split() for l in f if l.strip() and not l.startswith("#")][0]
    plane, index, expect = int(plane), int(index, 2), int(expect, 2)
    assert (plane, index, expect) == (3, 0b0011, 0x0088)
    q = np.zeros((1, 32), dtype=np.uint8)
    q[0, :4] = [8, 8, 0, 0]
    blob = pack_reference(q, np.ones((1, 1), np.float16), np.zeros((1, 1), np.float16), 4, 32)
    L = PackedLayout(1, 32, 4, 32, True)
    off, bit = L.code_bit_position(np.int64(0), np.int64(0), plane)
    nib = (int(blob[off]) >> int(bit)) & 15
    assert nib == index
    codes = sum(int(q[0, t]) << (4 * t) for t in range(4))
    assert oracle.repack_entry(plane, nib) == expect == codes
    # all planes of a random quadruple rebuild its bit-parallel codes
    q[0, :4] = [13, 2, 7, 10]
    blob = pack_reference(q, np.ones((1, 1), np.float16), np.zeros((1, 1), np.float16), 4, 32)
    word = 0
    for i in range(4):
        off, bit = L.code_bit_position(np.int64(0), np.int64(0), i)
        word |= oracle.repack_entry(i, (int(blob[off]) >> int(bit)) & 15)
    assert word == 13 | (2 << 4) | (7 << 8) | (10 << 12)


def _tag(n, j, p):
    """A distinct finite fp16 value for every (token, table, pattern), given by its bit pattern."""
    return np.uint16(0x0400 + (n * 64 + j) * 16 + p).view(np.float16)


@pytest.mark.parametrize("N,NP", [(1, 1), (2, 2), (3, 4), (4, 4), (5, 8), (8, 8)])
def test_table_buffer_layout_decodes_a_hand_built_buffer(N, NP):
    """Documented table buffer: fp16 entry (n, j, p) at element (j * 16 + p) * NP + n with the tokens padded
    to NP and K to a multiple of 128; fp32 sums of quantization group G at element G * NP + n after the
    tables.  Build such a buffer element by element with recognisable values and read it back."""
    K, group = 160, 32  # 2 tiles (the second partly padding): 64 tables, 8 groups in the buffer
    nkt, tables, groups = 2, 64, 8
    t = np.zeros(tables * 16 * NP, dtype=np.float16)
    sgs = np.zeros(groups * NP, dtype=np.float32)
    for n in range(NP):
        for j in range(tables):
            for p in range(16):
                t[(j * 16 + p) * NP + n] = _tag(n, j, p) if (n < N and j < K // 4) else np.float16(-7)
        for G in range(groups):
            sgs[G * NP + n] = n * 100.0 + G if (n < N and G < K // group) else -9.0
    buf = np.concatenate([t.view(np.uint8), sgs.view(np.uint8)])
    assert buf.size == nkt * 1024 * NP + groups * NP * 4
    T, S = lut_layout_decode(buf, N, K, group)
    assert T.shape == (N, K // 4, 16) and S.shape == (N, K // group)
    for n in range(N):
        for j in range(K // 4):
            for p in range(16):
                assert T[n, j, p].view(np.uint16) == _tag(n, j, p).view(np.uint16)
        for G in range(K // group):
            assert float(S[n, G]) == n * 100.0 + G
