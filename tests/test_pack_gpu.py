"""tman_pack_weights / tman_unpack_weights against the reference layout function: bit-exact."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_11248_amd as tman
import synth
from gpu_helpers import dev, pack, rand_case, to_dev

pytestmark = pytest.mark.gpu

CASES = [
    # M, K, bits, group, has_zero
    (256, 512, 4, 64, True),     # BASELINE config 0
    (70, 96, 4, 32, True),       # ragged rows, K below one tile
    (33, 384, 2, 64, True),      # K = 1.5 tiles
    (64, 256, 2, 32, True),
    (96, 1024, 4, 128, True),
    (40, 768, 1, 64, False),     # sign plane, scale only
    (32, 256, 1, 128, True),     # 1-bit affine
    (1, 32, 2, 32, True),        # smallest legal shape
    (130, 2816, 2, 64, True),    # 11 tiles: odd tile count
]


@pytest.mark.parametrize("M,K,bits,group,hz", CASES)
def test_pack_matches_reference_and_round_trips(oracle_lib, M, K, bits, group, hz):
    q, s, z, _ = rand_case(100 + M + K + bits, M, K, 1, bits, group, hz)
    shape = tman.Shape(M, K, bits, group, hz)
    blob = pack(shape, q, s, z)
    torch.cuda.synchronize()
    ref = oracle.pack_reference(q, s, z, bits, group)
    got = blob.cpu().numpy()
    assert got.shape == ref.shape
    assert np.array_equal(got[:128], ref[:128]), "header differs"
    assert np.array_equal(got, ref)
    # inverse on the GPU
    q2 = torch.full((M, K), 0xEE, dtype=torch.uint8, device=dev())
    s2 = torch.zeros((M, K // group), dtype=torch.float16, device=dev())
    z2 = torch.zeros((M, K // group), dtype=torch.float16, device=dev()) if hz else None
    tman.tman_unpack_weights(shape, blob, q2, s2, z2)
    torch.cuda.synchronize()
    assert np.array_equal(q2.cpu().numpy(), q)
    assert np.array_equal(s2.cpu().numpy().view(np.uint16), s.view(np.uint16))
    if hz:
        assert np.array_equal(z2.cpu().numpy().view(np.uint16), z.view(np.uint16))


def test_pack_ignores_bits_above_the_code_width(oracle_lib):
    M, K, bits, group = 64, 256, 2, 64
    q, s, z, _ = rand_case(7, M, K, 1, bits, group)
    shape = tman.Shape(M, K, bits, group)
    dirty = q | np.uint8(0xF0)
    assert np.array_equal(pack(shape, dirty, s, z).cpu().numpy(), pack(shape, q, s, z).cpu().numpy())


def test_lookup_indices_read_from_the_blob(oracle_lib):
    """Index generation: nibble u of a plane word is the 4-bit table index of the oracle's definition."""
    M, K, bits, group = 64, 512, 4, 64
    q, s, z, _ = rand_case(8, M, K, 1, bits, group)
    blob = pack(tman.Shape(M, K, bits, group), q, s, z).cpu().numpy()
    idx = oracle.lut_indices(q, bits, 4)  # [i][m][j]
    L = oracle.PackedLayout(M, K, bits, group, True)
    rng = np.random.default_rng(0)
    for _ in range(500):
        i, m, j = int(rng.integers(bits)), int(rng.integers(M)), int(rng.integers(K // 4))
        off, bit = L.code_bit_position(m, 4 * j, i)
        assert bit % 4 == 0
        assert (int(blob[off]) >> bit) & 15 == idx[i, m, j]


def test_device_code_generator_matches_host():
    for bits in (1, 2, 4):
        a = synth.uniform_codes(0xABCDEF + bits, 100003, bits, start=17)
        b = synth.uniform_codes_torch(0xABCDEF + bits, 100003, bits, dev(), start=17).cpu().numpy()
        assert np.array_equal(a, b)
