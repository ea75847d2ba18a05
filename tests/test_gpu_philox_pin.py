"""Pin of the oracle's Philox4x32-10 (and of the GPU library's) against an implementation neither side wrote:
rocRAND's host generator, driven through its C API.  rocRAND's Philox stream is the plain sequence of one engine:
output words 4i .. 4i+3 are the generator's block for counter (lo32(i), hi32(i), 0, 0) under key (lo32(seed), hi32(seed)),
and an offset of 4k words starts the stream at counter k.  A wrong multiplier, Weyl constant, round count, word
order inside a round or a swapped key half in the oracle fails this test.  Marked gpu only because rocRAND's host
generator allocates through the HIP runtime and refuses to work on a machine without a device."""
import ctypes as C

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu

ROCRAND_RNG_PSEUDO_PHILOX4_32_10 = 404      # rocrand_rng_type in rocrand/rocrand.h


def rocrand_words(seed: int, offset_words: int, n: int) -> np.ndarray:
    L = C.CDLL("/opt/rocm/lib/librocrand.so")
    gen = C.c_void_p()
    assert L.rocrand_create_generator_host(C.byref(gen), ROCRAND_RNG_PSEUDO_PHILOX4_32_10) == 0
    try:
        assert L.rocrand_set_seed(gen, C.c_ulonglong(seed)) == 0
        assert L.rocrand_set_offset(gen, C.c_ulonglong(offset_words)) == 0
        out = np.zeros(n, np.uint32)
        assert L.rocrand_generate(gen, out.ctypes.data_as(C.c_void_p), C.c_size_t(n)) == 0
    finally:
        L.rocrand_destroy_generator(gen)
    return out


@pytest.mark.parametrize("seed", [0, 1, 12345678901234567, 0xFFFFFFFF00000000, 2**64 - 1])
@pytest.mark.parametrize("first_counter", [0, 5, 2**32 - 3, 2**32 + 5, 7 * 2**32 + 123456789])
def test_oracle_philox_equals_rocrand(seed, first_counter):
    n_blocks = 512
    got = rocrand_words(seed, 4 * first_counter, 4 * n_blocks).reshape(n_blocks, 4)
    for i in range(n_blocks):
        c = first_counter + i                                   # 64-bit counter: low word c0, high word c1
        want = oracle.philox(seed, c & 0xFFFFFFFF, c >> 32, 0, 0)
        assert (got[i] == want).all(), (seed, c, [hex(x) for x in got[i]], [hex(x) for x in want])


def test_gpu_philox_equals_rocrand():
    import paper_2604_05417_amd as M
    seed, n = 0x0123456789ABCDEF, 100_000
    for c1 in (0, 9):
        got = rocrand_words(seed, 4 * (c1 << 32), 4 * n).reshape(n, 4)
        mine = M.philox_words(seed, 0, n, c1, 0, 0).cpu().numpy().view(np.uint32)
        assert np.array_equal(mine, got)
