"""The library's position-id helpers (host-only C ABI calls) against the oracle, element by element."""
import os

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2401_09486_amd", "libloma.so")
pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libloma.so not built")


@pytest.mark.parametrize("t,c,n", [(2, 3, 2), (4, 4, 4), (16, 4, 28), (32, 8, 60), (1, 1, 5), (5, 7, 3), (16, 16, 9)])
def test_position_ids_match_the_oracle(t, c, n):
    from oracle import loma_positions as lp
    from paper_2401_09486_amd import loma
    for code, name in ((loma.POS_INTERMITTENT, lp.INTERMITTENT), (loma.POS_CONTIGUOUS, lp.CONTIGUOUS)):
        assert loma.sample_position_ids(t, c, n, code) == lp.sample_position_ids(t, c, n, name).tolist()
        for chunk in (0, 1, n - 1, 511):
            ids = loma.memory_position_ids(t, c, chunk, code)
            assert ids == lp.memory_position_ids(chunk, t, c, name).tolist()
            # the generation loop's ids at the compression that creates this chunk's memory
            assert ids == lp.compress_position_ids((chunk + 1) * t * c, t, c, chunk, name).tolist()
            # an arithmetic progression, as the *_rope entry points take it
            step = c if code == loma.POS_INTERMITTENT else 1
            assert all(b - a == step for a, b in zip(ids, ids[1:]))


def test_position_id_helpers_reject_bad_arguments():
    import ctypes
    from paper_2401_09486_amd import loma
    buf = (ctypes.c_int * 64)()
    lib = loma.lib
    assert lib.loma_memory_position_ids(0, 4, 0, 0, buf) == loma.ERR_INVALID_ARG
    assert lib.loma_memory_position_ids(4, 4, -1, 0, buf) == loma.ERR_INVALID_ARG
    assert lib.loma_memory_position_ids(4, 4, 0, 2, buf) == loma.ERR_INVALID_ARG
    assert lib.loma_memory_position_ids(4, 4, 0, 0, None) == loma.ERR_INVALID_ARG
    assert lib.loma_memory_position_ids(16, 16, 1 << 24, 0, buf) == loma.ERR_UNSUPPORTED      # ids beyond int
    assert lib.loma_sample_position_ids(4, 4, 0, 0, buf) == loma.ERR_INVALID_ARG
    assert lib.loma_sample_position_ids(4, 4, 1, 7, buf) == loma.ERR_INVALID_ARG
    # rope entry points: bad positions / theta are caught before anything else
    P = 0x10000
    a = [P] * 7 + [P + 0x100, 1, 8, 128, 16, 4, 4, 80]
    assert lib.loma_compress_step_rope(*a, 0.1, 1, -1, 4, 10000.0, None) == loma.ERR_INVALID_ARG
    assert lib.loma_compress_step_rope(*a, 0.1, 1, 3, 4, 0.0, None) == loma.ERR_INVALID_ARG
    assert lib.loma_compress_step_rope(*a, 0.1, 0, 3, 4, 10000.0, None) == loma.ERR_UNSUPPORTED        # f32 data
    assert lib.loma_compress_step_rope(P, P, P, P, P, P, P, P, 1, 8, 128, 16, 4, 4, 80, 0.1, 1, 3, 4, 10000.0, None) == loma.ERR_INVALID_ARG   # out aliases q_mem
    d = [P] * 8 + [1, 8, 128, 16, 4, 4, 64, 3]
    assert lib.loma_decode_attn_rope(*d, 0.1, 1, -5, 10000.0, P, 1 << 30, None) == loma.ERR_INVALID_ARG
    assert lib.loma_decode_attn_rope(*d, 0.1, 1, 5, float("nan"), P, 1 << 30, None) == loma.ERR_INVALID_ARG
    assert lib.loma_decode_attn_rope(*d, 0.1, 0, 5, 10000.0, P, 1 << 30, None) == loma.ERR_UNSUPPORTED
