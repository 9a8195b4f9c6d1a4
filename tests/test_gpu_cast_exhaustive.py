"""The pseudo-gradient's FP32 -> binary16 rounding on the GPU against the oracle's integer-only
cast for all 2^32 float patterns (NaNs compare by class and sign, everything else bit for bit)."""
import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(900)
def test_all_float_patterns():
    import torch
    import paper_2407_07852_amd as D
    chunk = 1 << 28
    src = torch.empty(chunk, dtype=torch.int32, device="cuda")
    dst = torch.empty(chunk, dtype=torch.int16, device="cuda")
    base = torch.arange(chunk, dtype=torch.int64, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    for c in range(16):
        first = c * chunk
        # the chunk's bit patterns, as int32 with wrap-around
        src.copy_(((base + first + (1 << 31)) % (1 << 32) - (1 << 31)).to(torch.int32))
        D.diloco_cast_f32_to_f16(src.data_ptr(), dst.data_ptr(), chunk, stream)
        got = dst.cpu().numpy().view(np.uint16)
        want = oracle.cast_pattern_range(first, chunk)
        pat_hi = (np.arange(first, first + chunk, dtype=np.uint64) & 0x7FFFFFFF)
        nan = pat_hi > 0x7F800000
        assert np.array_equal(got[~nan], want[~nan]), "chunk %d" % c
        if nan.any():
            assert ((got[nan] & 0x7C00) == 0x7C00).all() and ((got[nan] & 0x3FF) != 0).all()
            assert np.array_equal(got[nan] >> 15, want[nan] >> 15)
        print("cast chunk %2d/16 ok" % (c + 1), flush=True)
