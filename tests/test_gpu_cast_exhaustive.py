"""The pseudo-gradient's FP32 -> binary16 and FP32 -> bfloat16 roundings on the GPU against the
oracle's integer-only casts for all 2^32 float patterns (NaNs compare by class and sign, everything else bit for bit)."""
import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.gpu


@pytest.mark.timeout(900)
@pytest.mark.parametrize("fmt", ["f16", "bf16"])
def test_all_float_patterns(fmt):
    import torch
    import paper_2407_07852_amd as D
    gpu_cast = D.diloco_cast_f32_to_f16 if fmt == "f16" else D.diloco_cast_f32_to_bf16
    cpu_cast = oracle.cast_pattern_range if fmt == "f16" else oracle.cast_pattern_range_bf16
    exp_mask, frac_mask = (0x7C00, 0x3FF) if fmt == "f16" else (0x7F80, 0x7F)
    chunk = 1 << 28
    src = torch.empty(chunk, dtype=torch.int32, device="cuda")
    dst = torch.empty(chunk, dtype=torch.int16, device="cuda")
    base = torch.arange(chunk, dtype=torch.int64, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    for c in range(16):
        first = c * chunk
        # the chunk's bit patterns, as int32 with wrap-around
        src.copy_(((base + first + (1 << 31)) % (1 << 32) - (1 << 31)).to(torch.int32))
        gpu_cast(src.data_ptr(), dst.data_ptr(), chunk, stream)
        got = dst.cpu().numpy().view(np.uint16)
        want = cpu_cast(first, chunk)
        pat_hi = (np.arange(first, first + chunk, dtype=np.uint64) & 0x7FFFFFFF)
        nan = pat_hi > 0x7F800000
        assert np.array_equal(got[~nan], want[~nan]), "chunk %d" % c
        if nan.any():
            assert ((got[nan] & exp_mask) == exp_mask).all() and ((got[nan] & frac_mask) != 0).all()
            assert np.array_equal(got[nan] >> 15, want[nan] >> 15)
        print("%s cast chunk %2d/16 ok" % (fmt, c + 1), flush=True)
