"""The allocation-free row quantiser (pahq_quantize_rows_noalloc, through the C ABI on device tensors the
test owns) against pahq_quantize_rows: codes and scales bit for bit, two calls in a row, the second
smaller (the static per-row maxima of the first call must not leak into it)."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


def _rows(rng, rows, cols):
    x = (rng.standard_normal((rows, cols)) * rng.uniform(1e-4, 300, (rows, 1))).astype(np.float32)
    x[min(3, rows - 1)] = 0.0                           # a zero row: scale 1, codes 0
    x[0, :] = np.float32(1e-30)
    return x


def test_noalloc_row_quantiser_matches_the_model_bound_one():
    import torch
    import paper_2510_23264_amd as P
    shape, w, clean, corrupt, spec = synth.make_workload("cfg1")
    gm = P.Model(shape, w, spec["B"], spec["S"], max_batch_edges=8)
    try:
        rng = np.random.default_rng(17)
        # first call large (maxima up to 300 * 5 sigma in every slot it uses), then smaller ones whose
        # rows have much smaller maxima: a slot that was not cleared would change their scales
        for rows, cols, amp in ((700, 5000, 1.0), (37, 100, 1e-3), (5, 12290, 1e-2), (1, 1, 1.0), (64, 4096, 1e-4)):
            x = _rows(rng, rows, cols) * np.float32(amp)
            xd = torch.from_numpy(x).cuda()
            codes = torch.full((rows, cols), 0xAA, dtype=torch.uint8, device="cuda")
            scales = torch.full((rows,), -1.0, dtype=torch.float32, device="cuda")
            P.quantize_rows_noalloc(xd, codes, scales)
            torch.cuda.synchronize()
            want_c, want_s = gm.quantize_rows(x)
            assert (scales.cpu().numpy().view(np.uint32) == want_s.view(np.uint32)).all(), (rows, cols)
            assert (codes.cpu().numpy() == want_c).all(), (rows, cols)
        # limits: more rows than the static array holds is an error, not a truncation; nothing to do is fine
        lib = P.lib()
        assert lib.pahq_quantize_rows_noalloc(None, None, 32769, 8, None, None) == -7
        assert lib.pahq_quantize_rows_noalloc(None, None, 0, 8, None, None) == 0
        assert lib.pahq_quantize_rows_noalloc(None, None, 4, 0, None, None) == -1
        assert lib.pahq_quantize_rows_noalloc(None, None, 4, 8, None, None) == -1
    finally:
        gm.close()
