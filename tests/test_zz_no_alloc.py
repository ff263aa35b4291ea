"""GPU check of leann_adc_noalloc (the entry point for callers that cannot allocate): its output must equal
leann_adc's bit for bit (same kernels, the lookup tables in the library's fixed array), on two calls in a row, the
second with a smaller input, and sizes beyond the fixed array must be rejected."""
import numpy as np
import pytest

import leann_inputs as li
from gpu_util import say, to_dev

pytestmark = pytest.mark.gpu


def test_noalloc_adc_equals_adc_twice_in_a_row(orc):
    import torch
    import paper_2506_08276_amd as L
    L.load_library()
    ctx = L.leann_create(li.TINY, to_dev(li.encoder_weights(li.TINY, 1)))
    try:
        rng = np.random.default_rng(12)
        d, m_sub, n = 768, 32, 6000
        x = rng.standard_normal((n, d)).astype(np.float32)
        x /= np.linalg.norm(x, axis=1, keepdims=True)
        cb, _ = orc.pq_train(x, m_sub, 2, 7)
        codes = orc.pq_encode(x, cb)
        pq = L.leann_pq_import(ctx, cb, codes)
        for nq, nc in ((128, 2500), (5, 33)):  # the second call is smaller: stale tables of the first stay behind it
            say(f"adc_noalloc nq={nq} nc={nc}")
            q = rng.standard_normal((nq, d)).astype(np.float32)
            q /= np.linalg.norm(q, axis=1, keepdims=True)
            cand = rng.integers(0, n, size=(nq, nc)).astype(np.uint32)
            qd, cd = to_dev(q), to_dev(cand)
            want = L.leann_adc(ctx, qd, pq, cd)
            got = torch.full((nq, nc), float("nan"), dtype=torch.float32, device="cuda:0")
            L.leann_adc_noalloc(ctx, qd, pq, cd, got)
            torch.cuda.synchronize()
            assert torch.equal(got, want)
            # and against the oracle, to the ADC bound
            for qi in (0, nq - 1):
                ref, l1 = orc.adc(orc.lut(q[qi], cb), codes, cand[qi])
                assert np.all(np.abs(got[qi].cpu().numpy() - ref) <= 1e-4 * np.maximum(np.abs(ref), l1))
        # an id outside the table: -inf at its position, the rest unchanged, no error status
        cand[1, 2] = n
        got2 = torch.empty((nq, nc), dtype=torch.float32, device="cuda:0")
        L.leann_adc_noalloc(ctx, qd, pq, to_dev(cand), got2)
        torch.cuda.synchronize()
        assert got2[1, 2].item() == float("-inf")
        got2[1, 2] = want[1, 2]
        assert torch.equal(got2, want)
        # beyond the fixed array: rejected, nothing written
        say("adc_noalloc nq=129 (rejected)")
        big_q = to_dev(np.zeros((129, d), np.float32))
        big_c = to_dev(np.zeros((129, 4), np.uint32))
        out = torch.full((129, 4), 7.0, dtype=torch.float32, device="cuda:0")
        with pytest.raises(L.LeannError) as ei:
            L.leann_adc_noalloc(ctx, big_q, pq, big_c, out)
        assert ei.value.status == -5
        torch.cuda.synchronize()
        assert bool((out == 7.0).all())
        L.leann_pq_free(pq)
    finally:
        L.leann_destroy(ctx)
