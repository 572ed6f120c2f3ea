"""The worker-process front end of the oracle returns exactly what direct oracle calls return."""
import numpy as np

from tests import helpers as H
from tests import oracle_pool as P
from tests import synth
from tests.test_gpu_fullsize import draft_task, one_head_per_pair, verify_task


def test_pool_results_equal_direct_oracle_calls():
    lay = synth.make_layer(1, "cpu", ctx_len=[320, 200], n_q_heads=8, n_kv_heads=2, quant_bits=(4,), keep=[40, 20],
                           keep_first=4, keep_last=8, win=[8, 4], tail_len=[3, 0])
    kw = H.draft_kwargs(lay, bits=4, use_pool=True, use_keep=True, use_tail=True)
    samples = one_head_per_pair(lay)
    assert len(samples) == 4 and len({(b, h // 4) for b, h in samples}) == 4
    try:
        refs = P.run(P.draft_task, [draft_task(lay, kw, b, h) for (b, h) in samples])
        ref, lse = H.oracle_draft(lay, kw)
        for (b, h), r in zip(samples, refs):
            assert np.array_equal(r[0][0][0], ref[b, h]) and r[0][0][1] == lse[b, h]
        rr = P.run(P.verify_task, [verify_task(lay, 1, 5, [0, 3])])
        vref, vlse = H.oracle_verify(lay)
        assert np.array_equal(rr[0][0][0], vref[8 + 0, 5]) and np.array_equal(rr[0][1][0], vref[8 + 3, 5])
        assert rr[0][1][1] == vlse[8 + 3, 5]
    finally:
        P.shutdown()
