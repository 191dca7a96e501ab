"""The entry point that allocates nothing (nt_q8_output_layer_static) against the entry point it is a variant of
(nt_debug_q8_output_layer), through the C ABI: bit-equal logits and arg-max on two calls in a row, the second on
a smaller input, so that what the first call left in the library's static scratch must not show."""
import numpy as np
import pytest

import nt_synth

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_equals_the_arena_entry_point():
    import torch
    import paper_2109_08003_amd as nt
    assert torch.cuda.is_available(), "this test needs the MI355X"
    nt.load_library()
    cfg = nt_synth.model_config("C1", q8_output=1, n_enc=1)
    blob = nt_synth.make_weights(cfg, seed=0, random_affine=True)
    gm = nt.Model(cfg, blob, max_batch_tokens=4096, pipeline_lanes=1)
    d, V = cfg["d_model"], cfg["vocab"]
    rng = np.random.default_rng(17)
    for R in (1024, 137):                                   # the largest supported input first, then a smaller one
        h = torch.from_numpy(rng.normal(0, 1, (R, d)).astype(np.float32)).cuda()
        want_am = torch.full((R,), -1, dtype=torch.int32, device="cuda")
        want_lg = torch.empty((R, V), dtype=torch.float32, device="cuda")
        gm.debug_q8_output_layer(h, want_am, want_lg)
        got_am = torch.full((R,), -2, dtype=torch.int32, device="cuda")
        got_lg = torch.full((R, V), float("nan"), dtype=torch.float32, device="cuda")
        gm.q8_output_layer_static(h, got_am, got_lg)
        torch.cuda.synchronize()
        assert torch.equal(got_am, want_am), R
        assert torch.equal(got_lg.view(torch.int32), want_lg.view(torch.int32)), R
        assert int(want_am.min()) >= 0 and int(want_am.max()) < V
    # beyond the stated maximum: a clear error, nothing launched
    h = torch.zeros((1025, d), dtype=torch.float32, device="cuda")
    with pytest.raises(nt.NtError) as e:
        gm.q8_output_layer_static(h, torch.empty(1025, dtype=torch.int32, device="cuda"))
    assert e.value.code == -6
    gm.close()
