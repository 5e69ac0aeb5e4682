"""The entry point that allocates nothing (smha_forward_static) against smha_forward, through the C ABI."""
import numpy as np
import pytest

import oracle
import workloads as W

pytestmark = pytest.mark.gpu


def test_static_workspace_entry_point_matches_forward_on_two_calls_in_a_row():
    """Two calls in a row through the library's own workspace array, the second with a smaller input (a quarter of the
    heads, half the head size): each output equals smha_forward's bit for bit (the merge of
    split 128-row groups runs in a fixed order) and matches the oracle; an unprepared shape is refused."""
    import torch
    import paper_2506_06095_amd as smha
    assert torch.cuda.is_available(), "this test needs the GPU"
    gen = torch.Generator(device="cuda").manual_seed(21)
    cases = [
        (W.MaskSpec(flags=W.BIGBIRD, block=64, n_window_blocks=3, n_global_blocks=2, n_random_blocks=2, seed=4), 1, 8, 4096, 128),
        (W.MaskSpec(flags=W.WINDOW | W.GLOBAL, window_left=32, window_right=32, n_global=70), 1, 2, 4096, 64),
    ]
    for spec, B, H, S, d in cases:
        with smha.Plan.from_desc(spec, B, H, S, head_dim=d, force=smha.SMHA_KERNEL_BLOCK) as plan:
            assert plan.info()["n_split_rows"] > 0              # the call really uses the workspace and its counters
            q, k, v = (torch.randn(B, H, S, d, device="cuda", generator=gen).half() for _ in range(3))
            out = torch.full_like(q, float("nan"))
            with pytest.raises(smha.SmhaError):                 # nothing prepared yet: the entry point may not allocate
                plan.forward_static(q, k, v, out)
            plan.prepare(B, H, d)
            for rep in range(2):                                # (the second call finds the counters as the first left them)
                out.fill_(float("nan"))
                plan.forward_static(q, k, v, out)
                torch.cuda.synchronize()
                want = plan.forward(q, k, v)
                torch.cuda.synchronize()
                assert torch.equal(out, want), (S, rep)
            masks = W.dense_mask(spec, B, H, S)
            Qb, Kb, Vb = (x.cpu().numpy().view(np.uint16) for x in (q, k, v))
            h = H - 1
            ref = oracle.masked_attention(*(np.ascontiguousarray(x[:1, h:h + 1]) for x in (Qb, Kb, Vb)), "f16", masks)
            got = out[:1, h:h + 1].float().cpu().numpy().astype(np.float64)
            assert np.abs(got - ref).max() <= 5e-3
            assert np.linalg.norm(got - ref) / np.linalg.norm(ref) <= 1e-3
