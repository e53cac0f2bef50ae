"""metok_prefill_prune_static (the entry point for callers that cannot allocate a workspace) against
metok_prefill_prune on the same inputs: every output bit for bit, on two calls in a row, the second with a
smaller input, so that what the first call left in the shared static array is shown not to matter."""
import numpy as np
import pytest
import torch

from paper_2506_02850_amd import synth

pytestmark = pytest.mark.gpu


def i32(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).cuda()


def make_case(seed, n_frames, tpf, n_events, n_text, D, Hq, Hkv, dh, dtype, vis_start):
    rng = np.random.Generator(np.random.PCG64(seed))
    ev = synth.token_events_for_frames(rng, n_frames, tpf, n_events)
    layer = synth.prefill_layer(seed + 1, ev, n_events, n_text, D, Hq, Hkv, dh, dtype, vis_start=vis_start)
    seg = (1 - layer.event_is_key[layer.token_event]).astype(np.int32)
    return layer, seg


def run_both(B, layer, seg, quotas):
    dt = layer.dtype
    args = dict(q_text=synth.to_torch(layer.q_text, dt, "cuda"), k_all=synth.to_torch(layer.k_all, dt, "cuda"),
                token_event=i32(layer.token_event), event_weight=torch.from_numpy(layer.event_weight).cuda())
    hidden = synth.to_torch(layer.hidden, dt, "cuda")
    tseg = i32(seg)
    ref = B.metok_prefill_prune(hidden, layer.vis_start, layer.n_vis, tseg, quotas, **args)
    # outputs of the static call are allocated beforehand and poisoned: the call itself allocates nothing
    out = {n: torch.full_like(t, -7 if t.dtype == torch.int32 else 3) for n, t in ref.items()}
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    got = B.metok_prefill_prune_static(hidden, layer.vis_start, layer.n_vis, tseg, quotas, out=out, **args)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for name, t in ref.items():
        assert got[name].data_ptr() == out[name].data_ptr()
        assert torch.equal(got[name], t), f"{name} differs between the static-scratch call and metok_prefill_prune"


def test_static_scratch_call_matches_the_workspace_call_twice_in_a_row():
    from paper_2506_02850_amd import binding as B
    assert B.metok_static_scratch_bytes() == 8 << 20
    # first call: LongVA head layout, 96 frames x 144 tokens (13824 visual keys, 14 selection tiles), 64 text rows
    big, seg_big = make_case(901, 96, 144, 13, 64, 256, 28, 4, 128, "bf16", 0)
    n_key, n_non = int((seg_big == 0).sum()), int((seg_big == 1).sum())
    run_both(B, big, seg_big, B.metok_retention_quotas(1, 0.55, 0.5, n_key, n_non))
    # second call, smaller and of another shape: fewer keys, other heads, a system prefix, fp32
    small, seg_small = make_case(902, 11, 24, 4, 19, 48, 6, 3, 64, "f32", 5)
    n_key, n_non = int((seg_small == 0).sum()), int((seg_small == 1).sum())
    run_both(B, small, seg_small, B.metok_retention_quotas(1, 0.55, 0.5, n_key, n_non))
