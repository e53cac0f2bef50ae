"""GPU parity of metok_prefill_prune_batched against the CPU oracle: every video of a batch is checked like a call of
metok_prefill_prune on that video alone (scores within tolerance, the selection bit-exact on the GPU's own scores,
the compaction bit-exact), and entries behind a video's own kept count are left untouched."""
import numpy as np
import pytest
import torch

from oracle import metok_oracle as O
from paper_2506_02850_amd import synth
from tests.test_gpu_stage2 import check_prune, i32, make_layer, mk

pytestmark = pytest.mark.gpu

SENTINEL = -7


def stack(layers, field, dtype=None):
    arrs = [getattr(l, field) for l in layers]
    a = np.stack(arrs)
    return a if dtype is None else a.astype(dtype)


def run_batched(layers, segs, quotas, use_weight=True, orig=None, Tq=None, score_mode=0, in_place=False):
    Bm = mk()
    l0 = layers[0]
    dt = l0.dtype
    Tq = l0.n_text if Tq is None else Tq
    qs = [l.q_text[:, l.n_text - Tq:, :] for l in layers]
    B = len(layers)
    n_keep = [int(sum(q)) for q in quotas]
    keep_stride = max(n_keep) + 3                                  # padded on purpose
    S = l0.hidden.shape[0]
    out_stride = S if in_place else S - l0.n_vis + max(n_keep) + 2
    hidden = synth.to_torch(stack(layers, "hidden"), dt, "cuda")
    out = {name: torch.full((B, keep_stride), SENTINEL, dtype=torch.int32, device="cuda")
           for name in ("kept_idx", "token_seg_out", "token_event_out", "orig_idx_out")}
    out["orig_idx_out"] = torch.full((B, keep_stride + 5), SENTINEL, dtype=torch.int32, device="cuda")     # its own stride
    hidden_out = hidden if in_place else torch.full((B, out_stride, l0.hidden.shape[1]), float(SENTINEL), dtype=hidden.dtype, device="cuda")
    res = Bm.metok_prefill_prune_batched(
        hidden, l0.vis_start, l0.n_vis, i32(np.stack(segs)), quotas,
        q_text=synth.to_torch(np.stack(qs), dt, "cuda"), k_all=synth.to_torch(stack(layers, "k_all"), dt, "cuda"),
        token_event=i32(stack(layers, "token_event")),
        event_weight=torch.from_numpy(stack(layers, "event_weight", np.float32)).cuda() if use_weight else None,
        orig_idx=None if orig is None else i32(np.pad(np.stack(orig), ((0, 0), (0, 4)), constant_values=-1)),     # its own stride
        score_mode=score_mode,
        hidden_out=hidden_out, out=out, keep_stride=keep_stride, out_row_stride=out_stride)
    torch.cuda.synchronize()
    assert res["n_keep"] == n_keep
    host = {n: (t.float() if t.dtype == torch.bfloat16 else t).cpu().numpy() for n, t in res.items() if n != "n_keep"}
    per_video = []
    for b in range(B):
        rows = S - l0.n_vis + n_keep[b]
        got = dict(scores=host["scores"][b], kept_idx=host["kept_idx"][b, :n_keep[b]], hidden_out=host["hidden_out"][b, :rows],
                   token_seg_out=host["token_seg_out"][b, :n_keep[b]], token_event_out=host["token_event_out"][b, :n_keep[b]],
                   orig_idx_out=host["orig_idx_out"][b, :n_keep[b]])
        for name in ("kept_idx", "token_seg_out", "token_event_out", "orig_idx_out"):
            assert (host[name][b, n_keep[b]:] == SENTINEL).all(), f"video {b}: {name} written behind its kept count"
        if not in_place:
            assert (host["hidden_out"][b, rows:] == SENTINEL).all(), f"video {b}: hidden_out written behind its rows"
        per_video.append((got, qs[b]))
    return per_video


def layers_of(seeds, *shape, **kw):
    return [make_layer(s, *shape, **kw) for s in seeds]


def two_class_quotas(layer, rng, keep_key, keep_non):
    seg = (rng.random(layer.n_vis) < 0.45).astype(np.int32)
    return seg, [int(np.ceil(keep_key * int((seg == 0).sum()))), int(np.ceil(keep_non * int((seg == 1).sum())))]


@pytest.mark.parametrize("dtype,dh,Hq,Hkv,n_text,vis_start,score_mode", [
    ("bf16", 128, 28, 4, 40, 0, 0),          # LongVA / OV-7B heads
    ("bf16", 64, 14, 2, 24, 5, 0),           # OV-0.5B heads, system prefix
    ("f32", 64, 8, 8, 17, 3, 1),             # MHA, fp32, softmax over the visual keys only
    ("bf16", 128, 40, 40, 19, 0, 0),         # VILA-13B heads: five row splits of the score grid
])
def test_batched_levels_match_the_oracle_per_video(dtype, dh, Hq, Hkv, n_text, vis_start, score_mode):
    rng = np.random.default_rng(41)
    layers = layers_of([1100, 1200, 1300], 24, 100, 5, n_text, 48, Hq, Hkv, dh, dtype, vis_start=vis_start)
    segs, quotas = [], []
    for b, l in enumerate(layers):                                   # a different kept count in every video
        seg, q = two_class_quotas(l, rng, 0.3 + 0.2 * b, 0.1 * (b + 1))
        segs.append(seg); quotas.append(q)
    orig = [rng.permutation(l.n_vis).astype(np.int32) for l in layers]
    for b, (got, q) in enumerate(run_batched(layers, segs, quotas, orig=orig, score_mode=score_mode)):
        check_prune(layers[b], segs[b], quotas[b], got, q, orig_idx=orig[b], score_mode=score_mode)


def test_batch_of_eight_at_the_second_level_size_and_one_video_batches():
    # 18432 visual + 128 text keys, eight videos: each score workgroup walks 72 key subtiles (one video alone: 9)
    layers = layers_of(range(2000, 2800, 100), 128, 144, 8, 128, 64, 28, 4, 128, "bf16")
    segs = [np.zeros(l.n_vis, dtype=np.int32) for l in layers]
    quotas = [[l.n_vis // 2] for l in layers]
    for b, (got, q) in enumerate(run_batched(layers, segs, quotas, Tq=64)):
        if b in (0, 5, 7):                                         # the oracle's attention takes seconds per video
            check_prune(layers[b], segs[b], quotas[b], got, q)
    # a batch of one is the plain call
    got, q = run_batched(layers[:1], segs[:1], quotas[:1], Tq=64)[0]
    check_prune(layers[0], segs[0], quotas[0], got, q)


def test_batched_selection_on_supplied_scores_general_path_and_ties():
    Bm = mk()
    rng = np.random.default_rng(8)
    B, n, D = 4, 5000, 8
    hidden = rng.standard_normal((B, n + 3, D)).astype(np.float32)
    for n_seg in (3, 9):                                            # fast selection / one workgroup per class
        seg = rng.integers(0, n_seg, size=(B, n)).astype(np.int32)
        scores = np.round(rng.standard_normal((B, n)), 1).astype(np.float32)          # heavy exact ties
        scores[2] = 0.25                                            # one video with all scores equal
        quotas = [[int(rng.integers(0, int((seg[b] == c).sum()) + 1)) for c in range(n_seg)] for b in range(B)]
        quotas[3] = [0] * n_seg                                     # one video keeps nothing
        out = Bm.metok_prefill_prune_batched(torch.from_numpy(hidden).cuda(), 2, n, i32(seg), quotas,
                                             scores=torch.from_numpy(scores).cuda())
        torch.cuda.synchronize()
        for b in range(B):
            k = out["n_keep"][b]
            kept = O.segmented_topk(scores[b], seg[b], quotas[b])
            np.testing.assert_array_equal(out["kept_idx"][b, :k].cpu().numpy(), kept)
            np.testing.assert_array_equal(out["hidden_out"][b, :3 + k].cpu().numpy(), O.compact_hidden(hidden[b], 2, n, kept))
            np.testing.assert_array_equal(out["token_seg_out"][b, :k].cpu().numpy(), seg[b][kept])


def test_batched_in_place():
    rng = np.random.default_rng(15)
    layers = layers_of([3100, 3200, 3300], 16, 64, 4, 12, 256, 8, 2, 64, "bf16", vis_start=2)
    segs, quotas = [], []
    for b, l in enumerate(layers):
        seg, q = two_class_quotas(l, rng, 0.5, 0.2 + 0.3 * b)
        segs.append(seg); quotas.append(q)
    for b, (got, q) in enumerate(run_batched(layers, segs, quotas, in_place=True)):
        check_prune(layers[b], segs[b], quotas[b], got, q)


def test_batched_argument_errors():
    Bm = mk()
    hidden = torch.zeros((2, 20, 16), device="cuda")
    seg = torch.zeros((2, 10), dtype=torch.int32, device="cuda")
    sc = torch.zeros((2, 10), device="cuda")
    with pytest.raises(Bm.MetokError) as e:
        Bm.metok_prefill_prune_batched(hidden, 0, 10, seg, [[3], [5]], scores=sc, keep_stride=4)        # below the larger video
    assert "keep_stride" in str(e.value)
    with pytest.raises(Bm.MetokError):
        Bm.metok_prefill_prune_batched(hidden, 0, 10, seg, [[3], [11]], scores=sc)                      # quota > n_vis
    big = torch.zeros((65, 4, 16), device="cuda")
    with pytest.raises(Bm.MetokError) as e:
        Bm.metok_prefill_prune_batched(big, 0, 2, torch.zeros((65, 2), dtype=torch.int32, device="cuda"), [[1]] * 65,
                                       scores=torch.zeros((65, 2), device="cuda"))
    assert "batch" in str(e.value)
    assert Bm.lib().metok_prefill_prune_batched_workspace_bytes(65, 20, 0, 0, 0, 0, 10, 0) == 0
