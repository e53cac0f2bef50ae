"""One step of bench.py's workload, launched the way bench.py times it -- 8 LongVA-7B-shaped 256-frame videos,
stage 1 and the three pruning levels as batched calls (28 launches) replayed from one HIP graph, then one in-place
KV compaction of the 28-layer cache -- checked against the CPU oracle: whole outputs where the oracle finishes in
seconds (stage 1 of a video, the scores of a level), sampled rows for the bulk tensors.  The same for bench.py's
--per-video launch (one call per video on 8 streams, one graph) and for the KV pass on its own stream."""
import numpy as np
import pytest
import torch

from oracle import metok_oracle as O
from tests.parity import RTOL, assert_pooled_bf16_strict, assert_rel, near_tie_report

pytestmark = pytest.mark.gpu


def f64(t):
    return t.float().cpu().numpy().astype(np.float64)


@pytest.mark.parametrize("mode,kv_overlap", [("batched", False), ("per-video", False), ("batched", True)])
def test_one_bench_step_matches_the_oracle(mode, kv_overlap):
    import bench
    w = bench.Workload(8, "cuda:0", 8)
    w.mode = mode
    n_text, counts, n_in = bench.N_TEXT, w.counts, w.n_in
    S = bench.N_VIS + n_text

    # slabs of the cache as they are before the in-place compaction (one per pruning level, one untouched layer)
    slabs = [(0, 0, 1, 2), (3, 1, 0, 0), (9, 0, 5, 3), (12, 1, 7, 1), (27, 0, 2, 2)]       # (layer, K|V, video, head)
    before = {s: (w.v_layers if s[1] else w.k_layers)[s[0]][s[2], s[3]].clone() for s in slabs}

    w.stages_1_2()                       # eager once, so that every code object is loaded before the capture
    torch.cuda.synchronize()
    w.configure(mode, kv_overlap=kv_overlap, use_graph=True)
    w.step()                             # graph replay of stages 1-2 + KV compaction (index lists of set 0)
    torch.cuda.synchronize()

    grid = (bench.GRID, bench.GRID)
    for b, levels in ((0, (0, 2)), (5, (1,))):
        print(f"video {b}: stage 1", flush=True)
        V = w.feats[b].float().cpu().numpy()
        t = w.text[b].float().cpu().numpy()
        out = w.s1_out[b]
        Ssim = O.adjacent_frame_cosine(V)
        assert_rel(out["sim"].cpu().numpy(), Ssim, RTOL["bf16"], "sim", scale=np.abs(Ssim).max())
        es, fe = O.event_boundaries(Ssim, bench.N_EVENTS)
        np.testing.assert_array_equal(out["event_start"].cpu().numpy(), es)
        np.testing.assert_array_equal(out["frame_event"].cpu().numpy(), fe)
        assert_rel(out["frame_score"].cpu().numpy(), O.frame_text_score(V, t), RTOL["bf16"], "frame_score")
        np.testing.assert_array_equal(out["frame_offsets"].cpu().numpy(), 144 * np.arange(bench.FRAMES + 1))
        np.testing.assert_array_equal(out["frame_stride"].cpu().numpy(), np.full(bench.FRAMES, 2))
        tok_event = np.repeat(fe, 144).astype(np.int32)
        np.testing.assert_array_equal(out["token_event"].cpu().numpy(), tok_event)
        for i in (0, 17 + b, 128, 255):
            ref = O.pool_frame(V[i], grid, 2)
            got = f64(out["out_tokens"][144 * i:144 * (i + 1)])
            assert_pooled_bf16_strict(got, ref, f"video {b} frame {i}")
            assert float((got != O.round_to_bf16(ref)).mean()) < 1e-3
        del V

        # the chain of metadata the three levels carry, re-derived by the oracle from the GPU's own scores
        ev, orig = tok_event, np.arange(bench.N_VIS)
        for lv in range(3):
            n, c = n_in[lv], counts[lv]
            po = w.prune_out[b][lv]
            scores = po["scores"].cpu().numpy()
            kept = po["kept_idx"].cpu().numpy()
            seg = np.zeros(n, dtype=np.int32)
            np.testing.assert_array_equal(kept, O.segmented_topk(scores, seg, [c]))
            if lv in levels:
                print(f"video {b}: scores of level {lv + 1} ({n} visual keys)", flush=True)
                q = f64(w.Q[b][lv])
                k = f64(w.K[b][lv])
                a = O.text_to_visual_attention(q, k, 0, n)
                s_or = O.event_weighted_scores(a, ev, w.weight[b].cpu().numpy().astype(np.float64))
                worst = assert_rel(scores, s_or, RTOL["bf16"], "scores")
                rep = near_tie_report(s_or, seg, [c], kept, O.segmented_topk(s_or, seg, [c]))
                print(f"  worst rel err {worst:.2e}, near-tie band {rep}", flush=True)
            hidden_in = w.hidden0[b] if lv == 0 else w.hidden_out[b][lv - 1]
            rows = np.concatenate([kept, np.arange(n, n + n_text)])
            ref_rows = O.compact_hidden(np.arange(n + n_text)[:, None], 0, n, kept)[:, 0]
            np.testing.assert_array_equal(rows, ref_rows)
            assert torch.equal(w.hidden_out[b][lv], hidden_in[torch.from_numpy(ref_rows).cuda()])
            np.testing.assert_array_equal(po["token_event_out"].cpu().numpy(), ev[kept])
            np.testing.assert_array_equal(po["orig_idx_out"].cpu().numpy(), orig[kept])
            ev, orig = ev[kept], orig[kept]
            # the retained original positions are what the KV compaction of this level's layers uses
            np.testing.assert_array_equal(w.idx_level[lv][b, :c].cpu().numpy(), orig)
            np.testing.assert_array_equal(w.idx_level[lv][b, c:].cpu().numpy(), np.arange(bench.N_VIS, S))

    print("KV cache", flush=True)
    want_len = []
    for l in range(bench.N_LAYERS):
        level = sum(1 for x in bench.L_H if l >= x)
        want_len.append(S if level == 0 else counts[level - 1] + n_text)
    np.testing.assert_array_equal(w.new_len.cpu().numpy(), want_len)
    for s in slabs:
        l, which, b, h = s
        level = sum(1 for x in bench.L_H if l >= x)
        idx = None if level == 0 else w.idx_level[level - 1][b].cpu().numpy()
        ref = O.kv_compact(before[s].view(torch.int16).cpu().numpy(), idx)
        got = (w.v_layers if which else w.k_layers)[l][b, h, :ref.shape[0]].view(torch.int16).cpu().numpy()
        assert np.array_equal(got, ref), f"layer {l} {'V' if which else 'K'} video {b} head {h}"
