"""GPU parity of metok_segment_compress (stage 1 in one call) against the CPU oracle and against the two
separate calls.  With every stride equal to 2 on an even grid the pooled tokens come out of the statistics
pass (one read of the frame features); they must then be bit-identical to what the two-pass path writes,
because both add the four cells of a window in the same order."""
import numpy as np
import pytest
import torch

from oracle import metok_oracle as O
from paper_2506_02850_amd import synth
from tests.parity import (RTOL, assert_pooled_bf16, assert_pooled_bf16_strict, assert_rel, assert_rows_close,
                          frame_score_scale)

pytestmark = pytest.mark.gpu


def mk():
    from paper_2506_02850_amd import binding
    return binding


def run_both(v, grid, k, alpha, beta, s1, s2, out_dtype, sim_mode=0, edge=0, reduce_=0):
    B = mk()
    feats = synth.to_torch(v.feats, v.dtype, "cuda")
    text = synth.to_torch(v.text_emb, v.dtype, "cuda")
    odt = torch.bfloat16 if out_dtype == "bf16" else torch.float32
    one = B.metok_segment_compress(feats, grid[0], grid[1], k, text, alpha, beta, s1, s2, sim_mode=sim_mode,
                                   event_reduce=reduce_, pool_edge=edge, out_dtype=odt)
    seg = B.metok_segment_events(feats, k, text, sim_mode=sim_mode)
    two = B.metok_compress_encoder_tokens(feats, grid[0], grid[1], seg["event_start"], alpha, beta, s1, s2,
                                          frame_score=seg["frame_score"], event_reduce=reduce_, pool_edge=edge, out_dtype=odt)
    torch.cuda.synchronize()
    return one, seg, two


def check(v, grid, k, alpha, beta, s1, s2, out_dtype, sim_mode=0, edge=0, reduce_=0, expect_strides=None, strict=False):
    """strict: the named configurations, held to the plain bars (see tests/parity.py)."""
    one, seg, two = run_both(v, grid, k, alpha, beta, s1, s2, out_dtype, sim_mode, edge, reduce_)
    rtol = RTOL[v.dtype]
    got = {n: (t.float() if t.dtype == torch.bfloat16 else t).cpu().numpy() for n, t in one.items()}
    # segmentation and scores against the oracle
    S = O.adjacent_frame_cosine(v.feats, sim_mode)
    if v.feats.shape[0] > 1:
        assert_rel(got["sim"], S, rtol, "sim", scale=np.abs(S).max())
    es, fe = O.event_boundaries(S, k)
    np.testing.assert_array_equal(got["event_start"], es)
    np.testing.assert_array_equal(got["frame_event"], fe)
    f_or = O.frame_text_score(v.feats, v.text_emb)
    assert_rel(got["frame_score"], f_or, rtol, "frame_score", scale=None if strict else frame_score_scale(v.feats, v.text_emb))
    # plan re-derived by the oracle from the GPU's own frame scores, pooled tokens against the exact means
    ref = O.compress_encoder_tokens(v.feats, grid, None, es, alpha, beta, s1, s2, reduce_, edge,
                                    frame_score=got["frame_score"].astype(np.float64))
    for name in ("event_is_key", "frame_is_key", "frame_stride", "frame_offsets"):
        np.testing.assert_array_equal(got[name], ref[name], err_msg=name)
    # ref's event scores are the oracle's reduction of the GPU's own frame scores: only the reduction differs
    assert_rel(got["event_score"], ref["event_score"], 1e-5, "event_score", scale=np.abs(f_or).max())
    M = int(ref["frame_offsets"][-1])
    np.testing.assert_array_equal(got["token_event"][:M], ref["token_event"])
    tokens = got["out_tokens"][:M]
    if out_dtype == "f32":
        assert_rows_close(tokens, ref["tokens"], rtol, "pooled tokens")
    else:
        cells = int(ref["frame_stride"].max()) ** 2
        if strict:
            assert_pooled_bf16_strict(tokens, ref["tokens"], "pooled tokens")
        else:
            assert_pooled_bf16(tokens, ref["tokens"], np.abs(v.feats).max(), cells, "pooled tokens")
        assert float((tokens.astype(np.float64) != O.round_to_bf16(ref["tokens"])).mean()) < 1e-3
    if expect_strides is not None:
        assert set(got["frame_stride"].tolist()) <= set(expect_strides)
    # the two separate calls: same decisions, bit-identical tokens
    for name in ("event_start", "frame_event"):
        assert torch.equal(one[name], seg[name]), name
    for name in ("event_is_key", "frame_is_key", "frame_stride", "frame_offsets"):
        assert torch.equal(one[name], two[name]), name
    assert torch.equal(one["token_event"][:M], two["token_event"][:M])
    assert torch.equal(one["out_tokens"][:M], two["out_tokens"][:M]), "one-call and two-call pooled tokens differ"
    return got


@pytest.mark.parametrize("out_dtype", ["bf16", "f32"])
def test_uniform_stride_two_encoder_config(out_dtype):
    # 32 x 576 x 1024 bf16, 8 events: 144 tokens per frame out of the statistics pass
    sh = synth.ENCODER
    got = check(synth.video_for(sh), sh.grid, sh.n_events, 1.0, 1.0, 2, 2, out_dtype, expect_strides={2}, strict=True)
    np.testing.assert_array_equal(got["frame_offsets"], 144 * np.arange(33))
    np.testing.assert_array_equal(got["event_start"], synth.video_for(sh).event_start)


@pytest.mark.parametrize("T,grid,d,dtype,k,alpha,beta,s1,s2", [
    (9, (4, 4), 64, "f32", 4, 1.0, 0.5, 2, 2),          # tiny grid, fp32, 16 chunks: most lanes idle
    (12, (6, 10), 512, "bf16", 3, 1.0, 1.0, 2, 2),      # 15 windows: the last workgroup is ragged
    (7, (8, 6), 1152, "bf16", 3, 1.0, 0.4, 2, 2),       # 144 chunks: three chunks per lane
    (10, (6, 6), 1024, "f32", 4, 1.0, 0.4, 2, 2),       # 256 chunks: four per lane
    (1, (4, 6), 128, "bf16", 1, 1.0, 1.0, 2, 2),        # single frame
    (2, (2, 2), 8, "bf16", 2, 1.0, 1.0, 2, 2),          # one window per frame
    (40, (4, 6), 2048, "bf16", 7, 1.0, 0.5, 2, 2),      # 256 chunks of bf16, several frame runs
    (6, (2, 2), 64, "f32", 2, 0.5, 0.5, 2, 3),          # 2, 3, 4, 6 all clamp to the 2 x 2 grid
    (8, (6, 6), 64, "f32", 3, 0.5, 0.5, 1, 1),          # not uniform (1 and 2): two passes
])
def test_one_call_shapes(T, grid, d, dtype, k, alpha, beta, s1, s2):
    v = synth.planted_video(777 + T + d, T, grid, d, min(k, T), 1, T, 0.15, dtype)
    for out_dtype in ("f32", "bf16"):
        check(v, grid, k, alpha, beta, s1, s2, out_dtype)


@pytest.mark.parametrize("case", ["odd grid", "adaptive", "token mean", "ceil edge", "wide rows"])
def test_one_call_falls_back_to_two_passes(case):
    if case == "odd grid":            # SigLIP 27 x 27, uniform stride 2: the last row and column are dropped
        v = synth.planted_video(31, 6, (27, 27), 64, 2, 2, 4, 0.15, "bf16")
        got = check(v, (27, 27), 2, 1.0, 1.0, 2, 2, "bf16", expect_strides={2})
        assert int(got["frame_offsets"][-1]) == 6 * 169
    elif case == "adaptive":          # the paper's LongVA setting
        v = synth.video_for(synth.ENCODER)
        check(v, (24, 24), 8, 0.5, 0.45, 2, 3, "bf16", expect_strides={2, 3, 4, 6}, strict=True)
    elif case == "token mean":
        v = synth.planted_video(32, 8, (4, 4), 64, 3, 1, 8, 0.15, "f32")
        check(v, (4, 4), 3, 1.0, 1.0, 2, 2, "f32", sim_mode=O.SIM_TOKEN_MEAN)
    elif case == "ceil edge":
        v = synth.planted_video(33, 5, (5, 7), 24, 2, 1, 5, 0.15, "f32")
        check(v, (5, 7), 2, 1.0, 1.0, 2, 2, "f32", edge=O.POOL_CEIL)
    else:                             # 4096 fp32 = 1024 chunks: too wide for the one-pass kernel
        v = synth.planted_video(34, 5, (2, 2), 4096, 2, 1, 5, 0.15, "f32")
        check(v, (2, 2), 2, 1.0, 1.0, 2, 2, "f32")


def test_one_call_at_256_frames_and_errors():
    B = mk()
    sh = synth.ENCODER_256
    v = synth.video_for(sh)
    got = check(v, sh.grid, sh.n_events, 1.0, 1.0, 2, 2, "bf16", expect_strides={2}, strict=True)
    assert int(got["frame_offsets"][-1]) == 256 * 144
    feats = torch.zeros((4, 16, 64), dtype=torch.float32, device="cuda")
    text = torch.ones(64, device="cuda")
    with pytest.raises(B.MetokError) as e:
        B.metok_segment_compress(feats, 4, 4, 9, text, 1.0, 1.0, 2, 2)
    assert e.value.code == -1 and "k must be" in str(e.value)
    with pytest.raises(B.MetokError) as e:
        B.metok_segment_compress(feats, 4, 4, 2, text, 1.0, 1.0, 2, 2, out={"out_tokens": torch.zeros((3, 64), device="cuda")})
    assert e.value.code == -4
    with pytest.raises(B.MetokError):
        B.metok_segment_compress(feats, 4, 4, 2, text, 1.0, 1.5, 2, 2)


@pytest.mark.parametrize("T,grid,d,dtype,k,alpha,beta,s1,s2,out_dtype", [
    (12, (6, 10), 512, "bf16", 3, 1.0, 1.0, 2, 2, "bf16"),     # one pass, ragged last workgroup
    (40, (4, 6), 2048, "bf16", 7, 1.0, 0.5, 2, 2, "f32"),      # one pass, several frame runs
    (10, (6, 6), 1024, "f32", 4, 1.0, 0.4, 2, 2, "f32"),       # one pass, fp32
    (9, (6, 6), 64, "bf16", 3, 0.5, 0.45, 2, 3, "bf16"),       # adaptive strides: two passes, each kernel once for the batch
    (21, (27, 27), 1152, "bf16", 5, 0.5, 0.4, 2, 3, "f32"),    # SigLIP grid, the OneVision setting, fp32 output
    (13, (5, 7), 24, "f32", 4, 0.3, 0.5, 1, 2, "f32"),         # odd grid, fp32, s / alpha rounds up
])
def test_batched_one_call_equals_the_single_video_call(T, grid, d, dtype, k, alpha, beta, s1, s2, out_dtype):
    """metok_segment_compress_batched: every video of the batch bit-identical to metok_segment_compress on that video
    (which `check` above holds against the oracle), the segmentation of one video also directly against the oracle."""
    B = mk()
    videos = [synth.planted_video(900 + 17 * b + T, T, grid, d, k, 1, T, 0.15, dtype) for b in range(3)]
    feats = synth.to_torch(np.stack([v.feats for v in videos]), dtype, "cuda")
    text = synth.to_torch(np.stack([v.text_emb for v in videos]), dtype, "cuda")
    odt = torch.bfloat16 if out_dtype == "bf16" else torch.float32
    got = B.metok_segment_compress_batched(feats, grid[0], grid[1], k, text, alpha, beta, s1, s2, out_dtype=odt)
    torch.cuda.synchronize()
    for b, v in enumerate(videos):
        one = B.metok_segment_compress(feats[b], grid[0], grid[1], k, text[b], alpha, beta, s1, s2, out_dtype=odt)
        torch.cuda.synchronize()
        M = int(one["frame_offsets"][-1])
        for name, t in one.items():
            rows = M if name in ("out_tokens", "token_event") else t.shape[0]
            assert torch.equal(got[name][b][:rows], t[:rows]), f"video {b}: {name}"
    es, fe = O.event_boundaries(O.adjacent_frame_cosine(videos[1].feats, 0), k)
    np.testing.assert_array_equal(got["event_start"][1].cpu().numpy(), es)
    np.testing.assert_array_equal(got["frame_event"][1].cpu().numpy(), fe)


def test_batched_one_call_at_256_frames_against_the_oracle():
    """Two 256-frame videos in one batched call: decisions and pooled tokens of the second video against the oracle."""
    B = mk()
    sh = synth.ENCODER_256
    v0, v1 = synth.video_for(sh), synth.planted_video(4242, sh.T, sh.grid, sh.d, sh.n_events, 8, 64, 0.15, "bf16")
    feats = synth.to_torch(np.stack([v0.feats, v1.feats]), "bf16", "cuda")
    text = synth.to_torch(np.stack([v0.text_emb, v1.text_emb]), "bf16", "cuda")
    got = B.metok_segment_compress_batched(feats, sh.grid[0], sh.grid[1], sh.n_events, text, 1.0, 1.0, 2, 2)
    torch.cuda.synchronize()
    g = {n: (t[1].float() if t.dtype == torch.bfloat16 else t[1]).cpu().numpy() for n, t in got.items()}
    S = O.adjacent_frame_cosine(v1.feats, 0)
    assert_rel(g["sim"], S, RTOL["bf16"], "sim", scale=np.abs(S).max())
    es, fe = O.event_boundaries(S, sh.n_events)
    np.testing.assert_array_equal(g["event_start"], es)
    np.testing.assert_array_equal(g["frame_event"], fe)
    assert_rel(g["frame_score"], O.frame_text_score(v1.feats, v1.text_emb), RTOL["bf16"], "frame_score")
    ref = O.compress_encoder_tokens(v1.feats, sh.grid, None, es, 1.0, 1.0, 2, 2, 0, 0, frame_score=g["frame_score"].astype(np.float64))
    for name in ("event_is_key", "frame_is_key", "frame_stride", "frame_offsets"):
        np.testing.assert_array_equal(g[name], ref[name], err_msg=name)
    np.testing.assert_array_equal(g["token_event"], ref["token_event"])
    assert_pooled_bf16_strict(g["out_tokens"], ref["tokens"], "pooled tokens")
    with pytest.raises(B.MetokError) as e:
        B.metok_segment_compress_batched(feats[:, :4].contiguous(), sh.grid[0], sh.grid[1], 2, text, 1.0, 1.0, 2, 2,
                                         workspace=torch.zeros(1024, dtype=torch.uint8, device="cuda"))
    assert "workspace" in str(e.value)
