"""GPU parity of stage 1 (metok_segment_events, metok_compress_encoder_tokens) against the CPU oracle."""
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


def run_segment(v: synth.Video, k: int, with_text=True, sim_mode=0):
    B = mk()
    feats = synth.to_torch(v.feats, v.dtype, "cuda")
    text = synth.to_torch(v.text_emb, v.dtype, "cuda") if with_text else None
    out = B.metok_segment_events(feats, k, text, sim_mode=sim_mode)
    torch.cuda.synchronize()
    return feats, text, {n: t.cpu().numpy() for n, t in out.items()}


def check_segment(v: synth.Video, k: int, got, with_text=True, sim_mode=0, strict=False):
    """strict: the named configurations, frame scores relative to the oracle's own value."""
    rtol = RTOL[v.dtype]
    S = O.adjacent_frame_cosine(v.feats, sim_mode)
    T = v.feats.shape[0]
    if T > 1:
        # cross-event similarities sit near 0: compare against the largest similarity
        assert_rel(got["sim"], S, rtol, "sim", scale=np.abs(S).max())
    es, fe = O.event_boundaries(S, k)
    if k > 1 and T > 2:
        # the boundary decision must not sit inside a near-tie band (the generators guarantee a wide gap)
        srt = np.sort(S)
        if k - 1 < len(srt):
            assert srt[k - 1] - srt[k - 2] > 1e-3 * abs(srt[k - 2]), "generator produced a near-tie at the boundary threshold"
    np.testing.assert_array_equal(got["event_start"], es)
    np.testing.assert_array_equal(got["frame_event"], fe)
    if with_text:
        f = O.frame_text_score(v.feats, v.text_emb)
        assert_rel(got["frame_score"], f, rtol, "frame_score", scale=None if strict else frame_score_scale(v.feats, v.text_emb))


@pytest.mark.parametrize("shapes", [synth.TINY, synth.ENCODER], ids=["tiny", "encoder"])
def test_segment_events_configs(shapes):
    v = synth.video_for(shapes)
    _, _, got = run_segment(v, shapes.n_events)
    check_segment(v, shapes.n_events, got, strict=True)
    np.testing.assert_array_equal(got["event_start"], v.event_start)      # planted boundaries recovered


@pytest.mark.parametrize("T,grid,d,dtype,k", [
    (5, (3, 5), 40, "bf16", 3),        # ragged: N = 15 tokens, d = 5 chunks
    (9, (7, 7), 1152, "bf16", 4),      # SigLIP width: 144 chunks -> whole-wave token groups
    (6, (5, 5), 132, "f32", 2),        # 33 chunks
    (1, (4, 4), 64, "f32", 1),         # single frame
    (2, (2, 2), 8, "bf16", 2),         # smallest pair, every frame its own event
    (40, (4, 6), 2048, "bf16", 7),     # several frame runs, 256 chunks
    (12, (3, 3), 4096, "f32", 12),     # widest supported fp32 rows, k = T
])
def test_segment_events_shapes(T, grid, d, dtype, k):
    n_events = min(k, T)
    v = synth.planted_video(1234 + T + d, T, grid, d, n_events, 1, T, 0.15, dtype)
    _, _, got = run_segment(v, k)
    check_segment(v, k, got)


@pytest.mark.parametrize("sim_mode", [O.SIM_TOKEN_MEAN, O.SIM_POOLED], ids=["token_mean", "pooled"])
@pytest.mark.parametrize("T,grid,d,dtype,k,with_text", [
    (8, (4, 4), 64, "f32", 3, True),           # the tiny configuration
    (5, (3, 5), 40, "bf16", 3, True),          # ragged: 15 tokens, 5 chunks
    (9, (7, 7), 1152, "bf16", 4, False),       # whole-wave token groups, no text pass
    (64, (24, 24), 1024, "bf16", 8, True),     # the encoder configuration
    (40, (4, 6), 2048, "bf16", 7, True),       # several frame runs per workgroup column
    (1, (4, 4), 64, "f32", 1, True),           # single frame: no similarities
    (12, (3, 3), 4096, "f32", 12, False),      # widest fp32 rows, k = T
])
def test_segment_events_alternative_similarity_readings(sim_mode, T, grid, d, dtype, k, with_text):
    v = synth.planted_video(4321 + T + d, T, grid, d, min(k, T), 1, T, 0.15, dtype)
    _, _, got = run_segment(v, k, with_text=with_text, sim_mode=sim_mode)
    check_segment(v, k, got, with_text=with_text, sim_mode=sim_mode)
    assert ("frame_score" in got) == with_text


def test_segment_similarity_modes_differ_and_bad_mode_is_rejected():
    B = mk()
    v = synth.planted_video(99, 10, (4, 4), 64, 3, 1, 10, 0.4, "f32")
    sims = [run_segment(v, 3, sim_mode=m)[2]["sim"] for m in (0, 1, 2)]
    # with token noise of this size the three readings give visibly different numbers
    assert np.abs(sims[0] - sims[1]).max() > 1e-4 and np.abs(sims[0] - sims[2]).max() > 1e-4
    with pytest.raises(B.MetokError):
        run_segment(v, 3, sim_mode=3)


def test_segment_without_text_and_equal_frames():
    v = synth.planted_video(77, 10, (4, 4), 64, 1, 10, 10, 0.0, "f32")     # sigma 0: all frames identical
    _, _, got = run_segment(v, 4, with_text=False)
    np.testing.assert_allclose(got["sim"], np.ones(9), rtol=1e-6)
    np.testing.assert_array_equal(got["event_start"], [0, 1, 2, 3, 10])    # ties -> lowest indices
    assert "frame_score" not in got


def test_segment_zero_frames_guard():
    feats = np.zeros((4, 6, 16), dtype=np.float32)
    feats[2] = 1.0
    v = synth.Video(feats=feats, text_emb=np.ones(16, dtype=np.float32), dtype="f32", grid=(2, 3), n_events=1,
                    event_start=np.array([0, 4]), centroids=np.zeros((1, 16)), text_weights=np.ones(1), sigma=0.0)
    _, _, got = run_segment(v, 2)
    np.testing.assert_array_equal(got["sim"], [0.0, 0.0, 0.0])
    np.testing.assert_allclose(got["frame_score"], [0.0, 0.0, 1.0, 0.0], rtol=1e-6)
    np.testing.assert_array_equal(got["event_start"], [0, 1, 4])


def compress_case(v: synth.Video, grid, k, alpha, beta, s1, s2, event_reduce, edge, out_dtype, fused=True, strict=False):
    B = mk()
    feats, text, seg = run_segment(v, k)
    es_dev = torch.from_numpy(seg["event_start"]).cuda()
    fs_dev = torch.from_numpy(seg["frame_score"]).cuda() if fused else None
    out = B.metok_compress_encoder_tokens(feats, grid[0], grid[1], es_dev, alpha, beta, s1, s2,
                                          text_emb=text, frame_score=fs_dev, event_reduce=event_reduce,
                                          pool_edge=edge, out_dtype=torch.bfloat16 if out_dtype == "bf16" else torch.float32)
    torch.cuda.synchronize()
    got = {n: (t.float() if t.dtype == torch.bfloat16 else t).cpu().numpy() for n, t in out.items()}
    rtol = RTOL[v.dtype]

    # frame scores as the oracle computes them; the decisions are then re-derived by the oracle from
    # the GPU's own float32 scores, so that an fp32-vs-fp64 rounding of a score cannot flip a ranking unnoticed
    f_or = O.frame_text_score(v.feats, v.text_emb)
    assert_rel(got["frame_score"], f_or, rtol, "frame_score", scale=None if strict else frame_score_scale(v.feats, v.text_emb))
    ref = O.compress_encoder_tokens(v.feats, grid, v.text_emb, seg["event_start"], alpha, beta, s1, s2,
                                    event_reduce, edge, frame_score=got["frame_score"].astype(np.float64))
    ref_own = O.compress_encoder_tokens(v.feats, grid, v.text_emb, seg["event_start"], alpha, beta, s1, s2,
                                        event_reduce, edge)
    # an event score is a mean (or max) of signed frame scores: error relative to their magnitude
    assert_rel(got["event_score"], ref_own["event_score"], rtol, "event_score",
               scale=None if strict else frame_score_scale(v.feats, v.text_emb).max())
    np.testing.assert_array_equal(got["event_is_key"], ref["event_is_key"])
    np.testing.assert_array_equal(got["frame_is_key"], ref["frame_is_key"])
    np.testing.assert_array_equal(got["frame_stride"], ref["frame_stride"])
    np.testing.assert_array_equal(got["frame_offsets"], ref["frame_offsets"])
    M = int(ref["frame_offsets"][-1])
    np.testing.assert_array_equal(got["token_event"][:M], ref["token_event"])
    # the oracle's own decisions agree unless a ranking sits within rounding distance (never with these generators)
    np.testing.assert_array_equal(ref["frame_stride"], ref_own["frame_stride"])
    tokens = got["out_tokens"][:M]
    if out_dtype == "f32":
        assert_rows_close(tokens, ref["tokens"], rtol, "pooled tokens")
    else:
        # bf16 output: within one bf16 ulp of the exact mean; exact agreement with the rounded oracle mean
        # except for rare double-rounding flips (fp32 mean -> bf16 vs fp64 mean -> bf16)
        cells = int(ref["frame_stride"].max()) ** 2
        if strict:
            assert_pooled_bf16_strict(tokens, ref["tokens"], "pooled tokens")
        else:
            assert_pooled_bf16(tokens, ref["tokens"], np.abs(v.feats).max(), cells, "pooled tokens")
        mismatch = float((tokens.astype(np.float64) != O.round_to_bf16(ref["tokens"])).mean())
        assert mismatch < 1e-3, f"bf16 rounding mismatch fraction {mismatch}"
    return got, ref


def test_compress_tiny_both_settings():
    v = synth.video_for(synth.TINY)
    got, _ = compress_case(v, (4, 4), 4, 1.0, 1.0, 2, 2, O.EVENT_REDUCE_MEAN, O.POOL_FLOOR, "f32", strict=True)
    assert int(got["frame_offsets"][-1]) == 32 and set(got["frame_stride"].tolist()) == {2}
    got, _ = compress_case(v, (4, 4), 4, 0.5, 0.5, 1, 2, O.EVENT_REDUCE_MEAN, O.POOL_FLOOR, "f32", strict=True)
    assert set(got["frame_stride"].tolist()) <= {1, 2, 4}


@pytest.mark.parametrize("out_dtype", ["f32", "bf16"])
def test_compress_encoder_config(out_dtype):
    v = synth.video_for(synth.ENCODER)
    # uniform stride 2: exactly 144 tokens per frame
    got, _ = compress_case(v, (24, 24), 8, 1.0, 1.0, 2, 2, O.EVENT_REDUCE_MEAN, O.POOL_FLOOR, out_dtype, strict=True)
    assert int(got["frame_offsets"][-1]) == 32 * 144
    # the paper's LongVA setting: (s1, s2) = (2, 3), alpha = 0.5, beta = 0.45
    got, ref = compress_case(v, (24, 24), 8, 0.5, 0.45, 2, 3, O.EVENT_REDUCE_MEAN, O.POOL_FLOOR, out_dtype, strict=True)
    rows = np.diff(got["frame_offsets"])
    assert set(rows.tolist()) <= {144, 64, 36, 16} and len(set(rows.tolist())) == 4


@pytest.mark.parametrize("grid,d,dtype,s1,s2,alpha,edge,reduce_,fused", [
    ((27, 27), 64, "bf16", 2, 3, 0.5, O.POOL_FLOOR, O.EVENT_REDUCE_MEAN, True),    # SigLIP grid, floor: 169/81/36/16
    ((27, 27), 64, "bf16", 2, 3, 0.5, O.POOL_CEIL, O.EVENT_REDUCE_MAX, False),     # ceil: partial edge windows
    ((5, 7), 24, "f32", 1, 2, 0.3, O.POOL_CEIL, O.EVENT_REDUCE_MEAN, False),       # non-square, s/alpha rounds up
    ((6, 10), 1152, "bf16", 3, 4, 0.7, O.POOL_FLOOR, O.EVENT_REDUCE_MAX, True),    # wide rows, 144 chunks
    ((4, 4), 16, "f32", 5, 9, 0.5, O.POOL_FLOOR, O.EVENT_REDUCE_MEAN, True),       # strides clamp to the grid
])
def test_compress_shapes(grid, d, dtype, s1, s2, alpha, edge, reduce_, fused):
    T, k = 11, 4
    v = synth.planted_video(99 + d, T, grid, d, k, 1, 6, 0.1, dtype)
    for out_dtype in ("f32", "bf16"):
        compress_case(v, grid, k, alpha, 0.4, s1, s2, reduce_, edge, out_dtype, fused=fused)


def test_maximum_frame_count():
    """T = METOK_MAX_FRAMES: the one-workgroup kernels rank 8191 similarities / 8192 frames, eight per thread."""
    B = mk()
    T, grid, d, k = 8192, (2, 2), 64, 61
    v = synth.planted_video(8192, T, grid, d, k, 1, T, 0.15, "bf16")
    _, _, got = run_segment(v, k)
    check_segment(v, k, got)
    np.testing.assert_array_equal(got["event_start"], v.event_start)
    compress_case(v, grid, k, 0.5, 0.45, 1, 2, O.EVENT_REDUCE_MEAN, O.POOL_FLOOR, "f32")
    # every frame its own event: k = T, all T - 1 similarities are boundaries
    feats = synth.to_torch(v.feats, v.dtype, "cuda")
    out = B.metok_segment_events(feats, T)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out["event_start"].cpu().numpy(), np.arange(T + 1))
    np.testing.assert_array_equal(out["frame_event"].cpu().numpy(), np.arange(T))
    with pytest.raises(B.MetokError):
        B.metok_segment_events(torch.zeros((T + 1, 4, 8), dtype=torch.float32, device="cuda"), 2)


@pytest.mark.parametrize("T,k", [(4096, 37), (3000, 2999), (2049, 2), (5000, 1)])
def test_long_videos_with_tied_similarities(T, k):
    """Above 2048 frames the boundaries come from a radix select of the (k-1)-th lowest similarity; equal similarities
    are taken lowest index first.  Frames drawn from four distinct vectors make most adjacent pairs tie exactly (the
    same two vectors give the same fp32 cosine wherever they meet), at the threshold too."""
    B = mk()
    rng = np.random.default_rng(T + k)
    basis = rng.standard_normal((4, 2, 16)).astype(np.float32)
    pick = rng.integers(0, 4, size=T)
    feats_np = basis[pick]
    out = B.metok_segment_events(torch.from_numpy(feats_np).cuda(), k)
    torch.cuda.synchronize()
    sim_gpu = out["sim"].cpu().numpy()
    assert len(np.unique(sim_gpu)) <= 10                             # 4 + 6 unordered pairs of vectors
    S = O.adjacent_frame_cosine(feats_np.astype(np.float64))
    assert_rel(sim_gpu, S, RTOL["f32"], "sim", scale=np.abs(S).max())
    # the decision is checked on the GPU's own fp32 similarities (ties are exact there), bit for bit
    es, fe = O.event_boundaries(sim_gpu, k)
    np.testing.assert_array_equal(out["event_start"].cpu().numpy(), es)
    np.testing.assert_array_equal(out["frame_event"].cpu().numpy(), fe)


@pytest.mark.parametrize("T,starts", [(5000, [0, 5000]), (4099, [0, 1, 4098, 4099]), (3001, [0, 7, 1501, 3001]),
                                      (3000, list(range(3001))), (4100, [0] + list(range(1100, 4101)))])
def test_key_frames_of_long_events_with_tied_scores(T, starts):
    """Algorithm 1's key frames inside events of thousands of frames, and key events among thousands of events: up to
    1024 items every item is ranked against all others (keys read from LDS four at a time, so event starts that are
    not multiples of four matter), beyond that the n-th largest key is found bit by bit; equal scores lowest index
    first either way.  Frames drawn from four vectors tie exactly in their frame-text score."""
    B = mk()
    rng = np.random.default_rng(T)
    basis = rng.standard_normal((4, 4, 16)).astype(np.float32)
    feats_np = basis[rng.integers(0, 4, size=T)]
    text_np = rng.standard_normal(16).astype(np.float32)
    es = np.asarray(starts, dtype=np.int32)
    out = B.metok_compress_encoder_tokens(torch.from_numpy(feats_np).cuda(), 2, 2, torch.from_numpy(es).cuda(), 0.5, 0.45, 1, 2,
                                          text_emb=torch.from_numpy(text_np).cuda(), out_dtype=torch.float32)
    torch.cuda.synchronize()
    fs = out["frame_score"].cpu().numpy()
    assert len(np.unique(fs)) <= 4
    ref = O.compress_encoder_tokens(feats_np.astype(np.float64), (2, 2), text_np.astype(np.float64), es, 0.5, 0.45, 1, 2,
                                    O.EVENT_REDUCE_MEAN, O.POOL_FLOOR, frame_score=fs.astype(np.float64))
    np.testing.assert_array_equal(out["frame_is_key"].cpu().numpy(), ref["frame_is_key"])
    np.testing.assert_array_equal(out["event_is_key"].cpu().numpy(), ref["event_is_key"])
    np.testing.assert_array_equal(out["frame_stride"].cpu().numpy(), ref["frame_stride"])
    np.testing.assert_array_equal(out["frame_offsets"].cpu().numpy(), ref["frame_offsets"])
    # ceil(0.45 len) key frames in every event
    for a, b in zip(starts[:-1], starts[1:]):
        assert int(out["frame_is_key"][a:b].sum()) == int(np.ceil(0.45 * (b - a) - 1e-9))


def test_argument_errors_are_reported():
    B = mk()
    feats = torch.zeros((4, 4, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(B.MetokError) as e:
        B.metok_segment_events(feats, 5)
    assert e.value.code == -1 and "k must be" in str(e.value)
    with pytest.raises(B.MetokError):
        B.metok_segment_events(torch.zeros((4, 4, 6), dtype=torch.float32, device="cuda"), 2)      # d % 4
    es = torch.tensor([0, 4], dtype=torch.int32, device="cuda")
    with pytest.raises(B.MetokError) as e:
        B.metok_compress_encoder_tokens(feats, 2, 2, es, 0.5, 0.5, 2, 2, text_emb=torch.zeros(64, device="cuda"),
                                        out_tokens=torch.zeros((3, 64), device="cuda"))
    assert e.value.code == -4
    with pytest.raises(B.MetokError):
        B.metok_compress_encoder_tokens(feats, 2, 2, es, 1.5, 0.5, 2, 2, text_emb=torch.zeros(64, device="cuda"))
    with pytest.raises(ValueError):
        B.metok_segment_events(feats.cpu(), 2)
