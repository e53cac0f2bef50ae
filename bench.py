#!/usr/bin/env python3
"""Throughput of METok's token-compression hot path on one MI355X.

One step = one pass of stages 1-3 over a batch of synthetic, LongVA-7B-shaped 256-frame videos:

  stage 1  per video: metok_segment_compress (segmentation, scores, plan and pooling in one call) on
           CLIP-ViT-L/336-shaped features [256, 576, 1024] bf16 (16 planted events, uniform stride 2 ->
           256 x 144 tokens, so the pooled tokens come out of the statistics pass: one read of the features);
  stage 2  per video: three metok_prefill_prune levels (keep 0.5 / 0.5 / 0.5 of the current count) on
           hidden states [36864 + 128, 3584] bf16 with 28 query / 4 kv heads of 128 and the last 64 text
           positions as queries; event ids come from stage 1, retained indices are carried level to level;
  stage 3  the whole batch: metok_kv_compact of a 28-layer KV cache [8, 4, 36992, 128] bf16 (K and V) to
           the per-layer retained sets of stage 2 (levels start at layers 3, 10, 19) plus the text rows.

All inputs are resident in HBM before the timed region.  `value` is visual tokens entering stage 1 per
second.  The JSON line also carries the roofline of the dominant kernel (the KV compaction, HBM bound;
duration measured with events on the launch stream inside the timed region) and the CPU oracle timed
on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
FRAMES, GRID, D_VIS = 256, 24, 1024
N_EVENTS = 16
TOK_PER_FRAME = 144
N_VIS = FRAMES * TOK_PER_FRAME           # 36864
N_TEXT, TQ = 128, 64
D_HID, HQ, HKV, DH = 3584, 28, 4, 128
N_LAYERS, L_H = 28, (3, 10, 19)
KEEP = (0.5, 0.5, 0.5)


def level_counts():
    out, n = [], N_VIS
    for r in KEEP:
        n = int(math.ceil(r * n - 1e-9))
        out.append(n)
    return out                                   # 18432, 9216, 4608


class Workload:
    def __init__(self, batch: int, device: str, n_streams: int = 8, seed: int = 250602850 + 4):
        import torch
        from paper_2506_02850_amd import binding, synth

        self.torch, self.B, self.batch, self.dev = torch, binding, batch, device
        gen = torch.Generator(device=device)
        gen.manual_seed(seed)
        bf = torch.bfloat16
        counts = level_counts()
        self.counts = counts
        self.n_in = [N_VIS] + counts[:-1]
        rng = np.random.Generator(np.random.PCG64(seed))

        # ---- stage 1 inputs: planted events, unit centroid + N(0, 0.2^2) noise per entry
        self.feats, self.text = [], []
        for b in range(batch):
            lens = synth.event_lengths(rng, FRAMES, N_EVENTS, 4, 40)
            cent = torch.from_numpy(synth.unit_rows(rng, N_EVENTS, D_VIS)).to(device)
            frame_event = torch.from_numpy(np.repeat(np.arange(N_EVENTS), lens)).to(device)
            f = torch.randn((FRAMES, GRID * GRID, D_VIS), generator=gen, device=device, dtype=torch.float32)
            f.mul_(0.2).add_(cent[frame_event][:, None, :])
            self.feats.append(f.to(bf))
            w = torch.linspace(1.0, 0.2, N_EVENTS, device=device)[torch.randperm(N_EVENTS, generator=gen, device=device)]
            t = (w[:, None] * cent).sum(0)
            self.text.append((t / t.norm()).to(bf))
            del f
        # ---- stage 2 inputs
        S0 = N_VIS + N_TEXT
        self.hidden0 = [torch.randn((S0, D_HID), generator=gen, device=device, dtype=bf) for _ in range(batch)]
        self.K = [[torch.randn((HKV, n + N_TEXT, DH), generator=gen, device=device, dtype=bf) for n in self.n_in]
                  for _ in range(batch)]
        self.Q = [[torch.randn((HQ, TQ, DH), generator=gen, device=device, dtype=bf) for _ in self.n_in]
                  for _ in range(batch)]
        self.weight = [torch.rand(N_EVENTS, generator=gen, device=device) + 0.5 for _ in range(batch)]
        self.seg0 = torch.zeros(N_VIS, dtype=torch.int32, device=device)
        self.hidden_out = [[torch.empty((c + N_TEXT, D_HID), dtype=bf, device=device) for c in counts]
                           for _ in range(batch)]
        # ---- stage 3: KV cache and per-level index lists [B, kept + text]; the text part is fixed
        self.k_layers = [torch.empty((batch, HKV, S0, DH), dtype=bf, device=device).normal_(generator=gen)
                         for _ in range(N_LAYERS)]
        self.v_layers = [torch.empty((batch, HKV, S0, DH), dtype=bf, device=device).normal_(generator=gen)
                         for _ in range(N_LAYERS)]
        text_rows = torch.arange(N_VIS, S0, dtype=torch.int32, device=device)
        self.idx_level = []
        for c in counts:
            t = torch.empty((batch, c + N_TEXT), dtype=torch.int32, device=device)
            t[:, c:] = text_rows
            t[:, :c] = torch.arange(c, dtype=torch.int32, device=device)      # overwritten by stage 2
            self.idx_level.append(t)
        self.idx_layers = []
        for l in range(N_LAYERS):
            level = sum(1 for b in L_H if l >= b)
            self.idx_layers.append(None if level == 0 else self.idx_level[level - 1])
        self.new_len = torch.empty(N_LAYERS, dtype=torch.int32, device=device)
        self.kv_ws = torch.empty(binding.metok_kv_compact_workspace_bytes(N_LAYERS, batch, HKV, S0, DH, binding.BF16),
                                 dtype=torch.uint8, device=device)
        # ---- preallocated outputs and workspaces (nothing is allocated inside a step)
        lib = binding.lib()
        # Videos are independent until stage 3, so their stage-1/2 calls are spread over a few streams: the
        # one-workgroup planning and selection kernels of one video then overlap with the streaming kernels
        # of another.  One workspace per stream (calls on a stream are ordered, so they can share it).
        self.n_streams = max(1, min(n_streams, batch))
        self.graph = None
        self.streams = [torch.cuda.Stream(device=device) for _ in range(self.n_streams)] if self.n_streams > 1 else []
        self.ws1 = [torch.empty(max(lib.metok_segment_events_workspace_bytes(FRAMES, GRID * GRID, D_VIS, binding.BF16),
                                    lib.metok_compress_encoder_tokens_workspace_bytes(FRAMES, GRID, GRID, D_VIS, binding.BF16)),
                                dtype=torch.uint8, device=device) for _ in range(self.n_streams)]
        self.ws2 = [torch.empty(lib.metok_prefill_prune_workspace_bytes(S0, HQ, HKV, DH, TQ, N_VIS, binding.BF16),
                                dtype=torch.uint8, device=device) for _ in range(self.n_streams)]
        i32, f32, u8 = torch.int32, torch.float32, torch.uint8
        self.seg_out = [dict(sim=torch.empty(FRAMES - 1, dtype=f32, device=device),
                             event_start=torch.empty(N_EVENTS + 1, dtype=i32, device=device),
                             frame_event=torch.empty(FRAMES, dtype=i32, device=device),
                             frame_score=torch.empty(FRAMES, dtype=f32, device=device)) for _ in range(batch)]
        self.cmp_out = [dict(out_tokens=torch.empty((N_VIS, D_VIS), dtype=bf, device=device),
                             frame_offsets=torch.empty(FRAMES + 1, dtype=i32, device=device),
                             token_event=torch.empty(N_VIS, dtype=i32, device=device),
                             event_is_key=torch.empty(N_EVENTS, dtype=u8, device=device),
                             frame_is_key=torch.empty(FRAMES, dtype=u8, device=device),
                             frame_stride=torch.empty(FRAMES, dtype=i32, device=device),
                             event_score=torch.empty(N_EVENTS, dtype=f32, device=device),
                             frame_score=torch.empty(FRAMES, dtype=f32, device=device)) for _ in range(batch)]
        self.s1_out = [{**self.seg_out[b], **self.cmp_out[b]} for b in range(batch)]
        self.prune_out = [[dict(scores=torch.empty(n, dtype=f32, device=device),
                                kept_idx=torch.empty(c, dtype=i32, device=device),
                                token_seg_out=torch.empty(c, dtype=i32, device=device),
                                token_event_out=torch.empty(c, dtype=i32, device=device),
                                orig_idx_out=self.idx_level[lv][b, :c])
                           for lv, (n, c) in enumerate(zip(self.n_in, counts))] for b in range(batch)]
        torch.cuda.synchronize()

    # algorithmic bytes (what the method itself must move)
    def stage1_bytes(self):
        read = FRAMES * GRID * GRID * D_VIS * 2          # uniform stride 2: statistics and pooling share one pass over V
        return self.batch * (read + N_VIS * D_VIS * 2)

    def gather_bytes(self):
        return self.batch * sum(2 * (c + N_TEXT) * D_HID * 2 for c in self.counts)

    def kv_rows(self):
        per_video = 0
        for l in range(N_LAYERS):
            level = sum(1 for b in L_H if l >= b)
            if level:
                per_video += self.counts[level - 1] + N_TEXT
        return per_video                           # kept token-layers per video (256,640)

    def kv_bytes(self):
        idx_bytes = self.batch * self.kv_rows() * 4
        return self.batch * self.kv_rows() * HKV * DH * 2 * 2 * 2 + idx_bytes     # K and V, read + write

    def score_flops(self):
        return self.batch * sum(2 * 2 * HQ * TQ * (n + N_TEXT) * DH for n in self.n_in)      # two passes

    def stage1(self, b):
        ws = self.ws1[b % self.n_streams]
        return self.B.metok_segment_compress(self.feats[b], GRID, GRID, N_EVENTS, self.text[b], 1.0, 1.0, 2, 2,
                                             workspace=ws, out=self.s1_out[b])

    def stage2(self, b, token_event):
        B = self.B
        ws2 = self.ws2[b % self.n_streams]
        h, tseg, tev, orig = self.hidden0[b], self.seg0, token_event, None
        for lv, (n, c) in enumerate(zip(self.n_in, self.counts)):
            r = B.metok_prefill_prune(h, 0, n, tseg, [c], q_text=self.Q[b][lv], k_all=self.K[b][lv], token_event=tev,
                                      event_weight=self.weight[b], orig_idx=orig, hidden_out=self.hidden_out[b][lv],
                                      workspace=ws2, out=self.prune_out[b][lv])
            h, tseg, tev, orig = r["hidden_out"], r["token_seg_out"], r["token_event_out"], r["orig_idx_out"]

    def stage3(self):
        self.B.metok_kv_compact(self.k_layers, self.v_layers, self.idx_layers, new_len=self.new_len, workspace=self.kv_ws)

    def stages_1_2(self):
        """Stage 1 and the three pruning levels of every video, spread over the streams, joined on the current stream."""
        torch = self.torch
        if self.streams:
            main = torch.cuda.current_stream()
            for i, st in enumerate(self.streams):
                st.wait_stream(main)                   # the previous step's KV compaction still reads the index lists
                with torch.cuda.stream(st):
                    for b in range(i, self.batch, self.n_streams):
                        cmp = self.stage1(b)
                        self.stage2(b, cmp["token_event"])
            for st in self.streams:
                main.wait_stream(st)
        else:
            for b in range(self.batch):
                cmp = self.stage1(b)
                self.stage2(b, cmp["token_event"])

    def capture(self):
        """Records the stage-1/2 launches of one step (about 270 kernels on 8 streams) into a HIP graph.  The
        library calls only launch kernels on the stream they are given (no allocation, copy, memset or
        synchronisation), so they can be captured as they are; the KV compaction stays an ordinary launch so
        that it can be bracketed by events."""
        torch = self.torch
        self.graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(self.graph, stream=side):
                self.stages_1_2()
        torch.cuda.current_stream().wait_stream(side)

    def step(self, kv_events=None):
        if self.graph is not None:
            self.graph.replay()
        else:
            self.stages_1_2()
        if kv_events is not None:
            kv_events[0].record()
        self.stage3()
        if kv_events is not None:
            kv_events[1].record()


def time_stages(w: Workload, reps: int):
    """Per-stage GPU time (ms per step), measured after the timed region; informational."""
    torch = w.torch
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(reps)]
    for r in range(reps):
        ev[r][0].record()
        toks = [w.stage1(b)["token_event"] for b in range(w.batch)]
        ev[r][1].record()
        for b in range(w.batch):
            w.stage2(b, toks[b])
        ev[r][2].record()
        w.stage3()
        ev[r][3].record()
    torch.cuda.synchronize()
    return [float(np.median([ev[r][i].elapsed_time(ev[r][i + 1]) for r in range(reps)])) for i in range(3)]


def cpu_baseline(n_videos: int = 8):
    """The oracle, unchanged, single-threaded, on whole videos of the same workload: stage 1 on 256 frames, the
    three pruning levels, and the KV compaction of the video's 25 moving layers -- for n_videos videos (8 = the
    batch of one step; inputs from the seeded CPU generators; only the oracle calls are timed: about 1.3 s per
    video on the MI355X machine's host, 6 s on the build container)."""
    from threadpoolctl import threadpool_limits

    from oracle import metok_oracle as O
    from paper_2506_02850_amd import synth

    counts = level_counts()
    t_stage = [0.0, 0.0, 0.0]
    with threadpool_limits(limits=1):
        for vid in range(n_videos):
            # stage 1: 256 frames, uniform stride 2
            v = synth.planted_video(100 + vid, FRAMES, (GRID, GRID), D_VIS, N_EVENTS, 4, 40, 0.2, "bf16")
            t0 = time.perf_counter()
            S = O.adjacent_frame_cosine(v.feats)
            es, _ = O.event_boundaries(S, N_EVENTS)
            cmp = O.compress_encoder_tokens(v.feats, (GRID, GRID), v.text_emb, es, 1.0, 1.0, 2, 2)
            t_stage[0] += time.perf_counter() - t0
            ev = cmp["token_event"]
            del v, cmp
            # stage 2: three levels, fresh activations per level, metadata carried
            seg = np.zeros(N_VIS, dtype=np.int32)
            kept_sets = []
            orig = np.arange(N_VIS)
            for lv, c in enumerate(counts):
                layer = synth.prefill_layer(200 + 10 * vid + lv, ev, N_EVENTS, N_TEXT, D_HID, HQ, HKV, DH, "bf16")
                t0 = time.perf_counter()
                r = O.prefill_prune(layer.hidden, layer.q_text[:, N_TEXT - TQ:], layer.k_all, 0, ev.shape[0], seg, ev,
                                    layer.event_weight, [c])
                t_stage[1] += time.perf_counter() - t0
                kept = r["kept_idx"]
                ev, seg, orig = ev[kept], seg[kept], orig[kept]
                kept_sets.append(orig.astype(np.int32))
                del layer, r
            # stage 3: the video's 25 moving layers, K and V of 4 heads each
            S0 = N_VIS + N_TEXT
            sched = synth.kv_layer_schedule(N_LAYERS, L_H, N_VIS, N_TEXT, kept_sets)
            slab = np.random.default_rng(vid).integers(-32768, 32767, size=(S0, DH), dtype=np.int16)
            t0 = time.perf_counter()
            for l in range(N_LAYERS):
                if sched[l] is None:
                    continue
                for _ in range(HKV * 2):
                    O.kv_compact(slab, sched[l])
            t_stage[2] += time.perf_counter() - t0
    total = sum(t_stage)
    return dict(value=n_videos * FRAMES * GRID * GRID / total, unit="tokens/s", cores=1, kind="oracle",
                sample=f"{n_videos} whole videos (one step has 8): stage 1 on 256 frames, three pruning levels, KV compaction of "
                       "25 layers x 4 heads x (K, V); oracle calls only, one thread",
                seconds_by_stage=[round(t, 3) for t in t_stage], seconds=round(total, 3))


def read_traffic():
    """HBM bytes per KV-compaction launch from the committed rocprofv3 counter summary, if present."""
    path = os.path.join(ROOT, "profiles", "kv_compact_longva256_b8_pmc.txt")
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch"):
                    return float(line.split()[1])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--streams", type=int, default=8, help="streams that share the per-video stage-1/2 work")
    ap.add_argument("--no-graph", action="store_true", help="launch the stage-1/2 kernels one by one instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", choices=["all", "kv", "copy", "prune"], default="all",
                    help="kv / copy / prune: run only the KV compaction, the calibration copy or the stage-2 calls "
                         "(for profiler counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import torch

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU (there is no CPU path)")
    from paper_2506_02850_amd import binding

    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.only == "copy":
        n = 1 << 30
        src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(args.warmup + args.steps):
            binding.metok_calib_copy(dst, src)
        torch.cuda.synchronize()
        print(json.dumps({"calib_copy_bytes": n}))
        return

    w = Workload(args.batch, dev, args.streams)
    if args.only == "kv":
        for b in range(args.batch):                      # index lists as the full pipeline produces them
            w.stage2(b, w.stage1(b)["token_event"])
        for _ in range(args.warmup + args.steps):
            w.stage3()
        torch.cuda.synchronize()
        print(json.dumps({"kv_bytes_per_launch": w.kv_bytes()}))
        return

    if args.only == "prune":
        toks = [w.stage1(b)["token_event"] for b in range(args.batch)]
        for _ in range(args.warmup + args.steps):
            for b in range(args.batch):
                w.stage2(b, toks[b])
        torch.cuda.synchronize()
        print(json.dumps({"score_flops_per_step": w.score_flops()}))
        return

    w.step()                                             # eager once: loads code objects before any capture
    torch.cuda.synchronize()
    if not args.no_graph:
        w.capture()
    for _ in range(args.warmup):
        w.step()
    torch.cuda.synchronize()
    kv_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for s in range(args.steps):
        w.step(kv_ev[s])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    kv_ms = float(np.mean([a.elapsed_time(b) for a, b in kv_ev]))
    stage_ms = time_stages(w, 5)
    tokens_per_step = args.batch * FRAMES * GRID * GRID
    ms_per_step = elapsed * 1e3 / args.steps
    achieved = w.kv_bytes() / (kv_ms * 1e-3) / 1e9
    out = {
        "metric": "visual tokens processed/sec through stages 1-3",
        "value": tokens_per_step / (elapsed / args.steps),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "LongVA-7B-shaped, 256 frames: hierarchical prefill + decoding KV compaction configs "
                               "chained behind stage 1 at 256 x 576 x 1024",
                   "batch_videos": args.batch, "frames": FRAMES, "tokens_per_frame_in": GRID * GRID,
                   "tokens_per_frame_pooled": TOK_PER_FRAME, "prune_levels": level_counts(), "text_tokens": N_TEXT,
                   "text_queries": TQ, "kv_layers": N_LAYERS, "L_H": list(L_H), "streams": w.n_streams,
                   "launch": "eager" if w.graph is None else "stages 1-2 replayed from one HIP graph, KV compaction launched directly"},
        "roofline": {"kernel": "move_rows_kernel", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": read_traffic(),
                     "algorithmic_bytes_per_launch": w.kv_bytes(), "ms_per_launch": kv_ms},
        "stages": {"stage1_ms": stage_ms[0], "stage2_ms": stage_ms[1], "stage3_ms": stage_ms[2],
                   "stage1_GBs": w.stage1_bytes() / stage_ms[0] / 1e6,
                   "stage2_gather_bytes": w.gather_bytes(), "stage2_score_flops": w.score_flops(),
                   "stage3_GBs": w.kv_bytes() / stage_ms[2] / 1e6},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
