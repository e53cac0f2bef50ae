#!/usr/bin/env python3
"""Throughput of METok's token-compression hot path on one MI355X.

One step = one pass of stages 1-3 over a batch of synthetic, LongVA-7B-shaped 256-frame videos:

  stage 1  the batch in one call: metok_segment_compress_batched (segmentation, scores, plan and pooling) on
           CLIP-ViT-L/336-shaped features [8, 256, 576, 1024] bf16 (16 planted events per video, uniform stride 2 ->
           256 x 144 tokens, so the pooled tokens come out of the statistics pass: one read of the features);
  stage 2  the batch in one call per level: three metok_prefill_prune_batched levels (keep 0.5 / 0.5 / 0.5 of the
           current count) on hidden states [8, 36864 + 128, 3584] bf16 with 28 query / 4 kv heads of 128 and the
           last 64 text positions as queries; keys carry a per-event mean shift and the queries lean towards one
           target event; event ids come from stage 1, retained indices are carried level to level;
  stage 3  the whole batch: metok_kv_compact of a 28-layer KV cache [8, 4, 36992, 128] bf16 (K and V) to
           the per-layer retained sets of stage 2 (levels start at layers 3, 10, 19) plus the text rows.

--per-video runs stages 1-2 as one call per video on 8 streams instead (the same kernels with one video per launch).

All inputs are resident in HBM before the timed region.  `value` is visual tokens entering stage 1 per
second.  The JSON line also carries
  roofline      the dominant kernel (the in-place row mover of the KV compaction, HBM bound), its duration taken
                from events the library records around that kernel inside the timed region;
  kernel_fractions_of_peak   every streaming kernel's fraction of the HBM peak and every score pass's fraction of the
                bf16 MFMA peak, side by side (the figures of `stages`);
  stages        per kernel family, measured in the same run right after the timed region with the same event
                hook: duration (min / median), algorithmic GB/s or TFLOP/s and the fraction of the peak; per
                stage the tokens entering it per second;
  configs       call-level timings of the encoder, single-level prefill, hierarchical prefill and KV
                configurations on their own;
  cpu_baseline  the CPU oracle on the same workload, one thread; cpu_baseline_all_cores: the same oracle, one
                video per worker process.  Both run before the GPU is touched.
"""
from __future__ import annotations

import argparse
import ctypes
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
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 MFMA, published
FRAMES, GRID, D_VIS = 256, 24, 1024
N_EVENTS = 16
TOK_PER_FRAME = 144
N_VIS = FRAMES * TOK_PER_FRAME           # 36864
N_TEXT, TQ = 128, 64
D_HID, HQ, HKV, DH = 3584, 28, 4, 128
N_LAYERS, L_H = 28, (3, 10, 19)
KEEP = (0.5, 0.5, 0.5)
ADAPTIVE = dict(alpha=0.5, beta=0.45, s1=2, s2=3)      # the LongVA setting of the appendix "Implementation Details"

# kernel ids of metok_trace_kernel (include/metok.h)
TRACE = dict(frame_stats=1, pool=2, frame_stats_pool2=3, segment=4, plan=5, row_stats=6, col_sums=7, select=8,
             write_index=9, gather_rows=10, move_rows=11)


def level_counts():
    out, n = [], N_VIS
    for r in KEEP:
        n = int(math.ceil(r * n - 1e-9))
        out.append(n)
    return out                                   # 18432, 9216, 4608


class HipEvents:
    """hipEvent_t handles for the library's kernel trace hook (plain HIP through ctypes; torch's Event objects do not
    expose their handle before the first record)."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        rc = self.hip.hipEventCreate(ctypes.byref(ev))
        if rc != 0 or not ev.value:
            raise RuntimeError(f"hipEventCreate failed ({rc})")
        return ev

    def elapsed_ms(self, a, b) -> float:
        if self.hip.hipEventSynchronize(b) != 0:
            raise RuntimeError("hipEventSynchronize failed")
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b)
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return float(ms.value)


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
        S0 = N_VIS + N_TEXT
        lib = binding.lib()
        i32, f32, u8 = torch.int32, torch.float32, torch.uint8

        # ---- stage 1 inputs: planted events, unit centroid + N(0, 0.2^2) noise per entry.  Every tensor of the batch is one
        # allocation with a leading video dimension (the batched calls take them whole); the per-video lists are views.
        self.feats_b = torch.empty((batch, FRAMES, GRID * GRID, D_VIS), dtype=bf, device=device)
        self.text_b = torch.empty((batch, D_VIS), dtype=bf, device=device)
        planted_events = []
        for b in range(batch):
            lens = synth.event_lengths(rng, FRAMES, N_EVENTS, 4, 40)
            cent = torch.from_numpy(synth.unit_rows(rng, N_EVENTS, D_VIS)).to(device)
            frame_event = torch.from_numpy(np.repeat(np.arange(N_EVENTS), lens)).to(device)
            planted_events.append(frame_event)
            f = torch.randn((FRAMES, GRID * GRID, D_VIS), generator=gen, device=device, dtype=torch.float32)
            f.mul_(0.2).add_(cent[frame_event][:, None, :])
            self.feats_b[b] = f.to(bf)
            w = torch.linspace(1.0, 0.2, N_EVENTS, device=device)[torch.randperm(N_EVENTS, generator=gen, device=device)]
            t = (w[:, None] * cent).sum(0)
            self.text_b[b] = (t / t.norm()).to(bf)
            del f
        self.feats = [self.feats_b[b] for b in range(batch)]
        self.text = [self.text_b[b] for b in range(batch)]
        # ---- preallocated outputs and workspaces (nothing is allocated inside a step)
        self.n_streams = max(1, min(n_streams, batch))
        self.mode, self.kv_overlap, self.graphs, self.step_no, self.split = "batched", False, [], 0, 1
        self.streams = [torch.cuda.Stream(device=device) for _ in range(self.n_streams)] if self.n_streams > 1 else []
        self.ws1_b = torch.empty(lib.metok_segment_compress_batched_workspace_bytes(batch, FRAMES, GRID, GRID, D_VIS, binding.BF16),
                                 dtype=torch.uint8, device=device)
        self.ws2_b = torch.empty(lib.metok_prefill_prune_batched_workspace_bytes(batch, S0, HQ, HKV, DH, TQ, N_VIS, binding.BF16),
                                 dtype=torch.uint8, device=device)
        # the per-video calls (one workspace per stream: calls on a stream are ordered, so they can share it)
        self.ws1 = [torch.empty(lib.metok_segment_compress_workspace_bytes(FRAMES, GRID, GRID, D_VIS, binding.BF16),
                                dtype=torch.uint8, device=device) for _ in range(self.n_streams)]
        self.ws2 = [torch.empty(lib.metok_prefill_prune_workspace_bytes(S0, HQ, HKV, DH, TQ, N_VIS, binding.BF16),
                                dtype=torch.uint8, device=device) for _ in range(self.n_streams)]

        def stage1_outputs(lead):
            return dict(sim=torch.empty(lead + (FRAMES - 1,), dtype=f32, device=device),
                        event_start=torch.empty(lead + (N_EVENTS + 1,), dtype=i32, device=device),
                        frame_event=torch.empty(lead + (FRAMES,), dtype=i32, device=device),
                        frame_score=torch.empty(lead + (FRAMES,), dtype=f32, device=device),
                        out_tokens=torch.empty(lead + (N_VIS, D_VIS), dtype=bf, device=device),
                        frame_offsets=torch.empty(lead + (FRAMES + 1,), dtype=i32, device=device),
                        token_event=torch.empty(lead + (N_VIS,), dtype=i32, device=device),
                        event_is_key=torch.empty(lead + (N_EVENTS,), dtype=u8, device=device),
                        frame_is_key=torch.empty(lead + (FRAMES,), dtype=u8, device=device),
                        frame_stride=torch.empty(lead + (FRAMES,), dtype=i32, device=device),
                        event_score=torch.empty(lead + (N_EVENTS,), dtype=f32, device=device))
        self.s1_out_b = stage1_outputs((batch,))
        self.s1_out = [{k: v[b] for k, v in self.s1_out_b.items()} for b in range(batch)]
        self.s1_adaptive_out = stage1_outputs(())        # the two-pass adaptive setting is measured on one video at a time

        # ---- stage 3: KV cache and per-level index lists [B, kept + text]; the text part is fixed.  Two sets of lists:
        # the KV compaction of one step reads one set while the next step's pruning already fills the other.
        self.k_layers = [torch.empty((batch, HKV, S0, DH), dtype=bf, device=device).normal_(generator=gen)
                         for _ in range(N_LAYERS)]
        self.v_layers = [torch.empty((batch, HKV, S0, DH), dtype=bf, device=device).normal_(generator=gen)
                         for _ in range(N_LAYERS)]
        text_rows = torch.arange(N_VIS, S0, dtype=torch.int32, device=device)
        self.idx_level_sets, self.idx_layers_sets = [], []
        for _ in range(2):
            levels = []
            for c in counts:
                t = torch.empty((batch, c + N_TEXT), dtype=torch.int32, device=device)
                t[:, c:] = text_rows
                t[:, :c] = torch.arange(c, dtype=torch.int32, device=device)      # overwritten by stage 2
                levels.append(t)
            self.idx_level_sets.append(levels)
            self.idx_layers_sets.append([None if sum(1 for b in L_H if l >= b) == 0 else levels[sum(1 for b in L_H if l >= b) - 1]
                                         for l in range(N_LAYERS)])
        self.idx_level, self.idx_layers = self.idx_level_sets[0], self.idx_layers_sets[0]
        self.new_len = torch.empty(N_LAYERS, dtype=torch.int32, device=device)
        self.kv_ws = torch.empty(binding.metok_kv_compact_workspace_bytes(N_LAYERS, batch, HKV, S0, DH, binding.BF16),
                                 dtype=torch.uint8, device=device)

        # ---- stage 2 inputs with the event structure of the parity generators (synth.prefill_layer): keys of an
        # event share a mean shift, the text queries lean towards one target event, hidden rows carry a per-event
        # shift.  The keys of level 2 and 3 belong to the survivors of the level before, so the levels are run
        # once here, in order, to learn which tokens those are (the timed steps repeat exactly these selections).
        self.seg0_b = torch.zeros((batch, N_VIS), dtype=torch.int32, device=device)
        self.seg0 = self.seg0_b[0]
        self.hidden_out_b = [torch.empty((batch, c + N_TEXT, D_HID), dtype=bf, device=device) for c in counts]
        self.hidden_out = [[self.hidden_out_b[lv][b] for lv in range(len(counts))] for b in range(batch)]
        shared = [dict(scores=torch.empty((batch, n), dtype=f32, device=device),
                       kept_idx=torch.empty((batch, c), dtype=i32, device=device),
                       token_seg_out=torch.empty((batch, c), dtype=i32, device=device),
                       token_event_out=torch.empty((batch, c), dtype=i32, device=device))
                  for n, c in zip(self.n_in, counts)]
        # orig_idx_out of a level is the leading block of that level's KV index lists (its own stride: kept + text)
        self.prune_out_b_sets = [[dict(shared[lv], orig_idx_out=self.idx_level_sets[p][lv]) for lv in range(len(counts))]
                                 for p in range(2)]
        self.prune_out = [[dict({k: v[b] for k, v in shared[lv].items()}, orig_idx_out=self.idx_level[lv][b, :c])
                           for lv, c in enumerate(counts)] for b in range(batch)]
        self.hidden0_b = torch.empty((batch, S0, D_HID), dtype=bf, device=device)
        self.weight_b = torch.rand((batch, N_EVENTS), generator=gen, device=device) + 0.5
        self.Q_b = [torch.empty((batch, HQ, TQ, DH), dtype=bf, device=device) for _ in self.n_in]
        self.K_b = [torch.empty((batch, HKV, n + N_TEXT, DH), dtype=bf, device=device) for n in self.n_in]
        mus = []
        for b in range(batch):
            mu = torch.randn((N_EVENTS, DH), generator=gen, device=device)
            target = int(torch.randint(0, N_EVENTS, (1,), generator=gen, device=device))
            shift = torch.randn(N_EVENTS, generator=gen, device=device)
            tev = planted_events[b].repeat_interleave(TOK_PER_FRAME)            # event of every pooled token
            h = torch.randn((S0, D_HID), generator=gen, device=device, dtype=torch.float32)
            h[:N_VIS] += shift[tev][:, None]
            self.hidden0_b[b] = h.to(bf)
            del h
            for lv in range(len(self.n_in)):
                self.Q_b[lv][b] = (torch.randn((HQ, TQ, DH), generator=gen, device=device) + 0.5 * mu[target]).to(bf)
            mus.append(mu)
        self.hidden0 = [self.hidden0_b[b] for b in range(batch)]
        self.weight = [self.weight_b[b] for b in range(batch)]
        self.Q = [[self.Q_b[lv][b] for lv in range(len(self.n_in))] for b in range(batch)]
        self.K = [[self.K_b[lv][b] for lv in range(len(self.n_in))] for b in range(batch)]
        tev_b = torch.stack([planted_events[b].repeat_interleave(TOK_PER_FRAME) for b in range(batch)]).to(torch.int32)
        for lv, n in enumerate(self.n_in):
            for b in range(batch):
                k = torch.randn((HKV, n + N_TEXT, DH), generator=gen, device=device)
                k[:, :n] += 0.5 * mus[b][tev_b[b].long()][None]
                self.K_b[lv][b] = k.to(bf)
                del k
            if lv + 1 < len(self.n_in):
                tev_b = self.prune_level_batched(lv, tev_b, 0)["token_event_out"].clone()
        torch.cuda.synchronize()

    # ---- algorithmic bytes / flops (what the method itself must move or compute)
    def stage1_fused_bytes(self):                  # per video: one read of V, pooled tokens written
        return FRAMES * GRID * GRID * D_VIS * 2 + N_VIS * D_VIS * 2

    def gather_bytes(self, lv):                    # per video and level: every output row read and written once
        return 2 * (self.counts[lv] + N_TEXT) * D_HID * 2

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

    def score_flops(self, lv):                     # per video and level, one pass over the keys
        return 2 * HQ * TQ * (self.n_in[lv] + N_TEXT) * DH

    # ---- the calls
    def stage1(self, b):
        ws = self.ws1[b % self.n_streams]
        return self.B.metok_segment_compress(self.feats[b], GRID, GRID, N_EVENTS, self.text[b], 1.0, 1.0, 2, 2,
                                             workspace=ws, out=self.s1_out[b])

    def stage1_adaptive(self, b):
        """Algorithm 1 with the paper's LongVA strides: two passes over the features (statistics, then pooling)."""
        ws, o, a = self.ws1[0], self.s1_adaptive_out, ADAPTIVE
        seg = self.B.metok_segment_events(self.feats[b], N_EVENTS, self.text[b], workspace=ws, out=o)
        return self.B.metok_compress_encoder_tokens(self.feats[b], GRID, GRID, seg["event_start"], a["alpha"], a["beta"], a["s1"], a["s2"],
                                                    frame_score=seg["frame_score"], workspace=ws, out=o)

    def prune_level(self, b, lv, token_event):
        n, c = self.n_in[lv], self.counts[lv]
        prev = self.prune_out[b][lv - 1] if lv > 0 else None
        h = self.hidden0[b] if lv == 0 else self.hidden_out[b][lv - 1]
        tseg = self.seg0 if lv == 0 else prev["token_seg_out"]
        orig = None if lv == 0 else prev["orig_idx_out"]
        return self.B.metok_prefill_prune(h, 0, n, tseg, [c], q_text=self.Q[b][lv], k_all=self.K[b][lv], token_event=token_event,
                                          event_weight=self.weight[b], orig_idx=orig, hidden_out=self.hidden_out[b][lv],
                                          workspace=self.ws2[b % self.n_streams], out=self.prune_out[b][lv])

    def stage1_batched(self, part=None):
        """Stage 1 of the whole batch in one call (part = (first video, end, workspace): of a share of the batch)."""
        b0, b1, ws = part if part is not None else (0, self.batch, self.ws1_b)
        return self.B.metok_segment_compress_batched(self.feats_b[b0:b1], GRID, GRID, N_EVENTS, self.text_b[b0:b1], 1.0, 1.0, 2, 2,
                                                     workspace=ws, out={k: v[b0:b1] for k, v in self.s1_out_b.items()})

    def prune_level_batched(self, lv, token_event, p, part=None):
        """Level lv of the whole batch (or of a share of it) in one call; p selects the set of KV index lists that receives
        the retained indices."""
        b0, b1, ws = part if part is not None else (0, self.batch, self.ws2_b)
        n, c = self.n_in[lv], self.counts[lv]
        cut = lambda d: {k: v[b0:b1] for k, v in d.items()}
        prev = cut(self.prune_out_b_sets[p][lv - 1]) if lv > 0 else None
        h = self.hidden0_b if lv == 0 else self.hidden_out_b[lv - 1]
        tseg = self.seg0_b[b0:b1] if lv == 0 else prev["token_seg_out"]
        orig = None if lv == 0 else prev["orig_idx_out"]
        return self.B.metok_prefill_prune_batched(h[b0:b1], 0, n, tseg, [[c]] * (b1 - b0), q_text=self.Q_b[lv][b0:b1],
                                                  k_all=self.K_b[lv][b0:b1], token_event=token_event,
                                                  event_weight=self.weight_b[b0:b1], orig_idx=orig,
                                                  hidden_out=self.hidden_out_b[lv][b0:b1], workspace=ws,
                                                  out=cut(self.prune_out_b_sets[p][lv]))

    def stage2_batched(self, token_event, p=0, part=None):
        tev = token_event
        for lv in range(len(self.n_in)):
            tev = self.prune_level_batched(lv, tev, p, part)["token_event_out"]

    def stage2(self, b, token_event):
        tev = token_event
        for lv in range(len(self.n_in)):
            tev = self.prune_level(b, lv, tev)["token_event_out"]

    def stage3(self, p=0):
        self.B.metok_kv_compact(self.k_layers, self.v_layers, self.idx_layers_sets[p], new_len=self.new_len, workspace=self.kv_ws)

    def stages_1_2_per_video(self):
        """Stage 1 and the three pruning levels of every video as calls of their own, spread over the streams and joined
        on the current stream."""
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

    def stages_1_2(self, p=0):
        """Stage 1 and the three pruning levels of the batch; the retained indices go to set p of the KV index lists."""
        if self.mode == "per-video":
            return self.stages_1_2_per_video()
        if self.split <= 1:
            cmp = self.stage1_batched()
            self.stage2_batched(cmp["token_event"], p)
            return
        # the batch in `split` shares, each on a stream of its own: the ALU-bound score passes of one share can then run
        # beside the HBM-bound kernels of another
        torch = self.torch
        main = torch.cuda.current_stream()
        per = (self.batch + self.split - 1) // self.split
        for i in range(self.split):
            b0, b1 = i * per, min(self.batch, (i + 1) * per)
            if b0 >= b1:
                continue
            st = self.streams[i]
            st.wait_stream(main)
            with torch.cuda.stream(st):
                cmp = self.stage1_batched((b0, b1, self.ws1_parts[i]))
                self.stage2_batched(cmp["token_event"], p, (b0, b1, self.ws2_parts[i]))
        for i in range(self.split):
            main.wait_stream(self.streams[i])

    def configure(self, mode="batched", kv_overlap=False, use_graph=True, split=1):
        """mode: "batched" (one call per stage and level for the whole batch: 28 launches per step) or "per-video" (one
        call per video, 8 streams: about 230 launches).  kv_overlap: the KV compaction of a step runs on a stream of its
        own, beside the next step's stages 1-2 (which fill the other set of index lists).  use_graph: the stage-1/2 launches
        are replayed from a HIP graph.  The library calls only launch kernels on the stream they are given (no allocation,
        copy, memset or synchronisation), so they can be captured as they are; the KV compaction stays an ordinary launch
        so that the library can bracket its kernel with events."""
        torch = self.torch
        self.mode = mode
        self.split = max(1, min(int(split), len(self.streams) if self.streams else 1)) if mode == "batched" else 1
        if self.split > 1:
            lib, S0 = self.B.lib(), N_VIS + N_TEXT
            per = (self.batch + self.split - 1) // self.split
            self.ws1_parts = [torch.empty(lib.metok_segment_compress_batched_workspace_bytes(per, FRAMES, GRID, GRID, D_VIS, self.B.BF16),
                                          dtype=torch.uint8, device=self.dev) for _ in range(self.split)]
            self.ws2_parts = [torch.empty(lib.metok_prefill_prune_batched_workspace_bytes(per, S0, HQ, HKV, DH, TQ, N_VIS, self.B.BF16),
                                          dtype=torch.uint8, device=self.dev) for _ in range(self.split)]
        self.kv_overlap = bool(kv_overlap) and mode == "batched"
        self.step_no = 0
        self.kv_stream = torch.cuda.Stream(device=self.dev) if self.kv_overlap else None
        self.filled = [torch.cuda.Event() for _ in range(2)]        # stages 1-2 have filled set p
        self.consumed = [torch.cuda.Event() for _ in range(2)]      # the KV compaction has read set p
        self.graphs = []
        if use_graph:
            for p in range(2 if self.kv_overlap else 1):
                g = torch.cuda.CUDAGraph()
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    with torch.cuda.graph(g, stream=side):
                        self.stages_1_2(p)
                torch.cuda.current_stream().wait_stream(side)
                self.graphs.append(g)

    def step(self, kv_events=None):
        torch = self.torch
        p = self.step_no % 2 if self.kv_overlap else 0
        main = torch.cuda.current_stream()
        if self.kv_overlap and self.step_no >= 2:
            main.wait_event(self.consumed[p])                       # the KV pass of two steps ago has finished with set p
        if self.graphs:
            self.graphs[p].replay()
        else:
            self.stages_1_2(p)

        def kv():
            if kv_events is not None:
                self.B.lib().metok_trace_kernel(TRACE["move_rows"], kv_events[0], kv_events[1])
            self.stage3(p)
            if kv_events is not None:
                self.B.lib().metok_trace_kernel(0, None, None)

        if self.kv_overlap:
            self.filled[p].record(main)
            with torch.cuda.stream(self.kv_stream):
                self.kv_stream.wait_event(self.filled[p])
                kv()
                self.consumed[p].record(self.kv_stream)
        else:
            kv()
        self.step_no += 1


def stats_us(ms_list):
    a = np.asarray(ms_list, dtype=np.float64) * 1e3
    return dict(us_min=round(float(a.min()), 2), us_median=round(float(np.median(a)), 2), launches=int(a.size))


def hbm_entry(ms_list, nbytes, kernel):
    e = dict(kernel=kernel, **stats_us(ms_list), algorithmic_bytes=int(nbytes))
    e["GBs"] = round(nbytes / (e["us_median"] * 1e-6) / 1e9, 1)
    e["frac_of_hbm_peak"] = round(e["GBs"] / HBM_PEAK_GBS, 4)
    return e


def time_kernels(w: Workload, hev: HipEvents, reps: int):
    """Per kernel family, in this run: the library brackets the named kernel with our events (metok_trace_kernel), so the
    one-workgroup planning kernels of a call are not charged to the streaming kernels."""
    torch, lib = w.torch, w.B.lib()
    a, b_ev = hev.create(), hev.create()

    def traced(kernel, call):
        lib.metok_trace_kernel(TRACE[kernel], a, b_ev)
        try:
            res = call()
        finally:
            lib.metok_trace_kernel(0, None, None)
        return hev.elapsed_ms(a, b_ev), res

    out = {}
    videos = list(range(w.batch))
    # in the batched mode one launch covers the whole batch: bytes and flops per launch scale with it
    batched = w.mode == "batched"
    nb = w.batch if batched else 1
    units = [None] * w.batch if batched else videos
    # stage 1, one pass (uniform stride 2)
    s1 = (lambda v: w.stage1_batched()) if batched else w.stage1
    ms = [traced("frame_stats_pool2", lambda v=v: s1(v))[0] for _ in range(reps) for v in units]
    e = hbm_entry(ms, nb * w.stage1_fused_bytes(), "frame_stats_pool2_kernel")
    e["videos_per_launch"] = nb
    e["workload"] = "[256, 576, 1024] bf16 per video, every frame pooled 2 x 2: statistics and pooled tokens from one read"
    out["stage1_one_pass"] = e
    # stage 1, the paper's adaptive strides: statistics pass, then pooling pass
    ms_stats, ms_pool, rows = [], [], []
    for _ in range(reps):
        for v in videos:
            t, _ = traced("frame_stats", lambda v=v: w.stage1_adaptive(v))
            ms_stats.append(t)
            t, res = traced("pool", lambda v=v: w.stage1_adaptive(v))
            ms_pool.append(t)
            if len(rows) < len(videos):
                rows.append(int(res["frame_offsets"][-1]))
    v_bytes = FRAMES * GRID * GRID * D_VIS * 2
    out["stage1_adaptive_statistics"] = hbm_entry(ms_stats, v_bytes, "frame_stats_kernel")
    pool_bytes = v_bytes + int(np.mean(rows)) * D_VIS * 2
    e = hbm_entry(ms_pool, pool_bytes, "pool_kernel")
    e["pooled_rows_per_video_mean"] = float(np.mean(rows))
    e["workload"] = "[256, 576, 1024] bf16, (s1, s2) = (2, 3), alpha = 0.5, beta = 0.45: strides 2 / 3 / 4 / 6 per frame"
    out["stage1_adaptive_pooling"] = e
    if batched:
        # the same two kernels with the whole batch per launch (metok_segment_compress_batched), outputs of their own
        ad = ADAPTIVE
        call = lambda o=None: w.B.metok_segment_compress_batched(w.feats_b, GRID, GRID, N_EVENTS, w.text_b, ad["alpha"], ad["beta"],
                                                                 ad["s1"], ad["s2"], workspace=w.ws1_b, out=o)
        bufs = call()
        ms_stats = [traced("frame_stats", lambda: call(bufs))[0] for _ in range(reps * 4)]
        ms_pool = [traced("pool", lambda: call(bufs))[0] for _ in range(reps * 4)]
        rows_b = int(bufs["frame_offsets"][:, -1].sum())
        e = hbm_entry(ms_stats, nb * v_bytes, "frame_stats_kernel")
        e["videos_per_launch"] = nb
        out["stage1_adaptive_statistics_batched"] = e
        e = hbm_entry(ms_pool, nb * v_bytes + rows_b * D_VIS * 2, "pool_kernel")
        e["videos_per_launch"] = nb
        out["stage1_adaptive_pooling_batched"] = e
        del bufs
    # stage 2 per level
    toks = [w.s1_out[v]["token_event"] for v in videos]
    for lv in range(len(w.n_in)):
        if batched:
            tev_b = w.s1_out_b["token_event"] if lv == 0 else w.prune_out_b_sets[0][lv - 1]["token_event_out"]
            level = lambda v, lv=lv, tev_b=tev_b: w.prune_level_batched(lv, tev_b, 0)
        else:
            tev = [toks[v] if lv == 0 else w.prune_out[v][lv - 1]["token_event_out"] for v in videos]
            level = lambda v, lv=lv, tev=tev: w.prune_level(v, lv, tev[v])
        entry = dict(visual_tokens_in=w.n_in[lv], kept=w.counts[lv], videos_per_launch=nb)
        for kernel in ("row_stats", "col_sums"):
            ms = [traced(kernel, lambda v=v: level(v))[0] for _ in range(reps) for v in units]
            k = dict(kernel=kernel + "_kernel", **stats_us(ms), flops=nb * w.score_flops(lv))
            k["TFLOPs"] = round(k["flops"] / (k["us_median"] * 1e-6) / 1e12, 1)
            k["frac_of_bf16_mfma_peak"] = round(k["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS, 4)
            # the keys of the level are streamed once per pass: pass 1 reads all S keys, pass 2 the visual ones
            key_rows = w.n_in[lv] + (N_TEXT if kernel == "row_stats" else 0)
            k["key_stream_bytes"] = nb * HKV * key_rows * DH * 2
            k["key_stream_GBs"] = round(k["key_stream_bytes"] / (k["us_median"] * 1e-6) / 1e9, 1)
            entry[kernel] = k
        for kernel in ("select", "write_index"):
            ms = [traced(kernel, lambda v=v: level(v))[0] for _ in range(reps) for v in units]
            entry[kernel] = dict(kernel=("score_hist_kernel + candidate_kernel" if kernel == "select" else kernel + "_kernel"), **stats_us(ms))
        ms = [traced("gather_rows", lambda v=v: level(v))[0] for _ in range(reps) for v in units]
        entry["gather_rows"] = hbm_entry(ms, nb * w.gather_bytes(lv), "gather_rows_kernel")
        out[f"stage2_level{lv + 1}"] = entry
    torch.cuda.synchronize()
    return out


def time_stages(w: Workload, reps: int):
    """Whole stages back to back on one stream (every kernel of the stage, also the one-workgroup ones): ms per step
    and the tokens entering the stage per second."""
    torch = w.torch
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(reps)]
    for r in range(reps):
        ev[r][0].record()
        if w.mode == "batched":
            tok_b = w.stage1_batched()["token_event"]
            ev[r][1].record()
            w.stage2_batched(tok_b, 0)
        else:
            toks = [w.stage1(b)["token_event"] for b in range(w.batch)]
            ev[r][1].record()
            for b in range(w.batch):
                w.stage2(b, toks[b])
        ev[r][2].record()
        w.stage3()
        ev[r][3].record()
    torch.cuda.synchronize()
    ms = [float(np.median([ev[r][i].elapsed_time(ev[r][i + 1]) for r in range(reps)])) for i in range(3)]
    tokens = [w.batch * FRAMES * GRID * GRID, w.batch * N_VIS, w.batch * N_VIS]
    return {f"stage{i + 1}": dict(ms_per_step_alone=round(ms[i], 4), tokens_in_per_step=tokens[i],
                                 tokens_in_per_s=round(tokens[i] / (ms[i] * 1e-3), 1)) for i in range(3)}


def time_configs(w: Workload, reps: int):
    """The named configurations on their own (call-level GPU time, every kernel of the call included)."""
    torch, B = w.torch, w.B
    out = {}

    def timed(call, n_calls=reps):
        call()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_calls)]
        for a, b in evs:
            a.record()
            call()
            b.record()
        torch.cuda.synchronize()
        t = [a.elapsed_time(b) for a, b in evs]
        return dict(ms_min=round(float(np.min(t)), 4), ms_median=round(float(np.median(t)), 4))

    # encoder configuration: 32 frames x 576 x 1024 (37.7 MB: resident in the last-level cache after the first pass)
    f32 = w.feats[0][:32].contiguous()
    e = timed(lambda: B.metok_segment_compress(f32, GRID, GRID, 8, w.text[0], 1.0, 1.0, 2, 2))
    e["tokens_in_per_s"] = round(32 * GRID * GRID / (e["ms_median"] * 1e-3), 1)
    out["encoder_32_frames_uniform"] = e
    a = ADAPTIVE
    e = timed(lambda: B.metok_segment_compress(f32, GRID, GRID, 8, w.text[0], a["alpha"], a["beta"], a["s1"], a["s2"]))
    e["tokens_in_per_s"] = round(32 * GRID * GRID / (e["ms_median"] * 1e-3), 1)
    out["encoder_32_frames_adaptive"] = e
    # prefill configuration: 128 x 144 visual + 64 text rows, one level, keep 25 %
    nv, nt = 128 * TOK_PER_FRAME, 64
    hid = w.hidden0[0][: nv + nt]
    k = w.K[0][0][:, : nv + nt].contiguous()
    tev = w.s1_out[0]["token_event"][:nv]
    seg = w.seg0[:nv]
    e = timed(lambda: B.metok_prefill_prune(hid, 0, nv, seg, [nv // 4], q_text=w.Q[0][0], k_all=k, token_event=tev,
                                            event_weight=w.weight[0]))
    e["tokens_in_per_s"] = round(nv / (e["ms_median"] * 1e-3), 1)
    out["prefill_18432_keep_quarter"] = e
    # hierarchical configuration: the three levels of one video
    e = timed(lambda: w.stage2(0, w.s1_out[0]["token_event"]))
    e["tokens_in_per_s"] = round(N_VIS / (e["ms_median"] * 1e-3), 1)
    out["hierarchical_36864_three_levels"] = e
    e = timed(lambda: w.stage2_batched(w.s1_out_b["token_event"], 0))
    e["tokens_in_per_s"] = round(w.batch * N_VIS / (e["ms_median"] * 1e-3), 1)
    out["hierarchical_36864_three_levels_batch8_one_call_per_level"] = e
    # decoding configuration: the batch's KV cache
    e = timed(w.stage3)
    e["tokens_in_per_s"] = round(w.batch * N_VIS / (e["ms_median"] * 1e-3), 1)
    e["GBs"] = round(w.kv_bytes() / (e["ms_median"] * 1e-3) / 1e9, 1)
    out["kv_28_layers_batch8"] = e
    # the paper's own stage-3 rule on the same cache: every visual row leaves from layer l1 on, only the 128 text rows move
    # (a latency case: 25 layers x 8 videos x 4 heads x (K, V) x 128 rows of 256 bytes = 52 MB each way)
    text_only = torch.arange(N_VIS, N_VIS + N_TEXT, dtype=torch.int32, device=w.dev).repeat(w.batch, 1)
    paper_idx = [None if l < L_H[0] else text_only for l in range(N_LAYERS)]
    paper_len = torch.empty_like(w.new_len)
    e = timed(lambda: B.metok_kv_compact(w.k_layers, w.v_layers, paper_idx, new_len=paper_len, workspace=w.kv_ws))
    out["kv_28_layers_batch8_paper_rule_text_rows_only_from_l1"] = e
    # the paper's LongVA setting of stage 1 (strides 2 / 3 / 4 / 6 per frame: two passes over the features) for the whole batch;
    # overwrites the stage-1 outputs, so it comes after the configurations that read them
    e = timed(lambda: B.metok_segment_compress_batched(w.feats_b, GRID, GRID, N_EVENTS, w.text_b, a["alpha"], a["beta"], a["s1"], a["s2"],
                                                       workspace=w.ws1_b, out=w.s1_out_b))
    e["tokens_in_per_s"] = round(w.batch * FRAMES * GRID * GRID / (e["ms_median"] * 1e-3), 1)
    e["GBs"] = round(w.batch * (2 * FRAMES * GRID * GRID * D_VIS * 2 + int(w.s1_out_b["frame_offsets"][:, -1].float().mean()) * D_VIS * 2)
                     / (e["ms_median"] * 1e-3) / 1e9, 1)
    out["encoder_256_frames_adaptive_batch8"] = e
    e = timed(lambda: B.metok_segment_compress(w.feats[0], GRID, GRID, N_EVENTS, w.text[0], a["alpha"], a["beta"], a["s1"], a["s2"],
                                               workspace=w.ws1[0], out=w.s1_out[0]))
    e["tokens_in_per_s"] = round(FRAMES * GRID * GRID / (e["ms_median"] * 1e-3), 1)
    out["encoder_256_frames_adaptive_one_video"] = e
    # the same cache as page pools (pages of 16 rows; the dense cache's memory reinterpreted, contents do not matter for the
    # timing): rows moved through the page table against tables rewritten.  Runs last: it scrambles the cache.
    ps = 16
    S0 = N_VIS + N_TEXT
    pages_per_seq, n_pages = S0 // ps, w.batch * (S0 // ps)
    kp = [k.view(n_pages, HKV, ps, DH) for k in w.k_layers]
    vp = [v.view(n_pages, HKV, ps, DH) for v in w.v_layers]
    table = torch.randperm(n_pages, device=w.dev).to(torch.int32).view(w.batch, pages_per_seq)
    level_of = [sum(1 for b in L_H if l >= b) for l in range(N_LAYERS)]
    text_rows = torch.arange(N_VIS, S0, dtype=torch.int32, device=w.dev).repeat(w.batch, 1)
    keep_pages = torch.sort(torch.randperm(N_VIS // ps, device=w.dev)[: N_VIS // ps // 2]).values.to(torch.int32)
    block_rows = (keep_pages[:, None] * ps + torch.arange(ps, dtype=torch.int32, device=w.dev)[None, :]).reshape(-1)
    block_idx = torch.cat([block_rows, text_rows[0]]).repeat(w.batch, 1).contiguous()
    cases = {"paper_rule_text_rows_only_from_l1": [None if lv == 0 else text_rows for lv in level_of],
             "whole_pages_dropped_half_of_the_visual_pages": [None if lv == 0 else block_idx for lv in level_of],
             "stage2_retained_sets": w.idx_layers}
    for name, idx in cases.items():
        res = B.metok_kv_relink_paged(kp, vp, table, idx)
        e = timed(lambda: B.metok_kv_relink_paged(kp, vp, table, idx, workspace=res["workspace"]))
        e["rows_copied_per_layer_and_video_max"] = int(res["rows_copied"].max())
        e["pages_released"] = int(res["n_free"].sum())
        out["kv_paged_relink_" + name] = e
    e = timed(lambda: B.metok_kv_compact_paged(kp, vp, table, w.idx_layers))
    e["GBs"] = round(w.kv_bytes() / (e["ms_median"] * 1e-3) / 1e9, 1)
    out["kv_paged_move_rows_stage2_retained_sets"] = e
    return out


# -------------------------------------------------------------------------------------------------
# CPU oracle legs (run before the GPU is initialised; the oracle is used as it stands)
# -------------------------------------------------------------------------------------------------
def oracle_video(vid: int):
    """One whole video through the oracle: stage 1 on 256 frames, the three pruning levels with fresh activations, the KV
    compaction of its 25 moving layers x 4 heads x (K, V).  Returns the seconds spent inside oracle calls per stage
    (the seeded generators that make the inputs are not timed)."""
    from oracle import metok_oracle as O
    from paper_2506_02850_amd import synth

    counts = level_counts()
    t_stage = [0.0, 0.0, 0.0]
    v = synth.planted_video(100 + vid, FRAMES, (GRID, GRID), D_VIS, N_EVENTS, 4, 40, 0.2, "bf16")
    t0 = time.perf_counter()
    S = O.adjacent_frame_cosine(v.feats)
    es, _ = O.event_boundaries(S, N_EVENTS)
    cmp = O.compress_encoder_tokens(v.feats, (GRID, GRID), v.text_emb, es, 1.0, 1.0, 2, 2)
    t_stage[0] += time.perf_counter() - t0
    ev = cmp["token_event"]
    del v, cmp
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
    return t_stage


def _oracle_worker(vid: int):
    from threadpoolctl import threadpool_limits

    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        stages = oracle_video(vid)
        return stages, time.perf_counter() - t0


def cpu_baseline(n_videos: int):
    """The oracle, unchanged, single-threaded, on whole videos of the same workload."""
    from threadpoolctl import threadpool_limits

    t_stage = [0.0, 0.0, 0.0]
    with threadpool_limits(limits=1):
        for vid in range(n_videos):
            for i, t in enumerate(oracle_video(vid)):
                t_stage[i] += t
    total = sum(t_stage)
    return dict(value=n_videos * FRAMES * GRID * GRID / total, unit="tokens/s", cores=1, kind="oracle",
                sample=f"{n_videos} whole videos (one step has 8; every video has its own seed): stage 1 on 256 frames, three pruning levels, KV compaction of "
                       "25 layers x 4 heads x (K, V); oracle calls only, one thread",
                seconds_by_stage=[round(t, 3) for t in t_stage], seconds=round(total, 3))


def cpu_baseline_all_cores(n_videos: int):
    """The same oracle on several host cores: one video per worker process (each single-threaded), at most 16 workers.
    The rate is videos finished per second of the workers' oracle calls running side by side."""
    import multiprocessing as mp

    nproc = os.cpu_count() or 1
    workers = max(1, min(n_videos, nproc, 16))
    ctx = mp.get_context("spawn")
    t0 = time.perf_counter()
    with ctx.Pool(workers) as pool:
        res = pool.map(_oracle_worker, range(n_videos), chunksize=1)
    wall = time.perf_counter() - t0
    oracle_s = [sum(stages) for stages, _ in res]
    # workers run concurrently: the oracle part of the wall clock is the longest chain of oracle calls on one worker
    rounds = (n_videos + workers - 1) // workers
    busy = max(oracle_s) * rounds
    return dict(value=n_videos * FRAMES * GRID * GRID / busy, unit="tokens/s", cores=workers, nproc=nproc, kind="oracle",
                sample=f"{n_videos} whole videos, one per worker process, {workers} processes side by side (host reports {nproc} "
                       "cores); per video as in cpu_baseline; rate = tokens / (slowest worker's oracle seconds x rounds)",
                oracle_seconds_per_video=[round(t, 3) for t in oracle_s], wall_seconds_with_input_generation=round(wall, 3))


def read_traffic():
    """HBM bytes per KV-compaction launch from the committed rocprofv3 counter summary, if present (a file-sourced
    figure: it is not measured in this run)."""
    path = os.path.join(ROOT, "profiles", "move_rows_longva256_b8_pmc.txt")
    try:
        with open(path) as fh:
            for line in fh:
                if line.startswith("traffic_bytes_per_launch"):
                    return float(line.split()[1]), (os.path.relpath(path, ROOT) + ": rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of `bench.py --only kv`, "
                                                    "scaled by the same counters on a plain copy; a separate run, not measured in this one")
    except OSError:
        pass
    return None, None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--streams", type=int, default=8, help="streams that share the per-video stage-1/2 work")
    ap.add_argument("--no-graph", action="store_true", help="launch the stage-1/2 kernels one by one instead of replaying a HIP graph")
    ap.add_argument("--per-video", action="store_true", help="one library call per video and stage on 8 streams instead of the batched calls")
    ap.add_argument("--split", type=int, default=1, help="run stages 1-2 on this many shares of the batch, each on its own stream")
    ap.add_argument("--kv-overlap", action="store_true",
                    help="run the KV compaction of a step on a stream of its own, beside the next step's stages 1-2 (higher whole-job rate, "
                         "but the two HBM-bound parts then share the memory system and the KV kernel's own duration grows by half)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-videos", type=int, default=12, help="videos of the single-thread oracle leg (the all-cores leg takes 8)")
    ap.add_argument("--kernel-reps", type=int, default=3, help="repetitions (x 8 videos) of the per-kernel measurements")
    ap.add_argument("--only", choices=["all", "kv", "copy", "prune", "stage1", "stage1_adaptive"], default="all",
                    help="run only one part (for profiler runs): the KV compaction, the calibration copy, the stage-2 calls, "
                         "the one-pass stage 1 or the two-pass adaptive stage 1")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    # the CPU legs come first: worker processes are started before this process touches the GPU
    cpu = {}
    if args.only == "all" and not args.no_cpu_baseline:
        cpu["cpu_baseline"] = cpu_baseline(args.cpu_videos)
        cpu["cpu_baseline_all_cores"] = cpu_baseline_all_cores(8)

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
        if args.per_video:
            toks = [w.stage1(b)["token_event"] for b in range(args.batch)]
            for _ in range(args.warmup + args.steps):
                for b in range(args.batch):
                    w.stage2(b, toks[b])
        else:
            tok_b = w.stage1_batched()["token_event"]
            for _ in range(args.warmup + args.steps):
                w.stage2_batched(tok_b, 0)
        torch.cuda.synchronize()
        print(json.dumps({"score_flops_per_step": sum(2 * w.score_flops(lv) for lv in range(3)) * args.batch}))
        return
    if args.only in ("stage1", "stage1_adaptive"):
        call = w.stage1 if args.only == "stage1" else w.stage1_adaptive
        for _ in range(args.warmup + args.steps):
            if args.only == "stage1" and not args.per_video:
                w.stage1_batched()
                continue
            for b in range(args.batch):
                call(b)
        torch.cuda.synchronize()
        print(json.dumps({"stage1_feature_bytes_per_video": FRAMES * GRID * GRID * D_VIS * 2}))
        return

    hev = HipEvents()
    w.mode = "per-video" if args.per_video else "batched"
    w.step()                                             # eager once: loads code objects before any capture
    torch.cuda.synchronize()
    w.configure(w.mode, kv_overlap=args.kv_overlap, use_graph=not args.no_graph, split=args.split)
    for _ in range(args.warmup):
        w.step()
    torch.cuda.synchronize()
    kv_ev = [(hev.create(), hev.create()) for _ in range(args.steps)]
    step_ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    step_ev[0].record()
    for s in range(args.steps):
        w.step(kv_ev[s])
        step_ev[s + 1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    kv_all = [hev.elapsed_ms(a, b) for a, b in kv_ev]
    kv_ms = float(np.mean(kv_all))
    # step boundaries on the main stream; with the KV compaction on its own stream a step's KV pass ends inside the next step
    step_ms = [step_ev[s].elapsed_time(step_ev[s + 1]) for s in range(args.steps)]
    err_word = int(w.kv_ws[:4].view(torch.int32)[0])
    if err_word != 0:
        sys.exit("the KV compaction reported an expired wait: results are invalid")
    tokens_per_step = args.batch * FRAMES * GRID * GRID
    ms_per_step = elapsed * 1e3 / args.steps
    achieved = w.kv_bytes() / (kv_ms * 1e-3) / 1e9
    traffic, traffic_file = read_traffic()
    stages = time_stages(w, 5)
    stages["stage3"]["GBs"] = round(w.kv_bytes() / (stages["stage3"]["ms_per_step_alone"] * 1e-3) / 1e9, 1)
    stages.update(time_kernels(w, hev, args.kernel_reps))
    stages["stage3_kv_compaction"] = hbm_entry(kv_all, w.kv_bytes(), "move_rows_kernel")
    # every streaming kernel's fraction of the HBM peak and every score pass's fraction of the bf16 MFMA peak, side by side
    fractions = {"hbm": {}, "mfma_bf16": {}}
    for name, e in stages.items():
        if isinstance(e, dict) and "frac_of_hbm_peak" in e:
            fractions["hbm"][e.get("kernel", name) + " (" + name + ")"] = e["frac_of_hbm_peak"]
        for sub, k in (e.items() if isinstance(e, dict) else ()):
            if isinstance(k, dict) and "frac_of_hbm_peak" in k:
                fractions["hbm"][k["kernel"] + " (" + name + ")"] = k["frac_of_hbm_peak"]
            if isinstance(k, dict) and "frac_of_bf16_mfma_peak" in k:
                fractions["mfma_bf16"][k["kernel"] + " (" + name + ")"] = k["frac_of_bf16_mfma_peak"]
    out = {
        "metric": "visual tokens processed/sec through stages 1-3",
        "value": tokens_per_step / (elapsed / args.steps),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_min": round(float(np.min(step_ms)), 4), "ms_per_step_median": round(float(np.median(step_ms)), 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "LongVA-7B-shaped, 256 frames: hierarchical prefill + decoding KV compaction configs "
                               "chained behind stage 1 at 256 x 576 x 1024",
                   "batch_videos": args.batch, "frames": FRAMES, "tokens_per_frame_in": GRID * GRID,
                   "tokens_per_frame_pooled": TOK_PER_FRAME, "prune_levels": level_counts(), "text_tokens": N_TEXT,
                   "text_queries": TQ, "kv_layers": N_LAYERS, "L_H": list(L_H), "streams": w.n_streams,
                   "stage2_inputs": "keys 0.5 mu_event + N(0,1), queries N(0,1) + 0.5 mu_target, hidden N(0,1) + event shift",
                   "calls": "one call per stage and level for the whole batch" if w.mode == "batched" else "one call per video, stage and level",
                   "launch": ("eager" if not w.graphs else "stages 1-2 replayed from a HIP graph, KV compaction launched directly")
                             + ("; the KV compaction of a step runs on its own stream beside the next step's stages 1-2 (two sets of index lists)"
                                if w.kv_overlap else "; one stream")},
        "value_in_pooled_tokens_per_s": args.batch * N_VIS / (elapsed / args.steps),
        "roofline": {"kernel": "move_rows_kernel", "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_file,
                     "algorithmic_bytes_per_launch": w.kv_bytes(), "ms_per_launch": kv_ms,
                     "ms_per_launch_min": round(float(np.min(kv_all)), 4), "ms_per_launch_median": round(float(np.median(kv_all)), 4)},
        "kernel_fractions_of_peak": fractions,
        "stages": stages,
        "configs": time_configs(w, 10),
    }
    out.update(cpu)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
