"""Seeded random sweeps on the GPU: many small cases with random sizes, class counts, quotas, tie structure,
index lists and page tables, each compared bit for bit with the oracle.  They complement the hand-picked cases
of the per-stage files."""
import numpy as np
import pytest
import torch

from oracle import metok_oracle as O
from tests.test_gpu_stage3 import as_device, as_host, fill_cache, mk

pytestmark = pytest.mark.gpu


def test_selection_and_compaction_random_cases():
    B = mk()
    rng = np.random.default_rng(123)
    for it in range(80):
        n = int(rng.integers(1, 7000))
        n_seg = int(rng.integers(1, 6))
        seg = rng.integers(0, n_seg, size=n).astype(np.int32)
        kind = it % 4
        if kind == 0:
            scores = rng.standard_normal(n)
        elif kind == 1:
            scores = np.round(rng.standard_normal(n), int(rng.integers(0, 3)))          # many exact ties
        elif kind == 2:
            scores = rng.choice([0.0, 1.0, -1.0, 0.5], size=n)                          # four values only
        else:
            scores = np.abs(rng.standard_normal(n)) * 1e-4                              # attention-like magnitudes
        scores = scores.astype(np.float32)
        quotas = [int(rng.integers(0, int((seg == s).sum()) + 1)) for s in range(n_seg)]
        vis_start, n_text, D = int(rng.integers(0, 3)), int(rng.integers(1, 4)), 8
        hidden = rng.standard_normal((vis_start + n + n_text, D)).astype(np.float32)
        out = B.metok_prefill_prune(torch.from_numpy(hidden).cuda(), vis_start, n, torch.from_numpy(seg).cuda(), quotas,
                                    scores=torch.from_numpy(scores).cuda())
        torch.cuda.synchronize()
        want = O.segmented_topk(scores, seg, quotas)
        np.testing.assert_array_equal(out["kept_idx"].cpu().numpy(), want, err_msg=f"case {it}: n={n} quotas={quotas}")
        np.testing.assert_array_equal(out["hidden_out"].cpu().numpy(), O.compact_hidden(hidden, vis_start, n, want))
        np.testing.assert_array_equal(out["token_seg_out"].cpu().numpy(), seg[want])


def random_index_list(rng, S, B):
    """Ascending positions with random structure: identity prefix, dense runs, sparse stretches."""
    rows = []
    n_keep = int(rng.integers(0, S + 1))
    for _ in range(B):
        style = int(rng.integers(0, 3))
        if style == 0:
            ix = np.sort(rng.choice(S, n_keep, replace=False))
        elif style == 1:                                   # identity prefix, then a random tail
            head = int(rng.integers(0, n_keep + 1))
            tail = np.sort(rng.choice(np.arange(head, S), n_keep - head, replace=False)) if n_keep > head else np.zeros(0, dtype=np.int64)
            ix = np.concatenate([np.arange(head), tail])
        else:                                              # the last n_keep rows (everything moves as one block)
            ix = np.arange(S - n_keep, S)
        rows.append(ix)
    return np.stack(rows).astype(np.int32)


def test_kv_compaction_random_cases_dense_and_paged():
    Bm = mk()
    rng = np.random.default_rng(321)
    for it in range(12):
        L, B, H = int(rng.integers(1, 4)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
        page_size = int(rng.choice([1, 4, 16, 19]))
        pages = int(rng.integers(1, 40))
        S = pages * page_size
        dh16 = int(rng.choice([8, 64, 128, 264]))
        dtype = "bf16" if it % 3 else "f32"
        if dtype == "f32" and dh16 % 16:
            dh16 = 64
        lists = [None if rng.random() < 0.25 else random_index_list(rng, S, B) for _ in range(L)]
        ks, vs = fill_cache(L, B, H, S, dh16, dtype)
        # dense
        kd, vd = [as_device(k, dtype) for k in ks], [as_device(v, dtype) for v in vs]
        idx_dev = [None if ix is None else torch.from_numpy(ix).cuda() for ix in lists]
        Bm.metok_kv_compact(kd, vd, idx_dev)
        # paged, through a random table
        n_pages = B * pages + 3
        table = rng.permutation(n_pages)[:B * pages].reshape(B, pages).astype(np.int32)

        def pooled(dense):
            pool = np.zeros((n_pages, H, page_size, dh16), dtype=np.int16)
            for b in range(B):
                for p, page in enumerate(table[b]):
                    pool[page] = dense[b, :, p * page_size:(p + 1) * page_size]
            return pool

        kp, vp = [as_device(pooled(k), dtype) for k in ks], [as_device(pooled(v), dtype) for v in vs]
        Bm.metok_kv_compact_paged(kp, vp, torch.from_numpy(table).cuda(), idx_dev)
        torch.cuda.synchronize()
        for l in range(L):
            for dense, dev, pdev in ((ks[l], kd[l], kp[l]), (vs[l], vd[l], vp[l])):
                got = as_host(dev).reshape(B, H, S, dh16)
                pool = as_host(pdev).reshape(n_pages, H, page_size, dh16)
                for b in range(B):
                    logical = np.concatenate([pool[page] for page in table[b]], axis=1)
                    for h in range(H):
                        ref = O.kv_compact(dense[b, h], None if lists[l] is None else lists[l][b])
                        assert np.array_equal(got[b, h, :ref.shape[0]], ref), f"case {it} dense layer {l}"
                        assert np.array_equal(logical[h, :ref.shape[0]], ref), f"case {it} paged layer {l}"


def test_stage1_random_cases_one_call_and_two_calls():
    from paper_2506_02850_amd import synth
    from tests.test_gpu_stage1_one_call import check

    rng = np.random.default_rng(77)
    for it in range(24):
        T = int(rng.integers(2, 30))
        grid = (int(rng.integers(1, 9)) * (2 if it % 2 == 0 else 1), int(rng.integers(1, 9)) * (2 if it % 2 == 0 else 1))
        dtype = "bf16" if it % 3 else "f32"
        d = 8 * int(rng.integers(1, 40))                          # bf16 output rows need a multiple of 8
        k = int(rng.integers(1, min(T, 6) + 1))
        if it % 2 == 0:
            alpha, s1, s2 = 1.0, 2, 2                              # uniform stride 2 on an even grid: the one-pass kernel
        else:
            alpha, s1, s2 = float(rng.choice([0.3, 0.5, 1.0])), int(rng.integers(1, 4)), int(rng.integers(1, 4))
        beta = float(rng.choice([0.4, 0.5, 1.0]))
        edge = int(rng.integers(0, 2))
        reduce_ = int(rng.integers(0, 2))
        v = synth.planted_video(5000 + it, T, grid, d, k, 1, T, 0.12, dtype)
        for out_dtype in ("f32", "bf16"):
            check(v, grid, k, alpha, beta, s1, s2, out_dtype, edge=edge, reduce_=reduce_)


def test_stage2_scores_random_cases():
    from paper_2506_02850_amd import synth
    from tests.test_gpu_stage2 import check_prune, run_prune

    rng = np.random.default_rng(99)
    for it in range(20):
        dtype = "bf16" if it % 4 else "f32"
        dh = int(rng.choice([32, 64, 128, 256] if dtype == "bf16" else [32, 64, 128]))
        Hkv = int(rng.integers(1, 5))
        Hq = Hkv * int(rng.integers(1, 8))
        n_text = int(rng.integers(1, 70))
        Tq = int(rng.integers(1, n_text + 1))
        vis_start = int(rng.integers(0, 40))
        n_events = int(rng.integers(1, 6))
        n_vis = int(rng.integers(1, 1500))
        token_event = np.sort(rng.integers(0, n_events, size=n_vis)).astype(np.int32)
        layer = synth.prefill_layer(7000 + it, token_event, n_events, n_text, 16, Hq, Hkv, dh, dtype, vis_start=vis_start)
        seg = rng.integers(0, 2, size=n_vis).astype(np.int32)
        quotas = [int(rng.integers(0, int((seg == s).sum()) + 1)) for s in range(2)]
        mode = int(rng.integers(0, 2))
        got, q = run_prune(layer, seg, quotas, use_weight=bool(it % 2), Tq=Tq, score_mode=mode)
        check_prune(layer, seg, quotas, got, q, use_weight=bool(it % 2), score_mode=mode)
