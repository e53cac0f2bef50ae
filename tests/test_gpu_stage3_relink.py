"""GPU parity of metok_kv_relink_paged against the CPU oracle.  A dense cache filled with the per-row-unique pattern is
scattered into page pools through a random page table; after the call
  * the new page tables, the released pages and the count of copied rows equal the oracle's index transformation;
  * every logical row read back through the NEW table equals the oracle's row copy of the dense cache, bit for bit;
  * relinked pages and pages that belong to no sequence hold exactly the bytes they held before."""
import numpy as np
import pytest
import torch

from oracle import metok_oracle as O
from tests.test_gpu_stage3 import as_device, as_host, fill_cache, mk
from tests.test_gpu_stage3_paged import nested_lists, to_pages

pytestmark = pytest.mark.gpu


def run_relink(L, B, H, pages_per_seq, page_size, dh16, dtype, idx_lists, seed=0, spare_pages=5, len_in=None):
    Bm = mk()
    S = pages_per_seq * page_size
    rng = np.random.default_rng(seed)
    n_pages = B * pages_per_seq + spare_pages
    table = rng.permutation(n_pages)[:B * pages_per_seq].reshape(B, pages_per_seq).astype(np.int32)
    ks, vs = fill_cache(L, B, H, S, dh16, dtype)
    kp = [to_pages(k, table, n_pages, page_size) for k in ks]
    vp = [to_pages(v, table, n_pages, page_size) for v in vs]
    kd = [as_device(k, dtype) for k in kp]
    vd = [as_device(v, dtype) for v in vp]
    idx_dev = [None if ix is None else torch.from_numpy(np.ascontiguousarray(ix, dtype=np.int32)).cuda() for ix in idx_lists]
    out = Bm.metok_kv_relink_paged(kd, vd, torch.from_numpy(table).cuda(), idx_dev, len_in=len_in)
    torch.cuda.synchronize()
    assert int(out["workspace"][:4].view(torch.int32)[0]) == 0, "a bounded wait inside the row mover expired"
    lens = [S] * L if len_in is None else list(len_in)
    np.testing.assert_array_equal(out["new_len"].cpu().numpy(), [lens[l] if ix is None else ix.shape[1] for l, ix in enumerate(idx_lists)])
    tout = out["page_table_out"].cpu().numpy()
    freed = out["free_pages"].cpu().numpy()
    n_free = out["n_free"].cpu().numpy()
    copied = out["rows_copied"].cpu().numpy()
    owned = set(table.reshape(-1).tolist())
    total_copied = 0
    for l in range(L):
        pools = [(ks[l], kp[l], as_host(kd[l]).reshape(n_pages, H, page_size, dh16), "K"),
                 (vs[l], vp[l], as_host(vd[l]).reshape(n_pages, H, page_size, dh16), "V")]
        for dense, before, pool, name in pools:
            for page in range(n_pages):
                if page not in owned:
                    assert np.array_equal(pool[page], before[page]), f"layer {l} {name}: spare page {page} was written"
        for b in range(B):
            if idx_lists[l] is None:
                np.testing.assert_array_equal(tout[l, b], table[b])
                assert n_free[l, b] == 0 and copied[l, b] == 0
                continue
            ix = idx_lists[l][b]
            ref = O.kv_relink_pages(ix, lens[l], page_size, table[b])
            n_new = len(ref["table_out"])
            np.testing.assert_array_equal(tout[l, b, :n_new], ref["table_out"], err_msg=f"layer {l} video {b}: new table")
            assert (tout[l, b, n_new:] == -1).all()
            assert n_free[l, b] == len(ref["free_pages"])
            np.testing.assert_array_equal(freed[l, b, :n_free[l, b]], ref["free_pages"], err_msg=f"layer {l} video {b}: released pages")
            assert copied[l, b] == ref["rows_copied"]
            total_copied += int(copied[l, b])
            if n_new == 0:                                   # a layer that keeps nothing: every page was released
                continue
            for dense, before, pool, name in pools:
                # relinked pages were not written at all
                for D, whole in enumerate(ref["relinked"]):
                    if whole:
                        assert np.array_equal(pool[tout[l, b, D]], before[tout[l, b, D]]), f"layer {l} {name} video {b}: relinked page {D} changed"
                logical = np.concatenate([pool[page] for page in tout[l, b, :n_new]], axis=1)          # [H, n_new * ps, dh]
                for h in range(H):
                    want = O.kv_compact(dense[b, h], ix)
                    assert np.array_equal(logical[h, :want.shape[0]], want), f"layer {l} {name} video {b} head {h}"
    return out, total_copied


@pytest.mark.parametrize("dtype,dh16,page_size", [("bf16", 128, 16), ("bf16", 64, 7), ("f32", 64, 32), ("bf16", 8, 1)])
def test_relink_matches_the_oracle_on_scattered_keeps(dtype, dh16, page_size):
    rng = np.random.default_rng(21)
    B, H, pages = 3, 2, 23
    S = pages * page_size
    n_text = min(9, S // 4)
    n_vis = S - n_text
    lists = nested_lists(rng, B, n_vis, n_text, [n_vis // 2, n_vis // 5, 0])
    run_relink(4, B, H, pages, page_size, dh16, dtype, [None] + lists, seed=3)


def test_paper_rule_moves_nothing_when_the_visual_span_ends_on_a_page():
    """Sec. 3.3: layers below l_1 untouched, the others keep the text rows only.  256 x 144 visual rows end on a page
    boundary for pages of 16, so the text pages are relinked: no row is copied and all 2304 visual pages are released."""
    B, H, ps = 2, 4, 16
    n_vis, n_text = 256 * 144, 128
    pages = (n_vis + n_text) // ps
    sched = O.kv_text_only_schedule(4, 2, n_vis, n_text)
    lists = [None if s is None else np.stack([s] * B).astype(np.int32) for s in sched]
    out, copied = run_relink(4, B, H, pages, ps, 128, "bf16", lists, seed=5)
    assert copied == 0
    np.testing.assert_array_equal(out["n_free"].cpu().numpy(), [[0, 0], [0, 0], [n_vis // ps] * 2, [n_vis // ps] * 2])


def test_unaligned_text_rows_and_block_aligned_drops():
    B, H, ps, pages = 2, 2, 16, 40
    S = pages * ps
    # (a) text rows that start inside a page: every one of them is copied, at most ceil(50 / 16) + 1 pages are written
    text = np.arange(S - 50, S, dtype=np.int32)
    # (b) whole pages dropped at random: every kept page is relinked, nothing is copied
    rng = np.random.default_rng(9)
    keep_pages = np.sort(rng.choice(pages, 17, replace=False))
    blocks = (keep_pages[:, None] * ps + np.arange(ps)[None, :]).reshape(-1).astype(np.int32)
    # (c) a kept head that stays in place, then scattered rows
    head = np.concatenate([np.arange(300), np.arange(310, S, 3)]).astype(np.int32)
    lists = [np.stack([text] * B), np.stack([blocks] * B), np.stack([head] * B)]
    out, _ = run_relink(3, B, H, pages, ps, 128, "bf16", lists, seed=6)
    copied = out["rows_copied"].cpu().numpy()
    assert (copied[0] == 50).all() and (copied[1] == 0).all()
    assert (out["n_free"].cpu().numpy()[1] == pages - 17).all()


def test_tiles_without_copies_among_tiles_with_copies_over_two_launches():
    """Only the tiles that copy rows get a workgroup.  45 layers (two launches of the row mover), pages of 24 rows
    that straddle the 512-row tiles, and per layer a different mix: a kept prefix, whole pages dropped at random
    (tiles with nothing to copy), scattered rows (tiles that copy), whole pages again behind them (their homes
    depend on the copies before them), untouched and empty layers in between."""
    rng = np.random.default_rng(77)
    L, B, H, ps, pages = 45, 2, 2, 24, 130
    S = pages * ps
    lists = []
    for l in range(L):
        if l % 11 == 5:
            lists.append(None)
            continue
        if l == 7:
            lists.append(np.zeros((B, 0), dtype=np.int32))
            continue
        per_video = []
        n_keep = None
        for b in range(B):
            prefix = int(rng.integers(0, 30))
            mid_end = int(rng.integers(60, 90))
            whole = np.sort(rng.choice(np.arange(prefix, mid_end), size=(mid_end - prefix) // 2, replace=False))
            tail_pages = np.sort(rng.choice(np.arange(mid_end + 20, pages), size=6, replace=False))
            rows = np.concatenate([np.arange(prefix * ps),
                                   (whole[:, None] * ps + np.arange(ps)[None, :]).reshape(-1),
                                   np.sort(rng.choice(np.arange(mid_end * ps, (mid_end + 20) * ps), size=200 + 24 * (l % 3), replace=False)),
                                   (tail_pages[:, None] * ps + np.arange(ps)[None, :]).reshape(-1)]).astype(np.int32)
            n_keep = len(rows) if n_keep is None else min(n_keep, len(rows))
            per_video.append(rows)
        lists.append(np.stack([r[:n_keep] for r in per_video]))
    out, copied = run_relink(L, B, H, pages, ps, 128, "bf16", lists, seed=8)
    assert copied > 0


def test_relinking_twice_with_per_layer_tables_and_shorter_layers():
    """The tables a first call wrote are the input of a second one (one table per layer, per-layer lengths)."""
    Bm = mk()
    rng = np.random.default_rng(31)
    L, B, H, ps, pages, dh = 2, 2, 2, 8, 30, 64
    S = pages * ps
    n_pages = B * pages + 4
    table = rng.permutation(n_pages)[:B * pages].reshape(B, pages).astype(np.int32)
    ks, vs = fill_cache(L, B, H, S, dh, "bf16")
    kd = [as_device(to_pages(k, table, n_pages, ps), "bf16") for k in ks]
    vd = [as_device(to_pages(v, table, n_pages, ps), "bf16") for v in vs]
    first = [np.stack([np.sort(rng.choice(S, n, replace=False)) for _ in range(B)]).astype(np.int32) for n in (150, 97)]
    out1 = Bm.metok_kv_relink_paged(kd, vd, torch.from_numpy(table).cuda(), [torch.from_numpy(x).cuda() for x in first])
    second = [np.stack([np.sort(rng.choice(first[l].shape[1], n, replace=False)) for _ in range(B)]).astype(np.int32)
              for l, n in enumerate((60, 97))]                      # layer 1 keeps everything the second time
    out2 = Bm.metok_kv_relink_paged(kd, vd, out1["page_table_out"], [torch.from_numpy(x).cuda() for x in second],
                                    len_in=[150, 97])
    torch.cuda.synchronize()
    assert int(out2["workspace"][:4].view(torch.int32)[0]) == 0
    t1 = out1["page_table_out"].cpu().numpy()
    t2 = out2["page_table_out"].cpu().numpy()
    for l in range(L):
        for dense, dev in ((ks[l], kd[l]), (vs[l], vd[l])):
            pool = as_host(dev).reshape(n_pages, H, ps, dh)
            for b in range(B):
                ref = O.kv_relink_pages(second[l][b], first[l].shape[1], ps, t1[l, b])
                np.testing.assert_array_equal(t2[l, b, :len(ref["table_out"])], ref["table_out"])
                assert int(out2["rows_copied"][l, b]) == ref["rows_copied"]
                rows = first[l][b][second[l][b]]                     # the two keeps composed, in rows of the first cache
                logical = np.concatenate([pool[p] for p in t2[l, b, :len(ref["table_out"])]], axis=1)
                for h in range(H):
                    assert np.array_equal(logical[h, :len(rows)], O.kv_compact(dense[b, h], rows))
    assert (out2["rows_copied"].cpu().numpy()[1] == 0).all()          # an identity keep relinks every page


def test_relink_longva_shaped_and_errors():
    rng = np.random.default_rng(12)
    B, H, ps = 1, 4, 16
    pages = (36864 + 128) // ps
    lists = nested_lists(rng, B, 36864, 128, [18432, 4608])
    run_relink(2, B, H, pages, ps, 128, "bf16", lists, seed=7, spare_pages=3)
    Bm = mk()
    pool = torch.zeros((8, 2, 4, 64), dtype=torch.bfloat16, device="cuda")
    table = torch.arange(8, dtype=torch.int32, device="cuda").reshape(2, 4)
    with pytest.raises(Bm.MetokError):
        Bm.metok_kv_relink_paged([pool], [pool], table, [torch.zeros((2, 17), dtype=torch.int32, device="cuda")])   # n_keep > capacity
    with pytest.raises(Bm.MetokError):
        Bm.metok_kv_relink_paged([pool], [pool], table, [torch.zeros((2, 9), dtype=torch.int32, device="cuda")], len_in=[8])
    with pytest.raises(ValueError):
        Bm.metok_kv_relink_paged([pool], [pool], table.to(torch.int64), [torch.zeros((2, 3), dtype=torch.int32, device="cuda")])
