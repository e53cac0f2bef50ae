"""GPU parity of metok_kv_compact_paged against the CPU oracle.  A dense cache filled with the per-row-unique
pattern is scattered into page pools through a random page table; after the paged compaction every logical row
read back through the table must equal the oracle's row copy of the dense cache, bit for bit, and pages that
belong to no sequence must be untouched."""
import numpy as np
import pytest
import torch

from oracle import metok_oracle as O
from paper_2506_02850_amd import synth
from tests.test_gpu_stage3 import as_device, as_host, fill_cache, mk

pytestmark = pytest.mark.gpu


def to_pages(dense, table, n_pages, page_size):
    """dense [B, H, S, dh] -> pool [n_pages, H, page_size, dh]; unused pages carry a marker."""
    B, H, S, dh = dense.shape
    pool = np.full((n_pages, H, page_size, dh), 0x5A5A, dtype=np.int16)
    for b in range(B):
        for p, page in enumerate(table[b]):
            rows = dense[b, :, p * page_size:(p + 1) * page_size]
            pool[page, :, :rows.shape[1]] = rows
    return pool


def run_paged(L, B, H, pages_per_seq, page_size, dh16, dtype, idx_lists, seed=0, spare_pages=5):
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
    new_len = Bm.metok_kv_compact_paged(kd, vd, torch.from_numpy(table).cuda(), idx_dev)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(new_len.cpu().numpy(), [S if ix is None else ix.shape[1] for ix in idx_lists])
    used = set(table.reshape(-1).tolist())
    for l in range(L):
        for dense, before, dev, name in ((ks[l], kp[l], kd[l], "K"), (vs[l], vp[l], vd[l], "V")):
            pool = as_host(dev).reshape(n_pages, H, page_size, dh16)
            for page in range(n_pages):
                if page not in used:
                    assert np.array_equal(pool[page], before[page]), f"layer {l} {name}: spare page {page} was written"
            for b in range(B):
                logical = np.concatenate([pool[page] for page in table[b]], axis=1)          # [H, S, dh]
                for h in range(H):
                    ix = None if idx_lists[l] is None else idx_lists[l][b]
                    ref = O.kv_compact(dense[b, h], ix)
                    assert np.array_equal(logical[h, :ref.shape[0]], ref), f"layer {l} {name} video {b} head {h}"


def nested_lists(rng, B, n_vis, n_text, counts):
    out = []
    for c in counts:
        rows = [np.concatenate([np.sort(rng.choice(n_vis, c, replace=False)), np.arange(n_vis, n_vis + n_text)]) for _ in range(B)]
        out.append(np.stack(rows).astype(np.int32))
    return out


@pytest.mark.parametrize("dtype,dh16,page_size", [("bf16", 128, 16), ("bf16", 64, 7), ("f32", 64, 32), ("bf16", 8, 1)])
def test_paged_compaction_matches_dense_semantics(dtype, dh16, page_size):
    rng = np.random.default_rng(11)
    B, H, pages = 3, 2, 23
    S = pages * page_size
    n_text = min(9, S // 4)
    n_vis = S - n_text
    lists = nested_lists(rng, B, n_vis, n_text, [n_vis // 2, n_vis // 5, 0])
    run_paged(4, B, H, pages, page_size, dh16, dtype, [None] + lists, seed=3)


def test_paged_text_only_rule_and_identity_prefix():
    # layers below l1 untouched, the others keep the text rows only (Sec. 3.3); plus a list whose head stays in place
    B, H, pages, ps = 2, 4, 40, 16
    S = pages * ps
    n_text = 50
    sched = O.kv_text_only_schedule(5, 2, S - n_text, n_text)
    lists = [None if s is None else np.stack([s] * B).astype(np.int32) for s in sched]
    keep_head = np.concatenate([np.arange(300), np.arange(310, S, 3)]).astype(np.int32)
    lists[4] = np.stack([keep_head] * B)
    run_paged(5, B, H, pages, ps, 128, "bf16", lists, seed=5)


def test_paged_longva_shaped_pages_and_errors():
    # one video of the decoding configuration's length: 36864 + 128 rows in 2312 pages of 16, 4 heads x 128
    rng = np.random.default_rng(12)
    B, H, ps = 1, 4, 16
    pages = (36864 + 128) // ps
    lists = nested_lists(rng, B, 36864, 128, [18432, 4608])
    run_paged(2, B, H, pages, ps, 128, "bf16", lists, seed=7, spare_pages=3)
    Bm = mk()
    pool = torch.zeros((8, 2, 4, 64), dtype=torch.bfloat16, device="cuda")
    table = torch.arange(8, dtype=torch.int32, device="cuda").reshape(2, 4)
    idx = torch.zeros((2, 3), dtype=torch.int32, device="cuda")
    with pytest.raises(Bm.MetokError):
        Bm.metok_kv_compact_paged([pool], [pool], table, [torch.zeros((2, 17), dtype=torch.int32, device="cuda")])   # n_keep > capacity
    with pytest.raises(ValueError):
        Bm.metok_kv_compact_paged([pool], [pool], table.to(torch.int64), [idx])
    # a page id outside the pool is never dereferenced: the rows that need it are skipped
    bad = table.clone(); bad[0, 3] = 99
    src = torch.arange(8 * 2 * 4 * 64, device="cuda").reshape(8, 2, 4, 64).to(torch.bfloat16)
    k, v = src.clone(), src.clone()
    Bm.metok_kv_compact_paged([k], [v], bad, [torch.tensor([[1, 13, 14], [2, 3, 5]], dtype=torch.int32, device="cuda")])
    torch.cuda.synchronize()
    assert torch.equal(k[0, :, 0], src[0, :, 1])                      # video 0, row 0 <- row 1 (page 0)
    assert torch.equal(k[0, :, 1], src[0, :, 1])                      # row 1 <- row 13 lives in the bad page: skipped
