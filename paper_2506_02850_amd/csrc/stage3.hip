// Stage 3 (Sec. 3.3): in-place compaction of the KV cache to the retained rows, and the in-place row
// mover it is built on (also used by metok_prefill_prune when hidden_out == hidden).
//
// A slab is one [S_cap, row] matrix that is compacted on its own: K or V of one layer, one video, one kv
// head (or a 16-byte-aligned column slice of it when a row is wider than one workgroup pass).  Inside a
// slab row i must receive row idx[i] >= i, idx strictly ascending.
//
// The destination rows of a slab are cut into tiles of R rows and a workgroup moves ONE tile: it loads
// the tile's source rows into registers (8 pieces of 16 bytes per thread, all in flight together), waits
// until they have landed, and stores them.  Many tiles of one slab are in flight on different CUs at the
// same time, so the sources of a tile are one long sequential sweep (R rows of a contiguous span) and the
// destinations one contiguous block of R rows: few, long DRAM streams instead of one short stream per
// slab.  Measured on MI355X (28-layer LongVA-shaped cache, batch 8): 5.9 TB/s against 5.2 TB/s for one
// workgroup per slab walking its tiles in order.
//
// Ordering.  A tile's stores may overwrite rows that EARLIER tiles of the slab still have to read (a
// source lies at or after its destination).  Later tiles only read rows at or after their own first row,
// which lie behind every row this tile writes.  So:
//   - inside a tile, a barrier separates "all my sources are in registers" from "I store";
//   - across tiles, a tile publishes a flag once its sources are in registers, and before storing it
//     waits for the flags of the earlier tiles whose sources fall into its destination rows [r0, r1).
//     Those are the destination rows lo <= i < hi with lo = #{idx < r0}, hi = min(#{idx < r1}, r0): a
//     contiguous run, found with two 64-ary searches that overlap the loads in flight; it spans at most a
//     few tiles.
// Tiles are handed out by an atomic ticket in ascending order inside a slab, so a tile only ever waits
// for tiles whose workgroups are already running, and a running workgroup publishes its flag before it
// waits for anything: the waits always end.  They are bounded nevertheless: a wait that expires sets the
// error word of the workspace and the tile is not stored.
// Different slabs never alias, so they need no ordering; the column slices and the K / V halves of one
// (layer, video) share the index list and are interleaved tile by tile.
//
// The paged variant moves the same logical rows through a page table: logical row p of video b lives in
// page table[b][p / page_size], slot p % page_size, of a per-layer pool [n_pages, Hkv, page_size, dh].
// The ordering argument is about logical rows; it carries over because distinct logical rows of a video
// are distinct physical rows as long as no page appears twice in the table.
//
// With relinked page tables (metok_kv_relink_paged) the planning kernel decides which tiles copy anything at
// all: it raises the flags of the others itself and writes the tiles with work, ascending inside a (layer,
// video), to a list; only the first (length of the list) x (slabs per video) workgroups of the mover take a
// ticket, and the ticket order is the order of the list, so the argument about the waits is unchanged.
#include "common.h"

namespace metok {

constexpr int kMoveThreads = 1024;
constexpr int kMoveInFlight = 8;        // 16-byte pieces per thread: 1024 x 8 x 16 B = 128 KB per tile

namespace {
int g_spin_limit = 1 << 24;             // polls of one flag before a wait is given up (tens of seconds)
}

struct MoveArgs {
    RowMoveLayer layer[kMaxLayersPerLaunch];
    int n_layers;
    int B, Hkv, n_which;  // slabs of a layer: B videos x Hkv heads x n_which buffers (K, V)
    int parts;            // column slices per row
    int lanes_per_row;    // 16-byte pieces per column slice
    int rows_per_step;    // kMoveThreads / lanes_per_row
    int tiles_max;        // flag slots per slab
    int total_items;      // tiles of all slabs of this launch
    int spin_limit;
    int64_t S_cap;
    int64_t row_bytes;
    uint32_t* flags;      // [n_layers][B * Hkv * n_which * parts][tiles_max]
    uint32_t* ticket;     // this launch's tile counter
    uint32_t* error;      // set to 1 if a bounded wait expired
    // paged variants only
    const int32_t* page_table;   // [B, pages_per_seq] (relink: the tables the rows are read through, + layer_id * table_in_layer_stride)
    int page_size, pages_per_seq;
    int64_t n_pages_pool;
    // relink variant only: rows are written through the new tables; home_page[D] is the OLD logical page whose
    // physical page the new logical page D occupies
    int64_t table_in_layer_stride;
    const int32_t* table_out;    // [L, B, pages_per_seq]
    const int32_t* home_page;    // [L, B, pages_per_seq]
    // (video, tile) groups of this launch that have rows to copy, written by the planning kernel: group ids
    // first_item / n_sub + video * tiles + tile, ascending within a (layer, video); *n_work of them
    const int32_t* worklist;
    const uint32_t* n_work;
};

enum { kMoveDense = 0, kMovePaged = 1, kMoveRelink = 2 };

// First position p in idx[0, n) with idx[p] >= key (n if there is none), for ascending idx; all 64 lanes
// of the calling wave take part: each round probes 64 positions, three rounds cover 2^18 entries.
// Terminates for any contents of idx (the range shrinks every round).
__device__ __forceinline__ int wave_lower_bound(const int32_t* __restrict__ idx, int n, int key) {
    const int lane = threadIdx.x & 63;
    int lo = 0, len = n;        // positions below lo are < key; position lo + len is >= key or the end of the range
    while (len > 0) {
        const int step = (len + 63) / 64;
        const int p = lo + (lane + 1) * step - 1;
        const bool ge = p >= lo + len ? true : idx[p] >= key;
        const unsigned long long m = __ballot(ge);
        if (m == 0ull) { lo += len; break; }                       // every probe is below key and the last one is the last position
        const int first = __ffsll(static_cast<long long>(m)) - 1;
        const int new_lo = lo + first * step;                      // one past the probe of lane first - 1
        int new_end = lo + (first + 1) * step - 1;                 // the probe of lane first
        if (new_end > lo + len) new_end = lo + len;
        len = new_end - new_lo;
        lo = new_lo;
    }
    return lo;
}

template <int MODE>
__global__ __launch_bounds__(kMoveThreads) void move_rows_kernel(const MoveArgs args) {
    constexpr bool PAGED = MODE != kMoveDense;
    constexpr int U = kMoveInFlight;
    __shared__ int s_item, s_lo, s_hi;
    const int n_sub = args.Hkv * args.n_which * args.parts;
    // With relinked tables only the tiles on the work list run: the first n_work * n_sub workgroups take one ticket
    // each, the others leave before they touch the counter.
    const int64_t n_items = MODE == kMoveRelink ? static_cast<int64_t>(*args.n_work) * n_sub : args.total_items;
    if (MODE == kMoveRelink && static_cast<int64_t>(blockIdx.x) >= n_items) return;
    if (threadIdx.x == 0) s_item = static_cast<int>(atomicAdd(args.ticket, 1u));
    __syncthreads();
    int item = s_item;
    if (item >= n_items) return;
    if (MODE == kMoveRelink) {
        const int k = item / n_sub;
        item = args.worklist[k] * n_sub + (item - k * n_sub);
    }
    int slot = 0;
    while (slot + 1 < args.n_layers && args.layer[slot + 1].first_item <= item) ++slot;
    const RowMoveLayer& L = args.layer[slot];
    // item -> (video, tile, sub-slab): the sub-slabs of one video share its index list and advance together
    const int local = item - L.first_item;
    const int b = local / (n_sub * L.tiles);
    int rem = local - b * n_sub * L.tiles;
    const int tile = rem / n_sub;
    int sub = rem - tile * n_sub;
    const int part = sub % args.parts; sub /= args.parts;
    const int which = sub % args.n_which;
    const int head = sub / args.n_which;

    const int rows = L.n_keep;
    const int32_t* __restrict__ idx = L.idx + static_cast<int64_t>(b) * rows;
    char* pool = which ? L.v : L.k;
    char* base = pool + (static_cast<int64_t>(b) * args.Hkv + head) * args.S_cap * args.row_bytes;      // dense slab
    const int32_t* __restrict__ table = PAGED ? args.page_table + (MODE == kMoveRelink ? L.layer_id * args.table_in_layer_stride : 0) +
                                                    static_cast<int64_t>(b) * args.pages_per_seq : nullptr;
    const int64_t lb = (static_cast<int64_t>(L.layer_id) * args.B + b) * args.pages_per_seq;
    const int32_t* __restrict__ table_dst = MODE == kMoveRelink ? args.table_out + lb : table;
    uint32_t* flags = args.flags + (static_cast<size_t>(L.flag_slot) * args.B * n_sub + static_cast<size_t>(b) * n_sub + (rem - tile * n_sub)) *
                                       args.tiles_max;

    const int lpr = args.lanes_per_row;
    const int rps = args.rows_per_step;
    const int R = rps * U;
    const int r0 = tile * R;
    const int r_in = threadIdx.x / lpr;
    const int col = (part * lpr + (threadIdx.x - r_in * lpr)) * 16;
    const bool active = r_in < rps;                               // threads beyond the last whole row idle
    const uint32_t s_cap = static_cast<uint32_t>(args.S_cap);

    // The loads of a tile are requested in batches without any branch between them -- first the U index entries, then
    // (paged) the 2 U page-table entries, then the U row pieces -- so that all pieces of a thread are in flight
    // together.  (With a branch around each load the compiler has to wait for every earlier load before the next
    // one, and the eight pieces of a thread went to memory one after the other.)  A piece that does not move reads
    // the first 16 bytes of the pool instead, a valid address, and is never stored.
    uint32_t src_row[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int i = r0 + u * rps + r_in;
        src_row[u] = static_cast<uint32_t>(idx[i < rows ? i : rows - 1]);
    }
    u32x4_t v[U];
    char* dst[U];                                                 // nullptr: this piece does not move
    if (!PAGED) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = r0 + u * rps + r_in;
            const uint32_t sr = src_row[u];
            // rows that stay where they are need no copy; positions outside (i, S_cap) are skipped
            const bool moves = active && i < rows && sr > static_cast<uint32_t>(i) && sr < s_cap;
            const char* src = moves ? base + static_cast<int64_t>(sr) * args.row_bytes + col : pool;
            dst[u] = moves ? base + static_cast<int64_t>(i) * args.row_bytes + col : nullptr;
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src));
        }
    } else {
        // logical row r of this (video, head) lives in page table[r / page_size], slot r % page_size; a page id that
        // is not a page of the pool makes the piece stay.  With relinked tables "stays where it is" is about the
        // physical row: a row of a relinked page never moves, a row with the same logical position moves if its page
        // changed.
        const uint32_t ps = static_cast<uint32_t>(args.page_size);
        const uint32_t last_page = static_cast<uint32_t>(args.pages_per_seq - 1);
        int page_s[U], page_d[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = r0 + u * rps + r_in;
            const uint32_t ps_idx = src_row[u] / ps, pd_idx = static_cast<uint32_t>(i < rows ? i : rows - 1) / ps;
            page_s[u] = table[ps_idx < last_page ? ps_idx : last_page];
            page_d[u] = table_dst[pd_idx < last_page ? pd_idx : last_page];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int i = r0 + u * rps + r_in;
            const uint32_t sr = src_row[u];
            const bool in_range = active && i < rows && sr < s_cap &&
                                  (MODE == kMoveRelink ? sr >= static_cast<uint32_t>(i) : sr > static_cast<uint32_t>(i));
            const bool pages_ok = page_s[u] >= 0 && page_s[u] < args.n_pages_pool && page_d[u] >= 0 && page_d[u] < args.n_pages_pool;
            const int64_t prow_s = (static_cast<int64_t>(page_s[u]) * args.Hkv + head) * args.page_size + sr % ps;
            const int64_t prow_d = (static_cast<int64_t>(page_d[u]) * args.Hkv + head) * args.page_size + static_cast<uint32_t>(i) % ps;
            const bool moves = in_range && pages_ok && prow_s != prow_d;
            const char* src = moves ? pool + prow_s * args.row_bytes + col : pool;
            dst[u] = moves ? pool + prow_d * args.row_bytes + col : nullptr;
            v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src));
        }
    }
    // Destination rows [lo, hi) of earlier tiles take their sources from the rows this tile overwrites: its own
    // destination rows [r0, r1), or with relinked tables the old logical rows of the pages its new pages occupy
    // (home pages ascend with the new page and never lie after it, so those readers are earlier tiles too).
    const int r1 = min(r0 + R, rows);
    const int wave = threadIdx.x >> 6;
    if (wave < 2) {
        int key = wave == 0 ? r0 : r1;
        if (MODE == kMoveRelink && r1 > r0) {
            const int ps = args.page_size, d0 = r0 / ps, d1 = (r1 - 1) / ps;
            int ext = wave == 0 ? 0x7fffffff : -1;                // wave 0: lowest home page of the tile, wave 1: highest
            for (int D = d0 + (threadIdx.x & 63); D <= d1; D += 64) {
                const int h = args.home_page[lb + D];
                ext = wave == 0 ? min(ext, h) : max(ext, h);
            }
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const int o = __shfl_xor(ext, off, 64);
                ext = wave == 0 ? min(ext, o) : max(ext, o);
            }
            const int64_t k64 = wave == 0 ? static_cast<int64_t>(ext) * ps : (static_cast<int64_t>(ext) + 1) * ps;
            key = k64 > 0x7fffffff ? 0x7fffffff : static_cast<int>(k64);
        }
        const int pos = wave_lower_bound(idx, r0, key);
        if ((threadIdx.x & 63) == 0) { if (wave == 0) s_lo = pos; else s_hi = pos; }
    }
    // every source piece of this tile is in registers before the flag goes up and before any thread stores
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) __hip_atomic_store(&flags[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const int lo = s_lo, hi = s_hi;                               // both <= r0
    bool ok = true;
    if (lo < hi) {
        const int t_lo = lo / R, t_hi = (hi - 1) / R;             // earlier tiles of this slab: t_hi < tile
        for (int t = t_lo + static_cast<int>(threadIdx.x); t <= t_hi; t += kMoveThreads) {
            int polls = 0;
            while (__hip_atomic_load(&flags[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0u) {
                if (++polls > args.spin_limit) { ok = false; break; }
                __builtin_amdgcn_s_sleep(8);
            }
        }
    }
    if (!__syncthreads_and(ok ? 1 : 0)) {
        if (threadIdx.x == 0) atomicOr(args.error, 1u);
        return;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (dst[u] != nullptr) __builtin_nontemporal_store(v[u], reinterpret_cast<u32x4_t*>(dst[u]));
}

// Clears the words the move kernels will use (flags, tickets, error word) and writes the per-layer lengths.
__global__ __launch_bounds__(256) void move_init_kernel(uint32_t* __restrict__ words, size_t n_words, int32_t* __restrict__ new_len,
                                                        const LengthTable lengths) {
    const size_t stride = static_cast<size_t>(gridDim.x) * 256;
    for (size_t i = static_cast<size_t>(blockIdx.x) * 256 + threadIdx.x; i < n_words; i += stride) words[i] = 0u;
    if (new_len != nullptr && blockIdx.x == 0 && static_cast<int>(threadIdx.x) < lengths.n) new_len[threadIdx.x] = lengths.len[threadIdx.x];
}

// ---------------------------------------------------------------------------------------------
// Page relinking (Sec. 3.3 on a paged cache): instead of moving every kept row, a new page table is
// written per layer and video.  A new logical page whose rows are exactly one whole old page (all kept,
// in order, aligned) simply takes over that page's physical page; the other new pages are filled by row
// copies into physical pages the sequence already owns, and the pages left over are reported as free.
//
// Plan, one workgroup per (layer, video):
//   1. new page D is "relinked" to old page P iff idx[D ps + t] = P ps + t for all its rows;
//   2. the old pages that are not taken over this way are "free", in ascending order;
//   3. the k-th new page that is not relinked takes the k-th free old page as its home.  Among the old pages
//      0..D at most D - k are taken over by relinks, so that home is at most D: a copied page never lands
//      behind its own logical position, and the rows it overwrites were read by new pages at or before it.
//      This is what lets the row mover order its tiles exactly as in the plain compaction.
//   4. table_out[D] = table_in[home[D]]; the free old pages beyond the ones used as homes are released.
// ---------------------------------------------------------------------------------------------

struct PlanLayer {
    const int32_t* idx; int32_t n_keep; int32_t len_in;
    // the layer's place in the row mover's launches (filled by launch_row_moves; launch < 0: the mover skips the layer)
    int32_t group_base;      // first_item / n_sub
    int16_t flag_slot, launch;
};
struct PlanArgs {
    PlanLayer layer[METOK_MAX_LAYERS];
    // row mover geometry and work lists (filled by launch_row_moves)
    int rows_per_tile, n_sub, tiles_max;
    uint32_t* flags;         // the mover's progress flags
    uint32_t* n_work;        // [launches] counters, zero before this kernel
    int32_t* worklist;       // [L, B, tiles_max]; the list of launch k starts at entry k * kMaxLayersPerLaunch * B * tiles_max
    int B, page_size, pages_per_seq;
    int64_t S_cap, table_in_layer_stride;
    const int32_t* table_in;
    int32_t* table_out;      // [L, B, pps]
    int32_t* free_pages;     // [L, B, pps]
    int32_t* n_free;         // [L, B]
    int32_t* rows_copied;    // [L, B]
    int32_t* home;           // [L, B, pps]  scratch kept for the row mover
    int32_t* used;           // [L, B, pps]  scratch
    int32_t* free_by_rank;   // [L, B, pps]  scratch
    int32_t* relinked;       // [L, B, pps]  scratch
};

constexpr int kPlanThreads = 1024;

__global__ __launch_bounds__(kPlanThreads) void relink_plan_kernel(const PlanArgs a) {
    __shared__ int scan_scratch[17];
    __shared__ int s_count, s_base;
    const int l = blockIdx.y, b = blockIdx.x, tid = threadIdx.x;
    const int pps = a.pages_per_seq, ps = a.page_size;
    const int64_t lb = (static_cast<int64_t>(l) * a.B + b) * pps;
    const int32_t* __restrict__ tin = a.table_in + l * a.table_in_layer_stride + static_cast<int64_t>(b) * pps;
    int32_t* tout = a.table_out + lb;
    int32_t* freed = a.free_pages + lb;
    int32_t* home = a.home + lb;
    int32_t* used = a.used + lb;
    int32_t* fbr = a.free_by_rank + lb;
    int32_t* rel = a.relinked + lb;
    const PlanLayer& L = a.layer[l];
    if (L.idx == nullptr) {                      // untouched layer: the table is carried over
        for (int D = tid; D < pps; D += kPlanThreads) { tout[D] = tin[D]; home[D] = D; freed[D] = -1; }
        if (tid == 0) { a.n_free[static_cast<int64_t>(l) * a.B + b] = 0; a.rows_copied[static_cast<int64_t>(l) * a.B + b] = 0; }
        return;
    }
    const int n = L.n_keep;
    const int32_t* __restrict__ idx = L.idx + static_cast<int64_t>(b) * n;
    const int np_old = (L.len_in + ps - 1) / ps, nd = (n + ps - 1) / ps;
    for (int j = tid; j < pps; j += kPlanThreads) { used[j] = 0; freed[j] = -1; }
    __syncthreads();
    // 1. which new pages are whole old pages
    for (int D = tid; D < nd; D += kPlanThreads) {
        const int rows_d = min(ps, n - D * ps);
        const int s0 = idx[D * ps];
        bool ok = s0 >= 0 && s0 % ps == 0 && static_cast<int64_t>(s0) + rows_d <= L.len_in;
        for (int t = 1; ok && t < rows_d; ++t) ok = idx[D * ps + t] == s0 + t;
        rel[D] = ok ? 1 : 0;
        home[D] = ok ? s0 / ps : -1;
        if (ok) used[s0 / ps] = 1;
    }
    __syncthreads();
    // 1b. the row mover's work list: a tile of destination rows whose new pages are all old pages as they stand has
    // nothing to copy (block-aligned drops, kept prefixes); its progress flags go up here so that no tile waits for
    // it, and it gets no workgroup.  The other tiles of this (layer, video) are appended in ascending order to the
    // list of the layer's launch, in a range reserved with one atomic.
    if (L.launch >= 0) {
        const int R = a.rows_per_tile, tiles = (n + R - 1) / R;
        auto has_work = [&](int t) {
            const int64_t end = min(static_cast<int64_t>(t + 1) * R, static_cast<int64_t>(n));
            const int d1 = static_cast<int>((end - 1) / ps);
            for (int D = static_cast<int>(static_cast<int64_t>(t) * R / ps); D <= d1; ++D)
                if (rel[D] == 0) return 1;
            return 0;
        };
        int n_mine = 0;
        for (int base = 0; base < tiles; base += kPlanThreads) {
            const int t = base + tid;
            n_mine += __syncthreads_count(t < tiles && has_work(t));
        }
        if (tid == 0) s_base = n_mine ? static_cast<int>(atomicAdd(a.n_work + L.launch, static_cast<uint32_t>(n_mine))) : 0;
        __syncthreads();
        int32_t* list = a.worklist + static_cast<int64_t>(L.launch) * kMaxLayersPerLaunch * a.B * a.tiles_max + s_base;
        uint32_t* flags = a.flags + (static_cast<size_t>(L.flag_slot) * a.B + b) * a.n_sub * a.tiles_max;
        int done = 0;
        for (int base = 0; base < tiles; base += kPlanThreads) {
            const int t = base + tid;
            const int f = (t < tiles) ? has_work(t) : 0;
            int tot = 0;
            const int ex = block_exclusive_scan(f, scan_scratch, &tot);
            if (f) list[done + ex] = L.group_base + b * tiles + t;
            else if (t < tiles)
                for (int sub = 0; sub < a.n_sub; ++sub) flags[static_cast<size_t>(sub) * a.tiles_max + t] = 1u;
            done += tot;
        }
    }
    // 2. free old pages in ascending order
    int carry = 0;
    for (int base = 0; base < np_old; base += kPlanThreads) {
        const int j = base + tid;
        const int f = (j < np_old && used[j] == 0) ? 1 : 0;
        int tot = 0;
        const int ex = block_exclusive_scan(f, scan_scratch, &tot);
        if (f) fbr[carry + ex] = j;
        carry += tot;
    }
    const int total_free = carry;
    __syncthreads();
    // 3. homes of the new pages that are filled by copies
    carry = 0;
    for (int base = 0; base < nd; base += kPlanThreads) {
        const int D = base + tid;
        const int f = (D < nd && rel[D] == 0) ? 1 : 0;
        int tot = 0;
        const int ex = block_exclusive_scan(f, scan_scratch, &tot);
        if (f) home[D] = carry + ex < total_free ? fbr[carry + ex] : D;      // the bound only fails for n_keep > len_in, refused by the host
        carry += tot;
    }
    const int n_copied_pages = carry;
    __syncthreads();
    // 4. the new table and the released pages
    for (int D = tid; D < pps; D += kPlanThreads) {
        int page = -1;
        if (D < nd) { const int h = home[D]; page = (h >= 0 && h < pps) ? tin[h] : -1; }
        tout[D] = page;
    }
    for (int r = n_copied_pages + tid; r < total_free; r += kPlanThreads) freed[r - n_copied_pages] = tin[fbr[r]];
    // rows that change their physical place
    int mine = 0;
    for (int d = tid; d < n; d += kPlanThreads) {
        const int s = idx[d];
        if (s >= d && s < a.S_cap && static_cast<int64_t>(home[d / ps]) * ps + d % ps != s) ++mine;
    }
    if (tid == 0) s_count = 0;
    __syncthreads();
    if (mine) atomicAdd(&s_count, mine);
    __syncthreads();
    if (tid == 0) {
        a.n_free[static_cast<int64_t>(l) * a.B + b] = total_free > n_copied_pages ? total_free - n_copied_pages : 0;
        a.rows_copied[static_cast<int64_t>(l) * a.B + b] = s_count;
    }
}

// four [L, B, pages_per_seq] tables and the mover's work lists [L, B, tiles_max]
static size_t relink_scratch_bytes(int L, int B, int pages_per_seq, int64_t tiles_max) {
    return 4 * round_up(static_cast<size_t>(L) * B * pages_per_seq * sizeof(int32_t), 256) +
           round_up(static_cast<size_t>(L) * B * static_cast<size_t>(tiles_max) * sizeof(int32_t), 256);
}


RowMoveGeom row_move_geom(int64_t row_bytes) {
    RowMoveGeom g;
    const int chunks = static_cast<int>(row_bytes / 16);
    // split a row into column slices only when it is too wide for one workgroup pass
    int parts = 1;
    while (chunks / parts > kMoveThreads || chunks % parts) ++parts;
    g.parts = parts;
    g.lanes_per_row = chunks / parts;
    g.rows_per_step = kMoveThreads / g.lanes_per_row;
    g.rows_per_tile = g.rows_per_step * kMoveInFlight;
    return g;
}

// words: [0] error, [1 .. 1 + launches) tickets, [1 + launches .. 1 + 2 launches) work-list lengths (relinked tables),
// then padding to 64 words, then the flags
static int move_launches(int L) { return (L + kMaxLayersPerLaunch - 1) / kMaxLayersPerLaunch; }
static size_t move_header_words(int L) { return round_up(1 + 2 * static_cast<size_t>(move_launches(L)), 64); }

size_t row_move_workspace_bytes(int L, int B, int Hkv, int n_which, int64_t S_cap, int64_t row_bytes) {
    const RowMoveGeom g = row_move_geom(row_bytes);
    const size_t tiles = static_cast<size_t>((S_cap + g.rows_per_tile - 1) / g.rows_per_tile);
    const size_t flags = static_cast<size_t>(L) * B * Hkv * n_which * g.parts * tiles;
    return round_up((move_header_words(L) + flags) * sizeof(uint32_t), 256);
}

// Host side of both stage-3 calls and of the in-place hidden-state compaction.  layers[i] needs k (v if
// n_which == 2), idx and n_keep; layers with n_keep == 0 must have been left out by the caller.
int launch_row_moves(RowMoveLayer* layers, int n_active, int B, int Hkv, int n_which, int64_t S_cap, int64_t row_bytes,
                     const int32_t* page_table, int page_size, int pages_per_seq, int64_t n_pages_pool,
                     int32_t* new_len, const int32_t* host_len, int L_total,
                     void* workspace, size_t workspace_bytes, hipStream_t st, const RelinkTables* relink) {
    const RowMoveGeom g = row_move_geom(row_bytes);
    const size_t need = row_move_workspace_bytes(L_total, B, Hkv, n_which, S_cap, row_bytes);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15u))
        return fail(METOK_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    uint32_t* words = static_cast<uint32_t*>(workspace);
    const size_t header = move_header_words(L_total);
    const int n_sub = Hkv * n_which * g.parts;
    const int tiles_max = static_cast<int>((S_cap + g.rows_per_tile - 1) / g.rows_per_tile);
    const size_t used_words = header + static_cast<size_t>(n_active) * B * n_sub * tiles_max;

    // one small launch clears the flags / tickets / error word and writes the lengths (L_total <= METOK_MAX_LAYERS)
    LengthTable lengths;
    lengths.n = new_len ? L_total : 0;
    for (int l = 0; l < lengths.n; ++l) lengths.len[l] = host_len[l];
    unsigned init_blocks = static_cast<unsigned>((used_words + 1023) / 1024);
    if (init_blocks < 1) init_blocks = 1;
    if (init_blocks > 1024) init_blocks = 1024;
    hipLaunchKernelGGL(move_init_kernel, dim3(init_blocks), dim3(256), 0, st, words, used_words, new_len, lengths);
    int rc = check_launch("row move init");
    if (rc) return rc;

    // the place of every layer in the launches
    const int n_launches = move_launches(L_total);
    int64_t launch_items[(METOK_MAX_LAYERS + kMaxLayersPerLaunch - 1) / kMaxLayersPerLaunch] = {};
    for (int first = 0, launch = 0; first < n_active; first += kMaxLayersPerLaunch, ++launch) {
        const int n_here = (n_active - first < kMaxLayersPerLaunch) ? n_active - first : kMaxLayersPerLaunch;
        int64_t items = 0;
        for (int i = 0; i < n_here; ++i) {
            RowMoveLayer& Lr = layers[first + i];
            Lr.tiles = (Lr.n_keep + g.rows_per_tile - 1) / g.rows_per_tile;
            if (items > INT32_MAX) return fail(METOK_ERR_INVALID_ARG, "too many tiles for one launch");
            Lr.first_item = static_cast<int32_t>(items);
            Lr.flag_slot = first + i;
            items += static_cast<int64_t>(Lr.tiles) * B * n_sub;
        }
        if (items > INT32_MAX) return fail(METOK_ERR_INVALID_ARG, "too many tiles for one launch");
        launch_items[launch] = items;
    }
    if (relink) {
        // the planning kernel runs between the clearing of the flags and the moves: it raises the flags of the tiles
        // that have nothing to copy and lists the others
        PlanArgs& plan = *relink->plan;
        for (int l = 0; l < METOK_MAX_LAYERS; ++l) { plan.layer[l].group_base = 0; plan.layer[l].flag_slot = 0; plan.layer[l].launch = -1; }
        for (int i = 0; i < n_active; ++i) {
            PlanLayer& pl = plan.layer[layers[i].layer_id];
            pl.group_base = layers[i].first_item / n_sub;
            pl.flag_slot = static_cast<int16_t>(layers[i].flag_slot);
            pl.launch = static_cast<int16_t>(i / kMaxLayersPerLaunch);
        }
        plan.rows_per_tile = g.rows_per_tile; plan.n_sub = n_sub; plan.tiles_max = tiles_max;
        plan.flags = words + header; plan.n_work = words + 1 + n_launches;
        hipLaunchKernelGGL(relink_plan_kernel, dim3(B, L_total), dim3(kPlanThreads), 0, st, plan);
        rc = check_launch("relink plan");
        if (rc) return rc;
    }

    for (int first = 0, launch = 0; first < n_active; first += kMaxLayersPerLaunch, ++launch) {
        MoveArgs args;
        args.n_layers = (n_active - first < kMaxLayersPerLaunch) ? n_active - first : kMaxLayersPerLaunch;
        for (int i = 0; i < args.n_layers; ++i) args.layer[i] = layers[first + i];
        const int64_t items = launch_items[launch];
        args.B = B; args.Hkv = Hkv; args.n_which = n_which; args.parts = g.parts; args.lanes_per_row = g.lanes_per_row;
        args.rows_per_step = g.rows_per_step; args.tiles_max = tiles_max; args.total_items = static_cast<int>(items);
        args.spin_limit = g_spin_limit;
        args.S_cap = S_cap; args.row_bytes = row_bytes;
        args.flags = words + header; args.ticket = words + 1 + launch; args.error = words;
        args.page_table = page_table; args.page_size = page_size; args.pages_per_seq = pages_per_seq; args.n_pages_pool = n_pages_pool;
        args.table_in_layer_stride = relink ? relink->table_in_layer_stride : 0;
        args.table_out = relink ? relink->table_out : nullptr;
        args.home_page = relink ? relink->home_page : nullptr;
        args.worklist = relink ? relink->plan->worklist + static_cast<int64_t>(launch) * kMaxLayersPerLaunch * B * tiles_max : nullptr;
        args.n_work = relink ? words + 1 + n_launches + launch : nullptr;
        if (items == 0) continue;
        if (relink)
            { TraceScope trace_scope(METOK_TRACE_MOVE_ROWS, st); hipLaunchKernelGGL(move_rows_kernel<kMoveRelink>, dim3(static_cast<unsigned>(items)), dim3(kMoveThreads), 0, st, args); }
        else if (page_table)
            { TraceScope trace_scope(METOK_TRACE_MOVE_ROWS, st); hipLaunchKernelGGL(move_rows_kernel<kMovePaged>, dim3(static_cast<unsigned>(items)), dim3(kMoveThreads), 0, st, args); }
        else
            { TraceScope trace_scope(METOK_TRACE_MOVE_ROWS, st); hipLaunchKernelGGL(move_rows_kernel<kMoveDense>, dim3(static_cast<unsigned>(items)), dim3(kMoveThreads), 0, st, args); }
        rc = check_launch("move_rows");
        if (rc) return rc;
    }
    return METOK_OK;
}

}  // namespace metok

using namespace metok;

// Shared host path.  Dense: page_table == nullptr.  Paged: S_cap = pages_per_seq * page_size.
static int compact_impl(void* const* k_layers, void* const* v_layers, int L, int B, int Hkv,
                        int64_t S_cap, int dh, int dtype,
                        const int32_t* const* idx, const int32_t* n_keep, int32_t* new_len,
                        const int32_t* page_table, int page_size, int pages_per_seq, int64_t n_pages_pool,
                        void* workspace, size_t workspace_bytes, void* stream) {
    if (dtype != METOK_F32 && dtype != METOK_BF16) return fail(METOK_ERR_INVALID_ARG, "unknown dtype %d", dtype);
    if (L < 1 || L > METOK_MAX_LAYERS) return fail(METOK_ERR_INVALID_ARG, "L must be in [1, %d], got %d", METOK_MAX_LAYERS, L);
    if (B < 1 || Hkv < 1 || dh < 1 || S_cap < 1 || S_cap > INT32_MAX)
        return fail(METOK_ERR_INVALID_ARG, "B, Hkv, dh, S_cap must be positive and S_cap < 2^31");
    if (!k_layers || !v_layers || !idx || !n_keep) return fail(METOK_ERR_INVALID_ARG, "NULL layer table");
    const int64_t row_bytes = static_cast<int64_t>(dh) * static_cast<int64_t>(dtype_size(dtype));
    if (row_bytes % 16 != 0) return fail(METOK_ERR_INVALID_ARG, "dh * sizeof(dtype) = %lld is not a multiple of 16", (long long)row_bytes);
    if (row_bytes / 16 > kMoveThreads * 64) return fail(METOK_ERR_UNSUPPORTED, "rows longer than %d bytes", kMoveThreads * 1024);
    if (static_cast<int64_t>(B) * Hkv * 2 > (1 << 20)) return fail(METOK_ERR_INVALID_ARG, "B * Hkv too large");

    // layers that move data, largest first so that the long slabs start early
    int order[METOK_MAX_LAYERS];
    int n_active = 0;
    for (int l = 0; l < L; ++l) {
        if (!idx[l]) continue;
        if (n_keep[l] < 0 || n_keep[l] > S_cap)
            return fail(METOK_ERR_INVALID_ARG, "n_keep[%d] = %d outside [0, S_cap]", l, n_keep[l]);
        if (!k_layers[l] || !v_layers[l] || !aligned16(k_layers[l]) || !aligned16(v_layers[l]) ||
            (reinterpret_cast<uintptr_t>(idx[l]) & 3u))
            return fail(METOK_ERR_INVALID_ARG, "layer %d: NULL or misaligned pointer", l);
        if (n_keep[l] == 0) continue;
        order[n_active++] = l;
    }
    for (int i = 1; i < n_active; ++i) {          // insertion sort, stable, by n_keep descending
        int l = order[i], j = i;
        while (j > 0 && n_keep[order[j - 1]] < n_keep[l]) { order[j] = order[j - 1]; --j; }
        order[j] = l;
    }
    RowMoveLayer layers[METOK_MAX_LAYERS];
    for (int i = 0; i < n_active; ++i) {
        const int l = order[i];
        layers[i].k = static_cast<char*>(k_layers[l]);
        layers[i].v = static_cast<char*>(v_layers[l]);
        layers[i].idx = idx[l];
        layers[i].n_keep = n_keep[l];
        layers[i].first_item = 0; layers[i].tiles = 0; layers[i].flag_slot = 0; layers[i].layer_id = l;
    }
    int32_t host_len[METOK_MAX_LAYERS];
    for (int l = 0; l < L; ++l) host_len[l] = idx[l] ? n_keep[l] : static_cast<int32_t>(S_cap);
    return launch_row_moves(layers, n_active, B, Hkv, 2, S_cap, row_bytes, page_table, page_size, pages_per_seq, n_pages_pool,
                            new_len, host_len, L, workspace, workspace_bytes, static_cast<hipStream_t>(stream), nullptr);
}

extern "C" size_t metok_kv_compact_workspace_bytes(int L, int B, int Hkv, int64_t S_cap, int dh, int dtype) {
    if (L < 1 || L > METOK_MAX_LAYERS || B < 1 || Hkv < 1 || S_cap < 1 || S_cap > INT32_MAX || dh < 1 ||
        (dtype != METOK_F32 && dtype != METOK_BF16))
        return 0;
    const int64_t row_bytes = static_cast<int64_t>(dh) * static_cast<int64_t>(dtype_size(dtype));
    if (row_bytes % 16 != 0 || row_bytes / 16 > kMoveThreads * 64) return 0;
    return row_move_workspace_bytes(L, B, Hkv, 2, S_cap, row_bytes);
}

extern "C" int metok_kv_compact(void* const* k_layers, void* const* v_layers, int L, int B, int Hkv,
                                int64_t S_cap, int dh, int dtype,
                                const int32_t* const* idx, const int32_t* n_keep, int32_t* new_len,
                                void* workspace, size_t workspace_bytes, void* stream) {
    clear_error();
    return compact_impl(k_layers, v_layers, L, B, Hkv, S_cap, dh, dtype, idx, n_keep, new_len, nullptr, 0, 0, 0,
                        workspace, workspace_bytes, stream);
}

extern "C" int metok_kv_compact_paged(void* const* k_pools, void* const* v_pools, int L, int B, int Hkv,
                                      int64_t n_pages_pool, int page_size, int dh, int dtype,
                                      const int32_t* page_table, int pages_per_seq,
                                      const int32_t* const* idx, const int32_t* n_keep, int32_t* new_len,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    clear_error();
    if (!page_table || (reinterpret_cast<uintptr_t>(page_table) & 3u)) return fail(METOK_ERR_INVALID_ARG, "page_table NULL or misaligned");
    if (page_size < 1 || pages_per_seq < 1 || n_pages_pool < 1 || n_pages_pool > INT32_MAX)
        return fail(METOK_ERR_INVALID_ARG, "page_size, pages_per_seq and n_pages_pool must be positive");
    const int64_t S_cap = static_cast<int64_t>(pages_per_seq) * page_size;
    if (S_cap > INT32_MAX) return fail(METOK_ERR_INVALID_ARG, "pages_per_seq * page_size must be below 2^31");
    return compact_impl(k_pools, v_pools, L, B, Hkv, S_cap, dh, dtype, idx, n_keep, new_len, page_table, page_size, pages_per_seq,
                        n_pages_pool, workspace, workspace_bytes, stream);
}

// Test hook: how often a tile polls one flag before it gives its wait up (default 2^24).  With 0 every
// wait that does not succeed at once expires, which exercises the error word without stalling anything.
extern "C" int metok_debug_set_move_spin_limit(int polls) {
    clear_error();
    if (polls < 0) return fail(METOK_ERR_INVALID_ARG, "polls must be non-negative");
    g_spin_limit = polls;
    return METOK_OK;
}


extern "C" size_t metok_kv_relink_paged_workspace_bytes(int L, int B, int Hkv, int page_size, int pages_per_seq, int dh, int dtype) {
    if (L < 1 || L > METOK_MAX_LAYERS || B < 1 || Hkv < 1 || page_size < 1 || pages_per_seq < 1 || dh < 1 ||
        (dtype != METOK_F32 && dtype != METOK_BF16))
        return 0;
    const int64_t S_cap = static_cast<int64_t>(pages_per_seq) * page_size;
    const int64_t row_bytes = static_cast<int64_t>(dh) * static_cast<int64_t>(dtype_size(dtype));
    if (S_cap > INT32_MAX || row_bytes % 16 != 0 || row_bytes / 16 > kMoveThreads * 64) return 0;
    const RowMoveGeom g = row_move_geom(row_bytes);
    return row_move_workspace_bytes(L, B, Hkv, 2, S_cap, row_bytes) +
           relink_scratch_bytes(L, B, pages_per_seq, (S_cap + g.rows_per_tile - 1) / g.rows_per_tile);
}

extern "C" int metok_kv_relink_paged(void* const* k_pools, void* const* v_pools, int L, int B, int Hkv,
                                     int64_t n_pages_pool, int page_size, int dh, int dtype,
                                     const int32_t* page_table_in, int64_t table_in_layer_stride, int pages_per_seq,
                                     const int32_t* len_in,
                                     const int32_t* const* idx, const int32_t* n_keep,
                                     int32_t* page_table_out, int32_t* free_pages, int32_t* n_free, int32_t* rows_copied,
                                     int32_t* new_len,
                                     void* workspace, size_t workspace_bytes, void* stream) {
    clear_error();
    if (dtype != METOK_F32 && dtype != METOK_BF16) return fail(METOK_ERR_INVALID_ARG, "unknown dtype %d", dtype);
    if (L < 1 || L > METOK_MAX_LAYERS) return fail(METOK_ERR_INVALID_ARG, "L must be in [1, %d], got %d", METOK_MAX_LAYERS, L);
    if (B < 1 || B > 65535 || Hkv < 1 || dh < 1) return fail(METOK_ERR_INVALID_ARG, "B (at most 65535), Hkv and dh must be positive");
    if (page_size < 1 || pages_per_seq < 1 || n_pages_pool < 1 || n_pages_pool > INT32_MAX)
        return fail(METOK_ERR_INVALID_ARG, "page_size, pages_per_seq and n_pages_pool must be positive");
    const int64_t S_cap = static_cast<int64_t>(pages_per_seq) * page_size;
    if (S_cap > INT32_MAX) return fail(METOK_ERR_INVALID_ARG, "pages_per_seq * page_size must be below 2^31");
    if (!k_pools || !v_pools || !idx || !n_keep) return fail(METOK_ERR_INVALID_ARG, "NULL layer table");
    if (!page_table_in || !page_table_out || !free_pages || !n_free || !rows_copied ||
        ((reinterpret_cast<uintptr_t>(page_table_in) | reinterpret_cast<uintptr_t>(page_table_out) | reinterpret_cast<uintptr_t>(free_pages) |
          reinterpret_cast<uintptr_t>(n_free) | reinterpret_cast<uintptr_t>(rows_copied)) & 3u))
        return fail(METOK_ERR_INVALID_ARG, "page tables and counters must be non-NULL and 4-byte aligned");
    if (table_in_layer_stride != 0 && table_in_layer_stride != static_cast<int64_t>(B) * pages_per_seq)
        return fail(METOK_ERR_INVALID_ARG, "table_in_layer_stride must be 0 (one table for all layers) or B * pages_per_seq");
    {   // the new tables must not overwrite the tables the rows are read through
        const char* a0 = reinterpret_cast<const char*>(page_table_in);
        const char* a1 = a0 + (table_in_layer_stride ? static_cast<size_t>(L) : 1) * B * pages_per_seq * sizeof(int32_t);
        const char* b0 = reinterpret_cast<const char*>(page_table_out);
        const char* b1 = b0 + static_cast<size_t>(L) * B * pages_per_seq * sizeof(int32_t);
        if (a0 < b1 && b0 < a1) return fail(METOK_ERR_INVALID_ARG, "page_table_out overlaps page_table_in");
    }
    const int64_t row_bytes = static_cast<int64_t>(dh) * static_cast<int64_t>(dtype_size(dtype));
    if (row_bytes % 16 != 0) return fail(METOK_ERR_INVALID_ARG, "dh * sizeof(dtype) = %lld is not a multiple of 16", (long long)row_bytes);
    if (row_bytes / 16 > kMoveThreads * 64) return fail(METOK_ERR_UNSUPPORTED, "rows longer than %d bytes", kMoveThreads * 1024);
    const size_t need = metok_kv_relink_paged_workspace_bytes(L, B, Hkv, page_size, pages_per_seq, dh, dtype);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 15u))
        return fail(METOK_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);

    PlanArgs plan;
    int order[METOK_MAX_LAYERS];
    int n_active = 0;
    int32_t host_len[METOK_MAX_LAYERS];
    for (int l = 0; l < L; ++l) {
        const int32_t cur = len_in ? len_in[l] : static_cast<int32_t>(S_cap);
        if (cur < 0 || cur > S_cap) return fail(METOK_ERR_INVALID_ARG, "len_in[%d] = %d outside [0, pages_per_seq * page_size]", l, cur);
        plan.layer[l].idx = idx[l];
        plan.layer[l].n_keep = idx[l] ? n_keep[l] : 0;
        plan.layer[l].len_in = cur;
        host_len[l] = idx[l] ? n_keep[l] : cur;
        if (!idx[l]) continue;
        if (n_keep[l] < 0 || n_keep[l] > cur) return fail(METOK_ERR_INVALID_ARG, "n_keep[%d] = %d outside [0, len_in]", l, n_keep[l]);
        if (!k_pools[l] || !v_pools[l] || !aligned16(k_pools[l]) || !aligned16(v_pools[l]) || (reinterpret_cast<uintptr_t>(idx[l]) & 3u))
            return fail(METOK_ERR_INVALID_ARG, "layer %d: NULL or misaligned pointer", l);
        if (n_keep[l] == 0) continue;
        order[n_active++] = l;
    }
    for (int l = L; l < METOK_MAX_LAYERS; ++l) { plan.layer[l].idx = nullptr; plan.layer[l].n_keep = 0; plan.layer[l].len_in = 0; }
    for (int i = 1; i < n_active; ++i) {          // insertion sort, stable, by n_keep descending
        int l = order[i], j = i;
        while (j > 0 && n_keep[order[j - 1]] < n_keep[l]) { order[j] = order[j - 1]; --j; }
        order[j] = l;
    }
    char* ws = static_cast<char*>(workspace);
    const size_t move_bytes = row_move_workspace_bytes(L, B, Hkv, 2, S_cap, row_bytes);
    const size_t slot = round_up(static_cast<size_t>(L) * B * pages_per_seq * sizeof(int32_t), 256);
    plan.B = B; plan.page_size = page_size; plan.pages_per_seq = pages_per_seq; plan.S_cap = S_cap;
    plan.table_in_layer_stride = table_in_layer_stride; plan.table_in = page_table_in;
    plan.table_out = page_table_out; plan.free_pages = free_pages; plan.n_free = n_free; plan.rows_copied = rows_copied;
    plan.home = reinterpret_cast<int32_t*>(ws + move_bytes);
    plan.used = reinterpret_cast<int32_t*>(ws + move_bytes + slot);
    plan.free_by_rank = reinterpret_cast<int32_t*>(ws + move_bytes + 2 * slot);
    plan.relinked = reinterpret_cast<int32_t*>(ws + move_bytes + 3 * slot);
    plan.worklist = reinterpret_cast<int32_t*>(ws + move_bytes + 4 * slot);
    hipStream_t st = static_cast<hipStream_t>(stream);

    RowMoveLayer layers[METOK_MAX_LAYERS];
    for (int i = 0; i < n_active; ++i) {
        const int l = order[i];
        layers[i].k = static_cast<char*>(k_pools[l]);
        layers[i].v = static_cast<char*>(v_pools[l]);
        layers[i].idx = idx[l];
        layers[i].n_keep = n_keep[l];
        layers[i].first_item = 0; layers[i].tiles = 0; layers[i].flag_slot = 0; layers[i].layer_id = l;
    }
    RelinkTables tables;
    tables.table_in_layer_stride = table_in_layer_stride; tables.table_out = page_table_out; tables.home_page = plan.home; tables.plan = &plan;
    return launch_row_moves(layers, n_active, B, Hkv, 2, S_cap, row_bytes, page_table_in, page_size, pages_per_seq, n_pages_pool,
                            new_len, host_len, L, workspace, move_bytes, st, &tables);
}
