// Stage 3 (Sec. 3.3): in-place compaction of the KV cache to the retained rows.
//
// A slab is one [S_cap, dh] matrix: K or V of one layer, one video, one kv head.  Inside a slab
// row i must receive row idx[i] >= i.  One workgroup owns a slab (or a 16-byte-aligned column
// slice of it) and walks it in ascending tiles of rows: all loads of a tile complete, the workgroup
// meets at a barrier, then the tile is stored.  Later tiles only read rows at or above their own first
// row, which no earlier store has touched, so no row is overwritten before it is read.
// Different slabs and different column slices never alias, so workgroups need no ordering.
//
// The paged variant moves the same logical rows through a page table: logical row p of video b lives in
// page table[b][p / page_size], slot p % page_size, of a per-layer pool [n_pages, Hkv, page_size, dh].
// The ordering argument is about logical rows; it carries over because distinct logical rows of a video
// are distinct physical rows as long as no page appears twice in the table.
#include "common.h"

namespace metok {

constexpr int kMaxLayersPerLaunch = 40;
// Measured on MI355X (28-layer LongVA-shaped cache, batch 8): 1024-thread workgroups that keep ONE
// 16-byte load per thread in flight and use non-temporal accesses reach 5.1 TB/s; 256-thread groups
// with 8 loads in flight per thread only 2.6 TB/s, because every slab then runs at once and the DRAM
// pages of 3200 interleaved read/write streams thrash.  Two resident workgroups per CU = 512 slabs.
constexpr int kCompactThreads = 1024;

struct CompactLayer {
    char* k;             // [B, Hkv, S_cap, row_bytes]
    char* v;
    const int32_t* idx;  // [B, n_keep]
    int32_t n_keep;
    int32_t layer_id;
};

struct CompactArgs {
    CompactLayer layer[kMaxLayersPerLaunch];
    int n_layers;
    int B, Hkv;
    int parts;            // column slices per row
    int lanes_per_row;    // 16-byte chunks per column slice
    int rows_per_tile;    // kCompactThreads / lanes_per_row
    int64_t S_cap;
    int64_t row_bytes;
    // paged variant only
    const int32_t* page_table;   // [B, pages_per_seq]
    int page_size, pages_per_seq;
    int64_t n_pages_pool;
};

template <bool PAGED>
__global__ __launch_bounds__(kCompactThreads) void kv_compact_kernel(const CompactArgs args) {
    // block -> (layer slot, video, head, K|V, column slice); layer slots are sorted by work, largest first
    const int units_per_layer = args.B * args.Hkv * 2 * args.parts;
    const int slot = blockIdx.x / units_per_layer;
    int rem = blockIdx.x - slot * units_per_layer;
    const int part = rem % args.parts; rem /= args.parts;
    const int which = rem & 1; rem >>= 1;
    const int head = rem % args.Hkv;
    const int b = rem / args.Hkv;

    const CompactLayer& L = args.layer[slot];
    const int rows = L.n_keep;
    const int32_t* __restrict__ idx = L.idx + static_cast<int64_t>(b) * rows;
    char* pool = which ? L.v : L.k;
    char* base = pool + (static_cast<int64_t>(b) * args.Hkv + head) * args.S_cap * args.row_bytes;      // dense slab
    const int32_t* __restrict__ table = PAGED ? args.page_table + static_cast<int64_t>(b) * args.pages_per_seq : nullptr;

    const int lpr = args.lanes_per_row;
    const int r_in_tile = threadIdx.x / lpr;
    const int col = (part * lpr + (threadIdx.x - r_in_tile * lpr)) * 16;
    const bool active = r_in_tile < args.rows_per_tile;          // threads beyond the last whole row idle
    const uint32_t s_cap = static_cast<uint32_t>(args.S_cap);

    // address of logical row r of this (video, head); nullptr if its page id is not a page of the pool
    auto row_ptr = [&](uint32_t r) -> char* {
        if (!PAGED) return base + static_cast<int64_t>(r) * args.row_bytes;
        const int page = table[r / static_cast<uint32_t>(args.page_size)];
        if (page < 0 || page >= args.n_pages_pool) return nullptr;
        const int64_t prow = (static_cast<int64_t>(page) * args.Hkv + head) * args.page_size + r % static_cast<uint32_t>(args.page_size);
        return pool + prow * args.row_bytes;
    };

    for (int tile = 0; tile < rows; tile += args.rows_per_tile) {
        const int i = tile + r_in_tile;
        u32x4_t v;
        bool move = false;
        char* dst = nullptr;                                      // paged only: looked up before the barrier
        if (active && i < rows) {
            const uint32_t s = static_cast<uint32_t>(idx[i]);
            // rows that stay where they are need no copy; positions outside [i, S_cap) are skipped
            if (s > static_cast<uint32_t>(i) && s < s_cap) {
                const char* src = row_ptr(s);
                if (PAGED) {
                    dst = row_ptr(static_cast<uint32_t>(i));
                    move = src != nullptr && dst != nullptr;
                } else {
                    move = true;
                }
                if (move) v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src + col));
            }
        }
        // every load of this tile has returned before any thread of the workgroup stores into it
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (move) {
            char* out = PAGED ? dst : base + static_cast<int64_t>(i) * args.row_bytes;
            __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(out + col));
        }
    }
}

__global__ void write_lengths_kernel(int32_t* out, const CompactArgs args) {
    // one thread per layer slot of this launch
    int i = threadIdx.x;
    if (i < args.n_layers) out[args.layer[i].layer_id] = args.layer[i].n_keep;
}

}  // namespace metok

using namespace metok;

// Shared host path.  Dense: page_table == nullptr.  Paged: S_cap = pages_per_seq * page_size.
static int compact_impl(void* const* k_layers, void* const* v_layers, int L, int B, int Hkv,
                        int64_t S_cap, int dh, int dtype,
                        const int32_t* const* idx, const int32_t* n_keep, int32_t* new_len,
                        const int32_t* page_table, int page_size, int pages_per_seq, int64_t n_pages_pool,
                        void* stream) {
    if (dtype != METOK_F32 && dtype != METOK_BF16) return fail(METOK_ERR_INVALID_ARG, "unknown dtype %d", dtype);
    if (L < 1 || L > METOK_MAX_LAYERS) return fail(METOK_ERR_INVALID_ARG, "L must be in [1, %d], got %d", METOK_MAX_LAYERS, L);
    if (B < 1 || Hkv < 1 || dh < 1 || S_cap < 1 || S_cap > INT32_MAX)
        return fail(METOK_ERR_INVALID_ARG, "B, Hkv, dh, S_cap must be positive and S_cap < 2^31");
    if (!k_layers || !v_layers || !idx || !n_keep) return fail(METOK_ERR_INVALID_ARG, "NULL layer table");
    const int64_t row_bytes = static_cast<int64_t>(dh) * static_cast<int64_t>(dtype_size(dtype));
    if (row_bytes % 16 != 0) return fail(METOK_ERR_INVALID_ARG, "dh * sizeof(dtype) = %lld is not a multiple of 16", (long long)row_bytes);
    const int chunks = static_cast<int>(row_bytes / 16);
    if (chunks > kCompactThreads * 64) return fail(METOK_ERR_UNSUPPORTED, "rows longer than %d bytes", kCompactThreads * 1024);
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

    // split a row into column slices only when it is too wide for one workgroup pass
    int parts = 1;
    while (chunks / parts > kCompactThreads || chunks % parts) ++parts;
    const int lanes_per_row = chunks / parts;
    hipStream_t st = static_cast<hipStream_t>(stream);

    int32_t host_len[METOK_MAX_LAYERS];
    for (int l = 0; l < L; ++l) host_len[l] = idx[l] ? n_keep[l] : static_cast<int32_t>(S_cap);

    for (int first = 0; first < n_active; first += kMaxLayersPerLaunch) {
        CompactArgs args;
        args.n_layers = (n_active - first < kMaxLayersPerLaunch) ? n_active - first : kMaxLayersPerLaunch;
        for (int i = 0; i < args.n_layers; ++i) {
            const int l = order[first + i];
            args.layer[i].k = static_cast<char*>(k_layers[l]);
            args.layer[i].v = static_cast<char*>(v_layers[l]);
            args.layer[i].idx = idx[l];
            args.layer[i].n_keep = n_keep[l];
            args.layer[i].layer_id = l;
        }
        args.B = B; args.Hkv = Hkv; args.parts = parts; args.lanes_per_row = lanes_per_row;
        args.rows_per_tile = kCompactThreads / lanes_per_row;
        args.S_cap = S_cap; args.row_bytes = row_bytes;
        args.page_table = page_table; args.page_size = page_size; args.pages_per_seq = pages_per_seq; args.n_pages_pool = n_pages_pool;
        const int64_t blocks = static_cast<int64_t>(args.n_layers) * B * Hkv * 2 * parts;
        if (blocks > 0x7fffffff) return fail(METOK_ERR_INVALID_ARG, "too many slabs for one launch");
        if (page_table)
            hipLaunchKernelGGL(kv_compact_kernel<true>, dim3(static_cast<unsigned>(blocks)), dim3(kCompactThreads), 0, st, args);
        else
            hipLaunchKernelGGL(kv_compact_kernel<false>, dim3(static_cast<unsigned>(blocks)), dim3(kCompactThreads), 0, st, args);
        int rc = check_launch("kv_compact");
        if (rc) return rc;
    }
    if (new_len) {
        // all L lengths, in layer order, through the same kernel-argument path (no host buffer is read later)
        for (int first = 0; first < L; first += kMaxLayersPerLaunch) {
            CompactArgs args;
            args.n_layers = (L - first < kMaxLayersPerLaunch) ? L - first : kMaxLayersPerLaunch;
            for (int i = 0; i < args.n_layers; ++i) {
                args.layer[i].k = nullptr; args.layer[i].v = nullptr; args.layer[i].idx = nullptr;
                args.layer[i].n_keep = host_len[first + i];
                args.layer[i].layer_id = first + i;
            }
            args.B = B; args.Hkv = Hkv; args.parts = 1; args.lanes_per_row = 1; args.rows_per_tile = 1;
            args.S_cap = S_cap; args.row_bytes = row_bytes;
            args.page_table = nullptr; args.page_size = 0; args.pages_per_seq = 0; args.n_pages_pool = 0;
            hipLaunchKernelGGL(write_lengths_kernel, dim3(1), dim3(64), 0, st, new_len, args);
            int rc = check_launch("kv_compact lengths");
            if (rc) return rc;
        }
    }
    return METOK_OK;
}

extern "C" int metok_kv_compact(void* const* k_layers, void* const* v_layers, int L, int B, int Hkv,
                                int64_t S_cap, int dh, int dtype,
                                const int32_t* const* idx, const int32_t* n_keep, int32_t* new_len,
                                void* stream) {
    clear_error();
    return compact_impl(k_layers, v_layers, L, B, Hkv, S_cap, dh, dtype, idx, n_keep, new_len, nullptr, 0, 0, 0, stream);
}

extern "C" int metok_kv_compact_paged(void* const* k_pools, void* const* v_pools, int L, int B, int Hkv,
                                      int64_t n_pages_pool, int page_size, int dh, int dtype,
                                      const int32_t* page_table, int pages_per_seq,
                                      const int32_t* const* idx, const int32_t* n_keep, int32_t* new_len,
                                      void* stream) {
    clear_error();
    if (!page_table || (reinterpret_cast<uintptr_t>(page_table) & 3u)) return fail(METOK_ERR_INVALID_ARG, "page_table NULL or misaligned");
    if (page_size < 1 || pages_per_seq < 1 || n_pages_pool < 1 || n_pages_pool > INT32_MAX)
        return fail(METOK_ERR_INVALID_ARG, "page_size, pages_per_seq and n_pages_pool must be positive");
    const int64_t S_cap = static_cast<int64_t>(pages_per_seq) * page_size;
    if (S_cap > INT32_MAX) return fail(METOK_ERR_INVALID_ARG, "pages_per_seq * page_size must be below 2^31");
    return compact_impl(k_pools, v_pools, L, B, Hkv, S_cap, dh, dtype, idx, n_keep, new_len, page_table, page_size, pages_per_seq,
                        n_pages_pool, stream);
}
