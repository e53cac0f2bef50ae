// Shared host/device helpers of the METok HIP library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>
#include <type_traits>

#include "metok.h"

namespace metok {

// ---------------------------------------------------------------------------------------------
// error reporting
// ---------------------------------------------------------------------------------------------
char* error_buffer();                       // thread-local, 512 bytes
int fail(int code, const char* fmt, ...);   // formats into the buffer, returns code
int check_launch(const char* what);         // hipGetLastError -> METOK_ERR_DEVICE
void clear_error();

// Measurement hook (metok_trace_kernel): brackets the launches of one kernel family with the caller's events.
struct KernelTrace { int kernel; hipEvent_t begin, end; };
KernelTrace& kernel_trace();                // thread-local
struct TraceScope {
    hipStream_t st;
    bool armed;
    TraceScope(int kernel, hipStream_t stream) : st(stream) {
        const KernelTrace& t = kernel_trace();
        armed = t.kernel == kernel && t.begin != nullptr && t.end != nullptr;
        if (armed) (void)hipEventRecord(t.begin, st);
    }
    ~TraceScope() { if (armed) (void)hipEventRecord(kernel_trace().end, st); }
};

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline size_t dtype_size(int dtype) { return dtype == METOK_BF16 ? 2 : 4; }
int ceil_ratio(double x);                   // ceil(x - 1e-9)

constexpr int kWave = 64;

// ---------------------------------------------------------------------------------------------
// in-place row mover (stage3.hip): row i of a slab receives row idx[i] >= i.  Used by the KV
// compaction and by metok_prefill_prune when its output aliases its input.
// ---------------------------------------------------------------------------------------------
constexpr int kMaxLayersPerLaunch = 40;

struct RowMoveLayer {
    char* k;             // [B, Hkv, S_cap, row_bytes]
    char* v;             // second buffer of the layer (n_which == 2), else unused
    const int32_t* idx;  // [B, n_keep]
    int32_t n_keep;
    int32_t first_item;  // filled by launch_row_moves
    int32_t tiles;       // filled by launch_row_moves
    int32_t flag_slot;   // filled by launch_row_moves
    int32_t layer_id;    // index of the layer in per-layer tables (relink variant)
};

struct PlanArgs;                     // arguments of the planning kernel of the relink variant
struct RelinkTables {
    int64_t table_in_layer_stride;   // 0: one input table shared by the layers
    const int32_t* table_out;        // [L, B, pages_per_seq]
    const int32_t* home_page;        // [L, B, pages_per_seq]
    PlanArgs* plan;                  // launch_row_moves fills in the mover's geometry and launches the planning kernel
};

struct RowMoveGeom { int parts, lanes_per_row, rows_per_step, rows_per_tile; };

struct LengthTable { int n; int32_t len[METOK_MAX_LAYERS]; };

RowMoveGeom row_move_geom(int64_t row_bytes);
size_t row_move_workspace_bytes(int L, int B, int Hkv, int n_which, int64_t S_cap, int64_t row_bytes);
int launch_row_moves(RowMoveLayer* layers, int n_active, int B, int Hkv, int n_which, int64_t S_cap, int64_t row_bytes,
                     const int32_t* page_table, int page_size, int pages_per_seq, int64_t n_pages_pool,
                     int32_t* new_len, const int32_t* host_len, int L_total,
                     void* workspace, size_t workspace_bytes, hipStream_t st, const RelinkTables* relink);

// ---------------------------------------------------------------------------------------------
// device helpers
// ---------------------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));   // 16 bytes, accepted by the non-temporal builtins

struct bf16_t { uint16_t bits; };           // storage type of a bf16 element

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// Two fp32 values -> packed bf16 pair, round to nearest even: gfx950 converts a pair with one instruction.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    typedef __bf16 bf16x2v_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    const bf16x2v_t r = __builtin_convertvector(v, bf16x2v_t);
    return __builtin_bit_cast(uint32_t, r);
}

// Streaming 16-byte load / store (non-temporal): on MI355X a read-once pass over a few hundred MB runs
// at about 6.5 TB/s with this hint and at about 3.2 TB/s without it.
__device__ __forceinline__ uint4 load_stream(const uint4* p) {
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream(uint4* p, const uint4& v) {
    const u32x4_t t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<u32x4_t*>(p));
}

// acc += a.lo * b.lo + a.hi * b.hi on two packed bf16 pairs, fp32 accumulate.
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), acc, false);
}

// 16-byte chunk arithmetic for the two element types.
template <typename T> struct Elem;
template <> struct Elem<bf16_t> {
    static constexpr int kVec = 8;
    static __device__ __forceinline__ float dot(const uint4& a, const uint4& b, float acc) {
        acc = dot2_bf16(a.x, b.x, acc);
        acc = dot2_bf16(a.y, b.y, acc);
        acc = dot2_bf16(a.z, b.z, acc);
        acc = dot2_bf16(a.w, b.w, acc);
        return acc;
    }
    static __device__ __forceinline__ void accumulate(const uint4& a, float (&acc)[8]) {
        acc[0] += bf16_lo(a.x); acc[1] += bf16_hi(a.x);
        acc[2] += bf16_lo(a.y); acc[3] += bf16_hi(a.y);
        acc[4] += bf16_lo(a.z); acc[5] += bf16_hi(a.z);
        acc[6] += bf16_lo(a.w); acc[7] += bf16_hi(a.w);
    }
};
template <> struct Elem<float> {
    static constexpr int kVec = 4;
    static __device__ __forceinline__ float dot(const uint4& a, const uint4& b, float acc) {
        acc = fmaf(__uint_as_float(a.x), __uint_as_float(b.x), acc);
        acc = fmaf(__uint_as_float(a.y), __uint_as_float(b.y), acc);
        acc = fmaf(__uint_as_float(a.z), __uint_as_float(b.z), acc);
        acc = fmaf(__uint_as_float(a.w), __uint_as_float(b.w), acc);
        return acc;
    }
    static __device__ __forceinline__ void accumulate(const uint4& a, float (&acc)[8]) {
        acc[0] += __uint_as_float(a.x); acc[1] += __uint_as_float(a.y);
        acc[2] += __uint_as_float(a.z); acc[3] += __uint_as_float(a.w);
    }
};

// Order-preserving map from float to uint32: a < b  <=>  key(a) < key(b) (-0 == +0, NaNs at the ends).
__device__ __forceinline__ uint32_t ordered_key(float x) {
    uint32_t u = __float_as_uint(x);
    if (u == 0x80000000u) u = 0u;              // -0 and +0 are the same score
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Sum over the 16 lanes of a DPP row; every lane of the row receives the total.
__device__ __forceinline__ float row16_sum(float v) {
    // row_ror:n rotates within each group of 16 lanes (dpp_ctrl 0x120 + n)
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x128, 0xf, 0xf, false));
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x124, 0xf, 0xf, false));
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x122, 0xf, 0xf, false));
    v += __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(v), 0x121, 0xf, 0xf, false));
    return v;
}
// Sum over all 64 lanes of the wave; every lane receives the total.
__device__ __forceinline__ float wave_sum(float v) {
    v = row16_sum(v);
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    return v;
}
template <int G> __device__ __forceinline__ float group_sum(float v) {
    static_assert(G == 16 || G == 64, "token groups are one DPP row or one wave");
    return G == 16 ? row16_sum(v) : wave_sum(v);
}

// A batch of videos runs as one launch with blockIdx.z = video.  Pointer of that video, `bytes` (or `elems`
// elements) apart from its neighbours; NULL stays NULL.  A launch without a batch has blockIdx.z = 0.
template <typename P> __device__ __forceinline__ P* of_video(P* p, int64_t bytes) {
    using B = typename std::conditional<std::is_const<P>::value, const char, char>::type;
    return p ? reinterpret_cast<P*>(reinterpret_cast<B*>(p) + static_cast<int64_t>(blockIdx.z) * bytes) : p;
}
template <typename P> __device__ __forceinline__ P* of_video_elems(P* p, int64_t elems) {
    return p ? p + static_cast<int64_t>(blockIdx.z) * elems : p;
}

// Exclusive prefix sum of one int per thread over a block of up to 1024 threads.
// `scratch` is 17 ints of LDS; returns the exclusive prefix and stores the block total in *total.
__device__ __forceinline__ int block_exclusive_scan(int v, int* scratch, int* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = (blockDim.x + 63) >> 6;
    int incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int up = __shfl_up(incl, off, 64);
        if (lane >= off) incl += up;
    }
    __syncthreads();                       // scratch may still be read from a previous call
    if (lane == 63) scratch[wave] = incl;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int w = 0; w < nwaves; ++w) { int t = scratch[w]; scratch[w] = run; run += t; }
        scratch[16] = run;
    }
    __syncthreads();
    *total = scratch[16];
    return scratch[wave] + incl - v;
}

}  // namespace metok
