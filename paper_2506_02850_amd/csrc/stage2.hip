// Stage 2 (Sec. 3.2.2): one level of hierarchical pruning.
//
//   pack_q_kernel        text queries -> MFMA fragment order, once per call
//   row_stats_kernel     MFMA pass 1 over all keys: per (head, text query) running max and sum of the
//                        causal softmax, in the log2 domain, per workgroup
//   merge_stats_kernel   merges the per-workgroup (max, sum) pairs into one normaliser per row
//   col_sums_kernel      MFMA pass 2 over the visual keys: recomputes the logits and adds up the
//                        probabilities of every visual key over the rows of a workgroup
//   score_hist_kernel    score_j = w_e(j) * mean probability; per 1024-token tile a histogram of the leading key
//                        bits per retention class; the workgroup that arrives last finds each class's bucket
//   candidate_kernel     per tile: tokens above the bucket counted, tokens inside it listed; the workgroup that
//                        arrives last finishes the radix select on the list -> class threshold, number of equal
//                        scores still kept, output offset of every tile
//   prepare_kernel, select_kernel   the same two steps for more than four classes or more than 40 tiles: one
//                        workgroup per class walks all keys
//   write_index_kernel   one workgroup per 1024-token tile: keep rule (lowest index first among equal
//                        scores), prefix sums -> ascending kept index list and carried metadata
//   gather_rows_kernel   compaction of the hidden states (hidden_index_kernel + the row mover of stage 3 when
//                        the output is the input buffer)
//
// A batch of videos of one shape runs as one launch of every kernel: blockIdx.z is the video, every pointer
// advances by that video's stride, and the per-video workspaces lie one after the other.
//
// Both MFMA passes are query-stationary: a wave keeps the fragments of its own 32-row blocks of queries in
// registers and the workgroup streams its range of keys through LDS.  The contraction index may be
// permuted freely as long as both operands agree; here lane half h = lane/32 owns the contiguous half h
// of the head dimension, so every fragment is a contiguous 16-byte chunk of a row.
#include <mutex>

#include "common.h"

namespace metok {

constexpr int kScoreThreads = 512;
constexpr int kScoreWaves = kScoreThreads / 64;
constexpr float kNegBig = -1.0e30f;
constexpr float kPosBig = 1.0e30f;

// v_exp_f32 without the denormal-range fix-up of exp2f(): arguments here are <= 0 and a result below
// 2^-126 may flush to zero (it is a softmax term that small).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
    static constexpr int kChunkElems = 8;          // one 16-byte chunk feeds one 32x32x16 MFMA
    static constexpr int kMfmaPerChunk = 1;
    static __device__ __forceinline__ f32x16_t mma(const uint4& a, const uint4& b, f32x16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mma<float> {
    static constexpr int kChunkElems = 4;          // one chunk feeds four 32x32x2 MFMAs
    static constexpr int kMfmaPerChunk = 4;
    static __device__ __forceinline__ f32x16_t mma(const uint4& a, const uint4& b, f32x16_t c) {
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
        return c;
    }
};

struct ScoreGeom {
    int64_t S;
    int Hq, Hkv, group, dh, Tq;
    int R;              // rows per kv head = group * Tq
    int rb_total;       // 32-row blocks per kv head
    int rbw;            // row blocks per workgroup (<= kScoreWaves * RBW)
    int rs;             // row splits per kv head
    int vis_start, n_vis;
    int64_t key_begin, key_end;   // keys the softmax of pass 1 normalises over (before the causal mask)
    float scale_log2;   // log2(e) / sqrt(dh)
    // a batch of videos runs as one launch, blockIdx.z = video: distances between consecutive videos
    int64_t q_video, k_video;     // elements of q_text / k_all
    int64_t ws_video;             // bytes of workspace
};


// Kept visual tokens of every video of a batch (the quotas of a video added up), passed by value.
struct BatchKeep { int32_t n[METOK_MAX_BATCH]; };

// ---------------------------------------------------------------------------------------------
// Both MFMA passes are query-stationary: wave w of a workgroup keeps the fragments of its own row
// blocks (local blocks w, w + 8, ...) in registers for the whole kernel, and the workgroup streams its
// contiguous range of keys through LDS, one stage of SUBS 32-key subtiles at a time (kStageBuffers
// stages in LDS, one barrier per stage).  A stage is stored in fragment order,
//     kbuf[(sub * NCH + c) * 64 + lane],   lane = key % 32 + 32 * half,
// so a wave reads the NCH fragments of a subtile with conflict-free 16-byte LDS reads and uses them
// against every row block it owns.
// ---------------------------------------------------------------------------------------------
template <typename T, int NCH, int SUBS>
struct KeyStage {
    static constexpr int kKeys = SUBS * 32;
    static constexpr int kSlots = SUBS * NCH * 64;                 // 16-byte pieces per stage
    static constexpr int kPerThread = (kSlots + kScoreThreads - 1) / kScoreThreads;

    // piece id -> (key in stage, half, chunk); the key runs fastest so that the LDS writes of a wave are contiguous
    static __device__ __forceinline__ void load(u32x4_t (&v)[kPerThread], const T* __restrict__ k_head, int64_t j0, int64_t S, int dh) {
        constexpr int CE = Mma<T>::kChunkElems;
#pragma unroll
        for (int u = 0; u < kPerThread; ++u) {
            int id = threadIdx.x + u * kScoreThreads;
            id = id < kSlots ? id : 0;                              // surplus threads repeat piece 0 and do not store it
            const int jl = id % kKeys, p = id / kKeys;
            int64_t j = j0 + jl;
            j = j < S ? j : S - 1;                                  // stages may overhang the sequence; masked later
            // S < 2^31: one 32 x 32 -> 64 bit multiply instead of a 64-bit one in every stage
            const size_t row = static_cast<size_t>(static_cast<uint32_t>(j)) * static_cast<uint32_t>(dh);
            v[u] = *reinterpret_cast<const u32x4_t*>(k_head + row + (p / NCH) * (dh / 2) + (p % NCH) * CE);
        }
    }
    // UNCHECKED_ROUNDS: rounds in which every thread of the workgroup owns a piece skip the bounds check,
    // which keeps a branch out of the caller's loop body.
    template <bool UNCHECKED_ROUNDS = false>
    static __device__ __forceinline__ void store(const u32x4_t (&v)[kPerThread], uint4* __restrict__ kbuf) {
#pragma unroll
        for (int u = 0; u < kPerThread; ++u) {
            const int id = threadIdx.x + u * kScoreThreads;
            const int jl = id % kKeys, p = id / kKeys;
            if ((UNCHECKED_ROUNDS && (u + 1) * kScoreThreads <= kSlots) || id < kSlots)
                reinterpret_cast<u32x4_t*>(kbuf)[((jl >> 5) * NCH + (p % NCH)) * 64 + (jl & 31) + 32 * (p / NCH)] = v[u];
        }
    }
};

// Query fragments in MFMA operand order, written once per call and read by every workgroup of both passes:
//     qfrag[((kvh * rb_total + rb) * NCH + c) * 64 + lane],  row = 32 rb + lane % 32, half = lane / 32,
// 16 bytes each (elements half * dh/2 + c * CE ... of the row); rows past the last query are zero.
// A wave then fetches a fragment with one fully coalesced 1 KB load instead of 64 strided 16-byte pieces.
// As the first kernel of a call it also clears the counters and histograms of the later kernels (`clear`, n_clear words).
template <typename T, int NCH>
__global__ __launch_bounds__(256) void pack_q_kernel(const T* __restrict__ q_text, const ScoreGeom g, uint4* __restrict__ qfrag,
                                                     uint32_t* __restrict__ clear, int n_clear) {
    constexpr int CE = Mma<T>::kChunkElems;
    q_text = of_video_elems(q_text, g.q_video); qfrag = of_video(qfrag, g.ws_video); clear = of_video(clear, g.ws_video);
    const int idx = blockIdx.x * 256 + threadIdx.x;
    for (int i = idx; i < n_clear; i += gridDim.x * 256) clear[i] = 0u;
    const int total = g.Hkv * g.rb_total * NCH * 64;
    if (idx >= total) return;
    const int lane = idx & 63, c = (idx >> 6) % NCH, rbg = idx / (64 * NCH);
    const int kvh = rbg / g.rb_total, rb = rbg % g.rb_total;
    const int r = rb * 32 + (lane & 31);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (r < g.R) {
        const int hq = kvh * g.group + r / g.Tq, qi = r % g.Tq;
        v = *reinterpret_cast<const uint4*>(q_text + (static_cast<size_t>(hq) * g.Tq + qi) * g.dh + (lane >> 5) * (g.dh / 2) + c * CE);
    }
    qfrag[idx] = v;
}

// q[i][c] belongs to the wave's local row block wave + 8 i.
template <int NCH, int RBW>
__device__ __forceinline__ void load_qfrag(uint4 (&q)[RBW][NCH], const uint4* __restrict__ qfrag, const ScoreGeom& g, int kvh,
                                           int rb0, int nrb, int wave, int lane) {
#pragma unroll
    for (int i = 0; i < RBW; ++i) {
        const int rbl = wave + kScoreWaves * i;
        const bool ok = rbl < nrb;
        const uint4* src = qfrag + (static_cast<size_t>(kvh) * g.rb_total + rb0 + (ok ? rbl : 0)) * NCH * 64 + lane;
#pragma unroll
        for (int c = 0; c < NCH; ++c) q[i][c] = ok ? src[c * 64] : make_uint4(0, 0, 0, 0);
    }
}

template <typename T, int NCH>
__device__ __forceinline__ f32x16_t mma_chain(const uint4 (&a)[NCH], const uint4 (&b)[NCH]) {
    f32x16_t acc = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < NCH; ++c) acc = Mma<T>::mma(a[c], b[c], acc);
    return acc;
}

__device__ __forceinline__ float max3(float a, float b, float c) { return fmaxf(fmaxf(a, b), c); }

// Online softmax step of one lane over its 16 accumulators when every key is visible (log2 domain).
__device__ __forceinline__ void softmax_step_full(const f32x16_t& acc, float scale_log2, float& m, float& l) {
    const float t0 = max3(acc[0], acc[1], acc[2]), t1 = max3(acc[3], acc[4], acc[5]), t2 = max3(acc[6], acc[7], acc[8]),
                t3 = max3(acc[9], acc[10], acc[11]), t4 = max3(acc[12], acc[13], acc[14]);
    const float tmax = max3(max3(t0, t1, t2), max3(t3, t4, acc[15]), acc[15]);
    const float m_new = fmaxf(m, tmax * scale_log2);        // the scale is positive: max commutes with it
    float sum = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) sum += fast_exp2(fmaf(acc[e], scale_log2, -m_new));
    l = l * fast_exp2(m - m_new) + sum;
    m = m_new;
}

// Keeps the MFMA chain that produces `acc` inside the scheduling region in which it was written: the value counts as
// used (and changed) here, so the chain cannot sink towards its first real use in a later region.
__device__ __forceinline__ void pin_accumulators(f32x16_t& acc) { asm volatile("" : "+v"(acc)); }

// Asks the scheduler to place `valu` vector instructions after each of the next `mfmas` MFMAs of the
// region, so that the softmax arithmetic of one block runs while the matrix pipe works on the next block.
template <int MFMAS, int VALU>
__device__ __forceinline__ void interleave_mfma_valu() {
#pragma unroll
    for (int z = 0; z < MFMAS; ++z) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x002, VALU, 0);
    }
}

// Online softmax step of one lane over its 16 accumulators with the causal / range mask applied:
// accumulator e is key j0 + 8 (e / 4) + 4 h + e % 4 and is visible iff that offset is <= lim.
__device__ __forceinline__ void softmax_step_masked(const f32x16_t& acc, float scale_log2, int h, int lim, float& m, float& l) {
    bool vis[16];
    float tmax = kNegBig;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        vis[e] = 8 * (e >> 2) + 4 * h + (e & 3) <= lim;
        if (vis[e]) tmax = fmaxf(tmax, acc[e] * scale_log2);
    }
    const float m_new = fmaxf(m, tmax);
    float sum = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) sum += vis[e] ? fast_exp2(fmaf(acc[e], scale_log2, -m_new)) : 0.f;
    l = l * fast_exp2(m - m_new) + sum;
    m = m_new;
}

constexpr int kStageBuffers = 3;       // LDS stages: one in use, one ready (its first fragments are read early), one being filled

// ---------------------------------------------------------------------------------------------
// pass 1: blockIdx.x owns sub_per_wg consecutive 32-key subtiles of [key_begin, key_end),
// blockIdx.y = kvh * rs + split.  The product is taken as keys x queries, so a lane's 16 accumulators
// are 16 keys of ONE query row (row = lane % 32) and the online softmax state is one (max, sum) pair
// per lane and row block, in the log2 domain.
// pstat[((y * gridDim.x + x) * rbw * 32 + local_row) * 2 + {0, 1}]
//
// Key stages are fetched two ahead (global -> registers at the top of a stage, registers -> LDS at its
// end, one barrier per stage).  A wave that owns two row blocks runs the stages in which every key is
// visible to every query as one software pipeline over the blocks (subtile, row block): the MFMA chain
// of block b + 1 is interleaved with the softmax arithmetic of block b, also across the barrier, and the
// fragments of the next stage's first subtile are read from LDS as soon as their registers are free.
// Stages that need the mask, and workgroups with fewer row blocks than waves, take the plain path.
// ---------------------------------------------------------------------------------------------
template <typename T, int NCH, int RBW, int SUBS>
__global__ __launch_bounds__(kScoreThreads) void row_stats_kernel(const uint4* __restrict__ qfrag, const T* __restrict__ k_all,
                                                                  const ScoreGeom g, int sub_per_wg, float* __restrict__ pstat) {
    using Stage = KeyStage<T, NCH, SUBS>;
    extern __shared__ uint4 lds[];                      // kStageBuffers stages
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h = lane >> 5;
    const int kvh = blockIdx.y / g.rs, split = blockIdx.y % g.rs;
    const int rb0 = split * g.rbw;
    const int nrb = min(g.rbw, g.rb_total - rb0);
    const int nrb_w = nrb > wave ? (nrb - wave + kScoreWaves - 1) / kScoreWaves : 0;     // row blocks of this wave
    qfrag = of_video(qfrag, g.ws_video); pstat = of_video(pstat, g.ws_video);
    const T* k_head = of_video_elems(k_all, g.k_video) + static_cast<size_t>(kvh) * g.S * g.dh;

    const int64_t kb = g.key_begin + static_cast<int64_t>(blockIdx.x) * sub_per_wg * 32;
    const int64_t ke = min(g.key_end, kb + static_cast<int64_t>(sub_per_wg) * 32);
    const int n_stage = static_cast<int>((ke - kb + Stage::kKeys - 1) / Stage::kKeys);
    const int64_t text_start = g.S - g.Tq;
    const int64_t full_end = text_start < ke ? text_start : ke;

    // the first two key stages and the query fragments are requested together: one memory round trip
    u32x4_t kv[Stage::kPerThread], kv1[Stage::kPerThread];
    Stage::load(kv, k_head, kb, g.S, g.dh);
    Stage::load(kv1, k_head, kb + (n_stage > 1 ? Stage::kKeys : 0), g.S, g.dh);
    uint4 q[RBW][NCH];
    load_qfrag<NCH, RBW>(q, qfrag, g, kvh, rb0, nrb, wave, lane);
    float m[RBW], l[RBW];
#pragma unroll
    for (int i = 0; i < RBW; ++i) { m[i] = kNegBig; l[i] = 0.f; }
    Stage::store(kv, lds);
    if (n_stage > 1) Stage::store(kv1, lds + Stage::kSlots);
    // Every load issued so far has to land before the loop: with query loads still pending at its head the
    // first use of a fragment inside would wait for ALL outstanding loads, the prefetch of later stages included.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();

    auto stage_buf = [&](int s) { return lds + (s % kStageBuffers) * Stage::kSlots; };
    auto prefetch = [&](int s) {          // global -> registers for stage s + 2
        if (s + 2 < n_stage) Stage::load(kv, k_head, kb + static_cast<int64_t>(s + 2) * Stage::kKeys, g.S, g.dh);
    };
    auto publish = [&](int s) {           // registers -> LDS; that buffer was last read before the previous barrier
        if (s + 2 < n_stage) Stage::store(kv, stage_buf(s + 2));
        __syncthreads();
    };

    int s = 0;
    if constexpr (RBW == 2 && SUBS == 2) {
        // leading stages whose 64 keys are all visible to every query
        // The choice is the same for every wave of the workgroup (all waves must meet at the same barriers):
        // with at least one row block per wave, waves that own a single block run the second chain on the
        // zero fragments load_qfrag gave them; its statistics belong to a padding row and are ignored.
        int n_fast = 0;
        if (nrb >= kScoreWaves) {
            const int64_t f = (full_end - kb) / Stage::kKeys;
            n_fast = f < 0 ? 0 : (f > n_stage ? n_stage : static_cast<int>(f));
        }
        if (n_fast > 0) {
            constexpr int kMfmas = NCH * Mma<T>::kMfmaPerChunk;
            constexpr int kValu = (64 + kMfmas - 1) / kMfmas;
            uint4 kf0[NCH], kf1[NCH];
#pragma unroll
            for (int c = 0; c < NCH; ++c) kf0[c] = lds[c * 64 + lane];
            f32x16_t A = mma_chain<T, NCH>(kf0, q[0]), B;
            // The body is branch-free so that the whole stage is one scheduling region: loads and stores
            // that a conditional would skip are done anyway on clamped addresses (a stage is fetched twice,
            // a free buffer is overwritten, the chain started for a stage that is not fast is dropped).
            for (; s < n_fast; ++s) {
                const uint4* kbuf = stage_buf(s);
                const int s2 = s + 2 < n_stage ? s + 2 : n_stage - 1;
                Stage::load(kv, k_head, kb + static_cast<int64_t>(s2) * Stage::kKeys, g.S, g.dh);
#pragma unroll
                for (int c = 0; c < NCH; ++c) kf1[c] = kbuf[(NCH + c) * 64 + lane];
                __builtin_amdgcn_sched_barrier(0);
                B = mma_chain<T, NCH>(kf0, q[1]);
                softmax_step_full(A, g.scale_log2, m[0], l[0]);
                interleave_mfma_valu<kMfmas, kValu>();
                pin_accumulators(B);
                __builtin_amdgcn_sched_barrier(0);
                {   // subtile 0 of the next stage: published before the previous barrier
                    const uint4* knext = stage_buf(s + 1);
#pragma unroll
                    for (int c = 0; c < NCH; ++c) kf0[c] = knext[c * 64 + lane];
                }
                __builtin_amdgcn_sched_barrier(0);
                A = mma_chain<T, NCH>(kf1, q[0]);
                softmax_step_full(B, g.scale_log2, m[1], l[1]);
                interleave_mfma_valu<kMfmas, kValu>();
                pin_accumulators(A);
                __builtin_amdgcn_sched_barrier(0);
                B = mma_chain<T, NCH>(kf1, q[1]);
                softmax_step_full(A, g.scale_log2, m[0], l[0]);
                interleave_mfma_valu<kMfmas, kValu>();
                pin_accumulators(B);
                __builtin_amdgcn_sched_barrier(0);
                Stage::template store<true>(kv, stage_buf(s + 2));
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
                A = mma_chain<T, NCH>(kf0, q[0]);
                softmax_step_full(B, g.scale_log2, m[1], l[1]);
                interleave_mfma_valu<kMfmas, kValu>();
                pin_accumulators(A);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    for (; s < n_stage; ++s) {
        const uint4* kbuf = stage_buf(s);
        const int64_t js = kb + static_cast<int64_t>(s) * Stage::kKeys;
        prefetch(s);
#pragma unroll
        for (int sub = 0; sub < SUBS; ++sub) {
            const int64_t j0 = js + sub * 32;
            if (j0 < ke && nrb_w > 0) {
                uint4 kf[NCH];
#pragma unroll
                for (int c = 0; c < NCH; ++c) kf[c] = kbuf[(sub * NCH + c) * 64 + lane];
                const bool full = j0 + 32 <= full_end;      // every key of the subtile is visible to every query
#pragma unroll
                for (int i = 0; i < RBW; ++i) {
                    if (i < nrb_w) {
                        const f32x16_t acc = mma_chain<T, NCH>(kf, q[i]);
                        if (full) {
                            softmax_step_full(acc, g.scale_log2, m[i], l[i]);
                        } else {
                            const int r = (rb0 + wave + kScoreWaves * i) * 32 + (lane & 31);
                            int64_t last = text_start + (r % g.Tq);            // causal: keys 0..last, and below ke
                            last = last < ke - 1 ? last : ke - 1;
                            const int64_t d = last - j0;
                            const int lim = d < 0 ? -1 : (d > 31 ? 31 : static_cast<int>(d));
                            softmax_step_masked(acc, g.scale_log2, h, lim, m[i], l[i]);
                        }
                    }
                }
            }
        }
        publish(s);
    }
    // the two lane halves hold different keys of the same row
    const int rows_per_y = g.rbw * 32;
#pragma unroll
    for (int i = 0; i < RBW; ++i) {
        const int rbl = wave + kScoreWaves * i;
        if (rbl < g.rbw) {
            const float m2 = __shfl_xor(m[i], 32, 64), l2 = __shfl_xor(l[i], 32, 64);
            const float mm = fmaxf(m[i], m2);
            const float ll = l[i] * fast_exp2(m[i] - mm) + l2 * fast_exp2(m2 - mm);
            if (h == 0) {
                float* dst = pstat + ((static_cast<size_t>(blockIdx.y) * gridDim.x + blockIdx.x) * rows_per_y + rbl * 32 + lane) * 2;
                dst[0] = mm;
                dst[1] = ll;
            }
        }
    }
}

// norm[y * rbw * 32 + local_row] = log2-domain normaliser max + log2(sum) of the row (+big for padding rows).
// Sixteen lanes share a row: each merges every 16th partial, then the lanes are merged pairwise.
__global__ __launch_bounds__(256) void merge_stats_kernel(const float* __restrict__ pstat, const ScoreGeom g, int nx,
                                                          float* __restrict__ norm) {
    const int rows_per_y = g.rbw * 32;
    const int total = g.Hkv * g.rs * rows_per_y;
    pstat = of_video(pstat, g.ws_video); norm = of_video(norm, g.ws_video);
    const int i = blockIdx.x * 16 + (threadIdx.x >> 4);
    const int p = threadIdx.x & 15;
    float mm = kNegBig, ll = 0.f;
    int y = 0, lr = 0;
    if (i < total) {
        y = i / rows_per_y; lr = i % rows_per_y;
        for (int x = p; x < nx; x += 16) {
            const float* src = pstat + ((static_cast<size_t>(y) * nx + x) * rows_per_y + lr) * 2;
            const float m2 = src[0], l2 = src[1];
            const float mx = fmaxf(mm, m2);
            ll = ll * fast_exp2(mm - mx) + l2 * fast_exp2(m2 - mx);
            mm = mx;
        }
    }
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) {
        const float m2 = __shfl_xor(mm, off, 16), l2 = __shfl_xor(ll, off, 16);
        const float mx = fmaxf(mm, m2);
        ll = ll * fast_exp2(mm - mx) + l2 * fast_exp2(m2 - mx);
        mm = mx;
    }
    if (i < total && p == 0) {
        const int r = (y % g.rs) * rows_per_y + lr;
        norm[i] = (r < g.R && ll > 0.f) ? mm + log2f(ll) : kPosBig;
    }
}

// ---------------------------------------------------------------------------------------------
// pass 2: queries x keys, a lane's 16 accumulators are 16 rows of ONE key (key = lane % 32), and the
// normalisers of those rows stay in registers.  blockIdx.x owns sub_per_wg consecutive subtiles of the
// visual keys.  The eight per-wave partial column sums of a stage are added in wave order through LDS.
// colpart[y * n_vis + j] = sum over the rows of workgroup-row y of the probability of visual key j.
// ---------------------------------------------------------------------------------------------
template <typename T, int NCH, int RBW, int SUBS>
__global__ __launch_bounds__(kScoreThreads) void col_sums_kernel(const uint4* __restrict__ qfrag, const T* __restrict__ k_all,
                                                                 const ScoreGeom g, int sub_per_wg, const float* __restrict__ norm,
                                                                 float* __restrict__ colpart) {
    using Stage = KeyStage<T, NCH, SUBS>;
    extern __shared__ uint4 lds[];                      // two stages, then the column partials [2][waves][stage keys]
    float* cs = reinterpret_cast<float*>(lds + 2 * Stage::kSlots);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, h = lane >> 5;
    const int kvh = blockIdx.y / g.rs, split = blockIdx.y % g.rs;
    const int rb0 = split * g.rbw;
    const int nrb = min(g.rbw, g.rb_total - rb0);
    const int nrb_w = nrb > wave ? (nrb - wave + kScoreWaves - 1) / kScoreWaves : 0;
    qfrag = of_video(qfrag, g.ws_video); norm = of_video(norm, g.ws_video); colpart = of_video(colpart, g.ws_video);
    const T* k_head = of_video_elems(k_all, g.k_video) + static_cast<size_t>(kvh) * g.S * g.dh;

    const int vb = blockIdx.x * sub_per_wg * 32;                       // visual keys [vb, ve) of this workgroup
    const int ve = min(g.n_vis, vb + sub_per_wg * 32);
    const int n_stage = (ve - vb + Stage::kKeys - 1) / Stage::kKeys;
    u32x4_t kv[Stage::kPerThread];
    Stage::load(kv, k_head, static_cast<int64_t>(g.vis_start) + vb, g.S, g.dh);

    uint4 q[RBW][NCH];
    load_qfrag<NCH, RBW>(q, qfrag, g, kvh, rb0, nrb, wave, lane);
    // accumulator e <-> query row 32 rbl + 8 (e / 4) + 4 h + e % 4
    float cr[RBW][16];
#pragma unroll
    for (int i = 0; i < RBW; ++i) {
        const int rbl = wave + kScoreWaves * i;
        const float* src = norm + static_cast<size_t>(blockIdx.y) * g.rbw * 32 + (rbl < g.rbw ? rbl : 0) * 32 + 4 * h;
#pragma unroll
        for (int b4 = 0; b4 < 4; ++b4) {
            const float4 c4 = *reinterpret_cast<const float4*>(src + 8 * b4);
            cr[i][4 * b4 + 0] = c4.x; cr[i][4 * b4 + 1] = c4.y; cr[i][4 * b4 + 2] = c4.z; cr[i][4 * b4 + 3] = c4.w;
        }
    }
    Stage::store(kv, lds);
    __builtin_amdgcn_s_waitcnt(0);      // queries and normalisers have landed: see row_stats_kernel
    __syncthreads();
    for (int s = 0; s < n_stage; ++s) {
        const uint4* kbuf = lds + (s & 1) * Stage::kSlots;
        float* csb = cs + (s & 1) * (kScoreWaves * Stage::kKeys);
        const int vs = vb + s * Stage::kKeys;
        if (s + 1 < n_stage) Stage::load(kv, k_head, static_cast<int64_t>(g.vis_start) + vs + Stage::kKeys, g.S, g.dh);
#pragma unroll
        for (int sub = 0; sub < SUBS; ++sub) {
            if (vs + sub * 32 < ve) {
                float colsum = 0.f;
                if (nrb_w > 0) {
                    uint4 kf[NCH];
#pragma unroll
                    for (int c = 0; c < NCH; ++c) kf[c] = kbuf[(sub * NCH + c) * 64 + lane];
#pragma unroll
                    for (int i = 0; i < RBW; ++i) {
                        if (i < nrb_w) {
                            const f32x16_t acc = mma_chain<T, NCH>(q[i], kf);
#pragma unroll
                            for (int e = 0; e < 16; ++e) colsum += fast_exp2(fmaf(acc[e], g.scale_log2, -cr[i][e]));
                        }
                    }
                    colsum += __shfl_xor(colsum, 32, 64);
                }
                if (h == 0) csb[wave * Stage::kKeys + sub * 32 + lane] = colsum;
            }
        }
        if (s + 1 < n_stage) Stage::store(kv, lds + ((s + 1) & 1) * Stage::kSlots);
        __syncthreads();
        if (threadIdx.x < Stage::kKeys) {
            const int j = vs + threadIdx.x;
            if (j < ve) {
                float a = 0.f;
#pragma unroll
                for (int w = 0; w < kScoreWaves; ++w) a += csb[w * Stage::kKeys + threadIdx.x];
                colpart[static_cast<size_t>(blockIdx.y) * g.n_vis + j] = a;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// scores, selection, scan, gather
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void prepare_kernel(const float* __restrict__ colpart, int n_parts, int n_vis, float rows_total,
                                                      const int32_t* __restrict__ token_event, const float* __restrict__ event_weight,
                                                      int n_events, float* __restrict__ scores, int64_t ws_video) {
    colpart = of_video(colpart, ws_video); token_event = of_video_elems(token_event, n_vis);
    event_weight = of_video_elems(event_weight, n_events); scores = of_video_elems(scores, n_vis);
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n_vis) return;
    float a = 0.f;
    for (int p = 0; p < n_parts; ++p) a += colpart[static_cast<size_t>(p) * n_vis + j];
    a = a / rows_total;
    if (event_weight) {
        int e = token_event[j];
        e = e < 0 ? 0 : (e >= n_events ? n_events - 1 : e);
        a *= event_weight[e];
    }
    scores[j] = a;
}

struct Quotas { int32_t q[METOK_MAX_SEGMENTS]; };

constexpr int kSelThreads = 1024;      // also the tile size of the selection: tile i = tokens [1024 i, 1024 i + 1024)
constexpr int kSelCache = 40;          // keys per thread held in registers (n_vis <= 40960)
constexpr int kSelCand = 4096;         // candidates kept in an LDS list once the first digit is fixed

// One workgroup per retention class.  Radix select of the quota-th largest key of the class: digits of up
// to 11 bits, starting at the highest bit in which the keys of the class differ.  Outputs: the threshold
// key tau and the number of tokens equal to tau that are still kept (sel_info[2 seg], [2 seg + 1];
// 0x7fffffff = every one), and per 1024-token tile the number of class members above tau (gt_count) and
// equal to it (eq_count).  The keep rule itself -- above tau, or equal and among the first `remaining`
// equal ones by index -- is applied by write_index_kernel.
// Thread t owns tokens t, t + 1024, ... (token i of a thread lies in tile i); with CACHED their keys stay
// in registers.  Attention scores share their top key bits, so a thread aggregates runs of equal digits
// before touching the LDS histogram, and once the first digit is fixed the remaining candidates (if at
// most kSelCand) move to an LDS list for the other digits.
template <bool CACHED>
__global__ __launch_bounds__(kSelThreads) void select_kernel(const float* __restrict__ scores, const int32_t* __restrict__ token_seg,
                                                             int n_vis, int n_tiles, const Quotas quotas,
                                                             int32_t* __restrict__ gt_count, int32_t* __restrict__ eq_count,
                                                             uint32_t* __restrict__ sel_info) {
    __shared__ int hist[2 * kSelThreads];      // 2048 bins: one 11-bit digit
    __shared__ int scan_scratch[17];
    __shared__ int s_digit, s_remaining, s_count, s_ncand;
    __shared__ uint32_t s_or, s_and;
    __shared__ uint32_t cand[kSelCand];
    __shared__ int cnt[2][64];
    const int seg = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int quota = quotas.q[seg];
    int32_t* my_gt = gt_count + static_cast<size_t>(seg) * n_tiles;
    int32_t* my_eq = eq_count + static_cast<size_t>(seg) * n_tiles;

    uint32_t key[CACHED ? kSelCache : 1];
    uint64_t member = 0;
    int mine = 0;
    if (CACHED) {
        // unconditional, clamped loads first so that all of them are in flight together
        int sv[kSelCache];
#pragma unroll
        for (int i = 0; i < kSelCache; ++i) {
            const int j = min(tid + i * kSelThreads, n_vis - 1);
            sv[i] = token_seg[j];
            key[i] = __float_as_uint(scores[j]);
        }
#pragma unroll
        for (int i = 0; i < kSelCache; ++i) {
            key[i] = ordered_key(__uint_as_float(key[i]));
            if (tid + i * kSelThreads < n_vis && sv[i] == seg) member |= 1ull << i;
        }
        mine = __popcll(member);
    } else {
        for (int i = 0; i < n_tiles; ++i) {
            const int j = tid + i * kSelThreads;
            mine += (j < n_vis && token_seg[j] == seg) ? 1 : 0;
        }
    }
    // f(key) for every token of the class owned by this thread
    auto for_each_key = [&](auto&& f) {
        if (CACHED) {
#pragma unroll
            for (int i = 0; i < kSelCache; ++i)
                if (member & (1ull << i)) f(key[i]);
        } else {
            for (int i = 0; i < n_tiles; ++i) {
                const int j = tid + i * kSelThreads;
                if (j < n_vis && token_seg[j] == seg) f(ordered_key(scores[j]));
            }
        }
    };
    if (tid == 0) { s_digit = 0; s_remaining = 0; s_count = 0; s_ncand = 0; s_or = 0u; s_and = 0xffffffffu; }
    int pop = 0;
    block_exclusive_scan(mine, scan_scratch, &pop);
    // bits on which the keys of the class differ: the radix digits start at the highest of them, so that the
    // first digit already separates scores that share sign, exponent and leading mantissa bits
    {
        uint32_t o = 0u, a = 0xffffffffu;
        for_each_key([&](uint32_t k) { o |= k; a &= k; });
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) { o |= __shfl_xor(o, off, 64); a &= __shfl_xor(a, off, 64); }
        if (lane == 0) { atomicOr(&s_or, o); atomicAnd(&s_and, a); }
        __syncthreads();
    }

    // keep rule: key > tau, or key == tau and fewer than `remaining` equal keys of the class precede the token
    uint32_t tau = 0;
    int remaining = 0x7fffffff;
    if (quota <= 0) {
        tau = 0xffffffffu; remaining = 0;                 // nothing is kept
    } else if (quota < pop) {
        const uint32_t differ = s_or ^ s_and;
        const int width = differ ? 32 - __clz(differ) : 0;             // the low `width` bits vary, the rest is common
        uint32_t prefix = width >= 32 ? 0u : (s_and & (0xffffffffu << width));
        int count_equal = pop;                                          // width 0: all keys are equal
        remaining = quota;
        bool use_list = false;
        // digits of up to 11 bits from the highest differing bit down (at most three rounds)
        for (int top = width; top > 0; top -= 11) {
            const int bits = top < 11 ? top : 11;
            const int shift = top - bits;
            const int bins = 1 << bits;
            const uint32_t dmask = static_cast<uint32_t>(bins - 1);
            const uint32_t hi_mask = top >= 32 ? 0u : (0xffffffffu << top);
            hist[tid] = 0; hist[tid + kSelThreads] = 0;
            __syncthreads();
            if (use_list) {
                for (int c = tid; c < s_ncand; c += kSelThreads) {
                    const uint32_t k = cand[c];
                    if ((k & hi_mask) == prefix) atomicAdd(&hist[(k >> shift) & dmask], 1);
                }
            } else {
                int run_digit = -1, run_count = 0;
                for_each_key([&](uint32_t k) {
                    if ((k & hi_mask) == prefix) {
                        const int d = static_cast<int>((k >> shift) & dmask);
                        if (d == run_digit) ++run_count;
                        else {
                            if (run_count) atomicAdd(&hist[run_digit], run_count);
                            run_digit = d; run_count = 1;
                        }
                    }
                });
                if (run_count) atomicAdd(&hist[run_digit], run_count);
            }
            __syncthreads();
            // thread t looks at digits bins-1-2t and bins-2-2t; exclusive scan = keys with a larger digit
            const int d0 = bins - 1 - 2 * tid, d1 = d0 - 1;
            const int v0 = d0 >= 0 ? hist[d0] : 0, v1 = d1 >= 0 ? hist[d1] : 0;
            int total = 0;
            const int excl = block_exclusive_scan(v0 + v1, scan_scratch, &total);
            if (excl < remaining && excl + v0 >= remaining) {
                s_digit = d0; s_remaining = remaining - excl; s_count = v0;
            } else if (excl + v0 < remaining && excl + v0 + v1 >= remaining) {
                s_digit = d1; s_remaining = remaining - excl - v0; s_count = v1;
            }
            __syncthreads();
            prefix |= static_cast<uint32_t>(s_digit) << shift;
            remaining = s_remaining;
            count_equal = s_count;
            if (!use_list && shift > 0 && count_equal <= kSelCand) {
                // the keys that still match move to the LDS list for the remaining digits
                const uint32_t fixed = 0xffffffffu << shift;
                for_each_key([&](uint32_t k) {
                    if ((k & fixed) == prefix) cand[atomicAdd(&s_ncand, 1)] = k;
                });
                use_list = true;
            }
            __syncthreads();
        }
        tau = prefix;
        if (remaining >= count_equal) remaining = 0x7fffffff;      // every token equal to the threshold is kept
    }

    if (tid == 0) {
        sel_info[2 * seg] = tau;
        sel_info[2 * seg + 1] = static_cast<uint32_t>(remaining);
    }
    // per-tile counts, tiles in groups of 64: lane i of a wave keeps the wave's counts of tile g0 + i
    for (int g0 = 0; g0 < n_tiles; g0 += 64) {
        if (tid < 128) cnt[tid >> 6][tid & 63] = 0;
        __syncthreads();
        const int g1 = min(n_tiles, g0 + 64);
        int my_gt_count = 0, my_eq_count = 0;
        auto tile_body = [&](int i, bool is_member, uint32_t k) {
            const unsigned long long gt = __ballot(is_member && k > tau), eq = __ballot(is_member && k == tau);
            if (lane == i - g0) { my_gt_count = __popcll(gt); my_eq_count = __popcll(eq); }
        };
        if (CACHED) {
#pragma unroll
            for (int i = 0; i < kSelCache; ++i)
                if (i >= g0 && i < g1) tile_body(i, (member >> i) & 1ull, key[i]);
        } else {
            for (int i = g0; i < g1; ++i) {
                const int j = tid + i * kSelThreads;
                const bool is_member = j < n_vis && token_seg[j] == seg;
                tile_body(i, is_member, is_member ? ordered_key(scores[j]) : 0u);
            }
        }
        if (my_gt_count) atomicAdd(&cnt[0][lane], my_gt_count);
        if (my_eq_count) atomicAdd(&cnt[1][lane], my_eq_count);
        __syncthreads();
        if (tid < g1 - g0) { my_gt[g0 + tid] = cnt[0][tid]; my_eq[g0 + tid] = cnt[1][tid]; }
        __syncthreads();
    }
}

// One workgroup per 1024-token tile: applies the keep rule (key above the class threshold, or equal to it and
// among the first `remaining` equal keys of the class by index), finds the position of the tile's first kept
// token from the per-class tile counts, and writes the kept index list and carried metadata in ascending order.
constexpr int kIdxThreads = 256;

__global__ __launch_bounds__(kIdxThreads) void write_index_kernel(
    const float* __restrict__ scores, const uint32_t* __restrict__ sel_info, const int32_t* __restrict__ gt_count,
    const int32_t* __restrict__ eq_count, const int32_t* __restrict__ token_seg,
    int n_vis, int n_seg, int n_tiles, int total_keep, const int32_t* __restrict__ token_event,
    const int32_t* __restrict__ orig_idx_in, int32_t* __restrict__ kept_idx, int32_t* __restrict__ token_seg_out,
    int32_t* __restrict__ token_event_out, int32_t* __restrict__ orig_idx_out,
    const int32_t* __restrict__ given_tile_off, const int32_t* __restrict__ given_eq_before /*[class][kSelCache]*/,
    int64_t ws_video, int64_t keep_stride, int64_t orig_idx_in_stride, int64_t orig_idx_stride, const BatchKeep keeps) {
    __shared__ int scan_scratch[17];
    __shared__ uint32_t s_tau[METOK_MAX_SEGMENTS];
    __shared__ int s_rem[METOK_MAX_SEGMENTS], s_eq_before[METOK_MAX_SEGMENTS];
    __shared__ int tie_seg[kSelThreads];
    const int tile = blockIdx.x, tid = threadIdx.x;
    total_keep = keeps.n[blockIdx.z];
    scores = of_video_elems(scores, n_vis); token_seg = of_video_elems(token_seg, n_vis);
    token_event = of_video_elems(token_event, n_vis); orig_idx_in = of_video_elems(orig_idx_in, orig_idx_in_stride);
    sel_info = of_video(sel_info, ws_video); gt_count = of_video(gt_count, ws_video); eq_count = of_video(eq_count, ws_video);
    given_tile_off = of_video(given_tile_off, ws_video); given_eq_before = of_video(given_eq_before, ws_video);
    kept_idx = of_video_elems(kept_idx, keep_stride); token_seg_out = of_video_elems(token_seg_out, keep_stride);
    token_event_out = of_video_elems(token_event_out, keep_stride); orig_idx_out = of_video_elems(orig_idx_out, orig_idx_stride);
    // kept tokens in earlier tiles: given by the fast path, else thread s walks the tiles of class s
    int before = 0;
    if (given_tile_off != nullptr) {
        for (int sg = tid; sg < n_seg; sg += kIdxThreads) {
            s_tau[sg] = sel_info[2 * sg]; s_rem[sg] = static_cast<int>(sel_info[2 * sg + 1]);
            s_eq_before[sg] = given_eq_before[sg * kSelCache + tile];
        }
        if (tid == 0) before = given_tile_off[tile];
    } else
    for (int sg = tid; sg < n_seg; sg += kIdxThreads) {
        const uint32_t tau = sel_info[2 * sg];
        const int rem = static_cast<int>(sel_info[2 * sg + 1]);
        int eqcum = 0;
        for (int t = 0; t < tile; ++t) {
            const int eq = eq_count[static_cast<size_t>(sg) * n_tiles + t];
            const int room = rem > eqcum ? rem - eqcum : 0;
            before += gt_count[static_cast<size_t>(sg) * n_tiles + t] + (eq < room ? eq : room);
            eqcum += eq;
        }
        s_tau[sg] = tau; s_rem[sg] = rem; s_eq_before[sg] = eqcum;
    }
    int tile_off = 0;
    block_exclusive_scan(before, scan_scratch, &tile_off);      // its barriers also publish the tables above
    // four consecutive tokens per thread
    const int j0 = tile * kSelThreads + tid * 4;
    bool keep[4], tie[4];
    int sv[4];
    bool any_tie = false;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int j = min(j0 + u, n_vis - 1);
        sv[u] = token_seg[j];
        const uint32_t key = ordered_key(scores[j]);
        const bool ok = (j0 + u < n_vis) && sv[u] >= 0 && sv[u] < n_seg;
        const int sg = ok ? sv[u] : 0;
        keep[u] = ok && key > s_tau[sg];
        tie[u] = ok && key == s_tau[sg];
        if (tie[u] && s_rem[sg] == 0x7fffffff) { keep[u] = true; tie[u] = false; }      // every equal key is kept
        if (tie[u] && s_rem[sg] <= s_eq_before[sg]) tie[u] = false;                      // the equal keys kept lie in earlier tiles
        any_tie = any_tie || tie[u];
        tie_seg[tid * 4 + u] = tie[u] ? sg : -1;
    }
    if (__syncthreads_or(any_tie ? 1 : 0)) {
        // rank of an undecided equal key among the equal keys of its class (ties are rare; the walk is short)
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (tie[u]) {
                int rank = s_eq_before[sv[u]];
                for (int q = 0; q < tid * 4 + u; ++q) rank += tie_seg[q] == sv[u] ? 1 : 0;
                keep[u] = rank < s_rem[sv[u]];
            }
        }
    }
    int mine = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) mine += keep[u] ? 1 : 0;
    int total = 0;
    int pos = tile_off + block_exclusive_scan(mine, scan_scratch, &total);
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        if (keep[u]) {
            const int j = j0 + u;
            if (pos < total_keep) {
                kept_idx[pos] = j;
                if (token_seg_out) token_seg_out[pos] = sv[u];
                if (token_event_out) token_event_out[pos] = token_event[j];
                if (orig_idx_out) orig_idx_out[pos] = orig_idx_in ? orig_idx_in[j] : j;
            }
            ++pos;
        }
    }
    // fewer survivors than announced (a quota above its class population): the last tile pads the tail so
    // that the gather stays in bounds
    if (tile == n_tiles - 1) {
        for (int p = tile_off + total + tid; p < total_keep; p += kIdxThreads) {
            kept_idx[p] = 0;
            if (token_seg_out) token_seg_out[p] = 0;
            if (token_event_out) token_event_out[p] = 0;
            if (orig_idx_out) orig_idx_out[p] = 0;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Fast selection path: at most kFastSeg retention classes and at most kFastTiles tiles of 1024 tokens.
// The single-workgroup radix select above costs 20-25 us at 36864 tokens, most of it barriers of a 1024-thread
// workgroup; here the token-parallel parts run on one workgroup per tile and only the short serial parts run
// on the workgroup that arrives last at an atomic counter (it is the one that knows every other workgroup's
// results are complete; nobody waits for anybody):
//   score_hist_kernel   per tile: scores (what prepare_kernel does on the general path), histogram of the top 11 key bits per class
//                       -> global histogram.  Last workgroup: per class the histogram bucket that holds the
//                       quota-th largest key, how many keys of that bucket are still needed, or keep all / none.
//   candidate_kernel    per tile: tokens above the bucket are kept for sure (counted per tile), tokens inside it are
//                       appended to a candidate list.  Last workgroup: radix select of the remaining 21 bits on the
//                       list -> class threshold and number of equal keys kept; per tile the candidates above / equal
//                       to it; exclusive sums over the tiles -> output offset of every tile.
//   write_index_kernel  per tile, as before, with the offsets given.
// Results are the same integers as on the general path: the keep rule (key above the threshold, or equal and among
// the first equal keys by index) does not depend on how the threshold was found.
// ---------------------------------------------------------------------------------------------
constexpr int kFastSeg = 4;
constexpr int kFastTiles = kSelCache;
static_assert(kFastTiles <= 64, "the finishing workgroup scans the tiles with one wave, a lane per tile");
constexpr uint32_t kKeepAll = 0x7fffffffu;

struct FastSel {
    // cleared before the first kernel that uses them
    uint32_t arrive_a, arrive_b, cand_total, pad;
    int32_t hist[kFastSeg][2048];
    // written before they are read
    int32_t state[kFastSeg][4];             // bucket digit, keys of the bucket still needed, bucket population, mode
    int32_t tile_sure[kFastSeg][kFastTiles];
    int32_t tile_off[kFastTiles];
    int32_t eq_before[kFastSeg][kFastTiles];
    uint32_t sel_info[kFastSeg][2];         // threshold key, equal keys kept (kKeepAll = every one)
};
constexpr int kFastClearWords = 4 + kFastSeg * 2048;
static size_t fast_state_bytes() { return round_up(sizeof(FastSel), 256); }
enum { kModeSearch = 0, kModeNone = 1, kModeAll = 2 };

struct FastArgs {
    FastSel* fs;
    uint32_t* cand_key;                     // [n_vis]
    uint32_t* cand_tok;                     // [n_vis]: class << 24 | token
    const float* colpart;                   // NULL: scores are given
    int n_parts;
    float rows_total;
    const int32_t* token_event;
    const float* event_weight;
    int n_events;
    float* scores;
    const int32_t* token_seg;
    int n_vis, n_seg;
    int64_t ws_video;                       // bytes between the workspaces of consecutive videos
    int32_t quota[METOK_MAX_BATCH][kFastSeg];
};
// The arguments as video blockIdx.z sees them: its pointers and the scalars; the quota table stays in the kernel
// arguments (a private copy of it would live in scratch memory).
struct FastView {
    FastSel* fs;
    uint32_t* cand_key;
    uint32_t* cand_tok;
    const float* colpart;
    int n_parts;
    float rows_total;
    const int32_t* token_event;
    const float* event_weight;
    int n_events;
    float* scores;
    const int32_t* token_seg;
    int n_vis, n_seg;
};
__device__ __forceinline__ FastView to_video(const FastArgs& a) {
    FastView v;
    v.fs = of_video(a.fs, a.ws_video); v.cand_key = of_video(a.cand_key, a.ws_video); v.cand_tok = of_video(a.cand_tok, a.ws_video);
    v.colpart = of_video(a.colpart, a.ws_video);
    v.n_parts = a.n_parts; v.rows_total = a.rows_total; v.n_events = a.n_events; v.n_vis = a.n_vis; v.n_seg = a.n_seg;
    v.token_event = of_video_elems(a.token_event, a.n_vis); v.event_weight = of_video_elems(a.event_weight, a.n_events);
    v.scores = of_video_elems(a.scores, a.n_vis); v.token_seg = of_video_elems(a.token_seg, a.n_vis);
    return v;
}

// Values handed from one workgroup to another inside a kernel travel through device-scope accesses (they pass the
// caches that are not coherent between the chip's dies), so that no whole-cache write-back or invalidate is needed:
// the writers store, wait until their stores have completed, meet at a barrier and count their arrival; the workgroup
// that arrives last loads.
template <typename V> __device__ __forceinline__ void store_shared_between_workgroups(V* p, V v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename V> __device__ __forceinline__ V load_shared_between_workgroups(const V* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Called by every thread of the workgroup after its last store: true in the workgroup that arrives last of gridDim.x.
__device__ __forceinline__ bool arrive_and_check_last(uint32_t* counter, int* s_flag) {
    __builtin_amdgcn_s_waitcnt(0);          // this thread's stores and atomics have completed
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t ticket = __hip_atomic_fetch_add(counter, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *s_flag = ticket == gridDim.x - 1 ? 1 : 0;
    }
    __syncthreads();
    return *s_flag != 0;
}

__global__ __launch_bounds__(256) void clear_words_kernel(uint32_t* __restrict__ words, int n, int64_t ws_video) {
    words = of_video(words, ws_video);
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) words[i] = 0u;
}

// Orders the LDS traffic of one wave's lanes among themselves: LDS serves a wave's instructions in issue order, so
// only the compiler has to be kept from moving accesses across this point.
__device__ __forceinline__ void wave_sync() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// One wave walks a histogram in LDS from the largest digit down and returns the digit at which the running count
// reaches `need`, how many keys of that digit are still needed and how many keys the digit holds.  bins is 1024 or 2048.
__device__ __forceinline__ void wave_find_bucket(const int* hist, int bins, int need, int* digit, int* rem, int* cnt) {
    const int lane = threadIdx.x & 63;
    const int per = bins / 64;
    const int hi = bins - 1 - lane * per;                          // the largest digit of this lane
    int mine_sum = 0;
    for (int u = 0; u < per; ++u) mine_sum += hist[hi - u];
    int incl = mine_sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(incl, off, 64);
        if (lane >= off) incl += up;
    }
    const int excl = incl - mine_sum;
    const bool mine = excl < need && incl >= need;
    int d = 0, r = 0, c = 0;
    if (mine) {
        int run = excl;
        for (int u = 0; u < per; ++u) {
            const int v = hist[hi - u];
            if (run + v >= need) { d = hi - u; r = need - run; c = v; break; }
            run += v;
        }
    }
    const unsigned long long m = __ballot(mine);
    const int src = m ? __ffsll(static_cast<long long>(m)) - 1 : 0;
    *digit = __shfl(d, src, 64); *rem = __shfl(r, src, 64); *cnt = __shfl(c, src, 64);
}
// population of a histogram (one wave)
__device__ __forceinline__ int wave_hist_total(const int* hist, int bins) {
    const int lane = threadIdx.x & 63;
    int s = 0;
    for (int i = lane; i < bins; i += 64) s += hist[i];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off, 64);
    return s;
}

__global__ __launch_bounds__(kSelThreads) void score_hist_kernel(const FastArgs args) {
    __shared__ int hist[kFastSeg * 2048];
    __shared__ int s_last;
    const FastView a = to_video(args);
    const int tid = threadIdx.x;
    const int j = blockIdx.x * kSelThreads + tid;
    for (int i = tid; i < a.n_seg * 2048; i += kSelThreads) hist[i] = 0;
    float sc = 0.f;
    int sg = -1;
    if (j < a.n_vis) {
        if (a.colpart) {
            // the partial sums of the workgroup rows, added in order; four loads are requested together (a part past the
            // last one reads the last one again and is not added)
            float acc = 0.f;
            for (int p0 = 0; p0 < a.n_parts; p0 += 4) {
                float v[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int p = p0 + u < a.n_parts ? p0 + u : a.n_parts - 1;
                    v[u] = a.colpart[static_cast<size_t>(p) * a.n_vis + j];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) acc += p0 + u < a.n_parts ? v[u] : 0.f;
            }
            acc = acc / a.rows_total;
            if (a.event_weight) {
                int e = a.token_event[j];
                e = e < 0 ? 0 : (e >= a.n_events ? a.n_events - 1 : e);
                acc *= a.event_weight[e];
            }
            sc = acc;
            a.scores[j] = sc;
        } else {
            sc = a.scores[j];
        }
        const int s = a.token_seg[j];
        sg = (s >= 0 && s < a.n_seg) ? s : -1;
    }
    const uint32_t key = ordered_key(sc);
    __syncthreads();
    if (sg >= 0) atomicAdd(&hist[sg * 2048 + (key >> 21)], 1);
    __syncthreads();
    int32_t* ghist = &a.fs->hist[0][0];
    for (int i = tid; i < a.n_seg * 2048; i += kSelThreads) {
        const int v = hist[i];
        if (v) atomicAdd(&ghist[i], v);
    }
    if (!arrive_and_check_last(&a.fs->arrive_a, &s_last)) return;
    // last workgroup: the complete histograms come back into LDS, then one wave finds every class's bucket (no more barriers)
    {
        constexpr int kPer = kFastSeg * 2048 / kSelThreads;
        int32_t h[kPer];
#pragma unroll
        for (int u = 0; u < kPer; ++u) h[u] = load_shared_between_workgroups(&ghist[tid + u * kSelThreads]);      // the block holds kFastSeg rows
#pragma unroll
        for (int u = 0; u < kPer; ++u) hist[tid + u * kSelThreads] = h[u];
    }
    __syncthreads();
    if (tid >= 64) return;
    for (int c = 0; c < a.n_seg; ++c) {
        const int quota = args.quota[blockIdx.z][c];
        const int pop = wave_hist_total(hist + c * 2048, 2048);
        int digit = 0, rem = 0, cnt = 0;
        const int mode = quota <= 0 ? kModeNone : (quota >= pop ? kModeAll : kModeSearch);
        if (mode == kModeSearch) wave_find_bucket(hist + c * 2048, 2048, quota, &digit, &rem, &cnt);
        if (tid == 0) { a.fs->state[c][0] = digit; a.fs->state[c][1] = rem; a.fs->state[c][2] = cnt; a.fs->state[c][3] = mode; }
    }
}

constexpr int kCandRegs = 8;             // candidates a thread of the finishing workgroup keeps in registers

__global__ __launch_bounds__(kSelThreads) void candidate_kernel(const FastArgs args) {
    __shared__ int lhist[kFastSeg * 2048];
    __shared__ int s_last, s_sure[kFastSeg], s_mode[kFastSeg], s_need[kFastSeg], s_cnt[kFastSeg];
    __shared__ uint32_t s_tau[kFastSeg], s_keep_eq[kFastSeg], s_prefix[kFastSeg];
    __shared__ int t_gt[kFastSeg][kFastTiles], t_eq[kFastSeg][kFastTiles];
    const int tid = threadIdx.x, lane = tid & 63;
    const int j = blockIdx.x * kSelThreads + tid;
    const FastView a = to_video(args);
    if (tid < kFastSeg) s_sure[tid] = 0;
    int sg = -1;
    uint32_t key = 0u;
    if (j < a.n_vis) {
        key = ordered_key(a.scores[j]);
        const int s = a.token_seg[j];
        sg = (s >= 0 && s < a.n_seg) ? s : -1;
    }
    bool sure = false, cand = false;
    if (sg >= 0) {
        const int mode = a.fs->state[sg][3], digit = a.fs->state[sg][0];
        const int d = static_cast<int>(key >> 21);
        sure = mode == kModeAll || (mode == kModeSearch && d > digit);
        cand = mode == kModeSearch && d == digit;
    }
    __syncthreads();
    for (int c = 0; c < a.n_seg; ++c) {
        const unsigned long long m = __ballot(sure && sg == c);
        if (lane == 0 && m) atomicAdd(&s_sure[c], __popcll(m));
    }
    {   // candidates of a wave take consecutive slots of the list
        const unsigned long long m = __ballot(cand);
        if (m) {
            const int leader = __ffsll(static_cast<long long>(m)) - 1;
            uint32_t base = 0u;
            if (lane == leader) base = atomicAdd(&a.fs->cand_total, static_cast<uint32_t>(__popcll(m)));
            base = __shfl(base, leader, 64);
            if (cand) {
                const uint32_t pos = base + __popcll(m & ((1ull << lane) - 1ull));
                if (pos < static_cast<uint32_t>(a.n_vis)) {
                    store_shared_between_workgroups(&a.cand_key[pos], key);
                    store_shared_between_workgroups(&a.cand_tok[pos], (static_cast<uint32_t>(sg) << 24) | static_cast<uint32_t>(j));
                }
            }
        }
    }
    __syncthreads();
    if (tid < a.n_seg) store_shared_between_workgroups(&a.fs->tile_sure[tid][blockIdx.x], s_sure[tid]);
    if (!arrive_and_check_last(&a.fs->arrive_b, &s_last)) return;

    // ---- last workgroup: every thread keeps up to eight candidates in registers; the searches of all classes run
    //      side by side, one wave per class walking that class's histogram ----
    const int n_tiles = gridDim.x;
    int m = static_cast<int>(load_shared_between_workgroups(&a.fs->cand_total));
    m = m < a.n_vis ? m : a.n_vis;
    const bool in_regs = m <= kCandRegs * kSelThreads;
    uint32_t ck[kCandRegs];
    int cm[kCandRegs];                                              // class << 6 | tile, -1: no candidate
    {
        // all loads are requested before the first is used: no branch between them (a slot past the list reads the
        // list's last entry again and is dropped)
        uint32_t tok[kCandRegs];
        const int last = m > 0 ? m - 1 : 0;
#pragma unroll
        for (int u = 0; u < kCandRegs; ++u) {
            const int i = tid + u * kSelThreads;
            const int ic = i < last ? i : last;
            tok[u] = load_shared_between_workgroups(&a.cand_tok[ic]);
            ck[u] = load_shared_between_workgroups(&a.cand_key[ic]);
        }
#pragma unroll
        for (int u = 0; u < kCandRegs; ++u) {
            const int i = tid + u * kSelThreads;
            const bool have = in_regs && i < m;
            cm[u] = have ? static_cast<int>(((tok[u] >> 24) << 6) | (((tok[u] & 0xffffffu) >> 10) & 63u)) : -1;
            ck[u] = have ? ck[u] : 0u;
        }
    }
    // f(key, class, tile) for every candidate; a list too long for the registers is walked in memory
    auto for_each_candidate = [&](auto&& f) {
        if (in_regs) {
#pragma unroll
            for (int u = 0; u < kCandRegs; ++u)
                if (cm[u] >= 0) f(ck[u], cm[u] >> 6, cm[u] & 63);
        } else {
            for (int i = tid; i < m; i += kSelThreads) {
                const uint32_t tok = load_shared_between_workgroups(&a.cand_tok[i]);
                f(load_shared_between_workgroups(&a.cand_key[i]), static_cast<int>(tok >> 24), static_cast<int>((tok & 0xffffffu) >> 10));
            }
        }
    };
    for (int i = tid; i < kFastSeg * kFastTiles; i += kSelThreads) {
        const int c = i / kFastTiles, t = i % kFastTiles;
        (&t_gt[0][0])[i] = (c < a.n_seg && t < n_tiles) ? load_shared_between_workgroups(&a.fs->tile_sure[c][t]) : 0;      // kept for sure
        (&t_eq[0][0])[i] = 0;
    }
    if (tid < kFastSeg) {
        const bool live = tid < a.n_seg;
        s_mode[tid] = live ? a.fs->state[tid][3] : kModeNone;
        s_prefix[tid] = live ? static_cast<uint32_t>(a.fs->state[tid][0]) << 21 : 0u;
        s_need[tid] = live ? a.fs->state[tid][1] : 0;
        s_cnt[tid] = live ? a.fs->state[tid][2] : 0;
    }
    __syncthreads();
    // the remaining 21 key bits of every class's quota-th largest key, 11 then 10 bits
    for (int top = 21; top > 0; top -= 11) {
        const int bits = top < 11 ? top : 11, shift = top - bits, bins = 1 << bits;
        const uint32_t hi_mask = 0xffffffffu << top, dmask = static_cast<uint32_t>(bins - 1);
        for (int i = tid; i < kFastSeg * 2048; i += kSelThreads) lhist[i] = 0;
        __syncthreads();
        for_each_candidate([&](uint32_t k, int cls, int) {
            if (s_mode[cls] == kModeSearch && (k & hi_mask) == s_prefix[cls]) atomicAdd(&lhist[cls * 2048 + ((k >> shift) & dmask)], 1);
        });
        __syncthreads();
        const int w = tid >> 6;
        if (w < a.n_seg && s_mode[w] == kModeSearch) {
            int digit = 0, need = 0, cnt = 0;
            wave_find_bucket(lhist + w * 2048, bins, s_need[w], &digit, &need, &cnt);
            wave_sync();
            if (lane == 0) { s_prefix[w] |= static_cast<uint32_t>(digit) << shift; s_need[w] = need; s_cnt[w] = cnt; }
        }
        __syncthreads();
    }
    if (tid < a.n_seg) {
        const int mode = s_mode[tid];
        uint32_t tau = 0u, keep_eq = kKeepAll;                      // kModeAll: every key is above or equal to 0
        if (mode == kModeNone) { tau = 0xffffffffu; keep_eq = 0u; }
        if (mode == kModeSearch) { tau = s_prefix[tid]; keep_eq = s_need[tid] >= s_cnt[tid] ? kKeepAll : static_cast<uint32_t>(s_need[tid]); }
        s_tau[tid] = tau; s_keep_eq[tid] = keep_eq;
        a.fs->sel_info[tid][0] = tau; a.fs->sel_info[tid][1] = keep_eq;
    }
    __syncthreads();
    // per tile and class: candidates above / equal to the threshold (t_gt already holds the tokens kept for sure)
    for_each_candidate([&](uint32_t k, int cls, int tile) {
        if (cls < a.n_seg && tile < n_tiles) {
            if (k > s_tau[cls]) atomicAdd(&t_gt[cls][tile], 1);
            else if (k == s_tau[cls]) atomicAdd(&t_eq[cls][tile], 1);
        }
    });
    __syncthreads();
    if (tid >= 64) return;
    // one wave, lane = tile (at most kFastTiles <= 64): per class the equal keys before every tile and the equal keys a
    // tile still keeps (the first keep_eq by index), then the output offset of every tile
    const bool live = lane < n_tiles;
    int kept = 0;
    for (int c = 0; c < a.n_seg; ++c) {
        const int eq = live ? t_eq[c][lane] : 0;
        int incl = eq;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off, 64);
            if (lane >= off) incl += up;
        }
        const int before = incl - eq;
        const uint32_t keep_eq = s_keep_eq[c];
        int room = keep_eq == kKeepAll ? eq : static_cast<int>(keep_eq) - before;
        room = room < 0 ? 0 : room;
        if (live) {
            a.fs->eq_before[c][lane] = before;
            kept += t_gt[c][lane] + (eq < room ? eq : room);
        }
    }
    int incl = kept;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int up = __shfl_up(incl, off, 64);
        if (lane >= off) incl += up;
    }
    if (live) a.fs->tile_off[lane] = incl - kept;
}

// Source row of every output row of the compacted sequence [prefix; kept visual rows; text rows].
__global__ __launch_bounds__(256) void hidden_index_kernel(int32_t* __restrict__ src_row, int out_rows, int vis_start, int n_vis, int n_keep,
                                                           const int32_t* __restrict__ kept_idx) {
    const int r = blockIdx.x * 256 + threadIdx.x;
    if (r >= out_rows) return;
    int s;
    if (r < vis_start) s = r;
    else if (r < vis_start + n_keep) {
        int kidx = kept_idx[r - vis_start];
        kidx = kidx < 0 ? 0 : (kidx >= n_vis ? n_vis - 1 : kidx);
        s = vis_start + kidx;
    } else s = r - n_keep + n_vis;
    src_row[r] = s;
}

constexpr int kGatherThreads = 256;

// One 16-byte chunk per thread, non-temporal (the copy pattern that measured fastest on MI355X).
__global__ __launch_bounds__(kGatherThreads) void gather_rows_kernel(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst,
                                                                     int64_t S, int64_t out_row_stride, int chunks_per_row, int vis_start,
                                                                     int n_vis, const int32_t* __restrict__ kept_idx, int64_t keep_stride,
                                                                     const BatchKeep keeps) {
    const int n_keep = keeps.n[blockIdx.z];
    const int64_t out_rows = S - n_vis + n_keep;
    src = of_video_elems(src, S * chunks_per_row); dst = of_video_elems(dst, out_row_stride * chunks_per_row);
    kept_idx = of_video_elems(kept_idx, keep_stride);
    const int64_t gidx = static_cast<int64_t>(blockIdx.x) * kGatherThreads + threadIdx.x;
    const int64_t r = gidx / chunks_per_row;
    if (r >= out_rows) return;
    const int c = static_cast<int>(gidx - r * chunks_per_row);
    int64_t s;
    if (r < vis_start) s = r;
    else if (r < static_cast<int64_t>(vis_start) + n_keep) {
        int kidx = kept_idx[r - vis_start];
        kidx = kidx < 0 ? 0 : (kidx >= n_vis ? n_vis - 1 : kidx);
        s = vis_start + kidx;
    } else s = r - n_keep + n_vis;
    __builtin_nontemporal_store(__builtin_nontemporal_load(src + s * chunks_per_row + c), dst + r * chunks_per_row + c);
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
// selection scratch: per-class tile counts above / equal to the threshold [2][METOK_MAX_SEGMENTS][n_tiles], then
// (threshold, equal keys kept) per class
static int select_tiles(int n_vis) { return (n_vis + kSelThreads - 1) / kSelThreads; }
static size_t select_count_bytes(int n_vis) {
    return round_up(static_cast<size_t>(METOK_MAX_SEGMENTS) * select_tiles(n_vis) * sizeof(int32_t), 256);
}
static size_t select_general_bytes(int n_vis) { return 2 * select_count_bytes(n_vis) + METOK_MAX_SEGMENTS * 2 * sizeof(uint32_t); }
// then the fast path: its state block and the candidate list (key and token of at most min(n_vis, 40960) candidates)
static size_t fast_state_bytes();
static size_t select_bytes(int n_vis) {
    const size_t cand = round_up(static_cast<size_t>(n_vis < kSelCache * kSelThreads ? n_vis : kSelCache * kSelThreads) * sizeof(uint32_t), 256);
    return select_general_bytes(n_vis) + fast_state_bytes() + 2 * cand;
}

// In-place compaction (hidden_out == hidden): the source row of every output row as an index list, and the
// progress flags of the row mover.  Rows of at most kInPlaceMaxRowBytes keep a row inside one workgroup
// pass, so a tile has at least eight rows and the flag count is bounded by the sequence length alone.
constexpr int64_t kInPlaceMaxRowBytes = 16384;
static size_t inplace_index_bytes(int64_t S) { return round_up(static_cast<size_t>(S) * sizeof(int32_t), 256); }
static size_t inplace_bytes(int64_t S) {
    return inplace_index_bytes(S) + round_up((64 + static_cast<size_t>((S + 7) / 8)) * sizeof(uint32_t), 256);
}

static int chunk_count(int dh, int dtype) { return dtype == METOK_BF16 ? dh / 16 : dh / 8; }     // 16-byte chunks per lane

// Row blocks a wave keeps in registers: two while the fragments of a block take at most 32 VGPRs, else one.
static int row_blocks_per_wave(int nch) { return nch <= 8 ? 2 : 1; }

static bool make_geom(int64_t S, int Hq, int Hkv, int dh, int Tq, int vis_start, int n_vis, int dtype, int score_mode,
                      ScoreGeom* g) {
    g->S = S; g->Hq = Hq; g->Hkv = Hkv; g->group = Hq / Hkv; g->dh = dh; g->Tq = Tq;
    g->R = g->group * Tq;
    g->rb_total = (g->R + 31) / 32;
    const int nch = chunk_count(dh, dtype);
    if (nch > 16) return false;
    const int cap = kScoreWaves * row_blocks_per_wave(nch);
    g->rs = (g->rb_total + cap - 1) / cap;
    g->rbw = (g->rb_total + g->rs - 1) / g->rs;
    g->vis_start = vis_start; g->n_vis = n_vis;
    g->key_begin = score_mode == METOK_SCORE_VISUAL_ONLY ? vis_start : 0;
    g->key_end = score_mode == METOK_SCORE_VISUAL_ONLY ? static_cast<int64_t>(vis_start) + n_vis : S;
    g->scale_log2 = static_cast<float>(1.4426950408889634 / sqrt(static_cast<double>(dh)));
    return true;
}

struct ScorePlan {
    int nx1, nx2;                   // workgroups along the keys in pass 1 / pass 2
    int per1, per2;                 // 32-key subtiles per workgroup
    size_t off_qfrag, off_pstat, off_norm, off_colpart, off_sel, off_inplace, total;
};

constexpr int kScoreSlots = 256;    // one 512-thread workgroup per CU

static void plan_score(const ScoreGeom& g, int n_vis, int nch, int batch, ScorePlan* p) {
    const int ny = g.Hkv * g.rs;
    const int64_t rows_of_grid = static_cast<int64_t>(ny) * batch;          // the videos of a batch share the chip's slots
    const int nx0 = kScoreSlots / rows_of_grid < 1 ? 1 : static_cast<int>(kScoreSlots / rows_of_grid);
    auto pick = [&](int64_t subtiles, int* per) {
        int64_t nx = nx0 < subtiles ? nx0 : subtiles;
        if (nx < 1) nx = 1;
        *per = static_cast<int>((subtiles + nx - 1) / nx);
        if (*per < 1) *per = 1;
        nx = (subtiles + *per - 1) / *per;                  // smallest grid with the same critical path
        return static_cast<int>(nx < 1 ? 1 : nx);
    };
    p->nx1 = pick((g.key_end - g.key_begin + 31) / 32, &p->per1);
    p->nx2 = pick((static_cast<int64_t>(n_vis) + 31) / 32, &p->per2);
    // the partial statistics are sized for the widest pass-1 grid of either score mode, so one
    // workspace query serves both
    int64_t nx1_cap = nx0;
    const int64_t sub_all = (g.S + 31) / 32;
    if (nx1_cap > sub_all) nx1_cap = sub_all;
    size_t off = 0;
    p->off_qfrag = off;   off += static_cast<size_t>(g.Hkv) * g.rb_total * nch * 1024;
    p->off_pstat = off;   off += round_up(static_cast<size_t>(ny) * nx1_cap * g.rbw * 32 * 2 * sizeof(float), 256);
    p->off_norm = off;    off += round_up(static_cast<size_t>(ny) * g.rbw * 32 * sizeof(float), 256);
    p->off_colpart = off; off += round_up(static_cast<size_t>(ny) * n_vis * sizeof(float), 256);
    p->off_sel = off;     off += select_bytes(n_vis);
    p->off_inplace = off; off += inplace_bytes(g.S);
    p->total = round_up(off, 256);
}

static bool dh_supported(int dh, int dtype) {
    if (dtype == METOK_BF16) return dh == 32 || dh == 64 || dh == 128 || dh == 256;
    return dh == 32 || dh == 64 || dh == 128;
}

template <typename T, int NCH>
static void launch_scores(const void* q, const void* k, const ScoreGeom& g, const ScorePlan& p, char* ws, int batch, hipStream_t st) {
    constexpr int RBW = NCH <= 8 ? 2 : 1;
    constexpr int SUBS = NCH <= 8 ? 2 : 1;
    using Stage = KeyStage<T, NCH, SUBS>;
    const size_t lds1 = kStageBuffers * static_cast<size_t>(Stage::kSlots) * sizeof(uint4);
    const size_t lds2 = 2 * static_cast<size_t>(Stage::kSlots) * sizeof(uint4) + 2 * static_cast<size_t>(kScoreWaves) * Stage::kKeys * sizeof(float);
    const int ny = g.Hkv * g.rs;
    uint4* qfrag = reinterpret_cast<uint4*>(ws + p.off_qfrag);
    float* pstat = reinterpret_cast<float*>(ws + p.off_pstat);
    float* norm = reinterpret_cast<float*>(ws + p.off_norm);
    float* colpart = reinterpret_cast<float*>(ws + p.off_colpart);
    const int qslots = g.Hkv * g.rb_total * NCH * 64;
    const unsigned nb = static_cast<unsigned>(batch);
    hipLaunchKernelGGL((pack_q_kernel<T, NCH>), dim3((qslots + 255) / 256, 1, nb), dim3(256), 0, st, static_cast<const T*>(q), g, qfrag,
                       reinterpret_cast<uint32_t*>(ws + p.off_sel + select_general_bytes(g.n_vis)), kFastClearWords);
    { TraceScope trace_scope(METOK_TRACE_ROW_STATS, st); hipLaunchKernelGGL((row_stats_kernel<T, NCH, RBW, SUBS>), dim3(p.nx1, ny, nb), dim3(kScoreThreads), lds1, st,
                       qfrag, static_cast<const T*>(k), g, p.per1, pstat); }
    const int total_rows = ny * g.rbw * 32;
    hipLaunchKernelGGL(merge_stats_kernel, dim3((total_rows + 15) / 16, 1, nb), dim3(256), 0, st, pstat, g, p.nx1, norm);
    { TraceScope trace_scope(METOK_TRACE_COL_SUMS, st); hipLaunchKernelGGL((col_sums_kernel<T, NCH, RBW, SUBS>), dim3(p.nx2, ny, nb), dim3(kScoreThreads), lds2, st,
                       qfrag, static_cast<const T*>(k), g, p.per2, norm, colpart); }
}

}  // namespace metok

using namespace metok;

// Workspace of ONE video of a batch of `batch` videos (the batch's videos lie one after the other).
static size_t video_workspace_bytes(int batch, int64_t S, int Hq, int Hkv, int dh, int Tq, int n_vis, int dtype) {
    if (n_vis < 0 || S < 1 || batch < 1) return 0;
    ScoreGeom g;
    ScorePlan p;
    if (Hq >= 1 && Hkv >= 1 && Tq >= 1 && Hq % Hkv == 0 && dh_supported(dh, dtype) &&
        make_geom(S, Hq, Hkv, dh, Tq, 0, n_vis, dtype, METOK_SCORE_CAUSAL_ALL, &g)) {
        plan_score(g, n_vis, chunk_count(dh, dtype), batch, &p);
        return p.total;
    }
    return round_up(select_bytes(n_vis) + inplace_bytes(S), 256);      // no attention pass (scores supplied by the caller)
}

extern "C" size_t metok_prefill_prune_workspace_bytes(int64_t S, int Hq, int Hkv, int dh, int Tq, int n_vis, int dtype) {
    return video_workspace_bytes(1, S, Hq, Hkv, dh, Tq, n_vis, dtype);
}

extern "C" size_t metok_prefill_prune_batched_workspace_bytes(int batch, int64_t S, int Hq, int Hkv, int dh, int Tq, int n_vis, int dtype) {
    if (batch < 1 || batch > METOK_MAX_BATCH) return 0;
    return static_cast<size_t>(batch) * video_workspace_bytes(batch, S, Hq, Hkv, dh, Tq, n_vis, dtype);
}

// Shared body of metok_prefill_prune, metok_prefill_prune_batched and metok_prefill_prune_static: `workspace` is the
// caller's buffer or the library's static scratch array; nothing below allocates.  Every array carries a leading
// dimension of `batch` videos (tightly packed inputs; outputs keep_stride entries / out_row_stride rows apart); every
// kernel takes the video from blockIdx.z.
static int prune_impl(int batch, const void* hidden, int64_t S, int D, int dtype,
                      const void* q_text, const void* k_all, int Hq, int Hkv, int dh, int Tq,
                      int score_mode, int vis_start, int n_vis,
                      const int32_t* token_seg, const int32_t* token_event,
                      const float* event_weight, int n_events,
                      int n_seg, const int32_t* seg_quota,
                      const int32_t* orig_idx_in, int64_t orig_idx_in_stride,
                      float* scores, int32_t* kept_idx, int64_t keep_stride, void* hidden_out, int64_t out_row_stride,
                      int32_t* token_seg_out, int32_t* token_event_out, int32_t* orig_idx_out, int64_t orig_idx_stride,
                      void* workspace, size_t workspace_bytes, void* stream) {
    if (batch < 1 || batch > METOK_MAX_BATCH) return fail(METOK_ERR_INVALID_ARG, "batch must be in [1, %d]", METOK_MAX_BATCH);
    if (dtype != METOK_F32 && dtype != METOK_BF16) return fail(METOK_ERR_INVALID_ARG, "unknown dtype %d", dtype);
    if (S < 1 || S > INT32_MAX || D < 1) return fail(METOK_ERR_INVALID_ARG, "S must be in [1, 2^31) and D positive");
    if (vis_start < 0 || n_vis < 1 || static_cast<int64_t>(vis_start) + n_vis > S)
        return fail(METOK_ERR_INVALID_ARG, "visual span [%d, %d + %d) does not fit S = %lld", vis_start, vis_start, n_vis, (long long)S);
    const size_t row_bytes = static_cast<size_t>(D) * dtype_size(dtype);
    if (row_bytes % 16) return fail(METOK_ERR_INVALID_ARG, "D * sizeof(dtype) must be a multiple of 16");
    if (!hidden || !hidden_out || !aligned16(hidden) || !aligned16(hidden_out))
        return fail(METOK_ERR_INVALID_ARG, "hidden / hidden_out NULL or not 16-byte aligned");
    if (!token_seg || !scores || !seg_quota) return fail(METOK_ERR_INVALID_ARG, "NULL pointer argument");
    if (n_seg < 1 || n_seg > METOK_MAX_SEGMENTS) return fail(METOK_ERR_INVALID_ARG, "n_seg must be in [1, %d]", METOK_MAX_SEGMENTS);
    if (!token_event && (event_weight || token_event_out)) return fail(METOK_ERR_INVALID_ARG, "token_event is NULL but needed");
    if (event_weight && n_events < 1) return fail(METOK_ERR_INVALID_ARG, "event_weight given with n_events < 1");
    BatchKeep keeps;
    int64_t max_keep = 0;
    for (int b = 0; b < METOK_MAX_BATCH; ++b) keeps.n[b] = 0;
    for (int b = 0; b < batch; ++b) {
        int64_t total_keep = 0;
        for (int s = 0; s < n_seg; ++s) {
            const int32_t q = seg_quota[static_cast<size_t>(b) * n_seg + s];
            if (q < 0 || q > n_vis) return fail(METOK_ERR_INVALID_ARG, "seg_quota[%d] = %d of video %d outside [0, n_vis]", s, q, b);
            total_keep += q;
        }
        if (total_keep > n_vis) return fail(METOK_ERR_INVALID_ARG, "quotas of video %d add up to %lld > n_vis = %d", b, (long long)total_keep, n_vis);
        keeps.n[b] = static_cast<int32_t>(total_keep);
        max_keep = total_keep > max_keep ? total_keep : max_keep;
    }
    if (max_keep > 0 && !kept_idx) return fail(METOK_ERR_INVALID_ARG, "kept_idx is NULL");
    const int64_t max_out_rows = S - n_vis + max_keep;
    if (batch > 1 && (keep_stride < max_keep || out_row_stride < max_out_rows))
        return fail(METOK_ERR_INVALID_ARG, "keep_stride = %lld / out_row_stride = %lld below the largest video's %lld kept tokens / %lld rows",
                    (long long)keep_stride, (long long)out_row_stride, (long long)max_keep, (long long)max_out_rows);
    if (batch > 1 && orig_idx_out && orig_idx_stride < max_keep)
        return fail(METOK_ERR_INVALID_ARG, "orig_idx_stride = %lld below the largest video's %lld kept tokens", (long long)orig_idx_stride, (long long)max_keep);
    if (batch > 1 && orig_idx_in && orig_idx_in_stride < n_vis)
        return fail(METOK_ERR_INVALID_ARG, "orig_idx_in_stride = %lld below n_vis = %d", (long long)orig_idx_in_stride, n_vis);
    if (batch == 1) { keep_stride = max_keep; out_row_stride = max_out_rows; orig_idx_stride = max_keep; orig_idx_in_stride = n_vis; }
    // hidden_out == hidden compacts in place (every kept row moves towards the front: source >= destination);
    // any other overlap is refused
    const bool in_place = hidden_out == hidden;
    if (!in_place) {
        const char* a0 = static_cast<const char*>(hidden); const char* a1 = a0 + static_cast<size_t>(batch) * S * row_bytes;
        const char* b0 = static_cast<const char*>(hidden_out);
        const char* b1 = b0 + (static_cast<size_t>(batch - 1) * out_row_stride + max_out_rows) * row_bytes;
        if (a0 < b1 && b0 < a1) return fail(METOK_ERR_INVALID_ARG, "hidden_out overlaps hidden without being the same buffer");
    } else {
        if (static_cast<int64_t>(row_bytes) > kInPlaceMaxRowBytes)
            return fail(METOK_ERR_UNSUPPORTED, "in-place compaction needs rows of at most %lld bytes, got %zu", (long long)kInPlaceMaxRowBytes, row_bytes);
        if (batch > 1 && out_row_stride != S)
            return fail(METOK_ERR_INVALID_ARG, "in-place compaction of a batch keeps every video where it is: out_row_stride must be S");
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    char* ws = static_cast<char*>(workspace);
    int rc;
    char* sel;
    char* inplace_ws;
    const float* colpart = nullptr;
    int n_parts = 0;
    const unsigned nb = static_cast<unsigned>(batch);
    const int64_t ws_video = static_cast<int64_t>(video_workspace_bytes(batch, S, q_text ? Hq : 0, q_text ? Hkv : 0, q_text ? dh : 0,
                                                                        q_text ? Tq : 0, n_vis, dtype));
    const int n_tiles = select_tiles(n_vis);
    const bool fast = n_seg <= kFastSeg && n_tiles <= kFastTiles;       // else the general one-workgroup-per-class select
    if (q_text) {
        if (!k_all || !aligned16(q_text) || !aligned16(k_all)) return fail(METOK_ERR_INVALID_ARG, "q_text / k_all NULL or misaligned");
        if (Hq < 1 || Hkv < 1 || Hq % Hkv) return fail(METOK_ERR_INVALID_ARG, "Hq = %d must be a positive multiple of Hkv = %d", Hq, Hkv);
        if (!dh_supported(dh, dtype)) return fail(METOK_ERR_UNSUPPORTED, "head dimension %d is not supported for this dtype", dh);
        if (Tq < 1 || static_cast<int64_t>(Tq) > S - vis_start - n_vis)
            return fail(METOK_ERR_INVALID_ARG, "Tq = %d must be in [1, number of text rows = %lld]", Tq, (long long)(S - vis_start - n_vis));
        if (score_mode != METOK_SCORE_CAUSAL_ALL && score_mode != METOK_SCORE_VISUAL_ONLY)
            return fail(METOK_ERR_INVALID_ARG, "unknown score_mode %d", score_mode);
        ScoreGeom g;
        if (!make_geom(S, Hq, Hkv, dh, Tq, vis_start, n_vis, dtype, score_mode, &g)) return fail(METOK_ERR_UNSUPPORTED, "head dimension too large");
        if (static_cast<int64_t>(g.Hkv) * g.rs > 65535) return fail(METOK_ERR_UNSUPPORTED, "too many query rows");
        ScorePlan p;
        plan_score(g, n_vis, chunk_count(dh, dtype), batch, &p);
        g.q_video = static_cast<int64_t>(Hq) * Tq * dh; g.k_video = static_cast<int64_t>(Hkv) * S * dh; g.ws_video = ws_video;
        if (static_cast<int64_t>(p.total) != ws_video) return fail(METOK_ERR_DEVICE, "internal: workspace plan mismatch");
        if (!workspace || workspace_bytes < p.total * batch || !aligned16(workspace))
            return fail(METOK_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", p.total * batch, workspace_bytes);
        const int nch = chunk_count(dh, dtype);
        if (dtype == METOK_BF16) {
            switch (nch) {
                case 2: launch_scores<bf16_t, 2>(q_text, k_all, g, p, ws, batch, st); break;
                case 4: launch_scores<bf16_t, 4>(q_text, k_all, g, p, ws, batch, st); break;
                case 8: launch_scores<bf16_t, 8>(q_text, k_all, g, p, ws, batch, st); break;
                default: launch_scores<bf16_t, 16>(q_text, k_all, g, p, ws, batch, st); break;
            }
        } else {
            switch (nch) {
                case 4: launch_scores<float, 4>(q_text, k_all, g, p, ws, batch, st); break;
                case 8: launch_scores<float, 8>(q_text, k_all, g, p, ws, batch, st); break;
                default: launch_scores<float, 16>(q_text, k_all, g, p, ws, batch, st); break;
            }
        }
        if ((rc = check_launch("attention scores"))) return rc;
        sel = ws + p.off_sel;
        inplace_ws = ws + p.off_inplace;
        colpart = reinterpret_cast<const float*>(ws + p.off_colpart);
        n_parts = g.Hkv * g.rs;
        if (!fast) {
            hipLaunchKernelGGL(prepare_kernel, dim3((n_vis + 255) / 256, 1, nb), dim3(256), 0, st, colpart, n_parts, n_vis,
                               static_cast<float>(static_cast<int64_t>(Hq) * Tq), token_event, event_weight, n_events, scores, ws_video);
            if ((rc = check_launch("prepare"))) return rc;
        }
    } else {
        const size_t need = static_cast<size_t>(ws_video) * batch;
        if (!workspace || workspace_bytes < need || !aligned16(workspace))
            return fail(METOK_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
        sel = ws;
        inplace_ws = ws + select_bytes(n_vis);
        if (fast) {      // no packing kernel runs on this path: clear the fast path's counters and histograms here
            hipLaunchKernelGGL(clear_words_kernel, dim3(8, 1, nb), dim3(256), 0, st, reinterpret_cast<uint32_t*>(sel + select_general_bytes(n_vis)),
                               kFastClearWords, ws_video);
            if ((rc = check_launch("clear"))) return rc;
        }
    }
    int32_t* gt_count = reinterpret_cast<int32_t*>(sel);
    int32_t* eq_count = reinterpret_cast<int32_t*>(sel + select_count_bytes(n_vis));
    uint32_t* sel_info = reinterpret_cast<uint32_t*>(sel + 2 * select_count_bytes(n_vis));
    const int32_t* tile_off = nullptr;
    const int32_t* eq_before = nullptr;
    if (fast) {
        FastArgs fa;
        fa.fs = reinterpret_cast<FastSel*>(sel + select_general_bytes(n_vis));
        const size_t cand = round_up(static_cast<size_t>(n_vis) * sizeof(uint32_t), 256);
        fa.cand_key = reinterpret_cast<uint32_t*>(sel + select_general_bytes(n_vis) + fast_state_bytes());
        fa.cand_tok = reinterpret_cast<uint32_t*>(sel + select_general_bytes(n_vis) + fast_state_bytes() + cand);
        fa.colpart = colpart; fa.n_parts = n_parts; fa.rows_total = static_cast<float>(static_cast<int64_t>(Hq) * Tq);
        fa.token_event = token_event; fa.event_weight = event_weight; fa.n_events = n_events;
        fa.scores = scores; fa.token_seg = token_seg; fa.n_vis = n_vis; fa.n_seg = n_seg; fa.ws_video = ws_video;
        for (int b = 0; b < METOK_MAX_BATCH; ++b)
            for (int c = 0; c < kFastSeg; ++c) fa.quota[b][c] = (b < batch && c < n_seg) ? seg_quota[static_cast<size_t>(b) * n_seg + c] : 0;
        {
            TraceScope trace_scope(METOK_TRACE_SELECT, st);          // both selection kernels
            hipLaunchKernelGGL(score_hist_kernel, dim3(n_tiles, 1, nb), dim3(kSelThreads), 0, st, fa);
            hipLaunchKernelGGL(candidate_kernel, dim3(n_tiles, 1, nb), dim3(kSelThreads), 0, st, fa);
        }
        if ((rc = check_launch("select"))) return rc;
        sel_info = &fa.fs->sel_info[0][0];
        tile_off = fa.fs->tile_off;
        eq_before = &fa.fs->eq_before[0][0];
    } else {
        // the general selection takes its quotas by value: one launch per video
        TraceScope trace_scope(METOK_TRACE_SELECT, st);
        for (int b = 0; b < batch; ++b) {
            Quotas quotas;
            for (int c = 0; c < METOK_MAX_SEGMENTS; ++c) quotas.q[c] = c < n_seg ? seg_quota[static_cast<size_t>(b) * n_seg + c] : 0;
            const float* sc_b = scores + static_cast<size_t>(b) * n_vis;
            const int32_t* seg_b = token_seg + static_cast<size_t>(b) * n_vis;
            auto at = [&](auto* ptr) { return reinterpret_cast<decltype(ptr)>(reinterpret_cast<char*>(ptr) + static_cast<size_t>(b) * ws_video); };
            if (n_vis <= kSelCache * kSelThreads)
                hipLaunchKernelGGL(select_kernel<true>, dim3(n_seg), dim3(kSelThreads), 0, st, sc_b, seg_b, n_vis, n_tiles, quotas,
                                   at(gt_count), at(eq_count), at(sel_info));
            else
                hipLaunchKernelGGL(select_kernel<false>, dim3(n_seg), dim3(kSelThreads), 0, st, sc_b, seg_b, n_vis, n_tiles, quotas,
                                   at(gt_count), at(eq_count), at(sel_info));
        }
        if ((rc = check_launch("select"))) return rc;
    }
    { TraceScope trace_scope(METOK_TRACE_WRITE_INDEX, st); hipLaunchKernelGGL(write_index_kernel, dim3(n_tiles, 1, nb), dim3(kIdxThreads), 0, st, scores, sel_info, gt_count, eq_count, token_seg, n_vis, n_seg,
                       n_tiles, 0, token_event, orig_idx_in, kept_idx, token_seg_out,
                       token_event_out, orig_idx_out, tile_off, eq_before, ws_video, keep_stride, orig_idx_in_stride, orig_idx_stride, keeps); }
    if ((rc = check_launch("write index"))) return rc;
    if (in_place) {
        // the row mover takes one sequence per call here: the videos of a batch go one after the other
        for (int b = 0; b < batch; ++b) {
            const int64_t out_rows = S - n_vis + keeps.n[b];
            if (out_rows == 0) continue;
            char* ws_b = inplace_ws + static_cast<size_t>(b) * ws_video;
            int32_t* src_row = reinterpret_cast<int32_t*>(ws_b);
            hipLaunchKernelGGL(hidden_index_kernel, dim3(static_cast<unsigned>((out_rows + 255) / 256)), dim3(256), 0, st, src_row,
                               static_cast<int>(out_rows), vis_start, n_vis, keeps.n[b], kept_idx + static_cast<size_t>(b) * keep_stride);
            if ((rc = check_launch("hidden index"))) return rc;
            RowMoveLayer layer;
            layer.k = static_cast<char*>(hidden_out) + static_cast<size_t>(b) * S * row_bytes; layer.v = nullptr; layer.idx = src_row;
            layer.n_keep = static_cast<int32_t>(out_rows);
            layer.first_item = 0; layer.tiles = 0; layer.flag_slot = 0; layer.layer_id = 0;
            rc = launch_row_moves(&layer, 1, 1, 1, 1, S, static_cast<int64_t>(row_bytes), nullptr, 0, 0, 0, nullptr, nullptr, 1,
                                  ws_b + inplace_index_bytes(S), inplace_bytes(S) - inplace_index_bytes(S), st, nullptr);
            if (rc) return rc;
        }
        return METOK_OK;
    }
    const int chunks_per_row = static_cast<int>(row_bytes / 16);
    const int64_t blocks = (max_out_rows * chunks_per_row + kGatherThreads - 1) / kGatherThreads;
    if (blocks > 0x7fffffff) return fail(METOK_ERR_INVALID_ARG, "hidden_out too large for one launch");
    if (blocks == 0) return METOK_OK;
    { TraceScope trace_scope(METOK_TRACE_GATHER_ROWS, st); hipLaunchKernelGGL(gather_rows_kernel, dim3(static_cast<unsigned>(blocks), 1, nb), dim3(kGatherThreads), 0, st,
                       static_cast<const u32x4_t*>(hidden), static_cast<u32x4_t*>(hidden_out), S, out_row_stride, chunks_per_row,
                       vis_start, n_vis, kept_idx, keep_stride, keeps); }
    return check_launch("gather");
}

extern "C" int metok_prefill_prune(const void* hidden, int64_t S, int D, int dtype,
                                   const void* q_text, const void* k_all, int Hq, int Hkv, int dh, int Tq,
                                   int score_mode, int vis_start, int n_vis,
                                   const int32_t* token_seg, const int32_t* token_event,
                                   const float* event_weight, int n_events,
                                   int n_seg, const int32_t* seg_quota,
                                   const int32_t* orig_idx_in,
                                   float* scores, int32_t* kept_idx, void* hidden_out,
                                   int32_t* token_seg_out, int32_t* token_event_out, int32_t* orig_idx_out,
                                   void* workspace, size_t workspace_bytes, void* stream) {
    clear_error();
    return prune_impl(1, hidden, S, D, dtype, q_text, k_all, Hq, Hkv, dh, Tq, score_mode, vis_start, n_vis, token_seg, token_event,
                      event_weight, n_events, n_seg, seg_quota, orig_idx_in, 0, scores, kept_idx, 0, hidden_out, 0, token_seg_out,
                      token_event_out, orig_idx_out, 0, workspace, workspace_bytes, stream);
}

extern "C" int metok_prefill_prune_batched(int batch, const void* hidden, int64_t S, int D, int dtype,
                                           const void* q_text, const void* k_all, int Hq, int Hkv, int dh, int Tq,
                                           int score_mode, int vis_start, int n_vis,
                                           const int32_t* token_seg, const int32_t* token_event,
                                           const float* event_weight, int n_events,
                                           int n_seg, const int32_t* seg_quota,
                                           const int32_t* orig_idx_in, int64_t orig_idx_in_stride,
                                           float* scores, int32_t* kept_idx, int64_t keep_stride,
                                           void* hidden_out, int64_t out_row_stride,
                                           int32_t* token_seg_out, int32_t* token_event_out,
                                           int32_t* orig_idx_out, int64_t orig_idx_stride,
                                           void* workspace, size_t workspace_bytes, void* stream) {
    clear_error();
    return prune_impl(batch, hidden, S, D, dtype, q_text, k_all, Hq, Hkv, dh, Tq, score_mode, vis_start, n_vis, token_seg, token_event,
                      event_weight, n_events, n_seg, seg_quota, orig_idx_in, orig_idx_in_stride, scores, kept_idx, keep_stride, hidden_out, out_row_stride,
                      token_seg_out, token_event_out, orig_idx_out, orig_idx_stride, workspace, workspace_bytes, stream);
}

// ---------------------------------------------------------------------------------------------
// metok_prefill_prune_static: the same call for callers that cannot allocate a workspace.  The scratch
// memory is a fixed array in the library's device image; every GPU holds its own copy at its own address,
// looked up once per device.  In host code the array's name is only a handle for that lookup: kernels
// and the shared body above always receive the looked-up device address.
// ---------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[METOK_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {nullptr};
}  // namespace

// Device address of this GPU's copy of `scratch` (cached after the first call on the device).
static int static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(METOK_ERR_DEVICE, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(METOK_ERR_UNSUPPORTED, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return fail(METOK_ERR_DEVICE, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return METOK_OK;
}

extern "C" size_t metok_static_scratch_bytes(void) { return METOK_STATIC_SCRATCH_BYTES; }

extern "C" int metok_prefill_prune_static(const void* hidden, int64_t S, int D, int dtype,
                                          const void* q_text, const void* k_all, int Hq, int Hkv, int dh, int Tq,
                                          int score_mode, int vis_start, int n_vis,
                                          const int32_t* token_seg, const int32_t* token_event,
                                          const float* event_weight, int n_events,
                                          int n_seg, const int32_t* seg_quota,
                                          const int32_t* orig_idx_in,
                                          float* scores, int32_t* kept_idx, void* hidden_out,
                                          int32_t* token_seg_out, int32_t* token_event_out, int32_t* orig_idx_out,
                                          void* stream) {
    clear_error();
    // the size check comes first so that an oversized request is refused before anything touches the device
    const size_t need = metok_prefill_prune_workspace_bytes(S, q_text ? Hq : 0, q_text ? Hkv : 0, q_text ? dh : 0, q_text ? Tq : 0,
                                                            n_vis, dtype);
    if (need > METOK_STATIC_SCRATCH_BYTES)
        return fail(METOK_ERR_WORKSPACE, "this shape needs %zu bytes of scratch memory, the static array holds %zu: use metok_prefill_prune "
                    "with a caller-provided workspace", need, static_cast<size_t>(METOK_STATIC_SCRATCH_BYTES));
    void* ws = nullptr;
    int rc = static_scratch(&ws);
    if (rc) return rc;
    return prune_impl(1, hidden, S, D, dtype, q_text, k_all, Hq, Hkv, dh, Tq, score_mode, vis_start, n_vis, token_seg, token_event,
                      event_weight, n_events, n_seg, seg_quota, orig_idx_in, 0, scores, kept_idx, 0, hidden_out, 0, token_seg_out,
                      token_event_out, orig_idx_out, 0, ws, METOK_STATIC_SCRATCH_BYTES, stream);
}
