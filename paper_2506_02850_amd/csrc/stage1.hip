// Stage 1 (Sec. 3.2.1, Algorithm 1): event segmentation, key event / key frame identification
// and adaptive pooling of the frame features V [T, N, d].
//
// Kernels
//   frame_stats_kernel   one streaming pass over V: per frame |v_i|^2 and <v_i, v_{i+1}> (Eq. 4) and
//                        the mean per-token cosine with the text embedding (Eq. 5)
//   segment_kernel       one workgroup: T-1 cosines, the k-1 lowest become boundaries
//   plan_kernel          one workgroup: event scores, key events, key frames, strides, row offsets
//   pool_kernel          second streaming pass: s x s mean pooling of every frame, packed output
//   frame_stats_pool2_kernel   statistics and 2 x 2 pooling from ONE pass, when every frame's stride is 2
//   frame_mean_kernel, frame_score_kernel, fill_token_event_kernel   small helpers of the other readings / paths
//
// In the one-pass call a batch of videos of one shape runs as one launch of every kernel: blockIdx.z is the
// video, every pointer advances by that video's stride.
#include "common.h"

namespace metok {

constexpr int kStatsThreads = 256;
constexpr int kStatsWaves = kStatsThreads / 64;
constexpr float kZeroNorm = 1e-12f;

// ---------------------------------------------------------------------------------------------
// frame_stats_kernel
//
// A token row (d elements) is spread over G lanes in 16-byte chunks (lane j of the group takes
// chunks j, j+G, ...; at most KL chunks per lane).  A wave therefore works on TPW = 64/G tokens at a
// time ("wave chunk" cw = blockIdx.x * 4 + wave of the frame's tokens).  blockIdx.y selects a run of
// consecutive frames; the wave walks its run keeping the rows of the previous and the current frame in
// registers, so that every frame is read once (plus one extra frame per run for the pair that straddles two
// runs): at step t it takes <v_{t-1}, v_t>, then requests frame t + 1 into the registers of frame t - 1 and
// works on frame t while those loads are in flight.  Waves are independent (no LDS, no barrier).
//
// part[(t * C + cw) * 3 + {0,1,2}] = over the tokens of wave chunk cw of frame t:
//     sum |v|^2,  sum <v_t, v_{t+1}> (token-mean mode: sum of cos(v_t[n], v_{t+1}[n])),  sum of cos(token, text)
//
// Cross-lane sums use v_permlane32_swap / v_permlane16_swap: they exchange halves of two registers, so one
// swap and one add fold two values at once.
// ---------------------------------------------------------------------------------------------
// low half of the wave: a summed over the lane pairs (l, l + 32); high half: b likewise
__device__ __forceinline__ float swap32_add(float a, float b) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// even 16-lane rows: a of the rows (r, r + 1) added; odd rows: b likewise
__device__ __forceinline__ float swap16_add(float a, float b) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

template <typename T, int G, int KL>
__global__ __launch_bounds__(kStatsThreads) void frame_stats_kernel(
    const T* __restrict__ feats, const T* __restrict__ text, int T_frames, int N, int d,
    int frames_per_run, int do_pair, int sim_mode, float* __restrict__ part, int C, int64_t ws_video) {
    using E = Elem<T>;
    static_assert(G == 16 || G == 64, "token groups are one DPP row or one wave");
    feats = of_video_elems(feats, static_cast<int64_t>(T_frames) * N * d); text = of_video_elems(text, d);
    part = of_video(part, ws_video);
    constexpr int TPW = 64 / G;                 // tokens per wave
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int sub = lane % G, tw = lane / G;
    const int cw = blockIdx.x * kStatsWaves + wave;
    if (cw >= C) return;                        // there is no barrier below: a wave may leave on its own
    const int n = cw * TPW + tw;
    const bool tok_ok = n < N;
    const int nchunks = d / E::kVec;
    const int t0 = blockIdx.y * frames_per_run;
    const int t1 = min(T_frames, t0 + frames_per_run);
    const uint4 zero = make_uint4(0, 0, 0, 0);
    const size_t row_chunks = static_cast<size_t>(nchunks);

    // text embedding chunks and its norm
    uint4 txt[KL];
    float tn2 = 0.f;
    const bool do_text = text != nullptr;
#pragma unroll
    for (int k = 0; k < KL; ++k) {
        const int c = sub + k * G;
        txt[k] = (do_text && c < nchunks) ? reinterpret_cast<const uint4*>(text)[c] : zero;
        tn2 = E::dot(txt[k], txt[k], tn2);
    }
    const float tnorm = sqrtf(group_sum<G>(tn2));

    // Loads are branch-free (a lane past the last chunk or token reads a valid address again and its data is masked
    // where it is used), so that the compiler can count the loads in flight and wait for exactly the older ones.
    bool valid[KL];
    int chc[KL];
#pragma unroll
    for (int k = 0; k < KL; ++k) {
        const int c = sub + k * G;
        valid[k] = tok_ok && c < nchunks;
        chc[k] = c < nchunks ? c : nchunks - 1;
    }
    auto load_row = [&](int t, uint4 (&dst)[KL]) {
        const uint4* row = reinterpret_cast<const uint4*>(feats) + (static_cast<size_t>(t) * N + (tok_ok ? n : 0)) * row_chunks;
#pragma unroll
        for (int k = 0; k < KL; ++k) dst[k] = load_stream(row + chc[k]);
    };

    const int t_last = (do_pair && t1 < T_frames) ? t1 : t1 - 1;      // last frame that is loaded
    float p_prev = 0.f;
    // the partial sums of a step are stored at the start of the next one, after that step's wait: a store issued just
    // before a wait for loads would be waited for as well
    float st_cd = 0.f, st_p = 0.f, st_c = 0.f;
    int st_t = -1;                                                    // frame whose sums are pending (-1: none)
    bool st_own = false;
    auto flush = [&]() {
        if (st_t < 0) return;
        if (lane == 0) {
            if (st_t > t0) part[(static_cast<size_t>(st_t - 1) * C + cw) * 3 + 1] = st_cd;
            if (st_own) part[(static_cast<size_t>(st_t) * C + cw) * 3 + 0] = st_p;
        }
        if (G == 16 ? lane == 32 : lane == 0) {
            if (st_own) part[(static_cast<size_t>(st_t) * C + cw) * 3 + 2] = st_c;
        }
    };
    // X holds frame t, W frame t - 1; after the pair product W receives frame t + 1 (LOAD: there is such a frame)
    auto step = [&](int t, uint4 (&W)[KL], uint4 (&X)[KL], auto load_tag) {
        constexpr bool LOAD = decltype(load_tag)::value;
        const bool own = t < t1;                                      // frame t belongs to this run
        float p = 0.f, q = 0.f, cd = 0.f;
        const bool pair = do_pair && t > t0;
#pragma unroll
        for (int k = 0; k < KL; ++k) {                                // the first use of X: the only wait of the step
            const float ck = E::dot(W[k], X[k], 0.f);
            cd += (pair && valid[k]) ? ck : 0.f;
        }
        __builtin_amdgcn_sched_barrier(0);
        flush();
        if (LOAD) load_row(t + 1, W);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < KL; ++k) {
            const float pk = E::dot(X[k], X[k], 0.f);
            p += valid[k] ? pk : 0.f;
            q = E::dot(X[k], txt[k], q);                              // txt is zero past the last chunk
        }
        if (!own) q = 0.f;
        // per token (one 16-lane row, or the whole wave): every lane of the group gets the token's sums
        p = row16_sum(p); q = row16_sum(q); cd = row16_sum(cd);
        if (G == 64) {
            // rows 0 / 2 of the wave end up with the whole token's |v|^2 / text product; bring both to every lane
            float a = swap32_add(p, q);
            a = swap16_add(a, a);
            const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(a), false, false);
            p = __uint_as_float(r[0]); q = __uint_as_float(r[1]);
            cd = swap32_add(cd, cd);
            cd = swap16_add(cd, cd);                                  // rows 0 and 2: all four rows
        }
        if (sim_mode == METOK_SIM_TOKEN_MEAN) {                       // cosine of the matching tokens of frames t-1 and t
            const float dn = sqrtf(p_prev) * sqrtf(p);
            cd = (tok_ok && !(dn < kZeroNorm)) ? cd / dn : 0.f;
        }
        p_prev = p;
        const float den = sqrtf(p) * tnorm;
        const float cosv = (own && do_text && tok_ok && !(den < kZeroNorm)) ? q / den : 0.f;
        if (!own) p = 0.f;
        if (G == 16) {
            // the four tokens of the wave: rows -> lane 0 (|v|^2, pair) and lane 32 (cosine)
            float a = swap32_add(p, cosv);
            a = swap16_add(a, a);
            p = a;                                                    // lane 0: sum |v|^2; lane 32: sum of cosines
            cd = swap32_add(cd, cd);
            cd = swap16_add(cd, cd);
        }
        // slot 1 of frame t-1 holds <v_{t-1}, v_t>; slots 0 and 2 belong to frame t
        st_t = t; st_own = own; st_cd = cd; st_p = p; st_c = G == 16 ? p : cosv;
    };
    const std::integral_constant<bool, true> with_load;
    const std::integral_constant<bool, false> without_load;
    uint4 A[KL], B[KL];
#pragma unroll
    for (int k = 0; k < KL; ++k) B[k] = zero;
    load_row(t0, A);
    int t = t0;
    for (; t + 2 <= t_last; t += 2) {                                 // straight-line pairs of steps, each requesting a frame
        step(t, B, A, with_load);
        step(t + 1, A, B, with_load);
    }
    if (t + 1 <= t_last) {
        step(t, B, A, with_load);
        step(t + 1, A, B, without_load);
    } else if (t <= t_last) {
        step(t, B, A, without_load);
    }
    flush();
    // the pair slot of the very last frame is never read; define it
    if (lane == 0 && t1 == T_frames) part[(static_cast<size_t>(T_frames - 1) * C + cw) * 3 + 1] = 0.f;
}

// ---------------------------------------------------------------------------------------------
// segment_kernel: one workgroup of 1024 threads.
// ---------------------------------------------------------------------------------------------
constexpr int kSegThreads = 1024;
constexpr int kRankLoopFrames = 2048;      // up to here every thread ranks its frames against all others

__global__ __launch_bounds__(kSegThreads) void segment_kernel(
    const float* __restrict__ part, int C, int T, int N, int k, int have_text, int sim_mode,
    float* __restrict__ sim, int32_t* __restrict__ event_start, int32_t* __restrict__ frame_event,
    float* __restrict__ frame_score, float* __restrict__ frame_norm2, float* __restrict__ pair_dot, int64_t ws_video) {
    __shared__ __align__(16) uint32_t key[METOK_MAX_FRAMES + 8];      // ordered keys of S_i, padded with the largest key
    __shared__ int scan_scratch[17];
    const int tid = threadIdx.x;
    part = of_video(part, ws_video); frame_norm2 = of_video(frame_norm2, ws_video); pair_dot = of_video(pair_dot, ws_video);
    sim = of_video_elems(sim, T - 1); event_start = of_video_elems(event_start, k + 1);
    frame_event = of_video_elems(frame_event, T); frame_score = of_video_elems(frame_score, T);

    // per-frame totals: the 3 C partial sums of a frame are contiguous (|v|^2, pair product, cosine sum, repeated C
    // times).  A wave takes four frames at a time; a lane reads the floats lane, lane + 64, ... of each and adds every
    // value to the total of its component; the lane totals are combined by a fixed butterfly, so the result does not
    // depend on timing.  The 16 loads of a step are requested together, without a branch between them (a position past
    // the end reads the last one again and is not added).
    {
        constexpr int kWaves = kSegThreads / 64, kBatch = 4, kRounds = 4;
        const int lane = tid & 63, wave = tid >> 6;
        const int n = 3 * C;
        for (int tb = wave; tb < T; tb += kWaves * kBatch) {
            float acc[kBatch][3];
#pragma unroll
            for (int u = 0; u < kBatch; ++u) { acc[u][0] = 0.f; acc[u][1] = 0.f; acc[u][2] = 0.f; }
            for (int e0 = 0; e0 < n; e0 += 64 * kRounds) {
                float v[kBatch][kRounds];
#pragma unroll
                for (int u = 0; u < kBatch; ++u) {
                    const int t = tb + u * kWaves < T ? tb + u * kWaves : T - 1;
                    const float* src = part + static_cast<size_t>(t) * n;
#pragma unroll
                    for (int r = 0; r < kRounds; ++r) {
                        const int e = e0 + 64 * r + lane;
                        v[u][r] = src[e < n ? e : n - 1];
                    }
                }
#pragma unroll
                for (int r = 0; r < kRounds; ++r) {
                    const int e = e0 + 64 * r + lane;
                    const int comp = e < n ? e % 3 : 3;
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) {
                        acc[u][0] += comp == 0 ? v[u][r] : 0.f;
                        acc[u][1] += comp == 1 ? v[u][r] : 0.f;
                        acc[u][2] += comp == 2 ? v[u][r] : 0.f;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < kBatch; ++u) {
                const int t = tb + u * kWaves;
                const float a = wave_sum(acc[u][0]), b = wave_sum(acc[u][1]), c3 = wave_sum(acc[u][2]);
                if (lane == 0 && t < T) {
                    frame_norm2[t] = a;
                    pair_dot[t] = b;
                    if (have_text && frame_score) frame_score[t] = c3 / static_cast<float>(N);
                }
            }
        }
    }
    __syncthreads();
    // Eq. 4
    for (int t = tid; t < T - 1; t += kSegThreads) {
        const float den = sqrtf(frame_norm2[t]) * sqrtf(frame_norm2[t + 1]);
        const float s = sim_mode == METOK_SIM_TOKEN_MEAN ? pair_dot[t] / static_cast<float>(N)
                                                         : ((den < kZeroNorm) ? 0.f : pair_dot[t] / den);
        sim[t] = s;
        key[t] = ordered_key(s);
    }
    const int n_pairs = T - 1, n_quads = (n_pairs + 3) / 4;
    if (tid < 4 && n_pairs + tid < n_quads * 4) key[n_pairs + tid] = 0xffffffffu;      // never below a real key, and at a higher index
    __syncthreads();
    // the k-1 lowest similarities under the order (value, index) are boundaries
    const int per = (T + kSegThreads - 1) / kSegThreads;      // frames per thread, consecutive
    uint32_t my_flags = 0;                                    // bit j: frame tid*per + j opens an event (per <= 8)
    if (T > kRankLoopFrames) {
        // Long videos: the (k-1)-th lowest key by a radix select over the keys in LDS (four 8-bit digits), then
        // "below it, or equal to it and among the first equal keys by index" -- the same set as the rank rule
        // below, in O(T) instead of O(T^2 / threads) compares.
        __shared__ int hist[256];
        __shared__ uint32_t s_prefix;
        __shared__ int s_need;
        if (tid == 0) { s_prefix = 0u; s_need = k - 1; }
        for (int shift = 24; shift >= 0 && k > 1; shift -= 8) {
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            const uint32_t prefix = s_prefix, himask = shift == 24 ? 0u : 0xffffffffu << (shift + 8);
            for (int i = tid; i < n_pairs; i += kSegThreads)
                if ((key[i] & himask) == prefix) atomicAdd(&hist[(key[i] >> shift) & 255u], 1);
            __syncthreads();
            if (tid < 64) {                                   // one wave: four bins per lane, ascending
                const int need = s_need;
                int c[4], mine = 0;
                for (int u = 0; u < 4; ++u) { c[u] = hist[4 * tid + u]; mine += c[u]; }
                int incl = mine;
                for (int off = 1; off < 64; off <<= 1) { const int up = __shfl_up(incl, off, 64); if (tid >= off) incl += up; }
                int run = incl - mine;
                if (run < need && incl >= need) {             // exactly one lane: the digit holding the need-th lowest key
                    for (int u = 0; u < 4; ++u) {
                        if (run + c[u] >= need) { s_prefix = prefix | (static_cast<uint32_t>(4 * tid + u) << shift); s_need = need - run; break; }
                        run += c[u];
                    }
                }
            }
            __syncthreads();
        }
        const uint32_t tau = s_prefix;
        const int take_equal = s_need;                        // equal keys that still are boundaries, lowest index first
        int n_eq = 0;
        for (int j = 0; j < per; ++j) {
            const int f = tid * per + j;
            if (k > 1 && f >= 1 && f < T) {
                if (key[f - 1] < tau) my_flags |= 1u << j;
                n_eq += key[f - 1] == tau ? 1 : 0;
            }
        }
        int total_eq = 0;
        int eq_rank = block_exclusive_scan(n_eq, scan_scratch, &total_eq);
        for (int j = 0; j < per; ++j) {
            const int f = tid * per + j;
            if (k > 1 && f >= 1 && f < T && key[f - 1] == tau) {
                if (eq_rank < take_equal) my_flags |= 1u << j;
                ++eq_rank;
            }
        }
    } else
    for (int j = 0; j < per; ++j) {
        const int f = tid * per + j;                          // frame f opens an event if pair f-1 is a boundary
        if (f >= 1 && f < T) {
            const int i = f - 1;
            const uint32_t ki = key[i];
            int rank = 0;
            const uint4* key4 = reinterpret_cast<const uint4*>(key);          // four keys per LDS read, all lanes the same address
#pragma unroll 4
            for (int q = 0; q < n_quads; ++q) {
                const uint4 km = key4[q];
                const int m = 4 * q;
                rank += (km.x < ki || (km.x == ki && m < i)) ? 1 : 0;
                rank += (km.y < ki || (km.y == ki && m + 1 < i)) ? 1 : 0;
                rank += (km.z < ki || (km.z == ki && m + 2 < i)) ? 1 : 0;
                rank += (km.w < ki || (km.w == ki && m + 3 < i)) ? 1 : 0;
            }
            if (rank < k - 1) my_flags |= 1u << j;
        }
    }
    int total = 0;
    int prefix = block_exclusive_scan(__popc(my_flags), scan_scratch, &total);
    // frame_event[f] = number of event openings at or before f
    int ev = prefix;
    for (int j = 0; j < per; ++j) {
        const int f = tid * per + j;
        if (f < T) {
            if (my_flags & (1u << j)) {
                ++ev;
                if (ev <= k - 1) event_start[ev] = f;         // total == k-1 by construction; the guard is for NaN input
            }
            frame_event[f] = ev < k ? ev : k - 1;
        }
    }
    if (tid == 0) {
        event_start[0] = 0;
        event_start[k] = T;
    }
}

// Token-mean vector of every frame (pooled reading of Eq. 4): mean[t][:] = (1/N) sum_n v_t[n][:], fp32.
// A workgroup takes one frame and 64 chunk columns; its four waves split the tokens and are added in order.
template <typename T>
__global__ __launch_bounds__(256) void frame_mean_kernel(const T* __restrict__ feats, int N, int d, float* __restrict__ mean) {
    using E = Elem<T>;
    __shared__ float red[4][64][8];
    const int t = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nchunks = d / E::kVec;
    const int c = blockIdx.y * 64 + lane;
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (c < nchunks) {
        const uint4* base = reinterpret_cast<const uint4*>(feats) + static_cast<size_t>(t) * N * nchunks + c;
        int n = wave;
        for (; n + 12 < N; n += 16) {                  // four independent loads in flight
            const uint4 a = load_stream(base + static_cast<size_t>(n) * nchunks), b = load_stream(base + static_cast<size_t>(n + 4) * nchunks),
                        e = load_stream(base + static_cast<size_t>(n + 8) * nchunks), f = load_stream(base + static_cast<size_t>(n + 12) * nchunks);
            E::accumulate(a, acc); E::accumulate(b, acc); E::accumulate(e, acc); E::accumulate(f, acc);
        }
        for (; n < N; n += 4) E::accumulate(load_stream(base + static_cast<size_t>(n) * nchunks), acc);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) red[wave][lane][i] = acc[i];
    __syncthreads();
    if (wave == 0 && c < nchunks) {
        for (int i = 0; i < E::kVec; ++i)
            mean[static_cast<size_t>(t) * d + static_cast<size_t>(c) * E::kVec + i] =
                (((red[0][lane][i] + red[1][lane][i]) + red[2][lane][i]) + red[3][lane][i]) / static_cast<float>(N);
    }
}

// Eq. 5 on its own: frame_score[t] = (sum of the chunk partials of the token cosines) / N, one wave per frame.
__global__ __launch_bounds__(kSegThreads) void frame_score_kernel(const float* __restrict__ part, int C, int T, int N,
                                                                  float* __restrict__ frame_score) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int t = wave; t < T; t += kSegThreads / 64) {
        float fs = 0.f;
        for (int c = lane; c < C; c += 64) fs += part[(static_cast<size_t>(t) * C + c) * 3 + 2];
        fs = wave_sum(fs);
        if (lane == 0) frame_score[t] = fs / static_cast<float>(N);
    }
}

// ---------------------------------------------------------------------------------------------
// plan_kernel: one workgroup.  Event scores, key events, key frames, strides and output offsets.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ int pooled_side(int g, int s, int edge) {
    return edge == METOK_POOL_FLOOR ? max(1, g / s) : (g + s - 1) / s;
}

// The n largest of keys[a, b) under (key descending, index ascending), found by the whole workgroup without comparing
// item against item: the n-th largest key bit by bit (32 counting rounds), then the keys above it and, of the keys
// equal to it, the first ones by index (an exclusive scan over the threads in index order).  The calling thread owns the
// contiguous items first_owned .. first_owned + per - 1 (per <= 32); bit j of the result says whether item
// first_owned + j is among the n.  Every thread of the workgroup must call it with the same a, b, n.
__device__ __forceinline__ uint32_t block_top_n_flags(const uint32_t* keys, int a, int b, int n, int first_owned, int per,
                                                      int* scan_scratch) {
    const int tid = threadIdx.x;
    if (n <= 0) return 0u;
    uint32_t tau = 0u;
    int total = 0;
    for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = tau | (1u << bit);
        int c = 0;
        for (int m = a + tid; m < b; m += static_cast<int>(blockDim.x)) c += keys[m] >= cand ? 1 : 0;
        block_exclusive_scan(c, scan_scratch, &total);
        if (total >= n) tau = cand;
    }
    int c_gt = 0;
    for (int m = a + tid; m < b; m += static_cast<int>(blockDim.x)) c_gt += keys[m] > tau ? 1 : 0;
    block_exclusive_scan(c_gt, scan_scratch, &total);
    const int need = n - total;                                // equal keys still kept
    int eq_mine = 0;
    for (int j = 0; j < per; ++j) {
        const int f = first_owned + j;
        eq_mine += (f >= a && f < b && keys[f] == tau) ? 1 : 0;
    }
    int eq_run = block_exclusive_scan(eq_mine, scan_scratch, &total);
    uint32_t flags = 0u;
    for (int j = 0; j < per; ++j) {
        const int f = first_owned + j;
        if (f >= a && f < b) {
            const uint32_t kf = keys[f];
            if (kf > tau || (kf == tau && eq_run < need)) flags |= 1u << j;
            eq_run += kf == tau ? 1 : 0;
        }
    }
    return flags;
}

__global__ __launch_bounds__(kSegThreads) void plan_kernel(
    const float* __restrict__ frame_score, const int32_t* __restrict__ event_start, int T, int k,
    int n_key_events, double beta, int s_key_kf, int s_key_nf, int s_non_kf, int s_non_nf,
    int grid_h, int grid_w, int event_reduce, int pool_edge,
    float* __restrict__ event_score, uint8_t* __restrict__ event_is_key, uint8_t* __restrict__ frame_is_key,
    int32_t* __restrict__ frame_stride, int32_t* __restrict__ frame_offsets, int32_t* __restrict__ frame_event_ws,
    float* __restrict__ frame_score_out, int64_t ws_video) {
    __shared__ __align__(16) uint32_t ekey[METOK_MAX_FRAMES];    // ordered keys of the event scores (k <= T), then of the frame scores
    __shared__ uint8_t ev_key[METOK_MAX_FRAMES];
    __shared__ int scan_scratch[17];
    const int tid = threadIdx.x;
    frame_score = of_video_elems(frame_score, T); event_start = of_video_elems(event_start, k + 1);
    event_score = of_video_elems(event_score, k); event_is_key = of_video_elems(event_is_key, k);
    frame_is_key = of_video_elems(frame_is_key, T); frame_stride = of_video_elems(frame_stride, T);
    frame_offsets = of_video_elems(frame_offsets, T + 1); frame_event_ws = of_video(frame_event_ws, ws_video);
    frame_score_out = of_video_elems(frame_score_out, T);

    // event score: mean (Sec. 3.2.1) or max (Algorithm 1) of the frame scores, frames in index order
    for (int e = tid; e < k; e += kSegThreads) {
        int a = event_start[e], b = event_start[e + 1];
        a = max(0, min(a, T)); b = max(a, min(b, T));
        float acc = (event_reduce == METOK_EVENT_MAX) ? -INFINITY : 0.f;
        for (int f = a; f < b; ++f) acc = (event_reduce == METOK_EVENT_MAX) ? fmaxf(acc, frame_score[f]) : acc + frame_score[f];
        if (event_reduce != METOK_EVENT_MAX) acc = (b > a) ? acc / static_cast<float>(b - a) : 0.f;
        event_score[e] = acc;
        ekey[e] = ordered_key(acc);
    }
    __syncthreads();
    // key events: rank under (score descending, index ascending); beyond kLongEvent events without the all-pairs ranking
    constexpr int kLongEvent = 1024;
    if (k <= kLongEvent) {
        for (int e = tid; e < k; e += kSegThreads) {
            const uint32_t ke = ekey[e];
            int rank = 0;
            for (int m = 0; m < k; ++m) rank += (ekey[m] > ke || (ekey[m] == ke && m < e)) ? 1 : 0;
            const uint8_t is_key = rank < n_key_events ? 1 : 0;
            ev_key[e] = is_key;
            event_is_key[e] = is_key;
        }
    } else {
        const int per_e = (k + kSegThreads - 1) / kSegThreads;
        const uint32_t flags = block_top_n_flags(ekey, 0, k, min(n_key_events, k), tid * per_e, per_e, scan_scratch);
        for (int j = 0; j < per_e; ++j) {
            const int e = tid * per_e + j;
            if (e < k) { const uint8_t is_key = (flags >> j & 1u) ? 1 : 0; ev_key[e] = is_key; event_is_key[e] = is_key; }
        }
    }
    __syncthreads();
    // the frame scores as ordered keys in LDS (the event keys are no longer needed): the ranking below reads every key
    // of a frame's event, four per 16-byte read
    for (int f = tid; f < T; f += kSegThreads) ekey[f] = ordered_key(frame_score[f]);
    __syncthreads();
    const int per = (T + kSegThreads - 1) / kSegThreads;      // thread tid owns frames tid * per .. tid * per + per - 1
    // Events longer than kLongEvent frames (at most 7 of them) do not rank frame against frame either.
    __shared__ int long_list[8];
    __shared__ int n_long_s;
    if (tid == 0) n_long_s = 0;
    __syncthreads();
    for (int e = tid; e < k; e += kSegThreads) {
        int a = event_start[e], b = event_start[e + 1];
        a = max(0, min(a, T)); b = max(a, min(b, T));
        if (b - a > kLongEvent) { const int p = atomicAdd(&n_long_s, 1); if (p < 8) long_list[p] = e; }
    }
    __syncthreads();
    const int n_long = min(n_long_s, 8);
    uint32_t long_flags = 0u;                                  // bit j: frame tid * per + j is a key frame of a long event
    for (int li = 0; li < n_long; ++li) {
        const int e = long_list[li];
        int a = event_start[e], b = event_start[e + 1];
        a = max(0, min(a, T)); b = max(a, min(b, T));
        const int len = b - a;
        const int n_kf = min(len, static_cast<int>(ceil(beta * static_cast<double>(len) - 1e-9)));
        long_flags |= block_top_n_flags(ekey, a, b, n_kf, tid * per, per, scan_scratch);
    }
    // per frame: event id (binary search), rank inside the event, stride, pooled row count
    int counts[8];
    int mine = 0;
    for (int j = 0; j < per; ++j) {
        const int f = tid * per + j;
        counts[j] = 0;
        if (f < T) {
            int lo = 0, hi = k - 1;                       // last event whose start is <= f
            while (lo < hi) {
                const int mid = (lo + hi + 1) >> 1;
                if (event_start[mid] <= f) lo = mid; else hi = mid - 1;
            }
            const int e = lo;
            int a = event_start[e], b = event_start[e + 1];
            a = max(0, min(a, T)); b = max(a, min(b, T));
            const uint32_t kf = ekey[f];
            const int len = b - a;
            int n_kf = static_cast<int>(ceil(beta * static_cast<double>(len) - 1e-9));
            n_kf = min(len, n_kf);
            bool kf_flag;
            if (len > kLongEvent) {
                kf_flag = (long_flags >> j & 1u) != 0u;
            } else {
                int rank = 0;
                auto count = [&](uint32_t km, int m) { rank += (km > kf || (km == kf && m < f)) ? 1 : 0; };
                int m = a;
                for (; m < b && (m & 3); ++m) count(ekey[m], m);
                for (; m + 4 <= b; m += 4) {
                    const uint4 q = *reinterpret_cast<const uint4*>(&ekey[m]);
                    count(q.x, m); count(q.y, m + 1); count(q.z, m + 2); count(q.w, m + 3);
                }
                for (; m < b; ++m) count(ekey[m], m);
                kf_flag = rank < n_kf;
            }
            const bool ek_flag = ev_key[e] != 0;
            int s = ek_flag ? (kf_flag ? s_key_kf : s_key_nf) : (kf_flag ? s_non_kf : s_non_nf);
            frame_is_key[f] = kf_flag ? 1 : 0;
            frame_stride[f] = s;
            frame_event_ws[f] = e;
            if (frame_score_out) frame_score_out[f] = frame_score[f];
            counts[j] = pooled_side(grid_h, s, pool_edge) * pooled_side(grid_w, s, pool_edge);
            mine += counts[j];
        }
    }
    int total = 0;
    int run = block_exclusive_scan(mine, scan_scratch, &total);
    for (int j = 0; j < per; ++j) {
        const int f = tid * per + j;
        if (f < T) {
            frame_offsets[f] = run;
            run += counts[j];
        }
    }
    if (tid == 0) frame_offsets[T] = total;
}

// ---------------------------------------------------------------------------------------------
// pool_kernel: blockIdx.y = frame; the waves of the frame's workgroups share its work items.
// A work item is (pooled row, column part of 64 chunks); a lane owns one 16-byte input chunk
// of every cell of the window and writes the pooled chunk.
// ---------------------------------------------------------------------------------------------
constexpr int kPoolThreads = 256;

template <typename TO> struct Store;
template <> struct Store<float> {
    // 4 or 8 fp32 values -> 16 or 32 bytes
    static __device__ __forceinline__ void put(float* row, int chunk, int vec, const float (&a)[8]) {
        uint4* dst = reinterpret_cast<uint4*>(row + static_cast<size_t>(chunk) * vec);
        store_stream(dst, make_uint4(__float_as_uint(a[0]), __float_as_uint(a[1]), __float_as_uint(a[2]), __float_as_uint(a[3])));
        if (vec == 8)
            store_stream(dst + 1, make_uint4(__float_as_uint(a[4]), __float_as_uint(a[5]), __float_as_uint(a[6]), __float_as_uint(a[7])));
    }
};
template <> struct Store<bf16_t> {
    static __device__ __forceinline__ void put(bf16_t* row, int chunk, int vec, const float (&a)[8]) {
        uint32_t* dst = reinterpret_cast<uint32_t*>(row + static_cast<size_t>(chunk) * vec);
        if (vec == 8) {
            store_stream(reinterpret_cast<uint4*>(dst), make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]),
                                                                   pack_bf16x2(a[4], a[5]), pack_bf16x2(a[6], a[7])));
        } else {
            *reinterpret_cast<uint2*>(dst) = make_uint2(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]));
        }
    }
};

template <typename TI, typename TO>
__global__ __launch_bounds__(kPoolThreads) void pool_kernel(
    const TI* __restrict__ feats, int grid_h, int grid_w, int d,
    const int32_t* __restrict__ frame_stride, const int32_t* __restrict__ frame_offsets,
    const int32_t* __restrict__ frame_event, int pool_edge, int64_t capacity_rows,
    TO* __restrict__ out, int32_t* __restrict__ token_event, int T_frames, int64_t ws_video) {
    using E = Elem<TI>;
    feats = of_video_elems(feats, static_cast<int64_t>(T_frames) * grid_h * grid_w * d);
    frame_stride = of_video_elems(frame_stride, T_frames); frame_offsets = of_video_elems(frame_offsets, T_frames + 1);
    frame_event = of_video(frame_event, ws_video);
    out = of_video_elems(out, capacity_rows * d); token_event = of_video_elems(token_event, capacity_rows);
    const int f = blockIdx.y;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int s = frame_stride[f];
    const int oh = pooled_side(grid_h, s, pool_edge), ow = pooled_side(grid_w, s, pool_edge);
    const int base = frame_offsets[f];
    const int ev = frame_event[f];
    const int nchunks = d / E::kVec;
    const int colparts = (nchunks + 63) / 64;
    const int items = oh * ow * colparts;
    const uint4* frame = reinterpret_cast<const uint4*>(feats) + static_cast<size_t>(f) * grid_h * grid_w * nchunks;
    const int stride_items = gridDim.x * (kPoolThreads / 64);

    for (int item = blockIdx.x * (kPoolThreads / 64) + wave; item < items; item += stride_items) {
        const int orow = item / colparts;
        const int chunk = (item - orow * colparts) * 64 + lane;
        const int oy = orow / ow, ox = orow - oy * ow;
        const int y0 = oy * s, y1 = min(y0 + s, grid_h);
        const int x0 = ox * s, x1 = min(x0 + s, grid_w);
        const int64_t out_row = static_cast<int64_t>(base) + orow;
        if (out_row >= capacity_rows) continue;              // cannot happen when the caller sized the buffer as required
        if (chunk < nchunks) {
            float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            for (int y = y0; y < y1; ++y) {
                const uint4* cell = frame + (static_cast<size_t>(y) * grid_w + x0) * nchunks + chunk;
                int x = x0;
                for (; x + 4 <= x1; x += 4) {                 // four independent loads in flight
                    const uint4 a = load_stream(cell), b = load_stream(cell + nchunks),
                                c = load_stream(cell + 2 * static_cast<size_t>(nchunks)),
                                e = load_stream(cell + 3 * static_cast<size_t>(nchunks));
                    E::accumulate(a, acc); E::accumulate(b, acc); E::accumulate(c, acc); E::accumulate(e, acc);
                    cell += 4 * static_cast<size_t>(nchunks);
                }
                for (; x < x1; ++x) {
                    E::accumulate(load_stream(cell), acc);
                    cell += nchunks;
                }
            }
            const float cnt = static_cast<float>((y1 - y0) * (x1 - x0));
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = acc[i] / cnt;
            Store<TO>::put(out + out_row * d, chunk, E::kVec, acc);
        }
        if (lane == 0 && item - orow * colparts == 0) token_event[out_row] = ev;
    }
}

// ---------------------------------------------------------------------------------------------
// frame_stats_pool2_kernel: the statistics of frame_stats_kernel (Eq. 4 over all entries, Eq. 5) and the
// 2 x 2 mean pooling of every frame in ONE pass over V, for the case in which every frame is pooled with
// stride 2 whatever the segmentation turns out to be (all four strides of the adaptive rule equal 2), on
// a grid with even sides.  A wave owns one pooling window: lane j holds the 16-byte chunks j, j + 64, ...
// (at most KL) of the window's four tokens, so the pooled chunk is a sum inside the lane (cells in the
// order (y, x), (y, x+1), (y+1, x), (y+1, x+1), the order pool_kernel uses) and the per-token reductions
// run over the whole wave.  blockIdx.y = run of frames; a wave walks its run with two row sets: while it
// works on frame t the rows of frame t + 1 are in flight, and <v_t, v_{t+1}> is taken when they land.
// Waves are independent (no LDS, no barrier): each writes its own partials
//     part[(t * n_win + w) * 3 + {0, 1, 2}] = sum |v|^2, <v_t, v_{t+1}>, sum of cos(token, text)
// over the four tokens of window w of frame t.  pooled[(t * n_win + w) * d ...] receives the pooled token.
//
// Reductions.  The eight per-token sums of a frame (|v|^2 and <v, text> of four tokens) are reduced together:
// v_permlane32_swap / v_permlane16_swap exchange halves of two registers, so one swap and one add fold two
// values at once, and after two such steps every 16-lane row holds one pair of values to finish with DPP
// adds -- about 45 vector instructions per frame instead of nine separate 64-lane reductions.
// ---------------------------------------------------------------------------------------------
template <typename T, int KL, typename TO>
__global__ __launch_bounds__(kStatsThreads) void frame_stats_pool2_kernel(
    const T* __restrict__ feats, const T* __restrict__ text, int T_frames, int grid_h, int grid_w, int d,
    int frames_per_run, float* __restrict__ part, TO* __restrict__ pooled, int64_t pooled_video, int64_t ws_video) {
    using E = Elem<T>;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ow = grid_w / 2, n_win = (grid_h / 2) * ow, N = grid_h * grid_w;
    feats = of_video_elems(feats, static_cast<int64_t>(T_frames) * N * d); text = of_video_elems(text, d);
    part = of_video(part, ws_video); pooled = of_video_elems(pooled, pooled_video);
    const int w = blockIdx.x * kStatsWaves + wave;
    if (w >= n_win) return;                                          // there is no barrier below: a wave may leave on its own
    const int wy = w / ow, wx = w % ow;
    const int nchunks = d / E::kVec;
    const int t0 = blockIdx.y * frames_per_run;
    const int t1 = min(T_frames, t0 + frames_per_run);
    const uint4 zero = make_uint4(0, 0, 0, 0);
    int tok[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) tok[c] = (2 * wy + (c >> 1)) * grid_w + 2 * wx + (c & 1);

    uint4 txt[KL];
    float tn2 = 0.f;
#pragma unroll
    for (int k = 0; k < KL; ++k) {
        const int ch = lane + 64 * k;
        txt[k] = ch < nchunks ? reinterpret_cast<const uint4*>(text)[ch] : zero;
        tn2 = E::dot(txt[k], txt[k], tn2);
    }
    const float tnorm = sqrtf(wave_sum(tn2));

    // Loads are branch-free -- lanes past the last chunk read the row's last chunk again, the step behind the last frame
    // reads the last frame again -- so that the compiler can count the loads in flight and wait for exactly the
    // older ones; what such a lane loaded is masked where it is used.
    bool valid[KL];
    int chc[KL];
#pragma unroll
    for (int k = 0; k < KL; ++k) {
        const int ch = lane + 64 * k;
        valid[k] = ch < nchunks;
        chc[k] = valid[k] ? ch : nchunks - 1;
    }
    auto load_rows = [&](int t, uint4 (&dst)[4][KL]) {
        const int tc = t < T_frames ? t : T_frames - 1;
        const uint4* frame = reinterpret_cast<const uint4*>(feats) + static_cast<size_t>(tc) * N * nchunks;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const uint4* row = frame + static_cast<size_t>(tok[c]) * nchunks;
#pragma unroll
            for (int k = 0; k < KL; ++k) dst[c][k] = load_stream(row + chc[k]);
        }
    };
    // X holds frame t; Y receives frame t + 1 while X is worked on.  Order inside a step: request Y, all arithmetic
    // on X alone, then <X, Y> (the first use of Y: the only wait of the step), then the stores -- a store issued
    // earlier would be waited for together with Y.
    auto step = [&](int t, uint4 (&X)[4][KL], uint4 (&Y)[4][KL]) {
        const bool has_next = t + 1 < T_frames;
        load_rows(t + 1, Y);
        float p[4], q[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            p[c] = 0.f; q[c] = 0.f;
#pragma unroll
            for (int k = 0; k < KL; ++k) {
                const float pk = E::dot(X[c][k], X[c][k], 0.f);
                p[c] += valid[k] ? pk : 0.f;
                q[c] = E::dot(X[c][k], txt[k], q[c]);               // txt is zero past the last chunk
            }
        }
        float pooled_acc[KL][8];
#pragma unroll
        for (int k = 0; k < KL; ++k) {
#pragma unroll
            for (int i = 0; i < 8; ++i) pooled_acc[k][i] = 0.f;
#pragma unroll
            for (int c = 0; c < 4; ++c) E::accumulate(X[c][k], pooled_acc[k]);
#pragma unroll
            for (int i = 0; i < 8; ++i) pooled_acc[k][i] = pooled_acc[k][i] / 4.f;
        }
        // after the two halving steps rows 0 / 1 hold |v|^2 of the tokens (0, 2) / (1, 3) in (u0, u1), rows 2 / 3 their text products
        const float s0 = swap32_add(p[0], q[0]), s1 = swap32_add(p[1], q[1]), s2 = swap32_add(p[2], q[2]), s3 = swap32_add(p[3], q[3]);
        const float u0 = row16_sum(swap16_add(s0, s1)), u1 = row16_sum(swap16_add(s2, s3));
        // both halves of the wave get the norms (first result) and the text products (second result) of their tokens
        const auto r0 = __builtin_amdgcn_permlane32_swap(__float_as_uint(u0), __float_as_uint(u0), false, false);
        const auto r1 = __builtin_amdgcn_permlane32_swap(__float_as_uint(u1), __float_as_uint(u1), false, false);
        const float pa = __uint_as_float(r0[0]), qa = __uint_as_float(r0[1]), pb = __uint_as_float(r1[0]), qb = __uint_as_float(r1[1]);
        const float da = sqrtf(pa) * tnorm, db = sqrtf(pb) * tnorm;
        const float cosv = (!(da < kZeroNorm) ? qa / da : 0.f) + (!(db < kZeroNorm) ? qb / db : 0.f);
        const float tot = swap16_add(cosv, pa + pb);                  // row 0: the four cosines added; row 1: the four |v|^2 added
        __builtin_amdgcn_sched_barrier(0);
        float cd = 0.f;
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int k = 0; k < KL; ++k) {
                const float ck = E::dot(X[c][k], Y[c][k], 0.f);
                cd += (valid[k] && has_next) ? ck : 0.f;
            }
        cd = row16_sum(cd);
        cd = swap32_add(cd, cd);
        cd = swap16_add(cd, cd);                                      // row 0: all four rows
        __builtin_amdgcn_sched_barrier(0);
        TO* out_row = pooled + (static_cast<size_t>(t) * n_win + w) * d;
#pragma unroll
        for (int k = 0; k < KL; ++k)
            if (valid[k]) Store<TO>::put(out_row, lane + 64 * k, E::kVec, pooled_acc[k]);
        float* dst = part + (static_cast<size_t>(t) * n_win + w) * 3;
        if (lane == 0) { dst[1] = cd; dst[2] = tot; }
        if (lane == 16) dst[0] = tot;
    };
    uint4 A[4][KL], B[4][KL];
    load_rows(t0, A);
    // the first frame has landed before the loop: inside it the only wait is the one for the frame requested in the same step
    __builtin_amdgcn_s_waitcnt(0);
    for (int t = t0; t < t1; t += 2) {
        step(t, A, B);
        if (t + 1 < t1) step(t + 1, B, A);
    }
}

// token_event of uniformly pooled frames: rows_per_frame consecutive rows carry their frame's event id.
__global__ __launch_bounds__(256) void fill_token_event_kernel(const int32_t* __restrict__ frame_event, int T, int rows_per_frame,
                                                               int32_t* __restrict__ token_event, int64_t rows_video) {
    frame_event = of_video_elems(frame_event, T); token_event = of_video_elems(token_event, rows_video);
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < T * rows_per_frame) token_event[i] = frame_event[i / rows_per_frame];
}

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
struct StatsPlan {
    int G, KL, tok_per_wg, C, frames_per_run, runs;
};

static bool plan_stats(int T, int N, int d, int dtype, StatsPlan* p) {
    const int vec = dtype == METOK_BF16 ? 8 : 4;
    if (d % vec) return false;
    const int nchunks = d / vec;
    int G = 16, KL = 0;
    for (int g : {16, 64}) {
        for (int kl : {1, 2, 4, 8, 16}) {
            if (g == 16 && kl == 16) continue;
            if (g * kl >= nchunks) { G = g; KL = kl; break; }
        }
        if (KL) break;
    }
    if (!KL) return false;
    p->G = G; p->KL = KL;
    p->tok_per_wg = kStatsWaves * (64 / G);
    p->C = (N + 64 / G - 1) / (64 / G);                 // wave chunks per frame: one partial triple each
    // about 2048 waves to fill 256 CUs twice over, but runs of at least 4 frames so that the extra frame read
    // per run stays a small fraction
    int runs = (2048 + p->C - 1) / p->C;
    int fpr = (T + runs - 1) / runs;
    if (fpr < 4) fpr = 4;
    // runs advance in step, their frames lie fpr frames apart: multiples of 8 frames put the runs' reads on the
    // same DRAM channels and banks (measured 20 % slower)
    if (fpr % 8 == 0) ++fpr;
    if (fpr > T) fpr = T;
    p->frames_per_run = fpr;
    p->runs = (T + fpr - 1) / fpr;
    return true;
}

template <typename T, int G, int KL>
static void launch_stats(const void* feats, const void* text, int Tf, int N, int d, const StatsPlan& p, int do_pair,
                         int sim_mode, float* part, hipStream_t st, int batch, int64_t ws_video) {
    { TraceScope trace_scope(METOK_TRACE_FRAME_STATS, st); hipLaunchKernelGGL((frame_stats_kernel<T, G, KL>), dim3((p.C + kStatsWaves - 1) / kStatsWaves, p.runs, batch), dim3(kStatsThreads), 0, st,
                       static_cast<const T*>(feats), static_cast<const T*>(text), Tf, N, d, p.frames_per_run, do_pair,
                       sim_mode, part, p.C, ws_video); }
}

template <typename T>
static bool dispatch_stats(const void* feats, const void* text, int Tf, int N, int d, const StatsPlan& p, int do_pair,
                           int sim_mode, float* part, hipStream_t st, int batch = 1, int64_t ws_video = 0) {
#define METOK_STATS_CASE(g, kl) \
    if (p.G == g && p.KL == kl) { launch_stats<T, g, kl>(feats, text, Tf, N, d, p, do_pair, sim_mode, part, st, batch, ws_video); return true; }
    METOK_STATS_CASE(16, 1) METOK_STATS_CASE(16, 2) METOK_STATS_CASE(16, 4) METOK_STATS_CASE(16, 8)
    METOK_STATS_CASE(64, 1) METOK_STATS_CASE(64, 2) METOK_STATS_CASE(64, 4) METOK_STATS_CASE(64, 8) METOK_STATS_CASE(64, 16)
#undef METOK_STATS_CASE
    return false;
}

static size_t stats_part_bytes(int T, const StatsPlan& p) {
    return round_up(static_cast<size_t>(T) * p.C * 3 * sizeof(float), 256);
}

static int check_feats(const void* feats, int dtype, int T, int N, int d, StatsPlan* p) {
    if (dtype != METOK_F32 && dtype != METOK_BF16) return fail(METOK_ERR_INVALID_ARG, "unknown dtype %d", dtype);
    if (T < 1 || T > METOK_MAX_FRAMES) return fail(METOK_ERR_INVALID_ARG, "T must be in [1, %d], got %d", METOK_MAX_FRAMES, T);
    if (N < 1 || d < 1) return fail(METOK_ERR_INVALID_ARG, "N and d must be positive");
    if (static_cast<int64_t>(T) * N > INT32_MAX) return fail(METOK_ERR_INVALID_ARG, "T * N must fit int32");
    if (!feats || !aligned16(feats)) return fail(METOK_ERR_INVALID_ARG, "feats is NULL or not 16-byte aligned");
    if (!plan_stats(T, N, d, dtype, p))
        return fail(METOK_ERR_UNSUPPORTED, "d = %d: need a multiple of %d and at most %d", d, dtype == METOK_BF16 ? 8 : 4,
                    dtype == METOK_BF16 ? 8192 : 4096);
    return METOK_OK;
}

}  // namespace metok

using namespace metok;

// workspace: [chunk partials of V] [norm2 T] [pair T] [token-mean vectors T*d fp32] [chunk partials of the means]
static size_t mean_bytes(int T, int d) { return round_up(static_cast<size_t>(T) * d * sizeof(float), 256); }

extern "C" size_t metok_segment_events_workspace_bytes(int T, int N, int d, int dtype) {
    StatsPlan p, pm;
    if (T < 1 || N < 1 || d < 1 || !plan_stats(T, N, d, dtype, &p)) return 0;
    size_t total = stats_part_bytes(T, p) + 2 * round_up(static_cast<size_t>(T) * sizeof(float), 256);
    if (plan_stats(T, 1, d, METOK_F32, &pm)) total += mean_bytes(T, d) + stats_part_bytes(T, pm);     // pooled mode
    return total;
}

extern "C" int metok_segment_events(const void* feats, int dtype, int T, int N, int d,
                                    const void* text_emb, int k, int sim_mode,
                                    float* sim, int32_t* event_start, int32_t* frame_event,
                                    float* frame_score,
                                    void* workspace, size_t workspace_bytes, void* stream) {
    clear_error();
    StatsPlan p;
    int rc = check_feats(feats, dtype, T, N, d, &p);
    if (rc) return rc;
    if (sim_mode != METOK_SIM_FLAT && sim_mode != METOK_SIM_TOKEN_MEAN && sim_mode != METOK_SIM_POOLED)
        return fail(METOK_ERR_INVALID_ARG, "unknown sim_mode %d", sim_mode);
    if (k < 1 || k > T) return fail(METOK_ERR_INVALID_ARG, "k must be in [1, T] (k=%d, T=%d)", k, T);
    if (!event_start || !frame_event || (T > 1 && !sim)) return fail(METOK_ERR_INVALID_ARG, "NULL output pointer");
    if (frame_score && !text_emb) return fail(METOK_ERR_INVALID_ARG, "frame_score requested without text_emb");
    if (text_emb && !aligned16(text_emb)) return fail(METOK_ERR_INVALID_ARG, "text_emb not 16-byte aligned");
    StatsPlan pm;
    const bool can_pool = plan_stats(T, 1, d, METOK_F32, &pm);
    if (sim_mode == METOK_SIM_POOLED && !can_pool)
        return fail(METOK_ERR_UNSUPPORTED, "pooled similarity needs d <= 4096, got %d", d);
    const size_t need = metok_segment_events_workspace_bytes(T, N, d, dtype);
    if (!workspace || workspace_bytes < need || !aligned16(workspace))
        return fail(METOK_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    char* ws = static_cast<char*>(workspace);
    const size_t tslot = round_up(static_cast<size_t>(T) * sizeof(float), 256);
    float* part = reinterpret_cast<float*>(ws);
    float* norm2 = reinterpret_cast<float*>(ws + stats_part_bytes(T, p));
    float* pair_dot = reinterpret_cast<float*>(ws + stats_part_bytes(T, p) + tslot);
    hipStream_t st = static_cast<hipStream_t>(stream);

    if (sim_mode != METOK_SIM_POOLED) {
        const bool ok = dtype == METOK_BF16 ? dispatch_stats<bf16_t>(feats, text_emb, T, N, d, p, 1, sim_mode, part, st)
                                            : dispatch_stats<float>(feats, text_emb, T, N, d, p, 1, sim_mode, part, st);
        if (!ok) return fail(METOK_ERR_UNSUPPORTED, "no frame-statistics kernel for d = %d", d);
        if ((rc = check_launch("frame_stats"))) return rc;
        { TraceScope trace_scope(METOK_TRACE_SEGMENT, st); hipLaunchKernelGGL(segment_kernel, dim3(1), dim3(kSegThreads), 0, st, part, p.C, T, N, k, text_emb ? 1 : 0, sim_mode,
                           sim, event_start, frame_event, frame_score, norm2, pair_dot, static_cast<int64_t>(0)); }
        return check_launch("segment");
    }
    // pooled reading: Eq. 5 (if wanted) from the tokens, Eq. 4 from the frames' mean tokens (a [T, 1, d] fp32 "video")
    if (text_emb && frame_score) {
        const bool ok = dtype == METOK_BF16 ? dispatch_stats<bf16_t>(feats, text_emb, T, N, d, p, 0, METOK_SIM_FLAT, part, st)
                                            : dispatch_stats<float>(feats, text_emb, T, N, d, p, 0, METOK_SIM_FLAT, part, st);
        if (!ok) return fail(METOK_ERR_UNSUPPORTED, "no frame-statistics kernel for d = %d", d);
        if ((rc = check_launch("frame_stats"))) return rc;
        hipLaunchKernelGGL(frame_score_kernel, dim3(1), dim3(kSegThreads), 0, st, part, p.C, T, N, frame_score);
        if ((rc = check_launch("frame_score"))) return rc;
    }
    float* mean = reinterpret_cast<float*>(ws + stats_part_bytes(T, p) + 2 * tslot);
    float* part_m = reinterpret_cast<float*>(ws + stats_part_bytes(T, p) + 2 * tslot + mean_bytes(T, d));
    const int vec = dtype == METOK_BF16 ? 8 : 4;
    dim3 mgrid(T, (d / vec + 63) / 64);
    if (dtype == METOK_BF16)
        hipLaunchKernelGGL(frame_mean_kernel<bf16_t>, mgrid, dim3(256), 0, st, static_cast<const bf16_t*>(feats), N, d, mean);
    else
        hipLaunchKernelGGL(frame_mean_kernel<float>, mgrid, dim3(256), 0, st, static_cast<const float*>(feats), N, d, mean);
    if ((rc = check_launch("frame_mean"))) return rc;
    if (!dispatch_stats<float>(mean, nullptr, T, 1, d, pm, 1, METOK_SIM_FLAT, part_m, st))
        return fail(METOK_ERR_UNSUPPORTED, "no frame-statistics kernel for d = %d", d);
    if ((rc = check_launch("frame_stats (means)"))) return rc;
    { TraceScope trace_scope(METOK_TRACE_SEGMENT, st); hipLaunchKernelGGL(segment_kernel, dim3(1), dim3(kSegThreads), 0, st, part_m, pm.C, T, 1, k, 0, METOK_SIM_FLAT,
                       sim, event_start, frame_event, static_cast<float*>(nullptr), norm2, pair_dot, static_cast<int64_t>(0)); }
    return check_launch("segment");
}

// Pooled rows when every frame takes the smaller of the two strides (s / alpha >= s, so no frame yields more).
static int64_t worst_case_rows(int T, int grid_h, int grid_w, int s1, int s2, int pool_edge) {
    const int gmax = grid_h > grid_w ? grid_h : grid_w;
    int s_min = s1 < s2 ? s1 : s2;
    s_min = s_min < 1 ? 1 : (s_min > gmax ? gmax : s_min);
    auto side = [&](int g) { return pool_edge == METOK_POOL_FLOOR ? (g / s_min > 1 ? g / s_min : 1) : (g + s_min - 1) / s_min; };
    return static_cast<int64_t>(T) * side(grid_h) * side(grid_w);
}

extern "C" int64_t metok_compress_encoder_tokens_capacity_rows(int T, int grid_h, int grid_w, int s1, int s2, int pool_edge) {
    if (T < 1 || T > METOK_MAX_FRAMES || grid_h < 1 || grid_w < 1 || static_cast<int64_t>(grid_h) * grid_w > (1 << 24) || s1 < 1 || s2 < 1 ||
        (pool_edge != METOK_POOL_FLOOR && pool_edge != METOK_POOL_CEIL))
        return -1;
    return worst_case_rows(T, grid_h, grid_w, s1, s2, pool_edge);
}

extern "C" size_t metok_compress_encoder_tokens_workspace_bytes(int T, int grid_h, int grid_w, int d, int dtype) {
    StatsPlan p;
    if (T < 1 || grid_h < 1 || grid_w < 1 || d < 1 || !plan_stats(T, grid_h * grid_w, d, dtype, &p)) return 0;
    // stats partials + frame norms + frame scores + frame -> event table
    return stats_part_bytes(T, p) + 3 * round_up(static_cast<size_t>(T) * sizeof(float), 256);
}

extern "C" int metok_compress_encoder_tokens(const void* feats, int dtype, int T, int grid_h, int grid_w, int d,
                                             const void* text_emb, const float* frame_score_in,
                                             const int32_t* event_start, int k,
                                             double alpha, double beta, int s1, int s2,
                                             int event_reduce, int pool_edge,
                                             void* out_tokens, int64_t out_capacity_rows, int out_dtype,
                                             int32_t* frame_offsets, int32_t* token_event,
                                             uint8_t* event_is_key, uint8_t* frame_is_key,
                                             int32_t* frame_stride, float* event_score, float* frame_score_out,
                                             void* workspace, size_t workspace_bytes, void* stream) {
    clear_error();
    if (grid_h < 1 || grid_w < 1 || static_cast<int64_t>(grid_h) * grid_w > (1 << 24))
        return fail(METOK_ERR_INVALID_ARG, "bad patch grid %d x %d", grid_h, grid_w);
    const int N = grid_h * grid_w;
    StatsPlan p;
    int rc = check_feats(feats, dtype, T, N, d, &p);
    if (rc) return rc;
    if (out_dtype != METOK_F32 && out_dtype != METOK_BF16) return fail(METOK_ERR_INVALID_ARG, "unknown out_dtype %d", out_dtype);
    if (k < 1 || k > T) return fail(METOK_ERR_INVALID_ARG, "k must be in [1, T] (k=%d, T=%d)", k, T);
    if (!(alpha > 0.0 && alpha <= 1.0) || !(beta > 0.0 && beta <= 1.0))
        return fail(METOK_ERR_INVALID_ARG, "need 0 < alpha, beta <= 1 (alpha=%g beta=%g)", alpha, beta);
    if (s1 < 1 || s2 < 1) return fail(METOK_ERR_INVALID_ARG, "strides must be >= 1 (s1=%d s2=%d)", s1, s2);
    if (event_reduce != METOK_EVENT_MEAN && event_reduce != METOK_EVENT_MAX)
        return fail(METOK_ERR_INVALID_ARG, "unknown event_reduce %d", event_reduce);
    if (pool_edge != METOK_POOL_FLOOR && pool_edge != METOK_POOL_CEIL)
        return fail(METOK_ERR_INVALID_ARG, "unknown pool_edge %d", pool_edge);
    if (!frame_score_in && !text_emb) return fail(METOK_ERR_INVALID_ARG, "need text_emb or frame_score_in");
    if (text_emb && !aligned16(text_emb)) return fail(METOK_ERR_INVALID_ARG, "text_emb not 16-byte aligned");
    if (!event_start || !out_tokens || !frame_offsets || !token_event || !event_is_key || !frame_is_key ||
        !frame_stride || !event_score)
        return fail(METOK_ERR_INVALID_ARG, "NULL pointer argument");
    if (!aligned16(out_tokens)) return fail(METOK_ERR_INVALID_ARG, "out_tokens not 16-byte aligned");
    if ((static_cast<size_t>(d) * dtype_size(out_dtype)) % 16)
        return fail(METOK_ERR_INVALID_ARG, "d * sizeof(out_dtype) must be a multiple of 16");

    const int gmax = grid_h > grid_w ? grid_h : grid_w;
    auto clamp_stride = [&](double s) { int v = ceil_ratio(s); return v < 1 ? 1 : (v > gmax ? gmax : v); };
    const int s_key_kf = clamp_stride(s1), s_key_nf = clamp_stride(s2);
    const int s_non_kf = clamp_stride(s1 / alpha), s_non_nf = clamp_stride(s2 / alpha);
    const int64_t worst = worst_case_rows(T, grid_h, grid_w, s1, s2, pool_edge);
    if (out_capacity_rows < worst)
        return fail(METOK_ERR_CAPACITY, "out_capacity_rows = %lld, worst case needs %lld", (long long)out_capacity_rows, (long long)worst);
    if (worst > INT32_MAX) return fail(METOK_ERR_INVALID_ARG, "pooled row count must fit int32");

    const size_t need = metok_compress_encoder_tokens_workspace_bytes(T, grid_h, grid_w, d, dtype);
    if (!workspace || workspace_bytes < need || !aligned16(workspace))
        return fail(METOK_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace_bytes);
    char* ws = static_cast<char*>(workspace);
    float* part = reinterpret_cast<float*>(ws);
    const size_t tslot = round_up(static_cast<size_t>(T) * sizeof(float), 256);
    float* norm2 = reinterpret_cast<float*>(ws + stats_part_bytes(T, p));
    float* score_ws = reinterpret_cast<float*>(ws + stats_part_bytes(T, p) + tslot);
    int32_t* frame_event_ws = reinterpret_cast<int32_t*>(ws + stats_part_bytes(T, p) + 2 * tslot);
    hipStream_t st = static_cast<hipStream_t>(stream);

    const float* scores = frame_score_in;
    if (!scores) {
        // Eq. 5 pass on its own (no adjacent-frame products)
        const bool ok = dtype == METOK_BF16 ? dispatch_stats<bf16_t>(feats, text_emb, T, N, d, p, 0, METOK_SIM_FLAT, part, st)
                                            : dispatch_stats<float>(feats, text_emb, T, N, d, p, 0, METOK_SIM_FLAT, part, st);
        if (!ok) return fail(METOK_ERR_UNSUPPORTED, "no frame-statistics kernel for d = %d", d);
        if ((rc = check_launch("frame_stats"))) return rc;
        hipLaunchKernelGGL(frame_score_kernel, dim3(1), dim3(kSegThreads), 0, st, part, p.C, T, N, score_ws);
        if ((rc = check_launch("frame_score"))) return rc;
        scores = score_ws;
    }
    (void)norm2;
    const int n_key_events = ceil_ratio(alpha * k) > k ? k : ceil_ratio(alpha * k);
    { TraceScope trace_scope(METOK_TRACE_PLAN, st); hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kSegThreads), 0, st, scores, event_start, T, k, n_key_events, beta,
                       s_key_kf, s_key_nf, s_non_kf, s_non_nf, grid_h, grid_w, event_reduce, pool_edge,
                       event_score, event_is_key, frame_is_key, frame_stride, frame_offsets, frame_event_ws,
                       frame_score_out, static_cast<int64_t>(0)); }
    if ((rc = check_launch("plan"))) return rc;

    const int wg_per_frame = 36;      // 144 waves per frame; 18 to 72 workgroups measured within 3 % of each other
    dim3 grid(wg_per_frame, T);
#define METOK_POOL_CASE(TI, TO) \
    { TraceScope trace_scope(METOK_TRACE_POOL, st); \
      hipLaunchKernelGGL((pool_kernel<TI, TO>), grid, dim3(kPoolThreads), 0, st, static_cast<const TI*>(feats), grid_h, grid_w, d, \
                         frame_stride, frame_offsets, frame_event_ws, pool_edge, out_capacity_rows, static_cast<TO*>(out_tokens), token_event, \
                         T, static_cast<int64_t>(0)); }
    if (dtype == METOK_BF16 && out_dtype == METOK_BF16) METOK_POOL_CASE(bf16_t, bf16_t)
    else if (dtype == METOK_BF16 && out_dtype == METOK_F32) METOK_POOL_CASE(bf16_t, float)
    else if (dtype == METOK_F32 && out_dtype == METOK_BF16) METOK_POOL_CASE(float, bf16_t)
    else METOK_POOL_CASE(float, float)
#undef METOK_POOL_CASE
    return check_launch("pool");
}

// ---------------------------------------------------------------------------------------------
// Stage 1 in one call.  When every frame is pooled with stride 2 whatever the segmentation decides
// (all four strides of the adaptive rule are 2, even grid), the statistics and the pooled tokens come
// out of ONE pass over V; otherwise the two calls above run back to back (two passes over V).
// ---------------------------------------------------------------------------------------------
// one-pass path: one partial triple per pooling window and frame, then the per-frame arrays of the small kernels
static size_t fused_part_bytes(int T, int grid_h, int grid_w) {
    return round_up(static_cast<size_t>(T) * (grid_h / 2) * (grid_w / 2) * 3 * sizeof(float), 256);
}

extern "C" size_t metok_segment_compress_workspace_bytes(int T, int grid_h, int grid_w, int d, int dtype) {
    if (grid_h < 1 || grid_w < 1 || T < 1) return 0;
    const size_t a = metok_segment_events_workspace_bytes(T, grid_h * grid_w, d, dtype);
    const size_t b = metok_compress_encoder_tokens_workspace_bytes(T, grid_h, grid_w, d, dtype);
    const size_t c = fused_part_bytes(T, grid_h, grid_w) + 3 * round_up(static_cast<size_t>(T) * sizeof(float), 256);
    const size_t ab = a > b ? a : b;
    return round_up(ab > c ? ab : c, 256);
}

// Streaming kernels here run fastest with FEW waves per CU: each wave keeps a whole frame step of loads in flight, and
// more resident waves only queue more requests at the memory system (measured for the one-pass kernel, 8 videos:
// 636 us with 8 workgroups per CU, 612 us with 2, 580 us with 1).  The launch therefore asks for more than half of a
// CU's 160 KB of LDS, which the kernel never touches: one workgroup per CU.
constexpr unsigned kOneWorkgroupPerCuLds = 96 * 1024;

template <typename T, typename TO>
static bool launch_stats_pool2(const void* feats, const void* text, int Tf, int grid_h, int grid_w, int d, int kl, int C, int fpr,
                               int runs, float* part, void* pooled, int batch, int64_t pooled_video, int64_t ws_video, hipStream_t st) {
#define METOK_FUSED_CASE(KLV) \
    if (kl == KLV) { \
        static bool lds_allowed[64] = {false};        /* per device: the attribute belongs to the device's copy of the kernel */ \
        int dev = 0; \
        if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return false; \
        if (!lds_allowed[dev]) { \
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(&frame_stats_pool2_kernel<T, KLV, TO>), \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kOneWorkgroupPerCuLds) != hipSuccess) return false; \
            lds_allowed[dev] = true; \
        } \
        { TraceScope trace_scope(METOK_TRACE_FRAME_STATS_POOL2, st); hipLaunchKernelGGL((frame_stats_pool2_kernel<T, KLV, TO>), dim3(C, runs, batch), dim3(kStatsThreads), kOneWorkgroupPerCuLds, st, static_cast<const T*>(feats), \
                           static_cast<const T*>(text), Tf, grid_h, grid_w, d, fpr, part, static_cast<TO*>(pooled), pooled_video, ws_video); } \
        return true; \
    }
    METOK_FUSED_CASE(1) METOK_FUSED_CASE(2) METOK_FUSED_CASE(3) METOK_FUSED_CASE(4)
#undef METOK_FUSED_CASE
    return false;
}

// Shared body of metok_segment_compress (batch = 1) and metok_segment_compress_batched: every array carries a leading
// dimension of `batch` videos, the workspace one slice per video; every kernel takes the video from blockIdx.z.
static int segment_compress_impl(int batch, const void* feats, int dtype, int T, int grid_h, int grid_w, int d,
                                 const void* text_emb, int k, int sim_mode,
                                 double alpha, double beta, int s1, int s2, int event_reduce, int pool_edge,
                                 float* sim, int32_t* event_start, int32_t* frame_event,
                                 void* out_tokens, int64_t out_capacity_rows, int out_dtype,
                                 int32_t* frame_offsets, int32_t* token_event,
                                 uint8_t* event_is_key, uint8_t* frame_is_key,
                                 int32_t* frame_stride, float* event_score, float* frame_score,
                                 void* workspace, size_t workspace_bytes, void* stream) {
    if (batch < 1 || batch > METOK_MAX_BATCH) return fail(METOK_ERR_INVALID_ARG, "batch must be in [1, %d]", METOK_MAX_BATCH);
    if (grid_h < 1 || grid_w < 1) return fail(METOK_ERR_INVALID_ARG, "grid sides must be positive");
    if (!text_emb || !frame_score) return fail(METOK_ERR_INVALID_ARG, "text_emb and frame_score are required (Eq. 5 drives the pooling plan)");
    const int N = grid_h * grid_w;
    const size_t need = metok_segment_compress_workspace_bytes(T, grid_h, grid_w, d, dtype);        // per video, a multiple of 256
    if (need && (!workspace || workspace_bytes < need * batch || !aligned16(workspace)))
        return fail(METOK_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need * batch, workspace_bytes);
    const int64_t ws_video = static_cast<int64_t>(need);

    // can the pooled tokens be produced inside the statistics pass?
    bool fused = sim_mode == METOK_SIM_FLAT && grid_h % 2 == 0 && grid_w % 2 == 0 && alpha > 0.0 && alpha <= 1.0 && s1 >= 1 && s2 >= 1 &&
                 (dtype == METOK_F32 || dtype == METOK_BF16) && (out_dtype == METOK_F32 || out_dtype == METOK_BF16);
    if (fused) {
        const int gmax = grid_h > grid_w ? grid_h : grid_w;
        auto clamp_stride = [&](double s) { int v = ceil_ratio(s); return v < 1 ? 1 : (v > gmax ? gmax : v); };
        fused = clamp_stride(s1) == 2 && clamp_stride(s2) == 2 && clamp_stride(s1 / alpha) == 2 && clamp_stride(s2 / alpha) == 2;
    }
    const int vec = dtype == METOK_BF16 ? 8 : 4;
    const int kl = (d > 0 && d % vec == 0) ? (d / vec + 63) / 64 : 0;
    if (kl < 1 || kl > 4) fused = false;
    if (!fused && batch > 1 && (sim_mode == METOK_SIM_FLAT || sim_mode == METOK_SIM_TOKEN_MEAN)) {
        // two passes (statistics, then pooling with the strides of Algorithm 1), each kernel once for the whole batch
        StatsPlan p;
        int rc = check_feats(feats, dtype, T, N, d, &p);
        if (rc) return rc;
        if (out_dtype != METOK_F32 && out_dtype != METOK_BF16) return fail(METOK_ERR_INVALID_ARG, "unknown out_dtype %d", out_dtype);
        if (k < 1 || k > T) return fail(METOK_ERR_INVALID_ARG, "k must be in [1, T] (k=%d, T=%d)", k, T);
        if (!(alpha > 0.0 && alpha <= 1.0) || !(beta > 0.0 && beta <= 1.0))
            return fail(METOK_ERR_INVALID_ARG, "need 0 < alpha, beta <= 1 (alpha=%g beta=%g)", alpha, beta);
        if (s1 < 1 || s2 < 1) return fail(METOK_ERR_INVALID_ARG, "strides must be >= 1 (s1=%d s2=%d)", s1, s2);
        if (event_reduce != METOK_EVENT_MEAN && event_reduce != METOK_EVENT_MAX)
            return fail(METOK_ERR_INVALID_ARG, "unknown event_reduce %d", event_reduce);
        if (pool_edge != METOK_POOL_FLOOR && pool_edge != METOK_POOL_CEIL)
            return fail(METOK_ERR_INVALID_ARG, "unknown pool_edge %d", pool_edge);
        if (!event_start || !frame_event || (T > 1 && !sim) || !out_tokens || !frame_offsets || !token_event || !event_is_key ||
            !frame_is_key || !frame_stride || !event_score)
            return fail(METOK_ERR_INVALID_ARG, "NULL pointer argument");
        if (!aligned16(text_emb) || !aligned16(out_tokens)) return fail(METOK_ERR_INVALID_ARG, "text_emb / out_tokens not 16-byte aligned");
        if ((static_cast<size_t>(d) * dtype_size(dtype)) % 16 || (static_cast<size_t>(d) * dtype_size(out_dtype)) % 16)
            return fail(METOK_ERR_INVALID_ARG, "d * sizeof(dtype) must be a multiple of 16 for the features and the pooled tokens");
        if (static_cast<int64_t>(grid_h) * grid_w > (1 << 24)) return fail(METOK_ERR_INVALID_ARG, "bad patch grid %d x %d", grid_h, grid_w);
        const int gmax = grid_h > grid_w ? grid_h : grid_w;
        auto clamp_stride = [&](double v) { int c = ceil_ratio(v); return c < 1 ? 1 : (c > gmax ? gmax : c); };
        const int64_t worst = worst_case_rows(T, grid_h, grid_w, s1, s2, pool_edge);
        if (out_capacity_rows < worst)
            return fail(METOK_ERR_CAPACITY, "out_capacity_rows = %lld, worst case needs %lld", (long long)out_capacity_rows, (long long)worst);
        if (worst > INT32_MAX) return fail(METOK_ERR_INVALID_ARG, "pooled row count must fit int32");
        char* ws = static_cast<char*>(workspace);
        const size_t tslot = round_up(static_cast<size_t>(T) * sizeof(float), 256);
        float* part = reinterpret_cast<float*>(ws);
        float* norm2 = reinterpret_cast<float*>(ws + stats_part_bytes(T, p));
        float* pair_dot = reinterpret_cast<float*>(ws + stats_part_bytes(T, p) + tslot);
        int32_t* frame_event_ws = reinterpret_cast<int32_t*>(ws + stats_part_bytes(T, p) + 2 * tslot);
        hipStream_t st = static_cast<hipStream_t>(stream);
        const unsigned nb = static_cast<unsigned>(batch);
        const bool ok = dtype == METOK_BF16 ? dispatch_stats<bf16_t>(feats, text_emb, T, N, d, p, 1, sim_mode, part, st, batch, ws_video)
                                            : dispatch_stats<float>(feats, text_emb, T, N, d, p, 1, sim_mode, part, st, batch, ws_video);
        if (!ok) return fail(METOK_ERR_UNSUPPORTED, "no frame-statistics kernel for d = %d", d);
        if ((rc = check_launch("frame_stats"))) return rc;
        { TraceScope trace_scope(METOK_TRACE_SEGMENT, st); hipLaunchKernelGGL(segment_kernel, dim3(1, 1, nb), dim3(kSegThreads), 0, st, part, p.C, T, N, k, 1, sim_mode,
                           sim, event_start, frame_event, frame_score, norm2, pair_dot, ws_video); }
        if ((rc = check_launch("segment"))) return rc;
        const int n_key_events = ceil_ratio(alpha * k) > k ? k : ceil_ratio(alpha * k);
        { TraceScope trace_scope(METOK_TRACE_PLAN, st); hipLaunchKernelGGL(plan_kernel, dim3(1, 1, nb), dim3(kSegThreads), 0, st, frame_score, event_start, T, k, n_key_events, beta,
                           clamp_stride(s1), clamp_stride(s2), clamp_stride(s1 / alpha), clamp_stride(s2 / alpha), grid_h, grid_w, event_reduce, pool_edge,
                           event_score, event_is_key, frame_is_key, frame_stride, frame_offsets, frame_event_ws,
                           static_cast<float*>(nullptr), ws_video); }
        if ((rc = check_launch("plan"))) return rc;
        dim3 grid(36, T, nb);
#define METOK_POOL_CASE(TI, TO) \
        { TraceScope trace_scope(METOK_TRACE_POOL, st); \
          hipLaunchKernelGGL((pool_kernel<TI, TO>), grid, dim3(kPoolThreads), 0, st, static_cast<const TI*>(feats), grid_h, grid_w, d, \
                             frame_stride, frame_offsets, frame_event_ws, pool_edge, out_capacity_rows, static_cast<TO*>(out_tokens), token_event, \
                             T, ws_video); }
        if (dtype == METOK_BF16 && out_dtype == METOK_BF16) METOK_POOL_CASE(bf16_t, bf16_t)
        else if (dtype == METOK_BF16 && out_dtype == METOK_F32) METOK_POOL_CASE(bf16_t, float)
        else if (dtype == METOK_F32 && out_dtype == METOK_BF16) METOK_POOL_CASE(float, bf16_t)
        else METOK_POOL_CASE(float, float)
#undef METOK_POOL_CASE
        return check_launch("pool");
    }
    if (!fused) {
        // a single video, or the reading of Eq. 4 that needs the extra pass over token means: the two stage-1 calls
        // (statistics, then pooling with the strides of Algorithm 1), one video after the other
        const size_t in_es = dtype_size(dtype), out_es = dtype_size(out_dtype);
        for (int b = 0; b < batch; ++b) {
            auto at = [&](auto* ptr, int64_t elems) { return ptr ? ptr + static_cast<int64_t>(b) * elems : ptr; };
            const char* f_b = static_cast<const char*>(feats) + static_cast<size_t>(b) * T * N * d * in_es;
            const char* t_b = static_cast<const char*>(text_emb) + static_cast<size_t>(b) * d * in_es;
            char* o_b = out_tokens ? static_cast<char*>(out_tokens) + static_cast<size_t>(b) * out_capacity_rows * d * out_es : nullptr;
            char* ws_b = static_cast<char*>(workspace) + static_cast<size_t>(b) * ws_video;
            int32_t* es_b = at(event_start, k + 1);
            float* fs_b = at(frame_score, T);
            int rc = metok_segment_events(f_b, dtype, T, N, d, t_b, k, sim_mode, at(sim, T - 1), es_b, at(frame_event, T), fs_b,
                                          ws_b, need, stream);
            if (rc) return rc;
            rc = metok_compress_encoder_tokens(f_b, dtype, T, grid_h, grid_w, d, nullptr, fs_b, es_b, k, alpha, beta, s1, s2,
                                               event_reduce, pool_edge, o_b, out_capacity_rows, out_dtype, at(frame_offsets, T + 1),
                                               at(token_event, out_capacity_rows), at(event_is_key, k), at(frame_is_key, T),
                                               at(frame_stride, T), at(event_score, k), nullptr, ws_b, need, stream);
            if (rc) return rc;
        }
        return METOK_OK;
    }
    // ---- one pass over V ------------------------------------------------------------------------
    StatsPlan p;
    int rc = check_feats(feats, dtype, T, N, d, &p);
    if (rc) return rc;
    if (k < 1 || k > T) return fail(METOK_ERR_INVALID_ARG, "k must be in [1, T] (k=%d, T=%d)", k, T);
    if (!(beta > 0.0 && beta <= 1.0)) return fail(METOK_ERR_INVALID_ARG, "need 0 < beta <= 1 (beta=%g)", beta);
    if (event_reduce != METOK_EVENT_MEAN && event_reduce != METOK_EVENT_MAX)
        return fail(METOK_ERR_INVALID_ARG, "unknown event_reduce %d", event_reduce);
    if (pool_edge != METOK_POOL_FLOOR && pool_edge != METOK_POOL_CEIL)
        return fail(METOK_ERR_INVALID_ARG, "unknown pool_edge %d", pool_edge);
    if (!event_start || !frame_event || (T > 1 && !sim) || !out_tokens || !frame_offsets || !token_event || !event_is_key ||
        !frame_is_key || !frame_stride || !event_score)
        return fail(METOK_ERR_INVALID_ARG, "NULL pointer argument");
    if (!aligned16(text_emb) || !aligned16(out_tokens)) return fail(METOK_ERR_INVALID_ARG, "text_emb / out_tokens not 16-byte aligned");
    if ((static_cast<size_t>(d) * dtype_size(out_dtype)) % 16)
        return fail(METOK_ERR_INVALID_ARG, "d * sizeof(out_dtype) must be a multiple of 16");
    const int n_win = (grid_h / 2) * (grid_w / 2);
    const int64_t rows = static_cast<int64_t>(T) * n_win;
    if (out_capacity_rows < rows)
        return fail(METOK_ERR_CAPACITY, "out_capacity_rows = %lld, worst case needs %lld", (long long)out_capacity_rows, (long long)rows);
    if (rows > INT32_MAX) return fail(METOK_ERR_INVALID_ARG, "pooled row count must fit int32");

    const int C = (n_win + kStatsWaves - 1) / kStatsWaves;          // workgroups per run of frames
    int runs = (2048 + C * kStatsWaves - 1) / (C * kStatsWaves);
    int fpr = (T + runs - 1) / runs;
    if (fpr < 4) fpr = 4;
    // Runs advance in step, so their frames lie fpr frames apart: a distance that is a multiple of 8 frames puts the
    // runs' reads on the same DRAM channels and banks (16 or 32 frames per run measured 20 % slower than 18 or 21).
    if (fpr % 8 == 0) ++fpr;
    if (fpr > T) fpr = T;
    runs = (T + fpr - 1) / fpr;
    char* ws = static_cast<char*>(workspace);
    const size_t part_bytes = fused_part_bytes(T, grid_h, grid_w);
    const size_t tslot = round_up(static_cast<size_t>(T) * sizeof(float), 256);
    float* part = reinterpret_cast<float*>(ws);
    float* norm2 = reinterpret_cast<float*>(ws + part_bytes);
    float* pair_dot = reinterpret_cast<float*>(ws + part_bytes + tslot);
    int32_t* frame_event_ws = reinterpret_cast<int32_t*>(ws + part_bytes + 2 * tslot);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t pooled_video = out_capacity_rows * d;
    const unsigned nb = static_cast<unsigned>(batch);
    bool ok;
    if (dtype == METOK_BF16)
        ok = out_dtype == METOK_BF16 ? launch_stats_pool2<bf16_t, bf16_t>(feats, text_emb, T, grid_h, grid_w, d, kl, C, fpr, runs, part, out_tokens, batch, pooled_video, ws_video, st)
                                     : launch_stats_pool2<bf16_t, float>(feats, text_emb, T, grid_h, grid_w, d, kl, C, fpr, runs, part, out_tokens, batch, pooled_video, ws_video, st);
    else
        ok = out_dtype == METOK_BF16 ? launch_stats_pool2<float, bf16_t>(feats, text_emb, T, grid_h, grid_w, d, kl, C, fpr, runs, part, out_tokens, batch, pooled_video, ws_video, st)
                                     : launch_stats_pool2<float, float>(feats, text_emb, T, grid_h, grid_w, d, kl, C, fpr, runs, part, out_tokens, batch, pooled_video, ws_video, st);
    if (!ok) return fail(METOK_ERR_UNSUPPORTED, "no fused kernel for d = %d", d);
    if ((rc = check_launch("frame_stats_pool2"))) return rc;
    { TraceScope trace_scope(METOK_TRACE_SEGMENT, st); hipLaunchKernelGGL(segment_kernel, dim3(1, 1, nb), dim3(kSegThreads), 0, st, part, n_win, T, N, k, 1, METOK_SIM_FLAT,
                       sim, event_start, frame_event, frame_score, norm2, pair_dot, ws_video); }
    if ((rc = check_launch("segment"))) return rc;
    const int n_key_events = ceil_ratio(alpha * k) > k ? k : ceil_ratio(alpha * k);
    { TraceScope trace_scope(METOK_TRACE_PLAN, st); hipLaunchKernelGGL(plan_kernel, dim3(1, 1, nb), dim3(kSegThreads), 0, st, frame_score, event_start, T, k, n_key_events, beta,
                       2, 2, 2, 2, grid_h, grid_w, event_reduce, pool_edge,
                       event_score, event_is_key, frame_is_key, frame_stride, frame_offsets, frame_event_ws,
                       static_cast<float*>(nullptr), ws_video); }
    if ((rc = check_launch("plan"))) return rc;
    hipLaunchKernelGGL(fill_token_event_kernel, dim3(static_cast<unsigned>((rows + 255) / 256), 1, nb), dim3(256), 0, st, frame_event, T, n_win,
                       token_event, out_capacity_rows);
    return check_launch("token events");
}

extern "C" int metok_segment_compress(const void* feats, int dtype, int T, int grid_h, int grid_w, int d,
                                      const void* text_emb, int k, int sim_mode,
                                      double alpha, double beta, int s1, int s2, int event_reduce, int pool_edge,
                                      float* sim, int32_t* event_start, int32_t* frame_event,
                                      void* out_tokens, int64_t out_capacity_rows, int out_dtype,
                                      int32_t* frame_offsets, int32_t* token_event,
                                      uint8_t* event_is_key, uint8_t* frame_is_key,
                                      int32_t* frame_stride, float* event_score, float* frame_score,
                                      void* workspace, size_t workspace_bytes, void* stream) {
    clear_error();
    return segment_compress_impl(1, feats, dtype, T, grid_h, grid_w, d, text_emb, k, sim_mode, alpha, beta, s1, s2, event_reduce, pool_edge,
                                 sim, event_start, frame_event, out_tokens, out_capacity_rows, out_dtype, frame_offsets, token_event,
                                 event_is_key, frame_is_key, frame_stride, event_score, frame_score, workspace, workspace_bytes, stream);
}

extern "C" size_t metok_segment_compress_batched_workspace_bytes(int batch, int T, int grid_h, int grid_w, int d, int dtype) {
    if (batch < 1 || batch > METOK_MAX_BATCH) return 0;
    return static_cast<size_t>(batch) * metok_segment_compress_workspace_bytes(T, grid_h, grid_w, d, dtype);
}

extern "C" int metok_segment_compress_batched(int batch, const void* feats, int dtype, int T, int grid_h, int grid_w, int d,
                                              const void* text_emb, int k, int sim_mode,
                                              double alpha, double beta, int s1, int s2, int event_reduce, int pool_edge,
                                              float* sim, int32_t* event_start, int32_t* frame_event,
                                              void* out_tokens, int64_t out_capacity_rows, int out_dtype,
                                              int32_t* frame_offsets, int32_t* token_event,
                                              uint8_t* event_is_key, uint8_t* frame_is_key,
                                              int32_t* frame_stride, float* event_score, float* frame_score,
                                              void* workspace, size_t workspace_bytes, void* stream) {
    clear_error();
    return segment_compress_impl(batch, feats, dtype, T, grid_h, grid_w, d, text_emb, k, sim_mode, alpha, beta, s1, s2, event_reduce,
                                 pool_edge, sim, event_start, frame_event, out_tokens, out_capacity_rows, out_dtype, frame_offsets,
                                 token_event, event_is_key, frame_is_key, frame_stride, event_score, frame_score, workspace,
                                 workspace_bytes, stream);
}
