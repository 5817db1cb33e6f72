// Shared declarations of the HIP implementation: handle layouts, error plumbing, wave/block primitives.
// gfx950 only: 64-wide wavefronts are assumed throughout.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "csv_decode.h"

// ---------------------------------------------------------------------------------------------- handles
struct csv_index {
    int V, d, C;
    int device;
    uint16_t* Wp;    // [V*d] bf16, rows permuted so that every cluster is a contiguous range
    float* bp;       // [V]   permuted bias (zeros when the head has none)
    int32_t* perm;   // [V]   permuted row -> original token id
    float* mu;       // [C*d] centroids, float32
    float* R;        // [C]   stored radii
    float* bmax;     // [C]   per-cluster bias maximum (-inf for an empty cluster)
    int32_t* n;      // [C]   rows per cluster
    int32_t* off;    // [C+1] first permuted row of each cluster
    float* lnn;      // [C]   ln n_c (-inf for an empty cluster)
};

enum { ST_ACTIVE = 0, ST_DONE = 1, ST_FALLBACK = 2, ST_INVALID = 3 };

struct SeqState {
    int status;
    int m0, m1;       // clusters open after round 0 / planned for round 1
    int fb_slot;      // row of the fallback logits buffer
    float theta0, Z0; // k-th largest logit and log-sum-exp after round 0
    int pad[2];
};

struct csv_workspace {
    int B_max, K_cap, V, d, C, Npad;   // Npad: C rounded up to a power of two (sort width)
    int n_chunks;                      // fallback top-k chunks per sequence
    int device;
    float* U;          // [B*C]      cluster bounds
    float* hnorm;      // [B]
    int32_t* order;    // [B*C]      cluster ids by descending bound
    float* su;         // [B*C]      bounds in that order
    float* T;          // [B*(C+1)]  log tail mass with the first m clusters open
    int32_t* P;        // [B*(C+1)]  rows in the first m clusters
    SeqState* st;      // [B]
    int32_t* rstart;   // [B]        first position of slog/rowmap to score this round
    int32_t* rcount;   // [B]        positions to score this round (0: nothing to do)
    float* slog;       // [B*K_cap]  logits of opened rows, in opening order
    int32_t* rowmap;   // [B*K_cap]  permuted row index of each opened position
    int32_t* counters; // [16]       [0] = number of fallback sequences this step
    int32_t* fb_list;  // [B]        sequences that fall back this step
    int32_t* all_list; // [B]        0..B-1 (csv_full_logits runs the fallback product over everyone)
    float* fb_logits;  // [B*V]      full logits of fallback sequences (permuted row order)
    float* cand_val;   // [B*n_chunks*CSV_MAX_K] per-chunk top-k candidates
    int32_t* cand_id;  //            their token ids
    float* cand_max;   // [B*n_chunks] per-chunk max logit
    float* cand_sum;   // [B*n_chunks] per-chunk sum exp(l - max)
    // optional per-stage timing (csv_profile_begin / csv_profile_end)
    hipEvent_t* prof_ev;   // (CSV_PROFILE_STAGES + 1) events per recorded step
    int prof_cap;          // steps the event pool holds
    int prof_n;            // steps recorded so far
    int prof_on;
};

// ---------------------------------------------------------------------------------------------- errors
void csv_set_error(const char* fmt, ...);

#define CSV_HIP(call)                                                                       \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess) {                                                             \
            csv_set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
            return CSV_EHIP;                                                                \
        }                                                                                   \
    } while (0)

#define CSV_LAUNCH_CHECK(name)                                                              \
    do {                                                                                    \
        hipError_t e_ = hipGetLastError();                                                  \
        if (e_ != hipSuccess) {                                                             \
            csv_set_error("launch of %s failed: %s", name, hipGetErrorString(e_));          \
            return CSV_EHIP;                                                                \
        }                                                                                   \
    } while (0)

// ---------------------------------------------------------------------------------------------- device primitives
#define CSV_WAVE 64

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// sum_j w_j * h_j over eight bf16 pairs packed in two 128-bit words, added to acc
__device__ __forceinline__ float dot8_bf16(const uint4& w, const uint4& h, float acc) {
    acc = fmaf(bf16_lo(w.x), bf16_lo(h.x), acc);
    acc = fmaf(bf16_hi(w.x), bf16_hi(h.x), acc);
    acc = fmaf(bf16_lo(w.y), bf16_lo(h.y), acc);
    acc = fmaf(bf16_hi(w.y), bf16_hi(h.y), acc);
    acc = fmaf(bf16_lo(w.z), bf16_lo(h.z), acc);
    acc = fmaf(bf16_hi(w.z), bf16_hi(h.z), acc);
    acc = fmaf(bf16_lo(w.w), bf16_lo(h.w), acc);
    acc = fmaf(bf16_hi(w.w), bf16_hi(h.w), acc);
    return acc;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, CSV_WAVE);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, CSV_WAVE));
    return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, CSV_WAVE);
    return v;
}
__device__ __forceinline__ int wave_min_i(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, CSV_WAVE));
    return v;
}

// Block-wide reductions in a fixed order (deterministic).  red: >= 16 words of LDS.  All threads get the result.
__device__ __forceinline__ float block_sum(float v, float* red) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_sum(v);
    __syncthreads();
    if (lane == 0) red[w] = v;
    __syncthreads();
    float r = 0.f;
    for (int i = 0; i < nw; ++i) r += red[i];
    return r;
}
__device__ __forceinline__ float block_max(float v, float* red) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_max(v);
    __syncthreads();
    if (lane == 0) red[w] = v;
    __syncthreads();
    float r = red[0];
    for (int i = 1; i < nw; ++i) r = fmaxf(r, red[i]);
    return r;
}
__device__ __forceinline__ int block_sum_i(int v, int* red) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_sum_i(v);
    __syncthreads();
    if (lane == 0) red[w] = v;
    __syncthreads();
    int r = 0;
    for (int i = 0; i < nw; ++i) r += red[i];
    return r;
}
__device__ __forceinline__ int block_min_i(int v, int* red) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_min_i(v);
    __syncthreads();
    if (lane == 0) red[w] = v;
    __syncthreads();
    int r = red[0];
    for (int i = 1; i < nw; ++i) r = min(r, red[i]);
    return r;
}

// Monotone map float -> uint32: a > b  <=>  fkey(a) > fkey(b)  (for non-NaN values; -0 < +0)
__device__ __forceinline__ uint32_t fkey(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float fkey_inv(uint32_t k) {
    uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __uint_as_float(u);
}

// a (+) b for log-sum-exp partials (m = running max, s = sum of exp(x - m)); (-inf, 0) is the identity
struct LseAcc {
    float m, s;
};
__device__ __forceinline__ LseAcc lse_combine(LseAcc a, LseAcc b) {
    if (a.s == 0.f) return b;
    if (b.s == 0.f) return a;
    LseAcc r;
    r.m = fmaxf(a.m, b.m);
    r.s = a.s * expf(a.m - r.m) + b.s * expf(b.m - r.m);
    return r;
}
__device__ __forceinline__ float lse_value(LseAcc a) { return a.s == 0.f ? -INFINITY : a.m + logf(a.s); }

// ---------------------------------------------------------------------------------------------- internal entry points
int csv_index_alloc(int V, int d, int C, csv_index** out);
