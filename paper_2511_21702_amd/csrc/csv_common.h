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
    uint16_t* mu16;  // [C*d] the same centroids as bf16 when they are stored rounded (NULL otherwise); mu then holds
                     //       the rounded values too
    float* R;        // [C]   stored radii
    float* bmax;     // [C]   per-cluster bias maximum (-inf for an empty cluster)
    int32_t* n;      // [C]   rows per cluster
    int32_t* off;    // [C+1] first permuted row of each cluster
    float* lnn;      // [C]   ln n_c (-inf for an empty cluster)
    int4* cmeta;     // [C]   {first permuted row, rows, bit pattern of ln n_c, 0}: what the seed selection needs of a
                     //       cluster in one 128-bit load
    float4* ang;     // [C] angular index (spherical clustering): {cos, sin of the angular radius, largest, smallest row norm},
                     //     all with slack; mu then holds unit directions and R is unused.  NULL = Euclidean index
    float2* bt;      // [C*bt_m] top-m bias table: pairs (radius, bias) per cluster, unused entries (0, -inf); NULL = none
    int bt_m;        // entries per cluster (0 = no table)
    float ln_nmax;   // ln of the largest cluster size
    int n_max;       // the largest cluster size
};

enum { ST_ACTIVE = 0, ST_DONE = 1, ST_FALLBACK = 2, ST_INVALID = 3 };
// counters[]: [CNT_FALLBACK] sequences that fall back this step; [CNT_ABORT] set when a bounded wait ran out;
// [CNT_TAIL_NEEDED] set by whoever queues work for after round 0 (tiles of a later round or of an oversize seed
// prefix, a fallback): what follows round 0 looks at this one word first;
// [CNT_BARRIER + i] arrivals at the i-th grid barrier of the tail kernel (2r, 2r+1: after the GEMV and after the
// certification of round r; 2*CSV_MAX_ROUNDS + j: the fallback phases); [CNT_TILES + r*CSV_MAX_BATCH + b] row tiles
// of sequence b in round r's work list; [CNT_CHUNKS + r*CSV_MAX_BATCH + b] chunk blocks of round r's certification
// that have published their partial results; [CNT_ARRIVE + b] blocks of the round-0 kernel that have finished their
// share of sequence b's seed rows; [CNT_R0_DONE] sequences whose round 0 is settled (certified, planned, handed over
// or invalid): what the blocks that run the tail inside the round-0 launch wait for.
// All are zeroed by the bound kernel at the start of a step.
enum { CNT_FALLBACK = 0, CNT_ABORT = 1, CNT_TAIL_NEEDED = 2, CNT_R0_DONE = 3, CNT_BARRIER = 16, CNT_TILES = 64, CNT_CHUNKS = 64 + CSV_MAX_ROUNDS * CSV_MAX_BATCH,
       CNT_ARRIVE = 64 + 2 * CSV_MAX_ROUNDS * CSV_MAX_BATCH, CNT_TOTAL = 64 + (2 * CSV_MAX_ROUNDS + 1) * CSV_MAX_BATCH,
       // not reset: bit i = whether the step i steps back needed anything after round 0 (kept behind the reset range)
       CNT_HISTORY = CNT_TOTAL,
       // not reset either: set when a step gave up while logits were still on their way through the round-0 slots
       // (the next step's bound kernel then refills the slots with the "empty" pattern before anything reads them)
       CNT_SLOTS_DIRTY = CNT_TOTAL + 1, CNT_ALLOC = CNT_TOTAL + 16 };

// A cluster's position in the bound order is carried by one 64-bit key: monotone image of U_c in the high word,
// ~c in the low word.  Larger key = larger bound, equal bounds = smaller cluster id first.  Empty clusters have key 0.
// The open set of a sequence is always {c : key_c >= kappa}.
struct SeqState {
    int status;
    int n_open;               // clusters open
    int n_rows;               // rows scored or planned so far (= positions used in slog / sid)
    int rounds;               // scoring rounds completed
    unsigned long long kappa; // threshold key of the open set
    float nxtU;               // largest bound among unopened clusters (-inf if none)
    float T;                  // log tail mass  log sum_{unopened} n_c exp(U_c)
    int fb_slot;              // row of the fallback logits buffer
    float theta;              // k-th largest logit scored so far (-inf: unknown): a later round's top-k starts from it
    int pad[2];
};

// Work item of the gathered GEMV: nrows (<= 8) consecutive rows of W' from row0, results to positions pos.. of sequence b.
struct Tile {
    int b, row0, nrows, pos;
};

#define CSV_SLOT_ROWS 4096    // seed rows a sequence can pass through the round-0 slots (= rows one block certifies from LDS)
#define CSV_SLOT_EMPTY 0xFFFFFFFFFFFFFFFFull

struct csv_workspace {
    int B_max, K_cap, V, d, C, Npad;   // Npad: C rounded up to a power of two (sort width)
    int n_chunks;                      // fallback top-k chunks per sequence
    int sp_chunks, cand_chunks;        // certification chunks per sequence; chunk stride of the candidate buffers
    int tile_stride;                   // entries of each sequence's region of a tile list
    int tail_grid;                     // blocks of the tail kernel (all resident together)
    int spin_limit;                    // polls a grid barrier waits before the step is given up
    int round0_capacity;               // blocks of the round-0 kernel that are resident together
    int split_min_B;                   // > 0: batches of at least this many sequences run the tail as one launch per
                                       // phase; 0: decided per step from the recent steps' history
    int* h_history;                    // pinned host word the bound kernel copies the history to (read without a sync)
    int* d_history;                    // the same word as the device sees it
    size_t tail_lds;                   // its dynamic LDS
    size_t fused_lds;                  // dynamic LDS of the launch that holds round 0 and the tail together
    int fused_ok;                      // that launch fits one block per compute unit
    int device;
    float* U;          // [B*C]      cluster bounds
    float* bound_partial; // K-slice partial sums of the batched (MFMA) bound product
    float* hnorm;      // [B]
    SeqState* st;      // [B]
    int32_t* sel;      // [B*C]      opened cluster ids
    float* slog;       // [B*K_cap]  logits of opened rows
    unsigned long long* slots; // [B*CSV_SLOT_ROWS] round 0: one (token id, logit) word per seed row, "empty" = all ones
    int32_t* sid;      // [B*K_cap]  their original token ids
    Tile* tiles[2];    // work lists of round 0 / round 1
    int32_t* counters; // [CNT_TOTAL]
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

// sum_j w_j * h_j over eight bf16 pairs packed in two 128-bit words, added to acc.  v_dot2c_f32_bf16 takes two
// bf16 pairs as they sit in memory and adds both products to a float32 accumulator: one instruction where
// widening both operands and two FMAs would be six (these loops are bound by instruction issue, not by arithmetic).
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 csv_bf16x2_t;
__device__ __forceinline__ float dot2_bf16(uint32_t w, uint32_t h, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(csv_bf16x2_t, w), __builtin_bit_cast(csv_bf16x2_t, h), acc, false);
}
__device__ __forceinline__ float dot8_bf16(const uint4& w, const uint4& h, float acc) {
    acc = dot2_bf16(w.x, h.x, acc);
    acc = dot2_bf16(w.y, h.y, acc);
    acc = dot2_bf16(w.z, h.z, acc);
    acc = dot2_bf16(w.w, h.w, acc);
    return acc;
}

// Wave-wide reductions with DPP lane exchanges (no LDS traffic): pairs, quads, half rows and rows of 16 lanes by
// quad_perm / row_half_mirror / row_mirror, then row_bcast15 and row_bcast31 carry the row totals to lane 63, whose
// value is broadcast.  Must be called with all 64 lanes active.  The combination order is fixed, so results are
// reproducible run to run.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ int dpp_move(int old, int src) {
    return __builtin_amdgcn_update_dpp(old, src, CTRL, ROW_MASK, 0xf, false);
}
#define CSV_DPP_REDUCE(T, TOI, FROMI, OP, IDENT)                                              \
    {                                                                                         \
        v = OP(v, FROMI(dpp_move<0xB1, 0xf>(TOI(v), TOI(v))));  /* quad_perm [1,0,3,2] */     \
        v = OP(v, FROMI(dpp_move<0x4E, 0xf>(TOI(v), TOI(v))));  /* quad_perm [2,3,0,1] */     \
        v = OP(v, FROMI(dpp_move<0x141, 0xf>(TOI(v), TOI(v)))); /* row_half_mirror */         \
        v = OP(v, FROMI(dpp_move<0x140, 0xf>(TOI(v), TOI(v)))); /* row_mirror */              \
        v = OP(v, FROMI(dpp_move<0x142, 0xa>(TOI((T)(IDENT)), TOI(v)))); /* row_bcast15 */    \
        v = OP(v, FROMI(dpp_move<0x143, 0xc>(TOI((T)(IDENT)), TOI(v)))); /* row_bcast31 */    \
        return FROMI(__builtin_amdgcn_readlane(TOI(v), 63));                                  \
    }
__device__ __forceinline__ float csv_addf(float a, float b) { return a + b; }
__device__ __forceinline__ int csv_addi(int a, int b) { return a + b; }
__device__ __forceinline__ int csv_mini(int a, int b) { return a < b ? a : b; }
__device__ __forceinline__ unsigned csv_maxu(unsigned a, unsigned b) { return a > b ? a : b; }
__device__ __forceinline__ int csv_id_i(int x) { return x; }
__device__ __forceinline__ int csv_u2i(unsigned x) { return (int)x; }
__device__ __forceinline__ unsigned csv_i2u(int x) { return (unsigned)x; }

__device__ __forceinline__ float wave_sum(float v) CSV_DPP_REDUCE(float, __float_as_int, __int_as_float, csv_addf, 0.f)
__device__ __forceinline__ float wave_max(float v) CSV_DPP_REDUCE(float, __float_as_int, __int_as_float, fmaxf, -INFINITY)
__device__ __forceinline__ int wave_sum_i(int v) CSV_DPP_REDUCE(int, csv_id_i, csv_id_i, csv_addi, 0)
__device__ __forceinline__ int wave_min_i(int v) CSV_DPP_REDUCE(int, csv_id_i, csv_id_i, csv_mini, 0x7fffffff)
__device__ __forceinline__ unsigned wave_max_u(unsigned v) CSV_DPP_REDUCE(unsigned, csv_u2i, csv_i2u, csv_maxu, 0u)

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

__device__ __forceinline__ unsigned long long wave_max_u64(unsigned long long v) {
    const unsigned hi = (unsigned)(v >> 32), lo = (unsigned)v;
    const unsigned mhi = wave_max_u(hi);
    const unsigned mlo = wave_max_u(hi == mhi ? lo : 0u);
    return ((unsigned long long)mhi << 32) | mlo;
}
// red: >= 16 64-bit words of LDS
__device__ __forceinline__ unsigned long long block_max_u64(unsigned long long v, unsigned long long* red) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_max_u64(v);
    __syncthreads();
    if (lane == 0) red[w] = v;
    __syncthreads();
    unsigned long long r = red[0];
    for (int i = 1; i < nw; ++i) r = red[i] > r ? red[i] : r;
    return r;
}

// The two largest of a set of distinct 64-bit keys (0 = none), reduced in one pass: the seed selection needs the
// best unopened cluster and the one after it, and one reduction of pairs is cheaper than two reductions in a row.
struct Top2 {
    unsigned long long a, b;   // a > b, or 0 when absent
};
__device__ __forceinline__ Top2 top2_merge(Top2 x, Top2 y) {
    const bool xg = x.a > y.a;
    Top2 r;
    r.a = xg ? x.a : y.a;
    const unsigned long long loser = xg ? y.a : x.a, second = xg ? x.b : y.b;   // the winner's own runner-up
    r.b = loser > second ? loser : second;
    return r;
}
__device__ __forceinline__ Top2 top2_push(Top2 t, unsigned long long k) {
    if (k > t.a) {
        t.b = t.a;
        t.a = k;
    } else if (k > t.b) {
        t.b = k;
    }
    return t;
}
template <int CTRL, int ROW_MASK, bool KEEP>
__device__ __forceinline__ Top2 top2_dpp_step(Top2 v) {
    // KEEP: lanes the move does not reach combine with their own value; otherwise with the identity (0, 0)
    const int a_lo = (int)(unsigned)v.a, a_hi = (int)(unsigned)(v.a >> 32), b_lo = (int)(unsigned)v.b, b_hi = (int)(unsigned)(v.b >> 32);
    Top2 y;
    y.a = ((unsigned long long)(unsigned)dpp_move<CTRL, ROW_MASK>(KEEP ? a_hi : 0, a_hi) << 32) | (unsigned)dpp_move<CTRL, ROW_MASK>(KEEP ? a_lo : 0, a_lo);
    y.b = ((unsigned long long)(unsigned)dpp_move<CTRL, ROW_MASK>(KEEP ? b_hi : 0, b_hi) << 32) | (unsigned)dpp_move<CTRL, ROW_MASK>(KEEP ? b_lo : 0, b_lo);
    return y;
}
__device__ __forceinline__ Top2 wave_top2(Top2 v) {
    // a lane never meets its own value in the first four steps (the moves are permutations); keys are distinct, so
    // merging a pair with a pair that shares an element cannot happen before the broadcast steps, where the partner is
    // another row's total
    v = top2_merge(v, top2_dpp_step<0xB1, 0xf, true>(v));    // quad_perm [1,0,3,2]
    v = top2_merge(v, top2_dpp_step<0x4E, 0xf, true>(v));    // quad_perm [2,3,0,1]
    v = top2_merge(v, top2_dpp_step<0x141, 0xf, true>(v));   // row_half_mirror
    v = top2_merge(v, top2_dpp_step<0x140, 0xf, true>(v));   // row_mirror
    v = top2_merge(v, top2_dpp_step<0x142, 0xa, false>(v));  // row_bcast15 into rows 1 and 3
    v = top2_merge(v, top2_dpp_step<0x143, 0xc, false>(v));  // row_bcast31 into rows 2 and 3
    Top2 r;
    r.a = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v.a >> 32), 63) << 32) | (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v.a, 63);
    r.b = ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v.b >> 32), 63) << 32) | (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v.b, 63);
    return r;
}
// red: >= 32 64-bit words of LDS
__device__ __forceinline__ Top2 block_top2(Top2 v, unsigned long long* red) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_top2(v);
    __syncthreads();
    if (lane == 0) {
        red[2 * w] = v.a;
        red[2 * w + 1] = v.b;
    }
    __syncthreads();
    Top2 r;
    r.a = red[0];
    r.b = red[1];
    for (int i = 1; i < nw; ++i) r = top2_merge(r, Top2{red[2 * i], red[2 * i + 1]});
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
// fold one more value into a running partial
__device__ __forceinline__ LseAcc lse_push(LseAcc a, float x) {
    if (x == -INFINITY) return a;
    if (a.s == 0.f) {
        a.m = x;
        a.s = 1.f;
    } else if (x > a.m) {
        a.s = a.s * expf(a.m - x) + 1.f;
        a.m = x;
    } else {
        a.s += expf(x - a.m);
    }
    return a;
}
__device__ __forceinline__ float lse_value(LseAcc a) { return a.s == 0.f ? -INFINITY : a.m + logf(a.s); }

// ---------------------------------------------------------------------------------------------- internal entry points
int csv_index_alloc(int V, int d, int C, csv_index** out);
int csv_index_pack_cmeta(csv_index* x, hipStream_t st);   // fills cmeta from off and lnn (both final)
