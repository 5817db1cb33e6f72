// Per-step kernels of the certified sub-vocabulary LM-head path and the entry points that enqueue them.
//
//   bound1_kernel / bound_kernel / bound_mfma_kernel + bound_finish_kernel
//                      U[b,c] = <mu_c,h_b> + R_c ||h_b|| + bmax_c  for 1, 2..4 and more sequences   (Eq. "cluster_bound")
//   round0_kernel      per sequence: shortest prefix of the bound order holding >= max(k,1) rows, next bound, log tail
//                      mass (Algorithm 1: queue, PopMax); logits of the prefix rows of W' (Algorithm 1: sparse GEMV);
//                      top-k, log-sum-exp and both certificates, or the plan of the next round
//                                                                                      (Definitions 1-2, Theorems 1-2)
//   tail_kernel        only when some sequence needs it: further rounds (tile GEMV + certification), then all V logits,
//                      top-k and log-sum-exp for the sequences that fall back                          (Eq. "logit")
//   full_gemv_kernel / full_mfma_kernel   all V logits as an entry point of their own
//
// Everything is enqueued on the caller's stream; decisions (round 1, fallback) are taken on the device.
// The open set of a sequence is {c : key_c >= kappa} for a 64-bit key that encodes (bound, cluster id), so the
// common path needs reductions only; the bound order is sorted only when the softmax test asks for a longer prefix.
#include "csv_common.h"

#include <math.h>
#include <type_traits>
#include <stdarg.h>
#include <stdlib.h>
#include <string.h>
#include <pthread.h>

// ------------------------------------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";
void csv_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}
extern "C" const char* csv_last_error(void) { return g_err; }

typedef unsigned long long u64;

// ------------------------------------------------------------------------------------------------ arguments
struct StepArgs {
    int V, d, C;
    const uint16_t* Wp;
    const float* bp;
    const int32_t* perm;
    const float* mu;
    const uint16_t* mu16;   // bf16 copy of the centroids, or NULL
    const float* R;
    const float* bmax;
    const int32_t* n;
    const int32_t* off;
    const float* lnn;
    const int4* cmeta;      // per cluster {first row, rows, bits of ln n, 0}
    const float2* bt;       // top-m bias table, [C * bt_m] pairs (radius, bias), or NULL
    const float4* ang;      // angular index: {cos, sin of the angular radius, largest, smallest row norm} per cluster, or NULL
    int bt_m;
    float ln_nmax;
    int B, B_max, K_cap, Npad, n_chunks, tile_stride;
    int sp_chunks;     // most STAGE_CAP-sized chunks a sequence's scored rows can span
    int cand_chunks;   // chunk stride of the candidate buffers
    int tail_lds;      // dynamic LDS bytes of the tail kernel
    int spin_limit;    // polls a grid barrier of the tail kernel waits before it gives the step up
    int* host_history; // pinned host word for the history of steps that needed the tail (device-visible address)
    int r0_h_off;      // offset of h in the round-0 kernel's LDS arena, in 128-bit units (behind the cluster data)
    float* U;
    float* hnorm;
    float* bound_partial;   // [BOUND_KS_MAX * B * C] K-slice partial sums of the batched bound product
    SeqState* st;
    int32_t* sel;
    float* slog;
    int32_t* sid;
    u64* slots;        // [B*CSV_SLOT_ROWS] round-0 hand-over words
    Tile* tiles[2];
    int32_t* counters;
    int32_t* fb_list;
    float* fb_logits;
    float* cand_val;
    int32_t* cand_id;
    float* cand_max;
    float* cand_sum;
    const uint16_t* h;
    int k, K_max, combine, use_k, use_s;
    int max_rounds, delta_clusters, relax;   // fallback levels
    float lam;   // ln(eps/(1-eps)); +inf when eps >= 1
    float lam2;  // the same for the relaxed tolerance 2 eps
    float top_p; // nucleus mass asked for (0 = none)
    csv_step_out out;
};

#define TILE_ROWS 8        // rows per work item of the gathered GEMV (4 waves x 2 rows)
#define SEQ_THREADS 512    // block size of the per-sequence kernels (seed, cert, fallback top-k)
#define STAGE_CAP 4096     // scored logits kept in LDS by cert_kernel when a sequence has at most this many
static_assert(STAGE_CAP == CSV_SLOT_ROWS, "the round-0 slots hold exactly what one block certifies from LDS");
#define FB_CHUNK 8192      // rows per block of the fallback top-k first stage
#define FULL_G 4           // sequences per pass of the vector full-vocabulary product
#define BIGQ 32            // clusters whose tiles are written cooperatively per emit call

#define CSV_STATIC_MAX_DEVICES 64   // devices the per-device host tables of this file cover

// Key of a value for ordering: -0 and +0 compare equal.
__device__ __forceinline__ uint32_t lkey(float v) { return fkey(v + 0.0f); }
__device__ __forceinline__ u64 ckey(float U, int c) { return ((u64)lkey(U) << 32) | (u64)(0xFFFFFFFFu - (uint32_t)c); }
__device__ __forceinline__ float ckey_bound(u64 k) { return fkey_inv((uint32_t)(k >> 32)); }

// Zero the step's counters: the fixed slots and, of every per-sequence row, the entries of the B sequences in use.
// Before that, whether the previous step needed anything after round 0 is shifted into the history word (device
// copy behind the reset range, and a pinned host copy that the next calls read without synchronising).
__device__ __forceinline__ void reset_step_counters(int* counters, int B, int nthreads, int* host_history, u64* slots, int B_max) {
    constexpr int rows = (CNT_TOTAL - CNT_TILES) / CSV_MAX_BATCH;
    if (counters[CNT_SLOTS_DIRTY] != 0) {     // an earlier step gave up with logits still on their way: empty every slot
        for (size_t i = threadIdx.x; i < (size_t)B_max * CSV_SLOT_ROWS; i += nthreads) slots[i] = CSV_SLOT_EMPTY;
        __syncthreads();
        if (threadIdx.x == 0) counters[CNT_SLOTS_DIRTY] = 0;
    }
    if (threadIdx.x == 0) {      // low half: steps that needed the tail; high half: steps with a fallback
        const unsigned old = (unsigned)counters[CNT_HISTORY];
        const unsigned lo = ((old << 1) | (unsigned)(counters[CNT_TAIL_NEEDED] != 0)) & 0xffffu;
        const unsigned hi = (((old >> 16) << 1) | (unsigned)(counters[CNT_FALLBACK] != 0)) & 0x7fffu;
        const int h = (int)(lo | (hi << 16));
        counters[CNT_HISTORY] = h;
        if (host_history) *host_history = h;
    }
    __syncthreads();             // called by every thread of one block: the zeroing below must not overtake the reads
    for (int i = threadIdx.x; i < CNT_TILES + rows * B; i += nthreads) {
        const int j = i - CNT_TILES;
        counters[i < CNT_TILES ? i : CNT_TILES + (j / B) * CSV_MAX_BATCH + (j % B)] = 0;
    }
}

// ================================================================================================ bounds
// What a cluster adds to <mu_c,h>: R_c ||h|| + max bias (Eq. "cluster_bound"), or, with a top-m bias table, the
// largest of its m terms rho_j ||h|| + beta_j (the m-1 tokens with the largest biases one by one, the rest together).
// With an angular index (spherical clustering) mu_c is a unit direction and the bound is
//   rho ||h|| cos(phi - theta_c) = rho (t cos(theta_c) + sqrt(||h||^2 - t^2) sin(theta_c)),  t = <mu_c,h> = ||h|| cos(phi),
// outside the cluster's cone and rho_max ||h|| inside it; rho is the largest row norm for a positive value, the smallest
// for a negative one.
__device__ __forceinline__ float bound_value(const StepArgs& a, int c, float dot, float Rc, float bm, float hn) {
    if (a.ang) {
        const float4 g = a.ang[c];
        const float perp = sqrtf(fmaxf(hn * hn - dot * dot, 0.f));
        const float v = dot * g.x + perp * g.y;
        const float val = dot >= hn * g.x ? g.z * hn : (v >= 0.f ? g.z * v : g.w * v);
        return val + bm;
    }
    if (!a.bt) return dot + Rc * hn + bm;
    const float2* t = a.bt + (size_t)c * a.bt_m;
    float best = -INFINITY;
    for (int j = 0; j < a.bt_m; ++j) {
        const float2 e = t[j];
        best = fmaxf(best, fmaf(e.x, hn, e.y));
    }
    return dot + best;
}

// Block = 8 waves = 8/WPC clusters x WPC column slices (WPC = 1, 2 or 4, chosen so that a wave's slice of the
// centroid row is at most 8 KB = one batch of eight 128-bit loads per lane), BT sequences per block.
// Order of requests matters: a wave's loads return in order, so h (needed first, to fill LDS and for ||h||) is
// requested before the centroid slice, and the slice is in flight while h is staged and the norms are taken.
// Blocks are dealt round-robin to the 8 XCDs, so group g = (block % 8) * groups_per_xcd + block / 8 keeps
// every XCD on the same centroid slice step after step.
#define BOUND_PF 8
// A "unit" is one 128-bit load of a centroid row: four float32 values, or eight bfloat16 values when the index
// stores its centroids rounded (MU16).  The matching piece of h is 8 resp. 16 bytes of bf16.
template <bool MU16>
__device__ __forceinline__ const uint4* mu_row(const StepArgs& a, int c) {
    return MU16 ? reinterpret_cast<const uint4*>(a.mu16 + (size_t)c * a.d) : reinterpret_cast<const uint4*>(a.mu + (size_t)c * a.d);
}
template <bool MU16>
__device__ __forceinline__ int mu_units(int d) { return MU16 ? d >> 3 : d >> 2; }
// acc += <unit of mu, matching piece of h>;  hrow: the sequence's h as 32-bit words (two bf16 each)
template <bool MU16, class HP>
__device__ __forceinline__ float mu_fma(const uint4& m, HP hrow, int unit, float acc) {
    if constexpr (MU16) {
        const uint4 hv = reinterpret_cast<const uint4*>(hrow)[unit];
        return dot8_bf16(m, hv, acc);
    } else {
        const uint2 hv = reinterpret_cast<const uint2*>(hrow)[unit];
        acc = fmaf(__uint_as_float(m.x), bf16_lo(hv.x), acc);
        acc = fmaf(__uint_as_float(m.y), bf16_hi(hv.x), acc);
        acc = fmaf(__uint_as_float(m.z), bf16_lo(hv.y), acc);
        acc = fmaf(__uint_as_float(m.w), bf16_hi(hv.y), acc);
        return acc;
    }
}
#define BOUND_THREADS 512
#define BOUND_LDS_MAX (128 * 1024)   // h of up to 8 sequences of d = 8192 in LDS: one block serves all 8, the centroids are read once
#define BOUND_HREG 8       // 128-bit pieces of h per thread: 8 x 512 x 16 B covers the 64 KB that BT sequences may take in LDS
// 2..4 sequences: h of the block's BT sequences is staged in LDS once, then every wave walks over whole clusters
// (cluster = wave index among all waves of the grid, then + their number, ...): a centroid row goes through the wave
// in chunks of BOUND_PFB 128-bit loads per lane, the next chunk (of this or of the wave's next cluster) always
// requested before the current one is used, and nothing in the loop waits for another wave.  With more clusters
// than resident waves the staging of h is paid once per block, not once per cluster.
#ifndef BOUND_PFB
#define BOUND_PFB 16      // 128-bit loads per lane and chunk of a centroid row (two chunks in flight)
#endif
template <int BT, bool MU16>
__global__ __launch_bounds__(BOUND_THREADS) void bound_kernel(StepArgs a, float* __restrict__ U_out, float* __restrict__ hn_out,
                                                              int reset_counters) {
    extern __shared__ uint4 hs4[];
    __shared__ float hn[BT];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int b0 = blockIdx.y * BT;
    const int nb = min(BT, a.B - b0);
    const int nch = a.d >> 3, nq = mu_units<MU16>(a.d), C = a.C;
    const int GW = gridDim.x * (BOUND_THREADS / 64);
    const int nchk = (nq + 64 * BOUND_PFB - 1) / (64 * BOUND_PFB);
    int c = blockIdx.x * (BOUND_THREADS / 64) + wave, chunk = 0;
    uint4 pfA[BOUND_PFB], pfB[BOUND_PFB];
    auto issue = [&](uint4 (&buf)[BOUND_PFB], int cc, int ch) {      // unconditional loads from clamped addresses, then a select
        const uint4* mrow = mu_row<MU16>(a, min(cc, C - 1));
#pragma unroll
        for (int j = 0; j < BOUND_PFB; ++j) {
            const int i = ch * 64 * BOUND_PFB + lane + 64 * j;
            const uint4 v = mrow[min(i, nq - 1)];
            buf[j] = (cc < C && i < nq) ? v : make_uint4(0, 0, 0, 0);
        }
    };
    issue(pfA, c, 0);                 // in flight while h is staged
    const uint4* hsrc = reinterpret_cast<const uint4*>(a.h) + (size_t)b0 * nch;
    for (int base = 0; base < BT * nch; base += BOUND_HREG * BOUND_THREADS) {
        uint4 hreg[BOUND_HREG];
#pragma unroll
        for (int q = 0; q < BOUND_HREG; ++q) {
            const int i = base + tid + q * BOUND_THREADS;
            const uint4 v = hsrc[min(i, nb * nch - 1)];
            hreg[q] = i < nb * nch ? v : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < BOUND_HREG; ++q) {
            const int i = base + tid + q * BOUND_THREADS;
            if (i < BT * nch) hs4[i] = hreg[q];
        }
    }
    if (reset_counters && blockIdx.x == 0 && blockIdx.y == 0)
        reset_step_counters(a.counters, a.B, BOUND_THREADS, a.host_history, a.slots, a.B_max);
    __syncthreads();
    for (int s = wave; s < BT; s += BOUND_THREADS / 64) {
        float acc = 0.f;
        for (int i = lane; i < nch; i += 64) {
            uint4 v = hs4[s * nch + i];
            acc = dot8_bf16(v, v, acc);
        }
        acc = wave_sum(acc);
        if (lane == 0) hn[s] = sqrtf(acc);
    }
    __syncthreads();
    if (blockIdx.x == 0 && tid < nb && hn_out) hn_out[b0 + tid] = hn[tid];

    float acc[BT];
#pragma unroll
    for (int s = 0; s < BT; ++s) acc[s] = 0.f;
    // one trip: request the chunk after (c, chunk) into `nxt`, use `cur`, finish the cluster when that was its last chunk
    auto trip = [&](uint4 (&cur)[BOUND_PFB], uint4 (&nxt)[BOUND_PFB]) {
        const bool last = chunk + 1 == nchk;
        const int c2 = last ? c + GW : c, ch2 = last ? 0 : chunk + 1;
        float Rc = 0.f, bm = 0.f;
        int ncl = 0;
        if (last) {                    // every lane the same address; needed only after the reduction below
            Rc = a.R[c];
            bm = a.bmax[c];
            ncl = a.n[c];
        }
        if (c2 < C) issue(nxt, c2, ch2);
#pragma unroll
        for (int j = 0; j < BOUND_PFB; ++j) {
            const int i = min(chunk * 64 * BOUND_PFB + lane + 64 * j, nq - 1);     // units past the row are zero
#pragma unroll
            for (int s = 0; s < BT; ++s) acc[s] = mu_fma<MU16>(cur[j], hs4 + s * nch, i, acc[s]);
        }
        if (last) {
#pragma unroll
            for (int s = 0; s < BT; ++s) {
                const float t = wave_sum(acc[s]);
                if (lane == 0 && s < nb) U_out[(size_t)(b0 + s) * C + c] = ncl == 0 ? -INFINITY : bound_value(a, c, t, Rc, bm, hn[s]);
                acc[s] = 0.f;
            }
        }
        c = c2;
        chunk = ch2;
    };
    while (c < C) {
        trip(pfA, pfB);
        if (c >= C) break;
        trip(pfB, pfA);
    }
}

// One sequence (B = 1): no LDS staging at all.  h is 2d bytes that every wave of the device reads, so it comes from
// L2 / L1 with the same addresses in every block; each wave takes its slice of h straight from global memory next to
// its centroid slice, and ||h||^2 is the sum of the slices' partial sums of squares (slice order: the same value
// in every block).
template <bool MU16>
__global__ __launch_bounds__(BOUND_THREADS) void bound1_kernel(StepArgs a, float* __restrict__ U_out, float* __restrict__ hn_out,
                                                               int reset_counters, int groups, int groups_per_xcd, int wpc) {
    __shared__ float part[BOUND_THREADS / 64], parth[BOUND_THREADS / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nq = mu_units<MU16>(a.d);
    const int cpb = (BOUND_THREADS / 64) / wpc, cl = wave / wpc, slice = wave - cl * wpc;
    const int g = (blockIdx.x & 7) * groups_per_xcd + (blockIdx.x >> 3);
    const int c = g * cpb + cl;
    const bool valid = g < groups && c < a.C;
    const int seg = (nq + wpc - 1) / wpc, lo = slice * seg, hi = min(nq, lo + seg);
    const uint4* mrow = mu_row<MU16>(a, valid ? c : 0);
    typedef typename std::conditional<MU16, uint4, uint2>::type hpiece;   // the piece of h that goes with one unit
    const hpiece* hp = reinterpret_cast<const hpiece*>(a.h);
    uint4 pf[BOUND_PF];
    hpiece ph[BOUND_PF];
#pragma unroll
    for (int j = 0; j < BOUND_PF; ++j) {
        const int i = lo + lane + 64 * j;
        pf[j] = (valid && i < hi) ? mrow[i] : make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < BOUND_PF; ++j) {
        const int i = lo + lane + 64 * j;
        ph[j] = i < hi ? hp[i] : hpiece{};
    }
    float Rc = 0.f, bm = 0.f;
    int ncl = 0;
    if (valid && slice == 0 && lane == 0) {
        Rc = a.R[c];
        bm = a.bmax[c];
        ncl = a.n[c];
    }
    if (reset_counters && blockIdx.x == 0)
        reset_step_counters(a.counters, a.B, BOUND_THREADS, a.host_history, a.slots, a.B_max);
    float acc = 0.f, hh = 0.f;
    auto step = [&](const uint4& m, const hpiece& hv) {
        acc = mu_fma<MU16>(m, &hv, 0, acc);
        const uint32_t* w = reinterpret_cast<const uint32_t*>(&hv);
#pragma unroll
        for (int e = 0; e < (int)(sizeof(hpiece) / 4); ++e) {
            hh = fmaf(bf16_lo(w[e]), bf16_lo(w[e]), hh);
            hh = fmaf(bf16_hi(w[e]), bf16_hi(w[e]), hh);
        }
    };
#pragma unroll
    for (int j = 0; j < BOUND_PF; ++j) step(pf[j], ph[j]);
#pragma unroll 4
    for (int i = lo + lane + 64 * BOUND_PF; i < hi; i += 64) {
        const uint4 m = valid ? mrow[i] : make_uint4(0, 0, 0, 0);
        step(m, hp[i]);
    }
    acc = wave_sum(acc);
    hh = wave_sum(hh);
    if (lane == 0) {
        part[wave] = acc;
        parth[wave] = hh;
    }
    __syncthreads();
    if (slice == 0 && lane == 0) {
        float t = part[wave], th = parth[wave];
        for (int q = 1; q < wpc; ++q) {
            t += part[wave + q];
            th += parth[wave + q];
        }
        const float hn = sqrtf(th);
        if (blockIdx.x == 0 && wave == 0 && hn_out) hn_out[0] = hn;
        if (valid) U_out[c] = ncl == 0 ? -INFINITY : bound_value(a, c, t, Rc, bm, hn);
    }
}

// Bounds for larger batches (B >= BOUND_MFMA_MIN_B): [C x d] fp32 centroids times [d x B] bf16 hidden states is a dense contraction,
// done with v_mfma_f32_16x16x32_bf16.  A float32 centroid value is split exactly into three bf16 pieces
// (x = hi + mid + lo, 8 mantissa bits each), so three MFMAs per k-block give the float32-exact products with float32
// accumulation; the split costs a handful of vector instructions per value, independent of B.
// A wave owns 16 clusters and one slice of K; lane (li, g) feeds cluster/sequence li with the eight k values
// 32 kb + 8 g.  Partial sums of the K slices go to P[slice][sequence][cluster]; bound_finish_kernel adds them in a
// fixed order together with R_c ||h|| + bmax_c, so the result does not depend on scheduling.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4_t;

__device__ __forceinline__ void split3_bf16(const float4& x0, const float4& x1, uint4& hi, uint4& mid, uint4& lo) {
    const float v[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
    uint32_t h[8], m[8], l[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        h[i] = __float_as_uint(v[i]) & 0xffff0000u;
        const float r1 = v[i] - __uint_as_float(h[i]);
        m[i] = __float_as_uint(r1) & 0xffff0000u;
        const float r2 = r1 - __uint_as_float(m[i]);
        l[i] = __float_as_uint(r2) & 0xffff0000u;
    }
    hi = make_uint4((h[0] >> 16) | h[1], (h[2] >> 16) | h[3], (h[4] >> 16) | h[5], (h[6] >> 16) | h[7]);
    mid = make_uint4((m[0] >> 16) | m[1], (m[2] >> 16) | m[3], (m[4] >> 16) | m[5], (m[6] >> 16) | m[7]);
    lo = make_uint4((l[0] >> 16) | l[1], (l[2] >> 16) | l[3], (l[4] >> 16) | l[5], (l[6] >> 16) | l[7]);
}

#define BOUND_TILES_PER_BLOCK 8   // waves of a block: each owns 16 clusters, all share the block's K slice (and its h in LDS)
#define BOUND_MFMA_MIN_B 5       // from this many sequences on the MFMA product is faster than the vector kernel, whose reads of h
                                 // from LDS (eight sequences: 128 bytes per lane for 16 bytes of a centroid) bound it: 15 vs 23 us at B = 8
#ifndef BOUND_BLOCK_TARGET
#define BOUND_BLOCK_TARGET 256   // (groups of cluster tiles x K slices) aimed at: one block per compute unit (64..2048 swept)
#endif
#define BOUND_KS_MAX 32
#ifndef BOUND_PIPE
#define BOUND_PIPE 4             // k-blocks (of 32) a wave has requested ahead: 8 KB of float32 centroids
#endif
#define BOUND_LDS_KB 48          // most LDS for the h of one K slice (1 KB per k-block and 16 sequences)
__device__ __forceinline__ uint4 keep_if(bool c, const uint4& v) {     // v or zero, component by component (no select between objects in memory)
    return make_uint4(c ? v.x : 0u, c ? v.y : 0u, c ? v.z : 0u, c ? v.w : 0u);
}
__device__ __forceinline__ void lds_barrier() {      // all LDS accesses of the block's waves are done; global loads stay in flight
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Grid (groups of 8 cluster tiles, K slices).  The block's slice of h goes to LDS once, in fragment order (1 KB per
// k-block and sequence tile, read without bank conflicts), zero where the sequence, the k-block or k itself lies
// outside: centroid values can then be read from clamped addresses without a select, which would be waited for right
// behind the load.  Every wave has BOUND_PIPE k-blocks of its 16 centroid rows requested ahead; a register buffer is
// requested again as soon as its values are split.  The last chunk is a copy of the loop body without requests, so
// that the waits the compiler places are counted at compile time.
template <int NT, bool MU16>
__global__ __launch_bounds__(512) void bound_mfma_kernel(StepArgs a, float* __restrict__ P, int seq0, int KS, int kb_per_slice,
                                                         int reset_counters) {
    extern __shared__ uint4 bound_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, g = lane >> 4;
    if (reset_counters && blockIdx.x == 0 && blockIdx.y == 0)
        reset_step_counters(a.counters, a.B, 512, a.host_history, a.slots, a.B_max);
    const int ks = blockIdx.y;
    const int nkb = (a.d + 31) >> 5;
    const int kb0 = ks * kb_per_slice, kb1 = min(nkb, kb0 + kb_per_slice);      // the host gives every slice at least one k-block
    const int nchunk = (kb1 - kb0 + BOUND_PIPE - 1) / BOUND_PIPE;
    const int c0 = (blockIdx.x * BOUND_TILES_PER_BLOCK + wave) * 16;            // past C: the wave computes a copy of the last rows and stores nothing
    const size_t crow = (size_t)min(c0 + li, a.C - 1) * a.d;
    const uint4* ap = MU16 ? reinterpret_cast<const uint4*>(a.mu16 + crow) : reinterpret_cast<const uint4*>(a.mu + crow);
    uint4 X[BOUND_PIPE][MU16 ? 1 : 2];
    auto load_x = [&](int u, int kb) {          // the lane's eight values of k-block kb, or (k past d) eight finite values that meet zeros
        const int k = min(kb * 32 + g * 8, a.d - 8);
        if constexpr (MU16) {
            X[u][0] = ap[k >> 3];
        } else {
            X[u][0] = ap[k >> 2];
            X[u][1] = ap[(k >> 2) + 1];
        }
    };
    // h first (older loads are waited for first), then the centroid requests, which stay in flight across the staging
    constexpr int HS = (BOUND_LDS_KB * 64 + 511) / 512;           // staged 128-bit pieces per thread at most
    const int items = nchunk * BOUND_PIPE * NT * 64;
    const uint4* hsrc = reinterpret_cast<const uint4*>(a.h);
    uint4 hreg[HS];
    bool hok[HS];
#pragma unroll
    for (int q = 0; q < HS; ++q) {
        const int it = tid + q * 512;
        const int ln = it & 63, t = (it >> 6) % NT, kbl = (it >> 6) / NT;
        const int sq = seq0 + t * 16 + (ln & 15), kb = kb0 + kbl, k = kb * 32 + (ln >> 4) * 8;
        hok[q] = it < items && sq < a.B && kb < kb1 && k < a.d;
        hreg[q] = make_uint4(0, 0, 0, 0);
        if (it < items) hreg[q] = hsrc[(size_t)(hok[q] ? sq : 0) * (a.d >> 3) + (hok[q] ? k >> 3 : 0)];
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < BOUND_PIPE; ++u) load_x(u, kb0 + u);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int q = 0; q < HS; ++q) {
        const int it = tid + q * 512;
        if (it < items) bound_lds[it] = keep_if(hok[q], hreg[q]);
    }
    lds_barrier();
    floatx4_t acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    auto chunk = [&](auto more_t, int c) {
        constexpr bool more = decltype(more_t)::value;
#pragma unroll
        for (int u = 0; u < BOUND_PIPE; ++u) {
            const uint4* hb = bound_lds + ((c * BOUND_PIPE + u) * NT << 6) + lane;
            if constexpr (MU16) {       // bf16 centroids feed the MFMA as they are
                const bf16x8_t xv = __builtin_bit_cast(bf16x8_t, X[u][0]);
                __builtin_amdgcn_sched_barrier(0);
                if (more) load_x(u, kb0 + (c + 1) * BOUND_PIPE + u);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, hb[t << 6]), xv, acc[t], 0, 0, 0);
            } else {
                uint4 hi, mid, lo;
                split3_bf16(__builtin_bit_cast(float4, X[u][0]), __builtin_bit_cast(float4, X[u][1]), hi, mid, lo);
                __builtin_amdgcn_sched_barrier(0);
                if (more) load_x(u, kb0 + (c + 1) * BOUND_PIPE + u);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const bf16x8_t bv = __builtin_bit_cast(bf16x8_t, hb[t << 6]);
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bv, __builtin_bit_cast(bf16x8_t, hi), acc[t], 0, 0, 0);
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bv, __builtin_bit_cast(bf16x8_t, mid), acc[t], 0, 0, 0);
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bv, __builtin_bit_cast(bf16x8_t, lo), acc[t], 0, 0, 0);
                }
            }
        }
    };
    for (int c = 0; c + 1 < nchunk; ++c) chunk(std::true_type{}, c);
    chunk(std::false_type{}, nchunk - 1);
    // h is the first operand: accumulator register r of lane (li, g) is  [sequence 4g + r][cluster li], so the 16
    // lanes of a group store 64 contiguous bytes of one sequence's partial bounds
    const int c = c0 + li;
    if (c < a.C) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int sq = seq0 + t * 16 + 4 * g + r;
                if (sq < a.B) P[((size_t)ks * a.B + sq) * a.C + c] = acc[t][r];
            }
    }
}

// Block (x, b): ||h_b|| (every block of the sequence recomputes it: d values), then for 256 clusters
// U[b,c] = sum of the K-slice partials (ascending slice) + R_c ||h_b|| + bmax_c.
__global__ __launch_bounds__(256) void bound_finish_kernel(StepArgs a, const float* __restrict__ P, int KS,
                                                           float* __restrict__ U_out, float* __restrict__ hn_out) {
    __shared__ float red[16];
    const int b = blockIdx.y, tid = threadIdx.x;
    const int c = blockIdx.x * 256 + tid;
    const bool in = c < a.C;
    float part[BOUND_KS_MAX];
#pragma unroll
    for (int ks = 0; ks < BOUND_KS_MAX; ++ks) part[ks] = (in && ks < KS) ? P[((size_t)ks * a.B + b) * a.C + c] : 0.f;
    const float Rc = in ? a.R[c] : 0.f, bm = in ? a.bmax[c] : 0.f;
    const int nc = in ? a.n[c] : 0;
    const uint4* hsrc = reinterpret_cast<const uint4*>(a.h) + (size_t)b * (a.d >> 3);
    float ss = 0.f;
    for (int i = tid; i < (a.d >> 3); i += 256) {
        const uint4 v = hsrc[i];
        ss = dot8_bf16(v, v, ss);
    }
    const float hn = sqrtf(block_sum(ss, red));
    if (blockIdx.x == 0 && tid == 0 && hn_out) hn_out[b] = hn;
    if (!in) return;
    float u = 0.f;
#pragma unroll
    for (int ks = 0; ks < BOUND_KS_MAX; ++ks) u += part[ks];
    U_out[(size_t)b * a.C + c] = nc == 0 ? -INFINITY : bound_value(a, c, u, Rc, bm, hn);
}

// ================================================================================================ block scans
// Combination of everything owned by the threads AFTER this one (exclusive suffix), for log-sum-exp partials.
__device__ __forceinline__ LseAcc block_excl_suffix_lse(LseAcc v, LseAcc* wtot) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    LseAcc x = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        LseAcc y;
        y.m = __shfl_down(x.m, o, CSV_WAVE);
        y.s = __shfl_down(x.s, o, CSV_WAVE);
        if (lane + o < 64) x = lse_combine(x, y);
    }
    LseAcc after;
    after.m = __shfl_down(x.m, 1, CSV_WAVE);
    after.s = __shfl_down(x.s, 1, CSV_WAVE);
    if (lane == 63) {
        after.m = -INFINITY;
        after.s = 0.f;
    }
    __syncthreads();
    if (lane == 0) wtot[w] = x;
    __syncthreads();
    LseAcc tail;
    tail.m = -INFINITY;
    tail.s = 0.f;
    for (int i = nw - 1; i > w; --i) tail = lse_combine(wtot[i], tail);
    return lse_combine(after, tail);
}

// ================================================================================================ shared LDS of the per-sequence kernels
struct BigItem {
    int row0, n, pos, tbase;
};
#define CAND_CAP SEQ_THREADS
#define RANK_DIRECT 256      // up to this many values are ranked against each other directly (a multiple of four, at most SEQ_THREADS)
struct SeqShared {
    unsigned hist[256];
    float redf[16];
    int redi[16];
    int scan3[48];
    int rank[SEQ_THREADS];
    u64 redu[32];
    LseAcc redl[16];
    unsigned sel, rem, eq, cnt;
    int tbase, nbig;
    BigItem big[BIGQ];
    float wval[CSV_MAX_K];
    int wid[CSV_MAX_K];
};
// Later rounds collect the values at or above the previous round's k-th logit, and their ids, behind the staged
// logits in the dynamic LDS (a region the cluster data of a large index covers anyway).
#define CAND_OFF (STAGE_CAP * 8)
#define CAND_BYTES ((CAND_CAP + 4) * 4 + CAND_CAP * 4)

// ================================================================================================ helpers shared by seed/cert
__device__ __forceinline__ void write_invalid(const StepArgs& a, int b) {
    for (int t = threadIdx.x; t < a.k; t += blockDim.x) {
        a.out.d_ids[(size_t)b * a.k + t] = -1;
        a.out.d_logits[(size_t)b * a.k + t] = NAN;
        if (a.out.d_probs) a.out.d_probs[(size_t)b * a.k + t] = NAN;
        if (a.out.d_cum) a.out.d_cum[(size_t)b * a.k + t] = NAN;
    }
    if (threadIdx.x == 0 && a.out.d_nucleus) a.out.d_nucleus[b] = 0;
    if (threadIdx.x == 0) {
        a.out.d_lse[b] = NAN;
        a.out.d_flags[b] = CSV_FLAG_INVALID_INPUT;
        a.out.d_n_rows[b] = 0;
        a.out.d_n_clusters[b] = 0;
        if (a.out.d_rounds) a.out.d_rounds[b] = 0;
        a.st[b].status = ST_INVALID;
    }
}

// Called by one thread: hand sequence b to the full-vocabulary path.
__device__ __forceinline__ void push_fallback(const StepArgs& a, int b, int rounds) {
    const int slot = atomicAdd(&a.counters[CNT_FALLBACK], 1);
    __hip_atomic_store(&a.counters[CNT_TAIL_NEEDED], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    a.fb_list[slot] = b;
    a.st[b].status = ST_FALLBACK;
    a.st[b].fb_slot = slot;
    if (a.out.d_rounds) a.out.d_rounds[b] = rounds;
}

// Per-sequence cluster data in LDS: keys[Npad], first permuted row of each cluster offl[C+1], and
// vl[c] = ln n_c + U_c (the cluster's term of the log tail mass; -inf for an empty cluster).
struct ClusterLds {
    u64* keys;
    int* offl;
    float* vl;
};
__device__ __forceinline__ ClusterLds carve_clusters(u64* arena, int Npad, int C) {
    ClusterLds L;
    L.keys = arena;
    L.offl = reinterpret_cast<int*>(arena + Npad);
    L.vl = reinterpret_cast<float*>(L.offl + C + 1);
    return L;
}
__device__ __forceinline__ void load_clusters(const StepArgs& a, int b, const ClusterLds& L) {
    const int tid = threadIdx.x, nt = blockDim.x;
    // four clusters per thread and trip, all sixteen loads issued before the first use (n_c = off[c+1] - off[c])
    for (int c0 = 0; c0 < a.C; c0 += 4 * nt) {
        float u[4], ln[4];
        int o0[4], o1[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = c0 + q * nt + tid;
            const bool in = c < a.C;
            u[q] = in ? a.U[(size_t)b * a.C + c] : 0.f;
            ln[q] = in ? a.lnn[c] : 0.f;
            o0[q] = in ? a.off[c] : 0;
            o1[q] = in ? a.off[c + 1] : 0;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = c0 + q * nt + tid;
            if (c < a.C) {
                const bool some = o1[q] > o0[q];
                L.offl[c] = o0[q];
                if (c == a.C - 1) L.offl[a.C] = o1[q];
                L.keys[c] = some ? ckey(u[q], c) : 0ull;
                L.vl[c] = some ? ln[q] + u[q] : -INFINITY;
            }
        }
    }
}

// Exclusive prefix sums of three ints per thread in one pass.  wtot: 48 ints of LDS.
__device__ __forceinline__ void block_excl_scan3(int& v0, int& v1, int& v2, int* wtot, int& t0, int& t1, int& t2) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    int x0 = v0, x1 = v1, x2 = v2;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int y0 = __shfl_up(x0, o, CSV_WAVE), y1 = __shfl_up(x1, o, CSV_WAVE), y2 = __shfl_up(x2, o, CSV_WAVE);
        if (lane >= o) {
            x0 += y0;
            x1 += y1;
            x2 += y2;
        }
    }
    __syncthreads();
    if (lane == 63) {
        wtot[w] = x0;
        wtot[16 + w] = x1;
        wtot[32 + w] = x2;
    }
    __syncthreads();
    int b0 = 0, b1 = 0, b2 = 0;
    t0 = t1 = t2 = 0;
    for (int i = 0; i < nw; ++i) {
        const int a0 = wtot[i], a1 = wtot[16 + i], a2 = wtot[32 + i];
        if (i < w) {
            b0 += a0;
            b1 += a1;
            b2 += a2;
        }
        t0 += a0;
        t1 += a1;
        t2 += a2;
    }
    v0 = b0 + x0 - v0;
    v1 = b1 + x1 - v1;
    v2 = b2 + x2 - v2;
}

// Opens every cluster c with flag(c): its rows get consecutive positions from pos_base on (cluster id order), its
// row tiles go to the sequence's region of the round's work list (two lists, used by even and odd rounds), its id is appended to the sequence's list of
// opened clusters.  All threads of the block call; flag must be the same function of c in both passes.
template <class FlagFn>
__device__ __forceinline__ void emit_clusters(const StepArgs& a, int b, int round, int pos_base, int sel_base, FlagFn flag,
                                              const ClusterLds& L, SeqShared& s) {
    const int tid = threadIdx.x, nt = blockDim.x, C = a.C;
    const int E = (C + nt - 1) / nt;
    const int c0 = min(C, tid * E), c1 = min(C, c0 + E);
    int cnt = 0, rows = 0, tiles = 0;
    for (int c = c0; c < c1; ++c)
        if (flag(c)) {
            const int n = L.offl[c + 1] - L.offl[c];
            cnt += 1;
            rows += n;
            tiles += (n + TILE_ROWS - 1) / TILE_ROWS;
        }
    int tot_cnt, tot_rows, tot_tiles;
    block_excl_scan3(cnt, rows, tiles, s.scan3, tot_cnt, tot_rows, tot_tiles);
    if (tid == 0) {
        a.counters[CNT_TILES + round * CSV_MAX_BATCH + b] = tot_tiles;
        __hip_atomic_store(&a.counters[CNT_TAIL_NEEDED], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s.nbig = 0;
    }
    __syncthreads();
    Tile* tl = a.tiles[round & 1] + (size_t)b * a.tile_stride;
    int tb = tiles, pos = pos_base + rows, si = sel_base + cnt;
    for (int c = c0; c < c1; ++c)
        if (flag(c)) {
            const int r0 = L.offl[c], n = L.offl[c + 1] - r0, ntc = (n + TILE_ROWS - 1) / TILE_ROWS;
            a.sel[(size_t)b * C + si++] = c;
            int slot = BIGQ;
            if (ntc > 16) slot = atomicAdd(&s.nbig, 1);
            if (slot < BIGQ) {
                BigItem it;
                it.row0 = r0; it.n = n; it.pos = pos; it.tbase = tb;
                s.big[slot] = it;
            } else {
                for (int t = 0; t < ntc; ++t) {
                    Tile x;
                    x.b = b; x.row0 = r0 + t * TILE_ROWS; x.nrows = min(TILE_ROWS, n - t * TILE_ROWS); x.pos = pos + t * TILE_ROWS;
                    tl[tb + t] = x;
                }
            }
            tb += ntc;
            pos += n;
        }
    __syncthreads();
    const int nbig = min(s.nbig, BIGQ);
    for (int q = 0; q < nbig; ++q) {
        const BigItem it = s.big[q];
        const int ntc = (it.n + TILE_ROWS - 1) / TILE_ROWS;
        for (int t = tid; t < ntc; t += nt) {
            Tile x;
            x.b = b; x.row0 = it.row0 + t * TILE_ROWS; x.nrows = min(TILE_ROWS, it.n - t * TILE_ROWS); x.pos = it.pos + t * TILE_ROWS;
            tl[it.tbase + t] = x;
        }
    }
    __syncthreads();
}

// Largest bound and log tail mass over the unopened clusters {c : 0 < key_c < kappa}: a max pass, then a sum pass.
__device__ __forceinline__ void tail_stats(const StepArgs& a, const ClusterLds& L, u64 kappa, SeqShared& s, float& nxtU, float& T) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    u64 best = 0;
    float vmax = -INFINITY;
    for (int c = threadIdx.x; c < a.C; c += blockDim.x) {
        const u64 kx = L.keys[c];
        if (kx != 0 && kx < kappa) {
            best = kx > best ? kx : best;
            vmax = fmaxf(vmax, L.vl[c]);
        }
    }
    best = wave_max_u64(best);
    vmax = wave_max(vmax);
    __syncthreads();
    if (lane == 0) {
        s.redu[w] = best;
        s.redf[w] = vmax;
    }
    __syncthreads();
    best = s.redu[0];
    vmax = s.redf[0];
    for (int i = 1; i < nw; ++i) {
        best = s.redu[i] > best ? s.redu[i] : best;
        vmax = fmaxf(vmax, s.redf[i]);
    }
    float sum = 0.f;
    if (vmax > -INFINITY)
        for (int c = threadIdx.x; c < a.C; c += blockDim.x) {
            const u64 kx = L.keys[c];
            if (kx != 0 && kx < kappa) sum += expf(L.vl[c] - vmax);
        }
    sum = block_sum(sum, s.redf);
    nxtU = best ? ckey_bound(best) : -INFINITY;
    T = vmax > -INFINITY ? vmax + logf(sum) : -INFINITY;
}

// ================================================================================================ gathered GEMV
// Work item = up to TILE_ROWS consecutive rows of W' for one sequence; one row per wave (8 waves).  Tiles of
// sequence b sit in its own region of the round's list; a prefix over the per-sequence counts maps a global tile
// number to (sequence, tile).  A block takes a contiguous run of tiles and has two of them in flight: both tiles' rows are requested in full (up to
// 16 KB per row) before anything is reduced, and the descriptors of the next pair are requested behind them, so an
// iteration costs one memory round trip for 16 rows.  h of the two tiles' sequences sits in two LDS slots (bf16)
// that are refilled only when the sequence changes.  128-bit loads, float32 accumulation, DPP wave reduction.
#define TILE_PF 16         // 128-bit pieces of a row requested at once per lane: a whole row up to d = 8192
struct GemvShared {
    int pre[CSV_MAX_BATCH + 1];
    int wsum[16];
};
// block / nblocks: this block's position in the set of blocks that share the work.  hs4: 2 * d * 2 bytes of LDS.
__device__ __forceinline__ void gemv_tiles_device(const StepArgs& a, int round, uint4* hs4, GemvShared& gs, int block, int nblocks) {
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6;
    {
        const int mine = tid < a.B ? a.counters[CNT_TILES + round * CSV_MAX_BATCH + tid] : 0;
        int x = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int y = __shfl_up(x, o, CSV_WAVE);
            if (lane >= o) x += y;
        }
        __syncthreads();
        if (lane == 63) gs.wsum[wave] = x;
        __syncthreads();
        int base = 0;
        for (int i = 0; i < wave; ++i) base += gs.wsum[i];
        if (tid == 0) gs.pre[0] = 0;
        if (tid < CSV_MAX_BATCH) gs.pre[tid + 1] = base + x;
        __syncthreads();
    }
    const int total = gs.pre[a.B];
    const int nch = a.d >> 3;
    const Tile* tl = a.tiles[round & 1];
    auto fetch = [&](int g) {        // descriptor of global tile g; an empty tile past the end
        Tile t;
        t.b = 0; t.row0 = 0; t.nrows = 0; t.pos = 0;
        if (g < total) {
            int lo = 0, hi = a.B;   // largest b with pre[b] <= g
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (gs.pre[mid] <= g) lo = mid; else hi = mid;
            }
            t = tl[(size_t)lo * a.tile_stride + (g - gs.pre[lo])];
        }
        return t;
    };
    // a block takes a contiguous run of the list: mostly one sequence (h is staged once or twice per block, not
    // once per tile) and neighbouring rows
    const int per = (total + nblocks - 1) / nblocks;
    const int g0 = block * per, g1 = min(total, g0 + per);
    int cached[2] = {-1, -1};
    Tile tA = fetch(g0 < g1 ? g0 : total), tB = fetch(g0 + 1 < g1 ? g0 + 1 : total);
    for (int g = g0; g < g1; g += 2) {
        const Tile t[2] = {tA, tB};
        uint4 pf[2][TILE_PF];
        const uint4* w[2];
        float bias[2];
        int ids[2];
        bool act[2];
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            act[q] = wave < t[q].nrows;
            const int r = t[q].row0 + (act[q] ? wave : 0);
            w[q] = reinterpret_cast<const uint4*>(a.Wp + (size_t)r * a.d);
#pragma unroll
            for (int j = 0; j < TILE_PF; ++j) {
                const int i = lane + 64 * j;
                pf[q][j] = (act[q] && i < nch) ? w[q][i] : make_uint4(0, 0, 0, 0);
            }
            bias[q] = 0.f;
            ids[q] = 0;
            if (act[q] && lane == 0) {
                bias[q] = a.bp[r];
                ids[q] = a.perm[r];
            }
        }
        // next pair's descriptors ride behind the row requests
        tA = fetch(g + 2 < g1 ? g + 2 : total);
        tB = fetch(g + 3 < g1 ? g + 3 : total);
        // h of the two sequences: slot q holds the sequence of tile q
        bool staged = false;
#pragma unroll
        for (int q = 0; q < 2; ++q)
            if (t[q].nrows > 0 && cached[q] != t[q].b) {
                if (!staged) __syncthreads();          // everyone is done with the slots' previous contents
                staged = true;
                const uint4* hsrc = reinterpret_cast<const uint4*>(a.h) + (size_t)t[q].b * nch;
                for (int i = tid; i < nch; i += nt) hs4[q * nch + i] = hsrc[i];
                cached[q] = t[q].b;
            }
        if (staged) __syncthreads();
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            if (!act[q]) continue;
            const uint4* hq = hs4 + q * nch;
            float acc = 0.f;
#pragma unroll
            for (int j = 0; j < TILE_PF; ++j) {
                const int i = lane + 64 * j;
                if (i < nch) acc = dot8_bf16(pf[q][j], hq[i], acc);
            }
            for (int i = lane + 64 * TILE_PF; i < nch; i += 64) acc = dot8_bf16(w[q][i], hq[i], acc);
            acc = wave_sum(acc);
            if (lane == 0) {
                const size_t o = (size_t)t[q].b * a.K_cap + t[q].pos + wave;
                a.slog[o] = acc + bias[q];
                a.sid[o] = ids[q];
            }
        }
    }
}

// Copy n 32-bit words from global memory to LDS.  Every trip issues eight loads per thread before the first
// store, also in the ragged last trip (out-of-range lanes load nothing), so a copy of up to 8 x blockDim words is
// one memory round trip.
template <class T>
__device__ __forceinline__ void stage_to_lds(T* dst, const T* __restrict__ src, int n) {
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int i = tid; i < n; i += 8 * nt) {
        T r[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) r[q] = i + q * nt < n ? src[i + q * nt] : T(0);
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (i + q * nt < n) dst[i + q * nt] = r[q];
    }
}
// Two arrays of the same length at once (logits and token ids): both arrays' loads are in flight together.
__device__ __forceinline__ void stage2_to_lds(float* dv, const float* __restrict__ sv, int* di, const int* __restrict__ si, int n) {
    const int tid = threadIdx.x, nt = blockDim.x;
    for (int i = tid; i < n; i += 8 * nt) {
        float rv[8];
        int ri[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const bool in = i + q * nt < n;
            rv[q] = in ? sv[i + q * nt] : 0.f;
            ri[q] = in ? si[i + q * nt] : 0;
        }
#pragma unroll
        for (int q = 0; q < 8; ++q)
            if (i + q * nt < n) {
                dv[i + q * nt] = rv[q];
                di[i + q * nt] = ri[q];
            }
    }
}

// ================================================================================================ block top-k
// kk-th largest key among the elements for which key(i, kx) returns true (1 <= kk <= their number).
// On return: kth = that key, need_eq = how many elements equal to it belong to the largest kk, n_eq = how many equal it.
// Needs blockDim.x >= 256.
template <class KeyFn>
__device__ __forceinline__ void radix_select(int n, unsigned kk, KeyFn key, SeqShared& s, unsigned& kth,
                                             unsigned& need_eq, unsigned& n_eq) {
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, w = tid >> 6, nw = (nt + 63) >> 6;
    // Bytes that all keys share from the top need no pass (logits of one cluster differ only in their low bits,
    // and a histogram pass over a shared byte would send every element to the same bin).
    unsigned kmin = 0xffffffffu, kmax = 0u;
    for (int i = tid; i < n; i += nt) {
        unsigned kx;
        if (key(i, kx)) {
            kmin = kx < kmin ? kx : kmin;
            kmax = kx > kmax ? kx : kmax;
        }
    }
    kmax = wave_max_u(kmax);
    kmin = ~wave_max_u(~kmin);
    __syncthreads();
    if (lane == 0) {
        s.hist[w] = kmax;
        s.hist[16 + w] = kmin;
    }
    __syncthreads();
    for (int i = 0; i < nw; ++i) {
        kmax = s.hist[i] > kmax ? s.hist[i] : kmax;
        kmin = s.hist[16 + i] < kmin ? s.hist[16 + i] : kmin;
    }
    __syncthreads();
    const unsigned diff = kmin ^ kmax;
    int first_shift = 24;
    unsigned prefix = 0, mask = 0, rem = kk, eq = 0;
    while (first_shift > 0 && ((diff >> first_shift) & 0xffu) == 0) {
        prefix |= kmax & (0xffu << first_shift);
        mask |= 0xffu << first_shift;
        first_shift -= 8;
    }
    for (int shift = first_shift; shift >= 0; shift -= 8) {
        for (int t = tid; t < 256; t += nt) s.hist[t] = 0;
        __syncthreads();
        for (int i0 = 0; i0 < n; i0 += nt) {
            const int i = i0 + tid;
            unsigned kx = 0;
            const bool in = i < n && key(i, kx) && (kx & mask) == prefix;
            const unsigned dg = (kx >> shift) & 255u;
            // one atomic per wave when every participating lane has the same digit
            const unsigned long long act = __ballot(in);
            if (act) {
                const unsigned d0 = __shfl(dg, __ffsll((long long)act) - 1, CSV_WAVE);
                const unsigned long long same = __ballot(in && dg == d0);
                if (same == act) {
                    if (lane == __ffsll((long long)act) - 1) atomicAdd(&s.hist[d0], (unsigned)__popcll(act));
                } else if (in) {
                    atomicAdd(&s.hist[dg], 1u);
                }
            }
        }
        __syncthreads();
        if (tid < 64) {
            // lane l owns bins 4l..4l+3; suffix sums by a descending scan inside the first wave
            const unsigned h0 = s.hist[4 * lane], h1 = s.hist[4 * lane + 1], h2 = s.hist[4 * lane + 2], h3 = s.hist[4 * lane + 3];
            const unsigned mine = h0 + h1 + h2 + h3;
            unsigned x = mine;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const unsigned y = __shfl_down(x, o, CSV_WAVE);
                if (lane + o < 64) x += y;
            }
            const unsigned gt3 = x - mine;          // elements in bins above 4l+3
            const unsigned gt2 = gt3 + h3, gt1 = gt2 + h2, gt0 = gt1 + h1, ge0 = gt0 + h0;
            if (ge0 >= rem && gt3 < rem) {           // the kk-th falls into one of my bins
                unsigned selb, gt, cntb;
                if (gt2 >= rem) { selb = 3; gt = gt3; cntb = h3; }
                else if (gt1 >= rem) { selb = 2; gt = gt2; cntb = h2; }
                else if (gt0 >= rem) { selb = 1; gt = gt1; cntb = h1; }
                else { selb = 0; gt = gt0; cntb = h0; }
                s.sel = 4u * lane + selb;
                s.rem = rem - gt;
                s.eq = cntb;
            }
        }
        __syncthreads();
        prefix |= s.sel << shift;
        mask |= 0xffu << shift;
        rem = s.rem;
        eq = s.eq;
        if (shift > 0 && eq <= 256u) {
            // few candidates left in the selected bin: list them and rank them directly instead of more passes
            __syncthreads();
            if (tid == 0) s.cnt = 0;
            __syncthreads();
            for (int i = tid; i < n; i += nt) {
                unsigned kx = 0;
                if (key(i, kx) && (kx & mask) == prefix) s.hist[atomicAdd(&s.cnt, 1u)] = kx;
            }
            __syncthreads();
            if (tid < (int)eq) {
                const unsigned v = s.hist[tid];
                unsigned gt = 0, ge = 0;
                for (unsigned j = 0; j < eq; ++j) {
                    const unsigned x = s.hist[j];
                    gt += x > v;
                    ge += x >= v;
                }
                if (gt < rem && rem <= ge) {     // every thread holding this value writes the same three numbers
                    s.sel = v;
                    s.rem = rem - gt;
                    s.eq = ge - gt;
                }
            }
            __syncthreads();
            kth = s.sel;
            need_eq = s.rem;
            n_eq = s.eq;
            __syncthreads();
            return;
        }
    }
    kth = prefix;
    need_eq = rem;
    n_eq = eq;
}

// Largest min(k,n) of n values in order (value descending, id ascending).  Result in s.wval / s.wid.
// val(i) and id_of(i) may read LDS or global memory.  Returns min(k,n).
template <class ValFn, class IdFn>
__device__ __forceinline__ int block_topk(int n, int k, ValFn val, IdFn id_of, SeqShared& s) {
    const int tid = threadIdx.x, nt = blockDim.x;
    const int kk = min(k, n);
    if (kk <= 0) return 0;
    if (n <= nt) {
        // rank of every element = number of larger values.  The n x n comparisons are spread over all threads:
        // thread (e, slice) compares element e with one slice of the others and adds its count (larger values in
        // the low half, equal values in the high half) to rank[e].  Ids are looked at only by elements that have
        // an equal somewhere else.  blockDim.x must be a power of two.
        int lg = 0;
        while ((1 << lg) < n) ++lg;
        const int npad = 1 << lg, slices = nt >> lg;
        const int e = tid & (npad - 1), sl = tid >> lg;
        __syncthreads();
        if (tid < npad) s.rank[tid] = 0;
        __syncthreads();
        const int len = ((n + slices - 1) / slices + 3) & ~3;
        const int j0 = sl * len, j1 = min(n, j0 + len);
        if (e < n && j0 < j1) {
            const float v = val(e);
            int gt = 0, eq = 0;
            int j = j0;
#pragma unroll 2
            for (; j + 4 <= j1; j += 4) {
                const float q0 = val(j), q1 = val(j + 1), q2 = val(j + 2), q3 = val(j + 3);
                gt += (q0 > v) + (q1 > v) + (q2 > v) + (q3 > v);
                eq += (q0 == v) + (q1 == v) + (q2 == v) + (q3 == v);
            }
            for (; j < j1; ++j) {
                const float vj = val(j);
                gt += vj > v;
                eq += vj == v;
            }
            atomicAdd(&s.rank[e], gt | (eq << 16));
        }
        __syncthreads();
        if (tid < n) {
            const float v = val(tid);
            const int id = id_of(tid);
            const int packed = s.rank[tid];
            int rank = packed & 0xffff;
            if ((packed >> 16) > 1)
                for (int i = 0; i < n; ++i)
                    if (val(i) == v && id_of(i) < id) rank += 1;
            if (rank < kk) {
                s.wval[rank] = v;
                s.wid[rank] = id;
            }
        }
        __syncthreads();
        return kk;
    }
    if (kk < n) {
        unsigned kth, need, neq;
        radix_select(n, (unsigned)kk, [&](int i, unsigned& kx) { kx = lkey(val(i)); return true; }, s, kth, need, neq);
        unsigned idkey = 0;   // boundary elements win when ~id >= idkey
        if (need < neq) {
            unsigned u1, u2;
            radix_select(n, need,
                         [&](int i, unsigned& kx) {
                             if (lkey(val(i)) != kth) return false;
                             kx = ~(unsigned)id_of(i);
                             return true;
                         },
                         s, idkey, u1, u2);
        }
        if (tid == 0) s.cnt = 0;
        __syncthreads();
        for (int i = tid; i < n; i += nt) {
            const float v = val(i);
            const unsigned kx = lkey(v);
            if (kx >= kth) {
                const int id = id_of(i);
                if (kx > kth || (~(unsigned)id) >= idkey) {
                    const unsigned slot = atomicAdd(&s.cnt, 1u);
                    if (slot < CSV_MAX_K) {
                        s.wval[slot] = v;
                        s.wid[slot] = id;
                    }
                }
            }
        }
        __syncthreads();
    } else {
        for (int i = tid; i < n; i += nt) {
            s.wval[i] = val(i);
            s.wid[i] = id_of(i);
        }
        __syncthreads();
    }
    // order the winners in place: ranks first, then a permuted write (CSV_MAX_K <= 4 * 256 threads)
    float mv[4];
    int mi[4], mr[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int t = tid + e * nt;
        mr[e] = -1;
        if (t < kk) {
            const float v = s.wval[t];
            const int id = s.wid[t];
            int rank = 0;
            for (int j = 0; j < kk; ++j) {
                const float vj = s.wval[j];
                rank += (vj > v) || (vj == v && s.wid[j] < id);
            }
            mv[e] = v; mi[e] = id; mr[e] = rank;
        }
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (mr[e] >= 0) {
            s.wval[mr[e]] = mv[e];
            s.wid[mr[e]] = mi[e];
        }
    __syncthreads();
    return kk;
}

// max and sum exp(x - max) of n values, fixed reduction order
template <class ValFn>
__device__ __forceinline__ LseAcc block_lse(int n, ValFn val, SeqShared& s) {
    float mx = -INFINITY;
    for (int i = threadIdx.x; i < n; i += blockDim.x) mx = fmaxf(mx, val(i));
    mx = block_max(mx, s.redf);
    float sm = 0.f;
    if (mx > -INFINITY)
        for (int i = threadIdx.x; i < n; i += blockDim.x) sm += expf(val(i) - mx);
    sm = block_sum(sm, s.redf);
    LseAcc r;
    r.m = mx;
    r.s = sm;
    return r;
}

// ================================================================================================ prefix search
// The shortest prefix of the bound order, no shorter than the open one, whose log tail mass is within lam of Z0
// (Theorem 2): returns the key of its last cluster.  In terms of keys: the largest key kappa <= kappa0 such that the
// clusters below it weigh  sum_{key_c < kappa} n_c exp(U_c)  <=  exp(Z0 + lam).  No sort: the key is found digit by
// digit from the top (eight bits a pass).  Among the keys that share the digits fixed so far, the clusters of a
// smaller digit all lie below those of a larger one, so a digit can hold the answer when it is not empty and the
// weight below its smallest key (everything below the fixed digits, plus the smaller digits) is within the limit;
// the largest such digit is taken.  Weights are summed as 64-bit fixed point relative to the limit (2^-40 steps, each
// term capped at 2^9, which already exceeds the limit of 1): integer sums do not depend on the order of the atomic
// additions, so the result is the same in every run.  Leaves the cluster data in LDS as it is.  Uses s.rank and s.hist.
__device__ __forceinline__ u64 softmax_prefix_key(const StepArgs& a, const ClusterLds& L, u64 kappa0, float Z0, SeqShared& s) {
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63;
    u64* H = reinterpret_cast<u64*>(s.rank);               // 256 weights
    unsigned* cnt = s.hist;                                // 256 counts
    const float shift = Z0 + a.lam;
    const u64 LIMIT = 1ull << 40;
    u64 prefix = 0, base = 0;
    for (int sb = 56; sb >= 0; sb -= 8) {
        if (sb == 24 || sb == 16) {                        // bits 16..31 of ~c: ones for every cluster id below 65536
            prefix |= 0xffull << sb;
            continue;
        }
        if (tid < 256) {
            H[tid] = 0ull;
            cnt[tid] = 0u;
        }
        __syncthreads();
        for (int c = tid; c < a.C; c += nt) {
            const u64 kx = L.keys[c];
            const bool match = sb == 56 || ((kx ^ prefix) >> (sb + 8)) == 0;
            if (kx != 0 && kx <= kappa0 && match) {
                const float e = expf(fminf(L.vl[c] - shift, 6.f));         // e^6 < 2^9
                const unsigned dg = (unsigned)(kx >> sb) & 255u;
                atomicAdd(reinterpret_cast<unsigned long long*>(&H[dg]), (unsigned long long)(e * 1099511627776.f));
                atomicAdd(&cnt[dg], 1u);
            }
        }
        __syncthreads();
        if (tid < 64) {
            // lane l owns digits 4l..4l+3; weights below a digit by an ascending scan inside the first wave
            u64 h[4];
            unsigned n4[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                h[q] = H[4 * lane + q];
                n4[q] = cnt[4 * lane + q];
            }
            const u64 mine = h[0] + h[1] + h[2] + h[3];
            u64 x = mine;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const u64 y = __shfl_up(x, o, CSV_WAVE);
                if (lane >= o) x += y;
            }
            u64 below[4];
            below[0] = base + (x - mine);
            below[1] = below[0] + h[0];
            below[2] = below[1] + h[1];
            below[3] = below[2] + h[2];
            int pick = -1;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (n4[q] != 0 && below[q] <= LIMIT) pick = 4 * lane + q;
            const int best = (int)wave_max_u((unsigned)(pick + 1)) - 1;
            if (best >= 0 && (best >> 2) == lane) {
                s.sel = (unsigned)best;
                s.redu[0] = below[best & 3];
            }
            if (best < 0 && lane == 0) {                  // cannot happen (the smallest key has nothing below it); stay defined
                s.sel = 0u;
                s.redu[0] = base;
            }
        }
        __syncthreads();
        prefix |= (u64)s.sel << sb;
        base = s.redu[0];
    }
    __syncthreads();
    return prefix;
}

// Ordered top-kk (value descending, id ascending) of len <= blockDim.x values V in LDS with ids I; V is followed by
// -inf up to the next multiple of four.  One pass, one barrier: thread (e, slice) compares value e with one slice of
// the others (larger ones, equal ones) and notes the slice's maximum; after the barrier thread e adds the slices'
// counts to its rank (ids are looked at only among equal values) and writes itself to its place in s.wval / s.wid.
// Returns the largest value; v is the value of element threadIdx.x (threadIdx.x < len).  The caller's next barrier
// publishes the list.  blockDim.x is a power of two.
__device__ __forceinline__ float rank_small(const float* V, const int* I, int len, int kk, SeqShared& s, float& v) {
    const int tid = threadIdx.x, nt = blockDim.x;
    int lg = 5;
    while ((1 << lg) < len) ++lg;
    const int npad = 1 << lg, slices = nt >> lg;           // slices <= 16
    const int e = tid & (npad - 1), sl = tid >> lg;
    const int len4 = (len + 3) >> 2;                         // slices of whole float4's
    const int seg4 = (len4 + slices - 1) / slices;
    const int q0 = min(len4, sl * seg4), q1 = min(len4, q0 + seg4);
    const float ve = V[min(e, max(len, 1) - 1)];
    int gt = 0, eq = 0;
    float mx = -INFINITY;
    const float4* v4 = reinterpret_cast<const float4*>(V);
#pragma unroll 8
    for (int q = q0; q < q1; ++q) {
        const float4 x = v4[q];
        gt += (x.x > ve) + (x.y > ve) + (x.z > ve) + (x.w > ve);
        eq += (x.x == ve) + (x.y == ve) + (x.z == ve) + (x.w == ve);
        mx = fmaxf(fmaxf(mx, fmaxf(x.x, x.y)), fmaxf(x.z, x.w));
    }
    s.rank[tid] = gt | (eq << 16);                          // rank[sl * npad + e]
    if (e == 0) s.redf[sl] = mx;
    __syncthreads();
    float vmax = s.redf[0];
    for (int q = 1; q < slices; ++q) vmax = fmaxf(vmax, s.redf[q]);
    v = ve;                                                 // tid < len <= npad: e is tid
    if (tid < len) {
        int packed = 0;
        for (int q = 0; q < slices; ++q) packed += s.rank[q * npad + tid];
        int rank = packed & 0xffff;
        const int id = I[tid];
        if ((packed >> 16) > 1)
            for (int i = 0; i < len; ++i)
                if (V[i] == v && I[i] < id) rank += 1;
        if (rank < kk) {
            s.wval[rank] = v;
            s.wid[rank] = id;
        }
    }
    return vmax;
}

// Ordered top-kk of m <= blockDim.x candidates V / I in LDS (one per thread), none of them below lo: a counting
// sort into 256 equal-width buckets between lo and hi, largest values first, then every candidate whose bucket starts within the first
// kk places ranks itself against the members of its bucket (equal values by id); values above hi share the first bucket.  Exact for any distribution of the
// values (a crowded bucket only costs time); the comparisons of rank_small grow with m * m, these with m.  V / I are
// reordered (bucket by bucket; the order inside a bucket depends on timing, the ranks do not).  The caller's next
// barrier publishes s.wval / s.wid.  Uses s.hist, s.rank, s.redi.
__device__ __forceinline__ void rank_buckets(float* V, int* I, int m, int kk, float lo, float hi, SeqShared& s) {
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const float scale = (hi > lo && lo > -INFINITY && hi < INFINITY) ? 255.f / (hi - lo) : 0.f;
    float v = 0.f;
    int id = 0, d = 0;
    if (tid < m) {
        v = V[tid];
        id = I[tid];
        d = scale > 0.f ? 255 - min(255, max(0, (int)((v - lo) * scale))) : 0;
    }
    if (tid < 256) s.hist[tid] = 0;
    __syncthreads();
    unsigned slot = 0;
    if (tid < m) slot = atomicAdd(&s.hist[d], 1u);
    __syncthreads();
    if (tid < 256) {
        const int c = (int)s.hist[tid];
        int x = c;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int y = __shfl_up(x, o, CSV_WAVE);
            if (lane >= o) x += y;
        }
        if (lane == 63) s.redi[w] = x;
        s.rank[tid] = x - c;                                // first place of the bucket, counted within its wave of buckets
    }
    __syncthreads();
    int start = 0, cnt = 0;
    if (tid < m) {
        start = s.rank[d];
        for (int i = 0; i < (d >> 6); ++i) start += s.redi[i];
        cnt = (int)s.hist[d];
        V[start + (int)slot] = v;
        I[start + (int)slot] = id;
    }
    __syncthreads();
    if (tid < m && start < kk) {
        int r = start;
#pragma unroll 4
        for (int j = start; j < start + cnt; ++j) {
            const float x = V[j];
            r += (x > v || (x == v && I[j] < id)) ? 1 : 0;
        }
        if (r < kk) {
            s.wval[r] = v;
            s.wid[r] = id;
        }
    }
}
#define RANK_BUCKETS_MIN 128     // more candidates than this (with a finite range) take rank_buckets instead of rank_small

// Ordered top-k of len > RANK_DIRECT values staged at the start of the dynamic LDS (ranking all of them against each
// other costs len^2 comparisons: 10 us at 512).  Everything below a threshold that k of the values are known to reach
// is out; the values at or above it (usually few more than k) are collected behind the staged data and ranked in one
// pass.  First threshold: theta, a value the caller knows k of the values to reach (-inf: none).  Failing that, or
// when more than CAND_CAP values reach it: the k-th largest of RANK_DIRECT group maxima.  short_ok: the values are one chunk of several
// and fewer than k of them may reach theta (the merged lists still hold the overall top-k).  The collected order
// depends on timing, the ranking does not.  On success s.wval / s.wid hold kkv entries once the caller has passed a
// barrier, vmax is the largest value; on failure (k > RANK_DIRECT, too many survivors) nothing is decided.
// MERGE: the values are lists of several chunks, unused places marked by the id 0x7fffffff (and the value -inf): those are
// left out, and the first attempt also runs without a threshold (len may then be RANK_DIRECT or less).
// LATE_IDS: idf reads global memory: the candidates are collected with their positions and all look their ids up
// together afterwards (a load in the collecting loop would be waited for in every trip that collects something).
template <bool MERGE = false, bool LATE_IDS = false, class IdFn>
__device__ __forceinline__ bool threshold_topk(int len, int k, float theta, bool short_ok, IdFn idf, SeqShared& s, int& kkv, float& vmax) {
    extern __shared__ __align__(16) u64 arena[];
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63;
    const float* V = reinterpret_cast<const float*>(arena);
    const int k0 = min(k, len);
    auto attempt = [&](float th) -> bool {
        float* wmax = reinterpret_cast<float*>(s.redu);        // not s.hist / s.redf: the ranking writes those while others still read here
        float* cval = reinterpret_cast<float*>(reinterpret_cast<char*>(arena) + CAND_OFF);
        int* cid = reinterpret_cast<int*>(cval + CAND_CAP + 4);
        if (tid < CAND_CAP) cval[tid] = -INFINITY;
        if (tid < 4) cval[CAND_CAP + tid] = -INFINITY;
        if (tid == 0) s.cnt = 0;
        __syncthreads();
        float mx = -INFINITY, over = 0.f;                  // over: sum of (v - th) over the collected values
        for (int i0 = 0; i0 < len; i0 += nt) {
            const int i = i0 + tid;
            const float v = i < len ? V[i] : -INFINITY;
            mx = fmaxf(mx, v);
            const bool in = i < len && v >= th && (!MERGE || idf(i) != 0x7fffffff);
            if (in) over += v - th;
            const unsigned long long bal = __ballot(in);
            if (bal) {
                const int lead = __ffsll((long long)bal) - 1;
                unsigned base = 0;
                if (lane == lead) base = atomicAdd(&s.cnt, (unsigned)__popcll(bal));
                base = __shfl(base, lead, CSV_WAVE);
                const unsigned slot = base + (unsigned)__popcll(bal & ((1ull << lane) - 1ull));
                if (in && slot < CAND_CAP) {
                    cval[slot] = v;
                    cid[slot] = LATE_IDS ? i : idf(i);
                }
            }
        }
        mx = wave_max(mx);
        over = wave_sum(over);
        if (lane == 0) {
            wmax[tid >> 6] = mx;
            wmax[16 + (tid >> 6)] = over;
        }
        __syncthreads();
        const int m = (int)s.cnt;
        if (m > CAND_CAP || (!short_ok && m < k0)) return false;
        vmax = wmax[0];
        for (int q = 1; q < (nt >> 6); ++q) vmax = fmaxf(vmax, wmax[q]);
        if (LATE_IDS) {
            if (tid < m) cid[tid] = idf(cid[tid]);
            __syncthreads();
        }
        kkv = min(k, m);
        if (m > RANK_BUCKETS_MIN && th > -INFINITY) {
            // the values thin out above the threshold: equal-width buckets up to eight times their mean excess hold a
            // few values each, whatever lies beyond (a handful of outstanding logits) shares the first bucket
            float tot = 0.f;
            for (int q = 0; q < (nt >> 6); ++q) tot += wmax[16 + q];
            rank_buckets(cval, cid, m, kkv, th, fminf(vmax, th + 8.f * tot / (float)m), s);
        } else {
            float v;
            rank_small(cval, cid, m, kkv, s, v);
        }
        return true;
    };
    bool ok = false;
    if (MERGE || theta > -INFINITY) ok = attempt(theta);
    if (!ok && k <= RANK_DIRECT && len > RANK_DIRECT) {
        // RANK_DIRECT group maxima (group g: the values i with i % RANK_DIRECT == g; len > RANK_DIRECT, so no group is
        // empty): k of them, hence k of the values, reach their k-th largest, and since the largest values mostly sit
        // in different groups few more do
        float* cval = reinterpret_cast<float*>(reinterpret_cast<char*>(arena) + CAND_OFF);
        float mx = -INFINITY;
        for (int i = tid; i < len; i += nt) mx = fmaxf(mx, V[i]);
        __syncthreads();
        if (tid < CAND_CAP) cval[tid] = mx;
        __syncthreads();
        float m2 = -INFINITY;
        if (tid < RANK_DIRECT) {
            m2 = cval[tid];
            for (int j = tid + RANK_DIRECT; j < min(nt, CAND_CAP); j += RANK_DIRECT) m2 = fmaxf(m2, cval[j]);
        }
        __syncthreads();
        if (tid < RANK_DIRECT) cval[tid] = m2;
        __syncthreads();
        float v;
        rank_small(cval, reinterpret_cast<const int*>(cval), RANK_DIRECT, k, s, v);      // only the k-th value is wanted: any ids do
        __syncthreads();
        const float th = fmaxf(s.wval[k - 1], theta);
        __syncthreads();
        ok = attempt(th);
    }
    return ok;
}

// ================================================================================================ certified distribution
// Optional outputs (Section III, top-p certification): over the returned list, in its order, the sub-vocabulary
// probabilities p~_t = exp(l_t - Z_S), their running sums, and the length of the shortest prefix whose running sum
// reaches top_p (0: not reached within the list).  kk entries of s.wval are valid; Z is the log-sum-exp that goes
// to d_lse.  Every thread of the block calls.  Each running sum is taken in list order by one thread.
__device__ __forceinline__ void write_distribution(const StepArgs& a, int b, int kk, float Z, SeqShared& s) {
    if (!a.out.d_probs && !a.out.d_cum && !a.out.d_nucleus) return;
    const int tid = threadIdx.x, nt = blockDim.x;
    int below = 0;
    for (int t = tid; t < a.k; t += nt) {
        float p = 0.f, cum = 0.f;
        const int last = min(t, kk - 1);
        for (int j = 0; j <= last; ++j) {
            const float pj = expf(s.wval[j] - Z);
            cum += pj;
            if (j == t) p = pj;
        }
        if (a.out.d_probs) a.out.d_probs[(size_t)b * a.k + t] = p;
        if (a.out.d_cum) a.out.d_cum[(size_t)b * a.k + t] = cum;
        below += (t < kk && cum < a.top_p) ? 1 : 0;
    }
    if (a.out.d_nucleus) {
        below = block_sum_i(below, s.redi);
        if (tid == 0) a.out.d_nucleus[b] = (a.top_p > 0.f && below < kk) ? below + 1 : 0;
    }
}

// ================================================================================================ certification
// One block per sequence.  round 0: certify, or plan round 1 (or fall back on budget); round 1: certify or fall back.
// Sequences with more than STAGE_CAP scored rows are handled by several blocks: each takes one chunk of STAGE_CAP
// logits, publishes the chunk's top-k candidates and log-sum-exp partial, and the block that arrives last (a
// device-scope counter; nobody waits) merges them and goes on to the tests.
// staged: the caller has already put the sequence's logits and ids where the staging below would put them
// Returns true when the sequence is finished (its outputs are written), false when work was queued for later phases
// (another round, the full vocabulary) or nothing was done.
// THRESH: compile the threshold selection for more than RANK_DIRECT values.  The fused step kernel leaves it out (its
// rare larger selections take the general path): with that code in the kernel a single-sequence step took 0.3 us
// longer, although the step never runs it.
template <bool THRESH>
__device__ __forceinline__ bool cert_body(const StepArgs& a, int b, int chunk, int round, const SeqState& st, SeqShared& s,
                                          bool staged = false, int* settled_count = nullptr) {
    extern __shared__ __align__(16) u64 arena[];
    const int tid = threadIdx.x, nt = blockDim.x, C = a.C;
    if (st.status != ST_ACTIVE || st.rounds != round) return false;
    const int n = st.n_rows;
    const int nchunks = (n + STAGE_CAP - 1) / STAGE_CAP;
    if (chunk >= nchunks) return false;
    const int c0 = chunk * STAGE_CAP, len = min(STAGE_CAP, n - c0);
    if (!staged) {
        const float* gv = a.slog + (size_t)b * a.K_cap + c0;
        const int32_t* gi = a.sid + (size_t)b * a.K_cap + c0;
        stage2_to_lds(reinterpret_cast<float*>(arena), gv, reinterpret_cast<int*>(arena) + STAGE_CAP, gi, len);
        if (tid < 4 && len + tid < STAGE_CAP) reinterpret_cast<float*>(arena)[len + tid] = -INFINITY;   // see the small path below
        __syncthreads();
    }
    // the accessors name the LDS array itself so that the reads compile to LDS instructions
    auto val = [](int i) { return reinterpret_cast<const float*>(arena)[i]; };
    auto idf = [](int i) { return reinterpret_cast<const int*>(arena)[STAGE_CAP + i]; };
    // with a top-k the largest logit is already known when the sum is taken: one block reduction instead of two
    LseAcc l;
    int kkv = min(a.k, len);                 // entries of the ordered list this chunk contributes
    bool have_topk = false;
    if (a.use_k && len <= RANK_DIRECT) {
        // few values: ordered top-k and log-sum-exp in one pass with two barriers
        float v;
        const float vmax = rank_small(reinterpret_cast<const float*>(arena), reinterpret_cast<const int*>(arena) + STAGE_CAP, len, kkv, s, v);
        float pe = (tid < len && vmax > -INFINITY) ? expf(v - vmax) : 0.f;
        pe = wave_sum(pe);
        float* wsum = reinterpret_cast<float*>(s.hist);
        if ((tid & 63) == 0) wsum[tid >> 6] = pe;
        __syncthreads();
        float tot = 0.f;
        for (int q = 0; q < (nt >> 6); ++q) tot += wsum[q];
        l.m = vmax;
        l.s = tot;
        have_topk = true;
    } else if (THRESH && a.use_k) {
        // more values: through a threshold (see threshold_topk); the log-sum-exp runs over all values
        float vmax;
        if (threshold_topk(len, a.k, st.theta, nchunks > 1, idf, s, kkv, vmax)) {
            float sm = 0.f;
            if (vmax > -INFINITY)
                for (int i = tid; i < len; i += nt) sm += expf(val(i) - vmax);
            l.m = vmax;
            l.s = block_sum(sm, s.redf);
            have_topk = true;
        }
    }
    if (have_topk) {
        // list and log-sum-exp are set
    } else if (a.use_k) {
        block_topk(len, a.k, val, idf, s);
        l.m = s.wval[0];
        float sm = 0.f;
        if (l.m > -INFINITY)
            for (int i = tid; i < len; i += nt) sm += expf(val(i) - l.m);
        l.s = block_sum(sm, s.redf);
    } else {
        l = block_lse(len, val, s);
    }
    if (nchunks > 1) {
        const size_t pb = (size_t)b * a.cand_chunks, pc = pb + chunk;
        const int kk = kkv;
        for (int t = tid; t < a.k; t += nt) {
            a.cand_val[pc * a.k + t] = t < kk ? s.wval[t] : -INFINITY;
            a.cand_id[pc * a.k + t] = t < kk ? s.wid[t] : 0x7fffffff;
        }
        if (tid == 0) {
            a.cand_max[pc] = l.m;
            a.cand_sum[pc] = l.s;
        }
        __threadfence();
        __syncthreads();
        if (tid == 0) s.sel = atomicAdd(&a.counters[CNT_CHUNKS + round * CSV_MAX_BATCH + b], 1) == nchunks - 1;
        __syncthreads();
        if (!s.sel) return false;
        __threadfence();
        float mx = -INFINITY;
        for (int i = tid; i < nchunks; i += nt) mx = fmaxf(mx, a.cand_max[pb + i]);
        mx = block_max(mx, s.redf);
        float sm = 0.f;
        for (int i = tid; i < nchunks; i += nt) sm += a.cand_sum[pb + i] * expf(a.cand_max[pb + i] - mx);
        l.m = mx;
        l.s = block_sum(sm, s.redf);
        if (a.use_k) {
            const float* cv = a.cand_val + pb * a.k;
            const int32_t* ci = a.cand_id + pb * a.k;
            const int nc = nchunks * a.k;
            if (nc <= STAGE_CAP) {
                __syncthreads();
                stage2_to_lds(reinterpret_cast<float*>(arena), cv, reinterpret_cast<int*>(arena) + STAGE_CAP, ci, nc);
                __syncthreads();
                bool merged = false;
                if (THRESH) {
                    int kq;
                    float vm;
                    merged = threshold_topk<true>(nc, a.k, st.theta, false, idf, s, kq, vm);
                    __syncthreads();
                }
                if (!merged) block_topk(nc, a.k, val, idf, s);
            } else {
                block_topk(nc, a.k, [&](int i) { return cv[i]; }, [&](int i) { return ci[i]; }, s);
            }
        }
    }
    const float Z = lse_value(l);
    float theta = -INFINITY;
    if (a.use_k) theta = s.wval[a.k - 1];
    const bool tk = (st.nxtU == -INFINITY) || (st.nxtU < theta);
    const bool sm = (st.T - Z <= a.lam) || (st.T == -INFINITY);
    bool ok;
    if (a.combine == CSV_COMBINE_ALL)
        ok = (tk || !a.use_k) && (sm || !a.use_s);
    else
        ok = (tk && a.use_k) || (sm && a.use_s);

    auto finish = [&](unsigned flags) {
        // the fused step kernel's parked blocks wait for this count: a finished sequence leaves nothing for them to
        // read, so they are told before the outputs are written rather than after
        if (settled_count && tid == 0) atomicAdd(settled_count, 1);
        for (int t = tid; t < a.k; t += nt) {
            a.out.d_ids[(size_t)b * a.k + t] = s.wid[t];
            a.out.d_logits[(size_t)b * a.k + t] = s.wval[t];
        }
        if (a.use_k) write_distribution(a, b, min(a.k, n), Z, s);
        if (a.out.d_sel_clusters)
            for (int j = tid; j < st.n_open; j += nt) a.out.d_sel_clusters[(size_t)b * C + j] = a.sel[(size_t)b * C + j];
        if (tid == 0) {
            a.out.d_lse[b] = Z;
            a.out.d_flags[b] = flags;
            a.out.d_n_rows[b] = n;
            a.out.d_n_clusters[b] = st.n_open;
            if (a.out.d_rounds) a.out.d_rounds[b] = round + 1;
            a.st[b].status = ST_DONE;
        }
    };
    if (ok) {
        finish(((tk && a.use_k) ? CSV_FLAG_TOPK_CERT : 0u) | ((sm && a.use_s) ? CSV_FLAG_SOFTMAX_CERT : 0u));
        return true;
    }
    if (round + 1 < a.max_rounds) {
        // ---- plan the next round: the open set grows from {key >= kappa0} to {key >= kappa1}
        __syncthreads();                                   // the staged logits are dead; the arena is reused
        const ClusterLds L = carve_clusters(arena, a.Npad, C);
        const u64 kappa0 = st.kappa;
        u64 kappa_a = kappa0, kappa_s = kappa0;
        if (a.use_k && !tk) kappa_a = (u64)lkey(theta) << 32;                 // every cluster with U_c >= theta
        bool intact = false;                               // the by-cluster data is in LDS
        if (a.use_s && !sm) {
            load_clusters(a, b, L);
            __syncthreads();
            bool hopeless = false;
            if (a.use_k && !tk && a.combine == CSV_COMBINE_ALL && a.delta_clusters == 0) {
                // when the top-k threshold alone opens more rows than allowed, the joint plan (a superset) does too:
                // the sorted prefix search for the softmax threshold would change nothing
                int r2 = 0;
                for (int c = tid; c < C; c += nt) {
                    const u64 kx = L.keys[c];
                    if (kx >= kappa_a && kx < kappa0 && kx != 0) r2 += L.offl[c + 1] - L.offl[c];
                }
                hopeless = n + block_sum_i(r2, s.redi) > a.K_max;
            }
            if (!hopeless) kappa_s = softmax_prefix_key(a, L, kappa0, Z, s);
            intact = true;
        }
        u64 kappa1;
        if (a.use_k && a.use_s)
            kappa1 = a.combine == CSV_COMBINE_ALL ? (kappa_a < kappa_s ? kappa_a : kappa_s) : (kappa_a > kappa_s ? kappa_a : kappa_s);
        else
            kappa1 = a.use_k ? kappa_a : kappa_s;
        if (!intact) {
            load_clusters(a, b, L);
            __syncthreads();
        }
        int cnt = 0, rows = 0;
        for (int c = tid; c < C; c += nt) {
            const u64 kx = L.keys[c];
            if (kx >= kappa1 && kx < kappa0 && kx != 0) {
                cnt += 1;
                rows += L.offl[c + 1] - L.offl[c];
            }
        }
        cnt = block_sum_i(cnt, s.redi);
        rows = block_sum_i(rows, s.redi);
        bool expand = n + rows <= a.K_max;
        if (!expand) {
            if (tid == 0) {          // sizes of the plan that did not fit (reported if the sequence falls back)
                a.st[b].n_open = st.n_open + cnt;
                a.st[b].n_rows = n + rows;
            }
            // partial expansion: the next clusters of the bound order, at most delta_clusters of them, not past
            // the planned set, while the rows stay within the budget
            u64 kp = kappa0;
            int add = 0, radd = 0;
            for (int i = 0; i < a.delta_clusters; ++i) {
                u64 best = 0;
                for (int c = tid; c < C; c += nt) {
                    const u64 kx = L.keys[c];
                    if (kx < kp && kx > best) best = kx;
                }
                best = block_max_u64(best, s.redu);
                if (best == 0 || best < kappa1) break;
                const int cw = (int)(0xFFFFFFFFu - (uint32_t)best);
                const int nr = L.offl[cw + 1] - L.offl[cw];
                if (n + radd + nr > a.K_max) break;
                kp = best;
                add += 1;
                radd += nr;
            }
            if (add > 0) {
                kappa1 = kp;
                cnt = add;
                rows = radd;
                expand = true;
            }
        }
        if (expand) {
            auto isnew = [&](int c) { const u64 kx = L.keys[c]; return kx >= kappa1 && kx < kappa0 && kx != 0; };
            float nxtU, T1;
            tail_stats(a, L, kappa1, s, nxtU, T1);
            emit_clusters(a, b, round + 1, n, st.n_open, isnew, L, s);
            if (tid == 0) {
                SeqState o = st;
                o.n_open = st.n_open + cnt; o.n_rows = n + rows; o.rounds = round + 1; o.kappa = kappa1; o.nxtU = nxtU; o.T = T1;
                o.theta = (a.use_k && n >= a.k) ? theta : -INFINITY;
                a.st[b] = o;
            }
            return false;
        }
    }
    // ---- no further expansion: the relaxed tolerance, then the full vocabulary
    if (a.relax && a.use_s) {
        const bool sm2 = (st.T - Z <= a.lam2) || (st.T == -INFINITY);
        const bool ok2 = a.combine == CSV_COMBINE_ALL ? ((tk || !a.use_k) && sm2) : ((tk && a.use_k) || sm2);
        if (ok2) {
            finish(((tk && a.use_k) ? CSV_FLAG_TOPK_CERT : 0u) | (sm ? CSV_FLAG_SOFTMAX_CERT : (sm2 ? CSV_FLAG_SOFTMAX_RELAXED : 0u)));
            return true;
        }
    }
    if (tid == 0) push_fallback(a, b, round + 1);
    return false;
}

template <bool THRESH>
__device__ __forceinline__ void cert_device(const StepArgs& a, int b, int chunk, int round, SeqShared& s) {
    const SeqState st = a.st[b];
    cert_body<THRESH>(a, b, chunk, round, st, s);
}

// ================================================================================================ round 0
// Grid (NB, B): the NB blocks of a sequence each derive the same seed prefix from the sequence's bounds (the
// prefix is a handful of clusters found by repeated block-wide arg-max over the keys, no sort), so no block
// waits for another to plan the work; they share the prefix rows wave by wave, and the block that arrives last at
// the sequence's counter (nobody waits) certifies, or plans round 1, or hands the sequence to the full product.
// A prefix with more rows than the NB blocks should score themselves (one giant cluster) goes to the round-0
// work list instead and is scored and certified by the tail kernel with the whole device.
#define ROUND0_ROWS_PER_BLOCK 4     // rows of the largest possible seed prefix per block (2..8 swept: 3-4 fastest; 8 costs 1 us)
#define ROUND0_NB_MAX 64           // most blocks of a sequence in the round-0 kernel (8..128 swept: 32-64 fastest)
#define ROUND0_ROWS_PER_WAVE 8     // with at most 32 blocks of 8 waves a sequence: no more than 2048 <= STAGE_CAP rows;
                                   // with a single block: 64 rows, larger prefixes go to the tail kernel
#define ROUND0_HREG 4     // 128-bit pieces of h a thread carries in registers across the seed (d <= 4 * 8 * SEQ_THREADS)
// log tail mass of the clusters below the threshold key kappa, shifted by an upper bound of its largest term
// (nxt: the largest unopened key, 0 if none; nxtU: its bound)
__device__ __forceinline__ float seed_tail_mass(const StepArgs& a, const ClusterLds& L, u64 kappa, u64 nxt, float nxtU, SeqShared& s) {
    if (!nxt) return -INFINITY;
    const float shift = a.ln_nmax + nxtU;
    float sum = 0.f;
    for (int c = threadIdx.x; c < a.C; c += blockDim.x) {
        const u64 kx = L.keys[c];
        if (kx != 0 && kx < kappa) sum += expf(L.vl[c] - shift);
    }
    sum = block_sum(sum, s.redf);
    return shift + logf(sum);
}
__device__ __forceinline__ SeqState seed_state(int m0, int rows, u64 kappa, float nxtU, float T0) {
    SeqState st;
    st.status = ST_ACTIVE; st.n_open = m0; st.n_rows = rows; st.rounds = 0; st.kappa = kappa; st.nxtU = nxtU; st.T = T0;
    st.fb_slot = -1; st.theta = -INFINITY; st.pad[0] = st.pad[1] = 0;
    return st;
}

// Seed selection for indexes of at most 64 * SEED_E clusters.  The block stages the sequence's bounds and ln n_c
// in LDS once (one barrier, shared with the staging of h); after that every wave works alone: lane l looks at
// clusters l, l + 64, ..., the wave takes the arg-max of the 64-bit keys and fetches the winner's packed metadata.
// Every wave of every block of the sequence gets the same answer.  When the best cluster alone holds max(k,1) rows
// (the common case: clusters larger than k) it is the whole seed prefix; the wave requests its row and only then
// takes, from the same registers, the next bound and the log tail mass of everything else, while the row is in
// flight.  Otherwise the caller falls through to the general selection.
#define SEED_E 16
struct WaveSeed {
    int c, row0, rows;
    u64 kappa;
    float u[SEED_E], l[SEED_E];     // bounds and ln n of the lane's clusters (-inf: empty or out of range)
};
// sU, sL, sR: LDS copies of U[b,:], of ln n_c and of {first row, rows} per cluster.  All LDS reads are issued from
// clamped indexes before anything is compared (a conditional read would put every read in a basic block of its own,
// one LDS round trip after the other).
__device__ __forceinline__ void wave_seed_pick(const StepArgs& a, const float* sU, const float* sL, const int2* sR, WaveSeed& r) {
    const int lane = threadIdx.x & 63, C = a.C;
#pragma unroll
    for (int i = 0; i < SEED_E; ++i) {
        const int cc = min(lane + 64 * i, C - 1);
        r.u[i] = sU[cc];
        r.l[i] = sL[cc];
    }
    // 32-bit keys: the largest bound first, then the smallest cluster id among its holders (the order of the 64-bit keys)
    unsigned bk = 0;
    int bc = 0x7fffffff;
#pragma unroll
    for (int i = 0; i < SEED_E; ++i) {
        const int c = lane + 64 * i;
        const bool some = c < C && r.l[i] > -INFINITY;
        r.u[i] = some ? r.u[i] : -INFINITY;
        r.l[i] = some ? r.l[i] : -INFINITY;
        const unsigned kx = some ? lkey(r.u[i]) : 0u;      // lkey is never 0 for a bound that is not NaN
        const bool better = kx > bk;                       // c grows with i: a tie keeps the smaller id
        bk = better ? kx : bk;
        bc = better ? c : bc;
    }
    const unsigned top = wave_max_u(bk);
    const int cw = wave_min_i((bk == top && top != 0u) ? bc : 0x7fffffff);
    r.kappa = 0;
    r.c = 0;
    r.row0 = 0;
    r.rows = 0;
    if (top != 0u) {
        const int2 rr = sR[cw];
        r.c = cw;
        r.row0 = rr.x;
        r.rows = rr.y;
        r.kappa = ((u64)top << 32) | (u64)(0xFFFFFFFFu - (uint32_t)cw);
    }
}
// next bound and log tail mass with cluster r.c open and everything else unopened
__device__ __forceinline__ void wave_seed_tail(const StepArgs& a, const WaveSeed& r, float& nxtU, float& T0) {
    const int lane = threadIdx.x & 63;
    float mx = -INFINITY;
    float v[SEED_E];
#pragma unroll
    for (int i = 0; i < SEED_E; ++i) {
        const bool rest = (lane + 64 * i) != r.c;          // empty and out-of-range clusters already carry -inf
        v[i] = rest ? r.l[i] + r.u[i] : -INFINITY;
        mx = fmaxf(mx, rest ? r.u[i] : -INFINITY);
    }
    mx = wave_max(mx + 0.0f);
    nxtU = mx;
    T0 = -INFINITY;
    if (mx == -INFINITY) return;                              // the prefix is the whole vocabulary
    const float shift = a.ln_nmax + nxtU;
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < SEED_E; ++i) sum += expf(v[i] - shift);     // exp(-inf) = 0
    sum = wave_sum(sum);
    T0 = shift + logf(sum);
}

// One sequence's round 0 as seen by block j of its NB blocks.  Returns nonzero in the one block that settled the
// sequence: 1 when the sequence is finished (certified, or flagged invalid), 2 when it left work for later phases
// (a planned round, a hand-over, a fallback) or gave up.
// settled_count: where a sequence that finishes here is counted as soon as that is decided (the return value is then 3).
__device__ __forceinline__ int round0_device(const StepArgs& a, int b, int j, int NB, SeqShared& s, int* settled_count = nullptr) {
    extern __shared__ __align__(16) u64 arena[];
    const int tid = threadIdx.x, nt = SEQ_THREADS, lane = tid & 63, wave = tid >> 6, C = a.C;
    const int nch = a.d >> 3;
    const ClusterLds L = carve_clusters(arena, a.Npad, C);
    // h is requested now and parked in registers: it moves to LDS once the cluster data there is dead
    uint4 hreg[ROUND0_HREG];
    {
        const uint4* hsrc = reinterpret_cast<const uint4*>(a.h) + (size_t)b * nch;
#pragma unroll
        for (int q = 0; q < ROUND0_HREG; ++q) {
            const int i = tid + q * nt;
            hreg[q] = i < nch ? hsrc[i] : make_uint4(0, 0, 0, 0);
        }
    }
    const float hn = a.hnorm[b];
    if (j == 0 && tid == 0) a.out.d_flags[b] = CSV_FLAG_ABORTED;   // pending: overwritten by whichever path finishes the sequence
    const int need = max(a.k, 1);
    const int GW = NB * (nt >> 6);
    const int cap_rows = min(GW * ROUND0_ROWS_PER_WAVE, STAGE_CAP);
    int* scl = s.wid;
    int* spos = reinterpret_cast<int*>(s.wval);
    int rows = 0, m0 = 0;
    u64 kappa = ~0ull, nxt = 0;
    float nxtU, T0;
    uint4* hs4 = reinterpret_cast<uint4*>(arena) + a.r0_h_off;
    u64* slots = a.slots + (size_t)b * CSV_SLOT_ROWS;
    uint4 pf[TILE_PF];
    const uint4* w = nullptr;
    float bias = 0.f;
    int id = 0;
    auto request_row = [&](int r) {       // unconditional loads from clamped addresses, then a select: no branches
        w = reinterpret_cast<const uint4*>(a.Wp + (size_t)r * a.d);
#pragma unroll
        for (int q = 0; q < TILE_PF; ++q) {
            const int i = lane + 64 * q;
            const uint4 v = w[min(i, nch - 1)];
            pf[q] = i < nch ? v : make_uint4(0, 0, 0, 0);
        }
        bias = a.bp[r];                   // every lane the same address: one transaction
        id = a.perm[r];
    };
    int p = wave * NB + j;   // neighbouring rows go to different compute units
    bool fast = false;
    WaveSeed ws;
    ws.row0 = 0;
    if (C <= 64 * SEED_E && nch <= ROUND0_HREG * nt) {
        // bounds, ln n and h to LDS with one barrier; then every wave picks the seed cluster by itself
        float* sU = reinterpret_cast<float*>(arena);
        float* sL = sU + C;
        int2* sR = reinterpret_cast<int2*>(sL + C + (C & 1));
        {
            const float* Ub = a.U + (size_t)b * C;
            float ru[2];
            int4 rm[2];
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int cc = min(tid + q * nt, C - 1);
                ru[q] = Ub[cc];
                rm[q] = a.cmeta[cc];
            }
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int c = tid + q * nt;
                if (c < C) {
                    sU[c] = ru[q];
                    sL[c] = __int_as_float(rm[q].z);
                    sR[c] = make_int2(rm[q].x, rm[q].y);
                }
            }
#pragma unroll
            for (int q = 0; q < ROUND0_HREG; ++q) {
                const int i = tid + q * nt;
                if (i < nch) hs4[i] = hreg[q];
            }
        }
        __syncthreads();
        if (!isfinite(hn)) {
            if (j == 0) write_invalid(a, b);
            return j == 0 ? 1 : 0;
        }
        wave_seed_pick(a, sU, sL, sR, ws);
        fast = ws.kappa != 0 && ws.rows >= need && ws.rows <= cap_rows && ws.rows <= a.K_max;
        if (!fast) __syncthreads();          // every wave has read the staged bounds: the general path reuses the LDS
    }
    if (fast) {
        // the prefix is one cluster: the row first, then the next bound and the tail mass while it is in flight
        m0 = 1; rows = ws.rows; kappa = ws.kappa;
        if (p < rows) request_row(ws.row0 + p);
        if (j == 0 && tid == 0) a.sel[(size_t)b * C] = ws.c;
        nxtU = -INFINITY;        // the next bound and the tail mass are needed by the certifying block only: taken after its rows
        T0 = -INFINITY;
    } else {
        load_clusters(a, b, L);
        if (!isfinite(hn)) {
            if (j == 0) write_invalid(a, b);
            return j == 0 ? 1 : 0;
        }
        __syncthreads();
        // Open clusters one at a time by block-wide arg-max until max(k,1) rows are open.  Every opened cluster has
        // at least one row, so at most max(k,1) <= CSV_MAX_K clusters open: their ids and positions fit the k-sized
        // arrays.  Nothing is written to global memory inside the loop (a store would be waited for at the next barrier).
        while (true) {
            // the best unopened cluster and the one after it, in one reduction: when the best completes the prefix,
            // the runner-up is already the next unopened bound
            Top2 t2{0ull, 0ull};
            for (int c = tid; c < C; c += nt) {
                const u64 kx = L.keys[c];
                if (kx < kappa) t2 = top2_push(t2, kx);
            }
            t2 = block_top2(t2, s.redu);
            if (t2.a == 0) {                   // nothing left to open
                nxt = 0;
                break;
            }
            const int cw = (int)(0xFFFFFFFFu - (uint32_t)t2.a);
            if (tid == 0) {
                scl[m0] = cw;
                spos[m0] = rows;
            }
            rows += L.offl[cw + 1] - L.offl[cw];
            m0 += 1;
            kappa = t2.a;
            if (rows >= need) {
                nxt = t2.b;
                break;
            }
        }
        if (rows > a.K_max) {
            if (j == 0 && tid == 0) {
                a.st[b].n_open = m0;
                a.st[b].n_rows = rows;
                push_fallback(a, b, 0);
            }
            return j == 0 ? 2 : 0;
        }
        __syncthreads();   // scl / spos complete
        if (j == 0)
            for (int i = tid; i < m0; i += nt) a.sel[(size_t)b * C + i] = scl[i];
        nxtU = nxt ? ckey_bound(nxt) : -INFINITY;
        if (rows > cap_rows || nch > ROUND0_HREG * nt) {
            // too much for these blocks: the first block queues the prefix for the tail
            if (j != 0) return 0;
            T0 = seed_tail_mass(a, L, kappa, nxt, nxtU, s);
            Tile* tl = a.tiles[0] + (size_t)b * a.tile_stride;
            int ntile = 0;
            for (int i = 0; i < m0; ++i) {
                const int r0 = L.offl[scl[i]], p0 = spos[i], n = (i + 1 < m0 ? spos[i + 1] : rows) - p0;
                const int ntc = (n + TILE_ROWS - 1) / TILE_ROWS;
                for (int t = tid; t < ntc; t += nt) {
                    Tile x;
                    x.b = b; x.row0 = r0 + t * TILE_ROWS; x.nrows = min(TILE_ROWS, n - t * TILE_ROWS); x.pos = p0 + t * TILE_ROWS;
                    tl[ntile + t] = x;
                }
                ntile += ntc;
            }
            if (tid == 0) {
                a.counters[CNT_TILES + b] = ntile;
                __hip_atomic_store(&a.counters[CNT_TAIL_NEEDED], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                a.st[b] = seed_state(m0, rows, kappa, nxtU, T0);
            }
            return 2;
        }
        // h goes to its own LDS region behind the cluster data; the wave's first row is requested before the tail
        // mass is summed, so that sum runs while the loads are in flight
#pragma unroll
        for (int q = 0; q < ROUND0_HREG; ++q) {
            const int i = tid + q * nt;
            if (i < nch) hs4[i] = hreg[q];
        }
    }
    auto row_of = [&](int pp) {
        if (fast) return ws.row0 + pp;
        int lo = 0, hi = m0;   // largest i with spos[i] <= pp
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (spos[mid] <= pp) lo = mid; else hi = mid;
        }
        return L.offl[scl[lo]] + (pp - spos[lo]);
    };
    if (!fast) {
        if (p < rows) request_row(row_of(p));
        __syncthreads();                   // h staged (the fast path staged it before its barrier)
    }
    while (p < rows) {
        float acc = 0.f, acc2 = 0.f;          // two chains: a dependent FMA costs two issue slots of a lone wave
#pragma unroll
        for (int q = 0; q < TILE_PF; q += 2) {     // pieces past the row are zero and h is finite: no branch needed
            const int i = lane + 64 * q;
            acc = dot8_bf16(pf[q], hs4[min(i, nch - 1)], acc);
            acc2 = dot8_bf16(pf[q + 1], hs4[min(i + 64, nch - 1)], acc2);
        }
        acc += acc2;
        int i = lane + 64 * TILE_PF;
        for (; i + 192 < nch; i += 256) {
            const uint4 x0 = w[i], x1 = w[i + 64], x2 = w[i + 128], x3 = w[i + 192];
            acc = dot8_bf16(x0, hs4[i], acc);
            acc = dot8_bf16(x1, hs4[i + 64], acc);
            acc = dot8_bf16(x2, hs4[i + 128], acc);
            acc = dot8_bf16(x3, hs4[i + 192], acc);
        }
        for (; i < nch; i += 64) acc = dot8_bf16(w[i], hs4[i], acc);
        acc = wave_sum(acc);
        if (lane == 0)      // one word carries the row's token id and logit: whoever reads it gets both or neither
            __hip_atomic_store(&slots[p], ((u64)(uint32_t)id << 32) | (u64)__float_as_uint(acc + bias), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        p += GW;
        if (p < rows) request_row(row_of(p));
    }
    // Block 0 of the sequence collects: each of its threads waits for its rows' words (no counter, no fence: a word
    // is either still empty or complete), puts the logit and the id where the certification expects its staged
    // input, copies them to the row arrays that later rounds read, and empties the word for the next step.  All NB
    // blocks of a sequence are resident together (the host sizes the grid so), and the wait is bounded.
    if (j != 0) return 0;
    // the tail mass, which only this block needs, while the other blocks' words are on their way (the cluster data
    // in LDS is still whole: h sits behind it)
    if (fast) wave_seed_tail(a, ws, nxtU, T0);
    else T0 = seed_tail_mass(a, L, kappa, nxt, nxtU, s);
    const SeqState st = seed_state(m0, rows, kappa, nxtU, T0);
    __syncthreads();                       // every wave is done with h in LDS: the staging area overlaps it
    float* sv = reinterpret_cast<float*>(arena);
    int* si = reinterpret_cast<int*>(arena) + STAGE_CAP;
    int gave_up = 0;
    for (int t = tid; t < rows; t += nt) {
        u64 v;
        int spins = 0;
        while ((v = __hip_atomic_load(&slots[t], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) == CSV_SLOT_EMPTY) {
            if (++spins > a.spin_limit) {
                gave_up = 1;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        if (gave_up) break;
        __hip_atomic_store(&slots[t], CSV_SLOT_EMPTY, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float lv = __uint_as_float((uint32_t)v);
        const int iv = (int)(uint32_t)(v >> 32);
        sv[t] = lv;
        si[t] = iv;
        a.slog[(size_t)b * a.K_cap + t] = lv;
        a.sid[(size_t)b * a.K_cap + t] = iv;
    }
    if (tid < 4 && rows + tid < STAGE_CAP) sv[rows + tid] = -INFINITY;     // the certification reads the values four at a time
    if (__syncthreads_or(gave_up)) {
        // a row never arrived: the step is given up for this sequence (flag ABORTED stays); words may still arrive
        // later, so the next step has to empty the slots before it uses them
        if (tid == 0) {
            atomicExch(&a.counters[CNT_ABORT], 1);
            __hip_atomic_store(&a.counters[CNT_SLOTS_DIRTY], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        return 2;
    }
    return cert_body<false>(a, b, 0, 0, st, s, true, settled_count) ? (settled_count ? 3 : 1) : 2;     // every path of it that leaves work behind writes the state it needs
}

// ================================================================================================ Algorithm 1's own order
// One cluster per iteration, the tests after every opening: the shortest certifying prefix of the bound order
// (Algorithm 1, Section III-C).  A reference mode, not the fast path: one block per sequence does everything itself, so
// an iteration is a block-wide arg-max, the rows of one cluster (a row per wave at a time) and a top-k update, with
// no dependency between blocks.  Dynamic LDS: staged values and ids with the candidates behind them (as the
// certification lays them out), then the sequence's cluster data, then h.
#define ALG1_PIECE 2048            // rows of a cluster scored between two updates of the list (a piece plus the list fit the staging area)
#define ALG1_CL_OFF (CAND_OFF + CAND_BYTES + 16)      // bytes; a multiple of 16
static_assert(ALG1_PIECE + CSV_MAX_K <= STAGE_CAP && ALG1_CL_OFF % 16 == 0, "Algorithm-1 mode: staging layout");
__global__ __launch_bounds__(SEQ_THREADS) void alg1_kernel(StepArgs a, int h_off16) {
    extern __shared__ __align__(16) u64 arena[];
    __shared__ SeqShared s;
    const int b = blockIdx.x, tid = threadIdx.x, nt = SEQ_THREADS, lane = tid & 63, wave = tid >> 6, C = a.C;
    const int nch = a.d >> 3;
    float* sv = reinterpret_cast<float*>(arena);
    int* si = reinterpret_cast<int*>(arena) + STAGE_CAP;
    const ClusterLds L = carve_clusters(reinterpret_cast<u64*>(reinterpret_cast<char*>(arena) + ALG1_CL_OFF), a.Npad, C);
    uint4* hs4 = reinterpret_cast<uint4*>(arena) + h_off16;
    auto val = [](int i) { return reinterpret_cast<const float*>(arena)[i]; };
    auto idf = [](int i) { return reinterpret_cast<const int*>(arena)[STAGE_CAP + i]; };
    const float hn = a.hnorm[b];
    if (!isfinite(hn)) {
        write_invalid(a, b);
        return;
    }
    load_clusters(a, b, L);
    for (int i = tid; i < nch; i += nt) hs4[i] = (reinterpret_cast<const uint4*>(a.h) + (size_t)b * nch)[i];
    __syncthreads();
    u64 kappa = ~0ull;
    int rows = 0, m = 0, kcur = 0;         // rows scored, clusters open, entries of the list in s.wval / s.wid
    LseAcc run;
    run.m = -INFINITY;
    run.s = 0.f;
    while (true) {
        // ---- both tests on the open prefix (m = 0: nothing scored, only "no cluster at all" certifies)
        float nxtU, T;
        tail_stats(a, L, kappa, s, nxtU, T);
        __syncthreads();
        const float Z = lse_value(run);
        const float theta = (a.use_k && kcur >= a.k) ? s.wval[a.k - 1] : -INFINITY;
        const bool none_left = nxtU == -INFINITY;
        const bool tk = none_left || (kcur >= a.k && nxtU < theta);
        const bool sm = none_left || (rows > 0 && T - Z <= a.lam);
        const bool tk_ok = a.use_k ? tk : (a.combine == CSV_COMBINE_ALL);
        const bool sm_ok = a.use_s ? sm : (a.combine == CSV_COMBINE_ALL);
        const bool ok = a.combine == CSV_COMBINE_ALL ? (tk_ok && sm_ok) : (tk_ok || sm_ok);
        if (ok) {
            for (int t = tid; t < a.k; t += nt) {
                a.out.d_ids[(size_t)b * a.k + t] = t < kcur ? s.wid[t] : -1;
                a.out.d_logits[(size_t)b * a.k + t] = t < kcur ? s.wval[t] : -INFINITY;
            }
            if (a.use_k) write_distribution(a, b, kcur, Z, s);
            if (tid == 0) {
                a.out.d_lse[b] = Z;
                a.out.d_flags[b] = ((tk && a.use_k) ? CSV_FLAG_TOPK_CERT : 0u) | ((sm && a.use_s) ? CSV_FLAG_SOFTMAX_CERT : 0u);
                a.out.d_n_rows[b] = rows;
                a.out.d_n_clusters[b] = m;
                if (a.out.d_rounds) a.out.d_rounds[b] = m;
                a.st[b].status = ST_DONE;
            }
            if (a.out.d_sel_clusters)
                for (int j = tid; j < m; j += nt)       // written by thread 0 of this block: read past the first-level cache
                    a.out.d_sel_clusters[(size_t)b * C + j] = __hip_atomic_load(&a.sel[(size_t)b * C + j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        // ---- open the next cluster of the bound order; the budget is tested before its rows are scored
        u64 best = 0;
        for (int c = tid; c < C; c += nt) {
            const u64 kx = L.keys[c];
            if (kx < kappa && kx > best) best = kx;
        }
        best = block_max_u64(best, s.redu);
        const int cw = (int)(0xFFFFFFFFu - (uint32_t)best);       // best != 0: some cluster is unopened, or the tests had held
        const int r0 = L.offl[cw], nc = L.offl[cw + 1] - r0;
        if (rows + nc > a.K_max) {
            if (tid == 0) {
                a.st[b].n_open = m + 1;
                a.st[b].n_rows = rows + nc;
                push_fallback(a, b, m + 1);
            }
            return;
        }
        if (tid == 0) a.sel[(size_t)b * C + m] = cw;
        kappa = best;
        m += 1;
        for (int p0 = 0; p0 < nc; p0 += ALG1_PIECE) {
            const int P = min(ALG1_PIECE, nc - p0);
            __syncthreads();                                  // the staging area is free
            // two rows per wave at a time, a whole row (up to TILE_PF pieces per lane) requested before anything is added up
            for (int p = 2 * wave; p < P; p += 2 * (nt >> 6)) {
                uint4 pf[2][TILE_PF];
                const uint4* w[2];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    w[q] = reinterpret_cast<const uint4*>(a.Wp + (size_t)(r0 + p0 + min(p + q, P - 1)) * a.d);
#pragma unroll
                    for (int j = 0; j < TILE_PF; ++j) pf[q][j] = w[q][min(lane + 64 * j, nch - 1)];
                }
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    float acc = 0.f;
#pragma unroll
                    for (int j = 0; j < TILE_PF; ++j) {
                        const int i = lane + 64 * j;
                        if (i < nch) acc = dot8_bf16(pf[q][j], hs4[i], acc);
                    }
                    for (int i = lane + 64 * TILE_PF; i < nch; i += 64) acc = dot8_bf16(w[q][i], hs4[i], acc);
                    acc = wave_sum(acc);
                    if (lane == 0 && p + q < P) {
                        const int r = r0 + p0 + p + q;
                        sv[p + q] = acc + a.bp[r];
                        si[p + q] = a.perm[r];
                    }
                }
            }
            __syncthreads();
            // log-sum-exp of the piece joins the running one; the list joins the piece and the top k of both is the new list
            const LseAcc lp = block_lse(P, val, s);
            run = lse_combine(run, lp);
            __syncthreads();
            for (int t = tid; t < kcur; t += nt) {
                sv[P + t] = s.wval[t];
                si[P + t] = s.wid[t];
            }
            const int ntot = P + kcur;
            if (tid < 4 && ntot + tid < STAGE_CAP) sv[ntot + tid] = -INFINITY;
            __syncthreads();
            if (a.use_k) {
                const int knew = min(a.k, ntot);
                bool done = false;
                if (ntot <= RANK_DIRECT) {
                    float v;
                    rank_small(sv, si, ntot, knew, s, v);
                    done = true;
                } else {
                    int kk = 0;
                    float vmax;
                    done = threshold_topk(ntot, a.k, kcur >= a.k ? s.wval[a.k - 1] : -INFINITY, false, idf, s, kk, vmax);
                }
                __syncthreads();
                if (!done) block_topk(ntot, a.k, val, idf, s);
                kcur = knew;
            }
            rows += P;
        }
        __syncthreads();
    }
}

// ================================================================================================ full-vocabulary product
struct FullArgs {
    int V, d;
    const uint16_t* Wp;
    const float* bp;
    const int32_t* perm;
    const uint16_t* h;
    const int32_t* list;    // sequences to score
    const int32_t* n_ptr;   // device count of entries in list, or NULL
    int n_fixed;            // count when n_ptr is NULL
    float* out;             // [slot*out_stride + row]
    long long out_stride;
    int scatter;            // 1: write at the original token id instead of the permuted row
};

// Vector path: FULL_G sequences per pass over W', h of the pass in LDS, two rows per wave at a time.
__device__ __forceinline__ void full_gemv_device(const FullArgs& f, int n, uint4* hs4, int block, int nblocks) {
    const int tid = threadIdx.x, nt = blockDim.x, lane = tid & 63, wave = tid >> 6;
    const int nch = f.d >> 3;
    const int rpt = (nt >> 6) * 2;                 // rows per tile: two per wave
    const int ntiles = (f.V + rpt - 1) / rpt;
    for (int g0 = 0; g0 < n; g0 += FULL_G) {
        const int ng = min(FULL_G, n - g0);
        __syncthreads();
        for (int i = tid; i < FULL_G * nch; i += nt) {
            const int s = i / nch, j = i - s * nch;
            hs4[i] = s < ng ? (reinterpret_cast<const uint4*>(f.h) + (size_t)f.list[g0 + s] * nch)[j] : make_uint4(0, 0, 0, 0);
        }
        __syncthreads();
        for (int tile = block; tile < ntiles; tile += nblocks) {
            const int r0 = tile * rpt + wave * 2;
            if (r0 >= f.V) continue;
            const bool two = r0 + 1 < f.V;
            const int r1 = two ? r0 + 1 : r0;
            const uint4* w0 = reinterpret_cast<const uint4*>(f.Wp + (size_t)r0 * f.d);
            const uint4* w1 = reinterpret_cast<const uint4*>(f.Wp + (size_t)r1 * f.d);
            float acc0[FULL_G], acc1[FULL_G];
#pragma unroll
            for (int s = 0; s < FULL_G; ++s) acc0[s] = acc1[s] = 0.f;
            int i = lane;
            for (; i + 64 < nch; i += 128) {
                const uint4 a0 = w0[i], a1 = w0[i + 64];
                const uint4 c0 = w1[i], c1 = w1[i + 64];
#pragma unroll
                for (int s = 0; s < FULL_G; ++s) {
                    if (s < ng) {
                        const uint4 h0 = hs4[s * nch + i], h1 = hs4[s * nch + i + 64];
                        acc0[s] = dot8_bf16(a0, h0, acc0[s]);
                        acc1[s] = dot8_bf16(c0, h0, acc1[s]);
                        acc0[s] = dot8_bf16(a1, h1, acc0[s]);
                        acc1[s] = dot8_bf16(c1, h1, acc1[s]);
                    }
                }
            }
            for (; i < nch; i += 64) {
                const uint4 a0 = w0[i], c0 = w1[i];
#pragma unroll
                for (int s = 0; s < FULL_G; ++s) {
                    if (s < ng) {
                        const uint4 h0 = hs4[s * nch + i];
                        acc0[s] = dot8_bf16(a0, h0, acc0[s]);
                        acc1[s] = dot8_bf16(c0, h0, acc1[s]);
                    }
                }
            }
#pragma unroll
            for (int s = 0; s < FULL_G; ++s) {
                if (s < ng) {
                    const float v0 = wave_sum(acc0[s]), v1 = wave_sum(acc1[s]);
                    if (lane == 0) {
                        float* dst = f.out + (size_t)(g0 + s) * f.out_stride;
                        dst[f.scatter ? f.perm[r0] : r0] = v0 + f.bp[r0];
                        if (two) dst[f.scatter ? f.perm[r1] : r1] = v1 + f.bp[r1];
                    }
                }
            }
        }
    }
}

__global__ __launch_bounds__(256) void full_gemv_kernel(FullArgs f) {
    extern __shared__ uint4 hs4[];
    const int n = f.n_ptr ? *f.n_ptr : f.n_fixed;
    if (n <= 0) return;
    full_gemv_device(f, n, hs4, blockIdx.x, gridDim.x);
}

// MFMA path of the full-vocabulary product, used when more than FULL_G sequences share the pass over W' (then it
// is a real dense contraction: [V x d] . [d x n]).  v_mfma_f32_16x16x32_bf16.  A block of eight waves owns
// 128 TW consecutive rows of W' at a time, a wave 16 TW of them (TW row tiles) for 16 NT sequences, and keeps the
// logits of its tiles in accumulator registers over the whole of K: every logit is written once.
//   h  (shared by all waves) moves through LDS in chunks of one to four K blocks of 128, already in fragment order
//      (the 64 lanes of a fragment read 1 KB contiguously: no bank conflicts), double-buffered: while a chunk is
//      consumed the next one is fetched into registers and stored to the other buffer; one barrier per chunk, which
//      waits for LDS traffic only, so the W' loads in flight cross it.  A fragment read from LDS serves TW MFMAs.
//   W' goes straight from global memory to registers: lane (li = lane%16, g = lane/16) feeds row li of a tile and, for
//      the jj-th MFMA of a K block, the eight k values at  128 block + 32 jj + 8 g.  A wave always has a chunk's worth
//      of K blocks requested ahead (register buffer kb is refilled for the next chunk as soon as its MFMAs are
//      issued): 8 to 32 KB per wave in flight at any time, in 256-byte runs per row.
// h is fed as the first operand and W' as the second, so accumulator register r of lane (li, g) is
// out[sequence 4g + r][row li]: stores are 64-byte runs per sequence instead of 4-byte pieces 4V bytes apart.
#define MFMA_THREADS 512
#define MFMA_LDS (64 * 1024)        // two buffers of K blocks x 4 fragments x 1 KB x groups of 16 sequences: at most 2x4
template <int NT, int TW, int MFMA_PIPE>
__device__ __forceinline__ void full_mfma_device(const FullArgs& f, int n, int seq0, uint4* lds, int block, int nblocks) {
    constexpr int NW = MFMA_THREADS / 64;
    constexpr int CH = MFMA_PIPE * 4 * NT * 64;       // 16-byte pieces per LDS buffer
    constexpr int SPT = CH / MFMA_THREADS;            // pieces a thread stages per chunk
    static_assert(CH % MFMA_THREADS == 0 && NW % NT == 0 && 2 * CH * 16 <= MFMA_LDS, "staging layout");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, g = lane >> 4;
    const int ntiles = (f.V + 15) >> 4;
    const int nq = f.d >> 3;                          // 16-byte pieces per row
    const int nsb = (f.d + 127) >> 7;                 // K blocks of 128
    const int nchunk = (nsb + MFMA_PIPE - 1) / MFMA_PIPE;
    const int ngroups = (ntiles + NW * TW - 1) / (NW * TW);
    // Staging: piece p = tid + 512 s of a buffer is lane p % 64 = lane of fragment p / 64 = (4 kb + jj) NT + t.  NT divides
    // the eight waves, so t, and with it the sequence 16 t + li, is the same for every piece a thread stages.
    const int st_sq = seq0 + (wave % NT) * 16 + li;
    const bool st_on = st_sq < n;
    const uint4* st_h = reinterpret_cast<const uint4*>(f.h) + (size_t)f.list[st_on ? st_sq : seq0] * nq;
    for (int grp = block; grp < ngroups; grp += nblocks) {
        const int tile0 = (grp * NW + wave) * TW;
        const uint4* ap[TW];
#pragma unroll
        for (int tw = 0; tw < TW; ++tw) ap[tw] = reinterpret_cast<const uint4*>(f.Wp + (size_t)min((tile0 + tw) * 16 + li, f.V - 1) * f.d);
        floatx4_t acc[TW][NT];
#pragma unroll
        for (int tw = 0; tw < TW; ++tw)
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[tw][t] = floatx4_t{0.f, 0.f, 0.f, 0.f};
        uint4 A[MFMA_PIPE][TW][4];
        uint4 sreg[SPT];
        // Nothing is done to a loaded value before its MFMA or its LDS store: an instruction on it would be waited for
        // where it stands, right behind the load.  Past the end of a row W' is read from a clamped address (the row's
        // own last piece) and meets zeros staged for h there; the zeros are selected when the piece is stored.
        auto load_A = [&](int kb, int sb) {           // K block sb of the wave's rows
#pragma unroll
            for (int tw = 0; tw < TW; ++tw)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) A[kb][tw][jj] = ap[tw][min(sb * 16 + jj * 4 + g, nq - 1)];
        };
        auto stage_q = [&](int c, int s) {
            const int kbjj = wave / NT + (NW / NT) * s;
            return (c * MFMA_PIPE + (kbjj >> 2)) * 16 + (kbjj & 3) * 4 + g;
        };
        auto stage_load = [&](int c) {
#pragma unroll
            for (int s = 0; s < SPT; ++s) sreg[s] = st_h[min(stage_q(c, s), nq - 1)];
        };
        auto stage_store = [&](uint4* buf, int c) {
#pragma unroll
            for (int s = 0; s < SPT; ++s) buf[tid + MFMA_THREADS * s] = keep_if(st_on && stage_q(c, s) < nq, sreg[s]);
        };
        stage_load(0);
#pragma unroll
        for (int kb = 0; kb < MFMA_PIPE; ++kb) load_A(kb, kb);
        stage_store(lds, 0);
        lds_barrier();
        // The last chunk is a copy of the loop body without the requests for a next one: with the requests under a
        // condition the compiler could not count, at compile time, how many younger loads a wait may leave open.
        auto chunk = [&](auto more_t, int c) {
            constexpr bool more = decltype(more_t)::value;
            const uint4* cur = lds + (c & 1) * CH;
            if (more) stage_load(c + 1);
            __builtin_amdgcn_sched_barrier(0);      // requests are issued where they are written: the scheduler would sink them
#pragma unroll
            for (int kb = 0; kb < MFMA_PIPE; ++kb) {
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        const uint4 Bv = cur[(((kb * 4 + jj) * NT + t) << 6) + lane];
#pragma unroll
                        for (int tw = 0; tw < TW; ++tw)
                            acc[tw][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, Bv),
                                                                                 __builtin_bit_cast(bf16x8_t, A[kb][tw][jj]), acc[tw][t], 0, 0, 0);
                    }
                __builtin_amdgcn_sched_barrier(0);
                if (more) load_A(kb, (c + 1) * MFMA_PIPE + kb);
                __builtin_amdgcn_sched_barrier(0);
            }
            if (more) stage_store(lds + ((c + 1) & 1) * CH, c + 1);
            lds_barrier();          // the chunk just consumed may be overwritten, the next one is complete
        };
        for (int c = 0; c + 1 < nchunk; ++c) chunk(std::true_type{}, c);
        chunk(std::false_type{}, nchunk - 1);
#pragma unroll
        for (int tw = 0; tw < TW; ++tw) {
            const int row = (tile0 + tw) * 16 + li;
            if (row < f.V) {
                const float bias = f.bp[row];
                const size_t col = f.scatter ? (size_t)f.perm[row] : (size_t)row;
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int sq = seq0 + t * 16 + 4 * g + r;
                        if (sq < n) f.out[(size_t)sq * f.out_stride + col] = acc[tw][t][r] + bias;
                    }
            }
        }
    }
}

// All n sequences through the MFMA path: up to 64 per pass over W'.  Two K blocks (of 128) are requested ahead: four
// measured 2-8 % slower at d = 8192 for up to 32 sequences (and spill with 64), one no faster, eight far slower.  The groups of 128 TW rows are dealt to the blocks in rounds:
// two row tiles per wave (a fragment of h read from LDS then serves two MFMAs) unless one tile per wave saves a
// round's worth of idle blocks.  Four tiles per wave with half the K blocks ahead measured 4-7 % slower at d = 8192.
template <int TW>
__device__ __forceinline__ void full_mfma_pass(const FullArgs& f, int n, uint4* lds, int block, int nblocks) {
    for (int s0 = 0; s0 < n; s0 += 64) {
        const int m = n - s0;
        if (m <= 16) full_mfma_device<1, TW, 2>(f, n, s0, lds, block, nblocks);
        else if (m <= 32) full_mfma_device<2, TW, 2>(f, n, s0, lds, block, nblocks);
        else full_mfma_device<4, TW, 2>(f, n, s0, lds, block, nblocks);
    }
}
__device__ __forceinline__ void full_mfma_all(const FullArgs& f, int n, uint4* lds, int block, int nblocks) {
    const int ntiles = (f.V + 15) >> 4, NW = MFMA_THREADS / 64;
    auto cost = [&](int tw) {           // rounds of groups x time of a group
        const int groups = (ntiles + NW * tw - 1) / (NW * tw);
        return (groups + nblocks - 1) / nblocks * tw;
    };
    if (cost(2) <= cost(1)) full_mfma_pass<2>(f, n, lds, block, nblocks);
    else full_mfma_pass<1>(f, n, lds, block, nblocks);
}

__global__ __launch_bounds__(MFMA_THREADS) void full_mfma_kernel(FullArgs f) {
    extern __shared__ uint4 mfma_lds[];
    const int n = f.n_ptr ? *f.n_ptr : f.n_fixed;
    if (n <= 0) return;
    full_mfma_all(f, n, mfma_lds, blockIdx.x, gridDim.x);
}

// The first stage for k <= RANK_DIRECT < n with the chunk's logits in registers (blockDim.x = SEQ_THREADS, sixteen values
// a thread): no staging, two passes over the registers.  Pass one: the thread's maximum, hence the maxima of 256 groups
// (the values i with i % 256 == g); their k-th largest is a threshold that k values reach (each thread counts the
// groups above its own, over half of them), their largest the chunk's maximum.  Pass two: the sum for the log-sum-exp,
// in block_lse's order (the same bits), and the values at or above the threshold, which are ranked like any other
// candidates.  Returns false (nothing decided) when more than CAND_CAP values reach the threshold.
template <class IdFn>
__device__ __forceinline__ bool fb_topk_regs(const float* __restrict__ vals, int n, int k, IdFn idf, SeqShared& s, LseAcc& l, int& kk) {
    extern __shared__ __align__(16) u64 arena[];
    constexpr int PER = FB_CHUNK / SEQ_THREADS;
    const int tid = threadIdx.x, lane = tid & 63;
    float v[PER];
    // all sixteen loads first, from clamped addresses; values past the end are replaced afterwards (a select behind each
    // load would be waited for where it stands: sixteen round trips one after the other)
#pragma unroll
    for (int j = 0; j < PER; ++j) v[j] = vals[min(tid + SEQ_THREADS * j, n - 1)];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int j = 0; j < PER; ++j)
        if (tid + SEQ_THREADS * j >= n) v[j] = -INFINITY;
    float* gm = reinterpret_cast<float*>(arena);
    float* cval = reinterpret_cast<float*>(reinterpret_cast<char*>(arena) + CAND_OFF);
    int* cid = reinterpret_cast<int*>(cval + CAND_CAP + 4);
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < PER; ++j) mx = fmaxf(mx, v[j]);
    gm[tid] = mx;
    if (tid < CAND_CAP) cval[tid] = -INFINITY;
    if (tid < 4) cval[CAND_CAP + tid] = -INFINITY;
    if (tid == 0) {
        s.cnt = 0;
        s.eq = 0xFFFFFFFFu;
    }
    __syncthreads();
    const int e = tid & 255, half = tid >> 8;
    const float ve = fmaxf(gm[e], gm[e + 256]);                  // the maximum of group e
    int gt = 0;
    const float4* gm4 = reinterpret_cast<const float4*>(gm);
#pragma unroll 8
    for (int q = half * 32; q < half * 32 + 32; ++q) {
        const float4 x = gm4[q], y = gm4[64 + q];
        gt += (fmaxf(x.x, y.x) > ve) + (fmaxf(x.y, y.y) > ve) + (fmaxf(x.z, y.z) > ve) + (fmaxf(x.w, y.w) > ve);
    }
    s.rank[tid] = gt;
    __syncthreads();
    if (tid < 256) {
        const int g = s.rank[tid] + s.rank[tid + 256];           // groups with a larger maximum
        if (g < k) atomicMin(&s.eq, lkey(ve));                   // the k-th largest is the smallest of those with fewer than k above
        if (g == 0) s.rem = __float_as_uint(ve);                 // the chunk's maximum (equal writes if it comes twice)
    }
    __syncthreads();
    const float th = fkey_inv(s.eq), vmax = __uint_as_float(s.rem);
    float sm = 0.f, over = 0.f;
#pragma unroll
    for (int j = 0; j < PER; ++j) {
        const int i = tid + SEQ_THREADS * j;
        if (vmax > -INFINITY && i < n) sm += expf(v[j] - vmax);
        const bool in = i < n && v[j] >= th;
        if (in) over += v[j] - th;
        const unsigned long long bal = __ballot(in);
        if (bal) {
            const int lead = __ffsll((long long)bal) - 1;
            unsigned base = 0;
            if (lane == lead) base = atomicAdd(&s.cnt, (unsigned)__popcll(bal));
            base = __shfl(base, lead, CSV_WAVE);
            const unsigned slot = base + (unsigned)__popcll(bal & ((1ull << lane) - 1ull));
            if (in && slot < CAND_CAP) {
                cval[slot] = v[j];
                cid[slot] = i;           // the token id is looked up below, for all candidates at once: a load from global
            }                            // memory in this loop would be waited for in every trip that collects something
        }
    }
    over = wave_sum(over);
    float* wover = reinterpret_cast<float*>(s.redu);
    if (lane == 0) wover[tid >> 6] = over;
    l.m = vmax;
    l.s = block_sum(sm, reinterpret_cast<float*>(s.redl));        // its barriers also publish the candidates and wover; not s.redf, which the ranking writes
    const int m = (int)s.cnt;
    if (m > CAND_CAP) return false;
    if (tid < m) cid[tid] = idf(cid[tid]);
    __syncthreads();
    kk = min(k, m);
    if (m > RANK_BUCKETS_MIN && th > -INFINITY) {
        float tot = 0.f;
        for (int q = 0; q < (SEQ_THREADS >> 6); ++q) tot += wover[q];
        rank_buckets(cval, cid, m, kk, th, fminf(vmax, th + 8.f * tot / (float)m), s);
    } else {
        float dummy;
        rank_small(cval, cid, m, kk, s, dummy);
    }
    return true;
}

// First stage of top-k / log-sum-exp over V: one block per (chunk of rows, fallback slot).  The chunk's logits
// are staged in LDS; token ids come from the permutation only for elements at the selection boundary.
template <bool THRESH>
__device__ __forceinline__ void fb_topk_device(const StepArgs& a, int slot, int chunk, SeqShared& s) {
    extern __shared__ __align__(16) u64 arena[];
    const int tid = threadIdx.x, nt = blockDim.x;
    const int c0 = chunk * FB_CHUNK;
    const int n = min(FB_CHUNK, a.V - c0);
    const float* vals = a.fb_logits + (size_t)slot * a.V + c0;
    auto idf = [&](int i) { return a.perm[c0 + i]; };
    const size_t pc = (size_t)slot * a.n_chunks + chunk;
    if (THRESH && a.k > 0 && a.k <= RANK_DIRECT && n > RANK_DIRECT) {
        LseAcc lr;
        int kr = 0;
        const bool done = fb_topk_regs(vals, n, a.k, idf, s, lr, kr);
        __syncthreads();
        if (done) {
            if (tid == 0) {
                a.cand_max[pc] = lr.m;
                a.cand_sum[pc] = lr.s;
            }
            for (int t = tid; t < a.k; t += nt) {
                a.cand_val[pc * a.k + t] = t < kr ? s.wval[t] : -INFINITY;
                a.cand_id[pc * a.k + t] = t < kr ? s.wid[t] : 0x7fffffff;
            }
            return;
        }
    }
    stage_to_lds(reinterpret_cast<float*>(arena), vals, n);
    __syncthreads();
    auto val = [](int i) { return reinterpret_cast<const float*>(arena)[i]; };
    const LseAcc l = block_lse(n, val, s);
    if (tid == 0) {
        a.cand_max[pc] = l.m;
        a.cand_sum[pc] = l.s;
    }
    if (a.k > 0) {
        int kk = 0;
        float vmax;
        bool done = false;
        if (THRESH && n > RANK_DIRECT) {
            __syncthreads();
            done = threshold_topk<false, true>(n, a.k, -INFINITY, false, idf, s, kk, vmax);
            __syncthreads();
        }
        if (!done) kk = block_topk(n, a.k, val, idf, s);
        for (int t = tid; t < a.k; t += nt) {
            a.cand_val[pc * a.k + t] = t < kk ? s.wval[t] : -INFINITY;
            a.cand_id[pc * a.k + t] = t < kk ? s.wid[t] : 0x7fffffff;
        }
    }
}

// Second stage: merge the chunk candidates of one fallback sequence and write its outputs.
template <bool THRESH>
__device__ __forceinline__ void fb_final_device(const StepArgs& a, int slot, SeqShared& s) {
    extern __shared__ __align__(16) u64 arena[];
    const int tid = threadIdx.x, nt = blockDim.x;
    const int b = a.fb_list[slot];
    const float* cm = a.cand_max + (size_t)slot * a.n_chunks;
    const float* cs = a.cand_sum + (size_t)slot * a.n_chunks;
    float mx = -INFINITY;
    for (int i = tid; i < a.n_chunks; i += nt) mx = fmaxf(mx, cm[i]);
    mx = block_max(mx, s.redf);
    float sm = 0.f;
    for (int i = tid; i < a.n_chunks; i += nt) sm += cs[i] * expf(cm[i] - mx);
    sm = block_sum(sm, s.redf);
    if (a.k > 0) {
        const float* cv = a.cand_val + (size_t)slot * a.n_chunks * a.k;
        const int32_t* ci = a.cand_id + (size_t)slot * a.n_chunks * a.k;
        const int n = a.n_chunks * a.k;
        if (n <= STAGE_CAP) {
            stage2_to_lds(reinterpret_cast<float*>(arena), cv, reinterpret_cast<int*>(arena) + STAGE_CAP, ci, n);
            __syncthreads();
            auto sval = [](int i) { return reinterpret_cast<const float*>(arena)[i]; };
            auto sid = [](int i) { return reinterpret_cast<const int*>(arena)[STAGE_CAP + i]; };
            int kk = 0;
            float vmax;
            bool done = false;
            if (THRESH && n > RANK_DIRECT) {
                done = threshold_topk(n, a.k, -INFINITY, false, sid, s, kk, vmax);
                __syncthreads();
            }
            if (!done) block_topk(n, a.k, sval, sid, s);
        } else {
            block_topk(n, a.k, [&](int i) { return cv[i]; }, [&](int i) { return ci[i]; }, s);
        }
        for (int t = tid; t < a.k; t += nt) {
            a.out.d_ids[(size_t)b * a.k + t] = s.wid[t];
            a.out.d_logits[(size_t)b * a.k + t] = s.wval[t];
        }
        write_distribution(a, b, min(a.k, a.V), mx + logf(sm), s);
    }
    if (tid == 0) {
        a.out.d_lse[b] = mx + logf(sm);
        a.out.d_flags[b] = CSV_FLAG_FALLBACK | CSV_FLAG_TOPK_CERT | CSV_FLAG_SOFTMAX_CERT;
        a.out.d_n_rows[b] = a.V;
        a.out.d_n_clusters[b] = a.C;
        if (a.out.d_fallback_count) atomicAdd(a.out.d_fallback_count, 1ull);
    }
}

// ================================================================================================ tail of a step
// Everything that is rarely needed runs in ONE kernel, so that a step whose sequences were all certified in round 0
// pays for one (immediately returning) launch instead of five: round-1 gathered GEMV, round-1 certification, the
// full-vocabulary product for fallback sequences, and the two stages of their top-k / log-sum-exp.  The phases
// depend on each other grid-wide, so the blocks meet at barriers built on device-scope atomics.  The grid is sized
// by the host so that all blocks are resident together; every wait is bounded: a block that waits too long raises
// the abort flag and every block leaves (the step's unfinished sequences keep the INVALID flag seed_kernel gave them).
#define TAIL_THREADS 512
static_assert(TAIL_THREADS == SEQ_THREADS, "the per-sequence phases assume one block size");
#define TAIL_SPIN_LIMIT (1 << 22)

// Returns false when the step was aborted.  Each barrier of a step uses its own counter.
__device__ __forceinline__ bool grid_barrier(int* counters, int which, int nblocks, int* s_flag, int spin_limit) {
    __syncthreads();
    if (threadIdx.x == 0) {
        __threadfence();
        atomicAdd(&counters[CNT_BARRIER + which], 1);
        int ok = 1, spins = 0;
        // relaxed polls (an acquire per poll would invalidate the XCD's L2 every time); the fence below acquires once
        while (__hip_atomic_load(&counters[CNT_BARRIER + which], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < nblocks) {
            if (__hip_atomic_load(&counters[CNT_ABORT], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) { ok = 0; break; }
            if (++spins > spin_limit) {
                atomicExch(&counters[CNT_ABORT], 1);
                ok = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(32);
        }
        __threadfence();
        *s_flag = ok;
    }
    __syncthreads();
    return *s_flag != 0;
}

// block / nblocks: this block's position among the blocks that run the tail together (all resident).
template <bool THRESH>
__device__ __forceinline__ void tail_device(const StepArgs& a, const FullArgs& f, int fallback_only, int block, int nblocks,
                                            SeqShared& s, GemvShared& gs, int* s_flag) {
    extern __shared__ __align__(16) u64 arena[];
    const int tid = threadIdx.x;
    if (a.counters[CNT_TAIL_NEEDED] == 0) return;      // the common case at small batches: one word, no reduction
    if (fallback_only && a.counters[CNT_FALLBACK] == 0) return;
    // is any sequence waiting for round 0 (a seed prefix too large for the round-0 blocks), for round 1 or for the
    // full product?  Every block reads the same, settled values.
    int mine0 = 0, mine1 = 0;
    if (tid < a.B) {
        mine0 = a.counters[CNT_TILES + tid];
        mine1 = a.counters[CNT_TILES + CSV_MAX_BATCH + tid];
    }
    const int n_fb0 = a.counters[CNT_FALLBACK];
    int tiles0 = block_sum_i(mine0, s.redi);
    int tiles = block_sum_i(mine1, s.redi);
    if (fallback_only) tiles0 = tiles = 0;      // the rounds ran as launches of their own
    if (tiles0 == 0 && tiles == 0 && n_fb0 == 0) return;

    // Rounds: the GEMV over the round's work list, then the certification, which may plan the next round.
    // Round 0 is here only for seed prefixes that the round-0 blocks handed over.
    for (int r = tiles0 > 0 ? 0 : 1; r < a.max_rounds && !fallback_only; ++r) {
        if (r > 0) {
            if (r > 1 || tiles0 > 0) {   // planned by a certification earlier in this kernel: read past the barrier
                const int mine = tid < a.B ? __hip_atomic_load(&a.counters[CNT_TILES + r * CSV_MAX_BATCH + tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0;
                tiles = block_sum_i(mine, s.redi);
            }
            if (tiles == 0) break;
        }
        gemv_tiles_device(a, r, reinterpret_cast<uint4*>(arena), gs, block, nblocks);
        if (!grid_barrier(a.counters, 2 * r, nblocks, s_flag, a.spin_limit)) return;
        // chunk-major items: the first chunks of all sequences (often the only ones with work) go to distinct blocks
        for (int item = block; item < a.B * a.sp_chunks; item += nblocks) {
            cert_device<THRESH>(a, item % a.B, item / a.B, r, s);
            __syncthreads();
        }
        if (!grid_barrier(a.counters, 2 * r + 1, nblocks, s_flag, a.spin_limit)) return;
    }
    const int n_fb = __hip_atomic_load(&a.counters[CNT_FALLBACK], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
    if (n_fb == 0) return;
    // the same rule as the separate launches, so that a sequence's logits do not depend on how the step was launched
    if (n_fb > FULL_G)
        full_mfma_all(f, n_fb, reinterpret_cast<uint4*>(arena), block, nblocks);
    else
        full_gemv_device(f, n_fb, reinterpret_cast<uint4*>(arena), block, nblocks);
    if (!grid_barrier(a.counters, 2 * CSV_MAX_ROUNDS, nblocks, s_flag, a.spin_limit)) return;
    for (int item = block; item < n_fb * a.n_chunks; item += nblocks) {
        fb_topk_device<THRESH>(a, item / a.n_chunks, item % a.n_chunks, s);
        __syncthreads();
    }
    if (!grid_barrier(a.counters, 2 * CSV_MAX_ROUNDS + 1, nblocks, s_flag, a.spin_limit)) return;
    for (int slot = block; slot < n_fb; slot += nblocks) {
        fb_final_device<THRESH>(a, slot, s);
        __syncthreads();
    }
}

__global__ __launch_bounds__(TAIL_THREADS) void tail_kernel(StepArgs a, FullArgs f, int fallback_only) {
    __shared__ SeqShared s;
    __shared__ GemvShared gs;
    __shared__ int s_flag;
    tail_device<true>(a, f, fallback_only, blockIdx.x, gridDim.x, s, gs, &s_flag);
}

// ------------------------------------------------------------------------------------------------ round 0 as a launch
// Plain form, grid NB x B: round 0 only; what follows is launched separately.
__global__ __launch_bounds__(SEQ_THREADS) void round0_kernel(StepArgs a, int NB) {
    __shared__ SeqShared s;
    round0_device(a, blockIdx.x / NB, blockIdx.x % NB, NB, s);
}

// Fused form, used while recent steps rarely needed anything after round 0: the first NB x B blocks run round 0,
// the remaining blocks are the tail's blocks, parked until every sequence's round 0 is settled.  When nothing is
// queued for them (the common case) they leave at once: the step has saved a kernel launch.  Otherwise they run the
// tail exactly as tail_kernel does (the round-0 blocks have left by then; the tail's blocks are all resident: the
// host sizes the grid for one block per compute unit).  Blocks start in index order, so the blocks waited for are
// already running when a parked block starts; the wait is bounded all the same (the poll limit of the grid barriers).
__global__ __launch_bounds__(SEQ_THREADS) void step_kernel(StepArgs a, FullArgs f, int NB) {
    __shared__ SeqShared s;
    __shared__ GemvShared gs;
    __shared__ int s_flag;
    const int n0 = NB * a.B;
    if ((int)blockIdx.x < n0) {
        const int settled = round0_device(a, blockIdx.x / NB, blockIdx.x % NB, NB, s, &a.counters[CNT_R0_DONE]);
        if (!settled || settled == 3) return;          // 3: finished and already counted
        __syncthreads();                      // all of the block's writes are issued
        if (threadIdx.x == 0) {
            // One word tells the parked blocks both things: sequences settled (low half) and whether any of them
            // left work for the tail (high half).  Work is released before the count; a finished sequence left
            // nothing for the tail to read.
            if (settled == 2) __threadfence();
            atomicAdd(&a.counters[CNT_R0_DONE], settled == 2 ? 0x10001 : 1);
        }
        return;
    }
    if (threadIdx.x == 0) {
        int ok = 1, spins = 0, v;
        while (((v = __hip_atomic_load(&a.counters[CNT_R0_DONE], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) & 0xffff) < a.B) {
            if (++spins > a.spin_limit) {
                atomicExch(&a.counters[CNT_ABORT], 1);
                ok = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(4);
        }
        if (ok && (v >> 16) == 0) ok = 0;     // every sequence finished in round 0: nothing to do, nothing to acquire
        if (ok) __threadfence();              // acquire
        s_flag = ok;
    }
    __syncthreads();
    if (!s_flag) return;
    tail_device<false>(a, f, 0, (int)blockIdx.x - n0, (int)gridDim.x - n0, s, gs, &s_flag);   // the lean form: see cert_body
}

// ------------------------------------------------------------------------------------------------ the tail, one launch per phase
// The same phases as tail_kernel as separate launches, used while recent steps needed them: a kernel boundary
// costs about 2.5 us on this machine, a grid barrier among 256 resident blocks 14-24 us (every block's device-scope
// release and acquire writes back and invalidates its XCD's L2).  Every kernel finds out on the device whether it
// has anything to do.
__global__ __launch_bounds__(TAIL_THREADS, 2) void round_gemv_kernel(StepArgs a, int r) {
    extern __shared__ __align__(16) u64 arena[];
    __shared__ GemvShared gs;
    if (a.counters[CNT_TAIL_NEEDED] == 0) return;
    gemv_tiles_device(a, r, reinterpret_cast<uint4*>(arena), gs, blockIdx.x, gridDim.x);
}

__global__ __launch_bounds__(SEQ_THREADS) void round_cert_kernel(StepArgs a, int r) {   // grid (B, chunks per sequence)
    __shared__ SeqShared s;
    if (a.counters[CNT_TAIL_NEEDED] == 0) return;
    cert_device<true>(a, blockIdx.x, blockIdx.y, r, s);
}

// Up to FULL_G fallback sequences take the vector product, more the MFMA product, which needs a compute unit's whole
// register file.  A batch of at most FULL_G sequences launches the first kernel, a larger one the second, which holds
// both products and picks by the number of fallback sequences.
__global__ __launch_bounds__(TAIL_THREADS, 2) void fb_product_kernel(StepArgs a, FullArgs f) {
    extern __shared__ __align__(16) u64 arena[];
    const int n_fb = a.counters[CNT_FALLBACK];
    if (n_fb == 0 || n_fb > FULL_G) return;
    full_gemv_device(f, n_fb, reinterpret_cast<uint4*>(arena), blockIdx.x, gridDim.x);
}

__global__ __launch_bounds__(MFMA_THREADS) void fb_product_mfma_kernel(StepArgs a, FullArgs f) {
    extern __shared__ uint4 mfma_lds[];
    const int n_fb = a.counters[CNT_FALLBACK];
    if (n_fb == 0) return;
    if (n_fb > FULL_G) full_mfma_all(f, n_fb, mfma_lds, blockIdx.x, gridDim.x);
    else full_gemv_device(f, n_fb, mfma_lds, blockIdx.x, gridDim.x);
}

__global__ __launch_bounds__(SEQ_THREADS) void fb_topk_kernel(StepArgs a) {             // grid (chunks of V, B)
    __shared__ SeqShared s;
    if ((int)blockIdx.y >= a.counters[CNT_FALLBACK]) return;
    fb_topk_device<true>(a, blockIdx.y, blockIdx.x, s);
}

__global__ __launch_bounds__(SEQ_THREADS) void fb_final_kernel(StepArgs a) {            // grid B
    __shared__ SeqShared s;
    if ((int)blockIdx.x >= a.counters[CNT_FALLBACK]) return;
    fb_final_device<true>(a, blockIdx.x, s);
}

// ================================================================================================ host side
static void profile_release(csv_workspace* ws);

static int next_pow2(int x) {
    int p = 1;
    while (p < x) p <<= 1;
    return p;
}

// dynamic LDS of the per-sequence kernels
static size_t seed_lds(const csv_workspace* ws) {
    const size_t general = (size_t)ws->Npad * 8 + (size_t)ws->C * 8 + 8;       // keys, offsets, tail terms
    const size_t staged = (size_t)ws->C * 16 + 32;                             // bounds, ln n, {first row, rows} (small indexes)
    return general > staged ? general : staged;
}
static size_t cert_lds(const csv_workspace* ws) {
    const size_t plan = seed_lds(ws), stage = (size_t)CAND_OFF + CAND_BYTES;      // staged logits and ids, then the candidates of a later round
    return plan > stage ? plan : stage;
}
static size_t round0_h_off(const csv_workspace* ws) { return (seed_lds(ws) + 15) / 16 * 16; }
static size_t round0_lds(const csv_workspace* ws) {
    const size_t c = cert_lds(ws), h = round0_h_off(ws) + (size_t)ws->d * 2;
    return c > h ? c : h;
}

static void fill_args(StepArgs& a, const csv_workspace* ws, const csv_index* idx) {
    memset(&a, 0, sizeof(a));
    a.V = idx->V; a.d = idx->d; a.C = idx->C;
    a.Wp = idx->Wp; a.bp = idx->bp; a.perm = idx->perm; a.mu = idx->mu; a.mu16 = idx->mu16; a.R = idx->R; a.bmax = idx->bmax;
    a.n = idx->n; a.off = idx->off; a.lnn = idx->lnn; a.cmeta = idx->cmeta; a.bt = idx->bt; a.bt_m = idx->bt_m; a.ang = idx->ang; a.ln_nmax = idx->ln_nmax;
    a.K_cap = ws->K_cap; a.Npad = ws->Npad; a.n_chunks = ws->n_chunks; a.tile_stride = ws->tile_stride; a.sp_chunks = ws->sp_chunks; a.cand_chunks = ws->cand_chunks;
    a.U = ws->U; a.hnorm = ws->hnorm; a.bound_partial = ws->bound_partial; a.st = ws->st; a.sel = ws->sel; a.slog = ws->slog; a.sid = ws->sid; a.slots = ws->slots; a.B_max = ws->B_max;
    a.tiles[0] = ws->tiles[0]; a.tiles[1] = ws->tiles[1]; a.counters = ws->counters;
    a.r0_h_off = (int)(round0_h_off(ws) / 16);
    a.tail_lds = (int)ws->tail_lds;
    a.spin_limit = ws->spin_limit;
    a.host_history = ws->d_history;
    a.fb_list = ws->fb_list; a.fb_logits = ws->fb_logits; a.cand_val = ws->cand_val; a.cand_id = ws->cand_id;
    a.cand_max = ws->cand_max; a.cand_sum = ws->cand_sum;
}

static int check_pair(const csv_workspace* ws, const csv_index* idx, const void* d_h, int B) {
    if (!ws || !idx || !d_h) { csv_set_error("null workspace, index or h"); return CSV_EINVAL; }
    if (ws->V != idx->V || ws->d != idx->d || ws->C != idx->C) { csv_set_error("workspace was created for another index shape"); return CSV_ESHAPE; }
    if (B < 1 || B > ws->B_max) { csv_set_error("B=%d outside 1..%d", B, ws->B_max); return CSV_ESHAPE; }
    return CSV_OK;
}

// The dynamic-LDS limit of a kernel is one attribute per process and device, shared by every workspace: it is only
// ever raised, so a workspace created later with smaller needs cannot take away what an earlier one's launches rely on.
enum { K_ROUND0, K_STEP, K_TAIL, K_RCERT, K_FBPROD, K_FBPRODM, K_FULLMFMA, K_ALG1, K_BOUND0, K_NKERN = K_BOUND0 + 8 };
static size_t g_lds_limit[CSV_STATIC_MAX_DEVICES][K_NKERN];
static pthread_mutex_t g_attr_lock = PTHREAD_MUTEX_INITIALIZER;
#define CSV_STATIC_LDS_MAX 16384     // at least the static shared memory of any kernel here
static hipError_t raise_lds(int dev, int which, const void* fn, size_t bytes) {
    if (dev < 0 || dev >= CSV_STATIC_MAX_DEVICES) return hipErrorInvalidDevice;
    hipError_t e = hipSuccess;
    pthread_mutex_lock(&g_attr_lock);
    if (bytes > g_lds_limit[dev][which]) {
        if (bytes + CSV_STATIC_LDS_MAX > 65536) e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e == hipSuccess) g_lds_limit[dev][which] = bytes;
    }
    pthread_mutex_unlock(&g_attr_lock);
    return e;
}

// K slices of the batched bound product and k-blocks (of 32) per slice: enough slices that (groups of cluster tiles x
// slices) fills the device, a whole number of request chunks per slice, a slice's h within BOUND_LDS_KB of LDS, at most
// BOUND_KS_MAX slices (the partial buffer holds KS x B x C floats).  B decides how many sequence tiles a block carries.
static int bound_mfma_nt(int B) { return B > 32 ? 4 : (B > 16 ? 2 : 1); }
static void bound_mfma_plan(int C, int d, int B, int& KS, int& kbs) {
    const int tiles = (C + 15) / 16, groups = (tiles + BOUND_TILES_PER_BLOCK - 1) / BOUND_TILES_PER_BLOCK, nkb = (d + 31) / 32;
    KS = (BOUND_BLOCK_TARGET + groups - 1) / groups;
    if (KS > BOUND_KS_MAX) KS = BOUND_KS_MAX;
    if (KS > nkb) KS = nkb;
    kbs = (nkb + KS - 1) / KS;
    kbs = (kbs + BOUND_PIPE - 1) / BOUND_PIPE * BOUND_PIPE;     // whole chunks
    const int cap = BOUND_LDS_KB / bound_mfma_nt(B) / BOUND_PIPE * BOUND_PIPE;
    if (kbs > cap) kbs = cap;                                   // d <= 8192: 256 k-blocks in at most 32 slices of 8 always fit
    KS = (nkb + kbs - 1) / kbs;
}

static int launch_bounds_kernel(const StepArgs& a, float* U, float* hn, int reset, hipStream_t st) {
    if (a.B >= BOUND_MFMA_MIN_B) {
        const int tiles = (a.C + 15) / 16;
        int KS, kbs;
        bound_mfma_plan(a.C, a.d, a.B, KS, kbs);
        dim3 grid((tiles + BOUND_TILES_PER_BLOCK - 1) / BOUND_TILES_PER_BLOCK, KS);
        for (int s0 = 0; s0 < a.B; s0 += 64) {
            const int nseq = a.B - s0 < 64 ? a.B - s0 : 64;
            const int r = reset && s0 == 0;
            const int nt = nseq <= 16 ? 1 : (nseq <= 32 ? 2 : 4);
            const size_t lds = (size_t)kbs * nt * 1024;
            if (a.mu16) {
                if (nt == 1) bound_mfma_kernel<1, true><<<grid, 512, lds, st>>>(a, a.bound_partial, s0, KS, kbs, r);
                else if (nt == 2) bound_mfma_kernel<2, true><<<grid, 512, lds, st>>>(a, a.bound_partial, s0, KS, kbs, r);
                else bound_mfma_kernel<4, true><<<grid, 512, lds, st>>>(a, a.bound_partial, s0, KS, kbs, r);
            } else {
                if (nt == 1) bound_mfma_kernel<1, false><<<grid, 512, lds, st>>>(a, a.bound_partial, s0, KS, kbs, r);
                else if (nt == 2) bound_mfma_kernel<2, false><<<grid, 512, lds, st>>>(a, a.bound_partial, s0, KS, kbs, r);
                else bound_mfma_kernel<4, false><<<grid, 512, lds, st>>>(a, a.bound_partial, s0, KS, kbs, r);
            }
            CSV_LAUNCH_CHECK("bound_mfma_kernel");
        }
        bound_finish_kernel<<<dim3((a.C + 255) / 256, a.B), 256, 0, st>>>(a, a.bound_partial, KS, U, hn);
        CSV_LAUNCH_CHECK("bound_finish_kernel");
        return CSV_OK;
    }
    int bt = 1;
    while (bt < a.B && bt < 4) bt <<= 1;       // B <= 4 here (more sequences take the MFMA product)
    while (bt > 1 && (size_t)bt * a.d * 2 > BOUND_LDS_MAX) bt >>= 1;
    const bool m16 = a.mu16 != nullptr;
    const size_t lds = (size_t)bt * a.d * 2;
    if (a.B == 1) {
        const int nq = m16 ? a.d >> 3 : a.d >> 2;     // 128-bit units per centroid row
        int wpc = 1;
        while (wpc < 4 && (nq + wpc - 1) / wpc > 64 * BOUND_PF) wpc <<= 1;
        const int cpb = (BOUND_THREADS / 64) / wpc;
        const int groups = (a.C + cpb - 1) / cpb;
        const int gpx = (groups + 7) / 8;
        if (m16) bound1_kernel<true><<<gpx * 8, BOUND_THREADS, 0, st>>>(a, U, hn, reset, groups, gpx, wpc);
        else bound1_kernel<false><<<gpx * 8, BOUND_THREADS, 0, st>>>(a, U, hn, reset, groups, gpx, wpc);
        CSV_LAUNCH_CHECK("bound1_kernel");
        return CSV_OK;
    }
    int dev = 0, cus = 0;
    CSV_HIP(hipGetDevice(&dev));
    CSV_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    // as many blocks as are resident together (LDS decides), at most one wave per cluster
    int per_cu = (int)((size_t)(150 * 1024) / (lds + 1024));
    per_cu = per_cu < 1 ? 1 : (per_cu > 4 ? 4 : per_cu);
    int gx = (a.C + (BOUND_THREADS / 64) - 1) / (BOUND_THREADS / 64);
    if (gx > cus * per_cu) gx = cus * per_cu;
    dim3 grid(gx, (a.B + bt - 1) / bt);
    if (lds + 4096 > 65536) {        // more dynamic LDS than the default limit: raise this variant's attribute (only ever upwards)
        const void* fn = nullptr;
        switch (bt) {
            case 2: fn = m16 ? (const void*)bound_kernel<2, true> : (const void*)bound_kernel<2, false>; break;
            case 4: fn = m16 ? (const void*)bound_kernel<4, true> : (const void*)bound_kernel<4, false>; break;
            default: fn = m16 ? (const void*)bound_kernel<1, true> : (const void*)bound_kernel<1, false>; break;
        }
        const int slot = K_BOUND0 + (bt == 1 ? 0 : bt == 2 ? 1 : bt == 4 ? 2 : 3) * 2 + (m16 ? 1 : 0);
        CSV_HIP(raise_lds(dev, slot, fn, BOUND_LDS_MAX));
    }
#define CSV_BOUND_LAUNCH(BT)                                                                   \
    do {                                                                                       \
        if (m16) bound_kernel<BT, true><<<grid, BOUND_THREADS, lds, st>>>(a, U, hn, reset);    \
        else bound_kernel<BT, false><<<grid, BOUND_THREADS, lds, st>>>(a, U, hn, reset);       \
    } while (0)
    switch (bt) {
        case 1: CSV_BOUND_LAUNCH(1); break;        // 2..4 sequences of rows too long for two of them in LDS
        case 2: CSV_BOUND_LAUNCH(2); break;
        default: CSV_BOUND_LAUNCH(4); break;
    }
#undef CSV_BOUND_LAUNCH
    CSV_LAUNCH_CHECK("bound_kernel");
    return CSV_OK;
}

// out[s][perm[r]] = tmp[s][r]: coalesced reads, scattered 4-byte writes, kept out of the streaming product kernel
__global__ __launch_bounds__(256) void unpermute_kernel(const float* __restrict__ tmp, const int32_t* __restrict__ perm, int V,
                                                        float* __restrict__ out) {
    const int r = blockIdx.x * 256 + threadIdx.x, s = blockIdx.y;
    if (r < V) out[(size_t)s * V + perm[r]] = tmp[(size_t)s * V + r];
}

// tmp: [n_fixed x V] scratch for the MFMA path when the result is wanted in token-id order (may be NULL otherwise)
static int launch_full(const csv_index* idx, const uint16_t* d_h, const int32_t* list, const int32_t* n_ptr, int n_fixed,
                       float* out, long long stride, int scatter, float* tmp, hipStream_t st) {
    FullArgs f;
    f.V = idx->V; f.d = idx->d; f.Wp = idx->Wp; f.bp = idx->bp; f.perm = idx->perm; f.h = d_h;
    f.list = list; f.n_ptr = n_ptr; f.n_fixed = n_fixed; f.out = out; f.out_stride = stride; f.scatter = scatter;
    if (!n_ptr && n_fixed > FULL_G) {
        int dev = 0, cus = 0;
        CSV_HIP(hipGetDevice(&dev));
        CSV_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
        const bool two_step = scatter && tmp && stride == idx->V;
        if (two_step) {
            f.out = tmp;
            f.scatter = 0;
        }
        full_mfma_kernel<<<cus, MFMA_THREADS, MFMA_LDS, st>>>(f);
        CSV_LAUNCH_CHECK("full_mfma_kernel");
        if (two_step) {
            unpermute_kernel<<<dim3((idx->V + 255) / 256, n_fixed), 256, 0, st>>>(tmp, idx->perm, idx->V, out);
            CSV_LAUNCH_CHECK("unpermute_kernel");
        }
        return CSV_OK;
    }
    const int ntiles = (idx->V + 7) / 8;
    const int grid = ntiles < 2048 ? ntiles : 2048;
    full_gemv_kernel<<<grid, 256, (size_t)FULL_G * idx->d * 2, st>>>(f);
    CSV_LAUNCH_CHECK("full_gemv_kernel");
    return CSV_OK;
}

extern "C" int csv_workspace_create(const csv_index* idx, int B_max, int K_cap_rows, csv_workspace** out) {
    if (out) *out = nullptr;
    if (!idx || !out) { csv_set_error("null index or out"); return CSV_EINVAL; }
    if (B_max < 1 || B_max > CSV_MAX_BATCH) { csv_set_error("B_max=%d outside 1..%d", B_max, CSV_MAX_BATCH); return CSV_ESHAPE; }
    if (K_cap_rows < 0 || K_cap_rows > idx->V) { csv_set_error("K_cap_rows=%d outside 0..V", K_cap_rows); return CSV_EINVAL; }
    if ((size_t)FULL_G * idx->d * 2 > 65536) { csv_set_error("d=%d too large for the LDS staging of h", idx->d); return CSV_ESHAPE; }
    csv_workspace* ws = (csv_workspace*)calloc(1, sizeof(csv_workspace));
    if (!ws) { csv_set_error("host allocation failed"); return CSV_ENOMEM; }
    ws->B_max = B_max; ws->K_cap = K_cap_rows > 0 ? K_cap_rows : 1; ws->V = idx->V; ws->d = idx->d; ws->C = idx->C;
    ws->Npad = next_pow2(idx->C);
    ws->n_chunks = (idx->V + FB_CHUNK - 1) / FB_CHUNK;
    ws->device = idx->device;
    ws->sp_chunks = (ws->K_cap + STAGE_CAP - 1) / STAGE_CAP;
    ws->cand_chunks = ws->n_chunks > ws->sp_chunks ? ws->n_chunks : ws->sp_chunks;
    const size_t B = B_max, C = idx->C, V = idx->V, K = ws->K_cap, NC = ws->cand_chunks;
    ws->tile_stride = (int)(K / TILE_ROWS + C + 1);
    const size_t tcap = B * (size_t)ws->tile_stride;
    hipError_t e = hipSuccess;
    auto A = [&](void** p, size_t bytes) { if (e == hipSuccess) e = hipMalloc(p, bytes ? bytes : 16); };
    A((void**)&ws->U, B * C * 4); A((void**)&ws->bound_partial, B_max >= BOUND_MFMA_MIN_B ? B * C * 4 * BOUND_KS_MAX : 16); A((void**)&ws->hnorm, B * 4); A((void**)&ws->st, B * sizeof(SeqState));
    A((void**)&ws->sel, B * C * 4); A((void**)&ws->slog, B * K * 4); A((void**)&ws->sid, B * K * 4);
    A((void**)&ws->slots, B * CSV_SLOT_ROWS * 8);
    A((void**)&ws->tiles[0], tcap * sizeof(Tile)); A((void**)&ws->tiles[1], tcap * sizeof(Tile));
    A((void**)&ws->counters, CNT_ALLOC * 4); A((void**)&ws->fb_list, B * 4); A((void**)&ws->all_list, B * 4);
    A((void**)&ws->fb_logits, B * V * 4); A((void**)&ws->cand_val, B * NC * CSV_MAX_K * 4); A((void**)&ws->cand_id, B * NC * CSV_MAX_K * 4);
    A((void**)&ws->cand_max, B * NC * 4); A((void**)&ws->cand_sum, B * NC * 4);
    if (e == hipSuccess) e = hipMemset(ws->counters, 0, CNT_ALLOC * 4);
    if (e == hipSuccess) e = hipHostMalloc((void**)&ws->h_history, 64, hipHostMallocDefault);
    if (e == hipSuccess) {
        *ws->h_history = 0;
        e = hipHostGetDevicePointer((void**)&ws->d_history, ws->h_history, 0);
    }
    if (e == hipSuccess) e = hipMemset(ws->slots, 0xFF, B * CSV_SLOT_ROWS * 8);     // every slot empty
    if (e == hipSuccess) e = hipMemset(ws->st, 0, B * sizeof(SeqState));
    if (e == hipSuccess) e = hipMemset(ws->tiles[0], 0, tcap * sizeof(Tile));
    if (e == hipSuccess) e = hipMemset(ws->tiles[1], 0, tcap * sizeof(Tile));
    if (e == hipSuccess) {
        int32_t* tmp = (int32_t*)malloc(B * 4);
        for (size_t i = 0; i < B; ++i) tmp[i] = (int32_t)i;
        e = hipMemcpy(ws->all_list, tmp, B * 4, hipMemcpyHostToDevice);
        free(tmp);
    }
    // the per-sequence kernels may need more dynamic LDS than the default limit when C is large
    if (e == hipSuccess) e = raise_lds(ws->device, K_FULLMFMA, (const void*)full_mfma_kernel, MFMA_LDS);
    if (e == hipSuccess) e = raise_lds(ws->device, K_ROUND0, (const void*)round0_kernel, round0_lds(ws));
    if (e == hipSuccess) {
        size_t l = cert_lds(ws);
        const size_t cand[] = {(size_t)FULL_G * idx->d * 2 /* also covers the two h slots of the tile loop */, (size_t)FB_CHUNK * 4, (size_t)STAGE_CAP * 8,
                               B_max > FULL_G ? (size_t)MFMA_LDS : 0 /* more than FULL_G fallback sequences: the MFMA product's h fragments */};
        for (size_t c : cand) l = c > l ? c : l;
        ws->tail_lds = l;
        e = raise_lds(ws->device, K_TAIL, (const void*)tail_kernel, l);
        int per_cu = 0, dev = 0, cus = 0;
        if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, tail_kernel, TAIL_THREADS, l);
        if (e == hipSuccess) e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess && (per_cu < 1 || cus < 1)) {
            csv_set_error("tail kernel does not fit a compute unit (dynamic LDS %zu bytes)", l);
            csv_workspace_free(ws);
            return CSV_ESHAPE;
        }
        // All blocks of the tail kernel must be resident together, which the occupancy check above guarantees
        // for one block per compute unit.  A second block per unit measured slower at every batch size: the
        // grid barriers cost more with twice the arrivals, and the row loops already keep enough loads in flight.
        ws->tail_grid = cus;
        ws->spin_limit = TAIL_SPIN_LIMIT;
        ws->split_min_B = 0;      // decided per step from the history
        if (e == hipSuccess) e = raise_lds(ws->device, K_RCERT, (const void*)round_cert_kernel, cert_lds(ws));
        if (e == hipSuccess) e = raise_lds(ws->device, K_FBPROD, (const void*)fb_product_kernel, (size_t)FULL_G * idx->d * 2);
        if (e == hipSuccess) e = raise_lds(ws->device, K_FBPRODM, (const void*)fb_product_mfma_kernel, MFMA_LDS);
        int r0_per_cu = 0;
        if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&r0_per_cu, round0_kernel, SEQ_THREADS, round0_lds(ws));
        if (e == hipSuccess && r0_per_cu < 1) {
            csv_set_error("round-0 kernel does not fit a compute unit (dynamic LDS %zu bytes)", round0_lds(ws));
            csv_workspace_free(ws);
            return CSV_ESHAPE;
        }
        ws->round0_capacity = r0_per_cu * cus;
        // round 0 and the tail in one launch: every block of that grid (one per compute unit) must be resident
        ws->fused_lds = round0_lds(ws) > l ? round0_lds(ws) : l;
        int fused_per_cu = 0;
        if (e == hipSuccess) e = raise_lds(ws->device, K_STEP, (const void*)step_kernel, ws->fused_lds);
        if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&fused_per_cu, step_kernel, SEQ_THREADS, ws->fused_lds);
        ws->fused_ok = fused_per_cu >= 1;
    }
    if (e != hipSuccess) {
        csv_set_error("workspace allocation failed: %s", hipGetErrorString(e));
        csv_workspace_free(ws);
        return e == hipErrorOutOfMemory ? CSV_ENOMEM : CSV_EHIP;
    }
    *out = ws;
    return CSV_OK;
}

extern "C" void csv_workspace_free(csv_workspace* ws) {
    if (!ws) return;
    void* ptrs[] = {ws->U, ws->bound_partial, ws->hnorm, ws->st, ws->sel, ws->slog, ws->sid, ws->slots, ws->tiles[0], ws->tiles[1],
                    ws->counters, ws->fb_list, ws->all_list, ws->fb_logits, ws->cand_val, ws->cand_id, ws->cand_max, ws->cand_sum};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    if (ws->h_history) (void)hipHostFree(ws->h_history);
    profile_release(ws);
    free(ws);
}

extern "C" int csv_bounds(csv_workspace* ws, const csv_index* idx, const uint16_t* d_h, int B, float* d_U, float* d_hnorm,
                          void* stream) {
    int rc = check_pair(ws, idx, d_h, B);
    if (rc) return rc;
    if (!d_U) { csv_set_error("null d_U"); return CSV_EINVAL; }
    StepArgs a;
    fill_args(a, ws, idx);
    a.B = B; a.h = d_h;
    return launch_bounds_kernel(a, d_U, d_hnorm, 0, (hipStream_t)stream);
}

// ------------------------------------------------------------------------------------------------ bounds without a workspace
// For callers that cannot allocate: the K-slice partial sums of the batched bound product (the only scratch the
// bound kernels use) live in a file-scope device array instead of a workspace buffer.  Every GPU holds its own copy
// of the array at its own address; the address is looked up once per device and handed to the kernels as an argument.
#define CSV_STATIC_SCRATCH_BYTES (8u << 20)
static __device__ __align__(256) unsigned char scratch[CSV_STATIC_SCRATCH_BYTES];
static void* g_scratch_ptr[CSV_STATIC_MAX_DEVICES];          // per device: address of `scratch` there (NULL = not looked up yet)
static pthread_mutex_t g_scratch_lock = PTHREAD_MUTEX_INITIALIZER;

// Address of the array on the current device (looked up on the first call there).
static int static_scratch(int dev, void** out) {
    if (dev < 0 || dev >= CSV_STATIC_MAX_DEVICES) { csv_set_error("device %d outside 0..%d", dev, CSV_STATIC_MAX_DEVICES - 1); return CSV_EINVAL; }
    pthread_mutex_lock(&g_scratch_lock);
    void* p = g_scratch_ptr[dev];
    if (!p) {
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            pthread_mutex_unlock(&g_scratch_lock);
            csv_set_error("hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
            return CSV_EHIP;
        }
        g_scratch_ptr[dev] = p;
    }
    pthread_mutex_unlock(&g_scratch_lock);
    *out = p;
    return CSV_OK;
}

extern "C" int csv_bounds_static(const csv_index* idx, const uint16_t* d_h, int B, float* d_U, float* d_hnorm, void* stream) {
    if (!idx || !d_h || !d_U) { csv_set_error("null index, h or d_U"); return CSV_EINVAL; }
    if (B < 1 || B > CSV_MAX_BATCH) { csv_set_error("B=%d outside 1..%d", B, CSV_MAX_BATCH); return CSV_ESHAPE; }
    int dev = -1;
    CSV_HIP(hipGetDevice(&dev));
    if (dev != idx->device) { csv_set_error("the index lives on device %d, the current device is %d", idx->device, dev); return CSV_EINVAL; }
    StepArgs a;
    memset(&a, 0, sizeof(a));
    a.V = idx->V; a.d = idx->d; a.C = idx->C;
    a.mu = idx->mu; a.mu16 = idx->mu16; a.R = idx->R; a.bmax = idx->bmax; a.n = idx->n; a.bt = idx->bt; a.bt_m = idx->bt_m; a.ang = idx->ang;
    a.B = B; a.h = d_h;
    if (B >= BOUND_MFMA_MIN_B) {       // the batched product is the only bound kernel with scratch: KS x B x C partial sums
        int KS, kbs;
        bound_mfma_plan(idx->C, idx->d, B, KS, kbs);
        const size_t need = (size_t)KS * B * idx->C * sizeof(float);
        if (need > CSV_STATIC_SCRATCH_BYTES) {
            csv_set_error("B=%d sequences x C=%d clusters need %zu bytes of partial sums, the static scratch holds %u: "
                          "use csv_bounds with a workspace", B, idx->C, need, CSV_STATIC_SCRATCH_BYTES);
            return CSV_ESHAPE;
        }
        void* p = nullptr;
        const int rc = static_scratch(dev, &p);
        if (rc) return rc;
        a.bound_partial = (float*)p;
    }
    return launch_bounds_kernel(a, d_U, d_hnorm, 0, (hipStream_t)stream);
}

extern "C" int csv_full_logits(csv_workspace* ws, const csv_index* idx, const uint16_t* d_h, int B, float* d_logits,
                               void* stream) {
    int rc = check_pair(ws, idx, d_h, B);
    if (rc) return rc;
    if (!d_logits) { csv_set_error("null d_logits"); return CSV_EINVAL; }
    return launch_full(idx, d_h, ws->all_list, nullptr, B, d_logits, idx->V, 1, ws->fb_logits, (hipStream_t)stream);
}

extern "C" int csv_decode_step(csv_workspace* ws, const csv_index* idx, const uint16_t* d_h, int B,
                               const csv_step_params* p, const csv_step_out* o, void* stream) {
    int rc = check_pair(ws, idx, d_h, B);
    if (rc) return rc;
    if (!p || !o) { csv_set_error("null params or out"); return CSV_EINVAL; }
    const bool use_k = p->k >= 1, use_s = p->eps > 0.f;
    if (!use_k && !use_s) { csv_set_error("both certificates disabled (k=%d, eps=%g)", p->k, (double)p->eps); return CSV_EINVAL; }
    if (p->k < 0 || p->k > CSV_MAX_K || p->k > idx->V) { csv_set_error("k=%d outside 0..min(V,%d)", p->k, CSV_MAX_K); return CSV_EINVAL; }
    if (p->K_max_rows < 0 || p->K_max_rows > ws->K_cap) { csv_set_error("K_max_rows=%d exceeds workspace capacity %d", p->K_max_rows, ws->K_cap); return CSV_EINVAL; }
    if (p->combine != CSV_COMBINE_ALL && p->combine != CSV_COMBINE_ANY) { csv_set_error("bad combine=%d", p->combine); return CSV_EINVAL; }
    const int max_rounds = p->max_rounds == 0 ? 2 : p->max_rounds;
    if (max_rounds < 2 || max_rounds > CSV_MAX_ROUNDS) { csv_set_error("max_rounds=%d outside 2..%d", p->max_rounds, CSV_MAX_ROUNDS); return CSV_EINVAL; }
    if (p->delta_clusters < 0) { csv_set_error("delta_clusters=%d is negative", p->delta_clusters); return CSV_EINVAL; }
    if (!o->d_lse || !o->d_flags || !o->d_n_rows || !o->d_n_clusters || (use_k && (!o->d_ids || !o->d_logits))) {
        csv_set_error("null output buffer");
        return CSV_EINVAL;
    }
    hipStream_t st = (hipStream_t)stream;
    StepArgs a;
    fill_args(a, ws, idx);
    a.B = B; a.h = d_h; a.k = p->k; a.K_max = p->K_max_rows; a.combine = p->combine; a.use_k = use_k; a.use_s = use_s;
    if (!use_s) a.lam = -INFINITY;
    else if (p->eps >= 1.f) a.lam = INFINITY;
    else a.lam = (float)log((double)p->eps / (1.0 - (double)p->eps));
    a.max_rounds = max_rounds; a.delta_clusters = p->delta_clusters; a.relax = p->relax != 0;
    if (!(p->top_p >= 0.f && p->top_p <= 1.f)) { csv_set_error("top_p=%g outside 0..1", (double)p->top_p); return CSV_EINVAL; }
    a.top_p = p->top_p;
    if (!use_s) a.lam2 = -INFINITY;
    else if (2.0 * (double)p->eps >= 1.0) a.lam2 = INFINITY;
    else a.lam2 = (float)log(2.0 * (double)p->eps / (1.0 - 2.0 * (double)p->eps));
    a.out = *o;

    hipEvent_t* ev = nullptr;
    if (ws->prof_on && ws->prof_n < ws->prof_cap) ev = ws->prof_ev + (size_t)ws->prof_n++ * (CSV_PROFILE_STAGES + 1);
#define CSV_MARK(i) do { if (ev) CSV_HIP(hipEventRecord(ev[i], st)); } while (0)
    CSV_MARK(0);
    rc = launch_bounds_kernel(a, ws->U, ws->hnorm, 1, st);
    if (rc) return rc;
    CSV_MARK(1);
    FullArgs f;
    f.V = idx->V; f.d = idx->d; f.Wp = idx->Wp; f.bp = idx->bp; f.perm = idx->perm; f.h = d_h;
    f.list = ws->fb_list; f.n_ptr = nullptr; f.n_fixed = 0; f.out = ws->fb_logits; f.out_stride = idx->V; f.scatter = 0;
    if (p->schedule == CSV_SCHEDULE_ALG1) {
        // Algorithm 1's own order: one block per sequence opens one cluster per iteration; then the fallback launches
        const size_t general = (size_t)ws->Npad * 8 + (size_t)ws->C * 8 + 8;
        const size_t h_off = (ALG1_CL_OFF + general + 15) / 16 * 16;
        const size_t lds = h_off + (size_t)idx->d * 2;
        if (lds + sizeof(SeqShared) + 256 > 160u * 1024u) {
            csv_set_error("schedule=ALG1: C=%d, d=%d need %zu bytes of LDS per block, more than a compute unit has", idx->C, idx->d, lds);
            return CSV_ESHAPE;
        }
        if (p->max_rounds > 2 || p->delta_clusters != 0 || p->relax) {
            csv_set_error("schedule=ALG1 has no fallback levels (max_rounds, delta_clusters, relax must be 0)");
            return CSV_EINVAL;
        }
        CSV_HIP(raise_lds(ws->device, K_ALG1, (const void*)alg1_kernel, lds));
        alg1_kernel<<<B, SEQ_THREADS, lds, st>>>(a, (int)(h_off / 16));
        CSV_LAUNCH_CHECK("alg1_kernel");
        CSV_MARK(2);
        if (B > FULL_G) {
            fb_product_mfma_kernel<<<ws->tail_grid, MFMA_THREADS, MFMA_LDS, st>>>(a, f);
            CSV_LAUNCH_CHECK("fb_product_mfma_kernel");
        } else {
            fb_product_kernel<<<ws->tail_grid, TAIL_THREADS, (size_t)FULL_G * idx->d * 2, st>>>(a, f);
            CSV_LAUNCH_CHECK("fb_product_kernel");
        }
        fb_topk_kernel<<<dim3(ws->n_chunks, B), SEQ_THREADS, (size_t)CAND_OFF + CAND_BYTES, st>>>(a);
        CSV_LAUNCH_CHECK("fb_topk_kernel");
        fb_final_kernel<<<B, SEQ_THREADS, (size_t)CAND_OFF + CAND_BYTES, st>>>(a);
        CSV_LAUNCH_CHECK("fb_final_kernel");
        CSV_MARK(3);
        return CSV_OK;
    }
    if (p->schedule != CSV_SCHEDULE_ROUNDS) { csv_set_error("bad schedule=%d", p->schedule); return CSV_EINVAL; }
    // One launch per phase pays when the tail is needed (kernel boundaries instead of grid barriers: 30 % of a
    // step even at B = 1), the single kernel when it is not (one launch that returns at once instead of seven).
    // Unless the caller fixed the choice, follow the recent steps: the bound kernel keeps a bit per step in a
    // pinned host word, read here without synchronising (it may lag a few steps; either choice is correct).
    bool split, fb_launches = true;
    const unsigned history = (unsigned)*(volatile int*)ws->h_history;
    if (ws->split_min_B > 0) {
        split = B >= ws->split_min_B;
    } else {
        split = __builtin_popcount(history & 0xffu) >= 2;
        // the three fallback phases as launches of their own only while fallbacks occur; otherwise one launch
        // of the single kernel restricted to them, which returns at once when nobody fell back
        fb_launches = (history >> 16) != 0;         // any of the last 15 steps
    }
    // blocks per sequence in round 0: as many as stay resident together (a second wave of blocks would double the
    // kernel's time), at most ROUND0_NB_MAX, and no more than the largest possible seed prefix needs at
    // ROUND0_ROWS_PER_BLOCK rows a block (max(k,1) - 1 rows before its last cluster plus that cluster)
    const long long prefix_max = (long long)(p->k > 1 ? p->k : 1) - 1 + idx->n_max;
    int nb = ws->round0_capacity / B;
    nb = nb < 1 ? 1 : (nb > ROUND0_NB_MAX ? ROUND0_NB_MAX : nb);
    {
        const long long want = (prefix_max + ROUND0_ROWS_PER_BLOCK - 1) / ROUND0_ROWS_PER_BLOCK;
        if (want < nb) nb = (int)(want < 1 ? 1 : want);
    }
    // the tail's blocks ride in the round-0 launch when they all fit next to the round-0 blocks (one block per unit)
    const bool fused = !split && ws->fused_ok && nb * B * 2 <= ws->tail_grid;
    if (fused) {
        step_kernel<<<ws->tail_grid, SEQ_THREADS, ws->fused_lds, st>>>(a, f, nb);
        CSV_LAUNCH_CHECK("step_kernel");
    } else {
        round0_kernel<<<nb * B, SEQ_THREADS, round0_lds(ws), st>>>(a, nb);
        CSV_LAUNCH_CHECK("round0_kernel");
    }
    CSV_MARK(2);
    if (!fused) {
        if (!split) {
            // one launch that returns at once when no sequence needs it
            tail_kernel<<<ws->tail_grid, TAIL_THREADS, ws->tail_lds, st>>>(a, f, 0);
            CSV_LAUNCH_CHECK("tail_kernel");
        } else {
            const size_t hl = (size_t)2 * idx->d * 2;
            // Round 0 appears here only for seed prefixes that the round-0 kernel hands over.  A prefix holds fewer
            // than max(k,1) rows before its last cluster, so with small clusters that cannot happen: no launches.
            const long long cap = (long long)nb * (SEQ_THREADS / 64) * ROUND0_ROWS_PER_WAVE;
            const bool may_hand_over = prefix_max > (cap < STAGE_CAP ? cap : STAGE_CAP) || (idx->d >> 3) > ROUND0_HREG * SEQ_THREADS;
            for (int r = may_hand_over ? 0 : 1; r < max_rounds; ++r) {
                round_gemv_kernel<<<ws->tail_grid, TAIL_THREADS, hl, st>>>(a, r);   // more blocks measured slower
                CSV_LAUNCH_CHECK("round_gemv_kernel");
                round_cert_kernel<<<dim3(B, ws->sp_chunks), SEQ_THREADS, cert_lds(ws), st>>>(a, r);
                CSV_LAUNCH_CHECK("round_cert_kernel");
            }
            if (fb_launches) {
                if (B > FULL_G) {
                    fb_product_mfma_kernel<<<ws->tail_grid, MFMA_THREADS, MFMA_LDS, st>>>(a, f);
                    CSV_LAUNCH_CHECK("fb_product_mfma_kernel");
                } else {
                    fb_product_kernel<<<ws->tail_grid, TAIL_THREADS, (size_t)FULL_G * idx->d * 2, st>>>(a, f);
                    CSV_LAUNCH_CHECK("fb_product_kernel");
                }
                fb_topk_kernel<<<dim3(ws->n_chunks, B), SEQ_THREADS, (size_t)CAND_OFF + CAND_BYTES, st>>>(a);
                CSV_LAUNCH_CHECK("fb_topk_kernel");
                fb_final_kernel<<<B, SEQ_THREADS, (size_t)CAND_OFF + CAND_BYTES, st>>>(a);
                CSV_LAUNCH_CHECK("fb_final_kernel");
            } else {
                tail_kernel<<<ws->tail_grid, TAIL_THREADS, ws->tail_lds, st>>>(a, f, 1);
                CSV_LAUNCH_CHECK("tail_kernel");
            }
        }
    }
    CSV_MARK(3);
#undef CSV_MARK
    return CSV_OK;
}

extern "C" int csv_workspace_set_tail_split(csv_workspace* ws, int min_batch) {
    if (!ws) { csv_set_error("null workspace"); return CSV_EINVAL; }
    if (min_batch < 0) { csv_set_error("min_batch=%d is negative", min_batch); return CSV_EINVAL; }
    ws->split_min_B = min_batch;
    return CSV_OK;
}

extern "C" int csv_workspace_set_spin_limit(csv_workspace* ws, int polls) {
    if (!ws) { csv_set_error("null workspace"); return CSV_EINVAL; }
    if (polls < 0) { csv_set_error("polls=%d is negative", polls); return CSV_EINVAL; }
    ws->spin_limit = polls == 0 ? TAIL_SPIN_LIMIT : polls;
    return CSV_OK;
}

// ------------------------------------------------------------------------------------------------ stage timing
static void profile_release(csv_workspace* ws) {
    if (ws->prof_ev) {
        for (size_t i = 0; i < (size_t)ws->prof_cap * (CSV_PROFILE_STAGES + 1); ++i)
            if (ws->prof_ev[i]) (void)hipEventDestroy(ws->prof_ev[i]);
        free(ws->prof_ev);
    }
    ws->prof_ev = nullptr;
    ws->prof_cap = ws->prof_n = ws->prof_on = 0;
}

extern "C" int csv_profile_begin(csv_workspace* ws, int max_steps) {
    if (!ws || max_steps < 1 || max_steps > (1 << 16)) { csv_set_error("bad workspace or max_steps"); return CSV_EINVAL; }
    profile_release(ws);
    const size_t n = (size_t)max_steps * (CSV_PROFILE_STAGES + 1);
    ws->prof_ev = (hipEvent_t*)calloc(n, sizeof(hipEvent_t));
    if (!ws->prof_ev) { csv_set_error("host allocation failed"); return CSV_ENOMEM; }
    ws->prof_cap = max_steps;
    for (size_t i = 0; i < n; ++i) {
        hipError_t e = hipEventCreate(&ws->prof_ev[i]);
        if (e != hipSuccess) {
            csv_set_error("hipEventCreate failed: %s", hipGetErrorString(e));
            profile_release(ws);
            return CSV_EHIP;
        }
    }
    ws->prof_on = 1;
    return CSV_OK;
}

extern "C" int csv_profile_end(csv_workspace* ws, float* h_stage_ms, int* h_steps) {
    if (!ws || !h_stage_ms || !h_steps) { csv_set_error("null argument"); return CSV_EINVAL; }
    for (int i = 0; i < CSV_PROFILE_STAGES; ++i) h_stage_ms[i] = 0.f;
    *h_steps = ws->prof_n;
    int rc = CSV_OK;
    for (int s = 0; s < ws->prof_n && rc == CSV_OK; ++s) {
        hipEvent_t* ev = ws->prof_ev + (size_t)s * (CSV_PROFILE_STAGES + 1);
        hipError_t e = hipEventSynchronize(ev[CSV_PROFILE_STAGES]);
        for (int i = 0; i < CSV_PROFILE_STAGES && e == hipSuccess; ++i) {
            float ms = 0.f;
            e = hipEventElapsedTime(&ms, ev[i], ev[i + 1]);
            h_stage_ms[i] += ms;
        }
        if (e != hipSuccess) {
            csv_set_error("event timing failed: %s", hipGetErrorString(e));
            rc = CSV_EHIP;
        }
    }
    profile_release(ws);
    return rc;
}

// ------------------------------------------------------------------------------------------------ adaptive budget
extern "C" int csv_kmax_init(csv_kmax_ctl* c, int K0, int K_min, int K_cap, double alpha, double rho_target, int literal) {
    if (!c) { csv_set_error("null controller"); return CSV_EINVAL; }
    if (K_min < 0 || K_cap < K_min || K0 < K_min || K0 > K_cap) { csv_set_error("need 0 <= K_min <= K0 <= K_cap (got %d, %d, %d)", K_min, K0, K_cap); return CSV_EINVAL; }
    if (!(alpha >= 0.0) || !(rho_target >= 0.0 && rho_target <= 1.0)) { csv_set_error("bad alpha=%g or rho_target=%g", alpha, rho_target); return CSV_EINVAL; }
    c->K_max = (double)K0; c->alpha = alpha; c->rho_target = rho_target; c->K_min = K_min; c->K_cap = K_cap; c->literal = literal != 0;
    return CSV_OK;
}

extern "C" int csv_kmax_update(csv_kmax_ctl* c, int n_fallback, int n_sequences) {
    if (!c) { csv_set_error("null controller"); return CSV_EINVAL; }
    if (n_sequences < 1 || n_fallback < 0 || n_fallback > n_sequences) { csv_set_error("bad counts %d of %d", n_fallback, n_sequences); return CSV_EINVAL; }
    const double rho = (double)n_fallback / (double)n_sequences;
    const double err = c->literal ? (c->rho_target - rho) : (rho - c->rho_target);
    double K = c->K_max * (1.0 + c->alpha * err);
    // the state itself stays inside the range, so a long run at one end does not have to be unwound
    if (K < (double)c->K_min) K = (double)c->K_min;
    if (K > (double)c->K_cap) K = (double)c->K_cap;
    c->K_max = K;
    return (int)floor(K);
}
