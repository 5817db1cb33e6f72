// Offline preprocessing: Lloyd's k-means over the rows of W, cluster metadata (centroid, radius, bias maximum)
// and the row permutation that makes every cluster contiguous (Section III-A.1; Section IV "Offline Preprocessing").
// Off the per-step hot path: clarity over speed, float64 accumulation for the metadata.
#include "csv_common.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

// ------------------------------------------------------------------------------------------------ kernels
// W'[r] = W[perm[r]], b'[r] = b[perm[r]] (0 without bias).  One block per permuted row.
__global__ __launch_bounds__(256) void gather_rows_kernel(const uint16_t* __restrict__ W, const float* __restrict__ b,
                                                          const int32_t* __restrict__ perm, int V, int d,
                                                          uint16_t* __restrict__ Wp, float* __restrict__ bp) {
    const int r = blockIdx.x;
    if (r >= V) return;
    const int src = perm[r];
    const uint4* s = reinterpret_cast<const uint4*>(W + (size_t)src * d);
    uint4* t = reinterpret_cast<uint4*>(Wp + (size_t)r * d);
    for (int i = threadIdx.x; i < (d >> 3); i += 256) t[i] = s[i];
    if (threadIdx.x == 0) bp[r] = b ? b[src] : 0.f;
}

// mu_c = mean of the cluster's rows, accumulated in float64 row by row, stored as float32.
// An empty cluster keeps its centroid (Lloyd) or is zeroed (final metadata).
__global__ __launch_bounds__(256) void centroid_kernel(const uint16_t* __restrict__ Wp, const int32_t* __restrict__ off, int d,
                                                       int zero_empty, float* __restrict__ mu) {
    const int c = blockIdx.x;
    const int col = blockIdx.y * 256 + threadIdx.x;
    if (col >= d) return;
    const int r0 = off[c], r1 = off[c + 1];
    if (r1 == r0) {
        if (zero_empty) mu[(size_t)c * d + col] = 0.f;
        return;
    }
    double sum = 0.0;
    for (int r = r0; r < r1; ++r) sum += (double)__uint_as_float((uint32_t)Wp[(size_t)r * d + col] << 16);
    mu[(size_t)c * d + col] = (float)(sum / (double)(r1 - r0));
}

__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, CSV_WAVE);
    return v;
}

// R_c = max_i ||W_i - mu_c||_2 to the stored float32 centroid, in float64; stored radius
// roundup_f32(R_c (1+rho) + rho ||mu_c||); bias maximum; ln n_c.
// Pass 1, one wave per permuted row (so a cluster of any size is spread over the whole device): squared distance in
// float64, folded into d2max[c] with an integer atomic max (non-negative doubles order like their bit patterns).
__global__ __launch_bounds__(256) void row_dist_kernel(const uint16_t* __restrict__ Wp, const int32_t* __restrict__ off,
                                                       const float* __restrict__ mu, int V, int d, int C,
                                                       unsigned long long* __restrict__ d2max, double* __restrict__ d2row) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= V) return;
    int lo = 0, hi = C;                       // cluster of the row: largest c with off[c] <= r
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= r) lo = mid; else hi = mid;
    }
    const uint4* w = reinterpret_cast<const uint4*>(Wp + (size_t)r * d);
    const float4* m = reinterpret_cast<const float4*>(mu + (size_t)lo * d);
    double acc = 0.0;
    for (int q = lane; q < (d >> 3); q += 64) {
        const uint4 x = w[q];
        const float4 m0 = m[2 * q], m1 = m[2 * q + 1];
        const uint32_t xs[4] = {x.x, x.y, x.z, x.w};
        const float ms[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const double d0 = (double)__uint_as_float(xs[e] << 16) - (double)ms[2 * e];
            const double d1 = (double)__uint_as_float(xs[e] & 0xffff0000u) - (double)ms[2 * e + 1];
            acc = fma(d0, d0, acc);
            acc = fma(d1, d1, acc);
        }
    }
    acc = wave_sum_d(acc);
    if (lane == 0) {
        atomicMax(&d2max[lo], (unsigned long long)__double_as_longlong(acc));
        if (d2row) d2row[r] = acc;          // squared distance of every row, for the bias table
    }
}

// Top-m bias table of one cluster (one block per cluster): the m-1 rows with the largest bias (equal biases: the
// earlier permuted row, i.e. the smaller token id) get entries of their own (distance to the centroid, bias); the
// remaining rows share one entry (their largest distance, their largest bias).  Radii are stored like R_c:
// roundup_f32(r (1+rho) + rho ||mu_c||).  Unused entries are (0, -inf).
__global__ __launch_bounds__(256) void bias_table_kernel(const float* __restrict__ bp, const int32_t* __restrict__ off,
                                                         const float* __restrict__ mu, int d, double rho, int m,
                                                         const double* __restrict__ d2row, float2* __restrict__ bt) {
    __shared__ float sb[256];
    __shared__ int si[256];
    __shared__ double sd[256];
    __shared__ int picked[CSV_MAX_BIAS_TABLE];
    __shared__ double mun;
    const int c = blockIdx.x, tid = threadIdx.x;
    const int r0 = off[c], r1 = off[c + 1], n = r1 - r0;
    float2* out = bt + (size_t)c * m;
    for (int j = tid; j < m; j += 256) out[j] = make_float2(0.f, -INFINITY);
    if (n == 0) return;
    {
        double acc = 0.0;
        for (int j = tid; j < d; j += 256) acc += (double)mu[(size_t)c * d + j] * (double)mu[(size_t)c * d + j];
        sd[tid] = acc;
        __syncthreads();
        for (int o = 128; o > 0; o >>= 1) {
            if (tid < o) sd[tid] += sd[tid + o];
            __syncthreads();
        }
        if (tid == 0) mun = sqrt(sd[0]);
        __syncthreads();
    }
    auto store = [&](int slot, double d2, float bias) {
        const double x = sqrt(d2) * (1.0 + rho) + rho * mun;
        float y = (float)x;
        if ((double)y < x) y = nextafterf(y, INFINITY);
        out[slot] = make_float2(y, bias);
    };
    const int ne = min(m - 1, n);
    for (int e = 0; e < ne; ++e) {
        // arg-max of (bias, -row) over the rows not picked yet
        float bb = -INFINITY;
        int bi = 0x7fffffff;
        for (int r = r0 + tid; r < r1; r += 256) {
            bool taken = false;
            for (int q = 0; q < e; ++q) taken |= picked[q] == r;
            const float v = bp[r];
            if (!taken && (v > bb || (v == bb && r < bi))) {
                bb = v;
                bi = r;
            }
        }
        sb[tid] = bb;
        si[tid] = bi;
        __syncthreads();
        for (int o = 128; o > 0; o >>= 1) {
            if (tid < o) {
                const float v = sb[tid + o];
                const int i = si[tid + o];
                if (v > sb[tid] || (v == sb[tid] && i < si[tid])) {
                    sb[tid] = v;
                    si[tid] = i;
                }
            }
            __syncthreads();
        }
        if (tid == 0) {
            picked[e] = si[0];
            store(e, d2row[si[0]], sb[0]);
        }
        __syncthreads();
    }
    if (n > ne) {       // the rest: largest distance and largest bias among the rows not picked
        float bb = -INFINITY;
        double dd = 0.0;
        for (int r = r0 + tid; r < r1; r += 256) {
            bool taken = false;
            for (int q = 0; q < ne; ++q) taken |= picked[q] == r;
            if (!taken) {
                bb = fmaxf(bb, bp[r]);
                dd = fmax(dd, d2row[r]);
            }
        }
        sb[tid] = bb;
        sd[tid] = dd;
        __syncthreads();
        for (int o = 128; o > 0; o >>= 1) {
            if (tid < o) {
                sb[tid] = fmaxf(sb[tid], sb[tid + o]);
                sd[tid] = fmax(sd[tid], sd[tid + o]);
            }
            __syncthreads();
        }
        if (tid == 0) store(ne, sd[0], sb[0]);
    }
}

// Pass 2, one block per cluster: bias maximum, ||mu_c||, the stored radius and ln n_c.
__global__ __launch_bounds__(256) void radius_finish_kernel(const float* __restrict__ bp, const int32_t* __restrict__ off,
                                                            const float* __restrict__ mu, int d, double rho,
                                                            const unsigned long long* __restrict__ d2max,
                                                            float* __restrict__ R, float* __restrict__ bmax,
                                                            float* __restrict__ lnn) {
    __shared__ float wb[4];
    __shared__ double wm[4];
    const int c = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r0 = off[c], r1 = off[c + 1];
    const float* m = mu + (size_t)c * d;
    float bm = -INFINITY;
    for (int r = r0 + tid; r < r1; r += 256) bm = fmaxf(bm, bp[r]);
    bm = wave_max(bm);
    double acc = 0.0;
    for (int j = tid; j < d; j += 256) acc += (double)m[j] * (double)m[j];
    acc = wave_sum_d(acc);
    if (lane == 0) {
        wb[wave] = bm;
        wm[wave] = acc;
    }
    __syncthreads();
    if (tid == 0) {
        const int n = r1 - r0;
        if (n == 0) {
            R[c] = 0.f;
            bmax[c] = -INFINITY;
            lnn[c] = -INFINITY;
        } else {
            const double mun2 = (wm[0] + wm[1]) + (wm[2] + wm[3]);
            const double d2 = __longlong_as_double((long long)d2max[c]);
            const double x = sqrt(d2) * (1.0 + rho) + rho * sqrt(mun2);
            float y = (float)x;
            if ((double)y < x) y = nextafterf(y, INFINITY);
            R[c] = y;
            bmax[c] = fmaxf(fmaxf(wb[0], wb[1]), fmaxf(wb[2], wb[3]));
            lnn[c] = (float)log((double)n);
        }
    }
}

// Lloyd assignment: labels[i] = argmin_c ||W_i - mu_c||^2, ties to the smaller cluster id.
// ||W_i - mu_c||^2 = ||W_i||^2 - 2 <W_i,mu_c> + ||mu_c||^2 and the first term does not depend on c, so the work is the
// dense contraction [V x d] . [d x C]: v_mfma_f32_16x16x32_bf16 with the rows of W (bf16) as one operand and the float32
// centroids, split exactly into three bf16 pieces (three MFMAs per k-block give float32-exact products), as the other.
// Block = 8 waves = 128 rows x AS_NT*16 clusters; a wave owns 16 rows and keeps their AS_NT accumulator tiles over the
// whole of K.  The centroid pieces are shared by the 8 waves: they are split while they are staged into LDS, one K
// chunk at a time, already in fragment order; the rows of W go straight from global memory to registers.
// Accumulator register r of lane (li, g) is [row 4g + r][cluster li]: the arg-min over a tile's 16 clusters is a
// reduction inside a 16-lane DPP row.  Each block writes, per row, the best (distance, cluster) of its cluster group;
// assign_reduce_kernel picks the best over the groups.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 as_bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float as_floatx4_t;
#define CSV_ANGLE_SLACK (1.0 / 4096.0)     // added to every angular radius (radians), next to the relative slack
#define AS_NT 4                 // cluster tiles of 16 per block
#define AS_KC 256               // K chunk staged in LDS: AS_NT*16 clusters x 3 pieces x AS_KC x 2 bytes = 96 KB
#define AS_THREADS 512
#define AS_LDS (AS_NT * 16 * 3 * AS_KC * 2)

__device__ __forceinline__ void as_split3(const float4& x0, const float4& x1, uint4& hi, uint4& mid, uint4& lo) {
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
// minimum over the 16 lanes of a DPP row (lanes 16g .. 16g+15); every lane of the row gets it
__device__ __forceinline__ unsigned row16_min_u(unsigned v) {
    v = min(v, (unsigned)dpp_move<0xB1, 0xf>((int)v, (int)v));    // quad_perm [1,0,3,2]
    v = min(v, (unsigned)dpp_move<0x4E, 0xf>((int)v, (int)v));    // quad_perm [2,3,0,1]
    v = min(v, (unsigned)dpp_move<0x141, 0xf>((int)v, (int)v));   // row_half_mirror
    v = min(v, (unsigned)dpp_move<0x140, 0xf>((int)v, (int)v));   // row_mirror
    return v;
}

// unit != 0 (spherical clustering): every direction counts as of length one, so the arg-min is the largest cosine
__global__ __launch_bounds__(256) void centroid_norm_kernel(const float* __restrict__ mu, int d, int unit, float* __restrict__ cn) {
    __shared__ double red[4];
    const int c = blockIdx.x, tid = threadIdx.x;
    if (unit) {
        if (tid == 0) cn[c] = 1.f;
        return;
    }
    double acc = 0.0;
    for (int j = tid; j < d; j += 256) acc += (double)mu[(size_t)c * d + j] * (double)mu[(size_t)c * d + j];
    acc = wave_sum_d(acc);
    if ((tid & 63) == 0) red[tid >> 6] = acc;
    __syncthreads();
    if (tid == 0) cn[c] = (float)((red[0] + red[1]) + (red[2] + red[3]));
}

// grid (cluster groups, row tiles of 128).  cand_key[row * G + group] = monotone key of the best distance, cand_c = its cluster.
__global__ __launch_bounds__(AS_THREADS) void assign_mfma_kernel(const uint16_t* __restrict__ W, const float* __restrict__ mu,
                                                                 const float* __restrict__ cn, int V, int d, int C, int G,
                                                                 unsigned* __restrict__ cand_key, int32_t* __restrict__ cand_c) {
    extern __shared__ uint4 as_lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, g = lane >> 4;
    const int group = blockIdx.x, cb = group * AS_NT * 16;
    const int r0 = blockIdx.y * 128 + wave * 16;
    const int nq = d >> 3;                                   // 16-byte pieces per row of W
    const uint4* ap = reinterpret_cast<const uint4*>(W + (size_t)min(r0 + li, V - 1) * d);
    as_floatx4_t acc[AS_NT];
#pragma unroll
    for (int t = 0; t < AS_NT; ++t) acc[t] = as_floatx4_t{0.f, 0.f, 0.f, 0.f};
    const uint4 zero = make_uint4(0, 0, 0, 0);
    for (int k0 = 0; k0 < d; k0 += AS_KC) {
        __syncthreads();
        // stage: piece (cluster cl of the group, q-th run of 8 k values of the chunk) -> three fragments.
        // fragment slot of (kb = q / 4, piece s, tile t) is ((kb * 3 + s) * AS_NT + t) * 64 + (q % 4) * 16 + (cl % 16)
        for (int p = tid; p < AS_NT * 16 * (AS_KC / 8); p += AS_THREADS) {
            const int cl = p / (AS_KC / 8), q = p - cl * (AS_KC / 8);
            const int c = cb + cl, k = k0 + q * 8;
            uint4 hi = zero, mid = zero, lo = zero;
            if (c < C && k < d) {                            // d is a multiple of 8: the eight values are all in or all out
                const float4* src = reinterpret_cast<const float4*>(mu + (size_t)c * d + k);
                as_split3(src[0], src[1], hi, mid, lo);
            }
            const int base = (q >> 2) * 3 * AS_NT * 64 + (cl >> 4) * 64 + (q & 3) * 16 + (cl & 15);
            as_lds[base] = hi;
            as_lds[base + AS_NT * 64] = mid;
            as_lds[base + 2 * AS_NT * 64] = lo;
        }
        __syncthreads();
#pragma unroll 2
        for (int kb = 0; kb < AS_KC / 32; ++kb) {
            const int q = ((k0 + kb * 32) >> 3) + g;         // this lane's 16-byte piece of its row
            const uint4 av = ap[min(q, nq - 1)];
            const as_bf16x8_t A = __builtin_bit_cast(as_bf16x8_t, q < nq ? av : zero);
#pragma unroll
            for (int sp = 0; sp < 3; ++sp)
#pragma unroll
                for (int t = 0; t < AS_NT; ++t) {
                    const uint4 Bv = as_lds[((kb * 3 + sp) * AS_NT + t) * 64 + lane];
                    acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A, __builtin_bit_cast(as_bf16x8_t, Bv), acc[t], 0, 0, 0);
                }
        }
    }
    // ||mu_c||^2 - 2 <W_i,mu_c> for row 4g + r and cluster cb + 16t + li; best over the tiles, then over the 16 lanes of the row
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        unsigned bk = 0xffffffffu;
        int bc = 0x7fffffff;
#pragma unroll
        for (int t = 0; t < AS_NT; ++t) {
            const int c = cb + 16 * t + li;
            const float v = c < C ? cn[c] - 2.f * acc[t][r] : INFINITY;
            const unsigned kx = c < C ? fkey(v + 0.0f) : 0xffffffffu;
            if (kx < bk) {                                   // tiles in ascending cluster order: a tie keeps the smaller id
                bk = kx;
                bc = c;
            }
        }
        const unsigned m = row16_min_u(bk);
        const int cm = (int)row16_min_u(bk == m ? (unsigned)bc : 0x7fffffffu);
        const int row = r0 + 4 * g + r;
        if (li == 0 && row < V) {
            cand_key[(size_t)row * G + group] = m;
            cand_c[(size_t)row * G + group] = cm;
        }
    }
}

__global__ __launch_bounds__(256) void assign_reduce_kernel(const unsigned* __restrict__ cand_key, const int32_t* __restrict__ cand_c,
                                                            int V, int G, int32_t* __restrict__ labels) {
    const int row = blockIdx.x * 256 + threadIdx.x;
    if (row >= V) return;
    unsigned bk = 0xffffffffu;
    int bc = 0x7fffffff;
    for (int gq = 0; gq < G; ++gq) {                         // groups in ascending cluster order: a tie keeps the smaller id
        const unsigned kx = cand_key[(size_t)row * G + gq];
        if (kx < bk) {
            bk = kx;
            bc = cand_c[(size_t)row * G + gq];
        }
    }
    labels[row] = bc;
}

// mu[c] = row init_rows[c] of W widened to float32 (starting centroids).
__global__ __launch_bounds__(256) void init_centroid_kernel(const uint16_t* __restrict__ W, const int32_t* __restrict__ rows,
                                                            int d, float* __restrict__ mu) {
    const int c = blockIdx.x;
    const uint16_t* w = W + (size_t)rows[c] * d;
    for (int j = threadIdx.x; j < d; j += 256) mu[(size_t)c * d + j] = __uint_as_float((uint32_t)w[j] << 16);
}

// ------------------------------------------------------------------------------------------------ spherical clustering
// (Section III, "Advanced Theoretical Improvements", spherical clustering metrics)
// ||W_r|| of every row (original or permuted order, whichever W is), float64.  One wave per row.
__global__ __launch_bounds__(256) void row_norm_kernel(const uint16_t* __restrict__ W, int V, int d, double* __restrict__ nrm) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= V) return;
    const uint4* w = reinterpret_cast<const uint4*>(W + (size_t)r * d);
    double acc = 0.0;
    for (int q = lane; q < (d >> 3); q += 64) {
        const uint4 x = w[q];
        const uint32_t xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const double a0 = (double)__uint_as_float(xs[e] << 16), a1 = (double)__uint_as_float(xs[e] & 0xffff0000u);
            acc = fma(a0, a0, acc);
            acc = fma(a1, a1, acc);
        }
    }
    acc = wave_sum_d(acc);
    if (lane == 0) nrm[r] = sqrt(acc);
}

// Starting directions: row init_rows[c] of W, normalised, as float32.
__global__ __launch_bounds__(256) void init_direction_kernel(const uint16_t* __restrict__ W, const int32_t* __restrict__ rows,
                                                             const double* __restrict__ nrm, int d, float* __restrict__ mu) {
    const int c = blockIdx.x;
    const uint16_t* w = W + (size_t)rows[c] * d;
    const double nr = nrm[rows[c]];
    for (int j = threadIdx.x; j < d; j += 256) {
        const double v = (double)__uint_as_float((uint32_t)w[j] << 16);
        mu[(size_t)c * d + j] = (float)(nr > 0.0 ? v / nr : v);
    }
}

// sums[c][col] = sum over the cluster's rows of W'[r][col] / ||W'[r]||, float64, row by row (nrm in permuted order).
__global__ __launch_bounds__(256) void direction_sum_kernel(const uint16_t* __restrict__ Wp, const int32_t* __restrict__ off,
                                                            const double* __restrict__ nrm, int d, double* __restrict__ sums) {
    const int c = blockIdx.x;
    const int col = blockIdx.y * 256 + threadIdx.x;
    if (col >= d) return;
    const int r0 = off[c], r1 = off[c + 1];
    double sum = 0.0;
    for (int r = r0; r < r1; ++r) {
        const double nr = nrm[r];
        const double v = (double)__uint_as_float((uint32_t)Wp[(size_t)r * d + col] << 16);
        sum += nr > 0.0 ? v / nr : v;
    }
    sums[(size_t)c * d + col] = sum;
}

// mu[c] = sums[c] / ||sums[c]|| as float32; an empty cluster keeps its direction (Lloyd) or is zeroed (final metadata).
__global__ __launch_bounds__(256) void direction_finish_kernel(const double* __restrict__ sums, const int32_t* __restrict__ off, int d,
                                                               int zero_empty, float* __restrict__ mu) {
    __shared__ double red[4];
    const int c = blockIdx.x, tid = threadIdx.x;
    if (off[c + 1] == off[c]) {
        if (zero_empty)
            for (int j = tid; j < d; j += 256) mu[(size_t)c * d + j] = 0.f;
        return;
    }
    double acc = 0.0;
    for (int j = tid; j < d; j += 256) acc += sums[(size_t)c * d + j] * sums[(size_t)c * d + j];
    acc = wave_sum_d(acc);
    if ((tid & 63) == 0) red[tid >> 6] = acc;
    __syncthreads();
    const double nr = sqrt((red[0] + red[1]) + (red[2] + red[3]));
    for (int j = tid; j < d; j += 256) {
        const double v = sums[(size_t)c * d + j];
        mu[(size_t)c * d + j] = (float)(nr > 0.0 ? v / nr : v);
    }
}

// Per row (one wave): cosine to its cluster's stored direction and its norm, folded into per-cluster extremes with
// integer atomics: cosines are shifted by +2 (positive doubles order like their bit patterns).
// ext[c] = {min (cos + 2), max ||w||^2 bits, min ||w||^2 bits}
__global__ __launch_bounds__(256) void row_angle_kernel(const uint16_t* __restrict__ Wp, const int32_t* __restrict__ off,
                                                        const float* __restrict__ mu, int V, int d, int C,
                                                        unsigned long long* __restrict__ ext) {
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (r >= V) return;
    int lo = 0, hi = C;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (off[mid] <= r) lo = mid; else hi = mid;
    }
    const uint4* w = reinterpret_cast<const uint4*>(Wp + (size_t)r * d);
    const float4* m = reinterpret_cast<const float4*>(mu + (size_t)lo * d);
    double ww = 0.0, wm = 0.0, mm = 0.0;
    for (int q = lane; q < (d >> 3); q += 64) {
        const uint4 x = w[q];
        const float4 m0 = m[2 * q], m1 = m[2 * q + 1];
        const uint32_t xs[4] = {x.x, x.y, x.z, x.w};
        const float ms[8] = {m0.x, m0.y, m0.z, m0.w, m1.x, m1.y, m1.z, m1.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const double a0 = (double)__uint_as_float(xs[e] << 16), a1 = (double)__uint_as_float(xs[e] & 0xffff0000u);
            const double b0 = (double)ms[2 * e], b1 = (double)ms[2 * e + 1];
            ww = fma(a0, a0, ww); ww = fma(a1, a1, ww);
            wm = fma(a0, b0, wm); wm = fma(a1, b1, wm);
            mm = fma(b0, b0, mm); mm = fma(b1, b1, mm);
        }
    }
    ww = wave_sum_d(ww);
    wm = wave_sum_d(wm);
    mm = wave_sum_d(mm);
    if (lane == 0) {
        const double nw = sqrt(ww), nm = sqrt(mm);
        double cs = nw > 0.0 ? wm / (nw * (nm > 0.0 ? nm : 1.0)) : 1.0;
        cs = fmin(1.0, fmax(-1.0, cs));
        atomicMin(&ext[3 * lo], (unsigned long long)__double_as_longlong(cs + 2.0));
        atomicMax(&ext[3 * lo + 1], (unsigned long long)__double_as_longlong(ww));
        atomicMin(&ext[3 * lo + 2], (unsigned long long)__double_as_longlong(ww));
    }
}

// ang[c] = {cos, sin of the angular radius with slack, largest norm (1+slack) rounded up, smallest (1-slack) rounded down}
__global__ __launch_bounds__(256) void angular_finish_kernel(const int32_t* __restrict__ off, int C, double slack, double angle_slack,
                                                             const unsigned long long* __restrict__ ext, float4* __restrict__ ang) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= C) return;
    if (off[c + 1] == off[c]) {
        ang[c] = make_float4(1.f, 0.f, 0.f, 0.f);
        return;
    }
    const double mincos = __longlong_as_double((long long)ext[3 * c]) - 2.0;
    double theta = acos(fmin(1.0, fmax(-1.0, mincos)));
    const double pi = 3.14159265358979323846;
    theta = fmin(pi, theta * (1.0 + slack) + angle_slack);
    auto up = [](double x) { float y = (float)x; if ((double)y < x) y = nextafterf(y, INFINITY); return y; };
    auto down = [](double x) { float y = (float)x; if ((double)y > x) y = nextafterf(y, -INFINITY); return y; };
    const float ct = theta < pi ? down(cos(theta)) : -1.f;
    const float st = up(sin(theta));
    const double nmax = sqrt(__longlong_as_double((long long)ext[3 * c + 1])), nmin = sqrt(__longlong_as_double((long long)ext[3 * c + 2]));
    ang[c] = make_float4(ct, st, up(nmax * (1.0 + slack)), down(nmin * (1.0 - slack)));
}

// cmeta[c] = {off[c], off[c+1] - off[c], bits of ln n_c, 0}
__global__ __launch_bounds__(256) void pack_cmeta_kernel(const int32_t* __restrict__ off, const float* __restrict__ lnn, int C,
                                                         int4* __restrict__ cmeta) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c < C) cmeta[c] = make_int4(off[c], off[c + 1] - off[c], __float_as_int(lnn[c]), 0);
}

// ------------------------------------------------------------------------------------------------ host side
int csv_index_pack_cmeta(csv_index* x, hipStream_t st) {
    pack_cmeta_kernel<<<(x->C + 255) / 256, 256, 0, st>>>(x->off, x->lnn, x->C, x->cmeta);
    CSV_LAUNCH_CHECK("pack_cmeta_kernel");
    return CSV_OK;
}

static int check_shape(int V, int d, int C) {
    if (V < 1 || d < 8 || (d & 7) != 0) { csv_set_error("need V >= 1 and d a positive multiple of 8 (V=%d, d=%d)", V, d); return CSV_ESHAPE; }
    if (C < 1 || C > V || C > CSV_MAX_CLUSTERS) { csv_set_error("C=%d outside 1..min(V,%d)", C, CSV_MAX_CLUSTERS); return CSV_ESHAPE; }
    return CSV_OK;
}

int csv_index_alloc(int V, int d, int C, csv_index** out) {
    csv_index* x = (csv_index*)calloc(1, sizeof(csv_index));
    if (!x) { csv_set_error("host allocation failed"); return CSV_ENOMEM; }
    x->V = V; x->d = d; x->C = C;
    hipError_t e = hipGetDevice(&x->device);
    auto A = [&](void** p, size_t bytes) { if (e == hipSuccess) e = hipMalloc(p, bytes); };
    A((void**)&x->Wp, (size_t)V * d * 2); A((void**)&x->bp, (size_t)V * 4); A((void**)&x->perm, (size_t)V * 4);
    A((void**)&x->mu, (size_t)C * d * 4); A((void**)&x->R, (size_t)C * 4); A((void**)&x->bmax, (size_t)C * 4);
    A((void**)&x->n, (size_t)C * 4); A((void**)&x->off, (size_t)(C + 1) * 4); A((void**)&x->lnn, (size_t)C * 4);
    A((void**)&x->cmeta, (size_t)C * sizeof(int4));
    if (e != hipSuccess) {
        csv_set_error("index allocation failed: %s", hipGetErrorString(e));
        csv_index_free(x);
        return e == hipErrorOutOfMemory ? CSV_ENOMEM : CSV_EHIP;
    }
    *out = x;
    return CSV_OK;
}

extern "C" void csv_index_free(csv_index* x) {
    if (!x) return;
    void* ptrs[] = {x->Wp, x->bp, x->perm, x->mu, x->mu16, x->R, x->bmax, x->n, x->off, x->lnn, x->cmeta, x->bt, x->ang};
    for (void* p : ptrs)
        if (p) (void)hipFree(p);
    free(x);
}

extern "C" int csv_index_dims(const csv_index* x, int* V, int* d, int* C) {
    if (!x) { csv_set_error("null index"); return CSV_EINVAL; }
    if (V) *V = x->V;
    if (d) *d = x->d;
    if (C) *C = x->C;
    return CSV_OK;
}

// Centroids stored as bfloat16: mu is rounded in place (nearest even) and the 16-bit patterns go to mu16.
// check != 0: nothing is rounded; *bad is set when a value is not already a bfloat16.
__global__ __launch_bounds__(256) void centroid_bf16_kernel(float* __restrict__ mu, uint16_t* __restrict__ mu16, size_t n, int check,
                                                            int* __restrict__ bad) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const uint32_t u = __float_as_uint(mu[i]);
    if (check) {
        if (u & 0xffffu) *bad = 1;
        mu16[i] = (uint16_t)(u >> 16);
        return;
    }
    const uint32_t r = (u + 0x7fffu + ((u >> 16) & 1u)) & 0xffff0000u;
    mu[i] = __uint_as_float(r);
    mu16[i] = (uint16_t)(r >> 16);
}

static int store_centroids_bf16(csv_index* x, int check, hipStream_t st) {
    const size_t n = (size_t)x->C * x->d;
    if (!x->mu16 && hipMalloc((void**)&x->mu16, n * 2) != hipSuccess) { csv_set_error("out of device memory (bf16 centroids)"); return CSV_ENOMEM; }
    int* d_bad = nullptr;
    if (hipMalloc((void**)&d_bad, 4) != hipSuccess) { csv_set_error("out of device memory"); return CSV_ENOMEM; }
    int h_bad = 0;
    hipError_t e = hipMemsetAsync(d_bad, 0, 4, st);
    if (e == hipSuccess) {
        centroid_bf16_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(x->mu, x->mu16, n, check, d_bad);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipMemcpyAsync(&h_bad, d_bad, 4, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    (void)hipFree(d_bad);
    if (e != hipSuccess) { csv_set_error("bf16 centroid conversion failed: %s", hipGetErrorString(e)); return CSV_EHIP; }
    if (h_bad) {
        (void)hipFree(x->mu16);
        x->mu16 = nullptr;
        csv_set_error("centroids are not bfloat16 values: the radii of this index were not measured to rounded centroids");
        return CSV_EINVAL;
    }
    return CSV_OK;
}

extern "C" int csv_index_use_bf16_centroids(csv_index* x, void* stream) {
    if (!x) { csv_set_error("null index"); return CSV_EINVAL; }
    if (x->mu16) return CSV_OK;
    return store_centroids_bf16(x, 1, (hipStream_t)stream);
}

// labels -> sizes, offsets and the permutation (clusters in id order, tokens by ascending id inside a cluster)
static int layout_from_labels(const int32_t* labels, int V, int C, std::vector<int32_t>& n, std::vector<int32_t>& off,
                              std::vector<int32_t>& perm) {
    n.assign(C, 0);
    for (int i = 0; i < V; ++i) {
        if (labels[i] < 0 || labels[i] >= C) { csv_set_error("label %d of token %d outside 0..C-1", labels[i], i); return CSV_EINVAL; }
        n[labels[i]]++;
    }
    off.assign(C + 1, 0);
    for (int c = 0; c < C; ++c) off[c + 1] = off[c] + n[c];
    perm.resize(V);
    std::vector<int32_t> cur(off.begin(), off.end() - 1);
    for (int i = 0; i < V; ++i) perm[cur[labels[i]]++] = i;
    return CSV_OK;
}

static int upload_layout(csv_index* x, const std::vector<int32_t>& n, const std::vector<int32_t>& off,
                         const std::vector<int32_t>& perm, hipStream_t st) {
    CSV_HIP(hipMemcpyAsync(x->n, n.data(), (size_t)x->C * 4, hipMemcpyHostToDevice, st));
    CSV_HIP(hipMemcpyAsync(x->off, off.data(), (size_t)(x->C + 1) * 4, hipMemcpyHostToDevice, st));
    CSV_HIP(hipMemcpyAsync(x->perm, perm.data(), (size_t)x->V * 4, hipMemcpyHostToDevice, st));
    CSV_HIP(hipStreamSynchronize(st));   // the host vectors may go away after this
    return CSV_OK;
}

static int gather(csv_index* x, const uint16_t* d_W, const float* d_b, hipStream_t st) {
    gather_rows_kernel<<<x->V, 256, 0, st>>>(d_W, d_b, x->perm, x->V, x->d, x->Wp, x->bp);
    CSV_LAUNCH_CHECK("gather_rows_kernel");
    return CSV_OK;
}

extern "C" int csv_build_index(const uint16_t* d_W, const float* d_b, int V, int d, int C, const csv_build_opts* o,
                               void* stream, csv_index** out) {
    if (out) *out = nullptr;
    if (!d_W || !o || !out) { csv_set_error("null W, opts or out"); return CSV_EINVAL; }
    int rc = check_shape(V, d, C);
    if (rc) return rc;
    if (o->iters < 0 || !(o->radius_slack >= 0.f)) { csv_set_error("iters and radius_slack must be >= 0"); return CSV_EINVAL; }
    if (o->bias_table_m < 0 || o->bias_table_m > CSV_MAX_BIAS_TABLE) { csv_set_error("bias_table_m=%d outside 0..%d", o->bias_table_m, CSV_MAX_BIAS_TABLE); return CSV_EINVAL; }

    hipStream_t st = (hipStream_t)stream;
    csv_index* x = nullptr;
    rc = csv_index_alloc(V, d, C, &x);
    if (rc) return rc;
    int32_t* d_labels = nullptr;
    std::vector<int32_t> labels(V), n, off, perm;
    // scratch of the assignment: per row and cluster group the best (distance key, cluster); centroid norms
    unsigned* d_ckey = nullptr;
    int32_t* d_cc = nullptr;
    float* d_cn = nullptr;
    // spherical clustering: row norms in original and in permuted order, float64 sums of unit rows
    const int sph = o->spherical != 0;
    double *d_nrm = nullptr, *d_nrmp = nullptr, *d_sums = nullptr;
    auto free_scratch = [&]() {
        if (d_labels) (void)hipFree(d_labels);
        if (d_ckey) (void)hipFree(d_ckey);
        if (d_cc) (void)hipFree(d_cc);
        if (d_cn) (void)hipFree(d_cn);
        if (d_nrm) (void)hipFree(d_nrm);
        if (d_nrmp) (void)hipFree(d_nrmp);
        if (d_sums) (void)hipFree(d_sums);
    };
    auto fail = [&](int code) {
        free_scratch();
        csv_index_free(x);
        return code;
    };
    if (hipMalloc((void**)&d_labels, (size_t)V * 4) != hipSuccess) { csv_set_error("label buffer allocation failed"); return fail(CSV_ENOMEM); }
    const dim3 cgrid(C, (d + 255) / 256);
    if (sph) {
        if (o->centroid_bf16 || o->bias_table_m >= 2) { csv_set_error("spherical clustering takes neither bf16 centroids nor a bias table"); return fail(CSV_EINVAL); }
        if (hipMalloc((void**)&d_nrm, (size_t)V * 8) != hipSuccess || hipMalloc((void**)&d_nrmp, (size_t)V * 8) != hipSuccess ||
            hipMalloc((void**)&d_sums, (size_t)C * d * 8) != hipSuccess) { csv_set_error("out of device memory (spherical clustering scratch)"); return fail(CSV_ENOMEM); }
        row_norm_kernel<<<(V + 3) / 4, 256, 0, st>>>(d_W, V, d, d_nrm);
        if (hipGetLastError() != hipSuccess) { csv_set_error("launch of row_norm_kernel failed"); return fail(CSV_EHIP); }
    }
    const int G = (C + AS_NT * 16 - 1) / (AS_NT * 16);
    auto assign = [&]() -> int {
        if (!d_ckey) {
            if (hipMalloc((void**)&d_ckey, (size_t)V * G * 4) != hipSuccess || hipMalloc((void**)&d_cc, (size_t)V * G * 4) != hipSuccess ||
                hipMalloc((void**)&d_cn, (size_t)C * 4) != hipSuccess) { csv_set_error("out of device memory (assignment scratch)"); return CSV_ENOMEM; }
            CSV_HIP(hipFuncSetAttribute((const void*)assign_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, AS_LDS));
        }
        centroid_norm_kernel<<<C, 256, 0, st>>>(x->mu, d, sph, d_cn);
        CSV_LAUNCH_CHECK("centroid_norm_kernel");
        assign_mfma_kernel<<<dim3(G, (V + 127) / 128), AS_THREADS, AS_LDS, st>>>(d_W, x->mu, d_cn, V, d, C, G, d_ckey, d_cc);
        CSV_LAUNCH_CHECK("assign_mfma_kernel");
        assign_reduce_kernel<<<(V + 255) / 256, 256, 0, st>>>(d_ckey, d_cc, V, G, d_labels);
        CSV_LAUNCH_CHECK("assign_reduce_kernel");
        CSV_HIP(hipMemcpyAsync(labels.data(), d_labels, (size_t)V * 4, hipMemcpyDeviceToHost, st));
        CSV_HIP(hipStreamSynchronize(st));
        return CSV_OK;
    };
    if (o->h_init_labels) {
        memcpy(labels.data(), o->h_init_labels, (size_t)V * 4);
    } else {
        // seeding rule when the caller names no rows: C tokens evenly spread over the vocabulary, token floor(c V / C)
        std::vector<int32_t> seed(C);
        for (int c = 0; c < C; ++c) seed[c] = o->h_init_rows ? o->h_init_rows[c] : (int32_t)((long long)c * V / C);
        for (int c = 0; c < C; ++c)
            if (seed[c] < 0 || seed[c] >= V) { csv_set_error("init row %d outside 0..V-1", seed[c]); return fail(CSV_EINVAL); }
        // x->n doubles as the staging buffer for the starting rows
        if (hipMemcpy(x->n, seed.data(), (size_t)C * 4, hipMemcpyHostToDevice) != hipSuccess) { csv_set_error("copy of init rows failed"); return fail(CSV_EHIP); }
        if (sph) init_direction_kernel<<<C, 256, 0, st>>>(d_W, x->n, d_nrm, d, x->mu);
        else init_centroid_kernel<<<C, 256, 0, st>>>(d_W, x->n, d, x->mu);
        if ((rc = assign())) return fail(rc);
    }
    for (int it = 0;; ++it) {
        if ((rc = layout_from_labels(labels.data(), V, C, n, off, perm))) return fail(rc);
        if ((rc = upload_layout(x, n, off, perm, st))) return fail(rc);
        if ((rc = gather(x, d_W, d_b, st))) return fail(rc);
        const bool last = it == o->iters;
        if (sph) {
            row_norm_kernel<<<(V + 3) / 4, 256, 0, st>>>(x->Wp, V, d, d_nrmp);
            direction_sum_kernel<<<cgrid, 256, 0, st>>>(x->Wp, x->off, d_nrmp, d, d_sums);
            direction_finish_kernel<<<C, 256, 0, st>>>(d_sums, x->off, d, last ? 1 : 0, x->mu);
        } else {
            centroid_kernel<<<cgrid, 256, 0, st>>>(x->Wp, x->off, d, last ? 1 : 0, x->mu);
        }
        if (hipGetLastError() != hipSuccess) { csv_set_error("launch of the centroid kernels failed"); return fail(CSV_EHIP); }
        if (last) break;
        if ((rc = assign())) return fail(rc);
    }
    {
        int nmax = 1;
        for (int c = 0; c < C; ++c) nmax = n[c] > nmax ? n[c] : nmax;
        x->ln_nmax = (float)log((double)nmax);
        x->n_max = nmax;
    }
    if (o->centroid_bf16 && (rc = store_centroids_bf16(x, 0, st))) return fail(rc);
    unsigned long long* d_d2max = nullptr;
    double* d_d2row = nullptr;
    const int bt_m = o->bias_table_m >= 2 ? o->bias_table_m : 0;
    if (hipMalloc((void**)&d_d2max, (size_t)C * 8) != hipSuccess) { csv_set_error("out of device memory (radius scratch)"); return fail(CSV_ENOMEM); }
    if (bt_m && (hipMalloc((void**)&d_d2row, (size_t)V * 8) != hipSuccess || hipMalloc((void**)&x->bt, (size_t)C * bt_m * sizeof(float2)) != hipSuccess)) {
        (void)hipFree(d_d2max);
        if (d_d2row) (void)hipFree(d_d2row);
        csv_set_error("out of device memory (bias table)");
        return fail(CSV_ENOMEM);
    }
    x->bt_m = bt_m;
    bool launched = hipMemsetAsync(d_d2max, 0, (size_t)C * 8, st) == hipSuccess;
    if (launched) {
        row_dist_kernel<<<(V + 3) / 4, 256, 0, st>>>(x->Wp, x->off, x->mu, V, d, C, d_d2max, d_d2row);
        launched = hipGetLastError() == hipSuccess;
    }
    if (launched && bt_m) {
        bias_table_kernel<<<C, 256, 0, st>>>(x->bp, x->off, x->mu, d, (double)o->radius_slack, bt_m, d_d2row, x->bt);
        launched = hipGetLastError() == hipSuccess;
    }
    if (launched) {
        radius_finish_kernel<<<C, 256, 0, st>>>(x->bp, x->off, x->mu, d, (double)o->radius_slack, d_d2max, x->R, x->bmax, x->lnn);
        launched = hipGetLastError() == hipSuccess;
    }
    if (launched) launched = csv_index_pack_cmeta(x, st) == CSV_OK;
    unsigned long long* d_ext = nullptr;
    if (launched && sph) {          // angular metadata in place of the Euclidean radius (which stays unused)
        std::vector<unsigned long long> init((size_t)3 * C);
        for (int c = 0; c < C; ++c) {
            init[3 * c] = ~0ull;
            init[3 * c + 1] = 0ull;
            init[3 * c + 2] = ~0ull;
        }
        launched = hipMalloc((void**)&d_ext, (size_t)3 * C * 8) == hipSuccess && hipMalloc((void**)&x->ang, (size_t)C * sizeof(float4)) == hipSuccess &&
                   hipMemcpy(d_ext, init.data(), (size_t)3 * C * 8, hipMemcpyHostToDevice) == hipSuccess;
        if (launched) {
            row_angle_kernel<<<(V + 3) / 4, 256, 0, st>>>(x->Wp, x->off, x->mu, V, d, C, d_ext);
            angular_finish_kernel<<<(C + 255) / 256, 256, 0, st>>>(x->off, C, (double)o->radius_slack, CSV_ANGLE_SLACK, d_ext, x->ang);
            launched = hipGetLastError() == hipSuccess;
        }
    }
    const bool synced = hipStreamSynchronize(st) == hipSuccess;
    if (d_ext) (void)hipFree(d_ext);
    (void)hipFree(d_d2max);
    if (d_d2row) (void)hipFree(d_d2row);
    if (!launched) { csv_set_error("launch of the radius kernels failed"); return fail(CSV_EHIP); }
    if (!synced) { csv_set_error("index build failed on the device: %s", hipGetErrorString(hipGetLastError())); return fail(CSV_EHIP); }
    free_scratch();
    *out = x;
    return CSV_OK;
}

extern "C" int csv_index_from_arrays(const uint16_t* d_W, const float* d_b, int V, int d, int C, const float* h_mu,
                                     const float* h_R, const float* h_bmax, const int32_t* h_n, const int32_t* h_perm,
                                     void* stream, csv_index** out) {
    if (out) *out = nullptr;
    if (!d_W || !h_mu || !h_R || !h_bmax || !h_n || !h_perm || !out) { csv_set_error("null argument"); return CSV_EINVAL; }
    int rc = check_shape(V, d, C);
    if (rc) return rc;
    std::vector<int32_t> n(h_n, h_n + C), off(C + 1, 0), perm(h_perm, h_perm + V);
    std::vector<float> lnn(C);
    for (int c = 0; c < C; ++c) {
        if (n[c] < 0) { csv_set_error("negative cluster size"); return CSV_EINVAL; }
        off[c + 1] = off[c] + n[c];
        lnn[c] = n[c] > 0 ? (float)log((double)n[c]) : -INFINITY;
    }
    if (off[C] != V) { csv_set_error("cluster sizes sum to %d, not V=%d", off[C], V); return CSV_EINVAL; }
    std::vector<char> seen(V, 0);
    for (int i = 0; i < V; ++i) {
        if (perm[i] < 0 || perm[i] >= V || seen[perm[i]]) { csv_set_error("h_perm is not a permutation of 0..V-1"); return CSV_EINVAL; }
        seen[perm[i]] = 1;
    }
    hipStream_t st = (hipStream_t)stream;
    csv_index* x = nullptr;
    rc = csv_index_alloc(V, d, C, &x);
    if (rc) return rc;
    auto fail = [&](int code) { csv_index_free(x); return code; };
    {
        int nmax = 1;
        for (int c = 0; c < C; ++c) nmax = n[c] > nmax ? n[c] : nmax;
        x->ln_nmax = (float)log((double)nmax);
        x->n_max = nmax;
    }
    hipError_t e = hipMemcpyAsync(x->mu, h_mu, (size_t)C * d * 4, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(x->R, h_R, (size_t)C * 4, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(x->bmax, h_bmax, (size_t)C * 4, hipMemcpyHostToDevice, st);
    if (e == hipSuccess) e = hipMemcpyAsync(x->lnn, lnn.data(), (size_t)C * 4, hipMemcpyHostToDevice, st);
    if (e != hipSuccess) { csv_set_error("metadata upload failed: %s", hipGetErrorString(e)); return fail(CSV_EHIP); }
    if ((rc = upload_layout(x, n, off, perm, st))) return fail(rc);
    if ((rc = gather(x, d_W, d_b, st))) return fail(rc);
    if ((rc = csv_index_pack_cmeta(x, st))) return fail(rc);
    if (hipStreamSynchronize(st) != hipSuccess) { csv_set_error("index import failed on the device"); return fail(CSV_EHIP); }
    *out = x;
    return CSV_OK;
}

extern "C" int csv_index_export(const csv_index* x, float* h_mu, float* h_R, float* h_bmax, int32_t* h_n, int32_t* h_perm) {
    if (!x) { csv_set_error("null index"); return CSV_EINVAL; }
    if (h_mu) CSV_HIP(hipMemcpy(h_mu, x->mu, (size_t)x->C * x->d * 4, hipMemcpyDeviceToHost));
    if (h_R) CSV_HIP(hipMemcpy(h_R, x->R, (size_t)x->C * 4, hipMemcpyDeviceToHost));
    if (h_bmax) CSV_HIP(hipMemcpy(h_bmax, x->bmax, (size_t)x->C * 4, hipMemcpyDeviceToHost));
    if (h_n) CSV_HIP(hipMemcpy(h_n, x->n, (size_t)x->C * 4, hipMemcpyDeviceToHost));
    if (h_perm) CSV_HIP(hipMemcpy(h_perm, x->perm, (size_t)x->V * 4, hipMemcpyDeviceToHost));
    return CSV_OK;
}

extern "C" int csv_index_set_bias_table(csv_index* x, int m, const float* h_table, void* stream) {
    if (!x) { csv_set_error("null index"); return CSV_EINVAL; }
    if (m < 0 || m > CSV_MAX_BIAS_TABLE || (m >= 1 && !h_table)) { csv_set_error("bias table: m=%d outside 0..%d, or null table", m, CSV_MAX_BIAS_TABLE); return CSV_EINVAL; }
    hipStream_t st = (hipStream_t)stream;
    if (x->bt) {
        CSV_HIP(hipStreamSynchronize(st));
        (void)hipFree(x->bt);
        x->bt = nullptr;
        x->bt_m = 0;
    }
    if (m == 0) return CSV_OK;
    const size_t bytes = (size_t)x->C * m * sizeof(float2);
    if (hipMalloc((void**)&x->bt, bytes) != hipSuccess) { csv_set_error("out of device memory (bias table)"); return CSV_ENOMEM; }
    CSV_HIP(hipMemcpyAsync(x->bt, h_table, bytes, hipMemcpyHostToDevice, st));
    CSV_HIP(hipStreamSynchronize(st));
    x->bt_m = m;
    return CSV_OK;
}

extern "C" int csv_index_get_bias_table(const csv_index* x, int* m, float* h_table) {
    if (!x || !m) { csv_set_error("null index or m"); return CSV_EINVAL; }
    *m = x->bt_m;
    if (h_table && x->bt_m) CSV_HIP(hipMemcpy(h_table, x->bt, (size_t)x->C * x->bt_m * sizeof(float2), hipMemcpyDeviceToHost));
    return CSV_OK;
}

extern "C" int csv_index_set_angular(csv_index* x, const float* h_ang, void* stream) {
    if (!x) { csv_set_error("null index"); return CSV_EINVAL; }
    hipStream_t st = (hipStream_t)stream;
    if (!h_ang) {
        if (x->ang) {
            CSV_HIP(hipStreamSynchronize(st));
            (void)hipFree(x->ang);
            x->ang = nullptr;
        }
        return CSV_OK;
    }
    if (x->bt || x->mu16) { csv_set_error("an angular index takes neither a bias table nor bf16 centroids"); return CSV_EINVAL; }
    if (!x->ang && hipMalloc((void**)&x->ang, (size_t)x->C * sizeof(float4)) != hipSuccess) { csv_set_error("out of device memory (angular metadata)"); return CSV_ENOMEM; }
    CSV_HIP(hipMemcpyAsync(x->ang, h_ang, (size_t)x->C * sizeof(float4), hipMemcpyHostToDevice, st));
    CSV_HIP(hipStreamSynchronize(st));
    return CSV_OK;
}

extern "C" int csv_index_get_angular(const csv_index* x, int* present, float* h_ang) {
    if (!x || !present) { csv_set_error("null index or present"); return CSV_EINVAL; }
    *present = x->ang != nullptr;
    if (h_ang && x->ang) CSV_HIP(hipMemcpy(h_ang, x->ang, (size_t)x->C * sizeof(float4), hipMemcpyDeviceToHost));
    return CSV_OK;
}
