// Trainer-side kernels: merge of the solvers' updates (paper Section 4.1: "merge updates, broadcast
// model") and the duality gap that solvers report as convergence metric (Section 4.1, Section 5.1).
#pragma once
#include <hip/hip_runtime.h>
#include "device_types.hpp"
#include "mem.hpp"
#include "sdca_rowwise.hpp"

namespace chicle {

// Elastic net (paper Section 2.2: generalised linear models): with the regulariser lambda (|w|^2 / 2 +
// l1 |w|_1) the solvers' updates add up in the dual image v, which is what the double-precision vector
// holds, and the shared vector is w_j = sign(v_j) max(|v_j| - l1, 0).  l1 = 0: w = v.
__device__ __forceinline__ double soft_threshold(double v, double l1)
{
    const double a = fabs(v) - l1;
    return a > 0.0 ? copysign(a, v) : 0.0;
}
// The shared vector as the gap kernels read it: the float mirror holds w itself, the double vector holds v.
__device__ __forceinline__ float shared_at(const float *w, int64_t c, double) { return w[c]; }
__device__ __forceinline__ double shared_at(const double *v, int64_t c, double l1) { return soft_threshold(v[c], l1); }

// u_k <- 0 for k < K (a solver fetching the model starts with no update of its own).
__global__ __launch_bounds__(256) void clear_private(float *u_all, int64_t ld_v, int64_t d4, int K)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < d4; j += stride)
        for (int k = 0; k < K; ++k) reinterpret_cast<float4 *>(u_all + (int64_t)k * ld_v)[j] = z;
}

// w <- w + sum_k Delta w_k with Delta w_k = u_k / sigma, then u_k <- 0 for all k (merge, broadcast).
// The shared vector is kept in double (w64) with a float mirror (w32) for the kernels that gather it.
// One pass: reads K + 1 vectors, writes K + 2 vectors, four columns per thread (ld_v and the
// buffers are 16-byte aligned; d is handled up to its padded length, the padding holds zeros).
__global__ __launch_bounds__(256) void aggregate_broadcast(double *w64, float *w32, float *u_all,
                                                           int64_t ld_v, int64_t d4, int K, float inv_sigma, double l1)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    double2 *wd = reinterpret_cast<double2 *>(w64);
    float4 *wf = reinterpret_cast<float4 *>(w32);
    const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < d4; j += stride) {
        float4 acc = z;
        for (int k = 0; k < K; ++k) {
            float4 *uk = reinterpret_cast<float4 *>(u_all + (int64_t)k * ld_v) + j;
            const float4 x = *uk;
            acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
            *uk = z;
        }
        double2 lo = wd[2 * j], hi = wd[2 * j + 1];
        lo.x += (double)(acc.x * inv_sigma); lo.y += (double)(acc.y * inv_sigma);
        hi.x += (double)(acc.z * inv_sigma); hi.y += (double)(acc.w * inv_sigma);
        wd[2 * j] = lo; wd[2 * j + 1] = hi;
        wf[j] = make_float4((float)soft_threshold(lo.x, l1), (float)soft_threshold(lo.y, l1),
                            (float)soft_threshold(hi.x, l1), (float)soft_threshold(hi.y, l1));
    }
}

// out <- Delta w_solver, or sum_k Delta w_k when solver < 0 (read-back helper).
__global__ __launch_bounds__(256) void delta_w_out(const float *u_all, int64_t ld_v, int64_t d, int K,
                                                   int solver, float inv_sigma, float *out)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < d; j += stride) {
        float acc = 0.f;
        if (solver >= 0) acc = u_all[(int64_t)solver * ld_v + j];
        else for (int k = 0; k < K; ++k) acc += u_all[(int64_t)k * ld_v + j];
        out[j] = acc * inv_sigma;
    }
}

// The merge where private vectors are stored compactly (see layout.hpp).  A workgroup takes 256 consecutive
// words of 32 columns (8192 columns) and walks the solvers: a solver's entries for these columns are one
// contiguous run of its compact vector, which the workgroup reads (and clears) with coalesced accesses into
// LDS; each thread then picks the entries of its own word out of the run, in order, by the word's bits.
// u_off[k]: where solver k's compact vector starts in u.  Reads and clears only what the solvers touched.
// Where there are few words (few workgroups), the solvers are divided over gridDim.y slices as well; the
// slices then add their sums into the double-precision vector with atomic adds and the float mirror is
// refreshed by a pass of its own (mirror_from_double).
constexpr int AGG_WORDS = 256;                       // words (threads) per workgroup
__global__ __launch_bounds__(AGG_WORDS) void aggregate_compact(double *w64, float *w32, float *u, const int64_t *__restrict__ u_off,
                                                               const unsigned *__restrict__ bits, const int32_t *__restrict__ pref,
                                                               int64_t words, int64_t d, int K, float inv_sigma, double l1)
{
    __shared__ float run[AGG_WORDS * 33];            // a run is at most all columns of the workgroup (32 per word;
                                                     // 33: the sums are laid out one word per padded row at the end)
    __shared__ unsigned touched[AGG_WORDS];
    __shared__ int run_begin, run_end;
    const int tid = threadIdx.x;
    const int64_t j = (int64_t)blockIdx.x * AGG_WORDS + tid;
    const bool live = j < words;
    const int last = (int)min((int64_t)AGG_WORDS, words - (int64_t)blockIdx.x * AGG_WORDS) - 1;   // last live thread
    float acc[32];
#pragma unroll
    for (int b = 0; b < 32; ++b) acc[b] = 0.f;
    unsigned any = 0;
    // (the next solver's word and prefix are requested before this solver's run is waited for)
    const int per = (K + (int)gridDim.y - 1) / (int)gridDim.y;
    const int k0 = (int)blockIdx.y * per, k1 = min(K, k0 + per);
    unsigned m_next = live && k0 < k1 ? bits[(int64_t)k0 * words + j] : 0u;
    int pf_next = live && k0 < k1 ? pref[(int64_t)k0 * words + j] : 0;
    for (int k = k0; k < k1; ++k) {
        const unsigned m = m_next;
        const int pf = pf_next;
        if (k + 1 < k1 && live) { m_next = bits[(int64_t)(k + 1) * words + j]; pf_next = pref[(int64_t)(k + 1) * words + j]; }
        if (tid == 0) run_begin = pf;
        if (tid == last) run_end = pf + __popc(m);
        __syncthreads();
        const int begin = run_begin, len = run_end - begin;
        float *uk = u + u_off[k] + begin;
        for (int i = tid; i < len; i += AGG_WORDS) { run[i] = uk[i]; uk[i] = 0.f; }
        __syncthreads();
        any |= m;
        int r = pf - begin;
#pragma unroll
        for (int b = 0; b < 32; ++b)
            if (m & (1u << b)) acc[b] += run[r++];
        __syncthreads();                             // the run is overwritten by the next solver's
    }
    // the sums go through LDS so that the shared vector is updated with coalesced accesses
    touched[tid] = any;
#pragma unroll
    for (int b = 0; b < 32; ++b) run[tid * 33 + b] = acc[b];
    __syncthreads();
    const int64_t c0 = (int64_t)blockIdx.x * AGG_WORDS * 32;
    for (int i = tid; i < AGG_WORDS * 32; i += AGG_WORDS) {
        const int64_t c = c0 + i;
        if (c < d && (touched[i >> 5] & (1u << (i & 31)))) {
            const double add = (double)(run[(i >> 5) * 33 + (i & 31)] * inv_sigma);
            if (gridDim.y == 1) {
                const double x = w64[c] + add;
                w64[c] = x;
                w32[c] = (float)soft_threshold(x, l1);
            } else {
                atomicAdd(&w64[c], add);
            }
        }
    }
}

// The same merge for thinly occupied vectors (long rows over many columns: a solver holds a few of every
// hundred columns).  A solver's run for a workgroup's 8192 columns is then a few hundred floats, and staging
// it through LDS costs three workgroup barriers and a dependent trip to memory per solver.  Here every thread
// picks the entries of its own word straight from memory - neighbouring threads read neighbouring short
// pieces of the run, so the lines are shared inside the wavefront - and keeps its 32 sums in LDS (row tid of
// a padded array, touched by that thread alone until the end), with no barrier inside the walk over the
// solvers; the next solver's word and prefix are requested before this solver's entries are waited for.
__global__ __launch_bounds__(AGG_WORDS) void aggregate_compact_thin(double *w64, float *w32, float *u, const int64_t *__restrict__ u_off,
                                                                    const unsigned *__restrict__ bits, const int32_t *__restrict__ pref,
                                                                    int64_t words, int64_t d, int K, float inv_sigma, double l1)
{
    __shared__ float sums[AGG_WORDS * 33];
    __shared__ unsigned touched[AGG_WORDS];
    const int tid = threadIdx.x;
    const int64_t j = (int64_t)blockIdx.x * AGG_WORDS + tid;
    const bool live = j < words;
    float *mine = sums + tid * 33;
#pragma unroll
    for (int b = 0; b < 32; ++b) mine[b] = 0.f;
    unsigned any = 0;
    const int per = (K + (int)gridDim.y - 1) / (int)gridDim.y;              // slices of solvers, as above
    const int k0 = (int)blockIdx.y * per, k1 = min(K, k0 + per);
    unsigned m_next = live && k0 < k1 ? bits[(int64_t)k0 * words + j] : 0u;
    int pf_next = live && k0 < k1 ? pref[(int64_t)k0 * words + j] : 0;
    for (int k = k0; k < k1; ++k) {
        unsigned m = m_next;
        const int pf = pf_next;
        if (k + 1 < k1 && live) { m_next = bits[(int64_t)(k + 1) * words + j]; pf_next = pref[(int64_t)(k + 1) * words + j]; }
        any |= m;
        float *uk = u + u_off[k] + pf;
        while (m) {                                  // four entries per trip
            float v[4];
            int b[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                b[q] = m ? __ffs(m) - 1 : -1;
                m &= m - 1;
                v[q] = b[q] >= 0 ? uk[q] : 0.f;
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (b[q] >= 0) { uk[q] = 0.f; mine[b[q]] += v[q]; }
            uk += 4;
        }
    }
    touched[tid] = any;
    __syncthreads();
    const int64_t c0 = (int64_t)blockIdx.x * AGG_WORDS * 32;
    for (int i = tid; i < AGG_WORDS * 32; i += AGG_WORDS) {
        const int64_t c = c0 + i;
        if (c < d && (touched[i >> 5] & (1u << (i & 31)))) {
            const double add = (double)(sums[(i >> 5) * 33 + (i & 31)] * inv_sigma);
            if (gridDim.y == 1) {
                const double x = w64[c] + add;
                w64[c] = x;
                w32[c] = (float)soft_threshold(x, l1);
            } else {
                atomicAdd(&w64[c], add);
            }
        }
    }
}

__global__ __launch_bounds__(256) void mirror_from_double(const double *__restrict__ w64, float *w32, int64_t d, double l1)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < d; c += stride) w32[c] = (float)soft_threshold(w64[c], l1);
}

// Read-back helper for compact private vectors: out <- Delta w_solver, or sum_k Delta w_k when solver < 0.
__global__ __launch_bounds__(256) void delta_w_out_compact(const float *u, const int64_t *__restrict__ u_off,
                                                           const unsigned *__restrict__ bits, const int32_t *__restrict__ pref,
                                                           int64_t words, int64_t d, int K, int solver, float inv_sigma,
                                                           float *out)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < d; c += stride) {
        float acc = 0.f;
        const int64_t j = c >> 5;
        const unsigned bit = 1u << (c & 31);
        for (int k = solver >= 0 ? solver : 0; k < (solver >= 0 ? solver + 1 : K); ++k) {
            const unsigned m = bits[(int64_t)k * words + j];
            if (m & bit) acc += u[u_off[k] + pref[(int64_t)k * words + j] + __popc(m & (bit - 1u))];
        }
        out[c] = acc * inv_sigma;
    }
}

__device__ __forceinline__ double wave_sum_d(double x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

// Workgroup sum of two doubles -> thread 0 writes them.  256 threads.
__device__ __forceinline__ void block_sum2_store(double a, double b, double *out_a, double *out_b)
{
    __shared__ double ra[4], rb[4];
    a = wave_sum_d(a);
    b = wave_sum_d(b);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { ra[wave] = a; rb[wave] = b; }
    __syncthreads();
    if (threadIdx.x == 0) {
        *out_a = ra[0] + ra[1] + ra[2] + ra[3];
        *out_b = rb[0] + rb[1] + rb[2] + rb[3];
    }
}

// Per-row loss and conjugate terms of the gap; also leaves the residual rw of every row in the chunk
// for the next local pass (hinge: 1 - y z, squared: y - z with z = x_i . w).  WT is the type the dot
// product is gathered and accumulated in: double for the squared loss, whose steps cancel y - z - alpha
// down to the size of the update near convergence; float for hinge.
// LPR lanes cooperate on one row (LPR divides 64).  Each workgroup writes one partial (loss sum,
// conjugate sum) in double.
//   hinge   : loss = max(0, 1 - y z),   conj = loss^*(-a) = -a
//   squared : loss = (z - y)^2 / 2,     conj = a^2/2 - a y
//   logistic: loss = log(1 + exp(-y z)), conj = a log a + (1 - a) log(1 - a); rw = -y z
template <int LOSS, typename WT>
__device__ __forceinline__ void gap_row_terms(RowState *st, WT z, double &s_loss, double &s_conj)
{
    const float y = st->y, a = st->alpha;
    if (LOSS == 0) {
        const WT rw = (WT)1 - (WT)y * z;
        st->rw = (float)rw;
        s_loss += (double)(rw > (WT)0 ? rw : (WT)0);
        s_conj += (double)(-a);
    } else if (LOSS == 2) {
        const double m = -(double)y * (double)z;
        st->rw = (float)m;
        s_loss += fmax(m, 0.0) + log1p(exp(-fabs(m)));
        const double ad = (double)a, bd = 1.0 - (double)a;
        s_conj += (ad > 0.0 ? ad * log(ad) : 0.0) + (bd > 0.0 ? bd * log(bd) : 0.0);
    } else {
        const WT rw = (WT)y - z;
        st->rw = (float)rw;
        s_loss += 0.5 * (double)rw * (double)rw;
        s_conj += 0.5 * (double)a * (double)a - (double)a * (double)y;
    }
}

// Grid: (workgroups per chunk, chunks).  Every group of LPR lanes walks rows of its chunk with a fixed
// stride and keeps two rows in flight.  Partial sums are indexed by the linear workgroup id.
template <int LOSS, int LPR, typename WT>
__global__ __launch_bounds__(256) void gap_rows_csr(const ChunkDev *__restrict__ chunks,
                                                    const WT *__restrict__ w, double l1,
                                                    double *part_loss, double *part_conj)
{
    constexpr int GROUPS = 256 / LPR;
    const int sub = threadIdx.x % LPR;
    const int grp = threadIdx.x / LPR;
    const ChunkDev &ch = chunks[blockIdx.y];
    const int n_rows = ch.n_rows;
    const int32_t *__restrict__ rp = ch.row_ptr;
    const int32_t *__restrict__ col = ch.col;
    const float *__restrict__ val = ch.val;
    const int stride = gridDim.x * GROUPS;
    double s_loss = 0.0, s_conj = 0.0;
    for (int r0 = blockIdx.x * GROUPS + grp; r0 < n_rows; r0 += 2 * stride) {
        const int r1 = r0 + stride;
        const bool two = r1 < n_rows;
        const int b0 = rp[r0], e0 = rp[r0 + 1];
        const int b1 = two ? rp[r1] : 0, e1 = two ? rp[r1 + 1] : 0;
        WT z0 = 0, z1 = 0;
        int p0 = b0 + sub, p1 = b1 + sub;
        while (p0 < e0 || p1 < e1) {           // both rows advance together: their loads overlap
            int c0 = 0, c1 = 0;
            float v0 = 0.f, v1 = 0.f;
            if (p0 < e0) { c0 = col[p0]; v0 = val[p0]; }
            if (p1 < e1) { c1 = col[p1]; v1 = val[p1]; }
            z0 += (WT)v0 * shared_at(w, c0, l1);
            z1 += (WT)v1 * shared_at(w, c1, l1);
            p0 += LPR; p1 += LPR;
        }
#pragma unroll
        for (int o = LPR / 2; o > 0; o >>= 1) { z0 += __shfl_xor(z0, o, 64); z1 += __shfl_xor(z1, o, 64); }
        if (sub == 0) {
            gap_row_terms<LOSS, WT>(ch.st + r0, z0, s_loss, s_conj);
            if (two) gap_row_terms<LOSS, WT>(ch.st + r1, z1, s_loss, s_conj);
        }
    }
    const int part = blockIdx.y * gridDim.x + blockIdx.x;
    block_sum2_store(s_loss, s_conj, &part_loss[part], &part_conj[part]);
}

// ---- the row pass for long rows over a shared vector far larger than a cache ------------------------------
// A row of a thousand entries spread over twenty million columns makes a thousand lonely 4-byte reads of the
// shared vector, every one of which misses the L2 cache of its compute-unit group and moves a whole line
// over the fabric.  Here the columns are cut into slices of 2 MB of the shared vector.  Rows are sorted by
// column, so a row's entries inside a slice are one contiguous run; off[s * n_total + row] = first entry of the
// row (relative to its start) with column >= s << shift, for s = 0 .. S, is built once per data set.
// Workgroup 8 i + x takes slice 8 (i / n_items) + x: the eight cache partitions (workgroups are dealt round
// robin over them) work on eight neighbouring slices of the same rows at the same time, each partition
// keeps its own slice of the shared vector in its L2, and the lines of entries that two neighbouring slices
// share are fetched from memory once.  Partial dot products are added into z[row] with atomic adds; a second
// kernel turns z into the rows' residuals and the loss and conjugate sums, and clears z for the next pass.
constexpr int SLICE_BYTES_LOG2 = 21;
constexpr int SLICE_SEG = 256;                      // rows per workgroup
constexpr int SLICE_LANES = 16;                     // lanes per row
constexpr int SLICE_ROWS_IN_FLIGHT = 8;             // rows a lane group works on at the same time

// Grid: (workgroups over rows, chunks); one wavefront per row.
__global__ __launch_bounds__(256) void slice_offsets(const ChunkDev *__restrict__ chunks, int shift, int S,
                                                     int64_t n_total, int32_t *off)
{
    const ChunkDev &ch = chunks[blockIdx.y];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int r = blockIdx.x * 4 + wave; r < ch.n_rows; r += gridDim.x * 4) {
        const int b = ch.row_ptr[r], e = ch.row_ptr[r + 1];
        int32_t *o = off + ch.row_base + r;
        // entry p opens every slice after its predecessor's up to its own; the row's end opens all that remain
        for (int p = b + lane; p <= e; p += 64) {
            const int sp = p < e ? ch.col[p] >> shift : S;
            const int sq = p > b ? ch.col[p - 1] >> shift : -1;
            for (int t = sq + 1; t <= sp; ++t) o[(int64_t)t * n_total] = p - b;
        }
    }
}

template <typename WT>
__global__ __launch_bounds__(256) void gap_rows_sliced(const ChunkDev *__restrict__ chunks, const WT *__restrict__ w,
                                                       double l1, const int32_t *__restrict__ off, int64_t n_total,
                                                       int S, int segs_per_chunk, int n_items, WT *z)
{
    __shared__ int s_b[SLICE_SEG], s_e[SLICE_SEG];
    const int x = (int)blockIdx.x % L2_PARTITIONS, i = (int)blockIdx.x / L2_PARTITIONS;
    const int slice = L2_PARTITIONS * (i / n_items) + x, item = i % n_items;
    if (slice >= S) return;
    const ChunkDev &ch = chunks[item / segs_per_chunk];
    const int r0 = (item % segs_per_chunk) * SLICE_SEG;
    if (r0 >= ch.n_rows) return;
    const int nr = min(SLICE_SEG, ch.n_rows - r0);
    const int t = threadIdx.x;
    if (t < nr) {
        const int start = ch.row_ptr[r0 + t];
        const int64_t row = (int64_t)ch.row_base + r0 + t;
        s_b[t] = start + off[(int64_t)slice * n_total + row];
        s_e[t] = start + off[(int64_t)(slice + 1) * n_total + row];
    }
    __syncthreads();
    const int32_t *__restrict__ col = ch.col;
    const float *__restrict__ val = ch.val;
    const int sub = t % SLICE_LANES, grp = t / SLICE_LANES;
    constexpr int GROUPS = 256 / SLICE_LANES, RF = SLICE_ROWS_IN_FLIGHT;
    for (int rb = grp; rb < nr; rb += GROUPS * RF) {
        int b[RF], e[RF], c[RF];
        float v[RF];
        WT acc[RF];
#pragma unroll
        for (int k = 0; k < RF; ++k) {
            const int r = rb + k * GROUPS;
            b[k] = r < nr ? s_b[r] : 0;
            e[k] = r < nr ? s_e[r] : 0;
            const bool has = b[k] + sub < e[k];
            c[k] = has ? col[b[k] + sub] : 0;
            v[k] = has ? val[b[k] + sub] : 0.f;
        }
#pragma unroll
        for (int k = 0; k < RF; ++k) acc[k] = (WT)v[k] * shared_at(w, c[k], l1);
#pragma unroll
        for (int k = 0; k < RF; ++k)                 // runs longer than the lane group
            for (int p = b[k] + SLICE_LANES + sub; p < e[k]; p += SLICE_LANES) acc[k] += (WT)val[p] * shared_at(w, col[p], l1);
#pragma unroll
        for (int k = 0; k < RF; ++k) {
#pragma unroll
            for (int o = SLICE_LANES / 2; o > 0; o >>= 1) acc[k] += __shfl_xor(acc[k], o, 64);
            if (sub == 0 && e[k] > b[k]) atomicAdd(&z[(int64_t)ch.row_base + r0 + rb + k * GROUPS], acc[k]);
        }
    }
}

// Grid: (workgroups per chunk, chunks); a thread per row.  Partial sums by linear workgroup id, as above.
template <int LOSS, typename WT>
__global__ __launch_bounds__(256) void gap_rows_from_z(const ChunkDev *__restrict__ chunks, WT *z,
                                                       double *part_loss, double *part_conj)
{
    const ChunkDev &ch = chunks[blockIdx.y];
    double s_loss = 0.0, s_conj = 0.0;
    for (int r = blockIdx.x * 256 + threadIdx.x; r < ch.n_rows; r += gridDim.x * 256) {
        const WT zi = z[(int64_t)ch.row_base + r];
        z[(int64_t)ch.row_base + r] = (WT)0;
        gap_row_terms<LOSS, WT>(ch.st + r, zi, s_loss, s_conj);
    }
    const int part = blockIdx.y * gridDim.x + blockIdx.x;
    block_sum2_store(s_loss, s_conj, &part_loss[part], &part_conj[part]);
}

// The same row pass where the columns are numbered by popularity: the first n_hot entries of w are
// copied into LDS once per workgroup and the frequent columns of every row are gathered from there;
// only the rare columns go to the cache hierarchy.  1024 threads; dynamic LDS = n_hot * sizeof(WT).
constexpr int GAP_HOT_THREADS = 1024;
constexpr int GAP_HOT_BYTES = 48 * 1024;
constexpr int GAP_HOT_MAX_LPR = 16;         // lanes per row at most; a lane takes 4 consecutive entries

template <int LOSS, int LPR, typename WT>
__global__ __launch_bounds__(GAP_HOT_THREADS) void gap_rows_csr_hot(const ChunkDev *__restrict__ chunks,
                                                                    const WT *__restrict__ w, double l1, int n_hot,
                                                                    double *part_loss, double *part_conj)
{
    extern __shared__ __align__(16) unsigned char gap_hot_raw[];
    WT *hot = reinterpret_cast<WT *>(gap_hot_raw);
    __shared__ double ra[GAP_HOT_THREADS / 64], rb[GAP_HOT_THREADS / 64];
    // LPR lanes per row, as many whole rows per wavefront as fit (LPR need not divide 64: with rows of 40
    // entries ten lanes carry a row and six rows share a wavefront; the lanes left over idle)
    constexpr int ROWS_PER_WAVE = 64 / LPR;
    constexpr int GROUPS = (GAP_HOT_THREADS / 64) * ROWS_PER_WAVE;
    const int lane = threadIdx.x & 63;
    const int sub = lane % LPR;
    const bool idle = lane >= ROWS_PER_WAVE * LPR;
    const int grp = (threadIdx.x >> 6) * ROWS_PER_WAVE + lane / LPR;
    const ChunkDev &ch = chunks[blockIdx.y];
    const int n_rows = ch.n_rows;
    const int32_t *__restrict__ rp = ch.row_ptr;
    const int32_t *__restrict__ col = ch.col;
    const float *__restrict__ val = ch.val;
    const int stride = gridDim.x * GROUPS;
    for (int i = threadIdx.x; i < n_hot; i += GAP_HOT_THREADS) hot[i] = shared_at(w, i, l1);
    __syncthreads();
    double s_loss = 0.0, s_conj = 0.0;
    // (the trip count is the same for all lanes of a wavefront: the shuffles below need every lane)
    for (int rb = blockIdx.x * GROUPS; rb < n_rows; rb += 2 * stride) {
        const int r0 = rb + grp;
        const int r1 = r0 + stride;
        const bool one = !idle && r0 < n_rows;
        const bool two = !idle && r1 < n_rows;
        const int b0 = one ? rp[r0] : 0, e0 = one ? rp[r0 + 1] : 0;
        const int b1 = two ? rp[r1] : 0, e1 = two ? rp[r1 + 1] : 0;
        WT z0 = 0, z1 = 0;
        // Each lane takes 4 consecutive entries of its row with one 16-byte load per array (the vector
        // memory pipeline is busy per instruction, not per byte, here); rows are at most 4 * LPR long where
        // this kernel is used, and every chunk's arrays are followed by readable slack.
        {
            const int p0 = b0 + 4 * sub, p1 = b1 + 4 * sub;
            int4_a4 c0 = {0, 0, 0, 0}, c1 = {0, 0, 0, 0};
            float4_a4 v0 = {0.f, 0.f, 0.f, 0.f}, v1 = {0.f, 0.f, 0.f, 0.f};
            if (p0 < e0) { c0 = gld4(col + p0); v0 = gld4(val + p0); }
            if (p1 < e1) { c1 = gld4(col + p1); v1 = gld4(val + p1); }
            WT w0[4], w1[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool in0 = p0 + k < e0, in1 = p1 + k < e1;
                const int a0 = in0 ? c0[k] : 0, a1 = in1 ? c1[k] : 0;
                w0[k] = a0 < n_hot ? hot[a0] : shared_at(w, a0, l1);
                w1[k] = a1 < n_hot ? hot[a1] : shared_at(w, a1, l1);
                if (!in0) v0[k] = 0.f;
                if (!in1) v1[k] = 0.f;
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                z0 += (WT)v0[k] * w0[k];
                z1 += (WT)v1[k] * w1[k];
            }
        }
        // sum over the row's lanes into its first lane
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) {
            const WT y0 = __shfl_down(z0, o, 64), y1 = __shfl_down(z1, o, 64);
            if (sub < o && sub + o < LPR) { z0 += y0; z1 += y1; }
        }
        if (sub == 0) {
            if (one) gap_row_terms<LOSS, WT>(ch.st + r0, z0, s_loss, s_conj);
            if (two) gap_row_terms<LOSS, WT>(ch.st + r1, z1, s_loss, s_conj);
        }
    }
    s_loss = wave_sum_d(s_loss);
    s_conj = wave_sum_d(s_conj);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { ra[wave] = s_loss; rb[wave] = s_conj; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double a = 0.0, b = 0.0;
        for (int i = 0; i < GAP_HOT_THREADS / 64; ++i) { a += ra[i]; b += rb[i]; }
        const int part = blockIdx.y * gridDim.x + blockIdx.x;
        part_loss[part] = a;
        part_conj[part] = b;
    }
}

// Dense rows: LPR lanes per row, strided over the d columns.  Same grid as the sparse kernel.
template <int LOSS, int LPR, typename WT>
__global__ __launch_bounds__(256) void gap_rows_dense(const ChunkDev *__restrict__ chunks, int d,
                                                      const WT *__restrict__ w, double l1,
                                                      double *part_loss, double *part_conj)
{
    constexpr int GROUPS = 256 / LPR;
    const int sub = threadIdx.x % LPR;
    const int grp = threadIdx.x / LPR;
    const ChunkDev &ch = chunks[blockIdx.y];
    double s_loss = 0.0, s_conj = 0.0;
    for (int r = blockIdx.x * GROUPS + grp; r < ch.n_rows; r += gridDim.x * GROUPS) {
        const float *x = ch.val + (int64_t)r * d;
        WT z = 0;
        for (int p = sub; p < d; p += LPR) z += (WT)x[p] * shared_at(w, p, l1);
#pragma unroll
        for (int o = LPR / 2; o > 0; o >>= 1) z += __shfl_xor(z, o, 64);
        if (sub == 0) gap_row_terms<LOSS, WT>(ch.st + r, z, s_loss, s_conj);
    }
    const int part = blockIdx.y * gridDim.x + blockIdx.x;
    block_sum2_store(s_loss, s_conj, &part_loss[part], &part_conj[part]);
}

// |w|^2 and |w|_1 partials in double (w = the soft-thresholded image of the double vector).
__global__ __launch_bounds__(256) void wsq_partial(const double *__restrict__ v, int64_t d, double l1,
                                                   double *part_wsq, double *part_wabs)
{
    double s = 0.0, t = 0.0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < d; j += 4 * stride) {
        double x[4];                                 // four loads in flight per thread
#pragma unroll
        for (int q = 0; q < 4; ++q) x[q] = j + q * stride < d ? v[j + q * stride] : 0.0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const double y = soft_threshold(x[q], l1);
            s += y * y;
            t += fabs(y);
        }
    }
    block_sum2_store(s, t, &part_wsq[blockIdx.x], &part_wabs[blockIdx.x]);
}

// out[0] = sum loss, out[1] = sum conj, out[2] = |w|^2, out[3] = the kernels' error flag, out[4] = |w|_1; one workgroup,
// fixed summation order.  out may be host memory mapped into the device's address space.
__global__ __launch_bounds__(256) void gap_finish(const double *part_loss, const double *part_conj,
                                                  int n_row_parts, const double *part_wsq, const double *part_wabs,
                                                  int n_w_parts, const int *err, double *out)
{
    double a = 0.0, b = 0.0, c = 0.0, e = 0.0;
    for (int i = threadIdx.x; i < n_row_parts; i += 256) { a += part_loss[i]; b += part_conj[i]; }
    for (int i = threadIdx.x; i < n_w_parts; i += 256) { c += part_wsq[i]; e += part_wabs[i]; }
    __shared__ double ra[4], rb[4], rc[4], re[4];
    a = wave_sum_d(a); b = wave_sum_d(b); c = wave_sum_d(c); e = wave_sum_d(e);
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { ra[wave] = a; rb[wave] = b; rc[wave] = c; re[wave] = e; }
    __syncthreads();
    if (threadIdx.x == 0) {
        out[0] = ra[0] + ra[1] + ra[2] + ra[3];
        out[1] = rb[0] + rb[1] + rb[2] + rb[3];
        out[2] = rc[0] + rc[1] + rc[2] + rc[3];
        out[3] = (double)*err;
        out[4] = re[0] + re[1] + re[2] + re[3];
    }
}

}  // namespace chicle
