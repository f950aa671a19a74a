// Local solver, one coordinate step at a time (paper Section 2.2: L = 1, H = all local samples).
//
// One workgroup per solver.  Every step is: row dot product against the solver's private vector
// (workgroup reduction), closed-form dual step, alpha update inside the chunk, scatter of the row
// into the private vector.  With v_k = w + sigma * Delta w_k the CoCoA subproblem step is a plain
// coordinate step against v_k:
//     hinge   : a' = clip(a + c (1 - y z) / q, 0, 1),  c = lambda n / sigma,  z = x_i . v_k
//     squared : delta = (y - z - a) / (1 + q / c)
//     v_k += (delta s / c) x_i,  s = y (hinge) or 1 (squared).
// The private vector is stored as its difference u_k = v_k - w (zero when the pass starts).  The part
// of a step that depends on w alone is the per-row residual rw that the gap pass left in the chunk
// (hinge: 1 - y x_i.w, squared: y - x_i.w, formed in double from the double-precision w), so a step
// needs only x_i . u_k on top of it.  Keeping the small quantities apart from the O(1) ones keeps fp32
// rounding relative to the update: near convergence y - z - a is a difference of nearly equal numbers.
#pragma once
#include <hip/hip_runtime.h>
#include "device_types.hpp"
#include "mem.hpp"

namespace chicle {

// Logistic loss, one dual step: a' = 1 / (1 + exp(-s)) with s the root of f(s) = m - s - r (a'(s) - a),
// where m = -y z and r = q / c; returns a' - a.  f decreases strictly (slope in [-1 - r/4, -1]) and, a'
// lying in (0, 1), its root lies in [m - r (1 - a), m + r a].  Newton steps from s0 inside that bracket; a
// bisection step whenever Newton would leave it or fails to halve the last step (r can be in the
// hundreds, where plain Newton cycles between the two flat ends of the sigmoid).  *root receives s.
__device__ __forceinline__ float logistic_step(float m, float r, float a, float s0, float *root = nullptr)
{
    float lo = m - r * (1.0f - a), hi = m + r * a;
    float s = fminf(fmaxf(s0, lo), hi), dx_old = hi - lo, dx = dx_old, ap, f, df;
    auto eval = [&]() {
        const float e = __expf(-fabsf(s));
        ap = s >= 0.f ? 1.0f / (1.0f + e) : e / (1.0f + e);
        f = (m - s) - r * (ap - a);
        df = -(1.0f + r * ap * (1.0f - ap));
    };
    eval();
    for (int it = 0; it < 48; ++it) {
        const bool leaves = ((s - hi) * df - f) * ((s - lo) * df - f) > 0.f;
        dx_old = dx;
        if (leaves || fabsf(2.0f * f) > fabsf(dx_old * df)) { dx = 0.5f * (hi - lo); s = lo + dx; }
        else { dx = f / df; s -= dx; }
        eval();
        if (f > 0.f) lo = s; else hi = s;
        if (fabsf(dx) <= 1e-7f * (1.0f + fabsf(s))) break;     // the step is below fp32 resolution of s
    }
    if (root) *root = s;
    return ap - a;
}

// One dual step of the logistic loss computed by a whole wavefront from uniform arguments (see
// logistic_step for the equation).  f decreases strictly, so the 64 lanes evaluate it at 64 evenly spaced
// points of the bracket and the first lane with f <= 0 narrows the bracket 63-fold; when the bracket is so
// narrow that a chord of f misses the root by less than fp32 resolution (|f''| <= 0.0963 r, |f'| >= 1:
// error <= 0.012 h^2 r), the root and a' are read off the chord.  [lo, lo + w] is a bracket of the root:
// the general one, [m - r (1 - a), m + r a], costs two evaluations for r of order one and four for r in
// the hundreds; no derivative, no iteration that could cycle.
__device__ __forceinline__ float logistic_step_wave(float m, float r, float a, float lo, float w, int lane)
{
    const float frac = (float)lane * (1.0f / 63.0f);
    float s = 0.f, ap = 0.f, f = 0.f;
    int k = 1;
    for (int it = 0; it < 8; ++it) {
        s = fmaf(frac, w, lo);
        const float e = __expf(-fabsf(s));
        const float t = __builtin_amdgcn_rcpf(1.0f + e);
        ap = s >= 0.f ? t : e * t;
        f = (m - s) - r * (ap - a);
        const unsigned long long pos = __ballot(f > 0.f);
        k = ~pos ? __builtin_ctzll(~pos) : 64;
        k = min(max(k, 1), 63);
        const float h = w * (1.0f / 63.0f);
        if (h * h * r <= 4e-6f || h <= 1e-7f * (1.0f + fabsf(lo))) break;
        lo = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s), k - 1));
        w = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s), k)) - lo;
    }
    const float f0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(f), k - 1));
    const float f1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(f), k));
    const float a0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ap), k - 1));
    const float a1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(ap), k));
    const float den = f0 - f1;
    const float th = den > 0.f ? fminf(fmaxf(f0 * __builtin_amdgcn_rcpf(den), 0.f), 1.f) : 0.5f;
    return fmaf(th, a1 - a0, a0) - a;
}

// rw: residual at w (see above; logistic: -y x_i.w); xu = x_i . u_k.  The arguments are the same in every
// lane of a wavefront (the logistic step is computed by the wavefront as a whole).
template <int LOSS>
__device__ __forceinline__ float dual_step(float a, float y, float rw, float xu, float q, float c)
{
    if (LOSS == 0) {
        float an = a + c * (rw - y * xu) / q;
        an = fminf(fmaxf(an, 0.0f), 1.0f);
        return an - a;
    }
    if (LOSS == 2) {
        // (taken from the first lane so that the compiler knows them to be uniform)
        const float m = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(rw - y * xu)));
        const float r = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(q / c)));
        const float a1 = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(a)));
        return logistic_step_wave(m, r, a1, m - r * (1.0f - a1), r, threadIdx.x & 63);
    }
    return (rw - xu - a) / (1.0f + q / c);
}

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
    return x;
}

// Sum over the workgroup; every thread gets the result.  red: BLOCK/64 floats of LDS.
template <int BLOCK>
__device__ __forceinline__ float block_sum(float x, float *red)
{
    x = wave_sum(x);
    if (BLOCK == 64) return x;
    const int wave = threadIdx.x >> 6;
    __syncthreads();                       // red may still be read from the previous use
    if ((threadIdx.x & 63) == 0) red[wave] = x;
    __syncthreads();
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < BLOCK / 64; ++i) s += red[i];
    return s;
}

// Largest j in [0, n) with prefix[j] <= lr (prefix ascending, prefix[0] = 0).
__device__ __forceinline__ int find_chunk(const int *prefix, int n, int lr)
{
    int lo = 0, hi = n - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (prefix[mid] <= lr) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// What a step needs to know about its row; len = 0 marks a row to skip.
struct RowMeta {
    const int32_t *col;
    const float *val;
    RowState *st;
    int len;
    float y, alpha, q, rw;
};

// Sparse rows of any length.  The step itself is gather - reduce - step - scatter; everything that does
// not depend on the private vector is fetched ahead by a small software pipeline so that a step costs
// one trip to memory (the gather) instead of five dependent ones:
//     step t issues   the order entry of row t+4, the chunk lookup and state loads of row t+3,
//     publishes       the resolved row t+2 in LDS (thread 0 does these three),
//     loads           the first EPT * BLOCK entries of row t+1 into registers (all threads),
//     computes        row t.
// The scatter uses atomic adds that are not waited for: accesses of one compute unit to one address
// are served in order, and the gathers read past the vector cache (ld_l2).
// Dynamic LDS: max_list chunk descriptors, then max_list local-row prefixes.
template <int LOSS, int BLOCK, int EPT>
__global__ __launch_bounds__(BLOCK) void sdca_rowwise_csr(
    const ChunkDev *__restrict__ chunks, const SolverDev *__restrict__ solvers,
    const int32_t *__restrict__ solver_chunks, const int32_t *__restrict__ solver_prefix,
    const int32_t *__restrict__ perm, float *u_all, int64_t ld_v, int max_list, RoundScalars sc, int *err,
    const int64_t *__restrict__ u_off)
{
    // u_off != nullptr: private vectors are stored compactly, solver k's at u_all + u_off[k], and every
    // entry's index into it is found in the array behind the chunk's column ids
    extern __shared__ __align__(16) unsigned char rw_smem[];
    __shared__ float red[BLOCK / 64];
    __shared__ RowMeta ring[4];
    const SolverDev S = solvers[blockIdx.x];
    ChunkDev *l_desc = reinterpret_cast<ChunkDev *>(rw_smem);
    int *l_prefix = reinterpret_cast<int *>(l_desc + max_list);
    const int tid = threadIdx.x;
    stamp_solver(sc, 0);
    for (int i = tid; i < S.n_chunks; i += BLOCK) {
        l_desc[i] = chunks[solver_chunks[S.list_begin + i]];
        l_prefix[i] = solver_prefix[S.list_begin + i];
    }
    __syncthreads();
    float *u = u_off ? u_all + u_off[blockIdx.x] : u_all + (int64_t)blockIdx.x * ld_v;
    const int32_t *pk = perm + S.perm_off;
    const int n = S.n_rows;

    // thread 0: rows being resolved
    int p_val = -1;                       // order entry of the row resolved next step
    int m_ci = -1, m_r = 0;               // row whose state loads are in flight
    int2_a4 m_rp = {0, 0};
    float4_v m_st = {0.f, 0.f, 0.f, 0.f};
    // all threads: entries of the current and of the next row
    int c_c[EPT], n_c[EPT];
    float c_v[EPT], n_v[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) { c_c[e] = n_c[e] = 0; c_v[e] = n_v[e] = 0.f; }

    for (int t = -4; t < n; ++t) {
        if (tid == 0) {
            // publish row t + 2 (state loads issued last step)
            if (t + 2 >= 0 && t + 2 < n) {
                RowMeta m;
                m.col = nullptr; m.val = nullptr; m.st = nullptr; m.len = 0;
                m.y = m_st.x; m.alpha = m_st.y; m.q = m_st.z; m.rw = m_st.w;
                const int len = m_rp.y - m_rp.x;
                if (m_ci >= 0 && m.q != 0.f && len > 0) {
                    const ChunkDev &ch = l_desc[m_ci];
                    m.col = (u_off ? chunk_compact_ids(ch) : ch.col) + m_rp.x;
                    m.val = ch.val + m_rp.x; m.st = ch.st + m_r; m.len = len;
                }
                ring[(t + 2) & 3] = m;
            }
            // state loads of row t + 3
            m_ci = -1;
            if (t + 3 >= 0 && t + 3 < n) {
                if ((unsigned)p_val >= (unsigned)n) {
                    atomicOr(err, ERR_PERM_RANGE);
                } else {
                    m_ci = find_chunk(l_prefix, S.n_chunks, p_val);
                    m_r = p_val - l_prefix[m_ci];
                    const ChunkDev &ch = l_desc[m_ci];
                    m_rp = gld2(ch.row_ptr + m_r);
                    m_st = gld_state(ch.st + m_r);
                }
            }
            // order entry of row t + 4
            p_val = (t + 4 >= 0 && t + 4 < n) ? pk[t + 4] : -1;
        }
        // The gather of row t is requested first and the entries of row t + 1 (published last step) after it:
        // loads return in the order they were issued, so the step does not wait for the next row's entries,
        // which come from memory.
        const RowMeta m = ring[t & 3];                            // (t < 0: an unused slot)
        const bool step = t >= 0 && m.len > 0;                    // uniform over the workgroup
        float got[EPT];
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            got[e] = 0.f;
            if (step && tid + e * BLOCK < m.len) got[e] = gather_entry(u, c_c[e]);
        }
        if (t + 1 >= 0 && t + 1 < n) {
            const RowMeta &mn = ring[(t + 1) & 3];
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const int p = tid + e * BLOCK;
                n_c[e] = 0; n_v[e] = 0.f;
                if (p < mn.len) { n_c[e] = gld(mn.col + p); n_v[e] = gld(mn.val + p); }
            }
        }
        {
            if (step) {
                float part = 0.f;
#pragma unroll
                for (int e = 0; e < EPT; ++e) part += c_v[e] * got[e];
                for (int p = tid + EPT * BLOCK; p < m.len; p += BLOCK) part += gld(m.val + p) * gather_entry(u, gld(m.col + p));
                const float xu = block_sum<BLOCK>(part, red);
                const float delta = dual_step<LOSS>(m.alpha, m.y, m.rw, xu, m.q, sc.c);
                if (tid == 0) {
                    float an = m.alpha + delta;                      // a + (clip(..) - a) can leave [0, 1] by an ulp
                    if (LOSS != 1) an = fminf(fmaxf(an, 0.f), 1.f);
                    gst(&m.st->alpha, an);
                }
                const float coef = delta * (LOSS == 1 ? 1.0f : m.y) * sc.inv_c;
                if (coef != 0.0f) {
#pragma unroll
                    for (int e = 0; e < EPT; ++e)
                        if (tid + e * BLOCK < m.len) add_entry(u, c_c[e], coef * c_v[e]);
                    for (int p = tid + EPT * BLOCK; p < m.len; p += BLOCK)
                        add_entry(u, gld(m.col + p), coef * gld(m.val + p));
                }
            }
        }
#pragma unroll
        for (int e = 0; e < EPT; ++e) { c_c[e] = n_c[e]; c_v[e] = n_v[e]; }
        __syncthreads();   // ring slots written this step are read next step; orders scatter before gather
    }
    stamp_solver(sc, 1);
}

// Dense rows.  The private vector is staged in LDS when it fits (V_LDS), else it stays in HBM.
// Dynamic LDS: 2 * max_list ints, then d floats when V_LDS.
template <int LOSS, int BLOCK, bool V_LDS>
__global__ __launch_bounds__(BLOCK) void sdca_rowwise_dense(
    const ChunkDev *__restrict__ chunks, const SolverDev *__restrict__ solvers,
    const int32_t *__restrict__ solver_chunks, const int32_t *__restrict__ solver_prefix,
    const int32_t *__restrict__ perm, float *u_all, int64_t ld_v, int d, int max_list,
    RoundScalars sc, int *err)
{
    extern __shared__ int lists[];
    __shared__ float red[BLOCK / 64];
    const SolverDev S = solvers[blockIdx.x];
    int *l_chunk = lists;
    int *l_prefix = lists + max_list;
    float *v_lds = reinterpret_cast<float *>(lists + 2 * max_list);
    float *v_glb = u_all + (int64_t)blockIdx.x * ld_v;
    const int tid = threadIdx.x;
    stamp_solver(sc, 0);
    for (int i = tid; i < S.n_chunks; i += BLOCK) {
        l_chunk[i] = solver_chunks[S.list_begin + i];
        l_prefix[i] = solver_prefix[S.list_begin + i];
    }
    if (V_LDS)
        for (int i = tid; i < d; i += BLOCK) v_lds[i] = v_glb[i];
    __syncthreads();
    float *v = V_LDS ? v_lds : v_glb;
    const int32_t *pk = perm + S.perm_off;

    for (int t = 0; t < S.n_rows; ++t) {
        const int lr = pk[t];
        if ((unsigned)lr >= (unsigned)S.n_rows) {
            if (tid == 0) atomicOr(err, ERR_PERM_RANGE);
            continue;
        }
        const int j = find_chunk(l_prefix, S.n_chunks, lr);
        const ChunkDev &ch = chunks[l_chunk[j]];
        const int r = lr - l_prefix[j];
        const RowState st = ch.st[r];
        const float q = st.q;
        if (q == 0.0f) continue;
        const float *x = ch.val + (int64_t)r * d;
        const float y = st.y;
        const float a = st.alpha;
        const float rw = st.rw;
        float part = 0.0f;
        for (int p = tid; p < d; p += BLOCK) part += x[p] * v[p];
        const float xu = block_sum<BLOCK>(part, red);
        const float delta = dual_step<LOSS>(a, y, rw, xu, q, sc.c);
        if (tid == 0) {
            float an = a + delta;
            if (LOSS != 1) an = fminf(fmaxf(an, 0.f), 1.f);
            ch.st[r].alpha = an;
        }
        const float coef = delta * (LOSS == 1 ? 1.0f : y) * sc.inv_c;
        if (coef != 0.0f)
            for (int p = tid; p < d; p += BLOCK) v[p] += coef * x[p];
        __syncthreads();
    }
    if (V_LDS)
        for (int i = tid; i < d; i += BLOCK) v_glb[i] = v_lds[i];
    stamp_solver(sc, 1);
}

}  // namespace chicle
