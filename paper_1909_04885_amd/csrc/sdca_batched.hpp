// Local solver, blocks of 64 coordinate steps at a time, same sequence of steps as the row-wise
// solver (paper Section 2.2: L = 1, strictly sequential coordinates; H = all local samples).
//
// For a block of rows taken in visiting order, everything a step needs from earlier steps of the
// block is a scalar recurrence over the rows' Gram matrix G_ij = x_i . x_j:
//     z_i = z_i(start of block) + sum_{j<i} (delta_j s_j / c) G_ij ,   delta_i = step_i(z_i).
// With t_i the unclipped step of row i (hinge: t = (c/q)(1 - y z), delta = clamp(t, -alpha, 1-alpha);
// squared: t = delta = c/(c+q) (y - alpha - z)) the recurrence becomes
//     delta_j = clamp_j(t_j);   t_i += delta_j T_ij,
//     T_ij = -y_i y_j G_ij / q_i (hinge),   T_ij = -G_ij / (c + q_i) (squared),
// three dependent instructions per step in one wavefront (lane i owns t_i).  The dot products with
// the private vector (gather), the alpha updates and the scatter into the private vector are done a
// block at a time by the other wavefronts of the workgroup, off the critical path; the matrices T
// depend on the data and the visiting order only and are produced beforehand by a separate kernel
// that runs on the whole chip.  Block b's dot products see the private vector with blocks <= b-2
// applied; block b-1 enters through the cross part of T.  Exact arithmetic gives the row-wise
// solver's result; in floating point only the summation order differs.
#pragma once
#include <hip/hip_runtime.h>
#include "device_types.hpp"
#include "sdca_rowwise.hpp"

namespace chicle {

constexpr int BATCH = 64;                    // rows per block = lanes of the chain wavefront
constexpr int TILE_W = 2 * BATCH;            // T rows: previous block (cross part), then own block
constexpr int TILE_FLOATS = BATCH * TILE_W;  // layout [jp][i]: jp in [0,128), i in [0,64)
constexpr int GRAM_MAX_ROW = 48;             // longest sparse row the batched solver accepts
constexpr int LPR = 8;                       // helper lanes per row
constexpr int ENT = GRAM_MAX_ROW / LPR;      // entries per helper lane
constexpr int HELPER_WAVES = BATCH * LPR / 64;
constexpr int BATCHED_THREADS = 64 + BATCH * LPR;
constexpr int RING = 8;

// What the helpers know about one row of a block.
struct RowSlot {
    const int32_t *col;
    const float *val;
    float *alpha_p;
    int len;          // 0 for a missing, empty or rejected row
    float y, alpha, q, zw;
};

// Resolve local row lr of a solver (lists in LDS or global) into a RowSlot; len = 0 if unusable.
__device__ __forceinline__ RowSlot locate_row(const ChunkDev *__restrict__ chunks, const int *l_chunk,
                                              const int *l_prefix, int n_list, int n_rows, int lr,
                                              int *err)
{
    RowSlot s;
    s.col = nullptr; s.val = nullptr; s.alpha_p = nullptr; s.len = 0;
    s.y = 0.f; s.alpha = 0.f; s.q = 0.f; s.zw = 0.f;
    if (lr < 0) return s;
    if (lr >= n_rows) { atomicOr(err, ERR_PERM_RANGE); return s; }
    const int j = find_chunk(l_prefix, n_list, lr);
    const ChunkDev &ch = chunks[l_chunk[j]];
    const int r = lr - l_prefix[j];
    const int b = ch.row_ptr[r], e = ch.row_ptr[r + 1];
    s.q = ch.q[r];
    if (s.q == 0.f || e - b > GRAM_MAX_ROW) return s;
    s.col = ch.col + b; s.val = ch.val + b; s.alpha_p = ch.alpha + r; s.len = e - b;
    s.y = ch.y[r]; s.alpha = ch.alpha[r]; s.zw = ch.zw[r];
    return s;
}

// ------------------------------------------------------------------------------------------------
// Gram blocks, reference form: every pair by a merge of the two sorted rows staged in LDS.
// One workgroup per block.  tile_solver[tile] = solver that owns the tile.
template <int LOSS>
__global__ __launch_bounds__(256) void gram_tiles_merge(
    const ChunkDev *__restrict__ chunks, const SolverDev *__restrict__ solvers,
    const int32_t *__restrict__ solver_chunks, const int32_t *__restrict__ solver_prefix,
    const int32_t *__restrict__ perm, const int32_t *__restrict__ tile_solver, float *tiles, float c,
    int *err)
{
    __shared__ int e_col[TILE_W * GRAM_MAX_ROW];
    __shared__ float e_val[TILE_W * GRAM_MAX_ROW];
    __shared__ int r_len[TILE_W];
    __shared__ float r_sgn[TILE_W];
    __shared__ float r_scale[BATCH];
    const int tile = blockIdx.x;
    const int k = tile_solver[tile];
    const SolverDev S = solvers[k];
    const int beta = tile - S.tile_begin;
    const int tid = threadIdx.x;
    if (tid < TILE_W) {
        const int b = tid < BATCH ? beta - 1 : beta;
        const int t = b * BATCH + (tid & (BATCH - 1));
        int lr = -1;
        if (b >= 0 && t < S.n_rows) lr = perm[S.perm_off + t];
        const RowSlot s = locate_row(chunks, solver_chunks + S.list_begin, solver_prefix + S.list_begin,
                                     S.n_chunks, S.n_rows, lr, err);
        r_len[tid] = s.len;
        r_sgn[tid] = LOSS == 0 ? s.y : 1.f;
        for (int p = 0; p < s.len; ++p) {
            e_col[tid * GRAM_MAX_ROW + p] = s.col[p];
            e_val[tid * GRAM_MAX_ROW + p] = s.val[p];
        }
        if (tid >= BATCH)
            r_scale[tid - BATCH] = s.len == 0 ? 0.f : (LOSS == 0 ? -1.f / s.q : -1.f / (c + s.q));
    }
    __syncthreads();
    float *out = tiles + (int64_t)tile * TILE_FLOATS;
    for (int idx = tid; idx < TILE_FLOATS; idx += 256) {
        const int jp = idx >> 6, i = idx & 63;
        float g = 0.f;
        if (jp < BATCH || jp - BATCH < i) {
            const int *ca = e_col + (BATCH + i) * GRAM_MAX_ROW, *cb = e_col + jp * GRAM_MAX_ROW;
            const float *va = e_val + (BATCH + i) * GRAM_MAX_ROW, *vb = e_val + jp * GRAM_MAX_ROW;
            const int la = r_len[BATCH + i], lb = r_len[jp];
            int pa = 0, pb = 0;
            while (pa < la && pb < lb) {
                const int x = ca[pa], yv = cb[pb];
                if (x == yv) { g += va[pa] * vb[pb]; ++pa; ++pb; }
                else if (x < yv) ++pa;
                else ++pb;
            }
            g *= r_scale[i] * r_sgn[BATCH + i] * r_sgn[jp];
        }
        out[idx] = g;
    }
}

// ------------------------------------------------------------------------------------------------
// Workgroup-internal barrier among the helper wavefronts only (the chain wavefront keeps running).
// cnt lives in LDS and only grows; target = arrivals expected so far.
__device__ __forceinline__ void helper_barrier(int *cnt, int target)
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    if ((threadIdx.x & 63) == 0) atomicAdd(cnt, 1);
    while (__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < target)
        __builtin_amdgcn_s_sleep(1);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

template <int LOSS>
__device__ __forceinline__ float clamp_step(float t, float lo, float hi)
{
    return LOSS == 0 ? __builtin_amdgcn_fmed3f(t, lo, hi) : t;
}

struct BatchedShared {
    RowSlot rows[RING][BATCH];
    float t0[RING][BATCH], lo[RING][BATCH], hi[RING][BATCH];
    float delta[2][BATCH];
    float Tw[2][BATCH][BATCH];   // own part of block i's T: [j][lane]
    float Tx[2][BATCH][BATCH];   // cross part of block i+1's T: [j][lane]
    int hb;
};

// The chain: 64 sequential steps of one block.  Lane i owns row i.
template <int LOSS>
__device__ __forceinline__ void chain_block(BatchedShared &sh, int i, int lane, float &x_carry)
{
    const int ring = i & (RING - 1), buf = i & 1;
    float t = sh.t0[ring][lane] + x_carry;
    const float lo = sh.lo[ring][lane], hi = sh.hi[ring][lane];
    float x = 0.f;
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
        const float d = clamp_step<LOSS>(t, lo, hi);
        const float s = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(d), j));
        t = fmaf(s, sh.Tw[buf][j][lane], t);
        x = fmaf(s, sh.Tx[buf][j][lane], x);
    }
    sh.delta[buf][lane] = clamp_step<LOSS>(t, lo, hi);
    x_carry = x;
}

// One workgroup per solver: wavefront 0 runs the chain, the others gather, scatter and stage.
// Dynamic LDS: BatchedShared, then max_list chunk descriptors and max_list local-row prefixes.
template <int LOSS>
__global__ __launch_bounds__(BATCHED_THREADS) void sdca_batched_csr(
    const ChunkDev *__restrict__ chunks, const SolverDev *__restrict__ solvers,
    const int32_t *__restrict__ solver_chunks, const int32_t *__restrict__ solver_prefix,
    const int32_t *__restrict__ perm, const float *__restrict__ tiles, float *u_all, int64_t ld_v,
    int max_list, RoundScalars sc, int *err)
{
    extern __shared__ __align__(16) unsigned char smem[];
    BatchedShared &sh = *reinterpret_cast<BatchedShared *>(smem);
    ChunkDev *l_desc = reinterpret_cast<ChunkDev *>(smem + sizeof(BatchedShared));
    int *l_prefix = reinterpret_cast<int *>(l_desc + max_list);
    const SolverDev S = solvers[blockIdx.x];
    const int tid = threadIdx.x;
    for (int i = tid; i < S.n_chunks; i += BATCHED_THREADS) {
        l_desc[i] = chunks[solver_chunks[S.list_begin + i]];
        l_prefix[i] = solver_prefix[S.list_begin + i];
    }
    if (tid == 0) sh.hb = 0;
    __syncthreads();
    float *u = u_all + (int64_t)blockIdx.x * ld_v;
    const int32_t *pk = perm + S.perm_off;
    const float *my_tiles = tiles + (int64_t)S.tile_begin * TILE_FLOATS;
    const int nb = (S.n_rows + BATCH - 1) / BATCH;
    const bool is_chain = tid < 64;
    const int lane = tid & 63;
    // helper coordinates
    const int hl = tid - 64, rho = hl >> 3, sub = hl & (LPR - 1);

    // helper pipeline registers
    int p_cur = -1, p_next = -1;                 // visiting-order entries (sub == 0 lanes)
    int m_ci = -1, m_r = 0, m_rp0 = 0, m_rp1 = 0;   // row being resolved: loads in flight
    float m_q = 0.f, m_y = 0.f, m_a = 0.f, m_zw = 0.f;
    int g_col[ENT], s_col[ENT], gn_col[ENT], sn_col[ENT];
    float g_val[ENT], s_val[ENT], gn_val[ENT], sn_val[ENT];
#pragma unroll
    for (int e = 0; e < ENT; ++e) {
        g_col[e] = s_col[e] = gn_col[e] = sn_col[e] = 0;
        g_val[e] = s_val[e] = gn_val[e] = sn_val[e] = 0.f;
    }
    float x_carry = 0.f;
    int hb_target = 0;

    for (int i = -5; i <= nb; ++i) {
        if (is_chain) {
            if (i >= 0 && i < nb) chain_block<LOSS>(sh, i, lane, x_carry);
        } else {
            // 1. publish the row of block i + 3 whose state loads were issued last iteration
            if (sub == 0 && i + 3 >= 0 && i + 3 < nb) {
                RowSlot s;
                s.col = nullptr; s.val = nullptr; s.alpha_p = nullptr; s.len = 0;
                s.y = m_y; s.alpha = m_a; s.q = m_q; s.zw = m_zw;
                const int len = m_rp1 - m_rp0;
                if (m_ci >= 0 && m_q != 0.f && len > 0 && len <= GRAM_MAX_ROW) {
                    const ChunkDev &ch = l_desc[m_ci];
                    s.col = ch.col + m_rp0; s.val = ch.val + m_rp0; s.alpha_p = ch.alpha + m_r;
                    s.len = len;
                }
                sh.rows[(i + 3) & (RING - 1)][rho] = s;
            }
            // 2. issue the state loads of block i + 4 from the order entry read last iteration
            m_ci = -1;
            if (sub == 0 && i + 4 >= 0 && i + 4 < nb && p_cur >= 0) {
                if (p_cur >= S.n_rows) {
                    atomicOr(err, ERR_PERM_RANGE);
                } else {
                    m_ci = find_chunk(l_prefix, S.n_chunks, p_cur);
                    m_r = p_cur - l_prefix[m_ci];
                    const ChunkDev &ch = l_desc[m_ci];
                    m_rp0 = ch.row_ptr[m_r]; m_rp1 = ch.row_ptr[m_r + 1];
                    m_q = ch.q[m_r]; m_y = ch.y[m_r]; m_a = ch.alpha[m_r]; m_zw = ch.zw[m_r];
                }
            }
            // 3. read the order entry of block i + 5
            p_next = -1;
            if (sub == 0 && i + 5 >= 0 && i + 5 < nb) {
                const int t = (i + 5) * BATCH + rho;
                if (t < S.n_rows) p_next = pk[t];
            }
            // 4. fetch the entries of block i + 2 (for its gather) and of block i (for its scatter)
#pragma unroll
            for (int e = 0; e < ENT; ++e) { gn_col[e] = 0; gn_val[e] = 0.f; sn_col[e] = 0; sn_val[e] = 0.f; }
            if (i + 2 >= 0 && i + 2 < nb) {
                const RowSlot &r = sh.rows[(i + 2) & (RING - 1)][rho];
                const int len = r.len;
#pragma unroll
                for (int e = 0; e < ENT; ++e) {
                    const int p = sub + e * LPR;
                    if (p < len) { gn_col[e] = r.col[p]; gn_val[e] = r.val[p]; }
                }
            }
            if (i >= 0 && i < nb) {
                const RowSlot &r = sh.rows[i & (RING - 1)][rho];
                const int len = r.len;
#pragma unroll
                for (int e = 0; e < ENT; ++e) {
                    const int p = sub + e * LPR;
                    if (p < len) { sn_col[e] = r.col[p]; sn_val[e] = r.val[p]; }
                }
            }
            // tile staging loads for iteration i + 1: own part of T(i+1), cross part of T(i+2)
            float4 tw_a = make_float4(0.f, 0.f, 0.f, 0.f), tw_b = tw_a, tx_a = tw_a, tx_b = tw_a;
            if (i + 1 >= 0 && i + 1 < nb) {
                const float4 *src = reinterpret_cast<const float4 *>(
                    my_tiles + (int64_t)(i + 1) * TILE_FLOATS + BATCH * BATCH);
                tw_a = src[hl]; tw_b = src[hl + 512];
            }
            if (i + 2 >= 0 && i + 2 < nb) {
                const float4 *src = reinterpret_cast<const float4 *>(my_tiles + (int64_t)(i + 2) * TILE_FLOATS);
                tx_a = src[hl]; tx_b = src[hl + 512];
            }
            // 5. scatter block i - 1: alpha and the private vector
            if (i - 1 >= 0 && i - 1 < nb) {
                const RowSlot &r = sh.rows[(i - 1) & (RING - 1)][rho];
                const float dl = sh.delta[(i - 1) & 1][rho];
                if (r.len > 0 && dl != 0.f) {
                    const float coef = dl * (LOSS == 0 ? r.y : 1.f) * sc.inv_c;
#pragma unroll
                    for (int e = 0; e < ENT; ++e)
                        if (sub + e * LPR < r.len) unsafeAtomicAdd(&u[s_col[e]], coef * s_val[e]);
                    if (sub == 0) {
                        float an = r.alpha + dl;
                        if (LOSS == 0) an = fminf(fmaxf(an, 0.f), 1.f);
                        *r.alpha_p = an;
                    }
                }
            }
            // 6. all scatters of block i - 1 are performed before any gather of block i + 1
            hb_target += HELPER_WAVES;
            helper_barrier(&sh.hb, hb_target);
            // 7. gather block i + 1 against the private vector (blocks <= i - 1 applied)
            if (i + 1 >= 0 && i + 1 < nb) {
                const RowSlot &r = sh.rows[(i + 1) & (RING - 1)][rho];
                float part = 0.f;
#pragma unroll
                for (int e = 0; e < ENT; ++e)
                    if (sub + e * LPR < r.len)
                        part += g_val[e] * __hip_atomic_load(&u[g_col[e]], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                part += __shfl_xor(part, 1, 64);
                part += __shfl_xor(part, 2, 64);
                part += __shfl_xor(part, 4, 64);
                if (sub == 0) {
                    const int ring = (i + 1) & (RING - 1);
                    float t0 = 0.f, lo = 0.f, hi = 0.f;
                    if (r.len > 0) {
                        const float z = r.zw + part;
                        if (LOSS == 0) {
                            t0 = (sc.c / r.q) * (1.f - r.y * z);
                            lo = -r.alpha; hi = 1.f - r.alpha;
                        } else {
                            t0 = (sc.c / (sc.c + r.q)) * (r.y - r.alpha - z);
                        }
                    }
                    sh.t0[ring][rho] = t0; sh.lo[ring][rho] = lo; sh.hi[ring][rho] = hi;
                }
            }
            // 8. publish the staged tile parts for iteration i + 1
            {
                const int buf = (i + 1) & 1;
                float4 *dw = reinterpret_cast<float4 *>(&sh.Tw[buf][0][0]);
                float4 *dx = reinterpret_cast<float4 *>(&sh.Tx[buf][0][0]);
                dw[hl] = tw_a; dw[hl + 512] = tw_b;
                dx[hl] = tx_a; dx[hl + 512] = tx_b;
            }
            // 9. rotate the pipeline registers
#pragma unroll
            for (int e = 0; e < ENT; ++e) {
                g_col[e] = gn_col[e]; g_val[e] = gn_val[e];
                s_col[e] = sn_col[e]; s_val[e] = sn_val[e];
            }
            p_cur = p_next;
        }
        __syncthreads();
    }
}

}  // namespace chicle
