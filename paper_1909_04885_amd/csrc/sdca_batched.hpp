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
// three dependent instructions per step in one wavefront (lane i owns t_i).  The logistic loss keeps
// m_i = -y_i z_i in place of t_i and solves each step's scalar equation inside the recurrence.  The dot products with
// the private vector (gather), the alpha updates and the scatter into the private vector are done a
// block at a time by the other wavefronts of the workgroup, off the critical path; the matrices T
// depend on the data and the visiting order only and are produced beforehand by a separate kernel
// that runs on the whole chip.  Block b's dot products see the private vector with blocks <= b-2
// applied; block b-1 enters through the cross part of T.  Exact arithmetic gives the row-wise
// solver's result; in floating point only the summation order differs.
#pragma once
#include <hip/hip_runtime.h>
#include "device_types.hpp"
#include "mem.hpp"
#include "sdca_rowwise.hpp"

namespace chicle {

constexpr int BATCH = 64;                    // rows per block = lanes of the chain wavefront
constexpr int TILE_W = 2 * BATCH;            // T rows: previous block (cross part), then own block
constexpr int TILE_FLOATS = BATCH * TILE_W;  // layout [jp][i]: jp in [0,128), i in [0,64)
constexpr int GRAM_MAX_ROW = 48;             // longest sparse row the batched solver accepts
constexpr int LPR = 8;                       // helper lanes per row
constexpr int ENT = GRAM_MAX_ROW / LPR;      // entries per helper lane
constexpr int HELPER_WAVES = BATCH * LPR / 64;
constexpr int SERVICE_WAVES = 2;              // row resolution and tile staging
constexpr int BATCHED_THREADS = 64 + BATCH * LPR + 64 * SERVICE_WAVES;
constexpr int RING = 8;
// The head of the private vector (popular columns) is kept in LDS for the whole pass, in double: LDS
// atomic adds on doubles run at the rate of the LDS pipeline on this hardware, those on floats are
// serialised lane by lane (about 3 cycles per lane).  It takes whatever LDS the rest leaves free.
constexpr int LDS_BYTES = 160 * 1024;
constexpr int WARM_AHEAD = 6;                 // blocks a warming workgroup may run ahead of its solver
constexpr int WARM_WAVES = 4;                 // its wavefronts at work

// What the helpers know about one row of a block.
struct RowSlot {
    const int32_t *col;   // always readable for ENT * LPR entries (a dummy row when len = 0)
    const float *val;
    RowState *st;
    int len;              // 0 for a missing, empty or rejected row
    float y, alpha, q, rw;
};

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
    int dead;                    // split solver: a wait for a partner workgroup has given up
    int xflag;                   // split solver: iteration whose ring words are in xv
    int gcount;                  // split solver, tail: helper wavefronts whose gathered values have arrived
    float xv[BATCH];             // split solver: what the partner sent (steps, or partial dot products)
};

// The chain: 64 sequential steps of one block.  Lane i owns row i.
template <int LOSS>
__device__ __forceinline__ void chain_block(BatchedShared &sh, int i, int lane, float &x_carry, float inv_c)
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

// The same for the logistic loss, whose step has no closed form.  Lane i owns m_i = -y_i z_i; step j is
// solved by the whole wavefront from lane j's values, then
//     m_i += delta_j T_ij,   T_ij = -y_i y_j G_ij / c.
// The helpers have solved every row's equation for its m at the start of the block (slot t0; the root in
// slot lo).  The root moves in the direction of m and by no more (ds/dm = 1 / (1 + r a'(1 - a')) lies in
// (0, 1]), so by the time of the row's turn it lies between the old root and the old root + (m - t0): a
// bracket as narrow as the block's own corrections, for which one evaluation is usually enough.
template <>
__device__ __forceinline__ void chain_block<2>(BatchedShared &sh, int i, int lane, float &x_carry, float inv_c)
{
    const int ring = i & (RING - 1), buf = i & 1;
    const float m0 = sh.t0[ring][lane], s0 = sh.lo[ring][lane];
    float m = m0 + x_carry;
    const RowSlot &row = sh.rows[ring][lane];
    const float a = row.alpha, r = row.len > 0 ? row.q * inv_c : 0.f;      // r = 0 marks a row to skip
    float x = 0.f, mine = 0.f;
#pragma unroll 2
    for (int j = 0; j < BATCH; ++j) {
        const float mj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m), j));
        const float aj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a), j));
        const float rj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(r), j));
        const float dm = mj - __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m0), j));
        const float sj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s0), j));
        float d = 0.f;
        if (rj > 0.f) d = logistic_step_wave(mj, rj, aj, sj + fminf(dm, 0.f), fabsf(dm), lane);
        m = fmaf(d, sh.Tw[buf][j][lane], m);
        x = fmaf(d, sh.Tx[buf][j][lane], x);
        mine = lane == j ? d : mine;
    }
    sh.delta[buf][lane] = mine;
    x_carry = x;
}

// One workgroup per solver: wavefront 0 runs the chain, eight wavefronts gather and scatter, two
// resolve the rows of coming blocks and stage the tiles.
// Dynamic LDS: BatchedShared, then max_list chunk descriptors, max_list local-row prefixes, then (at byte offset hot_off) n_hot doubles.
template <int LOSS>
__global__ __launch_bounds__(BATCHED_THREADS) void sdca_batched_csr(
    const ChunkDev *__restrict__ chunks, const SolverDev *__restrict__ solvers,
    const int32_t *__restrict__ solver_chunks, const int32_t *__restrict__ solver_prefix,
    const int32_t *__restrict__ perm, const float *__restrict__ tiles, float *u_all, int64_t ld_v,
    const int64_t *__restrict__ u_off, int max_list, int n_hot, int hot_off, RoundScalars sc, int *err, int *progress, int first_warmer)
{
    extern __shared__ __align__(16) unsigned char smem[];
    BatchedShared &sh = *reinterpret_cast<BatchedShared *>(smem);
    ChunkDev *l_desc = reinterpret_cast<ChunkDev *>(smem + sizeof(BatchedShared));
    int *l_prefix = reinterpret_cast<int *>(l_desc + max_list);
    // Workgroups [0, K) are the solvers; workgroup first_warmer + k runs ahead of solver k and only reads
    // what that solver is about to read, so that the data is in the L2 both share (first_warmer is a
    // multiple of the number of L2 partitions workgroups are dealt over).
    const bool warmer = (int)blockIdx.x >= first_warmer;
    const int sid = warmer ? (int)blockIdx.x - first_warmer : (int)blockIdx.x;
    if (sid >= sc.K) return;
    const SolverDev S = solvers[sid];
    const int tid = threadIdx.x;
    if (!warmer) stamp_solver(sc, sid, 0);
    for (int i = tid; i < S.n_chunks; i += BATCHED_THREADS) {
        l_desc[i] = chunks[solver_chunks[S.list_begin + i]];
        if (u_off) l_desc[i].col = chunk_compact_ids(l_desc[i]);     // compact private vector: its indices, not column ids
        l_prefix[i] = solver_prefix[S.list_begin + i];
    }
    if (warmer) {
        // WARM_WAVES wavefronts, one block each in turn, one lane per row: order entry -> row extent ->
        // column ids -> the private vector's lines outside the LDS-resident head.  Nothing is kept.
        __syncthreads();
        const int wv = tid >> 6, ln = tid & 63;
        if (wv >= WARM_WAVES) return;
        const int n_blocks = (S.n_rows + BATCH - 1) / BATCH;
        const float *uw = u_off ? u_all + u_off[sid] : u_all + (int64_t)sid * ld_v;
        const int32_t *pkw = perm + S.perm_off;
        for (int b = wv; b < n_blocks; b += WARM_WAVES) {
            // stay within WARM_AHEAD blocks of the solver (its last value ends every wait)
            while (__hip_atomic_load(progress + sid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) + WARM_AHEAD < b)
                __builtin_amdgcn_s_sleep(16);
            const int t = b * BATCH + ln;
            if (t >= S.n_rows) continue;
            const int p = pkw[t];
            if (p < 0 || p >= S.n_rows) continue;
            const int ci = find_chunk(l_prefix, S.n_chunks, p);
            const int r = p - l_prefix[ci];
            const ChunkDev &ch = l_desc[ci];
            const int2_a4 rp = gld2(ch.row_ptr + r);
            const int len = min(rp.y - rp.x, GRAM_MAX_ROW);
            if (len <= 0) continue;
            float sink = 0.f;
            for (int e = 0; e < len; e += 16) sink += gld(ch.val + rp.x + e);      // one touch per 64 bytes
            int cc[GRAM_MAX_ROW];
#pragma unroll
            for (int e = 0; e < GRAM_MAX_ROW; ++e) cc[e] = gld(ch.col + rp.x + min(e, len - 1));   // all in flight
            float uv[GRAM_MAX_ROW];
#pragma unroll
            for (int e = 0; e < GRAM_MAX_ROW; ++e) {
                uv[e] = 0.f;
                if (cc[e] >= n_hot) uv[e] = uw[cc[e]];
            }
#pragma unroll
            for (int e = 0; e < GRAM_MAX_ROW; ++e) sink += uv[e];
            asm volatile("" ::"v"(sink));
        }
        return;
    }
    // columns [0, n_hot) of the private vector live here for the whole pass (it starts at zero)
    double *hot = reinterpret_cast<double *>(smem + hot_off);
    for (int i = tid; i < n_hot; i += BATCHED_THREADS) hot[i] = 0.0;
    if (tid == 0) sh.hb = 0;
    __syncthreads();
    float *u = u_off ? u_all + u_off[sid] : u_all + (int64_t)sid * ld_v;
    const int32_t *pk = perm + S.perm_off;
    const float *my_tiles = tiles + (int64_t)S.tile_begin * TILE_FLOATS;
    const int nb = (S.n_rows + BATCH - 1) / BATCH;
    // roles: wavefront 0 runs the chain, 1..8 gather and scatter, 9..10 resolve rows and stage tiles
    const bool is_chain = tid < 64;
    const bool is_service = tid >= 64 + BATCH * LPR;
    const int lane = tid & 63;
    const int hl = tid - 64, rho = hl / LPR, sub = hl & (LPR - 1);     // helper coordinates
    const int sw = (tid - 64 - BATCH * LPR) >> 6;                     // service wavefront 0 or 1

    // service pipeline registers (wavefront 9: one lane per row of a block)
    int p_cur = -1;                                  // visiting-order entry read last iteration
    int m_ci = -1, m_r = 0;                          // row being resolved: loads in flight
    int2_a4 m_rp = {0, 0};
    float4_v m_st = {0.f, 0.f, 0.f, 0.f};          // kept whole until it is used (y, alpha, q, rw)
    // Entries of a row segment (ENT consecutive entries per helper lane) travel through four stages:
    // in (loads in flight) -> g (gathered this iteration) -> c (its block is in the chain) -> s (scattered).
    int in_c[ENT], g_c[ENT], c_c[ENT], s_c[ENT];
    float in_v[ENT], g_v[ENT], c_v[ENT], s_v[ENT];
#pragma unroll
    for (int e = 0; e < ENT; ++e) {
        in_c[e] = g_c[e] = c_c[e] = s_c[e] = 0;
        in_v[e] = g_v[e] = c_v[e] = s_v[e] = 0.f;
    }
    int in_len = 0;
    float x_carry = 0.f;
    int hb_target = 0;
    float4 stage[16];                                // service wavefronts: tile part fetched ahead
    bool staged = false;
    if (nb == 0) {                                   // a solver without rows (uniform for the workgroup)
        stamp_solver(sc, sid, 1);
        return;
    }

    for (int i = -5; i <= nb; ++i) {
        if (tid == BATCHED_THREADS - 1 && i > 0)
            __hip_atomic_store(progress + sid, i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (is_chain) {
            if (i >= 0 && i < nb) chain_block<LOSS>(sh, i, lane, x_carry, sc.inv_c);
        } else if (is_service) {
            // tiles for iteration i + 1 (wavefront 9: own part of T(i+1), wavefront 10: cross part of
            // T(i+2), 16 KB each) were fetched into registers during the last iteration
            {
                const int buf = (i + 1) & 1;
                float4 *dst = reinterpret_cast<float4 *>(sw == 0 ? &sh.Tw[buf][0][0] : &sh.Tx[buf][0][0]);
#pragma unroll
                for (int j = 0; j < 16; ++j) dst[lane + 64 * j] = staged ? stage[j] : make_float4(0.f, 0.f, 0.f, 0.f);
            }
            if (sw == 0) {
                // 1. publish the row of block i + 3 whose state loads were issued last iteration
                if (i + 3 >= 0 && i + 3 < nb) {
                    RowSlot s;
                    s.col = l_desc[0].col; s.val = l_desc[0].val; s.st = nullptr; s.len = 0;
                    s.y = m_st.x; s.alpha = m_st.y; s.q = m_st.z; s.rw = m_st.w;
                    const int len = m_rp.y - m_rp.x;
                    if (m_ci >= 0 && s.q != 0.f && len > 0 && len <= GRAM_MAX_ROW) {
                        const ChunkDev &ch = l_desc[m_ci];
                        s.col = ch.col + m_rp.x; s.val = ch.val + m_rp.x; s.st = ch.st + m_r;
                        s.len = len;
                    }
                    sh.rows[(i + 3) & (RING - 1)][lane] = s;
                }
                // 2. issue the state loads of block i + 4 from the order entry read last iteration
                m_ci = -1;
                if (i + 4 >= 0 && i + 4 < nb && (i + 4) * BATCH + lane < S.n_rows) {
                    if (p_cur < 0 || p_cur >= S.n_rows) {
                        atomicOr(err, ERR_PERM_RANGE);
                    } else {
                        m_ci = find_chunk(l_prefix, S.n_chunks, p_cur);
                        m_r = p_cur - l_prefix[m_ci];
                        const ChunkDev &ch = l_desc[m_ci];
                        m_rp = gld2(ch.row_ptr + m_r);
                        m_st = gld_state(ch.st + m_r);
                    }
                }
                // 3. read the order entry of block i + 5 (always some valid position: the value is only
                //    looked at next iteration, under the range test of step 2, so nothing waits for it here)
                p_cur = gld(pk + min(max((i + 5) * BATCH + lane, 0), S.n_rows - 1));
            }
            // the next iteration's tiles are requested once the helpers have issued their scatters: bulk
            // loads then queue behind the gather's loads in the vector memory pipeline, not in front of them
            hb_target += HELPER_WAVES;
            while (__hip_atomic_load(&sh.hb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < hb_target)
                __builtin_amdgcn_s_sleep(2);
            {
                const int tb = sw == 0 ? i + 2 : i + 3;
                staged = tb >= 0 && tb < nb;
                if (staged) {
                    const float4 *src = reinterpret_cast<const float4 *>(
                        my_tiles + (int64_t)tb * TILE_FLOATS + (sw == 0 ? BATCH * BATCH : 0));
#pragma unroll
                    for (int j = 0; j < 16; ++j) stage[j] = src[lane + 64 * j];
                }
            }
        } else {
            // 4. fetch this lane's segment of the row of block i + 2 (unconditional vector loads; the
            //    entries beyond the row's length are masked when the set moves on)
            if (i + 2 >= 0 && i + 2 < nb) {
                const RowSlot &r = sh.rows[(i + 2) & (RING - 1)][rho];
                // lane sub takes positions sub, sub + 8, ...: the row is sorted by column popularity, so
                // for one e the eight lanes of a row hold neighbouring ranks and the split "popular
                // column in LDS / other column in HBM" is nearly uniform over the wavefront
                const int32_t *cp = r.col + sub;
                const float *vp = r.val + sub;
                in_len = r.len;
#pragma unroll
                for (int e = 0; e < ENT; ++e) { in_c[e] = gld(cp + e * LPR); in_v[e] = gld(vp + e * LPR); }
            } else {
                in_len = 0;
            }
            // 5. scatter block i - 1: alpha and the private vector (masked entries carry value 0)
            if (i - 1 >= 0 && i - 1 < nb) {
                const RowSlot &r = sh.rows[(i - 1) & (RING - 1)][rho];
                const float dl = sh.delta[(i - 1) & 1][rho];
                if (r.len > 0 && dl != 0.f) {
                    const float coef = dl * (LOSS == 1 ? 1.f : r.y) * sc.inv_c;
#pragma unroll
                    for (int e = 0; e < ENT; ++e)
                        if (s_v[e] != 0.f) {
                            if (s_c[e] < n_hot) atomicAdd(&hot[s_c[e]], (double)(coef * s_v[e]));
                            else unsafeAtomicAdd(&u[s_c[e]], coef * s_v[e]);
                        }
                    if (sub == 0) {
                        float an = r.alpha + dl;
                        if (LOSS != 1) an = fminf(fmaxf(an, 0.f), 1.f);
                        gst(&r.st->alpha, an);
                    }
                }
            }
            // 6. all scatters of block i - 1 are performed before any gather of block i + 1
            hb_target += HELPER_WAVES;
            helper_barrier(&sh.hb, hb_target);
            // 7. gather block i + 1 against the private vector (blocks <= i - 1 applied)
            if (i + 1 >= 0 && i + 1 < nb) {
                const RowSlot &r = sh.rows[(i + 1) & (RING - 1)][rho];
                // All loads are issued before the first use so that one round trip covers the gather;
                // cold_v and hot_v are separate so that neither branch has to wait for its own load.
                // Masked entries hold value 0 and are skipped.
                float cold_v[ENT], hot_v[ENT];
#pragma unroll
                for (int e = 0; e < ENT; ++e) {
                    cold_v[e] = 0.f;
                    if (g_v[e] != 0.f && g_c[e] >= n_hot)
                        cold_v[e] = __hip_atomic_load(u + g_c[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
#pragma unroll
                for (int e = 0; e < ENT; ++e) {
                    hot_v[e] = 0.f;
                    if (g_v[e] != 0.f && g_c[e] < n_hot) hot_v[e] = (float)hot[g_c[e]];
                }
                float part = 0.f;
#pragma unroll
                for (int e = 0; e < ENT; ++e) part += g_v[e] * (cold_v[e] + hot_v[e]);
#pragma unroll
                for (int o = 1; o < LPR; o <<= 1) part += __shfl_xor(part, o, 64);
                if (sub == 0) {
                    const int ring = (i + 1) & (RING - 1);
                    float t0 = 0.f, lo = 0.f, hi = 0.f;
                    if (r.len > 0) {
                        if (LOSS == 0) {
                            t0 = (sc.c / r.q) * (r.rw - r.y * part);
                            lo = -r.alpha; hi = 1.f - r.alpha;
                        } else if (LOSS == 1) {
                            t0 = (sc.c / (sc.c + r.q)) * (r.rw - r.alpha - part);
                        } else {
                            t0 = r.rw - r.y * part;
                            const float rr = r.q * sc.inv_c;
                            logistic_step(t0, rr, r.alpha, t0 + rr * (r.alpha - 0.5f), &lo);   // lo: the root for t0
                        }
                    }
                    sh.t0[ring][rho] = t0; sh.lo[ring][rho] = lo; sh.hi[ring][rho] = hi;
                }
            }
            // 8. move the entry sets one stage on; the incoming set is masked to the row's length
#pragma unroll
            for (int e = 0; e < ENT; ++e) {
                s_c[e] = c_c[e]; s_v[e] = c_v[e];
                c_c[e] = g_c[e]; c_v[e] = g_v[e];
                const bool live = sub + e * LPR < in_len;
                g_c[e] = live ? in_c[e] : 0;
                g_v[e] = live ? in_v[e] : 0.f;
            }
        }
        __syncthreads();
    }
    for (int i = tid; i < n_hot; i += BATCHED_THREADS) u[i] = (float)hot[i];
    stamp_solver(sc, sid, 1);
}

}  // namespace chicle
