// Batched local solver with every solver spread over two or three compute units (paper Section 4.2: a
// solver may use all the processors of its node; Section 2.2: L = 1, the coordinate steps keep their order).
//
// One compute unit gets a memory request served every few cycles, whatever its size.  Per block of 64 steps
// the single-workgroup solver (sdca_batched.hpp) asks for the block's entries, its tile of T, and for some
// five hundred lonely 4-byte reads and as many atomic adds in the unpopular part of the private vector; the
// last two take about half of its requests and it waits for both inside every block.  Here the columns of
// the private vector are divided:
//   - the head workgroup keeps the popular columns [0, n_hot) in LDS, runs the recurrence, stages the tiles;
//     its gathers and scatters touch LDS only;
//   - one or two tail workgroups on the same L2 partition own the other columns (two: by parity), in memory.
// For every block the tail hands the head 64 partial dot products and the head hands the tail the 64 steps,
// through rings of 64-bit words in memory.  A word carries its value together with the number of the block
// it belongs to, so no fence is needed; every wait is bounded: a workgroup that waits too long raises the
// error flag, stops waiting for the rest of the pass and finishes.
//
// The order of operations is that of the single-workgroup solver: block b's dot products see the private
// vector with blocks <= b-2 applied, block b-1 enters through the cross part of T.
#pragma once
#include <hip/hip_runtime.h>
#include "device_types.hpp"
#include "mem.hpp"
#include "sdca_batched.hpp"

namespace chicle {

constexpr int SPLIT_RING = 8;                  // blocks a ring holds
constexpr int SPLIT_MAX_TAILS = 2;
constexpr int SPLIT_WORDS = (1 + SPLIT_MAX_TAILS) * SPLIT_RING * BATCH + 8;   // 64-bit words per solver
constexpr int SPLIT_SPIN_LIMIT = 1 << 22;      // polls before a wait for the partner gives up
constexpr int SPLIT_THREADS = BATCHED_THREADS + 64;   // the single-workgroup solver's wavefronts and one that polls the rings

__device__ __forceinline__ void ring_put(unsigned long long *p, float v, int tag)
{
    const unsigned long long w = ((unsigned long long)(unsigned)tag << 32) | (unsigned long long)__float_as_uint(v);
    __hip_atomic_store(p, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The wait of a polling wavefront (all 64 lanes, one ring word each), with several polls in flight: a poll is
// a trip to L2 and back, so with one at a time an arrival is noticed a trip and a half later on average;
// with POLL_DEPTH of them, issued a fraction of a trip apart, the one that sees it is already on its way.
// PROGRESS: the same polls also fetch two progress words of the other tail, and the wait ends when the ring
// words carry `tag` and those words have reached want_added / want_gathered.  Bounded: after SPLIT_SPIN_LIMIT
// polls the wait gives up, raises the error flag and sets *dead (LDS), which makes every later wait of the
// workgroup return at once, so a lost partner costs one time-out, not one per block.
constexpr int POLL_DEPTH = 1;
template <bool PROGRESS>
__device__ __forceinline__ float ring_wait(const unsigned long long *word, int tag, const unsigned long long *added,
                                           int want_added, const unsigned long long *gathered, int want_gathered,
                                           int *dead, int *err)
{
    unsigned long long v[POLL_DEPTH], a[POLL_DEPTH], g[POLL_DEPTH];
#define RING_POLL(k)                                                                                        \
    do {                                                                                                    \
        v[k] = __hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);                         \
        if (PROGRESS) {                                                                                     \
            a[k] = __hip_atomic_load(added, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);                    \
            g[k] = __hip_atomic_load(gathered, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);                 \
        }                                                                                                   \
    } while (0)
#pragma unroll
    for (int k = 0; k < POLL_DEPTH; ++k) {
        RING_POLL(k);
        if (k + 1 < POLL_DEPTH) __builtin_amdgcn_s_sleep(2);
    }
    int spins = 0;
    for (;;) {
#pragma unroll
        for (int k = 0; k < POLL_DEPTH; ++k) {
            bool ok = (int)(v[k] >> 32) == tag;
            if (PROGRESS) ok = ok && (int)a[k] >= want_added && (int)g[k] >= want_gathered;
            if (__builtin_amdgcn_ballot_w64(!ok) == 0ull) return __uint_as_float((unsigned)v[k]);   // every lane's word is here
            if (POLL_DEPTH == 1) __builtin_amdgcn_s_sleep(1);
            RING_POLL(k);
        }
        spins += POLL_DEPTH;
        if (spins > SPLIT_SPIN_LIMIT || __hip_atomic_load(dead, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)) {
            if (spins > SPLIT_SPIN_LIMIT) {
                __hip_atomic_store(dead, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                atomicOr(err, ERR_PARTNER_TIMEOUT);
            }
            return 0.f;
        }
    }
#undef RING_POLL
}

// Barrier among the helper wavefronts that orders their LDS traffic only (it does not wait for loads from
// memory that are still in flight).
__device__ __forceinline__ void helper_barrier_lds(int *cnt, int target)
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if ((threadIdx.x & 63) == 0) atomicAdd(cnt, 1);
    while (__hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < target)
        __builtin_amdgcn_s_sleep(1);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}

// Sum over the LPR = 8 lanes that share a row, in every one of them, by data-parallel-primitive moves (the
// neighbour inside pairs, the other pair of the quad, then the mirrored half of the eight): register to
// register, where a shuffle goes through the LDS crossbar and costs a trip's latency each time.
__device__ __forceinline__ float sum_over_row_lanes(float v)
{
    static_assert(LPR == 8, "the moves below cover groups of eight lanes");
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, false));   // row_half_mirror
    return v;
}

// Wait until an LDS word that only grows has reached `target`.
__device__ __forceinline__ void wait_flag(const int *flag, int target)
{
    while (__hip_atomic_load(flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) < target)
        __builtin_amdgcn_s_sleep(1);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
}

// The row resolver both kinds of workgroup run in one wavefront (one lane per row of a block).  A workgroup
// works through the blocks first, first + stride, ...; call x publishes the rows of its (x+3)-th block,
// requests row extents and state of the (x+4)-th and reads the order entries of the (x+5)-th.  Its registers
// live across iterations.
struct RowResolver {
    int p_cur = -1, m_ci = -1, m_r = 0;
    int2_a4 m_rp = {0, 0};
    float4_v m_st = {0.f, 0.f, 0.f, 0.f};

    __device__ __forceinline__ void step(RowSlot (*rows)[BATCH], int ring_mask, const ChunkDev *l_desc,
                                         const int *l_prefix, const SolverDev &S, const int32_t *pk, int x, int first,
                                         int stride, int n_own, int lane, int *err, bool report)
    {
        if (x + 3 >= 0 && x + 3 < n_own) {
            RowSlot s;
            s.col = l_desc[0].col; s.val = l_desc[0].val; s.st = nullptr; s.len = 0;
            s.y = m_st.x; s.alpha = m_st.y; s.q = m_st.z; s.rw = m_st.w;
            const int len = m_rp.y - m_rp.x;
            if (m_ci >= 0 && s.q != 0.f && len > 0 && len <= GRAM_MAX_ROW) {
                const ChunkDev &ch = l_desc[m_ci];
                s.col = ch.col + m_rp.x; s.val = ch.val + m_rp.x; s.st = ch.st + m_r;
                s.len = len;
            }
            rows[(x + 3) & ring_mask][lane] = s;
        }
        m_ci = -1;
        if (x + 4 >= 0 && x + 4 < n_own && (first + stride * (x + 4)) * BATCH + lane < S.n_rows) {
            if (p_cur < 0 || p_cur >= S.n_rows) {
                if (report) atomicOr(err, ERR_PERM_RANGE);
            } else {
                m_ci = find_chunk(l_prefix, S.n_chunks, p_cur);
                m_r = p_cur - l_prefix[m_ci];
                const ChunkDev &ch = l_desc[m_ci];
                m_rp = gld2(ch.row_ptr + m_r);
                m_st = gld_state(ch.st + m_r);
            }
        }
        // always some valid position: the value is only looked at next iteration, under the range test above
        p_cur = gld(pk + min(max((first + stride * (x + 5)) * BATCH + lane, 0), S.n_rows - 1));
    }
};

struct SplitArgs {
    const ChunkDev *chunks;
    const SolverDev *solvers;
    const int32_t *solver_chunks, *solver_prefix, *perm;
    const float *tiles;
    float *u_all;
    int64_t ld_v;
    const int64_t *u_off;       // compact private vectors: where each solver's starts (else nullptr)
    int max_list, n_hot, hot_off;
    RoundScalars sc;
    int *err;
    int n_tails;
    unsigned long long *xchg_all;
};

// Common start of both kinds of workgroup: the solver's chunk list into LDS.
__device__ __forceinline__ void split_stage_lists(unsigned char *smem, const SplitArgs &A, const SolverDev &S,
                                                  ChunkDev *l_desc, int *l_prefix)
{
    for (int i = threadIdx.x; i < S.n_chunks; i += SPLIT_THREADS) {
        l_desc[i] = A.chunks[A.solver_chunks[S.list_begin + i]];
        if (A.u_off) l_desc[i].col = chunk_compact_ids(l_desc[i]);     // compact private vector: its indices, not column ids
        l_prefix[i] = A.solver_prefix[S.list_begin + i];
    }
}

// ---- the head workgroup: recurrence, tiles, the popular columns in LDS -------------------------------------
// Wavefront 0 runs the chain, 1..8 gather and scatter (LDS only), 9..10 resolve rows and stage the tiles, 11
// fetches the tails' partial sums.  One loop per role, all with the same number of iterations and one
// workgroup barrier per iteration, so that the registers of one role are not kept alive through the code of
// the others.
template <int LOSS>
__device__ __forceinline__ void split_head(unsigned char *smem, const SplitArgs &A, int sid)
{
    BatchedShared &sh = *reinterpret_cast<BatchedShared *>(smem);
    ChunkDev *l_desc = reinterpret_cast<ChunkDev *>(smem + sizeof(BatchedShared));
    int *l_prefix = reinterpret_cast<int *>(l_desc + A.max_list);
    const SolverDev S = A.solvers[sid];
    const RoundScalars &sc = A.sc;
    const int tid = threadIdx.x, n_hot = A.n_hot;
    stamp_solver(sc, sid, 0);
    split_stage_lists(smem, A, S, l_desc, l_prefix);
    double *hot = reinterpret_cast<double *>(smem + A.hot_off);
    for (int i = tid; i < n_hot; i += SPLIT_THREADS) hot[i] = 0.0;
    if (tid == 0) { sh.hb = 0; sh.dead = 0; sh.xflag = 0; }
    __syncthreads();
    float *u = A.u_off ? A.u_all + A.u_off[sid] : A.u_all + (int64_t)sid * A.ld_v;
    const int32_t *pk = A.perm + S.perm_off;
    const float *my_tiles = A.tiles + (int64_t)S.tile_begin * TILE_FLOATS;
    unsigned long long *x_steps = A.xchg_all + (int64_t)sid * SPLIT_WORDS;
    unsigned long long *x_parts = x_steps + SPLIT_RING * BATCH;
    const int nb = (S.n_rows + BATCH - 1) / BATCH;
    const int lane = tid & 63, wave = tid >> 6;
    const int hl = tid - 64, rho = hl / LPR, sub = hl & (LPR - 1);     // helper coordinates
    if (nb == 0) {                                   // a solver without rows (uniform for its workgroups)
        stamp_solver(sc, sid, 1);
        return;
    }
#define HEAD_ITERATIONS for (int i = -6; i <= nb; ++i)
    if (wave == 0) {
        float x_carry = 0.f;
        HEAD_ITERATIONS {
            if (i >= 0 && i < nb) {
                chain_block<LOSS>(sh, i, lane, x_carry, sc.inv_c);
                // the tails add these steps into their columns
                if (A.n_tails > 0) ring_put(x_steps + (i & (SPLIT_RING - 1)) * BATCH + lane, sh.delta[i & 1][lane], i + 1);
            }
            __syncthreads();
        }
    } else if (wave == 11) {
        // What the tail sends for this iteration, fetched by a wavefront that has no other loads in flight
        // (loads return in the order they were issued) and handed on through LDS.
        HEAD_ITERATIONS {
            if (A.n_tails > 0 && i + 1 >= 0 && i + 1 < nb) {
                const int t = (i + 1) % A.n_tails;                   // the tail that owns block i + 1
                sh.xv[lane] = ring_wait<false>(x_parts + (t * SPLIT_RING + ((i + 1) & (SPLIT_RING - 1))) * BATCH + lane, i + 2,
                                               nullptr, 0, nullptr, 0, &sh.dead, A.err);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                if (lane == 0) __hip_atomic_store(&sh.xflag, i + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            __syncthreads();
        }
    } else if (wave >= 9) {
        const int sw = wave - 9;
        RowResolver resolver;
        float4 stage[16];                                // tile part fetched ahead
        bool staged = false;
        HEAD_ITERATIONS {
            // tiles for iteration i + 1 (wavefront 9: own part of T(i+1), wavefront 10: cross part of T(i+2),
            // 16 KB each) were fetched into registers during the last iteration
            const int buf = (i + 1) & 1;
            float4 *dst = reinterpret_cast<float4 *>(sw == 0 ? &sh.Tw[buf][0][0] : &sh.Tx[buf][0][0]);
#pragma unroll
            for (int j = 0; j < 16; ++j) dst[lane + 64 * j] = staged ? stage[j] : make_float4(0.f, 0.f, 0.f, 0.f);
            // (one block further ahead than the tails' resolvers: the helpers ask for a block's entries three
            // iterations before they gather it)
            if (sw == 0) resolver.step(sh.rows, RING - 1, l_desc, l_prefix, S, pk, i + 1, 0, 1, nb, lane, A.err, true);
            const int tb = sw == 0 ? i + 2 : i + 3;
            staged = tb >= 0 && tb < nb;
            if (staged) {
                const float4 *src = reinterpret_cast<const float4 *>(
                    my_tiles + (int64_t)tb * TILE_FLOATS + (sw == 0 ? BATCH * BATCH : 0));
#pragma unroll
                for (int j = 0; j < 16; ++j) stage[j] = src[lane + 64 * j];
            }
            __syncthreads();
        }
    } else {
        // Entries of a row segment (ENT entries per helper lane) travel through five stages:
        // ld (loads in flight) -> ar (arrived: asked for one iteration ago) -> g (gathered this iteration) ->
        // c (its block is in the chain) -> s (scattered).  Loads get a whole iteration before anything looks at
        // them; ld and ar swap register sets from one iteration to the next (nothing moves a register that a
        // load is still due to write).  Only entries in the head's columns are kept; the others are masked when
        // the set leaves ar.
        int a_c[ENT], b_c[ENT], g_c[ENT], c_c[ENT], s_c[ENT];
        float a_v[ENT], b_v[ENT], g_v[ENT], c_v[ENT], s_v[ENT];
#pragma unroll
        for (int e = 0; e < ENT; ++e) {
            a_c[e] = b_c[e] = g_c[e] = c_c[e] = s_c[e] = 0;
            a_v[e] = b_v[e] = g_v[e] = c_v[e] = s_v[e] = 0.f;
        }
        int a_len = 0, b_len = 0, hb_target = 0;
        auto iteration = [&](const int i, int (&ld_c)[ENT], float (&ld_v)[ENT], int &ld_len,
                             const int (&ar_c)[ENT], const float (&ar_v)[ENT], const int ar_len) {
            // 0. what this iteration needs of the rows of blocks i + 3, i - 1 and i + 1 (published at least one
            //    iteration ago) and the steps of block i - 1, read together: one trip to LDS instead of one per use
            const bool has_in = i + 3 >= 0 && i + 3 < nb, has_s = i - 1 >= 0 && i - 1 < nb, has_g = i + 1 >= 0 && i + 1 < nb;
            const RowSlot r_in = sh.rows[(i + 3) & (RING - 1)][rho];
            const RowSlot r_s = sh.rows[(i - 1) & (RING - 1)][rho];
            const RowSlot r_g = sh.rows[(i + 1) & (RING - 1)][rho];
            const float dl = sh.delta[(i - 1) & 1][rho];
            // 1. this lane's segment of the row of block i + 3 (unconditional vector loads)
            if (has_in) {
                const int32_t *cp = r_in.col + sub;
                const float *vp = r_in.val + sub;
                ld_len = r_in.len;
#pragma unroll
                for (int e = 0; e < ENT; ++e) { ld_c[e] = gld(cp + e * LPR); ld_v[e] = gld(vp + e * LPR); }
            } else {
                ld_len = 0;
            }
            // 2. block i - 1 is added to the head of the private vector
            if (has_s && r_s.len > 0 && dl != 0.f) {
                const float coef = dl * (LOSS == 1 ? 1.f : r_s.y) * sc.inv_c;
#pragma unroll
                for (int e = 0; e < ENT; ++e)
                    if (s_v[e] != 0.f) atomicAdd(&hot[s_c[e]], (double)(coef * s_v[e]));
                if (sub == 0) {
                    float an = r_s.alpha + dl;
                    if (LOSS != 1) an = fminf(fmaxf(an, 0.f), 1.f);
                    gst(&r_s.st->alpha, an);
                }
            }
            // 3. ... completely, before block i + 1 is gathered (LDS traffic only)
            hb_target += HELPER_WAVES;
            helper_barrier_lds(&sh.hb, hb_target);
            // 4. gather block i + 1 (blocks <= i - 1 applied)
            if (has_g) {
                float got[ENT];
#pragma unroll
                for (int e = 0; e < ENT; ++e) got[e] = (float)hot[g_c[e]];   // (masked entries: column 0 times 0)
                float part = 0.f;
#pragma unroll
                for (int e = 0; e < ENT; ++e) part += g_v[e] * got[e];
                part = sum_over_row_lanes(part);
                if (sub == 0) {
                    // everything that does not need the tails' share is done before it is waited for: what follows
                    // the wait is on the path between the workgroups
                    const int ring = (i + 1) & (RING - 1);
                    const bool live = r_g.len > 0;
                    float scale = 0.f, lo = 0.f, hi = 0.f;
                    if (live && LOSS == 0) { scale = sc.c / r_g.q; lo = -r_g.alpha; hi = 1.f - r_g.alpha; }
                    if (live && LOSS == 1) scale = sc.c / (sc.c + r_g.q);
                    if (LOSS != 2) { sh.lo[ring][rho] = lo; sh.hi[ring][rho] = hi; }
                    if (A.n_tails > 0) {
                        wait_flag(&sh.xflag, i + 2);
                        part += sh.xv[rho];                               // the tails' share of x_i . u
                    }
                    float t0 = 0.f;
                    if (live) {
                        if (LOSS == 0) {
                            t0 = scale * (r_g.rw - r_g.y * part);
                        } else if (LOSS == 1) {
                            t0 = scale * (r_g.rw - r_g.alpha - part);
                        } else {
                            t0 = r_g.rw - r_g.y * part;
                            const float rr = r_g.q * sc.inv_c;
                            logistic_step(t0, rr, r_g.alpha, t0 + rr * (r_g.alpha - 0.5f), &lo);   // lo: the root for t0
                        }
                    }
                    sh.t0[ring][rho] = t0;
                    if (LOSS == 2) { sh.lo[ring][rho] = lo; sh.hi[ring][rho] = hi; }
                }
            }
            // 5. move the entry sets one stage on; the set that arrived (block i + 2) is masked to the row's
            //    length and to the head's columns
#pragma unroll
            for (int e = 0; e < ENT; ++e) {
                s_c[e] = c_c[e]; s_v[e] = c_v[e];
                c_c[e] = g_c[e]; c_v[e] = g_v[e];
                const bool live = sub + e * LPR < ar_len && ar_c[e] < n_hot;
                g_c[e] = live ? ar_c[e] : 0;
                g_v[e] = live ? ar_v[e] : 0.f;
            }
            __syncthreads();
        };
        for (int i = -6; i <= nb; i += 2) {          // HEAD_ITERATIONS, two at a time
            iteration(i, a_c, a_v, a_len, b_c, b_v, b_len);
            if (i + 1 <= nb) iteration(i + 1, b_c, b_v, b_len, a_c, a_v, a_len);
        }
    }
#undef HEAD_ITERATIONS
    for (int i = tid; i < n_hot; i += SPLIT_THREADS) u[i] = (float)hot[i];
    stamp_solver(sc, sid, 1);
}

// ---- a tail workgroup: the unpopular columns, in memory -----------------------------------------------------
// Tail t of n (n = 1 or 2) owns the blocks t, t + n, t + 2n, ... of its solver: for each of them, in turn, it
// adds the block two before it (whose steps have just arrived) to the private vector, waits until that has
// been performed, gathers the block's dot products and hands them over.  With two tails the block two before
// is the tail's own previous block, and everything older that the other tail adds must have been performed as
// well: each tail publishes the last block it has added, after its fence, and waits for the other's where it
// needs it (that block was added a whole iteration earlier, so the wait is normally over when it begins).
// In the other direction, block b must not be added before the other tail has gathered block b + 1 (which
// sees blocks <= b - 1 only; block b reaches it through T): each tail also publishes the last block it has
// gathered, and an add waits for that.
// A tail works ahead of the head where nothing depends on the steps: it resolves its rows some blocks ahead
// and touches their entries several iterations before either workgroup asks for them, so that both find
// them in the L2 they share.
// Wavefronts 1..8 add and gather, 9 resolves rows, 10 touches entries, 11 waits for the steps (and for the
// other tail); wavefront 0 only keeps the barriers.  TE: entries per helper lane, taken from the end of the
// row, where its unpopular columns are (rows are sorted by popularity): TE * LPR must cover the largest
// number of entries a row has in the tails' columns (checked on the host).
constexpr int TAIL_WARM = 3;                        // iterations the touches run ahead of the tail's own loads
constexpr int TAIL_RING = 2 * RING;                 // resolved rows of the tail's blocks j - 2 .. j + TAIL_WARM + 2

template <int LOSS, int TE>
__device__ __forceinline__ void split_tail(unsigned char *smem, const SplitArgs &A, int sid, int tail)
{
    BatchedShared &sh = *reinterpret_cast<BatchedShared *>(smem);
    ChunkDev *l_desc = reinterpret_cast<ChunkDev *>(smem + sizeof(BatchedShared));
    int *l_prefix = reinterpret_cast<int *>(l_desc + A.max_list);
    RowSlot (*rows)[BATCH] = reinterpret_cast<RowSlot (*)[BATCH]>(smem + A.hot_off);     // the head's place for the popular columns
    const SolverDev S = A.solvers[sid];
    const RoundScalars &sc = A.sc;
    const int tid = threadIdx.x, n_hot = A.n_hot, n_tails = A.n_tails;
    split_stage_lists(smem, A, S, l_desc, l_prefix);
    if (tid == 0) { sh.hb = 0; sh.dead = 0; sh.xflag = 0; sh.gcount = 0; }
    __syncthreads();
    float *u = A.u_off ? A.u_all + A.u_off[sid] : A.u_all + (int64_t)sid * A.ld_v;
    const int32_t *pk = A.perm + S.perm_off;
    unsigned long long *x_steps = A.xchg_all + (int64_t)sid * SPLIT_WORDS;
    unsigned long long *x_parts = x_steps + (1 + tail) * SPLIT_RING * BATCH;
    // progress[t]: 1 + the last block tail t has added to the private vector (0: none yet);
    // progress[2 + t]: 1 + the last block it has gathered
    unsigned long long *progress = x_steps + (1 + SPLIT_MAX_TAILS) * SPLIT_RING * BATCH;
    const int nb = (S.n_rows + BATCH - 1) / BATCH;
    const int n_own = nb > tail ? (nb - tail + n_tails - 1) / n_tails : 0;      // this tail's blocks
    const int back = 2 / n_tails;                                               // own iterations between gather and add
    const int lane = tid & 63, wave = tid >> 6;
    const int hl = tid - 64, rho = hl / LPR, sub = hl & (LPR - 1);
    if (n_own == 0) return;
    auto block_of = [&](int j) { return tail + n_tails * j; };
#define TAIL_ITERATIONS for (int j = -(TAIL_WARM + 3); j < n_own + back; ++j)
    if (wave == 11) {
        TAIL_ITERATIONS {
            const int ja = j - back;                                     // own block that is added this iteration
            if (ja >= 0 && ja < n_own) {
                const int b = block_of(ja);
                // the steps of block b; with two tails also: has the other tail performed every add before b
                // (b - 1 is its latest), and has it gathered block b + 1?  All fetched by the same polls.
                const unsigned long long *word = x_steps + (b & (SPLIT_RING - 1)) * BATCH + lane;
                if (n_tails == 2)
                    sh.xv[lane] = ring_wait<true>(word, b + 1, progress + (1 - tail), b, progress + 2 + (1 - tail),
                                                  b + 1 < nb ? b + 2 : 0, &sh.dead, A.err);
                else
                    sh.xv[lane] = ring_wait<false>(word, b + 1, nullptr, 0, nullptr, 0, &sh.dead, A.err);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // (polls still in flight are not waited for)
                if (lane == 0) __hip_atomic_store(&sh.xflag, ja + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            }
            __syncthreads();
        }
    } else if (wave == 9) {
        RowResolver resolver;
        TAIL_ITERATIONS {
            // publishes the rows of own block j + TAIL_WARM + 1
            resolver.step(rows, TAIL_RING - 1, l_desc, l_prefix, S, pk, j + TAIL_WARM - 2, tail, n_tails, n_own, lane, A.err, false);
            __syncthreads();
        }
    } else if (wave == 10) {
        TAIL_ITERATIONS {
            // one touch per 64 bytes of the entries of own block j + TAIL_WARM (published last iteration);
            // nothing is kept
            if (j + TAIL_WARM >= 0 && j + TAIL_WARM < n_own) {
                const RowSlot &r = rows[(j + TAIL_WARM) & (TAIL_RING - 1)][lane];
                if (r.len > 0) {
                    float sink = 0.f;
#pragma unroll
                    for (int o = 0; o < GRAM_MAX_ROW; o += 16) {
                        const int e = min(o, r.len - 1);
                        sink += gld(r.val + e) + __int_as_float(gld(r.col + e));
                    }
                    sink += gld(r.val + r.len - 1) + __int_as_float(gld(r.col + r.len - 1));
                    asm volatile("" ::"v"(sink));
                }
            }
            __syncthreads();
        }
    } else if (wave == 0) {
        TAIL_ITERATIONS { __syncthreads(); }
    } else {
        // st[0]: the own block that is gathered (j); st[back]: the one that is added (j - back)
        int in_c[TE], st_c[3][TE];
        float in_v[TE], st_v[3][TE];
#pragma unroll
        for (int e = 0; e < TE; ++e) {
            in_c[e] = 0; in_v[e] = 0.f;
#pragma unroll
            for (int k = 0; k < 3; ++k) { st_c[k][e] = 0; st_v[k][e] = 0.f; }
        }
        int in_len = 0, in_base = 0, hb_target = 0;
        TAIL_ITERATIONS {
            // 1. this lane's segment of the row of own block j + 1: the last TE * LPR entries
            if (j + 1 >= 0 && j + 1 < n_own) {
                const RowSlot &r = rows[(j + 1) & (TAIL_RING - 1)][rho];
                in_len = r.len;
                in_base = max(in_len - TE * LPR, 0);
                const int32_t *cp = r.col + in_base + sub;
                const float *vp = r.val + in_base + sub;
#pragma unroll
                for (int e = 0; e < TE; ++e) { in_c[e] = gld(cp + e * LPR); in_v[e] = gld(vp + e * LPR); }
            } else {
                in_len = 0;
            }
            // 2. the steps of own block j - back have arrived: it is added to the private vector
            const int ja = j - back;
            if (ja >= 0 && ja < n_own) {
                const RowSlot &r = rows[ja & (TAIL_RING - 1)][rho];
                wait_flag(&sh.xflag, ja + 1);
                const float dl = sh.xv[rho];
                if (r.len > 0 && dl != 0.f) {
                    const float coef = dl * (LOSS == 1 ? 1.f : r.y) * sc.inv_c;
#pragma unroll
                    for (int e = 0; e < TE; ++e) {
                        const int c = back == 1 ? st_c[1][e] : st_c[2][e];
                        const float v = back == 1 ? st_v[1][e] : st_v[2][e];
                        if (v != 0.f) unsafeAtomicAdd(&u[c], coef * v);
                    }
                }
            }
            // 3. ... completely, before the next block is gathered; the other tail may rely on it from here on
            hb_target += HELPER_WAVES;
            helper_barrier(&sh.hb, hb_target);
            if (tid == 64 && ja >= 0 && ja < n_own)
                __hip_atomic_store(progress + tail, (unsigned long long)(block_of(ja) + 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // 4. gather own block j and hand the partial sums over
            if (j >= 0 && j < n_own) {
                float got[TE];
#pragma unroll
                for (int e = 0; e < TE; ++e) {
                    got[e] = 0.f;
                    if (st_v[0][e] != 0.f) got[e] = ld_l2(u + st_c[0][e]);
                }
                // the values are here: once all helper wavefronts have theirs, the other tail may add block b + 1
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
                if (lane == 0 && atomicAdd(&sh.gcount, 1) + 1 == HELPER_WAVES * (j + 1))
                    __hip_atomic_store(progress + 2 + tail, (unsigned long long)(block_of(j) + 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                float part = 0.f;
#pragma unroll
                for (int e = 0; e < TE; ++e) part += st_v[0][e] * got[e];
                part = sum_over_row_lanes(part);
                const int b = block_of(j);
                if (sub == 0) ring_put(x_parts + (b & (SPLIT_RING - 1)) * BATCH + rho, part, b + 1);
            }
            // 5. move the entry sets one stage on; the incoming set is masked to the row's length and to the
            //    tails' columns
#pragma unroll
            for (int e = 0; e < TE; ++e) {
                st_c[2][e] = st_c[1][e]; st_v[2][e] = st_v[1][e];
                st_c[1][e] = st_c[0][e]; st_v[1][e] = st_v[0][e];
                const bool live = in_base + sub + e * LPR < in_len && in_c[e] >= n_hot;
                st_c[0][e] = live ? in_c[e] : 0;
                st_v[0][e] = live ? in_v[e] : 0.f;
            }
            __syncthreads();
        }
    }
#undef TAIL_ITERATIONS
}

// Workgroup role * k_pad + k: role 0 is the head of solver k, roles 1 .. n_tails are its tails (k_pad is a
// multiple of the number of L2 partitions workgroups are dealt over, so all of them share one).
// xchg_all: SPLIT_WORDS zeroed 64-bit words per solver: the ring of steps, one ring of partial dot products
// per tail, the tails' progress words.
// Dynamic LDS: BatchedShared, then max_list chunk descriptors, max_list local-row prefixes, then (at byte
// offset hot_off) n_hot doubles in the head, the resolved rows in a tail.
template <int LOSS, int TE>
__global__ __launch_bounds__(SPLIT_THREADS) void sdca_batched_split(SplitArgs A, int k_pad)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int role = (int)blockIdx.x / k_pad, sid = (int)blockIdx.x % k_pad;
    if (sid >= A.sc.K) return;
    if (role == 0) split_head<LOSS>(smem, A, sid);
    else split_tail<LOSS, TE>(smem, A, sid, role - 1);
}

}  // namespace chicle
