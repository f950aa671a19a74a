// Row-wise local solver for long sparse rows with every solver spread over several compute units (paper
// Section 4.2: a solver may use all the processors of its node; Section 2.2: L = 1, the coordinate steps
// keep their order).
//
// One compute unit serves a scattered 4-byte access about every seven cycles, so a row of a thousand entries
// costs one workgroup some ten thousand cycles per step (gather, then atomic adds).  Here G workgroups (a
// cluster, all on one L2 partition) share every step of their solver: member g owns the columns
// [g d / G, (g+1) d / G) of the private vector, so of every row the contiguous run of entries that falls
// into that range (rows are sorted by column; the run's bounds come from a table built on the device when
// the chunks are assigned).  Per step each member forms its partial dot product, publishes it in a small
// ring in memory, reads the partial sums of the others, and then every member takes the same dual step from
// the same numbers (summed in member order, so all members get the same bits) and adds its own run of the
// row into its own columns.  One trip between compute units per step; a column is only ever touched by one
// compute unit, whose accesses to one address are served in order, so - as in the single-workgroup solver
// - the adds are not waited for.
//
// Every ring word carries its value together with the step it belongs to (no fences); every wait is bounded:
// a member that waits too long raises the error flag, stops waiting for the rest of the pass and finishes.
#pragma once
#include <hip/hip_runtime.h>
#include "device_types.hpp"
#include "mem.hpp"
#include "sdca_rowwise.hpp"

namespace chicle {

constexpr int CLUSTER_MAX = 4;                // members of a cluster at most
constexpr int CLUSTER_RING = 4;               // steps in flight in the ring
constexpr int CLUSTER_WORDS = CLUSTER_RING * CLUSTER_MAX;   // 64-bit words per solver
constexpr int CLUSTER_SPIN_LIMIT = 1 << 23;   // polls before a wait for another member gives up

// entry offsets, relative to the row's start, at which the columns of members 1 .. CLUSTER_MAX-1 begin
constexpr int SPLITS_PER_ROW = CLUSTER_MAX - 1;

// split[(row_base + r) * SPLITS_PER_ROW + g - 1] = first entry of row r with column >= g * d / G, for
// g = 1 .. G-1.  Grid: (blocks over rows, chunk), one thread per row.
__global__ __launch_bounds__(256) void row_split_offsets(const ChunkDev *__restrict__ chunks, int d, int G,
                                                         int32_t *split)
{
    const ChunkDev &ch = chunks[blockIdx.y];
    for (int r = blockIdx.x * 256 + threadIdx.x; r < ch.n_rows; r += gridDim.x * 256) {
        const int b = ch.row_ptr[r], e = ch.row_ptr[r + 1];
        for (int g = 1; g < G; ++g) {
            const int bound = (int)((int64_t)g * d / G);
            int lo = b, hi = e;                  // first p in [b, e) with col[p] >= bound
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (ch.col[mid] < bound) lo = mid + 1; else hi = mid;
            }
            split[((int64_t)ch.row_base + r) * SPLITS_PER_ROW + g - 1] = lo - b;
        }
    }
}

// One ring word: a partial sum tagged with its step + 1 (the ring is zeroed before the launch).
__device__ __forceinline__ void cluster_put(unsigned long long *p, float v, int tag)
{
    const unsigned long long w = ((unsigned long long)(unsigned)tag << 32) | (unsigned long long)__float_as_uint(v);
    __hip_atomic_store(p, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float cluster_get(const unsigned long long *p, int tag, int *dead, int *err)
{
    unsigned long long v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int spins = 0;
    while ((int)(v >> 32) != tag) {
        if (++spins > CLUSTER_SPIN_LIMIT || __hip_atomic_load(dead, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP)) {
            if (spins > CLUSTER_SPIN_LIMIT) {
                __hip_atomic_store(dead, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                atomicOr(err, ERR_PARTNER_TIMEOUT);
            }
            return 0.f;
        }
        __builtin_amdgcn_s_sleep(1);
        v = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    return __uint_as_float((unsigned)v);
}

// A resolved row as one member of the cluster sees it.
struct ClusterRow {
    const int32_t *col;     // this member's run of the row (indices into the private vector)
    const float *val;
    RowState *st;
    int len;                // length of the run (0: nothing here, or the row takes no step)
    int fast;               // every member's run fits the registers: the row may be gathered one step early
    float y, alpha, q, rw;  // q = 0: the row takes no step
};
constexpr int CLUSTER_ROWS = 8;               // resolved rows kept in LDS

// Sum over the wavefront, the same in every lane: four data-parallel-primitive moves inside rows of 16 lanes,
// then the four row sums are read as scalars.
__device__ __forceinline__ float cluster_wave_sum(float v)
{
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, false));    // quad_perm [1,0,3,2]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, false));    // quad_perm [2,3,0,1]
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, false));   // row_half_mirror
    v += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, false));   // row_mirror
    const int w = __float_as_int(v);
    return (__int_as_float(__builtin_amdgcn_readlane(w, 0)) + __int_as_float(__builtin_amdgcn_readlane(w, 16))) +
           (__int_as_float(__builtin_amdgcn_readlane(w, 32)) + __int_as_float(__builtin_amdgcn_readlane(w, 48)));
}

// Workgroup g * k_pad + k is member g of solver k's cluster (k_pad is a multiple of the number of L2
// partitions workgroups are dealt over, so a cluster shares one).
//
// A step's critical path is the trip of the partial sums between the members.  Everything else is moved off
// it: one thread resolves rows five steps ahead, all threads fetch a row's run of entries three steps ahead, and
// the gather of row t + 2 is requested while the sums of row t + 1 travel, i.e. before row t + 1 has been added
// to the private vector.  What that gather misses is exactly coef(t+1) * (x(t+1) . x(t+2)) over the member's
// columns, so the member forms that dot product meanwhile (the run of row t + 1 sits sorted in LDS, every
// lane looks its entries of row t + 2 up by bisection) and adds the correction when the step of row t + 1 is
// known: the same steps in the same order, in exact arithmetic the same numbers.  Rows of which some
// member's run does not fit the registers (EPT * BLOCK entries) are gathered after their predecessor has been
// added, as in the single-workgroup solver, with the surplus read from memory.
// ring: CLUSTER_WORDS zeroed 64-bit words per solver.
// Dynamic LDS: max_list chunk descriptors, then max_list local-row prefixes.
template <int LOSS, int BLOCK, int EPT>
__global__ __launch_bounds__(BLOCK) void sdca_rowwise_csr_cluster(
    const ChunkDev *__restrict__ chunks, const SolverDev *__restrict__ solvers,
    const int32_t *__restrict__ solver_chunks, const int32_t *__restrict__ solver_prefix,
    const int32_t *__restrict__ perm, float *u_all, int64_t ld_v, int max_list, RoundScalars sc, int *err,
    int k_pad, int G, const int32_t *__restrict__ split, unsigned long long *ring_all,
    const int64_t *__restrict__ u_off)
{
    // u_off: as in sdca_rowwise_csr (compact private vectors; the members' runs are still ranges of columns,
    // and the compact indices ascend with the columns)
    constexpr int CAP = EPT * BLOCK;
    extern __shared__ __align__(16) unsigned char rw_smem[];
    __shared__ float red[2][BLOCK / 64];
    __shared__ ClusterRow rows[CLUSTER_ROWS];
    __shared__ float parts[2][CLUSTER_MAX];
    __shared__ int run_col[3][CAP];            // the runs of the last three rows, for the pair products
    __shared__ float run_val[3][CAP];
    __shared__ int dead;
    const int sid = (int)blockIdx.x % k_pad, g = (int)blockIdx.x / k_pad;
    if (sid >= sc.K) return;
    const SolverDev S = solvers[sid];
    ChunkDev *l_desc = reinterpret_cast<ChunkDev *>(rw_smem);
    int *l_prefix = reinterpret_cast<int *>(l_desc + max_list);
    const int tid = threadIdx.x;
    if (g == 0) stamp_solver(sc, sid, 0);
    for (int i = tid; i < S.n_chunks; i += BLOCK) {
        l_desc[i] = chunks[solver_chunks[S.list_begin + i]];
        l_prefix[i] = solver_prefix[S.list_begin + i];
    }
    if (tid == 0) dead = 0;
    __syncthreads();
    float *u = u_off ? u_all + u_off[sid] : u_all + (int64_t)sid * ld_v;
    const int32_t *pk = perm + S.perm_off;
    unsigned long long *ring = ring_all + (int64_t)sid * CLUSTER_WORDS;
    const int n = S.n_rows;

    // one thread of the last wavefront resolves rows (the first wavefront waits for the other members' sums)
    constexpr int RESOLVER = BLOCK - 64;
    int p_val = -1;
    int m_ci = -1, m_r = 0, m_s1 = 0, m_s2 = 0, m_s3 = 0;
    int2_a4 m_rp = {0, 0};
    float4_v m_st = {0.f, 0.f, 0.f, 0.f};
    // all threads: this member's entries of rows t (0), t + 1 (1), t + 2 (2), t + 3 (3: loads in flight), the
    // gathered values of rows t + 1 and t + 2, and this thread's share of the pair products
    int c0[EPT], c1[EPT], c2[EPT], c3[EPT];
    float v0[EPT], v1[EPT], v2[EPT], v3[EPT], got1[EPT], got2[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
        c0[e] = c1[e] = c2[e] = c3[e] = 0;
        v0[e] = v1[e] = v2[e] = v3[e] = got1[e] = got2[e] = 0.f;
    }
    float g1 = 0.f, g2 = 0.f, mine1 = 0.f;
    bool early1 = false;                       // row t + 1 was gathered before row t was added

    // block sum with the wave sums formed by moves between registers; red[which] alternates between the uses
    auto sum_all = [&](float x, int which) {
        x = cluster_wave_sum(x);
        if ((tid & 63) == 0) red[which][tid >> 6] = x;
        __syncthreads();
        float s = 0.f;
#pragma unroll
        for (int i = 0; i < BLOCK / 64; ++i) s += red[which][i];
        return s;
    };

    for (int t = -6; t < n; ++t) {
        if (tid == RESOLVER) {
            // publish row t + 4: col / val point at this member's run of the row, len is the run's length (it
            // may be 0), q = 0 marks a row that takes no step
            if (t + 4 >= 0 && t + 4 < n) {
                ClusterRow m;
                m.col = nullptr; m.val = nullptr; m.st = nullptr; m.len = 0; m.fast = 1;
                m.y = m_st.x; m.alpha = m_st.y; m.q = 0.f; m.rw = m_st.w;
                const int len = m_rp.y - m_rp.x;
                if (m_ci >= 0 && m_st.z != 0.f && len > 0) {
                    const ChunkDev &ch = l_desc[m_ci];
                    // bounds of the members' runs: 0, s1, s2, s3, len (only the first G - 1 splits exist)
                    const int b1 = G > 1 ? m_s1 : len, b2 = G > 2 ? m_s2 : len, b3 = G > 3 ? m_s3 : len;
                    const int lo = g == 0 ? 0 : g == 1 ? b1 : g == 2 ? b2 : b3;
                    const int hi = g == 0 ? b1 : g == 1 ? b2 : g == 2 ? b3 : len;
                    const int longest = max(max(b1, b2 - b1), max(b3 - b2, len - b3));
                    m.col = (u_off ? chunk_compact_ids(ch) : ch.col) + m_rp.x + lo;
                    m.val = ch.val + m_rp.x + lo; m.st = ch.st + m_r;
                    m.len = hi - lo;
                    m.fast = longest <= CAP;
                    m.q = m_st.z;
                }
                rows[(t + 4) & (CLUSTER_ROWS - 1)] = m;
            }
            // state loads of row t + 5
            m_ci = -1;
            if (t + 5 >= 0 && t + 5 < n) {
                if ((unsigned)p_val >= (unsigned)n) {
                    if (g == 0) atomicOr(err, ERR_PERM_RANGE);
                } else {
                    m_ci = find_chunk(l_prefix, S.n_chunks, p_val);
                    m_r = p_val - l_prefix[m_ci];
                    const ChunkDev &ch = l_desc[m_ci];
                    m_rp = gld2(ch.row_ptr + m_r);
                    m_st = gld_state(ch.st + m_r);
                    const int32_t *sp = split + ((int64_t)ch.row_base + m_r) * SPLITS_PER_ROW;
                    m_s1 = G > 1 ? gld(sp) : 0;
                    m_s2 = G > 2 ? gld(sp + 1) : 0;
                    m_s3 = G > 3 ? gld(sp + 2) : 0;
                }
            }
            // order entry of row t + 6
            p_val = (t + 6 >= 0 && t + 6 < n) ? pk[t + 6] : -1;
        }
        // entries of row t + 3 (published last step), requested first: they have the whole step to arrive
        int len3 = 0;
        if (t + 3 >= 0 && t + 3 < n) {
            const ClusterRow &m3 = rows[(t + 3) & (CLUSTER_ROWS - 1)];
            len3 = min(m3.len, CAP);
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const int p = tid + e * BLOCK;
                c3[e] = 0; v3[e] = 0.f;
                if (p < len3) { c3[e] = gld(m3.col + p); v3[e] = gld(m3.val + p); }
            }
        }
        // ---- row t: the members' partial sums (sent last step) -> the step -> the adds
        const bool in0 = t >= 0;
        const ClusterRow m0 = rows[t & (CLUSTER_ROWS - 1)];              // (t < 0: an unused slot)
        const bool step0 = in0 && m0.q != 0.f;                            // uniform over the cluster
        float coef0 = 0.f;
        if (step0) {
            unsigned long long *slot = ring + (t & (CLUSTER_RING - 1)) * CLUSTER_MAX;
            if (tid < G) parts[t & 1][tid] = tid == g ? mine1 : cluster_get(slot + tid, t + 1, &dead, err);
            __syncthreads();
            float xu = 0.f;
            for (int j = 0; j < G; ++j) xu += parts[t & 1][j];            // the same order in every member
            const float delta = dual_step<LOSS>(m0.alpha, m0.y, m0.rw, xu, m0.q, sc.c);
            if (tid == 0 && g == 0) {
                float an = m0.alpha + delta;                              // a + (clip(..) - a) can leave [0, 1] by an ulp
                if (LOSS != 1) an = fminf(fmaxf(an, 0.f), 1.f);
                gst(&m0.st->alpha, an);
            }
            coef0 = delta * (LOSS == 1 ? 1.0f : m0.y) * sc.inv_c;
        }
        auto add_row_t = [&]() {
            if (coef0 != 0.0f) {
#pragma unroll
                for (int e = 0; e < EPT; ++e)
                    if (tid + e * BLOCK < m0.len) add_entry(u, c0[e], coef0 * v0[e]);
                for (int p = tid + CAP; p < m0.len; p += BLOCK)
                    add_entry(u, gld(m0.col + p), coef0 * gld(m0.val + p));
            }
        };
        // ---- row t + 1: its partial sum, corrected for row t where it was gathered early, is sent off.  Where it
        //      was, the adds of row t wait until the sum is on its way: they are not on the path between the members.
        const bool in1 = t + 1 >= 0 && t + 1 < n;
        const ClusterRow m1 = rows[(t + 1) & (CLUSTER_ROWS - 1)];
        const bool step1 = in1 && m1.q != 0.f;
        const bool adds_first = step1 && !early1;
        if (adds_first) add_row_t();
        if (step1) {
            float part = 0.f;
            if (!early1) {
                __syncthreads();                     // every wavefront has issued its adds of row t before any gathers
#pragma unroll
                for (int e = 0; e < EPT; ++e) got1[e] = tid + e * BLOCK < m1.len ? gather_entry(u, c1[e]) : 0.f;
                for (int p = tid + CAP; p < m1.len; p += BLOCK) part += gld(m1.val + p) * gather_entry(u, gld(m1.col + p));
            }
#pragma unroll
            for (int e = 0; e < EPT; ++e) part += v1[e] * got1[e];
            if (early1) part = fmaf(coef0, g1, part);
            mine1 = sum_all(part, (t + 1) & 1);
            if (tid == 0) cluster_put(ring + ((t + 1) & (CLUSTER_RING - 1)) * CLUSTER_MAX + g, mine1, t + 2);
        }
        if (!adds_first) add_row_t();
        // ---- row t + 2: gathered now, while the sums of row t + 1 travel, together with its product with row t + 1
        const bool in2 = t + 2 >= 0 && t + 2 < n;
        const ClusterRow m2 = rows[(t + 2) & (CLUSTER_ROWS - 1)];
        const bool early2 = in2 && m2.q != 0.f && m2.fast && (!step1 || m1.fast);
        g2 = 0.f;
        if (early2) {
            __syncthreads();                         // every wavefront has issued its adds of row t before any gathers
#pragma unroll
            for (int e = 0; e < EPT; ++e) got2[e] = tid + e * BLOCK < m2.len ? gather_entry(u, c2[e]) : 0.f;
            const int len1 = step1 ? m1.len : 0;
            if (len1 > 0 && m2.len > 0) {
                const int *rc = run_col[(t + 1 + 3) % 3];
                const float *rv = run_val[(t + 1 + 3) % 3];
                const int used = (m2.len + BLOCK - 1) / BLOCK;   // register slots the run of row t + 2 occupies (uniform)
                int pos[EPT];
#pragma unroll
                for (int e = 0; e < EPT; ++e) pos[e] = 0;
#pragma unroll
                for (int s = CAP; s > 0; s >>= 1) {              // pos = entries of the run below this column (CAP is a power of two)
                    if (s > len1) continue;                      // (uniform: such a stride cannot be taken)
#pragma unroll
                    for (int e = 0; e < EPT; ++e) {
                        if (e >= used) continue;
                        const int q = pos[e] + s;
                        if (q <= len1 && rc[q - 1] < vec_index(c2[e])) pos[e] = q;
                    }
                }
#pragma unroll
                for (int e = 0; e < EPT; ++e)
                    if (tid + e * BLOCK < m2.len && pos[e] < len1 && rc[pos[e]] == c2[e]) g2 = fmaf(v2[e], rv[pos[e]], g2);   // (an entry no other row shares has its sign bit set and matches nothing)
            }
        }
        // ---- one stage on; the run of row t + 3 goes to LDS for the pair products of the next two steps
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            c0[e] = c1[e]; v0[e] = v1[e];
            c1[e] = c2[e]; v1[e] = v2[e]; got1[e] = got2[e];
            c2[e] = c3[e]; v2[e] = v3[e];
        }
        g1 = g2; early1 = early2;
        if (t + 3 >= 0 && t + 3 < n) {
            int *rc = run_col[(t + 3 + 3) % 3];
            float *rv = run_val[(t + 3 + 3) % 3];
#pragma unroll
            for (int e = 0; e < EPT; ++e) {
                const int p = tid + e * BLOCK;
                if (p < len3) { rc[p] = vec_index(c2[e]); rv[p] = v2[e]; }
            }
        }
        __syncthreads();   // rows, runs and ring slots written this step are read in the next ones
    }
    if (g == 0) stamp_solver(sc, sid, 1);
}

}  // namespace chicle
