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

// Workgroup g * k_pad + k is member g of solver k's cluster (k_pad is a multiple of the number of L2
// partitions workgroups are dealt over, so a cluster shares one).  The software pipeline is that of
// sdca_rowwise_csr: thread 0 resolves rows ahead, all threads fetch the next row's run of entries while the
// current row is computed.  ring: CLUSTER_WORDS zeroed 64-bit words per solver.
// Dynamic LDS: max_list chunk descriptors, then max_list local-row prefixes.
template <int LOSS, int BLOCK, int EPT>
__global__ __launch_bounds__(BLOCK) void sdca_rowwise_csr_cluster(
    const ChunkDev *__restrict__ chunks, const SolverDev *__restrict__ solvers,
    const int32_t *__restrict__ solver_chunks, const int32_t *__restrict__ solver_prefix,
    const int32_t *__restrict__ perm, float *u_all, int64_t ld_v, int max_list, RoundScalars sc, int *err,
    int k_pad, int G, const int32_t *__restrict__ split, unsigned long long *ring_all,
    const int64_t *__restrict__ u_off)
{
    // u_off: as in sdca_rowwise_csr (compact private vectors; the members' runs are still ranges of columns)
    extern __shared__ __align__(16) unsigned char rw_smem[];
    __shared__ float red[BLOCK / 64];
    __shared__ RowMeta ring_rows[4];
    __shared__ float parts[2][CLUSTER_MAX];
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

    // thread 0: rows being resolved
    int p_val = -1;
    int m_ci = -1, m_r = 0, m_lo = 0, m_hi = 0;
    int2_a4 m_rp = {0, 0};
    float4_v m_st = {0.f, 0.f, 0.f, 0.f};
    // all threads: this member's entries of the current and of the next row
    int c_c[EPT], n_c[EPT];
    float c_v[EPT], n_v[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) { c_c[e] = n_c[e] = 0; c_v[e] = n_v[e] = 0.f; }

    for (int t = -4; t < n; ++t) {
        if (tid == 0) {
            // publish row t + 2: RowMeta.col / val point at this member's run of the row, len is the run's
            // length (it may be 0), and q = 0 marks a row that takes no step
            if (t + 2 >= 0 && t + 2 < n) {
                RowMeta m;
                m.col = nullptr; m.val = nullptr; m.st = nullptr; m.len = 0;
                m.y = m_st.x; m.alpha = m_st.y; m.q = 0.f; m.rw = m_st.w;
                const int len = m_rp.y - m_rp.x;
                if (m_ci >= 0 && m_st.z != 0.f && len > 0) {
                    const ChunkDev &ch = l_desc[m_ci];
                    const int lo = g == 0 ? 0 : m_lo, hi = g == G - 1 ? len : m_hi;
                    m.col = (u_off ? chunk_compact_ids(ch) : ch.col) + m_rp.x + lo;
                    m.val = ch.val + m_rp.x + lo; m.st = ch.st + m_r;
                    m.len = hi - lo;
                    m.q = m_st.z;
                }
                ring_rows[(t + 2) & 3] = m;
            }
            // state loads of row t + 3
            m_ci = -1;
            if (t + 3 >= 0 && t + 3 < n) {
                if ((unsigned)p_val >= (unsigned)n) {
                    if (g == 0) atomicOr(err, ERR_PERM_RANGE);
                } else {
                    m_ci = find_chunk(l_prefix, S.n_chunks, p_val);
                    m_r = p_val - l_prefix[m_ci];
                    const ChunkDev &ch = l_desc[m_ci];
                    m_rp = gld2(ch.row_ptr + m_r);
                    m_st = gld_state(ch.st + m_r);
                    const int32_t *sp = split + ((int64_t)ch.row_base + m_r) * SPLITS_PER_ROW;
                    m_lo = g > 0 ? gld(sp + g - 1) : 0;
                    m_hi = g < G - 1 ? gld(sp + g) : 0;
                }
            }
            // order entry of row t + 4
            p_val = (t + 4 >= 0 && t + 4 < n) ? pk[t + 4] : -1;
        }
        // The gather of row t is requested first and this member's entries of row t + 1 (published last step)
        // after it: loads return in the order they were issued, so the step does not wait for the next
        // row's entries, which come from memory.
        const RowMeta m = ring_rows[t & 3];                       // (t < 0: an unused slot)
        const bool step = t >= 0 && m.q != 0.f;                   // the row takes a step (uniform over the cluster)
        float got[EPT];
#pragma unroll
        for (int e = 0; e < EPT; ++e) {
            got[e] = 0.f;
            if (step && tid + e * BLOCK < m.len) got[e] = ld_l2(u + c_c[e]);
        }
        if (t + 1 >= 0 && t + 1 < n) {
            const RowMeta &mn = ring_rows[(t + 1) & 3];
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
                for (int p = tid + EPT * BLOCK; p < m.len; p += BLOCK) part += gld(m.val + p) * ld_l2(u + gld(m.col + p));
                const float mine = block_sum<BLOCK>(part, red);
                // exchange the partial sums: slot t % CLUSTER_RING, one word per member
                unsigned long long *slot = ring + (t & (CLUSTER_RING - 1)) * CLUSTER_MAX;
                if (tid == 0) cluster_put(slot + g, mine, t + 1);
                if (tid < G) parts[t & 1][tid] = tid == g ? mine : cluster_get(slot + tid, t + 1, &dead, err);
                __syncthreads();
                float xu = 0.f;
                for (int j = 0; j < G; ++j) xu += parts[t & 1][j];         // the same order in every member
                const float delta = dual_step<LOSS>(m.alpha, m.y, m.rw, xu, m.q, sc.c);
                if (tid == 0 && g == 0) {
                    float an = m.alpha + delta;                      // a + (clip(..) - a) can leave [0, 1] by an ulp
                    if (LOSS != 1) an = fminf(fmaxf(an, 0.f), 1.f);
                    gst(&m.st->alpha, an);
                }
                const float coef = delta * (LOSS == 1 ? 1.0f : m.y) * sc.inv_c;
                if (coef != 0.0f) {
#pragma unroll
                    for (int e = 0; e < EPT; ++e)
                        if (tid + e * BLOCK < m.len) unsafeAtomicAdd(u + c_c[e], coef * c_v[e]);
                    for (int p = tid + EPT * BLOCK; p < m.len; p += BLOCK)
                        unsafeAtomicAdd(u + gld(m.col + p), coef * gld(m.val + p));
                }
            }
        }
#pragma unroll
        for (int e = 0; e < EPT; ++e) { c_c[e] = n_c[e]; c_v[e] = n_v[e]; }
        __syncthreads();   // ring slots written this step are read next step; orders scatter before gather
    }
    if (g == 0) stamp_solver(sc, sid, 1);
}

}  // namespace chicle
