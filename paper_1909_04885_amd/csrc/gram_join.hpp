// Gram blocks of the batched solver, fast form.
//
// A tile couples the 64 rows of one block (i) with the 64 rows of the previous block and the earlier
// rows of the same block (jp): T[jp][i] = scale_i s_i s_j (x_i . x_j).  Columns are stored as popularity
// ranks, so a row's entries split by a range test:
//   - popular columns (rank < GRAM_DENSE): the window's values go into a small dense matrix in LDS and
//     their contribution is a register-tiled dense product (every row has most of these columns);
//   - all other columns: a hash join in LDS.  Entries are inserted into an open-addressing table keyed
//     by column, counted per slot, laid out as posting lists by a scan, and every entry of a block row
//     walks the (short) list of its column, adding its products with float atomics in LDS.
// The summation order of the join is not fixed, so tiles can differ in the last bits between runs.
#pragma once
#include <hip/hip_runtime.h>
#include "device_types.hpp"
#include "sdca_batched.hpp"

namespace chicle {

constexpr int GRAM_DENSE = 32;                        // columns handled by the dense product
constexpr int GRAM_THREADS = 1024;
constexpr int GRAM_SLOTS = 8192;                      // hash slots (>= window entries / 0.75)
constexpr int GRAM_ENTRIES = TILE_W * GRAM_MAX_ROW;   // 6144 entry positions: row slot * 48 + p
constexpr int G_LD = BATCH + 1;                       // padded row of the accumulator tile

struct GramShared {
    float G[TILE_W][G_LD];                 // accumulators [jp][i]
    float A[GRAM_DENSE][TILE_W];           // dense part, [column][window row]
    float e_val[GRAM_ENTRIES];             // values of the sparse-part entries
    int keys[GRAM_SLOTS];                  // column per slot during insertion, then fill cursors
    unsigned short e_slot[GRAM_ENTRIES];   // hash slot per entry, NO_SLOT for dense/absent entries
    unsigned short start[GRAM_SLOTS];      // entries per slot, then exclusive scan = list begin
    unsigned short post[GRAM_ENTRIES];     // posting lists: entry positions grouped by slot
    const int32_t *r_col[TILE_W];
    const float *r_val[TILE_W];
    int r_len[TILE_W];
    float r_sgn[TILE_W];
    float r_scale[BATCH];
    int scan[GRAM_THREADS / 64];
};

constexpr unsigned short NO_SLOT = 0xffff;
constexpr int EMPTY_KEY = -1;

__device__ __forceinline__ int gram_hash(int col) { return (int)(((unsigned)col * 2654435761u) >> 19); }

// row_chunk[perm_off + lr] = chunk of the solver's local row lr; chunk_first[c] = local index of the
// chunk's first row inside its solver.
template <int LOSS>
__global__ __launch_bounds__(GRAM_THREADS) void gram_tiles_join(
    const ChunkDev *__restrict__ chunks, const SolverDev *__restrict__ solvers,
    const int32_t *__restrict__ row_chunk, const int32_t *__restrict__ chunk_first,
    const int32_t *__restrict__ perm, const int32_t *__restrict__ tile_solver, float *tiles, float c,
    int *err)
{
    extern __shared__ __align__(16) unsigned char gsm[];
    GramShared &sh = *reinterpret_cast<GramShared *>(gsm);
    const int tile = blockIdx.x;
    const int k = tile_solver[tile];
    const SolverDev S = solvers[k];
    const int beta = tile - S.tile_begin;
    const int tid = threadIdx.x;

    // ---- rows of the window; clear the tables meanwhile
    if (tid < TILE_W) {
        const int b = tid < BATCH ? beta - 1 : beta;
        const int t = b * BATCH + (tid & (BATCH - 1));
        int len = 0;
        float sgn = 1.f, scale = 0.f;
        const int32_t *cp = nullptr;
        const float *vp = nullptr;
        if (b >= 0 && t < S.n_rows) {
            const int lr = perm[S.perm_off + t];
            if ((unsigned)lr >= (unsigned)S.n_rows) {
                atomicOr(err, ERR_PERM_RANGE);
            } else {
                const int ci = row_chunk[S.perm_off + lr];
                const ChunkDev &ch = chunks[ci];
                const int r = lr - chunk_first[ci];
                const int rb = ch.row_ptr[r], re = ch.row_ptr[r + 1];
                const RowState st = ch.st[r];
                if (st.q != 0.f && re - rb <= GRAM_MAX_ROW) {
                    len = re - rb; cp = ch.col + rb; vp = ch.val + rb;
                    sgn = LOSS == 0 ? st.y : 1.f;
                    scale = LOSS == 0 ? -1.f / st.q : -1.f / (c + st.q);
                }
            }
        }
        sh.r_col[tid] = cp; sh.r_val[tid] = vp; sh.r_len[tid] = len; sh.r_sgn[tid] = sgn;
        if (tid >= BATCH) sh.r_scale[tid - BATCH] = scale;
    }
    for (int i = tid; i < GRAM_SLOTS; i += GRAM_THREADS) { sh.keys[i] = EMPTY_KEY; sh.start[i] = 0; }
    for (int i = tid; i < GRAM_DENSE * TILE_W; i += GRAM_THREADS) (&sh.A[0][0])[i] = 0.f;
    __syncthreads();

    // ---- stage the entries: dense part into A, the rest into the hash table (count per slot)
    for (int idx = tid; idx < GRAM_ENTRIES; idx += GRAM_THREADS) {
        const int s = idx / GRAM_MAX_ROW, p = idx - s * GRAM_MAX_ROW;
        unsigned short slot = NO_SLOT;
        if (p < sh.r_len[s]) {
            const int col = gld(sh.r_col[s] + p);
            const float v = gld(sh.r_val[s] + p);
            if (col < GRAM_DENSE) {
                sh.A[col][s] = v;
            } else {
                int h = gram_hash(col);
                for (;;) {                       // ends: at most GRAM_ENTRIES < GRAM_SLOTS keys are inserted
                    const int prev = atomicCAS(&sh.keys[h], EMPTY_KEY, col);
                    if (prev == EMPTY_KEY || prev == col) break;
                    h = (h + 1) & (GRAM_SLOTS - 1);
                }
                slot = (unsigned short)h;
                sh.e_val[idx] = v;
                // two 16-bit counters share a word
                atomicAdd(reinterpret_cast<unsigned int *>(sh.start) + (h >> 1), (h & 1) ? 0x10000u : 1u);
            }
        }
        sh.e_slot[idx] = slot;
    }
    __syncthreads();

    // ---- exclusive scan of the slot counts (8 slots per thread), cursors into keys[]
    {
        const int base = tid * (GRAM_SLOTS / GRAM_THREADS);
        int cnt[GRAM_SLOTS / GRAM_THREADS], sum = 0;
#pragma unroll
        for (int j = 0; j < GRAM_SLOTS / GRAM_THREADS; ++j) { cnt[j] = sh.start[base + j]; sum += cnt[j]; }
        int incl = sum;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int y = __shfl_up(incl, o, 64);
            if ((tid & 63) >= o) incl += y;
        }
        if ((tid & 63) == 63) sh.scan[tid >> 6] = incl;
        __syncthreads();
        int off = incl - sum;
        for (int w = 0; w < (tid >> 6); ++w) off += sh.scan[w];
#pragma unroll
        for (int j = 0; j < GRAM_SLOTS / GRAM_THREADS; ++j) {
            sh.start[base + j] = (unsigned short)off;
            sh.keys[base + j] = off;
            off += cnt[j];
        }
    }
    __syncthreads();

    // ---- fill the posting lists
    for (int idx = tid; idx < GRAM_ENTRIES; idx += GRAM_THREADS) {
        const unsigned short slot = sh.e_slot[idx];
        if (slot != NO_SLOT) {
            const int pos = atomicAdd(&sh.keys[slot], 1);
            sh.post[pos] = (unsigned short)idx;
        }
    }
    // ---- dense part: G[jp][i] = sum_h A[h][64 + i] A[h][jp]; thread -> 4 values of i, 2 of jp
    {
        const int i0 = (tid & 15) * 4, j0 = (tid >> 4) * 2;
        float acc[2][4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll 8
        for (int h = 0; h < GRAM_DENSE; ++h) {
            const float4 ai = *reinterpret_cast<const float4 *>(&sh.A[h][BATCH + i0]);
            const float2 aj = *reinterpret_cast<const float2 *>(&sh.A[h][j0]);
            acc[0][0] += aj.x * ai.x; acc[0][1] += aj.x * ai.y; acc[0][2] += aj.x * ai.z; acc[0][3] += aj.x * ai.w;
            acc[1][0] += aj.y * ai.x; acc[1][1] += aj.y * ai.y; acc[1][2] += aj.y * ai.z; acc[1][3] += aj.y * ai.w;
        }
#pragma unroll
        for (int a = 0; a < 2; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) sh.G[j0 + a][i0 + b] = acc[a][b];
    }
    __syncthreads();

    // ---- sparse part: every entry of a block row meets the other entries of its column
    for (int idx = BATCH * GRAM_MAX_ROW + tid; idx < GRAM_ENTRIES; idx += GRAM_THREADS) {
        const unsigned short slot = sh.e_slot[idx];
        if (slot == NO_SLOT) continue;
        const int i = idx / GRAM_MAX_ROW - BATCH;
        const float a = sh.e_val[idx];
        const int pb = sh.start[slot], pe = sh.keys[slot];
        for (int p = pb; p < pe; ++p) {
            const int f = sh.post[p];
            const int sf = f / GRAM_MAX_ROW;
            if (sf < BATCH || sf - BATCH < i) atomicAdd(&sh.G[sf][i], a * sh.e_val[f]);
        }
    }
    __syncthreads();

    // ---- scale and write out, coalesced over i
    float *out = tiles + (int64_t)tile * TILE_FLOATS;
    for (int idx = tid; idx < TILE_FLOATS; idx += GRAM_THREADS) {
        const int jp = idx >> 6, i = idx & 63;
        float g = 0.f;
        if (jp < BATCH || jp - BATCH < i) g = sh.G[jp][i] * sh.r_scale[i] * sh.r_sgn[BATCH + i] * sh.r_sgn[jp];
        out[idx] = g;
    }
}

// Fill row_chunk for one (solver, chunk) list entry per workgroup.
__global__ __launch_bounds__(256) void fill_row_chunk(const ChunkDev *__restrict__ chunks,
                                                      const int32_t *__restrict__ solver_chunks,
                                                      const int32_t *__restrict__ list_base, int32_t *row_chunk)
{
    const int ci = solver_chunks[blockIdx.x];
    const int n = chunks[ci].n_rows;
    int32_t *dst = row_chunk + list_base[blockIdx.x];
    for (int r = threadIdx.x; r < n; r += 256) dst[r] = ci;
}

}  // namespace chicle
