// Gram blocks of the batched solver.
//
// A tile couples the 64 rows of one block (i) with the 64 rows of the previous block and the earlier
// rows of the same block (jp): T[jp][i] = scale_i s_i s_j (x_i . x_j).  Columns are stored as popularity
// ranks, so a row's entries split by a range test:
//   - popular columns (rank < GRAM_DENSE): the window's values go into a small dense matrix in LDS and
//     their contribution is a dense product on the matrix cores, fp32 in and out (the rows share so many
//     of these columns that the join's lists would be long);
//   - all other columns: a hash join in LDS.  Entries are inserted into an open-addressing table keyed
//     by column, counted per slot, laid out as posting lists (row, value) by a scan, and every entry of
//     a block row walks the short list of its column, adding its products with float atomics in LDS.
// The summation order of the join is not fixed, so tiles can differ in the last bits between runs.
//
// Each workgroup owns a contiguous range of tiles and works through it; the row lookups of the next
// tile (visiting order -> chunk -> row offsets, a chain of dependent loads) are spread over the phases
// of the current tile so that their latency is hidden.
#pragma once
#include <hip/hip_runtime.h>
#include "device_types.hpp"
#include "sdca_batched.hpp"

namespace chicle {

constexpr int GRAM_DENSE = 64;                        // columns handled by the dense product
constexpr int GRAM_THREADS = 1024;
constexpr int GRAM_SLOTS = 8192;                      // hash slots (> window entries, so probing ends)
constexpr int GRAM_ENTRIES = TILE_W * GRAM_MAX_ROW;   // 6144 entry positions: row slot * 48 + p
constexpr int GRAM_EPT = GRAM_ENTRIES / GRAM_THREADS; // entry positions per thread
constexpr int G_LD = BATCH + 1;                       // padded row of the accumulator tile

struct GramRows {                                     // the 128 rows of a window
    const int32_t *col[TILE_W];
    const float *val[TILE_W];
    int len[TILE_W];
    float sgn[TILE_W];
    float scale[BATCH];
};

// The accumulators are doubles: the join adds into them with LDS atomics, and on this hardware those run
// at the rate of the LDS pipeline for doubles while they are serialised lane by lane for floats.  The
// dense slab A is only alive from the clearing of the tables to the end of the dense product, when G is
// not; it occupies the tail of G's storage.
struct GramShared {
    union {
        double G[TILE_W][G_LD];            // accumulators [jp][i]
        struct {
            unsigned char before_A[sizeof(double) * TILE_W * G_LD - sizeof(float) * GRAM_DENSE * TILE_W];
            float A[GRAM_DENSE][TILE_W];   // dense part, [column][window row]
        } d;
    };
    int keys[GRAM_SLOTS];                  // column per slot during insertion, then fill cursors
    unsigned short start[GRAM_SLOTS];      // entries per slot, then exclusive scan = list begin
    float post_val[GRAM_ENTRIES];          // posting lists grouped by slot: value ...
    unsigned char post_row[GRAM_ENTRIES];  // ... and window row of each member
    GramRows rows[3];                      // current tile and the two after it
    int scan[GRAM_THREADS / 64];
};

constexpr int EMPTY_KEY = -1;

__device__ __forceinline__ int gram_hash(int col) { return (int)(((unsigned)col * 2654435761u) >> 19); }

// Row lookups of one window, one row per thread (tid < 128), as four steps of dependent loads.
struct RowLookup {
    int lr, ci, r;
    const int32_t *row_ptr, *colp;
    const float *valp;
    const RowState *stp;
    int2_a4 rp;
    float4_v st;
    bool live;
};

// row_chunk[perm_off + lr] = chunk of the solver's local row lr; chunk_first[c] = local index of the
// chunk's first row inside its solver.
template <int LOSS>
__global__ __launch_bounds__(GRAM_THREADS) void gram_tiles_join(
    const ChunkDev *__restrict__ chunks, const SolverDev *__restrict__ solvers,
    const int32_t *__restrict__ row_chunk, const int32_t *__restrict__ chunk_first,
    const int32_t *__restrict__ perm, const int32_t *__restrict__ tile_solver, float *tiles, int n_tiles,
    float c, int *err)
{
    extern __shared__ __align__(16) unsigned char gsm[];
    GramShared &sh = *reinterpret_cast<GramShared *>(gsm);
    const int tid = threadIdx.x;
    const int per = (n_tiles + gridDim.x - 1) / gridDim.x;
    const int t_begin = blockIdx.x * per;
    const int t_end = min(n_tiles, t_begin + per);
    if (t_begin >= t_end) return;

    const int32_t *dummy_col = chunks[0].col;      // readable for at least GRAM_MAX_ROW entries
    const float *dummy_val = chunks[0].val;
    RowLookup L;
    SolverDev LS;
    // step 1: visiting-order entry of this thread's row in window `tile`
    auto lookup1 = [&](int tile) {
        L.live = false; L.lr = -1;
        if (tid >= TILE_W || tile >= t_end) return;
        LS = solvers[tile_solver[tile]];
        const int beta = tile - LS.tile_begin;
        const int b = tid < BATCH ? beta - 1 : beta;
        const int t = b * BATCH + (tid & (BATCH - 1));
        if (b >= 0 && t < LS.n_rows) { L.lr = gld(perm + LS.perm_off + t); L.live = true; }
    };
    auto lookup2 = [&]() {       // -> chunk id
        if (!L.live) return;
        if ((unsigned)L.lr >= (unsigned)LS.n_rows) { atomicOr(err, ERR_PERM_RANGE); L.live = false; return; }
        L.ci = gld(row_chunk + LS.perm_off + L.lr);
    };
    auto lookup3 = [&]() {       // -> chunk descriptor
        if (!L.live) return;
        const ChunkDev &ch = chunks[L.ci];
        L.r = L.lr - gld(chunk_first + L.ci);
        L.row_ptr = ch.row_ptr; L.colp = ch.col; L.valp = ch.val; L.stp = ch.st;
    };
    auto lookup4 = [&]() {       // -> row offsets and state
        if (!L.live) return;
        L.rp = gld2(L.row_ptr + L.r);
        L.st = gld_state(L.stp + L.r);
    };
    auto publish = [&](GramRows &R) {
        if (tid >= TILE_W) return;
        int len = 0;
        float sgn = 1.f, scale = 0.f;
        const int32_t *cp = nullptr;
        const float *vp = nullptr;
        if (L.live) {
            const int n = L.rp.y - L.rp.x;
            const float q = L.st.z;
            if (q != 0.f && n > 0 && n <= GRAM_MAX_ROW) {
                len = n; cp = L.colp + L.rp.x; vp = L.valp + L.rp.x;
                sgn = LOSS == 1 ? 1.f : L.st.x;
                scale = LOSS == 0 ? -1.f / q : LOSS == 1 ? -1.f / (c + q) : -1.f / c;
            }
        }
        if (len == 0) { cp = dummy_col; vp = dummy_val; }
        R.col[tid] = cp; R.val[tid] = vp; R.len[tid] = len; R.sgn[tid] = sgn;
        if (tid >= BATCH) R.scale[tid - BATCH] = scale;
    };

    // Rows are known two tiles ahead (the lookups of tile + 2 are spread over the phases of the current
    // tile), entries one tile ahead: a thread holds the same entry positions of the block rows in every
    // tile, so the 64 rows that are "previous block" in the next tile are already in its registers and only
    // the next tile's own rows are requested, a whole tile before they are used.
    lookup1(t_begin); lookup2(); lookup3(); lookup4(); publish(sh.rows[0]);
    lookup1(t_begin + 1); lookup2(); lookup3(); lookup4(); publish(sh.rows[1]);
    __syncthreads();
    constexpr int HALF = GRAM_EPT / 2;             // entry positions per thread in the previous block's rows
    int e_col[GRAM_EPT], n_col[HALF];
    float e_val[GRAM_EPT], n_val[HALF];
#pragma unroll
    for (int k = 0; k < GRAM_EPT; ++k) {           // first tile: all 128 rows
        const int idx = tid + k * GRAM_THREADS;
        const int s = idx / GRAM_MAX_ROW, p = idx - s * GRAM_MAX_ROW;
        e_col[k] = gld(sh.rows[0].col[s] + p); e_val[k] = gld(sh.rows[0].val[s] + p);
    }

    for (int tile = t_begin; tile < t_end; ++tile) {
        const int slot = (tile - t_begin) % 3;
        GramRows &R = sh.rows[slot];
        // ---- request the next tile's own rows; clear the tables; lookup of tile + 2, step 1
        bool e_live[GRAM_EPT];
#pragma unroll
        for (int k = 0; k < GRAM_EPT; ++k) {
            const int idx = tid + k * GRAM_THREADS;
            const int s = idx / GRAM_MAX_ROW, p = idx - s * GRAM_MAX_ROW;
            // (loads are unconditional: a row without entries points at readable dummy data and the store
            // keeps slack behind every chunk; e_live masks them)
            e_live[k] = p < R.len[s];
        }
        if (tile + 1 < t_end) {
            const GramRows &N = sh.rows[(slot + 1) % 3];
#pragma unroll
            for (int k = 0; k < HALF; ++k) {
                const int idx = tid + (k + HALF) * GRAM_THREADS;
                const int s = idx / GRAM_MAX_ROW, p = idx - s * GRAM_MAX_ROW;
                n_col[k] = gld(N.col[s] + p); n_val[k] = gld(N.val[s] + p);
            }
        }
        lookup1(tile + 2);
        {
            // 16-byte stores: keys <- EMPTY_KEY (all ones), start <- 0, A <- 0
            uint4 *kq = reinterpret_cast<uint4 *>(sh.keys);
            for (int i = tid; i < GRAM_SLOTS / 4; i += GRAM_THREADS) kq[i] = make_uint4(~0u, ~0u, ~0u, ~0u);
            uint4 *sq = reinterpret_cast<uint4 *>(sh.start);
            for (int i = tid; i < GRAM_SLOTS / 8; i += GRAM_THREADS) sq[i] = make_uint4(0u, 0u, 0u, 0u);
            uint4 *aq = reinterpret_cast<uint4 *>(&sh.d.A[0][0]);
            for (int i = tid; i < GRAM_DENSE * TILE_W / 4; i += GRAM_THREADS) aq[i] = make_uint4(0u, 0u, 0u, 0u);
        }
        __syncthreads();

        // ---- dense part into A, the rest into the hash table (count per slot)
        int e_slot[GRAM_EPT], first[GRAM_EPT];
#pragma unroll
        for (int k = 0; k < GRAM_EPT; ++k) {       // first probes of all entries in flight together
            const int idx = tid + k * GRAM_THREADS;
            const int s = idx / GRAM_MAX_ROW;
            e_slot[k] = -1; first[k] = EMPTY_KEY;
            if (e_live[k]) {
                if (e_col[k] < GRAM_DENSE) sh.d.A[e_col[k]][s] = e_val[k];
                else {
                    e_slot[k] = gram_hash(e_col[k]);
                    first[k] = atomicCAS(&sh.keys[e_slot[k]], EMPTY_KEY, e_col[k]);
                }
            }
        }
#pragma unroll
        for (int k = 0; k < GRAM_EPT; ++k) {
            if (e_slot[k] < 0) continue;
            int h = e_slot[k], prev = first[k];
            while (prev != EMPTY_KEY && prev != e_col[k]) {   // ends: fewer keys than slots are inserted
                h = (h + 1) & (GRAM_SLOTS - 1);
                prev = atomicCAS(&sh.keys[h], EMPTY_KEY, e_col[k]);
            }
            e_slot[k] = h;
            // two 16-bit counters share a word
            atomicAdd(reinterpret_cast<unsigned int *>(sh.start) + (h >> 1), (h & 1) ? 0x10000u : 1u);
        }
        lookup2();
        __syncthreads();

        // ---- exclusive scan of the slot counts (8 slots per thread), cursors into keys[]
        {
            const int base = tid * (GRAM_SLOTS / GRAM_THREADS);
            static_assert(GRAM_SLOTS / GRAM_THREADS == 8, "a thread's counts are one 16-byte word");
            const uint4 packed = *reinterpret_cast<const uint4 *>(&sh.start[base]);
            const unsigned pw[4] = {packed.x, packed.y, packed.z, packed.w};
            int cnt[8], sum = 0;
#pragma unroll
            for (int j = 0; j < 8; ++j) { cnt[j] = (pw[j >> 1] >> ((j & 1) * 16)) & 0xffffu; sum += cnt[j]; }
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
            int cur[8];
            unsigned st[4] = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                cur[j] = off;
                st[j >> 1] |= (unsigned)off << ((j & 1) * 16);
                off += cnt[j];
            }
            *reinterpret_cast<uint4 *>(&sh.start[base]) = make_uint4(st[0], st[1], st[2], st[3]);
            *reinterpret_cast<int4 *>(&sh.keys[base]) = make_int4(cur[0], cur[1], cur[2], cur[3]);
            *reinterpret_cast<int4 *>(&sh.keys[base + 4]) = make_int4(cur[4], cur[5], cur[6], cur[7]);
        }
        lookup3();
        __syncthreads();

        // ---- fill the posting lists
#pragma unroll
        for (int k = 0; k < GRAM_EPT; ++k)
            if (e_slot[k] >= 0) {
                const int pos = atomicAdd(&sh.keys[e_slot[k]], 1);
                sh.post_val[pos] = e_val[k];
                sh.post_row[pos] = (unsigned char)((tid + k * GRAM_THREADS) / GRAM_MAX_ROW);
            }
        // ---- dense part: G[jp][i] = sum_h A[h][jp] A[h][64 + i] on the matrix cores (fp32 in and out).  A
        //      32 x 2 by 2 x 32 product takes A[l % 32][l / 32] and B[l / 32][l % 32] from lane l; wavefront
        //      w < 8 owns the 32 x 32 block (jp block w / 2, i block w % 2).  The block of own rows 96..127
        //      against rows 64..95 lies above the diagonal and is not needed.
        {
            typedef float floatx16 __attribute__((ext_vector_type(16)));
            const int wv = tid >> 6, lane = tid & 63;
            const int tj = wv >> 1, ti = wv & 1;
            const bool mine = wv < 8 && !(tj == 3 && ti == 0);
            floatx16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
            if (mine) {
                const float *pa = &sh.d.A[lane >> 5][32 * tj + (lane & 31)];
                const float *pb = &sh.d.A[lane >> 5][BATCH + 32 * ti + (lane & 31)];
#pragma unroll 8
                for (int h = 0; h < GRAM_DENSE; h += 2)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[h * TILE_W], pb[h * TILE_W], acc, 0, 0, 0);
            }
            lookup4();
            __syncthreads();                 // every read of A is done: G may take its place
            // result layout: register r of lane l is row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32
            if (wv < 8) {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    sh.G[32 * tj + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)][32 * ti + (lane & 31)] = (double)acc[r];
            }
        }
        __syncthreads();

        // ---- sparse part: every entry of a block row meets the other members of its column's list
#pragma unroll
        for (int k = HALF; k < GRAM_EPT; ++k) {                  // positions of the block rows (64 .. 127)
            if (e_slot[k] < 0) continue;
            const int i = (tid + k * GRAM_THREADS) / GRAM_MAX_ROW - BATCH;
            const float a = e_val[k];
            const int pb = sh.start[e_slot[k]], pe = sh.keys[e_slot[k]];
            for (int p = pb; p < pe; p += 4) {          // four list members per round of LDS latency
                int sf[4];
                float vf[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int pj = min(p + j, pe - 1);
                    sf[j] = sh.post_row[pj]; vf[j] = sh.post_val[pj];
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if (p + j < pe && (sf[j] < BATCH || sf[j] - BATCH < i)) atomicAdd(&sh.G[sf[j]][i], (double)(a * vf[j]));
            }
        }
        publish(sh.rows[(slot + 2) % 3]);
        __syncthreads();

        // ---- scale and write out, coalesced over i (a thread's i is the same for all its values)
        {
            float *out = tiles + (int64_t)tile * TILE_FLOATS;
            const int i = tid & 63;
            const float si = R.scale[i] * R.sgn[BATCH + i];
#pragma unroll
            for (int k = 0; k < TILE_FLOATS / GRAM_THREADS; ++k) {
                const int jp = (tid >> 6) + k * (GRAM_THREADS / 64);
                float g = 0.f;
                if (jp < BATCH || jp - BATCH < i) g = (float)sh.G[jp][i] * si * R.sgn[jp];
                out[jp * BATCH + i] = g;
            }
        }
        // this tile's own rows are the next tile's previous block; its own rows have arrived by now
#pragma unroll
        for (int k = 0; k < HALF; ++k) {
            e_col[k] = e_col[k + HALF]; e_val[k] = e_val[k + HALF];
            e_col[k + HALF] = n_col[k]; e_val[k + HALF] = n_val[k];
        }
        __syncthreads();     // G has been read: the next tile may clear A, which lies inside it
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
