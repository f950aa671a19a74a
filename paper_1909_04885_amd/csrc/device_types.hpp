// Plain structs shared by host code and kernels of the CoCoA-round library.
#pragma once
#include <stdint.h>

namespace chicle {

// Per-sample state that travels with its row (paper Section 4.4).  One record per row so that a
// randomly visited row costs one 16-byte access.
struct RowState {
    float y;        // label / target
    float alpha;    // dual variable
    float q;        // squared row norm
    float rw;       // residual at the current shared vector, refreshed by the gap pass in double:
                    // 1 - y x_i.w (hinge), y - x_i.w (squared)
};

// One data chunk as the kernels see it (paper Section 4.4: sparse or dense rows plus per-sample
// state in one contiguous block; all pointers point into that block).
struct ChunkDev {
    const int32_t *row_ptr;   // CSR: n_rows + 1 chunk-local offsets; dense: nullptr
    const int32_t *col;       // CSR column ids; dense: nullptr
    const float *val;         // CSR values, or dense row-major n_rows x d
    RowState *st;             // per-row state, one 16-byte record per row
    int32_t n_rows;
    int32_t row_base;         // index of the chunk's first row in context-wide per-row tables
    int64_t nnz;              // stored entries
};

// Readable entries past the last row of a chunk (kernels read short rows with fixed-width loads), and the
// length in entries of a chunk's per-entry arrays in the store (a multiple of 64 entries = 256 bytes).
constexpr int ENTRY_SLACK = 64;
__host__ __device__ inline int64_t padded_entries(int64_t nnz) { return (nnz + ENTRY_SLACK + 63) / 64 * 64; }
// Where private vectors are stored compactly (long sparse rows), a chunk's column ids are followed by an
// array of the same length that holds, for every entry, the index of its column in the compact private
// vector of the solver that owns the chunk.
__host__ __device__ inline const int32_t *chunk_compact_ids(const ChunkDev &ch) { return ch.col + padded_entries(ch.nnz); }

// One local solver under the current assignment.
struct SolverDev {
    int64_t perm_off;         // where this solver's visiting order starts in the concatenated array
    int32_t list_begin;       // first entry of this solver in solver_chunks[] / solver_prefix[]
    int32_t n_chunks;
    int32_t n_rows;
    int32_t tile_begin;       // first Gram tile of this solver (batched solver); batches = ceil(n_rows/64)
};

// Scalars of one round.
struct RoundScalars {
    float c;        // lambda n / sigma
    float inv_c;    // sigma / (lambda n)
    float inv_sigma;
    int32_t K;
    long long *ticks;   // per solver: constant-rate clock at the start and at the end of its pass
};

// Start / end stamps of a solver's pass (Section 4.5: task runtimes are what the rebalancing policy
// learns from).  One lane per workgroup writes them.
__device__ __forceinline__ void stamp_solver(const RoundScalars &sc, int solver, int which)
{
    if (threadIdx.x == 0 && sc.ticks) sc.ticks[2 * solver + which] = (long long)wall_clock64();
}
__device__ __forceinline__ void stamp_solver(const RoundScalars &sc, int which) { stamp_solver(sc, blockIdx.x, which); }

constexpr int L2_PARTITIONS = 8;         // workgroup i is dispatched to L2 partition (compute-unit group) i mod 8

constexpr int ERR_PERM_RANGE = 1;
constexpr int ERR_PARTNER_TIMEOUT = 2;   // the workgroups that share a solver lost each other

}  // namespace chicle
