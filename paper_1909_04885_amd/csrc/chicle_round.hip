// C ABI of the CoCoA round (see include/chicle_round.h for the contract of every call).
// Host logic: chunk store carved from a caller-supplied arena, chunk -> solver tables, launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <numeric>
#include <string>
#include <vector>

#include "../../include/chicle_round.h"
#include "aggregate_gap.hpp"
#include "device_types.hpp"
#include "gram_join.hpp"
#include "layout.hpp"
#include "policies.hpp"
#include "sdca_batched.hpp"
#include "sdca_batched_dense.hpp"
#include "sdca_batched_split.hpp"
#include "sdca_rowwise.hpp"
#include "sdca_rowwise_cluster.hpp"

using namespace chicle;

namespace {

constexpr size_t ALIGN = 256;
constexpr int GAP_PARTS = 8192;        // workgroups (and partial sums) of the gap row kernels, at least
constexpr int WSQ_PARTS = 512;
constexpr int MAX_LIST_LDS = 768;      // chunks one solver may own (their descriptors are staged in LDS)
constexpr int DENSE_V_LDS_MAX_D = 8192;
constexpr int BATCHED_MAX_LIST = MAX_LIST_LDS;  // chunk descriptors of one solver the batched solver stages in LDS (they take
                                               // the place of columns of the private vector's LDS-resident head)
constexpr int RENUMBER_MAX_ROW = 64;   // rows are re-sorted by one thread each: short rows only
#ifndef SPLIT_TAILS
#define SPLIT_TAILS 2        // tail workgroups per solver of the split batched solver (1 or 2)
#endif
constexpr int SLICES_MIN = 4;         // fewer slices of the shared vector than this: the plain gap row pass
constexpr double LONG_ROW_AVG = 96.0;  // sparse rows longer than this on average: the row-wise solver uses whole workgroups per row

enum State { ST_LOADING = 0, ST_READY = 1, ST_EPOCH_DONE = 2 };

inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }
inline int64_t pad_d(int64_t d) { return (d + 63) / 64 * 64; }
inline int64_t tiles_cap(int64_t n_total, int32_t max_solvers) { return n_total / BATCH + max_solvers + 1; }

struct Seg {
    hipEvent_t start = nullptr, stop = nullptr;
    bool recorded = false;
};

// Partial sums of the gap kernels: one (loss, conjugate) pair per workgroup of the row pass, |w|^2 partials.
struct GapScratch {
    double *loss = nullptr, *conj = nullptr, *wsq = nullptr, *unused = nullptr;
    int parts = 0;            // length of loss[] and conj[]
};

// Scratch of chicle_gap_noalloc: a fixed array in the code object, one copy per GPU, kept until the process
// ends.  Layout: GAP_PARTS loss partials, GAP_PARTS conjugate partials, 2 * WSQ_PARTS for |w|^2.
constexpr int STATIC_SCRATCH_DOUBLES = 2 * GAP_PARTS + 2 * WSQ_PARTS;
constexpr int MAX_DEVICES = 64;

}  // namespace

static __device__ __align__(256) double scratch[STATIC_SCRATCH_DOUBLES];

namespace {

// Device address of `scratch` on the current device (in host code the array's name is not one), looked
// up once per device.
double *scratch_ptr[MAX_DEVICES];
bool scratch_known[MAX_DEVICES];
std::mutex scratch_mutex;

hipError_t static_scratch_of_current_device(double **out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_known[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        scratch_ptr[dev] = (double *)p;
        scratch_known[dev] = true;
    }
    *out = scratch_ptr[dev];
    return hipSuccess;
}

}  // namespace

struct chicle_ctx {
    int loss = 0;
    int64_t n_total = 0;
    int32_t d = 0;
    int64_t ld_v = 0;
    double lambda = 0;
    double l1 = 0;             // elastic net: regulariser lambda (|w|^2 / 2 + l1 |w|_1); w64 then holds the dual image
    int32_t n_chunks = 0, max_solvers = 0;
    bool dense = false;        // chunks stored as dense row-major matrices
    bool api_dense = false;    // chunks arrive through chicle_load_chunk_dense
    int64_t total_entries = 0;
    char *arena = nullptr;
    size_t arena_bytes = 0, used = 0;
    hipStream_t stream = nullptr;
    State state = ST_LOADING;
    int solver_kind = CHICLE_SOLVER_AUTO;

    // fixed regions
    ChunkDev *chunks_dev = nullptr;
    SolverDev *solvers_dev = nullptr;
    int32_t *solver_chunks_dev = nullptr, *solver_prefix_dev = nullptr, *item_prefix_dev = nullptr;
    double *w64 = nullptr;     // shared vector (internal column order), double precision
    float *w = nullptr;        // its float mirror, gathered by the float kernels
    float *u = nullptr;        // private vectors as differences u_k = v_k - w, max_solvers x ld_v
    float *tmp_a = nullptr, *tmp_b = nullptr;   // d floats each: staging of host transfers
    int32_t *rank_of = nullptr, *col_of = nullptr;   // column renumbering tables (device)
    bool renumbered = false;
    int32_t max_row_len = 0;
    float *tiles[2] = {nullptr, nullptr};   // Gram tiles: one set in use by the chain, one being prepared
    int tile_buf = 0;                       // set the next chain kernel reads
    hipStream_t side = nullptr;             // stream of Gram kernels prepared ahead
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    // Visiting orders announced for the next pass are copied here when they are announced (two buffers: the
    // running pass may itself read announced orders), so the caller's buffer is not referred to afterwards.
    int32_t *perm_ahead[2] = {nullptr, nullptr};
    int ahead_buf = 0;                      // buffer the next announcement goes to
    bool ahead_valid = false;               // perm_ahead[1 - ahead_buf] holds the orders of the next pass
    bool ahead_tiles = false;               // ... and their Gram tiles are in tiles[1 - tile_buf] (side stream)
    int32_t *tile_solver_dev = nullptr;
    int32_t *row_chunk_dev = nullptr, *chunk_first_dev = nullptr, *list_base_dev = nullptr;
    int64_t max_tiles = 0;
    int32_t n_tiles = 0;
    bool zw_valid = true;      // the rows' residuals match w (set at load time for w = 0)
    int32_t *perm_stage = nullptr;
    GapScratch gap_scratch;           // in the arena
    double *static_scratch = nullptr; // this device's copy of the fixed scratch array (chicle_gap_noalloc)
    double *gap_host = nullptr;       // 4 doubles of pinned host memory the gap's last kernel writes into ...
    double *gap_host_dev = nullptr;   // ... through this device address
    int *err_dev = nullptr;
    int *progress_dev = nullptr;      // per solver: block its batched pass has reached
    unsigned long long *split_ring_dev = nullptr;   // per solver: rings between the workgroups that share it
    bool split_allowed = true;        // the batched solver may spread a solver over several compute units
    int max_tail_entries = 0;         // most entries a row has outside the columns the batched solver keeps on chip
    // long sparse rows: several workgroups (a cluster) share every solver of the row-wise pass
    bool long_rows = false;           // average row longer than LONG_ROW_AVG
    int32_t *row_split_dev = nullptr; // per row: where the columns of cluster members 1.. begin
    unsigned long long *cluster_ring_dev = nullptr;
    int cluster = 1;                  // members per solver under the current assignment
    int split_built_for = 0;          // cluster size row_split_dev was built for
    int32_t *slice_off_dev = nullptr; // long rows: (slices + 1) x n_total run boundaries of the sliced gap row pass
    double *slice_z_dev = nullptr;    // n_total partial dot products (float or double), zero between passes
    int gap_slices = 0, gap_slice_shift = 0;   // 0: the sliced row pass is not in use
    bool cluster_allowed = true;
    // Sparse chunks: private vectors are stored compactly (a solver touches a small part of the columns)
    bool compact = false;
    int64_t words = 0;                // 32-column words per bitmap
    unsigned *bits_dev = nullptr;     // max_solvers x words: columns a solver's chunks contain
    unsigned *multi_dev = nullptr;    // long rows: the same layout, columns that more than one row of the solver holds
    int32_t *pref_dev = nullptr;      // max_solvers x words: set bits before each word
    int32_t *count_dev = nullptr;     // max_solvers: columns per solver
    int64_t *u_off_dev = nullptr;     // max_solvers: start of each solver's compact vector in u
    int32_t *chunk_owner_dev = nullptr;
    int64_t u_capacity = 0;           // floats in u
    int64_t u_used = 0;               // floats of u in use under the current assignment (compact storage)
    int cu_count = 0;                 // compute units of the device
    long long *ticks_dev = nullptr;   // 2 per solver: clock at start / end of its last pass
    int wall_khz = 0;                 // rate of that clock
    bool epoch_ran = false;

    // host mirrors
    std::vector<ChunkDev> chunks;
    std::vector<char> loaded;
    int32_t n_loaded = 0;
    int64_t rows_loaded = 0, entries_loaded = 0;
    int32_t K = 0;
    std::vector<int32_t> chunk_to_solver;
    std::vector<SolverDev> solvers;
    int max_list = 0;
    int gap_lpr = 64, gap_items = 0, gap_hot_grid = 0;

    bool profiling = false;
    Seg seg[CHICLE_SEG_COUNT];
    std::string err;
};

namespace {

int fail(chicle_ctx *c, int code, const char *fmt, ...)
{
    if (c) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        c->err = buf;
    }
    return code;
}

#define HIP_TRY(c, expr)                                                                         \
    do {                                                                                         \
        hipError_t e_ = (expr);                                                                  \
        if (e_ != hipSuccess)                                                                    \
            return fail((c), CHICLE_EDEVICE, "%s: %s", #expr, hipGetErrorString(e_));            \
    } while (0)

void *carve(chicle_ctx *c, size_t bytes)
{
    const size_t need = align_up(bytes);
    if (c->used + need > c->arena_bytes) return nullptr;
    void *p = c->arena + c->used;
    c->used += need;
    return p;
}

// Floats of private-vector storage: dense, one vector per solver; compact (long rows): a solver's vector
// holds only the columns its chunks contain, so all of them together hold at most one float per entry.
int64_t private_floats(int64_t total_entries, int64_t ld, int32_t max_solvers, bool long_rows)
{
    const int64_t dense = ld * (int64_t)max_solvers;
    return long_rows ? std::min(dense, total_entries + 64 * (int64_t)max_solvers) : dense;
}

// Columns [0, forced) of a compact vector are always present (the batched solver keeps them on chip and
// addresses them by column id); at most this many.

// Slices of the sliced gap row pass at most (the shared vector in double).
int max_slices(int32_t d)
{
    const int shift = SLICE_BYTES_LOG2 - 3;
    return (int)(((int64_t)d + (1 << shift) - 1) >> shift);
}

size_t fixed_bytes(int64_t n_total, int32_t d, int32_t n_chunks, int32_t max_solvers, bool long_rows, bool compact,
                   int64_t n_total_entries_hint)
{
    const int64_t ld = pad_d(d);
    size_t s = 0;
    s += align_up(sizeof(ChunkDev) * (size_t)n_chunks);
    s += align_up(sizeof(SolverDev) * (size_t)max_solvers);
    s += 2 * align_up(sizeof(int32_t) * (size_t)n_chunks);
    s += align_up(sizeof(int32_t) * ((size_t)n_chunks + 1));
    s += align_up(sizeof(float) * (size_t)ld) * 3;                       // w, tmp_a, tmp_b
    s += align_up(sizeof(double) * (size_t)ld);                          // w in double
    s += align_up(sizeof(float) * (size_t)private_floats(n_total_entries_hint, ld, max_solvers, long_rows));   // private vectors
    s += 2 * align_up(sizeof(int32_t) * (size_t)d);                      // renumbering tables
    s += 2 * align_up(sizeof(float) * (size_t)TILE_FLOATS * (size_t)tiles_cap(n_total, max_solvers));
    s += align_up(sizeof(int32_t) * (size_t)tiles_cap(n_total, max_solvers));
    s += 4 * align_up(sizeof(int32_t) * (size_t)n_total);                // perm staging, announced orders (2), row -> chunk
    s += 2 * align_up(sizeof(int32_t) * (size_t)n_chunks);               // chunk_first, list_base
    s += 2 * align_up(sizeof(double) * (size_t)std::max(GAP_PARTS, 2 * n_chunks)) + 2 * align_up(sizeof(double) * WSQ_PARTS);
    s += align_up(sizeof(int));
    s += align_up(sizeof(long long) * 2 * (size_t)max_solvers);
    s += align_up(sizeof(int) * (size_t)max_solvers);
    s += align_up(sizeof(unsigned long long) * (size_t)SPLIT_WORDS * (size_t)max_solvers);   // rings of the split batched solver
    if (long_rows) {
        s += align_up(sizeof(int32_t) * ((size_t)max_slices(d) + 1) * (size_t)n_total) + align_up(sizeof(double) * (size_t)n_total);
        s += align_up(sizeof(int32_t) * (size_t)SPLITS_PER_ROW * (size_t)n_total);
        s += align_up(sizeof(unsigned long long) * (size_t)CLUSTER_WORDS * (size_t)max_solvers);
    }
    if (compact) {
        const size_t words = ((size_t)d + 31) / 32;
        s += 2 * align_up(sizeof(int32_t) * words * (size_t)max_solvers);          // column bitmaps, prefix counts
        if (long_rows) s += align_up(sizeof(int32_t) * words * (size_t)max_solvers);   // columns held by several rows
        s += align_up(sizeof(int32_t) * (size_t)max_solvers) + align_up(sizeof(int64_t) * (size_t)max_solvers);
        s += align_up(sizeof(int32_t) * (size_t)n_chunks);
    }
    return s;
}

size_t chunk_bytes(bool dense, bool compact, int64_t n_rows, int64_t entries)
{
    size_t s = 0;
    if (!dense) {
        s += align_up(sizeof(int32_t) * (size_t)(n_rows + 1));
        s += align_up(sizeof(int32_t) * (size_t)(entries + ENTRY_SLACK)) * (compact ? 2 : 1);   // column ids (+ compact ids)
    }
    s += align_up(sizeof(float) * (size_t)(entries + ENTRY_SLACK));
    s += align_up(sizeof(RowState) * (size_t)n_rows);
    return s;
}

void seg_begin(chicle_ctx *c, int s)
{
    if (c->profiling) (void)hipEventRecord(c->seg[s].start, c->stream);
}
void seg_end(chicle_ctx *c, int s)
{
    if (c->profiling) {
        (void)hipEventRecord(c->seg[s].stop, c->stream);
        c->seg[s].recorded = true;
    }
}

int check_deferred(chicle_ctx *c)
{
    int flag = 0;
    HIP_TRY(c, hipMemcpyAsync(&flag, c->err_dev, sizeof(int), hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (flag) {
        HIP_TRY(c, hipMemsetAsync(c->err_dev, 0, sizeof(int), c->stream));
        if (flag & ERR_PERM_RANGE)
            return fail(c, CHICLE_EDEVICE, "a visiting-order entry was outside [0, rows of its solver)");
        if (flag & ERR_PARTNER_TIMEOUT)
            return fail(c, CHICLE_EDEVICE, "the workgroups that share a solver lost each other; the pass is invalid");
        return fail(c, CHICLE_EDEVICE, "kernel error flag %d", flag);
    }
    return CHICLE_OK;
}

int grid_for(int64_t items, int per_block, int cap)
{
    int64_t g = (items + per_block - 1) / per_block;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (int)g;
}

void clear_device_words(chicle_ctx *c, void *p, int64_t n_words)
{
    hipLaunchKernelGGL(clear_words, dim3(grid_for(n_words, 256, 256)), dim3(256), 0, c->stream, (unsigned *)p, n_words);
}

int clear_all_private(chicle_ctx *c)
{
    if (c->K <= 0) return CHICLE_OK;
    if (c->compact) {
        HIP_TRY(c, hipMemsetAsync(c->u, 0, sizeof(float) * (size_t)c->u_used, c->stream));
        return CHICLE_OK;
    }
    const int64_t d4 = c->ld_v / 4;
    hipLaunchKernelGGL(clear_private, dim3(grid_for(d4, 256, 4096)), dim3(256), 0, c->stream, c->u,
                       c->ld_v, d4, c->K);
    HIP_TRY(c, hipGetLastError());
    return CHICLE_OK;
}

RoundScalars scalars(const chicle_ctx *c)
{
    RoundScalars s;
    const double cc = c->lambda * (double)c->n_total / (double)c->K;
    s.c = (float)cc;
    s.inv_c = (float)(1.0 / cc);
    s.inv_sigma = (float)(1.0 / (double)c->K);
    s.K = c->K;
    s.ticks = c->ticks_dev;
    return s;
}

// Dense rows short enough for the batched solver are stored with explicit column ids (row-major,
// columns 0 .. d-1): twice the bytes of the dense form, and every machinery for short sparse rows
// applies to them unchanged.
bool dense_as_csr(int32_t d) { return d <= GRAM_MAX_ROW; }

bool batched_eligible(const chicle_ctx *c)
{
    return !c->dense && c->max_row_len <= GRAM_MAX_ROW && c->max_list <= BATCHED_MAX_LIST;
}

// LDS layout of the batched solvers: BatchedShared, the solver's chunk descriptors and row prefixes, then
// the head of the private vector (the most popular columns, as many as fit), in double.
struct BatchedLayout { size_t hot_off, bytes; int n_hot; };
BatchedLayout batched_layout(const chicle_ctx *c)
{
    BatchedLayout L;
    const int ml = std::max(c->max_list, 1);
    L.hot_off = (sizeof(BatchedShared) + (sizeof(ChunkDev) + sizeof(int)) * (size_t)ml + 15) & ~(size_t)15;
    L.n_hot = (int)std::min<int64_t>((int64_t)((LDS_BYTES - L.hot_off) / sizeof(double)) & ~(int64_t)63, c->d);
    L.bytes = L.hot_off + sizeof(double) * (size_t)L.n_hot;
    return L;
}

// Dense rows too wide to be stored with column ids, narrow enough for a block of 64 to sit in LDS.
bool dense_blocked_eligible(const chicle_ctx *c)
{
    return c->dense && c->d <= DB_MAX_D;
}

template <int LOSS>
int launch_dense_blocked(chicle_ctx *c, const int32_t *perm)
{
    const RoundScalars sc = scalars(c);
    const int ml = std::max(c->max_list, 1);
    const size_t sh = sizeof(float) * db_lds_floats((int)c->d) + 2 * sizeof(int) * (size_t)ml;
    auto kern = sdca_batched_dense<LOSS>;
    HIP_TRY(c, hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh));
    hipLaunchKernelGGL(kern, dim3(c->K), dim3(DB_THREADS), sh, c->stream, c->chunks_dev, c->solvers_dev,
                       c->solver_chunks_dev, c->solver_prefix_dev, perm, c->u, c->ld_v, (int)c->d, ml, sc,
                       c->err_dev);
    HIP_TRY(c, hipGetLastError());
    return CHICLE_OK;
}

template <int LOSS>
int launch_rowwise(chicle_ctx *c, const int32_t *perm)
{
    const RoundScalars sc = scalars(c);
    const size_t list_bytes = 2 * sizeof(int) * (size_t)std::max(c->max_list, 1);
    if (c->dense) {
        const bool v_lds = c->d <= DENSE_V_LDS_MAX_D;
        const size_t sh = list_bytes + (v_lds ? sizeof(float) * (size_t)c->d : 0);
        if (v_lds)
            hipLaunchKernelGGL((sdca_rowwise_dense<LOSS, 64, true>), dim3(c->K), dim3(64), sh, c->stream,
                               c->chunks_dev, c->solvers_dev, c->solver_chunks_dev, c->solver_prefix_dev,
                               perm, c->u, c->ld_v, (int)c->d, std::max(c->max_list, 1), sc, c->err_dev);
        else
            hipLaunchKernelGGL((sdca_rowwise_dense<LOSS, 256, false>), dim3(c->K), dim3(256), sh, c->stream,
                               c->chunks_dev, c->solvers_dev, c->solver_chunks_dev, c->solver_prefix_dev,
                               perm, c->u, c->ld_v, (int)c->d, std::max(c->max_list, 1), sc, c->err_dev);
    } else {
        const double avg = c->n_total ? (double)c->total_entries / (double)c->n_total : 0.0;
        const int ml = std::max(c->max_list, 1);
        const size_t sh = (sizeof(ChunkDev) + sizeof(int)) * (size_t)ml;
        if (c->long_rows && c->cluster > 1 && c->cluster_allowed) {
            // every solver shared by a cluster of workgroups on one L2 partition, each owning a range of columns
            const int k_pad = (c->K + L2_PARTITIONS - 1) / L2_PARTITIONS * L2_PARTITIONS;
            clear_device_words(c, c->cluster_ring_dev, 2 * (int64_t)CLUSTER_WORDS * c->K);
            hipLaunchKernelGGL((sdca_rowwise_csr_cluster<LOSS, 512, 2>), dim3(k_pad * c->cluster), dim3(512), sh, c->stream,
                               c->chunks_dev, c->solvers_dev, c->solver_chunks_dev, c->solver_prefix_dev,
                               perm, c->u, c->ld_v, ml, sc, c->err_dev, k_pad, c->cluster, c->row_split_dev,
                               c->cluster_ring_dev, c->u_off_dev);
        } else if (avg <= LONG_ROW_AVG)
            hipLaunchKernelGGL((sdca_rowwise_csr<LOSS, 64, 2>), dim3(c->K), dim3(64), sh, c->stream,
                               c->chunks_dev, c->solvers_dev, c->solver_chunks_dev, c->solver_prefix_dev,
                               perm, c->u, c->ld_v, ml, sc, c->err_dev, (const int64_t *)(c->compact ? c->u_off_dev : nullptr));
        else
            hipLaunchKernelGGL((sdca_rowwise_csr<LOSS, 512, 4>), dim3(c->K), dim3(512), sh, c->stream,
                               c->chunks_dev, c->solvers_dev, c->solver_chunks_dev, c->solver_prefix_dev,
                               perm, c->u, c->ld_v, ml, sc, c->err_dev, (const int64_t *)c->u_off_dev);
    }
    HIP_TRY(c, hipGetLastError());
    return CHICLE_OK;
}

// Gram tiles of the given visiting orders into tile set `buf`, on `stream`.
template <int LOSS>
int launch_gram(chicle_ctx *c, const int32_t *perm, int buf, hipStream_t stream)
{
    const RoundScalars sc = scalars(c);
    if (c->n_tiles > 0) {
        auto kern = gram_tiles_join<LOSS>;
        HIP_TRY(c, hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)sizeof(GramShared)));
        // each workgroup takes a contiguous run of tiles (neighbouring tiles share half their rows)
        const int grid = std::min(c->n_tiles, 2048);
        hipLaunchKernelGGL(kern, dim3(grid), dim3(GRAM_THREADS), sizeof(GramShared), stream,
                           c->chunks_dev, c->solvers_dev, c->row_chunk_dev, c->chunk_first_dev, perm,
                           c->tile_solver_dev, c->tiles[buf], c->n_tiles, sc.c, c->err_dev);
    }
    HIP_TRY(c, hipGetLastError());
    return CHICLE_OK;
}

// The batched local pass.  Tiles of `perm` come from the set prepared ahead when there is one, else
// they are computed first on the main stream.  With perm_next, the tiles of the next pass are started
// on the side stream so that they run beside this pass's chain kernel (which occupies K of the 256
// compute units); they depend on the data and the orders only.
template <int LOSS>
int launch_batched(chicle_ctx *c, const int32_t *perm, bool tiles_ready, const int32_t *perm_next)
{
    const RoundScalars sc = scalars(c);
    int rc;
    if (tiles_ready) {
        c->tile_buf = 1 - c->tile_buf;
        HIP_TRY(c, hipStreamWaitEvent(c->stream, c->ev_join, 0));
    } else {
        if (c->ahead_tiles) HIP_TRY(c, hipStreamWaitEvent(c->stream, c->ev_join, 0));   // unused, but let it finish
        seg_begin(c, CHICLE_SEG_EPOCH_GRAM);
        rc = launch_gram<LOSS>(c, perm, c->tile_buf, c->stream);
        seg_end(c, CHICLE_SEG_EPOCH_GRAM);
        if (rc) return rc;
    }
    c->ahead_tiles = false;
    if (perm_next) HIP_TRY(c, hipEventRecord(c->ev_fork, c->stream));   // everything enqueued so far
    const int ml = std::max(c->max_list, 1);
    const BatchedLayout lay = batched_layout(c);
    const size_t hot_off = lay.hot_off, sh = lay.bytes;
    const int n_hot = lay.n_hot;
    const int64_t *u_off = c->compact ? c->u_off_dev : nullptr;
    const int k_pad = (c->K + L2_PARTITIONS - 1) / L2_PARTITIONS * L2_PARTITIONS;
    // Columns outside the LDS-resident head, and compute units to spare: every solver gets a head workgroup
    // and SPLIT_TAILS tail workgroups (all of them must be resident together: they wait for each other).
    // (where every column is in the LDS-resident head there is nothing for tails to do: the head workgroups run
    // alone, and their gathers and scatters never leave LDS)
    const int n_tails = n_hot < c->d ? SPLIT_TAILS : 0;
    const bool split = c->split_allowed && (1 + n_tails) * k_pad <= c->cu_count &&
                       (n_tails == 0 || sizeof(double) * (size_t)n_hot >= 2 * RING * BATCH * sizeof(RowSlot));   // a tail keeps its rows there
    if (split) {
        SplitArgs A;
        A.chunks = c->chunks_dev; A.solvers = c->solvers_dev; A.solver_chunks = c->solver_chunks_dev;
        A.solver_prefix = c->solver_prefix_dev; A.perm = perm; A.tiles = c->tiles[c->tile_buf]; A.u_all = c->u;
        A.ld_v = c->ld_v; A.u_off = u_off; A.max_list = ml; A.n_hot = n_hot; A.hot_off = (int)hot_off; A.sc = sc;
        A.err = c->err_dev; A.n_tails = n_tails; A.xchg_all = c->split_ring_dev;
        // a tail's helper lanes take the last 24 entries of a row where that covers every row's unpopular columns
        const bool short_tail = c->compact && c->max_tail_entries <= 3 * LPR;
        auto kern = short_tail ? sdca_batched_split<LOSS, 3> : sdca_batched_split<LOSS, ENT>;
        HIP_TRY(c, hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh));
        clear_device_words(c, c->split_ring_dev, 2 * (int64_t)SPLIT_WORDS * c->K);
        seg_begin(c, CHICLE_SEG_EPOCH_CHAIN);
        hipLaunchKernelGGL(kern, dim3((1 + n_tails) * k_pad), dim3(SPLIT_THREADS), sh, c->stream, A, k_pad);
        seg_end(c, CHICLE_SEG_EPOCH_CHAIN);
    } else {
        auto kern = sdca_batched_csr<LOSS>;
        HIP_TRY(c, hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh));
        const int first_warmer = k_pad;
        clear_device_words(c, c->progress_dev, c->K);
        seg_begin(c, CHICLE_SEG_EPOCH_CHAIN);
        hipLaunchKernelGGL(kern, dim3(first_warmer + c->K), dim3(BATCHED_THREADS), sh, c->stream, c->chunks_dev,
                           c->solvers_dev, c->solver_chunks_dev, c->solver_prefix_dev, perm, c->tiles[c->tile_buf], c->u,
                           c->ld_v, u_off, ml, n_hot, (int)hot_off, sc, c->err_dev, c->progress_dev, first_warmer);
        seg_end(c, CHICLE_SEG_EPOCH_CHAIN);
    }
    HIP_TRY(c, hipGetLastError());
    if (perm_next) {
        // the other tile set was last read by the previous pass's chain kernel, which precedes ev_fork
        HIP_TRY(c, hipStreamWaitEvent(c->side, c->ev_fork, 0));
        if (c->profiling) (void)hipEventRecord(c->seg[CHICLE_SEG_EPOCH_GRAM].start, c->side);
        rc = launch_gram<LOSS>(c, perm_next, 1 - c->tile_buf, c->side);
        if (c->profiling) {
            (void)hipEventRecord(c->seg[CHICLE_SEG_EPOCH_GRAM].stop, c->side);
            c->seg[CHICLE_SEG_EPOCH_GRAM].recorded = true;
        }
        if (rc) return rc;
        HIP_TRY(c, hipEventRecord(c->ev_join, c->side));
        c->ahead_tiles = true;
    }
    return CHICLE_OK;
}

// Work prepared ahead refers to the solver tables: finish it before they change.
int drop_ahead(chicle_ctx *c)
{
    if (c->side) HIP_TRY(c, hipStreamSynchronize(c->side));
    c->ahead_tiles = false;
    c->ahead_valid = false;
    return CHICLE_OK;
}

template <int LOSS, int LPRG, typename WT>
void launch_gap_rows_t(chicle_ctx *c, int grid_x, const WT *w, const GapScratch &gs)
{
    const dim3 grid(grid_x, c->n_chunks);
    if (c->gap_hot_grid > 0) {
        // lanes per row: the fewest that cover the longest row with 4 entries each
        const int n_hot = (int)std::min<int64_t>(c->d, GAP_HOT_BYTES / (int)sizeof(WT));
        const dim3 hg(c->gap_hot_grid, c->n_chunks);
        const size_t sh = n_hot * sizeof(WT);
        const int need = (c->max_row_len + 3) / 4;
#define CHICLE_GAP_HOT(L)                                                                                   \
        hipLaunchKernelGGL((gap_rows_csr_hot<LOSS, L, WT>), hg, dim3(GAP_HOT_THREADS), sh, c->stream,      \
                           c->chunks_dev, w, c->l1, n_hot, gs.loss, gs.conj)
        if (need <= 4) CHICLE_GAP_HOT(4);
        else if (need <= 8) CHICLE_GAP_HOT(8);
        else if (need <= 10) CHICLE_GAP_HOT(10);
        else if (need <= 12) CHICLE_GAP_HOT(12);
        else CHICLE_GAP_HOT(16);
#undef CHICLE_GAP_HOT
    } else if (c->dense)
        hipLaunchKernelGGL((gap_rows_dense<LOSS, LPRG, WT>), grid, dim3(256), 0, c->stream, c->chunks_dev,
                           (int)c->d, w, c->l1, gs.loss, gs.conj);
    else
        hipLaunchKernelGGL((gap_rows_csr<LOSS, LPRG, WT>), grid, dim3(256), 0, c->stream, c->chunks_dev, w, c->l1,
                           gs.loss, gs.conj);
}

// Squared loss: dot products in double against the double w (its steps cancel y - z - alpha down to the
// size of the update); logistic: in double as well (loss and conjugate nearly cancel in the gap close to
// the optimum); hinge: float against the float mirror.
template <int LOSS, int LPRG>
void launch_gap_rows(chicle_ctx *c, int grid, const GapScratch &gs)
{
    if (LOSS != 0) launch_gap_rows_t<LOSS, LPRG, double>(c, grid, c->w64, gs);
    else launch_gap_rows_t<LOSS, LPRG, float>(c, grid, c->w, gs);
}

template <int LOSS>
void launch_gap_lpr(chicle_ctx *c, int grid, const GapScratch &gs)
{
    switch (c->gap_lpr) {
        case 4: launch_gap_rows<LOSS, 4>(c, grid, gs); break;
        case 8: launch_gap_rows<LOSS, 8>(c, grid, gs); break;
        case 16: launch_gap_rows<LOSS, 16>(c, grid, gs); break;
        case 32: launch_gap_rows<LOSS, 32>(c, grid, gs); break;
        default: launch_gap_rows<LOSS, 64>(c, grid, gs); break;
    }
}

// The row pass of the gap: z_i = x_i . w into the chunks, loss and conjugate partial sums.
int run_row_pass(chicle_ctx *c, int *grid_out, const GapScratch &gs)
{
    // workgroups per chunk: enough to fill the chip several times over, within the partial-sum arrays
    int max_rows = 1;
    for (const ChunkDev &ch : c->chunks) max_rows = std::max(max_rows, ch.n_rows);
    const int rows_per_wg = 2 * (256 / c->gap_lpr);
    int gx = std::min((max_rows + rows_per_wg - 1) / rows_per_wg, std::max(1, 8192 / c->n_chunks));
    gx = std::max(1, std::min(gx, gs.parts / c->n_chunks));
    // popularity-numbered columns: frequent part of w from LDS, few large workgroups per chunk
    c->gap_hot_grid = 0;
    if (c->renumbered && !c->dense && c->max_row_len <= 4 * GAP_HOT_MAX_LPR) {
        const int lpr = std::max(4, (c->max_row_len + 3) / 4);
        const int rows_per_hot_wg = 2 * (GAP_HOT_THREADS / 64) * (64 / lpr);
        gx = std::max(1, std::min(std::min(2, (max_rows + rows_per_hot_wg - 1) / rows_per_hot_wg),
                                  gs.parts / c->n_chunks));
        c->gap_hot_grid = gx;
    }
    if (c->gap_slices > 0) {
        const int segs = (max_rows + SLICE_SEG - 1) / SLICE_SEG, n_items = segs * c->n_chunks;
        const unsigned blocks = (unsigned)((c->gap_slices + L2_PARTITIONS - 1) / L2_PARTITIONS * L2_PARTITIONS) * (unsigned)n_items;
        gx = std::max(1, std::min((max_rows + 255) / 256, gs.parts / c->n_chunks));
        const dim3 fg(gx, c->n_chunks);
        if (c->loss == CHICLE_LOSS_HINGE) {
            float *z = (float *)c->slice_z_dev;
            hipLaunchKernelGGL(gap_rows_sliced<float>, dim3(blocks), dim3(256), 0, c->stream, c->chunks_dev, (const float *)c->w, c->l1,
                               c->slice_off_dev, c->n_total, c->gap_slices, segs, n_items, z);
            hipLaunchKernelGGL((gap_rows_from_z<0, float>), fg, dim3(256), 0, c->stream, c->chunks_dev, z, gs.loss, gs.conj);
        } else {
            hipLaunchKernelGGL(gap_rows_sliced<double>, dim3(blocks), dim3(256), 0, c->stream, c->chunks_dev, (const double *)c->w64, c->l1,
                               c->slice_off_dev, c->n_total, c->gap_slices, segs, n_items, c->slice_z_dev);
            if (c->loss == CHICLE_LOSS_SQUARED)
                hipLaunchKernelGGL((gap_rows_from_z<1, double>), fg, dim3(256), 0, c->stream, c->chunks_dev, c->slice_z_dev, gs.loss, gs.conj);
            else
                hipLaunchKernelGGL((gap_rows_from_z<2, double>), fg, dim3(256), 0, c->stream, c->chunks_dev, c->slice_z_dev, gs.loss, gs.conj);
        }
    } else if (c->loss == CHICLE_LOSS_HINGE) launch_gap_lpr<0>(c, gx, gs);
    else if (c->loss == CHICLE_LOSS_SQUARED) launch_gap_lpr<1>(c, gx, gs);
    else launch_gap_lpr<2>(c, gx, gs);
    HIP_TRY(c, hipGetLastError());
    c->zw_valid = true;
    if (grid_out) *grid_out = gx * c->n_chunks;
    return CHICLE_OK;
}

int choose_lpr(double avg_row_len)
{
    if (avg_row_len <= 6) return 4;
    if (avg_row_len <= 12) return 8;
    if (avg_row_len <= 48) return 16;
    return 64;
}

// Greedy table of chicle_balance; integers only.
void greedy_table(const int64_t *load, int32_t n_chunks, int32_t K, const int32_t *speed, int32_t *out)
{
    std::vector<int32_t> order(n_chunks);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(),
                     [&](int32_t a, int32_t b) { return load[a] > load[b]; });
    std::vector<int64_t> L(K, 0);
    for (int32_t c : order) {
        int32_t best = 0;
        for (int32_t k = 1; k < K; ++k) {
            const __int128 fk = (__int128)(L[k] + load[c]) * (speed ? speed[best] : 1);
            const __int128 fb = (__int128)(L[best] + load[c]) * (speed ? speed[k] : 1);
            if (fk < fb) best = k;
        }
        out[c] = best;
        L[best] += load[c];
    }
}

// Once, when every chunk is in HBM: renumber the columns by popularity and re-sort the rows.
int renumber_columns(chicle_ctx *c)
{
    int32_t *count = c->rank_of;   // the table is built in place of the counts
    HIP_TRY(c, hipMemsetAsync(count, 0, sizeof(int32_t) * (size_t)c->d, c->stream));
    hipLaunchKernelGGL(count_columns, dim3(c->n_chunks), dim3(256), 0, c->stream, c->chunks_dev, count);
    HIP_TRY(c, hipGetLastError());
    std::vector<int32_t> cnt(c->d), order(c->d), rank(c->d);
    HIP_TRY(c, hipMemcpyAsync(cnt.data(), count, sizeof(int32_t) * (size_t)c->d, hipMemcpyDeviceToHost, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return cnt[a] > cnt[b]; });
    for (int32_t r = 0; r < c->d; ++r) rank[order[r]] = r;
    HIP_TRY(c, hipMemcpyAsync(c->rank_of, rank.data(), sizeof(int32_t) * (size_t)c->d, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->col_of, order.data(), sizeof(int32_t) * (size_t)c->d, hipMemcpyHostToDevice, c->stream));
    int max_rows = 1;
    for (const ChunkDev &ch : c->chunks) max_rows = std::max(max_rows, ch.n_rows);
    hipLaunchKernelGGL(renumber_rows, dim3(grid_for(max_rows, 256, 64), c->n_chunks), dim3(256), 0, c->stream,
                       c->chunks_dev, c->rank_of);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->renumbered = true;
    return CHICLE_OK;
}

}  // namespace

extern "C" {

size_t chicle_arena_bytes(int64_t n_total, int64_t total_entries, int32_t d, int32_t n_chunks,
                          int32_t max_solvers, int32_t dense)
{
    if (n_total <= 0 || total_entries < 0 || d <= 0 || n_chunks <= 0 || max_solvers <= 0) return 0;
    const bool long_rows = !dense && (double)total_entries > LONG_ROW_AVG * (double)n_total;
    const bool compact = !dense;
    size_t s = fixed_bytes(n_total, d, n_chunks, max_solvers, long_rows, compact, total_entries);
    // chunk blocks: exact array bytes plus alignment slack per array and chunk
    const size_t per_chunk_slack = 8 * ALIGN + 2 * sizeof(float) * ENTRY_SLACK;
    if (dense && !dense_as_csr(d))
        s += sizeof(float) * (size_t)total_entries + 4 * sizeof(float) * (size_t)n_total;
    else
        s += (sizeof(int32_t) * (compact ? 2 : 1) + sizeof(float)) * ((size_t)total_entries + (size_t)n_chunks) +
             sizeof(int32_t) * ((size_t)n_total + (size_t)n_chunks) + 4 * sizeof(float) * (size_t)n_total;
    s += (per_chunk_slack + (compact ? ALIGN + sizeof(int32_t) * ENTRY_SLACK : 0)) * (size_t)n_chunks;
    return s + ALIGN;
}

int chicle_create(chicle_ctx **out, int32_t loss, int64_t n_total, int32_t d, double lambda,
                  int32_t n_chunks, int32_t max_solvers, int32_t dense, int64_t total_entries,
                  void *device_arena, size_t arena_bytes, void *hip_stream)
{
    if (!out) return CHICLE_EINVAL;
    *out = nullptr;
    if ((loss != CHICLE_LOSS_HINGE && loss != CHICLE_LOSS_SQUARED && loss != CHICLE_LOSS_LOGISTIC) || n_total <= 0 ||
        n_total > INT32_MAX || d <= 0 || !(lambda > 0.0) || n_chunks <= 0 || max_solvers <= 0 ||
        total_entries < 0 || !device_arena || ((uintptr_t)device_arena % ALIGN) != 0)
        return CHICLE_EINVAL;
    const size_t need = chicle_arena_bytes(n_total, total_entries, d, n_chunks, max_solvers, dense);
    if (arena_bytes < need) return CHICLE_ENOMEM;
    chicle_ctx *c = new (std::nothrow) chicle_ctx();
    if (!c) return CHICLE_ENOMEM;
    c->loss = loss; c->n_total = n_total; c->d = d; c->ld_v = pad_d(d); c->lambda = lambda;
    c->n_chunks = n_chunks; c->max_solvers = max_solvers;
    c->api_dense = dense != 0;
    c->dense = c->api_dense && !dense_as_csr(d);
    c->total_entries = total_entries;
    c->arena = (char *)device_arena; c->arena_bytes = arena_bytes;
    c->stream = (hipStream_t)hip_stream;
    c->max_tiles = tiles_cap(n_total, max_solvers);

    c->chunks_dev = (ChunkDev *)carve(c, sizeof(ChunkDev) * (size_t)n_chunks);
    c->solvers_dev = (SolverDev *)carve(c, sizeof(SolverDev) * (size_t)max_solvers);
    c->solver_chunks_dev = (int32_t *)carve(c, sizeof(int32_t) * (size_t)n_chunks);
    c->solver_prefix_dev = (int32_t *)carve(c, sizeof(int32_t) * (size_t)n_chunks);
    c->item_prefix_dev = (int32_t *)carve(c, sizeof(int32_t) * ((size_t)n_chunks + 1));
    c->w = (float *)carve(c, sizeof(float) * (size_t)c->ld_v);
    c->w64 = (double *)carve(c, sizeof(double) * (size_t)c->ld_v);
    c->tmp_a = (float *)carve(c, sizeof(float) * (size_t)c->ld_v);
    c->tmp_b = (float *)carve(c, sizeof(float) * (size_t)c->ld_v);
    c->long_rows = !c->api_dense && (double)total_entries > LONG_ROW_AVG * (double)n_total;
    c->compact = !c->api_dense;
    c->u_capacity = private_floats(total_entries, c->ld_v, max_solvers, c->long_rows);
    c->u = (float *)carve(c, sizeof(float) * (size_t)c->u_capacity);
    c->rank_of = (int32_t *)carve(c, sizeof(int32_t) * (size_t)d);
    c->col_of = (int32_t *)carve(c, sizeof(int32_t) * (size_t)d);
    c->tiles[0] = (float *)carve(c, sizeof(float) * (size_t)TILE_FLOATS * (size_t)c->max_tiles);
    c->tiles[1] = (float *)carve(c, sizeof(float) * (size_t)TILE_FLOATS * (size_t)c->max_tiles);
    c->tile_solver_dev = (int32_t *)carve(c, sizeof(int32_t) * (size_t)c->max_tiles);
    c->perm_stage = (int32_t *)carve(c, sizeof(int32_t) * (size_t)n_total);
    c->perm_ahead[0] = (int32_t *)carve(c, sizeof(int32_t) * (size_t)n_total);
    c->perm_ahead[1] = (int32_t *)carve(c, sizeof(int32_t) * (size_t)n_total);
    c->row_chunk_dev = (int32_t *)carve(c, sizeof(int32_t) * (size_t)n_total);
    c->chunk_first_dev = (int32_t *)carve(c, sizeof(int32_t) * (size_t)n_chunks);
    c->list_base_dev = (int32_t *)carve(c, sizeof(int32_t) * (size_t)n_chunks);
    c->gap_scratch.parts = std::max(GAP_PARTS, 2 * n_chunks);
    c->gap_scratch.loss = (double *)carve(c, sizeof(double) * (size_t)c->gap_scratch.parts);
    c->gap_scratch.conj = (double *)carve(c, sizeof(double) * (size_t)c->gap_scratch.parts);
    c->gap_scratch.wsq = (double *)carve(c, sizeof(double) * WSQ_PARTS);
    c->gap_scratch.unused = (double *)carve(c, sizeof(double) * WSQ_PARTS);
    c->err_dev = (int *)carve(c, sizeof(int));
    c->ticks_dev = (long long *)carve(c, sizeof(long long) * 2 * (size_t)max_solvers);
    c->progress_dev = (int *)carve(c, sizeof(int) * (size_t)max_solvers);
    c->split_ring_dev = (unsigned long long *)carve(c, sizeof(unsigned long long) * (size_t)SPLIT_WORDS * (size_t)max_solvers);
    if (c->long_rows) {
        c->slice_off_dev = (int32_t *)carve(c, sizeof(int32_t) * ((size_t)max_slices(d) + 1) * (size_t)n_total);
        c->slice_z_dev = (double *)carve(c, sizeof(double) * (size_t)n_total);
        c->row_split_dev = (int32_t *)carve(c, sizeof(int32_t) * (size_t)SPLITS_PER_ROW * (size_t)n_total);
        c->cluster_ring_dev = (unsigned long long *)carve(c, sizeof(unsigned long long) * (size_t)CLUSTER_WORDS * (size_t)max_solvers);
    }
    if (c->compact) {
        c->words = ((int64_t)d + 31) / 32;
        c->bits_dev = (unsigned *)carve(c, sizeof(unsigned) * (size_t)c->words * (size_t)max_solvers);
        c->pref_dev = (int32_t *)carve(c, sizeof(int32_t) * (size_t)c->words * (size_t)max_solvers);
        if (c->long_rows) c->multi_dev = (unsigned *)carve(c, sizeof(unsigned) * (size_t)c->words * (size_t)max_solvers);
        c->count_dev = (int32_t *)carve(c, sizeof(int32_t) * (size_t)max_solvers);
        c->u_off_dev = (int64_t *)carve(c, sizeof(int64_t) * (size_t)max_solvers);
        c->chunk_owner_dev = (int32_t *)carve(c, sizeof(int32_t) * (size_t)n_chunks);
    }
    if (!c->err_dev || !c->ticks_dev || !c->progress_dev || !c->split_ring_dev || (c->long_rows && (!c->cluster_ring_dev || !c->slice_z_dev)) || (c->compact && (!c->chunk_owner_dev || (c->long_rows && !c->multi_dev)))) { delete c; return CHICLE_ENOMEM; }

    c->chunks.assign(n_chunks, ChunkDev{});
    c->loaded.assign(n_chunks, 0);
    bool ok = hipMemsetAsync(c->w, 0, sizeof(float) * (size_t)c->ld_v, c->stream) == hipSuccess &&
              hipMemsetAsync(c->w64, 0, sizeof(double) * (size_t)c->ld_v, c->stream) == hipSuccess &&
              hipMemsetAsync(c->tmp_a, 0, sizeof(float) * (size_t)c->ld_v, c->stream) == hipSuccess &&
              hipMemsetAsync(c->tmp_b, 0, sizeof(float) * (size_t)c->ld_v, c->stream) == hipSuccess &&
              hipMemsetAsync(c->u, 0, sizeof(float) * (size_t)c->u_capacity, c->stream) == hipSuccess &&
              hipMemsetAsync(c->err_dev, 0, sizeof(int), c->stream) == hipSuccess &&
              (!c->long_rows || hipMemsetAsync(c->slice_z_dev, 0, sizeof(double) * (size_t)n_total, c->stream) == hipSuccess) &&
              hipMemsetAsync(c->ticks_dev, 0, sizeof(long long) * 2 * (size_t)max_solvers, c->stream) == hipSuccess;
    {
        int dev = 0;
        ok = ok && hipGetDevice(&dev) == hipSuccess &&
             hipDeviceGetAttribute(&c->wall_khz, hipDeviceAttributeWallClockRate, dev) == hipSuccess && c->wall_khz > 0 &&
             hipDeviceGetAttribute(&c->cu_count, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && c->cu_count > 0;
    }
    for (int s = 0; ok && s < CHICLE_SEG_COUNT; ++s)
        ok = hipEventCreate(&c->seg[s].start) == hipSuccess && hipEventCreate(&c->seg[s].stop) == hipSuccess;
    ok = ok && hipHostMalloc((void **)&c->gap_host, sizeof(double) * 8, hipHostMallocMapped) == hipSuccess &&
         hipHostGetDevicePointer((void **)&c->gap_host_dev, c->gap_host, 0) == hipSuccess;
    ok = ok && static_scratch_of_current_device(&c->static_scratch) == hipSuccess;
    ok = ok && hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking) == hipSuccess &&
         hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) == hipSuccess &&
         hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) == hipSuccess;
    if (!ok) { chicle_destroy(c); return CHICLE_EDEVICE; }
    *out = c;
    return CHICLE_OK;
}

static int load_common(chicle_ctx *c, int32_t chunk_id, int32_t n_rows, int64_t entries)
{
    if (c->state != ST_LOADING) return fail(c, CHICLE_ESTATE, "chunks can only be loaded before the first assign");
    if (chunk_id < 0 || chunk_id >= c->n_chunks) return fail(c, CHICLE_EINVAL, "chunk id %d out of range", chunk_id);
    if (c->loaded[chunk_id]) return fail(c, CHICLE_EINVAL, "chunk %d already loaded", chunk_id);
    if (n_rows <= 0) return fail(c, CHICLE_EINVAL, "chunk %d: n_rows must be positive", chunk_id);
    if (c->rows_loaded + n_rows > c->n_total) return fail(c, CHICLE_EINVAL, "more rows than n_total");
    if (c->entries_loaded + entries > c->total_entries)
        return fail(c, CHICLE_EINVAL, "more stored entries than total_entries");
    if (c->used + chunk_bytes(c->dense, c->compact, n_rows, entries) > c->arena_bytes)
        return fail(c, CHICLE_ENOMEM, "chunk store full");
    return CHICLE_OK;
}

static int check_state_arrays(chicle_ctx *c, int32_t chunk_id, int32_t n_rows, const float *y,
                              const float *alpha0)
{
    if (!y) return fail(c, CHICLE_EINVAL, "chunk %d: y is NULL", chunk_id);
    for (int32_t r = 0; r < n_rows; ++r) {
        if (!std::isfinite(y[r])) return fail(c, CHICLE_EINVAL, "chunk %d row %d: label not finite", chunk_id, r);
        if (c->loss != CHICLE_LOSS_SQUARED && y[r] != 1.0f && y[r] != -1.0f)
            return fail(c, CHICLE_EINVAL, "chunk %d row %d: hinge label must be +1 or -1", chunk_id, r);
        if (alpha0) {
            if (!std::isfinite(alpha0[r])) return fail(c, CHICLE_EINVAL, "chunk %d row %d: alpha not finite", chunk_id, r);
            if (c->loss != CHICLE_LOSS_SQUARED && (alpha0[r] < 0.0f || alpha0[r] > 1.0f))
                return fail(c, CHICLE_EINVAL, "chunk %d row %d: hinge alpha outside [0,1]", chunk_id, r);
        }
    }
    return CHICLE_OK;
}

static int finish_load(chicle_ctx *c, int32_t chunk_id, ChunkDev &ch, const float *y, const float *alpha0,
                       const std::vector<float> &q)
{
    const size_t nb = sizeof(RowState) * (size_t)ch.n_rows;
    RowState *sd = (RowState *)carve(c, nb);
    if (!sd) return fail(c, CHICLE_ENOMEM, "chunk store full");
    ch.st = sd;
    std::vector<RowState> st(ch.n_rows);
    for (int32_t r = 0; r < ch.n_rows; ++r) {
        st[r].y = y[r]; st[r].alpha = alpha0 ? alpha0[r] : 0.f; st[r].q = q[r];
        st[r].rw = c->loss == CHICLE_LOSS_HINGE ? 1.f : c->loss == CHICLE_LOSS_SQUARED ? y[r] : 0.f;   // residual at w = 0
    }
    HIP_TRY(c, hipMemcpyAsync(sd, st.data(), nb, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));   // host arrays are the caller's again on return
    c->chunks[chunk_id] = ch;
    c->loaded[chunk_id] = 1;
    c->n_loaded += 1;
    c->rows_loaded += ch.n_rows;
    c->entries_loaded += ch.nnz;
    return CHICLE_OK;
}

static int load_csr(chicle_ctx *c, int32_t chunk_id, int32_t n_rows, const int32_t *row_ptr,
                    const int32_t *col, const float *val, const float *y, const float *alpha0);

int chicle_load_chunk_csr(chicle_ctx *c, int32_t chunk_id, int32_t n_rows, const int32_t *row_ptr,
                          const int32_t *col, const float *val, const float *y, const float *alpha0)
{
    if (!c) return CHICLE_EINVAL;
    if (c->api_dense) return fail(c, CHICLE_EINVAL, "context holds dense chunks");
    return load_csr(c, chunk_id, n_rows, row_ptr, col, val, y, alpha0);
}

static int load_csr(chicle_ctx *c, int32_t chunk_id, int32_t n_rows, const int32_t *row_ptr,
                    const int32_t *col, const float *val, const float *y, const float *alpha0)
{
    if (!row_ptr || n_rows <= 0) return fail(c, CHICLE_EINVAL, "chunk %d: row_ptr NULL or no rows", chunk_id);
    if (row_ptr[0] != 0) return fail(c, CHICLE_EINVAL, "chunk %d: row_ptr[0] must be 0", chunk_id);
    for (int32_t r = 0; r < n_rows; ++r)
        if (row_ptr[r + 1] < row_ptr[r]) return fail(c, CHICLE_EINVAL, "chunk %d: row_ptr decreases at row %d", chunk_id, r);
    const int64_t nnz = row_ptr[n_rows];
    int rc = load_common(c, chunk_id, n_rows, nnz);
    if (rc) return rc;
    if (nnz > 0 && (!col || !val)) return fail(c, CHICLE_EINVAL, "chunk %d: col/val NULL", chunk_id);
    rc = check_state_arrays(c, chunk_id, n_rows, y, alpha0);
    if (rc) return rc;
    std::vector<float> q(n_rows);
    int32_t longest = 0;
    for (int32_t r = 0; r < n_rows; ++r) {
        double s = 0.0;
        for (int32_t p = row_ptr[r]; p < row_ptr[r + 1]; ++p) {
            if (col[p] < 0 || col[p] >= c->d) return fail(c, CHICLE_EINVAL, "chunk %d row %d: column %d outside [0,d)", chunk_id, r, col[p]);
            if (p > row_ptr[r] && col[p] <= col[p - 1]) return fail(c, CHICLE_EINVAL, "chunk %d row %d: columns not strictly ascending", chunk_id, r);
            if (!std::isfinite(val[p])) return fail(c, CHICLE_EINVAL, "chunk %d row %d: value not finite", chunk_id, r);
            s += (double)val[p] * (double)val[p];
        }
        q[r] = (float)s;
        longest = std::max(longest, row_ptr[r + 1] - row_ptr[r]);
    }
    ChunkDev ch{};
    ch.n_rows = n_rows; ch.nnz = nnz; ch.row_base = (int32_t)c->rows_loaded;
    int32_t *rp = (int32_t *)carve(c, sizeof(int32_t) * (size_t)(n_rows + 1));
    // a few entries of slack: kernels read short rows with fixed-width vector loads
    int32_t *cd = (int32_t *)carve(c, sizeof(int32_t) * (size_t)(nnz + ENTRY_SLACK));
    if (c->compact) {      // compact ids, filled at every assign; must lie where chunk_compact_ids() looks
        int32_t *ci = (int32_t *)carve(c, sizeof(int32_t) * (size_t)(nnz + ENTRY_SLACK));
        if (!ci || ci != cd + padded_entries(nnz)) return fail(c, CHICLE_ENOMEM, "chunk store full");
    }
    float *vd = (float *)carve(c, sizeof(float) * (size_t)(nnz + ENTRY_SLACK));
    if (!vd) return fail(c, CHICLE_ENOMEM, "chunk store full");
    ch.row_ptr = rp; ch.col = cd; ch.val = vd;
    HIP_TRY(c, hipMemcpyAsync(rp, row_ptr, sizeof(int32_t) * (size_t)(n_rows + 1), hipMemcpyHostToDevice, c->stream));
    if (nnz > 0) {
        HIP_TRY(c, hipMemcpyAsync(cd, col, sizeof(int32_t) * (size_t)nnz, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemcpyAsync(vd, val, sizeof(float) * (size_t)nnz, hipMemcpyHostToDevice, c->stream));
    }
    rc = finish_load(c, chunk_id, ch, y, alpha0, q);
    if (rc == CHICLE_OK) c->max_row_len = std::max(c->max_row_len, longest);
    return rc;
}

int chicle_load_chunk_dense(chicle_ctx *c, int32_t chunk_id, int32_t n_rows, const float *X,
                            const float *y, const float *alpha0)
{
    if (!c) return CHICLE_EINVAL;
    if (!c->api_dense) return fail(c, CHICLE_EINVAL, "context holds CSR chunks");
    if (!X || n_rows <= 0) return fail(c, CHICLE_EINVAL, "chunk %d: X NULL or no rows", chunk_id);
    const int64_t entries = (int64_t)n_rows * c->d;
    if (!c->dense) {                       // short dense rows: explicit column ids
        if (entries > INT32_MAX) return fail(c, CHICLE_EINVAL, "chunk %d too large", chunk_id);
        std::vector<int32_t> rp(n_rows + 1), cols((size_t)entries);
        for (int32_t r = 0; r <= n_rows; ++r) rp[r] = r * c->d;
        for (int64_t p = 0; p < entries; ++p) cols[p] = (int32_t)(p % c->d);
        return load_csr(c, chunk_id, n_rows, rp.data(), cols.data(), X, y, alpha0);
    }
    int rc = load_common(c, chunk_id, n_rows, entries);
    if (rc) return rc;
    rc = check_state_arrays(c, chunk_id, n_rows, y, alpha0);
    if (rc) return rc;
    std::vector<float> q(n_rows);
    for (int32_t r = 0; r < n_rows; ++r) {
        double s = 0.0;
        const float *x = X + (int64_t)r * c->d;
        for (int32_t j = 0; j < c->d; ++j) {
            if (!std::isfinite(x[j])) return fail(c, CHICLE_EINVAL, "chunk %d row %d: value not finite", chunk_id, r);
            s += (double)x[j] * (double)x[j];
        }
        q[r] = (float)s;
    }
    ChunkDev ch{};
    ch.n_rows = n_rows; ch.nnz = entries; ch.row_base = (int32_t)c->rows_loaded;
    float *xd = (float *)carve(c, sizeof(float) * (size_t)entries);
    if (!xd) return fail(c, CHICLE_ENOMEM, "chunk store full");
    ch.val = xd;
    HIP_TRY(c, hipMemcpyAsync(xd, X, sizeof(float) * (size_t)entries, hipMemcpyHostToDevice, c->stream));
    rc = finish_load(c, chunk_id, ch, y, alpha0, q);
    if (rc == CHICLE_OK) c->max_row_len = c->d;
    return rc;
}

int chicle_balance(const int64_t *chunk_load, int32_t n_chunks, int32_t K, const int32_t *speed_q,
                   int32_t *chunk_to_solver_out)
{
    if (!chunk_load || !chunk_to_solver_out || n_chunks < 0 || K <= 0) return CHICLE_EINVAL;
    for (int32_t i = 0; i < n_chunks; ++i)
        if (chunk_load[i] < 0) return CHICLE_EINVAL;
    if (speed_q)
        for (int32_t k = 0; k < K; ++k)
            if (speed_q[k] <= 0) return CHICLE_EINVAL;
    greedy_table(chunk_load, n_chunks, K, speed_q, chunk_to_solver_out);
    return CHICLE_OK;
}

int chicle_assign(chicle_ctx *c, int32_t K, const int32_t *chunk_to_solver)
{
    if (!c) return CHICLE_EINVAL;
    if (c->state == ST_EPOCH_DONE)
        return fail(c, CHICLE_ESTATE, "solvers own the chunks until their updates are aggregated");
    if (K <= 0 || K > c->max_solvers) return fail(c, CHICLE_EINVAL, "K=%d outside [1, max_solvers=%d]", K, c->max_solvers);
    if (!chunk_to_solver) return fail(c, CHICLE_EINVAL, "table is NULL");
    if (c->n_loaded != c->n_chunks) return fail(c, CHICLE_EINVAL, "%d of %d chunks loaded", c->n_loaded, c->n_chunks);
    if (c->rows_loaded != c->n_total) return fail(c, CHICLE_EINVAL, "chunks hold %lld rows, n_total is %lld", (long long)c->rows_loaded, (long long)c->n_total);
    { const int rc0 = drop_ahead(c); if (rc0) return rc0; }
    std::vector<int32_t> count(K, 0);
    for (int32_t i = 0; i < c->n_chunks; ++i) {
        if (chunk_to_solver[i] < 0 || chunk_to_solver[i] >= K)
            return fail(c, CHICLE_EINVAL, "chunk %d assigned to solver %d, K=%d", i, chunk_to_solver[i], K);
        count[chunk_to_solver[i]] += 1;
    }
    int max_list = 0;
    for (int32_t k = 0; k < K; ++k) max_list = std::max(max_list, count[k]);
    if (max_list > MAX_LIST_LDS) return fail(c, CHICLE_EINVAL, "a solver owns %d chunks, limit %d", max_list, MAX_LIST_LDS);

    std::vector<SolverDev> sol(K);
    std::vector<int32_t> list(c->n_chunks), prefix(c->n_chunks), chunk_first(c->n_chunks), list_base(c->n_chunks);
    int32_t pos = 0, tile = 0;
    int64_t perm_off = 0;
    for (int32_t k = 0; k < K; ++k) {
        sol[k].list_begin = pos; sol[k].n_chunks = count[k]; sol[k].perm_off = perm_off;
        int32_t rows = 0;
        for (int32_t i = 0; i < c->n_chunks; ++i) {        // ascending chunk id
            if (chunk_to_solver[i] != k) continue;
            list[pos] = i; prefix[pos] = rows; chunk_first[i] = rows; list_base[pos] = (int32_t)(perm_off + rows);
            rows += c->chunks[i].n_rows; ++pos;
        }
        sol[k].n_rows = rows;
        sol[k].tile_begin = tile;
        tile += (rows + BATCH - 1) / BATCH;
        perm_off += rows;
    }
    if (tile > c->max_tiles) return fail(c, CHICLE_ENOMEM, "tile scratch too small");
    std::vector<int32_t> tile_solver(std::max(tile, 1));
    for (int32_t k = 0; k < K; ++k)
        for (int32_t t = sol[k].tile_begin; t < sol[k].tile_begin + (sol[k].n_rows + BATCH - 1) / BATCH; ++t)
            tile_solver[t] = k;
    // work items of the gap kernels: blocks of 256/LPR rows inside a chunk
    const double avg = c->dense ? (double)c->d : (double)c->total_entries / (double)c->n_total;
    c->gap_lpr = choose_lpr(avg);
    const int rows_per_item = 256 / c->gap_lpr;
    std::vector<int32_t> items(c->n_chunks + 1, 0);
    for (int32_t i = 0; i < c->n_chunks; ++i)
        items[i + 1] = items[i] + (c->chunks[i].n_rows + rows_per_item - 1) / rows_per_item;

    // Stream order keeps earlier kernels ahead of these copies; wait before the host vectors go away.
    HIP_TRY(c, hipMemcpyAsync(c->chunks_dev, c->chunks.data(), sizeof(ChunkDev) * (size_t)c->n_chunks, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->solvers_dev, sol.data(), sizeof(SolverDev) * (size_t)K, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->solver_chunks_dev, list.data(), sizeof(int32_t) * (size_t)c->n_chunks, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->solver_prefix_dev, prefix.data(), sizeof(int32_t) * (size_t)c->n_chunks, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->item_prefix_dev, items.data(), sizeof(int32_t) * ((size_t)c->n_chunks + 1), hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->tile_solver_dev, tile_solver.data(), sizeof(int32_t) * (size_t)tile, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->chunk_first_dev, chunk_first.data(), sizeof(int32_t) * (size_t)c->n_chunks, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipMemcpyAsync(c->list_base_dev, list_base.data(), sizeof(int32_t) * (size_t)c->n_chunks, hipMemcpyHostToDevice, c->stream));
    hipLaunchKernelGGL(fill_row_chunk, dim3(c->n_chunks), dim3(256), 0, c->stream, c->chunks_dev,
                       c->solver_chunks_dev, c->list_base_dev, c->row_chunk_dev);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    if (c->state == ST_LOADING && !c->dense && c->max_row_len <= RENUMBER_MAX_ROW) {
        const int rc = renumber_columns(c);
        if (rc) return rc;
    }
    c->K = K;
    c->chunk_to_solver.assign(chunk_to_solver, chunk_to_solver + c->n_chunks);
    c->solvers = sol;
    c->max_list = max_list;
    c->n_tiles = tile;
    c->gap_items = items[c->n_chunks];
    c->state = ST_READY;
    c->cluster = 1;
    if (c->compact) {
        // Compact private vectors: which columns each solver's chunks contain, where each of them lives in
        // the solver's vector, and that index for every stored entry.  The columns the batched solver keeps
        // on chip are present in every solver's vector, at their own index.
        int64_t max_nnz = 1;
        for (const ChunkDev &ch : c->chunks) max_nnz = std::max(max_nnz, padded_entries(ch.nnz));
        const dim3 egrid(grid_for(max_nnz, 256, 1024), c->n_chunks);
        HIP_TRY(c, hipMemcpyAsync(c->chunk_owner_dev, chunk_to_solver, sizeof(int32_t) * (size_t)c->n_chunks, hipMemcpyHostToDevice, c->stream));
        HIP_TRY(c, hipMemsetAsync(c->bits_dev, 0, sizeof(unsigned) * (size_t)c->words * (size_t)K, c->stream));
        if (c->multi_dev) HIP_TRY(c, hipMemsetAsync(c->multi_dev, 0, sizeof(unsigned) * (size_t)c->words * (size_t)K, c->stream));
        hipLaunchKernelGGL(mark_columns, egrid, dim3(256), 0, c->stream, c->chunks_dev, c->chunk_owner_dev, c->bits_dev, c->words, c->multi_dev);
        const int forced = batched_eligible(c) ? batched_layout(c).n_hot : 0;
        if (forced > 0)
            hipLaunchKernelGGL(force_columns, dim3(K), dim3(256), 0, c->stream, c->bits_dev, c->words, forced);
        hipLaunchKernelGGL(prefix_columns, dim3(K), dim3(1024), 0, c->stream, c->bits_dev, c->pref_dev, c->words, c->count_dev);
        HIP_TRY(c, hipGetLastError());
        std::vector<int32_t> cnt(K);
        HIP_TRY(c, hipMemcpyAsync(cnt.data(), c->count_dev, sizeof(int32_t) * (size_t)K, hipMemcpyDeviceToHost, c->stream));
        HIP_TRY(c, hipStreamSynchronize(c->stream));
        std::vector<int64_t> off(K);
        int64_t used = 0;
        for (int32_t k = 0; k < K; ++k) { off[k] = used; used += ((int64_t)cnt[k] + 63) / 64 * 64; }
        if (used > c->u_capacity) return fail(c, CHICLE_ENOMEM, "private vectors need %lld floats, %lld reserved", (long long)used, (long long)c->u_capacity);
        c->u_used = used;
        HIP_TRY(c, hipMemcpyAsync(c->u_off_dev, off.data(), sizeof(int64_t) * (size_t)K, hipMemcpyHostToDevice, c->stream));
        hipLaunchKernelGGL(compact_indices, egrid, dim3(256), 0, c->stream, c->chunks_dev, c->chunk_owner_dev, c->bits_dev,
                           c->pref_dev, c->words, (const unsigned *)c->multi_dev);
        HIP_TRY(c, hipGetLastError());
        if (forced > 0) {
            int max_rows = 1;
            for (const ChunkDev &ch : c->chunks) max_rows = std::max(max_rows, ch.n_rows);
            HIP_TRY(c, hipMemsetAsync(c->count_dev, 0, sizeof(int32_t), c->stream));
            hipLaunchKernelGGL(max_entries_beyond, dim3(grid_for(max_rows, 256, 64), c->n_chunks), dim3(256), 0, c->stream,
                               c->chunks_dev, forced, c->count_dev);
            HIP_TRY(c, hipGetLastError());
            HIP_TRY(c, hipMemcpyAsync(&c->max_tail_entries, c->count_dev, sizeof(int32_t), hipMemcpyDeviceToHost, c->stream));
        }
        HIP_TRY(c, hipStreamSynchronize(c->stream));      // cnt, off and the caller's table go out of scope
    }
    if (c->long_rows) {
        // as many workgroups per solver as the chip has compute units for, each owning a range of columns
        const int k_pad = (K + L2_PARTITIONS - 1) / L2_PARTITIONS * L2_PARTITIONS;
        c->cluster = std::max(1, std::min(CLUSTER_MAX, c->cu_count / k_pad));
        if (c->cluster > 1 && c->split_built_for != c->cluster) {
            int max_rows = 1;
            for (const ChunkDev &ch : c->chunks) max_rows = std::max(max_rows, ch.n_rows);
            hipLaunchKernelGGL(row_split_offsets, dim3(grid_for(max_rows, 256, 64), c->n_chunks), dim3(256), 0, c->stream,
                               c->chunks_dev, (int)c->d, c->cluster, c->row_split_dev);
            HIP_TRY(c, hipGetLastError());
            c->split_built_for = c->cluster;
        }
        // the sliced gap row pass, where the shared vector is several slices long (built once: data only)
        if (c->gap_slices == 0) {
            const int shift = SLICE_BYTES_LOG2 - (c->loss == CHICLE_LOSS_HINGE ? 2 : 3);
            const int S = (int)(((int64_t)c->d + (1 << shift) - 1) >> shift);
            if (S >= SLICES_MIN) {
                int max_rows = 1;
                for (const ChunkDev &ch : c->chunks) max_rows = std::max(max_rows, ch.n_rows);
                hipLaunchKernelGGL(slice_offsets, dim3(grid_for(max_rows, 4, 256), c->n_chunks), dim3(256), 0, c->stream,
                                   c->chunks_dev, shift, S, c->n_total, c->slice_off_dev);
                HIP_TRY(c, hipGetLastError());
                c->gap_slices = S; c->gap_slice_shift = shift;
            }
        }
    }
    return clear_all_private(c);
}

int chicle_solver_rows(chicle_ctx *c, int64_t *rows_out)
{
    if (!c || !rows_out) return CHICLE_EINVAL;
    if (c->state == ST_LOADING) return fail(c, CHICLE_ESTATE, "no assignment yet");
    for (int32_t k = 0; k < c->K; ++k) rows_out[k] = c->solvers[k].n_rows;
    return CHICLE_OK;
}

int chicle_set_solver(chicle_ctx *c, int32_t kind)
{
    if (!c) return CHICLE_EINVAL;
    if (kind != CHICLE_SOLVER_AUTO && kind != CHICLE_SOLVER_ROWWISE && kind != CHICLE_SOLVER_BATCHED &&
        kind != CHICLE_SOLVER_ROWWISE_ONE_CU && kind != CHICLE_SOLVER_BATCHED_ONE_CU)
        return fail(c, CHICLE_EINVAL, "unknown solver kind %d", kind);
    c->cluster_allowed = kind != CHICLE_SOLVER_ROWWISE_ONE_CU;
    c->split_allowed = kind != CHICLE_SOLVER_BATCHED_ONE_CU;
    c->solver_kind = kind == CHICLE_SOLVER_ROWWISE_ONE_CU ? CHICLE_SOLVER_ROWWISE : kind == CHICLE_SOLVER_BATCHED_ONE_CU ? CHICLE_SOLVER_BATCHED : kind;
    return CHICLE_OK;
}

int chicle_set_l1(chicle_ctx *c, double l1)
{
    if (!c) return CHICLE_EINVAL;
    if (!(l1 >= 0.0) || !std::isfinite(l1)) return fail(c, CHICLE_EINVAL, "l1 must be finite and >= 0");
    if (c->state == ST_EPOCH_DONE) return fail(c, CHICLE_ESTATE, "aggregate first");
    c->l1 = l1;
    if (c->state != ST_LOADING) {      // the shared vector is the threshold's image of what the solvers have summed so far
        hipLaunchKernelGGL(mirror_from_double, dim3(grid_for(c->d, 256, 2048)), dim3(256), 0, c->stream, c->w64, c->w,
                           (int64_t)c->d, c->l1);
        HIP_TRY(c, hipGetLastError());
        c->zw_valid = false;
    }
    return CHICLE_OK;
}

int chicle_local_epoch(chicle_ctx *c, const int32_t *perm_device)
{
    if (!c) return CHICLE_EINVAL;
    if (!perm_device) return fail(c, CHICLE_EINVAL, "perm is NULL");
    return chicle_local_epoch_ahead(c, perm_device, nullptr);
}

int chicle_local_epoch_ahead(chicle_ctx *c, const int32_t *perm_device, const int32_t *perm_next_device)
{
    if (!c) return CHICLE_EINVAL;
    if (c->state != ST_READY) return fail(c, CHICLE_ESTATE, c->state == ST_LOADING ? "assign first" : "aggregate before the next local epoch");
    if (!perm_device && !c->ahead_valid)
        return fail(c, CHICLE_EINVAL, "perm is NULL and the previous pass announced no orders (or an assign dropped them)");
    // NULL: the orders the previous call announced, from the library's own copy of them
    const bool announced = perm_device == nullptr;
    const bool tiles_ready = announced && c->ahead_tiles;
    if (announced) perm_device = c->perm_ahead[1 - c->ahead_buf];
    c->ahead_valid = false;
    if (perm_next_device) {
        // Copied on the context's stream, so the caller's buffer is an ordinary stream-ordered input.
        HIP_TRY(c, hipMemcpyAsync(c->perm_ahead[c->ahead_buf], perm_next_device, sizeof(int32_t) * (size_t)c->n_total,
                                  hipMemcpyDeviceToDevice, c->stream));
        perm_next_device = c->perm_ahead[c->ahead_buf];
        c->ahead_buf = 1 - c->ahead_buf;
        c->ahead_valid = true;
    }
    bool batched = false, dense_blocked = false;
    if (c->solver_kind == CHICLE_SOLVER_BATCHED) {
        dense_blocked = dense_blocked_eligible(c);
        if (!dense_blocked && !batched_eligible(c))
            return fail(c, CHICLE_EINVAL, "batched solver needs sparse rows of at most %d entries and at most %d chunks per solver, or dense rows of at most %d columns", GRAM_MAX_ROW, BATCHED_MAX_LIST, DB_MAX_D);
        batched = !dense_blocked;
    } else if (c->solver_kind == CHICLE_SOLVER_AUTO) {
        batched = batched_eligible(c);
        dense_blocked = !batched && dense_blocked_eligible(c);
    }
    seg_begin(c, CHICLE_SEG_LOCAL_EPOCH);
    int rc = CHICLE_OK;
    if (!c->zw_valid) rc = run_row_pass(c, nullptr, c->gap_scratch);     // x_i . w for the current w
    if (rc == CHICLE_OK) {
        if (batched) {
            rc = c->loss == CHICLE_LOSS_HINGE ? launch_batched<0>(c, perm_device, tiles_ready, perm_next_device)
                 : c->loss == CHICLE_LOSS_SQUARED ? launch_batched<1>(c, perm_device, tiles_ready, perm_next_device)
                                                  : launch_batched<2>(c, perm_device, tiles_ready, perm_next_device);
        } else if (dense_blocked) {
            seg_begin(c, CHICLE_SEG_EPOCH_CHAIN);
            rc = c->loss == CHICLE_LOSS_HINGE ? launch_dense_blocked<0>(c, perm_device)
                 : c->loss == CHICLE_LOSS_SQUARED ? launch_dense_blocked<1>(c, perm_device)
                                                  : launch_dense_blocked<2>(c, perm_device);
            seg_end(c, CHICLE_SEG_EPOCH_CHAIN);
        } else {
            seg_begin(c, CHICLE_SEG_EPOCH_CHAIN);
            rc = c->loss == CHICLE_LOSS_HINGE ? launch_rowwise<0>(c, perm_device)
                 : c->loss == CHICLE_LOSS_SQUARED ? launch_rowwise<1>(c, perm_device)
                                                  : launch_rowwise<2>(c, perm_device);
            seg_end(c, CHICLE_SEG_EPOCH_CHAIN);
        }
    }
    seg_end(c, CHICLE_SEG_LOCAL_EPOCH);
    if (rc) return rc;
    c->state = ST_EPOCH_DONE;
    c->epoch_ran = true;
    return CHICLE_OK;
}

int chicle_local_epoch_host_perm(chicle_ctx *c, const int32_t *perm_host)
{
    if (!c) return CHICLE_EINVAL;
    if (c->state != ST_READY) return fail(c, CHICLE_ESTATE, c->state == ST_LOADING ? "assign first" : "aggregate before the next local epoch");
    if (!perm_host) return fail(c, CHICLE_EINVAL, "perm is NULL");
    HIP_TRY(c, hipMemcpyAsync(c->perm_stage, perm_host, sizeof(int32_t) * (size_t)c->n_total, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return chicle_local_epoch(c, c->perm_stage);
}

int chicle_aggregate(chicle_ctx *c)
{
    if (!c) return CHICLE_EINVAL;
    if (c->state != ST_EPOCH_DONE) return fail(c, CHICLE_ESTATE, "no local epoch pending");
    seg_begin(c, CHICLE_SEG_AGGREGATE);
    const int64_t d4 = c->ld_v / 4;
    if (c->compact) {
        // few words: the solvers are divided over slices too, so that the chip is filled
        const unsigned gx = (unsigned)((c->words + AGG_WORDS - 1) / AGG_WORDS);
        const unsigned gy = (unsigned)std::max(1, std::min(c->K, (int)(1024 / gx)));
        // thinly occupied vectors (under an eighth of the columns per solver on average): entries are picked
        // straight from memory
        if (c->u_used * 8 < (int64_t)c->K * (int64_t)c->d)
            hipLaunchKernelGGL(aggregate_compact_thin, dim3(gx, gy), dim3(AGG_WORDS), 0, c->stream, c->w64, c->w,
                               c->u, c->u_off_dev, c->bits_dev, c->pref_dev, c->words, (int64_t)c->d, c->K,
                               (float)(1.0 / (double)c->K), c->l1);
        else
        hipLaunchKernelGGL(aggregate_compact, dim3(gx, gy), dim3(AGG_WORDS), 0, c->stream, c->w64, c->w,
                           c->u, c->u_off_dev, c->bits_dev, c->pref_dev, c->words, (int64_t)c->d, c->K,
                           (float)(1.0 / (double)c->K), c->l1);
        if (gy > 1)
            hipLaunchKernelGGL(mirror_from_double, dim3(grid_for(c->d, 256, 2048)), dim3(256), 0, c->stream, c->w64, c->w, (int64_t)c->d, c->l1);
    } else
        hipLaunchKernelGGL(aggregate_broadcast, dim3(grid_for(d4, 256, 4096)), dim3(256), 0, c->stream, c->w64, c->w,
                           c->u, c->ld_v, d4, c->K, (float)(1.0 / (double)c->K), c->l1);
    seg_end(c, CHICLE_SEG_AGGREGATE);
    HIP_TRY(c, hipGetLastError());
    c->zw_valid = false;
    c->state = ST_READY;
    return CHICLE_OK;
}

static int gap_with(chicle_ctx *c, const GapScratch &gs, double *primal, double *dual, double *gap)
{
    if (c->state != ST_READY) return fail(c, CHICLE_ESTATE, "gap is defined on the aggregated state");
    seg_begin(c, CHICLE_SEG_GAP);
    int grid = 1;
    int rc = run_row_pass(c, &grid, gs);
    if (rc) { seg_end(c, CHICLE_SEG_GAP); return rc; }
    const int gw = grid_for(c->d, 256 * 8, WSQ_PARTS);
    hipLaunchKernelGGL(wsq_partial, dim3(gw), dim3(256), 0, c->stream, c->w64, (int64_t)c->d, c->l1, gs.wsq, gs.unused);
    hipLaunchKernelGGL(gap_finish, dim3(1), dim3(256), 0, c->stream, gs.loss, gs.conj, grid,
                       gs.wsq, gs.unused, gw, c->err_dev, c->gap_host_dev);
    seg_end(c, CHICLE_SEG_GAP);
    HIP_TRY(c, hipGetLastError());
    // the sums and the error flag arrive in pinned host memory with the end of the kernel: no copy to wait for
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    const double *h = c->gap_host;
    if (h[3] != 0.0) {
        const int flag = (int)h[3];
        HIP_TRY(c, hipMemsetAsync(c->err_dev, 0, sizeof(int), c->stream));
        if (flag & ERR_PERM_RANGE)
            return fail(c, CHICLE_EDEVICE, "a visiting-order entry was outside [0, rows of its solver)");
        if (flag & ERR_PARTNER_TIMEOUT)
            return fail(c, CHICLE_EDEVICE, "the workgroups that share a solver lost each other; the pass is invalid");
        return fail(c, CHICLE_EDEVICE, "kernel error flag %d", flag);
    }
    const double n = (double)c->n_total;
    const double P = c->lambda * (0.5 * h[2] + c->l1 * h[4]) + h[0] / n;     // (the regulariser's conjugate at the dual image is |w|^2 / 2)
    const double D = -0.5 * c->lambda * h[2] - h[1] / n;
    if (primal) *primal = P;
    if (dual) *dual = D;
    if (gap) *gap = P - D;
    return CHICLE_OK;
}

int chicle_gap(chicle_ctx *c, double *primal, double *dual, double *gap)
{
    if (!c) return CHICLE_EINVAL;
    return gap_with(c, c->gap_scratch, primal, dual, gap);
}

int chicle_gap_noalloc(chicle_ctx *c, double *primal, double *dual, double *gap)
{
    if (!c) return CHICLE_EINVAL;
    if (2 * (int64_t)c->n_chunks > GAP_PARTS)
        return fail(c, CHICLE_EINVAL, "%d chunks: the fixed scratch holds partial sums for at most %d", c->n_chunks, GAP_PARTS / 2);
    if (!c->static_scratch) return fail(c, CHICLE_EDEVICE, "the fixed scratch array was not found on this device");
    GapScratch gs;
    gs.loss = c->static_scratch;
    gs.conj = gs.loss + GAP_PARTS;
    gs.wsq = gs.conj + GAP_PARTS;
    gs.unused = gs.wsq + WSQ_PARTS;
    gs.parts = GAP_PARTS;
    return gap_with(c, gs, primal, dual, gap);
}

// d floats in internal order on the device -> caller's order on the host.
static int read_vector(chicle_ctx *c, const float *src_internal, float scale, float *host_out)
{
    hipLaunchKernelGGL(to_caller_order<float>, dim3(grid_for(c->d, 256, 4096)), dim3(256), 0, c->stream,
                       src_internal, c->renumbered ? c->col_of : (const int32_t *)nullptr, (int64_t)c->d,
                       scale, c->tmp_b);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipMemcpyAsync(host_out, c->tmp_b, sizeof(float) * (size_t)c->d, hipMemcpyDeviceToHost, c->stream));
    return check_deferred(c);
}

int chicle_get_w(chicle_ctx *c, float *w_out)
{
    if (!c || !w_out) return CHICLE_EINVAL;
    return read_vector(c, c->w, 1.0f, w_out);
}

int chicle_set_w(chicle_ctx *c, const float *w_in)
{
    if (!c || !w_in) return CHICLE_EINVAL;
    if (c->state == ST_EPOCH_DONE) return fail(c, CHICLE_ESTATE, "aggregate first");
    if (c->state == ST_LOADING) return fail(c, CHICLE_ESTATE, "assign first (the column order is fixed at the first assign)");
    if (c->l1 > 0.0) return fail(c, CHICLE_ESTATE, "with l1 > 0 the state is the dual image, which w does not determine");
    for (int32_t j = 0; j < c->d; ++j)
        if (!std::isfinite(w_in[j])) return fail(c, CHICLE_EINVAL, "w not finite at %d", j);
    HIP_TRY(c, hipMemcpyAsync(c->tmp_b, w_in, sizeof(float) * (size_t)c->d, hipMemcpyHostToDevice, c->stream));
    hipLaunchKernelGGL(from_caller_order, dim3(grid_for(c->d, 256, 4096)), dim3(256), 0, c->stream, c->tmp_b,
                       c->renumbered ? c->col_of : (const int32_t *)nullptr, (int64_t)c->d, c->w64, c->w);
    HIP_TRY(c, hipGetLastError());
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    c->zw_valid = false;
    return CHICLE_OK;
}

int chicle_get_delta_w(chicle_ctx *c, int32_t solver, float *dw_out)
{
    if (!c || !dw_out) return CHICLE_EINVAL;
    if (c->state != ST_EPOCH_DONE) return fail(c, CHICLE_ESTATE, "updates exist only between local_epoch and aggregate");
    if (solver < -1 || solver >= c->K) return fail(c, CHICLE_EINVAL, "solver %d, K=%d", solver, c->K);
    if (c->compact)
        hipLaunchKernelGGL(delta_w_out_compact, dim3(grid_for(c->d, 256, 4096)), dim3(256), 0, c->stream, c->u, c->u_off_dev,
                           c->bits_dev, c->pref_dev, c->words, (int64_t)c->d, c->K, solver, (float)(1.0 / (double)c->K), c->tmp_a);
    else
        hipLaunchKernelGGL(delta_w_out, dim3(grid_for(c->d, 256, 4096)), dim3(256), 0, c->stream, c->u, c->ld_v,
                           (int64_t)c->d, c->K, solver, (float)(1.0 / (double)c->K), c->tmp_a);
    HIP_TRY(c, hipGetLastError());
    return read_vector(c, c->tmp_a, 1.0f, dw_out);
}

int chicle_get_alpha(chicle_ctx *c, int32_t chunk_id, float *alpha_out)
{
    if (!c || !alpha_out) return CHICLE_EINVAL;
    if (chunk_id < 0 || chunk_id >= c->n_chunks || !c->loaded[chunk_id]) return fail(c, CHICLE_EINVAL, "chunk %d not loaded", chunk_id);
    const ChunkDev &ch = c->chunks[chunk_id];
    HIP_TRY(c, hipMemcpy2DAsync(alpha_out, sizeof(float), &ch.st->alpha, sizeof(RowState), sizeof(float),
                                (size_t)ch.n_rows, hipMemcpyDeviceToHost, c->stream));
    return check_deferred(c);
}

int chicle_set_alpha(chicle_ctx *c, int32_t chunk_id, const float *alpha_in)
{
    if (!c || !alpha_in) return CHICLE_EINVAL;
    if (c->state == ST_EPOCH_DONE) return fail(c, CHICLE_ESTATE, "solvers own the chunks until their updates are aggregated");
    if (chunk_id < 0 || chunk_id >= c->n_chunks || !c->loaded[chunk_id]) return fail(c, CHICLE_EINVAL, "chunk %d not loaded", chunk_id);
    const ChunkDev &ch = c->chunks[chunk_id];
    for (int32_t r = 0; r < ch.n_rows; ++r) {
        if (!std::isfinite(alpha_in[r])) return fail(c, CHICLE_EINVAL, "alpha not finite at row %d", r);
        if (c->loss != CHICLE_LOSS_SQUARED && (alpha_in[r] < 0.f || alpha_in[r] > 1.f))
            return fail(c, CHICLE_EINVAL, "hinge alpha outside [0,1] at row %d", r);
    }
    HIP_TRY(c, hipMemcpy2DAsync(&ch.st->alpha, sizeof(RowState), alpha_in, sizeof(float), sizeof(float),
                                (size_t)ch.n_rows, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, hipStreamSynchronize(c->stream));
    return CHICLE_OK;
}

int chicle_get_assignment(chicle_ctx *c, int32_t *chunk_to_solver_out, int32_t *K_out)
{
    if (!c) return CHICLE_EINVAL;
    if (c->state == ST_LOADING) return fail(c, CHICLE_ESTATE, "no assignment yet");
    if (chunk_to_solver_out) std::memcpy(chunk_to_solver_out, c->chunk_to_solver.data(), sizeof(int32_t) * (size_t)c->n_chunks);
    if (K_out) *K_out = c->K;
    return CHICLE_OK;
}

int chicle_solver_ms(chicle_ctx *c, float *ms_out)
{
    if (!c) return CHICLE_EINVAL;
    if (!ms_out) return fail(c, CHICLE_EINVAL, "output is NULL");
    if (!c->epoch_ran) return fail(c, CHICLE_ESTATE, "no local epoch has run");
    std::vector<long long> t(2 * (size_t)c->K);
    HIP_TRY(c, hipMemcpyAsync(t.data(), c->ticks_dev, sizeof(long long) * t.size(), hipMemcpyDeviceToHost, c->stream));
    const int rc = check_deferred(c);
    if (rc) return rc;
    for (int k = 0; k < c->K; ++k) ms_out[k] = (float)((double)(t[2 * k + 1] - t[2 * k]) / (double)c->wall_khz);
    return CHICLE_OK;
}

double chicle_projected_iteration_time(int32_t K_tasks, int32_t nodes, int32_t n_slow, double slow_factor,
                                       int32_t base_nodes)
{
    if (K_tasks < 0 || nodes <= 0 || n_slow < 0 || n_slow > nodes || base_nodes <= 0 ||
        (n_slow > 0 && !(slow_factor > 0.0)))
        return -1.0;
    return projected_iteration_time(K_tasks, nodes, n_slow, slow_factor, base_nodes);
}

int32_t chicle_next_solver_count(const double *gap, int32_t n_gaps, int32_t K, int32_t K_min,
                                 double stall_ratio, int32_t patience, int32_t since_change)
{
    if (!gap || n_gaps < 1 || K < 1 || K_min < 1 || !(stall_ratio > 0.0 && stall_ratio <= 1.0) ||
        patience < 1 || since_change < 0)
        return -1;
    return next_solver_count(gap, n_gaps, K, K_min, stall_ratio, patience, since_change);
}

static bool table_ok(const int32_t *t, int32_t n_chunks, int32_t K)
{
    if (!t || n_chunks < 0 || K <= 0) return false;
    for (int32_t i = 0; i < n_chunks; ++i)
        if (t[i] < 0 || t[i] >= K) return false;
    return true;
}

int chicle_scale_out(const int32_t *chunk_to_solver, int32_t n_chunks, int32_t K_old, int32_t K_new,
                     const uint32_t *draw, int32_t *chunk_to_solver_out)
{
    if (!table_ok(chunk_to_solver, n_chunks, K_old) || K_new <= K_old || !draw || !chunk_to_solver_out)
        return CHICLE_EINVAL;
    scale_out_table(n_chunks, chunk_to_solver, K_old, K_new, draw, chunk_to_solver_out);
    return CHICLE_OK;
}

int chicle_scale_in(const int32_t *chunk_to_solver, int32_t n_chunks, int32_t K_old, int32_t K_new,
                    int32_t *chunk_to_solver_out)
{
    if (!table_ok(chunk_to_solver, n_chunks, K_old) || K_new <= 0 || K_new >= K_old || !chunk_to_solver_out)
        return CHICLE_EINVAL;
    scale_in_table(n_chunks, chunk_to_solver, K_old, K_new, chunk_to_solver_out);
    return CHICLE_OK;
}

int chicle_rebalance(const int64_t *chunk_load, int32_t n_chunks, int32_t K, const double *unit_time,
                     int32_t n_iterations, int32_t max_moves, int32_t *chunk_to_solver, int32_t *n_moved_out)
{
    if (!chunk_load || !table_ok(chunk_to_solver, n_chunks, K) || !unit_time || n_iterations <= 0 || max_moves < 0)
        return CHICLE_EINVAL;
    for (int32_t i = 0; i < n_chunks; ++i)
        if (chunk_load[i] < 0) return CHICLE_EINVAL;
    for (int64_t i = 0; i < (int64_t)n_iterations * K; ++i)
        if (!(unit_time[i] > 0.0) || !std::isfinite(unit_time[i])) return CHICLE_EINVAL;
    const int moved = rebalance_table(chunk_load, n_chunks, K, unit_time, n_iterations, max_moves, chunk_to_solver);
    if (n_moved_out) *n_moved_out = moved;
    return CHICLE_OK;
}

int chicle_sync(chicle_ctx *c)
{
    if (!c) return CHICLE_EINVAL;
    return check_deferred(c);
}

int chicle_set_profiling(chicle_ctx *c, int32_t on)
{
    if (!c) return CHICLE_EINVAL;
    c->profiling = on != 0;
    return CHICLE_OK;
}

int chicle_last_kernel_ms(chicle_ctx *c, int32_t segment, float *ms_out)
{
    if (!c || !ms_out || segment < 0 || segment >= CHICLE_SEG_COUNT) return CHICLE_EINVAL;
    if (!c->seg[segment].recorded) return fail(c, CHICLE_ESTATE, "segment %d was not recorded (profiling off, or not run)", segment);
    HIP_TRY(c, hipEventSynchronize(c->seg[segment].stop));
    HIP_TRY(c, hipEventElapsedTime(ms_out, c->seg[segment].start, c->seg[segment].stop));
    return CHICLE_OK;
}

int chicle_debug_gram(chicle_ctx *c, const int32_t *perm_device, float *tiles_out, int64_t capacity_floats,
                      int32_t *n_tiles_out)
{
    if (!c || !perm_device) return CHICLE_EINVAL;
    if (c->state != ST_READY) return fail(c, CHICLE_ESTATE, "needs an assignment and no pending epoch");
    if (!batched_eligible(c)) return fail(c, CHICLE_EINVAL, "batched solver not available for this data");
    if (n_tiles_out) *n_tiles_out = c->n_tiles;
    int rc = drop_ahead(c);
    if (rc) return rc;
    rc = c->loss == CHICLE_LOSS_HINGE ? launch_gram<0>(c, perm_device, c->tile_buf, c->stream)
         : c->loss == CHICLE_LOSS_SQUARED ? launch_gram<1>(c, perm_device, c->tile_buf, c->stream)
                                          : launch_gram<2>(c, perm_device, c->tile_buf, c->stream);
    if (rc) return rc;
    if (tiles_out) {
        const int64_t want = (int64_t)c->n_tiles * TILE_FLOATS;
        if (capacity_floats < want) return fail(c, CHICLE_EINVAL, "need room for %lld floats", (long long)want);
        HIP_TRY(c, hipMemcpyAsync(tiles_out, c->tiles[c->tile_buf], sizeof(float) * (size_t)want, hipMemcpyDeviceToHost, c->stream));
    }
    return check_deferred(c);
}

const char *chicle_last_error(chicle_ctx *c) { return c ? c->err.c_str() : "null context"; }

void chicle_destroy(chicle_ctx *c)
{
    if (!c) return;
    if (c->side) (void)hipStreamSynchronize(c->side);
    (void)hipStreamSynchronize(c->stream);
    if (c->gap_host) (void)hipHostFree(c->gap_host);
    if (c->side) (void)hipStreamDestroy(c->side);
    if (c->ev_fork) (void)hipEventDestroy(c->ev_fork);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    for (int s = 0; s < CHICLE_SEG_COUNT; ++s) {
        if (c->seg[s].start) (void)hipEventDestroy(c->seg[s].start);
        if (c->seg[s].stop) (void)hipEventDestroy(c->seg[s].stop);
    }
    delete c;
}

}  // extern "C"
