// Chunk-store layout kernels: column ids are stored as popularity ranks.
//
// When all chunks are in HBM the columns are renumbered once by how often they occur (most frequent
// column = id 0) and every row is re-sorted by the new ids.  Frequent columns then have small ids, so
// a solver can keep the frequently touched head of its private vector in LDS by a plain range test
// and the rows' frequent entries come first.  The shared vector and the private vectors live in the
// renumbered space; the read/write entry points translate to and from the caller's column ids.
#pragma once
#include <hip/hip_runtime.h>
#include "device_types.hpp"

namespace chicle {

// count[col] += 1 for every stored entry.  One workgroup per chunk.
__global__ __launch_bounds__(256) void count_columns(const ChunkDev *__restrict__ chunks, int *count)
{
    const ChunkDev &ch = chunks[blockIdx.x];
    for (int64_t p = threadIdx.x; p < ch.nnz; p += 256) atomicAdd(&count[ch.col[p]], 1);
}

// col <- rank_of[col] and insertion sort of each row by the new ids (values move with their ids).
// One thread per row; rows are short where this is used.  Grid: (blocks over rows, chunk).
__global__ __launch_bounds__(256) void renumber_rows(const ChunkDev *__restrict__ chunks,
                                                     const int32_t *__restrict__ rank_of)
{
    const ChunkDev &ch = chunks[blockIdx.y];
    int32_t *col = const_cast<int32_t *>(ch.col);
    float *val = const_cast<float *>(ch.val);
    for (int r = blockIdx.x * 256 + threadIdx.x; r < ch.n_rows; r += gridDim.x * 256) {
        const int b = ch.row_ptr[r], e = ch.row_ptr[r + 1];
        for (int p = b; p < e; ++p) {
            const int c = rank_of[col[p]];
            const float v = val[p];
            int s = p;
            while (s > b && col[s - 1] > c) {
                col[s] = col[s - 1];
                val[s] = val[s - 1];
                --s;
            }
            col[s] = c;
            val[s] = v;
        }
    }
}

// ---- compact private vectors (sparse rows: a solver touches a small part of the columns) ----
// Per solver a bitmap of the columns its chunks contain and, per 32-column word, the number of set bits
// before it: column c of solver k lives at index pref[k][c >> 5] + popcount(bits[k][c >> 5] below bit c & 31)
// of that solver's compact vector.

// bits[owner[chunk]][c >> 5] |= 1 << (c & 31) for every entry.  Grid: (blocks over entries, chunk).
// multi (may be null): the same layout, a bit is set when a second entry of the solver's chunks holds the column
// (the columns inside a row are distinct, so that is another row).
__global__ __launch_bounds__(256) void mark_columns(const ChunkDev *__restrict__ chunks, const int32_t *__restrict__ owner,
                                                    unsigned *bits, int64_t words, unsigned *multi)
{
    const ChunkDev &ch = chunks[blockIdx.y];
    unsigned *mine = bits + (int64_t)owner[blockIdx.y] * words;
    unsigned *more = multi ? multi + (int64_t)owner[blockIdx.y] * words : nullptr;
    for (int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x; p < ch.nnz; p += (int64_t)gridDim.x * 256) {
        const int c = ch.col[p];
        const unsigned bit = 1u << (c & 31);
        const unsigned old = atomicOr(mine + (c >> 5), bit);
        if (more && (old & bit)) atomicOr(more + (c >> 5), bit);
    }
}

// Columns [0, n) are present in every solver's vector: sets their bits.  One workgroup per solver.
__global__ __launch_bounds__(256) void force_columns(unsigned *bits, int64_t words, int n)
{
    unsigned *mine = bits + (int64_t)blockIdx.x * words;
    for (int j = threadIdx.x; j * 32 < n; j += 256) {
        const int left = n - j * 32;
        mine[j] |= left >= 32 ? 0xffffffffu : ((1u << left) - 1u);
    }
}

// pref[k][j] = number of set bits in bits[k][0 .. j); count[k] = all of them.  One workgroup of 1024 per solver.
__global__ __launch_bounds__(1024) void prefix_columns(const unsigned *__restrict__ bits, int32_t *pref, int64_t words,
                                                       int32_t *count)
{
    __shared__ int wave_sum[16];
    __shared__ int carry;
    const unsigned *b = bits + (int64_t)blockIdx.x * words;
    int32_t *p = pref + (int64_t)blockIdx.x * words;
    if (threadIdx.x == 0) carry = 0;
    __syncthreads();
    for (int64_t base = 0; base < words; base += 1024) {
        const int64_t j = base + threadIdx.x;
        const int v = j < words ? __popc(b[j]) : 0;
        int incl = v;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int y = __shfl_up(incl, o, 64);
            if ((threadIdx.x & 63) >= o) incl += y;
        }
        if ((threadIdx.x & 63) == 63) wave_sum[threadIdx.x >> 6] = incl;
        __syncthreads();
        int off = carry;
        for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) off += wave_sum[w];
        if (j < words) p[j] = off + incl - v;
        __syncthreads();
        if (threadIdx.x == 1023) carry = off + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) count[blockIdx.x] = carry;
}

// The compact index of every entry, written behind the chunk's column ids.  Grid: (blocks over entries, chunk).
// multi (may be null): see mark_columns; an entry whose column no other row of the solver holds gets the sign
// bit (UNIQUE_COLUMN in mem.hpp).
__global__ __launch_bounds__(256) void compact_indices(const ChunkDev *__restrict__ chunks, const int32_t *__restrict__ owner,
                                                       const unsigned *__restrict__ bits, const int32_t *__restrict__ pref,
                                                       int64_t words, const unsigned *__restrict__ multi)
{
    const ChunkDev &ch = chunks[blockIdx.y];
    const int64_t k = owner[blockIdx.y];
    const unsigned *b = bits + k * words;
    const int32_t *pf = pref + k * words;
    int32_t *out = const_cast<int32_t *>(chunk_compact_ids(ch));
    const int64_t n = padded_entries(ch.nnz);
    for (int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x; p < n; p += (int64_t)gridDim.x * 256) {
        int idx = 0;                                   // the slack behind the last row points at index 0
        if (p < ch.nnz) {
            const int c = ch.col[p];
            idx = pf[c >> 5] + __popc(b[c >> 5] & ((1u << (c & 31)) - 1u));
            if (multi && !(multi[k * words + (c >> 5)] & (1u << (c & 31)))) idx |= (int)0x80000000;
        }
        out[p] = idx;
    }
}

// *out = the largest number of entries any row has at compact indices >= n (the columns the batched solver
// does not keep on chip).  Grid: (blocks over rows, chunk), one thread per row; *out starts at 0.
__global__ __launch_bounds__(256) void max_entries_beyond(const ChunkDev *__restrict__ chunks, int n, int *out)
{
    const ChunkDev &ch = chunks[blockIdx.y];
    const int32_t *cid = chunk_compact_ids(ch);
    int most = 0;
    for (int r = blockIdx.x * 256 + threadIdx.x; r < ch.n_rows; r += gridDim.x * 256) {
        int cnt = 0;
        for (int p = ch.row_ptr[r]; p < ch.row_ptr[r + 1]; ++p) cnt += cid[p] >= n;
        most = max(most, cnt);
    }
    if (most > 0) atomicMax(out, most);
}

// out[col_of[r]] = in[r] * scale (internal order -> caller's column ids).
template <typename T>
__global__ __launch_bounds__(256) void to_caller_order(const T *__restrict__ in,
                                                       const int32_t *__restrict__ col_of, int64_t d,
                                                       float scale, float *out)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < d; r += stride)
        out[col_of ? col_of[r] : r] = (float)in[r] * scale;
}

// out64[r] = out32[r] = in[col_of[r]] (caller's column ids -> internal order).
__global__ __launch_bounds__(256) void from_caller_order(const float *__restrict__ in,
                                                         const int32_t *__restrict__ col_of, int64_t d,
                                                         double *out64, float *out32)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; r < d; r += stride) {
        const float x = in[col_of ? col_of[r] : r];
        out64[r] = (double)x;
        out32[r] = x;
    }
}

}  // namespace chicle
