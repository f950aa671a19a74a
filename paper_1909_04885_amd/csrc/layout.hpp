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
