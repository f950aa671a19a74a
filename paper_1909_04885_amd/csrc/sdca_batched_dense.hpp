// Local solver for dense rows of moderate width, blocks of 64 coordinate steps at a time; the same
// sequence of steps as the row-wise solver (paper Section 2.2: L = 1, H = all local samples).
//
// With the private vector and a block of rows in LDS nothing of a block touches HBM but the rows
// themselves, so the blocks are taken strictly one after the other (no lookahead, no cross term):
//   rows of the block -> LDS;  G = X_b X_b^T (a dense contraction: matrix cores, fp32 in / fp32 out);
//   t0 = unclipped steps against the private vector;  the recurrence of sdca_batched.hpp over the
//   strictly lower part of G (all three losses);  u += X_b^T coef;  alpha.
// fp32 matrix instructions give twice the multiply-adds per cycle of the vector units here (packed fp32
// vector operations are not used in this library).
#pragma once
#include <hip/hip_runtime.h>
#include "device_types.hpp"
#include "mem.hpp"
#include "sdca_batched.hpp"
#include "sdca_rowwise.hpp"

namespace chicle {

constexpr int DB_THREADS = 512;          // 8 wavefronts: 4 output tiles of 32 x 32, two halves of the columns
constexpr int DB_MAX_D = 320;            // widest row whose block fits LDS beside the rest
constexpr int DB_G_LD = BATCH + 1;

typedef float floatx16 __attribute__((ext_vector_type(16)));

// Dynamic LDS, in floats: X[64][ldx] | Gp[2][64][65] | T[64][65] | u[ldx] | per-row arrays (8 x 64) |
// then max_list chunk ids and max_list local-row prefixes (ints).  Rows are padded with zeros to a multiple
// of 16 columns (the Gram loop takes 8 columns per half and step); ldx = that + 4 keeps rows 16-byte
// aligned and spreads them over the banks.
__host__ __device__ inline int db_dpad(int d) { return (d + 15) & ~15; }
__host__ __device__ inline int db_ldx(int d) { return db_dpad(d) + 4; }
__host__ __device__ inline size_t db_lds_floats(int d)
{
    return (size_t)BATCH * db_ldx(d) + 3 * (size_t)BATCH * DB_G_LD + db_ldx(d) + 8 * BATCH;
}

template <int LOSS>
__global__ __launch_bounds__(DB_THREADS) void sdca_batched_dense(
    const ChunkDev *__restrict__ chunks, const SolverDev *__restrict__ solvers,
    const int32_t *__restrict__ solver_chunks, const int32_t *__restrict__ solver_prefix,
    const int32_t *__restrict__ perm, float *u_all, int64_t ld_v, int d, int max_list, RoundScalars sc,
    int *err)
{
    extern __shared__ __align__(16) float db_smem[];
    const int ldx = db_ldx(d), d2 = db_dpad(d);
    float *X = db_smem;                                  // [64][ldx], columns d .. d2-1 zero
    float *Gp = X + BATCH * ldx;                         // [2][64][65] partial Gram matrices
    float *T = Gp + 2 * BATCH * DB_G_LD;                 // [j][i], zero for j >= i
    float *u = T + BATCH * DB_G_LD;                      // private vector (difference to w)
    float *r_y = u + ldx, *r_a = r_y + BATCH, *r_q = r_a + BATCH, *r_rw = r_q + BATCH;
    float *r_t0 = r_rw + BATCH, *r_lo = r_t0 + BATCH, *r_hi = r_lo + BATCH, *r_dl = r_hi + BATCH;
    int *l_chunk = reinterpret_cast<int *>(r_dl + BATCH);
    int *l_prefix = l_chunk + max_list;
    __shared__ const float *r_x[BATCH];                  // row data (nullptr: row skipped)
    __shared__ RowState *r_st[BATCH];

    const SolverDev S = solvers[blockIdx.x];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    stamp_solver(sc, 0);
    float *u_glb = u_all + (int64_t)blockIdx.x * ld_v;
    for (int i = tid; i < S.n_chunks; i += DB_THREADS) {
        l_chunk[i] = solver_chunks[S.list_begin + i];
        l_prefix[i] = solver_prefix[S.list_begin + i];
    }
    for (int i = tid; i < ldx; i += DB_THREADS) u[i] = i < d ? u_glb[i] : 0.f;
    for (int i = tid; i < BATCH * DB_G_LD; i += DB_THREADS) T[i] = 0.f;
    __syncthreads();
    const int32_t *pk = perm + S.perm_off;
    const int nb = (S.n_rows + BATCH - 1) / BATCH;

    for (int b = 0; b < nb; ++b) {
        // 1. the block's rows: state and address
        if (tid < BATCH) {
            const int t = b * BATCH + tid;
            const float *xp = nullptr;
            RowState *sp = nullptr;
            float4_v st = {0.f, 0.f, 0.f, 0.f};
            if (t < S.n_rows) {
                const int lr = pk[t];
                if ((unsigned)lr >= (unsigned)S.n_rows) {
                    atomicOr(err, ERR_PERM_RANGE);
                } else {
                    const int j = find_chunk(l_prefix, S.n_chunks, lr);
                    const ChunkDev &ch = chunks[l_chunk[j]];
                    const int r = lr - l_prefix[j];
                    st = gld_state(ch.st + r);
                    if (st.z != 0.f) { xp = ch.val + (int64_t)r * d; sp = ch.st + r; }
                }
            }
            r_x[tid] = xp; r_st[tid] = sp;
            r_y[tid] = st.x; r_a[tid] = st.y; r_q[tid] = st.z; r_rw[tid] = st.w;
        }
        __syncthreads();
        // 2. rows into LDS (a skipped row is all zero: it then takes part in nothing)
        for (int idx = tid; idx < BATCH * d2; idx += DB_THREADS) {
            const int row = idx / d2, k = idx - row * d2;
            const float *xp = r_x[row];
            X[row * ldx + k] = (xp != nullptr && k < d) ? xp[k] : 0.f;
        }
        __syncthreads();
        // 3. G = X X^T on the matrix cores: wavefront -> (tile row, tile column, half of the columns).
        //    A 32 x 2 by 2 x 32 product takes A[l % 32][l / 32] and B[l / 32][l % 32] from lane l.  Any
        //    pairing of the columns works for a dot product: per 8 columns a lane reads 4 consecutive ones
        //    (the lower four for lanes 0..31, the upper four for the others) with one 16-byte LDS read per
        //    operand and feeds them to 4 products.
        {
            const int ti = wv & 1, tj = (wv >> 1) & 1, kh = wv >> 2;
            const float *pa = X + (32 * ti + (lane & 31)) * ldx + 4 * (lane >> 5);
            const float *pb = X + (32 * tj + (lane & 31)) * ldx + 4 * (lane >> 5);
            floatx16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
            const int k0 = kh * (d2 / 2), k1 = k0 + d2 / 2;          // d2 / 2 is a multiple of 8
            for (int k = k0; k < k1; k += 8) {
                const float4 a = *reinterpret_cast<const float4 *>(pa + k);
                const float4 bq = *reinterpret_cast<const float4 *>(pb + k);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, bq.x, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, bq.y, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, bq.z, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, bq.w, acc, 0, 0, 0);
            }
            // result layout: register r of lane l is row 8 (r / 4) + 4 (l / 32) + r % 4, column l % 32
            float *g = Gp + kh * BATCH * DB_G_LD;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                g[(32 * ti + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * DB_G_LD + 32 * tj + (lane & 31)] = acc[r];
        }
        //    and the dot products with the private vector: 8 lanes per row
        {
            const int row = tid >> 3, sub = tid & 7;
            float part = 0.f;
            for (int k = sub; k < d; k += 8) part += X[row * ldx + k] * u[k];
            part += __shfl_xor(part, 1, 64); part += __shfl_xor(part, 2, 64); part += __shfl_xor(part, 4, 64);
            if (sub == 0) {
                float t0 = 0.f, lo = 0.f, hi = 0.f;
                const float q = r_q[row];
                if (q != 0.f) {
                    if (LOSS == 0) {
                        t0 = (sc.c / q) * (r_rw[row] - r_y[row] * part);
                        lo = -r_a[row]; hi = 1.f - r_a[row];
                    } else if (LOSS == 1) {
                        t0 = (sc.c / (sc.c + q)) * (r_rw[row] - r_a[row] - part);
                    } else {
                        // logistic: t0 = m = -y z, hi = r = q / c, lo = the root of the row's equation for this m
                        t0 = r_rw[row] - r_y[row] * part;
                        hi = q * sc.inv_c;
                        logistic_step(t0, hi, r_a[row], t0 + hi * (r_a[row] - 0.5f), &lo);
                    }
                }
                r_t0[row] = t0; r_lo[row] = lo; r_hi[row] = hi;
            }
        }
        __syncthreads();
        // 4. T[j][i] for j < i (the rest stays zero)
        for (int idx = tid; idx < BATCH * BATCH; idx += DB_THREADS) {
            const int j = idx >> 6, i = idx & 63;
            float v = 0.f;
            const float q = r_q[i];
            if (j < i && q != 0.f) {
                const float g = Gp[j * DB_G_LD + i] + Gp[BATCH * DB_G_LD + j * DB_G_LD + i];
                v = LOSS == 0 ? -r_y[i] * r_y[j] * g / q : LOSS == 1 ? -g / (sc.c + q) : -r_y[i] * r_y[j] * g * sc.inv_c;
            }
            T[j * DB_G_LD + i] = v;
        }
        __syncthreads();
        // 5. the recurrence (one wavefront)
        if (wv == 0) {
            float t = r_t0[lane], dl;
            const float lo = r_lo[lane], hi = r_hi[lane];
            if (LOSS == 2) {
                // lane i keeps m_i; step j is solved by the whole wavefront from a bracket between the root
                // found for the row's m at the start of the block and that root moved by the change of m
                const float a = r_a[lane];
                dl = 0.f;
#pragma unroll 2
                for (int j = 0; j < BATCH; ++j) {
                    const float mj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(t), j));
                    const float aj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(a), j));
                    const float rj = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(hi), j));
                    const float dm = mj - r_t0[j];
                    float dj = 0.f;
                    if (rj > 0.f) dj = logistic_step_wave(mj, rj, aj, r_lo[j] + fminf(dm, 0.f), fabsf(dm), lane);
                    t = fmaf(dj, T[j * DB_G_LD + lane], t);
                    dl = lane == j ? dj : dl;
                }
            } else {
#pragma unroll 8
                for (int j = 0; j < BATCH; ++j) {
                    const float dj = clamp_step<LOSS>(t, lo, hi);
                    const float s = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(dj), j));
                    t = fmaf(s, T[j * DB_G_LD + lane], t);
                }
                dl = clamp_step<LOSS>(t, lo, hi);
            }
            if (r_st[lane] != nullptr) {
                float an = r_a[lane] + dl;
                if (LOSS != 1) an = fminf(fmaxf(an, 0.f), 1.f);
                gst(&r_st[lane]->alpha, an);
            }
            // coefficient of the row in the update of the private vector, in place of its delta
            r_dl[lane] = dl * (LOSS == 1 ? 1.f : r_y[lane]) * sc.inv_c;
        }
        __syncthreads();
        // 6. u += X^T coef, one column per thread
        for (int k = tid; k < d; k += DB_THREADS) {
            float acc = u[k];
#pragma unroll 8
            for (int row = 0; row < BATCH; ++row) acc = fmaf(r_dl[row], X[row * ldx + k], acc);
            u[k] = acc;
        }
        __syncthreads();
    }
    for (int i = tid; i < d; i += DB_THREADS) u_glb[i] = u[i];
    stamp_solver(sc, 1);
}

}  // namespace chicle
