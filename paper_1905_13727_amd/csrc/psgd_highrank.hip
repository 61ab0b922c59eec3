// Matrix-core kernels: ranks above 8 (up to 64) and bf16 gradients / bf16 output.
//
// At rank 16..64 the three products of a PowerSGD step (arXiv 1905.13727, Algorithm 1: P = M Q,
// Q = M^T P_hat, P_hat Q^T) are dense enough for the matrix cores: 2 r flops per element and
// sweep, still under the HBM balance point, but far too many for the vector ALUs next to the
// loads.  All three use v_mfma_f32_16x16x4_f32 (fp32 in, fp32 accumulate: M = g + e is an fp32
// quantity even when g arrives as bf16, and the parity bar is 1e-5).  The rank axis is padded to
// NT tiles of 16.  Every matrix must have a row length that is a multiple of 4.
//
//   k_hr_right<NT, BF>   M = g + e (g fp32 or bf16) written over e; P_w = M Q           (Alg. 2, Alg. 1)
//   k_hr_gram / k_hr_chol / k_hr_apply   mean P, Gram matrix in fp64, Cholesky factor, P_hat = P R^-1:
//                        the orthonormal factor Gram-Schmidt yields (remark "Orthogonalization is a
//                        linear operation"), for panels of any height                    (Alg. 1)
//   k_hr_left<NT>        Q_w = M^T P_hat, one partial per wavefront's row strip          (Alg. 1)
//   k_hr_decomp<NT, BF>  Delta' = P_hat Q^T, e' = M - Delta', Delta' stored fp32 or bf16  (Alg. 1, Alg. 2)
//   k_hr_vec<BFI, BFO>   mean of the vector-shaped tensors                                (Alg. 1 line 1)
//
// Lane roles of the 16x16x4 instruction (lane l, li = l % 16, kb = l / 16): A[li][kb], B[kb][li],
// D[4 kb + v][li] in register v.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <type_traits>

#include "psgd_device.h"
#include "psgd_internal.h"

namespace psgd {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned short bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float((unsigned)h << 16); }

// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <bool BF>
__device__ __forceinline__ v4f load_grad4(const void* base, int64_t idx) {
    if constexpr (BF) {
        typedef unsigned short us4 __attribute__((ext_vector_type(4)));
        const us4 h = __builtin_nontemporal_load(reinterpret_cast<const us4*>(static_cast<const bf16_t*>(base) + idx));
        return v4f{bf16_to_f32(h.x), bf16_to_f32(h.y), bf16_to_f32(h.z), bf16_to_f32(h.w)};
    } else {
        return __builtin_nontemporal_load(reinterpret_cast<const v4f*>(static_cast<const float*>(base) + idx));
    }
}

template <bool BF>
__device__ __forceinline__ void store_out4(void* base, int64_t idx, v4f v) {
    if constexpr (BF) {
        typedef unsigned short us4 __attribute__((ext_vector_type(4)));
        us4 h;
        h.x = f32_to_bf16(v.x); h.y = f32_to_bf16(v.y); h.z = f32_to_bf16(v.z); h.w = f32_to_bf16(v.w);
        *reinterpret_cast<us4*>(static_cast<bf16_t*>(base) + idx) = h;
    } else {
        *reinterpret_cast<v4f*>(static_cast<float*>(base) + idx) = v;
    }
}

// ---- k_hr_right: P_w = M Q ------------------------------------------------------------------------------
// A wavefront owns a strip of rows (16 at a time) and walks the whole row in chunks of 64 columns;
// per chunk it fetches the Q block of the chunk (B operands) and, for each 16-row step of its strip,
// loads g and e, stores M and issues 16 NT instructions.  The accumulators of all steps stay in
// registers across the chunks, so nothing is split over columns: one partial per worker.//
// Above rank 8 the products are accumulated in fp64 (v_mfma_f64_16x16x4_f64, the fp32 operands widen
// exactly): with r columns P spans singular directions whose weights differ by (sigma_1 / sigma_r)^2,
// and the orthogonalisation divides every column by its own norm, so an error that is small against the
// largest column is not small against the smallest.  fp32 accumulation leaves P_hat 2-3e-5 off at
// r = 16 on a 1/k spectrum; fp64 accumulation (one rounding to fp32 at the end) keeps it at 1e-6.
// The fp64 output tile is D[4 v + kb][li] (fp32: D[4 kb + v][li]).
constexpr int kHrRightRows = 256;    // rows per workgroup

typedef double v4d __attribute__((ext_vector_type(4)));

template <int NT, bool BF, bool F64>
__global__ __launch_bounds__(kBlock) void k_hr_right(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                     const void* __restrict__ grad, float* __restrict__ err,
                                                     const float* __restrict__ q, float* __restrict__ ws,
                                                     int64_t gstride, int64_t estride) {
    // register budget: accumulators for STEPS 16-row steps and the B operands of U 16-column groups
    constexpr int STEPS = (F64 && NT == 4) ? 1 : ((F64 && NT == 2) || NT == 4 ? 2 : 4);
    constexpr int U = (F64 && NT >= 2) ? 2 : 4;
    constexpr int ROWS_W = kHrRightRows / kWavesPerBlock;   // 64 rows per wavefront, in passes of 16 STEPS
    typedef typename std::conditional<F64, v4d, v4f>::type acc_t;
    typedef typename std::conditional<F64, double, float>::type b_t;
    const Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int w = blockIdx.y;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int li = lane & 15, kb = lane >> 4;
    const int ri = d.r, m = d.m, n = d.n;
    const int64_t goff = (int64_t)w * gstride + d.off;
    float* e = err + (int64_t)w * estride + d.off;
    const int row_end = min(n, t.row0 + t.nrows);

    for (int pass = 0; pass < ROWS_W / (16 * STEPS); ++pass) {
        const int row_w = t.row0 + wave * ROWS_W + pass * 16 * STEPS;
        if (row_w >= row_end) break;
        acc_t acc[STEPS][NT];
#pragma unroll
        for (int s = 0; s < STEPS; ++s)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[s][nt] = acc_t{0, 0, 0, 0};

        for (int c0 = 0; c0 < m; c0 += 16 * U) {
            // B operands of the chunk: Q[c0 + 16 u + 4 kb + c][16 nt + li]
            b_t bq[U][4][NT];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int col = c0 + 16 * u + 4 * kb + c;
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        const int j = 16 * nt + li;
                        bq[u][c][nt] = (col < m && j < ri) ? (b_t)q[d.q_off + (int64_t)col * ri + j] : (b_t)0;
                    }
                }
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const int row = row_w + 16 * s + li;
                const bool row_ok = row < row_end;
                v4f gv[U], ev[U];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int col = c0 + 16 * u + 4 * kb;
                    gv[u] = v4f{0.f, 0.f, 0.f, 0.f};
                    ev[u] = v4f{0.f, 0.f, 0.f, 0.f};
                    if (row_ok && col < m) {
                        gv[u] = load_grad4<BF>(grad, goff + (int64_t)row * m + col);
                        ev[u] = *reinterpret_cast<const v4f*>(e + (int64_t)row * m + col);
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int col = c0 + 16 * u + 4 * kb;
                    const v4f mv = gv[u] + ev[u];
                    if (row_ok && col < m) *reinterpret_cast<v4f*>(e + (int64_t)row * m + col) = mv;
#pragma unroll
                    for (int c = 0; c < 4; ++c)
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt) {
                            if constexpr (F64)
                                acc[s][nt] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)mv[c], bq[u][c][nt], acc[s][nt], 0, 0, 0);
                            else
                                acc[s][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(mv[c], bq[u][c][nt], acc[s][nt], 0, 0, 0);
                        }
                }
            }
        }
#pragma unroll
        for (int s = 0; s < STEPS; ++s)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int j = 16 * nt + li;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int row = row_w + 16 * s + (F64 ? 4 * v + kb : 4 * kb + v);
                    if (j < ri && row < row_end)
                        ws[d.ppart_off + ((int64_t)w * n + row) * ri + j] = (float)acc[s][nt][v];
                }
            }
    }
}

// ---- orthonormal factor by Cholesky-QR, any panel height, rank up to 64 ---------------------------------
constexpr int kHrMaxRank = PSGD_MAX_RANK;
constexpr int kHrGramRows = 128;   // panel rows staged in LDS at a time by the Gram kernel

// Row block of kGramRows rows: mean P (sum over workers, * 1/W) -> P buffer; Gram matrix of the block in
// fp64 -> gram[block][r*r].  Thread t owns entries (a, b) with a * r + b = t, t + 256, ...
__global__ __launch_bounds__(kBlock) void k_hr_gram(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                    const float* __restrict__ ws, float* __restrict__ p,
                                                    double* __restrict__ gram, int workers) {
    __shared__ float rows[kHrGramRows][kHrMaxRank + 1];
    const Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int r = d.r, tid = threadIdx.x;
    const int64_t nr = (int64_t)d.n * r;
    const float inv_w = 1.0f / (float)workers;
    const int nent = r * r;
    constexpr int EPT = (kHrMaxRank * kHrMaxRank + kBlock - 1) / kBlock;   // entries per thread
    double g[EPT];
#pragma unroll
    for (int x = 0; x < EPT; ++x) g[x] = 0.0;
    for (int r0 = t.row0; r0 < t.row0 + t.nrows; r0 += kHrGramRows) {
        const int nrow = min(kHrGramRows, t.row0 + t.nrows - r0);
        __syncthreads();
        for (int idx = tid; idx < nrow * r; idx += kBlock) {
            const int i = idx / r, k = idx - i * r;
            const int64_t at = (int64_t)(r0 + i) * r + k;
            float s = 0.f;
            for (int w = 0; w < workers; ++w) s += ws[d.ppart_off + (int64_t)w * nr + at];
            s *= inv_w;
            rows[i][k] = s;
            p[d.p_off + at] = s;
        }
        __syncthreads();
#pragma unroll
        for (int x = 0; x < EPT; ++x) {
            const int ent = tid + x * kBlock;
            if (ent < nent) {
                const int a = ent / r, b = ent - a * r;
                double acc = g[x];
                for (int i = 0; i < nrow; ++i) acc += (double)rows[i][a] * (double)rows[i][b];
                g[x] = acc;
            }
        }
    }
#pragma unroll
    for (int x = 0; x < EPT; ++x) {
        const int ent = tid + x * kBlock;
        if (ent < nent) gram[d.gram_off + (int64_t)t.part * nent + ent] = g[x];
    }
}

// One workgroup per matrix: Gram = sum of the blocks' matrices (block order), Cholesky factor R (upper,
// G = R^T R) in fp64, stored with the reciprocals of its diagonal (0 for a column whose pivot is <= 1e-30:
// that column of P_hat is zero); what is stored at chol[chol_off ..] is R^-1 (r x r, upper triangular).
__global__ __launch_bounds__(kBlock) void k_hr_chol(const MatDesc* __restrict__ mats, const double* __restrict__ gram,
                                                    double* __restrict__ chol) {
    __shared__ double G[kHrMaxRank][kHrMaxRank + 1];
    __shared__ double rinv[kHrMaxRank];
    const MatDesc d = mats[blockIdx.x];
    const int r = d.r, tid = threadIdx.x, nent = r * r;
    for (int ent = tid; ent < nent; ent += kBlock) {
        const double* src = gram + d.gram_off + ent;
        double v = 0.0;
        int b = 0;
        for (; b + 8 <= d.n_gblock; b += 8) {
            double x[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) x[u] = src[(int64_t)(b + u) * nent];
#pragma unroll
            for (int u = 0; u < 8; ++u) v += x[u];
        }
        for (; b < d.n_gblock; ++b) v += src[(int64_t)b * nent];
        G[ent / r][ent % r] = v;
    }
    __syncthreads();
    // right-looking Cholesky, row j of R at a time; G's upper triangle is overwritten by R
    for (int j = 0; j < r; ++j) {
        if (tid == 0) {
            const double piv = G[j][j];
            if (piv <= 1e-30) {
                rinv[j] = 0.0;
                G[j][j] = 0.0;
            } else {
                const double rjj = sqrt(piv);
                G[j][j] = rjj;
                rinv[j] = 1.0 / rjj;
            }
        }
        __syncthreads();
        const double ri_j = rinv[j];
        for (int c = j + 1 + tid; c < r; c += kBlock) G[j][c] = G[j][c] * ri_j;   // 0 for a dead column
        __syncthreads();
        // trailing update: G[a][b] -= R[j][a] R[j][b] for j < a <= b
        const int rem = r - j - 1;
        for (int idx = tid; idx < rem * rem; idx += kBlock) {
            const int a = j + 1 + idx / rem, b = j + 1 + idx % rem;
            if (b >= a) G[a][b] -= G[j][a] * G[j][b];
        }
        __syncthreads();
    }
    // inverse of R by back substitution, one column per thread: R x = e_c.  A dead column (reciprocal 0)
    // gets x = 0 and, its row of R being zero, takes no part in the others.
    __shared__ double X[kHrMaxRank][kHrMaxRank + 1];
    if (tid < r) {
        const int c = tid;
        for (int i = r - 1; i > c; --i) X[i][c] = 0.0;
        X[c][c] = rinv[c];
        for (int i = c - 1; i >= 0; --i) {
            double v = 0.0;
            for (int k = i + 1; k <= c; ++k) v += G[i][k] * X[k][c];
            X[i][c] = -v * rinv[i];
        }
    }
    __syncthreads();
    double* dst = chol + d.chol_off;
    for (int ent = tid; ent < nent; ent += kBlock) dst[ent] = X[ent / r][ent % r];
}

// P_hat = P R^-1 (R^-1 upper triangular, fp64), row by row, in place in the P buffer.
template <int RMAX>
__global__ __launch_bounds__(kBlock) void k_hr_apply(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                     const double* __restrict__ chol, float* __restrict__ p) {
    __shared__ double X[RMAX][RMAX + 1];
    const Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int r = d.r, tid = threadIdx.x, nent = r * r;
    const double* src = chol + d.chol_off;
    for (int ent = tid; ent < RMAX * RMAX; ent += kBlock) {
        const int a = ent / RMAX, b = ent % RMAX;
        X[a][b] = (a < r && b < r) ? src[a * r + b] : 0.0;
    }
    (void)nent;
    __syncthreads();
    for (int i = t.row0 + tid; i < t.row0 + t.nrows; i += kBlock) {
        float* row = p + d.p_off + (int64_t)i * r;
        float pb[RMAX];
#pragma unroll
        for (int k = 0; k < RMAX; ++k) pb[k] = k < r ? row[k] : 0.f;
        for (int j = 0; j < r; ++j) {
            double acc = 0.0;
#pragma unroll
            for (int k = 0; k < RMAX; ++k) acc += (double)pb[k] * X[k][j];   // X[k][j] = 0 for k > j
            row[j] = (float)acc;
        }
    }
}

// ---- k_hr_left: Q_w = M^T P_hat ----------------------------------------------------------------------------
// Lane (kb, li) loads 16 bytes at row 4 t + kb, columns c0 + 64 g + 4 li .. + 3; component c of that load
// is the A operand of the instruction that accumulates the columns c0 + 64 g + 4 i + c (i = 0..15).
// B operand: P_hat[row 4 t + kb][16 nt + li].  A wavefront walks its strip of rows 16 at a time (four
// such loads per column group in flight) and writes one partial Q per strip.
constexpr int kHrLeftGroups = 2;   // 64-column groups per wavefront (128 columns)

template <int NT>
__global__ __launch_bounds__(kBlock) void k_hr_left(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                    const float* __restrict__ err, const float* __restrict__ p,
                                                    float* __restrict__ ws, int64_t estride) {
    constexpr int NG = kHrLeftGroups;
    const Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int w = blockIdx.y;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int li = lane & 15, kb = lane >> 4;
    const int ri = d.r, m = d.m, n = d.n;
    const float* e = err + (int64_t)w * estride + d.off;
    const int c0 = t.vec0;                       // first column of the workgroup's chunk
    // rows of this wavefront
    int rb, rn;
    wave_rows(t.nrows, wave, &rb, &rn);
    const int r_begin = t.row0 + rb, r_end = r_begin + rn;

    v4f acc[NG][4][NT];
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[g][c][nt] = v4f{0.f, 0.f, 0.f, 0.f};

    for (int r0 = r_begin; r0 < r_end; r0 += 16) {
        v4f a[4][NG];
        float b[4][NT];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int row = r0 + 4 * s + kb;
            const bool ok = row < r_end;
            const int row_c = ok ? row : r_end - 1;     // a real row: its product is switched off through B
#pragma unroll
            for (int g = 0; g < NG; ++g) {
                const int col = c0 + 64 * g + 4 * li;
                a[s][g] = v4f{0.f, 0.f, 0.f, 0.f};
                if (col < m && col < c0 + t.nvec) a[s][g] = *reinterpret_cast<const v4f*>(e + (int64_t)row_c * m + col);
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int j = 16 * nt + li;
                b[s][nt] = (ok && j < ri) ? p[d.p_off + (int64_t)row * ri + j] : 0.f;
            }
        }
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[g][c][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s][g][c], b[s][nt], acc[g][c][nt], 0, 0, 0);
    }
    // acc[g][c][nt][v] = Q[c0 + 64 g + 4 (4 kb + v) + c][16 nt + li] for this strip
    const int part = (w * d.n_rblock) + t.part * kWavesPerBlock + wave;
    float* dst = ws + d.qpart_off + (int64_t)part * m * ri;
#pragma unroll
    for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int j = 16 * nt + li;
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int col = c0 + 64 * g + 4 * (4 * kb + v) + c;
                    if (j < ri && col < m && col < c0 + t.nvec) dst[(int64_t)col * ri + j] = acc[g][c][nt][v];
                }
            }
}

// ---- k_hr_decomp: Delta' = P_hat Q^T, e' = M - Delta' -------------------------------------------------------
// The product is formed transposed, (Q block 16 x K) (P_hat^T K x 16): A[li][kb] = Q[col0 + li][4 kk + kb],
// B[kb][li] = P_hat[row0 + li][4 kk + kb], so that lane (kb, li) ends up with Delta'[row0 + li][col0 + 4 kb + v],
// v = 0..3: four consecutive columns of one row, the same 16 bytes it loads of M and stores of e' and Delta'.
constexpr int kHrDecompBlocks = 8;   // 16-column blocks per wavefront (128 columns)

template <int NT, bool BF>
__global__ __launch_bounds__(kBlock) void k_hr_decomp(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                      float* __restrict__ err, const float* __restrict__ p,
                                                      const float* __restrict__ q, void* __restrict__ out,
                                                      int64_t estride) {
    constexpr int KK = 4 * NT;   // instructions per 16 x 16 block (K = 16 NT in steps of 4)
    constexpr int CB = kHrDecompBlocks;
    const Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int w = blockIdx.y;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int li = lane & 15, kb = lane >> 4;
    const int ri = d.r, m = d.m;
    float* e = err + (int64_t)w * estride + d.off;
    const int c0 = t.vec0;
    const int c_end = min(m, c0 + t.nvec);

    float aq[CB][KK];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) {
        const int col = c0 + 16 * cb + li;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const int k = 4 * kk + kb;
            aq[cb][kk] = (col < c_end && k < ri) ? q[d.q_off + (int64_t)col * ri + k] : 0.f;
        }
    }
    int rb, rn;
    wave_rows(t.nrows, wave, &rb, &rn);
    const int r_begin = t.row0 + rb, r_end = r_begin + rn;
    for (int r0 = r_begin; r0 < r_end; r0 += 16) {
        const int row = r0 + li;
        const bool row_ok = row < r_end;
        float bp[KK];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            const int k = 4 * kk + kb;
            bp[kk] = (row_ok && k < ri) ? p[d.p_off + (int64_t)row * ri + k] : 0.f;
        }
        v4f mv[CB];
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            const int col = c0 + 16 * cb + 4 * kb;
            mv[cb] = v4f{0.f, 0.f, 0.f, 0.f};
            if (row_ok && col < c_end) mv[cb] = *reinterpret_cast<const v4f*>(e + (int64_t)row * m + col);
        }
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(aq[cb][kk], bp[kk], acc, 0, 0, 0);
            const int col = c0 + 16 * cb + 4 * kb;
            if (row_ok && col < c_end) {
                *reinterpret_cast<v4f*>(e + (int64_t)row * m + col) = mv[cb] - acc;
                if (w == 0) store_out4<BF>(out, d.off + (int64_t)row * m + col, acc);
            }
        }
    }
}

template <bool BFI, bool BFO>
__global__ __launch_bounds__(kBlock) void k_hr_vec(const void* __restrict__ grad, void* __restrict__ out, int workers,
                                                   int64_t gstride, int64_t n_mat_elems, int64_t n_vec) {
    const float inv_w = 1.0f / (float)workers;
    for (int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x; idx < n_vec; idx += (int64_t)gridDim.x * kBlock) {
        float s = 0.f;
        for (int w = 0; w < workers; ++w) {
            const int64_t at = (int64_t)w * gstride + n_mat_elems + idx;
            if constexpr (BFI) s += bf16_to_f32(static_cast<const bf16_t*>(grad)[at]);
            else s += static_cast<const float*>(grad)[at];
        }
        s *= inv_w;
        if constexpr (BFO) static_cast<bf16_t*>(out)[n_mat_elems + idx] = f32_to_bf16(s);
        else static_cast<float*>(out)[n_mat_elems + idx] = s;
    }
}

// ---- host side ------------------------------------------------------------------------------------------------

static psgd_status hr_fail(psgd_plan* plan, const char* what) {
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) return PSGD_OK;
    plan->last_error = std::string(what) + ": " + hipGetErrorString(e);
    return PSGD_EHIP;
}

#define HR_CHECK(what)                          \
    do {                                        \
        psgd_status st_ = hr_fail(plan, what);  \
        if (st_ != PSGD_OK) return st_;         \
    } while (0)

#define HR_MARK(i)                                                                               \
    do {                                                                                         \
        if (plan->profiling && hipEventRecord(static_cast<hipEvent_t>(plan->events[i]), s) != hipSuccess) { \
            plan->last_error = "hipEventRecord";                                                 \
            return PSGD_EHIP;                                                                    \
        }                                                                                        \
    } while (0)

template <int NT>
static void hr_launch_right(psgd_plan* plan, const void* grad, float* err, const float* q, float* ws, hipStream_t s) {
    dim3 grid((unsigned)plan->hr_tiles1.size(), (unsigned)plan->workers);
    const bool bf = plan->grad_dtype == PSGD_BF16, f64 = plan->rank > kValuMaxRank;
#define HR_RIGHT(BFV, F64V)                                                                                       \
    hipLaunchKernelGGL((k_hr_right<NT, BFV, F64V>), grid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.hr_tiles1, \
                       grad, err, q, ws, plan->sizes.grad_stride, plan->sizes.err_stride)
    if (bf && f64) HR_RIGHT(true, true);
    else if (bf) HR_RIGHT(true, false);
    else if (f64) HR_RIGHT(false, true);
    else HR_RIGHT(false, false);
#undef HR_RIGHT
}

template <int NT>
static void hr_launch_decomp(psgd_plan* plan, float* err, const float* p, const float* q, void* out, hipStream_t s) {
    dim3 grid((unsigned)plan->hr_tiles4.size(), (unsigned)plan->workers);
    if (plan->out_dtype == PSGD_BF16)
        hipLaunchKernelGGL((k_hr_decomp<NT, true>), grid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.hr_tiles4, err, p, q,
                           out, plan->sizes.err_stride);
    else
        hipLaunchKernelGGL((k_hr_decomp<NT, false>), grid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.hr_tiles4, err, p, q,
                           out, plan->sizes.err_stride);
}

static double* hr_doubles(psgd_plan* plan, void* workspace) {
    const size_t float_bytes = (size_t)(plan->ws_ppart_floats + plan->ws_qpart_floats) * sizeof(float);
    return reinterpret_cast<double*>(static_cast<char*>(workspace) + (float_bytes + 255) / 256 * 256);
}

psgd_status hr_compress(psgd_plan* plan, const void* grad, float* err, float* q, float* p, void* workspace,
                        void* stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* ws = static_cast<float*>(workspace);
    if (plan->mats.empty()) return PSGD_OK;
    const int nt = plan->hr_nt;
    HR_MARK(0);
    if (nt == 1) hr_launch_right<1>(plan, grad, err, q, ws, s);
    else if (nt == 2) hr_launch_right<2>(plan, grad, err, q, ws, s);
    else hr_launch_right<4>(plan, grad, err, q, ws, s);
    HR_CHECK("launch k_hr_right");
    HR_MARK(1);
    double* gram = hr_doubles(plan, workspace);
    double* chol = gram + plan->ws_gram_doubles;
    hipLaunchKernelGGL(k_hr_gram, dim3((unsigned)plan->tiles_gram.size()), dim3(kBlock), 0, s, plan->dev.mats,
                       plan->dev.tiles_gram, ws, p, gram, plan->workers);
    HR_CHECK("launch k_hr_gram");
    hipLaunchKernelGGL(k_hr_chol, dim3((unsigned)plan->mats.size()), dim3(kBlock), 0, s, plan->dev.mats, gram, chol);
    HR_CHECK("launch k_hr_chol");
    if (plan->rank <= 16)
        hipLaunchKernelGGL((k_hr_apply<16>), dim3((unsigned)plan->tiles_gram.size()), dim3(kBlock), 0, s, plan->dev.mats,
                           plan->dev.tiles_gram, chol, p);
    else if (plan->rank <= 32)
        hipLaunchKernelGGL((k_hr_apply<32>), dim3((unsigned)plan->tiles_gram.size()), dim3(kBlock), 0, s, plan->dev.mats,
                           plan->dev.tiles_gram, chol, p);
    else
        hipLaunchKernelGGL((k_hr_apply<64>), dim3((unsigned)plan->tiles_gram.size()), dim3(kBlock), 0, s, plan->dev.mats,
                           plan->dev.tiles_gram, chol, p);
    HR_CHECK("launch k_hr_apply");
    HR_MARK(2);
    {
        dim3 grid((unsigned)plan->hr_tiles3.size(), (unsigned)plan->workers);
        if (nt == 1)
            hipLaunchKernelGGL((k_hr_left<1>), grid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.hr_tiles3, err, p, ws,
                               plan->sizes.err_stride);
        else if (nt == 2)
            hipLaunchKernelGGL((k_hr_left<2>), grid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.hr_tiles3, err, p, ws,
                               plan->sizes.err_stride);
        else
            hipLaunchKernelGGL((k_hr_left<4>), grid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.hr_tiles3, err, p, ws,
                               plan->sizes.err_stride);
    }
    HR_CHECK("launch k_hr_left");
    HR_MARK(3);
    psgd_status st = launch_q_reduce(plan, ws, q, stream);
    if (st != PSGD_OK) return st;
    HR_MARK(4);
    return PSGD_OK;
}

psgd_status hr_decompress(psgd_plan* plan, const float* p, const float* q, float* err, const void* grad, void* out,
                          void* stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int nt = plan->hr_nt;
    HR_MARK(5);
    if (!plan->hr_tiles4.empty()) {
        if (nt == 1) hr_launch_decomp<1>(plan, err, p, q, out, s);
        else if (nt == 2) hr_launch_decomp<2>(plan, err, p, q, out, s);
        else hr_launch_decomp<4>(plan, err, p, q, out, s);
        HR_CHECK("launch k_hr_decomp");
    }
    const int64_t L = plan->sizes.n_vec_elems;
    if (L > 0) {
        const unsigned blocks = (unsigned)std::min<int64_t>(1024, (L + kBlock - 1) / kBlock);
        const bool bi = plan->grad_dtype == PSGD_BF16, bo = plan->out_dtype == PSGD_BF16;
        if (bi && bo)
            hipLaunchKernelGGL((k_hr_vec<true, true>), dim3(blocks), dim3(kBlock), 0, s, grad, out, plan->workers,
                               plan->sizes.grad_stride, plan->sizes.n_mat_elems, L);
        else if (bi)
            hipLaunchKernelGGL((k_hr_vec<true, false>), dim3(blocks), dim3(kBlock), 0, s, grad, out, plan->workers,
                               plan->sizes.grad_stride, plan->sizes.n_mat_elems, L);
        else if (bo)
            hipLaunchKernelGGL((k_hr_vec<false, true>), dim3(blocks), dim3(kBlock), 0, s, grad, out, plan->workers,
                               plan->sizes.grad_stride, plan->sizes.n_mat_elems, L);
        else
            hipLaunchKernelGGL((k_hr_vec<false, false>), dim3(blocks), dim3(kBlock), 0, s, grad, out, plan->workers,
                               plan->sizes.grad_stride, plan->sizes.n_mat_elems, L);
        HR_CHECK("launch k_hr_vec");
    }
    HR_MARK(6);
    return finish_profiled_step(plan);
}

}  // namespace psgd
