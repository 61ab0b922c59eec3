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
//   k_hr_left<NT, ..>    Q_w = M^T P_hat, one partial per wavefront's row strip          (Alg. 1)
//   k_hr_decomp<NT, OM>  Delta' = P_hat Q^T, e' = M - Delta', Delta' stored fp32 or bf16, or folded into the
//                        momentum / parameter update                                     (Alg. 1, Alg. 2)
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

// four gradient elements, read once (non-temporal): as they come (8 or 16 bytes, kept that way while in flight), and widened
template <bool BF>
struct grad4 { typedef typename std::conditional<BF, v2u, v4u>::type raw; };
template <bool BF>
__device__ __forceinline__ typename grad4<BF>::raw buf_load_grad4_raw(buf_rsrc r, unsigned off) {
    if constexpr (BF) return __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, 2);
    else return __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 2);
}
__device__ __forceinline__ v4f grad4_widen(v2u x) {
    return v4f{__uint_as_float(x.x << 16), __uint_as_float(x.x & 0xffff0000u), __uint_as_float(x.y << 16),
               __uint_as_float(x.y & 0xffff0000u)};
}
__device__ __forceinline__ v4f grad4_widen(v4u x) {
    return v4f{__uint_as_float(x.x), __uint_as_float(x.y), __uint_as_float(x.z), __uint_as_float(x.w)};
}

// ---- k_hr_right: P_w = M Q ------------------------------------------------------------------------------
// A workgroup owns a block of rows and walks the whole row in chunks of 128 or 64 columns.  Global memory is
// touched in row-contiguous pieces only (a load instruction covers 2 rows x 128 or 4 rows x 64 columns); M = g + e goes back over e in the same shape and into a 16 x chunk tile in
// LDS private to the wavefront, from which the lanes fetch their A operands (row li, columns
// 16 u + 4 kb ..+3).  The Q rows of the chunk (B operands) are staged in LDS once per workgroup, double
// buffered, one barrier per chunk.  g and e of the next 16-row step are in flight while the current
// one is multiplied.  The accumulators of the wavefront's 16 STEPS rows stay in registers across the
// chunks.  Rows longer than the plan's column limit are split over workgroups, one partial P per worker
// and column range, summed (in index order) by k_hr_gram.
//
// The products are accumulated in fp64 (v_mfma_f64_16x16x4_f64, the fp32 operands widen
// exactly): with r columns P spans singular directions whose weights differ by (sigma_1 / sigma_r)^2,
// and the orthogonalisation divides every column by its own norm, so an error that is small against the
// largest column is not small against the smallest.  fp32 accumulation leaves P_hat 2-3e-5 off at
// r = 16 on a 1/k spectrum; fp64 accumulation (one rounding to fp32 at the end) keeps it at 1e-6.
// The fp64 output tile is D[4 v + kb][li] (fp32: D[4 kb + v][li]).
// columns per chunk: 128 (a load instruction covers 2 rows x 128 columns: 512-byte runs of e, 256-byte runs of bf16 g;
// a plain pass over g, e, M with that shape moves 5.9 TB/s here, with 4 rows x 64 columns 5.0) where the staged Q
// chunks leave room for two workgroups per compute unit, 64 at three and four rank tiles
constexpr int hr_chunk(int nt) { return nt <= 2 ? 128 : 64; }

typedef double v4d __attribute__((ext_vector_type(4)));

template <int NT, bool BF, bool F64, bool STREAM>
__global__ __launch_bounds__(kBlock, 2) void k_hr_right(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                        const void* __restrict__ grad, float* __restrict__ err,
                                                        const float* __restrict__ q, float* __restrict__ ws,
                                                        int64_t gstride, int64_t estride, int add) {
    constexpr int STEPS = 2;                          // 16-row steps per wavefront and pass: 128 rows per workgroup and pass
    constexpr int RP = 16 * NT;                       // padded rank
    constexpr int BST = RP + 4;                       // floats per LDS row of the staged Q chunk
    constexpr int CH = hr_chunk(NT);                  // columns per chunk
    constexpr int AST = CH + 4;                       // floats per LDS row of an A tile (b128 reads of 16 rows spread over the banks)
    constexpr int LPR = CH / 4;                       // loader lanes per row
    constexpr int RPI = kWave / LPR;                  // rows per load instruction
    constexpr int NI = 16 / RPI;                      // load instructions per 16-row step
    constexpr int BPT = CH * RP / kBlock;             // staged Q elements per thread
    typedef typename std::conditional<F64, v4d, v4f>::type acc_t;
    typedef typename std::conditional<F64, double, float>::type b_t;
    __shared__ float Bs[2][CH][BST];
    __shared__ __attribute__((aligned(16))) float As[kWavesPerBlock][16][AST];

    const Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int w = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, kb = lane >> 4;      // matrix-core roles
    const int lr = lane / LPR, lc = 4 * (lane % LPR);   // loader roles: row within the rows of an instruction, first column
    const int ri = d.r, m = d.m, n = d.n;
    constexpr int GS = BF ? 2 : 4;                  // bytes per gradient element
    const char* gmat = static_cast<const char*>(grad) + ((int64_t)w * gstride + d.off) * GS;
    float* emat = err + (int64_t)w * estride + d.off;
    const int row_end = min(n, t.row0 + t.nrows);
    const int col0 = t.vec0;   // first of this workgroup's columns (a multiple of 64); they end with the row or at a multiple of 64
    const int col_end = min(m, col0 + t.nvec);
    const int nchunks = (t.nvec + CH - 1) / CH;
    const int part = w * d.n_cchunk + t.part;
    float (*at)[AST] = As[wave];

    // Q rows of a chunk: element idx of the CH x RP block is Q[c0 + idx / RP][idx % RP]; rows past the
    // matrix fall outside the buffer (zero), padded rank columns get the out-of-range offset themselves
    const buf_rsrc qres = make_rsrc(q + d.q_off, (int64_t)m * ri * 4);
    // (thread tid stages elements tid + k * 256: the same rank column tid % RP in rows 256 / RP apart)
    const unsigned qoff0 = tid % RP < ri ? (unsigned)((tid / RP) * ri + tid % RP) * 4u : kOutOfRange;
    const unsigned qstep = (unsigned)((kBlock / RP) * ri * 4);
    // an unwanted request (past the last chunk) goes through a descriptor with an empty range: nothing is fetched,
    // and no branch surrounds the request, so the waits count exactly what is outstanding
    const buf_rsrc nores = make_rsrc(q + d.q_off, 0);
    auto stage_load = [&](int c0, bool wanted, float (&br)[BPT]) {
        const buf_rsrc res = wanted ? qres : nores;
#pragma unroll
        for (int k = 0; k < BPT; ++k)
            br[k] = buf_load_f32(res, qoff0 == kOutOfRange ? kOutOfRange : qoff0 + (unsigned)k * qstep + (unsigned)(c0 * ri * 4));
    };
    auto stage_store = [&](int buf, const float (&br)[BPT]) {
#pragma unroll
        for (int k = 0; k < BPT; ++k) {
            const int idx = tid + k * kBlock;
            Bs[buf][idx / RP][idx % RP] = br[k];
        }
    };

    for (int row_p = t.row0; row_p < row_end; row_p += kWavesPerBlock * 16 * STEPS) {
        const int row_w = row_p + wave * 16 * STEPS;
        acc_t acc[STEPS][NT];
#pragma unroll
        for (int s = 0; s < STEPS; ++s)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[s][nt] = acc_t{0, 0, 0, 0};

        // Buffer descriptors whose range ends with the last valid row of the strip: the lanes' offsets
        // (4 i + lr) m + lc are the same for every step and chunk, only the scalar offset moves, and rows
        // past the end read zeros / drop their stores.  Columns past the row end (last chunk) are sent
        // out of range explicitly.
        const int rows_w = max(0, min(16 * STEPS, row_end - row_w));
        const int64_t base_w = (int64_t)min(row_w, row_end) * m;
        // add == 0 (one more iteration on the M already stored): the gradient descriptor is empty (zeros are read),
        // and so is the one M would be stored through
        const buf_rsrc eres = make_rsrc(emat + base_w, (int64_t)rows_w * m * 4);
        const buf_rsrc esto = make_rsrc(emat + base_w, add ? (int64_t)rows_w * m * 4 : 0);
        const buf_rsrc gres = make_rsrc(gmat + base_w * GS, add ? (int64_t)rows_w * m * GS : 0);
        unsigned voff[NI];
#pragma unroll
        for (int i = 0; i < NI; ++i) voff[i] = (unsigned)(RPI * i + lr) * (unsigned)m + (unsigned)lc;
        // a step s starts 16 s rows further down: added to the lane offset (the range check looks at the lane
        // offset only)
        typedef typename grad4<BF>::raw graw_t;
        auto data_load = [&](int c0, int s, bool wanted, graw_t (&gv)[NI], v4f (&ev)[NI]) {
            const bool col_ok = c0 + lc < col_end;   // the workgroup's columns may end inside a chunk
            const buf_rsrc gr = wanted ? gres : nores, er = wanted ? eres : nores;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const unsigned el = voff[i] + (unsigned)(16 * s * m + c0);
                gv[i] = buf_load_grad4_raw<BF>(gr, col_ok ? el * GS : kOutOfRange);
                ev[i] = buf_load_v4f_policy<STREAM ? 2 : 0>(er, col_ok ? el * 4u : kOutOfRange);
            }
        };

        float br[BPT];
        __syncthreads();   // the previous pass has finished with Bs
        stage_load(col0, true, br);
        stage_store(0, br);
        graw_t gn[NI];
        v4f en[NI];
        data_load(col0, 0, true, gn, en);
        for (int ch = 0; ch < nchunks; ++ch) {
            const int c0 = col0 + ch * CH;
            const int buf = ch & 1;
            __syncthreads();   // Bs[buf] is complete; Bs[buf ^ 1] is no longer read
            // requests past the last chunk are sent out of range (nothing is fetched): no branch around a request,
            // so the waits below count exactly what is outstanding
            const bool more = ch + 1 < nchunks;
            stage_load(c0 + CH, more, br);
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                {
                    const bool col_ok = c0 + lc < col_end;
#pragma unroll
                    for (int i = 0; i < NI; ++i) {
                        const v4f mv = grad4_widen(gn[i]) + en[i];
                        const unsigned el = voff[i] + (unsigned)(16 * s * m + c0);
                        buf_store_v4f_policy<STREAM ? 2 : 0>(esto, col_ok ? el * 4u : kOutOfRange, mv);
                        *reinterpret_cast<v4f*>(&at[RPI * i + lr][lc]) = mv;
                    }
                }
                // g and e of the next step (or of the next chunk's first step)
                if (s + 1 < STEPS) data_load(c0, s + 1, true, gn, en);
                else data_load(c0 + CH, 0, more, gn, en);
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int u = 0; u < CH / 16; ++u) {
                    const v4f a = *reinterpret_cast<const v4f*>(&at[li][16 * u + 4 * kb]);
#pragma unroll
                    for (int c = 0; c < 4; ++c)
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt) {
                            const float b = Bs[buf][16 * u + 4 * kb + c][16 * nt + li];
                            if constexpr (F64)
                                acc[s][nt] = __builtin_amdgcn_mfma_f64_16x16x4f64((double)a[c], (double)b, acc[s][nt], 0, 0, 0);
                            else
                                acc[s][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[c], b, acc[s][nt], 0, 0, 0);
                        }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
            if (more) stage_store(buf ^ 1, br);
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
                        ws[d.ppart_off + ((int64_t)part * n + row) * ri + j] = (float)acc[s][nt][v];
                }
            }
    }
}

// ---- orthonormal factor by Cholesky-QR, any panel height, rank up to 64 ---------------------------------
constexpr int kHrMaxRank = PSGD_MAX_RANK;
constexpr int kHrGramRows = 128;   // panel rows staged in LDS at a time by the Gram kernel

// Row block: mean P (sum over workers and column ranges, * 1/W) -> P buffer; Gram matrix of the block in fp64 ->
// gram[block][r*r].  The block is staged 128 rows at a time in LDS; the Gram matrix is accumulated on the fp64
// matrix cores: output tile (ta, tb) of 16 x 16 entries is sum over rows of P[row][16 ta + i] P[row][16 tb + j],
// four rows per instruction (A[i][k] = P[4 s + k][16 ta + i], B[k][j] = P[4 s + k][16 tb + j]); the NT^2 tiles
// are dealt to the four wavefronts.  Rows beyond the block and rank columns beyond r are zero in LDS.
template <int NT>
__global__ __launch_bounds__(kBlock) void k_hr_gram(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                    const float* __restrict__ ws, float* __restrict__ p,
                                                    double* __restrict__ gram, int workers) {
    constexpr int RP = 16 * NT;
    constexpr int TPW = (NT * NT + kWavesPerBlock - 1) / kWavesPerBlock;   // output tiles per wavefront
    __shared__ float rows[kHrGramRows][RP + 1];
    const Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int r = d.r, tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    const int li = lane & 15, kb = lane >> 4;
    const int64_t nr = (int64_t)d.n * r;
    const float inv_w = 1.0f / (float)workers;
    const int nparts = workers * d.n_cchunk;
    v4d acc[TPW];
#pragma unroll
    for (int x = 0; x < TPW; ++x) acc[x] = v4d{0.0, 0.0, 0.0, 0.0};
    for (int r0 = t.row0; r0 < t.row0 + t.nrows; r0 += kHrGramRows) {
        const int nrow = min(kHrGramRows, t.row0 + t.nrows - r0);
        __syncthreads();
        // every thread's EPT elements of a partial slice are requested together (out-of-range ones through an
        // offset beyond the descriptor), slice after slice in slice order
        constexpr int EPT = kHrGramRows * RP / kBlock;
        float v[EPT];
        unsigned off[EPT];
#pragma unroll
        for (int x = 0; x < EPT; ++x) {
            const int idx = tid + x * kBlock;
            const int i = idx / RP, k = idx % RP;
            v[x] = 0.f;
            off[x] = (i < nrow && k < r) ? (unsigned)(((int64_t)(r0 + i) * r + k) * 4) : kOutOfRange;
        }
        for (int w = 0; w < nparts; ++w) {
            const buf_rsrc pres = make_rsrc(ws + d.ppart_off + (int64_t)w * nr, nr * 4);   // one slice: n r floats
            float t4[EPT];
#pragma unroll
            for (int x = 0; x < EPT; ++x) t4[x] = buf_load_f32(pres, off[x]);
#pragma unroll
            for (int x = 0; x < EPT; ++x) v[x] += t4[x];
        }
#pragma unroll
        for (int x = 0; x < EPT; ++x) {
            const int idx = tid + x * kBlock;
            const int i = idx / RP, k = idx % RP;
            v[x] *= inv_w;
            if (i < nrow && k < r) p[d.p_off + (int64_t)(r0 + i) * r + k] = v[x];
            rows[i][k] = v[x];
        }
        __syncthreads();
#pragma unroll
        for (int x = 0; x < TPW; ++x) {
            const int pair = wave + x * kWavesPerBlock;
            if (pair < NT * NT) {
                const int ta = pair / NT, tb = pair % NT;
#pragma unroll 8
                for (int s = 0; s < kHrGramRows / 4; ++s) {
                    const double av = (double)rows[4 * s + kb][16 * ta + li];
                    const double bv = (double)rows[4 * s + kb][16 * tb + li];
                    acc[x] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv, acc[x], 0, 0, 0);
                }
            }
        }
    }
    const int nent = r * r;
#pragma unroll
    for (int x = 0; x < TPW; ++x) {
        const int pair = wave + x * kWavesPerBlock;
        if (pair < NT * NT) {
            const int ta = pair / NT, tb = pair % NT;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int ga = 16 * ta + 4 * v + kb, gb = 16 * tb + li;   // fp64 output tile: D[4 v + kb][li]
                if (ga < r && gb < r) gram[d.gram_off + (int64_t)t.part * nent + ga * r + gb] = acc[x][v];
            }
        }
    }
}

// One workgroup per matrix: Gram = sum of the blocks' matrices (block order), Cholesky factor R (upper,
// G = R^T R) in fp64, stored with the reciprocals of its diagonal (0 for a column whose pivot is <= 1e-30:
// that column of P_hat is zero); what is stored at chol[chol_off ..] is R^-1 (r x r, upper triangular).
__global__ __launch_bounds__(kBlock) void k_hr_chol(const MatDesc* __restrict__ mats, const double* __restrict__ gram,
                                                    double* __restrict__ chol) {
    __shared__ double G[kHrMaxRank][kHrMaxRank + 1];    // Gram matrix; the trailing part is updated in place
    __shared__ double Rm[kHrMaxRank][kHrMaxRank + 1];   // its Cholesky factor (upper)
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
    // right-looking Cholesky, row j of R at a time.  Every thread takes the root and the reciprocal of the pivot itself
    // (same value, same arithmetic) and scales the entries of row j that it needs, so a column costs one barrier; the
    // trailing update G[a][b] -= R[j][a] R[j][b] (j < a <= b) runs over 16 x 16 blocks of the upper triangle, one
    // entry per thread.  Row j of G is not written again once its turn has come; R is kept beside it.
    const int ta = tid >> 4, tb = tid & 15;
    for (int j = 0; j < r; ++j) {
        const double piv = G[j][j];
        const bool dead = piv <= 1e-30;
        const double rjj = dead ? 0.0 : sqrt(piv);
        const double ri_j = dead ? 0.0 : 1.0 / rjj;   // 0 for a dead column: its row of R is zero
        if (tid == 0) {
            rinv[j] = ri_j;
            Rm[j][j] = rjj;
        }
        for (int c = j + 1 + tid; c < r; c += kBlock) Rm[j][c] = G[j][c] * ri_j;
        for (int a0 = j + 1; a0 < r; a0 += 16) {
            const int a = a0 + ta;
            const double ra = a < r ? G[j][a] * ri_j : 0.0;
            for (int b0 = a0; b0 < r; b0 += 16) {
                const int b = b0 + tb;
                if (a < r && b < r && b >= a) G[a][b] -= ra * (G[j][b] * ri_j);
            }
        }
        __syncthreads();
    }
    // inverse of R by back substitution, one column per thread: R x = e_c.  A dead column (reciprocal 0)
    // gets x = 0 and, its row of R being zero, takes no part in the others.  X takes G's place.
    double (&X)[kHrMaxRank][kHrMaxRank + 1] = G;
    if (tid < r) {
        const int c = tid;
        for (int i = r - 1; i > c; --i) X[i][c] = 0.0;
        X[c][c] = rinv[c];
        for (int i = c - 1; i >= 0; --i) {
            double v = 0.0;
            int k = i + 1;
            for (; k + 8 <= c + 1; k += 8) {   // eight products' operands requested together, added in the order of k
                double gv[8], xv[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    gv[u] = Rm[i][k + u];
                    xv[u] = X[k + u][c];
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) v += gv[u] * xv[u];
            }
            for (; k <= c; ++k) v += Rm[i][k] * X[k][c];
            X[i][c] = -v * rinv[i];
        }
    }
    __syncthreads();
    double* dst = chol + d.chol_off;
    for (int ent = tid; ent < nent; ent += kBlock) dst[ent] = X[ent / r][ent % r];
}

// P_hat = P R^-1 (R^-1 upper triangular, fp64), in place in the P buffer, on the fp64 matrix cores: output tile
// (16 rows, rank tile tj) = sum over k of P[row][k] X[k][16 tj + j], four k per instruction.  A wavefront takes
// 16 rows at a time and reads them (all rank columns) before it writes any of them.
template <int NT>
__global__ __launch_bounds__(kBlock) void k_hr_apply(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                     const double* __restrict__ chol, float* __restrict__ p) {
    constexpr int RP = 16 * NT;
    __shared__ double X[RP][RP + 1];
    const Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int r = d.r, tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    const int li = lane & 15, kb = lane >> 4;
    const double* src = chol + d.chol_off;
    {
        constexpr int XPT = RP * RP / kBlock;   // all requested before the first is stored
        double xv[XPT];
#pragma unroll
        for (int x = 0; x < XPT; ++x) {
            const int ent = tid + x * kBlock;
            const int a = ent / RP, b = ent % RP;
            xv[x] = src[(a < r && b < r) ? a * r + b : 0];
        }
#pragma unroll
        for (int x = 0; x < XPT; ++x) {
            const int ent = tid + x * kBlock;
            const int a = ent / RP, b = ent % RP;
            X[a][b] = (a < r && b < r) ? xv[x] : 0.0;
        }
    }
    __syncthreads();
    const int row_end = t.row0 + t.nrows;
    const buf_rsrc pres = make_rsrc(p + d.p_off, (int64_t)d.n * r * 4);
    for (int r0 = t.row0 + 16 * wave; r0 < row_end; r0 += 16 * kWavesPerBlock) {
        // A operands: P[r0 + li][4 s + kb] for s = 0 .. RP / 4 - 1
        double av[RP / 4];
#pragma unroll
        for (int s = 0; s < RP / 4; ++s) {
            const int k = 4 * s + kb;
            const unsigned off = (r0 + li < row_end && k < r) ? (unsigned)(((int64_t)(r0 + li) * r + k) * 4) : kOutOfRange;
            av[s] = (double)buf_load_f32(pres, off);
        }
        v4d acc[NT];
#pragma unroll
        for (int tj = 0; tj < NT; ++tj) {
            acc[tj] = v4d{0.0, 0.0, 0.0, 0.0};
#pragma unroll
            for (int s = 0; s < RP / 4; ++s)
                acc[tj] = __builtin_amdgcn_mfma_f64_16x16x4f64(av[s], X[4 * s + kb][16 * tj + li], acc[tj], 0, 0, 0);
        }
        // every lane's loads of these 16 rows are complete (their values were consumed) before the stores
#pragma unroll
        for (int tj = 0; tj < NT; ++tj)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = r0 + 4 * v + kb, j = 16 * tj + li;   // D[4 v + kb][li]
                if (row < row_end && j < r) p[d.p_off + (int64_t)row * r + j] = (float)acc[tj][v];
            }
    }
}

// ---- k_hr_left: Q_w = M^T P_hat ----------------------------------------------------------------------------
// Lane (kb, li) loads 16 bytes at row 4 t + kb, columns c0 + 64 g + 4 li .. + 3; component c of that load
// is the A operand of the instruction that accumulates the columns c0 + 64 g + 4 i + c (i = 0..15).
// B operand: P_hat[row 4 t + kb][16 nt + li].  A wavefront walks its strip of rows 16 at a time (four
// such loads per column group in flight); the workgroup's four strips are added in LDS and one partial Q per
// row block is written.
constexpr int kHrLeftGroups = 2;   // 64-column groups per wavefront (128 columns)

// STREAM: M is larger than the memory-side cache: it is read with non-temporal loads, which keeps it from pushing out
// lines that still wait to be written back
template <int NT, bool STREAM>
__global__ __launch_bounds__(kBlock) void k_hr_left(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                    const float* __restrict__ err, const float* __restrict__ p,
                                                    float* __restrict__ ws, float* __restrict__ q, int workers,
                                                    int64_t estride) {
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

    // The 16 rows of a step: four loads of M per column group and the lane's P_hat entries, through descriptors that
    // end with the strip's last row (rows past it read zeros, a lane without column or rank index is out of range):
    // no branch surrounds a request, so the waits count exactly what is outstanding.
    const buf_rsrc eres = make_rsrc(e + (int64_t)r_begin * m, (int64_t)rn * m * 4);
    const buf_rsrc pres = make_rsrc(p + d.p_off + (int64_t)r_begin * ri, (int64_t)rn * ri * 4);
    unsigned eo[NG], po[NT];   // element offsets of row kb of a step
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        const int col = c0 + 64 * g + 4 * li;
        eo[g] = (col < m && col < c0 + t.nvec) ? (unsigned)(kb * m + col) : kOutOfRange;
    }
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int j = 16 * nt + li;
        po[nt] = j < ri ? (unsigned)(kb * ri + j) : kOutOfRange;
    }
    auto load_step = [&](int r_rel, v4f (&a)[4][NG], float (&b)[4][NT]) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int g = 0; g < NG; ++g)
                a[s][g] = buf_load_v4f_policy<STREAM ? 2 : 0>(
                    eres, eo[g] == kOutOfRange ? kOutOfRange : (eo[g] + (unsigned)((r_rel + 4 * s) * m)) * 4u);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                b[s][nt] = buf_load_f32(pres, po[nt] == kOutOfRange ? kOutOfRange : (po[nt] + (unsigned)((r_rel + 4 * s) * ri)) * 4u);
        }
    };
    auto multiply = [&](const v4f (&a)[4][NG], const float (&b)[4][NT]) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int g = 0; g < NG; ++g)
#pragma unroll
                for (int c = 0; c < 4; ++c)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[g][c][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[s][g][c], b[s][nt], acc[g][c][nt], 0, 0, 0);
    };
    // the next step's loads are in flight while the current step is multiplied
    v4f an[4][NG];
    float bn[4][NT];
    load_step(0, an, bn);
    for (int r0 = 0; r0 < rn; r0 += 16) {
        v4f a[4][NG];
        float b[4][NT];
#pragma unroll
        for (int s = 0; s < 4; ++s) {
#pragma unroll
            for (int g = 0; g < NG; ++g) a[s][g] = an[s][g];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) b[s][nt] = bn[s][nt];
        }
        load_step(r0 + 16, an, bn);   // past the strip's last row: out of range, nothing is fetched
        multiply(a, b);
    }
    // acc[g][c][nt][v] = Q[c0 + 64 g + 4 (4 kb + v) + c][16 nt + li] for this strip.  The four strips of the
    // workgroup are added through LDS as (s0 + s1) + (s2 + s3), so that one partial per row block is written.
    constexpr int ACC = NG * 4 * NT;   // accumulator vectors per lane
    __shared__ v4f stage[2][ACC][kWave];
    auto put = [&](int slot) {
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) stage[slot][(g * 4 + c) * NT + nt][lane] = acc[g][c][nt];
    };
    auto take = [&](int slot) {
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[g][c][nt] += stage[slot][(g * 4 + c) * NT + nt][lane];
    };
    if (wave & 1) put(wave >> 1);
    __syncthreads();
    if (!(wave & 1)) take(wave >> 1);
    __syncthreads();
    if (wave == 2) put(0);
    __syncthreads();
    if (wave != 0) return;
    take(0);
    // the only partial of its matrix is the result itself (mean over one worker): it goes straight into Q
    const int part = w * d.n_rblock + t.part;
    float* dst = workers * d.n_rblock == 1 ? q + d.q_off : ws + d.qpart_off + (int64_t)part * m * ri;
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
// v = 0..3: four consecutive columns of one row.  A 16 x 16 block is then 16 rows of 64 bytes, too short a run for
// the memory system (a plain pass with that shape reads and writes 5.0 TB/s here, with runs of 512 bytes 5.8), so
// the eight blocks of a 16-row step go through a tile in LDS private to the wavefront and memory is touched in a
// second lane layout: lane (h, j) holds row 2 i + h, columns 4 j .. 4 j + 3 of the step's 16 x 128 piece, i = 0..7,
// i.e. every load and store instruction covers two runs of 512 bytes.  The Q rows of the workgroup's 128 columns
// are staged in LDS once; M and P_hat of the next 16-row step are in flight while the current one is multiplied.
// Buffer addressing: each wavefront's descriptors end with its last row.  STREAM: sets beyond the memory-side
// cache read M and write e' and Delta' around the caches.
constexpr int kHrDecompBlocks = 8;   // 16-column blocks per wavefront (128 columns)
constexpr int kHrDecompStride = 16 * kHrDecompBlocks + 4;   // floats per row of the wavefront's tile in LDS

template <bool BF, int AUX>
__device__ __forceinline__ void buf_store_out4(buf_rsrc r, unsigned off, v4f v) {
    if constexpr (BF) {
        v2u x;
        x.x = pack_bf16x2(v.x, v.y);
        x.y = pack_bf16x2(v.z, v.w);
        __builtin_amdgcn_raw_buffer_store_b64(x, r, (int)off, 0, AUX);
    } else {
        buf_store_v4f_policy<AUX>(r, off, v);
    }
}

// OM: what becomes of Delta': 0 stored as fp32, 1 stored as bf16, 2 not stored but folded into the momentum and
// parameter buffers (Algorithm 2's last two lines)
template <int NT, int OM, bool STREAM>
__global__ __launch_bounds__(kBlock, 2) void k_hr_decomp(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                         float* __restrict__ err, const float* __restrict__ p,
                                                         const float* __restrict__ q, void* __restrict__ out,
                                                         int64_t estride, UpdateArgs upd) {
    constexpr bool BF = OM == 1;
    constexpr bool UPD = OM == 2;
    constexpr int KK = 4 * NT;   // instructions per 16 x 16 block (K = 16 NT in steps of 4)
    constexpr int CB = kHrDecompBlocks;
    constexpr int RP = 16 * NT;
    constexpr int QST = RP + 4;  // floats per LDS row of the staged Q block
    constexpr int OS = BF ? 2 : 4;
    constexpr int AUX = STREAM ? 2 : 0;
    __shared__ float Qs[16 * CB][QST];
    __shared__ __attribute__((aligned(16))) float Ds[kWavesPerBlock][16][kHrDecompStride];
    const Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int w = blockIdx.y;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, kb = lane >> 4;
    const int ri = d.r, m = d.m;
    const int c0 = t.vec0;
    const int c_end = min(m, c0 + t.nvec);

    {
        const buf_rsrc qres = make_rsrc(q + d.q_off, (int64_t)m * ri * 4);
        constexpr int QPT = 16 * CB * RP / kBlock;   // staged elements per thread: all requested before the first is stored
        float qv[QPT];
#pragma unroll
        for (int x = 0; x < QPT; ++x) {
            const int idx = tid + x * kBlock;
            const int col = idx / RP, k = idx % RP;
            const unsigned off = (k < ri && c0 + col < c_end) ? (unsigned)((c0 + col) * ri + k) * 4u : kOutOfRange;
            qv[x] = buf_load_f32(qres, off);
        }
#pragma unroll
        for (int x = 0; x < QPT; ++x) {
            const int idx = tid + x * kBlock;
            Qs[idx / RP][idx % RP] = qv[x];
        }
    }
    __syncthreads();

    int rb, rn;
    wave_rows(t.nrows, wave, &rb, &rn);
    const int r_begin = t.row0 + rb;
    const int64_t ebase = (int64_t)r_begin * m;
    const buf_rsrc eres = make_rsrc(err + (int64_t)w * estride + d.off + ebase, (int64_t)rn * m * 4);
    // Delta' (or momentum and parameters) belong to worker 0's workgroups: the others get empty ranges
    const buf_rsrc ores = make_rsrc(UPD ? nullptr : static_cast<char*>(out) + (d.off + ebase) * OS,
                                    (!UPD && w == 0) ? (int64_t)rn * m * OS : 0);
    const buf_rsrc mres = make_rsrc(UPD ? upd.mom + d.off + ebase : nullptr, (UPD && w == 0) ? (int64_t)rn * m * 4 : 0);
    const buf_rsrc xres = make_rsrc(UPD ? upd.param + d.off + ebase : nullptr, (UPD && w == 0) ? (int64_t)rn * m * 4 : 0);
    const buf_rsrc pres = make_rsrc(p + d.p_off + (int64_t)r_begin * ri, (int64_t)rn * ri * 4);
    // lane offsets in elements, relative to the first row of the strip; out of range where the column (of M) or
    // the rank index (of P_hat) does not exist
    const int h = lane >> 5, j = lane & 31;
    const int mcol = c0 + 4 * j;
    const unsigned eo = mcol < c_end ? (unsigned)(h * m + mcol) : kOutOfRange;   // row h of the step, this lane's columns
    unsigned po[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) {
        const int k = 4 * kk + kb;
        po[kk] = k < ri ? (unsigned)(li * ri + k) : kOutOfRange;
    }
    // an out-of-range marker stays out of range after scaling and stepping: the element offsets below are
    // under 2^26, so it is kept apart by using byte offsets only at the access
    auto e_off = [&](int i, int step_el, int bytes) -> unsigned {
        return eo == kOutOfRange ? kOutOfRange : (eo + (unsigned)(2 * i * m) + (unsigned)step_el) * (unsigned)bytes;
    };
    auto load_step = [&](int r_rel, v4f (&mv)[CB], float (&bp)[KK]) {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
            bp[kk] = buf_load_f32(pres, po[kk] == kOutOfRange ? kOutOfRange : (po[kk] + (unsigned)(r_rel * ri)) * 4u);
#pragma unroll
        for (int i = 0; i < CB; ++i) mv[i] = buf_load_v4f_policy<AUX>(eres, e_off(i, r_rel * m, 4));
    };

    float (*dt)[kHrDecompStride] = Ds[wave];
    v4f mvn[CB];
    float bpn[KK];
    load_step(0, mvn, bpn);
    for (int r_rel = 0; r_rel < rn; r_rel += 16) {
        v4f mv[CB];
        float bp[KK];
#pragma unroll
        for (int i = 0; i < CB; ++i) mv[i] = mvn[i];
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) bp[kk] = bpn[kk];
        load_step(r_rel + 16, mvn, bpn);   // past the strip's last row: out of range, nothing is fetched
        // at two and four rank tiles the Q operands are fetched from LDS at every step instead of being kept
        // in registers for the whole strip (64 or 128 of them)
        v4f mo[UPD ? CB : 1], pa[UPD ? CB : 1];
        if constexpr (UPD) {   // momentum and parameters of this step: requested before the products are issued
#pragma unroll
            for (int i = 0; i < CB; ++i) {
                mo[i] = buf_load_v4f(mres, e_off(i, r_rel * m, 4));
                pa[i] = buf_load_v4f(xres, e_off(i, r_rel * m, 4));
            }
        }
        if constexpr (NT >= 2) asm volatile("" ::: "memory");
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) {
            v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
                acc = __builtin_amdgcn_mfma_f32_16x16x4f32(Qs[16 * cb + li][4 * kk + kb], bp[kk], acc, 0, 0, 0);
            *reinterpret_cast<v4f*>(&dt[li][16 * cb + 4 * kb]) = acc;
        }
        wave_lds_done();
#pragma unroll
        for (int i = 0; i < CB; ++i) {
            const v4f acc = *reinterpret_cast<const v4f*>(&dt[2 * i + h][4 * j]);
            buf_store_v4f_policy<AUX>(eres, e_off(i, r_rel * m, 4), mv[i] - acc);
            if constexpr (UPD) {
                float m4[4] = {mo[i].x, mo[i].y, mo[i].z, mo[i].w}, x4[4] = {pa[i].x, pa[i].y, pa[i].z, pa[i].w};
                const float d4[4] = {acc.x, acc.y, acc.z, acc.w};
                momentum_step<4>(m4, x4, d4, upd.lr, upd.lam);
                buf_store_v4f(mres, e_off(i, r_rel * m, 4), v4f{m4[0], m4[1], m4[2], m4[3]});
                buf_store_v4f(xres, e_off(i, r_rel * m, 4), v4f{x4[0], x4[1], x4[2], x4[3]});
            } else {
                buf_store_out4<BF, AUX>(ores, e_off(i, r_rel * m, OS), acc);   // dropped for workers other than the first (empty range)
            }
        }
        wave_lds_done();   // the tile is written again in the next step
    }
}

template <bool BFI, bool BFO>
__global__ __launch_bounds__(kBlock) void k_hr_vec(const void* __restrict__ grad, void* __restrict__ out, int workers,
                                                   int64_t gstride, int64_t n_mat_elems, int64_t n_vec, UpdateArgs upd) {
    const float inv_w = 1.0f / (float)workers;
    for (int64_t idx = (int64_t)blockIdx.x * kBlock + threadIdx.x; idx < n_vec; idx += (int64_t)gridDim.x * kBlock) {
        float s = 0.f;
        for (int w = 0; w < workers; ++w) {
            const int64_t at = (int64_t)w * gstride + n_mat_elems + idx;
            if constexpr (BFI) s += bf16_to_f32(static_cast<const bf16_t*>(grad)[at]);
            else s += static_cast<const float*>(grad)[at];
        }
        s *= inv_w;
        if (upd.mom) {
            float m1[1] = {upd.mom[n_mat_elems + idx]}, x1[1] = {upd.param[n_mat_elems + idx]};
            const float d1[1] = {s};
            momentum_step<1>(m1, x1, d1, upd.lr, upd.lam);
            upd.mom[n_mat_elems + idx] = m1[0];
            upd.param[n_mat_elems + idx] = x1[0];
        } else if constexpr (BFO) {
            static_cast<bf16_t*>(out)[n_mat_elems + idx] = f32_to_bf16(s);
        } else {
            static_cast<float*>(out)[n_mat_elems + idx] = s;
        }
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
static void hr_launch_right(psgd_plan* plan, const void* grad, float* err, const float* q, float* ws, hipStream_t s,
                            bool add) {
    dim3 grid((unsigned)plan->hr_tiles1.size(), (unsigned)plan->workers);
    // fp64 accumulation at every rank of this path: it costs nothing next to the loads (2.88 against 2.92 ms on
    // the transformer set) and at rank 4 fp32 accumulation left P_hat up to 8e-6 off after two steps
    // Sets beyond the memory-side cache: e is read and M written around the caches (non-temporal), as the streaming
    // path does (transformer subset, rank 16: k_hr_right -3 %, and k_hr_left, which then finds less of its M pushed
    // out by lines nobody reads again, -7 %).  The same hint on k_hr_decomp's 64-byte pieces costs 40 %.
#define HR_RIGHT(BFV, STREAMV)                                                                                             \
    hipLaunchKernelGGL((k_hr_right<NT, BFV, true, STREAMV>), grid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.hr_tiles1, \
                       grad, err, q, ws, plan->sizes.grad_stride, plan->sizes.err_stride, add ? 1 : 0)
    if (plan->stream_hints) {
        if (plan->grad_dtype == PSGD_BF16) HR_RIGHT(true, true);
        else HR_RIGHT(false, true);
    } else {
        if (plan->grad_dtype == PSGD_BF16) HR_RIGHT(true, false);
        else HR_RIGHT(false, false);
    }
#undef HR_RIGHT
}

template <int NT>
static void hr_launch_decomp(psgd_plan* plan, float* err, const float* p, const float* q, void* out, hipStream_t s,
                             const UpdateArgs& upd) {
    dim3 grid((unsigned)plan->hr_tiles4.size(), (unsigned)plan->workers);
#define HR_DECOMP(OMV, STREAMV)                                                                                                \
    hipLaunchKernelGGL((k_hr_decomp<NT, OMV, STREAMV>), grid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.hr_tiles4, err, p, q, \
                       out, plan->sizes.err_stride, upd)
    if (plan->stream_hints) {
        if (upd.mom) HR_DECOMP(2, true);
        else if (plan->out_dtype == PSGD_BF16) HR_DECOMP(1, true);
        else HR_DECOMP(0, true);
    } else {
        if (upd.mom) HR_DECOMP(2, false);
        else if (plan->out_dtype == PSGD_BF16) HR_DECOMP(1, false);
        else HR_DECOMP(0, false);
    }
#undef HR_DECOMP
}

static double* hr_doubles(psgd_plan* plan, void* workspace) {
    const size_t float_bytes = (size_t)(plan->ws_ppart_floats + plan->ws_qpart_floats) * sizeof(float);
    return reinterpret_cast<double*>(static_cast<char*>(workspace) + (float_bytes + 255) / 256 * 256);
}

psgd_status hr_compress(psgd_plan* plan, const void* grad, float* err, float* q, float* p, void* workspace,
                        void* stream, bool add) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* ws = static_cast<float*>(workspace);
    if (plan->mats.empty()) return PSGD_OK;
    const int nt = plan->hr_nt;
    HR_MARK(0);
    plan->compress_marked = plan->profiling;
    if (nt == 1) hr_launch_right<1>(plan, grad, err, q, ws, s, add);
    else if (nt == 2) hr_launch_right<2>(plan, grad, err, q, ws, s, add);
    else hr_launch_right<4>(plan, grad, err, q, ws, s, add);
    HR_CHECK("launch k_hr_right");
    HR_MARK(1);
    double* gram = hr_doubles(plan, workspace);
    double* chol = gram + plan->ws_gram_doubles;
    const dim3 ggrid((unsigned)plan->tiles_gram.size());
    if (nt == 1)
        hipLaunchKernelGGL((k_hr_gram<1>), ggrid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.tiles_gram, ws, p, gram,
                           plan->workers);
    else if (nt == 2)
        hipLaunchKernelGGL((k_hr_gram<2>), ggrid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.tiles_gram, ws, p, gram,
                           plan->workers);
    else
        hipLaunchKernelGGL((k_hr_gram<4>), ggrid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.tiles_gram, ws, p, gram,
                           plan->workers);
    HR_CHECK("launch k_hr_gram");
    hipLaunchKernelGGL(k_hr_chol, dim3((unsigned)plan->mats.size()), dim3(kBlock), 0, s, plan->dev.mats, gram, chol);
    HR_CHECK("launch k_hr_chol");
    if (nt == 1)
        hipLaunchKernelGGL((k_hr_apply<1>), ggrid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.tiles_gram, chol, p);
    else if (nt == 2)
        hipLaunchKernelGGL((k_hr_apply<2>), ggrid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.tiles_gram, chol, p);
    else
        hipLaunchKernelGGL((k_hr_apply<4>), ggrid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.tiles_gram, chol, p);
    HR_CHECK("launch k_hr_apply");
    HR_MARK(2);
    {
        dim3 grid((unsigned)plan->hr_tiles3.size(), (unsigned)plan->workers);
#define HR_LAUNCH_LEFT(NTV, STREAMV)                                                                                   \
    hipLaunchKernelGGL((k_hr_left<NTV, STREAMV>), grid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.hr_tiles3, err, p, ws, \
                       q, plan->workers, plan->sizes.err_stride)
        if (plan->stream_hints) {
            if (nt == 1) HR_LAUNCH_LEFT(1, true);
            else if (nt == 2) HR_LAUNCH_LEFT(2, true);
            else HR_LAUNCH_LEFT(4, true);
        } else {
            if (nt == 1) HR_LAUNCH_LEFT(1, false);
            else if (nt == 2) HR_LAUNCH_LEFT(2, false);
            else HR_LAUNCH_LEFT(4, false);
        }
#undef HR_LAUNCH_LEFT
    }
    HR_CHECK("launch k_hr_left");
    HR_MARK(3);
    psgd_status st = launch_q_reduce(plan, ws, q, stream);
    if (st != PSGD_OK) return st;
    HR_MARK(4);
    return PSGD_OK;
}

// mean over the workers of the vector-shaped tensors (any mix of fp32 / bf16 gradients and output)
psgd_status launch_vector_mean(psgd_plan* plan, const void* grad, void* out, void* stream, const UpdateArgs& upd) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t L = plan->sizes.n_vec_elems;
    if (L > 0) {
        const unsigned blocks = (unsigned)std::min<int64_t>(1024, (L + kBlock - 1) / kBlock);
        const bool bi = plan->grad_dtype == PSGD_BF16, bo = plan->out_dtype == PSGD_BF16;
        if (bi && bo)
            hipLaunchKernelGGL((k_hr_vec<true, true>), dim3(blocks), dim3(kBlock), 0, s, grad, out, plan->workers,
                               plan->sizes.grad_stride, plan->sizes.n_mat_elems, L, upd);
        else if (bi)
            hipLaunchKernelGGL((k_hr_vec<true, false>), dim3(blocks), dim3(kBlock), 0, s, grad, out, plan->workers,
                               plan->sizes.grad_stride, plan->sizes.n_mat_elems, L, upd);
        else if (bo)
            hipLaunchKernelGGL((k_hr_vec<false, true>), dim3(blocks), dim3(kBlock), 0, s, grad, out, plan->workers,
                               plan->sizes.grad_stride, plan->sizes.n_mat_elems, L, upd);
        else
            hipLaunchKernelGGL((k_hr_vec<false, false>), dim3(blocks), dim3(kBlock), 0, s, grad, out, plan->workers,
                               plan->sizes.grad_stride, plan->sizes.n_mat_elems, L, upd);
        HR_CHECK("launch k_hr_vec");
    }
    return PSGD_OK;
}

psgd_status hr_decompress(psgd_plan* plan, const float* p, const float* q, float* err, const void* grad, void* out,
                          void* stream, const UpdateArgs& upd) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int nt = plan->hr_nt;
    HR_MARK(5);
    if (!plan->hr_tiles4.empty()) {
        if (nt == 1) hr_launch_decomp<1>(plan, err, p, q, out, s, upd);
        else if (nt == 2) hr_launch_decomp<2>(plan, err, p, q, out, s, upd);
        else hr_launch_decomp<4>(plan, err, p, q, out, s, upd);
        HR_CHECK("launch k_hr_decomp");
    }
    psgd_status vs = launch_vector_mean(plan, grad, out, stream, upd);
    if (vs != PSGD_OK) return vs;
    HR_MARK(6);
    return finish_profiled_step(plan);
}

}  // namespace psgd
