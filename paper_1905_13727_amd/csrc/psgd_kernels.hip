// HIP kernels for gfx950 (MI355X) and their launchers.
//
// One PowerSGD step (arXiv 1905.13727, Algorithm 1 inside the error-feedback
// loop of Algorithm 2) is five to seven grouped launches over work-lists built by the
// planner; every launch covers all matrices of the model and all W workers:
//
//   k_ef_right    M_w = g_w + e_w (stored in e_w's place) fused with the row dot
//                 products of P_w = M_w Q               (Alg. 2 "Delta_w", Alg. 1 "P <- M Q");
//                 without the add, one more subspace iteration on a stored M (Appendix G.7)
//   k_gram_chol   mean over workers / column chunks, then the orthonormal factor Gram-Schmidt
//                 gives, by Cholesky-QR over many workgroups in one launch; k_gram,
//                 k_chol_apply: the same in two launches (Alg. 1 "all reduce mean", "orthogonalize";
//                 Remark "Orthogonalization is a linear operation")
//   k_ortho       the same by Gram-Schmidt in LDS, one workgroup per matrix, for the panels of at
//                 most ortho_rows rows (a tuning key; 0 by default: none)
//   k_left        column sums of Q_w = M_w^T P_hat      (Alg. 1 "Q <- M^T P_hat")
//   k_q_reduce    mean over workers / row blocks        (Alg. 1 second "all reduce mean"); also
//                 pre-reduces the partial P when there are many
//   k_decomp      Delta' = P_hat Q^T fused with e_w = M_w - Delta' and with the
//                 mean of the vector-shaped tensors     (Alg. 1 "decompress", Alg. 2 error memory);
//                 optionally with Alg. 2's momentum and parameter update instead of storing Delta'
//
// All reductions run in a fixed order (no float atomics): results are
// bit-reproducible from run to run.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "psgd_device.h"
#include "psgd_internal.h"

namespace psgd {

// ---- k_ef_right: M = g + e, P_w[i,:] = sum_j M[i,j] Q[j,:] ---------------------------------------
//
// A wavefront owns a strip of rows and a chunk of at most 64*NV*V columns.  Each lane keeps
// the Q rows of its columns in registers for the whole strip, streams g and e with V-wide
// loads, writes M over e, and the wavefront reduces R dot products per row.  Partial sums
// of different column chunks / workers go to separate slices of the workspace.

// ADD = false: one more subspace iteration on an update that already sits in e (nothing is added, e is not written)
// GBF: the gradient is stored as bf16 (M = g + e is an fp32 quantity either way)
template <int R, int V, int NV, bool ADD, bool GBF>
__device__ __forceinline__ void ef_right_tile(const Tile& t, const MatDesc& d, const void* __restrict__ g,
                                              float* __restrict__ e, const float* __restrict__ q,
                                              float* __restrict__ ppart) {
    constexpr unsigned GS = GBF ? 2u : 4u;   // bytes per gradient element
    // rows per step: all their loads are in flight together; RS * R results fit the 64 lanes
    constexpr int RS = (16 / NV) * R <= kWave ? 16 / NV : 8;
    static_assert(RS * R <= kWave, "one lane per (row, rank) result of a step");
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ri = d.r;

    float qr[NV][V][R];
    bool valid[NV];
    int col[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int jv = lane + kWave * v;
        valid[v] = jv < t.nvec;
        col[v] = (t.vec0 + jv) * V;
        load_factor_rows<R, V>(q + d.q_off + (int64_t)col[v] * ri, ri, valid[v], qr[v]);
    }

    int rb, rn;
    wave_rows(t.nrows, wave, &rb, &rn);
    const int i_begin = t.row0 + rb, i_end = i_begin + rn;
    // Descriptors over the rows of this wavefront's strip: a lane whose columns do not exist carries an
    // out-of-range offset, a row past the strip lies beyond the range by itself; such loads return zero and
    // such stores are dropped, so no access sits behind a branch and the waits count exactly what is outstanding.
    const int64_t strip = d.off + (int64_t)i_begin * d.m;
    const buf_rsrc gres = make_rsrc(static_cast<const char*>(g) + strip * GS, ADD ? (int64_t)rn * d.m * GS : 0);
    const buf_rsrc eres = make_rsrc(e + strip, (int64_t)rn * d.m * 4);
    unsigned coff[NV], goff[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        coff[v] = valid[v] ? (unsigned)col[v] * 4u : kOutOfRange;
        goff[v] = valid[v] ? (unsigned)col[v] * GS : kOutOfRange;
    }
    for (int i0 = i_begin; i0 < i_end; i0 += RS) {
        const int rows = min(RS, i_end - i0);
        const unsigned row_off = (unsigned)(i0 - i_begin) * (unsigned)d.m * 4u;
        float mv[RS][NV][V];
        // every load of the step is issued before anything is used
        if constexpr (ADD) {
#pragma unroll
            for (int i = 0; i < RS; ++i)
#pragma unroll
                for (int v = 0; v < NV; ++v)
                    buf_ld_grad<V, GBF>(gres, goff[v] + (row_off / 4u + (unsigned)i * (unsigned)d.m) * GS, mv[i][v]);
        } else {
#pragma unroll
            for (int i = 0; i < RS; ++i)
#pragma unroll
                for (int v = 0; v < NV; ++v)
#pragma unroll
                    for (int x = 0; x < V; ++x) mv[i][v][x] = 0.f;
        }
        // e in two halves of the step's rows (registers): all loads of a half in flight, then add and store
        constexpr int RH = RS / 2;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            float ev[RH][NV][V];
#pragma unroll
            for (int i = 0; i < RH; ++i)
#pragma unroll
                for (int v = 0; v < NV; ++v)
                    buf_ldv<V>(eres, coff[v] + row_off + (unsigned)(h * RH + i) * (unsigned)d.m * 4u, ev[i][v]);
#pragma unroll
            for (int i = 0; i < RH; ++i)
#pragma unroll
                for (int v = 0; v < NV; ++v) {
#pragma unroll
                    for (int x = 0; x < V; ++x) mv[h * RH + i][v][x] += ev[i][v][x];
                    if constexpr (ADD)
                        buf_stv<V>(eres, coff[v] + row_off + (unsigned)(h * RH + i) * (unsigned)d.m * 4u, mv[h * RH + i][v]);
                }
        }
        // RS * R dot products, reduced over the wavefront all at once; lane i * R + k receives the result of
        // (row i, rank k).  Rows past the strip were read as zeros.
        float part[RS * R];
#pragma unroll
        for (int i = 0; i < RS; ++i)
#pragma unroll
            for (int k = 0; k < R; ++k) {
                float s = 0.f;
#pragma unroll
                for (int v = 0; v < NV; ++v)
#pragma unroll
                    for (int x = 0; x < V; ++x) s = fmaf(mv[i][v][x], qr[v][x][k], s);
                part[i * R + k] = s;
            }
        const float mine = lane_sums<RS * R>(part);
        const int li = lane / R, lk = lane % R;
        if (li < rows && lk < ri)
            ppart[d.ppart_off + ((int64_t)t.part * d.n + i0 + li) * ri + lk] = mine;
    }
}

template <int R, int NV, bool ADD, bool GBF>
__global__ __launch_bounds__(kBlock) void k_ef_right(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                     const void* __restrict__ grad, float* __restrict__ err,
                                                     const float* __restrict__ q, float* __restrict__ ws,
                                                     int64_t gstride, int64_t estride) {
    Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int w = blockIdx.y;
    const void* g = static_cast<const char*>(grad) + (int64_t)w * gstride * (GBF ? 2 : 4);
    float* e = err + (int64_t)w * estride;
    t.part += w * d.n_cchunk;   // partial slices: [worker][column chunk]
    if (d.vec == 4) ef_right_tile<R, 4, NV, ADD, GBF>(t, d, g, e, q, ws);
    else if (d.vec == 2) ef_right_tile<R, 2, NV, ADD, GBF>(t, d, g, e, q, ws);
    else ef_right_tile<R, 1, NV, ADD, GBF>(t, d, g, e, q, ws);
}

// sum of `nparts` partial slices (stride `stride` floats) at `src`, in slice order, eight loads in flight
__device__ __forceinline__ float sum_parts(const float* __restrict__ src, int nparts, int64_t stride) {
    float s = 0.f;
    int c = 0;
    for (; c + 8 <= nparts; c += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = src[(int64_t)(c + u) * stride];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; c < nparts; ++c) s += src[(int64_t)c * stride];
    return s;
}

// the same for the r <= R values of one panel row at once: the loads of all columns and of several slices are in
// flight together; per column the slices are added in slice order, as in sum_parts (bit-identical to it)
template <int R>
__device__ __forceinline__ void sum_parts_row(const float* __restrict__ src, int r, int nparts, int64_t stride,
                                              float (&row)[R]) {
    constexpr int U = R <= 2 ? 8 : (R <= 4 ? 4 : 2);
#pragma unroll
    for (int k = 0; k < R; ++k) row[k] = 0.f;
    int c = 0;
    for (; c + U <= nparts; c += U) {
        float v[U][R];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int k = 0; k < R; ++k) v[u][k] = k < r ? src[(int64_t)(c + u) * stride + k] : 0.f;
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int k = 0; k < R; ++k) row[k] += v[u][k];
    }
    for (; c < nparts; ++c)
#pragma unroll
        for (int k = 0; k < R; ++k)
            if (k < r) row[k] += src[(int64_t)c * stride + k];
}

__global__ __launch_bounds__(kOrthoBlock) void k_ortho(const MatDesc* __restrict__ mats, const int32_t* __restrict__ which,
                                                       const float* __restrict__ ws, float* __restrict__ p, int workers,
                                                       int pre_reduced) {
    __shared__ float panel[kPanelFloats];
    __shared__ double red[kOrthoBlock / kWave][kValuMaxRank];
    const MatDesc d = mats[which[blockIdx.x]];
    const int n = d.n, r = d.r;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int64_t nr = (int64_t)n * r;    // <= kPanelFloats (planner)
    float* P = panel;
    const float inv_w = 1.0f / (float)workers;
    const int nparts = pre_reduced ? 1 : workers * d.n_cchunk;

    // mean over workers / column chunks: four panel elements per thread in flight
    for (int64_t base = tid; base < nr; base += 4 * kOrthoBlock) {
        float s[4] = {0.f, 0.f, 0.f, 0.f};
        for (int c = 0; c < nparts; ++c) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t idx = base + (int64_t)u * kOrthoBlock;
                v[u] = idx < nr ? ws[d.ppart_off + (int64_t)c * nr + idx] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) s[u] += v[u];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t idx = base + (int64_t)u * kOrthoBlock;
            if (idx < nr) P[idx] = s[u] * inv_w;
        }
    }
    __syncthreads();

    for (int j = 0; j < r; ++j) {
        double s[kValuMaxRank];
#pragma unroll
        for (int k = 0; k < kValuMaxRank; ++k) s[k] = 0.0;
        for (int i = tid; i < n; i += kOrthoBlock) {
            const float* row = P + (int64_t)i * r;
            const double pj = (double)row[j];
#pragma unroll
            for (int k = 0; k < kValuMaxRank; ++k)
                if (k >= j && k < r) s[k] += pj * (double)row[k];
        }
#pragma unroll
        for (int k = 0; k < kValuMaxRank; ++k) {
            if (k >= j && k < r) {
                const double v = wave_sum(s[k]);
                if (lane == 0) red[wave][k] = v;
            }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < kValuMaxRank; ++k) {
            if (k >= j && k < r) {
                double v = 0.0;
                for (int wv = 0; wv < kOrthoBlock / kWave; ++wv) v += red[wv][k];
                s[k] = v;
            }
        }
        double sjj = 0.0;
#pragma unroll
        for (int k = 0; k < kValuMaxRank; ++k)
            if (k == j) sjj = s[k];
        if (sjj <= 1e-30) {
            for (int i = tid; i < n; i += kOrthoBlock) P[(int64_t)i * r + j] = 0.f;
        } else {
            const double inv = 1.0 / sqrt(sjj);
            double c[kValuMaxRank];
#pragma unroll
            for (int k = 0; k < kValuMaxRank; ++k) c[k] = s[k] / sjj;
            for (int i = tid; i < n; i += kOrthoBlock) {
                float* row = P + (int64_t)i * r;
                const double pj = (double)row[j];
                row[j] = (float)(pj * inv);
#pragma unroll
                for (int k = 0; k < kValuMaxRank; ++k)
                    if (k > j && k < r) row[k] = (float)((double)row[k] - c[k] * pj);
            }
        }
        __syncthreads();
    }
    float* dst = p + d.p_off;
    for (int64_t idx = tid; idx < nr; idx += kOrthoBlock) dst[idx] = panel[idx];
}

// ---- the same orthonormal factor by Cholesky-QR over row blocks (every panel not given to k_ortho) ----
//
// Gram-Schmidt yields P_hat = P R^-1 with R upper triangular, positive diagonal (the paper's remark
// "Orthogonalization is a linear operation"); that R is the Cholesky factor of the Gram matrix
// P^T P.  The factor is computed that way, over many
// workgroups: k_gram sums the partials into the mean P (stored in the P buffer) and reduces the
// Gram matrix of its row block in fp64; k_chol_apply adds the blocks' Gram matrices in a fixed order,
// factorises (fp64, r <= 8) and solves P_hat R = P row by row.  A pivot <= 1e-30 (the squared norm
// Gram-Schmidt would find for that column at its turn) gives a zero column.

__global__ __launch_bounds__(kBlock) void k_gram(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                 const float* __restrict__ ws, float* __restrict__ p,
                                                 double* __restrict__ gram, int workers, int pre_reduced) {
    __shared__ double red[kWavesPerBlock][kValuMaxRank * kValuMaxRank];
    const Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int r = d.r, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int64_t nr = (int64_t)d.n * r;
    const float inv_w = 1.0f / (float)workers;
    const int nparts = pre_reduced ? 1 : workers * d.n_cchunk;
    double g[kValuMaxRank][kValuMaxRank];
#pragma unroll
    for (int a = 0; a < kValuMaxRank; ++a)
#pragma unroll
        for (int b = 0; b < kValuMaxRank; ++b) g[a][b] = 0.0;
    for (int i = t.row0 + tid; i < t.row0 + t.nrows; i += kBlock) {
        float row[kValuMaxRank];
        sum_parts_row<kValuMaxRank>(ws + d.ppart_off + (int64_t)i * r, r, nparts, nr, row);
#pragma unroll
        for (int k = 0; k < kValuMaxRank; ++k) {
            row[k] *= inv_w;
            if (k < r) p[d.p_off + (int64_t)i * r + k] = row[k];
        }
#pragma unroll
        for (int a = 0; a < kValuMaxRank; ++a)
#pragma unroll
            for (int b = a; b < kValuMaxRank; ++b)
                if (b < r) g[a][b] += (double)row[a] * (double)row[b];
    }
#pragma unroll
    for (int a = 0; a < kValuMaxRank; ++a)
#pragma unroll
        for (int b = a; b < kValuMaxRank; ++b)
            if (b < r) {
                const double v = wave_sum(g[a][b]);
                if (lane == 0) red[wave][a * kValuMaxRank + b] = v;
            }
    __syncthreads();
    if (tid < r * r) {
        const int a = tid / r, b = tid % r;
        double v = 0.0;
        if (b >= a)
            for (int wv = 0; wv < kWavesPerBlock; ++wv) v += red[wv][a * kValuMaxRank + b];
        gram[d.gram_off + (int64_t)t.part * r * r + tid] = v;   // upper triangle, zeros below
    }
}

__global__ __launch_bounds__(kBlock) void k_chol_apply(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                       const double* __restrict__ gram, float* __restrict__ p) {
    constexpr int kMaxSlices = 16;
    __shared__ double part[kMaxSlices][kValuMaxRank * kValuMaxRank];
    __shared__ double Gs[kValuMaxRank * kValuMaxRank];  // the summed Gram matrix, r x r
    __shared__ double Rm[kValuMaxRank][kValuMaxRank];   // upper triangular factor
    __shared__ double rinv[kValuMaxRank];               // 1 / R_jj, 0 for a zero column
    const Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int r = d.r, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    // Gram matrix = sum of the row blocks' matrices: the blocks are cut into consecutive slices (4, 8 or 16 of
    // them, as many as lanes allow: one lane per matrix entry and slice), each slice summed in block order,
    // then the slices in slice order
    const int nent = r * r;
    const int per_wave = nent <= 16 ? 4 : (nent <= 32 ? 2 : 1);   // slices per wavefront
    const int nslices = kWavesPerBlock * per_wave;
    {
        const int lanes_per = kWave / per_wave;
        const int ent = lane % lanes_per, sl = wave * per_wave + lane / lanes_per;
        if (ent < nent) {
            const int per = (d.n_gblock + nslices - 1) / nslices;
            const int b0 = min(d.n_gblock, sl * per), b1 = min(d.n_gblock, b0 + per);
            const double* src = gram + d.gram_off + ent;
            const int64_t stride = nent;
            double v = 0.0;
            int b = b0;
            for (; b + 8 <= b1; b += 8) {   // eight loads in flight, added in block order
                double x[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) x[u] = src[(int64_t)(b + u) * stride];
#pragma unroll
                for (int u = 0; u < 8; ++u) v += x[u];
            }
            for (; b < b1; ++b) v += src[(int64_t)b * stride];
            part[sl][ent] = v;
        }
    }
    __syncthreads();
    if (tid < nent) {   // one thread per entry adds the slices, in slice order
        double v = 0.0;
        for (int sl = 0; sl < nslices; ++sl) v += part[sl][tid];
        Gs[tid] = v;
    }
    __syncthreads();
    if (tid == 0) {
        // Every index below is a compile-time constant (loops unrolled to the largest rank, rows and columns
        // past r switched off by predicates), so the matrix lives in registers; R overwrites G's upper triangle.
        double G[kValuMaxRank][kValuMaxRank];
#pragma unroll
        for (int a = 0; a < kValuMaxRank; ++a)
#pragma unroll
            for (int b = a; b < kValuMaxRank; ++b) G[a][b] = b < r ? Gs[a * r + b] : 0.0;
        // Cholesky, row by row of R (upper): R_jj = sqrt(G_jj - sum_k R_kj^2), R_jc = (G_jc - sum_k R_kj R_kc) / R_jj
#pragma unroll
        for (int j = 0; j < kValuMaxRank; ++j) {
            if (j < r) {
                double piv = G[j][j];
#pragma unroll
                for (int k = 0; k < j; ++k) piv -= G[k][j] * G[k][j];
                const bool dead = piv <= 1e-30;
                const double rjj = dead ? 0.0 : sqrt(piv);
                const double rj = dead ? 0.0 : 1.0 / rjj;
                rinv[j] = rj;
                G[j][j] = rjj;
                Rm[j][j] = rjj;
#pragma unroll
                for (int c = j + 1; c < kValuMaxRank; ++c) {
                    double v = G[j][c];
#pragma unroll
                    for (int k = 0; k < j; ++k) v -= G[k][j] * G[k][c];
                    v = dead ? 0.0 : v * rj;     // a zero column takes no part in the later ones
                    G[j][c] = v;
                    if (c < r) Rm[j][c] = v;
                }
            }
        }
    }
    __syncthreads();
    for (int i = t.row0 + tid; i < t.row0 + t.nrows; i += kBlock) {
        float* row = p + d.p_off + (int64_t)i * r;
        double ph[kValuMaxRank];
#pragma unroll
        for (int j = 0; j < kValuMaxRank; ++j) {
            if (j < r) {
                double v = (double)row[j];
#pragma unroll
                for (int k = 0; k < kValuMaxRank; ++k)
                    if (k < j) v -= ph[k] * Rm[k][j];
                ph[j] = v * rinv[j];
            } else {
                ph[j] = 0.0;
            }
        }
#pragma unroll
        for (int j = 0; j < kValuMaxRank; ++j)
            if (j < r) row[j] = (float)ph[j];
    }
}

// ---- k_gram_chol: k_gram and k_chol_apply in one launch ----------------------------------------------------
//
// One workgroup per row block (at most kGramRows = kBlock rows, one per thread), as in the pair above, and the same
// sums in the same order: the results are bit-identical.  The block's Gram matrix goes to a plan-owned mailbox of
// {value, epoch} slots (two slots per double); the workgroup then collects the Gram matrices of all row blocks
// of its matrix, factorises the sum and solves for its own rows of P_hat, which never left the registers.  This
// saves a launch, a drain and refill of the machine, and the second reading of P.  The workgroups of a matrix wait
// for each other, so they must be co-resident (checked when the tables are uploaded); every wait is bounded.
template <int R>
__global__ __launch_bounds__(kBlock) void k_gram_chol(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                      const float* __restrict__ ws, float* __restrict__ p,
                                                      slot_t* __restrict__ mail_gram, unsigned* __restrict__ sync,
                                                      int workers, int pre_reduced, unsigned spin_limit) {
    constexpr int kMaxSlices = 16;
    constexpr int kAhead = 4;   // slots requested before the first is looked at
    constexpr int E = kValuMaxRank * kValuMaxRank;
    __shared__ double red[kWavesPerBlock][E];
    __shared__ double part[kMaxSlices][E];
    __shared__ double Gs[E];
    __shared__ double Rm[kValuMaxRank][kValuMaxRank];
    __shared__ double rinv[kValuMaxRank];
    unsigned epoch = 0;
    if ((threadIdx.x & (kWave - 1)) == 0) epoch = ld_dev(sync + res_sync_epoch());
    epoch = __builtin_amdgcn_readfirstlane(epoch);
    unsigned* err_word = sync + res_sync_err();
    const Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int r = d.r, tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6;
    const int64_t nr = (int64_t)d.n * r;
    const float inv_w = 1.0f / (float)workers;
    const int nparts = pre_reduced ? 1 : workers * d.n_cchunk;
    const int i = t.row0 + tid;
    const bool have = tid < t.nrows;

    float row[R];
    double g[R][R];
#pragma unroll
    for (int k = 0; k < R; ++k) row[k] = 0.f;
    if (have) {
        sum_parts_row<R>(ws + d.ppart_off + (int64_t)i * r, r, nparts, nr, row);
#pragma unroll
        for (int k = 0; k < R; ++k) row[k] *= inv_w;
    }
#pragma unroll
    for (int a = 0; a < R; ++a)
#pragma unroll
        for (int b = a; b < R; ++b) g[a][b] = (b < r && have) ? (double)row[a] * (double)row[b] : 0.0;
#pragma unroll
    for (int a = 0; a < R; ++a)
#pragma unroll
        for (int b = a; b < R; ++b)
            if (b < r) {
                const double v = wave_sum(g[a][b]);
                if (lane == 0) red[wave][a * kValuMaxRank + b] = v;
            }
    __syncthreads();
    const int nent = r * r;
    if (tid < nent) {
        const int a = tid / r, b = tid % r;
        double v = 0.0;
        if (b >= a)
            for (int wv = 0; wv < kWavesPerBlock; ++wv) v += red[wv][a * kValuMaxRank + b];
        post_double(mail_gram + 2 * (d.gram_off + (int64_t)t.part * nent + tid), v, epoch);   // upper triangle, zeros below
    }
    // The matrix's last row block sits furthest down the launch and tends to deliver last: one wavefront watches its
    // first slot with one lane, the others wait at a barrier, before all lanes fetch all blocks (polling everything
    // from the start costs more than it finds: 12 blocks requested at once instead of 4 made the kernel 10 % slower).
    if (wave == 0) await_tag(mail_gram + 2 * (d.gram_off + (int64_t)(d.n_gblock - 1) * nent), epoch, err_word, spin_limit);
    __syncthreads();
    // sum of all row blocks' matrices: consecutive slices of blocks (one lane per entry and slice), each added in
    // block order, then the slices in slice order
    const int per_wave = nent <= 16 ? 4 : (nent <= 32 ? 2 : 1);
    const int nslices = kWavesPerBlock * per_wave;
    {
        const int lanes_per = kWave / per_wave;
        const int ent = lane % lanes_per, sl = wave * per_wave + lane / lanes_per;
        if (ent < nent) {
            const int per = (d.n_gblock + nslices - 1) / nslices;
            const int b0 = min(d.n_gblock, sl * per), b1 = min(d.n_gblock, b0 + per);
            const slot_t* src = mail_gram + 2 * (d.gram_off + ent);
            const int64_t stride = 2 * (int64_t)nent;
            double v = 0.0;
            int b = b0;
            for (; b + kAhead <= b1; b += kAhead) {
                slot_t lo[kAhead], hi[kAhead];
#pragma unroll
                for (int u = 0; u < kAhead; ++u) {
                    lo[u] = fetch(src + (int64_t)(b + u) * stride);
                    hi[u] = fetch(src + (int64_t)(b + u) * stride + 1);
                }
#pragma unroll
                for (int u = 0; u < kAhead; ++u) v += take_double(src + (int64_t)(b + u) * stride, lo[u], hi[u], epoch, err_word, spin_limit);
            }
            for (; b < b1; ++b) {
                const slot_t* s2 = src + (int64_t)b * stride;
                v += take_double(s2, fetch(s2), fetch(s2 + 1), epoch, err_word, spin_limit);
            }
            part[sl][ent] = v;
        }
    }
    __syncthreads();
    if (tid < nent) {   // one thread per entry adds the slices, in slice order
        double v = 0.0;
        for (int sl = 0; sl < nslices; ++sl) v += part[sl][tid];
        Gs[tid] = v;
    }
    __syncthreads();
    if (tid == 0) {
        double G[R][R];
#pragma unroll
        for (int a = 0; a < R; ++a)
#pragma unroll
            for (int b = a; b < R; ++b) G[a][b] = b < r ? Gs[a * r + b] : 0.0;
        // Cholesky, row by row of R (upper): R_jj = sqrt(G_jj - sum_k R_kj^2), R_jc = (G_jc - sum_k R_kj R_kc) / R_jj
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if (j < r) {
                double piv = G[j][j];
#pragma unroll
                for (int k = 0; k < j; ++k) piv -= G[k][j] * G[k][j];
                const bool dead = piv <= 1e-30;
                const double rjj = dead ? 0.0 : sqrt(piv);
                const double rj = dead ? 0.0 : 1.0 / rjj;
                rinv[j] = rj;
                G[j][j] = rjj;
                Rm[j][j] = rjj;
#pragma unroll
                for (int c = j + 1; c < R; ++c) {
                    double v = G[j][c];
#pragma unroll
                    for (int k = 0; k < j; ++k) v -= G[k][j] * G[k][c];
                    v = dead ? 0.0 : v * rj;     // a zero column takes no part in the later ones
                    G[j][c] = v;
                    if (c < r) Rm[j][c] = v;
                }
            }
        }
    }
    __syncthreads();
    if (have) {
        double ph[R];
#pragma unroll
        for (int j = 0; j < R; ++j) {
            if (j < r) {
                double v = (double)row[j];
#pragma unroll
                for (int k = 0; k < R; ++k)
                    if (k < j) v -= ph[k] * Rm[k][j];
                ph[j] = v * rinv[j];
            } else {
                ph[j] = 0.0;
            }
        }
#pragma unroll
        for (int j = 0; j < R; ++j)
            if (j < r) p[d.p_off + (int64_t)i * r + j] = (float)ph[j];
    }
    // the workgroup that finishes last advances the epoch for the next launch
    __syncthreads();
    if (tid == 0) {
        unsigned* done = sync + res_sync_done();
        if (add_dev(done, 1u) == gridDim.x - 1u) {
            add_dev(done, 0u - gridDim.x);
            st_dev(sync + res_sync_epoch(), epoch + 1u);
        }
    }
}

// ---- k_left: Q_w[j,:] = sum_i M[i,j] P_hat[i,:] ---------------------------------------------------
//
// A lane owns NV column vectors and keeps their V*R running sums in registers while its
// wavefront walks down a strip of rows.  The P_hat rows of a 64-row group are loaded one
// row per lane and broadcast with readlane.  The four wavefronts of a workgroup walk four
// strips of the same columns; their sums are added in LDS in a fixed order and written as
// one partial per (row block, worker).

// STREAM: M is larger than the memory-side cache and will not be found there by the next sweep either way; reading it
// with non-temporal loads keeps it from pushing out lines that are still waiting to be written back.
template <int R, int V, int NV, bool STREAM>
__device__ __forceinline__ void left_tile(const Tile& t, const MatDesc& d, const float* __restrict__ e,
                                          const float* __restrict__ p, float* __restrict__ qpart, float* lds) {
    constexpr int RU = 8;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ri = d.r;
    float acc[NV][V][R];
    bool valid[NV];
    int col[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int jv = lane + kWave * v;
        valid[v] = jv < t.nvec;
        col[v] = (t.vec0 + jv) * V;
#pragma unroll
        for (int x = 0; x < V; ++x)
#pragma unroll
            for (int k = 0; k < R; ++k) acc[v][x][k] = 0.f;
    }
    int rb, rn;
    wave_rows(t.nrows, wave, &rb, &rn);
    // descriptor over the rows of this wavefront's strip: missing columns carry an out-of-range offset, rows past
    // the strip lie beyond the range; both read zeros (and zero rows of P_hat), so nothing sits behind a branch
    const buf_rsrc eres = make_rsrc(e + d.off + (int64_t)(t.row0 + rb) * d.m, (int64_t)rn * d.m * 4);
    unsigned coff[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) coff[v] = valid[v] ? (unsigned)col[v] * 4u : kOutOfRange;
    for (int g0 = 0; g0 < rn; g0 += kWave) {
        const int gr = min(kWave, rn - g0);
        const int i0 = t.row0 + rb + g0;
        float pr1[1][R];
        load_factor_rows<R, 1>(p + d.p_off + (int64_t)(i0 + lane) * ri, ri, lane < gr, pr1);
        float (&pr)[R] = pr1[0];
        for (int ii = 0; ii < gr; ii += RU) {
            float x[RU][NV][V];
            const unsigned row_off = (unsigned)(g0 + ii) * (unsigned)d.m * 4u;
#pragma unroll
            for (int u = 0; u < RU; ++u)
#pragma unroll
                for (int v = 0; v < NV; ++v) buf_ldv<V>(eres, coff[v] + row_off + (unsigned)u * (unsigned)d.m * 4u, x[u][v], STREAM);
#pragma unroll
            for (int u = 0; u < RU; ++u) {
                float pk[R];   // lanes at or past gr hold zeros: rows past the group contribute nothing
#pragma unroll
                for (int k = 0; k < R; ++k) pk[k] = lane_bcast(pr[k], min(ii + u, kWave - 1));
#pragma unroll
                for (int v = 0; v < NV; ++v)
#pragma unroll
                    for (int xx = 0; xx < V; ++xx)
#pragma unroll
                        for (int k = 0; k < R; ++k) acc[v][xx][k] = fmaf(x[u][v][xx], pk[k], acc[v][xx][k]);
            }
        }
    }
    // fixed-order sum over the 4 wavefronts: 1, 2, 3 deposit, 0 adds them in that order
    constexpr int PER_LANE = NV * V * R;
    if (wave > 0) {
        float* dst = lds + ((wave - 1) * kWave + lane) * PER_LANE;
#pragma unroll
        for (int v = 0; v < NV; ++v)
#pragma unroll
            for (int x = 0; x < V; ++x)
#pragma unroll
                for (int k = 0; k < R; ++k) dst[(v * V + x) * R + k] = acc[v][x][k];
    }
    __syncthreads();
    if (wave == 0) {
        for (int wv = 0; wv < kWavesPerBlock - 1; ++wv) {
            const float* src = lds + (wv * kWave + lane) * PER_LANE;
#pragma unroll
            for (int v = 0; v < NV; ++v)
#pragma unroll
                for (int x = 0; x < V; ++x)
#pragma unroll
                    for (int k = 0; k < R; ++k) acc[v][x][k] += src[(v * V + x) * R + k];
        }
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            if (valid[v]) {
                float* dst = qpart + d.qpart_off + ((int64_t)t.part * d.m + col[v]) * ri;
#pragma unroll
                for (int x = 0; x < V; ++x)
#pragma unroll
                    for (int k = 0; k < R; ++k)
                        if (k < ri) dst[x * ri + k] = acc[v][x][k];
            }
        }
    }
}

template <int R, int NV, bool STREAM>
__global__ __launch_bounds__(kBlock) void k_left(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                 const float* __restrict__ err, const float* __restrict__ p,
                                                 float* __restrict__ ws, int64_t estride) {
    __shared__ float lds[(kWavesPerBlock - 1) * kWave * NV * 4 * R];
    Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int w = blockIdx.y;
    const float* e = err + (int64_t)w * estride;
    float* qp = ws;
    t.part += w * d.n_rblock;   // partial slices: [worker][row block]
    if (d.vec == 4) left_tile<R, 4, NV, STREAM>(t, d, e, p, qp, lds);
    else if (d.vec == 2) left_tile<R, 2, NV, STREAM>(t, d, e, p, qp, lds);
    else left_tile<R, 1, NV, STREAM>(t, d, e, p, qp, lds);
}

// ---- k_q_reduce: Q = (1/W) sum over workers and row blocks of the partials ------------------------

// 64 elements per workgroup; wavefront g adds slice g of the partials (slice order), then the four slices
// are added in slice order.  for_p = 0: partial Q -> Q (mean over workers).  for_p = 1: partial P -> first
// partial slice (plain sum; used when there are many slices, so that the orthogonalisation reads one).
__global__ __launch_bounds__(kBlock) void k_q_reduce(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                     float* __restrict__ ws, float* __restrict__ q, int workers,
                                                     int for_p) {
    __shared__ float part[kWavesPerBlock][kWave];
    const Tile t = tiles[blockIdx.x];
    const MatDesc d = mats[t.mat];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    const int64_t stride = for_p ? (int64_t)d.n * d.r : (int64_t)d.m * d.r;
    const int nparts = workers * (for_p ? d.n_cchunk : d.n_rblock);
    float* src = ws + (for_p ? d.ppart_off : d.qpart_off);
    const int per = (nparts + kWavesPerBlock - 1) / kWavesPerBlock;
    const int b0 = min(nparts, wave * per), b1 = min(nparts, b0 + per);
    float s = 0.f;
    if (lane < t.nelem) s = sum_parts(src + (int64_t)b0 * stride + t.elem0 + lane, b1 - b0, stride);
    part[wave][lane] = s;
    __syncthreads();   // every slice of these 64 elements has been read before slice 0 is overwritten
    if (wave == 0 && lane < t.nelem) {
        const float v = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
        if (for_p) src[t.elem0 + lane] = v;
        else q[d.q_off + t.elem0 + lane] = v * (1.0f / (float)workers);
    }
}

// ---- k_decomp: Delta' = P_hat Q^T, e_w = M_w - Delta', vectors averaged ---------------------------

// STREAM (see left_tile): M is read with non-temporal loads and the new error memory written with non-temporal stores;
// otherwise it is Delta' that is written with non-temporal stores
// OBF: Delta' is stored as bf16
template <int R, int V, int NV, bool UPD, bool STREAM, bool OBF>
__device__ __forceinline__ void decomp_tile(const Tile& t, const MatDesc& d, float* __restrict__ e,
                                            const float* __restrict__ p, const float* __restrict__ q,
                                            void* __restrict__ out, bool write_out, const UpdateArgs& upd) {
    constexpr int RU = UPD ? 4 : 8;   // rows whose loads are in flight together (momentum and parameters ride along)
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ri = d.r;
    float qr[NV][V][R];
    bool valid[NV];
    int col[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int jv = lane + kWave * v;
        valid[v] = jv < t.nvec;
        col[v] = (t.vec0 + jv) * V;
        load_factor_rows<R, V>(q + d.q_off + (int64_t)col[v] * ri, ri, valid[v], qr[v]);
    }
    int rb, rn;
    wave_rows(t.nrows, wave, &rb, &rn);
    for (int g0 = 0; g0 < rn; g0 += kWave) {
        const int gr = min(kWave, rn - g0);
        const int i0 = t.row0 + rb + g0;
        float pr1[1][R];
        load_factor_rows<R, 1>(p + d.p_off + (int64_t)(i0 + lane) * ri, ri, lane < gr, pr1);
        float (&pr)[R] = pr1[0];
        for (int ii = 0; ii < gr; ii += RU) {
            float x[RU][NV][V];
            float mo[UPD ? RU : 1][NV][V], pa[UPD ? RU : 1][NV][V];
#pragma unroll
            for (int u = 0; u < RU; ++u) {
                if (ii + u < gr) {
                    const int64_t row = d.off + (int64_t)(i0 + ii + u) * d.m;
#pragma unroll
                    for (int v = 0; v < NV; ++v)
                        if (valid[v]) {
                            if constexpr (STREAM) ldv_stream<V>(e + row + col[v], x[u][v]);
                            else ldv<V>(e + row + col[v], x[u][v]);
                            if constexpr (UPD) {
                                if (write_out) {
                                    ldv<V>(upd.mom + row + col[v], mo[u][v]);
                                    ldv<V>(upd.param + row + col[v], pa[u][v]);
                                }
                            }
                        }
                }
            }
#pragma unroll
            for (int u = 0; u < RU; ++u) {
                if (ii + u < gr) {
                    const int64_t row = d.off + (int64_t)(i0 + ii + u) * d.m;
                    float pk[R];
#pragma unroll
                    for (int k = 0; k < R; ++k) pk[k] = lane_bcast(pr[k], ii + u);
#pragma unroll
                    for (int v = 0; v < NV; ++v)
                        if (valid[v]) {
                            float dl[V], en[V];
#pragma unroll
                            for (int xx = 0; xx < V; ++xx) {
                                float s = 0.f;
#pragma unroll
                                for (int k = 0; k < R; ++k) s = fmaf(pk[k], qr[v][xx][k], s);
                                dl[xx] = s;
                                en[xx] = x[u][v][xx] - s;
                            }
                            if constexpr (STREAM) stv_stream<V>(e + row + col[v], en);
                            else stv<V>(e + row + col[v], en);
                            if (write_out) {
                                if constexpr (UPD) {
                                    momentum_step<V>(mo[u][v], pa[u][v], dl, upd.lr, upd.lam);
                                    stv<V>(upd.mom + row + col[v], mo[u][v]);
                                    stv<V>(upd.param + row + col[v], pa[u][v]);
                                } else {
                                    // a set that fits the memory-side cache: Delta' goes around it, M and e' stay
                                    st_out<V, OBF, !STREAM>(out, row + col[v], dl);
                                }
                            }
                        }
                }
            }
        }
    }
}

// The slices of the vector region are handled here when gradients and output are fp32 (`grad`, `outv` typed
// accordingly); with bf16 data a kernel of its own does them and vec_here is 0.
template <int R, int NV, bool UPD, bool STREAM, bool OBF>
__global__ __launch_bounds__(kBlock) void k_decomp(const MatDesc* __restrict__ mats, const Tile* __restrict__ tiles,
                                                   float* __restrict__ err, const float* __restrict__ p,
                                                   const float* __restrict__ q, const float* __restrict__ grad,
                                                   void* __restrict__ outv, int workers, int64_t gstride,
                                                   int64_t estride, int64_t n_mat_elems, UpdateArgs upd, int vec_here) {
    const Tile t = tiles[blockIdx.x];
    const int w = blockIdx.y;
    if (t.mat < 0) {
        if (w != 0 || !vec_here) return;
        float* out = static_cast<float*>(outv);
        const float inv_w = 1.0f / (float)workers;
        for (int64_t idx = t.elem0 + threadIdx.x; idx < t.elem0 + t.nelem; idx += kBlock) {
            float s = 0.f;
            for (int ww = 0; ww < workers; ++ww) s += grad[(int64_t)ww * gstride + n_mat_elems + idx];
            if constexpr (UPD) {
                float m1[1] = {upd.mom[n_mat_elems + idx]}, x1[1] = {upd.param[n_mat_elems + idx]};
                const float d1[1] = {s * inv_w};
                momentum_step<1>(m1, x1, d1, upd.lr, upd.lam);
                upd.mom[n_mat_elems + idx] = m1[0];
                upd.param[n_mat_elems + idx] = x1[0];
            } else {
                out[n_mat_elems + idx] = s * inv_w;
            }
        }
        return;
    }
    const MatDesc d = mats[t.mat];
    float* e = err + (int64_t)w * estride;
    if (d.vec == 4) decomp_tile<R, 4, NV, UPD, STREAM, OBF>(t, d, e, p, q, outv, w == 0, upd);
    else if (d.vec == 2) decomp_tile<R, 2, NV, UPD, STREAM, OBF>(t, d, e, p, q, outv, w == 0, upd);
    else decomp_tile<R, 1, NV, UPD, STREAM, OBF>(t, d, e, p, q, outv, w == 0, upd);
}

// ---- host side ------------------------------------------------------------------------------------

// Workspace owned by the library, for callers that cannot allocate (psgd_step_static): one array per GPU, part of
// the loaded code object, held until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; its device address differs from GPU to GPU and is looked up once per device, with that
// device current, when a plan's tables are uploaded there.
static __device__ __align__(256) unsigned char scratch[PSGD_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};   // device address of `scratch` on each GPU (nullptr: not looked up yet)
static std::mutex g_scratch_mutex;

static hipError_t scratch_address(int device, void** out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));   // the current device's copy
        if (e != hipSuccess) return e;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return hipSuccess;
}

static psgd_status hip_fail(psgd_plan* plan, hipError_t err, const char* what) {
    plan->last_error = std::string(what) + ": " + hipGetErrorString(err);
    return err == hipErrorOutOfMemory ? PSGD_ENOMEM : PSGD_EHIP;
}

#define PSGD_HIP(call, what)                                   \
    do {                                                       \
        hipError_t e_ = (call);                                \
        if (e_ != hipSuccess) return hip_fail(plan, e_, what); \
    } while (0)

psgd_status set_profiling(psgd_plan* plan, bool enable) {
    if (enable == plan->profiling) return PSGD_OK;
    if (enable) {
        for (auto& ev : plan->events) {
            hipEvent_t e = nullptr;
            PSGD_HIP(hipEventCreate(&e), "hipEventCreate");
            ev = e;
        }
    } else {
        for (auto& ev : plan->events) {
            if (ev) (void)hipEventDestroy(static_cast<hipEvent_t>(ev));
            ev = nullptr;
        }
    }
    plan->profiling = enable;
    plan->compress_marked = false;
    return PSGD_OK;
}

#define PSGD_MARK(i)                                                                                \
    do {                                                                                            \
        if (plan->profiling) PSGD_HIP(hipEventRecord(static_cast<hipEvent_t>(plan->events[i]), s), "hipEventRecord"); \
    } while (0)

void free_tables(psgd_plan* plan) {
    (void)set_profiling(plan, false);
    if (plan->dev.base) {
        (void)hipFree(plan->dev.base);
        plan->dev = DeviceTables();
    }
    plan->uploaded = false;
}

// k_gram_chol: the row blocks of a matrix wait for each other, so the one-launch form is taken only when the whole
// grid fits the device at once (no assumption about the order in which workgroups are started).
static psgd_status gram_fused_check_device(psgd_plan* plan) {
    plan->gram_fused = false;
    if (plan->hr || !plan->tuning.gram_fused || plan->tiles_gram.empty()) return PSGD_OK;
    int dev = 0, cus = 0, occ = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PSGD_EHIP;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return PSGD_EHIP;
    hipError_t e = hipErrorInvalidValue;
    switch (plan->rank) {
        case 1: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_gram_chol<1>, kBlock, 0); break;
        case 2: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_gram_chol<2>, kBlock, 0); break;
        case 3: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_gram_chol<3>, kBlock, 0); break;
        case 4: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_gram_chol<4>, kBlock, 0); break;
        case 5: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_gram_chol<5>, kBlock, 0); break;
        case 6: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_gram_chol<6>, kBlock, 0); break;
        case 7: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_gram_chol<7>, kBlock, 0); break;
        case 8: e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_gram_chol<8>, kBlock, 0); break;
        default: break;
    }
    if (e != hipSuccess) return hip_fail(plan, e, "occupancy(k_gram_chol)");
    // gram_fused = 2 skips the test (diagnostic: lets a test see the waits time out)
    plan->gram_fused = plan->tuning.gram_fused == 2 || (int64_t)cus * occ >= (int64_t)plan->tiles_gram.size();
    return PSGD_OK;
}

psgd_status upload_tables(psgd_plan* plan) {
    if (plan->uploaded) return PSGD_OK;
    PSGD_HIP(hipGetDevice(&plan->device), "hipGetDevice");
    PSGD_HIP(scratch_address(plan->device, &plan->static_ws), "hipGetSymbolAddress(static workspace)");
    if (!plan->hr && plan->tuning.resident) {   // lays the resident tiling out for this device
        psgd_status st = resident_check_device(plan);
        if (st != PSGD_OK) return st;
    }
    {
        psgd_status st = gram_fused_check_device(plan);
        if (st != PSGD_OK) return st;
    }
    struct Piece { const void* src; size_t bytes; size_t at; };
    Piece pieces[23] = {
        {plan->mats.data(), plan->mats.size() * sizeof(MatDesc), 0},
        {plan->tiles1.data(), plan->tiles1.size() * sizeof(Tile), 0},
        {plan->tiles3.data(), plan->tiles3.size() * sizeof(Tile), 0},
        {plan->tiles4.data(), plan->tiles4.size() * sizeof(Tile), 0},
        {plan->tilesq.data(), plan->tilesq.size() * sizeof(Tile), 0},
        {plan->res_mats.data(), plan->res_mats.size() * sizeof(MatDesc), 0},
        {plan->res_tiles.data(), plan->res_tiles.size() * sizeof(RTile), 0},
        {nullptr, (size_t)plan->res_sync_words * sizeof(unsigned), 0},   // zero-filled, epoch set below
        {nullptr, plan->tuning.res_trace ? (size_t)plan->res_blocks * kWavesPerBlock * kResTracePoints * sizeof(unsigned long long) : 0, 0},
        {nullptr, (size_t)plan->res_mail_slots * sizeof(unsigned long long), 0},   // zero-filled: tag 0 never matches
        {plan->tiles_gram.data(), plan->tiles_gram.size() * sizeof(Tile), 0},
        {plan->small_mats.data(), plan->small_mats.size() * sizeof(int32_t), 0},
        {plan->tilesp.data(), plan->tilesp.size() * sizeof(Tile), 0},
        {plan->hr_tiles1.data(), plan->hr_tiles1.size() * sizeof(Tile), 0},
        {plan->hr_tiles3.data(), plan->hr_tiles3.size() * sizeof(Tile), 0},
        {plan->hr_tiles4.data(), plan->hr_tiles4.size() * sizeof(Tile), 0},
        {nullptr, plan->gram_fused ? (size_t)kResSyncWords * sizeof(unsigned) : 0, 0},                   // zero-filled, epoch set below
        {nullptr, plan->gram_fused ? (size_t)plan->ws_gram_doubles * 2 * sizeof(unsigned long long) : 0, 0},   // zero-filled: tag 0 never matches
        {plan->tiles4u.data(), plan->tiles4u.size() * sizeof(Tile), 0},
        {plan->flat_first.data(), plan->flat_first.size() * sizeof(int64_t), 0},
        {plan->kept_slice_mat.data(), plan->kept_slice_mat.size() * sizeof(int32_t), 0},
        {plan->kept_slice_first.data(), plan->kept_slice_first.size() * sizeof(int64_t), 0},
        {plan->mat_tensor.data(), plan->mat_tensor.size() * sizeof(int32_t), 0},
    };
    size_t total = 0;
    for (Piece& pc : pieces) {
        pc.at = total;
        total += (pc.bytes + 255) / 256 * 256;
    }
    total += 256;
    std::vector<char> host(total, 0);
    for (const Piece& pc : pieces)
        if (pc.src && pc.bytes) std::memcpy(host.data() + pc.at, pc.src, pc.bytes);
    if (plan->res_sync_words) {
        const unsigned one = 1;   // epochs start at 1
        std::memcpy(host.data() + pieces[7].at + res_sync_epoch() * sizeof(unsigned), &one, sizeof(one));
    }
    if (plan->gram_fused) {
        const unsigned one = 1;   // epochs start at 1
        std::memcpy(host.data() + pieces[16].at + res_sync_epoch() * sizeof(unsigned), &one, sizeof(one));
    }
    void* base = nullptr;
    PSGD_HIP(hipMalloc(&base, total), "hipMalloc(descriptor tables)");
    hipError_t ce = hipMemcpy(base, host.data(), total, hipMemcpyHostToDevice);
    if (ce != hipSuccess) {
        (void)hipFree(base);
        return hip_fail(plan, ce, "hipMemcpy(descriptor tables)");
    }
    char* b = static_cast<char*>(base);
    plan->dev.base = base;
    plan->dev.mats = reinterpret_cast<MatDesc*>(b + pieces[0].at);
    plan->dev.tiles1 = reinterpret_cast<Tile*>(b + pieces[1].at);
    plan->dev.tiles3 = reinterpret_cast<Tile*>(b + pieces[2].at);
    plan->dev.tiles4 = reinterpret_cast<Tile*>(b + pieces[3].at);
    plan->dev.tilesq = reinterpret_cast<Tile*>(b + pieces[4].at);
    plan->dev.res_mats = reinterpret_cast<MatDesc*>(b + pieces[5].at);
    plan->dev.res_tiles = reinterpret_cast<RTile*>(b + pieces[6].at);
    plan->dev.res_sync = reinterpret_cast<unsigned*>(b + pieces[7].at);
    plan->dev.res_trace = pieces[8].bytes ? reinterpret_cast<unsigned long long*>(b + pieces[8].at) : nullptr;
    plan->dev.res_mail = reinterpret_cast<unsigned long long*>(b + pieces[9].at);
    plan->dev.tiles_gram = reinterpret_cast<Tile*>(b + pieces[10].at);
    plan->dev.small_mats = reinterpret_cast<int32_t*>(b + pieces[11].at);
    plan->dev.tilesp = reinterpret_cast<Tile*>(b + pieces[12].at);
    plan->dev.hr_tiles1 = reinterpret_cast<Tile*>(b + pieces[13].at);
    plan->dev.hr_tiles3 = reinterpret_cast<Tile*>(b + pieces[14].at);
    plan->dev.hr_tiles4 = reinterpret_cast<Tile*>(b + pieces[15].at);
    plan->dev.gram_sync = plan->gram_fused ? reinterpret_cast<unsigned*>(b + pieces[16].at) : nullptr;
    plan->dev.gram_mail = plan->gram_fused ? reinterpret_cast<unsigned long long*>(b + pieces[17].at) : nullptr;
    plan->dev.tiles4u = plan->tiles4u.empty() ? nullptr : reinterpret_cast<Tile*>(b + pieces[18].at);
    plan->dev.flat_first = reinterpret_cast<int64_t*>(b + pieces[19].at);
    plan->dev.kept_slice_mat = reinterpret_cast<int32_t*>(b + pieces[20].at);
    plan->dev.kept_slice_first = reinterpret_cast<int64_t*>(b + pieces[21].at);
    plan->dev.mat_tensor = reinterpret_cast<int32_t*>(b + pieces[22].at);
    plan->uploaded = true;
    return PSGD_OK;
}

psgd_status read_trace(psgd_plan* plan, uint64_t* out, int64_t capacity, int64_t* n_written) {
    *n_written = 0;
    if (!plan->uploaded || !plan->dev.res_trace) return PSGD_OK;
    const int64_t n = std::min<int64_t>(capacity, (int64_t)plan->res_blocks * kWavesPerBlock * kResTracePoints);
    PSGD_HIP(hipDeviceSynchronize(), "hipDeviceSynchronize");
    PSGD_HIP(hipMemcpy(out, plan->dev.res_trace, (size_t)n * sizeof(uint64_t), hipMemcpyDeviceToHost), "hipMemcpy(trace)");
    *n_written = n;
    return PSGD_OK;
}

// The library-owned workspace of the device the plan lives on, for a plan whose tables are there already and whose
// workspace fits it; nothing is allocated here.
psgd_status static_workspace(psgd_plan* plan, void** ws) {
    if (!plan->uploaded || !plan->static_ws) {
        plan->last_error = "psgd_step_static: the plan's tables are not on the device yet (psgd_plan_check, or any "
                           "other GPU call on the plan, uploads them; that first call allocates)";
        return PSGD_EINVAL;
    }
    if (plan->sizes.workspace_bytes > (int64_t)PSGD_STATIC_WORKSPACE_BYTES) {
        plan->last_error = "psgd_step_static: the plan needs " + std::to_string(plan->sizes.workspace_bytes) +
                           " bytes of workspace, the library-owned one holds " +
                           std::to_string((long long)PSGD_STATIC_WORKSPACE_BYTES);
        return PSGD_EUNSUPPORTED;
    }
    int dev = -1;
    PSGD_HIP(hipGetDevice(&dev), "hipGetDevice");
    if (dev != plan->device) {
        plan->last_error = "psgd_step_static: the current device is not the one the plan's tables were uploaded to";
        return PSGD_EINVAL;
    }
    *ws = plan->static_ws;
    return PSGD_OK;
}

// Waits for the stream; reports a wait that gave up in one of the kernels whose workgroups wait for each other,
// resets that kernel's hand-over words and switches its mode off for the rest of the plan's life: the step then
// runs on the kernels that need no co-residency (streaming sweeps; Gram matrices and factorisation in two launches).
psgd_status check_plan(psgd_plan* plan, void* stream) {
    if (!plan->uploaded) return upload_tables(plan);   // nothing has run yet: just bring the tables to the device
    PSGD_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)), "hipStreamSynchronize");
    if (plan->gram_fused && plan->dev.gram_sync) {
        unsigned flag = 0;
        PSGD_HIP(hipMemcpy(&flag, plan->dev.gram_sync + res_sync_err(), sizeof(flag), hipMemcpyDeviceToHost),
                 "hipMemcpy(error word)");
        if (flag) {
            // start over: empty mailbox, epoch 1, no finished workgroups
            PSGD_HIP(hipMemset(plan->dev.gram_mail, 0, (size_t)plan->ws_gram_doubles * 2 * sizeof(unsigned long long)),
                     "hipMemset(mailbox)");
            PSGD_HIP(hipMemset(plan->dev.gram_sync, 0, (size_t)kResSyncWords * sizeof(unsigned)), "hipMemset(sync words)");
            const unsigned one = 1;
            PSGD_HIP(hipMemcpy(plan->dev.gram_sync + res_sync_epoch(), &one, sizeof(one), hipMemcpyHostToDevice),
                     "hipMemcpy(epoch)");
            if (plan->tuning.gram_fused != 2) plan->gram_fused = false;   // 2: the diagnostic setting keeps the mode
            plan->last_error = "k_gram_chol: a wait timed out (row blocks not co-resident: is the GPU shared?); "
                               "the plan continues with the two-launch factorisation";
            return PSGD_EHIP;
        }
    }
    if (!plan->resident_ok || !plan->res_sync_words) return PSGD_OK;
    unsigned flag = 0;
    PSGD_HIP(hipMemcpy(&flag, plan->dev.res_sync + res_sync_err(), sizeof(flag), hipMemcpyDeviceToHost),
             "hipMemcpy(barrier error word)");
    if (flag) {
        // start over: empty mailbox, epoch 1, no finished workgroups
        PSGD_HIP(hipMemset(plan->dev.res_mail, 0, (size_t)plan->res_mail_slots * sizeof(unsigned long long)),
                 "hipMemset(mailbox)");
        PSGD_HIP(hipMemset(plan->dev.res_sync, 0, (size_t)plan->res_sync_words * sizeof(unsigned)),
                 "hipMemset(sync words)");
        const unsigned one = 1;
        PSGD_HIP(hipMemcpy(plan->dev.res_sync + res_sync_epoch(), &one, sizeof(one), hipMemcpyHostToDevice),
                 "hipMemcpy(epoch)");
        plan->resident_ok = false;
        plan->last_error = "resident kernel: a wait timed out (grid not co-resident: is the GPU shared?); "
                           "the plan continues on the streaming kernels";
        return PSGD_EHIP;
    }
    return PSGD_OK;
}

template <int R>
static void launch_ef_right(psgd_plan* plan, const void* grad, float* err, const float* q, float* ws,
                            hipStream_t s, bool add) {
    dim3 grid((unsigned)plan->tiles1.size(), (unsigned)plan->workers);
#define PSGD_LAUNCH_RIGHT(NVV, ADDV, GBFV)                                                                             \
    hipLaunchKernelGGL((k_ef_right<R, NVV, ADDV, GBFV>), grid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.tiles1,   \
                       grad, err, q, ws, plan->sizes.grad_stride, plan->sizes.err_stride)
    if (!add) {   // the gradient is not read
        if (plan->tuning.k1_nv == 1) PSGD_LAUNCH_RIGHT(1, false, false);
        else PSGD_LAUNCH_RIGHT(2, false, false);
    } else if (plan->grad_dtype == PSGD_BF16) {
        if (plan->tuning.k1_nv == 1) PSGD_LAUNCH_RIGHT(1, true, true);
        else PSGD_LAUNCH_RIGHT(2, true, true);
    } else {
        if (plan->tuning.k1_nv == 1) PSGD_LAUNCH_RIGHT(1, true, false);
        else PSGD_LAUNCH_RIGHT(2, true, false);
    }
#undef PSGD_LAUNCH_RIGHT
}

template <int R>
static void launch_left(psgd_plan* plan, const float* err, const float* p, float* ws, hipStream_t s) {
    dim3 grid((unsigned)plan->tiles3.size(), (unsigned)plan->workers);
#define PSGD_LAUNCH_LEFT(NVV, STREAMV)                                                                                 \
    hipLaunchKernelGGL((k_left<R, NVV, STREAMV>), grid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.tiles3, err, p, ws, \
                       plan->sizes.err_stride)
    if (plan->stream_hints) {
        if (plan->tuning.k3_nv == 1) PSGD_LAUNCH_LEFT(1, true);
        else PSGD_LAUNCH_LEFT(2, true);
    } else {
        if (plan->tuning.k3_nv == 1) PSGD_LAUNCH_LEFT(1, false);
        else PSGD_LAUNCH_LEFT(2, false);
    }
#undef PSGD_LAUNCH_LEFT
}

template <int R>
static void launch_decomp(psgd_plan* plan, float* err, const float* p, const float* q, const void* grad, void* out,
                          hipStream_t s, const UpdateArgs& upd) {
    // fused with the update: tiles of its own where the planner made some
    const bool own_tiles = upd.mom && plan->dev.tiles4u;
    const Tile* tiles = own_tiles ? plan->dev.tiles4u : plan->dev.tiles4;
    dim3 grid((unsigned)(own_tiles ? plan->tiles4u.size() : plan->tiles4.size()), (unsigned)plan->workers);
    // bf16 gradients or output: the vector region has a kernel of its own
    const int vec_here = plan->grad_dtype == PSGD_F32 && plan->out_dtype == PSGD_F32 ? 1 : 0;
#define PSGD_LAUNCH_DECOMP(NVV, UPDV, STREAMV, OBFV)                                                                    \
    hipLaunchKernelGGL((k_decomp<R, NVV, UPDV, STREAMV, OBFV>), grid, dim3(kBlock), 0, s, plan->dev.mats,               \
                       tiles, err, p, q, static_cast<const float*>(grad), out, plan->workers,                           \
                       plan->sizes.grad_stride, plan->sizes.err_stride, plan->sizes.n_mat_elems, upd, vec_here)
#define PSGD_LAUNCH_DECOMP_NV(UPDV, STREAMV)                                     \
    do {                                                                         \
        if (plan->tuning.k4_nv == 1) PSGD_LAUNCH_DECOMP(1, UPDV, STREAMV, false); \
        else PSGD_LAUNCH_DECOMP(2, UPDV, STREAMV, false);                        \
    } while (0)
    if (upd.mom) {   // Delta' is not stored
        if (plan->stream_hints) PSGD_LAUNCH_DECOMP_NV(true, true);
        else PSGD_LAUNCH_DECOMP_NV(true, false);
    } else if (plan->out_dtype == PSGD_BF16) {   // one column vector per lane (planner)
        if (plan->stream_hints) PSGD_LAUNCH_DECOMP(1, false, true, true);
        else PSGD_LAUNCH_DECOMP(1, false, false, true);
    } else {
        if (plan->stream_hints) PSGD_LAUNCH_DECOMP_NV(false, true);
        else PSGD_LAUNCH_DECOMP_NV(false, false);
    }
#undef PSGD_LAUNCH_DECOMP_NV
#undef PSGD_LAUNCH_DECOMP
}

#define PSGD_RANK_SWITCH(fn, ...)                       \
    switch (plan->rank) {                               \
        case 1: fn<1>(__VA_ARGS__); break;              \
        case 2: fn<2>(__VA_ARGS__); break;              \
        case 3: fn<3>(__VA_ARGS__); break;              \
        case 4: fn<4>(__VA_ARGS__); break;              \
        case 5: fn<5>(__VA_ARGS__); break;              \
        case 6: fn<6>(__VA_ARGS__); break;              \
        case 7: fn<7>(__VA_ARGS__); break;              \
        case 8: fn<8>(__VA_ARGS__); break;              \
        default: return PSGD_EUNSUPPORTED;              \
    }

static psgd_status check_ready(psgd_plan* plan) {
    if (!plan->uploaded) {
        psgd_status st = upload_tables(plan);
        if (st != PSGD_OK) return st;
    }
    return PSGD_OK;
}

psgd_status launch_compress(psgd_plan* plan, const void* grad, float* err, float* q, float* p, void* workspace,
                            void* stream, bool add) {
    psgd_status st = check_ready(plan);
    if (st != PSGD_OK) return st;
    if (plan->hr) return hr_compress(plan, grad, err, q, p, workspace, stream, add);
    hipStream_t s = static_cast<hipStream_t>(stream);
    float* ws = static_cast<float*>(workspace);
    const void* g = grad;
    if (plan->mats.empty()) return PSGD_OK;

    PSGD_MARK(0);
    plan->compress_marked = plan->profiling;
    PSGD_RANK_SWITCH(launch_ef_right, plan, g, err, q, ws, s, add);
    PSGD_HIP(hipGetLastError(), "launch k_ef_right");
    PSGD_MARK(1);

    const int pre_reduced = plan->p_pre_reduce ? 1 : 0;
    if (pre_reduced) {
        hipLaunchKernelGGL(k_q_reduce, dim3((unsigned)plan->tilesp.size()), dim3(kBlock), 0, s, plan->dev.mats,
                           plan->dev.tilesp, ws, static_cast<float*>(nullptr), plan->workers, 1);
        PSGD_HIP(hipGetLastError(), "launch k_q_reduce (partial P)");
    }
    if (!plan->small_mats.empty()) {
        hipLaunchKernelGGL(k_ortho, dim3((unsigned)plan->small_mats.size()), dim3(kOrthoBlock), 0, s, plan->dev.mats,
                           plan->dev.small_mats, ws, p, plan->workers, pre_reduced);
        PSGD_HIP(hipGetLastError(), "launch k_ortho");
    }
    if (!plan->tiles_gram.empty() && plan->gram_fused) {
        hipError_t ge = hipSuccess;
        const dim3 ggrid((unsigned)plan->tiles_gram.size());
        slot_t* gmail = reinterpret_cast<slot_t*>(plan->dev.gram_mail);
#define PSGD_LAUNCH_GRAM_CHOL(RR)                                                                                     \
    hipLaunchKernelGGL((k_gram_chol<RR>), ggrid, dim3(kBlock), 0, s, plan->dev.mats, plan->dev.tiles_gram, ws, p, gmail, \
                       plan->dev.gram_sync, plan->workers, pre_reduced, (unsigned)plan->tuning.gram_spin)
        switch (plan->rank) {
            case 1: PSGD_LAUNCH_GRAM_CHOL(1); break;
            case 2: PSGD_LAUNCH_GRAM_CHOL(2); break;
            case 3: PSGD_LAUNCH_GRAM_CHOL(3); break;
            case 4: PSGD_LAUNCH_GRAM_CHOL(4); break;
            case 5: PSGD_LAUNCH_GRAM_CHOL(5); break;
            case 6: PSGD_LAUNCH_GRAM_CHOL(6); break;
            case 7: PSGD_LAUNCH_GRAM_CHOL(7); break;
            case 8: PSGD_LAUNCH_GRAM_CHOL(8); break;
            default: ge = hipErrorInvalidValue; break;
        }
#undef PSGD_LAUNCH_GRAM_CHOL
        if (ge == hipSuccess) ge = hipGetLastError();
        PSGD_HIP(ge, "launch k_gram_chol");
    } else if (!plan->tiles_gram.empty()) {
        const size_t float_bytes = (size_t)(plan->ws_ppart_floats + plan->ws_qpart_floats) * sizeof(float);
        double* gram = reinterpret_cast<double*>(static_cast<char*>(workspace) + (float_bytes + 255) / 256 * 256);
        hipLaunchKernelGGL(k_gram, dim3((unsigned)plan->tiles_gram.size()), dim3(kBlock), 0, s, plan->dev.mats,
                           plan->dev.tiles_gram, ws, p, gram, plan->workers, pre_reduced);
        PSGD_HIP(hipGetLastError(), "launch k_gram");
        hipLaunchKernelGGL(k_chol_apply, dim3((unsigned)plan->tiles_gram.size()), dim3(kBlock), 0, s, plan->dev.mats,
                           plan->dev.tiles_gram, gram, p);
        PSGD_HIP(hipGetLastError(), "launch k_chol_apply");
    }
    PSGD_MARK(2);

    PSGD_RANK_SWITCH(launch_left, plan, err, p, ws, s);
    PSGD_HIP(hipGetLastError(), "launch k_left");
    PSGD_MARK(3);

    st = launch_q_reduce(plan, ws, q, stream);
    if (st != PSGD_OK) return st;
    PSGD_MARK(4);
    return PSGD_OK;
}

psgd_status launch_q_reduce(psgd_plan* plan, float* ws, float* q, void* stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (plan->tilesq.empty()) return PSGD_OK;   // every Q was written directly
    hipLaunchKernelGGL(k_q_reduce, dim3((unsigned)plan->tilesq.size()), dim3(kBlock), 0, s, plan->dev.mats,
                       plan->dev.tilesq, ws, q, plan->workers, 0);
    PSGD_HIP(hipGetLastError(), "launch k_q_reduce");
    return PSGD_OK;
}

psgd_status launch_decompress(psgd_plan* plan, const float* p, const float* q, float* err, const void* grad, void* out,
                              void* workspace, void* stream, const UpdateArgs& upd) {
    (void)workspace;
    psgd_status st = check_ready(plan);
    if (st != PSGD_OK) return st;
    if (plan->hr) return hr_decompress(plan, p, q, err, grad, out, stream, upd);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (plan->tiles4.empty()) return PSGD_OK;
    PSGD_MARK(5);
    PSGD_RANK_SWITCH(launch_decomp, plan, err, p, q, grad, out, s, upd);
    PSGD_HIP(hipGetLastError(), "launch k_decomp");
    if (plan->grad_dtype != PSGD_F32 || plan->out_dtype != PSGD_F32) {
        psgd_status vs = launch_vector_mean(plan, grad, out, stream, upd);
        if (vs != PSGD_OK) return vs;
    }
    PSGD_MARK(6);
    return finish_profiled_step(plan);
}

// measurement mode: wait for the step, then add its per-kernel times (compress must have run first)
psgd_status finish_profiled_step(psgd_plan* plan) {
    if (!plan->profiling) return PSGD_OK;
    if (!plan->compress_marked) return PSGD_OK;   // no psgd_compress recorded its events since profiling was switched on
    PSGD_HIP(hipEventSynchronize(static_cast<hipEvent_t>(plan->events[6])), "hipEventSynchronize");
    static const int first[5] = {0, 1, 2, 3, 5};
    for (int k = 0; k < 5; ++k) {
        float ms = 0.f;
        hipError_t e = hipEventElapsedTime(&ms, static_cast<hipEvent_t>(plan->events[first[k]]),
                                           static_cast<hipEvent_t>(plan->events[first[k] + 1]));
        if (e != hipSuccess) return hip_fail(plan, e, "hipEventElapsedTime");
        plan->kernel_ms[k] += ms;
    }
    ++plan->profiled_steps;
    return PSGD_OK;
}

}  // namespace psgd
