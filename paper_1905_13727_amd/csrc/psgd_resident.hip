// Resident PowerSGD step for models whose update matrices fit in the register files of the chip
// (MI355X: 256 CUs x 512 KB of vector registers).
//
// One kernel does the whole step of arXiv 1905.13727 (Algorithm 1 inside the error-feedback loop
// of Algorithm 2) for W = 1.  Each wavefront owns one tile (a strip of rows x 64 column vectors)
// of one matrix and keeps M = g + e of that tile in registers from the first load to the last
// store, so that HBM sees each matrix element exactly once in (g, e) and once out (e', Delta'):
//
//   phase A   load g, e; M = g + e (Alg. 2);  row dot products of P = M Q (Alg. 1) -> partial P per
//             column chunk; the wavefront with the first chunk of a strip adds the strip's chunks;
//             the wavefront with the first tile of a matrix runs Gram-Schmidt on the n x r panel
//             (Alg. 1 "orthogonalize") and publishes P_hat
//   phase B   (needs this strip's rows of P_hat)  Q = M^T P_hat from the registers -> partial Q per
//             run of strips (consecutive wavefronts of a workgroup with the same column chunk); the
//             first wavefront of every run adds the chunk's runs and hands Q to its run through LDS
//   phase C   (needs this chunk's rows of Q)  Delta' = P_hat Q^T (Alg. 1 "decompress"),
//             e' = M - Delta' (Alg. 2), each stored once
//
// The two "needs" are the two global dependencies of the method (all of P before P_hat, all of Q
// before P_hat Q^T), taken per strip and per column chunk instead of as grid-wide barriers.
//
// Everything that crosses wavefronts travels through a plan-owned MAILBOX of 64-bit slots
// {value, tag}: the producer writes the float together with the step's epoch in one 8-byte
// device-scope store (written through to memory), the consumer polls the slot with device-scope
// loads until the tag equals the epoch.  There are no counters, no flags and no cache-wide
// write-backs or invalidates on the critical path; a hand-over costs one memory round trip.  The
// epoch is a device word read by every wavefront at kernel start and advanced by the workgroup
// that finishes last, so stale slots of earlier steps never match.  All sums run in a fixed order.
//
// The grid must be co-resident (the launcher checks the occupancy).  Every wait is bounded: a
// wavefront that polls longer than kSpinLimit rounds raises the error word and goes on, so the
// kernel always terminates.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>

#include "psgd_device.h"
#include "psgd_internal.h"

namespace psgd {

constexpr int kResRowsPerLane = kResMaxN / kWave;   // rows of the Gram-Schmidt panel a lane holds

struct ResArgs {
    const MatDesc* mats;         // resident descriptors: ppart_off / qpart_off are mailbox offsets (slots)
    const RTile* tiles;
    const float* grad;
    float* err;
    float* q;
    float* p;
    float* out;
    slot_t* mail;
    unsigned* sync;              // error word, epoch word, finished-workgroup count
    int32_t nblocks;
    int64_t n_mat_elems;
    unsigned long long* trace;   // diagnostic: kResTracePoints timestamps per workgroup, or nullptr
    unsigned spin;               // polls before a wait gives up
    int32_t iters;               // subspace iterations per step (ITER kernels; 1 otherwise)
    UpdateArgs upd;              // UPD kernels: momentum / parameter buffers and step sizes (Algorithm 2's last lines)
};

__device__ __forceinline__ void trace_mark(const ResArgs& a, int point) {
    if (a.trace && (threadIdx.x & (kWave - 1)) == 0)
        a.trace[((size_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)) * kResTracePoints + point] = wall_clock64();
}
__device__ __forceinline__ void trace_mark_wave(const ResArgs& a, int point) { trace_mark(a, point); }

// ---- Gram-Schmidt by one wavefront -------------------------------------------------------------------
// Rows lane, lane + 64, ... of the n x r panel are held in registers (n <= kResMaxN).  Column by
// column, left to right: squared norm and dot products with the columns to the right in fp64, reduced
// over the wavefront; normalise; remove the component from the columns to the right (modified
// Gram-Schmidt).  A column whose squared norm is <= 1e-30 at its turn becomes zero.
template <int R>
__device__ __forceinline__ void gram_schmidt_rows(float (&P)[kResRowsPerLane][R], int ri) {
#pragma unroll
    for (int c = 0; c < R; ++c) {
        if (c < ri) {
            double s[R];
#pragma unroll
            for (int k = 0; k < R; ++k) s[k] = 0.0;
#pragma unroll
            for (int j = 0; j < kResRowsPerLane; ++j) {
                const double pc = (double)P[j][c];
#pragma unroll
                for (int k = c; k < R; ++k) s[k] += pc * (double)P[j][k];
            }
#pragma unroll
            for (int k = c; k < R; ++k) s[k] = wave_sum(s[k]);
            const double scc = s[c];
            if (scc <= 1e-30) {
#pragma unroll
                for (int j = 0; j < kResRowsPerLane; ++j) P[j][c] = 0.f;
            } else {
                const double inv = 1.0 / sqrt(scc);
#pragma unroll
                for (int j = 0; j < kResRowsPerLane; ++j) {
                    const double pc = (double)P[j][c];
                    P[j][c] = (float)(pc * inv);
#pragma unroll
                    for (int k = c + 1; k < R; ++k) P[j][k] = (float)((double)P[j][k] - (s[k] / scc) * pc);
                }
            }
        }
    }
}

// ---- the step, for a workgroup whose tiles use V-wide row accesses ---------------------------------------
// ITER: several subspace iterations on the resident tile (Appendix G.7): P = M Q, orthogonalise, Q = M^T P_hat
// repeated a.iters times before the decompression, each round under its own mailbox tag epoch0 + round.
// RT: rows of the tile the code is written out for (the strips of the plan are no taller).
template <int R, int V, bool UPD, bool ITER, int RT>
__device__ __forceinline__ void resident_body(const ResArgs& a, const RTile& t, float* lds, unsigned epoch0) {
    const int lane_id = threadIdx.x & (kWave - 1);
    const int lane = lane_id;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool active = t.mat >= 0;
    const MatDesc d = a.mats[active ? t.mat : 0];
    const int ri = d.r;
    const bool valid = active && lane < t.nvec;
    const int col = (t.vec0 + lane) * V;
    const int nrows = active ? t.nrows : 0;
    const int64_t tile_off = d.off + (int64_t)t.row0 * d.m + col;
    unsigned* err_word = a.sync + res_sync_err();
    // mailbox regions of this matrix (slots)
    const int64_t nr = (int64_t)d.n * ri, mr = (int64_t)d.m * ri;
    slot_t* mail_base = a.mail;

    // ---------------- phase A ----------------
    trace_mark(a, 0);
    if (a.trace && lane == 0) {
        unsigned long long* tr = a.trace + ((size_t)blockIdx.x * kWavesPerBlock + wave) * kResTracePoints;
        tr[12] = (unsigned long long)(long long)t.mat;
        // with the wavefront's place on the chip in the upper halves: hardware id (compute unit, shader array and
        // engine, SIMD, slot) and accelerator die
        const unsigned long long hw_id = __builtin_amdgcn_s_getreg((31 << 11) | 4);    // HW_ID, all 32 bits
        const unsigned long long xcc_id = __builtin_amdgcn_s_getreg((31 << 11) | 20);  // XCC_ID, all 32 bits
        tr[13] = (unsigned long long)(unsigned)t.ppart | (hw_id << 32);
        tr[14] = (unsigned long long)(unsigned)t.row0 | (xcc_id << 32);
        tr[15] = (unsigned long long)(t.qrun_len > 0 ? t.qpart : -1);
    }
    float M[RT][V];
    float qr[V][R];
    load_factor_rows<R, V>(a.q + d.q_off + (int64_t)col * ri, ri, valid, qr);
    {
        // strip descriptor: rows past the strip are beyond the range, a lane without columns is out of range
        const int64_t strip = d.off + (int64_t)t.row0 * d.m;
        const buf_rsrc gres = make_rsrc(a.grad + strip, (int64_t)nrows * d.m * 4);
        const buf_rsrc eres = make_rsrc(a.err + strip, (int64_t)nrows * d.m * 4);
        const unsigned coff = valid ? (unsigned)col * 4u : kOutOfRange;
        // g and e are read once per step: non-temporal loads, which claim no cache lines.  Behind caches full of
        // another kernel's unwritten lines (a training step: the backward pass has just run) every claimed line first
        // forces one of those out to memory: 53.6 -> 45.8 us for the step at rank 2 with e read this way; steps
        // run back to back with nothing between them lose 0.5 us (their e then no longer waits in the memory-side
        // cache to be overwritten in place)
#pragma unroll
        for (int i = 0; i < RT; ++i) buf_ldv<V>(gres, coff + (unsigned)i * (unsigned)d.m * 4u, M[i], true);
        if constexpr (RT > 24) {
            // the tallest strips have no room for a second whole tile of registers: e in two halves, all loads of a
            // half in flight together (row by row behind single loads the phase is bound by their latency)
            constexpr int H = RT / 2;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float e[H][V];
#pragma unroll
                for (int i = 0; i < H; ++i) buf_ldv<V>(eres, coff + (unsigned)(h * H + i) * (unsigned)d.m * 4u, e[i], true);
#pragma unroll
                for (int i = 0; i < H; ++i)
#pragma unroll
                    for (int x = 0; x < V; ++x) M[h * H + i][x] += e[i][x];
            }
        } else {
            float e[RT][V];
#pragma unroll
            for (int i = 0; i < RT; ++i) buf_ldv<V>(eres, coff + (unsigned)i * (unsigned)d.m * 4u, e[i], true);
#pragma unroll
            for (int i = 0; i < RT; ++i)
#pragma unroll
                for (int x = 0; x < V; ++x) M[i][x] += e[i][x];
        }
    }
    const int iters = ITER ? a.iters : 1;
    float pr[R];
    for (int it = 0; it < iters; ++it) {
    const unsigned epoch = epoch0 + (unsigned)it;
    int lane = lane_id;
    if constexpr (ITER) {
        // the slot addresses are formed anew in every round: computed once before the loop they would all be held
        // in registers across it, which the tile of M leaves no room for
        asm volatile("" : "+s"(mail_base));
        asm volatile("" : "+v"(lane));
    }
    slot_t* mail_pp = mail_base + d.ppart_off;            // partial P   [n_cchunk][n][r]
    slot_t* mail_pb = mail_pp + (int64_t)d.n_cchunk * nr; // mean P      [n][r]
    slot_t* mail_ph = mail_pb + nr;                       // P_hat       [n][r]
    slot_t* mail_qp = mail_base + d.qpart_off;            // partial Q   [n_rblock][m][r]
    {
        // the strip's row dot products: lane i receives row i's (rows past the strip were read as zeros)
        float mine[R];
        // rank by rank, all rows of the strip reduced over the wavefront together (one reduction per row and rank
        // instead: +1.5 us at rank 3, +0.9 us at rank 4)
#pragma unroll
        for (int k = 0; k < R; ++k) {
            float part[RT];
#pragma unroll
            for (int i = 0; i < RT; ++i) {
                float s = 0.f;
#pragma unroll
                for (int x = 0; x < V; ++x) s = fmaf(M[i][x], qr[x][k], s);
                part[i] = s;
            }
            mine[k] = lane_sums<RT>(part);
        }
        if (lane < nrows) {
            // mailbox layouts are [..][k][row] (and [..][x][k][column vector] for Q): consecutive lanes
            // write consecutive slots, so one store instruction fills whole memory lines
            slot_t* dst = mail_pp + (int64_t)t.ppart * nr + t.row0 + lane;
#pragma unroll
            for (int k = 0; k < R; ++k)
                if (k < ri) post(dst + (int64_t)k * d.n, mine[k], epoch);
        }
    }
    trace_mark(a, 1);
    if (active && t.ppart == 0 && t.row0 == 0) trace_mark_wave(a, 7);
    if (active && t.ppart == 0) {
        // This wavefront holds the first column chunk of its strip: it adds the strip's chunks in chunk
        // order into the rows of the mean P (W = 1: the mean over workers is the value itself).
        const int nval = nrows * ri;   // <= 128
        // The strip's last column chunk sits furthest down the tile list and tends to deliver last: one lane watches
        // its slot before all lanes poll all chunks.  (A wavefront that polls everything for microseconds fills its
        // compute unit's memory pipeline, and the loads of the other workgroup on that unit land 2-3 us late.)
        await_tag(mail_pp + (int64_t)(d.n_cchunk - 1) * nr + t.row0, epoch, err_word, a.spin);
        for (int u = 0; u * kWave < nval; ++u) {
            const int idx = lane + kWave * u;
            const bool mine = idx < nval;
            const int idx_c = mine ? idx : nval - 1;
            const int64_t at = (int64_t)(idx_c / nrows) * d.n + t.row0 + idx_c % nrows;   // [k][row]
            float s = 0.f;
            constexpr int CG = 20;   // chunk partials polled together
            for (int c0 = 0; c0 < d.n_cchunk; c0 += CG) {
                slot_t w[CG];
                await([&]() {
#pragma unroll
                    for (int cc = 0; cc < CG; ++cc)
                        w[cc] = fetch(mail_pp + (int64_t)min(c0 + cc, d.n_cchunk - 1) * nr + at);
                    bool ok = true;
#pragma unroll
                    for (int cc = 0; cc < CG; ++cc) ok &= arrived(w[cc], epoch);
                    return ok;
                }, err_word, epoch, a.spin);
#pragma unroll
                for (int cc = 0; cc < CG; ++cc)
                    if (c0 + cc < d.n_cchunk) s += value_of(w[cc]);
            }
            if (mine) post(mail_pb + at, s, epoch);
        }
        if (t.row0 == 0) {
            // ... and this one also holds the first strip: it orthogonalises the matrix's panel.
            trace_mark_wave(a, 8);
            float P[kResRowsPerLane][R];
            {
                // again one lane first, on the matrix's last row (its last strip is furthest down the tile list)
                await_tag(mail_pb + (d.n - 1), epoch, err_word, a.spin);
                slot_t w[kResRowsPerLane][R];
                await([&]() {
#pragma unroll
                    for (int j = 0; j < kResRowsPerLane; ++j)
#pragma unroll
                        for (int k = 0; k < R; ++k)
                            w[j][k] = fetch(mail_pb + (int64_t)min(k, ri - 1) * d.n + min(lane + kWave * j, d.n - 1));
                    bool ok = true;
#pragma unroll
                    for (int j = 0; j < kResRowsPerLane; ++j)
#pragma unroll
                        for (int k = 0; k < R; ++k) ok &= arrived(w[j][k], epoch);
                    return ok;
                }, err_word, epoch, a.spin);
#pragma unroll
                for (int j = 0; j < kResRowsPerLane; ++j)
#pragma unroll
                    for (int k = 0; k < R; ++k)
                        P[j][k] = (lane + kWave * j < d.n && k < ri) ? value_of(w[j][k]) : 0.f;
            }
            trace_mark_wave(a, 9);
            gram_schmidt_rows<R>(P, ri);
            trace_mark_wave(a, 10);
#pragma unroll
            for (int j = 0; j < kResRowsPerLane; ++j) {
                const int row = lane + kWave * j;
                if (row < d.n) {
#pragma unroll
                    for (int k = 0; k < R; ++k)
                        if (k < ri) {
                            post(mail_ph + (int64_t)k * d.n + row, P[j][k], epoch);
                            a.p[d.p_off + (int64_t)row * ri + k] = P[j][k];
                        }
                }
            }
            trace_mark_wave(a, 11);
        }
    }
    trace_mark(a, 2);

    // ---------------- phase B ----------------
#pragma unroll
    for (int k = 0; k < R; ++k) pr[k] = 0.f;
    // The workgroup's first wavefront watches for P_hat (one lane, one slot); the others wait for it at a barrier,
    // which costs no memory traffic.  Its strips are mostly consecutive strips of one matrix and get their rows at
    // the same time; they meet at the barrier of the sum of Q a moment later anyway.
    if (active && wave == 0) await_tag(mail_ph + t.row0, epoch, err_word, a.spin);
    __syncthreads();
    if (active) {
        slot_t w[R];
        const int64_t my_row = t.row0 + min(lane, nrows - 1);
        await([&]() {
#pragma unroll
            for (int k = 0; k < R; ++k) w[k] = fetch(mail_ph + (int64_t)min(k, ri - 1) * d.n + my_row);
            bool ok = true;
#pragma unroll
            for (int k = 0; k < R; ++k) ok &= arrived(w[k], epoch);
            return ok;
        }, err_word, epoch, a.spin);
#pragma unroll
        for (int k = 0; k < R; ++k) pr[k] = (lane < nrows && k < ri) ? value_of(w[k]) : 0.f;
    }
    trace_mark(a, 3);
    float acc[V][R];
#pragma unroll
    for (int x = 0; x < V; ++x)
#pragma unroll
        for (int k = 0; k < R; ++k) acc[x][k] = 0.f;
#pragma unroll
    for (int i = 0; i < RT; ++i) {   // rows past the strip: M was read as zeros and P_hat is zero there, no branch needed
#pragma unroll
        for (int k = 0; k < R; ++k) {
            const float pk = lane_bcast(pr[k], i);
#pragma unroll
            for (int x = 0; x < V; ++x) acc[x][k] = fmaf(M[i][x], pk, acc[x][k]);
        }
    }
    // add the sums of a run of wavefronts (strips of the same column chunk) in LDS, fixed order
#pragma unroll
    for (int x = 0; x < V; ++x)
#pragma unroll
        for (int k = 0; k < R; ++k) lds[((wave * V + x) * R + k) * kWave + lane] = acc[x][k];
    __syncthreads();
    if (active && t.qrun_len > 0) {
        for (int w2 = 1; w2 < t.qrun_len; ++w2) {
#pragma unroll
            for (int x = 0; x < V; ++x)
#pragma unroll
                for (int k = 0; k < R; ++k) acc[x][k] += lds[(((wave + w2) * V + x) * R + k) * kWave + lane];
        }
        const int64_t nvec_m = d.m / V;                       // column vectors of the matrix
        const int64_t jv = t.vec0 + min(lane, t.nvec - 1);    // this lane's (idle lanes: a wanted) column vector
        if (valid) {
            slot_t* dst = mail_qp + (int64_t)t.qpart * mr + jv;   // [x][k][column vector]
#pragma unroll
            for (int x = 0; x < V; ++x)
#pragma unroll
                for (int k = 0; k < R; ++k)
                    if (k < ri) post(dst + (int64_t)(x * ri + k) * nvec_m, acc[x][k], epoch);
        }
        {
            // Every run of this column chunk adds the chunk's partials itself, in run order (the same sum in each of
            // them): Q is then one trip through memory away from the partials, not two, and only the runs' first
            // wavefronts poll.  The chunk's first run also stores Q.
            if (t.qpart == 0 && !(t.ppart == 0 && t.row0 == 0)) trace_mark_wave(a, 8);
            float s[V][R];
#pragma unroll
            for (int x = 0; x < V; ++x)
#pragma unroll
                for (int k = 0; k < R; ++k) s[x][k] = 0.f;
            constexpr int PG = V * R >= 16 ? 1 : (V * R >= 8 ? 2 : 4);   // run partials polled together
            const slot_t* src_c = mail_qp + jv;
            for (int p0 = 0; p0 < t.nqparts; p0 += PG) {
                slot_t w[PG][V][R];
                await([&]() {
#pragma unroll
                    for (int u = 0; u < PG; ++u)
#pragma unroll
                        for (int x = 0; x < V; ++x)
#pragma unroll
                            for (int k = 0; k < R; ++k)
                                w[u][x][k] = fetch(src_c + (int64_t)min(p0 + u, t.nqparts - 1) * mr +
                                                   (int64_t)(x * ri + min(k, ri - 1)) * nvec_m);
                    bool ok = true;
#pragma unroll
                    for (int u = 0; u < PG; ++u)
#pragma unroll
                        for (int x = 0; x < V; ++x)
#pragma unroll
                            for (int k = 0; k < R; ++k) ok &= arrived(w[u][x][k], epoch);
                    return ok;
                }, err_word, epoch, a.spin);
#pragma unroll
                for (int u = 0; u < PG; ++u)
#pragma unroll
                    for (int x = 0; x < V; ++x)
#pragma unroll
                        for (int k = 0; k < R; ++k)
                            if (p0 + u < t.nqparts) s[x][k] += value_of(w[u][x][k]);
                if (t.qpart == 0 && !(t.ppart == 0 && t.row0 == 0)) trace_mark_wave(a, 9 + min(p0 / PG, 2));
            }
            if (t.qpart == 0 && valid) {
#pragma unroll
                for (int x = 0; x < V; ++x)
#pragma unroll
                    for (int k = 0; k < R; ++k)
                        if (k < ri) a.q[d.q_off + (int64_t)(col + x) * ri + k] = s[x][k];   // W = 1: mean = sum
            }
            // Q goes to the wavefronts of the run through shared memory (their own sums there have been read above)
            for (int w2 = 0; w2 < t.qrun_len; ++w2) {
#pragma unroll
                for (int x = 0; x < V; ++x)
#pragma unroll
                    for (int k = 0; k < R; ++k) lds[(((wave + w2) * V + x) * R + k) * kWave + lane] = s[x][k];
            }
        }
    }
    trace_mark(a, 4);
    __syncthreads();

    // this chunk's rows of Q, for the decompression or the next round's P = M Q
#pragma unroll
    for (int x = 0; x < V; ++x)
#pragma unroll
        for (int k = 0; k < R; ++k) qr[x][k] = 0.f;
    if (active) {
#pragma unroll
        for (int x = 0; x < V; ++x)
#pragma unroll
            for (int k = 0; k < R; ++k)
                qr[x][k] = (valid && k < ri) ? lds[((wave * V + x) * R + k) * kWave + lane] : 0.f;
    }
    if constexpr (ITER) {
        if (it + 1 < iters) __syncthreads();   // shared memory is written again in the next round
    }
    }   // rounds

    // ---------------- phase C ----------------
    float (&qb)[V][R] = qr;
    trace_mark(a, 5);
    constexpr int CG = UPD ? 4 : 1;   // rows whose momentum / parameter loads are in flight together
#pragma unroll
    for (int i0 = 0; i0 < RT; i0 += CG) {
        float mo[CG][V], pa[CG][V];
        if constexpr (UPD) {
#pragma unroll
            for (int u = 0; u < CG; ++u)
                if (i0 + u < RT && i0 + u < nrows && valid) {
                    ldv<V>(a.upd.mom + tile_off + (int64_t)(i0 + u) * d.m, mo[u]);
                    ldv<V>(a.upd.param + tile_off + (int64_t)(i0 + u) * d.m, pa[u]);
                }
        }
#pragma unroll
        for (int u = 0; u < CG; ++u) {
            const int i = i0 + u;
            if (i < RT && i < nrows) {
                float pk[R];
#pragma unroll
                for (int k = 0; k < R; ++k) pk[k] = lane_bcast(pr[k], i);
                if (valid) {
                    float dl[V], en[V];
#pragma unroll
                    for (int x = 0; x < V; ++x) {
                        float s = 0.f;
#pragma unroll
                        for (int k = 0; k < R; ++k) s = fmaf(pk[k], qb[x][k], s);
                        dl[x] = s;
                        en[x] = M[i < RT ? i : 0][x] - s;
                    }
                    stv<V>(a.err + tile_off + (int64_t)i * d.m, en);
                    if constexpr (UPD) {
                        momentum_step<V>(mo[u], pa[u], dl, a.upd.lr, a.upd.lam);
                        stv<V>(a.upd.mom + tile_off + (int64_t)i * d.m, mo[u]);
                        stv<V>(a.upd.param + tile_off + (int64_t)i * d.m, pa[u]);
                    } else {
                        stv_stream<V>(a.out + tile_off + (int64_t)i * d.m, dl);   // written once: around the caches, which keep e
                    }
                }
            }
        }
    }
    if (t.mat == -1) {
        // vector-shaped tensors, W = 1: Delta' is the gradient itself
        for (int64_t idx = t.elem0 + lane; idx < t.elem0 + t.nelem; idx += kWave) {
            const float dl1[1] = {a.grad[a.n_mat_elems + idx]};
            if constexpr (UPD) {
                float m1[1] = {a.upd.mom[a.n_mat_elems + idx]}, x1[1] = {a.upd.param[a.n_mat_elems + idx]};
                momentum_step<1>(m1, x1, dl1, a.upd.lr, a.upd.lam);
                a.upd.mom[a.n_mat_elems + idx] = m1[0];
                a.upd.param[a.n_mat_elems + idx] = x1[0];
            } else {
                a.out[a.n_mat_elems + idx] = dl1[0];
            }
        }
    }
    trace_mark(a, 6);
}

template <int R, bool UPD, bool ITER, int RT>
__global__ __launch_bounds__(kBlock, 2) void k_resident(ResArgs a) {
    __shared__ float lds[kWavesPerBlock * 4 * R * kWave];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    // the epoch cannot change before every workgroup of this launch has finished
    unsigned epoch = 0;
    if ((threadIdx.x & (kWave - 1)) == 0) epoch = ld_dev(a.sync + res_sync_epoch());
    epoch = __builtin_amdgcn_readfirstlane(epoch);
    const RTile t = a.tiles[blockIdx.x * kWavesPerBlock + wave];
    // all tiles of a workgroup use the same access width; the first slot is never idle
    const RTile t0 = a.tiles[blockIdx.x * kWavesPerBlock];
    const int vec = t0.mat >= 0 ? a.mats[t0.mat].vec : 4;
    if (vec == 4) resident_body<R, 4, UPD, ITER, RT>(a, t, lds, epoch);
    else if (vec == 2) resident_body<R, 2, UPD, ITER, RT>(a, t, lds, epoch);
    else resident_body<R, 1, UPD, ITER, RT>(a, t, lds, epoch);
    // the workgroup that finishes last advances the epoch for the next launch
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned* done = a.sync + res_sync_done();
        if (add_dev(done, 1u) == (unsigned)a.nblocks - 1u) {
            add_dev(done, 0u - (unsigned)a.nblocks);
            st_dev(a.sync + res_sync_epoch(), epoch + (ITER ? (unsigned)a.iters : 1u));   // one tag per round
        }
    }
}

// ---- host side --------------------------------------------------------------------------------------------

// The kernels are written out for 24-row tiles and, at rank 1 and 2, for 32-row tiles as well; a plan whose strips
// are at most 24 rows tall (the ResNet18-shaped set: 23) runs the shorter code, a quarter less work in every phase.
template <int R, int RT>
static hipError_t launch_k_resident_rt(const ResArgs& a, int blocks, hipStream_t s, int* max_blocks_per_cu) {
    if (max_blocks_per_cu) {
        // every variant must be co-resident
        int occ[3] = {0, 0, 0};
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ[0], k_resident<R, false, false, RT>, kBlock, 0);
        if (e != hipSuccess) return e;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ[1], k_resident<R, true, false, RT>, kBlock, 0);
        if (e != hipSuccess) return e;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ[2], k_resident<R, false, true, RT>, kBlock, 0);
        if (e != hipSuccess) return e;
        *max_blocks_per_cu = std::min(occ[0], std::min(occ[1], occ[2]));
        return hipSuccess;
    }
    if (a.upd.mom) hipLaunchKernelGGL((k_resident<R, true, false, RT>), dim3((unsigned)blocks), dim3(kBlock), 0, s, a);
    else if (a.iters > 1) hipLaunchKernelGGL((k_resident<R, false, true, RT>), dim3((unsigned)blocks), dim3(kBlock), 0, s, a);
    else hipLaunchKernelGGL((k_resident<R, false, false, RT>), dim3((unsigned)blocks), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

template <int R>
static hipError_t launch_k_resident(const ResArgs& a, int blocks, hipStream_t s, int* max_blocks_per_cu, int strip_rows) {
    if constexpr (res_rows_for_rank(R) > 24) {
        if (max_blocks_per_cu) {   // the smaller of the two variants' occupancies
            int o24 = 0, o32 = 0;
            hipError_t e = launch_k_resident_rt<R, 24>(a, blocks, s, &o24);
            if (e != hipSuccess) return e;
            e = launch_k_resident_rt<R, 32>(a, blocks, s, &o32);
            if (e != hipSuccess) return e;
            *max_blocks_per_cu = std::min(o24, o32);
            return hipSuccess;
        }
        if (strip_rows > 24) return launch_k_resident_rt<R, 32>(a, blocks, s, nullptr);
    }
    return launch_k_resident_rt<R, 24>(a, blocks, s, max_blocks_per_cu);
}

static hipError_t dispatch_resident(int rank, const ResArgs& a, int blocks, hipStream_t s, int* occ, int strip_rows) {
    switch (rank) {
        case 1: return launch_k_resident<1>(a, blocks, s, occ, strip_rows);
        case 2: return launch_k_resident<2>(a, blocks, s, occ, strip_rows);
        case 3: return launch_k_resident<3>(a, blocks, s, occ, strip_rows);
        case 4: return launch_k_resident<4>(a, blocks, s, occ, strip_rows);
        default: return hipErrorInvalidValue;
    }
}

// Once per plan, when its tables are uploaded: the resident tiling is laid out again for the number of workgroups
// THIS device holds at once (compute units x workgroups per unit of the kernel); the planner's own figure is a
// provisional one, since it runs without a device.  A model that does not fit streams instead.
psgd_status resident_check_device(psgd_plan* plan) {
    if (plan->rank > kResMaxRank || plan->workers != 1) return PSGD_OK;   // never resident: nothing to lay out
    int dev = 0, cus = 0, occ = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PSGD_EHIP;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return PSGD_EHIP;
    ResArgs dummy{};
    if (dispatch_resident(plan->rank, dummy, 0, nullptr, &occ, 0) != hipSuccess) return PSGD_EHIP;
    if (plan->tuning.resident == 2) return PSGD_OK;   // diagnostic: keep the planner's grid whatever the device holds
    build_resident(plan, (int64_t)cus * std::min(occ, kResBlocksPerCU));
    return PSGD_OK;
}

// The step on the streaming kernels: what a plan without (or no longer with) a resident tiling runs.
static psgd_status streamed_step(psgd_plan* plan, const void* grad, float* err, float* q, float* p, void* out,
                                 void* workspace, void* stream, const UpdateArgs& upd, int iterations) {
    psgd_status st = launch_compress(plan, grad, err, q, p, workspace, stream);
    for (int it = 1; it < iterations && st == PSGD_OK; ++it)
        st = launch_compress(plan, err, err, q, p, workspace, stream, false);
    if (st != PSGD_OK) return st;
    return launch_decompress(plan, p, q, err, grad, out, workspace, stream, upd);
}

psgd_status launch_resident_step(psgd_plan* plan, const void* grad, float* err, float* q, float* p, void* out,
                                 void* workspace, void* stream, const UpdateArgs& upd, int iterations) {
    if (!plan->uploaded) {
        psgd_status st = upload_tables(plan);
        if (st != PSGD_OK) return st;
    }
    // the upload may have found that the grid does not fit this device; a wait that gave up switches the mode off
    if (!plan->resident_ok) return streamed_step(plan, grad, err, q, p, out, workspace, stream, upd, iterations);
    hipStream_t s = static_cast<hipStream_t>(stream);
    ResArgs a{};
    a.upd = upd;
    a.mats = plan->dev.res_mats;
    a.tiles = plan->dev.res_tiles;
    a.grad = static_cast<const float*>(grad);
    a.err = err;
    a.q = q;
    a.p = p;
    a.out = static_cast<float*>(out);
    a.mail = reinterpret_cast<slot_t*>(plan->dev.res_mail);
    a.sync = plan->dev.res_sync;
    a.nblocks = plan->res_blocks;
    a.n_mat_elems = plan->sizes.n_mat_elems;
    a.trace = plan->dev.res_trace;
    a.spin = (unsigned)plan->tuning.res_spin;
    a.iters = iterations;
    if (plan->profiling) {
        hipError_t e = hipEventRecord(static_cast<hipEvent_t>(plan->events[0]), s);
        if (e != hipSuccess) { plan->last_error = hipGetErrorString(e); return PSGD_EHIP; }
    }
    hipError_t e = dispatch_resident(plan->rank, a, plan->res_blocks, s, nullptr, plan->res_strip_rows);
    if (e != hipSuccess) {
        plan->last_error = std::string("launch k_resident: ") + hipGetErrorString(e);
        return PSGD_EHIP;
    }
    if (plan->profiling) {
        hipEvent_t e0 = static_cast<hipEvent_t>(plan->events[0]), e1 = static_cast<hipEvent_t>(plan->events[1]);
        float ms = 0.f;
        if (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
            hipEventElapsedTime(&ms, e0, e1) != hipSuccess) {
            plan->last_error = "resident step: event timing failed";
            return PSGD_EHIP;
        }
        plan->kernel_ms[PSGD_KERNEL_RESIDENT] += ms;
        ++plan->profiled_steps;
    }
    return PSGD_OK;
}

}  // namespace psgd
