// Resident PowerSGD step for models whose update matrices fit in the register files of the chip
// (MI355X: 256 CUs x 512 KB of vector registers).
//
// One kernel does the whole step of arXiv 1905.13727 (Algorithm 1 inside the error-feedback loop
// of Algorithm 2) for W = 1.  Each wavefront owns one tile (a strip of rows x 64 column vectors)
// of one matrix and keeps M = g + e of that tile in registers from the first load to the last
// store, so that HBM sees each matrix element exactly once in (g, e) and once out (e', Delta'):
//
//   phase A   load g, e; M = g + e (Alg. 2);  row dot products of P = M Q (Alg. 1) -> partial P;
//             the wavefront that completes a matrix's partials runs Gram-Schmidt on its n x r
//             panel (Alg. 1 "orthogonalize") and publishes P_hat
//   -- wait until this matrix's P_hat is published --
//   phase B   Q = M^T P_hat from the registers -> partial Q per run of strips; the wavefront
//             that completes a column chunk's partials adds them and publishes Q
//   -- wait until this column chunk's Q is published --
//   phase C   Delta' = P_hat Q^T (Alg. 1 "decompress"), e' = M - Delta' (Alg. 2), stored once
//
// The two waits are the two global dependencies of the method (all of P before P_hat, all of Q
// before P_hat Q^T), taken per matrix and per column chunk instead of as grid-wide barriers, so
// that a small matrix does not wait for a large one.  Everything that crosses workgroups
// (partials, P_hat, Q, counters, flags) moves through device-scope relaxed atomics, which are
// written through to memory and read from there, so no cache-wide write-back or invalidate is
// needed; a wavefront only waits for its own stores to be acknowledged before it signals.
// All sums run in a fixed order.
//
// The grid must be co-resident (the launcher checks the occupancy).  Every wait is bounded: a
// wavefront that polls longer than kSpinLimit iterations raises the error word and goes on, so
// the kernel always terminates.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>

#include "psgd_device.h"
#include "psgd_internal.h"

namespace psgd {

constexpr unsigned kSpinLimit = 1u << 21;
constexpr int kResRowsPerLane = kResMaxN / kWave;   // rows of the Gram-Schmidt panel a lane holds

struct ResArgs {
    const MatDesc* mats;
    const RTile* tiles;
    const float* grad;
    float* err;
    float* q;
    float* p;
    float* out;
    float* ws;
    unsigned* sync;
    int32_t ngroups;
    int32_t nblocks;
    int32_t n_mats;
    int32_t n_cntq;
    int32_t n_cnts;
    int64_t flags_at;            // word offset of the readiness flags in `sync`
    int64_t n_mat_elems;
    unsigned long long* trace;   // diagnostic: kResTracePoints timestamps per workgroup, or nullptr
};

__device__ __forceinline__ void trace_mark(const ResArgs& a, int point) {
    if (a.trace && threadIdx.x == 0) a.trace[(size_t)blockIdx.x * kResTracePoints + point] = wall_clock64();
}

// ---- readiness flags -----------------------------------------------------------------------------------
// One word per matrix ("P_hat is published") and one per column chunk ("Q is published").  A flag only
// ever grows: the publisher stores (value at kernel start) + 1 after its data is in memory, consumers
// wait until the word differs from the value they read at kernel start.  A consumer reads that value
// before it contributes to the result the flag stands for, so it cannot miss the change; no word
// needs a reset between launches.
// Each flag has kResFlagCopies copies on separate 256-byte lines so that the wavefronts polling a
// big matrix's flag do not queue on one memory channel; one lane per wavefront polls.
__device__ __forceinline__ unsigned* flag_word(unsigned* flags, int flag, int copy) {
    return flags + ((int64_t)flag * kResFlagCopies + copy) * kSyncLineWords;
}

__device__ __forceinline__ unsigned read_flag(unsigned* flags, int flag, int copy) {
    unsigned v = 0;
    if ((threadIdx.x & (kWave - 1)) == 0) v = ld_dev(flag_word(flags, flag, copy));
    return __builtin_amdgcn_readfirstlane(v);
}

__device__ __forceinline__ void publish_flag(unsigned* flags, int flag, unsigned value) {
    const int lane = threadIdx.x & (kWave - 1);
    if (lane < kResFlagCopies) st_dev(flag_word(flags, flag, lane), value);
}

__device__ __forceinline__ void wait_flag(unsigned* flags, int flag, int copy, unsigned seen_at_start,
                                          unsigned* err_word) {
    unsigned spins = 0;
    while (read_flag(flags, flag, copy) == seen_at_start) {
        __builtin_amdgcn_s_sleep(4);
        if (++spins > kSpinLimit) {
            st_dev(err_word, 1u);
            break;
        }
    }
    wave_mem_done();
}

// ---- Gram-Schmidt by one wavefront -------------------------------------------------------------------
// In place on the n x r panel p_io (the mean P on entry, P_hat on exit), accessed with device-scope
// loads and stores.  Panel rows lane, lane + 64, ... are held in registers (n <= kResMaxN).  Column by column, left to
// right: squared norm and dot products with the columns to the right in fp64, reduced over the
// wavefront; normalise; remove the component from the columns to the right (modified Gram-Schmidt).
// A column whose squared norm is <= 1e-30 at its turn becomes zero.
template <int R>
__device__ __forceinline__ void gram_schmidt_wave(const MatDesc& d, float* p_io) {
    const int lane = threadIdx.x & (kWave - 1);
    const int n = d.n, ri = d.r;
    float P[kResRowsPerLane][R];
#pragma unroll
    for (int j = 0; j < kResRowsPerLane; ++j) {
        const int row = lane + kWave * j;
#pragma unroll
        for (int k = 0; k < R; ++k) P[j][k] = (row < n && k < ri) ? ld_dev(p_io + (int64_t)row * ri + k) : 0.f;
    }
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
#pragma unroll
    for (int j = 0; j < kResRowsPerLane; ++j) {
        const int row = lane + kWave * j;
        if (row < n) {
#pragma unroll
            for (int k = 0; k < R; ++k)
                if (k < ri) st_dev(p_io + (int64_t)row * ri + k, P[j][k]);
        }
    }
}

// ---- the step, for a workgroup whose tiles use V-wide row accesses ---------------------------------------
template <int R, int V>
__device__ __forceinline__ void resident_body(const ResArgs& a, const RTile& t, float* lds) {
    constexpr int RT = kResRows;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool active = t.mat >= 0;
    const MatDesc d = a.mats[active ? t.mat : 0];
    const int ri = d.r;
    const bool valid = active && lane < t.nvec;
    const int col = (t.vec0 + lane) * V;
    const int nrows = active ? t.nrows : 0;
    const int64_t tile_off = d.off + (int64_t)t.row0 * d.m + col;
    unsigned* cnt_p = a.sync + res_sync_cntp(a.ngroups);   // one arrival counter per matrix ...
    unsigned* cnt_q = cnt_p + a.n_mats;                    // ... one per column chunk ...
    unsigned* cnt_s = cnt_q + a.n_cntq;                    // ... one per strip,
    // then the readiness flags, on lines of their own: per matrix, then per column chunk
    unsigned* flags = a.sync + a.flags_at;
    const int fl_p = active ? t.mat : 0, fl_q = active ? a.n_mats + t.cntq : 0;
    const int copy = (blockIdx.x * kWavesPerBlock + wave) % kResFlagCopies;
    unsigned* err_word = a.sync + res_sync_err();
    unsigned fp0 = 0, fq0 = 0;
    if (active) {
        fp0 = read_flag(flags, fl_p, copy);
        fq0 = read_flag(flags, fl_q, copy);
    }

    // ---------------- phase A ----------------
    trace_mark(a, 0);
    float M[RT][V];
    float qr[V][R];
#pragma unroll
    for (int x = 0; x < V; ++x)
#pragma unroll
        for (int k = 0; k < R; ++k)
            qr[x][k] = (valid && k < ri) ? a.q[d.q_off + (int64_t)(col + x) * ri + k] : 0.f;
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        if (i < nrows && valid) {
            ldv_stream<V>(a.grad + tile_off + (int64_t)i * d.m, M[i]);
        } else {
#pragma unroll
            for (int x = 0; x < V; ++x) M[i][x] = 0.f;
        }
    }
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        if (i < nrows && valid) {
            float e[V];
            ldv<V>(a.err + tile_off + (int64_t)i * d.m, e);
#pragma unroll
            for (int x = 0; x < V; ++x) M[i][x] += e[x];
        }
    }
    {
        float mine[R];
#pragma unroll
        for (int k = 0; k < R; ++k) mine[k] = 0.f;
#pragma unroll
        for (int i = 0; i < RT; ++i) {
            if (i < nrows) {
#pragma unroll
                for (int k = 0; k < R; ++k) {
                    float s = 0.f;
#pragma unroll
                    for (int x = 0; x < V; ++x) s = fmaf(M[i][x], qr[x][k], s);
                    s = wave_sum(s);
                    if (lane == i) mine[k] = s;
                }
            }
        }
        if (lane < nrows) {
            float* dst = a.ws + d.ppart_off + ((int64_t)t.ppart * d.n + t.row0 + lane) * ri;
#pragma unroll
            for (int k = 0; k < R; ++k)
                if (k < ri) st_dev(dst + k, mine[k]);
        }
    }
    trace_mark(a, 1);
    if (active) {
        wave_mem_done();
        // the wavefront that brings the last column chunk of a strip adds the chunks (fixed order) into the
        // mean P rows of the strip (W = 1: the mean over workers is the value itself), kept in the P buffer
        int last = 0;
        if (lane == 0) {
            last = add_dev(cnt_s + t.cnts, 1u) == (unsigned)d.n_cchunk - 1u;
            if (last) add_dev(cnt_s + t.cnts, 0u - (unsigned)d.n_cchunk);
        }
        last = __builtin_amdgcn_readfirstlane(last);
        if (last) {
            const int nval = nrows * ri;                   // <= 128
            const float* src = a.ws + d.ppart_off + (int64_t)t.row0 * ri;
            float* dst = a.p + d.p_off + (int64_t)t.row0 * ri;
            const int64_t cstride = (int64_t)d.n * ri;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int idx = lane + kWave * u;
                if (idx < nval) {
                    float s = 0.f;
                    for (int c0 = 0; c0 < d.n_cchunk; c0 += 16) {
                        float v[16];
#pragma unroll
                        for (int cc = 0; cc < 16; ++cc) v[cc] = (c0 + cc < d.n_cchunk) ? ld_dev(src + (c0 + cc) * cstride + idx) : 0.f;
#pragma unroll
                        for (int cc = 0; cc < 16; ++cc) s += v[cc];
                    }
                    st_dev(dst + idx, s);
                }
            }
            wave_mem_done();
            // the wavefront that completes the last strip of a matrix orthogonalises its panel
            int last_m = 0;
            if (lane == 0) {
                last_m = add_dev(cnt_p + t.mat, 1u) == (unsigned)t.nstrips_mat - 1u;
                if (last_m) add_dev(cnt_p + t.mat, 0u - (unsigned)t.nstrips_mat);
            }
            last_m = __builtin_amdgcn_readfirstlane(last_m);
            if (last_m) {
                gram_schmidt_wave<R>(d, a.p + d.p_off);
                wave_mem_done();
                publish_flag(flags, fl_p, fp0 + 1u);
            }
        }
    }
    trace_mark(a, 2);
    if (active) wait_flag(flags, fl_p, copy, fp0, err_word);
    trace_mark(a, 3);

    // ---------------- phase B ----------------
    float pr[R];
#pragma unroll
    for (int k = 0; k < R; ++k)
        pr[k] = (lane < nrows && k < ri) ? ld_dev(a.p + d.p_off + (int64_t)(t.row0 + lane) * ri + k) : 0.f;
    float acc[V][R];
#pragma unroll
    for (int x = 0; x < V; ++x)
#pragma unroll
        for (int k = 0; k < R; ++k) acc[x][k] = 0.f;
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        if (i < nrows) {
#pragma unroll
            for (int k = 0; k < R; ++k) {
                const float pk = lane_bcast(pr[k], i);
#pragma unroll
                for (int x = 0; x < V; ++x) acc[x][k] = fmaf(M[i][x], pk, acc[x][k]);
            }
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
        float* qpart = a.ws + d.qpart_off;
        const int64_t mr = (int64_t)d.m * ri;
        if (valid) {
            float* dst = qpart + (int64_t)t.qpart * mr + (int64_t)col * ri;
#pragma unroll
            for (int x = 0; x < V; ++x)
#pragma unroll
                for (int k = 0; k < R; ++k)
                    if (k < ri) st_dev(dst + x * ri + k, acc[x][k]);
        }
        wave_mem_done();
        int last = 0;
        if (lane == 0) {
            unsigned* c = cnt_q + t.cntq;
            last = add_dev(c, 1u) == (unsigned)t.nqparts - 1u;
            if (last) add_dev(c, 0u - (unsigned)t.nqparts);
        }
        last = __builtin_amdgcn_readfirstlane(last);
        if (last && valid) {
            // add the runs' partials in run order; loads of four runs at a time are in flight together
            float* qdst = a.q + d.q_off + (int64_t)col * ri;
            const float* src = qpart + (int64_t)col * ri;
            float s[V][R];
#pragma unroll
            for (int x = 0; x < V; ++x)
#pragma unroll
                for (int k = 0; k < R; ++k) s[x][k] = 0.f;
            for (int p0 = 0; p0 < t.nqparts; p0 += 4) {
                float v[4][V][R];
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int x = 0; x < V; ++x)
#pragma unroll
                        for (int k = 0; k < R; ++k)
                            v[u][x][k] = (p0 + u < t.nqparts && k < ri) ? ld_dev(src + (int64_t)(p0 + u) * mr + x * ri + k) : 0.f;
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int x = 0; x < V; ++x)
#pragma unroll
                        for (int k = 0; k < R; ++k) s[x][k] += v[u][x][k];
            }
#pragma unroll
            for (int x = 0; x < V; ++x)
#pragma unroll
                for (int k = 0; k < R; ++k)
                    if (k < ri) st_dev(qdst + x * ri + k, s[x][k]);   // W = 1: the mean is the sum
        }
        if (last) {
            wave_mem_done();
            publish_flag(flags, fl_q, fq0 + 1u);
        }
    }
    trace_mark(a, 4);
    if (active) wait_flag(flags, fl_q, copy, fq0, err_word);
    trace_mark(a, 5);

    // ---------------- phase C ----------------
    float qb[V][R];
#pragma unroll
    for (int x = 0; x < V; ++x)
#pragma unroll
        for (int k = 0; k < R; ++k)
            qb[x][k] = (valid && k < ri) ? ld_dev(a.q + d.q_off + (int64_t)(col + x) * ri + k) : 0.f;
#pragma unroll
    for (int i = 0; i < RT; ++i) {
        if (i < nrows) {
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
                    en[x] = M[i][x] - s;
                }
                stv<V>(a.err + tile_off + (int64_t)i * d.m, en);
                stv<V>(a.out + tile_off + (int64_t)i * d.m, dl);
            }
        }
    }
    if (t.mat == -1) {
        // vector-shaped tensors, W = 1: Delta' is the gradient itself
        for (int64_t idx = t.elem0 + lane; idx < t.elem0 + t.nelem; idx += kWave)
            a.out[a.n_mat_elems + idx] = a.grad[a.n_mat_elems + idx];
    }
    trace_mark(a, 6);
}

template <int R>
__global__ __launch_bounds__(kBlock, 2) void k_resident(ResArgs a) {
    __shared__ float lds[kWavesPerBlock * 4 * R * kWave];
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const RTile t = a.tiles[blockIdx.x * kWavesPerBlock + wave];
    // all tiles of a workgroup use the same access width; the first slot is never idle
    const RTile t0 = a.tiles[blockIdx.x * kWavesPerBlock];
    const int vec = t0.mat >= 0 ? a.mats[t0.mat].vec : 4;
    if (vec == 4) resident_body<R, 4>(a, t, lds);
    else if (vec == 2) resident_body<R, 2>(a, t, lds);
    else resident_body<R, 1>(a, t, lds);
}

// ---- host side --------------------------------------------------------------------------------------------

template <int R>
static hipError_t launch_k_resident(const ResArgs& a, int blocks, hipStream_t s, int* max_blocks_per_cu) {
    if (max_blocks_per_cu) {
        hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(max_blocks_per_cu, k_resident<R>, kBlock, 0);
        if (e != hipSuccess) return e;
        return hipSuccess;
    }
    hipLaunchKernelGGL((k_resident<R>), dim3((unsigned)blocks), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

static hipError_t dispatch_resident(int rank, const ResArgs& a, int blocks, hipStream_t s, int* occ) {
    switch (rank) {
        case 1: return launch_k_resident<1>(a, blocks, s, occ);
        case 2: return launch_k_resident<2>(a, blocks, s, occ);
        case 3: return launch_k_resident<3>(a, blocks, s, occ);
        case 4: return launch_k_resident<4>(a, blocks, s, occ);
        default: return hipErrorInvalidValue;
    }
}

// Checks, once per plan, that the resident grid fits the device all at once.
psgd_status resident_check_device(psgd_plan* plan) {
    int dev = 0, cus = 0, occ = 0;
    if (hipGetDevice(&dev) != hipSuccess) return PSGD_EHIP;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return PSGD_EHIP;
    ResArgs dummy{};
    if (dispatch_resident(plan->rank, dummy, 0, nullptr, &occ) != hipSuccess) return PSGD_EHIP;
    if ((int64_t)cus * occ < plan->res_blocks) {
        plan->resident_ok = false;   // not co-resident on this device: the streaming path takes over
    }
    return PSGD_OK;
}

psgd_status launch_resident_step(psgd_plan* plan, const void* grad, float* err, float* q, float* p, void* out,
                                 void* workspace, void* stream) {
    if (!plan->uploaded) {
        psgd_status st = upload_tables(plan);
        if (st != PSGD_OK) return st;
        if (!plan->resident_ok) {   // upload found that the grid does not fit this device
            st = launch_compress(plan, grad, err, q, p, workspace, stream);
            if (st != PSGD_OK) return st;
            return launch_decompress(plan, p, q, err, grad, out, workspace, stream);
        }
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    ResArgs a{};
    a.mats = plan->dev.res_mats;
    a.tiles = plan->dev.res_tiles;
    a.grad = static_cast<const float*>(grad);
    a.err = err;
    a.q = q;
    a.p = p;
    a.out = static_cast<float*>(out);
    a.ws = static_cast<float*>(workspace);
    a.sync = plan->dev.res_sync;
    a.nblocks = plan->res_blocks;
    a.ngroups = (plan->res_blocks + kResBarrierFanIn - 1) / kResBarrierFanIn;
    a.n_mats = (int32_t)plan->mats.size();
    a.n_cntq = plan->res_n_cntq;
    a.n_cnts = plan->res_n_cnts;
    a.flags_at = plan->res_flags_at;
    a.n_mat_elems = plan->sizes.n_mat_elems;
    a.trace = plan->dev.res_trace;
    if (plan->profiling) {
        hipError_t e = hipEventRecord(static_cast<hipEvent_t>(plan->events[0]), s);
        if (e != hipSuccess) { plan->last_error = hipGetErrorString(e); return PSGD_EHIP; }
    }
    hipError_t e = dispatch_resident(plan->rank, a, plan->res_blocks, s, nullptr);
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
