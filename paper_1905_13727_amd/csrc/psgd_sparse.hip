// The two linear baselines of arXiv 1905.13727, Appendix G, that run inside the error-feedback loop of
// Algorithm 2 in the place of PowerSGD: "Random Block compression" and "Random K compression".
//
// Both keep b = (n + m) r entries of the flattened update M_w = g_w + e_w of each matrix (the same entries on
// every worker), average them over the workers, decompress to a matrix that is zero elsewhere, and leave
// e_w = M_w - decompressed in the error memory.  Only the kept entries couple the workers, and they are fewer
// than one in a hundred, so a step is two launches:
//
//   k_ef_add_zero   every element: M_w = g_w + e_w written over e_w, Delta' = 0 (by worker 0's workgroups); the
//                   vector-shaped tensors' mean.  A pure stream: 12 + 4 / W bytes per element and worker.
//   k_kept_entries  one lane per kept entry: mean over the workers of M_w at that position -> Delta', the packed
//                   value buffer, and e_w = M_w - mean for every worker.
//
// After the first launch the error memory of every position outside the kept set already holds its final value
// (nothing is sent from there: Delta' = 0, e_w = M_w).
#include <hip/hip_runtime.h>

#include <string>

#include "psgd_device.h"
#include "psgd_internal.h"

namespace psgd {

static_assert(kFlatTileElems == kBlock * 4, "one 16-byte access per lane and array");

// blockIdx.x: slice of kFlatTileElems elements; slices [first[i], first[i+1]) belong to matrix i, those from
// first[n_mats] on to the vector region.  blockIdx.y: worker.
__global__ __launch_bounds__(kBlock) void k_ef_add_zero(const MatDesc* __restrict__ mats, const int64_t* __restrict__ first,
                                                        int n_mats, const float* __restrict__ grad,
                                                        float* __restrict__ err, float* __restrict__ out, int workers,
                                                        int64_t gstride, int64_t estride, int64_t n_mat_elems,
                                                        int64_t n_vec_elems) {
    const int64_t slice = blockIdx.x;
    const int w = blockIdx.y;
    if (slice >= first[n_mats]) {
        // vector-shaped tensors: aggregated uncompressed (mean over the workers), no error memory
        if (w != 0) return;
        const float inv_w = 1.0f / (float)workers;
        const int64_t e0 = (slice - first[n_mats]) * kFlatTileElems;
        const int64_t e1 = e0 + kFlatTileElems < n_vec_elems ? e0 + kFlatTileElems : n_vec_elems;
        for (int64_t idx = e0 + threadIdx.x; idx < e1; idx += kBlock) {
            float s = 0.f;
            for (int ww = 0; ww < workers; ++ww) s += grad[(int64_t)ww * gstride + n_mat_elems + idx];
            out[n_mat_elems + idx] = s * inv_w;
        }
        return;
    }
    // the matrix this slice belongs to: the last i with first[i] <= slice (the same in every lane)
    int lo = 0, hi = n_mats - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (first[mid] <= slice) lo = mid;
        else hi = mid - 1;
    }
    const MatDesc d = mats[lo];
    const int64_t nm = (int64_t)d.n * d.m;
    const int64_t e0 = (slice - first[lo]) * kFlatTileElems;
    const int nelem = (int)(nm - e0 < kFlatTileElems ? nm - e0 : kFlatTileElems);
    const float* g = grad + (int64_t)w * gstride + d.off + e0;
    float* e = err + (int64_t)w * estride + d.off + e0;
    float* o = out + d.off + e0;
    // matrices start on multiples of 64 elements and slices on multiples of kFlatTileElems: the 16-byte accesses
    // are aligned; a matrix's last few elements (n m not a multiple of 4) go one by one
    const int v = threadIdx.x;
    if (4 * v + 4 <= nelem) {
        const f4 gv = __builtin_nontemporal_load(reinterpret_cast<const f4*>(g) + v);   // read once
        const f4 ev = reinterpret_cast<const f4*>(e)[v];
        reinterpret_cast<f4*>(e)[v] = gv + ev;
        if (w == 0) __builtin_nontemporal_store(f4{0.f, 0.f, 0.f, 0.f}, reinterpret_cast<f4*>(o) + v);
    } else {
        for (int i = 4 * v; i < nelem; ++i) {
            e[i] = g[i] + e[i];
            if (w == 0) o[i] = 0.f;
        }
    }
}

// blockIdx.x: a slice of kBlock kept entries of one matrix (tile: mat, elem0 = first entry, nelem = count)
__global__ __launch_bounds__(kBlock) void k_kept_entries(const MatDesc* __restrict__ mats, const int32_t* __restrict__ slice_mat,
                                                         const int64_t* __restrict__ slice_first,
                                                         const int32_t* __restrict__ mat_tensor,
                                                         float* __restrict__ err, float* __restrict__ out,
                                                         float* __restrict__ vals, const int64_t* __restrict__ starts,
                                                         const int64_t* __restrict__ indices, int workers,
                                                         int64_t estride) {
    const int mi = slice_mat[blockIdx.x];
    const MatDesc d = mats[mi];
    const int64_t j = slice_first[blockIdx.x] + threadIdx.x;   // entry of this matrix
    if (j >= d.kept) return;
    const int64_t nm = (int64_t)d.n * d.m;
    int64_t pos;
    if (starts) {
        // Random Block: the slice M(s : s + b), cut at the end of the vector
        int64_t s = starts[mat_tensor[mi]];
        s = s < 0 ? 0 : (s >= nm ? nm - 1 : s);
        pos = s + j;
    } else {
        pos = indices[d.kept_off + j];   // Random K: the j-th sampled position
    }
    if (pos < 0 || pos >= nm) {
        vals[d.kept_off + j] = 0.f;
        return;
    }
    float* e = err + d.off + pos;
    float s = 0.f;
    for (int w = 0; w < workers; ++w) s += e[(int64_t)w * estride];   // M_w as the first launch left it; worker order
    const float mean = s * (1.0f / (float)workers);
    vals[d.kept_off + j] = mean;
    out[d.off + pos] = mean;
    for (int w = 0; w < workers; ++w) e[(int64_t)w * estride] -= mean;
}

psgd_status launch_sparse_step(psgd_plan* plan, const void* grad, float* err, const int64_t* starts,
                               const int64_t* indices, float* vals, void* out, void* stream) {
    if (!plan->uploaded) {
        psgd_status st = upload_tables(plan);
        if (st != PSGD_OK) return st;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    auto mark = [&](int i) -> bool {   // measurement mode: an event before / between / after the two launches
        if (!plan->profiling) return true;
        hipError_t e = hipEventRecord(static_cast<hipEvent_t>(plan->events[i]), s);
        if (e != hipSuccess) plan->last_error = std::string("hipEventRecord: ") + hipGetErrorString(e);
        return e == hipSuccess;
    };
    if (!mark(0)) return PSGD_EHIP;
    const int64_t slices = plan->flat_tiles + plan->flat_vec_tiles;
    if (slices > 0x7fffffffLL) {
        plan->last_error = "baseline step: more than 2^31 slices of 1024 elements";
        return PSGD_EUNSUPPORTED;
    }
    if (slices > 0) {
        hipLaunchKernelGGL(k_ef_add_zero, dim3((unsigned)slices, (unsigned)plan->workers), dim3(kBlock), 0, s,
                           plan->dev.mats, plan->dev.flat_first, (int)plan->mats.size(), static_cast<const float*>(grad), err,
                           static_cast<float*>(out), plan->workers, plan->sizes.grad_stride, plan->sizes.err_stride,
                           plan->sizes.n_mat_elems, plan->sizes.n_vec_elems);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) { plan->last_error = std::string("launch k_ef_add_zero: ") + hipGetErrorString(e); return PSGD_EHIP; }
    }
    if (!mark(1)) return PSGD_EHIP;
    if (plan->kept_slices > 0) {
        hipLaunchKernelGGL(k_kept_entries, dim3((unsigned)plan->kept_slices), dim3(kBlock), 0, s, plan->dev.mats,
                           plan->dev.kept_slice_mat, plan->dev.kept_slice_first, plan->dev.mat_tensor, err,
                           static_cast<float*>(out), vals, starts, indices, plan->workers, plan->sizes.err_stride);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) { plan->last_error = std::string("launch k_kept_entries: ") + hipGetErrorString(e); return PSGD_EHIP; }
    }
    if (!mark(2)) return PSGD_EHIP;
    if (plan->profiling) {
        hipEvent_t ev[3] = {static_cast<hipEvent_t>(plan->events[0]), static_cast<hipEvent_t>(plan->events[1]),
                            static_cast<hipEvent_t>(plan->events[2])};
        float a = 0.f, b = 0.f;
        if (hipEventSynchronize(ev[2]) != hipSuccess || hipEventElapsedTime(&a, ev[0], ev[1]) != hipSuccess ||
            hipEventElapsedTime(&b, ev[1], ev[2]) != hipSuccess) {
            plan->last_error = "baseline step: event timing failed";
            return PSGD_EHIP;
        }
        plan->kernel_ms[PSGD_KERNEL_EF_ADD_ZERO] += a;
        plan->kernel_ms[PSGD_KERNEL_KEPT_ENTRIES] += b;
        ++plan->profiled_steps;
    }
    return PSGD_OK;
}

}  // namespace psgd
