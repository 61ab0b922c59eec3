// Device-side helpers shared by the streaming kernels and the resident kernel (gfx950).
#ifndef PSGD_DEVICE_H
#define PSGD_DEVICE_H

#include <hip/hip_runtime.h>

#include "psgd_internal.h"

namespace psgd {

typedef float f2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));

// ---- V-wide row accesses -----------------------------------------------------------------------

template <int V>
__device__ __forceinline__ void ldv(const float* p, float (&x)[V]);
template <>
__device__ __forceinline__ void ldv<1>(const float* p, float (&x)[1]) { x[0] = *p; }
template <>
__device__ __forceinline__ void ldv<2>(const float* p, float (&x)[2]) {
    f2 t = *reinterpret_cast<const f2*>(p);
    x[0] = t.x; x[1] = t.y;
}
template <>
__device__ __forceinline__ void ldv<4>(const float* p, float (&x)[4]) {
    f4 t = *reinterpret_cast<const f4*>(p);
    x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
}

// streamed-once data (the gradient): non-temporal so that it does not evict M from the caches
template <int V>
__device__ __forceinline__ void ldv_stream(const float* p, float (&x)[V]);
template <>
__device__ __forceinline__ void ldv_stream<1>(const float* p, float (&x)[1]) { x[0] = __builtin_nontemporal_load(p); }
template <>
__device__ __forceinline__ void ldv_stream<2>(const float* p, float (&x)[2]) {
    f2 t = __builtin_nontemporal_load(reinterpret_cast<const f2*>(p));
    x[0] = t.x; x[1] = t.y;
}
template <>
__device__ __forceinline__ void ldv_stream<4>(const float* p, float (&x)[4]) {
    f4 t = __builtin_nontemporal_load(reinterpret_cast<const f4*>(p));
    x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
}

template <int V>
__device__ __forceinline__ void stv(float* p, const float (&x)[V]);
template <>
__device__ __forceinline__ void stv<1>(float* p, const float (&x)[1]) { *p = x[0]; }
template <>
__device__ __forceinline__ void stv<2>(float* p, const float (&x)[2]) {
    f2 t; t.x = x[0]; t.y = x[1];
    *reinterpret_cast<f2*>(p) = t;
}
template <>
__device__ __forceinline__ void stv<4>(float* p, const float (&x)[4]) {
    f4 t; t.x = x[0]; t.y = x[1]; t.z = x[2]; t.w = x[3];
    *reinterpret_cast<f4*>(p) = t;
}

// written once and not read again soon (an error memory larger than the caches): non-temporal
template <int V>
__device__ __forceinline__ void stv_stream(float* p, const float (&x)[V]) {
    if constexpr (V == 4) {
        f4 t; t.x = x[0]; t.y = x[1]; t.z = x[2]; t.w = x[3];
        __builtin_nontemporal_store(t, reinterpret_cast<f4*>(p));
    } else if constexpr (V == 2) {
        f2 t; t.x = x[0]; t.y = x[1];
        __builtin_nontemporal_store(t, reinterpret_cast<f2*>(p));
    } else {
        __builtin_nontemporal_store(x[0], p);
    }
}

typedef float v4f __attribute__((ext_vector_type(4)));

// ---- buffer addressing ----------------------------------------------------------------------------------
// Raw buffer descriptors (base, byte range) let a wavefront address a tile with one 32-bit lane offset per
// access: a lane whose offset lies at or beyond the range reads zeros and its stores are dropped, so ragged
// tiles need no branches.  The whole address goes into the lane offset (the scalar offset operand is not
// part of the range check).  Ranges and offsets stay below 2^31 bytes (row lengths are limited when the
// plan is made), which makes kOutOfRange, and kOutOfRange plus any valid offset, out of range for every
// descriptor.
typedef __amdgpu_buffer_rsrc_t buf_rsrc;
typedef unsigned v4u __attribute__((ext_vector_type(4)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));
constexpr unsigned kOutOfRange = 0x80000000u;
constexpr int kRsrcFlags = 0x00020000;   // raw 32-bit data format word of gfx9-family descriptors

// base and bytes must be the same in every lane of the wavefront; they are moved to scalar registers here so
// that the descriptor is one (a descriptor held in vector registers makes every access a loop over its values)
__device__ __forceinline__ buf_rsrc make_rsrc(const void* base, int64_t bytes) {
    const unsigned long long b = reinterpret_cast<unsigned long long>(base);
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)b);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(b >> 32));
    const int nb = __builtin_amdgcn_readfirstlane((int)bytes);
    return __builtin_amdgcn_make_buffer_rsrc(reinterpret_cast<void*>(((unsigned long long)hi << 32) | lo), 0, nb, kRsrcFlags);
}
__device__ __forceinline__ float buf_load_f32(buf_rsrc r, unsigned off) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0));
}
__device__ __forceinline__ v4f buf_load_v4f(buf_rsrc r, unsigned off) {
    const v4u x = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
    return v4f{__uint_as_float(x.x), __uint_as_float(x.y), __uint_as_float(x.z), __uint_as_float(x.w)};
}
// the same two with a cache policy word (0: none, 2: non-temporal)
template <int AUX>
__device__ __forceinline__ v4f buf_load_v4f_policy(buf_rsrc r, unsigned off) {
    const v4u x = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, AUX);
    return v4f{__uint_as_float(x.x), __uint_as_float(x.y), __uint_as_float(x.z), __uint_as_float(x.w)};
}
template <int AUX>
__device__ __forceinline__ void buf_store_v4f_policy(buf_rsrc r, unsigned off, v4f v) {
    const v4u x{__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
    __builtin_amdgcn_raw_buffer_store_b128(x, r, (int)off, 0, AUX);
}
__device__ __forceinline__ void buf_store_v4f(buf_rsrc r, unsigned off, v4f v) {
    const v4u x{__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
    __builtin_amdgcn_raw_buffer_store_b128(x, r, (int)off, 0, 0);
}
// V consecutive floats through a descriptor (V = 1, 2, 4); `stream`: read once (non-temporal)
template <int V>
__device__ __forceinline__ void buf_ldv(buf_rsrc r, unsigned off, float (&x)[V], bool stream = false) {
    if constexpr (V == 4) {
        const v4u t = stream ? __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 2)
                             : __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
        x[0] = __uint_as_float(t.x); x[1] = __uint_as_float(t.y); x[2] = __uint_as_float(t.z); x[3] = __uint_as_float(t.w);
    } else if constexpr (V == 2) {
        const v2u t = stream ? __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, 2)
                             : __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, 0);
        x[0] = __uint_as_float(t.x); x[1] = __uint_as_float(t.y);
    } else {
        x[0] = __uint_as_float(stream ? __builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 2)
                                      : __builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 0));
    }
}
template <int V>
__device__ __forceinline__ void buf_stv(buf_rsrc r, unsigned off, const float (&x)[V]) {
    if constexpr (V == 4) {
        const v4u t{__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3])};
        __builtin_amdgcn_raw_buffer_store_b128(t, r, (int)off, 0, 0);
    } else if constexpr (V == 2) {
        const v2u t{__float_as_uint(x[0]), __float_as_uint(x[1])};
        __builtin_amdgcn_raw_buffer_store_b64(t, r, (int)off, 0, 0);
    } else {
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(x[0]), r, (int)off, 0, 0);
    }
}

// ---- bf16 gradients and output -----------------------------------------------------------------------------
typedef unsigned short bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float((unsigned)h << 16); }

// fp32 -> bf16, round to nearest even (NaN stays NaN): the conversion instruction of the matrix-core generation
typedef float v2f __attribute__((ext_vector_type(2)));
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
    const v2bf y = __builtin_convertvector(v2f{lo, hi}, v2bf);
    unsigned u;
    __builtin_memcpy(&u, &y, 4);
    return u;
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

// V consecutive gradient elements through a descriptor, read once (non-temporal); `off` in bytes.  BF: the
// gradient is stored as bf16: 8-, 4- or 2-byte loads of four, two or one value, widened exactly.
template <int V, bool BF>
__device__ __forceinline__ void buf_ld_grad(buf_rsrc r, unsigned off, float (&x)[V]) {
    if constexpr (BF) {
        if constexpr (V == 4) {
            const v2u t = __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, 2);
            x[0] = __uint_as_float(t.x << 16); x[1] = __uint_as_float(t.x & 0xffff0000u);
            x[2] = __uint_as_float(t.y << 16); x[3] = __uint_as_float(t.y & 0xffff0000u);
        } else if constexpr (V == 2) {
            const unsigned t = __builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, 2);
            x[0] = __uint_as_float(t << 16); x[1] = __uint_as_float(t & 0xffff0000u);
        } else {
            const unsigned t = (unsigned)(unsigned short)__builtin_amdgcn_raw_buffer_load_b16(r, (int)off, 0, 2);
            x[0] = __uint_as_float(t << 16);
        }
    } else {
        buf_ldv<V>(r, off, x, true);
    }
}

// V consecutive elements of the output at element index `at`; BF: stored as bf16 (round to nearest even).
// NT: non-temporal.
template <int V, bool BF, bool NT>
__device__ __forceinline__ void st_out(void* out, int64_t at, const float (&x)[V]) {
    if constexpr (BF) {
        bf16_t* base = static_cast<bf16_t*>(out) + at;
        if constexpr (V == 4) {
            typedef unsigned u2 __attribute__((ext_vector_type(2)));
            u2 t;
            t.x = pack_bf16x2(x[0], x[1]);
            t.y = pack_bf16x2(x[2], x[3]);
            u2* dst = reinterpret_cast<u2*>(base);
            if constexpr (NT) __builtin_nontemporal_store(t, dst);
            else *dst = t;
        } else if constexpr (V == 2) {
            const unsigned t = pack_bf16x2(x[0], x[1]);
            unsigned* dst = reinterpret_cast<unsigned*>(base);
            if constexpr (NT) __builtin_nontemporal_store(t, dst);
            else *dst = t;
        } else {
            const bf16_t t = f32_to_bf16(x[0]);
            if constexpr (NT) __builtin_nontemporal_store(t, base);
            else *base = t;
        }
    } else {
        if constexpr (NT) stv_stream<V>(static_cast<float*>(out) + at, x);
        else stv<V>(static_cast<float*>(out) + at, x);
    }
}

// Rows of a factor that belong to V consecutive matrix columns (or rows): the V * ri consecutive floats at
// `rows` -> f[V][R], zero beyond ri and everything zero when !valid.  With ri == R (the usual case; ri < R
// only for matrices smaller than the rank) they are fetched with the widest aligned vector loads instead of
// V * R scattered dwords.  `rows` must be 16-byte aligned when V * R is a multiple of 4, 8-byte aligned when
// it is even (factor offsets are multiples of 4 floats and the first column is a multiple of V).
template <int R, int V>
__device__ __forceinline__ void load_factor_rows(const float* rows, int ri, bool valid, float (&f)[V][R]) {
    constexpr int N = V * R;
    constexpr int WD = N % 4 == 0 ? 4 : (N % 2 == 0 ? 2 : 1);
    if (ri == R) {
        float buf[N];
        if (valid) {
#pragma unroll
            for (int j = 0; j < N / WD; ++j) {
                float t[WD];
                ldv<WD>(rows + WD * j, t);
#pragma unroll
                for (int x = 0; x < WD; ++x) buf[WD * j + x] = t[x];
            }
        } else {
#pragma unroll
            for (int j = 0; j < N; ++j) buf[j] = 0.f;
        }
#pragma unroll
        for (int x = 0; x < V; ++x)
#pragma unroll
            for (int k = 0; k < R; ++k) f[x][k] = buf[x * R + k];
    } else {
#pragma unroll
        for (int x = 0; x < V; ++x)
#pragma unroll
            for (int k = 0; k < R; ++k) f[x][k] = (valid && k < ri) ? rows[x * ri + k] : 0.f;
    }
}

// Algorithm 2, last two lines, for V consecutive elements whose momentum and parameter values have been loaded:
// m <- lambda m + Delta' ; x <- x - gamma (Delta' + m).
template <int V>
__device__ __forceinline__ void momentum_step(float (&m)[V], float (&x)[V], const float (&dl)[V], float lr, float lam) {
#pragma unroll
    for (int i = 0; i < V; ++i) {
        m[i] = fmaf(lam, m[i], dl[i]);
        x[i] = fmaf(-lr, dl[i] + m[i], x[i]);
    }
}

// ---- wavefront helpers ---------------------------------------------------------------------------

__device__ __forceinline__ float lane_bcast(float v, int src_lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), src_lane));
}

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}

// Sum over the 64 lanes, same value returned in every lane, fixed order: data-parallel-primitive
// adds inside each row of 16 lanes (lane^1, lane^2, mirrored 8, mirrored 16), then the four row
// sums are read out and added as (row0 + row1) + (row2 + row3).
__device__ __forceinline__ float wave_sum(float v) {
    v += dpp_mov<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_mov<0x141>(v);  // row_half_mirror
    v += dpp_mov<0x140>(v);  // row_mirror
    const float s0 = lane_bcast(v, 0), s1 = lane_bcast(v, 16), s2 = lane_bcast(v, 32), s3 = lane_bcast(v, 48);
    return (s0 + s1) + (s2 + s3);
}

template <int CTRL>
__device__ __forceinline__ double dpp_mov(double v) {
    const long long b = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xffffffffLL), CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xf, 0xf, true);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

__device__ __forceinline__ double lane_bcast(double v, int src_lane) {
    const long long b = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_readlane((int)(b & 0xffffffffLL), src_lane);
    const int hi = __builtin_amdgcn_readlane((int)(b >> 32), src_lane);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}

__device__ __forceinline__ double wave_sum(double v) {
    v += dpp_mov<0xB1>(v);
    v += dpp_mov<0x4E>(v);
    v += dpp_mov<0x141>(v);
    v += dpp_mov<0x140>(v);
    const double s0 = lane_bcast(v, 0), s1 = lane_bcast(v, 16), s2 = lane_bcast(v, 32), s3 = lane_bcast(v, 48);
    return (s0 + s1) + (s2 + s3);
}

// N sums over the 64 lanes at once: every lane brings N addends x[0..N-1]; on return lane L (L < N) holds the sum
// over all lanes of x[L].  Within each row of 16 lanes the values are handed over in halves (mirror, half mirror,
// the two quad swaps): a lane keeps the half whose index bit equals its own lane bit and adds its partner's copy
// of it, so 16 values per lane shrink to one in 15 exchanges instead of 16 separate reductions; the four rows'
// results are then added through two cross-lane reads.  Fixed order, the same in every call.
template <int N>
__device__ __forceinline__ float lane_sums(const float (&x)[N]) {
    static_assert(N >= 1 && N <= kWave, "one result per lane");
    constexpr int G = (N + 15) / 16;
    const int lane = threadIdx.x & (kWave - 1);
    const bool b3 = (lane & 8) != 0, b2 = (lane & 4) != 0, b1 = (lane & 2) != 0, b0 = (lane & 1) != 0;
    float res[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        float a16[16], a8[8], a4[4], a2[2];
#pragma unroll
        for (int j = 0; j < 16; ++j) a16[j] = 16 * g + j < N ? x[16 * g + j] : 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) a8[j] = (b3 ? a16[j + 8] : a16[j]) + dpp_mov<0x140>(b3 ? a16[j] : a16[j + 8]);   // row_mirror
#pragma unroll
        for (int j = 0; j < 4; ++j) a4[j] = (b2 ? a8[j + 4] : a8[j]) + dpp_mov<0x141>(b2 ? a8[j] : a8[j + 4]);       // row_half_mirror
#pragma unroll
        for (int j = 0; j < 2; ++j) a2[j] = (b1 ? a4[j + 2] : a4[j]) + dpp_mov<0x1B>(b1 ? a4[j] : a4[j + 2]);        // quad_perm [3,2,1,0]
        float v = (b0 ? a2[1] : a2[0]) + dpp_mov<0xB1>(b0 ? a2[0] : a2[1]);                                          // quad_perm [1,0,3,2]
        // lane L now holds, for index 16 g + (L & 15), the sum over its row of 16 lanes
        v += __int_as_float(__builtin_amdgcn_ds_bpermute((lane ^ 16) << 2, __float_as_int(v)));
        v += __int_as_float(__builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __float_as_int(v)));
        res[g] = v;
    }
    float out = res[0];
#pragma unroll
    for (int g = 1; g < G; ++g)
        if ((lane >> 4) == g) out = res[g];
    return out;
}

// rows [*begin, *begin + *count) of a tile's `total` rows that wavefront `wave` of 4 handles
__device__ __forceinline__ void wave_rows(int total, int wave, int* begin, int* count) {
    const int base = total / kWavesPerBlock, rem = total % kWavesPerBlock;
    *begin = wave * base + (wave < rem ? wave : rem);
    *count = base + (wave < rem ? 1 : 0);
}

// ---- accesses that are coherent across the whole GPU inside one kernel ----------------------------
//
// The eight accelerator dies have one L2 each.  Data that one workgroup writes and another reads
// within the same kernel goes through device-scope relaxed atomics: the store is written through
// to memory and the load is served from there, so no cache-wide write-back or invalidate is needed.

__device__ __forceinline__ float ld_dev(const float* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(float* p, float v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned ld_dev(const unsigned* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(unsigned* p, unsigned v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned add_dev(unsigned* p, unsigned v) {
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- mailbox: values that cross workgroups inside one kernel ---------------------------------------------
// A slot holds {value, tag} in 64 bits.  The producer writes the float together with the step's epoch in one
// 8-byte device-scope store, the consumer polls the slot with device-scope loads until the tag equals the
// epoch: the value is its own arrival flag, and no cache-wide write-back or invalidate is involved.  Every
// wait is bounded: after a limit of rounds the waiter writes the launch's epoch into an error word and goes on,
// so a kernel always ends.  The error word is only ever compared with the epoch of the running launch (a waiter
// that sees it gives up at once instead of timing out slot after slot): what an earlier launch left there does
// not shorten any wait of a later one.  The host reads the word as "some launch since the last check gave up".
typedef unsigned long long slot_t;
constexpr unsigned kSpinLimit = 1u << 21;   // default poll limit of the resident kernel's waits

__device__ __forceinline__ void post(slot_t* slot, float v, unsigned epoch) {
    const slot_t w = ((slot_t)epoch << 32) | (slot_t)__float_as_uint(v);
    __hip_atomic_store(slot, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Polling is written as: issue all loads of an attempt back to back (`fetch`, unconditional, so that
// no branch forces a wait between them; lanes or slots that are not wanted re-read a wanted one),
// then look at the tags.
__device__ __forceinline__ slot_t fetch(const slot_t* slot) {
    return __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ bool arrived(slot_t w, unsigned epoch) { return (unsigned)(w >> 32) == epoch; }
__device__ __forceinline__ float value_of(slot_t w) { return __uint_as_float((unsigned)(w & 0xffffffffULL)); }

// true when the wait should be abandoned: the limit is reached, or (looked at every 16 rounds, far longer than
// a wait lasts when all is well) another waiter of this launch has given up.  Uniform over the wavefront.
__device__ __forceinline__ bool give_up(unsigned spins, unsigned limit, const unsigned* err_word, unsigned epoch) {
    if (spins > limit) return true;
    if ((spins & 15u) != 0u) return false;
    unsigned seen = 0;
    if ((threadIdx.x & (kWave - 1)) == 0) seen = ld_dev(err_word);
    return __builtin_amdgcn_readfirstlane(seen) == epoch;
}

// Wait for a group of slots: every lane polls the slots it needs (`attempt()` returns true when all of
// them carry this step's tag) until the whole wavefront has them.  For the few wavefronts that reduce.
// All lanes of the wavefront call it together.
template <typename F>
__device__ __forceinline__ void await(F attempt, unsigned* err_word, unsigned epoch, unsigned limit) {
    unsigned spins = 0;
    for (;;) {
        const bool ok = attempt();
        if (__all(ok)) break;
        __builtin_amdgcn_s_sleep(2);
        if (give_up(++spins, limit, err_word, epoch)) {
            st_dev(err_word, epoch);
            break;
        }
    }
}

// Before a long wait: one lane watches a single slot (`probe`, the same address for the whole wavefront) at a
// relaxed pace, so that the waiting wavefronts put little load on the memory system (a wavefront that polls all its
// slots with all lanes also delays the loads of the other workgroup on its compute unit); once the slot carries this
// step's tag the rest is about to land and the caller polls the slots it needs with await().  False when the wait
// was given up.
__device__ __forceinline__ bool await_tag(const slot_t* probe, unsigned epoch, unsigned* err_word, unsigned limit) {
    unsigned spins = 0;
    for (;;) {
        unsigned tag = epoch;
        if ((threadIdx.x & (kWave - 1)) == 0)
            tag = (unsigned)(__hip_atomic_load(probe, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 32);
        if (__builtin_amdgcn_readfirstlane(tag) == epoch) return true;
        __builtin_amdgcn_s_sleep(6);
        if (give_up(++spins, limit, err_word, epoch)) {
            st_dev(err_word, epoch);
            return false;
        }
    }
}

// One slot, waited for by this lane alone (other lanes of the wavefront may be waiting for theirs).  Gives up after
// `limit` rounds, or as soon as another waiter of this launch has given up (the error word is looked at every 16
// rounds), so that a broken hand-over ends the kernel quickly.
__device__ __forceinline__ unsigned take_bits(const slot_t* slot, slot_t first, unsigned epoch, unsigned* err_word,
                                              unsigned limit) {
    slot_t w = first;
    unsigned spins = 0;
    while (!arrived(w, epoch)) {
        __builtin_amdgcn_s_sleep(2);
        w = fetch(slot);
        ++spins;
        if ((spins & 15u) == 0u && (spins > limit || ld_dev(err_word) == epoch)) {
            st_dev(err_word, epoch);
            break;
        }
    }
    return (unsigned)(w & 0xffffffffULL);
}

// A double travels as two slots (low word, high word), each with the tag.
__device__ __forceinline__ void post_double(slot_t* pair, double v, unsigned epoch) {
    const unsigned long long b = (unsigned long long)__double_as_longlong(v);
    __hip_atomic_store(pair, ((slot_t)epoch << 32) | (b & 0xffffffffULL), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(pair + 1, ((slot_t)epoch << 32) | (b >> 32), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double take_double(const slot_t* pair, slot_t first_lo, slot_t first_hi, unsigned epoch,
                                              unsigned* err_word, unsigned limit) {
    const unsigned lo = take_bits(pair, first_lo, epoch, err_word, limit);
    const unsigned hi = take_bits(pair + 1, first_hi, epoch, err_word, limit);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}

// Shared memory written by lanes of this wavefront is read by other lanes of the same wavefront (or the reverse)
// across this point: the wavefront's LDS operations complete in order, the compiler must not move them.
__device__ __forceinline__ void wave_lds_done() {
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

// Wait until every memory operation this wavefront has issued is complete (loads returned, stores
// acknowledged), and keep the compiler from moving memory operations across this point.
__device__ __forceinline__ void wave_mem_done() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_s_waitcnt(0);
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

}  // namespace psgd

#endif
