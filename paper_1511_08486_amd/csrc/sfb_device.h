// Device-side helpers shared by the SFB kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sfb {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint16_t bf16_t;  // storage only: the upper 16 bits of an IEEE fp32

constexpr int kWave = 64;
constexpr int kXcds = 8;  // MI355X: 8 accelerator dies, each with its own L2

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Round to nearest, ties to even.  NaN stays NaN (quiet bit forced).
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// Four consecutive elements of one row starting at column `col`, widened to fp32.
// Elements at or beyond `ncols` read as 0.  `vec` promises that `row + col` is
// suitably aligned for a single wide load (checked on the host).
__device__ __forceinline__ f32x4 load4(const float* __restrict__ row, int64_t col, int64_t ncols, bool vec) {
    f32x4 r = {0.f, 0.f, 0.f, 0.f};
    if (vec && col + 3 < ncols) {
        r = *reinterpret_cast<const f32x4*>(row + col);
    } else {
        if (col + 0 < ncols) r.x = row[col + 0];
        if (col + 1 < ncols) r.y = row[col + 1];
        if (col + 2 < ncols) r.z = row[col + 2];
        if (col + 3 < ncols) r.w = row[col + 3];
    }
    return r;
}

__device__ __forceinline__ f32x4 load4(const bf16_t* __restrict__ row, int64_t col, int64_t ncols, bool vec) {
    f32x4 r = {0.f, 0.f, 0.f, 0.f};
    if (vec && col + 3 < ncols) {
        uint2 p = *reinterpret_cast<const uint2*>(row + col);
        r.x = __uint_as_float(p.x << 16);
        r.y = __uint_as_float(p.x & 0xffff0000u);
        r.z = __uint_as_float(p.y << 16);
        r.w = __uint_as_float(p.y & 0xffff0000u);
    } else {
        if (col + 0 < ncols) r.x = bf16_to_f32(row[col + 0]);
        if (col + 1 < ncols) r.y = bf16_to_f32(row[col + 1]);
        if (col + 2 < ncols) r.z = bf16_to_f32(row[col + 2]);
        if (col + 3 < ncols) r.w = bf16_to_f32(row[col + 3]);
    }
    return r;
}

// Four consecutive elements of row `row` starting at column `col`, for any alignment and any
// shape, without a branch: every element is loaded from an address clamped into the matrix
// (which must have at least one row and one column) and replaced by 0 if it lies outside.
// Independent scalar loads: slower per byte than load4's wide path, but all in flight at once.
__device__ __forceinline__ f32x4 load4_clamped(const float* __restrict__ base, int64_t row, int64_t ld, int64_t nrows,
                                               int64_t col, int64_t ncols) {
    const float* p = base + (row < nrows ? row : nrows - 1) * ld;
    const bool rin = row < nrows;
    f32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int64_t c = col + e;
        const float v = p[c < ncols ? c : ncols - 1];
        r[e] = (rin && c < ncols) ? v : 0.f;
    }
    return r;
}
__device__ __forceinline__ f32x4 load4_clamped(const bf16_t* __restrict__ base, int64_t row, int64_t ld, int64_t nrows,
                                               int64_t col, int64_t ncols) {
    const bf16_t* p = base + (row < nrows ? row : nrows - 1) * ld;
    const bool rin = row < nrows;
    f32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int64_t c = col + e;
        const float v = bf16_to_f32(p[c < ncols ? c : ncols - 1]);
        r[e] = (rin && c < ncols) ? v : 0.f;
    }
    return r;
}

// The same four clamped scalar loads WITHOUT the zeroing select: nothing is computed from the
// loaded words, so a prefetch can keep them in registers without the wait for them moving up
// to the loads.  The consumer masks the elements outside the matrix (in_matrix4) when it uses
// them.  bf16 comes back as its bit pattern, zero-extended by the load itself.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x4 load4_clamped_raw(const float* __restrict__ base, int64_t row, int64_t ld,
                                                   int64_t nrows, int64_t col, int64_t ncols) {
    const float* p = base + (row < nrows ? row : nrows - 1) * ld;
    f32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = p[col + e < ncols ? col + e : ncols - 1];
    return r;
}
__device__ __forceinline__ u32x4 load4_clamped_raw(const bf16_t* __restrict__ base, int64_t row, int64_t ld,
                                                   int64_t nrows, int64_t col, int64_t ncols) {
    const bf16_t* p = base + (row < nrows ? row : nrows - 1) * ld;
    u32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = p[col + e < ncols ? col + e : ncols - 1];
    return r;
}
__device__ __forceinline__ f32x4 widen4(u32x4 bits) {
    f32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = __uint_as_float(bits[e] << 16);
    return r;
}
// v with the elements at columns >= ncols (or all of it, if !row_ok) replaced by 0
__device__ __forceinline__ f32x4 in_matrix4(f32x4 v, bool row_ok, int64_t col, int64_t ncols) {
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = (row_ok && col + e < ncols) ? v[e] : 0.f;
    return v;
}

// Unguarded, aligned 4-element loads for the fast paths (the caller clamps the address
// into the matrix and discards what it must not use: no branches around memory ops).
__device__ __forceinline__ f32x4 ldg4(const float* __restrict__ p) { return *reinterpret_cast<const f32x4*>(p); }
__device__ __forceinline__ f32x4 ldg4(const bf16_t* __restrict__ p) {
    const uint2 q = *reinterpret_cast<const uint2*>(p);
    f32x4 r;
    r.x = __uint_as_float(q.x << 16);
    r.y = __uint_as_float(q.x & 0xffff0000u);
    r.z = __uint_as_float(q.y << 16);
    r.w = __uint_as_float(q.y & 0xffff0000u);
    return r;
}

// Raw (unconverted) 4-element loads: what a prefetch keeps in registers until it is staged.
template <typename T> struct RawOf;
template <> struct RawOf<float> { typedef f32x4 type; };
template <> struct RawOf<bf16_t> { typedef uint2 type; };
__device__ __forceinline__ f32x4 ldraw4(const float* __restrict__ p) { return *reinterpret_cast<const f32x4*>(p); }
__device__ __forceinline__ uint2 ldraw4(const bf16_t* __restrict__ p) { return *reinterpret_cast<const uint2*>(p); }
__device__ __forceinline__ f32x4 widen4(f32x4 v) { return v; }
__device__ __forceinline__ f32x4 widen4(uint2 q) {
    f32x4 r;
    r.x = __uint_as_float(q.x << 16);
    r.y = __uint_as_float(q.x & 0xffff0000u);
    r.z = __uint_as_float(q.y << 16);
    r.w = __uint_as_float(q.y & 0xffff0000u);
    return r;
}
// fp32 values that are exact bf16 (they were widened from bf16) back to their raw form
template <typename T> __device__ __forceinline__ typename RawOf<T>::type to_raw(f32x4 v);
template <> __device__ __forceinline__ f32x4 to_raw<float>(f32x4 v) { return v; }
template <> __device__ __forceinline__ uint2 to_raw<bf16_t>(f32x4 v) {
    uint2 q;
    q.x = (__float_as_uint(v.x) >> 16) | (__float_as_uint(v.y) & 0xffff0000u);
    q.y = (__float_as_uint(v.z) >> 16) | (__float_as_uint(v.w) & 0xffff0000u);
    return q;
}

// Entrywise proximal operator (Section 2.1), applied to an updated entry of W before it is
// stored: kind 0 none, 1 w * a (squared l2: a = 1 / (1 + eta lam)), 2 soft threshold at
// a = eta lam (l1).  `kind` is uniform over the launch.
__device__ __forceinline__ float prox_entry(float w, int kind, float a) {
    if (kind == 1) return w * a;
    if (kind == 2) return w > a ? w - a : (w < -a ? w + a : 0.f);
    return w;
}
__device__ __forceinline__ f32x4 prox_entry4(f32x4 w, int kind, float a) {
    if (kind == 0) return w;
    return f32x4{prox_entry(w.x, kind, a), prox_entry(w.y, kind, a), prox_entry(w.z, kind, a), prox_entry(w.w, kind, a)};
}

__device__ __forceinline__ void store4(float* __restrict__ row, int64_t col, int64_t ncols, bool vec, f32x4 v) {
    if (vec && col + 3 < ncols) {
        *reinterpret_cast<f32x4*>(row + col) = v;
    } else {
        if (col + 0 < ncols) row[col + 0] = v.x;
        if (col + 1 < ncols) row[col + 1] = v.y;
        if (col + 2 < ncols) row[col + 2] = v.z;
        if (col + 3 < ncols) row[col + 3] = v.w;
    }
}

__device__ __forceinline__ void store4(bf16_t* __restrict__ row, int64_t col, int64_t ncols, bool vec, f32x4 v) {
    if (vec && col + 3 < ncols) {
        uint2 p;
        p.x = (uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16);
        p.y = (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16);
        *reinterpret_cast<uint2*>(row + col) = p;
    } else {
        if (col + 0 < ncols) row[col + 0] = f32_to_bf16(v.x);
        if (col + 1 < ncols) row[col + 1] = f32_to_bf16(v.y);
        if (col + 2 < ncols) row[col + 2] = f32_to_bf16(v.z);
        if (col + 3 < ncols) row[col + 3] = f32_to_bf16(v.w);
    }
}

// Two fp32 values -> two bf16 (round to nearest even) packed in one word, first value in the low half.
typedef float sfb_f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 sfb_bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b) {
    const sfb_f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, sfb_bf16x2));
}
// Exact three-way split of two fp32 values into bf16 terms, x = h + m + l (3 x 8 significand bits
// cover fp32's 24; both differences are exact in fp32).  Outputs are packed pairs as cvt_pk_bf16.
__device__ __forceinline__ void split3_pair(float x0, float x1, uint32_t& h, uint32_t& m, uint32_t& l) {
    h = cvt_pk_bf16(x0, x1);
    const float r0 = x0 - __uint_as_float(h << 16), r1 = x1 - __uint_as_float(h & 0xffff0000u);
    m = cvt_pk_bf16(r0, r1);
    const float s0 = r0 - __uint_as_float(m << 16), s1 = r1 - __uint_as_float(m & 0xffff0000u);
    l = cvt_pk_bf16(s0, s1);
}

// LDS-DMA: one wavefront-wide instruction moves 64 x 16 bytes from per-lane global addresses
// to LDS; lane i lands at lds_addr + 16*i.  lds_addr must be wavefront-uniform (it travels in
// M0).  The compiler does not see the LDS write: the caller orders it by hand with
// wait_vmcnt (the vector-memory counter retires in order) and a barrier.
__device__ __forceinline__ void lds_dma16(const float* g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(g) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Workgroups are handed to the 8 dies round-robin by linear id.  Renumber so that each
// die owns one contiguous range of tile ids (tiles that share operands then share an L2).
__device__ __forceinline__ int xcd_contiguous_id(int linear_id, int total) {
    const int xcd = linear_id % kXcds;
    const int slot = linear_id / kXcds;
    const int q = total / kXcds, r = total % kXcds;
    return xcd * q + (xcd < r ? xcd : r) + slot;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

}  // namespace sfb
