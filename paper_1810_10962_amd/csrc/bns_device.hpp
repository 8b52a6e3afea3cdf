// Device-side building blocks: 128-bit vector access for fp32 / bf16 storage,
// wave64 and block reductions, and division by launch-uniform divisors.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bns {

constexpr int kWave = 64;     // gfx950 wavefront
constexpr int kBlock = 256;   // threads per block in every kernel (4 waves)

// ---------------------------------------------------------------------------
// Division of a 32-bit dividend (< 2^31) by a divisor fixed for the launch:
// round-up multiplier method (Granlund & Montgomery 1994).  q = (mulhi(n, mul) + n) >> shift.
// ---------------------------------------------------------------------------
struct FastDiv {
    uint32_t mul, shift, d;
};

inline FastDiv make_fastdiv(uint32_t d) {  // host; d >= 1
    FastDiv f;
    f.d = d;
    uint32_t l = 0;
    while ((uint64_t(1) << l) < d) ++l;     // ceil(log2 d)
    f.shift = l;
    f.mul = uint32_t(((uint64_t(1) << 32) * ((uint64_t(1) << l) - d)) / d + 1);
    return f;
}

__device__ __forceinline__ uint32_t fdiv(uint32_t n, const FastDiv& f) {
    return (__umulhi(n, f.mul) + n) >> f.shift;
}

// ---------------------------------------------------------------------------
// Storage types.  bf16 is handled as raw 16-bit patterns: widening is a shift,
// narrowing is the hardware conversion (round to nearest, ties to even; NaN stays NaN).
// ---------------------------------------------------------------------------
struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float bf16_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Two floats -> two bf16 packed in one dword (lo in bits 0..15): v_cvt_pk_bf16_f32 on gfx950.
typedef __bf16 bf16x2_native __attribute__((ext_vector_type(2)));
typedef float f32x2_native __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const f32x2_native v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_native));
}
__device__ __forceinline__ uint32_t f32_to_bf16(float f) { return pack_bf16x2(f, 0.f) & 0xFFFFu; }

// Vec<T, V>: V consecutive elements of storage type T, moved with one access of
// V * sizeof(T) bytes and exposed as V floats.
template <typename T, int V>
struct Vec;

template <>
struct Vec<float, 1> {
    float f[1];
    __device__ __forceinline__ void load(const float* p) { f[0] = *p; }
    __device__ __forceinline__ void load_nt(const float* p) { f[0] = __builtin_nontemporal_load(p); }
    __device__ __forceinline__ void store(float* p) const { *p = f[0]; }
    __device__ __forceinline__ void store_nt(float* p) const { __builtin_nontemporal_store(f[0], p); }
};

template <>
struct Vec<float, 4> {
    float f[4];
    typedef float v4 __attribute__((ext_vector_type(4)));
    __device__ __forceinline__ void load(const float* p) {
        v4 v = *reinterpret_cast<const v4*>(p);
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    __device__ __forceinline__ void load_nt(const float* p) {
        v4 v = __builtin_nontemporal_load(reinterpret_cast<const v4*>(p));
        f[0] = v.x; f[1] = v.y; f[2] = v.z; f[3] = v.w;
    }
    __device__ __forceinline__ void store(float* p) const {
        v4 v = {f[0], f[1], f[2], f[3]};
        *reinterpret_cast<v4*>(p) = v;
    }
    __device__ __forceinline__ void store_nt(float* p) const {
        v4 v = {f[0], f[1], f[2], f[3]};
        __builtin_nontemporal_store(v, reinterpret_cast<v4*>(p));
    }
};

template <>
struct Vec<bf16_t, 1> {
    float f[1];
    __device__ __forceinline__ void load(const bf16_t* p) { f[0] = bf16_to_f32(p->bits); }
    __device__ __forceinline__ void load_nt(const bf16_t* p) { load(p); }
    __device__ __forceinline__ void store(bf16_t* p) const { p->bits = uint16_t(f32_to_bf16(f[0])); }
    __device__ __forceinline__ void store_nt(bf16_t* p) const { store(p); }
};

template <>
struct Vec<bf16_t, 4> {
    float f[4];
    typedef uint32_t u2 __attribute__((ext_vector_type(2)));
    __device__ __forceinline__ void unpack(u2 v) {
        f[0] = bf16_to_f32(v.x & 0xFFFFu); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
        f[2] = bf16_to_f32(v.y & 0xFFFFu); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
    }
    __device__ __forceinline__ u2 pack() const {
        u2 v;
        v.x = pack_bf16x2(f[0], f[1]);
        v.y = pack_bf16x2(f[2], f[3]);
        return v;
    }
    __device__ __forceinline__ void load(const bf16_t* p) { unpack(*reinterpret_cast<const u2*>(p)); }
    __device__ __forceinline__ void load_nt(const bf16_t* p) {
        unpack(__builtin_nontemporal_load(reinterpret_cast<const u2*>(p)));
    }
    __device__ __forceinline__ void store(bf16_t* p) const { *reinterpret_cast<u2*>(p) = pack(); }
    __device__ __forceinline__ void store_nt(bf16_t* p) const {
        __builtin_nontemporal_store(pack(), reinterpret_cast<u2*>(p));
    }
};

template <>
struct Vec<bf16_t, 8> {
    float f[8];
    typedef uint32_t u4 __attribute__((ext_vector_type(4)));
    __device__ __forceinline__ void unpack(u4 v) {
        f[0] = bf16_to_f32(v.x & 0xFFFFu); f[1] = __uint_as_float(v.x & 0xFFFF0000u);
        f[2] = bf16_to_f32(v.y & 0xFFFFu); f[3] = __uint_as_float(v.y & 0xFFFF0000u);
        f[4] = bf16_to_f32(v.z & 0xFFFFu); f[5] = __uint_as_float(v.z & 0xFFFF0000u);
        f[6] = bf16_to_f32(v.w & 0xFFFFu); f[7] = __uint_as_float(v.w & 0xFFFF0000u);
    }
    __device__ __forceinline__ u4 pack() const {
        u4 v;
        v.x = pack_bf16x2(f[0], f[1]);
        v.y = pack_bf16x2(f[2], f[3]);
        v.z = pack_bf16x2(f[4], f[5]);
        v.w = pack_bf16x2(f[6], f[7]);
        return v;
    }
    __device__ __forceinline__ void load(const bf16_t* p) { unpack(*reinterpret_cast<const u4*>(p)); }
    __device__ __forceinline__ void load_nt(const bf16_t* p) {
        unpack(__builtin_nontemporal_load(reinterpret_cast<const u4*>(p)));
    }
    __device__ __forceinline__ void store(bf16_t* p) const { *reinterpret_cast<u4*>(p) = pack(); }
    __device__ __forceinline__ void store_nt(bf16_t* p) const {
        __builtin_nontemporal_store(pack(), reinterpret_cast<u4*>(p));
    }
};

template <typename T>
__device__ __forceinline__ float load_scalar(const T* p);
template <>
__device__ __forceinline__ float load_scalar<float>(const float* p) { return *p; }
template <>
__device__ __forceinline__ float load_scalar<bf16_t>(const bf16_t* p) { return bf16_to_f32(p->bits); }

// ---------------------------------------------------------------------------
// Reductions.  Wave: butterfly over the 64 lanes with cross-lane shuffles (fixed
// pattern, so the rounding order never changes).  Block: one value per wave through
// LDS, then the first wave adds the four in index order.
// ---------------------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// fp64 butterfly over the wave (fixed pattern): used by the finalize kernels, one wave per channel.
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// Sum of two values over a block of NT threads; result valid in thread 0.  `lds` holds
// 2 * (NT / kWave) floats.
template <int NT = kBlock>
__device__ __forceinline__ void block_sum2(float& a, float& b, float* lds) {
    a = wave_sum(a);
    b = wave_sum(b);
    const int wave = threadIdx.x / kWave, lane = threadIdx.x % kWave;
    constexpr int nw = NT / kWave;
    if (lane == 0) {
        lds[wave] = a;
        lds[nw + wave] = b;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float sa = lds[0], sb = lds[nw];
#pragma unroll
        for (int w = 1; w < nw; ++w) {
            sa += lds[w];
            sb += lds[nw + w];
        }
        a = sa;
        b = sb;
    }
}

}  // namespace bns
