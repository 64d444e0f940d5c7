// Device-side helpers shared by the gfx950 kernels of this library (storage types, packing,
// workgroup-to-XCD mapping).  Wave size is 64 everywhere.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hyena.h"

namespace hy {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// Storage element tags.
struct F32 {
    static constexpr int kBytes = 4;
};
struct BF16 {
    static constexpr int kBytes = 2;
};

// N 32-bit words moved with one memory instruction when N is 1, 2 or 4.
template <int N>
struct Words {
    uint32_t w[N];
};

template <int N>
__device__ __forceinline__ Words<N> load_words(const void* p) {
    Words<N> r;
    if constexpr (N == 4) {
        uint4 t = *reinterpret_cast<const uint4*>(p);
        r.w[0] = t.x; r.w[1] = t.y; r.w[2] = t.z; r.w[3] = t.w;
    } else if constexpr (N == 2) {
        uint2 t = *reinterpret_cast<const uint2*>(p);
        r.w[0] = t.x; r.w[1] = t.y;
    } else {
        static_assert(N == 1, "1, 2 or 4 words");
        r.w[0] = *reinterpret_cast<const uint32_t*>(p);
    }
    return r;
}

template <int N>
__device__ __forceinline__ void store_words(void* p, const Words<N>& r) {
    if constexpr (N == 4) {
        *reinterpret_cast<uint4*>(p) = make_uint4(r.w[0], r.w[1], r.w[2], r.w[3]);
    } else if constexpr (N == 2) {
        *reinterpret_cast<uint2*>(p) = make_uint2(r.w[0], r.w[1]);
    } else {
        static_assert(N == 1, "1, 2 or 4 words");
        *reinterpret_cast<uint32_t*>(p) = r.w[0];
    }
}

// Streaming variants: the non-temporal hint keeps once-touched activations from displacing other
// lines in L2 and the memory-side cache.  Measured on MI355X: a 3-read/1-write stream of 64 MiB arrays
// runs ~10% faster with the hint on both loads and stores.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

template <int N>
__device__ __forceinline__ Words<N> load_words_nt(const void* p) {
    Words<N> r;
    if constexpr (N == 4) {
        u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
        r.w[0] = t.x; r.w[1] = t.y; r.w[2] = t.z; r.w[3] = t.w;
    } else if constexpr (N == 2) {
        u32x2_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x2_t*>(p));
        r.w[0] = t.x; r.w[1] = t.y;
    } else {
        static_assert(N == 1, "1, 2 or 4 words");
        r.w[0] = __builtin_nontemporal_load(reinterpret_cast<const uint32_t*>(p));
    }
    return r;
}

template <int N>
__device__ __forceinline__ void store_words_nt(void* p, const Words<N>& r) {
    if constexpr (N == 4) {
        u32x4_t t = {r.w[0], r.w[1], r.w[2], r.w[3]};
        __builtin_nontemporal_store(t, reinterpret_cast<u32x4_t*>(p));
    } else if constexpr (N == 2) {
        u32x2_t t = {r.w[0], r.w[1]};
        __builtin_nontemporal_store(t, reinterpret_cast<u32x2_t*>(p));
    } else {
        static_assert(N == 1, "1, 2 or 4 words");
        __builtin_nontemporal_store(r.w[0], reinterpret_cast<uint32_t*>(p));
    }
}

template <int N>
__device__ __forceinline__ Words<N> zero_words() {
    Words<N> r;
#pragma unroll
    for (int i = 0; i < N; ++i) r.w[i] = 0u;
    return r;
}

// Two floats -> packed bf16 pair (round to nearest even, the hardware conversion of gfx950).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    f32x2_t x = {lo, hi};
    bf16x2_t b = __builtin_convertvector(x, bf16x2_t);
    return __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// VEC elements of storage type T <-> VEC floats.  VEC * bytes must be 2 (one bf16), 4, 8 or 16.
template <typename T, int VEC>
struct Pack {
    static constexpr int kBytes = VEC * T::kBytes;
    static constexpr int kWords = kBytes >= 4 ? kBytes / 4 : 1;
    using Raw = Words<kWords>;

    static __device__ __forceinline__ Raw load(const void* p) {
        if constexpr (kBytes == 2) {
            Raw r;
            r.w[0] = *reinterpret_cast<const uint16_t*>(p);
            return r;
        } else {
            return load_words<kWords>(p);
        }
    }
    static __device__ __forceinline__ void store(void* p, const Raw& r) {
        if constexpr (kBytes == 2) {
            *reinterpret_cast<uint16_t*>(p) = static_cast<uint16_t>(r.w[0]);
        } else {
            store_words<kWords>(p, r);
        }
    }
    // streaming (non-temporal) forms for data touched once
    static __device__ __forceinline__ Raw load_nt(const void* p) {
        if constexpr (kBytes == 2) {
            Raw r;
            r.w[0] = __builtin_nontemporal_load(reinterpret_cast<const uint16_t*>(p));
            return r;
        } else {
            return load_words_nt<kWords>(p);
        }
    }
    static __device__ __forceinline__ void store_nt(void* p, const Raw& r) {
        if constexpr (kBytes == 2) {
            __builtin_nontemporal_store(static_cast<uint16_t>(r.w[0]), reinterpret_cast<uint16_t*>(p));
        } else {
            store_words_nt<kWords>(p, r);
        }
    }
    static __device__ __forceinline__ void unpack(const Raw& r, float (&f)[VEC]) {
        if constexpr (T::kBytes == 4) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) f[i] = __uint_as_float(r.w[i]);
        } else if constexpr (VEC == 1) {
            f[0] = bf16_lo(r.w[0]);
        } else {
#pragma unroll
            for (int i = 0; i < VEC / 2; ++i) {
                f[2 * i] = bf16_lo(r.w[i]);
                f[2 * i + 1] = bf16_hi(r.w[i]);
            }
        }
    }
    static __device__ __forceinline__ Raw pack(const float (&f)[VEC]) {
        Raw r;
        if constexpr (T::kBytes == 4) {
#pragma unroll
            for (int i = 0; i < VEC; ++i) r.w[i] = __float_as_uint(f[i]);
        } else if constexpr (VEC == 1) {
            r.w[0] = pack_bf16x2(f[0], 0.0f) & 0xffffu;
        } else {
#pragma unroll
            for (int i = 0; i < VEC / 2; ++i) r.w[i] = pack_bf16x2(f[2 * i], f[2 * i + 1]);
        }
        return r;
    }
};

// Note on workgroup order: workgroups are dealt to the 8 XCDs round-robin by launch index.  Every kernel
// here keeps the plain launch order with the fastest-varying tile index along a row, so that all XCDs
// sweep one compact address window together; giving each XCD its own contiguous range of tiles was
// measured slower on MI355X for all of them (copy, stencil, MR).

}  // namespace hy
