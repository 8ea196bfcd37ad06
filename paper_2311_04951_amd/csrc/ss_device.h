// Device-side building blocks shared by the kernels: 16-byte operand chunks, the MFMA wrappers for
// the two storage types, bf16 rounding and the hi/lo split of fp32 activations.
//
// Operand convention used by every contraction in this library (gfx950, wave64):
//   D[i][j] += sum_k A[i][k] * B[k][j]   with a 16x16 output tile per wavefront.
//   A = the operand streamed from HBM in its storage type (weights, cached keys, cached values),
//   B = the small fp32 "activation" operand (hidden rows, queries, softmax weights).
// Lane l = (c = l & 15, g = l >> 4) supplies, for one "k-block" of 4*E contraction indices,
//   A[i = c][k = g*E .. g*E+E-1]  and  B[k = g*E .. g*E+E-1][j = c]      (one 16-byte chunk each)
// and receives D[i = 4*g + v][j = c] in accumulator register v = 0..3.
//   bf16 storage: E = 8, one v_mfma_f32_16x16x32_bf16 per chunk pair; the fp32 activation is split
//                 into hi + lo bf16 parts (two MFMAs), which keeps ~16 mantissa bits of it.
//   f32 storage:  E = 4, four v_mfma_f32_16x16x4_f32 per chunk pair (exact fp32 products).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ss {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

struct bf16_t {
    uint16_t bits;
};

template <typename T> struct Traits;
template <> struct Traits<bf16_t> {
    static constexpr int E = 8;      // elements per 16-byte chunk
    static constexpr int PLANES = 2; // activation planes: hi, lo
};
template <> struct Traits<float> {
    static constexpr int E = 4;
    static constexpr int PLANES = 1;
};

__device__ __forceinline__ uint32_t f2u(float x) { return __builtin_bit_cast(uint32_t, x); }
__device__ __forceinline__ float u2f(uint32_t x) { return __builtin_bit_cast(float, x); }

// fp32 -> bf16, round to nearest even (finite inputs; NaN/Inf pass through the high half).
__device__ __forceinline__ uint32_t bf16_rne(float x) {
    uint32_t u = f2u(x);
    if ((u & 0x7f800000u) == 0x7f800000u) return u >> 16;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return u2f(b << 16); }

__device__ __forceinline__ float to_f32(bf16_t x) { return bf16_bits_to_f32(x.bits); }
__device__ __forceinline__ float to_f32(float x) { return x; }

template <typename T> __device__ __forceinline__ T to_storage(float x);
template <> __device__ __forceinline__ bf16_t to_storage<bf16_t>(float x) { return bf16_t{(uint16_t)bf16_rne(x)}; }
template <> __device__ __forceinline__ float to_storage<float>(float x) { return x; }

__device__ __forceinline__ u32x4 ld16(const void *p) { return *reinterpret_cast<const u32x4 *>(p); }
// non-temporal load.  Measured on the 7B-shaped layer: where a wave-level load covers half of each 128-byte line
// it touches (16 rows x 64 bytes: the MFMA operand layout of bf16 and int8 matrices and of the cache) the plain
// load is the faster one (the other half of the line, asked for by the next instruction or by a neighbouring wave,
// then hits; the counters showed 20 to 40 % more bytes fetched with the non-temporal form), so only the int4
// kernel, whose loads cover whole lines, still uses this.
__device__ __forceinline__ u32x4 ld16_stream(const void *p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}
// 16-byte load through a pointer that is known to be global memory although the compiler cannot see
// it (pointers read from a descriptor in memory are generic): keeps it a global_load, not a flat_load,
// which matters for wait counting (flat loads can return out of order and force vmcnt(0))
__device__ __forceinline__ u32x4 ld16_global(const void *p) {
    typedef const u32x4 __attribute__((address_space(1))) * gptr;
    return *(gptr)(p);
}
__device__ __forceinline__ float ldf_global(const float *p) {
    typedef const float __attribute__((address_space(1))) * gptr;
    return *(gptr)(p);
}
__device__ __forceinline__ u32x4 zero16() { return u32x4{0u, 0u, 0u, 0u}; }

// The activation (B) operand of one k-block.
template <typename T> struct Act {
    u32x4 p[Traits<T>::PLANES];
};

// Activation planes in memory: element (row, col) of plane pl lives at base[pl*plane + row*ld + col].
template <typename T> struct ActPlanes {
    T *base;
    size_t plane; // elements between planes
    int ld;       // elements between rows
};

template <typename T> __device__ __forceinline__ Act<T> load_act(const ActPlanes<T> &a, size_t off) {
    Act<T> r;
#pragma unroll
    for (int pl = 0; pl < Traits<T>::PLANES; ++pl) r.p[pl] = ld16(a.base + pl * a.plane + off);
    return r;
}
template <typename T> __device__ __forceinline__ Act<T> zero_act() {
    Act<T> r;
#pragma unroll
    for (int pl = 0; pl < Traits<T>::PLANES; ++pl) r.p[pl] = zero16();
    return r;
}

// store one fp32 activation value as planes (bf16: hi + lo; f32: itself)
__device__ __forceinline__ void store_act(const ActPlanes<bf16_t> &a, size_t off, float x) {
    uint32_t hi = bf16_rne(x);
    uint32_t lo = bf16_rne(x - bf16_bits_to_f32(hi));
    a.base[off].bits = (uint16_t)hi;
    a.base[a.plane + off].bits = (uint16_t)lo;
}
__device__ __forceinline__ void store_act(const ActPlanes<float> &a, size_t off, float x) { a.base[off] = x; }

// pack E fp32 values held by one lane into the activation operand of a k-block
__device__ __forceinline__ Act<bf16_t> pack_act(const float (&x)[8], bf16_t) {
    Act<bf16_t> r;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        uint32_t h0 = bf16_rne(x[2 * j]), h1 = bf16_rne(x[2 * j + 1]);
        uint32_t l0 = bf16_rne(x[2 * j] - bf16_bits_to_f32(h0));
        uint32_t l1 = bf16_rne(x[2 * j + 1] - bf16_bits_to_f32(h1));
        r.p[0][j] = h0 | (h1 << 16);
        r.p[1][j] = l0 | (l1 << 16);
    }
    return r;
}
__device__ __forceinline__ Act<float> pack_act(const float (&x)[4], float) {
    Act<float> r;
#pragma unroll
    for (int j = 0; j < 4; ++j) r.p[0][j] = f2u(x[j]);
    return r;
}

// acc[i][j] += sum over the k-block of a[i][k] * b[k][j]
__device__ __forceinline__ f32x4 mma(f32x4 acc, u32x4 a, const Act<bf16_t> &b) {
    bf16x8 av = __builtin_bit_cast(bf16x8, a);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, b.p[0]), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, b.p[1]), acc, 0, 0, 0);
    return acc;
}
__device__ __forceinline__ f32x4 mma(f32x4 acc, u32x4 a, const Act<float> &b) {
#pragma unroll
    for (int j = 0; j < 4; ++j) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(u2f(a[j]), u2f(b.p[0][j]), acc, 0, 0, 0);
    return acc;
}

// ---- agent-coherent accesses ------------------------------------------------------------------
// Data that one workgroup writes and another reads INSIDE one kernel (persistent verify kernel) is
// moved with relaxed agent-scope atomics: they are performed at the memory side, so no cache
// write-back / invalidate is needed at the device-wide barriers (the L2 of each XCD is private).
__device__ __forceinline__ float ld_coh(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_coh(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_coh(bf16_t *p, bf16_t v) {
    __hip_atomic_store(reinterpret_cast<uint16_t *>(p), v.bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long ld_coh64(const void *p) {
    return __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// 16-byte chunk as two coherent 8-byte loads
__device__ __forceinline__ u32x4 ld16_coh(const void *p) {
    const unsigned long long a = ld_coh64(p), b = ld_coh64(reinterpret_cast<const char *>(p) + 8);
    return u32x4{(uint32_t)a, (uint32_t)(a >> 32), (uint32_t)b, (uint32_t)(b >> 32)};
}
// 16-byte agent-coherent load (sc0 sc1: performed at the memory side, like the relaxed agent-scope
// atomics above, but four dwords per lane) through a raw buffer resource over `base`; `byte_off` < 4 GiB
__device__ __forceinline__ u32x4 ld16_coh_buf(const void *base, uint32_t byte_off) {
    const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, 0x7fffffff, 0x00020000);
    return __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 1 | 16);
}
template <typename T> __device__ __forceinline__ Act<T> load_act_coh(const ActPlanes<T> &a, size_t off) {
    Act<T> r;
#pragma unroll
    for (int pl = 0; pl < Traits<T>::PLANES; ++pl) r.p[pl] = ld16_coh_buf(a.base, (uint32_t)((pl * a.plane + off) * sizeof(T)));
    return r;
}
// The all-ones bit pattern is reserved (the persistent kernel uses it for "not written yet"): a NaN
// that happens to carry it is stored as another NaN.
__device__ __forceinline__ void store_act_coh(const ActPlanes<bf16_t> &a, size_t off, float x) {
    uint32_t hi = bf16_rne(x);
    uint32_t lo = bf16_rne(x - bf16_bits_to_f32(hi));
    hi = hi == 0xffffu ? 0xffc0u : hi;
    lo = lo == 0xffffu ? 0xffc0u : lo;
    st_coh(a.base + off, bf16_t{(uint16_t)hi});
    st_coh(a.base + a.plane + off, bf16_t{(uint16_t)lo});
}
__device__ __forceinline__ void store_act_coh(const ActPlanes<float> &a, size_t off, float x) {
    st_coh(a.base + off, f2u(x) == 0xffffffffu ? u2f(0xffc00000u) : x);
}

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o);
    return x;
}

} // namespace ss
