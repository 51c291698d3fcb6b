// Device-side helpers shared by the HIP kernels (gfx950 / CDNA4, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace anr {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;

// v_mfma_f32_32x32x2_f32: D(32x32) += A(32x2) * B(2x32), fp32 throughout.
// Lane l supplies A[i = l%32][k = l/32] and B[k = l/32][j = l%32].
// Register r of lane l holds D[i = 8*(r/4) + 4*(l/32) + r%4][j = l%32].
__device__ __forceinline__ f32x16 mfma32(float a, float b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// v_mfma_f32_16x16x4_f32: D(16x16) += A(16x4) * B(4x16).
// Lane l supplies A[i = l%16][k = l/16] and B[k = l/16][j = l%16].
// Register r of lane l holds D[i = 4*(l/16) + r][j = l%16].
__device__ __forceinline__ f32x4 mfma16(float a, float b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x4 ldg4(const float* p)
{
    return *reinterpret_cast<const f32x4*>(p);
}

__device__ __forceinline__ void stg4(float* p, f32x4 v)
{
    *reinterpret_cast<f32x4*>(p) = v;
}

// Non-temporal store of a result that the kernel never reads again.  An ordinary store leaves
// the line dirty in L2, and all dirty lines are written back when the kernel ends: a serial tail
// that a 25 MB stream pays with 6.8 instead of 5.4 us (copy) or 9.4 instead of 7.0 us (the TBS batch
// matmul).  Only for stores that cover whole 128-byte lines per instruction: scattered 16-byte pieces
// were measured slower this way (the 56x56 convolution: 43.7 against 38.8 us), since they lose the
// write combining L2 gives them.
__device__ __forceinline__ void stg4_nt(float* p, f32x4 v)
{
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(p));
}
// the same policy as the `aux` operand of a raw buffer store (the nt bit of gfx950's cache policy)
constexpr int kBufferNonTemporal = 2;

__device__ __forceinline__ f32x4 zero4()
{
    f32x4 z = {0.f, 0.f, 0.f, 0.f};
    return z;
}

// Kernel arguments are read through the scalar cache, and the compiler fetches each where it is
// first used: a kernel with large argument structs starts with several dependent round trips to
// memory and nothing else to do meanwhile.  This requests one word of each 64-byte line of the
// first BYTES bytes of the argument block in one go and waits for them; the compiler's own reads
// then hit the scalar cache.  The loads and their wait are one asm statement, so the registers
// they write stay reserved until the data is there.
template <int BYTES>
__device__ __forceinline__ void touch_kernel_arguments()
{
    constexpr int LINES = (BYTES + 63) / 64;
    static_assert(LINES >= 1 && LINES <= 8, "one to eight lines");
    auto ka = __builtin_amdgcn_kernarg_segment_ptr();
    uint32_t t[8];
    if constexpr (LINES == 8)
        asm volatile(
                     "s_load_dword %0, %8, 0x0\n\t"
                     "s_load_dword %1, %8, 0x40\n\t"
                     "s_load_dword %2, %8, 0x80\n\t"
                     "s_load_dword %3, %8, 0xc0\n\t"
                     "s_load_dword %4, %8, 0x100\n\t"
                     "s_load_dword %5, %8, 0x140\n\t"
                     "s_load_dword %6, %8, 0x180\n\t"
                     "s_load_dword %7, %8, 0x1c0\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&s"(t[0]), "=&s"(t[1]), "=&s"(t[2]), "=&s"(t[3]), "=&s"(t[4]), "=&s"(t[5]), "=&s"(t[6]), "=&s"(t[7])
                     : "s"(ka)
                     : "memory");
    else if constexpr (LINES == 7)
        asm volatile(
                     "s_load_dword %0, %7, 0x0\n\t"
                     "s_load_dword %1, %7, 0x40\n\t"
                     "s_load_dword %2, %7, 0x80\n\t"
                     "s_load_dword %3, %7, 0xc0\n\t"
                     "s_load_dword %4, %7, 0x100\n\t"
                     "s_load_dword %5, %7, 0x140\n\t"
                     "s_load_dword %6, %7, 0x180\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&s"(t[0]), "=&s"(t[1]), "=&s"(t[2]), "=&s"(t[3]), "=&s"(t[4]), "=&s"(t[5]), "=&s"(t[6])
                     : "s"(ka)
                     : "memory");
    else if constexpr (LINES == 6)
        asm volatile(
                     "s_load_dword %0, %6, 0x0\n\t"
                     "s_load_dword %1, %6, 0x40\n\t"
                     "s_load_dword %2, %6, 0x80\n\t"
                     "s_load_dword %3, %6, 0xc0\n\t"
                     "s_load_dword %4, %6, 0x100\n\t"
                     "s_load_dword %5, %6, 0x140\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&s"(t[0]), "=&s"(t[1]), "=&s"(t[2]), "=&s"(t[3]), "=&s"(t[4]), "=&s"(t[5])
                     : "s"(ka)
                     : "memory");
    else if constexpr (LINES == 5)
        asm volatile(
                     "s_load_dword %0, %5, 0x0\n\t"
                     "s_load_dword %1, %5, 0x40\n\t"
                     "s_load_dword %2, %5, 0x80\n\t"
                     "s_load_dword %3, %5, 0xc0\n\t"
                     "s_load_dword %4, %5, 0x100\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&s"(t[0]), "=&s"(t[1]), "=&s"(t[2]), "=&s"(t[3]), "=&s"(t[4])
                     : "s"(ka)
                     : "memory");
    else if constexpr (LINES == 4)
        asm volatile(
                     "s_load_dword %0, %4, 0x0\n\t"
                     "s_load_dword %1, %4, 0x40\n\t"
                     "s_load_dword %2, %4, 0x80\n\t"
                     "s_load_dword %3, %4, 0xc0\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&s"(t[0]), "=&s"(t[1]), "=&s"(t[2]), "=&s"(t[3])
                     : "s"(ka)
                     : "memory");
    else if constexpr (LINES == 3)
        asm volatile(
                     "s_load_dword %0, %3, 0x0\n\t"
                     "s_load_dword %1, %3, 0x40\n\t"
                     "s_load_dword %2, %3, 0x80\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&s"(t[0]), "=&s"(t[1]), "=&s"(t[2])
                     : "s"(ka)
                     : "memory");
    else if constexpr (LINES == 2)
        asm volatile(
                     "s_load_dword %0, %2, 0x0\n\t"
                     "s_load_dword %1, %2, 0x40\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&s"(t[0]), "=&s"(t[1])
                     : "s"(ka)
                     : "memory");
    else if constexpr (LINES == 1)
        asm volatile(
                     "s_load_dword %0, %1, 0x0\n\t"
                     "s_waitcnt lgkmcnt(0)"
                     : "=&s"(t[0])
                     : "s"(ka)
                     : "memory");
}

// floor(n / d) for 0 <= n < 2^31 as one multiply-high and one shift (Granlund-Montgomery
// round-up method: mul = ceil(2^(31+l) / d), l = ceil(log2 d), quotient = (n*mul) >> (31+l)).
struct FastDiv {
    uint32_t mul, shr;
    __device__ __forceinline__ int div(int n) const
    {
        return mul ? (int)(__umulhi((uint32_t)n, mul) >> shr) : n;
    }
};

inline FastDiv make_fastdiv(int d)
{
    FastDiv f{0u, 0u};
    if (d <= 1) return f;
    int l = 0;
    while ((1ll << l) < d) ++l;
    f.mul = (uint32_t)((((uint64_t)1 << (31 + l)) + (uint64_t)d - 1) / (uint64_t)d);
    f.shr = (uint32_t)(l - 1);
    return f;
}

}  // namespace anr
