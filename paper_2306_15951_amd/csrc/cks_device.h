// Shared device-side definitions for the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>

namespace cks {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;  // four 64-lane wavefronts per workgroup, one per SIMD
constexpr int kXcds = 8;       // MI355X: 8 accelerator dies, each with its own L2

// Mathematical ceiling of a / b for b > 0 and any a.
__host__ __device__ inline int cdiv_any(int a, int b) { return a >= 0 ? (a + b - 1) / b : -((-a) / b); }

// v_mfma_f32_32x32x2_f32:  D(32x32) += A(32x2) * B(2x32).
// Lane l supplies A[l%32][l/32] and B[l/32][l%32]; register r of D in lane l is
// D[8*(r/4) + 4*(l/32) + r%4][l%32].
__device__ inline floatx16 mfma32(float a, float b, floatx16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

// Division of a non-negative 31-bit number by a divisor fixed on the host: one multiply-high and a
// shift.  The compiler's own expansion of a division by a kernel argument runs through the float
// reciprocal on the vector ALU even for wave-uniform operands, and vector ALU time is MFMA time.
// mul = ceil(2^(31 + ceil(log2 d)) / d), shr = ceil(log2 d) - 1  (d >= 2); exact for 0 <= x < 2^31.
struct FastDiv {
    int d;
    unsigned mul, shr;
};
inline FastDiv make_fastdiv(int d)
{
    FastDiv f{d, 0u, 0u};
    if (d > 1) {
        unsigned lg = 0;
        while ((1ll << lg) < d) ++lg;
        const unsigned long long p2 = 1ull << (31 + lg);
        f.mul = (unsigned)((p2 + (unsigned long long)d - 1) / (unsigned long long)d);
        f.shr = lg - 1;
    }
    return f;
}
__device__ inline int fdiv(int x, const FastDiv &f) { return f.d == 1 ? x : (int)(__umulhi((unsigned)x, f.mul) >> f.shr); }
__device__ inline int fmod(int x, const FastDiv &f) { return x - fdiv(x, f) * f.d; }

// Workgroups are handed to the 8 dies round-robin.  Map the hardware block id
// to a work item so that each die gets one contiguous range of work items;
// neighbours in that order share operands and therefore that die's L2.
__device__ inline int xcd_contiguous_work(int bid, int per_xcd) { return (bid % kXcds) * per_xcd + bid / kXcds; }

// 4 consecutive floats from p, elements at or beyond `valid` replaced by 0 and
// never read.  VEC: p is 16-byte aligned and valid is a multiple of 4.
template <bool VEC>
__device__ inline float4 load4(const float *p, int valid)
{
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (VEC) {
        if (valid > 0) v = *reinterpret_cast<const float4 *>(p);
    } else {
        if (valid > 0) v.x = p[0];
        if (valid > 1) v.y = p[1];
        if (valid > 2) v.z = p[2];
        if (valid > 3) v.w = p[3];
    }
    return v;
}

}  // namespace cks
