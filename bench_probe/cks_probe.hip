// Measurement probes for the benchmark (not part of the operators' path): what the fp32 matrix cores of
// this chip sustain with operands that are not constants, and the shader clock while a kernel runs.
// Built into bench_probe/libcks_probe.so by the package's build step; see cks_probe.h.
#include "cks_probe.h"

#include <hip/hip_runtime.h>

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ inline float pseudo_random(unsigned i)   // in [-1, 1): values only have to differ, bit patterns toggle
{
    i = i * 2654435761u + 12345u;
    i ^= i >> 15;
    i *= 2246822519u;
    i ^= i >> 13;
    return (float)(int)(i & 0xffff) / 32768.f - 1.f;
}

// Two independent accumulator chains per wave, operands in registers: the matrix pipe alone.
__global__ void __launch_bounds__(256) mfma_registers(float *out, int iters, int random)
{
    float a[4], b[4];
    for (int e = 0; e < 4; ++e) {
        a[e] = random ? pseudo_random(threadIdx.x * 8 + e + blockIdx.x * 4096) : 1.0f;
        b[e] = random ? pseudo_random(threadIdx.x * 8 + 4 + e + blockIdx.x * 4096) : 1.0f;
    }
    floatx16 acc0, acc1;
    for (int r = 0; r < 16; ++r) { acc0[r] = 0.f; acc1[r] = 0.f; }
    for (int t = 0; t < iters; ++t) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], b[e], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(b[e], a[e], acc1, 0, 0, 0);
        }
    }
    float s = 0.f;
    for (int r = 0; r < 16; ++r) s += acc0[r] + acc1[r];
    if (s == 123.456f) out[threadIdx.x] = s;   // never true for these inputs; keeps the loop alive
}

// The K loop of the general kernels without its global side: per chunk of 32, four 16-byte fragment
// reads per operand from a [64][36] LDS tile feed 16 MFMAs of one 32x32 accumulator; a workgroup barrier
// per chunk.  `items` work items of `chunks` chunks per workgroup.
constexpr int LDK = 36, BM = 64, BN = 64;
__global__ void __launch_bounds__(256) mfma_lds(float *out, int chunks, int items, int random)
{
    extern __shared__ __align__(16) float smem[];
    float *As = smem, *Bs = smem + 2 * BM * LDK;
    for (int i = threadIdx.x; i < 2 * (BM + BN) * LDK; i += 256) smem[i] = random ? pseudo_random(i + blockIdx.x * 77777) : 1.0f;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, wm = wave >> 1, wn = wave & 1;
    const int frow = lane & 31, fk = (lane >> 5) * 4;
    const float *Ar = As + (wm * 32 + frow) * LDK + fk, *Br = Bs + (wn * 32 + frow) * LDK + fk;
    float s = 0.f;
    for (int it = 0; it < items; ++it) {
        floatx16 acc;
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        for (int t = 0; t < chunks; t += 2) {
#pragma unroll
            for (int buf = 0; buf < 2; ++buf) {
                float4 a = *reinterpret_cast<const float4 *>(Ar + buf * BM * LDK), b = *reinterpret_cast<const float4 *>(Br + buf * BN * LDK);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    float4 an = a, bn = b;
                    if (kk < 3) {
                        an = *reinterpret_cast<const float4 *>(Ar + buf * BM * LDK + (kk + 1) * 8);
                        bn = *reinterpret_cast<const float4 *>(Br + buf * BN * LDK + (kk + 1) * 8);
                    }
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
                    if (kk < 3) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
                    a = an; b = bn;
                }
                __syncthreads();
            }
        }
        for (int r = 0; r < 16; ++r) s += acc[r];
    }
    if (s == 123.456f) out[threadIdx.x] = s;
}

// One lane samples the 100 MHz wall clock and the shader clock counter n times, sleeping in between.
__global__ void clock_samples(long long *buf, int n, int sleeps)
{
    if (threadIdx.x != 0) return;
    for (int i = 0; i < n; ++i) {
        buf[2 * i] = wall_clock64();
        buf[2 * i + 1] = clock64();
        for (int j = 0; j < sleeps; ++j) __builtin_amdgcn_s_sleep(127);
    }
}

inline int done() { return hipGetLastError() == hipSuccess ? 0 : -4; }

}  // namespace

extern "C" {

int cks_probe_mfma_registers(float *out, int blocks, int iters, int random, void *stream)
{
    if (!out || blocks <= 0 || iters <= 0 || iters > (1 << 24)) return -2;
    hipLaunchKernelGGL(mfma_registers, dim3(blocks), dim3(256), 0, (hipStream_t)stream, out, iters, random);
    return done();
}

int cks_probe_mfma_lds(float *out, int blocks, int chunks, int items, int random, void *stream)
{
    if (!out || blocks <= 0 || chunks <= 0 || (chunks & 1) || items <= 0 || (long long)chunks * items > (1 << 24)) return -2;
    hipLaunchKernelGGL(mfma_lds, dim3(blocks), dim3(256), (size_t)2 * (BM + BN) * LDK * sizeof(float), (hipStream_t)stream, out, chunks, items, random);
    return done();
}

int cks_probe_clock_samples(long long *buf, int n, int sleeps, void *stream)
{
    if (!buf || n <= 0 || n > (1 << 16) || sleeps < 0 || sleeps > 1024) return -2;
    hipLaunchKernelGGL(clock_samples, dim3(1), dim3(64), 0, (hipStream_t)stream, buf, n, sleeps);
    return done();
}

}  // extern "C"
