// Loads that go from global memory straight into LDS, and the hand-scheduled LDS reads that go with them.
//
// gfx950 buffer loads can deposit their data in LDS instead of vector registers ("buffer_load_dword[x4] ... lds"):
// lane l's 4 or 16 bytes land at  LDS base (wave-uniform, in M0) + size * l.  A lane whose offset is out of the
// descriptor's range writes zeros.  The compiler makes every LDS read it can see wait for all such loads in
// flight (it cannot tell which buffer they fill), so kernels that want loading and multiplying to overlap read
// their fragments with the inline-assembly helpers below and place the waits by hand; each wait passes the
// values it releases through itself, which orders their consumers behind it.
//
// The assembly exists in the device pass only: the host pass compiles kernel bodies for their launch stubs
// and knows neither the vector-register constraint nor these builtins.
#pragma once
#include "cks_device.h"

namespace cks {

typedef float floatx4v __attribute__((ext_vector_type(4)));
typedef float floatx2v __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) float lds_float_t;

template <int OFF>
__device__ __forceinline__ floatx4v lds_read_b128(unsigned addr)
{
    static_assert(OFF >= 0 && OFF < 65536, "LDS immediate offset");
    floatx4v v = {0.f, 0.f, 0.f, 0.f};
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
#else
    (void)addr;
#endif
    return v;
}
// two floats OFF0 and OFF1 dwords behind addr (each below 256)
template <int OFF0, int OFF1>
__device__ __forceinline__ floatx2v lds_read2_b32(unsigned addr)
{
    static_assert(OFF0 >= 0 && OFF0 < 256 && OFF1 >= 0 && OFF1 < 256, "ds_read2 offsets are 8-bit dword counts");
    floatx2v v = {0.f, 0.f};
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("ds_read2_b32 %0, %1 offset0:%2 offset1:%3" : "=v"(v) : "v"(addr), "n"(OFF0), "n"(OFF1));
#else
    (void)addr;
#endif
    return v;
}
// Wait until at most PENDING LDS reads are in flight.  The values it releases pass through it, so that
// their consumers are ordered behind the wait.
template <int PENDING>
__device__ __forceinline__ void lds_wait(floatx4v &a, floatx4v &b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_waitcnt lgkmcnt(%2)" : "+v"(a), "+v"(b) : "n"(PENDING));
#endif
}
template <int PENDING>
__device__ __forceinline__ void lds_wait(floatx4v &a, floatx4v &b, floatx4v &c)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(a), "+v"(b), "+v"(c) : "n"(PENDING));
#endif
}
template <int PENDING>
__device__ __forceinline__ void lds_wait(floatx4v &a, floatx4v &b, floatx4v &c, floatx4v &d)
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(PENDING));
#endif
}
// 16 bytes per lane from a raw buffer (byte offset voff per lane + scalar soff) to LDS: the wave's pieces land
// at dst + 16 * lane; dst must be wave-uniform.
__device__ __forceinline__ void load16_to_lds(__amdgpu_buffer_rsrc_t rsrc, float *dst, unsigned voff, int soff)
{
#if defined(__HIP_DEVICE_COMPILE__)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_float_t *)dst, 16, voff, soff, 0, 0);
#else
    (void)rsrc; (void)dst; (void)voff; (void)soff;
#endif
}
__device__ __forceinline__ void vmem_wait_all()
{
#if defined(__HIP_DEVICE_COMPILE__)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
}

}  // namespace cks
