// Helpers shared by the matrix-core kernels: exact e4m3 -> fp16 decode, global-address-space
// accessors, the XCD-aware tile order, and the direct-to-LDS slab pipeline primitives.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pahq {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v2h __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// Eight e4m3 codes (two 32-bit words) -> eight fp16 values with the hardware
// converter (V_CVT_SCALEF32_PK_F16_FP8, scale 1): exact for every finite code,
// subnormals and signed zero included (checked over all 254 codes on gfx950).
__device__ __forceinline__ v8h decode8(uint32_t w0, uint32_t w1) {
  union { v8h h; v2h p[4]; } r;
  r.p[0] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w0, 1.0f, false);
  r.p[1] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w0, 1.0f, true);
  r.p[2] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w1, 1.0f, false);
  r.p[3] = __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(w1, 1.0f, true);
  return r.h;
}


// Pointers that arrive inside descriptor structs are generic to the compiler; every one of them points to
// global memory.  Saying so turns FLAT accesses (which may touch LDS and therefore wait for the
// slab loads in flight) into GLOBAL ones.
#define GCF(p) ((const __attribute__((address_space(1))) float*)(p))
#define GF(p) ((__attribute__((address_space(1))) float*)(p))
__device__ __forceinline__ float4 gload4(const float* p) {
  v4f v = *(const __attribute__((address_space(1))) v4f*)p;
  return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void gstore4(float* p, float4 v) {
  *(__attribute__((address_space(1))) v4f*)p = (v4f){v.x, v.y, v.z, v.w};
}
// A load marked non-temporal, for data that is read once.
__device__ __forceinline__ float4 gload4_nt(const float* p) {
  v4f v = __builtin_nontemporal_load((const __attribute__((address_space(1))) v4f*)p);
  return make_float4(v[0], v[1], v[2], v[3]);
}
// The same store marked non-temporal: a result tile that nothing reads again before it has left the L2 anyway
// should not push the operands the neighbouring tiles still need out of it.
__device__ __forceinline__ void gstore4_nt(float* p, float4 v) {
  __builtin_nontemporal_store((v4f){v.x, v.y, v.z, v.w}, (__attribute__((address_space(1))) v4f*)p);
}

// XCD-aware tile order: workgroup id w runs on XCD w % 8; that XCD gets the
// contiguous range [x * chunk, (x+1) * chunk) of the linear tile index.
__device__ __forceinline__ int xcd_tile(int wg, int total) {
  int chunk = (total + 7) >> 3;
  return (wg & 7) * chunk + (wg >> 3);
}

// The slab loads, the waits for them and the workgroup barriers are written as volatile assembly
// with a memory clobber.  The compiler's own wait insertion treats a load into LDS as something
// every later LDS read may depend on wherever control flow merges, and waits for all of them
// (and for the stores in flight) at exactly the points where this kernel wants them outstanding;
// __syncthreads() adds a fence that waits for every global store.  What must be ordered is spelled
// out instead: a wave waits for its own slab loads (s_waitcnt vmcnt) before the barrier that
// publishes a stage, and has consumed its operand reads (their values fed MFMAs) before the
// barrier that frees it.  Waits the compiler adds for ordinary loads count fewer operations than
// are in flight, which only makes them stricter.
__device__ __forceinline__ void slab_load16(const uint8_t* g, uint32_t lds_addr) {
  // M0 = wave-uniform LDS base; lane l writes bytes [16 l, 16 l + 16) behind it
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_addr) : "memory");
}
// one dword per lane: lane l writes LDS bytes [4 l, 4 l + 4) behind the base
__device__ __forceinline__ void lds_load4(const void* g, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(g), "s"(lds_addr) : "memory");
}
// at most N vector-memory operations of this wave still outstanding (they retire in issue order)
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }
// "Everything has arrived" is said with the builtin, so that the compiler also knows that its own
// loads (scales, bias) are complete and does not wait for them again in the middle of a slab.
// 0x0F70: vmcnt(0), expcnt and lgkmcnt left at their maxima.
__device__ __forceinline__ void wait_all_then_barrier() {
  asm volatile("" ::: "memory");       // no load may be moved below the wait
  __builtin_amdgcn_s_waitcnt(0x0F70);
  wg_barrier();
}
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}


}  // namespace pahq
