// Device-side helpers: bfloat16 storage type, 8-wide vector loads/stores, wavefront reductions.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace sp {

typedef __bf16 bf16;

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __builtin_bit_cast(float, b << 16); }
__device__ __forceinline__ uint32_t float_to_bf16_bits(float f) {
  return (uint32_t) __builtin_bit_cast(uint16_t, (bf16)f);  // round to nearest even
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  return float_to_bf16_bits(lo) | (float_to_bf16_bits(hi) << 16);
}

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16 v) { return (float)v; }
template <class T> __device__ __forceinline__ T from_float(float v);
template <> __device__ __forceinline__ float from_float<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_float<bf16>(float v) { return (bf16)v; }

// 8 consecutive elements <-> 8 floats; p must be 16-byte aligned for bf16, 32 for float
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16* p, float (&v)[8]) {
  uint4 u = *reinterpret_cast<const uint4*>(p);
  v[0] = bf16_bits_to_float(u.x & 0xffffu); v[1] = bf16_bits_to_float(u.x >> 16);
  v[2] = bf16_bits_to_float(u.y & 0xffffu); v[3] = bf16_bits_to_float(u.y >> 16);
  v[4] = bf16_bits_to_float(u.z & 0xffffu); v[5] = bf16_bits_to_float(u.z >> 16);
  v[6] = bf16_bits_to_float(u.w & 0xffffu); v[7] = bf16_bits_to_float(u.w >> 16);
}
// 8 bf16 values held as 16 bytes -> 8 floats
__device__ __forceinline__ void unpack8(const uint4& v, float (&x)[8]) {
  const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) { x[2 * e] = bf16_bits_to_float(w[e] & 0xffffu); x[2 * e + 1] = bf16_bits_to_float(w[e] >> 16); }
}
// Tells the compiler that the four registers (and `after`) may have changed: values derived from them before this
// point are not kept alive for reuse after it (a kernel that holds many packed values and unpacks them in several
// passes would otherwise keep the unpacked floats of the first pass, at twice the registers), and nothing derived
// from v after this point is computed before `after` has its value, which keeps the pieces of an unrolled loop in
// sequence where the scheduler would otherwise unpack all of them at once.
__device__ __forceinline__ void forget_derived(uint4& v, float& after) {
  asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w), "+v"(after));
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16* p, const float (&v)[8]) {
  uint4 u;
  u.x = pack_bf16(v[0], v[1]); u.y = pack_bf16(v[2], v[3]); u.z = pack_bf16(v[4], v[5]); u.w = pack_bf16(v[6], v[7]);
  *reinterpret_cast<uint4*>(p) = u;
}

// The same stores with the streaming hint: for outputs far larger than the L2s that the next kernel reads once
// (a matrix product's output tile); measured 1.5 us less per round of 256 x 256 tiles than plain stores.
__device__ __forceinline__ void store16_stream(void* p, const uint4& u) {
  typedef __attribute__((ext_vector_type(4))) unsigned int u4;
  const u4 w = {u.x, u.y, u.z, u.w};
  __builtin_nontemporal_store(w, reinterpret_cast<u4*>(p));
}
__device__ __forceinline__ uint4 load16_stream(const void* p) {
  typedef __attribute__((ext_vector_type(4))) unsigned int u4;
  const u4 w = __builtin_nontemporal_load(reinterpret_cast<const u4*>(p));
  return make_uint4(w[0], w[1], w[2], w[3]);
}
__device__ __forceinline__ void store8_stream(bf16* p, const float (&v)[8]) {
  uint4 u;
  u.x = pack_bf16(v[0], v[1]); u.y = pack_bf16(v[2], v[3]); u.z = pack_bf16(v[4], v[5]); u.w = pack_bf16(v[6], v[7]);
  store16_stream(p, u);
}

// ---- buffer loads: 16 bytes at byte offset voff of a raw buffer; zero when voff is at or past its end
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
__device__ __forceinline__ rsrc_t make_rsrc(const void* p, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ u32x4 buffer_load16(rsrc_t rsrc, uint32_t voff) {
  typedef __attribute__((ext_vector_type(4))) int i32x4_;
  return __builtin_bit_cast(u32x4, (i32x4_)__builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voff, 0, 0));
}

// ---- buffer loads with the LDS modifier (memory -> LDS without passing through registers), written as
// assembly so that the compiler's wait insertion does not see them: it would otherwise make the first LDS
// read after every such load wait for it (it cannot tell that the read is from another buffer), which would
// undo any prefetch.  One instruction copies 64 x 16 bytes (or 64 x 4) from the lanes' buffer offsets to LDS at
// lds .. lds + 1024 (256) in lane order; an offset at or past the descriptor's size delivers zeros.  Counted
// by vmcnt like any load: the caller waits for them by hand (s_waitcnt) before a barrier.
typedef __attribute__((address_space(3))) void* lds_ptr;
__device__ __forceinline__ u32x4 make_desc(const void* p, uint32_t bytes) {   // raw buffer descriptor as 4 words
  const uint64_t a = (uint64_t)p;
  u32x4 d = {(uint32_t)a, (uint32_t)(a >> 32) & 0xffffu, bytes, 0x00020000u};
  return d;
}
// The statements overwrite m0 and say so in their clobber lists, so that the compiler re-creates any m0 value of
// its own after them.  m0 is a register the compiler never allocates, and clang warns about such a register on a
// clobber list whatever the reason: the warning is switched off for these two statements only.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void load_to_lds16(u32x4 desc, lds_ptr lds, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(lds), "v"(voff), "s"(desc) : "memory", "m0");
}
__device__ __forceinline__ void load_to_lds4(u32x4 desc, lds_ptr lds, uint32_t voff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, 0 offen lds" ::"s"(lds), "v"(voff), "s"(desc) : "memory", "m0");
}
#pragma clang diagnostic pop

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}

}  // namespace sp
