// Types and small device helpers shared by every kernel of libodma.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "odma.h"
#include "plan_types.h"

namespace {

constexpr int BLK = ODMA_BLOCK_TOKENS;
constexpr int PLAN_THREADS = 1024;
constexpr int PLAN_LDS_REQ = 8192;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));

// Block-table entries are read through the constant address space: with a wave-uniform index the load is then a
// scalar one (its own counter), where a load from the global address space becomes a vector load that queues behind
// the K/V tile loads in flight -- and the next tile's address would have to wait for all of them.  The table is
// written before the launch and by nobody during it.
typedef const int32_t __attribute__((address_space(4))) const_i32;
__device__ __forceinline__ const const_i32* as_constant(const int32_t* p) { return (const const_i32*)(uintptr_t)p; }

using odma_plan::PlanHeader;
using odma_plan::Item;
using odma_plan::ReqInfo;

struct DecodeArgs {
  const char* k;         // layer base of the K pool
  const char* v;
  const void* q;
  void* out;
  const int64_t* offsets;
  const int32_t* lengths;
  const int32_t* bt;
  int32_t bt_stride;
  const PlanHeader* hdr;
  const Item* items;
  const ReqInfo* req;
  float2* part_ml;
  float* part_o;
  int32_t n, Hq, Hkv, G, D;
  int64_t head_stride;   // bytes between KV-head planes of one layer
  float scale_log2;      // sm_scale * log2(e)
  int32_t out_bf16;
};

__device__ __forceinline__ int rfl(int x) { return __builtin_amdgcn_readfirstlane(x); }

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
  return x;
}
__device__ __forceinline__ float bf16_bits_to_float(unsigned short b) {
  return __uint_as_float((unsigned int)b << 16);
}
__device__ __forceinline__ unsigned short float_to_bf16_bits(float f) {
  __bf16 h = (__bf16)f;   // round to nearest even (v_cvt_pk_bf16_f32)
  return __builtin_bit_cast(unsigned short, h);
}

}  // namespace
