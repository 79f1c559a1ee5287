// Pieces shared by the MFMA GEMM kernels: vector types, the fused epilogue on 8 consecutive output
// columns, and the kernel that sums split-k partials in fixed order.
#pragma once
#include "common.h"

namespace mslt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;   // first-class 16-byte register value
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_void_t;

constexpr int EPI_LD = 68;                             // floats per staged row of a wavefront quarter

// ---- epilogue on 8 consecutive columns ------------------------------------------------------
static __device__ __forceinline__ void unpack8(const uint4& u, float (&f)[8]) {
  const uint32_t* w = reinterpret_cast<const uint32_t*>(&u);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(w[i] << 16);
    f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
  }
}
static __device__ __forceinline__ uint4 pack8(const float (&f)[8]) {
  uint4 u;
  uint32_t* w = reinterpret_cast<uint32_t*>(&u);
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = pack_bf16x2(f[2 * i], f[2 * i + 1]);
  return u;
}
// true when the epilogue reads the per-element operand (stored GELU derivative or addend)
static __device__ __forceinline__ bool epilogue_reads_aux(const Epilogue& e) {
  return e.act == EPI_MUL || (e.act == EPI_ADD && !e.aux_f32);   // an fp32 addend is read where it is used
}
static __device__ __forceinline__ uint4 load_aux8(const Epilogue& e, int m, int n) {
  return *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16*>(e.aux) + (size_t)m * e.ldaux + n);
}
// raw: the 8 per-element operand values of this position (only read when the epilogue uses them);
// callers load it well ahead so its latency is not paid here
// EXTRAS: the rarely used parts (dropout of the result, accumulation into the output) are compiled
// into a second copy of the epilogue, so that the common one carries none of their code.
template <bool EXTRAS>
static __device__ __forceinline__ void epilogue8(const Epilogue& e, int m, int n, float (&v)[8], const float (&bias)[8],
                                          const uint4& raw) {
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] += bias[i];
  if (EXTRAS && e.drop.thr) {
    const uint64_t quad = ((uint64_t)m * e.drop_ld + n) >> 2;     // n and drop_ld are multiples of 4
    const uint64_t r0 = drop_quad(e.drop, quad), r1 = drop_quad(e.drop, quad + 1);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[i] *= drop_field(e.drop, r0, i);
      v[4 + i] *= drop_field(e.drop, r1, i);
    }
  }
  size_t o = (size_t)m * e.ldo + n;
  if (e.act == EPI_GELU) {
    float d[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) gelu_both_fast(v[i], v[i], d[i]);
    if (e.out2) {
      uint4 q;
      q.x = enc_dgelu(d[0]) | (enc_dgelu(d[1]) << 16);
      q.y = enc_dgelu(d[2]) | (enc_dgelu(d[3]) << 16);
      q.z = enc_dgelu(d[4]) | (enc_dgelu(d[5]) << 16);
      q.w = enc_dgelu(d[6]) | (enc_dgelu(d[7]) << 16);
      *reinterpret_cast<uint4*>(reinterpret_cast<bf16*>(e.out2) + o) = q;
    }
  } else if (e.act == EPI_MUL) {
    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      v[2 * i] *= dec_dgelu(w[i] & 0xffffu);
      v[2 * i + 1] *= dec_dgelu(w[i] >> 16);
    }
  } else if (e.act == EPI_ADD) {
    if (e.aux_f32) {
      const float* a = reinterpret_cast<const float*>(e.aux) + (size_t)m * e.ldaux + n;
      const float4 a0 = *reinterpret_cast<const float4*>(a), a1 = *reinterpret_cast<const float4*>(a + 4);
      v[0] += a0.x; v[1] += a0.y; v[2] += a0.z; v[3] += a0.w;
      v[4] += a1.x; v[5] += a1.y; v[6] += a1.z; v[7] += a1.w;
    } else {
      float u[8];
      unpack8(raw, u);
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] += u[i];
    }
  }
  if (e.out_f32) {
    float* p = reinterpret_cast<float*>(e.out) + o;
    if (EXTRAS && e.accumulate) {
      const float4 a0 = *reinterpret_cast<const float4*>(p), a1 = *reinterpret_cast<const float4*>(p + 4);
      v[0] += a0.x; v[1] += a0.y; v[2] += a0.z; v[3] += a0.w;
      v[4] += a1.x; v[5] += a1.y; v[6] += a1.z; v[7] += a1.w;
    }
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
  } else {
    *reinterpret_cast<uint4*>(reinterpret_cast<bf16*>(e.out) + o) = pack8(v);
  }
}

// sums the split-k partials [splitk][M][N] in split order and applies the epilogue (defined with the 128-wide kernel)
__global__ void k_splitk_reduce(const float* __restrict__ partials, int splitk, int M, int N, Epilogue e);

}  // namespace mslt
