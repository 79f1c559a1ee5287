// Guarded SIMT GEMM: C(m,n) = sum_k A(m,k) B(n,k) with the shared epilogue, any shape and any
// leading dimension, fp32 accumulation.  64x64 output tile per 256-thread workgroup, 4x4 outputs
// per thread, operands staged through LDS in slabs of 16 along k.  This is the fp32-mode GEMM
// and the fallback of the bf16 path for shapes the MFMA kernel does not take.
#include "common.h"

namespace mslt {

template <typename AT>
__device__ inline void epilogue_store(const Epilogue& e, int m, int n, float acc) {
  float v = acc;
  if (e.bias) v += e.bias[n];
  if (e.drop.thr) v *= drop_factor(e.drop, (uint64_t)m * e.drop_ld + n);
  size_t o = (size_t)m * e.ldo + n;
  if (e.act == EPI_GELU) {
    float g;
    gelu_both_f(v, v, g);
    if (e.out2) st_dgelu(reinterpret_cast<AT*>(e.out2) + o, g);
  } else if (e.act == EPI_MUL) {
    v *= ld_dgelu(reinterpret_cast<const AT*>(e.aux) + (size_t)m * e.ldaux + n);
  } else if (e.act == EPI_ADD) {
    v += e.aux_f32 ? reinterpret_cast<const float*>(e.aux)[(size_t)m * e.ldaux + n]
                   : ldf(reinterpret_cast<const AT*>(e.aux) + (size_t)m * e.ldaux + n);
  }
  if (e.out_f32)
    reinterpret_cast<float*>(e.out)[o] = e.accumulate ? reinterpret_cast<float*>(e.out)[o] + v : v;
  else
    stf(reinterpret_cast<AT*>(e.out) + o, v);
}

template <typename AT>
__global__ void __launch_bounds__(256) k_gemm_simt(GemmDesc d) {
  constexpr int BM = 64, BN = 64, BK = 16;
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const AT* A = reinterpret_cast<const AT*>(d.A);
  const AT* B = reinterpret_cast<const AT*>(d.B);
  int tid = threadIdx.x;
  int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  int tm = (tid / 16) * 4, tn = (tid % 16) * 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < d.K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int idx = tid + i * 256;
      int mm, kk;
      if (d.a_kcontig) { mm = idx / BK; kk = idx % BK; } else { mm = idx % BM; kk = idx / BM; }
      int gm = m0 + mm, gk = k0 + kk;
      float v = 0.f;
      if (gm < d.M && gk < d.K) v = ldf(A + (d.a_kcontig ? (size_t)gm * d.lda + gk : (size_t)gk * d.lda + gm));
      As[kk][mm] = v;
      int nn;
      if (d.b_kcontig) { nn = idx / BK; kk = idx % BK; } else { nn = idx % BN; kk = idx / BN; }
      int gn = n0 + nn;
      gk = k0 + kk;
      v = 0.f;
      if (gn < d.N && gk < d.K) v = ldf(B + (d.b_kcontig ? (size_t)gn * d.ldb + gk : (size_t)gk * d.ldb + gn));
      Bs[kk][nn] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][tm + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tn + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + tm + i;
    if (m >= d.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tn + j;
      if (n < d.N) epilogue_store<AT>(d.epi, m, n, acc[i][j]);
    }
  }
}

hipError_t gemm_simt(int dtype, const GemmDesc& d, hipStream_t s) {
  if (d.M <= 0 || d.N <= 0) return hipSuccess;
  dim3 grid((d.N + 63) / 64, (d.M + 63) / 64), block(256);
  if (dtype == 0)
    k_gemm_simt<float><<<grid, block, 0, s>>>(d);
  else
    k_gemm_simt<bf16><<<grid, block, 0, s>>>(d);
  return hipGetLastError();
}

}  // namespace mslt
