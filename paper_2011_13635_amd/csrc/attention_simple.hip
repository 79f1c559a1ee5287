// Guarded reference attention kernels (any sequence length, head width up to 128): one
// wavefront per query row (forward, dQ) or per key row (dK, dV).  Used in fp32 mode and as the
// fallback of the bf16 path for shapes the MFMA kernels do not take.  Scores are recomputed in
// the backward from Q, K and the stored row log-sum-exp; no S x S matrix ever reaches memory.
#include "common.h"

namespace mslt {

// forward: ctx[i,:] = sum_j softmax_j(q_i.k_j*scale + bias_j) v_j ; lse[i] = log sum_j exp(score_ij)
template <typename AT>
__global__ void __launch_bounds__(64) k_attn_fwd_simple(const AT* __restrict__ qkv, AT* __restrict__ ctx,
                                                        float* __restrict__ lse, const int32_t* __restrict__ am, int S,
                                                        int nh, int dh, float scale, float mask_bias,
                                                        DropSpec drop, float* __restrict__ ctx32) {
  extern __shared__ float sm[];  // q[dh] | p[S]
  float* q = sm;
  float* p = sm + dh;
  int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  int H = nh * dh, ld = 3 * H, lane = threadIdx.x;
  const AT* base = qkv + (size_t)b * S * ld;
  for (int d = lane; d < dh; d += 64) q[d] = ldf(base + (size_t)i * ld + h * dh + d);
  __syncthreads();
  float mx = -INFINITY;
  for (int j = lane; j < S; j += 64) {
    const AT* kr = base + (size_t)j * ld + H + h * dh;
    float acc = 0.f;
    for (int d = 0; d < dh; ++d) acc += q[d] * ldf(kr + d);
    float sc = acc * scale + (am[b * S + j] ? 0.f : mask_bias);
    p[j] = sc;
    mx = fmaxf(mx, sc);
  }
  mx = wave_max(mx);
  float se = 0.f;
  for (int j = lane; j < S; j += 64) {
    float e = __expf(p[j] - mx);
    p[j] = e;
    se += e;
  }
  se = wave_sum(se);
  if (drop.thr) {   // the normaliser is that of the undropped probabilities
    const uint64_t rowbase = (((uint64_t)b * nh + h) * S + i) * S;
    for (int j = lane; j < S; j += 64) p[j] *= drop_factor(drop, rowbase + j);
  }
  __syncthreads();
  float inv = 1.0f / se;
  for (int d = lane; d < dh; d += 64) {
    float acc = 0.f;
    for (int j = 0; j < S; ++j) acc += p[j] * ldf(base + (size_t)j * ld + 2 * H + h * dh + d);
    stf(ctx + ((size_t)b * S + i) * H + h * dh + d, acc * inv);
    if (ctx32 != nullptr) ctx32[((size_t)b * S + i) * H + h * dh + d] = acc * inv;
  }
  if (lse != nullptr && lane == 0) lse[((size_t)b * nh + h) * S + i] = mx + __logf(se);
}

// backward, query side: delta_i = dctx_i . ctx_i ; dA_ij = P_ij (dctx_i . v_j - delta_i) ; dq_i = scale sum_j dA_ij k_j
template <typename AT>
__global__ void __launch_bounds__(64) k_attn_bwd_q(const AT* __restrict__ qkv, const AT* __restrict__ ctx,
                                                   const AT* __restrict__ dctx, const float* __restrict__ lse,
                                                   float* __restrict__ delta, AT* __restrict__ dqkv,
                                                   const int32_t* __restrict__ am, int S, int nh, int dh, float scale,
                                                   float mask_bias, DropSpec drop, const float* __restrict__ ctx32) {
  extern __shared__ float sm[];  // q[dh] | dc[dh] | da[S]
  float* q = sm;
  float* dc = sm + dh;
  float* da = sm + 2 * dh;
  int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  int H = nh * dh, ld = 3 * H, lane = threadIdx.x;
  const AT* base = qkv + (size_t)b * S * ld;
  size_t row = (size_t)b * S + i;
  float dl = 0.f;
  for (int d = lane; d < dh; d += 64) {
    q[d] = ldf(base + (size_t)i * ld + h * dh + d);
    float g = ldf(dctx + row * H + h * dh + d);
    dc[d] = g;
    dl += g * (ctx32 != nullptr ? ctx32[row * H + h * dh + d] : ldf(ctx + row * H + h * dh + d));
  }
  dl = wave_sum(dl);
  __syncthreads();
  float l = lse[((size_t)b * nh + h) * S + i];
  for (int j = lane; j < S; j += 64) {
    const AT* kr = base + (size_t)j * ld + H + h * dh;
    const AT* vr = base + (size_t)j * ld + 2 * H + h * dh;
    float s = 0.f, dp = 0.f;
    for (int d = 0; d < dh; ++d) {
      s += q[d] * ldf(kr + d);
      dp += dc[d] * ldf(vr + d);
    }
    float pij = __expf(s * scale + (am[b * S + j] ? 0.f : mask_bias) - l);
    if (drop.thr) dp *= drop_factor(drop, (((uint64_t)b * nh + h) * S + i) * S + j);
    da[j] = pij * (dp - dl);
  }
  __syncthreads();
  for (int d = lane; d < dh; d += 64) {
    float acc = 0.f;
    for (int j = 0; j < S; ++j) acc += da[j] * ldf(base + (size_t)j * ld + H + h * dh + d);
    stf(dqkv + row * ld + h * dh + d, acc * scale);
  }
  if (lane == 0) delta[((size_t)b * nh + h) * S + i] = dl;
}

// backward, key side: dv_j = sum_i P_ij dctx_i ; dk_j = scale sum_i dA_ij q_i
template <typename AT>
__global__ void __launch_bounds__(64) k_attn_bwd_kv(const AT* __restrict__ qkv, const AT* __restrict__ dctx,
                                                    const float* __restrict__ lse, const float* __restrict__ delta,
                                                    AT* __restrict__ dqkv, const int32_t* __restrict__ am, int S, int nh,
                                                    int dh, float scale, float mask_bias, DropSpec drop) {
  extern __shared__ float sm[];  // k[dh] | v[dh] | p[S] | da[S]
  float* k = sm;
  float* v = sm + dh;
  float* p = sm + 2 * dh;
  float* da = sm + 2 * dh + S;
  int j = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  int H = nh * dh, ld = 3 * H, lane = threadIdx.x;
  const AT* base = qkv + (size_t)b * S * ld;
  for (int d = lane; d < dh; d += 64) {
    k[d] = ldf(base + (size_t)j * ld + H + h * dh + d);
    v[d] = ldf(base + (size_t)j * ld + 2 * H + h * dh + d);
  }
  __syncthreads();
  float bias = am[b * S + j] ? 0.f : mask_bias;
  for (int i = lane; i < S; i += 64) {
    const AT* qr = base + (size_t)i * ld + h * dh;
    const AT* gr = dctx + ((size_t)b * S + i) * H + h * dh;
    float s = 0.f, dp = 0.f;
    for (int d = 0; d < dh; ++d) {
      s += k[d] * ldf(qr + d);
      dp += v[d] * ldf(gr + d);
    }
    size_t li = ((size_t)b * nh + h) * S + i;
    float pij = __expf(s * scale + bias - lse[li]);
    float kf = drop.thr ? drop_factor(drop, (((uint64_t)b * nh + h) * S + i) * S + j) : 1.f;
    p[i] = pij * kf;                      // dropped probability (for dV)
    da[i] = pij * (dp * kf - delta[li]);
  }
  __syncthreads();
  size_t row = (size_t)b * S + j;
  for (int d = lane; d < dh; d += 64) {
    float av = 0.f, ak = 0.f;
    for (int i = 0; i < S; ++i) {
      av += p[i] * ldf(dctx + ((size_t)b * S + i) * H + h * dh + d);
      ak += da[i] * ldf(base + (size_t)i * ld + h * dh + d);
    }
    stf(dqkv + row * ld + 2 * H + h * dh + d, av);
    stf(dqkv + row * ld + H + h * dh + d, ak * scale);
  }
}

template <typename AT>
static hipError_t fwd_t(const AttnDesc& a, hipStream_t s) {
  dim3 grid(a.S, a.nh, a.B);
  size_t sh = (size_t)(a.dh + a.S) * sizeof(float);
  k_attn_fwd_simple<AT><<<grid, dim3(64), sh, s>>>((const AT*)a.qkv, (AT*)a.ctx, a.lse, a.attn_mask, a.S, a.nh, a.dh,
                                                   1.0f / sqrtf((float)a.dh), a.mask_bias, a.drop, a.ctx_f32);
  return hipGetLastError();
}
hipError_t attention_fwd_simple(int dtype, const AttnDesc& a, hipStream_t s) {
  return dtype == 0 ? fwd_t<float>(a, s) : fwd_t<bf16>(a, s);
}

template <typename AT>
static hipError_t bwd_t(const AttnBwdDesc& a, hipStream_t s) {
  dim3 grid(a.S, a.nh, a.B);
  float scale = 1.0f / sqrtf((float)a.dh);
  k_attn_bwd_q<AT><<<grid, dim3(64), (size_t)(2 * a.dh + a.S) * sizeof(float), s>>>(
      (const AT*)a.qkv, (const AT*)a.ctx, (const AT*)a.dctx, a.lse, a.delta, (AT*)a.dqkv, a.attn_mask, a.S, a.nh, a.dh,
      scale, a.mask_bias, a.drop, a.ctx_f32);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  k_attn_bwd_kv<AT><<<grid, dim3(64), (size_t)(2 * a.dh + 2 * a.S) * sizeof(float), s>>>(
      (const AT*)a.qkv, (const AT*)a.dctx, a.lse, a.delta, (AT*)a.dqkv, a.attn_mask, a.S, a.nh, a.dh, scale,
      a.mask_bias, a.drop);
  return hipGetLastError();
}
hipError_t attention_bwd_simple(int dtype, const AttnBwdDesc& a, hipStream_t s) {
  return dtype == 0 ? bwd_t<float>(a, s) : bwd_t<bf16>(a, s);
}

}  // namespace mslt
