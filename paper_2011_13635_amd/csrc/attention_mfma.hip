// bf16 MFMA attention for gfx950, head width 64, sequence length a multiple of 128.
//
// Forward: softmax(Q K^T / sqrt(d) + key mask) V with the scale, mask and softmax fused between
// the two products; the S x S scores never leave registers.  Backward: scores are recomputed
// from Q, K and the stored row log-sum-exp, in two kernels that each keep one operand family
// resident: a query-side kernel (dQ, and delta = rowsum(dC * C)) and a key-side kernel (dK, dV).
//
// All products are v_mfma_f32_32x32x16_bf16 and are arranged transposed, so that the index the
// softmax runs along sits in a lane's registers:
//   query side:  S^T[key,q] = K Q^T      -> a lane owns one query column, its registers the keys
//                O^T[d,q]   = V^T P^T    -> P^T feeds the second product straight from registers
//   key side:    S[q,key]   = Q K^T      -> a lane owns one key column, its registers the queries
//                dV^T[d,key] = dC^T P,  dK^T[d,key] = Q^T dS
// The accumulator layout of one product is used directly as the B operand of the next one by
// agreeing on a permuted order of the contraction index (the order in which a lane's registers
// hold it); the A operand (V^T, K^T, Q^T, dC^T) is written to LDS transposed and in that order.
// One 256-thread workgroup handles 128 queries (or keys) of one (batch, head): 32 per wavefront.
#include "common.h"

namespace mslt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

constexpr int DH = 64;        // head width
constexpr int TILE = 128;     // rows per LDS tile
constexpr int TLD = 136;      // row stride (elements) of a transposed tile [64][128+8]

__device__ __forceinline__ int swz8(int row) { return ((row >> 1) & 7) ^ ((row >> 4) & 7); }

// Row-major tile [128][64] from global rows of stride ld, 16-byte chunks XOR-swizzled per row.
__device__ __forceinline__ void load_tile_rows(bf16* __restrict__ lds, const bf16* __restrict__ g, size_t ld, int tid) {
  int c = tid & 7, r = tid >> 3;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    int row = r + 32 * p;
    u32x4_t v = *reinterpret_cast<const u32x4_t*>(g + (size_t)row * ld + 8 * c);
    *reinterpret_cast<u32x4_t*>(lds + row * DH + 8 * (c ^ swz8(row))) = v;
  }
}
__device__ __forceinline__ bf16x8_t frag_rows(const bf16* __restrict__ lds, int row, int chunk) {
  return *reinterpret_cast<const bf16x8_t*>(lds + row * DH + 8 * (chunk ^ swz8(row)));
}

// Position of row r (0..127) of a tile along the contraction axis of a transposed tile: within
// each block of 32 the order is the one in which an accumulator lane holds its 16 rows, i.e.
// slot s of lane-half h in the c-th 16-wide MFMA step is row 8*(2c + s/4) + 4h + s%4.
__device__ __forceinline__ int perm_pos(int r) {
  int blk = r & ~31, o = r & 31;
  int c = o >> 4, s4 = (o >> 3) & 1, h = (o >> 2) & 1, j = o & 3;
  return blk + c * 16 + h * 8 + s4 * 4 + j;
}

// Transposed tile [64 d][128 rows permuted] from global rows of stride ld: each thread takes 4
// consecutive rows x 8 d, transposes in registers and writes eight 8-byte pieces.
__device__ __forceinline__ void put4(bf16* __restrict__ lds, int d, int pos, uint32_t a, uint32_t b, uint32_t c,
                                     uint32_t e, uint32_t sel) {
  u32x2_t o;
  o.x = __builtin_amdgcn_perm(b, a, sel);
  o.y = __builtin_amdgcn_perm(e, c, sel);
  *reinterpret_cast<u32x2_t*>(lds + d * TLD + pos) = o;
}
__device__ __forceinline__ void load_tile_transposed(bf16* __restrict__ lds, const bf16* __restrict__ g, size_t ld,
                                                     int tid) {
  int rg = tid >> 3, dg = tid & 7;  // rows 4rg..4rg+3, d 8dg..8dg+7
  const bf16* q = g + (size_t)(4 * rg) * ld + 8 * dg;
  u32x4_t v0 = *reinterpret_cast<const u32x4_t*>(q);
  u32x4_t v1 = *reinterpret_cast<const u32x4_t*>(q + ld);
  u32x4_t v2 = *reinterpret_cast<const u32x4_t*>(q + 2 * ld);
  u32x4_t v3 = *reinterpret_cast<const u32x4_t*>(q + 3 * ld);
  int pos = perm_pos(4 * rg), d = 8 * dg;
  const uint32_t LO = 0x05040100u, HI = 0x07060302u;
  put4(lds, d + 0, pos, v0.x, v1.x, v2.x, v3.x, LO);
  put4(lds, d + 1, pos, v0.x, v1.x, v2.x, v3.x, HI);
  put4(lds, d + 2, pos, v0.y, v1.y, v2.y, v3.y, LO);
  put4(lds, d + 3, pos, v0.y, v1.y, v2.y, v3.y, HI);
  put4(lds, d + 4, pos, v0.z, v1.z, v2.z, v3.z, LO);
  put4(lds, d + 5, pos, v0.z, v1.z, v2.z, v3.z, HI);
  put4(lds, d + 6, pos, v0.w, v1.w, v2.w, v3.w, LO);
  put4(lds, d + 7, pos, v0.w, v1.w, v2.w, v3.w, HI);
}
// A-operand fragment of a transposed tile: row d, the 8 contraction slots of (block kb, step c, half h)
__device__ __forceinline__ bf16x8_t frag_transposed(const bf16* __restrict__ lds, int d, int kb, int c, int half) {
  return *reinterpret_cast<const bf16x8_t*>(lds + d * TLD + kb * 32 + c * 16 + half * 8);
}

__device__ __forceinline__ uint32_t pack2(float a, float b) { return pack_bf16x2(a, b); }
// registers 8c..8c+7 of an accumulator block -> B operand of the c-th 16-wide step
__device__ __forceinline__ bf16x8_t pack_frag(const f32x16_t& p, int c) {
  u32x4_t u;
  u.x = pack2(p[8 * c + 0], p[8 * c + 1]);
  u.y = pack2(p[8 * c + 2], p[8 * c + 3]);
  u.z = pack2(p[8 * c + 4], p[8 * c + 5]);
  u.w = pack2(p[8 * c + 6], p[8 * c + 7]);
  return __builtin_bit_cast(bf16x8_t, u);
}
__device__ __forceinline__ f32x16_t zero16() {
  f32x16_t z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.f;
  return z;
}
#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a), (b), (c), 0, 0, 0)

// 4 consecutive d of 32 rows: accumulator block (lane = row index n, registers = d) to global
// out[(row0 + n)*ld + d0 + 8g + 4half + j] with optional scale, 8-byte stores
__device__ __forceinline__ void store_acc_T(bf16* __restrict__ out, size_t ld, int n, int half, const f32x16_t& a,
                                            float scale) {
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    u32x2_t o;
    o.x = pack2(a[4 * g] * scale, a[4 * g + 1] * scale);
    o.y = pack2(a[4 * g + 2] * scale, a[4 * g + 3] * scale);
    *reinterpret_cast<u32x2_t*>(out + (size_t)n * ld + 8 * g + 4 * half) = o;
  }
}

__device__ __forceinline__ void store_acc_T_f32(float* __restrict__ out, size_t ld, int n, int half, const f32x16_t& a,
                                                float scale) {
#pragma unroll
  for (int g = 0; g < 4; ++g)
    *reinterpret_cast<float4*>(out + (size_t)n * ld + 8 * g + 4 * half) =
        make_float4(a[4 * g] * scale, a[4 * g + 1] * scale, a[4 * g + 2] * scale, a[4 * g + 3] * scale);
}
// 8 consecutive values of the context row for delta: from the fp32 copy when there is one
__device__ __forceinline__ void load_ctx8(const bf16* __restrict__ ctx, const float* __restrict__ ctx32, size_t o,
                                          float (&c)[8]) {
  if (ctx32 != nullptr) {
    float4 a = *reinterpret_cast<const float4*>(ctx32 + o), b = *reinterpret_cast<const float4*>(ctx32 + o + 4);
    c[0] = a.x; c[1] = a.y; c[2] = a.z; c[3] = a.w; c[4] = b.x; c[5] = b.y; c[6] = b.z; c[7] = b.w;
  } else {
    bf16x8_t v = *reinterpret_cast<const bf16x8_t*>(ctx + o);
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = (float)v[i];
  }
}

// ---- forward --------------------------------------------------------------------------------
// The K and V^T tiles of one step (one key tile of one work item) as they sit in registers between the
// global loads and the LDS writes: issued one step ahead, so that the loads of step i+1 are in flight
// while step i computes.
struct KvRegs {
  u32x4_t k[4], v[4];
  float bias;
};
__device__ __forceinline__ void fetch_kv(KvRegs& r, const bf16* __restrict__ kbase, const bf16* __restrict__ vbase,
                                         size_t ld, const int32_t* __restrict__ am_row, float mask_bias, int tid) {
  const int c = tid & 7, rr = tid >> 3;
#pragma unroll
  for (int p = 0; p < 4; ++p) r.k[p] = *reinterpret_cast<const u32x4_t*>(kbase + (size_t)(rr + 32 * p) * ld + 8 * c);
  const bf16* q = vbase + (size_t)(4 * rr) * ld + 8 * c;     // rows 4rr..4rr+3, d 8c..8c+7
#pragma unroll
  for (int p = 0; p < 4; ++p) r.v[p] = *reinterpret_cast<const u32x4_t*>(q + p * ld);
  r.bias = (tid < TILE) ? (am_row[tid] ? 0.f : mask_bias) : 0.f;
}
__device__ __forceinline__ void commit_kv(const KvRegs& r, bf16* __restrict__ Ks, bf16* __restrict__ Vt,
                                          float* __restrict__ bias, int tid) {
  const int c = tid & 7, rr = tid >> 3;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    int row = rr + 32 * p;
    *reinterpret_cast<u32x4_t*>(Ks + row * DH + 8 * (c ^ swz8(row))) = r.k[p];
  }
  const int pos = perm_pos(4 * rr), d = 8 * c;
  const uint32_t LO = 0x05040100u, HI = 0x07060302u;
  put4(Vt, d + 0, pos, r.v[0].x, r.v[1].x, r.v[2].x, r.v[3].x, LO);
  put4(Vt, d + 1, pos, r.v[0].x, r.v[1].x, r.v[2].x, r.v[3].x, HI);
  put4(Vt, d + 2, pos, r.v[0].y, r.v[1].y, r.v[2].y, r.v[3].y, LO);
  put4(Vt, d + 3, pos, r.v[0].y, r.v[1].y, r.v[2].y, r.v[3].y, HI);
  put4(Vt, d + 4, pos, r.v[0].z, r.v[1].z, r.v[2].z, r.v[3].z, LO);
  put4(Vt, d + 5, pos, r.v[0].z, r.v[1].z, r.v[2].z, r.v[3].z, HI);
  put4(Vt, d + 6, pos, r.v[0].w, r.v[1].w, r.v[2].w, r.v[3].w, LO);
  put4(Vt, d + 7, pos, r.v[0].w, r.v[1].w, r.v[2].w, r.v[3].w, HI);
  if (tid < TILE) bias[tid] = r.bias;
}

constexpr int FWD_BUF_ELEMS = TILE * DH + DH * TLD;                     // K rows + V^T of one step
constexpr int FWD_LDS_BYTES = 2 * (FWD_BUF_ELEMS * 2 + TILE * 4);       // two steps

// One workgroup takes `per_wg` consecutive work items (item = 128 queries of one (batch, head), numbered
// query tile fastest, then head, then batch) and walks their key tiles as one sequence of steps over two
// LDS buffers: while step i runs on one buffer, the K/V rows (and, at an item's first step, the Q
// fragments) of step i+1 are already on their way from memory.
template <bool DROP>
__global__ void __launch_bounds__(256, 2) k_attn_fwd_mfma(const bf16* __restrict__ qkv, bf16* __restrict__ ctx,
                                                       float* __restrict__ lse, const int32_t* __restrict__ am, int S,
                                                       int nh, float scale, float mask_bias, DropSpec drop,
                                                       float* __restrict__ ctx32, int n_items, int per_wg) {
  extern __shared__ __attribute__((aligned(16))) unsigned char fwd_lds[];
  bf16* const tiles = reinterpret_cast<bf16*>(fwd_lds);
  float* const biases = reinterpret_cast<float*>(fwd_lds + 2 * FWD_BUF_ELEMS * 2);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 31, half = lane >> 5;
  const int H = nh * DH, nkt = S / TILE;
  const size_t ld = 3 * (size_t)H;
  const int first = blockIdx.x * per_wg;
  const int count = min(per_wg, n_items - first);
  if (count <= 0) return;
  const int steps = count * nkt;
  // scores, running maximum and sum live in the base-2 domain: exp(x) = 2^(x log2 e) with the factor folded
  // into the score scale and the mask bias, so that a probability costs one subtraction and one v_exp_f32
  constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;
  const float scale2 = scale * LOG2E;
  mask_bias *= LOG2E;

  // addresses of a step
  auto item_of = [&](int step, int& b, int& h, int& qt, int& kt) {
    const int it = first + step / nkt;
    kt = step % nkt;
    qt = it % nkt;
    h = (it / nkt) % nh;
    b = it / (nkt * nh);
  };
  KvRegs regs;
  bf16x8_t qn[4];
  auto fetch = [&](int step) {
    int b, h, qt, kt;
    item_of(step, b, h, qt, kt);
    const bf16* base = qkv + (size_t)b * S * ld + h * DH;
    fetch_kv(regs, base + H + (size_t)kt * TILE * ld, base + 2 * H + (size_t)kt * TILE * ld, ld,
             am + (size_t)b * S + kt * TILE, mask_bias, tid);
    if (kt == 0) {
      const int q = qt * TILE + wave * 32 + n;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks)
        qn[ks] = *reinterpret_cast<const bf16x8_t*>(base + (size_t)q * ld + 16 * ks + 8 * half);
    }
  };

  fetch(0);
  commit_kv(regs, tiles, tiles + TILE * DH, biases, tid);
  __syncthreads();

  bf16x8_t qf[4];
  float m_run = -INFINITY, l_run = 0.f;
  f32x16_t o0 = zero16(), o1 = zero16();
#pragma unroll 1
  for (int step = 0; step < steps; ++step) {
    int b, h, qt, kt;
    item_of(step, b, h, qt, kt);
    const bf16* Ks = tiles + (step & 1) * FWD_BUF_ELEMS;
    const bf16* Vt = Ks + TILE * DH;
    const float* bias = biases + (step & 1) * TILE;
    const int q = qt * TILE + wave * 32 + n;  // this lane's query inside the sequence
    if (kt == 0) {
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) qf[ks] = qn[ks];
      m_run = -INFINITY;
      l_run = 0.f;
      o0 = zero16();
      o1 = zero16();
    }
    if (step + 1 < steps) fetch(step + 1);

    // the tile's keys go through the running softmax in two halves of 64: half the score registers
#pragma unroll 1
    for (int kh = 0; kh < 2; ++kh) {
      f32x16_t s[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        s[j] = zero16();
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) s[j] = MFMA(frag_rows(Ks, (2 * kh + j) * 32 + n, 2 * ks + half), qf[ks], s[j]);
      }
      float tmax = -INFINITY;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          float4 bb = *reinterpret_cast<const float4*>(&bias[(2 * kh + j) * 32 + 8 * g + 4 * half]);
          s[j][4 * g + 0] = s[j][4 * g + 0] * scale2 + bb.x;
          s[j][4 * g + 1] = s[j][4 * g + 1] * scale2 + bb.y;
          s[j][4 * g + 2] = s[j][4 * g + 2] * scale2 + bb.z;
          s[j][4 * g + 3] = s[j][4 * g + 3] * scale2 + bb.w;
          tmax = fmaxf(tmax, fmaxf(fmaxf(s[j][4 * g], s[j][4 * g + 1]), fmaxf(s[j][4 * g + 2], s[j][4 * g + 3])));
        }
      tmax = fmaxf(tmax, __shfl_xor(tmax, 32, 64));
      float m_new = fmaxf(m_run, tmax);
      float alpha = __builtin_amdgcn_exp2f(m_run - m_new);   // 0 on an item's first half tile (m_run = -inf)
      float psum = 0.f;
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float p = __builtin_amdgcn_exp2f(s[j][r] - m_new);
          s[j][r] = p;
          psum += p;
        }
      l_run = l_run * alpha + psum;
      m_run = m_new;
      if constexpr (DROP) {   // the row sum above is of the undropped probabilities; the product below uses the kept ones
        const uint64_t rowbase = (((uint64_t)b * nh + h) * S + q) * S + (uint64_t)kt * TILE;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            const uint64_t r = drop_quad(drop, (rowbase + (2 * kh + j) * 32 + 8 * g + 4 * half) >> 2);
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) s[j][4 * g + jj] *= drop_field(drop, r, jj);
          }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        o0[r] *= alpha;
        o1[r] *= alpha;
      }
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int c = 0; c < 2; ++c) {
          bf16x8_t pf = pack_frag(s[j], c);
          o0 = MFMA(frag_transposed(Vt, n, 2 * kh + j, c, half), pf, o0);
          o1 = MFMA(frag_transposed(Vt, 32 + n, 2 * kh + j, c, half), pf, o1);
        }
    }
    if (kt == nkt - 1) {
      float l_tot = l_run + __shfl_xor(l_run, 32, 64);
      float inv = 1.0f / l_tot;
      bf16* out = ctx + ((size_t)b * S + qt * TILE + wave * 32) * H + h * DH;
      store_acc_T(out, H, n, half, o0, inv);
      store_acc_T(out + 32, H, n, half, o1, inv);
      if (ctx32 != nullptr) {
        float* out32 = ctx32 + ((size_t)b * S + qt * TILE + wave * 32) * H + h * DH;
        store_acc_T_f32(out32, H, n, half, o0, inv);
        store_acc_T_f32(out32 + 32, H, n, half, o1, inv);
      }
      if (lse != nullptr && half == 0) lse[((size_t)b * nh + h) * S + q] = (m_run + __builtin_amdgcn_logf(l_tot)) * LN2;
    }
    if (step + 1 < steps) {
      bf16* Kn = tiles + ((step + 1) & 1) * FWD_BUF_ELEMS;
      commit_kv(regs, Kn, Kn + TILE * DH, biases + ((step + 1) & 1) * TILE, tid);
    }
    __syncthreads();
  }
}

// ---- backward, query side: delta and dQ -----------------------------------------------------
template <bool DROP>
__global__ void __launch_bounds__(256) k_attn_bwd_q_mfma(const bf16* __restrict__ qkv, const bf16* __restrict__ ctx,
                                                         const bf16* __restrict__ dctx, const float* __restrict__ lse,
                                                         float* __restrict__ delta, bf16* __restrict__ dqkv,
                                                         const int32_t* __restrict__ am, int S, int nh, float scale,
                                                         float mask_bias, DropSpec drop,
                                                         const float* __restrict__ ctx32) {
  __shared__ __attribute__((aligned(16))) bf16 Ks[TILE * DH];
  __shared__ __attribute__((aligned(16))) bf16 Vs[TILE * DH];
  __shared__ __attribute__((aligned(16))) bf16 Kt[DH * TLD];
  __shared__ __attribute__((aligned(16))) float bias[TILE];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 31, half = lane >> 5;
  const int qt = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int H = nh * DH;
  const size_t ld = 3 * (size_t)H;
  const bf16* base = qkv + (size_t)b * S * ld + h * DH;
  const int q = qt * TILE + wave * 32 + n;
  const size_t tok = (size_t)b * S + q;
  const uint64_t rowbase = (((uint64_t)b * nh + h) * S + q) * S;   // element index of P[b, h, q, 0]

  bf16x8_t qf[4], gf[4];
  float dl = 0.f;
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    qf[ks] = *reinterpret_cast<const bf16x8_t*>(base + (size_t)q * ld + 16 * ks + 8 * half);
    gf[ks] = *reinterpret_cast<const bf16x8_t*>(dctx + tok * H + h * DH + 16 * ks + 8 * half);
    float cf[8];
    load_ctx8(ctx, ctx32, tok * H + h * DH + 16 * ks + 8 * half, cf);
#pragma unroll
    for (int i = 0; i < 8; ++i) dl += (float)gf[ks][i] * cf[i];
  }
  dl += __shfl_xor(dl, 32, 64);
  const float l = lse[((size_t)b * nh + h) * S + q];
  if (half == 0) delta[((size_t)b * nh + h) * S + q] = dl;

  f32x16_t dq0 = zero16(), dq1 = zero16();
  for (int kt = 0; kt < S / TILE; ++kt) {
    if (kt > 0) __syncthreads();
    const bf16* kbase = base + H + (size_t)kt * TILE * ld;
    load_tile_rows(Ks, kbase, ld, tid);
    load_tile_rows(Vs, base + 2 * H + (size_t)kt * TILE * ld, ld, tid);
    load_tile_transposed(Kt, kbase, ld, tid);
    if (tid < TILE) bias[tid] = am[b * S + kt * TILE + tid] ? 0.f : mask_bias;
    __syncthreads();
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      f32x16_t s = zero16(), dp = zero16();
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        s = MFMA(frag_rows(Ks, kb * 32 + n, 2 * ks + half), qf[ks], s);
        dp = MFMA(frag_rows(Vs, kb * 32 + n, 2 * ks + half), gf[ks], dp);
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float4 bb = *reinterpret_cast<const float4*>(&bias[kb * 32 + 8 * g + 4 * half]);
        float bv[4] = {bb.x, bb.y, bb.z, bb.w};
        float kf4[4] = {1.f, 1.f, 1.f, 1.f};
        if constexpr (DROP) {
          const uint64_t r = drop_quad(drop, (rowbase + (uint64_t)kt * TILE + kb * 32 + 8 * g + 4 * half) >> 2);
#pragma unroll
          for (int j = 0; j < 4; ++j) kf4[j] = drop_field(drop, r, j);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float p = __expf(s[4 * g + j] * scale + bv[j] - l);
          s[4 * g + j] = p * (dp[4 * g + j] * kf4[j] - dl);   // dS^T (dP passes through the dropout mask)
        }
      }
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        bf16x8_t df = pack_frag(s, c);
        dq0 = MFMA(frag_transposed(Kt, n, kb, c, half), df, dq0);
        dq1 = MFMA(frag_transposed(Kt, 32 + n, kb, c, half), df, dq1);
      }
    }
  }
  bf16* out = dqkv + ((size_t)b * S + qt * TILE + wave * 32) * ld + h * DH;
  store_acc_T(out, ld, n, half, dq0, scale);
  store_acc_T(out + 32, ld, n, half, dq1, scale);
}

// ---- backward, key side: dK and dV ----------------------------------------------------------
// (two wavefronts per SIMD asked for: the accumulators then stay in VGPRs, where the softmax arithmetic reads
//  them without v_accvgpr moves, and two workgroups share a compute unit; the dropout variant would spill)
template <bool DROP>
__global__ void __launch_bounds__(256, DROP ? 1 : 2) k_attn_bwd_kv_mfma(const bf16* __restrict__ qkv, const bf16* __restrict__ dctx,
                                                          const float* __restrict__ lse,
                                                          const float* __restrict__ delta, bf16* __restrict__ dqkv,
                                                          const int32_t* __restrict__ am, int S, int nh, float scale,
                                                          float mask_bias, DropSpec drop) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_kv[];   // KV_LDS_BYTES
  bf16* Qs = reinterpret_cast<bf16*>(smem_kv);
  bf16* Gs = Qs + TILE * DH;
  bf16* Qt = Gs + TILE * DH;
  bf16* Gt = Qt + DH * TLD;
  float* lse_s = reinterpret_cast<float*>(Gt + DH * TLD);
  float* dl_s = lse_s + TILE;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 31, half = lane >> 5;
  const int kt = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
  const int H = nh * DH;
  const size_t ld = 3 * (size_t)H;
  const bf16* base = qkv + (size_t)b * S * ld + h * DH;
  const int key = kt * TILE + wave * 32 + n;  // this lane's key
  const uint64_t headbase = ((uint64_t)b * nh + h) * S;          // row index of P[b, h, 0, :]

  bf16x8_t kf[4], vf[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    kf[ks] = *reinterpret_cast<const bf16x8_t*>(base + H + (size_t)key * ld + 16 * ks + 8 * half);
    vf[ks] = *reinterpret_cast<const bf16x8_t*>(base + 2 * H + (size_t)key * ld + 16 * ks + 8 * half);
  }
  const float kbias = am[b * S + key] ? 0.f : mask_bias;

  f32x16_t dk0 = zero16(), dk1 = zero16(), dv0 = zero16(), dv1 = zero16();
  for (int qt = 0; qt < S / TILE; ++qt) {
    if (qt > 0) __syncthreads();
    const bf16* qbase = base + (size_t)qt * TILE * ld;
    const bf16* gbase = dctx + ((size_t)b * S + qt * TILE) * H + h * DH;
    load_tile_rows(Qs, qbase, ld, tid);
    load_tile_rows(Gs, gbase, H, tid);
    load_tile_transposed(Qt, qbase, ld, tid);
    load_tile_transposed(Gt, gbase, H, tid);
    if (tid < TILE) {
      lse_s[tid] = lse[((size_t)b * nh + h) * S + qt * TILE + tid];
      dl_s[tid] = delta[((size_t)b * nh + h) * S + qt * TILE + tid];
    }
    __syncthreads();
#pragma unroll
    for (int qb = 0; qb < 4; ++qb) {
      f32x16_t s = zero16(), dp = zero16();   // S[q,key] and dP[q,key]: lane = key, registers = queries
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        s = MFMA(frag_rows(Qs, qb * 32 + n, 2 * ks + half), kf[ks], s);
        dp = MFMA(frag_rows(Gs, qb * 32 + n, 2 * ks + half), vf[ks], dp);
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float4 ll = *reinterpret_cast<const float4*>(&lse_s[qb * 32 + 8 * g + 4 * half]);
        float4 dd = *reinterpret_cast<const float4*>(&dl_s[qb * 32 + 8 * g + 4 * half]);
        float lv[4] = {ll.x, ll.y, ll.z, ll.w}, dv[4] = {dd.x, dd.y, dd.z, dd.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float p = __expf(s[4 * g + j] * scale + kbias - lv[j]);
          float kf1 = 1.f;
          if constexpr (DROP) kf1 = drop_factor(drop, (headbase + (uint64_t)qt * TILE + qb * 32 + 8 * g + 4 * half + j) * S + key);
          s[4 * g + j] = p * kf1;                                   // dropped P (for dV)
          dp[4 * g + j] = p * (dp[4 * g + j] * kf1 - dv[j]);        // dS
        }
      }
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        bf16x8_t pf = pack_frag(s, c), df = pack_frag(dp, c);
        dv0 = MFMA(frag_transposed(Gt, n, qb, c, half), pf, dv0);
        dv1 = MFMA(frag_transposed(Gt, 32 + n, qb, c, half), pf, dv1);
        dk0 = MFMA(frag_transposed(Qt, n, qb, c, half), df, dk0);
        dk1 = MFMA(frag_transposed(Qt, 32 + n, qb, c, half), df, dk1);
      }
    }
  }
  bf16* out = dqkv + ((size_t)b * S + kt * TILE + wave * 32) * ld + h * DH;
  store_acc_T(out + H, ld, n, half, dk0, scale);
  store_acc_T(out + H + 32, ld, n, half, dk1, scale);
  store_acc_T(out + 2 * H, ld, n, half, dv0, 1.0f);
  store_acc_T(out + 2 * H + 32, ld, n, half, dv1, 1.0f);
}

// ---- backward for one-tile sequences (S = 128): both sides in one launch ----------------------
// One 512-thread workgroup per (batch, head).  All eight wavefronts first stage Q, K, V and dC
// (row tiles for the first products, transposed tiles for the second ones), the row log-sum-exp,
// the key bias and delta = rowsum(dC * C) in LDS; then wavefronts 0..3 run the query side (dQ)
// and wavefronts 4..7 the key side (dK, dV) next to each other, with the same arithmetic as the
// two kernels above.  Every operand is read from memory once and delta never leaves the chip.
constexpr int ONE_LDS_BYTES = (4 * TILE * DH + 3 * DH * TLD) * 2 + 3 * TILE * 4;

template <bool DROP>
__global__ void __launch_bounds__(512) k_attn_bwd_one_tile(const bf16* __restrict__ qkv, const bf16* __restrict__ ctx,
                                                           const bf16* __restrict__ dctx,
                                                           const float* __restrict__ lse, bf16* __restrict__ dqkv,
                                                           const int32_t* __restrict__ am, int nh, float scale,
                                                           float mask_bias, DropSpec drop,
                                                           const float* __restrict__ ctx32) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_one[];   // ONE_LDS_BYTES
  bf16* Ks = reinterpret_cast<bf16*>(smem_one);
  bf16* Vs = Ks + TILE * DH;
  bf16* Qs = Vs + TILE * DH;
  bf16* Gs = Qs + TILE * DH;
  bf16* Kt = Gs + TILE * DH;
  bf16* Qt = Kt + DH * TLD;
  bf16* Gt = Qt + DH * TLD;
  float* lse_s = reinterpret_cast<float*>(Gt + DH * TLD);
  float* dl_s = lse_s + TILE;
  float* bias = dl_s + TILE;
  constexpr int S = TILE;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n = lane & 31, half = lane >> 5;
  const int h = blockIdx.x, b = blockIdx.y;
  const int H = nh * DH;
  const size_t ld = 3 * (size_t)H;
  const bf16* base = qkv + (size_t)b * S * ld + h * DH;
  const bf16* gbase = dctx + (size_t)b * S * H + h * DH;

  // staging: the two halves of the workgroup take different tiles
  if (tid < 256) {
    load_tile_rows(Ks, base + H, ld, tid);
    load_tile_rows(Vs, base + 2 * H, ld, tid);
    load_tile_transposed(Kt, base + H, ld, tid);
    load_tile_rows(Gs, gbase, H, tid);
  } else {
    load_tile_rows(Qs, base, ld, tid - 256);
    load_tile_transposed(Qt, base, ld, tid - 256);
    load_tile_transposed(Gt, gbase, H, tid - 256);
  }
  {
    // delta[q] = sum_d dC[q,d] * C[q,d]: four threads per query, 16 d each
    const int q = tid >> 2, part = tid & 3;
    const size_t o = ((size_t)b * S + q) * H + h * DH + 16 * part;
    float dl = 0.f;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      bf16x8_t g = *reinterpret_cast<const bf16x8_t*>(dctx + o + 8 * j);
      float c[8];
      load_ctx8(ctx, ctx32, o + 8 * j, c);
#pragma unroll
      for (int i = 0; i < 8; ++i) dl += (float)g[i] * c[i];
    }
    dl += __shfl_xor(dl, 1, 64);
    dl += __shfl_xor(dl, 2, 64);
    if (part == 0) dl_s[q] = dl;
  }
  if (tid < TILE) lse_s[tid] = lse[((size_t)b * nh + h) * S + tid];
  else if (tid < 2 * TILE) bias[tid - TILE] = am[b * S + tid - TILE] ? 0.f : mask_bias;
  __syncthreads();

  if (wave < 4) {
    // query side: lane owns query q, registers run over keys
    const int q = wave * 32 + n;
    const uint64_t rowbase = (((uint64_t)b * nh + h) * S + q) * S;
    bf16x8_t qf[4], gf[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      qf[ks] = *reinterpret_cast<const bf16x8_t*>(base + (size_t)q * ld + 16 * ks + 8 * half);
      gf[ks] = *reinterpret_cast<const bf16x8_t*>(gbase + (size_t)q * H + 16 * ks + 8 * half);
    }
    const float l = lse_s[q], dl = dl_s[q];
    f32x16_t dq0 = zero16(), dq1 = zero16();
#pragma unroll
    for (int kb = 0; kb < 4; ++kb) {
      f32x16_t s = zero16(), dp = zero16();
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        s = MFMA(frag_rows(Ks, kb * 32 + n, 2 * ks + half), qf[ks], s);
        dp = MFMA(frag_rows(Vs, kb * 32 + n, 2 * ks + half), gf[ks], dp);
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float4 bb = *reinterpret_cast<const float4*>(&bias[kb * 32 + 8 * g + 4 * half]);
        float bv[4] = {bb.x, bb.y, bb.z, bb.w};
        float kf4[4] = {1.f, 1.f, 1.f, 1.f};
        if constexpr (DROP) {
          const uint64_t r = drop_quad(drop, (rowbase + kb * 32 + 8 * g + 4 * half) >> 2);
#pragma unroll
          for (int j = 0; j < 4; ++j) kf4[j] = drop_field(drop, r, j);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float p = __expf(s[4 * g + j] * scale + bv[j] - l);
          s[4 * g + j] = p * (dp[4 * g + j] * kf4[j] - dl);   // dS^T (dP passes through the dropout mask)
        }
      }
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        bf16x8_t df = pack_frag(s, c);
        dq0 = MFMA(frag_transposed(Kt, n, kb, c, half), df, dq0);
        dq1 = MFMA(frag_transposed(Kt, 32 + n, kb, c, half), df, dq1);
      }
    }
    bf16* out = dqkv + ((size_t)b * S + wave * 32) * ld + h * DH;
    store_acc_T(out, ld, n, half, dq0, scale);
    store_acc_T(out + 32, ld, n, half, dq1, scale);
  } else {
    // key side: lane owns a key, registers run over queries
    const int w = wave - 4;
    const int key = w * 32 + n;
    const uint64_t headbase = ((uint64_t)b * nh + h) * S;
    bf16x8_t kf[4], vf[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      kf[ks] = *reinterpret_cast<const bf16x8_t*>(base + H + (size_t)key * ld + 16 * ks + 8 * half);
      vf[ks] = *reinterpret_cast<const bf16x8_t*>(base + 2 * H + (size_t)key * ld + 16 * ks + 8 * half);
    }
    const float kbias = bias[key];
    f32x16_t dk0 = zero16(), dk1 = zero16(), dv0 = zero16(), dv1 = zero16();
#pragma unroll
    for (int qb = 0; qb < 4; ++qb) {
      f32x16_t s = zero16(), dp = zero16();
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        s = MFMA(frag_rows(Qs, qb * 32 + n, 2 * ks + half), kf[ks], s);
        dp = MFMA(frag_rows(Gs, qb * 32 + n, 2 * ks + half), vf[ks], dp);
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float4 ll = *reinterpret_cast<const float4*>(&lse_s[qb * 32 + 8 * g + 4 * half]);
        float4 dd = *reinterpret_cast<const float4*>(&dl_s[qb * 32 + 8 * g + 4 * half]);
        float lv[4] = {ll.x, ll.y, ll.z, ll.w}, dv[4] = {dd.x, dd.y, dd.z, dd.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float p = __expf(s[4 * g + j] * scale + kbias - lv[j]);
          float kf1 = 1.f;
          if constexpr (DROP) kf1 = drop_factor(drop, (headbase + qb * 32 + 8 * g + 4 * half + j) * S + key);
          s[4 * g + j] = p * kf1;                                   // dropped P (for dV)
          dp[4 * g + j] = p * (dp[4 * g + j] * kf1 - dv[j]);        // dS
        }
      }
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        bf16x8_t pf = pack_frag(s, c), df = pack_frag(dp, c);
        dv0 = MFMA(frag_transposed(Gt, n, qb, c, half), pf, dv0);
        dv1 = MFMA(frag_transposed(Gt, 32 + n, qb, c, half), pf, dv1);
        dk0 = MFMA(frag_transposed(Qt, n, qb, c, half), df, dk0);
        dk1 = MFMA(frag_transposed(Qt, 32 + n, qb, c, half), df, dk1);
      }
    }
    bf16* out = dqkv + ((size_t)b * S + w * 32) * ld + h * DH;
    store_acc_T(out + H, ld, n, half, dk0, scale);
    store_acc_T(out + H + 32, ld, n, half, dk1, scale);
    store_acc_T(out + 2 * H, ld, n, half, dv0, 1.0f);
    store_acc_T(out + 2 * H + 32, ld, n, half, dv1, 1.0f);
  }
}

constexpr int KV_LDS_BYTES = (2 * TILE * DH + 2 * DH * TLD) * 2 + 2 * TILE * 4;

bool attention_mfma_supported(int S, int dh) { return dh == DH && S >= TILE && S % TILE == 0; }

template <bool DROP>
static hipError_t attention_fwd_mfma_t(const AttnDesc& a, hipStream_t s) {
  static bool attr_set = false;     // one flag per instantiation
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_attn_fwd_mfma<DROP>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, FWD_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  // two workgroups fit a compute unit (LDS and registers); up to that many, one item each keeps the most
  // units busy, beyond it a workgroup walks several items so that loads run ahead of the arithmetic
  const int n_items = a.B * a.nh * (a.S / TILE);
  const int slots = 2 * 256;
  const int per_wg = (n_items + slots - 1) / slots;
  const int n_wg = (n_items + per_wg - 1) / per_wg;
  k_attn_fwd_mfma<DROP><<<dim3(n_wg), dim3(256), FWD_LDS_BYTES, s>>>(
      (const bf16*)a.qkv, (bf16*)a.ctx, a.lse, a.attn_mask, a.S, a.nh, 1.0f / sqrtf((float)a.dh), a.mask_bias, a.drop,
      a.ctx_f32, n_items, per_wg);
  return hipGetLastError();
}
hipError_t attention_fwd_mfma(const AttnDesc& a, hipStream_t s) {
  if (!attention_mfma_supported(a.S, a.dh)) return hipErrorInvalidValue;
  // dropout is a compile-time variant so that the plain kernels carry none of its registers
  return a.drop.thr ? attention_fwd_mfma_t<true>(a, s) : attention_fwd_mfma_t<false>(a, s);
}

template <bool DROP>
static hipError_t attention_bwd_mfma_t(const AttnBwdDesc& a, hipStream_t s) {
  dim3 grid(a.S / TILE, a.nh, a.B);
  float scale = 1.0f / sqrtf((float)a.dh);
  if (a.S == TILE) {
    static bool one_attr_set = false;     // one flag per instantiation
    if (!one_attr_set) {
      hipError_t e1 = hipFuncSetAttribute(reinterpret_cast<const void*>(k_attn_bwd_one_tile<DROP>),
                                          hipFuncAttributeMaxDynamicSharedMemorySize, ONE_LDS_BYTES);
      if (e1 != hipSuccess) return e1;
      one_attr_set = true;
    }
    k_attn_bwd_one_tile<DROP><<<dim3(a.nh, a.B), dim3(512), ONE_LDS_BYTES, s>>>(
        (const bf16*)a.qkv, (const bf16*)a.ctx, (const bf16*)a.dctx, a.lse, (bf16*)a.dqkv, a.attn_mask, a.nh, scale,
        a.mask_bias, a.drop, a.ctx_f32);
    return hipGetLastError();
  }
  k_attn_bwd_q_mfma<DROP><<<grid, dim3(256), 0, s>>>((const bf16*)a.qkv, (const bf16*)a.ctx, (const bf16*)a.dctx, a.lse,
                                                     a.delta, (bf16*)a.dqkv, a.attn_mask, a.S, a.nh, scale, a.mask_bias,
                                                     a.drop, a.ctx_f32);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  static bool attr_set = false;
  if (!attr_set) {
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_attn_bwd_kv_mfma<DROP>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, KV_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  k_attn_bwd_kv_mfma<DROP><<<grid, dim3(256), KV_LDS_BYTES, s>>>((const bf16*)a.qkv, (const bf16*)a.dctx, a.lse, a.delta,
                                                                 (bf16*)a.dqkv, a.attn_mask, a.S, a.nh, scale,
                                                                 a.mask_bias, a.drop);
  return hipGetLastError();
}
hipError_t attention_bwd_mfma(const AttnBwdDesc& a, hipStream_t s) {
  if (!attention_mfma_supported(a.S, a.dh)) return hipErrorInvalidValue;
  // dropout is a compile-time variant so that the plain kernels carry none of its registers
  return a.drop.thr ? attention_bwd_mfma_t<true>(a, s) : attention_bwd_mfma_t<false>(a, s);
}

}  // namespace mslt
