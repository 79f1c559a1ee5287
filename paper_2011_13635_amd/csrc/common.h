// Shared device helpers and the launcher interface between the kernel files and the host logic.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace mslt {

// ---- bf16 storage type with round-to-nearest-even conversion -------------------------------
struct bf16 {
  uint16_t x;
};

__host__ __device__ inline float bf2f(bf16 v) {
  union { uint32_t u; float f; } c;
  c.u = ((uint32_t)v.x) << 16;
  return c.f;
}
typedef __bf16 hw_bf16x2_t __attribute__((ext_vector_type(2)));
typedef float hw_f32x2_t __attribute__((ext_vector_type(2)));
// fp32 -> bf16, round to nearest even, in hardware (v_cvt_pk_bf16_f32 on gfx950)
__device__ inline uint32_t pack_bf16x2(float lo, float hi) {
  hw_f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, hw_bf16x2_t));
}
__device__ inline bf16 f2bf(float f) {
  bf16 r;
  r.x = (uint16_t)(pack_bf16x2(f, 0.f) & 0xffffu);
  return r;
}

__device__ inline float ldf(const float* p) { return *p; }
__device__ inline float ldf(const bf16* p) { return bf2f(*p); }
__device__ inline void stf(float* p, float v) { *p = v; }
__device__ inline void stf(bf16* p, float v) { *p = f2bf(v); }

// The GELU derivative kept from the forward pass for the backward pass.  fp32 mode keeps the
// float.  bf16 mode keeps 16-bit fixed point (value + 0.25) * 32768 in the 2-byte slot: the
// derivative lies in [-0.13, 1.13], so the step of 3.05e-5 is two orders of magnitude finer than
// a bf16 number near 1 (and finer than evaluating the derivative at a bf16-rounded argument).
__device__ inline uint32_t enc_dgelu(float d) { return __float2uint_rn(fmaf(d, 32768.f, 8192.f)); }
__device__ inline float dec_dgelu(uint32_t q) { return fmaf((float)q, 1.0f / 32768.f, -0.25f); }
__device__ inline float ld_dgelu(const float* p) { return *p; }
__device__ inline float ld_dgelu(const bf16* p) { return dec_dgelu(p->x); }
__device__ inline void st_dgelu(float* p, float d) { *p = d; }
__device__ inline void st_dgelu(bf16* p, float d) { p->x = (uint16_t)enc_dgelu(d); }

// ---- dropout keep decisions ------------------------------------------------------------------
// Counter-based, so that they can be recomputed anywhere (forward, backward, a checker): the
// SplitMix64 output function (Steele, Lea, Flood 2014) of key + quad * GOLDEN decides the four
// elements 4*quad .. 4*quad+3 of a tensor (C-order element index) with its four 16-bit fields,
// lowest field first: an element is kept iff its field >= thr = round(p * 65536), and kept values
// are scaled by 1 / (1 - p).  The key mixes the caller's seed with (step, layer, site).
constexpr uint64_t DROP_GOLDEN = 0x9E3779B97F4A7C15ull;
enum DropSite { SITE_EMBEDDING = 0, SITE_ATTN_PROBS = 1, SITE_ATTN_OUT = 2, SITE_FFN_OUT = 3 };
struct DropSpec {
  uint64_t key = 0;
  uint32_t thr = 0;     // 0: dropout off
  float scale = 1.f;
};
__host__ __device__ inline uint64_t mix64(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}
inline uint64_t drop_key(uint64_t seed, uint64_t step, int layer, int site) {
  uint64_t stream = (step << 20) | ((uint64_t)layer << 4) | (uint64_t)site;
  return mix64(seed ^ mix64(stream + DROP_GOLDEN));
}
__device__ inline uint64_t drop_quad(const DropSpec& d, uint64_t quad) { return mix64(d.key + quad * DROP_GOLDEN); }
__device__ inline float drop_field(const DropSpec& d, uint64_t r, int field) {
  return (uint32_t)((r >> (16 * field)) & 0xffffu) >= d.thr ? d.scale : 0.f;
}
__device__ inline float drop_factor(const DropSpec& d, uint64_t elem) {
  return drop_field(d, drop_quad(d, elem >> 2), (int)(elem & 3));
}

// ---- wavefront (64 lanes) reductions --------------------------------------------------------
__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// erf-form GELU for the bf16 path: erf from the three-term rational-exponential formula of
// Abramowitz & Stegun 7.1.25 (|error| <= 2.5e-5, far below bf16 resolution); the Gaussian factor
// is shared between Phi and phi.  One reciprocal and one exp2 per element.
__device__ inline void gelu_parts_fast(float u, float& cdf, float& pdf) {
  float x = fabsf(u) * 0.70710678118654752440f;
  float t = __builtin_amdgcn_rcpf(fmaf(0.47047f, x, 1.0f));
  float e = __builtin_amdgcn_exp2f(-1.4426950408889634f * x * x);   // exp(-x^2) = exp(-u^2/2)
  float poly = t * fmaf(t, fmaf(t, 0.7478556f, -0.0958798f), 0.3480242f);
  float erfc_half = 0.5f * poly * e;                                 // (1 - erf(x)) / 2
  cdf = u >= 0.f ? 1.0f - erfc_half : erfc_half;
  pdf = 0.39894228040143267794f * e;
}
// value and derivative together (the forward epilogue stores the derivative for the backward pass)
__device__ inline void gelu_both_fast(float u, float& val, float& grad) {
  float c, p;
  gelu_parts_fast(u, c, p);
  val = u * c;
  grad = fmaf(u, p, c);
}
// erf-form GELU and its derivative with the library erf (fp32 mode)
__device__ inline void gelu_both_f(float u, float& val, float& grad) {
  float cdf = 0.5f * (1.0f + erff(u * 0.70710678118654752440f));
  float pdf = 0.39894228040143267794f * __expf(-0.5f * u * u);
  val = u * cdf;
  grad = cdf + u * pdf;
}

// ---- GEMM interface -------------------------------------------------------------------------
// C(m,n) = sum_k A(m,k) * B(n,k), fp32 accumulation, followed by an epilogue.
// Each operand has unit stride along exactly one of its two indices:
//   a_kcontig: A(m,k) = A[m*lda + k]   else A(m,k) = A[k*lda + m]   (same for B with n)
enum EpiAct { EPI_NONE = 0, EPI_GELU = 1, EPI_MUL = 2, EPI_ADD = 3 };

struct Epilogue {
  void* out = nullptr;      // [M, ldo]; element type: float if out_f32 else the activation type
  int ldo = 0;
  int out_f32 = 0;
  const float* bias = nullptr;  // per column n, or null
  int act = EPI_NONE;
  void* out2 = nullptr;     // EPI_GELU: GELU'(pre-activation) for the backward pass (st_dgelu format), may be null
  const void* aux = nullptr;  // EPI_MUL: the stored GELU derivative D[m,n] (ld_dgelu format); EPI_ADD: addend R[m,n]
  int ldaux = 0;
  int aux_f32 = 0;          // EPI_ADD: the addend is fp32 whatever the activation type (wide residual gradients)
  DropSpec drop;            // dropout of (acc + bias) before the activation / addend; element index m * drop_ld + n
  int drop_ld = 0;          // logical row width of the dropped tensor (a multiple of 4)
  int accumulate = 0;       // fp32 output only: out += result (gradient of a parameter set shared by several layers)
};

struct GemmDesc {
  const void* A = nullptr;
  const void* B = nullptr;
  int M = 0, N = 0, K = 0;
  int lda = 0, ldb = 0;
  int a_kcontig = 1, b_kcontig = 1;
  Epilogue epi;
};

// dtype: 0 = float operands, 1 = bf16 operands.
// Guarded SIMT kernel: any shape, any leading dimension.
hipError_t gemm_simt(int dtype, const GemmDesc& d, hipStream_t s);
// MFMA kernel (bf16 only): M, N multiples of 128, K multiple of 64 (per split), all loads in
// bounds by construction (padded buffers).  splitk > 1 writes fp32 partials to `partials`
// ([splitk][M][N]) and reduces them in fixed order into the epilogue.
bool gemm_mfma_supported(const GemmDesc& d);
// force_tile_m: 0 = choose the M-tile height (128 or 256 rows) from the shape.
int gemm_mfma_tile_m(const GemmDesc& d);
// force_dma: -1 = default choice, 0/1 = k-contiguous operands through registers / direct to LDS.
hipError_t gemm_mfma(const GemmDesc& d, int splitk, float* partials, hipStream_t s, int force_tile_m = 0,
                     int force_dma = -1);

// Large-tile MFMA kernel (bf16 only): tile_m x tile_n of 256x256, 256x128 or 128x256, both operands loaded
// global -> LDS directly in any of the three layouts; M % tile_m == 0, N % tile_n == 0.
// rk: k extent of a ring stage, 32 or 64 (K % rk == 0).
bool gemm_ring_supported(const GemmDesc& d, int tile_m, int tile_n, int rk);
// Up to gemm_ring_group_max() products whose operands are both k-strided (weight gradients) as one launch of
// tile_m x tile_n tiles (128x128, 256x128 or 256x256), none of them split; each must pass
// gemm_ring_supported(d, tile_m, tile_n, 64).
int gemm_ring_group_max();
hipError_t gemm_ring_grouped_tn(const GemmDesc* d, int n, int tile_m, int tile_n, hipStream_t s);
// keep_partials: with splitk > 1, leave the partial sums in `partials` and skip the kernel that adds them (the
// caller adds them later, see ReduceJob); only for a plain fp32 result (no bias, activation, addend or dropout)
hipError_t gemm_ring(const GemmDesc& d, int tile_m, int tile_n, int rk, int splitk, float* partials, hipStream_t s,
                     bool keep_partials = false);

// ---- attention ------------------------------------------------------------------------------
struct AttnDesc {
  const void* qkv;    // [T, 3H] rows = tokens: Q | K | V, head h at columns h*dh
  void* ctx;          // [T, H]
  float* lse;         // [B, nh, S] natural log-sum-exp of the masked scaled scores, or null
  const int32_t* attn_mask;  // [B, S]
  int B, S, nh, dh;
  float mask_bias;
  DropSpec drop;      // dropout of the attention probabilities; element index ((b*nh + h)*S + q)*S + key
  float* ctx_f32 = nullptr;   // optional second copy of ctx in fp32, unrounded, for the backward pass (see AttnBwdDesc)
};
struct AttnBwdDesc {
  const void* qkv;
  const void* ctx;
  const void* dctx;   // [T, H]
  const float* lse;
  float* delta;       // scratch [B, nh, S]
  void* dqkv;         // [T, 3H]
  const int32_t* attn_mask;
  int B, S, nh, dh;
  float mask_bias;
  DropSpec drop;      // as in AttnDesc
  // The backward needs delta = rowsum(dC * C) to equal sum_key P * dP of the probabilities it
  // recomputes; with C rounded to bf16 the two differ by 2^-9 |C||dC|, the rows of dS no longer sum
  // to zero, and that residual times the (large) common part of the keys ends up in dQ.  So when the
  // forward kept an unrounded fp32 copy of C, delta is taken from that.
  const float* ctx_f32 = nullptr;
};
hipError_t attention_fwd_simple(int dtype, const AttnDesc& d, hipStream_t s);
hipError_t attention_bwd_simple(int dtype, const AttnBwdDesc& d, hipStream_t s);
bool attention_mfma_supported(int S, int dh);
hipError_t attention_fwd_mfma(const AttnDesc& d, hipStream_t s);
hipError_t attention_bwd_mfma(const AttnBwdDesc& d, hipStream_t s);

// ---- row-wise and element-wise kernels ------------------------------------------------------
hipError_t fill_zero(void* p, size_t bytes, hipStream_t s);
hipError_t cast_f32_to_bf16(const float* src, bf16* dst, size_t n, hipStream_t s);
hipError_t widen_to_f32(int dtype, const void* src, float* dst, size_t n, hipStream_t s);

// checks the batch and compacts predicted positions.  counters[0] = M, counters[1] = error bits
// (1 id range, 2 type range, 4 label range, 8 mask value).  inv[t] = j if t is the j-th predicted
// position else -1.
// pos/lab hold at most `cap` entries; counters[0] still reports the true count.
hipError_t batch_scan(const int32_t* ids, const int32_t* tt, const int32_t* am, const int32_t* labels, int T, int vocab,
                      int type_vocab, int cap, int32_t* pos, int32_t* lab, int32_t* inv, int32_t* counters,
                      int cls_every, const int32_t* nsp_labels, int n_seq, hipStream_t s);

struct LnStash {
  void* xhat = nullptr;   // [rows, H] activation type, or null
  float* rstd = nullptr;  // [rows] or null
};
hipError_t embed_ln_fwd(int dtype, const int32_t* ids, const int32_t* tt, int S, const float* word, const float* pos,
                        const float* type, const float* g, const float* b, float eps, void* out, LnStash st, int T,
                        int H, int vocab, int type_vocab, const DropSpec& drop, hipStream_t s);
// out = LN(a + r) (r may be null)
hipError_t add_ln_fwd(int dtype, const void* a, const void* r, const float* g, const float* b, float eps, void* out,
                      LnStash st, int rows, int H, hipStream_t s);
// Dropout around a LayerNorm in the backward pass.  in: the LayerNorm output was dropped (embedding
// block), so dy is multiplied by the keep factors first.  out: the LayerNorm input was residual +
// dropout(y); then dzm receives dz times the keep factors (the gradient of y) next to dz (the
// gradient of the residual), and the column sums are those of dzm.  rowmap (or null): token row of
// each of the first n_mapped rows, for the element index of compacted rows.
struct LnBwdDrop {
  DropSpec in, out;
  void* dzm = nullptr;
  const int32_t* rowmap = nullptr;
  int n_mapped = 0;
  int accumulate = 0;   // dgamma, dbeta and the column sums are added to what the outputs hold
};
// A sum of partial results that may be carried out later, many at a time in one launch (reduce_batch):
// out[c] (+)= sum over p < n_partials of partial[p*N + c], partials added in index order.  `flat` picks the
// work split for few partials of many elements (split-k partial products); otherwise the split is the one for
// many partials of a row (column sums).  Two jobs of one batch must not write the same output.
struct ReduceJob {
  const float* partial;
  float* out;
  uint32_t n_partials, N;
  uint32_t first_block;    // set by reduce_batch
  uint32_t flags;          // 1 = add to what out holds, 2 = flat
};
inline ReduceJob reduce_job(const float* partial, float* out, int n_partials, size_t N, bool accumulate, bool flat) {
  return ReduceJob{partial, out, (uint32_t)n_partials, (uint32_t)N, 0u, (accumulate ? 1u : 0u) | (flat ? 2u : 0u)};
}
hipError_t reduce_batch(ReduceJob* jobs, int n, hipStream_t s);

// dz from dy, xhat, rstd, gamma; dgamma, dbeta and (if dzsum != null) the column sums of dz (of dzm
// with output dropout) via partials in scratch (ln_bwd_scratch_floats(rows, H) floats).
// dy_f32: dy is fp32 whatever the activation type; dz32 (or null): a second, unrounded fp32 copy of dz
// (the residual branch of the backward pass carries fp32 in bf16 mode, see model.hip).
hipError_t ln_bwd(int dtype, const void* dy, const void* xhat, const float* rstd, const float* g, void* dz, float* dg,
                  float* db, float* dzsum, float* scratch, int rows, int H, const LnBwdDrop& dd, hipStream_t s,
                  int dy_f32 = 0, float* dz32 = nullptr, ReduceJob* later = nullptr, int* n_later = nullptr);
// column sums of Y[rows, N] (leading dimension ld) into out[N]; scratch holds ceil(rows/64)*N floats
// later (ln_bwd: room for 3, *n_later receives the count): the sums of the partials are not launched but
// described there for reduce_batch; scratch must then stay untouched until that batch has run
hipError_t colsum(int dtype, const void* y, int ld, int rows, int N, float* out, float* scratch, hipStream_t s,
                  int accumulate = 0, ReduceJob* later = nullptr);   // accumulate: out += sums
size_t colsum_scratch_floats(int rows, int N);
size_t ln_bwd_scratch_floats(int rows, int H);

hipError_t mul_dgelu(int dtype, const void* dg, const void* d, void* du, size_t n, hipStream_t s);
struct GatherDesc { const void* src; void* dst; int row_bytes; };
constexpr int GATHER_MAX = 8;
struct GatherArgs { GatherDesc d[GATHER_MAX]; };
// for each of the n arrays: dst row j = j < M ? src row pos[j] : zeros, j < Mpad; rows are raw bytes
// (row_bytes a multiple of 4)
hipError_t gather_rows_multi(const GatherDesc* descs, int n, const int32_t* pos, int M, int Mpad, hipStream_t s);
hipError_t scatter_rows(int dtype, const void* dxm, const int32_t* inv, int rows_total, int T, int H, void* out,
                        hipStream_t s);
// cross-entropy over logits [Mpad, ldz] of the activation type: writes dZ (same type, zero in padded rows
// and columns; dz may be the logits buffer itself), per-row loss and lse; loss_out = mean over the
// labelled rows in fixed order.
// (rows whose label is negative are only there for the next-sentence head: zero dZ, no loss; Mn = rows with a label)
hipError_t ce_fwd_bwd(int dtype, const void* logits, int ldz, const int32_t* lab, int M, int Mn, int Mpad, int V,
                      void* dz, float* row_loss, float* lse, float* loss_out, hipStream_t s);
// next-sentence head: small row-wise pieces around its three products
hipError_t gather_first_tokens(int dtype, const void* x, int S, int H, int n_seq, void* out, hipStream_t s);
hipError_t tanh_inplace(int dtype, void* u, size_t n, hipStream_t s);
hipError_t tanh_bwd(int dtype, const void* dp, const void* p, void* du, size_t n, hipStream_t s);
hipError_t nsp_ce(int dtype, const float* z, const int32_t* y, int n_seq, void* dz, float* loss, hipStream_t s);
hipError_t add_first_token_rows(int dtype, const void* dxc, const int32_t* inv, int S, int H, int n_seq, void* dxm,
                                hipStream_t s);

// embedding backward (first stage / retraining only): adds the gather contribution into gword,
// writes gpos (all gpos_rows rows) and gtype.  rank/order hold T ints, cnt/start round_up(vocab,4)
// ints, blockcnt embed_bwd_int_scratch(T, vocab) ints, scratch ceil(T/64)*type_vocab*H floats,
// partial T*H floats.
size_t embed_bwd_int_scratch(int T, int vocab);
hipError_t embed_bwd(int dtype, const void* dz, const int32_t* ids, const int32_t* tt, int B, int S, int H, int vocab,
                     int type_vocab, float* gword, float* gpos, float* gtype, int32_t* rank, int32_t* cnt,
                     int32_t* start, int32_t* order, int32_t* blockcnt, int gpos_rows, float* scratch, float* partial,
                     hipStream_t s);

// ---- optimizer ------------------------------------------------------------------------------
struct OptTensor {   // one logical tensor, device-side descriptor
  unsigned long long offset;
  unsigned long long count;
  int decays;
  int first_chunk;  // index of its first chunk in the global chunk list
  int n_chunks;
  int pad_;
};
struct OptHyper {
  int kind;
  float lr, beta1, beta2, eps, wd;
  int bias_correction;
  // device pointer to the loss of the step whose gradients are applied, or null: when set, the
  // update kernels do nothing unless that value is finite (lets an update be queued behind a step
  // before the host has seen its loss)
  const float* gate = nullptr;
};
constexpr int OPT_CHUNK = 16384;  // elements per workgroup
// Updates tensors [tensor0, tensor0+n_tensors), whose chunks are [chunk0, chunk0+n_chunks).
// tsteps[i] is tensor i's step count (already incremented for this update).
// chunk_norms: 2 floats per chunk; ratio: 1 float per tensor (LAMB only).
hipError_t bump_steps(int32_t* tsteps, int tensor0, int n_tensors, const float* gate, hipStream_t s);
hipError_t optimizer_step(const OptHyper& h, const OptTensor* tensors, const int32_t* tsteps, int tensor0,
                          int n_tensors, const int32_t* chunk_tensor, int chunk0, int n_chunks, float* w,
                          const float* g, float* m, float* v, bf16* shadow, float* chunk_norms, float* ratio,
                          hipStream_t s);

}  // namespace mslt
