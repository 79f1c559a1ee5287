// Row-wise, element-wise and indexing kernels of the MSLT stage step: embedding + LayerNorm,
// residual + LayerNorm and its backward, column sums for bias gradients, masked-row
// compaction / gather / scatter, cross-entropy over the vocabulary logits, embedding backward.
// All are bound by HBM traffic; rows are handled one wavefront (64 lanes) per row with the row
// held in registers, reductions by cross-lane shuffles.  No atomics on floating point: every
// reduction has a fixed order, so results are bitwise reproducible.
#include "common.h"

namespace mslt {

// ---- small vector helpers -------------------------------------------------------------------
__device__ inline float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ inline float4 load4(const bf16* p) {
  uint2 r = *reinterpret_cast<const uint2*>(p);
  float4 o;
  o.x = __uint_as_float(r.x << 16);
  o.y = __uint_as_float(r.x & 0xffff0000u);
  o.z = __uint_as_float(r.y << 16);
  o.w = __uint_as_float(r.y & 0xffff0000u);
  return o;
}
// Loads of a row's tail are made unconditional: lanes past the row end re-read column 0 (always in
// bounds) and drop the value, so that all loads of a thread issue back to back instead of one
// guarded load-and-wait at a time.
__device__ inline int ldcol(int c, int H) { return c < H ? c : 0; }
__device__ inline float4 keep4(bool keep, float4 v) { return keep ? v : make_float4(0.f, 0.f, 0.f, 0.f); }
// dropout factors of the 4 consecutive elements starting at element index e (a multiple of 4)
__device__ inline float4 drop4(const DropSpec& d, uint64_t e) {
  const uint64_t r = drop_quad(d, e >> 2);
  return make_float4(drop_field(d, r, 0), drop_field(d, r, 1), drop_field(d, r, 2), drop_field(d, r, 3));
}
__device__ inline float4 mul4(float4 a, float4 b) { return make_float4(a.x * b.x, a.y * b.y, a.z * b.z, a.w * b.w); }
__device__ inline void store4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
__device__ inline void store4(bf16* p, float4 v) {
  uint2 r;
  r.x = pack_bf16x2(v.x, v.y);
  r.y = pack_bf16x2(v.z, v.w);
  *reinterpret_cast<uint2*>(p) = r;
}

// ---- fill / cast ----------------------------------------------------------------------------
__global__ void k_fill_zero(uint32_t* p, size_t n_words) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t n4 = n_words / 4;
  uint4 z = make_uint4(0, 0, 0, 0);
  for (size_t j = i; j < n4; j += stride) reinterpret_cast<uint4*>(p)[j] = z;
  for (size_t j = n4 * 4 + i; j < n_words; j += stride) p[j] = 0;
}
hipError_t fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  if (bytes % 4 != 0 || (reinterpret_cast<uintptr_t>(p) % 16) != 0) return hipErrorInvalidValue;
  size_t words = bytes / 4;
  size_t blocks = (words / 4 + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 8192) blocks = 8192;
  k_fill_zero<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(reinterpret_cast<uint32_t*>(p), words);
  return hipGetLastError();
}

__global__ void k_cast_bf16(const float* __restrict__ src, bf16* __restrict__ dst, size_t n) {
  size_t i = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * 4;
  size_t stride = (size_t)gridDim.x * blockDim.x * 4;
  for (; i + 3 < n; i += stride) store4(dst + i, load4(src + i));
  // tail (n not a multiple of 4): handled by the first threads
  size_t t = (n / 4) * 4 + (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t < n) dst[t] = f2bf(src[t]);
}
hipError_t cast_f32_to_bf16(const float* src, bf16* dst, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n / 4 + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 8192) blocks = 8192;
  k_cast_bf16<<<dim3((unsigned)blocks), dim3(256), 0, s>>>(src, dst, n);
  return hipGetLastError();
}

template <typename AT>
__global__ void k_widen(const AT* __restrict__ src, float* __restrict__ dst, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) dst[i] = ldf(src + i);
}
hipError_t widen_to_f32(int dtype, const void* src, float* dst, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  if (dtype == 0)
    k_widen<float><<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const float*)src, dst, n);
  else
    k_widen<bf16><<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const bf16*)src, dst, n);
  return hipGetLastError();
}

// ---- batch check + compaction of predicted positions (integer, exact) -----------------------
__global__ void __launch_bounds__(1024) k_batch_scan(const int32_t* __restrict__ ids, const int32_t* __restrict__ tt,
                                                     const int32_t* __restrict__ am, const int32_t* __restrict__ labels,
                                                     int T, int vocab, int type_vocab, int cap, int32_t* pos,
                                                     int32_t* lab, int32_t* inv, int32_t* counters, int cls_every,
                                                     const int32_t* __restrict__ nsp_labels, int n_seq) {
  // cls_every > 0 (next-sentence head on): the first token of every sequence (t % cls_every == 0)
  // joins the compacted rows even without a label, because the classifier sends a gradient there;
  // its entry in lab stays -100.  counters: [0] rows, [1] error bits, [2] rows with a label.
  // One workgroup walks the tokens in chunks of 1024 (coalesced); inside a chunk the rank of a
  // predicted position is a wavefront ballot prefix plus the totals of the wavefronts before it.
  __shared__ int wtot[16];
  __shared__ int bad_all;
  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  if (tid == 0) bad_all = 0;
  __syncthreads();
  int base = 0, bad = 0, labelled = 0;
  if (nsp_labels != nullptr)
    for (int i = tid; i < n_seq; i += 1024) {
      int y = nsp_labels[i];
      if (y != 0 && y != 1) bad |= 16;
    }
  for (int c0 = 0; c0 < T; c0 += 1024) {
    const int t = c0 + tid;
    const bool in = t < T;
    int l = -100;
    if (in) {
      int id = ids[t];
      if (id < 0 || id >= vocab) bad |= 1;
      int ty = tt[t];
      if (ty < 0 || ty >= type_vocab) bad |= 2;
      int a = am[t];
      if (a != 0 && a != 1) bad |= 8;
      l = labels[t];
    }
    const bool has_label = in && l != -100;
    if (has_label && (l < 0 || l >= vocab)) bad |= 4;
    const bool v = has_label || (in && cls_every > 0 && t % cls_every == 0);
    labelled += __popcll(__ballot(has_label));       // the same count in every lane of the wavefront
    const unsigned long long mask = __ballot(v);
    const int within = __popcll(mask & ((1ull << lane) - 1ull));
    if (lane == 0) wtot[w] = __popcll(mask);
    __syncthreads();
    int before = 0, tot = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      int x = wtot[j];
      before += j < w ? x : 0;
      tot += x;
    }
    if (in) {
      const int off = base + before + within;
      if (v && off < cap) {
        pos[off] = t;
        lab[off] = l;
        inv[t] = off;
      } else {
        inv[t] = -1;
      }
    }
    base += tot;
    __syncthreads();
  }
  if (bad) atomicOr(&bad_all, bad);
  if (lane == 0) wtot[w] = labelled;
  __syncthreads();
  if (tid == 0) {
    int n = 0;
    for (int j = 0; j < 16; ++j) n += wtot[j];
    counters[0] = base;
    counters[1] = bad_all;
    counters[2] = n;
  }
}
hipError_t batch_scan(const int32_t* ids, const int32_t* tt, const int32_t* am, const int32_t* labels, int T, int vocab,
                      int type_vocab, int cap, int32_t* pos, int32_t* lab, int32_t* inv, int32_t* counters,
                      int cls_every, const int32_t* nsp_labels, int n_seq, hipStream_t s) {
  k_batch_scan<<<dim3(1), dim3(1024), 0, s>>>(ids, tt, am, labels, T, vocab, type_vocab, cap, pos, lab, inv, counters,
                                              cls_every, nsp_labels, n_seq);
  return hipGetLastError();
}

// ---- LayerNorm forward on a row held in registers -------------------------------------------
// NV = float4 per lane: a row of up to 256*NV elements lives in one wavefront's registers.
template <typename AT, int NV>
__device__ inline void ln_row_finish(float4 (&z)[NV], int H, int lane, const float* __restrict__ g,
                                     const float* __restrict__ b, float eps, AT* __restrict__ out,
                                     AT* __restrict__ xhat, float* __restrict__ rstd_out,
                                     const DropSpec& drop = DropSpec(), uint64_t drop_base = 0) {
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int c = (i * 64 + lane) * 4;
    if (c < H) sum += (z[i].x + z[i].y) + (z[i].z + z[i].w);
  }
  float mu = wave_sum(sum) / (float)H;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int c = (i * 64 + lane) * 4;
    if (c < H) {
      z[i].x -= mu; z[i].y -= mu; z[i].z -= mu; z[i].w -= mu;
      sq += (z[i].x * z[i].x + z[i].y * z[i].y) + (z[i].z * z[i].z + z[i].w * z[i].w);
    }
  }
  float var = wave_sum(sq) / (float)H;
  float rstd = 1.0f / sqrtf(var + eps);
  if (rstd_out != nullptr && lane == 0) *rstd_out = rstd;
  float4 gg[NV], bb[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int c = ldcol((i * 64 + lane) * 4, H);
    gg[i] = load4(g + c);
    bb[i] = load4(b + c);
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int c = (i * 64 + lane) * 4;
    if (c < H) {
      float4 xh = make_float4(z[i].x * rstd, z[i].y * rstd, z[i].z * rstd, z[i].w * rstd);
      if (xhat != nullptr) store4(xhat + c, xh);
      float4 y = make_float4(xh.x * gg[i].x + bb[i].x, xh.y * gg[i].y + bb[i].y, xh.z * gg[i].z + bb[i].z,
                             xh.w * gg[i].w + bb[i].w);
      if (drop.thr) y = mul4(y, drop4(drop, drop_base + c));     // dropout of the LayerNorm output
      store4(out + c, y);
    }
  }
}

template <typename AT, int NV>
__global__ void __launch_bounds__(256) k_embed_ln(const int32_t* __restrict__ ids, const int32_t* __restrict__ tt, int S,
                                                  const float* __restrict__ word, const float* __restrict__ pos,
                                                  const float* __restrict__ type, const float* __restrict__ g,
                                                  const float* __restrict__ b, float eps, AT* __restrict__ out,
                                                  AT* __restrict__ xhat, float* __restrict__ rstd, int T, int H,
                                                  int vocab, int type_vocab, DropSpec drop) {
  int lane = threadIdx.x & 63;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= T) return;
  // ids are clamped for memory safety only: a batch with ids out of range is rejected by the
  // batch check, whose verdict the host reads while this kernel may already be running
  const float* w = word + (size_t)min(max(ids[row], 0), vocab - 1) * H;
  const float* p = pos + (size_t)(row % S) * H;
  const float* ty = type + (size_t)min(max(tt[row], 0), type_vocab - 1) * H;
  float4 z[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int c = ldcol((i * 64 + lane) * 4, H);
    float4 a = load4(w + c), b2 = load4(p + c), c2 = load4(ty + c);
    z[i] = make_float4(a.x + b2.x + c2.x, a.y + b2.y + c2.y, a.z + b2.z + c2.z, a.w + b2.w + c2.w);
  }
  ln_row_finish<AT, NV>(z, H, lane, g, b, eps, out + (size_t)row * H, xhat ? xhat + (size_t)row * H : nullptr,
                        rstd ? rstd + row : nullptr, drop, (uint64_t)row * H);
}
static inline int ln_nv(int H) { return H <= 512 ? 2 : H <= 1024 ? 4 : 8; }
#define LN_DISPATCH(H, CALL)         \
  switch (ln_nv(H)) {                \
    case 2: { constexpr int NV = 2; CALL; } break; \
    case 4: { constexpr int NV = 4; CALL; } break; \
    default: { constexpr int NV = 8; CALL; } break; \
  }
hipError_t embed_ln_fwd(int dtype, const int32_t* ids, const int32_t* tt, int S, const float* word, const float* pos,
                        const float* type, const float* g, const float* b, float eps, void* out, LnStash st, int T,
                        int H, int vocab, int type_vocab, const DropSpec& drop, hipStream_t s) {
  dim3 grid((T + 3) / 4), block(256);
  if (dtype == 0) {
    LN_DISPATCH(H, (k_embed_ln<float, NV><<<grid, block, 0, s>>>(ids, tt, S, word, pos, type, g, b, eps, (float*)out,
                                                                 (float*)st.xhat, st.rstd, T, H, vocab, type_vocab, drop)));
  } else {
    LN_DISPATCH(H, (k_embed_ln<bf16, NV><<<grid, block, 0, s>>>(ids, tt, S, word, pos, type, g, b, eps, (bf16*)out,
                                                                (bf16*)st.xhat, st.rstd, T, H, vocab, type_vocab, drop)));
  }
  return hipGetLastError();
}

template <typename AT, int NV>
__global__ void __launch_bounds__(256) k_add_ln(const AT* __restrict__ a, const AT* __restrict__ r,
                                                const float* __restrict__ g, const float* __restrict__ b, float eps,
                                                AT* __restrict__ out, AT* __restrict__ xhat, float* __restrict__ rstd,
                                                int rows, int H) {
  int lane = threadIdx.x & 63;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const AT* pa = a + (size_t)row * H;
  const AT* pr = r ? r + (size_t)row * H : nullptr;
  float4 z[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) z[i] = load4(pa + ldcol((i * 64 + lane) * 4, H));
  if (pr) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      float4 y = load4(pr + ldcol((i * 64 + lane) * 4, H));
      z[i].x += y.x; z[i].y += y.y; z[i].z += y.z; z[i].w += y.w;
    }
  }
  ln_row_finish<AT, NV>(z, H, lane, g, b, eps, out + (size_t)row * H, xhat ? xhat + (size_t)row * H : nullptr,
                        rstd ? rstd + row : nullptr);
}
hipError_t add_ln_fwd(int dtype, const void* a, const void* r, const float* g, const float* b, float eps, void* out,
                      LnStash st, int rows, int H, hipStream_t s) {
  dim3 grid((rows + 3) / 4), block(256);
  if (dtype == 0) {
    LN_DISPATCH(H, (k_add_ln<float, NV><<<grid, block, 0, s>>>((const float*)a, (const float*)r, g, b, eps, (float*)out,
                                                               (float*)st.xhat, st.rstd, rows, H)));
  } else {
    LN_DISPATCH(H, (k_add_ln<bf16, NV><<<grid, block, 0, s>>>((const bf16*)a, (const bf16*)r, g, b, eps, (bf16*)out,
                                                              (bf16*)st.xhat, st.rstd, rows, H)));
  }
  return hipGetLastError();
}

// ---- reduction of partial column sums: out[c] = sum_p partial[p][c], fixed order ------------
// Up to three arrays per launch (blockIdx.y).  1024 threads = 32 columns x 32 partial-lanes; lane
// j adds partials j, j+32, ... in order, then the 32 lane sums are added in lane order.
struct ReduceArgs {
  const float* partial[3];
  float* out[3];
  int accumulate;     // add to what out holds (gradients of a parameter set shared by several layers)
};
__global__ void __launch_bounds__(1024) k_reduce_partials(ReduceArgs a, int n_partials, int N) {
  __shared__ float sh[32][33];
  const float* __restrict__ partial = a.partial[blockIdx.y];
  int cl = threadIdx.x & 31, pl = threadIdx.x >> 5;
  int c = blockIdx.x * 32 + cl;
  float acc = 0.f;
  if (c < N) {
    int p = pl;
    for (; p + 96 < n_partials; p += 128) {   // four independent loads in flight
      float v0 = partial[(size_t)p * N + c], v1 = partial[(size_t)(p + 32) * N + c];
      float v2 = partial[(size_t)(p + 64) * N + c], v3 = partial[(size_t)(p + 96) * N + c];
      acc += v0; acc += v1; acc += v2; acc += v3;
    }
    for (; p < n_partials; p += 32) acc += partial[(size_t)p * N + c];
  }
  sh[pl][cl] = acc;
  __syncthreads();
  if (pl == 0 && c < N) {
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < 32; ++j) v += sh[j][cl];
    a.out[blockIdx.y][c] = a.accumulate ? a.out[blockIdx.y][c] + v : v;
  }
}
static hipError_t reduce_partials(const float* partial, int n_partials, int N, float* out, hipStream_t s,
                                  int accumulate = 0) {
  ReduceArgs a{{partial, nullptr, nullptr}, {out, nullptr, nullptr}, accumulate};
  k_reduce_partials<<<dim3((N + 31) / 32, 1), dim3(1024), 0, s>>>(a, n_partials, N);
  return hipGetLastError();
}

// ---- many such sums in one launch ------------------------------------------------------------
// The job table travels in the kernel arguments.  A workgroup finds its job by its index; a row job uses the
// arithmetic of k_reduce_partials (same order of additions, so the result does not depend on whether a sum
// was carried out at once or later), a flat job adds the partials of four consecutive elements per thread.
constexpr int REDUCE_BATCH_JOBS = 112;
struct ReduceBatch {
  ReduceJob job[REDUCE_BATCH_JOBS];
  int n;
};
__global__ void __launch_bounds__(1024) k_reduce_batch(ReduceBatch b) {
  __shared__ float sh[32][33];
  int lo = 0, hi = b.n - 1;
  while (lo < hi) {
    int mid = (lo + hi + 1) >> 1;
    if (b.job[mid].first_block <= blockIdx.x) lo = mid; else hi = mid - 1;
  }
  const ReduceJob j = b.job[lo];
  const uint32_t blk = blockIdx.x - j.first_block;
  const float* __restrict__ partial = j.partial;
  const size_t N = j.N;
  const int n_partials = (int)j.n_partials;
  if (j.flags & 2u) {
    const size_t i = ((size_t)blk * 1024 + threadIdx.x) * 4;
    if (i >= N) return;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int p = 0; p < n_partials; ++p) {
      float4 a = *reinterpret_cast<const float4*>(partial + (size_t)p * N + i);
      v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
    }
    float4* o = reinterpret_cast<float4*>(j.out + i);
    if (j.flags & 1u) {
      float4 old = *o;
      v.x += old.x; v.y += old.y; v.z += old.z; v.w += old.w;
    }
    *o = v;
    return;
  }
  int cl = threadIdx.x & 31, pl = threadIdx.x >> 5;
  size_t c = (size_t)blk * 32 + cl;
  float acc = 0.f;
  if (c < N) {
    int p = pl;
    for (; p + 96 < n_partials; p += 128) {
      float v0 = partial[(size_t)p * N + c], v1 = partial[(size_t)(p + 32) * N + c];
      float v2 = partial[(size_t)(p + 64) * N + c], v3 = partial[(size_t)(p + 96) * N + c];
      acc += v0; acc += v1; acc += v2; acc += v3;
    }
    for (; p < n_partials; p += 32) acc += partial[(size_t)p * N + c];
  }
  sh[pl][cl] = acc;
  __syncthreads();
  if (pl == 0 && c < N) {
    float v = 0.f;
#pragma unroll
    for (int jj = 0; jj < 32; ++jj) v += sh[jj][cl];
    j.out[c] = (j.flags & 1u) ? j.out[c] + v : v;
  }
}
hipError_t reduce_batch(ReduceJob* jobs, int n, hipStream_t s) {
  for (int at = 0; at < n; at += REDUCE_BATCH_JOBS) {
    ReduceBatch b;
    b.n = n - at < REDUCE_BATCH_JOBS ? n - at : REDUCE_BATCH_JOBS;
    uint32_t blocks = 0;
    for (int i = 0; i < b.n; ++i) {
      ReduceJob& j = jobs[at + i];
      if (j.flags & 2u) {
        if (j.N % 4 || ((reinterpret_cast<uintptr_t>(j.partial) | reinterpret_cast<uintptr_t>(j.out)) & 15))
          return hipErrorInvalidValue;
      }
      j.first_block = blocks;
      blocks += (j.flags & 2u) ? (j.N + 4095) / 4096 : (j.N + 31) / 32;
      b.job[i] = j;
    }
    if (blocks == 0) continue;
    k_reduce_batch<<<dim3(blocks), dim3(1024), 0, s>>>(b);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

// ---- LayerNorm backward ---------------------------------------------------------------------
// One wavefront handles R consecutive rows (all loads issued before the row reductions), four
// wavefronts per workgroup; the workgroup leaves one partial row each of dgamma = sum dy*xhat,
// dbeta = sum dy and sum dz (the bias gradient of the linear layer in front of the LayerNorm).
static inline int lnb_rows_per_wave(int H) { return ln_nv(H) == 8 ? 2 : 4; }
size_t ln_bwd_scratch_floats(int rows, int H) {
  int rpb = 4 * lnb_rows_per_wave(H);
  return (size_t)3 * ((rows + rpb - 1) / rpb) * H;
}

// DROP: the dropout variants are a second compiled copy, so that the plain kernel carries none of their code
// DYT: type of dy (the activation type, or float for the wide residual gradient); dz32: optional fp32 copy of dz
template <typename AT, typename DYT, int NV, int R, bool DROP>
__global__ void __launch_bounds__(256) k_ln_bwd(const DYT* __restrict__ dy, const AT* __restrict__ xhat,
                                                const float* __restrict__ rstd, const float* __restrict__ g,
                                                AT* __restrict__ dz, float* __restrict__ dz32, float* __restrict__ part_g,
                                                float* __restrict__ part_b, float* __restrict__ part_z, int rows,
                                                int H, LnBwdDrop dd) {
  __shared__ float red[3][256 * NV];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float4 gg[NV], ag[NV], ab[NV], az[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    int c = (i * 64 + lane) * 4;
    ag[i] = ab[i] = az[i] = make_float4(0, 0, 0, 0);
    gg[i] = keep4(c < H, load4(g + ldcol(c, H)));
  }
  const int row0 = (blockIdx.x * 4 + wave) * R;
  const float invH = 1.0f / (float)H;
  float4 d[R][NV], x[R][NV];
  float rs[R];
#pragma unroll
  for (int rr = 0; rr < R; ++rr) {
    const int row = row0 + rr;
    const bool ok = row < rows;
    const size_t ro = (size_t)(ok ? row : rows - 1) * H;     // rows past the end re-read the last row
    rs[rr] = rstd[ok ? row : rows - 1];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = (i * 64 + lane) * 4;
      d[rr][i] = load4(dy + ro + ldcol(c, H));
      x[rr][i] = load4(xhat + ro + ldcol(c, H));
    }
  }
#pragma unroll
  for (int rr = 0; rr < R; ++rr) {
    const bool ok = row0 + rr < rows;
    if (!ok) rs[rr] = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const bool keep = ok && (i * 64 + lane) * 4 < H;
      d[rr][i] = keep4(keep, d[rr][i]);
      x[rr][i] = keep4(keep, x[rr][i]);
      // the LayerNorm output went through dropout (embedding block): so does its gradient
      if (DROP && dd.in.thr && keep) d[rr][i] = mul4(d[rr][i], drop4(dd.in, (uint64_t)(row0 + rr) * H + (i * 64 + lane) * 4));
    }
  }
#pragma unroll
  for (int rr = 0; rr < R; ++rr) {
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      float4 y = d[rr][i], xx = x[rr][i];
      ag[i].x += y.x * xx.x; ag[i].y += y.y * xx.y; ag[i].z += y.z * xx.z; ag[i].w += y.w * xx.w;
      ab[i].x += y.x; ab[i].y += y.y; ab[i].z += y.z; ab[i].w += y.w;
      y = make_float4(y.x * gg[i].x, y.y * gg[i].y, y.z * gg[i].z, y.w * gg[i].w);
      d[rr][i] = y;
      s1 += (y.x + y.y) + (y.z + y.w);
      s2 += (y.x * xx.x + y.y * xx.y) + (y.z * xx.z + y.w * xx.w);
    }
    float m1 = wave_sum(s1) * invH, m2 = wave_sum(s2) * invH;
    int row = row0 + rr;
    if (row < rows) {
      // the LayerNorm input was residual + dropout(linear output): the linear output's gradient is
      // dz times the same keep factors (element index by token row: compacted rows go through rowmap)
      uint64_t tok = (uint64_t)row;
      if (DROP && dd.out.thr && dd.rowmap) tok = row < dd.n_mapped ? (uint64_t)dd.rowmap[row] : 0;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        int c = (i * 64 + lane) * 4;
        if (c < H) {
          float4 y = d[rr][i], xx = x[rr][i];
          float4 o = make_float4((y.x - m1 - xx.x * m2) * rs[rr], (y.y - m1 - xx.y * m2) * rs[rr],
                                 (y.z - m1 - xx.z * m2) * rs[rr], (y.w - m1 - xx.w * m2) * rs[rr]);
          store4(dz + (size_t)row * H + c, o);
          if (dz32) *reinterpret_cast<float4*>(dz32 + (size_t)row * H + c) = o;
          if (DROP && dd.out.thr) {
            o = mul4(o, drop4(dd.out, tok * H + c));
            store4(reinterpret_cast<AT*>(dd.dzm) + (size_t)row * H + c, o);
          }
          az[i].x += o.x; az[i].y += o.y; az[i].z += o.z; az[i].w += o.w;
        }
      }
    }
  }
  // cross-wave reduction of the three per-column sums, waves added in order 0,1,2,3
#pragma unroll
  for (int pass = 0; pass < 3; ++pass) {
    float4* acc = pass == 0 ? ag : pass == 1 ? ab : az;
    if (wave > 0) {
#pragma unroll
      for (int i = 0; i < NV; ++i) *reinterpret_cast<float4*>(&red[wave - 1][(i * 64 + lane) * 4]) = acc[i];
    }
    __syncthreads();
    if (wave == 0) {
      float* dst = (pass == 0 ? part_g : pass == 1 ? part_b : part_z) + (size_t)blockIdx.x * H;
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        int c = (i * 64 + lane) * 4;
        if (c < H) {
          float4 v = acc[i];
#pragma unroll
          for (int w = 0; w < 3; ++w) {
            float4 o = *reinterpret_cast<float4*>(&red[w][c]);
            v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
          }
          *reinterpret_cast<float4*>(dst + c) = v;
        }
      }
    }
    __syncthreads();
  }
}
template <typename AT, typename DYT>
static hipError_t ln_bwd_t(const DYT* dy, const AT* xhat, const float* rstd, const float* g, AT* dz, float* dz32, float* dg,
                           float* db, float* dzsum, float* scratch, int rows, int H, const LnBwdDrop& dd, hipStream_t s,
                           ReduceJob* later, int* n_later) {
  if (dd.out.thr && dd.dzm == nullptr) return hipErrorInvalidValue;
  if (later != nullptr && n_later == nullptr) return hipErrorInvalidValue;
  if ((dd.out.thr || dd.in.thr) && H % 4) return hipErrorInvalidValue;
  int R = lnb_rows_per_wave(H);
  int nb = (rows + 4 * R - 1) / (4 * R);
  float* pg = scratch;
  float* pb = pg + (size_t)nb * H;
  float* pz = pb + (size_t)nb * H;
  const bool drop = dd.in.thr || dd.out.thr;
#define MSLT_LNB(NV, R)                                                                                                   \
  do {                                                                                                                    \
    if (drop) k_ln_bwd<AT, DYT, NV, R, true><<<dim3(nb), dim3(256), 0, s>>>(dy, xhat, rstd, g, dz, dz32, pg, pb, pz, rows, H, dd);  \
    else k_ln_bwd<AT, DYT, NV, R, false><<<dim3(nb), dim3(256), 0, s>>>(dy, xhat, rstd, g, dz, dz32, pg, pb, pz, rows, H, dd);      \
  } while (0)
  switch (ln_nv(H)) {
    case 2: MSLT_LNB(2, 4); break;
    case 4: MSLT_LNB(4, 4); break;
    default: MSLT_LNB(8, 2); break;
  }
#undef MSLT_LNB
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (later != nullptr) {
    int n = 0;
    later[n++] = reduce_job(pg, dg, nb, (size_t)H, dd.accumulate, false);
    later[n++] = reduce_job(pb, db, nb, (size_t)H, dd.accumulate, false);
    if (dzsum) later[n++] = reduce_job(pz, dzsum, nb, (size_t)H, dd.accumulate, false);
    *n_later = n;
    return hipSuccess;
  }
  ReduceArgs a{{pg, pb, pz}, {dg, db, dzsum}, dd.accumulate};
  k_reduce_partials<<<dim3((H + 31) / 32, dzsum ? 3 : 2), dim3(1024), 0, s>>>(a, nb, H);
  return hipGetLastError();
}
hipError_t ln_bwd(int dtype, const void* dy, const void* xhat, const float* rstd, const float* g, void* dz, float* dg,
                  float* db, float* dzsum, float* scratch, int rows, int H, const LnBwdDrop& dd, hipStream_t s, int dy_f32,
                  float* dz32, ReduceJob* later, int* n_later) {
  if (dtype == 0)
    return ln_bwd_t<float, float>((const float*)dy, (const float*)xhat, rstd, g, (float*)dz, dz32, dg, db, dzsum, scratch, rows,
                                  H, dd, s, later, n_later);
  if (dy_f32)
    return ln_bwd_t<bf16, float>((const float*)dy, (const bf16*)xhat, rstd, g, (bf16*)dz, dz32, dg, db, dzsum, scratch, rows, H,
                                 dd, s, later, n_later);
  return ln_bwd_t<bf16, bf16>((const bf16*)dy, (const bf16*)xhat, rstd, g, (bf16*)dz, dz32, dg, db, dzsum, scratch, rows, H, dd, s,
                              later, n_later);
}

// ---- column sums (bias gradients) -----------------------------------------------------------
// Vector path (N, ld multiples of 8): a workgroup takes 64 columns x 256 rows as 8 column-threads
// (8 columns = 16 or 32 bytes each) x 32 row-lanes; row-lanes are added in lane order through LDS.
constexpr int CS_ROWS = 64;        // rows per partial, scalar path
constexpr int CSV_ROWS = 256;      // rows per partial, vector path
size_t colsum_scratch_floats(int rows, int N) { return (size_t)((rows + CS_ROWS - 1) / CS_ROWS) * N; }

__device__ inline void load8(const float* p, float (&v)[8]) {
  float4 a = load4(p), b = load4(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ inline void load8(const bf16* p, float (&v)[8]) {
  uint4 r = *reinterpret_cast<const uint4*>(p);
  v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
  v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
  v[4] = __uint_as_float(r.z << 16); v[5] = __uint_as_float(r.z & 0xffff0000u);
  v[6] = __uint_as_float(r.w << 16); v[7] = __uint_as_float(r.w & 0xffff0000u);
}
template <typename AT>
__global__ void __launch_bounds__(256) k_colsum_vec(const AT* __restrict__ y, int ld, int rows, int N,
                                                    float* __restrict__ partial) {
  __shared__ float sh[32][65];
  int ct = threadIdx.x & 7, rl = threadIdx.x >> 3;
  int c = blockIdx.x * 64 + ct * 8;
  int r0 = blockIdx.y * CSV_ROWS;
  float acc[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (c < N) {
    // rows past the end re-read the last row and are dropped, so the loads issue back to back
    float v[CSV_ROWS / 32][8];
#pragma unroll
    for (int it = 0; it < CSV_ROWS / 32; ++it) {
      int r = r0 + it * 32 + rl;
      load8(y + (size_t)(r < rows ? r : rows - 1) * ld + c, v[it]);
    }
#pragma unroll
    for (int it = 0; it < CSV_ROWS / 32; ++it) {
      const bool ok = r0 + it * 32 + rl < rows;
#pragma unroll
      for (int i = 0; i < 8; ++i) acc[i] += ok ? v[it][i] : 0.f;
    }
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) sh[rl][ct * 8 + i] = acc[i];
  __syncthreads();
  if (threadIdx.x < 64) {
    int cc = blockIdx.x * 64 + threadIdx.x;
    if (cc < N) {
      float v = 0.f;
#pragma unroll
      for (int j = 0; j < 32; ++j) v += sh[j][threadIdx.x];
      partial[(size_t)blockIdx.y * N + cc] = v;
    }
  }
}
template <typename AT>
__global__ void __launch_bounds__(256) k_colsum_partial(const AT* __restrict__ y, int ld, int rows, int N,
                                                        float* __restrict__ partial) {
  int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= N) return;
  int r0 = blockIdx.y * CS_ROWS, r1 = min(rows, r0 + CS_ROWS);
  float acc = 0.f;
  for (int r = r0; r < r1; ++r) acc += ldf(y + (size_t)r * ld + c);
  partial[(size_t)blockIdx.y * N + c] = acc;
}
hipError_t colsum(int dtype, const void* y, int ld, int rows, int N, float* out, float* scratch, hipStream_t s,
                  int accumulate, ReduceJob* later) {
  bool vec = (N % 8 == 0) && (ld % 8 == 0) && ((reinterpret_cast<uintptr_t>(y) & 31) == 0);
  int nchunks;
  if (vec) {
    nchunks = (rows + CSV_ROWS - 1) / CSV_ROWS;
    dim3 grid((N + 63) / 64, nchunks), block(256);
    if (dtype == 0)
      k_colsum_vec<float><<<grid, block, 0, s>>>((const float*)y, ld, rows, N, scratch);
    else
      k_colsum_vec<bf16><<<grid, block, 0, s>>>((const bf16*)y, ld, rows, N, scratch);
  } else {
    nchunks = (rows + CS_ROWS - 1) / CS_ROWS;
    dim3 grid((N + 255) / 256, nchunks), block(256);
    if (dtype == 0)
      k_colsum_partial<float><<<grid, block, 0, s>>>((const float*)y, ld, rows, N, scratch);
    else
      k_colsum_partial<bf16><<<grid, block, 0, s>>>((const bf16*)y, ld, rows, N, scratch);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (later != nullptr) {
    *later = reduce_job(scratch, out, nchunks, (size_t)N, accumulate != 0, false);
    return hipSuccess;
  }
  return reduce_partials(scratch, nchunks, N, out, s, accumulate);
}

// ---- GELU backward of the head: gradient times the derivative stored by the forward epilogue
// (the layers fuse this into the GEMM epilogue) -------------------------------------------------
template <typename AT>
__global__ void k_mul_dgelu(const AT* __restrict__ dg, const AT* __restrict__ d, AT* __restrict__ du, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) stf(du + i, ldf(dg + i) * ld_dgelu(d + i));
}
hipError_t mul_dgelu(int dtype, const void* dg, const void* u, void* du, size_t n, hipStream_t s) {
  if (n == 0) return hipSuccess;
  size_t blocks = (n + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  if (dtype == 0)
    k_mul_dgelu<float><<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const float*)dg, (const float*)u, (float*)du, n);
  else
    k_mul_dgelu<bf16><<<dim3((unsigned)blocks), dim3(256), 0, s>>>((const bf16*)dg, (const bf16*)u, (bf16*)du, n);
  return hipGetLastError();
}

// ---- gather of predicted rows / scatter of their gradients ----------------------------------
// Gathers rows pos[0..M) of up to GATHER_MAX arrays in one launch (blockIdx.y picks the array) and
// zero-fills rows [M, Mpad).  Rows are copied as raw bytes, whatever they encode.
template <typename U>
__device__ inline void copy_row(char* __restrict__ o, const char* __restrict__ src, int row_bytes) {
  for (int c = threadIdx.x * (int)sizeof(U); c < row_bytes; c += blockDim.x * (int)sizeof(U)) {
    U v = U();
    if (src) v = *reinterpret_cast<const U*>(src + c);
    *reinterpret_cast<U*>(o + c) = v;
  }
}
__global__ void __launch_bounds__(64) k_gather_multi(GatherArgs a, const int32_t* __restrict__ pos, int M) {
  const int j = blockIdx.x;
  const GatherDesc g = a.d[blockIdx.y];
  char* o = reinterpret_cast<char*>(g.dst) + (size_t)j * g.row_bytes;
  const char* src = j < M ? reinterpret_cast<const char*>(g.src) + (size_t)pos[j] * g.row_bytes : nullptr;
  if (g.row_bytes % 16 == 0) copy_row<uint4>(o, src, g.row_bytes);
  else if (g.row_bytes % 8 == 0) copy_row<uint2>(o, src, g.row_bytes);
  else copy_row<uint32_t>(o, src, g.row_bytes);
}
hipError_t gather_rows_multi(const GatherDesc* descs, int n, const int32_t* pos, int M, int Mpad, hipStream_t s) {
  if (n < 1 || n > GATHER_MAX) return hipErrorInvalidValue;
  GatherArgs a;
  for (int i = 0; i < n; ++i) {
    if (descs[i].row_bytes <= 0 || descs[i].row_bytes % 4) return hipErrorInvalidValue;
    a.d[i] = descs[i];
  }
  for (int i = n; i < GATHER_MAX; ++i) a.d[i] = descs[0];
  k_gather_multi<<<dim3(Mpad, n), dim3(64), 0, s>>>(a, pos, M);
  return hipGetLastError();
}

template <typename AT>
__global__ void k_scatter_rows(const AT* __restrict__ dxm, const int32_t* __restrict__ inv, int T, int H,
                               AT* __restrict__ out) {
  int t = blockIdx.x;
  int j = t < T ? inv[t] : -1;
  AT* o = out + (size_t)t * H;
  if (j >= 0) {
    const AT* src = dxm + (size_t)j * H;
    for (int c = threadIdx.x * 4; c < H; c += blockDim.x * 4) store4(o + c, load4(src + c));
  } else {
    for (int c = threadIdx.x * 4; c < H; c += blockDim.x * 4) store4(o + c, make_float4(0, 0, 0, 0));
  }
}
hipError_t scatter_rows(int dtype, const void* dxm, const int32_t* inv, int rows_total, int T, int H, void* out,
                        hipStream_t s) {
  if (dtype == 0)
    k_scatter_rows<float><<<dim3(rows_total), dim3(64), 0, s>>>((const float*)dxm, inv, T, H, (float*)out);
  else
    k_scatter_rows<bf16><<<dim3(rows_total), dim3(64), 0, s>>>((const bf16*)dxm, inv, T, H, (bf16*)out);
  return hipGetLastError();
}

// ---- cross-entropy over the vocabulary ------------------------------------------------------
__device__ inline float block_reduce_sum_256(float v, float* sh) {
  v = wave_sum(v);
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}
__device__ inline float block_reduce_max_256(float v, float* sh) {
  v = wave_max(v);
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) sh[wave] = v;
  __syncthreads();
  return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
}

// Cross-entropy over the logits of the predicted rows, forward and backward in one pass per row.  The
// logits are of the activation type (bf16 logits halve the traffic of the largest tensor of the head;
// their rounding, 2^-9 relative per logit, averages out in the log-sum-exp and is an order below the
// rounding of dZ itself).  dz may be the logits buffer itself: a row is overwritten only after the
// kernel has taken everything it needs from it.
template <typename AT>
__global__ void __launch_bounds__(256) k_ce(const AT* __restrict__ logits, int ldz, const int32_t* __restrict__ lab,
                                            int M, int Mn, int V, AT* dz, float* __restrict__ row_loss,
                                            float* __restrict__ lse_out) {
  __shared__ float sh[4];
  int j = blockIdx.x;
  AT* d = dz + (size_t)j * ldz;
  if (j >= M || lab[j] < 0) {      // padding row, or a row that is only there for the next-sentence head
    for (int c = threadIdx.x; c < ldz; c += 256) stf(d + c, 0.f);
    if (j < M && threadIdx.x == 0) { row_loss[j] = 0.f; lse_out[j] = 0.f; }
    return;
  }
  const AT* z = logits + (size_t)j * ldz;
  float mx = -INFINITY;
  for (int c = threadIdx.x; c < V; c += 256) mx = fmaxf(mx, ldf(z + c));
  mx = block_reduce_max_256(mx, sh);
  float se = 0.f;
  for (int c = threadIdx.x; c < V; c += 256) se += __expf(ldf(z + c) - mx);
  se = block_reduce_sum_256(se, sh);
  float lse = mx + __logf(se);
  int y = lab[j];
  const float zy = ldf(z + y);     // before the row is overwritten (dz may alias the logits)
  __syncthreads();
  float invM = 1.0f / (float)Mn;
  for (int c = threadIdx.x; c < ldz; c += 256) {
    float v = 0.f;
    if (c < V) v = (__expf(ldf(z + c) - lse) - (c == y ? 1.0f : 0.0f)) * invM;
    stf(d + c, v);
  }
  if (threadIdx.x == 0) {
    row_loss[j] = lse - zy;
    lse_out[j] = lse;
  }
}
// Same, with the row of logits resident in LDS (V elements of dynamic LDS): one global read of the
// logits and one write of dZ per row, 1024 threads per row.
template <typename AT>
__global__ void __launch_bounds__(1024) k_ce_lds(const AT* __restrict__ logits, int ldz, const int32_t* __restrict__ lab,
                                                 int M, int Mn, int V, AT* dz, float* __restrict__ row_loss,
                                                 float* __restrict__ lse_out) {
  extern __shared__ __attribute__((aligned(16))) unsigned char row_raw[];
  AT* row = reinterpret_cast<AT*>(row_raw);
  __shared__ float sh[16];
  const int j = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  AT* d = dz + (size_t)j * ldz;
  if (j >= M || lab[j] < 0) {      // padding row, or a row that is only there for the next-sentence head
    for (int c = tid * 4; c < ldz; c += 4096) store4(d + c, make_float4(0, 0, 0, 0));
    if (j < M && tid == 0) { row_loss[j] = 0.f; lse_out[j] = 0.f; }
    return;
  }
  const AT* z = logits + (size_t)j * ldz;
  const int V4 = V & ~3;
  float mx = -INFINITY;
  for (int c = tid * 4; c < V4; c += 4096) {
    float4 v = load4(z + c);
    store4(row + c, v);              // exact: the values are of type AT already
    mx = fmaxf(mx, fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w)));
  }
  for (int c = V4 + tid; c < V; c += 1024) {
    float v = ldf(z + c);
    stf(row + c, v);
    mx = fmaxf(mx, v);
  }
  mx = wave_max(mx);
  if (lane == 0) sh[wave] = mx;
  __syncthreads();
  mx = sh[0];
#pragma unroll
  for (int w = 1; w < 16; ++w) mx = fmaxf(mx, sh[w]);
  float se = 0.f;
  for (int c = tid; c < V; c += 1024) se += __expf(ldf(row + c) - mx);
  se = wave_sum(se);
  __syncthreads();
  if (lane == 0) sh[wave] = se;
  __syncthreads();
  se = 0.f;
#pragma unroll
  for (int w = 0; w < 16; ++w) se += sh[w];
  const float lse = mx + __logf(se);
  const int y = lab[j];
  const float invM = 1.0f / (float)Mn;
  for (int c = tid * 4; c < ldz; c += 4096) {
    float o[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int cc = c + i;
      o[i] = cc < V ? (__expf(ldf(row + cc) - lse) - (cc == y ? 1.0f : 0.0f)) * invM : 0.f;
    }
    store4(d + c, make_float4(o[0], o[1], o[2], o[3]));
  }
  if (tid == 0) {
    row_loss[j] = lse - ldf(row + y);
    lse_out[j] = lse;
  }
}
__global__ void __launch_bounds__(256) k_mean_rows(const float* __restrict__ v, int M, int Mn, float* __restrict__ out) {
  __shared__ float sh[256];
  float acc = 0.f;
  for (int i = threadIdx.x; i < M; i += 256) acc += v[i];
  sh[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = sh[0] / (float)Mn;     // mean over the rows that carry a label
}
hipError_t ce_fwd_bwd(int dtype, const void* logits, int ldz, const int32_t* lab, int M, int Mn, int Mpad, int V,
                      void* dz, float* row_loss, float* lse, float* loss_out, hipStream_t s) {
  const size_t row_bytes = (size_t)V * (dtype ? 2 : 4);
  hipError_t e;
  if (row_bytes <= 150 * 1024 && ldz % 4 == 0) {
    static bool attr_set = false;
    if (!attr_set) {
      if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_ce_lds<float>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024)) != hipSuccess) return e;
      if ((e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_ce_lds<bf16>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024)) != hipSuccess) return e;
      attr_set = true;
    }
    if (dtype == 0)
      k_ce_lds<float><<<dim3(Mpad), dim3(1024), row_bytes, s>>>((const float*)logits, ldz, lab, M, Mn, V, (float*)dz, row_loss, lse);
    else
      k_ce_lds<bf16><<<dim3(Mpad), dim3(1024), row_bytes, s>>>((const bf16*)logits, ldz, lab, M, Mn, V, (bf16*)dz, row_loss, lse);
  } else if (dtype == 0) {
    k_ce<float><<<dim3(Mpad), dim3(256), 0, s>>>((const float*)logits, ldz, lab, M, Mn, V, (float*)dz, row_loss, lse);
  } else {
    k_ce<bf16><<<dim3(Mpad), dim3(256), 0, s>>>((const bf16*)logits, ldz, lab, M, Mn, V, (bf16*)dz, row_loss, lse);
  }
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  k_mean_rows<<<dim3(1), dim3(256), 0, s>>>(row_loss, M, Mn, loss_out);
  return hipGetLastError();
}

// ---- embedding backward (first stage and retraining only) -----------------------------------
// Word rows: tokens are grouped by id with their original order kept inside a group (a stable
// counting sort), so each vocabulary row is summed in ascending token order: deterministic, no
// floating-point atomics.  Stable position of token t = start[id] + (occurrences of id in earlier
// blocks of 256 tokens) + (occurrences earlier in t's own block).
constexpr int RK_BLOCK = 256;
__global__ void __launch_bounds__(RK_BLOCK) k_rank_local(const int32_t* __restrict__ ids, int T, int V,
                                                        int32_t* __restrict__ rank, int32_t* __restrict__ blockcnt) {
  __shared__ int tile[RK_BLOCK];
  const int t = blockIdx.x * RK_BLOCK + threadIdx.x;
  const int id = t < T ? ids[t] : -1;
  tile[threadIdx.x] = id;
  __syncthreads();
  int before = 0, after = 0;
#pragma unroll 8
  for (int j = 0; j < RK_BLOCK; ++j) {
    int same = tile[j] == id ? 1 : 0;
    before += (j < (int)threadIdx.x) ? same : 0;
    after += (j > (int)threadIdx.x) ? same : 0;
  }
  if (t < T) {
    rank[t] = before;
    if (after == 0) blockcnt[(size_t)blockIdx.x * V + id] = before + 1;   // last occurrence in the block
  }
}
// per id: exclusive prefix over the blocks (in place) and the total count
__global__ void k_block_prefix(int32_t* __restrict__ blockcnt, int nblocks, int V, int32_t* __restrict__ cnt) {
  int v = blockIdx.x * blockDim.x + threadIdx.x;
  if (v >= V) return;
  int run = 0;
  for (int b = 0; b < nblocks; ++b) {
    int c = blockcnt[(size_t)b * V + v];
    blockcnt[(size_t)b * V + v] = run;
    run += c;
  }
  cnt[v] = run;
}
// exclusive scan of n ints in three small launches: 1024-element blocks, their totals, the fix-up
__global__ void __launch_bounds__(1024) k_scan_blocks(const int32_t* __restrict__ in, int n, int32_t* __restrict__ out,
                                                      int32_t* __restrict__ totals) {
  __shared__ int sc[1024];
  int i = blockIdx.x * 1024 + threadIdx.x;
  int v = i < n ? in[i] : 0;
  sc[threadIdx.x] = v;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    int a = (int)threadIdx.x >= o ? sc[threadIdx.x - o] : 0;
    __syncthreads();
    sc[threadIdx.x] += a;
    __syncthreads();
  }
  if (i < n) out[i] = sc[threadIdx.x] - v;
  if (threadIdx.x == 1023) totals[blockIdx.x] = sc[1023];
}
__global__ void __launch_bounds__(1024) k_scan_totals(int32_t* __restrict__ totals, int nb) {
  __shared__ int sc[1024];
  int v = (int)threadIdx.x < nb ? totals[threadIdx.x] : 0;
  sc[threadIdx.x] = v;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    int a = (int)threadIdx.x >= o ? sc[threadIdx.x - o] : 0;
    __syncthreads();
    sc[threadIdx.x] += a;
    __syncthreads();
  }
  if ((int)threadIdx.x < nb) totals[threadIdx.x] = sc[threadIdx.x] - v;
}
__global__ void __launch_bounds__(1024) k_scan_add(int32_t* __restrict__ out, int n, const int32_t* __restrict__ totals) {
  int i = blockIdx.x * 1024 + threadIdx.x;
  if (i < n) out[i] += totals[blockIdx.x];
}
__global__ void k_token_order(const int32_t* __restrict__ ids, const int32_t* __restrict__ rank,
                              const int32_t* __restrict__ start, const int32_t* __restrict__ blockcnt, int T, int V,
                              int32_t* __restrict__ order) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= T) return;
  int id = ids[t];
  order[start[id] + blockcnt[(size_t)(t / RK_BLOCK) * V + id] + rank[t]] = t;
}
size_t embed_bwd_int_scratch(int T, int vocab) {   // ints: per-block counts + scan totals
  return (size_t)((T + RK_BLOCK - 1) / RK_BLOCK) * vocab + 1024;
}
// Level 1: the id-sorted token list is cut into chunks of WG_CHUNK positions; a workgroup adds, in
// order, the rows of every run of equal ids inside its chunk and leaves the sum at the row of the
// run's first position in `partial` [T, H].
constexpr int WG_CHUNK = 32;
template <typename AT>
__global__ void __launch_bounds__(256) k_word_grad_chunks(const AT* __restrict__ dz, const int32_t* __restrict__ ids,
                                                          const int32_t* __restrict__ order, int T, int H,
                                                          float* __restrict__ partial) {
  __shared__ int tok[WG_CHUNK], tid_of[WG_CHUNK];
  const int p0 = blockIdx.x * WG_CHUNK, n = min(WG_CHUNK, T - p0);
  if ((int)threadIdx.x < n) {
    int t = order[p0 + threadIdx.x];
    tok[threadIdx.x] = t;
    tid_of[threadIdx.x] = ids[t];
  }
  __syncthreads();
  for (int c = threadIdx.x * 4; c < H; c += 1024) {
    float4 acc = make_float4(0, 0, 0, 0);
    int run_start = 0;
    for (int i = 0; i < n; ++i) {
      if (i > 0 && tid_of[i] != tid_of[i - 1]) {
        store4(partial + (size_t)(p0 + run_start) * H + c, acc);
        acc = make_float4(0, 0, 0, 0);
        run_start = i;
      }
      float4 v = load4(dz + (size_t)tok[i] * H + c);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    store4(partial + (size_t)(p0 + run_start) * H + c, acc);
  }
}
// Level 2: one workgroup per vocabulary row adds the row's chunk partials in chunk order.
__global__ void __launch_bounds__(256) k_word_grad_rows(const float* __restrict__ partial, const int32_t* __restrict__ cnt,
                                                        const int32_t* __restrict__ start, int H,
                                                        float* __restrict__ gword) {
  const int v = blockIdx.x, n = cnt[v];
  if (n == 0) return;
  const int s0 = start[v], s1 = s0 + n;
  for (int c = threadIdx.x * 4; c < H; c += 1024) {
    float4 acc = make_float4(0, 0, 0, 0);
    for (int p = s0; p < s1; p = (p / WG_CHUNK + 1) * WG_CHUNK) {   // run of v in each chunk starts at p
      float4 x = load4(partial + (size_t)p * H + c);
      acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
    }
    float4 g = load4(gword + (size_t)v * H + c);
    store4(gword + (size_t)v * H + c, make_float4(g.x + acc.x, g.y + acc.y, g.z + acc.z, g.w + acc.w));
  }
}
template <typename AT>
__global__ void k_pos_grad(const AT* __restrict__ dz, int B, int S, int H, int rows_total, float* __restrict__ gpos) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)rows_total * H) return;
  int s = (int)(i / H), c = (int)(i % H);
  float acc = 0.f;
  if (s < S)
    for (int b = 0; b < B; ++b) acc += ldf(dz + ((size_t)b * S + s) * H + c);
  gpos[i] = acc;
}
template <typename AT>
__global__ void __launch_bounds__(256) k_type_partial(const AT* __restrict__ dz, const int32_t* __restrict__ tt, int T,
                                                      int H, int type_vocab, float* __restrict__ partial) {
  int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= H) return;
  int r0 = blockIdx.y * CS_ROWS, r1 = min(T, r0 + CS_ROWS);
  float acc[4] = {0.f, 0.f, 0.f, 0.f};
  for (int r = r0; r < r1; ++r) {
    float v = ldf(dz + (size_t)r * H + c);
    int ty = tt[r];
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[k] += (ty == k) ? v : 0.f;
  }
  for (int k = 0; k < type_vocab; ++k) partial[((size_t)blockIdx.y * type_vocab + k) * H + c] = acc[k];
}
template <typename AT>
static hipError_t embed_bwd_t(const AT* dz, const int32_t* ids, const int32_t* tt, int B, int S, int H, int vocab,
                              int type_vocab, float* gword, float* gpos, float* gtype, int32_t* rank, int32_t* cnt,
                              int32_t* start, int32_t* order, int32_t* blockcnt, int gpos_rows, float* scratch, float* partial,
                              hipStream_t s) {
  int T = B * S;
  int nblk = (T + RK_BLOCK - 1) / RK_BLOCK, nsb = (vocab + 1023) / 1024;
  if (nsb > 1024) return hipErrorInvalidValue;   // vocabulary above 2^20 rows is not supported here
  int32_t* totals = blockcnt + (size_t)nblk * vocab;
  hipError_t e = fill_zero(blockcnt, ((size_t)nblk * vocab + 3) / 4 * 16, s);
  if (e != hipSuccess) return e;
  k_rank_local<<<dim3(nblk), dim3(RK_BLOCK), 0, s>>>(ids, T, vocab, rank, blockcnt);
  k_block_prefix<<<dim3((vocab + 255) / 256), dim3(256), 0, s>>>(blockcnt, nblk, vocab, cnt);
  k_scan_blocks<<<dim3(nsb), dim3(1024), 0, s>>>(cnt, vocab, start, totals);
  k_scan_totals<<<dim3(1), dim3(1024), 0, s>>>(totals, nsb);
  k_scan_add<<<dim3(nsb), dim3(1024), 0, s>>>(start, vocab, totals);
  k_token_order<<<dim3((T + 255) / 256), dim3(256), 0, s>>>(ids, rank, start, blockcnt, T, vocab, order);
  k_word_grad_chunks<AT><<<dim3((T + WG_CHUNK - 1) / WG_CHUNK), dim3(256), 0, s>>>(dz, ids, order, T, H, partial);
  k_word_grad_rows<<<dim3(vocab), dim3(256), 0, s>>>(partial, cnt, start, H, gword);
  size_t np = (size_t)gpos_rows * H;
  k_pos_grad<AT><<<dim3((unsigned)((np + 255) / 256)), dim3(256), 0, s>>>(dz, B, S, H, gpos_rows, gpos);
  int nchunks = (T + CS_ROWS - 1) / CS_ROWS;
  k_type_partial<AT><<<dim3((H + 255) / 256, nchunks), dim3(256), 0, s>>>(dz, tt, T, H, type_vocab, scratch);
  int N = type_vocab * H;
  return reduce_partials(scratch, nchunks, N, gtype, s);
}
hipError_t embed_bwd(int dtype, const void* dz, const int32_t* ids, const int32_t* tt, int B, int S, int H, int vocab,
                     int type_vocab, float* gword, float* gpos, float* gtype, int32_t* rank, int32_t* cnt,
                     int32_t* start, int32_t* order, int32_t* blockcnt, int gpos_rows, float* scratch, float* partial,
                     hipStream_t s) {
  if (dtype == 0)
    return embed_bwd_t<float>((const float*)dz, ids, tt, B, S, H, vocab, type_vocab, gword, gpos, gtype, rank, cnt,
                              start, order, blockcnt, gpos_rows, scratch, partial, s);
  return embed_bwd_t<bf16>((const bf16*)dz, ids, tt, B, S, H, vocab, type_vocab, gword, gpos, gtype, rank, cnt, start,
                           order, blockcnt, gpos_rows, scratch, partial, s);
}

// ---- fused multi-tensor Adam / LAMB ---------------------------------------------------------
// One workgroup per chunk of OPT_CHUNK elements of one logical tensor.
// Pass 1 updates the moments; Adam also applies the step.  LAMB leaves per-chunk sums of w^2 and
// u^2, a second kernel adds them per tensor in chunk order, and pass 2 recomputes u from the new
// moments and applies the step with the tensor's trust ratio.
__device__ inline bool gate_closed(const float* gate) { return gate != nullptr && !isfinite(*gate); }
__global__ void k_bump_steps(int32_t* tsteps, int tensor0, int n, const float* gate) {
  if (gate_closed(gate)) return;
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) tsteps[tensor0 + i] += 1;
}
hipError_t bump_steps(int32_t* tsteps, int tensor0, int n_tensors, const float* gate, hipStream_t s) {
  if (n_tensors <= 0) return hipSuccess;
  k_bump_steps<<<dim3((n_tensors + 63) / 64), dim3(64), 0, s>>>(tsteps, tensor0, n_tensors, gate);
  return hipGetLastError();
}
__device__ inline void opt_corrections(const OptHyper& h, int t, float& c1, float& c2) {
  if (h.bias_correction) {
    c1 = (float)(1.0 / (1.0 - pow((double)h.beta1, (double)t)));
    c2 = (float)(1.0 / (1.0 - pow((double)h.beta2, (double)t)));
  } else {
    c1 = 1.f;
    c2 = 1.f;
  }
}
__global__ void __launch_bounds__(256) k_opt_pass1(OptHyper h, const OptTensor* __restrict__ tensors,
                                                   const int32_t* __restrict__ tsteps,
                                                   const int32_t* __restrict__ chunk_tensor, int chunk0,
                                                   float* __restrict__ w, const float* __restrict__ g,
                                                   float* __restrict__ m, float* __restrict__ v,
                                                   bf16* __restrict__ shadow, float* __restrict__ chunk_norms) {
  __shared__ float sh[4];
  if (gate_closed(h.gate)) return;
  int chunk = chunk0 + blockIdx.x;
  int ti = chunk_tensor[chunk];
  OptTensor tn = tensors[ti];
  size_t lo = (size_t)(chunk - tn.first_chunk) * OPT_CHUNK;
  size_t hi = lo + OPT_CHUNK < tn.count ? lo + OPT_CHUNK : (size_t)tn.count;
  float c1, c2;
  opt_corrections(h, tsteps[ti], c1, c2);
  float wd = tn.decays ? h.wd : 0.f;
  float sw = 0.f, su = 0.f;
  for (size_t i = lo + threadIdx.x; i < hi; i += 256) {
    size_t a = tn.offset + i;
    float gi = g[a], wi = w[a];
    float mi = h.beta1 * m[a] + (1.f - h.beta1) * gi;
    float vi = h.beta2 * v[a] + (1.f - h.beta2) * gi * gi;
    m[a] = mi;
    v[a] = vi;
    float u = (mi * c1) / (sqrtf(vi * c2) + h.eps) + wd * wi;
    if (h.kind == 0) {
      wi -= h.lr * u;
      w[a] = wi;
      if (shadow) shadow[a] = f2bf(wi);
    } else {
      sw += wi * wi;
      su += u * u;
    }
  }
  if (h.kind != 0) {
    sw = block_reduce_sum_256(sw, sh);
    su = block_reduce_sum_256(su, sh);
    if (threadIdx.x == 0) {
      chunk_norms[2 * (size_t)chunk] = sw;
      chunk_norms[2 * (size_t)chunk + 1] = su;
    }
  }
}
// one wavefront per tensor: lane j adds chunks j, j+64, ... in that order, then the lanes are added in a fixed
// butterfly order, so the ratio is the same in every run
__global__ void __launch_bounds__(64) k_lamb_ratio(const OptTensor* __restrict__ tensors, int tensor0, int n_tensors,
                                                   const float* __restrict__ chunk_norms, float* __restrict__ ratio) {
  const int i = blockIdx.x, lane = threadIdx.x;
  if (i >= n_tensors) return;
  OptTensor tn = tensors[tensor0 + i];
  float sw = 0.f, su = 0.f;
  for (int c = lane; c < tn.n_chunks; c += 64) {
    sw += chunk_norms[2 * (size_t)(tn.first_chunk + c)];
    su += chunk_norms[2 * (size_t)(tn.first_chunk + c) + 1];
  }
  sw = wave_sum(sw);
  su = wave_sum(su);
  if (lane == 0) {
    float wn = sqrtf(sw), un = sqrtf(su);
    ratio[tensor0 + i] = (wn > 0.f && un > 0.f) ? wn / un : 1.0f;
  }
}
__global__ void __launch_bounds__(256) k_lamb_pass2(OptHyper h, const OptTensor* __restrict__ tensors,
                                                    const int32_t* __restrict__ tsteps,
                                                    const int32_t* __restrict__ chunk_tensor, int chunk0,
                                                    float* __restrict__ w, const float* __restrict__ m,
                                                    const float* __restrict__ v, bf16* __restrict__ shadow,
                                                    const float* __restrict__ ratio) {
  if (gate_closed(h.gate)) return;
  int chunk = chunk0 + blockIdx.x;
  int ti = chunk_tensor[chunk];
  OptTensor tn = tensors[ti];
  size_t lo = (size_t)(chunk - tn.first_chunk) * OPT_CHUNK;
  size_t hi = lo + OPT_CHUNK < tn.count ? lo + OPT_CHUNK : (size_t)tn.count;
  float c1, c2;
  opt_corrections(h, tsteps[ti], c1, c2);
  float wd = tn.decays ? h.wd : 0.f;
  float step = h.lr * ratio[ti];
  for (size_t i = lo + threadIdx.x; i < hi; i += 256) {
    size_t a = tn.offset + i;
    float wi = w[a];
    float u = (m[a] * c1) / (sqrtf(v[a] * c2) + h.eps) + wd * wi;
    wi -= step * u;
    w[a] = wi;
    if (shadow) shadow[a] = f2bf(wi);
  }
}
hipError_t optimizer_step(const OptHyper& h, const OptTensor* tensors, const int32_t* tsteps, int tensor0,
                          int n_tensors, const int32_t* chunk_tensor, int chunk0, int n_chunks, float* w,
                          const float* g, float* m, float* v, bf16* shadow, float* chunk_norms, float* ratio,
                          hipStream_t s) {
  if (n_chunks <= 0) return hipSuccess;
  k_opt_pass1<<<dim3(n_chunks), dim3(256), 0, s>>>(h, tensors, tsteps, chunk_tensor, chunk0, w, g, m, v, shadow,
                                                   chunk_norms);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || h.kind == 0) return e;
  k_lamb_ratio<<<dim3(n_tensors), dim3(64), 0, s>>>(tensors, tensor0, n_tensors, chunk_norms, ratio);
  k_lamb_pass2<<<dim3(n_chunks), dim3(256), 0, s>>>(h, tensors, tsteps, chunk_tensor, chunk0, w, m, v, shadow, ratio);
  return hipGetLastError();
}

// ---- next-sentence head (pooler + two-way classifier on the first token of every sequence) ----
// These work on batch-many rows: a few thousand elements, small launches.
template <typename AT>
__global__ void k_gather_first_tokens(const AT* __restrict__ x, int S, int H, AT* __restrict__ out) {
  int b = blockIdx.x;
  for (int c = threadIdx.x; c < H; c += blockDim.x) out[(size_t)b * H + c] = x[(size_t)b * S * H + c];
}
template <typename AT>
__global__ void k_tanh_inplace(AT* __restrict__ u, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) stf(u + i, tanhf(ldf(u + i)));
}
// du = dp * (1 - p^2)
template <typename AT>
__global__ void k_tanh_bwd(const AT* __restrict__ dp, const AT* __restrict__ p, AT* __restrict__ du, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    float t = ldf(p + i);
    stf(du + i, ldf(dp + i) * (1.0f - t * t));
  }
}
// two-way cross-entropy: dz = (softmax(z) - onehot) / n_seq, *loss += mean loss (one workgroup)
template <typename AT>
__global__ void __launch_bounds__(256) k_nsp_ce(const float* __restrict__ z, const int32_t* __restrict__ y, int n_seq,
                                                AT* __restrict__ dz, float* __restrict__ loss) {
  __shared__ float sh[256];
  float acc = 0.f;
  const float inv = 1.0f / (float)n_seq;
  for (int b = threadIdx.x; b < n_seq; b += 256) {
    float z0 = z[2 * b], z1 = z[2 * b + 1];
    float mx = fmaxf(z0, z1);
    float lse = mx + __logf(__expf(z0 - mx) + __expf(z1 - mx));
    int yy = y[b] != 0;
    acc += lse - (yy ? z1 : z0);
    stf(dz + 2 * b, (__expf(z0 - lse) - (yy ? 0.f : 1.f)) * inv);
    stf(dz + 2 * b + 1, (__expf(z1 - lse) - (yy ? 1.f : 0.f)) * inv);
  }
  sh[threadIdx.x] = acc;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss += sh[0] * inv;
}
// dxm[inv[b*S], :] += dxc[b, :]: the classifier's gradient joins the compacted rows of the last layer's output
template <typename AT>
__global__ void k_add_first_token_rows(const AT* __restrict__ dxc, const int32_t* __restrict__ inv, int S, int H,
                                       AT* __restrict__ dxm) {
  int b = blockIdx.x;
  int j = inv[(size_t)b * S];
  if (j < 0) return;
  for (int c = threadIdx.x; c < H; c += blockDim.x) {
    AT* d = dxm + (size_t)j * H + c;
    stf(d, ldf(d) + ldf(dxc + (size_t)b * H + c));
  }
}
#define MSLT_BY_DTYPE(CALL_F, CALL_B) do { if (dtype == 0) { CALL_F; } else { CALL_B; } } while (0)
hipError_t gather_first_tokens(int dtype, const void* x, int S, int H, int n_seq, void* out, hipStream_t s) {
  MSLT_BY_DTYPE((k_gather_first_tokens<float><<<dim3(n_seq), dim3(256), 0, s>>>((const float*)x, S, H, (float*)out)),
                (k_gather_first_tokens<bf16><<<dim3(n_seq), dim3(256), 0, s>>>((const bf16*)x, S, H, (bf16*)out)));
  return hipGetLastError();
}
hipError_t tanh_inplace(int dtype, void* u, size_t n, hipStream_t s) {
  dim3 grid((unsigned)((n + 255) / 256));
  MSLT_BY_DTYPE((k_tanh_inplace<float><<<grid, dim3(256), 0, s>>>((float*)u, n)),
                (k_tanh_inplace<bf16><<<grid, dim3(256), 0, s>>>((bf16*)u, n)));
  return hipGetLastError();
}
hipError_t tanh_bwd(int dtype, const void* dp, const void* p, void* du, size_t n, hipStream_t s) {
  dim3 grid((unsigned)((n + 255) / 256));
  MSLT_BY_DTYPE((k_tanh_bwd<float><<<grid, dim3(256), 0, s>>>((const float*)dp, (const float*)p, (float*)du, n)),
                (k_tanh_bwd<bf16><<<grid, dim3(256), 0, s>>>((const bf16*)dp, (const bf16*)p, (bf16*)du, n)));
  return hipGetLastError();
}
hipError_t nsp_ce(int dtype, const float* z, const int32_t* y, int n_seq, void* dz, float* loss, hipStream_t s) {
  MSLT_BY_DTYPE((k_nsp_ce<float><<<dim3(1), dim3(256), 0, s>>>(z, y, n_seq, (float*)dz, loss)),
                (k_nsp_ce<bf16><<<dim3(1), dim3(256), 0, s>>>(z, y, n_seq, (bf16*)dz, loss)));
  return hipGetLastError();
}
hipError_t add_first_token_rows(int dtype, const void* dxc, const int32_t* inv, int S, int H, int n_seq, void* dxm,
                                hipStream_t s) {
  MSLT_BY_DTYPE((k_add_first_token_rows<float><<<dim3(n_seq), dim3(256), 0, s>>>((const float*)dxc, inv, S, H, (float*)dxm)),
                (k_add_first_token_rows<bf16><<<dim3(n_seq), dim3(256), 0, s>>>((const bf16*)dxc, inv, S, H, (bf16*)dxm)));
  return hipGetLastError();
}
#undef MSLT_BY_DTYPE

}  // namespace mslt
