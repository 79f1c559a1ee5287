// bf16 MFMA GEMM for gfx950: C(m,n) = sum_k A(m,k) B(n,k), fp32 accumulation, shared epilogue.
//
// A workgroup of BM/64 x 2 wavefronts computes a BM x 128 tile of C (BM = 256: eight wavefronts,
// BM = 128: four); each wavefront owns a 64x64 quarter as 2x2 blocks of
// v_mfma_f32_32x32x16_bf16.  The k loop advances 64 at a time through two LDS stages: while the
// matrix cores work on stage s, later operand slabs travel global -> registers -> LDS stage s^1,
// two k tiles ahead, and the memory instructions of a tile are spread between the MFMAs of its
// four 16-wide steps.  Both operands sit in LDS as [rows][64 k] bf16 with the 16-byte chunks of
// a row XOR-swizzled by the row index, so the 16-byte fragment reads of the MFMA layout (lane =
// row, 8 consecutive k) are free of bank conflicts without padding.  An operand whose k index is
// the strided one in memory (the weight in dX = dY.W, both operands in dW = dY^T.X) is transposed
// in registers on its way into LDS, so every product of the training step runs through this one
// kernel and no transposed copy of an activation or weight ever goes to HBM.  The 256-row tile
// moves 25 % fewer bytes through the vector L1 per FLOP than the 128-row one (the L1 -> LDS path
// is as scarce as the matrix cores at 128x128) and is used for long contractions with enough
// tiles.  The epilogue stages each wavefront's quarter in LDS and writes 16-byte rows: bias, GELU
// (which also stores GELU' for the backward pass), multiply by that stored derivative, or residual
// add are fused there.  With split-k the tile's
// partial sums go to an fp32 workspace and a second kernel adds the splits in a fixed order
// (deterministic, no atomics).
#include "common.h"
#include "gemm_epilogue.h"
#include <type_traits>

namespace mslt {

constexpr int BN = 128, BK = 64;
constexpr int PF = 2;                                  // prefetch distance in k tiles
constexpr int lds_bytes(int BM) {
  int main_bytes = 2 * (BM + BN) * BK * 2;             // two stages of both operands
  int epi_bytes = (BM / 64) * 2 * 64 * EPI_LD * 4;     // one 64 x EPI_LD fp32 quarter per wavefront
  return epi_bytes > main_bytes ? epi_bytes : main_bytes;
}

// 16-byte chunk swizzle of a 128-byte LDS row
__device__ __forceinline__ int swz(int row) { return ((row >> 1) & 7) ^ ((row >> 4) & 7); }

struct MfmaParams {
  const bf16* A;
  const bf16* B;
  int M, N, K;       // K = contraction length of this launch (all splits together)
  int lda, ldb;
  int splitk;
  int tiles_m, tiles_n;
  float* partials;   // [splitk][M][N] when splitk > 1
  Epilogue epi;
};

// ---- global -> register -> LDS slabs --------------------------------------------------------
// Up to four 16-byte registers per thread and operand.  Named members of native vector type (not
// an array, not a struct vector) so that the compiler keeps them in VGPRs across the MFMA block.
struct Slab {
  u32x4_t v0, v1, v2, v3;
};
__device__ __forceinline__ u32x4_t& slab_reg(Slab& s, int i) { return i == 0 ? s.v0 : i == 1 ? s.v1 : i == 2 ? s.v2 : s.v3; }
__device__ __forceinline__ const u32x4_t& slab_reg(const Slab& s, int i) {
  return i == 0 ? s.v0 : i == 1 ? s.v1 : i == 2 ? s.v2 : s.v3;
}
__device__ __forceinline__ uint32_t word_of(const u32x4_t& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }

// An operand slab is ROWS x 64 k, moved by NT threads, LPT = ROWS*8/NT 16-byte loads per thread.
//   k-contiguous operand [rows][ld]: load i of thread t is chunk t%8 of row t/8 + (NT/8)*i.
//   k-strided operand [k][ld]: thread t takes 8 rows (16 bytes) 8*(t % (ROWS/8)) of the LPT
//   consecutive k starting at LPT*(t / (ROWS/8)); load i is k number i of those.
template <bool KC, int ROWS, int NT, int I>
__device__ __forceinline__ void load_one(const bf16* __restrict__ base, int ld, int row0, int k0, int tid, Slab& s) {
  constexpr int LPT = ROWS * 8 / NT, RG = ROWS / 8;
  static_assert(I < LPT, "load index");
  if constexpr (KC)
    slab_reg(s, I) = *reinterpret_cast<const u32x4_t*>(base + (size_t)(row0 + (tid >> 3) + (NT / 8) * I) * ld + k0 + 8 * (tid & 7));
  else
    slab_reg(s, I) = *reinterpret_cast<const u32x4_t*>(base + (size_t)(k0 + LPT * (tid / RG) + I) * ld + row0 + 8 * (tid % RG));
}
template <bool KC, int ROWS, int NT>
__device__ __forceinline__ void load_slab(const bf16* __restrict__ base, int ld, int row0, int k0, int tid, Slab& s) {
  constexpr int LPT = ROWS * 8 / NT;
  load_one<KC, ROWS, NT, 0>(base, ld, row0, k0, tid, s);
  load_one<KC, ROWS, NT, 1>(base, ld, row0, k0, tid, s);
  if constexpr (LPT == 4) {
    load_one<KC, ROWS, NT, 2>(base, ld, row0, k0, tid, s);
    load_one<KC, ROWS, NT, 3>(base, ld, row0, k0, tid, s);
  }
}
// Quarter Q (0..3) of the slab's loads / LDS stores, so that the memory instructions of a k tile
// can be spread between the MFMAs of the four 16-wide steps.
template <bool KC, int ROWS, int NT, int Q>
__device__ __forceinline__ void load_part(const bf16* __restrict__ base, int ld, int row0, int k0, int tid, Slab& s) {
  constexpr int LPT = ROWS * 8 / NT;
  if constexpr (LPT == 4) load_one<KC, ROWS, NT, Q>(base, ld, row0, k0, tid, s);
  if constexpr (LPT == 2 && (Q & 1) == 0) load_one<KC, ROWS, NT, Q / 2>(base, ld, row0, k0, tid, s);
}
template <bool KC, int ROWS, int NT, int Q>
__device__ __forceinline__ void store_part(bf16* __restrict__ lds, int tid, const Slab& s) {
  constexpr int LPT = ROWS * 8 / NT, RG = ROWS / 8;
  if constexpr (KC) {
    if constexpr (LPT == 4 || (Q & 1) == 1) {
      constexpr int I = LPT == 4 ? Q : Q / 2;
      int c = tid & 7, r = (tid >> 3) + (NT / 8) * I;
      *reinterpret_cast<u32x4_t*>(lds + r * BK + 8 * (c ^ swz(r))) = slab_reg(s, I);
    }
  } else {
    // rows 8cg+2Q and 8cg+2Q+1 get their LPT k values: low / high halves of word Q of the loads
    int cg = tid % RG, kg = tid / RG, r = 8 * cg + 2 * Q;
    uint32_t a = word_of(s.v0, Q), b = word_of(s.v1, Q);
    if constexpr (LPT == 4) {
      uint32_t c = word_of(s.v2, Q), d = word_of(s.v3, Q);
      u32x2_t lo, hi;
      lo.x = __builtin_amdgcn_perm(b, a, 0x05040100u); lo.y = __builtin_amdgcn_perm(d, c, 0x05040100u);
      hi.x = __builtin_amdgcn_perm(b, a, 0x07060302u); hi.y = __builtin_amdgcn_perm(d, c, 0x07060302u);
      *reinterpret_cast<u32x2_t*>(lds + r * BK + 8 * ((kg >> 1) ^ swz(r)) + 4 * (kg & 1)) = lo;
      *reinterpret_cast<u32x2_t*>(lds + (r + 1) * BK + 8 * ((kg >> 1) ^ swz(r + 1)) + 4 * (kg & 1)) = hi;
    } else {
      uint32_t lo = __builtin_amdgcn_perm(b, a, 0x05040100u), hi = __builtin_amdgcn_perm(b, a, 0x07060302u);
      *reinterpret_cast<uint32_t*>(lds + r * BK + 8 * ((kg >> 2) ^ swz(r)) + 2 * (kg & 3)) = lo;
      *reinterpret_cast<uint32_t*>(lds + (r + 1) * BK + 8 * ((kg >> 2) ^ swz(r + 1)) + 2 * (kg & 3)) = hi;
    }
  }
}
template <bool KC, int ROWS, int NT>
__device__ __forceinline__ void store_slab(bf16* __restrict__ lds, int tid, const Slab& s) {
  store_part<KC, ROWS, NT, 0>(lds, tid, s);
  store_part<KC, ROWS, NT, 1>(lds, tid, s);
  store_part<KC, ROWS, NT, 2>(lds, tid, s);
  store_part<KC, ROWS, NT, 3>(lds, tid, s);
}

// Direct global -> LDS load of quarter Q of a k-contiguous slab (no register staging): lane i of
// a wavefront lands at its LDS base + 16*i bytes, i.e. eight whole 128-byte rows per instruction,
// so each lane fetches the global chunk that belongs at its (row, swizzled chunk) position.
template <int ROWS, int NT, int Q>
__device__ __forceinline__ void dma_part(const bf16* __restrict__ base, int ld, int row0, int k0, int tid, bf16* lds) {
  constexpr int LPT = ROWS * 8 / NT;
  if constexpr (LPT == 4 || (Q & 1) == 0) {
    constexpr int I = LPT == 4 ? Q : Q / 2;
    const int row = (tid >> 3) + (NT / 8) * I;
    const int c = (tid & 7) ^ swz(row);
    const bf16* src = base + (size_t)(row0 + row) * ld + k0 + 8 * c;
    const int wave_row0 = __builtin_amdgcn_readfirstlane((tid >> 6) * 8 + (NT / 8) * I);
    __builtin_amdgcn_global_load_lds((global_void_t*)src, (lds_void_t*)(lds + wave_row0 * BK), 16, 0, 0);
  }
}
template <int ROWS, int NT>
__device__ __forceinline__ void dma_slab(const bf16* __restrict__ base, int ld, int row0, int k0, int tid, bf16* lds) {
  dma_part<ROWS, NT, 0>(base, ld, row0, k0, tid, lds);
  dma_part<ROWS, NT, 1>(base, ld, row0, k0, tid, lds);
  dma_part<ROWS, NT, 2>(base, ld, row0, k0, tid, lds);
  dma_part<ROWS, NT, 3>(base, ld, row0, k0, tid, lds);
}

__device__ __forceinline__ bf16x8_t lds_frag(const bf16* __restrict__ lds, int row, int chunk) {
  return *reinterpret_cast<const bf16x8_t*>(lds + row * BK + 8 * (chunk ^ swz(row)));
}

// ---- the kernel -----------------------------------------------------------------------------
// Operand modes: how an operand slab gets from global memory into LDS.
enum { OP_STRIDED = 0, OP_KC = 1, OP_KC_DMA = 2 };

template <int BM, int AMODE, int BMODE>
__global__ void __launch_bounds__(2 * BM) k_gemm_mfma(MfmaParams p) {
  constexpr bool A_KC = AMODE != OP_STRIDED, B_KC = BMODE != OP_STRIDED;
  constexpr bool A_DMA = AMODE == OP_KC_DMA, B_DMA = BMODE == OP_KC_DMA;
  constexpr int NT = 2 * BM;                       // threads: BM/64 x 2 wavefronts
  constexpr int STAGE_ELEMS = (BM + BN) * BK;      // bf16 elements per pipeline stage
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* lds = reinterpret_cast<bf16*>(smem);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  // workgroup -> (split, tile): consecutive ids go round-robin to the 8 XCDs, so give each XCD a
  // contiguous range of tiles (row-major over the tile grid) to keep its L2 working set small
  const int total = p.tiles_m * p.tiles_n * p.splitk;
  int pid = blockIdx.x;
  {
    int per = (total + 7) >> 3, tall = total & 7;
    if (tall == 0) tall = 8;
    int xcd = pid & 7, local = pid >> 3;
    pid = xcd < tall ? xcd * per + local : tall * per + (xcd - tall) * (per - 1) + local;
  }
  const int tiles = p.tiles_m * p.tiles_n;
  const int split = pid / tiles;
  const int tile = pid - split * tiles;
  // Consecutive tiles run at the same time on one XCD and share its L2: order them in bands of
  // GROUP_M tile rows, column by column inside a band, so that the concurrent set is a block of
  // about GROUP_M x 64/GROUP_M tiles (few distinct operand panels) instead of one long tile row.
#ifndef MSLT_GROUP_M
#define MSLT_GROUP_M 8
#endif
  int tm, tn;
  {
    constexpr int G = MSLT_GROUP_M;
    const int band = tile / (G * p.tiles_n);
    const int first = band * G;
    const int rows = p.tiles_m - first < G ? p.tiles_m - first : G;
    const int in_band = tile - band * G * p.tiles_n;
    tm = first + in_band % rows;
    tn = in_band / rows;
  }
  const int m0 = tm * BM, n0 = tn * BN;
  // split s takes k tiles [s*nkt/splitk, (s+1)*nkt/splitk): sizes differ by at most one tile
  const int nkt = p.K / BK;
  const int kt_lo = (int)((long long)split * nkt / p.splitk);
  const int kbeg = kt_lo * BK;
  const int nk = (int)((long long)(split + 1) * nkt / p.splitk) - kt_lo;

  f32x16_t acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Software pipeline: PF register sets hold the slabs of tiles kt+1 .. kt+PF while tile kt is
  // multiplied out of LDS.  Tile t lives in set t % PF; the loop is unrolled by PF so that every
  // set has a static name, and its body is branch-free (tile indices past the end are clamped: the
  // duplicate loads and the last LDS store are never consumed), which lets the compiler keep the
  // loads of later tiles in flight across iterations instead of draining them at every join.
  // An operand in OP_KC_DMA mode skips the registers: the slab of tile kt+1 is loaded straight into
  // LDS stage (kt+1)&1 during iteration kt and awaited (vmcnt) before the closing barrier.
  Slab ra[PF], rb[PF];
#pragma unroll
  for (int j = 0; j < PF; ++j) {
    int t = j < nk ? j : nk - 1;
    if constexpr (!A_DMA) load_slab<A_KC, BM, NT>(p.A, p.lda, m0, kbeg + t * BK, tid, ra[j]);
    if constexpr (!B_DMA) load_slab<B_KC, BN, NT>(p.B, p.ldb, n0, kbeg + t * BK, tid, rb[j]);
  }
  if constexpr (A_DMA) dma_slab<BM, NT>(p.A, p.lda, m0, kbeg, tid, lds);
  else store_slab<A_KC, BM, NT>(lds, tid, ra[0]);
  if constexpr (B_DMA) dma_slab<BN, NT>(p.B, p.ldb, n0, kbeg, tid, lds + BM * BK);
  else store_slab<B_KC, BN, NT>(lds + BM * BK, tid, rb[0]);
  if constexpr (A_DMA || B_DMA) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  __syncthreads();

  const int arow = 64 * wm + (lane & 31), brow = 64 * wn + (lane & 31), half = lane >> 5;
  auto body = [&](Slab& la, Slab& lb, const Slab& na, const Slab& nb, int kt) {
    // la/lb: set of tile kt (free: refilled with tile kt+PF); na/nb: set of tile kt+1 (goes to LDS).
    // The four 16-wide steps each carry a quarter of the global loads and of the LDS stores and
    // prefetch the fragments of the next step, so that memory instructions issue in the shadow of
    // the MFMAs instead of in separate phases; sched_barrier keeps the steps apart.
    const bf16* sa = lds + (kt & 1) * STAGE_ELEMS;
    const bf16* sb = sa + BM * BK;
    bf16* da = lds + ((kt + 1) & 1) * STAGE_ELEMS;
    bf16* db = da + BM * BK;
    const int tn2 = kt + PF < nk ? kt + PF : nk - 1;
    const int kn = kbeg + tn2 * BK;                                  // register prefetch: tile kt+PF
    const int kd = kbeg + (kt + 1 < nk ? kt + 1 : nk - 1) * BK;      // direct loads: tile kt+1
    bf16x8_t fa[2][2], fb[2][2];
    fa[0][0] = lds_frag(sa, arow, half);
    fa[0][1] = lds_frag(sa, arow + 32, half);
    fb[0][0] = lds_frag(sb, brow, half);
    fb[0][1] = lds_frag(sb, brow + 32, half);
#define MSLT_GEMM_STEP(KS)                                                                          \
    {                                                                                               \
      constexpr int cur = (KS) & 1, nxt = cur ^ 1;                                                  \
      if constexpr ((KS) < 3) {                                                                     \
        fa[nxt][0] = lds_frag(sa, arow, 2 * ((KS) + 1) + half);                                     \
        fa[nxt][1] = lds_frag(sa, arow + 32, 2 * ((KS) + 1) + half);                                \
        fb[nxt][0] = lds_frag(sb, brow, 2 * ((KS) + 1) + half);                                     \
        fb[nxt][1] = lds_frag(sb, brow + 32, 2 * ((KS) + 1) + half);                                \
      }                                                                                             \
      if constexpr (A_DMA) dma_part<BM, NT, (KS)>(p.A, p.lda, m0, kd, tid, da);                     \
      else load_part<A_KC, BM, NT, (KS)>(p.A, p.lda, m0, kn, tid, la);                              \
      if constexpr (B_DMA) dma_part<BN, NT, (KS)>(p.B, p.ldb, n0, kd, tid, db);                     \
      else load_part<B_KC, BN, NT, (KS)>(p.B, p.ldb, n0, kn, tid, lb);                              \
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][0], fb[cur][0], acc[0][0], 0, 0, 0); \
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][0], fb[cur][1], acc[0][1], 0, 0, 0); \
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][1], fb[cur][0], acc[1][0], 0, 0, 0); \
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[cur][1], fb[cur][1], acc[1][1], 0, 0, 0); \
      if constexpr (!A_DMA) store_part<A_KC, BM, NT, (KS)>(da, tid, na);                            \
      if constexpr (!B_DMA) store_part<B_KC, BN, NT, (KS)>(db, tid, nb);                            \
      __builtin_amdgcn_sched_barrier(0);                                                            \
    }
    MSLT_GEMM_STEP(0)
    MSLT_GEMM_STEP(1)
    MSLT_GEMM_STEP(2)
    MSLT_GEMM_STEP(3)
#undef MSLT_GEMM_STEP
    if constexpr (A_DMA || B_DMA) __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): direct loads landed
    __syncthreads();
  };
  int kt = 0;
  for (; kt + PF <= nk; kt += PF) {
#pragma unroll
    for (int j = 0; j < PF; ++j) body(ra[j], rb[j], ra[(j + 1) % PF], rb[(j + 1) % PF], kt + j);
  }
#pragma unroll
  for (int j = 0; j < PF - 1; ++j)
    if (kt + j < nk) body(ra[j], rb[j], ra[(j + 1) % PF], rb[(j + 1) % PF], kt + j);

  // Epilogue operands first: the bias and the per-element operand are requested before the
  // accumulators are staged, so their memory latency runs under the staging and its barrier.
  const int cc = 8 * (lane & 7);
  const int n = n0 + 64 * wn + cc;
  const int mrow = m0 + 64 * wm + (lane >> 3);      // first of this lane's 8 rows (stride 8)
  Epilogue e = p.epi;
  float bias[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) bias[i] = 0.f;
  uint4 raw[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) raw[i] = make_uint4(0, 0, 0, 0);
  if (p.splitk > 1) {
    e = Epilogue();
    e.out = p.partials + (size_t)split * p.M * p.N;
    e.ldo = p.N;
    e.out_f32 = 1;
  } else {
    if (epilogue_reads_aux(e)) {
#pragma unroll
      for (int i = 0; i < 8; ++i) raw[i] = load_aux8(e, mrow + 8 * i, n);
    }
    if (e.bias) {
      float4 b0 = *reinterpret_cast<const float4*>(e.bias + n), b1 = *reinterpret_cast<const float4*>(e.bias + n + 4);
      bias[0] = b0.x; bias[1] = b0.y; bias[2] = b0.z; bias[3] = b0.w;
      bias[4] = b1.x; bias[5] = b1.y; bias[6] = b1.z; bias[7] = b1.w;
    }
  }

  // stage this wavefront's 64x64 quarter in LDS (all operand reads are behind the last barrier)
  float* stage = reinterpret_cast<float*>(smem) + wave * 64 * EPI_LD;
#pragma unroll
  for (int bi = 0; bi < 2; ++bi)
#pragma unroll
    for (int bj = 0; bj < 2; ++bj)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int row = 32 * bi + 8 * (r >> 2) + 4 * half + (r & 3);
        stage[row * EPI_LD + 32 * bj + (lane & 31)] = acc[bi][bj][r];
      }
  __syncthreads();

  auto finish = [&](auto extras) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      int row = 8 * i + (lane >> 3);
      float4 x0 = *reinterpret_cast<const float4*>(stage + row * EPI_LD + cc);
      float4 x1 = *reinterpret_cast<const float4*>(stage + row * EPI_LD + cc + 4);
      float v[8] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w};
      epilogue8<decltype(extras)::value>(e, mrow + 8 * i, n, v, bias, raw[i]);
    }
  };
  if (e.drop.thr || e.accumulate) finish(std::true_type());
  else finish(std::false_type());
}

// sums the split-k partials in split order and applies the epilogue; 8 columns per thread
__global__ void __launch_bounds__(256) k_splitk_reduce(const float* __restrict__ partials, int splitk, int M, int N,
                                                       Epilogue e) {
  size_t idx = ((size_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (idx >= (size_t)M * N) return;
  int m = (int)(idx / N), n = (int)(idx % N);
  uint4 raw = make_uint4(0, 0, 0, 0);
  if (epilogue_reads_aux(e)) raw = load_aux8(e, m, n);
  float v[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  for (int s = 0; s < splitk; ++s) {
    const float* q = partials + (size_t)s * M * N + idx;
    float4 a = *reinterpret_cast<const float4*>(q), b = *reinterpret_cast<const float4*>(q + 4);
    v[0] += a.x; v[1] += a.y; v[2] += a.z; v[3] += a.w;
    v[4] += b.x; v[5] += b.y; v[6] += b.z; v[7] += b.w;
  }
  float bias[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (e.bias) {
#pragma unroll
    for (int i = 0; i < 8; ++i) bias[i] = e.bias[n + i];
  }
  if (e.drop.thr || e.accumulate) epilogue8<true>(e, m, n, v, bias, raw);
  else epilogue8<false>(e, m, n, v, bias, raw);
}

bool gemm_mfma_supported(const GemmDesc& d) {
  if (d.M <= 0 || d.N <= 0 || d.K <= 0) return false;
  if (d.M % 128 || d.N % BN || d.K % BK) return false;
  if (d.lda % 8 || d.ldb % 8 || d.epi.ldo % 8) return false;
  if ((d.epi.act == EPI_MUL || d.epi.act == EPI_ADD) && d.epi.ldaux % 8) return false;
  if (d.epi.drop.thr && d.epi.drop_ld % 4) return false;
  if (d.epi.accumulate && !d.epi.out_f32) return false;
  auto al = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
  if (!al(d.A) || !al(d.B) || !al(d.epi.out) || !al(d.epi.out2) || !al(d.epi.aux) || !al(d.epi.bias)) return false;
  return true;
}

// The tall tile pays off for long contractions with at least one full wave of tall tiles (measured:
// 8192^3 runs at 1054 vs 852 TFLOP/s), and, inside the training step, for the products with a narrow
// output (N <= 1024: output projection, second feed-forward layer and the data gradients that end in
// the hidden size): there a 128-row tiling leaves the last round of workgroups partly empty, and with
// a second kernel chain running beside it fewer, larger workgroups finish sooner.  Measured in the
// step (same box, alternating), this rule against 128-row tiles everywhere: 3 % of the step at
// hidden 768, 1.5 % at hidden 1024; NN products gain only at hidden 1024 and lose 1 % at 768, where
// two resident 128-row workgroups per CU overlap their prologues and epilogues better.  Wide outputs
// stay at 128 rows (the tall tile costs 3.5 % of the step there).
int gemm_mfma_tile_m(const GemmDesc& d) {
  if (d.M % 256) return 128;
  if (d.K >= 4096 && (d.M / 256) * (d.N / BN) >= 256) return 256;
  if (d.a_kcontig && d.M >= 2048 && d.N <= 1024 && (d.b_kcontig || d.N == 1024)) return 256;
  return 128;
}

template <int BM, int AMODE, int BMODE>
static hipError_t launch_mode(const MfmaParams& p, dim3 grid, hipStream_t s) {
  constexpr int LDS = lds_bytes(BM);
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_mfma<BM, AMODE, BMODE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  k_gemm_mfma<BM, AMODE, BMODE><<<grid, dim3(2 * BM), LDS, s>>>(p);
  return hipGetLastError();
}
// k-contiguous operands go global -> LDS directly (use_dma) or through registers
template <int BM>
static hipError_t launch(const GemmDesc& d, const MfmaParams& p, dim3 grid, hipStream_t s, bool use_dma) {
  if (d.a_kcontig && d.b_kcontig)
    return use_dma ? launch_mode<BM, OP_KC_DMA, OP_KC_DMA>(p, grid, s) : launch_mode<BM, OP_KC, OP_KC>(p, grid, s);
  if (d.a_kcontig && !d.b_kcontig)
    return use_dma ? launch_mode<BM, OP_KC_DMA, OP_STRIDED>(p, grid, s) : launch_mode<BM, OP_KC, OP_STRIDED>(p, grid, s);
  if (!d.a_kcontig && d.b_kcontig)
    return use_dma ? launch_mode<BM, OP_STRIDED, OP_KC_DMA>(p, grid, s) : launch_mode<BM, OP_STRIDED, OP_KC>(p, grid, s);
  return launch_mode<BM, OP_STRIDED, OP_STRIDED>(p, grid, s);
}

hipError_t gemm_mfma(const GemmDesc& d, int splitk, float* partials, hipStream_t s, int force_tile_m, int force_dma) {
  if (!gemm_mfma_supported(d)) return hipErrorInvalidValue;
  if (splitk < 1 || splitk > d.K / BK) return hipErrorInvalidValue;
  if (splitk > 1 && partials == nullptr) return hipErrorInvalidValue;
  const int bm = force_tile_m ? force_tile_m : gemm_mfma_tile_m(d);
  if ((bm != 128 && bm != 256) || d.M % bm) return hipErrorInvalidValue;
  MfmaParams p;
  p.A = reinterpret_cast<const bf16*>(d.A);
  p.B = reinterpret_cast<const bf16*>(d.B);
  p.M = d.M; p.N = d.N; p.K = d.K;
  p.lda = d.lda; p.ldb = d.ldb;
  p.splitk = splitk;
  p.tiles_m = d.M / bm; p.tiles_n = d.N / BN;
  p.partials = partials;
  p.epi = d.epi;
  dim3 grid((unsigned)(p.tiles_m * p.tiles_n * splitk));
  // Direct global -> LDS loads hide only one iteration of latency (two LDS stages); measured, they win
  // for NT products whose tiles fit in one round of resident workgroups and lose otherwise.
  const bool dma_default = d.a_kcontig && d.b_kcontig && bm == 128 && p.tiles_m * p.tiles_n * splitk <= 512;
  const bool use_dma = force_dma >= 0 ? force_dma != 0 : dma_default;
  hipError_t e = bm == 256 ? launch<256>(d, p, grid, s, use_dma) : launch<128>(d, p, grid, s, use_dma);
  if (e != hipSuccess || splitk == 1) return e;
  size_t n8 = (size_t)d.M * d.N / 8;
  k_splitk_reduce<<<dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, s>>>(partials, splitk, d.M, d.N, d.epi);
  return hipGetLastError();
}

}  // namespace mslt
