// Large-tile bf16 MFMA GEMM for gfx950: C(m,n) = sum_k A(m,k) B(n,k), fp32 accumulation, shared
// epilogue.  Made for the products of the training step that have enough output tiles: the
// operand feed (global memory -> vector L1 -> LDS) is what bounds a 128x128 tile, and a 256x256
// tile moves half the bytes per MFMA.
//
// A workgroup of eight wavefronts owns a TM x TN tile (256x256: 2x4 wavefronts of 128x64;
// 256x128 and 128x256: 64x64 per wavefront).  Both operands travel global memory -> LDS
// directly (buffer loads with the LDS bit, 16 bytes per lane, no register staging) through a
// ring of NS stages of 32 k each, NS-1 tiles ahead of the matrix cores; one workgroup barrier
// per 32 k.  An operand whose k index is contiguous in memory sits in LDS as [rows][32 k] with
// the four 16-byte chunks of a row XOR-swizzled by the row index, and its MFMA fragments are
// plain 16-byte reads.  An operand whose k index is the strided one (the weight in dX = dY.W,
// both operands in dW = dY^T.X) is copied as it lies, [32 k][rows], with the 16-byte chunks of a
// k row XOR-swizzled by k, and its fragments come from the transposing LDS read
// (ds_read_b64_tr_b16: sixteen lanes that each fetch four consecutive rows of one k receive four
// consecutive k of one row), so no operand is ever transposed in registers or in HBM.
// The loads of a lane differ from one k tile to the next only in a scalar offset, so the k loop
// carries no address arithmetic in vector registers.
#include "common.h"
#include "gemm_epilogue.h"
#include <type_traits>

namespace mslt {

namespace ring {

typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(8))) short s16x8_t;

struct Params {
  const bf16* A;
  const bf16* B;
  int M, N, K;       // K = contraction length of this launch (all splits together)
  int lda, ldb;
  int splitk;
  int tiles_m, tiles_n;
  float* partials;   // [splitk][M][N] when splitk > 1
  Epilogue epi;
};

// ---- operand movers ---------------------------------------------------------------------------
// One buffer load moves 64 lanes x 16 bytes into 1024 consecutive LDS bytes (lane i lands at
// base + 16 i); which global chunk a lane fetches is free, which is where the swizzles live.
// RK is the k extent of a ring stage: 64 for a k-contiguous operand makes every row segment a whole
// 128-byte cache line (eight adjacent lanes), which halves the number of L2 requests against 32.
//
// k-contiguous operand, stage layout [ROWS][RK k]:
//   RK = 32 (64-byte rows): instruction q covers rows 16q .. 16q+15; lane -> row 16q + lane/4, slot
//   lane%4, which holds k chunk slot ^ ((row>>2)&3).
//   RK = 64 (128-byte rows): instruction q covers rows 8q .. 8q+7; lane -> row 8q + lane/8, slot
//   lane%8, which holds k chunk slot ^ ((row>>1)&7).
// k-strided operand, stage layout [RK k][ROWS]: a k row is ROWS/8 chunks; chunk c of k row k sits in
// slot c ^ ((k&3)<<2).  ROWS = 256: instruction q covers k rows 2q, 2q+1; ROWS = 128: 4q .. 4q+3.
template <bool KC, int ROWS, int RK, int NWAVES>
struct Mover {
  static constexpr int INSTR = ROWS * RK * 2 / 1024;       // per stage
  static constexpr int IPW = INSTR / NWAVES;               // per wavefront
  static constexpr int KPI = 1024 / (ROWS * 2);            // k rows per instruction (k-strided)
  static constexpr int RPI = 1024 / (RK * 2);              // rows per instruction (k-contiguous)
  static_assert(IPW >= 1 && IPW <= 8, "rows per tile");
  int voff[2];     // per-lane byte offset of even / odd instructions (relative to the tile's first row, k = 0)
  __device__ __forceinline__ void init(int lane, int ld) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      if constexpr (KC && RK == 32) {
        voff[j] = ((lane >> 2) * ld + 8 * ((lane & 3) ^ ((lane >> 4) & 3))) * 2;
      } else if constexpr (KC) {
        // row = 8q + lane/8 with q = IPW*wave + j', IPW even or q parity = j' parity: (row>>1)&7 = (4(q&1) + lane/16)&7
        voff[j] = ((lane >> 3) * ld + 8 * ((lane & 7) ^ ((4 * j + (lane >> 4)) & 7))) * 2;
      } else if constexpr (ROWS == 256) {
        const int kk = lane >> 5, slot = lane & 31;     // k = 2q + kk, k&3 = (2(q&1) + kk)&3
        voff[j] = kk * ld * 2 + ((slot ^ (((2 * j + kk) & 3) << 2)) << 4);
      } else {
        const int kk = lane >> 4, slot = lane & 15;     // k = 4q + kk, k&3 = kk
        voff[j] = kk * ld * 2 + ((slot ^ (kk << 2)) << 4);
      }
    }
  }
  // queues the loads of the tile at contraction offset k0 (elements) into the stage at `lds`
  __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rsrc, int ld, int k0, int wave, bf16* lds) const {
    static_assert(IPW == 1 || IPW % 2 == 0, "instruction parity follows j");
#pragma unroll
    for (int j = 0; j < IPW; ++j) {
      const int q = wave * IPW + j;
      int soff;
      if constexpr (KC) soff = (q * RPI * ld + k0) * 2;
      else soff = (k0 + q * KPI) * ld * 2;
      // with one instruction per wavefront its parity is the wavefront's
      const int par = IPW == 1 ? (wave & 1) : (j & 1);
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_t*)(lds + q * 512), 16, voff[par], soff, 0, 0);
    }
  }
};

// ---- MFMA fragments ----------------------------------------------------------------------------
// Fragment of v_mfma_f32_32x32x16_bf16: lane l holds row l%32, k = 8*(l/32) .. +7 of a 32 x 16 block.
// The transposing read is written as inline assembly: through the builtin the compiler cannot tell it
// from an access that aliases the loads into LDS still in flight and waits for all of them before
// every read, which would undo the ring.  Its completion is awaited by hand (lgkmcnt) before the
// MFMAs that consume it.
template <bool KC, int ROWS, int NBLK, int RK>
struct Frags {
  static constexpr int STEPS = RK / 16;
  static constexpr int OPS = KC ? NBLK : 2 * NBLK;          // LDS instructions per 16-wide step
  int off[KC ? STEPS : NBLK];   // KC: element offsets inside a stage; k-strided: byte offsets
  // row_base: first row of this wavefront's part of the tile
  __device__ __forceinline__ void init(int lane, int row_base) {
    if constexpr (KC) {
      const int row = row_base + (lane & 31), half = lane >> 5;
      const int sw = RK == 32 ? (lane >> 2) & 3 : (lane >> 1) & 7;    // row_base % 32 == 0
#pragma unroll
      for (int s = 0; s < STEPS; ++s) off[s] = row * RK + 8 * ((2 * s + half) ^ sw);
    } else {
      const int blk = lane >> 4, j = lane & 15;
#pragma unroll
      for (int i = 0; i < NBLK; ++i) {
        const int e = row_base + 32 * i + 16 * (blk & 1) + 4 * (j & 3);      // first of this lane's four rows
        off[i] = 2 * ((8 * (blk >> 1) + (j >> 2)) * ROWS + ((((e >> 3) ^ ((j >> 2) << 2))) << 3) + (e & 7));
      }
    }
  }
  // block i (32 rows), 16-wide k step s of the stage at `st`; stage_bytes: LDS byte address of the stage
  __device__ __forceinline__ bf16x8_t get(const bf16* st, unsigned stage_bytes, int i, int s) const {
    if constexpr (KC) {
      return *reinterpret_cast<const bf16x8_t*>(st + off[s] + i * 32 * RK);
    } else {
      s16x8_t v;
      const unsigned addr = stage_bytes + (unsigned)off[i] + (unsigned)(32 * s * ROWS);
      // early-clobber outputs: the data of the first read may arrive before the second read has taken its address
      asm volatile("ds_read_b64_tr_b16 %0, %2\n\tds_read_b64_tr_b16 %1, %2 offset:%3"
                   : "=&v"(reinterpret_cast<s16x4_t*>(&v)[0]), "=&v"(reinterpret_cast<s16x4_t*>(&v)[1])
                   : "v"(addr), "n"(8 * ROWS));
      return __builtin_bit_cast(bf16x8_t, v);
    }
  }
};

constexpr int n_waves(int TM, int TN) { return TM * TN >= 256 * 128 ? 8 : 4; }
constexpr int lds_bytes(int TM, int TN, int RK, int NS) {
  int main_bytes = NS * (TM + TN) * RK * 2;
  int epi_bytes = n_waves(TM, TN) * 64 * EPI_LD * 4;
  return epi_bytes > main_bytes ? epi_bytes : main_bytes;
}

// s_waitcnt immediate: vmcnt <= vm (63: untouched), lgkmcnt <= lgkm (15: untouched), expcnt untouched
constexpr int waitcnt_imm(int vm, int lgkm) { return (vm & 15) | 0x70 | ((vm >> 4) << 14) | (lgkm << 8); }

// One workgroup's tile of one product; wg: the workgroup's index among the product's workgroups (the index
// of the launch, or of the product's range of a grouped launch, which starts at a multiple of 8 so that
// wg % 8 is still the XCD the hardware has put the workgroup on).
template <int TM, int TN, int RK, int NS, bool A_KC, bool B_KC>
__device__ __forceinline__ void ring_tile(const Params& p, const int wg) {
  constexpr int NWAVES = n_waves(TM, TN);
  constexpr int WN = TN == 256 ? 4 : 2, WM = NWAVES / WN;         // wavefront grid
  constexpr int WTM = TM / WM, WTN = TN / WN;                     // wavefront tile: 128x64 or 64x64
  constexpr int MI = WTM / 32, NI = WTN / 32;
  static_assert(NI == 2 && (MI == 2 || MI == 4), "wavefront tile");
  constexpr int STAGE = (TM + TN) * RK;                           // bf16 elements per stage
  constexpr int STEPS = RK / 16;
  typedef Mover<A_KC, TM, RK, NWAVES> MoverA;
  typedef Mover<B_KC, TN, RK, NWAVES> MoverB;
  typedef Frags<A_KC, TM, MI, RK> FragsA;
  typedef Frags<B_KC, TN, NI, RK> FragsB;
  constexpr int LPT = MoverA::IPW + MoverB::IPW;                  // loads per lane and tile
  static_assert((NS - 2) * LPT < 64, "vmcnt range");
  constexpr int WAIT_TILE = waitcnt_imm((NS - 2) * LPT, 0);       // the oldest tile in flight has landed, LDS reads done
  constexpr bool HAND_WAIT = !A_KC || !B_KC;                      // some LDS reads are invisible to the compiler
  constexpr int WAIT_OLDER = waitcnt_imm(63, FragsA::OPS + FragsB::OPS);   // all but the newest batch of LDS reads done
  static_assert(FragsA::OPS + FragsB::OPS < 15, "lgkmcnt range");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  bf16* lds = reinterpret_cast<bf16*>(smem);
  const unsigned lds_base = (unsigned)(uintptr_t)(lds_void_t*)lds;   // LDS byte address of the dynamic segment
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;

  // workgroup -> (split, tile): consecutive ids go round-robin to the 8 XCDs, so give each XCD a
  // contiguous range of tiles, ordered in bands of 8 tile rows, column by column inside a band (the
  // tiles that run together on an XCD then share few operand panels in its L2)
  const int total = p.tiles_m * p.tiles_n * p.splitk;
  if (wg >= total) return;      // padding of a grouped launch (the whole workgroup leaves)
  int pid = wg;
  {
    int per = (total + 7) >> 3, tall = total & 7;
    if (tall == 0) tall = 8;
    int xcd = pid & 7, local = pid >> 3;
    pid = xcd < tall ? xcd * per + local : tall * per + (xcd - tall) * (per - 1) + local;
  }
  const int tiles = p.tiles_m * p.tiles_n;
  const int split = pid / tiles;
  const int tile = pid - split * tiles;
  int tm, tn;
  {
    constexpr int G = 8;
    const int band = tile / (G * p.tiles_n);
    const int first = band * G;
    const int rows = p.tiles_m - first < G ? p.tiles_m - first : G;
    const int in_band = tile - band * G * p.tiles_n;
    tm = first + in_band % rows;
    tn = in_band / rows;
  }
  const int m0 = tm * TM, n0 = tn * TN;
  const int nkt = p.K / RK;
  const int kt_lo = (int)((long long)split * nkt / p.splitk);
  const int kbeg = kt_lo * RK;
  const int nk = (int)((long long)(split + 1) * nkt / p.splitk) - kt_lo;

  // buffer resources based at the tile's first row (k-contiguous: row m0 of [rows][ld]; k-strided:
  // column m0 of [k][ld]); every offset below stays far under 2^31 (checked on the host)
  const bf16* abase = A_KC ? p.A + (size_t)m0 * p.lda : p.A + m0;
  const bf16* bbase = B_KC ? p.B + (size_t)n0 * p.ldb : p.B + n0;
  __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc((void*)abase, 0, 0x7fffffff, 0x00020000);
  __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc((void*)bbase, 0, 0x7fffffff, 0x00020000);
  MoverA ma; ma.init(lane, p.lda);
  MoverB mb; mb.init(lane, p.ldb);
  FragsA fa; fa.init(lane, WTM * wm);
  FragsB fb; fb.init(lane, WTN * wn);

  f32x16_t acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // tile t lives in stage t % NS; indices past the end are clamped (their loads land in a stage nobody
  // reads any more), which keeps the count of loads in flight the same in every iteration
  auto issue = [&](int t, int stage) {
    const int k0 = kbeg + (t < nk ? t : nk - 1) * RK;
    bf16* s = lds + stage * STAGE;
    ma.issue(ra, p.lda, k0, wave, s);
    mb.issue(rb, p.ldb, k0, wave, s + TM * RK);
  };
  bf16x8_t a[2][MI], b[2][NI];     // fragments of two consecutive 16-wide steps
  auto read_frags = [&](int buf, int stage, int step) {
    const bf16* sa = lds + stage * STAGE;
    const unsigned sab = lds_base + (unsigned)(stage * STAGE * 2);
#pragma unroll
    for (int i = 0; i < MI; ++i) a[buf][i] = fa.get(sa, sab, i, step);
#pragma unroll
    for (int j = 0; j < NI; ++j) b[buf][j] = fb.get(sa + TM * RK, sab + TM * RK * 2, j, step);
  };
#pragma unroll
  for (int t = 0; t < NS - 1; ++t) issue(t, t);
  __builtin_amdgcn_s_waitcnt(WAIT_TILE);      // tile 0 has landed (this wavefront's part)
  __builtin_amdgcn_s_barrier();               // ... and everybody's
  asm volatile("" ::: "memory");
  read_frags(0, 0, 0);

  // One iteration = one k tile of RK.  Entering it, the step-0 fragments of tile t are on their way to
  // registers.  Tile t+NS-1 is requested into the stage tile t-1 occupied (every wavefront has passed
  // the barrier that ended iteration t-1, behind all its reads of that stage).  Each 16-wide step
  // first requests the fragments of the next step, then multiplies its own; before the last step,
  // once tile t+1 has landed, comes the barrier, and the fragments requested there are step 0 of
  // tile t+1, so the last step is multiplied under their latency.  (Requesting tile t+NS right behind
  // the barrier instead, a step earlier, was measured and is no faster: the loop is not latency-bound.)
  auto body = [&](int t, int st, int st_next, int st_dma) {
    issue(t + NS - 1, st_dma);
#pragma unroll
    for (int s = 0; s < STEPS; ++s) {
      const int cur = s & 1, nxt = cur ^ 1;
      if (s + 1 < STEPS) {
        read_frags(nxt, st, s + 1);
        if constexpr (HAND_WAIT) __builtin_amdgcn_s_waitcnt(WAIT_OLDER);
        __builtin_amdgcn_sched_barrier(0);
      } else {
        __builtin_amdgcn_s_waitcnt(WAIT_TILE);
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        read_frags(nxt, st_next, 0);
        __builtin_amdgcn_sched_barrier(0);
      }
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Registers written by the hand-issued reads must hold their data wherever control flow joins: the
  // compiler is free to copy them there and does not know that they are still in flight.
  auto settle = [&]() {
    if constexpr (HAND_WAIT) __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, 0));
  };
  settle();
  int t = 0;
  for (; t + NS <= nk; t += NS) {
#pragma unroll
    for (int s = 0; s < NS; ++s) body(t + s, s, (s + 1) % NS, (s + NS - 1) % NS);
    settle();
  }
#pragma unroll
  for (int s = 0; s < NS - 1; ++s)
    if (t + s < nk) {
      body(t + s, s, (s + 1) % NS, (s + NS - 1) % NS);
      settle();
    }
  __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, 0));   // the clamped extra loads still write LDS; the last fragment reads
  __syncthreads();

  // ---- epilogue: each wavefront stages 64x64 quarters of its tile in LDS and writes 16-byte rows ----
  const int half = lane >> 5;
  const int cc = 8 * (lane & 7);
  Epilogue e = p.epi;
  const bool to_partials = p.splitk > 1;
  if (to_partials) {
    e = Epilogue();
    e.out = p.partials + (size_t)split * p.M * p.N;
    e.ldo = p.N;
    e.out_f32 = 1;
  }
  const int n = n0 + WTN * wn + cc;
  float bias[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) bias[i] = 0.f;
  if (e.bias) {
    float4 q0 = *reinterpret_cast<const float4*>(e.bias + n), q1 = *reinterpret_cast<const float4*>(e.bias + n + 4);
    bias[0] = q0.x; bias[1] = q0.y; bias[2] = q0.z; bias[3] = q0.w;
    bias[4] = q1.x; bias[5] = q1.y; bias[6] = q1.z; bias[7] = q1.w;
  }
  float* stage = reinterpret_cast<float*>(smem) + wave * 64 * EPI_LD;
#pragma unroll
  for (int pass = 0; pass < MI / 2; ++pass) {
    const int mrow = m0 + WTM * wm + 64 * pass + (lane >> 3);     // first of this lane's 8 rows (stride 8)
    uint4 raw[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) raw[i] = make_uint4(0, 0, 0, 0);
    if (epilogue_reads_aux(e)) {
#pragma unroll
      for (int i = 0; i < 8; ++i) raw[i] = load_aux8(e, mrow + 8 * i, n);
    }
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
      for (int bj = 0; bj < 2; ++bj)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          int row = 32 * bi + 8 * (r >> 2) + 4 * half + (r & 3);
          stage[row * EPI_LD + 32 * bj + (lane & 31)] = acc[2 * pass + bi][bj][r];
        }
    // the staging area is private to the wavefront: its LDS operations complete in order
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
}

template <int TM, int TN, int RK, int NS, bool A_KC, bool B_KC>
__global__ void __launch_bounds__(64 * n_waves(TM, TN)) k_gemm_ring(Params p) {
  ring_tile<TM, TN, RK, NS, A_KC, B_KC>(p, (int)blockIdx.x);
}
// Several products of one operand layout in one launch: product g owns the workgroups first[g] .. first[g+1]-1.
// Products too small to fill the chip one by one (the weight gradients of a layer) then need no split of their
// contraction, hence no partial sums in memory.
constexpr int GROUP_MAX = 4;
struct GroupParams {
  Params p[GROUP_MAX];
  int first[GROUP_MAX + 1];
  int n;
};
template <int TM, int TN, int RK, int NS, bool A_KC, bool B_KC>
__global__ void __launch_bounds__(64 * n_waves(TM, TN)) k_gemm_ring_grouped(GroupParams gp) {
  int g = 0;
  while (g + 1 < gp.n && (int)blockIdx.x >= gp.first[g + 1]) ++g;
  ring_tile<TM, TN, RK, NS, A_KC, B_KC>(gp.p[g], (int)blockIdx.x - gp.first[g]);
}

// ring depth: what fits the 160 KB of LDS of a compute unit, at most 6 stages
constexpr int ring_depth(int TM, int TN, int RK) {
  if (TM == 128 && TN == 128) return 64 * 1024 / ((TM + TN) * RK * 2);   // two workgroups per compute unit
  int n = 160 * 1024 / ((TM + TN) * RK * 2);
  return n > 6 ? 6 : n;
}
// every tile shape in every operand layout
#define MSLT_RING_INSTANCES(TM, TN, RK)                                                      \
  template __global__ void k_gemm_ring<TM, TN, RK, ring_depth(TM, TN, RK), true, true>(Params);   \
  template __global__ void k_gemm_ring<TM, TN, RK, ring_depth(TM, TN, RK), true, false>(Params);  \
  template __global__ void k_gemm_ring<TM, TN, RK, ring_depth(TM, TN, RK), false, true>(Params);  \
  template __global__ void k_gemm_ring<TM, TN, RK, ring_depth(TM, TN, RK), false, false>(Params);
template __global__ void k_gemm_ring_grouped<128, 128, 64, ring_depth(128, 128, 64), false, false>(GroupParams);
template __global__ void k_gemm_ring_grouped<256, 256, 64, ring_depth(256, 256, 64), false, false>(GroupParams);
template __global__ void k_gemm_ring_grouped<256, 128, 64, ring_depth(256, 128, 64), false, false>(GroupParams);
MSLT_RING_INSTANCES(256, 256, 64)
MSLT_RING_INSTANCES(256, 128, 64)
MSLT_RING_INSTANCES(128, 256, 64)
MSLT_RING_INSTANCES(128, 128, 64)
MSLT_RING_INSTANCES(256, 256, 32)
MSLT_RING_INSTANCES(256, 128, 32)
MSLT_RING_INSTANCES(128, 256, 32)
#undef MSLT_RING_INSTANCES

template <int TM, int TN, int RK, bool A_KC, bool B_KC>
static hipError_t launch_one(const Params& p, dim3 grid, hipStream_t s) {
  constexpr int NS = ring_depth(TM, TN, RK);
  constexpr int LDS = lds_bytes(TM, TN, RK, NS);
  static_assert(LDS <= 160 * 1024, "LDS of a gfx950 compute unit");
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_ring<TM, TN, RK, NS, A_KC, B_KC>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  k_gemm_ring<TM, TN, RK, NS, A_KC, B_KC><<<grid, dim3(64 * n_waves(TM, TN)), LDS, s>>>(p);
  return hipGetLastError();
}
template <int TM, int TN, int RK>
static hipError_t launch_layout(const GemmDesc& d, const Params& p, dim3 grid, hipStream_t s) {
  if (d.a_kcontig && d.b_kcontig) return launch_one<TM, TN, RK, true, true>(p, grid, s);
  if (d.a_kcontig) return launch_one<TM, TN, RK, true, false>(p, grid, s);
  if (d.b_kcontig) return launch_one<TM, TN, RK, false, true>(p, grid, s);
  return launch_one<TM, TN, RK, false, false>(p, grid, s);
}

}  // namespace ring

static void ring_params(const GemmDesc& d, int tile_m, int tile_n, int splitk, float* partials, ring::Params* p) {
  p->A = reinterpret_cast<const bf16*>(d.A);
  p->B = reinterpret_cast<const bf16*>(d.B);
  p->M = d.M; p->N = d.N; p->K = d.K;
  p->lda = d.lda; p->ldb = d.ldb;
  p->splitk = splitk;
  p->tiles_m = d.M / tile_m; p->tiles_n = d.N / tile_n;
  p->partials = partials;
  p->epi = d.epi;
}

int gemm_ring_group_max() { return ring::GROUP_MAX; }
template <int TM, int TN>
static hipError_t grouped_tn(const GemmDesc* d, int n, hipStream_t s) {
  using namespace ring;
  constexpr int RK = 64, NS = ring_depth(TM, TN, RK), LDS = lds_bytes(TM, TN, RK, NS);
  static_assert(LDS <= 160 * 1024, "LDS of a gfx950 compute unit");
  GroupParams gp;
  gp.n = n;
  int at = 0;
  for (int i = 0; i < n; ++i) {
    if (d[i].a_kcontig || d[i].b_kcontig || !gemm_ring_supported(d[i], TM, TN, RK)) return hipErrorInvalidValue;
    ring_params(d[i], TM, TN, 1, nullptr, &gp.p[i]);
    gp.first[i] = at;
    at += (gp.p[i].tiles_m * gp.p[i].tiles_n + 7) & ~7;      // every product starts on XCD 0
  }
  for (int i = n; i <= GROUP_MAX; ++i) gp.first[i] = at;
  static bool attr_set = false;       // one flag per tile size
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_gemm_ring_grouped<TM, TN, RK, NS, false, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  k_gemm_ring_grouped<TM, TN, RK, NS, false, false><<<dim3((unsigned)at), dim3(64 * n_waves(TM, TN)), LDS, s>>>(gp);
  return hipGetLastError();
}
hipError_t gemm_ring_grouped_tn(const GemmDesc* d, int n, int tile_m, int tile_n, hipStream_t s) {
  if (n < 1 || n > ring::GROUP_MAX) return hipErrorInvalidValue;
  if (tile_m == 128 && tile_n == 128) return grouped_tn<128, 128>(d, n, s);
  if (tile_m == 256 && tile_n == 128) return grouped_tn<256, 128>(d, n, s);
  if (tile_m == 256 && tile_n == 256) return grouped_tn<256, 256>(d, n, s);
  return hipErrorInvalidValue;
}

bool gemm_ring_supported(const GemmDesc& d, int tile_m, int tile_n, int rk) {
  if (rk != 32 && rk != 64) return false;
  if (d.M <= 0 || d.N <= 0 || d.K <= 0) return false;
  if (d.lda % 8 || d.ldb % 8 || d.epi.ldo % 8) return false;
  if ((d.epi.act == EPI_MUL || d.epi.act == EPI_ADD) && d.epi.ldaux % 8) return false;
  if (d.epi.drop.thr && d.epi.drop_ld % 4) return false;
  if (d.epi.accumulate && !d.epi.out_f32) return false;
  auto al = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
  if (!al(d.A) || !al(d.B) || !al(d.epi.out) || !al(d.epi.out2) || !al(d.epi.aux) || !al(d.epi.bias)) return false;
  if (!((tile_m == 256 && tile_n == 256) || (tile_m == 256 && tile_n == 128) || (tile_m == 128 && tile_n == 256) ||
        (tile_m == 128 && tile_n == 128 && rk == 64)))
    return false;
  if (d.M % tile_m || d.N % tile_n || d.K % rk) return false;
  // byte offsets inside a tile's buffer view stay below 2^31
  const long long a_span = d.a_kcontig ? (long long)tile_m * d.lda + d.K : (long long)d.K * d.lda + tile_m;
  const long long b_span = d.b_kcontig ? (long long)tile_n * d.ldb + d.K : (long long)d.K * d.ldb + tile_n;
  if (2 * a_span >= 0x7fffffffLL || 2 * b_span >= 0x7fffffffLL) return false;
  return true;
}

hipError_t gemm_ring(const GemmDesc& d, int tile_m, int tile_n, int rk, int splitk, float* partials, hipStream_t s,
                     bool keep_partials) {
  if (!gemm_ring_supported(d, tile_m, tile_n, rk)) return hipErrorInvalidValue;
  if (keep_partials && (!d.epi.out_f32 || d.epi.bias || d.epi.act != EPI_NONE || d.epi.drop.thr || d.epi.out2))
    return hipErrorInvalidValue;
  if (splitk < 1 || splitk > d.K / rk) return hipErrorInvalidValue;
  if (splitk > 1 && partials == nullptr) return hipErrorInvalidValue;
  ring::Params p;
  p.A = reinterpret_cast<const bf16*>(d.A);
  p.B = reinterpret_cast<const bf16*>(d.B);
  p.M = d.M; p.N = d.N; p.K = d.K;
  p.lda = d.lda; p.ldb = d.ldb;
  p.splitk = splitk;
  p.tiles_m = d.M / tile_m; p.tiles_n = d.N / tile_n;
  p.partials = partials;
  p.epi = d.epi;
  dim3 grid((unsigned)(p.tiles_m * p.tiles_n * splitk));
  hipError_t e;
  if (rk == 64) {
    if (tile_m == 256 && tile_n == 256) e = ring::launch_layout<256, 256, 64>(d, p, grid, s);
    else if (tile_m == 256) e = ring::launch_layout<256, 128, 64>(d, p, grid, s);
    else if (tile_n == 256) e = ring::launch_layout<128, 256, 64>(d, p, grid, s);
    else e = ring::launch_layout<128, 128, 64>(d, p, grid, s);
  } else {
    if (tile_m == 256 && tile_n == 256) e = ring::launch_layout<256, 256, 32>(d, p, grid, s);
    else if (tile_m == 256) e = ring::launch_layout<256, 128, 32>(d, p, grid, s);
    else e = ring::launch_layout<128, 256, 32>(d, p, grid, s);
  }
  if (e != hipSuccess || splitk == 1 || keep_partials) return e;
  size_t n8 = (size_t)d.M * d.N / 8;
  k_splitk_reduce<<<dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, s>>>(partials, splitk, d.M, d.N, d.epi);
  return hipGetLastError();
}

}  // namespace mslt
