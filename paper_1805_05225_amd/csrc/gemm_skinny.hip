// Products with few rows (M <= about a thousand): the stepped decoder cell (Sec. 7, Listing 1: "s", an LSTM cell fed by
// 620 + 2000 values for 64 sentences x beam 12 = 768 rows), and the linear layers around it ("s_tr", "readout", the
// output layer).  The throughput kernels of gemm_nt.hip use 256 x 256 tiles: 768 rows x 4000 columns are 48 tiles, so
// K had to be cut into ranges whose partial products went through memory (61 MB per step) and a second pass.  Here a
// work-group owns 96 rows x 128 columns - 768 x 4096 is exactly 256 tiles, one per compute unit - and walks the
// whole K, so the result is complete in the work-group and the epilogue can finish the job:
//   * plain:  C = A B^T + bias, optionally max(0, .), float or bfloat16;
//   * cell:   the 128 columns are the four gates of 32 hidden units (the packed weights are ordered that way), and
//             the epilogue adds the bias, applies the LSTM cell and writes y, h', c' - no pre-activations in memory.
//
// C[M,N] = A[M,K] B[N,K]^T, both operands bfloat16, k-contiguous, rows 16-byte aligned, K a multiple of 8.
// Eight wavefronts: wavefront (kq, wc) owns the 96 x 64 block of column half wc (3 x 2 MFMA blocks of 32x32x16) for
// k-step kq of every 64-wide stage (five fragment reads for six MFMAs; with 96 x 32 per wavefront the LDS reads took
// longer than the MFMAs); the four shares are added in the epilogue.  Two wavefronts per SIMD.  Operands travel from global memory straight into LDS (16 bytes
// per lane, 1 KiB per wavefront instruction = 8 rows of 128 bytes), four stages of 64 k, one barrier per stage; bank conflicts
// are avoided by placement: the 16-byte slot p of row r holds k-chunk p ^ ((r >> 1) & 7).  What bounds it is the path
// from L2 to LDS (about 47 bytes per clock and compute unit, measured for the large kernels): 28 KiB per stage
// against 384 clocks of MFMA work, i.e. about 600 clocks per stage.
//
// A second tile shape, 64 rows x 64 columns (every wavefront one k-step of a 64 x 32 block), serves products whose
// 96 x 128 tiles would occupy less than half the device (the decoder's query projection and readout, 768 x 1000: 64 tiles
// against 192): what bounds the kernel is the rate at which ONE compute unit pulls operands from L2, so more, smaller
// tiles finish sooner although they move more bytes in total.
#include "recurrent_dev.h"

namespace lstm {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
constexpr int kBufFlags = 0x00020000;   // raw buffer descriptor word 3 for gfx9-family devices
constexpr int kRow = 128;                          // bytes per LDS row (64 bfloat16)
constexpr int kDepth = 4;                          // stages in LDS: three in flight while one is multiplied (2: +20 %, 3 and 5: the same)
// Tile geometry for wavefront blocks of BI x BJ MFMA blocks (32 x 32): the tile is 32 BI rows x 64 BJ columns.
template <int BI, int BJ>
struct Geo {
  static constexpr int kTM = 32 * BI, kTN = 64 * BJ;
  static constexpr int kAop = kTM * kRow, kBop = kTN * kRow, kStage = kAop + kBop;   // <3,2>: 12 + 16 KiB
  static constexpr int kLoads = (kTM + kTN) / 8;                                      // wavefront-loads per stage
  static constexpr int kPerWave = (kLoads + 7) / 8;                                   // issued by every wavefront per stage
  static constexpr int kDummy = kDepth * kStage;      // 4 KiB that the surplus loads of a stage write zeros to (see the kernel)
  static constexpr int kEpStride = kTN + 4;           // floats per staged row
  static constexpr int kLds = kDummy + 4096;          // <3,2>: 118784 bytes; the epilogue's staging reuses the stages
  static_assert(kTM * kEpStride * 4 <= kDummy, "the epilogue's staging must fit into the stage buffers");
};
constexpr unsigned kParked = 0x7ffffff0u;

struct SkinnyArgs {
  const char* A; const char* B; void* C; const float* bias;
  int M, N, K;
  long lda, ldb, ldc;                    // elements
  long sAz, sBz, sCz, sbiasz; int nz;    // blockIdx.z batches independent problems (the two directions)
  int out_bf16, relu;
  // cell epilogue (cell != 0): N = 128 * ceil(n / 32), column 128 * tile + 32 * gate + unit; bias is [4n] gate-major
  int cell, n;
  const float* h_in; const float* c_in; float* h_out; float* c_out; uint16_t* y; long ldy; float* cs; const int* lens;
};

__device__ __forceinline__ void load_to_lds_b128(const u32x4& rsrc, unsigned lds_addr, unsigned voff, unsigned soff) {
  asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" ::"s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory");
}
__device__ __forceinline__ u32x4 make_rsrc(const void* base, unsigned bytes) {
  const unsigned long long a = (unsigned long long)base;
  u32x4 r;
  r[0] = __builtin_amdgcn_readfirstlane((unsigned)a);
  r[1] = __builtin_amdgcn_readfirstlane((unsigned)(a >> 32) & 0xffffu);
  r[2] = __builtin_amdgcn_readfirstlane(bytes);
  r[3] = kBufFlags;
  return r;
}
__device__ __forceinline__ f32x16 mma32(uint4 a, uint4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// Work-group -> tile.  Work-groups are dealt to the eight XCDs round-robin (blockIdx & 7 is the XCD).  The tiles an XCD
// runs at a time should share operand panels out of its L2: with tiles_m <= 32 row tiles, an XCD takes all row tiles of
// 32 / bm column tiles at a time (bm = tiles_m rounded up to a power of two); otherwise tiles are dealt row-major.
// s_waitcnt operand for vmcnt(n) lgkmcnt(0): vmcnt's low four bits sit in bits 3:0, its upper two in bits 15:14
constexpr int vm_wait(unsigned n) { return (int)(0x0070u | (n & 15u) | ((n >> 4) << 14)); }
struct Tile { int tm, tn, pos; bool live; };
__host__ __device__ inline int pow2_at_least(int v) { int p = 1; while (p < v) p <<= 1; return p; }
__device__ __forceinline__ Tile tile_of(int tiles_m, int tiles_n) {
  Tile t = {0, 0, 0, false};
  const int bid = blockIdx.x;
  if (tiles_m <= 32) {
    const int bm = pow2_at_least(tiles_m), bn = 32 / bm;
    const int xcd = bid & 7, slot = bid >> 3, group = (slot / 32) * 8 + xcd, pos = slot % 32;
    t.tm = pos % bm; t.tn = group * bn + pos / bm; t.pos = pos;
    t.live = t.tm < tiles_m && t.tn < tiles_n;
  } else {
    t.tm = bid % tiles_m; t.tn = bid / tiles_m; t.pos = bid & 31;
    t.live = t.tn < tiles_n;
  }
  return t;
}
inline int grid_for(int tiles_m, int tiles_n) {
  if (tiles_m <= 32) {
    const int bm = pow2_at_least(tiles_m), bn = 32 / bm;
    const int groups = cdiv(tiles_n, bn);
    return cdiv(groups, 8) * 8 * 32;
  }
  return tiles_m * tiles_n;
}

template <int BI, int BJ, bool CELL>
__global__ __launch_bounds__(512) void skinny_kernel(SkinnyArgs g) {
  typedef Geo<BI, BJ> G;
  constexpr int kTM = G::kTM, kTN = G::kTN, kAop = G::kAop, kStage = G::kStage, kLoads = G::kLoads, kDummy = G::kDummy,
                kEpStride = G::kEpStride, kPerWave = G::kPerWave;
  static_assert(!CELL || (BI == 3 && BJ == 2), "the cell epilogue expects the four gates of 32 units in a tile's 128 columns");
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kq = wave >> 1, wc = wave & 1;          // k-step of a stage (0..3) and column half (32 BJ columns) of this wavefront
  const int r = lane & 31, gq = lane >> 5;
  const int tiles_m = (g.M + kTM - 1) / kTM, tiles_n = (g.N + kTN - 1) / kTN;
  const Tile tl = tile_of(tiles_m, tiles_n);
  if (!tl.live) return;
  const int m0 = tl.tm * kTM, n0 = tl.tn * kTN, z = blockIdx.z;
  const int K = g.K, nstage = (K + 63) / 64;
  // The work-groups of an XCD that share an operand panel would ask for the same lines at the same time, and all of
  // them would wait for the one fetch from beyond L2 (whose rate per compute unit is a quarter of the L2's).  So each
  // of the 32 work-groups an XCD runs together starts at a different k and wraps around: a line is fetched once and
  // found in L2 by the others when their turn comes (the sum over k does not care about the order).
  const int rot = (int)(((long)tl.pos * nstage) >> 5);

  f32x16 acc[BI][BJ];
#pragma unroll
  for (int i = 0; i < BI; ++i)
#pragma unroll
    for (int j = 0; j < BJ; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // Loads: wavefront-load q of a stage (q = wave + 8 i) fills rows 8 q' .. 8 q' + 7 of A (q < kTM / 8) or B (q < kLoads);
  // lane l fills slot l & 7 of row l >> 3 of those, i.e. fetches k-chunk (l & 7) ^ swizzle(row).  Rows past the operand's
  // end and chunks past K point outside the buffer descriptor and arrive as zeros.  Every wavefront issues the same
  // number of loads per stage, so that one wait count serves all of them: surplus ones (q >= kLoads; four in the 96 x 128
  // tile) have every lane parked and write their zeros to a spare 4 KiB of LDS without touching memory.
  unsigned voff[kPerWave], dst[kPerWave];
  int chunk[kPerWave];
  bool is_b[kPerWave];
  const long a_bytes = (long)g.M * g.lda * 2, b_bytes = (long)g.N * g.ldb * 2;
#pragma unroll
  for (int i = 0; i < kPerWave; ++i) {
    const int q = wave + 8 * i;
    const bool real = q < kLoads;
    is_b[i] = q >= kTM / 8;
    const int rg = is_b[i] ? q - kTM / 8 : q;
    const int rl = rg * 8 + (lane >> 3);
    chunk[i] = real ? (lane & 7) ^ ((rl >> 1) & 7) : 0x10000;            // surplus load: "past K" in every stage
    const long row = (is_b[i] ? n0 : m0) + rl;
    const bool inside = real && (is_b[i] ? row < g.N : row < g.M);
    const long off = row * (is_b[i] ? g.ldb : g.lda) * 2 + (chunk[i] & 7) * 16;
    voff[i] = (inside && off <= 0x7fffff00L) ? (unsigned)off : kParked;
    dst[i] = real ? (unsigned)((is_b[i] ? kAop : 0) + rg * 1024) : 0u;
  }
  const unsigned lds_base = (unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)lds;
  const u32x4 ra = make_rsrc(g.A + g.sAz * z * 2, a_bytes > 0x7fffff00L ? 0x7fffff00u : (unsigned)a_bytes);
  const u32x4 rb = make_rsrc(g.B + g.sBz * z * 2, b_bytes > 0x7fffff00L ? 0x7fffff00u : (unsigned)b_bytes);
  auto issue = [&](int it) __attribute__((always_inline)) {
    const unsigned buf = lds_base + (unsigned)(it % kDepth) * kStage;
    const int kt = it + rot < nstage ? it + rot : it + rot - nstage;       // which 64 k this stage holds
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      const bool past = kt * 64 + chunk[i] * 8 >= K;           // ragged last k-tile (and every surplus load)
      const unsigned where = wave + 8 * i >= kLoads ? lds_base + kDummy + (unsigned)(wave & 3) * 1024u : buf + dst[i];
      load_to_lds_b128(is_b[i] ? rb : ra, where, past ? kParked : voff[i], (unsigned)kt * 128u);
    }
  };
  // Fragment reads: row (i*32 + r) of A / (wc*32*BJ + j*32 + r) of B, k-chunk 2 kq + gq, in slot (2 kq + gq) ^ ((row >> 1) & 7)
  const int slot = ((2 * kq + gq) ^ ((r >> 1) & 7)) * 16;
  const int fa_off = r * kRow + slot, fb_off = kAop + (wc * 32 * BJ + r) * kRow + slot;

  // Pipeline: while the MFMAs of stage it run (fragments in registers), the fragments of stage it+1 are read from LDS
  // and the loads of stages it+2 .. it+4 are in flight (a load from beyond L2 takes longer than two stages of MFMAs:
  // with one stage ahead the loop ran at memory latency, 1700 clocks per stage; and with fragment reads and MFMAs of
  // one stage in program order the compiler made every MFMA wait for its own LDS read).  Loads complete in issue
  // order, four per wavefront and stage: when at most 8 are outstanding, everything up to the stage two behind the
  // newest has landed.  A buffer is overwritten one iteration after every wavefront has passed the barrier behind
  // which it read the buffer's fragments (and waited for them).
  uint4 fa[2][BI], fb[2][BJ];                      // [register set][row block], [register set][column block]
  auto read_a = [&](int it, int set, int i) __attribute__((always_inline)) {
    fa[set][i] = *(const uint4*)(lds + (it % kDepth) * kStage + fa_off + i * 32 * kRow);
  };
  auto read_b = [&](int it, int set, int j) __attribute__((always_inline)) {
    fb[set][j] = *(const uint4*)(lds + (it % kDepth) * kStage + fb_off + j * 32 * kRow);
  };
  auto wait_stage = [&](int newer) __attribute__((always_inline)) {       // `newer` stages were issued behind the awaited one
    if (newer >= 4) __builtin_amdgcn_s_waitcnt(vm_wait(4 * kPerWave));
    else if (newer == 3) __builtin_amdgcn_s_waitcnt(vm_wait(3 * kPerWave));
    else if (newer == 2) __builtin_amdgcn_s_waitcnt(vm_wait(2 * kPerWave));
    else if (newer == 1) __builtin_amdgcn_s_waitcnt(vm_wait(kPerWave));
    else __builtin_amdgcn_s_waitcnt(vm_wait(0));
  };
#pragma unroll
  for (int j = 0; j < kDepth; ++j)
    if (j < nstage) issue(j);
  wait_stage(min(nstage - 1, kDepth - 1));
  __syncthreads();
  // fragment read number q of a stage, in the order the MFMAs will want them: B block 0, the A blocks, the other B blocks
  auto read_nr = [&](int it, int set, int q) __attribute__((always_inline)) {
    if (q == 0) read_b(it, set, 0);
    else if (q <= BI) read_a(it, set, q - 1);
    else if (q < BI + BJ) read_b(it, set, q - BI);
  };
#pragma unroll
  for (int q = 0; q < BI + BJ; ++q) read_nr(0, 0, q);
  // The MFMAs of a stage in the order (row block, column block) = (0,0) (1,0) .. (0,1) (1,1) ..; with `next`, one
  // fragment read of the following stage goes out behind each MFMA (96 x 128 tile: behind the first five of six),
  // what is left of them behind the last.  (All reads in front of the MFMAs held the MFMAs back until the LDS had
  // taken them: reads and MFMAs of a stage then ran one after the other.)
  auto mfmas = [&](int set, bool next, int it_next) __attribute__((always_inline)) {
#pragma unroll
    for (int m = 0; m < BI * BJ; ++m) {
      const int i = m % BI, j = m / BI;
      acc[i][j] = mma32(fa[set][i], fb[set][j], acc[i][j]);
      if (next) {
        __builtin_amdgcn_sched_barrier(0);
        read_nr(it_next, set ^ 1, m);
        if (m == BI * BJ - 1) {
#pragma unroll
          for (int q = BI * BJ; q < BI + BJ; ++q) read_nr(it_next, set ^ 1, q);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  // one stage with a successor.  No branch between the successor's reads and the MFMAs: where two paths with different
  // numbers of pending LDS reads met in front of the MFMAs, the compiler made them wait for every read.
  auto step = [&](int it, int set) __attribute__((always_inline)) {
    wait_stage(min(nstage - 2 - it, kDepth - 2));                         // stage it+1 landed; own fragment reads of stage it done
    __syncthreads();
    if (it + kDepth < nstage) issue(it + kDepth);                         // into the buffer of stage it, now in registers everywhere
    __builtin_amdgcn_sched_barrier(0);
    mfmas(set, true, it + 1);
    __builtin_amdgcn_sched_barrier(0);
  };
  int it = 0;
  for (; it + 2 < nstage; it += 2) {
    step(it, 0);
    step(it + 1, 1);
  }
  if (it + 2 == nstage) {
    step(it, 0);
    mfmas(1, false, 0);
  } else {
    mfmas(0, false, 0);
  }
  __syncthreads();                                 // the stage buffers are free for the epilogue

  // Epilogue.  The four k-steps' shares meet in LDS (the stage buffers are free), one after the other:
  // acc[i][j][v] is row i*32 + 8 (v / 4) + 4 gq + v % 4, column wc*32*BJ + j*32 + r.
  float* ep = (float*)lds;
#pragma unroll
  for (int round = 3; round >= 0; --round) {
    if (kq == round) {
#pragma unroll
      for (int i = 0; i < BI; ++i)
#pragma unroll
        for (int j = 0; j < BJ; ++j)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float* e = &ep[(i * 32 + 8 * (v >> 2) + 4 * gq + (v & 3)) * kEpStride + wc * 32 * BJ + j * 32 + r];
            *e = round == 3 ? acc[i][j][v] : *e + acc[i][j][v];
          }
    }
    __syncthreads();
  }
  if constexpr (!CELL) {
    // thread -> (row, four columns): kTN / 4 threads per row, 512 / (kTN / 4) rows per pass
    constexpr int kTpr = kTN / 4;
    const int c4 = (tid % kTpr) * 4, col = n0 + c4;
    const float* bias = g.bias ? g.bias + g.sbiasz * z : nullptr;
    float bv[4] = {0.f, 0.f, 0.f, 0.f};
    if (bias) {
#pragma unroll
      for (int k = 0; k < 4; ++k) if (col + k < g.N) bv[k] = bias[col + k];
    }
    const bool vec = (g.ldc % 4 == 0) && ((((uintptr_t)g.C) & 15u) == 0) && (g.sCz % 4 == 0) && col + 3 < g.N;
    for (int rr = tid / kTpr; rr < kTM; rr += 512 / kTpr) {
      const int row = m0 + rr;
      if (row >= g.M || col >= g.N) continue;
      const float4 val = *(const float4*)&ep[rr * kEpStride + c4];
      float e[4] = {val.x + bv[0], val.y + bv[1], val.z + bv[2], val.w + bv[3]};
      if (g.relu) {
#pragma unroll
        for (int k = 0; k < 4; ++k) e[k] = e[k] > 0.f ? e[k] : 0.f;
      }
      const long off = g.sCz * z + (long)row * g.ldc + col;
      if (g.out_bf16) {
        uint16_t* Cb = (uint16_t*)g.C + off;
        if (vec) {
          uint2 o;
          o.x = f2bf_bits(e[0]) | ((unsigned)f2bf_bits(e[1]) << 16);
          o.y = f2bf_bits(e[2]) | ((unsigned)f2bf_bits(e[3]) << 16);
          *(uint2*)Cb = o;
        } else {
#pragma unroll
          for (int k = 0; k < 4; ++k) if (col + k < g.N) Cb[k] = f2bf_bits(e[k]);
        }
      } else {
        float* Cf = (float*)g.C + off;
        if (vec) *(float4*)Cf = make_float4(e[0], e[1], e[2], e[3]);
        else {
#pragma unroll
          for (int k = 0; k < 4; ++k) if (col + k < g.N) Cf[k] = e[k];
        }
      }
    }
  } else {
    // thread -> (unit of the tile, row): 32 threads per row, 16 rows per pass; staged columns 32 q + unit
    const int uu = tid & 31, j = tl.tn * 32 + uu, n = g.n;
    if (j < n) {
      float bv[4] = {0.f, 0.f, 0.f, 0.f};
      if (g.bias) {
#pragma unroll
        for (int q = 0; q < 4; ++q) bv[q] = g.bias[(long)z * 4 * n + q * n + j];
      }
      for (int rr = tid >> 5; rr < kTM; rr += 16) {
        const int b = m0 + rr;
        if (b >= g.M) break;
        const long si = ((long)z * g.M + b) * n + j;
        const bool valid = clamp_len(g.lens, b, 1) > 0;
        float c = g.c_in ? g.c_in[si] : 0.f, h = 0.f;
        if (valid) {
          float zh[4];
#pragma unroll
          for (int q = 0; q < 4; ++q) zh[q] = ep[rr * kEpStride + q * 32 + uu] + bv[q];
          const float zx[4] = {0.f, 0.f, 0.f, 0.f};
          const CellOut o = lstm_cell(zh, zx, c);
          c = o.c; h = o.h;
        }
        g.y[(long)b * g.ldy + (long)z * n + j] = f2bf_bits(h);
        if (g.cs) g.cs[si] = c;
        if (g.c_out) g.c_out[si] = c;
        if (g.h_out) g.h_out[si] = valid ? h : (g.h_in ? g.h_in[si] : 0.f);
      }
    }
  }
}

template <int BI, int BJ, bool CELL>
hipError_t launch_as(const SkinnyArgs& a, hipStream_t s) {
  typedef Geo<BI, BJ> G;
  static std::atomic<unsigned long long> attr_set{0};
  const hipError_t ea = once_per_device(attr_set, [] {
    return hipFuncSetAttribute((const void*)skinny_kernel<BI, BJ, CELL>, hipFuncAttributeMaxDynamicSharedMemorySize, G::kLds);
  });
  if (ea != hipSuccess) return ea;
  const dim3 grid(grid_for(cdiv(a.M, G::kTM), cdiv(a.N, G::kTN)), 1, a.nz);
  hipLaunchKernelGGL((skinny_kernel<BI, BJ, CELL>), grid, dim3(512), G::kLds, s, a);
  return hipGetLastError();
}
hipError_t launch(const SkinnyArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0 || a.nz <= 0) return hipSuccess;
  if (a.cell) return launch_as<3, 2, true>(a, s);
  // fewer 96 x 128 tiles than half the device has compute units: 64 x 64 tiles
  if ((long)cdiv(a.M, 96) * cdiv(a.N, 128) * a.nz < 128) return launch_as<2, 1, false>(a, s);
  return launch_as<3, 2, false>(a, s);
}

// Wcell[d][128 t + 32 q + u][k] = [W_x^T | 0 | W_h^T | 0] row (q n + 32 t + u), zero for units past n; a 64 x 64 tile of
// (k, packed row) per work-group: rows of W are read along the packed-row axis in runs of 32 consecutive columns.
__global__ __launch_bounds__(256) void pack_wcell_kernel(const uint16_t* Wx, const uint16_t* Wh, uint16_t* Wc, int n_in, int n_in_pad, int n,
                                                         int Kc, int Np) {
  __shared__ uint16_t tile[64][66];
  const int N4 = 4 * n;
  const int d = blockIdx.z;
  Wx += (long)d * n_in * N4;
  Wh += (long)d * n * N4;
  Wc += (long)d * Np * Kc;
  const int k0 = blockIdx.x * 64, p0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  {
    const int p = p0 + tx, t = p >> 7, q = (p >> 5) & 3, u = p & 31, j = t * 32 + u;
    const int col = q * n + j;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int k = k0 + ty + 4 * i;
      uint16_t v = 0;
      if (p < Np && j < n) {
        if (k < n_in) v = Wx[(long)k * N4 + col];
        else if (k >= n_in_pad && k < n_in_pad + n) v = Wh[(long)(k - n_in_pad) * N4 + col];
      }
      tile[ty + 4 * i][tx] = v;
    }
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int p = p0 + ty + 4 * i, k = k0 + tx;
    if (p < Np && k < Kc) Wc[(long)p * Kc + k] = tile[tx][ty + 4 * i];
  }
}

}  // namespace

bool gemm_skinny_ok(const GemmArgs& g) {
  const auto a16 = [](const void* p) { return ((uintptr_t)p & 15u) == 0; };
  // only where the 256 x 256 tiles of the throughput kernel would leave most of the device idle (it is the faster one
  // from about half a device's worth of tiles: 768 x 20000 x 1000 takes 49 us there and 72 us here)
  if ((long)cdiv(g.M, 256) * cdiv(g.N, 256) * g.nz >= 128) return false;
  return g.in_bf16 && g.a_kcontig && g.b_kcontig && !g.lens && g.M <= kSkinnyMaxRows && g.nseg == 1 && !g.a_rows && !g.c_rows && !g.m_dev &&
         !g.k_dev && !g.accumulate && g.ksplit <= 1 && g.K % 8 == 0 && g.lda % 8 == 0 && g.ldb % 8 == 0 && g.sAz % 8 == 0 && g.sBz % 8 == 0 &&
         a16(g.A) && a16(g.B) && (long)g.N * g.ldb * 2 <= 0x7fffff00L;
}
hipError_t launch_gemm_skinny(const GemmArgs& g, bool relu, hipStream_t s) {
  SkinnyArgs a = {};
  a.A = (const char*)g.A; a.B = (const char*)g.B; a.C = g.C; a.bias = g.bias;
  a.M = g.M; a.N = g.N; a.K = g.K; a.lda = g.lda; a.ldb = g.ldb; a.ldc = g.ldc;
  a.sAz = g.sAz; a.sBz = g.sBz; a.sCz = g.sCz; a.sbiasz = g.sbiasz; a.nz = g.nz;
  a.out_bf16 = g.out_bf16; a.relu = relu;
  return launch(a, s);
}
hipError_t launch_pack_wcell(const void* W_x, const void* W_h, void* Wcell, int n_in, int n_in_pad, int n, int Kc, int ndir, hipStream_t s) {
  const int Np = 128 * cdiv(n, 32);
  hipLaunchKernelGGL(pack_wcell_kernel, dim3(cdiv(Kc, 64), cdiv(Np, 64), ndir), dim3(256), 0, s, (const uint16_t*)W_x, (const uint16_t*)W_h,
                     (uint16_t*)Wcell, n_in, n_in_pad, n, Kc, Np);
  return hipGetLastError();
}
hipError_t launch_step_cell(const void* Acat, const void* Wcell, const float* bias, const float* h_in, const float* c_in, float* h_out,
                            float* c_out, void* y, long ldy, float* cs, const int* lens, int B, int n, int Kc, int ndir, hipStream_t s) {
  SkinnyArgs a = {};
  const int Np = 128 * cdiv(n, 32);
  a.A = (const char*)Acat; a.B = (const char*)Wcell; a.bias = bias;
  a.M = B; a.N = Np; a.K = Kc; a.lda = Kc; a.ldb = Kc;
  a.sAz = (long)B * Kc; a.sBz = (long)Np * Kc; a.nz = ndir;
  a.cell = 1; a.n = n; a.h_in = h_in; a.c_in = c_in; a.h_out = h_out; a.c_out = c_out; a.y = (uint16_t*)y; a.ldy = ldy; a.cs = cs; a.lens = lens;
  return launch(a, s);
}

}  // namespace lstm
