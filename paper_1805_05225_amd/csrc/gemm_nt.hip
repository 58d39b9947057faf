// Fast path of the hoisted matrix products for bfloat16 storage.
//
// All four products of a layer (Zx = X W_x + b, dX = DZ W_x^T, dW_x = X^T DZ, dW_h = Hprev^T DZ;
// paper Sec. 3: work moved out of the recurrent loop) are brought into ONE shape,
//     C[M,N] (+)= sum_seg A_seg[M,K] . B_seg[N,K]^T  (+ bias[N]),
// with both operands k-contiguous, rows 16-byte aligned and K a multiple of 8.  Operands that are
// stored the other way round (W_x for Zx; X, Hprev and DZ for the weight gradients) are transposed
// once by `launch_transpose` below - a bandwidth-bound pass that costs a few percent of the product
// it feeds - instead of being transposed on the fly inside the MFMA loop.
//
// gemm_dl8_* (operands loaded straight into LDS, eight wavefronts; described where it is defined) serves every K that
// is a multiple of 8; gemm_tn8_f32 serves the k-major operand pair of the weight gradients.
#include "common.h"
#include "recurrent_dev.h"
#include <algorithm>

namespace lstm {
namespace {

constexpr int kT = 256;                   // tile edge (both M and N)
constexpr int kKB = 64;                   // k per stage (bf16 elements)
constexpr int kSupM = 8, kSupN = 4;   // tiles per XCD-resident block (kSupM * kSupN = 32 CUs)

struct NtArgs {
  const char* A; const char* B; void* C; const float* bias;
  int M, N, K;
  long lda, ldb, ldc;                     // elements
  long sAz, sBz, sCz, sbiasz; int nz;
  int nseg; long sAseg, sBseg;
  int accumulate;
  const int* a_rows; const int* c_rows;   // logical row -> physical row of A / of C (NULL: identity)
  const int* k_rows; int k_phys_rows;     // k-major kernel: k -> row of A and B in memory (NULL: identity), rows in memory
  const int* m_dev; const int* k_dev;     // device-resident M / K (NULL: use M / K above)
  int a_phys_rows;                        // rows of A in memory when a_rows is given
  int ksplit;                             // > 1: K is cut into that many ranges, each adds its part to C atomically ...
  float* parts; long sPart;               // ... or, if parts != NULL, stores it at parts + (z * ksplit + range) * sPart (layout of C)
  int blocked;                            // tile raster: 1 = blocks of kSupM x kSupN tiles per XCD, 0 = bands of 8 tile columns
};

__device__ __forceinline__ f32x16 mma(uint4 a, uint4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
constexpr int kBufFlags = 0x00020000;   // raw buffer descriptor word 3 for gfx9-family devices

// What every kernel variant needs to know about its tile.
struct TileCoord { int M, K, m0, n0, z, ks, ksplit, pos; bool live; };
__device__ __forceinline__ TileCoord tile_coord(const NtArgs& g) {
  TileCoord t;
  t.live = false;
  t.pos = 0;                                        // place inside the XCD's block of tiles (blocked raster; else 0)
  t.M = g.m_dev ? min(g.M, *g.m_dev) : g.M;        // the grid is sized for g.M; surplus tiles leave at once
  t.K = g.k_dev ? min(g.K, *g.k_dev) : g.K;
  const int tiles_m = (g.M + kT - 1) / kT, tiles_n = (g.N + kT - 1) / kT;
  const int bid = blockIdx.x;
  int tm, tn;
  if (g.blocked) {
    // Work-groups are dealt to the eight XCDs round-robin, so blockIdx & 7 is the XCD and blockIdx >> 3 counts the
    // work-groups of that XCD in launch order.  The 32 work-groups an XCD runs at a time form a block of
    // kSupM x kSupN tiles: kSupM + kSupN operand panels feed kSupM * kSupN tiles out of that XCD's L2.
    const int sup_m = (tiles_m + kSupM - 1) / kSupM, sup_n = (tiles_n + kSupN - 1) / kSupN;
    const int xcd = bid & 7, slot = bid >> 3;
    const int sup = (slot / (kSupM * kSupN)) * 8 + xcd, pos = slot % (kSupM * kSupN);
    if (sup >= sup_m * sup_n) return t;
    const int sn = sup % sup_n, sm = sup / sup_n;
    tm = sm * kSupM + pos / kSupN; tn = sn * kSupN + pos % kSupN;
    t.pos = pos;
    if (tm >= tiles_m || tn >= tiles_n) return t;
  } else {
    // few tiles: bands of 8 tile columns, row-major inside a band; every XCD keeps one B tile column in its L2
    const int band = bid / (8 * tiles_m);
    const int width = min(8, tiles_n - band * 8);
    const int rel = bid - band * 8 * tiles_m;
    tn = band * 8 + rel % width; tm = rel / width;
  }
  t.m0 = tm * kT; t.n0 = tn * kT;
  if (t.m0 >= t.M) return t;
  t.ksplit = g.ksplit > 1 ? g.ksplit : 1;
  t.z = blockIdx.y / t.ksplit; t.ks = blockIdx.y - t.z * t.ksplit;
  t.live = true;
  return t;
}

// Writes a work-group's 256x256 accumulator tile to C.  The tile is held by 2 x (8 / TN) wavefronts, each
// 4 x TN MFMA blocks of 32x32 (TN = 4: 2x2 wavefronts of 128x128; TN = 2: 2x4 wavefronts of 128x64).
template <typename TC, int TN>
__device__ __forceinline__ void store_tile(f32x16 (&acc)[4][TN], char* lds, const NtArgs& g, int M, int m0, int n0, int z, int ks,
                                           int ksplit) {
  constexpr int WN = 8 / TN, NW = 2 * WN;            // wavefronts along N, wavefronts in all
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave / WN, wn = wave % WN;
  const int r = lane & 31, gq = lane >> 5;
  // Epilogue.  A lane holds column (lane % 32), rows 8*(v/4) + 4*(lane/32) + v%4 of each 32x32 block: stored as
  // it is that would be 128-byte pieces, eight of them per row at different times.  The tile goes through LDS
  // instead (two halves of 128 rows, the main loop's buffers are free by now) and leaves as whole rows: one
  // wavefront store = 256 consecutive columns of one row.
  const bool to_parts = ksplit > 1 && g.parts != nullptr;      // this K range keeps its own copy: plain stores, no atomics
  TC* C = to_parts ? (TC*)(g.parts + ((long)z * ksplit + ks) * g.sPart) : (TC*)g.C + g.sCz * z;
  const float* bias = g.bias ? g.bias + g.sbiasz * z : nullptr;
  constexpr int kEpStride = 260;                      // floats per staged row (16-byte aligned, off the bank period)
  float* ep = (float*)lds;
  const bool vec_ok = (g.ldc % 4 == 0) && (((uintptr_t)C & 15u) == 0);
  float bv[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int col = n0 + wn * (TN * 32) + j * 32 + r;
    bv[j] = (bias && ks == 0 && col < g.N) ? bias[col] : 0.f;
  }
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    __syncthreads();                                   // LDS free: main loop done / previous half stored
#pragma unroll
    for (int ii = 0; ii < 2; ++ii)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int rowl = wm * 64 + ii * 32 + 8 * (v >> 2) + 4 * gq + (v & 3);
          ep[rowl * kEpStride + wn * (TN * 32) + j * 32 + r] = acc[2 * half + ii][j][v] + bv[j];
        }
    __syncthreads();
    const int col = n0 + lane * 4;
    for (int rr = 0; rr < 128 / NW; ++rr) {
      const int rowl = wave * (128 / NW) + rr;
      const int row = m0 + (rowl >> 6) * 128 + half * 64 + (rowl & 63);
      if (row >= M) break;                             // rows ascend with rr inside a wave's share
      if (col >= g.N) continue;
      const float4 val = *(const float4*)&ep[rowl * kEpStride + lane * 4];
      const float e[4] = {val.x, val.y, val.z, val.w};
      const long off = (long)((g.c_rows && !to_parts) ? g.c_rows[row] : row) * g.ldc + col;     // parts keep the packed rows
      const bool whole = vec_ok && col + 3 < g.N;
      if constexpr (sizeof(TC) == 4) {
        float* Cf = (float*)C + off;
        if (ksplit > 1 && !to_parts) {
#pragma unroll
          for (int k = 0; k < 4; ++k)
            if (col + k < g.N) unsafeAtomicAdd(Cf + k, e[k]);
        } else if (whole) {
          float4 o = val;
          if (g.accumulate && !to_parts) {
            const float4 old = *(const float4*)Cf;
            o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w;
          }
          *(float4*)Cf = o;
        } else {
#pragma unroll
          for (int k = 0; k < 4; ++k)
            if (col + k < g.N) Cf[k] = (g.accumulate && !to_parts) ? Cf[k] + e[k] : e[k];
        }
      } else {
        uint16_t* Cb = (uint16_t*)C + off;
        if (whole) {
          uint2 o;
          o.x = f2bf_bits(e[0]) | ((unsigned)f2bf_bits(e[1]) << 16);
          o.y = f2bf_bits(e[2]) | ((unsigned)f2bf_bits(e[3]) << 16);
          *(uint2*)Cb = o;
        } else {
#pragma unroll
          for (int k = 0; k < 4; ++k)
            if (col + k < g.N) Cb[k] = f2bf_bits(e[k]);
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------------------
// Same product with the operands brought from global memory straight into LDS (16-byte-per-lane buffer loads
// with the LDS destination: no staging registers, no LDS store instructions), for K a multiple of 64.
//
// LDS holds two stages of [A | B], each operand 256 rows of 128 bytes (64 bf16), unpadded: a wavefront-wide
// load fills 1 KiB = 8 consecutive rows, lane l writing bytes 16*l of it.  Bank conflicts of the fragment reads
// are avoided by the placement instead of padding: the 16-byte slot p of row r holds k-chunk p ^ ((r >> 1) & 7),
// which the loading lane arranges by choosing WHICH global chunk it fetches.
//
// Wavefronts: 2 x (8 / TN), each 4 x TN MFMA blocks; the kernels below use TN = 2: eight wavefronts of 128x64,
// two per SIMD, so one wavefront's LDS reads and waits hide behind the other's MFMAs (four wavefronts of 128x128
// measured 15-20 % slower).  Measured on the device: what bounds this kernel is the path from L2 to LDS - with the
// MFMAs taken out the loop needs the same number of cycles (about 3500 per stage against 2050 of MFMA work), because
// a fifth of a stage's lines is a first touch per XCD and the work-groups sharing a panel wait for the same miss.
//
// Loop, per stage `it` (k advances 64 = four MFMA k-steps): fragments of k-step s+1 are read while the MFMAs of
// step s run.  Before the last k-step the wavefront waits for its own loads of stage it+1 and meets the others at
// the barrier; after it every load of stage it+1 has landed and every read of stage it's buffer has completed,
// so the loads of stage it+2 are issued into that buffer and the first fragments of stage it+1 are read - both
// under the MFMAs of the last k-step.  A load therefore has a whole stage of MFMAs to complete.
constexpr int kDlRow = 128;                  // bytes per LDS row
constexpr int kDlOp = kT * kDlRow;           // one operand, one stage (32 KiB)
constexpr int kDlStage = 2 * kDlOp;
constexpr int kDlLds = 133120;               // max(two stages, the epilogue's staging of 128 rows x 260 floats)
// A buffer load whose data goes to LDS (M0 = wavefront-uniform LDS byte address; lane l writes M0 + size * l) instead of
// registers.  Written as assembly on purpose: the compiler makes every later LDS read wait for ALL such loads
// it knows to be in flight (it cannot tell that they fill the other stage), which would serialise loads and MFMAs.
// The kernel orders them itself with explicit vmcnt waits and barriers.  Nothing else in these kernels uses M0.
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

template <typename TC, int TN, bool RAGGED>
__device__ __forceinline__ void gemm_dl_body(const NtArgs& g) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  constexpr int WN = 8 / TN, NW = 2 * WN, NLD = 32 / NW;       // loads per wavefront, operand and stage
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const int r = lane & 31, gq = lane >> 5;

  const TileCoord tc = tile_coord(g);
  if (!tc.live) return;
  const int M = tc.M, K = tc.K, m0 = tc.m0, n0 = tc.n0, z = tc.z, ks = tc.ks, ksplit = tc.ksplit;

  f32x16 acc[4][TN];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // K is a multiple of 8 (whole 16-byte chunks).  The last k-tile of a segment may hold fewer than 8 chunks: the lanes
  // that would fetch a chunk past K point outside the buffer descriptor for that tile and their slots arrive as zeros.
  const int ktiles = (K + kKB - 1) / kKB;
  const int tail_chunks = (K - (ktiles - 1) * kKB) >> 3;       // 1 .. 8 chunks in the last k-tile
  const bool ragged = RAGGED && tail_chunks < 8;              // RAGGED = false: the launcher saw K % 64 == 0
  const int nstage = ktiles * g.nseg;
  const int it0 = (int)((long)nstage * ks / ksplit);
  const int total = (int)((long)nstage * (ks + 1) / ksplit) - it0;

  // Loads.  Wavefront-load i of this wavefront fills rows 8 * (i * NW + wave) .. + 7 of an operand; lane l fills
  // slot l & 7 of row (l >> 3) of those, i.e. fetches k-chunk (l & 7) ^ swizzle(row).  Rows past the operand's end
  // point outside the buffer descriptor and arrive as zeros.
  // The order in which a work-group asks for the row groups of a stage is rotated by its place in the XCD's block of
  // tiles: the 4 (8) work-groups that share an A (B) panel each start with a different quarter (half) of it, so the
  // first request for a line - the one that has to fetch it from beyond L2 - goes out early in every work-group's
  // burst instead of all sharers asking for the same lines in the same order.
  const int rotA = tc.pos % kSupN, rotB = (tc.pos / kSupN) >> 1;
  unsigned voa[NLD], vob[NLD], lda_off[NLD], ldb_off[NLD];
  bool a_past[NLD], b_past[NLD];                                // this lane's chunk lies past K in a ragged last k-tile
  {
    const long a_rows_mem = g.a_rows ? g.a_phys_rows : M;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int ia = (i + rotA) % NLD, ib = (i + rotB) % NLD;
      lda_off[i] = ia * NW * 1024; ldb_off[i] = kDlOp + ib * NW * 1024;
      const int rl = (ia * NW + wave) * 8 + (lane >> 3), rlb = (ib * NW + wave) * 8 + (lane >> 3);
      const int chunk = (lane & 7) ^ ((rl >> 1) & 7), chunkb = (lane & 7) ^ ((rlb >> 1) & 7);
      long ra = m0 + rl;
      if (g.a_rows) ra = ra < M ? (long)g.a_rows[ra] : 0x7fffffffL; else if (ra >= M) ra = 0x7fffffffL;
      long rb = n0 + rlb;
      if (rb >= g.N) rb = 0x7fffffffL;
      const long oa = (ra * g.lda) * 2 + chunk * 16, ob = (rb * g.ldb) * 2 + chunkb * 16;
      voa[i] = (ra >= a_rows_mem || oa > 0x7ffffff0L) ? 0x7ffffff0u : (unsigned)oa;
      vob[i] = (rb >= g.N || ob > 0x7ffffff0L) ? 0x7ffffff0u : (unsigned)ob;
      a_past[i] = chunk >= tail_chunks; b_past[i] = chunkb >= tail_chunks;
    }
  }
  const long a_bytes = (long)(g.a_rows ? g.a_phys_rows : M) * g.lda * 2, b_bytes = (long)g.N * g.ldb * 2;
  const unsigned lds_base = (unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)lds;
  const int a_rec = a_bytes > 0x7fffffffL ? 0x7fffffff : (int)a_bytes, b_rec = b_bytes > 0x7fffffffL ? 0x7fffffff : (int)b_bytes;
  // Wavefront-loads of a stage are numbered 0 .. 2*NLD-1 (even: A, odd: B); `issue` enqueues numbers [first, last).
  auto issue = [&](int rel_it, int buf, int first, int last) __attribute__((always_inline)) {
    const int it = it0 + rel_it;
    const int seg = it / ktiles, kt = it - seg * ktiles;
    const u32x4 ra = make_rsrc(g.A + (g.sAz * z + g.sAseg * seg) * 2, (unsigned)a_rec);
    const u32x4 rb = make_rsrc(g.B + (g.sBz * z + g.sBseg * seg) * 2, (unsigned)b_rec);
    const unsigned dst = lds_base + buf * kDlStage + wave * 1024;
    const unsigned koff = kt * (kKB * 2);
    const bool cut = ragged && kt == ktiles - 1;
#pragma unroll
    for (int q = 0; q < 2 * NLD; ++q) {
      if (q < first || q >= last) continue;
      const int i = q >> 1;
      if (q & 1) load_to_lds_b128(rb, dst + ldb_off[i], (cut && b_past[i]) ? 0x7ffffff0u : vob[i], koff);
      else load_to_lds_b128(ra, dst + lda_off[i], (cut && a_past[i]) ? 0x7ffffff0u : voa[i], koff);
    }
  };
  constexpr int NQ = 2 * NLD;                               // wavefront-loads per stage and wavefront

  // Fragment reads: row (wm*128 + i*32 + r) of A / (wn*TN*32 + j*32 + r) of B, k-chunk 2*s + gq, which sits in
  // slot (2*s + gq) ^ ((r >> 1) & 7): one XOR with s * 32 per k-step on a per-lane base offset.
  const int fa_off = (wm * 128 + r) * kDlRow + ((gq ^ ((r >> 1) & 7)) * 16);
  const int fb_off = kDlOp + (wn * TN * 32 + r) * kDlRow + ((gq ^ ((r >> 1) & 7)) * 16);
  uint4 fa[2][4], fb[2][TN];
  auto read_frags = [&](int buf, int s, int c) __attribute__((always_inline)) {
    const char* base = lds + buf * kDlStage;
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[c][i] = *(const uint4*)(base + (fa_off ^ (s * 32)) + i * 32 * kDlRow);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[c][j] = *(const uint4*)(base + (fb_off ^ (s * 32)) + j * 32 * kDlRow);
  };

  // One k-step: the MFMAs of fragment buffer c.  With `ld`, the NQ wavefront-loads of stage `ld_it` go out between
  // them, one after every second MFMA, the rest behind the last.  (Spreading them over three k-steps measured
  // slower: the last ones then have too little time left; so did L2 prefetches of the coming stages.)
  auto kstep = [&](int c, bool ld, int ld_it, int ld_buf) __attribute__((always_inline)) {
    int q = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        acc[i][j] = mma(fa[c][i], fb[c][j], acc[i][j]);
        if (((i * TN + j) & 1) && q < NQ) {
          if (ld) issue(ld_it, ld_buf, q, q + 1);
          ++q;
        }
      }
    if (q < NQ && ld) issue(ld_it, ld_buf, q, NQ);
  };

  if (total > 0) {
    issue(0, 0, 0, NQ);
    __builtin_amdgcn_s_waitcnt(0x0f70);            // vmcnt(0)
    __syncthreads();
    if (total > 1) issue(1, 1, 0, NQ);
    read_frags(0, 0, 0);
  }
  for (int it = 0; it < total; ++it) {
    const int cur = it & 1;
    read_frags(cur, 1, 1);
    __builtin_amdgcn_sched_barrier(0);
    kstep(0, false, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(cur, 2, 0);
    __builtin_amdgcn_sched_barrier(0);
    kstep(1, false, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(cur, 3, 1);
    __builtin_amdgcn_sched_barrier(0);
    kstep(0, false, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
    // last k-step: stage it+1 must be in LDS and this stage's buffer free
    if (it + 1 < total) {
      __builtin_amdgcn_s_waitcnt(0x0070);          // vmcnt(0) lgkmcnt(0): own loads of stage it+1 landed, own reads of this stage done
      __syncthreads();
      read_frags(cur ^ 1, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    kstep(1, it + 2 < total, it + 2, cur);
    __builtin_amdgcn_sched_barrier(0);
  }
  store_tile<TC, TN>(acc, lds, g, M, m0, n0, z, ks, ksplit);
}

// ---------------------------------------------------------------------------------------------------------
// The weight-gradient shape, C[M,N] = sum_k A[k][m] B[k][n] with BOTH operands stored k-major (a row per frame:
// dW_x = X^T DZ, dW_h = Hprev^T DZ; float C), without transposing anything in memory.  Same tile, wavefront
// layout, stage pipeline and epilogue as gemm_dl_body; what differs is how a stage sits in LDS and how MFMA
// fragments leave it:
//   * a stage is 64 k-rows of 256 columns (512 bytes) per operand; a wavefront-load brings two whole rows (full
//     lines).  Row k may be any row of the operand in memory (`k_rows`: the packed list of real frames), looked up
//     one stage ahead of the load that needs it;
//   * MFMA wants, per lane, 8 consecutive k of ONE column, which in a k-major tile are 512 bytes apart.  The LDS
//     transpose read (8 bytes per lane, 16-bit elements) does that turn inside each group of 16 lanes: lane s
//     supplies the address of row kbase + s/4, columns cbase + 4*(s%4) .. +3, and lane l receives column cbase + l
//     of rows kbase .. kbase+3 (layout measured on the device).  Two such reads make one MFMA operand;
//   * the four rows a 16-lane group reads together lie 512 bytes apart, i.e. in the same banks; so the 64-byte
//     blocks of row k are stored XORed with k % 4 (again by choosing which global chunk a loading lane fetches).
template <typename TC>
__device__ __forceinline__ void gemm_tn_body(const NtArgs& g) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  constexpr int TN = 2, WN = 4, NW = 8, NLD = 4;               // 8 wavefronts of 128x64; 4 wavefront-loads per operand
  constexpr int kRow = 512;                                    // bytes per k-row of a stage (256 columns)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;

  const TileCoord tc = tile_coord(g);
  if (!tc.live) return;
  const int M = tc.M, K = tc.K, m0 = tc.m0, n0 = tc.n0, z = tc.z, ks = tc.ks, ksplit = tc.ksplit;

  f32x16 acc[4][TN];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int nstage = (K + kKB - 1) / kKB;                      // rows past K arrive as zeros
  const int it0 = (int)((long)nstage * ks / ksplit);
  const int total = (int)((long)nstage * (ks + 1) / ksplit) - it0;

  // Loads.  Wavefront-load i of this wavefront fills k-rows 2*(i*NW + wave) and +1 of the stage; lane l fills
  // 16-byte slot l % 32 of row l / 32, i.e. fetches column chunk (l % 32) ^ 4*(k % 4).
  const int krow_in_stage = 2 * wave + (lane >> 5);            // + 2*NW*i
  const int chunk = (lane & 31) ^ (4 * (krow_in_stage & 3));   // 2*NW*i is a multiple of 4
  const bool a_col_ok = m0 + chunk * 8 < M, b_col_ok = n0 + chunk * 8 < g.N;
  const long a_col = ((long)m0 + chunk * 8) * 2, b_col = ((long)n0 + chunk * 8) * 2;
  const long a_rows_mem = g.k_rows ? g.k_phys_rows : K;
  const long a_bytes = a_rows_mem * g.lda * 2, b_bytes = a_rows_mem * g.ldb * 2;
  const unsigned a_rec = a_bytes > 0x7fffffffL ? 0x7fffffffu : (unsigned)a_bytes, b_rec = b_bytes > 0x7fffffffL ? 0x7fffffffu : (unsigned)b_bytes;
  const u32x4 ra = make_rsrc(g.A + g.sAz * z * 2, a_rec), rb = make_rsrc(g.B + g.sBz * z * 2, b_rec);
  const unsigned lds_base = (unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)lds;
  // Work-groups that run side by side on an XCD all want the same 64 frame rows of a stage; each starts its burst
  // of wavefront-loads with a different quarter of them, so that the first request for a line goes out early in
  // some work-group's burst.
  const int rot = (int)(blockIdx.x >> 3) % NLD;
  // Memory rows of the stage whose loads go out next.  A wavefront-load covers rows k and k+1 of the list, the same
  // for all lanes of a half, so the look-up is a scalar load of two consecutive entries - written as assembly and
  // waited for by hand (together with the operand loads, before the barrier of the next stage): the compiler would
  // wait for a look-up it knows about right where it is issued, and with vector loads that wait would also
  // cover every operand load in flight.  The list must be readable up to the next multiple of 64 entries.
  typedef __attribute__((ext_vector_type(2))) int i32x2;
  i32x2 prow2[NLD];
  int pk0 = 0;
  auto lookup = [&](int rel_it) __attribute__((always_inline)) {
    pk0 = (it0 + rel_it) * kKB + krow_in_stage;                // k of wavefront-load 0 for this lane; load i adds 2 * NW * i
    if (g.k_rows && rel_it < total) {
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        const int* p = g.k_rows + (long)(it0 + rel_it) * kKB + 2 * (NW * ((i + rot) % NLD) + wave);
        asm volatile("s_load_dwordx2 %0, %1, 0x0" : "=s"(prow2[i]) : "s"(p) : "memory");
      }
    }
  };
  auto row_of = [&](int i) __attribute__((always_inline)) {
    return g.k_rows ? ((lane >> 5) ? prow2[i][1] : prow2[i][0]) : pk0 + 2 * NW * ((i + rot) % NLD);
  };
  auto issue = [&](int buf, int first, int last) __attribute__((always_inline)) {
    const unsigned dst = lds_base + buf * kDlStage + wave * 1024;
#pragma unroll
    for (int q = 0; q < 2 * NLD; ++q) {
      if (q < first || q >= last) continue;
      const int i = q >> 1;
      const int row = row_of(i), ir = (i + rot) % NLD;
      const bool row_ok = pk0 + 2 * NW * ir < K && row >= 0 && row < a_rows_mem;
      if (q & 1) {
        const long o = (long)row * g.ldb * 2 + b_col;
        load_to_lds_b128(rb, dst + kDlOp + ir * NW * 1024, (row_ok && b_col_ok && o <= 0x7ffffff0L) ? (unsigned)o : 0x7ffffff0u, 0);
      } else {
        const long o = (long)row * g.lda * 2 + a_col;
        load_to_lds_b128(ra, dst + ir * NW * 1024, (row_ok && a_col_ok && o <= 0x7ffffff0L) ? (unsigned)o : 0x7ffffff0u, 0);
      }
    }
  };
  constexpr int NQ = 2 * NLD;

  // Fragment reads (see the head of this function).  Lane L = 32*kg + 16*grp + l: source row kg*8 + l/4 (+4 for the
  // second read) of the 16-row k-step, columns block*32 + grp*16 + 4*(l%4) .. +3, 64-byte blocks XORed with row % 4.
  const int l16 = lane & 15, grp = (lane >> 4) & 1, kg = lane >> 5;
  const int fr_row = (kg * 8 + (l16 >> 2)) * kRow, fr_sw = (l16 >> 2) & 3, fr_low = grp * 32 + (l16 & 3) * 8;
  int fa_off[4], fb_off[TN];
#pragma unroll
  for (int i = 0; i < 4; ++i) fa_off[i] = fr_row + ((((wm * 4 + i) ^ fr_sw) & 7) << 6) + fr_low;          // column block wm*4 + i of 8
#pragma unroll
  for (int j = 0; j < TN; ++j) fb_off[j] = kDlOp + fr_row + ((((wn * TN + j) ^ fr_sw) & 7) << 6) + fr_low;
  typedef __attribute__((ext_vector_type(4))) short s16x4;
  uint4 fa[2][4], fb[2][TN];
  auto tr_read = [&](const char* p) __attribute__((always_inline)) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p + 4 * kRow));
    const uint2 l2 = __builtin_bit_cast(uint2, lo), h2 = __builtin_bit_cast(uint2, hi);
    return make_uint4(l2.x, l2.y, h2.x, h2.y);
  };
  auto read_frags = [&](int buf, int s, int c) __attribute__((always_inline)) {
    const char* base = lds + buf * kDlStage + s * 16 * kRow;
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[c][i] = tr_read(base + fa_off[i]);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[c][j] = tr_read(base + fb_off[j]);
  };
  auto kstep = [&](int c, bool ld, int ld_buf) __attribute__((always_inline)) {
    int q = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        acc[i][j] = mma(fa[c][i], fb[c][j], acc[i][j]);
        if (((i * TN + j) & 1) && q < NQ) {
          if (ld) issue(ld_buf, q, q + 1);
          ++q;
        }
      }
    if (q < NQ && ld) issue(ld_buf, q, NQ);
  };

  if (total > 0) {
    lookup(0);
    __builtin_amdgcn_s_waitcnt(0xc07f);            // lgkmcnt(0): the look-up
    issue(0, 0, NQ);
    lookup(1);
    __builtin_amdgcn_s_waitcnt(0x0070);            // vmcnt(0) lgkmcnt(0)
    __syncthreads();
    if (total > 1) issue(1, 0, NQ);
    lookup(2);
    read_frags(0, 0, 0);
  }
  for (int it = 0; it < total; ++it) {
    const int cur = it & 1;
    read_frags(cur, 1, 1);
    __builtin_amdgcn_sched_barrier(0);
    kstep(0, false, 0);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(cur, 2, 0);
    __builtin_amdgcn_sched_barrier(0);
    kstep(1, false, 0);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(cur, 3, 1);
    __builtin_amdgcn_sched_barrier(0);
    kstep(0, false, 0);
    __builtin_amdgcn_sched_barrier(0);
    if (it + 1 < total) {
      __builtin_amdgcn_s_waitcnt(0x0070);          // vmcnt(0) lgkmcnt(0): own loads of stage it+1 (and row look-ups) landed, own reads done
      __syncthreads();
      read_frags(cur ^ 1, 0, 0);
    }
    __builtin_amdgcn_sched_barrier(0);
    kstep(1, it + 2 < total, cur);                 // loads of stage it+2 (rows looked up during the previous stage)
    __builtin_amdgcn_sched_barrier(0);
    lookup(it + 3);
  }
  store_tile<TC, TN>(acc, lds, g, M, m0, n0, z, ks, ksplit);
}
__global__ __launch_bounds__(512, 1) void gemm_tn8_f32_kernel(NtArgs g) { gemm_tn_body<float>(g); }

// (kernels with literal launch bounds: a bound that depends on a template parameter loses the host-side stub)
template <bool RAGGED> __global__ __launch_bounds__(512, 1) void gemm_dl8_f32_kernel(NtArgs g) { gemm_dl_body<float, 2, RAGGED>(g); }
template <bool RAGGED> __global__ __launch_bounds__(512, 1) void gemm_dl8_bf16_kernel(NtArgs g) { gemm_dl_body<uint16_t, 2, RAGGED>(g); }

// C[z][m][n] (+)= sum over the K ranges of parts[z][range][m][n]  (parts in the layout of C, one after the other)
__global__ void sum_parts_kernel(const float* parts, float* C, int M, int N, long ldc, long sCz, long sPart, int ksplit, int accumulate,
                                 long total) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int n = (int)(idx % N);
  const long rest = idx / N;
  const int m = (int)(rest % M);
  const long z = rest / M;
  const long off = (long)m * ldc + n;
  float v = accumulate ? C[z * sCz + off] : 0.f;
  for (int ks = 0; ks < ksplit; ++ks) v += __builtin_nontemporal_load(parts + (z * ksplit + ks) * sPart + off);
  C[z * sCz + off] = v;
}

// The same for a bfloat16 C without z: C[rows[m]][n] = sum over the K ranges of parts[range][m][n], m below *m_dev
// when given (the rows above it were never computed); four columns per lane.
__global__ void sum_parts_bf16_kernel(const float* parts, uint16_t* C, int M, int N, long ldc, long sPart, int ksplit, const int* c_rows,
                                      const int* m_dev) {
  const int nq = (N + 3) / 4;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const int m = (int)(idx / nq), n = (int)(idx % nq) * 4;
  if (m >= (m_dev ? min(M, *m_dev) : M)) return;
  const long src = (long)m * ldc + n, dst = (long)(c_rows ? c_rows[m] : m) * ldc + n;
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  const bool whole = n + 3 < N && ldc % 4 == 0;
  for (int ks = 0; ks < ksplit; ++ks) {
    const float* p = parts + ks * sPart + src;
    if (whole) {
      typedef __attribute__((ext_vector_type(4))) float f32x4_;
      const f32x4_ q = __builtin_nontemporal_load((const f32x4_*)p);
      v[0] += q[0]; v[1] += q[1]; v[2] += q[2]; v[3] += q[3];
    } else {
      for (int k = 0; k < 4; ++k)
        if (n + k < N) v[k] += p[k];
    }
  }
  if (whole && (((uintptr_t)C & 7u) == 0)) {
    uint2 o;
    o.x = f2bf_bits(v[0]) | ((unsigned)f2bf_bits(v[1]) << 16);
    o.y = f2bf_bits(v[2]) | ((unsigned)f2bf_bits(v[3]) << 16);
    *(uint2*)(C + dst) = o;
  } else {
    for (int k = 0; k < 4; ++k)
      if (n + k < N) C[dst + k] = f2bf_bits(v[k]);
  }
}

// dst[c][r] = keep(r) ? src[r][c] : 0 for r < R, c < C ; dst rows are padded with zeros up to ldd.
// keep(r): rows of src are frames (t = r / Bt, b = r % Bt), kept iff lens == NULL or t < lens[b].
// With `cidx` (compact index of every frame, -1 for padded frames) the kept frames are packed instead:
// dst[c][cidx[r]] = src[r][c]; columns past the last kept frame are left to zero_tail_kernel.
__global__ __launch_bounds__(256) void transpose_kernel(const uint16_t* src, uint16_t* dst, int R, int C, long lds_, long ldd,
                                                        long s_src, long s_dst, const int* lens, int Bt, int T, const int* cidx) {
  __shared__ uint16_t tile[64][66];
  src += s_src * blockIdx.z;
  dst += s_dst * blockIdx.z;
  const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int rr = r0 + ty + 4 * i, cc = c0 + tx;
    uint16_t v = 0;
    if (rr < R && cc < C) {
      bool keep = true;
      if (lens) {
        const int t = rr / Bt, b = rr - t * Bt;
        int L = lens[b];
        L = L < 0 ? 0 : (L > T ? T : L);
        keep = t < L;
      }
      if (cidx) keep = cidx[rr] >= 0;
      if (keep) v = src[(long)rr * lds_ + cc];
    }
    tile[ty + 4 * i][tx] = v;
  }
  __syncthreads();
  if (cidx) {
    const int rr = r0 + tx;
    const int dcol = rr < R ? cidx[rr] : -1;
    if (dcol < 0) return;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int cc = c0 + ty + 4 * i;
      if (cc < C) dst[(long)cc * ldd + dcol] = tile[tx][ty + 4 * i];
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int cc = c0 + ty + 4 * i, rr = r0 + tx;
    if (cc < C && rr < ldd) dst[(long)cc * ldd + rr] = tile[tx][ty + 4 * i];
  }
}

// Same operation for 16-byte aligned operands (C, lds_, ldd, strides all multiples of 8 elements), written around
// the destination: a work-group produces 64 consecutive destination columns (packed frames when `fidx` maps them
// back to source rows) for 256 source columns.  Source rows are read as 16-byte vectors, the tile is turned in
// LDS, and every destination row receives one aligned 128-byte run.  Columns from the last kept frame up to
// the next multiple of 64 (packed) or up to ldd (not packed) are written as zeros here.
__global__ __launch_bounds__(256) void transpose_frames_kernel(const uint16_t* src, uint16_t* dst, int R, int C, long lds_, long ldd,
                                                               long s_src, long s_dst, const int* lens, int Bt, int T,
                                                               const int* fidx, const int* count) {
  __shared__ __attribute__((aligned(16))) uint16_t tile[64][264];
  src += s_src * blockIdx.z;
  dst += s_dst * blockIdx.z;
  const int tid = threadIdx.x;
  const int f0 = blockIdx.x * 64, c0 = blockIdx.y * 256;
  const int nkeep = fidx ? min(count[0], R) : R;
  if (fidx && f0 >= count[1]) return;            // past the zeroed tail of the packed columns
  {
    const int cv = tid & 31, fr = tid >> 5;
    const int col = c0 + cv * 8;
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
      const int f = pass * 8 + fr, c = f0 + f;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (c < nkeep && col < C) {
        const int row = fidx ? fidx[c] : c;
        bool keep = row >= 0 && row < R;
        if (keep && lens && !fidx) {
          const int t = row / Bt, b = row - t * Bt;
          int L = lens[b];
          L = L < 0 ? 0 : (L > T ? T : L);
          keep = t < L;
        }
        if (keep) v = *(const uint4*)(src + (long)row * lds_ + col);
      }
      *(uint4*)&tile[f][cv * 8] = v;
    }
  }
  __syncthreads();
  {
    const int g = tid & 7, cl = tid >> 3;          // 8 lanes cover the 64 columns (128 bytes) of one destination row
    const int c = f0 + g * 8;
    if (c >= ldd) return;
#pragma unroll
    for (int pass = 0; pass < 8; ++pass) {
      const int sc = cl + 32 * pass;               // source column inside the tile
      if (c0 + sc >= C) break;
      uint16_t e[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) e[k] = tile[g * 8 + k][sc];
      uint4 o;
      o.x = e[0] | ((unsigned)e[1] << 16); o.y = e[2] | ((unsigned)e[3] << 16);
      o.z = e[4] | ((unsigned)e[5] << 16); o.w = e[6] | ((unsigned)e[7] << 16);
      *(uint4*)(dst + (long)(c0 + sc) * ldd + c) = o;
    }
  }
}

// dst[row][count[0] .. count[1]) = 0 for every row: the k tail of packed operands (count[1] = count[0] rounded up to 64)
__global__ void zero_tail_kernel(uint16_t* dst, long rows, long ldd, const int* count) {
  const int k0 = count[0], k1 = count[1];
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const long row = idx >> 6;
  const int k = k0 + (int)(idx & 63);
  if (row < rows && k < k1 && k < ldd) dst[row * ldd + k] = 0;
}

// Frame map of a batch of end-padded sequences: frame (t, b) is kept iff t < lens[b].  Kept frames are numbered
// in (t, b) order: cidx[t*B + b] = that number or -1, fidx[number] = t*B + b, count[0] = how many are kept,
// count[1] = count[0] rounded up to a multiple of 64.  One wavefront per time step.
__global__ __launch_bounds__(256) void frame_map_kernel(const int* lens, int T, int B, int* cidx, int* fidx, int* count) {
  frame_map_body(blockIdx.x, lens, T, B, cidx, fidx, count);
}

// dst[r][c] = src[r][c] for c < C, zero for C <= c < ldd  (rows made 16-byte aligned)
__global__ void pad_rows_kernel(const uint16_t* src, uint16_t* dst, long R, int C, int ldd) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= R * ldd) return;
  const long rr = idx / ldd;
  const int cc = (int)(idx - rr * ldd);
  dst[idx] = cc < C ? src[rr * C + cc] : (uint16_t)0;
}

}  // namespace

bool gemm_nt_ok(const GemmArgs& g) {
  const auto a16 = [](const void* p) { return ((uintptr_t)p & 15u) == 0; };
  const long lim = 0x7fffff00L;     // operands are addressed with 32-bit byte offsets
  if ((long)g.M * g.lda * 2 > lim || (long)g.N * g.ldb * 2 > lim) return false;
  if (g.k_dev && g.K % 64 != 0) return false;     // a device-resident K counts whole 64-wide stages
  return g.in_bf16 && g.a_kcontig && g.b_kcontig && !g.lens && g.K % 8 == 0 && g.lda % 8 == 0 && g.ldb % 8 == 0 &&
         g.sAz % 8 == 0 && g.sBz % 8 == 0 && g.sAseg % 8 == 0 && g.sBseg % 8 == 0 && a16(g.A) && a16(g.B);
}

// second half of a product whose K ranges stored their parts side by side: C (+)= their sum
static hipError_t sum_parts(const NtArgs& a, hipStream_t s) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !a.parts) return e;
  const long total = (long)a.nz * a.M * a.N;
  hipLaunchKernelGGL(sum_parts_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, a.parts, (float*)a.C, a.M, a.N, a.ldc, a.sCz, a.sPart, a.ksplit,
                     a.accumulate, total);
  return hipGetLastError();
}

bool gemm_tn_ok(const GemmArgs& g) {
  const auto a16 = [](const void* p) { return ((uintptr_t)p & 15u) == 0; };
  const long lim = 0x7fffff00L;     // operands are addressed with 32-bit byte offsets
  const long rows = g.k_rows ? g.k_phys_rows : g.K;
  if (rows * g.lda * 2 > lim || rows * g.ldb * 2 > lim) return false;
  return g.in_bf16 && !g.out_bf16 && !g.a_kcontig && !g.b_kcontig && !g.lens && g.nseg == 1 && !g.a_rows && !g.c_rows && !g.m_dev &&
         g.lda % 8 == 0 && g.ldb % 8 == 0 && g.sAz % 8 == 0 && g.sBz % 8 == 0 && a16(g.A) && a16(g.B);
}

hipError_t launch_gemm_tn(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0 || g.nz <= 0) return hipSuccess;
  NtArgs a = {};
  a.A = (const char*)g.A; a.B = (const char*)g.B; a.C = g.C; a.bias = g.bias;
  a.M = g.M; a.N = g.N; a.K = g.K; a.lda = g.lda; a.ldb = g.ldb; a.ldc = g.ldc;
  a.sAz = g.sAz; a.sBz = g.sBz; a.sCz = g.sCz; a.sbiasz = g.sbiasz; a.nz = g.nz; a.nseg = 1;
  a.accumulate = g.accumulate; a.k_dev = g.k_dev; a.k_rows = g.k_rows; a.k_phys_rows = g.k_phys_rows;
  a.ksplit = g.ksplit > 1 ? g.ksplit : 1;
  a.parts = a.ksplit > 1 ? g.parts : nullptr; a.sPart = (long)g.M * g.ldc;
  const int sups = cdiv(cdiv(g.M, kT), kSupM) * cdiv(cdiv(g.N, kT), kSupN);
  a.blocked = sups >= 32 ? 1 : 0;
  const int tiles = a.blocked ? cdiv(sups, 8) * 8 * kSupM * kSupN : cdiv(g.M, kT) * cdiv(g.N, kT);
  static std::atomic<unsigned long long> attr_set{0};
  const hipError_t ea = once_per_device(attr_set, [] {
    return hipFuncSetAttribute((const void*)gemm_tn8_f32_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kDlLds);
  });
  if (ea != hipSuccess) return ea;
  hipLaunchKernelGGL(gemm_tn8_f32_kernel, dim3(tiles, g.nz * a.ksplit), dim3(512), kDlLds, s, a);
  return sum_parts(a, s);
}

hipError_t launch_gemm_nt(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0 || g.nz <= 0) return hipSuccess;
  NtArgs a;
  a.A = (const char*)g.A; a.B = (const char*)g.B; a.C = g.C; a.bias = g.bias;
  a.M = g.M; a.N = g.N; a.K = g.K; a.lda = g.lda; a.ldb = g.ldb; a.ldc = g.ldc;
  a.sAz = g.sAz; a.sBz = g.sBz; a.sCz = g.sCz; a.sbiasz = g.sbiasz; a.nz = g.nz;
  a.nseg = g.nseg; a.sAseg = g.sAseg; a.sBseg = g.sBseg; a.accumulate = g.accumulate;
  a.a_rows = g.a_rows; a.c_rows = g.c_rows; a.m_dev = g.m_dev; a.k_dev = g.k_dev; a.a_phys_rows = g.a_phys_rows;
  // bfloat16 output over K ranges: float parts (packed rows) from the float kernel, then one pass that adds them,
  // rounds once and scatters the rows; needs the direct-to-LDS kernel (segments and ranges share its stage counter)
  const bool dl = !g.k_dev || g.K % kKB == 0;
  const bool parts_bf16 = g.out_bf16 && g.ksplit > 1 && g.parts && dl && g.nz == 1 && !g.accumulate && !g.bias;
  a.ksplit = (g.ksplit > 1 && ((!g.out_bf16 && g.nseg == 1) || parts_bf16)) ? g.ksplit : 1;
  a.parts = a.ksplit > 1 && (!g.c_rows || parts_bf16) ? g.parts : nullptr; a.sPart = (long)g.M * g.ldc;
  // the blocked raster pays when every XCD gets several blocks; with few tiles it would leave XCDs idle
  const int sups = cdiv(cdiv(g.M, kT), kSupM) * cdiv(cdiv(g.N, kT), kSupN);
  a.blocked = sups >= 32 ? 1 : 0;
  const int tiles = a.blocked ? cdiv(sups, 8) * 8 * kSupM * kSupN : cdiv(g.M, kT) * cdiv(g.N, kT);
  // operands go straight into LDS; K any multiple of 8 (a device-resident K is a multiple of 64 by contract, and so
  // must then be the host's bound on it)
  if (dl) {
    static std::atomic<unsigned long long> dl_attr_set{0};
    const hipError_t ea = once_per_device(dl_attr_set, [] {
      for (const void* k : {(const void*)gemm_dl8_f32_kernel<false>, (const void*)gemm_dl8_f32_kernel<true>,
                            (const void*)gemm_dl8_bf16_kernel<false>, (const void*)gemm_dl8_bf16_kernel<true>}) {
        const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kDlLds);
        if (e != hipSuccess) return e;
      }
      return hipSuccess;
    });
    if (ea != hipSuccess) return ea;
    const dim3 grid(tiles, g.nz * a.ksplit);
    const bool ragged = g.K % kKB != 0, bf = g.out_bf16 && !parts_bf16;
    if (bf && ragged) hipLaunchKernelGGL(gemm_dl8_bf16_kernel<true>, grid, dim3(512), kDlLds, s, a);
    else if (bf) hipLaunchKernelGGL(gemm_dl8_bf16_kernel<false>, grid, dim3(512), kDlLds, s, a);
    else if (ragged) hipLaunchKernelGGL(gemm_dl8_f32_kernel<true>, grid, dim3(512), kDlLds, s, a);
    else hipLaunchKernelGGL(gemm_dl8_f32_kernel<false>, grid, dim3(512), kDlLds, s, a);
    if (parts_bf16) {
      const hipError_t e = hipGetLastError();
      if (e != hipSuccess) return e;
      const long total = (long)a.M * ((a.N + 3) / 4);
      hipLaunchKernelGGL(sum_parts_bf16_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, a.parts, (uint16_t*)a.C, a.M, a.N, a.ldc, a.sPart,
                         a.ksplit, a.c_rows, a.m_dev);
      return hipGetLastError();
    }
    return sum_parts(a, s);
  }
  return hipErrorInvalidValue;       // unreachable: gemm_nt_ok() refuses a device-resident K whose bound is not a multiple of 64
}


hipError_t launch_transpose(const void* src, void* dst, int R, int C, long ld_src, long ld_dst, int nz, long s_src, long s_dst,
                            const int* lens, int Bt, int T, hipStream_t s, const int* cidx, const int* fidx, const int* count) {
  if (R <= 0 || C <= 0 || nz <= 0) return hipSuccess;
  const bool aligned = C % 8 == 0 && ld_src % 8 == 0 && ld_dst % 8 == 0 && s_src % 8 == 0 && s_dst % 8 == 0 &&
                       ((uintptr_t)src & 15u) == 0 && ((uintptr_t)dst & 15u) == 0;
  if (aligned) {
    hipLaunchKernelGGL(transpose_frames_kernel, dim3(cdiv(ld_dst, 64), cdiv(C, 256), nz), dim3(256), 0, s, (const uint16_t*)src,
                       (uint16_t*)dst, R, C, ld_src, ld_dst, s_src, s_dst, lens, Bt, T, cidx ? fidx : nullptr, count);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(transpose_kernel, dim3(cdiv(ld_dst, 64), cdiv(C, 64), nz), dim3(256), 0, s, (const uint16_t*)src,
                     (uint16_t*)dst, R, C, ld_src, ld_dst, s_src, s_dst, lens, Bt, T, cidx);
  if (cidx) {                           // packed columns: zero from the last kept frame to the next multiple of 64
    for (int z = 0; z < nz; ++z)
      hipLaunchKernelGGL(zero_tail_kernel, dim3(cdiv((long)C * 64, 256)), dim3(256), 0, s, (uint16_t*)dst + s_dst * z, (long)C,
                         ld_dst, count);
  }
  return hipGetLastError();
}

hipError_t launch_frame_map(const int* lens, int T, int B, int* cidx, int* fidx, int* count, hipStream_t s) {
  if (T <= 0 || B <= 0) return hipSuccess;
  hipLaunchKernelGGL(frame_map_kernel, dim3(cdiv(T, 4)), dim3(256), 0, s, lens, T, B, cidx, fidx, count);
  return hipGetLastError();
}

hipError_t launch_pad_rows(const void* src, void* dst, long R, int C, int ld_dst, hipStream_t s) {
  if (R <= 0) return hipSuccess;
  const long total = R * ld_dst;
  hipLaunchKernelGGL(pad_rows_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, (const uint16_t*)src, (uint16_t*)dst, R, C, ld_dst);
  return hipGetLastError();
}

}  // namespace lstm
