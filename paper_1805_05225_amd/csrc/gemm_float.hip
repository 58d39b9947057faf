// The hoisted products in float storage (paper Sec. 3: work taken out of the recurrent loop), float in, float out,
// float MFMA (16x16x4), operands used as they lie in memory:
//     <AK, BK> = <true,  false>   Zx   = X W_x + b      A[M][K] rows of frames,  B[K][N]
//                <true,  true >   dX   = DZ W_x^T       A[M][K],                 B[N][K]     (summed over `nseg` directions)
//                <false, false>   dW   = X^T DZ         A[K][M], B[K][N]: a row per frame in both
//     C[z][M][N] (+)= sum_seg sum_k A . B  (+ bias[N])
//
// Tile 128 x 128, four wavefronts of 64 x 64 (4 x 4 MFMA blocks), k advances 32 per stage, two stages in LDS
// (65 KiB: two work-groups per compute unit, so one's barrier and waits hide behind the other's MFMAs).  The operands
// go from global memory straight into LDS (16 bytes per lane, no staging registers, no LDS store instructions); a
// wavefront-load writes 1 KiB, lane l its bytes 16 l .., and what a lane fetches is chosen so that the fragment
// reads meet no bank conflicts:
//   * k-major operand (a memory row is one k): a float MFMA wants ONE value per lane, element (k-row = lane / 16,
//     column = lane % 16) of a 4 x 16 block - 16 lanes reading 16 consecutive floats, no transposition needed.  A
//     stage is 16 pieces of 1 KiB + 16 bytes; piece p holds k-rows p and p + 16 of the stage (512 bytes each).
//   * k-contiguous operand (a memory row is a row of the tile): a stage is 128 rows of 128 bytes, unpadded; the
//     16-byte slot s of row r holds k-chunk s ^ ((r >> 1) & 7).  A lane reads 16 bytes: four consecutive k of its row.
// Since a k-contiguous lane gets four consecutive k at once, the MFMAs walk k in this order: step s (0..3) of group
// G (0..1) of a stage multiplies, in its lane group q (0..3), k = 16 G + 4 q + s.  Both operands follow it, so every
// k meets its partner; a k-major fragment of that step reads k-rows 16 G + s + {0, 4, 8, 12}: four pieces that lie
// 4 x 1040 bytes apart, 16 banks from one another.
// The MFMA takes the B fragment (columns n) as its row operand and the A fragment as its column operand: a lane then
// holds four CONSECUTIVE n of one row m of C and stores them as 16 bytes.
// Rows of a k-contiguous A (and of C) may be mapped (`a_rows`, `c_rows`, `m_dev`: the packed list of real frames), as
// may the k-rows of a k-major pair (`k_rows`, `k_dev`), looked up one stage ahead.
#include "common.h"
#include <algorithm>

namespace lstm {
namespace {

constexpr int kTile = 128, kKS = 32;
constexpr int kPiece = 1024 + 16;                // k-major: bytes per piece (k-rows p and p + 16, padding)
constexpr int kOp = 16 * kPiece;                 // one operand, one stage (a k-contiguous one uses 16 KiB of it)
constexpr int kStage = 2 * kOp;
constexpr int kLds = 2 * kStage;                 // 66 560
constexpr int kBufFlags = 0x00020000;            // raw buffer descriptor word 3 for gfx9-family devices
constexpr unsigned kParked = 0x7ffffff0u;        // offset outside every descriptor: the load returns zeros

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;

struct FArgs {
  const char* A; const char* B; float* C; const float* bias;
  int M, N, K;
  long lda, ldb, ldc;                            // elements
  long sAz, sBz, sCz, sbiasz;
  int nseg; long sAseg, sBseg;
  int accumulate;
  const int* a_rows; const int* c_rows; int a_phys_rows; const int* m_dev;
  const int* k_rows; int k_phys_rows; const int* k_dev;
  int ksplit;                                    // > 1: every K range adds its part to C atomically ...
  float* parts; long sPart;                      // ... or (ksplit == 8 only) stores it at parts + (z * 8 + range) * sPart, rows
                                                 // packed, and range r is worked on by XCD r alone
  int tiles_m, tiles_n, per_xcd;
  unsigned a_bytes, b_bytes;                     // extent of one segment of A / B in memory
};

// A buffer load whose data goes to LDS (M0 = wavefront-uniform LDS byte address; lane l writes M0 + 16 l).  Written as
// assembly so that the compiler does not make later LDS reads wait for loads that fill the other stage; the kernel
// orders them with an explicit vmcnt(0) and the barrier of every stage.  Nothing else here uses M0.
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

template <bool AK, bool BK>
__device__ __forceinline__ void gemm_float_body(const FArgs& g) {
  static_assert(AK || !BK, "a k-major A with a k-contiguous B is not a product of the layer");
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  // Work-groups are dealt to the eight XCDs round-robin: an XCD takes a run of consecutive tiles, column-major, i.e.
  // all row tiles of a few tile columns - the A panels and those few B panels are what its L2 has to hold.
  // With `parts` (few tiles, long K: dX) every XCD takes ALL tiles for one eighth of K instead: its L2 then holds that
  // eighth of B for good and streams that eighth of A once, and no operand byte is fetched by two XCDs.  The tiles
  // of one row panel (same rows of A) are neighbours in launch order, so they run side by side.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const bool by_range = g.parts != nullptr;
  const int t = by_range ? slot : xcd * g.per_xcd + slot;
  if ((!by_range && slot >= g.per_xcd) || t >= g.tiles_m * g.tiles_n) return;
  const int m0 = (by_range ? t / g.tiles_n : t % g.tiles_m) * kTile, n0 = (by_range ? t % g.tiles_n : t / g.tiles_m) * kTile;
  const int M = g.m_dev ? min(g.M, *g.m_dev) : g.M;              // the grid is sized for g.M; surplus tiles leave at once
  if (m0 >= M) return;
  const int ksplit = g.ksplit > 1 ? g.ksplit : 1;
  const int z = by_range ? blockIdx.y : blockIdx.y / ksplit, ks = by_range ? xcd : blockIdx.y - z * ksplit;
  const int K = g.k_dev ? min(g.K, *g.k_dev) : g.K;
  const int sps = max((K + kKS - 1) / kKS, 1);                   // stages per segment; what lies past K arrives as zeros
  const int nstage = K > 0 ? sps * g.nseg : 0;
  const int it0 = (int)((long)nstage * ks / ksplit);
  const int total = (int)((long)nstage * (ks + 1) / ksplit) - it0;
  if (total <= 0 && !by_range && (ksplit > 1 || g.accumulate)) return;        // nothing to add

  const unsigned lds_base = (unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)lds;
  // ---- loads ----
  // k-major operand: wavefront-load i of this wavefront writes piece p = 4 wave + i; its lower 32 lanes fetch k-row p
  // of the stage, the upper 32 k-row p + 16; lane l fetches columns 4 (l % 32) .. + 3 of the tile.
  const int half = lane >> 5, chunk32 = lane & 31;
  const int k_lane = 16 * half + 4 * wave;                       // k of wavefront-load 0 inside a stage; load i adds i
  const long krows_mem = g.k_rows ? g.k_phys_rows : K;
  const bool am_col_ok = m0 + chunk32 * 4 < g.M, bm_col_ok = n0 + chunk32 * 4 < g.N;
  const unsigned am_col = (unsigned)(m0 + chunk32 * 4) * 4u, bm_col = (unsigned)(n0 + chunk32 * 4) * 4u;
  // k-contiguous operand: wavefront-load i writes tile rows 32 wave + 8 i .. + 7; lane l fills slot l % 8 of row l / 8
  // of those, i.e. fetches k-chunk (l % 8) ^ ((row >> 1) & 7).  The rows do not change from stage to stage.
  unsigned ak_row[4], bk_row[4];                                 // byte offset of the lane's row (kParked: no such row)
  int ak_kc[4], bk_kc[4];                                        // first k of the chunk the lane fetches, within a stage
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 32 * wave + 8 * i + (lane >> 3);
    const int kc = 4 * ((lane & 7) ^ ((r >> 1) & 7));
    ak_kc[i] = bk_kc[i] = kc;
    ak_row[i] = bk_row[i] = kParked;
    if (AK) {
      long ra = m0 + r;
      const long rows_mem = g.a_rows ? g.a_phys_rows : g.M;
      if (ra < M) {
        if (g.a_rows) ra = g.a_rows[ra];
        if (ra >= 0 && ra < rows_mem) ak_row[i] = (unsigned)(ra * g.lda * 4);
      }
    }
    if (BK) {
      const long rb = n0 + r;
      if (rb < g.N) bk_row[i] = (unsigned)(rb * g.ldb * 4);
    }
  }
  auto lookup = [&](int rel_it) -> int4 {                        // memory rows of the four k this lane fetches (k-major pair)
    const int it = it0 + rel_it, seg = it / sps;
    const int k = (it - seg * sps) * kKS + k_lane;
    if (!AK && !BK && g.k_rows && rel_it < total) return *(const int4*)(g.k_rows + k);   // (readable up to a multiple of 64)
    return make_int4(k, k + 1, k + 2, k + 3);
  };
  auto issue = [&](int rel_it, int buf, const int4& rows) __attribute__((always_inline)) {
    const int it = it0 + rel_it, seg = it / sps;
    const int k0 = (it - seg * sps) * kKS;
    const u32x4 ra = make_rsrc(g.A + (g.sAz * z + g.sAseg * seg) * 4, g.a_bytes);
    const u32x4 rb = make_rsrc(g.B + (g.sBz * z + g.sBseg * seg) * 4, g.b_bytes);
    const int r[4] = {rows.x, rows.y, rows.z, rows.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool row_ok = k0 + k_lane + i < K && r[i] >= 0 && r[i] < krows_mem;
      if (AK) {
        const bool ok = ak_row[i] != kParked && k0 + ak_kc[i] < K;
        load_to_lds_b128(ra, lds_base + buf * kStage + (4 * wave + i) * 1024, ok ? ak_row[i] + (unsigned)ak_kc[i] * 4u : kParked, (unsigned)k0 * 4u);
      } else {
        load_to_lds_b128(ra, lds_base + buf * kStage + (4 * wave + i) * kPiece,
                         row_ok && am_col_ok ? (unsigned)r[i] * (unsigned)(g.lda * 4) + am_col : kParked, 0u);
      }
      if (BK) {
        const bool ok = bk_row[i] != kParked && k0 + bk_kc[i] < K;
        load_to_lds_b128(rb, lds_base + buf * kStage + kOp + (4 * wave + i) * 1024, ok ? bk_row[i] + (unsigned)bk_kc[i] * 4u : kParked, (unsigned)k0 * 4u);
      } else {
        load_to_lds_b128(rb, lds_base + buf * kStage + kOp + (4 * wave + i) * kPiece,
                         row_ok && bm_col_ok ? (unsigned)r[i] * (unsigned)(g.ldb * 4) + bm_col : kParked, 0u);
      }
    }
  };

  // ---- fragment reads ----
  // Lane l = 16 q + i16.  k-major: k-row 16 G + 4 q + s -> piece 4 q + s, half G, column block * 16 + i16.
  // k-contiguous: row block * 16 + i16, k-chunk 4 G + q in slot (4 G + q) ^ ((row >> 1) & 7) (the blocks' row offsets
  // are multiples of 16, so the XOR term depends on i16 only).
  const int q = lane >> 4, i16 = lane & 15;
  const int sw = (i16 >> 1) & 7;
  const char* fa_base[2];                                        // per group G (k-major: the same for both)
  const char* fb_base[2];
#pragma unroll
  for (int G = 0; G < 2; ++G) {
    fa_base[G] = AK ? lds + (wm * 64 + i16) * 128 + (((4 * G + q) ^ sw) * 16) : lds + 4 * q * kPiece + (wm * 64 + i16) * 4 + G * 512;
    fb_base[G] = BK ? lds + kOp + (wn * 64 + i16) * 128 + (((4 * G + q) ^ sw) * 16) : lds + kOp + 4 * q * kPiece + (wn * 64 + i16) * 4 + G * 512;
  }
  f32x4 acc[4][4];                                               // [m block][n block]; element v: n = 4 q + v
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};
  // Fragments.  A k-contiguous operand is read a group at a time (16 bytes per lane and block = the four steps of the
  // group), a k-major one a step at a time (4 bytes per lane and block); both are read ahead of their use, a piece
  // behind each step's MFMAs, so that only the first read of a stage is waited for.
  float fa[2][4][4], fb[2][4][4];                                // k-contiguous: [group][block][step]; k-major: [step % 2][block][0]
  auto read_a = [&](int buf, int e, int blk) __attribute__((always_inline)) {       // e = 4 G + s
    const int G = e >> 2, sx = e & 3;
    if (AK) {
      const float4 v = *(const float4*)(fa_base[G] + buf * kStage + blk * 2048);
      fa[G][blk][0] = v.x; fa[G][blk][1] = v.y; fa[G][blk][2] = v.z; fa[G][blk][3] = v.w;
    } else {
      fa[e & 1][blk][0] = *(const float*)(fa_base[G] + buf * kStage + sx * kPiece + blk * 64);
    }
  };
  auto read_b = [&](int buf, int e, int blk) __attribute__((always_inline)) {
    const int G = e >> 2, sx = e & 3;
    if (BK) {
      const float4 v = *(const float4*)(fb_base[G] + buf * kStage + blk * 2048);
      fb[G][blk][0] = v.x; fb[G][blk][1] = v.y; fb[G][blk][2] = v.z; fb[G][blk][3] = v.w;
    } else {
      fb[e & 1][blk][0] = *(const float*)(fb_base[G] + buf * kStage + sx * kPiece + blk * 64);
    }
  };

  int4 rows_next = lookup(0);
  if (total > 0) {
    issue(0, 0, rows_next);
    rows_next = lookup(1);
  }
  for (int it = 0; it < total; ++it) {
    const int cur = it & 1;
    __builtin_amdgcn_s_waitcnt(0x0070);            // vmcnt(0) lgkmcnt(0): this wavefront's loads of stage `it` (and the look-up) are in
    __syncthreads();                               // everybody's are, and everybody has finished reading the other buffer
    if (it + 1 < total) issue(it + 1, cur ^ 1, rows_next);
    rows_next = lookup(it + 2);
    // (fenced: left alone, the compiler moves each read down to its first use and waits for it there)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int blk = 0; blk < 4; ++blk) {
      read_a(cur, 0, blk);
      read_b(cur, 0, blk);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      __builtin_amdgcn_sched_barrier(0);
      // k-major: the next step, all four blocks; k-contiguous: during group 0, block e of group 1
#pragma unroll
      for (int blk = 0; blk < 4; ++blk) {
        if (!AK && e + 1 < 8) read_a(cur, e + 1, blk);
        if (!BK && e + 1 < 8) read_b(cur, e + 1, blk);
      }
      if (AK && e < 4) read_a(cur, 4, e);
      if (BK && e < 4) read_b(cur, 4, e);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float av = AK ? fa[e >> 2][i][e & 3] : fa[e & 1][i][0];
          const float bv = BK ? fb[e >> 2][j][e & 3] : fb[e & 1][j][0];
          acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(bv, av, acc[i][j], 0, 0, 0);
        }
    }
  }

  // Epilogue: lane l holds C[m = block_m * 16 + l % 16][n = block_n * 16 + 4 (l / 16) .. + 3].
  float* C = by_range ? g.parts + ((long)z * 8 + ks) * g.sPart : g.C + g.sCz * z;
  const float* bias = (g.bias && ks == 0) ? g.bias + g.sbiasz * z : nullptr;
  const bool vec_ok = (g.ldc % 4 == 0) && (((uintptr_t)C & 15u) == 0);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = m0 + wm * 64 + i * 16 + i16;
    if (row >= M) continue;
    const long prow = (g.c_rows && !by_range) ? g.c_rows[row] : row;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + wn * 64 + j * 16 + 4 * q;
      if (col >= g.N) continue;
      float* p = C + prow * g.ldc + col;
      float e[4] = {acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]};
      if (bias) {
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (col + v < g.N) e[v] += bias[col + v];
      }
      if (ksplit > 1 && !by_range) {
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (col + v < g.N) unsafeAtomicAdd(p + v, e[v]);
      } else if (vec_ok && col + 3 < g.N) {
        float4 o = make_float4(e[0], e[1], e[2], e[3]);
        if (g.accumulate && !by_range) {
          const float4 old = *(const float4*)p;
          o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w;
        }
        *(float4*)p = o;
      } else {
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (col + v < g.N) p[v] = (g.accumulate && !by_range) ? p[v] + e[v] : e[v];
      }
    }
  }
}

// C[z][rows[m]][n] (+)= sum over the eight K ranges of parts[z][range][m][n], m below *m_dev when given; four columns per lane.
__global__ void sum_ranges_kernel(const float* parts, float* C, int M, int N, long ldc, long sCz, long sPart, const int* c_rows,
                                  const int* m_dev, int accumulate) {
  const int nq = (N + 3) / 4;
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  const int m = (int)(idx / nq), n = (int)(idx % nq) * 4, z = blockIdx.y;
  if (m >= (m_dev ? min(M, *m_dev) : M)) return;
  const long src = (long)m * ldc + n;
  float* dst = C + sCz * z + (long)(c_rows ? c_rows[m] : m) * ldc + n;
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  const bool whole = n + 3 < N && ldc % 4 == 0 && (((uintptr_t)(C + sCz * z) & 15u) == 0);
  if (accumulate)
    for (int k = 0; k < 4; ++k)
      if (n + k < N) v[k] = dst[k];
  for (int r = 0; r < 8; ++r) {
    const float* p = parts + ((long)z * 8 + r) * sPart + src;
    if (whole) {
      const f32x4 q4 = __builtin_nontemporal_load((const f32x4*)p);
      v[0] += q4[0]; v[1] += q4[1]; v[2] += q4[2]; v[3] += q4[3];
    } else {
      for (int k = 0; k < 4; ++k)
        if (n + k < N) v[k] += p[k];
    }
  }
  if (whole) *(float4*)dst = make_float4(v[0], v[1], v[2], v[3]);
  else
    for (int k = 0; k < 4; ++k)
      if (n + k < N) dst[k] = v[k];
}

__global__ __launch_bounds__(256, 2) void gemm_float_nn_kernel(FArgs g) { gemm_float_body<true, false>(g); }
__global__ __launch_bounds__(256, 2) void gemm_float_nt_kernel(FArgs g) { gemm_float_body<true, true>(g); }
__global__ __launch_bounds__(256, 2) void gemm_float_tn_kernel(FArgs g) { gemm_float_body<false, false>(g); }

}  // namespace

bool gemm_float_ok(const GemmArgs& g) {
  const auto a16 = [](const void* p) { return ((uintptr_t)p & 15u) == 0; };
  const auto m4 = [](long v) { return v % 4 == 0; };
  const long lim = 0x7fffff00L;                                  // operands are addressed with 32-bit byte offsets
  if (g.in_bf16 || g.out_bf16 || g.lens || g.nseg < 1 || (!g.a_kcontig && g.b_kcontig)) return false;
  if (g.parts && (g.ksplit != 8 || g.bias || !m4(g.ldc) || !a16(g.parts))) return false;   // parts: eight ranges, one per XCD
  if (!a16(g.A) || !a16(g.B) || !m4(g.lda) || !m4(g.ldb) || !m4(g.sAz) || !m4(g.sBz) || !m4(g.sAseg) || !m4(g.sBseg)) return false;
  const bool tn = !g.a_kcontig && !g.b_kcontig;
  if (g.k_rows && (!tn || !a16(g.k_rows))) return false;
  if ((g.a_rows || g.m_dev) && !g.a_kcontig) return false;
  if (g.c_rows && !g.a_kcontig) return false;
  if (tn && g.nseg != 1) return false;
  if ((g.a_kcontig || g.b_kcontig) && !m4(g.K)) return false;    // 16-byte chunks along k must not straddle K
  if (!g.a_kcontig && !m4(g.M)) return false;                    // ... nor along the columns of a k-major operand
  if (!g.b_kcontig && !m4(g.N)) return false;
  const long a_rows_mem = g.a_kcontig ? (g.a_rows ? g.a_phys_rows : g.M) : (g.k_rows ? g.k_phys_rows : g.K);
  const long b_rows_mem = g.b_kcontig ? g.N : (g.k_rows ? g.k_phys_rows : g.K);
  return a_rows_mem * g.lda * 4 <= lim && b_rows_mem * g.ldb * 4 <= lim;
}

hipError_t launch_gemm_float(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0 || g.nz <= 0) return hipSuccess;
  FArgs a = {};
  a.A = (const char*)g.A; a.B = (const char*)g.B; a.C = (float*)g.C; a.bias = g.bias;
  a.M = g.M; a.N = g.N; a.K = g.K; a.lda = g.lda; a.ldb = g.ldb; a.ldc = g.ldc;
  a.sAz = g.sAz; a.sBz = g.sBz; a.sCz = g.sCz; a.sbiasz = g.sbiasz; a.nseg = g.nseg; a.sAseg = g.sAseg; a.sBseg = g.sBseg;
  a.accumulate = g.accumulate;
  a.a_rows = g.a_rows; a.c_rows = g.c_rows; a.a_phys_rows = g.a_phys_rows; a.m_dev = g.m_dev;
  a.k_rows = g.k_rows; a.k_phys_rows = g.k_phys_rows; a.k_dev = g.k_dev;
  a.ksplit = g.ksplit > 1 ? g.ksplit : 1;
  a.parts = g.parts; a.sPart = (long)g.M * g.ldc;
  a.tiles_m = cdiv(g.M, kTile); a.tiles_n = cdiv(g.N, kTile);
  a.per_xcd = cdiv(a.tiles_m * a.tiles_n, 8);
  const long a_rows_mem = g.a_kcontig ? (g.a_rows ? g.a_phys_rows : g.M) : (g.k_rows ? g.k_phys_rows : g.K);
  const long b_rows_mem = g.b_kcontig ? g.N : (g.k_rows ? g.k_phys_rows : g.K);
  a.a_bytes = (unsigned)(a_rows_mem * g.lda * 4); a.b_bytes = (unsigned)(b_rows_mem * g.ldb * 4);
  static std::atomic<unsigned long long> attr_set{0};
  const hipError_t ea = once_per_device(attr_set, [] {
    for (const void* k : {(const void*)gemm_float_nn_kernel, (const void*)gemm_float_nt_kernel, (const void*)gemm_float_tn_kernel}) {
      const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  });
  if (ea != hipSuccess) return ea;
  const dim3 grid = a.parts ? dim3(a.tiles_m * a.tiles_n * 8, g.nz) : dim3(a.per_xcd * 8, g.nz * a.ksplit), block(256);
  if (g.a_kcontig && g.b_kcontig) hipLaunchKernelGGL(gemm_float_nt_kernel, grid, block, kLds, s, a);
  else if (g.a_kcontig) hipLaunchKernelGGL(gemm_float_nn_kernel, grid, block, kLds, s, a);
  else hipLaunchKernelGGL(gemm_float_tn_kernel, grid, block, kLds, s, a);
  if (a.parts) {
    const long lanes = (long)g.M * ((g.N + 3) / 4);
    hipLaunchKernelGGL(sum_ranges_kernel, dim3((unsigned)cdiv(lanes, 256L), g.nz), dim3(256), 0, s, a.parts, a.C, g.M, g.N, g.ldc, g.sCz, a.sPart,
                       g.c_rows, g.m_dev, g.accumulate);
  }
  return hipGetLastError();
}

}  // namespace lstm
