// Hoisted matrix products of the LSTM layer on the gfx950 matrix cores.
//
// Everything that does not depend on the recurrent state is taken out of the time loop
// (paper Sec. 3 and Sec. 7: computation is moved out of the recurrent loop) and done here as
// one large product per layer:
//   forward   Zx  = X   W_x + b        (A k-contiguous, B n-contiguous)
//   backward  dX  = DZ  W_x^T          (A k-contiguous, B k-contiguous, summed over directions)
//             dW_x = X^T  DZ           (A m-contiguous, B n-contiguous, K = all frames, masked)
//             dW_h = Hprev^T DZ        (same shape of problem)
//
// One kernel template covers the four layout combinations.  A 128x128 output tile is computed
// by 256 threads = 4 wavefronts (2x2), each owning a 64x64 sub-tile as 2x2 MFMA 32x32 blocks.
// Operand tiles are staged through LDS in k-contiguous rows of 128 bytes (+16 bytes padding, so
// 16-byte fragment reads of 16 consecutive rows fall into distinct banks).  Operands that are
// stored with m / n contiguous are transposed in registers on their way into LDS.  Global loads
// for tile i+1 are issued before the MFMAs of tile i (register staging, two LDS buffers).
#include "common.h"

namespace lstm {
namespace {

constexpr int kBM = 128, kBN = 128;
constexpr int kRowBytes = 128;            // bytes of k per LDS row: 64 bf16 or 32 float
constexpr int kLdsStride = 144;           // row stride in LDS (bytes)
constexpr int kTileBytes = kBM * kLdsStride;
constexpr int kThreads = 256;

template <typename T> struct Mma;
template <> struct Mma<bf16_t> {
  __device__ static f32x16 run(uint4 a, uint4 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};
template <> struct Mma<float> {
  // a 16-byte chunk holds 4 k per lane group; MFMA e contracts k-pair {e (lanes 0-31), 4+e (lanes 32-63)}
  __device__ static f32x16 run(uint4 a, uint4 b, f32x16 c) {
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    return c;
  }
};

// ---- k-contiguous operand: rows of the tile are rows of memory -------------------------------
// 128 rows x 8 chunks of 16 bytes; thread handles chunks tid + 256*i, i = 0..3
template <typename T>
__device__ __forceinline__ void fetch_kcontig(uint32_t (&st)[16], const char* base, long ld, int rows, int row0,
                                              int K, int k0, int vec, int tid, const int (&prow)[4]) {
  constexpr int ES = sizeof(T), EPC = 16 / ES;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int c = tid + kThreads * i;
    int row = row0 + (c >> 3), k = k0 + (c & 7) * EPC;
    uint32_t w0 = 0, w1 = 0, w2 = 0, w3 = 0;
    if (row < rows && k < K) {
      const char* p = base + ((long)prow[i] * ld + k) * ES;                       // prow[i]: where logical row `row` lies in memory
      if (vec >= 16 && k + EPC <= K) {
        uint4 v = *(const uint4*)p;
        w0 = v.x; w1 = v.y; w2 = v.z; w3 = v.w;
      } else if (vec >= 8 && k + EPC <= K) {
        uint2 v0 = *(const uint2*)p, v1 = *(const uint2*)(p + 8);
        w0 = v0.x; w1 = v0.y; w2 = v1.x; w3 = v1.y;
      } else {
        uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (ES == 4) {
            if (k + j < K) w[j] = *(const uint32_t*)(p + 4 * j);
          } else {
            int ke = k + 2 * j;
            if (vec >= 4 && ke + 2 <= K) w[j] = *(const uint32_t*)(p + 4 * j);
            else {
              uint32_t lo = ke < K ? *(const uint16_t*)(p + 4 * j) : 0u;
              uint32_t hi = ke + 1 < K ? *(const uint16_t*)(p + 4 * j + 2) : 0u;
              w[j] = lo | (hi << 16);
            }
          }
        }
        w0 = w[0]; w1 = w[1]; w2 = w[2]; w3 = w[3];
      }
    }
    st[4 * i] = w0; st[4 * i + 1] = w1; st[4 * i + 2] = w2; st[4 * i + 3] = w3;
  }
}
__device__ __forceinline__ void commit_kcontig(const uint32_t (&st)[16], char* lds, int tid) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int c = tid + kThreads * i;
    *(uint4*)(lds + (c >> 3) * kLdsStride + (c & 7) * 16) = make_uint4(st[4 * i], st[4 * i + 1], st[4 * i + 2], st[4 * i + 3]);
  }
}

// ---- m-contiguous operand: rows of memory are k, the tile is transposed in registers ----------
// frame mask: row k of the K axis is frame (t = k / Bt, b = k % Bt), valid iff t < lens[b]
// bf16: micro-tile of 8 k x 2 m (eight 4-byte loads), two micro-tiles per thread
template <bool MASK>
__device__ __forceinline__ void fetch_mcontig_bf16(uint32_t (&st)[16], const char* base, long ld, int cols, int col0,
                                                   int K, int k0, int vec, int tid, const int* lens, int Bt, int T, const int* krows) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    int c = tid + kThreads * i;
    int m = col0 + 2 * (c & 63), kb = __builtin_amdgcn_readfirstlane(k0 + (c >> 6) * 8);   // (the same in every lane of a wavefront)
    // The frame mask is fetched independently of the data and applied afterwards, so the data loads
    // never wait for the seq_lens loads.
    uint32_t keep = 0xffu;
    if (MASK) {
      int ft = kb / Bt, fb = kb - ft * Bt;                  // frame (t, b) of row kb, advanced incrementally
      keep = 0u;
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        if (kb + kk < K) { int L = lens[fb]; L = L < 0 ? 0 : (L > T ? T : L); keep |= (ft < L ? 1u : 0u) << kk; }
        if (++fb == Bt) { fb = 0; ++ft; }
      }
    }
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      int k = kb + kk;
      uint32_t w = 0;
      if (k < K && m < cols) {
        const char* p = base + ((long)(krows ? krows[k] : k) * ld + m) * 2;   // k is the same in every lane: a scalar look-up
        if (vec >= 4 && m + 1 < cols) w = *(const uint32_t*)p;
        else {
          w = *(const uint16_t*)p;
          if (m + 1 < cols) w |= ((uint32_t) * (const uint16_t*)(p + 2)) << 16;
        }
      }
      st[8 * i + kk] = ((keep >> kk) & 1u) ? w : 0u;
    }
  }
}
__device__ __forceinline__ void commit_mcontig_bf16(const uint32_t (&st)[16], char* lds, int tid) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    int c = tid + kThreads * i;
    int r = 2 * (c & 63), kc = c >> 6;
    uint32_t lo[4], hi[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint32_t a = st[8 * i + 2 * j], b = st[8 * i + 2 * j + 1];
      lo[j] = (a & 0xffffu) | (b << 16);
      hi[j] = (a >> 16) | (b & 0xffff0000u);
    }
    *(uint4*)(lds + r * kLdsStride + kc * 16) = make_uint4(lo[0], lo[1], lo[2], lo[3]);
    *(uint4*)(lds + (r + 1) * kLdsStride + kc * 16) = make_uint4(hi[0], hi[1], hi[2], hi[3]);
  }
}
// float: micro-tile of 4 k x 1 m, four per thread
template <bool MASK>
__device__ __forceinline__ void fetch_mcontig_f32(uint32_t (&st)[16], const char* base, long ld, int cols, int col0,
                                                  int K, int k0, int tid, const int* lens, int Bt, int T, const int* krows) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int c = tid + kThreads * i;
    int m = col0 + (c & 127), kb = __builtin_amdgcn_readfirstlane(k0 + (c >> 7) * 4);     // (the same in every lane of a wavefront)
    uint32_t keep = 0xfu;
    if (MASK) {
      int ft = kb / Bt, fb = kb - ft * Bt;
      keep = 0u;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        if (kb + kk < K) { int L = lens[fb]; L = L < 0 ? 0 : (L > T ? T : L); keep |= (ft < L ? 1u : 0u) << kk; }
        if (++fb == Bt) { fb = 0; ++ft; }
      }
    }
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      int k = kb + kk;
      uint32_t w = (k < K && m < cols) ? *(const uint32_t*)(base + ((long)(krows ? krows[k] : k) * ld + m) * 4) : 0u;   // scalar look-up
      st[4 * i + kk] = ((keep >> kk) & 1u) ? w : 0u;
    }
  }
}
__device__ __forceinline__ void commit_mcontig_f32(const uint32_t (&st)[16], char* lds, int tid) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int c = tid + kThreads * i;
    *(uint4*)(lds + (c & 127) * kLdsStride + (c >> 7) * 16) = make_uint4(st[4 * i], st[4 * i + 1], st[4 * i + 2], st[4 * i + 3]);
  }
}

template <typename T, bool AK, bool BK, bool MASK>
struct Stager {
  static constexpr int EPT = kRowBytes / (int)sizeof(T);   // k per tile: 64 bf16 / 32 float
  // M, K: the extents in force (the arguments', or what the device-side counts cut them down to)
  __device__ static void fetchA(uint32_t (&st)[16], const GemmArgs& g, const char* A, int M, int K, int m0, int k0, int tid,
                                const int (&prow)[4]) {
    if constexpr (AK) fetch_kcontig<T>(st, A, g.lda, M, m0, K, k0, g.vecA, tid, prow);
    else if constexpr (sizeof(T) == 2) fetch_mcontig_bf16<MASK>(st, A, g.lda, M, m0, K, k0, g.vecA, tid, g.lens, g.Bt, g.T, g.k_rows);
    else fetch_mcontig_f32<MASK>(st, A, g.lda, M, m0, K, k0, tid, g.lens, g.Bt, g.T, g.k_rows);
  }
  __device__ static void fetchB(uint32_t (&st)[16], const GemmArgs& g, const char* B, int K, int n0, int k0, int tid,
                                const int (&prow)[4]) {
    if constexpr (BK) fetch_kcontig<T>(st, B, g.ldb, g.N, n0, K, k0, g.vecB, tid, prow);
    else if constexpr (sizeof(T) == 2) fetch_mcontig_bf16<false>(st, B, g.ldb, g.N, n0, K, k0, g.vecB, tid, nullptr, 1, 0, AK ? nullptr : g.k_rows);
    else fetch_mcontig_f32<false>(st, B, g.ldb, g.N, n0, K, k0, tid, nullptr, 1, 0, AK ? nullptr : g.k_rows);
  }
  __device__ static void commitA(const uint32_t (&st)[16], char* lds, int tid) {
    if constexpr (AK) commit_kcontig(st, lds, tid);
    else if constexpr (sizeof(T) == 2) commit_mcontig_bf16(st, lds, tid);
    else commit_mcontig_f32(st, lds, tid);
  }
  __device__ static void commitB(const uint32_t (&st)[16], char* lds, int tid) {
    if constexpr (BK) commit_kcontig(st, lds, tid);
    else if constexpr (sizeof(T) == 2) commit_mcontig_bf16(st, lds, tid);
    else commit_mcontig_f32(st, lds, tid);
  }
};

template <typename T, typename TC, bool AK, bool BK, bool MASK>
__global__ __launch_bounds__(kThreads, 2) void gemm_kernel(GemmArgs g) {
  using S = Stager<T, AK, BK, MASK>;
  __shared__ __attribute__((aligned(16))) char lds[4 * kTileBytes];   // A0 B0 A1 B1
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int r = lane & 31, gq = lane >> 5;

  // tile raster: bands of 8 tile-columns, row-major inside a band, so that the eight XCDs
  // (work-groups are dealt to them round-robin) each keep one B tile-column in their L2.
  const int tiles_m = (g.M + kBM - 1) / kBM, tiles_n = (g.N + kBN - 1) / kBN;
  int bid = blockIdx.x;
  const int band = bid / (8 * tiles_m);
  const int width = min(8, tiles_n - band * 8);
  const int rel = bid - band * 8 * tiles_m;
  const int tn = band * 8 + rel % width, tm = rel / width;
  const int m0 = tm * kBM, n0 = tn * kBN;
  // blockIdx.y = problem z and, with ksplit > 1 (float C holding zeros or the value to add to), the range of the K axis
  // that this work-group multiplies; the ranges' parts meet in C by atomic adds
  const int ks = g.ksplit > 1 ? g.ksplit : 1;
  const int z = blockIdx.y / ks, range = blockIdx.y - z * ks;
  // Row maps and device-side extents (the frames that are real, numbered on the device): logical row r of a k-contiguous A
  // and of C is row a_rows[r] / c_rows[r] in memory, M is cut down to *m_dev; with both operands m-contiguous, row k of
  // the K axis is row k_rows[k] of A and of B, K cut down to *k_dev.
  const int M = g.m_dev ? min(g.M, *g.m_dev) : g.M;
  const int K = g.k_dev ? min(g.K, *g.k_dev) : g.K;
  if (m0 >= M) return;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // where the rows this thread stages lie in memory (k-contiguous operands: the same rows in every stage)
  int arow[4], brow[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int ra = m0 + ((tid + kThreads * i) >> 3);
    arow[i] = (AK && g.a_rows && ra < M) ? g.a_rows[ra] : ra;
    brow[i] = n0 + ((tid + kThreads * i) >> 3);
  }
  const int ktiles = (K + S::EPT - 1) / S::EPT;
  const int total = ktiles * g.nseg;
  uint32_t sa[16], sb[16];
  auto fetch = [&](int it) {
    int seg = it / ktiles, kt = it - seg * ktiles;
    const char* A = (const char*)g.A + (g.sAz * z + g.sAseg * seg) * (long)sizeof(T);
    const char* B = (const char*)g.B + (g.sBz * z + g.sBseg * seg) * (long)sizeof(T);
    S::fetchA(sa, g, A, M, K, m0, kt * S::EPT, tid, arow);
    S::fetchB(sb, g, B, K, n0, kt * S::EPT, tid, brow);
  };
  const int it_begin = (int)((long)total * range / ks), it_end = (int)((long)total * (range + 1) / ks);
  if (it_end > it_begin) {
    fetch(it_begin);
    S::commitA(sa, lds, tid);
    S::commitB(sb, lds + kTileBytes, tid);
  }
  __syncthreads();
  for (int it = it_begin; it < it_end; ++it) {
    const int cur = (it - it_begin) & 1;
    if (it + 1 < it_end) fetch(it + 1);
    const char* As = lds + cur * 2 * kTileBytes + (wm * 64 + r) * kLdsStride + gq * 16;
    const char* Bs = lds + cur * 2 * kTileBytes + kTileBytes + (wn * 64 + r) * kLdsStride + gq * 16;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint4 a0 = *(const uint4*)(As + j * 32), a1 = *(const uint4*)(As + 32 * kLdsStride + j * 32);
      uint4 b0 = *(const uint4*)(Bs + j * 32), b1 = *(const uint4*)(Bs + 32 * kLdsStride + j * 32);
      acc[0][0] = Mma<T>::run(a0, b0, acc[0][0]);
      acc[0][1] = Mma<T>::run(a0, b1, acc[0][1]);
      acc[1][0] = Mma<T>::run(a1, b0, acc[1][0]);
      acc[1][1] = Mma<T>::run(a1, b1, acc[1][1]);
    }
    if (it + 1 < it_end) {
      S::commitA(sa, lds + (cur ^ 1) * 2 * kTileBytes, tid);
      S::commitB(sb, lds + (cur ^ 1) * 2 * kTileBytes + kTileBytes, tid);
    }
    __syncthreads();
  }

  // epilogue: lane holds column (lane % 32), rows 8*(v/4) + 4*(lane/32) + v%4 of each 32x32 block
  TC* C = (TC*)g.C + g.sCz * z;
  const float* bias = g.bias ? g.bias + g.sbiasz * z : nullptr;
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int col = n0 + wn * 64 + j * 32 + r;
    if (col >= g.N) continue;
    const float bv = (bias && range == 0) ? bias[col] : 0.f;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * gq + (v & 3);
        if (row < M) {
          float val = acc[i][j][v] + bv;
          long off = (long)(g.c_rows ? g.c_rows[row] : row) * g.ldc + col;
          if constexpr (sizeof(TC) == 4) {
            if (ks > 1) unsafeAtomicAdd((float*)C + off, val);
            else {
              if (g.accumulate) val += ((float*)C)[off];
              ((float*)C)[off] = val;
            }
          } else {
            ((uint16_t*)C)[off] = f2bf_bits(val);
          }
        }
      }
  }
}

template <typename T, typename TC>
hipError_t dispatch(const GemmArgs& g, hipStream_t s) {
  const int tiles_m = (g.M + kBM - 1) / kBM, tiles_n = (g.N + kBN - 1) / kBN;
  if (g.ksplit > 1 && (sizeof(TC) != 4 || g.parts)) return hipErrorInvalidValue;   // ranges of K: float C, added atomically
  dim3 grid(tiles_m * tiles_n, g.nz * (g.ksplit > 1 ? g.ksplit : 1)), block(kThreads);
  if (g.a_kcontig && !g.b_kcontig) hipLaunchKernelGGL((gemm_kernel<T, TC, true, false, false>), grid, block, 0, s, g);
  else if (g.a_kcontig && g.b_kcontig) hipLaunchKernelGGL((gemm_kernel<T, TC, true, true, false>), grid, block, 0, s, g);
  else if (!g.a_kcontig && !g.b_kcontig && g.lens) hipLaunchKernelGGL((gemm_kernel<T, TC, false, false, true>), grid, block, 0, s, g);
  else if (!g.a_kcontig && !g.b_kcontig) hipLaunchKernelGGL((gemm_kernel<T, TC, false, false, false>), grid, block, 0, s, g);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0 || g.nz <= 0) return hipSuccess;
  if (gemm_skinny_ok(g)) return launch_gemm_skinny(g, false, s);
  if (gemm_nt_ok(g)) return launch_gemm_nt(g, s);
  if (gemm_tn_ok(g)) return launch_gemm_tn(g, s);
  if (gemm_float_ok(g)) return launch_gemm_float(g, s);
  if (g.in_bf16) {
    if (g.out_bf16) return dispatch<bf16_t, bf16_t>(g, s);
    return dispatch<bf16_t, float>(g, s);
  }
  if (g.out_bf16) return hipErrorInvalidValue;
  return dispatch<float, float>(g, s);
}

}  // namespace lstm
