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
// Kernel: 256x256 output tile per work-group of 4 wavefronts (2x2), each wavefront a 128x128
// sub-tile = 4x4 MFMA 32x32x16 blocks (256 accumulator registers).  K advances 64 at a time through
// two LDS stages (rows of 128 bytes + 16 bytes padding; 144 KiB of the 160 KiB LDS).  Global loads run two
// stages ahead of the MFMAs (one stage in registers, one in LDS); fragments are double-buffered in registers.
// Per 16-wide k step a wavefront issues 8 LDS reads for 16 MFMAs, half the LDS bandwidth a 128x128
// work-group tile would need.
#include "common.h"

namespace lstm {
namespace {

constexpr int kT = 256;                   // tile edge (both M and N)
constexpr int kKB = 64;                   // k per stage (bf16 elements)
constexpr int kStride = 144;              // LDS row stride in bytes
constexpr int kOpBytes = kT * kStride;    // one operand, one stage
constexpr int kThreads = 256;

struct NtArgs {
  const char* A; const char* B; void* C; const float* bias;
  int M, N, K;
  long lda, ldb, ldc;                     // elements
  long sAz, sBz, sCz, sbiasz; int nz;
  int nseg; long sAseg, sBseg;
  int accumulate;
};

__device__ __forceinline__ f32x16 mma(uint4 a, uint4 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
constexpr int kBufFlags = 0x00020000;   // raw buffer descriptor word 3 for gfx9-family devices

// One operand of one stage: 256 rows x 8 chunks of 16 bytes; thread handles chunks tid + 256*i, i < 8.
// Loads go through a buffer descriptor covering exactly the operand's rows: rows past the end read as zero
// in hardware, so only the K tail needs a mask (and only in the last stage of a segment).
struct OperandLoader {
  __amdgpu_buffer_rsrc_t rs;
  unsigned voff[8];                     // byte offset of chunk i at k = 0
  int kc8;                              // first k of this thread's chunk inside a stage
  __device__ __forceinline__ void init(const char* base, long ld, int rows, int row0, int tid) {
    const long bytes = (long)rows * ld * 2;
    rs = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, bytes > 0x7fffffffL ? 0x7fffffff : (int)bytes, kBufFlags);
    kc8 = (tid & 7) * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const long row = row0 + ((tid + kThreads * i) >> 3);
      const long off = (row * ld + kc8) * 2;
      voff[i] = off > 0x7ffffff0L ? 0x7ffffff0u : (unsigned)off;      // past-the-end rows land outside the descriptor
    }
  }
  template <bool TAIL>
  __device__ __forceinline__ void fetch(uint4 (&st)[8], int k0, int K) const {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const u32x4 x = __builtin_amdgcn_raw_buffer_load_b128(rs, voff[i] + k0 * 2, 0, 0);
      const bool keep = !TAIL || k0 + kc8 < K;
      st[i] = keep ? make_uint4(x[0], x[1], x[2], x[3]) : make_uint4(0, 0, 0, 0);
    }
  }
};
__device__ __forceinline__ void commit(const uint4 (&st)[8], char* lds, int tid) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int c = tid + kThreads * i;
    *(uint4*)(lds + (c >> 3) * kStride + (c & 7) * 16) = st[i];
  }
}

template <typename TC>
__global__ __launch_bounds__(kThreads, 1) void gemm_nt_kernel(NtArgs g) {
  extern __shared__ __attribute__((aligned(16))) char lds[];   // [stage][A | B]
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave >> 1, wn = wave & 1;
  const int r = lane & 31, gq = lane >> 5;

  // tile raster: bands of 8 tile-columns, row-major inside a band: the eight XCDs (work-groups are dealt to
  // them round-robin) each keep one B tile-column in their L2 while the A tiles stream through
  const int tiles_m = (g.M + kT - 1) / kT, tiles_n = (g.N + kT - 1) / kT;
  const int bid = blockIdx.x;
  const int band = bid / (8 * tiles_m);
  const int width = min(8, tiles_n - band * 8);
  const int rel = bid - band * 8 * tiles_m;
  const int tn = band * 8 + rel % width, tm = rel / width;
  const int m0 = tm * kT, n0 = tn * kT;
  const int z = blockIdx.y;

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int ktiles = (g.K + kKB - 1) / kKB;
  const bool ktail = (g.K % kKB) != 0;
  const int total = ktiles * g.nseg;
  OperandLoader la, lb;
  int seg_loaded = -1;
  uint4 sa[8], sb[8];
  // stage `it`: segment it / ktiles, k offset (it % ktiles) * 64
  auto fetch_a = [&](int it) {
    const int seg = it / ktiles, kt = it - seg * ktiles;
    if (seg != seg_loaded) {
      la.init(g.A + (g.sAz * z + g.sAseg * seg) * 2, g.lda, g.M, m0, tid);
      lb.init(g.B + (g.sBz * z + g.sBseg * seg) * 2, g.ldb, g.N, n0, tid);
      seg_loaded = seg;
    }
    if (ktail && kt == ktiles - 1) la.fetch<true>(sa, kt * kKB, g.K); else la.fetch<false>(sa, kt * kKB, g.K);
  };
  auto fetch_b = [&](int it) {
    const int seg = it / ktiles, kt = it - seg * ktiles;
    if (ktail && kt == ktiles - 1) lb.fetch<true>(sb, kt * kKB, g.K); else lb.fetch<false>(sb, kt * kKB, g.K);
  };
  // prologue: stage 0 into LDS buffer 0, stage 1 into registers
  if (total > 0) {
    fetch_a(0); fetch_b(0);
    commit(sa, lds, tid);
    commit(sb, lds + kOpBytes, tid);
    if (total > 1) { fetch_a(1); fetch_b(1); }
  }
  __syncthreads();

  // Main loop.  While stage `it` is multiplied out of LDS buffer it&1: the registers holding stage it+1 are
  // written to the other buffer (k-steps 0-1), then the loads of stage it+2 are issued (k-steps 2-3), so every
  // global load has a whole stage of MFMAs to complete.  Fragments for k-step s+1 are read from LDS while
  // the 16 MFMAs of step s run; the scheduling barriers keep the compiler from collapsing that overlap.
  // (Moving the barrier to mid-stage and pre-reading the next stage's first fragments measured slower.)
  for (int it = 0; it < total; ++it) {
    const int cur = it & 1;
    const char* As = lds + cur * 2 * kOpBytes + (wm * 128 + r) * kStride + gq * 16;
    const char* Bs = lds + cur * 2 * kOpBytes + kOpBytes + (wn * 128 + r) * kStride + gq * 16;
    char* nxt = lds + (cur ^ 1) * 2 * kOpBytes;
    uint4 fa[2][4], fb[2][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      fa[0][i] = *(const uint4*)(As + i * 32 * kStride);
      fb[0][i] = *(const uint4*)(Bs + i * 32 * kStride);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int c = s & 1;
      if (s < 3) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          fa[c ^ 1][i] = *(const uint4*)(As + i * 32 * kStride + (s + 1) * 32);
          fb[c ^ 1][i] = *(const uint4*)(Bs + i * 32 * kStride + (s + 1) * 32);
        }
      }
      if (it + 1 < total) {
        if (s == 0) commit(sa, nxt, tid);
        if (s == 1) commit(sb, nxt + kOpBytes, tid);
      }
      if (it + 2 < total) {
        if (s == 2) fetch_a(it + 2);
        if (s == 3) fetch_b(it + 2);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = mma(fa[c][i], fb[c][j], acc[i][j]);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
  }

  // epilogue: a lane holds column (lane % 32), rows 8*(v/4) + 4*(lane/32) + v%4 of each 32x32 block
  TC* C = (TC*)g.C + g.sCz * z;
  const float* bias = g.bias ? g.bias + g.sbiasz * z : nullptr;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int col = n0 + wn * 128 + j * 32 + r;
    if (col >= g.N) continue;
    const float bv = bias ? bias[col] : 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * 128 + i * 32 + 8 * (v >> 2) + 4 * gq + (v & 3);
        if (row < g.M) {
          float val = acc[i][j][v] + bv;
          const long off = (long)row * g.ldc + col;
          if constexpr (sizeof(TC) == 4) {
            if (g.accumulate) val += ((float*)C)[off];
            ((float*)C)[off] = val;
          } else {
            ((uint16_t*)C)[off] = f2bf_bits(val);
          }
        }
      }
  }
}

// dst[c][r] = keep(r) ? src[r][c] : 0 for r < R, c < C ; dst rows are padded with zeros up to ldd.
// keep(r): rows of src are frames (t = r / Bt, b = r % Bt), kept iff lens == NULL or t < lens[b].
__global__ __launch_bounds__(256) void transpose_kernel(const uint16_t* src, uint16_t* dst, int R, int C, long lds_, long ldd,
                                                        long s_src, long s_dst, const int* lens, int Bt, int T) {
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
      if (keep) v = src[(long)rr * lds_ + cc];
    }
    tile[ty + 4 * i][tx] = v;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int cc = c0 + ty + 4 * i, rr = r0 + tx;
    if (cc < C && rr < ldd) dst[(long)cc * ldd + rr] = tile[tx][ty + 4 * i];
  }
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
  return g.in_bf16 && g.a_kcontig && g.b_kcontig && !g.lens && g.K % 8 == 0 && g.lda % 8 == 0 && g.ldb % 8 == 0 &&
         g.sAz % 8 == 0 && g.sBz % 8 == 0 && g.sAseg % 8 == 0 && g.sBseg % 8 == 0 && a16(g.A) && a16(g.B);
}

hipError_t launch_gemm_nt(const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0 || g.nz <= 0) return hipSuccess;
  NtArgs a;
  a.A = (const char*)g.A; a.B = (const char*)g.B; a.C = g.C; a.bias = g.bias;
  a.M = g.M; a.N = g.N; a.K = g.K; a.lda = g.lda; a.ldb = g.ldb; a.ldc = g.ldc;
  a.sAz = g.sAz; a.sBz = g.sBz; a.sCz = g.sCz; a.sbiasz = g.sbiasz; a.nz = g.nz;
  a.nseg = g.nseg; a.sAseg = g.sAseg; a.sBseg = g.sBseg; a.accumulate = g.accumulate;
  const int tiles = cdiv(g.M, kT) * cdiv(g.N, kT);
  const size_t shmem = 4 * kOpBytes;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_nt_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e == hipSuccess) e = hipFuncSetAttribute((const void*)gemm_nt_kernel<uint16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shmem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  if (g.out_bf16) hipLaunchKernelGGL(gemm_nt_kernel<uint16_t>, dim3(tiles, g.nz), dim3(kThreads), shmem, s, a);
  else hipLaunchKernelGGL(gemm_nt_kernel<float>, dim3(tiles, g.nz), dim3(kThreads), shmem, s, a);
  return hipGetLastError();
}

hipError_t launch_transpose(const void* src, void* dst, int R, int C, long ld_src, long ld_dst, int nz, long s_src, long s_dst,
                            const int* lens, int Bt, int T, hipStream_t s) {
  if (R <= 0 || C <= 0 || nz <= 0) return hipSuccess;
  hipLaunchKernelGGL(transpose_kernel, dim3(cdiv(ld_dst, 64), cdiv(C, 64), nz), dim3(256), 0, s, (const uint16_t*)src,
                     (uint16_t*)dst, R, C, ld_src, ld_dst, s_src, s_dst, lens, Bt, T);
  return hipGetLastError();
}

hipError_t launch_pad_rows(const void* src, void* dst, long R, int C, int ld_dst, hipStream_t s) {
  if (R <= 0) return hipSuccess;
  const long total = R * ld_dst;
  hipLaunchKernelGGL(pad_rows_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, (const uint16_t*)src, (uint16_t*)dst, R, C, ld_dst);
  return hipGetLastError();
}

}  // namespace lstm
