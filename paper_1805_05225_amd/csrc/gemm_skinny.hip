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
// Eight wavefronts: wavefront (kg, wn) owns the 96 x 32 block of column group wn (three 32x32x16 MFMA blocks) for the
// k-steps 2 kg, 2 kg + 1 of every 64-wide stage; the two halves are added in the epilogue.  Two wavefronts per SIMD,
// so one's LDS reads hide behind the other's MFMAs.  Operands travel from global memory straight into LDS (16 bytes
// per lane, 1 KiB per wavefront instruction = 8 rows of 128 bytes), two stages, one barrier per stage; bank conflicts
// are avoided by placement: the 16-byte slot p of row r holds k-chunk p ^ ((r >> 1) & 7).  What bounds it is the path
// from L2 to LDS (about 47 bytes per clock and compute unit, measured for the large kernels): 28 KiB per stage
// against 384 clocks of MFMA work, i.e. about 600 clocks per stage.
#include "recurrent_dev.h"

namespace lstm {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
constexpr int kBufFlags = 0x00020000;   // raw buffer descriptor word 3 for gfx9-family devices
constexpr int kTM = 96, kTN = 128;
constexpr int kRow = 128;                          // bytes per LDS row (64 bfloat16)
constexpr int kAop = kTM * kRow, kBop = kTN * kRow, kStage = kAop + kBop;      // 12 + 16 KiB
constexpr int kLoads = (kTM + kTN) / 8;            // wavefront-loads per stage: 12 for A, 16 for B
constexpr int kEpStride = kTN + 4;                 // floats per staged row
constexpr int kLds = 2 * kStage > kTM * kEpStride * 4 ? 2 * kStage : kTM * kEpStride * 4;     // 57344 bytes
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
// runs at a time should share operand panels out of its L2: with tiles_m <= 8 row tiles, an XCD takes all row tiles of
// 32 / bm column tiles at a time (bm = tiles_m rounded up to a power of two); otherwise tiles are dealt row-major.
struct Tile { int tm, tn; bool live; };
__device__ __forceinline__ Tile tile_of(int tiles_m, int tiles_n) {
  Tile t = {0, 0, false};
  const int bid = blockIdx.x;
  if (tiles_m <= 8) {
    const int bm = tiles_m <= 1 ? 1 : tiles_m <= 2 ? 2 : tiles_m <= 4 ? 4 : 8, bn = 32 / bm;
    const int xcd = bid & 7, slot = bid >> 3, group = (slot / 32) * 8 + xcd, pos = slot % 32;
    t.tm = pos % bm; t.tn = group * bn + pos / bm;
    t.live = t.tm < tiles_m && t.tn < tiles_n;
  } else {
    t.tm = bid % tiles_m; t.tn = bid / tiles_m;
    t.live = t.tn < tiles_n;
  }
  return t;
}
inline int grid_for(int tiles_m, int tiles_n) {
  if (tiles_m <= 8) {
    const int bm = tiles_m <= 1 ? 1 : tiles_m <= 2 ? 2 : tiles_m <= 4 ? 4 : 8, bn = 32 / bm;
    const int groups = cdiv(tiles_n, bn);
    return cdiv(groups, 8) * 8 * 32;
  }
  return tiles_m * tiles_n;
}

template <bool CELL>
__global__ __launch_bounds__(512) void skinny_kernel(SkinnyArgs g) {
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int kg = wave >> 2, wn = wave & 3;
  const int r = lane & 31, gq = lane >> 5;
  const int tiles_m = (g.M + kTM - 1) / kTM, tiles_n = (g.N + kTN - 1) / kTN;
  const Tile tl = tile_of(tiles_m, tiles_n);
  if (!tl.live) return;
  const int m0 = tl.tm * kTM, n0 = tl.tn * kTN, z = blockIdx.z;
  const int K = g.K, nstage = (K + 63) / 64;

  f32x16 acc[3];
#pragma unroll
  for (int i = 0; i < 3; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

  // Loads: wavefront-load q of a stage (q = wave + 8 i) fills rows 8 q' .. 8 q' + 7 of A (q < 12) or B; lane l fills
  // slot l & 7 of row l >> 3 of those, i.e. fetches k-chunk (l & 7) ^ swizzle(row).  Rows past the operand's end and
  // chunks past K point outside the buffer descriptor and arrive as zeros.
  constexpr int kPerWave = (kLoads + 7) / 8;       // 4 (the last round has 4 loads for 8 wavefronts)
  unsigned voff[kPerWave], dst[kPerWave];
  int chunk[kPerWave];
  bool is_b[kPerWave], on[kPerWave];
  const long a_bytes = (long)g.M * g.lda * 2, b_bytes = (long)g.N * g.ldb * 2;
#pragma unroll
  for (int i = 0; i < kPerWave; ++i) {
    const int q = wave + 8 * i;
    on[i] = q < kLoads;
    is_b[i] = q >= kTM / 8;
    const int rg = is_b[i] ? q - kTM / 8 : q;
    const int rl = rg * 8 + (lane >> 3);
    chunk[i] = (lane & 7) ^ ((rl >> 1) & 7);
    const long row = (is_b[i] ? n0 : m0) + rl;
    const bool inside = is_b[i] ? row < g.N : row < g.M;
    const long off = row * (is_b[i] ? g.ldb : g.lda) * 2 + chunk[i] * 16;
    voff[i] = (inside && off <= 0x7fffff00L) ? (unsigned)off : kParked;
    dst[i] = (unsigned)((is_b[i] ? kAop : 0) + rg * 1024);
  }
  const unsigned lds_base = (unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)lds;
  const u32x4 ra = make_rsrc(g.A + g.sAz * z * 2, a_bytes > 0x7fffff00L ? 0x7fffff00u : (unsigned)a_bytes);
  const u32x4 rb = make_rsrc(g.B + g.sBz * z * 2, b_bytes > 0x7fffff00L ? 0x7fffff00u : (unsigned)b_bytes);
  auto issue = [&](int it, int buf) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < kPerWave; ++i) {
      if (!on[i]) continue;                                    // wave-uniform
      const bool past = it * 64 + chunk[i] * 8 >= K;           // ragged last stage
      load_to_lds_b128(is_b[i] ? rb : ra, lds_base + buf * kStage + dst[i], past ? kParked : voff[i], (unsigned)it * 128u);
    }
  };
  // Fragment reads: row (i*32 + r) of A / (wn*32 + r) of B, k-chunk 2 s + gq, in slot (2 s + gq) ^ ((row >> 1) & 7)
  const int sw = (r >> 1) & 7;
  const int fa_off = r * kRow, fb_off = kAop + (wn * 32 + r) * kRow;

  issue(0, 0);
  __builtin_amdgcn_s_waitcnt(0x0f70);              // vmcnt(0)
  __syncthreads();
  for (int it = 0; it < nstage; ++it) {
    const int cur = it & 1;
    if (it + 1 < nstage) issue(it + 1, cur ^ 1);   // the other buffer was last read before the barrier that ended stage it - 1
    const char* base = lds + cur * kStage;
    uint4 fa[2][3], fb[2];
#pragma unroll
    for (int ss = 0; ss < 2; ++ss) {
      const int slot = ((2 * (2 * kg + ss) + gq) ^ sw) * 16;
#pragma unroll
      for (int i = 0; i < 3; ++i) fa[ss][i] = *(const uint4*)(base + fa_off + i * 32 * kRow + slot);
      fb[ss] = *(const uint4*)(base + fb_off + slot);
    }
#pragma unroll
    for (int ss = 0; ss < 2; ++ss)
#pragma unroll
      for (int i = 0; i < 3; ++i) acc[i] = mma32(fa[ss][i], fb[ss], acc[i]);
    __builtin_amdgcn_s_waitcnt(0x0070);            // vmcnt(0) lgkmcnt(0): own loads of the next stage landed, own reads done
    __syncthreads();
  }

  // Epilogue.  The two k-halves meet in LDS (the stage buffers are free: the loop ended with a barrier):
  // acc[i][v] is row i*32 + 8 (v / 4) + 4 gq + v % 4, column wn*32 + r.
  float* ep = (float*)lds;
  if (kg == 1) {
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) ep[(i * 32 + 8 * (v >> 2) + 4 * gq + (v & 3)) * kEpStride + wn * 32 + r] = acc[i][v];
  }
  __syncthreads();
  if (kg == 0) {
#pragma unroll
    for (int i = 0; i < 3; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) ep[(i * 32 + 8 * (v >> 2) + 4 * gq + (v & 3)) * kEpStride + wn * 32 + r] += acc[i][v];
  }
  __syncthreads();
  if constexpr (!CELL) {
    // thread -> (row, four columns): 32 threads per row, 16 rows per pass
    const int c4 = (tid & 31) * 4, col = n0 + c4;
    const float* bias = g.bias ? g.bias + g.sbiasz * z : nullptr;
    float bv[4] = {0.f, 0.f, 0.f, 0.f};
    if (bias) {
#pragma unroll
      for (int k = 0; k < 4; ++k) if (col + k < g.N) bv[k] = bias[col + k];
    }
    const bool vec = (g.ldc % 4 == 0) && ((((uintptr_t)g.C) & 15u) == 0) && (g.sCz % 4 == 0) && col + 3 < g.N;
    for (int rr = tid >> 5; rr < kTM; rr += 16) {
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

hipError_t launch(const SkinnyArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0 || a.nz <= 0) return hipSuccess;
  static bool attr_set = false;
  if (!attr_set) {
    for (const void* k : {(const void*)skinny_kernel<false>, (const void*)skinny_kernel<true>}) {
      const hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kLds);
      if (e != hipSuccess) return e;
    }
    attr_set = true;
  }
  const dim3 grid(grid_for(cdiv(a.M, kTM), cdiv(a.N, kTN)), 1, a.nz);
  if (a.cell) hipLaunchKernelGGL(skinny_kernel<true>, grid, dim3(512), kLds, s, a);
  else hipLaunchKernelGGL(skinny_kernel<false>, grid, dim3(512), kLds, s, a);
  return hipGetLastError();
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
