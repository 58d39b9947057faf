// One time step of an LSTM layer for many rows at once (inference, bfloat16 storage): the stepped decoder cell,
// whose input of a step is an embedding concatenated with a context vector (paper Sec. 7, Listing 1: a
// recurrent unit of 1000 cells fed by 620 + 2000 values, stepped once per output word for every beam entry).
//
// With T = 1 nothing can be hoisted and nothing stays resident: the step is ONE dense product
//     z[B, 4n] = [x_t | h_{t-1}] . [W_x ; W_h] + b
// over the concatenated reduction axis (MFMA bound: B = 768 rows against 29 MB of weights), followed by the
// pointwise cell update.  The weights are packed once into the k-contiguous layout of the fast GEMM,
// Wcat[4n][Kc] = [W_x^T | 0 | W_h^T | 0] (x part padded to a multiple of 8, Kc a multiple of 64), and may be
// kept across calls (LSTM_FLAG_WEIGHTS_PACKED).
#include "recurrent_dev.h"

namespace lstm {
namespace {

// Wcat[d][col][k] for a 64 x 64 tile of (k, col): rows of W are read along col, rows of Wcat written along k.
__global__ __launch_bounds__(256) void pack_wcat_kernel(const uint16_t* Wx, const uint16_t* Wh, uint16_t* Wcat, int n_in, int n_in_pad, int n,
                                                        int Kc) {
  __shared__ uint16_t tile[64][66];
  const int N4 = 4 * n;
  const int d = blockIdx.z;
  Wx += (long)d * n_in * N4;
  Wh += (long)d * n * N4;
  Wcat += (long)d * N4 * Kc;
  const int k0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int k = k0 + ty + 4 * i, col = c0 + tx;
    uint16_t v = 0;
    if (col < N4) {
      if (k < n_in) v = Wx[(long)k * N4 + col];
      else if (k >= n_in_pad && k < n_in_pad + n) v = Wh[(long)(k - n_in_pad) * N4 + col];
    }
    tile[ty + 4 * i][tx] = v;
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int col = c0 + ty + 4 * i, k = k0 + tx;
    if (col < N4 && k < Kc) Wcat[(long)col * Kc + k] = tile[tx][ty + 4 * i];
  }
}

// Acat[d][b][k] = x[b][k] (k < n_in), bf16(h[d][b][k - n_in_pad]) (n_in_pad <= k < n_in_pad + n; h == NULL: zeros), 0 elsewhere.
// One thread writes eight consecutive k (16 bytes; Kc and n_in_pad are multiples of 8).
__global__ void concat_kernel(const uint16_t* x, const float* h, uint16_t* Acat, int B, int n_in, int n_in_pad, int n, int Kc, long total8) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total8) return;
  const int k8 = Kc / 8;
  const int k = (int)(idx % k8) * 8;
  const long rest = idx / k8;
  const int b = (int)(rest % B), d = (int)(rest / B);
  uint4 o;
  if (k + 8 <= n_in && n_in % 4 == 0) {                    // whole chunk of x, rows 8-byte aligned
    const uint2* xp = (const uint2*)(x + (long)b * n_in + k);
    const uint2 lo = xp[0], hi = xp[1];
    o = make_uint4(lo.x, lo.y, hi.x, hi.y);
  } else if (h && k >= n_in_pad && k + 8 <= n_in_pad + n && n % 4 == 0 && (((uintptr_t)h) & 15) == 0) {   // whole chunk of h, rows 16-byte aligned
    const float4* hp = (const float4*)(h + ((long)d * B + b) * n + (k - n_in_pad));
    const float4 lo = hp[0], hi = hp[1];
    o.x = f2bf_bits(lo.x) | ((unsigned)f2bf_bits(lo.y) << 16); o.y = f2bf_bits(lo.z) | ((unsigned)f2bf_bits(lo.w) << 16);
    o.z = f2bf_bits(hi.x) | ((unsigned)f2bf_bits(hi.y) << 16); o.w = f2bf_bits(hi.z) | ((unsigned)f2bf_bits(hi.w) << 16);
  } else {
    uint16_t v[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int kk = k + e;
      v[e] = 0;
      if (kk < n_in) v[e] = x[(long)b * n_in + kk];
      else if (h && kk >= n_in_pad && kk < n_in_pad + n) v[e] = f2bf_bits(h[((long)d * B + b) * n + (kk - n_in_pad)]);
    }
    o.x = v[0] | ((unsigned)v[1] << 16); o.y = v[2] | ((unsigned)v[3] << 16);
    o.z = v[4] | ((unsigned)v[5] << 16); o.w = v[6] | ((unsigned)v[7] << 16);
  }
  *(uint4*)(Acat + idx * 8) = o;
}

// Pointwise cell update of the single frame from bias + the partial products.  h_in / c_in: state entering the step
// (NULL = zeros), h_out / c_out: state leaving it (either may be NULL).  A row with length 0 keeps its state and
// outputs zero.  One thread per (row, unit): four units per thread with 16-byte accesses measured slower (too few
// wavefronts left to cover the latency of the partial-product reads).
__global__ void cell_step_kernel(const float* z, long part, int nparts, const float* bias, const float* h_in, const float* c_in,
                                 float* h_out, float* c_out, uint16_t* y, long ldy, float* cs, const int* lens, int B, int n, long total) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int j = (int)(idx % n);
  const long rest = idx / n;
  const int b = (int)(rest % B), d = (int)(rest / B);
  const long si = ((long)d * B + b) * n + j;
  const bool valid = clamp_len(lens, b, 1) > 0;
  float c = c_in ? c_in[si] : 0.f, h = 0.f;
  if (valid) {
    float zh[4] = {0.f, 0.f, 0.f, 0.f};
    if (bias) {
#pragma unroll
      for (int q = 0; q < 4; ++q) zh[q] = bias[(long)d * 4 * n + q * n + j];
    }
    const float* zp = z + (long)d * nparts * part + (long)b * 4 * n + j;
    for (int ks = 0; ks < nparts; ++ks) {
#pragma unroll
      for (int q = 0; q < 4; ++q) zh[q] += __builtin_nontemporal_load(zp + ks * part + q * n);
    }
    const float zx[4] = {0.f, 0.f, 0.f, 0.f};
    const CellOut o = lstm_cell(zh, zx, c);
    c = o.c; h = o.h;
  }
  y[(long)b * ldy + (long)d * n + j] = f2bf_bits(h);
  if (cs) cs[si] = c;
  if (c_out) c_out[si] = c;
  if (h_out) h_out[si] = valid ? h : (h_in ? h_in[si] : 0.f);
}

}  // namespace

hipError_t launch_pack_wcat(const void* W_x, const void* W_h, void* Wcat, int n_in, int n_in_pad, int n, int Kc, int ndir, hipStream_t s) {
  hipLaunchKernelGGL(pack_wcat_kernel, dim3(cdiv(Kc, 64), cdiv(4L * n, 64), ndir), dim3(256), 0, s, (const uint16_t*)W_x, (const uint16_t*)W_h,
                     (uint16_t*)Wcat, n_in, n_in_pad, n, Kc);
  return hipGetLastError();
}
hipError_t launch_concat_xh(const void* x, const float* h, void* Acat, int B, int n_in, int n_in_pad, int n, int Kc, int ndir, hipStream_t s) {
  const long total8 = (long)ndir * B * (Kc / 8);
  if (total8 <= 0) return hipSuccess;
  hipLaunchKernelGGL(concat_kernel, dim3(cdiv(total8, 256)), dim3(256), 0, s, (const uint16_t*)x, h, (uint16_t*)Acat, B, n_in, n_in_pad, n, Kc,
                     total8);
  return hipGetLastError();
}
hipError_t launch_cell_step(const float* z, long part, int nparts, const float* bias, const float* h_in, const float* c_in, float* h_out,
                            float* c_out, void* y, long ldy, float* cs, const int* lens, int B, int n, int ndir, hipStream_t s) {
  const long total = (long)ndir * B * n;
  if (total <= 0) return hipSuccess;
  hipLaunchKernelGGL(cell_step_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, z, part, nparts, bias, h_in, c_in, h_out, c_out, (uint16_t*)y,
                     ldy, cs, lens, B, n, total);
  return hipGetLastError();
}

}  // namespace lstm
