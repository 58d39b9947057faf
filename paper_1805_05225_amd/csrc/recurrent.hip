// The recurrent part of the LSTM layer: what cannot leave the time loop.
//
// Forward step  (one launch per time step, both directions of a bidirectional layer in the same
// launch):   z_t = Zx_t + h W_h ;  gates ;  c' = f c + i g ;  h' = o tanh(c') ;  sequence mask.
// Backward step:  Dh = dz_{next} W_h^T  (the matrix product of the previous backward step's gate
// gradients), then the gate gradients dz_t of this frame.
//
// Decomposition.  A work-group owns a few hidden units and ALL of their gate columns
// (forward: 8 units = 32 columns for 32 batch rows; backward: 16 units for 16 batch rows).  So the cell update
// is local to the work-group and only h_t (forward) or dz_t (backward) crosses work-groups
// between steps.  The small-M product runs on MFMA 16x16 tiles with the K axis split over the
// four wavefronts, followed by a reduction through LDS and the pointwise epilogue.
//
// Operands are kept in "fragment order": the exact register image of an MFMA operand, one
// 16-byte chunk per lane, so every operand load is one fully coalesced 1 KiB read per wavefront:
//   chunk (tile, kc, lane = g*16 + r) element e  <->  row/col r of the 16-wide tile,
//   k = kc*KC + g*E + e,  E = elements per 16 bytes, KC = 4E.
// W_h is packed once per call; h_t / dz_t are written in this order by the step that makes them.
#include "recurrent_dev.h"

namespace lstm {
namespace {

// Work-group -> (unit tile, row block, direction).  The work-groups that share a unit tile read the same slice of the
// packed W_h, 32 MB in all for two directions of n = 1000 in float: as much as the eight XCDs' L2 caches hold together,
// so it streams in from the memory side in every step - once per row block if those work-groups sit on different
// XCDs.  Work-groups are dealt to the XCDs round-robin in launch order, so the row blocks of one unit tile are given
// numbers 8 apart: they run on one XCD at about the same time and the slice comes in once.
struct StepCoord { int tile, rb, dir; bool live; };
__device__ __forceinline__ StepCoord step_coord(int ntile, int nrb) {
  const int ntile8 = (ntile + 7) / 8;
  const int lin = blockIdx.x, t8 = lin & 7, r = lin >> 3;
  StepCoord c;
  c.rb = r % nrb;
  const int g = r / nrb;
  c.tile = (g % ntile8) * 8 + t8;
  c.dir = g / ntile8;
  c.live = c.tile < ntile;
  return c;
}
inline int step_grid(int ntile, int nrb, int ndir) { return ndir * ((ntile + 7) / 8) * nrb * 8; }

// ------------------------------------------------------------------------------------------------
// forward step
template <typename T>
__global__ __launch_bounds__(256) void step_fwd_kernel(FwdArgs a) {
  __shared__ float red[4][32][33];
  const StepCoord sc = step_coord((a.n + 7) / 8, (a.B + 31) / 32);
  if (!sc.live) return;
  const FwdDir& d = a.d[sc.dir];
  const int tile = sc.tile, rb = sc.rb;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nkc = a.nkc;

  f32x4 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = (f32x4){0.f, 0.f, 0.f, 0.f};

  const uint4* hA0 = d.hin + ((long)(rb * 2 + 0) * nkc) * 64 + lane;
  const uint4* hA1 = d.hin + ((long)(rb * 2 + 1) * nkc) * 64 + lane;
  const uint4* wB0 = d.Wf + ((long)(tile * 2 + 0) * nkc) * 64 + lane;
  const uint4* wB1 = d.Wf + ((long)(tile * 2 + 1) * nkc) * 64 + lane;
#pragma unroll 4
  for (int kc = wave; kc < nkc; kc += 4) {
    uint4 a0 = hA0[(long)kc * 64], a1 = hA1[(long)kc * 64];
    uint4 b0 = wB0[(long)kc * 64], b1 = wB1[(long)kc * 64];
    acc[0][0] = Mma16<T>::run(a0, b0, acc[0][0]);
    acc[0][1] = Mma16<T>::run(a0, b1, acc[0][1]);
    acc[1][0] = Mma16<T>::run(a1, b0, acc[1][0]);
    acc[1][1] = Mma16<T>::run(a1, b1, acc[1][1]);
  }
  // accumulator of a 16x16 block: lane holds column lane%16, rows 4*(lane/16) + v
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) red[wave][i * 16 + 4 * (lane >> 4) + v][j * 16 + (lane & 15)] = acc[i][j][v];
  __syncthreads();

  const int r = tid >> 3, u = tid & 7;
  const int b = rb * 32 + r, j = tile * 8 + u;
  if (b >= a.B || j >= a.n) return;
  float z[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) z[q] = red[0][r][q * 8 + u] + red[1][r][q * 8 + u] + red[2][r][q * 8 + u] + red[3][r][q * 8 + u];

  const int n = a.n;
  const bool valid = d.t < clamp_len(a.lens, b, a.T);
  float* gp = d.gates + (long)b * 4 * n + j;
  const float c_prev = d.cstate[(long)b * n + j];
  const float h_prev = d.hstate[(long)b * n + j];
  float h_new = h_prev, c_new = c_prev, yv = 0.f;
  if (valid) {
    const float gi = sigmoidf_(z[0] + gp[0]);
    const float gf = sigmoidf_(z[1] + gp[n]);
    const float gg = tanhf_(z[2] + gp[2 * n]);
    const float go = sigmoidf_(z[3] + gp[3 * n]);
    c_new = gf * c_prev + gi * gg;
    h_new = go * tanhf_(c_new);
    yv = h_new;
    if (a.write_gates) { gp[0] = gi; gp[n] = gf; gp[2 * n] = gg; gp[3 * n] = go; }
    d.cstate[(long)b * n + j] = c_new;
    d.hstate[(long)b * n + j] = h_new;
  }
  Store<T>::store(d.hout, frag_offset<T>(b, j, nkc), h_new);
  Store<T>::store(d.y, (long)b * d.ldy + j, yv);
  if (d.cs) d.cs[(long)b * n + j] = c_new;
  if (d.hprev) Store<T>::store(d.hprev, (long)b * n + j, h_prev);
}

// ------------------------------------------------------------------------------------------------
// backward step: a work-group owns 16 units for one tile of 16 batch rows
template <typename T>
__global__ __launch_bounds__(256) void step_bwd_kernel(BwdArgs a) {
  __shared__ float red[4][16][17];
  const StepCoord sc = step_coord((a.n + 15) / 16, (a.B + 15) / 16);
  if (!sc.live) return;
  const BwdDir& d = a.d[sc.dir];
  const int tile = sc.tile, rt = sc.rb;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nkc = a.nkc, n = a.n;

  if (a.do_matmul) {
    f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
    const uint4* Ap = d.dzin + ((long)rt * nkc) * 64 + lane;
    const uint4* Bp = d.Wb + ((long)tile * nkc) * 64 + lane;
#pragma unroll 8
    for (int kc = wave; kc < nkc; kc += 4) acc = Mma16<T>::run(Ap[(long)kc * 64], Bp[(long)kc * 64], acc);
#pragma unroll
    for (int v = 0; v < 4; ++v) red[wave][4 * (lane >> 4) + v][lane & 15] = acc[v];
  }
  __syncthreads();

  const int r = tid >> 4, u = tid & 15;
  const int b = rt * 16 + r, j = tile * 16 + u;
  if (b >= a.B || j >= n) return;
  const int L = clamp_len(a.lens, b, a.T);
  float Dh = d.Dh[(long)b * n + j];
  if (a.do_matmul && d.t_next < L) Dh = red[0][r][u] + red[1][r][u] + red[2][r][u] + red[3][r][u];
  d.Dh[(long)b * n + j] = Dh;
  if (!a.do_pointwise) return;
  float dz[4] = {0.f, 0.f, 0.f, 0.f};
  if (d.t < L) {
    const float* gp = d.gates + (long)b * 4 * n + j;
    const float c_prev = d.cprev ? d.cprev[(long)b * n + j] : 0.f;
    const float dh = Store<T>::load(d.dy, (long)b * d.lddy + j) + Dh;
    float Dc = d.Dc[(long)b * n + j];
    lstm_cell_grad(gp[0], gp[n], gp[2 * n], gp[3 * n], d.cs[(long)b * n + j], c_prev, dh, Dc, dz);
    d.Dc[(long)b * n + j] = Dc;
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    Store<T>::store(d.DZ, (long)b * 4 * n + q * n + j, dz[q]);
    Store<T>::store(d.dzout, frag_offset<T>(b, q * n + j, nkc), dz[q]);
  }
}

// ------------------------------------------------------------------------------------------------
// packing
// forward: chunk index = ((dir*ntiles + tile)*2 + ct)*nkc + kc)*64 + lane ; column ct*16 + (lane%16) of the
// work-group's 32 columns is gate q = col/8, unit tile*8 + col%8.
template <typename T>
__global__ void pack_wh_fwd_kernel(const T* W, uint4* out, int n, int nkc, long total) {
  constexpr int E = Store<T>::kPerChunk, KC = 4 * E;
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  int lane = idx & 63;
  long rest = idx >> 6;
  int kc = rest % nkc; rest /= nkc;
  int ct = rest & 1; rest >>= 1;
  int ntiles = (n + 7) / 8;
  int tile = rest % ntiles;
  int dir = rest / ntiles;
  int col = ct * 16 + (lane & 15), g = lane >> 4;
  int q = col >> 3, unit = tile * 8 + (col & 7);
  const T* Wd = W + (long)dir * n * 4 * n;
  T v[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    int k = kc * KC + g * E + e;
    v[e] = (k < n && unit < n) ? Wd[(long)k * 4 * n + q * n + unit] : (T)0.f;
  }
  out[idx] = *(uint4*)v;
}
// backward: chunk index = ((dir*ntiles + tile)*nkc + kc)*64 + lane ; column lane%16 = unit tile*16 + c,
// k runs over the 4n gate columns: element = W_h[unit][k]
template <typename T>
__global__ void pack_wh_bwd_kernel(const T* W, uint4* out, int n, int nkc, long total) {
  constexpr int E = Store<T>::kPerChunk, KC = 4 * E;
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  int lane = idx & 63;
  long rest = idx >> 6;
  int kc = rest % nkc; rest /= nkc;
  int ntiles = (n + 15) / 16;
  int tile = rest % ntiles;
  int dir = rest / ntiles;
  int unit = tile * 16 + (lane & 15), g = lane >> 4;
  const T* Wd = W + (long)dir * n * 4 * n;
  T v[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    int k = kc * KC + g * E + e;
    v[e] = (k < 4 * n && unit < n) ? Wd[(long)unit * 4 * n + k] : (T)0.f;
  }
  out[idx] = *(uint4*)v;
}
// state: chunk index = ((dir*nrt + rt)*nkc + kc)*64 + lane
template <typename T>
__global__ void pack_state_kernel(const float* h, uint4* f0, uint4* f1, int B, int n, int nkc, int nrt, long total) {
  constexpr int E = Store<T>::kPerChunk, KC = 4 * E;
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  int lane = idx & 63;
  long rest = idx >> 6;
  int kc = rest % nkc; rest /= nkc;
  int rt = rest % nrt;
  int dir = rest / nrt;
  int row = rt * 16 + (lane & 15), g = lane >> 4;
  T v[E];
#pragma unroll
  for (int e = 0; e < E; ++e) {
    int k = kc * KC + g * E + e;
    v[e] = (row < B && k < n) ? (T)h[((long)dir * B + row) * n + k] : (T)0.f;
  }
  f0[idx] = *(uint4*)v;
  f1[idx] = *(uint4*)v;
}

__global__ void fill_zero_kernel(uint32_t* p, size_t nwords, int tail16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
  if (i == 0 && tail16) ((uint16_t*)(p + nwords))[0] = 0;
  for (; i < nwords; i += stride) p[i] = 0u;
}
// several fills in one launch: block b works on the region whose block range holds b
__global__ void fill_zero_many_kernel(ZeroRegions r) {
  int k = 0;
#pragma unroll
  for (int j = 1; j < ZeroRegions::kMax; ++j)
    if (j < r.count && (int)blockIdx.x >= r.first_block[j]) k = j;
  uint32_t* p = (uint32_t*)r.ptr[k];
  const size_t nwords = r.words[k];
  const size_t nb = (size_t)(r.first_block[k + 1] - r.first_block[k]);
  size_t i = (size_t)(blockIdx.x - r.first_block[k]) * blockDim.x + threadIdx.x;
  for (; i < nwords; i += nb * blockDim.x) p[i] = 0u;
}
__global__ void copy_kernel(uint32_t* dst, const uint32_t* src, size_t nwords) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x, stride = (size_t)gridDim.x * blockDim.x;
  for (; i < nwords; i += stride) dst[i] = src[i];
}

// column sums in two deterministic passes: partial sums over row slices, then a sum over slices
constexpr int kColsumSplit = kColsumSlices;
template <typename T>
__global__ void colsum_part_kernel(const T* DZ, float* part, int rows, int ncols, long sDZ) {
  int c = blockIdx.x * blockDim.x + threadIdx.x, sp = blockIdx.y, dir = blockIdx.z;
  if (c >= ncols) return;
  int per = (rows + kColsumSplit - 1) / kColsumSplit;
  int r0 = sp * per, r1 = min(rows, r0 + per);
  const T* p = DZ + dir * sDZ;
  float s = 0.f;
  for (int r = r0; r < r1; ++r) s += (float)p[(long)r * ncols + c];
  part[((long)dir * kColsumSplit + sp) * ncols + c] = s;
}
__global__ void colsum_final_kernel(const float* part, float* db, int ncols, int nslices, int accumulate) {
  int c = blockIdx.x * blockDim.x + threadIdx.x, dir = blockIdx.y;
  if (c >= ncols) return;
  float s = 0.f;
  const float* p = part + (long)dir * kColsumSplit * ncols + c;
  int sp = 0;
  for (; sp + 8 <= nslices; sp += 8) {                   // eight loads in flight (one at a time, each costs a trip to memory)
    float v[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) v[k] = p[(long)(sp + k) * ncols];
#pragma unroll
    for (int k = 0; k < 8; ++k) s += v[k];
  }
  for (; sp < nslices; ++sp) s += p[(long)sp * ncols];
  float* o = db + (long)dir * ncols + c;
  *o = accumulate ? *o + s : s;
}

}  // namespace

hipError_t launch_step_fwd(const FwdArgs& a, bool bf16, hipStream_t s) {
  dim3 grid(step_grid(cdiv(a.n, 8), cdiv(a.B, 32), a.ndir)), block(256);
  if (bf16) hipLaunchKernelGGL(step_fwd_kernel<bf16_t>, grid, block, 0, s, a);
  else hipLaunchKernelGGL(step_fwd_kernel<float>, grid, block, 0, s, a);
  return hipGetLastError();
}
hipError_t launch_step_bwd(const BwdArgs& a, bool bf16, hipStream_t s) {
  dim3 grid(step_grid(cdiv(a.n, 16), cdiv(a.B, 16), a.ndir)), block(256);
  if (bf16) hipLaunchKernelGGL(step_bwd_kernel<bf16_t>, grid, block, 0, s, a);
  else hipLaunchKernelGGL(step_bwd_kernel<float>, grid, block, 0, s, a);
  return hipGetLastError();
}
hipError_t launch_pack_wh_fwd(const void* W, uint4* Wf, int n, int nkc, int ndir, bool bf16, hipStream_t s) {
  long total = (long)ndir * cdiv(n, 8) * 2 * nkc * 64;
  dim3 grid(cdiv(total, 256)), block(256);
  if (bf16) hipLaunchKernelGGL(pack_wh_fwd_kernel<bf16_t>, grid, block, 0, s, (const bf16_t*)W, Wf, n, nkc, total);
  else hipLaunchKernelGGL(pack_wh_fwd_kernel<float>, grid, block, 0, s, (const float*)W, Wf, n, nkc, total);
  return hipGetLastError();
}
hipError_t launch_pack_wh_bwd(const void* W, uint4* Wb, int n, int nkc, int ndir, bool bf16, hipStream_t s) {
  long total = (long)ndir * cdiv(n, 16) * nkc * 64;
  dim3 grid(cdiv(total, 256)), block(256);
  if (bf16) hipLaunchKernelGGL(pack_wh_bwd_kernel<bf16_t>, grid, block, 0, s, (const bf16_t*)W, Wb, n, nkc, total);
  else hipLaunchKernelGGL(pack_wh_bwd_kernel<float>, grid, block, 0, s, (const float*)W, Wb, n, nkc, total);
  return hipGetLastError();
}
hipError_t launch_pack_state(const float* h, uint4* f0, uint4* f1, int B, int n, int nkc, int nrt, int ndir, bool bf16,
                             hipStream_t s) {
  long total = (long)ndir * nrt * nkc * 64;
  dim3 grid(cdiv(total, 256)), block(256);
  if (bf16) hipLaunchKernelGGL(pack_state_kernel<bf16_t>, grid, block, 0, s, h, f0, f1, B, n, nkc, nrt, total);
  else hipLaunchKernelGGL(pack_state_kernel<float>, grid, block, 0, s, h, f0, f1, B, n, nkc, nrt, total);
  return hipGetLastError();
}
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  size_t nw = bytes / 4;
  int blocks = (int)((nw + 255) / 256 > 4096 ? 4096 : (nw + 255) / 256);
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, s, (uint32_t*)p, nw, (int)((bytes & 2) != 0));
  return hipGetLastError();
}
void ZeroRegions::add(void* p, size_t bytes) {
  if (bytes == 0 || count >= kMax) { overflow |= bytes != 0; return; }
  const size_t nw = bytes / 4;
  const size_t blocks = std::min<size_t>((nw + 1023) / 1024, 512);      // a few words per lane
  ptr[count] = p; words[count] = nw;
  first_block[count + 1] = first_block[count] + (int)std::max<size_t>(blocks, 1);
  ++count;
}
hipError_t launch_fill_zero_many(const ZeroRegions& r, hipStream_t s) {
  if (r.overflow) return hipErrorInvalidValue;
  if (r.count == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_many_kernel, dim3(r.first_block[r.count]), dim3(256), 0, s, r);
  return hipGetLastError();
}
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s) {
  if (bytes == 0) return hipSuccess;
  size_t nw = bytes / 4;
  int blocks = (int)((nw + 255) / 256 > 4096 ? 4096 : (nw + 255) / 256);
  hipLaunchKernelGGL(copy_kernel, dim3(blocks), dim3(256), 0, s, (uint32_t*)dst, (const uint32_t*)src, nw);
  return hipGetLastError();
}
hipError_t launch_colsum(const void* DZ, float* db, float* part, int rows, int ncols, int ndir, long sDZ, bool bf16,
                         int accumulate, hipStream_t s) {
  dim3 grid(cdiv(ncols, 256), kColsumSplit, ndir), block(256);
  if (bf16) hipLaunchKernelGGL(colsum_part_kernel<bf16_t>, grid, block, 0, s, (const bf16_t*)DZ, part, rows, ncols, sDZ);
  else hipLaunchKernelGGL(colsum_part_kernel<float>, grid, block, 0, s, (const float*)DZ, part, rows, ncols, sDZ);
  hipLaunchKernelGGL(colsum_final_kernel, dim3(cdiv(ncols, 256), ndir), block, 0, s, part, db, ncols, kColsumSplit, accumulate);
  return hipGetLastError();
}
hipError_t launch_colsum_final(const float* part, float* db, int ncols, int ndir, int nslices, int accumulate, hipStream_t s) {
  hipLaunchKernelGGL(colsum_final_kernel, dim3(cdiv(ncols, 256), ndir), dim3(256), 0, s, part, db, ncols, nslices, accumulate);
  return hipGetLastError();
}

}  // namespace lstm
