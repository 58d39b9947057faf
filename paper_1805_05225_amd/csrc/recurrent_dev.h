// Device helpers shared by the per-step and the persistent recurrent kernels.
#pragma once
#include "common.h"

namespace lstm {
namespace {

// Frame map of a batch of end-padded sequences (see launch_frame_map), the work of one block of 256 threads: four time steps,
// one wavefront each.  Shared by the kernel of its own and by the set-up kernel of the single-launch loops.
__device__ __forceinline__ void frame_map_body(int block, const int* lens, int T, int B, int* cidx, int* fidx, int* count) {
  const int lane = threadIdx.x & 63;
  const int t = block * 4 + (threadIdx.x >> 6);
  if (t >= T) return;
  // kept frames before time t: sum over b of min(len_b, t)
  long before = 0, all = 0;
  for (int b = lane; b < B; b += 64) {
    int L = lens[b];
    L = L < 0 ? 0 : (L > T ? T : L);
    before += L < t ? L : t;
    all += L;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    before += __shfl_xor(before, o);
    all += __shfl_xor(all, o);
  }
  if (t == 0 && lane == 0) {
    count[0] = (int)all;
    count[1] = (int)((all + 63) / 64 * 64);
  }
  int base = (int)before;
  for (int b0 = 0; b0 < B; b0 += 64) {
    const int b = b0 + lane;
    bool keep = false;
    if (b < B) {
      int L = lens[b];
      L = L < 0 ? 0 : (L > T ? T : L);
      keep = t < L;
    }
    const unsigned long long m = __builtin_amdgcn_ballot_w64(keep);
    const int mine = base + __popcll(m & ((1ull << lane) - 1ull));
    if (b < B) cidx[(long)t * B + b] = keep ? mine : -1;
    if (keep) fidx[mine] = t * B + b;
    base += __popcll(m);
  }
}

template <typename T> struct Mma16;
template <> struct Mma16<bf16_t> {
  __device__ static f32x4 run(uint4 a, uint4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
};
template <> struct Mma16<float> {
  __device__ static f32x4 run(uint4 a, uint4 b, f32x4 c) {
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.x), __uint_as_float(b.x), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.y), __uint_as_float(b.y), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.z), __uint_as_float(b.z), c, 0, 0, 0);
    c = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(a.w), __uint_as_float(b.w), c, 0, 0, 0);
    return c;
  }
};

// element offset (in elements of T) of (row, k) inside a fragment-ordered buffer with nkc chunks per row tile
template <typename T>
__device__ __forceinline__ long frag_offset(int row, int k, int nkc) {
  constexpr int E = Store<T>::kPerChunk, KC = 4 * E;
  int rt = row >> 4, r = row & 15;
  int kc = k / KC, rem = k - kc * KC;
  int g = rem / E, e = rem - g * E;
  return ((((long)rt * nkc + kc) * 64 + g * 16 + r) * E + e);
}

// Reciprocals through the hardware approximation (1 ulp): a correctly rounded float division is ten dependent
// instructions, and with one wavefront per SIMD the recurrent kernels pay for every one of them in every step.
__device__ __forceinline__ float sigmoidf_(float x) { return __builtin_amdgcn_rcpf(1.f + __expf(-x)); }
__device__ __forceinline__ float tanhf_(float x) { return 1.f - 2.f * __builtin_amdgcn_rcpf(1.f + __expf(2.f * x)); }
__device__ __forceinline__ int clamp_len(const int* lens, int b, int T) {
  if (!lens) return T;
  int L = lens[b];
  return L < 0 ? 0 : (L > T ? T : L);
}


// One LSTM cell update in float.  zh = h W_h part, zx = x W_x + b part, both ordered i|f|g|o.
struct CellOut { float gi, gf, gg, go, c, h; };
__device__ __forceinline__ CellOut lstm_cell(const float (&zh)[4], const float (&zx)[4], float c_prev) {
  CellOut o;
  o.gi = sigmoidf_(zh[0] + zx[0]);
  o.gf = sigmoidf_(zh[1] + zx[1]);
  o.gg = tanhf_(zh[2] + zx[2]);
  o.go = sigmoidf_(zh[3] + zx[3]);
  o.c = o.gf * c_prev + o.gi * o.gg;
  o.h = o.go * tanhf_(o.c);
  return o;
}
// Gate gradients of one valid frame.  dh = dy + carried Dh; Dc is updated in place.
__device__ __forceinline__ void lstm_cell_grad(float gi, float gf, float gg, float go, float c_new, float c_prev, float dh,
                                               float& Dc, float (&dz)[4]) {
  const float tc = tanhf_(c_new);
  const float dc = Dc + dh * go * (1.f - tc * tc);
  Dc = dc * gf;
  dz[0] = dc * gg * gi * (1.f - gi);
  dz[1] = dc * c_prev * gf * (1.f - gf);
  dz[2] = dc * gi * (1.f - gg * gg);
  dz[3] = dh * tc * go * (1.f - go);
}

}  // namespace
}  // namespace lstm
