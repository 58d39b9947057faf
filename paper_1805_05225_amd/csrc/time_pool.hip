// Max-pooling in time between encoder layers (the speech encoder of the paper's attention model on Switchboard pools in
// the time dimension between its bidirectional layers, a factor of 8 in total; window and padding are this library's
// reading: non-overlapping windows of `pool` frames taken inside every sequence, short last window allowed).
//
// Both kernels stream: every input element is read once and every output element written once, 16 bytes per lane
// where the row length allows it.  One work-group handles a few consecutive windows of one row of the batch; the
// bound is HBM.
#include "common.h"

namespace lstm {
namespace {

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kVec = 4;                       // elements per 16 bytes
  __device__ static float get(const uint4& v, int i) { return __uint_as_float(((const unsigned*)&v)[i]); }
  __device__ static void put(uint4& v, int i, float f) { ((unsigned*)&v)[i] = __float_as_uint(f); }
};
template <> struct Elem<bf16_t> {
  static constexpr int kVec = 8;
  __device__ static float get(const uint4& v, int i) { return bf_bits2f(((const uint16_t*)&v)[i]); }
  __device__ static void put(uint4& v, int i, float f) { ((uint16_t*)&v)[i] = f2bf_bits(f); }     // f is a bf16 value already: exact
};

__device__ __forceinline__ int row_len(const int* lens, int b, int T) {
  if (!lens) return T;
  const int L = lens[b];
  return L < 0 ? 0 : (L > T ? T : L);
}

constexpr int kFramesPerBlock = 4;                     // output frames one work-group handles: enough loads in flight per lane to stream

// out[tp][b][:] = max over the valid frames of window tp of row b; arg = offset of the earliest maximum; zero where
// the output frame is padding.  VEC: 16-byte accesses (F a multiple of the vector width, aligned rows).
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void time_pool_fwd_kernel(const T* __restrict__ y, long ldy, const int* __restrict__ lens, T* __restrict__ out,
                                                             long ldo, uint8_t* __restrict__ arg, int* __restrict__ lens_out, int Tn, int B,
                                                             int F, int pool) {
  constexpr int V = VEC ? Elem<T>::kVec : 1;
  const int b = blockIdx.y;
  const int L = row_len(lens, b, Tn), Tp = (Tn + pool - 1) / pool;
  if (blockIdx.x == 0 && threadIdx.x == 0 && lens_out) lens_out[b] = (L + pool - 1) / pool;
  for (int f = threadIdx.x * V; f < F; f += blockDim.x * V) {
#pragma unroll
    for (int k = 0; k < kFramesPerBlock; ++k) {
      const int tp = blockIdx.x * kFramesPerBlock + k;
      if (tp >= Tp) break;
      const int t0 = tp * pool, t1 = min(t0 + pool, L);
      const long orow = (long)tp * B + b;
      float best[V];
      uint8_t which[V];
#pragma unroll
      for (int i = 0; i < V; ++i) { best[i] = 0.f; which[i] = 0; }
      for (int t = t0; t < t1; ++t) {
        const T* src = y + ((long)t * B + b) * ldy + f;
        float v[V];
        if (VEC) {
          typedef __attribute__((ext_vector_type(4))) unsigned u32x4_;
          const u32x4_ r4 = __builtin_nontemporal_load((const u32x4_*)src);      // read once: keep it out of the caches' way
          const uint4 raw = make_uint4(r4[0], r4[1], r4[2], r4[3]);
#pragma unroll
          for (int i = 0; i < V; ++i) v[i] = Elem<T>::get(raw, i);
        } else {
          v[0] = Store<T>::load(src, 0);
        }
#pragma unroll
        for (int i = 0; i < V; ++i)
          if (t == t0 || v[i] > best[i]) { best[i] = v[i]; which[i] = (uint8_t)(t - t0); }     // strictly greater: ties keep the earliest
      }
      if (VEC) {
        uint4 o;
#pragma unroll
        for (int i = 0; i < V; ++i) Elem<T>::put(o, i, best[i]);
        *(uint4*)(out + orow * ldo + f) = o;
      } else {
        Store<T>::store(out, orow * ldo + f, best[0]);
      }
      if (arg && t0 < L) {                                     // padded output frames: the backward pass never reads their bytes
        if (VEC) {                                             // V bytes at once (F, hence every row of arg, is a multiple of V)
          unsigned w[2] = {0u, 0u};
#pragma unroll
          for (int i = 0; i < V; ++i) w[i >> 2] |= (unsigned)which[i] << (8 * (i & 3));
          if (V == 8) *(uint2*)(arg + orow * F + f) = make_uint2(w[0], w[1]);
          else *(unsigned*)(arg + orow * F + f) = w[0];
        } else {
          arg[orow * F + f] = which[0];
        }
      }
    }
  }
}

// The frames of window tp of row b: dy = dout[tp] where arg says the frame supplied the maximum, else 0; padded frames 0.
// dout and arg are read once per window, every frame of dy is written (zeros included: nothing has to be cleared first).
template <typename T, bool VEC>
__global__ __launch_bounds__(256) void time_pool_bwd_kernel(const T* __restrict__ dout, long ldo, const uint8_t* __restrict__ arg,
                                                             const int* __restrict__ lens, T* __restrict__ dy, long ldy, int Tn, int B, int F,
                                                             int pool) {
  constexpr int V = VEC ? Elem<T>::kVec : 1;
  const int b = blockIdx.y;
  const int L = row_len(lens, b, Tn), Tp = (Tn + pool - 1) / pool;
  for (int f = threadIdx.x * V; f < F; f += blockDim.x * V) {
#pragma unroll
    for (int k = 0; k < kFramesPerBlock; ++k) {
      const int tp = blockIdx.x * kFramesPerBlock + k;
      if (tp >= Tp) break;
      const int t0 = tp * pool, t1 = min(t0 + pool, Tn);
      const long orow = (long)tp * B + b;
      const bool any = t0 < L;                                 // the window holds at least one valid frame
      uint4 g = make_uint4(0, 0, 0, 0);
      uint8_t which[V];
#pragma unroll
      for (int i = 0; i < V; ++i) which[i] = 0;
      float g1 = 0.f;
      if (any) {
        if (VEC) {
          g = *(const uint4*)(dout + orow * ldo + f);
          unsigned w[2] = {0u, 0u};
          if (V == 8) { const uint2 a2 = *(const uint2*)(arg + orow * F + f); w[0] = a2.x; w[1] = a2.y; }
          else w[0] = *(const unsigned*)(arg + orow * F + f);
#pragma unroll
          for (int i = 0; i < V; ++i) which[i] = (uint8_t)(w[i >> 2] >> (8 * (i & 3)));
        } else {
          g1 = Store<T>::load(dout, orow * ldo + f);
          which[0] = arg[orow * F + f];
        }
      }
      for (int t = t0; t < t1; ++t) {
        const long irow = (long)t * B + b;
        const int off = t - t0;
        if (VEC) {
          uint4 o = make_uint4(0, 0, 0, 0);
          if (t < L) {
#pragma unroll
            for (int i = 0; i < V; ++i)
              if (which[i] == off) Elem<T>::put(o, i, Elem<T>::get(g, i));
          }
          *(uint4*)(dy + irow * ldy + f) = o;
        } else {
          Store<T>::store(dy, irow * ldy + f, (t < L && which[0] == off) ? g1 : 0.f);
        }
      }
    }
  }
}

template <typename T>
hipError_t pool_fwd(const void* y, long ldy, const int* lens, void* out, long ldo, uint8_t* arg, int* lens_out, int Tn, int B, int F, int pool,
                    hipStream_t s) {
  const int Tp = (Tn + pool - 1) / pool;
  if (Tp == 0 || B == 0) return hipSuccess;
  constexpr int V = Elem<T>::kVec;
  const bool vec = F % V == 0 && ldy % V == 0 && ldo % V == 0 && (((uintptr_t)y | (uintptr_t)out) & 15u) == 0;
  const dim3 grid((Tp + kFramesPerBlock - 1) / kFramesPerBlock, B);
  if (vec) hipLaunchKernelGGL((time_pool_fwd_kernel<T, true>), grid, dim3(256), 0, s, (const T*)y, ldy, lens, (T*)out, ldo, arg, lens_out, Tn, B, F, pool);
  else hipLaunchKernelGGL((time_pool_fwd_kernel<T, false>), grid, dim3(256), 0, s, (const T*)y, ldy, lens, (T*)out, ldo, arg, lens_out, Tn, B, F, pool);
  return hipGetLastError();
}
template <typename T>
hipError_t pool_bwd(const void* dout, long ldo, const uint8_t* arg, const int* lens, void* dy, long ldy, int Tn, int B, int F, int pool,
                    hipStream_t s) {
  if (Tn == 0 || B == 0) return hipSuccess;
  constexpr int V = Elem<T>::kVec;
  const bool vec = F % V == 0 && ldy % V == 0 && ldo % V == 0 && (((uintptr_t)dy | (uintptr_t)dout) & 15u) == 0;
  const dim3 grid(((Tn + pool - 1) / pool + kFramesPerBlock - 1) / kFramesPerBlock, B);
  if (vec) hipLaunchKernelGGL((time_pool_bwd_kernel<T, true>), grid, dim3(256), 0, s, (const T*)dout, ldo, arg, lens, (T*)dy, ldy, Tn, B, F, pool);
  else hipLaunchKernelGGL((time_pool_bwd_kernel<T, false>), grid, dim3(256), 0, s, (const T*)dout, ldo, arg, lens, (T*)dy, ldy, Tn, B, F, pool);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_time_pool_fwd(bool bf16, const void* y, long ldy, const int* lens, void* out, long ldo, uint8_t* arg, int* lens_out, int T,
                                int B, int F, int pool, hipStream_t s) {
  return bf16 ? pool_fwd<bf16_t>(y, ldy, lens, out, ldo, arg, lens_out, T, B, F, pool, s)
              : pool_fwd<float>(y, ldy, lens, out, ldo, arg, lens_out, T, B, F, pool, s);
}
hipError_t launch_time_pool_bwd(bool bf16, const void* dout, long ldo, const uint8_t* arg, const int* lens, void* dy, long ldy, int T, int B,
                                int F, int pool, hipStream_t s) {
  return bf16 ? pool_bwd<bf16_t>(dout, ldo, arg, lens, dy, ldy, T, B, F, pool, s)
              : pool_bwd<float>(dout, ldo, arg, lens, dy, ldy, T, B, F, pool, s);
}

}  // namespace lstm
