// Persistent recurrent kernels: the whole time loop of a layer in ONE launch.
//
// The per-step kernels pay a launch per time step and re-read their W_h slice from the memory
// system every step.  Here each work-group loads its slice of the packed W_h into registers once
// (bf16, n = 1024: 64 KiB per work-group forward, 128 KiB backward) and then walks all T steps.
// Only h_t (forward) or dz_t (backward) crosses work-groups: it is written in MFMA fragment
// order to a two-deep ring in global memory, and the work-groups of one (direction, row block)
// meet at a monotonically increasing counter between steps:
//
//   producer:  stores ; __syncthreads ; thread 0: release fence (agent scope), counter += 1
//   consumer:  wave 0 polls the counter (bounded), acquire fence (agent scope) ; __syncthreads ; loads
//
// The eight XCDs of the device have separate L2 caches, so the agent-scope fences are what makes
// the ring visible across them.  Two ring slots suffice: a work-group can write slot s for step
// t+1 only after every work-group has signalled step t, i.e. after all reads of slot s for step
// t-1 have been issued and consumed.
//
// Every wait is bounded: when `spin_limit` polls pass without progress the work-group raises the
// error word sync[0] and leaves; all others notice the word in their own waits and leave too, so
// the grid always drains.  The launch is cooperative, which guarantees that all work-groups are
// resident together (otherwise the launch is refused and the caller uses the per-step kernels).
#include "recurrent_dev.h"

namespace lstm {
namespace {

__device__ __forceinline__ unsigned ld_relaxed(const unsigned* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Executed by wave 0 only.  Returns true when *cnt >= target was observed.
__device__ __forceinline__ bool wait_counter(const unsigned* cnt, unsigned target, unsigned* err, unsigned limit) {
  for (unsigned i = 0; i < limit; ++i) {
    if (ld_relaxed(cnt) >= target) return true;
    if ((i & 31u) == 31u && ld_relaxed(err) != 0u) return false;
    __builtin_amdgcn_s_sleep(1);
  }
  __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return false;
}

// ------------------------------------------------------------------------------------------------
template <typename ST, int NIT>
__global__ __launch_bounds__(256) void persist_fwd_kernel(PFwdArgs a) {
  __shared__ float red[4][32][33];
  __shared__ int s_ok;
  const PFwdDir& d = a.d[blockIdx.z];
  const int tile = blockIdx.x, rb = blockIdx.y, ntiles = gridDim.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nkc = a.nkc, n = a.n, B = a.B, T = a.T;
  unsigned* err = a.sync;
  unsigned* cnt = a.sync + 1 + blockIdx.z * gridDim.y + rb;

  // this work-group's slice of W_h, resident in registers for the whole sequence
  uint4 w0[NIT], w1[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int kc = wave + 4 * it;
    w0[it] = w1[it] = make_uint4(0, 0, 0, 0);
    if (kc < nkc) {
      w0[it] = d.Wf[((long)(tile * 2 + 0) * nkc + kc) * 64 + lane];
      w1[it] = d.Wf[((long)(tile * 2 + 1) * nkc + kc) * 64 + lane];
    }
  }

  const int r = tid >> 3, u = tid & 7;
  const int b = rb * 32 + r, j = tile * 8 + u;
  const bool active = b < B && j < n;
  float c = 0.f, h = 0.f;
  int L = 0;
  if (active) {
    c = d.cstate[(long)b * n + j];
    h = d.hstate[(long)b * n + j];
    L = clamp_len(a.lens, b, T);
  }
  const long hoff = active ? frag_offset<ST>(b, j, nkc) : 0;

  for (int tau = 0; tau < T; ++tau) {
    const int t = d.rev ? T - 1 - tau : tau;
    // the input projection of this frame does not depend on the recurrence: fetch it before waiting
    float* gp = d.gates + ((long)t * B + b) * 4 * n + j;
    float zx[4] = {0.f, 0.f, 0.f, 0.f};
    const bool valid = active && t < L;
    if (valid) { zx[0] = gp[0]; zx[1] = gp[n]; zx[2] = gp[2 * n]; zx[3] = gp[3 * n]; }

    if (tau > 0) {
      if (wave == 0) {
        const bool ok = wait_counter(cnt, (unsigned)tau * ntiles, err, a.spin_limit);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        if (lane == 0) s_ok = ok;
      }
      __syncthreads();
      if (!s_ok) break;
    }
    const uint4* hin = (tau & 1) ? d.hfrag1 : d.hfrag0;
    void* hout = (tau & 1) ? (void*)d.hfrag0 : (void*)d.hfrag1;

    f32x4 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) acc[i][jj] = (f32x4){0.f, 0.f, 0.f, 0.f};
    const uint4* hA0 = hin + ((long)(rb * 2 + 0) * nkc) * 64 + lane;
    const uint4* hA1 = hin + ((long)(rb * 2 + 1) * nkc) * 64 + lane;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
      const int kc = wave + 4 * it;
      if (kc < nkc) {
        const uint4 a0 = hA0[(long)kc * 64], a1 = hA1[(long)kc * 64];
        acc[0][0] = Mma16<ST>::run(a0, w0[it], acc[0][0]);
        acc[0][1] = Mma16<ST>::run(a0, w1[it], acc[0][1]);
        acc[1][0] = Mma16<ST>::run(a1, w0[it], acc[1][0]);
        acc[1][1] = Mma16<ST>::run(a1, w1[it], acc[1][1]);
      }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][i * 16 + 4 * (lane >> 4) + v][jj * 16 + (lane & 15)] = acc[i][jj][v];
    __syncthreads();

    if (active) {
      const float h_prev = h;
      float yv = 0.f;
      if (valid) {
        float zh[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) zh[q] = red[0][r][q * 8 + u] + red[1][r][q * 8 + u] + red[2][r][q * 8 + u] + red[3][r][q * 8 + u];
        const CellOut o = lstm_cell(zh, zx, c);
        c = o.c; h = o.h; yv = o.h;
        if (a.write_gates) { gp[0] = o.gi; gp[n] = o.gf; gp[2 * n] = o.gg; gp[3 * n] = o.go; }
      }
      Store<ST>::store(hout, hoff, h);
      Store<ST>::store(d.y, ((long)t * B + b) * d.ldy + j, yv);
      if (d.cs) d.cs[((long)t * B + b) * n + j] = c;
      if (d.hprev) Store<ST>::store(d.hprev, ((long)t * B + b) * n + j, h_prev);
    }
    __syncthreads();
    if (tid == 0) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  if (active) {
    d.cstate[(long)b * n + j] = c;
    d.hstate[(long)b * n + j] = h;
  }
}

// ------------------------------------------------------------------------------------------------
template <typename ST, int NIT>
__global__ __launch_bounds__(256) void persist_bwd_kernel(PBwdArgs a) {
  __shared__ float red[4][16][17];
  __shared__ int s_ok;
  const PBwdDir& d = a.d[blockIdx.z];
  const int tile = blockIdx.x, rt = blockIdx.y, ntiles = gridDim.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nkc = a.nkc, n = a.n, B = a.B, T = a.T;
  unsigned* err = a.sync;
  unsigned* cnt = a.sync + 1 + blockIdx.z * gridDim.y + rt;

  uint4 w[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int kc = wave + 4 * it;
    w[it] = kc < nkc ? d.Wb[((long)tile * nkc + kc) * 64 + lane] : make_uint4(0, 0, 0, 0);
  }

  const int r = tid >> 4, u = tid & 15;
  const int b = rt * 16 + r, j = tile * 16 + u;
  const bool active = b < B && j < n;
  float Dh = 0.f, Dc = 0.f;
  int L = 0;
  if (active) {
    Dh = d.Dh[(long)b * n + j];
    Dc = d.Dc[(long)b * n + j];
    L = clamp_len(a.lens, b, T);
  }
  long zoff[4] = {0, 0, 0, 0};
  if (active) {
#pragma unroll
    for (int q = 0; q < 4; ++q) zoff[q] = frag_offset<ST>(b, q * n + j, nkc);
  }

  for (int tau = T - 1; tau >= -1; --tau) {
    const int t = d.rev ? T - 1 - tau : tau;             // frame of this step (out of range when tau == -1)
    const int t_next = d.rev ? t - 1 : t + 1;            // frame of the previous backward step
    const bool pointwise = tau >= 0;
    const bool valid = pointwise && active && t < L;
    // everything the gate gradients need except Dh is independent of the recurrence: fetch it first
    float gi = 0.f, gf = 0.f, gg = 0.f, go = 0.f, c_new = 0.f, c_prev = 0.f, dyv = 0.f;
    if (valid) {
      const float* gp = d.gates + ((long)t * B + b) * 4 * n + j;
      gi = gp[0]; gf = gp[n]; gg = gp[2 * n]; go = gp[3 * n];
      c_new = d.cs[((long)t * B + b) * n + j];
      const int tp = d.rev ? t + 1 : t - 1;               // frame processed just before t in the forward pass
      if (tp >= 0 && tp < T) c_prev = d.cs[((long)tp * B + b) * n + j];
      else if (d.c0) c_prev = d.c0[(long)b * n + j];
      dyv = Store<ST>::load(d.dy, ((long)t * B + b) * d.lddy + j);
    }

    if (tau < T - 1) {
      if (wave == 0) {
        const bool ok = wait_counter(cnt, (unsigned)(T - 1 - tau) * ntiles, err, a.spin_limit);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        if (lane == 0) s_ok = ok;
      }
      __syncthreads();
      if (!s_ok) break;
      const uint4* zin = ((tau + 1) & 1) ? d.dzfrag1 : d.dzfrag0;
      const uint4* Ap = zin + ((long)rt * nkc) * 64 + lane;
      f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int it = 0; it < NIT; ++it) {
        const int kc = wave + 4 * it;
        if (kc < nkc) acc = Mma16<ST>::run(Ap[(long)kc * 64], w[it], acc);
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) red[wave][4 * (lane >> 4) + v][lane & 15] = acc[v];
      __syncthreads();
      if (active && t_next < L) Dh = red[0][r][u] + red[1][r][u] + red[2][r][u] + red[3][r][u];
    }
    if (pointwise) {
      if (active) {
        float dz[4] = {0.f, 0.f, 0.f, 0.f};
        if (valid) lstm_cell_grad(gi, gf, gg, go, c_new, c_prev, dyv + Dh, Dc, dz);
        void* zout = (tau & 1) ? (void*)d.dzfrag1 : (void*)d.dzfrag0;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          Store<ST>::store(d.DZ, ((long)t * B + b) * 4 * n + q * n + j, dz[q]);
          Store<ST>::store(zout, zoff[q], dz[q]);
        }
      }
      __syncthreads();
      if (tid == 0) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  if (active) {
    d.Dh[(long)b * n + j] = Dh;
    d.Dc[(long)b * n + j] = Dc;
  }
}

template <typename K, typename A>
hipError_t coop(K kernel, dim3 grid, const A& a, hipStream_t s) {
  A copy = a;
  void* args[] = {&copy};
  return hipLaunchCooperativeKernel((const void*)kernel, grid, dim3(256), args, 0, s);
}

}  // namespace

hipError_t launch_persist_fwd(const PFwdArgs& a, bool bf16, hipStream_t s) {
  dim3 grid(cdiv(a.n, 8), cdiv(a.B, 32), a.ndir);
  if (bf16) {
    if (a.nkc > kPersistFwdMaxNkcBf16) return hipErrorCooperativeLaunchTooLarge;
    return coop(persist_fwd_kernel<bf16_t, kPersistFwdMaxNkcBf16 / 4>, grid, a, s);
  }
  if (a.nkc > kPersistFwdMaxNkcF32) return hipErrorCooperativeLaunchTooLarge;
  return coop(persist_fwd_kernel<float, kPersistFwdMaxNkcF32 / 4>, grid, a, s);
}

hipError_t launch_persist_bwd(const PBwdArgs& a, bool bf16, hipStream_t s) {
  dim3 grid(cdiv(a.n, 16), cdiv(a.B, 16), a.ndir);
  if (bf16) {
    if (a.nkc > kPersistBwdMaxNkcBf16) return hipErrorCooperativeLaunchTooLarge;
    return coop(persist_bwd_kernel<bf16_t, kPersistBwdMaxNkcBf16 / 4>, grid, a, s);
  }
  if (a.nkc > kPersistBwdMaxNkcF32) return hipErrorCooperativeLaunchTooLarge;
  return coop(persist_bwd_kernel<float, kPersistBwdMaxNkcF32 / 4>, grid, a, s);
}

}  // namespace lstm
