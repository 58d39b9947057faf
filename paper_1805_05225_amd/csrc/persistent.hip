// Single-launch recurrent kernels: the whole time loop of a layer in ONE launch (bfloat16 storage).
//
// The per-step kernels pay a launch per time step and re-read their W_h slice from the memory
// system every step.  Here each work-group (16 hidden units x 16 batch rows) loads its slice of
// the packed W_h into registers once and then walks all T steps.
//
// Only h_t (forward) or dz_t (backward) crosses work-groups.  Measurements on this device showed
// that a counter barrier is the wrong tool: atomics on one address serialise at ~16 ns each
// (4 us for 256 work-groups) and agent-scope fences cost microseconds more.  So there is no
// barrier and no fence here.  The exchanged data lives in a two-slot ring whose every 8-byte unit
// holds three bf16 values and a 16-bit step tag, written with one 64-bit agent-scope atomic store
// and read with cache-bypassing 16-byte loads.  A consumer simply re-reads its operands until
// every tag shows the step it is waiting for: value and "ready" flag arrive in the same atomic
// unit, so no ordering between different addresses is ever needed.
//
// Two ring slots suffice: a work-group writes slot s for step t+1 only after it has seen every
// tag of step t, i.e. after every work-group has finished step t and therefore finished reading
// slot s (which held step t-1).
//
// Every wait is bounded: after `spin_limit` polls the wave raises the error word sync[0], stops
// waiting for the rest of the launch and runs to the end (results are then invalid and the word
// says so); every other wave notices the word in its own wait loop and does the same, so the
// grid always drains.  The launch is cooperative, which guarantees that all work-groups are
// resident together (otherwise the launch is refused and the caller uses the per-step kernels).
#include "recurrent_dev.h"

namespace lstm {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// Optional in-kernel phase clocks (build with -DLSTM_PROF; prints from a few work-groups at the end).
#ifdef LSTM_PROF
#define PROF_DECL long long pt_[8] = {0, 0, 0, 0, 0, 0, 0, 0}; long long pc_ = wall_clock64(); unsigned npoll_ = 0;
#define PROF_MARK(i) { long long now_ = wall_clock64(); pt_[i] += now_ - pc_; pc_ = now_; }
#define PROF_POLLS(n) npoll_ += (n);
#define PROF_DUMP(name, steps) if ((tid & 63) == 0 && (blockIdx.x % 23) == 0 && blockIdx.y == 0) \
  printf("%s wg(%d,%d,%d) wave %d: ns/step poll %lld mma %lld red+cell %lld publish %lld other %lld polls/step %.2f\n", name, blockIdx.x, blockIdx.y, blockIdx.z, tid >> 6, \
         pt_[0] * 10 / (steps), pt_[1] * 10 / (steps), pt_[2] * 10 / (steps), pt_[3] * 10 / (steps), pt_[4] * 10 / (steps), (double)npoll_ / (steps));
#else
#define PROF_DECL
#define PROF_MARK(i)
#define PROF_POLLS(n)
#define PROF_DUMP(name, steps)
#endif
constexpr int kBufFlags = 0x00020000;   // raw buffer descriptor word 3 for gfx9-family devices
// cache policy of the polling loads: bit 4 = coherent at agent scope (bypasses the XCD-local L2),
// bit 31 = volatile, so the compiler re-issues the load in every poll
constexpr int kSc1 = (int)(16u | 0x80000000u);

__device__ __forceinline__ unsigned ld_relaxed(const unsigned* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_relaxed(unsigned* p, unsigned v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Ring reads.  One wavefront owns chunks kc = wave + 4*it of its row tile.  Reads of freshly written
// remote data are latency-bound per compute unit and degrade when more than ~12 KiB per wavefront is in
// flight, so (a) a wave first polls ONE chunk (its last) until that shows the awaited tag, which is cheap
// while the producers are still busy, and only then (b) fetches its operands in batches of at most 12
// chunks, checking every tag; a batch with a stale tag is simply fetched again.
struct RingReader {
  __amdgpu_buffer_rsrc_t rs;
  int nkc, nchunk_valid, wave, lane;
  unsigned tag;
  unsigned* err;
  unsigned limit;

  __device__ __forceinline__ u32x4 load(int kc) const {
    return __builtin_amdgcn_raw_buffer_load_b128(rs, (kc * 64 + lane) * 16, 0, kSc1);
  }
  __device__ __forceinline__ bool chunk_fresh(const u32x4& x, int kc) const {
    return kc * 4 + (lane >> 4) >= nchunk_valid || ((x[1] >> 16) == tag && (x[3] >> 16) == tag);
  }
  // bounded wait on the wave's last chunk; returns the number of polls (diagnostics only)
  __device__ __forceinline__ unsigned wait_sample(bool& dead) const {
    if (dead || wave >= nkc) return 0;
    const int kc = wave + 4 * ((nkc - 1 - wave) / 4);          // last chunk of this wave
    for (unsigned poll = 0;; ++poll) {
      const u32x4 x = load(kc);
      if (__all(chunk_fresh(x, kc))) return poll + 1;
      if (poll >= limit || ((poll & 63u) == 63u && ld_relaxed(err) != 0u)) {
        st_relaxed(err, 1u);
        dead = true;
        return poll + 1;
      }
    }
  }
  template <int N>
  __device__ __forceinline__ void issue(u32x4 (&x)[N], int it0) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int kc = wave + 4 * (it0 + i);
      x[i] = (u32x4){0u, 0u, 0u, 0u};
      if (kc < nkc) x[i] = load(kc);
    }
  }
  // checks the tags of a fetched batch (fetching it again while any is stale) and strips them
  template <int N>
  __device__ __forceinline__ void settle(u32x4 (&x)[N], uint4 (&av)[N], int it0, bool& dead) const {
    for (unsigned poll = 0;; ++poll) {
      bool fresh = true;
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const int kc = wave + 4 * (it0 + i);
        if (kc < nkc) fresh = fresh && chunk_fresh(x[i], kc);
      }
      if (dead || __all(fresh)) break;
      if (poll >= limit || ((poll & 63u) == 63u && ld_relaxed(err) != 0u)) {
        st_relaxed(err, 1u);
        dead = true;
        break;
      }
      issue<N>(x, it0);
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int kc = wave + 4 * (it0 + i);
      const bool use = kc < nkc && kc * 4 + (lane >> 4) < nchunk_valid;
      av[i] = use ? make_uint4(x[i][0], x[i][1] & 0xffffu, x[i][2], x[i][3] & 0xffffu) : make_uint4(0, 0, 0, 0);
    }
  }
};

__device__ __forceinline__ RingReader make_reader(const uint4* base, int nkc, int nchunk_valid, int wave, int lane, unsigned tag,
                                                   unsigned* err, unsigned limit) {
  RingReader r;
  r.rs = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, nkc * 1024, kBufFlags);
  r.nkc = nkc; r.nchunk_valid = nchunk_valid; r.wave = wave; r.lane = lane; r.tag = tag; r.err = err; r.limit = limit;
  return r;
}

__device__ __forceinline__ void store_unit(uint4* ring, long unit_index, unsigned v0, unsigned v1, unsigned v2, unsigned tag) {
  const unsigned long long u = (unsigned long long)(v0 | (v1 << 16)) | ((unsigned long long)(v2 | (tag << 16)) << 32);
  __hip_atomic_store((unsigned long long*)ring + unit_index, u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ------------------------------------------------------------------------------------------------
// forward: z[16 rows, 4 gates x 16 units] = h[16 rows, K] W[K, 64]
template <int NIT>
__global__ __launch_bounds__(256) void persist_fwd_kernel(PFwdArgs a) {
  __shared__ float red[4][16][65];
  __shared__ unsigned short hb[16][18];
  const PFwdDir& d = a.d[blockIdx.z];
  const int tile = blockIdx.x, rt = blockIdx.y, ntiles = gridDim.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nkc = a.nkc, n = a.n, B = a.B, T = a.T;
  unsigned* err = a.sync;
  bool dead = false;

  uint4 w[NIT][4];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int kc = wave + 4 * it;
#pragma unroll
    for (int q = 0; q < 4; ++q)
      w[it][q] = kc < nkc ? d.Wf[((long)(tile * 4 + q) * nkc + kc) * 64 + lane] : make_uint4(0, 0, 0, 0);
  }

  const int r = tid >> 4, u = tid & 15;
  const int b = rt * 16 + r, j = tile * 16 + u;
  const bool active = b < B && j < n;
  float c = 0.f, h = 0.f;
  int L = 0;
  if (active) {
    c = d.cstate[(long)b * n + j];
    h = d.hstate[(long)b * n + j];
    L = clamp_len(a.lens, b, T);
  }
  // the unit this thread publishes (threads 0..95): row r2, unit m of this producer's 6
  const int r2 = tid / 6, m = tid - 6 * r2;
  const int cch = tile * 3 + (m >> 1);
  const long unit_index = (((long)rt * nkc + (cch >> 2)) * 64 + (cch & 3) * 16 + r2) * 2 + (m & 1);

  // x W_x + b of a frame does not depend on the recurrence: it is fetched one step ahead
  float zx[4] = {0.f, 0.f, 0.f, 0.f}, zx_next[4] = {0.f, 0.f, 0.f, 0.f};
  auto fetch_zx = [&](int tau, float (&z)[4]) {
    const int t = d.rev ? T - 1 - tau : tau;
    if (tau < T && active && t < L) {
      const float* gp = d.gates + ((long)t * B + b) * 4 * n + j;
      z[0] = gp[0]; z[1] = gp[n]; z[2] = gp[2 * n]; z[3] = gp[3 * n];
    }
  };
  fetch_zx(0, zx);
  PROF_DECL
  for (int tau = 0; tau < T; ++tau) {
    const int t = d.rev ? T - 1 - tau : tau;
    const bool valid = active && t < L;
    PROF_MARK(4)
    const uint4* rin = ((tau & 1) ? d.ring1 : d.ring0) + (long)rt * nkc * 64;
    uint4* rout = (tau & 1) ? d.ring0 : d.ring1;
    const RingReader rd = make_reader(rin, nkc, ntiles * 3, wave, lane, (unsigned)(tau + 1) & 0xffffu, err, a.spin_limit);
    const unsigned np_ = rd.wait_sample(dead);
    (void)np_;
    PROF_POLLS(np_)
    u32x4 raw[NIT];
    uint4 av[NIT];
    rd.issue<NIT>(raw, 0);
    fetch_zx(tau + 1, zx_next);
    rd.settle<NIT>(raw, av, 0, dead);
    PROF_MARK(0)

    f32x4 acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] = (f32x4){0.f, 0.f, 0.f, 0.f};
    // chunks beyond nkc hold zeros in both operands, so no guard is needed around the MFMAs
#pragma unroll
    for (int it = 0; it < NIT; ++it)
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[q] = Mma16<bf16_t>::run(av[it], w[it][q], acc[q]);
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int v = 0; v < 4; ++v) red[wave][4 * (lane >> 4) + v][q * 16 + (lane & 15)] = acc[q][v];
    PROF_MARK(1)
    __syncthreads();

    const float h_prev = h;
    CellOut o = {};
    if (valid) {
      float zh[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) zh[q] = red[0][r][q * 16 + u] + red[1][r][q * 16 + u] + red[2][r][q * 16 + u] + red[3][r][q * 16 + u];
      o = lstm_cell(zh, zx, c);
      c = o.c; h = o.h;
    }
    hb[r][u] = f2bf_bits(h);          // inactive threads hold h = 0: padding rows / units publish zeros
    __syncthreads();
    PROF_MARK(2)
    if (tid < 96) {                   // the recurrence's critical store goes out first
      const int v0 = 3 * m;
      const unsigned x0 = hb[r2][v0], x1 = v0 + 1 < 16 ? hb[r2][v0 + 1] : 0u, x2 = v0 + 2 < 16 ? hb[r2][v0 + 2] : 0u;
      store_unit(rout, unit_index, x0, x1, x2, (unsigned)(tau + 2) & 0xffffu);
    }
    if (active) {                     // layer outputs and what the backward pass needs
      Store<bf16_t>::store(d.y, ((long)t * B + b) * d.ldy + j, valid ? h : 0.f);
      if (d.cs) d.cs[((long)t * B + b) * n + j] = c;
      if (d.hprev) Store<bf16_t>::store(d.hprev, ((long)t * B + b) * n + j, h_prev);
      if (valid && a.write_gates) {
        float* gp = d.gates + ((long)t * B + b) * 4 * n + j;
        gp[0] = o.gi; gp[n] = o.gf; gp[2 * n] = o.gg; gp[3 * n] = o.go;
      }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) zx[q] = zx_next[q];
    PROF_MARK(3)
  }
  PROF_DUMP("fwd", T)
  if (active) {
    d.cstate[(long)b * n + j] = c;
    d.hstate[(long)b * n + j] = h;
  }
}

// ------------------------------------------------------------------------------------------------
// backward: Dh[16 rows, 16 units] = dz[16 rows, K] W^T[K, 16], then the gate gradients of this frame
struct BwdIn { float gi, gf, gg, go, c_new, c_prev, dy; };

template <int NIT>
__global__ __launch_bounds__(256) void persist_bwd_kernel(PBwdArgs a) {
  constexpr int NB = 4, BS = NIT / NB;           // operand batches per step
  static_assert(NIT % NB == 0, "operands are fetched in equal batches");
  __shared__ float red[4][16][17];
  __shared__ unsigned short zb[16][66];
  const PBwdDir& d = a.d[blockIdx.z];
  const int tile = blockIdx.x, rt = blockIdx.y, ntiles = gridDim.x;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nkc = a.nkc, n = a.n, B = a.B, T = a.T;
  unsigned* err = a.sync;
  bool dead = false;

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
  // everything the gate gradients need except Dh is independent of the recurrence: fetched one step ahead
  auto fetch_in = [&](int tau) {
    BwdIn in = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    const int t = d.rev ? T - 1 - tau : tau;
    if (tau >= 0 && active && t < L) {
      const float* gp = d.gates + ((long)t * B + b) * 4 * n + j;
      in.gi = gp[0]; in.gf = gp[n]; in.gg = gp[2 * n]; in.go = gp[3 * n];
      in.c_new = d.cs[((long)t * B + b) * n + j];
      const int tp = d.rev ? t + 1 : t - 1;               // frame processed just before t in the forward pass
      if (tp >= 0 && tp < T) in.c_prev = d.cs[((long)tp * B + b) * n + j];
      else if (d.c0) in.c_prev = d.c0[(long)b * n + j];
      in.dy = Store<bf16_t>::load(d.dy, ((long)t * B + b) * d.lddy + j);
    }
    return in;
  };
  BwdIn in = fetch_in(T - 1);

  PROF_DECL
  for (int tau = T - 1; tau >= -1; --tau) {
    PROF_MARK(4)
    const int sigma = T - 1 - tau;                       // count of backward steps done before this one
    const int t = d.rev ? T - 1 - tau : tau;             // frame of this step (out of range when tau == -1)
    const int t_next = d.rev ? t - 1 : t + 1;            // frame of the previous backward step
    const bool pointwise = tau >= 0;
    const bool valid = pointwise && active && t < L;
    BwdIn in_next = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

    if (sigma > 0) {
      const uint4* rin = (((sigma - 1) & 1) ? d.ring1 : d.ring0) + (long)rt * nkc * 64;
      const RingReader rd = make_reader(rin, nkc, ntiles * 11, wave, lane, (unsigned)sigma & 0xffffu, err, a.spin_limit);
      const unsigned np_ = rd.wait_sample(dead);
      (void)np_;
      PROF_POLLS(np_)
      f32x4 acc[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[q] = (f32x4){0.f, 0.f, 0.f, 0.f};
      u32x4 raw[2][BS];
      uint4 av[BS];
      rd.issue<BS>(raw[0], 0);
      in_next = fetch_in(tau - 1);
#pragma unroll
      for (int bt = 0; bt < NB; ++bt) {
        if (bt + 1 < NB) rd.issue<BS>(raw[(bt + 1) & 1], (bt + 1) * BS);
        rd.settle<BS>(raw[bt & 1], av, bt * BS, dead);
        PROF_MARK(0)
        // chunks beyond nkc hold zeros in both operands, so no guard is needed around the MFMAs
#pragma unroll
        for (int i = 0; i < BS; ++i) acc[(bt * BS + i) & 3] = Mma16<bf16_t>::run(av[i], w[bt * BS + i], acc[(bt * BS + i) & 3]);
        PROF_MARK(1)
      }
#pragma unroll
      for (int v = 0; v < 4; ++v) red[wave][4 * (lane >> 4) + v][lane & 15] = (acc[0][v] + acc[1][v]) + (acc[2][v] + acc[3][v]);
      __syncthreads();
      if (active && t_next < L) Dh = red[0][r][u] + red[1][r][u] + red[2][r][u] + red[3][r][u];
    } else {
      in_next = fetch_in(tau - 1);
    }
    if (pointwise) {
      float dz[4] = {0.f, 0.f, 0.f, 0.f};
      if (valid) lstm_cell_grad(in.gi, in.gf, in.gg, in.go, in.c_new, in.c_prev, in.dy + Dh, Dc, dz);
      unsigned short bits[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        bits[q] = f2bf_bits(dz[q]);
        zb[r][q * 16 + u] = bits[q];                       // inactive threads publish zeros
      }
      __syncthreads();
      PROF_MARK(2)
      uint4* rout = (sigma & 1) ? d.ring1 : d.ring0;
      const unsigned tag_out = (unsigned)(sigma + 1) & 0xffffu;
#pragma unroll
      for (int round = 0; round < 2; ++round) {
        const int id = tid + 256 * round;
        if (id < 16 * 22) {
          const int r2 = id / 22, m = id - 22 * r2, v0 = 3 * m;
          const unsigned x0 = zb[r2][v0], x1 = v0 + 1 < 64 ? zb[r2][v0 + 1] : 0u, x2 = v0 + 2 < 64 ? zb[r2][v0 + 2] : 0u;
          const int cch = tile * 11 + (m >> 1);
          const long unit_index = (((long)rt * nkc + (cch >> 2)) * 64 + (cch & 3) * 16 + r2) * 2 + (m & 1);
          store_unit(rout, unit_index, x0, x1, x2, tag_out);
        }
      }
      if (active) {
#pragma unroll
        for (int q = 0; q < 4; ++q) ((unsigned short*)d.DZ)[((long)t * B + b) * 4 * n + q * n + j] = bits[q];
      }
      __syncthreads();                                      // zb and red are reused by the next step
      PROF_MARK(3)
    }
    in = in_next;
  }
  PROF_DUMP("bwd", T)
  if (active) {
    d.Dh[(long)b * n + j] = Dh;
    d.Dc[(long)b * n + j] = Dc;
  }
}

// ------------------------------------------------------------------------------------------------
// packing for the ring layout
// forward weights: chunk index = (((dir*ntile + tile)*4 + q)*nkc + kc)*64 + lane
__global__ void pack_wh_fwd_ll_kernel(const bf16_t* W, uint4* out, int n, int nkc, long total) {
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int lane = idx & 63;
  long rest = idx >> 6;
  const int kc = rest % nkc; rest /= nkc;
  const int q = rest & 3; rest >>= 2;
  const int ntile = (n + 15) / 16;
  const int tile = rest % ntile, dir = rest / ntile;
  const int j = tile * 16 + (lane & 15), g = lane >> 4;
  const bf16_t* Wd = W + (long)dir * n * 4 * n;
  bf16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int s = (kc * 4 + g) * 8 + e;
    const int p = s / kLLSlotsFwd, val = ll_slot_value(s - p * kLLSlotsFwd, kLLValsFwd);
    const int k = p * 16 + val;
    v[e] = (val >= 0 && k < n && j < n) ? Wd[(long)k * 4 * n + q * n + j] : (bf16_t)0.f;
  }
  out[idx] = *(uint4*)v;
}
// backward weights: chunk index = ((dir*ntile + tile)*nkc + kc)*64 + lane ; K runs over the producers' dz values
__global__ void pack_wh_bwd_ll_kernel(const bf16_t* W, uint4* out, int n, int nkc, long total) {
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int lane = idx & 63;
  long rest = idx >> 6;
  const int kc = rest % nkc; rest /= nkc;
  const int ntile = (n + 15) / 16;
  const int tile = rest % ntile, dir = rest / ntile;
  const int unit = tile * 16 + (lane & 15), g = lane >> 4;
  const bf16_t* Wd = W + (long)dir * n * 4 * n;
  bf16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int s = (kc * 4 + g) * 8 + e;
    const int p = s / kLLSlotsBwd, val = ll_slot_value(s - p * kLLSlotsBwd, kLLValsBwd);
    const int ju = p * 16 + (val & 15), q = val >> 4;
    v[e] = (val >= 0 && ju < n && unit < n) ? Wd[(long)unit * 4 * n + q * n + ju] : (bf16_t)0.f;
  }
  out[idx] = *(uint4*)v;
}
// initial state: unit index = ((((dir*nrt + rt)*nkc + kc)*64 + lane)*2 + half) ; ring0 gets h with tag 1, ring1 zeros
__global__ void pack_state_ll_kernel(const float* h, uint4* ring0, uint4* ring1, int B, int n, int nkc, int nrt, long total) {
  long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int half = idx & 1, lane = (idx >> 1) & 63;
  long rest = idx >> 7;
  const int kc = rest % nkc; rest /= nkc;
  const int rt = rest % nrt, dir = rest / nrt;
  const int row = rt * 16 + (lane & 15), g = lane >> 4;
  const int U = (kc * 4 + g) * 2 + half;       // unit-of-three index along K
  const int p = U / 6, m = U - 6 * p;
  unsigned x[3];
#pragma unroll
  for (int e = 0; e < 3; ++e) {
    const int val = 3 * m + e, k = p * 16 + val;
    x[e] = (val < 16 && k < n && row < B) ? (unsigned)f2bf_bits(h[((long)dir * B + row) * n + k]) : 0u;
  }
  ((unsigned long long*)ring0)[idx] = (unsigned long long)(x[0] | (x[1] << 16)) | ((unsigned long long)(x[2] | (1u << 16)) << 32);
  ((unsigned long long*)ring1)[idx] = 0ull;
}

// Cooperative launch; refuses (without launching) a grid that cannot be resident all at once.
template <typename K, typename A>
hipError_t coop(K kernel, dim3 grid, const A& a, hipStream_t s) {
  static int capacity = -1;             // work-groups of this kernel the current device can hold at once
  if (capacity < 0) {
    int dev = 0, per_cu = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 256, 0) != hipSuccess)
      return hipErrorUnknown;
    capacity = per_cu * prop.multiProcessorCount;
  }
  if ((long)grid.x * grid.y * grid.z > capacity) return hipErrorCooperativeLaunchTooLarge;
  A copy = a;
  void* args[] = {&copy};
  return hipLaunchCooperativeKernel((const void*)kernel, grid, dim3(256), args, 0, s);
}

}  // namespace

hipError_t launch_persist_fwd(const PFwdArgs& a, hipStream_t s) {
  if (a.nkc > kLLMaxNkcFwd) return hipErrorCooperativeLaunchTooLarge;
  return coop(persist_fwd_kernel<kLLMaxNkcFwd / 4>, dim3(cdiv(a.n, 16), cdiv(a.B, 16), a.ndir), a, s);
}
hipError_t launch_persist_bwd(const PBwdArgs& a, hipStream_t s) {
  if (a.nkc > kLLMaxNkcBwd) return hipErrorCooperativeLaunchTooLarge;
  return coop(persist_bwd_kernel<kLLMaxNkcBwd / 4>, dim3(cdiv(a.n, 16), cdiv(a.B, 16), a.ndir), a, s);
}
hipError_t launch_pack_wh_fwd_ll(const void* W, uint4* Wf, int n, int nkc, int ndir, hipStream_t s) {
  long total = (long)ndir * cdiv(n, 16) * 4 * nkc * 64;
  hipLaunchKernelGGL(pack_wh_fwd_ll_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, (const bf16_t*)W, Wf, n, nkc, total);
  return hipGetLastError();
}
hipError_t launch_pack_wh_bwd_ll(const void* W, uint4* Wb, int n, int nkc, int ndir, hipStream_t s) {
  long total = (long)ndir * cdiv(n, 16) * nkc * 64;
  hipLaunchKernelGGL(pack_wh_bwd_ll_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, (const bf16_t*)W, Wb, n, nkc, total);
  return hipGetLastError();
}
hipError_t launch_pack_state_ll(const float* h, uint4* ring0, uint4* ring1, int B, int n, int nkc, int nrt, int ndir,
                                hipStream_t s) {
  long total = (long)ndir * nrt * nkc * 64 * 2;
  hipLaunchKernelGGL(pack_state_ll_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, h, ring0, ring1, B, n, nkc, nrt, total);
  return hipGetLastError();
}

}  // namespace lstm
