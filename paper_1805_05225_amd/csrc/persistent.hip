// Single-launch recurrent kernels: the whole time loop of a layer in ONE launch (bfloat16 storage).
//
// The per-step kernels pay a launch per time step and re-read their W_h slice from the memory
// system every step.  Here each work-group (32 hidden units x 8 batch rows, or x 16 rows for batches
// that the 8-row form cannot hold in one launch) loads its slice of the packed W_h into registers once and
// then walks all T steps.
//
// Only h_t (forward) or partial sums of Dh (backward) cross work-groups.  Measurements on this device
// showed that a counter barrier is the wrong tool: atomics on one address serialise at ~16 ns each
// (4 us for 256 work-groups) and agent-scope fences cost microseconds more.  So there is no
// barrier and no fence here.  The exchanged data lives in a two-slot ring whose every 8-byte unit
// holds its values AND a tag of the step that wrote it (four bf16 values, the tag one bit that their
// range leaves free), written with one 64-bit store and read with cache-bypassing 16-byte loads.  A consumer simply re-reads an operand until
// its tags show the step it is waiting for: value and "ready" flag arrive in the same atomic
// unit, so no ordering between different addresses is ever needed.
//
// Two ring slots suffice: a work-group writes slot s for step t+1 only after it has seen every
// tag of step t, i.e. after every work-group has finished step t and therefore finished reading
// slot s (which held step t-1).
//
// Every wait is bounded: after `spin_limit` polls the wave raises the error word sync[0], stops
// waiting for the rest of the launch and runs to the end (results are then invalid and the word
// says so); every other wave notices the word in its own wait loop and does the same, so the
// grid always drains.  The grid is checked against what the device holds at once; the launch is
// cooperative unless the caller vouches that nothing else occupies the device.
#include "recurrent_dev.h"
#include <type_traits>
#include <algorithm>
#include <map>
#include <mutex>

namespace lstm {
namespace {

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// Optional in-kernel phase clocks (build with -DLSTM_PROF; prints from a few work-groups at the end).
#ifdef LSTM_PROF
#define PROF_DECL long long pt_[8] = {0, 0, 0, 0, 0, 0, 0, 0}; long long pc_ = wall_clock64(); unsigned npoll_ = 0, nredo_ = 0;
#define PROF_MARK(i) { long long now_ = wall_clock64(); pt_[i] += now_ - pc_; pc_ = now_; }
#define PROF_POLLS(n) npoll_ += (n);
#define PROF_REDO(n) nredo_ += (n);
#define PROF_DUMP(name, steps) if ((tid & 63) == 0 && (blockIdx.x % 23) == 0 && blockIdx.y == 0) \
  printf("%s wg(%d,%d,%d) wave %d: ns/step sample %lld stream %lld mma %lld red+cell %lld publish %lld other %lld polls/step %.2f loads fetched again per 1000 steps %.1f\n", name, blockIdx.x, blockIdx.y, blockIdx.z, (int)(threadIdx.x >> 6), \
         pt_[5] * 10 / (steps), pt_[0] * 10 / (steps), pt_[1] * 10 / (steps), pt_[2] * 10 / (steps), pt_[3] * 10 / (steps), pt_[4] * 10 / (steps), (double)npoll_ / (steps), 1000.0 * nredo_ / (steps));
#else
#define PROF_DECL
#define PROF_MARK(i)
#define PROF_POLLS(n)
#define PROF_REDO(n)
#define PROF_DUMP(name, steps)
#endif
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
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
// flight, so (a) a wave first polls the first two of its loads until they show the awaited tag, which is cheap
// while the producers are still busy, and only then (b) fetches the rest, checking every tag; a load whose tags
// are stale is fetched again on its own (fix_up_batch, or an immediate re-issue through LDS), never the whole set.
//
// Nothing in the stream is predicated.  The buffer descriptor covers exactly the nkc chunks of the row tile,
// so a load past the end (chunks the template bound adds beyond nkc, lanes whose rows this work-group does
// not own: their offset is parked far outside) returns zeros from the bounds check without touching memory.
// Padding units inside the ring hold zero values (nobody writes them after the initial fill), so masking off
// the tags is all the clean-up an operand needs.  Keeping branches and lane masks out of this loop
// matters: with them the instruction stream between two loads, not the memory system, set the step time.
// Order in which a work-group walks the nitv loads of its row tile: rotated by `rot`, so that the work-groups of
// one XCD, which all read the same tile at the same time, do not all ask the same L2 channel for the same lines.
__device__ __forceinline__ int rot_index(int i, int rot, int nitv) {
  const int j = i + rot;
  return i >= nitv ? i : (j >= nitv ? j - nitv : j);
}
struct RingReader {
  __amdgpu_buffer_rsrc_t rs;
  int rot, nitv;                         // load i of the stream fetches iteration (i + rot) mod nitv of the row tile
  unsigned voff;                         // byte offset of this lane's first load (parked out of range if the lane is off)
  unsigned it_bytes;                     // byte distance between consecutive loads of a lane
  int lim, lim_step;                     // load `it` carries awaited tags for this lane iff lim_step*it < lim
  unsigned tag;                          // the awaited tag as it sits in the upper half of a unit's second dword
  unsigned* err;
  unsigned limit;

  __device__ __forceinline__ int it_of(int i) const { return rot_index(i, rot, nitv); }
  __device__ __forceinline__ u32x4 load_it(int it) const {
    return __builtin_amdgcn_raw_buffer_load_b128(rs, voff + (unsigned)it * it_bytes, 0, kSc1);
  }
  __device__ __forceinline__ bool expects(int it) const { return lim_step * it < lim; }   // does this lane's unit of load `it` carry a tag?
  // Tag differences of one load, per lane: a bit above the low half iff one of the lane's two tags is not `tagw >> 16`.
  // Lanes whose units carry no tag (padding inside the ring, chunks past the end) report nothing, whatever they read.
  __device__ __forceinline__ unsigned tag_diff(const u32x4& x, int it, unsigned tagw) const {
    const unsigned t = (x[1] ^ tagw) | (x[3] ^ tagw);
    return expects(it) ? t & kLLFwdTagBit : 0u;
  }
  __device__ __forceinline__ unsigned stale_bits(const u32x4& x, int it) const {
    const unsigned d = ((x[1] >> 16) ^ tag) | ((x[3] >> 16) ^ tag);
    return lim_step * it < lim ? d & (kLLFwdTagBit >> 16) : 0u;
  }
  // Second pass over the loads marked in `redo`, all of them in flight at once: every round fetches those still
  // marked, hands the ones whose tags have all turned to `use` (operand as loaded, tags included) and keeps the
  // rest for the next round (bounded).
  template <int NIT, int OFF = 0, typename F>
  __device__ __forceinline__ void fix_up_batch(unsigned long long redo, bool& dead, F&& use) const {
    redo &= ((1ull << NIT) - 1ull) << OFF;                    // loads OFF .. OFF + NIT - 1 of the stream
    for (unsigned poll = 0; redo != 0ull && !dead; ++poll) {
      u32x4 x[NIT];
#pragma unroll
      for (int i = 0; i < NIT; ++i)
        if ((redo >> (i + OFF)) & 1ull) x[i] = load_it(it_of(i + OFF));
#pragma unroll
      for (int i = 0; i < NIT; ++i) {
        if (!((redo >> (i + OFF)) & 1ull)) continue;
        if (__builtin_amdgcn_ballot_w64(stale_bits(x[i], it_of(i + OFF)) != 0u) == 0ull) {
          use(i + OFF, x[i]);
          redo &= ~(1ull << (i + OFF));
        }
      }
      if (redo != 0ull && (poll >= limit || ((poll & 63u) == 63u && ld_relaxed(err) != 0u))) {
        st_relaxed(err, 1u);
        dead = true;
      }
    }
  }
};

// `nchunk_valid` counts the 16-lane groups (quarter chunks) that producers write; `lane_on` is false for lanes
// whose fragment rows belong to another work-group.
__device__ __forceinline__ RingReader make_reader(const uint4* base, int nkc, int nchunk_valid, int wave, int lane, unsigned tag,
                                                   unsigned* err, unsigned limit, int rot, bool lane_on = true) {
  RingReader r;
  r.nitv = (nkc + 3) / 4; r.rot = rot;
  r.rs = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, nkc * 1024, kBufFlags);
  r.voff = lane_on ? (unsigned)(wave * 1024 + lane * 16) : 0x7ff00000u;
  r.it_bytes = 4096u;
  r.lim = lane_on ? nchunk_valid - (lane >> 4) - 4 * wave : -0x40000000;
  r.lim_step = 16;
  r.tag = tag; r.err = err; r.limit = limit;
  return r;
}

// Reader for a work-group that owns only 8 of a row tile's 16 rows (`half` selects which).  A load would
// leave half the lanes idle, and the time of a ring read goes with the number of loads, not their bytes; so one
// load serves TWO chunks: lanes whose fragment row is below 8 fetch our rows of chunk wave + 8*it, the others
// our rows of chunk wave + 8*it + 4.  The registers as loaded are the A operand of the first chunk with our rows
// in fragment rows 0-7 (rows 8-15 hold the other chunk's data: rows of a matrix product are independent, and
// those output rows are never read); rotating each group of 16 lanes by 8 gives the operand of the second.
__device__ __forceinline__ RingReader make_reader_half(const uint4* base, int nkc, int nchunk_valid, int wave, int lane, int half,
                                                        unsigned tag, unsigned* err, unsigned limit, int rot) {
  RingReader r;
  r.nitv = (nkc + 7) / 8; r.rot = rot;
  const int row = lane & 15, g = lane >> 4, second = row >> 3;
  r.rs = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, nkc * 1024, kBufFlags);
  r.voff = (unsigned)((wave + 4 * second) * 1024 + (g * 16 + half * 8 + (row & 7)) * 16);
  r.it_bytes = 8192u;
  r.lim = nchunk_valid - g - 4 * wave - 16 * second;
  r.lim_step = 32;
  r.tag = tag; r.err = err; r.limit = limit;
  return r;
}
__device__ __forceinline__ uint4 rotate_rows_by_8(uint4 v) {
  constexpr int kRowRor8 = 0x128;        // DPP control: rotate right by 8 inside each row of 16 lanes
  uint4 o;
  o.x = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v.x, kRowRor8, 0xf, 0xf, false);
  o.y = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v.y, kRowRor8, 0xf, 0xf, false);
  o.z = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v.z, kRowRor8, 0xf, 0xf, false);
  o.w = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v.w, kRowRor8, 0xf, 0xf, false);
  return o;
}

// two floats -> two bf16 (round to nearest even) in one register, low half first
__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_;
  const bf16x2_ r = __builtin_convertvector((f32x2_){lo, hi}, bf16x2_);
  return __builtin_bit_cast(unsigned, r);
}
// Streaming accesses of the recurrent kernels (every byte touched once): marked non-temporal so that they do not
// push the exchange ring, which is re-read every step, out of the L2.
__device__ __forceinline__ float ld_stream(const float* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ unsigned short ld_stream(const unsigned short* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void st_stream(float* p, float v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ void st_stream(unsigned short* p, unsigned short v) { __builtin_nontemporal_store(v, p); }

// --- W_h in accumulation registers ---------------------------------------------------------------------------
// The register file of a wavefront is 256 architectural + 256 accumulation registers.  A W_h slice larger than
// what is left of the first 256 is parked by the compiler in accumulation registers and copied back, four moves
// per MFMA, before every use - with one wavefront per SIMD those moves are on the critical path.  MFMA can read
// its B operand from accumulation registers directly, so the slice is loaded straight into them and the products
// are issued through inline assembly.  The compiler does not see an MFMA in that text, so the wait states the
// hardware needs between the last MFMA and the first read of its result are inserted by hand (mfma_settle).
__device__ __forceinline__ u32x4 load_to_agpr(const uint4* p) {
  u32x4 r;
  asm volatile("global_load_dwordx4 %0, %1, off" : "=a"(r) : "v"(p) : "memory");
  return r;
}
__device__ __forceinline__ void agpr_loads_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// acc += A (16 rows x 32 k, vector registers) x B (32 k x 16 columns, accumulation registers)
__device__ __forceinline__ void mfma_b_agpr(f32x4& acc, const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_b_vgpr(f32x4& acc, const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "v"(b));
}
// acc = A x B: the first product of a chain takes the constant 0 as its addend, so the accumulators need no clearing
// (64 moves per step in the backward kernel, and the wait states between them and the first MFMA).  The result may not share
// registers with an operand: early clobber.
__device__ __forceinline__ void mfma_b_agpr_first(f32x4& acc, const u32x4& a, const u32x4& b) {
  asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "a"(b));
}
// The float MFMA (16x16x4): A one float per lane in a vector register, B one float per lane in an accumulation register.
__device__ __forceinline__ void mfma4_b_agpr(f32x4& acc, float a, unsigned b) {
  asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+v"(acc) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma4_b_agpr_first(f32x4& acc, float a, unsigned b) {
  asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, 0" : "=&v"(acc) : "v"(a), "a"(b));
}
__device__ __forceinline__ void mfma_settle(f32x4& a0) { asm volatile("s_nop 15\n\ts_nop 3" : "+v"(a0)); }
// Wait states between the last ordinary (vector ALU, DPP, LDS) write of registers and an MFMA reading them.  For
// MFMAs it emits itself the compiler knows what the hardware needs; for these it cannot, and an MFMA issued right
// behind DPP moves was observed to read the old register contents.
// first MFMA of a pair behind which a preparation step of the next pair is placed (the next pair's loads were
// issued together with this pair's and have had that much more time to arrive)
#ifndef LSTM_PREP_DELAY
#define LSTM_PREP_DELAY 6
#endif
constexpr int kPrepDelay = LSTM_PREP_DELAY;
#ifndef LSTM_OPERAND_NOPS
#define LSTM_OPERAND_NOPS "7"
#endif
// s_waitcnt vmcnt(n) for an n that is constant after unrolling (0 .. 15; the instruction takes an immediate).
// Where a kernel consumes a ring load while younger stores are in flight it waits with this, n = the number of
// YOUNGER LOADS: loads return in the order of issue among themselves, but stores were seen to be acknowledged ahead of
// older loads that bypass L2, so a count that includes the younger stores - what the compiler emits - can be reached
// while the load is still on its way.
// The wait names the registers it is for: an assembly statement that "rewrites" them, so that no instruction reading them can
// be scheduled in front of it (in straight-line code the compiler would otherwise be free to, with only its own wait before them).
#define LSTM_WAIT_CASE(N) case N: asm volatile("s_waitcnt vmcnt(" #N ")" : "+v"(x)); break;
__device__ __forceinline__ void wait_loads_but(int n, u32x4& x) {
  switch (n < 15 ? n : 15) {
    LSTM_WAIT_CASE(0) LSTM_WAIT_CASE(1) LSTM_WAIT_CASE(2) LSTM_WAIT_CASE(3) LSTM_WAIT_CASE(4) LSTM_WAIT_CASE(5) LSTM_WAIT_CASE(6) LSTM_WAIT_CASE(7)
    LSTM_WAIT_CASE(8) LSTM_WAIT_CASE(9) LSTM_WAIT_CASE(10) LSTM_WAIT_CASE(11) LSTM_WAIT_CASE(12) LSTM_WAIT_CASE(13) LSTM_WAIT_CASE(14)
    default: asm volatile("s_waitcnt vmcnt(15)" : "+v"(x)); break;
  }
}
#undef LSTM_WAIT_CASE
// f(integral_constant<0>) ... f(integral_constant<N - 1>): a loop whose counter is a constant expression in the body
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (N > 0) {
    static_for<N - 1>(f);
    f(std::integral_constant<int, N - 1>{});
  }
}
__device__ __forceinline__ void operands_settle(u32x4& a, u32x4& b) { asm volatile("s_nop " LSTM_OPERAND_NOPS : "+v"(a), "+v"(b)); }
__device__ __forceinline__ void operands_settle(u32x4& a, u32x4& b, u32x4& c, u32x4& d) {
  asm volatile("s_nop " LSTM_OPERAND_NOPS : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}
__device__ __forceinline__ void operands_settle(f32x4& a, f32x4& b, f32x4& c, f32x4& d) {
  asm volatile("s_nop " LSTM_OPERAND_NOPS : "+v"(a), "+v"(b), "+v"(c), "+v"(d));
}
// 20 wait states: more than any MFMA of this shape needs before its result may be read or overwritten
__device__ __forceinline__ void mfma_settle(f32x4& a0, f32x4& a1, f32x4& a2, f32x4& a3) {
  asm volatile("s_nop 15\n\ts_nop 3" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3));
}
__device__ __forceinline__ void mfma_settle(f32x4& a0, f32x4& a1, f32x4& a2, f32x4& a3, f32x4& a4, f32x4& a5, f32x4& a6, f32x4& a7) {
  asm volatile("s_nop 15\n\ts_nop 3" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7));
}

// Is every work-group of this one's exchange group on the same XCD?  Then their ring stores need not be written
// through to memory: the XCD's L2 is the point where those work-groups meet (measured: one-way latency 212 ns
// instead of 350, and the ring's store traffic stays out of the fabric).  Each work-group publishes the XCD it runs on
// (hardware register XCC_ID) in `tab` (zero-filled by the host, one word per work-group, a group's words consecutive
// from `group_base`) and reads the group's words; anything but "all equal to mine" - a word still unset after the
// poll limit included - means "not local", and the caller then uses agent-scope stores as before.  The verdict
// needs no agreement: a work-group that says "local" has seen every member on its own XCD.
__device__ __forceinline__ bool group_is_xcd_local(unsigned* tab, int group_base, int members, int me, unsigned limit) {
  __shared__ int verdict;
  if (threadIdx.x == 0) {
    const unsigned mine = (__builtin_amdgcn_s_getreg(((4 - 1) << 11) | 20) & 15u) + 1u;     // XCC_ID, bits 3:0
    st_relaxed(&tab[group_base + me], mine);
    bool same = true;
    for (int p = 0; p < members && same; ++p) {
      unsigned v = 0u;
      for (unsigned poll = 0; poll < limit; ++poll) {
        v = ld_relaxed(&tab[group_base + p]);
        if (v != 0u) break;
      }
      same = v == mine;
    }
    verdict = same ? 1 : 0;
  }
  __syncthreads();
  return verdict != 0;
}

// Work-group -> (unit tile, row tile, direction).  Work-groups are dealt to the 8 XCDs round-robin in launch
// order, and every work-group of one (direction, row tile) group reads the same ring tile each step.  When the
// shape allows it the groups are laid out so that each XCD serves a single group: its L2 then fetches one
// ring tile per step instead of all of them.  Any bijection is correct; this one is only faster.
struct WgCoord { int tile, rt, dir; };
__device__ __forceinline__ WgCoord wg_coord() {
  const int ntiles = gridDim.x, nrt = gridDim.y, ndir = gridDim.z;
  const int groups = nrt * ndir, total = ntiles * groups;
  const int lin = blockIdx.x + ntiles * (blockIdx.y + nrt * blockIdx.z);
  WgCoord c = {(int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z};
  if (groups <= 8 && 8 % groups == 0 && total % 8 == 0) {
    const int xcd = lin & 7, slot = lin >> 3, per_group = 8 / groups;     // XCDs per group
    const int group = xcd % groups;
    c.tile = xcd / groups + per_group * slot;
    c.rt = group % nrt;
    c.dir = group / nrt;
  }
  return c;
}

// ------------------------------------------------------------------------------------------------
// forward: z[8 rows, 4 gates x 32 units] = h[8 rows, K] W[K, 128].  A work-group owns 32 units for 8 batch rows
// (half a row tile); one load serves two chunks (see make_reader_half).  The W_h slice fills the 256 accumulation
// registers of every lane (n = 1024: 8 register sets of 8 fragments).
template <int NIT>
__global__ __launch_bounds__(256) void persist_fwd8_kernel(PFwdArgs a) {
  __shared__ float red[2][4][8][129];                    // two copies, used by even and odd steps: one barrier per step
  const WgCoord wg = wg_coord();
  const PFwdDir d = a.d[wg.dir];       // a copy: fields read through a reference are fetched again in every time step
  const int tile2 = wg.tile, rt = a.rt0 + (wg.rt >> 1), half = wg.rt & 1;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int nkc = a.nkc, n = a.n, B = a.B, T = a.T;
  const int ntiles16 = (n + 15) / 16;
  unsigned* err = a.sync;
  bool dead = false;

  const int nitv = (nkc + 7) / 8, rot = tile2 % nitv;
  // Register sets 2p, 2p+1 hold the two chunks that load p of the stream fetches.  The first kAccIts sets fill the
  // 256 accumulation registers, the rest sit in vector registers.  Sets of chunks past the end (or of a unit tile
  // past the end) are loaded from a chunk of zeros that the host keeps behind the packed weights.
  constexpr int kAccIts = NIT < 8 ? NIT : 8;
  u32x4 wa[kAccIts][2][4];
  u32x4 wv[NIT - kAccIts > 0 ? NIT - kAccIts : 1][2][4];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int kc = wave + 4 * (2 * rot_index(it >> 1, rot, nitv) + (it & 1));
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
      const int t16 = tile2 * 2 + ct;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint4* src = (kc < nkc && t16 < ntiles16) ? &d.Wf[((long)(t16 * 4 + q) * nkc + kc) * 64 + lane] : &d.Wzero[lane];
        if (it < kAccIts) wa[it][ct][q] = load_to_agpr(src);
        else wv[it - kAccIts][ct][q] = *(const u32x4*)src;
      }
    }
  }
  agpr_loads_done();

  const int r8 = tid >> 5, u = tid & 31;                 // pointwise pair of this thread: row r8 of the half, unit u of 32
  const int b = rt * 16 + half * 8 + r8, j = tile2 * 32 + u;
  const bool active = b < B && j < n;
  float c = 0.f, h = 0.f;
  int L = 0;
  if (active) {
    c = d.cstate[(long)b * n + j];
    h = d.hstate[(long)b * n + j];
    L = clamp_len(a.lens, b, T);
  }
  // The unit this thread publishes.  A unit is four consecutive units' h of one row (the tag is a bit of the fourth), and a
  // row's 32 units sit in 32 consecutive lanes, so the thread of every fourth unit takes its neighbours' values
  // through DPP shifts: no staging in shared memory, no second barrier.  m = which unit of the 16-unit tile (0..3).
  const int pp = u >> 4, m = (u & 15) >> 2;
  const int t16p = tile2 * 2 + pp;
  const int cch = t16p * 2 + (m >> 1);
  const long unit_index = (((long)rt * nkc + (cch >> 2)) * 64 + (cch & 3) * 16 + half * 8 + r8) * 2 + (m & 1);
  const bool publishes = (u & 3) == 0 && t16p < ntiles16;
  const bool local = a.xcc != nullptr &&
                     group_is_xcd_local(a.xcc, (wg.dir * (int)gridDim.y + wg.rt) * (int)gridDim.x, gridDim.x, tile2, a.spin_limit);
  // Has this row had a frame yet?  Until then it publishes zeros, not the initial state it carries: that state's product
  // with W_h has been added to the pre-activations of the row's first frame by the host side, and what travels
  // through the ring must keep |h| <= 1 (the tag bit).
  bool started = false;

  // x W_x + b of a frame is read through a buffer descriptor that covers exactly that frame: a lane with nothing to
  // fetch (row past the batch, unit past n, frame past the row's length) has its offset parked outside and gets zeros
  // without touching memory, as does every lane once the frames are used up (zero-sized descriptor).  Nothing is
  // predicated, so every step issues the same four loads: with loads that may or may not have been issued the
  // compiler has to assume the fewest when it places the waits.
  // The outputs go the same way: one descriptor per array and frame (zero-sized if the array is absent), offsets
  // that never change, parked where a lane has nothing to store; and so does the ring store, whose descriptor ends
  // below the parking offset.  Frame sizes in bytes: gates [B,4n] float, y [B,ldy] bf16, cs [B,n] float, hprev [B,n] bf16.
  constexpr unsigned kParked = 0x7ff00000u;
  const unsigned g_bytes = (unsigned)B * 4u * n * 4u, y_bytes = (unsigned)B * d.ldy * 2u, s_bytes = (unsigned)B * n * 4u;
  const unsigned g_off = active ? ((unsigned)b * 4u * n + j) * 4u : kParked;
  const unsigned y_off = active ? ((unsigned)b * d.ldy + j) * 2u : kParked;
  const unsigned s_off = active ? ((unsigned)b * n + j) * 4u : kParked;        // (half of it in the bf16 array; still parked)
  const unsigned pub_off = publishes ? (unsigned)unit_index * 8u : kParked;
  auto frame_of = [&](const void* base, int t, unsigned bytes, bool present = true) {
    return __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)base + (unsigned long long)(unsigned)t * bytes), 0, present && base != nullptr ? bytes : 0u, kBufFlags);
  };
  auto fetch_zx = [&](int tau, float (&z)[4]) {
    const bool ok = tau < T;
    const int t = d.rev ? T - 1 - tau : tau;
    const __amdgpu_buffer_rsrc_t rg =
        __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)d.gates + (unsigned long long)(unsigned)(ok ? t : 0) * g_bytes), 0, ok ? g_bytes : 0u, kBufFlags);
    const unsigned go = t < L ? g_off : kParked;           // (L is 0 in lanes without a row)
#pragma unroll
    for (int q = 0; q < 4; ++q) z[q] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(rg, go, (unsigned)q * 4u * n, 2));   // 2: non-temporal
  };
  float zx_a[4], zx_b[4];
  unsigned h_prev_bits = pack_bf16x2(h, 0.f) & 0xffffu;     // what hprev receives: h before the step, as bf16
  fetch_zx(0, zx_a);
  PROF_DECL
  // One time step.  `zx` holds this step's x W_x + b and `zx_next` receives the next step's; the loop below calls it
  // with the two in alternating roles, because a copy at the end of a step would have to wait for the loads (and,
  // counted with them, the step's stores) at that point.
  auto step = [&](const int tau, const float (&zx)[4], float (&zx_next)[4], auto parity) __attribute__((always_inline)) {
    float (&red_)[4][8][129] = red[decltype(parity)::value];
    const int t = d.rev ? T - 1 - tau : tau;
    const bool valid = active && t < L;
    PROF_MARK(4)
    const uint4* rin = ((tau & 1) ? d.ring1 : d.ring0) + (long)rt * nkc * 64;
    uint4* rout = (tau & 1) ? d.ring0 : d.ring1;
    RingReader rd = make_reader_half(rin, nkc, ntiles16 * 2, wave, lane, half, ll_fwd_tag((unsigned)tau) << 14, err, a.spin_limit, rot);
    f32x4 acc[2][4];
    {
      // One MFMA of register set `it` into accumulator (ct, q).
      auto mma_one = [&](int it, int ct, int q, const u32x4& a_op) __attribute__((always_inline)) {
        if (it < kAccIts) mfma_b_agpr(acc[ct][q], a_op, wa[it < kAccIts ? it : 0][ct][q]);
        else mfma_b_vgpr(acc[ct][q], a_op, wv[it >= kAccIts ? it - kAccIts : 0][ct][q]);
      };
      auto use_single = [&](int p, const u32x4& raw) {     // a load fetched again after the stream, tags still in it
        const uint4 av_ = make_uint4(raw[0], raw[1] & ~kLLFwdTagBit, raw[2], raw[3] & ~kLLFwdTagBit);
        const uint4 av2_ = rotate_rows_by_8(av_);
        u32x4 av = {av_.x, av_.y, av_.z, av_.w}, av2 = {av2_.x, av2_.y, av2_.z, av2_.w};
        operands_settle(av, av2);
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            mma_one(2 * p, ct, q, av);
            mma_one(2 * p + 1, ct, q, av2);
          }
      };
      // The stream.  The loads are consumed in pairs: a pair is four chunks, and every accumulator takes its four
      // products in a row.  An MFMA of this shape issues every 16 cycles (7.05 ns measured, in any order of the
      // accumulators) and occupies the issue slot of the wavefront for 4 of them: one independent instruction behind
      // it is free (7.4 ns per MFMA measured), three dependent ones are not (12.4 ns).  What turns the next pair's loads
      // into operands (tag test, masking the tags off, the rotated copies) is cut into single instructions, and one
      // is placed behind each of the first MFMAs of the pair before: there it costs nothing, in front of the pair's
      // own MFMAs it was a fifth of the step.  A pair with a stale tag in any lane is skipped (wave-uniform branch)
      // and both its loads are fetched again by fix_up.
      static_assert((NIT / 2) % 2 == 0, "loads are consumed in pairs");
      constexpr int NL = NIT / 2, NP = NL / 2, kPrepSteps = 14;
      u32x4 x[NL];
      const unsigned tagw = rd.tag << 16;
      // The poll IS the first pair of loads: they are repeated (bounded) until all their tags have turned, and what
      // the last round fetched is kept.  Only then are the other loads issued; their round trip passes behind the
      // first pair's MFMAs instead of in front of the whole stream (a poll of its own followed by all loads cost one
      // round trip more per step, a tenth of it).  (Nine times out of ten the first round succeeds; yet issuing
      // everything at once without looking was measured slower: the values arrive while the poll is in flight.)
      for (unsigned poll = 0;; ++poll) {
        x[0] = rd.load_it(rd.it_of(0));
        x[1] = rd.load_it(rd.it_of(1));
        // The accumulators are cleared while the poll is in flight.  (By moves: starting each chain with an MFMA that
        // adds to the constant 0, as the backward kernel does, was measured 10 % slower per step here.)
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
          for (int q = 0; q < 4; ++q) acc[ct][q] = (f32x4){0.f, 0.f, 0.f, 0.f};
        operands_settle(acc[0][0], acc[0][1], acc[0][2], acc[0][3]);
        operands_settle(acc[1][0], acc[1][1], acc[1][2], acc[1][3]);
        __builtin_amdgcn_sched_barrier(0);
        if (dead) break;
        const unsigned stale = rd.tag_diff(x[0], rd.it_of(0), tagw) | rd.tag_diff(x[1], rd.it_of(1), tagw);
        if (__builtin_amdgcn_ballot_w64(stale > 0xffffu) == 0ull) break;
        if (poll >= rd.limit || ((poll & 63u) == 63u && ld_relaxed(err) != 0u)) {
          st_relaxed(err, 1u);
          dead = true;
          break;
        }
        PROF_POLLS(1)
      }
      PROF_MARK(5)
#pragma unroll
      for (int i = 2; i < NL; ++i) x[i] = rd.load_it(rd.it_of(i));
      __builtin_amdgcn_sched_barrier(0);
      u32x4 ops[NP][4];                                    // [0] load 2p as fetched, [1] its rows rotated by 8, [2], [3]: load 2p+1
      unsigned bad[NP];                                    // tag mismatches of the pair, per lane, in the upper 16 bits
      auto prep = [&](int p, int k) __attribute__((always_inline)) {
        const int second = k >= kPrepSteps / 2, i = 2 * p + second, kk = second ? k - kPrepSteps / 2 : k;
        if (kk == 0) {
          const unsigned m = rd.tag_diff(x[i], rd.it_of(i), tagw);
          bad[p] = second ? (bad[p] | m) : m;
        } else if (kk == 1) {
          x[i][1] &= ~kLLFwdTagBit;
        } else if (kk == 2) {
          x[i][3] &= ~kLLFwdTagBit;
          ops[p][2 * second] = x[i];
        } else {
          ops[p][2 * second + 1][kk - 3] = (unsigned)__builtin_amdgcn_mov_dpp((int)x[i][kk - 3], 0x128, 0xf, 0xf, false);
        }
      };
      unsigned long long redo = 0ull;
#pragma unroll
      for (int k = 0; k < kPrepSteps; ++k) prep(0, k);
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        __builtin_amdgcn_sched_barrier(0);
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(bad[p] > 0xffffu) == 0ull, 1)) {
          operands_settle(ops[p][0], ops[p][1], ops[p][2], ops[p][3]);
          // The next frame's x W_x + b, from HBM, goes out where this wavefront's last ring load has arrived.  The CU hands
          // loads back in the order of issue, other wavefronts' included: a pair earlier, it holds up the ring loads still
          // in flight (+17 % per step); behind the last pair's MFMAs, where it used to be, it is in the next step's poll's way (+3 %).
          if (p == NP - 1) fetch_zx(tau + 1, zx_next);
#pragma unroll
          for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
              for (int o = 0; o < 4; ++o) {
                mma_one(4 * p + o, ct, q, ops[p][o]);
                // the second pair's loads were issued just before the first pair's MFMAs: their turn comes late
                const int m = (ct * 4 + q) * 4 + o - (p == 0 ? 32 - kPrepSteps : kPrepDelay);
                if (p + 1 < NP && m >= 0 && m < kPrepSteps) {
                  __builtin_amdgcn_sched_barrier(0);
                  prep(p + 1, m);
                  __builtin_amdgcn_sched_barrier(0);
                }

              }
        } else {                                           // rare once the sample has turned
          redo |= 3ull << (2 * p);
          if (p == NP - 1) fetch_zx(tau + 1, zx_next);
          if (p + 1 < NP) {
            // The empty statement makes the loads' registers new values on this path: instructions that are the
            // same on both paths are moved in front of the branch, and with them the wait for the next pair's loads.
            asm volatile("" : "+v"(x[2 * p + 2]), "+v"(x[2 * p + 3]));
#pragma unroll
            for (int k = 0; k < kPrepSteps; ++k) prep(p + 1, k);
          }
        }
      }
      PROF_REDO(__popcll(redo))
      if (redo) {
        rd.fix_up_batch<NL>(redo, dead, use_single);
        // (nothing of that is outstanding any more - said with an instruction the compiler takes note of: it cannot tell
        // from the loop's exits, and would make whatever reuses those registers below wait for every load in flight)
        __builtin_amdgcn_s_waitcnt(0x0f70);                // vmcnt(0)
      }
      mfma_settle(acc[0][0], acc[0][1], acc[0][2], acc[0][3], acc[1][0], acc[1][1], acc[1][2], acc[1][3]);
    }
    PROF_MARK(0)
    // accumulator rows 4*(lane/16) + v; this work-group's rows sit in fragment rows 0..7
    if (lane < 32) {
#pragma unroll
      for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int v = 0; v < 4; ++v) red_[wave][4 * (lane >> 4) + v][q * 32 + ct * 16 + (lane & 15)] = acc[ct][q][v];
    }
    PROF_MARK(1)
    __syncthreads();

    CellOut o = {};
    if (valid) {
      float zh[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) zh[q] = red_[0][r8][q * 32 + u] + red_[1][r8][q * 32 + u] + red_[2][r8][q * 32 + u] + red_[3][r8][q * 32 + u];
      o = lstm_cell(zh, zx, c);
      c = o.c; h = o.h;
    }
    const unsigned h_bits = pack_bf16x2(h, 0.f) & 0xffffu; // inactive threads hold h = 0: padding rows / units publish zeros
    started = started || valid;
    PROF_MARK(2)
    {                                 // the recurrence's critical store goes out first
      // h of the next three units of the tile (DPP row_shl:1, :2, :3; past the row of 16 lanes: zero)
      const unsigned x0 = started ? h_bits : 0u;
      const unsigned x1 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)x0, 0x101, 0xf, 0xf, true);
      const unsigned x2 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)x0, 0x102, 0xf, 0xf, true);
      const unsigned x3 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)x0, 0x103, 0xf, 0xf, true);
      const u32x2 unit = {x0 | (x1 << 16), x2 | (x3 << 16) | (ll_fwd_tag((unsigned)tau + 1u) << 30)};
      const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc((void*)((tau & 1) ? d.ring0 : d.ring1), 0, kParked, kBufFlags);
      // 1: workgroup scope, stays in this XCD's L2;  16: agent scope, written through
      if (local) __builtin_amdgcn_raw_buffer_store_b64(unit, ro, pub_off, 0, 1);
      else __builtin_amdgcn_raw_buffer_store_b64(unit, ro, pub_off, 0, 16);
    }
    {                                 // layer outputs and what the backward pass needs (2: non-temporal)
      __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(valid ? h_bits : 0u), frame_of(d.y, t, y_bytes), y_off, 0, 2);
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(c), frame_of(d.cs, t, s_bytes), s_off, 0, 2);
      __builtin_amdgcn_raw_buffer_store_b16((unsigned short)h_prev_bits, frame_of(d.hprev, t, s_bytes >> 1), s_off >> 1, 0, 2);
      const __amdgpu_buffer_rsrc_t rw = frame_of(d.gates, t, g_bytes, a.write_gates != 0);
      const unsigned gw = valid ? g_off : kParked;
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o.gi), rw, gw, 0u, 2);
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o.gf), rw, gw, 4u * n, 2);
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o.gg), rw, gw, 8u * n, 2);
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o.go), rw, gw, 12u * n, 2);
    }
    h_prev_bits = h_bits;
    PROF_MARK(3)
  };
  for (int tau = 0; tau < T; tau += 2) {
    step(tau, zx_a, zx_b, std::integral_constant<int, 0>{});
    if (tau + 1 < T) step(tau + 1, zx_b, zx_a, std::integral_constant<int, 1>{});
  }
  PROF_DUMP("fwd8", T)
  if (active) {
    d.cstate[(long)b * n + j] = c;
    d.hstate[(long)b * n + j] = h;
  }
}

// ------------------------------------------------------------------------------------------------
// forward, third decomposition: a work-group owns 32 units for all 16 rows of a row tile.  For batches of more than
// 32 rows: 64 rows x 2 directions are then 256 work-groups, one launch, where the 32 x 8 form needs two launches
// that each walk all T steps.  Every MFMA row is a real row (96 MFMAs per wavefront and step, as in the 32 x 8 form,
// for twice the rows), a load is one whole chunk (12 loads per wavefront and step instead of 6), and a thread
// updates two cells (rows r8 and r8 + 8).  Ring layout, tags and publishing are those of the 32 x 8 form.
template <int NIT>
__global__ __launch_bounds__(256) void persist_fwd16r_kernel(PFwdArgs a) {
  __shared__ float red[2][4][16][129];                   // two copies, used by even and odd steps: one barrier per step
  // x W_x + b of the next frame, fetched one step ahead by loads that write LDS instead of registers (the register
  // file has no room for two sets of 8 values per thread): [set][wavefront][row k, gate q][lane], each thread reading
  // back exactly what it asked for, so no barrier is involved - only the loads' completion.
  __shared__ float zxs[2][4][8][64];
  __shared__ u32x4 rbuf[4][NIT][64];                     // the ring loads of a step: [wavefront][load][lane], written by the memory unit
  const WgCoord wg = wg_coord();
  const PFwdDir d = a.d[wg.dir];       // a copy: fields read through a reference are fetched again in every time step
  const int tile2 = wg.tile, rt = a.rt0 + wg.rt;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // (told to be wave-uniform: it forms scalar LDS addresses below)
  const int nkc = a.nkc, n = a.n, B = a.B, T = a.T;
  const int ntiles16 = (n + 15) / 16;
  unsigned* err = a.sync;
  bool dead = false;

  const int nitv = (nkc + 3) / 4, rot = tile2 % nitv;
  // Register set `it` holds the chunk that load `it` of the stream fetches; the first kAccIts sets fill the 256
  // accumulation registers, the rest sit in vector registers (as in the 32 x 8 form).
  constexpr int kAccIts = NIT < 8 ? NIT : 8;
  u32x4 wa[kAccIts][2][4];
  u32x4 wv[NIT - kAccIts > 0 ? NIT - kAccIts : 1][2][4];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    const int kc = wave + 4 * rot_index(it, rot, nitv);
#pragma unroll
    for (int ct = 0; ct < 2; ++ct) {
      const int t16 = tile2 * 2 + ct;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint4* src = (kc < nkc && t16 < ntiles16) ? &d.Wf[((long)(t16 * 4 + q) * nkc + kc) * 64 + lane] : &d.Wzero[lane];
        if (it < kAccIts) wa[it][ct][q] = load_to_agpr(src);
        else wv[it - kAccIts][ct][q] = *(const u32x4*)src;
      }
    }
  }
  agpr_loads_done();

  const int r8 = tid >> 5, u = tid & 31;                 // pointwise pairs of this thread: rows r8 and r8 + 8, unit u of 32
  const int j = tile2 * 32 + u;
  float c[2] = {0.f, 0.f}, h[2] = {0.f, 0.f};
  int L[2] = {0, 0};
  bool active[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int b = rt * 16 + r8 + 8 * k;
    active[k] = b < B && j < n;
    if (active[k]) {
      c[k] = d.cstate[(long)b * n + j];
      h[k] = d.hstate[(long)b * n + j];
      L[k] = clamp_len(a.lens, b, T);
    }
  }
  const int pp = u >> 4, m = (u & 15) >> 2;                // the unit (four units' h, see the 32 x 8 kernel) this thread publishes
  const int t16p = tile2 * 2 + pp;
  const int cch = t16p * 2 + (m >> 1);
  const bool publishes = (u & 3) == 0 && t16p < ntiles16;
  bool started[2] = {false, false};                      // (see the 32 x 8 kernel)
  const bool local = a.xcc != nullptr &&
                     group_is_xcd_local(a.xcc, (wg.dir * (int)gridDim.y + wg.rt) * (int)gridDim.x, gridDim.x, tile2, a.spin_limit);

  constexpr unsigned kParked = 0x7ff00000u;
  const unsigned g_bytes = (unsigned)B * 4u * n * 4u, y_bytes = (unsigned)B * d.ldy * 2u, s_bytes = (unsigned)B * n * 4u;
  // offsets of row r8 inside a frame; row r8 + 8 lies a wave-uniform distance behind it (a row of the second half
  // that exists implies its partner in the first half does), which keeps four registers free
  const unsigned b0 = (unsigned)(rt * 16 + r8);
  const unsigned g_off0 = active[0] ? (b0 * 4u * n + j) * 4u : kParked;
  const unsigned y_off0 = active[0] ? (b0 * d.ldy + j) * 2u : kParked;
  const unsigned s_off0 = active[0] ? (b0 * n + j) * 4u : kParked;
  const unsigned pub_off0 = publishes ? (unsigned)((((long)rt * nkc + (cch >> 2)) * 64 + (cch & 3) * 16 + r8) * 2 + (m & 1)) * 8u : kParked;
  auto g_off = [&](int k) { return k == 0 ? g_off0 : (active[1] ? g_off0 + 8u * 4u * n * 4u : kParked); };
  auto y_off = [&](int k) { return k == 0 ? y_off0 : (active[1] ? y_off0 + 8u * (unsigned)d.ldy * 2u : kParked); };
  auto s_off = [&](int k) { return k == 0 ? s_off0 : (active[1] ? s_off0 + 8u * n * 4u : kParked); };
  auto pub_off = [&](int k) { return k == 0 ? pub_off0 : (publishes ? pub_off0 + 8u * 16u : kParked); };
  auto frame_of = [&](const void* base, int t, unsigned bytes, bool present = true) {
    return __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)base + (unsigned long long)(unsigned)t * bytes), 0, present && base != nullptr ? bytes : 0u, kBufFlags);
  };
  const unsigned zxs_base = (unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)&zxs[0][0][0][0];
  const unsigned rbuf_base = (unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)&rbuf[0][0][0];
  // (assembly: the compiler makes every later LDS read wait for all loads of this kind that it knows to be in flight;
  // the kernel counts them itself - see the wait in front of the cell update)
  auto fetch_zx = [&](int tau, int set) __attribute__((always_inline)) {
    const bool ok = tau < T;
    const int t = d.rev ? T - 1 - tau : tau;
    const __amdgpu_buffer_rsrc_t rg =
        __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)d.gates + (unsigned long long)(unsigned)(ok ? t : 0) * g_bytes), 0, ok ? g_bytes : 0u, kBufFlags);
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const unsigned go = t < L[k] ? g_off(k) : kParked;     // (L is 0 in lanes without a row)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const unsigned dst = zxs_base + (unsigned)(((set * 4 + wave) * 8 + k * 4 + q) * 256);
        asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dword %1, %2, %3 offen nt lds" ::"s"(dst), "v"(go), "s"(rg), "s"((unsigned)q * 4u * n) : "memory");
      }
    }
  };
  unsigned h_prev_bits[2] = {pack_bf16x2(h[0], 0.f) & 0xffffu, pack_bf16x2(h[1], 0.f) & 0xffffu};
  fetch_zx(0, 0);
  PROF_DECL
  auto step = [&](const int tau, auto parity) __attribute__((always_inline)) {
    constexpr int kSet = decltype(parity)::value;
    float (&red_)[4][16][129] = red[decltype(parity)::value];
    const int t = d.rev ? T - 1 - tau : tau;
    PROF_MARK(4)
    const uint4* rin = ((tau & 1) ? d.ring1 : d.ring0) + (long)rt * nkc * 64;
    RingReader rd = make_reader(rin, nkc, ntiles16 * 2, wave, lane, ll_fwd_tag((unsigned)tau) << 14, err, a.spin_limit, rot);
    f32x4 acc[2][4];
    {
      auto mma_one = [&](int it, int ct, int q, const u32x4& a_op) __attribute__((always_inline)) {
        if (it < kAccIts) mfma_b_agpr(acc[ct][q], a_op, wa[it < kAccIts ? it : 0][ct][q]);
        else mfma_b_vgpr(acc[ct][q], a_op, wv[it >= kAccIts ? it - kAccIts : 0][ct][q]);
      };
      auto use_single = [&](int i, const u32x4& raw) {     // a load fetched again after the stream, tags still in it
        u32x4 av = {raw[0], raw[1] & ~kLLFwdTagBit, raw[2], raw[3] & ~kLLFwdTagBit}, dummy = av;
        operands_settle(av, dummy);
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
          for (int q = 0; q < 4; ++q) mma_one(i, ct, q, av);
      };
      // The loads are consumed in pairs (two chunks, 16 MFMAs); what turns the next pair's loads into operands (tag
      // test, masking the tags off) is cut into single instructions that follow the first MFMAs of the pair before.
      static_assert(NIT % 2 == 0, "loads are consumed in pairs");
      constexpr int NP = NIT / 2, kPrepSteps = 6;
      // The first pair of loads is the poll and lands in registers.  The others are written to LDS by the memory
      // unit (rbuf: no registers are held while they are in flight, so all of them fly at once) and are read back
      // a pair ahead of their MFMAs; loads complete in the order of issue, which is what the counted waits rely on.
      u32x4 x[2][2];
      const unsigned tagw = rd.tag << 16;
      auto issue_dma = [&](int i) __attribute__((always_inline)) {
        const unsigned dst = rbuf_base + (unsigned)(wave * NIT + i) * 1024u, soff = (unsigned)rd.it_of(i) * rd.it_bytes;
        asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen sc1 lds" ::"s"(dst), "v"(rd.voff), "s"(rd.rs), "s"(soff) : "memory");
      };
      // (Fetching everything along with the first poll - stale loads now being cheap to repeat - was measured 15 % slower
      // per step: the polled pair then returns behind 10 KiB of other loads, most of which are repeated anyway.)
      for (unsigned poll = 0;; ++poll) {
        x[0][0] = rd.load_it(rd.it_of(0));
        x[0][1] = rd.load_it(rd.it_of(1));
        __builtin_amdgcn_sched_barrier(0);
        if (poll == 0) {
#pragma unroll
          for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[ct][q] = (f32x4){0.f, 0.f, 0.f, 0.f};
          operands_settle(acc[0][0], acc[0][1], acc[0][2], acc[0][3]);
          operands_settle(acc[1][0], acc[1][1], acc[1][2], acc[1][3]);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (dead) break;
        const unsigned stale = rd.tag_diff(x[0][0], rd.it_of(0), tagw) | rd.tag_diff(x[0][1], rd.it_of(1), tagw);
        if (__builtin_amdgcn_ballot_w64(stale > 0xffffu) == 0ull) break;
        if (poll >= rd.limit || ((poll & 63u) == 63u && ld_relaxed(err) != 0u)) {
          st_relaxed(err, 1u);
          dead = true;
          break;
        }
        PROF_POLLS(1)
      }
      PROF_MARK(5)
#pragma unroll
      for (int i = 2; i < NIT; ++i) issue_dma(i);
      __builtin_amdgcn_sched_barrier(0);
      unsigned bad[NP];
      // pair p + 1 becomes operands behind MFMA `at` of pair p: wait for its loads, read them from LDS (step -1);
      // tag test and masking (steps 0 .. kPrepSteps - 1) follow a few MFMAs later, when the LDS reads have returned
      auto prep = [&](auto P, int k) __attribute__((always_inline)) {
        constexpr int p = decltype(P)::value;
        u32x4 (&xp)[2] = x[p & 1];
        if (k < 0) {
          asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NIT - 2 - 2 * p) : "memory");     // all but the loads behind this pair have landed
          xp[0] = rbuf[wave][2 * p][lane];
          xp[1] = rbuf[wave][2 * p + 1][lane];
          return;
        }
        const int second = k >= kPrepSteps / 2, i = 2 * p + second, kk = second ? k - kPrepSteps / 2 : k;
        u32x4& xi = xp[second];
        if (kk == 0) {
          const unsigned mm = rd.tag_diff(xi, rd.it_of(i), tagw);
          bad[p] = second ? (bad[p] | mm) : mm;
        } else if (kk == 1) {
          xi[1] &= ~kLLFwdTagBit;
        } else {
          xi[3] &= ~kLLFwdTagBit;
        }
      };
      unsigned long long redo = 0ull;
      bool zx_asked = false;
#pragma unroll
      for (int k = 0; k < kPrepSteps; ++k) prep(std::integral_constant<int, 0>{}, k);
      static_for<NP>([&](auto P) __attribute__((always_inline)) {
        constexpr int p = decltype(P)::value;
        constexpr std::integral_constant<int, (p + 1 < NP ? p + 1 : p)> P1{};
        // the second pair's loads have just been issued: reading them early would only stall this pair's MFMAs
        constexpr int read_at = p == 0 ? 15 : 2, prep_at = p == 0 ? 16 : 9;
        __builtin_amdgcn_sched_barrier(0);
        if (__builtin_expect(__builtin_amdgcn_ballot_w64(bad[p] > 0xffffu) == 0ull, 1)) {
          operands_settle(x[p & 1][0], x[p & 1][1]);
          // The next frame's x W_x + b goes out where this wavefront's last ring load has arrived (see the 32 x 8 kernel) -
          // unless a pair is being fetched again: the second look below waits for everything in flight, and these come from HBM.
          if (p == NP - 1 && redo == 0ull) {
            fetch_zx(tau + 1, kSet ^ 1);
            zx_asked = true;
          }
#pragma unroll
          for (int o = 0; o < 2; ++o)
#pragma unroll
            for (int ct = 0; ct < 2; ++ct)
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                mma_one(2 * p + o, ct, q, x[p & 1][o]);
                const int mm = (o * 2 + ct) * 4 + q;
                if (p + 1 < NP && (mm == read_at || (mm >= prep_at && mm < prep_at + kPrepSteps))) {
                  __builtin_amdgcn_sched_barrier(0);
                  prep(P1, mm == read_at ? -1 : mm - prep_at);
                  __builtin_amdgcn_sched_barrier(0);
                }
              }
          if (p + 1 < NP) {
#pragma unroll
            for (int k = 0; k < kPrepSteps; ++k)
              if (prep_at + k >= 16) prep(P1, k);            // what did not fit behind this pair's MFMAs
          }
        } else {
          // Stale: the pair's loads are issued again at once, behind the others, and looked at after the last pair, so
          // their round trip passes behind the MFMAs still to come.  (The counted waits of later pairs then wait for
          // up to that many loads more than they need: loads complete in order, so they wait for no less.)
          redo |= 3ull << (2 * p);
          if (p > 0) {
            issue_dma(2 * p);
            issue_dma(2 * p + 1);
          }
          if (p + 1 < NP) {
#pragma unroll
            for (int k = -1; k < kPrepSteps; ++k) prep(P1, k);
          }
        }
      });
      if (redo >> 2) {                                     // the second look at what was fetched again
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        static_for<NP - 1>([&](auto P) __attribute__((always_inline)) {
          constexpr int p = decltype(P)::value + 1;
          if ((redo >> (2 * p)) & 1ull) {
            const u32x4 y0 = rbuf[wave][2 * p][lane], y1 = rbuf[wave][2 * p + 1][lane];
            if (__builtin_amdgcn_ballot_w64((rd.stale_bits(y0, rd.it_of(2 * p)) | rd.stale_bits(y1, rd.it_of(2 * p + 1))) != 0u) == 0ull) {
              use_single(2 * p, y0);
              use_single(2 * p + 1, y1);
              redo &= ~(3ull << (2 * p));
            }
          }
        });
      }
      PROF_REDO(__popcll(redo))
      if (redo) {                                          // (a quarter of the loads at a time: registers)
        rd.template fix_up_batch<NIT / 4, 0>(redo, dead, use_single);
        rd.template fix_up_batch<NIT / 4, NIT / 4>(redo, dead, use_single);
        rd.template fix_up_batch<NIT / 4, NIT / 2>(redo, dead, use_single);
        rd.template fix_up_batch<NIT / 4, 3 * (NIT / 4)>(redo, dead, use_single);
      }
      mfma_settle(acc[0][0], acc[0][1], acc[0][2], acc[0][3], acc[1][0], acc[1][1], acc[1][2], acc[1][3]);
      if (!zx_asked) fetch_zx(tau + 1, kSet ^ 1);
    }
    PROF_MARK(0)
    // (LDS addresses are formed anew in every step: hoisted out of the loop they stay in registers the loop does not have)
    int lane_ = lane, u_ = u, r8_ = r8;
    asm volatile("" : "+v"(lane_), "+v"(u_), "+v"(r8_));
    // accumulator rows 4*(lane/16) + v: every row is one of this work-group's
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int v = 0; v < 4; ++v) red_[wave][4 * (lane_ >> 4) + v][q * 32 + ct * 16 + (lane_ & 15)] = acc[ct][q][v];
    PROF_MARK(1)
    // this frame's x W_x + b was asked for one step ago: everything but the 8 loads just issued has completed
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
    __syncthreads();
    const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc((void*)((tau & 1) ? d.ring0 : d.ring1), 0, kParked, kBufFlags);
    const __amdgpu_buffer_rsrc_t ry = frame_of(d.y, t, y_bytes), rc = frame_of(d.cs, t, s_bytes), rh = frame_of(d.hprev, t, s_bytes >> 1);
    const __amdgpu_buffer_rsrc_t rw = frame_of(d.gates, t, g_bytes, a.write_gates != 0);
    // both cells first, then both ring stores (the recurrence's critical stores, close together so that the two halves
    // of a row tile turn their tags at about the same time), then the outputs
    CellOut o[2] = {};
    bool valid[2];
    unsigned h_bits[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const int rr = r8_ + 8 * k;
      valid[k] = active[k] && t < L[k];
      if (valid[k]) {
        float zh[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) zh[q] = red_[0][rr][q * 32 + u_] + red_[1][rr][q * 32 + u_] + red_[2][rr][q * 32 + u_] + red_[3][rr][q * 32 + u_];
        float zx[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) zx[q] = zxs[kSet][wave][k * 4 + q][lane_];
        o[k] = lstm_cell(zh, zx, c[k]);
        c[k] = o[k].c; h[k] = o[k].h;
      }
      h_bits[k] = pack_bf16x2(h[k], 0.f) & 0xffffu;         // inactive threads hold h = 0: padding rows / units publish zeros
      started[k] = started[k] || valid[k];
    }
    PROF_MARK(2)
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const unsigned x0 = started[k] ? h_bits[k] : 0u;
      const unsigned x1 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)x0, 0x101, 0xf, 0xf, true);
      const unsigned x2 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)x0, 0x102, 0xf, 0xf, true);
      const unsigned x3 = (unsigned)__builtin_amdgcn_update_dpp(0, (int)x0, 0x103, 0xf, 0xf, true);
      const u32x2 unit = {x0 | (x1 << 16), x2 | (x3 << 16) | (ll_fwd_tag((unsigned)tau + 1u) << 30)};
      if (local) __builtin_amdgcn_raw_buffer_store_b64(unit, ro, pub_off(k), 0, 1);
      else __builtin_amdgcn_raw_buffer_store_b64(unit, ro, pub_off(k), 0, 16);
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {          // layer outputs and what the backward pass needs (2: non-temporal)
      __builtin_amdgcn_raw_buffer_store_b16((unsigned short)(valid[k] ? h_bits[k] : 0u), ry, y_off(k), 0, 2);
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(c[k]), rc, s_off(k), 0, 2);
      __builtin_amdgcn_raw_buffer_store_b16((unsigned short)h_prev_bits[k], rh, s_off(k) >> 1, 0, 2);
      const unsigned gw = valid[k] ? g_off(k) : kParked;
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o[k].gi), rw, gw, 0u, 2);
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o[k].gf), rw, gw, 4u * n, 2);
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o[k].gg), rw, gw, 8u * n, 2);
      __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(o[k].go), rw, gw, 12u * n, 2);
      h_prev_bits[k] = h_bits[k];
    }
    PROF_MARK(3)
  };
  for (int tau = 0; tau < T; tau += 2) {
    step(tau, std::integral_constant<int, 0>{});
    if (tau + 1 < T) step(tau + 1, std::integral_constant<int, 1>{});
  }
  PROF_DUMP("fwd16r", T)
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int b = rt * 16 + r8 + 8 * k;
    if (active[k]) {
      d.cstate[(long)b * n + j] = c[k];
      d.hstate[(long)b * n + j] = h[k];
    }
  }
}

// ------------------------------------------------------------------------------------------------
// backward, third decomposition ("partial sums"): no dz crosses work-groups.  A work-group still owns 32 units for
// 8 rows, but it multiplies ITS dz (8 rows x 128 gate columns) by the matching 128 rows of W_h^T for ALL n outputs
// and publishes, per destination tile of 32 units, a partial sum of Dh (bf16).  A consumer adds the partial sums
// of its tile from all producers: 1 KiB per producer, 32 KiB per step at n = 1024, where reading dz itself takes
// 88 KiB.  The ring read is what bounds the backward step, so this is the fastest of the three forms.  Dh is
// therefore a sum of bf16-rounded partial sums (accumulated in float), not a float product of bf16-rounded dz.
//
// With one wavefront per SIMD every instruction's latency is exposed (about 2 ns each), so the formats are chosen
// to keep instruction counts low: an 8-byte unit holds values of ONE output for four ROWS, which
// is how an MFMA accumulator lane holds them, so a producer stores straight from its accumulators - no staging,
// no cross-lane moves.  Ring layout per direction and slot:
//   [row group][destination tile][producer tile][32 outputs][2 row halves] x 8 bytes (rows 4g .. 4g+3 as bf16).
// The tag is ONE BIT, bit 14 of the fourth value (see the forward ring): the partial sums travel scaled by 2^-32 - the
// packed W_h carries the factor, so the MFMAs deliver them scaled, and the consumer multiplies its sum by 2^32 - which
// leaves that bit 0 for every partial sum below 2^33 in magnitude and changes no other bit of any value above 2^-94
// (a power of two commutes with every rounding on the way).  A partial sum of 2^33 or more cannot be exchanged: its
// unit looks stale or fresh at random; gradients of that size are past use, and the case mostly ends in an expired wait.
// Half the bytes and half the ring loads of the format this replaces (3 values + a 16-bit tag per unit, 16 bytes per lane).
// W_h slice in registers: w[kc][c] = B fragment of gate kc (K = this tile's 32 units) for column tile
// wave*16 + c of the n outputs.
constexpr int kPartBytes = 512;                           // one (producer, destination tile)
constexpr float kPartScale = 1.f / 4294967296.f;          // 2^-32
// tag bit of the partial sums that backward step sigma (= T-1-tau) consumes: written by step sigma - 1 into slot
// (sigma - 1) & 1; alternates between consecutive uses of a slot and is 1 at the first, so zero-filled slots look unwritten
__device__ __forceinline__ unsigned part_tag(int sigma) { return ((((unsigned)sigma - 1u) >> 1) & 1u) ^ 1u; }

template <int NPW>                                        // producers per wavefront at most: n <= 128 * NPW
__global__ __launch_bounds__(256) void persist_bwdp_kernel(PBwdArgs a) {
  __shared__ float red[8][8][33];                        // [wavefront, producer of the pair][row][output]
  __shared__ __attribute__((aligned(16))) unsigned short zb[8][136];
  const WgCoord wg = wg_coord();
  const PBwdDir d = a.d[wg.dir];       // a copy: fields read through a reference are fetched again in every time step
  const int J = wg.tile, R = 2 * a.rt0 + wg.rt, ntile2 = gridDim.x;     // R: row group of 8 rows, counted over the whole batch
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n = a.n, B = a.B, T = a.T;
  unsigned* err = a.sync;
  bool dead = false;

  u32x4 w[4][16];                                        // all 256 accumulation registers
#pragma unroll
  for (int kc = 0; kc < 4; ++kc)
#pragma unroll
    for (int c = 0; c < 16; ++c) w[kc][c] = load_to_agpr(&d.Wb[((((long)J * 4 + wave) * 4 + kc) * 16 + c) * 64 + lane]);
  agpr_loads_done();

  const int r8 = tid >> 5, u = tid & 31;                 // pointwise pair of this thread
  const int b = R * 8 + r8, j = J * 32 + u;
  const bool active = b < B && j < n;
  float Dh = 0.f, Dc = 0.f;
  float dbsum[4] = {0.f, 0.f, 0.f, 0.f};
  int L = 0;
  if (active) {
    Dh = d.Dh[(long)b * n + j];
    Dc = d.Dc[(long)b * n + j];
    L = clamp_len(a.lens, b, T);
  }
  // What the gate gradients of one frame need.  dy stays as the 16 bits that were loaded: a conversion right behind
  // the load would make the wavefront wait for it - and for every load in front of it - where it is issued.
  struct In { float gi, gf, gg, go, c_new, c_prev; unsigned dy_bits; };
  // The per-frame arrays are read through buffer descriptors that cover exactly one frame: the frame's address is
  // scalar arithmetic, a lane's offset inside the frame never changes, and a lane with nothing to fetch (row past the
  // batch, unit past n, frame past the row's length) has its offset parked outside the frame and gets zeros without
  // touching memory - as does every lane when the frame itself does not exist (zero-sized descriptor).  Nothing is
  // predicated, so every step issues the same six loads; with loads that may or may not have been issued the
  // compiler has to assume the fewest, and made the wavefront wait for the loads of the NEXT frame, just issued and
  // on their way from HBM, where it only needed those of this one.
  constexpr unsigned kParked = 0x7ff00000u;
  const unsigned g_bytes = (unsigned)B * 4u * n * 4u, s_bytes = (unsigned)B * n * 4u, y_bytes = (unsigned)B * d.lddy * 2u;
  const unsigned g_off = active ? ((unsigned)b * 4u * n + j) * 4u : kParked;
  const unsigned s_off = active ? ((unsigned)b * n + j) * 4u : kParked;
  const unsigned y_off = active ? ((unsigned)b * d.lddy + j) * 2u : kParked;
  auto frame_of = [&](const void* base, int t, unsigned bytes) {
    const bool ok = t >= 0 && t < T;
    return __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)base + (unsigned long long)(unsigned)(ok ? t : 0) * bytes), 0, ok ? bytes : 0u, kBufFlags);
  };
  auto ld_f = [&](__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {     // 2: non-temporal
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 2));
  };
  auto fetch_in = [&](int tau) {
    const int t = tau < 0 ? -1 : (d.rev ? T - 1 - tau : tau);
    const bool lane_on = t < L;                            // (L is 0 in lanes without a row)
    const unsigned go = lane_on ? g_off : kParked, so = lane_on ? s_off : kParked, yo = lane_on ? y_off : kParked;
    In in;
    const __amdgpu_buffer_rsrc_t rg = frame_of(d.gates, t, g_bytes);
    in.gi = ld_f(rg, go, 0u); in.gf = ld_f(rg, go, 4u * n); in.gg = ld_f(rg, go, 8u * n); in.go = ld_f(rg, go, 12u * n);
    const int tp = d.rev ? t + 1 : t - 1;                  // the frame before t in processing order
    const bool inside = t >= 0 && tp >= 0 && tp < T, initial = t >= 0 && !inside && d.c0 != nullptr;
    const __amdgpu_buffer_rsrc_t rp = initial ? __builtin_amdgcn_make_buffer_rsrc((void*)d.c0, 0, s_bytes, kBufFlags)
                                              : frame_of(d.cs, inside ? tp : -1, s_bytes);
    // The cell state entering frame t is the state leaving the frame before it, which is the NEXT backward step's
    // frame: that step takes its c_new from here instead of loading it again (one load per step less).  So the value is
    // also fetched where frame t itself is padding but the frame before it is real (direction +1, t = the row's length).
    in.c_prev = ld_f(rp, (d.rev ? t : t - 1) < L ? s_off : kParked, 0u);
    in.c_new = 0.f;                                        // supplied by the caller
    in.dy_bits = __builtin_amdgcn_raw_buffer_load_b16(frame_of(d.dy, t, y_bytes), yo, 0, 2);
    return in;
  };
  // entries of DZ, which this thread stores: a pointer that moves by one frame per step
  const long row_last = (long)(d.rev ? 0 : T - 1) * B + b, g_step = (d.rev ? (long)B : -(long)B) * 4 * n;
  unsigned short* dz_p = (unsigned short*)d.DZ + row_last * 4 * n + j;
  In in_a = fetch_in(T - 1), in_b = in_a;
  {                                                        // the first frame's own cell state: the only one loaded as such
    const int t0 = d.rev ? 0 : T - 1;
    in_a.c_new = ld_f(frame_of(d.cs, t0, s_bytes), t0 < L ? s_off : kParked, 0u);
  }

  // consumer side: a load covers two producers' blocks; lane reads output lane%32, all eight rows, of producer lane/32
  const int ccol = lane & 31, chalf = lane >> 5;
  const int nitv = (ntile2 + 7) / 8, rot = J % nitv;
  const long ring_tile = ((long)R * ntile2 + J) * ntile2 * (kPartBytes / 16);     // uint4 index of [R][J][0]
  // producer side: lanes 0..31 hold rows 4*(lane/16) .. +3 of output column lane%16 of each accumulator tile
  const int pg = (lane >> 4) & 1, pcol = lane & 15;
  // (the verdict comes out of shared memory; the compiler has to be told that it is the same in every lane, or the
  // two copies of the publishing code below become one divergent region)
  const bool local = __builtin_amdgcn_readfirstlane((int)(a.xcc != nullptr &&
                     group_is_xcd_local(a.xcc, (wg.dir * (int)gridDim.y + wg.rt) * ntile2, ntile2, J, a.spin_limit))) != 0;
  // byte offset, from row group R's part of the ring, of what this lane stores for accumulator tile c: destination tile
  // wave*8 + c/2 (one past the last falls outside the buffer), this producer's block, output column, row half.  Lanes
  // 32..63 hold copies of the same rows; their offset is parked outside the buffer and the store is dropped.
  unsigned pub_off[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) {
    const int Jd = wave * 8 + (c >> 1);
    pub_off[c] = lane < 32 ? (unsigned)(((Jd * ntile2 + J) * 32 + (c & 1) * 16 + pcol) * 2 + pg) * 8u : 0xfff00000u;
  }

  PROF_DECL
  // One time step.  `in` holds the inputs of this step's frame and `in_next` receives those of the next; the loop
  // below calls it with the two in alternating roles, because a copy at the end of a step would have to wait for
  // the loads (and, counted with them, the step's stores) at that point.
  // `ring_c`: the step reads partial sums (every step but the first); `pointwise_c`: it has a frame (every step but the
  // last, which only collects the Dh that leaves the layer).  Constants of the call, so that the loop below is free
  // of the two exceptions: with them inside, the compiler's wait counts in the loop allowed for paths it never takes.
  auto step = [&](const int tau, const In& in, In& in_next, auto ring_c, auto pointwise_c) __attribute__((always_inline)) {
    PROF_MARK(4)
    // (told to be wave-uniform: computed next to per-lane uses of tau it ends up in vector registers, and a buffer
    // descriptor derived from it is then applied lane by lane in a loop)
    const int sigma = __builtin_amdgcn_readfirstlane(T - 1 - tau);
    const int t = d.rev ? T - 1 - tau : tau;
    const int t_next = d.rev ? t - 1 : t + 1;
    constexpr bool pointwise = decltype(pointwise_c)::value;
    const bool valid = pointwise && active && t < L;

    // The gate gradients of a valid frame, dh = dy + Dh (recurrent_dev.h has the plain form):
    //   dc = Dc + dh go (1 - tanh(c)^2), Dc' = dc gf, dz = (dc gg gi (1-gi), dc c_prev gf (1-gf), dc gi (1-gg^2), dh tanh(c) go (1-go)).
    // Everything that does not involve dh or Dc is computed while the ring loads are in flight.
    float f_c = 0.f, f_i = 0.f, f_f = 0.f, f_g = 0.f, f_o = 0.f;
    auto factors = [&]() __attribute__((always_inline)) {
      if (valid) {
        const float tc = tanhf_(in.c_new);
        f_c = in.go * (1.f - tc * tc);
        f_i = in.gg * in.gi * (1.f - in.gi);
        f_f = in.c_prev * in.gf * (1.f - in.gf);
        f_g = in.gi * (1.f - in.gg * in.gg);
        f_o = tc * in.go * (1.f - in.go);
      }
    };
    if constexpr (decltype(ring_c)::value) {
      RingReader rd;
      rd.rs = __builtin_amdgcn_make_buffer_rsrc((void*)((((sigma - 1) & 1) ? d.ring1 : d.ring0) + ring_tile), 0, ntile2 * kPartBytes,
                                                kBufFlags);
      // load `it` of this wavefront covers producers 2 * (wave + 4 * it) and the one after it (1 KiB)
      rd.voff = (unsigned)(wave * 2 * kPartBytes + lane * 16);
      rd.it_bytes = 8u * kPartBytes;
      rd.lim = ntile2 - 2 * wave - chalf; rd.lim_step = 8;
      rd.tag = part_tag(sigma) << 14; rd.err = err; rd.limit = a.spin_limit;
      rd.nitv = nitv; rd.rot = rot;
      constexpr int NLD = NPW / 2;                          // loads per wavefront
      float ps[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      {
        // The sums need no masking but the tag bit's: the shifts drop the other halves.  With one wavefront per SIMD what
        // bounds this phase is its instruction stream, and a verdict per load (compare, branch, or worse a ballot
        // handed to scalar registers) costs as much as the additions themselves.  So the loads behind the poll are
        // taken together: their values are added into sums of their own without looking, the tag differences are ORed
        // per lane, and one compare and branch decides whether those sums count.  If not, the loads are fetched
        // again, all at once, by fix_up_batch.
        auto add = [&](float (&acc)[8], const u32x4& v) __attribute__((always_inline)) {
          acc[0] += __uint_as_float(v[0] << 16); acc[1] += __uint_as_float(v[0] & 0xffff0000u);
          acc[2] += __uint_as_float(v[1] << 16); acc[3] += __uint_as_float(v[1] & (0xffff0000u & ~kLLFwdTagBit));
          acc[4] += __uint_as_float(v[2] << 16); acc[5] += __uint_as_float(v[2] & 0xffff0000u);
          acc[6] += __uint_as_float(v[3] << 16); acc[7] += __uint_as_float(v[3] & (0xffff0000u & ~kLLFwdTagBit));
        };
        static_assert(NLD >= 2, "the poll is two loads");
        u32x4 x[NLD];
        const unsigned tagw = rd.tag << 16;
        // The poll is the first two loads, repeated (bounded) until their tags have turned and then kept; the others
        // are issued behind it (see the forward kernel).
        for (unsigned poll = 0;; ++poll) {
          x[0] = rd.load_it(rd.it_of(0));
          x[1] = rd.load_it(rd.it_of(1));
          if (dead) break;
          const unsigned stale = rd.tag_diff(x[0], rd.it_of(0), tagw) | rd.tag_diff(x[1], rd.it_of(1), tagw);
          if (__builtin_amdgcn_ballot_w64(stale > 0xffffu) == 0ull) break;
          if (poll >= rd.limit || ((poll & 63u) == 63u && ld_relaxed(err) != 0u)) {
            st_relaxed(err, 1u);
            dead = true;
            break;
          }
          PROF_POLLS(1)
        }
        PROF_MARK(5)
        // Nothing is outstanding here (the poll has just been waited for, and loads complete in order).  Said with an
        // instruction the compiler takes note of: otherwise it makes the pointwise part below wait for this frame's
        // inputs, asked for a step ago, with a count that also waits for the next frame's, just asked for.
        __builtin_amdgcn_s_waitcnt(0x0f70);                // vmcnt(0)
#pragma unroll
        for (int i = 2; i < NLD; ++i) x[i] = rd.load_it(rd.it_of(i));
        __builtin_amdgcn_sched_barrier(0);
        // while those loads are on their way: the polled loads' values, and the part of the gate gradients that
        // does not need Dh
        add(ps, x[0]);
        add(ps, x[1]);
        factors();
        __builtin_amdgcn_sched_barrier(0);
        unsigned long long redo = 0ull;
        if (NLD > 2) {
          float pg[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          unsigned bad = 0u;
#pragma unroll
          for (int i = 2; i < NLD; ++i) {
            __builtin_amdgcn_sched_barrier(0);             // each load is waited for and consumed in turn
            bad |= rd.tag_diff(x[i], rd.it_of(i), tagw);
            add(pg, x[i]);
          }
          __builtin_amdgcn_sched_barrier(0);
          if (__builtin_expect(__builtin_amdgcn_ballot_w64(bad > 0xffffu) == 0ull, 1)) {
#pragma unroll
            for (int v = 0; v < 8; ++v) ps[v] += pg[v];
          } else {
            redo |= ((1ull << NLD) - 1ull) & ~3ull;
          }
        }
        PROF_REDO(__popcll(redo))
        if (redo) {
          rd.fix_up_batch<NLD>(redo, dead, [&](int, const u32x4& v) __attribute__((always_inline)) { add(ps, v); });
          // (nothing of that is outstanding any more - said with an instruction the compiler takes note of: it cannot tell
          // from the loop's exits, and would make whatever reuses those registers below wait for every load in flight)
          __builtin_amdgcn_s_waitcnt(0x0f70);              // vmcnt(0)
        }
        // The next frame's inputs, from HBM.  Loads complete in the order of issue: asked for in front of the groups
        // above (where their latency would be covered best) they held up every ring load behind them - a tenth of the step.
        in_next = fetch_in(tau - 1);
        in_next.c_new = in.c_prev;
      }
      PROF_MARK(0)
#pragma unroll
      for (int v = 0; v < 8; ++v) red[2 * wave + chalf][v][ccol] = ps[v];
      __syncthreads();
      if (active && t_next < L) {
        float sum = 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) sum += red[k][r8][u];
        Dh = sum * (1.f / kPartScale);                     // the partial sums travel scaled (see above)
      }
    } else {
      factors();
      in_next = fetch_in(tau - 1);
      in_next.c_new = in.c_prev;
    }
    if (pointwise) {
      float dz[4] = {0.f, 0.f, 0.f, 0.f};
      if (valid) {
        const float dh = bf_bits2f((unsigned short)in.dy_bits) + Dh, dc = Dc + dh * f_c;
        Dc = dc * in.gf;
        dz[0] = dc * f_i; dz[1] = dc * f_f; dz[2] = dc * f_g; dz[3] = dh * f_o;
      }
      const unsigned b01 = pack_bf16x2(dz[0], dz[1]), b23 = pack_bf16x2(dz[2], dz[3]);
      const unsigned short bits[4] = {(unsigned short)b01, (unsigned short)(b01 >> 16), (unsigned short)b23, (unsigned short)(b23 >> 16)};
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        dbsum[q] += dz[q];
        zb[r8][q * 32 + u] = bits[q];                      // inactive threads contribute zeros
      }
      __syncthreads();
      PROF_MARK(2)
      // partial sums of Dh for all n outputs: [16 rows (8 real, repeated), K = 128] x [128, 256 outputs of this wave],
      // in four groups of four column tiles: while the MFMAs of one group run, the previous group's results are
      // converted and stored.  One 16-byte store per accumulator tile: the 32 storing lanes of a wavefront cover 512
      // consecutive bytes.  Each 8-byte half carries its own tag in its upper dword, so the only thing relied on
      // beyond the 64-bit units of the other kernels is that an aligned 16-byte lane store is not split below 8 bytes.
      const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc(
          (void*)(((sigma & 1) ? d.ring1 : d.ring0) + (long)R * ntile2 * ntile2 * (kPartBytes / 16)), 0, ntile2 * ntile2 * kPartBytes, kBufFlags);
      const unsigned tag_hi = part_tag(sigma + 1) << 30;
      u32x4 av[4];
#pragma unroll
      for (int kc = 0; kc < 4; ++kc) av[kc] = *(const u32x4*)&zb[lane & 7][kc * 32 + (lane >> 4) * 8];
      f32x4 acc[16];
      // Sixteen column tiles, the k loop inside.  An MFMA of this shape issues every 16 cycles, of which the wavefront's
      // issue slot is taken for 4 (see the forward kernel for the measurements).  What publishes a tile (two conversions,
      // three moves and one store) is cut into single instructions that follow the MFMAs of the tile two behind it:
      // by then its last result has been written (more than the 20 wait states mfma_settle would spend), the
      // instructions cost little there, and only the last two tiles are published behind the last MFMA (with groups of
      // four tiles, as this was first written, a whole group's publishing - a quarter of it - trailed the stream).
      // Nothing is predicated: lanes that hold no result have their store offset parked outside the buffer (pub_off),
      // and the two cache policies are two copies of the code.
      constexpr int kPubSteps = 4, kPubLag = 2;             // a tile is published behind the MFMAs of the tile kPubLag after it
      auto mma_publish = [&](auto local_c) __attribute__((always_inline)) {
        constexpr bool kLocal = decltype(local_c)::value;
        u32x2 val[4];
        auto pub_step = [&](int c, int kk) __attribute__((always_inline)) {
          u32x2& v = val[c & 3];
          if (kk == 0) v[0] = pack_bf16x2(acc[c][0], acc[c][1]);
          else if (kk == 1) v[1] = pack_bf16x2(acc[c][2], acc[c][3]);
          else if (kk == 2) v[1] |= tag_hi;                  // (bit 14 of the fourth value is 0 below 2^33: see the format)
          else __builtin_amdgcn_raw_buffer_store_b64(v, ro, pub_off[c], 0, kLocal ? 0 : 16);   // 16: sc1, agent scope, written through
        };
        operands_settle(av[0], av[1], av[2], av[3]);
#pragma unroll
        for (int c = 0; c < 16; ++c)
#pragma unroll
          for (int kc = 0; kc < 4; ++kc) {
            if (kc == 0) mfma_b_agpr_first(acc[c], av[kc], w[kc][c]);
            else mfma_b_agpr(acc[c], av[kc], w[kc][c]);
            if (c >= kPubLag) {                              // one step of the earlier tile behind each MFMA
              __builtin_amdgcn_sched_barrier(0);
              pub_step(c - kPubLag, kc);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        mfma_settle(acc[12], acc[13], acc[14], acc[15]);
#pragma unroll
        for (int c = 16 - kPubLag; c < 16; ++c)
#pragma unroll
          for (int k = 0; k < kPubSteps; ++k) pub_step(c, k);
      };
      if (local) mma_publish(std::true_type{});
      else mma_publish(std::false_type{});
      PROF_MARK(1)
      if (active) {
#pragma unroll
        for (int q = 0; q < 4; ++q) st_stream(dz_p + q * n, bits[q]);
      }
      dz_p += g_step;
      PROF_MARK(3)
    }
  };
  // (tau is told to be wave-uniform: computed next to per-lane uses it ends up in vector registers)
  constexpr std::true_type yes{};
  constexpr std::false_type no{};
  step(T - 1, in_a, in_b, no, yes);                        // (T >= 2)
  int tau = T - 2;
  for (; tau >= 1; tau = __builtin_amdgcn_readfirstlane(tau) - 2) {
    step(tau, in_b, in_a, yes, yes);
    step(__builtin_amdgcn_readfirstlane(tau - 1), in_a, in_b, yes, yes);
  }
  if (tau == 0) {
    step(0, in_b, in_a, yes, yes);
    step(-1, in_a, in_b, yes, no);
  } else {
    step(-1, in_b, in_a, yes, no);
  }
  PROF_DUMP("bwdp", T)
  if (active) {
    d.Dh[(long)b * n + j] = Dh;
    d.Dc[(long)b * n + j] = Dc;
  }
  if (d.dbpart) {                       // bias gradient: sum this work-group's 8 rows, one slice per row group
    __shared__ float dbred[8][129];
#pragma unroll
    for (int q = 0; q < 4; ++q) dbred[r8][q * 32 + u] = dbsum[q];
    __syncthreads();
    if (tid < 128) {
      const int q = tid >> 5, uu = tid & 31, jj = J * 32 + uu;
      float sum = 0.f;
#pragma unroll
      for (int rr = 0; rr < 8; ++rr) sum += dbred[rr][q * 32 + uu];
      if (jj < n) d.dbpart[(long)R * 4 * n + q * n + jj] = sum;
    }
  }
}

// The same kernel for work-groups of 16 rows (two per thread: rows r8 and r8 + 8 of the group), for batches that the
// 8-row form cannot hold in one launch.  The MFMAs and the publishing stores are the same instructions with all 64 lanes
// doing real work (the 8-row form computes every row twice); a (producer, destination tile) block is 1 KiB -
// [32 outputs][4 row quarters] x 8 bytes -, a consumer's load covers one producer (lane = output lane/2, row half lane%2),
// so a wavefront reads eight loads per step instead of four, and the pointwise part runs twice.
template <int NPW>                                        // producers per wavefront at most: n <= 128 * NPW
__global__ __launch_bounds__(256) void persist_bwdp16_kernel(PBwdArgs a) {
  __shared__ float red[4][16][33];                       // [wavefront][row][output]
  __shared__ __attribute__((aligned(16))) unsigned short zb[16][136];
  constexpr int kBlock = 2 * kPartBytes;                 // one (producer, destination tile)
  const WgCoord wg = wg_coord();
  const PBwdDir d = a.d[wg.dir];       // a copy: fields read through a reference are fetched again in every time step
  const int J = wg.tile, R = a.rt0 + wg.rt, ntile2 = gridDim.x;         // R: row group of 16 rows, counted over the whole batch
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n = a.n, B = a.B, T = a.T;
  unsigned* err = a.sync;
  bool dead = false;

  u32x4 w[4][16];                                        // all 256 accumulation registers
#pragma unroll
  for (int kc = 0; kc < 4; ++kc)
#pragma unroll
    for (int c = 0; c < 16; ++c) w[kc][c] = load_to_agpr(&d.Wb[((((long)J * 4 + wave) * 4 + kc) * 16 + c) * 64 + lane]);
  agpr_loads_done();

  const int r8 = tid >> 5, u = tid & 31;                 // pointwise pairs of this thread: rows r8 and r8 + 8, unit u
  const int b0 = R * 16 + r8, j = J * 32 + u;
  bool active[2];
  float Dh[2], Dc[2];
  float dbsum[4] = {0.f, 0.f, 0.f, 0.f};
  int L[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int b = b0 + 8 * k;
    active[k] = b < B && j < n;
    Dh[k] = 0.f; Dc[k] = 0.f; L[k] = 0;
    if (active[k]) {
      Dh[k] = d.Dh[(long)b * n + j];
      Dc[k] = d.Dc[(long)b * n + j];
      L[k] = clamp_len(a.lens, b, T);
    }
  }
  // What the gate gradients of one frame need.  dy stays as the 16 bits that were loaded: a conversion right behind
  // the load would make the wavefront wait for it - and for every load in front of it - where it is issued.
  struct In { float gi, gf, gg, go, c_new, c_prev; unsigned dy_bits; };
  // The per-frame arrays are read through buffer descriptors that cover exactly one frame: the frame's address is
  // scalar arithmetic, a lane's offset inside the frame never changes, and a lane with nothing to fetch (row past the
  // batch, unit past n, frame past the row's length) has its offset parked outside the frame and gets zeros without
  // touching memory - as does every lane when the frame itself does not exist (zero-sized descriptor).  Nothing is
  // predicated, so every step issues the same six loads; with loads that may or may not have been issued the
  // compiler has to assume the fewest, and made the wavefront wait for the loads of the NEXT frame, just issued and
  // on their way from HBM, where it only needed those of this one.
  constexpr unsigned kParked = 0x7ff00000u;
  const unsigned g_bytes = (unsigned)B * 4u * n * 4u, s_bytes = (unsigned)B * n * 4u, y_bytes = (unsigned)B * d.lddy * 2u;
  // offsets of row r8 inside a frame; row r8 + 8 lies a wave-uniform distance behind it (and exists only if row r8 does)
  const unsigned g_off0 = active[0] ? ((unsigned)b0 * 4u * n + j) * 4u : kParked;
  const unsigned s_off0 = active[0] ? ((unsigned)b0 * n + j) * 4u : kParked;
  const unsigned y_off0 = active[0] ? ((unsigned)b0 * d.lddy + j) * 2u : kParked;
  auto g_off = [&](int k) { return k == 0 ? g_off0 : (active[1] ? g_off0 + 8u * 4u * n * 4u : kParked); };
  auto s_off = [&](int k) { return k == 0 ? s_off0 : (active[1] ? s_off0 + 8u * n * 4u : kParked); };
  auto y_off = [&](int k) { return k == 0 ? y_off0 : (active[1] ? y_off0 + 8u * (unsigned)d.lddy * 2u : kParked); };
  auto frame_of = [&](const void* base, int t, unsigned bytes) {
    const bool ok = t >= 0 && t < T;
    return __builtin_amdgcn_make_buffer_rsrc((void*)((const char*)base + (unsigned long long)(unsigned)(ok ? t : 0) * bytes), 0, ok ? bytes : 0u, kBufFlags);
  };
  auto ld_f = [&](__amdgpu_buffer_rsrc_t r, unsigned voff, unsigned soff) {     // 2: non-temporal
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 2));
  };
  auto fetch_in = [&](int tau, int k) {
    const int t = tau < 0 ? -1 : (d.rev ? T - 1 - tau : tau);
    const bool lane_on = t < L[k];                         // (L is 0 in lanes without a row)
    const unsigned go = lane_on ? g_off(k) : kParked, yo = lane_on ? y_off(k) : kParked;
    In in;
    const __amdgpu_buffer_rsrc_t rg = frame_of(d.gates, t, g_bytes);
    in.gi = ld_f(rg, go, 0u); in.gf = ld_f(rg, go, 4u * n); in.gg = ld_f(rg, go, 8u * n); in.go = ld_f(rg, go, 12u * n);
    const int tp = d.rev ? t + 1 : t - 1;                  // the frame before t in processing order
    const bool inside = t >= 0 && tp >= 0 && tp < T, initial = t >= 0 && !inside && d.c0 != nullptr;
    const __amdgpu_buffer_rsrc_t rp = initial ? __builtin_amdgcn_make_buffer_rsrc((void*)d.c0, 0, s_bytes, kBufFlags)
                                              : frame_of(d.cs, inside ? tp : -1, s_bytes);
    // The cell state entering frame t is the state leaving the frame before it, which is the NEXT backward step's
    // frame: that step takes its c_new from here instead of loading it again (one load per step less).  So the value is
    // also fetched where frame t itself is padding but the frame before it is real (direction +1, t = the row's length).
    in.c_prev = ld_f(rp, (d.rev ? t : t - 1) < L[k] ? s_off(k) : kParked, 0u);
    in.c_new = 0.f;                                        // supplied by the caller
    in.dy_bits = __builtin_amdgcn_raw_buffer_load_b16(frame_of(d.dy, t, y_bytes), yo, 0, 2);
    return in;
  };
  // entries of DZ, which this thread stores: a pointer that moves by one frame per step
  const long row_last = (long)(d.rev ? 0 : T - 1) * B + b0, g_step = (d.rev ? (long)B : -(long)B) * 4 * n;
  unsigned short* dz_p = (unsigned short*)d.DZ + row_last * 4 * n + j;
  In in_a[2], in_b[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    in_a[k] = fetch_in(T - 1, k);
    in_b[k] = in_a[k];
    const int t0 = d.rev ? 0 : T - 1;                      // the first frame's own cell state: the only one loaded as such
    in_a[k].c_new = ld_f(frame_of(d.cs, t0, s_bytes), t0 < L[k] ? s_off(k) : kParked, 0u);
  }

  // consumer side: a load covers one producer's block; lane reads output lane/2, rows 8 * (lane%2) .. + 7
  const int ccol = lane >> 1, chalf = lane & 1;
  const int nitv = (ntile2 + 3) / 4, rot = J % nitv;
  const long ring_tile = ((long)R * ntile2 + J) * ntile2 * (kBlock / 16);         // uint4 index of [R][J][0]
  // producer side: lane holds rows 4*(lane/16) .. +3 of output column lane%16 of each accumulator tile
  const int pq = lane >> 4, pcol = lane & 15;
  // (the verdict comes out of shared memory; the compiler has to be told that it is the same in every lane, or the
  // two copies of the publishing code below become one divergent region)
  const bool local = __builtin_amdgcn_readfirstlane((int)(a.xcc != nullptr &&
                     group_is_xcd_local(a.xcc, (wg.dir * (int)gridDim.y + wg.rt) * ntile2, ntile2, J, a.spin_limit))) != 0;
  // byte offset, from row group R's part of the ring, of what this lane stores for accumulator tile c: destination tile
  // wave*8 + c/2 (one past the last falls outside the buffer), this producer's block, output column, row quarter
  unsigned pub_off[16];
#pragma unroll
  for (int c = 0; c < 16; ++c) {
    const int Jd = wave * 8 + (c >> 1);
    pub_off[c] = (unsigned)(((Jd * ntile2 + J) * 32 + (c & 1) * 16 + pcol) * 4 + pq) * 8u;
  }

  PROF_DECL
  // One time step.  `in` holds the inputs of this step's frame and `in_next` receives those of the next; the loop
  // below calls it with the two in alternating roles, because a copy at the end of a step would have to wait for
  // the loads (and, counted with them, the step's stores) at that point.
  // `ring_c`: the step reads partial sums (every step but the first); `pointwise_c`: it has a frame (every step but the
  // last, which only collects the Dh that leaves the layer).  Constants of the call, so that the loop below is free
  // of the two exceptions: with them inside, the compiler's wait counts in the loop allowed for paths it never takes.
  auto step = [&](const int tau, const In (&in)[2], In (&in_next)[2], auto ring_c, auto pointwise_c) __attribute__((always_inline)) {
    PROF_MARK(4)
    // (told to be wave-uniform: computed next to per-lane uses of tau it ends up in vector registers, and a buffer
    // descriptor derived from it is then applied lane by lane in a loop)
    const int sigma = __builtin_amdgcn_readfirstlane(T - 1 - tau);
    const int t = d.rev ? T - 1 - tau : tau;
    const int t_next = d.rev ? t - 1 : t + 1;
    constexpr bool pointwise = decltype(pointwise_c)::value;
    bool valid[2];
#pragma unroll
    for (int k = 0; k < 2; ++k) valid[k] = pointwise && active[k] && t < L[k];

    // The gate gradients of a valid frame, dh = dy + Dh (recurrent_dev.h has the plain form):
    //   dc = Dc + dh go (1 - tanh(c)^2), Dc' = dc gf, dz = (dc gg gi (1-gi), dc c_prev gf (1-gf), dc gi (1-gg^2), dh tanh(c) go (1-go)).
    // Everything that does not involve dh or Dc is computed while the ring loads are in flight.
    float f_c[2], f_i[2], f_f[2], f_g[2], f_o[2];
    auto factors = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        f_c[k] = 0.f; f_i[k] = 0.f; f_f[k] = 0.f; f_g[k] = 0.f; f_o[k] = 0.f;
        if (valid[k]) {
          const float tc = tanhf_(in[k].c_new);
          f_c[k] = in[k].go * (1.f - tc * tc);
          f_i[k] = in[k].gg * in[k].gi * (1.f - in[k].gi);
          f_f[k] = in[k].c_prev * in[k].gf * (1.f - in[k].gf);
          f_g[k] = in[k].gi * (1.f - in[k].gg * in[k].gg);
          f_o[k] = tc * in[k].go * (1.f - in[k].go);
        }
      }
    };
    auto fetch_next = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        in_next[k] = fetch_in(tau - 1, k);
        in_next[k].c_new = in[k].c_prev;
      }
    };
    if constexpr (decltype(ring_c)::value) {
      RingReader rd;
      rd.rs = __builtin_amdgcn_make_buffer_rsrc((void*)((((sigma - 1) & 1) ? d.ring1 : d.ring0) + ring_tile), 0, ntile2 * kBlock,
                                                kBufFlags);
      // load `it` of this wavefront covers producer wave + 4 * it (1 KiB)
      rd.voff = (unsigned)(wave * kBlock + lane * 16);
      rd.it_bytes = 4u * kBlock;
      rd.lim = ntile2 - wave; rd.lim_step = 4;
      rd.tag = part_tag(sigma) << 14; rd.err = err; rd.limit = a.spin_limit;
      rd.nitv = nitv; rd.rot = rot;
      constexpr int NLD = NPW;                              // loads per wavefront
      float ps[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      {
        // The sums need no masking but the tag bit's: the shifts drop the other halves.  With one wavefront per SIMD what
        // bounds this phase is its instruction stream, and a verdict per load (compare, branch, or worse a ballot
        // handed to scalar registers) costs as much as the additions themselves.  So the loads behind the poll are
        // taken together: their values are added into sums of their own without looking, the tag differences are ORed
        // per lane, and one compare and branch decides whether those sums count.  If not, the loads are fetched
        // again, all at once, by fix_up_batch.
        auto add = [&](float (&acc)[8], const u32x4& v) __attribute__((always_inline)) {
          acc[0] += __uint_as_float(v[0] << 16); acc[1] += __uint_as_float(v[0] & 0xffff0000u);
          acc[2] += __uint_as_float(v[1] << 16); acc[3] += __uint_as_float(v[1] & (0xffff0000u & ~kLLFwdTagBit));
          acc[4] += __uint_as_float(v[2] << 16); acc[5] += __uint_as_float(v[2] & 0xffff0000u);
          acc[6] += __uint_as_float(v[3] << 16); acc[7] += __uint_as_float(v[3] & (0xffff0000u & ~kLLFwdTagBit));
        };
        static_assert(NLD >= 2, "the poll is two loads");
        u32x4 x[NLD];
        const unsigned tagw = rd.tag << 16;
        // The poll is the first two loads, repeated (bounded) until their tags have turned and then kept; the others
        // are issued behind it (see the forward kernel).
        for (unsigned poll = 0;; ++poll) {
          x[0] = rd.load_it(rd.it_of(0));
          x[1] = rd.load_it(rd.it_of(1));
          if (dead) break;
          const unsigned stale = rd.tag_diff(x[0], rd.it_of(0), tagw) | rd.tag_diff(x[1], rd.it_of(1), tagw);
          if (__builtin_amdgcn_ballot_w64(stale > 0xffffu) == 0ull) break;
          if (poll >= rd.limit || ((poll & 63u) == 63u && ld_relaxed(err) != 0u)) {
            st_relaxed(err, 1u);
            dead = true;
            break;
          }
          PROF_POLLS(1)
        }
        PROF_MARK(5)
        // Nothing is outstanding here (the poll has just been waited for, and loads complete in order).  Said with an
        // instruction the compiler takes note of: otherwise it makes the pointwise part below wait for this frame's
        // inputs, asked for a step ago, with a count that also waits for the next frame's, just asked for.
        __builtin_amdgcn_s_waitcnt(0x0f70);                // vmcnt(0)
#pragma unroll
        for (int i = 2; i < NLD; ++i) x[i] = rd.load_it(rd.it_of(i));
        __builtin_amdgcn_sched_barrier(0);
        // while those loads are on their way: the polled loads' values, and the part of the gate gradients that
        // does not need Dh
        add(ps, x[0]);
        add(ps, x[1]);
        factors();
        __builtin_amdgcn_sched_barrier(0);
        unsigned long long redo = 0ull;
        constexpr int kGroup = (NLD - 2) / 2;              // the other loads: two groups
#pragma unroll
        for (int g = 0; g < 2; ++g) {
          const int i0 = 2 + g * kGroup, i1 = g == 0 ? 2 + kGroup : NLD;
          float pg[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          unsigned bad = 0u;
#pragma unroll
          for (int i = i0; i < i1; ++i) {
            __builtin_amdgcn_sched_barrier(0);             // each load is waited for and consumed in turn
            bad |= rd.tag_diff(x[i], rd.it_of(i), tagw);
            add(pg, x[i]);
          }
          __builtin_amdgcn_sched_barrier(0);
          if (__builtin_expect(__builtin_amdgcn_ballot_w64(bad > 0xffffu) == 0ull, 1)) {
#pragma unroll
            for (int v = 0; v < 8; ++v) ps[v] += pg[v];
          } else {
            redo |= ((1ull << i1) - 1ull) & ~((1ull << i0) - 1ull);
          }
        }
        PROF_REDO(__popcll(redo))
        if (redo) {
          rd.fix_up_batch<NLD>(redo, dead, [&](int, const u32x4& v) __attribute__((always_inline)) { add(ps, v); });
          // (nothing of that is outstanding any more - said with an instruction the compiler takes note of: it cannot tell
          // from the loop's exits, and would make whatever reuses those registers below wait for every load in flight)
          __builtin_amdgcn_s_waitcnt(0x0f70);              // vmcnt(0)
        }
        // The next frame's inputs, from HBM.  Loads complete in the order of issue: asked for in front of the groups
        // above (where their latency would be covered best) they held up every ring load behind them - a tenth of the step.
        fetch_next();
      }
      PROF_MARK(0)
#pragma unroll
      for (int v = 0; v < 8; ++v) red[wave][8 * chalf + v][ccol] = ps[v];
      __syncthreads();
#pragma unroll
      for (int k = 0; k < 2; ++k)
        if (active[k] && t_next < L[k]) {
          const int rr = r8 + 8 * k;
          Dh[k] = (red[0][rr][u] + red[1][rr][u] + red[2][rr][u] + red[3][rr][u]) * (1.f / kPartScale);   // the partial sums travel scaled
        }
    } else {
      factors();
      fetch_next();
    }
    if (pointwise) {
      unsigned short bits[2][4];
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        float dz[4] = {0.f, 0.f, 0.f, 0.f};
        if (valid[k]) {
          const float dh = bf_bits2f((unsigned short)in[k].dy_bits) + Dh[k], dc = Dc[k] + dh * f_c[k];
          Dc[k] = dc * in[k].gf;
          dz[0] = dc * f_i[k]; dz[1] = dc * f_f[k]; dz[2] = dc * f_g[k]; dz[3] = dh * f_o[k];
        }
        const unsigned b01 = pack_bf16x2(dz[0], dz[1]), b23 = pack_bf16x2(dz[2], dz[3]);
        bits[k][0] = (unsigned short)b01; bits[k][1] = (unsigned short)(b01 >> 16);
        bits[k][2] = (unsigned short)b23; bits[k][3] = (unsigned short)(b23 >> 16);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          dbsum[q] += dz[q];
          zb[r8 + 8 * k][q * 32 + u] = bits[k][q];         // inactive threads contribute zeros
        }
      }
      __syncthreads();
      PROF_MARK(2)
      // partial sums of Dh for all n outputs: [16 rows, K = 128] x [128, 256 outputs of this wave],
      // in four groups of four column tiles: while the MFMAs of one group run, the previous group's results are
      // converted and stored.  One 16-byte store per accumulator tile: the 32 storing lanes of a wavefront cover 512
      // consecutive bytes.  Each 8-byte half carries its own tag in its upper dword, so the only thing relied on
      // beyond the 64-bit units of the other kernels is that an aligned 16-byte lane store is not split below 8 bytes.
      const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc(
          (void*)(((sigma & 1) ? d.ring1 : d.ring0) + (long)R * ntile2 * ntile2 * (kBlock / 16)), 0, ntile2 * ntile2 * kBlock, kBufFlags);
      const unsigned tag_hi = part_tag(sigma + 1) << 30;
      u32x4 av[4];
#pragma unroll
      for (int kc = 0; kc < 4; ++kc) av[kc] = *(const u32x4*)&zb[lane & 15][kc * 32 + (lane >> 4) * 8];
      f32x4 acc[16];
      // Sixteen column tiles, the k loop inside.  An MFMA of this shape issues every 16 cycles, of which the wavefront's
      // issue slot is taken for 4 (see the forward kernel for the measurements).  What publishes a tile (two conversions,
      // three moves and one store) is cut into single instructions that follow the MFMAs of the tile two behind it:
      // by then its last result has been written (more than the 20 wait states mfma_settle would spend), the
      // instructions cost little there, and only the last two tiles are published behind the last MFMA (with groups of
      // four tiles, as this was first written, a whole group's publishing - a quarter of it - trailed the stream).
      // Nothing is predicated: lanes that hold no result have their store offset parked outside the buffer (pub_off),
      // and the two cache policies are two copies of the code.
      constexpr int kPubSteps = 4, kPubLag = 2;             // a tile is published behind the MFMAs of the tile kPubLag after it
      auto mma_publish = [&](auto local_c) __attribute__((always_inline)) {
        constexpr bool kLocal = decltype(local_c)::value;
        u32x2 val[4];
        auto pub_step = [&](int c, int kk) __attribute__((always_inline)) {
          u32x2& v = val[c & 3];
          if (kk == 0) v[0] = pack_bf16x2(acc[c][0], acc[c][1]);
          else if (kk == 1) v[1] = pack_bf16x2(acc[c][2], acc[c][3]);
          else if (kk == 2) v[1] |= tag_hi;                  // (bit 14 of the fourth value is 0 below 2^33: see the format)
          else __builtin_amdgcn_raw_buffer_store_b64(v, ro, pub_off[c], 0, kLocal ? 0 : 16);   // 16: sc1, agent scope, written through
        };
        operands_settle(av[0], av[1], av[2], av[3]);
#pragma unroll
        for (int c = 0; c < 16; ++c)
#pragma unroll
          for (int kc = 0; kc < 4; ++kc) {
            if (kc == 0) mfma_b_agpr_first(acc[c], av[kc], w[kc][c]);
            else mfma_b_agpr(acc[c], av[kc], w[kc][c]);
            if (c >= kPubLag) {                              // one step of the earlier tile behind each MFMA
              __builtin_amdgcn_sched_barrier(0);
              pub_step(c - kPubLag, kc);
              __builtin_amdgcn_sched_barrier(0);
            }
          }
        mfma_settle(acc[12], acc[13], acc[14], acc[15]);
#pragma unroll
        for (int c = 16 - kPubLag; c < 16; ++c)
#pragma unroll
          for (int k = 0; k < kPubSteps; ++k) pub_step(c, k);
      };
      if (local) mma_publish(std::true_type{});
      else mma_publish(std::false_type{});
      PROF_MARK(1)
#pragma unroll
      for (int k = 0; k < 2; ++k)
        if (active[k]) {
#pragma unroll
          for (int q = 0; q < 4; ++q) st_stream(dz_p + (long)k * 8 * 4 * n + q * n, bits[k][q]);
        }
      dz_p += g_step;
      PROF_MARK(3)
    }
  };
  // (tau is told to be wave-uniform: computed next to per-lane uses it ends up in vector registers)
  constexpr std::true_type yes{};
  constexpr std::false_type no{};
  step(T - 1, in_a, in_b, no, yes);                        // (T >= 2)
  int tau = T - 2;
  for (; tau >= 1; tau = __builtin_amdgcn_readfirstlane(tau) - 2) {
    step(tau, in_b, in_a, yes, yes);
    step(__builtin_amdgcn_readfirstlane(tau - 1), in_a, in_b, yes, yes);
  }
  if (tau == 0) {
    step(0, in_b, in_a, yes, yes);
    step(-1, in_a, in_b, yes, no);
  } else {
    step(-1, in_b, in_a, yes, no);
  }
  PROF_DUMP("bwdp16", T)
#pragma unroll
  for (int k = 0; k < 2; ++k)
    if (active[k]) {
      d.Dh[(long)(b0 + 8 * k) * n + j] = Dh[k];
      d.Dc[(long)(b0 + 8 * k) * n + j] = Dc[k];
    }
  if (d.dbpart) {                       // bias gradient: sum this work-group's 16 rows into the first of its two slices (the other stays zero)
    __shared__ float dbred[8][129];
#pragma unroll
    for (int q = 0; q < 4; ++q) dbred[r8][q * 32 + u] = dbsum[q];
    __syncthreads();
    if (tid < 128) {
      const int q = tid >> 5, uu = tid & 31, jj = J * 32 + uu;
      float sum = 0.f;
#pragma unroll
      for (int rr = 0; rr < 8; ++rr) sum += dbred[rr][q * 32 + uu];
      if (jj < n) d.dbpart[(long)2 * R * 4 * n + q * n + jj] = sum;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// forward, float storage.  The float MFMA (16x16x4) runs at a sixteenth of the bfloat16 rate: 7.1 us per step for 64 rows
// x 2 directions of n = 1000 on the whole device, so here the matrix cores bound the step, and the exchange has to stay
// out of their way.  Two things compete with them.  (1) Every work-group reads the whole h of its rows in float, from
// beyond L2 (an exchange group spans several XCDs), so rows per work-group are traded against copies of W_h: a work-group
// owns 16 units - 64 gate columns, four MFMA column tiles - for a slab of 32 rows: 63 x 2 slabs x 2 directions = 252
// work-groups for config 2, W_h held twice on the device (256 registers per lane: the per-step kernel's packed slices of
// two 8-unit tiles), 128 KiB of ring read per work-group and step (with 8 units x 64 rows, 256 KiB, the step took 13.8 us
// against 11 for its products alone).  (2) The round trip of the exchange - reduce, cell, publish, and the consumers' loads,
// about 2.5 us - which nothing overlaps if all rows move in lock step (12.0 us per step).  The two row tiles of a slab
// are different batch rows, i.e. independent recurrences: they are walked HALF A STEP APART, one's products running
// while the other's h travels.
// The K axis is split over the four wavefronts (chunks of 16 k, wavefront w takes chunks w, w + 4, ...), their accumulators
// meet in LDS, a thread updates one cell per row tile, and two neighbouring units are published as ONE 8-byte unit of the
// ring: two float h values, the tag in bit 30 of the second (|h| < 1 leaves the top exponent bit 0, as bit 14 of a
// bfloat16 value in the other kernels).  The ring is the per-step kernel's fragment-ordered h buffer [row tile][chunk][lane]
// x 16 bytes, a lane's 16 bytes being two such units, so the reader of the other kernels applies unchanged.  An initial
// hidden state never enters the ring (it is not bounded by 1): rows publish zeros until their first frame is done, and
// launch_h0_term has added h0 W_h to that frame's pre-activations.
template <int NCH>                                         // chunks per wavefront at most: n <= 64 * NCH
__global__ __launch_bounds__(256) void persist_fwd_f32_kernel(PFwdArgs a) {
  __shared__ float red[4][16][65];
  const int tile = blockIdx.x, dir = blockIdx.z;           // tile: 16 units
  const PFwdDir d = a.d[dir];          // a copy: fields read through a reference are fetched again in every time step
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nkc = a.nkc, n = a.n, B = a.B, T = a.T;
  const int rt_base = a.rt0 + 2 * (int)blockIdx.y;         // first 16-row tile of this work-group's slab
  const int nrt_here = min(2, (B + 15) / 16 - rt_base);
  const int ntile8 = (n + 7) / 8;
  unsigned* err = a.sync;
  bool dead = false;

  // W_h slice: chunk kc = wave + 4 it; column tile ct = tile of 8 units (ct >> 1), its gates i,f (ct & 1 = 0) or g,o
  // (the per-step kernel's packing)
  // It fills the 256 accumulation registers of every lane and the MFMAs read it there (inline assembly, as in the bfloat16
  // kernels).  A chunk past the end of K or a column tile past n takes the last valid one's weights instead of zeros: the h
  // values of such a chunk arrive as zeros (the ring's descriptor ends before them), and such columns are never stored.
  u32x4 w[NCH][4];
#pragma unroll
  for (int it = 0; it < NCH; ++it) {
    const int kc = min(wave + 4 * it, nkc - 1);
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) {
      const int tile8 = min(tile * 2 + (ct >> 1), ntile8 - 1);
      w[it][ct] = load_to_agpr(&d.Wf[((long)(tile8 * 2 + (ct & 1)) * nkc + kc) * 64 + lane]);
    }
  }
  agpr_loads_done();

  // pointwise: row r16 of each row tile, unit u of the tile's 16
  const int r16 = tid >> 4, u = tid & 15;
  const int j = tile * 16 + u;
  float c[2] = {0.f, 0.f}, h[2] = {0.f, 0.f};
  int L[2] = {0, 0};
  bool active[2];
  // A row publishes zeros until its first frame has been processed: its initial hidden state (not bounded by 1, so not
  // fit for the ring) reaches that frame through the pre-activations instead (launch_h0_term).
  bool started[2] = {false, false};
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int b = (rt_base + k) * 16 + r16;
    active[k] = k < nrt_here && b < B && j < n;
    if (active[k]) {
      c[k] = d.cstate[(long)b * n + j];
      h[k] = d.hstate[(long)b * n + j];
      L[k] = clamp_len(a.lens, b, T);
    }
  }
  // The even unit of a pair publishes both: chunk j / 16, lane group (j % 16) / 4, half ((j % 4) / 2) of that lane's 16 bytes
  constexpr unsigned kParked = 0x7ff00000u;
  const bool publishes = (u & 1) == 0 && j < n;            // (n is a multiple of 8: the odd partner exists as well)
  const unsigned pub_in_tile = (unsigned)((((long)(j >> 4) * 64 + ((j & 15) >> 2) * 16 + r16) * 2 + ((j >> 1) & 1)) * 8);
  const unsigned ring_bytes = (unsigned)((B + 15) / 16) * nkc * 1024u;
  const long fg = (long)B * 4 * n, fy = (long)B * d.ldy, fs = (long)B * n;     // elements per frame
  // columns of this thread's cell among the work-group's 64: 32 per tile of 8 units, then gate q, unit
  const int col0 = (u >> 3) * 32 + (u & 7);
  PROF_DECL
  // The first half of a half step's ring loads goes out before the reduction and the cell update of the half step
  // before it (their values were published half a step earlier) and is there when the products begin; the second half
  // goes out then and arrives behind the first half's products.  (All of them early does not fit the register file.)
#ifndef LSTM_FWD_F32_EARLY
#define LSTM_FWD_F32_EARLY (NCH / 2)
#endif
  constexpr int kEarly = LSTM_FWD_F32_EARLY;
  u32x4 x[NCH];
  auto reader = [&](int tau, int k) __attribute__((always_inline)) {
    return make_reader(((tau & 1) ? d.ring1 : d.ring0) + (long)(rt_base + k) * nkc * 64, nkc, (n + 3) / 4, wave, lane,
                       ll_fwd_tag((unsigned)tau) << 14, err, a.spin_limit, 0);
  };
  auto issue_loads = [&](int tau, int k) __attribute__((always_inline)) {
    const RingReader rn = reader(tau, k);
#pragma unroll
    for (int it = 0; it < kEarly; ++it) x[it] = rn.load_it(it);
  };
  if (T > 0) issue_loads(0, 0);

  for (int tau = 0; tau < T; ++tau) {
    const int t = d.rev ? T - 1 - tau : tau;
    const unsigned tag = ll_fwd_tag((unsigned)tau) << 14, tagw = tag << 16;
#pragma unroll
    for (int k = 0; k < 2; ++k) {                          // the slab's two row tiles, half a step apart
      if (k >= nrt_here) break;                            // (the same in every work-group of the launch)
      PROF_MARK(4)
      const int b = (rt_base + k) * 16 + r16;
      const bool valid = active[k] && t < L[k];
      // this frame's x W_x + b: in flight while the products run
      float zx[4];
#pragma unroll
      for (int q = 0; q < 4; ++q) zx[q] = valid ? d.gates[t * fg + (long)b * 4 * n + q * n + j] : 0.f;
      f32x4 acc[4];
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) acc[ct] = (f32x4){0.f, 0.f, 0.f, 0.f};
      operands_settle(acc[0], acc[1], acc[2], acc[3]);     // (the MFMAs are assembly text: wait states by hand)
      const RingReader rd = reader(tau, k);
      auto use = [&](int it, const u32x4& x) __attribute__((always_inline)) {
        u32x4 av = {x[0], x[1] & ~kLLFwdTagBit, x[2], x[3] & ~kLLFwdTagBit};
        asm volatile("s_nop 4" : "+v"(av));                // masked just now by the vector ALU
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int ct = 0; ct < 4; ++ct) mfma4_b_agpr(acc[ct], __uint_as_float(av[e]), w[it][ct][e]);
      };
#pragma unroll
      for (int it = kEarly; it < NCH; ++it) x[it] = rd.load_it(it);
      // a load with a stale tag is fetched again (bounded) - rare, since the values were published half a step ago
      unsigned long long redo = 0ull;
#pragma unroll
      for (int it = 0; it < NCH; ++it) {
        wait_loads_but(NCH - 1 - it, x[it]);               // (the first half went out before the last half step's stores)
        if (__builtin_amdgcn_ballot_w64(rd.tag_diff(x[it], it, tagw) != 0u) == 0ull) use(it, x[it]);
        else { redo |= 1ull << it; PROF_REDO(1) }
      }
      if (redo) rd.template fix_up_batch<NCH>(redo, dead, use);
      if (k + 1 < nrt_here) issue_loads(tau, k + 1);
      else if (tau + 1 < T) issue_loads(tau + 1, 0);
      mfma_settle(acc[0], acc[1], acc[2], acc[3]);         // (behind the loads: their issue covers part of the wait)
      PROF_MARK(0)
      // accumulator rows 4 * (lane / 16) + v of the row tile, column lane % 16 of the column tile
#pragma unroll
      for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][4 * (lane >> 4) + v][ct * 16 + (lane & 15)] = acc[ct][v];
      PROF_MARK(1)
      __syncthreads();
      const float hprev = h[k];
      CellOut o = {};
      if (valid) {
        float zh[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int col = col0 + q * 8;
          zh[q] = red[0][r16][col] + red[1][r16][col] + red[2][r16][col] + red[3][r16][col];
        }
        o = lstm_cell(zh, zx, c[k]);
        c[k] = o.c; h[k] = o.h;
      }
      started[k] = started[k] || valid;
      __syncthreads();                // (the accumulators of the other row tile may be written)
      PROF_MARK(2)
      {                               // the recurrence's critical store goes out first (16: agent scope, written through)
        const unsigned h_pub = started[k] ? __float_as_uint(h[k]) : 0u;
        const unsigned h_odd = (unsigned)__builtin_amdgcn_mov_dpp((int)h_pub, 0xB1, 0xf, 0xf, false);   // quad_perm [1,0,3,2]: the neighbour's h
        const u32x2 unit = {h_pub, h_odd | (ll_fwd_tag((unsigned)tau + 1u) << 30)};
        const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc((void*)((tau & 1) ? d.ring0 : d.ring1), 0, ring_bytes, kBufFlags);
        __builtin_amdgcn_raw_buffer_store_b64(unit, ro, publishes ? (unsigned)(rt_base + k) * (unsigned)nkc * 1024u + pub_in_tile : kParked, 0, 16);
      }
      if (active[k]) {                // layer outputs and what the backward pass needs
        ((float*)d.y)[t * fy + (long)b * d.ldy + j] = valid ? h[k] : 0.f;
        if (d.cs) d.cs[t * fs + (long)b * n + j] = c[k];
        if (d.hprev) ((float*)d.hprev)[t * fs + (long)b * n + j] = hprev;
        if (valid && a.write_gates) {
          float* gp = d.gates + t * fg + (long)b * 4 * n + j;
          gp[0] = o.gi; gp[n] = o.gf; gp[2 * n] = o.gg; gp[3 * n] = o.go;
        }
      }
      PROF_MARK(3)
    }
  }
  PROF_DUMP("fwdf32", T)
#pragma unroll
  for (int k = 0; k < 2; ++k)
    if (active[k]) {
      const int b = (rt_base + k) * 16 + r16;
      d.cstate[(long)b * n + j] = c[k];
      d.hstate[(long)b * n + j] = h[k];
    }
}

// ------------------------------------------------------------------------------------------------
// backward, float storage: partial sums of Dh, as in the bfloat16 kernels, in the decomposition of the float forward
// kernel (16 units x a slab of 32 rows per work-group, the slab's two row tiles half a step apart).  A work-group
// multiplies ITS dz (16 rows x 64 gate columns, through LDS, never leaving the compute unit) by the matching 64 rows of W_h^T
// for ALL n outputs - 256 registers per lane hold that slice, 16 column tiles x 16 k-steps per wavefront - and publishes,
// per destination tile of 16 units, the accumulator tile as it stands: a lane's four floats (rows 4g .. 4g+3 of one output)
// are two 8-byte units, the tag bit 30 of each unit's second float.  Partial sums are not bounded by 1, so they travel scaled
// by 2^-32 (the packed W_h^T carries the factor; the consumer multiplies its sum by 2^32): bit 30 is then 0 for every partial
// sum below 2^33 in magnitude, and no other bit of a value above 2^-94 changes.  A consumer adds the blocks of its tile from
// all producers (1 KiB each, one 16-byte load per lane: the producer's accumulator layout), wavefront w taking producers
// w, w + 4, ..., and the four sums meet in LDS.
// Ring per direction and slot: [row tile][destination tile][producer tile] x 1 KiB.  K axis of the product: gate column
// kappa = 16 kg + s of the work-group's 64 (gate kappa / 16, unit kappa % 16) is k-step s of lane group kg, so that a lane
// reads its sixteen A values from sixteen consecutive floats of a dz row in LDS.
template <int NCT>                                         // column tiles per wavefront at most: n <= 64 * NCT
__global__ __launch_bounds__(256) void persist_bwd_f32_kernel(PBwdArgs a) {
  __shared__ float red[4][16][17];                         // [wavefront][row][output]
  __shared__ __attribute__((aligned(16))) float zb[16][68];// dz of the row tile in hand: [row][gate column kappa]
  const int J = blockIdx.x, dir = blockIdx.z;              // J: tile of 16 units
  const PBwdDir d = a.d[dir];          // a copy: fields read through a reference are fetched again in every time step
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = a.n, B = a.B, T = a.T;
  const int ntile = (n + 15) / 16;
  const int rt_base = a.rt0 + 2 * (int)blockIdx.y;         // first 16-row tile of this work-group's slab
  const int nrt_here = min(2, (B + 15) / 16 - rt_base);
  unsigned* err = a.sync;
  bool dead = false;

  // W_h^T slice: column tile wave + 4 ci of the outputs, k-step s (launch_pack_wh_bwd_f32p)
  // It fills the 256 accumulation registers of every lane and stays there: the MFMAs read it from them (inline assembly, as in
  // the bfloat16 kernels; left to the compiler the slice is spread over both register files and copied back before every use, with
  // the architectural registers filled to the last one).
  u32x4 w[NCT][4];
#pragma unroll
  for (int ci = 0; ci < NCT; ++ci)
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) w[ci][s4] = load_to_agpr((const uint4*)d.Wb + ((((long)J * 4 + wave) * NCT + ci) * 4 + s4) * 64 + lane);
  agpr_loads_done();

  // pointwise: row r16 of each row tile, unit u of the tile's 16
  const int r16 = tid >> 4, u = tid & 15;
  const int j = J * 16 + u;
  float Dh[2] = {0.f, 0.f}, Dc[2] = {0.f, 0.f};
  float dbsum[4] = {0.f, 0.f, 0.f, 0.f};                    // bias gradient of this thread's unit over its two rows and all frames
  int L[2] = {0, 0};
  bool active[2];
#pragma unroll
  for (int k = 0; k < 2; ++k) {
    const int b = (rt_base + k) * 16 + r16;
    active[k] = k < nrt_here && b < B && j < n;
    if (active[k]) {
      Dh[k] = d.Dh[(long)b * n + j];
      Dc[k] = d.Dc[(long)b * n + j];
      L[k] = clamp_len(a.lens, b, T);
    }
  }
  const long fg = (long)B * 4 * n, fy = (long)B * d.lddy, fs = (long)B * n;    // elements per frame
  const unsigned ring_bytes = (unsigned)((B + 15) / 16) * (unsigned)ntile * (unsigned)ntile * 1024u;
  PROF_DECL
  // The reader of the partial sums that step sigma consumes for row tile k.  In a slab of two row tiles they are collected
  // DURING the products of the half step before (the other row tile's): what they fetch was published half a step
  // earlier, the loads run kWin ahead of the additions, one load and one addition behind each column tile's MFMAs, and
  // the matrix cores do not wait for the exchange.  `ps_c` / `redo_c` carry the sums (or, if a tag was stale, the order to fetch
  // everything again) into the next half step.
#ifndef LSTM_BWD_F32_WIN
#define LSTM_BWD_F32_WIN 6
#endif
  constexpr int kWin = LSTM_BWD_F32_WIN;
  static_assert(kWin >= 1 && kWin <= 16 && kWin <= NCT, "wait_loads_but covers up to 15 younger loads");
  u32x4 x[NCT];
  float ps_c[4] = {0.f, 0.f, 0.f, 0.f};
  unsigned long long redo_c = 0ull;
  bool have_c = false;
  auto reader = [&](int sigma, int k) __attribute__((always_inline)) {
    RingReader rd;
    const long tile_base = (((long)(rt_base + k) * ntile + J) * ntile) * 64;                   // uint4 index of [row tile][J][0]
    rd.rs = __builtin_amdgcn_make_buffer_rsrc((void*)((((sigma - 1) & 1) ? d.ring1 : d.ring0) + tile_base), 0, ntile * 1024, kBufFlags);
    rd.voff = (unsigned)(wave * 1024 + lane * 16);       // load `it` of this wavefront covers producer wave + 4 it
    rd.it_bytes = 4096u;
    rd.lim = ntile - wave; rd.lim_step = 4;
    rd.tag = part_tag(sigma) << 14; rd.err = err; rd.limit = a.spin_limit;
    rd.nitv = (ntile + 3) / 4; rd.rot = 0;
    return rd;
  };
  auto add_to = [](float (&ps)[4], const u32x4& v) __attribute__((always_inline)) {
    ps[0] += __uint_as_float(v[0]); ps[1] += __uint_as_float(v[1] & ~kLLFwdTagBit);
    ps[2] += __uint_as_float(v[2]); ps[3] += __uint_as_float(v[3] & ~kLLFwdTagBit);
  };

  // Steps sigma = 0 .. T-1 work on frames (the last frame in processing order first); step T only collects the Dh that
  // leaves the layer.
  for (int sigma = 0; sigma <= T; ++sigma) {
    const int tau = T - 1 - sigma;                         // position in processing order; -1 in the collecting step
    const int t = d.rev ? T - 1 - tau : tau;               // this step's frame (outside [0, T) in the collecting step)
    const int t_next = d.rev ? t - 1 : t + 1;              // the frame of the step before: where the partial sums come from
    const bool pointwise = sigma < T;
#pragma unroll
    for (int k = 0; k < 2; ++k) {                          // the slab's two row tiles, half a step apart
      if (k >= nrt_here) break;                            // (the same in every work-group of the launch)
      PROF_MARK(4)
      const int b = (rt_base + k) * 16 + r16;
      const bool valid = pointwise && active[k] && t < L[k];
      // what the gate gradients of the frame need: in flight while the partial sums are collected
      float gi = 0.f, gf = 0.f, gg = 0.f, go = 0.f, c_new = 0.f, c_prev = 0.f, dy = 0.f;
      if (valid) {
        const float* gp = d.gates + t * fg + (long)b * 4 * n + j;
        gi = gp[0]; gf = gp[n]; gg = gp[2 * n]; go = gp[3 * n];
        c_new = d.cs[t * fs + (long)b * n + j];
        const int tp = d.rev ? t + 1 : t - 1;              // the frame before t in processing order
        c_prev = (tp >= 0 && tp < T) ? d.cs[tp * fs + (long)b * n + j] : (d.c0 ? d.c0[(long)b * n + j] : 0.f);
        dy = ((const float*)d.dy)[t * fy + (long)b * d.lddy + j];
      }
      if (sigma > 0) {                                     // the partial sums of Dh that the step before published
        const RingReader rd = reader(sigma, k);
        const unsigned tagw = rd.tag << 16;
        float ps[4] = {ps_c[0], ps_c[1], ps_c[2], ps_c[3]};
        unsigned long long redo = redo_c;
        auto add = [&](int, const u32x4& v) __attribute__((always_inline)) { add_to(ps, v); };
        if (!have_c) {
          // nothing was collected ahead: a slab of one row tile has no other half step to hide behind (what it consumes
          // is published by the half step before it), and the collecting step follows no products
#pragma unroll
          for (int v = 0; v < 4; ++v) ps[v] = 0.f;
          redo = 0ull;
#pragma unroll
          for (int it = 0; it < NCT; ++it) x[it] = rd.load_it(it);
#pragma unroll
          for (int it = 0; it < NCT; ++it) {
            if (__builtin_amdgcn_ballot_w64(rd.tag_diff(x[it], it, tagw) != 0u) == 0ull) add(it, x[it]);
            else { redo |= 1ull << it; PROF_REDO(1) }
          }
        }
        if (redo) rd.template fix_up_batch<NCT>(redo, dead, add);
        // a lane's sums: rows 4 (lane / 16) + v of output lane % 16
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][4 * (lane >> 4) + v][lane & 15] = ps[v];
      }
      PROF_MARK(0)
      __syncthreads();
      if (sigma > 0 && active[k] && t_next >= 0 && t_next < L[k])
        Dh[k] = (red[0][r16][u] + red[1][r16][u] + red[2][r16][u] + red[3][r16][u]) * (1.f / kPartScale);
      float dz[4] = {0.f, 0.f, 0.f, 0.f};
      if (valid) lstm_cell_grad(gi, gf, gg, go, c_new, c_prev, dy + Dh[k], Dc[k], dz);
      if (pointwise) {
#pragma unroll
        for (int q = 0; q < 4; ++q) dbsum[q] += dz[q];       // (zero where the frame is padding)
#pragma unroll
        for (int q = 0; q < 4; ++q) zb[r16][q * 16 + u] = dz[q];
        if (active[k]) {
          float* zp = (float*)d.DZ + t * fg + (long)b * 4 * n + j;
          zp[0] = dz[0]; zp[n] = dz[1]; zp[2 * n] = dz[2]; zp[3 * n] = dz[3];
        }
      }
      PROF_MARK(2)
      __syncthreads();
      have_c = false;
      if (pointwise) {
        // what the next half step consumes (the other row tile's partial sums, published half a step ago) is collected here
        const int k_n = k ^ 1, sigma_n = k == 0 ? sigma : sigma + 1;
        const bool collect = nrt_here == 2 && sigma_n >= 1 && sigma_n <= T;
        const RingReader rn = reader(sigma_n, k_n);
        const unsigned tagw_n = rn.tag << 16;
        float psn[4] = {0.f, 0.f, 0.f, 0.f};
        unsigned stale_n = 0u;
        if (collect) {
#pragma unroll
          for (int it = 0; it < kWin; ++it) x[it] = rn.load_it(it);
        }
        // A operand: row lane % 16, gate columns 16 (lane / 16) .. + 15
        float av[16];
#pragma unroll
        for (int s4 = 0; s4 < 4; ++s4) {
          const float4 v = *(const float4*)&zb[lane & 15][(lane >> 4) * 16 + 4 * s4];
          av[4 * s4] = v.x; av[4 * s4 + 1] = v.y; av[4 * s4 + 2] = v.z; av[4 * s4 + 3] = v.w;
        }
        const unsigned tag_hi = part_tag(sigma + 1) << 30;
        const __amdgpu_buffer_rsrc_t ro = __builtin_amdgcn_make_buffer_rsrc((void*)((sigma & 1) ? d.ring1 : d.ring0), 0, ring_bytes, kBufFlags);
        // destination tile wave + 4 ci (one past the last: parked), this producer's block
        const unsigned pub0 = (unsigned)((((rt_base + k) * ntile + wave) * ntile + J) * 1024 + lane * 16);
        // The accumulator of column tile ci is published behind the MFMAs of column tile ci + 1: by then its last MFMA has long
        // finished (the compiler does not see the MFMAs in the assembly text and inserts no wait states for their results).
        auto publish = [&](int ci, const f32x4& acc) __attribute__((always_inline)) {
          const u32x4 unit = {__float_as_uint(acc[0]), __float_as_uint(acc[1]) | tag_hi, __float_as_uint(acc[2]), __float_as_uint(acc[3]) | tag_hi};
          const unsigned off = wave + 4 * ci < ntile ? pub0 + (unsigned)(4 * ci) * (unsigned)ntile * 1024u : 0x7ff00000u;
          __builtin_amdgcn_raw_buffer_store_b128(unit, ro, off, 0, 16);    // 16: agent scope, written through
        };
        f32x4 acc2[2];
#pragma unroll
        for (int ci = 0; ci < NCT; ++ci) {
          f32x4& acc = acc2[ci & 1];
#pragma unroll
          for (int s = 0; s < 16; ++s) {
            if (s == 0) mfma4_b_agpr_first(acc, av[0], w[ci][0][0]);
            else mfma4_b_agpr(acc, av[s], w[ci][s >> 2][s & 3]);
          }
          if (ci > 0) publish(ci - 1, acc2[(ci - 1) & 1]);
          if (collect) {                                   // (behind the MFMAs just issued: they run while this does)
            wait_loads_but((NCT - 1 - ci) < (kWin - 1) ? (NCT - 1 - ci) : (kWin - 1), x[ci % kWin]);     // the younger loads: the window's others
            stale_n |= rn.tag_diff(x[ci % kWin], ci, tagw_n);      // looked at once, behind the last load
            add_to(psn, x[ci % kWin]);
            if (ci + kWin < NCT) x[ci % kWin] = rn.load_it(ci + kWin);
          }
        }
        mfma_settle(acc2[(NCT - 1) & 1]);
        publish(NCT - 1, acc2[(NCT - 1) & 1]);
        if (collect) {
          // The tags are looked at once, here: a test and a branch per load cost a twentieth of the step.  A stale tag anywhere
          // (a tenth of the half steps): the sums are dropped and the next half step fetches every load again.
          const bool again = __builtin_amdgcn_ballot_w64(stale_n != 0u) != 0ull;
          if (again) { PROF_REDO(NCT) }
#pragma unroll
          for (int v = 0; v < 4; ++v) ps_c[v] = again ? 0.f : psn[v];
          redo_c = again ? (1ull << NCT) - 1ull : 0ull;
          have_c = true;
        }
      }
      PROF_MARK(1)
    }
  }
  PROF_DUMP("bwdf32", T)
#pragma unroll
  for (int k = 0; k < 2; ++k)
    if (active[k]) {
      const int b = (rt_base + k) * 16 + r16;
      d.Dh[(long)b * n + j] = Dh[k];
      d.Dc[(long)b * n + j] = Dc[k];
    }
  if (d.dbpart) {                       // bias gradient: this work-group's 32 rows summed into the first of the slab's four slices (the others stay zero)
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) zb[r16][q * 16 + u] = dbsum[q];
    __syncthreads();
    if (tid < 64) {
      const int q = tid >> 4, uu = tid & 15, jj = J * 16 + uu;
      float sum = 0.f;
#pragma unroll
      for (int rr = 0; rr < 16; ++rr) sum += zb[rr][q * 16 + uu];
      if (jj < n) d.dbpart[(long)2 * rt_base * 4 * n + q * n + jj] = sum;
    }
  }
}

// ------------------------------------------------------------------------------------------------
// packing for the ring layout
// forward weights: chunk index = (((dir*ntile + tile)*4 + q)*nkc + kc)*64 + lane
__device__ __forceinline__ void pack_wh_fwd_ll_body(long idx, const bf16_t* W, uint4* out, int n, int nkc, long total) {
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
    const int k = (kc * 4 + g) * 8 + e;                    // forward ring: slot = unit index (kLLSlotsFwd = kLLValsFwd)
    v[e] = (k < n && j < n) ? Wd[(long)k * 4 * n + q * n + j] : (bf16_t)0.f;
  }
  out[idx] = *(uint4*)v;
}
// partial-sum backward kernel: chunk index = ((((dir*ntile2 + J)*4 + wave)*4 + kc)*16 + c)*64 + lane ; B fragment of
// gate kc, K = the 32 units of tile J, columns = outputs (wave*16 + c)*16 .. +15
__device__ __forceinline__ void pack_wh_bwdp_body(long idx, const bf16_t* W, uint4* out, int n, int ntile2, long total) {
  if (idx >= total) return;
  const int lane = idx & 63, c = (idx >> 6) & 15, kc = (idx >> 10) & 3, wave = (idx >> 12) & 3;
  const long rest = idx >> 14;
  const int J = rest % ntile2, dir = rest / ntile2;
  const int jout = (wave * 16 + c) * 16 + (lane & 15), g = lane >> 4;
  const bf16_t* Wd = W + (long)dir * n * 4 * n;
  bf16_t v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int unit = J * 32 + g * 8 + e;
    // (scaled by 2^-32, exactly: the partial sums of Dh leave the MFMAs scaled, which keeps a bit of their bf16 form free)
    v[e] = (jout < n && unit < n) ? (bf16_t)((float)Wd[(long)jout * 4 * n + kc * n + unit] * kPartScale) : (bf16_t)0.f;
  }
  out[idx] = *(uint4*)v;
}
// Initial contents of the forward ring, one 8-byte unit per thread: slot 0 = zeros that carry the tag of step 0, slot 1 = zeros.
__device__ __forceinline__ void pack_state_ll_body(long idx, uint4* ring0, uint4* ring1, long total) {
  if (idx >= total) return;
  ((unsigned long long*)ring0)[idx] = (unsigned long long)(ll_fwd_tag(0u) * kLLFwdTagBit) << 32;
  ((unsigned long long*)ring1)[idx] = 0ull;
}
// Everything a bfloat16 single-launch loop needs set up, in ONE launch (three kernels in a row cost three start-ups and run one
// after the other; none of them depends on another): blocks [0, first_pack) clear the regions of `z` (as fill_zero_many_kernel does),
// blocks [first_pack, first_ring) bring W_h into the kernel's order (forward: ring order; backward: the partial-sum kernel's),
// blocks [first_ring, first_map) (forward only) write the initial ring, blocks from first_map on number the real frames
// (frame_map_body) when the products that follow go over real frames only.
struct PrepArgs {
  ZeroRegions z;
  const bf16_t* W; uint4* Wout; int n, nk; long w_total;   // nk: nkc (forward) / ntile2 (backward)
  uint4* ring0; uint4* ring1; long ring_total;
  const int* lens; int T, B; int* cidx; int* fidx; int* count;     // frame map (cidx == NULL: none)
  int first_pack, first_ring, first_map, backward;
};
__global__ __launch_bounds__(256) void prep_ll_kernel(PrepArgs a) {
  const int bid = blockIdx.x;
  if (bid < a.first_pack) {
    int k = 0;
#pragma unroll
    for (int j = 1; j < ZeroRegions::kMax; ++j)
      if (j < a.z.count && bid >= a.z.first_block[j]) k = j;
    uint32_t* p = (uint32_t*)a.z.ptr[k];
    const size_t nwords = a.z.words[k];
    const size_t nb = (size_t)(a.z.first_block[k + 1] - a.z.first_block[k]);
    for (size_t i = (size_t)(bid - a.z.first_block[k]) * 256 + threadIdx.x; i < nwords; i += nb * 256) p[i] = 0u;
  } else if (bid < a.first_ring) {
    const long idx = (long)(bid - a.first_pack) * 256 + threadIdx.x;
    if (a.backward) pack_wh_bwdp_body(idx, a.W, a.Wout, a.n, a.nk, a.w_total);
    else pack_wh_fwd_ll_body(idx, a.W, a.Wout, a.n, a.nk, a.w_total);
  } else if (bid < a.first_map) {
    pack_state_ll_body((long)(bid - a.first_ring) * 256 + threadIdx.x, a.ring0, a.ring1, a.ring_total);
  } else {
    frame_map_body(bid - a.first_map, a.lens, a.T, a.B, a.cidx, a.fidx, a.count);
  }
}
// The initial state's share of the first frame: gates[t0(b)][b][col] += sum_k bf16(h0[b][k]) W_h[k][col], t0 = the row's
// first frame in processing order.  One thread per column, a row per blockIdx.y; W_h rows are read coalesced.  Runs only
// when the caller passes an initial state.
template <typename TW>                                     // bfloat16 storage: h0 rounded as the recurrence would feed it
__global__ __launch_bounds__(256) void h0_term_kernel(const float* h0, const TW* W, float* gates, long gates_stride, const int* lens,
                                                      int T, int B, int n, int rev0, int rev1) {
  const int col = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y, dir = blockIdx.z;
  const int L = clamp_len(lens, b, T);
  if (col >= 4 * n || L <= 0) return;
  const float* hb = h0 + ((long)dir * B + b) * n;
  const TW* Wd = W + (long)dir * n * 4 * n + col;
  float acc = 0.f;
  for (int k = 0; k < n; ++k) acc += (sizeof(TW) == 2 ? bf_bits2f(f2bf_bits(hb[k])) : hb[k]) * (float)Wd[(long)k * 4 * n];
  const int t0 = (dir == 0 ? rev0 : rev1) ? L - 1 : 0;
  gates[dir * gates_stride + ((long)t0 * B + b) * 4 * n + col] += acc;
}

std::mutex g_capacity_mu;
std::map<std::pair<int, const void*>, int> g_capacity;    // (device, kernel) -> work-groups of the kernel that device holds at once

// How many work-groups of `kernel` the current device holds at once (0 if that cannot be found out).
template <typename K>
int capacity(K kernel) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return 0; }
  std::lock_guard<std::mutex> lock(g_capacity_mu);
  const auto key = std::make_pair(dev, (const void*)kernel);
  auto it = g_capacity.find(key);
  if (it == g_capacity.end()) {
    int per_cu = 0;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess ||
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, 256, 0) != hipSuccess) {
      (void)hipGetLastError();
      return 0;
    }
    it = g_capacity.emplace(key, per_cu * prop.multiProcessorCount).first;
  }
  return it->second;
}
// Can `grid` be resident all at once (the condition of a cooperative launch)?
template <typename K>
bool fits_device(K kernel, dim3 grid) { return (long)grid.x * grid.y * grid.z <= capacity(kernel); }

// Cooperative launches over the batch in slabs of whole 16-row tiles.  A work-group owns `rows_per_y` rows (16 or 8),
// so one row tile takes grid.x * (16 / rows_per_y) * ndir work-groups; as many row tiles as the device can hold at
// once go into one launch (the kernels need every work-group of a launch resident together), the rest follow in
// further launches on the same stream: batch rows never interact, each launch walks all T steps of its rows.
// Between launches the table in which exchange groups record their XCD is cleared again.  Returns
// hipErrorCooperativeLaunchTooLarge without launching anything if not even one row tile fits.
// Return values: hipSuccess; hipErrorCooperativeLaunchTooLarge = NOTHING was launched (the caller may use another
// kernel form or the per-step path on the untouched state); any other error = a later slab failed after earlier
// slabs had already advanced the state of their rows, so the call as a whole has failed and nothing may be re-run.
template <typename K, typename A>
hipError_t coop_slabs(K kernel, int grid_x, int rows_per_y, const A& a, hipStream_t s) {
  const int per_rt = 16 / rows_per_y, nrt = cdiv(a.B, 16);
  const long cap = capacity(kernel);
  const long slab = cap / ((long)grid_x * per_rt * a.ndir);            // row tiles per launch
  if (slab < 1) return hipErrorCooperativeLaunchTooLarge;
  for (int rt0 = 0; rt0 < nrt; rt0 += (int)slab) {
    A copy = a;
    copy.rt0 = rt0;
    const int here = (int)std::min<long>(slab, nrt - rt0);
    const dim3 grid(grid_x, per_rt * here, a.ndir);
    if (rt0 > 0 && a.xcc) {
      const hipError_t e = launch_fill_zero(a.xcc, (size_t)grid_x * per_rt * slab * a.ndir * 4, s);
      if (e != hipSuccess) return e == hipErrorCooperativeLaunchTooLarge ? hipErrorLaunchFailure : e;
    }
    void* args[] = {&copy};
    // (the grid has been checked against what the device holds at once either way; a cooperative launch goes through a
    // queue of its own, and crossing to it and back leaves the device idle for tens of microseconds)
    const hipError_t e = a.plain_launch ? hipLaunchKernel((const void*)kernel, grid, dim3(256), args, 0, s)
                                        : hipLaunchCooperativeKernel((const void*)kernel, grid, dim3(256), args, 0, s);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      if (rt0 == 0) return hipErrorCooperativeLaunchTooLarge;          // the first launch was refused: nothing has run
      return e == hipErrorCooperativeLaunchTooLarge ? hipErrorLaunchFailure : e;
    }
  }
  return hipSuccess;
}
// The kernels address a frame's arrays with 32-bit byte offsets and park idle lanes at offset 0x7ff00000: every frame
// array (gate pre-activations [B][4n] float, outputs [B][ld] bf16) and every ring must end below that offset.
inline bool offsets_fit(long B, long n, long ld_out, long ring_bytes) {
  const long lim = 0x7ff00000L;
  return B * 4 * n * 4 < lim && B * ld_out * 2 < lim && ring_bytes < lim;
}
template <typename K>
bool slab_fits(K kernel, int grid_x, int rows_per_y, int ndir) {
  return capacity(kernel) >= (long)grid_x * (16 / rows_per_y) * ndir;
}

}  // namespace

hipError_t launch_persist_fwd(const PFwdArgs& a, hipStream_t s) {
  if (a.nkc > kLLMaxNkcFwd) return hipErrorCooperativeLaunchTooLarge;
  if (!offsets_fit(a.B, a.n, std::max(a.d[0].ldy, a.d[a.ndir - 1].ldy), (long)cdiv(a.B, 16) * a.nkc * 1024)) return hipErrorCooperativeLaunchTooLarge;
  const int t32 = cdiv(cdiv(a.n, 16), 2), nrt = cdiv(a.B, 16);
  // more rows than the 32 x 8 form holds in one launch: 32 units x 16 rows, if that takes a single launch
  if ((long)t32 * 2 * nrt * a.ndir > capacity(persist_fwd8_kernel<kLLMaxNkcFwd / 4>) &&
      (long)t32 * nrt * a.ndir <= capacity(persist_fwd16r_kernel<kLLMaxNkcFwd / 4>)) {
    const hipError_t e16 = coop_slabs(persist_fwd16r_kernel<kLLMaxNkcFwd / 4>, t32, 16, a, s);
    if (e16 != hipErrorCooperativeLaunchTooLarge) return e16;
    (void)hipGetLastError();
  }
  // 32 units x 8 rows per work-group
  return coop_slabs(persist_fwd8_kernel<kLLMaxNkcFwd / 4>, t32, 8, a, s);
}
// Would launch_persist_fwd launch anything?  (Asked before the initial state's term is added to the pre-activations,
// which only the single-launch kernels expect there.)
bool persist_fwd_fits(const PFwdArgs& a) {
  if (a.nkc > kLLMaxNkcFwd) return false;
  if (!offsets_fit(a.B, a.n, std::max(a.d[0].ldy, a.d[a.ndir - 1].ldy), (long)cdiv(a.B, 16) * a.nkc * 1024)) return false;
  const int t32 = cdiv(cdiv(a.n, 16), 2);
  return slab_fits(persist_fwd8_kernel<kLLMaxNkcFwd / 4>, t32, 8, a.ndir);
}
bool persist_bwd_fits(const PBwdArgs& a) {
  const int t32 = cdiv(cdiv(a.n, 16), 2);
  if (!offsets_fit(a.B, a.n, std::max(a.d[0].lddy, a.d[a.ndir - 1].lddy), (long)bwdp_ring_bytes(a.B, a.n))) return false;
  return a.n <= 1024 && slab_fits(persist_bwdp_kernel<8>, t32, 8, a.ndir);
}
hipError_t launch_persist_bwd(const PBwdArgs& a, hipStream_t s) {
  const int t32 = cdiv(cdiv(a.n, 16), 2);
  // more rows than the 8-row form holds in one launch: 16 rows per work-group, if that takes a single launch
  const int nrt = cdiv(a.B, 16);
  if ((long)t32 * 2 * nrt * a.ndir > capacity(persist_bwdp_kernel<8>) && (long)t32 * nrt * a.ndir <= capacity(persist_bwdp16_kernel<8>)) {
    const hipError_t e16 = coop_slabs(persist_bwdp16_kernel<8>, t32, 16, a, s);
    if (e16 != hipErrorCooperativeLaunchTooLarge) return e16;
    (void)hipGetLastError();
  }
  return coop_slabs(persist_bwdp_kernel<8>, t32, 8, a, s);
}
hipError_t launch_prep_fwd_ll(const ZeroRegions& z, const void* W, uint4* Wf, int n, int nkc, int ndir, uint4* ring0, uint4* ring1,
                              int nrt, const FrameMapArgs& fm, hipStream_t s) {
  if (z.overflow) return hipErrorInvalidValue;
  PrepArgs a = {};
  a.z = z; a.W = (const bf16_t*)W; a.Wout = Wf; a.n = n; a.nk = nkc; a.w_total = (long)ndir * cdiv(n, 16) * 4 * nkc * 64;
  a.ring0 = ring0; a.ring1 = ring1; a.ring_total = (long)ndir * nrt * nkc * 64 * 2;
  a.first_pack = z.count ? z.first_block[z.count] : 0;
  a.first_ring = a.first_pack + cdiv(a.w_total, 256);
  a.first_map = a.first_ring + cdiv(a.ring_total, 256);
  a.backward = 0;
  a.lens = fm.lens; a.T = fm.T; a.B = fm.B; a.cidx = fm.cidx; a.fidx = fm.fidx; a.count = fm.count;
  hipLaunchKernelGGL(prep_ll_kernel, dim3(a.first_map + (fm.cidx ? cdiv(fm.T, 4) : 0)), dim3(256), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_prep_bwd_ll(const ZeroRegions& z, const void* W, uint4* Wb, int n, int ndir, const FrameMapArgs& fm, hipStream_t s) {
  if (z.overflow) return hipErrorInvalidValue;
  PrepArgs a = {};
  a.z = z; a.W = (const bf16_t*)W; a.Wout = Wb; a.n = n; a.nk = cdiv(n, 32); a.w_total = (long)ndir * a.nk * 4 * 4 * 16 * 64;
  a.first_pack = z.count ? z.first_block[z.count] : 0;
  a.first_ring = a.first_pack + cdiv(a.w_total, 256);
  a.first_map = a.first_ring;
  a.backward = 1;
  a.lens = fm.lens; a.T = fm.T; a.B = fm.B; a.cidx = fm.cidx; a.fidx = fm.fidx; a.count = fm.count;
  hipLaunchKernelGGL(prep_ll_kernel, dim3(a.first_map + (fm.cidx ? cdiv(fm.T, 4) : 0)), dim3(256), 0, s, a);
  return hipGetLastError();
}
// float ring, before the first step: slot 0 holds zeros that carry the tag of step 0 in every unit, slot 1 is cleared
__global__ void init_ring_f32_kernel(uint4* ring0, uint4* ring1, long total) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const unsigned t = ll_fwd_tag(0u) << 30;
  ring0[idx] = make_uint4(0u, t, 0u, t);
  ring1[idx] = make_uint4(0u, 0u, 0u, 0u);
}
bool persist_fwd_f32_fits(const PFwdArgs& a) {
  constexpr int kNch = 16;
  if (a.n % 8 != 0 || a.nkc > 4 * kNch || a.T < 2) return false;
  const long ring_bytes = (long)cdiv(a.B, 16) * a.nkc * 1024;
  if (ring_bytes >= 0x7ff00000L) return false;
  for (int d = 0; d < a.ndir; ++d) {
    const PFwdDir& f = a.d[d];
    if ((((uintptr_t)f.y | (uintptr_t)f.cs | (uintptr_t)f.hprev | (uintptr_t)f.gates | (uintptr_t)f.hstate | (uintptr_t)f.cstate) & 7) || (f.ldy & 1))
      return false;
  }
  return (long)cdiv(a.n, 16) * a.ndir <= capacity(persist_fwd_f32_kernel<kNch>);
}
// As many slabs of 32 rows per launch as the device holds at once (each launch walks all T steps of its rows; batch
// rows never interact).
hipError_t launch_persist_fwd_f32(const PFwdArgs& a, hipStream_t s) {
  constexpr int kNch = 16;
  if (!persist_fwd_f32_fits(a)) return hipErrorCooperativeLaunchTooLarge;
  const int nrt = cdiv(a.B, 16), nslab = cdiv(nrt, 2), grid_x = cdiv(a.n, 16);
  const int per_launch = (int)std::min<long>(nslab, capacity(persist_fwd_f32_kernel<kNch>) / ((long)grid_x * a.ndir));
  {
    const long total = (long)nrt * a.nkc * 64;
    for (int d = 0; d < a.ndir; ++d)
      hipLaunchKernelGGL(init_ring_f32_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, a.d[d].ring0, a.d[d].ring1, total);
    if (hipGetLastError() != hipSuccess) return hipErrorLaunchFailure;
  }
  for (int slab0 = 0; slab0 < nslab; slab0 += per_launch) {
    PFwdArgs copy = a;
    copy.rt0 = 2 * slab0;
    const dim3 grid(grid_x, std::min(per_launch, nslab - slab0), a.ndir);
    void* args[] = {&copy};
    const hipError_t e = a.plain_launch ? hipLaunchKernel((const void*)persist_fwd_f32_kernel<kNch>, grid, dim3(256), args, 0, s)
                                        : hipLaunchCooperativeKernel((const void*)persist_fwd_f32_kernel<kNch>, grid, dim3(256), args, 0, s);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      if (slab0 == 0) return hipErrorCooperativeLaunchTooLarge;        // the first launch was refused: nothing has run
      return e == hipErrorCooperativeLaunchTooLarge ? hipErrorLaunchFailure : e;
    }
  }
  return hipSuccess;
}
// W_h^T for the float partial-sum backward kernel, scaled by 2^-32: float index
// ((((dir*ntile + J)*4 + wave)*NCT + ci)*16 + s)*64 + lane holds W_h[unit (wave + 4 ci)*16 + lane%16][gate column
// (kappa/16)*n + J*16 + kappa%16], kappa = 16 (lane/16) + s; stored so that a lane's k-steps 4 s4 .. 4 s4 + 3 are one float4:
// float4 index ((((dir*ntile + J)*4 + wave)*NCT + ci)*4 + s4)*64 + lane.
__global__ void pack_wh_bwd_f32p_kernel(const float* W, float* out, int n, int ntile, int nct, long total) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int e = idx & 3;
  long rest = idx >> 2;
  const int lane = rest & 63; rest >>= 6;
  const int s4 = rest & 3; rest >>= 2;
  const int ci = rest % nct; rest /= nct;
  const int wave = rest & 3; rest >>= 2;
  const int J = rest % ntile, dir = rest / ntile;
  const int s = 4 * s4 + e, kappa = 16 * (lane >> 4) + s;
  const int unit_in = (wave + 4 * ci) * 16 + (lane & 15), unit_out = J * 16 + (kappa & 15), q = kappa >> 4;
  const float* Wd = W + (long)dir * n * 4 * n;
  out[idx] = (unit_in < n && unit_out < n) ? Wd[(long)unit_in * 4 * n + q * n + unit_out] * kPartScale : 0.f;
}
constexpr int kBwdF32Nct = 16;
bool persist_bwd_f32_fits(const PBwdArgs& a) {
  if (a.n % 8 != 0 || a.n > 64 * kBwdF32Nct || a.T < 2) return false;
  const long ntile = cdiv(a.n, 16);
  if ((long)cdiv(a.B, 16) * ntile * ntile * 1024 >= 0x7ff00000L) return false;
  return ntile * a.ndir <= capacity(persist_bwd_f32_kernel<kBwdF32Nct>);
}
hipError_t launch_pack_wh_bwd_f32p(const void* W, void* Wb, int n, int ndir, hipStream_t s) {
  const int ntile = cdiv(n, 16);
  const long total = (long)ndir * ntile * 4 * kBwdF32Nct * 16 * 64;
  hipLaunchKernelGGL(pack_wh_bwd_f32p_kernel, dim3(cdiv(total, 256)), dim3(256), 0, s, (const float*)W, (float*)Wb, n, ntile, kBwdF32Nct, total);
  return hipGetLastError();
}
// As many slabs of 32 rows per launch as the device holds at once; the rings must hold zeros.
hipError_t launch_persist_bwd_f32(const PBwdArgs& a, hipStream_t s) {
  if (!persist_bwd_f32_fits(a)) return hipErrorCooperativeLaunchTooLarge;
  const int nrt = cdiv(a.B, 16), nslab = cdiv(nrt, 2), grid_x = cdiv(a.n, 16);
  const int per_launch = (int)std::min<long>(nslab, capacity(persist_bwd_f32_kernel<kBwdF32Nct>) / ((long)grid_x * a.ndir));
  for (int slab0 = 0; slab0 < nslab; slab0 += per_launch) {
    PBwdArgs copy = a;
    copy.rt0 = 2 * slab0;
    const dim3 grid(grid_x, std::min(per_launch, nslab - slab0), a.ndir);
    void* args[] = {&copy};
    const hipError_t e = a.plain_launch ? hipLaunchKernel((const void*)persist_bwd_f32_kernel<kBwdF32Nct>, grid, dim3(256), args, 0, s)
                                        : hipLaunchCooperativeKernel((const void*)persist_bwd_f32_kernel<kBwdF32Nct>, grid, dim3(256), args, 0, s);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      if (slab0 == 0) return hipErrorCooperativeLaunchTooLarge;        // the first launch was refused: nothing has run
      return e == hipErrorCooperativeLaunchTooLarge ? hipErrorLaunchFailure : e;
    }
  }
  return hipSuccess;
}
hipError_t launch_h0_term(const float* h0, const void* W_h, bool bf16, float* gates, long gates_stride, const int* lens, int T, int B, int n,
                          int ndir, int rev0, int rev1, hipStream_t s) {
  if (B <= 0 || T <= 0) return hipSuccess;
  const dim3 grid(cdiv(4L * n, 256), B, ndir);
  if (bf16) hipLaunchKernelGGL(h0_term_kernel<bf16_t>, grid, dim3(256), 0, s, h0, (const bf16_t*)W_h, gates, gates_stride, lens, T, B, n, rev0, rev1);
  else hipLaunchKernelGGL(h0_term_kernel<float>, grid, dim3(256), 0, s, h0, (const float*)W_h, gates, gates_stride, lens, T, B, n, rev0, rev1);
  return hipGetLastError();
}

}  // namespace lstm
