// One step of batched beam search on the device (Sec. 3, Table 2: decoding is a batched beam search that runs on the GPU, beam
// size 12; Listing 1: "output_prob" softmax over the labels, "output" chooses, "trg" embeds the choice):
//
//     cand[q, b, v] = score[q, b] + logits[r, v] - logsumexp(logits[r, :]),  r = q * beam + b
//     the `beam` largest candidates of sentence q, best first, equal ones by ascending b * V + v  -> score', src, label
//     state rows follow their hypotheses: out[q * beam + k] = in[q * beam + src[q, k]]
//     trg[r] = W_trg[label[r]] + b_trg
//
// No candidate list of beam * V entries is ever sorted: a sentence's best `beam` candidates contain at most `beam` from one
// row, so every row first picks its own best `beam` labels in one pass over its logits (beam_row_kernel, a work-group of
// four wavefronts per row), and one wavefront per sentence merges the beam * beam survivors (beam_merge_kernel).  Nothing
// returns to the host.
#include <algorithm>
#include <mutex>
#include <type_traits>

#include "../../include/lstm_abi.h"
#include "common.h"

namespace lstm {
namespace {

constexpr int kBeamMax = 16;
constexpr int kVocabMax = 1 << 26;    // beam * V must fit an int32 flat index

// Scratch of lstm_beam_step_static: Q * beam * beam survivors (value and label) at most kStaticCands of each, e.g. 256
// sentences at beam 16.  512 KiB of every device the library runs on, held until the process ends.
constexpr uint64_t kStaticCands = 1u << 16;
constexpr int kStaticDevices = 64;
static __device__ __align__(256) unsigned char scratch[2 * kStaticCands * 4];
std::mutex g_static_mu;
void* g_static_ptr[kStaticDevices] = {};   // device address of `scratch` per device, from hipGetSymbolAddress

// (value, index) pairs ordered by larger value first, then smaller index: `better(a, b)` = a comes before b
struct Cand { float v; int i; };
__device__ __forceinline__ bool better(const Cand& a, const Cand& b) { return (a.v > b.v) | ((a.v == b.v) & (a.i < b.i)); }
// field by field: selecting between two structs made the compiler store both to scratch memory and load one back
__device__ __forceinline__ Cand pick(const Cand& a, const Cand& b) {
  const bool t = better(a, b);
  Cand c;
  c.v = t ? a.v : b.v;
  c.i = t ? a.i : b.i;
  return c;
}
// The best candidate of the wavefront, in every lane.  Six combining steps through DPP moves (neighbour in the quad, other
// pair of the quad, mirrored half row, mirrored row, last lane of the row before, last lane of the first half), after
// which lane 63 holds the result; 64 lanes of `__shfl_xor` took six dependent trips through the LDS crossbar per value.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ Cand dpp_step(const Cand& c) {
  Cand d;   // lanes that the move does not reach (row mask, row_bcast sources out of range) keep their own candidate
  d.v = __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(c.v), __float_as_int(c.v), CTRL, ROW_MASK, 0xf, false));
  d.i = __builtin_amdgcn_update_dpp(c.i, c.i, CTRL, ROW_MASK, 0xf, false);
  return pick(c, d);
}
__device__ __forceinline__ Cand wave_best(Cand c) {
  c = dpp_step<0xB1, 0xf>(c);       // quad_perm [1,0,3,2]
  c = dpp_step<0x4E, 0xf>(c);       // quad_perm [2,3,0,1]
  c = dpp_step<0x141, 0xf>(c);      // row_half_mirror
  c = dpp_step<0x140, 0xf>(c);      // row_mirror: every lane holds the best of its row of 16
  c = dpp_step<0x142, 0xa>(c);      // row_bcast15 into rows 1 and 3
  c = dpp_step<0x143, 0xc>(c);      // row_bcast31 into rows 2 and 3
  Cand w;
  w.v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(c.v), 63));
  w.i = __builtin_amdgcn_readlane(c.i, 63);
  return w;
}
// A lane's best CAP candidates so far, best first.
template <int CAP>
struct TopList {
  float v[CAP];
  int i[CAP];
  __device__ __forceinline__ void clear() {
#pragma unroll
    for (int p = 0; p < CAP; ++p) { v[p] = -__builtin_inff(); i[p] = 0x7fffffff; }
  }
  // insert c, dropping the last entry; ORDERED: the caller offers candidates in ascending index order, so one that
  // equals an entry in value comes after it and a value comparison is enough
  template <bool ORDERED>
  __device__ __forceinline__ void insert(const Cand& c) {
    const auto before = [&](int p) { return ORDERED ? c.v > v[p] : better(c, Cand{v[p], i[p]}); };
#pragma unroll
    for (int p = CAP - 1; p > 0; --p) {
      const bool shift = before(p - 1), here = before(p);
      v[p] = shift ? v[p - 1] : (here ? c.v : v[p]);
      i[p] = shift ? i[p - 1] : (here ? c.i : i[p]);
    }
    const bool first = before(0);
    v[0] = first ? c.v : v[0];
    i[0] = first ? c.i : i[0];
  }
  __device__ __forceinline__ void pop() {
#pragma unroll
    for (int p = 0; p + 1 < CAP; ++p) { v[p] = v[p + 1]; i[p] = i[p + 1]; }
    v[CAP - 1] = -__builtin_inff();
    i[CAP - 1] = 0x7fffffff;
  }
};

// The wavefront's best `beam` candidates out of its 64 lists, best first: `beam` rounds in which every lane offers the
// head of its list and the lane that wins drops it.  emit(k, winner) runs in every lane.
template <int CAP, typename F>
__device__ __forceinline__ void wave_select(TopList<CAP>& t, int beam, F emit) {
  for (int k = 0; k < beam; ++k) {
    const Cand head = {t.v[0], t.i[0]};
    const Cand win = wave_best(head);
    if (win.i == head.i && win.i != 0x7fffffff) t.pop();        // indices are unique, so exactly one lane owns the winner
    emit(k, win);
  }
}

// Row r of the logits, one work-group of four wavefronts, each with a quarter of the row: a single pass with a running
// logsumexp.  Sorted lists per lane cost a hundred instructions for the whole wavefront whenever ONE lane has to insert, and
// with 64 lists some lane nearly always has (59 us for 768 rows of 20000).  Instead a wavefront keeps a bound that at least
// `beam` of the entries it has seen reach - the `beam`-th largest of its 64 lanes' running maxima, found by bisection over
// the ordered bit patterns with ballots, renewed once per round of loads - and appends whatever reaches the bound to its
// candidate buffer in LDS (ballot, count, one store per value): an entry strictly below the bound has `beam` entries in
// front of it and can be dropped.  A typical row leaves a few hundred candidates, from which `beam` rounds of "every lane
// offers its best, the wavefront picks" take the row's best, equal values by ascending label.  Should a buffer run short of
// a round's worth of room (rows that keep rising), it is first cut down to its best `beam` the same way.
// Writes cand_val[r][k] = score[r] + logits[r][label] - logsumexp and cand_lab[r][k].
constexpr int kRowU = 4;                         // loads of 16 bytes in flight per lane
constexpr int kRowRound = 64 * kRowU * 4;        // entries per wavefront and round of loads
constexpr int kRowCap = kRowRound + 512;         // candidate buffer per wavefront (4 x 12 KiB per work-group)
// LDS traffic between the lanes of ONE wavefront: its LDS instructions execute in program order, so all that is needed is
// that the compiler keeps them in that order
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
__global__ __launch_bounds__(256) void beam_row_kernel(const float* __restrict__ logits, long ld, const float* __restrict__ score,
                                                        float* __restrict__ cand_val, int* __restrict__ cand_lab, int V, int beam) {
  __shared__ float bv[4 * kRowCap];
  __shared__ int bi[4 * kRowCap];
  __shared__ int cnt[4];
  __shared__ float part_m[4], part_z[4], part_b[4];
  __shared__ float fv[64];                                      // the row's finalists (see the end)
  __shared__ int fi[64];
  __shared__ int fcount;
  if (threadIdx.x == 0) fcount = 0;
  const int r = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* src = logits + (long)r * ld;
  const float kNegInf = -__builtin_inff();
  float m = kNegInf, z = 0.f;                                    // running maximum and sum of exp(x - m) of this lane's entries
  const auto fold = [&](float gm, float gz) {                    // merge (gm, gz) into (m, z)
    const float mn = fmaxf(m, gm);
    if (mn > kNegInf) z = z * __expf(m - mn) + gz * __expf(gm - mn);
    m = mn;
  };
  const int need = min(beam, 64);
  float bound = kNegInf;
  const auto renew_bound = [&]() {                               // the need-th largest of the lanes' maxima m, rounded down
    const unsigned f = __float_as_uint(m);
    const unsigned key = ((f & 0x80000000u) ? ~f : (f | 0x80000000u)) >> 12;     // larger float => key not smaller; 20 bits
    unsigned lo = 0u, hi = 0xfffffu;
    while (lo < hi) {
      const unsigned mid = lo + ((hi - lo) >> 1) + 1u;
      if (__popcll(__ballot(key >= mid)) >= need) lo = mid; else hi = mid - 1u;
    }
    // lo = the need-th largest key: at least `need` maxima are at or above the smallest float with that key.  Keys at or
    // below that of -inf mean fewer than `need` lanes hold anything yet.
    const unsigned full = lo << 12;                               // the smallest ordered pattern with this key
    bound = lo <= (0x007fffffu >> 12) ? kNegInf : __uint_as_float((full & 0x80000000u) ? (full & 0x7fffffffu) : ~full);
  };
  float* wbv = bv + wave * kRowCap;
  int* wbi = bi + wave * kRowCap;
  int count = 0;                                                 // candidates in this wavefront's buffer (the same in every lane)
  const auto append = [&](bool keep, float x, int label) {       // wavefront-wide: every lane calls it
    const unsigned long long mask = __ballot(keep);
    if (mask == 0ull) return;
    if (keep) {
      const int pos = count + (int)__popcll(mask & ((1ull << lane) - 1ull));
      wbv[pos] = x;
      wbi[pos] = label;
    }
    count += (int)__popcll(mask);
  };
  // One round of picking over this wavefront's buffer (ALL = false, `count` entries) or all four (counts in cnt[]): the
  // best candidate, which leaves its buffer.  Runs in one wavefront.  (Counts in a private array indexed by the loop
  // would live in scratch memory: a trip to memory per buffer and round.)
  const auto pick_best = [&](auto all) {
    constexpr bool ALL = decltype(all)::value;
    Cand mine = {kNegInf, 0x7fffffff};
    int at = -1;
#pragma unroll
    for (int w = 0; w < (ALL ? 4 : 1); ++w) {
      const int buf = ALL ? w : wave, n = ALL ? cnt[w] : count;
      for (int p = lane; p < n; p += 64) {
        const int q = buf * kRowCap + p;
        const Cand cd = {bv[q], bi[q]};
        if (cd.i != 0x7fffffff && better(cd, mine)) { mine = cd; at = q; }
      }
    }
    const Cand win = wave_best(mine);
    if (at >= 0 && win.i == mine.i) bi[at] = 0x7fffffff;         // labels are unique, so exactly one lane owns the winner
    wave_lds_sync();
    return win;
  };
  const auto make_room = [&]() {                                 // before a round: room for all its entries
    if (count <= kRowCap - kRowRound) return;
    wave_lds_sync();
    Cand kept = {kNegInf, 0x7fffffff};
    for (int k = 0; k < need; ++k) {
      const Cand win = pick_best(std::false_type{});
      if (lane == k) kept = win;
    }
    count = 0;
    append(kept.i != 0x7fffffff, kept.v, kept.i);
    wave_lds_sync();
  };
  const bool vec = (ld & 3) == 0 && ((uintptr_t)logits & 15) == 0;
  const int n4 = vec ? V >> 2 : 0;
  const int q4 = (n4 + 3) >> 2, end4 = min(n4, (wave + 1) * q4);  // this wavefront's 16-byte pieces: [wave * q4, end4)
  for (int base = wave * q4; base < end4; base += 64 * kRowU) {
    float4 x4[kRowU];
    float g[kRowU];
#pragma unroll
    for (int u = 0; u < kRowU; ++u) x4[u] = ((const float4*)src)[min(base + lane + u * 64, end4 - 1)];
#pragma unroll
    for (int u = 0; u < kRowU; ++u) {
      const float gm = fmaxf(fmaxf(x4[u].x, x4[u].y), fmaxf(x4[u].z, x4[u].w));
      g[u] = base + lane + u * 64 < end4 ? gm : kNegInf;
      if (g[u] > kNegInf) fold(gm, __expf(x4[u].x - gm) + __expf(x4[u].y - gm) + __expf(x4[u].z - gm) + __expf(x4[u].w - gm));
    }
    renew_bound();                                               // counts this round's entries as well
    make_room();
#pragma unroll
    for (int u = 0; u < kRowU; ++u) {
      const bool any = g[u] > kNegInf && g[u] >= bound;
      if (__ballot(any) == 0ull) continue;
      const int i4 = base + lane + u * 64;
      const float x[4] = {x4[u].x, x4[u].y, x4[u].z, x4[u].w};
#pragma unroll
      for (int e = 0; e < 4; ++e) append(any && x[e] > kNegInf && x[e] >= bound, x[e], 4 * i4 + e);
    }
  }
  for (int base = 4 * n4 + wave * 64 * kRowU; base < V; base += 4 * 64 * kRowU) {   // what 16-byte loads do not cover
    float x[kRowU];
#pragma unroll
    for (int u = 0; u < kRowU; ++u) {
      const int i = base + lane + u * 64;
      x[u] = i < V ? src[i] : kNegInf;
      if (x[u] > kNegInf) fold(x[u], 1.f);
    }
    renew_bound();
    make_room();
#pragma unroll
    for (int u = 0; u < kRowU; ++u) append(x[u] > kNegInf && x[u] >= bound, x[u], base + lane + u * 64);
  }
  // logsumexp of this wavefront's part, then of the whole row
  float mw = m;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mw = fmaxf(mw, __shfl_xor(mw, o));
  float zw = mw > kNegInf ? z * __expf(m - mw) : 0.f;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) zw += __shfl_xor(zw, o);
  if (lane == 0) { part_m[wave] = mw; part_z[wave] = zw; cnt[wave] = count; part_b[wave] = bound; }
  __syncthreads();
  // Finalists: every one of the row's best `beam` reaches the largest of the four wavefronts' bounds (at least `beam`
  // entries of that wavefront's quarter do).  Each wavefront copies its candidates at or above it to a common list of 64;
  // if they fit - they nearly always do: a few dozen - the first wavefront ranks them in registers (a candidate's place
  // is the number of better ones: no rounds, nothing through LDS), else it picks from the four buffers round by round.
  const float top_bound = fmaxf(fmaxf(part_b[0], part_b[1]), fmaxf(part_b[2], part_b[3]));
  for (int p0 = 0; p0 < count; p0 += 64) {
    const int p = p0 + lane;
    const bool keep = p < count && wbv[p] >= top_bound;
    const unsigned long long mask = __ballot(keep);
    if (mask == 0ull) continue;
    int base = 0;
    if (lane == 0) base = atomicAdd(&fcount, (int)__popcll(mask));
    base = __builtin_amdgcn_readfirstlane(base);
    const int pos = base + (int)__popcll(mask & ((1ull << lane) - 1ull));
    if (keep && pos < 64) { fv[pos] = wbv[p]; fi[pos] = wbi[p]; }
  }
  __syncthreads();
  if (wave != 0) return;
  const float mr = fmaxf(fmaxf(part_m[0], part_m[1]), fmaxf(part_m[2], part_m[3]));
  float zr = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) zr += part_m[w] > kNegInf ? part_z[w] * __expf(part_m[w] - mr) : 0.f;
  const float lse = mr + __logf(zr);
  const float sc = score[r];
  const int total = fcount;
  if (total <= 64) {
    const Cand mine = {lane < total ? fv[lane] : kNegInf, lane < total ? fi[lane] : 0x7fffffff};
    int place = 0;
    for (int j = 0; j < total; ++j) {
      const Cand other = {__int_as_float(__builtin_amdgcn_readlane(__float_as_int(mine.v), j)), __builtin_amdgcn_readlane(mine.i, j)};
      place += better(other, mine) ? 1 : 0;
    }
    if (lane < total && place < beam) {
      cand_val[(long)r * beam + place] = sc + (mine.v - lse);
      cand_lab[(long)r * beam + place] = mine.i;
    }
    if (lane >= total && lane < beam) {                          // fewer than `beam` usable labels in the row: the rest never wins
      cand_val[(long)r * beam + lane] = kNegInf;
      cand_lab[(long)r * beam + lane] = 0;
    }
    return;
  }
  // lane k keeps the k-th best and stores it at the end
  Cand kept = {kNegInf, 0x7fffffff};
  for (int k = 0; k < beam; ++k) {
    const Cand win = pick_best(std::true_type{});
    if (lane == k) kept = win;
  }
  if (lane < beam) {
    const bool found = kept.i != 0x7fffffff;
    cand_val[(long)r * beam + lane] = found ? sc + (kept.v - lse) : kNegInf;
    cand_lab[(long)r * beam + lane] = found ? kept.i : 0;
  }
}

// The beam * beam survivors of sentence q = blockIdx.x, one wavefront: the best `beam`, by value and then by flat index
// b * V + label.
__global__ __launch_bounds__(64) void beam_merge_kernel(const float* __restrict__ cand_val, const int* __restrict__ cand_lab,
                                                         float* __restrict__ score_out, int* __restrict__ src_out,
                                                         int* __restrict__ label_out, int V, int beam) {
  const int q = blockIdx.x, lane = threadIdx.x;
  TopList<4> t;                                                 // beam * beam / 64 <= 4 candidates per lane
  t.clear();
  for (int c = lane; c < beam * beam; c += 64) {
    const float val = cand_val[(long)q * beam * beam + c];
    const int flat = (c / beam) * V + cand_lab[(long)q * beam * beam + c];
    // a row with fewer than `beam` labels pads with (-inf, label 0): give the padding indices that cannot collide
    t.insert<false>(Cand{val, val == -__builtin_inff() ? 0x7ffffffe - c : flat});
  }
  Cand kept = {-__builtin_inff(), 0x7fffffff};
  wave_select(t, beam, [&](int k, const Cand& win) { if (lane == k) kept = win; });
  if (lane < beam) {
    const bool real = kept.i < beam * V;
    score_out[q * beam + lane] = kept.v;
    src_out[q * beam + lane] = real ? kept.i / V : 0;
    label_out[q * beam + lane] = real ? kept.i % V : 0;
  }
}

// out[q * beam + k][0..width) = in[q * beam + src[q * beam + k]][0..width) for up to kGatherMax arrays in one launch.  Array i
// is copied in units of unit[i] bytes (16, 8, 4 or 2: the widest that its row length, leading dimensions and base addresses
// allow), one unit per thread; blocks [first_block[i], first_block[i+1]) work on array i.
constexpr int kGatherMax = 8;
struct GatherArgs {
  const char* in[kGatherMax]; char* out[kGatherMax];
  long ld_in[kGatherMax], ld_out[kGatherMax];          // bytes
  int units[kGatherMax], unit[kGatherMax];             // units per row; bytes per unit
  int first_block[kGatherMax + 1];
  int count, rows, beam;
  const int* src;
};
__global__ __launch_bounds__(256) void beam_gather_kernel(GatherArgs a) {
  int i = 0;
#pragma unroll
  for (int j = 1; j < kGatherMax; ++j)
    if (j < a.count && (int)blockIdx.x >= a.first_block[j]) i = j;
  const long idx = (long)((int)blockIdx.x - a.first_block[i]) * 256 + threadIdx.x;
  const int upr = a.units[i];
  if (idx >= (long)a.rows * upr) return;
  const int r = (int)(idx / upr), c = (int)(idx - (long)r * upr);
  int s = a.src[r];
  s = s < 0 ? 0 : (s >= a.beam ? a.beam - 1 : s);
  const int u = a.unit[i];
  const char* pi = a.in[i] + ((long)(r / a.beam) * a.beam + s) * a.ld_in[i] + (long)c * u;
  char* po = a.out[i] + (long)r * a.ld_out[i] + (long)c * u;
  if (u == 16) *(uint4*)po = *(const uint4*)pi;
  else if (u == 8) *(uint2*)po = *(const uint2*)pi;
  else if (u == 4) *(uint32_t*)po = *(const uint32_t*)pi;
  else *(uint16_t*)po = *(const uint16_t*)pi;
}

// trg[r] = W[label[r]] + b (bfloat16 table and result, float bias); labels outside [0, V) give the bias alone
__global__ void embed_kernel(const int* __restrict__ label, const uint16_t* __restrict__ W, const float* __restrict__ b,
                             uint16_t* __restrict__ out, long ld_out, int rows, int n, int V) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)rows * n) return;
  const int r = (int)(idx / n), c = (int)(idx % n);
  const int l = label[r];
  const float w = (l >= 0 && l < V) ? bf_bits2f(W[(long)l * n + c]) : 0.f;
  out[(long)r * ld_out + c] = f2bf_bits(w + (b ? b[c] : 0.f));
}

}  // namespace
}  // namespace lstm

using namespace lstm;

extern "C" {

static int beam_dims(int Q, int beam, int V) {
  if (Q < 0 || beam < 1 || V < 1 || (long)Q * beam > 0x7fffffffL / 16) return LSTM_ERR_DIM;
  if (beam > kBeamMax || V > kVocabMax) return LSTM_ERR_UNSUPPORTED;
  return LSTM_OK;
}

int lstm_beam_query(int Q, int beam, int V, uint64_t* workspace_bytes) {
  if (!workspace_bytes) return LSTM_ERR_NULL;
  const int rc = beam_dims(Q, beam, V);
  if (rc) return rc;
  *workspace_bytes = 256 + 2 * (((uint64_t)Q * beam * beam * 4 + 255) / 256 * 256);
  return LSTM_OK;
}

// both kernels of a step; cand_val / cand_lab hold Q * beam * beam entries each
static int beam_launch(int Q, int beam, int V, const float* logits, int64_t ld, const float* score_in, float* score_out, int32_t* src,
                       int32_t* label, float* cand_val, int* cand_lab, hipStream_t st) {
  hipLaunchKernelGGL(beam_row_kernel, dim3(Q * beam), dim3(256), 0, st, logits, (long)ld, score_in, cand_val, cand_lab, V, beam);
  hipLaunchKernelGGL(beam_merge_kernel, dim3(Q), dim3(64), 0, st, cand_val, cand_lab, score_out, src, label, V, beam);
  if (hipGetLastError() != hipSuccess) return LSTM_ERR_HIP;
  return LSTM_OK;
}

static int beam_step_args(int Q, int beam, int V, const float* logits, int64_t ld, const float* score_in, float* score_out, int32_t* src,
                          int32_t* label) {
  if (!logits || !score_in || !score_out || !src || !label) return LSTM_ERR_NULL;
  const int rc = beam_dims(Q, beam, V);
  if (rc) return rc;
  if (ld < V) return LSTM_ERR_DIM;
  if (((uintptr_t)logits | (uintptr_t)score_in | (uintptr_t)score_out | (uintptr_t)src | (uintptr_t)label) & 3) return LSTM_ERR_ALIGN;
  return LSTM_OK;
}

int lstm_beam_step(int Q, int beam, int V, const float* logits, int64_t ld, const float* score_in, float* score_out, int32_t* src,
                   int32_t* label, void* workspace, uint64_t workspace_bytes, void* stream) {
  if (!workspace) return LSTM_ERR_NULL;
  int rc = beam_step_args(Q, beam, V, logits, ld, score_in, score_out, src, label);
  if (rc) return rc;
  uint64_t need = 0;
  lstm_beam_query(Q, beam, V, &need);
  if (workspace_bytes < need) return LSTM_ERR_SIZE;
  if (Q == 0) return LSTM_OK;
  if ((rc = device_ok())) return rc;
  char* ws = (char*)(((uintptr_t)workspace + 255) / 256 * 256);
  float* cand_val = (float*)ws;
  int* cand_lab = (int*)(ws + ((size_t)Q * beam * beam * 4 + 255) / 256 * 256);
  return beam_launch(Q, beam, V, logits, ld, score_in, score_out, src, label, cand_val, cand_lab, (hipStream_t)stream);
}

// The same step for callers that cannot allocate: the survivors of the rows (the only scratch of the step) go to a
// device array that is part of the library's image.  Its address on each device is looked up once, with that device
// current, and kept; host code never uses the array's name for anything else.
int lstm_beam_step_static(int Q, int beam, int V, const float* logits, int64_t ld, const float* score_in, float* score_out,
                          int32_t* src, int32_t* label, void* stream) {
  int rc = beam_step_args(Q, beam, V, logits, ld, score_in, score_out, src, label);
  if (rc) return rc;
  if ((uint64_t)Q * beam * beam > kStaticCands) return LSTM_ERR_SIZE;
  if (Q == 0) return LSTM_OK;
  if ((rc = device_ok())) return rc;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kStaticDevices) { (void)hipGetLastError(); return LSTM_ERR_HIP; }
  char* base = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
      void* p = nullptr;
      if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) { (void)hipGetLastError(); return LSTM_ERR_HIP; }
      g_static_ptr[dev] = p;
    }
    base = (char*)g_static_ptr[dev];
  }
  // every entry the merge reads is written by the row kernel of the same call: nothing has to be cleared
  return beam_launch(Q, beam, V, logits, ld, score_in, score_out, src, label, (float*)base, (int*)(base + kStaticCands * 4),
                     (hipStream_t)stream);
}

int lstm_beam_gather_many(int Q, int beam, int count, const lstm_gather_item* items, const int32_t* src, void* stream) {
  if (!items || !src) return LSTM_ERR_NULL;
  if (count < 1 || count > kGatherMax) return LSTM_ERR_DIM;
  if (Q < 0 || beam < 1 || (long)Q * beam > 0x7fffffffL / 16) return LSTM_ERR_DIM;
  if ((uintptr_t)src & 3) return LSTM_ERR_ALIGN;
  GatherArgs a = {};
  a.count = count; a.rows = Q * beam; a.beam = beam; a.src = src;
  for (int i = 0; i < count; ++i) {
    const lstm_gather_item& it = items[i];
    if (!it.in || !it.out) return LSTM_ERR_NULL;
    if (it.width < 1 || it.ld_in < it.width || it.ld_out < it.width) return LSTM_ERR_DIM;
    if (it.elem_bytes != 2 && it.elem_bytes != 4) return LSTM_ERR_UNSUPPORTED;
    if (((uintptr_t)it.in | (uintptr_t)it.out) & (uintptr_t)(it.elem_bytes - 1)) return LSTM_ERR_ALIGN;
    if (it.in == it.out) return LSTM_ERR_UNSUPPORTED;             // rows are read while others are written
    const long row_bytes = (long)it.width * it.elem_bytes, lbi = (long)it.ld_in * it.elem_bytes, lbo = (long)it.ld_out * it.elem_bytes;
    const uintptr_t all = (uintptr_t)it.in | (uintptr_t)it.out | (uintptr_t)row_bytes | (uintptr_t)lbi | (uintptr_t)lbo;
    const int u = !(all & 15) ? 16 : !(all & 7) ? 8 : !(all & 3) ? 4 : 2;
    a.in[i] = (const char*)it.in; a.out[i] = (char*)it.out; a.ld_in[i] = lbi; a.ld_out[i] = lbo;
    a.unit[i] = u; a.units[i] = (int)(row_bytes / u);
    const long blocks = ((long)a.rows * a.units[i] + 255) / 256;
    if (blocks + a.first_block[i] > 0x7fffffffL) return LSTM_ERR_DIM;
    a.first_block[i + 1] = a.first_block[i] + (int)blocks;
  }
  if (Q == 0) return LSTM_OK;
  int rc = device_ok();
  if (rc) return rc;
  hipLaunchKernelGGL(beam_gather_kernel, dim3((unsigned)a.first_block[count]), dim3(256), 0, (hipStream_t)stream, a);
  if (hipGetLastError() != hipSuccess) return LSTM_ERR_HIP;
  return LSTM_OK;
}

int lstm_beam_gather(int elem_bytes, int Q, int beam, int width, const void* in, int64_t ld_in, const int32_t* src, void* out,
                     int64_t ld_out, void* stream) {
  if (!in || !src || !out) return LSTM_ERR_NULL;
  const lstm_gather_item it = {elem_bytes, width, in, ld_in, out, ld_out};
  return lstm_beam_gather_many(Q, beam, 1, &it, src, stream);
}

int lstm_embed(int B, int n, int V, const int32_t* label, const void* W_trg, const float* b_trg, void* out, int64_t ld_out, void* stream) {
  if (!label || !W_trg || !out) return LSTM_ERR_NULL;
  if (B < 0 || n < 1 || V < 1 || ld_out < n || (long)B * n > 0x7fffffffL) return LSTM_ERR_DIM;
  if ((((uintptr_t)W_trg | (uintptr_t)out) & 1) || (((uintptr_t)label | (uintptr_t)b_trg) & 3)) return LSTM_ERR_ALIGN;
  if (B == 0) return LSTM_OK;
  int rc = device_ok();
  if (rc) return rc;
  const long total = (long)B * n;
  hipLaunchKernelGGL(embed_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream, label, (const uint16_t*)W_trg, b_trg,
                     (uint16_t*)out, (long)ld_out, B, n, V);
  if (hipGetLastError() != hipSuccess) return LSTM_ERR_HIP;
  return LSTM_OK;
}

}  // extern "C"
