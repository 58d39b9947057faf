// One step of batched beam search on the device (Sec. 3, Table 2: decoding is a batched beam search that runs on the GPU, beam
// size 12; Listing 1: "output_prob" softmax over the labels, "output" chooses, "trg" embeds the choice):
//
//     cand[q, b, v] = score[q, b] + logits[r, v] - logsumexp(logits[r, :]),  r = q * beam + b
//     the `beam` largest candidates of sentence q, best first, equal ones by ascending b * V + v  -> score', src, label
//     state rows follow their hypotheses: out[q * beam + k] = in[q * beam + src[q, k]]
//     trg[r] = W_trg[label[r]] + b_trg
//
// No candidate list of beam * V entries is ever sorted: a sentence's best `beam` candidates contain at most `beam` from one
// row, so every row first picks its own best `beam` labels in one pass over its logits (beam_row_kernel, a wavefront per
// row), and one wavefront per sentence merges the beam * beam survivors (beam_merge_kernel).  Nothing returns to the host.
#include <algorithm>
#include <mutex>

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
__device__ __forceinline__ bool better(const Cand& a, const Cand& b) { return a.v > b.v || (a.v == b.v && a.i < b.i); }
__device__ __forceinline__ Cand pick(const Cand& a, const Cand& b) { return better(a, b) ? a : b; }
__device__ __forceinline__ Cand wave_best(Cand c) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    Cand d;
    d.v = __shfl_xor(c.v, o);
    d.i = __shfl_xor(c.i, o);
    c = pick(c, d);
  }
  return c;
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

// Row r of the logits, one wavefront: a single pass over the row in which every lane keeps the best 16 of the entries it
// sees (in registers; an insertion is needed ever more rarely as the list fills up with large values) and a running
// logsumexp, then wave_select.  Writes cand_val[r][k] = score[r] + logits[r][label] - logsumexp and cand_lab[r][k].
// (Four wavefronts per row, each with a quarter of the row and a second merge, measured slower: 63 -> 77 us.)
template <int CAP>
__global__ __launch_bounds__(64) void beam_row_kernel(const float* __restrict__ logits, long ld, const float* __restrict__ score,
                                                       float* __restrict__ cand_val, int* __restrict__ cand_lab, int V, int beam) {
  const int r = blockIdx.x, lane = threadIdx.x;
  const float* src = logits + (long)r * ld;
  TopList<CAP> t;
  t.clear();
  float m = -__builtin_inff(), z = 0.f;                          // running maximum and sum of exp(x - m) of this lane's entries
  const auto fold = [&](float gm, float gz) {                    // merge (gm, gz) into (m, z)
    const float mn = fmaxf(m, gm);
    if (mn > -__builtin_inff()) z = z * __expf(m - mn) + gz * __expf(gm - mn);
    m = mn;
  };
  const bool vec = (ld & 3) == 0 && ((uintptr_t)logits & 15) == 0;
  const int n4 = vec ? V >> 2 : 0;
  constexpr int kU = 8;                                          // loads of 16 bytes in flight per lane
  // Inserting is a hundred instructions for the whole wavefront whenever ONE lane needs it, and with 64 private lists
  // some lane nearly always does.  So entries are first held against a bound that at least `beam` entries seen so far
  // reach: the `beam`-th largest of the 64 list heads, found by bisection over the ordered bit patterns with ballots,
  // renewed once per round of loads.  Whatever lies strictly below it cannot be among the row's best `beam`.
  float bound = -__builtin_inff();
  const int need = min(beam, 64);
  const auto renew_bound = [&]() {
    const unsigned f = __float_as_uint(t.v[0]);
    const unsigned key = (f & 0x80000000u) ? ~f : (f | 0x80000000u);             // larger float <=> larger key
    unsigned lo = 0u, hi = 0xffffffffu;
    while (lo < hi) {
      const unsigned mid = lo + ((hi - lo) >> 1) + 1u;
      if (__popcll(__ballot(key >= mid)) >= need) lo = mid; else hi = mid - 1u;
    }
    // lo = the need-th largest key; keys at or below that of -inf mean fewer than `need` lanes hold anything yet
    bound = lo <= 0x007fffffu ? -__builtin_inff() : __uint_as_float((lo & 0x80000000u) ? (lo & 0x7fffffffu) : ~lo);
  };
  for (int i0 = lane; i0 < n4; i0 += 64 * kU) {
    float4 x4[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) x4[u] = ((const float4*)src)[min(i0 + u * 64, n4 - 1)];
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      const int i4 = i0 + u * 64;
      if (i4 < n4) {
        const float x[4] = {x4[u].x, x4[u].y, x4[u].z, x4[u].w};
        const float gm = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
        if (gm > -__builtin_inff()) fold(gm, __expf(x[0] - gm) + __expf(x[1] - gm) + __expf(x[2] - gm) + __expf(x[3] - gm));
        if (gm >= bound && gm > t.v[CAP - 1]) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (x[e] >= bound && x[e] > t.v[CAP - 1]) t.template insert<true>(Cand{x[e], 4 * i4 + e});
        }
      }
    }
    renew_bound();
  }
  for (int i = 4 * n4 + lane; i < V; i += 64) {
    const float x = src[i];
    if (x > -__builtin_inff()) fold(x, 1.f);
    if (x > t.v[CAP - 1]) t.template insert<true>(Cand{x, i});
  }
  // logsumexp of the whole row
  float mw = m;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mw = fmaxf(mw, __shfl_xor(mw, o));
  float zw = mw > -__builtin_inff() ? z * __expf(m - mw) : 0.f;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) zw += __shfl_xor(zw, o);
  const float lse = mw + __logf(zw);
  const float sc = score[r];
  wave_select(t, beam, [&](int k, const Cand& win) {
    if (lane == 0) {
      const bool found = win.i != 0x7fffffff;                    // fewer than `beam` usable labels in the row: the rest never wins
      cand_val[(long)r * beam + k] = found ? sc + (win.v - lse) : -__builtin_inff();
      cand_lab[(long)r * beam + k] = found ? win.i : 0;
    }
  });
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
  wave_select(t, beam, [&](int k, const Cand& win) {
    if (lane == 0) {
      const bool real = win.i < beam * V;
      score_out[q * beam + k] = win.v;
      src_out[q * beam + k] = real ? win.i / V : 0;
      label_out[q * beam + k] = real ? win.i % V : 0;
    }
  });
}

// out[q * beam + k][0..width) = in[q * beam + src[q * beam + k]][0..width), elements of `esz` bytes copied as bytes pairs
__global__ void beam_gather_kernel(const uint16_t* __restrict__ in, long ld_in, const int* __restrict__ src, uint16_t* __restrict__ out,
                                   long ld_out, int rows, int beam, int halves) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)rows * halves) return;
  const int r = (int)(idx / halves), c = (int)(idx % halves);
  int s = src[r];
  s = s < 0 ? 0 : (s >= beam ? beam - 1 : s);
  out[(long)r * ld_out + c] = in[((long)(r / beam) * beam + s) * ld_in + c];
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
  // a lane's list holds as many entries as the beam asks for (in the worst case all of the row's best lie in one lane)
  if (beam <= 4) hipLaunchKernelGGL(beam_row_kernel<4>, dim3(Q * beam), dim3(64), 0, st, logits, (long)ld, score_in, cand_val, cand_lab, V, beam);
  else if (beam <= 8) hipLaunchKernelGGL(beam_row_kernel<8>, dim3(Q * beam), dim3(64), 0, st, logits, (long)ld, score_in, cand_val, cand_lab, V, beam);
  else if (beam <= 12) hipLaunchKernelGGL(beam_row_kernel<12>, dim3(Q * beam), dim3(64), 0, st, logits, (long)ld, score_in, cand_val, cand_lab, V, beam);
  else hipLaunchKernelGGL(beam_row_kernel<16>, dim3(Q * beam), dim3(64), 0, st, logits, (long)ld, score_in, cand_val, cand_lab, V, beam);
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

int lstm_beam_gather(int elem_bytes, int Q, int beam, int width, const void* in, int64_t ld_in, const int32_t* src, void* out,
                     int64_t ld_out, void* stream) {
  if (!in || !src || !out) return LSTM_ERR_NULL;
  if (Q < 0 || beam < 1 || width < 1 || ld_in < width || ld_out < width || (long)Q * beam > 0x7fffffffL / 16) return LSTM_ERR_DIM;
  if (elem_bytes != 2 && elem_bytes != 4) return LSTM_ERR_UNSUPPORTED;
  if ((((uintptr_t)in | (uintptr_t)out) & (elem_bytes - 1)) || ((uintptr_t)src & 3)) return LSTM_ERR_ALIGN;
  if (in == out) return LSTM_ERR_UNSUPPORTED;                     // rows are read while others are written
  if (Q == 0) return LSTM_OK;
  int rc = device_ok();
  if (rc) return rc;
  const int halves = width * (elem_bytes / 2), rows = Q * beam;
  const long total = (long)rows * halves;
  hipLaunchKernelGGL(beam_gather_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, (hipStream_t)stream, (const uint16_t*)in,
                     (long)ld_in * (elem_bytes / 2), src, (uint16_t*)out, (long)ld_out * (elem_bytes / 2), rows, beam, halves);
  if (hipGetLastError() != hipSuccess) return LSTM_ERR_HIP;
  return LSTM_OK;
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
