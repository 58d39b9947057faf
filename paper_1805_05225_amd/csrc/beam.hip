// One step of batched beam search on the device (Sec. 4: decoding is a batched beam search that runs on the GPU, beam
// size 12; Listing 1: "output_prob" softmax over the labels, "output" chooses, "trg" embeds the choice):
//
//     cand[q, b, v] = score[q, b] + logits[r, v] - logsumexp(logits[r, :]),  r = q * beam + b
//     the `beam` largest candidates of sentence q, best first, equal ones by ascending b * V + v  -> score', src, label
//     state rows follow their hypotheses: out[q * beam + k] = in[q * beam + src[q, k]]
//     trg[r] = W_trg[label[r]] + b_trg
//
// No candidate list of beam * V entries is ever sorted: a sentence's best `beam` candidates contain at most `beam` from one
// row, so every row first picks its own best `beam` labels out of a copy of the row in LDS (beam_row_kernel), and one small
// work-group per sentence merges the beam * beam survivors (beam_merge_kernel).  Nothing returns to the host.
#include <algorithm>

#include "../../include/lstm_abi.h"
#include "common.h"

namespace lstm {
namespace {

constexpr int kBeamMax = 16;
constexpr int kVocabMax = 32768;      // a row of logits must fit into LDS as floats (128 KiB)

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
// best candidate of the work-group (256 lanes); every lane receives it.  `slot` = 4 entries of LDS scratch.
__device__ __forceinline__ Cand block_best(Cand c, Cand* slot) {
  c = wave_best(c);
  __syncthreads();                                              // the previous round's readers are done with `slot`
  if ((threadIdx.x & 63) == 0) slot[threadIdx.x >> 6] = c;
  __syncthreads();
  return pick(pick(slot[0], slot[1]), pick(slot[2], slot[3]));
}

// Row r of the logits: logsumexp, then the row's best `beam` labels, each found as the best entry that comes after the
// previous pick in the order above (so nothing has to be marked or removed).  Writes cand_val[r][k] = score[r] +
// logits[r][label] - logsumexp and cand_lab[r][k] = label.  Dynamic LDS: V floats.
__global__ __launch_bounds__(256) void beam_row_kernel(const float* __restrict__ logits, long ld, const float* __restrict__ score,
                                                        float* __restrict__ cand_val, int* __restrict__ cand_lab, int V, int beam) {
  extern __shared__ float row[];
  __shared__ Cand slot[4];
  __shared__ float fsum[4];
  const int r = blockIdx.x, tid = threadIdx.x;
  const float* src = logits + (long)r * ld;
  const Cand none = {-__builtin_inff(), 0x7fffffff};
  Cand best = none;
  for (int i = tid; i < V; i += 256) {
    const float x = src[i];
    row[i] = x;
    const Cand c = {x, i};
    best = pick(best, c);
  }
  best = block_best(best, slot);                                // also makes the whole row visible
  const float m = best.v;
  float z = 0.f;
  for (int i = tid; i < V; i += 256) z += __expf(row[i] - m);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) z += __shfl_xor(z, o);
  if ((tid & 63) == 0) fsum[tid >> 6] = z;
  __syncthreads();
  const float lse = m + __logf(fsum[0] + fsum[1] + fsum[2] + fsum[3]);
  const float sc = score[r];
  Cand prev = best;
  for (int k = 0; k < beam; ++k) {
    if (k > 0) {
      Cand c = none;
      for (int i = tid; i < V; i += 256) {
        const Cand x = {row[i], i};
        if (better(prev, x)) c = pick(c, x);                    // strictly after the previous pick
      }
      prev = block_best(c, slot);
    }
    if (tid == 0) {
      const bool found = prev.i < V;                             // fewer than `beam` labels in the row: the rest never wins
      cand_val[(long)r * beam + k] = found ? sc + (prev.v - lse) : -__builtin_inff();
      cand_lab[(long)r * beam + k] = found ? prev.i : 0;
    }
  }
}

// The beam * beam survivors of sentence q = blockIdx.x: the best `beam`, by value and then by flat index b * V + label.
__global__ __launch_bounds__(256) void beam_merge_kernel(const float* __restrict__ cand_val, const int* __restrict__ cand_lab,
                                                          float* __restrict__ score_out, int* __restrict__ src_out,
                                                          int* __restrict__ label_out, int V, int beam) {
  __shared__ Cand slot[4];
  const int q = blockIdx.x, tid = threadIdx.x;
  const Cand none = {-__builtin_inff(), 0x7fffffff};
  Cand mine = none;
  if (tid < beam * beam) {
    const int b = tid / beam;
    mine.v = cand_val[(long)q * beam * beam + tid];
    mine.i = b * V + cand_lab[(long)q * beam * beam + tid];
  }
  Cand prev = none;
  for (int k = 0; k < beam; ++k) {
    const bool eligible = k == 0 || better(prev, mine);
    prev = block_best(eligible ? mine : none, slot);
    if (tid == 0) {
      // with every hypothesis at -inf no candidate is "better" than another after the first pick: flat indices still are
      score_out[q * beam + k] = prev.v;
      src_out[q * beam + k] = prev.i == 0x7fffffff ? 0 : prev.i / V;
      label_out[q * beam + k] = prev.i == 0x7fffffff ? 0 : prev.i % V;
    }
  }
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

int lstm_beam_step(int Q, int beam, int V, const float* logits, int64_t ld, const float* score_in, float* score_out, int32_t* src,
                   int32_t* label, void* workspace, uint64_t workspace_bytes, void* stream) {
  if (!logits || !score_in || !score_out || !src || !label || !workspace) return LSTM_ERR_NULL;
  int rc = beam_dims(Q, beam, V);
  if (rc) return rc;
  if (ld < V) return LSTM_ERR_DIM;
  if (((uintptr_t)logits | (uintptr_t)score_in | (uintptr_t)score_out | (uintptr_t)src | (uintptr_t)label) & 3) return LSTM_ERR_ALIGN;
  uint64_t need = 0;
  lstm_beam_query(Q, beam, V, &need);
  if (workspace_bytes < need) return LSTM_ERR_SIZE;
  if (Q == 0) return LSTM_OK;
  if ((rc = device_ok())) return rc;
  hipStream_t st = (hipStream_t)stream;
  char* ws = (char*)(((uintptr_t)workspace + 255) / 256 * 256);
  float* cand_val = (float*)ws;
  int* cand_lab = (int*)(ws + ((size_t)Q * beam * beam * 4 + 255) / 256 * 256);
  static bool attr_set = false;
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)beam_row_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kVocabMax * 4) != hipSuccess) {
      (void)hipGetLastError();
      return LSTM_ERR_HIP;
    }
    attr_set = true;
  }
  hipLaunchKernelGGL(beam_row_kernel, dim3(Q * beam), dim3(256), (size_t)V * 4, st, logits, (long)ld, score_in, cand_val, cand_lab, V, beam);
  hipLaunchKernelGGL(beam_merge_kernel, dim3(Q), dim3(256), 0, st, cand_val, cand_lab, score_out, src, label, V, beam);
  if (hipGetLastError() != hipSuccess) return LSTM_ERR_HIP;
  return LSTM_OK;
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
