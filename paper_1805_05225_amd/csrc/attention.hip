// One step of the attention decoder between the stepped LSTM cell and the readout (Listing 1, sub-network of layer
// "output": "s_tr", "weight_feedback", "e_in", "e_tanh", "e", "a", "accum_a", "att", "readout"):
//
//     s_tr[r]   = s[r] W_s + b_s                                       one product over all rows (MFMA)
//     e[r, j]   = v . tanh(ctx[j, q(r)] + accum[r, j] w_fb + b_fb + s_tr[r]) + b_e      att_energy_kernel (vector ALU)
//     a[r, :]   = softmax of e[r, :] over j < src_lens[q(r)],  accum' = accum + a        att_context_kernel (its first part)
//     att[r]    = sum_j a[r, j] H[j, q(r)]                                               att_context_kernel (reads H once per sentence)
//     readout   = max(0, [s, trg, att] W_r + b_r)                      one product + bias_relu_kernel
//
// q(r) = r / beam: the hypotheses of a sentence are neighbours in the decoder batch, so one work-group serves all of
// them from a single read of the sentence's ctx / H rows.  Storage: ctx, H, s, att, readout bfloat16; s_tr, e, a, accum
// float; all arithmetic float.
#include <algorithm>

#include "../../include/lstm_abi.h"
#include "common.h"
#include "recurrent_dev.h"
#include <type_traits>

namespace lstm {
namespace {

constexpr int kMaxBeam = 16;          // hypotheses per sentence (register budget of the energy kernel)
constexpr int kMaxS = 1024;           // source positions: beam x S weights sit in LDS
constexpr int kJB = 2;                // source positions per work-group of the energy kernel (measured: 1: 31 us, 2: 27, 4: 29, 8: 41)
constexpr int kPartStride = 260;      // floats per partial-sum row in LDS: 4 * value + slot hits 64 different banks

__device__ __forceinline__ int src_len(const int* lens, int q, int S) {
  if (!lens) return S;
  const int L = lens[q];
  return L < 0 ? 0 : (L > S ? S : L);
}

// e[r][j] for the rows of sentence q = blockIdx.y and the kJB positions from blockIdx.x * kJB.  A lane owns the
// attention features k = lane, lane + 256, ...: it loads ctx[j][q][k] once and uses it for every hypothesis of the
// sentence.  The beam x kJB partial sums of the 256 lanes are added through LDS.
__global__ __launch_bounds__(256) void att_energy_kernel(const uint16_t* __restrict__ ctx, const float* __restrict__ s_tr,
                                                          const float* __restrict__ accum, const float* __restrict__ w_fb,
                                                          const float* __restrict__ b_fb, const float* __restrict__ v, float b_e,
                                                          const int* __restrict__ lens, float* __restrict__ e, int S, int Q, int beam,
                                                          int A) {
  __shared__ float part[32 * kPartStride];                     // 32 (hypothesis, position) pairs at a time
  const int q = blockIdx.y, j0 = blockIdx.x * kJB, tid = threadIdx.x;
  const int L = src_len(lens, q, S);
  if (j0 >= L) return;
  const int nj = min(kJB, L - j0);
  // tanh(x) = 1 - 2 / (1 + 2^(x * 2 log2 e)): with every addend of x scaled by 2 log2 e beforehand an element costs
  // multiply-add, add, exp2, add, reciprocal, multiply-add; the "1" of every term is added once per lane (vsum).
  constexpr float kScale = 2.8853900817779268f;                // 2 log2(e)
  float sum[kMaxBeam][kJB];
#pragma unroll
  for (int r = 0; r < kMaxBeam; ++r)
#pragma unroll
    for (int j = 0; j < kJB; ++j) sum[r][j] = 0.f;
  float vsum = 0.f;
  // the accumulated weights of the beam x kJB (row, position) pairs: the same for every lane and every k
  float ac[kMaxBeam][kJB];
#pragma unroll
  for (int r = 0; r < kMaxBeam; ++r)
#pragma unroll
    for (int j = 0; j < kJB; ++j) ac[r][j] = (r < beam && j < nj) ? accum[((long)q * beam + r) * S + j0 + j] : 0.f;
  for (int k = tid; k < A; k += 256) {
    // every load of this k goes out before the first use: inside the uniform branches below each would be waited for
    // on its own, one L2 latency per hypothesis (measured: 47 -> 30 us).  Fetching the next k's operands ahead of
    // this k's arithmetic as well measured no faster.
    float c[kJB], st[kMaxBeam];
#pragma unroll
    for (int j = 0; j < kJB; ++j) c[j] = bf_bits2f(ctx[((long)(j0 + min(j, nj - 1)) * Q + q) * A + k]);
#pragma unroll
    for (int r = 0; r < kMaxBeam; ++r) st[r] = s_tr[((long)q * beam + min(r, beam - 1)) * A + k];
    const float bf = b_fb[k], wf = kScale * w_fb[k], vk = v[k], m2v = -2.f * vk;
#pragma unroll
    for (int j = 0; j < kJB; ++j) c[j] = kScale * (c[j] + bf);
    vsum += vk;
#pragma unroll
    for (int r = 0; r < kMaxBeam; ++r) {
      if (r < beam) {                                          // uniform: a scalar branch
        const float s2 = kScale * st[r];
#pragma unroll
        for (int j = 0; j < kJB; ++j) {
          const float x2 = __builtin_fmaf(ac[r][j], wf, c[j]) + s2;
          sum[r][j] = __builtin_fmaf(__builtin_amdgcn_rcpf(__builtin_amdgcn_exp2f(x2) + 1.f), m2v, sum[r][j]);
        }
      }
    }
  }
#pragma unroll
  for (int r = 0; r < kMaxBeam; ++r)
#pragma unroll
    for (int j = 0; j < kJB; ++j) sum[r][j] += vsum;
  // the partial sums of 32 (hypothesis, position) pairs at a time: kRows hypotheses x kJB positions
  constexpr int kRows = 32 / kJB < kMaxBeam ? 32 / kJB : kMaxBeam;
#pragma unroll
  for (int grp = 0; grp < kMaxBeam / kRows; ++grp) {
    if (grp * kRows >= beam) break;
    if (grp) __syncthreads();                                   // the previous group has been read
#pragma unroll
    for (int rr = 0; rr < kRows; ++rr)
      if (grp * kRows + rr < beam) {
#pragma unroll
        for (int j = 0; j < kJB; ++j) part[(rr * kJB + j) * kPartStride + tid] = sum[grp * kRows + rr][j];
      }
    __syncthreads();
    // value `vid` (= rr * kJB + j) is added up by four lanes, each taking every fourth of the 256 partial sums
    const int vid = tid >> 2, sub = tid & 3;
    const int r = grp * kRows + vid / kJB, j = vid % kJB;
    const bool live = vid < kRows * kJB && r < beam;
    float t = 0.f;
    if (live) {
      for (int i = 0; i < 64; ++i) t += part[vid * kPartStride + 4 * i + sub];
    }
    t += __shfl_xor(t, 1);
    t += __shfl_xor(t, 2);
    if (sub == 0 && live && j < nj) e[((long)q * beam + r) * S + j0 + j] = t + b_e;
  }
}

// a[r, :] = softmax of e[r, :] over the valid positions, accum' = accum + a, and att[r] = sum_j a[r][j] H[j][q], for
// the hypotheses of sentence q = blockIdx.y and the 128 features from blockIdx.x * 128.  Every work-group of a sentence
// works the softmax out for itself (beam x S exponentials from one round of loads: cheaper than a launch of its own and
// a pass through memory); the one with blockIdx.x == 0 writes a and accum'.  Softmax: 16 lanes per hypothesis, e staged
// in LDS.  Context: lane l of every wavefront owns features 2l, 2l + 1 of the slice, the four wavefronts share the
// source positions (wavefront w takes j = w, w + 4, ...), kU loads in flight per lane, and their partial sums meet in
// LDS.  H is read once for all hypotheses of the sentence.  Dynamic LDS: S * kMaxBeam floats, w[j][r] (rows r >= beam
// up to the next multiple of 4 hold zeros).
__global__ __launch_bounds__(256) void att_context_kernel(const uint16_t* __restrict__ H, const float* __restrict__ e,
                                                           const float* __restrict__ accum_in, const int* __restrict__ lens,
                                                           float* __restrict__ a_out, float* __restrict__ accum_out,
                                                           uint16_t* __restrict__ att, long ldatt, int S, int Q, int beam, int E) {
  extern __shared__ float w[];
  __shared__ float red[3][kMaxBeam * 2][64];
  const int q = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int L = src_len(lens, q, S);
  const int nb4 = (beam + 3) >> 2;                              // groups of four hypotheses
  {
    const int r = tid >> 4, l = tid & 15;                       // beam <= 16: one group of 16 lanes per hypothesis
    const long row = (long)q * beam + r;
    float m = -3.0e38f;
    if (r < beam) {
      for (int j = l; j < L; j += 16) {
        const float ev = e[row * S + j];
        w[j * kMaxBeam + r] = ev;
        m = fmaxf(m, ev);
      }
    } else if (r < nb4 * 4) {
      for (int j = l; j < L; j += 16) w[j * kMaxBeam + r] = 0.f;
    }
    // a lane reads back only what it wrote itself until the weights are complete
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if (r < beam) {
      float z = 0.f;
      for (int j = l; j < L; j += 16) {
        const float p = __expf(w[j * kMaxBeam + r] - m);
        w[j * kMaxBeam + r] = p;
        z += p;
      }
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) z += __shfl_xor(z, o);
      const float inv = L > 0 ? 1.f / z : 0.f;
      for (int j = l; j < L; j += 16) w[j * kMaxBeam + r] *= inv;
      if (blockIdx.x == 0) {
        for (int j = l; j < S; j += 16) {
          const float p = j < L ? w[j * kMaxBeam + r] : 0.f;
          if (a_out) a_out[row * S + j] = p;
          accum_out[row * S + j] = j < L ? accum_in[row * S + j] + p : 0.f;
        }
      }
    }
  }
  __syncthreads();
  const int f = (blockIdx.x * 64 + lane) * 2;
  const bool live = f < E;
  float acc[kMaxBeam][2];
#pragma unroll
  for (int r = 0; r < kMaxBeam; ++r) acc[r][0] = acc[r][1] = 0.f;
  const uint16_t* Hq = H + (long)q * E + (live ? f : 0);        // E even, rows 4-byte aligned
  const long jstride = (long)Q * E;
  constexpr int kU = 8;
  for (int j = wave; j < L; j += 4 * kU) {
    unsigned hh[kU];
#pragma unroll
    for (int u = 0; u < kU; ++u) hh[u] = *(const unsigned*)(Hq + min(j + 4 * u, L - 1) * jstride);
#pragma unroll
    for (int u = 0; u < kU; ++u) {
      if (j + 4 * u >= L) break;                                // uniform within the wavefront
      const float h0 = __uint_as_float(hh[u] << 16), h1 = __uint_as_float(hh[u] & 0xffff0000u);
      const float4* wj = (const float4*)(w + (j + 4 * u) * kMaxBeam);
#pragma unroll
      for (int g = 0; g < kMaxBeam / 4; ++g)
        if (g < nb4) {                                          // uniform
          const float4 p = wj[g];
          acc[4 * g + 0][0] += p.x * h0; acc[4 * g + 0][1] += p.x * h1;
          acc[4 * g + 1][0] += p.y * h0; acc[4 * g + 1][1] += p.y * h1;
          acc[4 * g + 2][0] += p.z * h0; acc[4 * g + 2][1] += p.z * h1;
          acc[4 * g + 3][0] += p.w * h0; acc[4 * g + 3][1] += p.w * h1;
        }
    }
  }
  if (wave > 0) {
#pragma unroll
    for (int r = 0; r < kMaxBeam; ++r)
      if (r < beam) { red[wave - 1][2 * r][lane] = acc[r][0]; red[wave - 1][2 * r + 1][lane] = acc[r][1]; }
  }
  __syncthreads();
  if (wave > 0 || !live) return;
#pragma unroll
  for (int r = 0; r < kMaxBeam; ++r)
    if (r < beam) {
      const float s0 = acc[r][0] + red[0][2 * r][lane] + red[1][2 * r][lane] + red[2][2 * r][lane];
      const float s1 = acc[r][1] + red[0][2 * r + 1][lane] + red[1][2 * r + 1][lane] + red[2][2 * r + 1][lane];
      const unsigned o = (unsigned)f2bf_bits(s0) | ((unsigned)f2bf_bits(s1) << 16);
      *(unsigned*)(att + ((long)q * beam + r) * ldatt + f) = o;
    }
}

// out = bfloat16(max(0, z)) for a float z[M][N] that already holds product + bias
__global__ void relu_bf16_kernel(const float* __restrict__ z, uint16_t* __restrict__ out, int M, int N, long ldo) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)M * N) return;
  const int m = (int)(idx / N), n = (int)(idx % N);
  out[(long)m * ldo + n] = f2bf_bits(fmaxf(z[idx], 0.f));
}

// cat[r] = [s[r] | trg[r] | att[r] | zeros up to ldc]: the three inputs of the readout side by side (16-bit elements, any
// row strides)
// V elements per thread (V = 4: 8-byte accesses, when every piece starts and ends on a multiple of 4 elements and all
// rows are 8-byte aligned; K .. ldc-1 is then the zero padding, ldc a multiple of 8).
template <int V>
__global__ void concat3_kernel(const uint16_t* __restrict__ x0, long ld0, int k0, const uint16_t* __restrict__ x1, long ld1, int k1,
                               const uint16_t* __restrict__ x2, long ld2, int k2, uint16_t* __restrict__ cat, long ldc, int B) {
  typedef typename std::conditional<V == 4, uint2, uint16_t>::type vec_t;
  const int K = k0 + k1 + k2;                                  // columns K .. ldc-1 of cat are padding: zeros
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x, per_row = ldc / V;
  if (idx >= (long)B * per_row) return;
  const int r = (int)(idx / per_row), k = (int)(idx % per_row) * V;
  const uint16_t* src = k < k0 ? x0 + (long)r * ld0 + k : (k < k0 + k1 ? x1 + (long)r * ld1 + k - k0 : x2 + (long)r * ld2 + k - k0 - k1);
  vec_t v = {};
  if (k < K) v = *(const vec_t*)src;
  *(vec_t*)(cat + (long)r * ldc + k) = v;
}
hipError_t launch_concat3(const uint16_t* x0, long ld0, int k0, const uint16_t* x1, long ld1, int k1, const uint16_t* x2, long ld2, int k2,
                          uint16_t* cat, long ldc, int B, hipStream_t s) {
  const bool v4 = ((k0 | k1 | k2 | (int)(ld0 & 3) | (int)(ld1 & 3) | (int)(ld2 & 3) | (int)(ldc & 3)) & 3) == 0 &&
                  ((((uintptr_t)x0) | ((uintptr_t)x1) | ((uintptr_t)x2) | ((uintptr_t)cat)) & 7) == 0;
  if (v4) {
    const long total = (long)B * (ldc / 4);
    hipLaunchKernelGGL(concat3_kernel<4>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, x0, ld0, k0, x1, ld1, k1, x2, ld2, k2, cat, ldc, B);
  } else {
    const long total = (long)B * ldc;
    hipLaunchKernelGGL(concat3_kernel<1>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, x0, ld0, k0, x1, ld1, k1, x2, ld2, k2, cat, ldc, B);
  }
  return hipGetLastError();
}

inline size_t up256(size_t x) { return (x + 255) / 256 * 256; }

// C[M][N] float = A[M][lda] (bf16) . W[N][ldw]^T (bf16, a row per output) + bias, K cut into ranges when the product has
// few output tiles; `parts` holds ksplit * M * N floats.
hipError_t linear_rows(const void* A, long lda, const void* W, long ldw, const float* bias, float* C, int M, int N, int K, float* parts,
                       int ksplit, hipStream_t s) {
  GemmArgs g = {};
  g.A = A; g.B = W; g.C = C; g.bias = bias; g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldw; g.ldc = N;
  g.nz = 1; g.nseg = 1; g.a_kcontig = true; g.b_kcontig = true; g.in_bf16 = true; g.out_bf16 = false;
  const auto vec = [](const void* p, long ld) { int v = 16; while (v > 2 && (((uintptr_t)p % v) || ((ld * 2) % v))) v >>= 1; return v; };
  g.vecA = vec(A, lda); g.vecB = vec(W, ldw);
  if (gemm_skinny_ok(g)) return launch_gemm_skinny(g, false, s);       // few rows: one work-group per tile walks the whole K
  if (ksplit > 1 && gemm_nt_ok(g)) { g.ksplit = ksplit; g.parts = parts; }
  return launch_gemm(g, s);
}
int ranges_for(int M, int N, int K) {
  const long tiles = (long)((M + 255) / 256) * ((N + 255) / 256), stages = (K + 63) / 64;
  return (int)std::max(1L, std::min(std::min(256 / std::max(tiles, 1L), stages / 4), 8L));
}

}  // namespace
}  // namespace lstm

using namespace lstm;

extern "C" {

static int att_check(const lstm_att_desc* d) {
  if (!d) return LSTM_ERR_NULL;
  if (d->S < 1 || d->Q < 0 || d->beam < 1 || d->A < 1 || d->E < 2 || d->n < 1 || d->Q > 65535 || (long)d->Q * d->beam > 0x7fffffffL / d->S)
    return LSTM_ERR_DIM;
  if (d->beam > kMaxBeam || d->S > kMaxS || (d->E & 1)) return LSTM_ERR_UNSUPPORTED;
  return LSTM_OK;
}

int lstm_attention_query(const lstm_att_desc* d, uint64_t* workspace_bytes) {
  int rc = att_check(d);
  if (rc) return rc;
  if (!workspace_bytes) return LSTM_ERR_NULL;
  const size_t B = (size_t)d->Q * d->beam;
  const int ks = ranges_for((int)B, d->A, d->n);
  *workspace_bytes = 256 + up256(B * d->A * 4) + up256(B * d->S * 4) + (ks > 1 ? up256((size_t)ks * B * d->A * 4) : 0) + up256(B * d->S * 4);
  return LSTM_OK;
}

int lstm_attention_step(const lstm_att_desc* d, const void* enc, const void* enc_ctx, const int32_t* src_lens, const void* s, int64_t ld_s,
                        const void* W_s, const float* b_s, const float* w_fb, const float* b_fb, const float* v, float b_e,
                        const float* accum_in, float* accum_out, float* a, void* att, int64_t ld_att, void* workspace, void* stream) {
  int rc = att_check(d);
  if (rc) return rc;
  if (!enc || !enc_ctx || !s || !W_s || !b_s || !w_fb || !b_fb || !v || !accum_in || !accum_out || !att || !workspace) return LSTM_ERR_NULL;
  if (ld_s < d->n || ld_att < d->E) return LSTM_ERR_DIM;
  if ((ld_att & 1) || ((uintptr_t)att & 3) || ((uintptr_t)enc & 3) || ((uintptr_t)enc_ctx & 1) || ((uintptr_t)s & 1) || ((uintptr_t)W_s & 1) ||
      (((uintptr_t)b_s | (uintptr_t)w_fb | (uintptr_t)b_fb | (uintptr_t)v | (uintptr_t)accum_in | (uintptr_t)accum_out | (uintptr_t)a) & 3))
    return LSTM_ERR_ALIGN;
  uint64_t need = 0;
  lstm_attention_query(d, &need);
  if (d->workspace_bytes < need) return LSTM_ERR_SIZE;
  if (d->Q == 0) return LSTM_OK;
  if ((rc = device_ok())) return rc;
  hipStream_t st = (hipStream_t)stream;
  const int B = d->Q * d->beam;
  char* ws = (char*)(((uintptr_t)workspace + 255) / 256 * 256);
  float* s_tr = (float*)ws;
  float* e = (float*)(ws + up256((size_t)B * d->A * 4));
  float* parts = (float*)(ws + up256((size_t)B * d->A * 4) + up256((size_t)B * d->S * 4));
  const int ks = ranges_for(B, d->A, d->n);
  if (linear_rows(s, ld_s, W_s, d->n, b_s, s_tr, B, d->A, d->n, parts, ks, st) != hipSuccess) { (void)hipGetLastError(); return LSTM_ERR_HIP; }
  hipLaunchKernelGGL(att_energy_kernel, dim3((d->S + kJB - 1) / kJB, d->Q), dim3(256), 0, st, (const uint16_t*)enc_ctx, s_tr, accum_in, w_fb,
                     b_fb, v, b_e, src_lens, e, d->S, d->Q, d->beam, d->A);
  static std::atomic<unsigned long long> attr_set{0};            // S = 1024 needs 64 KiB of dynamic LDS beside the static arrays
  if (once_per_device(attr_set, [] {
        return hipFuncSetAttribute((const void*)att_context_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, kMaxS * kMaxBeam * 4);
      }) != hipSuccess) {
    (void)hipGetLastError();
    return LSTM_ERR_HIP;
  }
  hipLaunchKernelGGL(att_context_kernel, dim3((d->E / 2 + 63) / 64, d->Q), dim3(256), (size_t)d->S * kMaxBeam * 4, st, (const uint16_t*)enc,
                     e, accum_in, src_lens, a, accum_out, (uint16_t*)att, (long)ld_att, d->S, d->Q, d->beam, d->E);
  if (hipGetLastError() != hipSuccess) return LSTM_ERR_HIP;
  return LSTM_OK;
}

static int readout_dims(int B, int R, int n, int n_trg, int E) {
  if (B < 0 || R < 1 || n < 1 || n_trg < 0 || E < 0 || (long)n + n_trg + E > 0x7fffff || (long)B * R > 0x7fffffffL ||
      (long)B * ((long)n + n_trg + E) > 0x7fffffffL)
    return LSTM_ERR_DIM;
  return LSTM_OK;
}
static long readout_kpad(int n, int n_trg, int E) { return ((long)n + n_trg + E + 7) / 8 * 8; }     // rows of whole 16-byte chunks

int lstm_readout_query(int B, int R, int n, int n_trg, int E, uint64_t* workspace_bytes) {
  if (!workspace_bytes) return LSTM_ERR_NULL;
  const int rc = readout_dims(B, R, n, n_trg, E);
  if (rc) return rc;
  const long Kp = readout_kpad(n, n_trg, E);
  const int ks = ranges_for(B, R, (int)Kp);
  *workspace_bytes = 256 + up256((size_t)R * Kp * 2) + up256((size_t)B * Kp * 2) + up256((size_t)B * R * 4) +
                     (ks > 1 ? up256((size_t)ks * B * R * 4) : 0);
  return LSTM_OK;
}

int lstm_readout(int flags, int B, int R, const void* s, int64_t ld_s, int n, const void* trg, int64_t ld_trg, int n_trg, const void* att,
                 int64_t ld_att, int E, const void* W_r, const float* b_r, void* out, int64_t ld_out, void* workspace,
                 uint64_t workspace_bytes, void* stream) {
  if (!s || (!trg && n_trg > 0) || (!att && E > 0) || !W_r || !out || !workspace) return LSTM_ERR_NULL;
  if (flags & ~LSTM_FLAG_WEIGHTS_PACKED) return LSTM_ERR_UNSUPPORTED;
  int rc = readout_dims(B, R, n, n_trg, E);
  if (rc) return rc;
  if (ld_s < n || ld_trg < n_trg || ld_att < E || ld_out < R) return LSTM_ERR_DIM;
  if ((((uintptr_t)s | (uintptr_t)trg | (uintptr_t)att | (uintptr_t)W_r | (uintptr_t)out) & 1) || ((uintptr_t)b_r & 3)) return LSTM_ERR_ALIGN;
  uint64_t need = 0;
  lstm_readout_query(B, R, n, n_trg, E, &need);
  if (workspace_bytes < need) return LSTM_ERR_SIZE;
  if (B == 0) return LSTM_OK;
  if ((rc = device_ok())) return rc;
  hipStream_t st = (hipStream_t)stream;
  const int K = n + n_trg + E;
  const long Kp = readout_kpad(n, n_trg, E);
  char* ws = (char*)(((uintptr_t)workspace + 255) / 256 * 256);
  // workspace: W_r with its rows padded with zeros to whole 16-byte chunks (kept between calls under
  // LSTM_FLAG_WEIGHTS_PACKED), the concatenated inputs padded the same way, the float product, the K ranges' parts
  uint16_t* Wp = (uint16_t*)ws;
  uint16_t* cat = (uint16_t*)(ws + up256((size_t)R * Kp * 2));
  float* z = (float*)((char*)cat + up256((size_t)B * Kp * 2));
  float* parts = (float*)((char*)z + up256((size_t)B * R * 4));
  if (!(flags & LSTM_FLAG_WEIGHTS_PACKED) && launch_pad_rows(W_r, Wp, R, K, (int)Kp, st) != hipSuccess) { (void)hipGetLastError(); return LSTM_ERR_HIP; }
  if (launch_concat3((const uint16_t*)s, (long)ld_s, n, (const uint16_t*)trg, (long)ld_trg, n_trg, (const uint16_t*)att, (long)ld_att, E, cat,
                     Kp, B, st) != hipSuccess) { (void)hipGetLastError(); return LSTM_ERR_HIP; }
  {                                  // few rows: bias, max(0, .) and the rounding happen in the product's epilogue
    GemmArgs g = {};
    g.A = cat; g.B = Wp; g.C = out; g.bias = b_r; g.M = B; g.N = R; g.K = (int)Kp; g.lda = Kp; g.ldb = Kp; g.ldc = ld_out;
    g.nz = 1; g.nseg = 1; g.a_kcontig = true; g.b_kcontig = true; g.in_bf16 = true; g.out_bf16 = true; g.vecA = 16; g.vecB = 16;
    if (gemm_skinny_ok(g)) {
      if (launch_gemm_skinny(g, true, st) != hipSuccess) { (void)hipGetLastError(); return LSTM_ERR_HIP; }
      return LSTM_OK;
    }
  }
  if (linear_rows(cat, Kp, Wp, Kp, b_r, z, B, R, (int)Kp, parts, ranges_for(B, R, (int)Kp), st) != hipSuccess) { (void)hipGetLastError(); return LSTM_ERR_HIP; }
  const long total = (long)B * R;
  hipLaunchKernelGGL(relu_bf16_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, z, (uint16_t*)out, B, R, (long)ld_out);
  if (hipGetLastError() != hipSuccess) return LSTM_ERR_HIP;
  return LSTM_OK;
}

}  // extern "C"
