// Host side of the C ABI: argument validation, buffer planning and the launch sequences.
// No device code lives here.  Validation never touches the HIP runtime, so every argument error
// can be produced on a machine without a GPU.
#include "../../include/lstm_abi.h"
#include "common.h"

#include <string.h>
#include <stdlib.h>
#include <algorithm>
#include <vector>

namespace lstm {
namespace {

constexpr size_t kAlign = 256;
constexpr unsigned kSpinLimit = 1u << 20;   // polls before a single-launch kernel's wait gives up (about a second)
inline size_t up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct Plan {
  int T, B, n_in, n, D;
  bool bf16;
  size_t esz;
  int nkc_f, nkc_b, nrt, ntile_f, ntile_b;
  int nkc_ll_f, ntile16;                    // ring layout of the single-launch forward kernels
  // reserve: per direction [gates float T*B*4n][hprev storage T*B*n]
  size_t res_gates, res_hprev, res_dir_stride, reserve_bytes;
  // workspace
  size_t ws_Wf, ws_Wb, ws_hfrag0, ws_hfrag1, ws_dzfrag0, ws_dzfrag1, ws_hstate, ws_cstate, ws_Dh, ws_Dc, ws_DZ, ws_Zx,
      ws_colsum, ws_sync, sync_bytes, ws_WxT, ws_xpad, ws_XT, ws_DZT, ws_HT, ws_cidx, ws_fidx, ws_count, ws_Wcat, ws_Acat, ws_parts, workspace_bytes;
  int ks_dwx, ks_dwh, ks_dx;                // K ranges of the weight-gradient products and of dX (few output tiles: the whole device works on them)
  bool single_step, step_fused; int Kc, ksplit;         // T == 1 inference in bfloat16: the step is one product over [x | h], K cut in ksplit ranges
  bool fast_gemm; int n_in_pad; long TBp;   // bf16 products through the k-contiguous kernel (operands transposed once)
  size_t hfrag_bytes, dzfrag_bytes, DZ_dir_elems, Zx_dir_elems, Wf_bytes;
};

int make_plan(const lstm_desc* d, int bidir, Plan* p) {
  if (!d) return LSTM_ERR_NULL;
  if (d->T < 0 || d->B < 0 || d->n_in < 1 || d->n < 1) return LSTM_ERR_DIM;
  const long TB = (long)d->T * d->B;
  if (TB >= (1L << 31) || (long)d->n * 4 >= (1L << 29) || d->n_in >= (1 << 29) || d->B >= (1 << 24)) return LSTM_ERR_DIM;
  if (d->dtype != LSTM_F32 && d->dtype != LSTM_BF16_F32STATE) return LSTM_ERR_UNSUPPORTED;
  if (d->flags & ~(LSTM_FLAG_ACCUMULATE | LSTM_FLAG_PER_STEP | LSTM_FLAG_INFERENCE | LSTM_FLAG_WEIGHTS_PACKED | LSTM_FLAG_PLAIN_LAUNCH)) return LSTM_ERR_UNSUPPORTED;
  if (d->reserved != 0) return LSTM_ERR_UNSUPPORTED;
  p->T = d->T; p->B = d->B; p->n_in = d->n_in; p->n = d->n; p->D = bidir ? 2 : 1;
  p->bf16 = d->dtype == LSTM_BF16_F32STATE;
  p->esz = p->bf16 ? 2 : 4;
  const int KC = p->bf16 ? 32 : 16;                 // k covered by one fragment chunk index
  p->nkc_f = cdiv(d->n, KC);
  p->nkc_b = cdiv(4L * d->n, KC);
  p->nrt = 2 * cdiv(d->B > 0 ? d->B : 1, 32);       // 16-row tiles, two per work-group row block
  p->ntile_f = cdiv(d->n, 8);
  p->ntile_b = cdiv(d->n, 16);
  p->ntile16 = cdiv(d->n, 16);
  p->nkc_ll_f = ll_nkc(d->n, kLLSlotsFwd);
  const size_t n = d->n, D = p->D, B = d->B;
  const bool infer = d->flags & LSTM_FLAG_INFERENCE;
  p->res_gates = 0;
  p->res_hprev = up(TB * 4 * n * 4);
  p->res_dir_stride = p->res_hprev + up(TB * n * p->esz);
  p->reserve_bytes = D * p->res_dir_stride + kAlign;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += up(bytes); return at; };
  // error word, per-row-tile words, then one word per work-group of a single-launch kernel (its XCD)
  p->sync_bytes = up((64 + 2 * (size_t)p->nrt) * 4 + D * 2 * (size_t)p->nrt * cdiv(d->n, 32) * 4);
  p->ws_sync = take(p->sync_bytes);              // first, so that lstm_sync_status() finds it without a plan
  p->Wf_bytes = D * std::max((size_t)p->ntile_f * 2 * p->nkc_f, (size_t)p->ntile16 * 4 * p->nkc_ll_f) * 1024;
  p->ws_Wf = take(p->Wf_bytes + 1024);            // packed W_h, then one chunk of zeros
  const bool part = p->bf16 && d->n <= 1024;          // the partial-sum backward kernel may be chosen
  // float storage: the single-launch backward kernel (batches of up to 256 rows: its rings grow with B n^2 / 16)
  const bool part32 = !p->bf16 && d->n % 8 == 0 && d->n <= 1024 && d->B <= 256;
  p->ws_Wb = take(infer ? 0 : D * std::max({(size_t)p->ntile_b * p->nkc_b * 1024, part ? bwdp_wh_bytes(d->n) : (size_t)0,
                                            part32 ? bwd_f32_wh_bytes(d->n) : (size_t)0}));
  p->hfrag_bytes = D * p->nrt * (size_t)std::max(p->nkc_f, p->nkc_ll_f) * 1024;
  p->dzfrag_bytes = D * std::max({p->nrt * (size_t)p->nkc_b * 1024, part ? bwdp_ring_bytes(d->B, d->n) : (size_t)0,
                                  part32 ? bwd_f32_ring_bytes(d->B, d->n) : (size_t)0});
  p->ws_hfrag0 = take(p->hfrag_bytes);
  p->ws_hfrag1 = take(p->hfrag_bytes);
  p->ws_dzfrag0 = take(infer ? 0 : p->dzfrag_bytes);
  p->ws_dzfrag1 = take(infer ? 0 : p->dzfrag_bytes);
  p->ws_hstate = take(D * B * n * 4);
  p->ws_cstate = take(D * B * n * 4);
  p->ws_Dh = take(infer ? 0 : D * B * n * 4);
  p->ws_Dc = take(infer ? 0 : D * B * n * 4);
  p->DZ_dir_elems = up(TB * 4 * n * p->esz) / p->esz;
  p->ws_DZ = take(infer ? 0 : D * p->DZ_dir_elems * p->esz);
  p->Zx_dir_elems = up(TB * 4 * n * 4) / 4;
  // T == 1 inference, bfloat16: few output tiles, so K is cut into ranges that separate work-groups multiply (each at
  // least four 64-wide stages); their partial products lie side by side and the cell kernel adds them
  p->single_step = p->bf16 && d->n % 2 == 0 && infer && d->T == 1 && !(d->flags & LSTM_FLAG_PER_STEP);
  // k extent of the input projection: a multiple of 8 (16-byte rows), and for narrow inputs a multiple of 64 so that
  // the product runs through the kernel that loads straight into LDS (x is then copied into zero-padded rows)
  p->n_in_pad = d->n_in < 256 ? (d->n_in + 63) / 64 * 64 : (d->n_in + 7) / 8 * 8;
  // The step's product has few rows: a work-group of the skinny-row kernel walks the whole K and applies the cell in its
  // epilogue (B <= kSkinnyMaxRows); larger batches go through the throughput kernel, K cut into ranges whose partial
  // products lie side by side for the cell kernel to add.
  p->step_fused = p->single_step && d->B <= kSkinnyMaxRows;
  {
    const long tiles = (long)cdiv(B > 0 ? B : 1, 256) * cdiv(4L * d->n, 256) * p->D;
    const long stages = cdiv((long)p->n_in_pad + d->n, 64);
    p->ksplit = p->step_fused ? 1 : (int)std::max(1L, std::min(std::min(256 / tiles, stages / 4), 8L));
    p->Kc = cdiv((long)p->n_in_pad + d->n, 64L * p->ksplit) * 64 * p->ksplit;
  }
  p->ws_Zx = take(infer && !p->step_fused ? D * p->Zx_dir_elems * 4 * (p->single_step ? p->ksplit : 1) : 0);
  p->ws_colsum = take(infer ? 0 : D * 64 * 4 * n * 4);
  // transposed / padded operand copies for the fast bf16 products
  p->fast_gemm = p->bf16 && d->n % 2 == 0;
  p->TBp = (TB + 63) / 64 * 64;
  const bool fg = p->fast_gemm;
  p->ws_WxT = take(fg ? D * 4 * n * p->n_in_pad * 2 : 0);
  p->ws_xpad = take(fg && p->n_in_pad != d->n_in ? TB * p->n_in_pad * 2 : 0);
  p->ws_XT = take(fg && !infer ? (size_t)d->n_in * p->TBp * 2 : 0);
  p->ws_DZT = take(fg && !infer ? D * 4 * n * p->TBp * 2 : 0);
  p->ws_HT = take(fg && !infer ? D * n * p->TBp * 2 : 0);
  // frame map of the batch (which frames are real), used to leave padded frames out of the products
  const bool fm = fg || !p->bf16;             // (float storage: its product kernels take the same row maps)
  p->ws_cidx = take(fm ? (size_t)TB * 4 : 0);
  p->ws_fidx = take(fm ? (size_t)p->TBp * 4 : 0);
  p->ws_count = take(fm ? 256 : 0);
  p->ws_Wcat = take(p->single_step ? D * std::max((size_t)4 * n, wcell_rows(d->n)) * p->Kc * 2 : 0);
  p->ws_Acat = take(p->single_step ? D * B * p->Kc * 2 : 0);
  // weight-gradient products with few output tiles cut K into ranges whose partial results are summed afterwards
  const auto ksplit_for = [&](long M, long N) {
    const long tiles = (long)cdiv(M, 256) * cdiv(N, 256) * p->D;
    const long want = 256 / (tiles > 0 ? tiles : 1);
    const long most = p->TBp / 1024 > 0 ? p->TBp / 1024 : 1;        // every range keeps at least 16 stages of 64 frames
    return (int)std::max(1L, std::min(std::min(want, most), 8L));
  };
  // dX on a short batch has few output tiles too (rows = frames): K = 4n per direction cut into ranges of >= 16 stages
  {
    const long tiles = (long)cdiv(TB, 256) * cdiv(d->n_in, 256), stages = (long)p->D * cdiv(4L * d->n, 64);
    // (tiles counts the padded frames; about two thirds of them are real with the benchmarks' length mixes, and only those
    // rows' tiles do any work: 384 instead of 256 work-groups are aimed at.  Config 3: 160 tiles, 96 of them real, two
    // ranges instead of one: dX 1.44 -> 0.89 ms per step.)
    p->ks_dx = fg && !infer && p->bf16 && tiles > 0 ? (int)std::max(1L, std::min(std::min(384 / tiles, stages / 16), 8L)) : 1;
    // float storage: 128 x 128 tiles; with fewer than 512 of them each XCD takes an eighth of K for all tiles (gemm_float.hip)
    const long tiles_f = (long)cdiv(TB, 128) * cdiv(d->n_in, 128), stages_f = (long)p->D * cdiv(4L * d->n, 32);
    if (!p->bf16 && !infer && tiles_f > 0 && tiles_f < 512 && stages_f >= 64) p->ks_dx = 8;
  }
  p->ks_dwx = fg && !infer ? ksplit_for(d->n_in, 4L * d->n) : 1;
  p->ks_dwh = fg && !infer ? ksplit_for(d->n, 4L * d->n) : 1;
  p->ws_parts = take(std::max({p->ks_dwx > 1 ? D * p->ks_dwx * d->n_in * 4 * n * 4 : 0, p->ks_dwh > 1 ? D * p->ks_dwh * n * 4 * n * 4 : 0,
                               p->ks_dx > 1 ? (size_t)p->ks_dx * TB * d->n_in * 4 : 0}));
  p->workspace_bytes = o + kAlign;
  return LSTM_OK;
}

bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }

int widest(long ld_elems, long s1, long s2, size_t esz, int cap) {
  int v = cap;
  while (v > (int)esz && ((ld_elems * (long)esz) % v || (s1 * (long)esz) % v || (s2 * (long)esz) % v)) v >>= 1;
  return v;
}

int check_device() {                 // is the current device one this library is built for?  (looked up once per device)
  static std::atomic<unsigned long long> known_good{0};
  const hipError_t e = once_per_device(known_good, [] {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return hipErrorInvalidDevice;
    return strncmp(prop.gcnArchName, "gfx950", 6) == 0 ? hipSuccess : hipErrorInvalidDevice;
  });
  if (e != hipSuccess) { (void)hipGetLastError(); return LSTM_ERR_HIP; }
  return 0;
}

// ---- optional phase timing (hipEvents on the caller's stream) -----------------------------------
struct PhaseRec { int phase; long launches; hipEvent_t e0, e1; };
int g_profile = 0;              // 0 off, 1 recurrent loops and hoisted products, 2 every phase
std::vector<PhaseRec> g_recs;

struct Phase {
  int idx = -1;
  hipStream_t s;
  Phase(int phase, long launches, hipStream_t stream) : s(stream) {
    if (!g_profile) return;
    // (an event between two kernels leaves the device idle for some microseconds: the short set-up phases are
    // bracketed only on request)
    if (g_profile < 2 && (phase == LSTM_PHASE_PREP || phase == LSTM_PHASE_DB)) return;
    PhaseRec r{phase, launches, nullptr, nullptr};
    if (hipEventCreate(&r.e0) != hipSuccess || hipEventCreate(&r.e1) != hipSuccess) { (void)hipGetLastError(); return; }
    (void)hipEventRecord(r.e0, s);
    g_recs.push_back(r);
    idx = (int)g_recs.size() - 1;
  }
  ~Phase() { if (idx >= 0) (void)hipEventRecord(g_recs[idx].e1, s); }
};

#define HIPCHK(expr) do { if ((expr) != hipSuccess) { (void)hipGetLastError(); return LSTM_ERR_HIP; } } while (0)

int run_fwd(const lstm_desc* desc, int bidir, const void* x, const void* W_x, const void* W_h, const void* b,
            const void* h0, const void* c0, const int32_t* seq_lens, void* y, void* c, void* hT, void* cT, void* reserve,
            void* workspace, void* stream) {
  Plan p;
  int rc = make_plan(desc, bidir, &p);
  if (rc) return rc;
  if (!bidir && desc->direction != 1 && desc->direction != -1) return LSTM_ERR_DIRECTION;
  const bool infer = desc->flags & LSTM_FLAG_INFERENCE;
  if (!x || !W_x || !W_h || !y || !workspace) return LSTM_ERR_NULL;
  if (!infer && (!reserve || !c)) return LSTM_ERR_NULL;
  const void* ptrs[] = {x, W_x, W_h, b, h0, c0, seq_lens, y, c, hT, cT, reserve, workspace};
  for (const void* q : ptrs) if (misaligned(q)) return LSTM_ERR_ALIGN;
  if (desc->workspace_bytes < p.workspace_bytes) return LSTM_ERR_SIZE;
  if (!infer && desc->reserve_bytes < p.reserve_bytes) return LSTM_ERR_SIZE;
  if (p.B == 0) return LSTM_OK;
  if ((rc = check_device())) return rc;

  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)(((uintptr_t)workspace + kAlign - 1) / kAlign * kAlign);
  char* rs = reserve ? (char*)(((uintptr_t)reserve + kAlign - 1) / kAlign * kAlign) : nullptr;
  const size_t n = p.n, B = p.B, D = p.D, T = p.T;
  float* hstate = (float*)(ws + p.ws_hstate);
  float* cstate = (float*)(ws + p.ws_cstate);
  const size_t state_bytes = D * B * n * 4;

  if (p.single_step) {
    // the stepped cell: z = [x | h] [W_x ; W_h] + b as one product over all rows, then the cell update
    const long Kc = p.Kc;
    char* Wcat = ws + p.ws_Wcat;
    char* Acat = ws + p.ws_Acat;
    float* z = (float*)(ws + p.ws_Zx);
    {
      Phase ph(LSTM_PHASE_PREP, 2, s);
      if (!(desc->flags & LSTM_FLAG_WEIGHTS_PACKED)) {
        if (p.step_fused) HIPCHK(launch_pack_wcell(W_x, W_h, Wcat, p.n_in, p.n_in_pad, p.n, p.Kc, p.D, s));
        else HIPCHK(launch_pack_wcat(W_x, W_h, Wcat, p.n_in, p.n_in_pad, p.n, p.Kc, p.D, s));
      }
      HIPCHK(launch_concat_xh(x, (const float*)h0, Acat, p.B, p.n_in, p.n_in_pad, p.n, p.Kc, p.D, s));
    }
    if (p.step_fused) {                // product, bias, cell update and outputs in one kernel
      Phase ph(LSTM_PHASE_LOOP_FWD, 1, s);
      HIPCHK(launch_step_cell(Acat, Wcat, (const float*)b, (const float*)h0, (const float*)c0, (float*)hT, (float*)cT, y, (long)(D * n),
                              (float*)c, seq_lens, p.B, p.n, p.Kc, p.D, s));
      return LSTM_OK;
    }
    // batch index of the product = K range: A and B advance by Kr columns, C by one partial result
    const long Kr = Kc / p.ksplit, part = (long)p.Zx_dir_elems;
    {
      Phase ph(LSTM_PHASE_GEMM_ZX, (long)D, s);
      for (size_t d = 0; d < D; ++d) {
        GemmArgs g = {};
        g.A = Acat + d * B * Kc * 2; g.B = Wcat + d * (4 * n) * Kc * 2; g.C = z + d * p.ksplit * part;
        g.M = p.B; g.N = 4 * p.n; g.K = (int)Kr; g.lda = Kc; g.ldb = Kc; g.ldc = 4 * n;
        g.sAz = Kr; g.sBz = Kr; g.sCz = part; g.nz = p.ksplit; g.nseg = 1;
        g.a_kcontig = true; g.b_kcontig = true; g.in_bf16 = true; g.out_bf16 = false; g.vecA = 16; g.vecB = 16;
        HIPCHK(launch_gemm(g, s));
      }
    }
    {
      Phase ph(LSTM_PHASE_LOOP_FWD, 1, s);
      HIPCHK(launch_cell_step(z, part, p.ksplit, (const float*)b, (const float*)h0, (const float*)c0, (float*)hT, (float*)cT, y,
                              (long)(D * n), (float*)c, seq_lens, p.B, p.n, p.D, s));
    }
    return LSTM_OK;
  }
  bool frames_mapped = false;            // the frame map was written by the set-up launch
  {
    Phase ph(LSTM_PHASE_PREP, 5, s);
    ZeroRegions z;
    z.add(ws + p.ws_sync, p.sync_bytes);
    if (h0) HIPCHK(launch_copy(hstate, h0, state_bytes, s)); else z.add(hstate, state_bytes);
    if (c0) HIPCHK(launch_copy(cstate, c0, state_bytes, s)); else z.add(cstate, state_bytes);
    if (p.bf16 && !(desc->flags & LSTM_FLAG_PER_STEP) && T >= 2 && p.nkc_ll_f <= kLLMaxNkcFwd)
      z.add(ws + p.ws_Wf + p.Wf_bytes, 1024);              // the chunk of zeros behind the packed W_h (single-launch path)
    // (on the single-launch path the fills, the packed W_h and the initial ring are one launch)
    if (p.bf16 && !(desc->flags & LSTM_FLAG_PER_STEP) && T >= 2 && p.nkc_ll_f <= kLLMaxNkcFwd) {
      FrameMapArgs fm = {};
      if (p.fast_gemm && seq_lens) {   // the input projection below goes over the real frames
        fm = {seq_lens, p.T, p.B, (int*)(ws + p.ws_cidx), (int*)(ws + p.ws_fidx), (int*)(ws + p.ws_count)};
        frames_mapped = true;
      }
      HIPCHK(launch_prep_fwd_ll(z, W_h, (uint4*)(ws + p.ws_Wf), p.n, p.nkc_ll_f, p.D, (uint4*)(ws + p.ws_hfrag0), (uint4*)(ws + p.ws_hfrag1),
                                p.nrt, fm, s));
    } else HIPCHK(launch_fill_zero_many(z, s));
  }
  // single-launch path: bf16 storage, at least two steps, register budget of the kernel
  bool use_ll = p.bf16 && !(desc->flags & LSTM_FLAG_PER_STEP) && T >= 2 && p.nkc_ll_f <= kLLMaxNkcFwd;
  auto pack_fwd = [&]() -> int {            // the per-step kernels' order (also what a single-launch path that does not start falls back to)
    Phase ph(LSTM_PHASE_PREP, 2, s);
    HIPCHK(launch_pack_wh_fwd(W_h, (uint4*)(ws + p.ws_Wf), p.n, p.nkc_f, p.D, p.bf16, s));
    HIPCHK(launch_pack_state(hstate, (uint4*)(ws + p.ws_hfrag0), (uint4*)(ws + p.ws_hfrag1), p.B, p.n, p.nkc_f, p.nrt,
                             p.D, p.bf16, s));
    return LSTM_OK;
  };
  if (T > 0 && !use_ll) {
    if ((rc = pack_fwd())) return rc;
  }
  if (T > 0) {
    // hoisted input projection for all frames and both directions: Zx = X W_x + b
    float* gates = infer ? (float*)(ws + p.ws_Zx) : (float*)(rs + p.res_gates);
    const long gates_stride = infer ? (long)p.Zx_dir_elems : (long)(p.res_dir_stride / 4);
    GemmArgs g = {};
    g.A = x; g.B = W_x; g.C = gates; g.bias = (const float*)b;
    g.M = (int)(T * B); g.N = 4 * p.n; g.K = p.n_in;
    g.lda = p.n_in; g.ldb = 4 * n; g.ldc = 4 * n;
    g.sAz = 0; g.sBz = (long)p.n_in * 4 * n; g.sCz = gates_stride; g.sbiasz = 4 * n; g.nz = p.D;
    g.nseg = 1; g.a_kcontig = true; g.b_kcontig = false; g.in_bf16 = p.bf16; g.out_bf16 = false;
    g.vecA = widest(g.lda, 0, 0, p.esz, 16);
    g.vecB = widest(g.ldb, g.sBz, 0, p.esz, 4);
    {
      Phase ph(LSTM_PHASE_GEMM_ZX, 1, s);
      if (p.fast_gemm) {                 // W_x is transposed once so that both operands are k-contiguous
        HIPCHK(launch_transpose(W_x, ws + p.ws_WxT, p.n_in, 4 * p.n, 4 * n, p.n_in_pad, p.D, (long)p.n_in * 4 * n,
                                (long)(4 * n) * p.n_in_pad, nullptr, 1, 0, s));
        if (p.n_in_pad != p.n_in) {      // rows of x are not 16-byte aligned, or narrow: zero-padded copy
          HIPCHK(launch_pad_rows(x, ws + p.ws_xpad, (long)(T * B), p.n_in, p.n_in_pad, s));
          g.A = ws + p.ws_xpad;
        }
        g.B = ws + p.ws_WxT; g.K = p.n_in_pad; g.lda = p.n_in_pad; g.ldb = p.n_in_pad;
        g.sBz = (long)(4 * n) * p.n_in_pad; g.b_kcontig = true;
        if (seq_lens && gemm_nt_ok(g)) {
          // only real frames are projected: row r of the product is frame fidx[r]; the pre-activations of padded
          // frames stay unwritten and are never read
          int* fidx = (int*)(ws + p.ws_fidx);
          int* count = (int*)(ws + p.ws_count);
          if (!frames_mapped) HIPCHK(launch_frame_map(seq_lens, p.T, p.B, (int*)(ws + p.ws_cidx), fidx, count, s));
          g.a_rows = fidx; g.c_rows = fidx; g.a_phys_rows = g.M; g.m_dev = count;
        }
      } else if (!p.bf16 && seq_lens) {  // float storage: the same selection of real frames
        int* fidx = (int*)(ws + p.ws_fidx);
        int* count = (int*)(ws + p.ws_count);
        HIPCHK(launch_frame_map(seq_lens, p.T, p.B, (int*)(ws + p.ws_cidx), fidx, count, s));
        g.a_rows = fidx; g.c_rows = fidx; g.a_phys_rows = g.M; g.m_dev = count;
      }
      HIPCHK(launch_gemm(g, s));
    }

    bool done = false;
    if (use_ll) {
      PFwdArgs pa = {};
      pa.lens = seq_lens; pa.B = p.B; pa.n = p.n; pa.nkc = p.nkc_ll_f; pa.T = p.T; pa.ndir = p.D; pa.write_gates = infer ? 0 : 1;
      pa.plain_launch = (desc->flags & LSTM_FLAG_PLAIN_LAUNCH) != 0;
      pa.sync = (unsigned*)(ws + p.ws_sync); pa.spin_limit = kSpinLimit;
      pa.xcc = (unsigned*)(ws + p.ws_sync) + 64 + 2 * (size_t)p.nrt;
      const size_t frag_dir = (size_t)p.nrt * p.nkc_ll_f * 1024;
      for (size_t d = 0; d < D; ++d) {
        PFwdDir& fd = pa.d[d];
        fd.Wf = (const uint4*)(ws + p.ws_Wf + d * (size_t)p.ntile16 * 4 * p.nkc_ll_f * 1024);
        fd.Wzero = (const uint4*)(ws + p.ws_Wf + p.Wf_bytes);
        fd.ring0 = (uint4*)(ws + p.ws_hfrag0 + d * frag_dir);
        fd.ring1 = (uint4*)(ws + p.ws_hfrag1 + d * frag_dir);
        fd.gates = gates + d * gates_stride;
        fd.hstate = hstate + d * B * n;
        fd.cstate = cstate + d * B * n;
        fd.y = (char*)y + d * n * p.esz;
        fd.ldy = (long)(D * n);
        fd.cs = c ? (float*)c + d * T * B * n : nullptr;
        fd.hprev = infer ? nullptr : rs + d * p.res_dir_stride + p.res_hprev;
        fd.rev = bidir ? d == 1 : desc->direction == -1;
      }
      hipError_t e = hipErrorCooperativeLaunchTooLarge;
      if (persist_fwd_fits(pa)) {
        // The initial state does not travel through the exchange ring (what does must keep |h| <= 1): its product with W_h
        // goes into the pre-activations of every row's first frame, and the kernels start from zeros in the ring.
        if (h0) {
          Phase ph(LSTM_PHASE_PREP, 1, s);
          HIPCHK(launch_h0_term((const float*)h0, W_h, true, gates, gates_stride, seq_lens, p.T, p.B, p.n, p.D, pa.d[0].rev, pa.d[D - 1].rev, s));
        }
        Phase ph(LSTM_PHASE_LOOP_FWD, 1, s);
        e = launch_persist_fwd(pa, s);
        if (e == hipErrorCooperativeLaunchTooLarge && h0) e = hipErrorLaunchFailure;   // the pre-activations are no longer what the per-step path expects
      }
      if (e == hipSuccess) done = true;
      else if (e == hipErrorCooperativeLaunchTooLarge) {   // nothing was launched (does not fit on the device all at once): one launch per step
        (void)hipGetLastError();
        if ((rc = pack_fwd())) return rc;
      } else {                                      // a later batch slab failed after earlier ones ran: no second attempt on advanced state
        (void)hipGetLastError();
        return LSTM_ERR_HIP;
      }
    }
    // float storage: one launch for the whole time loop as well (the kernel works on the per-step path's packed W_h and
    // h buffers)
    if (!done && !p.bf16 && !(desc->flags & LSTM_FLAG_PER_STEP) && T >= 2 && p.n % 8 == 0) {
      PFwdArgs pa = {};
      pa.lens = seq_lens; pa.B = p.B; pa.n = p.n; pa.nkc = p.nkc_f; pa.T = p.T; pa.ndir = p.D; pa.write_gates = infer ? 0 : 1;
      pa.plain_launch = (desc->flags & LSTM_FLAG_PLAIN_LAUNCH) != 0;
      pa.sync = (unsigned*)(ws + p.ws_sync); pa.spin_limit = kSpinLimit;
      const size_t frag_dir = (size_t)p.nrt * p.nkc_f * 1024;
      for (size_t d = 0; d < D; ++d) {
        PFwdDir& fd = pa.d[d];
        fd.Wf = (const uint4*)(ws + p.ws_Wf + d * (size_t)p.ntile_f * 2 * p.nkc_f * 1024);
        fd.ring0 = (uint4*)(ws + p.ws_hfrag0 + d * frag_dir);
        fd.ring1 = (uint4*)(ws + p.ws_hfrag1 + d * frag_dir);
        fd.gates = gates + d * gates_stride;
        fd.hstate = hstate + d * B * n;
        fd.cstate = cstate + d * B * n;
        fd.y = (char*)y + d * n * p.esz;
        fd.ldy = (long)(D * n);
        fd.cs = c ? (float*)c + d * T * B * n : nullptr;
        fd.hprev = infer ? nullptr : rs + d * p.res_dir_stride + p.res_hprev;
        fd.rev = bidir ? d == 1 : desc->direction == -1;
      }
      hipError_t e = hipErrorCooperativeLaunchTooLarge;
      if (persist_fwd_f32_fits(pa)) {
        if (h0) {   // (as on the bfloat16 path: the initial state enters through the pre-activations of every row's first frame)
          Phase ph(LSTM_PHASE_PREP, 1, s);
          HIPCHK(launch_h0_term((const float*)h0, W_h, false, gates, gates_stride, seq_lens, p.T, p.B, p.n, p.D, pa.d[0].rev, pa.d[D - 1].rev, s));
        }
        Phase ph(LSTM_PHASE_LOOP_FWD, 1, s);
        e = launch_persist_fwd_f32(pa, s);
        if (e == hipErrorCooperativeLaunchTooLarge && h0) e = hipErrorLaunchFailure;   // the pre-activations are no longer what the per-step path expects
      }
      if (e == hipSuccess) done = true;
      else if (e == hipErrorCooperativeLaunchTooLarge) {   // nothing of the loop ran, but the h buffers may have been initialised for it
        (void)hipGetLastError();
        if ((rc = pack_fwd())) return rc;
      } else {
        (void)hipGetLastError();
        return LSTM_ERR_HIP;
      }
    }
    if (!done) {
    Phase ph(LSTM_PHASE_LOOP_FWD, (long)T, s);
    FwdArgs a = {};
    a.lens = seq_lens; a.B = p.B; a.n = p.n; a.nkc = p.nkc_f; a.T = p.T; a.ndir = p.D; a.write_gates = infer ? 0 : 1;
    const size_t frag_dir = (size_t)p.nrt * p.nkc_f * 1024;
    for (size_t tau = 0; tau < T; ++tau) {
      for (size_t d = 0; d < D; ++d) {
        const bool rev = bidir ? d == 1 : desc->direction == -1;
        const size_t t = rev ? T - 1 - tau : tau;
        FwdDir& fd = a.d[d];
        fd.Wf = (const uint4*)(ws + p.ws_Wf + d * (size_t)p.ntile_f * 2 * p.nkc_f * 1024);
        fd.hin = (const uint4*)(ws + ((tau & 1) ? p.ws_hfrag1 : p.ws_hfrag0) + d * frag_dir);
        fd.hout = ws + ((tau & 1) ? p.ws_hfrag0 : p.ws_hfrag1) + d * frag_dir;
        fd.gates = gates + d * gates_stride + t * B * 4 * n;
        fd.hstate = hstate + d * B * n;
        fd.cstate = cstate + d * B * n;
        fd.y = (char*)y + (t * B * D * n + d * n) * p.esz;
        fd.ldy = (long)(D * n);
        fd.cs = c ? (float*)c + (d * T + t) * B * n : nullptr;
        fd.hprev = infer ? nullptr : rs + d * p.res_dir_stride + p.res_hprev + t * B * n * p.esz;
        fd.t = (int)t;
      }
      HIPCHK(launch_step_fwd(a, p.bf16, s));
    }
    }
  }
  Phase ph(LSTM_PHASE_PREP, 2, s);
  if (hT) HIPCHK(launch_copy(hT, hstate, state_bytes, s));
  if (cT) HIPCHK(launch_copy(cT, cstate, state_bytes, s));
  return LSTM_OK;
}

int run_bwd(const lstm_desc* desc, int bidir, const void* x, const void* W_x, const void* W_h, const void* h0,
            const void* c0, const int32_t* seq_lens, const void* y, const void* c, const void* reserve, const void* dy,
            const void* dhT, const void* dcT, void* dx, void* dW_x, void* dW_h, void* db, void* dh0, void* dc0,
            void* workspace, void* stream) {
  Plan p;
  int rc = make_plan(desc, bidir, &p);
  if (rc) return rc;
  if (!bidir && desc->direction != 1 && desc->direction != -1) return LSTM_ERR_DIRECTION;
  if (desc->flags & LSTM_FLAG_INFERENCE) return LSTM_ERR_UNSUPPORTED;
  if (!x || !W_x || !W_h || !c || !reserve || !dy || !dW_x || !dW_h || !db || !workspace) return LSTM_ERR_NULL;
  const void* ptrs[] = {x, W_x, W_h, h0, c0, seq_lens, y, c, reserve, dy, dhT, dcT, dx, dW_x, dW_h, db, dh0, dc0, workspace};
  for (const void* q : ptrs) if (misaligned(q)) return LSTM_ERR_ALIGN;
  if (desc->workspace_bytes < p.workspace_bytes || desc->reserve_bytes < p.reserve_bytes) return LSTM_ERR_SIZE;
  if ((rc = check_device())) return rc;

  hipStream_t s = (hipStream_t)stream;
  char* ws = (char*)(((uintptr_t)workspace + kAlign - 1) / kAlign * kAlign);
  const char* rs = (const char*)(((uintptr_t)reserve + kAlign - 1) / kAlign * kAlign);
  const size_t n = p.n, B = p.B, D = p.D, T = p.T, n_in = p.n_in;
  const int acc = (desc->flags & LSTM_FLAG_ACCUMULATE) ? 1 : 0;
  float* Dh = (float*)(ws + p.ws_Dh);
  float* Dc = (float*)(ws + p.ws_Dc);
  const size_t state_bytes = D * B * n * 4;
  if (B > 0 && T == 0) HIPCHK(launch_fill_zero(ws + p.ws_sync, p.sync_bytes, s));
  if (B == 0 || T == 0) {          // no frames: parameter gradients are zero, state gradients pass through
    if (!acc) {
      HIPCHK(launch_fill_zero(dW_x, D * n_in * 4 * n * 4, s));
      HIPCHK(launch_fill_zero(dW_h, D * n * 4 * n * 4, s));
      HIPCHK(launch_fill_zero(db, D * 4 * n * 4, s));
    }
    if (B > 0) {
      if (dh0) { if (dhT) HIPCHK(launch_copy(dh0, dhT, state_bytes, s)); else HIPCHK(launch_fill_zero(dh0, state_bytes, s)); }
      if (dc0) { if (dcT) HIPCHK(launch_copy(dc0, dcT, state_bytes, s)); else HIPCHK(launch_fill_zero(dc0, state_bytes, s)); }
    }
    return LSTM_OK;
  }
  // With sequence lengths given, the products behind the loop run over the real frames only (about two thirds of T*B for
  // the length mix of speech batches): frames are numbered once, row-indexed products gather / scatter through
  // that numbering and the transposed operands of the weight gradients are packed by it.
  const int TB = (int)(T * B);
  const bool compact = (p.fast_gemm || !p.bf16) && seq_lens && TB > 0;
  // single-launch path: bf16 storage, at least two steps, and the kernel fits the device
  PBwdArgs pa = {};
  pa.lens = seq_lens; pa.B = p.B; pa.n = p.n; pa.T = p.T; pa.ndir = p.D;
  pa.plain_launch = (desc->flags & LSTM_FLAG_PLAIN_LAUNCH) != 0;
  pa.sync = (unsigned*)(ws + p.ws_sync); pa.spin_limit = kSpinLimit;
  pa.xcc = (unsigned*)(ws + p.ws_sync) + 64 + 2 * (size_t)p.nrt;
  for (size_t d = 0; d < D; ++d) pa.d[d].lddy = (long)(D * n);       // (the check looks at the frame sizes)
  const bool use_ll = p.bf16 && !(desc->flags & LSTM_FLAG_PER_STEP) && T >= 2 && persist_bwd_fits(pa);
  const bool use_ll32 = !p.bf16 && !(desc->flags & LSTM_FLAG_PER_STEP) && T >= 2 && p.n % 8 == 0 && p.n <= 1024 && p.B <= 256 &&
                        persist_bwd_f32_fits(pa);
  bool dx_cleared = false;
  {
    Phase ph(LSTM_PHASE_PREP, 5, s);
    ZeroRegions z;
    z.add(ws + p.ws_sync, p.sync_bytes);
    if (dhT) HIPCHK(launch_copy(Dh, dhT, state_bytes, s)); else z.add(Dh, state_bytes);
    if (dcT) HIPCHK(launch_copy(Dc, dcT, state_bytes, s)); else z.add(Dc, state_bytes);
    z.add(ws + p.ws_dzfrag0, p.dzfrag_bytes);
    z.add(ws + p.ws_dzfrag1, p.dzfrag_bytes);
    if (2 * p.nrt <= kColsumSlices) z.add(ws + p.ws_colsum, D * kColsumSlices * 4 * n * 4);   // bias-gradient slices of row groups the grid lacks
    // (the bfloat16 single-launch path clears and packs W_h^T in one launch)
    if (use_ll) {
      FrameMapArgs fm = {};
      if (compact) fm = {seq_lens, p.T, p.B, (int*)(ws + p.ws_cidx), (int*)(ws + p.ws_fidx), (int*)(ws + p.ws_count)};
      if (compact && dx && ((size_t)TB * n_in * p.esz) % 4 == 0) {   // dX is scattered to the real frames' rows: the padded frames' rows are cleared here
        z.add(dx, (size_t)TB * n_in * p.esz);
        dx_cleared = true;
      }
      HIPCHK(launch_prep_bwd_ll(z, W_h, (uint4*)(ws + p.ws_Wb), p.n, p.D, fm, s));
    } else HIPCHK(launch_fill_zero_many(z, s));
  }
  if (!use_ll) {
    Phase ph(LSTM_PHASE_PREP, 1, s);
    if (use_ll32) HIPCHK(launch_pack_wh_bwd_f32p(W_h, ws + p.ws_Wb, p.n, p.D, s));
    else HIPCHK(launch_pack_wh_bwd(W_h, (uint4*)(ws + p.ws_Wb), p.n, p.nkc_b, p.D, p.bf16, s));
  }

  const size_t frag_dir = (size_t)p.nrt * p.nkc_b * 1024;
  char* DZ = ws + p.ws_DZ;
  bool done = false;
  const bool db_in_loop = (use_ll || use_ll32) && 2 * p.nrt <= kColsumSlices;   // the single-launch kernels also sum the bias gradient
  if (use_ll || use_ll32) {
    const size_t ring_dir = use_ll ? bwdp_ring_bytes(p.B, p.n) : bwd_f32_ring_bytes(p.B, p.n);
    const size_t wb_dir = use_ll ? bwdp_wh_bytes(p.n) : bwd_f32_wh_bytes(p.n);
    for (size_t d = 0; d < D; ++d) {
      PBwdDir& bd = pa.d[d];
      bd.Wb = (const uint4*)(ws + p.ws_Wb + d * wb_dir);
      bd.ring0 = (uint4*)(ws + p.ws_dzfrag0 + d * ring_dir);
      bd.ring1 = (uint4*)(ws + p.ws_dzfrag1 + d * ring_dir);
      bd.gates = (const float*)(rs + d * p.res_dir_stride + p.res_gates);
      bd.cs = (const float*)c + d * T * B * n;
      bd.c0 = c0 ? (const float*)c0 + d * B * n : nullptr;
      bd.dy = (const char*)dy + d * n * p.esz;
      bd.lddy = (long)(D * n);
      bd.DZ = DZ + d * p.DZ_dir_elems * p.esz;
      bd.Dh = Dh + d * B * n;
      bd.Dc = Dc + d * B * n;
      bd.dbpart = db_in_loop ? (float*)(ws + p.ws_colsum) + d * kColsumSlices * 4 * n : nullptr;
      bd.rev = bidir ? d == 1 : desc->direction == -1;
    }
    hipError_t e;
    {
      Phase ph(LSTM_PHASE_LOOP_BWD, 1, s);
      e = use_ll ? launch_persist_bwd(pa, s) : launch_persist_bwd_f32(pa, s);
    }
    if (e == hipSuccess) done = true;
    else if (e != hipErrorCooperativeLaunchTooLarge) {   // a later batch slab failed after earlier ones ran
      (void)hipGetLastError();
      return LSTM_ERR_HIP;
    } else {
      (void)hipGetLastError();
      Phase ph(LSTM_PHASE_PREP, 1, s);
      HIPCHK(launch_pack_wh_bwd(W_h, (uint4*)(ws + p.ws_Wb), p.n, p.nkc_b, p.D, p.bf16, s));
    }
  }
  BwdArgs a = {};
  a.lens = seq_lens; a.B = p.B; a.n = p.n; a.nkc = p.nkc_b; a.T = p.T; a.ndir = p.D;
  if (!done) {
  Phase ph(LSTM_PHASE_LOOP_BWD, (long)T + 1, s);
  for (long tau = (long)T - 1; tau >= -1; --tau) {
    a.do_matmul = tau < (long)T - 1;
    a.do_pointwise = tau >= 0;
    for (size_t d = 0; d < D; ++d) {
      const bool rev = bidir ? d == 1 : desc->direction == -1;
      const long t = rev ? (long)T - 1 - tau : tau;            // frame of this step (out of range when tau == -1)
      const long t_next = rev ? t - 1 : t + 1;                 // frame of the previous backward step
      BwdDir& bd = a.d[d];
      bd.Wb = (const uint4*)(ws + p.ws_Wb + d * (size_t)p.ntile_b * p.nkc_b * 1024);
      bd.dzin = (const uint4*)(ws + (((tau + 1) & 1) ? p.ws_dzfrag1 : p.ws_dzfrag0) + d * frag_dir);
      bd.dzout = ws + ((tau & 1) ? p.ws_dzfrag1 : p.ws_dzfrag0) + d * frag_dir;
      bd.Dh = Dh + d * B * n;
      bd.Dc = Dc + d * B * n;
      bd.t = (int)t; bd.t_next = (int)t_next;
      if (tau >= 0) {
        const float* cs = (const float*)c + d * T * B * n;
        const long tp = rev ? t + 1 : t - 1;                   // frame processed just before t in the forward pass
        bd.gates = (const float*)(rs + d * p.res_dir_stride + p.res_gates) + t * B * 4 * n;
        bd.cs = cs + t * B * n;
        bd.cprev = (tp >= 0 && tp < (long)T) ? cs + tp * B * n : (c0 ? (const float*)c0 + d * B * n : nullptr);
        bd.dy = (const char*)dy + (t * B * D * n + d * n) * p.esz;
        bd.lddy = (long)(D * n);
        bd.DZ = DZ + (d * p.DZ_dir_elems + t * B * 4 * n) * p.esz;
      }
    }
    HIPCHK(launch_step_bwd(a, p.bf16, s));
  }
  }
  {
    Phase ph(LSTM_PHASE_PREP, 2, s);
    if (dh0) HIPCHK(launch_copy(dh0, Dh, state_bytes, s));
    if (dc0) HIPCHK(launch_copy(dc0, Dc, state_bytes, s));
  }

  int* cidx = (int*)(ws + p.ws_cidx);
  int* fidx = (int*)(ws + p.ws_fidx);
  int* count = (int*)(ws + p.ws_count);
  const auto fits = [](long rows, long ld) { return rows * ld * 2 <= 0x7fffff00L; };
  const bool compact_w = compact && fits(p.n_in, p.TBp) && fits(4L * p.n, p.TBp) && fits(p.n, p.TBp);
  if (compact && !use_ll) {          // (the bfloat16 single-launch path numbered the frames in its set-up launch)
    Phase ph(LSTM_PHASE_PREP, 1, s);
    HIPCHK(launch_frame_map(seq_lens, p.T, p.B, cidx, fidx, count, s));
  }
  if (dx) {                        // dX = sum over directions of DZ W_x^T
    GemmArgs g = {};
    g.A = DZ; g.B = W_x; g.C = dx;
    g.M = TB; g.N = p.n_in; g.K = 4 * p.n;
    g.lda = 4 * n; g.ldb = 4 * n; g.ldc = n_in; g.nz = 1;
    g.nseg = p.D; g.sAseg = (long)p.DZ_dir_elems; g.sBseg = (long)(n_in * 4 * n);
    g.a_kcontig = true; g.b_kcontig = true; g.in_bf16 = p.bf16; g.out_bf16 = p.bf16;
    g.vecA = widest(g.lda, g.sAseg, 0, p.esz, 16);
    g.vecB = widest(g.ldb, g.sBseg, 0, p.esz, 16);
    Phase ph(LSTM_PHASE_GEMM_DX, 1, s);
    if (compact && (gemm_nt_ok(g) || !p.bf16)) {      // rows of padded frames: zero, and left out of the product
      if (!dx_cleared) HIPCHK(launch_fill_zero(dx, (size_t)TB * n_in * p.esz, s));
      g.a_rows = fidx; g.c_rows = fidx; g.a_phys_rows = TB; g.m_dev = count;
    }
    if (p.ks_dx > 1 && gemm_nt_ok(g)) { g.ksplit = p.ks_dx; g.parts = (float*)(ws + p.ws_parts); }
    if (!p.bf16 && p.ks_dx == 8) {
      g.ksplit = 8; g.parts = (float*)(ws + p.ws_parts);
      if (!gemm_float_ok(g)) { g.ksplit = 0; g.parts = nullptr; }
    }
    if (!p.bf16 && !g.parts) {
      // float storage, shapes the eight-range form above does not take: rows = frames and n_in columns give few 128 x 128 tiles (config 2: 85 with real
      // frames), so K = 4n per direction is cut into ranges that add their parts to the zero-filled dx atomically
      const long tiles = (long)cdiv(TB, 128) * cdiv(p.n_in, 128), stages = (long)p.D * cdiv(4L * p.n, 32);
      const int ks = (int)std::max(1L, std::min(std::min(384 / std::max(tiles, 1L), stages / 16), 8L));
      if (ks > 1) {
        if (!compact) HIPCHK(launch_fill_zero(dx, (size_t)TB * n_in * p.esz, s));
        g.ksplit = ks;
      }
    }
    HIPCHK(launch_gemm(g, s));
  }
  // Weight gradients straight from the frame-major tensors (a row per frame in X, Hprev and DZ: both operands of
  // X^T DZ are k-major), over the packed list of real frames when lengths are given.
  auto frame_major = [&](const void* A, long lda, long sAz, int M, void* C, int ks) {
    GemmArgs g = {};
    g.A = A; g.B = DZ; g.C = C;
    g.M = M; g.N = 4 * p.n; g.K = (int)TB; g.lda = lda; g.ldb = 4 * n; g.ldc = 4 * n;
    g.sAz = sAz; g.sBz = (long)p.DZ_dir_elems; g.sCz = (long)M * 4 * n; g.nz = p.D; g.nseg = 1;
    g.a_kcontig = false; g.b_kcontig = false; g.in_bf16 = true; g.out_bf16 = false; g.accumulate = acc;
    g.vecA = 16; g.vecB = 16;
    if (compact) { g.k_rows = fidx; g.k_phys_rows = (int)TB; g.k_dev = count; }
    if (ks > 1) { g.ksplit = ks; g.parts = (float*)(ws + p.ws_parts); }
    return g;
  };
  const GemmArgs gx = frame_major(x, n_in, 0, p.n_in, dW_x, p.ks_dwx);
  const GemmArgs gh = frame_major(rs + p.res_hprev, n, (long)(p.res_dir_stride / 2), p.n, dW_h, p.ks_dwh);
  if (p.fast_gemm && (!seq_lens || compact) && gemm_tn_ok(gx) && gemm_tn_ok(gh)) {
    {
      Phase ph(LSTM_PHASE_GEMM_DWX, 1, s);
      HIPCHK(launch_gemm(gx, s));
    }
    {
      Phase ph(LSTM_PHASE_GEMM_DWH, 1, s);
      HIPCHK(launch_gemm(gh, s));
    }
  } else if (p.fast_gemm) {        // operands transposed once: everything k-contiguous
    const long TBp = p.TBp;
    {
      Phase ph(LSTM_PHASE_GEMM_DWX, 3, s);
      const int* cmap = compact_w ? cidx : nullptr;
      HIPCHK(launch_transpose(DZ, ws + p.ws_DZT, TB, 4 * p.n, 4 * n, TBp, p.D, (long)p.DZ_dir_elems, (long)(4 * n) * TBp,
                              nullptr, 1, 0, s, cmap, fidx, count));
      HIPCHK(launch_transpose(x, ws + p.ws_XT, TB, p.n_in, n_in, TBp, 1, 0, 0, seq_lens, p.B, p.T, s, cmap, fidx, count));
      GemmArgs g = {};
      g.A = ws + p.ws_XT; g.B = ws + p.ws_DZT; g.C = dW_x;
      g.M = p.n_in; g.N = 4 * p.n; g.K = (int)TBp; g.lda = TBp; g.ldb = TBp; g.ldc = 4 * n;
      g.sAz = 0; g.sBz = (long)(4 * n) * TBp; g.sCz = (long)(n_in * 4 * n); g.nz = p.D; g.nseg = 1;
      g.a_kcontig = true; g.b_kcontig = true; g.in_bf16 = true; g.out_bf16 = false; g.accumulate = acc;
      g.vecA = 16; g.vecB = 16;
      if (compact_w) g.k_dev = count + 1;
      if (gemm_nt_ok(g) && p.ks_dwx > 1) { g.ksplit = p.ks_dwx; g.parts = (float*)(ws + p.ws_parts); }
      HIPCHK(launch_gemm(g, s));
    }
    {
      Phase ph(LSTM_PHASE_GEMM_DWH, 2, s);
      HIPCHK(launch_transpose(rs + p.res_hprev, ws + p.ws_HT, TB, p.n, n, TBp, p.D, (long)(p.res_dir_stride / 2), (long)n * TBp,
                              nullptr, 1, 0, s, compact_w ? cidx : nullptr, fidx, count));
      GemmArgs g = {};
      g.A = ws + p.ws_HT; g.B = ws + p.ws_DZT; g.C = dW_h;
      g.M = p.n; g.N = 4 * p.n; g.K = (int)TBp; g.lda = TBp; g.ldb = TBp; g.ldc = 4 * n;
      g.sAz = (long)n * TBp; g.sBz = (long)(4 * n) * TBp; g.sCz = (long)(n * 4 * n); g.nz = p.D; g.nseg = 1;
      g.a_kcontig = true; g.b_kcontig = true; g.in_bf16 = true; g.out_bf16 = false; g.accumulate = acc;
      g.vecA = 16; g.vecB = 16;
      if (compact_w) g.k_dev = count + 1;
      if (gemm_nt_ok(g) && p.ks_dwh > 1) { g.ksplit = p.ks_dwh; g.parts = (float*)(ws + p.ws_parts); }
      HIPCHK(launch_gemm(g, s));
    }
  } else {                         // dW_x = X^T DZ, padded frames of X masked out
    GemmArgs g = {};
    g.A = x; g.B = DZ; g.C = dW_x;
    g.M = p.n_in; g.N = 4 * p.n; g.K = TB;
    g.lda = n_in; g.ldb = 4 * n; g.ldc = 4 * n;
    g.sAz = 0; g.sBz = (long)p.DZ_dir_elems; g.sCz = (long)(n_in * 4 * n); g.nz = p.D; g.nseg = 1;
    g.a_kcontig = false; g.b_kcontig = false; g.in_bf16 = p.bf16; g.out_bf16 = false; g.accumulate = acc;
    if (compact) { g.k_rows = fidx; g.k_phys_rows = (int)TB; g.k_dev = count; }   // the real frames only
    else { g.lens = seq_lens; g.Bt = p.B; g.T = p.T; }                              // (or every frame, padded ones read as zero)
    g.vecA = widest(g.lda, 0, 0, p.esz, 4);
    g.vecB = widest(g.ldb, g.sBz, 0, p.esz, 4);
    {
      Phase ph(LSTM_PHASE_GEMM_DWX, 1, s);
      HIPCHK(launch_gemm(g, s));
    }
    // dW_h = Hprev^T DZ
    g.A = rs + p.res_hprev; g.C = dW_h; g.M = p.n; g.lda = n;
    g.sAz = (long)(p.res_dir_stride / p.esz); g.sCz = (long)(n * 4 * n);
    g.lens = nullptr;
    g.vecA = widest(g.lda, g.sAz, 0, p.esz, 4);
    Phase ph(LSTM_PHASE_GEMM_DWH, 1, s);
    HIPCHK(launch_gemm(g, s));
  }
  Phase ph(LSTM_PHASE_DB, 2, s);
  if (done && db_in_loop) {
    HIPCHK(launch_colsum_final((const float*)(ws + p.ws_colsum), (float*)db, 4 * p.n, p.D, 2 * p.nrt, acc, s));
    return LSTM_OK;
  }
  HIPCHK(launch_colsum(DZ, (float*)db, (float*)(ws + p.ws_colsum), TB, 4 * p.n, p.D, (long)p.DZ_dir_elems, p.bf16, acc, s));
  return LSTM_OK;
}

}  // namespace
int device_ok() { return check_device(); }
}  // namespace lstm

extern "C" {

int lstm_query(const lstm_desc* desc, int bidirectional, size_t* reserve_bytes, size_t* workspace_bytes) {
  lstm::Plan p;
  int rc = lstm::make_plan(desc, bidirectional, &p);
  if (rc) return rc;
  if (!reserve_bytes || !workspace_bytes) return LSTM_ERR_NULL;
  *reserve_bytes = (desc->flags & LSTM_FLAG_INFERENCE) ? 0 : p.reserve_bytes;
  *workspace_bytes = p.workspace_bytes;
  return LSTM_OK;
}

int lstm_fwd(const lstm_desc* desc, const void* x, const void* W_x, const void* W_h, const void* b, const void* h0,
             const void* c0, const int32_t* seq_lens, void* y, void* c, void* hT, void* cT, void* reserve, void* workspace,
             void* stream) {
  return lstm::run_fwd(desc, 0, x, W_x, W_h, b, h0, c0, seq_lens, y, c, hT, cT, reserve, workspace, stream);
}
int blstm_fwd(const lstm_desc* desc, const void* x, const void* W_x, const void* W_h, const void* b, const void* h0,
              const void* c0, const int32_t* seq_lens, void* y, void* c, void* hT, void* cT, void* reserve, void* workspace,
              void* stream) {
  return lstm::run_fwd(desc, 1, x, W_x, W_h, b, h0, c0, seq_lens, y, c, hT, cT, reserve, workspace, stream);
}
int lstm_bwd(const lstm_desc* desc, const void* x, const void* W_x, const void* W_h, const void* h0, const void* c0,
             const int32_t* seq_lens, const void* y, const void* c, const void* reserve, const void* dy, const void* dhT,
             const void* dcT, void* dx, void* dW_x, void* dW_h, void* db, void* dh0, void* dc0, void* workspace,
             void* stream) {
  return lstm::run_bwd(desc, 0, x, W_x, W_h, h0, c0, seq_lens, y, c, reserve, dy, dhT, dcT, dx, dW_x, dW_h, db, dh0, dc0,
                       workspace, stream);
}
int blstm_bwd(const lstm_desc* desc, const void* x, const void* W_x, const void* W_h, const void* h0, const void* c0,
              const int32_t* seq_lens, const void* y, const void* c, const void* reserve, const void* dy, const void* dhT,
              const void* dcT, void* dx, void* dW_x, void* dW_h, void* db, void* dh0, void* dc0, void* workspace,
              void* stream) {
  return lstm::run_bwd(desc, 1, x, W_x, W_h, h0, c0, seq_lens, y, c, reserve, dy, dhT, dcT, dx, dW_x, dW_h, db, dh0, dc0,
                       workspace, stream);
}

int lstm_gemm(int in_bf16, int out_bf16, int a_kcontig, int b_kcontig, int M, int N, int K, const void* A, int64_t lda,
              const void* B, int64_t ldb, void* C, int64_t ldc, const float* bias, int accumulate, const int32_t* lens,
              int Bt, int T, void* stream) {
  using namespace lstm;
  if (!A || !B || !C) return LSTM_ERR_NULL;
  if (M < 0 || N < 0 || K < 0 || lda < 1 || ldb < 1 || ldc < 1) return LSTM_ERR_DIM;
  if ((out_bf16 && !in_bf16) || (!a_kcontig && b_kcontig) || (lens && (a_kcontig || Bt < 1)) || (accumulate && out_bf16))
    return LSTM_ERR_UNSUPPORTED;
  const size_t esz = in_bf16 ? 2 : 4;
  if (((uintptr_t)A | (uintptr_t)B) & (esz - 1) || ((uintptr_t)C & (out_bf16 ? 1 : 3))) return LSTM_ERR_ALIGN;
  int rc = check_device();
  if (rc) return rc;
  GemmArgs g = {};
  g.A = A; g.B = B; g.C = C; g.bias = bias; g.M = M; g.N = N; g.K = K; g.lda = lda; g.ldb = ldb; g.ldc = ldc;
  g.nz = 1; g.nseg = 1; g.a_kcontig = a_kcontig; g.b_kcontig = b_kcontig; g.in_bf16 = in_bf16; g.out_bf16 = out_bf16;
  g.accumulate = accumulate; g.lens = lens; g.Bt = Bt; g.T = T;
  auto ptr_vec = [&](const void* p, int cap) { int v = cap; while (v > (int)esz && ((uintptr_t)p % v)) v >>= 1; return v; };
  g.vecA = std::min(widest(lda, 0, 0, esz, a_kcontig ? 16 : 4), ptr_vec(A, a_kcontig ? 16 : 4));
  g.vecB = std::min(widest(ldb, 0, 0, esz, b_kcontig ? 16 : 4), ptr_vec(B, b_kcontig ? 16 : 4));
  if (launch_gemm(g, (hipStream_t)stream) != hipSuccess) { (void)hipGetLastError(); return LSTM_ERR_HIP; }
  return LSTM_OK;
}

static int pool_args(int dtype, int T, int B, int F, int pool, const void* a, int64_t lda, const void* o, int64_t ldo) {
  if (!a || !o) return LSTM_ERR_NULL;
  if (T < 0 || B < 0 || F < 1 || pool < 1 || pool > 255 || lda < F || ldo < F || B > 65535) return LSTM_ERR_DIM;
  if (dtype != LSTM_F32 && dtype != LSTM_BF16_F32STATE) return LSTM_ERR_UNSUPPORTED;
  const uintptr_t mask = dtype == LSTM_F32 ? 3 : 1;
  if (((uintptr_t)a | (uintptr_t)o) & mask) return LSTM_ERR_ALIGN;
  return LSTM_OK;
}

int lstm_time_pool_fwd(int dtype, int T, int B, int F, int pool, const void* y, int64_t ldy, const int32_t* seq_lens, void* out,
                       int64_t ldo, uint8_t* arg, int32_t* lens_out, void* stream) {
  int rc = pool_args(dtype, T, B, F, pool, y, ldy, out, ldo);
  if (rc) return rc;
  if ((rc = lstm::check_device())) return rc;
  if (lstm::launch_time_pool_fwd(dtype == LSTM_BF16_F32STATE, y, ldy, seq_lens, out, ldo, arg, lens_out, T, B, F, pool,
                                 (hipStream_t)stream) != hipSuccess) {
    (void)hipGetLastError();
    return LSTM_ERR_HIP;
  }
  return LSTM_OK;
}

int lstm_time_pool_bwd(int dtype, int T, int B, int F, int pool, const void* dout, int64_t ldo, const uint8_t* arg,
                       const int32_t* seq_lens, void* dy, int64_t ldy, void* stream) {
  int rc = pool_args(dtype, T, B, F, pool, dout, ldo, dy, ldy);
  if (rc) return rc;
  if (!arg) return LSTM_ERR_NULL;
  if ((rc = lstm::check_device())) return rc;
  if (lstm::launch_time_pool_bwd(dtype == LSTM_BF16_F32STATE, dout, ldo, arg, seq_lens, dy, ldy, T, B, F, pool,
                                 (hipStream_t)stream) != hipSuccess) {
    (void)hipGetLastError();
    return LSTM_ERR_HIP;
  }
  return LSTM_OK;
}

int lstm_sync_status(const void* workspace, int32_t* timed_out) {
  if (!workspace || !timed_out) return LSTM_ERR_NULL;
  const char* ws = (const char*)(((uintptr_t)workspace + lstm::kAlign - 1) / lstm::kAlign * lstm::kAlign);
  uint32_t word = 0;
  if (hipMemcpy(&word, ws, 4, hipMemcpyDeviceToHost) != hipSuccess) { (void)hipGetLastError(); return LSTM_ERR_HIP; }
  *timed_out = word != 0;
  return LSTM_OK;
}

int lstm_profile_enable(int on) {
  lstm::g_profile = on < 0 ? 0 : on > 2 ? 2 : on;
  return LSTM_OK;
}
int lstm_profile_read(double* ms, int64_t* launches) {
  if (!ms || !launches) return LSTM_ERR_NULL;
  int rc = LSTM_OK;
  for (auto& r : lstm::g_recs) {
    float t = 0.f;
    if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&t, r.e0, r.e1) != hipSuccess) {
      (void)hipGetLastError();
      rc = LSTM_ERR_HIP;
    } else {
      ms[r.phase] += t;
      launches[r.phase] += r.launches;
    }
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  lstm::g_recs.clear();
  return rc;
}

const char* lstm_strerror(int status) {
  switch (status) {
    case LSTM_OK: return "ok";
    case LSTM_ERR_NULL: return "a required pointer is NULL";
    case LSTM_ERR_DIM: return "bad dimension";
    case LSTM_ERR_DIRECTION: return "direction must be +1 or -1";
    case LSTM_ERR_UNSUPPORTED: return "unsupported dtype or flag";
    case LSTM_ERR_ALIGN: return "pointer is not 16-byte aligned";
    case LSTM_ERR_SIZE: return "reserve or workspace too small (see lstm_query)";
    case LSTM_ERR_HIP: return "HIP runtime error or device is not gfx950";
    default: return "unknown status";
  }
}

}  // extern "C"
