// Internal declarations shared by the translation units of the library (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>

namespace lstm {

typedef __bf16 bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// round-to-nearest-even float -> bf16 bits, NaN kept quiet
__device__ __forceinline__ uint16_t f2bf_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf_bits2f(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// Storage-type helpers: T is float or bf16_t.
template <typename T> struct Store;
template <> struct Store<float> {
  static constexpr int kBytes = 4;
  static constexpr int kPerChunk = 4;                      // elements in a 16-byte chunk
  __device__ static float load(const void* p, long i) { return ((const float*)p)[i]; }
  __device__ static void store(void* p, long i, float v) { ((float*)p)[i] = v; }
};
template <> struct Store<bf16_t> {
  static constexpr int kBytes = 2;
  static constexpr int kPerChunk = 8;
  __device__ static float load(const void* p, long i) { return bf_bits2f(((const uint16_t*)p)[i]); }
  __device__ static void store(void* p, long i, float v) { ((uint16_t*)p)[i] = f2bf_bits(v); }
};

// ------------------------------------------------------------------------------------------
// Hoisted GEMM:  C[m,n] (+)= sum_seg sum_k A(m,k) B(k,n) + bias[n]
//   a_kcontig: A is stored [M][lda] (k contiguous); otherwise [K][lda] (m contiguous).
//   b_kcontig: B is stored [N][ldb] (k contiguous); otherwise [K][ldb] (n contiguous).
// blockIdx.z batches independent problems (pointer strides s*z, in elements).
// nseg > 1 sums over several (A,B) pairs (strides s*seg): used to add both directions' dX.
// lens != NULL masks rows of the K axis: row k is a frame (t = k / Bt, b = k % Bt) and is read
// as zero unless t < lens[b]  (so values stored at padded frames never enter dW_x).
struct GemmArgs {
  const void* A; const void* B; void* C; const float* bias;
  int M, N, K;
  long lda, ldb, ldc;
  long sAz, sBz, sCz, sbiasz;
  int nz;
  int nseg; long sAseg, sBseg;
  int vecA, vecB;            // widest aligned access (bytes) usable on A / B: 16, 8, 4 or 2
  int accumulate;            // C += result (float C only)
  const int* lens; int Bt; int T;
  bool a_kcontig, b_kcontig;
  bool in_bf16, out_bf16;
  // Row maps (the fast kernels and the generic one; not the few-rows kernel, and not together with `parts` or ksplit there):
  const int* a_rows; const int* c_rows;   // k-contiguous A: logical row r of A / C lives at physical row a_rows[r] / c_rows[r]
  int a_phys_rows;                        // rows of A in memory when a_rows is given
  const int* m_dev; const int* k_dev;     // M / K read from device memory (capped by M / K above, which size the grid)
  const int* k_rows; int k_phys_rows;     // both operands k-major: k -> row of A and of B in memory; rows each holds in memory
  int ksplit;                             // > 1: K cut into that many ranges whose parts are ADDED to C atomically
                                          // (float C, nseg == 1; C must hold zeros or the value to add to) ...
  float* parts;                           // ... or, if not NULL (nz * ksplit * M * ldc floats, no c_rows): every range stores
                                          // its part there and a second kernel writes C (+)= their sum (`accumulate` honoured)
};
hipError_t launch_gemm(const GemmArgs& g, hipStream_t s);
// Fast bfloat16 kernel for problems with both operands k-contiguous, 16-byte aligned rows and K % 8 == 0
// (launch_gemm routes such problems to it by itself).
bool gemm_nt_ok(const GemmArgs& g);
hipError_t launch_gemm_nt(const GemmArgs& g, hipStream_t s);
// Fast bfloat16 kernel for the opposite storage: both operands k-major (A[K][lda], B[K][ldb], 16-byte aligned rows),
// float C.  Row k of both operands is row k_rows[k] in memory if k_rows is given (launch_gemm routes to it by itself).
bool gemm_tn_ok(const GemmArgs& g);
hipError_t launch_gemm_tn(const GemmArgs& g, hipStream_t s);
// Float storage (gemm_float.hip): operands as they lie in memory, rows 16-byte aligned, extents along 16-byte chunks
// multiples of 4 (K for a k-contiguous operand, M / N for a k-major one); row maps, device-resident M / K, segments
// and atomic K ranges as above (launch_gemm routes to it by itself; what it does not take goes to the generic kernel).
bool gemm_float_ok(const GemmArgs& g);
hipError_t launch_gemm_float(const GemmArgs& g, hipStream_t s);
// Products with few rows (gemm_skinny.hip): both operands k-contiguous bfloat16 with 16-byte aligned rows, K % 8 == 0,
// M <= kSkinnyMaxRows, one segment, no row maps, no K ranges: a work-group owns 96 x 128 of C for the whole K, so bias,
// max(0, .) and the rounding to bfloat16 happen in its epilogue (launch_gemm routes such problems to it by itself).
constexpr int kSkinnyMaxRows = 1024;
bool gemm_skinny_ok(const GemmArgs& g);
hipError_t launch_gemm_skinny(const GemmArgs& g, bool relu, hipStream_t s);
// dst[c][r] = src[r][c] (16-bit elements), r < R, c < C, dst rows zero-padded up to ld_dst; nz problems with
// strides s_src / s_dst.  lens != NULL: rows of src are frames (t = r / Bt, b = r % Bt) and are read as zero
// unless t < lens[b].  With cidx / fidx / count from launch_frame_map the kept frames are packed instead: column
// cidx[r] receives row r, padded frames are dropped, and columns count[0] .. count[1]-1 are zeroed (ld_dst must
// then be a multiple of 64).
hipError_t launch_transpose(const void* src, void* dst, int R, int C, long ld_src, long ld_dst, int nz, long s_src, long s_dst,
                            const int* lens, int Bt, int T, hipStream_t s, const int* cidx = nullptr, const int* fidx = nullptr,
                            const int* count = nullptr);
// Numbers the frames (t, b) with t < lens[b] in (t, b) order: cidx[T*B] frame -> number or -1, fidx[number] -> frame,
// count[0] = how many, count[1] = that rounded up to a multiple of 64.
hipError_t launch_frame_map(const int* lens, int T, int B, int* cidx, int* fidx, int* count, hipStream_t s);
// dst[r][0..ld_dst) = src[r][0..C) followed by zeros (16-bit elements)
hipError_t launch_pad_rows(const void* src, void* dst, long R, int C, int ld_dst, hipStream_t s);

// ------------------------------------------------------------------------------------------
// Recurrent part.  Fragment geometry of the 16x16 MFMA used by the step kernels: a 16-byte chunk
// per lane holds kPerChunk consecutive k; lane = g*16 + r with r the row (A) or column (B) inside
// a 16-wide tile and g in 0..3; one chunk index kc covers KC = 4*kPerChunk values of k:
//   k = kc*KC + g*kPerChunk + e.
struct FwdDir {
  const uint4* Wf;    // packed W_h: [unit tile of 8][2 column tiles][nkc][64] chunks
  const uint4* hin;   // h entering the step, fragment order: [row tile of 16][nkc][64] chunks
  void* hout;         // h leaving the step, same layout
  float* gates;       // frame slab [B][4n]: in = x W_x + b, out = activations i|f|g|o
  float* hstate;      // [B][n] float running state
  float* cstate;
  void* y; long ldy;  // row b of this frame's output at y + b*ldy (storage type)
  float* cs;          // frame slab [B][n] or NULL
  void* hprev;        // frame slab [B][n] (storage type) or NULL
  int t;              // frame index of this step
};
struct FwdArgs {
  FwdDir d[2];
  const int* lens;
  int B, n, nkc, T, ndir, write_gates;
};
hipError_t launch_step_fwd(const FwdArgs& a, bool bf16, hipStream_t s);

struct BwdDir {
  const uint4* Wb;    // packed W_h^T: [unit tile of 16][nkc][64] chunks, k runs over the 4n gate columns
  const uint4* dzin;  // dz of the previous backward step, fragment order [row tile][nkc][64]
  void* dzout;
  const float* gates; // frame slab [B][4n] activations
  const float* cs;    // frame slab [B][n]: cell state after this frame
  const float* cprev; // [B][n]: cell state entering this frame (slab of the neighbouring frame or c0); NULL = 0
  const void* dy; long lddy;
  void* DZ;           // frame slab [B][4n] (storage type)
  float* Dh; float* Dc;   // [B][n] carried gradients
  int t;              // frame of this step (pointwise part)
  int t_next;         // frame whose dz sits in dzin (matmul part)
};
struct BwdArgs {
  BwdDir d[2];
  const int* lens;
  int B, n, nkc, T, ndir, do_matmul, do_pointwise;
};
hipError_t launch_step_bwd(const BwdArgs& a, bool bf16, hipStream_t s);

// Single-launch ("persistent") variants for bfloat16 storage: one launch runs every time step with
// W_h resident in registers.  What crosses work-groups (h_t forward, partial sums of Dh backward)
// travels through a two-slot ring in global memory whose every 8-byte unit carries its values AND a tag
// of the step that wrote it, so a consumer needs no barrier and no fence: it re-reads the ring until every
// tag shows the step it waits for.
//   Forward (h): the K axis of the ring is the unit index; an 8-byte unit carries four consecutive values of one row.
//   |h| <= 1, so bit 14 of a bf16 h (the top bit of the exponent) is always 0; in the fourth value that bit IS the
//   tag - one bit is enough to tell a slot's new contents from what the step two earlier left there - and the reader
//   clears it.  Chunks of 8 values x 64 lanes form MFMA A-fragments exactly as in the per-step kernels.
//   Backward (partial sums of Dh): same unit and tag; the layout is described at the kernels.
// sync[0] is an error word set when a bounded wait expires.
constexpr int kLLValsFwd = 16, kLLSlotsFwd = 16;     // 16 h values  -> 4 units  -> 2 chunks per producer and row
constexpr int kLLMaxNkcFwd = 32;                     // register budget of the kernels (n <= 1024)
constexpr unsigned kLLFwdTagBit = 0x40000000u;       // in the upper dword of a unit: bit 14 of the fourth value
inline int ll_nkc(int n, int slots) { return (int)((((long)(n + 15) / 16) * slots + 31) / 32); }
// The tag bit of the data that step tau consumes (written by step tau - 1 into slot tau & 1; the initial contents of
// slot 0 carry it for tau = 0): it alternates between consecutive uses of a slot and is 1 at a slot's first use, so a
// zero-filled slot never looks written.
__host__ __device__ inline unsigned ll_fwd_tag(unsigned tau) { return ((tau >> 1) & 1u) ^ 1u; }

struct PFwdDir {
  const uint4* Wf;    // [unit tile][gate][nkc][64] chunks
  const uint4* Wzero; // one chunk (64 x 16 bytes) of zeros
  uint4* ring0; uint4* ring1;   // [row tile][nkc][64] chunks each
  float* gates;       // [T][B][4n]
  float* hstate; float* cstate;
  void* y; long ldy;  // y + column offset of this direction; frame stride B*ldy
  float* cs;          // [T][B][n] or NULL
  void* hprev;        // [T][B][n] or NULL
  int rev;            // 0: t = tau, 1: t = T-1-tau
};
struct PFwdArgs {
  PFwdDir d[2];
  const int* lens;
  int B, n, nkc, T, ndir, write_gates;
  unsigned* sync; unsigned spin_limit;
  unsigned* xcc;      // NULL or one zeroed word per work-group (see PBwdArgs)
  int rt0;            // set by the launcher: first 16-row tile of the batch that this launch handles
  bool plain_launch;  // ordinary instead of cooperative launch (the caller vouches that the device is otherwise idle)
};
hipError_t launch_persist_fwd(const PFwdArgs& a, hipStream_t s);
bool persist_fwd_fits(const PFwdArgs& a);     // would launch_persist_fwd launch anything on this device?
// Float storage (an initial hidden state goes through launch_h0_term, as for bfloat16): Wf is the per-step kernel's packed W_h (launch_pack_wh_fwd), ring0 / ring1 its
// fragment-ordered h buffers (initialised here), y / hprev float; nkc = chunks of 16 k.
hipError_t launch_persist_fwd_f32(const PFwdArgs& a, hipStream_t s);
bool persist_fwd_f32_fits(const PFwdArgs& a);

struct PBwdDir {
  const uint4* Wb;    // as launch_prep_bwd_ll writes it
  uint4* ring0; uint4* ring1;
  const float* gates; const float* cs; const float* c0;
  const void* dy; long lddy;
  void* DZ;           // [T][B][4n]
  float* Dh; float* Dc;
  float* dbpart;      // NULL or [2 * row tiles][4n]: slice g receives the bias gradient summed over row group g (8 rows)
  int rev;
};
struct PBwdArgs {
  PBwdDir d[2];
  const int* lens;
  int B, n, T, ndir;
  unsigned* sync; unsigned spin_limit;
  unsigned* xcc;      // NULL or one zeroed word per work-group: lets an exchange group find out whether it shares an XCD
  int rt0;            // set by the launcher: first 16-row tile of the batch that this launch handles
  bool plain_launch;  // ordinary instead of cooperative launch (the caller vouches that the device is otherwise idle)
};
// Does the single-launch backward kernel (partial sums of Dh exchanged; W_h via launch_prep_bwd_ll, ring of
// bwdp_ring_bytes per direction and slot) fit the device for this problem?
bool persist_bwd_fits(const PBwdArgs& a);
hipError_t launch_persist_bwd(const PBwdArgs& a, hipStream_t s);
// Float storage: the same exchange of partial sums in float.  W_h^T via launch_pack_wh_bwd_f32p (bwd_f32_wh_bytes per
// direction), rings of bwd_f32_ring_bytes per direction and slot, zero-filled; gates, cs, dy, DZ float; dbpart unused.
bool persist_bwd_f32_fits(const PBwdArgs& a);
hipError_t launch_persist_bwd_f32(const PBwdArgs& a, hipStream_t s);
hipError_t launch_pack_wh_bwd_f32p(const void* W_h, void* Wb, int n, int ndir, hipStream_t s);
inline size_t bwd_f32_wh_bytes(int n) { return (size_t)((n + 15) / 16) * 4 * 16 * 16 * 64 * 4; }
inline size_t bwd_f32_ring_bytes(int B, int n) {
  const size_t tiles = (size_t)((n + 15) / 16), rts = 2 * (size_t)(((B > 0 ? B : 1) + 31) / 32);
  return rts * tiles * tiles * 1024;
}
inline size_t bwdp_wh_bytes(int n) { return (size_t)((n + 31) / 32) * 262144; }                  // per direction
inline size_t bwdp_ring_bytes(int B, int n) {                                                      // per direction and slot
  const size_t groups = 2 * (size_t)(((B > 0 ? B : 1) + 15) / 16), tiles = (size_t)((n + 31) / 32);
  return groups * tiles * tiles * 512;
}
// (launch_prep_fwd_ll: W_h in ring order; ring slot 0 = zeros carrying the tag of step 0, ring slot 1 cleared.  The initial state does
// not travel through the ring: launch_h0_term adds its product with W_h to the pre-activations of every row's first frame instead.)
// gates[first frame of row b][b][:] += bf16(h0[b]) . W_h for every row with a frame (forward: t = 0; reverse: t = len - 1),
// per direction; gates [T][B][4n] float with `gates_stride` elements between directions.
hipError_t launch_h0_term(const float* h0, const void* W_h, bool bf16, float* gates, long gates_stride, const int* lens, int T, int B, int n,
                          int ndir, int rev0, int rev1, hipStream_t s);

// Weight / state packing and small helpers (all enqueue-only).
hipError_t launch_pack_wh_fwd(const void* W_h, uint4* Wf, int n, int nkc, int ndir, bool bf16, hipStream_t s);
hipError_t launch_pack_wh_bwd(const void* W_h, uint4* Wb, int n, int nkc, int ndir, bool bf16, hipStream_t s);
// h (float [ndir][B][n]) -> fragment order, zero padded, written to both ping-pong buffers
hipError_t launch_pack_state(const float* h, uint4* frag0, uint4* frag1, int B, int n, int nkc, int nrt, int ndir,
                             bool bf16, hipStream_t s);
int device_ok();   // 0 if the current device is gfx950, else a negative lstm_status (cached after the first call)
hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s);                 // p 4-byte aligned, bytes % 2 == 0
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t s);   // bytes % 4 == 0
// Up to kMax regions cleared by one launch (the set-up of a layer clears half a dozen small buffers; one launch each
// costs more in launch gaps than in work).  Every region 4-byte aligned, bytes % 4 == 0.
struct ZeroRegions {
  static constexpr int kMax = 8;
  void* ptr[kMax];
  size_t words[kMax];
  int first_block[kMax + 1];
  int count;
  bool overflow;
  ZeroRegions() : ptr{}, words{}, first_block{}, count(0), overflow(false) {}
  void add(void* p, size_t bytes);
};
hipError_t launch_fill_zero_many(const ZeroRegions& r, hipStream_t s);
// The set-up of a bfloat16 single-launch loop in one launch: the fills of `z`, W_h in the kernel's order, (forward) the initial
// ring, and the frame map of launch_frame_map if fm.cidx is not NULL.
struct FrameMapArgs { const int* lens; int T, B; int* cidx; int* fidx; int* count; };
hipError_t launch_prep_fwd_ll(const ZeroRegions& z, const void* W, uint4* Wf, int n, int nkc, int ndir, uint4* ring0, uint4* ring1,
                              int nrt, const FrameMapArgs& fm, hipStream_t s);
hipError_t launch_prep_bwd_ll(const ZeroRegions& z, const void* W, uint4* Wb, int n, int ndir, const FrameMapArgs& fm, hipStream_t s);
// db[c] (+)= sum_rows DZ[row][c]; part = float scratch [nsplit][ncols] per direction
// db[dir][c] (+)= sum over the first nslices slices of part[dir][kColsumSlices][ncols]
constexpr int kColsumSlices = 64;
hipError_t launch_colsum_final(const float* part, float* db, int ncols, int ndir, int nslices, int accumulate, hipStream_t s);
hipError_t launch_colsum(const void* DZ, float* db, float* part, int rows, int ncols, int ndir, long sDZ,
                         bool bf16, int accumulate, hipStream_t s);

// One time step for all rows as a single product (inference, bfloat16 storage; see single_step.hip):
// Wcat[ndir][4n][Kc] = [W_x^T | 0 up to n_in_pad | W_h^T | 0 up to Kc]
hipError_t launch_pack_wcat(const void* W_x, const void* W_h, void* Wcat, int n_in, int n_in_pad, int n, int Kc, int ndir, hipStream_t s);
// Acat[ndir][B][Kc] = [x | 0 | bf16(h[dir]) | 0] in the same column layout (h == NULL: zeros)
// max-pooling in time (time_pool.hip); arg [T'][B][F] bytes, lens_out [B] may be NULL
hipError_t launch_time_pool_fwd(bool bf16, const void* y, long ldy, const int* lens, void* out, long ldo, uint8_t* arg, int* lens_out, int T,
                                int B, int F, int pool, hipStream_t s);
hipError_t launch_time_pool_bwd(bool bf16, const void* dout, long ldo, const uint8_t* arg, const int* lens, void* dy, long ldy, int T, int B,
                                int F, int pool, hipStream_t s);
hipError_t launch_concat_xh(const void* x, const float* h, void* Acat, int B, int n_in, int n_in_pad, int n, int Kc, int ndir, hipStream_t s);
// The same step with the cell update in the product's epilogue (gemm_skinny.hip):
// Wcell[ndir][128 * ceil(n/32)][Kc]: row 128 t + 32 q + u = row q n + 32 t + u of Wcat (zeros for units past n), so that
// a tile of 128 columns holds the four gates of 32 units.  Arguments of the step as for launch_cell_step.
inline size_t wcell_rows(int n) { return (size_t)128 * ((n + 31) / 32); }
hipError_t launch_pack_wcell(const void* W_x, const void* W_h, void* Wcell, int n_in, int n_in_pad, int n, int Kc, int ndir, hipStream_t s);
hipError_t launch_step_cell(const void* Acat, const void* Wcell, const float* bias, const float* h_in, const float* c_in, float* h_out,
                            float* c_out, void* y, long ldy, float* cs, const int* lens, int B, int n, int Kc, int ndir, hipStream_t s);
// cell update from the pre-activations z = bias + sum of `nparts` partial products, laid out [ndir][nparts][part floats]
// with [B][4n] inside a part.  h_in, c_in [ndir][B][n]: state entering the step (NULL = zeros); h_out, c_out: state
// leaving it (NULL = not wanted); y[B][ldy] (direction d at column d*n); cs[ndir][B][n] or NULL; rows with lens[b] < 1
// keep their state and output zero
hipError_t launch_cell_step(const float* z, long part, int nparts, const float* bias, const float* h_in, const float* c_in, float* h_out,
                            float* c_out, void* y, long ldy, float* cs, const int* lens, int B, int n, int ndir, hipStream_t s);

inline int cdiv(long a, long b) { return (int)((a + b - 1) / b); }

// Host-side set-up that HIP keeps per device (function attributes, what a device is and holds): done once on every
// device the library is used on, whichever thread gets there first.  `done` holds one bit per device ordinal (ordinals
// 64 apart share a bit: the set-up is then simply repeated); the set-up must be idempotent, since two threads may both run it.
template <typename F>
hipError_t once_per_device(std::atomic<unsigned long long>& done, F&& setup) {
  int dev = 0;
  const hipError_t eg = hipGetDevice(&dev);
  if (eg != hipSuccess) return eg;
  const unsigned long long bit = 1ull << (dev & 63);
  if (dev < 64 && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
  const hipError_t e = setup();
  if (e == hipSuccess && dev < 64) done.fetch_or(bit, std::memory_order_release);
  return e;
}

}  // namespace lstm
