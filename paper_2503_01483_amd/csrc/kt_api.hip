// kt_api.hip -- host side of libkurtail: argument checks, workspace layout, launch
// sequences, and the extern "C" boundary declared in include/kt.h.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/kt.h"
#include "kt_aux.h"
#include "kt_cayley_d128.h"
#include "kt_fused_d128.h"
#include "kt_hadamard.h"

namespace kt {

// ------------------------------------------------------------------ errors --------
static thread_local char g_err[512] = "";

static kt_status fail(kt_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

static bool launch_ok() { return hipGetLastError() == hipSuccess; }

// Kernels that use more than 64 KiB of dynamic LDS need the limit raised once per kernel AND per
// device (the attribute belongs to the device's copy of the code).  Remembers what has been set;
// safe to call from several host threads.
static bool ensure_dynamic_lds(const void* kernel, size_t bytes) {
  struct Entry { const void* kernel; int device; size_t bytes; };
  static std::mutex mu;
  static std::vector<Entry> done;
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess) return false;
  std::lock_guard<std::mutex> lock(mu);
  Entry* hit = nullptr;
  for (Entry& e : done)
    if (e.kernel == kernel && e.device == device) hit = &e;
  if (hit && hit->bytes >= bytes) return true;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) != hipSuccess) return false;
  if (hit) hit->bytes = bytes;
  else done.push_back({kernel, device, bytes});
  return true;
}

// ------------------------------------------------------------------ static scratch
// Device memory owned by the library image itself, for the one entry point that must not allocate
// (kt_cayley_step_static).  Every GPU the library runs on holds its own copy of the array at its own
// address until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress: the address a kernel can use is looked up once per device, with that device
// current, and kept in g_scratch_ptr; nothing else in this file may pass `scratch` itself anywhere.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static void* g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mu;

// Address of this device's copy of the scratch array (null on failure; text in kt_last_error()).
static void* static_scratch_of_current_device() {
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) {
    fail(KT_ERR_DEVICE, "no current HIP device (or device index beyond %d)", kMaxDevices - 1);
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    const hipError_t rc = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (rc != hipSuccess || !ptr) {
      fail(KT_ERR_DEVICE, "hipGetSymbolAddress(scratch) failed on device %d: %s", device, hipGetErrorString(rc));
      return nullptr;
    }
    g_scratch_ptr[device] = ptr;
  }
  return g_scratch_ptr[device];
}

// ------------------------------------------------------------------ profiling -----
// Optional event brackets around the large launches (see kt_profile_enable).
// Entry points running on several host threads may take records at the same time: the slot counter is
// atomic (a slot belongs to the scope that drew it); enabling, reading and resetting are not, as the header says.
struct ProfRecord { hipEvent_t start, stop; int id; };
static ProfRecord* g_prof = nullptr;
static int g_prof_cap = 0;
static std::atomic<int> g_prof_used{0};

struct ProfScope {
  ProfRecord* rec = nullptr;
  hipStream_t st;
  ProfScope(int id, hipStream_t s) : st(s) {
    if (g_prof && g_prof_used.load(std::memory_order_relaxed) < g_prof_cap) {
      const int slot = g_prof_used.fetch_add(1, std::memory_order_relaxed);
      if (slot >= g_prof_cap) return;  // another thread drew the last slot meanwhile
      rec = &g_prof[slot];
      rec->id = id;
      (void)hipEventRecord(rec->start, st);
    }
  }
  ~ProfScope() {
    if (rec) (void)hipEventRecord(rec->stop, st);
  }
};

// ------------------------------------------------------------------ tiles ---------
using bf16 = __bf16;
using TB_BIG = Tile<bf16, 256, 256, 2, 2>;   // d % 256 == 0
using TB_M128 = Tile<bf16, 128, 256, 1, 4>;  // features on m, d % 256 != 0
using TB_N128 = Tile<bf16, 256, 128, 4, 1>;  // features on n, d % 256 != 0
using TB_128 = Tile<bf16, 128, 128, 2, 2>;   // d x d outputs, d % 256 != 0
using TF = Tile<float, 128, 128, 2, 2>;      // fp32 path, every contraction

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

constexpr int kNumCUs = 256;
// Token-minor operands (X^T, G^T) are stored in blocks of this many tokens: within a block a
// feature row is contiguous, blocks follow each other feature-row-set by feature-row-set, so
// the 256 rows a tile streams together span 2 MiB per block instead of one page per row.
constexpr int64_t kTokenBlock = 4096;
constexpr int kHadMfmaFrom = 12;  // bf16 Hadamard factors of at least this order run on the matrix cores (measured: the vector kernel wins for 4 and 8)
constexpr int kSensBlocks = 1024;  // workgroups of the sensitivity sweeps
constexpr int kCayleyMaxIters = 32;
constexpr float kCayleyTol = 3e-7f;
constexpr int kCayleyFusedFrom = 6;  // three-term path: iterations from here on are single launches

#ifdef KT_PHASE_STAMPS
static int g_stamp_next = -1;  // developer build: slot the next GEMM launch records its phase stamps in (-1: none)
#endif

template <class TL, class Epi, bool ATN = false>
static bool launch_gemm(const void* A, int64_t lda, int64_t bsa, int M, const void* B, int64_t ldb,
                        int64_t bsb, int N, int64_t K, int slabs_per_split, int batch,
                        const Epi& epi, hipStream_t stream, int64_t k_block = 0,
                        int64_t block_stride_a = 0, int64_t block_stride_b = 0, int k_valid = 0) {
  // ATN: A is [K][lda] with the M index along its rows (see gemm_mainloop); K blocking applies to B only
  auto kern = gemm_nt_kernel<TL, Epi, ATN>;
  constexpr int lds_bytes = ATN ? 2 * (kAtnStageBytes + TL::B_BYTES) : TL::LDS_BYTES;
  // the kernel addresses the rows of a tile with 32-bit byte offsets from the tile's first row
  const int64_t esz = (int64_t)sizeof(typename TL::T);
  if ((ATN ? 127 : TL::BM - 1) * lda * esz + 512 > (int64_t)UINT32_MAX || (TL::BN - 1) * ldb * esz + 128 > (int64_t)UINT32_MAX)
    return false;
  if (ATN && (k_valid < 1 || k_valid > K)) return false;
  if (!ensure_dynamic_lds(reinterpret_cast<const void*>(kern), lds_bytes)) return false;
  GemmShape g;
  g.A = A; g.B = B; g.lda = lda; g.ldb = ldb;
  g.batch_stride_a = bsa; g.batch_stride_b = bsb;
  g.M = M; g.N = N;
  g.tiles_m = (int)ceil_div(M, TL::BM);
  g.tiles_n = (int)ceil_div(N, TL::BN);
  g.slabs_total = (int)(K / TL::BK);
  g.slabs_per_split = slabs_per_split > 0 ? slabs_per_split : g.slabs_total;
  g.split_k = (int)ceil_div(g.slabs_total, g.slabs_per_split);  // every split non-empty
  g.tiles_total = g.tiles_m * g.tiles_n * g.split_k;
  g.grid_padded = (int)round_up(g.tiles_total, 8);
  // K blocking: rows hold K in blocks of k_block elements, block b of a row starts
  // block_stride elements after block b-1 (k_block = 0: ordinary contiguous rows)
  g.slabs_per_block = k_block > 0 ? (int)(k_block / TL::BK) : (g.slabs_total > 0 ? g.slabs_total : 1);
  g.block_bytes_a = block_stride_a * (int64_t)sizeof(typename TL::T);
  g.block_bytes_b = block_stride_b * (int64_t)sizeof(typename TL::T);
  g.k_valid = k_valid;
#ifdef KT_PHASE_STAMPS
  g.stamp_slot = g_stamp_next >= 0 && g_stamp_next < kStampSlots ? g_stamp_next++ : -1;
#endif
  hipLaunchKernelGGL(kern, dim3(g.grid_padded, batch), dim3(TL::NT), lds_bytes, stream, g, epi);
  return launch_ok();
}

// K slabs per split so that `tiles` output tiles give about `target_wgs` workgroups
// (one per CU for 256 x 256 tiles, several for the small tiles that share a CU), with at
// least 8 slabs of work in each split.
static int choose_slabs_per_split(int64_t tiles, int64_t slabs_total, int64_t target_wgs) {
  int64_t s = ceil_div(target_wgs, tiles);
  const int64_t cap = slabs_total / 8 > 0 ? slabs_total / 8 : 1;
  if (s > cap) s = cap;
  if (s < 1) s = 1;
  return (int)ceil_div(slabs_total, s);
}

// ------------------------------------------------------------------ workspace -----
struct Carver {
  size_t off = 0;
  size_t take(size_t bytes) {
    const size_t o = off;
    off = (size_t)round_up((int64_t)(off + bytes), 256);
    return o;
  }
};

struct LossGradPlan {
  bool fused;      // d = 128 bf16: single-pass kernel, no token-minor copies
  int fused_wgs;   // workgroups per problem on the fused path
  bool fp32;
  size_t esz;
  int64_t ldt;     // padded token count of the token-minor copies (multiple of 128)
  int64_t tb;      // tokens per block of the token-minor copies (row length inside a block)
  int64_t nblk;    // blocks per feature row
  int P;           // moment partials per token
  int tiles_dd;    // tiles of the d x d output GEMM
  int slabs_per_split, split_k;
  size_t o_rt, o_part, o_coef, o_losspart, o_xt, o_gt, o_splitk, o_gstat, o_yt, total;
  int loss_blocks;
  bool keep_y;     // the forward pass writes Y (fp32, token-minor) and the backward pass reads it instead of recomputing it
};

// Up to this many bytes of kept Y, kt_workspace_bytes(KT_OP_LOSS_GRAD / KT_OP_POOLED_LOSS_GRAD) asks for the
// room to keep it (4 n d bytes per problem); beyond, for the recompute form.
constexpr int64_t kKeepYMaxBytes = (int64_t)64 << 30;

static LossGradPlan plan_loss_grad(int64_t batch, int64_t n, int64_t d, kt_dtype xdt, bool pooled = false,
                                   bool keep_y = false) {
  LossGradPlan p;
  p.keep_y = false;
  p.o_yt = 0;
  p.fp32 = (xdt == KT_F32);
  p.esz = p.fp32 ? 4 : 2;
  p.fused = !p.fp32 && d == 128 && !pooled;  // the pooled loss needs its global statistics before the gradient
  p.fused_wgs = 0;
  if (p.fused) {
    const int64_t tiles = ceil_div(n, kF128Tile);
    int64_t wgs = ceil_div(kNumCUs, batch);  // about one workgroup per CU over all problems
    p.fused_wgs = (int)(wgs < tiles ? wgs : tiles);
    p.ldt = p.tb = p.nblk = 0;
    p.P = p.tiles_dd = p.slabs_per_split = p.split_k = p.loss_blocks = 0;
    Carver c;
    p.o_rt = c.take((size_t)batch * d * d * p.esz);
    p.o_losspart = c.take((size_t)batch * p.fused_wgs * 8);
    p.o_splitk = c.take((size_t)p.fused_wgs * batch * d * d * 4);
    p.o_part = p.o_coef = p.o_xt = p.o_gt = p.o_gstat = 0;
    p.total = c.off;
    return p;
  }
  p.ldt = round_up(n, 128);
  p.tb = p.ldt < kTokenBlock ? p.ldt : kTokenBlock;
  p.nblk = ceil_div(p.ldt, p.tb);
  int64_t slabs;
  if (p.fp32) {
    p.P = (int)ceil_div(d, TF::BM) * TF::WGM;
    p.tiles_dd = (int)(ceil_div(d, TF::BM) * ceil_div(d, TF::BN));
    slabs = p.ldt / TF::BK;
  } else if (d % 256 == 0) {
    p.P = (int)(d / TB_BIG::BM) * TB_BIG::WGM;
    p.tiles_dd = (int)((d / 256) * (d / 256));
    slabs = p.ldt / TB_BIG::BK;
  } else {
    p.P = (int)ceil_div(d, TB_M128::BM) * TB_M128::WGM;
    p.tiles_dd = (int)(ceil_div(d, 128) * ceil_div(d, 128));
    slabs = p.ldt / TB_128::BK;
  }
  const bool big_tiles = !p.fp32 && d % 256 == 0;
  p.slabs_per_split = choose_slabs_per_split((int64_t)p.tiles_dd * batch, slabs,
                                             big_tiles ? kNumCUs : 4 * kNumCUs);
  p.split_k = (int)ceil_div(slabs, p.slabs_per_split);
  p.loss_blocks = (int)ceil_div(n, 256);
  Carver c;
  p.o_rt = c.take((size_t)batch * d * d * p.esz);
  p.o_part = c.take((size_t)batch * p.P * n * 16);
  p.o_coef = c.take((size_t)batch * n * 16);
  p.o_losspart = c.take((size_t)batch * p.loss_blocks * 8 * (pooled ? 4 : 1));
  p.o_gstat = c.take(pooled ? (size_t)batch * 4 * 8 : 0);
  p.o_xt = c.take(big_tiles ? 0 : (size_t)batch * d * p.nblk * p.tb * p.esz);  // big tiles read X as it is
  p.o_gt = c.take((size_t)batch * d * p.nblk * p.tb * p.esz);
  p.o_splitk = c.take(p.split_k > 1 ? (size_t)p.split_k * batch * d * d * 4 : 0);
  p.keep_y = keep_y;
  p.o_yt = c.take(keep_y ? (size_t)batch * d * p.nblk * p.tb * 4 : 0);
  p.total = c.off;
  return p;
}

// The plan kt_workspace_bytes recommends: Y kept when it is small enough and the path has a backward GEMM to save.
static bool keep_y_recommended(int64_t batch, int64_t n, int64_t d, kt_dtype xdt, bool pooled) {
  if (xdt == KT_BF16 && d == 128 && !pooled) return false;  // single-pass kernel
  return batch * round_up(n, 128) * d * 4 <= kKeepYMaxBytes;
}

struct CayleyPlan {
  bool split;  // three-term bf16 GEMMs on the bf16 matrix cores instead of fp32 MFMA
  size_t o_m, o_b, o_rt, o_zt, o_u0, o_u1, o_delta, o_g2, o_sq, o_scal, total;
  int g2_blocks;  // Cayley Adam: block partials of ||G||^2 per problem
};

// Large problems run their d^3 GEMMs as three-term bf16 products (about 2^-17 relative
// per term, 3x the flops at ~16x the rate of the fp32 matrix pipe); small ones, where the
// step costs microseconds anyway, stay in fp32.
static bool cayley_use_split(int64_t d) { return d >= 1024 && d % 256 == 0; }

static CayleyPlan plan_cayley(int64_t batch, int64_t d) {
  CayleyPlan p;
  Carver c;
  p.split = cayley_use_split(d);
  const size_t mat = (size_t)batch * d * d * 4;
  const size_t smat = (size_t)batch * d * d * 6;  // [d][3d] bf16
  p.o_m = c.take(mat);  // M = dR R^T; in the fp32 path later reused as the second U buffer
  p.o_b = c.take(p.split ? smat : mat);
  p.o_rt = c.take(mat);
  p.o_zt = c.take(mat);
  p.o_u0 = c.take(p.split ? smat : mat);
  p.o_u1 = p.split ? c.take(smat) : p.o_m;
  p.o_delta = c.take((size_t)batch * kCayleyMaxIters * 4);
  // Cayley Adam scalars: partial sums (fp64) and {r, alpha, ||W||, alpha/(2r)} per problem
  p.g2_blocks = (int)(ceil_div(d * d / 4, 256) < 1024 ? ceil_div(d * d / 4, 256) : 1024);
  p.o_g2 = c.take((size_t)batch * p.g2_blocks * 8);
  p.o_sq = c.take((size_t)batch * (d / 32) * (d / 32) * 8);
  p.o_scal = c.take((size_t)batch * 4 * 4);
  p.total = c.off;
  return p;
}

struct QuantPlan {
  bool fp32;
  size_t esz;
  int P, PN;
  // Scales computed here AND codes or errors wanted: Y goes through an fp32 staging buffer of at most
  // kQuantStageBytes, `problems` whole problems or `rows` tokens of one problem per launch pair.
  int64_t stage_problems, stage_rows;
  size_t o_rt, o_amax, o_scales, o_errpart, o_y, total;
};

// d = 4096, n = 131072: fake-quant measured alike from 64 MiB to 4 GiB; the quantisation figures, whose row
// kernel is one workgroup per token, lose 7 % at 256 MiB and nothing at 1 GiB
constexpr int64_t kQuantStageBytes = (int64_t)1 << 30;

// How many whole problems, or how many token rows of one problem, an fp32 staging buffer of at most
// kQuantStageBytes takes per launch pair (rotation GEMM + row kernel).
static void stage_slices(int64_t batch, int64_t n, int64_t d, int64_t* problems, int64_t* rows) {
  const int64_t cap = kQuantStageBytes / (4 * d) / 256 * 256;  // >= 16384 token rows at d <= 16384
  *rows = n < cap ? n : cap;
  *problems = n <= cap ? (cap / n < batch ? cap / n : batch) : 1;
}

static QuantPlan plan_quant(int64_t batch, int64_t n, int64_t d, kt_dtype xdt) {
  QuantPlan p;
  p.fp32 = (xdt == KT_F32);
  p.esz = p.fp32 ? 4 : 2;
  if (p.fp32) {
    p.P = (int)ceil_div(d, TF::BM) * TF::WGM;
    p.PN = (int)ceil_div(d, TF::BN) * TF::WGN;
  } else if (d % 256 == 0) {
    p.P = (int)(d / 256) * TB_BIG::WGM;
    p.PN = (int)(d / 256) * TB_BIG::WGN;
  } else {
    p.P = (int)ceil_div(d, TB_M128::BM) * TB_M128::WGM;
    p.PN = (int)ceil_div(d, TB_N128::BN) * TB_N128::WGN;
  }
  Carver c;
  p.o_rt = c.take((size_t)batch * d * d * p.esz);
  p.o_amax = c.take((size_t)batch * p.P * n * 4);
  p.o_scales = c.take((size_t)batch * n * 4);
  p.o_errpart = c.take((size_t)batch * p.P * n * 8);
  stage_slices(batch, n, d, &p.stage_problems, &p.stage_rows);
  p.o_y = c.take((size_t)p.stage_problems * p.stage_rows * d * 4);
  p.total = c.off;
  return p;
}

// ------------------------------------------------------------------ checks --------
static kt_status check_xr(const void* X, int64_t ldx, const void* R, int64_t ldr, int64_t batch,
                          int64_t n, int64_t d, kt_dtype xdt, kt_dtype rdt) {
  if (!X || !R) return fail(KT_ERR_INVALID_ARG, "X and R must not be null");
  if (batch < 1 || n < 1 || d < 1) return fail(KT_ERR_INVALID_ARG, "batch, n, d must be positive");
  if (xdt != KT_F32 && xdt != KT_BF16) return fail(KT_ERR_BAD_DTYPE, "x_dtype must be KT_F32 or KT_BF16");
  if (rdt != KT_F32 && rdt != KT_BF16) return fail(KT_ERR_BAD_DTYPE, "r_dtype must be KT_F32 or KT_BF16");
  if (xdt == KT_F32 && rdt != KT_F32)
    return fail(KT_ERR_BAD_DTYPE, "the fp32 path needs an fp32 R");
  if (d % 128 != 0) return fail(KT_ERR_BAD_SHAPE, "d = %lld is not a multiple of 128", (long long)d);
  // n is bounded so that 255 rows of a token-minor operand stay inside 32-bit byte offsets
  if (d > 16384 || n > (int64_t)1 << 22 || batch > 65535)
    return fail(KT_ERR_BAD_SHAPE, "size out of range (d <= 16384, n <= 2^22, batch <= 65535)");
  const int64_t align = xdt == KT_F32 ? 4 : 8;
  if (ldx < d || ldx % align != 0)
    return fail(KT_ERR_BAD_SHAPE, "ldx = %lld must be >= d and a multiple of %lld", (long long)ldx,
                (long long)align);
  if (ldr < d) return fail(KT_ERR_BAD_SHAPE, "ldr = %lld must be >= d", (long long)ldr);
  // 255 rows of X must stay inside 32-bit byte offsets (tiles are addressed from their first row)
  if (ldx > (int64_t)1 << 22 || ldr > (int64_t)1 << 22)
    return fail(KT_ERR_BAD_SHAPE, "ldx and ldr must not exceed 2^22 elements");
  if ((reinterpret_cast<uintptr_t>(X) & 15) != 0)
    return fail(KT_ERR_BAD_SHAPE, "X must be 16-byte aligned");
  return KT_OK;
}

static kt_status check_ws(void* ws, size_t have, size_t need) {
  if (!ws) return fail(KT_ERR_INVALID_ARG, "workspace must not be null");
  if ((reinterpret_cast<uintptr_t>(ws) & 255) != 0)
    return fail(KT_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  if (have < need)
    return fail(KT_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", have, need);
  return KT_OK;
}

// R (fp32 or bf16, row-major) -> R^T in the GEMM dtype.
template <typename Tout>
static bool prep_rt(const void* R, int64_t ldr, kt_dtype rdt, Tout* RT, int64_t batch, int64_t d,
                    hipStream_t st) {
  dim3 grid((unsigned)ceil_div(d, 64), (unsigned)ceil_div(d, 64), (unsigned)batch);
  if (rdt == KT_F32)
    hipLaunchKernelGGL((transpose_kernel<float, Tout>), grid, dim3(256), 0, st,
                       static_cast<const float*>(R), ldr, d * ldr, RT, d, d * d, (int)d, (int)d, (int)d, 0);
  else
    hipLaunchKernelGGL((transpose_kernel<bf16, Tout>), grid, dim3(256), 0, st,
                       static_cast<const bf16*>(R), ldr, d * ldr, RT, d, d * d, (int)d, (int)d, (int)d, 0);
  return launch_ok();
}

// ------------------------------------------------------------------ loss + grad ---
struct PooledArgs {  // paper-literal pooled loss (kurtosis over all entries after an RMSNorm)
  float rms_eps;
  float* kappa_out;  // [batch] or null
};

template <typename T, class TFWD, class TDD>
static kt_status run_loss_grad(const LossGradPlan& p, const void* X, int64_t ldx, const void* R,
                               int64_t ldr, kt_dtype rdt, int64_t batch, int64_t n, int64_t d,
                               float kappa_target, float* loss, float* row_kurt, float* dR,
                               char* ws, hipStream_t st, const PooledArgs* pooled = nullptr) {
  T* RT = reinterpret_cast<T*>(ws + p.o_rt);
  floatx4* part = reinterpret_cast<floatx4*>(ws + p.o_part);
  floatx4* coef = reinterpret_cast<floatx4*>(ws + p.o_coef);
  double* loss_part = reinterpret_cast<double*>(ws + p.o_losspart);
  T* XT = reinterpret_cast<T*>(ws + p.o_xt);
  T* GT = reinterpret_cast<T*>(ws + p.o_gt);
  float* splitk = reinterpret_cast<float*>(ws + p.o_splitk);
  const T* Xp = static_cast<const T*>(X);

  // a0: R -> R^T in the GEMM dtype
  if (!prep_rt<T>(R, ldr, rdt, RT, batch, d, st)) return fail(KT_ERR_DEVICE, "prep_rt launch failed");

  // a1: forward GEMM (features on m, tokens on n) with the moment epilogue; with keep_y it also writes Y
  const bool keep = p.keep_y && dR;
  float* YT = reinterpret_cast<float*>(ws + p.o_yt);
  {
    ProfScope prof(0, st);
    EpiMoments<TFWD> e;
    e.part = part; e.n_tokens = (int)n; e.d = (int)d; e.P = p.P;
    bool ok;
    if (keep) {
      EpiMomentsKeep<TFWD> ek;
      ek.mom = e; ek.YT = YT; ek.ldt = p.ldt; ek.tb = p.tb; ek.batch_stride = d * p.nblk * p.tb;
      ok = launch_gemm<TFWD>(RT, d, d * d, (int)d, Xp, ldx, n * ldx, (int)n, d, 0, (int)batch, ek, st);
    } else {
      ok = launch_gemm<TFWD>(RT, d, d * d, (int)d, Xp, ldx, n * ldx, (int)n, d, 0, (int)batch, e, st);
    }
    if (!ok) return fail(KT_ERR_DEVICE, "forward GEMM launch failed");
  }
  if (pooled) {
    // a2, pooled form: pooled sums -> global statistics and loss -> per-token coefficients
    double* gstat = reinterpret_cast<double*>(ws + p.o_gstat);
    hipLaunchKernelGGL(pooled_stage1_kernel, dim3(p.loss_blocks, (unsigned)batch), dim3(256), 0, st, part, p.P,
                       (int)n, (int)d, pooled->rms_eps, loss_part);
    hipLaunchKernelGGL(pooled_stage2_kernel, dim3((unsigned)batch), dim3(256), 0, st, loss_part, p.loss_blocks,
                       (int)n, (int)d, kappa_target, gstat, loss, pooled->kappa_out);
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "pooled statistics launch failed");
    if (!dR) return KT_OK;
    hipLaunchKernelGGL(pooled_stage3_kernel, dim3(p.loss_blocks, (unsigned)batch), dim3(256), 0, st, part, p.P,
                       (int)n, (int)d, pooled->rms_eps, gstat, coef);
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "pooled coefficient launch failed");
  } else {
  // a2: per-token finalisation and loss
  hipLaunchKernelGGL(finalize_rows_kernel, dim3(p.loss_blocks, (unsigned)batch), dim3(256), 0, st, part,
                     p.P, (int)n, (int)d, kappa_target, coef, row_kurt, loss_part);
  if (!launch_ok()) return fail(KT_ERR_DEVICE, "finalize_rows launch failed");
  hipLaunchKernelGGL(finalize_loss_kernel, dim3((unsigned)batch), dim3(256), 0, st, loss_part,
                     p.loss_blocks, (int)n, loss);
  if (!launch_ok()) return fail(KT_ERR_DEVICE, "finalize_loss launch failed");
  if (!dR) return KT_OK;
  }

  // bf16, d % 256 == 0: the last GEMM reads X as it is (transposing LDS reads); otherwise it needs a
  // token-minor copy of X (zero padded to ldt tokens)
  constexpr bool kXDirect = std::is_same<TDD, TB_BIG>::value;
  if (!kXDirect) {
    ProfScope prof(3, st);
    if (sizeof(T) == 2) {
      dim3 grid((unsigned)ceil_div(p.ldt, 128), (unsigned)(d / 64), (unsigned)batch);
      hipLaunchKernelGGL(transpose16_kernel, grid, dim3(256), 0, st, reinterpret_cast<const uint16_t*>(Xp),
                         ldx, n * ldx, reinterpret_cast<uint16_t*>(XT), p.tb, d * p.nblk * p.tb, (int)n,
                         (int)p.ldt, (int)d);
    } else {
      dim3 grid((unsigned)(p.ldt / 64), (unsigned)ceil_div(d, 64), (unsigned)batch);
      hipLaunchKernelGGL((transpose_kernel<T, T>), grid, dim3(256), 0, st, Xp, ldx, n * ldx, XT, p.tb,
                         d * p.nblk * p.tb, (int)n, (int)p.ldt, (int)d, 1);
    }
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "X transpose launch failed");
  }
  // a3: dL/dY token-minor, from the kept Y entry by entry or from a recomputed Y in the GEMM epilogue
  if (keep) {
    ProfScope prof(1, st);
    constexpr int kFeats = 8;
    dim3 grid((unsigned)ceil_div(p.ldt, 256), (unsigned)ceil_div(d, 4 * kFeats), (unsigned)batch);
    hipLaunchKernelGGL((grad_from_y_kernel<T, kFeats>), grid, dim3(256), 0, st, YT, coef, GT, p.ldt, p.tb,
                       d * p.nblk * p.tb, (int)n, (int)d);
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "gradient kernel launch failed");
  } else {
    ProfScope prof(1, st);
    EpiGrad<TFWD> e;
    e.coef = coef; e.GT = GT; e.ldt = p.ldt; e.tb = p.tb; e.batch_stride = d * p.nblk * p.tb;
    e.n_tokens = (int)n; e.d = (int)d;
    if (!launch_gemm<TFWD>(RT, d, d * d, (int)d, Xp, ldx, n * ldx, (int)n, d, 0, (int)batch, e, st))
      return fail(KT_ERR_DEVICE, "backward recompute GEMM launch failed");
  }
  // a4: dR = X^T G, split over tokens
  {
    ProfScope prof(2, st);
    EpiStore<TDD> e;
    e.ldc = d; e.M = (int)d; e.N = (int)d;
    if (p.split_k > 1) {
      e.C = splitk; e.batch_stride = d * d; e.split_stride = batch * d * d;
    } else {
      e.C = dR; e.batch_stride = d * d; e.split_stride = 0;
    }
    bool ok;
    if constexpr (kXDirect)
      ok = launch_gemm<TDD, EpiStore<TDD>, true>(Xp, ldx, n * ldx, (int)d, GT, p.tb, d * p.nblk * p.tb, (int)d, p.ldt,
                                                 p.slabs_per_split, (int)batch, e, st, p.tb, 0, d * p.tb, (int)n);
    else
      ok = launch_gemm<TDD>(XT, p.tb, d * p.nblk * p.tb, (int)d, GT, p.tb, d * p.nblk * p.tb, (int)d, p.ldt,
                            p.slabs_per_split, (int)batch, e, st, p.tb, d * p.tb, d * p.tb);
    if (!ok) return fail(KT_ERR_DEVICE, "gradient GEMM launch failed");
    if (p.split_k > 1) {
      const int64_t count = batch * d * d;
      hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)(ceil_div(count, 256) < 4096 ? ceil_div(count, 256) : 4096)),
                         dim3(256), 0, st, splitk, count, p.split_k, dR, count);
      if (!launch_ok()) return fail(KT_ERR_DEVICE, "split-K reduce launch failed");
    }
  }
  return KT_OK;
}

// d = 128, bf16: one pass over X (kt_fused_d128.h), then fixed-order reductions.
static kt_status run_loss_grad_fused(const LossGradPlan& p, const void* X, int64_t ldx, const void* R,
                                     int64_t ldr, kt_dtype rdt, int64_t batch, int64_t n, int64_t d,
                                     float kappa_target, float* loss, float* row_kurt, float* dR,
                                     char* ws, hipStream_t st) {
  if (!ensure_dynamic_lds(reinterpret_cast<const void*>(fused_d128_kernel), kF128LdsBytes))
    return fail(KT_ERR_DEVICE, "the fused d=128 kernel needs %d bytes of LDS per workgroup", kF128LdsBytes);
  bf16* RT = reinterpret_cast<bf16*>(ws + p.o_rt);
  double* loss_part = reinterpret_cast<double*>(ws + p.o_losspart);
  float* dR_part = reinterpret_cast<float*>(ws + p.o_splitk);
  if (!prep_rt<bf16>(R, ldr, rdt, RT, batch, d, st)) return fail(KT_ERR_DEVICE, "prep_rt launch failed");
  {
    ProfScope prof(0, st);
    hipLaunchKernelGGL(fused_d128_kernel, dim3(p.fused_wgs, (unsigned)batch), dim3(256), kF128LdsBytes, st,
                       static_cast<const bf16*>(X), ldx, n * ldx, RT, (int)n, kappa_target, row_kurt,
                       loss_part, dR_part, dR ? 1 : 0);
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "fused kernel launch failed");
  }
  hipLaunchKernelGGL(finalize_loss_kernel, dim3((unsigned)batch), dim3(256), 0, st, loss_part, p.fused_wgs,
                     (int)n, loss);
  if (!launch_ok()) return fail(KT_ERR_DEVICE, "finalize_loss launch failed");
  if (dR) {
    const int64_t count = batch * d * d;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)(ceil_div(count, 256) < 4096 ? ceil_div(count, 256) : 4096)),
                       dim3(256), 0, st, dR_part, count, p.fused_wgs, dR, count);
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "partial dR reduce launch failed");
  }
  return KT_OK;
}

// ------------------------------------------------------------------ fake-quant ----
template <typename T, class TFWD, class TQ>
static kt_status run_quant(const QuantPlan& p, const void* X, int64_t ldx, const void* R, int64_t ldr,
                           kt_dtype rdt, int64_t batch, int64_t n, int64_t d, float clip,
                           const float* scales_in, float* scales_out, int8_t* codes, float* err,
                           char* ws, hipStream_t st) {
  T* RT = reinterpret_cast<T*>(ws + p.o_rt);
  float* amax = reinterpret_cast<float*>(ws + p.o_amax);
  float* scales_ws = reinterpret_cast<float*>(ws + p.o_scales);
  float2* errpart = reinterpret_cast<float2*>(ws + p.o_errpart);
  const T* Xp = static_cast<const T*>(X);
  if (!prep_rt<T>(R, ldr, rdt, RT, batch, d, st)) return fail(KT_ERR_DEVICE, "prep_rt launch failed");
  const float* scales = scales_in;
  if (!scales_in && (codes || err)) {
    // One GEMM instead of two: Y = X R is staged in fp32 (token-major: tokens on the rows of the GEMM), a
    // row kernel takes the maximum and quantises.  4 n d bytes written and read against 2 n d^2 flop saved.
    float* Ybuf = reinterpret_cast<float*>(ws + p.o_y);
    for (int64_t b0 = 0; b0 < batch; b0 += p.stage_problems) {
      const int64_t nb = batch - b0 < p.stage_problems ? batch - b0 : p.stage_problems;
      for (int64_t t0 = 0; t0 < n; t0 += p.stage_rows) {
        const int64_t nt = n - t0 < p.stage_rows ? n - t0 : p.stage_rows;
        EpiStore<TQ> e;
        e.C = Ybuf; e.ldc = d; e.batch_stride = nt * d; e.split_stride = 0; e.M = (int)nt; e.N = (int)d;
        if (!launch_gemm<TQ>(Xp + (b0 * n + t0) * ldx, ldx, n * ldx, (int)nt, RT + b0 * d * d, d, d * d, (int)d, d,
                             0, (int)nb, e, st))
          return fail(KT_ERR_DEVICE, "rotation GEMM launch failed");
        const int64_t rows = nb * nt, row0 = b0 * n + t0;
        float* so = scales_out ? scales_out + row0 : nullptr;
        int8_t* co = codes ? codes + row0 * d : nullptr;
        float2* eo = err ? reinterpret_cast<float2*>(err) + row0 : nullptr;
        const dim3 grid((unsigned)ceil_div(rows, 4));
        if (d <= 1024)
          hipLaunchKernelGGL((quant_rows_kernel<4, true>), grid, dim3(256), 0, st, Ybuf, rows, (int)d, clip, so, co, eo);
        else if (d <= 4096)
          hipLaunchKernelGGL((quant_rows_kernel<16, true>), grid, dim3(256), 0, st, Ybuf, rows, (int)d, clip, so, co, eo);
        else if (d <= 8192)
          hipLaunchKernelGGL((quant_rows_kernel<32, true>), grid, dim3(256), 0, st, Ybuf, rows, (int)d, clip, so, co, eo);
        else
          hipLaunchKernelGGL((quant_rows_kernel<1, false>), grid, dim3(256), 0, st, Ybuf, rows, (int)d, clip, so, co, eo);
        if (!launch_ok()) return fail(KT_ERR_DEVICE, "row quantiser launch failed");
      }
    }
    return KT_OK;
  }
  if (!scales_in) {
    EpiAmax<TFWD> e;
    e.part = amax; e.n_tokens = (int)n; e.d = (int)d; e.P = p.P;
    if (!launch_gemm<TFWD>(RT, d, d * d, (int)d, Xp, ldx, n * ldx, (int)n, d, 0, (int)batch, e, st))
      return fail(KT_ERR_DEVICE, "amax GEMM launch failed");
    hipLaunchKernelGGL(quant_scale_kernel, dim3((unsigned)ceil_div(n, 256), (unsigned)batch), dim3(256),
                       0, st, amax, p.P, n, clip, scales_ws, scales_out);
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "scale kernel launch failed");
    scales = scales_ws;
  } else if (scales_out) {
    if (hipMemcpyAsync(scales_out, scales_in, (size_t)batch * n * 4, hipMemcpyDeviceToDevice, st) != hipSuccess)
      return fail(KT_ERR_DEVICE, "scale copy failed");
  }
  if (!codes && !err) return KT_OK;
  {
    EpiQuant<TFWD> e;
    e.scales = scales; e.codes = codes; e.err_part = err ? errpart : nullptr;
    e.n_tokens = (int)n; e.d = (int)d; e.P = p.P;
    if (!launch_gemm<TFWD>(RT, d, d * d, (int)d, Xp, ldx, n * ldx, (int)n, d, 0, (int)batch, e, st))
      return fail(KT_ERR_DEVICE, "quantise GEMM launch failed");
  }
  if (err) {
    hipLaunchKernelGGL(quant_err_kernel, dim3((unsigned)ceil_div(n, 256), (unsigned)batch), dim3(256), 0,
                       st, errpart, p.P, n, reinterpret_cast<float2*>(err));
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "error reduce launch failed");
  }
  return KT_OK;
}

}  // namespace kt

using namespace kt;

// =================================================================== C ABI =========
// d = 128: one workgroup per problem does the whole step (kt_cayley_d128.h).
template <bool ADAM>
static kt_status launch_cayley_d128(float* R, const float* G, void* R_lowp, int64_t batch, float half_coef,
                                    float* ortho_err, int32_t* info, const C128Adam& ad, hipStream_t st) {
  if (!ensure_dynamic_lds(reinterpret_cast<const void*>(cayley_d128_kernel<ADAM>), kC128LdsBytes))
    return fail(KT_ERR_DEVICE, "the d=128 Cayley kernel needs %d bytes of LDS per workgroup", kC128LdsBytes);
  hipLaunchKernelGGL(cayley_d128_kernel<ADAM>, dim3((unsigned)batch), dim3(256), kC128LdsBytes, st, R, G,
                     static_cast<__bf16*>(R_lowp), half_coef, ortho_err, info, kCayleyMaxIters, kCayleyTol, ad);
  if (!launch_ok()) return fail(KT_ERR_DEVICE, "Cayley d=128 launch failed");
  return KT_OK;
}

// Optional Cayley Adam part of a retraction: moments already updated, r in scal[4b].
struct AdamArgs {
  float* M;            // [batch][d][d] momentum: in = beta1 M + (1-beta1) G, out = r W R
  float lr, q, eps;
  float* scal;         // [batch][4] device scalars {r, alpha, ||W||, alpha/(2r)}
  double* sq_part;     // [batch][(d/32)^2] tile partials of ||S||^2
  float* scalars_out;  // [batch][3] {r, alpha, ||W||} for the caller, or null
};

// Shared by the two optimisers.  P = G R^T, S = half_coef (P - P^T), then the Cayley transform
// Z = (I + c S)^-1 (I - c S) R by the fixed point in transposed space (c = 1, or alpha/(2r) from
// device memory for Adam), R <- Z.  For Adam, between set-up and iteration: step scalars, and
// M <- S R (the momentum moved into the tangent space at R).
static kt_status cayley_run(const CayleyPlan& p, char* ws, float* R, const float* G, void* R_lowp, int64_t batch,
                            int64_t d, float half_coef, const AdamArgs* adam, float* ortho_err, int32_t* info,
                            hipStream_t st) {
  float* Mm = reinterpret_cast<float*>(ws + p.o_m);
  float* Bm = reinterpret_cast<float*>(ws + p.o_b);
  float* Rt = reinterpret_cast<float*>(ws + p.o_rt);
  float* Zt = reinterpret_cast<float*>(ws + p.o_zt);
  float* U[2] = {reinterpret_cast<float*>(ws + p.o_u0), reinterpret_cast<float*>(ws + p.o_u1)};
  unsigned* delta = reinterpret_cast<unsigned*>(ws + p.o_delta);
  const int D = (int)d;
  const int64_t dd = d * d;

  if (p.split) {
    // three-term bf16 path: operands live as [d][3d] bf16
    __bf16* Bs = reinterpret_cast<__bf16*>(ws + p.o_b);
    __bf16* Us[2] = {reinterpret_cast<__bf16*>(ws + p.o_u0), reinterpret_cast<__bf16*>(ws + p.o_u1)};
    const int64_t sd = 3 * d * d;
    const unsigned sb = (unsigned)(ceil_div(dd, 256) < 8192 ? ceil_div(dd, 256) : 8192);
    // M = dR R^T with dR as [hi|hi|lo] (in Us[0]) and R as [hi|lo|hi] (in Us[1])
    hipLaunchKernelGGL(split3_kernel, dim3(sb, 1, (unsigned)batch), dim3(256), 0, st, G, D, D, Us[0], 0);
    hipLaunchKernelGGL(split3_kernel, dim3(sb, 1, (unsigned)batch), dim3(256), 0, st, R, D, D, Us[1], 1);
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "split launch failed");
    // below d = 4096 a 256 x 256 tiling leaves most CUs without a tile: use 128 x 128 there
    const bool big = (d / 256) * (d / 256) * batch >= kNumCUs;
    auto product = [&](const __bf16* A3, const __bf16* B3, int it, float* Cdst = nullptr, float alpha = 1.f) -> bool {
      auto go = [&](auto tile_tag) -> bool {
        using TL = decltype(tile_tag);
        EpiCayleyProduct<TL> e;
        e.C = Cdst ? Cdst : Mm; e.alpha = alpha;
        e.ldc = d; e.batch_stride = dd; e.split_stride = 0; e.M = D; e.N = D;
        e.delta = delta; e.it = it; e.max_iters = kCayleyMaxIters; e.tol = kCayleyTol;
        return launch_gemm<TL>(A3, 3 * d, sd, D, B3, 3 * d, sd, D, 3 * d, 0, (int)batch, e, st);
      };
      return big ? go(TB_BIG{}) : go(TB_128{});
    };
    if (!product(Us[0], Us[1], 0)) return fail(KT_ERR_DEVICE, "dR R^T GEMM launch failed");
    hipLaunchKernelGGL(fill_u32_kernel, dim3(64), dim3(256), 0, st, delta, batch * kCayleyMaxIters, 0u);
    hipLaunchKernelGGL(cayley_setup_kernel, dim3(D / 32, D / 32, (unsigned)batch), dim3(256), 0, st, Mm, R,
                       D, half_coef, (float*)nullptr, Rt, Zt, (float*)nullptr, Bs, Us[0], adam ? adam->sq_part : nullptr);
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "Cayley set-up launch failed");
    if (adam) {
      hipLaunchKernelGGL(adam_scalars2_kernel, dim3((unsigned)batch), dim3(256), 0, st, adam->sq_part,
                         (int)((d / 32) * (d / 32)), adam->lr, adam->q, adam->eps, adam->scal, adam->scalars_out);
      if (!launch_ok()) return fail(KT_ERR_DEVICE, "Cayley Adam scalar launch failed");
      // M <- S R = (1/2) S (2 Rt)^T: S sits in Bs as [hi|lo|hi], 2 Rt in Us[0] as [hi|hi|lo]; the same three
      // cross terms come out whichever operand carries which layout
      if (!product(Bs, Us[0], 0, adam->M, 0.5f)) return fail(KT_ERR_DEVICE, "momentum projection GEMM launch failed");
    }
    const unsigned ub = (unsigned)(ceil_div(dd / 4, 256) < 512 ? ceil_div(dd / 4, 256) : 512);
    // The first iterations run as product + elementwise update (the faster pair when they do real
    // work); the later ones, which almost always only find the convergence flag set, as ONE launch
    // each with the update in the GEMM epilogue: half as many launches to skip through.
    auto fused_iteration = [&](int it) -> bool {
      auto go = [&](auto tile_tag) -> bool {
        using TL = decltype(tile_tag);
        EpiCayleyIter<TL> e;
        e.Rt = Rt; e.Zt = Zt; e.Unew = nullptr; e.Usplit = Us[(it + 1) & 1]; e.delta = delta;
        e.d = D; e.it = it; e.max_iters = kCayleyMaxIters; e.tol = kCayleyTol;
        e.bscale = adam ? adam->scal : nullptr;
        return launch_gemm<TL>(Us[it & 1], 3 * d, sd, D, Bs, 3 * d, sd, D, 3 * d, 0, (int)batch, e, st);
      };
      return big ? go(TB_BIG{}) : go(TB_128{});
    };
    for (int it = 0; it < kCayleyMaxIters; ++it) {
      if (it >= kCayleyFusedFrom) {
        if (!fused_iteration(it)) return fail(KT_ERR_DEVICE, "Cayley iteration launch failed");
        continue;
      }
      if (!product(Us[it & 1], Bs, it)) return fail(KT_ERR_DEVICE, "Cayley iteration launch failed");
      hipLaunchKernelGGL(cayley_update_kernel, dim3(ub, (unsigned)batch), dim3(256), 0, st, Mm, Rt, Zt,
                         Us[(it + 1) & 1], D, delta, it, kCayleyMaxIters, kCayleyTol, adam ? adam->scal : nullptr);
      if (!launch_ok()) return fail(KT_ERR_DEVICE, "Cayley update launch failed");
    }
  } else {
  // M = dR R^T
  {
    EpiStore<TF> e;
    e.C = Mm; e.ldc = d; e.batch_stride = dd; e.split_stride = 0; e.M = D; e.N = D;
    if (!launch_gemm<TF>(G, d, dd, D, R, d, dd, D, d, 0, (int)batch, e, st))
      return fail(KT_ERR_DEVICE, "dR R^T GEMM launch failed");
  }
  // delta[it] collects max |Zt_new - Zt_old| of iteration it through atomicMax
  hipLaunchKernelGGL(fill_u32_kernel, dim3(64), dim3(256), 0, st, delta, batch * kCayleyMaxIters, 0u);
  if (!launch_ok()) return fail(KT_ERR_DEVICE, "fill launch failed");
  hipLaunchKernelGGL(cayley_setup_kernel, dim3(D / 32, D / 32, (unsigned)batch), dim3(256), 0, st, Mm, R,
                     D, half_coef, Bm, Rt, Zt, U[0], (__bf16*)nullptr, (__bf16*)nullptr, adam ? adam->sq_part : nullptr);
  if (!launch_ok()) return fail(KT_ERR_DEVICE, "Cayley set-up launch failed");
  if (adam) {
    hipLaunchKernelGGL(adam_scalars2_kernel, dim3((unsigned)batch), dim3(256), 0, st, adam->sq_part,
                 (int)((d / 32) * (d / 32)), adam->lr, adam->q, adam->eps, adam->scal, adam->scalars_out);
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "Cayley Adam scalar launch failed");
    EpiStore<TF> e;  // M <- S R = S (Rt)^T
    e.C = adam->M; e.ldc = d; e.batch_stride = dd; e.split_stride = 0; e.M = D; e.N = D;
    if (!launch_gemm<TF>(Bm, d, dd, D, Rt, d, dd, D, d, 0, (int)batch, e, st))
      return fail(KT_ERR_DEVICE, "momentum projection GEMM launch failed");
  }
  // fixed point in transposed space: Zt <- Rt - U Bm^T, U <- Rt + Zt
  for (int it = 0; it < kCayleyMaxIters; ++it) {
    EpiCayleyIter<TF> e;
    e.Rt = Rt; e.Zt = Zt; e.Unew = U[(it + 1) & 1]; e.Usplit = nullptr; e.delta = delta;
    e.d = D; e.it = it; e.max_iters = kCayleyMaxIters; e.tol = kCayleyTol;
    e.bscale = adam ? adam->scal : nullptr;
    if (!launch_gemm<TF>(U[it & 1], d, dd, D, Bm, d, dd, D, d, 0, (int)batch, e, st))
      return fail(KT_ERR_DEVICE, "Cayley iteration launch failed");
  }
  }
  hipLaunchKernelGGL(cayley_finish_kernel, dim3(D / 32, D / 32, (unsigned)batch), dim3(256), 0, st, Zt, D,
                     R, static_cast<__bf16*>(R_lowp), delta, kCayleyMaxIters, kCayleyTol, info);
  if (!launch_ok()) return fail(KT_ERR_DEVICE, "Cayley wrap-up launch failed");
  if (ortho_err) {
    hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(256), 0, st, reinterpret_cast<unsigned*>(ortho_err),
                       batch, 0u);
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "fill launch failed");
    EpiOrtho<TF> e;
    e.err = reinterpret_cast<unsigned*>(ortho_err); e.d = D;
    // Zt Zt^T = R^T R
    if (!launch_gemm<TF>(Zt, d, dd, D, Zt, d, dd, D, d, 0, (int)batch, e, st))
      return fail(KT_ERR_DEVICE, "orthogonality GEMM launch failed");
    hipLaunchKernelGGL(ortho_diag_kernel, dim3(D, (unsigned)batch), dim3(256), 0, st, Zt, D,
                       reinterpret_cast<unsigned*>(ortho_err));
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "orthogonality diagonal launch failed");
  }
  return KT_OK;
}


// ------------------------------------------------------------- Hadamard rows ----
template <typename T, int LOG2D>
static kt_status launch_hadamard(const void* X, int64_t ldx, void* Y, int64_t ldy, const int8_t* signs, int64_t n,
                                 float scale, int sign_rows, hipStream_t st) {
  constexpr size_t lds = 4 * (size_t)kHadRegion * 4;
  if (!ensure_dynamic_lds(reinterpret_cast<const void*>(hadamard_rows_kernel<T, LOG2D>), lds))
    return fail(KT_ERR_DEVICE, "the Hadamard kernel needs %d bytes of LDS per workgroup", (int)lds);
  const int64_t rows = kHadChunk >> LOG2D, chunks = ceil_div(n, rows);
  const int64_t wgs = ceil_div(chunks, 4) < 2 * kNumCUs ? ceil_div(chunks, 4) : 2 * kNumCUs;
  hipLaunchKernelGGL((hadamard_rows_kernel<T, LOG2D>), dim3((unsigned)wgs), dim3(256), lds, st,
                     static_cast<const T*>(X), ldx, static_cast<T*>(Y), ldy, signs, n, scale, sign_rows);
  if (!launch_ok()) return fail(KT_ERR_DEVICE, "Hadamard launch failed");
  return KT_OK;
}

template <typename T>
static kt_status dispatch_hadamard(int log2d, const void* X, int64_t ldx, void* Y, int64_t ldy,
                                   const int8_t* signs, int64_t n, float scale, int sign_rows, hipStream_t st) {
  switch (log2d) {
    case 7: return launch_hadamard<T, 7>(X, ldx, Y, ldy, signs, n, scale, sign_rows, st);
    case 8: return launch_hadamard<T, 8>(X, ldx, Y, ldy, signs, n, scale, sign_rows, st);
    case 9: return launch_hadamard<T, 9>(X, ldx, Y, ldy, signs, n, scale, sign_rows, st);
    case 10: return launch_hadamard<T, 10>(X, ldx, Y, ldy, signs, n, scale, sign_rows, st);
    case 11: return launch_hadamard<T, 11>(X, ldx, Y, ldy, signs, n, scale, sign_rows, st);
    default: return launch_hadamard<T, 12>(X, ldx, Y, ldy, signs, n, scale, sign_rows, st);
  }
}

static bool is_prime(int64_t q) {
  if (q < 2) return false;
  for (int64_t t = 2; t * t <= q; ++t)
    if (q % t == 0) return false;
  return true;
}

// How a row length splits into H_d = H_m (x) S_p2 (stated in kt.h).  kind 0: H_m Sylvester,
// 1: Paley's first construction, 2: Paley's second.  False when there is no such split.
static bool hadamard_split(int64_t d, int* m, int* p2, int* kind) {
  int64_t r = d;
  int t = 0;
  while (r > 1 && (r & 1) == 0) { r >>= 1; ++t; }
  if (r == 1) {
    int64_t mm = 1;
    if (t > 12) mm = (int64_t(1) << (t - 12)) < 4 ? 4 : (int64_t(1) << (t - 12));
    *m = (int)mm; *p2 = (int)(d / mm); *kind = 0;
    return true;
  }
  for (int j = 2; j <= t; ++j) {
    const int64_t mm = r << j;
    if (mm > 256) break;
    const int k = is_prime(mm - 1) ? 1 : (is_prime(mm / 2 - 1) && (mm / 2 - 1) % 4 == 1) ? 2 : 0;
    if (k) { *m = (int)mm; *p2 = (int)(d / mm); *kind = k; return true; }
  }
  return false;
}

template <typename T>
static kt_status run_hadamard(const void* X, int64_t ldx, void* Y, int64_t ldy, const int8_t* signs, int64_t n,
                              int64_t d, int m, int p2, int kind, hipStream_t st) {
  int log2p = 0;
  while ((1 << log2p) < p2) ++log2p;
  const float scale = 1.0f / sqrtf((float)d);
  // the Sylvester factor on the m segments of every row (p2 consecutive elements at a * p2), X -> Y:
  // contiguous rows are one matrix of n * m short rows; otherwise one launch per segment
  if (ldx == d && ldy == d && n * m < ((int64_t)1 << 31)) {
    kt_status s = dispatch_hadamard<T>(log2p, X, p2, Y, p2, signs, n * m, scale, m, st);
    if (s != KT_OK) return s;
  } else {
    for (int a = 0; a < m; ++a) {
      kt_status s = dispatch_hadamard<T>(log2p, static_cast<const T*>(X) + (int64_t)a * p2, ldx,
                                         static_cast<T*>(Y) + (int64_t)a * p2, ldy,
                                         signs ? signs + (int64_t)a * p2 : nullptr, n, scale, 1, st);
      if (s != KT_OK) return s;
    }
  }
  if (m == 1) return KT_OK;
  // the order-m factor across the segments, in place on Y
  const int64_t tiles = n * (p2 / 128);
  const int64_t wgs = tiles < 8 * kNumCUs ? tiles : 8 * kNumCUs;
  if (sizeof(T) == 2 && m >= kHadMfmaFrom) {  // bf16: exact on the matrix cores
    const int MB = (m + 31) / 32, KS = (m + 15) / 16;
    int lognb = 0;  // blocks of 32 columns per wave: as many as keep m * NBW <= 128, fit the segment and 64 KiB of LDS
    while ((2 << lognb) * m <= 128 && (256 << lognb) <= p2 && 2 * 16 * KS * (512 << lognb) <= 65536) ++lognb;
    const size_t lds = (size_t)32 * MB * 32 * KS + (size_t)16 * KS * (256 << lognb) + (size_t)32 * MB * ((256 << lognb) + 16);
    if (!ensure_dynamic_lds(reinterpret_cast<const void*>(hadamard_cross_mfma_kernel), lds))
      return fail(KT_ERR_DEVICE, "the Hadamard factor kernel needs %zu bytes of LDS per workgroup", lds);
    const int64_t tiles_m = n * (p2 / (128 << lognb));
    const int64_t wgs_m = tiles_m < 8 * kNumCUs ? tiles_m : 8 * kNumCUs;
    hipLaunchKernelGGL(hadamard_cross_mfma_kernel, dim3((unsigned)wgs_m), dim3(256), lds, st,
                       reinterpret_cast<__bf16*>(Y), ldy, n, m, p2, kind, lognb);
  } else {
    int cgroups = m >= 12 ? 1 : (m == 8 ? 2 : 4);  // as in the kernel
    while (cgroups > 1 && p2 / 128 < cgroups) cgroups /= 2;
    const size_t lds = ((size_t)m * m + 128 * (size_t)cgroups * m) * 4 + (size_t)m;
    if (!ensure_dynamic_lds(reinterpret_cast<const void*>(hadamard_cross_kernel<T>), lds))
      return fail(KT_ERR_DEVICE, "the Hadamard factor kernel needs %zu bytes of LDS per workgroup", lds);
    hipLaunchKernelGGL((hadamard_cross_kernel<T>), dim3((unsigned)wgs), dim3(256), lds, st, static_cast<T*>(Y), ldy,
                       n, m, p2, kind);
  }
  if (!launch_ok()) return fail(KT_ERR_DEVICE, "Hadamard factor launch failed");
  return KT_OK;
}

extern "C" {

int32_t kt_version(void) { return 100; }

#ifndef KT_BUILD_ID
#define KT_BUILD_ID "unknown"
#endif
const char* kt_build_id(void) { return KT_BUILD_ID; }

const char* kt_last_error(void) { return g_err; }

size_t kt_workspace_bytes(kt_op op, int64_t batch, int64_t n, int64_t d, kt_dtype x_dtype) {
  if (batch < 1 || d < 1 || d % 128 != 0) return 0;
  if (x_dtype != KT_F32 && x_dtype != KT_BF16) return 0;
  switch (op) {
    case KT_OP_LOSS_GRAD:
      if (n < 1) return 0;
      return plan_loss_grad(batch, n, d, x_dtype, false, keep_y_recommended(batch, n, d, x_dtype, false)).total;
    case KT_OP_LOSS_GRAD_RECOMPUTE:
      if (n < 1) return 0;
      return plan_loss_grad(batch, n, d, x_dtype).total;
    case KT_OP_POOLED_LOSS_GRAD:
      if (n < 1) return 0;
      return plan_loss_grad(batch, n, d, x_dtype, true, keep_y_recommended(batch, n, d, x_dtype, true)).total;
    case KT_OP_POOLED_LOSS_GRAD_RECOMPUTE:
      if (n < 1) return 0;
      return plan_loss_grad(batch, n, d, x_dtype, true).total;
    case KT_OP_QUANT_METRICS:
      if (n < 1) return 0;
      {  // R^T and, when the caller does not ask for Y, an fp32 staging slice of it
        int64_t sp, sr;
        stage_slices(batch, n, d, &sp, &sr);
        return round_up(batch * d * d * (x_dtype == KT_F32 ? 4 : 2), 256) + (size_t)sp * sr * d * 4;
      }
    case KT_OP_FUSE_ROTATION:  // n = the other dimension k of the weight
      if (n < 1) return 0;
      return round_up(d * d * 4, 256) + (size_t)n * d * 4;
    case KT_OP_SENSITIVITY:
      return (size_t)kSensBlocks * kSensSteps * 8 + 1024;
    case KT_OP_CAYLEY:
      return plan_cayley(batch, d).total;
    case KT_OP_FAKEQUANT:
      if (n < 1) return 0;
      return plan_quant(batch, n, d, x_dtype).total;
    default:
      return 0;
  }
}

kt_status kt_kurtosis_loss_grad(const void* X, int64_t ldx, const void* R, int64_t ldr,
                                int64_t batch, int64_t n, int64_t d, kt_dtype x_dtype,
                                kt_dtype r_dtype, float kappa_target, float* loss, float* row_kurt,
                                float* dR, void* workspace, size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  kt_status s = check_xr(X, ldx, R, ldr, batch, n, d, x_dtype, r_dtype);
  if (s != KT_OK) return s;
  if (!loss) return fail(KT_ERR_INVALID_ARG, "loss must not be null");
  if (!(kappa_target >= 0.f)) return fail(KT_ERR_INVALID_ARG, "kappa_target must be >= 0");
  LossGradPlan p = plan_loss_grad(batch, n, d, x_dtype);
  s = check_ws(workspace, workspace_bytes, p.total);
  if (s != KT_OK) return s;
  if (!p.fused && dR) {  // room for Y: keep it instead of recomputing it (same result)
    const LossGradPlan pk = plan_loss_grad(batch, n, d, x_dtype, false, true);
    if (workspace_bytes >= pk.total) p = pk;
  }
  char* ws = static_cast<char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (p.fused)
    return run_loss_grad_fused(p, X, ldx, R, ldr, r_dtype, batch, n, d, kappa_target, loss, row_kurt, dR,
                               ws, st);
  if (p.fp32)
    return run_loss_grad<float, TF, TF>(p, X, ldx, R, ldr, r_dtype, batch, n, d, kappa_target, loss,
                                        row_kurt, dR, ws, st);
  if (d % 256 == 0)
    return run_loss_grad<bf16, TB_BIG, TB_BIG>(p, X, ldx, R, ldr, r_dtype, batch, n, d, kappa_target,
                                               loss, row_kurt, dR, ws, st);
  return run_loss_grad<bf16, TB_M128, TB_128>(p, X, ldx, R, ldr, r_dtype, batch, n, d, kappa_target,
                                              loss, row_kurt, dR, ws, st);
}

kt_status kt_pooled_kurtosis_loss_grad(const void* X, int64_t ldx, const void* R, int64_t ldr,
                                       int64_t batch, int64_t n, int64_t d, kt_dtype x_dtype,
                                       kt_dtype r_dtype, float kappa_target, float rms_eps, float* loss,
                                       float* kappa, float* dR, void* workspace, size_t workspace_bytes,
                                       void* stream) {
  g_err[0] = 0;
  kt_status s = check_xr(X, ldx, R, ldr, batch, n, d, x_dtype, r_dtype);
  if (s != KT_OK) return s;
  if (!loss) return fail(KT_ERR_INVALID_ARG, "loss must not be null");
  if (!(kappa_target >= 0.f)) return fail(KT_ERR_INVALID_ARG, "kappa_target must be >= 0");
  if (!(rms_eps >= 0.f)) return fail(KT_ERR_INVALID_ARG, "rms_eps must be >= 0");
  LossGradPlan p = plan_loss_grad(batch, n, d, x_dtype, true);
  s = check_ws(workspace, workspace_bytes, p.total);
  if (s != KT_OK) return s;
  if (dR) {
    const LossGradPlan pk = plan_loss_grad(batch, n, d, x_dtype, true, true);
    if (workspace_bytes >= pk.total) p = pk;
  }
  char* ws = static_cast<char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  PooledArgs pa;
  pa.rms_eps = rms_eps; pa.kappa_out = kappa;
  if (p.fp32)
    return run_loss_grad<float, TF, TF>(p, X, ldx, R, ldr, r_dtype, batch, n, d, kappa_target, loss, nullptr,
                                        dR, ws, st, &pa);
  if (d % 256 == 0)
    return run_loss_grad<bf16, TB_BIG, TB_BIG>(p, X, ldx, R, ldr, r_dtype, batch, n, d, kappa_target, loss,
                                               nullptr, dR, ws, st, &pa);
  return run_loss_grad<bf16, TB_M128, TB_128>(p, X, ldx, R, ldr, r_dtype, batch, n, d, kappa_target, loss,
                                              nullptr, dR, ws, st, &pa);
}

kt_status kt_cayley_step(float* R, const float* dR, void* R_lowp, int64_t batch, int64_t d, float lr,
                         float* ortho_err, int32_t* info, void* workspace, size_t workspace_bytes,
                         void* stream) {
  g_err[0] = 0;
  if (!R || !dR) return fail(KT_ERR_INVALID_ARG, "R and dR must not be null");
  if ((reinterpret_cast<uintptr_t>(R) | reinterpret_cast<uintptr_t>(dR)) & 15)
    return fail(KT_ERR_BAD_SHAPE, "R and dR must be 16-byte aligned");
  if (batch < 1 || d < 1) return fail(KT_ERR_INVALID_ARG, "batch and d must be positive");
  if (d % 128 != 0) return fail(KT_ERR_BAD_SHAPE, "d = %lld is not a multiple of 128", (long long)d);
  if (d > 16384 || batch > 65535) return fail(KT_ERR_BAD_SHAPE, "size out of range (d <= 16384, batch <= 65535)");
  if (!(lr == lr) || lr - lr != 0.f) return fail(KT_ERR_INVALID_ARG, "lr must be finite");
  const CayleyPlan p = plan_cayley(batch, d);
  kt_status s = check_ws(workspace, workspace_bytes, p.total);
  if (s != KT_OK) return s;
  char* ws = static_cast<char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope prof(4, st);
  if (d == 128)  // whole retraction of a problem inside one workgroup (kt_cayley_d128.h)
    return launch_cayley_d128<false>(R, dR, R_lowp, batch, 0.5f * lr, ortho_err, info, C128Adam{}, st);
  return cayley_run(p, ws, R, dR, R_lowp, batch, d, 0.5f * lr, nullptr, ortho_err, info, st);
}

kt_status kt_cayley_step_static(float* R, const float* dR, void* R_lowp, int64_t batch, int64_t d, float lr,
                                float* ortho_err, int32_t* info, void* stream) {
  g_err[0] = 0;
  if (!R || !dR) return fail(KT_ERR_INVALID_ARG, "R and dR must not be null");
  if (batch < 1 || d < 1) return fail(KT_ERR_INVALID_ARG, "batch and d must be positive");
  if (d % 128 != 0) return fail(KT_ERR_BAD_SHAPE, "d = %lld is not a multiple of 128", (long long)d);
  if (d > 16384 || batch > 65535) return fail(KT_ERR_BAD_SHAPE, "size out of range (d <= 16384, batch <= 65535)");
  if (!(lr == lr) || lr - lr != 0.f) return fail(KT_ERR_INVALID_ARG, "lr must be finite");
  const size_t need = plan_cayley(batch, d).total;
  if (need > kStaticScratchBytes)
    return fail(KT_ERR_NOT_SUPPORTED,
                "batch = %lld, d = %lld needs %zu bytes of scratch; the library's static scratch holds %zu "
                "(use kt_cayley_step with a workspace)", (long long)batch, (long long)d, need, kStaticScratchBytes);
  void* ws = static_scratch_of_current_device();
  if (!ws) return KT_ERR_DEVICE;
  // same checks, plan and launches as the workspace form; the fixed point clears its own counters
  // with a fill kernel, so whatever the previous call left in the array does not matter
  return kt_cayley_step(R, dR, R_lowp, batch, d, lr, ortho_err, info, ws, kStaticScratchBytes, stream);
}

kt_status kt_cayley_adam_step(float* R, const float* dR, float* M, float* v, int64_t step, void* R_lowp,
                              int64_t batch, int64_t d, float lr, float beta1, float beta2, float eps, float q,
                              float* ortho_err, int32_t* info, float* scalars, void* workspace,
                              size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  if (!R || !dR || !M || !v) return fail(KT_ERR_INVALID_ARG, "R, dR, M and v must not be null");
  if ((reinterpret_cast<uintptr_t>(R) | reinterpret_cast<uintptr_t>(dR) | reinterpret_cast<uintptr_t>(M)) & 15)
    return fail(KT_ERR_BAD_SHAPE, "R, dR and M must be 16-byte aligned");
  if (batch < 1 || d < 1) return fail(KT_ERR_INVALID_ARG, "batch and d must be positive");
  if (d % 128 != 0) return fail(KT_ERR_BAD_SHAPE, "d = %lld is not a multiple of 128", (long long)d);
  if (d > 16384 || batch > 65535) return fail(KT_ERR_BAD_SHAPE, "size out of range (d <= 16384, batch <= 65535)");
  if (step < 1) return fail(KT_ERR_INVALID_ARG, "step counts from 1");
  if (!(lr == lr) || lr - lr != 0.f) return fail(KT_ERR_INVALID_ARG, "lr must be finite");
  if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f))
    return fail(KT_ERR_INVALID_ARG, "beta1 and beta2 must lie in [0, 1)");
  if (!(eps >= 0.f) || !(q > 0.f)) return fail(KT_ERR_INVALID_ARG, "eps must be >= 0 and q > 0");
  const CayleyPlan p = plan_cayley(batch, d);
  kt_status s = check_ws(workspace, workspace_bytes, p.total);
  if (s != KT_OK) return s;
  char* ws = static_cast<char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope prof(4, st);
  const double c1 = 1.0 - pow((double)beta1, (double)step), c2 = 1.0 - pow((double)beta2, (double)step);
  if (d == 128) {
    C128Adam ad;
    ad.M = M; ad.v = v; ad.scalars_out = scalars; ad.lr = lr; ad.beta1 = beta1; ad.beta2 = beta2;
    ad.eps = eps; ad.q = q; ad.c1 = c1; ad.c2 = c2;
    return launch_cayley_d128<true>(R, dR, R_lowp, batch, 0.5f, ortho_err, info, ad, st);
  }
  AdamArgs a;
  a.M = M; a.lr = lr; a.q = q; a.eps = eps; a.scalars_out = scalars;
  a.scal = reinterpret_cast<float*>(ws + p.o_scal);
  a.sq_part = reinterpret_cast<double*>(ws + p.o_sq);
  double* g2_part = reinterpret_cast<double*>(ws + p.o_g2);
  hipLaunchKernelGGL(adam_moment_kernel, dim3((unsigned)p.g2_blocks, (unsigned)batch), dim3(256), 0, st, M, dR,
                     d * d, beta1, g2_part);
  hipLaunchKernelGGL(adam_scalars1_kernel, dim3((unsigned)batch), dim3(256), 0, st, g2_part, p.g2_blocks, v, beta2,
                     c1, c2, eps, a.scal);
  if (!launch_ok()) return fail(KT_ERR_DEVICE, "Cayley Adam moment launch failed");
  // P = M1 R^T, S = (P - P^T)/2 (= r W for orthogonal R), then the transform with c = alpha/(2r)
  return cayley_run(p, ws, R, M, R_lowp, batch, d, 0.5f, &a, ortho_err, info, st);
}

kt_status kt_rotate_fakequant_int4(const void* X, int64_t ldx, const void* R, int64_t ldr,
                                   int64_t batch, int64_t n, int64_t d, kt_dtype x_dtype,
                                   kt_dtype r_dtype, float clip_ratio, const float* scales_in,
                                   float* scales_out, int8_t* codes, float* err, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  kt_status s = check_xr(X, ldx, R, ldr, batch, n, d, x_dtype, r_dtype);
  if (s != KT_OK) return s;
  if (!(clip_ratio > 0.f && clip_ratio <= 1.f))
    return fail(KT_ERR_INVALID_ARG, "clip_ratio must be in (0, 1]");
  if (!scales_out && !codes && !err) return fail(KT_ERR_INVALID_ARG, "no output requested");
  if (reinterpret_cast<uintptr_t>(codes) & 15) return fail(KT_ERR_BAD_SHAPE, "codes must be 16-byte aligned");
  const QuantPlan p = plan_quant(batch, n, d, x_dtype);
  s = check_ws(workspace, workspace_bytes, p.total);
  if (s != KT_OK) return s;
  char* ws = static_cast<char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope prof(5, st);
  if (!p.fp32 && d == 128) {  // one pass over X (kt_fused_d128.h)
    bf16* RT = reinterpret_cast<bf16*>(ws + p.o_rt);
    if (!prep_rt<bf16>(R, ldr, r_dtype, RT, batch, d, st)) return fail(KT_ERR_DEVICE, "prep_rt launch failed");
    const int64_t tiles = ceil_div(n, 32);
    int64_t wgs = ceil_div(4 * kNumCUs, batch);  // about four workgroups per CU over all problems
    if (wgs > ceil_div(tiles, 4)) wgs = ceil_div(tiles, 4);
    hipLaunchKernelGGL(quant_d128_kernel, dim3((unsigned)wgs, (unsigned)batch), dim3(256), 0, st,
                       static_cast<const bf16*>(X), ldx, n * ldx, RT, (int)n, clip_ratio, scales_in, scales_out, codes,
                       reinterpret_cast<float2*>(err));
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "d=128 fake-quant launch failed");
    return KT_OK;
  }
  if (p.fp32)
    return run_quant<float, TF, TF>(p, X, ldx, R, ldr, r_dtype, batch, n, d, clip_ratio, scales_in,
                                    scales_out, codes, err, ws, st);
  if (d % 256 == 0)
    return run_quant<bf16, TB_BIG, TB_BIG>(p, X, ldx, R, ldr, r_dtype, batch, n, d, clip_ratio, scales_in,
                                           scales_out, codes, err, ws, st);
  return run_quant<bf16, TB_M128, TB_N128>(p, X, ldx, R, ldr, r_dtype, batch, n, d, clip_ratio, scales_in,
                                           scales_out, codes, err, ws, st);
}

kt_status kt_rotate_quant_metrics(const void* X, int64_t ldx, const void* R, int64_t ldr, int64_t batch,
                                  int64_t n, int64_t d, kt_dtype x_dtype, kt_dtype r_dtype, float quantile,
                                  float* Y, float* amax, float* threshold, float* err_sym, float* err_asym,
                                  int64_t* success, void* workspace, size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  kt_status s = check_xr(X, ldx, R, ldr, batch, n, d, x_dtype, r_dtype);
  if (s != KT_OK) return s;
  if (!(quantile > 0.f && quantile <= 1.f)) return fail(KT_ERR_INVALID_ARG, "quantile must be in (0, 1]");
  if (d > 8192) return fail(KT_ERR_NOT_SUPPORTED, "quantisation metrics keep a token row in registers: d <= 8192");
  const bool fp32 = x_dtype == KT_F32;
  const size_t rt_bytes = (size_t)round_up(batch * d * d * (fp32 ? 4 : 2), 256);
  // With Y wanted the whole rotation is one launch pair into the caller's buffer; without it Y passes through
  // a bounded staging slice, some problems or some token rows of one problem at a time.
  int64_t sp = batch, sr = n;
  if (!Y) stage_slices(batch, n, d, &sp, &sr);
  const size_t need = rt_bytes + (Y ? 0 : (size_t)sp * sr * d * 4);
  s = check_ws(workspace, workspace_bytes, need);
  if (s != KT_OK) return s;
  char* ws = static_cast<char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* Yb = Y ? Y : reinterpret_cast<float*>(ws + rt_bytes);
  ProfScope prof(5, st);
  // Y = X R, token-major (tokens on the rows of the GEMM): Y never feeds another GEMM here, the
  // row kernel wants whole token rows
  auto rotate = [&](auto t_tag, auto tile_tag) -> kt_status {
    using T = decltype(t_tag);
    using TL = decltype(tile_tag);
    T* RT = reinterpret_cast<T*>(ws);
    const T* Xp = static_cast<const T*>(X);
    if (!prep_rt<T>(R, ldr, r_dtype, RT, batch, d, st)) return fail(KT_ERR_DEVICE, "prep_rt launch failed");
    if (success) {
      hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(256), 0, st, reinterpret_cast<unsigned*>(success),
                         2 * batch, 0u);
    }
    for (int64_t b0 = 0; b0 < batch; b0 += sp) {
      const int64_t nb = batch - b0 < sp ? batch - b0 : sp;
      for (int64_t t0 = 0; t0 < n; t0 += sr) {
        const int64_t nt = n - t0 < sr ? n - t0 : sr, row0 = b0 * n + t0;
        EpiStore<TL> e;
        e.C = Yb; e.ldc = d; e.batch_stride = nt * d; e.split_stride = 0; e.M = (int)nt; e.N = (int)d;
        if (!launch_gemm<TL>(Xp + row0 * ldx, ldx, n * ldx, (int)nt, RT + b0 * d * d, d, d * d, (int)d, d, 0, (int)nb,
                             e, st))
          return fail(KT_ERR_DEVICE, "rotation GEMM launch failed");
        // the row in 4 / 8 / 16 / 32 float4 registers per lane; rows that fill them exactly skip every bounds test
        auto rows_kernel = d == 1024   ? quant_metrics_row_kernel<T, 4, true>
                           : d < 1024  ? quant_metrics_row_kernel<T, 4, false>
                           : d == 2048 ? quant_metrics_row_kernel<T, 8, true>
                           : d < 2048  ? quant_metrics_row_kernel<T, 8, false>
                           : d == 4096 ? quant_metrics_row_kernel<T, 16, true>
                           : d < 4096  ? quant_metrics_row_kernel<T, 16, false>
                           : d == 8192 ? quant_metrics_row_kernel<T, 32, true>
                                       : quant_metrics_row_kernel<T, 32, false>;
        const int64_t row_wgs = ceil_div(nt, 4) < ceil_div(16 * kNumCUs, nb) ? ceil_div(nt, 4) : ceil_div(16 * kNumCUs, nb);
        hipLaunchKernelGGL(rows_kernel, dim3((unsigned)row_wgs, (unsigned)nb), dim3(256), 0, st, Yb,
                           Xp + row0 * ldx, ldx, n * ldx, (int)nt, (int)d, (double)quantile,
                           amax ? amax + 2 * row0 : nullptr, threshold ? threshold + row0 : nullptr,
                           err_sym ? err_sym + 2 * row0 : nullptr, err_asym ? err_asym + 2 * row0 : nullptr,
                           success ? reinterpret_cast<unsigned long long*>(success) + b0 : nullptr);
        if (!launch_ok()) return fail(KT_ERR_DEVICE, "metrics kernel launch failed");
      }
    }
    return KT_OK;
  };
  if (fp32) return rotate(float{}, TF{});
  if (d % 256 == 0) return rotate(bf16{}, TB_BIG{});
  return rotate(bf16{}, TB_N128{});
}

kt_status kt_hadamard_rows(const void* X, int64_t ldx, void* Y, int64_t ldy, const int8_t* signs, int64_t n,
                           int64_t d, kt_dtype dtype, void* stream) {
  g_err[0] = 0;
  if (!X || !Y) return fail(KT_ERR_INVALID_ARG, "X and Y must not be null");
  if (n < 1) return fail(KT_ERR_INVALID_ARG, "n must be positive");
  if (dtype != KT_F32 && dtype != KT_BF16) return fail(KT_ERR_BAD_DTYPE, "dtype must be KT_F32 or KT_BF16");
  int m = 0, p2 = 0, kind = 0;
  if (d < 128 || d > 524288 || !hadamard_split(d, &m, &p2, &kind) || p2 < 128 || p2 > 4096 || m > 128)
    return fail(KT_ERR_BAD_SHAPE,
                "d = %lld: the Hadamard transform here needs d = m 2^k with 128 <= 2^k <= 4096 and m = 1, a power "
                "of two or a Paley order (q + 1 or 2 (q + 1), q prime) up to 128",
                (long long)d);
  const int64_t vec = dtype == KT_F32 ? 4 : 8;
  if (ldx < d || ldy < d || ldx % vec != 0 || ldy % vec != 0)
    return fail(KT_ERR_BAD_SHAPE, "ldx / ldy must be >= d and keep rows 16-byte aligned");
  if ((reinterpret_cast<uintptr_t>(X) | reinterpret_cast<uintptr_t>(Y)) & 15)
    return fail(KT_ERR_BAD_SHAPE, "X and Y must be 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  ProfScope prof(5, st);
  if (dtype == KT_F32) return run_hadamard<float>(X, ldx, Y, ldy, signs, n, d, m, p2, kind, st);
  return run_hadamard<bf16>(X, ldx, Y, ldy, signs, n, d, m, p2, kind, st);
}

kt_status kt_fuse_rotation(const float* W, int64_t ldw, const float* R, int64_t ldr, float* Wout, int64_t ldo,
                           int64_t k, int64_t d, int32_t side, void* workspace, size_t workspace_bytes,
                           void* stream) {
  g_err[0] = 0;
  if (!W || !R || !Wout) return fail(KT_ERR_INVALID_ARG, "W, R and Wout must not be null");
  if (k < 1 || d < 1) return fail(KT_ERR_INVALID_ARG, "k and d must be positive");
  if (side != 0 && side != 1) return fail(KT_ERR_INVALID_ARG, "side must be 0 (W R) or 1 (R^T W)");
  if (d % 128 != 0 || d > 16384) return fail(KT_ERR_BAD_SHAPE, "d = %lld is not a multiple of 128 (<= 16384)", (long long)d);
  if (k > (int64_t(1) << 22)) return fail(KT_ERR_BAD_SHAPE, "k out of range");
  const int64_t wcols = side == 0 ? d : k;
  if (ldw < wcols || ldo < wcols || ldr < d || ldw % 4 != 0 || ldo % 4 != 0 || ldr % 4 != 0)
    return fail(KT_ERR_BAD_SHAPE, "leading dimensions must cover the rows and keep them 16-byte aligned");
  if (side == 1 && k % 4 != 0) return fail(KT_ERR_BAD_SHAPE, "k must be a multiple of 4 for side 1");
  const size_t rt_bytes = (size_t)round_up(d * d * 4, 256);
  kt_status s = check_ws(workspace, workspace_bytes, rt_bytes + (side == 1 ? (size_t)k * d * 4 : 0));
  if (s != KT_OK) return s;
  char* ws = static_cast<char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* RT = reinterpret_cast<float*>(ws);
  if (!prep_rt<float>(R, ldr, KT_F32, RT, 1, d, st)) return fail(KT_ERR_DEVICE, "prep_rt launch failed");
  ProfScope prof(5, st);
  EpiStore<TF> e;
  e.C = Wout; e.ldc = ldo; e.batch_stride = 0; e.split_stride = 0;
  if (side == 0) {  // Wout [k][d] = W R = W (R^T)^T
    e.M = (int)k; e.N = (int)d;
    if (!launch_gemm<TF>(W, ldw, 0, (int)k, RT, d, 0, (int)d, d, 0, 1, e, st))
      return fail(KT_ERR_DEVICE, "fusion GEMM launch failed");
  } else {          // Wout [d][k] = R^T W = R^T (W^T)^T
    float* Wt = reinterpret_cast<float*>(ws + rt_bytes);
    hipLaunchKernelGGL(transpose_f32_kernel, dim3((unsigned)ceil_div(k, 32), (unsigned)ceil_div(d, 32)), dim3(256),
                       0, st, W, ldw, Wt, d, (int)d, (int)k);
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "weight transpose launch failed");
    e.M = (int)d; e.N = (int)k;
    if (!launch_gemm<TF>(RT, d, 0, (int)d, Wt, d, 0, (int)k, d, 0, 1, e, st))
      return fail(KT_ERR_DEVICE, "fusion GEMM launch failed");
  }
  return KT_OK;
}

kt_status kt_quant_sensitivity(const float* Y, int64_t count, int32_t bits, const float* alphas, int32_t n_alpha,
                               float* out, float* gamma, void* workspace, size_t workspace_bytes, void* stream) {
  g_err[0] = 0;
  if (!Y || !out) return fail(KT_ERR_INVALID_ARG, "Y and out must not be null");
  if (count < 1) return fail(KT_ERR_INVALID_ARG, "count must be positive");
  if (bits < 2 || bits > 8) return fail(KT_ERR_INVALID_ARG, "bits must be in [2, 8]");
  if (n_alpha < 0 || n_alpha > kSensSteps - 1) return fail(KT_ERR_INVALID_ARG, "at most 31 step fractions");
  if (n_alpha > 0 && (!alphas || !gamma)) return fail(KT_ERR_INVALID_ARG, "alphas and gamma must not be null");
  const size_t need = (size_t)kSensBlocks * kSensSteps * 8 + 1024;
  kt_status s = check_ws(workspace, workspace_bytes, need);
  if (s != KT_OK) return s;
  char* ws = static_cast<char*>(workspace);
  hipStream_t st = static_cast<hipStream_t>(stream);
  double* part = reinterpret_cast<double*>(ws);
  double* dst = reinterpret_cast<double*>(ws + (size_t)kSensBlocks * kSensSteps * 8);
  float* stt = reinterpret_cast<float*>(ws + (size_t)kSensBlocks * kSensSteps * 8 + 64);
  const float L = (float)((1 << (bits - 1)) - 1);
  const int nblocks = (int)(ceil_div(count, 256) < kSensBlocks ? ceil_div(count, 256) : kSensBlocks);
  ProfScope prof(5, st);
  hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(256), 0, st, reinterpret_cast<unsigned*>(stt), 64, 0u);
  hipLaunchKernelGGL(sens_amax_kernel, dim3(nblocks), dim3(256), 0, st, Y, count,
                     reinterpret_cast<unsigned*>(stt + 35));
  hipLaunchKernelGGL(sens_select_kernel, dim3(1), dim3(256), 0, st, part, nblocks, 0, count, -1, L, stt, dst, alphas,
                     (int)n_alpha, out, gamma);
  if (!launch_ok()) return fail(KT_ERR_DEVICE, "sensitivity set-up launch failed");
  for (int round = 0; round < 4; ++round) {
    const int ns = round < 3 ? kSensSteps : 1 + n_alpha;
    hipLaunchKernelGGL(sens_sweep_kernel, dim3(nblocks, (unsigned)ceil_div(ns, kSensPerBlock)), dim3(256), 0, st, Y, count, stt,
                       ns, L, part);
    hipLaunchKernelGGL(sens_select_kernel, dim3(1), dim3(256), 0, st, part, nblocks, ns, count, round, L, stt, dst,
                       alphas, (int)n_alpha, out, gamma);
    if (!launch_ok()) return fail(KT_ERR_DEVICE, "sensitivity sweep launch failed");
  }
  return KT_OK;
}

#ifdef KT_PHASE_STAMPS
// Developer build only: arm the phase stamps (the next kStampSlots GEMM launches record into slots 0, 1, ...) and
// read them back (synchronises the device).
void kt_debug_stamps_arm(void) { g_stamp_next = 0; }
int kt_debug_stamps_read(void* host_dst, size_t bytes) {
  g_stamp_next = -1;
  if (hipDeviceSynchronize() != hipSuccess) return -1;
  const size_t all = sizeof(unsigned long long) * kStampSlots * kStampWgs * kStampWords;
  return hipMemcpyFromSymbol(host_dst, HIP_SYMBOL(g_phase_stamps), bytes < all ? bytes : all) == hipSuccess ? 0 : -1;
}
#endif

kt_status kt_profile_reset(void) {
  g_prof_used.store(0);
  return KT_OK;
}

kt_status kt_profile_enable(int32_t max_records) {
  g_err[0] = 0;
  if (max_records < 0) return fail(KT_ERR_INVALID_ARG, "max_records must be >= 0");
  for (int i = 0; i < g_prof_cap; ++i) {
    (void)hipEventDestroy(g_prof[i].start);
    (void)hipEventDestroy(g_prof[i].stop);
  }
  delete[] g_prof;
  g_prof = nullptr;
  g_prof_cap = 0;
  g_prof_used.store(0);
  if (max_records == 0) return KT_OK;
  g_prof = new (std::nothrow) ProfRecord[max_records];  // no exception may cross the C boundary
  if (!g_prof) return fail(KT_ERR_INVALID_ARG, "cannot hold %d profile records", (int)max_records);
  for (int i = 0; i < max_records; ++i) {
    if (hipEventCreate(&g_prof[i].start) != hipSuccess || hipEventCreate(&g_prof[i].stop) != hipSuccess)
      return fail(KT_ERR_DEVICE, "hipEventCreate failed");
    g_prof_cap = i + 1;
  }
  return KT_OK;
}

kt_status kt_profile_read(int32_t kernel_id, double* total_ms, int32_t* launches) {
  g_err[0] = 0;
  if (!total_ms || !launches) return fail(KT_ERR_INVALID_ARG, "outputs must not be null");
  double tot = 0.0;
  int cnt = 0;
  const int used = g_prof_used.load() < g_prof_cap ? g_prof_used.load() : g_prof_cap;
  for (int i = 0; i < used; ++i) {
    if (g_prof[i].id != kernel_id) continue;
    if (hipEventSynchronize(g_prof[i].stop) != hipSuccess) return fail(KT_ERR_DEVICE, "event sync failed");
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, g_prof[i].start, g_prof[i].stop) != hipSuccess)
      return fail(KT_ERR_DEVICE, "event elapsed failed");
    tot += ms;
    ++cnt;
  }
  *total_ms = tot;
  *launches = cnt;
  return KT_OK;
}

}  // extern "C"
