// C ABI of libprac (see include/prac.h): argument checks, scratch planning and the
// sequence of kernel launches behind each entry point.
#include <algorithm>
#include <new>

#include "prac_internal.h"

// Scratch of the entry point that allocates nothing (prac_weight_grad_static): one block per GPU,
// part of the code object, held until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress; prac_create asks for the block's device address once per
// device (with that device current) and everything else uses that address.
static __device__ __align__(256) unsigned char scratch[PRAC_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = PRAC_MAX_DEVICES;
char* g_static_scratch[kMaxDevices] = {};  // device address of `scratch` on each GPU, set by prac_create

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline size_t esize(prac_dtype t) { return t == PRAC_BF16 ? 2 : 4; }
inline bool valid_dtype(int t) { return t == PRAC_F32 || t == PRAC_BF16; }
// token counts are 32-bit inside the kernels' launch arguments
inline bool bad_tokens(int64_t N) { return N < 1 || N >= ((int64_t)1 << 31); }

struct LpLayout {
  int64_t ldpt, ldpn;
  int nkb, ncb;  // fragment-order copy: 16-row blocks over round_up(d,256), 32-column blocks (multiple of 8)
  int nrb, nckb; // A-operand fragment copy: 32-row blocks over round_up(d,128), 16-column blocks over c
  size_t off_pn, off_pf, off_pa, bytes;
};
inline LpLayout lp_layout(int64_t d, int c) {
  LpLayout l;
  l.ldpt = round_up64(d, 64);
  l.ldpn = round_up64(c, 64);
  l.nkb = (int)(round_up64(d, 256) / 16);
  l.ncb = (int)round_up64((c + 31) / 32, 8);
  l.off_pn = ((size_t)c * l.ldpt * sizeof(bf16_t) + 255) & ~size_t(255);
  l.off_pf = (l.off_pn + (size_t)d * l.ldpn * sizeof(bf16_t) + 255) & ~size_t(255);
  l.nrb = (int)(round_up64(d, 128) / 32);
  l.nckb = (c + 15) / 16;
  l.off_pa = (l.off_pf + (size_t)l.nkb * l.ncb * 64 * 8 * sizeof(bf16_t) + 255) & ~size_t(255);
  l.bytes = l.off_pa + (size_t)l.nrb * l.nckb * 64 * 8 * sizeof(bf16_t);
  return l;
}
inline size_t packed_c_bytes(int64_t N, int c) {
  return (size_t)((N + 127) / 128) * 8 * ((c + 31) / 32) * 64 * 8 * sizeof(bf16_t);  // whole 128-token tiles
}

// split count for a reduction over K with `tiles` output tiles: fill the chip about
// twice over without making slabs shorter than `min_k`.
inline int pick_splits(int tiles, int64_t K, int n_cu, int min_k) {
  int s = (2 * n_cu + tiles - 1) / tiles;
  const int64_t cap = K / min_k;
  if (s > cap) s = (int)cap;
  if (s > 64) s = 64;
  return s < 1 ? 1 : s;
}

}  // namespace

int prac_ws_reserve(prac_ctx* ctx, size_t bytes) {
  if (bytes <= ctx->ws_bytes) return PRAC_OK;
  // Work already enqueued may still read the old block (on the ctx stream, or on a stream the ctx
  // was bound to earlier): wait for the device before replacing it.  Callers that must not wait
  // size the block up front (prac_workspace_bytes, prac_reserve_workspace).
  PRAC_HIP_TRY(ctx, hipDeviceSynchronize());
  if (ctx->ws) PRAC_HIP_TRY(ctx, hipFree(ctx->ws));
  ctx->ws = nullptr;
  ctx->ws_bytes = 0;
  const size_t want = bytes + bytes / 4;
  void* p = nullptr;
  hipError_t e = hipMalloc(&p, want);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    e = hipMalloc(&p, bytes);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      ctx->last_hip = (int)e;
      return PRAC_ENOMEM;
    }
    ctx->ws_bytes = bytes;
  } else {
    ctx->ws_bytes = want;
  }
  ctx->ws = reinterpret_cast<char*>(p);
  return PRAC_OK;
}

ProfScope::ProfScope(prac_ctx* c, int kind) : ctx(c) {
  c->ev_start = nullptr;
  c->ev_stop = nullptr;
  if (c->prof_kind != kind || kind == 0) return;
  if (c->prof_seen++ % c->prof_stride != 0) return;
  hipEvent_t ev[2] = {nullptr, nullptr};
  for (int i = 0; i < 2; ++i) {
    if (!c->prof_pool.empty()) {
      ev[i] = c->prof_pool.back();
      c->prof_pool.pop_back();
    } else if (hipEventCreate(&ev[i]) != hipSuccess) {
      (void)hipGetLastError();
      if (i == 1) c->prof_pool.push_back(ev[0]);
      return;
    }
  }
  c->prof_pairs.emplace_back(ev[0], ev[1]);
  c->ev_start = ev[0];
  c->ev_stop = ev[1];
}
ProfScope::~ProfScope() {
  // a launcher that did not take the pair leaves it unrecorded; prac_profile_read skips it
  ctx->ev_start = nullptr;
  ctx->ev_stop = nullptr;
}

namespace {
inline bool gram_fast(const void* X, prac_dtype xdt, int64_t rows, int64_t ldx, int64_t row_stride) {
  return xdt == PRAC_BF16 && aligned16(X) && ldx % 8 == 0 && rows < ((int64_t)1 << 31) &&
         ldx * (row_stride > 0 ? row_stride : 1) <= PRAC_MAX_STREAM_PITCH;
}
inline int gram_splits(int n_cu, int64_t d, int64_t rows) {
  const int tiles = (int)(((d + 127) / 128) * ((d + 127) / 128));
  return pick_splits(tiles, rows, n_cu, 512);
}
}  // namespace

namespace {
// Large Gram matrices run on the C^T dY kernel with X in both places (its streaming rate at
// d = 2048 is 2.5 times that of the tiled GEMM): X is first copied into the packed layout the
// kernel reads its C operand from.
inline bool gram_streaming(int64_t rows, int64_t d) { return rows >= 2048 && d >= 256; }
inline int gram_stream_splits(int n_cu, int64_t d, int64_t rows) {
  const int64_t tiles = ((d + 127) / 128) * ((d + 255) / 256);
  int64_t s = n_cu / tiles;
  if (s > rows / 256) s = rows / 256;
  if (s > 64) s = 64;
  return s < 1 ? 1 : (int)s;
}
struct GramPlan {
  bool streaming;
  int splits;
  size_t o_part, o_g, o_pack, bytes;
};
inline GramPlan plan_gram(int n_cu, int64_t rows, int64_t d, int64_t ldg) {
  GramPlan g{};
  g.streaming = gram_streaming(rows, d);
  g.splits = g.streaming ? gram_stream_splits(n_cu, d, rows) : gram_splits(n_cu, d, rows);
  WsPlan plan;
  g.o_part = plan.take(g.splits > 1 ? (size_t)g.splits * d * d * sizeof(float) : 0);
  g.o_g = plan.take(ldg == d ? 0 : (size_t)d * d * sizeof(float));
  g.o_pack = plan.take(g.streaming ? packed_c_bytes(rows, (int)d) : 0);
  g.bytes = plan.off;
  return g;
}
}  // namespace

size_t gram_scratch_bytes(int n_cu, const void* X, prac_dtype xdt, int64_t N, int64_t d, int64_t ldx,
                          int64_t row_stride, int64_t ldg) {
  const int64_t rows = (N + row_stride - 1) / row_stride;
  if (!gram_fast(X, xdt, rows, ldx, row_stride)) return 0;
  return plan_gram(n_cu, rows, d, ldg).bytes;
}

// G = Xs^T Xs with all scratch taken from `scratch` (gram_scratch_bytes of it).
int gram_device(prac_ctx* ctx, const void* X, prac_dtype xdt, int64_t N, int64_t d, int64_t ldx, int64_t row_stride,
                float* G, int64_t ldg, char* scratch) {
  const int64_t rows = (N + row_stride - 1) / row_stride;
  if (gram_fast(X, xdt, rows, ldx, row_stride)) {
    const GramPlan gp = plan_gram(ctx->n_cu, rows, d, ldg);
    const int splits = gp.splits;
    const size_t o_part = gp.o_part, o_g = gp.o_g;
    float* dense = ldg == d ? G : reinterpret_cast<float*>(scratch + o_g);
    float* partial = splits > 1 ? reinterpret_cast<float*>(scratch + o_part) : nullptr;
    int rc;
    if (gp.streaming) {
      const bf16_t* Xb = reinterpret_cast<const bf16_t*>(X);
      bf16_t* Xpk = reinterpret_cast<bf16_t*>(scratch + gp.o_pack);
      const int64_t ld = ldx * row_stride;
      rc = launch_pack_c(ctx, Xb, ld, (int)rows, (int)d, Xpk);
      if (rc) return rc;
      const int dm = (int)d;
      float* out = splits > 1 ? partial : dense;
      {
        ProfScope ps(ctx, PRAC_KERNEL_GRAM);
        rc = launch_ctdy_ws(ctx, Xpk, dm, (int)rows, 1, &Xb, &ld, &dm, &out, splits);
      }
      if (rc) return rc;
    } else {
      GemmBf16Args g{};
      g.A = reinterpret_cast<const bf16_t*>(X);
      g.lda = ldx * row_stride;
      g.M = (int)d;
      g.K = (int)rows;
      g.a_kc = false;
      g.b_kc = false;
      g.b0 = GemmOperandB{reinterpret_cast<const bf16_t*>(X), ldx * row_stride, (int)d, dense, d};
      g.b1 = GemmOperandB{nullptr, 0, 0, nullptr, 0};
      g.out_bf16 = false;
      g.beta = 0.f;
      g.splits = splits;
      g.partial = partial;
      g.tile_hint = 0;
      ProfScope ps(ctx, PRAC_KERNEL_GRAM);
      rc = launch_gemm_bf16(ctx, g);
      if (rc) return rc;
    }
    if (splits > 1) {
      rc = launch_reduce_slabs(ctx, partial, splits, (int64_t)d * d, dense, (int64_t)d * d, 1.f, 0.f);
      if (rc) return rc;
    }
    if (dense != G) return launch_cast_out(ctx, dense, d, G, PRAC_F32, ldg, (int)d, (int)d, 0.f);
    return PRAC_OK;
  }
  GemmGenArgs g{};
  g.A = X; g.B = X; g.adt = xdt; g.bdt = xdt;
  g.a_rs = 1; g.a_cs = ldx; g.b_rs = ldx; g.b_cs = 1;
  g.M = (int)d; g.N = (int)d; g.K = N; g.k_stride = row_stride;
  g.out = G; g.ldo = ldg; g.alpha = 1.f; g.beta = 0.f; g.acc64 = false; g.out64 = nullptr;
  return launch_gemm_generic(ctx, g);
}

extern "C" {

const char* prac_strerror(int s) {
  switch (s) {
    case PRAC_OK: return "ok";
    case PRAC_EINVAL: return "invalid argument";
    case PRAC_ENOMEM: return "out of device memory";
    case PRAC_EHIP: return "HIP runtime error";
    case PRAC_ENUMERIC: return "numeric breakdown";
    case PRAC_EUNSUPPORTED: return "unsupported request";
    case PRAC_ENOCTX: return "null context";
    case PRAC_ETOOBIG: return "request needs more scratch than the static block holds";
    default: return "unknown status";
  }
}

int prac_create(prac_ctx** out, int device, void* hip_stream) {
  if (!out || device < 0) return PRAC_EINVAL;
  *out = nullptr;
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) {
    (void)hipGetLastError();
    return PRAC_EHIP;
  }
  if (hipSetDevice(device) != hipSuccess) return PRAC_EHIP;
  prac_ctx* c = new (std::nothrow) prac_ctx();
  if (!c) return PRAC_ENOMEM;
  c->device = device;
  c->stream = reinterpret_cast<hipStream_t>(hip_stream);
  c->ws = nullptr;
  c->ws_bytes = 0;
  c->d_flag = nullptr;
  c->last_hip = 0;
  c->prof_kind = 0;
  c->prof_stride = 1;
  c->prof_seen = 0;
  c->ev_start = nullptr;
  c->ev_stop = nullptr;
  c->tune_splits = 0;
  c->tune_one_launch = 0;
  c->tune_tail = 0;
  c->d_sync = nullptr;
  hipDeviceProp_t prop;
  c->n_cu = (hipGetDeviceProperties(&prop, device) == hipSuccess) ? prop.multiProcessorCount : 256;
  // failure flag (256 bytes) followed by the counters of the one-launch weight gradient
  const size_t flag_bytes = 256 + PRAC_SYNC_BYTES;
  if (hipMalloc(reinterpret_cast<void**>(&c->d_flag), flag_bytes) != hipSuccess) {
    (void)hipGetLastError();
    delete c;
    return PRAC_EHIP;
  }
  c->d_sync = c->d_flag + 64;
  if (hipMemset(c->d_flag, 0, flag_bytes) != hipSuccess) {
    (void)hipGetLastError();
    (void)hipFree(c->d_flag);
    delete c;
    return PRAC_EHIP;
  }
  // address of this device's copy of the static scratch block (the device is current here)
  c->static_scratch = device < kMaxDevices ? g_static_scratch[device] : nullptr;
  if (!c->static_scratch) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
      (void)hipGetLastError();
      (void)hipFree(c->d_flag);
      delete c;
      return PRAC_EHIP;
    }
    c->static_scratch = reinterpret_cast<char*>(p);
    if (device < kMaxDevices) g_static_scratch[device] = c->static_scratch;
  }
  *out = c;
  return PRAC_OK;
}

int prac_destroy(prac_ctx* ctx) {
  if (!ctx) return PRAC_ENOCTX;
  (void)hipStreamSynchronize(ctx->stream);
  if (ctx->ws) (void)hipFree(ctx->ws);
  if (ctx->d_flag) (void)hipFree(ctx->d_flag);
  for (auto& pr : ctx->prof_pairs) {
    (void)hipEventDestroy(pr.first);
    (void)hipEventDestroy(pr.second);
  }
  for (auto& ev : ctx->prof_pool) (void)hipEventDestroy(ev);
  delete ctx;
  return PRAC_OK;
}

int prac_set_stream(prac_ctx* ctx, void* hip_stream) {
  if (!ctx) return PRAC_ENOCTX;
  ctx->stream = reinterpret_cast<hipStream_t>(hip_stream);
  return PRAC_OK;
}

int prac_sync_status(prac_ctx* ctx) {
  if (!ctx) return PRAC_ENOCTX;
  int flag = 0;
  PRAC_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  PRAC_HIP_TRY(ctx, hipMemcpy(&flag, ctx->d_flag, sizeof(int), hipMemcpyDeviceToHost));
  if (flag != 0) {
    PRAC_HIP_TRY(ctx, hipMemset(ctx->d_flag, 0, sizeof(int)));
    if (flag & 4) {
      // a wait between workgroups of the one-launch weight gradient gave up: its counters may be left
      // non-zero, clear them for the next launch  (bits 1 and 2 are the basis fit's: a pivot that was
      // not positive or a basis that did not come out orthonormal, an eigen-iteration that did not settle)
      PRAC_HIP_TRY(ctx, hipMemset(ctx->d_sync, 0, PRAC_SYNC_BYTES));
      return PRAC_EHIP;
    }
    return PRAC_ENUMERIC;
  }
  return PRAC_OK;
}

int prac_last_hip_error(const prac_ctx* ctx) { return ctx ? ctx->last_hip : 0; }

int prac_profile_select(prac_ctx* ctx, int kind) {
  if (kind < PRAC_KERNEL_NONE || kind > PRAC_KERNEL_SUM_P_T) return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  ctx->prof_kind = kind;
  ctx->prof_seen = 0;
  return PRAC_OK;
}

int prac_set_tuning(prac_ctx* ctx, int key, int value) {
  if (key == PRAC_TUNE_PROFILE_STRIDE) {
    if (value < 0 || value > 1024) return PRAC_EINVAL;
    if (!ctx) return PRAC_ENOCTX;
    ctx->prof_stride = value < 1 ? 1 : value;
    return PRAC_OK;
  }
  if (key == PRAC_TUNE_WGRAD_TAIL) {
    if (value < 0 || value > 2) return PRAC_EINVAL;
    if (!ctx) return PRAC_ENOCTX;
    ctx->tune_tail = value;
    return PRAC_OK;
  }
  if (key == PRAC_TUNE_WGRAD_ONE_LAUNCH) {
    if (value != 0 && value != 1) return PRAC_EINVAL;
    if (!ctx) return PRAC_ENOCTX;
    ctx->tune_one_launch = value;
    return PRAC_OK;
  }
  if (key != PRAC_TUNE_CTDY_SPLITS || value < 0 || value > 64) return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  ctx->tune_splits = value;
  return PRAC_OK;
}

int prac_profile_read_each(prac_ctx* ctx, float* each_ms, int64_t cap, int64_t* launches) {
  if (!launches || cap < 0 || (cap > 0 && !each_ms)) return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  PRAC_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  int64_t n = 0;
  for (auto& pr : ctx->prof_pairs) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, pr.first, pr.second) == hipSuccess) {
      if (n < cap) each_ms[n] = ms;
      ++n;
    } else {
      (void)hipGetLastError();  // a pair no launch took: its events were never recorded
    }
    ctx->prof_pool.push_back(pr.first);
    ctx->prof_pool.push_back(pr.second);
  }
  ctx->prof_pairs.clear();
  *launches = n;
  return PRAC_OK;
}

int prac_profile_read(prac_ctx* ctx, double* total_ms, int64_t* launches) {
  if (!total_ms || !launches) return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  std::vector<float> each(ctx->prof_pairs.size());
  int rc = prac_profile_read_each(ctx, each.data(), (int64_t)each.size(), launches);
  if (rc) return rc;
  double sum = 0.0;
  for (int64_t i = 0; i < *launches; ++i) sum += each[(size_t)i];
  *total_ms = sum;
  return PRAC_OK;
}

// ---------------------------------------------------------------- Gaussian draw
int prac_philox_words(prac_ctx* ctx, uint64_t seed, uint64_t draw, uint32_t stream, uint32_t* out, int64_t n) {
  if (n < 0 || (n > 0 && !out) || draw > 0xFFFFFFFFull) return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  return launch_philox(ctx, seed, (uint32_t)draw, stream, out, n, false);
}

int prac_philox_normal(prac_ctx* ctx, uint64_t seed, uint64_t draw, uint32_t stream, float* out, int64_t n) {
  if (n < 0 || (n > 0 && !out) || draw > 0xFFFFFFFFull) return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  return launch_philox(ctx, seed, (uint32_t)draw, stream, out, n, true);
}

// ------------------------------------------------------------------------- Gram
int prac_gram(prac_ctx* ctx, const void* X, prac_dtype xdt, int64_t N, int64_t d, int64_t ldx, int64_t row_stride,
              float* G, int64_t ldg) {
  if (!X || !G || !valid_dtype(xdt) || bad_tokens(N) || d < 1 || d > (1 << 20) || ldx < d || ldg < d || row_stride < 1)
    return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  const size_t need = gram_scratch_bytes(ctx->n_cu, X, xdt, N, d, ldx, row_stride, ldg);
  int rc = prac_ws_reserve(ctx, need);
  if (rc) return rc;
  return gram_device(ctx, X, xdt, N, d, ldx, row_stride, G, ldg, ctx->ws);
}

// ------------------------------------------------------------------------ basis
size_t prac_basis_lp_bytes(int64_t d, int c) {
  if (d < 1 || c < 1) return 0;
  return lp_layout(d, c).bytes;
}

int prac_pack_basis(prac_ctx* ctx, const float* P, int64_t d, int64_t ldp, int c, void* P_lp) {
  if (!P || !P_lp || d < 1 || c < 1 || c > d || ldp < c || !aligned16(P_lp)) return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  const LpLayout l = lp_layout(d, c);
  char* base = reinterpret_cast<char*>(P_lp);
  int rc = launch_pack_basis(ctx, P, d, ldp, c, reinterpret_cast<bf16_t*>(base), l.ldpt,
                             reinterpret_cast<bf16_t*>(base + l.off_pn), l.ldpn);
  if (rc) return rc;
  rc = launch_pack_pfrag(ctx, P, d, ldp, c, l.nkb, l.ncb, reinterpret_cast<bf16_t*>(base + l.off_pf));
  if (rc) return rc;
  return launch_pack_pafrag(ctx, P, d, ldp, c, l.nrb, l.nckb, reinterpret_cast<bf16_t*>(base + l.off_pa));
}

int prac_fit_basis(prac_ctx* ctx, const void* X, prac_dtype xdt, int64_t N, int64_t d, int64_t ldx, int k, int r,
                   uint64_t seed, uint64_t draw, int refresh, const prac_fit_opts* opts, float* P, int64_t ldp,
                   void* P_lp, float* scale) {
  if (!P || d < 1 || d > (1 << 20) || k < 0 || r < 0 || k + r < 1 || (int64_t)k + r > d || ldp < k + r ||
      draw > 0xFFFFFFFFull || (refresh & ~3) != 0)
    return PRAC_EINVAL;
  const bool need_x = (refresh & PRAC_REFRESH_PRINCIPAL) && k > 0;
  if (need_x && (!X || !valid_dtype(xdt) || bad_tokens(N) || ldx < d)) return PRAC_EINVAL;
  prac_fit_opts o{};
  if (opts) o = *opts;
  if (o.iters < 0 || o.row_stride < 0 || (o.warm_start != 0 && o.warm_start != 1)) return PRAC_EINVAL;
  if (o.iters == 0) o.iters = 8;
  if (o.row_stride == 0) o.row_stride = 1;
  if (P_lp && !aligned16(P_lp)) return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  if (scale) *scale = r > 0 ? (float)((double)(d - k) / (double)r) : 0.f;
  int rc = fit_basis_device(ctx, X, xdt, N, d, ldx, k, r, seed, (uint32_t)draw, refresh, o, P, ldp);
  if (rc) return rc;
  if (P_lp) return prac_pack_basis(ctx, P, d, ldp, k + r, P_lp);
  return PRAC_OK;
}

// --------------------------------------------------------------------- compress
size_t prac_compressed_bytes(int64_t N, int c, prac_dtype dt, int c_layout, int64_t ldc) {
  if (N < 1 || c < 1 || !valid_dtype(dt)) return 0;
  if (c_layout == PRAC_C_PACKED) return dt == PRAC_BF16 ? packed_c_bytes(N, c) : 0;
  if (c_layout != PRAC_C_ROWMAJOR || ldc < c) return 0;
  return (size_t)N * ldc * esize(dt);
}

int prac_unpack_compressed(prac_ctx* ctx, const void* Cpk, int64_t N, int c, void* C, int64_t ldc) {
  if (!Cpk || !C || bad_tokens(N) || c < 1 || ldc < c || !aligned16(Cpk)) return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  return launch_unpack_c(ctx, reinterpret_cast<const bf16_t*>(Cpk), (int)N, c, reinterpret_cast<bf16_t*>(C), ldc);
}

namespace {
// Scratch of one compress / fused-forward call.  fast: the bf16 kernels run (aligned bf16 X).
struct CompressPlan {
  size_t o_lp, o_w, o_tmp, o_c, bytes;
  int ncb_w;
};
CompressPlan plan_compress(bool fast, bool fused, bool packed, bool has_lp, prac_dtype xdt, int64_t N, int64_t d, int c,
                           int64_t m) {
  CompressPlan q{};
  WsPlan plan;
  if (fast) {
    const LpLayout l = lp_layout(d, c);
    q.o_lp = plan.take(has_lp ? 0 : l.bytes);
    q.ncb_w = fused ? (int)round_up64((m + 31) / 32, 8) : 0;  // whole 256-column groups
    q.o_w = plan.take(fused ? (size_t)l.nkb * q.ncb_w * 64 * 8 * sizeof(bf16_t) : 0);
  } else {
    const bool need_tmp = xdt == PRAC_BF16;
    q.o_tmp = plan.take(need_tmp ? (size_t)N * (c > m ? c : (size_t)m) * sizeof(float) : 0);
    q.o_c = plan.take(packed ? (size_t)N * round_up64(c, 8) * sizeof(bf16_t) : 0);
  }
  q.bytes = plan.off;
  return q;
}
}  // namespace

static int compress_impl(prac_ctx* ctx, const void* X, prac_dtype xdt, int64_t N, int64_t d, int64_t ldx,
                         const void* W, int64_t m, int64_t ldw, int w_layout, const float* P, const void* P_lp,
                         int64_t ldp, int c, void* Y, int64_t ldy, void* C, int64_t ldc, int c_layout) {
  const bool fused = W != nullptr;
  const bool packed = c_layout == PRAC_C_PACKED;
  const bool fast = xdt == PRAC_BF16 && aligned16(X) && ldx % 8 == 0 && ldx <= PRAC_MAX_STREAM_PITCH &&
                    N < ((int64_t)1 << 31);
  if (packed && (xdt != PRAC_BF16 || !aligned16(C))) return PRAC_EUNSUPPORTED;
  const CompressPlan q = plan_compress(fast, fused, packed, P_lp != nullptr, xdt, N, d, c, m);
  if (q.bytes) {
    int rc = prac_ws_reserve(ctx, q.bytes);
    if (rc) return rc;
  }
  if (fast) {
    const LpLayout l = lp_layout(d, c);
    const size_t o_lp = q.o_lp, o_w = q.o_w;
    const int ncb_w = q.ncb_w;
    int rc;
    const char* lp = reinterpret_cast<const char*>(P_lp);
    if (!lp) {
      rc = prac_pack_basis(ctx, P, d, ldp, c, ctx->ws + o_lp);
      if (rc) return rc;
      lp = ctx->ws + o_lp;
    }
    const bf16_t* Pf = reinterpret_cast<const bf16_t*>(lp + l.off_pf);
    if (!fused) {
      ProfScope ps(ctx, PRAC_KERNEL_COMPRESS);
      return launch_compress_ws(ctx, reinterpret_cast<const bf16_t*>(X), ldx, (int)N, (int)d, Pf, l.ncb, c,
                                reinterpret_cast<bf16_t*>(C), ldc, packed, nullptr, 0, 0, nullptr, 0);
    }
    // W changes every step, so it is put into fragment order on every call (a pure permutation
    // of its d x m elements), then one launch forms Y and C
    bf16_t* Wf = reinterpret_cast<bf16_t*>(ctx->ws + o_w);
    rc = launch_pack_wfrag(ctx, reinterpret_cast<const bf16_t*>(W), ldw, w_layout, d, (int)m, l.nkb, ncb_w, Wf);
    if (rc) return rc;
    ProfScope ps(ctx, PRAC_KERNEL_FUSED_FWD);
    return launch_compress_ws(ctx, reinterpret_cast<const bf16_t*>(X), ldx, (int)N, (int)d, Pf, l.ncb, c,
                              reinterpret_cast<bf16_t*>(C), ldc, packed, Wf, ncb_w, (int)m,
                              reinterpret_cast<bf16_t*>(Y), ldy);
  }
  // generic path: fp32 data (P used in fp32) or unaligned bf16
  const bool need_tmp = xdt == PRAC_BF16;
  const size_t o_tmp = q.o_tmp, o_c = q.o_c;
  float* tmp = need_tmp ? reinterpret_cast<float*>(ctx->ws + o_tmp) : nullptr;
  void* Crm = packed ? static_cast<void*>(ctx->ws + o_c) : C;
  const int64_t ldcrm = packed ? round_up64(c, 8) : ldc;
  GemmGenArgs g{};
  g.A = X; g.adt = xdt; g.a_rs = ldx; g.a_cs = 1;
  g.M = (int)N; g.K = d; g.k_stride = 1; g.alpha = 1.f; g.beta = 0.f; g.acc64 = false; g.out64 = nullptr;
  // C = X P
  g.B = P; g.bdt = PRAC_F32; g.b_rs = ldp; g.b_cs = 1; g.N = c;
  g.out = need_tmp ? tmp : reinterpret_cast<float*>(C);
  g.ldo = need_tmp ? c : ldc;
  int rc = launch_gemm_generic(ctx, g);
  if (rc) return rc;
  if (need_tmp) {
    rc = launch_cast_out(ctx, tmp, c, Crm, PRAC_BF16, ldcrm, (int)N, c, 0.f);
    if (rc) return rc;
    if (packed) {
      rc = launch_pack_c(ctx, reinterpret_cast<const bf16_t*>(Crm), ldcrm, (int)N, c, reinterpret_cast<bf16_t*>(C));
      if (rc) return rc;
    }
  }
  if (fused) {
    g.B = W; g.bdt = xdt; g.N = (int)m;
    if (w_layout == 1) { g.b_rs = 1; g.b_cs = ldw; } else { g.b_rs = ldw; g.b_cs = 1; }
    g.out = need_tmp ? tmp : reinterpret_cast<float*>(Y);
    g.ldo = need_tmp ? m : ldy;
    rc = launch_gemm_generic(ctx, g);
    if (rc) return rc;
    if (need_tmp) rc = launch_cast_out(ctx, tmp, m, Y, PRAC_BF16, ldy, (int)N, (int)m, 0.f);
  }
  return rc;
}

static bool bad_c_layout(int c_layout, int64_t ldc, int c) {
  if (c_layout == PRAC_C_PACKED) return false;
  return c_layout != PRAC_C_ROWMAJOR || ldc < c;
}

int prac_compress(prac_ctx* ctx, const void* X, prac_dtype xdt, int64_t N, int64_t d, int64_t ldx, const float* P,
                  const void* P_lp, int64_t ldp, int c, void* C, int64_t ldc, int c_layout) {
  if (!X || !P || !C || !valid_dtype(xdt) || bad_tokens(N) || d < 1 || d > (1 << 20) || c < 1 || c > d || ldx < d ||
      ldp < c || bad_c_layout(c_layout, ldc, c) || (P_lp && !aligned16(P_lp)))
    return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  return compress_impl(ctx, X, xdt, N, d, ldx, nullptr, 0, 0, 0, P, P_lp, ldp, c, nullptr, 0, C, ldc, c_layout);
}

int prac_compress_fused_fwd(prac_ctx* ctx, const void* X, prac_dtype xdt, int64_t N, int64_t d, int64_t ldx,
                            const void* W, int64_t m, int64_t ldw, int w_layout, const float* P, const void* P_lp,
                            int64_t ldp, int c, void* Y, int64_t ldy, void* C, int64_t ldc, int c_layout) {
  if (!X || !P || !C || !W || !Y || !valid_dtype(xdt) || bad_tokens(N) || d < 1 || d > (1 << 20) || c < 1 || c > d ||
      m < 1 || m > (1 << 20) || ldx < d || ldp < c || bad_c_layout(c_layout, ldc, c) || ldy < m ||
      (w_layout != 0 && w_layout != 1) || ldw < (w_layout == 1 ? d : m) || (P_lp && !aligned16(P_lp)))
    return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  return compress_impl(ctx, X, xdt, N, d, ldx, W, m, ldw, w_layout, P, P_lp, ldp, c, Y, ldy, C, ldc, c_layout);
}

}  // extern "C"

// ------------------------------------------------------------------ weight grad
namespace {

// One gradient through the strided kernels (fp32 data, unaligned bf16): T = C^T dY (fp32), scale
// the random rows, dW = P T.
struct WgradGenPlan {
  size_t o_t, o_dw, o_crm, bytes;
};
WgradGenPlan plan_wgrad_generic(int64_t N, int64_t d, int64_t m, int c, bool packed, prac_dtype odt) {
  WgradGenPlan q{};
  WsPlan plan;
  q.o_t = plan.take((size_t)c * m * sizeof(float));
  q.o_dw = plan.take(odt == PRAC_BF16 ? (size_t)d * m * sizeof(float) : 0);
  q.o_crm = plan.take(packed ? (size_t)N * c * sizeof(bf16_t) : 0);
  q.bytes = plan.off;
  return q;
}

int weight_grad_generic(prac_ctx* ctx, char* ws, const void* C, const void* dY, prac_dtype dt, int64_t N, int64_t m,
                        int64_t ldc, bool packed, int64_t lddy, const float* P, int64_t d, int64_t ldp, int k, int r,
                        float scale, void* dW, prac_dtype odt, int64_t lddw, float beta) {
  const int c = k + r;
  const WgradGenPlan q = plan_wgrad_generic(N, d, m, c, packed, odt);
  const size_t o_t = q.o_t, o_dw = q.o_dw, o_crm = q.o_crm;
  int rc;
  const void* Crm = C;
  int64_t ldcrm = ldc;
  if (packed) {
    rc = launch_unpack_c(ctx, reinterpret_cast<const bf16_t*>(C), (int)N, c, reinterpret_cast<bf16_t*>(ws + o_crm), c);
    if (rc) return rc;
    Crm = ws + o_crm;
    ldcrm = c;
  }
  float* T = reinterpret_cast<float*>(ws + o_t);
  GemmGenArgs g{};
  g.A = Crm; g.adt = dt; g.a_rs = 1; g.a_cs = ldcrm;
  g.B = dY; g.bdt = dt; g.b_rs = lddy; g.b_cs = 1;
  g.M = c; g.N = (int)m; g.K = N; g.k_stride = 1;
  g.out = T; g.ldo = m; g.alpha = 1.f; g.beta = 0.f; g.acc64 = false; g.out64 = nullptr;
  rc = launch_gemm_generic(ctx, g);
  if (rc) return rc;
  rc = launch_scale_rows(ctx, T, c, (int)m, m, k, scale);
  if (rc) return rc;
  GemmGenArgs h{};
  h.A = P; h.adt = PRAC_F32; h.a_rs = ldp; h.a_cs = 1;
  h.B = T; h.bdt = PRAC_F32; h.b_rs = m; h.b_cs = 1;
  h.M = (int)d; h.N = (int)m; h.K = c; h.k_stride = 1;
  h.alpha = 1.f; h.acc64 = false; h.out64 = nullptr;
  if (odt == PRAC_F32) {
    h.out = reinterpret_cast<float*>(dW); h.ldo = lddw; h.beta = beta;
    return launch_gemm_generic(ctx, h);
  }
  float* tmp = reinterpret_cast<float*>(ws + o_dw);
  h.out = tmp; h.ldo = m; h.beta = 0.f;
  rc = launch_gemm_generic(ctx, h);
  if (rc) return rc;
  return launch_cast_out(ctx, tmp, m, dW, PRAC_BF16, lddw, (int)d, (int)m, beta);
}

// n_out gradients from one C on the bf16 kernels: one launch forms the token-split slabs of every
// C^T dY_h, then each output gets its slab reduction and its dW_h = P T_h.
struct WgradPlan {
  int splits;
  bool fused;  // one launch (see launch_wgrad_fused) instead of three
  int nmb[PRAC_CTDY_MAX_OUT];
  size_t o_part[PRAC_CTDY_MAX_OUT], o_t[PRAC_CTDY_MAX_OUT], o_lp, o_cpk, bytes;
};
WgradPlan plan_wgrad_fast(int n_cu, int tune_splits, bool unfused, int64_t N, int64_t d, int c, int n_out,
                          const int64_t* m, bool packed, bool has_lp) {
  WgradPlan q{};
  const LpLayout l = lp_layout(d, c);
  int splits = unfused ? 0 : wgrad_fused_splits(n_cu, c, n_out, m, N, tune_splits);
  q.fused = splits > 0;
  if (!q.fused) {
    int tiles = 0;
    for (int h = 0; h < n_out; ++h) tiles += ((c + 255) / 256) * (int)((m[h] + 127) / 128);
    // one workgroup per CU at most: a second, partly filled round would cost a whole workgroup time
    splits = n_cu / tiles;
    if (splits > N / 256) splits = (int)(N / 256);
    if (splits < 1) splits = 1;
    if (splits > 64) splits = 64;
    if (tune_splits > 0) splits = tune_splits;
  }
  q.splits = splits;
  WsPlan plan;
  for (int h = 0; h < n_out; ++h) {
    q.nmb[h] = (int)round_up64((m[h] + 31) / 32, 4);  // 32-column blocks of T, whole 128-column tiles
    q.o_part[h] = plan.take((size_t)splits * c * m[h] * sizeof(float));
    q.o_t[h] = plan.take((size_t)l.nckb * q.nmb[h] * 64 * 8 * sizeof(bf16_t));
  }
  q.o_lp = plan.take(has_lp ? 0 : l.bytes);
  q.o_cpk = plan.take(packed ? 0 : packed_c_bytes(N, c));
  q.bytes = plan.off;
  return q;
}

int weight_grad_fast(prac_ctx* ctx, char* ws, int* cnt, const WgradPlan& q, const void* C, int64_t N, int64_t ldc, bool packed,
                     int n_out, const void* const* dY, const int64_t* m, const int64_t* lddy, const float* P,
                     const void* P_lp, int64_t d, int64_t ldp, int k, int r, float scale, void* const* dW,
                     prac_dtype odt, const int64_t* lddw, float beta) {
  const int c = k + r;
  const LpLayout l = lp_layout(d, c);
  const int splits = q.splits;
  int rc;
  const char* lp = reinterpret_cast<const char*>(P_lp);
  if (!lp) {
    rc = prac_pack_basis(ctx, P, d, ldp, c, ws + q.o_lp);
    if (rc) return rc;
    lp = ws + q.o_lp;
  }
  const bf16_t* Cpk = reinterpret_cast<const bf16_t*>(C);
  if (!packed) {
    rc = launch_pack_c(ctx, reinterpret_cast<const bf16_t*>(C), ldc, (int)N, c, reinterpret_cast<bf16_t*>(ws + q.o_cpk));
    if (rc) return rc;
    Cpk = reinterpret_cast<const bf16_t*>(ws + q.o_cpk);
  }
  const bf16_t* dYp[PRAC_CTDY_MAX_OUT];
  float* part[PRAC_CTDY_MAX_OUT];
  int mi[PRAC_CTDY_MAX_OUT];
  for (int h = 0; h < n_out; ++h) {
    dYp[h] = reinterpret_cast<const bf16_t*>(dY[h]);
    part[h] = reinterpret_cast<float*>(ws + q.o_part[h]);
    mi[h] = (int)m[h];
  }
  bf16_t* Tf[PRAC_CTDY_MAX_OUT];
  for (int h = 0; h < n_out; ++h) Tf[h] = reinterpret_cast<bf16_t*>(ws + q.o_t[h]);
  if (q.fused) {
    // one launch: slabs, their sum T (bf16, fragment order, random rows scaled) and dW_h = P T_h
    ProfScope ps(ctx, PRAC_KERNEL_WEIGHT_GRAD);
    return launch_wgrad_fused(ctx, Cpk, c, (int)N, n_out, dYp, lddy, mi, part, splits, k, scale, l.nckb, q.nmb, Tf,
                              reinterpret_cast<const bf16_t*>(lp + l.off_pa), (int)d, dW, lddw, odt == PRAC_BF16, beta,
                              cnt);
  }
  {  // T_h = C^T dY_h as `splits` partial slabs over the token range
    ProfScope ps(ctx, PRAC_KERNEL_CT_DY);
    rc = launch_ctdy_ws(ctx, Cpk, c, (int)N, n_out, dYp, lddy, mi, part, splits);
  }
  if (rc) return rc;
  // Slab sum, scaling factor and dW_h = P T_h in one launch where that is the faster form: measured on an
  // MI355X it is for c > 256 (rank 512 + 512 at d = m = 2048: 159 against 179 us per weight gradient), where
  // the two launches move a large T through memory and run the LDS-staged product; at c <= 256 the two
  // small launches overlap each other's start and end and win (61.6 against 66.8 us at the same d, m).
  // (every 512 rows of dW are one more workgroup per column block that repeats the slab sum: at d = 11008,
  // 22 of them, the one launch takes 180 us against 98 us for the two, so it is limited to d <= 2048)
  const bool tail_one = ctx->tune_tail == 2 || (ctx->tune_tail == 0 && l.nckb > 16 && d <= 2048);
  if (tail_one && sum_pt_eligible(n_out, mi, splits)) {
    ProfScope ps(ctx, PRAC_KERNEL_SUM_P_T);
    return launch_sum_pt(ctx, reinterpret_cast<const bf16_t*>(lp + l.off_pa), n_out, part, splits, c, k, scale, l.nckb,
                         (int)d, mi, dW, lddw, odt == PRAC_BF16, beta);
  }
  {  // T_h in fragment order (bf16): slabs summed, random rows weighted by the scaling factor
    ProfScope ps(ctx, PRAC_KERNEL_T_REDUCE);
    rc = launch_reduce_to_tfrag(ctx, n_out, part, splits, c, mi, k, scale, l.nckb, q.nmb, Tf);
  }
  if (rc) return rc;
  {
    ProfScope ps(ctx, PRAC_KERNEL_P_T);  // dW_h = P T_h, all outputs in one launch
    rc = launch_pt(ctx, reinterpret_cast<const bf16_t*>(lp + l.off_pa), n_out, Tf, (int)d, mi, l.nckb, q.nmb, dW, lddw,
                   odt == PRAC_BF16, beta);
  }
  if (rc) return rc;
  return PRAC_OK;
}

// Argument checks of the weight-gradient entry points (no ctx needed).
int wgrad_check(const void* C, prac_dtype dt, int64_t N, int64_t ldc, int c_layout, int n_out, const void* const* dY,
                const int64_t* m, const int64_t* lddy, const float* P, const void* P_lp, int64_t d, int64_t ldp, int k,
                int r, void* const* dW, prac_dtype odt, const int64_t* lddw) {
  if (!C || !dY || !m || !lddy || !dW || !lddw || !P || n_out < 1 || n_out > PRAC_MAX_SHARED || !valid_dtype(dt) ||
      !valid_dtype(odt) || bad_tokens(N) || d < 1 || d > (1 << 20) || k < 0 || r < 0 || k + r < 1 || (int64_t)k + r > d ||
      (c_layout != PRAC_C_PACKED && (c_layout != PRAC_C_ROWMAJOR || ldc < k + r)) || ldp < k + r ||
      (P_lp && !aligned16(P_lp)))
    return PRAC_EINVAL;
  for (int h = 0; h < n_out; ++h)
    if (!dY[h] || !dW[h] || m[h] < 1 || m[h] > (1 << 20) || lddy[h] < m[h] || lddw[h] < m[h]) return PRAC_EINVAL;
  return PRAC_OK;
}
bool wgrad_is_fast(prac_dtype dt, int64_t N, int n_out, const void* const* dY, const int64_t* lddy) {
  bool fast = dt == PRAC_BF16 && N < ((int64_t)1 << 31);
  for (int h = 0; h < n_out; ++h)
    fast = fast && aligned16(dY[h]) && lddy[h] % 8 == 0 && lddy[h] <= PRAC_MAX_STREAM_PITCH;
  return fast;
}

}  // namespace

extern "C" {

int prac_weight_grad(prac_ctx* ctx, const void* C, const void* dY, prac_dtype dt, int64_t N, int64_t m, int64_t ldc,
                     int c_layout, int64_t lddy, const float* P, const void* P_lp, int64_t d, int64_t ldp, int k,
                     int r, float scale, void* dW, prac_dtype odt, int64_t lddw, float beta) {
  return prac_weight_grad_shared(ctx, C, dt, N, ldc, c_layout, 1, &dY, &m, &lddy, P, P_lp, d, ldp, k, r, scale, &dW, odt,
                                 &lddw, beta);
}

int prac_weight_grad_static(prac_ctx* ctx, const void* C, const void* dY, prac_dtype dt, int64_t N, int64_t m,
                            int64_t ldc, int c_layout, int64_t lddy, const float* P, const void* P_lp, int64_t d,
                            int64_t ldp, int k, int r, float scale, void* dW, prac_dtype odt, int64_t lddw, float beta) {
  int rc = wgrad_check(C, dt, N, ldc, c_layout, 1, &dY, &m, &lddy, P, P_lp, d, ldp, k, r, &dW, odt, &lddw);
  if (rc) return rc;
  if (!ctx) return PRAC_ENOCTX;
  const bool packed = c_layout == PRAC_C_PACKED;
  if (packed && (dt != PRAC_BF16 || !aligned16(C))) return PRAC_EUNSUPPORTED;
  const bool fast = wgrad_is_fast(dt, N, 1, &dY, &lddy);
  WgradPlan q{};
  size_t need;
  if (fast) {
    q = plan_wgrad_fast(ctx->n_cu, ctx->tune_splits, ctx->tune_one_launch == 0, N, d, k + r, 1, &m, packed, P_lp != nullptr);
    need = q.bytes;
  } else {
    need = plan_wgrad_generic(N, d, m, k + r, packed, odt).bytes;
  }
  // the first 128 KB of the block are the counters of the one-launch weight gradient (zero when the code
  // object is loaded, and every launch leaves them zero)
  constexpr size_t kSync = PRAC_SYNC_BYTES;
  if (need > PRAC_STATIC_SCRATCH_BYTES - kSync) return PRAC_ETOOBIG;
  // no event pairs here (creating one allocates): this call is not profiled
  const int prof = ctx->prof_kind;
  ctx->prof_kind = PRAC_KERNEL_NONE;
  char* ws = ctx->static_scratch + kSync;
  if (fast)
    rc = weight_grad_fast(ctx, ws, reinterpret_cast<int*>(ctx->static_scratch), q, C, N, ldc, packed, 1, &dY, &m, &lddy, P, P_lp, d, ldp, k, r, scale, &dW, odt, &lddw,
                          beta);
  else
    rc = weight_grad_generic(ctx, ws, C, dY, dt, N, m, ldc, packed, lddy, P, d, ldp, k, r, scale, dW, odt, lddw, beta);
  ctx->prof_kind = prof;
  return rc;
}

int prac_weight_grad_shared(prac_ctx* ctx, const void* C, prac_dtype dt, int64_t N, int64_t ldc, int c_layout, int n_out,
                            const void* const* dY, const int64_t* m, const int64_t* lddy, const float* P,
                            const void* P_lp, int64_t d, int64_t ldp, int k, int r, float scale, void* const* dW,
                            prac_dtype odt, const int64_t* lddw, float beta) {
  int rc = wgrad_check(C, dt, N, ldc, c_layout, n_out, dY, m, lddy, P, P_lp, d, ldp, k, r, dW, odt, lddw);
  if (rc) return rc;
  if (!ctx) return PRAC_ENOCTX;
  const bool packed = c_layout == PRAC_C_PACKED;
  if (packed && (dt != PRAC_BF16 || !aligned16(C))) return PRAC_EUNSUPPORTED;
  if (wgrad_is_fast(dt, N, n_out, dY, lddy)) {
    const WgradPlan q = plan_wgrad_fast(ctx->n_cu, ctx->tune_splits, ctx->tune_one_launch == 0, N, d, k + r, n_out, m, packed,
                                        P_lp != nullptr);
    rc = prac_ws_reserve(ctx, q.bytes);
    if (rc) return rc;
    return weight_grad_fast(ctx, ctx->ws, ctx->d_sync, q, C, N, ldc, packed, n_out, dY, m, lddy, P, P_lp, d, ldp, k, r, scale, dW, odt,
                            lddw, beta);
  }
  size_t need = 0;
  for (int h = 0; h < n_out; ++h) need = std::max(need, plan_wgrad_generic(N, d, m[h], k + r, packed, odt).bytes);
  rc = prac_ws_reserve(ctx, need);
  if (rc) return rc;
  for (int h = 0; h < n_out; ++h) {
    rc = weight_grad_generic(ctx, ctx->ws, C, dY[h], dt, N, m[h], ldc, packed, lddy[h], P, d, ldp, k, r, scale, dW[h], odt,
                             lddw[h], beta);
    if (rc) return rc;
  }
  return PRAC_OK;
}

}  // extern "C"

// ------------------------------------------------------------------ reconstruction
namespace {
struct ReconPlan {
  bool fast, direct;
  int nkb, ncb;
  int64_t ldcrm;
  size_t o_pt, o_c, o_tmp, o_crm, bytes;
};
ReconPlan plan_reconstruct(bool fast, prac_dtype dt, int64_t N, int64_t d, int c, bool packed, int64_t ldc) {
  ReconPlan q{};
  q.fast = fast;
  WsPlan plan;
  if (fast) {
    q.nkb = (int)(round_up64(c, 256) / 16);
    q.ncb = (int)round_up64((d + 31) / 32, 8);
    q.direct = c <= 256;  // the dedicated kernel reads packed C itself
    q.ldcrm = packed ? round_up64(c, 8) : ldc;
    q.o_pt = plan.take((size_t)q.nkb * q.ncb * 64 * 8 * sizeof(bf16_t));
    q.o_c = plan.take(packed && !q.direct ? (size_t)N * q.ldcrm * sizeof(bf16_t) : 0);
  } else {
    q.o_tmp = plan.take(dt == PRAC_BF16 ? (size_t)N * d * sizeof(float) : 0);
    q.o_crm = plan.take(packed ? (size_t)N * c * sizeof(bf16_t) : 0);
  }
  q.bytes = plan.off;
  return q;
}
}  // namespace

int prac_reconstruct(prac_ctx* ctx, const void* C, prac_dtype dt, int64_t N, int64_t ldc, int c_layout, const float* P,
                     int64_t d, int64_t ldp, int k, int r, float scale, void* Xh, int64_t ldxh) {
  if (!C || !P || !Xh || !valid_dtype(dt) || bad_tokens(N) || d < 1 || d > (1 << 20) || k < 0 || r < 0 || k + r < 1 ||
      (int64_t)k + r > d || bad_c_layout(c_layout, ldc, k + r) || ldp < k + r || ldxh < d)
    return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  const int c = k + r;
  const bool packed = c_layout == PRAC_C_PACKED;
  if (packed && (dt != PRAC_BF16 || !aligned16(C))) return PRAC_EUNSUPPORTED;
  const bool rm_ok = !packed && aligned16(C) && ldc % 8 == 0 && ldc <= PRAC_MAX_STREAM_PITCH;
  const bool fast = dt == PRAC_BF16 && (packed || rm_ok) && N < ((int64_t)1 << 31);
  const ReconPlan q = plan_reconstruct(fast, dt, N, d, c, packed, ldc);
  if (q.bytes) {
    int rc = prac_ws_reserve(ctx, q.bytes);
    if (rc) return rc;
  }
  if (fast) {
    // Xh = C Ps^T is the forward-output launch of the compress kernel with C in the role of X
    // (its "feature" dimension is c) and Ps^T in the role of W.
    const int nkb = q.nkb, ncb = q.ncb;
    const int64_t ldcrm = q.ldcrm;
    bf16_t* Pt = reinterpret_cast<bf16_t*>(ctx->ws + q.o_pt);
    int rc = launch_pack_ptfrag(ctx, P, d, ldp, c, k, scale, nkb, ncb, Pt);
    if (rc) return rc;
    if (q.direct) {
      ProfScope ps(ctx, PRAC_KERNEL_RECONSTRUCT);
      return launch_reconstruct_ws(ctx, reinterpret_cast<const bf16_t*>(C), ldc, packed, (int)N, c, (int)d, Pt, ncb,
                                   reinterpret_cast<bf16_t*>(Xh), ldxh);
    }
    const bf16_t* Crm = reinterpret_cast<const bf16_t*>(C);
    if (packed) {
      rc = launch_unpack_c(ctx, reinterpret_cast<const bf16_t*>(C), (int)N, c, reinterpret_cast<bf16_t*>(ctx->ws + q.o_c),
                           ldcrm);
      if (rc) return rc;
      Crm = reinterpret_cast<const bf16_t*>(ctx->ws + q.o_c);
    }
    ProfScope ps(ctx, PRAC_KERNEL_RECONSTRUCT);
    return launch_compress_ws(ctx, Crm, ldcrm, (int)N, c, nullptr, 0, 0, nullptr, 0, false, Pt, ncb, (int)d,
                              reinterpret_cast<bf16_t*>(Xh), ldxh);
  }
  // generic path: Xh = C1 Q1^T, then Xh += scale * C2 Q2^T (fp32 sums)
  const bool need_tmp = dt == PRAC_BF16;
  const void* Crm = C;
  int64_t ldcrm = ldc;
  if (packed) {
    int rc = launch_unpack_c(ctx, reinterpret_cast<const bf16_t*>(C), (int)N, c,
                             reinterpret_cast<bf16_t*>(ctx->ws + q.o_crm), c);
    if (rc) return rc;
    Crm = ctx->ws + q.o_crm;
    ldcrm = c;
  }
  float* out = need_tmp ? reinterpret_cast<float*>(ctx->ws + q.o_tmp) : reinterpret_cast<float*>(Xh);
  const int64_t ldo = need_tmp ? d : ldxh;
  const size_t es = esize(dt);
  bool first = true;
  for (int part = 0; part < 2; ++part) {
    const int k0 = part == 0 ? 0 : k, kn = part == 0 ? k : r;
    if (kn == 0) continue;
    GemmGenArgs g{};
    g.A = reinterpret_cast<const char*>(Crm) + (size_t)k0 * es; g.adt = dt; g.a_rs = ldcrm; g.a_cs = 1;
    g.B = P + k0; g.bdt = PRAC_F32; g.b_rs = 1; g.b_cs = ldp;  // B(kk, n) = P[n][k0 + kk]
    g.M = (int)N; g.N = (int)d; g.K = kn; g.k_stride = 1;
    g.out = out; g.ldo = ldo; g.acc64 = false; g.out64 = nullptr;
    g.alpha = part == 0 ? 1.f : scale;
    g.beta = first ? 0.f : 1.f;
    first = false;
    int rc = launch_gemm_generic(ctx, g);
    if (rc) return rc;
  }
  if (need_tmp) return launch_cast_out(ctx, out, d, Xh, PRAC_BF16, ldxh, (int)N, (int)d, 0.f);
  return PRAC_OK;
}

// ------------------------------------------------------------------ scratch sizing
extern "C" {

size_t prac_workspace_bytes(const prac_ctx* ctx, const prac_call_shape* sh) {
  const size_t bad = ~(size_t)0;
  if (!sh || !valid_dtype(sh->dt) || sh->N < 1 || sh->N >= ((int64_t)1 << 31) || sh->d < 1 || sh->d > (1 << 20) ||
      sh->k < 0 || sh->r < 0 || (int64_t)sh->k + sh->r > sh->d)
    return bad;
  const int n_cu = ctx ? ctx->n_cu : 256;
  const int tune = ctx ? ctx->tune_splits : 0;
  const prac_dtype dt = (prac_dtype)sh->dt;
  const int c = sh->k + sh->r;
  const bool fast = dt == PRAC_BF16 && !sh->generic;
  const bool packed = sh->c_layout == PRAC_C_PACKED;
  // an unaligned pointer stands for "the strided kernels will run" where a plan looks at alignment
  const void* xptr = sh->generic ? reinterpret_cast<const void*>(uintptr_t(2)) : nullptr;
  const int64_t ldq = sh->generic ? sh->d : round_up64(sh->d, 8);  // row pitch the plan assumes for X
  switch (sh->op) {
    case PRAC_OP_GRAM:
      return gram_scratch_bytes(n_cu, xptr, dt, sh->N, sh->d, ldq, sh->fit.row_stride > 0 ? sh->fit.row_stride : 1, sh->d);
    case PRAC_OP_FIT_BASIS: {
      if (c < 1) return bad;
      prac_fit_opts o = sh->fit;
      if (o.iters == 0) o.iters = 8;
      if (o.row_stride == 0) o.row_stride = 1;
      size_t b = fit_scratch_bytes(n_cu, xptr, dt, sh->N, sh->d, ldq, sh->k, sh->r, sh->refresh, o);
      return b;  // the packed copy goes to the caller's P_lp, not to scratch
    }
    case PRAC_OP_COMPRESS:
    case PRAC_OP_FUSED_FWD: {
      if (c < 1) return bad;
      const bool fused = sh->op == PRAC_OP_FUSED_FWD;
      if (fused && (sh->n_out != 1 || sh->m[0] < 1)) return bad;
      return plan_compress(fast, fused, packed, sh->have_p_lp != 0, dt, sh->N, sh->d, c, fused ? sh->m[0] : 0).bytes;
    }
    case PRAC_OP_WEIGHT_GRAD: {
      if (c < 1 || sh->n_out < 1 || sh->n_out > PRAC_MAX_SHARED) return bad;
      for (int h = 0; h < sh->n_out; ++h)
        if (sh->m[h] < 1 || sh->m[h] > (1 << 20)) return bad;
      if (fast)
        return plan_wgrad_fast(n_cu, tune, !(ctx && ctx->tune_one_launch), sh->N, sh->d, c, sh->n_out, sh->m, packed,
                               sh->have_p_lp != 0).bytes;
      size_t need = 0;
      for (int h = 0; h < sh->n_out; ++h)
        need = std::max(need, plan_wgrad_generic(sh->N, sh->d, sh->m[h], c, packed,
                                                 sh->odt == PRAC_BF16 ? PRAC_BF16 : PRAC_F32).bytes);
      return need;
    }
    case PRAC_OP_RECONSTRUCT:
      if (c < 1) return bad;
      return plan_reconstruct(fast, dt, sh->N, sh->d, c, packed, c).bytes;
    default:
      return bad;
  }
}

int prac_reserve_workspace(prac_ctx* ctx, size_t bytes) {
  if (bytes == ~(size_t)0) return PRAC_EINVAL;
  if (!ctx) return PRAC_ENOCTX;
  return prac_ws_reserve(ctx, bytes);
}

int64_t prac_debug_fit_slab_margin(const prac_call_shape* sh) {
  if (!sh) return -1;
  prac_fit_opts o = sh->fit;
  if (o.iters == 0) o.iters = 8;
  if (o.row_stride == 0) o.row_stride = 1;
  return fit_slab_margin(256, (prac_dtype)sh->dt, sh->N, sh->d, sh->k, sh->r, sh->refresh, o);
}

}  // extern "C"
