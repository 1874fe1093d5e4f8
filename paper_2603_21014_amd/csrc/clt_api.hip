// C ABI of libclt (include/clt.h): argument validation, workspace planning and
// the order in which the kernels of a CLT train step are enqueued.  No
// arithmetic of the method lives here.
#include "../../include/clt.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <vector>

#include "common.h"

#include <algorithm>

using namespace clt;

namespace {

constexpr size_t ALIGN = 256;
inline size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

struct Plan {
  size_t norms, G, d_yhat, dpre, part_cols, part_cols2, part_cols3, part_rec, part_sp, part_dead, l0, flags, xcd_sync, n2_part, pre32, g_idx, g_val, g_counts, g_counts_w, dz_part,
         fl_off, fl_cnt, fl_tok, fl_val, fl_seg, total;
  int kcap;
  int ecap;
};

thread_local char g_err[256] = "";

void set_err(char* dst, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(dst, 256, fmt, ap);
  va_end(ap);
}

}  // namespace

enum KernelId {
  K_NORMS, K_ENC, K_DEC, K_LOSS_SP, K_LOSS_REC, K_LOSS_FINAL, K_COLRED, K_DZ, K_STE, K_DWENC, K_DWDEC,
  K_ADAM_WDEC, K_ADAM_WENC, K_ADAM_VEC, K_ZERO, K_DECIDE, K_COMPACT, K_GATHER, K_SP_FILL, K_GATHER_DZ, K_FLISTS,
  K_SP_DWDEC, K_TOPK, K_NORM_SUM, K_NORMALISE, K_NORMS_REUSE, K_COUNT
};
static const char* const kKernelNames[K_COUNT] = {
  "decoder_norms", "encoder_jumprelu_gemm", "decode_gemm", "loss_sparsity", "loss_reconstruction", "loss_final",
  "column_reduce", "dz_gemm", "ste_reduce", "dW_enc_gemm", "dW_dec_gemm", "adam_W_dec", "adam_W_enc",
  "adam_vectors", "zero_counters", "decode_decide", "compact_active", "gather_decode", "sparse_dpre_fill",
  "gather_dz", "feature_lists", "sparse_dW_dec", "topk_select", "activation_norm_sum", "normalise_activations",
  "decoder_norms_from_update"};

struct ProfSpan { int kernel; hipEvent_t a, b; };

struct clt_handle {
  bool prof_on = false;
  std::vector<ProfSpan> spans;          // recorded, not yet harvested
  std::vector<hipEvent_t> free_events;  // recycled events
  double prof_ms[K_COUNT] = {};
  int64_t prof_n[K_COUNT] = {};
  clt_config cfg;
  Dims D;
  bool bf16, int8;
  size_t esz;             // bytes per element of T
  char* ws;
  Plan plan;
  int stage;              // 0 = fresh, 1 = forward done, 2 = loss done
  bool n2_eligible;       // the configuration can hand decoder norms from the update to the next forward
  const void* n2_for;     // W_dec pointer whose updated row sums of squares sit in the workspace, or NULL
  float lambda0, lambda1;
  char err[256];
};

namespace {

int check_config(const clt_config* c, char* err) {
  if (!c) { set_err(err, "config is NULL"); return CLT_ERR_INVALID_ARG; }
  if (c->size != sizeof(clt_config)) {
    set_err(err, "config.size is %u, this library expects %zu", c->size, sizeof(clt_config));
    return CLT_ERR_INVALID_ARG;
  }
  if (c->L < 1 || c->L > 128 || c->B < 1 || c->d < 8 || c->F < 8 || (c->d % 8) || (c->F % 8)) {
    set_err(err, "unsupported shape L=%d d=%d F=%d B=%d (need 1<=L<=128, B>=1, d and F positive multiples of 8)",
            c->L, c->d, c->F, c->B);
    return CLT_ERR_SHAPE;
  }
  if ((double)c->L * c->B * (double)c->F >= 9.0e18 || (size_t)c->L * c->B > (size_t)1 << 31 ||
      (size_t)c->L * c->F >= (size_t)1 << 31) {
    set_err(err, "shape too large");
    return CLT_ERR_SHAPE;
  }
  if (c->dtype != CLT_DTYPE_F32 && c->dtype != CLT_DTYPE_BF16) { set_err(err, "bad dtype %d", c->dtype); return CLT_ERR_INVALID_ARG; }
  if (c->input_format != CLT_INPUT_NATIVE && c->input_format != CLT_INPUT_INT8_ROWSCALE) {
    set_err(err, "bad input_format %d", c->input_format);
    return CLT_ERR_INVALID_ARG;
  }
  if (c->input_format == CLT_INPUT_INT8_ROWSCALE && c->dtype != CLT_DTYPE_BF16) {
    set_err(err, "int8 inputs need dtype bf16");
    return CLT_ERR_INVALID_ARG;
  }
  if (c->master_weights != 0 && c->master_weights != 1) { set_err(err, "bad master_weights"); return CLT_ERR_INVALID_ARG; }
  if (c->decode_mode != CLT_DECODE_DENSE && c->decode_mode != CLT_DECODE_GATHER && c->decode_mode != CLT_DECODE_AUTO) {
    set_err(err, "bad decode_mode %d", c->decode_mode);
    return CLT_ERR_INVALID_ARG;
  }
  if (c->log_threshold != 0 && c->log_threshold != 1) { set_err(err, "bad log_threshold"); return CLT_ERR_INVALID_ARG; }
  if (c->reuse_decoder_norms != 0 && c->reuse_decoder_norms != 1) { set_err(err, "bad reuse_decoder_norms"); return CLT_ERR_INVALID_ARG; }
  if (c->activation != CLT_ACT_JUMPRELU && c->activation != CLT_ACT_TOPK) { set_err(err, "bad activation %d", c->activation); return CLT_ERR_INVALID_ARG; }
  if (c->activation == CLT_ACT_TOPK && (c->topk_k < 0 || c->topk_k > c->F)) {
    set_err(err, "topk_k must be in [0, F]");
    return CLT_ERR_INVALID_ARG;
  }
  if (c->activation == CLT_ACT_TOPK && c->log_threshold) { set_err(err, "log_threshold has no meaning with TopK"); return CLT_ERR_INVALID_ARG; }
  if (c->decode_mode == CLT_DECODE_AUTO && !(c->gather_density_threshold >= 0.f && c->gather_density_threshold <= 1.f)) {
    set_err(err, "gather_density_threshold must be in [0, 1]");
    return CLT_ERR_INVALID_ARG;
  }
  if (c->decode_mode == CLT_DECODE_AUTO &&
      !(c->list_backward_density_threshold >= 0.f && c->list_backward_density_threshold <= 1.f)) {
    set_err(err, "list_backward_density_threshold must be in [0, 1]");
    return CLT_ERR_INVALID_ARG;
  }
  if (!(c->C > 0.f) || !(c->ste_bandwidth > 0.f) || !(c->beta1 >= 0.f && c->beta1 < 1.f) ||
      !(c->beta2 >= 0.f && c->beta2 < 1.f) || !(c->adam_eps > 0.f)) {
    set_err(err, "bad scalar: need C>0, ste_bandwidth>0, 0<=beta<1, adam_eps>0");
    return CLT_ERR_INVALID_ARG;
  }
  return CLT_OK;
}

// AUTO: the density up to which the backward through the decoder takes the lists (0 = as the forward decode)
float backward_threshold(const clt_config* c) {
  return c->list_backward_density_threshold > 0.f ? c->list_backward_density_threshold : c->gather_density_threshold;
}

Plan make_plan(const clt_config* c) {
  const size_t L = c->L, d = c->d, F = c->F, B = c->B;
  const size_t esz = c->dtype == CLT_DTYPE_BF16 ? 2 : 4;
  // row blocks of the column-partial arrays: 32-row blocks of the reduction kernels, or the 128-row half
  // tiles of the dz epilogue that folds the straight-through reductions in (whichever is more)
  const size_t rbs = row_blocks(c->B) > fold_row_blocks(c->B) ? row_blocks(c->B) : fold_row_blocks(c->B);
  const size_t wide = F > d ? F : d;
  Plan p;
  size_t o = 0;
  p.norms = o;      o += align_up(L * F * 4);
  p.G = o;          o += align_up(L * F * 4);
  p.d_yhat = o;     o += align_up(L * B * d * esz);
  p.dpre = o;       o += align_up(L * B * F * esz);
  p.part_cols = o;  o += align_up(rbs * L * wide * 4);
  p.part_cols2 = o; o += align_up(rbs * L * F * 4);
  p.part_cols3 = o; o += align_up(rbs * L * F * 4);
  p.part_rec = o;   o += align_up(rbs * L * 8);
  p.part_sp = o;    o += align_up(rbs * L * 8);
  p.part_dead = o;  o += align_up(rbs * L * 8);
  p.l0 = o;         o += align_up(L * 4);
  p.flags = o;      o += align_up(4 * 4);
  p.xcd_sync = o;   o += align_up(8 * 64 * 4);   // pacing counters of the dense decode, one 256-byte line per XCD
  // row sums of squares of the updated decoder weights, [P][d / 64][F] (reuse_decoder_norms, eligible shapes only)
  const bool n2 = c->reuse_decoder_norms && c->dtype == CLT_DTYPE_BF16 && F % 256 == 0 && d % 256 == 0;
  // (per block and feature: d / 64 runs in the dense kernel's layout, 8 slots per 2048 columns in the row kernel's)
  p.n2_part = o;    o += align_up(n2 ? (L * (L + 1) / 2) * std::max<size_t>(d / 64, 8 * ((d + 2047) / 2048)) * F * 4 : 0);
  p.pre32 = o;      o += align_up(c->activation == CLT_ACT_TOPK ? L * B * F * 4 : 0);   // fp32 pre-activations for the selection
  // active-feature lists of the gather decode: forced gather must hold a fully dense row;
  // the automatic switch only ever gathers below the threshold, so rows are capped at a
  // multiple of it and a step with a longer row falls back to the dense decode
  p.kcap = 0;
  if (c->decode_mode == CLT_DECODE_GATHER) p.kcap = c->F;
  if (c->decode_mode == CLT_DECODE_AUTO) {
    size_t k = (size_t)(32.0 * std::max(c->gather_density_threshold, backward_threshold(c)) * F) + 64;
    k = (k + 7) / 8 * 8;
    p.kcap = (int)(k < F ? k : F);
  }
  const size_t lstride = p.kcap ? (size_t)list_stride(p.kcap) : 0;
  p.g_idx = o;      o += align_up(L * B * lstride * 4);
  p.g_val = o;      o += align_up(L * B * lstride * 4);
  p.g_counts = o;   o += align_up(L * B * 4);
  p.g_counts_w = o; o += align_up(L * B * 4);
  // per-feature token lists of the sparse backward (transpose of the row lists, same capacity)
  const size_t gathers = p.kcap ? 1 : 0;
  p.fl_off = o;     o += align_up(gathers * L * F * 4);
  p.fl_cnt = o;     o += align_up(gathers * L * F * 4);
  // (+16: the row kernel of dW_dec reads list entries four at a time, up to three past a list's end)
  p.fl_tok = o;     o += align_up(L * B * (size_t)p.kcap * 4 + (gathers ? 16 : 0));
  p.fl_val = o;     o += align_up(L * B * (size_t)p.kcap * 4 + (gathers ? 16 : 0));
  p.fl_seg = o;     o += align_up(gathers * FL_SEGS * L * F * 4);
  // partial dot products of the fused dz: (pair, column slice, entry), entries per layer capped (longer lists take
  // the separate gather kernel)
  int per_token = FUSED_DZ_ENTRIES_PER_TOKEN;
  if (c->decode_mode == CLT_DECODE_AUTO)      // what the backward threshold admits, a quarter more for window entries
    per_token = std::min(FUSED_DZ_ENTRIES_PER_TOKEN_MAX, (int)(1.25 * backward_threshold(c) * F) + 32);
  p.ecap = (int)(B * (size_t)std::min(p.kcap, per_token));
  p.dz_part = o;    o += align_up((L * (L + 1) / 2) * 8 * (size_t)p.ecap * 4);
  p.total = o;
  return p;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

#define REQ(h, ptr)                                                                   \
  do {                                                                                \
    if (!(ptr)) { set_err((h)->err, "%s: argument %s is NULL", __func__, #ptr); return CLT_ERR_INVALID_ARG; } \
    if (misaligned(ptr)) { set_err((h)->err, "%s: argument %s is not 16-byte aligned", __func__, #ptr); return CLT_ERR_ALIGN; } \
  } while (0)
#define OPT(h, ptr)                                                                   \
  do {                                                                                \
    if ((ptr) && misaligned(ptr)) { set_err((h)->err, "%s: argument %s is not 16-byte aligned", __func__, #ptr); return CLT_ERR_ALIGN; } \
  } while (0)
#define HIPCHK(h, expr)                                                               \
  do {                                                                                \
    hipError_t e__ = (expr);                                                          \
    if (e__ != hipSuccess) {                                                          \
      set_err((h)->err, "%s: %s failed: %s", __func__, #expr, hipGetErrorString(e__)); \
      return CLT_ERR_HIP;                                                             \
    }                                                                                 \
  } while (0)

hipEvent_t take_event(clt_handle* h) {
  if (!h->free_events.empty()) { hipEvent_t e = h->free_events.back(); h->free_events.pop_back(); return e; }
  hipEvent_t e = nullptr;
  if (hipEventCreate(&e) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
  return e;
}

// Enqueues one kernel; with profiling on, brackets it with events on the same stream.
#define RUN(h, s, kid, expr)                                                          \
  do {                                                                                \
    hipEvent_t ea__ = nullptr, eb__ = nullptr;                                        \
    if ((h)->prof_on && (h)->spans.size() < 65536) {                                  \
      ea__ = take_event(h); eb__ = take_event(h);                                     \
      if (ea__ && eb__) HIPCHK(h, hipEventRecord(ea__, s));                           \
    }                                                                                 \
    HIPCHK(h, expr);                                                                  \
    if (ea__ && eb__) {                                                               \
      HIPCHK(h, hipEventRecord(eb__, s));                                             \
      (h)->spans.push_back(ProfSpan{kid, ea__, eb__});                                \
    }                                                                                 \
  } while (0)

int check_tensors(clt_handle* h, const char* what, const clt_tensors* t, bool need_matrices_only) {
  if (!t) { set_err(h->err, "clt tensors '%s' is NULL", what); return CLT_ERR_INVALID_ARG; }
  const void* ptrs[5] = {t->W_enc, t->b_enc, t->theta, t->W_dec, t->b_dec};
  const char* names[5] = {"W_enc", "b_enc", "theta", "W_dec", "b_dec"};
  for (int i = 0; i < 5; ++i) {
    const bool matrix = (i == 0 || i == 3);
    if (need_matrices_only && !matrix) continue;
    if (!ptrs[i]) { set_err(h->err, "%s.%s is NULL", what, names[i]); return CLT_ERR_INVALID_ARG; }
    if (misaligned(ptrs[i])) { set_err(h->err, "%s.%s is not 16-byte aligned", what, names[i]); return CLT_ERR_ALIGN; }
  }
  return CLT_OK;
}

}  // namespace

extern "C" {

int clt_workspace_bytes(const clt_config* cfg, size_t* bytes) {
  if (!bytes) { set_err(g_err, "clt_workspace_bytes: bytes is NULL"); return CLT_ERR_INVALID_ARG; }
  const int rc = check_config(cfg, g_err);
  if (rc != CLT_OK) return rc;
  *bytes = make_plan(cfg).total;
  return CLT_OK;
}

int clt_init(clt_handle** handle, const clt_config* cfg, void* workspace, size_t workspace_bytes) {
  if (!handle) { set_err(g_err, "clt_init: handle is NULL"); return CLT_ERR_INVALID_ARG; }
  *handle = nullptr;
  const int rc = check_config(cfg, g_err);
  if (rc != CLT_OK) return rc;
  const Plan plan = make_plan(cfg);
  if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & (ALIGN - 1)) || workspace_bytes < plan.total) {
    set_err(g_err, "clt_init: workspace must be non-NULL, 256-byte aligned and at least %zu bytes (got %zu)",
            plan.total, workspace_bytes);
    return CLT_ERR_WORKSPACE;
  }
  int ndev = 0;
  hipError_t e = hipGetDeviceCount(&ndev);
  if (e != hipSuccess || ndev < 1) {
    set_err(g_err, "clt_init: no usable HIP device (%s)", e != hipSuccess ? hipGetErrorString(e) : "count 0");
    (void)hipGetLastError();
    return CLT_ERR_HIP;
  }
  if (cfg->dtype == CLT_DTYPE_BF16) {
    e = init_gemm_bf16();
    if (e != hipSuccess) {
      set_err(g_err, "clt_init: cannot configure the MFMA kernels (%s); this library needs a gfx950 device",
              hipGetErrorString(e));
      (void)hipGetLastError();
      return CLT_ERR_HIP;
    }
  }
  e = init_gather();
  if (e != hipSuccess) {
    set_err(g_err, "clt_init: cannot configure the gather kernels (%s)", hipGetErrorString(e));
    (void)hipGetLastError();
    return CLT_ERR_HIP;
  }
  {   // set-up for clt_norm_accumulate_static on this device (address of the library's own scratch array)
    double* unused = nullptr;
    e = static_scratch(&unused);
    if (e != hipSuccess) {
      set_err(g_err, "clt_init: cannot resolve the static scratch array (%s)", hipGetErrorString(e));
      (void)hipGetLastError();
      return CLT_ERR_HIP;
    }
  }
  clt_handle* h = new (std::nothrow) clt_handle;
  if (!h) { set_err(g_err, "clt_init: out of host memory"); return CLT_ERR_INVALID_ARG; }
  h->cfg = *cfg;
  h->D = Dims{cfg->L, cfg->d, cfg->F, cfg->B};
  h->bf16 = cfg->dtype == CLT_DTYPE_BF16;
  h->int8 = cfg->input_format == CLT_INPUT_INT8_ROWSCALE;
  h->esz = h->bf16 ? 2 : 4;
  h->ws = static_cast<char*>(workspace);
  h->plan = plan;
  h->stage = 0;
  h->n2_eligible = cfg->reuse_decoder_norms && h->bf16 && cfg->F % 256 == 0 && cfg->d % 256 == 0;
  h->n2_for = nullptr;
  h->lambda0 = 0.f;
  h->lambda1 = 0.f;
  h->err[0] = 0;
  *handle = h;
  return CLT_OK;
}

int clt_destroy(clt_handle* handle) {
  if (!handle) return CLT_OK;
  for (ProfSpan& sp : handle->spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
  for (hipEvent_t e : handle->free_events) (void)hipEventDestroy(e);
  delete handle;
  return CLT_OK;
}

int clt_profile_enable(clt_handle* h, int on) {
  if (!h) { set_err(g_err, "clt_profile_enable: handle is NULL"); return CLT_ERR_INVALID_ARG; }
  h->prof_on = on != 0;
  if (h->prof_on) {
    for (ProfSpan& sp : h->spans) { h->free_events.push_back(sp.a); h->free_events.push_back(sp.b); }
    h->spans.clear();
    for (int k = 0; k < K_COUNT; ++k) { h->prof_ms[k] = 0.0; h->prof_n[k] = 0; }
  }
  return CLT_OK;
}

int clt_profile_num_kernels(void) { return K_COUNT; }

int clt_profile_query(clt_handle* h, int kernel, const char** name, double* total_ms, int64_t* launches) {
  if (!h) { set_err(g_err, "clt_profile_query: handle is NULL"); return CLT_ERR_INVALID_ARG; }
  if (kernel < 0 || kernel >= K_COUNT || !name || !total_ms || !launches) {
    set_err(h->err, "clt_profile_query: bad argument");
    return CLT_ERR_INVALID_ARG;
  }
  for (ProfSpan& sp : h->spans) {       // harvest: waits for the recorded events
    float ms = 0.f;
    HIPCHK(h, hipEventSynchronize(sp.b));
    HIPCHK(h, hipEventElapsedTime(&ms, sp.a, sp.b));
    h->prof_ms[sp.kernel] += ms;
    h->prof_n[sp.kernel] += 1;
    h->free_events.push_back(sp.a);
    h->free_events.push_back(sp.b);
  }
  h->spans.clear();
  *name = kKernelNames[kernel];
  *total_ms = h->prof_ms[kernel];
  *launches = h->prof_n[kernel];
  return CLT_OK;
}

int clt_diag_mfma_loop(void* stream, int iters, int mode, void* buf, size_t buf_bytes, uint64_t* counters_dev,
                       double* flop, double* wall_clock_hz) {
  if (!counters_dev || misaligned(counters_dev) || iters < 1 || iters > (1 << 24) || mode < 0 || mode > 255) {
    set_err(g_err, "clt_diag_mfma_loop: counters_dev must be a 16-byte aligned device pointer to 4 x uint64, 1 <= iters <= 2^24, 0 <= mode <= 255");
    return CLT_ERR_INVALID_ARG;
  }
  int dev = 0, cus = 0, khz = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
      hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || cus < 1) {
    set_err(g_err, "clt_diag_mfma_loop: no usable HIP device");
    (void)hipGetLastError();
    return CLT_ERR_HIP;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  const size_t need = (size_t)cus * (DIAG_NEAR_BYTES + DIAG_FAR_BYTES);
  if (mode & (DIAG_LOADS_L2 | DIAG_LOADS_FAR)) {
    if (!(mode & DIAG_LOADS_L2) || !buf || misaligned(buf) || buf_bytes < need) {
      set_err(g_err, "clt_diag_mfma_loop: the load modes need mode bit 8 and a 16-byte aligned device buffer of at least %zu bytes", need);
      return CLT_ERR_INVALID_ARG;
    }
    const hipError_t ef = launch_diag_fill(s, buf, need, mode & DIAG_RANDOM_DATA);
    if (ef != hipSuccess) { set_err(g_err, "clt_diag_mfma_loop: fill failed: %s", hipGetErrorString(ef)); return CLT_ERR_HIP; }
  }
  const hipError_t e = launch_mfma_loop(s, cus, iters, mode, buf, reinterpret_cast<unsigned long long*>(counters_dev));
  if (e != hipSuccess) {
    set_err(g_err, "clt_diag_mfma_loop: mode %d is not built or the launch failed: %s", mode, hipGetErrorString(e));
    (void)hipGetLastError();
    return e == hipErrorInvalidValue ? CLT_ERR_INVALID_ARG : CLT_ERR_HIP;
  }
  if (flop) *flop = (double)cus * 8.0 * (double)iters * 32.0 * 32768.0;
  if (wall_clock_hz) *wall_clock_hz = 1e3 * (double)khz;
  return CLT_OK;
}

const char* clt_last_error(const clt_handle* handle) { return handle ? handle->err : g_err; }

int clt_workspace_view(const clt_handle* h, int which, void** ptr, size_t* bytes) {
  if (!h || !ptr || !bytes) return CLT_ERR_INVALID_ARG;
  const size_t L = h->D.L, d = h->D.d, F = h->D.F, B = h->D.B;
  switch (which) {
    case 0: *ptr = h->ws + h->plan.norms; *bytes = L * F * 4; break;
    case 1: *ptr = h->ws + h->plan.d_yhat; *bytes = L * B * d * h->esz; break;
    case 2: *ptr = h->ws + h->plan.dpre; *bytes = L * B * F * h->esz; break;
    case 3: *ptr = h->ws + h->plan.G; *bytes = L * F * 4; break;
    case 4: *ptr = h->ws + h->plan.flags; *bytes = 16; break;
    default: return CLT_ERR_INVALID_ARG;
  }
  return CLT_OK;
}

int clt_norm_accumulate(clt_handle* h, void* stream, const void* a, const float* a_scale, double* norm_sum) {
  if (!h) { set_err(g_err, "clt_norm_accumulate: handle is NULL"); return CLT_ERR_INVALID_ARG; }
  REQ(h, a); REQ(h, norm_sum);
  if (h->int8) REQ(h, a_scale);
  else if (a_scale) { set_err(h->err, "clt_norm_accumulate: a_scale given but input_format is native"); return CLT_ERR_INVALID_ARG; }
  hipStream_t s = static_cast<hipStream_t>(stream);
  // the per-block partial sums borrow the reconstruction loss's partials, which never outlive a clt_loss call
  double* part = reinterpret_cast<double*>(h->ws + h->plan.part_rec);
  RUN(h, s, K_NORM_SUM, launch_norm_accumulate(s, h->bf16, h->int8, h->D, a, a_scale, part, norm_sum));
  return CLT_OK;
}

int clt_norm_accumulate_static(void* stream, int32_t L, int32_t B, int32_t d, int32_t dtype, int32_t input_format,
                               const void* a, const float* a_scale, double* norm_sum) {
  const bool int8 = input_format == CLT_INPUT_INT8_ROWSCALE;
  if ((dtype != CLT_DTYPE_F32 && dtype != CLT_DTYPE_BF16) || (input_format != CLT_INPUT_NATIVE && !int8) ||
      (int8 && dtype != CLT_DTYPE_BF16)) {
    set_err(g_err, "clt_norm_accumulate_static: bad dtype %d / input_format %d", dtype, input_format);
    return CLT_ERR_INVALID_ARG;
  }
  if (L < 1 || L > 128 || B < 1 || d < 8 || (d % 8)) {
    set_err(g_err, "clt_norm_accumulate_static: unsupported shape L=%d B=%d d=%d (need 1<=L<=128, B>=1, d a positive multiple of 8)", L, B, d);
    return CLT_ERR_SHAPE;
  }
  const size_t need = (size_t)L * row_blocks(B);
  if (need > STATIC_SCRATCH_DOUBLES) {
    set_err(g_err, "clt_norm_accumulate_static: L * ceil(B/%d) = %zu partial sums exceed the library's static scratch of %zu; "
            "use clt_norm_accumulate with a workspace, or split the batch", LOSS_ROWS_PER_BLOCK, need, STATIC_SCRATCH_DOUBLES);
    return CLT_ERR_WORKSPACE;
  }
  if (!a || !norm_sum || (int8 && !a_scale)) {
    set_err(g_err, "clt_norm_accumulate_static: a, norm_sum%s must not be NULL", int8 ? ", a_scale" : "");
    return CLT_ERR_INVALID_ARG;
  }
  if (!int8 && a_scale) { set_err(g_err, "clt_norm_accumulate_static: a_scale given but input_format is native"); return CLT_ERR_INVALID_ARG; }
  if (misaligned(a) || misaligned(norm_sum) || (a_scale && misaligned(a_scale))) {
    set_err(g_err, "clt_norm_accumulate_static: a pointer is not 16-byte aligned");
    return CLT_ERR_ALIGN;
  }
  double* part = nullptr;
  hipError_t e = static_scratch(&part);
  if (e != hipSuccess) {
    set_err(g_err, "clt_norm_accumulate_static: cannot resolve the scratch array on this device: %s", hipGetErrorString(e));
    (void)hipGetLastError();
    return CLT_ERR_HIP;
  }
  e = launch_norm_accumulate(static_cast<hipStream_t>(stream), dtype == CLT_DTYPE_BF16, int8, Dims{L, d, 8, B}, a, a_scale,
                             part, norm_sum);
  if (e != hipSuccess) { set_err(g_err, "clt_norm_accumulate_static: launch failed: %s", hipGetErrorString(e)); return CLT_ERR_HIP; }
  return CLT_OK;
}

int clt_normalise(clt_handle* h, void* stream, const double* norm_sum, int64_t n_tokens, const void* a_in,
                  const float* scale_in, void* a_out, float* scale_out) {
  if (!h) { set_err(g_err, "clt_normalise: handle is NULL"); return CLT_ERR_INVALID_ARG; }
  REQ(h, norm_sum);
  if (n_tokens < 1) { set_err(h->err, "clt_normalise: n_tokens must be >= 1"); return CLT_ERR_INVALID_ARG; }
  if (h->int8) {
    REQ(h, scale_in); REQ(h, scale_out);
    if (a_in || a_out) {
      set_err(h->err, "clt_normalise: int8 rows are normalised through their scales; a_in and a_out must be NULL");
      return CLT_ERR_INVALID_ARG;
    }
  } else {
    REQ(h, a_in); REQ(h, a_out);
    if (scale_in || scale_out) {
      set_err(h->err, "clt_normalise: scales given but input_format is native");
      return CLT_ERR_INVALID_ARG;
    }
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  RUN(h, s, K_NORMALISE, launch_normalise(s, h->bf16, h->int8, h->D, norm_sum, (double)n_tokens, a_in, scale_in, a_out, scale_out));
  return CLT_OK;
}

int clt_forward(clt_handle* h, void* stream, const void* x, const float* x_scale, const void* W_enc,
                const float* b_enc, const float* theta, const void* W_dec, const float* b_dec, void* z, void* pre,
                uint8_t* act_class, float* y_hat, int32_t* l0_per_layer) {
  if (!h) { set_err(g_err, "clt_forward: handle is NULL"); return CLT_ERR_INVALID_ARG; }
  REQ(h, x); REQ(h, W_enc); REQ(h, b_enc); REQ(h, theta); REQ(h, W_dec); REQ(h, b_dec);
  REQ(h, z); REQ(h, act_class); REQ(h, y_hat);
  OPT(h, pre); OPT(h, l0_per_layer);
  if (h->int8) REQ(h, x_scale);
  else if (x_scale) { set_err(h->err, "clt_forward: x_scale given but input_format is native"); return CLT_ERR_INVALID_ARG; }
  hipStream_t s = static_cast<hipStream_t>(stream);
  h->stage = 0;
  float* norms = reinterpret_cast<float*>(h->ws + h->plan.norms);
  int32_t* l0 = l0_per_layer ? l0_per_layer : reinterpret_cast<int32_t*>(h->ws + h->plan.l0);
  int32_t* flags = reinterpret_cast<int32_t*>(h->ws + h->plan.flags);
  RUN(h, s, K_ZERO, launch_zero_i32(s, l0, h->D.L));
  if (h->n2_for && h->n2_for == W_dec)   // the last fused update left the sums of squares of exactly these weights
    RUN(h, s, K_NORMS_REUSE, launch_norms_from_partials(s, h->D, reinterpret_cast<const float*>(h->ws + h->plan.n2_part), norms,
                                                            h->cfg.decode_mode == CLT_DECODE_DENSE ? nullptr : flags, h->plan.kcap));
  else
    RUN(h, s, K_NORMS, launch_decoder_norms(s, h->bf16, h->D, W_dec, norms));
  h->n2_for = nullptr;
  const bool topk = h->cfg.activation == CLT_ACT_TOPK;
  float* pre32 = topk ? reinterpret_cast<float*>(h->ws + h->plan.pre32) : nullptr;
  EncArgs ea{x, x_scale, W_enc, b_enc, theta, h->cfg.ste_bandwidth, z, pre, act_class, l0,
             h->cfg.log_threshold != 0, pre32};
  const int mode = h->cfg.decode_mode;
  DecArgs da{z, W_dec, b_dec, y_hat, mode == CLT_DECODE_AUTO ? flags : nullptr, h->plan.kcap,
             reinterpret_cast<uint32_t*>(h->ws + h->plan.xcd_sync)};
  GatherLists gl{reinterpret_cast<int32_t*>(h->ws + h->plan.g_idx), reinterpret_cast<float*>(h->ws + h->plan.g_val),
                 reinterpret_cast<int32_t*>(h->ws + h->plan.g_counts),
                 reinterpret_cast<int32_t*>(h->ws + h->plan.g_counts_w), h->plan.kcap, list_stride(h->plan.kcap)};
  if (h->bf16) {
    RUN(h, s, K_ENC, launch_enc_bf16(s, h->D, ea, h->int8));
  } else {
    RUN(h, s, K_ENC, launch_enc_f32(s, h->D, ea));
  }
  if (topk) RUN(h, s, K_TOPK, launch_topk_select(s, h->bf16, h->D, pre32, h->cfg.topk_k, z, act_class, l0));
  if (mode != CLT_DECODE_DENSE) {   // Sec. 3.2: density monitor, then the gather path where it pays
    // (automatic mode with dz taken inside the row kernel of dW_dec: the backward works from the per-feature lists
    //  alone, so a row longer than the per-token lists hold does not stop it)
    RUN(h, s, K_DECIDE, launch_decode_decide(s, h->D, l0, h->cfg.gather_density_threshold, backward_threshold(&h->cfg),
                                             mode == CLT_DECODE_GATHER,
                                             mode == CLT_DECODE_AUTO && sparse_dwdec_takes_dz(h->D) && h->plan.ecap > 0,
                                             flags));
    RUN(h, s, K_COMPACT, launch_compact_active(s, h->bf16, h->D, z, act_class, gl, flags));
    RUN(h, s, K_GATHER, launch_gather_decode(s, h->bf16, h->D, gl, W_dec, b_dec, y_hat, flags));
  }
  if (mode != CLT_DECODE_GATHER) {
    if (h->bf16) RUN(h, s, K_DEC, launch_dec_bf16(s, h->D, da));
    else RUN(h, s, K_DEC, launch_dec_f32(s, h->D, da));
  }
  h->stage = 1;
  return CLT_OK;
}

int clt_loss(clt_handle* h, void* stream, const void* y, const float* y_scale, const float* y_hat, const void* z,
             const void* pre, const float* theta, float lambda0, float lambda1, float* loss_dev, float* loss_host) {
  if (!h) { set_err(g_err, "clt_loss: handle is NULL"); return CLT_ERR_INVALID_ARG; }
  REQ(h, y); REQ(h, y_hat); REQ(h, z); REQ(h, loss_dev);
  if (h->int8) REQ(h, y_scale);
  else if (y_scale) { set_err(h->err, "clt_loss: y_scale given but input_format is native"); return CLT_ERR_INVALID_ARG; }
  if (!(lambda0 >= 0.f)) { set_err(h->err, "clt_loss: lambda0 must be >= 0"); return CLT_ERR_INVALID_ARG; }
  if (!(lambda1 >= 0.f)) { set_err(h->err, "clt_loss: lambda1 must be >= 0"); return CLT_ERR_INVALID_ARG; }
  const bool dead = lambda1 > 0.f;
  if (dead && h->cfg.activation == CLT_ACT_TOPK) {
    set_err(h->err, "clt_loss: the dead-feature term (lambda1 > 0) needs a threshold; activation is TopK");
    return CLT_ERR_INVALID_ARG;
  }
  if (dead) { REQ(h, pre); REQ(h, theta); }
  if (h->stage < 1) { set_err(h->err, "clt_loss: call clt_forward first (decoder norms missing)"); return CLT_ERR_STATE; }
  hipStream_t s = static_cast<hipStream_t>(stream);
  const Dims D = h->D;
  const int rbs = row_blocks(D.B);
  float* norms = reinterpret_cast<float*>(h->ws + h->plan.norms);
  float* G = reinterpret_cast<float*>(h->ws + h->plan.G);
  float* part = reinterpret_cast<float*>(h->ws + h->plan.part_cols);
  float* part2 = reinterpret_cast<float*>(h->ws + h->plan.part_cols2);
  double* prec = reinterpret_cast<double*>(h->ws + h->plan.part_rec);
  double* psp = reinterpret_cast<double*>(h->ws + h->plan.part_sp);
  double* pdead = reinterpret_cast<double*>(h->ws + h->plan.part_dead);
  void* d_yhat = h->ws + h->plan.d_yhat;
  h->stage = 1;
  // sparsity (and dead-feature) terms first: their column partials are folded into G
  // before the same partial buffer is reused for the db_dec partials of the reconstruction pass
  RUN(h, s, K_LOSS_SP, launch_loss_sparsity(s, h->bf16, D, z, norms, h->cfg.C, psp, part, dead ? pre : nullptr, theta,
                                            h->cfg.log_threshold != 0, pdead, part2));
  RUN(h, s, K_COLRED, launch_col_reduce(s, part, rbs, D.L * D.F, lambda0 / (float)D.B, nullptr, 0.f, G));
  if (dead)
    RUN(h, s, K_COLRED, launch_col_reduce(s, part2, rbs, D.L * D.F, lambda1 / (float)D.B, nullptr, 0.f, G, true));
  RUN(h, s, K_LOSS_REC, launch_loss_rec(s, h->bf16, h->int8, D, y_hat, y, y_scale, d_yhat, prec, part));
  RUN(h, s, K_LOSS_FINAL, launch_loss_final(s, prec, rbs * D.L, psp, rbs * D.L, dead ? pdead : nullptr,
                                            1.0f / (float)D.B, lambda0, lambda1, loss_dev));
  h->lambda0 = lambda0;
  h->lambda1 = lambda1;
  h->stage = 2;
  if (loss_host) {
    HIPCHK(h, hipMemcpyAsync(loss_host, loss_dev, 4 * sizeof(float), hipMemcpyDeviceToHost, s));
    HIPCHK(h, hipStreamSynchronize(s));
  }
  return CLT_OK;
}

// Backward kernels in stream order.  With `fuse` set, the Adam update of W_enc and
// W_dec happens in the epilogues of the two weight-gradient GEMMs (the matrix
// gradients are written only where gW_enc / gW_dec are not NULL).
static int backward_impl(clt_handle* h, hipStream_t s, const void* x, const float* x_scale, const float* theta,
                         void* W_dec, void* W_enc, const void* z, const uint8_t* act_class, void* gW_enc,
                         float* gb_enc, float* gtheta, void* gW_dec, float* gb_dec, const AdamFuseArgs& fenc,
                         const AdamFuseArgs& fdec) {
  const Dims D = h->D;
  const int rbs = row_blocks(D.B);
  float* norms = reinterpret_cast<float*>(h->ws + h->plan.norms);
  float* G = reinterpret_cast<float*>(h->ws + h->plan.G);
  float* part = reinterpret_cast<float*>(h->ws + h->plan.part_cols);
  float* part2 = reinterpret_cast<float*>(h->ws + h->plan.part_cols2);
  void* d_yhat = h->ws + h->plan.d_yhat;
  float* part3 = reinterpret_cast<float*>(h->ws + h->plan.part_cols3);
  void* dpre = h->ws + h->plan.dpre;
  const float lam1_over_b = h->lambda1 / (float)D.B;

  // db_dec from the column partials that clt_loss left behind
  RUN(h, s, K_COLRED, launch_col_reduce(s, part, rbs, D.L * D.d, 1.0f, nullptr, 0.f, gb_dec));
  // Backward through the decoder: dense GEMMs, or the gather kernels on the lists of the forward
  // pass when the device-side switch selected them (AUTO enqueues both; the one not selected
  // returns at once).
  const int mode = h->cfg.decode_mode;
  int32_t* flags = reinterpret_cast<int32_t*>(h->ws + h->plan.flags);
  const int32_t* skip = mode == CLT_DECODE_AUTO ? flags : nullptr;
  const int kcap = h->plan.kcap;
  const float lam_c_over_b = h->lambda0 * h->cfg.C / (float)D.B;
  DzArgs za{d_yhat, W_dec, z, act_class, norms, lam_c_over_b, h->cfg.C, dpre, lam1_over_b, skip, kcap};
  // dense bf16 backward: the dz epilogue writes the final d pre and the column partials itself.  In the automatic mode
  // that holds for the steps that go backward densely; the others take the reduction kernel, whose partials come in
  // another number of row blocks, and the kernels that sum them look at the switch.
  const bool fold = h->bf16 && mode != CLT_DECODE_GATHER;
  if (fold) { za.x_scale = h->int8 ? x_scale : nullptr; za.part_theta = part; za.part_benc = part2; za.part_below = part3; }
  const int nparts = fold ? fold_row_blocks(D.B) : rbs;
  PartsSwitch psw;
  if (fold && mode == CLT_DECODE_AUTO) psw = PartsSwitch{flags, kcap, rbs};
  DWdecArgs wa{z, d_yhat, W_dec, G, norms, gW_dec, fdec, skip, kcap};
  if (h->n2_eligible && fdec.m) wa.n2_part = reinterpret_cast<float*>(h->ws + h->plan.n2_part);
  DWencArgs ea{x, dpre, gW_enc, W_enc, fenc};
  GatherLists gl{reinterpret_cast<int32_t*>(h->ws + h->plan.g_idx), reinterpret_cast<float*>(h->ws + h->plan.g_val),
                 reinterpret_cast<int32_t*>(h->ws + h->plan.g_counts),
                 reinterpret_cast<int32_t*>(h->ws + h->plan.g_counts_w), kcap, list_stride(kcap)};
  FeatureLists fl{reinterpret_cast<int32_t*>(h->ws + h->plan.fl_off), reinterpret_cast<int32_t*>(h->ws + h->plan.fl_cnt),
                  reinterpret_cast<int32_t*>(h->ws + h->plan.fl_tok), reinterpret_cast<float*>(h->ws + h->plan.fl_val),
                  reinterpret_cast<int32_t*>(h->ws + h->plan.fl_seg), kcap,
                  sparse_dwdec_takes_dz(D) && h->plan.ecap ? reinterpret_cast<float*>(h->ws + h->plan.dz_part) : nullptr,
                  h->plan.ecap};
  if (mode != CLT_DECODE_DENSE) {
    // The row kernel of dW_dec runs before the rest of the backward: when the lists are short enough it also takes
    // the dot products that make up dz at the listed entries, and the separate gather kernel stands down.  (It
    // updates W_dec in place when Adam is fused: nothing after it reads the decoder.)
    RUN(h, s, K_SP_FILL, launch_sparse_dpre_fill(s, h->bf16, D, act_class, norms, lam1_over_b, dpre, flags, kcap));
    RUN(h, s, K_FLISTS, launch_feature_lists(s, h->bf16, D, act_class, z, fl, flags, mode == CLT_DECODE_AUTO));
    // (automatic mode with dz taken inside the row kernel: lists too long for that send the backward to the dense
    //  kernels, so the separate gather kernel would only ever stand down)
    if (!(mode == CLT_DECODE_AUTO && fl.dz_part))
      RUN(h, s, K_GATHER_DZ, launch_gather_dz(s, h->bf16, D, gl, d_yhat, W_dec, norms, lam_c_over_b, h->cfg.C, dpre,
                                              flags, &fl));
    RUN(h, s, K_SP_DWDEC, launch_sparse_dwdec(s, h->bf16, D, fl, wa, flags));
    RUN(h, s, K_GATHER_DZ, launch_dz_from_partials(s, h->bf16, D, fl, norms, lam_c_over_b, h->cfg.C, dpre, flags));
  }
  if (mode != CLT_DECODE_GATHER) {
    if (h->bf16) RUN(h, s, K_DZ, launch_dz_bf16(s, D, za)); else RUN(h, s, K_DZ, launch_dz_f32(s, D, za));
  }
  if (!fold || mode == CLT_DECODE_AUTO)
    RUN(h, s, K_STE, launch_ste_reduce(s, h->bf16, D, dpre, act_class, h->int8 ? x_scale : nullptr, norms, lam1_over_b,
                                       part, part2, part3, fold ? flags : nullptr, kcap));
  if (h->cfg.activation == CLT_ACT_TOPK)     // no threshold: the window partials are all zero, and so is the gradient
    RUN(h, s, K_COLRED, launch_col_reduce(s, part, nparts, D.L * D.F, 1.0f, nullptr, 0.f, gtheta, false, psw));
  else
    RUN(h, s, K_COLRED, launch_dtheta_final(s, part, part3, nparts, D.L * D.F, theta, h->cfg.log_threshold != 0, norms,
                                            1.0f / h->cfg.ste_bandwidth, lam1_over_b, gtheta, psw));
  RUN(h, s, K_COLRED, launch_col_reduce(s, part2, nparts, D.L * D.F, 1.0f, nullptr, 0.f, gb_enc, false, psw));
  if (h->bf16) RUN(h, s, K_DWENC, launch_dwenc_bf16(s, D, ea, h->int8));
  else RUN(h, s, K_DWENC, launch_dwenc_f32(s, D, ea));
  if (mode != CLT_DECODE_GATHER) {
    if (h->bf16) RUN(h, s, K_DWDEC, launch_dwdec_bf16(s, D, wa)); else RUN(h, s, K_DWDEC, launch_dwdec_f32(s, D, wa));
  }
  h->stage = 1;   // the loss by-products are consumed; a new clt_loss is needed before the next backward
  return CLT_OK;
}

static AdamScalars adam_scalars(const clt_handle* h, int64_t t, float lr) {
  const double b1 = h->cfg.beta1, b2 = h->cfg.beta2;
  AdamScalars a;
  a.b1 = h->cfg.beta1; a.omb1 = (float)(1.0 - b1);
  a.b2 = h->cfg.beta2; a.omb2 = (float)(1.0 - b2);
  a.inv_bc2 = (float)(1.0 / (1.0 - pow(b2, (double)t)));
  a.neg_lr_over_bc1 = (float)(-(double)lr / (1.0 - pow(b1, (double)t)));
  a.eps = h->cfg.adam_eps;
  return a;
}

int clt_backward(clt_handle* h, void* stream, const void* x, const float* x_scale, const float* theta,
                 const void* W_dec, const void* z, const uint8_t* act_class, const clt_tensors* grads) {
  if (!h) { set_err(g_err, "clt_backward: handle is NULL"); return CLT_ERR_INVALID_ARG; }
  REQ(h, x); REQ(h, theta); REQ(h, W_dec); REQ(h, z); REQ(h, act_class);
  if (h->int8) REQ(h, x_scale);
  else if (x_scale) { set_err(h->err, "clt_backward: x_scale given but input_format is native"); return CLT_ERR_INVALID_ARG; }
  int rc = check_tensors(h, "grads", grads, false);
  if (rc != CLT_OK) return rc;
  if (h->stage < 2) { set_err(h->err, "clt_backward: call clt_forward and clt_loss first"); return CLT_ERR_STATE; }
  const AdamFuseArgs none{nullptr, nullptr, nullptr, AdamScalars{}};
  return backward_impl(h, static_cast<hipStream_t>(stream), x, x_scale, theta, const_cast<void*>(W_dec), nullptr, z,
                       act_class, grads->W_enc, grads->b_enc, grads->theta, grads->W_dec, grads->b_dec, none, none);
}

int clt_backward_adam_step(clt_handle* h, void* stream, const void* x, const float* x_scale, const void* z,
                           const uint8_t* act_class, int64_t t, float lr, const clt_tensors* params,
                           const clt_tensors* grads, const clt_tensors* m, const clt_tensors* v,
                           const clt_tensors* master) {
  if (!h) { set_err(g_err, "clt_backward_adam_step: handle is NULL"); return CLT_ERR_INVALID_ARG; }
  REQ(h, x); REQ(h, z); REQ(h, act_class);
  if (h->int8) REQ(h, x_scale);
  else if (x_scale) { set_err(h->err, "clt_backward_adam_step: x_scale given but input_format is native"); return CLT_ERR_INVALID_ARG; }
  if (t < 1) { set_err(h->err, "clt_backward_adam_step: step count t must be >= 1"); return CLT_ERR_INVALID_ARG; }
  if (!(lr >= 0.f)) { set_err(h->err, "clt_backward_adam_step: lr must be >= 0"); return CLT_ERR_INVALID_ARG; }
  int rc;
  if ((rc = check_tensors(h, "params", params, false)) != CLT_OK) return rc;
  if ((rc = check_tensors(h, "m", m, false)) != CLT_OK) return rc;
  if ((rc = check_tensors(h, "v", v, false)) != CLT_OK) return rc;
  if (!grads || !grads->b_enc || !grads->theta || !grads->b_dec) {
    set_err(h->err, "clt_backward_adam_step: grads->b_enc, theta and b_dec are required");
    return CLT_ERR_INVALID_ARG;
  }
  if (misaligned(grads->b_enc) || misaligned(grads->theta) || misaligned(grads->b_dec) ||
      (grads->W_enc && misaligned(grads->W_enc)) || (grads->W_dec && misaligned(grads->W_dec))) {
    set_err(h->err, "clt_backward_adam_step: a gradient pointer is not 16-byte aligned");
    return CLT_ERR_ALIGN;
  }
  if (h->cfg.master_weights) {
    if ((rc = check_tensors(h, "master", master, true)) != CLT_OK) return rc;
  } else if (master) {
    set_err(h->err, "clt_backward_adam_step: master given but config.master_weights is 0");
    return CLT_ERR_INVALID_ARG;
  }
  if (h->stage < 2) { set_err(h->err, "clt_backward_adam_step: call clt_forward and clt_loss first"); return CLT_ERR_STATE; }
  hipStream_t s = static_cast<hipStream_t>(stream);
  const Dims D = h->D;
  const AdamScalars a = adam_scalars(h, t, lr);
  const AdamFuseArgs fenc{(float*)m->W_enc, (float*)v->W_enc, master ? (float*)master->W_enc : nullptr, a};
  const AdamFuseArgs fdec{(float*)m->W_dec, (float*)v->W_dec, master ? (float*)master->W_dec : nullptr, a};
  h->n2_for = nullptr;
  rc = backward_impl(h, s, x, x_scale, params->theta, params->W_dec, params->W_enc, z, act_class, grads->W_enc,
                     grads->b_enc, grads->theta, grads->W_dec, grads->b_dec, fenc, fdec);
  if (rc != CLT_OK) return rc;
  // the weight-gradient kernel that ran (dense GEMM or row kernel) has updated W_dec and left the row sums of
  // squares of the new weights
  if (h->n2_eligible) h->n2_for = params->W_dec;
  RUN(h, s, K_ADAM_VEC, launch_adam_vector(s, (size_t)D.L * D.F, params->b_enc, grads->b_enc, m->b_enc, v->b_enc, a));
  RUN(h, s, K_ADAM_VEC, launch_adam_vector(s, (size_t)D.L * D.F, params->theta, grads->theta, m->theta, v->theta, a));
  RUN(h, s, K_ADAM_VEC, launch_adam_vector(s, (size_t)D.L * D.d, params->b_dec, grads->b_dec, m->b_dec, v->b_dec, a));
  return CLT_OK;
}

int clt_adam_step(clt_handle* h, void* stream, int64_t t, float lr, const clt_tensors* params,
                  const clt_tensors* grads, const clt_tensors* m, const clt_tensors* v, const clt_tensors* master) {
  if (!h) { set_err(g_err, "clt_adam_step: handle is NULL"); return CLT_ERR_INVALID_ARG; }
  if (t < 1) { set_err(h->err, "clt_adam_step: step count t must be >= 1"); return CLT_ERR_INVALID_ARG; }
  if (!(lr >= 0.f)) { set_err(h->err, "clt_adam_step: lr must be >= 0"); return CLT_ERR_INVALID_ARG; }
  int rc;
  if ((rc = check_tensors(h, "params", params, false)) != CLT_OK) return rc;
  if ((rc = check_tensors(h, "grads", grads, false)) != CLT_OK) return rc;
  if ((rc = check_tensors(h, "m", m, false)) != CLT_OK) return rc;
  if ((rc = check_tensors(h, "v", v, false)) != CLT_OK) return rc;
  if (h->cfg.master_weights) {
    if ((rc = check_tensors(h, "master", master, true)) != CLT_OK) return rc;
  } else if (master) {
    set_err(h->err, "clt_adam_step: master given but config.master_weights is 0");
    return CLT_ERR_INVALID_ARG;
  }
  hipStream_t s = static_cast<hipStream_t>(stream);
  const Dims D = h->D;
  const AdamScalars a = adam_scalars(h, t, lr);
  h->n2_for = nullptr;   // W_dec changes here without new row sums
  const size_t n_enc = (size_t)D.L * D.d * D.F, n_dec = (size_t)D.P() * D.F * D.d;
  RUN(h, s, K_ADAM_WDEC, launch_adam_matrix(s, h->bf16, n_dec, params->W_dec, grads->W_dec, (float*)m->W_dec, (float*)v->W_dec,
                               master ? (float*)master->W_dec : nullptr, a));
  RUN(h, s, K_ADAM_WENC, launch_adam_matrix(s, h->bf16, n_enc, params->W_enc, grads->W_enc, (float*)m->W_enc, (float*)v->W_enc,
                               master ? (float*)master->W_enc : nullptr, a));
  RUN(h, s, K_ADAM_VEC, launch_adam_vector(s, (size_t)D.L * D.F, params->b_enc, grads->b_enc, m->b_enc, v->b_enc, a));
  RUN(h, s, K_ADAM_VEC, launch_adam_vector(s, (size_t)D.L * D.F, params->theta, grads->theta, m->theta, v->theta, a));
  RUN(h, s, K_ADAM_VEC, launch_adam_vector(s, (size_t)D.L * D.d, params->b_dec, grads->b_dec, m->b_dec, v->b_dec, a));
  return CLT_OK;
}

}  // extern "C"
