// Shared declarations of the HIP side of libclt: problem dimensions, bf16
// helpers and the internal launch interface between the C ABI (clt_api.hip)
// and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace clt {

struct Dims {
  int L, d, F, B;
  __host__ __device__ int P() const { return L * (L + 1) / 2; }
};

// Packed index of decoder block (source l -> target lp), source-major (eq. 3).
__host__ __device__ inline int packed_index(int l, int lp, int L) {
  return l * L - (l * (l - 1)) / 2 + (lp - l);
}

typedef uint16_t bf16_t;  // raw bf16 bits

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// float -> bf16, round to nearest even (NaN stays NaN): gfx950's packed conversion instruction.
typedef __bf16 hw_bf16x2 __attribute__((ext_vector_type(2)));
typedef float hw_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const hw_f32x2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, hw_bf16x2));
}
__device__ __forceinline__ bf16_t f32_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.0f) & 0xffffu); }

// Streaming (non-temporal) 16- and 8-byte accesses for the optimizer state and weights in the
// update epilogues of the contractions: data touched once there should not displace the operand
// panels that the contractions reuse out of the L2.  (Kernels that do nothing but stream are
// faster with plain accesses and do not use these.)
typedef float nt_f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int nt_u32x2 __attribute__((ext_vector_type(2)));
#define CLT_NT_LOAD(p) __builtin_nontemporal_load(p)
#define CLT_NT_STORE(v, p) __builtin_nontemporal_store(v, p)
__device__ __forceinline__ nt_f32x4 nt_load_v4(const float* p) { return CLT_NT_LOAD(reinterpret_cast<const nt_f32x4*>(p)); }
__device__ __forceinline__ float4 nt_load_f4(const float* p) {
  const nt_f32x4 v = nt_load_v4(p);
  return make_float4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void nt_store_f4(float* p, float4 v) {
  const nt_f32x4 t = {v.x, v.y, v.z, v.w};
  CLT_NT_STORE(t, reinterpret_cast<nt_f32x4*>(p));
}

// Element-type traits for the two storage types.
template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
  static __device__ __forceinline__ void store4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
  static __device__ __forceinline__ float4 load4(const float* p) { return *reinterpret_cast<const float4*>(p); }
  static __device__ __forceinline__ float4 nt_load4(const float* p) { return nt_load_f4(p); }
  static __device__ __forceinline__ void nt_store4(float* p, float4 v) { nt_store_f4(p, v); }
  // 4 elements as they come out of memory; widen4() turns them into floats.  Code that wants loads
  // in flight across other work keeps the raw form until the values are used: arithmetic on a
  // loaded value is where the wait for that load goes.
  typedef float4 Raw4;
  static __device__ __forceinline__ Raw4 load_raw4(const float* p) { return load4(p); }
  static __device__ __forceinline__ Raw4 nt_load_raw4(const float* p) { return nt_load_f4(p); }
  static __device__ __forceinline__ float4 widen4(Raw4 r) { return r; }
  static __device__ __forceinline__ Raw4 narrow4(float4 v) { return v; }
  static __device__ __forceinline__ void nt_store_raw4(float* p, Raw4 v) { nt_store_f4(p, v); }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
  static __device__ __forceinline__ void store4(bf16_t* p, float4 v) {
    uint2 u;
    u.x = pack_bf16x2(v.x, v.y);
    u.y = pack_bf16x2(v.z, v.w);
    *reinterpret_cast<uint2*>(p) = u;
  }
  static __device__ __forceinline__ float4 load4(const bf16_t* p) {
    uint2 u = *reinterpret_cast<const uint2*>(p);
    return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
                       __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u));
  }
  static __device__ __forceinline__ float4 nt_load4(const bf16_t* p) {
    const nt_u32x2 u = CLT_NT_LOAD(reinterpret_cast<const nt_u32x2*>(p));
    return make_float4(__uint_as_float(u[0] << 16), __uint_as_float(u[0] & 0xffff0000u),
                       __uint_as_float(u[1] << 16), __uint_as_float(u[1] & 0xffff0000u));
  }
  static __device__ __forceinline__ void nt_store4(bf16_t* p, float4 v) {
    const nt_u32x2 u = {pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w)};
    CLT_NT_STORE(u, reinterpret_cast<nt_u32x2*>(p));
  }
  typedef nt_u32x2 Raw4;
  static __device__ __forceinline__ Raw4 load_raw4(const bf16_t* p) { return *reinterpret_cast<const nt_u32x2*>(p); }
  static __device__ __forceinline__ Raw4 nt_load_raw4(const bf16_t* p) { return CLT_NT_LOAD(reinterpret_cast<const nt_u32x2*>(p)); }
  static __device__ __forceinline__ float4 widen4(Raw4 u) {
    return make_float4(__uint_as_float(u[0] << 16), __uint_as_float(u[0] & 0xffff0000u),
                       __uint_as_float(u[1] << 16), __uint_as_float(u[1] & 0xffff0000u));
  }
  static __device__ __forceinline__ Raw4 narrow4(float4 v) {
    const Raw4 u = {pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w)};
    return u;
  }
  static __device__ __forceinline__ void nt_store_raw4(bf16_t* p, Raw4 u) { CLT_NT_STORE(u, reinterpret_cast<nt_u32x2*>(p)); }
};

// Adam (App. C Table 1) with bias correction, the step's scalars folded on the host:
//   m' = b1 m + (1-b1) g,  v' = b2 v + (1-b2) g^2,
//   p' = p - lr (m'/(1-b1^t)) / (sqrt(v'/(1-b2^t)) + eps)
struct AdamScalars { float b1, omb1, b2, omb2, inv_bc2, neg_lr_over_bc1, eps; };
// One element.  Square root and reciprocal are the hardware approximations (1 ulp each); the
// correctly rounded forms cost ten times the instructions in epilogues that are ALU-bound.
__device__ __forceinline__ void adam_element(float& p, float& m, float& v, float g, const AdamScalars& a) {
  m = fmaf(a.b1, m, a.omb1 * g);
  v = fmaf(a.b2, v, (a.omb2 * g) * g);
  const float den = __builtin_amdgcn_sqrtf(v * a.inv_bc2) + a.eps;
  p = fmaf(a.neg_lr_over_bc1 * m, __builtin_amdgcn_rcpf(den), p);
}

// Sum over each row of 16 lanes, result in all of them: four adds on data-parallel-primitive operands (swaps
// inside quads, then mirrored half rows and rows), no LDS round trips.
template <int CTRL> __device__ __forceinline__ float dpp_move(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_move<0x141>(v);   // row_half_mirror: the other quad of the half row
  v += dpp_move<0x140>(v);   // row_mirror: the other half row
  return v;
}

// act_class bits
constexpr uint8_t CLS_ACTIVE = 1;
constexpr uint8_t CLS_WINDOW = 2;
constexpr uint8_t CLS_BELOW = 4;   // pre < theta strictly (where the dead-feature term has a gradient)

// The stored threshold parameter is theta itself or tau = log(theta) (App. B writes exp(tau)).
__device__ __forceinline__ float threshold_value(float param, bool log_threshold) {
  return log_threshold ? expf(param) : param;
}

// ---------------------------------------------------------------------------
// Launch interface.  `bf16` selects the storage type T of matrices/activations.
// All functions enqueue on `s` and return the launch status.
// ---------------------------------------------------------------------------
struct EncArgs {       // pre = x W_enc + b_enc; JumpReLU; classes; L0 counts
  const void* x; const float* x_scale; const void* W_enc; const float* b_enc; const float* theta;
  float ste_eps; void* z; void* pre; uint8_t* cls; int32_t* l0;
  bool log_threshold;     // theta holds tau = log(theta)
  float* pre32 = nullptr; // TopK activation: store only the fp32 pre-activation (activation applied by launch_topk_select)
};
struct DecArgs {       // y_hat[lp] = sum_{l<=lp} z[l] W_dec[p(l,lp)] + b_dec[lp]
  const void* z; const void* W_dec; const float* b_dec; float* y_hat;
  const int32_t* skip_flags;   // optional decode switch (see GatherLists); NULL = always run
  int kcap;
  uint32_t* xcd_sync = nullptr;   // bf16 kernel: 8 x 64 words of pacing counters (zeroed by the launch), or NULL
};
struct DzArgs {        // dz[l] = sum_{lp>=l} dyhat[lp] W_dec[p(l,lp)]^T + g_sp, kept where active|window
  const void* d_yhat; const void* W_dec; const void* z; const uint8_t* cls; const float* norms;
  float lam_c_over_b; float C; void* dpre;
  float lam1_over_b;      // dead-feature coefficient lambda1 / B (0 = term off)
  const int32_t* skip_flags = nullptr;   // optional switch: stand down when the gather path is selected
  int kcap = 0;
  // bf16 kernel only, all four or none: the straight-through reductions folded into the epilogue (then dpre is
  // final and launch_ste_reduce is not needed).  Column partials per 128-row half tile, fold_row_blocks(B) of
  // them: [half tile][L][F].  x_scale: the row scales of int8 inputs, or NULL.
  const float* x_scale = nullptr; float* part_theta = nullptr; float* part_benc = nullptr; float* part_below = nullptr;
};
inline int fold_row_blocks(int B) { return 2 * ((B + 255) / 256); }
// Optional Adam fused into the two weight-gradient GEMMs (m == nullptr: plain gradient output)
struct AdamFuseArgs { float* m; float* v; float* master; AdamScalars a; };
struct DWdecArgs {     // dW_dec[p] = z[l]^T dyhat[lp] + (G/n)[l,f] W_dec[p][f,:]
  const void* z; const void* d_yhat; void* W_dec; const float* G; const float* norms; void* dW_dec;
  AdamFuseArgs fuse;
  const int32_t* skip_flags = nullptr;   // as in DzArgs
  int kcap = 0;
  // optional, bf16 kernel with the fused update and F, d multiples of 256: [P][d / 64][F] sums of squares of the
  // updated weights (see launch_norms_from_partials)
  float* n2_part = nullptr;
};
struct DWencArgs {     // dW_enc[l] = x[l]^T dpre[l]
  const void* x; const void* dpre; void* dW_enc; void* W_enc;
  AdamFuseArgs fuse;
};

hipError_t launch_enc_f32(hipStream_t s, Dims D, const EncArgs& a);
hipError_t launch_dec_f32(hipStream_t s, Dims D, const DecArgs& a);
hipError_t launch_dz_f32(hipStream_t s, Dims D, const DzArgs& a);
hipError_t launch_dwdec_f32(hipStream_t s, Dims D, const DWdecArgs& a);
hipError_t launch_dwenc_f32(hipStream_t s, Dims D, const DWencArgs& a);

hipError_t launch_enc_bf16(hipStream_t s, Dims D, const EncArgs& a, bool int8_x);
hipError_t launch_dec_bf16(hipStream_t s, Dims D, const DecArgs& a);
hipError_t launch_dz_bf16(hipStream_t s, Dims D, const DzArgs& a);
hipError_t launch_dwdec_bf16(hipStream_t s, Dims D, const DWdecArgs& a);
hipError_t launch_dwenc_bf16(hipStream_t s, Dims D, const DWencArgs& a, bool int8_x);
hipError_t init_gemm_bf16();   // one-time function attributes (LDS size)

// Elementwise / reduction kernels (kernels_elementwise.hip)
constexpr int LOSS_ROWS_PER_BLOCK = 32;   // token rows per block of the row-blocked reductions
inline int row_blocks(int B) { return (B + LOSS_ROWS_PER_BLOCK - 1) / LOSS_ROWS_PER_BLOCK; }

hipError_t launch_zero_i32(hipStream_t s, int32_t* p, int n);
// activation normalisation (Sec. 3.1): norm_sum[l] += sum over the B rows of ||a[l,b,:]||_2 (part: row_blocks(B)*L
// doubles of scratch); then a / c[l] with c[l] = norm_sum[l] / n_tokens, folded into the row scales for int8 rows
hipError_t launch_norm_accumulate(hipStream_t s, bool bf16, bool int8_a, Dims D, const void* a, const float* a_scale,
                                  double* part, double* norm_sum);
// Capacity of the library-owned scratch array (doubles) and its device address on the current GPU
constexpr size_t STATIC_SCRATCH_DOUBLES = 65536;
hipError_t static_scratch(double** ptr);
hipError_t launch_normalise(hipStream_t s, bool bf16, bool int8_a, Dims D, const double* norm_sum, double n_tokens,
                            const void* a_in, const float* scale_in, void* a_out, float* scale_out);
// TopK activation (Sec. 3.2): per (layer, token) row of pre32 [L,B,F] the k largest entries (lower index wins
// ties) -> z = pre there, 0 elsewhere; class byte CLS_ACTIVE or 0; l0[l] += k per row
hipError_t launch_topk_select(hipStream_t s, bool bf16, Dims D, const float* pre32, int k, void* z, uint8_t* cls,
                              int32_t* l0);
hipError_t launch_decoder_norms(hipStream_t s, bool bf16, Dims D, const void* W_dec, float* norms);
// the same norms from the partial sums of squares a fused weight-gradient launch left behind:
// n[l,f] = sqrt(sum over the blocks p(l, l..L-1) and their d / 64 column runs of n2_part[p][run][f]), in that order
// (flags: the device-side decode switch of the step that left the sums, NULL when only the dense kernels run)
hipError_t launch_norms_from_partials(hipStream_t s, Dims D, const float* n2_part, float* norms, const int32_t* flags,
                                      int kcap);
// L_rec partials, d_yhat = 2 r / B, column partials for db_dec
hipError_t launch_loss_rec(hipStream_t s, bool bf16, bool int8_y, Dims D, const float* y_hat, const void* y,
                           const float* y_scale, void* d_yhat, double* loss_part, float* col_part);
// L_sp partials and column partials of C z sech^2(C z n)
// with pre != NULL also the dead-feature partial sums: sum relu(theta - pre) n into dead_part and the column
// partials of relu(theta - pre) into dead_col_part
hipError_t launch_loss_sparsity(hipStream_t s, bool bf16, Dims D, const void* z, const float* norms, float C,
                                double* loss_part, float* col_part, const void* pre, const float* theta,
                                bool log_threshold, double* dead_part, float* dead_col_part);
// final loss: loss_dev = {rec + sp + dead, rec, sp, dead}
hipError_t launch_loss_final(hipStream_t s, const double* part_rec, int n_rec, const double* part_sp, int n_sp,
                             const double* part_dead_or_null, float inv_B, float lambda0, float lambda1,
                             float* loss_dev);
// Automatic mode: the column partials of the backward come in nparts row blocks when the dense dz epilogue wrote
// them and in nparts_lists when the list-driven backward ran (launch_ste_reduce); which, the device-side switch says.
struct PartsSwitch { const int32_t* flags = nullptr; int kcap = 0; int nparts_lists = 0; };
// out[c] = alpha * sum_r part[r][c] (fixed order), optionally times -(theta[c]/eps)
hipError_t launch_col_reduce(hipStream_t s, const float* part, int nparts, int ncols, float alpha,
                             const float* theta_or_null, float inv_eps, float* out, bool accumulate = false,
                             PartsSwitch sw = PartsSwitch{});
// dtheta[c] = -(theta/eps) sum_r part_win[r][c] + lam1_over_b * norms[c] * sum_r part_below[r][c], times theta
// when the parameter is log(theta)
hipError_t launch_dtheta_final(hipStream_t s, const float* part_win, const float* part_below, int nparts, int ncols,
                               const float* theta_param, bool log_threshold, const float* norms, float inv_eps,
                               float lam1_over_b, float* out, PartsSwitch sw = PartsSwitch{});
// reads dz kept where active|window: column partials for dtheta (window) and db_enc (active);
// zeroes entries that are in the window but not active so the buffer becomes dpre
// (entries that are below the threshold get the dead-feature gradient -lam1_over_b * n; part_below counts them)
// (only_if_lists: automatic mode with the dz epilogue doing this work for the dense backward -- the kernel then runs
//  only when the list-driven backward was selected)
hipError_t launch_ste_reduce(hipStream_t s, bool bf16, Dims D, void* dpre, const uint8_t* cls,
                             const float* row_scale_or_null, const float* norms, float lam1_over_b,
                             float* part_theta, float* part_benc, float* part_below,
                             const int32_t* only_if_lists = nullptr, int kcap = 0);

// p, g in T (or p in T with fp32 master); m, v float
hipError_t launch_adam_matrix(hipStream_t s, bool bf16, size_t n, void* p, const void* g, float* m, float* v,
                              float* master_or_null, AdamScalars a);
hipError_t launch_adam_vector(hipStream_t s, size_t n, float* p, const float* g, float* m, float* v, AdamScalars a);

// Diagnostic (kernels_diag.hip): the contraction kernel's instruction stream taken apart.  `workgroups` x 8 waves x
// iters x 64 v_mfma_f32_16x16x32_bf16; mode bits add the LDS and memory traffic of the real kernel; out[0] / out[1] =
// shader cycles / constant-rate ticks that wave 0 spent in its loop.  buf: workgroups * (NEAR + FAR) bytes when a
// load bit is set.
constexpr int DIAG_RANDOM_DATA = 1, DIAG_LDS_READS = 2, DIAG_LDS_WRITES = 4, DIAG_LOADS_L2 = 8, DIAG_LOADS_FAR = 16,
              DIAG_FOUR_WAVES = 32, DIAG_LDS_DMA = 64, DIAG_MFMA_32X32 = 128;
constexpr size_t DIAG_NEAR_BYTES = 64u << 10, DIAG_FAR_BYTES = 512u << 10;
hipError_t launch_mfma_loop(hipStream_t s, int workgroups, int iters, int mode, const void* buf, unsigned long long* out);
hipError_t launch_diag_fill(hipStream_t s, void* buf, size_t bytes, int random_data);

// ---- active-feature gather paths (kernels_gather.hip) -------------------------
// Device-side switch, 4 ints in the workspace:
//   [0] bit 0: the measured density allows the gather decode (or it is forced); bit 1: it allows the list-driven
//       backward through the decoder (or it is forced); bit 2: that backward does not need the row lists
//   [1] longest per-(layer, token) list seen by the compaction (active + window-only entries)
//   [2] path taken by the last forward: 1 dense, 2 gather
//   [3] longest per-layer total of the feature lists (see fused_dz_selected)
// The list-driven kernels run only when their bit of flags[0] is set and flags[1] <= kcap; the dense kernels that
// carry the same flags stand down in exactly that case.
__host__ __device__ inline bool gather_selected(const int32_t* flags, int kcap) {
  return (flags[0] & 1) != 0 && flags[1] <= kcap;
}
// The backward through the decoder (dz, dW_dec) has a switch of its own, flags[0] bit 1: its list-driven kernels pay
// up to a higher density than the gather decode does.
// Bit 2 says that this backward does not touch the per-(layer, token) lists (dz is taken inside the row kernel of
// dW_dec, which works from the per-feature lists; their capacity is checked when they are built): a token with more
// listed features than a row holds then only sends the forward decode back to the dense kernel.
__host__ __device__ inline bool lists_backward_selected(const int32_t* flags, int kcap) {
  return (flags[0] & 2) != 0 && ((flags[0] & 4) != 0 || flags[1] <= kcap);
}
// Per (layer, token) row of kcap slots: the active features in ascending order from the front
// (counts[row] of them, val = z), the inactive features inside the threshold window from the
// back (counts_w[row] of them, slot kcap-1 first, val = 0).  Rows are `stride` slots apart
// (list_stride(kcap): never a multiple of 4 KB, or the heads of all rows would share one L2 channel).
struct GatherLists { int32_t* idx; float* val; int32_t* counts; int32_t* counts_w; int kcap; int stride; };
__host__ __device__ inline int list_stride(int kcap) { return kcap + 32; }
// flags[0] = (sum l0 <= threshold * L*B*F) or forced; flags[1] = 0
hipError_t launch_decode_decide(hipStream_t s, Dims D, const int32_t* l0, float density_threshold,
                                float backward_density_threshold, int forced, bool backward_without_row_lists,
                                int32_t* flags);
hipError_t launch_compact_active(hipStream_t s, bool bf16, Dims D, const void* z, const uint8_t* cls, GatherLists g,
                                 int32_t* flags);
// y_hat[lp, b, :] = b_dec[lp] + sum_{l<=lp} sum_{active f} z[l,b,f] W_dec[p(l,lp)][f, :]; records the path in flags[2]
hipError_t launch_gather_decode(hipStream_t s, bool bf16, Dims D, GatherLists g, const void* W_dec,
                                const float* b_dec, float* y_hat, int32_t* flags);

// Sparse backward through the decoder (same switch).
// dpre := 0, or the dead-feature gradient -(lambda1/B) n where pre < theta and the entry is not listed
hipError_t launch_sparse_dpre_fill(hipStream_t s, bool bf16, Dims D, const uint8_t* cls, const float* norms,
                                   float lam1_over_b, void* dpre, const int32_t* flags, int kcap);
hipError_t init_gather();   // once per process, after the device is chosen
// Per (layer, feature): tokens on which the feature is active or inside the threshold window, ascending, with z
// (0 for the window-only ones; transpose of the row lists).
// Layer l's entries start at l * B * kcap; off is layer-local.  seg holds FL_SEGS x L*F partial counts.
constexpr int FL_SEGS = 16;
// dz_part / ecap: room for the partial dot products of the fused dz (see fused_dz_selected), P x 8 x ecap floats.
struct FeatureLists { int32_t* off; int32_t* cnt; int32_t* tok; float* val; int32_t* seg; int kcap; float* dz_part; int ecap; };
// flags[3] = longest per-layer total of the feature lists (raised by launch_feature_lists, cleared by
// launch_decode_decide).  While it fits ecap, the row kernel of dW_dec also takes the dot products d y_hat . W_dec of
// its (entry, target, column slice) and launch_dz_from_partials sums them into d pre; launch_gather_dz stands down.
__host__ __device__ inline bool fused_dz_selected(const int32_t* flags, const FeatureLists& fl) {
  return fl.dz_part != nullptr && lists_backward_selected(flags, fl.kcap) && flags[3] <= fl.ecap;
}
constexpr int FUSED_DZ_ENTRIES_PER_TOKEN = 128;      // forced gather mode: ecap = B * min(kcap, this)
constexpr int FUSED_DZ_ENTRIES_PER_TOKEN_MAX = 320;  // automatic mode: sized from the backward threshold, up to this
bool sparse_dwdec_takes_dz(Dims D);                  // whether launch_sparse_dwdec will use the kernel that can (else: dz_part = NULL)
// dz at the listed entries only: sum_{lp>=l} <d_yhat[lp,b,:], W_dec[p(l,lp)][f,:]> + sparsity gradient -> dpre[l,b,f]
hipError_t launch_gather_dz(hipStream_t s, bool bf16, Dims D, GatherLists g, const void* d_yhat, const void* W_dec,
                            const float* norms, float lam_c_over_b, float C, void* dpre, const int32_t* flags,
                            const FeatureLists* fused);      // fused: stands down when fused_dz_selected(flags, *fused)
// dense_when_too_long (automatic mode): a layer total beyond ecap clears bit 1 of flags[0], which hands the backward
// through the decoder back to the dense kernels.
hipError_t launch_feature_lists(hipStream_t s, bool bf16, Dims D, const uint8_t* cls, const void* z, FeatureLists fl,
                                int32_t* flags, bool dense_when_too_long);
// d pre at the listed entries from the partial dot products the row kernel of dW_dec left (fused_dz_selected only)
hipError_t launch_dz_from_partials(hipStream_t s, bool bf16, Dims D, FeatureLists fl, const float* norms,
                                   float lam_c_over_b, float C, void* dpre, const int32_t* flags);
// dW_dec[p(l,lp)][f,:] = sum_{b in list(l,f)} z[l,b,f] d_yhat[lp,b,:] + (G/n)[l,f] W_dec[p][f,:], with the optional
// fused Adam update of the row (every row is visited: Adam also moves rows without gradient)
// (a.n2_part, bf16 with the fused update and d a multiple of 64: the row kernel leaves the same sums of squares of the
// updated weights as the dense fused kernel)
hipError_t launch_sparse_dwdec(hipStream_t s, bool bf16, Dims D, FeatureLists fl, const DWdecArgs& a,
                               const int32_t* flags);

}  // namespace clt
