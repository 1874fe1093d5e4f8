// The five contractions of a CLT train step, each described as a "policy":
// operand addressing (which memory dimension is the contraction index K), the
// K segments of the triangular sums, and the fused epilogue.  The same policies
// drive the fp32 FMA kernel (kernels_gemm_f32.hip) and the bf16 MFMA kernel
// (kernels_gemm_bf16.hip).
//
// A policy exposes
//   A_KC / B_KC  true when the operand is contiguous along K in memory
//                (A element (m,k) at a[m*lda + k]; otherwise at a[k*lda + m];
//                 B element (k,n) at b[n*ldb + k] when B_KC, else b[k*ldb + n])
//   M, N, kseg   tile-space extents and the length of one K segment
//   ginfo(order) group visited at position `order` of the launch (longest K first)
//   nseg(gi), a_seg(gi,s), b_seg(gi,s)   K segments of a group
//   epi_begin(st, gi, col, ok, row0)   once per tile and lane: loads what depends on the lane's
//                columns only (biases, thresholds, norms) when `ok` (col inside the matrix); row0 is the
//                first row of the block whose rows this lane will see (wave-uniform in the bf16 kernel)
//   epi_load(regs, gi, pos)       issues the global loads the epilogue of that 4-column
//                group needs and keeps the results as loaded (no arithmetic on them here: that
//                is where the wait for the load would land).  The bf16 kernel calls it ahead of
//                use: EPI_BATCH / EPI_BATCH_LATE / EPI_BATCH_LAST groups ahead in the first
//                quarter / second quarter / second half of a wave's block
//   epi4(st, gi, pos, v, regs)    consumes 4 accumulators of one row, columns col..col+3
//   PERSISTENT   the bf16 kernel runs one workgroup per CU over many tiles (else one per tile)
//   UNIFORM_K    every group of a launch has the same K length
#pragma once
#include "common.h"

#include <type_traits>

namespace clt {

// Maps a workgroup index to (group order, tile row, tile column).
// Workgroups are dealt round-robin to the 8 XCDs, each with a private L2.  The
// XCDs form teams of S (1, 2, 4 or 8): a team works on one group at a time and
// each of its XCDs takes a contiguous 1/S of that group's tile list, sized so
// that the ~32 tiles an XCD has in flight belong to one group.  The list runs
// through column panels SN tiles wide, so those tiles form a compact 2-D block
// that shares few A and B panels in the XCD's L2.  Groups arrive sorted by
// decreasing K and are handed to the teams in snake order (0..n-1, n-1..0, ...),
// which balances the teams' total work for the triangular sums.
struct TileGrid {
  int G, mt, nt, per_xcd, S, nteams, rounds;
  static constexpr int SN = 8;
  __host__ __device__ static TileGrid make(int G, int M, int N, int TM, int TN) {
    TileGrid t;
    t.G = G;
    t.mt = (M + TM - 1) / TM;
    t.nt = (N + TN - 1) / TN;
    const int tiles = t.mt * t.nt;
    t.S = 1;
    while (t.S < 8 && tiles > 32 * t.S) t.S *= 2;
    t.nteams = 8 / t.S;
    t.per_xcd = (tiles + t.S - 1) / t.S;
    t.rounds = (G + t.nteams - 1) / t.nteams;
    return t;
  }
  __host__ __device__ int num_wg() const { return rounds * per_xcd * 8; }
  __device__ __forceinline__ bool decode(int wg, int& gorder, int& tm, int& tn) const {
    const int xcd = wg & 7, slot = wg >> 3;
    const int team = xcd / S, rank = xcd - team * S;
    const int round = slot / per_xcd;
    gorder = round * nteams + ((round & 1) ? nteams - 1 - team : team);
    if (gorder >= G) return false;
    const int t = rank * per_xcd + (slot - round * per_xcd);
    if (t >= mt * nt) return false;
    const int full = nt / SN, rem = nt - full * SN;
    const int tiles_full = full * mt * SN;
    if (t < tiles_full) {
      const int panel = t / (mt * SN), r = t - panel * mt * SN;
      tm = r / SN;
      tn = panel * SN + (r - tm * SN);
    } else {
      const int r = t - tiles_full;
      tm = r / rem;
      tn = full * SN + (r - tm * rem);
    }
    return true;
  }
};

// Where a 4-column group of the epilogue lands: row = ru + rl, col = cu + cl.  ru and cu are
// wave-uniform; rl and cl are the lane's fixed position inside its wave's block.  Element offsets
// are formed as a uniform 64-bit part (scalar registers) plus a 32-bit per-lane byte offset that
// is the same for every group of a tile, so the epilogue's memory accesses need no per-lane
// 64-bit arithmetic.
struct EpiPos {
  int ru, cu, rl, cl;
  float* lds = nullptr;   // bf16 kernel: 128 floats of LDS private to the wave, free for the policy during the epilogue
  __device__ __forceinline__ int row() const { return ru + rl; }
  __device__ __forceinline__ int col() const { return cu + cl; }
  // offsets of (row, col) in a row-major matrix with leading dimension ld that starts base_row rows in
  __device__ __forceinline__ size_t uoff(size_t base_row, int ld) const { return (base_row + ru) * (size_t)ld + cu; }
  __device__ __forceinline__ uint32_t loff(int ld) const { return (uint32_t)(rl * ld + cl); }
};
template <typename X>
__device__ __forceinline__ X* epi_ptr(X* base, size_t uoff, uint32_t loff) {
  typedef typename std::conditional<std::is_const<X>::value, const char, char>::type Byte;
  return reinterpret_cast<X*>(reinterpret_cast<Byte*>(base + uoff) + loff * (uint32_t)sizeof(X));
}

// Adam fused into a weight-gradient epilogue: the fp32 gradient of 4 consecutive
// parameters goes straight from the accumulators into the moments and the
// weights (App. C Table 1 update rule; same arithmetic as adam_kernel).
struct AdamFuse {
  float* m; float* v; float* master; AdamScalars a;   // m == nullptr: not fused
};
// Moments and the fp32 master parameter (when there is one) exactly as loaded; the stored weight
// travels beside them in its raw form.  Nothing is computed on any of them before adam_update4,
// so the loads stay in flight.
struct AdamRegs { float4 m, v, master; };
__device__ __forceinline__ void adam_load4(AdamRegs& r, const AdamFuse& f, size_t uo, uint32_t lo) {
  r.m = nt_load_f4(epi_ptr(f.m, uo, lo));
  r.v = nt_load_f4(epi_ptr(f.v, uo, lo));
  if (f.master) r.master = nt_load_f4(epi_ptr(f.master, uo, lo));
}
// Returns the four weights as stored (after rounding to T).
template <typename T>
__device__ __forceinline__ float4 adam_update4(const AdamFuse& f, T* w, size_t uo, uint32_t lo, const AdamRegs& r,
                                               typename Elem<T>::Raw4 w_raw, float4 g4) {
  const float4 m4 = r.m, v4 = r.v, p4 = f.master ? r.master : Elem<T>::widen4(w_raw);
  const float g[4] = {g4.x, g4.y, g4.z, g4.w};
  float mm[4] = {m4.x, m4.y, m4.z, m4.w}, vv[4] = {v4.x, v4.y, v4.z, v4.w}, pp[4] = {p4.x, p4.y, p4.z, p4.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) adam_element(pp[k], mm[k], vv[k], g[k], f.a);
  nt_store_f4(epi_ptr(f.m, uo, lo), make_float4(mm[0], mm[1], mm[2], mm[3]));
  nt_store_f4(epi_ptr(f.v, uo, lo), make_float4(vv[0], vv[1], vv[2], vv[3]));
  const float4 pn = make_float4(pp[0], pp[1], pp[2], pp[3]);
  if (f.master) nt_store_f4(epi_ptr(f.master, uo, lo), pn);
  const typename Elem<T>::Raw4 stored = Elem<T>::narrow4(pn);
  Elem<T>::nt_store_raw4(epi_ptr(w, uo, lo), stored);
  return Elem<T>::widen4(stored);
}

// ---------------------------------------------------------------------------
// Encoder: pre[l] = x[l] W_enc[l] + b_enc[l]  (eq. 1), JumpReLU epilogue.
// ---------------------------------------------------------------------------
template <typename T, typename TA = T>
struct EncPolicy {
  static constexpr bool XCD_SYNC = false;
  static constexpr bool A_KC = true, B_KC = false;
  typedef TA AType;
  Dims D;
  int M, N, kseg, lda, ldb;
  const TA* x; const T* W_enc; const float* b_enc; const float* theta; const float* x_scale;
  float half_eps; T* z; T* pre; uint8_t* cls; int32_t* l0;
  bool log_threshold;
  float* pre32;   // TopK activation: the epilogue only stores the fp32 pre-activation here (and pre); no z, classes, L0
  __device__ bool skip() const { return false; }
  struct GInfo { int l; };
  struct Epi { int count; float4 b, th; };
  __device__ GInfo ginfo(int order) const { return {order}; }
  __device__ int nseg(const GInfo&) const { return 1; }
  __device__ const TA* a_seg(const GInfo& g, int) const { return x + (size_t)g.l * D.B * D.d; }
  __device__ const T* b_seg(const GInfo& g, int) const { return W_enc + (size_t)g.l * D.d * D.F; }
  static constexpr int EPI_BATCH = 8, EPI_BATCH_LATE = 8, EPI_BATCH_LAST = 8;
  static constexpr bool PERSISTENT = true, UNIFORM_K = true;
  struct EpiRegs { float s; };
  __device__ void epi_begin(Epi& e, const GInfo& g, int col, bool ok, int row0) const {
    e.count = 0;
    e.b = e.th = make_float4(0.f, 0.f, 0.f, 0.f);
    if (ok) {
      const size_t vo = (size_t)g.l * D.F + col;
      e.b = *reinterpret_cast<const float4*>(b_enc + vo);
      if (!pre32) e.th = *reinterpret_cast<const float4*>(theta + vo);
      if (log_threshold) e.th = make_float4(expf(e.th.x), expf(e.th.y), expf(e.th.z), expf(e.th.w));
    }
  }
  __device__ void epi_load(EpiRegs& r, const GInfo& g, const EpiPos& pos) const {
    r.s = x_scale ? *epi_ptr(x_scale, (size_t)g.l * D.B + pos.ru, (uint32_t)pos.rl) : 1.0f;
  }
  __device__ void epi4(Epi& e, const GInfo& g, const EpiPos& pos, float4 v, const EpiRegs& r) const {
    const float4 b = e.b, th = e.th;
    if (x_scale) {   // int8 codes: the row scale multiplies the integer dot product
      const float s = r.s;
      v.x *= s; v.y *= s; v.z *= s; v.w *= s;
    }
    float p[4] = {v.x + b.x, v.y + b.y, v.z + b.z, v.w + b.w};
    if (pre32) {
      const size_t uo = pos.uoff((size_t)g.l * D.B, D.F);
      const uint32_t lo = pos.loff(D.F);
      *reinterpret_cast<float4*>(epi_ptr(pre32, uo, lo)) = make_float4(p[0], p[1], p[2], p[3]);
      if (pre) Elem<T>::store4(epi_ptr(pre, uo, lo), make_float4(p[0], p[1], p[2], p[3]));
      return;
    }
    const float t[4] = {th.x, th.y, th.z, th.w};
    float zz[4];
    uint32_t c4 = 0;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool act = p[i] > t[i];
      const bool win = fabsf(p[i] - t[i]) < half_eps;
      zz[i] = act ? p[i] : 0.0f;
      const uint32_t c = (act ? CLS_ACTIVE : 0u) | (win ? CLS_WINDOW : 0u) | (p[i] < t[i] ? CLS_BELOW : 0u);
      c4 |= c << (8 * i);
    }
    e.count += __popc(c4 & 0x01010101u);
    const size_t uo = pos.uoff((size_t)g.l * D.B, D.F);
    const uint32_t lo = pos.loff(D.F);
    Elem<T>::store4(epi_ptr(z, uo, lo), make_float4(zz[0], zz[1], zz[2], zz[3]));
    if (pre) Elem<T>::store4(epi_ptr(pre, uo, lo), make_float4(p[0], p[1], p[2], p[3]));
    *reinterpret_cast<uint32_t*>(epi_ptr(cls, uo, lo)) = c4;
  }
  __device__ void epi_end(Epi& e, const GInfo& g, float*) const {
    if (!l0) return;
    int c = e.count;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) c += __shfl_xor(c, off, 64);
    if ((threadIdx.x & 63) == 0 && c) atomicAdd(l0 + g.l, c);
  }
};

// ---------------------------------------------------------------------------
// Cross-layer decode (eq. 3): target lp, K runs over the sources l = 0..lp.
// ---------------------------------------------------------------------------
template <typename T>
struct DecPolicy {
  static constexpr bool XCD_SYNC = true;
  static constexpr bool A_KC = true, B_KC = false;
  typedef T AType;
  Dims D;
  int M, N, kseg, lda, ldb;
  const T* z; const T* W_dec; const float* b_dec; float* y_hat;
  const int32_t* skip_flags; int kcap;
  uint32_t* xcd_sync;   // 8 counters, 64 words apart, zero at launch (or NULL): see main_loop
  // the dense decode stands down when the device-side switch selected the gather path
  __device__ bool skip() const { return skip_flags && gather_selected(skip_flags, kcap); }
  struct GInfo { int lp; };
  struct Epi { float4 b; };
  __device__ GInfo ginfo(int order) const { return {D.L - 1 - order}; }   // longest K first
  __device__ int nseg(const GInfo& g) const { return g.lp + 1; }
  __device__ const T* a_seg(const GInfo&, int s) const { return z + (size_t)s * D.B * D.F; }
  __device__ const T* b_seg(const GInfo& g, int s) const {
    return W_dec + (size_t)packed_index(s, g.lp, D.L) * D.F * D.d;
  }
  static constexpr int EPI_BATCH = 8, EPI_BATCH_LATE = 8, EPI_BATCH_LAST = 8;
  static constexpr bool PERSISTENT = true, UNIFORM_K = false;
  struct EpiRegs {};
  __device__ void epi_begin(Epi& e, const GInfo& g, int col, bool ok, int row0) const {
    e.b = ok ? *reinterpret_cast<const float4*>(b_dec + (size_t)g.lp * D.d + col) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  __device__ void epi_load(EpiRegs&, const GInfo&, const EpiPos&) const {}
  __device__ void epi4(Epi& e, const GInfo& g, const EpiPos& pos, float4 v, const EpiRegs&) const {
    const float4 b = e.b;
    *reinterpret_cast<float4*>(epi_ptr(y_hat, pos.uoff((size_t)g.lp * D.B, D.d), pos.loff(D.d))) =
        make_float4(v.x + b.x, v.y + b.y, v.z + b.z, v.w + b.w);
  }
  __device__ void epi_end(Epi&, const GInfo&, float*) const {}
};

// ---------------------------------------------------------------------------
// dz[l] = sum_{lp>=l} dyhat[lp] W_dec[p(l,lp)]^T + sparsity gradient, kept
// where the feature is active or inside the threshold window (0 elsewhere).
// The sparsity gradient (lambda0 C / B) n sech^2(C z n) is evaluated as
// 4 e / (1 + e)^2 with e = exp(-2 |C z n|): no cancellation for large arguments
// and one hardware exponential per element.
// ---------------------------------------------------------------------------
// FOLD (bf16 kernel, dense mode): the epilogue also does what ste_reduce_kernel does after the plain
// variant -- it writes the final d pre (an inactive entry inside the threshold window only lends its dz
// to the threshold gradient; rows times the x scale for int8 inputs) and leaves, per 128-row half tile,
// the column sums of dz over the window (-> d theta), of d pre (-> d b_enc) and of the below-threshold
// count, summed in a fixed order: a lane over its 32 rows, then the 4 lanes that share its columns.
template <typename T, bool FOLD_ = false>
struct DzPolicy {
  static constexpr bool FOLD = FOLD_;
  static constexpr bool XCD_SYNC = false;
  static constexpr bool A_KC = true, B_KC = true;
  typedef T AType;
  Dims D;
  int M, N, kseg, lda, ldb;
  const T* d_yhat; const T* W_dec; const T* z; const uint8_t* cls; const float* norms;
  float lam_c_over_b, C; T* dpre;
  float lam1_over_b;
  const int32_t* skip_flags; int kcap;
  const float* x_scale; float* part_theta; float* part_benc; float* part_below;   // FOLD only
  // stands down when the device-side switch selected the sparse backward
  __device__ bool skip() const { return skip_flags && lists_backward_selected(skip_flags, kcap); }
  struct GInfo { int l; };
  // per column: -2 log2(e) C n, 4 (lambda0 C / B) n, -(lambda1 / B) n; FOLD: the three column sums and where they go
  struct Epi { float4 karg, kamp, dead; float4 st, sb, nb; int col, prow; bool ok; };
  __device__ GInfo ginfo(int order) const { return {order}; }             // K = (L-l) d, longest first
  __device__ int nseg(const GInfo& g) const { return D.L - g.l; }
  __device__ const T* a_seg(const GInfo& g, int s) const { return d_yhat + (size_t)(g.l + s) * D.B * D.d; }
  __device__ const T* b_seg(const GInfo& g, int s) const {
    return W_dec + (size_t)packed_index(g.l, g.l + s, D.L) * D.F * D.d;
  }
  static constexpr int EPI_BATCH = 8, EPI_BATCH_LATE = 8, EPI_BATCH_LAST = 8;
  static constexpr bool PERSISTENT = false, UNIFORM_K = false;   // measured: no faster as a tile loop (15.4 ms either way)
  struct EpiRegs { uint32_t c4; typename Elem<T>::Raw4 z4; float s; };
  __device__ void epi_begin(Epi& e, const GInfo& g, int col, bool ok, int row0) const {
    float4 n4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (ok) n4 = *reinterpret_cast<const float4*>(norms + (size_t)g.l * D.F + col);
    const float ka = -2.0f * 1.4426950408889634f * C, kb = 4.0f * lam_c_over_b, kd = 0.0f - lam1_over_b;
    e.karg = make_float4(ka * n4.x, ka * n4.y, ka * n4.z, ka * n4.w);
    e.kamp = make_float4(kb * n4.x, kb * n4.y, kb * n4.z, kb * n4.w);
    e.dead = make_float4(kd * n4.x, kd * n4.y, kd * n4.z, kd * n4.w);
    if (FOLD) {
      e.st = e.sb = e.nb = make_float4(0.f, 0.f, 0.f, 0.f);
      e.col = col;
      e.ok = ok;
      e.prow = row0 >> 7;     // the wave's 128-row half tile
    }
  }
  __device__ void epi_load(EpiRegs& r, const GInfo& g, const EpiPos& pos) const {
    const size_t uo = pos.uoff((size_t)g.l * D.B, D.F);
    const uint32_t lo = pos.loff(D.F);
    r.c4 = *reinterpret_cast<const uint32_t*>(epi_ptr(cls, uo, lo));
    r.z4 = Elem<T>::load_raw4(epi_ptr(z, uo, lo));
    if (FOLD) r.s = x_scale ? *epi_ptr(x_scale, (size_t)g.l * D.B + pos.ru, (uint32_t)pos.rl) : 1.0f;
  }
  __device__ void epi4(Epi& e, const GInfo& g, const EpiPos& pos, float4 v, const EpiRegs& r) const {
    const uint32_t c4 = r.c4;
    float4 out = make_float4(0.f, 0.f, 0.f, 0.f);
    const float dg[4] = {e.dead.x, e.dead.y, e.dead.z, e.dead.w};
    if (c4 & 0x03030303u) {          // some entry active or in the window: dz is kept there
      const float4 z4 = Elem<T>::widen4(r.z4);
      const float zz[4] = {z4.x, z4.y, z4.z, z4.w};
      const float vv[4] = {v.x, v.y, v.z, v.w};
      const float ka[4] = {e.karg.x, e.karg.y, e.karg.z, e.karg.w}, kb[4] = {e.kamp.x, e.kamp.y, e.kamp.z, e.kamp.w};
      float o[4], win[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float ex = __builtin_amdgcn_exp2f(ka[i] * fabsf(zz[i]));
        const float s = 1.0f + ex;
        const float gsp = kb[i] * ex * __builtin_amdgcn_rcpf(s * s);
        const uint32_t ci = (c4 >> (8 * i)) & 7u;
        const float dzv = vv[i] + gsp;
        // elsewhere only the dead-feature gradient of pre < theta
        const float below = (ci & CLS_BELOW) ? dg[i] + 0.0f : 0.0f;
        if (FOLD) {
          win[i] = (ci & CLS_WINDOW) ? dzv : 0.0f;
          o[i] = (ci & CLS_ACTIVE) ? dzv : below;
        } else {
          o[i] = (ci & 3u) ? dzv : below;
        }
      }
      out = make_float4(o[0], o[1], o[2], o[3]);
      if (FOLD) { e.st.x += win[0]; e.st.y += win[1]; e.st.z += win[2]; e.st.w += win[3]; }
    } else if (lam1_over_b != 0.f && c4) {
      out = make_float4((c4 & 0x4u) ? dg[0] : 0.f, (c4 & 0x400u) ? dg[1] : 0.f, (c4 & 0x40000u) ? dg[2] : 0.f,
                        (c4 & 0x4000000u) ? dg[3] : 0.f);
    }
    if (FOLD) {
      e.sb.x += out.x; e.sb.y += out.y; e.sb.z += out.z; e.sb.w += out.w;
      if (lam1_over_b != 0.f) {
        e.nb.x += (c4 & 0x4u) ? 1.f : 0.f; e.nb.y += (c4 & 0x400u) ? 1.f : 0.f;
        e.nb.z += (c4 & 0x40000u) ? 1.f : 0.f; e.nb.w += (c4 & 0x4000000u) ? 1.f : 0.f;
      }
      const float s = r.s;   // int8 inputs: the encoder-weight gradient contracts d pre with the integer codes
      out = make_float4(out.x * s, out.y * s, out.z * s, out.w * s);
    }
    Elem<T>::store4(epi_ptr(dpre, pos.uoff((size_t)g.l * D.B, D.F), pos.loff(D.F)), out);
  }
  __device__ void epi_end(Epi& e, const GInfo& g, float*) const {
    if (!FOLD) return;
    float* const dst[3] = {part_theta, part_benc, part_below};
    float4* const src[3] = {&e.st, &e.sb, &e.nb};
#pragma unroll
    for (int q = 0; q < 3; ++q) {
      if (q == 2 && lam1_over_b == 0.f) break;
      float a[4] = {src[q]->x, src[q]->y, src[q]->z, src[q]->w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {      // the 4 lanes that own these columns (lane / 16 = row inside a row group)
        a[i] += __shfl_xor(a[i], 16, 64);
        a[i] += __shfl_xor(a[i], 32, 64);
      }
      if (e.ok && (threadIdx.x & 48) == 0)
        *reinterpret_cast<float4*>(dst[q] + ((size_t)e.prow * D.L + g.l) * D.F + e.col) = make_float4(a[0], a[1], a[2], a[3]);
    }
  }
};

// ---------------------------------------------------------------------------
// dW_dec[p(l,lp)] = z[l]^T dyhat[lp] + (G[l,f] / n[l,f]) W_dec[p][f,:]
// ---------------------------------------------------------------------------
// ADAM: the update is fused into the epilogue (compile-time, so that the epilogue is one straight
// run of code and every wait counts exactly the loads that were issued).
// N2: the epilogue of the fused update also leaves the sums of squares of the updated weights (compile-time for
// the same reason as ADAM: one straight run of code).
template <typename T, bool ADAM, bool N2 = false>
struct DWdecPolicy {
  static constexpr bool XCD_SYNC = false;
  static constexpr bool A_KC = false, B_KC = false;
  typedef T AType;
  Dims D;
  int M, N, kseg, lda, ldb;
  const T* z; const T* d_yhat; T* W_dec; const float* G; const float* norms; T* dW_dec;   // dW_dec may be NULL when fused
  AdamFuse fuse;
  const int32_t* skip_flags; int kcap;
  int p0;   // first decoder block of this launch
  // optional (fused update, bf16 kernel, no edge tiles): sums of squares of the UPDATED weights over each run of
  // 64 columns of a row, [P][N / 64][F], from which the next step's decoder norms are formed without reading W_dec
  float* n2_part;
  __device__ bool skip() const { return skip_flags && lists_backward_selected(skip_flags, kcap); }
  struct GInfo { int p, l, lp; };
  struct Epi { int row0, run; };
  __device__ GInfo ginfo(int order) const {
    int l = 0, r = order + p0;
    while (r >= D.L - l) { r -= D.L - l; ++l; }
    return {order + p0, l, l + r};
  }
  __device__ int nseg(const GInfo&) const { return 1; }
  __device__ const T* a_seg(const GInfo& g, int) const { return z + (size_t)g.l * D.B * D.F; }
  __device__ const T* b_seg(const GInfo& g, int) const { return d_yhat + (size_t)g.lp * D.B * D.d; }
  // up to 16 registers per row group in flight: a short window while most accumulators are still live
  // (one group less with the sums of squares, whose registers come on top)
  static constexpr int EPI_BATCH = N2 ? 3 : 4, EPI_BATCH_LATE = N2 ? 6 : 8, EPI_BATCH_LAST = N2 ? 7 : 8;
  static constexpr bool PERSISTENT = true, UNIFORM_K = true;
  struct EpiRegs { float Gf, nf; typename Elem<T>::Raw4 w; AdamRegs ad; };
  __device__ void epi_begin(Epi& e, const GInfo&, int col, bool, int row0) const {
    e.row0 = row0;
    e.run = col >> 6;
  }
  __device__ void epi_load(EpiRegs& r, const GInfo& g, const EpiPos& pos) const {
    const size_t nf = (size_t)g.l * D.F + pos.ru;
    r.Gf = *epi_ptr(G, nf, (uint32_t)pos.rl);
    r.nf = *epi_ptr(norms, nf, (uint32_t)pos.rl);
    const size_t uo = pos.uoff((size_t)g.p * D.F, D.d);
    const uint32_t lo = pos.loff(D.d);
    r.w = Elem<T>::nt_load_raw4(epi_ptr(W_dec, uo, lo));
    if (ADAM) adam_load4(r.ad, fuse, uo, lo);
  }
  __device__ void epi4(Epi& e, const GInfo& g, const EpiPos& pos, float4 v, const EpiRegs& r) const {
    const float coef = r.Gf * __builtin_amdgcn_rcpf(fmaxf(r.nf, 1e-30f));
    const size_t uo = pos.uoff((size_t)g.p * D.F, D.d);
    const uint32_t lo = pos.loff(D.d);
    const float4 w = Elem<T>::widen4(r.w);
    const float4 gr = make_float4(fmaf(coef, w.x, v.x), fmaf(coef, w.y, v.y), fmaf(coef, w.z, v.z), fmaf(coef, w.w, v.w));
    if (!ADAM || dW_dec) Elem<T>::store4(epi_ptr(dW_dec, uo, lo), gr);
    if (ADAM) {
      const float4 wn = adam_update4<T>(fuse, W_dec, uo, lo, r.ad, r.w, gr);
      if (N2) {   // 16 lanes hold the 64 columns of one row of the wave's block
        const float s2 = row16_sum((wn.x * wn.x + wn.y * wn.y) + (wn.z * wn.z + wn.w * wn.w));
        // collected in the wave's LDS scratch (row inside the wave's 128-row block), written out once in epi_end
        if ((threadIdx.x & 15) == 0) pos.lds[(pos.ru - e.row0) + pos.rl] = s2;
      }
    }
  }
  __device__ void epi_end(Epi& e, const GInfo& g, float* lds) const {
    if (!ADAM || !N2) return;
    const int lane = threadIdx.x & 63;
    if (lane < 32) {    // the wave's 128 row sums, 512 contiguous bytes
      const float4 v = *reinterpret_cast<const float4*>(lds + 4 * lane);
      *reinterpret_cast<float4*>(n2_part + ((size_t)g.p * (N >> 6) + e.run) * (size_t)M + e.row0 + 4 * lane) = v;
    }
  }
};

// ---------------------------------------------------------------------------
// dW_enc[l] = x[l]^T dpre[l]
// ---------------------------------------------------------------------------
template <typename T, bool ADAM, typename TA = T>
struct DWencPolicy {
  static constexpr bool XCD_SYNC = false;
  static constexpr bool A_KC = false, B_KC = false;
  typedef TA AType;
  Dims D;
  int M, N, kseg, lda, ldb;
  const TA* x; const T* dpre; T* dW_enc;   // dW_enc may be NULL when fused
  T* W_enc; AdamFuse fuse;
  __device__ bool skip() const { return false; }
  struct GInfo { int l; };
  struct Epi {};
  __device__ GInfo ginfo(int order) const { return {order}; }
  __device__ int nseg(const GInfo&) const { return 1; }
  __device__ const TA* a_seg(const GInfo& g, int) const { return x + (size_t)g.l * D.B * D.d; }
  __device__ const T* b_seg(const GInfo& g, int) const { return dpre + (size_t)g.l * D.B * D.F; }
  static constexpr int EPI_BATCH = 4, EPI_BATCH_LATE = 8, EPI_BATCH_LAST = 8;
  static constexpr bool PERSISTENT = true, UNIFORM_K = true;
  struct EpiRegs { AdamRegs ad; typename Elem<T>::Raw4 w; };
  __device__ void epi_begin(Epi&, const GInfo&, int, bool, int) const {}
  __device__ void epi_load(EpiRegs& r, const GInfo& g, const EpiPos& pos) const {
    if (!ADAM) return;
    const size_t uo = pos.uoff((size_t)g.l * D.d, D.F);
    const uint32_t lo = pos.loff(D.F);
    adam_load4(r.ad, fuse, uo, lo);
    if (!fuse.master) r.w = Elem<T>::nt_load_raw4(epi_ptr(W_enc, uo, lo));
  }
  __device__ void epi4(Epi&, const GInfo& g, const EpiPos& pos, float4 v, const EpiRegs& r) const {
    const size_t uo = pos.uoff((size_t)g.l * D.d, D.F);
    const uint32_t lo = pos.loff(D.F);
    if (!ADAM || dW_enc) Elem<T>::store4(epi_ptr(dW_enc, uo, lo), v);
    if (ADAM) adam_update4<T>(fuse, W_enc, uo, lo, r.ad, r.w, v);
  }
  __device__ void epi_end(Epi&, const GInfo&, float*) const {}
};

}  // namespace clt
