// The five contractions of a CLT train step, each described as a "policy":
// operand addressing (which memory dimension is the contraction index K), the
// K segments of the triangular sums, and the fused epilogue.  The same policies
// drive the fp32 FMA kernel (gemm_f32.h) and the bf16 MFMA kernel
// (gemm_bf16.h).
//
// A policy exposes
//   A_KC / B_KC  true when the operand is contiguous along K in memory
//                (A element (m,k) at a[m*lda + k]; otherwise at a[k*lda + m];
//                 B element (k,n) at b[n*ldb + k] when B_KC, else b[k*ldb + n])
//   M, N, kseg   tile-space extents and the length of one K segment
//   ginfo(order) group visited at position `order` of the launch (longest K first)
//   nseg(gi), a_seg(gi,s), b_seg(gi,s)   K segments of a group
//   epi_load(regs, gi, row, col)  issues the global loads the epilogue of that 4-column
//                group needs (the kernels call it for a batch of groups first, so the
//                loads of the whole batch of EPI_BATCH groups are in flight together)
//   epi4(st, gi, row, col, v, regs)  consumes 4 accumulators of one row, columns col..col+3
#pragma once
#include "common.h"

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
  __device__ bool decode(int wg, int& gorder, int& tm, int& tn) const {
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

// Adam fused into a weight-gradient epilogue: the fp32 gradient of 4 consecutive
// parameters goes straight from the accumulators into the moments and the
// weights (App. C Table 1 update rule; same arithmetic as adam_kernel).
struct AdamFuse {
  float* m; float* v; float* master; AdamScalars a;   // m == nullptr: not fused
};
struct AdamRegs { float4 m, v, p; };   // moments and the fp32 parameter (master copy or widened weight)
template <typename T>
__device__ __forceinline__ void adam_load4(AdamRegs& r, const AdamFuse& f, const T* w, size_t o) {
  r.m = *reinterpret_cast<const float4*>(f.m + o);
  r.v = *reinterpret_cast<const float4*>(f.v + o);
  r.p = f.master ? *reinterpret_cast<const float4*>(f.master + o) : Elem<T>::load4(w + o);
}
template <typename T>
__device__ __forceinline__ void adam_update4(const AdamFuse& f, T* w, size_t o, const AdamRegs& r, float4 g4) {
  const float inv_bc1 = 1.0f / f.a.bc1, inv_bc2 = 1.0f / f.a.bc2;
  const float4 m4 = r.m, v4 = r.v, p4 = r.p;
  const float g[4] = {g4.x, g4.y, g4.z, g4.w};
  float mm[4] = {m4.x, m4.y, m4.z, m4.w}, vv[4] = {v4.x, v4.y, v4.z, v4.w}, pp[4] = {p4.x, p4.y, p4.z, p4.w};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    mm[k] = f.a.beta1 * mm[k] + (1.0f - f.a.beta1) * g[k];
    vv[k] = f.a.beta2 * vv[k] + (1.0f - f.a.beta2) * g[k] * g[k];
    pp[k] -= f.a.lr * (mm[k] * inv_bc1) / (sqrtf(vv[k] * inv_bc2) + f.a.eps);
  }
  *reinterpret_cast<float4*>(f.m + o) = make_float4(mm[0], mm[1], mm[2], mm[3]);
  *reinterpret_cast<float4*>(f.v + o) = make_float4(vv[0], vv[1], vv[2], vv[3]);
  const float4 pn = make_float4(pp[0], pp[1], pp[2], pp[3]);
  if (f.master) *reinterpret_cast<float4*>(f.master + o) = pn;
  Elem<T>::store4(w + o, pn);
}

__device__ __forceinline__ uint32_t pack_u8x4(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  return a | (b << 8) | (c << 16) | (d << 24);
}

// ---------------------------------------------------------------------------
// Encoder: pre[l] = x[l] W_enc[l] + b_enc[l]  (eq. 1), JumpReLU epilogue.
// ---------------------------------------------------------------------------
template <typename T, typename TA = T>
struct EncPolicy {
  static constexpr bool A_KC = true, B_KC = false;
  typedef TA AType;
  Dims D;
  int M, N, kseg, lda, ldb;
  const TA* x; const T* W_enc; const float* b_enc; const float* theta; const float* x_scale;
  float half_eps; T* z; T* pre; uint8_t* cls; int32_t* l0;
  bool log_threshold;
  __device__ bool skip() const { return false; }
  struct GInfo { int l; };
  struct Epi { int count; };
  __device__ GInfo ginfo(int order) const { return {order}; }
  __device__ int nseg(const GInfo&) const { return 1; }
  __device__ const TA* a_seg(const GInfo& g, int) const { return x + (size_t)g.l * D.B * D.d; }
  __device__ const T* b_seg(const GInfo& g, int) const { return W_enc + (size_t)g.l * D.d * D.F; }
  static constexpr int EPI_BATCH = 8, EPI_BATCH_LATE = 8;
  struct EpiRegs { float4 b, th; float s; };
  __device__ void epi_begin(Epi& e) const { e.count = 0; }
  __device__ void epi_load(EpiRegs& r, const GInfo& g, int row, int col) const {
    const size_t vo = (size_t)g.l * D.F + col;
    r.b = *reinterpret_cast<const float4*>(b_enc + vo);
    r.th = *reinterpret_cast<const float4*>(theta + vo);
    if (log_threshold) r.th = make_float4(expf(r.th.x), expf(r.th.y), expf(r.th.z), expf(r.th.w));
    r.s = x_scale ? x_scale[(size_t)g.l * D.B + row] : 1.0f;
  }
  __device__ void epi4(Epi& e, const GInfo& g, int row, int col, float4 v, const EpiRegs& r) const {
    const float4 b = r.b, th = r.th;
    if (x_scale) {   // int8 codes: the row scale multiplies the integer dot product
      const float s = r.s;
      v.x *= s; v.y *= s; v.z *= s; v.w *= s;
    }
    float p[4] = {v.x + b.x, v.y + b.y, v.z + b.z, v.w + b.w};
    const float t[4] = {th.x, th.y, th.z, th.w};
    float zz[4];
    uint32_t c[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const bool act = p[i] > t[i];
      const bool win = fabsf(p[i] - t[i]) < half_eps;
      zz[i] = act ? p[i] : 0.0f;
      c[i] = (act ? CLS_ACTIVE : 0) | (win ? CLS_WINDOW : 0) | (p[i] < t[i] ? CLS_BELOW : 0);
      e.count += act ? 1 : 0;
    }
    const size_t o = ((size_t)g.l * D.B + row) * D.F + col;
    Elem<T>::store4(z + o, make_float4(zz[0], zz[1], zz[2], zz[3]));
    if (pre) Elem<T>::store4(pre + o, make_float4(p[0], p[1], p[2], p[3]));
    *reinterpret_cast<uint32_t*>(cls + o) = pack_u8x4(c[0], c[1], c[2], c[3]);
  }
  __device__ void epi_end(Epi& e, const GInfo& g) const {
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
  static constexpr bool A_KC = true, B_KC = false;
  typedef T AType;
  Dims D;
  int M, N, kseg, lda, ldb;
  const T* z; const T* W_dec; const float* b_dec; float* y_hat;
  const int32_t* skip_flags; int kcap;
  // the dense decode stands down when the device-side switch selected the gather path
  __device__ bool skip() const { return skip_flags && skip_flags[0] != 0 && skip_flags[1] <= kcap; }
  struct GInfo { int lp; };
  struct Epi {};
  __device__ GInfo ginfo(int order) const { return {D.L - 1 - order}; }   // longest K first
  __device__ int nseg(const GInfo& g) const { return g.lp + 1; }
  __device__ const T* a_seg(const GInfo&, int s) const { return z + (size_t)s * D.B * D.F; }
  __device__ const T* b_seg(const GInfo& g, int s) const {
    return W_dec + (size_t)packed_index(s, g.lp, D.L) * D.F * D.d;
  }
  static constexpr int EPI_BATCH = 8, EPI_BATCH_LATE = 8;
  struct EpiRegs { float4 b; };
  __device__ void epi_begin(Epi&) const {}
  __device__ void epi_load(EpiRegs& r, const GInfo& g, int, int col) const {
    r.b = *reinterpret_cast<const float4*>(b_dec + (size_t)g.lp * D.d + col);
  }
  __device__ void epi4(Epi&, const GInfo& g, int row, int col, float4 v, const EpiRegs& r) const {
    const float4 b = r.b;
    *reinterpret_cast<float4*>(y_hat + ((size_t)g.lp * D.B + row) * D.d + col) =
        make_float4(v.x + b.x, v.y + b.y, v.z + b.z, v.w + b.w);
  }
  __device__ void epi_end(Epi&, const GInfo&) const {}
};

// ---------------------------------------------------------------------------
// dz[l] = sum_{lp>=l} dyhat[lp] W_dec[p(l,lp)]^T + sparsity gradient, kept
// where the feature is active or inside the threshold window (0 elsewhere).
// ---------------------------------------------------------------------------
template <typename T>
struct DzPolicy {
  static constexpr bool A_KC = true, B_KC = true;
  typedef T AType;
  Dims D;
  int M, N, kseg, lda, ldb;
  const T* d_yhat; const T* W_dec; const T* z; const uint8_t* cls; const float* norms;
  float lam_c_over_b, C; T* dpre;
  float lam1_over_b;
  __device__ bool skip() const { return false; }
  struct GInfo { int l; };
  struct Epi {};
  __device__ GInfo ginfo(int order) const { return {order}; }             // K = (L-l) d, longest first
  __device__ int nseg(const GInfo& g) const { return D.L - g.l; }
  __device__ const T* a_seg(const GInfo& g, int s) const { return d_yhat + (size_t)(g.l + s) * D.B * D.d; }
  __device__ const T* b_seg(const GInfo& g, int s) const {
    return W_dec + (size_t)packed_index(g.l, g.l + s, D.L) * D.F * D.d;
  }
  static constexpr int EPI_BATCH = 8, EPI_BATCH_LATE = 8;
  struct EpiRegs { uint32_t c4; float4 z4, n4; };
  __device__ void epi_begin(Epi&) const {}
  __device__ void epi_load(EpiRegs& r, const GInfo& g, int row, int col) const {
    const size_t o = ((size_t)g.l * D.B + row) * D.F + col;
    r.c4 = *reinterpret_cast<const uint32_t*>(cls + o);
    r.z4 = Elem<T>::load4(z + o);
    r.n4 = *reinterpret_cast<const float4*>(norms + (size_t)g.l * D.F + col);
  }
  __device__ void epi4(Epi&, const GInfo& g, int row, int col, float4 v, const EpiRegs& r) const {
    const size_t o = ((size_t)g.l * D.B + row) * D.F + col;
    const uint32_t c4 = r.c4;
    float4 out = make_float4(0.f, 0.f, 0.f, 0.f);
    const float4 n4 = r.n4;
    const float nn[4] = {n4.x, n4.y, n4.z, n4.w};
    if (c4 & 0x03030303u) {          // some entry active or in the window: dz is kept there
      const float4 z4 = r.z4;
      const float zz[4] = {z4.x, z4.y, z4.z, z4.w};
      const float vv[4] = {v.x, v.y, v.z, v.w};
      float r[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float t = tanhf(C * zz[i] * nn[i]);
        const float gsp = lam_c_over_b * nn[i] * (1.0f - t * t);
        const uint32_t ci = (c4 >> (8 * i)) & 7u;
        // elsewhere only the dead-feature gradient of pre < theta
        r[i] = (ci & 3u) ? vv[i] + gsp : ((ci & CLS_BELOW) ? 0.0f - lam1_over_b * nn[i] : 0.0f);
      }
      out = make_float4(r[0], r[1], r[2], r[3]);
    } else if (lam1_over_b != 0.f && c4) {
      out = make_float4((c4 & 0x4u) ? -lam1_over_b * nn[0] : 0.f, (c4 & 0x400u) ? -lam1_over_b * nn[1] : 0.f,
                        (c4 & 0x40000u) ? -lam1_over_b * nn[2] : 0.f, (c4 & 0x4000000u) ? -lam1_over_b * nn[3] : 0.f);
    }
    Elem<T>::store4(dpre + o, out);
  }
  __device__ void epi_end(Epi&, const GInfo&) const {}
};

// ---------------------------------------------------------------------------
// dW_dec[p(l,lp)] = z[l]^T dyhat[lp] + (G[l,f] / n[l,f]) W_dec[p][f,:]
// ---------------------------------------------------------------------------
template <typename T>
struct DWdecPolicy {
  static constexpr bool A_KC = false, B_KC = false;
  typedef T AType;
  Dims D;
  int M, N, kseg, lda, ldb;
  const T* z; const T* d_yhat; T* W_dec; const float* G; const float* norms; T* dW_dec;   // dW_dec may be NULL when fused
  AdamFuse fuse;
  int p0;   // first decoder block of this launch
  __device__ bool skip() const { return false; }
  struct GInfo { int p, l, lp; };
  struct Epi {};
  __device__ GInfo ginfo(int order) const {
    int l = 0, r = order + p0;
    while (r >= D.L - l) { r -= D.L - l; ++l; }
    return {order + p0, l, l + r};
  }
  __device__ int nseg(const GInfo&) const { return 1; }
  __device__ const T* a_seg(const GInfo& g, int) const { return z + (size_t)g.l * D.B * D.F; }
  __device__ const T* b_seg(const GInfo& g, int) const { return d_yhat + (size_t)g.lp * D.B * D.d; }
  // 18 registers per row group: 4 groups while most accumulators are still live, 8 afterwards
  static constexpr int EPI_BATCH = 4, EPI_BATCH_LATE = 8;
  struct EpiRegs { float Gf, nf; float4 w; AdamRegs ad; };
  __device__ void epi_begin(Epi&) const {}
  __device__ void epi_load(EpiRegs& r, const GInfo& g, int row, int col) const {
    const size_t nf = (size_t)g.l * D.F + row;
    r.Gf = G[nf];
    r.nf = norms[nf];
    const size_t o = ((size_t)g.p * D.F + row) * D.d + col;
    r.w = Elem<T>::load4(W_dec + o);
    if (fuse.m) adam_load4<T>(r.ad, fuse, W_dec, o);
  }
  __device__ void epi4(Epi&, const GInfo& g, int row, int col, float4 v, const EpiRegs& r) const {
    const float coef = r.Gf / fmaxf(r.nf, 1e-30f);
    const size_t o = ((size_t)g.p * D.F + row) * D.d + col;
    const float4 w = r.w;
    const float4 gr = make_float4(v.x + coef * w.x, v.y + coef * w.y, v.z + coef * w.z, v.w + coef * w.w);
    if (dW_dec) Elem<T>::store4(dW_dec + o, gr);
    if (fuse.m) adam_update4<T>(fuse, W_dec, o, r.ad, gr);
  }
  __device__ void epi_end(Epi&, const GInfo&) const {}
};

// ---------------------------------------------------------------------------
// dW_enc[l] = x[l]^T dpre[l]
// ---------------------------------------------------------------------------
template <typename T, typename TA = T>
struct DWencPolicy {
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
  static constexpr int EPI_BATCH = 4, EPI_BATCH_LATE = 8;
  struct EpiRegs { AdamRegs ad; };
  __device__ void epi_begin(Epi&) const {}
  __device__ void epi_load(EpiRegs& r, const GInfo& g, int row, int col) const {
    if (fuse.m) adam_load4<T>(r.ad, fuse, W_enc, ((size_t)g.l * D.d + row) * D.F + col);
  }
  __device__ void epi4(Epi&, const GInfo& g, int row, int col, float4 v, const EpiRegs& r) const {
    const size_t o = ((size_t)g.l * D.d + row) * D.F + col;
    if (dW_enc) Elem<T>::store4(dW_enc + o, v);
    if (fuse.m) adam_update4<T>(fuse, W_enc, o, r.ad, v);
  }
  __device__ void epi_end(Epi&, const GInfo&) const {}
};

}  // namespace clt
