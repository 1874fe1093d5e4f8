// Active-feature gather paths (paper Sec. 3.2 "Sparse Decode"): once training
// has pushed the activations into the sparse regime, each token looks up only
// the decoder rows of its active features, O(k d) instead of the dense O(F d)
// contraction.  The paper does this for the forward decode; the same lists also
// drive the two backward contractions through the decoder here.
//   decide    reads the per-layer active counts of the encoder epilogue and sets
//             the device-side switch (no host round trip);
//   compact   turns every (layer, token) row of z into an ordered list of
//             (feature, value) pairs, plus the inactive features inside the
//             threshold window (needed by the threshold gradient);
//   gather decode   one workgroup per (token, target layer): walks the sources
//             l <= l' and their lists, streams the 2d-byte decoder rows with
//             16-byte loads per lane and accumulates in fp32 registers;
//   gather dz       one workgroup per (layer, token): dot products of the listed
//             features' decoder rows with the token's d y_hat rows;
//   feature lists   transpose of the row lists: per (layer, feature) the tokens on
//             which it is active, built by a column scan in token order;
//   sparse dW_dec   one workgroup per (layer, feature, 8 targets): sums the few
//             d y_hat rows of the feature's tokens, adds the norm term and runs
//             the fused Adam update of the row.
// Every order of summation is fixed, so the results are bitwise reproducible
// (no floating-point atomics).  Decode and dz read B * k * P * d * sizeof(T)
// bytes of decoder rows (HBM/L2-bound); sparse dW_dec streams the optimizer
// state once, like a plain Adam pass, and reads its d y_hat rows out of the L2.
#include "common.h"

#include <cstdlib>

#include <type_traits>

namespace clt {
namespace {

__global__ void decode_decide_kernel(Dims D, const int32_t* __restrict__ l0, float thr, float thr_bwd, int forced,
                                     int rows_free, int32_t* __restrict__ flags) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  long long tot = 0;
  for (int l = 0; l < D.L; ++l) tot += l0[l];
  const double dens = (double)tot / ((double)D.L * D.B * D.F);
  flags[0] = ((forced || dens <= (double)thr) ? 1 : 0) | ((forced || dens <= (double)thr_bwd) ? 2 : 0) |
             (rows_free ? 4 : 0);
  flags[1] = 0;
  flags[2] = 1;
  flags[3] = 0;
}

// One wavefront per (layer, token) row; lanes take 16 consecutive features per pass (two 8-byte
// loads of class bytes: F is a multiple of 8, so a row start is 8-byte aligned), positions come
// from wave-wide exclusive scans of the per-lane counts: 8 passes and 16 scans for 8192 features.
// Active features fill the row's slots from the front, window-only features from the back.
// z is read only where a group of 4 features holds an active one.
__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int u = __shfl_up(v, off, 64);
    if (lane >= off) v += u;
  }
  return v;
}

template <typename T>
__global__ __launch_bounds__(256) void compact_active_kernel(Dims D, const T* __restrict__ z,
                                                             const uint8_t* __restrict__ cls, GatherLists g,
                                                             int32_t* __restrict__ flags) {
  // the row lists serve the gather decode, and the backward unless it works from the per-feature lists alone
  if (!((flags[0] & 1) || ((flags[0] & 2) && !(flags[0] & 4)))) return;
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);   // l * B + b
  if (row >= (long)D.L * D.B) return;
  const T* zr = z + (size_t)row * D.F;
  const uint8_t* cr = cls + (size_t)row * D.F;
  int32_t* oi = g.idx + (size_t)row * g.stride;
  float* ov = g.val + (size_t)row * g.stride;
  int base = 0, base_w = 0;
  for (int f0 = 0; f0 < D.F; f0 += 1024) {
    const int f = f0 + lane * 16;
    uint32_t c[4] = {0u, 0u, 0u, 0u};
    if (f < D.F) {
      const uint2 lo = *reinterpret_cast<const uint2*>(cr + f);
      c[0] = lo.x; c[1] = lo.y;
    }
    if (f + 8 < D.F) {
      const uint2 hi = *reinterpret_cast<const uint2*>(cr + f + 8);
      c[2] = hi.x; c[3] = hi.y;
    }
    uint32_t a[4], w[4];
    int n = 0, nw = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      a[j] = c[j] & 0x01010101u;                          // active
      w[j] = ((c[j] >> 1) & 0x01010101u) & ~a[j];         // in the window, not active
      n += __popc(a[j]);
      nw += __popc(w[j]);
    }
    const int incl = wave_incl_scan(n, lane), incl_w = wave_incl_scan(nw, lane);
    int pos = base + incl - n, pos_w = base_w + incl_w - nw;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if ((a[j] | w[j]) == 0u) continue;
      float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f);
      if (a[j]) z4 = Elem<T>::load4(zr + f + 4 * j);
      const float zz[4] = {z4.x, z4.y, z4.z, z4.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if ((a[j] >> (8 * i)) & 1u) {
          if (pos < g.kcap) { oi[pos] = f + 4 * j + i; ov[pos] = zz[i]; }
          ++pos;
        }
        if ((w[j] >> (8 * i)) & 1u) {
          if (pos_w < g.kcap) { oi[g.kcap - 1 - pos_w] = f + 4 * j + i; ov[g.kcap - 1 - pos_w] = 0.f; }
          ++pos_w;
        }
      }
    }
    base += __shfl(incl, 63, 64);
    base_w += __shfl(incl_w, 63, 64);
  }
  if (lane == 0) {
    g.counts[row] = base;
    g.counts_w[row] = base_w;
    // longest list so far; lists that collide make every gather kernel stand down.  The value only
    // grows, so a row that does not exceed what is already there (a stale read at worst costs an
    // atomic that changes nothing) leaves the one hot address alone.
    const int mine = base + base_w;
    if (mine > *reinterpret_cast<volatile const int32_t*>(flags + 1)) atomicMax(flags + 1, mine);
  }
}

// Address = wave-uniform base + the lane's fixed element offset (one 32-bit register per lane).
template <typename X>
__device__ __forceinline__ X* lane_ptr(X* uniform_base, uint32_t lane_elems) {   // base + lane offset, 32-bit lane part
  typedef typename std::conditional<std::is_const<X>::value, const char, char>::type Byte;
  return reinterpret_cast<X*>(reinterpret_cast<Byte*>(uniform_base) + lane_elems * (uint32_t)sizeof(X));
}

// 8 consecutive elements kept as loaded (16 bytes of bf16 or 32 bytes of fp32) until they are used
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> {
  typedef uint4 type;
  static __device__ __forceinline__ type load(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
  static __device__ __forceinline__ float dot(const type& a, const type& b, float acc) {
    const uint32_t x[4] = {a.x, a.y, a.z, a.w}, y[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      acc = fmaf(__uint_as_float(x[i] << 16), __uint_as_float(y[i] << 16), acc);
      acc = fmaf(__uint_as_float(x[i] & 0xffff0000u), __uint_as_float(y[i] & 0xffff0000u), acc);
    }
    return acc;
  }
};
template <> struct Raw8<float> {
  struct type { float4 lo, hi; };
  static __device__ __forceinline__ type load(const float* p) {
    return type{*reinterpret_cast<const float4*>(p), *reinterpret_cast<const float4*>(p + 4)};
  }
  static __device__ __forceinline__ float dot(const type& a, const type& b, float acc) {
    acc = fmaf(a.lo.x, b.lo.x, acc); acc = fmaf(a.lo.y, b.lo.y, acc); acc = fmaf(a.lo.z, b.lo.z, acc);
    acc = fmaf(a.lo.w, b.lo.w, acc); acc = fmaf(a.hi.x, b.hi.x, acc); acc = fmaf(a.hi.y, b.hi.y, acc);
    acc = fmaf(a.hi.z, b.hi.z, acc); acc = fmaf(a.hi.w, b.hi.w, acc);
    return acc;
  }
};

// One wavefront per (token, target, run of 256 columns): 4 columns per lane, the sources l <= l' and their lists in
// order.  Feature ids and values are wave-uniform, so a decoder row is a scalar base plus the lane's fixed column
// offset; eight rows are in flight for long lists, four for short ones.  The runs of a row are neighbours in the
// grid, and workgroups go round-robin to the XCDs: with d = 2048 an XCD always gets the same eighth of the columns,
// so the eight L2s hold disjoint parts of the decoder instead of eight copies of what is hot, and the long rows of
// a heavy-tailed batch are spread over eight CUs instead of going through one.
template <typename T, int U>
__device__ __forceinline__ void gather_rows(float (&acc)[4], const T* __restrict__ Wp, int ld, uint32_t col,
                                            const int32_t* __restrict__ ii, const float* __restrict__ vv, int j) {
  typename Elem<T>::Raw4 r[U];
  float v[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int f = __builtin_amdgcn_readfirstlane(ii[j + u]);
    v[u] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(vv[j + u])));
    r[u] = Elem<T>::load_raw4(lane_ptr(Wp + (size_t)f * ld, col));
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const float4 q = Elem<T>::widen4(r[u]);
    acc[0] = fmaf(v[u], q.x, acc[0]);
    acc[1] = fmaf(v[u], q.y, acc[1]);
    acc[2] = fmaf(v[u], q.z, acc[2]);
    acc[3] = fmaf(v[u], q.w, acc[3]);
  }
}

constexpr int GD_COLS = 256;      // columns per wavefront
template <typename T>
__global__ __launch_bounds__(64) void gather_decode_kernel(Dims D, GatherLists g, const T* __restrict__ W_dec,
                                                          const float* __restrict__ b_dec,
                                                          float* __restrict__ y_hat, int32_t* __restrict__ flags) {
  if (!gather_selected(flags, g.kcap)) return;
  const int ncs = (D.d + GD_COLS - 1) / GD_COLS;
  const int cs = (int)(blockIdx.x % ncs);
  const size_t bt = blockIdx.x / ncs;
  const int lp = D.L - 1 - (int)(bt / D.B);   // heaviest targets first
  const int b = (int)(bt % D.B);
  if (blockIdx.x == 0 && threadIdx.x == 0) flags[2] = 2;
  const int col = cs * GD_COLS + threadIdx.x * 4;
  if (col >= D.d) return;
  float acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) acc[i] = b_dec[(size_t)lp * D.d + col + i];
  for (int l = 0; l <= lp; ++l) {
    const size_t row = (size_t)l * D.B + b;
    const int cnt = g.counts[row];
    const int32_t* ii = g.idx + row * g.stride;
    const float* vv = g.val + row * g.stride;
    const T* Wp = W_dec + (size_t)packed_index(l, lp, D.L) * D.F * D.d;
    int j = 0;
    for (; j + 8 <= cnt; j += 8) gather_rows<T, 8>(acc, Wp, D.d, (uint32_t)col, ii, vv, j);
    if (j + 4 <= cnt) { gather_rows<T, 4>(acc, Wp, D.d, (uint32_t)col, ii, vv, j); j += 4; }
    for (; j < cnt; ++j) gather_rows<T, 1>(acc, Wp, D.d, (uint32_t)col, ii, vv, j);
  }
  *reinterpret_cast<float4*>(y_hat + ((size_t)lp * D.B + b) * D.d + col) = make_float4(acc[0], acc[1], acc[2], acc[3]);
}

// ---------------------------------------------------------------------------
// Sparse backward
// ---------------------------------------------------------------------------
template <typename T> struct Row8;      // 8 consecutive elements of a row as floats
template <> struct Row8<bf16_t> {
  static __device__ __forceinline__ void load(const bf16_t* p, float (&o)[8]) {
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) { o[2 * i] = __uint_as_float(w[i] << 16); o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u); }
  }
};
template <> struct Row8<float> {
  static __device__ __forceinline__ void load(const float* p, float (&o)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
  }
};

// dpre := 0 (or the dead-feature gradient below the threshold); the listed entries are overwritten by gather_dz.
template <typename T>
__global__ __launch_bounds__(256) void sparse_dpre_fill_kernel(Dims D, const uint8_t* __restrict__ cls,
                                                               const float* __restrict__ norms, float lam1_over_b,
                                                               T* __restrict__ dpre, const int32_t* __restrict__ flags,
                                                               int kcap) {
  if (!lists_backward_selected(flags, kcap)) return;
  const size_t n4 = (size_t)D.L * D.B * D.F / 4, per_layer4 = (size_t)D.B * D.F / 4;
  const int F4 = D.F / 4;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
    float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
    if (lam1_over_b != 0.f) {
      const uint32_t c4 = *reinterpret_cast<const uint32_t*>(cls + i * 4);
      if (c4 & 0x04040404u) {
        const int l = (int)(i / per_layer4), f = (int)(i % F4) * 4;
        const float4 n = *reinterpret_cast<const float4*>(norms + (size_t)l * D.F + f);
        o = make_float4((c4 & 0x4u) ? -lam1_over_b * n.x : 0.f, (c4 & 0x400u) ? -lam1_over_b * n.y : 0.f,
                        (c4 & 0x40000u) ? -lam1_over_b * n.z : 0.f, (c4 & 0x4000000u) ? -lam1_over_b * n.w : 0.f);
      }
    }
    Elem<T>::store4(dpre + i * 4, o);
  }
}

// One wavefront per listed entry: for each target l' >= l it streams the entry's decoder row and
// the token's d y_hat row (64 lanes x 8 columns, 4 passes in flight), keeps one partial dot
// product per lane and reduces over the wave at the end.  No workgroup barrier, few registers
// (93 registers with bf16 storage: five waves per SIMD), so many independent latency chains overlap.  A row's entries are dealt
// to GDZ_PARTS workgroups of 4 waves, so that the few very long rows of a heavy-tailed batch do
// not serialise on one workgroup.
constexpr int GDZ_PARTS = 8;
template <typename T>
__global__ __launch_bounds__(256) void gather_dz_kernel(Dims D, GatherLists g, const T* __restrict__ d_yhat,
                                                        const T* __restrict__ W_dec, const float* __restrict__ norms,
                                                        float lam_c_over_b, float C, T* __restrict__ dpre,
                                                        const int32_t* __restrict__ flags, FeatureLists fused) {
  if (!lists_backward_selected(flags, g.kcap) || fused_dz_selected(flags, fused)) return;
  const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long items = ((long)D.L * D.B + 7) / 8 * 8 * GDZ_PARTS;
  for (long it = blockIdx.x; it < items; it += gridDim.x) {      // layer 0 (most targets) first
    // items in groups of 8 rows x GDZ_PARTS parts, the row index fastest: workgroups go round-robin
    // to the 8 XCDs, so all parts of a row run on one XCD and share its L2
    const long grp = it / (8 * GDZ_PARTS);
    const int within = (int)(it % (8 * GDZ_PARTS));
    const long row = grp * 8 + (within & 7);
    const int part = within >> 3;
    if (row >= (long)D.L * D.B) continue;
    const int l = (int)(row / D.B), b = (int)(row % D.B);
    const int na = g.counts[row], n = na + g.counts_w[row];
    const int32_t* ii = g.idx + (size_t)row * g.stride;
    const float* vv = g.val + (size_t)row * g.stride;
    for (int e = part * 4 + wv; e < n; e += 4 * GDZ_PARTS) {
      const int slot = e < na ? e : g.kcap - 1 - (e - na);      // front: active entries, back: window-only
      const int fe = __builtin_amdgcn_readfirstlane(ii[slot]);
      float part_sum = 0.f;
      // the loads of two targets are in flight together
      auto targets = [&](auto nt_tag, int lp) {
        constexpr int NTG = decltype(nt_tag)::value;
        for (int c0 = 0; c0 < D.d; c0 += 2048) {
          typename Raw8<T>::type dy[NTG][4], wq[NTG][4];
#pragma unroll
          for (int t = 0; t < NTG; ++t) {
            const T* dyr = d_yhat + ((size_t)(lp + t) * D.B + b) * D.d;
            const T* wr = W_dec + ((size_t)packed_index(l, lp + t, D.L) * D.F + fe) * D.d;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const uint32_t col = (uint32_t)(c0 + q * 512 + lane * 8);
              if ((int)col < D.d) { dy[t][q] = Raw8<T>::load(lane_ptr(dyr, col)); wq[t][q] = Raw8<T>::load(lane_ptr(wr, col)); }
            }
          }
#pragma unroll
          for (int t = 0; t < NTG; ++t)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const uint32_t col = (uint32_t)(c0 + q * 512 + lane * 8);
              if ((int)col < D.d) part_sum = Raw8<T>::dot(wq[t][q], dy[t][q], part_sum);
            }
        }
      };
      int lp = l;
      for (; lp + 2 <= D.L; lp += 2) targets(std::integral_constant<int, 2>{}, lp);
      if (lp < D.L) targets(std::integral_constant<int, 1>{}, lp);
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) part_sum += __shfl_xor(part_sum, off, 64);
      if (lane == 0) {
        const float zv = vv[slot];
        const float nn = norms[(size_t)l * D.F + fe];
        const float ex = __builtin_amdgcn_exp2f(-2.0f * 1.4426950408889634f * C * nn * fabsf(zv));
        const float sden = 1.0f + ex;
        const float gsp = 4.0f * lam_c_over_b * nn * ex * __builtin_amdgcn_rcpf(sden * sden);
        Elem<T>::store(dpre + (size_t)row * D.F + fe, part_sum + gsp);
      }
    }
  }
}

// The same entries with the token's d y_hat rows staged in LDS: one workgroup of 16 waves per (layer, token) row,
// the rows of up to `tcap` targets (at most 64 KB) are copied to LDS once and every wave streams the decoder rows
// of its entries (four per batch of 64) against them, two targets' rows in flight.  Only decoder rows are left on the
// vector-memory path (d y_hat is fetched once per row instead of once per entry), and 64 registers allow eight waves
// per SIMD.  Launched with one workgroup per row, so long and short rows are balanced by the dispatcher; this is the
// kernel the library uses whenever a row of d y_hat fits LDS, gather_dz_kernel above is the fallback.
template <typename T> struct Raw8Lds;
template <> struct Raw8Lds<bf16_t> {
  static __device__ __forceinline__ Raw8<bf16_t>::type load(const bf16_t* p) { return *reinterpret_cast<const uint4*>(p); }
};
template <> struct Raw8Lds<float> {
  static __device__ __forceinline__ Raw8<float>::type load(const float* p) {
    return Raw8<float>::type{*reinterpret_cast<const float4*>(p), *reinterpret_cast<const float4*>(p + 4)};
  }
};
template <typename T>
__global__ __launch_bounds__(1024, 2) void gather_dz_lds_kernel(Dims D, GatherLists g, const T* __restrict__ d_yhat,
                                                                const T* __restrict__ W_dec,
                                                                const float* __restrict__ norms, float lam_c_over_b,
                                                                float C, T* __restrict__ dpre,
                                                                const int32_t* __restrict__ flags, int tcap,
                                                                FeatureLists fused) {
  extern __shared__ __align__(16) unsigned char gdz_smem[];
  T* dys = reinterpret_cast<T*>(gdz_smem);      // [tcap][d]
  if (!lists_backward_selected(flags, g.kcap) || fused_dz_selected(flags, fused)) return;
  const int tid = threadIdx.x, lane = tid & 63, wv = __builtin_amdgcn_readfirstlane(tid >> 6);
  constexpr int PIECE = 16 / (int)sizeof(T);      // elements per 16-byte piece
  const int ppr = D.d / PIECE;                    // pieces per row
  const long rows = (long)D.L * D.B;
  for (long row = blockIdx.x; row < rows; row += gridDim.x) {      // layer 0 (most targets) first
    const int l = (int)(row / D.B), b = (int)(row % D.B);
    const int na = g.counts[row], n = na + g.counts_w[row];
    const int32_t* ii = g.idx + (size_t)row * g.stride;
    const float* vv = g.val + (size_t)row * g.stride;
    for (int e0 = 0; e0 < n; e0 += 64) {
      float sum[4] = {0.f, 0.f, 0.f, 0.f};
      int slot[4], fe[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int e = e0 + u * 16 + wv;
        const int ec = e < n ? e : e0;                               // (a valid slot; nothing is computed or stored for it)
        slot[u] = ec < na ? ec : g.kcap - 1 - (ec - na);             // front: active entries, back: window-only
        fe[u] = __builtin_amdgcn_readfirstlane(ii[slot[u]]);
      }
      for (int lp0 = l; lp0 < D.L; lp0 += tcap) {
        const int tc = min(tcap, D.L - lp0);
        __syncthreads();                                             // the previous chunk's rows are no longer read
        for (int i = tid; i < tc * ppr; i += 1024) {
          const int t = i / ppr, c = (i - t * ppr) * PIECE;
          *reinterpret_cast<uint4*>(dys + (size_t)t * D.d + c) =
              *reinterpret_cast<const uint4*>(d_yhat + ((size_t)(lp0 + t) * D.B + b) * D.d + c);
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (e0 + u * 16 + wv >= n) continue;                       // wave-uniform
          float ps = sum[u];
          const T* wrow0 = W_dec + ((size_t)packed_index(l, lp0, D.L) * D.F + fe[u]) * D.d;
          const size_t blk = (size_t)D.F * D.d;
          for (int t = 0; t < tc; t += 2) {
            const bool two = t + 1 < tc;
            for (int c0 = 0; c0 < D.d; c0 += 2048) {
              typename Raw8<T>::type wq[2][4];
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const uint32_t col = (uint32_t)(c0 + q * 512 + lane * 8);
                if ((int)col < D.d) {
                  wq[0][q] = Raw8<T>::load(lane_ptr(wrow0 + (size_t)t * blk, col));
                  wq[1][q] = Raw8<T>::load(lane_ptr(wrow0 + (size_t)(two ? t + 1 : t) * blk, col));
                }
              }
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const uint32_t col = (uint32_t)(c0 + q * 512 + lane * 8);
                if ((int)col < D.d) {
                  ps = Raw8<T>::dot(wq[0][q], Raw8Lds<T>::load(dys + (size_t)t * D.d + col), ps);
                  if (two) ps = Raw8<T>::dot(wq[1][q], Raw8Lds<T>::load(dys + (size_t)(t + 1) * D.d + col), ps);
                }
              }
            }
          }
          sum[u] = ps;
        }
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        if (e0 + u * 16 + wv >= n) continue;
        float ps = sum[u];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) ps += __shfl_xor(ps, off, 64);
        if (lane == 0) {
          const float zv = vv[slot[u]];
          const float nn = norms[(size_t)l * D.F + fe[u]];
          const float ex = __builtin_amdgcn_exp2f(-2.0f * 1.4426950408889634f * C * nn * fabsf(zv));
          const float sden = 1.0f + ex;
          const float gsp = 4.0f * lam_c_over_b * nn * ex * __builtin_amdgcn_rcpf(sden * sden);
          Elem<T>::store(dpre + (size_t)row * D.F + fe[u], ps + gsp);
        }
      }
    }
  }
}

// ---- feature lists: column scan of the class bytes in FL_SEGS token segments ----
// Each thread owns 4 consecutive features of one layer and one token segment.
__global__ __launch_bounds__(256) void fl_count_kernel(Dims D, const uint8_t* __restrict__ cls, FeatureLists fl,
                                                       const int32_t* __restrict__ flags) {
  if (!lists_backward_selected(flags, fl.kcap)) return;
  const int LF4 = D.L * D.F / 4;
  const int q = blockIdx.x * 256 + threadIdx.x, sgm = blockIdx.y;
  if (q >= LF4) return;
  const int l = (q * 4) / D.F, f = (q * 4) % D.F;
  const int seg_len = (D.B + FL_SEGS - 1) / FL_SEGS;
  const int b0 = sgm * seg_len, b1 = min(D.B, b0 + seg_len);
  int c[4] = {0, 0, 0, 0};
#pragma unroll 8
  for (int b = b0; b < b1; ++b) {
    const uint32_t a4 = *reinterpret_cast<const uint32_t*>(cls + ((size_t)l * D.B + b) * D.F + f);
    const uint32_t listed = (a4 | (a4 >> 1)) & 0x01010101u;      // active, or inside the threshold window
#pragma unroll
    for (int i = 0; i < 4; ++i) c[i] += (int)((listed >> (8 * i)) & 1u);
  }
  int32_t* o = fl.seg + (size_t)sgm * D.L * D.F + (size_t)q * 4;
  o[0] = c[0]; o[1] = c[1]; o[2] = c[2]; o[3] = c[3];
}

// One workgroup of 1024 lanes per layer: layer-local exclusive scan over the features of the summed
// segment counts; the segment counts are turned into each segment's first slot.  A lane owns a
// run of consecutive features (8 at F = 8192, so neighbouring lanes share cache lines).
constexpr int FL_SCAN_THREADS = 1024;
__global__ __launch_bounds__(FL_SCAN_THREADS) void fl_scan_kernel(Dims D, FeatureLists fl,
                                                                  int32_t* __restrict__ flags, int dense_beyond) {
  if (!lists_backward_selected(flags, fl.kcap)) return;
  __shared__ int tot[FL_SCAN_THREADS];
  const int l = blockIdx.x, tid = threadIdx.x;
  const int per = (D.F + FL_SCAN_THREADS - 1) / FL_SCAN_THREADS;
  const int f0 = min(D.F, tid * per), f1 = min(D.F, f0 + per);
  const size_t LF = (size_t)D.L * D.F;
  int sum = 0;
  for (int f = f0; f < f1; ++f) {
    int c = 0;
    for (int sgm = 0; sgm < FL_SEGS; ++sgm) c += fl.seg[(size_t)sgm * LF + (size_t)l * D.F + f];
    sum += c;
  }
  tot[tid] = sum;
  __syncthreads();
  for (int off = 1; off < FL_SCAN_THREADS; off <<= 1) {   // inclusive scan of the lane totals
    const int v = tid >= off ? tot[tid - off] : 0;
    __syncthreads();
    tot[tid] += v;
    __syncthreads();
  }
  if (tid == FL_SCAN_THREADS - 1) {
    atomicMax(&flags[3], tot[tid]);      // the longest layer decides whether the fused dz has room
    // Automatic mode: lists too long for the fused dz are long enough for the dense kernels to win, so the backward
    // is handed back to them (they run after this kernel and look at the same bit; so do the list kernels).
    if (dense_beyond > 0 && tot[tid] > dense_beyond) atomicAnd(&flags[0], ~2);
  }
  int run = tot[tid] - sum;
  for (int f = f0; f < f1; ++f) {
    const size_t lf = (size_t)l * D.F + f;
    fl.off[lf] = run;
    int c = 0;
    for (int sgm = 0; sgm < FL_SEGS; ++sgm) {
      const int v = fl.seg[(size_t)sgm * LF + lf];
      fl.seg[(size_t)sgm * LF + lf] = run + c;
      c += v;
    }
    fl.cnt[lf] = c;
    run += c;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void fl_fill_kernel(Dims D, const uint8_t* __restrict__ cls, const T* __restrict__ z,
                                                      FeatureLists fl, const int32_t* __restrict__ flags) {
  if (!lists_backward_selected(flags, fl.kcap)) return;
  const int LF4 = D.L * D.F / 4;
  const int q = blockIdx.x * 256 + threadIdx.x, sgm = blockIdx.y;
  if (q >= LF4) return;
  const int l = (q * 4) / D.F, f = (q * 4) % D.F;
  const int seg_len = (D.B + FL_SEGS - 1) / FL_SEGS;
  const int b0 = sgm * seg_len, b1 = min(D.B, b0 + seg_len);
  const int32_t* so = fl.seg + (size_t)sgm * D.L * D.F + (size_t)q * 4;
  int pos[4] = {so[0], so[1], so[2], so[3]};
  const size_t base = (size_t)l * D.B * fl.kcap;        // layer l's region of the lists
  for (int bb = b0; bb < b1; bb += 8) {      // the class words of eight tokens in flight, then the (few) listed entries
    uint32_t c8[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      c8[u] = bb + u < b1 ? *reinterpret_cast<const uint32_t*>(cls + ((size_t)l * D.B + bb + u) * D.F + f) : 0u;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const uint32_t a4 = (c8[u] | (c8[u] >> 1)) & 0x01010101u;      // as counted: active or in the window (z = 0 there)
      if (!a4) continue;
      const int b = bb + u;
      const float4 z4 = Elem<T>::load4(z + ((size_t)l * D.B + b) * D.F + f);
      const float zz[4] = {z4.x, z4.y, z4.z, z4.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if ((a4 >> (8 * i)) & 1u) {
          fl.tok[base + pos[i]] = b;
          fl.val[base + pos[i]] = zz[i];
          ++pos[i];
        }
    }
  }
}

// One item = (layer l, feature f, pair of targets): a workgroup of 256 lanes, 8 columns each,
// requests the rows' weights and optimizer state, sums z * d y_hat rows over the feature's tokens (four tokens in
// flight) meanwhile, then finishes the row of both targets: norm term, optional gradient store, optional Adam update.  Most rows of a
// sparse step have no token at all and only stream their optimizer state.  Token indices and
// values are wave-uniform, so every address is a scalar base plus the lane's fixed column offset.
constexpr int SD_TCH = 2;

template <typename T, int NT, bool MASTER>
__device__ __forceinline__ void sparse_dwdec_rows(const Dims& D, int l, int f, int lp0, int cnt,
                                                  const int32_t* __restrict__ tk, const float* __restrict__ tv,
                                                  float coef, const T* __restrict__ d_yhat, T* __restrict__ W_dec,
                                                  T* __restrict__ dW_dec, const AdamFuseArgs& fuse, uint32_t col,
                                                  bool ok1, float* __restrict__ n2_part, int n2_slots, int n2_slot0) {
  // the lane owns columns col..col+3 and, when ok1, col+1024..col+1027: every access of the
  // workgroup is one contiguous run of 256 x 4 elements.
  // The rows' weights and optimizer state are requested first: they come from HBM and do not depend on the
  // token lists, so their latency lies under the gathering of the d y_hat rows below.
  // (native vector types: selects on the float4 class type would go through scratch memory)
  typename Elem<T>::Raw4 wr[NT][2];
  nt_f32x4 m4[NT][2], v4[NT][2], p4[NT][2];
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const size_t o = ((size_t)packed_index(l, lp0 + t, D.L) * D.F + f) * D.d;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      m4[t][h] = v4[t][h] = p4[t][h] = nt_f32x4{0.f, 0.f, 0.f, 0.f};
      wr[t][h] = Elem<T>::narrow4(make_float4(0.f, 0.f, 0.f, 0.f));
      if (h == 1 && !ok1) continue;
      const uint32_t ch = col + 1024 * h;
      wr[t][h] = Elem<T>::load_raw4(lane_ptr(W_dec + o, ch));
      if (fuse.m) {
        m4[t][h] = *reinterpret_cast<const nt_f32x4*>(lane_ptr(fuse.m + o, ch));
        v4[t][h] = *reinterpret_cast<const nt_f32x4*>(lane_ptr(fuse.v + o, ch));
        if (MASTER) p4[t][h] = *reinterpret_cast<const nt_f32x4*>(lane_ptr(fuse.master + o, ch));
      }
    }
  }
  float acc[NT][2][4];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int k = 0; k < 4; ++k) acc[t][h][k] = 0.f;
  int j = 0;
  for (; j + 4 <= cnt; j += 4) {
    // (the gathered rows stay in their storage type until they are used: half the registers for bf16)
    typename Elem<T>::Raw4 r[4][NT][2];
    float zv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int b = __builtin_amdgcn_readfirstlane(tk[j + u]);
      zv[u] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(tv[j + u])));
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const T* row = d_yhat + ((size_t)(lp0 + t) * D.B + b) * D.d;
        r[u][t][0] = Elem<T>::load_raw4(lane_ptr(row, col));
        r[u][t][1] = Elem<T>::load_raw4(lane_ptr(row, ok1 ? col + 1024 : col));
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const float4 q = Elem<T>::widen4(r[u][t][h]);
          acc[t][h][0] = fmaf(zv[u], q.x, acc[t][h][0]);
          acc[t][h][1] = fmaf(zv[u], q.y, acc[t][h][1]);
          acc[t][h][2] = fmaf(zv[u], q.z, acc[t][h][2]);
          acc[t][h][3] = fmaf(zv[u], q.w, acc[t][h][3]);
        }
  }
  for (; j < cnt; ++j) {
    const int b = __builtin_amdgcn_readfirstlane(tk[j]);
    const float zv = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(tv[j])));
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const T* row = d_yhat + ((size_t)(lp0 + t) * D.B + b) * D.d;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        if (h == 1 && !ok1) continue;
        const float4 r = Elem<T>::load4(lane_ptr(row, col + 1024 * h));
        acc[t][h][0] = fmaf(zv, r.x, acc[t][h][0]);
        acc[t][h][1] = fmaf(zv, r.y, acc[t][h][1]);
        acc[t][h][2] = fmaf(zv, r.z, acc[t][h][2]);
        acc[t][h][3] = fmaf(zv, r.w, acc[t][h][3]);
      }
    }
  }
  nt_f32x4 w[NT][2];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const float4 wl = Elem<T>::widen4(wr[t][h]);
      w[t][h] = nt_f32x4{wl.x, wl.y, wl.z, wl.w};
      if (!MASTER) p4[t][h] = w[t][h];
    }
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    const size_t o = ((size_t)packed_index(l, lp0 + t, D.L) * D.F + f) * D.d;
    float n2_half[2] = {0.f, 0.f};
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      if (h == 1 && !ok1) continue;
      const uint32_t ch = col + 1024 * h;
      const nt_f32x4 wq = w[t][h];
      const float g4[4] = {fmaf(coef, wq[0], acc[t][h][0]), fmaf(coef, wq[1], acc[t][h][1]),
                           fmaf(coef, wq[2], acc[t][h][2]), fmaf(coef, wq[3], acc[t][h][3])};
      if (dW_dec) Elem<T>::store4(lane_ptr(dW_dec + o, ch), make_float4(g4[0], g4[1], g4[2], g4[3]));
      if (fuse.m) {
        float mm[4] = {m4[t][h][0], m4[t][h][1], m4[t][h][2], m4[t][h][3]};
        float vv[4] = {v4[t][h][0], v4[t][h][1], v4[t][h][2], v4[t][h][3]};
        float pp[4] = {p4[t][h][0], p4[t][h][1], p4[t][h][2], p4[t][h][3]};
#pragma unroll
        for (int k = 0; k < 4; ++k) adam_element(pp[k], mm[k], vv[k], g4[k], fuse.a);
        *reinterpret_cast<float4*>(lane_ptr(fuse.m + o, ch)) = make_float4(mm[0], mm[1], mm[2], mm[3]);
        *reinterpret_cast<float4*>(lane_ptr(fuse.v + o, ch)) = make_float4(vv[0], vv[1], vv[2], vv[3]);
        const float4 pn = make_float4(pp[0], pp[1], pp[2], pp[3]);
        if (MASTER) *reinterpret_cast<float4*>(lane_ptr(fuse.master + o, ch)) = pn;
        const typename Elem<T>::Raw4 stored = Elem<T>::narrow4(pn);
        *reinterpret_cast<typename Elem<T>::Raw4*>(lane_ptr(W_dec + o, ch)) = stored;
        if (n2_part) {   // sum of squares of the wave's 256 weights as stored, for the next step's norms: one slot per wave and half
          const float4 wn = Elem<T>::widen4(stored);
          const int b16 = __float_as_int(row16_sum((wn.x * wn.x + wn.y * wn.y) + (wn.z * wn.z + wn.w * wn.w)));
          n2_half[h] = (__int_as_float(__builtin_amdgcn_readlane(b16, 0)) + __int_as_float(__builtin_amdgcn_readlane(b16, 16))) +
                       (__int_as_float(__builtin_amdgcn_readlane(b16, 32)) + __int_as_float(__builtin_amdgcn_readlane(b16, 48)));
        }
      }
    }
    if (n2_part && fuse.m && (threadIdx.x & 63) == 0)     // both halves of the wave's slot pair at once
      *reinterpret_cast<float2*>(n2_part + ((size_t)packed_index(l, lp0 + t, D.L) * D.F + f) * n2_slots + n2_slot0) =
          make_float2(n2_half[0], n2_half[1]);
  }
}

// MASTER: fp32 master weights travel with the moments (compile-time: their 16 registers are not held otherwise)
template <typename T, bool MASTER>
__global__ __launch_bounds__(256, 4) void sparse_dwdec_kernel(Dims D, FeatureLists fl, const T* __restrict__ d_yhat,
                                                           T* __restrict__ W_dec, const float* __restrict__ G,
                                                           const float* __restrict__ norms, T* __restrict__ dW_dec,
                                                           AdamFuseArgs fuse, const int32_t* __restrict__ flags,
                                                           float* __restrict__ n2_part) {
  if (!lists_backward_selected(flags, fl.kcap)) return;
  const int tid = threadIdx.x;
  const int chunks = (D.L + SD_TCH - 1) / SD_TCH;          // chunk slots per (l, f); those past L - l are empty
  const long items = (long)D.L * D.F * chunks;
  // what an item needs before its rows can be touched; fetched one item ahead
  struct Meta { int l, f, lp0, cnt, off; float Gf, nf; };
  auto fetch_meta = [&](long it) {
    Meta mt;
    // order (l, target pair, f): the workgroups in flight walk a few long contiguous row ranges
    mt.f = (int)(it % D.F);
    const long lc = it / D.F;
    const int c = (int)(lc % chunks);
    mt.l = (int)(lc / chunks);
    const long lf = (long)mt.l * D.F + mt.f;
    mt.lp0 = mt.l + c * SD_TCH;
    mt.cnt = 0; mt.off = 0; mt.Gf = 0.f; mt.nf = 1.f;
    if (mt.lp0 < D.L) { mt.cnt = fl.cnt[lf]; mt.off = fl.off[lf]; mt.Gf = G[lf]; mt.nf = norms[lf]; }
    return mt;
  };
  long it = blockIdx.x;
  if (it >= items) return;
  Meta cur = fetch_meta(it);
  for (; it < items; it += gridDim.x) {
    const long nx = it + gridDim.x;
    Meta nxt = cur;
    if (nx < items) nxt = fetch_meta(nx);
    if (cur.lp0 < D.L) {
      const int32_t* tk = fl.tok + (size_t)cur.l * D.B * fl.kcap + cur.off;
      const float* tv = fl.val + (size_t)cur.l * D.B * fl.kcap + cur.off;
      const float coef = cur.Gf * __builtin_amdgcn_rcpf(fmaxf(cur.nf, 1e-30f));
      // row sums of squares of the updated weights (n2_part, d a multiple of 256): [P][F][8 slots per 2048 columns],
      // slot = (wave, half) of the lanes that own the columns; slots whose columns do not exist hold zero
      const int n2_slots = 8 * ((D.d + 2047) / 2048);
      for (int c0 = 0; c0 < D.d; c0 += 2048) {
        const int col = c0 + tid * 4;
        const bool ok1 = col + 1024 < D.d;
        const int slot0 = (c0 >> 11) * 8 + (tid >> 6) * 2;
        if (n2_part && (tid & 63) == 0) {
          const int nt = cur.lp0 + 1 < D.L ? 2 : 1;
          for (int t = 0; t < nt; ++t) {
            float* q = n2_part + ((size_t)packed_index(cur.l, cur.lp0 + t, D.L) * D.F + cur.f) * n2_slots + slot0;
            if (col >= D.d) { q[0] = 0.f; q[1] = 0.f; }
          }
        }
        if (col >= D.d) continue;
        if (cur.lp0 + 1 < D.L)
          sparse_dwdec_rows<T, 2, MASTER>(D, cur.l, cur.f, cur.lp0, cur.cnt, tk, tv, coef, d_yhat, W_dec, dW_dec, fuse,
                                  (uint32_t)col, ok1, n2_part, n2_slots, slot0);
        else
          sparse_dwdec_rows<T, 1, MASTER>(D, cur.l, cur.f, cur.lp0, cur.cnt, tk, tv, coef, d_yhat, W_dec, dW_dec, fuse,
                                  (uint32_t)col, ok1, n2_part, n2_slots, slot0);
      }
    }
    cur = nxt;
  }
}

// Sums of four values over the wave at once: on return the lanes with lane % 4 == u hold the sum of the u-th value.
// Two exchange steps inside quads halve the values each lane carries, two rotations finish the rows of 16 lanes,
// two shuffles the four rows.
__device__ __forceinline__ float wave_sum4(float a, float b, float c, float d, int lane, int addr16, int addr32) {
  const bool o1 = lane & 1, o2 = lane & 2;
  const float r1 = (o1 ? b : a) + dpp_move<0xB1>(o1 ? a : b);      // even lanes: a of the pair, odd lanes: b
  const float r2 = (o1 ? d : c) + dpp_move<0xB1>(o1 ? c : d);
  float r = (o2 ? r2 : r1) + dpp_move<0x4E>(o2 ? r1 : r2);         // lane % 4 = 0, 1, 2, 3: a, b, c, d of the quad
  r += dpp_move<0x128>(r);                                          // row_ror:8
  r += dpp_move<0x124>(r);                                          // row_ror:4
  // (addr16 / addr32: byte addresses of lanes lane ^ 16 and lane ^ 32, computed once by the caller)
  r += __int_as_float(__builtin_amdgcn_ds_bpermute(addr16, __float_as_int(r)));
  r += __int_as_float(__builtin_amdgcn_ds_bpermute(addr32, __float_as_int(r)));
  return r;
}

// bf16 pairs as the dot-product instruction takes them
typedef __bf16 bf16x2_hw __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_hw, a), __builtin_bit_cast(bf16x2_hw, b), c, false);
}

// The same rows cut into eight column slices, one per XCD (workgroups go round-robin to the XCDs, so blockIdx & 7
// names the slice): an XCD's L2 then only ever sees its d/8 columns of d y_hat, and with the (source, target) pairs
// walked target-major that is B * d/8 elements at a time (2 MB at L=16 d=2048 B=4096), so the gathered d y_hat rows
// come out of the L2.  One wave per (pair, feature, slice), four consecutive features per workgroup, lanes own 4
// columns per pass of 256; 44-48 registers with bf16 storage, eight waves per SIMD.  The weights and optimizer state,
// touched once, are streamed with non-temporal accesses so that they do not displace the slice (plain accesses: 10 %
// slower).  The sums run over the feature's tokens in list order; with fp32 storage exactly as in the kernel above
// (same gradient and update, bit for bit).  At more than a few tokens per feature the kernel is bound by vector
// instruction issue, hence the bf16 token loop below.  This is the kernel the library uses whenever d is a
// multiple of 32.
#ifndef SD_ITEMS_PER_WG
#define SD_ITEMS_PER_WG 2
#endif
template <typename T, bool MASTER>
__global__ __launch_bounds__(256, sizeof(T) == 2 ? 8 : 6) void sparse_dwdec_sliced_kernel(Dims D, FeatureLists fl, const T* __restrict__ d_yhat,
                                                                     T* __restrict__ W_dec, const float* __restrict__ G,
                                                                     const float* __restrict__ norms, T* __restrict__ dW_dec,
                                                                     AdamFuseArgs fuse, const int32_t* __restrict__ flags,
                                                                     float* __restrict__ n2_part,
                                                                     const int32_t* __restrict__ fl_tok,
                                                                     const float* __restrict__ fl_val) {
  // (fl_tok, fl_val: fl.tok and fl.val once more, as parameters of their own that nothing else aliases: the wave-uniform
  //  reads of the token lists can then go through the scalar unit)
  if (!lists_backward_selected(flags, fl.kcap)) return;
  const int lane = threadIdx.x & 63, wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int addr16 = (lane ^ 16) << 2, addr32 = (lane ^ 32) << 2;
  const int slice = blockIdx.x & 7, wg = blockIdx.x >> 3, nwg = gridDim.x >> 3;      // (the grid is a multiple of 8)
  const int sw = D.d / 8, q4 = sw / 4;                     // slice width in columns and in lane quads (d % 32 == 0)
  const int passes = (q4 + 63) / 64;
  const int F4 = (D.F + 3) / 4;
  const long items = (long)(D.L * (D.L + 1) / 2) * F4;
  const bool dz_on = fused_dz_selected(flags, fl);
  struct Meta { int l, lp, f, cnt, off; float Gf, nf; };
  // (SD_ITEMS_PER_WG consecutive items per workgroup as long as the grid allows it: handed out in order by the
  //  dispatcher, the workgroups in flight stay within a narrow window of items, which is what keeps their d y_hat rows
  //  in the L2; more than one item, so that a launch that stands down costs fewer empty workgroups)
  for (long itb = (long)wg * SD_ITEMS_PER_WG; itb < items; itb += (long)nwg * SD_ITEMS_PER_WG)
  for (long it = itb; it < itb + SD_ITEMS_PER_WG && it < items; ++it) {
    Meta cur;
    const int pq = (int)(it / F4);                         // pair ordinal, target-major: (0,0) (0,1) (1,1) (0,2) ...
    cur.f = (int)(it % F4) * 4 + wv;
    int lpq = (int)((__builtin_amdgcn_sqrtf(8.0f * (float)pq + 1.0f) - 1.0f) * 0.5f);
    while ((lpq + 1) * (lpq + 2) / 2 <= pq) ++lpq;
    while (lpq * (lpq + 1) / 2 > pq) --lpq;
    cur.lp = lpq;
    cur.l = pq - lpq * (lpq + 1) / 2;
    if (cur.f < D.F) {
      const long lf = (long)cur.l * D.F + cur.f;
      cur.cnt = fl.cnt[lf]; cur.off = fl.off[lf]; cur.Gf = G[lf]; cur.nf = norms[lf];
      const int32_t* tk = fl_tok + (size_t)cur.l * D.B * fl.kcap + cur.off;
      const float* tv = fl_val + (size_t)cur.l * D.B * fl.kcap + cur.off;
      const float coef = cur.Gf * __builtin_amdgcn_rcpf(fmaxf(cur.nf, 1e-30f));
      const size_t o = ((size_t)packed_index(cur.l, cur.lp, D.L) * D.F + cur.f) * D.d;
      const T* dyt = d_yhat + (size_t)cur.lp * D.B * D.d;
      float* dz_out = dz_on ? fl.dz_part + ((size_t)packed_index(cur.l, cur.lp, D.L) * 8 + slice) * fl.ecap + cur.off : nullptr;
      for (int ps = 0; ps < passes; ++ps) {
        const int qd = ps * 64 + lane;
        const bool on = qd < q4;
        const uint32_t col = (uint32_t)(slice * sw + (on ? qd : 0) * 4);      // (idle lanes shadow quad 0, store nothing)
        typename Elem<T>::Raw4 wr;
        nt_f32x4 m4 = {0.f, 0.f, 0.f, 0.f}, v4 = m4, p4 = m4;
        wr = Elem<T>::nt_load_raw4(lane_ptr(W_dec + o, col));
        if (fuse.m) {
          m4 = nt_load_v4(lane_ptr(fuse.m + o, col));
          v4 = nt_load_v4(lane_ptr(fuse.v + o, col));
          if (MASTER) p4 = nt_load_v4(lane_ptr(fuse.master + o, col));
        }
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        // Fused dz: the token's d y_hat columns are in registers anyway, so their dot product with the row's weights
        // (before the update) costs four multiply-adds per lane and, for four tokens at a time, one sum over the
        // wave; lane t % 64 keeps token t's sum and the wave stores 64 of them at a time, one slot per
        // (pair, slice, entry).
        float dz_keep = 0.f;
        const float4 wl = Elem<T>::widen4(wr);
        auto dz_group = [&](int j0, int nval, const float (&pd)[4]) {      // tokens j0 .. j0 + nval - 1, j0 % 4 == 0
          const float r = wave_sum4(pd[0], pd[1], pd[2], pd[3], lane, addr16, addr32);
          if ((lane & 60) == (j0 & 63)) dz_keep = r;
          const int last = j0 + nval - 1;
          if ((last & 63) == 63 || last == cur.cnt - 1) {
            if (lane <= (last & 63)) {
              float* slot = dz_out + (last & ~63) + lane;
              *slot = ps == 0 ? dz_keep : *slot + dz_keep;      // (a slice wider than 256 columns: one pass after the other)
            }
          }
        };
        if constexpr (sizeof(T) == 2) {
          // bf16 storage.  The rows come through buffer loads (descriptor of the target's d y_hat, the lane's column
          // offset in a register, the token's row offset as the scalar operand: no vector arithmetic per token) and
          // stay packed: z * row enters the gradient two tokens at a time as a packed dot product (the two tokens'
          // values of a column brought into one register by a byte permute, (z_a, z_b) as the scalar operand; z is a
          // bf16 value, so nothing is rounded), the dz product two columns at a time.
          const __amdgpu_buffer_rsrc_t rows = __builtin_amdgcn_make_buffer_rsrc(
              const_cast<T*>(dyt), 0, (int)((size_t)D.B * D.d * 2), 0x00020000);
          const uint32_t voff = col * 2, row_bytes = (uint32_t)D.d * 2;
          const uint32_t wzx = on ? wr[0] : 0u, wzy = on ? wr[1] : 0u;
          for (int j = 0; j < cur.cnt; j += 4) {
            const int nval = cur.cnt - j < 4 ? cur.cnt - j : 4;
            nt_u32x2 q[4];
            uint32_t zb[4], bt[4];
            // (four list entries at once whatever nval is: past the feature's own entries lie other lists or, at the
            //  very end, the arrays that follow in the workspace; what is read there is replaced by token 0 with z = 0)
#pragma unroll
            for (int u = 0; u < 4; ++u) { bt[u] = (uint32_t)tk[j + u]; zb[u] = __float_as_uint(tv[j + u]); }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              if (u >= nval) { bt[u] = 0u; zb[u] = 0u; }
              q[u] = __builtin_amdgcn_raw_buffer_load_b64(rows, voff, bt[u] * row_bytes, 0);
            }
            float pd[4];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              const uint32_t zp = (zb[2 * h] >> 16) | (zb[2 * h + 1] & 0xffff0000u);
              const nt_u32x2 qa = q[2 * h], qb = q[2 * h + 1];
              acc[0] = dot2_bf16(__builtin_amdgcn_perm(qb[0], qa[0], 0x05040100u), zp, acc[0]);
              acc[1] = dot2_bf16(__builtin_amdgcn_perm(qb[0], qa[0], 0x07060302u), zp, acc[1]);
              acc[2] = dot2_bf16(__builtin_amdgcn_perm(qb[1], qa[1], 0x05040100u), zp, acc[2]);
              acc[3] = dot2_bf16(__builtin_amdgcn_perm(qb[1], qa[1], 0x07060302u), zp, acc[3]);
              pd[2 * h] = dot2_bf16(qa[0], wzx, dot2_bf16(qa[1], wzy, 0.f));
              pd[2 * h + 1] = dot2_bf16(qb[0], wzx, dot2_bf16(qb[1], wzy, 0.f));
            }
            if (dz_out) dz_group(j, nval, pd);
          }
        } else {
          const float4 wz = on ? wl : make_float4(0.f, 0.f, 0.f, 0.f);
          int j = 0;
          for (; j + 4 <= cur.cnt; j += 4) {
            typename Elem<T>::Raw4 r[4];
            float zv[4], pd[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const int b = __builtin_amdgcn_readfirstlane(tk[j + u]);
              zv[u] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(tv[j + u])));
              r[u] = Elem<T>::load_raw4(lane_ptr(dyt + (size_t)b * D.d, col));
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const float4 q = Elem<T>::widen4(r[u]);
              acc[0] = fmaf(zv[u], q.x, acc[0]);
              acc[1] = fmaf(zv[u], q.y, acc[1]);
              acc[2] = fmaf(zv[u], q.z, acc[2]);
              acc[3] = fmaf(zv[u], q.w, acc[3]);
              pd[u] = fmaf(wz.x, q.x, fmaf(wz.y, q.y, fmaf(wz.z, q.z, wz.w * q.w)));
            }
            if (dz_out) dz_group(j, 4, pd);
          }
          if (j < cur.cnt) {
            const int nval = cur.cnt - j;
            float pd[4] = {0.f, 0.f, 0.f, 0.f};
            for (int u = 0; u < nval; ++u) {
              const int b = __builtin_amdgcn_readfirstlane(tk[j + u]);
              const float zv = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(tv[j + u])));
              const float4 q = Elem<T>::widen4(Elem<T>::load_raw4(lane_ptr(dyt + (size_t)b * D.d, col)));
              acc[0] = fmaf(zv, q.x, acc[0]);
              acc[1] = fmaf(zv, q.y, acc[1]);
              acc[2] = fmaf(zv, q.z, acc[2]);
              acc[3] = fmaf(zv, q.w, acc[3]);
              const float pu = fmaf(wz.x, q.x, fmaf(wz.y, q.y, fmaf(wz.z, q.z, wz.w * q.w)));
              pd[0] = u == 0 ? pu : pd[0];
              pd[1] = u == 1 ? pu : pd[1];
              pd[2] = u == 2 ? pu : pd[2];
            }
            if (dz_out) dz_group(j, nval, pd);
          }
        }
        const float w4[4] = {wl.x, wl.y, wl.z, wl.w};
        float g4[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) g4[k] = fmaf(coef, w4[k], acc[k]);
        if (dW_dec && on) Elem<T>::store4(lane_ptr(dW_dec + o, col), make_float4(g4[0], g4[1], g4[2], g4[3]));
        if (fuse.m) {
          float mm[4] = {m4[0], m4[1], m4[2], m4[3]};
          float vv[4] = {v4[0], v4[1], v4[2], v4[3]};
          float pp[4];
#pragma unroll
          for (int k = 0; k < 4; ++k) pp[k] = MASTER ? p4[k] : w4[k];
#pragma unroll
          for (int k = 0; k < 4; ++k) adam_element(pp[k], mm[k], vv[k], g4[k], fuse.a);
          const float4 pn = make_float4(pp[0], pp[1], pp[2], pp[3]);
          const typename Elem<T>::Raw4 stored = Elem<T>::narrow4(pn);
          if (on) {
            nt_store_f4(lane_ptr(fuse.m + o, col), make_float4(mm[0], mm[1], mm[2], mm[3]));
            nt_store_f4(lane_ptr(fuse.v + o, col), make_float4(vv[0], vv[1], vv[2], vv[3]));
            if (MASTER) nt_store_f4(lane_ptr(fuse.master + o, col), pn);
            Elem<T>::nt_store_raw4(lane_ptr(W_dec + o, col), stored);
          }
          if (n2_part) {      // sum of squares of the pass's weights as stored, for the next step's norms: slot (slice, pass)
            const float4 wn = Elem<T>::widen4(stored);
            const float sq = on ? (wn.x * wn.x + wn.y * wn.y) + (wn.z * wn.z + wn.w * wn.w) : 0.f;
            const int b16 = __float_as_int(row16_sum(sq));
            const float tot = (__int_as_float(__builtin_amdgcn_readlane(b16, 0)) + __int_as_float(__builtin_amdgcn_readlane(b16, 16))) +
                              (__int_as_float(__builtin_amdgcn_readlane(b16, 32)) + __int_as_float(__builtin_amdgcn_readlane(b16, 48)));
            if (lane == 0)
              n2_part[((size_t)packed_index(cur.l, cur.lp, D.L) * D.F + cur.f) * (8 * passes) + slice * passes + ps] = tot;
          }
        }
      }
    }
  }
}

// Fused dz, second half: 16 lanes per (layer, feature) sum the partial dot products of each listed entry over the
// targets and the eight column slices, always in that order, add the gradient of the sparsity term and write d pre.
template <typename T>
__global__ __launch_bounds__(256) void dz_from_partials_kernel(Dims D, FeatureLists fl, const float* __restrict__ norms,
                                                               float lam_c_over_b, float C, T* __restrict__ dpre,
                                                               const int32_t* __restrict__ flags) {
  if (!fused_dz_selected(flags, fl)) return;
  const int sub = threadIdx.x & 15;
  const long lf = (long)blockIdx.x * 16 + (threadIdx.x >> 4);
  if (lf >= (long)D.L * D.F) return;
  const int l = (int)(lf / D.F), f = (int)(lf % D.F);
  const int cnt = fl.cnt[lf], off = fl.off[lf];
  const float nn = norms[lf];
  const int32_t* tk = fl.tok + (size_t)l * D.B * fl.kcap + off;
  const float* tv = fl.val + (size_t)l * D.B * fl.kcap + off;
  for (int j = sub; j < cnt; j += 16) {
    float acc = 0.f;
    for (int lp = l; lp < D.L; ++lp) {
      const float* q = fl.dz_part + (size_t)packed_index(l, lp, D.L) * 8 * fl.ecap + off + j;
#pragma unroll
      for (int s8 = 0; s8 < 8; ++s8) acc += q[(size_t)s8 * fl.ecap];
    }
    const float zv = tv[j];
    const float ex = __builtin_amdgcn_exp2f(-2.0f * 1.4426950408889634f * C * nn * fabsf(zv));
    const float sden = 1.0f + ex;
    const float gsp = 4.0f * lam_c_over_b * nn * ex * __builtin_amdgcn_rcpf(sden * sden);
    Elem<T>::store(dpre + ((size_t)l * D.B + tk[j]) * D.F + f, acc + gsp);
  }
}

}  // namespace

hipError_t launch_decode_decide(hipStream_t s, Dims D, const int32_t* l0, float density_threshold,
                                float backward_density_threshold, int forced, bool backward_without_row_lists,
                                int32_t* flags) {
  hipLaunchKernelGGL(decode_decide_kernel, dim3(1), dim3(64), 0, s, D, l0, density_threshold,
                     backward_density_threshold, forced, backward_without_row_lists ? 1 : 0, flags);
  return hipGetLastError();
}

hipError_t launch_compact_active(hipStream_t s, bool bf16, Dims D, const void* z, const uint8_t* cls, GatherLists g,
                                 int32_t* flags) {
  const long rows = (long)D.L * D.B;
  const dim3 grid((unsigned)((rows + 3) / 4));
  if (bf16)
    hipLaunchKernelGGL((compact_active_kernel<bf16_t>), grid, dim3(256), 0, s, D, (const bf16_t*)z, cls, g, flags);
  else
    hipLaunchKernelGGL((compact_active_kernel<float>), grid, dim3(256), 0, s, D, (const float*)z, cls, g, flags);
  return hipGetLastError();
}

hipError_t launch_gather_decode(hipStream_t s, bool bf16, Dims D, GatherLists g, const void* W_dec,
                                const float* b_dec, float* y_hat, int32_t* flags) {
  const size_t ncs = ((size_t)D.d + GD_COLS - 1) / GD_COLS;
  const dim3 grid((unsigned)((size_t)D.L * D.B * ncs));
  if (bf16)
    hipLaunchKernelGGL((gather_decode_kernel<bf16_t>), grid, dim3(64), 0, s, D, g, (const bf16_t*)W_dec, b_dec, y_hat,
                       flags);
  else
    hipLaunchKernelGGL((gather_decode_kernel<float>), grid, dim3(64), 0, s, D, g, (const float*)W_dec, b_dec, y_hat,
                       flags);
  return hipGetLastError();
}

hipError_t launch_sparse_dpre_fill(hipStream_t s, bool bf16, Dims D, const uint8_t* cls, const float* norms,
                                   float lam1_over_b, void* dpre, const int32_t* flags, int kcap) {
  const dim3 grid(256 * 16);
  if (bf16)
    hipLaunchKernelGGL((sparse_dpre_fill_kernel<bf16_t>), grid, dim3(256), 0, s, D, cls, norms, lam1_over_b,
                       (bf16_t*)dpre, flags, kcap);
  else
    hipLaunchKernelGGL((sparse_dpre_fill_kernel<float>), grid, dim3(256), 0, s, D, cls, norms, lam1_over_b,
                       (float*)dpre, flags, kcap);
  return hipGetLastError();
}

hipError_t launch_gather_dz(hipStream_t s, bool bf16, Dims D, GatherLists g, const void* d_yhat, const void* W_dec,
                            const float* norms, float lam_c_over_b, float C, void* dpre, const int32_t* flags,
                            const FeatureLists* fused) {
  FeatureLists fz{};
  if (fused) fz = *fused;
  const size_t esz = bf16 ? 2 : 4;
  int tcap = (int)(65536 / ((size_t)D.d * esz));      // targets whose d y_hat rows fit 64 KB of LDS
  if (tcap > D.L) tcap = D.L;
  if (D.d % 8 == 0 && tcap >= 1 && !getenv("CLT_GDZ_NO_LDS")) {
    // One workgroup per row, no loop over rows: the dispatcher hands rows out as workgroups retire, so the long
    // rows of a heavy-tailed batch (the same tokens in every layer) do not pile up on a few resident workgroups.
    const size_t rows = (size_t)D.L * D.B;
    const dim3 grid((unsigned)(rows < ((size_t)1 << 30) ? rows : ((size_t)1 << 30)));
    const size_t lds = (size_t)tcap * D.d * esz;
    if (bf16)
      hipLaunchKernelGGL((gather_dz_lds_kernel<bf16_t>), grid, dim3(1024), lds, s, D, g, (const bf16_t*)d_yhat,
                         (const bf16_t*)W_dec, norms, lam_c_over_b, C, (bf16_t*)dpre, flags, tcap, fz);
    else
      hipLaunchKernelGGL((gather_dz_lds_kernel<float>), grid, dim3(1024), lds, s, D, g, (const float*)d_yhat,
                         (const float*)W_dec, norms, lam_c_over_b, C, (float*)dpre, flags, tcap, fz);
    return hipGetLastError();
  }
  // rows too wide for LDS staging, or not a multiple of 8 columns (or CLT_GDZ_NO_LDS set, for comparison runs)
  const size_t items = ((size_t)D.L * D.B + 7) / 8 * 8 * GDZ_PARTS;
  const dim3 grid((unsigned)(items < 256 * 64 ? items : 256 * 64));
  if (bf16)
    hipLaunchKernelGGL((gather_dz_kernel<bf16_t>), grid, dim3(256), 0, s, D, g, (const bf16_t*)d_yhat,
                       (const bf16_t*)W_dec, norms, lam_c_over_b, C, (bf16_t*)dpre, flags, fz);
  else
    hipLaunchKernelGGL((gather_dz_kernel<float>), grid, dim3(256), 0, s, D, g, (const float*)d_yhat,
                       (const float*)W_dec, norms, lam_c_over_b, C, (float*)dpre, flags, fz);
  return hipGetLastError();
}
hipError_t init_gather() {
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gather_dz_lds_kernel<bf16_t>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&gather_dz_lds_kernel<float>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
}

hipError_t launch_feature_lists(hipStream_t s, bool bf16, Dims D, const uint8_t* cls, const void* z, FeatureLists fl,
                                int32_t* flags, bool dense_when_too_long) {
  const int LF4 = D.L * D.F / 4;
  const dim3 grid((LF4 + 255) / 256, FL_SEGS);
  hipLaunchKernelGGL(fl_count_kernel, grid, dim3(256), 0, s, D, cls, fl, flags);
  hipLaunchKernelGGL(fl_scan_kernel, dim3(D.L), dim3(FL_SCAN_THREADS), 0, s, D, fl, flags,
                     dense_when_too_long && fl.dz_part ? fl.ecap : 0);
  if (bf16)
    hipLaunchKernelGGL((fl_fill_kernel<bf16_t>), grid, dim3(256), 0, s, D, cls, (const bf16_t*)z, fl, flags);
  else
    hipLaunchKernelGGL((fl_fill_kernel<float>), grid, dim3(256), 0, s, D, cls, (const float*)z, fl, flags);
  return hipGetLastError();
}

// The sliced kernel: d in eight slices of whole lane quads, and one target's d y_hat within reach of a 32-bit byte offset
static bool sparse_dwdec_sliced(Dims D) {
  return D.d % 32 == 0 && (size_t)D.B * D.d * 2 < ((size_t)1 << 31) && !getenv("CLT_SD_ROWS");
}
bool sparse_dwdec_takes_dz(Dims D) { return sparse_dwdec_sliced(D) && !getenv("CLT_NO_FUSED_DZ"); }

hipError_t launch_dz_from_partials(hipStream_t s, bool bf16, Dims D, FeatureLists fl, const float* norms,
                                   float lam_c_over_b, float C, void* dpre, const int32_t* flags) {
  if (!fl.dz_part) return hipSuccess;
  const dim3 grid((unsigned)(((size_t)D.L * D.F + 15) / 16));
  if (bf16)
    hipLaunchKernelGGL((dz_from_partials_kernel<bf16_t>), grid, dim3(256), 0, s, D, fl, norms, lam_c_over_b, C,
                       (bf16_t*)dpre, flags);
  else
    hipLaunchKernelGGL((dz_from_partials_kernel<float>), grid, dim3(256), 0, s, D, fl, norms, lam_c_over_b, C,
                       (float*)dpre, flags);
  return hipGetLastError();
}

hipError_t launch_sparse_dwdec(hipStream_t s, bool bf16, Dims D, FeatureLists fl, const DWdecArgs& a,
                               const int32_t* flags) {
  const bool master = a.fuse.m && a.fuse.master;
  float* n2 = (bf16 && a.fuse.m && D.d % 256 == 0) ? a.n2_part : nullptr;
  // Both kernels get one workgroup per item while the grid allows it (see the comment in the sliced kernel).
  if (sparse_dwdec_sliced(D)) {
    const size_t per_xcd = ((size_t)(D.L * (D.L + 1) / 2) * ((D.F + 3) / 4) + SD_ITEMS_PER_WG - 1) / SD_ITEMS_PER_WG,
                 gx = (size_t)1 << 27;
    const dim3 grid((unsigned)(8 * (per_xcd < gx ? per_xcd : gx)));
#define CLT_SDS(T, M)                                                                                              \
  hipLaunchKernelGGL((sparse_dwdec_sliced_kernel<T, M>), grid, dim3(256), 0, s, D, fl, (const T*)a.d_yhat,         \
                     (T*)a.W_dec, a.G, a.norms, (T*)a.dW_dec, a.fuse, flags, n2, fl.tok, fl.val)
    if (bf16) { if (master) CLT_SDS(bf16_t, true); else CLT_SDS(bf16_t, false); }
    else { if (master) CLT_SDS(float, true); else CLT_SDS(float, false); }
#undef CLT_SDS
    return hipGetLastError();
  }
  // d not a multiple of 32 (or CLT_SD_ROWS set, for comparison runs): whole rows per workgroup
  const size_t items = (size_t)D.L * D.F * ((D.L + SD_TCH - 1) / SD_TCH), gcap = (size_t)1 << 30;
  const dim3 grid((unsigned)(items < gcap ? items : gcap));
#define CLT_SD(T, M)                                                                                              \
  hipLaunchKernelGGL((sparse_dwdec_kernel<T, M>), grid, dim3(256), 0, s, D, fl, (const T*)a.d_yhat, (T*)a.W_dec, a.G, \
                     a.norms, (T*)a.dW_dec, a.fuse, flags, n2)
  if (bf16) { if (master) CLT_SD(bf16_t, true); else CLT_SD(bf16_t, false); }
  else { if (master) CLT_SD(float, true); else CLT_SD(float, false); }
#undef CLT_SD
  return hipGetLastError();
}

}  // namespace clt
