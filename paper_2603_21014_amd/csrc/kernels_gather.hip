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

namespace clt {
namespace {

__global__ void decode_decide_kernel(Dims D, const int32_t* __restrict__ l0, float thr, int forced,
                                     int32_t* __restrict__ flags) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  long long tot = 0;
  for (int l = 0; l < D.L; ++l) tot += l0[l];
  const double dens = (double)tot / ((double)D.L * D.B * D.F);
  flags[0] = (forced || dens <= (double)thr) ? 1 : 0;
  flags[1] = 0;
  flags[2] = 1;
}

// One wavefront per (layer, token) row; lanes take 4 consecutive features per
// pass, positions come from wave-wide exclusive scans of the per-lane counts.
// Active features fill the row's slots from the front, window-only features from the back.
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
  if (flags[0] == 0) return;
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);   // l * B + b
  if (row >= (long)D.L * D.B) return;
  const T* zr = z + (size_t)row * D.F;
  const uint8_t* cr = cls + (size_t)row * D.F;
  int32_t* oi = g.idx + (size_t)row * g.kcap;
  float* ov = g.val + (size_t)row * g.kcap;
  int base = 0, base_w = 0;
  for (int f0 = 0; f0 < D.F; f0 += 256) {
    const int f = f0 + lane * 4;
    uint32_t c4 = 0;
    float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (f < D.F) {
      c4 = *reinterpret_cast<const uint32_t*>(cr + f);
      if (c4 & 0x01010101u) z4 = Elem<T>::load4(zr + f);
    }
    const uint32_t a4 = c4 & 0x01010101u;                       // active
    const uint32_t w4 = ((c4 >> 1) & 0x01010101u) & ~a4;        // in the window, not active
    const int n = __popc(a4), nw = __popc(w4);
    const int incl = wave_incl_scan(n, lane), incl_w = wave_incl_scan(nw, lane);
    int pos = base + incl - n, pos_w = base_w + incl_w - nw;
    const float zz[4] = {z4.x, z4.y, z4.z, z4.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if ((a4 >> (8 * i)) & 1u) {
        if (pos < g.kcap) { oi[pos] = f + i; ov[pos] = zz[i]; }
        ++pos;
      }
      if ((w4 >> (8 * i)) & 1u) {
        if (pos_w < g.kcap) { oi[g.kcap - 1 - pos_w] = f + i; ov[g.kcap - 1 - pos_w] = 0.f; }
        ++pos_w;
      }
    }
    base += __shfl(incl, 63, 64);
    base_w += __shfl(incl_w, 63, 64);
  }
  if (lane == 0) {
    g.counts[row] = base;
    g.counts_w[row] = base_w;
    atomicMax(flags + 1, base + base_w);     // lists that collide make every gather kernel stand down
  }
}

// Accumulates 8 columns per lane; d is walked in passes of 2048 columns.
template <typename T>
__global__ __launch_bounds__(256) void gather_decode_kernel(Dims D, GatherLists g, const T* __restrict__ W_dec,
                                                            const float* __restrict__ b_dec,
                                                            float* __restrict__ y_hat, int32_t* __restrict__ flags) {
  if (!gather_selected(flags, g.kcap)) return;
  const int lp = D.L - 1 - (int)(blockIdx.x / D.B);   // heaviest targets first
  const int b = (int)(blockIdx.x % D.B);
  if (blockIdx.x == 0 && threadIdx.x == 0) flags[2] = 2;
  for (int c0 = 0; c0 < D.d; c0 += 2048) {
    const int col = c0 + threadIdx.x * 8;
    const bool ok = col < D.d;
    float acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = ok ? b_dec[(size_t)lp * D.d + col + i] : 0.f;
    for (int l = 0; l <= lp; ++l) {
      const size_t row = (size_t)l * D.B + b;
      const int cnt = g.counts[row];
      const int32_t* ii = g.idx + row * g.kcap;
      const float* vv = g.val + row * g.kcap;
      const T* Wp = W_dec + (size_t)packed_index(l, lp, D.L) * D.F * D.d + col;
      int j = 0;
      for (; j + 4 <= cnt; j += 4) {          // four rows in flight per lane
        float4 r[4][2];
        float v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const T* rp = Wp + (size_t)ii[j + u] * D.d;
          v[u] = vv[j + u];
          if (ok) { r[u][0] = Elem<T>::load4(rp); r[u][1] = Elem<T>::load4(rp + 4); }
        }
        if (ok) {
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            acc[0] = fmaf(v[u], r[u][0].x, acc[0]); acc[1] = fmaf(v[u], r[u][0].y, acc[1]);
            acc[2] = fmaf(v[u], r[u][0].z, acc[2]); acc[3] = fmaf(v[u], r[u][0].w, acc[3]);
            acc[4] = fmaf(v[u], r[u][1].x, acc[4]); acc[5] = fmaf(v[u], r[u][1].y, acc[5]);
            acc[6] = fmaf(v[u], r[u][1].z, acc[6]); acc[7] = fmaf(v[u], r[u][1].w, acc[7]);
          }
        }
      }
      for (; j < cnt; ++j) {
        const T* rp = Wp + (size_t)ii[j] * D.d;
        const float v = vv[j];
        if (ok) {
          const float4 r0 = Elem<T>::load4(rp), r1 = Elem<T>::load4(rp + 4);
          acc[0] = fmaf(v, r0.x, acc[0]); acc[1] = fmaf(v, r0.y, acc[1]);
          acc[2] = fmaf(v, r0.z, acc[2]); acc[3] = fmaf(v, r0.w, acc[3]);
          acc[4] = fmaf(v, r1.x, acc[4]); acc[5] = fmaf(v, r1.y, acc[5]);
          acc[6] = fmaf(v, r1.z, acc[6]); acc[7] = fmaf(v, r1.w, acc[7]);
        }
      }
    }
    if (ok) {
      float* o = y_hat + ((size_t)lp * D.B + b) * D.d + col;
      *reinterpret_cast<float4*>(o) = make_float4(acc[0], acc[1], acc[2], acc[3]);
      *reinterpret_cast<float4*>(o + 4) = make_float4(acc[4], acc[5], acc[6], acc[7]);
    }
  }
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
  if (!gather_selected(flags, kcap)) return;
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

// One workgroup per (layer, token) row, 8 columns of d per lane, 8 listed entries per batch:
// for every target l' >= l the token's d y_hat columns are loaded once and multiplied with the
// decoder rows of the 8 entries; the 8 partial dot products are then summed over the workgroup.
template <typename T>
__global__ __launch_bounds__(256) void gather_dz_kernel(Dims D, GatherLists g, const T* __restrict__ d_yhat,
                                                        const T* __restrict__ W_dec, const float* __restrict__ norms,
                                                        float lam_c_over_b, float C, T* __restrict__ dpre,
                                                        const int32_t* __restrict__ flags) {
  if (!gather_selected(flags, g.kcap)) return;
  __shared__ float red[4][8];
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const long rows = (long)D.L * D.B;
  for (long row = blockIdx.x; row < rows; row += gridDim.x) {    // layer 0 (most targets) first
    const int l = (int)(row / D.B), b = (int)(row % D.B);
    const int na = g.counts[row], n = na + g.counts_w[row];
    const int32_t* ii = g.idx + (size_t)row * g.kcap;
    const float* vv = g.val + (size_t)row * g.kcap;
    for (int e0 = 0; e0 < n; e0 += 8) {
      int f[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int e = e0 + u;                                    // slot: front for active, back for window-only
        f[u] = e < n ? ii[e < na ? e : g.kcap - 1 - (e - na)] : -1;
      }
      float part[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      for (int c0 = 0; c0 < D.d; c0 += 2048) {
        const int col = c0 + tid * 8;
        if (col < D.d) {
          for (int lp = l; lp < D.L; ++lp) {
            float dy[8];
            Row8<T>::load(d_yhat + ((size_t)lp * D.B + b) * D.d + col, dy);
            const T* Wp = W_dec + (size_t)packed_index(l, lp, D.L) * D.F * D.d + col;
            float w[8][8];
#pragma unroll
            for (int u = 0; u < 8; ++u)
              if (f[u] >= 0) Row8<T>::load(Wp + (size_t)f[u] * D.d, w[u]);
#pragma unroll
            for (int u = 0; u < 8; ++u)
              if (f[u] >= 0) {
#pragma unroll
                for (int k = 0; k < 8; ++k) part[u] = fmaf(w[u][k], dy[k], part[u]);
              }
          }
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) part[u] += __shfl_xor(part[u], off, 64);
      }
      __syncthreads();                       // the previous batch's readers are done with red
      if (lane == 0) {
#pragma unroll
        for (int u = 0; u < 8; ++u) red[wv][u] = part[u];
      }
      __syncthreads();
      if (tid < 8 && e0 + tid < n) {
        const int e = e0 + tid;
        const int slot = e < na ? e : g.kcap - 1 - (e - na);
        const int fe = ii[slot];
        const float zv = vv[slot];
        const float nn = norms[(size_t)l * D.F + fe];
        const float ex = __builtin_amdgcn_exp2f(-2.0f * 1.4426950408889634f * C * nn * fabsf(zv));
        const float sden = 1.0f + ex;
        const float gsp = 4.0f * lam_c_over_b * nn * ex * __builtin_amdgcn_rcpf(sden * sden);
        const float dz = ((red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid])) + gsp;
        Elem<T>::store(dpre + (size_t)row * D.F + fe, dz);
      }
    }
  }
}

// ---- feature lists: column scan of the class bytes in FL_SEGS token segments ----
// Each thread owns 4 consecutive features of one layer and one token segment.
__global__ __launch_bounds__(256) void fl_count_kernel(Dims D, const uint8_t* __restrict__ cls, FeatureLists fl,
                                                       const int32_t* __restrict__ flags) {
  if (!gather_selected(flags, fl.kcap)) return;
  const int LF4 = D.L * D.F / 4;
  const int q = blockIdx.x * 256 + threadIdx.x, sgm = blockIdx.y;
  if (q >= LF4) return;
  const int l = (q * 4) / D.F, f = (q * 4) % D.F;
  const int seg_len = (D.B + FL_SEGS - 1) / FL_SEGS;
  const int b0 = sgm * seg_len, b1 = min(D.B, b0 + seg_len);
  int c[4] = {0, 0, 0, 0};
  for (int b = b0; b < b1; ++b) {
    const uint32_t a4 = *reinterpret_cast<const uint32_t*>(cls + ((size_t)l * D.B + b) * D.F + f);
#pragma unroll
    for (int i = 0; i < 4; ++i) c[i] += (int)((a4 >> (8 * i)) & 1u);
  }
  int32_t* o = fl.seg + (size_t)sgm * D.L * D.F + (size_t)q * 4;
  o[0] = c[0]; o[1] = c[1]; o[2] = c[2]; o[3] = c[3];
}

// One workgroup per layer: layer-local exclusive scan over the features of the summed segment
// counts; the segment counts are turned into each segment's first slot.
__global__ __launch_bounds__(256) void fl_scan_kernel(Dims D, FeatureLists fl, const int32_t* __restrict__ flags) {
  if (!gather_selected(flags, fl.kcap)) return;
  __shared__ int tot[256];
  const int l = blockIdx.x, tid = threadIdx.x;
  const int per = (D.F + 255) / 256;
  const int f0 = tid * per, f1 = min(D.F, f0 + per);
  const size_t LF = (size_t)D.L * D.F;
  int sum = 0;
  for (int f = f0; f < f1; ++f) {
    int c = 0;
    for (int sgm = 0; sgm < FL_SEGS; ++sgm) c += fl.seg[(size_t)sgm * LF + (size_t)l * D.F + f];
    sum += c;
  }
  tot[tid] = sum;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {              // inclusive scan of the 256 thread totals
    const int v = tid >= off ? tot[tid - off] : 0;
    __syncthreads();
    tot[tid] += v;
    __syncthreads();
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
  if (!gather_selected(flags, fl.kcap)) return;
  const int LF4 = D.L * D.F / 4;
  const int q = blockIdx.x * 256 + threadIdx.x, sgm = blockIdx.y;
  if (q >= LF4) return;
  const int l = (q * 4) / D.F, f = (q * 4) % D.F;
  const int seg_len = (D.B + FL_SEGS - 1) / FL_SEGS;
  const int b0 = sgm * seg_len, b1 = min(D.B, b0 + seg_len);
  const int32_t* so = fl.seg + (size_t)sgm * D.L * D.F + (size_t)q * 4;
  int pos[4] = {so[0], so[1], so[2], so[3]};
  const size_t base = (size_t)l * D.B * fl.kcap;        // layer l's region of the lists
  for (int b = b0; b < b1; ++b) {
    const size_t o = ((size_t)l * D.B + b) * D.F + f;
    const uint32_t a4 = *reinterpret_cast<const uint32_t*>(cls + o) & 0x01010101u;
    if (!a4) continue;
    const float4 z4 = Elem<T>::load4(z + o);
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

// One item = (layer l, feature f, chunk of up to 8 targets): a workgroup of 256 lanes, 8 columns
// each, sums z * d y_hat rows over the feature's tokens (two tokens in flight), then finishes the
// row of every target: norm term, optional gradient store, optional Adam update.
constexpr int SD_TCH = 8;
template <typename T>
__global__ __launch_bounds__(256) void sparse_dwdec_kernel(Dims D, FeatureLists fl, const T* __restrict__ d_yhat,
                                                           T* __restrict__ W_dec, const float* __restrict__ G,
                                                           const float* __restrict__ norms, T* __restrict__ dW_dec,
                                                           AdamFuseArgs fuse, const int32_t* __restrict__ flags) {
  if (!gather_selected(flags, fl.kcap)) return;
  const int tid = threadIdx.x;
  const int chunks = (D.L + SD_TCH - 1) / SD_TCH;          // chunk slots per (l, f); those past L - l are empty
  const long items = (long)D.L * D.F * chunks;
  for (long it = blockIdx.x; it < items; it += gridDim.x) {
    const int c = (int)(it % chunks);
    const long lf = it / chunks;
    const int l = (int)(lf / D.F), f = (int)(lf % D.F);
    const int lp0 = l + c * SD_TCH;
    if (lp0 >= D.L) continue;
    const int nt = min(SD_TCH, D.L - lp0);
    const int cnt = fl.cnt[lf];
    const int32_t* tk = fl.tok + (size_t)l * D.B * fl.kcap + fl.off[lf];
    const float* tv = fl.val + (size_t)l * D.B * fl.kcap + fl.off[lf];
    const float coef = G[lf] * __builtin_amdgcn_rcpf(fmaxf(norms[lf], 1e-30f));
    for (int c0 = 0; c0 < D.d; c0 += 2048) {
      const int col = c0 + tid * 8;
      if (col >= D.d) continue;
      float acc[SD_TCH][8];
#pragma unroll
      for (int t = 0; t < SD_TCH; ++t)
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[t][k] = 0.f;
      int j = 0;
      for (; j + 2 <= cnt; j += 2) {
        const int bA = tk[j], bB = tk[j + 1];
        const float vA = tv[j], vB = tv[j + 1];
        float rA[SD_TCH][8], rB[SD_TCH][8];
#pragma unroll
        for (int t = 0; t < SD_TCH; ++t)
          if (t < nt) {
            Row8<T>::load(d_yhat + ((size_t)(lp0 + t) * D.B + bA) * D.d + col, rA[t]);
            Row8<T>::load(d_yhat + ((size_t)(lp0 + t) * D.B + bB) * D.d + col, rB[t]);
          }
#pragma unroll
        for (int t = 0; t < SD_TCH; ++t)
          if (t < nt) {
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[t][k] = fmaf(vA, rA[t][k], acc[t][k]);
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[t][k] = fmaf(vB, rB[t][k], acc[t][k]);
          }
      }
      if (j < cnt) {
        const int bA = tk[j];
        const float vA = tv[j];
#pragma unroll
        for (int t = 0; t < SD_TCH; ++t)
          if (t < nt) {
            float rA[8];
            Row8<T>::load(d_yhat + ((size_t)(lp0 + t) * D.B + bA) * D.d + col, rA);
#pragma unroll
            for (int k = 0; k < 8; ++k) acc[t][k] = fmaf(vA, rA[k], acc[t][k]);
          }
      }
#pragma unroll
      for (int t = 0; t < SD_TCH; ++t)
        if (t < nt) {
          const size_t o = ((size_t)packed_index(l, lp0 + t, D.L) * D.F + f) * D.d + col;
#pragma unroll
          for (int h = 0; h < 2; ++h) {                   // two groups of 4 columns
            const size_t oh = o + 4 * h;
            const float4 w = Elem<T>::nt_load4(W_dec + oh);
            const float4 gr = make_float4(fmaf(coef, w.x, acc[t][4 * h]), fmaf(coef, w.y, acc[t][4 * h + 1]),
                                          fmaf(coef, w.z, acc[t][4 * h + 2]), fmaf(coef, w.w, acc[t][4 * h + 3]));
            if (dW_dec) Elem<T>::store4(dW_dec + oh, gr);
            if (fuse.m) {
              const float4 m4 = nt_load_f4(fuse.m + oh), v4 = nt_load_f4(fuse.v + oh);
              const float4 p4 = fuse.master ? nt_load_f4(fuse.master + oh) : w;
              const float g4[4] = {gr.x, gr.y, gr.z, gr.w};
              float mm[4] = {m4.x, m4.y, m4.z, m4.w}, vv[4] = {v4.x, v4.y, v4.z, v4.w};
              float pp[4] = {p4.x, p4.y, p4.z, p4.w};
#pragma unroll
              for (int k = 0; k < 4; ++k) adam_element(pp[k], mm[k], vv[k], g4[k], fuse.a);
              nt_store_f4(fuse.m + oh, make_float4(mm[0], mm[1], mm[2], mm[3]));
              nt_store_f4(fuse.v + oh, make_float4(vv[0], vv[1], vv[2], vv[3]));
              const float4 pn = make_float4(pp[0], pp[1], pp[2], pp[3]);
              if (fuse.master) nt_store_f4(fuse.master + oh, pn);
              Elem<T>::nt_store4(W_dec + oh, pn);
            }
          }
        }
    }
  }
}

}  // namespace

hipError_t launch_decode_decide(hipStream_t s, Dims D, const int32_t* l0, float density_threshold, int forced,
                                int32_t* flags) {
  hipLaunchKernelGGL(decode_decide_kernel, dim3(1), dim3(64), 0, s, D, l0, density_threshold, forced, flags);
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
  const dim3 grid((unsigned)((size_t)D.L * D.B));
  if (bf16)
    hipLaunchKernelGGL((gather_decode_kernel<bf16_t>), grid, dim3(256), 0, s, D, g, (const bf16_t*)W_dec, b_dec, y_hat,
                       flags);
  else
    hipLaunchKernelGGL((gather_decode_kernel<float>), grid, dim3(256), 0, s, D, g, (const float*)W_dec, b_dec, y_hat,
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
                            const float* norms, float lam_c_over_b, float C, void* dpre, const int32_t* flags) {
  const size_t rows = (size_t)D.L * D.B;
  const dim3 grid((unsigned)(rows < 256 * 64 ? rows : 256 * 64));
  if (bf16)
    hipLaunchKernelGGL((gather_dz_kernel<bf16_t>), grid, dim3(256), 0, s, D, g, (const bf16_t*)d_yhat,
                       (const bf16_t*)W_dec, norms, lam_c_over_b, C, (bf16_t*)dpre, flags);
  else
    hipLaunchKernelGGL((gather_dz_kernel<float>), grid, dim3(256), 0, s, D, g, (const float*)d_yhat,
                       (const float*)W_dec, norms, lam_c_over_b, C, (float*)dpre, flags);
  return hipGetLastError();
}

hipError_t launch_feature_lists(hipStream_t s, bool bf16, Dims D, const uint8_t* cls, const void* z, FeatureLists fl,
                                const int32_t* flags) {
  const int LF4 = D.L * D.F / 4;
  const dim3 grid((LF4 + 255) / 256, FL_SEGS);
  hipLaunchKernelGGL(fl_count_kernel, grid, dim3(256), 0, s, D, cls, fl, flags);
  hipLaunchKernelGGL(fl_scan_kernel, dim3(D.L), dim3(256), 0, s, D, fl, flags);
  if (bf16)
    hipLaunchKernelGGL((fl_fill_kernel<bf16_t>), grid, dim3(256), 0, s, D, cls, (const bf16_t*)z, fl, flags);
  else
    hipLaunchKernelGGL((fl_fill_kernel<float>), grid, dim3(256), 0, s, D, cls, (const float*)z, fl, flags);
  return hipGetLastError();
}

hipError_t launch_sparse_dwdec(hipStream_t s, bool bf16, Dims D, FeatureLists fl, const DWdecArgs& a,
                               const int32_t* flags) {
  const size_t items = (size_t)D.L * D.F * ((D.L + SD_TCH - 1) / SD_TCH);
  const dim3 grid((unsigned)(items < 256 * 64 ? items : 256 * 64));
  if (bf16)
    hipLaunchKernelGGL((sparse_dwdec_kernel<bf16_t>), grid, dim3(256), 0, s, D, fl, (const bf16_t*)a.d_yhat,
                       (bf16_t*)a.W_dec, a.G, a.norms, (bf16_t*)a.dW_dec, a.fuse, flags);
  else
    hipLaunchKernelGGL((sparse_dwdec_kernel<float>), grid, dim3(256), 0, s, D, fl, (const float*)a.d_yhat,
                       (float*)a.W_dec, a.G, a.norms, (float*)a.dW_dec, a.fuse, flags);
  return hipGetLastError();
}

}  // namespace clt
