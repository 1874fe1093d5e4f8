// HBM-bound kernels of the CLT train step: decoder norms, loss reductions with
// their fused gradient by-products, the threshold (straight-through) column
// reductions and Adam.  Reductions are two-stage with a fixed summation order
// (per-block partials, then one pass over the partials), so results are
// bitwise reproducible run to run.
#include "common.h"

namespace clt {
namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}
// sum over a 256-lane block; result valid in thread 0
__device__ __forceinline__ double block_sum_256(double v) {
  __shared__ double sh[4];
  v = wave_sum(v);
  if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
  __syncthreads();
  return sh[0] + sh[1] + sh[2] + sh[3];
}

__global__ void zero_i32_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// ---- decoder norms (App. B): one wavefront per (source layer, feature) -----
// The L-l blocks that leave source l are contiguous in the source-major packing,
// so feature f's rows are L-l runs of d contiguous elements.
template <typename T>
__global__ __launch_bounds__(256) void decoder_norms_kernel(Dims D, const T* __restrict__ W_dec,
                                                            float* __restrict__ norms) {
  const int lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);   // l * F + f
  if (row >= (long)D.L * D.F) return;
  const int l = (int)(row / D.F), f = (int)(row - (long)l * D.F);
  const T* base = W_dec + ((size_t)packed_index(l, l, D.L) * D.F + f) * D.d;
  float acc = 0.f;
  for (int s = 0; s < D.L - l; ++s) {
    const T* r = base + (size_t)s * D.F * D.d;
    for (int j = lane * 4; j < D.d; j += 256) {
      const float4 v = Elem<T>::load4(r + j);
      acc += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
  }
  acc = wave_sum(acc);
  if (lane == 0) norms[row] = sqrtf(acc);
}

// The same norms from sums of squares that the last fused update left, in a fixed order.  The dense kernel leaves
// them per (block, 64-column run, feature), [P][d / 64][F]; the list-driven row kernel per (block, feature, slot),
// [P][F][8 ceil(d / 2048)].  Which of the two ran is what the device-side switch decided in that step (flags).
__global__ __launch_bounds__(256) void norms_from_partials_kernel(Dims D, const float* __restrict__ n2_part,
                                                                  float* __restrict__ norms,
                                                                  const int32_t* __restrict__ flags, int kcap) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;      // l * F + f
  if (i >= (long)D.L * D.F) return;
  const int l = (int)(i / D.F), f = (int)(i - (long)l * D.F);
  float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (flags && lists_backward_selected(flags, kcap)) {
    const int slots = 8 * ((D.d + 2047) / 2048);
    const float* base = n2_part + ((size_t)packed_index(l, l, D.L) * D.F + f) * slots;
    for (int j = 0; j < D.L - l; ++j)
      for (int q = 0; q < slots; q += 8) {
        const float4 u = *reinterpret_cast<const float4*>(base + (size_t)j * D.F * slots + q);
        const float4 w = *reinterpret_cast<const float4*>(base + (size_t)j * D.F * slots + q + 4);
        a[0] += u.x; a[1] += u.y; a[2] += u.z; a[3] += u.w; a[4] += w.x; a[5] += w.y; a[6] += w.z; a[7] += w.w;
      }
  } else {
    const int runs = D.d >> 6;
    const float* base = n2_part + (size_t)packed_index(l, l, D.L) * runs * D.F + f;
    // eight independent chains keep eight loads in flight per lane; the order of the sum stays fixed
    const int n = (D.L - l) * runs;
    int j = 0;
    for (; j + 8 <= n; j += 8) {
#pragma unroll
      for (int q = 0; q < 8; ++q) a[q] += base[(size_t)(j + q) * D.F];
    }
    for (; j < n; ++j) a[j & 7] += base[(size_t)j * D.F];
  }
  norms[i] = sqrtf(((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7])));
}

// ---- reconstruction loss: r = y_hat - y; partial sum r^2; d_yhat = 2 r / B;
// column partial sums of d_yhat (for db_dec).  grid = (row blocks, L), each
// thread owns 4 consecutive columns and walks the block's rows.
template <typename T, bool INT8>
__global__ __launch_bounds__(256) void loss_rec_kernel(Dims D, const float* __restrict__ y_hat, const void* yv,
                                                       const float* __restrict__ y_scale, T* __restrict__ d_yhat,
                                                       double* __restrict__ loss_part, float* __restrict__ col_part) {
  const int rb = blockIdx.x, l = blockIdx.y;
  const int r0 = rb * LOSS_ROWS_PER_BLOCK, r1 = min(D.B, r0 + LOSS_ROWS_PER_BLOCK);
  const float two_over_b = 2.0f / (float)D.B;
  double sq = 0.0;
  for (int c = threadIdx.x * 4; c < D.d; c += 1024) {
    float4 cs = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int r = r0; r < r1; ++r) {
      const size_t o = ((size_t)l * D.B + r) * D.d + c;
      const float4 yh = *reinterpret_cast<const float4*>(y_hat + o);
      float4 y;
      if (INT8) {
        const uint32_t q = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const int8_t*>(yv) + o);
        const float s = y_scale[(size_t)l * D.B + r];
        y = make_float4(s * (float)(int8_t)q, s * (float)(int8_t)(q >> 8), s * (float)(int8_t)(q >> 16),
                        s * (float)(int8_t)(q >> 24));
      } else {
        y = Elem<T>::load4(reinterpret_cast<const T*>(yv) + o);
      }
      const float4 rr = make_float4(yh.x - y.x, yh.y - y.y, yh.z - y.z, yh.w - y.w);
      sq += (double)(rr.x * rr.x + rr.y * rr.y) + (double)(rr.z * rr.z + rr.w * rr.w);
      const float4 g = make_float4(two_over_b * rr.x, two_over_b * rr.y, two_over_b * rr.z, two_over_b * rr.w);
      Elem<T>::store4(d_yhat + o, g);
      cs.x += g.x; cs.y += g.y; cs.z += g.z; cs.w += g.w;
    }
    *reinterpret_cast<float4*>(col_part + ((size_t)rb * D.L + l) * D.d + c) = cs;
  }
  const double tot = block_sum_256(sq);
  if (threadIdx.x == 0) loss_part[(size_t)l * gridDim.x + rb] = tot;
}

// ---- sparsity loss: partial sum tanh(C z n); column partials of C z sech^2(C z n)
// (both from one hardware exponential).
// With DEAD also the App. B dead-feature term: partial sum relu(theta - pre) n and the
// column partials of relu(theta - pre) (its derivative w.r.t. the decoder norm).
template <typename T, bool DEAD>
__global__ __launch_bounds__(256) void loss_sparsity_kernel(Dims D, const T* __restrict__ z,
                                                            const float* __restrict__ norms, float C,
                                                            double* __restrict__ loss_part,
                                                            float* __restrict__ col_part, const T* __restrict__ pre,
                                                            const float* __restrict__ theta, bool log_threshold,
                                                            double* __restrict__ dead_part,
                                                            float* __restrict__ dead_col_part) {
  const int rb = blockIdx.x, l = blockIdx.y;
  const int r0 = rb * LOSS_ROWS_PER_BLOCK, r1 = min(D.B, r0 + LOSS_ROWS_PER_BLOCK);
  double sp = 0.0, dead = 0.0;
  for (int c = threadIdx.x * 4; c < D.F; c += 1024) {
    const float4 n4 = *reinterpret_cast<const float4*>(norms + (size_t)l * D.F + c);
    const float nn[4] = {n4.x, n4.y, n4.z, n4.w};
    const float cn[4] = {C * n4.x, C * n4.y, C * n4.z, C * n4.w};
    float th[4] = {0.f, 0.f, 0.f, 0.f};
    if (DEAD) {
      const float4 t4 = *reinterpret_cast<const float4*>(theta + (size_t)l * D.F + c);
      th[0] = threshold_value(t4.x, log_threshold); th[1] = threshold_value(t4.y, log_threshold);
      th[2] = threshold_value(t4.z, log_threshold); th[3] = threshold_value(t4.w, log_threshold);
    }
    float cs[4] = {0.f, 0.f, 0.f, 0.f}, ds[4] = {0.f, 0.f, 0.f, 0.f};
    float ts = 0.f, dsum = 0.f;
    for (int r = r0; r < r1; ++r) {
      const size_t o = ((size_t)l * D.B + r) * D.F + c;
      const float4 z4 = Elem<T>::load4(z + o);
      const float zz[4] = {z4.x, z4.y, z4.z, z4.w};
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (zz[i] != 0.f) {
          // e = exp(-2|u|): tanh|u| = (1 - e) / (1 + e), sech^2 u = 4 e / (1 + e)^2 (no cancellation for large u)
          const float u = cn[i] * zz[i];
          const float e = __builtin_amdgcn_exp2f(-2.0f * 1.4426950408889634f * fabsf(u));
          const float r = __builtin_amdgcn_rcpf(1.0f + e);
          ts += copysignf((1.0f - e) * r, u);
          cs[i] += C * zz[i] * (4.0f * e * r * r);
        }
      }
      if (DEAD) {
        const float4 p4 = Elem<T>::load4(pre + o);
        const float pp[4] = {p4.x, p4.y, p4.z, p4.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float g = fmaxf(th[i] - pp[i], 0.f);
          ds[i] += g;
          dsum += g * nn[i];
        }
      }
    }
    sp += (double)ts;
    dead += (double)dsum;
    const size_t po = ((size_t)rb * D.L + l) * D.F + c;
    *reinterpret_cast<float4*>(col_part + po) = make_float4(cs[0], cs[1], cs[2], cs[3]);
    if (DEAD) *reinterpret_cast<float4*>(dead_col_part + po) = make_float4(ds[0], ds[1], ds[2], ds[3]);
  }
  const double tot = block_sum_256(sp);
  if (threadIdx.x == 0) loss_part[(size_t)l * gridDim.x + rb] = tot;
  if (DEAD) {
    __syncthreads();
    const double dt = block_sum_256(dead);
    if (threadIdx.x == 0) dead_part[(size_t)l * gridDim.x + rb] = dt;
  }
}

__global__ __launch_bounds__(256) void loss_final_kernel(const double* part_rec, int n_rec, const double* part_sp,
                                                         int n_sp, const double* part_dead, float inv_B, float lambda0,
                                                         float lambda1, float* loss_dev) {
  double a = 0.0, b = 0.0, c = 0.0;
  for (int i = threadIdx.x; i < n_rec; i += 256) a += part_rec[i];
  for (int i = threadIdx.x; i < n_sp; i += 256) b += part_sp[i];
  if (part_dead)
    for (int i = threadIdx.x; i < n_sp; i += 256) c += part_dead[i];
  a = block_sum_256(a);
  __syncthreads();
  b = block_sum_256(b);
  __syncthreads();
  c = block_sum_256(c);
  if (threadIdx.x == 0) {
    const double rec = a * (double)inv_B, sp = b * (double)inv_B * (double)lambda0;
    const double dead = c * (double)inv_B * (double)lambda1;
    loss_dev[0] = (float)(rec + sp + dead);
    loss_dev[1] = (float)rec;
    loss_dev[2] = (float)sp;
    loss_dev[3] = (float)dead;
  }
}

__global__ __launch_bounds__(256) void col_reduce_kernel(const float* __restrict__ part, int nparts, int ncols,
                                                         float alpha, const float* __restrict__ theta, float inv_eps,
                                                         float* __restrict__ out, bool accumulate, PartsSwitch sw) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= ncols) return;
  if (sw.flags && lists_backward_selected(sw.flags, sw.kcap)) nparts = sw.nparts_lists;
  float s = 0.f;
  for (int r = 0; r < nparts; ++r) s += part[(size_t)r * ncols + c];
  s *= alpha;
  if (theta) s = (s == 0.f) ? 0.f : s * -(theta[c] * inv_eps);   // empty window: exactly 0, also for theta = inf
  out[c] = accumulate ? out[c] + s : s;
}

// Threshold gradient: straight-through part -(theta/eps) * (sum over window entries of dz), plus the
// dead-feature part (lambda1/B) n * #(pre < theta); times theta when the parameter is tau = log(theta).
__global__ __launch_bounds__(256) void dtheta_final_kernel(const float* __restrict__ part_win,
                                                           const float* __restrict__ part_below, int nparts,
                                                           int ncols, const float* __restrict__ theta_param,
                                                           bool log_threshold, const float* __restrict__ norms,
                                                           float inv_eps, float lam1_over_b,
                                                           float* __restrict__ out, PartsSwitch sw) {
  const int c = blockIdx.x * 256 + threadIdx.x;
  if (c >= ncols) return;
  if (sw.flags && lists_backward_selected(sw.flags, sw.kcap)) nparts = sw.nparts_lists;
  float w = 0.f, nb = 0.f;
  for (int r = 0; r < nparts; ++r) w += part_win[(size_t)r * ncols + c];
  if (lam1_over_b != 0.f)
    for (int r = 0; r < nparts; ++r) nb += part_below[(size_t)r * ncols + c];
  const float th = threshold_value(theta_param[c], log_threshold);
  float g = (w == 0.f) ? 0.f : w * -(th * inv_eps);   // empty window: exactly 0, also for theta = inf
  if (lam1_over_b != 0.f) g += lam1_over_b * norms[c] * nb;
  out[c] = log_threshold ? g * th : g;
}

// ---- straight-through reductions over the buffer that holds dz where a feature
// is active or in the threshold window, and the dead-feature gradient elsewhere
// below the threshold: column partials of dz over the window (-> dtheta), of the
// final dpre (-> db_enc) and of the below-threshold count; entries that are in the
// window but inactive are rewritten to their dpre value (dead-feature gradient or 0),
// so the buffer becomes dpre.  With a row scale (int8 inputs) dpre rows are also
// multiplied by it, because the encoder-weight gradient contracts them with the
// integer codes.
template <typename T>
__global__ __launch_bounds__(256) void ste_reduce_kernel(Dims D, T* __restrict__ dpre,
                                                         const uint8_t* __restrict__ cls,
                                                         const float* __restrict__ row_scale,
                                                         const float* __restrict__ norms, float lam1_over_b,
                                                         float* __restrict__ part_theta,
                                                         float* __restrict__ part_benc,
                                                         float* __restrict__ part_below,
                                                         const int32_t* __restrict__ only_if_lists, int kcap) {
  if (only_if_lists && !lists_backward_selected(only_if_lists, kcap)) return;
  const int rb = blockIdx.x, l = blockIdx.y;
  const int r0 = rb * LOSS_ROWS_PER_BLOCK, r1 = min(D.B, r0 + LOSS_ROWS_PER_BLOCK);
  const bool dead = lam1_over_b != 0.f;
  for (int c = threadIdx.x * 4; c < D.F; c += 1024) {
    float st[4] = {0.f, 0.f, 0.f, 0.f}, sb[4] = {0.f, 0.f, 0.f, 0.f}, nb[4] = {0.f, 0.f, 0.f, 0.f};
    float dg[4] = {0.f, 0.f, 0.f, 0.f};
    if (dead) {
      const float4 n4 = *reinterpret_cast<const float4*>(norms + (size_t)l * D.F + c);
      dg[0] = -lam1_over_b * n4.x; dg[1] = -lam1_over_b * n4.y; dg[2] = -lam1_over_b * n4.z; dg[3] = -lam1_over_b * n4.w;
    }
    for (int r = r0; r < r1; ++r) {
      const size_t o = ((size_t)l * D.B + r) * D.F + c;
      uint32_t c4 = *reinterpret_cast<const uint32_t*>(cls + o);
      if (!dead) c4 &= 0x03030303u;       // without the dead-feature term only active / window entries matter
      if (!c4) continue;
      const float4 g4 = Elem<T>::load4(dpre + o);
      float g[4] = {g4.x, g4.y, g4.z, g4.w};
      bool rewrite = row_scale != nullptr;
      const float s = row_scale ? row_scale[(size_t)l * D.B + r] : 1.0f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t ci = (c4 >> (8 * i)) & 7u;
        if (ci & CLS_WINDOW) st[i] += g[i];
        if (ci & CLS_BELOW) nb[i] += 1.0f;
        if (!(ci & CLS_ACTIVE) && (ci & CLS_WINDOW)) {   // held dz for the threshold gradient only
          g[i] = (ci & CLS_BELOW) ? dg[i] : 0.f;
          rewrite = true;
        }
        if (ci) {
          sb[i] += g[i];
          g[i] *= s;
        }
      }
      if (rewrite) Elem<T>::store4(dpre + o, make_float4(g[0], g[1], g[2], g[3]));
    }
    const size_t po = ((size_t)rb * D.L + l) * D.F + c;
    *reinterpret_cast<float4*>(part_theta + po) = make_float4(st[0], st[1], st[2], st[3]);
    *reinterpret_cast<float4*>(part_benc + po) = make_float4(sb[0], sb[1], sb[2], sb[3]);
    if (dead) *reinterpret_cast<float4*>(part_below + po) = make_float4(nb[0], nb[1], nb[2], nb[3]);
  }
}

// ---- Adam (App. C Table 1), 4 elements per lane --------------------------------
template <typename T, bool MASTER>
__global__ __launch_bounds__(256) void adam_kernel(size_t n4, T* __restrict__ p, const T* __restrict__ g,
                                                   float* __restrict__ m, float* __restrict__ v,
                                                   float* __restrict__ master, AdamScalars a) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
    const size_t o = i * 4;
    const float4 g4 = Elem<T>::load4(g + o);
    float4 m4 = *reinterpret_cast<const float4*>(m + o);
    float4 v4 = *reinterpret_cast<const float4*>(v + o);
    float4 p4 = MASTER ? *reinterpret_cast<const float4*>(master + o) : Elem<T>::load4(p + o);
    const float gg[4] = {g4.x, g4.y, g4.z, g4.w};
    float mm[4] = {m4.x, m4.y, m4.z, m4.w}, vv[4] = {v4.x, v4.y, v4.z, v4.w}, pp[4] = {p4.x, p4.y, p4.z, p4.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) adam_element(pp[k], mm[k], vv[k], gg[k], a);
    *reinterpret_cast<float4*>(m + o) = make_float4(mm[0], mm[1], mm[2], mm[3]);
    *reinterpret_cast<float4*>(v + o) = make_float4(vv[0], vv[1], vv[2], vv[3]);
    const float4 pn = make_float4(pp[0], pp[1], pp[2], pp[3]);
    if (MASTER) *reinterpret_cast<float4*>(master + o) = pn;
    Elem<T>::store4(p + o, pn);
  }
}

// ---- TopK activation: the k largest of a row's F fp32 pre-activations ----------------
// One workgroup per (layer, token) row.  A radix select over the order-preserving integer image
// of the floats finds the k-th largest value in four 8-bit passes (LDS histograms); a last pass
// writes z and the class bytes.  Entries equal to the k-th value are taken in index order until
// k entries are selected; that ordered count runs only for rows that have such ties to break.
#ifndef TOPK_HIST_COPIES
#define TOPK_HIST_COPIES 4
#endif
__device__ __forceinline__ uint32_t order_key(float x) {
  const uint32_t u = __float_as_uint(x);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);     // larger float <=> larger key (NaN sorts by its bits)
}

// NV4 > 0: the row (F <= 1024 * NV4) is held in registers, NV4 float4 per lane, and read from memory once;
// NV4 = 0: any F, every pass re-reads the row (it stays in the L2).
template <typename T, int NV4>
__global__ __launch_bounds__(256) void topk_select_kernel(Dims D, const float* __restrict__ pre32, int k,
                                                          T* __restrict__ z, uint8_t* __restrict__ cls,
                                                          int32_t* __restrict__ l0) {
  // (TOPK_HIST_COPIES histograms, one per lane residue: pre-activations share a few exponents, so most keys of the
  //  first pass fall into a handful of bins and atomics on one LDS word serialise)
  __shared__ int hist[TOPK_HIST_COPIES][256];
  __shared__ int sh_bin, sh_rem, scan[256], wtot[4];
  const int tid = threadIdx.x;
  const size_t row = blockIdx.x;
  const float* pr = pre32 + row * D.F;
  const int F4 = D.F / 4;
  const int rounds = NV4 > 0 ? NV4 : (F4 + 255) / 256;
  float4 held[NV4 > 0 ? NV4 : 1];
  if (NV4 > 0) {
#pragma unroll
    for (int j = 0; j < NV4; ++j) {
      const int q = tid + 256 * j;
      // padding sorts below every float (no float maps to key 0), so it is never selected
      held[j] = q < F4 ? *reinterpret_cast<const float4*>(pr + 4 * q) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
  auto value4 = [&](int j) -> float4 {        // the lane's j-th float4 (index 4 * (tid + 256 j)); in range only
    if (NV4 > 0) return held[j];
    return *reinterpret_cast<const float4*>(pr + 4 * (tid + 256 * j));
  };
  auto key4 = [&](int j, uint32_t (&key)[4]) {
    const int q = tid + 256 * j;
    if (q < F4) {
      const float4 v = value4(j);
      key[0] = order_key(v.x); key[1] = order_key(v.y); key[2] = order_key(v.z); key[3] = order_key(v.w);
    } else {
      key[0] = key[1] = key[2] = key[3] = 0u;
    }
  };

  uint32_t prefix = 0;
  int remaining = k;            // entries still to take among those whose key matches the prefix so far
  if (k > 0 && k < D.F) {
    for (int shift = 24; shift >= 0; shift -= 8) {
#pragma unroll
      for (int c = 0; c < TOPK_HIST_COPIES; ++c) hist[c][tid] = 0;
      __syncthreads();
      const uint32_t himask = shift == 24 ? 0u : (0xffffffffu << (shift + 8));
#pragma unroll NV4 > 0 ? NV4 : 1
      for (int j = 0; j < rounds; ++j) {
        uint32_t key[4];
        key4(j, key);
        if (tid + 256 * j < F4) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if ((key[i] & himask) == prefix) atomicAdd(&hist[tid & (TOPK_HIST_COPIES - 1)][(key[i] >> shift) & 255u], 1);
        }
      }
      __syncthreads();
      // the bin that holds the `remaining`-th largest entry: suffix sums over the 256 bins (lane = bin),
      // wave scans plus the totals of the higher waves
      {
        int h = 0;
#pragma unroll
        for (int c = 0; c < TOPK_HIST_COPIES; ++c) h += hist[c][tid];
        const int lane = tid & 63, wv = tid >> 6;
        int sfx = h;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const int u = __shfl_down(sfx, off, 64);
          if (lane + off < 64) sfx += u;
        }
        if (lane == 0) wtot[wv] = sfx;
        __syncthreads();
        for (int w2 = wv + 1; w2 < 4; ++w2) sfx += wtot[w2];
        const int above = sfx - h;                  // entries in higher bins
        if (above < remaining && remaining <= sfx) { sh_bin = tid; sh_rem = remaining - above; }
      }
      __syncthreads();
      prefix |= (uint32_t)sh_bin << shift;
      remaining = sh_rem;
      __syncthreads();
    }
  }
  // prefix = key of the k-th largest value; `remaining` of the entries equal to it are selected
  const bool all = k >= D.F, none = k <= 0;
  int eq_total = 0;
  if (!all && !none) {
    int c = 0;
#pragma unroll NV4 > 0 ? NV4 : 1
    for (int j = 0; j < rounds; ++j) {
      uint32_t key[4];
      key4(j, key);
      if (tid + 256 * j < F4) c += (key[0] == prefix) + (key[1] == prefix) + (key[2] == prefix) + (key[3] == prefix);
    }
    scan[tid] = c;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
      if (tid < off) scan[tid] += scan[tid + off];
      __syncthreads();
    }
    eq_total = scan[0];
    __syncthreads();
  }
  const bool ties = !all && !none && eq_total > remaining;     // uniform over the workgroup
  int taken_before = 0;                                         // equal entries in earlier float4 rounds
#pragma unroll NV4 > 0 ? NV4 : 1
  for (int j = 0; j < rounds; ++j) {
    const int q = tid + 256 * j;
    const bool in = q < F4;
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (in) v = value4(j);
    const float vv[4] = {v.x, v.y, v.z, v.w};
    uint32_t key[4];
    key4(j, key);
    int rank0 = 0;                                              // equal entries before this lane's first one
    if (ties) {
      const int c = in ? (key[0] == prefix) + (key[1] == prefix) + (key[2] == prefix) + (key[3] == prefix) : 0;
      scan[tid] = c;
      __syncthreads();
      for (int off = 1; off < 256; off <<= 1) {                 // inclusive scan over the 256 lanes
        const int u = tid >= off ? scan[tid - off] : 0;
        __syncthreads();
        scan[tid] += u;
        __syncthreads();
      }
      rank0 = taken_before + scan[tid] - c;
      taken_before += scan[255];
      __syncthreads();
    }
    if (in) {
      float zz[4];
      uint32_t c4 = 0;
      int r = rank0;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        bool sel = all || (!none && key[i] > prefix);
        if (!all && !none && key[i] == prefix) {
          sel = !ties || r < remaining;
          ++r;
        }
        zz[i] = sel ? vv[i] : 0.f;
        c4 |= (sel ? (uint32_t)CLS_ACTIVE : 0u) << (8 * i);
      }
      Elem<T>::store4(z + row * D.F + 4 * q, make_float4(zz[0], zz[1], zz[2], zz[3]));
      *reinterpret_cast<uint32_t*>(cls + row * D.F + 4 * q) = c4;
    }
  }
  // every row selects the same number of entries, so one row per layer books the whole layer
  // (a per-row add would send all B*L atomics of the launch to 16 addresses, one after the other)
  if (tid == 0 && l0 && row % D.B == 0) atomicAdd(l0 + (int)(row / D.B), D.B * (all ? D.F : (none ? 0 : k)));
}

// ---- activation normalisation (Sec. 3.1): the factor of a layer is the mean L2 norm of its
// token vectors over the first batches.  Stage 1: grid = (row blocks, L), one wave per row, each
// block leaves the sum of its rows' norms; stage 2 adds the blocks of a layer, in order, to the
// running sum.  int8 rows: the norm of the codes times |row scale|.
template <typename T, bool INT8>
__global__ __launch_bounds__(256) void row_norm_sum_kernel(Dims D, const void* __restrict__ av,
                                                           const float* __restrict__ a_scale,
                                                           double* __restrict__ part) {
  const int rb = blockIdx.x, l = blockIdx.y, lane = threadIdx.x & 63;
  const int r0 = rb * LOSS_ROWS_PER_BLOCK, r1 = min(D.B, r0 + LOSS_ROWS_PER_BLOCK);
  double s = 0.0;   // the same value in every lane of a wave
  for (int r = r0 + (threadIdx.x >> 6); r < r1; r += 4) {
    const size_t o = ((size_t)l * D.B + r) * D.d;
    float acc = 0.f;
    for (int j = lane * 4; j < D.d; j += 256) {
      float4 v;
      if (INT8) {
        const uint32_t q = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const int8_t*>(av) + o + j);
        v = make_float4((float)(int8_t)q, (float)(int8_t)(q >> 8), (float)(int8_t)(q >> 16), (float)(int8_t)(q >> 24));
      } else {
        v = Elem<T>::load4(reinterpret_cast<const T*>(av) + o + j);
      }
      acc += (v.x * v.x + v.y * v.y) + (v.z * v.z + v.w * v.w);
    }
    float n = sqrtf(wave_sum(acc));
    if (INT8) n *= fabsf(a_scale[(size_t)l * D.B + r]);
    s += (double)n;
  }
  __shared__ double sh[4];
  if (lane == 0) sh[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) part[(size_t)l * gridDim.x + rb] = (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

__global__ void norm_sum_final_kernel(int L, int nrb, const double* __restrict__ part, double* __restrict__ norm_sum) {
  const int l = blockIdx.x * blockDim.x + threadIdx.x;
  if (l >= L) return;
  double s = 0.0;
  for (int i = 0; i < nrb; ++i) s += part[(size_t)l * nrb + i];
  norm_sum[l] += s;
}

// 1 / c[l] = n_tokens / norm_sum[l]; a layer that summed to zero has no scale and keeps factor 1
__device__ __forceinline__ float inv_norm_factor(const double* norm_sum, int l, double n_tokens) {
  const double s = norm_sum[l];
  return s > 0.0 ? (float)(n_tokens / s) : 1.0f;
}

// int8 rows: the division folds into the dequantisation scale, the codes stay as they are
__global__ void normalise_scale_kernel(Dims D, const double* __restrict__ norm_sum, double n_tokens,
                                       const float* __restrict__ scale_in, float* __restrict__ scale_out) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)D.L * D.B) return;
  scale_out[i] = scale_in[i] * inv_norm_factor(norm_sum, (int)(i / D.B), n_tokens);
}

// native rows: a_out = a_in / c[l] (a_out may be a_in); grid = (chunks of a layer, L)
template <typename T>
__global__ __launch_bounds__(256) void normalise_rows_kernel(Dims D, const double* __restrict__ norm_sum,
                                                             double n_tokens, const T* a_in, T* a_out) {
  const int l = blockIdx.y;
  const float k = inv_norm_factor(norm_sum, l, n_tokens);
  const size_t n4 = (size_t)D.B * D.d / 4, base = (size_t)l * D.B * D.d;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += (size_t)gridDim.x * 256) {
    const float4 v = Elem<T>::load4(a_in + base + 4 * i);
    Elem<T>::store4(a_out + base + 4 * i, make_float4(k * v.x, k * v.y, k * v.z, k * v.w));
  }
}

// Scratch of the entry point that allocates nothing: the per-block partial sums of the activation-norm
// reduction, held in the library's own device memory instead of a caller workspace.  One copy per GPU
// for the life of the process (512 KB); every call on a GPU uses that GPU's copy.
static __device__ __align__(256) double scratch[STATIC_SCRATCH_DOUBLES];
constexpr int MAX_DEVICES = 64;
double* g_scratch_ptr[MAX_DEVICES] = {};   // device address of `scratch` on each GPU, resolved once

inline int grid_for(size_t n, int per_block, int cap) {
  size_t b = (n + per_block - 1) / per_block;
  if (b < 1) b = 1;
  if (b > (size_t)cap) b = cap;
  return (int)b;
}

}  // namespace

hipError_t launch_zero_i32(hipStream_t s, int32_t* p, int n) {
  hipLaunchKernelGGL(zero_i32_kernel, dim3((n + 255) / 256), dim3(256), 0, s, p, n);
  return hipGetLastError();
}

hipError_t launch_topk_select(hipStream_t s, bool bf16, Dims D, const float* pre32, int k, void* z, uint8_t* cls,
                              int32_t* l0) {
  const dim3 grid((unsigned)((size_t)D.L * D.B));
#define CLT_TOPK(T, NV4) \
  hipLaunchKernelGGL((topk_select_kernel<T, NV4>), grid, dim3(256), 0, s, D, pre32, k, (T*)z, cls, l0)
  const int nv4 = D.F <= 2048 ? 2 : (D.F <= 8192 ? 8 : 0);     // registers for rows up to 8192 features
  if (bf16) { if (nv4 == 2) CLT_TOPK(bf16_t, 2); else if (nv4 == 8) CLT_TOPK(bf16_t, 8); else CLT_TOPK(bf16_t, 0); }
  else { if (nv4 == 2) CLT_TOPK(float, 2); else if (nv4 == 8) CLT_TOPK(float, 8); else CLT_TOPK(float, 0); }
#undef CLT_TOPK
  return hipGetLastError();
}

hipError_t launch_decoder_norms(hipStream_t s, bool bf16, Dims D, const void* W_dec, float* norms) {
  const long rows = (long)D.L * D.F;
  const dim3 grid((unsigned)((rows + 3) / 4));
  if (bf16)
    hipLaunchKernelGGL((decoder_norms_kernel<bf16_t>), grid, dim3(256), 0, s, D, (const bf16_t*)W_dec, norms);
  else
    hipLaunchKernelGGL((decoder_norms_kernel<float>), grid, dim3(256), 0, s, D, (const float*)W_dec, norms);
  return hipGetLastError();
}

hipError_t launch_norms_from_partials(hipStream_t s, Dims D, const float* n2_part, float* norms, const int32_t* flags,
                                      int kcap) {
  const long rows = (long)D.L * D.F;
  hipLaunchKernelGGL(norms_from_partials_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0, s, D, n2_part, norms,
                     flags, kcap);
  return hipGetLastError();
}

hipError_t launch_loss_rec(hipStream_t s, bool bf16, bool int8_y, Dims D, const float* y_hat, const void* y,
                           const float* y_scale, void* d_yhat, double* loss_part, float* col_part) {
  const dim3 grid(row_blocks(D.B), D.L);
  if (!bf16)
    hipLaunchKernelGGL((loss_rec_kernel<float, false>), grid, dim3(256), 0, s, D, y_hat, y, y_scale, (float*)d_yhat,
                       loss_part, col_part);
  else if (int8_y)
    hipLaunchKernelGGL((loss_rec_kernel<bf16_t, true>), grid, dim3(256), 0, s, D, y_hat, y, y_scale,
                       (bf16_t*)d_yhat, loss_part, col_part);
  else
    hipLaunchKernelGGL((loss_rec_kernel<bf16_t, false>), grid, dim3(256), 0, s, D, y_hat, y, y_scale,
                       (bf16_t*)d_yhat, loss_part, col_part);
  return hipGetLastError();
}

hipError_t launch_loss_sparsity(hipStream_t s, bool bf16, Dims D, const void* z, const float* norms, float C,
                                double* loss_part, float* col_part, const void* pre, const float* theta,
                                bool log_threshold, double* dead_part, float* dead_col_part) {
  const dim3 grid(row_blocks(D.B), D.L);
#define CLT_LSP(T, DEAD)                                                                                      \
  hipLaunchKernelGGL((loss_sparsity_kernel<T, DEAD>), grid, dim3(256), 0, s, D, (const T*)z, norms, C, loss_part, \
                     col_part, (const T*)pre, theta, log_threshold, dead_part, dead_col_part)
  if (bf16) { if (pre) CLT_LSP(bf16_t, true); else CLT_LSP(bf16_t, false); }
  else { if (pre) CLT_LSP(float, true); else CLT_LSP(float, false); }
#undef CLT_LSP
  return hipGetLastError();
}

hipError_t launch_loss_final(hipStream_t s, const double* part_rec, int n_rec, const double* part_sp, int n_sp,
                             const double* part_dead_or_null, float inv_B, float lambda0, float lambda1,
                             float* loss_dev) {
  hipLaunchKernelGGL(loss_final_kernel, dim3(1), dim3(256), 0, s, part_rec, n_rec, part_sp, n_sp, part_dead_or_null,
                     inv_B, lambda0, lambda1, loss_dev);
  return hipGetLastError();
}

hipError_t launch_col_reduce(hipStream_t s, const float* part, int nparts, int ncols, float alpha,
                             const float* theta_or_null, float inv_eps, float* out, bool accumulate, PartsSwitch sw) {
  hipLaunchKernelGGL(col_reduce_kernel, dim3((ncols + 255) / 256), dim3(256), 0, s, part, nparts, ncols, alpha,
                     theta_or_null, inv_eps, out, accumulate, sw);
  return hipGetLastError();
}

hipError_t launch_dtheta_final(hipStream_t s, const float* part_win, const float* part_below, int nparts, int ncols,
                               const float* theta_param, bool log_threshold, const float* norms, float inv_eps,
                               float lam1_over_b, float* out, PartsSwitch sw) {
  hipLaunchKernelGGL(dtheta_final_kernel, dim3((ncols + 255) / 256), dim3(256), 0, s, part_win, part_below, nparts,
                     ncols, theta_param, log_threshold, norms, inv_eps, lam1_over_b, out, sw);
  return hipGetLastError();
}

hipError_t launch_ste_reduce(hipStream_t s, bool bf16, Dims D, void* dpre, const uint8_t* cls,
                             const float* row_scale_or_null, const float* norms, float lam1_over_b,
                             float* part_theta, float* part_benc, float* part_below,
                             const int32_t* only_if_lists, int kcap) {
  const dim3 grid(row_blocks(D.B), D.L);
  if (bf16)
    hipLaunchKernelGGL((ste_reduce_kernel<bf16_t>), grid, dim3(256), 0, s, D, (bf16_t*)dpre, cls, row_scale_or_null,
                       norms, lam1_over_b, part_theta, part_benc, part_below, only_if_lists, kcap);
  else
    hipLaunchKernelGGL((ste_reduce_kernel<float>), grid, dim3(256), 0, s, D, (float*)dpre, cls, row_scale_or_null,
                       norms, lam1_over_b, part_theta, part_benc, part_below, only_if_lists, kcap);
  return hipGetLastError();
}

hipError_t launch_adam_matrix(hipStream_t s, bool bf16, size_t n, void* p, const void* g, float* m, float* v,
                              float* master, AdamScalars a) {
  const size_t n4 = n / 4;   // matrices have a multiple of 64 elements (d, F multiples of 8)
  const dim3 grid(grid_for(n4, 256, 256 * 32));
  if (bf16) {
    if (master)
      hipLaunchKernelGGL((adam_kernel<bf16_t, true>), grid, dim3(256), 0, s, n4, (bf16_t*)p, (const bf16_t*)g, m, v,
                         master, a);
    else
      hipLaunchKernelGGL((adam_kernel<bf16_t, false>), grid, dim3(256), 0, s, n4, (bf16_t*)p, (const bf16_t*)g, m, v,
                         master, a);
  } else {
    if (master)
      hipLaunchKernelGGL((adam_kernel<float, true>), grid, dim3(256), 0, s, n4, (float*)p, (const float*)g, m, v,
                         master, a);
    else
      hipLaunchKernelGGL((adam_kernel<float, false>), grid, dim3(256), 0, s, n4, (float*)p, (const float*)g, m, v,
                         master, a);
  }
  return hipGetLastError();
}

hipError_t launch_adam_vector(hipStream_t s, size_t n, float* p, const float* g, float* m, float* v, AdamScalars a) {
  const size_t n4 = n / 4;   // vectors have L*F or L*d elements, multiples of 8
  hipLaunchKernelGGL((adam_kernel<float, false>), dim3(grid_for(n4, 256, 256 * 32)), dim3(256), 0, s, n4, p, g, m, v,
                     (float*)nullptr, a);
  return hipGetLastError();
}

hipError_t launch_norm_accumulate(hipStream_t s, bool bf16, bool int8_a, Dims D, const void* a, const float* a_scale,
                                  double* part, double* norm_sum) {
  const dim3 grid(row_blocks(D.B), D.L);
  if (!bf16)
    hipLaunchKernelGGL((row_norm_sum_kernel<float, false>), grid, dim3(256), 0, s, D, a, a_scale, part);
  else if (int8_a)
    hipLaunchKernelGGL((row_norm_sum_kernel<bf16_t, true>), grid, dim3(256), 0, s, D, a, a_scale, part);
  else
    hipLaunchKernelGGL((row_norm_sum_kernel<bf16_t, false>), grid, dim3(256), 0, s, D, a, a_scale, part);
  hipLaunchKernelGGL(norm_sum_final_kernel, dim3((D.L + 63) / 64), dim3(64), 0, s, D.L, (int)grid.x, part, norm_sum);
  return hipGetLastError();
}

// Device address of this GPU's `scratch` array (the array's name is only a host-side handle for
// hipGetSymbolAddress; kernels get the resolved pointer as an argument).  Resolved once per device,
// with that device current.
hipError_t static_scratch(double** ptr) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  double* p = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (!p) {
    e = hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    __atomic_store_n(&g_scratch_ptr[dev], p, __ATOMIC_RELEASE);   // every thread resolves the same address
  }
  *ptr = p;
  return hipSuccess;
}

hipError_t launch_normalise(hipStream_t s, bool bf16, bool int8_a, Dims D, const double* norm_sum, double n_tokens,
                            const void* a_in, const float* scale_in, void* a_out, float* scale_out) {
  if (int8_a) {
    const size_t n = (size_t)D.L * D.B;
    hipLaunchKernelGGL(normalise_scale_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, D, norm_sum,
                       n_tokens, scale_in, scale_out);
  } else {
    const dim3 grid(grid_for((size_t)D.B * D.d / 4, 256 * 4, 2048), D.L);
    if (bf16)
      hipLaunchKernelGGL((normalise_rows_kernel<bf16_t>), grid, dim3(256), 0, s, D, norm_sum, n_tokens,
                         (const bf16_t*)a_in, (bf16_t*)a_out);
    else
      hipLaunchKernelGGL((normalise_rows_kernel<float>), grid, dim3(256), 0, s, D, norm_sum, n_tokens,
                         (const float*)a_in, (float*)a_out);
  }
  return hipGetLastError();
}

}  // namespace clt
