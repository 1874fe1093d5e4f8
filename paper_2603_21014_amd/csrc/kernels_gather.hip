// Active-feature gather decode (paper Sec. 3.2 "Sparse Decode"): once training
// has pushed the activations into the sparse regime, each token looks up only
// the decoder rows of its active features and sums them, O(k d) instead of the
// dense O(F d) contraction.  Three kernels:
//   decide   reads the per-layer active counts of the encoder epilogue and sets
//            the device-side switch (no host round trip);
//   compact  turns every (layer, token) row of z into an ordered list of
//            (feature, value) pairs;
//   gather   one workgroup per (token, target layer): walks the sources
//            l <= l' and their lists, streams the 2d-byte decoder rows with
//            16-byte loads per lane and accumulates in fp32 registers.
// The row order inside a list and the order of the sources are fixed, so the
// result is bitwise reproducible (no atomics).  The path is HBM/L2-bound:
// B * k * P * d * sizeof(T) bytes of decoder rows per call.
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
// pass, positions come from a wave-wide exclusive scan of the per-lane counts.
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
  int base = 0;
  for (int f0 = 0; f0 < D.F; f0 += 256) {
    const int f = f0 + lane * 4;
    uint32_t c4 = 0;
    float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (f < D.F) {
      c4 = *reinterpret_cast<const uint32_t*>(cr + f) & 0x01010101u;   // active bits
      if (c4) z4 = Elem<T>::load4(zr + f);
    }
    const int n = __popc(c4);
    int incl = n;                                   // inclusive scan over the 64 lanes
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int v = __shfl_up(incl, off, 64);
      if (lane >= off) incl += v;
    }
    int pos = base + incl - n;
    const float zz[4] = {z4.x, z4.y, z4.z, z4.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if ((c4 >> (8 * i)) & 1u) {
        if (pos < g.kcap) { oi[pos] = f + i; ov[pos] = zz[i]; }
        ++pos;
      }
    }
    base += __shfl(incl, 63, 64);
  }
  if (lane == 0) {
    g.counts[row] = base;
    atomicMax(flags + 1, base);
  }
}

// Accumulates 8 columns per lane; d is walked in passes of 2048 columns.
template <typename T>
__global__ __launch_bounds__(256) void gather_decode_kernel(Dims D, GatherLists g, const T* __restrict__ W_dec,
                                                            const float* __restrict__ b_dec,
                                                            float* __restrict__ y_hat, int32_t* __restrict__ flags) {
  if (flags[0] == 0 || flags[1] > g.kcap) return;
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

}  // namespace clt
