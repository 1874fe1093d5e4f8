// fp32 path of the five CLT contractions: fp32 storage, fp32 FMA accumulate
// (no reduced-precision matrix mode), LDS-staged 64x64x16 tiles, one 4x4
// micro-tile per lane.  This is the exact-arithmetic path used by small fp32
// configurations; the bf16 MFMA path lives in kernels_gemm_bf16.hip.
#include "common.h"
#include "gemm_policies.h"

namespace clt {
namespace {

constexpr int FTM = 64, FTN = 64, FTK = 16;

template <class P>
__global__ __launch_bounds__(256) void gemm_f32_kernel(P p, TileGrid tg) {
  __shared__ float As[FTK][FTM + 4];
  __shared__ float Bs[FTK][FTN + 4];
  int gorder, tm, tn;
  if (!tg.decode(blockIdx.x, gorder, tm, tn) || p.skip()) return;
  const typename P::GInfo gi = p.ginfo(gorder);
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;
  const int m0 = tm * FTM, n0 = tn * FTN;
  const int M = p.M, N = p.N, kseg = p.kseg, nseg = p.nseg(gi);

  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  for (int s = 0; s < nseg; ++s) {
    const float* A = p.a_seg(gi, s);
    const float* Bm = p.b_seg(gi, s);
    for (int k0 = 0; k0 < kseg; k0 += FTK) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int idx = t + 256 * i;
        int m, k;
        if (P::A_KC) { m = idx >> 4; k = idx & 15; } else { k = idx >> 6; m = idx & 63; }
        float v = 0.f;
        if (m0 + m < M && k0 + k < kseg)
          v = P::A_KC ? A[(size_t)(m0 + m) * p.lda + k0 + k] : A[(size_t)(k0 + k) * p.lda + m0 + m];
        As[k][m] = v;
        int n;
        if (P::B_KC) { n = idx >> 4; k = idx & 15; } else { k = idx >> 6; n = idx & 63; }
        v = 0.f;
        if (n0 + n < N && k0 + k < kseg)
          v = P::B_KC ? Bm[(size_t)(n0 + n) * p.ldb + k0 + k] : Bm[(size_t)(k0 + k) * p.ldb + n0 + n];
        Bs[k][n] = v;
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < FTK; ++k) {
        const float4 a = *reinterpret_cast<const float4*>(&As[k][ty * 4]);
        const float4 b = *reinterpret_cast<const float4*>(&Bs[k][tx * 4]);
        const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
      }
      __syncthreads();
    }
  }

  typename P::Epi est;
  const int col = n0 + tx * 4;
  p.epi_begin(est, gi, col, col < N, m0);
  if (col < N) {
    typename P::EpiRegs er[4];
    EpiPos pos{m0, n0, 0, tx * 4};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      pos.rl = ty * 4 + i;
      if (pos.row() < M) p.epi_load(er[i], gi, pos);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      pos.rl = ty * 4 + i;
      if (pos.row() < M) p.epi4(est, gi, pos, make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]), er[i]);
    }
  }
  p.epi_end(est, gi, nullptr);
}

template <class P>
hipError_t launch(hipStream_t s, const P& p, int G) {
  const TileGrid tg = TileGrid::make(G, p.M, p.N, FTM, FTN);
  hipLaunchKernelGGL((gemm_f32_kernel<P>), dim3(tg.num_wg()), dim3(256), 0, s, p, tg);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_enc_f32(hipStream_t s, Dims D, const EncArgs& a) {
  EncPolicy<float> p{D, D.B, D.F, D.d, D.d, D.F,
                     (const float*)a.x, (const float*)a.W_enc, a.b_enc, a.theta, nullptr,
                     0.5f * a.ste_eps, (float*)a.z, (float*)a.pre, a.cls, a.l0, a.log_threshold, a.pre32};
  return launch(s, p, D.L);
}
hipError_t launch_dec_f32(hipStream_t s, Dims D, const DecArgs& a) {
  DecPolicy<float> p{D, D.B, D.d, D.F, D.F, D.d, (const float*)a.z, (const float*)a.W_dec, a.b_dec, a.y_hat, a.skip_flags, a.kcap, nullptr};
  return launch(s, p, D.L);
}
hipError_t launch_dz_f32(hipStream_t s, Dims D, const DzArgs& a) {
  DzPolicy<float> p{D, D.B, D.F, D.d, D.d, D.d,
                    (const float*)a.d_yhat, (const float*)a.W_dec, (const float*)a.z, a.cls, a.norms,
                    a.lam_c_over_b, a.C, (float*)a.dpre, a.lam1_over_b, a.skip_flags, a.kcap,
                    nullptr, nullptr, nullptr, nullptr};
  return launch(s, p, D.L);
}
template <bool ADAM>
static hipError_t launch_dwdec_mode(hipStream_t s, Dims D, const DWdecArgs& a) {
  DWdecPolicy<float, ADAM> p{D, D.F, D.d, D.B, D.F, D.d,
                             (const float*)a.z, (const float*)a.d_yhat, (float*)a.W_dec, a.G, a.norms,
                             (float*)a.dW_dec, AdamFuse{a.fuse.m, a.fuse.v, a.fuse.master, a.fuse.a}, a.skip_flags, a.kcap, 0, nullptr};
  // one launch per source layer, like the bf16 path
  for (int l = 0; l < D.L; ++l) {
    p.p0 = packed_index(l, l, D.L);
    const hipError_t e = launch(s, p, D.L - l);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}
hipError_t launch_dwdec_f32(hipStream_t s, Dims D, const DWdecArgs& a) {
  return a.fuse.m ? launch_dwdec_mode<true>(s, D, a) : launch_dwdec_mode<false>(s, D, a);
}
template <bool ADAM>
static hipError_t launch_dwenc_mode(hipStream_t s, Dims D, const DWencArgs& a) {
  DWencPolicy<float, ADAM> p{D, D.d, D.F, D.B, D.d, D.F, (const float*)a.x, (const float*)a.dpre, (float*)a.dW_enc,
                             (float*)a.W_enc, AdamFuse{a.fuse.m, a.fuse.v, a.fuse.master, a.fuse.a}};
  return launch(s, p, D.L);
}
hipError_t launch_dwenc_f32(hipStream_t s, Dims D, const DWencArgs& a) {
  return a.fuse.m ? launch_dwenc_mode<true>(s, D, a) : launch_dwenc_mode<false>(s, D, a);
}

}  // namespace clt
