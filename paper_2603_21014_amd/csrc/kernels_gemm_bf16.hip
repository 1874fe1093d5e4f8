// bf16 MFMA path of the five CLT contractions on gfx950 (CDNA4).
//
// One workgroup = 4 wavefronts (one per SIMD) computes a 256x256 output tile;
// each wavefront owns a 128x128 quadrant as 4x4 v_mfma_f32_32x32x16_bf16
// accumulators (256 accumulator registers per lane).  K advances in steps of
// 64 through two LDS stages (2 x 64 KB): while the MFMAs of step t run from one
// stage, the tile of step t+1 goes registers -> LDS into the other stage and
// the tile of step t+2 is fetched from HBM into registers.
//
// Both operands sit in LDS as [row][64 k] bf16 with the 16-byte chunk index
// xor-swizzled by the row, so that the MFMA fragment reads (one row per lane,
// 8 consecutive k) and the staging writes are bank-conflict free.  An operand
// whose memory layout is contiguous along K is copied as is; one that is
// strided along K (the row-major right-hand sides, and both operands of the
// weight-gradient GEMMs) is fetched as 8(k) x 8 blocks and transposed in
// registers with byte permutes before the LDS write, so no transposed copy of
// any tensor is ever materialised in HBM.
//
// The epilogue transposes accumulators through LDS so that every lane hands
// four consecutive columns of one row to the policy's fused epilogue, which
// then reads/writes global memory in 128-byte row segments.
#include "common.h"
#include "gemm_policies.h"

namespace clt {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
// native 16-byte register vector (HIP's uint4 is a class type; selects on it go through memory)
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int TM = 256, TN = 256, TK = 64;
constexpr int STAGE_ELEMS = 2 * 256 * TK;            // A tile + B tile, bf16 elements
constexpr int LDS_BYTES = 2 * STAGE_ELEMS * 2;       // two stages = 128 KB

// element offset of 16-byte chunk `c` (8 bf16) of tile row `row`
__device__ __forceinline__ int lds_off(int row, int c) {
  return row * TK + (((c ^ row ^ (row >> 3)) & 7) << 3);
}

__device__ __forceinline__ u32x4 ld16(const void* p) { return *reinterpret_cast<const u32x4*>(p); }

// int8 codes -> bf16 (exact: |q| <= 127 fits the 8-bit significand)
__device__ __forceinline__ uint32_t i8x2_to_bf16x2(int lo, int hi) {
  return (__float_as_uint((float)lo) >> 16) | (__float_as_uint((float)hi) & 0xffff0000u);
}
__device__ __forceinline__ u32x4 i8x8_to_bf16x8(u32x2 q) {
  u32x4 r;
  r[0] = i8x2_to_bf16x2((int)(int8_t)(q[0]), (int)(int8_t)(q[0] >> 8));
  r[1] = i8x2_to_bf16x2((int)(int8_t)(q[0] >> 16), (int)(int8_t)(q[0] >> 24));
  r[2] = i8x2_to_bf16x2((int)(int8_t)(q[1]), (int)(int8_t)(q[1] >> 8));
  r[3] = i8x2_to_bf16x2((int)(int8_t)(q[1] >> 16), (int)(int8_t)(q[1] >> 24));
  return r;
}
template <typename TE> __device__ __forceinline__ u32x4 load8(const TE* p);
template <> __device__ __forceinline__ u32x4 load8<bf16_t>(const bf16_t* p) { return ld16(p); }
template <> __device__ __forceinline__ u32x4 load8<int8_t>(const int8_t* p) {
  return i8x8_to_bf16x8(*reinterpret_cast<const u32x2*>(p));
}

// Fetch one 256(rows) x 64(k) operand tile into 8 x 16-byte registers per lane.
// KC: lane t takes chunk c = t%8 of rows t/8 + 32 i.  Otherwise lane t takes the
// 8(k) x 8(rows) block kb = t/32, nb = t%32.  Out-of-range chunks read as zero
// (the address is redirected to the tensor base, which is always readable).
template <bool KC, typename TE>
__device__ __forceinline__ void gload(u32x4 (&r)[8], const TE* base, int ld, int r0, int R, int k0, int kseg,
                                      int t) {
  const u32x4 zero = {0u, 0u, 0u, 0u};
  if (KC) {
    const int kk = k0 + ((t & 7) << 3);
    const bool kok = kk < kseg;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = r0 + (t >> 3) + 32 * i;
      const bool ok = kok && row < R;
      const u32x4 v = load8<TE>(base + (ok ? (size_t)row * ld + kk : (size_t)0));
      r[i] = ok ? v : zero;
    }
  } else {
    const int col = r0 + ((t & 31) << 3);
    const bool cok = col < R;
    const int kb = k0 + ((t >> 5) << 3);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const int k = kb + j;
      const bool ok = cok && k < kseg;
      const u32x4 v = load8<TE>(base + (ok ? (size_t)k * ld + col : (size_t)0));
      r[j] = ok ? v : zero;
    }
  }
}

template <bool KC>
__device__ __forceinline__ void sstore(bf16_t* lds, const u32x4 (&r)[8], int t) {
  if (KC) {
    const int c = t & 7;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = (t >> 3) + 32 * i;
      *reinterpret_cast<u32x4*>(lds + lds_off(row, c)) = r[i];
    }
  } else {
    const int nb = t & 31, kb = t >> 5;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
      u32x4 o;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t lo = r[2 * w][n >> 1], hi = r[2 * w + 1][n >> 1];
        o[w] = (n & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
      }
      *reinterpret_cast<u32x4*>(lds + lds_off(8 * nb + n, kb)) = o;
    }
  }
}

template <class P>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(P p, TileGrid tg) {
  extern __shared__ __align__(16) bf16_t smem[];
  int gorder, tm, tn;
  if (!tg.decode(blockIdx.x, gorder, tm, tn)) return;
  const typename P::GInfo gi = p.ginfo(gorder);
  typedef typename P::AType TA;

  const int t = threadIdx.x, lane = t & 63, w = t >> 6, wm = w >> 1, wn = w & 1;
  const int m0 = tm * TM, n0 = tn * TN;
  const int M = p.M, N = p.N, kseg = p.kseg, nseg = p.nseg(gi);
  const int nk = nseg * ((kseg + TK - 1) / TK);

  int ld_seg = 0, ld_k0 = 0;
  const TA* Aseg = p.a_seg(gi, 0);
  const bf16_t* Bseg = p.b_seg(gi, 0);
  u32x4 ra[8], rb[8];

  auto fetch = [&]() {
    gload<P::A_KC, TA>(ra, Aseg, p.lda, m0, M, ld_k0, kseg, t);
    gload<P::B_KC, bf16_t>(rb, Bseg, p.ldb, n0, N, ld_k0, kseg, t);
    ld_k0 += TK;
    if (ld_k0 >= kseg) {
      ld_k0 = 0;
      ++ld_seg;
      if (ld_seg < nseg) {
        Aseg = p.a_seg(gi, ld_seg);
        Bseg = p.b_seg(gi, ld_seg);
      }
    }
  };
  auto stage = [&](int st) {
    bf16_t* base = smem + st * STAGE_ELEMS;
    sstore<P::A_KC>(base, ra, t);
    sstore<P::B_KC>(base + 256 * TK, rb, t);
  };

  f32x16_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4 fa[2][4], fb[2][4];
  const int frow = lane & 31, fch = lane >> 5;
  auto frags = [&](int st, int kk, int buf) {
    const bf16_t* a = smem + st * STAGE_ELEMS;
    const bf16_t* b = a + 256 * TK;
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[buf][i] = ld16(a + lds_off(wm * 128 + i * 32 + frow, 2 * kk + fch));
#pragma unroll
    for (int j = 0; j < 4; ++j) fb[buf][j] = ld16(b + lds_off(wn * 128 + j * 32 + frow, 2 * kk + fch));
  };
  auto mfma = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fa[buf][i]),
                                                            __builtin_bit_cast(bf16x8_t, fb[buf][j]), acc[i][j], 0, 0,
                                                            0);
  };

  fetch();
  stage(0);
  if (nk > 1) fetch();
  __syncthreads();
  frags(0, 0, 0);
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) stage(cur ^ 1);
    if (kt + 2 < nk) fetch();
    frags(cur, 1, 1);
    mfma(0);
    frags(cur, 2, 0);
    mfma(1);
    frags(cur, 3, 1);
    mfma(0);
    __syncthreads();
    if (kt + 1 < nk) frags(cur ^ 1, 0, 0);
    mfma(1);
  }

  // ---- epilogue: accumulators -> LDS (wave-private 128x64 fp32) -> rows of 4 columns per lane
  __syncthreads();
  float* wl = reinterpret_cast<float*>(smem) + w * (128 * 64);
  typename P::Epi est;
  p.epi_begin(est);
#pragma unroll
  for (int jp = 0; jp < 4; jp += 2) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          wl[(i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3)) * 64 + jj * 32 + (lane & 31)] = acc[i][jp + jj][r];
    __syncthreads();
    const int c4 = (lane & 15) << 2;
    const int gcol = n0 + wn * 128 + jp * 32 + c4;
#pragma unroll 4
    for (int it = 0; it < 32; ++it) {
      const int row = it * 4 + (lane >> 4);
      const int grow = m0 + wm * 128 + row;
      const float4 v = *reinterpret_cast<const float4*>(wl + row * 64 + c4);
      if (grow < M && gcol < N) p.epi4(est, gi, grow, gcol, v);
    }
    __syncthreads();
  }
  p.epi_end(est, gi);
}

template <class P>
hipError_t launch(hipStream_t s, const P& p, int G) {
  const TileGrid tg = TileGrid::make(G, p.M, p.N, TM, TN);
  hipLaunchKernelGGL((gemm_bf16_kernel<P>), dim3(tg.num_wg()), dim3(256), LDS_BYTES, s, p, tg);
  return hipGetLastError();
}

template <class P>
hipError_t set_lds_attr() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<P>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
}

}  // namespace

hipError_t init_gemm_bf16() {
  hipError_t e;
  if ((e = set_lds_attr<EncPolicy<bf16_t>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<EncPolicy<bf16_t, int8_t>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DecPolicy<bf16_t>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DzPolicy<bf16_t>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DWdecPolicy<bf16_t>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DWencPolicy<bf16_t>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DWencPolicy<bf16_t, int8_t>>()) != hipSuccess) return e;
  return hipSuccess;
}

hipError_t launch_enc_bf16(hipStream_t s, Dims D, const EncArgs& a, bool int8_x) {
  if (int8_x) {
    EncPolicy<bf16_t, int8_t> p{D, D.B, D.F, D.d, D.d, D.F,
                                (const int8_t*)a.x, (const bf16_t*)a.W_enc, a.b_enc, a.theta, a.x_scale,
                                0.5f * a.ste_eps, (bf16_t*)a.z, (bf16_t*)a.pre, a.cls, a.l0};
    return launch(s, p, D.L);
  }
  EncPolicy<bf16_t> p{D, D.B, D.F, D.d, D.d, D.F,
                      (const bf16_t*)a.x, (const bf16_t*)a.W_enc, a.b_enc, a.theta, nullptr,
                      0.5f * a.ste_eps, (bf16_t*)a.z, (bf16_t*)a.pre, a.cls, a.l0};
  return launch(s, p, D.L);
}
hipError_t launch_dec_bf16(hipStream_t s, Dims D, const DecArgs& a) {
  DecPolicy<bf16_t> p{D, D.B, D.d, D.F, D.F, D.d, (const bf16_t*)a.z, (const bf16_t*)a.W_dec, a.b_dec, a.y_hat};
  return launch(s, p, D.L);
}
hipError_t launch_dz_bf16(hipStream_t s, Dims D, const DzArgs& a) {
  DzPolicy<bf16_t> p{D, D.B, D.F, D.d, D.d, D.d,
                     (const bf16_t*)a.d_yhat, (const bf16_t*)a.W_dec, (const bf16_t*)a.z, a.cls, a.norms,
                     a.lam_c_over_b, a.C, (bf16_t*)a.dpre};
  return launch(s, p, D.L);
}
hipError_t launch_dwdec_bf16(hipStream_t s, Dims D, const DWdecArgs& a) {
  DWdecPolicy<bf16_t> p{D, D.F, D.d, D.B, D.F, D.d,
                        (const bf16_t*)a.z, (const bf16_t*)a.d_yhat, (const bf16_t*)a.W_dec, a.G, a.norms,
                        (bf16_t*)a.dW_dec};
  return launch(s, p, D.P());
}
hipError_t launch_dwenc_bf16(hipStream_t s, Dims D, const DWencArgs& a, bool int8_x) {
  if (int8_x) {
    DWencPolicy<bf16_t, int8_t> p{D, D.d, D.F, D.B, D.d, D.F, (const int8_t*)a.x, (const bf16_t*)a.dpre,
                                  (bf16_t*)a.dW_enc};
    return launch(s, p, D.L);
  }
  DWencPolicy<bf16_t> p{D, D.d, D.F, D.B, D.d, D.F, (const bf16_t*)a.x, (const bf16_t*)a.dpre, (bf16_t*)a.dW_enc};
  return launch(s, p, D.L);
}

}  // namespace clt
