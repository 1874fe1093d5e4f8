// bf16 MFMA path of the five CLT contractions on gfx950 (CDNA4).
//
// One workgroup = 8 wavefronts (two per SIMD) computes a 256x256 output tile;
// each wavefront owns a 128x64 block as 8x4 v_mfma_f32_16x16x32_bf16
// accumulators (128 accumulator registers per lane; at the board's power limit
// this shape runs 14 % faster on real data than 32x32x16, whose accumulator
// traffic per flop is twice as large).  K advances in steps of
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

#include <cstdlib>
#include <type_traits>

namespace clt {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef f32x4_t acc_t[8][4];   // a wave's 128x64 block as 8x4 accumulators of 16x16
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
// 8 operand elements as they come out of memory (int8: the codes in the first two dwords), and
// their bf16 form.  The conversion happens when the tile goes to LDS, not at the load: arithmetic
// on a loaded register is where the wait for that load lands, and the loads of a tile are meant
// to stay in flight across the other group's compute phase.
template <typename TE> __device__ __forceinline__ u32x4 load8(const TE* p);
template <> __device__ __forceinline__ u32x4 load8<bf16_t>(const bf16_t* p) { return ld16(p); }
template <> __device__ __forceinline__ u32x4 load8<int8_t>(const int8_t* p) {
  const u32x2 q = *reinterpret_cast<const u32x2*>(p);
  u32x4 r = {q[0], q[1], 0u, 0u};
  return r;
}
template <typename TE> __device__ __forceinline__ u32x4 cook8(u32x4 raw);
template <> __device__ __forceinline__ u32x4 cook8<bf16_t>(u32x4 raw) { return raw; }
template <> __device__ __forceinline__ u32x4 cook8<int8_t>(u32x4 raw) {
  u32x2 q = {raw[0], raw[1]};
  return i8x8_to_bf16x8(q);
}

// ---------------------------------------------------------------------------
// Staging of one 256(rows) x 64(k) operand tile by 256 lanes (lt = 0..255),
// 8 x 16 bytes per lane.
//   K-contiguous operand: lane takes 16-byte chunk c = lt%8 of rows lt/8 + 32 i.
//   K-strided operand:    lane takes the 8(k) x 8(rows) block kb = lt/32, nb = lt%32
//                         and transposes it in registers before the LDS write.
// Addresses are a wave-uniform base (tile origin, advanced along K by the
// caller) plus one 32-bit per-lane byte offset that never changes, so a load
// needs a single address register.  The EDGE variants predicate every chunk
// and redirect out-of-range ones to the tensor base (always readable); those
// chunks reach LDS as zeros.
// ---------------------------------------------------------------------------
template <bool KC, typename TE>
struct Stager {
  uint32_t voff;       // per-lane byte offset inside the tile
  uint32_t step;       // byte distance between the lane's consecutive chunks (uniform)
  int r_lane, k_lane;  // EDGE only: first row / k index of this lane inside the tile

  __device__ __forceinline__ void init(int lt, int ld) {
    if (KC) {
      r_lane = lt >> 3; k_lane = (lt & 7) << 3;
      voff = (uint32_t)(((size_t)r_lane * ld + k_lane) * sizeof(TE));
      step = (uint32_t)(32u * ld * sizeof(TE));
    } else {
      r_lane = (lt & 31) << 3; k_lane = (lt >> 5) << 3;
      voff = (uint32_t)(((size_t)k_lane * ld + r_lane) * sizeof(TE));
      step = (uint32_t)(ld * sizeof(TE));
    }
  }
  // tile_base = operand + tile origin (row r0, k index k0), uniform
  // EDGE: chunks outside the matrix are read from the tensor base and must reach LDS as zeros.  A
  // K-contiguous operand remembers which chunks lie inside (bit i of `inside`) and zeroes the others
  // when the tile goes to LDS, so that nothing is computed on the loaded registers here; a
  // K-strided one zeroes them at once (its transposition mixes all 8 registers, and keeping the
  // predicates until then costs the predicated code more registers than it has).
  template <bool EDGE>
  __device__ __forceinline__ void load(u32x4 (&r)[8], uint32_t& inside, const TE* seg_base, const TE* tile_base,
                                       int rows_left, int k_left) const {
    const char* b = reinterpret_cast<const char*>(tile_base);
    uint32_t in = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const char* bi = b + (size_t)i * step;            // uniform
      if (!EDGE) {
        r[i] = load8<TE>(reinterpret_cast<const TE*>(bi + voff));
      } else {
        const bool ok = KC ? (r_lane + 32 * i < rows_left && k_lane < k_left)
                           : (r_lane < rows_left && k_lane + i < k_left);
        const TE* ptr = ok ? reinterpret_cast<const TE*>(bi + voff) : seg_base;
        const u32x4 v = load8<TE>(ptr);
        const u32x4 zero = {0u, 0u, 0u, 0u};
        if (KC) { r[i] = v; in |= (ok ? 1u : 0u) << i; }
        else r[i] = ok ? v : zero;
      }
    }
    if (EDGE && KC) inside = in;
  }
  template <bool EDGE>
  __device__ __forceinline__ void store(bf16_t* lds, const u32x4 (&r)[8], uint32_t inside, int lt) const {
    if (KC) {
      const int c = lt & 7;
      const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int row = (lt >> 3) + 32 * i;
        const u32x4 v = cook8<TE>(r[i]);
        *reinterpret_cast<u32x4*>(lds + lds_off(row, c)) = (!EDGE || ((inside >> i) & 1u)) ? v : zero;
      }
    } else {
      const int nb = lt & 31, kb = lt >> 5;
      u32x4 q[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) q[i] = cook8<TE>(r[i]);
#pragma unroll
      for (int n = 0; n < 8; ++n) {
        u32x4 o;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const uint32_t lo = q[2 * w][n >> 1], hi = q[2 * w + 1][n >> 1];
          o[w] = (n & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
        }
        *reinterpret_cast<u32x4*>(lds + lds_off(8 * nb + n, kb)) = o;
      }
    }
  }
};

constexpr int NTHREADS = 512;   // 8 wavefronts: two per SIMD, so one's memory phase hides under the other's MFMAs

// K loop of one output tile.  EDGE = false assumes the tile lies fully inside the
// matrices and kseg is a multiple of 64 (no predication at all).
template <class P, bool EDGE>
__device__ __forceinline__ void main_loop(const P& p, const typename P::GInfo& gi, int m0, int n0, bf16_t* smem,
                                          acc_t& acc, int t, uint32_t& sync_count) {
  typedef typename P::AType TA;
  const int lane = t & 63, w = t >> 6, wm = w >> 2, wn = w & 3;
  const int lt = t & 255;
  // waves 0-3 stage A, waves 4-7 stage B (waves w and w+4 share a SIMD, so each SIMD holds one of each group)
  const bool loads_a = __builtin_amdgcn_readfirstlane(w) < 4;
  const int kseg = p.kseg, nseg = p.nseg(gi);
  const int nk = nseg * ((kseg + TK - 1) / TK);

  Stager<P::A_KC, TA> sa;
  Stager<P::B_KC, bf16_t> sb;
  sa.init(lt, p.lda);
  sb.init(lt, p.ldb);

  // uniform cursors: current segment bases, k offset inside the segment
  int ld_seg = 0, ld_k0 = 0;
  const TA* Aseg = p.a_seg(gi, 0);
  const bf16_t* Bseg = p.b_seg(gi, 0);
  const size_t a_row0 = P::A_KC ? (size_t)m0 * p.lda : (size_t)m0;   // tile origin at k = 0
  const size_t b_row0 = P::B_KC ? (size_t)n0 * p.ldb : (size_t)n0;
  const size_t a_kstep = P::A_KC ? 1 : (size_t)p.lda, b_kstep = P::B_KC ? 1 : (size_t)p.ldb;
  u32x4 rg[8];
  uint32_t rg_inside = 0;   // EDGE, K-contiguous operand: which of the 8 chunks lie inside the matrix

  auto fetch = [&]() {
    if (loads_a) sa.template load<EDGE>(rg, rg_inside, Aseg, Aseg + a_row0 + ld_k0 * a_kstep, p.M - m0, kseg - ld_k0);
    else sb.template load<EDGE>(rg, rg_inside, Bseg, Bseg + b_row0 + ld_k0 * b_kstep, p.N - n0, kseg - ld_k0);
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
  // Keeping an XCD's workgroups in step (policies with an xcd_sync member, persistent launches only).  The 32
  // tiles an XCD works on share 12 operand panels through its 4 MB L2, which holds about ten K steps of them:
  // tiles that drift further apart fetch every panel from the fabric again.  At the start of every K segment
  // the workgroup books itself on its XCD's counter and its first wave waits, for a bounded time, until all
  // 32 have done so (every workgroup of an XCD walks the same groups in the same order, so the n-th booking
  // of each belongs together).  Only a pacing aid: a wait that runs into its bound just goes on.
  auto xcd_sync = [&]() {
    if constexpr (P::XCD_SYNC) {
      ++sync_count;
      if (p.xcd_sync && t == 0) {
        uint32_t* ctr = p.xcd_sync + (blockIdx.x & 7) * 64;
        const uint32_t want = (gridDim.x >> 3) * sync_count;
        __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int spin = 0; spin < 400; ++spin) {
          if (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= want) break;
          __builtin_amdgcn_s_sleep(2);
        }
      }
    }
  };
  auto stage = [&](int st) {
    bf16_t* base = smem + st * STAGE_ELEMS;
    if (loads_a) sa.template store<EDGE>(base, rg, rg_inside, lt);
    else sb.template store<EDGE>(base + 256 * TK, rg, rg_inside, lt);
  };

  // v_mfma_f32_16x16x32_bf16: a lane's fragment is 8 consecutive k of row lane%16; lane group lane/16 takes
  // one of the four 8-wide k chunks of a 32-wide slice.  Which chunk a group takes is free as long as A and B
  // agree: groups 0,1,2,3 take chunks 0,2,1,3.  A 16-byte LDS read is served in four passes of lanes
  // 8q..8q+7 together with 32+8q..32+8q+7; with this assignment the two halves of a pass read chunks c and
  // c^1 of the same 8 rows, which the swizzle puts on distinct banks (chunks in order: two-way conflicts on
  // every fragment read).  One K step = two slices; in each the four B fragments stay put while the A
  // fragments come four at a time: 4 groups of 16 MFMAs per K step.
  u32x4 fa[2][4], fb[2][4];
  const int frow = lane & 15, fch = ((lane >> 3) & 2) | (lane >> 5);
  auto read_a = [&](int st, int sl, int q, int buf) {
    const bf16_t* a = smem + st * STAGE_ELEMS;
#pragma unroll
    for (int i = 0; i < 4; ++i) fa[buf][i] = ld16(a + lds_off(wm * 128 + (4 * q + i) * 16 + frow, 4 * sl + fch));
  };
  auto read_b = [&](int st, int sl, int buf) {
    const bf16_t* b = smem + st * STAGE_ELEMS + 256 * TK;
#pragma unroll
    for (int j = 0; j < 4; ++j) fb[buf][j] = ld16(b + lds_off(wn * 64 + j * 16 + frow, 4 * sl + fch));
  };
  auto mfma_g = [&](int q, int abuf, int bbuf) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[4 * q + i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, fa[abuf][i]),
                                                                    __builtin_bit_cast(bf16x8_t, fb[bbuf][j]),
                                                                    acc[4 * q + i][j], 0, 0, 0);
  };
  // One K step = the 64 MFMAs of this wave on tile `kt`; the fragment reads of the next group overlap the
  // MFMAs of the current one, and the MFMAs of a tile's last group are held back until the first fragment
  // reads of the next tile are in flight (their operands stay in registers across the memory phase).
  auto mfma = [&](int) { mfma_g(1, 1, 1); };   // the group held back at the end of a K step
  const int first_kt = 0;
  auto compute = [&](int kt) {
    const int cur = kt & 1;
    __builtin_amdgcn_s_setprio(1);
    read_b(cur, 0, 0);
    read_a(cur, 0, 0, 0);
    if (kt != first_kt) mfma_g(1, 1, 1);   // last group of the previous tile, deferred to cover this read latency
    read_a(cur, 0, 1, 1);
    mfma_g(0, 0, 0);
    read_b(cur, 1, 1);
    read_a(cur, 1, 0, 0);
    mfma_g(1, 1, 0);
    read_a(cur, 1, 1, 1);
    mfma_g(0, 0, 1);
    __builtin_amdgcn_s_setprio(0);
  };

  // Ping-pong: the two wavefronts of a SIMD belong to different groups that run
  // half a K step apart, so the memory phase of one (wait for HBM data,
  // registers -> LDS, issue the next fetch) sits under the MFMA phase of the
  // other.  Every phase ends at a workgroup barrier; both groups execute the
  // same number of barriers.  Group A (waves 0-3) writes its half of tile k
  // right before computing it; group B (waves 4-7) writes its half of tile k+1
  // before computing tile k, so a stage is never written while the other group
  // still reads it: interval 2k = {A: memory(k), B: compute(k-1)}, interval 2k+1 =
  // {A: compute(k), B: memory(k+1)}; stage k&1 is written by A in 2k and by B in 2k-1
  // and read by both from 2k+1 (A) / 2k+2 (B) on, after a barrier.
  // (the prologue is repeated inside each branch on purpose: every branch then only ever
  // touches its own operand, which keeps the other operand's addressing out of its registers)
  if (loads_a) {
    fetch();
    stage(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      if (kt >= 1) stage(kt & 1);
      if (kt + 1 < nk) {
        if (ld_k0 == 0) xcd_sync();   // the fetch opens a new K segment
        fetch();
      }
      __syncthreads();
      compute(kt);
      __syncthreads();
    }
    mfma(1);
  } else {
    fetch();
    stage(0);
    if (nk > 1) fetch();
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
      if (kt >= 1) compute(kt - 1);
      __syncthreads();
      if (kt + 1 < nk) stage((kt + 1) & 1);
      if (kt + 2 < nk) fetch();
      __syncthreads();
    }
    compute(nk - 1);
    mfma(1);
  }
}

// Epilogue of one tile: accumulators -> LDS (wave-private 32 rows x 64 fp32) -> 4 consecutive
// columns of one row per lane -> the policy's fused epilogue.  The lane's position inside a row
// group never changes and the group's origin is wave-uniform (EpiPos), so the policy's memory
// accesses are a scalar base plus one fixed per-lane offset.  EDGE = false: the tile lies fully
// inside the matrix, no predicates.
template <class P, bool EDGE>
__device__ __forceinline__ void epilogue(const P& p, const typename P::GInfo& gi, int m0, int n0, bf16_t* smem,
                                         acc_t& acc, int t) {
  const int lane = t & 63, w = t >> 6;
  const int wu = __builtin_amdgcn_readfirstlane(w), wm = wu >> 2, wn = wu & 3;
  const int M = p.M, N = p.N;
  __syncthreads();
  float* wl = reinterpret_cast<float*>(smem) + wu * (32 * 64);
  EpiPos pos;
  // (the transposition uses the first 64 KB of LDS, 8 KB per wave; the policy's scratch lies behind it)
  pos.lds = reinterpret_cast<float*>(smem) + 8 * (32 * 64) + wu * 128;
  pos.cu = n0 + wn * 64;
  pos.cl = (lane & 15) << 2;
  pos.rl = lane >> 4;
  pos.ru = 0;
  const bool col_ok = !EDGE || pos.col() < N;
  typename P::Epi est;
  p.epi_begin(est, gi, pos.col(), col_ok, m0 + wm * 128);
  // The wave's block is 32 row groups of 4 rows (4 slabs of 8).  Each slab goes through the wave's
  // private LDS region (a wave's LDS accesses complete in issue order, so the transposition needs
  // no barrier).  The global loads the policy's epilogue needs run ahead of their use as a rolling
  // window: before group g is consumed the loads of all groups below g + depth have been issued, so
  // loads stay in flight while earlier groups are computed and stored.  The window deepens slab by
  // slab as the accumulators already written out stop occupying registers (predicated edge tiles
  // keep to 4: the predicates' registers come on top).
  constexpr int NG = 32;
  // look-ahead (in row groups) while group g is consumed
  auto depth = [](int g) constexpr {
    const int d = g < 8 ? P::EPI_BATCH : (g < 16 ? P::EPI_BATCH_LATE : P::EPI_BATCH_LAST);
    return (EDGE && d > 4) ? 4 : d;
  };
  typename P::EpiRegs er[NG];
  auto issue = [&](int g) {
    pos.ru = m0 + wm * 128 + g * 4;
    if (!EDGE || (col_ok && pos.row() < M)) p.epi_load(er[g], gi, pos);
  };
#pragma unroll
  for (int g = 0; g < depth(0); ++g) issue(g);
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    if ((g & 7) == 0) {
      const int i = g >> 3;
#pragma unroll
      for (int ii = 0; ii < 2; ++ii)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            wl[(16 * ii + 4 * (lane >> 4) + r) * 64 + j * 16 + (lane & 15)] = acc[2 * i + ii][j][r];
    }
    const int done = g == 0 ? depth(0) : g - 1 + depth(g - 1);
    const int want = g + depth(g);
#pragma unroll
    for (int q = (done < NG ? done : NG); q < (want < NG ? want : NG); ++q) issue(q);
    pos.ru = m0 + wm * 128 + g * 4;
    const float4 v = *reinterpret_cast<const float4*>(wl + ((g & 7) * 4 + pos.rl) * 64 + pos.cl);
    if (!EDGE || (col_ok && pos.row() < M)) p.epi4(est, gi, pos, v, er[g]);
  }
  p.epi_end(est, gi, pos.lds);
}

// P::PERSISTENT: the grid is one workgroup per CU and workgroup i runs tiles i, i + gridDim.x, ...
// of the XCD-aware tile order (gridDim.x is a multiple of 8, so all tiles of a workgroup belong
// to the XCD it runs on).  Between two tiles of a CU there is then neither a workgroup dispatch
// nor a wait for the finished tile's stores to drain (2 to 8 us per tile otherwise).
// INTERIOR: no tile of the launch touches an edge, only the unpredicated code is built in.
template <class P, bool INTERIOR>
__global__ __launch_bounds__(NTHREADS) void gemm_bf16_kernel(P p, TileGrid tg, int nwg) {
  extern __shared__ __align__(16) bf16_t smem[];
  if (p.skip()) return;
  constexpr bool LOOP = P::PERSISTENT && INTERIOR;   // (the predicated code has no registers to spare for the loop either)
  uint32_t sync_count = 0;   // K segments this workgroup has opened so far (see xcd_sync in main_loop)
  int vb = blockIdx.x;
  do {
    int gorder, tm, tn;
    if (!tg.decode(vb, gorder, tm, tn)) continue;
    const typename P::GInfo gi = p.ginfo(gorder);
    const int m0 = tm * TM, n0 = tn * TN;

    // wave w owns output rows (w/4)*128.., columns (w%4)*64..
    acc_t acc;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;

    // The thread index is made opaque once per tile: everything a lane derives from it (LDS
    // addresses, operand offsets, epilogue positions) is then recomputed per tile instead of
    // being hoisted out of this loop, where it would stay live across both phases of every tile
    // and push the kernel over its 256 registers.
    int t = threadIdx.x;
    asm volatile("" : "+v"(t));
    if (INTERIOR) {   // no tile of this launch touches an edge
      main_loop<P, false>(p, gi, m0, n0, smem, acc, t, sync_count);
      epilogue<P, false>(p, gi, m0, n0, smem, acc, t);
    } else {
      const bool inside = (m0 + TM <= p.M) && (n0 + TN <= p.N);
      if (inside && p.kseg % TK == 0) main_loop<P, false>(p, gi, m0, n0, smem, acc, t, sync_count);
      else main_loop<P, true>(p, gi, m0, n0, smem, acc, t, sync_count);
      if (inside) epilogue<P, false>(p, gi, m0, n0, smem, acc, t);
      else epilogue<P, true>(p, gi, m0, n0, smem, acc, t);
    }
    if (LOOP) __syncthreads();   // the next tile stages its operands in the LDS the epilogue transposed through
  } while (LOOP && (vb += gridDim.x) < nwg);
}

int g_num_wg_slots = 0;   // workgroups of a persistent grid: the CU count, rounded down to a multiple of 8

template <class P>
hipError_t launch(hipStream_t s, const P& p, int G) {
  const TileGrid tg = TileGrid::make(G, p.M, p.N, TM, TN);
  const int nwg = tg.num_wg();
  if (g_num_wg_slots < 8) return hipErrorNotInitialized;
  if (p.M % TM == 0 && p.N % TN == 0 && p.kseg % TK == 0) {
    // The tile loop gives every workgroup a fixed share (tiles i, i + grid, ...).  The shares are equal when all
    // groups have the same K, or when every workgroup meets every round of groups equally often (the slots of
    // a round are a multiple of the slots one pass of the grid covers; the snake order evens out the teams).
    // Otherwise the hardware's dispatch of one workgroup per tile, longest groups first, balances better.
    const int pass = g_num_wg_slots / 8;   // slots per XCD that one pass of the grid covers
    const bool even_shares = P::UNIFORM_K || tg.per_xcd % pass == 0;
    const int grid = (P::PERSISTENT && even_shares && nwg > g_num_wg_slots) ? g_num_wg_slots : nwg;
    if constexpr (P::XCD_SYNC) {
      // pacing needs every workgroup of an XCD to open the same K segments: a tile loop in which no slot is empty
      const bool full = grid < nwg && (tg.mt * tg.nt) % tg.S == 0 && G % tg.nteams == 0 && nwg % grid == 0;
      P q = p;
      if (!full || getenv("CLT_NO_XCD_PACING")) q.xcd_sync = nullptr;
      if (q.xcd_sync) {
        const hipError_t ez = launch_zero_i32(s, reinterpret_cast<int32_t*>(q.xcd_sync), 8 * 64);
        if (ez != hipSuccess) return ez;
      }
      hipLaunchKernelGGL((gemm_bf16_kernel<P, true>), dim3(grid), dim3(NTHREADS), LDS_BYTES, s, q, tg, nwg);
      return hipGetLastError();
    }
    hipLaunchKernelGGL((gemm_bf16_kernel<P, true>), dim3(grid), dim3(NTHREADS), LDS_BYTES, s, p, tg, nwg);
  } else {
    hipLaunchKernelGGL((gemm_bf16_kernel<P, false>), dim3(nwg), dim3(NTHREADS), LDS_BYTES, s, p, tg, nwg);
  }
  return hipGetLastError();
}

template <class P>
hipError_t set_lds_attr() {
  const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<P, true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
  if (e != hipSuccess) return e;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_bf16_kernel<P, false>),
                             hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
}

}  // namespace

hipError_t init_gemm_bf16() {
  hipError_t e;
  int dev = 0, cus = 0;
  if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
  if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
  g_num_wg_slots = cus >= 8 ? cus / 8 * 8 : 8;
  if ((e = set_lds_attr<EncPolicy<bf16_t>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<EncPolicy<bf16_t, int8_t>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DecPolicy<bf16_t>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DzPolicy<bf16_t>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DzPolicy<bf16_t, true>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DWdecPolicy<bf16_t, false>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DWdecPolicy<bf16_t, true>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DWdecPolicy<bf16_t, true, true>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DWencPolicy<bf16_t, false>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DWencPolicy<bf16_t, true>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DWencPolicy<bf16_t, false, int8_t>>()) != hipSuccess) return e;
  if ((e = set_lds_attr<DWencPolicy<bf16_t, true, int8_t>>()) != hipSuccess) return e;
  return hipSuccess;
}

hipError_t launch_enc_bf16(hipStream_t s, Dims D, const EncArgs& a, bool int8_x) {
  if (int8_x) {
    EncPolicy<bf16_t, int8_t> p{D, D.B, D.F, D.d, D.d, D.F,
                                (const int8_t*)a.x, (const bf16_t*)a.W_enc, a.b_enc, a.theta, a.x_scale,
                                0.5f * a.ste_eps, (bf16_t*)a.z, (bf16_t*)a.pre, a.cls, a.l0, a.log_threshold, a.pre32};
    return launch(s, p, D.L);
  }
  EncPolicy<bf16_t> p{D, D.B, D.F, D.d, D.d, D.F,
                      (const bf16_t*)a.x, (const bf16_t*)a.W_enc, a.b_enc, a.theta, nullptr,
                      0.5f * a.ste_eps, (bf16_t*)a.z, (bf16_t*)a.pre, a.cls, a.l0, a.log_threshold, a.pre32};
  return launch(s, p, D.L);
}
hipError_t launch_dec_bf16(hipStream_t s, Dims D, const DecArgs& a) {
  DecPolicy<bf16_t> p{D, D.B, D.d, D.F, D.F, D.d, (const bf16_t*)a.z, (const bf16_t*)a.W_dec, a.b_dec, a.y_hat, a.skip_flags, a.kcap,
                      a.xcd_sync};
  return launch(s, p, D.L);
}
template <bool FOLD>
static hipError_t launch_dz_mode(hipStream_t s, Dims D, const DzArgs& a) {
  DzPolicy<bf16_t, FOLD> p{D, D.B, D.F, D.d, D.d, D.d,
                           (const bf16_t*)a.d_yhat, (const bf16_t*)a.W_dec, (const bf16_t*)a.z, a.cls, a.norms,
                           a.lam_c_over_b, a.C, (bf16_t*)a.dpre, a.lam1_over_b, a.skip_flags, a.kcap,
                           a.x_scale, a.part_theta, a.part_benc, a.part_below};
  return launch(s, p, D.L);
}
hipError_t launch_dz_bf16(hipStream_t s, Dims D, const DzArgs& a) {
  return a.part_theta ? launch_dz_mode<true>(s, D, a) : launch_dz_mode<false>(s, D, a);
}
template <bool ADAM, bool N2>
static hipError_t launch_dwdec_mode(hipStream_t s, Dims D, const DWdecArgs& a) {
  DWdecPolicy<bf16_t, ADAM, N2> p{D, D.F, D.d, D.B, D.F, D.d,
                              (const bf16_t*)a.z, (const bf16_t*)a.d_yhat, (bf16_t*)a.W_dec, a.G, a.norms,
                              (bf16_t*)a.dW_dec, AdamFuse{a.fuse.m, a.fuse.v, a.fuse.master, a.fuse.a}, a.skip_flags, a.kcap, 0,
                              N2 ? a.n2_part : nullptr};
  // One launch per source layer: the tiles that share operand panels start together again at
  // every launch and stay in step along K, which keeps the panel reuse in the XCDs' L2s (same
  // run time as one long launch, but half the traffic to the fabric).  Layers whose blocks hold
  // fewer than 8 rounds of tiles for the CUs share a launch with the layers after them: a launch
  // that ends on a partly filled round leaves CUs idle, and short launches do so often.
  const int tiles_per_block = ((D.F + TM - 1) / TM) * ((D.d + TN - 1) / TN);
  const int min_blocks = (8 * g_num_wg_slots + tiles_per_block - 1) / tiles_per_block;
  for (int l = 0; l < D.L;) {
    int l1 = l, blocks = 0;
    do { blocks += D.L - l1; ++l1; } while (l1 < D.L && blocks < min_blocks);
    p.p0 = packed_index(l, l, D.L);
    const hipError_t e = launch(s, p, blocks);
    if (e != hipSuccess) return e;
    l = l1;
  }
  return hipSuccess;
}
hipError_t launch_dwdec_bf16(hipStream_t s, Dims D, const DWdecArgs& a) {
  if (!a.fuse.m) return launch_dwdec_mode<false, false>(s, D, a);
  // the row sums of squares need every tile to take the unpredicated epilogue (all 16 lanes of a row at work)
  if (a.n2_part && D.F % TM == 0 && D.d % TN == 0) return launch_dwdec_mode<true, true>(s, D, a);
  return launch_dwdec_mode<true, false>(s, D, a);
}
template <bool ADAM, typename TA>
static hipError_t launch_dwenc_mode(hipStream_t s, Dims D, const DWencArgs& a) {
  DWencPolicy<bf16_t, ADAM, TA> p{D, D.d, D.F, D.B, D.d, D.F, (const TA*)a.x, (const bf16_t*)a.dpre,
                                  (bf16_t*)a.dW_enc, (bf16_t*)a.W_enc, AdamFuse{a.fuse.m, a.fuse.v, a.fuse.master, a.fuse.a}};
  return launch(s, p, D.L);
}
hipError_t launch_dwenc_bf16(hipStream_t s, Dims D, const DWencArgs& a, bool int8_x) {
  if (int8_x) return a.fuse.m ? launch_dwenc_mode<true, int8_t>(s, D, a) : launch_dwenc_mode<false, int8_t>(s, D, a);
  return a.fuse.m ? launch_dwenc_mode<true, bf16_t>(s, D, a) : launch_dwenc_mode<false, bf16_t>(s, D, a);
}

}  // namespace clt
