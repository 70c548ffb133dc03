// De-quantise the packed weight back to a row-major [K,N] fp16/bf16 matrix.
// Same load + reinterpret + cast code as the matmul kernels (paper, Section
// "Efficient Low-Precision Support in LLMs"); the result is written to memory so
// that it can be compared bit for bit.  Compiled once per weight type (QG_WT).
#include "qg_decode.h"
#include "qg_static_for.h"

#ifndef QG_WT
#error "compile with -DQG_WT=<weight type index>"
#endif

namespace qg {

// MX: 8-bit exponent scales, one per 32 rows and column, applied by the scaled hardware converts
// (e2m1 / e4m3 weights on the first layout).
template <int WT, int ROUTE, int LY, bool MX = false>
__global__ __launch_bounds__(256) void dequant_kernel(DequantParams p) {
  typedef Decoder<WT, ROUTE, LY> D;
  typedef LayoutOf<LY> L;
  constexpr int BITS = D::BITS, RAW = D::RAW;
  const int l = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int KC = p.K / TILE_K;
  const int64_t chunk = (int64_t)blockIdx.x * 4 + wave;
  typename D::Uniform u;
  u.init();
  if constexpr (D::IS_LUT) {       // codebook indices: the replicated lookup table, built by the whole workgroup
    __shared__ __attribute__((aligned(16))) unsigned char lds_raw[D::TABLE_DWORDS * 4 + 512];
    uint32_t* table = reinterpret_cast<uint32_t*>(lds_raw);
    D::build(table, reinterpret_cast<uint16_t*>(lds_raw + D::TABLE_DWORDS * 4), D::fetch(p.T, threadIdx.x), threadIdx.x, 256);
    u.set_table(table, l);
  }
  if (chunk >= (int64_t)KC * (p.N / TILE_N)) return;
  const int nc = (int)(chunk / KC), kc = (int)(chunk % KC);

  uint32_t r[RAW];
  const uint4* src = reinterpret_cast<const uint4*>(p.W + chunk * (1024 * BITS));
#pragma unroll
  for (int i = 0; i < BITS; ++i) {
    uint4 q = src[i * 64 + l];
    r[4 * i + 0] = q.x; r[4 * i + 1] = q.y; r[4 * i + 2] = q.z; r[4 * i + 3] = q.w;
  }
  const int n0 = TILE_N * nc + L::pair_n(l, 0);
  static_for<L::STEPS>([&](auto Jc) __attribute__((always_inline)) {
    constexpr int J = decltype(Jc)::value;
    const int g = (TILE_K * kc + L::K_STEP * J) / p.group;
    uint2 sraw = make_uint2(0u, 0u);
    uint32_t zraw = 0u;
    if constexpr (MX) {
    } else if constexpr (L::NT == 4) {
      sraw = *reinterpret_cast<const uint2*>(p.S + (int64_t)g * p.N + n0);
      if constexpr (!D::IS_LUT)
        if (p.Z) zraw = *reinterpret_cast<const uint32_t*>(p.Z + (int64_t)g * p.N + n0);
    } else {
      sraw = make_uint2(*reinterpret_cast<const uint32_t*>(p.S + (int64_t)g * p.N + n0), 0u);
      if (p.Z) zraw = *reinterpret_cast<const uint16_t*>(p.Z + (int64_t)g * p.N + n0);
    }
    // all of the lane's columns for this k-step, then one store per row: the lane's
    // NT adjacent columns are 2*NT contiguous bytes, and the 16 (32) lanes of a k-block
    // together write 128 contiguous bytes of the row
    uint32_t o[L::NT][4];
    if constexpr (MX) {
      MxConsts mx;
      mx.make(*reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint8_t*>(p.S) + (int64_t)(4 * kc + J) * p.N + n0));
      static_for<4>([&](auto NTc) __attribute__((always_inline)) {
        constexpr int NT = decltype(NTc)::value;
        frag_mx<WT, ROUTE == ROUTE_BF16, J, NT>(r, mx, o[NT]);
      });
    } else {
      typename D::Consts gc;
      D::make_consts(gc, sraw, zraw, p.zbias, p.scale_bf16);
      static_for<L::NT>([&](auto NTc) __attribute__((always_inline)) {
        constexpr int NT = decltype(NTc)::value;
        D::template frag<J, NT>(r, gc, u, o[NT]);
      });
    }
    if constexpr (LY == 0) {
      if (p.frag_out) {            // the registers as they are, one 16-byte store per (k-step, sub-tile): 1 KiB per wavefront
        uint4* dst = reinterpret_cast<uint4*>(reinterpret_cast<uint8_t*>(p.out) + chunk * 16384) + l;
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) dst[(J * 4 + nt) * 64] = make_uint4(o[nt][0], o[nt][1], o[nt][2], o[nt][3]);
        return;
      }
    }
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      const int k = TILE_K * kc + L::pair_k(l, L::t0(J, 0) + v);
      uint16_t* row0 = p.out + (int64_t)k * p.N + n0;          // the pair's lo code: row k
      uint16_t* row1 = row0 + p.N;                              // its hi code: row k + 1
      if constexpr (L::NT == 4) {
        *reinterpret_cast<uint2*>(row0) = make_uint2((o[0][v] & 0xffffu) | (o[1][v] << 16), (o[2][v] & 0xffffu) | (o[3][v] << 16));
        *reinterpret_cast<uint2*>(row1) = make_uint2((o[0][v] >> 16) | (o[1][v] & 0xffff0000u), (o[2][v] >> 16) | (o[3][v] & 0xffff0000u));
      } else {
        *reinterpret_cast<uint32_t*>(row0) = (o[0][v] & 0xffffu) | (o[1][v] << 16);
        *reinterpret_cast<uint32_t*>(row1) = (o[0][v] >> 16) | (o[1][v] & 0xffff0000u);
      }
    }
  });
}

#define QG_CAT2(a, b) a##b
#define QG_CAT(a, b) QG_CAT2(a, b)

template <int LY>
static void launch_ly(const DequantParams& p, int route, dim3 grid, dim3 block, hipStream_t st) {
  if (route == ROUTE_F16) hipLaunchKernelGGL((dequant_kernel<QG_WT, ROUTE_F16, LY>), grid, block, 0, st, p);
  else                    hipLaunchKernelGGL((dequant_kernel<QG_WT, ROUTE_BF16, LY>), grid, block, 0, st, p);
}

int QG_CAT(dequant_launch_wt, QG_WT)(const DequantParams& p, int route, hipStream_t st) {
  int64_t nchunks = (int64_t)(p.K / TILE_K) * (p.N / TILE_N);
  dim3 grid((unsigned)((nchunks + 3) / 4)), block(256);
  if (p.scale_e8m0) {
#if QG_WT == 9 || QG_WT == 13
    if (p.layout != 0 || p.group != 32) return QG_EUNSUPPORTED;
    if (route == ROUTE_F16) hipLaunchKernelGGL((dequant_kernel<QG_WT, ROUTE_F16, 0, true>), grid, block, 0, st, p);
    else                    hipLaunchKernelGGL((dequant_kernel<QG_WT, ROUTE_BF16, 0, true>), grid, block, 0, st, p);
    return hipGetLastError() == hipSuccess ? QG_OK : QG_EHIP;
#else
    return QG_EUNSUPPORTED;
#endif
  }
#if QG_WT > 14
  if (p.layout != 0 || !p.T) return QG_EINVAL;          // codebook indices: first layout, with a table
  launch_ly<0>(p, route, grid, block, st);
#else
  if (p.layout == 0) launch_ly<0>(p, route, grid, block, st);
  else               launch_ly<1>(p, route, grid, block, st);
#endif
  return hipGetLastError() == hipSuccess ? QG_OK : QG_EHIP;
}

}  // namespace qg
