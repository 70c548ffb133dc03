// Decode-sized matmul (M <= 64): the weights are streamed from HBM exactly once.
//
// One workgroup of 8 wavefronts owns one 64-column strip of W and one slab of K;
// wavefront w takes every 8th 128x64 chunk of the slab.  Per chunk a lane issues
// BITS 16-byte loads for its codes and 4 16-byte loads per 16 rows of A, several
// chunks ahead of use (register ring, the software pipelining the paper calls
// essential in Sections "An Example of Tilus Program" and "End-to-End
// Performance"); codes are unpacked in registers and fed straight to the
// 16x16x32 matrix instruction with W as the row operand, so a lane's four
// accumulators per sub-tile are 16 consecutive columns of one row of C.  The K
// reduction runs inside the MFMA (across the four 8-wide k-blocks of lanes),
// then across the 8 wavefronts through LDS, then -- when K is also split over
// workgroups -- through fp32 partial tiles in a workspace, summed in a fixed
// order by whichever workgroup arrives last (no spinning, no atomics on data).
// Compiled once per weight type (QG_WT).
#include "qg_decode.h"
#include "qg_static_for.h"

#ifndef QG_WT
#error "compile with -DQG_WT=<weight type index>"
#endif

namespace qg {

typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
typedef _Float16 h8_t __attribute__((ext_vector_type(8)));
typedef __bf16 b8_t __attribute__((ext_vector_type(8)));
typedef float f4_t __attribute__((ext_vector_type(4)));

template <int ROUTE>
__device__ __forceinline__ f4_t mfma16(u4_t w, u4_t a, f4_t c) {
  if constexpr (ROUTE == ROUTE_F16)
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8_t, w), __builtin_bit_cast(h8_t, a), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(b8_t, w), __builtin_bit_cast(b8_t, a), c, 0, 0, 0);
}

template <int ROUTE>
__device__ __forceinline__ uint32_t pack_out(float lo, float hi) {
  f2_t f = {lo, hi};
  if constexpr (ROUTE == ROUTE_F16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, h2_t));
  else return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, b2_t));
}

constexpr int SMALL_WAVES = 8;

template <int BITS, int MT>
struct SmallCfg {
  static constexpr int per_stage = 4 * BITS + 16 * MT + 6;
  static constexpr int STAGES = (96 / per_stage) < 2 ? 2 : ((96 / per_stage) > 4 ? 4 : (96 / per_stage));
};

template <int WT, int ROUTE, int MT>
__global__ __launch_bounds__(SMALL_WAVES * 64) void small_kernel(GemmParams p) {
  typedef Decoder<WT, ROUTE> D;
  constexpr int BITS = D::BITS, RAW = D::RAW;
  constexpr int STAGES = SmallCfg<BITS, MT>::STAGES;

  const int tid = threadIdx.x, l = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int b = l >> 4, i16 = l & 15;
  const int nc = blockIdx.x, split = blockIdx.y;
  const int KC = p.K / TILE_K, NCH = p.N / TILE_N;
  const int c0 = split * p.chunks_per_split;
  const int c1 = min(KC, c0 + p.chunks_per_split);
  const int mine = (c1 - c0 > w) ? (c1 - c0 - w + SMALL_WAVES - 1) / SMALL_WAVES : 0;
  const int n0 = TILE_N * nc + 4 * i16;
  const bool two_groups = (p.group == 64);

  const uint4* wstrip = reinterpret_cast<const uint4*>(p.W + (int64_t)nc * KC * (1024 * BITS));
  // rows past M re-read row M-1; their results are never stored
  const uint16_t* arow[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) arow[mt] = p.A + (int64_t)min(mt * 16 + i16, p.M - 1) * p.K + 8 * b;

  struct Stage {
    uint32_t r[RAW];
    u4_t a[MT][4];
    uint2 s0, s1;
    uint32_t z0, z1;
  };
  Stage st[STAGES];

  auto issue = [&](Stage& s, int c) __attribute__((always_inline)) {
    const uint4* src = wstrip + (int64_t)c * (64 * BITS) + l;
#pragma unroll
    for (int i = 0; i < BITS; ++i) {
      uint4 q = src[i * 64];
      s.r[4 * i + 0] = q.x; s.r[4 * i + 1] = q.y; s.r[4 * i + 2] = q.z; s.r[4 * i + 3] = q.w;
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        s.a[mt][j] = *reinterpret_cast<const u4_t*>(arow[mt] + c * TILE_K + 32 * j);
    const int g0 = (p.group == 64) ? 2 * c : ((c >> p.gshift) & p.gmask);
    s.s0 = *reinterpret_cast<const uint2*>(p.S + (int64_t)g0 * p.N + n0);
    s.z0 = p.Z ? *reinterpret_cast<const uint32_t*>(p.Z + (int64_t)g0 * p.N + n0) : 0u;
    if (two_groups) {
      s.s1 = *reinterpret_cast<const uint2*>(p.S + (int64_t)(g0 + 1) * p.N + n0);
      s.z1 = p.Z ? *reinterpret_cast<const uint32_t*>(p.Z + (int64_t)(g0 + 1) * p.N + n0) : 0u;
    } else {
      s.s1 = s.s0; s.z1 = s.z0;
    }
  };

  f4_t acc[MT][4];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = (f4_t){0.f, 0.f, 0.f, 0.f};

  typename D::Uniform u;
  u.init();

  auto compute = [&](const Stage& s) __attribute__((always_inline)) {
    typename D::Consts gc0, gc1;
    D::make_consts(gc0, s.s0, s.z0, p.zbias, p.scale_bf16);
    if (two_groups) D::make_consts(gc1, s.s1, s.z1, p.zbias, p.scale_bf16);
    else gc1 = gc0;
    static_for<4>([&](auto Jc) __attribute__((always_inline)) {
      constexpr int J = decltype(Jc)::value;
      static_for<4>([&](auto NTc) __attribute__((always_inline)) {
        constexpr int NT = decltype(NTc)::value;
        uint32_t o[4];
        D::template frag<J, NT>(s.r, (J < 2) ? gc0 : gc1, u, o);
        u4_t wf = {o[0], o[1], o[2], o[3]};
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt][NT] = mfma16<ROUTE>(wf, s.a[mt][J], acc[mt][NT]);
      });
    });
  };

  // chunk index of my i-th chunk; indices past the end re-load my last chunk
  // (valid memory, result unused) so that the ring needs no branches on loads
  auto chunk_of = [&](int i) __attribute__((always_inline)) { return c0 + w + min(i, mine - 1) * SMALL_WAVES; };

  if (mine > 0) {
#pragma unroll
    for (int s = 0; s < STAGES; ++s)
      if (s < mine) issue(st[s], chunk_of(s));
    for (int i = 0; i < mine; i += STAGES) {
#pragma unroll
      for (int s = 0; s < STAGES; ++s) {
        if (i + s < mine) {
          compute(st[s]);
          if (i + s + STAGES < mine) issue(st[s], chunk_of(i + s + STAGES));
        }
      }
    }
  }

  // ---- reduce over the 8 wavefronts (LDS), one 16-row tile at a time -----------
  __shared__ float red[SMALL_WAVES][16][64];
  __shared__ int s_last;
  const int idx0 = 2 * w;                       // my two of the 16 column offsets
  float sum[MT][2];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    if (mt) __syncthreads();
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[w][4 * r + nt][l] = acc[mt][nt][r];   // row = column offset 4r+nt
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      float t = 0.f;
#pragma unroll
      for (int ww = 0; ww < SMALL_WAVES; ++ww) t += red[ww][idx0 + e][l];
      sum[mt][e] = t;
    }
  }

  const int ncol = TILE_N * nc + 16 * b + idx0;   // columns ncol, ncol+1 of row mt*16 + i16
  if (p.splitk > 1) {
    // Partial tiles cross workgroups (and XCDs, whose L2s are not coherent with
    // each other) through device-scope relaxed atomics: such stores write
    // through and such loads bypass the local caches, so no cache-wide
    // write-back or invalidate is needed.  Order: my stores complete (the
    // barrier waits for them), then one arrival count per workgroup; the
    // workgroup that counts splitk-1 earlier arrivals sums all tiles in split
    // order, so the result does not depend on arrival order.
    float* tile = p.ws + ((int64_t)split * NCH + nc) * (MT * 1024);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int e = 0; e < 2; ++e)
        __hip_atomic_store(tile + mt * 1024 + (idx0 + e) * 64 + l, sum[mt][e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // a workgroup barrier alone does not wait for outstanding global stores
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0)
      s_last = (__hip_atomic_fetch_add(&p.tickets[nc], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (unsigned)(p.splitk - 1));
    __syncthreads();
    if (!s_last) return;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        float t = 0.f;
        for (int sp = 0; sp < p.splitk; ++sp)
          t += __hip_atomic_load(p.ws + ((int64_t)sp * NCH + nc) * (MT * 1024) + mt * 1024 + (idx0 + e) * 64 + l,
                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sum[mt][e] = t;
      }
    if (tid == 0) __hip_atomic_store(&p.tickets[nc], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
  }
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = mt * 16 + i16;
    if (m < p.M)
      *reinterpret_cast<uint32_t*>(p.C + (int64_t)m * p.N + ncol) = pack_out<ROUTE>(sum[mt][0], sum[mt][1]);
  }
}

#define QG_CAT2(a, b) a##b
#define QG_CAT(a, b) QG_CAT2(a, b)

template <int ROUTE>
static int launch_route(const GemmParams& p, int mt, hipStream_t st) {
  dim3 grid((unsigned)(p.N / TILE_N), (unsigned)p.splitk), block(SMALL_WAVES * 64);
  switch (mt) {
    case 1: hipLaunchKernelGGL((small_kernel<QG_WT, ROUTE, 1>), grid, block, 0, st, p); break;
    case 2: hipLaunchKernelGGL((small_kernel<QG_WT, ROUTE, 2>), grid, block, 0, st, p); break;
    case 4: hipLaunchKernelGGL((small_kernel<QG_WT, ROUTE, 4>), grid, block, 0, st, p); break;
    default: return QG_EINVAL;
  }
  return hipGetLastError() == hipSuccess ? QG_OK : QG_EHIP;
}

int QG_CAT(small_launch_wt, QG_WT)(const GemmParams& p, int route, int mt, hipStream_t st) {
  return route == ROUTE_F16 ? launch_route<ROUTE_F16>(p, mt, st) : launch_route<ROUTE_BF16>(p, mt, st);
}

}  // namespace qg
