// Matrix-vector form of the decode-sized matmul (M <= 4), without the matrix cores: the measured
// alternative to the streaming kernel for the smallest batches.
//
// Same layout, same weight stream, same register ring as decode_kernel (one workgroup of NW
// wavefronts per 64-column strip and K-slab, wavefront w takes every NW-th 128x64 chunk, two
// chunks in flight), and the same in-register unpack.  What differs is the contraction: a lane
// keeps one fp32 partial sum per (row of A, own column) and adds to it with the two-element dot
// product instruction (v_dot2_f32_{f16,bf16}: a.lo*b.lo + a.hi*b.hi + c in fp32) -- one per
// operand register, so four vector instructions per k-step and column where the streaming
// kernel issues one matrix instruction per k-step and sub-tile.  The four lanes 16*b + i
// (k-blocks b = 0..3) hold partial sums of the same columns; they are added inside the wavefront
// with two lane permutes (xor 16, xor 32), then across the wavefronts through LDS, then -- when K
// is split over workgroups -- through the same fp32 partial tiles and arrival counters as the
// streaming kernel (the k-dimension parallelisation of Section "End-to-End Performance").
// For the bit-exact contract nothing changes: the products are formed from the same rounded
// weights, accumulated in fp32.
// Compiled once per weight type (QG_WT).
#include "qg_decode.h"
#include "qg_static_for.h"

#ifndef QG_WT
#error "compile with -DQG_WT=<weight type index>"
#endif

namespace qg {

typedef uint32_t u4_t __attribute__((ext_vector_type(4)));

template <int ROUTE>
__device__ __forceinline__ float dot2(uint32_t w, uint32_t a, float c) {
  if constexpr (ROUTE == ROUTE_F16) return __builtin_amdgcn_fdot2(as_h2(w), as_h2(a), c, false);
  else return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(b2_t, w), __builtin_bit_cast(b2_t, a), c, false);
}

template <int ROUTE>
__device__ __forceinline__ uint32_t pack_out2(float lo, float hi) {
  f2_t f = {lo, hi};
  if constexpr (ROUTE == ROUTE_F16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, h2_t));
  else return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, b2_t));
}

// MR = rows of A carried (1 or 4; rows past M repeat row M-1 and are never stored)
template <int WT, int ROUTE, int GPC, int NW, int MR>
__global__ __launch_bounds__(NW * 64) void gemv_kernel(GemmParams p) {
  typedef Decoder<WT, ROUTE> D;
  static_assert(!D::IS_LUT, "integer and float weight types only");
  constexpr int BITS = D::BITS, RAW = D::RAW, DEPTH = 2;

  const int tid = threadIdx.x, l = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = l >> 4, i16 = l & 15;
  const int nc = blockIdx.x, split = blockIdx.y;
  const int KC = p.K / TILE_K, NCH = p.N / TILE_N;
  const int c0 = split * p.chunks_per_split;
  const int c1 = min(KC, c0 + p.chunks_per_split);
  const int mine = (c1 - c0 > w) ? (c1 - c0 - w + NW - 1) / NW : 0;
  const int n0 = TILE_N * nc + 4 * i16;

  const uint4* wstrip = reinterpret_cast<const uint4*>(p.W + (int64_t)nc * KC * (1024 * BITS)) + l;
  const uint16_t* arow[MR];
#pragma unroll
  for (int mr = 0; mr < MR; ++mr) arow[mr] = p.A + (int64_t)min(mr, p.M - 1) * p.K + 8 * b;
  const uint8_t* zbase = p.Z ? p.Z : reinterpret_cast<const uint8_t*>(p.S);
  const uint32_t zmask = p.Z ? 0xffffffffu : 0u;

  struct Stage {
    uint32_t r[RAW];
    u4_t a[MR][4];         // the lane's 8 values of A per k-step: k = 32*j + 8*b .. +7
    uint2 s[GPC];
    uint32_t z[GPC];
  };
  Stage st[DEPTH];

  auto issue = [&](auto Sc, int c) __attribute__((always_inline)) {
    constexpr int S = decltype(Sc)::value;
    Stage& s = st[S];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int mr = 0; mr < MR; ++mr)
#pragma unroll
      for (int j = 0; j < 4; ++j) s.a[mr][j] = *reinterpret_cast<const u4_t*>(arow[mr] + c * TILE_K + 32 * j);
    const uint4* src = wstrip + (int64_t)c * (64 * BITS);
#pragma unroll
    for (int i = 0; i < BITS; ++i) {
      u4_t q = __builtin_nontemporal_load(reinterpret_cast<const u4_t*>(src + i * 64));
      s.r[4 * i + 0] = q.x; s.r[4 * i + 1] = q.y; s.r[4 * i + 2] = q.z; s.r[4 * i + 3] = q.w;
    }
    const int g0 = (GPC > 1) ? GPC * c : ((c >> p.gshift) & p.gmask);
#pragma unroll
    for (int g = 0; g < GPC; ++g) {
      s.s[g] = *reinterpret_cast<const uint2*>(p.S + (int64_t)(g0 + g) * p.N + n0);
      s.z[g] = *reinterpret_cast<const uint32_t*>(zbase + (int64_t)(g0 + g) * p.N + n0);
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  float acc[MR][4];
#pragma unroll
  for (int mr = 0; mr < MR; ++mr)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) acc[mr][nt] = 0.f;

  typename D::Uniform u;
  u.init();

  auto compute = [&](auto Sc) __attribute__((always_inline)) {
    constexpr int S = decltype(Sc)::value;
    Stage& s = st[S];
    typename D::Consts gc[GPC];
#pragma unroll
    for (int g = 0; g < GPC; ++g) D::make_consts(gc[g], s.s[g], s.z[g] & zmask, p.zbias, p.scale_bf16);
    static_for<4>([&](auto Jc) __attribute__((always_inline)) {
      constexpr int J = decltype(Jc)::value;
      static_for<4>([&](auto NTc) __attribute__((always_inline)) {
        constexpr int NT = decltype(NTc)::value;
        uint32_t o[4];
        D::template frag<J, NT>(s.r, gc[J * GPC / 4], u, o);      // the lane's 8 weights of column NT, k-step J
#pragma unroll
        for (int mr = 0; mr < MR; ++mr) {
          float t = acc[mr][NT];
          t = dot2<ROUTE>(o[0], s.a[mr][J].x, t);
          t = dot2<ROUTE>(o[1], s.a[mr][J].y, t);
          t = dot2<ROUTE>(o[2], s.a[mr][J].z, t);
          t = dot2<ROUTE>(o[3], s.a[mr][J].w, t);
          acc[mr][NT] = t;
        }
      });
    });
  };

  auto chunk_of = [&](int i) __attribute__((always_inline)) { return c0 + w + min(i, mine - 1) * NW; };

  if (mine > 0) {
    static_for<DEPTH>([&](auto Sc) __attribute__((always_inline)) { issue(Sc, chunk_of(decltype(Sc)::value)); });
    int i = 0;
    for (; i + 2 * DEPTH <= mine; i += DEPTH)
      static_for<DEPTH>([&](auto Sc) __attribute__((always_inline)) {
        compute(Sc);
        issue(Sc, chunk_of(i + decltype(Sc)::value + DEPTH));
      });
    static_for<DEPTH>([&](auto Sc) __attribute__((always_inline)) {
      constexpr int S = decltype(Sc)::value;
      if (i + S < mine) {
        compute(Sc);
        if (i + S + DEPTH < mine) issue(Sc, chunk_of(i + S + DEPTH));
      }
    });
    i += DEPTH;
    static_for<DEPTH>([&](auto Sc) __attribute__((always_inline)) {
      if (i + decltype(Sc)::value < mine) compute(Sc);
    });
  }

  // ---- inside the wavefront: the four k-blocks of lanes hold partial sums of the same columns ----
#pragma unroll
  for (int mr = 0; mr < MR; ++mr)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      float t = acc[mr][nt];
      t += __shfl_xor(t, 16);
      t += __shfl_xor(t, 32);
      acc[mr][nt] = t;                                   // every lane 16*b + i now has the sum for column 4*i + nt
    }

  // ---- across the wavefronts through LDS: red[w][mr][column 0..63] ----------------------------------
  __shared__ float red[NW * MR * 64];
  __shared__ int s_last;
  if (b == 0) {
#pragma unroll
    for (int mr = 0; mr < MR; ++mr)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) red[(w * MR + mr) * 64 + 4 * i16 + nt] = acc[mr][nt];
  }
  __syncthreads();
  // thread t < MR*64 owns output (row t / 64, column t % 64) from here on
  const bool owner = tid < MR * 64;
  const int orow = tid >> 6, ocol = tid & 63;
  float sum = 0.f;
  if (owner)
#pragma unroll
    for (int ww = 0; ww < NW; ++ww) sum += red[(ww * MR + orow) * 64 + ocol];

  if (p.splitk > 1) {
    // partial tiles cross workgroups through device-scope relaxed atomics, as in the streaming kernel
    float* tile = p.ws + ((int64_t)split * NCH + nc) * (MR * 64);
    if (owner && orow < p.M) __hip_atomic_store(tile + tid, sum, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (tid == 0)
      s_last = (__hip_atomic_fetch_add(&p.tickets[blockIdx.x], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (unsigned)(p.splitk - 1));
    __syncthreads();
    if (!s_last) return;
    sum = 0.f;
    if (owner && orow < p.M)
      for (int sp = 0; sp < p.splitk; ++sp)
        sum += __hip_atomic_load(p.ws + ((int64_t)sp * NCH + nc) * (MR * 64) + tid, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (tid == 0) __hip_atomic_store(&p.tickets[blockIdx.x], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  // store: two adjacent columns per even thread (the odd neighbour's sum comes over a lane permute)
  const float hi = __shfl_down(sum, 1);
  if (owner && orow < p.M && (ocol & 1) == 0)
    *reinterpret_cast<uint32_t*>(p.C + (int64_t)orow * p.N + TILE_N * nc + ocol) = pack_out2<ROUTE>(sum, hi);
}

#define QG_CAT2(a, b) a##b
#define QG_CAT(a, b) QG_CAT2(a, b)

template <int ROUTE, int GPC, int NW, int MR>
static int launch_gemv(const GemmParams& p, hipStream_t st) {
  dim3 grid((unsigned)(p.N / TILE_N), (unsigned)p.splitk), block(NW * 64);
  hipLaunchKernelGGL((gemv_kernel<QG_WT, ROUTE, GPC, NW, MR>), grid, block, 0, st, p);
  return hipGetLastError() == hipSuccess ? QG_OK : QG_EHIP;
}

template <int ROUTE, int GPC>
static int launch_gemv_shape(const GemmParams& p, int waves, hipStream_t st) {
  if (p.M > 4) return QG_EINVAL;
  // one row of A, or four (two and three rows ride in the four-row instantiation); 16 wavefronts per
  // strip exist for one row only (with four rows their ring does not fit the registers)
  if (p.M <= 1) {
    if (waves == 4) return launch_gemv<ROUTE, GPC, 4, 1>(p, st);
    if (waves == 8) return launch_gemv<ROUTE, GPC, 8, 1>(p, st);
    if (waves == 16) return launch_gemv<ROUTE, GPC, 16, 1>(p, st);
    return QG_EINVAL;
  }
  if (waves == 4) return launch_gemv<ROUTE, GPC, 4, 4>(p, st);
  if (waves == 8) return launch_gemv<ROUTE, GPC, 8, 4>(p, st);
  return QG_EINVAL;
}

// waves: wavefronts per strip (4, 8 or 16)
int QG_CAT(gemv_launch_wt, QG_WT)(const GemmParams& p, int route, int waves, hipStream_t st) {
  if (p.scale_e8m0) return QG_EUNSUPPORTED;
  const int gpc = (p.group == 32) ? 4 : (p.group == 64) ? 2 : 1;
  if (route == ROUTE_F16)
    return gpc == 4 ? launch_gemv_shape<ROUTE_F16, 4>(p, waves, st)
         : gpc == 2 ? launch_gemv_shape<ROUTE_F16, 2>(p, waves, st) : launch_gemv_shape<ROUTE_F16, 1>(p, waves, st);
  return gpc == 4 ? launch_gemv_shape<ROUTE_BF16, 4>(p, waves, st)
       : gpc == 2 ? launch_gemv_shape<ROUTE_BF16, 2>(p, waves, st) : launch_gemv_shape<ROUTE_BF16, 1>(p, waves, st);
}

}  // namespace qg
