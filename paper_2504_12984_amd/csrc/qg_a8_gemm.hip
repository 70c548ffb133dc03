// Matmul with int8 activations:  C[m,n] = a_scale[m] * sum_g s[g,n] * sum_{k in g} A8[m,k] * (q[k,n] - z[g,n]).
//
// The paper lists int8 beside float16 and bfloat16 as an activation type it supports (Section
// "Arbitrary Data Type Support") and says no more; the form above is this library's reading:
// integer weights only, exact integer sums inside a scale group (the integer matrix
// instruction), the group's weight scale applied to that sum, one fp32 scale per row of A.
//
// Same streaming design as the 16-bit-activation kernel for small M (the weights are read from
// HBM once, each wavefront keeps a ring of two 128x64 chunks in registers, K is reduced inside
// the matrix instruction, then across wavefronts in LDS, then -- if K is also split over
// workgroups -- through fp32 partial tiles and an arrival counter), on the third device layout:
// a lane's 16*BITS bytes are FOUR parallel byte streams (byte lane e of every register), quad t
// occupies bits [t*BITS, (t+1)*BITS) of each, so one shift + one mask turn a register into
// four int8 operands of v_mfma_i32_16x16x64_i8 at once (two more operations when the codes
// straddle a byte).  Codes stay unsigned (intk is stored offset-binary); the zero-point term is
// taken out afterwards through the row sums of A, which one extra matrix instruction with an
// all-ones operand delivers:  sum a (q - z) = sum a q - z sum a.
// Rows beyond 64 are served in blocks of 64 by the host (a first slice: no LDS-staged tile
// kernel for prefill-sized M yet).  Compiled once per code width (QG_BITS).
#include "qg_common.h"
#include "qg_static_for.h"

#ifndef QG_BITS
#error "compile with -DQG_BITS=<1..8>"
#endif

namespace qg {

typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
typedef int i4_t __attribute__((ext_vector_type(4)));
typedef float f2_t __attribute__((ext_vector_type(2)));
typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
typedef __bf16 b2_t __attribute__((ext_vector_type(2)));

// (a & mask) | orv as a plain expression (the compiler selects v_and_or_b32 itself).  The
// inline-asm form that the 16-bit kernels use -- there its result passes through further vector
// arithmetic -- gave wrong operands in lanes 0..15 of one quad when its result fed the matrix
// instruction directly; with the plain expression every code of every width decodes exactly.
__device__ __forceinline__ uint32_t and_or_a8(uint32_t a, uint32_t mask, uint32_t orv) { return (a & mask) | orv; }

// Quad T of the lane: four codes, one per byte lane, as four unsigned bytes of one register.
template <int BITS, int T>
__device__ __forceinline__ uint32_t quad(const uint32_t (&r)[4 * BITS]) {
  constexpr int bit = T * BITS, h = bit >> 3, p = bit & 7;
  constexpr uint32_t CODE = (1u << BITS) - 1u;
  constexpr uint32_t ALL = 0x01010101u;
  if constexpr (BITS == 8) {
    return r[h];
  } else if constexpr (p + BITS <= 8) {
    if constexpr (p == 0) return r[h] & (CODE * ALL);
    else return (r[h] >> p) & (CODE * ALL);
  } else {
    constexpr int n1 = 8 - p;                                   // bits of the code in register h
    constexpr uint32_t LOW = ((1u << n1) - 1u) * ALL, HIGH = (CODE & ~((1u << n1) - 1u)) * ALL;
    const uint32_t x = (r[h] >> p) & LOW;
    return and_or_a8(r[h + 1] << n1, HIGH, x);
  }
}

__device__ __forceinline__ uint32_t pack_out_a8(float lo, float hi, int out_bf16) {
  f2_t f = {lo, hi};
  const uint32_t h = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, h2_t));
  const uint32_t b = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, b2_t));
  return out_bf16 ? b : h;
}

template <int BITS, int GPC, int NW, int MT>
__global__ __launch_bounds__(NW * 64) void a8_kernel(A8Params p) {
  constexpr int RAW = 4 * BITS, DEPTH = 2;
  constexpr int ZOFF = (BITS == 8) ? 128 : 0;     // 8-bit codes enter the signed instruction as q - 128
  static_assert(16 % NW == 0, "wavefronts along K");

  const int tid = threadIdx.x, l = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int b = l >> 4, i16 = l & 15;
  const int nc = blockIdx.x, split = blockIdx.y;
  const int KC = p.K / TILE_K, NCH = p.N / TILE_N;
  const int c0 = split * p.chunks_per_split;
  const int c1 = min(KC, c0 + p.chunks_per_split);
  const int mine = (c1 - c0 > w) ? (c1 - c0 - w + NW - 1) / NW : 0;
  const int n16 = TILE_N * nc + 16 * b;           // the 16 output columns this lane accumulates

  const uint4* wstrip = reinterpret_cast<const uint4*>(p.W + (int64_t)nc * KC * (1024 * BITS)) + l;
  // MT tiles of 16 rows; rows past M re-read row M-1, their results are never stored
  const int8_t* arow[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) arow[mt] = p.A + (int64_t)min(mt * 16 + i16, p.M - 1) * p.K + 16 * b;
  // no zero-points: read (valid) scale bytes instead and mask them away
  const uint8_t* zbase = (p.Z ? p.Z : reinterpret_cast<const uint8_t*>(p.S)) + n16;
  const uint32_t zmask = p.Z ? 0xffu : 0u;
  const uint16_t* sbase = p.S + n16;

  struct Stage {
    uint32_t r[RAW];
    u4_t a[MT][2];          // 16 int8 of my row for each of the two 64-wide k-steps
    u4_t s[GPC][2];         // 16 scales
    u4_t z[GPC];            // 16 zero-points
  };
  Stage st[DEPTH];

  auto issue = [&](auto Sc, int c) __attribute__((always_inline)) {
    constexpr int S = decltype(Sc)::value;
    Stage& s = st[S];
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < 2; ++j) s.a[mt][j] = *reinterpret_cast<const u4_t*>(arow[mt] + c * TILE_K + 64 * j);
    const uint4* src = wstrip + (int64_t)c * (64 * BITS);
#pragma unroll
    for (int i = 0; i < BITS; ++i) {
      u4_t q = __builtin_nontemporal_load(reinterpret_cast<const u4_t*>(src + i * 64));
      s.r[4 * i + 0] = q.x; s.r[4 * i + 1] = q.y; s.r[4 * i + 2] = q.z; s.r[4 * i + 3] = q.w;
    }
    const int g0 = (GPC > 1) ? GPC * c : ((c >> p.gshift) & p.gmask);
#pragma unroll
    for (int g = 0; g < GPC; ++g) {
      const u4_t* sp = reinterpret_cast<const u4_t*>(sbase + (int64_t)(g0 + g) * p.N);
      s.s[g][0] = sp[0]; s.s[g][1] = sp[1];
      s.z[g] = *reinterpret_cast<const u4_t*>(zbase + (int64_t)(g0 + g) * p.N);
    }
    __builtin_amdgcn_sched_barrier(0);
  };

  float acc[MT][4][4];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int r = 0; r < 4; ++r) acc[mt][nt][r] = 0.f;

  const uint32_t bf_sel = p.scale_bf16 ? 0xffffffffu : 0u;
  const i4_t ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};

  auto compute = [&](auto Sc) __attribute__((always_inline)) {
    constexpr int S = decltype(Sc)::value;
    Stage& s = st[S];
    static_for<GPC>([&](auto Gc) __attribute__((always_inline)) {
      constexpr int G = decltype(Gc)::value;
      i4_t dq[MT][4], rs[MT];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt) {
        rs[mt] = (i4_t){0, 0, 0, 0};
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) dq[mt][nt] = (i4_t){0, 0, 0, 0};
      }
      constexpr int J0 = (GPC == 2) ? G : 0, J1 = (GPC == 2) ? G + 1 : 2;   // the k-steps of this group
      static_for<J1 - J0>([&](auto Jc) __attribute__((always_inline)) {
        constexpr int J = J0 + decltype(Jc)::value;
        static_for<4>([&](auto NTc) __attribute__((always_inline)) {
          constexpr int NT = decltype(NTc)::value;
          constexpr int T0 = (J * 4 + NT) * 4;
          uint32_t q0 = quad<BITS, T0 + 0>(s.r), q1 = quad<BITS, T0 + 1>(s.r);
          uint32_t q2 = quad<BITS, T0 + 2>(s.r), q3 = quad<BITS, T0 + 3>(s.r);
          if constexpr (BITS == 8) { q0 ^= 0x80808080u; q1 ^= 0x80808080u; q2 ^= 0x80808080u; q3 ^= 0x80808080u; }
          const i4_t wq = {(int)q0, (int)q1, (int)q2, (int)q3};
#pragma unroll
          for (int mt = 0; mt < MT; ++mt)
            dq[mt][NT] = __builtin_amdgcn_mfma_i32_16x16x64_i8(wq, __builtin_bit_cast(i4_t, s.a[mt][J]), dq[mt][NT], 0, 0, 0);
        });
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
          rs[mt] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, __builtin_bit_cast(i4_t, s.a[mt][J]), rs[mt], 0, 0, 0);
      });
      // scale of column n16 + 4r + nt times (the integer sum minus zero-point times row sum)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int c = 4 * r + nt;
          const uint32_t sw = s.s[G][c >> 3][(c & 7) >> 1];
          const uint32_t s16 = (c & 1) ? (sw >> 16) : (sw & 0xffffu);
          const uint32_t from_h = __builtin_bit_cast(uint32_t, (float)__builtin_bit_cast(_Float16, (uint16_t)s16));
          const float sf = __builtin_bit_cast(float, ((s16 << 16) & bf_sel) | (from_h & ~bf_sel));
          const int zq = (int)((s.z[G][c >> 2] >> (8 * (c & 3))) & zmask) + p.zbias - ZOFF;
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) {
            const int t = dq[mt][nt][r] - zq * rs[mt][r];
            acc[mt][nt][r] = __builtin_fmaf(sf, (float)t, acc[mt][nt][r]);
          }
        }
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

  // ---- reduce over the NW wavefronts through LDS, one 16-row tile at a time -----------------
  __shared__ float red[NW * 16 * 64];                      // [NW][16 column offsets][64 lanes]
  int* s_last = reinterpret_cast<int*>(red);               // reused once the sums are in registers
  constexpr int PER = 16 / NW;                             // column offsets per thread
  const int idx0 = PER * w;
  float sum[MT][PER];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const bool row_ok = mt * 16 + i16 < p.M;
    if (mt) __syncthreads();
    if (row_ok) {
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[(w * 16 + 4 * r + nt) * 64 + l] = acc[mt][nt][r];   // column offset 4r + nt
    }
    __syncthreads();
#pragma unroll
    for (int e = 0; e < PER; ++e) sum[mt][e] = 0.f;
    if (row_ok) {
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        float t = 0.f;
#pragma unroll
        for (int kk = 0; kk < NW; ++kk) t += red[(kk * 16 + idx0 + e) * 64 + l];
        sum[mt][e] = t;
      }
    }
  }

  if (p.splitk > 1) {
    // Partial tiles cross workgroups through device-scope relaxed atomics (write-through
    // stores, cache-bypassing loads) and one arrival counter per strip; the last arriver
    // sums the slabs in slab order, so the result does not depend on arrival order.
    float* tile = p.ws + ((int64_t)split * NCH + nc) * (MT * 1024);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
      if (mt * 16 + i16 < p.M) {
#pragma unroll
        for (int e = 0; e < PER; ++e)
          __hip_atomic_store(tile + mt * 1024 + (idx0 + e) * 64 + l, sum[mt][e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // a workgroup barrier alone does not wait for global stores
    __syncthreads();
    if (tid == 0)
      *s_last = (__hip_atomic_fetch_add(&p.tickets[blockIdx.x], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == (unsigned)(p.splitk - 1));
    __syncthreads();
    if (!*s_last) return;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int e = 0; e < PER; ++e) sum[mt][e] = 0.f;
    for (int sp = 0; sp < p.splitk; ++sp) {
      const float* src = p.ws + ((int64_t)sp * NCH + nc) * (MT * 1024);
      float v[MT][PER];
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int e = 0; e < PER; ++e) {
          v[mt][e] = 0.f;
          if (mt * 16 + i16 < p.M)
            v[mt][e] = __hip_atomic_load(src + mt * 1024 + (idx0 + e) * 64 + l, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int e = 0; e < PER; ++e) sum[mt][e] += v[mt][e];
    }
    if (tid == 0) __hip_atomic_store(&p.tickets[blockIdx.x], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
  }
  // ---- row scale, one rounding to the output type, store -----------------------------------
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = mt * 16 + i16;
    if (m < p.M) {
      const float as = p.a_scale ? p.a_scale[m] : 1.0f;
      uint16_t* dst = p.C + (int64_t)m * p.N + n16 + idx0;
      if constexpr (PER == 1) {
        dst[0] = (uint16_t)(pack_out_a8(sum[mt][0] * as, 0.f, p.out_bf16) & 0xffffu);
      } else {
#pragma unroll
        for (int e = 0; e + 1 < PER; e += 2)
          *reinterpret_cast<uint32_t*>(dst + e) = pack_out_a8(sum[mt][e] * as, sum[mt][e + 1] * as, p.out_bf16);
      }
    }
  }
}

#define QG_CAT2(a, b) a##b
#define QG_CAT(a, b) QG_CAT2(a, b)

template <int GPC, int NW, int MT>
static int launch_a8(const A8Params& p, hipStream_t st) {
  auto kern = a8_kernel<QG_BITS, GPC, NW, MT>;
  dim3 grid((unsigned)(p.N / TILE_N), (unsigned)p.splitk), block(NW * 64);
  hipLaunchKernelGGL(kern, grid, block, 0, st, p);
  return hipGetLastError() == hipSuccess ? QG_OK : QG_EHIP;
}

// waves: 8 wavefronts per strip, or 4 (short K); mt: row tiles 1, 2 or 4
int QG_CAT(a8_launch_bits, QG_BITS)(const A8Params& p, int waves, int mt, hipStream_t st) {
  const int gpc = (p.group == 64) ? 2 : 1;
#define QG_A8(GPC_, NW_, MT_) if (gpc == GPC_ && waves == NW_ && mt == MT_) return launch_a8<GPC_, NW_, MT_>(p, st);
  QG_A8(1, 8, 1) QG_A8(1, 8, 2) QG_A8(1, 8, 4) QG_A8(2, 8, 1) QG_A8(2, 8, 2) QG_A8(2, 8, 4)
  QG_A8(1, 4, 1) QG_A8(1, 4, 2) QG_A8(1, 4, 4) QG_A8(2, 4, 1) QG_A8(2, 4, 2) QG_A8(2, 4, 4)
#undef QG_A8
  return QG_EINVAL;
}

}  // namespace qg
