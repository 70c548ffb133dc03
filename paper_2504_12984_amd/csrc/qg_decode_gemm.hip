// Decode-sized matmul, M <= 64 (one, two or four tiles of 16 rows): the weights are streamed from HBM exactly once
// and the kernel is built to keep that stream saturated.
//
// One workgroup of NW wavefronts owns one 64-column strip of W and one slab of
// K; wavefront w takes every NW-th 128x64 chunk of the slab.  A wavefront keeps
// DEPTH chunks in flight at all times in a ring of registers (the software
// pipelining the paper calls essential, Sections "An Example of Tilus Program"
// and "End-to-End Performance"): per chunk BITS 16-byte loads of packed codes,
// four 16-byte loads of A (one per k-step, L2-resident), one load each of
// scales and zero-points.  The steady-state loop has no branches and refills a
// ring entry right after it has been consumed, so the compiler waits on exact
// outstanding-load counts instead of draining the queue.
// Codes are unpacked in registers and fed to the 16x16x32 matrix instruction
// with W as the row operand (the paper's load -> reinterpret -> cast -> mma
// pipeline, Section "Key Ideas", with no layout conversion and no trip through
// LDS).  The K reduction runs inside the MFMA (across the four 8-wide k-blocks
// of lanes), then across the wavefronts through LDS, then -- when K is also
// split over workgroups -- through fp32 partial tiles summed in split order by
// the last workgroup to arrive (the k-dimension parallelisation the paper names
// in Section "End-to-End Performance").
// Compiled once per weight type (QG_WT).
// QG_DBG_NODECODE / NOMFMA / NOSZ / NOREDUCE (never defined by the build) each cut one
// stage out for timing experiments -- results are wrong with them; QG_SZ_BCAST and
// QG_W_FIRST are two measured-and-rejected orderings of the scale and weight loads.
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

// Weights are used once: load them with the streaming (non-temporal) policy so that
// they do not push the re-used A rows out of the vector cache and L2 (measured:
// 5-10 % shorter kernels at 4..8 bits, M = 16).
__device__ __forceinline__ uint4 stream_load(const uint4* p) {
  u4_t v = __builtin_nontemporal_load(reinterpret_cast<const u4_t*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}

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

// MX: the scales are 8-bit exponents, one per 32 rows and column (GPC = 4), applied by the
// hardware converts of the e2m1 / e4m3 types; there are no zero-points.
template <int WT, int ROUTE, int GPC, int NW, int DEPTH, int MT, int NS = 1, bool MX = false>
__global__ __launch_bounds__(NW * 64) void decode_kernel(GemmParams p) {
  // NS adjacent strips per workgroup, NK wavefronts along K for each: wavefront w
  // works on strip w % NS and takes every NK-th chunk of the slab starting at
  // w / NS, so the NS wavefronts with the same w / NS walk the same K range at the
  // same pace and find each other's A rows in the vector cache.
  constexpr int NK = NW / NS;
  static_assert(NW % NS == 0 && 16 % NK == 0, "wavefront grid");
  typedef Decoder<WT, ROUTE> D;
  constexpr int BITS = D::BITS, RAW = D::RAW;

  const int tid = threadIdx.x, l = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int b = l >> 4, i16 = l & 15;
  const int ws = w % NS, wk = w / NS;                       // my strip and K position inside the workgroup
  const int nc = blockIdx.x * NS + ws, split = blockIdx.y;
  const int KC = p.K / TILE_K, NCH = p.N / TILE_N;
  const int c0 = split * p.chunks_per_split;
  const int c1 = min(KC, c0 + p.chunks_per_split);
  const int mine = (c1 - c0 > wk) ? (c1 - c0 - wk + NK - 1) / NK : 0;
  const int n0 = TILE_N * nc + 4 * i16;

  const uint4* wstrip = reinterpret_cast<const uint4*>(p.W + (int64_t)nc * KC * (1024 * BITS)) + l;
  // MT tiles of 16 rows; rows past M re-read row M-1, their results are never stored
  const uint16_t* arow[MT];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) arow[mt] = p.A + (int64_t)min(mt * 16 + i16, p.M - 1) * p.K + 8 * b;
  // no zero-points: read (valid) scale bytes instead and mask them away
  const uint8_t* zbase = p.Z ? p.Z : reinterpret_cast<const uint8_t*>(p.S);
  const uint32_t zmask = p.Z ? 0xffffffffu : 0u;

  struct Stage {
    uint32_t r[RAW];
    u4_t a[MT][4];
    uint2 s[GPC];          // GPC groups per chunk (group size 128 or more: 1; 64: 2; 32: 4)
    uint32_t z[GPC];
  };
  Stage st[DEPTH];

  auto issue = [&](auto Sc, int c) __attribute__((always_inline)) {
    constexpr int S = decltype(Sc)::value;
    Stage& s = st[S];
    __builtin_amdgcn_sched_barrier(0);         // stay below the last use of the entry being refilled,
                                               // so that the refill reuses the same registers
#ifndef QG_W_FIRST
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < 4; ++j) s.a[mt][j] = *reinterpret_cast<const u4_t*>(arow[mt] + c * TILE_K + 32 * j);
#endif
    const uint4* src = wstrip + (int64_t)c * (64 * BITS);
#pragma unroll
    for (int i = 0; i < BITS; ++i) {
      uint4 q = stream_load(src + i * 64);
      s.r[4 * i + 0] = q.x; s.r[4 * i + 1] = q.y; s.r[4 * i + 2] = q.z; s.r[4 * i + 3] = q.w;
    }
#ifdef QG_DBG_NOSZ
#pragma unroll
    for (int g = 0; g < GPC; ++g) { s.s[g] = make_uint2(0x3c003c00u, 0x3c003c00u); s.z[g] = 0x04040404u; }
    __builtin_amdgcn_sched_barrier(0);
    return;
#endif
    const int g0 = (GPC > 1) ? GPC * c : ((c >> p.gshift) & p.gmask);
    if constexpr (D::IS_LUT) {   // codebook indices: scales only
#pragma unroll
      for (int g = 0; g < GPC; ++g) s.s[g] = *reinterpret_cast<const uint2*>(p.S + (int64_t)(g0 + g) * p.N + n0);
      __builtin_amdgcn_sched_barrier(0);
      return;
    }
    if constexpr (MX) {          // four scale bytes (the lane's columns) per block of 32 rows, kept in the zero-point slot
#pragma unroll
      for (int g = 0; g < GPC; ++g)
        s.z[g] = *reinterpret_cast<const uint32_t*>(reinterpret_cast<const uint8_t*>(p.S) + (int64_t)(g0 + g) * p.N + n0);
      __builtin_amdgcn_sched_barrier(0);
      return;
    }
#ifdef QG_SZ_BCAST
    if (b == 0) {
#endif
#pragma unroll
    for (int g = 0; g < GPC; ++g) {
      s.s[g] = *reinterpret_cast<const uint2*>(p.S + (int64_t)(g0 + g) * p.N + n0);
      s.z[g] = *reinterpret_cast<const uint32_t*>(zbase + (int64_t)(g0 + g) * p.N + n0);
    }
#ifdef QG_SZ_BCAST
    }
#endif
#ifdef QG_W_FIRST
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int j = 0; j < 4; ++j) s.a[mt][j] = *reinterpret_cast<const u4_t*>(arow[mt] + c * TILE_K + 32 * j);
#endif
    __builtin_amdgcn_sched_barrier(0);
  };

  f4_t acc[MT][4];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = (f4_t){0.f, 0.f, 0.f, 0.f};

  typename D::Uniform u;
  u.init();
  auto compute = [&](auto Sc) __attribute__((always_inline)) {
    constexpr int S = decltype(Sc)::value;
    Stage& s = st[S];
    if constexpr (MX) {
      static_assert(GPC == 4, "one scale block per k-step");
      static_for<4>([&](auto Jc) __attribute__((always_inline)) {
        constexpr int J = decltype(Jc)::value;
        MxConsts mx;
        mx.make(s.z[J]);
        static_for<4>([&](auto NTc) __attribute__((always_inline)) {
          constexpr int NT = decltype(NTc)::value;
          uint32_t o[4];
          frag_mx<WT, ROUTE == ROUTE_BF16, J, NT>(s.r, mx, o);
          const u4_t wf = {o[0], o[1], o[2], o[3]};
#pragma unroll
          for (int mt = 0; mt < MT; ++mt) acc[mt][NT] = mfma16<ROUTE>(wf, s.a[mt][J], acc[mt][NT]);
        });
      });
      return;
    }
    typename D::Consts gc[GPC];
#ifdef QG_SZ_BCAST
    {
      const int ba = 4 * i16;
#pragma unroll
      for (int g = 0; g < GPC; ++g) {
        s.s[g].x = __builtin_amdgcn_ds_bpermute(ba, s.s[g].x); s.s[g].y = __builtin_amdgcn_ds_bpermute(ba, s.s[g].y);
        s.z[g] = __builtin_amdgcn_ds_bpermute(ba, s.z[g]);
      }
    }
#endif
#pragma unroll
    for (int g = 0; g < GPC; ++g) D::make_consts(gc[g], s.s[g], D::IS_LUT ? 0u : (s.z[g] & zmask), p.zbias, p.scale_bf16);
    static_for<4>([&](auto Jc) __attribute__((always_inline)) {
      constexpr int J = decltype(Jc)::value;
      static_for<4>([&](auto NTc) __attribute__((always_inline)) {
        constexpr int NT = decltype(NTc)::value;
        uint32_t o[4];
#ifdef QG_DBG_NODECODE
        o[0] = s.r[(J * 4 + NT) % RAW]; o[1] = s.r[(J * 4 + NT + 1) % RAW]; o[2] = s.r[(J * 4 + NT + 2) % RAW]; o[3] = s.r[(J * 4 + NT + 3) % RAW] ^ s.s[0].x ^ s.z[0];
#else
        D::template frag<J, NT>(s.r, gc[J * GPC / 4], u, o);          // k-step J lies in group J*GPC/4 of the chunk
#endif
        const u4_t wf = {o[0], o[1], o[2], o[3]};      // unpacked once, used by every row tile
#ifdef QG_DBG_NOMFMA
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt][NT][0] += __builtin_bit_cast(float, wf.x ^ wf.y ^ wf.z ^ wf.w ^ s.a[mt][J].x ^ s.a[mt][J].w);
#else
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt][NT] = mfma16<ROUTE>(wf, s.a[mt][J], acc[mt][NT]);
#endif
      });
    });
  };

  auto chunk_of = [&](int i) __attribute__((always_inline)) { return c0 + wk + min(i, mine - 1) * NK; };

  // LDS: the reduction buffer after the main loop; during it, for codebook indices, the
  // replicated lookup table (built by all wavefronts while the first loads are in flight)
  constexpr int RED_BYTES = NW * 16 * 64 * 4;
  constexpr int LUT_BYTES = [] { if constexpr (D::IS_LUT) return D::TABLE_DWORDS * 4 + 512; else return 0; }();
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[RED_BYTES > LUT_BYTES ? RED_BYTES : LUT_BYTES];

  static_assert(!D::IS_LUT || NW * 64 >= 256, "one level per thread");
  uint32_t my_level = 0;
  if constexpr (D::IS_LUT) my_level = D::fetch(p.T, tid);
  // prologue: DEPTH chunks in flight (past-the-end stages re-load my last chunk)
  if (mine > 0)
    static_for<DEPTH>([&](auto Sc) __attribute__((always_inline)) { issue(Sc, chunk_of(decltype(Sc)::value)); });
  if constexpr (D::IS_LUT) {
    uint32_t* table = reinterpret_cast<uint32_t*>(lds_raw);
    D::build(table, reinterpret_cast<uint16_t*>(lds_raw + D::TABLE_DWORDS * 4), my_level, tid, NW * 64);
    u.set_table(table, l);
  }
  if (mine > 0) {
    int i = 0;
    // steady state: no branches, so the compiler can wait on exact load counts
    for (; i + 2 * DEPTH <= mine; i += DEPTH)
      static_for<DEPTH>([&](auto Sc) __attribute__((always_inline)) {
        compute(Sc);
        issue(Sc, chunk_of(i + decltype(Sc)::value + DEPTH));
      });
    // drain
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
  if constexpr (D::IS_LUT) __syncthreads();                // every wavefront is done with the table
  float* red = reinterpret_cast<float*>(lds_raw);          // [NW][16 column offsets][64 lanes]
  int* s_last = reinterpret_cast<int*>(red);               // reused once the sums are in registers
  constexpr int PER = 16 / NK;                             // column offsets per thread
  const int idx0 = PER * wk;
  float sum[MT][PER];
#ifdef QG_DBG_NOREDUCE
#pragma unroll
  for (int mt = 0; mt < MT; ++mt)
#pragma unroll
    for (int e = 0; e < PER; ++e) sum[mt][e] = acc[mt][e & 3][(e >> 2) & 3];
  if (false)
#endif
  // lanes whose row is past M carry nothing: they stay out of the LDS traffic, of the
  // split-K exchange and of the final store
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
        for (int kk = 0; kk < NK; ++kk) t += red[((kk * NS + ws) * 16 + idx0 + e) * 64 + l];
        sum[mt][e] = t;
      }
    }
  }

  if (p.splitk > 1) {
    // Partial tiles cross workgroups (and XCDs, whose L2s are not coherent with
    // each other) through device-scope relaxed atomics: such stores write
    // through and such loads bypass the local caches, so no cache-wide
    // write-back or invalidate is needed.  Order: my stores complete, barrier,
    // one arrival count per workgroup; the workgroup that counts splitk-1
    // earlier arrivals sums all tiles in split order, so the result does not
    // depend on arrival order.
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
    // all loads of a split are issued before the first add (independent accumulators)
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
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    const int m = mt * 16 + i16;
    if (m < p.M) {
      uint16_t* dst = p.C + (int64_t)m * p.N + TILE_N * nc + 16 * b + idx0;
      if constexpr (PER == 1) {
        dst[0] = (uint16_t)(pack_out<ROUTE>(sum[mt][0], 0.f) & 0xffffu);
      } else {
#pragma unroll
        for (int e = 0; e + 1 < PER; e += 2) *reinterpret_cast<uint32_t*>(dst + e) = pack_out<ROUTE>(sum[mt][e], sum[mt][e + 1]);
      }
    }
  }
}

#define QG_CAT2(a, b) a##b
#define QG_CAT(a, b) QG_CAT2(a, b)

template <int ROUTE, int GPC, int NW, int DEPTH, int MT, int NS = 1, bool MX = false>
static int launch_cfg(const GemmParams& p, hipStream_t st) {
  if ((p.N / TILE_N) % NS) return QG_EINVAL;
  auto kern = decode_kernel<QG_WT, ROUTE, GPC, NW, DEPTH, MT, NS, MX>;
  dim3 grid((unsigned)(p.N / TILE_N / NS), (unsigned)p.splitk), block(NW * 64);
  hipLaunchKernelGGL(kern, grid, block, 0, st, p);
  return hipGetLastError() == hipSuccess ? QG_OK : QG_EHIP;
}

// variant = 10 * (row tiles: 1, 2, 4) + (0: 8 wavefronts per strip, 1: 4 wavefronts, 2: 16 wavefronts)
template <int ROUTE, int GPC>
static int launch_variant(const GemmParams& p, int variant, hipStream_t st) {
  if constexpr (GPC == 4 && (QG_WT == 9 || QG_WT == 13)) {
    if (p.scale_e8m0) {              // block-scaled e2m1 / e4m3: every arrangement, scaled converts
      switch (variant) {
        case 10: return launch_cfg<ROUTE, 4, 8, 2, 1, 1, true>(p, st);
        case 11: return launch_cfg<ROUTE, 4, 4, 2, 1, 1, true>(p, st);
        case 12: return launch_cfg<ROUTE, 4, 16, 2, 1, 1, true>(p, st);
        case 14: return launch_cfg<ROUTE, 4, 8, 2, 1, 2, true>(p, st);
        case 15: return launch_cfg<ROUTE, 4, 16, 2, 1, 2, true>(p, st);
        case 16: return launch_cfg<ROUTE, 4, 16, 2, 1, 4, true>(p, st);
        case 21: return launch_cfg<ROUTE, 4, 4, 2, 2, 1, true>(p, st);
        case 26: return launch_cfg<ROUTE, 4, 4, 2, 2, 2, true>(p, st);
        case 46: return launch_cfg<ROUTE, 4, 4, 2, 4, 2, true>(p, st);
        case 41: return launch_cfg<ROUTE, 4, 4, 2, 4, 1, true>(p, st);
        default: return QG_EINVAL;
      }
    }
  }
  if (p.scale_e8m0) return QG_EUNSUPPORTED;
  if constexpr (GPC == 4) {          // group size 32: the 4-wavefront arrangements only
    switch (variant) {
      case 11: return launch_cfg<ROUTE, 4, 4, 2, 1>(p, st);
      case 21: return launch_cfg<ROUTE, 4, 4, 2, 2>(p, st);
      case 41: return launch_cfg<ROUTE, 4, 4, 2, 4>(p, st);
      default: return QG_EINVAL;
    }
  } else {
  switch (variant) {
    case 10: return launch_cfg<ROUTE, GPC, 8, 2, 1>(p, st);
    case 11: return launch_cfg<ROUTE, GPC, 4, 2, 1>(p, st);
    case 12: return launch_cfg<ROUTE, GPC, 16, 2, 1>(p, st);
    case 14: return launch_cfg<ROUTE, GPC, 8, 2, 1, 2>(p, st);     // 2 strips x 4
    case 15: return launch_cfg<ROUTE, GPC, 16, 2, 1, 2>(p, st);    // 2 strips x 8
    case 16: return launch_cfg<ROUTE, GPC, 16, 2, 1, 4>(p, st);    // 4 strips x 4
    case 21: return launch_cfg<ROUTE, GPC, 4, 2, 2>(p, st);
    case 26: return launch_cfg<ROUTE, GPC, 4, 2, 2, 2>(p, st);     // 2 row tiles, 2 strips x 2
    case 46: return launch_cfg<ROUTE, GPC, 4, 2, 4, 2>(p, st);     // 4 row tiles, 2 strips x 2
    case 41: return launch_cfg<ROUTE, GPC, 4, 2, 4>(p, st);
    default: return QG_EINVAL;
  }
  }
}

// number of wavefronts along K per strip of a variant (the host sizes split-K with it)
int QG_CAT(decode_waves_wt, QG_WT)(int variant) {
  switch (variant) {
    case 10: return 8;
    case 12: return 16;
    case 14: case 16: return 4;
    case 26: case 46: return 2;
    case 15: return 8;
    default: return 4;
  }
}

int QG_CAT(decode_launch_wt, QG_WT)(const GemmParams& p, int route, int variant, hipStream_t st) {
  const int gpc = (p.group == 32) ? 4 : (p.group == 64) ? 2 : 1;       // groups per 128-row chunk
  if (route == ROUTE_F16)
    return gpc == 4 ? launch_variant<ROUTE_F16, 4>(p, variant, st)
         : gpc == 2 ? launch_variant<ROUTE_F16, 2>(p, variant, st) : launch_variant<ROUTE_F16, 1>(p, variant, st);
  return gpc == 4 ? launch_variant<ROUTE_BF16, 4>(p, variant, st)
       : gpc == 2 ? launch_variant<ROUTE_BF16, 2>(p, variant, st) : launch_variant<ROUTE_BF16, 1>(p, variant, st);
}

}  // namespace qg
