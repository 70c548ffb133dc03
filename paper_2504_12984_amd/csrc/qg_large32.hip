// Prefill-sized matmul for the 32-row layout: LDS-staged A, register-resident W,
// 32x32x16 MFMA.
//
// A workgroup of 4 wavefronts computes a BM x 256 tile of C.  Wavefront w owns
// 64 columns: it loads its own 128x64 weight chunk straight from global memory
// into registers (BITS 16-byte loads per lane, one chunk ahead of use), unpacks
// it in registers and uses it as the row operand of the matrix instruction --
// the weights never pass through LDS and are never exchanged between lanes,
// which is the paper's weight pipeline (Section "Key Ideas", steps 1-4) with the
// shared-memory hop removed because every wavefront needs different columns.
// The BM x 128 slab of A for the same K range is shared by the four wavefronts
// through LDS (double-buffered per chunk, filled through a register ring four
// k-steps ahead), so each unpacked weight is used BM times and each weight is
// unpacked M/BM times in total.
// Why the 32x32x16 instruction: one wavefront per SIMD issues it back to back at
// the full matrix rate (the 16x16x32 form reaches about 82 % that way), and its 32
// cycles hide five vector instructions instead of two, which is what the
// in-register unpack needs.
// Workgroup ids are remapped so that the workgroups resident on one XCD (ids
// congruent mod 8) form 4 x 8 panels of tiles that share A and W in that XCD's L2.
// Compiled once per weight type (QG_WT).
#include "qg_decode.h"
#include "qg_static_for.h"

#ifndef QG_WT
#error "compile with -DQG_WT=<weight type index>"
#endif

namespace qg {

typedef uint32_t u4_t __attribute__((ext_vector_type(4)));
typedef float f16_t __attribute__((ext_vector_type(16)));

// acc += w . a with the accumulator pinned to accumulation registers
template <int ROUTE>
__device__ __forceinline__ void mfma32_acc(f16_t& acc, const u4_t& w, const u4_t& a) {
  if constexpr (ROUTE == ROUTE_F16)
    asm volatile("v_mfma_f32_32x32x16_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(w), "v"(a));
  else
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(w), "v"(a));
}

template <int ROUTE>
__device__ __forceinline__ uint32_t pack_out32(float lo, float hi) {
  f2_t f = {lo, hi};
  if constexpr (ROUTE == ROUTE_F16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, h2_t));
  else return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, b2_t));
}

constexpr int L32_BN = 256;
constexpr int L32_GROUP_M = 4;   // m-tiles per L2 panel
constexpr int L32_AHEAD = 4;        // k-steps between the global load of an A piece and its LDS store (2, 4 or 8;
                                    // measured: no difference between them)
constexpr int L32_READ_AHEAD = 2;   // row tiles between the LDS read of an A fragment and its use (2..6 measure alike)

// LDS: the A slab of one chunk = 8 k-step slices, each [BM rows][2 pieces of 16 B]
// plus 32 bytes of padding; piece h of row r sits at slot h ^ swz(r).  A fragment
// read takes piece h of 32 consecutive rows (32-byte row stride): the swizzle makes
// the 16-byte bank groups distinct within any aligned run of 8 rows modulo 128
// bytes and of 16 rows modulo 256 bytes, whichever way the hardware splits a
// 16-byte-per-lane read.  The padding staggers the slices so that the 16 pieces of
// one row (two per slice), written by 16 adjacent lanes, fall in 16 different
// bank groups.
__device__ __forceinline__ int swz32(int r) { return ((r >> 2) ^ (r >> 3)) & 1; }
template <int BM>
struct Lds32 {
  static constexpr int SLICE = BM * 32 + 32;   // bytes
  static constexpr int BUF = LayoutOf<1>::STEPS * SLICE;
};

template <int WT, int ROUTE, bool TWO_GROUPS, int BM>
__global__ __launch_bounds__(256) void large32_kernel(GemmParams p, int tiles_m, int tiles_n, int per_xcd, int tn0) {
  typedef Decoder<WT, ROUTE, 1> D;
  typedef LayoutOf<1> LY;
  constexpr int BITS = D::BITS, RAW = D::RAW;
  constexpr int NS = LY::STEPS;                // 8 k-steps of 16 per chunk
  constexpr int MTS = BM / 32;                 // 32-row MFMA tiles per workgroup
  constexpr int PT = BM / 16;                  // 16-byte A pieces per thread per chunk
  constexpr int PPS = PT / NS;                 // ... per k-step
  constexpr int PB = 8 / MTS;                  // pairs unpacked per row tile
  typedef Lds32<BM> L;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

  // ---- which tile ----------------------------------------------------------------
  const int total = tiles_m * tiles_n;
  const int logical = (int)(blockIdx.x % 8) * per_xcd + (int)(blockIdx.x / 8);
  if (logical >= total) return;
  const int panel = L32_GROUP_M * tiles_n;
  const int first_m = (logical / panel) * L32_GROUP_M;
  const int gsize = min(tiles_m - first_m, L32_GROUP_M);
  const int tm = first_m + (logical % panel) % gsize;
  const int tn = tn0 + (logical % panel) / gsize;       // tn0: first column tile of this launch

  const int tid = threadIdx.x, l = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int h = l >> 5, i32 = l & 31;
  const int KC = p.K / TILE_K, NCH = p.N / TILE_N;
  const int m0 = tm * BM;
  const int ncw = tn * (L32_BN / TILE_N) + w;            // my 64-column strip
  const bool active = ncw < NCH;
  const int nc = active ? ncw : NCH - 1;                 // idle wavefronts shadow a valid strip
  const int n0 = TILE_N * nc + 2 * i32;
  // no zero-points: read (valid) scale bytes instead and mask them away
  const uint8_t* zbase = p.Z ? p.Z : reinterpret_cast<const uint8_t*>(p.S);
  const uint32_t zmask = p.Z ? 0xffffffffu : 0u;

  // ---- A staging: piece i of thread t is the 16 bytes at row (t/16) + 16*i, byte
  // 16*(t%16) of the chunk's 256-byte row segment (16 adjacent lanes read one
  // segment).  It lands in slice (t%16)/2, piece (t%16)%2 of that row.
  // Loads go through a buffer resource over A: the per-lane part of the address is one
  // 32-bit register (row and position inside the chunk's row segment), everything
  // uniform (which 16-row block, which chunk) is scalar, and rows past M -- byte
  // offsets at or beyond M*K*2 -- read as zeros by the resource's range check
  // instead of needing a clamp.  (The host checks M*K*2 < 2^32.)
  const int srow = tid >> 4, spc = tid & 15;
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(p.A), 0, (int)((uint32_t)p.M * (uint32_t)(2 * p.K)), 0x00020000);
  const uint32_t a_off0 = (uint32_t)(m0 + srow) * (uint32_t)(2 * p.K) + 16u * spc;
  const uint32_t a_step = 16u * (uint32_t)(2 * p.K);                      // 16 rows further
  const int a_dst = (spc >> 1) * L::SLICE + srow * 32 + 16 * ((spc & 1) ^ swz32(srow));   // + 512*i for piece i
  auto a_load = [&](int i, int c) __attribute__((always_inline)) {
    // the row part stays in the vector offset so that the range check sees it; chunks
    // past K (the padding chunk of an odd chunk count, the ring's look-ahead at the
    // end) are pushed out of range as well and read as zeros
    const uint32_t past = (c < KC) ? 0u : 0x80000000u;
    return __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)(a_off0 + (uint32_t)i * a_step + past),
                                                 min(c, KC - 1) * (2 * TILE_K), 0);
  };
  u4_t stage[L32_AHEAD][PPS];

  // ---- W prefetch: raw chunk + its scales / zero-points -------------------------------
  struct WStage {
    uint32_t r[RAW];
    uint32_t s0, s1;
    uint32_t z0, z1;
  };
  // All of these go through buffer resources too: the lane's part of the address is
  // a constant 32-bit register, the chunk / group part a scalar.  (The host checks that
  // the packed weight and the scale array are below 4 GiB.)
  const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(p.W), 0, (int)(uint32_t)((int64_t)p.K * p.N / 8 * BITS), 0x00020000);
  const __amdgpu_buffer_rsrc_t s_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(p.S), 0, (int)(uint32_t)((int64_t)(p.K / p.group) * p.N * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t z_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(zbase), 0, (int)(uint32_t)((int64_t)(p.K / p.group) * p.N), 0x00020000);
  const int w_lane = 16 * l, s_lane = 2 * n0, z_lane = n0;
  const int w_strip = nc * KC * (1024 * BITS);          // byte offset of my strip (scalar)
  // The loads of one chunk are 2 (4 with two groups per chunk) + BITS separate
  // pieces, so that the main loop can issue them a few at a time in different gaps
  // between matrix instructions.  Pieces: s0, z0, (s1, z1,) then BITS x 16 bytes of codes.
  constexpr int WMETA = TWO_GROUPS ? 4 : 2;
  constexpr int WPIECES = WMETA + BITS;
  auto w_piece = [&](WStage& s, int c, auto Ic) __attribute__((always_inline)) {
    constexpr int I = decltype(Ic)::value;
    c = min(c, KC - 1);
    if constexpr (I >= WMETA) {
      constexpr int B = I - WMETA;
      const u4_t q = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, w_lane, w_strip + c * (1024 * BITS) + B * 1024, 0);
      s.r[4 * B + 0] = q.x; s.r[4 * B + 1] = q.y; s.r[4 * B + 2] = q.z; s.r[4 * B + 3] = q.w;
    } else {
      const int g0 = TWO_GROUPS ? 2 * c : ((c >> p.gshift) & p.gmask);
      if constexpr (I == 0) s.s0 = __builtin_amdgcn_raw_buffer_load_b32(s_rsrc, s_lane, g0 * p.N * 2, 0);
      if constexpr (I == 1) s.z0 = __builtin_amdgcn_raw_buffer_load_b16(z_rsrc, z_lane, g0 * p.N, 0);
      if constexpr (I == 2) s.s1 = __builtin_amdgcn_raw_buffer_load_b32(s_rsrc, s_lane, (g0 + 1) * p.N * 2, 0);
      if constexpr (I == 3) s.z1 = __builtin_amdgcn_raw_buffer_load_b16(z_rsrc, z_lane, (g0 + 1) * p.N, 0);
    }
  };
  auto w_issue = [&](WStage& s, int c) __attribute__((always_inline)) {
    static_for<WPIECES>([&](auto Ic) __attribute__((always_inline)) { w_piece(s, c, Ic); });
  };
  // constants of one column of the first (G = 0) or second (G = 1) group of a chunk
  auto consts_col = [&](typename D::Consts& g, const WStage& s, auto Gc, int nt) __attribute__((always_inline)) {
    if constexpr (decltype(Gc)::value == 0) D::make_col(g, nt, make_uint2(s.s0, 0u), s.z0 & zmask, p.zbias, p.scale_bf16);
    else                                    D::make_col(g, nt, make_uint2(s.s1, 0u), s.z1 & zmask, p.zbias, p.scale_bf16);
  };

  // Accumulators live in the accumulation registers (AGPRs) for the whole
  // kernel; the matrix instruction is issued through asm so that the register
  // allocator cannot shuttle them through vector registers.
  f16_t acc[MTS][2];
#pragma unroll
  for (int mt = 0; mt < MTS; ++mt)
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.f;

  typename D::Uniform u;
  u.init();

  // ---- prologue: chunk 0's A slab into buffer 0, ring primed for chunk 1 --------------
  WStage wA, wB;
  w_issue(wA, 0);
#pragma unroll
  for (int i = 0; i < PT; ++i) *reinterpret_cast<u4_t*>(lds + a_dst + 512 * i) = a_load(i, 0);
#pragma unroll
  for (int s = 0; s < L32_AHEAD; ++s)
#pragma unroll
    for (int q = 0; q < PPS; ++q) stage[s][q] = a_load(PPS * s + q, 1);

  // my A fragment of row tile mt, k-step slice j: piece h of row mt*32 + i32
  const int a_rd = i32 * 32 + 16 * (h ^ swz32(i32));

  // Weight fragments are unpacked one k-step ahead of their use, and the unpack
  // of step J+1 is spread over the MFMAs of step J (PB pairs per 32-row tile),
  // so the vector ALU works in the shadow of the matrix pipeline.  Fragments
  // ping-pong between two register sets by k-step parity, weight stages and
  // their constants by chunk parity (the chunk loop is unrolled by two).
  //
  // With one wavefront per SIMD every instruction of any kind takes an issue slot
  // of that one wavefront, and only about five fit behind a 32x32x16 MFMA before
  // the matrix pipeline starts to idle.  So everything that is not an MFMA is cut
  // into small items and dealt out over the 2*MTS gaps of every k-step:
  //   gap after the first MFMA of a tile:   extract this tile's pairs, read the A
  //                                         fragment RA tiles ahead, round the
  //                                         previous tile's pairs
  //   gap after the second MFMA of a tile:  centre / widen this tile's pairs, plus
  //                                         ONE extra item: an A staging piece
  //                                         (store + next load), or one load of the
  //                                         next chunk's weights, or the constants
  //                                         of one column of the next chunk
  // Constants of a chunk's first (or only) group ping-pong with the weight stages; those
  // of its second group (group size 64) live in one set that is rebuilt in place at the
  // start of the chunk, after its last use by the chunk before and before its first use.
  typename D::Consts gA0, gB0, g1;
  consts_col(gA0, wA, std::integral_constant<int, 0>{}, 0);
  consts_col(gA0, wA, std::integral_constant<int, 0>{}, 1);
  u4_t wf[2][2];
  static_for<2>([&](auto NTc) __attribute__((always_inline)) {
    constexpr int NT = decltype(NTc)::value;
    uint32_t o[4];
    D::template frag<0, NT>(wA.r, gA0, u, o);
    wf[0][NT] = (u4_t){o[0], o[1], o[2], o[3]};
  });
  __syncthreads();

  // Extra-item table.  Tiles whose second gap carries an A staging piece: MT = 1 + q*(MTS/PPS).
  // The other tiles of the chunk, in order, are numbered FS = 0, 1, ...:
  //   FS 0, 1 (two groups per chunk only): this chunk's second-group constants, one column each
  //   then WPS pieces of the next chunk's weights per tile until all are issued
  //   from k-step 5 on: the next chunk's first-group constants, one column per tile
  //   (its scale loads went out in k-step 0 and have long arrived).
  constexpr int STAGE_EVERY = MTS / PPS;
  constexpr int FREE_PER_STEP = MTS - PPS;
  constexpr int WPS = (BM == 128) ? 2 : 1;             // shorter k-steps: issue the loads twice as densely
  constexpr int W0 = TWO_GROUPS ? 2 : 0;
  constexpr int WSLOTS = (WPIECES + WPS - 1) / WPS;
  static_assert(W0 + WSLOTS <= 3 * FREE_PER_STEP, "weight loads must be issued by the end of k-step 2");

  // one chunk: weights wc (constants gc0, g1) are consumed, wn is loaded and its
  // constants gn0 built; CUR is the LDS buffer holding this chunk's A slab
  auto chunk = [&](auto CURc, WStage& wc, WStage& wn, typename D::Consts& gc0, typename D::Consts& gn0,
                   int kc) __attribute__((always_inline)) {
    constexpr int CUR = decltype(CURc)::value, NXT = CUR ^ 1;
    // A fragments: flat index f = J*MTS + MT over the chunk, read RA tiles ahead
    const uint8_t* abase = lds + CUR * L::BUF + a_rd;
    auto a_read = [&](int f) __attribute__((always_inline)) {
      return *reinterpret_cast<const u4_t*>(abase + (f / MTS) * L::SLICE + (f % MTS) * (32 * 32));
    };
    constexpr int RA = L32_READ_AHEAD;
    u4_t ar[RA + 1];
#pragma unroll
    for (int f = 0; f < RA; ++f) ar[f] = a_read(f);
    static_for<NS>([&](auto Jc) __attribute__((always_inline)) {
      constexpr int J = decltype(Jc)::value;
      constexpr int JN = (J + 1) % NS;
      uint32_t nf[2][4];                 // fragments of k-step J+1 under construction
      uint32_t xe[PB];
      typename D::Mid mid[PB], mid_prev[PB];
      const typename D::Consts& g = (J < NS - 1) ? ((TWO_GROUPS && JN >= NS / 2) ? g1 : gc0) : gn0;
      const uint32_t (&rw)[RAW] = (J < NS - 1) ? wc.r : wn.r;
      static_for<MTS>([&](auto MTc) __attribute__((always_inline)) {
        constexpr int MT = decltype(MTc)::value;
        constexpr int F = J * MTS + MT;
        mfma32_acc<ROUTE>(acc[MT][0], wf[J & 1][0], ar[F % (RA + 1)]);
        __builtin_amdgcn_sched_barrier(0);
        static_for<PB>([&](auto Qc) __attribute__((always_inline)) {          // extract
          constexpr int Q = decltype(Qc)::value, R = MT * PB + Q;
          xe[Q] = D::template pair_e<LY::t0(JN, R / 4) + R % 4>(rw, u);
        });
        if constexpr (F + RA < NS * MTS) ar[(F + RA) % (RA + 1)] = a_read(F + RA);   // A fragment RA tiles ahead
        if constexpr (MT > 0) {                                               // scale-and-round of the previous tile
          static_for<PB>([&](auto Qc) __attribute__((always_inline)) {
            constexpr int Q = decltype(Qc)::value, R = (MT - 1) * PB + Q;
            nf[R / 4][R % 4] = D::pair_p(mid_prev[Q], g, R / 4);
          });
        }
        __builtin_amdgcn_sched_barrier(0);
        mfma32_acc<ROUTE>(acc[MT][1], wf[J & 1][1], ar[F % (RA + 1)]);
        __builtin_amdgcn_sched_barrier(0);
        static_for<PB>([&](auto Qc) __attribute__((always_inline)) {          // centre / widen
          constexpr int Q = decltype(Qc)::value, R = MT * PB + Q;
          mid[Q] = D::template pair_s<LY::t0(JN, R / 4) + R % 4>(xe[Q], g, R / 4);
        });
        // ---- the one extra item of this tile --------------------------------------------
        constexpr bool STAGES = (MT >= 1) && ((MT - 1) % STAGE_EVERY == 0);
        if constexpr (STAGES) {
          // A slab of the next chunk: store the piece loaded L32_AHEAD steps ago, then
          // start the load that will be stored L32_AHEAD steps from now
          constexpr int Q = (MT - 1) / STAGE_EVERY;
          constexpr int SET = J % L32_AHEAD;
          *reinterpret_cast<u4_t*>(lds + NXT * L::BUF + a_dst + 512 * (PPS * J + Q)) = stage[SET][Q];
          constexpr int TS = J + L32_AHEAD;            // target step, counted from this chunk's first
          stage[SET][Q] = a_load(PPS * (TS % NS) + Q, kc + 1 + TS / NS);
        } else {
          constexpr int BEFORE = (MT == 0) ? 0 : (MT - 1 - (MT - 1) / STAGE_EVERY);   // free tiles before MT in this step
          constexpr int FS = J * FREE_PER_STEP + BEFORE;
          if constexpr (TWO_GROUPS && FS < 2) consts_col(g1, wc, std::integral_constant<int, 1>{}, FS);
          static_for<WPS>([&](auto Xc) __attribute__((always_inline)) {
            constexpr int I = (FS - W0) * WPS + decltype(Xc)::value;
            if constexpr (FS >= W0 && I < WPIECES) w_piece(wn, kc + 1, std::integral_constant<int, I>{});
          });
          constexpr int CS = FS - 5 * FREE_PER_STEP;   // first free tiles of k-step 5
          if constexpr (CS == 0 || CS == 1) consts_col(gn0, wn, std::integral_constant<int, 0>{}, CS);
        }
#pragma unroll
        for (int q = 0; q < PB; ++q) mid_prev[q] = mid[q];
        __builtin_amdgcn_sched_barrier(0);
      });
      static_for<PB>([&](auto Qc) __attribute__((always_inline)) {            // last tile's scale-and-round
        constexpr int Q = decltype(Qc)::value, R = (MTS - 1) * PB + Q;
        nf[R / 4][R % 4] = D::pair_p(mid_prev[Q], g, R / 4);
      });
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) wf[JN & 1][nt] = (u4_t){nf[nt][0], nf[nt][1], nf[nt][2], nf[nt][3]};
    });
    __syncthreads();
  };

  // Chunks go in pairs (buffers, weight stages and constants alternate); an odd chunk
  // count is padded with one chunk whose A slab reads as zeros, which keeps the loop
  // free of a conditional tail.
  for (int kc = 0; kc < KC; kc += 2) {
    chunk(std::integral_constant<int, 0>{}, wA, wB, gA0, gB0, kc);
    chunk(std::integral_constant<int, 1>{}, wB, wA, gB0, gA0, kc + 1);
  }

  // the matrix pipeline may still be writing the accumulators (the compiler
  // does not see the asm MFMAs, so it inserts no wait states of its own)
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");

  // ---- epilogue: element r of a tile is row (column of C) 8*(r/4) + 4*h + r%4 of the
  // instruction, i.e. C column 16*(r/4) + 8*h + 2*(r%4) + nt of the strip, in C row
  // mt*32 + i32: eight consecutive columns per r/4
  if (!active) return;
#pragma unroll
  for (int mt = 0; mt < MTS; ++mt) {
    const int m = m0 + mt * 32 + i32;
    if (m < p.M) {
      uint16_t* crow = p.C + (int64_t)m * p.N + TILE_N * nc + 8 * h;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        u4_t o;
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) o[r4] = pack_out32<ROUTE>(acc[mt][0][4 * q + r4], acc[mt][1][4 * q + r4]);
        *reinterpret_cast<u4_t*>(crow + 16 * q) = o;
      }
    }
  }
}

#define QG_CAT2(a, b) a##b
#define QG_CAT(a, b) QG_CAT2(a, b)

// One launch over the column tiles [tn0, tn0 + tiles_n) and all row tiles of height BM.
template <int ROUTE, bool TG, int BM>
static int launch_bm(const GemmParams& p, hipStream_t st, int tn0, int tiles_n) {
  const int tiles_m = (p.M + BM - 1) / BM;
  const int total = tiles_m * tiles_n;
  const int per_xcd = (total + 7) / 8;
  const size_t lds_bytes = 2 * Lds32<BM>::BUF;
  auto kern = large32_kernel<QG_WT, ROUTE, TG, BM>;
  // raise the dynamic LDS limit once per instantiation and device
  static bool attr_done[64] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return QG_EHIP;
  if (!attr_done[dev]) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds_bytes) != hipSuccess)
      return QG_EHIP;
    attr_done[dev] = true;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)(8 * per_xcd)), dim3(256), lds_bytes, st, p, tiles_m, tiles_n, per_xcd, tn0);
  return hipGetLastError() == hipSuccess ? QG_OK : QG_EHIP;
}

template <int ROUTE>
static int launch_rows(const GemmParams& p, int bm, hipStream_t st, int tn0, int tiles_n) {
  const bool tg = (p.group == 64);
  if (bm == 128) return tg ? launch_bm<ROUTE, true, 128>(p, st, tn0, tiles_n) : launch_bm<ROUTE, false, 128>(p, st, tn0, tiles_n);
  if (bm == 256) return tg ? launch_bm<ROUTE, true, 256>(p, st, tn0, tiles_n) : launch_bm<ROUTE, false, 256>(p, st, tn0, tiles_n);
  return QG_EINVAL;
}

template <int ROUTE>
static int launch_route(const GemmParams& p, int bm, hipStream_t st) {
  const int tiles_n = (p.N + L32_BN - 1) / L32_BN;
  if (bm != 0) return launch_rows<ROUTE>(p, bm, st, 0, tiles_n);
  // Row-tile height by a small cost model: workgroups run in rounds of 256 (one per
  // CU), a tile costs its rows plus about 64 rows' worth of unpack and start-up.
  // 128 rows win when they fill a round that 256 rows leave half empty (M <= 256 on
  // 28672 columns, M = 384 on 57344: measured 20-30 % shorter), 256 rows otherwise.
  auto cost = [&](int rows, long cols) {
    const long tiles = ((p.M + rows - 1) / rows) * cols;
    return ((tiles + 255) / 256) * (rows + 64);
  };
  if (p.M <= 128) return launch_rows<ROUTE>(p, 128, st, 0, tiles_n);
  // Whole rounds of 256-row tiles first; the column tiles that would start a partly
  // filled last round go into a second launch with whichever height is cheaper for
  // them (M = 1024 on 57344 columns: 3.5 rounds become 3 + one round of 128-row tiles).
  const int tm256 = (p.M + 255) / 256;
  const long rounds = ((long)tm256 * tiles_n) / 256;
  const int tn_full = (int)((rounds * 256) / tm256 < tiles_n ? (rounds * 256) / tm256 : tiles_n);
  if (tn_full == 0) return launch_rows<ROUTE>(p, cost(128, tiles_n) < cost(256, tiles_n) ? 128 : 256, st, 0, tiles_n);
  int rc = launch_rows<ROUTE>(p, 256, st, 0, tn_full);
  if (rc != QG_OK || tn_full == tiles_n) return rc;
  const int rest = tiles_n - tn_full;
  return launch_rows<ROUTE>(p, cost(128, rest) < cost(256, rest) ? 128 : 256, st, tn_full, rest);
}

int QG_CAT(large32_launch_wt, QG_WT)(const GemmParams& p, int route, int bm, hipStream_t st) {
  return route == ROUTE_F16 ? launch_route<ROUTE_F16>(p, bm, st) : launch_route<ROUTE_BF16>(p, bm, st);
}

}  // namespace qg
