// Prefill-sized matmul: LDS-staged A, register-resident W, 16x16x32 MFMA.
//
// A workgroup of 4 wavefronts computes a BM x 256 tile of C.  Wavefront w owns
// 64 columns: it loads its own 128x64 weight chunk straight from global memory
// into registers (BITS 16-byte loads per lane, one chunk ahead of use), unpacks
// it in registers and uses it as the row operand of the matrix instruction --
// the weights never pass through LDS and are never exchanged between lanes,
// which is the paper's weight pipeline (Section "Key Ideas", steps 1-4) with the
// shared-memory hop removed because every wavefront needs different columns.
// The BM x 128 slab of A for the same K range is shared by the four wavefronts
// through LDS (double-buffered per chunk, XOR-swizzled 16-byte pieces, filled
// through a small register ring two k-steps ahead), so each unpacked weight is
// used BM times and each weight is unpacked M/BM times in total.
// Workgroup ids are remapped so that the workgroups resident on one XCD (ids
// congruent mod 8) form 4 x 8 panels of tiles that share A and W in that XCD's L2.
// Compiled once per weight type (QG_WT).
// QG_DBG_NOBARRIER / NOAFRAG / NOSTAGE / NOWLOAD (never defined by the build) each cut one stage out for
// timing experiments -- results are wrong with them.
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

// acc += w . a with the accumulator pinned to accumulation registers
template <int ROUTE>
__device__ __forceinline__ void mfma16_acc(f4_t& acc, const u4_t& w, const u4_t& a) {
  if constexpr (ROUTE == ROUTE_F16)
    asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(w), "v"(a));
  else
    asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(w), "v"(a));
}

template <int ROUTE>
__device__ __forceinline__ uint32_t pack_out(float lo, float hi) {
  f2_t f = {lo, hi};
  if constexpr (ROUTE == ROUTE_F16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, h2_t));
  else return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, b2_t));
}

constexpr int LARGE_BN = 256;
constexpr int LARGE_GROUP_M = 4;   // m-tiles per L2 panel

// LDS: A slab of one chunk = 4 k-step slices, each [BM rows][4 pieces of 16 B];
// piece p of row r is stored at slot p ^ lds_swizzle(r).  A fragment read takes
// one piece column of 16 consecutive rows (64-byte row stride = 4 four-bank
// groups): the swizzle makes the groups distinct both within every aligned run of
// 8 rows modulo 8 groups (32 banks) and within the 16 rows modulo 16 groups (64
// banks), whichever way the hardware splits a 16-byte-per-lane read.
__device__ __forceinline__ int lds_swizzle(int r) { return (((r >> 2) & 1) << 1) | (((r >> 1) ^ (r >> 3)) & 1); }
template <int BM>
struct LargeLds {
  static constexpr int SLICE = BM * 64;        // bytes
  static constexpr int BUF = 4 * SLICE;
};

template <int WT, int ROUTE, int GPC, int BM, bool MX = false>
__global__ __launch_bounds__(256) void large_kernel(GemmParams p, int tiles_m, int tiles_n, int per_xcd, int tn0) {
  // GPC = groups per 128-row chunk: 1 (group size 128 or more), 2 (64) or 4 (32)
  // MX: power-of-two block scales (8-bit exponents, one per 32 rows: GPC = 4) on e2m1 / e4m3 codes
  constexpr bool TWO_GROUPS = (GPC == 2), FOUR_GROUPS = (GPC == 4);
  static_assert(!MX || GPC == 4, "block scales: one per 32 rows");
  typedef typename DecoderFor<WT, ROUTE, MX>::type D;  // WT_DENSE16: weights already de-quantised, pass-through
  constexpr int BITS = D::BITS, RAW = D::RAW;
  constexpr int MTS = BM / 16;                 // 16-row MFMA tiles per workgroup
  constexpr int PIECES = BM * 4 / 256;         // 16-byte pieces per thread per slice
  typedef LargeLds<BM> L;
  extern __shared__ __attribute__((aligned(16))) uint8_t lds[];

  // ---- which tile ----------------------------------------------------------------
  // With split-K every tile is computed by p.splitk workgroups, one per slab of
  // chunks_per_split K-chunks; the slab is the slowest index, so the workgroups of a slab
  // keep the panel order among themselves.
  const int tiles = tiles_m * tiles_n;
  const int logical = (int)(blockIdx.x % 8) * per_xcd + (int)(blockIdx.x / 8);
  if (logical >= tiles * p.splitk) return;
  const int slab = logical / tiles, tile = logical % tiles;
  const int panel = LARGE_GROUP_M * tiles_n;
  const int first_m = (tile / panel) * LARGE_GROUP_M;
  const int gsize = min(tiles_m - first_m, LARGE_GROUP_M);
  const int tm = first_m + (tile % panel) % gsize;
  const int tn = tn0 + (tile % panel) / gsize;          // tn0: first column tile of this launch

  const int tid = threadIdx.x, l = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, kept in a scalar register
  const int b = l >> 4, i16 = l & 15;
  const int KC = p.K / TILE_K, NCH = p.N / TILE_N;
  const int kbeg = slab * p.chunks_per_split, kend = min(KC, kbeg + p.chunks_per_split);   // my K-chunks
  const int m0 = tm * BM;
  const int ncw = tn * (LARGE_BN / TILE_N) + w;          // my 64-column strip
  const bool active = ncw < NCH;
  const int nc = active ? ncw : NCH - 1;                 // idle wavefronts shadow a valid strip
  const int n0 = TILE_N * nc + 4 * i16;
  // no zero-points: read (valid) scale bytes instead and mask them away
  const uint8_t* zbase = p.Z ? p.Z : reinterpret_cast<const uint8_t*>(p.S);
  const uint32_t zmask = p.Z ? 0xffffffffu : 0u;

  // ---- A staging: thread t moves pieces q = t + 256*i, row = q/4, piece = q%4 ---------
  // Loads go through a buffer resource over A: the lane's part of the address is one
  // 32-bit register, which 64-row block and which k-step is scalar, and rows past M --
  // byte offsets at or beyond M*K*2 -- read as zeros by the resource's range check
  // instead of needing a clamp.  (The host checks M*K*2 < 2^32.)
  const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(p.A), 0, (int)((uint32_t)p.M * (uint32_t)(2 * p.K)), 0x00020000);
  const int srow = tid >> 2, spc = tid & 3;
  const uint32_t a_off0 = (uint32_t)(m0 + srow) * (uint32_t)(2 * p.K) + 16u * spc;
  const uint32_t a_step = 64u * (uint32_t)(2 * p.K);                      // 64 rows further
  const int a_dst0 = srow * 64 + 16 * (spc ^ lds_swizzle(srow));          // + 4096*i for piece i
  auto a_load = [&](int i, int kstep) __attribute__((always_inline)) {     // kstep = 4*chunk + slice
    // the row part stays in the vector offset so that the range check sees it; k-steps
    // past my last chunk (the padding chunk of an odd chunk count, the ring's look-ahead
    // at the end) are pushed out of range as well and read as zeros
    const uint32_t past = (kstep < 4 * kend) ? 0u : 0x80000000u;
    return __builtin_amdgcn_raw_buffer_load_b128(a_rsrc, (int)(a_off0 + (uint32_t)i * a_step + past),
                                                 min(kstep, 4 * KC - 1) * 64, 0);
  };
  // Staging registers: SETS sets of PIECES pieces; a piece is loaded SETS k-steps before it is
  // stored to LDS (2: half a chunk ahead; 4: a whole chunk ahead -- measured on the prefill
  // shapes: no difference, the loads are not late; 2 is the build's value).
#ifndef QG_STAGE_SETS
#define QG_STAGE_SETS 2
#endif
  constexpr int SETS = QG_STAGE_SETS;
  static_assert(SETS == 2 || SETS == 4, "staging distance");
  u4_t stage[SETS][PIECES];
  auto a_issue = [&](int set, int kstep) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < PIECES; ++i) stage[set][i] = a_load(i, kstep);
  };
  auto a_commit = [&](int set, int buf, int slice) __attribute__((always_inline)) {
#pragma unroll
    for (int i = 0; i < PIECES; ++i)
      *reinterpret_cast<u4_t*>(lds + buf * L::BUF + slice * L::SLICE + a_dst0 + 4096 * i) = stage[set][i];
  };

  // ---- W prefetch: raw chunk + its scales / zero-points -------------------------------
  struct WStage {
    uint32_t r[RAW];
    uint2 s0, s1, s2, s3;        // scales / zero-points of the chunk's groups (GPC of them in use)
    uint32_t z0, z1, z2, z3;
  };
  // Through buffer resources as well (the host checks that the packed weight and the
  // scale array are below 4 GiB): lane part constant, chunk / group part scalar.
  const __amdgpu_buffer_rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(p.W), 0, (int)(uint32_t)((int64_t)p.K * p.N / 8 * BITS), 0x00020000);
  const __amdgpu_buffer_rsrc_t s_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(p.S), 0, (int)(uint32_t)((int64_t)(p.K / p.group) * p.N * (D::IS_MX ? 1 : 2)), 0x00020000);
  const __amdgpu_buffer_rsrc_t z_rsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint8_t*>(zbase), 0, (int)(uint32_t)((int64_t)(p.K / p.group) * p.N), 0x00020000);
  const int w_lane = 16 * l, s_lane = 2 * n0, z_lane = n0;
  const int w_strip = nc * KC * (1024 * BITS);          // byte offset of my strip (scalar)
  // The loads of one chunk are 2 (4 with two groups per chunk) + BITS separate pieces,
  // so that the main loop can issue them a few at a time in different gaps between
  // matrix instructions.  Pieces: s0, z0, (s1, z1, (s2, z2, s3, z3,)) then BITS x 16 bytes of codes.
  constexpr int WMETA = !D::HAS_META ? 0 : (D::IS_MX ? GPC : 2 * GPC);      // block scales: one 4-byte load per group
  constexpr int WPIECES = WMETA + BITS;
  auto w_piece = [&](WStage& s, int c, auto Ic) __attribute__((always_inline)) {
    constexpr int I = decltype(Ic)::value;
    c = min(c, KC - 1);
    if constexpr (I >= WMETA) {
      constexpr int B = I - WMETA;
      const u4_t q = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, w_lane, w_strip + c * (1024 * BITS) + B * 1024, 0);
      s.r[4 * B + 0] = q.x; s.r[4 * B + 1] = q.y; s.r[4 * B + 2] = q.z; s.r[4 * B + 3] = q.w;
    } else {
      const int g0 = (GPC > 1) ? GPC * c : ((c >> p.gshift) & p.gmask);
      typedef uint32_t u2_t __attribute__((ext_vector_type(2)));
      if constexpr (D::IS_MX) {        // the lane's four scale bytes of group I, kept in the zero-point slot
        const uint32_t v = __builtin_amdgcn_raw_buffer_load_b32(s_rsrc, z_lane, (g0 + I) * p.N, 0);
        if constexpr (I == 0) s.z0 = v;
        if constexpr (I == 1) s.z1 = v;
        if constexpr (I == 2) s.z2 = v;
        if constexpr (I == 3) s.z3 = v;
      } else {
        if constexpr (I == 0) { const u2_t v = __builtin_amdgcn_raw_buffer_load_b64(s_rsrc, s_lane, g0 * p.N * 2, 0); s.s0 = make_uint2(v.x, v.y); }
        if constexpr (I == 1) s.z0 = __builtin_amdgcn_raw_buffer_load_b32(z_rsrc, z_lane, g0 * p.N, 0);
        if constexpr (I == 2) { const u2_t v = __builtin_amdgcn_raw_buffer_load_b64(s_rsrc, s_lane, (g0 + 1) * p.N * 2, 0); s.s1 = make_uint2(v.x, v.y); }
        if constexpr (I == 3) s.z1 = __builtin_amdgcn_raw_buffer_load_b32(z_rsrc, z_lane, (g0 + 1) * p.N, 0);
        if constexpr (I == 4) { const u2_t v = __builtin_amdgcn_raw_buffer_load_b64(s_rsrc, s_lane, (g0 + 2) * p.N * 2, 0); s.s2 = make_uint2(v.x, v.y); }
        if constexpr (I == 5) s.z2 = __builtin_amdgcn_raw_buffer_load_b32(z_rsrc, z_lane, (g0 + 2) * p.N, 0);
        if constexpr (I == 6) { const u2_t v = __builtin_amdgcn_raw_buffer_load_b64(s_rsrc, s_lane, (g0 + 3) * p.N * 2, 0); s.s3 = make_uint2(v.x, v.y); }
        if constexpr (I == 7) s.z3 = __builtin_amdgcn_raw_buffer_load_b32(z_rsrc, z_lane, (g0 + 3) * p.N, 0);
      }
    }
  };
  auto w_issue = [&](WStage& s, int c) __attribute__((always_inline)) {
    static_for<WPIECES>([&](auto Ic) __attribute__((always_inline)) { w_piece(s, c, Ic); });
  };
  // constants of one column of group G (0 .. GPC-1) of a chunk
  auto consts_col = [&](typename D::Consts& g, const WStage& s, auto Gc, int nt) __attribute__((always_inline)) {
    constexpr int G = decltype(Gc)::value;
    if constexpr (!D::HAS_META) return;
    const uint32_t zm = D::IS_MX ? 0xffffffffu : zmask;          // block scales travel in the zero-point slot: never masked
    if constexpr (G == 0) D::make_col(g, nt, s.s0, s.z0 & zm, p.zbias, p.scale_bf16);
    if constexpr (G == 1) D::make_col(g, nt, s.s1, s.z1 & zm, p.zbias, p.scale_bf16);
    if constexpr (G == 2) D::make_col(g, nt, s.s2, s.z2 & zm, p.zbias, p.scale_bf16);
    if constexpr (G == 3) D::make_col(g, nt, s.s3, s.z3 & zm, p.zbias, p.scale_bf16);
  };

  // Accumulators live in the accumulation registers (AGPRs) for the whole
  // kernel; the matrix instruction is issued through asm so that the register
  // allocator cannot shuttle them through vector registers.
  f4_t acc[MTS][4];
#pragma unroll
  for (int mt = 0; mt < MTS; ++mt)
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = (f4_t){0.f, 0.f, 0.f, 0.f};

  typename D::Uniform u;
  u.init();

  // ---- prologue: chunk 0's A slab into buffer 0, ring primed for chunk 1 --------------
  uint32_t my_level = 0;
  if constexpr (D::IS_LUT) my_level = D::fetch(p.T, tid);       // codebook indices: this thread's level of the table
  WStage wA, wB;
  w_issue(wA, kbeg);
  const int ks0 = 4 * kbeg;
  if constexpr (SETS == 2) {
    a_issue(0, ks0); a_issue(1, ks0 + 1);
    a_commit(0, 0, 0); a_issue(0, ks0 + 2);
    a_commit(1, 0, 1); a_issue(1, ks0 + 3);
    a_commit(0, 0, 2); a_issue(0, ks0 + 4);     // slice 0 of the second chunk
    a_commit(1, 0, 3); a_issue(1, ks0 + 5);     // slice 1 of the second chunk
  } else {
    a_issue(0, ks0); a_issue(1, ks0 + 1); a_issue(2, ks0 + 2); a_issue(3, ks0 + 3);
    a_commit(0, 0, 0); a_issue(0, ks0 + 4);     // the four slices of the second chunk
    a_commit(1, 0, 1); a_issue(1, ks0 + 5);
    a_commit(2, 0, 2); a_issue(2, ks0 + 6);
    a_commit(3, 0, 3); a_issue(3, ks0 + 7);
  }

  // my A fragment of row-tile mt, k-step slice j: piece b of row mt*16 + i16
  const int a_rd = i16 * 64 + 16 * (b ^ lds_swizzle(i16));

  // Codebook indices: the replicated lookup table sits behind the two A buffers; the 512 bytes
  // the build stages the levels in are borrowed from the second buffer, which nothing has
  // written yet.  (Two workgroup barriers inside; the first loads are already in flight.)
  if constexpr (D::IS_LUT) {
    uint32_t* table = reinterpret_cast<uint32_t*>(lds + 2 * L::BUF);
    D::build(table, reinterpret_cast<uint16_t*>(lds + L::BUF), my_level, tid, 256);
    u.set_table(table, l);
  }

  // Weight fragments are unpacked one k-step ahead of their use, and the unpack
  // of step J+1 is spread over the MFMAs of step J (one pair per 16-row tile),
  // so the vector ALU works in the shadow of the matrix pipeline.  Fragments
  // ping-pong between two register sets by k-step parity, weight stages and
  // their first-group constants by chunk parity (the chunk loop is unrolled by two);
  // the second-group constants (group size 64) live in one set rebuilt in place at
  // the start of each chunk.
  //
  // With one wavefront per SIMD every instruction of any kind takes an issue slot
  // of that one wavefront, and only about two fit behind a 16x16x32 MFMA before the
  // matrix pipeline starts to idle.  So everything that is not an MFMA is cut into
  // small items and dealt out over the four gaps of every row tile:
  //   gap 0: extract this tile's pair          gap 1: read the A fragment two tiles
  //   gap 2: centre / widen this tile's pair          ahead, round the previous pair
  //   gap 3: ONE extra item -- an A staging piece (store + next load), or a load of
  //          the next chunk's weights, or the constants of one column
  typename D::Consts gA0, gB0, g1;
  static_for<4>([&](auto NTc) __attribute__((always_inline)) {
    consts_col(gA0, wA, std::integral_constant<int, 0>{}, decltype(NTc)::value);
  });
  u4_t wf[2][4];
  static_for<4>([&](auto NTc) __attribute__((always_inline)) {
    constexpr int NT = decltype(NTc)::value;
    uint32_t o[4];
    D::template frag<0, NT>(wA.r, gA0, u, o);
    wf[0][NT] = (u4_t){o[0], o[1], o[2], o[3]};
  });
  __syncthreads();

  // Extra-item table, gap 3 of row tile MT in k-step J:
  //   MT % 4 == 0   store the A staging piece MT/4 loaded SETS k-steps ago
  //   MT % 4 == 2   start the load of that piece for SETS k-steps from now
  //   odd MT        (index MT/2 within the step) k-steps 0 and 1: WPS loads of the next
  //                 chunk's weights; last CSLOTS of k-step 2: the next chunk's first-group
  //                 constants, CPS columns each; first CSLOTS of k-step 3 (two groups per
  //                 chunk): the next chunk's second-group constants, rebuilt in place --
  //                 their last use was the unpack during k-step 2
  constexpr int FREE_PER_STEP = MTS / 2;
  constexpr int WPS = (WPIECES + 2 * FREE_PER_STEP - 1) / (2 * FREE_PER_STEP);   // weight loads per odd tile
  constexpr int WSLOTS = (WPIECES + WPS - 1) / WPS;
  constexpr int CPS = (4 + FREE_PER_STEP - 1) / FREE_PER_STEP;                  // constant columns per odd tile
  constexpr int CSLOTS = 4 / CPS;
  static_assert(MTS / 4 == PIECES, "one staging piece per four row tiles");
  static_assert(WSLOTS <= 2 * FREE_PER_STEP, "weight loads must be issued by the end of k-step 1");
  if constexpr (TWO_GROUPS) {
    static_for<4>([&](auto NTc) __attribute__((always_inline)) {
      consts_col(g1, wA, std::integral_constant<int, 1>{}, decltype(NTc)::value);
    });
  }
  // Four groups per chunk: every k-step has its own group.  Two constant sets alternate by
  // the parity of the k-step -- gA0 for steps 0 and 2, gB0 for steps 1 and 3, whatever the
  // chunk -- and while the unpack of step J+1 reads one, the other is rebuilt for step J+2
  // (groups 2 and 3 from this chunk's stage in k-steps 0 and 1, groups 0 and 1 of the next
  // chunk from its stage in k-steps 2 and 3).
  if constexpr (FOUR_GROUPS) {
    static_for<4>([&](auto NTc) __attribute__((always_inline)) {
      consts_col(gB0, wA, std::integral_constant<int, 1>{}, decltype(NTc)::value);
    });
  }

  // one chunk: weights wc (constants gc0, g1) are consumed, wn is loaded and its
  // constants gn0 built; CUR is the LDS buffer holding this chunk's A slab
  auto chunk = [&](auto CURc, WStage& wc, WStage& wn, typename D::Consts& gc0, typename D::Consts& gn0,
                   int kc) __attribute__((always_inline)) {
    constexpr int CUR = decltype(CURc)::value, NXT = CUR ^ 1;
    constexpr int PB = 16 / MTS;                       // pairs unpacked per row tile
    // A fragments: flat index f = J*MTS + MT over the chunk, read two tiles ahead
    const uint8_t* abase = lds + CUR * L::BUF + a_rd;
    auto a_read = [&](int f) __attribute__((always_inline)) {
#ifdef QG_DBG_NOAFRAG
      return (u4_t){0x3c003c00u + (uint32_t)f, 0x3c003c00u, 0x3c003c00u, (uint32_t)(uintptr_t)abase};
#else
      return *reinterpret_cast<const u4_t*>(abase + (f / MTS) * L::SLICE + (f % MTS) * (16 * 64));
#endif
    };
    u4_t ar[3];
    ar[0] = a_read(0);
    ar[1] = a_read(1);
    static_for<4>([&](auto Jc) __attribute__((always_inline)) {
      constexpr int J = decltype(Jc)::value;
      constexpr int JN = (J + 1) & 3;
      uint32_t nf[4][4];                 // fragment of k-step J+1 under construction
      typename D::Ext xe[PB];
      typename D::Mid mid[PB], mid_prev[PB];
      const typename D::Consts& g = FOUR_GROUPS ? ((JN & 1) ? gn0 : gc0)
                                                : (J < 3) ? ((TWO_GROUPS && JN >= 2) ? g1 : gc0) : gn0;
      const uint32_t (&rw)[RAW] = (J < 3) ? wc.r : wn.r;
      static_for<MTS>([&](auto MTc) __attribute__((always_inline)) {
        constexpr int MT = decltype(MTc)::value;
        constexpr int F = J * MTS + MT;
        mfma16_acc<ROUTE>(acc[MT][0], wf[J & 1][0], ar[F % 3]);
        __builtin_amdgcn_sched_barrier(0);
        static_for<PB>([&](auto Qc) __attribute__((always_inline)) {          // extract
          constexpr int Q = decltype(Qc)::value, R = MT * PB + Q;
          xe[Q] = D::template pair_e<(JN * 4 + R / 4) * 4 + R % 4>(rw, u);
        });
        __builtin_amdgcn_sched_barrier(0);
        mfma16_acc<ROUTE>(acc[MT][1], wf[J & 1][1], ar[F % 3]);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (F + 2 < 4 * MTS) ar[(F + 2) % 3] = a_read(F + 2);       // A fragment two tiles ahead
        if constexpr (MT > 0) {                                               // scale-and-round of the previous tile
          static_for<PB>([&](auto Qc) __attribute__((always_inline)) {
            constexpr int Q = decltype(Qc)::value, R = (MT - 1) * PB + Q;
            nf[R / 4][R % 4] = D::pair_p(mid_prev[Q], g, R / 4);
          });
        }
        __builtin_amdgcn_sched_barrier(0);
        mfma16_acc<ROUTE>(acc[MT][2], wf[J & 1][2], ar[F % 3]);
        __builtin_amdgcn_sched_barrier(0);
        static_for<PB>([&](auto Qc) __attribute__((always_inline)) {          // centre / widen
          constexpr int Q = decltype(Qc)::value, R = MT * PB + Q;
          mid[Q] = D::template pair_s<(JN * 4 + R / 4) * 4 + R % 4>(xe[Q], g, R / 4);
        });
        __builtin_amdgcn_sched_barrier(0);
        mfma16_acc<ROUTE>(acc[MT][3], wf[J & 1][3], ar[F % 3]);
        __builtin_amdgcn_sched_barrier(0);
        // ---- the one extra item of this tile --------------------------------------------
        if constexpr (MT % 4 == 0) {
#ifndef QG_DBG_NOSTAGE
          constexpr int I = MT / 4;
          *reinterpret_cast<u4_t*>(lds + NXT * L::BUF + J * L::SLICE + a_dst0 + 4096 * I) = stage[J % SETS][I];
#endif
        } else if constexpr (MT % 4 == 2) {
#ifndef QG_DBG_NOSTAGE
          constexpr int I = MT / 4;
          stage[J % SETS][I] = a_load(I, 4 * (kc + 1) + J + SETS);     // SETS k-steps from now
#endif
        } else {
          constexpr int IDX = MT / 2;                  // 0 .. FREE_PER_STEP-1
          constexpr int FS = J * FREE_PER_STEP + IDX;
#ifndef QG_DBG_NOWLOAD
          static_for<WPS>([&](auto Xc) __attribute__((always_inline)) {
            constexpr int I = FS * WPS + decltype(Xc)::value;
            if constexpr (I < WPIECES) w_piece(wn, kc + 1, std::integral_constant<int, I>{});
          });
#endif
          static_for<CPS>([&](auto Xc) __attribute__((always_inline)) {
            constexpr int X = decltype(Xc)::value;
            if constexpr (!FOUR_GROUPS && J == 2 && IDX >= FREE_PER_STEP - CSLOTS)
              consts_col(gn0, wn, std::integral_constant<int, 0>{}, (IDX - (FREE_PER_STEP - CSLOTS)) * CPS + X);
            if constexpr (TWO_GROUPS && J == 3 && IDX < CSLOTS)
              consts_col(g1, wn, std::integral_constant<int, 1>{}, IDX * CPS + X);
            if constexpr (FOUR_GROUPS && IDX >= FREE_PER_STEP - CSLOTS) {
              constexpr int COL = (IDX - (FREE_PER_STEP - CSLOTS)) * CPS + X;
              if constexpr (J == 0) consts_col(gc0, wc, std::integral_constant<int, 2>{}, COL);
              if constexpr (J == 1) consts_col(gn0, wc, std::integral_constant<int, 3>{}, COL);
              if constexpr (J == 2) consts_col(gc0, wn, std::integral_constant<int, 0>{}, COL);
              if constexpr (J == 3) consts_col(gn0, wn, std::integral_constant<int, 1>{}, COL);
            }
          });
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
      for (int nt = 0; nt < 4; ++nt) wf[JN & 1][nt] = (u4_t){nf[nt][0], nf[nt][1], nf[nt][2], nf[nt][3]};
    });
#ifndef QG_DBG_NOBARRIER
    __syncthreads();
#endif
  };

  // Chunks go in pairs (buffers, weight stages and constants alternate); an odd chunk
  // count is padded with one chunk whose A slab reads as zeros, which keeps the loop
  // free of a conditional tail (with one, the compiler merged tail and loop body and
  // shuffled the whole accumulator state around the merge).
  for (int kc = kbeg; kc < kend; kc += 2) {
    chunk(std::integral_constant<int, 0>{}, wA, wB, gA0, gB0, kc);
    if constexpr (FOUR_GROUPS) chunk(std::integral_constant<int, 1>{}, wB, wA, gA0, gB0, kc + 1);   // sets by k-step parity
    else                       chunk(std::integral_constant<int, 1>{}, wB, wA, gB0, gA0, kc + 1);   // sets by chunk parity
  }

  // the matrix pipeline may still be writing the accumulators (the compiler
  // does not see the asm MFMAs, so it inserts no wait states of its own)
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");

  // ---- split-K: partial tiles meet in the workspace ------------------------------------
  // Partial sums cross workgroups (and XCDs, whose L2s are not coherent with each other)
  // through 16-byte buffer stores and loads that carry the sc1 cache-policy bit, which is
  // what a device-scope relaxed atomic store / load compiles to on this target: the store
  // writes through, the load bypasses the local caches.  Every wavefront handles its own
  // 64-column strip of the tile by itself (no workgroup barrier after the main loop): its
  // stores complete, lane 0 draws a ticket of that strip, and the wavefront that draws the
  // last of the splitk tickets sums all slabs in slab order -- the result does not depend
  // on arrival order.  The read-back is the expensive part (measured: one CU sustains only
  // about 60 GB/s of such loads, and the four strips of a tile are in practice finished by
  // the same, slowest workgroup), which is what the host's cost model charges per MB.
  // Only the lower tiles use this (the host never splits 256-row tiles).
  if constexpr (BM <= 128) {
    if (p.splitk > 1) {
      if (!active) return;
      constexpr int SC1 = 16;                                   // cache policy: device coherence
      constexpr int TILE_BYTES = BM * LARGE_BN * 4;
      auto ws_rsrc = [&](int sp) __attribute__((always_inline)) {
        return __builtin_amdgcn_make_buffer_rsrc(p.ws + ((int64_t)tile * p.splitk + sp) * (BM * LARGE_BN), 0, TILE_BYTES, 0x00020000);
      };
      // lane layout of a partial tile: fragment (mt, nt) of thread tid at 16 * ((mt*4+nt)*256 + tid)
      // (QG_DBG_NOEXSTORE / QG_DBG_NOEXLOAD: diagnostic builds without the exchange / without the
      // read-back, wrong results, timing only; never defined by the build)
#ifndef QG_DBG_NOEXSTORE
      {
        const __amdgpu_buffer_rsrc_t mine = ws_rsrc(slab);
#pragma unroll
        for (int mt = 0; mt < MTS; ++mt)
          if (m0 + mt * 16 + i16 < p.M) {
#pragma unroll
            for (int nt = 0; nt < 4; ++nt)
              __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4_t, acc[mt][nt]), mine, 16 * tid, (mt * 4 + nt) * 4096, SC1);
          }
      }
#endif
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");           // my partial strip is out before my ticket is drawn
      unsigned* ticket = p.tickets + 4 * tile + w;
      unsigned drawn = 0;
      if (l == 0) drawn = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      drawn = __builtin_amdgcn_readfirstlane(drawn);
      if (drawn != (unsigned)(p.splitk - 1)) return;
#pragma unroll
      for (int mt = 0; mt < MTS; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt) acc[mt][nt] = (f4_t){0.f, 0.f, 0.f, 0.f};
#if !defined(QG_DBG_NOEXLOAD) && !defined(QG_DBG_NOEXSTORE)
      // two slabs' loads are in flight together (the second of an odd count is a repeat
      // of the last slab whose values are dropped)
      for (int sp = 0; sp < p.splitk; sp += 2) {
        const bool two = sp + 1 < p.splitk;
        const __amdgpu_buffer_rsrc_t r0 = ws_rsrc(sp), r1 = ws_rsrc(two ? sp + 1 : sp);
        u4_t v0[MTS][4], v1[MTS][4];
#pragma unroll
        for (int mt = 0; mt < MTS; ++mt)
#pragma unroll
          for (int nt = 0; nt < 4; ++nt) {
            v0[mt][nt] = v1[mt][nt] = (u4_t){0u, 0u, 0u, 0u};
            if (m0 + mt * 16 + i16 < p.M) {                       // rows past M were not written
              v0[mt][nt] = __builtin_amdgcn_raw_buffer_load_b128(r0, 16 * tid, (mt * 4 + nt) * 4096, SC1);
              v1[mt][nt] = __builtin_amdgcn_raw_buffer_load_b128(r1, 16 * tid, (mt * 4 + nt) * 4096, SC1);
            }
          }
#pragma unroll
        for (int mt = 0; mt < MTS; ++mt)
#pragma unroll
          for (int nt = 0; nt < 4; ++nt) {
            acc[mt][nt] += __builtin_bit_cast(f4_t, v0[mt][nt]);
            if (two) acc[mt][nt] += __builtin_bit_cast(f4_t, v1[mt][nt]);
          }
      }
#endif
      if (l == 0) __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // ready for the next call
    }
  }

  // ---- epilogue: a lane holds 16 consecutive columns of row mt*16 + i16 ---------------
  if (!active) return;
  const int ncol = TILE_N * nc + 16 * b;
#pragma unroll
  for (int mt = 0; mt < MTS; ++mt) {
    const int m = m0 + mt * 16 + i16;
    if (m < p.M) {
      uint32_t o[8];
#pragma unroll
      for (int r = 0; r < 4; ++r) {          // column offset 4r + nt
        o[2 * r + 0] = pack_out<ROUTE>(acc[mt][0][r], acc[mt][1][r]);
        o[2 * r + 1] = pack_out<ROUTE>(acc[mt][2][r], acc[mt][3][r]);
      }
      u4_t* dst = reinterpret_cast<u4_t*>(p.C + (int64_t)m * p.N + ncol);
      dst[0] = (u4_t){o[0], o[1], o[2], o[3]};
      dst[1] = (u4_t){o[4], o[5], o[6], o[7]};
    }
  }
}

#define QG_CAT2(a, b) a##b
#define QG_CAT(a, b) QG_CAT2(a, b)

// One launch over the column tiles [tn0, tn0 + tiles_n) and all row tiles of height BM.
template <int ROUTE, int GPC, int BM, bool MX = false>
static int launch_bm(const GemmParams& p, hipStream_t st, int tn0, int tiles_n) {
  const int tiles_m = (p.M + BM - 1) / BM;
  if (p.splitk > 1 && BM > 128) return QG_EINVAL;
  const int total = tiles_m * tiles_n * p.splitk;
  const int per_xcd = (total + 7) / 8;
  typedef typename DecoderFor<QG_WT, ROUTE, MX>::type D;
  size_t lds_bytes = 2 * LargeLds<BM>::BUF;
  if constexpr (D::IS_LUT) lds_bytes += (size_t)D::TABLE_DWORDS * 4;      // 256-row tiles + a 32 KiB table: exactly the 160 KiB of a CU
  auto kern = large_kernel<QG_WT, ROUTE, GPC, BM, MX>;
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
  const int gpc = (p.group == 32) ? 4 : (p.group == 64) ? 2 : 1;       // groups per 128-row chunk
  if (p.scale_e8m0) {
#if QG_WT == 9 || QG_WT == 13
    if (gpc != 4) return QG_EUNSUPPORTED;
    if (bm == 64) return launch_bm<ROUTE, 4, 64, true>(p, st, tn0, tiles_n);
    if (bm == 128) return launch_bm<ROUTE, 4, 128, true>(p, st, tn0, tiles_n);
    if (bm == 256) return launch_bm<ROUTE, 4, 256, true>(p, st, tn0, tiles_n);
    return QG_EINVAL;
#else
    return QG_EUNSUPPORTED;
#endif
  }
#define QG_ROWS(BM_)                                                              \
  if (bm == BM_)                                                                  \
    return gpc == 4 ? launch_bm<ROUTE, 4, BM_>(p, st, tn0, tiles_n)               \
         : gpc == 2 ? launch_bm<ROUTE, 2, BM_>(p, st, tn0, tiles_n) : launch_bm<ROUTE, 1, BM_>(p, st, tn0, tiles_n);
  QG_ROWS(64) QG_ROWS(128) QG_ROWS(256)
#undef QG_ROWS
  return QG_EINVAL;
}

template <int ROUTE>
static int launch_route(const GemmParams& p, int bm, hipStream_t st) {
  const int tiles_n = (p.N + LARGE_BN - 1) / LARGE_BN;
  if (bm != 0) return launch_rows<ROUTE>(p, bm, st, 0, tiles_n);
  // Row-tile height by a small cost model: workgroups run in rounds of 256 (one per
  // CU), a tile costs its rows plus about 64 rows' worth of unpack and start-up.
  // 128 rows win when they fill a round that 256 rows leave half empty (M <= 256 on
  // 28672 columns, M = 384 on 57344: measured 20-30 % shorter), 256 rows otherwise.
  auto cost = [&](int rows, long cols) {
    const long tiles = ((p.M + rows - 1) / rows) * cols;
    return ((tiles + 255) / 256) * (rows + 64);
  };
  // 128-row tiles that would occupy at most half of the CUs: 64-row tiles instead -- a tile
  // costs 0.89 of a 128-row one (the unpack per matrix instruction doubles) but twice as many
  // CUs work (measured 10-15 % shorter: M = 128 on 28672 columns, M = 256..512 on 8192)
  if (large_prefers_64_rows(p.M, p.N)) return launch_rows<ROUTE>(p, 64, st, 0, tiles_n);
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

int QG_CAT(large_launch_wt, QG_WT)(const GemmParams& p, int route, int bm, hipStream_t st) {
  return route == ROUTE_F16 ? launch_route<ROUTE_F16>(p, bm, st) : launch_route<ROUTE_BF16>(p, bm, st);
}

}  // namespace qg
