// Shared host/device definitions of the gfx950 quantised-matmul library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/qgemm.h"
#include "../../include/qgemm_tuning.h"

namespace qg {

// ---- the device layout ------------------------------------------------------
// W[K,N] is cut into tiles ("chunks") of 128 (K) x 64 (N) codes.  One chunk is
// read by one wavefront as BITS loads of 16 bytes per lane:
//     load i, lane l  ->  bytes [i*1024 + l*16, +16) of the chunk
// so a lane owns RAW = 4*BITS dwords r[0..RAW) = 128 codes, as 64 (lo, hi) pairs.
// Pair t sits in two parallel 16-bit streams: the lo code occupies bits
// [t*BITS, (t+1)*BITS) of the stream made of the LOW halves of r[0], r[1], ...,
// the hi code the same bits of the stream made of the HIGH halves.  A single
// mask operation therefore extracts both codes of a pair at once, already in
// the two 16-bit lanes of the register the matrix instruction reads.
//
// Which element a pair is:   t = (j*4 + nt)*4 + v
//     j  in 0..3   k-step of 32 inside the chunk
//     nt in 0..3   16-column sub-tile
//     v  in 0..3   register of the 4-register (8-element) MFMA operand
// lane l = 16*b + i (b = k-block 0..3, i = 0..15):
//     k = 128*kc + 32*j + 8*b + 2*v + {0 (lo), 1 (hi)}
//     n = 64*nc + 4*i + nt
// Chunks of one 64-column strip are contiguous along K:
//     byte offset of chunk (kc, nc) = (nc * (K/128) + kc) * 1024 * BITS
// A second layout (QG_LAYOUT_TILE128x64_R32) has the same chunks, streams and
// byte offsets and differs only in which element a pair is: it follows the
// operand shape of the 32x32x16 matrix instruction, whose lane l feeds row
// l % 32 with the eight k values 8*(l/32) .. +7:
//     t = (j*2 + nt)*4 + v,   j in 0..7 (k-step of 16), nt in 0..1, v in 0..3
//     lane l = 32*h + i:   k = 128*kc + 16*j + 8*h + 2*v + {0, 1},   n = 64*nc + 2*i + nt
// This is the paper's "reinterpret each tile as the bytes each thread loads and
// store the tile contiguously" (Section "Efficient Low-Precision Weight
// Loading"), with T = 64 lanes and n = 16*BITS bytes per lane, so n1 = 16.
// A third layout (QG_LAYOUT_TILE128x64_I8) serves the integer matrix instruction
// v_mfma_i32_16x16x64_i8, whose lane l = 16*b + i feeds row i with 16 consecutive k values
// as the 16 bytes of four registers.  Same chunks and byte offsets, but the lane's 4*BITS
// registers are FOUR parallel byte streams (byte lane e = bits [8e, 8e+8) of every register):
// quad t occupies bits [t*BITS, (t+1)*BITS) of each byte stream, so one shift and one mask
// turn a register into four int8 operands at once.
//     t = (j*4 + nt)*4 + v,   j in 0..1 (k-step of 64), nt in 0..3, v in 0..3 (operand register)
//     byte lane e of quad t:  k = 128*kc + 64*j + 16*b + 4*v + e,   n = 64*nc + 4*i + nt
constexpr int TILE_K = QG_TILE_K;
constexpr int TILE_N = QG_TILE_N;
constexpr int PAIRS = 64;
constexpr int NUM_LAYOUT = 3;
constexpr int QUADS = 32;
__host__ __device__ constexpr int quad_k(int l, int t) { return 64 * (t / 16) + 16 * (l / 16) + 4 * (t & 3); }
__host__ __device__ constexpr int quad_n(int l, int t) { return 4 * (l % 16) + ((t >> 2) & 3); }

// Per-layout shape: columns per lane (NT), k extent of one matrix instruction
// (K_STEP), steps per chunk, and the element (k of the lo code, n) offsets inside
// the chunk of pair t of lane l.
template <int LY>
struct LayoutOf {
  static constexpr int NT = LY == 0 ? 4 : 2;
  static constexpr int K_STEP = LY == 0 ? 32 : 16;
  static constexpr int STEPS = TILE_K / K_STEP;
  static constexpr int ROWS = LY == 0 ? 16 : 32;        // lanes per k-block
  __host__ __device__ static constexpr int t0(int j, int nt) { return (j * NT + nt) * 4; }
  __host__ __device__ static constexpr int pair_k(int l, int t) { return K_STEP * (t / (4 * NT)) + 8 * (l / ROWS) + 2 * (t & 3); }
  __host__ __device__ static constexpr int pair_n(int l, int t) { return NT * (l % ROWS) + ((t >> 2) % NT); }
};
__host__ __device__ constexpr int pair_k(int layout, int l, int t) { return layout == 0 ? LayoutOf<0>::pair_k(l, t) : LayoutOf<1>::pair_k(l, t); }
__host__ __device__ constexpr int pair_n(int layout, int l, int t) { return layout == 0 ? LayoutOf<0>::pair_n(l, t) : LayoutOf<1>::pair_n(l, t); }

// ---- weight-type index used to pick a kernel instantiation ---------------------
// 0..7   integer codes of 1..8 bits (uintk; intk is stored offset-binary and
//        differs only by a constant added to the zero-point)
// 8..13  floats e1m1, e2m1, e2m2, e3m2, e3m3, e4m3 (3..8 bits)
// Kernel-side indices beyond the interface's weight types:
// 14      16-bit weights already de-quantised (the tiled kernel's pass-through)
// 15..22  codebook indices of 1..8 bits (table lookup through LDS)
constexpr int NUM_WT = 14;
constexpr int WT_DENSE16 = NUM_WT;
constexpr int WT_LUT0 = NUM_WT + 1;
constexpr int NUM_LUT = 8;

__host__ __device__ constexpr bool wt_is_lut(int wt) { return wt >= WT_LUT0 && wt < WT_LUT0 + NUM_LUT; }
__host__ __device__ constexpr int wt_bits(int wt) { return wt < 8 ? wt + 1 : wt < NUM_WT ? wt - 8 + 3 : wt == WT_DENSE16 ? 16 : wt - WT_LUT0 + 1; }
__host__ __device__ constexpr bool wt_is_float(int wt) { return wt >= 8 && wt < NUM_WT; }
__host__ __device__ constexpr int wt_ebits(int wt) {
  return wt == 8 ? 1 : wt == 9 ? 2 : wt == 10 ? 2 : wt == 11 ? 3 : wt == 12 ? 3 : wt == 13 ? 4 : 0;
}
__host__ __device__ constexpr int wt_mbits(int wt) { return wt < 8 ? 0 : wt_bits(wt) - 1 - wt_ebits(wt); }

// Float types the hardware converts by itself (OCP FP4 e2m1, FP6 e3m2, FP8 e4m3 on
// gfx950).  Their codes sit in the lane's bytes in plain order -- code c of the lane at
// bits [c*bits, (c+1)*bits), pair t = codes (2t, 2t+1) -- which is the order the
// packed convert instructions read; every other type uses the two 16-bit streams.
// Codebook indices use the same plain order: extracting an index is then a bit-field extract.
__host__ __device__ constexpr bool wt_natural(int wt) { return wt == 9 || wt == 11 || wt == 13 || wt_is_lut(wt); }

inline int wt_index(const qg_wtype& t) {
  if (t.bits < 1 || t.bits > 8) return -1;
  if (t.kind == QG_UINT || t.kind == QG_INT) return (t.ebits == 0 && t.mbits == 0) ? t.bits - 1 : -1;
  if (t.kind == QG_FLOAT) {
    if (t.bits < 3 || 1 + t.ebits + t.mbits != t.bits || t.ebits < 1) return -1;
    int wt = 8 + t.bits - 3;
    return (wt_ebits(wt) == t.ebits) ? wt : -2;   // -2: valid split, no kernel
  }
  if (t.kind == QG_CODEBOOK) return (t.ebits == 0 && t.mbits == 0) ? WT_LUT0 + t.bits - 1 : -1;
  return -1;
}

// Rounding routes of the de-quantiser.
//   ROUTE_F16  activations fp16, scales fp16: exact packed-half subtract, one
//              packed-half multiply (rounds once, to nearest even)
//   ROUTE_BF16 activations bf16, scales fp16 or bf16: exact fp32 product
//              through fused multiply-add, one hardware fp32->bf16 rounding
constexpr int ROUTE_F16 = 0;
constexpr int ROUTE_BF16 = 1;
constexpr int NUM_ROUTE = 2;

struct DequantParams {
  const uint8_t* W;
  const uint16_t* S;
  const uint8_t* Z;
  const uint16_t* T;   // codebook: 2^bits half-precision levels (codebook indices only, else unused)
  uint16_t* out;
  int layout;
  int K, N, group;
  int zbias;        // added to every zero-point (2^(bits-1) for intk, else 0)
  int scale_bf16;   // scales are bf16 (only with ROUTE_BF16)
  int scale_e8m0;   // scales are 8-bit exponents, one per 32 rows (e2m1 / e4m3 weights, group 32, first layout)
  int frag_out;     // 0: out is [K,N] row-major; 1: out is in fragment order (first layout only):
                    // 16 KiB per chunk, the four registers of (k-step j, sub-tile nt) of lane l at
                    // byte (4*j + nt) * 1024 + 16 * l -- what the tiled kernel's pass-through reads
};

struct GemmParams {
  const uint16_t* A;
  const uint8_t* W;
  const uint16_t* S;
  const uint8_t* Z;
  const uint16_t* T;    // codebook: 2^bits half-precision levels (codebook indices only, else unused)
  uint16_t* C;
  float* ws;            // split-K partial sums
  unsigned* tickets;    // one arrival counter per output tile, zero between calls
  int M, N, K, group;
  int zbias, scale_bf16;
  int scale_e8m0;       // scales are 8-bit exponents (streaming kernel only; e2m1 / e4m3, group 32)
  int splitk;           // number of K-slabs (grid.y)
  int chunks_per_split; // K-chunks per slab (last slab may be shorter)
  // group index of K-chunk c without a division: group 64 -> 2c (two groups per
  // chunk), group 32 -> 4c (four); group 128*2^s -> (c >> gshift) & gmask, with gmask 0 when one group
  // spans all of K
  int gshift, gmask;
};

// Matmul with int8 activations (third layout, integer matrix instruction).
struct A8Params {
  const int8_t* A;        // [M, K] row-major
  const float* a_scale;   // [M] or null (= 1)
  const uint8_t* W;
  const uint16_t* S;
  const uint8_t* Z;
  uint16_t* C;
  float* ws;
  unsigned* tickets;
  int M, N, K, group;
  int zbias, scale_bf16, out_bf16;
  int splitk, chunks_per_split;
  int gshift, gmask;      // as in GemmParams
};

// Fills gshift/gmask; false if the group size has no shift form (128 * odd, != K).
template <class P>
inline bool set_group_index(P& p) {
  p.gshift = 0; p.gmask = ~0;
  if (p.group == 64 || p.group == 32) return true;
  if (p.group == p.K) { p.gmask = 0; return true; }
  int q = p.group / TILE_K;
  if (q < 1 || p.group % TILE_K || (q & (q - 1))) return false;
  while ((1 << p.gshift) < q) ++p.gshift;
  return true;
}

// The 16x16 tiled kernel's own choice of 64-row tiles: when 128-row tiles would occupy at
// most half of the 256 CUs (column tiles are 256 wide).
inline bool large_prefers_64_rows(int64_t M, int64_t N) { return ((M + 127) / 128) * ((N + 255) / 256) <= 128; }

typedef int (*dequant_launch_fn)(const DequantParams&, hipStream_t);
typedef int (*gemm_launch_fn)(const GemmParams&, int mt, hipStream_t);

}  // namespace qg
