// Compact storage and the offline re-layout of the weight.
//   pack_codes_kernel : one code per byte -> canonical gap-free bit stream
//                       (paper, Section "Storage of Low-Precision Data")
//   repack_kernel     : canonical [K,N] stream -> tiled device layout
//                       (paper, Section "Efficient Low-Precision Weight Loading",
//                       the "Change Layout" pre-processing step)
#include "qg_common.h"

namespace qg {

// Eight consecutive codes fill exactly `bits` bytes; one thread writes them.
__global__ __launch_bounds__(256) void pack_codes_kernel(const uint8_t* __restrict__ codes, int bits,
                                                         int64_t count, uint8_t* __restrict__ out,
                                                         int64_t out_bytes) {
  int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t e0 = g * 8;
  if (e0 >= count) return;
  const uint32_t mask = (1u << bits) - 1u;
  uint64_t acc = 0;
  for (int i = 0; i < 8; ++i) {
    uint64_t c = (e0 + i < count) ? (codes[e0 + i] & mask) : 0u;
    acc |= c << (i * bits);
  }
  int64_t b0 = g * bits;
  for (int i = 0; i < bits; ++i)
    if (b0 + i < out_bytes) out[b0 + i] = (uint8_t)(acc >> (8 * i));
}

__device__ __forceinline__ uint32_t fetch_code(const uint8_t* __restrict__ canon, int64_t canon_bytes,
                                               int64_t elem, int bits) {
  int64_t bit = elem * bits;
  int64_t byte = bit >> 3;
  int sh = (int)(bit & 7);
  uint32_t w = canon[byte];
  if (sh + bits > 8 && byte + 1 < canon_bytes) w |= (uint32_t)canon[byte + 1] << 8;
  return (w >> sh) & ((1u << bits) - 1u);
}

// One thread builds one lane's 4*bits dwords of one chunk (see qg_common.h for
// the element <-> (chunk, lane, pair) map) and writes them where load i of that
// lane will find them.
__global__ __launch_bounds__(256) void repack_kernel(const uint8_t* __restrict__ canon, int64_t canon_bytes,
                                                     uint32_t* __restrict__ out, int bits, int K, int N,
                                                     uint32_t flip, int natural, int layout) {
  const int KC = K / TILE_K;
  const int64_t nchunks = (int64_t)KC * (N / TILE_N);
  int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t chunk = gid >> 6;
  if (chunk >= nchunks) return;
  const int l = (int)(gid & 63);
  const int nc = (int)(chunk / KC), kc = (int)(chunk % KC);
  uint32_t* dst = out + chunk * (256 * bits);
  if (layout == QG_LAYOUT_TILE128x64_I8) {
    // four parallel byte streams: quad t at bits [t*bits, (t+1)*bits) of byte lane e of the registers
    for (int d = 0; d < 4 * bits; ++d) {
      uint32_t word = 0;
      int t0 = (8 * d) / bits, t1 = (8 * d + 7) / bits;
      if (t1 > QUADS - 1) t1 = QUADS - 1;
      for (int t = t0; t <= t1; ++t) {
        const int n = TILE_N * nc + quad_n(l, t);
        const int sh = t * bits - 8 * d;
        for (int e = 0; e < 4; ++e) {
          const int k = TILE_K * kc + quad_k(l, t) + e;
          const uint32_t code = fetch_code(canon, canon_bytes, (int64_t)k * N + n, bits) ^ flip;
          const uint32_t part = ((sh >= 0) ? (code << sh) : (code >> (-sh))) & 0xffu;
          word |= part << (8 * e);
        }
      }
      dst[(d >> 2) * 256 + l * 4 + (d & 3)] = word;
    }
    return;
  }
  if (natural) {
    // plain order: code c = 2t + {0 lo, 1 hi} of the lane at bits [c*bits, (c+1)*bits)
    for (int d = 0; d < 4 * bits; ++d) {
      uint32_t word = 0;
      int c0 = (32 * d) / bits, c1 = (32 * d + 31) / bits;
      if (c1 > 2 * PAIRS - 1) c1 = 2 * PAIRS - 1;
      for (int c = c0; c <= c1; ++c) {
        int t = c >> 1;
        int k = TILE_K * kc + pair_k(layout, l, t) + (c & 1);
        int n = TILE_N * nc + pair_n(layout, l, t);
        uint32_t code = fetch_code(canon, canon_bytes, (int64_t)k * N + n, bits);
        int sh = c * bits - 32 * d;
        word |= (sh >= 0) ? (code << sh) : (code >> (-sh));
      }
      dst[(d >> 2) * 256 + l * 4 + (d & 3)] = word;
    }
    return;
  }
  for (int d = 0; d < 4 * bits; ++d) {
    uint32_t lo = 0, hi = 0;
    int t0 = (16 * d) / bits, t1 = (16 * d + 15) / bits;
    if (t1 > PAIRS - 1) t1 = PAIRS - 1;
    for (int t = t0; t <= t1; ++t) {
      int k = TILE_K * kc + pair_k(layout, l, t);
      int n = TILE_N * nc + pair_n(layout, l, t);
      uint32_t clo = fetch_code(canon, canon_bytes, (int64_t)k * N + n, bits) ^ flip;
      uint32_t chi = fetch_code(canon, canon_bytes, (int64_t)(k + 1) * N + n, bits) ^ flip;
      int sh = t * bits - 16 * d;
      if (sh >= 0) { lo |= clo << sh; hi |= chi << sh; }
      else         { lo |= clo >> (-sh); hi |= chi >> (-sh); }
    }
    dst[(d >> 2) * 256 + l * 4 + (d & 3)] = (lo & 0xffffu) | (hi << 16);
  }
}

int launch_pack_codes(const uint8_t* codes, int bits, int64_t count, uint8_t* out, hipStream_t st) {
  int64_t groups = (count + 7) / 8;
  int64_t out_bytes = (count * bits + 7) / 8;
  if (groups == 0) return QG_OK;
  int64_t blocks = (groups + 255) / 256;
  hipLaunchKernelGGL(pack_codes_kernel, dim3((unsigned)blocks), dim3(256), 0, st, codes, bits, count, out, out_bytes);
  return hipGetLastError() == hipSuccess ? QG_OK : QG_EHIP;
}

int launch_repack(const uint8_t* canon, int bits, int K, int N, uint32_t flip, int natural, int layout, uint8_t* out, hipStream_t st) {
  int64_t nchunks = (int64_t)(K / TILE_K) * (N / TILE_N);
  int64_t canon_bytes = ((int64_t)K * N * bits + 7) / 8;
  int64_t blocks = (nchunks * 64 + 255) / 256;
  hipLaunchKernelGGL(repack_kernel, dim3((unsigned)blocks), dim3(256), 0, st, canon, canon_bytes,
                     reinterpret_cast<uint32_t*>(out), bits, K, N, flip, natural, layout);
  return hipGetLastError() == hipSuccess ? QG_OK : QG_EHIP;
}

}  // namespace qg
