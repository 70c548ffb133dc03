// C ABI of the library: argument checks, kernel choice, workspace.  No compute
// happens on the host.
#include <atomic>
#include <mutex>
#include <string>

#include "qg_common.h"

namespace qg {

int launch_pack_codes(const uint8_t*, int, int64_t, uint8_t*, hipStream_t);
int launch_probe_stream(const void*, size_t, void*, hipStream_t);
int launch_probe_mfma(int, int, int, int, void*, hipStream_t);
int launch_repack(const uint8_t*, int, int, int, uint32_t, int, int, uint8_t*, hipStream_t);

#define QG_FOR_ALL_WT(X) X(0) X(1) X(2) X(3) X(4) X(5) X(6) X(7) X(8) X(9) X(10) X(11) X(12) X(13)

#define QG_DECL(i)                                                            \
  int dequant_launch_wt##i(const DequantParams&, int, hipStream_t);           \
  int decode_launch_wt##i(const GemmParams&, int, int, hipStream_t);          \
  int decode_waves_wt##i(int);                                                \
  int large_launch_wt##i(const GemmParams&, int, int, hipStream_t);          \
  int large32_launch_wt##i(const GemmParams&, int, int, hipStream_t);        \
  int gemv_launch_wt##i(const GemmParams&, int, int, hipStream_t);
QG_FOR_ALL_WT(QG_DECL)
#undef QG_DECL
int large_launch_wt14(const GemmParams&, int, int, hipStream_t);
// codebook indices of 1..8 bits: kernel-side weight types WT_LUT0 .. WT_LUT0 + 7
#define QG_FOR_ALL_LUT(X) X(15) X(16) X(17) X(18) X(19) X(20) X(21) X(22)
#define QG_DECL(i)                                                            \
  int dequant_launch_wt##i(const DequantParams&, int, hipStream_t);           \
  int decode_launch_wt##i(const GemmParams&, int, int, hipStream_t);          \
  int large_launch_wt##i(const GemmParams&, int, int, hipStream_t);
QG_FOR_ALL_LUT(QG_DECL)
#undef QG_DECL
#define QG_DECL_A8(b) int a8_launch_bits##b(const A8Params&, int, int, hipStream_t);
QG_DECL_A8(1) QG_DECL_A8(2) QG_DECL_A8(3) QG_DECL_A8(4) QG_DECL_A8(5) QG_DECL_A8(6) QG_DECL_A8(7) QG_DECL_A8(8)
#undef QG_DECL_A8
typedef int (*a8_fn)(const A8Params&, int, int, hipStream_t);
static const a8_fn kA8[8] = {a8_launch_bits1, a8_launch_bits2, a8_launch_bits3, a8_launch_bits4,
                             a8_launch_bits5, a8_launch_bits6, a8_launch_bits7, a8_launch_bits8};

typedef int (*dq_fn)(const DequantParams&, int, hipStream_t);
typedef int (*gm_fn)(const GemmParams&, int, int, hipStream_t);
#define QG_ENT(i) dequant_launch_wt##i,
static const dq_fn kDequant[NUM_WT] = {QG_FOR_ALL_WT(QG_ENT)};
#undef QG_ENT
#define QG_ENT(i) large_launch_wt##i,
static const gm_fn kLarge[NUM_WT] = {QG_FOR_ALL_WT(QG_ENT)};
#undef QG_ENT
#define QG_ENT(i) large32_launch_wt##i,
static const gm_fn kLarge32[NUM_WT] = {QG_FOR_ALL_WT(QG_ENT)};
#undef QG_ENT
#define QG_ENT(i) decode_launch_wt##i,
static const gm_fn kDecode[NUM_WT] = {QG_FOR_ALL_WT(QG_ENT)};
#undef QG_ENT
#define QG_ENT(i) gemv_launch_wt##i,
static const gm_fn kGemv[NUM_WT] = {QG_FOR_ALL_WT(QG_ENT)};
#undef QG_ENT
#define QG_ENT(i) dequant_launch_wt##i,
static const dq_fn kDequantLut[NUM_LUT] = {QG_FOR_ALL_LUT(QG_ENT)};
#undef QG_ENT
#define QG_ENT(i) decode_launch_wt##i,
static const gm_fn kDecodeLut[NUM_LUT] = {QG_FOR_ALL_LUT(QG_ENT)};
#undef QG_ENT
#define QG_ENT(i) large_launch_wt##i,
static const gm_fn kLargeLut[NUM_LUT] = {QG_FOR_ALL_LUT(QG_ENT)};
#undef QG_ENT
typedef int (*waves_fn)(int);
#define QG_ENT(i) decode_waves_wt##i,
static const waves_fn kDecodeWaves[NUM_WT] = {QG_FOR_ALL_WT(QG_ENT)};
#undef QG_ENT

static thread_local std::string g_last_error;
// Experiment overrides (qg_set_knob): process-wide, read once per call with relaxed loads.
static std::atomic<int> g_knob[4] = {{0}, {0}, {0}, {0}};
static int knob(int i) { return g_knob[i].load(std::memory_order_relaxed); }

static int hip_fail(hipError_t e, const char* what) {
  g_last_error = std::string(what) + ": " + hipGetErrorString(e);
  return QG_EHIP;
}

// ---- split-K workspace (partial sums + arrival counters) -----------------------------------
// What the automatic plans can ask for is bounded: the streaming kernel splits K only while
// strips x slabs stay below 512 (16 KiB of partial sums each at most), the tiled kernel only
// while tiles x slabs stay within 256 (at most 128 x 256 fp32 each).  So every workspace has
// this one capacity; only forced split factors (the experiment knobs) can exceed it.
constexpr size_t WS_PARTIAL_BYTES = size_t(32) << 20;
constexpr size_t WS_TICKETS = 16384;
constexpr size_t WS_BYTES = WS_PARTIAL_BYTES + WS_TICKETS * sizeof(unsigned);

// qgemm: one workspace per device and stream.  Kernels of one stream run in order, so they
// can share a workspace; kernels of different streams may overlap, so each stream gets its
// own.  It is allocated once, on the first call of that (device, stream) that splits K, at
// the fixed capacity, and never freed or moved, so a HIP graph captured later keeps valid
// pointers.  (A forced split beyond the capacity gets a larger block; the old one is kept
// allocated for the same reason.)  The counters are zeroed by a memset enqueued on the
// stream ahead of the first kernel; nothing synchronises.
struct Workspace {
  int dev = -1;
  hipStream_t stream = nullptr;
  unsigned char* base = nullptr;
  size_t partial_bytes = 0;
  size_t ticket_count = 0;
};
static std::mutex g_ws_mutex;
static Workspace g_ws[32];
static int g_ws_used = 0;

static int get_workspace(size_t partial_bytes, size_t ticket_count, hipStream_t st, float** partial, unsigned** tickets) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  std::lock_guard<std::mutex> lock(g_ws_mutex);
  Workspace* found = nullptr;
  for (int i = 0; i < g_ws_used; ++i)
    if (g_ws[i].dev == dev && g_ws[i].stream == st) { found = &g_ws[i]; break; }
  if (!found) {
    if (g_ws_used == 32) { g_last_error = "split-K workspaces for more than 32 (device, stream) pairs"; return QG_EUNSUPPORTED; }
    found = &g_ws[g_ws_used++];
    found->dev = dev; found->stream = st;
  }
  Workspace& w = *found;
  if (w.partial_bytes < partial_bytes || w.ticket_count < ticket_count) {
    const size_t pb = partial_bytes < WS_PARTIAL_BYTES ? WS_PARTIAL_BYTES : ((partial_bytes + 255) & ~size_t(255));
    const size_t tc = ticket_count < WS_TICKETS ? WS_TICKETS : ticket_count;
    unsigned char* block = nullptr;
    e = hipMalloc(&block, pb + tc * sizeof(unsigned));
    if (e != hipSuccess) return hip_fail(e, "hipMalloc(workspace)");
    // counters start at zero; every kernel that uses them leaves them at zero
    e = hipMemsetAsync(block + pb, 0, tc * sizeof(unsigned), st);
    if (e != hipSuccess) { (void)hipFree(block); return hip_fail(e, "hipMemsetAsync(tickets)"); }
    w.base = block; w.partial_bytes = pb; w.ticket_count = tc;      // an earlier, smaller block stays allocated
  }
  *partial = reinterpret_cast<float*>(w.base);
  *tickets = reinterpret_cast<unsigned*>(w.base + w.partial_bytes);
  return QG_OK;
}

// qgemm_noalloc: the same workspace as one fixed array in device memory, part of the code
// object (zero when it is loaded), one copy per GPU.  Its address on a device is looked up
// once, with that device current, and kept; host code never uses the array's name otherwise.
// Partial sums need no clearing (a call reads back only slots it has written itself) and
// every arrival counter is returned to zero by the last arriver of the kernel that used it.
static __device__ __align__(256) unsigned char scratch[WS_BYTES];
static std::mutex g_scratch_mutex;
static unsigned char* g_scratch_ptr[64] = {};

// Looks the array's address up on the current device (first call there) and keeps it.
static int static_scratch_base(unsigned char** base) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  if (dev < 0 || dev >= 64) { g_last_error = "qgemm_noalloc: device index beyond 63"; return QG_EUNSUPPORTED; }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return hip_fail(e, "hipGetSymbolAddress(scratch)");
    g_scratch_ptr[dev] = static_cast<unsigned char*>(ptr);
  }
  *base = g_scratch_ptr[dev];
  return QG_OK;
}

static int get_static_scratch(size_t partial_bytes, size_t ticket_count, float** partial, unsigned** tickets) {
  if (partial_bytes > WS_PARTIAL_BYTES || ticket_count > WS_TICKETS) {
    g_last_error = "qgemm_noalloc: this call needs " + std::to_string(partial_bytes) + " bytes of split-K partial sums and " +
                   std::to_string(ticket_count) + " arrival counters; the fixed scratch holds " +
                   std::to_string(WS_PARTIAL_BYTES) + " bytes and " + std::to_string(WS_TICKETS) + " counters";
    return QG_EUNSUPPORTED;
  }
  unsigned char* base = nullptr;
  int rc = static_scratch_base(&base);
  if (rc != QG_OK) return rc;
  *partial = reinterpret_cast<float*>(base);
  *tickets = reinterpret_cast<unsigned*>(base + WS_PARTIAL_BYTES);
  return QG_OK;
}

enum WsMode { WS_PER_STREAM = 0, WS_STATIC = 1 };
static int acquire_ws(int mode, size_t partial_bytes, size_t ticket_count, hipStream_t st, GemmParams& p) {
  return mode == WS_STATIC ? get_static_scratch(partial_bytes, ticket_count, &p.ws, &p.tickets)
                           : get_workspace(partial_bytes, ticket_count, st, &p.ws, &p.tickets);
}

// ---- buffer of the de-quantise-first path (forced path 4) -------------------------------------
// The whole weight in 16 bits, K*N*2 bytes, rewritten by every call: one buffer per (device,
// stream), allocated on first use and replaced (after the stream has drained) when a larger
// weight arrives.  Only this explicitly selected path allocates beyond the fixed workspace.
struct DenseBuffer { int dev = -1; hipStream_t stream = nullptr; void* ptr = nullptr; size_t bytes = 0; };
static DenseBuffer g_dense[32];
static int g_dense_used = 0;

static int get_dense_buffer(size_t bytes, hipStream_t st, void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail(e, "hipGetDevice");
  std::lock_guard<std::mutex> lock(g_ws_mutex);
  DenseBuffer* found = nullptr;
  for (int i = 0; i < g_dense_used; ++i)
    if (g_dense[i].dev == dev && g_dense[i].stream == st) { found = &g_dense[i]; break; }
  if (!found) {
    if (g_dense_used == 32) { g_last_error = "de-quantised weight buffers for more than 32 (device, stream) pairs"; return QG_EUNSUPPORTED; }
    found = &g_dense[g_dense_used++];
    found->dev = dev; found->stream = st;
  }
  if (found->bytes < bytes) {
    if (found->ptr) {
      e = hipStreamSynchronize(st);                    // earlier calls on the stream may still read the old buffer
      if (e != hipSuccess) return hip_fail(e, "hipStreamSynchronize");
      (void)hipFree(found->ptr);
      found->ptr = nullptr; found->bytes = 0;
    }
    e = hipMalloc(&found->ptr, bytes);
    if (e != hipSuccess) return hip_fail(e, "hipMalloc(de-quantised weight)");
    found->bytes = bytes;
  }
  *out = found->ptr;
  return QG_OK;
}

static bool layout_ok(int layout) { return layout == QG_LAYOUT_TILE128x64 || layout == QG_LAYOUT_TILE128x64_R32; }
static bool pack_layout_ok(int layout) { return layout_ok(layout) || layout == QG_LAYOUT_TILE128x64_I8; }
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// `codebook`: the call brought a table of levels (the *_codebook entry points); a codebook weight
// type needs one and no other type takes one.
static int check_common(qg_wtype t, int layout, int act, int scale_dtype, int64_t group, int64_t K, int64_t N,
                        int* wt_out, int* route_out, bool codebook = false) {
  if (!layout_ok(layout)) return QG_EINVAL;
  int wt = wt_index(t);
  if (wt == -2) return QG_EUNSUPPORTED;
  if (wt < 0) return QG_EINVAL;
  if (wt_is_lut(wt) != codebook) return QG_EINVAL;
  if (codebook && (layout != QG_LAYOUT_TILE128x64 || scale_dtype == QG_E8M0)) return QG_EUNSUPPORTED;
  if (K <= 0 || N <= 0 || K % TILE_K || N % TILE_N || K > (1 << 24) || N > (1 << 24)) return QG_EINVAL;
  if (group <= 0 || K % group) return QG_EINVAL;
  if (!((group % TILE_K) == 0 || group == 64 || group == 32)) return QG_EINVAL;
  if ((act != QG_F16 && act != QG_BF16) || (scale_dtype != QG_F16 && scale_dtype != QG_BF16 && scale_dtype != QG_E8M0)) return QG_EINVAL;
  if (act == QG_F16 && scale_dtype == QG_BF16) return QG_EUNSUPPORTED;
  // power-of-two block scales: 32 rows per scale, e2m1 / e4m3 codes (the scaled hardware converts), first layout
  if (scale_dtype == QG_E8M0 && (group != 32 || !(wt == 9 || wt == 13) || layout != QG_LAYOUT_TILE128x64)) return QG_EUNSUPPORTED;
  *wt_out = wt;
  *route_out = (act == QG_F16) ? ROUTE_F16 : ROUTE_BF16;
  return QG_OK;
}

// tiles of 16 rows a wavefront of the streaming kernel carries for M rows (M <= 64)
static int row_tiles(int64_t M) { return M <= 16 ? 1 : (M <= 32 ? 2 : 4); }

// Streaming kernel (M <= 64): wavefront arrangement and split-K by shape.  Host arithmetic only.
// (mx: block-scaled weights -- group 32, but only four scale bytes per block and lane, so every
// arrangement has the registers for them)
static void plan_streaming(int M, int N, int K, int group, int wt, int* variant_out, int* splitk_out, int* cps_out,
                           bool mx = false) {
  const int KC = K / TILE_K, NCH = N / TILE_N;
  const int mt = row_tiles(M);
  int variant = 10 * mt + 1;                  // 4 wavefronts on one strip
  // One row tile, short K (at most 32 chunks): as many wavefronts per strip as leaves each
  // two chunks -- 16 (every load of the strip in flight at once) up to 4-bit codes, whose
  // ring fits the 128 registers 16 wavefronts leave each; 8 from 16 chunks on; else 4.
  // With enough strips for pairs of them, two strips per workgroup as for long K below
  // (measured on K = 1024 .. 4096, N = 8192 .. 57344, 3, 4 and 8 bits: within 10 % of the
  // best arrangement everywhere; 16 wavefronts on wide codes or one-chunk shares cost 2-3x).
  if (mt == 1 && KC <= 32) {
    const int bits = wt_bits(wt);
    if (NCH % 2 == 0 && NCH / 2 >= 192) {
      variant = 14;
      if (bits <= 6 && group != 64 && KC >= 16) variant = 15;
      if (variant == 15 && NCH % 4 == 0 && NCH / 4 >= 192) variant = 16;
    } else if (KC >= 32 && bits <= 4 && NCH >= 192) {      // enough strips to occupy most CUs unsplit
      variant = 12;
    } else if (KC >= 16) {
      variant = 10;
    }
  }
  // long K and enough strips to fill the chip with pairs of them: 8 wavefronts on 2
  // adjacent strips, 4 along K each -- wavefronts at the same K position share
  // their A rows in the vector cache (measured 2-4 % shorter at K = 8192, N = 28672;
  // with 2 or 4 row tiles: 2 strips x 2 wavefronts along K, 10-15 % shorter)
  // (with several row tiles also for short K: K = 4096, N = 28672, M = 24: 20.8 us against 22.4)
  if ((KC > 32 || mt > 1) && NCH % 2 == 0 && NCH / 2 >= 192) variant = (mt == 1) ? 14 : (mt == 2) ? 26 : 46;
  // up to 6 bits per code a wavefront needs few enough registers for 16 of them per
  // workgroup (2 strips x 8 along K): twice the wavefronts in flight, 1-6 % shorter
  if (KC > 32 && variant == 14 && wt_bits(wt) <= 6 && group != 64) variant = 15;
  // and with enough strips for groups of four: 4 strips x 4 along K, half as many, twice as
  // long-lived workgroups (measured 5-9 % shorter at K = 8192, N = 57344, 2 to 6 bits)
  if (KC > 32 && variant == 15 && NCH % 4 == 0 && NCH / 4 >= 192) variant = 16;
  // long K but too few strips to fill the chip (K is split over workgroups below): more
  // wavefronts per strip for narrow codes -- 16 up to 4 bits, 8 up to 6 (measured on
  // K = N = 8192: 11 % and 7 % shorter at 4 bits, no gain at 8)
  if (variant == 11 && KC > 32 && NCH <= 128) variant = wt_bits(wt) <= 4 ? 12 : (wt_bits(wt) <= 6 ? 10 : 11);
  // between 128 and 256 strips a split in two gives more workgroups than CUs: 8-wavefront
  // workgroups, two of which share a CU (K = 8192, N = 14336: 16.3 us against 19.3 with 16
  // wavefronts at 3 bits; 8-bit codes: two strips x 4 wavefronts, 23.5 against 27.3)
  if (variant == 11 && KC > 32 && NCH > 128 && NCH < 256) variant = wt_bits(wt) <= 6 ? 10 : (NCH % 2 == 0 ? 14 : 11);
  if (knob(3) > 0) variant = knob(3);
  if (group == 32 && !mx) variant = 10 * mt + 1;   // four groups per chunk: the 4-wavefront arrangements only
  const int waves = kDecodeWaves[wt_is_lut(wt) ? 0 : wt](variant);      // the same map for every type
  // Split K over workgroups only when the column strips alone cannot fill the
  // 256 CUs, and never below 4 chunks per wavefront (2 with 16 wavefronts per strip, or with a
  // short K on at most 128 strips: K = 4096, N = 4096 .. 8192 is 15-25 % shorter with 8
  // wavefronts and K in two).
  int splitk = knob(1);
  if (splitk <= 0) {
    splitk = 1;
    const int min_chunks = (waves >= 16 || (KC <= 32 && NCH <= 128)) ? 2 : 4;      // per wavefront
    // (several row tiles on 192 or more strips: no split -- K = 4096, N = 14336, M = 24 takes
    // 12.1 us unsplit against 14.7 in two)
    while (NCH * splitk < 256 && !(mt > 1 && NCH >= 192) && KC / (splitk * 2) >= min_chunks * waves) splitk *= 2;
    // long K and still at most half of the CUs busy: K in four, down to one chunk per wavefront
    // (K = 14336, N = 4096: 11.0 us against 16.2 with K in two; deeper splits lose to the exchange)
    while (KC > 32 && splitk < 4 && NCH * splitk <= 128 && KC / (splitk * 2) >= waves) splitk *= 2;
  }
  if (splitk > KC) splitk = KC;
  const int cps = (KC + splitk - 1) / splitk;
  *variant_out = variant;
  *splitk_out = (KC + cps - 1) / cps;
  *cps_out = cps;
}

// Matrix-vector kernel (forced path 5, M <= 4): wavefronts per strip and split-K.  Host arithmetic only.
static void plan_gemv(int M, int N, int K, int group, int wt, int* waves_out, int* splitk_out, int* cps_out) {
  const int KC = K / TILE_K, NCH = N / TILE_N;
  // as many wavefronts per strip as leaves each two chunks: 16 on long K for one row of A, codes of up to 4 bits and one
  // scale group per chunk (beyond that the ring does not fit the 128 registers 16 wavefronts leave each), 8 from 16 chunks on, else 4
  // (measured: 16 pay on short slabs only -- K = 4096, or long K on at most 128 strips, where K is split;
  // K = 8192 on 448 or 896 strips is 6-13 % shorter with 8)
  const bool short_slabs = KC == 32 || (KC > 32 && NCH <= 128);
  int waves = (short_slabs && wt_bits(wt) <= 4 && M == 1 && group >= TILE_K) ? 16 : (KC >= 16 ? 8 : 4);
  if (knob(3) == 4 || knob(3) == 8 || (knob(3) == 16 && M == 1)) waves = knob(3);      // 16 wavefronts: one row only
  int splitk = knob(1);
  if (splitk <= 0) {
    splitk = 1;
    // K over workgroups while the strips alone leave CUs idle and every wavefront keeps two chunks
    while (NCH * splitk < 256 && KC / (splitk * 2) >= 2 * waves) splitk *= 2;
  }
  if (splitk > KC) splitk = KC;
  const int cps = (KC + splitk - 1) / splitk;
  *waves_out = waves; *splitk_out = (KC + cps - 1) / cps; *cps_out = cps;
}

// One launch of the streaming kernel.
static int launch_streaming(GemmParams& p, int wt, int route, int ws_mode, hipStream_t st) {
  int variant;
  plan_streaming(p.M, p.N, p.K, p.group, wt, &variant, &p.splitk, &p.chunks_per_split, p.scale_e8m0 != 0);
  const int mt = row_tiles(p.M);
  if (variant / 10 != mt) { g_last_error = "wavefront arrangement does not cover M rows"; return QG_EINVAL; }
  if (p.splitk > 1) {
    const int NCH = p.N / TILE_N;
    size_t pbytes = (size_t)p.splitk * NCH * (size_t)(mt * 16 * TILE_N) * sizeof(float);
    int rc = acquire_ws(ws_mode, pbytes, (size_t)NCH, st, p);
    if (rc != QG_OK) return rc;
  }
  return wt_is_lut(wt) ? kDecodeLut[wt - WT_LUT0](p, route, variant, st) : kDecode[wt](p, route, variant, st);
}

// Tiled kernel of the first layout: row-tile height (0 = the kernel's own choice between
// 256 and 128 rows by rounds of workgroups) and split-K.  Host arithmetic only.
//
// Split-K serves the lower row tiles when they would leave CUs idle.  Candidates: 64- or
// 128-row tiles, K cut into 1, 2, 4 or 8 slabs of an even number of chunks (the kernel
// works in pairs of chunks), at most one workgroup per CU when split.  Cost in
// microseconds, fitted to measurements at K = 1024 .. 8192, N = 2048 .. 14336:
// chunks per workgroup x time per chunk (1.33 at up to 4 bits, + 0.33 per bit above,
// x 1.13 for 128 rows) + for the exchange of partial sums 5 + 0.4 per MB with 64-row
// tiles, 11 + 0.6 per MB with 128-row tiles.
// Up to 64 rows (one 64-row tile per column tile) a fit of its own, to K = 4096 .. 28672,
// N = 4096 .. 28672 at 4, 6 and 8 bits: 6 + chunks per workgroup x (1.41 + 0.11 per bit
// above 4; float codes, whose unpack is longer: 1.6 + 0.41 per bit above 4, + 0.4 without a
// hardware convert) + 1.2 per slab (the last arriver of a tile reads the slabs back one
// pair after the other).
static void plan_tiled(int64_t M, int64_t N, int64_t K, qg_wtype t, int* bm_out, int* splitk_out, int* cps_out,
                       double* cost_out = nullptr) {
  const int bits = t.bits;
  int bm = knob(2), splitk = knob(1);
  const int KC = (int)(K / TILE_K);
  const int64_t tiles_n = (N + 255) / 256;
  if (bm == 0 && (M <= 64 || large_prefers_64_rows(M, N))) {
    bm = 64;
    if (splitk <= 0 && M <= 64) {
      const int over = bits > 4 ? bits - 4 : 0;
      const bool hw_convert = (bits == 4 || bits == 6 || bits == 8);      // e2m1, e3m2, e4m3
      const double tc = (t.kind == QG_FLOAT) ? 1.6 + 0.41 * over + (hw_convert ? 0.0 : 0.4) : 1.41 + 0.11 * over;
      double best = 1e30;
      for (int sk = 1; sk <= 8; sk *= 2) {
        int cps = (KC + sk - 1) / sk;
        if (sk > 1 && (cps & 1)) ++cps;
        if (sk > 1 && (cps < 8 || tiles_n * sk > 256)) continue;       // short slabs do not pay for the exchange
        const double rounds = (double)((tiles_n * sk + 255) / 256);
        const double cost = 6.0 + rounds * cps * tc + (sk > 1 ? 1.2 * sk : 0.0);
        if (cost < best) { best = cost; splitk = sk; }
      }
      if (cost_out) *cost_out = best;
    } else if (splitk <= 0) {
      const double tc = 1.33 + 0.33 * (bits > 4 ? bits - 4 : 0);
      double best = 1e30;
      for (int cand_bm = 64; cand_bm <= 128; cand_bm *= 2)
        for (int sk = 1; sk <= 8; sk *= 2) {
          const int64_t tiles_m = (M + cand_bm - 1) / cand_bm;
          int cps = (KC + sk - 1) / sk;
          if (sk > 1 && (cps & 1)) ++cps;
          if (sk > 1 && (cps < 4 || tiles_m * tiles_n * sk > 256)) continue;
          const double rounds = (double)((tiles_m * tiles_n * sk + 255) / 256);
          const double mb = (double)sk * (double)(tiles_m * cand_bm) * (double)(tiles_n * 256) * 4.0 / 1e6;
          const double cost = rounds * cps * tc * (cand_bm == 64 ? 1.0 : 1.13) +
                              (sk > 1 ? (cand_bm == 64 ? 5.0 + 0.4 * mb : 11.0 + 0.6 * mb) : 0.0);
          if (cost < best) { best = cost; bm = cand_bm; splitk = sk; }
        }
      if (cost_out) *cost_out = best;
    }
  }
  if (splitk <= 0 || (bm != 64 && bm != 128)) splitk = 1;
  if (splitk > KC) splitk = KC;
  int cps = (KC + splitk - 1) / splitk;
  if (splitk > 1 && (cps & 1)) ++cps;
  *bm_out = bm;
  *splitk_out = (KC + cps - 1) / cps;
  *cps_out = cps;
}

// The tiled kernels' 32-bit byte offsets: A, the packed weight and the scale array each below 2 GiB.
static bool tiled_operands_fit(int64_t M, int64_t N, int64_t K, int64_t group, int bits) {
  const uint64_t lim = 1ull << 31;
  return (uint64_t)M * (uint64_t)K * 2u < lim && (uint64_t)K * (uint64_t)N / 8u * (uint64_t)bits < lim &&
         (uint64_t)(K / group) * (uint64_t)N * 2u < lim;
}

// path of the first layout: 1 = streaming kernel, 2 = tiled kernel, 3 = streaming kernel
// over blocks of 64 rows (forced only), 4 = de-quantise first (forced, or wide codebooks on many rows)
static int plan_path(int64_t M, int64_t N, int64_t K, int64_t group, qg_wtype t) {
  const int bits = t.bits;
  if (knob(0)) return knob(0);
  // Codebooks of more than 4 bits are looked up code by code (six vector instructions and two LDS
  // reads per pair), which no longer hides between the matrix instructions of the tiled kernel: from
  // about 1024 rows on the paper's prefill variant -- de-quantise once, then the 16-bit matmul -- is
  // faster (6 bits on K = 8192, N = 57344: 1.04 ms against 1.09 at M = 1024, 3.22 against 4.11 at 4096,
  // 9.22 against 12.33 at 12288).  It needs K*N*2 bytes of library-owned buffer below 2 GiB.
  if (t.kind == QG_CODEBOOK && bits > 4 && M >= 1024 && tiled_operands_fit(M, N, K, group, bits) &&
      (uint64_t)K * (uint64_t)N * 2u < (1ull << 31)) return 4;
  if (M > 64) return 2;
  // 33 .. 64 rows: the streaming kernel (4 row tiles per wavefront) re-reads A from L2 for
  // every 64-column strip -- measured 10 us + 2.2 us (+ 0.09 per bit above 4) per 1024 of K
  // at N = 8192 -- while the tiled kernel shares A through LDS among four strips and splits K
  // instead; it wins on all but the small problems (K = 8192, N = 28672, M = 64, 6 bits:
  // 59 us against 75; K = N = 8192: a tie; K = 14336, N = 4096: 32 against 26).
  if (M > 32 && (double)K * (double)N >= 16.0e6 && knob(1) == 0 &&
      knob(2) == 0 && knob(3) == 0) {
    double tiled = 1e30;
    int bm, sk, cps;
    plan_tiled(M, N, K, t, &bm, &sk, &cps, &tiled);
    const double streaming = 10.0 + (2.2 + 0.09 * (bits > 4 ? bits - 4 : 0)) * ((double)K / 1024.0) * ((double)N / 8192.0);
    if (tiled < 0.9 * streaming) return 2;          // both fits are good to about 10 %
  }
  return 1;
}

}  // namespace qg

using namespace qg;

extern "C" {

const char* qg_status_string(int status) {
  switch (status) {
    case QG_OK: return "ok";
    case QG_EINVAL: return "invalid argument";
    case QG_EUNSUPPORTED: return "valid request with no kernel";
    case QG_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

const char* qg_last_error(void) { return g_last_error.c_str(); }

size_t qg_canonical_bytes(int bits, int64_t count) {
  if (bits < 1 || bits > 8 || count < 0) return 0;
  return (size_t)((count * bits + 7) / 8);
}

size_t qgemm_packed_bytes(qg_wtype t, int layout, int64_t K, int64_t N) {
  if (!pack_layout_ok(layout) || wt_index(t) == -1) return 0;
  if (layout == QG_LAYOUT_TILE128x64_I8 && t.kind == QG_FLOAT) return 0;
  if (t.kind == QG_CODEBOOK && layout != QG_LAYOUT_TILE128x64) return 0;
  if (K <= 0 || N <= 0 || K % TILE_K || N % TILE_N) return 0;
  return (size_t)(K * N * t.bits / 8);
}

int qg_pack_codes(const uint8_t* codes, int bits, int64_t count, uint8_t* stream_out, void* stream) {
  if (bits < 1 || bits > 8 || count < 0) return QG_EINVAL;
  if (count == 0) return QG_OK;
  if (!codes || !stream_out) return QG_EINVAL;
  return launch_pack_codes(codes, bits, count, stream_out, static_cast<hipStream_t>(stream));
}

int repack(const void* canonical, qg_wtype t, int layout, int64_t K, int64_t N, void* packed_out, void* stream) {
  if (!pack_layout_ok(layout)) return QG_EINVAL;
  int wt = wt_index(t);
  if (wt == -1) return QG_EINVAL;   // any float split can be re-laid out; only the type must be well formed
  if (layout == QG_LAYOUT_TILE128x64_I8 && t.kind == QG_FLOAT) return QG_EUNSUPPORTED;   // integer weights only
  if (t.kind == QG_CODEBOOK && layout != QG_LAYOUT_TILE128x64) return QG_EUNSUPPORTED;   // the lookup kernels read the first layout
  if (!canonical || !packed_out || canonical == packed_out) return QG_EINVAL;
  if (K <= 0 || N <= 0 || K % TILE_K || N % TILE_N || K > (1 << 24) || N > (1 << 24)) return QG_EINVAL;
  if (!aligned16(packed_out)) return QG_EINVAL;
  uint32_t flip = (t.kind == QG_INT) ? (1u << (t.bits - 1)) : 0u;
  const int natural = (wt >= 0 && wt_natural(wt) && layout != QG_LAYOUT_TILE128x64_I8) ? 1 : 0;   // types decoded by the hardware converts
  return launch_repack(static_cast<const uint8_t*>(canonical), t.bits, (int)K, (int)N, flip, natural, layout,
                       static_cast<uint8_t*>(packed_out), static_cast<hipStream_t>(stream));
}

static int qdequant_run(const void* packed_W, const void* scales, const uint8_t* zeros, const void* codebook, bool with_codebook,
                        qg_wtype t, int layout, int act, int scale_dtype, int64_t group, int64_t K, int64_t N, void* W_out,
                        void* stream) {
  if (group == 0) group = K;               // 0 = one scale per output column
  int wt, route;
  int rc = check_common(t, layout, act, scale_dtype, group, K, N, &wt, &route, with_codebook);
  if (rc != QG_OK) return rc;
  if (!packed_W || !scales || !W_out || (with_codebook && !codebook)) return QG_EINVAL;
  if (!aligned16(packed_W) || !aligned16(scales) || !aligned16(W_out) || (zeros && !aligned16(zeros)) ||
      (codebook && (reinterpret_cast<uintptr_t>(codebook) & 1u))) return QG_EINVAL;
  DequantParams p;
  p.W = static_cast<const uint8_t*>(packed_W);
  p.S = static_cast<const uint16_t*>(scales);
  p.Z = zeros;
  p.T = static_cast<const uint16_t*>(codebook);
  p.out = static_cast<uint16_t*>(W_out);
  p.layout = layout;
  p.K = (int)K; p.N = (int)N; p.group = (int)group;
  p.zbias = (t.kind == QG_INT) ? (1 << (t.bits - 1)) : 0;
  p.scale_bf16 = (scale_dtype == QG_BF16);
  p.scale_e8m0 = (scale_dtype == QG_E8M0);
  if (p.scale_e8m0 && zeros) return QG_EINVAL;       // block scales come without zero-points
  p.frag_out = 0;
  if (wt_is_lut(wt)) return kDequantLut[wt - WT_LUT0](p, route, static_cast<hipStream_t>(stream));
  return kDequant[wt](p, route, static_cast<hipStream_t>(stream));
}

int qdequant(const void* packed_W, const void* scales, const uint8_t* zeros, qg_wtype t, int layout, int act,
             int scale_dtype, int64_t group, int64_t K, int64_t N, void* W_out, void* stream) {
  return qdequant_run(packed_W, scales, zeros, nullptr, false, t, layout, act, scale_dtype, group, K, N, W_out, stream);
}

int qdequant_codebook(const void* packed_W, const void* codebook, const void* scales, int bits, int act, int scale_dtype,
                      int64_t group, int64_t K, int64_t N, void* W_out, void* stream) {
  const qg_wtype t = {QG_CODEBOOK, bits, 0, 0};
  return qdequant_run(packed_W, scales, nullptr, codebook, true, t, QG_LAYOUT_TILE128x64, act, scale_dtype, group, K, N, W_out, stream);
}

static int qgemm_run(const void* A, const void* packed_W, const void* scales, const uint8_t* zeros, qg_wtype t, int layout,
                     int act, int scale_dtype, int64_t group, int64_t M, int64_t N, int64_t K, void* C, void* stream,
                     int ws_mode, const void* codebook = nullptr, bool with_codebook = false) {
  if (group == 0) group = K;               // 0 = one scale per output column
  int wt, route;
  int rc = check_common(t, layout, act, scale_dtype, group, K, N, &wt, &route, with_codebook);
  if (rc != QG_OK) return rc;
  if (M < 0 || M > (1 << 24)) return QG_EINVAL;
  if (ws_mode == WS_STATIC) {
    // every call with valid shapes, also one with M = 0 or one that will not split K, makes sure
    // the scratch array's address on this device is known: the first such call on a device is the
    // set-up (the runtime loads this library's device code then, if nothing of it has run yet),
    // which a caller that must not allocate later can do once with M = 0
    unsigned char* base = nullptr;
    rc = static_scratch_base(&base);
    if (rc != QG_OK) return rc;
  }
  if (M == 0) return QG_OK;
  if (!A || !packed_W || !scales || !C || (with_codebook && !codebook)) return QG_EINVAL;
  if (!aligned16(A) || !aligned16(packed_W) || !aligned16(scales) || !aligned16(C) || (zeros && !aligned16(zeros)) ||
      (codebook && (reinterpret_cast<uintptr_t>(codebook) & 1u))) return QG_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  // one handle value that names a different stream in every thread: the per-stream
  // workspaces (and the stream order the shared scratch relies on) cannot be keyed by it
  if (st == hipStreamPerThread) { g_last_error = "hipStreamPerThread is not accepted: pass a stream of your own"; return QG_EINVAL; }

  GemmParams p;
  p.A = static_cast<const uint16_t*>(A);
  p.W = static_cast<const uint8_t*>(packed_W);
  p.S = static_cast<const uint16_t*>(scales);
  p.Z = zeros;
  p.T = static_cast<const uint16_t*>(codebook);
  p.C = static_cast<uint16_t*>(C);
  p.ws = nullptr; p.tickets = nullptr;
  p.M = (int)M; p.N = (int)N; p.K = (int)K; p.group = (int)group;
  p.zbias = (t.kind == QG_INT) ? (1 << (t.bits - 1)) : 0;
  p.scale_bf16 = (scale_dtype == QG_BF16);
  p.scale_e8m0 = (scale_dtype == QG_E8M0);
  if (p.scale_e8m0 && zeros) return QG_EINVAL;       // block scales come without zero-points
  p.splitk = 1; p.chunks_per_split = (int)(K / TILE_K);
  if (!set_group_index(p)) return QG_EUNSUPPORTED;

  // The tiled kernels address A, the packed weight and the scales through buffer
  // resources with 32-bit byte offsets, some of them formed in signed arithmetic and A's
  // with the top bit used to push padding rows out of range: each operand stays below 2 GiB.
  const bool fits32 = tiled_operands_fit(M, N, K, group, t.bits);
  if (layout == QG_LAYOUT_TILE128x64_R32) {      // one kernel for every M
    if (!fits32 || group == 32) return QG_EUNSUPPORTED;      // the second layout's kernel has no variant for four groups per chunk
    return kLarge32[wt](p, route, knob(2), st);
  }

  int path = plan_path(M, N, K, group, t);
  if (p.scale_e8m0 && path == 4) return QG_EUNSUPPORTED;      // the de-quantise-first path has no block-scaled variant
  if (path == 1 && M > 64) return QG_EINVAL;
  if (path < 1 || path > 5) return QG_EINVAL;
  if (path == 5) {
    // The decode-sized product as matrix-vector products on the vector ALU (two-element dot
    // products, partial sums added across lanes with permutes): the measured alternative to
    // the matrix-core streaming kernel for M <= 4.  Forced only.
    if (M > 4 || wt_is_lut(wt)) return QG_EINVAL;
    if (p.scale_e8m0) return QG_EUNSUPPORTED;
    int waves;
    plan_gemv(p.M, p.N, p.K, p.group, wt, &waves, &p.splitk, &p.chunks_per_split);
    if (p.splitk > 1) {
      const int NCH = p.N / TILE_N;
      const int mr = M <= 1 ? 1 : 4;
      rc = acquire_ws(ws_mode, (size_t)p.splitk * NCH * (size_t)(mr * TILE_N) * sizeof(float), (size_t)NCH, st, p);
      if (rc != QG_OK) return rc;
    }
    return kGemv[wt](p, route, waves, st);
  }

  void* dense = nullptr;
  if (path == 4) {
    // The paper's prefill variant (Section "End-to-End Performance"): de-quantise the whole
    // weight to 16 bits once, then a plain 16-bit matmul -- here the same tiled kernel reading
    // ready-made operand registers instead of unpacking codes.
    const uint64_t dense_bytes = (uint64_t)K * (uint64_t)N * 2u;
    if (!fits32 || dense_bytes >= (1ull << 31)) return QG_EUNSUPPORTED;
    if (ws_mode == WS_STATIC) { g_last_error = "qgemm_noalloc: the de-quantise-first path needs a K*N*2-byte buffer"; return QG_EUNSUPPORTED; }
    rc = get_dense_buffer((size_t)dense_bytes, st, &dense);
    if (rc != QG_OK && knob(0) == 4) return rc;
    if (rc != QG_OK) path = 2;       // chosen by the library, no memory for the buffer: the fused kernel instead
  }
  if (path == 4) {
    DequantParams d;
    d.W = p.W; d.S = p.S; d.Z = p.Z; d.out = static_cast<uint16_t*>(dense);
    d.layout = QG_LAYOUT_TILE128x64; d.K = p.K; d.N = p.N; d.group = p.group; d.zbias = p.zbias; d.scale_bf16 = p.scale_bf16;
    d.scale_e8m0 = 0;
    d.frag_out = 1;
    d.T = p.T;
    rc = wt_is_lut(wt) ? kDequantLut[wt - WT_LUT0](d, route, st) : kDequant[wt](d, route, st);
    if (rc != QG_OK) return rc;
    GemmParams q = p;
    q.W = static_cast<const uint8_t*>(dense);
    q.Z = nullptr; q.group = p.K; q.zbias = 0;
    if (!set_group_index(q)) return QG_EINVAL;
    qg_wtype t16 = {QG_UINT, 4, 0, 0};               // cost model of the tiled kernel: nothing to unpack, as for a narrow code
    int bm;
    plan_tiled(M, N, K, t16, &bm, &q.splitk, &q.chunks_per_split);
    if (q.splitk > 1) {
      const int64_t tiles = ((M + bm - 1) / bm) * ((N + 255) / 256);
      rc = acquire_ws(ws_mode, (size_t)q.splitk * (size_t)tiles * (size_t)(bm * 256) * sizeof(float), (size_t)tiles * 4, st, q);
      if (rc != QG_OK) return rc;
    }
    return large_launch_wt14(q, route, bm, st);
  }

  if (path == 1 || path == 3) {
    // a forced arrangement must have the row tiles every block of rows needs, or rows would stay unwritten
    if (knob(3) > 0 && (group != 32 || p.scale_e8m0))
      for (int64_t r0 = 0; r0 < M; r0 += 64)
        if (knob(3) / 10 != row_tiles(M - r0 < 64 ? M - r0 : 64)) { g_last_error = "forced wavefront arrangement does not cover the rows of M"; return QG_EINVAL; }
    for (int64_t r0 = 0; r0 < M; r0 += 64) {
      GemmParams q = p;
      q.A = p.A + r0 * K;
      q.C = p.C + r0 * N;
      q.M = (int)((M - r0 < 64) ? (M - r0) : 64);
      rc = launch_streaming(q, wt, route, ws_mode, st);
      if (rc != QG_OK) return rc;
    }
    return QG_OK;
  }
  if (!fits32) return QG_EUNSUPPORTED;
  int bm;
  plan_tiled(M, N, K, t, &bm, &p.splitk, &p.chunks_per_split);
  if (p.splitk > 1) {
    const int64_t tiles = ((M + bm - 1) / bm) * ((N + 255) / 256);
    rc = acquire_ws(ws_mode, (size_t)p.splitk * (size_t)tiles * (size_t)(bm * 256) * sizeof(float), (size_t)tiles * 4, st, p);   // a ticket per 64-column strip
    if (rc != QG_OK) return rc;
  }
  return wt_is_lut(wt) ? kLargeLut[wt - WT_LUT0](p, route, bm, st) : kLarge[wt](p, route, bm, st);
}

int qgemm(const void* A, const void* packed_W, const void* scales, const uint8_t* zeros, qg_wtype t, int layout,
          int act, int scale_dtype, int64_t group, int64_t M, int64_t N, int64_t K, void* C, void* stream) {
  return qgemm_run(A, packed_W, scales, zeros, t, layout, act, scale_dtype, group, M, N, K, C, stream, WS_PER_STREAM);
}

int qgemm_noalloc(const void* A, const void* packed_W, const void* scales, const uint8_t* zeros, qg_wtype t, int layout,
                  int act, int scale_dtype, int64_t group, int64_t M, int64_t N, int64_t K, void* C, void* stream) {
  return qgemm_run(A, packed_W, scales, zeros, t, layout, act, scale_dtype, group, M, N, K, C, stream, WS_STATIC);
}

int qgemm_codebook(const void* A, const void* packed_W, const void* codebook, const void* scales, int bits, int act,
                   int scale_dtype, int64_t group, int64_t M, int64_t N, int64_t K, void* C, void* stream) {
  const qg_wtype t = {QG_CODEBOOK, bits, 0, 0};
  return qgemm_run(A, packed_W, scales, nullptr, t, QG_LAYOUT_TILE128x64, act, scale_dtype, group, M, N, K, C, stream,
                   WS_PER_STREAM, codebook, true);
}

// int8 activations: wavefronts per strip, row tiles and split-K of one block of at most 64 rows
static void plan_a8(int M, int N, int K, int* waves_out, int* splitk_out, int* cps_out) {
  const int KC = K / TILE_K, NCH = N / TILE_N;
  // eight wavefronts per strip on long K; four with four row tiles (their accumulators and
  // the ring do not fit the registers eight wavefronts leave each) and on short K
  int waves = (KC >= 16 && row_tiles(M) < 4) ? 8 : 4;
  int splitk = knob(1);
  if (splitk <= 0) {
    splitk = 1;
    // K over workgroups while the strips alone leave CUs idle and every wavefront keeps two chunks
    while (NCH * splitk < 256 && KC / (splitk * 2) >= 2 * waves) splitk *= 2;
  }
  if (splitk > KC) splitk = KC;
  const int cps = (KC + splitk - 1) / splitk;
  *waves_out = waves; *splitk_out = (KC + cps - 1) / cps; *cps_out = cps;
}

int qgemm_a8(const int8_t* A8, const float* a_scale, const void* packed_W, const void* scales, const uint8_t* zeros,
             qg_wtype t, int out_dtype, int scale_dtype, int64_t group, int64_t M, int64_t N, int64_t K, void* C,
             void* stream) {
  if (group == 0) group = K;
  int wt = wt_index(t);
  if (wt == -1) return QG_EINVAL;
  if (t.kind == QG_CODEBOOK) return QG_EINVAL;                    // no table in this call
  if (t.kind == QG_FLOAT) return QG_EUNSUPPORTED;                 // the integer instruction multiplies integers
  if (K <= 0 || N <= 0 || K % TILE_K || N % TILE_N || K > (1 << 24) || N > (1 << 24)) return QG_EINVAL;
  if (group <= 0 || K % group) return QG_EINVAL;
  if (group == 32) return QG_EUNSUPPORTED;                         // the instruction sums 64 values of k
  if (!((group % TILE_K) == 0 || group == 64)) return QG_EINVAL;
  if ((out_dtype != QG_F16 && out_dtype != QG_BF16) || (scale_dtype != QG_F16 && scale_dtype != QG_BF16)) return QG_EINVAL;
  if (M < 0 || M > (1 << 24)) return QG_EINVAL;
  if (M == 0) return QG_OK;
  if (!A8 || !packed_W || !scales || !C) return QG_EINVAL;
  if (!aligned16(A8) || !aligned16(packed_W) || !aligned16(scales) || !aligned16(C) || (zeros && !aligned16(zeros)) ||
      (a_scale && (reinterpret_cast<uintptr_t>(a_scale) & 3u))) return QG_EINVAL;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (st == hipStreamPerThread) { g_last_error = "hipStreamPerThread is not accepted: pass a stream of your own"; return QG_EINVAL; }

  A8Params p;
  p.A = A8; p.a_scale = a_scale;
  p.W = static_cast<const uint8_t*>(packed_W);
  p.S = static_cast<const uint16_t*>(scales);
  p.Z = zeros;
  p.C = static_cast<uint16_t*>(C);
  p.ws = nullptr; p.tickets = nullptr;
  p.N = (int)N; p.K = (int)K; p.group = (int)group;
  p.zbias = (t.kind == QG_INT) ? (1 << (t.bits - 1)) : 0;
  p.scale_bf16 = (scale_dtype == QG_BF16);
  p.out_bf16 = (out_dtype == QG_BF16);
  p.M = 0;
  if (!set_group_index(p)) return QG_EUNSUPPORTED;
  for (int64_t r0 = 0; r0 < M; r0 += 64) {
    A8Params q = p;
    q.A = p.A + r0 * K;
    q.a_scale = a_scale ? a_scale + r0 : nullptr;
    q.C = p.C + r0 * N;
    q.M = (int)((M - r0 < 64) ? (M - r0) : 64);
    int waves;
    plan_a8(q.M, q.N, q.K, &waves, &q.splitk, &q.chunks_per_split);
    const int mt = row_tiles(q.M);
    if (q.splitk > 1) {
      const int NCH = q.N / TILE_N;
      float* ws = nullptr; unsigned* tk = nullptr;
      int rc = get_workspace((size_t)q.splitk * NCH * (size_t)(mt * 16 * TILE_N) * sizeof(float), (size_t)NCH, st, &ws, &tk);
      if (rc != QG_OK) return rc;
      q.ws = ws; q.tickets = tk;
    }
    int rc = kA8[t.bits - 1](q, waves, mt, st);
    if (rc != QG_OK) return rc;
  }
  return QG_OK;
}

int qg_probe_stream_read(const void* buf, size_t bytes, void* sink, void* stream) {
  if (!buf || !sink || bytes < 16 || !aligned16(buf)) return QG_EINVAL;
  return launch_probe_stream(buf, bytes, sink, static_cast<hipStream_t>(stream));
}

int qg_probe_mfma(int bf16, int random_data, int iters, int waves_per_simd, void* sink, double* flops_out, void* stream) {
  if (!sink || iters < 1 || waves_per_simd < 1 || waves_per_simd > 8) return QG_EINVAL;
  // 8 instructions of 32*32*16*2 flop per iteration and wavefront, 4 wavefronts per block
  if (flops_out) *flops_out = 8.0 * 32768.0 * (double)iters * 4.0 * 256.0 * waves_per_simd;
  return launch_probe_mfma(bf16 != 0, random_data != 0, iters, waves_per_simd, sink, static_cast<hipStream_t>(stream));
}

int qg_plan(qg_wtype t, int layout, int act, int scale_dtype, int64_t group, int64_t M, int64_t N, int64_t K, int plan[5]) {
  if (group == 0) group = K;               // 0 = one scale per output column
  int wt, route;
  int rc = check_common(t, layout, act, scale_dtype, group, K, N, &wt, &route, t.kind == QG_CODEBOOK);
  if (rc != QG_OK) return rc;
  if (M < 1 || M > (1 << 24) || !plan) return QG_EINVAL;
  plan[0] = plan[1] = plan[2] = 0; plan[3] = 1; plan[4] = (int)(K / TILE_K);
  if (layout == QG_LAYOUT_TILE128x64_R32) {
    plan[0] = 2; plan[2] = knob(2);
    return (group == 32 || !tiled_operands_fit(M, N, K, group, t.bits)) ? QG_EUNSUPPORTED : QG_OK;
  }
  plan[0] = plan_path(M, N, K, group, t);
  if (scale_dtype == QG_E8M0 && plan[0] == 4) return QG_EUNSUPPORTED;   // the de-quantise-first path has no block-scaled variant
  if (plan[0] == 1 && M > 64) return QG_EINVAL;
  if (plan[0] == 1 || plan[0] == 3) {
    plan_streaming((int)(M < 64 ? M : 64), (int)N, (int)K, (int)group, wt, &plan[1], &plan[3], &plan[4], scale_dtype == QG_E8M0);
    if (knob(3) > 0 && (group != 32 || scale_dtype == QG_E8M0))
      for (int64_t r0 = 0; r0 < M; r0 += 64)
        if (knob(3) / 10 != row_tiles(M - r0 < 64 ? M - r0 : 64)) return QG_EINVAL;
  } else {
    if (plan[0] < 1 || plan[0] > 5) return QG_EINVAL;
    if (plan[0] == 5) {
      if (M > 4 || wt_is_lut(wt)) return QG_EINVAL;
      if (scale_dtype == QG_E8M0) return QG_EUNSUPPORTED;
      plan_gemv((int)M, (int)N, (int)K, (int)group, wt, &plan[1], &plan[3], &plan[4]);
      return QG_OK;
    }
    if (!tiled_operands_fit(M, N, K, group, t.bits)) return QG_EUNSUPPORTED;
    qg_wtype tt = t;
    if (plan[0] == 4) {
      if ((uint64_t)K * (uint64_t)N * 2u >= (1ull << 31)) return QG_EUNSUPPORTED;
      tt = qg_wtype{QG_UINT, 4, 0, 0};
    }
    plan_tiled(M, N, K, tt, &plan[2], &plan[3], &plan[4]);
  }
  return QG_OK;
}

int qg_set_knob(int knob, int value) {
  if (knob < 0 || knob >= 4) return 0;
  return g_knob[knob].exchange(value, std::memory_order_relaxed);
}

}  // extern "C"
