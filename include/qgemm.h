/*
 * qgemm.h -- C ABI of the MI355X (gfx950) mixed-precision matmul library
 *
 *     C[M,N] = A[M,K] . dequant(W[K,N])
 *
 * A and C are fp16 or bf16, W holds 1..8-bit codes (uintk, intk, small floats)
 * stored bit-packed with group-wise scales and zero-points.  The contraction is
 * the problem statement of the Tilus paper (arXiv 2504.12984, Section "An
 * Example of Tilus Program": C = A x B, A float16, B a low-bit type).  The
 * operations below are the pieces of that paper's data path:
 *
 *   qg_pack_codes       compact, gap-free storage of sub-byte values in a byte
 *                       array (Section "Storage of Low-Precision Data")
 *   repack              the offline "Change Layout" step: tile the weight and
 *                       store each tile as the byte string the threads will
 *                       load (Section "Efficient Low-Precision Support in LLMs",
 *                       "Efficient Low-Precision Weight Loading")
 *   qdequant            load + reinterpret + vectorised cast/de-quantise
 *                       (same section, "Efficient Casting"), written out to
 *                       memory so it can be checked bit for bit
 *   qgemm               the full kernel: pipelined weight load, in-register
 *                       cast, matrix-core accumulate, store (Sections "Key
 *                       Ideas" and "An Example of Tilus Program")
 *
 * Conventions common to every call
 *   - every pointer is DEVICE memory owned by the caller, 16-byte aligned;
 *   - work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *     default stream) and the call returns without synchronising;
 *   - the return value is a qg_status (0 = ok, negative = error, nothing was
 *     enqueued); no call throws, none frees caller memory;
 *   - qgemm may use a library-owned workspace for split-K partial sums: one per
 *     (device, stream), of one fixed size (32 MiB + 64 KiB, which covers every
 *     shape), allocated by the first call on that pair that splits K (one
 *     hipMalloc and one memset enqueued on the stream; nothing synchronises) and
 *     then never freed, moved or grown, so calls on different streams may overlap
 *     and a HIP graph captured later keeps valid pointers.  At most 32 (device,
 *     stream) pairs per process (QG_EUNSUPPORTED beyond); a stream that is
 *     destroyed and whose handle value is re-used simply inherits the workspace.
 *     hipStreamPerThread is refused (QG_EINVAL): the one handle value names a
 *     different stream in every thread.  Calls may be captured into a HIP graph
 *     once a call that splits K has run eagerly on the capture stream (so that
 *     nothing is allocated during the capture); every launch leaves counters and
 *     workspace ready for the next, so a graph can be replayed any number of
 *     times.  qgemm_noalloc is the same call with no allocation at all.
 *
 * De-quantisation (the paper names the step but prints no formula; this is the
 * standard affine group form):
 *        w[k,n] = rne_act( (value(code[k,n]) - z[k/g, n]) * s[k/g, n] )
 *   value(): uintk -> code; intk -> two's complement (int1 = {0,-1});
 *            floatk -> sign|exponent|mantissa, bias 2^(e-1)-1, subnormals, no
 *            infinities; e4m3's S.1111.111 is NaN and must not be used
 *   one rounding, to nearest even, to the activation type; the contraction
 *   accumulates products of A with these ROUNDED weights in fp32 and rounds
 *   the sum once (nearest even) to the activation type.
 */
#ifndef QGEMM_H_
#define QGEMM_H_

#include <stddef.h>
#include <stdint.h>

#define QG_API __attribute__((visibility("default")))

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { QG_OK = 0, QG_EINVAL = -1, QG_EUNSUPPORTED = -2, QG_EHIP = -3 } qg_status;
typedef enum { QG_UINT = 0, QG_INT = 1, QG_FLOAT = 2, QG_CODEBOOK = 3 } qg_kind;
typedef enum { QG_F16 = 0, QG_BF16 = 1, QG_E8M0 = 2 } qg_dtype;   /* activation / scale dtype; QG_E8M0: scales only */

/* Weight type.  uint/int: bits in 1..8, ebits = mbits = 0.  float: 1 + ebits +
 * mbits == bits; supported splits are the paper's representative set
 * e1m1, e2m1, e2m2, e3m2, e3m3, e4m3 (Section "Arbitrary Data Type Support").
 * codebook: bits in 1..8, ebits = mbits = 0; a code is an index into a table of 2^bits levels
 * that the *_codebook calls take (repack and qgemm_packed_bytes accept the kind, qdequant /
 * qgemm / qgemm_a8 answer QG_EINVAL: they have no table). */
typedef struct { int32_t kind, bits, ebits, mbits; } qg_wtype;

/* Device layouts.  In all of them W is cut into tiles of 128 (K) x 64 (N) codes; a tile
 * is 1024*bits bytes, read by one 64-lane wavefront as `bits` 16-byte loads per
 * lane, and the lane's 16*bits bytes hold exactly the 128 codes that lane feeds to
 * the matrix instruction (no exchange between lanes, no staging through LDS).
 * Tiles of one 64-column strip are contiguous along K.  intk codes are stored
 * offset-binary (sign bit flipped).  The layouts differ in which 128 codes a lane
 * owns, i.e. in the matrix instruction the kernels built for them use (the paper
 * transforms the weight for the program that will read it, Section "Efficient
 * Low-Precision Weight Loading"):
 *   QG_LAYOUT_TILE128x64      lane owns 4 columns; 16x16x32 instruction.  A streaming
 *                             kernel for M <= 64 and a tiled kernel (with split-K)
 *                             above; the default, and the faster one at every M.
 *   QG_LAYOUT_TILE128x64_R32  lane owns 2 columns; 32x32x16 instruction.  One tiled
 *                             kernel for every M (no split-K, no group size 32),
 *                             about 5 % slower than the first layout's on the prefill
 *                             shapes: the measured alternative, kept with its tests.
 *   QG_LAYOUT_TILE128x64_I8   for int8 activations (qgemm_a8): lane owns 4 columns, its bytes
 *                             are four parallel byte streams that unpack straight into the
 *                             int8 operands of the 16x16x64 integer instruction.  Integer
 *                             weight types only; qdequant and qgemm do not read it. */
#define QG_LAYOUT_TILE128x64 0
#define QG_LAYOUT_TILE128x64_R32 1
#define QG_LAYOUT_TILE128x64_I8 2
#define QG_TILE_K 128
#define QG_TILE_N 64

QG_API const char* qg_status_string(int status);
/* Text of the last HIP error seen by this library on the calling thread. */
QG_API const char* qg_last_error(void);

/* ceil(count*bits/8): bytes of the canonical little-endian bit stream -- values stored
 * back to back with no bit gaps (Section "Storage of Low-Precision Data"). */
QG_API size_t qg_canonical_bytes(int bits, int64_t count);

/* Bytes of the device layout for a [K,N] weight, or 0 if the shape is not tileable
 * (K % 128, N % 64) or the type is invalid.  The re-layout adds no padding: a tile of
 * BK x BN codes of b bits is BK*BN*b/8 bytes (the identity the paper states for its
 * int6 tile, Section "An Example of Tilus Program"), so the whole is K*N*bits/8. */
QG_API size_t qgemm_packed_bytes(qg_wtype t, int layout, int64_t K, int64_t N);

/* codes[count] (one code per byte, low `bits` bits) -> canonical stream:
 * element e occupies stream bits [e*bits, (e+1)*bits), stream bit j is bit
 * (j mod 8) of byte (j div 8).  `stream_out` must hold qg_canonical_bytes()
 * bytes; pad bits are written as zero.  QG_EINVAL on bad bits / null. */
QG_API int qg_pack_codes(const uint8_t* codes, int bits, int64_t count, uint8_t* stream_out, void* stream);

/* Canonical row-major [K,N] stream -> device layout.  `packed_out` must hold
 * qgemm_packed_bytes() bytes and must not alias the input.  QG_EINVAL on a
 * non-tileable shape, bad type or layout, null pointers. */
QG_API int repack(const void* canonical, qg_wtype t, int layout, int64_t K, int64_t N,
           void* packed_out, void* stream);

/* W_out[K,N] (row-major, `act` dtype) = rounded de-quantised weights.
 *   scales [K/group, N] row-major, dtype `scale_dtype` (QG_F16 or QG_BF16), or -- microscaling
 *          block scales, which the paper's closing section names as a finer-grained
 *          quantisation it could support -- QG_E8M0: one BYTE e per 32 rows and column, the
 *          scale is 2^(e - 127), e in 1 .. 254.  Block scales go with group == 32, no
 *          zero-points, the float types e2m1 and e4m3 (the 4- and 8-bit microscaling element
 *          types) and QG_LAYOUT_TILE128x64; anything else with QG_E8M0 is QG_EUNSUPPORTED.
 *          The hardware's scaled converts apply the scale, so a de-quantised pair of codes
 *          costs one instruction; qgemm runs such weights through the streaming and the tiled
 *          kernel of that layout like any other (only the de-quantise-first experiment path has
 *          no variant for them)
 *   zeros  [K/group, N] row-major uint8, or NULL for zero-point 0
 *   group  rows of W per scale, dividing K: 32, 64, 128 * 2^s, or K itself (= one scale per
 *          output column; 0 means the same).  128 * odd (other than K) is a valid group
 *          size this build has no kernel for: QG_EUNSUPPORTED.  Group size 32 exists in
 *          qdequant (both layouts) and in qgemm on QG_LAYOUT_TILE128x64; qgemm with group
 *          32 on QG_LAYOUT_TILE128x64_R32 is QG_EUNSUPPORTED.
 * QG_EINVAL on shape/group violations, QG_EUNSUPPORTED on an unsupported
 * float split or group size. */
QG_API int qdequant(const void* packed_W, const void* scales, const uint8_t* zeros, qg_wtype t,
             int layout, int act, int scale_dtype, int64_t group, int64_t K, int64_t N,
             void* W_out, void* stream);

/* C[M,N] (row-major, `act`) = A[M,K] (row-major, `act`) . dequant(W).
 * Arguments as for qdequant; M >= 1 is arbitrary, C is overwritten.
 * Path choice (by shape) is internal: M <= 64 streams the weights once through
 * a split-K kernel (1, 2 or 4 tiles of 16 rows per wavefront); larger M -- and
 * 33 <= M <= 64 on all but small problems -- use the LDS-staged tiled kernel, which also splits K (partial sums meet in a
 * workspace the library allocates on first use) when its 64- or
 * 128-row tiles would leave most CUs idle.  The tiled kernel needs M*K*2, the packed
 * weight and the scale array each below 2 GiB (QG_EUNSUPPORTED otherwise). */
QG_API int qgemm(const void* A, const void* packed_W, const void* scales, const uint8_t* zeros,
          qg_wtype t, int layout, int act, int scale_dtype, int64_t group,
          int64_t M, int64_t N, int64_t K, void* C, void* stream);

/* qgemm for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels,
 * same plan and therefore the same bits as qgemm, but the split-K partial sums and
 * arrival counters live in ONE fixed array in device memory that is part of the loaded
 * library (32 MiB + 64 KiB per GPU, held until the process ends); the call allocates
 * nothing, frees nothing and does not synchronise.
 *   - The first call on a device with valid shapes -- M = 0 will do, all pointers may then
 *     be NULL -- looks the array's address up on that device and keeps it (the HIP runtime
 *     loads this library's device code at that moment if none of it has been used yet,
 *     which is when the array comes to occupy device memory).  Make that call once before
 *     entering a region that must not touch the allocator, e.g. before a graph capture.
 *   - Every call on a GPU shares that GPU's array: calls that may overlap in time (on
 *     different streams, or from different threads onto streams that are not ordered
 *     with each other) race on it and give wrong sums.  Issue them on one stream, or
 *     order the streams, or use qgemm (one workspace per stream) for the overlapping ones.
 *   - Nothing needs to be cleared between calls: a call reads back only partial sums it
 *     wrote itself, and each arrival counter is returned to zero by the kernel that used it.
 *   - A request beyond the array (only a forced split factor, see qgemm_tuning.h, can
 *     make one) is refused with QG_EUNSUPPORTED and qg_last_error() says how much was
 *     asked for; nothing is enqueued.  Other errors as for qgemm. */
QG_API int qgemm_noalloc(const void* A, const void* packed_W, const void* scales, const uint8_t* zeros,
          qg_wtype t, int layout, int act, int scale_dtype, int64_t group,
          int64_t M, int64_t N, int64_t K, void* C, void* stream);

/* Matmul with int8 activations (Section "Arbitrary Data Type Support" names int8 as a supported
 * activation type and gives no formula; this is the library's reading, the standard W-k-bit /
 * A-8-bit form):
 *     C[m,n] = rne_out( a_scale[m] * sum_g s[g,n] * ( sum_{k in group g} A8[m,k] * (value(code[k,n]) - z[g,n]) ) )
 * The inner sum over the rows of one scale group is an exact integer (integer matrix
 * instruction, int32), the group's weight scale multiplies it and the groups are added in fp32,
 * the row's activation scale multiplies the total, one rounding to `out_dtype`.
 *   A8        [M, K] row-major int8, device, 16-byte aligned
 *   a_scale   [M] fp32, device, or NULL for 1
 *   packed_W  repack(..., QG_LAYOUT_TILE128x64_I8, ...) of a uintk or intk weight (floats: QG_EUNSUPPORTED)
 *   scales / zeros / scale_dtype / K, N as for qgemm; group 64, 128 * 2^s, K (or 0 = K);
 *   group 32 is QG_EUNSUPPORTED (the instruction sums 64 values of k)
 *   out_dtype QG_F16 or QG_BF16: dtype of C [M, N]
 * M >= 1 is arbitrary (rows are served in blocks of 64; there is no separate prefill kernel
 * yet).  Workspace, stream and error conventions as for qgemm. */
QG_API int qgemm_a8(const int8_t* A8, const float* a_scale, const void* packed_W, const void* scales,
             const uint8_t* zeros, qg_wtype t, int out_dtype, int scale_dtype, int64_t group,
             int64_t M, int64_t N, int64_t K, void* C, void* stream);

/* Codebook quantisation.  The paper's related-work section says a lookup instruction would
 * accommodate codebook schemes such as LCQ and gives no formula; this is the library's reading:
 *     w[k,n] = rne_act( codebook[code[k,n]] * s[k/g, n] )
 * one table of 2^bits levels per weight matrix, the group scale as in the affine form, no
 * zero-point (a table holds any offset), one rounding to the activation type.
 *   packed_W  repack(..., {QG_CODEBOOK, bits, 0, 0}, QG_LAYOUT_TILE128x64, ...) of the canonical
 *             stream of codes, bits in 1..8
 *   codebook  2^bits fp16 values (whatever `act` is), device, 2-byte aligned, read by every
 *             workgroup at kernel start
 *   scales / scale_dtype (QG_F16, or QG_BF16 with bf16 activations) / group / K, N / act as for
 *   qdequant and qgemm
 * The lookup is an LDS read from a table replicated over the 32 banks (up to 4 bits: one read
 * returns the two levels of a pair of codes; above: one read per code).  qgemm_codebook chooses
 * between the streaming and the tiled kernel as qgemm does (the experiment overrides of
 * qgemm_tuning.h apply); workspace, stream and error conventions as for qgemm.  One more choice
 * is automatic here: codes of more than 4 bits with M >= 1024 take the paper's prefill variant
 * (Section "End-to-End Performance": de-quantise the weight to 16 bits once, then a 16-bit
 * matmul), which is faster for them (their code-by-code lookup does not hide between the matrix
 * instructions).  It uses a library-owned buffer of K*N*2 bytes per (device, stream), allocated
 * on first use and replaced after a stream synchronisation when a larger weight arrives -- so
 * such a call may allocate and is not for graph capture; forcing the tiled kernel (knob 0 = 2)
 * avoids it, and so does the library itself when K*N*2 reaches 2 GiB or the allocation fails.  QG_EINVAL on a null table, bits outside 1..8 and
 * on the shape / group violations of qgemm. */
QG_API int qdequant_codebook(const void* packed_W, const void* codebook, const void* scales, int bits,
                      int act, int scale_dtype, int64_t group, int64_t K, int64_t N, void* W_out, void* stream);
QG_API int qgemm_codebook(const void* A, const void* packed_W, const void* codebook, const void* scales, int bits,
                   int act, int scale_dtype, int64_t group, int64_t M, int64_t N, int64_t K, void* C, void* stream);

/* What qgemm would launch for a shape: host arithmetic only, no GPU call, usable without
 * a device.  Arguments as for qgemm (M >= 1).  plan (host, 5 ints) receives
 *   [0] path: 1 = streaming kernel, 2 = tiled kernel, 3 = streaming kernel over blocks of 64 rows,
 *       4 = de-quantise first, then the tiled kernel on 16-bit weights (forced only),
 *       5 = matrix-vector kernel on the vector ALU, M <= 4 (forced only)
 *   [1] wavefront arrangement of the streaming kernel (the values of knob 3), 0 on path 2; on path 5
 *       the wavefronts per strip
 *   [2] row-tile height of the tiled kernel: 64 or 128, or 0 = whole rounds of 256-row
 *       tiles, then 128 or 256 rows for the rest (paths 2 and 4); 0 on paths 1 and 3
 *   [3] K-slabs (split-K factor; 1 = none)   [4] K-chunks of 128 per slab
 * The experiment overrides of qgemm_tuning.h apply as in qgemm.  Returns the status qgemm's
 * argument checks would return.  With t.kind == QG_CODEBOOK: what qgemm_codebook would launch. */
QG_API int qg_plan(qg_wtype t, int layout, int act, int scale_dtype, int64_t group,
            int64_t M, int64_t N, int64_t K, int plan[5]);

/* Measurement aids -- not part of the method (no passage of the paper defines
 * them): the two empirical ceilings bench.py quotes beside the published peaks.
 * Both enqueue one kernel on `stream` and return; the caller times them.
 * qg_probe_stream_read: reads `bytes` (>= 16; whole 16-byte units are read) from
 *   device buffer `buf` (16-byte aligned) once with 16-byte loads and discards
 *   them.  `sink`: >= 1 KiB of device memory, practically never written.
 * qg_probe_mfma: 256 * waves_per_simd workgroups of 4 wavefronts each run `iters`
 *   x 8 register-resident 32x32x16 matrix instructions (bf16 != 0: bf16 operands,
 *   else fp16) on constant (all ones) or pseudo-random operand data;
 *   *flops_out (host, may be NULL) receives the flop count of the launch.
 * QG_EINVAL on null / misaligned pointers or counts out of range. */
QG_API int qg_probe_stream_read(const void* buf, size_t bytes, void* sink, void* stream);
QG_API int qg_probe_mfma(int bf16, int random_data, int iters, int waves_per_simd, void* sink,
                         double* flops_out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* QGEMM_H_ */
