/*
 * ams.h -- C ABI of the MI355X (gfx950) AMS-Quant weight-only quantized Linear.
 *
 * The library implements the decode-time Linear of AMS-Quant (arxiv 2510.16045):
 * weights are stored in a non-integer bit-width floating-point format in which a
 * group of k consecutive input-channel weights shares its last mantissa bit
 * (Sec. 3.1), are restored to fp16 on the fly by bit operations (Sec. 3.2) and
 * multiplied by a skinny fp16 activation matrix (Sec. 3.3, Sec. 4.2).
 *
 * Conventions for every entry point
 *   - Return value: 0 (AMS_OK) or a negative AMS_ERR_* code; nothing throws or aborts
 *     (the host quantizer reports AMS_ERR_NOMEM when it cannot get its row buffers).
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device
 *     memory of the current device.  The caller owns every buffer.
 *   - Device entry points only enqueue work on `stream` (a hipStream_t passed as
 *     void*; NULL = the default stream); they never synchronize and never allocate.
 *   - fp16 values travel as uint16_t bit patterns (IEEE binary16).
 *   - W is [N, K]: N output channels (rows), K input channels; one fp16 scale per row.
 *   - A "code" is one weight's mini-float [S | E(2) | M(m)] with exponent bias 1,
 *     subnormals, and no inf/NaN (Sec. 2.2, Table 1): 6 bits for e2m3, 5 for e2m2, 4 for e2m1.
 */
#ifndef AMS_H_
#define AMS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Formats.  The two the paper builds kernels for (abstract; Sec. 3.2, Sec. 3.3 item 1),
 * the other shared-bit formats it evaluates (Sec. 4.1, FP(x-1).y with y = 1/k), and the
 * plain mini-floats it compares with (group size 1: no sharing, the search is a no-op).
 */
enum {
  AMS_FMT_FP533_E2M3 = 0, /* e2m3 codes, groups of 3 along K share the mantissa LSB: 16/3 bits per weight */
  AMS_FMT_FP425_E2M2 = 1, /* e2m2 codes, groups of 4 share it: 4.25 bits per weight */
  AMS_FMT_FP45_E2M2 = 2,  /* e2m2 codes, groups of 2 share it: 4.5 bits per weight */
  AMS_FMT_FP433_E2M2 = 3, /* e2m2 codes, groups of 3 share it: 13/3 bits per weight */
  AMS_FMT_FP6_E2M3 = 4,   /* plain e2m3: 6 bits per weight */
  AMS_FMT_FP5_E2M2 = 5,   /* plain e2m2: 5 bits per weight */
  AMS_FMT_FP4_E2M1 = 6    /* plain e2m1: 4 bits per weight */
};

enum {
  AMS_OK = 0,
  AMS_ERR_FORMAT = -1,    /* unknown fmt */
  AMS_ERR_SHAPE = -2,     /* N, K, M or a leading dimension out of range */
  AMS_ERR_NULL = -3,      /* a required pointer is NULL */
  AMS_ERR_ALIGN = -4,     /* a device pointer is not 16-byte aligned */
  AMS_ERR_NONFINITE = -5, /* a weight is inf or NaN */
  AMS_ERR_LAUNCH = -6,    /* the HIP runtime refused a launch (see hipGetLastError) */
  AMS_ERR_DEVICE = -7,    /* the current device is not a gfx950 GPU (returned by every device entry point) */
  AMS_ERR_SCRATCH = -8,   /* ams_linear_static_ws: the shape is beyond what the library's static scratch holds */
  AMS_ERR_NOMEM = -9      /* a host entry point could not get the memory for its row buffers */
};

#define AMS_MAX_M 32 /* largest activation batch of ams_linear / ams_fp16_linear (Table 3: batch 1..32) */

/* Version of the library and of its packed layout: 100 * major + minor.  A packed buffer is only valid
 * for the major version that wrote it (200: FP4.25 records carry their shared bits inside the lane chunks). */
int ams_version(void);
const char* ams_strerror(int code);

/*
 * Optional one-time set-up for the current device: checks that it is a gfx950 (else
 * AMS_ERR_DEVICE) and raises the dynamic-LDS limit of every Linear kernel (they use up to
 * 160 KiB).  Every device entry point does the same for itself on its first call, so this
 * is only REQUIRED before the first call of an entry point happens inside a HIP stream
 * capture (function attributes should not be changed while capturing).  Allocates nothing,
 * enqueues nothing; may be called any number of times, once per device that is used.
 */
int ams_init(void);

/* Group size k of the format (Sec. 3.1: the k weights that share their last mantissa bit; 1 to 4, 1 = plain
 * mini-float) and bits of one code (Sec. 2.2: sign + 2 exponent bits + mantissa; 4 to 6); 0 for an unknown fmt. */
int ams_group_size(int fmt);
int ams_code_bits(int fmt);

/*
 * Size in bytes of the packed weight buffer in this library's gfx950 layout
 * (what ams_pack writes and ams_dequant / ams_linear read): the result of the
 * "ahead-of-time weight packing" of Sec. 3.3 stage 1, arranged for 64-wide wavefronts.  The layout is opaque:
 * records of 16 rows x 96 weights (FP5.33, FP4.33, FP6) or 16 rows x 128 weights
 * (FP4.25, FP4.5, FP5, FP4), stored K-major in units of 1, 2 or 4 records (formats that
 * keep last mantissa bits beside their records: FP4.25 and FP4.33 four, FP4.5 and FP6 two),
 * so N is padded to a multiple of 16 and K to a multiple of 96 / 128 times that unit;
 * padding holds zero codes.  Without padding the size is exactly N * K * bits-per-weight / 8.
 */
int ams_packed_bytes(int fmt, int64_t N, int64_t K, size_t* bytes);

/*
 * Size in bytes of the paper's own packing: one uint16 per 3 weights for FP5.33
 * (Sec. 3.3 item 1), 17 uint16 per 64 weights for FP4.25 (Sec. 3.2); for the other
 * formats the densest whole-byte packing per row (9 bytes per 16 weights, 13 per 24,
 * 3 per 4, 5 per 8, 1 per 2).  This is the "algorithmic" byte count used when bandwidth is
 * reported.
 */
int ams_canonical_bytes(int fmt, int64_t N, int64_t K, size_t* bytes);

/*
 * Offline quantizer + packer (Sec. 3.1; Sec. 3.3 stage 1).  All pointers are host.
 *   W_fp16      [N, ldw] fp16 weights, row n at W_fp16 + n*ldw, ldw >= K
 *   packed      out, ams_packed_bytes() bytes
 *   scales_fp16 out, [N] fp16: s_n = fp16(max_k|W[n,k]| / Fmax) (Eq. 1), 1.0 for a row
 *               whose scale would be zero
 *   codes       out or NULL, [N, K] one byte per weight: the final code, whose last
 *               bit is the group's shared bit
 * Per row: RTN of W/s to the nearest code (ties to the even code, saturating);
 * then per group of k consecutive weights along K both values of the shared last
 * bit are tried and the one with the smaller fp64 sum of squared errors against
 * the original weights is kept (a tie keeps 0; a short last group counts only its
 * real members).  Deterministic.  Errors: FORMAT, SHAPE, NULL, NONFINITE.
 */
int ams_pack(int fmt, const uint16_t* W_fp16, int64_t N, int64_t K, int64_t ldw, void* packed,
             uint16_t* scales_fp16, uint8_t* codes);

/*
 * ams_pack with a choice of the search (everything else as ams_pack):
 *   AMS_SEARCH_SET_BIT  Sec. 3.1 as written: each member keeps the upper bits of its RTN
 *                       code and only its last bit is set to the tried value.
 *   AMS_SEARCH_REROUND  a variant that is not in the paper: for each tried value every
 *                       member is re-rounded to the nearest code that ends in it (ties to
 *                       the code whose upper part is even, saturating).  Never a larger
 *                       error; the packed layout and the kernels are the same.
 * Errors: as ams_pack; SHAPE for an unknown search.
 */
enum { AMS_SEARCH_SET_BIT = 0, AMS_SEARCH_REROUND = 1 };
int ams_pack_ex(int fmt, int search, const uint16_t* W_fp16, int64_t N, int64_t K, int64_t ldw, void* packed,
                uint16_t* scales_fp16, uint8_t* codes);

/*
 * ams_pack_ex with ONE scale for the whole matrix (per-tensor granularity, Sec. 5):
 * s = fp16(max over all of |W| / Fmax).  `scales_fp16` still receives N values (all the
 * same), so the result is used with ams_dequant / ams_linear unchanged.
 */
int ams_pack_per_tensor(int fmt, int search, const uint16_t* W_fp16, int64_t N, int64_t K, int64_t ldw, void* packed,
                        uint16_t* scales_fp16, uint8_t* codes);

/*
 * One scale per run of `scale_group` consecutive input channels of a row instead of
 * one per row (Sec. 5: the method "can be applied with any granularity ... per-group";
 * read as Eq. 1, RTN and the search applied to every run by itself).  scale_group must
 * be the record size of the format (96 for FP5.33 / FP4.33 / FP6, 128 for the others)
 * times a power of two; the last run of a row may be shorter.
 *   ams_group_scales_count  number of fp16 scales: ceil(K / scale_group) per row, rows
 *                           padded to a multiple of 16
 *   ams_pack_grouped        as ams_pack_ex; `scales_fp16` receives that many values in
 *                           the order the kernels read them: [strip of 16 rows][run][row
 *                           inside the strip] (1.0 for padding rows)
 *   ams_dequant_grouped / ams_linear_grouped
 *                           as ams_dequant / ams_linear with such a scale buffer (device)
 * Errors: as their per-row counterparts; SHAPE for a scale_group that is not allowed.
 */
int ams_group_scales_count(int fmt, int64_t N, int64_t K, int64_t scale_group, size_t* count);
int ams_pack_grouped(int fmt, int search, int64_t scale_group, const uint16_t* W_fp16, int64_t N, int64_t K, int64_t ldw,
                     void* packed, uint16_t* scales_fp16, uint8_t* codes);
int ams_dequant_grouped(int fmt, const void* W_packed, const uint16_t* scales, int64_t scale_group, uint16_t* W_out_fp16,
                        int64_t N, int64_t K, int scaled, void* stream);
int ams_linear_grouped(const void* W_packed, const uint16_t* scales, int64_t scale_group, const uint16_t* X, uint16_t* Y,
                       int M, int64_t N, int64_t K, int fmt, void* stream);

/*
 * The packing step alone (Sec. 3.3 stage 1; Sec. 3.2: remainders and shared bits stored in
 * standard words): pack codes that were produced elsewhere (e.g. read from the paper's layout) into
 * the gfx950 layout.  codes [N, K] as written by ams_pack; within a group all last
 * bits must agree (else AMS_ERR_SHAPE).  Host pointers.
 */
int ams_pack_codes(int fmt, const uint8_t* codes, int64_t N, int64_t K, void* packed);

/* Inverse of the layout step (the stitching of remainder and shared bit of Sec. 3.2 / Sec. 3.3 stage 2, done on
 * the host): packed (host) -> codes [N, K] (host).  Debug / tests. */
int ams_unpack_host(int fmt, const void* packed, int64_t N, int64_t K, uint8_t* codes);

/*
 * Bit-level restoration (Sec. 3.2, Sec. 3.3 stages 2-3) of a whole packed matrix.
 *   W_packed device, 16-byte aligned;  scales device [N] fp16 (may be NULL if !scaled)
 *   W_out    device [N, K] fp16 row-major, logical k order
 *   scaled=0: the code's own value (exact);  scaled=1: fp16_RNE(value * s_n) (Eq. 2)
 */
int ams_dequant(int fmt, const void* W_packed, const uint16_t* scales, uint16_t* W_out, int64_t N, int64_t K,
                int scaled, void* stream);

/*
 * The quantized Linear (Sec. 3.3; Sec. 4.2 "GEMV-like operations"):
 *   Y[m, n] = fp16( sum_k value(code[n,k]) * s_n * X[m, k] ),  fp32 accumulation.
 *   W_packed device (ams_pack layout), scales device [N] fp16,
 *   X device [M, K] fp16 row-major, Y device [M, N] fp16 row-major, 1 <= M <= AMS_MAX_M.
 * All four pointers must be 16-byte aligned.  X and Y must not alias.
 * Errors: FORMAT, NULL, SHAPE (M, N or K out of range), ALIGN, DEVICE, LAUNCH.
 * The first call of a kernel on a device raises that kernel's LDS limit: if it can happen inside a
 * stream capture, call ams_init() before.
 */
int ams_linear(const void* W_packed, const uint16_t* scales, const uint16_t* X, uint16_t* Y, int M, int64_t N,
               int64_t K, int fmt, void* stream);

/*
 * The unquantized fp16 Linear Y = X W^T (the W16A16 baseline of Sec. 4.2) written for
 * the same GPU, used as the denominator of the reported speed-ups.
 *   W device [N, K] fp16 row-major (K a multiple of 8), X [M, K], Y [M, N], 1 <= M <= AMS_MAX_M.
 */
int ams_fp16_linear(const uint16_t* W, const uint16_t* X, uint16_t* Y, int M, int64_t N, int64_t K, void* stream);

/*
 * ams_linear / ams_fp16_linear with a workspace (device, 16-byte aligned, at least
 * ams_linear_workspace_bytes() bytes, zero-filled once before its first use; the calls
 * leave it ready for the next one, of any shape).  With a workspace the kernel may cut K in slices
 * handled by different workgroups, which exchange fp32 partial tiles through it: shapes
 * with few output channels (e.g. the MLP down-projections of Sec. 4.2's table, N = 2560
 * to 5120) then use all compute units, and large batches stage less of X per workgroup.
 * Results differ from ams_linear only in the order of the fp32 sums (deterministic for a
 * given shape).  A workspace that is NULL or too small gives the behaviour of ams_linear.
 * Calls that overlap in time must not share a workspace.
 *   ams_linear_workspace_bytes  fmt = AMS_FMT_*, or -1 for the fp16 baseline; may return 0
 */
int ams_linear_workspace_bytes(int fmt, int M, int64_t N, int64_t K, size_t* bytes);
/* Which kernel and launch shape ams_linear (with_workspace = 0) or ams_linear_ws (1) would use for
 * this problem (fmt = -1: the fp16 baseline), as a short text for logs and tests: "column ..." (the
 * packed formats), "gemv ..." (the baseline at batches up to 4 whose activations fit in LDS), "sweep ..."
 * or "stream ..." (the baseline otherwise), followed by key=value pairs (workgroups, strips per
 * workgroup, slices of K, wavefronts, wavefronts per strip or strips per wavefront, phases of K, LDS
 * bytes, records ahead).  Host only, launches nothing. */
int ams_linear_plan(int fmt, int M, int64_t N, int64_t K, int with_workspace, char* text, size_t text_len);
int ams_linear_ws(const void* W_packed, const uint16_t* scales, const uint16_t* X, uint16_t* Y, int M, int64_t N,
                  int64_t K, int fmt, void* workspace, size_t workspace_bytes, void* stream);
int ams_fp16_linear_ws(const uint16_t* W, const uint16_t* X, uint16_t* Y, int M, int64_t N, int64_t K, void* workspace,
                       size_t workspace_bytes, void* stream);

/*
 * ams_linear_ws for callers that cannot allocate a workspace (code under HIP graph capture
 * that may not call hipMalloc, tight serving loops, harnesses that forbid allocation): the
 * split of K exchanges its partial tiles and arrival counters through a static device array
 * inside the library (64 KiB + 8 MiB per GPU, held until the process ends) instead of a
 * caller's buffer.  Same arguments, same kernels and bit-for-bit the same results as
 * ams_linear_ws with a large enough zero-filled workspace.  Allocates nothing.
 *   Limit: the workspace this shape's split needs (what ams_linear_workspace_bytes reports)
 *   must fit the array, i.e. be at most 64 KiB + 8 MiB: true for every shape with up to 16384
 *   output channels (8192 for M > 16) and for most larger ones, which are not split at all;
 *   beyond that AMS_ERR_SCRATCH, never a silently different plan (use ams_linear or ams_linear_ws).
 *   Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU
 *   (two streams, two threads) race and must be serialised by the caller.  Each call leaves
 *   the counters at zero for the next one; the array starts zero-filled when the library is loaded.
 *   If the first call on a device happens inside a stream capture, call ams_init() before the capture.
 * Errors: as ams_linear, plus SCRATCH.
 */
int ams_linear_static_ws(const void* W_packed, const uint16_t* scales, const uint16_t* X, uint16_t* Y, int M, int64_t N,
                         int64_t K, int fmt, void* stream);

/*
 * Measurement aid, not part of the method: a bare streaming read of the first
 * floor(bytes / 1024) KiB of `buf` (device, 16-byte aligned), front to back, 1 KiB per
 * wavefront load, two loads in flight per wavefront, 16 wavefronts on each of 256
 * workgroups: the window of memory that the Linear kernel's wavefronts read between them
 * moves through a packed matrix in the same way.  Nothing is computed, nothing stored.  Its
 * time is the read ceiling of this GPU at that size, the second denominator (beside the
 * 8 TB/s HBM peak) for the "saturate the memory subsystem" goal of Sec. 3.3; bytes < 1024
 * gives an empty launch of the same shape (the launch floor).  `sink` is a device
 * word the kernel may write (it practically never does) or NULL.
 */
int ams_read_probe(const void* buf, size_t bytes, uint32_t* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* AMS_H_ */
