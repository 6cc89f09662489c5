// HIP kernels (gfx950 / CDNA4) of the AMS-Quant weight-only quantized Linear:
// bit-level restoration of the packed weights (Sec. 3.2, Sec. 3.3 stages 2-3) fused
// with the skinny fp16 matmul of the decode stage (Sec. 4.2), and the fp16 baseline.
//
// One wavefront owns a strip of 16 output channels over a contiguous run of records;
// every lane loads its 16-byte chunk of a record with one dwordx4 (the whole record is
// one contiguous 1 KiB access), restores the fp16 pairs in registers and feeds them as
// the A operand of v_mfma_f32_16x16x32_f16.  The activations are staged once per
// workgroup in LDS in the operand order the restoration produces.  The wavefronts of
// a workgroup split K among themselves and combine their partial tiles through LDS,
// so no global workspace or atomics are needed.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "../../include/ams.h"
#include "ams_layout.h"

namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef unsigned short us2 __attribute__((ext_vector_type(2)));

constexpr int FMT_FP533 = AMS_FMT_FP533_E2M3;
constexpr int FMT_FP425 = AMS_FMT_FP425_E2M2;
constexpr int FMT_FP16 = 2;  // internal: unquantized row-major fp16 weights (baseline)

constexpr float kTwo14 = 16384.0f;  // restored patterns are value * 2^-14

__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (a & mask) | (b & ~mask); }

__device__ __forceinline__ uint32_t pk_mul_u16(uint32_t a, uint32_t c) {
  us2 x = __builtin_bit_cast(us2, a), y = __builtin_bit_cast(us2, c);
  return __builtin_bit_cast(uint32_t, (us2)(x * y));
}

// FP4.25 (Sec. 3.2): one 32-bit word = two groups of four 4-bit remainders, plus their
// two shared bits already placed at bits 8 and 24 of `sh`.  Produces the four fp16
// pairs (A_i low, B_i high) as bit patterns of value * 2^-14:
// sign -> bit 15, e1 e0 m1 -> bits 11..9, shared m0 -> bit 8.
__device__ __forceinline__ void restore_fp425(uint32_t s, uint32_t sh, uint32_t out[4]) {
  constexpr uint32_t M = 0x8E008E00u;
  out[0] = bfi(M, s, sh);
  out[1] = bfi(M, s << 3, sh);
  // members 2 and 3: sign and magnitude need different shifts; a packed 16-bit
  // multiply by (2^a + 2^b) makes both shifted copies at once
  out[2] = bfi(M, pk_mul_u16(s & 0x40384038u, 0x00420042u), sh);
  out[3] = bfi(M, pk_mul_u16(s & 0x20072007u, 0x02040204u), sh);
}

// Shared bits of a lane's FP4.25 record byte: bit d = group A of word d, bit 4+d = group B.
__device__ __forceinline__ uint32_t spread_shared_fp425(uint32_t byte) { return byte | (byte << 12); }
__device__ __forceinline__ uint32_t shared_of_word_fp425(uint32_t spread, int d) {
  return (spread << (8 - d)) & 0x01000100u;
}

// FP5.33 (Sec. 3.3 item 1): one 32-bit word = two half-words, each a whole group (three
// 5-bit remainders + the shared bit).  Produces three fp16 pairs (A_i low, B_i high):
// sign -> bit 15, e1 e0 m2 m1 -> bits 11..8, shared m0 -> bit 7.
__device__ __forceinline__ void restore_fp533(uint32_t s, uint32_t out[3]) {
  constexpr uint32_t M = 0x8F008F00u;
  const uint32_t sh = (s >> 5) & 0x00800080u;
  out[0] = bfi(M, s, sh);
  out[1] = bfi(0x80008000u, s << 1, ((s << 4) & 0x0F000F00u) | sh);
  out[2] = bfi(M, pk_mul_u16(s & 0x200F200Fu, 0x01040104u), sh);
}

template <int FMT>
struct Fmt;
template <>
struct Fmt<FMT_FP533> {
  static constexpr int REC_K = 96, REC_BYTES = 1024, N_MFMA = 3;
};
template <>
struct Fmt<FMT_FP425> {
  static constexpr int REC_K = 128, REC_BYTES = 1088, N_MFMA = 4;
};
template <>
struct Fmt<FMT_FP16> {
  static constexpr int REC_K = 128, REC_BYTES = 0, N_MFMA = 4;
};

// What one lane holds of one record.
template <int FMT>
struct LaneRec {
  u4 w;
};
template <>
struct LaneRec<FMT_FP425> {
  u4 w;
  uint32_t t;
};
template <>
struct LaneRec<FMT_FP16> {
  u4 w[4];
};

struct LinearArgs {
  const uint8_t* W;        // packed records, or row-major fp16 for the baseline
  const uint16_t* scales;  // [N] fp16, unused by the baseline
  const uint16_t* X;       // [M, K] fp16
  uint16_t* Y;             // [M, N] fp16
  int M, N, K;
  int n_rec;          // records per strip
  int recs_per_wave;  // L: records a wave takes per phase
  int x_stride;       // halfs between activation rows in LDS
};

template <int FMT>
__device__ __forceinline__ void load_rec(LaneRec<FMT>& r, const LinearArgs& a, int strip, int rec, int lane, bool valid) {
  if constexpr (FMT == FMT_FP16) {
    const int row = strip * 16 + (lane & 15);
    const int kq = lane >> 4;
#pragma unroll
    for (int d = 0; d < 4; d++) {
      const int k = rec * 128 + 32 * d + 8 * kq;
      const bool ok = valid && row < a.N && k < a.K;  // K is a multiple of 8
      const u4* p = (const u4*)(a.W + ((size_t)row * a.K + k) * 2);
      r.w[d] = ok ? __builtin_nontemporal_load(p) : u4{0, 0, 0, 0};
    }
  } else {
    const uint8_t* base = a.W + ((size_t)strip * a.n_rec + rec) * Fmt<FMT>::REC_BYTES;
    r.w = valid ? __builtin_nontemporal_load((const u4*)(base + lane * 16)) : u4{0, 0, 0, 0};
    if constexpr (FMT == FMT_FP425) r.t = valid ? (uint32_t)__builtin_nontemporal_load(base + 1024 + lane) : 0u;
  }
}

// Multiply one record (16 rows x REC_K) into the accumulators.  xrow points at this
// lane's activation row in LDS at the first operand slot of this record's K-quarter.
template <int FMT, int MT>
__device__ __forceinline__ void mac_rec(const LaneRec<FMT>& r, const _Float16* xrow, bool has_x0, bool has_x1, int x_hi_off,
                                        f4 acc[MT]) {
  h8 a[Fmt<FMT>::N_MFMA];
  if constexpr (FMT == FMT_FP425) {
    const uint32_t spread = spread_shared_fp425(r.t);
#pragma unroll
    for (int d = 0; d < 4; d++) {
      uint32_t o[4];
      restore_fp425(r.w[d], shared_of_word_fp425(spread, d), o);
      a[d] = __builtin_bit_cast(h8, u4{o[0], o[1], o[2], o[3]});
    }
  } else if constexpr (FMT == FMT_FP533) {
    uint32_t o[12];
#pragma unroll
    for (int d = 0; d < 4; d++) restore_fp533(r.w[d], &o[3 * d]);
#pragma unroll
    for (int u = 0; u < 3; u++) a[u] = __builtin_bit_cast(h8, u4{o[4 * u], o[4 * u + 1], o[4 * u + 2], o[4 * u + 3]});
  } else {
#pragma unroll
    for (int d = 0; d < 4; d++) a[d] = __builtin_bit_cast(h8, r.w[d]);
  }
  const h8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
  for (int u = 0; u < Fmt<FMT>::N_MFMA; u++) {
    // FP16 records interleave the K-quarters per MFMA (32 consecutive k each)
    const int off = FMT == FMT_FP16 ? 32 * u : 8 * u;
    h8 b0 = has_x0 ? *(const h8*)(xrow + off) : zero;
    acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[u], b0, acc[0], 0, 0, 0);
    if constexpr (MT == 2) {
      h8 b1 = has_x1 ? *(const h8*)(xrow + x_hi_off + off) : zero;
      acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[u], b1, acc[1], 0, 0, 0);
    }
  }
}

// Operand slot of activation k (relative to its record) in LDS.
template <int FMT>
__device__ __forceinline__ int x_slot(int kk) {
  if constexpr (FMT == FMT_FP425) {
    return (kk & ~7) + 2 * (kk & 3) + ((kk >> 2) & 1);
  } else if constexpr (FMT == FMT_FP533) {
    const int q = kk / 6, r = kk - 6 * q;
    const int h = r >= 3 ? 1 : 0;
    return 6 * q + 2 * (r - 3 * h) + h;
  } else {
    return kk;
  }
}

// Y[m, n] = fp16( s_n * sum_k value(code[n,k]) * X[m,k] ), one workgroup per strip of 16 rows.
// blockDim.x = 64 * S wavefronts; phase p covers records [p*S*L, (p+1)*S*L), wave w the
// L records starting at p*S*L + w*L.
template <int FMT, int MT, int LMAX>
__global__ void __launch_bounds__(1024) linear_kernel(LinearArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  _Float16* xs = (_Float16*)smem;
  constexpr int REC_K = Fmt<FMT>::REC_K;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int S = blockDim.x >> 6;
  const int strip = blockIdx.x;
  const int L = a.recs_per_wave;
  const int per_phase = S * L;
  const int m_lo = lane & 15, kq = lane >> 4;
  const bool has_x0 = m_lo < a.M, has_x1 = m_lo + 16 < a.M;

  f4 acc[MT];
#pragma unroll
  for (int i = 0; i < MT; i++) acc[i] = f4{0, 0, 0, 0};

  for (int rec0 = 0; rec0 < a.n_rec; rec0 += per_phase) {
    const int chunk_recs = min(per_phase, a.n_rec - rec0);
    // 1. issue this wave's weight loads for the phase
    LaneRec<FMT> recs[LMAX];
#pragma unroll
    for (int q = 0; q < LMAX; q++) {
      const int rl = wave * L + q;
      load_rec<FMT>(recs[q], a, strip, rec0 + rl, lane, q < L && rl < chunk_recs);
    }
    // 2. stage the activations of the phase in operand order (zero beyond K)
    if (rec0 > 0) __syncthreads();
    const int chunk_k = chunk_recs * REC_K;
    for (int idx = tid; idx < a.M * chunk_k; idx += blockDim.x) {
      const int m = idx / chunk_k, kk = idx - m * chunk_k;
      const int k = rec0 * REC_K + kk;
      const uint16_t v = k < a.K ? a.X[(size_t)m * a.K + k] : (uint16_t)0;
      const int rl = kk / REC_K, kr = kk - rl * REC_K;
      ((uint16_t*)xs)[m * a.x_stride + rl * REC_K + x_slot<FMT>(kr)] = v;
    }
    __syncthreads();
    // 3. restore + multiply
#pragma unroll
    for (int q = 0; q < LMAX; q++) {
      const int rl = wave * L + q;
      if (q < L && rl < chunk_recs) {
        const int lane_off = FMT == FMT_FP16 ? 8 * kq : (REC_K / 4) * kq;
        const _Float16* xrow = xs + m_lo * a.x_stride + rl * REC_K + lane_off;
        mac_rec<FMT, MT>(recs[q], xrow, has_x0, has_x1, 16 * a.x_stride, acc);
      }
    }
  }

  // cross-wave reduction of the 16 x 16 tiles, then scale, convert, store
  __syncthreads();
  f4* red = (f4*)smem;
#pragma unroll
  for (int i = 0; i < MT; i++) red[(wave * MT + i) * 64 + lane] = acc[i];
  __syncthreads();
  if (tid < 64 * MT) {
    const int mt = tid >> 6;
    f4 sum = {0, 0, 0, 0};
    for (int w = 0; w < S; w++) sum += red[(w * MT + mt) * 64 + lane];
    const int m = m_lo + 16 * mt;
    if (m < a.M) {
#pragma unroll
      for (int r = 0; r < 4; r++) {
        const int n = strip * 16 + 4 * kq + r;  // C[i][j]: lane = j + 16*(i/4), register i%4
        if (n < a.N) {
          float v = sum[r];
          if constexpr (FMT != FMT_FP16)
            v *= (float)__builtin_bit_cast(_Float16, a.scales[n]) * kTwo14;
          a.Y[(size_t)m * a.N + n] = __builtin_bit_cast(uint16_t, (_Float16)v);
        }
      }
    }
  }
}

// Restore a whole packed matrix to row-major fp16: one wavefront per record.
template <int FMT>
__global__ void __launch_bounds__(256) dequant_kernel(const uint8_t* W, const uint16_t* scales, uint16_t* out, int N, int K,
                                                      int n_rec, int64_t total_recs, int scaled) {
  const int lane = threadIdx.x & 63;
  const int64_t rec_id = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (rec_id >= total_recs) return;
  const int strip = (int)(rec_id / n_rec), rec = (int)(rec_id - (int64_t)strip * n_rec);
  const uint8_t* base = W + (size_t)rec_id * Fmt<FMT>::REC_BYTES;
  const u4 w = *(const u4*)(base + lane * 16);
  const int n = strip * 16 + (lane & 15);
  if (n >= N) return;
  float mul = kTwo14;
  if (scaled) mul *= (float)__builtin_bit_cast(_Float16, scales[n]);
  const int kbase = rec * Fmt<FMT>::REC_K + (lane >> 4) * (Fmt<FMT>::REC_K / 4);
  auto put = [&](int k, uint32_t bits16) {
    if (k < K) {
      // magnitude and sign apart: the exact product is rounded once, and a negative
      // zero code keeps its sign (a fused multiply-add with +0 would drop it)
      const float v = (float)__builtin_bit_cast(_Float16, (uint16_t)(bits16 & 0x7FFF)) * mul;
      out[(size_t)n * K + k] = (uint16_t)(__builtin_bit_cast(uint16_t, (_Float16)v) | (bits16 & 0x8000));
    }
  };
  if constexpr (FMT == FMT_FP425) {
    const uint32_t spread = spread_shared_fp425(base[1024 + lane]);
#pragma unroll
    for (int d = 0; d < 4; d++) {
      uint32_t o[4];
      restore_fp425(w[d], shared_of_word_fp425(spread, d), o);
#pragma unroll
      for (int i = 0; i < 4; i++) {
        put(kbase + 8 * d + i, o[i] & 0xFFFF);
        put(kbase + 8 * d + 4 + i, o[i] >> 16);
      }
    }
  } else {
#pragma unroll
    for (int d = 0; d < 4; d++) {
      uint32_t o[3];
      restore_fp533(w[d], o);
#pragma unroll
      for (int i = 0; i < 3; i++) {
        put(kbase + 6 * d + i, o[i] & 0xFFFF);
        put(kbase + 6 * d + 3 + i, o[i] >> 16);
      }
    }
  }
}

// ---- host-side launch logic -------------------------------------------------
constexpr int kXLdsBudget = 64 * 1024;  // bytes of LDS for staged activations per workgroup

struct Plan {
  int S, L, lmax, x_stride;
  size_t lds;
};

// Choose wavefronts per workgroup (S) and records per wave per phase (L).
Plan make_plan(int M, int64_t n_strips, int n_rec, int rec_k, int lmax_hi, int lmax_lo) {
  Plan p;
  int64_t want = (4096 + n_strips - 1) / n_strips;  // aim at >= 4096 wavefronts in the grid
  int S = (int)std::min<int64_t>(16, std::max<int64_t>(1, want));
  // keep at least ~4 records per wave when the grid is already large
  while (S > 1 && (n_rec + S - 1) / S < 4 && n_strips * (S / 2) >= 4096) S /= 2;
  S = std::min(S, n_rec);
  int L;
  for (;;) {
    const int per_wave = (n_rec + S - 1) / S;
    const int fit = kXLdsBudget / (M * S * rec_k * 2);
    L = std::min(std::min(per_wave, lmax_hi), fit);
    if (L >= 1 || S == 1) break;
    S = std::max(1, S / 2);
  }
  if (L < 1) L = 1;
  p.S = S;
  p.L = L;
  p.lmax = L <= lmax_lo ? lmax_lo : lmax_hi;
  p.x_stride = S * L * rec_k + 8;  // +8 halfs: rows 16 bytes apart modulo the bank span
  const size_t x_bytes = (size_t)M * p.x_stride * 2;
  const size_t red_bytes = (size_t)S * (M > 16 ? 2 : 1) * 64 * 16;
  p.lds = std::max(x_bytes, red_bytes);
  return p;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

template <int FMT, int MT, int LMAX>
int launch_linear(const LinearArgs& a, const Plan& p, int64_t n_strips, hipStream_t st) {
  auto kern = linear_kernel<FMT, MT, LMAX>;
  if (p.lds > 64 * 1024) {
    if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds) != hipSuccess)
      return AMS_ERR_LAUNCH;
  }
  hipLaunchKernelGGL(kern, dim3((unsigned)n_strips), dim3(64 * p.S), p.lds, st, a);
  return hipGetLastError() == hipSuccess ? AMS_OK : AMS_ERR_LAUNCH;
}

template <int FMT>
int run_linear(const void* W, const uint16_t* scales, const uint16_t* X, uint16_t* Y, int M, int64_t N, int64_t K,
               void* stream) {
  if (!W || !X || !Y || (FMT != FMT_FP16 && !scales)) return AMS_ERR_NULL;
  if (M < 1 || M > AMS_MAX_M || N <= 0 || K <= 0 || N > (1 << 24) || K > (1 << 24)) return AMS_ERR_SHAPE;
  if (FMT == FMT_FP16 && (K % 8) != 0) return AMS_ERR_SHAPE;
  if (!aligned16(W) || !aligned16(X) || !aligned16(Y) || (scales && !aligned16(scales))) return AMS_ERR_ALIGN;
  constexpr int REC_K = Fmt<FMT>::REC_K;
  const int64_t n_strips = (N + 15) / 16;
  const int n_rec = (int)((K + REC_K - 1) / REC_K);
  constexpr int HI = FMT == FMT_FP16 ? 4 : 16, LO = FMT == FMT_FP16 ? 1 : 4;
  const Plan p = make_plan(M, n_strips, n_rec, REC_K, HI, LO);
  LinearArgs a;
  a.W = (const uint8_t*)W;
  a.scales = scales;
  a.X = X;
  a.Y = Y;
  a.M = M;
  a.N = (int)N;
  a.K = (int)K;
  a.n_rec = n_rec;
  a.recs_per_wave = p.L;
  a.x_stride = p.x_stride;
  hipStream_t st = (hipStream_t)stream;
  if (M <= 16)
    return p.lmax == LO ? launch_linear<FMT, 1, LO>(a, p, n_strips, st) : launch_linear<FMT, 1, HI>(a, p, n_strips, st);
  return p.lmax == LO ? launch_linear<FMT, 2, LO>(a, p, n_strips, st) : launch_linear<FMT, 2, HI>(a, p, n_strips, st);
}

}  // namespace

extern "C" {

int ams_dequant(int fmt, const void* W_packed, const uint16_t* scales, uint16_t* W_out, int64_t N, int64_t K, int scaled,
                void* stream) {
  const ams::FormatInfo* fi = ams::format_info(fmt);
  if (!fi) return AMS_ERR_FORMAT;
  if (!W_packed || !W_out || (scaled && !scales)) return AMS_ERR_NULL;
  if (N <= 0 || K <= 0 || N > (1 << 24) || K > (1 << 24)) return AMS_ERR_SHAPE;
  if (!aligned16(W_packed)) return AMS_ERR_ALIGN;
  const int n_rec = (int)((K + fi->rec_k - 1) / fi->rec_k);
  const int64_t total = ((N + 15) / 16) * n_rec;
  const unsigned grid = (unsigned)((total + 3) / 4);
  hipStream_t st = (hipStream_t)stream;
  if (fmt == FMT_FP533)
    hipLaunchKernelGGL(dequant_kernel<FMT_FP533>, dim3(grid), dim3(256), 0, st, (const uint8_t*)W_packed, scales, W_out,
                       (int)N, (int)K, n_rec, total, scaled);
  else
    hipLaunchKernelGGL(dequant_kernel<FMT_FP425>, dim3(grid), dim3(256), 0, st, (const uint8_t*)W_packed, scales, W_out,
                       (int)N, (int)K, n_rec, total, scaled);
  return hipGetLastError() == hipSuccess ? AMS_OK : AMS_ERR_LAUNCH;
}

int ams_linear(const void* W_packed, const uint16_t* scales, const uint16_t* X, uint16_t* Y, int M, int64_t N, int64_t K,
               int fmt, void* stream) {
  if (fmt == FMT_FP533) return run_linear<FMT_FP533>(W_packed, scales, X, Y, M, N, K, stream);
  if (fmt == FMT_FP425) return run_linear<FMT_FP425>(W_packed, scales, X, Y, M, N, K, stream);
  return AMS_ERR_FORMAT;
}

int ams_fp16_linear(const uint16_t* W, const uint16_t* X, uint16_t* Y, int M, int64_t N, int64_t K, void* stream) {
  return run_linear<FMT_FP16>(W, nullptr, X, Y, M, N, K, stream);
}

}  // extern "C"
