// HIP kernels (gfx950 / CDNA4) of the AMS-Quant weight-only quantized Linear:
// bit-level restoration of the packed weights (Sec. 3.2, Sec. 3.3 stages 2-3) fused
// with the skinny fp16 matmul of the decode stage (Sec. 4.2), and the fp16 baseline.
//
// Every lane loads its 16-byte chunk of a record with one dwordx4 (a record is one
// contiguous 1 KiB access per wavefront), restores the fp16 pairs in registers and feeds
// them as the A operand of v_mfma_f32_16x16x32_f16; the activations are staged in LDS in
// the operand order the restoration produces.
//   column_kernel  the packed formats: a workgroup owns up to 16 neighbouring strips, every
//                  wavefront stays with one strip and walks K in step with all the others, so
//                  that the grid as a whole reads one contiguous, moving window of the K-major
//                  packed matrix; the partial tile of a strip never leaves its wavefront's
//                  registers until the end.
//   sweep_kernel / stream_kernel   the fp16 baseline (row-major weights).
// Partial tiles are combined through LDS, deterministically; only the entry points that take
// a workspace also split K over workgroups and exchange fp32 tiles through it.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>
#include <type_traits>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/ams.h"
#include "ams_layout.h"

namespace {

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef uint32_t u4 __attribute__((ext_vector_type(4)));
typedef unsigned short us2 __attribute__((ext_vector_type(2)));
typedef unsigned short us4 __attribute__((ext_vector_type(4)));

constexpr int FMT_FP533 = AMS_FMT_FP533_E2M3;
constexpr int FMT_FP425 = AMS_FMT_FP425_E2M2;
constexpr int FMT_FP45 = AMS_FMT_FP45_E2M2;
constexpr int FMT_FP433 = AMS_FMT_FP433_E2M2;
constexpr int FMT_FP6 = AMS_FMT_FP6_E2M3;
constexpr int FMT_FP5 = AMS_FMT_FP5_E2M2;
constexpr int FMT_FP4 = AMS_FMT_FP4_E2M1;
constexpr int FMT_FP16 = 100;  // internal: unquantized row-major fp16 weights (baseline)
static_assert(FMT_FP533 == ams::kFmtFp533 && FMT_FP425 == ams::kFmtFp425 && FMT_FP45 == ams::kFmtFp45 &&
              FMT_FP433 == ams::kFmtFp433 && FMT_FP6 == ams::kFmtFp6 && FMT_FP5 == ams::kFmtFp5 && FMT_FP4 == ams::kFmtFp4, "format numbers");

constexpr float kTwo14 = 16384.0f;  // restored patterns are value * 2^-14

__device__ __forceinline__ uint32_t bfi(uint32_t mask, uint32_t a, uint32_t b) { return (a & mask) | (b & ~mask); }

__device__ __forceinline__ uint32_t pk_mul_u16(uint32_t a, uint32_t c) {
  us2 x = __builtin_bit_cast(us2, a), y = __builtin_bit_cast(us2, c);
  return __builtin_bit_cast(uint32_t, (us2)(x * y));
}

// e2m2 formats (Sec. 3.2): one 32-bit word = two half-words of four 4-bit remainders.
// sh[t] holds the last mantissa bits of pair t already placed at bits 8 and 24.
// Produces the four fp16 pairs (A_t low, B_t high) as bit patterns of value * 2^-14:
// sign -> bit 15, e1 e0 m1 -> bits 11..9, last bit m0 -> bit 8.
__device__ __forceinline__ void restore_e2m2(uint32_t s, const uint32_t sh[4], uint32_t out[4]) {
  constexpr uint32_t M = 0x8E008E00u;
  out[0] = bfi(M, s, sh[0]);
  out[1] = bfi(M, s << 3, sh[1]);
  // members 2 and 3: sign and magnitude need different shifts; a packed 16-bit
  // multiply by (2^a + 2^b) makes both shifted copies at once
  out[2] = bfi(M, pk_mul_u16(s & 0x40384038u, 0x00420042u), sh[2]);
  out[3] = bfi(M, pk_mul_u16(s & 0x20072007u, 0x02040204u), sh[3]);
}
// FP4.25: the four members of a half-word are one group, one pair of shared bits per word
__device__ __forceinline__ void restore_fp425(uint32_t s, uint32_t sh, uint32_t out[4]) {
  const uint32_t same[4] = {sh, sh, sh, sh};
  restore_e2m2(s, same, out);
}

// Last bits kept in a side byte: bit t belongs to pair t's A half, bit 4+t to its B half.
__device__ __forceinline__ uint32_t spread_side_byte(uint32_t byte) { return byte | (byte << 12); }
__device__ __forceinline__ uint32_t pair_bits_e2m2(uint32_t spread, int t) { return (spread << (8 - t)) & 0x01000100u; }

// e2m3 formats (Sec. 3.3 item 1): one 32-bit word = two half-words of three 5-bit
// remainders; sh0..sh2 hold the last bits of the three pairs at bits 7 and 23.
// Produces three fp16 pairs (A_i low, B_i high): sign -> bit 15, e1 e0 m2 m1 ->
// bits 11..8, last bit m0 -> bit 7.
__device__ __forceinline__ void restore_e2m3(uint32_t s, uint32_t sh0, uint32_t sh1, uint32_t sh2, uint32_t out[3]) {
  constexpr uint32_t M = 0x8F008F00u;
  out[0] = bfi(M, s, sh0);
  {
    // member 1: magnitude and sign need different shifts; spelled out as and-or + bit-field
    // insert (left to itself the compiler makes two ands and a three-way or: one operation more)
    uint32_t t, r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(t) : "v"(s << 4), "s"(0x0F000F00u), "v"(sh1));
    asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(r) : "s"(0x80008000u), "v"(s << 1), "v"(t));
    out[1] = r;
  }
  out[2] = bfi(M, pk_mul_u16(s & 0x200F200Fu, 0x01040104u), sh2);
}
// FP5.33: each half-word is a whole group, its shared bit sits at bit 12
__device__ __forceinline__ void restore_fp533(uint32_t s, uint32_t out[3]) {
  const uint32_t sh = (s >> 5) & 0x00800080u;
  restore_e2m3(s, sh, sh, sh, out);
}

template <int FMT>
struct Fmt {
  static constexpr int REC_K = ams::kFormats[FMT].rec_k, REC_BYTES = ams::kFormats[FMT].rec_bytes,
                       CHUNK = ams::kFormats[FMT].chunk_bytes, SIDE = ams::kFormats[FMT].side_bytes,
                       PB = ams::kFormats[FMT].perm_block, N_MFMA = REC_K / 32,
                       SG = ams::side_group(ams::kFormats[FMT]),       // records per unit (a power of two)
                       CB = ams::chunk_block_bytes(ams::kFormats[FMT]),  // bytes of one record's lane chunks
                       UNIT = ams::unit_bytes(ams::kFormats[FMT]);
};
template <>
struct Fmt<FMT_FP16> {
  static constexpr int REC_K = 128, REC_BYTES = 0, CHUNK = 0, SIDE = 0, PB = 8, N_MFMA = 4, SG = 1, CB = 0, UNIT = 0;
};

// Input channel (inside its permutation block) of every operand slot of the block.
template <int FMT>
struct SlotChannel {
  int v[Fmt<FMT>::PB];
  constexpr SlotChannel() : v{} {
    for (int i = 0; i < Fmt<FMT>::PB; i++) v[i] = FMT == FMT_FP16 ? i : ams::slot_channel(FMT == FMT_FP16 ? 0 : FMT, i);
  }
};
template <int FMT>
__device__ constexpr int slot_channel(int s) {
  constexpr SlotChannel<FMT> tab{};
  return tab.v[s];
}

// What one lane holds of one record: the words of its chunk and, for formats with side bits,
// the lane's side dword of the record's unit (the record's own byte(s) are picked where it is restored).
template <int SIDE>
struct SideBits {
  uint32_t t;
};
template <>
struct SideBits<0> {};
template <int FMT>
struct LaneRec : SideBits<Fmt<FMT>::SIDE> {
  uint32_t w[Fmt<FMT>::CHUNK / 4];
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
  int n_rec;     // records per strip
  int x_stride;  // halfs between activation rows inside a wave's LDS region
  int x_region;  // halfs of one wave's LDS region
  int x_shift;   // log2 of the staging units per activation row, rounded up to a power of two
  int n_strips;  // strips of 16 output channels
  int spw;       // stream kernel: strips per workgroup
  int red_slots; // stream kernel: partial tiles a wave may park in LDS (strips its piece can touch)
  int piece_q, piece_r;  // stream kernel: pairs per wave in a full workgroup: quotient, remainder
  int rc;                // stream kernel: records per strip in one phase of K
  int n_sg, sg_shift;    // scales per run of input channels: runs per row, log2(records per run)
  // split of K over gk workgroups per strip (sweep kernel with a workspace): workgroups along N,
  // slices of K, per-slice partial tiles [gk][strip][MT][64] f4, per-strip arrival counters
  int gn, gk;
  int wps;  // wavefronts that share a strip (sweep kernel: the workgroup works on S / wps strips at a time)
  int wpa;  // column kernel: how many of a strip's wps wavefronts take records (the others idle: a count that divides the work evenly)
  f4* ws_tiles;
  unsigned* ws_count;
};

// One lane's part of a record: its chunk at `chunks` (one dwordx4, or three dwords that the
// compiler merges) and its dword of the unit's side block at `side`.
template <int FMT, bool NT, bool WITH_SIDE = true>
__device__ __forceinline__ void load_lane_rec(LaneRec<FMT>& r, const uint8_t* chunks, const uint8_t* side, int lane) {
  constexpr int CHUNK = Fmt<FMT>::CHUNK, SIDE = Fmt<FMT>::SIDE;
  auto ld = [](auto* p) { return NT ? __builtin_nontemporal_load(p) : *p; };
  if constexpr (CHUNK == 16) {
    const u4 v = ld((const u4*)(chunks + lane * 16));
    r.w[0] = v[0], r.w[1] = v[1], r.w[2] = v[2], r.w[3] = v[3];
  } else {
    const uint32_t* p = (const uint32_t*)(chunks + lane * CHUNK);
#pragma unroll
    for (int d = 0; d < CHUNK / 4; d++) r.w[d] = ld(p + d);
  }
  // WITH_SIDE = false: the caller keeps the group's side dword elsewhere
  if constexpr (SIDE != 0 && WITH_SIDE) r.t = ld((const uint32_t*)side + lane);
}

// The MFMA A operands of one record as packed fp16 pairs: o[4u + t] = elements 2t, 2t+1
// of the lane's row in MFMA u (bit patterns of value * 2^-14).
// side_shift: first bit of this record's side bits inside the unit's side dword (wave-uniform).
template <int FMT>
__device__ __forceinline__ void restore_rec(const LaneRec<FMT>& r, int side_shift, uint32_t (&o)[4 * Fmt<FMT>::N_MFMA]) {
  if constexpr (FMT == FMT_FP533) {
#pragma unroll
    for (int d = 0; d < 4; d++) restore_fp533(r.w[d], &o[3 * d]);
  } else if constexpr (FMT == FMT_FP6) {
    // side bits: bit 2d + (i-1) = member i of half A of word d, the same + 8 for half B
    const uint32_t t = r.t >> side_shift;
    const uint32_t spread = (t & 0xFFu) | ((t & 0xFF00u) << 8);
#pragma unroll
    for (int d = 0; d < 4; d++)
      restore_e2m3(r.w[d], (r.w[d] >> 5) & 0x00800080u, (spread << (7 - 2 * d)) & 0x00800080u, (spread << (6 - 2 * d)) & 0x00800080u,
                   &o[3 * d]);
  } else if constexpr (FMT == FMT_FP425) {
    const uint32_t spread = spread_side_byte(__builtin_amdgcn_ubfe(r.t, (uint32_t)side_shift, 8u));
#pragma unroll
    for (int d = 0; d < 4; d++) restore_fp425(r.w[d], pair_bits_e2m2(spread, d), &o[4 * d]);
  } else if constexpr (FMT == FMT_FP4) {
    // an e2m1 code is an e2m2 remainder whose last bit is 0
    const uint32_t none[4] = {0, 0, 0, 0};
#pragma unroll
    for (int d = 0; d < 4; d++) restore_e2m2(r.w[d], none, &o[4 * d]);
  } else {
    // FP4.33: one side byte for all words; FP4.5: one per two words; FP5: one per word
    constexpr int WORDS_PER_BYTE = FMT == FMT_FP433 ? 3 : (FMT == FMT_FP45 ? 2 : 1);
    const uint32_t t = Fmt<FMT>::SIDE == 4 ? r.t : __builtin_amdgcn_ubfe(r.t, (uint32_t)side_shift, (uint32_t)(8 * Fmt<FMT>::SIDE));
    uint32_t sh[4];
#pragma unroll
    for (int d = 0; d < Fmt<FMT>::CHUNK / 4; d++) {
      if (d % WORDS_PER_BYTE == 0) {
        const uint32_t spread = spread_side_byte(Fmt<FMT>::SIDE == 1 ? t : (t >> (8 * (d / WORDS_PER_BYTE))) & 0xFFu);
#pragma unroll
        for (int i = 0; i < 4; i++) sh[i] = pair_bits_e2m2(spread, i);
      }
      restore_e2m2(r.w[d], sh, &o[4 * d]);
    }
  }
}

// Unconditional loads of one record (rec must be a valid record of the strip).  NT: packed
// records bypass the caches' retention (they are read once per call, and a model's other
// layers pass through the caches before the next call); only tiny matrices use ordinary loads.
template <int FMT, bool NT = true>
__device__ __forceinline__ void load_rec(LaneRec<FMT>& r, const LinearArgs& a, int strip, int rec, int lane) {
  if constexpr (FMT == FMT_FP16) {
    // rows beyond N and K-chunks beyond K are redirected to the matrix's first 16 bytes
    // and zeroed afterwards: keeps the loads free of control flow
    const int row = strip * 16 + (lane & 15);
    const int kq = lane >> 4;
#pragma unroll
    for (int d = 0; d < 4; d++) {
      const int k = rec * 128 + 32 * d + 8 * kq;
      const bool ok = row < a.N && k < a.K;  // K is a multiple of 8
      const size_t off = ok ? ((size_t)row * a.K + k) * 2 : 0;
      const u4 v = *(const u4*)(a.W + off);  // cached: the two halves of a 128-byte line come from two loads
      const uint32_t keep = ok ? 0xFFFFFFFFu : 0u;
      r.w[d] = u4{v[0] & keep, v[1] & keep, v[2] & keep, v[3] & keep};
    }
  } else {
    // unit (rec / SG, strip) of the K-major packed matrix, record rec % SG inside it
    constexpr int SG = Fmt<FMT>::SG;
    const uint8_t* unit = a.W + ((size_t)(rec / SG) * a.n_strips + strip) * Fmt<FMT>::UNIT;
    load_lane_rec<FMT, NT>(r, unit + (rec % SG) * Fmt<FMT>::CB, unit + SG * Fmt<FMT>::CB, lane);
  }
}

// Multiply one record (16 rows x REC_K) into the accumulators.  x0 / x1 point at this
// lane's activation row(s) in LDS at the first operand slot of its K-quarter of the record.
// side_shift: see restore_rec (8 * SIDE * (rec % SG); 0 for formats without side bits).
template <int FMT, int MT>
__device__ __forceinline__ void mac_rec(const LaneRec<FMT>& r, const _Float16* x0, const _Float16* x1, f4 acc[MT], int side_shift = 0) {
  h8 a[Fmt<FMT>::N_MFMA];
  if constexpr (FMT == FMT_FP16) {
#pragma unroll
    for (int d = 0; d < 4; d++) a[d] = __builtin_bit_cast(h8, r.w[d]);
  } else {
    uint32_t o[4 * Fmt<FMT>::N_MFMA];
    restore_rec<FMT>(r, side_shift, o);
#pragma unroll
    for (int u = 0; u < Fmt<FMT>::N_MFMA; u++) a[u] = __builtin_bit_cast(h8, u4{o[4 * u], o[4 * u + 1], o[4 * u + 2], o[4 * u + 3]});
  }
#pragma unroll
  for (int u = 0; u < Fmt<FMT>::N_MFMA; u++) {
    // FP16 records interleave the K-quarters per MFMA (32 consecutive k each)
    const int off = FMT == FMT_FP16 ? 32 * u : 8 * u;
    acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[u], *(const h8*)(x0 + off), acc[0], 0, 0, 0);
    if constexpr (MT == 2) acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[u], *(const h8*)(x1 + off), acc[1], 0, 0, 0);
  }
}

// Operand slot of activation k (relative to its record) in LDS.
template <int FMT>
__device__ __forceinline__ int x_slot(int kk) {
  if constexpr (FMT == FMT_FP16) {
    return kk;
  } else {
    constexpr int PB = Fmt<FMT>::PB;
    const int blk = kk / PB, j = kk - blk * PB;
    int slot = 0;
    for (int s = 0; s < PB; s++)
      if (slot_channel<FMT>(s) == j) slot = s;
    return blk * PB + slot;
  }
}

// dword made of half `ia` (low) and half `ib` (high) of an array of packed half pairs
__device__ __forceinline__ uint32_t pick2(const uint32_t* in, int ia, int ib) {
  const uint32_t sel = (uint32_t)(2 * (ia & 1)) | (uint32_t)(2 * (ia & 1) + 1) << 8 | (uint32_t)(4 + 2 * (ib & 1)) << 16 |
                       (uint32_t)(5 + 2 * (ib & 1)) << 24;
  return __builtin_amdgcn_perm(in[ib >> 1], in[ia >> 1], sel);
}

// One permutation block of activations from input-channel order into operand order
// (packed pairs in, packed pairs out).
template <int FMT>
__device__ __forceinline__ void permute_unit(const uint32_t (&in)[Fmt<FMT>::PB / 2], uint32_t (&out)[Fmt<FMT>::PB / 2]) {
#pragma unroll
  for (int m = 0; m < Fmt<FMT>::PB / 2; m++) {
    if constexpr (FMT == FMT_FP16)
      out[m] = in[m];
    else
      out[m] = pick2(in, slot_channel<FMT>(2 * m), slot_channel<FMT>(2 * m + 1));
  }
}

// Activation staging.  A wave copies X[0..M) x [k0, k0+nk) into its LDS region in operand
// order (zero beyond K), nk a multiple of the record size.  The copy is split in a load
// half (global -> registers, no control flow around the loads) and a store half
// (permute + LDS write) so that the loads can be issued ahead of the weight stream.
// The work is cut in units of UNIT halfs; unit u covers row u >> x_shift, position
// u & (2^x_shift - 1) (rows are padded to a power of two of units).
template <int FMT>
struct XUnit {
  static constexpr int UNIT = Fmt<FMT>::PB;               // halfs permuted together
  static constexpr int CH = UNIT / 8;                     // 16-byte chunks per unit
  static constexpr int XU = 2;                            // units a lane moves in the first pass (in flight with the weights)
  static constexpr int XB = CH == 1 ? 8 : CH == 2 ? 4 : 2;  // units a lane moves in each further pass (all requested, then stored)
};

template <int FMT, int NU = XUnit<FMT>::XU>
struct XRegs {
  u4 c[NU][XUnit<FMT>::CH];
};

// Units u0 + i * nthr + idx, i < NU.
template <int FMT, int NU>
__device__ __forceinline__ void x_load(XRegs<FMT, NU>& xr, const LinearArgs& a, int k0, int nk, int u0, int idx, int nthr) {
  constexpr int UNIT = XUnit<FMT>::UNIT, CH = XUnit<FMT>::CH;
  const int upr = nk / UNIT;
#pragma unroll
  for (int i = 0; i < NU; i++) {
    const int u = u0 + i * nthr + idx;
    const int m = u >> a.x_shift, j = u & ((1 << a.x_shift) - 1);
    const int k = k0 + UNIT * j;
    const bool row_ok = m < a.M && j < upr;
#pragma unroll
    for (int e = 0; e < CH; e++) {
      const bool ok = row_ok && k + 8 * e < a.K;
      const size_t off = ok ? (size_t)m * a.K + k + 8 * e : 0;  // redirected loads are zeroed by x_store
      xr.c[i][e] = *(const u4*)(a.X + off);
    }
  }
}

template <int FMT, int NU>
__device__ __forceinline__ void x_store(const XRegs<FMT, NU>& xr, _Float16* xs, const LinearArgs& a, int k0, int nk, int u0,
                                        int idx, int nthr) {
  constexpr int UNIT = XUnit<FMT>::UNIT, CH = XUnit<FMT>::CH;
  const int upr = nk / UNIT;
#pragma unroll
  for (int i = 0; i < NU; i++) {
    const int u = u0 + i * nthr + idx;
    const int m = u >> a.x_shift, j = u & ((1 << a.x_shift) - 1);
    const int k = k0 + UNIT * j;
    uint32_t in[4 * CH], out[4 * CH];
#pragma unroll
    for (int e = 0; e < CH; e++) {
      const uint32_t keep = k + 8 * e < a.K ? 0xFFFFFFFFu : 0u;  // zero beyond K
      in[4 * e] = xr.c[i][e][0] & keep, in[4 * e + 1] = xr.c[i][e][1] & keep;
      in[4 * e + 2] = xr.c[i][e][2] & keep, in[4 * e + 3] = xr.c[i][e][3] & keep;
    }
    permute_unit<FMT>(in, out);
    if (m < a.M && j < upr) {
      u4* dst = (u4*)(xs + m * a.x_stride + UNIT * j);
#pragma unroll
      for (int e = 0; e < CH; e++) dst[e] = u4{out[4 * e], out[4 * e + 1], out[4 * e + 2], out[4 * e + 3]};
    }
  }
}

// Element-by-element staging for activations whose rows are not 16-byte aligned (K % 8 != 0).
template <int FMT>
__device__ __forceinline__ void stage_x_unaligned(_Float16* xs, const LinearArgs& a, int k0, int nk, int idx0, int nthr) {
  for (int idx = idx0; idx < a.M * nk; idx += nthr) {
    const int m = idx / nk, kk = idx - m * nk;
    const int k = k0 + kk;
    const uint16_t v = k < a.K ? a.X[(size_t)m * a.K + k] : (uint16_t)0;
    const int rl = kk / Fmt<FMT>::REC_K, kr = kk - rl * Fmt<FMT>::REC_K;
    ((uint16_t*)xs)[m * a.x_stride + rl * Fmt<FMT>::REC_K + x_slot<FMT>(kr)] = v;
  }
}

// fp16 bits of the scales of the four output channels a lane holds of a strip's tile
struct ScaleBits {
  uint16_t b[4];
};
template <int FMT>
__device__ __forceinline__ ScaleBits load_scale_bits(const LinearArgs& a, int strip, int lane) {
  ScaleBits sb = {{0x3C00, 0x3C00, 0x3C00, 0x3C00}};
  if constexpr (FMT != FMT_FP16) {
    const int n0 = strip * 16 + 4 * (lane >> 4);
#pragma unroll
    for (int r = 0; r < 4; r++) sb.b[r] = a.scales[min(n0 + r, a.N - 1)];  // clamped: rows beyond N are never stored
  }
  return sb;
}
// fp32 multipliers s_n * 2^14 (the baseline's "scales" are 1: its bits are 1.0 and no 2^14 is owed)
__device__ __forceinline__ f4 scales_from_bits(const ScaleBits& sb, float mul = kTwo14) {
  f4 sc;
#pragma unroll
  for (int r = 0; r < 4; r++) sc[r] = (float)__builtin_bit_cast(_Float16, sb.b[r]) * mul;
  return sc;
}
template <int FMT>
__device__ __forceinline__ f4 load_scales(const LinearArgs& a, int strip, int lane) {
  return scales_from_bits(load_scale_bits<FMT>(a, strip, lane), FMT == FMT_FP16 ? 1.0f : kTwo14);
}

// Multiply a finished 16x16 tile (C[i][j]: lane = j + 16*(i/4), register i%4) by the scales, convert, store.
template <int MT>
__device__ __forceinline__ void store_tile_scaled(const f4 t[MT], const f4 sc, const LinearArgs& a, int strip, int lane) {
  const int m_lo = lane & 15, kq = lane >> 4;
#pragma unroll
  for (int mt = 0; mt < MT; mt++) {
    const int m = m_lo + 16 * mt;
    if (m < a.M) {
      const int n0 = strip * 16 + 4 * kq;
      us4 h;
#pragma unroll
      for (int r = 0; r < 4; r++) h[r] = __builtin_bit_cast(uint16_t, (_Float16)(t[mt][r] * sc[r]));
      if (n0 + 3 < a.N && (a.N & 3) == 0) {  // the lane's four output channels are eight aligned bytes of Y's row m
        *(us4*)(a.Y + (size_t)m * a.N + n0) = h;
      } else {
#pragma unroll
        for (int r = 0; r < 4; r++)
          if (n0 + r < a.N) a.Y[(size_t)m * a.N + n0 + r] = h[r];
      }
    }
  }
}

// The streaming Linear.  A workgroup owns `spw` consecutive strips and walks K in
// phases of `rc` records per strip (one phase when the activations M x K fit in LDS).
// Inside a phase its work is the list of (strip, record) pairs in strip-major order;
// the S wavefronts cut that list into S equal contiguous pieces, whatever the strip
// boundaries, so every wave streams the same number of bytes through its register ring
// (records of a strip are adjacent in memory, and with one phase those of consecutive
// strips are too).  The pieces are the same in every phase, so a wave meets the same
// strips again: its partial 16x16 tiles live in LDS slots and are swapped in and out
// of the accumulator registers where its piece crosses a strip boundary.  The
// activations of a phase are staged once per workgroup in LDS (operand order).  After
// the last phase the wave holding a strip's first record adds the tiles of the waves
// after it, in wave order, scales and stores.  The grid is one resident round.
template <int MT, int LR>
__global__ void __launch_bounds__(1024) stream_kernel(LinearArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int FMT = FMT_FP16;  // the baseline's kernel: row-major fp16 weights
  constexpr int REC_K = Fmt<FMT>::REC_K;
  // All kernel arguments are pulled in at once: fetched piecemeal where they are first used,
  // each batch would be one more trip to memory in front of the first weight load.
  asm volatile("" ::"s"(a.W), "s"(a.scales), "s"(a.X), "s"(a.Y), "s"(a.M), "s"(a.N), "s"(a.K), "s"(a.n_rec), "s"(a.x_stride),
               "s"(a.x_region), "s"(a.x_shift), "s"(a.n_strips), "s"(a.spw), "s"(a.red_slots), "s"(a.piece_q), "s"(a.piece_r),
               "s"(a.rc));
  const int tid = threadIdx.x, lane = tid & 63, nthr = blockDim.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int S = nthr >> 6;
  const int strip0 = blockIdx.x * a.spw;
  const int ns = min(a.spw, a.n_strips - strip0);
  const int RC = a.rc;
  const int P = ns * RC;  // (strip, record) pairs of one phase
  // balanced pieces: wave w takes piece_q pairs, the first piece_r waves one more
  // (the host supplies the quotient for full workgroups: no 64-bit division in here)
  int piece_q = a.piece_q, piece_r = a.piece_r;
  if (ns != a.spw) {
    piece_q = (int)((unsigned)P / (unsigned)S);
    piece_r = P - piece_q * S;
  }
  const int g0 = wave * piece_q + min(wave, piece_r), g1 = g0 + piece_q + (wave < piece_r ? 1 : 0);
  const int g_last = max(g1 - 1, 0);
  // strip of the piece's first pair and its record inside the phase
  const int s_first = (int)((unsigned)min(g0, g_last) / (unsigned)RC);
  const int j_first = min(g0, g_last) - s_first * RC;
  _Float16* xs = (_Float16*)smem;
  f4* red = (f4*)(smem + (size_t)a.x_region * 2);  // [S][red_slots][MT][64]
  f4* const my_red = red + (size_t)wave * a.red_slots * MT * 64 + lane;  // this wave's tiles: [slot][MT][64]
  const int m_lo = lane & 15, kq = lane >> 4;
  const int lane_off = FMT == FMT_FP16 ? 8 * kq : (REC_K / 4) * kq;
  // lanes whose activation row does not exist read row 0: they only feed output columns never stored
  const _Float16* x0 = xs + (m_lo < a.M ? m_lo : 0) * a.x_stride + lane_off;
  const _Float16* x1 = xs + (m_lo + 16 < a.M ? m_lo + 16 : 0) * a.x_stride + lane_off;

  const bool vec_x = (a.K & 7) == 0;
  const int total_units = a.M << a.x_shift;
  const int units_per_pass = nthr * XUnit<FMT>::XU;
  const bool wave_has_x = vec_x && wave * 64 < total_units;  // wave-uniform
  const int chunk_k = RC * REC_K;
  __builtin_amdgcn_sched_barrier(0);

  for (int rec_base = 0; rec_base < a.n_rec; rec_base += RC) {
    // Activations of the phase, in operand order.  Units beyond the first pass (large M)
    // and unaligned rows are staged by loops that run to completion first; the first
    // pass is only requested here and stored after the head of the weight stream has
    // been requested too, so both are in flight together and the stream starts as soon
    // as its first record lands.  Waves whose units all fall outside skip the pass.
    if (rec_base > 0) __syncthreads();  // everyone is done with the previous phase's activations
    const int k0 = rec_base * REC_K;
    XRegs<FMT> xr;
    if (vec_x) {
      for (int u0 = units_per_pass; u0 < total_units; u0 += nthr * XUnit<FMT>::XB) {
        XRegs<FMT, XUnit<FMT>::XB> xb;
        x_load(xb, a, k0, chunk_k, u0, tid, nthr);
        x_store(xb, xs, a, k0, chunk_k, u0, tid, nthr);
      }
    } else {
      stage_x_unaligned<FMT>(xs, a, k0, chunk_k, tid, nthr);
    }
    if (wave_has_x) x_load(xr, a, k0, chunk_k, 0, tid, nthr);
    __builtin_amdgcn_sched_barrier(0);

    // the head of the weight stream: LR records in flight per wave.  The prefetch cursor
    // (pair index, strip, record in phase) is clamped to the piece's last pair; records
    // beyond the end of K (last phase) are redirected to the strip's last record and skipped.
    const int rec_hi = a.n_rec - 1 - rec_base;  // last valid record of this phase, relative
    int pp = min(g0, g_last), ps = s_first, pj = j_first;
    LaneRec<FMT> ring[LR];
#pragma unroll
    for (int q = 0; q < LR; q++) {
      load_rec<FMT>(ring[q], a, strip0 + ps, rec_base + min(pj, rec_hi), lane);
      if (pp < g_last) {
        pp++;
        if (++pj == RC) pj = 0, ps++;
      }
      __builtin_amdgcn_sched_barrier(0);  // issue in ring order: the oldest load is the first one needed
    }

    if (rec_base == 0) {
      // set-up that nothing above needs, done while the first loads are in flight: this wave's tile slots cleared
      for (int t = 0; t < a.red_slots * MT; t++) my_red[t * 64] = f4{0, 0, 0, 0};
    }
    if (wave_has_x) x_store(xr, xs, a, k0, chunk_k, 0, tid, nthr);
    __syncthreads();

    f4 acc[MT];
    f4* slot_ptr = my_red;
#pragma unroll
    for (int i = 0; i < MT; i++) acc[i] = slot_ptr[i * 64];
    int g = g0, j = j_first;

    // One pair: multiply, refill the ring slot; where the strip (or the piece) ends, the
    // tile goes back to its LDS slot and the next strip's tile comes in.  Nothing in
    // here touches global memory except the refill, so the ring drains one record at a time.
    auto step = [&](LaneRec<FMT>& slot) {
      if (j <= rec_hi) mac_rec<FMT, MT>(slot, x0 + j * REC_K, x1 + j * REC_K, acc);
      load_rec<FMT>(slot, a, strip0 + ps, rec_base + min(pj, rec_hi), lane);
      if (pp < g_last) {
        pp++;
        if (++pj == RC) pj = 0, ps++;
      }
      g++;
      j++;
      if (j == RC || g == g1) {
#pragma unroll
        for (int i = 0; i < MT; i++) slot_ptr[i * 64] = acc[i];
        if (j == RC) {
          slot_ptr += MT * 64;
          j = 0;
        }
#pragma unroll
        for (int i = 0; i < MT; i++) acc[i] = slot_ptr[i * 64];
      }
    };

    while (g + LR <= g1) {
#pragma unroll
      for (int q = 0; q < LR; q++) {
        step(ring[q]);
        // keep the refill right behind its record
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int q = 0; q < LR - 1; q++)
      if (g < g1) step(ring[q]);
  }

  // Finish the strips.  The wave that holds a strip's first pair owns it: it adds the
  // head tiles (slot 0) of the waves after it whose pieces still lie in that strip, in
  // wave order, and stores.  The tile reads do not depend on each other, so they overlap.
  __syncthreads();
  if (g1 > g0) {
    const int s_begin = j_first == 0 ? s_first : s_first + 1;  // first strip that starts inside this piece
    for (int s = s_begin; s * RC < g1; s++) {
      const int se = (s + 1) * RC;
      f4 sum[MT];
#pragma unroll
      for (int i = 0; i < MT; i++) sum[i] = red[(((size_t)wave * a.red_slots + (s - s_first)) * MT + i) * 64 + lane];
      if (se > g1) {  // the strip runs on into the pieces of the next nf waves
        int nf = 0;
        for (int w2 = wave + 1, h0 = g1; w2 < S && h0 < se; w2++) {
          const int len = piece_q + (w2 < piece_r ? 1 : 0);
          if (len == 0) break;
          h0 += len;
          nf++;
        }
        const f4* follower = red + (size_t)wave * a.red_slots * MT * 64 + lane;  // slot 0 of this wave; followers are whole waves further
        const int wave_stride = a.red_slots * MT * 64;
#pragma unroll
        for (int d = 1; d < 16; d++) {
          // reads are independent and unconditional (inside the tile area: wave index clamped);
          // selected, not multiplied: a tile that is not taken may be uninitialised LDS
          const f4* t = follower + min(d, S - 1 - wave) * wave_stride;
#pragma unroll
          for (int i = 0; i < MT; i++) {
            const f4 v = t[i * 64];
            sum[i] += d <= nf ? v : f4{0, 0, 0, 0};
          }
        }
      }
      store_tile_scaled<MT>(sum, f4{1.0f, 1.0f, 1.0f, 1.0f}, a, strip0 + s, lane);  // the baseline has no scales
    }
  }
}

// The sweeping Linear.  Strips are dealt to the workgroups round robin (workgroup g owns
// strips g, g + G, g + 2G, ...), and inside a workgroup the records of its strips, taken
// as one list in that order, are dealt to the S wavefronts record by record.  At any
// moment a workgroup therefore reads one contiguous run of S * LR records, and the whole
// grid reads a window of G neighbouring strips that moves through the matrix front to
// back: the order the memory system serves fastest (measured with bare read kernels, this
// beats per-wavefront contiguous pieces by 15-20 % on the Llama shapes, and two records in
// flight per wave beat four).  Every wave meets every strip of its workgroup, so it parks
// one partial 16x16 tile per strip in LDS (only the lanes of existing activation rows);
// after one barrier the strips are finished one per wave: the S tiles added in wave
// order, scaled, converted, stored.  The activations are staged once per workgroup in LDS
// in operand order; when M x K does not fit, K is walked in phases of rc records per strip
// and the parked tiles accumulate over the phases.  The grid is one resident round.
template <int MT, int LR, bool GROUPS = false>
__global__ void __launch_bounds__(1024) sweep_kernel(LinearArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int FMT = FMT_FP16;  // the baseline's kernel: row-major fp16 weights
  constexpr int REC_K = Fmt<FMT>::REC_K;
  asm volatile("" ::"s"(a.W), "s"(a.scales), "s"(a.X), "s"(a.Y), "s"(a.M), "s"(a.N), "s"(a.K), "s"(a.n_rec), "s"(a.x_stride),
               "s"(a.x_region), "s"(a.x_shift), "s"(a.n_strips), "s"(a.spw), "s"(a.rc), "s"(a.gn), "s"(a.gk), "s"(a.wps));
  const int tid = threadIdx.x, lane = tid & 63, nthr = blockDim.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int S = nthr >> 6;
  // workgroup = (position g along N, slice gk of K); without a split the grid is all along N
  const int G = a.gn;
  const int gk = a.gk > 1 ? (int)(blockIdx.x / (unsigned)G) : 0;
  const int g = (int)blockIdx.x - gk * G;
  const int ns = (a.n_strips - g + G - 1) / G;  // strips of this workgroup (>= 1)
  const int RC = a.rc;                          // records per strip in one phase of K
  // records [rec_lo, rec_hi) of every strip are this workgroup's slice of K
  const int rec_lo = a.gk > 1 ? (int)((unsigned)(gk * a.n_rec) / (unsigned)a.gk) : 0;
  const int rec_hi = a.gk > 1 ? (int)((unsigned)((gk + 1) * a.n_rec) / (unsigned)a.gk) : a.n_rec;
  const bool one_phase = RC >= rec_hi - rec_lo;
  const int mc = min(a.M, 16);  // activation rows of an MFMA tile that exist
  _Float16* xs = (_Float16*)smem;
  f4* parts = (f4*)(smem + (size_t)a.x_region * 2);  // [spw][wps][MT][4 K-quarters][mc]
  // The waves come in S / wps groups of wps; group vs owns the local strips vs, vs + sg, ...
  // and deals their records to its waves one by one (wps = S: all waves on one strip at a
  // time; fewer when the parked tiles, one per strip and wave of its group, must be fewer).
  // (GROUPS = false is the common case wps = S, spelled out so that it costs nothing.)
  const int wps = GROUPS ? a.wps : S;
  const int sg = GROUPS ? S / wps : 1;
  const int vs = GROUPS ? (int)((unsigned)wave / (unsigned)wps) : 0, vw = wave - vs * wps;
  const int ns_v = vs < ns ? (ns - vs + sg - 1) / sg : 0;  // strips of this wave's group
  // the group's j-th strip is local strip vs + j * sg = strip strip0 + j * strip_step of the
  // matrix; a group without strips reads (only reads) the workgroup's first strip
  const int strip0 = g + (ns_v > 0 ? vs : 0) * G, strip_step = (ns_v > 0 ? sg : 0) * G;
  const int m_lo = lane & 15, kq = lane >> 4;
  const int lane_off = FMT == FMT_FP16 ? 8 * kq : (REC_K / 4) * kq;
  // lanes whose activation row does not exist read row 0: they only feed output columns never stored
  const _Float16* x0 = xs + (m_lo < a.M ? m_lo : 0) * a.x_stride + lane_off;
  const _Float16* x1 = xs + (m_lo + 16 < a.M ? m_lo + 16 : 0) * a.x_stride + lane_off;
  const int part_f4 = MT * 4 * mc;  // f4 per parked tile
  // this wave's tile of its group's first strip; the next strips' tiles follow part_step apart
  f4* const my_part = parts + (size_t)((ns_v > 0 ? vs : 0) * wps + vw) * part_f4 + kq * mc + m_lo;
  const int part_step = sg * wps * part_f4;

  const bool vec_x = (a.K & 7) == 0;
  const int total_units = a.M << a.x_shift;
  const int units_per_pass = nthr * XUnit<FMT>::XU;
  const bool wave_has_x = vec_x && wave * 64 < total_units;  // wave-uniform
  const int chunk_k = RC * REC_K;
  __builtin_amdgcn_sched_barrier(0);

  // K is walked in phases of RC records per strip (one phase when all activations fit in LDS).
  for (int rec_base = rec_lo; rec_base < rec_hi; rec_base += RC) {
    const int n_rec = min(RC, rec_hi - rec_base);                 // records per strip in this phase
    const int total = ns_v * n_rec;                                  // records of this wave's group
    const int cnt = vw < total ? (total - vw + wps - 1) / wps : 0;  // records of this wave
    if (rec_base > rec_lo) __syncthreads();  // everyone is done with the previous phase's activations
    const int k0 = rec_base * REC_K;

    // Activations: units beyond the first pass (large M) and unaligned rows are staged by loops
    // that run to completion; the first pass is only requested here and stored behind the
    // head of the weight stream, so both are in flight together.
    XRegs<FMT> xr;
    if (vec_x) {
      for (int u0 = units_per_pass; u0 < total_units; u0 += nthr * XUnit<FMT>::XB) {
        XRegs<FMT, XUnit<FMT>::XB> xb;
        x_load(xb, a, k0, chunk_k, u0, tid, nthr);
        x_store(xb, xs, a, k0, chunk_k, u0, tid, nthr);
      }
    } else {
      stage_x_unaligned<FMT>(xs, a, k0, chunk_k, tid, nthr);
    }
    if (wave_has_x) x_load(xr, a, k0, chunk_k, 0, tid, nthr);
    __builtin_amdgcn_sched_barrier(0);

    // Head of the weight stream.  The prefetch cursor (position in the list, local strip,
    // record) stops at the wave's last record; a wave without records reads record 0.
    int pf = vw < total ? vw : 0, pj = 0, pr = pf;
    while (pr >= n_rec) pr -= n_rec, pj++;
    int cj = pj, cr = pr;  // strip (counted inside the group) and record (inside the phase) being multiplied

    // LR records are in flight while a record is being restored: the ring has one slot more,
    // and a step first requests the record LR places ahead into the slot freed by the step
    // before, then works on its own (a refill into the slot being read would have to wait
    // until the restoration has consumed it).
    constexpr int RS = LR + 1;
    struct Slot {
      LaneRec<FMT> r;
    };
    Slot ring[RS];
    auto request = [&](Slot& slot) {
      const int strip = strip0 + pj * strip_step;
      load_rec<FMT, false>(slot.r, a, strip, rec_base + pr, lane);
      if (pf + wps < total) {
        pf += wps, pr += wps;
        while (pr >= n_rec) pr -= n_rec, pj++;
      }
    };
#pragma unroll
    for (int q = 0; q < LR; q++) {
      request(ring[q]);
      __builtin_amdgcn_sched_barrier(0);  // issue in ring order: the oldest load is the first one needed
    }

    // while those are in flight: every tile slot cleared (a wave need not meet every strip when a
    // strip has fewer records than the workgroup has waves)
    if (rec_base == rec_lo)
      for (int i = tid; i < ns * wps * part_f4; i += nthr) parts[i] = f4{0, 0, 0, 0};
    if (wave_has_x) x_store(xr, xs, a, k0, chunk_k, 0, tid, nthr);
    __syncthreads();

    f4 acc[MT];
#pragma unroll
    for (int i = 0; i < MT; i++) acc[i] = f4{0, 0, 0, 0};
    bool pending = false;  // acc holds products that are not parked yet

    auto park = [&]() {
      if (m_lo < mc) {
        f4* t = my_part + cj * part_step;
        if (one_phase) {
#pragma unroll
          for (int i = 0; i < MT; i++) t[i * 4 * mc] = acc[i];
        } else {  // the slot belongs to this wave alone: a plain read-add-write
#pragma unroll
          for (int i = 0; i < MT; i++) t[i * 4 * mc] += acc[i];
        }
      }
#pragma unroll
      for (int i = 0; i < MT; i++) acc[i] = f4{0, 0, 0, 0};
    };
    // One record: request the one LR ahead, multiply, move on by S records; where that leaves
    // the strip, the tile is parked.  Only the request touches global memory.
    auto step = [&](Slot& slot, Slot& free_slot) {
      request(free_slot);
      __builtin_amdgcn_sched_barrier(0);
      mac_rec<FMT, MT>(slot.r, x0 + cr * REC_K, x1 + cr * REC_K, acc);
      pending = true;
      cr += wps;
      if (cr >= n_rec) {
        park();
        pending = false;
        do {
          cr -= n_rec, cj++;
        } while (cr >= n_rec);
      }
    };

    int i = 0;
    for (; i + RS <= cnt; i += RS) {
#pragma unroll
      for (int q = 0; q < RS; q++) {
        step(ring[q], ring[(q + LR) % RS]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
#pragma unroll
    for (int q = 0; q < RS - 1; q++)
      if (i + q < cnt) step(ring[q], ring[(q + LR) % RS]);
    if (pending) park();
  }

  // Finish the strips, one per wave: the wps parked tiles added in wave order.
  __syncthreads();
  for (int j = wave; j < ns; j += S) {
    f4 sum[MT];
#pragma unroll
    for (int t = 0; t < MT; t++) sum[t] = f4{0, 0, 0, 0};
    if (m_lo < mc) {
      const f4* t0 = parts + (size_t)j * wps * part_f4 + kq * mc + m_lo;
      for (int w = 0; w < wps; w++) {
#pragma unroll
        for (int t = 0; t < MT; t++) sum[t] += t0[(size_t)w * part_f4 + t * 4 * mc];
      }
    }
    const int strip = g + j * G;
    if (a.gk > 1) {
      // K is split over gk workgroups: every one leaves its partial tile in the workspace and
      // counts itself in; the one that arrives last adds all gk tiles in slice order (so the
      // result does not depend on who was last), finishes the strip and clears the counter
      // for the next call.  Nobody waits for anybody.
      // The tiles travel as device-scope relaxed atomic stores and loads (they go to the level
      // of the memory system all compute units share).  What orders them: the wave waits until
      // every one of its tile stores has been acknowledged (s_waitcnt vmcnt(0): on this target
      // stores count in vmcnt) before it counts itself in, and the last arriver's tile loads are
      // issued only after its own count has come back (the branch below depends on it).  A
      // device-scope fence would instead write back and invalidate the whole L2, which costs
      // more than the Linear itself.
      float* wt = (float*)(a.ws_tiles + ((size_t)gk * a.n_strips + strip) * MT * 64 + lane);
#pragma unroll
      for (int t = 0; t < MT; t++)
#pragma unroll
        for (int r = 0; r < 4; r++) __hip_atomic_store(wt + t * 256 + r, sum[t][r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      // all tile stores of this wave acknowledged; the compiler moves no memory access across either statement
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      unsigned before = 0;
      if (lane == 0) before = __hip_atomic_fetch_add(a.ws_count + strip, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      before = __builtin_amdgcn_readfirstlane(before);
      if (before != (unsigned)a.gk - 1) continue;
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the count has returned; the tile loads below are issued after it
#pragma unroll
      for (int t = 0; t < MT; t++) sum[t] = f4{0, 0, 0, 0};
      for (int q = 0; q < a.gk; q++) {
        const float* rt = (const float*)(a.ws_tiles + ((size_t)q * a.n_strips + strip) * MT * 64 + lane);
#pragma unroll
        for (int t = 0; t < MT; t++)
#pragma unroll
          for (int r = 0; r < 4; r++) sum[t][r] += __hip_atomic_load(rt + t * 256 + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      if (lane == 0) __hip_atomic_store(a.ws_count + strip, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    store_tile_scaled<MT>(sum, f4{1.0f, 1.0f, 1.0f, 1.0f}, a, strip, lane);  // the baseline has no scales
  }
}

// The fp16 baseline at small batches (Sec. 4.2's W16A16 GEMV): every wavefront owns whole rows of the
// row-major matrix, dealt round robin over all wavefronts of the grid, and reads a row as consecutive
// 1 KiB segments (one 16-byte load per lane, LR of them in flight), multiplies on the VALU (packed dot
// products into fp32, the lane's eight channels against the same eight of each activation row in LDS)
// and adds the 64 lanes of a row up when the row ends.  a.x_stride = halfs between activation rows in
// LDS (K rounded up to whole segments; the tail is zero).  K is a multiple of 8.
template <int MB, bool NT>
__global__ void __launch_bounds__(1024) gemv_fp16_kernel(LinearArgs a) {
  extern __shared__ __align__(16) uint8_t smem[];
  typedef _Float16 h2 __attribute__((ext_vector_type(2)));
  constexpr int LR = 2, RS = LR + 1, SEG = 512;  // halfs of a row one wavefront load covers
  _Float16* xs = (_Float16*)smem;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_seg = (a.K + SEG - 1) / SEG;
  const int kpad = a.x_stride;
  for (int u = tid; u < MB * (kpad / 8); u += 1024) {
    const int m = u / (kpad / 8), k = 8 * (u - m * (kpad / 8));
    u4 v = u4{0, 0, 0, 0};
    if (k < a.K) v = *(const u4*)(a.X + (size_t)m * a.K + k);
    *(u4*)(xs + (size_t)m * kpad + k) = v;
  }
  __syncthreads();

  const int n_waves = gridDim.x * 16;
  const int first = __builtin_amdgcn_readfirstlane(blockIdx.x * 16 + wave);  // this wave's first row
  const int n_rows = first < a.N ? (a.N - first + n_waves - 1) / n_waves : 0;
  const int total = n_rows * n_seg;  // segments this wave reads, row after row
  if (total == 0) return;
  const _Float16* W = (const _Float16*)a.W;
  u4 ring[RS];
  int rq = 0;  // next segment to request (clamped to the last: requests past the end are ignored)
  auto request = [&](u4& slot) {
    const int c = min(rq, total - 1);
    const int ri = c / n_seg, seg = c - ri * n_seg;
    const int k = seg * SEG + 8 * lane;
    const bool ok = k < a.K;
    const u4* p = (const u4*)(W + (size_t)(first + ri * n_waves) * a.K + (ok ? k : 0));
    const u4 v = NT ? __builtin_nontemporal_load(p) : *p;
    const uint32_t keep = ok ? 0xFFFFFFFFu : 0u;  // lanes beyond K re-read the row's start and drop it
    slot = u4{v[0] & keep, v[1] & keep, v[2] & keep, v[3] & keep};
    rq++;
  };
#pragma unroll
  for (int q = 0; q < LR; q++) {
    request(ring[q]);
    __builtin_amdgcn_sched_barrier(0);
  }
  float acc[MB];
#pragma unroll
  for (int m = 0; m < MB; m++) acc[m] = 0.0f;
  int row = first, seg = 0;
  auto step = [&](u4& slot, u4& free_slot) {
    request(free_slot);
    __builtin_amdgcn_sched_barrier(0);
    const h8 w = __builtin_bit_cast(h8, slot);
    const _Float16* x = xs + seg * SEG + 8 * lane;
#pragma unroll
    for (int m = 0; m < MB; m++) {
      const h8 xv = *(const h8*)(x + (size_t)m * kpad);
#pragma unroll
      for (int q = 0; q < 4; q++) acc[m] = __builtin_amdgcn_fdot2(h2{w[2 * q], w[2 * q + 1]}, h2{xv[2 * q], xv[2 * q + 1]}, acc[m], false);
    }
    if (++seg == n_seg) {  // the row is complete: add its 64 lanes up and store
#pragma unroll
      for (int m = 0; m < MB; m++) {
        float v = acc[m];
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
        if (lane == 0) a.Y[(size_t)m * a.N + row] = __builtin_bit_cast(uint16_t, (_Float16)v);
        acc[m] = 0.0f;
      }
      seg = 0;
      row += n_waves;
    }
  };
  int i = 0;
  for (; i + RS <= total; i += RS) {
#pragma unroll
    for (int q = 0; q < RS; q++) {
      step(ring[q], ring[(q + LR) % RS]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#pragma unroll
  for (int q = 0; q < RS - 1; q++)
    if (i + q < total) step(ring[q], ring[(q + LR) % RS]);
}

// Finish one strip with the complete tile of this workgroup's slice of K: times the scales, converted, stored; with
// K split over gk workgroups, through the workspace.
template <int MT>
__device__ __forceinline__ void finish_strip(const LinearArgs& a, int gk, int out_strip, f4 (&sum)[MT], const f4 sc, int lane) {
  if (a.gk > 1) {
    // K is split over gk workgroups: every one leaves its partial tile in the workspace and
    // counts itself in; the one that arrives last adds all gk tiles in slice order (so the
    // result does not depend on who was last), finishes the strip and clears the counter
    // for the next call.  Nobody waits for anybody.
    // The tiles travel as device-scope relaxed atomic stores and loads (they go to the level
    // of the memory system all compute units share).  What orders them: the wave waits until
    // every one of its tile stores has been acknowledged (s_waitcnt vmcnt(0): on this target
    // stores count in vmcnt) before it counts itself in, and the last arriver's tile loads are
    // issued only after its own count has come back (the branch below depends on it).  A
    // device-scope fence would instead write back and invalidate the whole L2, which costs
    // more than the Linear itself.
    float* wt = (float*)(a.ws_tiles + ((size_t)gk * a.n_strips + out_strip) * MT * 64 + lane);
#pragma unroll
    for (int t = 0; t < MT; t++)
#pragma unroll
      for (int r = 0; r < 4; r++) __hip_atomic_store(wt + t * 256 + r, sum[t][r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // all tile stores of this wave acknowledged; the compiler moves no memory access across either statement
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    unsigned before = 0;
    if (lane == 0) before = __hip_atomic_fetch_add(a.ws_count + out_strip, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    before = __builtin_amdgcn_readfirstlane(before);
    if (before != (unsigned)a.gk - 1) return;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the count has returned; the tile loads below are issued after it
#pragma unroll
    for (int t = 0; t < MT; t++) sum[t] = f4{0, 0, 0, 0};
    for (int q = 0; q < a.gk; q++) {
      const float* rt = (const float*)(a.ws_tiles + ((size_t)q * a.n_strips + out_strip) * MT * 64 + lane);
#pragma unroll
      for (int t = 0; t < MT; t++)
#pragma unroll
        for (int r = 0; r < 4; r++) sum[t][r] += __hip_atomic_load(rt + t * 256 + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (lane == 0) __hip_atomic_store(a.ws_count + out_strip, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  store_tile_scaled<MT>(sum, sc, a, out_strip, lane);
}

// The Linear on packed weights.  A workgroup owns up to 16 neighbouring strips (spw of them,
// one resident round of workgroups; more strips than 16 x 256 just means more workgroups) and
// has S / spw wavefronts on each: a wavefront stays with its strip and takes every wps-th
// record of it, in step with all other wavefronts of the grid.  With the K-major packed layout
// the grid as a whole then reads one contiguous window of memory that moves through the
// matrix front to back (measured with bare read kernels under a realistic amount of per-record
// arithmetic: 10-20 % faster than strips that are read as separate streams).  A strip's
// partial tile stays in its wavefront's accumulator registers for the whole of K, also across
// the phases K is walked in when the activations M x K do not fit in LDS; at the end the wps
// tiles of a strip are added in wave order through LDS (deterministic, no atomics), scaled,
// converted and stored; a wavefront that is alone on its strip (wps = 1) finishes it straight
// from its accumulators.  Each wave keeps LR records in flight beside the one it is restoring
// (two with 16 wavefronts per workgroup, three with 8: the host decides which).
// QD (formats with side bits): the records are dealt to a strip's wavefronts in whole side groups,
// so that a group's side dword is loaded once per group and not once per record; used where the
// groups of a phase divide evenly enough among the wavefronts (the host decides).
template <int FMT, int MT, bool NT, bool GS, bool QD = false, int LR = 2>
__global__ void __launch_bounds__(1024) column_kernel(LinearArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int REC_K = Fmt<FMT>::REC_K, SG = Fmt<FMT>::SG, RS = LR + 1;
  // the side-group deal has a ring of four slots and two side registers: a request must stay within the group after
  // the one being multiplied
  static_assert(!QD || LR == 2 || (LR == 3 && SG == 4), "records ahead in the side-group deal");
  asm volatile("" ::"s"(a.W), "s"(a.scales), "s"(a.X), "s"(a.Y), "s"(a.M), "s"(a.N), "s"(a.K), "s"(a.n_rec), "s"(a.x_stride),
               "s"(a.x_region), "s"(a.x_shift), "s"(a.n_strips), "s"(a.spw), "s"(a.rc), "s"(a.gn), "s"(a.gk), "s"(a.wps));
  const int tid = threadIdx.x, lane = tid & 63, nthr = blockDim.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int S = nthr >> 6;
  // workgroup = (position g along N, slice gk of K); without a split the grid is all along N
  const int G = a.gn;
  const int gk = a.gk > 1 ? (int)(blockIdx.x / (unsigned)G) : 0;
  const int g = (int)blockIdx.x - gk * G;
  const int s_first = g * a.spw;                      // this workgroup's strips: s_first .. s_first + ns - 1
  const int ns = min(a.spw, a.n_strips - s_first);    // >= 1
  const int wps = a.wps;                              // wavefronts per strip
  const int wj = (int)((unsigned)wave / (unsigned)wps), wk = wave - wj * wps;  // this wave: strip wj of the workgroup, lane wk of its K deal
  const bool has_strip = wj < ns && wk < a.wpa;
  const int strip = s_first + (wj < ns ? wj : 0);
  // records [rec_lo, rec_hi) of every strip are this workgroup's slice of K
  const int rec_lo = a.gk > 1 ? (int)((unsigned)(gk * a.n_rec) / (unsigned)a.gk) : 0;
  const int rec_hi = a.gk > 1 ? (int)((unsigned)((gk + 1) * a.n_rec) / (unsigned)a.gk) : a.n_rec;
  const int RC = a.rc;  // records per strip in one phase of K
  const int mc = min(a.M, 16);  // activation rows of an MFMA tile that exist
  _Float16* xs = (_Float16*)smem;
  f4* parts = (f4*)(smem + (size_t)a.x_region * 2);  // [spw][wps][MT][4 K-quarters][mc]
  const int m_lo = lane & 15, kq = lane >> 4;
  const int lane_off = (REC_K / 4) * kq;
  // lanes whose activation row does not exist read row 0: they only feed output columns never stored
  const _Float16* x0 = xs + (m_lo < a.M ? m_lo : 0) * a.x_stride + lane_off;
  const _Float16* x1 = xs + (m_lo + 16 < a.M ? m_lo + 16 : 0) * a.x_stride + lane_off;
  const int part_f4 = MT * 4 * mc;  // f4 per parked tile

  const bool vec_x = (a.K & 7) == 0;
  const int total_units = a.M << a.x_shift;
  const int units_per_pass = nthr * XUnit<FMT>::XU;
  const bool wave_has_x = vec_x && wave * 64 < total_units;  // wave-uniform
  const int chunk_k = RC * REC_K;
  // Scales of the strip this wave finishes (wave w finishes strip w of the workgroup): requested first, kept as raw
  // bits until the epilogue.  (With one scale per run of input channels, GS, the scales travel with the records.)
  ScaleBits scale0_bits = {{0x3C00, 0x3C00, 0x3C00, 0x3C00}};
  if constexpr (!GS) scale0_bits = load_scale_bits<FMT>(a, min(s_first + min(wave, ns - 1), a.n_strips - 1), lane);
  __builtin_amdgcn_sched_barrier(0);

  f4 acc[MT];
#pragma unroll
  for (int i = 0; i < MT; i++) acc[i] = f4{0, 0, 0, 0};

  // K is walked in phases of RC records per strip (one phase when all activations fit in LDS).
  for (int rec_base = rec_lo; rec_base < rec_hi; rec_base += RC) {
    const int n_rec = min(RC, rec_hi - rec_base);                                    // records per strip in this phase
    const int cnt = (has_strip && wk < n_rec) ? (n_rec - wk + wps - 1) / wps : 0;  // records of this wave
    if (rec_base > rec_lo) __syncthreads();  // everyone is done with the previous phase's activations
    const int k0 = rec_base * REC_K;

    // Activations: units beyond the first pass (large M) and unaligned rows are staged by loops
    // that run to completion; the first pass is only requested here and stored behind the
    // head of the weight stream, so both are in flight together.
    XRegs<FMT> xr;
    if (vec_x) {
      for (int u0 = units_per_pass; u0 < total_units; u0 += nthr * XUnit<FMT>::XB) {
        XRegs<FMT, XUnit<FMT>::XB> xb;
        x_load(xb, a, k0, chunk_k, u0, tid, nthr);
        x_store(xb, xs, a, k0, chunk_k, u0, tid, nthr);
      }
    } else {
      stage_x_unaligned<FMT>(xs, a, k0, chunk_k, tid, nthr);
    }
    if (wave_has_x) x_load(xr, a, k0, chunk_k, 0, tid, nthr);
    __builtin_amdgcn_sched_barrier(0);

    if constexpr (QD) {
      // Side groups dealt whole: the wave's records are its groups wk, wk + wpa, ... of the phase, member by
      // member.  Two groups per unrolled round, so that the ring slot of a record (its number mod 4), the side
      // register of its group (the group's number mod 2) and its place in the side dword are all fixed in the
      // code.  LR = 2 records ahead as above; a group's side dword is requested with its first record.
      constexpr int UN = 2 * SG;
      const int n_grp = (n_rec + SG - 1) / SG;  // the phase starts on a group boundary; a last group may run into the padding records
      const int wpa = a.wpa;
      const int cnt_g = (has_strip && wk < n_grp) ? (n_grp - wk + wpa - 1) / wpa : 0;
      const int total_e = cnt_g * SG, e_last = max(total_e - 1, 0);
      const int g_first = cnt_g > 0 ? wk : 0;
      LaneRec<FMT> ring[4];
      uint32_t side[2] = {0, 0};
      // e-th record of this wave (clamped to its last): group g_first + (e / SG) * wpa, member e % SG
      auto request = [&](int e, LaneRec<FMT>& slot, uint32_t& side_reg, bool with_side) {
        e = min(e, e_last);
        const int grp = rec_base / SG + g_first + (e / SG) * wpa;
        const uint8_t* unit = a.W + ((size_t)grp * a.n_strips + strip) * Fmt<FMT>::UNIT;
        load_lane_rec<FMT, NT, false>(slot, unit + (e % SG) * Fmt<FMT>::CB, nullptr, lane);
        if (with_side) {
          const uint32_t* sp = (const uint32_t*)(unit + SG * Fmt<FMT>::CB) + lane;
          side_reg = NT ? __builtin_nontemporal_load(sp) : *sp;
        }
      };
#pragma unroll
      for (int q = 0; q < LR; q++) {
        request(q, ring[q], side[(q / SG) & 1], q % SG == 0);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (wave_has_x) x_store(xr, xs, a, k0, chunk_k, 0, tid, nthr);
      __syncthreads();

      int rel = g_first * SG;  // first record of the group being multiplied, relative to the phase
      auto round_of = [&](int b, auto n_steps) {
#pragma unroll
        for (int u = 0; u < decltype(n_steps)::value; u++) {
          request(b + u + LR, ring[(u + LR) & 3], side[((u + LR) / SG) & 1], (u + LR) % SG == 0);
          __builtin_amdgcn_sched_barrier(0);
          LaneRec<FMT> cur = ring[u & 3];
          cur.t = side[(u / SG) & 1];
          const int kk = (rel + u % SG) * REC_K;
          mac_rec<FMT, MT>(cur, x0 + kk, x1 + kk, acc, 8 * Fmt<FMT>::SIDE * (u % SG));
          if (u % SG == SG - 1) rel += wpa * SG;
          __builtin_amdgcn_sched_barrier(0);
        }
      };
      int b = 0;
      for (; b + UN <= total_e; b += UN) round_of(b, std::integral_constant<int, UN>{});
      if (b < total_e) round_of(b, std::integral_constant<int, SG>{});  // an odd last group
    } else {
      // LR records are in flight while a record is being restored: the ring has one slot more,
      // and a step first requests the record LR places ahead into the slot freed by the step
      // before, then works on its own.  The request cursor stops at the wave's last record (a
      // wave without records requests, and ignores, the phase's first record of its strip).
      struct Slot {
        LaneRec<FMT> r;
        us4 gs;  // GS: the scales of this lane's four output channels for the record's run
      };
      Slot ring[RS];
      int pr = rec_base + (cnt > 0 ? wk : 0);                       // record the next request fetches
      const int pr_last = rec_base + (cnt > 0 ? wk + (cnt - 1) * wps : 0);
      auto request = [&](Slot& slot) {
        load_rec<FMT, NT>(slot.r, a, strip, pr, lane);
        if constexpr (GS)  // 8 bytes, the same for the 16 lanes of a K-quarter; cached: a run spans many records
          slot.gs = *(const us4*)(a.scales + ((size_t)strip * a.n_sg + (pr >> a.sg_shift)) * 16 + 4 * kq);
        pr = min(pr + wps, pr_last);
      };
  #pragma unroll
      for (int q = 0; q < LR; q++) {
        request(ring[q]);
        __builtin_amdgcn_sched_barrier(0);  // issue in ring order: the oldest load is the first one needed
      }
      if (wave_has_x) x_store(xr, xs, a, k0, chunk_k, 0, tid, nthr);
      __syncthreads();

      // One record: request the one LR ahead, restore, multiply, move on by wps records.
      int cr = wk;  // record being multiplied, relative to the phase
      auto step = [&](Slot& slot, Slot& free_slot) {
        request(free_slot);
        __builtin_amdgcn_sched_barrier(0);
        const int side_shift = 8 * Fmt<FMT>::SIDE * ((rec_base + cr) & (SG - 1));
        if constexpr (GS) {  // the record's own tile, times its run's scales (Eq. 2), then into the sum
          f4 t[MT];
  #pragma unroll
          for (int i = 0; i < MT; i++) t[i] = f4{0, 0, 0, 0};
          mac_rec<FMT, MT>(slot.r, x0 + cr * REC_K, x1 + cr * REC_K, t, side_shift);
          f4 sc;
  #pragma unroll
          for (int r = 0; r < 4; r++) sc[r] = (float)__builtin_bit_cast(_Float16, (uint16_t)slot.gs[r]);
  #pragma unroll
          for (int i = 0; i < MT; i++) acc[i] += t[i] * sc;
        } else {
          mac_rec<FMT, MT>(slot.r, x0 + cr * REC_K, x1 + cr * REC_K, acc, side_shift);
        }
        cr += wps;
      };
      int i = 0;
      for (; i + RS <= cnt; i += RS) {
  #pragma unroll
        for (int q = 0; q < RS; q++) {
          step(ring[q], ring[(q + LR) % RS]);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
  #pragma unroll
      for (int q = 0; q < RS - 1; q++)
        if (i + q < cnt) step(ring[q], ring[(q + LR) % RS]);
    }
  }

  // Finish strip j of the workgroup with its complete tile of this workgroup's slice of K.
  auto finish = [&](int j, f4 (&sum)[MT]) {
    const int out_strip = s_first + j;
    f4 sc;
    if constexpr (GS)
      sc = f4{kTwo14, kTwo14, kTwo14, kTwo14};
    else
      sc = j == wave ? scales_from_bits(scale0_bits, kTwo14) : load_scales<FMT>(a, out_strip, lane);
    finish_strip<MT>(a, gk, out_strip, sum, sc, lane);
  };
  // A wavefront that is alone on its strip finishes it straight from its accumulators.
  if (wps == 1) {
    if (wj < ns) finish(wj, acc);
    return;
  }
  // Otherwise one wave per strip adds the wps tiles of the strip in wave order, through LDS.
  if (wj < ns && m_lo < mc) {  // idle wavefronts of a strip leave a tile of zeros
    f4* t = parts + (size_t)(wj * wps + wk) * part_f4 + kq * mc + m_lo;
#pragma unroll
    for (int i = 0; i < MT; i++) t[i * 4 * mc] = acc[i];
  }
  __syncthreads();
  for (int j = wave; j < ns; j += S) {
    f4 sum[MT];
#pragma unroll
    for (int t = 0; t < MT; t++) sum[t] = f4{0, 0, 0, 0};
    if (m_lo < mc) {
      const f4* t0 = parts + (size_t)j * wps * part_f4 + kq * mc + m_lo;
      for (int w = 0; w < wps; w++) {
#pragma unroll
        for (int t = 0; t < MT; t++) sum[t] += t0[(size_t)w * part_f4 + t * 4 * mc];
      }
    }
    finish(j, sum);
  }
}

// The Linear on packed weights where a workgroup owns more strips than it has wavefronts: eight wavefronts, each
// alone on NS strips of the workgroup (wave w on strips w, w + wn, ...; wn = a.wpa wavefronts own strips), which it
// walks record by record side by side (record r of its first strip, record r of its second, record r + 1 ...), one
// accumulator tile per strip, three records ahead in a ring of four.  All strips of the workgroup are still read
// at the same record index at the same time (the contiguous window of the column kernel), the activations are
// staged as there, and every strip is finished straight from its wavefront's accumulators: no tiles in LDS, no
// barrier after the last record.  For the formats whose records carry no side groups (with the side groups of two
// strips dealt in turn FP4.25 was 1-3 % slower than with sixteen wavefronts on one strip each: measured, not kept).
template <int FMT, int MT, bool NT, int NS>
__global__ void __launch_bounds__(512) multi_kernel(LinearArgs a) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  constexpr int REC_K = Fmt<FMT>::REC_K, SG = Fmt<FMT>::SG, LR = 3;
  static_assert(NS == 2 || NS == 4, "strips per wavefront: the ring of four must hold whole rounds of them");
  asm volatile("" ::"s"(a.W), "s"(a.scales), "s"(a.X), "s"(a.Y), "s"(a.M), "s"(a.N), "s"(a.K), "s"(a.n_rec), "s"(a.x_stride),
               "s"(a.x_region), "s"(a.x_shift), "s"(a.n_strips), "s"(a.spw), "s"(a.rc), "s"(a.gn), "s"(a.gk), "s"(a.wpa));
  const int tid = threadIdx.x, lane = tid & 63, nthr = blockDim.x;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int G = a.gn;
  const int gk = a.gk > 1 ? (int)(blockIdx.x / (unsigned)G) : 0;
  const int g = (int)blockIdx.x - gk * G;
  const int s_first = g * a.spw;
  const int ns = min(a.spw, a.n_strips - s_first);  // >= 1
  const int wn = a.wpa;                             // wavefronts that own strips
  const bool has_strip = wave < wn && wave < ns;
  int sidx[NS];    // this wave's strips (those that do not exist stand for the workgroup's last: read, never finished)
  bool valid[NS];
#pragma unroll
  for (int i = 0; i < NS; i++) {
    valid[i] = wave < wn && wave + i * wn < ns;
    sidx[i] = s_first + min(wave + i * wn, ns - 1);
  }
  const int rec_lo = a.gk > 1 ? (int)((unsigned)(gk * a.n_rec) / (unsigned)a.gk) : 0;
  const int rec_hi = a.gk > 1 ? (int)((unsigned)((gk + 1) * a.n_rec) / (unsigned)a.gk) : a.n_rec;
  const int RC = a.rc;
  _Float16* xs = (_Float16*)smem;
  const int m_lo = lane & 15, kq = lane >> 4;
  const int lane_off = (REC_K / 4) * kq;
  const _Float16* x0 = xs + (m_lo < a.M ? m_lo : 0) * a.x_stride + lane_off;
  const _Float16* x1 = xs + (m_lo + 16 < a.M ? m_lo + 16 : 0) * a.x_stride + lane_off;
  const bool vec_x = (a.K & 7) == 0;
  const int total_units = a.M << a.x_shift;
  const int units_per_pass = nthr * XUnit<FMT>::XU;
  const bool wave_has_x = vec_x && wave * 64 < total_units;  // wave-uniform
  const int chunk_k = RC * REC_K;
  ScaleBits sb[NS];
#pragma unroll
  for (int i = 0; i < NS; i++) sb[i] = load_scale_bits<FMT>(a, sidx[i], lane);
  __builtin_amdgcn_sched_barrier(0);

  f4 acc[NS][MT];
#pragma unroll
  for (int i = 0; i < NS; i++)
#pragma unroll
    for (int t = 0; t < MT; t++) acc[i][t] = f4{0, 0, 0, 0};

  for (int rec_base = rec_lo; rec_base < rec_hi; rec_base += RC) {
    const int n_rec = min(RC, rec_hi - rec_base);
    if (rec_base > rec_lo) __syncthreads();  // everyone is done with the previous phase's activations
    const int k0 = rec_base * REC_K;
    XRegs<FMT> xr;
    if (vec_x) {
      for (int u0 = units_per_pass; u0 < total_units; u0 += nthr * XUnit<FMT>::XB) {
        XRegs<FMT, XUnit<FMT>::XB> xb;
        x_load(xb, a, k0, chunk_k, u0, tid, nthr);
        x_store(xb, xs, a, k0, chunk_k, u0, tid, nthr);
      }
    } else {
      stage_x_unaligned<FMT>(xs, a, k0, chunk_k, tid, nthr);
    }
    if (wave_has_x) x_load(xr, a, k0, chunk_k, 0, tid, nthr);
    __builtin_amdgcn_sched_barrier(0);

    LaneRec<FMT> ring[4];
    {
      // records e = 0 .. NS * n_rec - 1 of the phase: strip e % NS, record e / NS
      const int total_e = has_strip ? NS * n_rec : 0;
      int qr = 0;  // record of the next request, relative to the phase (stops at the last)
      auto request = [&](LaneRec<FMT>& slot, int i) {
        load_rec<FMT, NT>(slot, a, sidx[i], rec_base + min(qr, n_rec - 1), lane);
        if (i == NS - 1) qr++;
      };
#pragma unroll
      for (int q = 0; q < LR; q++) {
        request(ring[q], q % NS);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (wave_has_x) x_store(xr, xs, a, k0, chunk_k, 0, tid, nthr);
      __syncthreads();
      int cr = 0;  // record being multiplied, relative to the phase
      auto step = [&](auto uc) {
        constexpr int u = decltype(uc)::value;
        request(ring[(u + LR) & 3], (u + LR) % NS);
        __builtin_amdgcn_sched_barrier(0);
        const int side_shift = 8 * Fmt<FMT>::SIDE * ((rec_base + cr) & (SG - 1));
        mac_rec<FMT, MT>(ring[u & 3], x0 + cr * REC_K, x1 + cr * REC_K, acc[u % NS], side_shift);
        if (u % NS == NS - 1) cr++;
        __builtin_amdgcn_sched_barrier(0);
      };
      int e = 0;
      for (; e + 4 <= total_e; e += 4) {
        step(std::integral_constant<int, 0>{});
        step(std::integral_constant<int, 1>{});
        step(std::integral_constant<int, 2>{});
        step(std::integral_constant<int, 3>{});
      }
      if (e < total_e) {  // NS = 2 and an odd number of records: one more of each strip
        step(std::integral_constant<int, 0>{});
        step(std::integral_constant<int, 1>{});
      }
    }
  }

#pragma unroll
  for (int i = 0; i < NS; i++)
    if (valid[i]) finish_strip<MT>(a, gk, sidx[i], acc[i], scales_from_bits(sb[i], kTwo14), lane);
}

// Restore a whole packed matrix to row-major fp16: one wavefront per record.
template <int FMT>
__global__ void __launch_bounds__(256) dequant_kernel(const uint8_t* W, const uint16_t* scales, uint16_t* out, int N, int K,
                                                      int n_rec, int64_t total_recs, int scaled, int n_sg, int sg_shift) {
  const int lane = threadIdx.x & 63;
  const int64_t rec_id = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (rec_id >= total_recs) return;
  const int strip = (int)(rec_id / n_rec), rec = (int)(rec_id - (int64_t)strip * n_rec);
  constexpr int SG = Fmt<FMT>::SG;
  const int64_t n_strips = (N + 15) / 16;
  const uint8_t* unit = W + ((size_t)(rec / SG) * n_strips + strip) * Fmt<FMT>::UNIT;
  LaneRec<FMT> r;
  load_lane_rec<FMT, false>(r, unit + (rec % SG) * Fmt<FMT>::CB, unit + SG * Fmt<FMT>::CB, lane);
  const int n = strip * 16 + (lane & 15);
  if (n >= N) return;
  float mul = kTwo14;
  // one scale per row (sg_shift < 0) or per run of 2^sg_shift records: [strip][run][row in strip]
  if (scaled) mul *= (float)__builtin_bit_cast(_Float16, sg_shift < 0 ? scales[n] : scales[((size_t)strip * n_sg + (rec >> sg_shift)) * 16 + (lane & 15)]);
  const int kbase = rec * Fmt<FMT>::REC_K + (lane >> 4) * (Fmt<FMT>::REC_K / 4);
  auto put = [&](int k, uint32_t bits16) {
    if (k < K) {
      // magnitude and sign apart: the exact product is rounded once, and a negative
      // zero code keeps its sign (a fused multiply-add with +0 would drop it)
      const float v = (float)__builtin_bit_cast(_Float16, (uint16_t)(bits16 & 0x7FFF)) * mul;
      out[(size_t)n * K + k] = (uint16_t)(__builtin_bit_cast(uint16_t, (_Float16)v) | (bits16 & 0x8000));
    }
  };
  uint32_t o[4 * Fmt<FMT>::N_MFMA];
  restore_rec<FMT>(r, 8 * Fmt<FMT>::SIDE * (rec % SG), o);
  constexpr int PB = Fmt<FMT>::PB;
#pragma unroll
  for (int m = 0; m < 4 * Fmt<FMT>::N_MFMA; m++) {
    // pair m = operand slots 2m and 2m+1 of the lane chunk
    const int blk = (2 * m) / PB * PB;
    put(kbase + blk + slot_channel<FMT>(2 * m - blk), o[m] & 0xFFFF);
    put(kbase + blk + slot_channel<FMT>(2 * m + 1 - blk), o[m] >> 16);
  }
}

// Measurement aid: reads n_rec records of 1 KiB and discards them.  Record r goes to
// wavefront r mod (all wavefronts of the grid), two records in flight per wave: the
// fastest read order found on this GPU, the ceiling the Linear kernels are compared with.
__global__ void __launch_bounds__(1024) read_probe_kernel(const u4* __restrict__ p, int64_t n_rec, uint32_t* sink) {
  const int lane = threadIdx.x & 63;
  const int S = blockDim.x >> 6;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t first = (int64_t)blockIdx.x * S + wave, step = (int64_t)gridDim.x * S;
  // nothing to read (the launch-floor mode) or no record for this wave: no load at all
  if (first >= n_rec) return;
  const int64_t last = n_rec - 1;  // >= 0 here; every index below is clamped into [0, last]
  u4 ring[2];
  uint32_t acc = 0;
#pragma unroll
  for (int i = 0; i < 2; i++) ring[i] = __builtin_nontemporal_load(p + min(first + i * step, last) * 64 + lane);
  for (int64_t r = first; r < n_rec; r += 2 * step) {
#pragma unroll
    for (int i = 0; i < 2; i++) {
      const u4 v = ring[i];
      ring[i] = __builtin_nontemporal_load(p + min(r + (i + 2) * step, last) * 64 + lane);
      if (r + i * step < n_rec) acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
    }
  }
  if (acc == 0x9E3779B9u && sink) sink[0] = acc;  // keeps the loads alive; practically never true
}

// ---- host-side launch logic -------------------------------------------------
constexpr int kLdsMaxBytes = 160 * 1024;  // LDS of a gfx950 compute unit

// activations are staged in units of one permutation block
int x_unit(int fmt) { return fmt == FMT_FP16 ? 8 : ams::kFormats[fmt].perm_block; }

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

constexpr int kNumCU = 256;             // MI355X compute units
constexpr int kStreamLdsMax = kLdsMaxBytes;  // one workgroup per compute unit: all of it (measured: the phases of K this saves pay)

struct StreamPlan {
  bool ok;
  int S, lr, spw, grid, rc, x_shift, x_stride, x_region, red_slots;
  size_t lds;
};

// Launch shape of the streaming kernel: one workgroup of 16 wavefronts per CU, each
// owning an equal run of whole strips; K is walked in as few phases as the LDS allows
// (activations of a phase: M x rc records; plus the waves' tile slots).
StreamPlan make_stream_plan(int fmt, int M, int64_t n_strips, int n_rec, int rec_k) {
  StreamPlan p;
  const int mt = M > 16 ? 2 : 1;
  // strips per workgroup: one resident round, but at most 32 (a wave parks one tile per strip it touches)
  p.spw = (int)std::min<int64_t>(32, (n_strips + kNumCU - 1) / kNumCU);
  p.grid = (int)((n_strips + p.spw - 1) / p.spw);
  p.ok = false;
  for (int n_phase = 1; n_phase <= n_rec; n_phase++) {
    const int rc = (n_rec + n_phase - 1) / n_phase;
    if (n_phase > 1 && rc == (n_rec + n_phase - 2) / (n_phase - 1)) continue;  // same rc as before
    const int64_t P = (int64_t)p.spw * rc;
    const int S = (int)std::min<int64_t>(16, std::max<int64_t>(1, P));
    const int per_wave_max = (int)((P + S - 1) / S);
    const int slots = (per_wave_max - 1) / rc + 2;
    const int x_stride = rc * rec_k + 8;  // +8 halfs: consecutive rows start 16 bytes apart in the banks
    const size_t lds = (size_t)M * x_stride * 2 + (size_t)S * slots * mt * 64 * 16;
    if (lds > (size_t)kStreamLdsMax) continue;
    p.ok = true;
    p.rc = rc;
    p.S = S;
    p.red_slots = slots;
    p.x_stride = x_stride;
    p.x_region = M * x_stride;
    p.lds = lds;
    // measured on the Llama-8B/70B shapes: deeper rings only lengthen the drain at the end of the stream
    p.lr = fmt == FMT_FP16 ? 2 : 4;  // the baseline's records are four times larger
    while (p.lr > 2 && p.lr > per_wave_max) p.lr /= 2;
    const int units = rc * rec_k / x_unit(fmt);
    p.x_shift = 0;
    while ((1 << p.x_shift) < units) p.x_shift++;
    break;
  }
  return p;
}

struct SweepPlan {
  bool ok;
  int S, lr, spw, grid, gn, gk, wps, rc, x_shift, x_stride, x_region;
  size_t lds;
};

// Launch shape of the sweeping kernel: one resident round of workgroups of up to 16
// wavefronts; LDS holds one parked tile per (strip, wave) and the activations of one
// phase of K, in as few phases as fit.
// any_shape: this kernel must take the shape (no other kernel can): strips per workgroup
// are capped so that the parked tiles fit, whatever number of rounds and phases that takes.
// gk > 1: K is cut in gk slices, each with its own kNumCU / gk workgroups along N.
SweepPlan make_sweep_plan(int fmt, int M, int64_t n_strips, int n_rec_all, int rec_k, bool any_shape = false, int gk = 1) {
  SweepPlan p;
  const int mt = M > 16 ? 2 : 1;
  const int mc = std::min(M, 16);
  p.ok = false;
  p.gk = gk;
  if (!any_shape && n_strips > (int64_t)kNumCU * 64) return p;
  const int n_rec = (n_rec_all + gk - 1) / gk;  // records of the longest slice
  const int wg_along_n = kNumCU / gk;
  p.spw = (int)((n_strips + wg_along_n - 1) / wg_along_n);
  const size_t tile_bytes = (size_t)mt * 4 * mc * 16;  // one parked tile
  if (any_shape) p.spw = (int)std::max<int64_t>(1, std::min<int64_t>(p.spw, (48 * 1024) / tile_bytes));
  p.gn = (int)((n_strips + p.spw - 1) / p.spw);
  p.grid = p.gn * gk;
  // The baseline's records are four times larger (one in flight per wave).  Measured: at M <= 4 with every
  // compute unit busy it reads 8-14 % faster from 8 wavefronts with two records in flight each (the packed
  // formats do not: equal at M = 1, slower from M = 8).
  const bool few_waves = fmt == FMT_FP16 && M <= 4 && gk == 1 && !any_shape && n_strips >= kNumCU && p.spw <= 16;
  p.S = (int)std::min<int64_t>(few_waves ? 8 : 16, (int64_t)p.spw * (n_rec_all / gk));  // n_rec_all / gk: the shortest slice
  if (p.S < 1) return p;
  p.lr = fmt == FMT_FP16 ? (few_waves ? 2 : 1) : 2;
  // waves per strip: all of them unless the parked tiles (one per strip and wave of its group)
  // would take more than 48 KB; never fewer than leaves every group of waves a strip
  p.wps = p.S;
  if (p.S == 16)
    while (p.wps > 1 && (size_t)p.spw * p.wps * tile_bytes > 48 * 1024 && 16 / (p.wps / 2) <= p.spw) p.wps /= 2;
  const size_t parts = (size_t)p.spw * p.wps * tile_bytes;
  for (int n_phase = 1; n_phase <= (any_shape ? n_rec : 8) && n_phase <= n_rec; n_phase++) {
    const int rc = (n_rec + n_phase - 1) / n_phase;
    const int x_stride = rc * rec_k + 8;  // +8 halfs: consecutive rows start 16 bytes apart in the banks
    const size_t lds = (size_t)M * x_stride * 2 + parts;
    if (lds > (size_t)kStreamLdsMax) continue;
    // measured: with many parked tiles and more than four phases (two for the baseline's larger records) the
    // contiguous-piece kernel is faster
    if (!any_shape && n_phase > (fmt == FMT_FP16 ? 2 : 4) && parts > 32 * 1024) break;
    p.ok = true;
    p.rc = rc;
    p.x_stride = x_stride;
    p.x_region = M * x_stride;
    p.lds = lds;
    const int units = rc * rec_k / x_unit(fmt);
    p.x_shift = 0;
    while ((1 << p.x_shift) < units) p.x_shift++;
    break;
  }
  return p;
}

struct ColumnPlan {
  int S, spw, grid, gn, gk, wps, rc, n_phase, x_shift, x_stride, x_region;
  bool qd;  // records dealt in whole side groups
  int wpa;  // wavefronts of a strip that take records (= wps unless fewer divide the side groups evenly)
  int lr;   // records a wavefront keeps in flight beside the one it restores
  int ns;   // strips a wavefront owns alone (multi_kernel; 1: column_kernel); then wpa = wavefronts that own strips
  size_t lds;
};

// Launch shape of the packed formats' kernel for S wavefronts per workgroup that keep lr records in flight each: up
// to 16 neighbouring strips per workgroup (one resident round of workgroups where the matrix allows it), S / strips
// wavefronts on each strip; LDS holds the activations of one phase of K, in as few phases as fit,
// and one tile per wavefront for the final sum.  Every shape the entry points accept gets a plan.
// gk > 1: K is cut in gk slices, each with its own kNumCU / gk workgroups along N.
// allow_qd: the caller's variant can deal whole side groups (not with one scale per run of input channels).
ColumnPlan column_plan_for(int S, int lr, int fmt, int M, int64_t n_strips, int n_rec_all, int rec_k, int gk, bool allow_qd,
                           int ns = 1) {
  ColumnPlan p;
  p.ns = ns;
  const int sg = ams::side_group(ams::kFormats[fmt]);
  const int mt = M > 16 ? 2 : 1;
  const int mc = std::min(M, 16);
  p.gk = gk;
  p.S = S;
  p.lr = lr;
  const int n_rec = (n_rec_all + gk - 1) / gk;  // records of the longest slice
  const int wg_along_n = kNumCU / gk;
  p.spw = (int)std::min<int64_t>(16, (n_strips + wg_along_n - 1) / wg_along_n);
  p.gn = (int)((n_strips + p.spw - 1) / p.spw);
  p.grid = p.gn * gk;
  p.wps = ns > 1 ? 1 : p.S / p.spw;
  const size_t parts = ns > 1 ? 0 : (size_t)p.spw * p.wps * mt * 4 * mc * 16;  // at most 32 KiB
  // Whole side groups per wavefront where that divides the work evenly enough: the phases then start on group
  // boundaries, and every wavefront of a strip must get (nearly) the same number of groups.
  p.qd = false;
  for (int n_phase = 1;; n_phase++) {
    int rc = (n_rec + n_phase - 1) / n_phase;
    bool qd = allow_qd && sg > 1 && gk == 1;
    int wpa = p.wps;
    if (qd) {
      // the most wavefronts per strip, at least 7 of 8 of them, among which the groups divide within 20 %.  Measured
      // on eleven shapes and four formats: a wavefront with a fifth more records than the average costs less than
      // a side dword loaded with every record (each of a group's records is then read by another wavefront, and
      // each loads the group's 256 bytes of side bits again: 2-14 % slower), while leaving more than an eighth of
      // the wavefronts without records to make the groups divide costs more than it gains (up to 9 % slower)
      const int rcq = (rc + sg - 1) / sg * sg;
      const int groups = rcq / sg;
      qd = false;
      if ((size_t)M * (rcq * rec_k + 8) * 2 + parts <= (size_t)kLdsMaxBytes)
        for (int w = p.wps; w * 8 >= p.wps * 7 && w >= 1 && !qd; w--)
          if (groups >= w && (groups + w - 1) / w * w * 100 <= groups * 120) qd = true, wpa = w;
      if (qd) rc = rcq;
    }
    const int x_stride = rc * rec_k + 8;  // +8 halfs: consecutive rows start 16 bytes apart in the banks
    const size_t lds = (size_t)M * x_stride * 2 + parts;
    if (lds > (size_t)kLdsMaxBytes && rc > 1) continue;  // one record per phase always fits (32 rows x 136 halfs)
    p.qd = qd;
    p.wpa = ns > 1 ? (p.spw + ns - 1) / ns : wpa;
    p.rc = rc;
    p.n_phase = (n_rec + rc - 1) / rc;
    p.x_stride = x_stride;
    p.x_region = M * x_stride;
    p.lds = lds;
    const int units = rc * rec_k / x_unit(fmt);
    p.x_shift = 0;
    while ((1 << p.x_shift) < units) p.x_shift++;
    break;
  }
  return p;
}

// allow_qd: the caller's variant can deal whole side groups (not with one scale per run of input channels).
// allow_deep: the caller has the kernel with three records ahead (non-temporal loads, one scale per row).
ColumnPlan make_column_plan(int fmt, int M, int64_t n_strips, int n_rec_all, int rec_k, int gk = 1, bool allow_qd = true,
                            bool allow_deep = true) {
  const ColumnPlan p = column_plan_for(16, 2, fmt, M, n_strips, n_rec_all, rec_k, gk, allow_qd);
  // Eight wavefronts with three records ahead instead of sixteen with two: fewer wavefronts contend for the VALU
  // and nearly the same bytes are in flight.  Measured on fourteen shapes: formats whose records carry no side
  // groups are 1-7 % faster where the workgroups fill the chip, at least seven of the eight wavefronts get a strip
  // or an equal share of one, and a wavefront's stream is long enough to amortise the deeper ring's start; slower
  // elsewhere, and slower at larger batches (half the threads stage the activations) except where a wavefront is
  // alone on its strip and needs no sum through LDS at the end (up to a batch of 8).  With the side groups dealt
  // whole only that last case gains: FP4.25 0-8 % (kept), FP4.33 -4 % at K = 4096 and +3 % at K = 8192 (not kept).
  const int sg = ams::side_group(ams::kFormats[fmt]);
  const int n_rec = (n_rec_all + gk - 1) / gk;
  // More strips than eight wavefronts: two strips per wavefront, side by side (70B gate/up 50.8 -> 48.5 us, the
  // 128256 x 4096 vocabulary projection 55.1 -> 54.5, the same at K = 8192 +- 0; batches up to 8 measured).
  if (allow_deep && sg == 1 && gk == 1 && p.spw >= 9 && p.grid >= kNumCU * 7 / 8 && n_rec >= 8 && M <= 8)
    return column_plan_for(8, 3, fmt, M, n_strips, n_rec_all, rec_k, gk, allow_qd, 2);
  const int active = p.spw <= 8 ? (8 / p.spw) * p.spw : 0;  // of eight wavefronts, those that get records
  if (!allow_deep || gk != 1 || active < 7 || p.grid < kNumCU * 7 / 8 || (int64_t)n_rec * p.spw < 16 * active) return p;
  if (sg == 1 && (M <= 2 || (p.spw >= 7 && M <= 8))) return column_plan_for(8, 3, fmt, M, n_strips, n_rec_all, rec_k, gk, allow_qd);
  if (fmt == FMT_FP425 && allow_qd && p.spw >= 7 && M <= 16) {
    const ColumnPlan d = column_plan_for(8, 3, fmt, M, n_strips, n_rec_all, rec_k, gk, allow_qd);
    if (d.qd) return d;  // three records ahead exist for the side-group deal only
  }
  return p;
}

// Workspace of a split in gk slices: per-strip arrival counters, then the partial tiles.  The
// counter area has one size for every shape, so that a workspace that is reused for another
// shape never finds old tile data where it expects counters at zero.
constexpr int64_t kSplitMaxStrips = 16384;
constexpr size_t kSplitCounterBytes = (size_t)kSplitMaxStrips * 4;
size_t split_workspace_bytes(int M, int64_t n_strips, int gk) {
  return gk <= 1 ? 0 : kSplitCounterBytes + (size_t)gk * n_strips * (M > 16 ? 2 : 1) * 1024;
}

// The baseline's GEMV kernel takes batches up to 4 whose activations fit in LDS beside nothing else.
struct GemvPlan {
  bool ok;
  int kpad;    // K rounded up to whole 512-channel segments
  size_t lds;  // M rows of kpad halfs
};
GemvPlan make_gemv_plan(int M, int64_t K, int gk) {
  GemvPlan p;
  p.kpad = (int)((K + 511) / 512 * 512);
  p.lds = (size_t)M * p.kpad * 2;
  p.ok = M <= 4 && gk == 1 && K % 8 == 0 && p.lds <= (size_t)kLdsMaxBytes;
  return p;
}

constexpr int kMaxSplit = 8;  // most slices of K choose_split ever takes
// passed as the workspace by the entry point that uses the library's static scratch instead
void* const kStaticScratch = (void*)(uintptr_t)1;

// How many slices of K to use when a workspace is available.  A split pays when the strips
// alone do not fill the compute units evenly (e.g. 320 strips: 2 per workgroup on 160 CUs,
// against 5 strips x a quarter of K on 256) and when the batch is large (every workgroup
// stages the activations of its own slice of K only).  The estimate is bytes a workgroup
// moves: its weight records, half weight for the activations it stages (they come from
// L2), and a fixed charge for the exchange through the workspace (fitted to measurements on
// the Llama and Qwen shapes: below a batch of 4 the stream is bound by the memory system as a
// whole and a split never paid).
int choose_split(int fmt, int M, int64_t n_strips, int n_rec, int rec_k, int rec_bytes) {
  if (M < 4) return 1;
  int best = 1;
  double best_cost = 0;
  for (int gk = 1; gk <= kMaxSplit; gk *= 2) {
    if (gk > 1 && (n_rec / gk < 8 || n_strips > kSplitMaxStrips)) break;
    int spw, rc;
    double rounds = 1.0;  // the packed formats' workgroups take at most 16 strips: more of them means more rounds
    SweepPlan p;
    p.ok = true;
    if (fmt != FMT_FP16) {
      const ColumnPlan cp = make_column_plan(fmt, M, n_strips, n_rec, rec_k, gk);
      spw = cp.spw, rc = cp.rc;
      rounds = std::max(1.0, (double)cp.grid / kNumCU);
    } else {
      p = make_sweep_plan(fmt, M, n_strips, n_rec, rec_k, false, gk);
      spw = p.spw, rc = p.rc;
    }
    if (!p.ok) {
      if (gk > 1) continue;
      // without a split the shape would go to the contiguous-piece kernel: price that one
      const StreamPlan sp = make_stream_plan(fmt, M, n_strips, n_rec, rec_k);
      if (!sp.ok) continue;
      spw = sp.spw, rc = sp.rc;
    }
    const double slice = (double)((n_rec + gk - 1) / gk);
    const double n_phase = std::max(1.0, slice / rc);
    double cost = spw * slice * rec_bytes + 0.5 * M * slice * rec_k * 2 + 8192.0 * (n_phase - 1);
    if (gk > 1) cost += 49152.0 + 2048.0 * gk * spw * (M > 16 ? 2 : 1);
    cost *= rounds;
    if (best_cost == 0 || cost < best_cost) best = gk, best_cost = cost;
  }
  return best;
}

// Per-device state, set up once per device with that device current: whether it is the GPU
// this library is written for, and where this device's copy of the static scratch lives.
constexpr int kMaxDevices = 64;
struct DeviceState {
  int status;     // 0 = not looked at yet, 1 = usable, -1 = not a gfx950 with the expected resources
  void* scratch;  // device address of this device's `scratch` array
};
std::mutex g_dev_mu;
DeviceState g_dev[kMaxDevices];

// Scratch of the entry point that may not allocate (ams_linear_static_ws): the arrival counters
// and partial tiles of a split of K.  One copy per GPU, held until the process ends.  In host
// code this name is only a handle for hipGetSymbolAddress, never a device address.
constexpr size_t kStaticScratchBytes = ((size_t)64 << 10) + ((size_t)8 << 20);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// AMS_OK when the current device is a gfx950 with the compute units and LDS the launch plans
// assume; looked up once per device (no allocation, no synchronisation).
int device_state(DeviceState** out = nullptr) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return AMS_ERR_DEVICE;
  std::lock_guard<std::mutex> lock(g_dev_mu);
  DeviceState& d = g_dev[dev];
  if (d.status == 0) {
    hipDeviceProp_t prop;
    d.status = -1;
    if (hipGetDeviceProperties(&prop, dev) == hipSuccess && strncmp(prop.gcnArchName, "gfx950", 6) == 0 &&
        prop.multiProcessorCount >= 1 && prop.warpSize == 64) {
      void* ptr = nullptr;
      if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) == hipSuccess && ptr) {
        d.scratch = ptr;
        d.status = 1;
      }
    }
    (void)hipGetLastError();  // a failed query must not be reported by the caller's next HIP call
  }
  if (out) *out = &d;
  return d.status == 1 ? AMS_OK : AMS_ERR_DEVICE;
}

// Kernels that use more than 64 KiB of dynamic LDS must have their limit raised first;
// that is a per-function, per-device property, remembered here so it is done once.
bool raise_lds_limit(const void* kern) {
  struct Entry {
    const void* kern;
    int dev;
  };
  static std::mutex mu;
  static std::vector<Entry> done;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  std::lock_guard<std::mutex> lock(mu);
  for (const Entry& e : done)
    if (e.kern == kern && e.dev == dev) return true;
  if (hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsMaxBytes) != hipSuccess) return false;
  try {
    done.push_back({kern, dev});
  } catch (...) {  // out of host memory: the limit is raised, it is just not remembered
  }
  return true;
}

// grid == 0: only prepare the kernel (raise its LDS limit), launch nothing (ams_init)
template <class Kern>
int launch(Kern kern, const LinearArgs& a, unsigned grid, int S, size_t lds, hipStream_t st) {
  if ((grid == 0 || lds > 64 * 1024) && !raise_lds_limit((const void*)kern)) return AMS_ERR_LAUNCH;
  if (grid == 0) return AMS_OK;
  hipLaunchKernelGGL(kern, dim3(grid), dim3(64 * S), lds, st, a);
  return hipGetLastError() == hipSuccess ? AMS_OK : AMS_ERR_LAUNCH;
}

enum KernelKind { kSweep, kStream };

// The fp16 baseline's kernels by ring depth and wave grouping.
template <int MT>
int launch_fp16(KernelKind kind, int lr, const LinearArgs& a, unsigned grid, int S, size_t lds, hipStream_t st) {
  const bool groups = a.wps != S;  // wave groups per strip: their own instantiation, the common case stays lean
  if (kind == kSweep) {
    if (lr == 1) return groups ? launch(sweep_kernel<MT, 1, true>, a, grid, S, lds, st) : launch(sweep_kernel<MT, 1, false>, a, grid, S, lds, st);
    if (lr == 2 && !groups) return launch(sweep_kernel<MT, 2, false>, a, grid, S, lds, st);
  } else {
    switch (lr) {
      case 4: return launch(stream_kernel<MT, 4>, a, grid, S, lds, st);
      case 2: return launch(stream_kernel<MT, 2>, a, grid, S, lds, st);
    }
  }
  return AMS_ERR_LAUNCH;
}

// The baseline's GEMV kernel by batch size.
int launch_gemv(int M, bool nt, const LinearArgs& a, unsigned grid, size_t lds, hipStream_t st) {
  switch (M) {
    case 1: return nt ? launch(gemv_fp16_kernel<1, true>, a, grid, 16, lds, st) : launch(gemv_fp16_kernel<1, false>, a, grid, 16, lds, st);
    case 2: return nt ? launch(gemv_fp16_kernel<2, true>, a, grid, 16, lds, st) : launch(gemv_fp16_kernel<2, false>, a, grid, 16, lds, st);
    case 3: return nt ? launch(gemv_fp16_kernel<3, true>, a, grid, 16, lds, st) : launch(gemv_fp16_kernel<3, false>, a, grid, 16, lds, st);
    case 4: return nt ? launch(gemv_fp16_kernel<4, true>, a, grid, 16, lds, st) : launch(gemv_fp16_kernel<4, false>, a, grid, 16, lds, st);
  }
  return AMS_ERR_LAUNCH;
}

// The packed formats' kernel: nt = non-temporal weight loads, gs = one scale per run of input channels.
template <int FMT, int MT>
int launch_column(bool nt, bool gs, bool qd, int lr, const LinearArgs& a, unsigned grid, int S, size_t lds, hipStream_t st) {
  if (gs) return launch(column_kernel<FMT, MT, true, true>, a, grid, S, lds, st);
  if constexpr (Fmt<FMT>::SG == 1) {
    if (lr == 3) return nt ? launch(column_kernel<FMT, MT, true, false, false, 3>, a, grid, S, lds, st) : AMS_ERR_LAUNCH;
  }
  if constexpr (Fmt<FMT>::SG == 4) {
    if (qd && lr == 3) return nt ? launch(column_kernel<FMT, MT, true, false, true, 3>, a, grid, S, lds, st) : AMS_ERR_LAUNCH;
  }
  if constexpr (Fmt<FMT>::SG > 1) {
    if (qd)
      return nt ? launch(column_kernel<FMT, MT, true, false, true>, a, grid, S, lds, st)
                : launch(column_kernel<FMT, MT, false, false, true>, a, grid, S, lds, st);
  }
  return nt ? launch(column_kernel<FMT, MT, true, false>, a, grid, S, lds, st)
            : launch(column_kernel<FMT, MT, false, false>, a, grid, S, lds, st);
}

// Wavefronts that own two strips each (non-temporal loads, one scale per row).
template <int FMT, int MT>
int launch_multi(const LinearArgs& a, unsigned grid, int S, size_t lds, hipStream_t st) {
  if constexpr (Fmt<FMT>::SG == 1) return launch(multi_kernel<FMT, MT, true, 2>, a, grid, S, lds, st);
  return AMS_ERR_LAUNCH;
}

template <int FMT>
int run_linear(const void* W, const uint16_t* scales, const uint16_t* X, uint16_t* Y, int M, int64_t N, int64_t K,
               void* stream, int64_t scale_group = 0, void* workspace = nullptr, size_t ws_bytes = 0) {
  if (!W || !X || !Y || (FMT != FMT_FP16 && !scales)) return AMS_ERR_NULL;
  if (M < 1 || M > AMS_MAX_M || N <= 0 || K <= 0 || N > (1 << 24) || K > (1 << 24)) return AMS_ERR_SHAPE;
  if (FMT == FMT_FP16 && (K % 8) != 0) return AMS_ERR_SHAPE;
  if (!aligned16(W) || !aligned16(X) || !aligned16(Y) || (scales && !aligned16(scales))) return AMS_ERR_ALIGN;
  DeviceState* dev = nullptr;
  if (const int rc = device_state(&dev); rc != AMS_OK) return rc;
  const bool static_ws = workspace == kStaticScratch;
  if (static_ws) {  // the library's own scratch, this device's copy
    workspace = dev->scratch;
    ws_bytes = kStaticScratchBytes;
  }
  constexpr int REC_K = Fmt<FMT>::REC_K;
  const int64_t n_strips = (N + 15) / 16;
  const int n_rec = (int)((K + REC_K - 1) / REC_K);
  LinearArgs a;
  a.W = (const uint8_t*)W;
  a.scales = scales;
  a.X = X;
  a.Y = Y;
  a.M = M;
  a.N = (int)N;
  a.K = (int)K;
  a.n_rec = n_rec;
  a.n_strips = (int)n_strips;
  hipStream_t st = (hipStream_t)stream;
  a.n_sg = 0;
  a.sg_shift = 0;
  if (scale_group != 0) {  // one scale per run of scale_group = REC_K * 2^shift input channels
    int shift = -1;
    for (int j = 0; j < 20; j++)
      if (scale_group == (int64_t)REC_K << j) shift = j;
    if (shift < 0 || FMT == FMT_FP16) return AMS_ERR_SHAPE;
    a.sg_shift = shift;
    a.n_sg = (int)((K + scale_group - 1) / scale_group);
  }
  a.gn = 1;
  a.gk = 1;
  a.wps = 1;
  a.wpa = 1;
  a.ws_tiles = nullptr;
  a.ws_count = nullptr;
  a.red_slots = 0;
  a.piece_q = a.piece_r = 0;
  constexpr int REC_BYTES = FMT == FMT_FP16 ? 4096 : Fmt<FMT>::REC_BYTES;
  int gk = 1;
  if (workspace && scale_group == 0) {
    if (!aligned16(workspace)) return AMS_ERR_ALIGN;
    gk = choose_split(FMT, M, n_strips, n_rec, REC_K, REC_BYTES);
    if (split_workspace_bytes(M, n_strips, gk) > ws_bytes) {
      if (static_ws) return AMS_ERR_SCRATCH;  // beyond the static array: refused, never silently another plan
      gk = 1;                                 // a caller's workspace that is too small: no split
    }
  }
  auto use_split = [&](int plan_gk) {
    if (plan_gk > 1) {
      a.ws_count = (unsigned*)workspace;
      a.ws_tiles = (f4*)((uint8_t*)workspace + kSplitCounterBytes);
    }
  };
  if constexpr (FMT != FMT_FP16) {
    // Non-temporal loads for everything but tiny matrices.  Measured with every call reading weights that are not
    // in any cache (a model's layers in turn): equal or up to 5 % faster than ordinary loads at every size; ordinary
    // loads only win when the same few megabytes are read again call after call.
    const bool nt = n_strips * n_rec * (int64_t)REC_BYTES >= (2ll << 20);
    const ColumnPlan cp = make_column_plan(FMT, M, n_strips, n_rec, REC_K, gk, scale_group == 0, scale_group == 0 && nt);
    a.gn = cp.gn;
    a.gk = cp.gk;
    a.wps = cp.wps;
    a.wpa = cp.wpa;
    use_split(cp.gk);
    a.x_stride = cp.x_stride;
    a.x_region = cp.x_region;
    a.x_shift = cp.x_shift;
    a.spw = cp.spw;
    a.rc = cp.rc;
    if (cp.ns > 1) return M <= 16 ? launch_multi<FMT, 1>(a, cp.grid, cp.S, cp.lds, st) : launch_multi<FMT, 2>(a, cp.grid, cp.S, cp.lds, st);
    return M <= 16 ? launch_column<FMT, 1>(nt, scale_group != 0, cp.qd, cp.lr, a, cp.grid, cp.S, cp.lds, st)
                   : launch_column<FMT, 2>(nt, scale_group != 0, cp.qd, cp.lr, a, cp.grid, cp.S, cp.lds, st);
  } else {
    if (const GemvPlan gp = make_gemv_plan(M, K, gk); gp.ok) {
      a.x_stride = gp.kpad;
      const bool nt = N * K * 2 >= (2ll << 20);
      return launch_gemv(M, nt, a, kNumCU, gp.lds, st);
    }
    const SweepPlan wp = make_sweep_plan(FMT, M, n_strips, n_rec, REC_K, false, gk);
    if (wp.ok) {
      a.gn = wp.gn;
      a.gk = wp.gk;
      a.wps = wp.wps;
      use_split(wp.gk);
      a.x_stride = wp.x_stride;
      a.x_region = wp.x_region;
      a.x_shift = wp.x_shift;
      a.spw = wp.spw;
      a.rc = wp.rc;
      return M <= 16 ? launch_fp16<1>(kSweep, wp.lr, a, wp.grid, wp.S, wp.lds, st) : launch_fp16<2>(kSweep, wp.lr, a, wp.grid, wp.S, wp.lds, st);
    }
    const StreamPlan sp = make_stream_plan(FMT, M, n_strips, n_rec, REC_K);
    if (sp.ok) {
      a.x_stride = sp.x_stride;
      a.x_region = sp.x_region;
      a.x_shift = sp.x_shift;
      a.spw = sp.spw;
      a.red_slots = sp.red_slots;
      a.piece_q = (int)(((int64_t)sp.spw * sp.rc) / sp.S);
      a.piece_r = (int)(((int64_t)sp.spw * sp.rc) % sp.S);
      a.rc = sp.rc;
      return M <= 16 ? launch_fp16<1>(kStream, sp.lr, a, sp.grid, sp.S, sp.lds, st) : launch_fp16<2>(kStream, sp.lr, a, sp.grid, sp.S, sp.lds, st);
    }
    return AMS_ERR_SHAPE;  // not reached: the contiguous-piece plan accepts every shape the checks above let through
  }
}

// Raise the LDS limit of every Linear kernel of one weight format on the current device.
template <int FMT>
int prepare_format() {
  LinearArgs a = {};
  bool ok = true;
  if constexpr (FMT != FMT_FP16) {
    for (int nt = 0; nt < 2; nt++)
      for (int gs = 0; gs < 2; gs++)
        for (int qd = 0; qd < 2; qd++) {
          if (gs && (!nt || qd)) continue;
          ok &= launch_column<FMT, 1>(nt, gs, qd, 2, a, 0, 16, 0, nullptr) == AMS_OK;
          ok &= launch_column<FMT, 2>(nt, gs, qd, 2, a, 0, 16, 0, nullptr) == AMS_OK;
        }
    if constexpr (Fmt<FMT>::SG == 1) {
      ok &= launch_multi<FMT, 1>(a, 0, 8, 0, nullptr) == AMS_OK;
      ok &= launch_multi<FMT, 2>(a, 0, 8, 0, nullptr) == AMS_OK;
    }
    if constexpr (Fmt<FMT>::SG == 1 || Fmt<FMT>::SG == 4) {
      ok &= launch_column<FMT, 1>(true, false, Fmt<FMT>::SG == 4, 3, a, 0, 8, 0, nullptr) == AMS_OK;
      ok &= launch_column<FMT, 2>(true, false, Fmt<FMT>::SG == 4, 3, a, 0, 8, 0, nullptr) == AMS_OK;
    }
  } else {
    for (int m = 1; m <= 4; m++)
      for (int nt = 0; nt < 2; nt++) ok &= launch_gemv(m, nt != 0, a, 0, 0, nullptr) == AMS_OK;
    for (int groups = 0; groups < 2; groups++) {
      a.wps = groups ? 8 : 16;
      ok &= launch_fp16<1>(kSweep, 1, a, 0, 16, 0, nullptr) == AMS_OK;
      ok &= launch_fp16<2>(kSweep, 1, a, 0, 16, 0, nullptr) == AMS_OK;
    }
    a.wps = 16;
    ok &= launch_fp16<1>(kSweep, 2, a, 0, 16, 0, nullptr) == AMS_OK;
    ok &= launch_fp16<2>(kSweep, 2, a, 0, 16, 0, nullptr) == AMS_OK;
    for (int lr : {2, 4}) {
      ok &= launch_fp16<1>(kStream, lr, a, 0, 16, 0, nullptr) == AMS_OK;
      ok &= launch_fp16<2>(kStream, lr, a, 0, 16, 0, nullptr) == AMS_OK;
    }
  }
  (void)hipGetLastError();
  return ok ? AMS_OK : AMS_ERR_LAUNCH;
}

}  // namespace

extern "C" {

int ams_init(void) {
  if (const int rc = device_state(); rc != AMS_OK) return rc;
  int rc = prepare_format<FMT_FP533>();
  if (rc == AMS_OK) rc = prepare_format<FMT_FP425>();
  if (rc == AMS_OK) rc = prepare_format<FMT_FP45>();
  if (rc == AMS_OK) rc = prepare_format<FMT_FP433>();
  if (rc == AMS_OK) rc = prepare_format<FMT_FP6>();
  if (rc == AMS_OK) rc = prepare_format<FMT_FP5>();
  if (rc == AMS_OK) rc = prepare_format<FMT_FP4>();
  if (rc == AMS_OK) rc = prepare_format<FMT_FP16>();
  return rc;
}

int ams_linear_static_ws(const void* W_packed, const uint16_t* scales, const uint16_t* X, uint16_t* Y, int M, int64_t N,
                         int64_t K, int fmt, void* stream) {
  switch (fmt) {
    case FMT_FP533: return run_linear<FMT_FP533>(W_packed, scales, X, Y, M, N, K, stream, 0, kStaticScratch, 0);
    case FMT_FP425: return run_linear<FMT_FP425>(W_packed, scales, X, Y, M, N, K, stream, 0, kStaticScratch, 0);
    case FMT_FP45: return run_linear<FMT_FP45>(W_packed, scales, X, Y, M, N, K, stream, 0, kStaticScratch, 0);
    case FMT_FP433: return run_linear<FMT_FP433>(W_packed, scales, X, Y, M, N, K, stream, 0, kStaticScratch, 0);
    case FMT_FP6: return run_linear<FMT_FP6>(W_packed, scales, X, Y, M, N, K, stream, 0, kStaticScratch, 0);
    case FMT_FP5: return run_linear<FMT_FP5>(W_packed, scales, X, Y, M, N, K, stream, 0, kStaticScratch, 0);
    case FMT_FP4: return run_linear<FMT_FP4>(W_packed, scales, X, Y, M, N, K, stream, 0, kStaticScratch, 0);
  }
  return AMS_ERR_FORMAT;
}

int ams_dequant(int fmt, const void* W_packed, const uint16_t* scales, uint16_t* W_out, int64_t N, int64_t K, int scaled,
                void* stream) {
  return ams_dequant_grouped(fmt, W_packed, scales, 0, W_out, N, K, scaled, stream);
}

int ams_dequant_grouped(int fmt, const void* W_packed, const uint16_t* scales, int64_t scale_group, uint16_t* W_out,
                        int64_t N, int64_t K, int scaled, void* stream) {
  const ams::FormatInfo* fi = ams::format_info(fmt);
  if (!fi) return AMS_ERR_FORMAT;
  if (!W_packed || !W_out || (scaled && !scales)) return AMS_ERR_NULL;
  if (N <= 0 || K <= 0 || N > (1 << 24) || K > (1 << 24)) return AMS_ERR_SHAPE;
  if (!aligned16(W_packed)) return AMS_ERR_ALIGN;
  if (const int rc = device_state(); rc != AMS_OK) return rc;
  int sg_shift = -1, n_sg = 0;  // per-row scales
  if (scale_group != 0) {
    for (int j = 0; j < 20; j++)
      if (scale_group == (int64_t)fi->rec_k << j) sg_shift = j;
    if (sg_shift < 0) return AMS_ERR_SHAPE;
    n_sg = (int)((K + scale_group - 1) / scale_group);
  }
  const int n_rec = (int)((K + fi->rec_k - 1) / fi->rec_k);
  const int64_t total = ((N + 15) / 16) * n_rec;
  const unsigned grid = (unsigned)((total + 3) / 4);
  hipStream_t st = (hipStream_t)stream;
  auto go = [&](auto kern) {
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), 0, st, (const uint8_t*)W_packed, scales, W_out, (int)N, (int)K, n_rec, total, scaled, n_sg,
                       sg_shift);
  };
  switch (fmt) {
    case FMT_FP533: go(dequant_kernel<FMT_FP533>); break;
    case FMT_FP425: go(dequant_kernel<FMT_FP425>); break;
    case FMT_FP45: go(dequant_kernel<FMT_FP45>); break;
    case FMT_FP433: go(dequant_kernel<FMT_FP433>); break;
    case FMT_FP6: go(dequant_kernel<FMT_FP6>); break;
    case FMT_FP5: go(dequant_kernel<FMT_FP5>); break;
    default: go(dequant_kernel<FMT_FP4>); break;
  }
  return hipGetLastError() == hipSuccess ? AMS_OK : AMS_ERR_LAUNCH;
}

int ams_linear(const void* W_packed, const uint16_t* scales, const uint16_t* X, uint16_t* Y, int M, int64_t N, int64_t K,
               int fmt, void* stream) {
  switch (fmt) {
    case FMT_FP533: return run_linear<FMT_FP533>(W_packed, scales, X, Y, M, N, K, stream);
    case FMT_FP425: return run_linear<FMT_FP425>(W_packed, scales, X, Y, M, N, K, stream);
    case FMT_FP45: return run_linear<FMT_FP45>(W_packed, scales, X, Y, M, N, K, stream);
    case FMT_FP433: return run_linear<FMT_FP433>(W_packed, scales, X, Y, M, N, K, stream);
    case FMT_FP6: return run_linear<FMT_FP6>(W_packed, scales, X, Y, M, N, K, stream);
    case FMT_FP5: return run_linear<FMT_FP5>(W_packed, scales, X, Y, M, N, K, stream);
    case FMT_FP4: return run_linear<FMT_FP4>(W_packed, scales, X, Y, M, N, K, stream);
  }
  return AMS_ERR_FORMAT;
}

int ams_linear_grouped(const void* W_packed, const uint16_t* scales, int64_t scale_group, const uint16_t* X, uint16_t* Y,
                       int M, int64_t N, int64_t K, int fmt, void* stream) {
  if (scale_group <= 0) return AMS_ERR_SHAPE;
  switch (fmt) {
    case FMT_FP533: return run_linear<FMT_FP533>(W_packed, scales, X, Y, M, N, K, stream, scale_group);
    case FMT_FP425: return run_linear<FMT_FP425>(W_packed, scales, X, Y, M, N, K, stream, scale_group);
    case FMT_FP45: return run_linear<FMT_FP45>(W_packed, scales, X, Y, M, N, K, stream, scale_group);
    case FMT_FP433: return run_linear<FMT_FP433>(W_packed, scales, X, Y, M, N, K, stream, scale_group);
    case FMT_FP6: return run_linear<FMT_FP6>(W_packed, scales, X, Y, M, N, K, stream, scale_group);
    case FMT_FP5: return run_linear<FMT_FP5>(W_packed, scales, X, Y, M, N, K, stream, scale_group);
    case FMT_FP4: return run_linear<FMT_FP4>(W_packed, scales, X, Y, M, N, K, stream, scale_group);
  }
  return AMS_ERR_FORMAT;
}

int ams_linear_workspace_bytes(int fmt, int M, int64_t N, int64_t K, size_t* bytes) {
  if (!bytes) return AMS_ERR_NULL;
  if (M < 1 || M > AMS_MAX_M || N <= 0 || K <= 0 || N > (1 << 24) || K > (1 << 24)) return AMS_ERR_SHAPE;
  int rec_k = 128, rec_bytes = 4096, f = FMT_FP16;  // fmt < 0: the fp16 baseline
  if (fmt >= 0) {
    const ams::FormatInfo* fi = ams::format_info(fmt);
    if (!fi) return AMS_ERR_FORMAT;
    rec_k = fi->rec_k, rec_bytes = fi->rec_bytes, f = fmt;
  }
  const int64_t n_strips = (N + 15) / 16;
  const int n_rec = (int)((K + rec_k - 1) / rec_k);
  *bytes = split_workspace_bytes(M, n_strips, choose_split(f, M, n_strips, n_rec, rec_k, rec_bytes));
  return AMS_OK;
}

int ams_linear_plan(int fmt, int M, int64_t N, int64_t K, int with_workspace, char* text, size_t text_len) {
  if (!text || text_len == 0) return AMS_ERR_NULL;
  if (M < 1 || M > AMS_MAX_M || N <= 0 || K <= 0 || N > (1 << 24) || K > (1 << 24)) return AMS_ERR_SHAPE;
  int rec_k = 128, rec_bytes = 4096, f = FMT_FP16;
  if (fmt >= 0) {
    const ams::FormatInfo* fi = ams::format_info(fmt);
    if (!fi) return AMS_ERR_FORMAT;
    rec_k = fi->rec_k, rec_bytes = fi->rec_bytes, f = fmt;
  }
  const int64_t n_strips = (N + 15) / 16;
  const int n_rec = (int)((K + rec_k - 1) / rec_k);
  const int gk = with_workspace ? choose_split(f, M, n_strips, n_rec, rec_k, rec_bytes) : 1;
  if (f != FMT_FP16) {
    const bool nt = n_strips * n_rec * (int64_t)rec_bytes >= (2ll << 20);  // as run_linear decides it
    const ColumnPlan cp = make_column_plan(f, M, n_strips, n_rec, rec_k, gk, true, nt);
    snprintf(text, text_len, "column grid=%d strips_per_wg=%d k_slices=%d waves=%d waves_per_strip=%d phases=%d lds=%zu side_groups=%d active_per_strip=%d ahead=%d strips_per_wave=%d", cp.grid,
             cp.spw, cp.gk, cp.S, cp.wps, cp.n_phase, cp.lds, cp.qd ? 1 : 0, cp.ns > 1 ? 1 : cp.wpa, cp.lr, cp.ns);
    return AMS_OK;
  }
  if (const GemvPlan gp = make_gemv_plan(M, K, gk); gp.ok) {
    snprintf(text, text_len, "gemv grid=%d rows_per_wave=%d k_slices=1 waves=16 phases=1 lds=%zu", kNumCU,
             (int)((N + kNumCU * 16 - 1) / (kNumCU * 16)), gp.lds);
    return AMS_OK;
  }
  const SweepPlan wp = make_sweep_plan(f, M, n_strips, n_rec, rec_k, false, gk);
  if (wp.ok) {
    const int slice = (n_rec + gk - 1) / gk;
    snprintf(text, text_len, "sweep grid=%d strips_per_wg=%d k_slices=%d waves=%d waves_per_strip=%d phases=%d lds=%zu", wp.grid, wp.spw,
             wp.gk, wp.S, wp.wps, (slice + wp.rc - 1) / wp.rc, wp.lds);
    return AMS_OK;
  }
  const StreamPlan sp = make_stream_plan(f, M, n_strips, n_rec, rec_k);
  snprintf(text, text_len, "stream grid=%d strips_per_wg=%d k_slices=1 waves=%d phases=%d lds=%zu", sp.grid, sp.spw, sp.S,
           (n_rec + sp.rc - 1) / sp.rc, sp.lds);
  return AMS_OK;
}

int ams_linear_ws(const void* W_packed, const uint16_t* scales, const uint16_t* X, uint16_t* Y, int M, int64_t N, int64_t K,
                  int fmt, void* workspace, size_t workspace_bytes, void* stream) {
  switch (fmt) {
    case FMT_FP533: return run_linear<FMT_FP533>(W_packed, scales, X, Y, M, N, K, stream, 0, workspace, workspace_bytes);
    case FMT_FP425: return run_linear<FMT_FP425>(W_packed, scales, X, Y, M, N, K, stream, 0, workspace, workspace_bytes);
    case FMT_FP45: return run_linear<FMT_FP45>(W_packed, scales, X, Y, M, N, K, stream, 0, workspace, workspace_bytes);
    case FMT_FP433: return run_linear<FMT_FP433>(W_packed, scales, X, Y, M, N, K, stream, 0, workspace, workspace_bytes);
    case FMT_FP6: return run_linear<FMT_FP6>(W_packed, scales, X, Y, M, N, K, stream, 0, workspace, workspace_bytes);
    case FMT_FP5: return run_linear<FMT_FP5>(W_packed, scales, X, Y, M, N, K, stream, 0, workspace, workspace_bytes);
    case FMT_FP4: return run_linear<FMT_FP4>(W_packed, scales, X, Y, M, N, K, stream, 0, workspace, workspace_bytes);
  }
  return AMS_ERR_FORMAT;
}

int ams_fp16_linear_ws(const uint16_t* W, const uint16_t* X, uint16_t* Y, int M, int64_t N, int64_t K, void* workspace,
                       size_t workspace_bytes, void* stream) {
  return run_linear<FMT_FP16>(W, nullptr, X, Y, M, N, K, stream, 0, workspace, workspace_bytes);
}

int ams_fp16_linear(const uint16_t* W, const uint16_t* X, uint16_t* Y, int M, int64_t N, int64_t K, void* stream) {
  return run_linear<FMT_FP16>(W, nullptr, X, Y, M, N, K, stream);
}

int ams_read_probe(const void* buf, size_t bytes, uint32_t* sink, void* stream) {
  if (!buf) return AMS_ERR_NULL;
  if (!aligned16(buf)) return AMS_ERR_ALIGN;
  if (const int rc = device_state(); rc != AMS_OK) return rc;
  const int64_t n_rec = (int64_t)(bytes / 1024);
  // with nothing to read this is an empty launch of the same shape (the launch floor)
  const unsigned grid = n_rec == 0 ? 1u : (unsigned)std::min<int64_t>(kNumCU, (n_rec + 15) / 16);
  if (n_rec == 0)
    hipLaunchKernelGGL(read_probe_kernel, dim3(kNumCU), dim3(1024), 0, (hipStream_t)stream, (const u4*)buf, (int64_t)0, sink);
  else
    hipLaunchKernelGGL(read_probe_kernel, dim3(grid), dim3(1024), 0, (hipStream_t)stream, (const u4*)buf, n_rec, sink);
  return hipGetLastError() == hipSuccess ? AMS_OK : AMS_ERR_LAUNCH;
}

}  // extern "C"
