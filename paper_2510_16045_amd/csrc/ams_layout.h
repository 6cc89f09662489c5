// gfx950 packed-weight layout of the AMS-Quant formats, shared by the host packer
// and the device unpack code of this library.
//
// The paper packs FP5.33 as one uint16 per group of 3 weights and FP4.25 as 16
// nibble words + 1 shared-bit word per 64 weights (Sec. 3.2, Sec. 3.3 item 1).  The
// same information is kept here, but arranged for 64-wide wavefronts feeding
// 16x16x32 fp16 MFMA tiles:
//
//   * rows are cut into strips of 16 output channels, K into records of
//     REC_K weights (96 for FP5.33, 128 for FP4.25);
//   * a record is 64 lane chunks of 16 bytes, lane l = row (l & 15) of the strip,
//     K-quarter (l >> 4) of the record, so one wavefront load of a record is one
//     contiguous 1 KiB dwordx4 access and every lane already owns the operand slots
//     of its MFMA row;
//   * FP4.25 records carry 64 more bytes: lane l's byte holds the shared bits of its
//     8 groups (the "1 word of shared LSBs per 64 weights" of Sec. 3.2, kept per lane);
//   * the records of a strip are contiguous, strips follow each other.
//
// Inside a lane chunk each 32-bit word holds two groups, A in the low half-word and B
// in the high half-word, and the restored fp16 pairs are (A_i, B_i): that way the two
// shared bits of a pair sit 16 bits apart and one shift+mask places both.
//
// Restored values are produced as fp16 bit patterns equal to value * 2^-14: the
// bias-1 exponent and the mantissa are dropped into the low exponent bits / high
// mantissa bits of binary16 (bias 15), which maps subnormal codes onto fp16
// subnormals (Sec. 3.2's SHIFT/AND/OR restoration).  The factor 2^14 is applied in
// fp32 together with the row scale.
//
// Half-word layouts (bit 15 .. bit 0), chosen so that sign and magnitude fields land
// on fp16 bit 15 and bits 11.. with the fewest VALU operations:
//   FP4.25:  s0 s2 s3 s1 | mag0(3) | mag1(3) | mag2(3) | mag3(3)      mag = e1 e0 m1
//   FP5.33:  s0 s1 s2 sh | mag0(4) | mag1(4) | mag2(4)                mag = e1 e0 m2 m1
#ifndef AMS_LAYOUT_H_
#define AMS_LAYOUT_H_

#include <stdint.h>

namespace ams {

constexpr int kStripRows = 16;
constexpr int kLaneChunkBytes = 16;
constexpr int kLanes = 64;

struct FormatInfo {
  int group;       // weights sharing one last mantissa bit
  int code_bits;   // bits of a full code (sign + 2 exponent + mantissa)
  int rec_k;       // weights of one row inside a record
  int lane_k;      // weights of one lane chunk (rec_k / 4)
  int rec_bytes;   // bytes of a record
  double fmax;     // largest magnitude of the format
};

constexpr FormatInfo kFp533 = {3, 6, 96, 24, 1024, 7.5};
constexpr FormatInfo kFp425 = {4, 5, 128, 32, 1024 + 64, 7.0};

inline const FormatInfo* format_info(int fmt) {
  if (fmt == 0) return &kFp533;
  if (fmt == 1) return &kFp425;
  return nullptr;
}

inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

// Position of logical weight j (0..lane_k-1) of a lane chunk inside the lane's MFMA
// operand order: the restored pairs come out as (A_i, B_i) per 32-bit word, so the
// activations must be laid out in the same order.  Both functions are bijections of
// [0, lane_k).
//   FP4.25: word d = j/8, group half h = (j%8)/4, member i = j%4 -> slot 8d + 2i + h
//   FP5.33: word d = j/6, group half h = (j%6)/3, member i = j%3 -> slot 6d + 2i + h
inline int operand_slot_fp425(int j) { return (j & ~7) + 2 * (j & 3) + ((j >> 2) & 1); }
inline int operand_slot_fp533(int j) {
  int d = j / 6, r = j % 6;
  return 6 * d + 2 * (r % 3) + r / 3;
}

}  // namespace ams
#endif
