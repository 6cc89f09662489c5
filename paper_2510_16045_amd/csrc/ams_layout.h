// gfx950 packed-weight layout of the AMS-Quant formats, shared by the host packer
// and the device unpack code of this library.
//
// The paper packs FP5.33 as one uint16 per group of 3 weights and FP4.25 as 16
// nibble words + 1 shared-bit word per 64 weights (Sec. 3.2, Sec. 3.3 item 1).  The
// same information is kept here, but arranged for 64-wide wavefronts feeding
// 16x16x32 fp16 MFMA tiles:
//
//   * rows are cut into strips of 16 output channels, K into records of REC_K weights
//     (96 for the formats whose lane chunk holds 24 weights, 128 for those with 32);
//   * a record is 64 lane chunks (16 bytes, 12 for FP4.33), lane l = row (l & 15) of the
//     strip, K-quarter (l >> 4) of the record, so one wavefront load of a record is one
//     contiguous dwordx4 (dwordx3) access and every lane already owns the operand slots
//     of its MFMA row;
//   * formats whose last mantissa bits do not fit in the chunk carry them as side bits,
//     1, 2 or 4 bytes per lane and record (the "word of shared LSBs" of Sec. 3.2, kept per
//     lane so that no cross-lane traffic is needed).  So that they are read with ordinary
//     dword loads (byte loads per lane cost a wavefront far more than their 64 bytes), the
//     records of a strip come in side groups of 4 / side_bytes consecutive records: a unit
//     = the chunk blocks of the group's records, then one dword per lane whose byte(s) t
//     belong to record t of the group.  Formats without side bits have units of one record;
//   * the units are stored K-major: all strips' units of the first side group, then all
//     strips' units of the second, and so on: unit (g, s) at (g * n_strips + s) *
//     unit_bytes.  Wavefronts that each own a strip and walk K in step therefore read one
//     contiguous window of memory as a whole, which this GPU's memory system serves
//     10-20 % faster than strip-contiguous pieces that advance independently.
//
// A lane chunk is made of 32-bit words of two half-words (A low, B high); a half-word
// holds the remainders (code without its last bit) of 4 weights (e2m2: 4 bits each) or
// 3 weights (e2m3: 5 bits each, plus one spare bit).  The restored fp16 pairs are
// (A_i, B_i), so the last bits of a pair sit 16 bits apart and one shift+mask places
// both.  Half-word layouts (bit 15 .. bit 0), chosen so that sign and magnitude land on
// fp16 bit 15 and bits 11.. with the fewest VALU operations:
//   e2m2:  s0 s2 s3 s1 | mag0(3) | mag1(3) | mag2(3) | mag3(3)       mag = e1 e0 m1
//   e2m3:  s0 s1 s2 b  | mag0(4) | mag1(4) | mag2(4)                 mag = e1 e0 m2 m1
// (b = the group's shared bit for FP5.33, the last bit of member 0 for FP6).
//
// Which weights of a lane chunk form a sharing group (they are always k consecutive
// input channels, Sec. 3.1) and where their common last bit is kept:
//   FP4.25 (k=4)  the 4 members of a half-word; side byte, bit 4h + d
//   FP5.33 (k=3)  the 3 members of a half-word; bit 12 of the half-word
//   FP4.5  (k=2)  member i of half h in words 2q and 2q+1; side byte q, bit 4h + i
//   FP4.33 (k=3)  member i of half h in words 0, 1, 2;      side byte, bit 4h + i
//   FP5    (k=1)  every weight its own bit;                 side byte d, bit 4h + i
//   FP6    (k=1)  member 0: bit 12 of its half-word; members 1, 2: side 16 bits,
//                 bit 8h + 2d + (i - 1)
//   FP4    (e2m1) a nibble is the whole code: the e2m2 layout with every last bit 0
// With the groups of FP4.5 / FP4.33 running across words, the last bits needed for the
// four restored pairs of a word are the same for all words of the group.
//
// Restored values are produced as fp16 bit patterns equal to value * 2^-14: the
// bias-1 exponent and the mantissa are dropped into the low exponent bits / high
// mantissa bits of binary16 (bias 15), which maps subnormal codes onto fp16
// subnormals (Sec. 3.2's SHIFT/AND/OR restoration).  The factor 2^14 is applied in
// fp32 together with the row scale.
#ifndef AMS_LAYOUT_H_
#define AMS_LAYOUT_H_

#include <stdint.h>

namespace ams {

constexpr int kStripRows = 16;
constexpr int kLanes = 64;

// format numbers of the C ABI
constexpr int kFmtFp533 = 0, kFmtFp425 = 1, kFmtFp45 = 2, kFmtFp433 = 3, kFmtFp6 = 4, kFmtFp5 = 5, kFmtFp4 = 6, kNumFormats = 7;

struct FormatInfo {
  int group;        // weights sharing one last mantissa bit
  int code_bits;    // bits of a full code (sign + 2 exponent + mantissa)
  int rec_k;        // weights of one row inside a record
  int lane_k;       // weights of one lane chunk (rec_k / 4)
  int chunk_bytes;  // bytes of a lane chunk
  int side_bytes;   // bytes per lane behind the chunks
  int rec_bytes;    // bytes per record = 64 * (chunk_bytes + side_bytes)  (a unit is side_group records)
  int perm_block;   // operand slots and input channels are permuted inside blocks of this many weights
  double fmax;      // largest magnitude of the format
};

constexpr FormatInfo kFormats[kNumFormats] = {
    {3, 6, 96, 24, 16, 0, 1024, 24, 7.5},   // FP5.33-e2m3
    {4, 5, 128, 32, 16, 1, 1088, 8, 7.0},   // FP4.25-e2m2
    {2, 5, 128, 32, 16, 2, 1152, 16, 7.0},  // FP4.5-e2m2
    {3, 5, 96, 24, 12, 1, 832, 24, 7.0},    // FP4.33-e2m2
    {1, 6, 96, 24, 16, 2, 1152, 24, 7.5},   // FP6-e2m3
    {1, 5, 128, 32, 16, 4, 1280, 8, 7.0},   // FP5-e2m2
    {1, 4, 128, 32, 16, 0, 1024, 8, 6.0},   // FP4-e2m1
};

inline const FormatInfo* format_info(int fmt) { return fmt >= 0 && fmt < kNumFormats ? &kFormats[fmt] : nullptr; }

inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

// Records of a strip that share one block of side dwords (1 when the format has no side bits).
constexpr int side_group(const FormatInfo& f) { return f.side_bytes ? 4 / f.side_bytes : 1; }
constexpr int chunk_block_bytes(const FormatInfo& f) { return kLanes * f.chunk_bytes; }  // the lane chunks of one record
constexpr int unit_bytes(const FormatInfo& f) { return side_group(f) * chunk_block_bytes(f) + (f.side_bytes ? kLanes * 4 : 0); }

// Where record `rec` of strip `strip` lives in a packed matrix of n_strips strips: offset of its
// chunk block, offset of its unit's side dwords (lane l's dword at + 4 l), and the first bit of
// its side bits inside that dword.
struct RecordPlace {
  int64_t chunks, side;
  int side_shift;
};
inline RecordPlace record_place(const FormatInfo& f, int64_t n_strips, int64_t strip, int64_t rec) {
  const int sg = side_group(f);
  const int64_t unit = ((rec / sg) * n_strips + strip) * unit_bytes(f);
  const int sub = (int)(rec % sg);
  return {unit + (int64_t)sub * chunk_block_bytes(f), unit + (int64_t)sg * chunk_block_bytes(f), 8 * f.side_bytes * sub};
}
// bytes of a packed matrix: K is padded to whole side groups of records, N to whole strips
inline int64_t packed_bytes(const FormatInfo& f, int64_t N, int64_t K) {
  const int64_t n_rec = round_up(K, f.rec_k) / f.rec_k, sg = side_group(f);
  return (round_up(n_rec, sg) / sg) * (round_up(N, kStripRows) / kStripRows) * unit_bytes(f);
}

// Where weight j (0 .. lane_k-1, in input-channel order) of a lane chunk lives.
struct Place {
  int d, h, i;  // 32-bit word, half-word (0 = A), member inside the half-word
};
constexpr Place place(int fmt, int j) {
  switch (fmt) {
    case kFmtFp533:
    case kFmtFp6: return {j / 6, (j % 6) / 3, j % 3};
    case kFmtFp433: return {j % 3, (j / 3) / 4, (j / 3) % 4};
    case kFmtFp45: return {2 * (j / 16) + j % 2, ((j % 16) / 2) / 4, ((j % 16) / 2) % 4};
    default: return {j / 8, (j % 8) / 4, j % 4};  // FP4.25, FP5, FP4
  }
}

// Position of that weight in the lane's MFMA operand order (the activations are laid
// out in the same order): the restored pairs of a word come out as (A_i, B_i).
constexpr int operand_slot(int fmt, int j) {
  const Place p = place(fmt, j);
  return (fmt == kFmtFp533 || fmt == kFmtFp6) ? 2 * (3 * p.d + p.i) + p.h : 8 * p.d + 2 * p.i + p.h;
}

// The inverse inside one permutation block: input channel (relative to the block) of
// operand slot s (relative to the block).
constexpr int slot_channel(int fmt, int s) {
  const int pb = kFormats[fmt].perm_block;
  for (int j = 0; j < pb; j++)
    if (operand_slot(fmt, j) == s) return j;
  return -1;
}

// Bit of the lane's side bytes (taken as one little-endian integer) that holds the last
// mantissa bit of weight j, or -1 when it is kept in the half-word itself.
constexpr int side_bit(int fmt, int j) {
  const Place p = place(fmt, j);
  switch (fmt) {
    case kFmtFp425: return 4 * p.h + p.d;
    case kFmtFp433: return 4 * p.h + p.i;
    case kFmtFp45: return 8 * (p.d / 2) + 4 * p.h + p.i;
    case kFmtFp5: return 8 * p.d + 4 * p.h + p.i;
    case kFmtFp6: return p.i == 0 ? -1 : 8 * p.h + 2 * p.d + (p.i - 1);
    default: return -1;  // FP5.33: bit 12 of the half-word; FP4: there is none
  }
}

}  // namespace ams
#endif
