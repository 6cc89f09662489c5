// Host side of the AMS-Quant library: the offline quantizer (Sec. 3.1) and the
// packer into the gfx950 layout (Sec. 3.3 stage 1), plus the size queries.
// Compiled with -ffp-contract=off: the squared-error comparison of the adaptive
// search is specified as plain IEEE fp64 operations in member order.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <thread>
#include <vector>

#include "../../include/ams.h"
#include "ams_layout.h"

namespace {

using ams::FormatInfo;

// ---- binary16 <-> double -------------------------------------------------
inline double half_to_double(uint16_t h) {
  int s = h >> 15, e = (h >> 10) & 31, m = h & 1023;
  double v;
  if (e == 0)
    v = std::ldexp((double)m, -24);
  else if (e == 31)
    v = m ? NAN : INFINITY;
  else
    v = std::ldexp((double)(1024 + m), e - 25);
  return s ? -v : v;
}

// round-to-nearest-even conversion of a finite non-negative double
inline uint16_t double_to_half_bits(double a) {
  if (a == 0) return 0;
  int ex;
  (void)std::frexp(a, &ex);  // a = f * 2^ex, f in [0.5, 1)
  int e = ex - 1;            // a = 1.xxx * 2^e
  if (e < -14) e = -14;      // subnormal quantum 2^-24
  double q = std::nearbyint(std::ldexp(a, 10 - e));  // integer significand, RNE
  if (q >= 2048) {           // rounded up into the next binade
    q = 1024;
    e += 1;
  }
  if (e > 15) return 0x7C00;  // overflow to inf (cannot happen for absmax / Fmax)
  if (q < 1024) return (uint16_t)q;  // subnormal (or zero)
  return (uint16_t)(((e + 15) << 10) | ((int)q - 1024));
}

// ---- Sec. 2.2: magnitude of a magnitude code, bias 1 ----------------------
inline double magnitude(int mag_code, int mbits) {
  int e = mag_code >> mbits, m = mag_code & ((1 << mbits) - 1);
  if (e == 0) return std::ldexp((double)m, -mbits);
  return std::ldexp((double)((1 << mbits) + m), e - 1 - mbits);
}

// ---- Eq. 1: Round(t) = nearest magnitude, ties to the even code, saturating
inline int rtn_magnitude_code(double a, int mbits) {
  // the grid is uniform with step 2^-m below 2, 2^(1-m) in [2,4), 2^(2-m) from 4 on
  const int one = 1 << mbits;  // code of 1.0
  int sh = a < 2.0 ? 0 : (a < 4.0 ? 1 : 2);
  double r = std::nearbyint(std::ldexp(a, mbits - sh));  // round-half-even on the grid
  int code;
  if (sh == 0)
    code = (int)r;             // 0 .. 2*one
  else if (sh == 1)
    code = one + (int)r;       // r in [one, 2*one]
  else {
    if (r > 4.0 * one) r = 4.0 * one;  // keep the cast in range for huge inputs
    code = 2 * one + (int)r;   // r >= one
  }
  return std::min(code, 4 * one - 1);
}

// Re-rounding variant of the search (not in the paper): nearest magnitude among the codes
// that end in m0.  The candidates are walked in order; an exact tie between two
// neighbours goes to the one whose upper part (code >> 1) is even; inputs above the
// largest candidate land on it.
inline int reround_magnitude_code(double a, int mbits, int m0) {
  const int n_upper = 2 << mbits;  // 4 * 2^mbits magnitude codes, every other one
  int best = 0;
  double best_d = std::fabs(a - magnitude(m0, mbits));
  for (int j = 1; j < n_upper; j++) {
    const double d = std::fabs(a - magnitude(2 * j + m0, mbits));
    if (d < best_d || (d == best_d && (j & 1) == 0)) best = j, best_d = d;
  }
  return 2 * best + m0;
}

struct RowQuant {
  int mbits, group;
  double fmax;
  int search;  // AMS_SEARCH_*
};

// Quantize one row: scale (Eq. 1), RTN, adaptive search of each group's shared bit.
// Returns false on inf/NaN.
// Largest magnitude of a run of weights, or a negative number when one of them is inf or NaN.
double abs_max(const uint16_t* w, int64_t K) {
  double absmax = 0;
  for (int64_t k = 0; k < K; k++) {
    if (((w[k] >> 10) & 31) == 31) return -1.0;
    absmax = std::max(absmax, std::fabs(half_to_double(w[k])));
  }
  return absmax;
}

// Eq. 1: the fp16 scale for a given largest magnitude (1.0 where it would be zero)
uint16_t scale_bits(double absmax, double fmax) {
  const uint16_t sb = double_to_half_bits(absmax / fmax);
  return sb == 0 ? (uint16_t)0x3C00 : sb;
}

// forced_scale: 0 = the row's own scale (Eq. 1 per output channel), else the fp16 bits to use
bool quantize_row(const RowQuant& q, const uint16_t* w, int64_t K, uint8_t* codes, uint16_t* scale_out, uint16_t forced_scale = 0) {
  const double absmax = abs_max(w, K);
  if (absmax < 0) return false;
  const uint16_t sb = forced_scale ? forced_scale : scale_bits(absmax, q.fmax);
  *scale_out = sb;
  const double s = half_to_double(sb);
  const int sign_shift = 2 + q.mbits;
  for (int64_t k0 = 0; k0 < K; k0 += q.group) {
    const int n = (int)std::min<int64_t>(q.group, K - k0);
    int c[2][4];  // candidate codes of the members for shared bit 0 and 1
    double sse0 = 0, sse1 = 0;
    for (int i = 0; i < n; i++) {
      const double wv = half_to_double(w[k0 + i]);
      const double a = std::fabs(wv / s);
      int mc0, mc1;
      if (q.search == AMS_SEARCH_REROUND) {
        mc0 = reround_magnitude_code(a, q.mbits, 0);
        mc1 = reround_magnitude_code(a, q.mbits, 1);
      } else {  // Sec. 3.1: the RTN code with its last bit set to m0
        const int mc = rtn_magnitude_code(a, q.mbits);
        mc0 = mc & ~1;
        mc1 = mc | 1;
      }
      const int sign = (wv < 0 ? 1 : 0) << sign_shift;
      c[0][i] = mc0 | sign;
      c[1][i] = mc1 | sign;
      const double sg = wv < 0 ? -1.0 : 1.0;
      const double d0 = sg * magnitude(mc0, q.mbits) * s - wv;  // Eq. 2 with last bit 0
      const double d1 = sg * magnitude(mc1, q.mbits) * s - wv;  // ... with last bit 1
      sse0 = sse0 + d0 * d0;
      sse1 = sse1 + d1 * d1;
    }
    const int m0 = sse1 < sse0 ? 1 : 0;  // a tie keeps 0
    for (int i = 0; i < n; i++) codes[k0 + i] = (uint8_t)c[m0][i];
  }
  return true;
}

// ---- layout ---------------------------------------------------------------
inline bool is_e2m3(int fmt) { return fmt == ams::kFmtFp533 || fmt == ams::kFmtFp6; }

// Bit positions of member i's sign and magnitude inside a half-word, and the bit
// (or -1) of the half-word that holds a last mantissa bit.
inline int sign_pos(int fmt, int i) {
  if (is_e2m3(fmt)) return 15 - i;
  constexpr int pos[4] = {15, 12, 14, 13};
  return pos[i];
}
inline int mag_pos(int fmt, int i) { return is_e2m3(fmt) ? 8 - 4 * i : 9 - 3 * i; }

// Writes the records of strip t of a packed matrix of n_strips strips.  codes: 16 rows of K bytes
// (row pointer NULL = padding row).  Records beyond K that pad the last side group hold zero codes.
void pack_strip(int fmt, const FormatInfo& fi, const uint8_t* const rows[16], int64_t K, uint8_t* packed, int64_t n_strips, int64_t t) {
  const int64_t n_rec = ams::round_up(ams::round_up(K, fi.rec_k) / fi.rec_k, ams::side_group(fi));
  // FP4-e2m1 has no last bit beside its remainder: the nibble is the whole code
  const bool whole = fmt == ams::kFmtFp4;
  const int mag_bits = whole ? fi.code_bits - 1 : fi.code_bits - 2;  // bits of a remainder without its sign
  for (int64_t j = 0; j < n_rec; j++) {
    const ams::RecordPlace rp = ams::record_place(fi, n_strips, t, j);
    for (int l = 0; l < ams::kLanes; l++) {
      const uint8_t* row = rows[l & 15];
      const int64_t kbase = j * fi.rec_k + (int64_t)(l >> 4) * fi.lane_k;
      uint32_t words[4] = {0, 0, 0, 0};
      uint32_t side = 0;
      for (int q = 0; q < fi.lane_k; q++) {
        const int c = (row && kbase + q < K) ? row[kbase + q] : 0;  // padding is code 0
        const ams::Place p = ams::place(fmt, q);
        const uint32_t rem = whole ? (uint32_t)c : (uint32_t)c >> 1, lsb = whole ? 0u : (uint32_t)c & 1;
        uint32_t hw = (rem >> mag_bits) << sign_pos(fmt, p.i) | (rem & ((1u << mag_bits) - 1)) << mag_pos(fmt, p.i);
        const int sb = ams::side_bit(fmt, q);
        if (sb >= 0)
          side |= lsb << sb;  // members of a group agree (checked by the caller)
        else
          hw |= lsb << 12;
        words[p.d] |= hw << (16 * p.h);
      }
      std::memcpy(packed + rp.chunks + l * fi.chunk_bytes, words, (size_t)fi.chunk_bytes);
      // this record's bytes of the lane's side dword (little-endian); the other records of the group write theirs
      for (int b = 0; b < fi.side_bytes; b++) packed[rp.side + 4 * l + rp.side_shift / 8 + b] = (uint8_t)(side >> (8 * b));
    }
  }
}

void unpack_strip(int fmt, const FormatInfo& fi, const uint8_t* packed, int64_t n_strips, int64_t t, int64_t K, uint8_t* const rows[16]) {
  const int64_t n_rec = ams::round_up(K, fi.rec_k) / fi.rec_k;
  const bool whole = fmt == ams::kFmtFp4;
  const int mag_bits = whole ? fi.code_bits - 1 : fi.code_bits - 2;
  for (int64_t j = 0; j < n_rec; j++) {
    const ams::RecordPlace rp = ams::record_place(fi, n_strips, t, j);
    for (int l = 0; l < ams::kLanes; l++) {
      uint8_t* row = rows[l & 15];
      if (!row) continue;
      const int64_t kbase = j * fi.rec_k + (int64_t)(l >> 4) * fi.lane_k;
      uint32_t words[4] = {0, 0, 0, 0};
      std::memcpy(words, packed + rp.chunks + l * fi.chunk_bytes, (size_t)fi.chunk_bytes);
      uint32_t side = 0;
      for (int b = 0; b < fi.side_bytes; b++) side |= (uint32_t)packed[rp.side + 4 * l + rp.side_shift / 8 + b] << (8 * b);
      for (int q = 0; q < fi.lane_k; q++) {
        if (kbase + q >= K) continue;
        const ams::Place p = ams::place(fmt, q);
        const uint32_t hw = (words[p.d] >> (16 * p.h)) & 0xFFFF;
        const uint32_t rem = ((hw >> sign_pos(fmt, p.i)) & 1) << mag_bits | ((hw >> mag_pos(fmt, p.i)) & ((1u << mag_bits) - 1));
        const int sb = ams::side_bit(fmt, q);
        const uint32_t lsb = sb >= 0 ? (side >> sb) & 1 : (hw >> 12) & 1;
        row[kbase + q] = whole ? (uint8_t)rem : (uint8_t)(rem << 1 | lsb);
      }
    }
  }
}

int check_shape(int fmt, int64_t N, int64_t K) {
  if (!ams::format_info(fmt)) return AMS_ERR_FORMAT;
  if (N <= 0 || K <= 0 || N > (int64_t)1 << 24 || K > (int64_t)1 << 24) return AMS_ERR_SHAPE;
  return AMS_OK;
}

// Runs body(0 .. n-1) on up to 16 threads.  False when a body threw (the only thing these bodies can
// throw is std::bad_alloc from their row buffers); a thread that cannot be started just means fewer workers.
template <class F>
bool parallel_for(int64_t n, F&& body) {
  unsigned hw = std::thread::hardware_concurrency();
  int64_t nt = std::max<int64_t>(1, std::min<int64_t>({(int64_t)(hw ? hw : 1), (int64_t)16, n}));
  std::atomic<int64_t> next{0};
  std::atomic<int> failed{0};
  auto work = [&] {
    try {
      for (int64_t i; !failed.load() && (i = next.fetch_add(1)) < n;) body(i);
    } catch (...) {
      failed.store(1);
    }
  };
  std::vector<std::thread> th;
  try {
    th.reserve((size_t)nt);
    for (int64_t t = 1; t < nt; t++) th.emplace_back(work);
  } catch (...) {  // no more threads (or no memory for the list): the ones that exist, and this one, do the work
  }
  work();
  for (auto& t : th) t.join();
  return failed.load() == 0;
}

}  // namespace

extern "C" {

int ams_version(void) { return 200; }

const char* ams_strerror(int code) {
  switch (code) {
    case AMS_OK: return "ok";
    case AMS_ERR_FORMAT: return "unknown format";
    case AMS_ERR_SHAPE: return "shape or argument out of range";
    case AMS_ERR_NULL: return "null pointer";
    case AMS_ERR_ALIGN: return "device pointer not 16-byte aligned";
    case AMS_ERR_NONFINITE: return "weight is inf or NaN";
    case AMS_ERR_LAUNCH: return "kernel launch failed";
    case AMS_ERR_DEVICE: return "current device is not gfx950";
    case AMS_ERR_SCRATCH: return "problem too large for the library's static scratch (use ams_linear or ams_linear_ws)";
    case AMS_ERR_NOMEM: return "out of host memory";
    default: return "unknown error";
  }
}

int ams_group_size(int fmt) {
  const FormatInfo* fi = ams::format_info(fmt);
  return fi ? fi->group : 0;
}

int ams_code_bits(int fmt) {
  const FormatInfo* fi = ams::format_info(fmt);
  return fi ? fi->code_bits : 0;
}

int ams_packed_bytes(int fmt, int64_t N, int64_t K, size_t* bytes) {
  if (int rc = check_shape(fmt, N, K)) return rc;
  if (!bytes) return AMS_ERR_NULL;
  const FormatInfo& fi = *ams::format_info(fmt);
  *bytes = (size_t)ams::packed_bytes(fi, N, K);
  return AMS_OK;
}

int ams_canonical_bytes(int fmt, int64_t N, int64_t K, size_t* bytes) {
  if (int rc = check_shape(fmt, N, K)) return rc;
  if (!bytes) return AMS_ERR_NULL;
  switch (fmt) {
    case AMS_FMT_FP533_E2M3: *bytes = (size_t)2 * (size_t)((K + 2) / 3) * (size_t)N; break;     // one uint16 per 3 weights
    case AMS_FMT_FP425_E2M2: *bytes = (size_t)34 * (size_t)((K + 63) / 64) * (size_t)N; break;  // 17 uint16 per 64 weights
    case AMS_FMT_FP45_E2M2: *bytes = (size_t)9 * (size_t)((K + 15) / 16) * (size_t)N; break;    // 16 nibbles + 8 shared bits
    case AMS_FMT_FP433_E2M2: *bytes = (size_t)13 * (size_t)((K + 23) / 24) * (size_t)N; break;  // 24 nibbles + 8 shared bits
    case AMS_FMT_FP6_E2M3: *bytes = (size_t)3 * (size_t)((K + 3) / 4) * (size_t)N; break;       // 4 codes of 6 bits
    case AMS_FMT_FP5_E2M2: *bytes = (size_t)5 * (size_t)((K + 7) / 8) * (size_t)N; break;       // 8 codes of 5 bits
    default: *bytes = (size_t)((K + 1) / 2) * (size_t)N; break;                                 // FP4: 2 codes per byte
  }
  return AMS_OK;
}

int ams_pack(int fmt, const uint16_t* W, int64_t N, int64_t K, int64_t ldw, void* packed, uint16_t* scales,
             uint8_t* codes_out) {
  return ams_pack_ex(fmt, AMS_SEARCH_SET_BIT, W, N, K, ldw, packed, scales, codes_out);
}

namespace {
int pack_rows(int fmt, int search, bool per_tensor, const uint16_t* W, int64_t N, int64_t K, int64_t ldw, void* packed,
              uint16_t* scales, uint8_t* codes_out);
}

int ams_pack_ex(int fmt, int search, const uint16_t* W, int64_t N, int64_t K, int64_t ldw, void* packed, uint16_t* scales,
                uint8_t* codes_out) {
  return pack_rows(fmt, search, false, W, N, K, ldw, packed, scales, codes_out);
}

int ams_pack_per_tensor(int fmt, int search, const uint16_t* W, int64_t N, int64_t K, int64_t ldw, void* packed,
                        uint16_t* scales, uint8_t* codes_out) {
  return pack_rows(fmt, search, true, W, N, K, ldw, packed, scales, codes_out);
}

namespace {
int pack_rows(int fmt, int search, bool per_tensor, const uint16_t* W, int64_t N, int64_t K, int64_t ldw, void* packed,
              uint16_t* scales, uint8_t* codes_out) {
  if (int rc = check_shape(fmt, N, K)) return rc;
  if (search != AMS_SEARCH_SET_BIT && search != AMS_SEARCH_REROUND) return AMS_ERR_SHAPE;
  if (!W || !packed || !scales) return AMS_ERR_NULL;
  if (ldw < K) return AMS_ERR_SHAPE;
  const FormatInfo& fi = *ams::format_info(fmt);
  const RowQuant rq = {fi.code_bits - 3, fi.group, fi.fmax, search};
  const int64_t n_strips = ams::round_up(N, ams::kStripRows) / ams::kStripRows;
  uint16_t tensor_scale = 0;
  if (per_tensor) {  // Eq. 1 with the maximum over the whole matrix
    double absmax = 0;
    for (int64_t n = 0; n < N; n++) {
      const double m = abs_max(W + n * ldw, K);
      if (m < 0) return AMS_ERR_NONFINITE;
      absmax = std::max(absmax, m);
    }
    tensor_scale = scale_bits(absmax, fi.fmax);
  }
  std::atomic<int> bad{0};
  const bool done = parallel_for(n_strips, [&](int64_t t) {
    std::vector<uint8_t> buf((size_t)ams::kStripRows * K);
    const uint8_t* rows[16];
    for (int r = 0; r < 16; r++) {
      const int64_t n = t * 16 + r;
      if (n >= N) {
        rows[r] = nullptr;
        continue;
      }
      uint8_t* c = buf.data() + (size_t)r * K;
      if (!quantize_row(rq, W + n * ldw, K, c, scales + n, tensor_scale)) bad.store(1);
      rows[r] = c;
      if (codes_out) std::memcpy(codes_out + n * K, c, (size_t)K);
    }
    pack_strip(fmt, fi, rows, K, (uint8_t*)packed, n_strips, t);
  });
  if (!done) return AMS_ERR_NOMEM;
  return bad.load() ? AMS_ERR_NONFINITE : AMS_OK;
}
}  // namespace

// log2(scale_group / rec_k), or -1 when scale_group is not rec_k * 2^j
int scale_group_shift(const FormatInfo& fi, int64_t scale_group) {
  for (int j = 0; j < 20; j++)
    if (scale_group == (int64_t)fi.rec_k << j) return j;
  return -1;
}

int ams_group_scales_count(int fmt, int64_t N, int64_t K, int64_t scale_group, size_t* count) {
  if (int rc = check_shape(fmt, N, K)) return rc;
  if (!count) return AMS_ERR_NULL;
  const FormatInfo& fi = *ams::format_info(fmt);
  if (scale_group_shift(fi, scale_group) < 0) return AMS_ERR_SHAPE;
  *count = (size_t)(ams::round_up(N, ams::kStripRows)) * (size_t)((K + scale_group - 1) / scale_group);
  return AMS_OK;
}

int ams_pack_grouped(int fmt, int search, int64_t scale_group, const uint16_t* W, int64_t N, int64_t K, int64_t ldw,
                     void* packed, uint16_t* scales, uint8_t* codes_out) {
  if (int rc = check_shape(fmt, N, K)) return rc;
  if (search != AMS_SEARCH_SET_BIT && search != AMS_SEARCH_REROUND) return AMS_ERR_SHAPE;
  if (!W || !packed || !scales) return AMS_ERR_NULL;
  if (ldw < K) return AMS_ERR_SHAPE;
  const FormatInfo& fi = *ams::format_info(fmt);
  if (scale_group_shift(fi, scale_group) < 0) return AMS_ERR_SHAPE;
  const RowQuant rq = {fi.code_bits - 3, fi.group, fi.fmax, search};
  const int64_t n_strips = ams::round_up(N, ams::kStripRows) / ams::kStripRows;
  const int64_t n_sg = (K + scale_group - 1) / scale_group;
  std::atomic<int> bad{0};
  const bool done = parallel_for(n_strips, [&](int64_t t) {
    std::vector<uint8_t> buf((size_t)ams::kStripRows * K);
    const uint8_t* rows[16];
    for (int r = 0; r < 16; r++) {
      const int64_t n = t * 16 + r;
      uint16_t* srow = scales + (size_t)t * n_sg * 16 + r;  // [strip][run][row in strip]
      if (n >= N) {
        rows[r] = nullptr;
        for (int64_t j = 0; j < n_sg; j++) srow[j * 16] = 0x3C00;  // padding rows: 1.0
        continue;
      }
      uint8_t* c = buf.data() + (size_t)r * K;
      for (int64_t j = 0; j < n_sg; j++) {  // Eq. 1 and the search on every run by itself
        const int64_t a = j * scale_group, len = std::min<int64_t>(scale_group, K - a);
        if (!quantize_row(rq, W + n * ldw + a, len, c + a, srow + j * 16)) bad.store(1);
      }
      rows[r] = c;
      if (codes_out) std::memcpy(codes_out + n * K, c, (size_t)K);
    }
    pack_strip(fmt, fi, rows, K, (uint8_t*)packed, n_strips, t);
  });
  if (!done) return AMS_ERR_NOMEM;
  return bad.load() ? AMS_ERR_NONFINITE : AMS_OK;
}

int ams_pack_codes(int fmt, const uint8_t* codes, int64_t N, int64_t K, void* packed) {
  if (int rc = check_shape(fmt, N, K)) return rc;
  if (!codes || !packed) return AMS_ERR_NULL;
  const FormatInfo& fi = *ams::format_info(fmt);
  const int64_t n_strips = ams::round_up(N, ams::kStripRows) / ams::kStripRows;
  std::atomic<int> bad{0};
  parallel_for(n_strips, [&](int64_t t) {
    const uint8_t* rows[16];
    for (int r = 0; r < 16; r++) {
      const int64_t n = t * 16 + r;
      rows[r] = n < N ? codes + n * K : nullptr;
      if (n >= N) continue;
      for (int64_t k0 = 0; k0 < K; k0 += fi.group) {
        const int64_t k1 = std::min<int64_t>(K, k0 + fi.group);
        for (int64_t k = k0; k < k1; k++)
          if ((rows[r][k] >> fi.code_bits) || ((rows[r][k] ^ rows[r][k0]) & 1)) bad.store(1);
      }
    }
    pack_strip(fmt, fi, rows, K, (uint8_t*)packed, n_strips, t);
  });
  return bad.load() ? AMS_ERR_SHAPE : AMS_OK;
}

int ams_unpack_host(int fmt, const void* packed, int64_t N, int64_t K, uint8_t* codes) {
  if (int rc = check_shape(fmt, N, K)) return rc;
  if (!codes || !packed) return AMS_ERR_NULL;
  const FormatInfo& fi = *ams::format_info(fmt);
  const int64_t n_strips = ams::round_up(N, ams::kStripRows) / ams::kStripRows;
  parallel_for(n_strips, [&](int64_t t) {
    uint8_t* rows[16];
    for (int r = 0; r < 16; r++) rows[r] = t * 16 + r < N ? codes + (t * 16 + r) * K : nullptr;
    unpack_strip(fmt, fi, (const uint8_t*)packed, n_strips, t, K, rows);
  });
  return AMS_OK;
}

}  // extern "C"
