// The signed 8-bit dynamic code of the blockwise codec, built at compile time.
//
// "Compression techniques", item 1 (dynamic blockwise quantization).  A magnitude is
// 10^-e (0.1 + 0.9 (j + 1/2) / 2^f) with e = 0..6, f = 6 - e, j = 0..2^f - 1; over a common
// denominator that is the ratio of the integers 2^(f+1) + 9 (2j + 1) and 10^(e+1) 2^(f+1),
// evaluated as one double division and rounded once to float.  The table is the negated
// magnitudes, 0, the magnitudes and +1.0: 256 ascending floats.  Mid[j] is the float nearest
// to the mean of T[j] and T[j+1] (formed exactly in double).
//
// Encoding counts the midpoints strictly below a value v.  By the mirror symmetry of the first
// 255 entries this is
//     v >= +0 : 127 + #{ i in 0..127 : |v| >  P[i] }
//     v <  -0 : 127 - #{ i in 0..126 : |v| >= P[i] }          with P[i] = Mid[127 + i] > 0,
// and, positive floats being ordered like their bit patterns, both counts become
// "bits(|v|) + (v negative) > bits(P[i])" on integers (capped at 127 for negatives).
// The count is looked up rather than searched: the 14 leading bits of a positive float (8
// exponent bits, 6 mantissa bits) select a cell, and no cell holds more than one P[i] (checked
// at compile time), so  count = base[cell] + (bits > threshold[cell]).
#pragma once
#include <stdint.h>

namespace mmd8 {

constexpr int kCellShift = 17;                    // 32 - 1 sign bit - 14 index bits
constexpr uint32_t kNoThreshold = 0xffffffffu;    // compares greater than every bit pattern

struct CodeCell {
  uint32_t threshold;   // bits(P[i]) of the midpoint inside the cell, or kNoThreshold
  uint32_t base;        // number of midpoints below the cell
};

struct DynamicCode {
  static constexpr int kCellLo = 6728;            // one below the cell of P[0]
  static constexpr int kCellHi = 8128;            // cell of 1.0f: every P[i] lies below it
  static constexpr int kCells = kCellHi - kCellLo + 1;

  float T[256];
  float Mid[255];
  CodeCell cell[kCells];
  bool one_midpoint_per_cell;
};

constexpr DynamicCode make_dynamic_code() {
  DynamicCode d{};
  float mag[127] = {};
  int n = 0;
  for (int e = 6; e >= 0; --e) {
    const int f = 6 - e;
    long long den = 1;
    for (int i = 0; i <= e; ++i) den *= 10;
    den <<= (f + 1);
    for (int j = 0; j < (1 << f); ++j) {
      const long long num = (1ll << (f + 1)) + 9ll * (2 * j + 1);
      mag[n++] = (float)((double)num / (double)den);
    }
  }
  for (int i = 0; i < 127; ++i) {
    d.T[126 - i] = -mag[i];
    d.T[128 + i] = mag[i];
  }
  d.T[127] = 0.0f;
  d.T[255] = 1.0f;
  for (int j = 0; j < 255; ++j) d.Mid[j] = (float)(((double)d.T[j] + (double)d.T[j + 1]) / 2.0);

  d.one_midpoint_per_cell = true;
  for (int c = 0; c < DynamicCode::kCells; ++c) d.cell[c] = CodeCell{kNoThreshold, 0};
  uint32_t count_in_cell[DynamicCode::kCells] = {};
  for (int i = 0; i < 128; ++i) {
    const uint32_t bits = __builtin_bit_cast(uint32_t, d.Mid[127 + i]);
    const int c = (int)(bits >> kCellShift) - DynamicCode::kCellLo;
    if (c <= 0 || c >= DynamicCode::kCells - 1 || count_in_cell[c] != 0) d.one_midpoint_per_cell = false;
    if (c > 0 && c < DynamicCode::kCells - 1) {
      count_in_cell[c] += 1;
      d.cell[c].threshold = bits;
    }
  }
  uint32_t below = 0;
  for (int c = 0; c < DynamicCode::kCells; ++c) {
    d.cell[c].base = below;
    below += count_in_cell[c];
  }
  if (below != 128) d.one_midpoint_per_cell = false;
  return d;
}

}  // namespace mmd8
