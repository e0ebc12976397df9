// Host-side table construction for the quantizers of Section 3.5 (see stq_tables.h).
#include "stq_tables.h"

#include <cmath>
#include <cstring>

namespace stq {

static inline uint32_t f2u(float f) { uint32_t u; std::memcpy(&u, &f, 4); return u; }

// One table serves every width: level k of width b is 2^(-k * 2^(4-b)) = G[k << (9-b)] and the
// decision threshold between levels k and k+1 (their geometric mean) is G[(2k+1) << (8-b)].
float table_G(int j) { return static_cast<float>(std::exp2(-static_cast<double>(j) / 32.0)); }

float table_R(int b, int u) {
  const int qmax = (1 << (b - 1)) - 1;
  // quotient of two small integers: the double quotient rounds to the same fp32 as the exact one
  return static_cast<float>(static_cast<double>(u - qmax) / static_cast<double>(qmax));
}

float table_L(int b, int c) { return table_G((((1 << b) - 1) - c) << (9 - b)); }

float table_T(int b, int k) { return table_G((2 * k + 1) << (8 - b)); }

bool build_table_image(std::vector<uint32_t>& img) {
  img.assign(kTabWords, 0u);
  for (int b = kMinBits; b <= kMaxBits; ++b) {
    const int qmax = (1 << (b - 1)) - 1, kmax = (1 << b) - 1;
    for (int u = 0; u <= 2 * qmax; ++u) img[kTabROff + (1 << b) + u] = f2u(table_R(b, u));
    for (int c = 0; c <= kmax; ++c) img[kTabLOff + (1 << b) + c] = f2u(table_L(b, c));
    // thresholds as bit patterns; positive floats order like their bit patterns
    std::vector<uint32_t> tb(kmax);
    for (int k = 0; k < kmax; ++k) tb[k] = f2u(table_T(b, k));
    uint32_t* vq = &img[kTabVqOff + (b - 2) * kVqBuckets * 2];
    for (int idx = 0; idx < kVqBuckets; ++idx) {
      const bool last = idx == 0;  // the catch-all bucket below the lowest threshold
      const uint64_t lo = last ? 0 : (static_cast<uint64_t>(kVqLow + idx) << kVqShift);
      const uint64_t hi = idx == kVqBuckets - 1 ? (1ull << 32) : (static_cast<uint64_t>(kVqLow + idx + 1) << kVqShift);
      uint32_t base = 0, thr = 0xFFFFFFFFu;
      int inside = 0;
      for (int k = 0; k < kmax; ++k) {
        if (tb[k] < lo) ++base;
        else if (tb[k] < hi) { thr = tb[k]; ++inside; }
      }
      if (inside > 1 || (last && inside != 0)) return false;
      vq[2 * idx] = thr;     // code = base + (bits >= thr) = number of thresholds <= bits
      vq[2 * idx + 1] = base;
    }
  }
  return true;
}

void build_repack_lut(int state, int b_old, int b_new, uint8_t* out) {
  std::memset(out, 0, 256);
  if (state == 0) {
    const int qo = (1 << (b_old - 1)) - 1, qn = (1 << (b_new - 1)) - 1;
    for (int u = 0; u <= 2 * qo; ++u) {
      const float t = table_R(b_old, u) * static_cast<float>(qn);
      float r = std::nearbyintf(t);  // half to even in the default rounding mode
      if (r > static_cast<float>(qn)) r = static_cast<float>(qn);
      if (r < -static_cast<float>(qn)) r = -static_cast<float>(qn);
      out[u] = static_cast<uint8_t>(static_cast<int>(r) + qn);
    }
  } else {
    const int ko = (1 << b_old) - 1, kn = (1 << b_new) - 1;
    for (int c = 0; c <= ko; ++c) {
      const float rho = table_L(b_old, c);
      int code = 0;  // number of new thresholds at or below the old level's value
      for (int k = 0; k < kn; ++k) if (rho >= table_T(b_new, k)) ++code;
      out[c] = static_cast<uint8_t>(code);
    }
  }
}

}  // namespace stq
