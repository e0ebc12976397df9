// Host-side tables of the two block quantizers (Section 3.5 of the paper: linear
// symmetric codes for the first moment, logarithmic codes for the second) in the
// form the gfx950 kernels consume.  Pure host code, no HIP.
#pragma once
#include <cstdint>
#include <vector>

namespace stq {

constexpr int kGLen = 511;    // G[j] = fl32(2^(-j/32)), j = 0..510
constexpr int kMinBits = 2;
constexpr int kMaxBits = 8;

// Second-moment quantizer as a bucketed search over the bit pattern of
// rho = v / blockmax in (0, 1]:  bucket = max((bits(rho) >> kVqShift) - kVqLow, 0)  (one saturating
// subtraction), code = entry.base + (bits(rho) >= entry.thr).  Bucket width 2^18 ulps keeps at most
// one threshold per bucket for every width up to 8 bits.
constexpr int kVqShift = 18;
constexpr uint32_t kVqTop = 0x3F800000u >> kVqShift;  // the last bucket holds rho >= 1
constexpr int kVqBuckets = 514;                       // everything below + 16 octaves x 32 + the last
constexpr uint32_t kVqLow = kVqTop - (kVqBuckets - 1);
struct VqEntry { uint32_t thr; uint32_t base; };

// Offsets (in 32-bit words) inside the table image that stq_init uploads and every
// workgroup copies to LDS.
// R_b and L_b start at word (1<<b) of their 512-word regions, so that a code index can be OR-ed
// onto the table's base.
constexpr int kTabROff = 0;     // R_b[u] at kTabROff + (1<<b) + u
constexpr int kTabLOff = 512;   // L_b[c] at kTabLOff + (1<<b) + c
constexpr int kTabVqOff = 1024; // VqEntry table of width b at kTabVqOff + (b-2)*kVqBuckets*2
constexpr int kTabWords = kTabVqOff + 7 * kVqBuckets * 2;

float table_G(int j);
float table_R(int b, int u);  // value of first-moment code u at scale 1
float table_L(int b, int c);  // value of second-moment code c at scale 1
float table_T(int b, int k);  // threshold between second-moment levels k and k+1 at scale 1

// Fills `img` (kTabWords words).  Returns false if some bucket would hold two thresholds.
bool build_table_image(std::vector<uint32_t>& img);

// Code-domain conversion tables for a width change (scale of the block unchanged).
// state 0: first moment, 1: second moment.  out has 256 entries.
void build_repack_lut(int state, int b_old, int b_new, uint8_t* out);

}  // namespace stq
