// Constant tables of the LLVQ dequantiser: layout shared by the host-side builder
// (llvq_tables.cpp) and the gfx950 kernels (llvq_kernels.hip).
//
// The dequantiser of the paper's App. A needs, per index: shell/class lookup in cumulative tables,
// the unflattening of the class-local index into (r, s, I''), and a "local combinatorial
// reconstruction".  Here every one of these steps is a lookup in a small table held in LDS:
//   gs      4096 Golay words ordered by (weight, message)                      [paper Sec. 2.3]
//   bucket  top bits of the index -> first candidate class                      [App. A steps 1-2]
//   cls_off cumulative class offsets; cls: one ClassRec per class               [App. A steps 2-3]
//   split   ranking tables of the q-subsets of n slots (12 low + n-12 high)     [App. A step 4]
//   lut12   colex rank -> 12-bit mask, grouped by popcount
//   inner   rank of an arrangement of the minority values -> two bit planes
//   pdep6   deposit of <=6 compressed bits into a 6-bit mask
//   spread6 the same deposit, result spread to one nibble per position
#pragma once
#include <cstdint>
#include <vector>

namespace llvq {

struct alignas(16) ClassRec {
    double   invPP;      // 1/(P1*Pin), nudged upwards so that floor(x*invPP) == x / PP for x < 2^48
    uint32_t PP;         // P1 * Pin
    float    invP1;      // 1/P1 rounded up (exact quotients for dividends < 2^22)
    uint32_t f0;         // bit fields, see F0_* below
    uint32_t f1;         // bit fields, see F1_* below
    uint16_t P1;         // arrangements of the direct F1 word (1 when there is none)
    uint16_t tb1;        // first entry of the direct F1 word's table in `inner`
    uint16_t tb0;        // first entry of the outer domain's inner-word table in `inner`
    uint16_t sp;         // split entry of j is split[sp + j]
    uint32_t vt8_lo, vt8_hi;   // value of code 0..7 as fp8 e4m3 bytes (sign bit = bit 7)
    uint32_t vti_lo, vti_hi;   // value of code 0..7 as int8
};
static_assert(sizeof(ClassRec) == 48, "ClassRec layout");

// f0: [0] odd  [1] f1_direct (even class, 0 < w <= 16: F1 planes go through the codeword)
//     [2] outer_all (outer domain = all 24 positions: odd classes and w = 24)
//     [3..7] wm1 = max(w-1,0)  [8] forced-sign enable  [9] kappa (parity of negative F1 signs)
//     [10..14] B  [15..18] m  [19..23] n (slots of the outer domain)  [24..28] q (subset size)
enum { F0_ODD = 0, F0_F1DIRECT = 1, F0_OUTER_ALL = 2, F0_WM1 = 3, F0_FEN = 8, F0_KAPPA = 9,
       F0_B = 10, F0_M = 15, F0_N = 19, F0_Q = 24 };
// f1: [0..11] first Golay word of the class in gs  [12..13] code of A  [14..18] guess shift
//     [19..22] jmax  [23..28] row of the guess table
enum { F1_GOFF = 0, F1_ACODE = 12, F1_GSHIFT = 14, F1_JMAX = 19, F1_GROW = 23 };

struct alignas(16) SplitEnt {
    uint32_t base;       // number of subsets with fewer high slots
    float    inv;        // 1 / C(nl, q-j), rounded up
    uint16_t div;        // C(nl, q-j)
    uint16_t b12lo;      // lut12 base of popcount q-j
    uint16_t b12hi;      // lut12 base of popcount j
    uint16_t pad;
};
static_assert(sizeof(SplitEnt) == 16, "SplitEnt layout");

// Fixed byte offsets of the tables inside the blob (and inside LDS, where kernels copy the blob verbatim).
// They are compile-time constants so that the kernels can fold them into the offset field of the LDS
// instructions; the small, frequently read tables sit below 64 KB, the reach of that field.
constexpr uint32_t kOffGs      = 0;        // 4096 x u32
constexpr uint32_t kOffSpread6 = 16384;    // 4096 x u32
constexpr uint32_t kOffPdep6   = 32768;    // 4096 x u8
constexpr uint32_t kOffLut12   = 36864;    // 4096 x u16
constexpr uint32_t kOffBucket  = 45056;    // 4096 x u16
constexpr uint32_t kOffGuess   = 53248;    // up to 48 rows x 64 x u8
constexpr uint32_t kOffAtab    = 56320;    // 4 x {A, 1/A} doubles
constexpr uint32_t kOffClsOff  = 56384;    // (ncls + 1) x u64, ncls <= 383
constexpr uint32_t kOffRnorm   = 59456;    // 16 x float: 1/sqrt(16 m)
constexpr uint32_t kOffSplit   = 59520;    // up to 352 x SplitEnt
constexpr uint32_t kOffCls     = 65152;    // ncls x ClassRec
constexpr uint32_t kOffInner   = 83552;    // inner-word planes, u32
constexpr uint32_t kMaxBlob    = 162816;   // 159 KB; the last KB of the 160 KB of LDS is kernel scratch
constexpr uint32_t kBucketShift = 36;      // bucket index = I >> 36 (4096 buckets cover 48 bits)
constexpr uint32_t kGuessBuckets = 64;     // buckets of the subset-split guess table per (n, q)

struct TableLayout {
    uint32_t lds_bytes;      // bytes of the blob = bytes resident in LDS
    uint32_t ncls;
    uint32_t inner_entries;
    uint32_t pad;
    uint64_t npoints;        // N(m_max)
    float    rnorm[16];      // 1/sqrt(16 m)
};

// nibble slot (0..7) of chunk position 0..5 inside a spread6 entry
static constexpr int kNibbleSlot[6] = {0, 2, 1, 3, 4, 6};

struct Tables {
    TableLayout lay;
    uint64_t shell_off[16];  // index of the first point of shell m (N(m-1)); entries above m_max hold N(m_max)
    std::vector<unsigned char> blob;
};

// Builds every table for Lambda_24(m_max), 2 <= m_max <= 13.  Returns false on an internal inconsistency.
bool build_tables(int m_max, Tables& out);

}  // namespace llvq
