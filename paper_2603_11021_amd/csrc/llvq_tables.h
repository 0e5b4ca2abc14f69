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

// Fixed byte offsets of the tables inside the blob.  The first kLdsBytes of the blob are copied verbatim into LDS
// by every kernel; the offsets are compile-time constants so that the kernels can fold them into the offset field
// of the LDS instructions.  The two large tables that are read once or twice per block (the sorted Golay words and
// the inner-word planes) come last: a kernel either copies the whole blob into LDS or only the first kLdsBytes and
// reads those two through the vector L1/L2 (a shorter table copy per launch, at the price of three global gathers
// per block).
constexpr uint32_t kSpreadPitch = 65;      // dwords per mask row of spread6: entry (F, m) at F * 65 + m, so that equal m of
                                           // different masks (all-zero sources are frequent) fall into different LDS banks
constexpr uint32_t kPdepPitch  = 68;       // bytes per mask row of pdep6 (17 dwords, for the same reason)
constexpr uint32_t kOffSpread6 = 0;        // 64 x 65 x u32
constexpr uint32_t kOffPdep6   = 16640;    // 64 x 68 x u8
constexpr uint32_t kOffLut12   = 20992;    // 4096 x u16
constexpr uint32_t kOffBucket  = 29184;    // 4096 x u16: 8 x class id (the byte offset of its entry in cls_off)
constexpr uint32_t kOffGuess   = 37376;    // up to 48 rows x 64 x u8
constexpr uint32_t kOffAtab    = 40448;    // 4 x {A, 1/A} doubles
constexpr uint32_t kOffClsOff  = 40512;    // (ncls + 4) x u64, ncls <= 383: offsets, N, and three entries above every index
constexpr uint32_t kOffRnorm   = 43616;    // 16 x float: 1/sqrt(16 m)
constexpr uint32_t kOffSplit   = 43680;    // up to 352 x SplitEnt
constexpr uint32_t kOffCls     = 49312;    // ncls x ClassRec
constexpr uint32_t kLdsBytes   = 67712;    // end of the LDS-resident part
constexpr uint32_t kOffGs      = 67712;    // 4096 x u32 (global memory)
constexpr uint32_t kOffInner   = 84096;    // inner-word planes, u32 (global memory)
constexpr uint32_t kMaxBlob    = 84096 + 4 * 65536;   // the inner-word table bases are 16-bit entry numbers
constexpr uint32_t kBucketShift = 36;      // bucket index = I >> 36 (4096 buckets cover 48 bits)
constexpr uint32_t kGuessBuckets = 64;     // buckets of the subset-split guess table per (n, q)

struct TableLayout {
    uint32_t lds_bytes;      // first part of the blob: the tables every kernel keeps in LDS
    uint32_t blob_bytes;     // the whole blob (kernels that want all tables in LDS copy this many bytes)
    uint32_t ncls;
    uint32_t inner_entries;
    uint64_t npoints;        // N(m_max)
};

// ---- tables of the encoder-side index map (point -> index), a blob of their own ---------------------
// One record per class, in class order.  The point's class is found by hashing the key below; the code of each
// coordinate (the same nibble codes the decoder produces) comes from an 8-entry table indexed by |x| >> 1.
struct alignas(16) EncRec {
    uint64_t offset;            // index of the first point of the class
    uint32_t key;               // sum |x|^4  |  (sum |x|) << 20  |  parity << 29: identifies the leader
    uint32_t f0;                // the bit fields of ClassRec::f0
    uint32_t ctab_lo, ctab_hi;  // nibble code of the absolute value 2k (even classes) or 2k+1 (odd), k = 0..7
    uint32_t Pin;               // arrangements of the inner word of the outer domain
    uint32_t e1;                // bit fields, see E1_* below
    uint16_t P1;                // arrangements of the direct F1 word
    uint16_t sp;                // split entry of j is split[sp + j]
    uint16_t rad0[2];           // radices of the first two digits of the outer domain's inner word
    uint16_t rad1[2];           // the same for the direct F1 word
    uint32_t pad;
};
static_assert(sizeof(EncRec) == 48, "EncRec layout");
// e1: [0..11] first Golay word of the class in gs  [12..13] code of A  [14..15] digits of the outer inner word
//     [16..17] digits of the direct F1 word  [18] first symbol of the outer inner word (0 or 1)
enum { E1_GOFF = 0, E1_ACODE = 12, E1_DIG0 = 14, E1_DIG1 = 16, E1_SYM0 = 18 };

constexpr uint32_t kEncGs     = 0;        // 4096 x u32, the decoder's sorted Golay words
constexpr uint32_t kEncGinv   = 16384;    // 4096 x u16: low 12 bits of a word -> its position in gs
constexpr uint32_t kEncRank12 = 24576;    // 4096 x u16: colex rank of a 12-bit mask among the masks of its popcount
constexpr uint32_t kEncPext6  = 32768;    // 4096 x u8: extraction of the bits of a 6-bit source under a 6-bit mask
constexpr uint32_t kEncHash   = 36864;    // 2 x 512 x HashEnt: cuckoo table of the class keys
constexpr uint32_t kEncG16    = 45056;    // 16 x 17 x u16: masks of popcount p whose bits 12..15 are below H
constexpr uint32_t kEncSplit  = 46080;    // the decoder's SplitEnt array
constexpr uint32_t kEncCls    = 51712;    // ncls x EncRec
constexpr uint32_t kEncBlob   = 70144;    // 68.5 KB
constexpr uint32_t kEncHashBits = 9;      // slots per half of the cuckoo table

// a key sits in slot (key * mult[h]) >> (32 - kEncHashBits) of half h, for h = 0 or h = 1
struct HashEnt {
    uint32_t key;     // 0xFFFFFFFF: empty
    uint32_t cid;
};

struct EncLayout {
    uint32_t bytes;          // bytes of the encoder blob = bytes resident in LDS
    uint32_t ncls;
    uint32_t hash_mult[2];   // multipliers of the two halves of the cuckoo table
    uint32_t m_max;
};

// ---- tables of the nearest-point search: one record per class, read with wave-uniform (scalar) loads ----
// coef: the 24 coefficients the sorted input is multiplied with.  Odd class: +a for a = 1 (mod 4), -a for
// a = 3 (mod 4), in descending order.  Even class: the 2-mod-4 values in descending order (w of them), then the
// 0-mod-4 values in descending order.
struct alignas(128) SearchRec {
    float    coef[24];
    float    mul[2];     // score = <w, x> * mul[metric] + bias[metric]: {1 / sqrt(16 m), 1}
    float    bias[2];    //                                              {0, -||x||^2 / 2 = -8 m}
    float    amin2;      // twice the smallest 2-mod-4 value (0 when there is none): cost factor of the parity repair
    uint32_t kappa;      // parity that the number of negative F1 signs must have
    uint32_t cid;        // class id
    uint32_t w;          // Golay weight of the class (odd classes: 0)
};
static_assert(sizeof(SearchRec) == 128, "SearchRec layout");

// records are ordered: all odd classes, then the even classes grouped by weight 0, 8, 12, 16, 24
constexpr int kMaxSearchTiles = 16;
struct SearchLayout {
    uint32_t n_odd;
    uint32_t even_first[5];
    uint32_t even_count[5];
    uint32_t total;
    // the same records cut into tiles of 32 classes for the matrix cores; group 0 = odd, 1..5 = even weights 0, 8, 12, 16, 24
    uint32_t n_tiles;
    uint32_t grp_tile_first[6];
    uint32_t grp_tile_count[6];
    uint32_t tile_first_rec[kMaxSearchTiles];
    uint32_t tile_rows[kMaxSearchTiles];      // valid classes in the tile (the rest is padding)
};
// Matrix-core operands of a tile: A[tile][kb][lane] = eight bf16 values, class row lane % 32, k = 16 kb + 8 (lane / 32) + t.
// k = 0..23: the record's coef; even classes: k = 24 holds -amin2 when kappa = 0, k = 25 holds -amin2 when kappa = 1.
// Scale[tile][metric][lane / 32][r]: the factor (angular metric) or the offset (Euclidean metric) of the class in
// accumulator slot r (row 8 (r / 4) + 4 (lane / 32) + r % 4).  Padding rows repeat the first class of the tile.
constexpr uint32_t kSearchTileABytes = 2 * 64 * 16;
constexpr uint32_t kSearchTileScaleFloats = 2 * 2 * 16;

// nibble slot (0..7) of chunk position 0..5 inside a spread6 entry
static constexpr int kNibbleSlot[6] = {0, 2, 1, 3, 4, 6};

struct Tables {
    TableLayout lay;
    uint64_t shell_off[16];  // index of the first point of shell m (N(m-1)); entries above m_max hold N(m_max)
    std::vector<unsigned char> blob;
    EncLayout enc_lay;
    std::vector<unsigned char> enc_blob;
    SearchLayout search_lay;
    std::vector<SearchRec> search_recs;
    std::vector<uint16_t> search_tile_a;      // n_tiles x 2 x 64 x 8 bf16
    std::vector<float> search_tile_scale;     // n_tiles x kSearchTileScaleFloats
    std::vector<uint32_t> golay_sorted;   // the 4096 words in (weight, message) order
};

// Builds every table for Lambda_24(m_max), 2 <= m_max <= 13.  Returns false on an internal inconsistency.
bool build_tables(int m_max, Tables& out);

}  // namespace llvq
