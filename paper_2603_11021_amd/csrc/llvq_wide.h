// Dequantiser for the larger unions of shells, Lambda_24(m_max) with 14 <= m_max <= 19 (paper Table 1, row m = 19:
// 23,546,209,100,646,960 points, 55-bit indices; App. A steps 1-4).  Up to shell 19 there are 1,457 classes, up to six
// distinct absolute values per class (five up to shell 13), values up to 17 and arrangement ranks of 38 bits, which the
// table-driven decoder of llvq_decode_core.h is not laid out for (three-bit value codes, two symbol planes, class
// tables that fill LDS for 383 classes).  This one follows the same index format step by step with plain 64-bit
// integer arithmetic and loops over the 24 positions: class records and offsets stay in global memory, subsets are
// unranked against a table of binomial coefficients.  It is several times slower than the table-driven decoder and
// is used only by contexts created with m_max > 13.  The same source compiles for the host, where a test harness
// runs it against the tables without a GPU.
#pragma once
#include <cstdint>
#include <vector>

#if defined(__HIPCC__)
#define LLVQ_WHD __host__ __device__ inline
#else
#define LLVQ_WHD inline
#endif

namespace llvq {

constexpr int kWideMaxM = 19;
constexpr int kWideMaxMinor = 5;      // distinct values of the outer domain besides the outside value
constexpr int kWideMaxDirect = 4;     // distinct 2-mod-4 values of a direct F1 word

// flags of WideRec
enum { WF_ODD = 1, WF_F1DIRECT = 2, WF_OUTER_ALL = 4, WF_FEN = 8, WF_KAPPA = 16 };

struct alignas(16) WideRec {
    uint64_t Pin;                 // arrangements of the minority values on their q slots
    uint32_t P1;                  // arrangements of the direct F1 word (1 when there is none)
    uint32_t A;                   // Golay refinements of the class: 1, 759, 2576 or 4096
    float    rnorm;               // 1 / sqrt(16 m)
    uint16_t goff;                // first Golay word of the class in the (weight, message) order
    uint8_t  B, w, m, n, q, flags;
    uint8_t  nm, nd;              // numbers of minority values / of direct F1 values
    uint8_t  mc[kWideMaxMinor];   // multiplicities of the minority values, descending value order
    uint8_t  dc[kWideMaxDirect];  // multiplicities of the direct F1 values, descending value order
    int8_t   outside;             // value on the outer domain's slots outside U (signed for odd classes, see below)
    int8_t   mv[kWideMaxMinor];   // minority values; odd classes: the value taken where the Golay word has a 0
    int8_t   dv[kWideMaxDirect];  // direct F1 values
    uint8_t  pad[13];
};
static_assert(sizeof(WideRec) == 64, "WideRec layout");

struct WideLayout {
    uint32_t ncls;
    uint32_t m_max;
    uint64_t npoints;
};

// device / host views of the tables
struct WidePtrs {
    const WideRec*  recs;      // ncls records
    const uint64_t* cls_off;   // ncls + 1 cumulative class offsets (the last one is N)
    const uint32_t* gs;        // 4096 Golay words ordered by (weight, message)
    const uint32_t* binom;     // 25 x 25 binomial coefficients C(n, k) at [n * 25 + k]
    uint32_t ncls;
    uint64_t npoints;
};

LLVQ_WHD uint32_t wide_popc(uint32_t v) { return (uint32_t)__builtin_popcount(v); }

// the k-subset of {0 .. nbits-1} with colex rank `rank` (numeric order of the masks of popcount k)
LLVQ_WHD uint32_t wide_colex_unrank(const uint32_t* binom, int nbits, int k, uint32_t rank) {
    uint32_t mask = 0;
    for (int pos = nbits - 1; pos >= 0 && k > 0; pos--) {
        const uint32_t c = binom[pos * 25 + k];            // subsets of size k among positions below pos
        if (rank >= c) { mask |= 1u << pos; rank -= c; k--; }
    }
    return mask;
}

// the low bits of src laid onto the set bits of mask, lowest first
LLVQ_WHD uint32_t wide_deposit(uint32_t src, uint32_t mask) {
    uint32_t out = 0;
    while (mask) {
        const uint32_t low = mask & (0u - mask);
        if (src & 1u) out |= low;
        src >>= 1;
        mask ^= low;
    }
    return out;
}

// Lays the values of a word (multiplicities cnt[0..nv-1], descending value order) onto the set bits of `slots`
// according to the mixed-radix rank rho: digit of the largest value least significant, each digit the colex rank of
// the subset that value takes among the slots still free; the last value takes what is left.  occ[i] = positions of value i.
LLVQ_WHD void wide_inner_word(const uint32_t* binom, const uint8_t* cnt, int nv, uint64_t rho, uint32_t slots, uint32_t* occ) {
    uint32_t freemask = slots;
    for (int i = 0; i < nv; i++) {
        const int nfree = (int)wide_popc(freemask);
        if (i + 1 == nv) { occ[i] = freemask; break; }
        const uint32_t radix = binom[nfree * 25 + cnt[i]];
        const uint32_t digit = (uint32_t)(rho % radix);
        rho /= radix;
        occ[i] = wide_deposit(wide_colex_unrank(binom, nfree, cnt[i], digit), freemask);
        freemask &= ~occ[i];
    }
}

// Decodes index I < npoints into 24 int8 coordinates (six dwords, position order); returns the shell.
LLVQ_WHD uint32_t wide_decode(const WidePtrs& T, uint64_t I, uint32_t (&out)[6], float& rnorm) {
    // App. A steps 1-2: the class whose range of indices holds I
    uint32_t lo = 0, hi = T.ncls;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (I >= T.cls_off[mid]) lo = mid; else hi = mid;
    }
    const WideRec R = T.recs[lo];
    // step 3: r = Ic mod A, then B sign bits, then I'' = (d * Pin + rin) * P1 + rho1
    uint64_t t = I - T.cls_off[lo];
    const uint32_t r = (uint32_t)(t % R.A);
    t /= R.A;
    const uint32_t s = (uint32_t)(t & ((1ull << R.B) - 1ull));
    t >>= R.B;
    const uint32_t rho1 = (uint32_t)(t % R.P1);
    t /= R.P1;
    const uint64_t rin = t % R.Pin;
    const uint32_t d = (uint32_t)(t / R.Pin);
    // step 4: Golay word, placement, signs
    const uint32_t c = T.gs[R.goff + r];
    const bool odd = R.flags & WF_ODD, outer_all = R.flags & WF_OUTER_ALL, f1direct = R.flags & WF_F1DIRECT;
    const uint32_t om = outer_all ? 0xFFFFFFu : (~c & 0xFFFFFFu);
    // the q-subset U of the outer domain's n slots: slots 0..11 low, the rest high; ordered by the number j of high
    // slots, then the colex rank of the high part, then that of the low part
    const int n = R.n, q = R.q, nl = n < 12 ? n : 12, nh = n - nl;
    int j = q - nl > 0 ? q - nl : 0;
    const int jmax = q < nh ? q : nh;
    uint32_t base = 0;
    for (; j < jmax; j++) {
        const uint32_t cnt = T.binom[nh * 25 + j] * T.binom[nl * 25 + (q - j)];
        if (d < base + cnt) break;
        base += cnt;
    }
    const uint32_t dl = d - base, div = T.binom[nl * 25 + (q - j)];
    const uint32_t U_rel = wide_colex_unrank(T.binom, nl, q - j, dl % div) | (wide_colex_unrank(T.binom, nh, j, dl / div) << 12);
    const uint32_t U = wide_deposit(U_rel, om);
    uint32_t occ_m[kWideMaxMinor] = {0, 0, 0, 0, 0}, occ_d[kWideMaxDirect] = {0, 0, 0, 0};
    if (R.nm) wide_inner_word(T.binom, R.mc, R.nm, rin, U, occ_m);
    if (f1direct) wide_inner_word(T.binom, R.dc, R.nd, rho1, c, occ_d);
    // signs: even classes take w - 1 free bits on the word's support (the last slot is forced by condition (iii)),
    // then one bit per slot of U; odd classes are negated where the word has a 1
    uint32_t neg;
    if (odd) {
        neg = c;
    } else {
        const uint32_t wm1 = R.w ? R.w - 1u : 0u;
        uint32_t s1 = s & ((1u << wm1) - 1u);
        const uint32_t forced = ((R.flags & WF_FEN) ? 1u : 0u) & (((R.flags & WF_KAPPA) ? 1u : 0u) ^ wide_popc(s1)) & 1u;
        s1 |= forced << wm1;
        neg = wide_deposit(s1, c) | wide_deposit(s >> wm1, U);
    }
    int8_t x[24];
    for (int p = 0; p < 24; p++) {
        const uint32_t bit = 1u << p;
        int v = (om & ~U & bit) ? R.outside : 0;
        for (int i = 0; i < kWideMaxMinor; i++) if (occ_m[i] & bit) v = R.mv[i];
        for (int i = 0; i < kWideMaxDirect; i++) if (occ_d[i] & bit) v = R.dv[i];
        x[p] = (int8_t)((neg & bit) ? -v : v);
    }
    for (int k = 0; k < 6; k++)
        out[k] = (uint32_t)(uint8_t)x[4 * k] | ((uint32_t)(uint8_t)x[4 * k + 1] << 8) | ((uint32_t)(uint8_t)x[4 * k + 2] << 16) |
                 ((uint32_t)(uint8_t)x[4 * k + 3] << 24);
    rnorm = R.rnorm;
    return R.m;
}

// host-side tables of the wide decoder
struct WideTables {
    WideLayout lay;
    uint64_t shell_off[24];            // index of the first point of shell m (N(m-1)); entries above m_max hold N(m_max)
    std::vector<WideRec> recs;
    std::vector<uint64_t> cls_off;     // ncls + 1 entries
    std::vector<uint32_t> gs;          // 4096 Golay words in (weight, message) order
    std::vector<uint32_t> binom;       // 25 x 25
};

// Builds the tables for Lambda_24(m_max), 2 <= m_max <= 19.  Returns false on an internal inconsistency.
bool build_wide_tables(int m_max, WideTables& out);

}  // namespace llvq
