// Host-side builder of the dequantiser's constant tables (see llvq_tables.h for what each holds).
//
// What the tables encode, with the passages that define it:
//   - Golay words: cyclic (23,12) code of generator x^11+x^10+x^6+x^5+x^4+x^2+1 extended by a parity
//     bit at coordinate 23; words ordered by (weight, message)                        [paper Sec. 2.3]
//   - classes of a shell: multisets of 24 absolute values with sum of squares 16 m, all even with
//     #(2 mod 4) a Golay weight (and #(4 mod 8) even when that weight is 0), or all odd [Sec. 2.3-2.5]
//   - class cardinality A * 2^B * (arrangements on F1) * (arrangements on F0)          [Sec. 2.5]
//   - index order: shells by radius, classes contiguous, local digits r, s, I''       [Sec. 3.2, App. A]
// The orders the paper leaves free (class order, word order, sign-bit order, ranking of placements)
// are those of this library's index format; they are restated where each table is built.
#include "llvq_tables.h"
#include "llvq_wide.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <map>

namespace llvq {
namespace {

uint64_t g_binom[25][25];

void init_binom() {
    for (int n = 0; n <= 24; n++)
        for (int k = 0; k <= 24; k++)
            g_binom[n][k] = (k == 0) ? 1 : (n == 0 ? 0 : g_binom[n - 1][k - 1] + g_binom[n - 1][k]);
}

inline int popcnt(uint32_t v) { return __builtin_popcount(v); }

// masks of popcount p below 2^nbits in increasing numeric order (= colex order of the subsets)
std::vector<uint32_t> masks_in_colex_order(int nbits, int p) {
    std::vector<uint32_t> out;
    for (uint32_t m = 0; m < (1u << nbits); m++)
        if (popcnt(m) == p) out.push_back(m);
    return out;
}

// deposit the low bits of `src` into the set bits of `mask`, lowest first
uint32_t deposit(uint32_t src, uint32_t mask) {
    uint32_t out = 0;
    for (int pos = 0, k = 0; pos < 32; pos++)
        if ((mask >> pos) & 1u) { if ((src >> k) & 1u) out |= 1u << pos; k++; }
    return out;
}

struct Leader {
    std::vector<int> val, cnt;   // distinct absolute values descending, multiplicities
    int m = 0;
    bool odd = false;
    int w = 0;
    uint64_t A = 0, size = 0, offset = 0, P1 = 1, P0 = 1;
    int B = 0;
};

uint64_t multinomial(const std::vector<int>& c) {
    int n = 0;
    for (int v : c) n += v;
    uint64_t r = 1;
    for (int v : c) { r *= g_binom[n][v]; n -= v; }
    return r;
}

void enumerate(int m, bool odd, int v, int left, int leftsq, Leader& cur, std::vector<Leader>& out) {
    const int vmin = odd ? 1 : 0;
    if (v == vmin) {
        if (left * v * v != leftsq) return;
        Leader L = cur;
        if (left > 0) { L.val.push_back(v); L.cnt.push_back(left); }
        out.push_back(L);
        return;
    }
    for (int k = std::min(left, leftsq / (v * v)); k >= 0; k--) {
        if (k) { cur.val.push_back(v); cur.cnt.push_back(k); }
        enumerate(m, odd, v - 2, left - k, leftsq - k * v * v, cur, out);
        if (k) { cur.val.pop_back(); cur.cnt.pop_back(); }
    }
}

bool leader_less(const Leader& a, const Leader& b) {
    if (a.odd != b.odd) return !a.odd;
    if (a.w != b.w) return a.w < b.w;
    // descending-ordered leaders compared lexicographically
    std::vector<int> ea, eb;
    for (size_t i = 0; i < a.val.size(); i++) ea.insert(ea.end(), a.cnt[i], a.val[i]);
    for (size_t i = 0; i < b.val.size(); i++) eb.insert(eb.end(), b.cnt[i], b.val[i]);
    return ea < eb;
}

uint8_t fp8_e4m3(int v) {   // small non-negative integers are exact in e4m3 (bias 7)
    if (v == 0) return 0;
    int e = 0;
    while ((v >> (e + 1)) != 0) e++;
    int frac = ((v << 3) >> e) & 7;   // three mantissa bits below the leading one (v <= 15)
    return (uint8_t)(((e + 7) << 3) | frac);
}

template <typename T>
uint32_t append(std::vector<unsigned char>& blob, const std::vector<T>& v) {
    while (blob.size() % 16) blob.push_back(0);
    uint32_t off = (uint32_t)blob.size();
    const unsigned char* p = reinterpret_cast<const unsigned char*>(v.data());
    blob.insert(blob.end(), p, p + v.size() * sizeof(T));
    return off;
}



// The 4096 Golay words in (weight, message) order and every class of shells 2..m_max in index order (paper Sec. 2.3-2.5,
// 3.2): shell_off[m] receives N(m-1) for m <= m_max, `total` N(m_max).
bool enumerate_leaders(int m_max, std::vector<uint32_t>& gs, int (&woff)[25], std::vector<Leader>& cls, uint64_t* shell_off,
                       uint64_t& total) {
    init_binom();
    // ---- Golay words ----------------------------------------------------------------------------
    std::vector<uint32_t> word(4096);
    gs.clear();
    const uint32_t gen = 0xC75;
    for (uint32_t u = 0; u < 4096; u++) {
        uint32_t c = 0;
        for (int k = 0; k < 12; k++) if ((u >> k) & 1u) c ^= gen << k;
        if (popcnt(c) & 1) c |= 1u << 23;
        word[u] = c;
    }
    for (int wt = 0; wt <= 24; wt++) {
        woff[wt] = (int)gs.size();
        for (uint32_t u = 0; u < 4096; u++) if (popcnt(word[u]) == wt) gs.push_back(word[u]);
    }
    if (gs.size() != 4096 || woff[8] != 1 || woff[12] != 760 || woff[16] != 3336 || woff[24] != 4095) return false;

    // ---- classes ----------------------------------------------------------------------------------
    cls.clear();
    uint64_t running = 0;
    for (int m = 2; m <= m_max; m++) {
        shell_off[m] = running;
        std::vector<Leader> shell;
        int vmax = (int)std::floor(std::sqrt(16.0 * m) + 1e-9);
        for (int odd = 0; odd < 2; odd++) {
            Leader cur;
            std::vector<Leader> raw;
            int v0 = (vmax % 2 == odd) ? vmax : vmax - 1;
            enumerate(m, odd != 0, v0, 24, 16 * m, cur, raw);
            for (Leader& L : raw) {
                L.m = m; L.odd = odd != 0;
                if (L.odd) {
                    L.w = 0; L.A = 4096; L.B = 0; L.P1 = multinomial(L.cnt); L.P0 = 1;
                } else {
                    std::vector<int> c1, c0;
                    int w = 0, n4 = 0, nnz0 = 0;
                    for (size_t i = 0; i < L.val.size(); i++) {
                        if (L.val[i] % 4 == 2) { c1.push_back(L.cnt[i]); w += L.cnt[i]; }
                        else { c0.push_back(L.cnt[i]); if (L.val[i]) nnz0 += L.cnt[i]; }
                        if (L.val[i] % 8 == 4) n4 += L.cnt[i];
                    }
                    if (!(w == 0 || w == 8 || w == 12 || w == 16 || w == 24)) continue;
                    if (w == 0 && (n4 & 1)) continue;
                    L.w = w;
                    L.A = (w == 0 || w == 24) ? 1 : (w == 12 ? 2576 : 759);
                    L.B = (w ? w - 1 : 0) + nnz0;
                    L.P1 = multinomial(c1); L.P0 = multinomial(c0);
                }
                L.size = L.A * L.P1 * L.P0 << L.B;
                shell.push_back(L);
            }
        }
        std::sort(shell.begin(), shell.end(), leader_less);
        for (Leader& L : shell) { L.offset = running; running += L.size; cls.push_back(L); }
    }
    total = running;
    return true;
}

// How a class lays its values out (shared by the two decoders' table builders): the values that go through the Golay
// word directly, the outer domain's outside value and minority values, and the parity that condition (iii) forces on
// the number of negative F1 coordinates.
struct ClassShape {
    bool f1direct, outer_all;
    std::vector<int> mv, mc, dv, dc;     // minority values / direct F1 values, descending, with multiplicities
    int outside, n, q, kappa;
};

ClassShape shape_of(const Leader& L) {
    ClassShape S;
    S.f1direct = !L.odd && L.w > 0 && L.w <= 16;
    S.outer_all = L.odd || L.w == 24;
    std::vector<int> ov, oc;
    for (size_t i = 0; i < L.val.size(); i++) {
        bool isF1 = !L.odd && (L.val[i] % 4 == 2);
        if (S.f1direct && isF1) { S.dv.push_back(L.val[i]); S.dc.push_back(L.cnt[i]); }
        else { ov.push_back(L.val[i]); oc.push_back(L.cnt[i]); }
    }
    S.n = 0;
    for (int c : oc) S.n += c;
    // outside value: 0 for the F0 domain of even classes (whether present or not), otherwise the most
    // frequent value, ties towards the smaller value
    S.outside = 0;
    if (S.outer_all) {
        size_t best = 0;
        for (size_t i = 0; i < ov.size(); i++)
            if (oc[i] > oc[best] || (oc[i] == oc[best] && ov[i] < ov[best])) best = i;
        S.outside = ov[best];
    }
    for (size_t i = 0; i < ov.size(); i++) if (ov[i] != S.outside) { S.mv.push_back(ov[i]); S.mc.push_back(oc[i]); }
    S.q = 0;
    for (int c : S.mc) S.q += c;
    // parity of the number of negative signs on F1 (condition (iii) of L_even): with a = 4y on F0 and
    // a = 2 + 4u on F1, sum x = 4 (sum y + sum u + #negative F1) (mod 8) because 2w = 0 (mod 8).
    S.kappa = 0;
    if (!L.odd) for (size_t i = 0; i < L.val.size(); i++) {
        int t = (L.val[i] % 4 == 2) ? (L.val[i] - 2) / 4 : L.val[i] / 4;
        S.kappa ^= (t * L.cnt[i]) & 1;
    }
    return S;
}

}  // namespace

bool build_wide_tables(int m_max, WideTables& out) {
    if (m_max < 2 || m_max > kWideMaxM) return false;
    std::vector<Leader> cls;
    int woff[25];
    uint64_t total = 0;
    for (int m = 0; m < 24; m++) out.shell_off[m] = 0;
    if (!enumerate_leaders(m_max, out.gs, woff, cls, out.shell_off, total)) return false;
    for (int m = m_max + 1; m < 24; m++) out.shell_off[m] = total;
    if (total >= (1ull << 56)) return false;
    out.lay.ncls = (uint32_t)cls.size();
    out.lay.m_max = (uint32_t)m_max;
    out.lay.npoints = total;
    out.binom.assign(25 * 25, 0);
    for (int n = 0; n <= 24; n++)
        for (int k = 0; k <= 24; k++) {
            if (g_binom[n][k] > 0xFFFFFFFFull) return false;
            out.binom[n * 25 + k] = (uint32_t)g_binom[n][k];
        }
    out.recs.assign(cls.size(), WideRec{});
    out.cls_off.assign(cls.size() + 1, total);
    for (size_t ci = 0; ci < cls.size(); ci++) {
        const Leader& L = cls[ci];
        const ClassShape S = shape_of(L);
        WideRec R{};
        out.cls_off[ci] = L.offset;
        if (S.mv.size() > (size_t)kWideMaxMinor || S.dv.size() > (size_t)kWideMaxDirect) return false;
        const uint64_t Pin = multinomial(S.mc), P1 = S.f1direct ? multinomial(S.dc) : 1;
        if (g_binom[S.n][S.q] * Pin * P1 != L.P1 * L.P0 || P1 > 0xFFFFFFFFull) return false;     // consistency with the class cardinality
        R.Pin = Pin; R.P1 = (uint32_t)P1; R.A = (uint32_t)L.A;
        R.rnorm = (float)(1.0 / std::sqrt(16.0 * L.m));
        R.goff = (uint16_t)(L.odd ? 0 : woff[L.w]);
        R.B = (uint8_t)L.B; R.w = (uint8_t)L.w; R.m = (uint8_t)L.m; R.n = (uint8_t)S.n; R.q = (uint8_t)S.q;
        R.flags = (uint8_t)((L.odd ? WF_ODD : 0) | (S.f1direct ? WF_F1DIRECT : 0) | (S.outer_all ? WF_OUTER_ALL : 0) |
                            ((!L.odd && L.w > 0) ? WF_FEN : 0) | (S.kappa ? WF_KAPPA : 0));
        R.nm = (uint8_t)S.mv.size(); R.nd = (uint8_t)S.dv.size();
        // odd classes: the sign a coordinate takes where the Golay word has a 0 (+a for a = 1 mod 4, -a for a = 3 mod 4)
        auto signed_value = [&](int a) { return (int8_t)((L.odd && a % 4 == 3) ? -a : a); };
        R.outside = signed_value(S.outside);
        for (size_t i = 0; i < S.mv.size(); i++) { R.mv[i] = signed_value(S.mv[i]); R.mc[i] = (uint8_t)S.mc[i]; }
        for (size_t i = 0; i < S.dv.size(); i++) { R.dv[i] = (int8_t)S.dv[i]; R.dc[i] = (uint8_t)S.dc[i]; }
        out.recs[ci] = R;
    }
    return true;
}

bool build_tables(int m_max, Tables& out) {
    if (m_max < 2 || m_max > 13) return false;
    std::vector<uint32_t> gs;
    int woff[25];
    std::vector<Leader> cls;
    uint64_t running = 0, shell_off[24] = {};
    if (!enumerate_leaders(m_max, gs, woff, cls, shell_off, running)) return false;
    for (int m = 0; m < 16; m++) out.shell_off[m] = m <= m_max ? shell_off[m] : running;
    const uint32_t ncls = (uint32_t)cls.size();
    if (running >= (1ull << 48)) return false;

    // ---- lut12: colex rank -> mask, grouped by popcount ---------------------------------------------
    std::vector<uint16_t> lut12;
    int b12[14];
    for (int p = 0; p <= 12; p++) {
        b12[p] = (int)lut12.size();
        for (uint32_t mk : masks_in_colex_order(12, p)) lut12.push_back((uint16_t)mk);
    }
    b12[13] = (int)lut12.size();

    // ---- inner-word tables ------------------------------------------------------------------------
    // Pattern = multiplicities of the values of the word in descending value order, over q slots.
    // Entry rho: mixed radix, digit of the largest value least significant, each digit the colex rank of
    // the subset that value occupies among the slots still free; the smallest value takes the rest.
    // Planes: bit k of plane a/b = bit 0/1 of (symbol index + sym_base) of the value on slot k.
    std::vector<uint32_t> inner;
    std::map<std::pair<std::vector<int>, int>, uint32_t> inner_base;
    auto inner_table = [&](const std::vector<int>& cnt, int sym_base) -> int64_t {
        auto key = std::make_pair(cnt, sym_base);
        auto it = inner_base.find(key);
        if (it != inner_base.end()) return it->second;
        int q = 0;
        for (int c : cnt) q += c;
        if (q > 16 || (int)cnt.size() + sym_base > 4) return -1;
        uint64_t P = multinomial(cnt);
        uint32_t base = (uint32_t)inner.size();
        std::vector<std::vector<uint32_t>> cm(cnt.size());
        for (size_t i = 0; i < cnt.size(); i++) cm[i] = masks_in_colex_order(q, cnt[i]);   // over-long lists are harmless
        for (uint64_t rho = 0; rho < P; rho++) {
            uint64_t r = rho;
            uint32_t freemask = (q == 32) ? 0xFFFFFFFFu : ((1u << q) - 1u), pa = 0, pb = 0;
            for (size_t i = 0; i < cnt.size(); i++) {
                uint32_t occ;
                int nfree = popcnt(freemask);
                if (i + 1 == cnt.size()) occ = freemask;
                else {
                    uint64_t radix = g_binom[nfree][cnt[i]];
                    occ = deposit(cm[i][r % radix], freemask);
                    r /= radix;
                }
                int sym = (int)i + sym_base;
                if (sym & 1) pa |= occ;
                if (sym & 2) pb |= occ;
                freemask &= ~occ;
            }
            inner.push_back(pa | (pb << 16));
        }
        inner_base[key] = base;
        return base;
    };
    const int64_t dummy_tb = inner_table(std::vector<int>{}, 0);   // one all-zero entry
    if (dummy_tb != 0) return false;

    // ---- subset ranking tables ---------------------------------------------------------------------
    // q-subsets of n slots, slots 0..11 low, 12..n-1 high; order: number j of high slots, then colex rank
    // of the high part, then colex rank of the low part.
    std::vector<SplitEnt> split;
    std::vector<uint8_t> guess;
    struct SplitInfo { uint16_t sp; int shift, jmax, row; };
    std::map<std::pair<int, int>, SplitInfo> split_of;
    auto split_table = [&](int n, int q) -> SplitInfo {
        auto key = std::make_pair(n, q);
        auto it = split_of.find(key);
        if (it != split_of.end()) return it->second;
        int nl = std::min(n, 12), nh = n - nl;
        int jmin = std::max(0, q - nl), jmax = std::min(q, nh);
        SplitInfo si;
        si.sp = (uint16_t)((int)split.size() - jmin);      // entry of j is split[sp + j]
        si.jmax = jmax;
        si.row = (int)(guess.size() / kGuessBuckets);
        std::vector<uint64_t> bases;
        uint64_t base = 0;
        for (int j = jmin; j <= jmax; j++) {
            SplitEnt e{};
            uint64_t div = g_binom[nl][q - j];
            e.base = (uint32_t)base;
            e.div = (uint16_t)div;
            float inv = 1.0f / (float)div;
            while ((double)inv * (double)div < 1.0) inv = std::nextafterf(inv, 2.0f);
            e.inv = inv;
            e.b12lo = (uint16_t)b12[q - j];
            e.b12hi = (uint16_t)b12[j];
            split.push_back(e);
            bases.push_back(base);
            base += g_binom[nh][j] * div;
        }
        uint64_t total = base;                              // C(n, q)
        int shift = 0;
        while (((total - 1) >> shift) >= kGuessBuckets) shift++;
        si.shift = shift;
        for (uint32_t b = 0; b < kGuessBuckets; b++) {
            uint64_t d0 = (uint64_t)b << shift;
            int j = jmin;
            while (j < jmax && bases[j + 1 - jmin] <= d0) j++;
            guess.push_back((uint8_t)j);
        }
        split_of[key] = si;
        return si;
    };

    // ---- class records ---------------------------------------------------------------------------
    std::vector<ClassRec> recs(ncls);
    std::vector<EncRec> encs(ncls);
    std::vector<uint64_t> cls_off(ncls + 4, ~0ull);      // the search reads up to three entries past offset[ncls] = N
    for (uint32_t ci = 0; ci < ncls; ci++) {
        const Leader& L = cls[ci];
        ClassRec R{};
        cls_off[ci] = L.offset;
        const ClassShape S = shape_of(L);
        const bool f1direct = S.f1direct, outer_all = S.outer_all;
        const std::vector<int>&mv = S.mv, &mc = S.mc, &dv = S.dv, &dc = S.dc;
        const int n = S.n, q = S.q, outside = S.outside;
        uint64_t Pin = multinomial(mc);
        uint64_t P1 = f1direct ? multinomial(dc) : 1;
        // consistency with the class cardinality
        uint64_t arr = g_binom[n][q] * Pin * P1;
        if (arr != L.P1 * L.P0) return false;
        int sym_base0 = outer_all ? 0 : 1;
        int64_t tb0 = mc.empty() ? dummy_tb : inner_table(mc, sym_base0);
        int64_t tb1 = f1direct ? inner_table(dc, 0) : dummy_tb;
        if (tb0 < 0 || tb1 < 0 || tb0 > 0xFFFF || tb1 > 0xFFFF) return false;
        SplitInfo si = split_table(n, q);
        uint64_t PP = P1 * Pin;
        if (PP >= (1u << 22) || P1 > 0xFFFF) return false;
        R.PP = (uint32_t)PP;
        R.invPP = (1.0 / (double)PP) * (1.0 + std::ldexp(1.0, -50));
        float i1 = 1.0f / (float)P1;
        while ((double)i1 * (double)P1 < 1.0) i1 = std::nextafterf(i1, 2.0f);
        R.invP1 = i1;
        R.P1 = (uint16_t)P1; R.tb0 = (uint16_t)tb0; R.tb1 = (uint16_t)tb1; R.sp = si.sp;
        const int kappa = S.kappa;
        int acode = L.A == 1 ? 0 : (L.A == 759 ? 1 : (L.A == 2576 ? 2 : 3));
        int wm1 = (!L.odd && L.w > 0) ? L.w - 1 : 0;
        R.f0 = (uint32_t)(L.odd ? 1 : 0) << F0_ODD | (uint32_t)(f1direct ? 1 : 0) << F0_F1DIRECT |
               (uint32_t)(outer_all ? 1 : 0) << F0_OUTER_ALL | (uint32_t)wm1 << F0_WM1 |
               (uint32_t)((!L.odd && L.w > 0) ? 1 : 0) << F0_FEN | (uint32_t)kappa << F0_KAPPA |
               (uint32_t)L.B << F0_B | (uint32_t)L.m << F0_M | (uint32_t)n << F0_N | (uint32_t)q << F0_Q;
        int goff = L.odd ? 0 : woff[L.w];
        R.f1 = (uint32_t)goff << F1_GOFF | (uint32_t)acode << F1_ACODE | (uint32_t)si.shift << F1_GSHIFT |
               (uint32_t)si.jmax << F1_JMAX | (uint32_t)si.row << F1_GROW;
        // value of each nibble code.  Outer domain = all positions (odd, w = 24): code 0 = outside value,
        // 4 + i = i-th minority value.  Otherwise: 0 = zero, 1 + i = i-th nonzero F0 value, 4 + i = i-th F1 value.
        int code_val[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        if (outer_all) {
            code_val[0] = outside;
            for (size_t i = 0; i < mv.size(); i++) code_val[4 + i] = mv[i];
        } else {
            for (size_t i = 0; i < mv.size(); i++) code_val[1 + i] = mv[i];
            for (size_t i = 0; i < dv.size(); i++) code_val[4 + i] = dv[i];
        }
        uint64_t v8 = 0, vi = 0;
        for (int k = 0; k < 8; k++) {
            int v = code_val[k];
            bool neg = L.odd && (v % 4 == 3);      // odd classes: x_i = 1 + 2 c_i (mod 4); the word bit flips it again
            v8 |= (uint64_t)(fp8_e4m3(v) | (neg ? 0x80 : 0)) << (8 * k);
            vi |= (uint64_t)(uint8_t)(int8_t)(neg ? -v : v) << (8 * k);
        }
        R.vt8_lo = (uint32_t)v8; R.vt8_hi = (uint32_t)(v8 >> 32);
        R.vti_lo = (uint32_t)vi; R.vti_hi = (uint32_t)(vi >> 32);
        recs[ci] = R;

        // the same class seen from the encoder: key of the leader, code of each absolute value, ranking radices
        EncRec E{};
        E.offset = L.offset;
        uint64_t p1 = 0, p4 = 0;
        for (size_t i = 0; i < L.val.size(); i++) {
            uint64_t v = (uint64_t)L.val[i];
            p1 += v * L.cnt[i];
            p4 += v * v * v * v * L.cnt[i];
        }
        if (p4 >= (1u << 20) || p1 >= (1u << 9)) return false;
        E.key = (uint32_t)p4 | (uint32_t)p1 << 20 | (uint32_t)(L.odd ? 1 : 0) << 29;
        E.f0 = R.f0;
        uint8_t ctab[8];
        for (int k = 0; k < 8; k++) ctab[k] = 0xFF;
        auto set_code = [&](int value, int code) { ctab[value >> 1] = (uint8_t)code; };
        if (outer_all) {
            set_code(outside, 0);
            for (size_t i = 0; i < mv.size(); i++) set_code(mv[i], 4 + (int)i);
        } else {
            set_code(0, 0);
            for (size_t i = 0; i < mv.size(); i++) set_code(mv[i], 1 + (int)i);
            for (size_t i = 0; i < dv.size(); i++) set_code(dv[i], 4 + (int)i);
        }
        std::memcpy(&E.ctab_lo, ctab, 4);
        std::memcpy(&E.ctab_hi, ctab + 4, 4);
        E.Pin = (uint32_t)Pin;
        E.P1 = (uint16_t)P1;
        E.sp = si.sp;
        auto radices = [&](const std::vector<int>& cnt, uint16_t rad[2]) -> int {
            int slots = 0;
            for (int c : cnt) slots += c;
            rad[0] = rad[1] = 1;
            for (size_t i = 0; i + 1 < cnt.size(); i++) {
                if (i < 2) rad[i] = (uint16_t)g_binom[slots][cnt[i]];
                slots -= cnt[i];
            }
            return cnt.empty() ? 0 : (int)cnt.size() - 1;
        };
        const int dig0 = radices(mc, E.rad0);
        int dig1 = 0;
        E.rad1[0] = E.rad1[1] = 1;
        if (f1direct) dig1 = radices(dc, E.rad1);
        if (dig0 > 3 || dig1 > 3) return false;
        E.e1 = (uint32_t)goff << E1_GOFF | (uint32_t)acode << E1_ACODE | (uint32_t)dig0 << E1_DIG0 |
               (uint32_t)dig1 << E1_DIG1 | (uint32_t)sym_base0 << E1_SYM0;
        encs[ci] = E;
    }
    cls_off[ncls] = running;

    // ---- bucket table: index >> shift -> class holding the first index of the bucket --------------------
    const uint32_t bucket_shift = kBucketShift, nbuckets = 1u << (48 - kBucketShift);
    std::vector<uint16_t> bucket(nbuckets);
    for (uint32_t b = 0; b < nbuckets; b++) {
        uint64_t first = (uint64_t)b << bucket_shift;
        uint32_t ci = (uint32_t)(std::upper_bound(cls_off.begin(), cls_off.begin() + ncls, first) - cls_off.begin());
        bucket[b] = (uint16_t)(8u * (ci == 0 ? 0 : ci - 1));
    }

    // ---- 6-bit deposit tables ---------------------------------------------------------------------
    std::vector<uint8_t> pdep6(64 * kPdepPitch, 0);
    std::vector<uint32_t> spread6(64 * kSpreadPitch, 0);
    for (uint32_t F = 0; F < 64; F++)
        for (uint32_t mbits = 0; mbits < 64; mbits++) {
            uint32_t dep = deposit(mbits, F);
            pdep6[F * kPdepPitch + mbits] = (uint8_t)dep;
            uint32_t sp = 0;
            for (int p = 0; p < 6; p++) {
                if ((dep >> p) & 1u) sp |= 1u << (4 * kNibbleSlot[p]);
                if ((F >> p) & 1u) sp |= 4u << (4 * kNibbleSlot[p]);
            }
            spread6[F * kSpreadPitch + mbits] = sp;
        }

    // ---- blob ------------------------------------------------------------------------------------
    std::vector<double> atab = {1.0, 1.0, 759.0, (1.0 / 759.0) * (1.0 + std::ldexp(1.0, -50)),
                                2576.0, (1.0 / 2576.0) * (1.0 + std::ldexp(1.0, -50)), 4096.0, 1.0 / 4096.0};
    TableLayout lay{};
    const uint32_t inner_end = kOffInner + (uint32_t)(inner.size() * sizeof(uint32_t));
    if (guess.size() > kOffAtab - kOffGuess || cls_off.size() * 8 > kOffRnorm - kOffClsOff ||
        (split.size() + 1) * sizeof(SplitEnt) > kOffCls - kOffSplit || recs.size() * sizeof(ClassRec) > kLdsBytes - kOffCls ||
        inner_end > kMaxBlob)
        return false;
    std::vector<unsigned char> blob((inner_end + 15u) & ~15u, 0);
    auto put = [&](uint32_t off, const void* src, size_t bytes) { std::memcpy(blob.data() + off, src, bytes); };
    put(kOffGs, gs.data(), gs.size() * 4);
    put(kOffSpread6, spread6.data(), spread6.size() * 4);
    put(kOffPdep6, pdep6.data(), pdep6.size());
    put(kOffLut12, lut12.data(), lut12.size() * 2);
    put(kOffBucket, bucket.data(), bucket.size() * 2);
    put(kOffGuess, guess.data(), guess.size());
    put(kOffAtab, atab.data(), atab.size() * 8);
    put(kOffClsOff, cls_off.data(), cls_off.size() * 8);
    float rnorm[16];
    for (int m = 0; m < 16; m++) rnorm[m] = m >= 1 ? (float)(1.0 / std::sqrt(16.0 * m)) : 0.0f;
    put(kOffRnorm, rnorm, sizeof rnorm);
    put(kOffSplit, split.data(), split.size() * sizeof(SplitEnt));
    put(kOffCls, recs.data(), recs.size() * sizeof(ClassRec));
    put(kOffInner, inner.data(), inner.size() * 4);
    lay.lds_bytes = kLdsBytes;
    lay.blob_bytes = (uint32_t)blob.size();
    lay.ncls = ncls;
    lay.inner_entries = (uint32_t)inner.size();
    lay.npoints = running;
    out.lay = lay;
    out.blob.swap(blob);

    // ---- encoder blob ------------------------------------------------------------------------------
    // ginv: any 12 cyclically consecutive coordinates of a cyclic code are an information set, so the low 12
    // bits of a word identify it
    std::vector<uint16_t> ginv(4096, 0xFFFF);
    for (uint32_t k = 0; k < 4096; k++) {
        if (ginv[gs[k] & 0xFFFu] != 0xFFFF) return false;
        ginv[gs[k] & 0xFFFu] = (uint16_t)k;
    }
    std::vector<uint16_t> rank12(4096);
    for (int pc = 0; pc <= 12; pc++) {
        uint16_t rk = 0;
        for (uint32_t mk : masks_in_colex_order(12, pc)) rank12[mk] = rk++;
    }
    std::vector<uint8_t> pext6(4096);
    for (uint32_t F = 0; F < 64; F++)
        for (uint32_t src = 0; src < 64; src++) {
            uint32_t o = 0;
            for (int pos = 0, k = 0; pos < 6; pos++)
                if ((F >> pos) & 1u) { if ((src >> pos) & 1u) o |= 1u << k; k++; }
            pext6[F << 6 | (src ^ F)] = (uint8_t)o;            // XOR with the mask: equal sources of different masks in different LDS banks
        }
    // g16[H][p]: number of 16-bit masks of popcount p whose bits 12..15, read as a number, are below H
    std::vector<uint16_t> g16(16 * 17, 0);
    for (uint32_t H = 0; H < 16; H++)
        for (int pc = 0; pc <= 16; pc++) {
            uint64_t c = 0;
            for (uint32_t h = 0; h < H; h++) {
                int rest = pc - popcnt(h);
                if (rest >= 0 && rest <= 12) c += g_binom[12][rest];
            }
            if (c > 0xFFFF) return false;
            g16[H * 17 + pc] = (uint16_t)c;
        }
    // cuckoo hash of the class keys: every key sits in one of its two candidate slots
    const uint32_t hslots = 1u << kEncHashBits;
    std::vector<HashEnt> htab;
    uint32_t mult[2] = {0, 0};
    for (uint32_t attempt = 0; attempt < 64 && !mult[0]; attempt++) {
        const uint32_t m0 = 0x9E3779B1u + 2u * attempt * 0x632BE5ABu, m1 = 0x85EBCA77u + 2u * attempt * 0xC2B2AE3Du;
        htab.assign(2 * hslots, HashEnt{0xFFFFFFFFu, 0});
        bool ok = true;
        for (uint32_t ci = 0; ci < ncls && ok; ci++) {
            HashEnt cur{encs[ci].key, ci};
            int half = 0;
            ok = false;
            for (int kick = 0; kick < 200; kick++) {
                const uint32_t slot = half * hslots + ((cur.key * (half ? m1 : m0)) >> (32 - kEncHashBits));
                std::swap(cur, htab[slot]);
                if (cur.key == 0xFFFFFFFFu) { ok = true; break; }
                half ^= 1;
            }
        }
        if (ok) { mult[0] = m0; mult[1] = m1; }
    }
    if (!mult[0]) return false;
    if (split.size() * sizeof(SplitEnt) > kEncCls - kEncSplit || encs.size() * sizeof(EncRec) > kEncBlob - kEncCls) return false;
    std::vector<unsigned char> eb(kEncBlob, 0);
    auto eput = [&](uint32_t off, const void* src, size_t bytes) { std::memcpy(eb.data() + off, src, bytes); };
    eput(kEncGs, gs.data(), gs.size() * 4);
    eput(kEncGinv, ginv.data(), ginv.size() * 2);
    eput(kEncRank12, rank12.data(), rank12.size() * 2);
    eput(kEncPext6, pext6.data(), pext6.size());
    eput(kEncHash, htab.data(), htab.size() * sizeof(HashEnt));
    eput(kEncG16, g16.data(), g16.size() * 2);
    eput(kEncSplit, split.data(), split.size() * sizeof(SplitEnt));
    eput(kEncCls, encs.data(), encs.size() * sizeof(EncRec));
    out.enc_lay.bytes = kEncBlob;
    out.enc_lay.ncls = ncls;
    out.enc_lay.hash_mult[0] = mult[0];
    out.enc_lay.hash_mult[1] = mult[1];
    out.enc_lay.m_max = (uint32_t)m_max;
    out.enc_blob.swap(eb);

    // ---- nearest-point search records ------------------------------------------------------------------
    out.search_recs.clear();
    SearchLayout sl{};
    auto make_rec = [&](uint32_t ci) {
        const Leader& L = cls[ci];
        SearchRec S{};
        std::vector<float> co;
        if (L.odd) {
            for (size_t i = 0; i < L.val.size(); i++)
                for (int k = 0; k < L.cnt[i]; k++) co.push_back(L.val[i] % 4 == 1 ? (float)L.val[i] : -(float)L.val[i]);
            std::sort(co.begin(), co.end(), [](float a, float b) { return a > b; });
        } else {
            for (int pass = 0; pass < 2; pass++)
                for (size_t i = 0; i < L.val.size(); i++)
                    if ((L.val[i] % 4 == 2) == (pass == 0))
                        for (int k = 0; k < L.cnt[i]; k++) co.push_back((float)L.val[i]);
            if (L.w > 0) S.amin2 = 2.0f * co[L.w - 1];
        }
        for (int k = 0; k < 24; k++) S.coef[k] = co[k];
        S.mul[0] = (float)(1.0 / std::sqrt(16.0 * L.m));
        S.mul[1] = 1.0f;
        S.bias[0] = 0.0f;
        S.bias[1] = -8.0f * (float)L.m;
        S.kappa = (encs[ci].f0 >> F0_KAPPA) & 1u;
        S.cid = ci;
        S.w = L.odd ? 0u : (uint32_t)L.w;
        out.search_recs.push_back(S);
    };
    for (uint32_t ci = 0; ci < ncls; ci++) if (cls[ci].odd) make_rec(ci);
    sl.n_odd = (uint32_t)out.search_recs.size();
    const int weights[5] = {0, 8, 12, 16, 24};
    for (int g = 0; g < 5; g++) {
        sl.even_first[g] = (uint32_t)out.search_recs.size();
        for (uint32_t ci = 0; ci < ncls; ci++) if (!cls[ci].odd && cls[ci].w == weights[g]) make_rec(ci);
        sl.even_count[g] = (uint32_t)out.search_recs.size() - sl.even_first[g];
    }
    sl.total = (uint32_t)out.search_recs.size();
    if (sl.total != ncls) return false;
    // tiles of 32 classes, never across a group
    sl.n_tiles = 0;
    for (int g = 0; g < 6; g++) {
        const uint32_t first = g == 0 ? 0 : sl.even_first[g - 1], count = g == 0 ? sl.n_odd : sl.even_count[g - 1];
        sl.grp_tile_first[g] = sl.n_tiles;
        sl.grp_tile_count[g] = (count + 31) / 32;
        for (uint32_t t = 0; t < sl.grp_tile_count[g]; t++) {
            if (sl.n_tiles >= (uint32_t)kMaxSearchTiles) return false;
            sl.tile_first_rec[sl.n_tiles] = first + 32 * t;
            sl.tile_rows[sl.n_tiles] = std::min<uint32_t>(32, count - 32 * t);
            sl.n_tiles++;
        }
    }
    auto bf16_of = [](float v) -> uint16_t {          // exact for the small integers stored here
        uint32_t u;
        std::memcpy(&u, &v, 4);
        return (uint16_t)(u >> 16);
    };
    out.search_tile_a.assign((size_t)sl.n_tiles * 2 * 64 * 8, 0);
    out.search_tile_scale.assign((size_t)sl.n_tiles * kSearchTileScaleFloats, 0.0f);
    for (uint32_t tl = 0; tl < sl.n_tiles; tl++) {
        for (uint32_t row = 0; row < 32; row++) {
            // padding rows repeat the first class of the tile: they can tie with it but never win alone
            const SearchRec* S = &out.search_recs[sl.tile_first_rec[tl] + (row < sl.tile_rows[tl] ? row : 0)];
            float kvec[32];
            for (int k = 0; k < 32; k++) kvec[k] = 0.0f;
            {
                for (int k = 0; k < 24; k++) kvec[k] = S->coef[k];
                kvec[S->kappa ? 25 : 24] = -S->amin2;
                for (int k = 0; k < 32; k++) {
                    float back;
                    uint32_t u = (uint32_t)bf16_of(kvec[k]) << 16;
                    std::memcpy(&back, &u, 4);
                    if (back != kvec[k]) return false;
                }
            }
            for (int kb = 0; kb < 2; kb++)
                for (int h = 0; h < 2; h++)
                    for (int t = 0; t < 8; t++)
                        out.search_tile_a[(((size_t)tl * 2 + kb) * 64 + (32 * h + row)) * 8 + t] = bf16_of(kvec[16 * kb + 8 * h + t]);
            // accumulator slot of this row: row = 8 (r / 4) + 4 h + r % 4
            const uint32_t h = (row >> 2) & 1u, r = 4 * (row >> 3) + (row & 3u);
            float* sc = &out.search_tile_scale[(size_t)tl * kSearchTileScaleFloats];
            sc[0 * 32 + h * 16 + r] = S->mul[0];       // angular: score = <w, x> * mul
            sc[1 * 32 + h * 16 + r] = S->bias[1];      // Euclidean: score = <w, x> + bias
        }
    }
    out.search_lay = sl;
    out.golay_sorted = gs;
    return true;
}

}  // namespace llvq
