// Point -> index: the encoder side of the index map (paper Sec. 3.2), the inverse of llvq_decode_core.h.
// Written so that the same source compiles for the host, where a test harness runs it without a GPU.
//
// One call takes the 24 int8 coordinates of a vector (six dwords, position order) and returns its index in
// Lambda_24(m_max), or kInvalidIndex when the vector is not a point of the ball cut.  Membership is decided by
// the definition (paper Sec. 2.3, conditions (i)-(iii)) plus the norm; the index is then assembled as
//     I = offset(class) + ((I'' << B) + s) * A + r            [paper Sec. 3.2, App. A step 3 read backwards]
// with r the position of the Golay word among the words the class uses, s the free sign bits and I'' the rank
// of the arrangement, all in the orders of this library's index format.
#pragma once
#include <cstdint>

#include "llvq_decode_core.h"

namespace llvq {

constexpr uint64_t kInvalidIndex = ~0ull;

struct EncPtrs {
    TabBase base;               // the encoder blob in LDS (address 0 on the device, see TabBase)
    uint32_t hash_mult[2];
    uint32_t m_max;
};

LLVQ_HD EncPtrs make_enc_ptrs(TabBase base, const EncLayout& L) {
    EncPtrs T;
    T.base = base;
    T.hash_mult[0] = L.hash_mult[0];
    T.hash_mult[1] = L.hash_mult[1];
    T.m_max = L.m_max;
    return T;
}

template <typename V, uint32_t OFF>
LLVQ_HD V enc_at(const EncPtrs& T, uint32_t byte_off) {
    return tab_load<V>(T.base + OFF + byte_off);
}

// v holds one bit per byte (bit 0 of each byte): the four bits, byte 0 lowest
LLVQ_HD uint32_t gather4(uint32_t v) { return (v * 0x01020408u) >> 24; }

// sum of the four bytes of v, as unsigned numbers, plus acc
LLVQ_HD uint32_t sum_u8(uint32_t v, uint32_t acc) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_sad_u8(v, 0u, acc);
#else
    return acc + (v & 0xFFu) + ((v >> 8) & 0xFFu) + ((v >> 16) & 0xFFu) + (v >> 24);
#endif
}

// sum of the products of corresponding unsigned bytes of a and b, plus acc
LLVQ_HD uint32_t dot_u8(uint32_t a, uint32_t b, uint32_t acc) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_udot4(a, b, acc, false);
#else
    for (int k = 0; k < 4; k++) acc += ((a >> (8 * k)) & 0xFFu) * ((b >> (8 * k)) & 0xFFu);
    return acc;
#endif
}

// the bits of src under the set bits of mask, packed towards bit 0 (both below 2^24)
template <int CHUNKS>
LLVQ_HD uint32_t pext6n(const EncPtrs& T, uint32_t src, uint32_t mask) {
    uint32_t out = 0, off = 0;
#pragma unroll
    for (int k = 0; k < CHUNKS; k++) {
        const uint32_t mk = bfe6(mask, 6 * k);
        const uint32_t v = enc_at<uint8_t, kEncPext6>(T, (mk << 6) | (bfe6(src, 6 * k) ^ mk));
        out |= v << off;
        off += popc32(mk);
    }
    return out;
}

// colex rank of a mask below 2^16 among the masks of its popcount (= its rank in numeric order)
LLVQ_HD uint32_t colex_rank16(const EncPtrs& T, uint32_t mask) {
    const uint32_t H = (mask >> 12) & 15u, p = popc32(mask & 0xFFFFu);
    return (uint32_t)enc_at<uint16_t, kEncG16>(T, (H * 17u + p) * 2u) + (uint32_t)enc_at<uint16_t, kEncRank12>(T, (mask & 0xFFFu) * 2u);
}

// Rank of an inner word: symbols sym0, sym0+1, ... (two-bit codes in the planes a, b over q <= 16 slots), the
// digit of the first symbol least significant, each digit the colex rank of the slots of that symbol among the
// slots not taken by earlier symbols; the last symbol takes the rest and has no digit.
LLVQ_HD uint32_t inner_word_rank(const EncPtrs& T, uint32_t a, uint32_t b, uint32_t q, uint32_t ndig, uint32_t sym0,
                                 uint32_t rad0, uint32_t rad1) {
    const uint32_t qmask = (1u << q) - 1u;
    uint32_t rank = 0, free_slots = qmask, scale = 1;
    // every step is guarded wave-wide: most classes have one digit or none
    for (uint32_t i = 0; i < 3; i++) {
        if (!wave_any(i < ndig)) break;
        const uint32_t s = sym0 + i;
        const uint32_t occ = ((s & 1u) ? a : ~a) & ((s & 2u) ? b : ~b) & qmask;
        const uint32_t packed = i == 0 ? occ : pext6n<3>(T, occ, free_slots);
        const uint32_t digit = colex_rank16(T, packed);
        if (i < ndig) rank += digit * scale;
        scale *= i == 0 ? rad0 : rad1;
        free_slots &= ~occ;
    }
    return rank;
}

// x[0..5]: the 24 coordinates as int8, four per dword, position order
LLVQ_HD uint64_t encode_block(const EncPtrs& T, const uint32_t (&x)[6]) {
    // absolute values, sign mask, the bit (x - parity)/2 mod 2 of every coordinate, parity check
    uint32_t a[6], neg = 0, cw = 0, par_or = 0, par_and = 0xFFFFFFFFu, big = 0;
#pragma unroll
    for (int k = 0; k < 6; k++) {
        const uint32_t sg = (x[k] >> 7) & 0x01010101u;
        a[k] = (x[k] ^ (sg * 0xFFu)) + sg;                      // per byte (v ^ 0xFF) + 1 = -v, no carry leaves a byte
        neg |= gather4(sg) << (4 * k);
        cw |= gather4((x[k] >> 1) & 0x01010101u) << (4 * k);
        par_or |= x[k];
        par_and &= x[k];
        big |= a[k];
    }
    const uint32_t odd = x[0] & 1u;
    bool ok = ((odd ? par_and : ~par_or) & 0x01010101u) == 0x01010101u;         // condition (i): one parity
    ok = ok && (big & 0xF0F0F0F0u) == 0;                                         // |x| <= 15: fits the tables below
    // sums: sum |x|, sum x, sum x^2, sum x^4; squares of 2k (+1) from an eight-entry byte table
    const uint32_t sq_lo = odd ? 0x31190901u : 0x24100400u, sq_hi = odd ? 0xE1A97951u : 0xC4906440u;
    uint32_t p1 = 0, p2 = 0, p4 = 0, sumx = 0, sel[6];
#pragma unroll
    for (int k = 0; k < 6; k++) {
        sel[k] = (a[k] >> 1) & 0x07070707u;
        const uint32_t sq = byte_lut8(sq_hi, sq_lo, sel[k]);
        p1 = sum_u8(a[k], p1);
        p2 = sum_u8(sq, p2);
        p4 = dot_u8(sq, sq, p4);
        sumx = sum_u8(a[k] & ~(((x[k] >> 7) & 0x01010101u) * 0xFFu), sumx);      // positive part
    }
    // sum x = (sum of positive parts) - (sum of negative parts) = 2 * positive - sum |x|
    const uint32_t sx = 2u * sumx - p1;
    ok = ok && ((sx & 7u) == (odd ? 4u : 0u));                                   // condition (iii)
    const uint32_t m = p2 >> 4;
    ok = ok && (p2 & 15u) == 0 && m >= 2 && m <= T.m_max;
    // condition (ii): the word must be a Golay word; its position among the sorted words
    const uint32_t gi = enc_at<uint16_t, kEncGinv>(T, (cw & 0xFFFu) * 2u);
    ok = ok && enc_at<uint32_t, kEncGs>(T, gi * 4u) == cw;
    // the class: leaders are told apart by (parity, sum |x|, sum x^4)
    const uint32_t key = (p4 & 0xFFFFFu) | (p1 & 0x1FFu) << 20 | odd << 29;
    const HashEnt h0 = enc_at<HashEnt, kEncHash>(T, ((key * T.hash_mult[0]) >> (32 - kEncHashBits)) * (uint32_t)sizeof(HashEnt));
    const HashEnt h1 = enc_at<HashEnt, kEncHash + (sizeof(HashEnt) << kEncHashBits)>(T, ((key * T.hash_mult[1]) >> (32 - kEncHashBits)) * (uint32_t)sizeof(HashEnt));
    ok = ok && (h0.key == key || h1.key == key) && p4 < (1u << 20) && p1 < (1u << 9);
    const uint32_t cid = !ok ? 0u : (h0.key == key ? h0.cid : h1.cid);
    const EncRec R = enc_at<EncRec, kEncCls>(T, cid * (uint32_t)sizeof(EncRec));
    const uint32_t f0 = R.f0, e1 = R.e1;
    ok = ok && R.key == key && ((f0 >> F0_M) & 15u) == m;

    // nibble code of every coordinate and the three code planes over the 24 positions
    uint32_t pa = 0, pb = 0, pd = 0, unknown = 0;
#pragma unroll
    for (int k = 0; k < 6; k++) {
        const uint32_t code = byte_lut8(R.ctab_hi, R.ctab_lo, sel[k]);
        unknown |= code;
        pa |= gather4(code & 0x01010101u) << (4 * k);
        pb |= gather4((code >> 1) & 0x01010101u) << (4 * k);
        pd |= gather4((code >> 2) & 0x01010101u) << (4 * k);
    }
    ok = ok && (unknown & 0x08080808u) == 0;                     // every value belongs to the leader

    const bool outer_all = (f0 >> F0_OUTER_ALL) & 1u;
    const bool f1direct = (f0 >> F0_F1DIRECT) & 1u;
    const uint32_t n = (f0 >> F0_N) & 31u, q = (f0 >> F0_Q) & 31u, wm1 = (f0 >> F0_WM1) & 31u;
    // U: the positions of the outer domain that do not hold its outside value; Uc: the same as slots of the domain
    const uint32_t U = outer_all ? pd : ((pa | pb) & ~pd);
    const uint32_t dom = outer_all ? 0xFFFFFFu : (~cw & 0xFFFFFFu);
    const uint32_t Uc = pext6n<4>(T, U, dom);
    ok = ok && popc32(U) == q && popc32(dom) == n;
    // subset rank: number j of slots >= 12, then colex rank of the high part, then of the low part
    const uint32_t hi = Uc >> 12, lo = Uc & 0xFFFu, j = popc32(hi);
    const SplitEnt se = enc_at<SplitEnt, kEncSplit>(T, (uint32_t)(uint16_t)(R.sp + j) * (uint32_t)sizeof(SplitEnt));
    const uint32_t d = se.base + (uint32_t)enc_at<uint16_t, kEncRank12>(T, hi * 2u) * se.div +
                       (uint32_t)enc_at<uint16_t, kEncRank12>(T, lo * 2u);
    // inner word on the slots of U, direct word on the slots of the Golay word
    const uint32_t a0 = pext6n<4>(T, pa, U), b0 = pext6n<4>(T, pb, U);
    const uint32_t rin = inner_word_rank(T, a0, b0, q, (e1 >> E1_DIG0) & 3u, (e1 >> E1_SYM0) & 1u, R.rad0[0], R.rad0[1]);
    uint32_t rho1 = 0;
    const uint32_t cwm = f1direct ? cw : 0u;
    if (wave_any(f1direct && ((e1 >> E1_DIG1) & 3u) != 0)) {
        const uint32_t a1 = pext6n<4>(T, pa, cwm), b1 = pext6n<4>(T, pb, cwm);
        rho1 = inner_word_rank(T, a1, b1, f1direct ? wm1 + 1u : 0u, f1direct ? (e1 >> E1_DIG1) & 3u : 0u, 0u, R.rad1[0], R.rad1[1]);
    }
    const uint64_t Ipp = ((uint64_t)d * R.Pin + rin) * R.P1 + rho1;
    // sign bits: the first w-1 slots of the word, then the nonzero F0 coordinates; odd classes have none
    const bool is_odd = (f0 >> F0_ODD) & 1u;
    const uint32_t s1 = is_odd ? 0u : (pext6n<4>(T, neg, cw) & ((1u << wm1) - 1u));
    const uint32_t s0 = outer_all ? 0u : pext6n<4>(T, neg, U);
    const uint64_t s = (uint64_t)s1 | ((uint64_t)s0 << wm1);
    const uint32_t B = (f0 >> F0_B) & 31u;
    const uint32_t acode = (e1 >> E1_ACODE) & 3u;
    const uint32_t A = acode == 0 ? 1u : (acode == 1 ? 759u : (acode == 2 ? 2576u : 4096u));
    const uint32_t r = gi - ((e1 >> E1_GOFF) & 4095u);
    const uint64_t I = R.offset + ((Ipp << B) + s) * A + r;
    return ok ? I : kInvalidIndex;
}

}  // namespace llvq
