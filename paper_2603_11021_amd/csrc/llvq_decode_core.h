// Index -> block reconstruction shared by all kernels (paper App. A, steps 1-4), written so that the
// same source also compiles for the host, where a test harness runs it against the tables without a GPU.
//
// One call decodes one 48-bit index into four 32-bit words of six nibbles each.  Word j covers positions
// 6j..6j+5; position p of the chunk sits in nibble slot kNibbleSlot[p].  A nibble is
//     bit 3: sign,  bits 0..2: value code, an index into the class's 8-entry value table.
// Nothing here branches on the class: odd classes, even classes and the degenerate weights 0 and 24 run
// the same instruction stream with different class-record fields, so a wavefront holding 64 different
// classes does not diverge (the only data-dependent loops are the two short table searches).
#pragma once
#include <cstdint>
#include <cmath>
#include <type_traits>

#include "llvq_tables.h"

#if defined(__HIPCC__)
#define LLVQ_HD __host__ __device__ __forceinline__
#else
#define LLVQ_HD inline
#endif

namespace llvq {

// The tables are addressed as `base + constant offset + key`.  On the device `base` is an LDS pointer whose value
// the kernels make the literal address 0 (they use no static LDS, so their dynamic LDS starts there; the host side
// checks this per kernel): constant and base then fold into the offset field of the LDS instruction and a table
// address costs no addition.
#if defined(__HIP_DEVICE_COMPILE__)
#define LLVQ_LDS __attribute__((address_space(3)))
#else
#define LLVQ_LDS
#endif
typedef const LLVQ_LDS unsigned char* TabBase;

struct TabPtrs {
    TabBase base;                  // LDS-resident part of the blob
    const unsigned char* gbase;    // the whole blob in global memory (for kernels that keep only its first part in LDS)
    uint32_t ncls;
    uint64_t npoints;
};

LLVQ_HD TabPtrs make_tab_ptrs(TabBase base, const unsigned char* gbase, const TableLayout& L) {
    TabPtrs T;
    T.base = base;
    T.gbase = gbase;
    T.ncls = L.ncls;
    T.npoints = L.npoints;
    return T;
}

// a table element of type V at p: records are read as 16-byte pieces (an LDS pointer cannot bind to the reference
// a struct copy takes)
template <typename V>
LLVQ_HD V tab_load(TabBase p) {
#if defined(__HIP_DEVICE_COMPILE__)
    if constexpr (std::is_class<V>::value && sizeof(V) == 8) {
        typedef uint32_t Piece __attribute__((ext_vector_type(2)));
        const Piece v = *reinterpret_cast<const LLVQ_LDS Piece*>(p);
        struct Pieces { uint32_t q[2]; } t = {{v[0], v[1]}};
        return __builtin_bit_cast(V, t);
    } else if constexpr (std::is_class<V>::value) {
        static_assert(sizeof(V) % 16 == 0, "records are 8 bytes or multiples of 16 bytes");
        struct Pieces { uint32_t q[sizeof(V) / 4]; } t;
        typedef uint32_t Piece __attribute__((ext_vector_type(4)));
        const LLVQ_LDS Piece* src = reinterpret_cast<const LLVQ_LDS Piece*>(p);
        for (uint32_t i = 0; i < sizeof(V) / 16; i++) {
            const Piece v = src[i];
            t.q[4 * i] = v[0]; t.q[4 * i + 1] = v[1]; t.q[4 * i + 2] = v[2]; t.q[4 * i + 3] = v[3];
        }
        return __builtin_bit_cast(V, t);
    } else {
        return *reinterpret_cast<const LLVQ_LDS V*>(p);
    }
#else
    return *reinterpret_cast<const V*>(p);
#endif
}

// element `byte_off` bytes into the table at constant offset OFF
template <typename V, uint32_t OFF>
LLVQ_HD V tab_at(const TabPtrs& T, uint32_t byte_off) {
    return tab_load<V>(T.base + OFF + byte_off);
}

// the same for the tables that stay in global memory
template <typename V, uint32_t OFF>
LLVQ_HD V gtab_at(const TabPtrs& T, uint32_t byte_off) {
    return *reinterpret_cast<const V*>(T.gbase + OFF + byte_off);
}

// product of two numbers below 2^24 (the 24-bit multiplier runs at full rate, the 32-bit one does not)
LLVQ_HD uint32_t mul24(uint32_t a, uint32_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __umul24(a, b);
#else
    return a * b;
#endif
}

LLVQ_HD uint32_t popc32(uint32_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
    return (uint32_t)__popc(v);
#else
    return (uint32_t)__builtin_popcount(v);
#endif
}

// bits off..off+5 of v.  On the device the extraction is kept as one v_bfe_u32: written with shift and mask the
// compiler folds a following scale into the mask and ends up with more instructions per table address.
LLVQ_HD uint32_t bfe6(uint32_t v, uint32_t off) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_ubfe(v, off, 6u);
#else
    return (v >> off) & 63u;
#endif
}

// Entry (F, m) of spread6 is dword F * kSpreadPitch + m (the odd pitch spreads equal m of different masks over
// the LDS banks).  Fx = F * 4 * kSpreadPitch; the source is bits o..o+5 of plane (bits past the mask's
// popcount do not change the entry's value).
LLVQ_HD uint32_t spread6_at(const TabPtrs& T, uint32_t Fx, uint32_t plane, uint32_t o) {
    return tab_at<uint32_t, kOffSpread6>(T, Fx + (bfe6(plane, o) << 2));
}

// Marks a product that several table addresses share: without it the compiler repeats the multiplication inside
// every address (a multiply-add each) instead of adding to the product once computed.
LLVQ_HD void keep_product(uint32_t& v) {
#if defined(__HIP_DEVICE_COMPILE__)
    asm("" : "+v"(v));
#else
    (void)v;
#endif
}

// any boolean function of three words: bit i of the result is bit (a_i b_i c_i) of the truth table TT
// (a = 0xF0, b = 0xCC, c = 0xAA), one v_bitop3_b32 on the device
template <uint32_t TT>
LLVQ_HD uint32_t lut3(uint32_t a, uint32_t b, uint32_t c) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_bitop3_b32(a, b, c, TT);
#else
    uint32_t r = 0;
    for (uint32_t i = 0; i < 8; i++)
        if ((TT >> i) & 1u) r |= ((i & 4u) ? a : ~a) & ((i & 2u) ? b : ~b) & ((i & 1u) ? c : ~c);
    return r;
#endif
}

// true when `v` holds for any active lane of the wavefront (always true on the host, where it only gates work)
LLVQ_HD bool wave_any(bool v) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_ballot_w64(v) != 0;
#else
    (void)v;
    return true;
#endif
}

// loop condition shared by the lanes of a wavefront: true while any lane still has work (the host has one lane)
LLVQ_HD bool wave_or(bool v) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_ballot_w64(v) != 0;
#else
    return v;
#endif
}

struct BlockInfo {
    uint32_t cid;                // class id
    uint32_t m;                  // shell
    float rnorm;                 // 1/sqrt(16 m): the factor that normalises the block to the unit sphere
    uint32_t vt8_lo, vt8_hi;     // value table of the class, fp8 bytes
    uint32_t vti_lo, vti_hi;     // value table of the class, int8
};

// App. A steps 1-2: shell and class of an index (< npoints) in one search over the global class offsets
struct ClassHit {
    uint32_t cid;     // class id
    uint64_t Ic;      // index inside the class
};

LLVQ_HD ClassHit find_class(const TabPtrs& T, uint64_t I) {
    // the bucket of the top bits names the class of the bucket's first index; the class of I is that one or one of
    // the next few.  Three candidates are tested per round (their offsets are read together), so that the rare lane
    // whose bucket spans several small classes does not make its whole wavefront wait for one table read per class.
    // The class is carried as the byte offset of its cls_off entry, so the candidates' addresses are constants
    // apart; the table ends with offset[ncls] = N and three entries above every index, which no lane passes.
    uint32_t c8 = tab_at<uint16_t, kOffBucket>(T, (uint32_t)(I >> kBucketShift) * 2u);
    for (;;) {
        const uint64_t o1 = tab_at<uint64_t, kOffClsOff + 8>(T, c8);
        const uint64_t o2 = tab_at<uint64_t, kOffClsOff + 16>(T, c8);
        const uint64_t o3 = tab_at<uint64_t, kOffClsOff + 24>(T, c8);
        const bool p1 = I >= o1, p2 = I >= o2, p3 = I >= o3;     // monotone: p3 implies p2 implies p1
        c8 += (p1 ? 8u : 0u) + (p2 ? 8u : 0u) + (p3 ? 8u : 0u);
        if (!wave_or(p3)) break;
    }
    ClassHit h;
    h.cid = c8 >> 3;
    h.Ic = I - tab_at<uint64_t, kOffClsOff>(T, c8);
    return h;
}

// App. A step 3 for a block whose class is known: the digits r, s, I'' = (d, rin, rho1) and the first table
// reads that depend on them.  Everything the placement needs later is carried in a Front.
struct Front {
    uint32_t cid, f0, f1;
    uint32_t c;                  // the Golay word selected by r
    uint32_t e0, e1;             // symbol planes over the slots of U and over the F1 slots
    uint32_t s, d;               // sign bits, rank of the subset U
    uint32_t sp_j;               // split entry guessed for d (index into the split table)
    uint32_t vt8_lo, vt8_hi, vti_lo, vti_hi;
    float rnorm;
};

// BIG_GLOBAL: the Golay words and the inner-word planes are read from global memory instead of LDS
// (GS_LDS: only the inner-word planes are; the kernel has copied the blob up to kOffInner);
// REC_GLOBAL: so is the class record
template <bool BIG_GLOBAL = false, bool REC_GLOBAL = false, bool GS_LDS = false>
LLVQ_HD Front decode_front(const TabPtrs& T, const ClassHit& hit) {
    Front F;
    const ClassRec R = REC_GLOBAL ? gtab_at<ClassRec, kOffCls>(T, mul24(hit.cid, (uint32_t)sizeof(ClassRec)))
                                  : tab_at<ClassRec, kOffCls>(T, mul24(hit.cid, (uint32_t)sizeof(ClassRec)));
    const uint32_t f0 = R.f0, f1 = R.f1;
    // r = Ic mod A, then B sign bits, then the permutation rank I''.  All quotients are exact: the operands are
    // integers below 2^48 held in doubles and the reciprocals are nudged upwards.
    const uint32_t acode = (f1 >> F1_ACODE) & 3u;
    const double A = tab_at<double, kOffAtab>(T, acode * 16u);
    const double invA = tab_at<double, kOffAtab + 8>(T, acode * 16u);
    // Ic < 2^48 as a double: its bits under the exponent of 2^52, minus 2^52 (two instructions instead of two
    // conversions, a scaling and an addition)
    const double x = __builtin_bit_cast(double, hit.Ic | 0x4330000000000000ull) - 4503599627370496.0;
    const double q1 = floor(x * invA);
    const uint32_t r = (uint32_t)fma(-q1, A, x);
    const int B = (int)((f0 >> F0_B) & 31u);
    const double ipp = floor(ldexp(q1, -B));
    F.s = (uint32_t)fma(-ipp, ldexp(1.0, B), q1);
    // I'' = (d * Pin + rin) * P1 + rho1
    const double dd = floor(ipp * R.invPP);
    const uint32_t rem = (uint32_t)fma(-dd, (double)R.PP, ipp);
    F.d = (uint32_t)dd;
    const uint32_t rin = (uint32_t)((double)rem * (double)R.invP1);
    const uint32_t rho1 = rem - mul24(rin, R.P1);             // rem < 2^22
    const uint32_t oc = (((f1 >> F1_GOFF) & 4095u) + r) * 4u, o0 = (R.tb0 + rin) * 4u, o1 = (R.tb1 + rho1) * 4u;
    F.c = (BIG_GLOBAL && !GS_LDS) ? gtab_at<uint32_t, kOffGs>(T, oc) : tab_at<uint32_t, kOffGs>(T, oc);
    F.e0 = BIG_GLOBAL ? gtab_at<uint32_t, kOffInner>(T, o0) : tab_at<uint32_t, kOffInner>(T, o0);
    F.e1 = BIG_GLOBAL ? gtab_at<uint32_t, kOffInner>(T, o1) : tab_at<uint32_t, kOffInner>(T, o1);
    const uint32_t j = tab_at<uint8_t, kOffGuess>(T, ((f1 >> F1_GROW) & 63u) * kGuessBuckets + (F.d >> ((f1 >> F1_GSHIFT) & 31u)));
    F.sp_j = (uint32_t)(uint16_t)(R.sp + j) | (j << 16);
    F.cid = hit.cid; F.f0 = f0; F.f1 = f1;
    F.vt8_lo = R.vt8_lo; F.vt8_hi = R.vt8_hi; F.vti_lo = R.vti_lo; F.vti_hi = R.vti_hi;
    F.rnorm = tab_at<float, kOffRnorm>(T, (f0 >> (F0_M - 2)) & 60u);
    return F;
}

// App. A step 4, first part: the q-subset U of the outer domain's n slots with rank d, relative to the domain
// (bit i = slot i of the domain); needs only the digits, not the Golay word
LLVQ_HD uint32_t decode_subset(const TabPtrs& T, const Front& F) {
    uint32_t j = F.sp_j >> 16, eo = (F.sp_j & 0xFFFFu) * (uint32_t)sizeof(SplitEnt);
    SplitEnt e = tab_at<SplitEnt, kOffSplit>(T, eo);
    uint32_t nbase = tab_at<uint32_t, kOffSplit + sizeof(SplitEnt)>(T, eo);   // one past the last entry is never used
    const uint32_t jmax = (F.f1 >> F1_JMAX) & 15u;
    for (;;) {
        const bool more = j < jmax && F.d >= nbase;
        if (more) {
            j++;
            eo += (uint32_t)sizeof(SplitEnt);
            e = tab_at<SplitEnt, kOffSplit>(T, eo);
            nbase = tab_at<uint32_t, kOffSplit + sizeof(SplitEnt)>(T, eo);
        }
        if (!wave_or(more)) break;
    }
    const uint32_t dl = F.d - e.base;
    const uint32_t rk_hi = (uint32_t)((double)dl * (double)e.inv);
    const uint32_t rk_lo = dl - mul24(rk_hi, e.div);          // dl < C(24, 12) < 2^22
    return (uint32_t)tab_at<uint16_t, kOffLut12>(T, (e.b12lo + rk_lo) * 2u) |
           ((uint32_t)tab_at<uint16_t, kOffLut12>(T, (e.b12hi + rk_hi) * 2u) << 12);
}

// App. A step 4, second part: placement and signs for the subset U.  w[0..3] receive the nibble words of the block.
LLVQ_HD BlockInfo decode_place(const TabPtrs& T, const Front& F, uint32_t U, uint32_t (&w)[4]) {
    BlockInfo info;
    const uint32_t f0 = F.f0;
    info.cid = F.cid; info.m = (f0 >> F0_M) & 15u;
    info.rnorm = F.rnorm;
    info.vt8_lo = F.vt8_lo; info.vt8_hi = F.vt8_hi; info.vti_lo = F.vti_lo; info.vti_hi = F.vti_hi;
    {
        // 16-bit planes; the deposit ignores source bits past the popcount of its mask, so e0 serves as its own low plane
        const uint32_t a0 = F.e0, b0 = F.e0 >> 16, a1 = F.e1, b1 = F.e1 >> 16;
        // signs: w-1 free bits on F1 then one bit per nonzero F0 coordinate; the last F1 slot is forced so
        // that the number of negative F1 coordinates has the parity condition (iii) asks for
        const uint32_t wm1 = (f0 >> F0_WM1) & 31u;
        uint32_t s1 = F.s & ((1u << wm1) - 1u);
        const uint32_t forced = (f0 >> F0_FEN) & ((f0 >> F0_KAPPA) ^ popc32(s1)) & 1u;
        s1 |= forced << wm1;
        const uint32_t s0 = F.s >> wm1;

        const bool odd = (f0 >> F0_ODD) & 1u;
        const bool outer_all = (f0 >> F0_OUTER_ALL) & 1u;
        const uint32_t cw = F.c;
        const uint32_t om = outer_all ? 0xFFFFFFu : (~cw & 0xFFFFFFu);      // positions of the outer domain
        const uint32_t sm = odd ? 0xFFFFFFu : cw;                           // positions taking a bit of sb
        const uint32_t sb = odd ? cw : s1;                                  // odd: the word itself flips signs
        const uint32_t dkeep = outer_all ? 0x04044444u : 0u;                // keep U as the domain bit
        // The planes of the direct F1 word go through the same mask as the sign bits: where there is such a word
        // (even class, 0 < w <= 16) both masks are the Golay word; everywhere else the planes are zero (the class
        // points at an all-zero table entry), so only the mask bit of their entries has to be dropped.
        const uint32_t f1keep = ((f0 >> F0_F1DIRECT) & 1u) ? 0x04044444u : 0u;

        // the running bit offsets start from a zero the compiler does not see through: with a literal 0 it rewrites the
        // first chunk's bit-field extracts into shift-and-mask forms that cost one more instruction per table address
        uint32_t zero = 0;
        keep_product(zero);
        uint32_t o0 = zero, os = zero, ou = zero;
        // U in absolute positions, all four chunks first: their table reads depend on nothing the chunk loop computes,
        // and issued together they cost one trip to LDS instead of one per chunk
        uint32_t uks[4];
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const uint32_t omk = bfe6(om, 6 * k);
            uks[k] = tab_at<uint8_t, kOffPdep6>(T, omk * kPdepPitch + bfe6(U, ou));
            ou += popc32(omk);
        }
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const uint32_t uk = uks[k];
            const uint32_t smk = bfe6(sm, 6 * k);
            uint32_t ux = uk * (4u * kSpreadPitch), sx = smk * (4u * kSpreadPitch);
            keep_product(sx); keep_product(ux);
            const uint32_t gA1 = spread6_at(T, sx, a1, os);
            const uint32_t gB1 = spread6_at(T, sx, b1, os);
            const uint32_t gS1 = spread6_at(T, sx, sb, os);
            os += popc32(smk);
            const uint32_t gA0 = spread6_at(T, ux, a0, o0);
            const uint32_t gB0 = spread6_at(T, ux, b0, o0);
            const uint32_t gS0 = spread6_at(T, ux, s0, o0);
            o0 += popc32(uk);
            // an entry holds the deposited bits in bit 0 and the mask in bit 2 of its nibbles
            const uint32_t ones = 0x01011111u;
            const uint32_t ta = lut3<0xE0>(ones, gA1, gA0), tb = lut3<0xE0>(ones, gB1, gB0), ts = lut3<0xE0>(ones, gS1, gS0);
            uint32_t v = (tb << 1) | ta;
            v = (ts << 3) | v;
            v = (gA1 & f1keep) | v;
            w[k] = lut3<0xEA>(gA0, dkeep, v);
        }
    }
    return info;
}

// App. A step 4 in one call
LLVQ_HD BlockInfo decode_back(const TabPtrs& T, const Front& F, uint32_t (&w)[4]) {
    return decode_place(T, F, decode_subset(T, F), w);
}

// Decodes one index I (must be < npoints); w[0..3] receive the nibble words.
LLVQ_HD BlockInfo decode_block(const TabPtrs& T, uint64_t I, uint32_t (&w)[4]) {
    return decode_back(T, decode_front(T, find_class(T, I)), w);
}

// v_perm_b32-style byte select restricted to selector values 0..7: byte k of the result is byte sel_k of hi:lo
LLVQ_HD uint32_t byte_lut8(uint32_t hi, uint32_t lo, uint32_t sel) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_perm(hi, lo, sel);
#else
    const uint64_t tab = ((uint64_t)hi << 32) | lo;
    uint32_t out = 0;
    for (int k = 0; k < 4; k++) out |= (uint32_t)((tab >> (8 * ((sel >> (8 * k)) & 7u))) & 0xFFu) << (8 * k);
    return out;
#endif
}

// Value bytes of one nibble word through an 8-entry table whose bytes carry a sign in bit 7 (fp8) or are
// two's complement int8.  ev = positions (0,1,4,5) of the chunk, od = positions (2,3) in its low half.
LLVQ_HD void chunk_codes(uint32_t w, uint32_t& ev, uint32_t& od) {
    ev = w & 0x07070707u;
    od = (w >> 4) & 0x00000707u;
}

// 24 int8 coordinates of a decoded block, position order, as six dwords
LLVQ_HD void nibbles_to_i8(const uint32_t w[4], uint32_t vt_lo, uint32_t vt_hi, uint32_t out[6]) {
    uint32_t ev[4], od[4];
#pragma unroll
    for (int k = 0; k < 4; k++) {
        uint32_t ce, co;
        chunk_codes(w[k], ce, co);
        uint32_t ve = byte_lut8(vt_hi, vt_lo, ce), vo = byte_lut8(vt_hi, vt_lo, co) & 0xFFFFu;
        // negate the bytes whose sign bit is set: (v ^ m) + (m & 1) per byte, no carries because v != 0 there
        uint32_t me = ((w[k] >> 3) & 0x01010101u) * 0xFFu, mo = ((w[k] >> 7) & 0x00000101u) * 0xFFu;
        ev[k] = (ve ^ me) + (me & 0x01010101u);
        od[k] = (vo ^ mo) + (mo & 0x01010101u);
    }
    // chunk k holds (q0 q1 q4 q5) in ev and (q2 q3) in od; two chunks make three dwords in position order
#pragma unroll
    for (int h = 0; h < 2; h++) {
        const uint32_t e0 = ev[2 * h], o0 = od[2 * h], e1 = ev[2 * h + 1], o1 = od[2 * h + 1];
        out[3 * h + 0] = (e0 & 0xFFFFu) | (o0 << 16);                    // q0 q1 q2 q3
        out[3 * h + 1] = (e0 >> 16) | (e1 << 16);                        // q4 q5 q0' q1'
        out[3 * h + 2] = (o1 & 0xFFFFu) | (e1 & 0xFFFF0000u);            // q2' q3' q4' q5'
    }
}

}  // namespace llvq
