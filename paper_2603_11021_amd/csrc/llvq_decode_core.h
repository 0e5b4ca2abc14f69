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

#include "llvq_tables.h"

#if defined(__HIPCC__)
#define LLVQ_HD __host__ __device__ __forceinline__
#else
#define LLVQ_HD inline
#endif

namespace llvq {

// The tables are addressed as `base + constant offset + key`; on the device `base` is the start of LDS and
// the constant folds into the offset field of the LDS instruction.
struct TabPtrs {
    const unsigned char* base;     // LDS-resident part of the blob
    const unsigned char* gbase;    // the whole blob in global memory (for kernels that keep only its first part in LDS)
    uint32_t ncls;
    uint64_t npoints;
};

LLVQ_HD TabPtrs make_tab_ptrs(const unsigned char* base, const unsigned char* gbase, const TableLayout& L) {
    TabPtrs T;
    T.base = base;
    T.gbase = gbase;
    T.ncls = L.ncls;
    T.npoints = L.npoints;
    return T;
}

// element `byte_off` bytes into the table at constant offset OFF
template <typename V, uint32_t OFF>
LLVQ_HD V tab_at(const TabPtrs& T, uint32_t byte_off) {
    return *reinterpret_cast<const V*>(T.base + OFF + byte_off);
}

// the same for the tables that stay in global memory
template <typename V, uint32_t OFF>
LLVQ_HD V gtab_at(const TabPtrs& T, uint32_t byte_off) {
    return *reinterpret_cast<const V*>(T.gbase + OFF + byte_off);
}

LLVQ_HD uint32_t popc32(uint32_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
    return (uint32_t)__popc(v);
#else
    return (uint32_t)__builtin_popcount(v);
#endif
}

LLVQ_HD uint32_t bfe6(uint32_t v, uint32_t off) { return (v >> off) & 63u; }

// Entry (F, m) of the 6-bit deposit tables sits at F*64 + (m ^ F): the frequent all-zero sources of different
// masks then fall into different LDS banks instead of all into bank 0.
// spread6: byte offset of entry (F, bits o..o+5 of plane) given plane2 = plane << 2 and Fx = F * 0x104
LLVQ_HD uint32_t spread6_at(const TabPtrs& T, uint32_t Fx, uint32_t plane2, uint32_t o) {
    return tab_at<uint32_t, kOffSpread6>(T, ((plane2 >> o) & 0xFCu) ^ Fx);
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
    uint32_t cid = tab_at<uint16_t, kOffBucket>(T, (uint32_t)(I >> kBucketShift) * 2u);
    uint64_t off = tab_at<uint64_t, kOffClsOff>(T, cid * 8u);
    for (;;) {
        const uint32_t last = T.ncls;                       // offset[ncls] = npoints > I: never passed
        const uint32_t c1 = cid + 1 < last ? cid + 1 : last, c2 = cid + 2 < last ? cid + 2 : last, c3 = cid + 3 < last ? cid + 3 : last;
        const uint64_t o1 = tab_at<uint64_t, kOffClsOff>(T, c1 * 8u);
        const uint64_t o2 = tab_at<uint64_t, kOffClsOff>(T, c2 * 8u);
        const uint64_t o3 = tab_at<uint64_t, kOffClsOff>(T, c3 * 8u);
        const bool p1 = I >= o1, p2 = I >= o2, p3 = I >= o3;     // monotone: p3 implies p2 implies p1
        off = p3 ? o3 : (p2 ? o2 : (p1 ? o1 : off));
        cid = p3 ? c3 : (p2 ? c2 : (p1 ? c1 : cid));
        if (!wave_or(p3)) break;
    }
    ClassHit h;
    h.cid = cid;
    h.Ic = I - off;
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
template <bool BIG_GLOBAL = false>
LLVQ_HD Front decode_front(const TabPtrs& T, const ClassHit& hit) {
    Front F;
    const ClassRec R = tab_at<ClassRec, kOffCls>(T, hit.cid * (uint32_t)sizeof(ClassRec));
    const uint32_t f0 = R.f0, f1 = R.f1;
    // r = Ic mod A, then B sign bits, then the permutation rank I''.  All quotients are exact: the operands are
    // integers below 2^48 held in doubles and the reciprocals are nudged upwards.
    const uint32_t acode = (f1 >> F1_ACODE) & 3u;
    const double A = tab_at<double, kOffAtab>(T, acode * 16u);
    const double invA = tab_at<double, kOffAtab + 8>(T, acode * 16u);
    const double x = (double)hit.Ic;
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
    const uint32_t rho1 = rem - rin * R.P1;
    const uint32_t oc = (((f1 >> F1_GOFF) & 4095u) + r) * 4u, o0 = (R.tb0 + rin) * 4u, o1 = (R.tb1 + rho1) * 4u;
    F.c = BIG_GLOBAL ? gtab_at<uint32_t, kOffGs>(T, oc) : tab_at<uint32_t, kOffGs>(T, oc);
    F.e0 = BIG_GLOBAL ? gtab_at<uint32_t, kOffInner>(T, o0) : tab_at<uint32_t, kOffInner>(T, o0);
    F.e1 = BIG_GLOBAL ? gtab_at<uint32_t, kOffInner>(T, o1) : tab_at<uint32_t, kOffInner>(T, o1);
    const uint32_t j = tab_at<uint8_t, kOffGuess>(T, ((f1 >> F1_GROW) & 63u) * kGuessBuckets + (F.d >> ((f1 >> F1_GSHIFT) & 31u)));
    F.sp_j = (uint32_t)(uint16_t)(R.sp + j) | (j << 16);
    F.cid = hit.cid; F.f0 = f0; F.f1 = f1;
    F.vt8_lo = R.vt8_lo; F.vt8_hi = R.vt8_hi; F.vti_lo = R.vti_lo; F.vti_hi = R.vti_hi;
    F.rnorm = tab_at<float, kOffRnorm>(T, (f0 >> (F0_M - 2)) & 60u);
    return F;
}

// App. A step 4: placement and signs.  w[0..3] receive the nibble words of the block.
LLVQ_HD BlockInfo decode_back(const TabPtrs& T, const Front& F, uint32_t (&w)[4]) {
    // the q-subset U of the outer domain's n slots with rank d
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
    const uint32_t rk_lo = dl - rk_hi * e.div;
    const uint32_t U = (uint32_t)tab_at<uint16_t, kOffLut12>(T, (e.b12lo + rk_lo) * 2u) |
                       ((uint32_t)tab_at<uint16_t, kOffLut12>(T, (e.b12hi + rk_hi) * 2u) << 12);

    BlockInfo info;
    const uint32_t f0 = F.f0;
    info.cid = F.cid; info.m = (f0 >> F0_M) & 15u;
    info.rnorm = F.rnorm;
    info.vt8_lo = F.vt8_lo; info.vt8_hi = F.vt8_hi; info.vti_lo = F.vti_lo; info.vti_hi = F.vti_hi;
    {
        // planes pre-shifted by two: the deposit keys below are byte offsets into a table of dwords
        const uint32_t a0 = (F.e0 & 0xFFFFu) << 2, b0 = (F.e0 >> 16) << 2, a1 = (F.e1 & 0xFFFFu) << 2, b1 = (F.e1 >> 16) << 2;
        // signs: w-1 free bits on F1 then one bit per nonzero F0 coordinate; the last F1 slot is forced so
        // that the number of negative F1 coordinates has the parity condition (iii) asks for
        const uint32_t wm1 = (f0 >> F0_WM1) & 31u;
        uint32_t s1 = F.s & ((1u << wm1) - 1u);
        const uint32_t forced = (f0 >> F0_FEN) & ((f0 >> F0_KAPPA) ^ popc32(s1)) & 1u;
        s1 |= forced << wm1;
        const uint32_t s0 = (F.s >> wm1) << 2;

        const bool odd = (f0 >> F0_ODD) & 1u;
        const bool outer_all = (f0 >> F0_OUTER_ALL) & 1u;
        const uint32_t cw = F.c;
        const uint32_t cm = ((f0 >> F0_F1DIRECT) & 1u) ? cw : 0u;           // slots of the direct F1 word
        const uint32_t om = outer_all ? 0xFFFFFFu : (~cw & 0xFFFFFFu);      // positions of the outer domain
        const uint32_t sm = odd ? 0xFFFFFFu : cw;                           // positions taking a bit of sb
        const uint32_t sb = (odd ? cw : s1) << 2;                           // odd: the word itself flips signs
        const uint32_t dkeep = outer_all ? 0x04044444u : 0u;                // keep U as the domain bit

        uint32_t o1 = 0, o0 = 0, os = 0, ou = 0;
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const uint32_t omk = bfe6(om, 6 * k);
            const uint32_t uk = tab_at<uint8_t, kOffPdep6>(T, (omk << 6) | (bfe6(U, ou) ^ omk));   // U in absolute positions
            ou += popc32(omk);
            const uint32_t cmk = bfe6(cm, 6 * k), smk = bfe6(sm, 6 * k);
            const uint32_t cx = cmk * 0x104u, ux = uk * 0x104u, sx = smk * 0x104u;
            const uint32_t gA1 = spread6_at(T, cx, a1, o1);
            uint32_t gB = spread6_at(T, cx, b1, o1);
            o1 += popc32(cmk);
            const uint32_t gA0 = spread6_at(T, ux, a0, o0);
            gB |= spread6_at(T, ux, b0, o0);
            const uint32_t gS0 = spread6_at(T, ux, s0, o0);
            o0 += popc32(uk);
            const uint32_t gS1 = spread6_at(T, sx, sb, os);
            os += popc32(smk);
            const uint32_t ones = 0x01011111u;
            w[k] = ((gA1 | gA0) & ones) | ((gB & ones) << 1) | (((gS1 | gS0) & ones) << 3) |
                      (gA1 & 0x04044444u) | (gA0 & dkeep);
        }
    }
    return info;
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
