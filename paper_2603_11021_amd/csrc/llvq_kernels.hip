// gfx950 kernels and the C ABI of the LLVQ library (see include/llvq.h for the contract).
//
// Work decomposition: one lane decodes one 24-block.  The constant tables live in LDS (66 to 157 KB, one
// 1024-thread workgroup per compute unit); a table access is an LDS gather (short launches of the batch-1 product
// read the two largest tables from global memory instead), every other step is VALU work on registers.  The fused product streams 8 bytes per block from HBM (6-byte index + fp16 gain),
// decodes the block into fp8-coded weights in registers, converts them pairwise to fp16 and feeds
// v_dot2_f32_f16 against activations that consecutive lanes read as consecutive 48-byte runs.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <rocblas/rocblas.h>
#include <type_traits>

#include <cstdio>
#include <algorithm>
#include <cstring>
#include <new>
#include <atomic>
#include <string>
#include <mutex>

#include "../../include/llvq.h"
#include "llvq_decode_core.h"
#include "llvq_encode_core.h"
#include "llvq_tables.h"
#include "llvq_wide.h"

namespace {

using llvq::ClassRec;
using llvq::TableLayout;
using llvq::TabPtrs;

constexpr int kThreads = 1024;

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));

extern __shared__ __align__(16) unsigned char g_lds[];

// Address 0 of LDS as a table base.  The kernels here declare no static LDS, so the dynamic LDS that receives the
// tables starts at 0 (set_lds checks that per kernel); with the base a literal, table offsets fold into the LDS
// instructions.  (Formed from a variable: a literal 0 would be the null pointer, which is not address 0 in LDS.)
__device__ __forceinline__ llvq::TabBase lds_origin() {
    uint32_t zero = 0;
    return (llvq::TabBase)(uintptr_t)zero;
}

template <int THREADS = kThreads>
__device__ __forceinline__ void load_tables(const unsigned char* __restrict__ blob, uint32_t bytes) {
    // global -> LDS without staging in registers: one wave instruction moves 64 x 16 B to 1 KB of consecutive LDS
    // addresses (base in M0, wave-uniform); chunks of 1 KB are dealt round-robin to the waves
    const uint32_t n16 = bytes / 16;
    const uint32_t wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const uint32_t nchunk = (n16 + 63) / 64;
    // workgroups start at different chunks: all of them copy the same bytes at the same time, and in the same order
    // they would all queue at the same L2 channel
    const uint32_t rot = (blockIdx.x * 5u) % nchunk;
    for (uint32_t c0 = wave; c0 < nchunk; c0 += THREADS / 64) {
        const uint32_t c = c0 + rot < nchunk ? c0 + rot : c0 + rot - nchunk;
        const uint32_t k = c * 64 + lane;
        if (k < n16)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(blob + (size_t)k * 16),
                                             (__attribute__((address_space(3))) void*)(g_lds + c * 1024), 16, 0, 0);
    }
    __builtin_amdgcn_s_waitcnt(0);          // vmcnt(0): the wave's copies have landed
    __syncthreads();
}

// sum over the 64 lanes of a wavefront, valid in lane 63 only: four DPP adds inside each row of 16 lanes, then the
// row totals travel to the following rows (row_bcast:15 into rows 1 and 3, row_bcast:31 into rows 2 and 3)
__device__ __forceinline__ float wave_sum_to_last(float v) {
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));  // row_half_mirror
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x140, 0xF, 0xF, true));  // row_mirror
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x142, 0xA, 0xF, false)); // row_bcast:15
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x143, 0xC, 0xF, false)); // row_bcast:31
    return v;
}


// LDS atomics issued by one lane of a wave.  With an address the compiler can prove wave-uniform it first combines
// the values of all active lanes (a scan over the exec mask, a dozen instructions) before one lane performs the
// operation; here a single lane is active by construction, so the address is made to look lane-dependent and the
// operation compiles to the one LDS instruction.
__device__ __forceinline__ uint32_t lane_zero() {
    uint32_t z = 0;
    asm volatile("" : "+v"(z));
    return z;
}
__device__ __forceinline__ void lds_add_one_lane(float* p, float v) { atomicAdd(p + lane_zero(), v); }
__device__ __forceinline__ uint32_t lds_fetch_add_one_lane(uint32_t* p, uint32_t v) { return atomicAdd(p + lane_zero(), v); }

template <int FMT>
__device__ __forceinline__ uint64_t load_index(const void* __restrict__ idx, size_t k) {
    if constexpr (FMT == LLVQ_IDX_U64) {
        return reinterpret_cast<const uint64_t*>(idx)[k];             // callers mask: the top 16 bits may carry a gain
    } else if constexpr (FMT == LLVQ_IDX_U24) {
        const uint8_t* p = reinterpret_cast<const uint8_t*>(idx) + 3 * k;
        return (uint64_t)p[0] | ((uint64_t)p[1] << 8) | ((uint64_t)p[2] << 16);
    } else {
        const uint16_t* p = reinterpret_cast<const uint16_t*>(idx) + 3 * k;
        return (uint64_t)p[0] | ((uint64_t)p[1] << 16) | ((uint64_t)p[2] << 32);
    }
}

// bytes of a stored code word
template <int FMT> constexpr uint32_t kWordBytes = FMT == LLVQ_IDX_U64 ? 8u : FMT == LLVQ_IDX_U24 ? 3u : 6u;

// How a stored code word maps to (lattice index, gain): index = (word & mask) + base; the gain is either the
// per-block fp16 array or entry (word >> shape_bits) of a small table (gain bits carried inside the word).
struct Code {
    uint64_t base;
    uint64_t mask;
    const uint16_t* lut;       // nullptr: gains come from the per-block array or from the word itself
    uint32_t shape_bits;
    uint32_t lut_last;         // last valid entry of lut
    uint32_t gain_in_word;     // 64-bit words only, lut == nullptr: bits 48..63 of the word are the block's fp16 gain
    // true when the kernels have to read the per-block gain array
    __host__ __device__ bool gain_array() const { return lut == nullptr && !gain_in_word; }
};

template <int FMT>
__device__ __forceinline__ void load_block(const void* __restrict__ idx, const uint16_t* __restrict__ gain, const Code& cd,
                                           size_t k, uint64_t& I, uint16_t& g) {
    const uint64_t v = load_index<FMT>(idx, k);
    if (cd.lut) g = cd.lut[min((uint32_t)((v & 0xFFFFFFFFFFFFull) >> cd.shape_bits), cd.lut_last)];
    else if (FMT == LLVQ_IDX_U64 && cd.gain_in_word) g = (uint16_t)(v >> 48);
    else g = gain ? gain[k] : (uint16_t)0;
    I = (v & cd.mask) + cd.base;
}

// The same in two steps for software-pipelined loops: load_raw only issues the loads (nothing in it depends on a
// loaded value, so no wait is placed there), finish_block turns the loaded pieces into (index, gain) where they are used.
struct RawBlock {
    uint32_t a, b, c;          // pieces of the stored word as loaded
    uint16_t g;                // per-block gain as loaded
};

template <int FMT>
__device__ __forceinline__ void load_raw(const void* __restrict__ idx, const uint16_t* __restrict__ gain, bool gain_array, size_t k,
                                         RawBlock& r) {
    r.a = r.b = r.c = 0;
    if constexpr (FMT == LLVQ_IDX_U64) {
        const uint32_t* p = reinterpret_cast<const uint32_t*>(idx) + 2 * k;
        r.a = p[0]; r.b = p[1];
    } else if constexpr (FMT == LLVQ_IDX_U24) {
        const uint8_t* p = reinterpret_cast<const uint8_t*>(idx) + 3 * k;
        r.a = p[0]; r.b = p[1]; r.c = p[2];
    } else {
        // one 4-byte load (2-byte aligned) and one 2-byte load: the pieces stay as loaded until finish_block
        typedef uint32_t u32_align2 __attribute__((aligned(2)));
        const unsigned char* p = reinterpret_cast<const unsigned char*>(idx) + 6 * k;
        r.a = *reinterpret_cast<const u32_align2*>(p);
        r.c = *reinterpret_cast<const uint16_t*>(p + 4);
    }
    // always a load (from the index array itself when gains come from a table; the value is then ignored): a load under
    // a condition would make later waits in a pipelined loop conservative
    const uint16_t* gp = gain_array ? gain : reinterpret_cast<const uint16_t*>(idx);
    r.g = gp[k];
}

// The same loads for a block `k` (below 2^24) past a wave-uniform position of the arrays: the addresses are then a
// scalar base plus a 32-bit lane offset, one multiplication each.
template <int FMT>
__device__ __forceinline__ void load_raw_near(const unsigned char* __restrict__ idx0, const unsigned char* __restrict__ gain0,
                                              uint32_t k, RawBlock& r) {
    r.a = r.b = r.c = 0;
    if constexpr (FMT == LLVQ_IDX_U64) {
        const uint32_t* p = reinterpret_cast<const uint32_t*>(idx0 + llvq::mul24(k, 8u));
        r.a = p[0]; r.b = p[1];
    } else if constexpr (FMT == LLVQ_IDX_U24) {
        const uint8_t* p = idx0 + llvq::mul24(k, 3u);
        r.a = p[0]; r.b = p[1]; r.c = p[2];
    } else {
        typedef uint32_t u32_align2 __attribute__((aligned(2)));
        const unsigned char* p = idx0 + llvq::mul24(k, 6u);
        r.a = *reinterpret_cast<const u32_align2*>(p);
        r.c = *reinterpret_cast<const uint16_t*>(p + 4);
    }
    r.g = *reinterpret_cast<const uint16_t*>(gain0 + 2u * k);
}

template <int FMT>
__device__ __forceinline__ void finish_block(const RawBlock& r, const Code& cd, uint64_t& I, uint16_t& g) {
    uint64_t v;
    if constexpr (FMT == LLVQ_IDX_U64) v = ((uint64_t)r.a | ((uint64_t)r.b << 32)) & 0xFFFFFFFFFFFFull;
    else if constexpr (FMT == LLVQ_IDX_U24) v = (uint64_t)(r.a | (r.b << 8) | (r.c << 16));
    else v = (uint64_t)r.a | ((uint64_t)r.c << 32);
    g = cd.lut ? cd.lut[min((uint32_t)(v >> cd.shape_bits), cd.lut_last)] : r.g;
    if constexpr (FMT == LLVQ_IDX_U64) { if (cd.gain_in_word) g = (uint16_t)(r.b >> 16); }
    I = (v & cd.mask) + cd.base;
}

// How the bulk-decode kernels hand blocks to their lanes.  Both forms keep the position of a wave's blocks wave-uniform
// (`base`, a scalar) with the lane's block at base + t, and both walk the array grid-stride, so that the blocks in
// flight on the chip at any time are neighbours in memory.
//   fixed   (short launches): the workgroup takes every gridDim.x-th run of kThreads blocks; t = thread number
//   dynamic (long launches):  the workgroup takes every gridDim.x-th batch of 64 blocks; a wave decodes the workgroup's
//                             batches `wave` and `wave + 16` and then takes its next free one through a counter in LDS
//                             (the 4 bytes behind the tables), one batch ahead of the one it decodes; t = lane.  The SIMDs
//                             of a compute unit do not get through their batches at the same rate, and this evens it out.
template <bool DYNAMIC>
struct BatchDeal {
    size_t base, next, end;
    uint32_t t, taken;
    uint32_t* next_free;
    __device__ __forceinline__ size_t batch_start(uint32_t b) const { return ((size_t)b * gridDim.x + blockIdx.x) * 64; }
    __device__ __forceinline__ BatchDeal(size_t n, uint32_t table_bytes) {
        taken = 0;
        end = n;
        next_free = reinterpret_cast<uint32_t*>(g_lds + table_bytes);
        if constexpr (DYNAMIC) {
            const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
            t = threadIdx.x & 63;
            base = batch_start(wave);
            next = batch_start(wave + kThreads / 64);
            if (threadIdx.x == 0) *next_free = 2 * kThreads / 64;                  // covered by the barrier of load_tables
        } else {
            t = threadIdx.x;
            base = (size_t)blockIdx.x * kThreads;
            next = base + (size_t)gridDim.x * kThreads;
        }
    }
    // ask for the batch after `next` (its number arrives while this batch is decoded)
    __device__ __forceinline__ void take() {
        if constexpr (DYNAMIC) { if (t == 0) taken = lds_fetch_add_one_lane(next_free, 1u); }
    }
    __device__ __forceinline__ void advance() {
        base = next;
        if constexpr (DYNAMIC) next = batch_start(__builtin_amdgcn_readfirstlane(taken));
        else next += (size_t)gridDim.x * kThreads;
    }
};

// ---- llvq_decode_i8 ---------------------------------------------------------------------------------
// BIG_GLOBAL as in matmul_kernel below: with the two big tables in global memory the LDS part is 66 KB and two
// workgroups share a compute unit (eight waves per SIMD, 64 registers per lane), which wins on launches that are not
// dominated by their HBM traffic
template <int FMT, bool BIG_GLOBAL, bool DYNAMIC>
__global__ void __launch_bounds__(kThreads, BIG_GLOBAL ? 8 : 4) decode_i8_kernel(const unsigned char* __restrict__ blob, TableLayout lay,
                                                             const void* __restrict__ idx, Code cd, size_t n,
                                                             uint32_t* __restrict__ out) {
    BatchDeal<DYNAMIC> deal(n, BIG_GLOBAL ? lay.lds_bytes : lay.blob_bytes);
    load_tables(blob, BIG_GLOBAL ? lay.lds_bytes : lay.blob_bytes);
    const TabPtrs T = llvq::make_tab_ptrs(lds_origin(), blob, lay);
    // The streamed arrays are addressed as scalar base + 32-bit lane offset (BatchDeal).  The next word is requested
    // (always: past the end the last one is read again) before this block is decoded.
    const uint32_t t = deal.t;
    auto request = [&](size_t base, RawBlock& r) {
        const size_t b0 = base < n ? base : n - 1;
        const unsigned char* idx0 = reinterpret_cast<const unsigned char*>(idx) + b0 * kWordBytes<FMT>;
        load_raw_near<FMT>(idx0, idx0, (uint32_t)min((size_t)t, n - 1 - b0), r);
    };
    RawBlock raw, raw_next;
    if (deal.base < deal.end) request(deal.base, raw);
    for (; deal.base < deal.end; deal.advance(), raw = raw_next) {
        request(deal.next, raw_next);
        deal.take();
        const size_t base = deal.base;
        uint64_t I;
        uint16_t gdummy;
        finish_block<FMT>(raw, cd, I, gdummy);
        const bool ok = I < T.npoints;
        uint32_t w[4], o[6];
        const llvq::BlockInfo bi = llvq::decode_back(T, llvq::decode_front<BIG_GLOBAL>(T, llvq::find_class(T, ok ? I : 0)), w);
        llvq::nibbles_to_i8(w, bi.vti_lo, bi.vti_hi, o);
        if (base + t < n) {
            uint2* dst = reinterpret_cast<uint2*>(reinterpret_cast<unsigned char*>(out + 6 * base) + llvq::mul24(t, 24u));
            dst[0] = ok ? make_uint2(o[0], o[1]) : make_uint2(0, 0);
            dst[1] = ok ? make_uint2(o[2], o[3]) : make_uint2(0, 0);
            dst[2] = ok ? make_uint2(o[4], o[5]) : make_uint2(0, 0);
        }
    }
}

// fp8 (e4m3) byte pair -> two fp16 / bf16, exact for the small integers stored in the value tables
__device__ __forceinline__ half2_t fp8x2_to_f16(uint32_t v, bool hi) {
    return hi ? __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(v, 1.0f, true) : __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(v, 1.0f, false);
}
__device__ __forceinline__ bf16x2_t fp8x2_to_bf16(uint32_t v, bool hi) {
    return hi ? __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(v, 1.0f, true) : __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(v, 1.0f, false);
}

// signed fp8 bytes of chunk word w: fe = positions (0,1,4,5), fo = positions (2,3)
__device__ __forceinline__ void chunk_fp8(uint32_t w, uint32_t vt_lo, uint32_t vt_hi, uint32_t& fe, uint32_t& fo) {
    uint32_t ce, co;
    llvq::chunk_codes(w, ce, co);
    fe = llvq::byte_lut8(vt_hi, vt_lo, ce) ^ ((w << 4) & 0x80808080u);
    fo = llvq::byte_lut8(vt_hi, vt_lo, co) ^ (w & 0x00008080u);
}

// ---- llvq_decode (shape-gain reconstruction) ------------------------------------------------------------
template <int FMT, int OUT, bool BIG_GLOBAL>
__global__ void __launch_bounds__(kThreads, BIG_GLOBAL ? 8 : 4) dequant_kernel(const unsigned char* __restrict__ blob, TableLayout lay,
                                                           const void* __restrict__ idx, const uint16_t* __restrict__ gain,
                                                           Code cd, size_t n, void* __restrict__ out) {
    BatchDeal<!BIG_GLOBAL> deal(n, BIG_GLOBAL ? lay.lds_bytes : lay.blob_bytes);
    load_tables(blob, BIG_GLOBAL ? lay.lds_bytes : lay.blob_bytes);
    const TabPtrs T = llvq::make_tab_ptrs(lds_origin(), blob, lay);
    // batches and addressing as in decode_i8_kernel; the next word and gain are requested before this block is decoded
    const uint32_t t = deal.t;
    auto request = [&](size_t base, RawBlock& r) {
        const size_t b0 = base < n ? base : n - 1;
        const unsigned char* idx0 = reinterpret_cast<const unsigned char*>(idx) + b0 * kWordBytes<FMT>;
        const unsigned char* gain0 = cd.gain_array() ? reinterpret_cast<const unsigned char*>(gain + b0) : idx0;
        load_raw_near<FMT>(idx0, gain0, (uint32_t)min((size_t)t, n - 1 - b0), r);
    };
    RawBlock raw, raw_next;
    if (deal.base < deal.end) request(deal.base, raw);
    for (; deal.base < deal.end; deal.advance(), raw = raw_next) {
        request(deal.next, raw_next);
        deal.take();
        const size_t base = deal.base;
        const bool live = base + t < n;
        uint64_t I;
        uint16_t gb;
        finish_block<FMT>(raw, cd, I, gb);
        const bool ok = I < T.npoints;
        uint32_t w[4];
        const llvq::BlockInfo bi = llvq::decode_back(T, llvq::decode_front<BIG_GLOBAL>(T, llvq::find_class(T, ok ? I : 0)), w);
        const uint32_t vt_lo = bi.vt8_lo, vt_hi = bi.vt8_hi;
        const float g = __half2float(__ushort_as_half(gb));
        const float scale = ok ? g * bi.rnorm : 0.0f;
        // the signed fp8 bytes of a chunk come as pairs of positions (0,1), (2,3), (4,5); a pair is converted, scaled in
        // fp32 and rounded once to the output type
        typedef float float2_t __attribute__((ext_vector_type(2)));
        uint32_t pair[12];
#pragma unroll
        for (int c = 0; c < 4; c++) {
            uint32_t fe, fo;
            chunk_fp8(w[c], vt_lo, vt_hi, fe, fo);
            pair[3 * c + 0] = fe; pair[3 * c + 1] = fo; pair[3 * c + 2] = fe;
        }
        if constexpr (OUT == LLVQ_F32) {
            float2_t f[12];
#pragma unroll
            for (int i = 0; i < 12; i++)
                f[i] = (i % 3 == 2 ? __builtin_amdgcn_cvt_pk_f32_fp8(pair[i], true) : __builtin_amdgcn_cvt_pk_f32_fp8(pair[i], false)) * scale;
            float4* dst = reinterpret_cast<float4*>(reinterpret_cast<unsigned char*>(reinterpret_cast<float*>(out) + 24 * base) + llvq::mul24(t, 96u));
            if (live) {
#pragma unroll
                for (int i = 0; i < 6; i++) dst[i] = make_float4(f[2 * i][0], f[2 * i][1], f[2 * i + 1][0], f[2 * i + 1][1]);
            }
        } else {
            uint32_t pk[12];
#pragma unroll
            for (int i = 0; i < 12; i++) {
                // round to nearest even with the hardware conversions
                const float2_t f = (i % 3 == 2 ? __builtin_amdgcn_cvt_pk_f32_fp8(pair[i], true) : __builtin_amdgcn_cvt_pk_f32_fp8(pair[i], false)) * scale;
                if constexpr (OUT == LLVQ_F16) pk[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, half2_t));
                else pk[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
            }
            uint4* dst = reinterpret_cast<uint4*>(reinterpret_cast<unsigned char*>(reinterpret_cast<uint16_t*>(out) + 24 * base) + llvq::mul24(t, 48u));
            if (live) {
                dst[0] = make_uint4(pk[0], pk[1], pk[2], pk[3]);
                dst[1] = make_uint4(pk[4], pk[5], pk[6], pk[7]);
                dst[2] = make_uint4(pk[8], pk[9], pk[10], pk[11]);
            }
        }
    }
}

// ---- llvq_matmul, lane-per-block kernel ---------------------------------------------------------------
// A workgroup owns `rows_per_wg` consecutive rows, i.e. a contiguous run of rows_per_wg*KB blocks of the
// row-major index and gain arrays; wave-batches of 64 consecutive blocks are dealt to the 16 waves.  Per block and activation row the 24 products are accumulated by v_dot2_f32_f16 in fp32, scaled by
// gain/sqrt(16 m), reduced over the lanes that share an output row and added to that row's LDS accumulator.
constexpr int kMaxMChunk = 2;     // activation rows handled per pass over the indices
constexpr int kRowsPerPass = 64;  // output rows accumulated in LDS at a time

template <typename X2> struct Dot;
template <> struct Dot<half2_t> {
    static __device__ __forceinline__ half2_t cvt(uint32_t v, bool hi) { return fp8x2_to_f16(v, hi); }
    static __device__ __forceinline__ float dot(half2_t a, half2_t b, float c) { return __builtin_amdgcn_fdot2(a, b, c, false); }
};
template <> struct Dot<bf16x2_t> {
    static __device__ __forceinline__ bf16x2_t cvt(uint32_t v, bool hi) { return fp8x2_to_bf16(v, hi); }
    static __device__ __forceinline__ float dot(bf16x2_t a, bf16x2_t b, float c) { return __builtin_amdgcn_fdot2_f32_bf16(a, b, c, false); }
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// BIG_GLOBAL: only the small tables are copied into LDS and the Golay words and inner-word planes are read from global
// memory (short launches, where the table copy is a visible share); otherwise the whole blob is copied (long launches).
// DYNAMIC: after its first two batches a wave takes the next free batch instead of every 16th one (long launches: the
// SIMDs do not get through their batches at the same rate; short ones are faster with the fixed deal).
// MULTI: the rows are those of up to four matrices that share x, K and the word format, one after the other (`items`);
// a pass over the LDS accumulators never crosses from one matrix into the next.
constexpr int kMaxItems = 4;
struct MatItems {
    const void* idx[kMaxItems];
    const uint16_t* gain[kMaxItems];
    float* y[kMaxItems];
    int row_end[kMaxItems];        // rows of matrices 0..i together; entries past the last matrix repeat the total
    int tile_end[kMaxItems];       // the same in tiles of 32 rows, every matrix rounded up (mfma_kernel)
    int tile16_end[kMaxItems];     // the same in tiles of 16 rows (tile_kernel)
    int strip_end[kMaxItems];      // the same in strips of 128 rows (panel_kernel)
};

template <int FMT, typename X2, bool BIG_GLOBAL, bool DYNAMIC, bool MULTI = false>
__global__ void __launch_bounds__(kThreads) matmul_kernel(const unsigned char* __restrict__ blob, TableLayout lay,
                                                          const void* __restrict__ idx, const uint16_t* __restrict__ gain,
                                                          const uint32_t* __restrict__ x, int M, int N, int KB,
                                                          Code cd, uint32_t kb_magic, int rows_per_wg, int rows_per_pass, MatItems items,
                                                          float* __restrict__ y) {
    const int wg_r0 = blockIdx.x * rows_per_wg;
    const int wg_r1 = min(N, wg_r0 + rows_per_wg);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // scalar: loop control below is wave-uniform
    // The matrix that holds row r of the concatenation, and what a pass starting there works on: its arrays, its output,
    // its first row and the number of rows the pass may take (all wave-uniform).
    struct Pass { const void* idx; const uint16_t* gain; float* y; int first, rows, n_out; };
    auto pass_at = [&](int r) {
        Pass p = {idx, gain, y, 0, min(rows_per_pass, wg_r1 - r), N};
        if constexpr (MULTI) {
            int it = 0;
#pragma unroll
            for (int i = 0; i + 1 < kMaxItems; i++) {
                if (r >= items.row_end[i]) { it = i + 1; p.first = items.row_end[i]; }
            }
            p.idx = items.idx[it]; p.gain = items.gain[it]; p.y = items.y[it];
            p.rows = min(p.rows, items.row_end[it] - r);
            p.n_out = items.row_end[it] - p.first;
        }
        return p;
    };
    // the words of this wave's first batch are requested now: their trip from HBM overlaps the table copy below
    RawBlock first_raw;
    {
        const Pass p = pass_at(wg_r0);
        const uint32_t nblk = (uint32_t)p.rows * (uint32_t)KB;
        const size_t blk0 = (size_t)(wg_r0 - p.first) * KB;
        const unsigned char* idx0 = reinterpret_cast<const unsigned char*>(p.idx) + blk0 * kWordBytes<FMT>;
        const unsigned char* gain0 = cd.gain_array() ? reinterpret_cast<const unsigned char*>(p.gain + blk0) : idx0;
        load_raw_near<FMT>(idx0, gain0, min((uint32_t)wave * 64u + (uint32_t)lane, nblk - 1), first_raw);
    }
    // one workgroup per compute unit: the tables are copied once per launch and workgroup
    const uint32_t table_bytes = BIG_GLOBAL ? llvq::kOffInner : lay.blob_bytes;      // short launches: small tables + Golay words
    float* ysum = reinterpret_cast<float*>(g_lds + table_bytes);      // [kRowsPerPass][kMaxMChunk]
    // the first block number no wave has taken yet: the first two batches of a wave are fixed, after them it takes the
    // next free one, so waves on a SIMD that gets through its batches sooner end up with more of them
    uint32_t* next_free = reinterpret_cast<uint32_t*>(ysum + kRowsPerPass * kMaxMChunk);
    // the accumulators of the first pass are cleared here: the barrier that ends the table copy covers them too
    for (int i = threadIdx.x; i < kRowsPerPass * kMaxMChunk; i += kThreads) ysum[i] = 0.0f;
    if (DYNAMIC && threadIdx.x == 0) *next_free = 2 * kThreads;
    load_tables(blob, table_bytes);
    const TabPtrs T = llvq::make_tab_ptrs(lds_origin(), blob, lay);
    const size_t xpitch = (size_t)KB * 12;                              // dwords per activation row

    // rows_per_pass <= kRowsPerPass keeps a pass below 2^24 blocks (block numbers inside a pass go through 24-bit multiplies)
    int nrows = 0;
    for (int r0 = wg_r0; r0 < wg_r1; r0 += nrows) {
        const Pass ps = pass_at(r0);
        nrows = ps.rows;
        const uint32_t nblk = (uint32_t)nrows * (uint32_t)KB;
        const size_t blk0 = (size_t)(r0 - ps.first) * KB;
        // wave-uniform starts of this pass in the index and gain arrays (gains from a table: any readable address)
        const unsigned char* idx0 = reinterpret_cast<const unsigned char*>(ps.idx) + blk0 * kWordBytes<FMT>;
        const unsigned char* gain0 = cd.gain_array() ? reinterpret_cast<const unsigned char*>(ps.gain + blk0) : idx0;
        for (int m0 = 0; m0 < M; m0 += kMaxMChunk) {
            const int mc = min(kMaxMChunk, M - m0);
            if (r0 != wg_r0 || m0 != 0) {
                for (int i = threadIdx.x; i < nrows * kMaxMChunk; i += kThreads) ysum[i] = 0.0f;
                if (DYNAMIC && threadIdx.x == 0) *next_free = 2 * kThreads;
                __syncthreads();
            }
            // a wave starts with batches `wave` and `wave + 16` and then takes every 16th batch of 64 blocks or (DYNAMIC)
            // free batches one at a time, one batch ahead of the one it decodes.  Software pipeline over the batches: the indices and gains of
            // the next batch are requested before this one is decoded, and the next batch's class search and digit
            // extraction (a chain of dependent table reads) run before this batch's products, which hide their latency
            struct Fetch { RawBlock raw; uint32_t row, b; uint16_t g; bool live; };
            auto place = [&](uint32_t base, Fetch& f) {
                const uint32_t fb = base + lane;
                f.live = fb < nblk;
                const uint32_t fbc = f.live ? fb : nblk - 1;
                // fbc < 64*KB and KB < 8192: ceil(2^32/KB) is an exact reciprocal; otherwise divide
                f.row = kb_magic ? __umulhi(fbc, kb_magic) : fbc / (uint32_t)KB;
                f.b = fbc - llvq::mul24(f.row, (uint32_t)KB);
                return fbc;
            };
            auto fetch = [&](uint32_t base, Fetch& f) { load_raw_near<FMT>(idx0, gain0, place(base, f), f.raw); };
            auto front_of = [&](Fetch& f, bool& ok) {
                uint64_t I;
                finish_block<FMT>(f.raw, cd, I, f.g);
                ok = f.live && I < T.npoints;
                // long launches (all tables in LDS) read the class record through the otherwise idle vector cache: the LDS
                // gather pipe is as busy as the vector ALUs there, and three 16-byte gathers per block are a tenth of its load
                return llvq::decode_front<BIG_GLOBAL, !BIG_GLOBAL, true>(T, llvq::find_class(T, ok ? I : 0));
            };
            uint32_t base = (uint32_t)wave * 64, next = base + kThreads, taken = 0;
            Fetch cur, nxt;
            llvq::Front front_cur, front_nxt;
            bool ok_cur = false, ok_nxt = false;
            if (base < nblk) {
                if (r0 == wg_r0 && m0 == 0) {                        // the batch requested before the table copy
                    place(base, cur);
                    cur.raw = first_raw;
                } else {
                    fetch(base, cur);
                }
                front_cur = front_of(cur, ok_cur);
            }
            // one batch: kMore says whether another batch follows.  The two cases are separate copies of the code so that
            // each is straight-line with respect to its memory operations: a load inside a branch would make every later
            // wait count as if it had not been issued, i.e. wait for newer loads than it needs
            auto batch = [&](auto more_tag) {
                constexpr bool kMore = decltype(more_tag)::value;
                if constexpr (kMore) {
                    fetch(next, nxt);
                    if (DYNAMIC && lane == 0) taken = lds_fetch_add_one_lane(next_free, 64u);      // the batch after that one
                }
                u32x4 xq[1][3];
                {
                    const u32x4* xp = reinterpret_cast<const u32x4*>(reinterpret_cast<const unsigned char*>(x + (size_t)m0 * xpitch) + llvq::mul24(cur.b, 48u));
                    xq[0][0] = xp[0]; xq[0][1] = xp[1]; xq[0][2] = xp[2];
                }
                uint32_t w[1][4];
                llvq::BlockInfo bi[1];
                bi[0] = llvq::decode_back(T, front_cur, w[0]);
                if constexpr (kMore) front_nxt = front_of(nxt, ok_nxt);
                {
                    constexpr int u = 0;
                    const uint32_t vt_lo = bi[u].vt8_lo, vt_hi = bi[u].vt8_hi;
                    const float g = __half2float(__ushort_as_half(cur.g));
                    const float scale = ok_cur ? g * bi[u].rnorm : 0.0f;
                    X2 wt[12];
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        uint32_t fe, fo;
                        chunk_fp8(w[u][c], vt_lo, vt_hi, fe, fo);
                        wt[3 * c + 0] = Dot<X2>::cvt(fe, false);   // positions 6c+0, 6c+1
                        wt[3 * c + 1] = Dot<X2>::cvt(fo, false);   // positions 6c+2, 6c+3
                        wt[3 * c + 2] = Dot<X2>::cvt(fe, true);    // positions 6c+4, 6c+5
                    }
                    // rows are contiguous runs of lanes; with KB >= 64 a batch touches at most two rows
                    const uint32_t row = cur.row;
                    const uint32_t row_lo = __builtin_amdgcn_readfirstlane(row);
                    const uint32_t row_hi = __builtin_amdgcn_readlane(row, 63);
                    const bool two_rows = row_hi <= row_lo + 1;
                    for (int mi = 0; mi < mc; mi++) {
                        u32x4 x0 = xq[u][0], x1 = xq[u][1], x2 = xq[u][2];
                        if (mi > 0) {
                            const u32x4* xp = reinterpret_cast<const u32x4*>(reinterpret_cast<const unsigned char*>(x + (size_t)(m0 + mi) * xpitch) + llvq::mul24(cur.b, 48u));
                            x0 = xp[0]; x1 = xp[1]; x2 = xp[2];
                        }
                        const uint32_t xs[12] = {x0.x, x0.y, x0.z, x0.w, x1.x, x1.y, x1.z, x1.w, x2.x, x2.y, x2.z, x2.w};
                        float acc = 0.0f;
#pragma unroll
                        for (int i = 0; i < 12; i++) acc = Dot<X2>::dot(wt[i], __builtin_bit_cast(X2, xs[i]), acc);
                        float p = cur.live ? acc * scale : 0.0f;
                        if (row_hi == row_lo) {                                  // the whole batch lies in one row
                            const float s_all = wave_sum_to_last(p);
                            if (lane == 63) lds_add_one_lane(&ysum[row_lo * kMaxMChunk + mi], s_all);
                        } else if (two_rows) {
                            const float p_lo = row == row_lo ? p : 0.0f;
                            const float s_lo = wave_sum_to_last(p_lo), s_hi = wave_sum_to_last(p - p_lo);
                            if (lane == 63) {
                                lds_add_one_lane(&ysum[row_lo * kMaxMChunk + mi], s_lo);
                                lds_add_one_lane(&ysum[row_hi * kMaxMChunk + mi], s_hi);
                            }
                        } else {
                            // general case: segmented suffix sum over lanes of equal row
                            const uint32_t row_up = __shfl_up(row, 1);
                            const bool head = (lane == 0) || (row_up != row);
#pragma unroll
                            for (int off = 1; off < 64; off <<= 1) {
                                const float pv = __shfl_down(p, off);
                                const uint32_t rv = __shfl_down(row, off);
                                if (lane + off < 64 && rv == row) p += pv;
                            }
                            if (head && cur.live) atomicAdd(&ysum[row * kMaxMChunk + mi], p);
                        }
                    }
                }
            };
            while (next < nblk) {
                batch(std::true_type{});
                cur = nxt;
                front_cur = front_nxt;
                ok_cur = ok_nxt;
                base = next;
                next = DYNAMIC ? __builtin_amdgcn_readfirstlane(taken) : next + kThreads;
            }
            if (base < nblk) batch(std::false_type{});
            __syncthreads();
            for (int i = threadIdx.x; i < nrows * mc; i += kThreads) {
                const int rr = i / mc, mi = i - rr * mc;
                ps.y[(size_t)(m0 + mi) * ps.n_out + (r0 - ps.first) + rr] = ysum[rr * kMaxMChunk + mi];
            }
            __syncthreads();
        }
    }
}

// ---- llvq_matmul, MFMA kernel for 2 <= M (batched decode and prefill) --------------------------------------
// A wave owns 32 weight rows and two neighbouring blocks of 24 input channels per step: lanes 0..31 decode
// block b of rows r0..r0+31, lanes 32..63 block b+1 of the same rows.  The decoded block, scaled by
// gain/sqrt(16 m) and rounded to the activation type, is exactly the B operand of v_mfma_f32_32x32x16 (lane l
// supplies k = 8*(l/32)..+7 of column l%32), so the weights go from the decoder's registers straight into the
// matrix cores; the A operand (32 tokens x the same 16 channels) is read from global memory.  Three MFMAs consume
// the 24 channels of both blocks.  The block pairs of a row are cut into ranges that different workgroups take (split
// along K), partial tiles are added to y with fp32 atomics, y is cleared first by fill_kernel.
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));

// 16-byte stores over the aligned middle of p[0..n), single floats at its ends
__global__ void fill_kernel(float* __restrict__ p, size_t n, float v) {
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x, nthreads = (size_t)gridDim.x * blockDim.x;
    const size_t head = min(n, (size_t)(((16 - (reinterpret_cast<uintptr_t>(p) & 15)) & 15) / 4));
    float4* q = reinterpret_cast<float4*>(p + head);
    const size_t n4 = (n - head) / 4, tail = n - head - 4 * n4;
    for (size_t i = tid; i < n4; i += nthreads) q[i] = make_float4(v, v, v, v);
    if (tid < head) p[tid] = v;
    if (tid < tail) p[head + 4 * n4 + tid] = v;
}

// the same for the outputs of several matrices: blockIdx.y picks the matrix, M * (its rows) floats each
__global__ void fill_multi_kernel(MatItems items, int M, float v) {
    const int it = blockIdx.y;
    float* p = items.y[it];
    const size_t n = (size_t)M * (size_t)(items.row_end[it] - (it ? items.row_end[it - 1] : 0));
    const size_t tid = (size_t)blockIdx.x * blockDim.x + threadIdx.x, nthreads = (size_t)gridDim.x * blockDim.x;
    const size_t head = min(n, (size_t)(((16 - (reinterpret_cast<uintptr_t>(p) & 15)) & 15) / 4));
    float4* q = reinterpret_cast<float4*>(p + head);
    const size_t n4 = (n - head) / 4, tail = n - head - 4 * n4;
    for (size_t i = tid; i < n4; i += nthreads) q[i] = make_float4(v, v, v, v);
    if (tid < head) p[tid] = v;
    if (tid < tail) p[head + 4 * n4 + tid] = v;
}

// Mma<X2>::weights turns a pair of fp8-coded coordinates into kTerms dwords of scaled weights in the activation type.
// fp16: one term (11 significant bits).  bf16: two terms, the bf16 rounding of the fp32 product and the bf16 rounding of
// what that leaves (16 significant bits together; one term alone would put 2^-9 per weight into y), each contracted by
// its own MFMA against the same activations.
template <typename X2> struct Mma;
template <> struct Mma<half2_t> {
    static constexpr int kTerms = 1;
    static __device__ __forceinline__ void weights(uint32_t fp8, bool hi, float scale, uint32_t (&out)[1]) { out[0] = scaled(fp8, hi, scale); }
    static __device__ __forceinline__ uint32_t scaled(uint32_t fp8, bool hi, float scale) {
        const half2_t h = fp8x2_to_f16(fp8, hi);
        const _Float16 sh = (_Float16)scale;
        const half2_t r = h * half2_t{sh, sh};
        return __builtin_bit_cast(uint32_t, r);
    }
    // c += A B over 16 values of k: lane l holds k = 8 (l / 32) .. + 7 of row (A) or column (B) l % 32
    static __device__ __forceinline__ float16_t mma(u32x4 a, u32x4 b, float16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mma<bf16x2_t> {
    static constexpr int kTerms = 2;
    static __device__ __forceinline__ void weights(uint32_t fp8, bool hi, float scale, uint32_t (&out)[2]) {
        // fp8 pair -> fp32 pair, scale in fp32, round to nearest even with the hardware conversion; the remainder is exact
        typedef float float2_t __attribute__((ext_vector_type(2)));
        float2_t f = hi ? __builtin_amdgcn_cvt_pk_f32_fp8(fp8, true) : __builtin_amdgcn_cvt_pk_f32_fp8(fp8, false);
        f *= scale;
        const bf16x2_t top = __builtin_convertvector(f, bf16x2_t);
        const float2_t rest = f - __builtin_convertvector(top, float2_t);
        out[0] = __builtin_bit_cast(uint32_t, top);
        out[1] = __builtin_bit_cast(uint32_t, __builtin_convertvector(rest, bf16x2_t));
    }
    static __device__ __forceinline__ float16_t mma(u32x4 a, u32x4 b, float16_t c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};

constexpr int kGemmMinM = 96;       // from this many activation rows on, llvq_matmul_ws dequantises once and calls a dense GEMM
constexpr int kMfmaMinM = 3;        // from this many activation rows on, llvq_matmul uses the MFMA kernel
// THREADS x TOKTILES: more token tiles per pass over the weights need more accumulator registers, i.e. fewer
// waves per SIMD.  Used as 1024 threads x 2 tiles (64 tokens per pass) for 3 <= M <= 64; larger M takes prefill_kernel.
// MULTI: the row tiles are those of up to four matrices that share x, one matrix after the other (`items`).
template <int FMT, typename X2, int THREADS, int kTokTiles, bool MULTI = false>
__global__ void __launch_bounds__(THREADS) mfma_kernel(const unsigned char* __restrict__ blob, TableLayout lay,
                                                        const void* __restrict__ idx_in, const uint16_t* __restrict__ gain_in,
                                                        const uint32_t* __restrict__ x, int M, int N_in, int KB,
                                                        Code cd, uint32_t kranges, MatItems items, float* __restrict__ y_in) {
    constexpr int kWavesHere = THREADS / 64;
    load_tables<THREADS>(blob, lay.blob_bytes);
    const TabPtrs T = llvq::make_tab_ptrs(lds_origin(), blob, lay);
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 31, half = lane >> 5;
    // The waves of a workgroup own neighbouring row tiles and walk the same block pairs (the range blockIdx.y of the
    // kranges ranges a row is cut into), so they ask for the same activation lines at about the same time and the
    // vector cache serves fifteen of sixteen requests.  (Dealing the steps to the waves as one contiguous sequence made
    // every wave fetch its own activations from L2: at M = 64 that traffic, not the decode, set the time.)
    const uint32_t spt = ((uint32_t)KB + 1) / 2;                         // steps (block pairs) per row tile
    const uint32_t n_rt = MULTI ? (uint32_t)items.tile_end[kMaxItems - 1] : ((uint32_t)N_in + 31) / 32;
    const uint32_t rt_all = (uint32_t)blockIdx.x * kWavesHere + wave;
    const uint32_t s0 = (uint32_t)(((uint64_t)spt * blockIdx.y) / kranges);
    const uint32_t s1 = (uint32_t)(((uint64_t)spt * (blockIdx.y + 1)) / kranges);
    if (rt_all >= n_rt || s0 >= s1) return;
    // the matrix this wave's row tile belongs to (wave-uniform) and the tile's number inside it
    const void* idx = idx_in;
    const uint16_t* gain = gain_in;
    float* y = y_in;
    int N = N_in;
    uint32_t rt = rt_all;
    if constexpr (MULTI) {
        int it = 0, first_tile = 0, first_row = 0;
#pragma unroll
        for (int i = 0; i + 1 < kMaxItems; i++) {
            if (rt_all >= (uint32_t)items.tile_end[i]) { it = i + 1; first_tile = items.tile_end[i]; first_row = items.row_end[i]; }
        }
        idx = items.idx[it]; gain = items.gain[it]; y = items.y[it];
        N = items.row_end[it] - first_row;
        rt = rt_all - (uint32_t)first_tile;
    }
    const size_t xpitch = (size_t)KB * 12;                              // dwords per activation row

    for (int m0 = 0; m0 < M; m0 += 32 * kTokTiles) {
        const int ntile = min(kTokTiles, (M - m0 + 31) / 32);
        float16_t acc[kTokTiles];
#pragma unroll
        for (int t = 0; t < kTokTiles; t++) {
#pragma unroll
            for (int v = 0; v < 16; v++) acc[t][v] = 0.0f;
        }
        // activation rows of this lane as dword offsets, one per token tile (clamped: out-of-range tokens are never stored)
        uint32_t xoff[kTokTiles];
#pragma unroll
        for (int t = 0; t < kTokTiles; t++) xoff[t] = (uint32_t)min(M - 1, m0 + 32 * t + col) * (uint32_t)xpitch;

        // adds the accumulated tiles of weight-row tile `tile` to y and clears them
        auto flush = [&](uint32_t tile) {
            const int wrow = (int)tile * 32 + col;
            if (wrow < N) {
                // element offset of (token m0 + 4*half, weight row wrow); M*N < 2^32 is checked by the caller.
                // Register v of tile t belongs to token m0 + 32 t + 8 (v/4) + 4 half + v%4.
                uint32_t ot = (uint32_t)(m0 + 4 * half) * (uint32_t)N + (uint32_t)wrow;
                const uint32_t un = (uint32_t)N;
#pragma unroll
                for (int t = 0; t < kTokTiles; t++) {
                    if (t < ntile) {
                        const int tok0 = m0 + 32 * t + 4 * half;
                        const bool full = m0 + 32 * t + 32 <= M;
                        uint32_t og = ot;
#pragma unroll
                        for (int q = 0; q < 4; q++) {
                            uint32_t ov = og;
#pragma unroll
                            for (int r = 0; r < 4; r++) {
                                if (full || tok0 + 8 * q + r < M) atomicAdd(y + ov, acc[t][4 * q + r]);
                                ov += un;
                            }
                            og += 8 * un;
                        }
                    }
                    ot += 32 * un;
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
#pragma unroll
            for (int t = 0; t < kTokTiles; t++) {
#pragma unroll
                for (int v = 0; v < 16; v++) acc[t][v] = 0.0f;
            }
        };

        // the word and gain of the next step are requested before this step's block is decoded
        const int row = (int)rt * 32 + col;
        auto request = [&](uint32_t st, RawBlock& r) {
            const size_t k = (size_t)min(row, N - 1) * KB + min(2 * st + half, (uint32_t)KB - 1);
            load_raw<FMT>(idx, gain, cd.gain_array(), k, r);
        };
        RawBlock raw, raw_next;
        request(s0, raw);
        for (uint32_t st = s0; st < s1; st++, raw = raw_next) {
            request(min(st + 1, s1 - 1), raw_next);
            const uint32_t b = 2 * st + half;
            // this step's activation operands are requested before the block is decoded (each lane reads 48 bytes of a
            // different token row: the slowest loads of the step)
            const uint32_t bx = min(b, (uint32_t)KB - 1) * 12;
            u32x4 xa[kTokTiles <= 2 ? kTokTiles : 1][3];
            if constexpr (kTokTiles <= 2) {
#pragma unroll
                for (int t = 0; t < kTokTiles; t++) {
                    if (t < ntile) {
                        const u32x4* xp = reinterpret_cast<const u32x4*>(x + (size_t)(xoff[t] + bx));
                        xa[t][0] = xp[0]; xa[t][1] = xp[1]; xa[t][2] = xp[2];
                    }
                }
            }
            const bool live = row < N && b < (uint32_t)KB;
            uint64_t I;
            uint16_t gb;
            finish_block<FMT>(raw, cd, I, gb);
            const float g = __half2float(__ushort_as_half(gb));
            const bool ok = live && I < T.npoints;
            if (!ok) I = 0;
            uint32_t w[4];
            const llvq::BlockInfo bi = llvq::decode_block(T, I, w);
            const float scale = ok ? g * bi.rnorm : 0.0f;
            constexpr int kTerms = Mma<X2>::kTerms;
            uint32_t wt[kTerms][12];
#pragma unroll
            for (int c = 0; c < 4; c++) {
                uint32_t fe, fo, o[kTerms];
                chunk_fp8(w[c], bi.vt8_lo, bi.vt8_hi, fe, fo);
                Mma<X2>::weights(fe, false, scale, o);
#pragma unroll
                for (int r = 0; r < kTerms; r++) wt[r][3 * c + 0] = o[r];
                Mma<X2>::weights(fo, false, scale, o);
#pragma unroll
                for (int r = 0; r < kTerms; r++) wt[r][3 * c + 1] = o[r];
                Mma<X2>::weights(fe, true, scale, o);
#pragma unroll
                for (int r = 0; r < kTerms; r++) wt[r][3 * c + 2] = o[r];
            }
#pragma unroll
            for (int t = 0; t < kTokTiles; t++) {
                if (t < ntile) {
                    if constexpr (kTokTiles <= 2) {
#pragma unroll
                        for (int j = 0; j < 3; j++) {
#pragma unroll
                            for (int r = 0; r < kTerms; r++)
                                acc[t] = Mma<X2>::mma(xa[t][j], u32x4{wt[r][4 * j], wt[r][4 * j + 1], wt[r][4 * j + 2], wt[r][4 * j + 3]}, acc[t]);
                        }
                    } else {
                        const u32x4* xp = reinterpret_cast<const u32x4*>(x + (size_t)(xoff[t] + bx));
                        const u32x4 xl[3] = {xp[0], xp[1], xp[2]};
#pragma unroll
                        for (int j = 0; j < 3; j++) {
#pragma unroll
                            for (int r = 0; r < kTerms; r++)
                                acc[t] = Mma<X2>::mma(xl[j], u32x4{wt[r][4 * j], wt[r][4 * j + 1], wt[r][4 * j + 2], wt[r][4 * j + 3]}, acc[t]);
                        }
                    }
                }
                if (kTokTiles > 2 && (t & 1)) __builtin_amdgcn_sched_barrier(0);   // keep only two tiles of activations in flight
            }
        }
        flush(rt);
    }
}

// ---- llvq_matmul, batched decode (3 <= M <= 32): a row tile belongs to one workgroup, K is reduced inside it ------
// A step = 16 weight rows x 4 neighbouring blocks of 24 input channels: lane l decodes block 4 s + l / 16 of row l % 16
// of the tile.  The decoded block, scaled by gain / sqrt(16 m) and rounded to the activation type, is what
// v_mfma_f32_16x16x32 expects from that lane as its B operand (k = 8 (l / 16) .. + 7 of column l % 16); the A operand
// (16 tokens x the same channels) comes from global memory; three MFMAs consume the 24 channels of the four blocks.
// A workgroup owns whole row tiles, so every channel of a row is seen inside it: the steps of up to kTilePassSlots
// tiles (a pass) are dealt round-robin to the sixteen waves, each wave keeps the running 16 x 16 tile in its matrix-core
// accumulators and, when it leaves a row tile, stores it into a slot of its own in LDS; after a barrier the slots of a
// tile are added in a fixed order and y is written once with plain stores.  Nothing is cleared beforehand, nothing is
// combined with atomics, and the result does not depend on timing.  Only the small tables are kept in LDS (the Golay
// words and inner-word planes are read from global memory), which leaves 64 KB for the slots.
// bf16 activations: the scaled weight is split into two bf16 terms (its bf16 rounding and the bf16 rounding of the
// remainder, together 16 significant bits), six MFMAs per step: a single bf16 term (8 bits) would put 2^-9 per weight
// into y.
constexpr int kTileRows = 16;
constexpr int kTilePassSlots = 4;               // 16 x 16 tiles a wave can park in LDS per pass: 4 row tiles x 1 token tile or 2 x 2
typedef float float4_t __attribute__((ext_vector_type(4)));

template <typename X2> struct Mma16;
template <> struct Mma16<half2_t> {
    // c += A B over 32 values of k: lane l holds k = 8 (l / 16) .. + 7 of row (A) or column (B) l % 16
    static __device__ __forceinline__ float4_t mma(u32x4 a, u32x4 b, float4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, a), __builtin_bit_cast(half8_t, b), c, 0, 0, 0);
    }
};
template <> struct Mma16<bf16x2_t> {
    static __device__ __forceinline__ float4_t mma(u32x4 a, u32x4 b, float4_t c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
};

// TT: token tiles of 16 (M <= 16 TT); MULTI: the row tiles are those of up to four matrices that share x (`items`).
template <int FMT, typename X2, int TT, bool MULTI = false>
__global__ void __launch_bounds__(kThreads) tile_kernel(const unsigned char* __restrict__ blob, TableLayout lay,
                                                        const void* __restrict__ idx_in, const uint16_t* __restrict__ gain_in,
                                                        const uint32_t* __restrict__ x, int M, int N_in, int KB, Code cd,
                                                        int n_tiles, int tiles_per_wg, MatItems items, float* __restrict__ y_in) {
    constexpr int kWaves = kThreads / 64;
    constexpr int kPassTiles = kTilePassSlots / TT;                      // row tiles per pass
    constexpr int kTerms = Mma<X2>::kTerms;
    load_tables(blob, llvq::kOffInner);          // the small tables and the Golay words; the inner-word planes stay in global memory
    const TabPtrs T = llvq::make_tab_ptrs(lds_origin(), blob, lay);
    float* slots = reinterpret_cast<float*>(g_lds + llvq::kOffInner);      // [kWaves][kPassTiles][TT][256]
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = lane & 15, kgrp = lane >> 4;
    const uint32_t S = ((uint32_t)KB + 3) / 4;                            // steps per row tile
    const size_t xpitch = (size_t)KB * 12;                              // dwords per activation row
    const int wg_t0 = blockIdx.x * tiles_per_wg, wg_t1 = min(n_tiles, wg_t0 + tiles_per_wg);
    // The activation tile of a step (16 tokens x 96 channels per token tile) is fetched with four neighbouring lanes on
    // one token row (lane = 4 token + group: 16 rows per load instead of 64 distinct lines with the MFMA's own lane
    // order, which made the vector memory pipe the limit of this kernel) and turned into the MFMA's order through LDS.
    // The staging buffer is the slot the wave will park the current row tile in: until then it is free.  Unit (token t,
    // group g) of 16 bytes sits at g * 16 + (t + 2 g) % 16, which spreads a store over all banks.
    const int ld_tok = lane >> 2, ld_grp = lane & 3;
    uint32_t xoff[TT];                                   // row of the token this lane FETCHES, as a dword offset (clamped)
#pragma unroll
    for (int t = 0; t < TT; t++) xoff[t] = (uint32_t)min(M - 1, 16 * t + ld_tok) * (uint32_t)xpitch;
    const uint32_t st_unit = (uint32_t)(ld_grp * 16 + ((ld_tok + 2 * ld_grp) & 15)) * 4;      // in floats
    const uint32_t rd_unit = (uint32_t)(kgrp * 16 + ((col + 2 * kgrp) & 15)) * 4;

    // the matrix a row tile belongs to and the tile's first row inside it (wave-uniform)
    struct Mat { const void* idx; const uint16_t* gain; float* y; int N, row0; };
    auto mat_of = [&](int tile) {
        Mat m = {idx_in, gain_in, y_in, N_in, tile * kTileRows};
        if constexpr (MULTI) {
            int it = 0, first_tile = 0, first_row = 0;
#pragma unroll
            for (int i = 0; i + 1 < kMaxItems; i++) {
                if (tile >= items.tile16_end[i]) { it = i + 1; first_tile = items.tile16_end[i]; first_row = items.row_end[i]; }
            }
            m.idx = items.idx[it]; m.gain = items.gain[it]; m.y = items.y[it];
            m.N = items.row_end[it] - first_row;
            m.row0 = (tile - first_tile) * kTileRows;
        }
        return m;
    };

    for (int pt0 = wg_t0; pt0 < wg_t1; pt0 += kPassTiles) {
        const int np = min(kPassTiles, wg_t1 - pt0);
        const uint32_t nsteps = (uint32_t)np * S;
        // this wave's steps: e = wave, wave + 16, ...; step e is step e % S of pass tile e / S
        uint32_t e = (uint32_t)wave, tl = e / S, st = e - tl * S;
        float4_t acc[TT];
#pragma unroll
        for (int t = 0; t < TT; t++) acc[t] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};

        struct Blk { RawBlock raw; bool live; };
        auto fetch_blk = [&](uint32_t tile_local, uint32_t step, Blk& q) {
            const Mat m = mat_of(pt0 + (int)tile_local);
            const int row = m.row0 + col;
            const uint32_t b = 4 * step + (uint32_t)kgrp;
            q.live = row < m.N && b < (uint32_t)KB;
            const size_t k = (size_t)min(row, m.N - 1) * KB + min(b, (uint32_t)KB - 1);
            load_raw<FMT>(m.idx, m.gain, cd.gain_array(), k, q.raw);
        };
        auto front_of = [&](const Blk& q, bool& ok, uint16_t& gb) {
            uint64_t I;
            finish_block<FMT>(q.raw, cd, I, gb);
            ok = q.live && I < T.npoints;
            return llvq::decode_front<true, false, true>(T, llvq::find_class(T, ok ? I : 0));
        };
        Blk cur_blk, nxt_blk;
        llvq::Front F, Fn;
        bool ok_cur = false, ok_nxt = false;
        uint16_t g_cur = 0, g_nxt = 0;
        if (e < nsteps) {
            fetch_blk(tl, st, cur_blk);
            F = front_of(cur_blk, ok_cur, g_cur);
        }
        // one step; kMore: another step of this wave follows in the pass (two copies of the code, so that each is
        // straight-line with respect to its memory operations, as in matmul_kernel)
        auto step = [&](auto more_tag, uint32_t tl_n, uint32_t st_n) {
            constexpr bool kMore = decltype(more_tag)::value;
            if constexpr (kMore) fetch_blk(tl_n, st_n, nxt_blk);
            const uint32_t bx = min(4 * st + (uint32_t)ld_grp, (uint32_t)KB - 1) * 12;
            u32x4 xl[TT][3];
#pragma unroll
            for (int t = 0; t < TT; t++) {
                const u32x4* xp = reinterpret_cast<const u32x4*>(x + (size_t)(xoff[t] + bx));
                xl[t][0] = xp[0]; xl[t][1] = xp[1]; xl[t][2] = xp[2];
            }
            uint32_t w[4];
            const llvq::BlockInfo bi = llvq::decode_back(T, F, w);
            const float scale = ok_cur ? __half2float(__ushort_as_half(g_cur)) * bi.rnorm : 0.0f;
            uint32_t wt[kTerms][12];
#pragma unroll
            for (int c = 0; c < 4; c++) {
                uint32_t fe, fo, o[kTerms];
                chunk_fp8(w[c], bi.vt8_lo, bi.vt8_hi, fe, fo);
                Mma<X2>::weights(fe, false, scale, o);
#pragma unroll
                for (int r = 0; r < kTerms; r++) wt[r][3 * c + 0] = o[r];
                Mma<X2>::weights(fo, false, scale, o);
#pragma unroll
                for (int r = 0; r < kTerms; r++) wt[r][3 * c + 1] = o[r];
                Mma<X2>::weights(fe, true, scale, o);
#pragma unroll
                for (int r = 0; r < kTerms; r++) wt[r][3 * c + 2] = o[r];
            }
            if constexpr (kMore) Fn = front_of(nxt_blk, ok_nxt, g_nxt);
            // one channel group j at a time through the wave's buffer: LDS operations of a wave execute in order, so
            // the store of group j + 1 cannot overtake the loads of group j
            float* stage = slots + ((size_t)(wave * kPassTiles + (int)tl) * TT) * 256;
#pragma unroll
            for (int j = 0; j < 3; j++) {
                u32x4 xa[TT];
#pragma unroll
                for (int t = 0; t < TT; t++) *reinterpret_cast<u32x4*>(stage + t * 256 + st_unit) = xl[t][j];
#pragma unroll
                for (int t = 0; t < TT; t++) xa[t] = *reinterpret_cast<const u32x4*>(stage + t * 256 + rd_unit);
#pragma unroll
                for (int r = 0; r < kTerms; r++) {
                    const u32x4 bw = {wt[r][4 * j], wt[r][4 * j + 1], wt[r][4 * j + 2], wt[r][4 * j + 3]};
#pragma unroll
                    for (int t = 0; t < TT; t++) acc[t] = Mma16<X2>::mma(xa[t], bw, acc[t]);
                }
            }
            // leaving this row tile (or the pass): park the accumulated tile in this wave's slot and start from zero
            if (!kMore || tl_n != tl) {
                float* dst = stage + lane * 4;
#pragma unroll
                for (int t = 0; t < TT; t++) {
                    *reinterpret_cast<float4_t*>(dst + t * 256) = acc[t];
                    acc[t] = float4_t{0.0f, 0.0f, 0.0f, 0.0f};
                }
            }
        };
        while (e < nsteps) {
            // the wave's next step (wave-uniform scalars)
            const uint32_t e_n = e + kWaves;
            uint32_t tl_n = tl, st_n = st + kWaves;
            while (st_n >= S) { st_n -= S; tl_n++; }
            if (e_n < nsteps) {
                step(std::true_type{}, tl_n, st_n);
                F = Fn; ok_cur = ok_nxt; g_cur = g_nxt;
            } else {
                step(std::false_type{}, tl_n, st_n);
            }
            e = e_n; tl = tl_n; st = st_n;
        }
        __syncthreads();
        // tile tau of the pass got a partial tile from the waves (tau S + i) % 16, i < min(S, 16): added in that order.
        // Thread r of a group of 256 writes token r / 16, weight row r % 16 (neighbouring threads, neighbouring addresses).
        for (int u = threadIdx.x; u < np * TT * 256; u += kThreads) {
            const int tau = u / (TT * 256), rem = u - tau * (TT * 256), t = rem >> 8, r = rem & 255;
            const int tok_l = r >> 4, c = r & 15;
            const int src = (((tok_l >> 2) << 4) + c) * 4 + (tok_l & 3);        // lane (4 (tok / 4) ... ) register tok % 4
            const uint32_t first = (uint32_t)tau * S, cnt = min(S, (uint32_t)kWaves);
            float sum = 0.0f;
            for (uint32_t i = 0; i < cnt; i++) {
                const int wv = (int)((first + i) & (kWaves - 1));
                sum += slots[((size_t)(wv * kPassTiles + tau) * TT + t) * 256 + src];
            }
            const Mat m = mat_of(pt0 + tau);
            const int row = m.row0 + c, tok = 16 * t + tok_l;
            if (row < m.N && tok < M) m.y[(size_t)tok * m.N + row] = sum;
        }
        __syncthreads();
    }
}

// ---- llvq_matmul, prefill kernel for large M: activations shared through LDS, no split along K -----------------
// A workgroup of eight waves owns a strip of 256 weight rows (wave w: rows 32 w .. 32 w + 31 of the strip) and a pass of
// 256 tokens, and walks all block pairs of the rows.  Per step the activation tile of the step (256 tokens x 48 channels)
// is staged once in LDS and read by all eight waves as MFMA A operands, so it is fetched from L2 once per workgroup
// instead of once per wave; the decoded blocks are the B operands straight from the decoder's registers as in
// mfma_kernel.  A workgroup sees every channel of its rows, so y is written once with plain stores: no clearing, no
// atomics, results reproducible.  Only the small tables are kept in LDS (the Golay words and inner-word planes are
// read from global memory), which leaves room for two activation buffers.
// Shape used: 8 waves x 8 token tiles (strips of 256 rows, passes of 256 tokens; 128 accumulator registers, two waves per
// SIMD).  16 waves x 2 token tiles was measured for M <= 64 and lost to mfma_kernel (75.6 against 68 us on 14336 x 4104).
constexpr uint32_t kATokenPitch = 112;                 // bytes per token in the staged tile: 96 of data, padded so that rows stay 16-byte
                                                       // aligned (128-bit LDS accesses) and eight consecutive tokens cover all banks

template <int FMT, typename X2, int WAVES, int TT>
__global__ void __launch_bounds__(64 * WAVES) prefill_kernel(const unsigned char* __restrict__ blob, TableLayout lay,
                                                                   const void* __restrict__ idx, const uint16_t* __restrict__ gain,
                                                                   const uint32_t* __restrict__ x, int M, int N, int KB, Code cd,
                                                                   int ksplit, float* __restrict__ y) {
    constexpr int kPrefillThreads = 64 * WAVES, kPrefillTokens = 32 * TT, kPrefillRows = 32 * WAVES;
    constexpr uint32_t kABufBytes = kPrefillTokens * kATokenPitch;
    load_tables<kPrefillThreads>(blob, lay.lds_bytes);
    const TabPtrs T = llvq::make_tab_ptrs(lds_origin(), blob, lay);
    unsigned char* abuf = g_lds + lay.lds_bytes;                         // two buffers of kABufBytes
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 31, half = lane >> 5;
    // steps (block pairs) of a row; with ksplit > 1 the workgroups of blockIdx.z share them and add their parts to y
    const uint32_t spt_all = ((uint32_t)KB + 1) / 2;
    const uint32_t st_first = (uint32_t)(((uint64_t)spt_all * blockIdx.z) / (uint32_t)ksplit);
    const uint32_t spt = (uint32_t)(((uint64_t)spt_all * (blockIdx.z + 1)) / (uint32_t)ksplit);      // one past this workgroup's last step
    const int m0 = (int)blockIdx.y * kPrefillTokens;
    const int wrow = (int)blockIdx.x * kPrefillRows + wave * 32 + col;    // weight row of this lane
    const size_t xpitch = (size_t)KB * 12;                              // dwords per activation row

    // staging role of this thread: token (thread / 2) of the pass, block (thread % 2) of the pair
    const bool s_on = (int)(threadIdx.x >> 1) < kPrefillTokens;          // with more threads than staging work the rest sit out
    const int s_tok = min(M - 1, m0 + min((int)(threadIdx.x >> 1), kPrefillTokens - 1));
    const uint32_t s_part = threadIdx.x & 1u;
    const uint32_t* s_src = x + (size_t)s_tok * xpitch;
    unsigned char* s_dst = abuf + (uint32_t)min((int)(threadIdx.x >> 1), kPrefillTokens - 1) * kATokenPitch + s_part * 48u;
    auto stage_load = [&](uint32_t st, uint4 (&v)[3]) {
        const uint32_t b = min(2 * st + s_part, (uint32_t)KB - 1);       // past the last block: any valid data, its weights are zero
        const uint4* p = reinterpret_cast<const uint4*>(s_src + (size_t)b * 12);
        v[0] = p[0]; v[1] = p[1]; v[2] = p[2];
    };
    auto stage_store = [&](uint32_t buf, const uint4 (&v)[3]) {
        if (!s_on) return;
        uint4* d = reinterpret_cast<uint4*>(s_dst + buf * kABufBytes);
        d[0] = v[0]; d[1] = v[1]; d[2] = v[2];
    };

    float16_t acc[TT];
#pragma unroll
    for (int t = 0; t < TT; t++) {
#pragma unroll
        for (int v = 0; v < 16; v++) acc[t][v] = 0.0f;
    }
    // Software pipeline over the steps: the word of the next step is requested first, then this step's block is placed,
    // then the next step's class search and digit extraction run (their reads from global memory are in flight during
    // the matrix products), then the products of this step, then the next activation tile is put into LDS.
    struct Blk { RawBlock raw; bool live; };
    auto fetch_blk = [&](uint32_t st, Blk& q) {
        const uint32_t b = 2 * st + half;
        q.live = wrow < N && b < (uint32_t)KB;
        const size_t k = (size_t)min(wrow, N - 1) * KB + min(b, (uint32_t)KB - 1);
        load_raw<FMT>(idx, gain, cd.gain_array(), k, q.raw);
    };
    auto front_of = [&](const Blk& q, bool& ok, uint16_t& gb) {
        uint64_t I;
        finish_block<FMT>(q.raw, cd, I, gb);
        ok = q.live && I < T.npoints;
        return llvq::decode_front<true>(T, llvq::find_class(T, ok ? I : 0));
    };
    {
        uint4 v[3];
        stage_load(st_first, v);
        stage_store(st_first & 1u, v);
    }
    Blk cur_blk, nxt_blk;
    fetch_blk(st_first, cur_blk);
    bool ok_cur = false, ok_nxt = false;
    uint16_t g_cur = 0, g_nxt = 0;
    llvq::Front F = front_of(cur_blk, ok_cur, g_cur), Fn;
    __syncthreads();
    for (uint32_t st = st_first; st < spt; st++) {
        const uint32_t st_next = st + 1 < spt ? st + 1 : st;            // past the end the last step is requested again
        uint4 nextv[3];
        stage_load(st_next, nextv);
        fetch_blk(st_next, nxt_blk);
        uint32_t w[4];
        const llvq::BlockInfo bi = llvq::decode_back(T, F, w);
        const float scale = ok_cur ? __half2float(__ushort_as_half(g_cur)) * bi.rnorm : 0.0f;
        constexpr int kTerms = Mma<X2>::kTerms;
        uint32_t wt[kTerms][12];
#pragma unroll
        for (int c = 0; c < 4; c++) {
            uint32_t fe, fo, o[kTerms];
            chunk_fp8(w[c], bi.vt8_lo, bi.vt8_hi, fe, fo);
            Mma<X2>::weights(fe, false, scale, o);
#pragma unroll
            for (int r = 0; r < kTerms; r++) wt[r][3 * c + 0] = o[r];
            Mma<X2>::weights(fo, false, scale, o);
#pragma unroll
            for (int r = 0; r < kTerms; r++) wt[r][3 * c + 1] = o[r];
            Mma<X2>::weights(fe, true, scale, o);
#pragma unroll
            for (int r = 0; r < kTerms; r++) wt[r][3 * c + 2] = o[r];
        }
        Fn = front_of(nxt_blk, ok_nxt, g_nxt);
        // A operands from the staged tile: token 32 t + col, the lane half's block (48 bytes), k group j
        const unsigned char* arow = abuf + (st & 1u) * kABufBytes + (uint32_t)col * kATokenPitch + (uint32_t)half * 48u;
        // k group outermost: consecutive MFMAs go to different accumulators and do not wait for each other
#pragma unroll
        for (int j = 0; j < 3; j++) {
#pragma unroll
            for (int t = 0; t < TT; t++) {
                const u32x4 a = *reinterpret_cast<const u32x4*>(arow + (uint32_t)t * 32u * kATokenPitch + (uint32_t)j * 16u);
#pragma unroll
                for (int r = 0; r < kTerms; r++)
                    acc[t] = Mma<X2>::mma(a, u32x4{wt[r][4 * j], wt[r][4 * j + 1], wt[r][4 * j + 2], wt[r][4 * j + 3]}, acc[t]);
            }
        }
        stage_store((st + 1) & 1u, nextv);
        F = Fn;
        ok_cur = ok_nxt;
        g_cur = g_nxt;
        __syncthreads();
    }
    // y[token][wrow]: register v of tile t belongs to token m0 + 32 t + 8 (v / 4) + 4 half + v % 4
    if (wrow < N) {
#pragma unroll
        for (int t = 0; t < TT; t++) {
#pragma unroll
            for (int v = 0; v < 16; v++) {
                const int tok = m0 + 32 * t + 8 * (v / 4) + 4 * half + (v % 4);
                if (tok < M) {
                    if (ksplit == 1) y[(size_t)tok * N + wrow] = acc[t][v];
                    else atomicAdd(y + (size_t)tok * N + wrow, acc[t][v]);
                }
            }
        }
    }
}

// ---- llvq_matmul, prefill kernel for M >= kPanelMinM: decoded weights shared through LDS ------------------------
// The index decode costs the vector ALUs and the LDS gather pipe as much per block as 500 tokens cost the matrix cores,
// so a block should be decoded once per as many tokens as the accumulators can hold.  A workgroup of eight waves owns a
// panel of 128 weight rows x 512 tokens: wave w keeps ALL 128 rows x tokens 64 w .. 64 w + 63 (eight 32 x 32 tiles, 128
// accumulator registers), i.e. the waves split the tokens, not the rows.  Per step (a block pair = 48 channels) the four
// 32-row tiles are decoded by four of the waves (the two halves of the workgroup take turns, so a SIMD always hosts
// one decoding and one multiplying wave) and written to LDS as ready-made MFMA B operands; every wave reads the 12 KB
// of the step's weights from there and the A operands of its own 64 tokens from a private region of LDS that it fills
// itself with direct global-to-LDS loads (six lanes fetch the 96 bytes of a token row: few cache lines per load).  The
// region needs no barrier: the wave reads a step's operands into registers once its own loads have landed, and asks
// for the next step's rows after that.  One barrier per step publishes the weights.  Against prefill_kernel a step
// moves 18 KB instead of 24 KB per wave through LDS for twice the tokens per decoded block.
// The decode of a step is spread over two steps of its wave: class search and digits while the wave's half is off
// duty, placement, signs and scaling in the step before the weights are needed.
constexpr int kPanelRows = 128, kPanelTokens = 512, kPanelWaves = 8;
constexpr int kPanelMinM = 384;

// MULTI: the strips are those of up to four matrices that share x, one matrix after the other (`items`).
template <int FMT, typename X2, bool MULTI = false>
__global__ void __launch_bounds__(64 * kPanelWaves) panel_kernel(const unsigned char* __restrict__ blob, TableLayout lay,
                                                                   const void* __restrict__ idx_in, const uint16_t* __restrict__ gain_in,
                                                                   const uint32_t* __restrict__ x, int M, int N_in, int KB, Code cd,
                                                                   int ksplit, MatItems items, float* __restrict__ y_in) {
    // the matrix this workgroup's strip belongs to and the strip's first row inside it (wave-uniform)
    const void* idx = idx_in;
    const uint16_t* gain = gain_in;
    float* y = y_in;
    int N = N_in, strip = (int)blockIdx.x;
    if constexpr (MULTI) {
        int it = 0, first_strip = 0, first_row = 0;
#pragma unroll
        for (int i = 0; i + 1 < kMaxItems; i++) {
            if (strip >= items.strip_end[i]) { it = i + 1; first_strip = items.strip_end[i]; first_row = items.row_end[i]; }
        }
        idx = items.idx[it]; gain = items.gain[it]; y = items.y[it];
        N = items.row_end[it] - first_row;
        strip -= first_strip;
    }
    constexpr int kTerms = Mma<X2>::kTerms;
    constexpr int kBBufs = kTerms == 1 ? 2 : 1;                      // two-term weights: one buffer, a second barrier per step
    constexpr uint32_t kBBytes = 4 * 3 * 1024 * kTerms;              // [term][row tile][k group][lane] x 16 bytes
    constexpr uint32_t kARegion = 7 * 1024;                          // one wave's 64 token rows: seven staging instructions x 1 KB
    load_tables<64 * kPanelWaves>(blob, lay.lds_bytes);
    const TabPtrs T = llvq::make_tab_ptrs(lds_origin(), blob, lay);
    unsigned char* bbuf = g_lds + lay.lds_bytes;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    unsigned char* abuf = bbuf + kBBufs * kBBytes + (uint32_t)wave * kARegion;
    const int col = lane & 31, half = lane >> 5;
    const uint32_t spt_all = ((uint32_t)KB + 1) / 2;
    const uint32_t st_first = (uint32_t)(((uint64_t)spt_all * blockIdx.z) / (uint32_t)ksplit);
    const uint32_t st_end = (uint32_t)(((uint64_t)spt_all * (blockIdx.z + 1)) / (uint32_t)ksplit);
    const int row0 = strip * kPanelRows;
    const int m0 = (int)blockIdx.y * kPanelTokens + wave * 64;        // first token of this wave
    const uint32_t xpitch = (uint32_t)KB * 12u;                       // dwords per activation row

    // decoding role: row tile (wave % 4), steps of parity (wave / 4) counted from st_first
    const int drt = wave & 3;
    const uint32_t dpar = (uint32_t)wave >> 2;
    const int wrow = row0 + 32 * drt + col;
    struct Blk { RawBlock raw; bool live; };
    auto fetch_blk = [&](uint32_t st, Blk& q) {
        const uint32_t b = 2 * st + (uint32_t)half;
        q.live = wrow < N && b < (uint32_t)KB;
        const size_t k = (size_t)min(wrow, N - 1) * KB + min(b, (uint32_t)KB - 1);
        load_raw<FMT>(idx, gain, cd.gain_array(), k, q.raw);
    };
    // first part of a block's decode: class, digits and the subset U (everything that does not need the Golay word and
    // the inner-word planes, whose reads from global memory are left in flight)
    auto front_of = [&](const Blk& q, bool& ok, uint16_t& gb, uint32_t& U) {
        uint64_t I;
        finish_block<FMT>(q.raw, cd, I, gb);
        ok = q.live && I < T.npoints;
        const llvq::Front f = llvq::decode_front<true>(T, llvq::find_class(T, ok ? I : 0));
        U = llvq::decode_subset(T, f);
        return f;
    };
    // second part: placement, signs, scaling; the weights go to LDS as B operands of `buf`
    auto back_to_lds = [&](const llvq::Front& F, uint32_t U, bool ok, uint16_t gb, uint32_t buf) {
        uint32_t w[4];
        const llvq::BlockInfo bi = llvq::decode_place(T, F, U, w);
        const float scale = ok ? __half2float(__ushort_as_half(gb)) * bi.rnorm : 0.0f;
        uint32_t wt[kTerms][12];
#pragma unroll
        for (int c = 0; c < 4; c++) {
            uint32_t fe, fo, o[kTerms];
            chunk_fp8(w[c], bi.vt8_lo, bi.vt8_hi, fe, fo);
            Mma<X2>::weights(fe, false, scale, o);
#pragma unroll
            for (int r = 0; r < kTerms; r++) wt[r][3 * c + 0] = o[r];
            Mma<X2>::weights(fo, false, scale, o);
#pragma unroll
            for (int r = 0; r < kTerms; r++) wt[r][3 * c + 1] = o[r];
            Mma<X2>::weights(fe, true, scale, o);
#pragma unroll
            for (int r = 0; r < kTerms; r++) wt[r][3 * c + 2] = o[r];
        }
        unsigned char* dst = bbuf + buf * kBBytes + (uint32_t)(drt * 3) * 1024u + (uint32_t)lane * 16u;
#pragma unroll
        for (int r = 0; r < kTerms; r++) {
#pragma unroll
            for (int j = 0; j < 3; j++)
                *reinterpret_cast<u32x4*>(dst + (uint32_t)(r * 12 + j) * 1024u) = u32x4{wt[r][4 * j], wt[r][4 * j + 1], wt[r][4 * j + 2], wt[r][4 * j + 3]};
        }
    };

    // Staging of this wave's activation rows, global memory -> LDS without passing registers: one wave instruction moves
    // 64 x 16 bytes to 1 KB of consecutive LDS addresses.  Lane 6 k + q of instruction i fetches piece q (channels
    // 8 (q % 3) .. + 7 of block 2 st + q / 3) of token 10 i + k, so the 96 bytes of a token row are fetched by six
    // neighbouring lanes (few cache lines per instruction) and land at i * 1024 + k * 96; seven instructions cover the 64
    // tokens (lanes 60..63 and the tail of the last instruction fetch copies that nobody reads).
    const int s_tok = lane / 6, s_q = lane - 6 * s_tok;
    // byte offsets of this lane's seven token rows in x (M * KB * 48 < 2^32, checked by the host)
    uint32_t s_row[7];
#pragma unroll
    for (int i = 0; i < 7; i++) s_row[i] = (uint32_t)min(M - 1, m0 + min(10 * i + s_tok, 63)) * (xpitch * 4u) + (uint32_t)(s_q % 3) * 16u;
    auto stage_dma = [&](uint32_t st) {
        const uint32_t b = min(2 * st + (uint32_t)(s_q / 3), (uint32_t)KB - 1);      // past the last block: any valid data, its weights are zero
        const uint32_t boff = b * 48u;
#pragma unroll
        for (int i = 0; i < 7; i++)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(reinterpret_cast<const unsigned char*>(x) + (s_row[i] + boff)),
                                             (__attribute__((address_space(3))) void*)(abuf + i * 1024), 16, 0, 0);
    };
    // A operands of the staged step in the MFMA's order: token 32 t + col, the lane half's block, channel group j
    uint32_t a_off[2];
#pragma unroll
    for (int t = 0; t < 2; t++) a_off[t] = (uint32_t)((32 * t + col) / 10) * 1024u + (uint32_t)((32 * t + col) % 10) * 96u + (uint32_t)half * 48u;
    u32x4 a[3][2];
    auto read_a = [&]() {
#pragma unroll
        for (int j = 0; j < 3; j++) {
#pragma unroll
            for (int t = 0; t < 2; t++) a[j][t] = *reinterpret_cast<const u32x4*>(abuf + a_off[t] + (uint32_t)j * 16u);
        }
    };

    float16_t acc[4][2];
#pragma unroll
    for (int rt = 0; rt < 4; rt++) {
#pragma unroll
        for (int t = 0; t < 2; t++) {
#pragma unroll
            for (int v = 0; v < 16; v++) acc[rt][t][v] = 0.0f;
        }
    }

    // Prologue.  Relative step r = st - st_first; the half with parity r % 2 decodes step r.  Before the first step:
    // half 0 decodes step 0 completely and requests the word of step 2; half 1 does the first part of step 1.
    // Steps past the last one are replaced by the last one wherever something is requested or decoded ahead: the loop
    // then has no conditional assignments, and what is decoded in excess is never read.
    const uint32_t st_last = st_end - 1;
    Blk blk;
    llvq::Front F;
    uint32_t U = 0;
    bool ok = false;
    uint16_t gb = 0;
    fetch_blk(min(st_first + dpar, st_last), blk);
    F = front_of(blk, ok, gb, U);
    if (dpar == 0) {
        back_to_lds(F, U, ok, gb, 0);
        fetch_blk(min(st_first + 2, st_last), blk);
    }
    stage_dma(st_first);
    __builtin_amdgcn_s_waitcnt(0);              // vmcnt(0): the rows have landed
    read_a();
    __syncthreads();

    // s_waitcnt vmcnt(n): wait until at most n of this wave's loads are outstanding (they complete in order)
    auto wait_loads_but = [](auto n_tag) {
        constexpr unsigned n = decltype(n_tag)::value;
        __builtin_amdgcn_s_waitcnt((n & 15u) | (7u << 4) | (15u << 8) | ((n >> 4) << 14));
    };
    constexpr unsigned kFetchLoads = FMT == LLVQ_IDX_U24 ? 4u : 3u;      // loads of fetch_blk

    // One step.  kBack: this wave finishes the decode of step st + 1 (its half's turn); otherwise it starts that of
    // step st + 2.  The role alternates from step to step and is fixed per position in the loop below, so that every
    // value carried from one step to the next is assigned unconditionally: a load may then stay in flight across steps
    // (with an assignment under a condition the compiler copies the register where the paths join and waits for ALL
    // loads there, i.e. at the top of the next step, before the activation rows are requested).
    auto slot = [&](auto back_tag, uint32_t st) {
        constexpr bool kBack = decltype(back_tag)::value;
        const uint32_t r = st - st_first;
        const uint32_t bcur = kBBufs == 2 ? (r & 1u) : 0u, bnext = kBBufs == 2 ? ((r + 1) & 1u) : 0u;
        // the A operands of step st are in registers (read before the barrier that ended the last step), so the
        // activation rows of step st + 1 can be requested into the same region right away
        // (the decoding half asks after its decode: all eight waves asking at once right after the barrier queue at the
        // vector memory pipe, 56 KB per step, and every one of them waits for the issue of its seven loads)
        const uint32_t st_stage = min(st + 1, st_last);
        if (!(kBBufs == 2 && kBack)) stage_dma(st_stage);
        // second part of step st + 1 before the products: the other wave of this SIMD multiplies meanwhile
        if (kBBufs == 2 && kBack) {
            back_to_lds(F, U, ok, gb, bnext);
            fetch_blk(min(st + 3, st_last), blk);
            stage_dma(st_stage);
        }
        // The products of step st: B operands one channel group ahead.
        // Waves whose tokens lie past M work on copies of token M - 1 and store nothing at the end.
        {
            const unsigned char* brow = bbuf + bcur * kBBytes + (uint32_t)lane * 16u;
            // one term per weight: the operands of the next channel group are read while this one is multiplied; two
            // terms: twice the operands and twice the products per read, no room in the register file for reading ahead
            constexpr int kAhead = kTerms == 1 ? 1 : 0;
            u32x4 b[1 + kAhead][kTerms][4];
            auto load_b = [&](int j, u32x4 (&dst)[kTerms][4]) {
#pragma unroll
                for (int rr = 0; rr < kTerms; rr++) {
#pragma unroll
                    for (int rt = 0; rt < 4; rt++) dst[rr][rt] = *reinterpret_cast<const u32x4*>(brow + (uint32_t)(rr * 12 + rt * 3 + j) * 1024u);
                }
            };
            if (kAhead) load_b(0, b[0]);
#pragma unroll
            for (int j = 0; j < 3; j++) {
                if (kAhead) {
                    if (j + 1 < 3) load_b(j + 1, b[(j + 1) & kAhead]);
                    __builtin_amdgcn_sched_barrier(0);               // keep the reads ahead of the products they are not needed for
                } else {
                    load_b(j, b[0]);
                }
#pragma unroll
                for (int rt = 0; rt < 4; rt++) {
#pragma unroll
                    for (int rr = 0; rr < kTerms; rr++) {
#pragma unroll
                        for (int t = 0; t < 2; t++) acc[rt][t] = Mma<X2>::mma(a[j][t], b[j & kAhead][rr][rt], acc[rt][t]);
                    }
                }
            }
        }
        if (kBBufs == 1) {
            __syncthreads();                                         // every wave has read the weights of step st
            if (kBack) {
                back_to_lds(F, U, ok, gb, 0);
                fetch_blk(min(st + 3, st_last), blk);
            }
        }
        if (!kBack) F = front_of(blk, ok, gb, U);                    // first part of step st + 2 (its word was requested a step ago)
        // the rows of step st + 1 have landed in LDS once the loads requested after them are the only ones outstanding:
        // the three table reads that front_of leaves in flight, or the words requested behind the rows
        if (!kBack) wait_loads_but(std::integral_constant<unsigned, 3>{});
        else if (kBBufs == 1) wait_loads_but(std::integral_constant<unsigned, kFetchLoads>{});
        else wait_loads_but(std::integral_constant<unsigned, 0>{});
        read_a();
        __syncthreads();
    };
    {
        uint32_t st = st_first;
        if (dpar == 1) {                                             // relative steps 0, 2, ..: second part; 1, 3, ..: first part
            for (; st + 1 < st_end; st += 2) { slot(std::true_type{}, st); slot(std::false_type{}, st + 1); }
            if (st < st_end) slot(std::true_type{}, st);
        } else {
            for (; st + 1 < st_end; st += 2) { slot(std::false_type{}, st); slot(std::true_type{}, st + 1); }
            if (st < st_end) slot(std::false_type{}, st);
        }
    }

    // y[token][row]: register v of tile (rt, t) belongs to token m0 + 32 t + 8 (v / 4) + 4 half + v % 4, row row0 + 32 rt + col
#pragma unroll
    for (int rt = 0; rt < 4; rt++) {
        const int row = row0 + 32 * rt + col;
        if (row >= N) continue;
#pragma unroll
        for (int t = 0; t < 2; t++) {
#pragma unroll
            for (int v = 0; v < 16; v++) {
                const int tok = m0 + 32 * t + 8 * (v / 4) + 4 * half + (v % 4);
                if (tok < M) {
                    if (ksplit == 1) y[(size_t)tok * N + row] = acc[rt][t][v];
                    else atomicAdd(y + (size_t)tok * N + row, acc[rt][t][v]);
                }
            }
        }
    }
}

// ---- llvq_encode --------------------------------------------------------------------------------------
// One lane per vector: 24 bytes in, one index out.  The encoder's tables (68.5 KB) are copied to LDS first.
template <int FMT, bool DYNAMIC>
__global__ void __launch_bounds__(kThreads, 8) encode_kernel(const unsigned char* __restrict__ blob, llvq::EncLayout lay,
                                                          const uint2* __restrict__ pts, size_t n, void* __restrict__ idx,
                                                          size_t out_stride) {
    BatchDeal<DYNAMIC> deal(n, lay.bytes);
    load_tables(blob, lay.bytes);
    const llvq::EncPtrs T = llvq::make_enc_ptrs(lds_origin(), lay);
    for (; deal.base < deal.end; deal.advance()) {
        deal.take();
        const size_t k = deal.base + deal.t;
        if (k < n) {
            const uint2 p0 = pts[3 * k], p1 = pts[3 * k + 1], p2 = pts[3 * k + 2];
            const uint32_t x[6] = {p0.x, p0.y, p1.x, p1.y, p2.x, p2.y};
            const uint64_t I = llvq::encode_block(T, x);
            if constexpr (FMT == LLVQ_IDX_U64) {
                reinterpret_cast<uint64_t*>(idx)[k * out_stride] = I;
            } else {
                uint16_t* o = reinterpret_cast<uint16_t*>(idx) + 3 * k * out_stride;
                o[0] = (uint16_t)I; o[1] = (uint16_t)(I >> 16); o[2] = (uint16_t)(I >> 32);
            }
        }
    }
}

}  // namespace

#include "llvq_search_kernel.h"

namespace {

// ---- llvq_repack --------------------------------------------------------------------------------------
template <int FMT>
__global__ void repack_kernel(const void* __restrict__ idx, const uint16_t* __restrict__ gain, size_t n, uint64_t* __restrict__ out) {
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += (size_t)gridDim.x * blockDim.x)
        out[k] = (load_index<FMT>(idx, k) & 0xFFFFFFFFFFFFull) | ((uint64_t)gain[k] << 48);
}

// ---- llvq_validate ------------------------------------------------------------------------------------
template <int FMT>
__global__ void validate_kernel(const void* __restrict__ idx, size_t n, uint64_t index_mask, uint64_t npoints, unsigned long long* __restrict__ bad) {
    unsigned long long local = 0;
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += (size_t)gridDim.x * blockDim.x)
        local += (load_index<FMT>(idx, k) & index_mask) >= npoints;
    for (int off = 32; off > 0; off >>= 1) local += __shfl_down(local, off);
    if ((threadIdx.x & 63) == 0 && local) atomicAdd(bad, local);
}

// ---- llvq_validate_static: the same count without any allocation ----------------------------------------
// Partial counts, one per workgroup, live in a device array of the library itself.  Host code never passes the
// array by name: llvq_create asks the runtime for its address on the context's device and the launches pass that.
constexpr int kValidateStaticMaxWg = 1024;
constexpr int kValidateStaticThreads = 256;
static __device__ __align__(256) unsigned int g_validate_scratch[kValidateStaticMaxWg];

// every workgroup overwrites its own slot, so nothing has to be cleared between calls
template <int FMT>
__global__ void __launch_bounds__(kValidateStaticThreads) validate_partial_kernel(const void* __restrict__ idx, size_t n, uint64_t index_mask,
                                                                                  uint64_t npoints, unsigned int* __restrict__ partial) {
    __shared__ unsigned int wave_count[kValidateStaticThreads / 64];
    unsigned int local = 0;
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += (size_t)gridDim.x * blockDim.x)
        local += (load_index<FMT>(idx, k) & index_mask) >= npoints;
    for (int off = 32; off > 0; off >>= 1) local += __shfl_down(local, off);
    if ((threadIdx.x & 63) == 0) wave_count[threadIdx.x >> 6] = local;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned int total = 0;
        for (int w = 0; w < kValidateStaticThreads / 64; w++) total += wave_count[w];
        partial[blockIdx.x] = total;
    }
}

// one workgroup adds the first `nparts` partial counts (in a fixed order) and writes the total
__global__ void __launch_bounds__(kValidateStaticThreads) validate_sum_kernel(const unsigned int* __restrict__ partial, int nparts,
                                                                              unsigned long long* __restrict__ d_bad) {
    __shared__ unsigned long long wave_sum[kValidateStaticThreads / 64];
    unsigned long long local = 0;
    for (int i = threadIdx.x; i < nparts; i += kValidateStaticThreads) local += partial[i];
    for (int off = 32; off > 0; off >>= 1) local += __shfl_down(local, off);
    if ((threadIdx.x & 63) == 0) wave_sum[threadIdx.x >> 6] = local;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long total = 0;
        for (int w = 0; w < kValidateStaticThreads / 64; w++) total += wave_sum[w];
        *d_bad = total;
    }
}

}  // namespace

// ---- contexts with m_max > 13: the dequantiser of llvq_wide.h, one thread per block ----------------------------------
namespace {

constexpr uint64_t kWideIndexMask = (1ull << 56) - 1;      // 64-bit words of these contexts carry the index in their low 56 bits

template <int FMT>
__device__ __forceinline__ uint64_t wide_index(const void* __restrict__ idx, size_t k) {
    return load_index<FMT>(idx, k) & kWideIndexMask;
}

template <int FMT>
__global__ void __launch_bounds__(256) wide_decode_i8_kernel(llvq::WidePtrs T, const void* __restrict__ idx, size_t n, uint2* __restrict__ out) {
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += (size_t)gridDim.x * blockDim.x) {
        const uint64_t I = wide_index<FMT>(idx, k);
        uint32_t o[6] = {0, 0, 0, 0, 0, 0};
        float rnorm;
        if (I < T.npoints) llvq::wide_decode(T, I, o, rnorm);
        out[3 * k] = make_uint2(o[0], o[1]);
        out[3 * k + 1] = make_uint2(o[2], o[3]);
        out[3 * k + 2] = make_uint2(o[4], o[5]);
    }
}

__device__ __forceinline__ float wide_coord(const uint32_t (&o)[6], int i) { return (float)(int8_t)(o[i >> 2] >> (8 * (i & 3))); }

template <int FMT, int OUT>
__global__ void __launch_bounds__(256) wide_dequant_kernel(llvq::WidePtrs T, const void* __restrict__ idx, const uint16_t* __restrict__ gain,
                                                           size_t n, void* __restrict__ out) {
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += (size_t)gridDim.x * blockDim.x) {
        const uint64_t I = wide_index<FMT>(idx, k);
        uint32_t o[6] = {0, 0, 0, 0, 0, 0};
        float rnorm = 0.0f;
        if (I < T.npoints) llvq::wide_decode(T, I, o, rnorm);
        const float scale = __half2float(__ushort_as_half(gain[k])) * rnorm;
#pragma unroll
        for (int i = 0; i < 24; i++) {
            const float v = wide_coord(o, i) * scale;
            if constexpr (OUT == LLVQ_F32) reinterpret_cast<float*>(out)[24 * k + i] = v;
            else if constexpr (OUT == LLVQ_F16) reinterpret_cast<__half*>(out)[24 * k + i] = __float2half_rn(v);
            else reinterpret_cast<__bf16*>(out)[24 * k + i] = (__bf16)v;
        }
    }
}

// y must be zero when this kernel starts: every block adds its M partial dot products to y with atomic adds
template <int FMT, bool BF16>
__global__ void __launch_bounds__(256) wide_matmul_kernel(llvq::WidePtrs T, const uint16_t* __restrict__ x, int M, const void* __restrict__ idx,
                                                          const uint16_t* __restrict__ gain, int N, int KB, float* __restrict__ y) {
    const size_t n = (size_t)N * KB;
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += (size_t)gridDim.x * blockDim.x) {
        const uint64_t I = wide_index<FMT>(idx, k);
        if (I >= T.npoints) continue;                                   // the zero block contributes nothing
        uint32_t o[6];
        float rnorm;
        llvq::wide_decode(T, I, o, rnorm);
        const float scale = __half2float(__ushort_as_half(gain[k])) * rnorm;
        const size_t row = k / KB, b = k - row * KB;
        for (int m = 0; m < M; m++) {
            const uint16_t* xp = x + ((size_t)m * KB + b) * 24;
            float acc = 0.0f;
#pragma unroll
            for (int i = 0; i < 24; i++) {
                const float xv = BF16 ? __builtin_bit_cast(float, (uint32_t)xp[i] << 16) : __half2float(__ushort_as_half(xp[i]));
                acc = fmaf(wide_coord(o, i), xv, acc);
            }
            atomicAdd(y + (size_t)m * N + row, acc * scale);
        }
    }
}

}  // namespace

// ---- C ABI -------------------------------------------------------------------------------------------
struct llvq_ctx {
    int device = 0;
    int m_max = 0;
    int num_cu = 0;
    llvq::TableLayout lay{};
    llvq::EncLayout enc_lay{};
    uint64_t shell_off[16] = {};            // first index of each shell
    unsigned char* d_blob = nullptr;
    unsigned char* d_enc_blob = nullptr;
    llvq::SearchLayout search_lay{};
    llvq::SearchRec* d_search = nullptr;    // nearest-point search records
    uint32_t* d_words = nullptr;            // the 4096 Golay words in (weight, message) order
    uint4* d_tile_a = nullptr;              // matrix-core operands of the class tiles
    float* d_tile_scale = nullptr;          // per-class factor and offset in accumulator order
    unsigned long long* d_counter = nullptr;
    unsigned int* d_validate_scratch = nullptr;   // address of g_validate_scratch on this context's device (not owned)
    uint64_t index_mask = 0xFFFFFFFFFFFFull;      // bits of a stored word that hold the index (56 for 64-bit words of wide contexts)
    // contexts with m_max > 13: the tables of llvq_wide.h in global memory; the table-driven kernels are not available
    bool wide = false;
    llvq::WideRec* d_wrecs = nullptr;
    uint64_t* d_wcls_off = nullptr;
    uint32_t* d_wgs = nullptr;
    uint32_t* d_wbinom = nullptr;
    uint64_t wide_shell_off[24] = {};
    llvq::WidePtrs wide_ptrs() const { return llvq::WidePtrs{d_wrecs, d_wcls_off, d_wgs, d_wbinom, lay.ncls, lay.npoints}; }
    rocblas_handle blas = nullptr;          // created at the first llvq_matmul_ws call that takes the two-step path
    // text of the last failure: written under the lock (calls may fail on several threads at once), read without it
    std::mutex err_mu;
    char err[256] = {0};
    void set_error(const std::string& text) {
        std::lock_guard<std::mutex> hold(err_mu);
        std::snprintf(err, sizeof err, "%s", text.c_str());
    }
};

namespace {

int hip_fail(llvq_ctx* ctx, hipError_t e, const char* what) {
    if (ctx) ctx->set_error(std::string(what) + ": " + hipGetErrorString(e));
    return LLVQ_EHIP;
}

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_idx(const void* d_idx, int fmt) {
    if (!d_idx) return LLVQ_EINVAL;
    if (fmt == LLVQ_IDX_U48) return aligned(d_idx, 2) ? LLVQ_OK : LLVQ_EALIGN;
    if (fmt == LLVQ_IDX_U64) return aligned(d_idx, 8) ? LLVQ_OK : LLVQ_EALIGN;
    if (fmt == LLVQ_IDX_U24) return LLVQ_OK;
    return LLVQ_EINVAL;
}

// Sets the dynamic LDS size of a kernel.  The kernels address their tables from LDS address 0 (lds_origin), which
// holds only while a kernel declares no static LDS.  The kernel is a template argument, so the state below exists
// once per kernel instantiation: the static-LDS check runs at that kernel's first launch on a device, and the
// attribute is set again only when the size asked for changes.
constexpr int kMaxDevices = 64;
template <auto Kernel>
int set_lds(llvq_ctx* ctx, size_t bytes) {
    static std::atomic<size_t> configured[kMaxDevices];      // bytes + 1 of the last successful call on the device, 0: none yet
    const int dev = ctx->device;
    if (dev < kMaxDevices && configured[dev].load(std::memory_order_acquire) == bytes + 1) return LLVQ_OK;
    const void* fn = reinterpret_cast<const void*>(Kernel);
    hipFuncAttributes attr;
    hipError_t q = hipFuncGetAttributes(&attr, fn);
    if (q != hipSuccess) return hip_fail(ctx, q, "hipFuncGetAttributes");
    if (attr.sharedSizeBytes != 0) {
        ctx->set_error("a kernel that addresses its tables from LDS address 0 declares static LDS");
        return LLVQ_EHIP;
    }
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return hip_fail(ctx, e, "hipFuncSetAttribute");
    if (dev < kMaxDevices) configured[dev].store(bytes + 1, std::memory_order_release);
    return LLVQ_OK;
}

int grid_for(const llvq_ctx* ctx, size_t n, int per_cu = 1) {
    // grid-stride kernels: no more workgroups than fit the compute units at once, so that each copies the tables once
    size_t wgs = (n + kThreads - 1) / kThreads;
    size_t cap = (size_t)ctx->num_cu * per_cu;
    return (int)(wgs < 1 ? 1 : (wgs > cap ? cap : wgs));
}

}  // namespace

// Short launches keep only the small tables in LDS and run two workgroups per compute unit (see the kernels); long ones
// copy all tables and run one.  The crossover, in wave-batches of 64 blocks per compute unit, depends on how much the
// kernel stores (measured on 14336 x 4104 and on slices and multiples of it): int8 output about 768, 16-bit output about 64.
static bool small_launch(const llvq_ctx* ctx, size_t n, size_t batches_per_cu) { return n < (size_t)ctx->num_cu * 64 * batches_per_cu; }

template <int FMT>
static int launch_decode_i8(llvq_ctx* ctx, const void* d_idx, const Code& cd, size_t n, int8_t* d_out, hipStream_t st) {
    const bool small = small_launch(ctx, n, 768);
    // from about 3.5 batches per wave on, dealing the batches to the waves as they finish pays
    const bool dynamic = !small_launch(ctx, n, small ? 112 : 56);
    const size_t lds = (small ? ctx->lay.lds_bytes : ctx->lay.blob_bytes) + 16;       // + the batch counter
    const int grid = grid_for(ctx, n, small ? 2 : 1);
#define LLVQ_LAUNCH_I8(BG, DYN)                                                                                              \
    do {                                                                                                                     \
        if (int rc = set_lds<decode_i8_kernel<FMT, BG, DYN>>(ctx, lds)) return rc;                                           \
        hipLaunchKernelGGL((decode_i8_kernel<FMT, BG, DYN>), dim3(grid), dim3(kThreads), lds, st, ctx->d_blob, ctx->lay,     \
                           d_idx, cd, n, reinterpret_cast<uint32_t*>(d_out));                                                \
    } while (0)
    if (!small) LLVQ_LAUNCH_I8(false, true);
    else if (dynamic) LLVQ_LAUNCH_I8(true, true);
    else LLVQ_LAUNCH_I8(true, false);
#undef LLVQ_LAUNCH_I8
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? LLVQ_OK : hip_fail(ctx, e, "decode_i8 launch");
}

template <int FMT>
static int launch_dequant(llvq_ctx* ctx, const void* d_idx, const void* d_gain, const Code& cd, size_t n, void* d_out, int out_dtype, hipStream_t st) {
    // fp32 output is bound by its stores: it always takes the one-workgroup variant
    const bool small = small_launch(ctx, n, 64) && out_dtype != LLVQ_F32;
    const size_t lds = small ? ctx->lay.lds_bytes : ctx->lay.blob_bytes + 16;       // long launches: + the batch counter
    const int grid = grid_for(ctx, n, small ? 2 : 1);
    const uint16_t* g = reinterpret_cast<const uint16_t*>(d_gain);
#define LLVQ_LAUNCH_DQ(OUT, BG)                                                                                    \
    do {                                                                                                              \
        if (int rc = set_lds<dequant_kernel<FMT, OUT, BG>>(ctx, lds)) return rc;                                      \
        hipLaunchKernelGGL((dequant_kernel<FMT, OUT, BG>), dim3(grid), dim3(kThreads), lds, st, ctx->d_blob, ctx->lay, d_idx, g, cd, n, d_out); \
    } while (0)
    if (out_dtype == LLVQ_F16) { if (small) LLVQ_LAUNCH_DQ(LLVQ_F16, true); else LLVQ_LAUNCH_DQ(LLVQ_F16, false); }
    else if (out_dtype == LLVQ_BF16) { if (small) LLVQ_LAUNCH_DQ(LLVQ_BF16, true); else LLVQ_LAUNCH_DQ(LLVQ_BF16, false); }
    else LLVQ_LAUNCH_DQ(LLVQ_F32, false);
#undef LLVQ_LAUNCH_DQ
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? LLVQ_OK : hip_fail(ctx, e, "dequant launch");
}

// MULTI: N is the number of rows of all matrices of `items` together; d_idx, d_gain and d_y are not used
template <int FMT, typename X2, bool MULTI = false>
static int launch_matmul(llvq_ctx* ctx, const void* d_x, int M, const void* d_idx, const void* d_gain, const Code& cd, int N, int KB, float* d_y, hipStream_t st,
                         const MatItems& items = MatItems{}) {
    // one persistent workgroup per compute unit (the tables fill its LDS), rows split evenly among them
    int grid = ctx->num_cu < N ? ctx->num_cu : N;
    const int rows = (N + grid - 1) / grid;
    grid = (N + rows - 1) / rows;
    const uint32_t kb_magic = (KB > 1 && KB < 8192) ? (uint32_t)(((1ull << 32) + (uint64_t)KB - 1) / (uint64_t)KB) : 0u;
    // from 64 batches of 64 blocks per compute unit on (four per wave; measured on Llama-3-8B and 70B shapes), copying
    // all tables into LDS pays, and so does dealing the batches to the waves as they finish
    const bool short_launch = (size_t)N * (size_t)KB / 64 < (size_t)ctx->num_cu * 64;
    const size_t lds = (short_launch ? llvq::kOffInner : ctx->lay.blob_bytes) + (size_t)kRowsPerPass * kMaxMChunk * sizeof(float) + 16;   // row sums + batch counter
    const int rows_pass = std::max(1, std::min(kRowsPerPass, ((1 << 24) - 1) / KB));       // KB < 2^24 (checked by the caller)
#define LLVQ_LAUNCH_MATMUL(BG, DYN)                                                                                         \
    do {                                                                                                                    \
        if (int rc = set_lds<matmul_kernel<FMT, X2, BG, DYN, MULTI>>(ctx, lds)) return rc;                                  \
        hipLaunchKernelGGL((matmul_kernel<FMT, X2, BG, DYN, MULTI>), dim3(grid), dim3(kThreads), lds, st, ctx->d_blob,      \
                           ctx->lay, d_idx, reinterpret_cast<const uint16_t*>(d_gain), reinterpret_cast<const uint32_t*>(d_x), \
                           M, N, KB, cd, kb_magic, rows, rows_pass, items, d_y);                                             \
    } while (0)
    if (short_launch) LLVQ_LAUNCH_MATMUL(true, false);
    else LLVQ_LAUNCH_MATMUL(false, true);
#undef LLVQ_LAUNCH_MATMUL
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? LLVQ_OK : hip_fail(ctx, e, "matmul launch");
}

template <int FMT, typename X2, int THREADS, int TOKTILES, bool MULTI = false>
static int launch_mfma_cfg(llvq_ctx* ctx, const void* d_x, int M, const void* d_idx, const void* d_gain, const Code& cd, int N, int KB, float* d_y, hipStream_t st,
                           const MatItems& items = MatItems{}) {
    // workgroups = groups of row tiles (one tile per wave) x ranges of block pairs; enough ranges to fill the chip, but
    // at least two steps each to amortise the write-back of a partial tile
    constexpr uint32_t wpg = THREADS / 64;
    const uint32_t n_rt = MULTI ? (uint32_t)items.tile_end[kMaxItems - 1] : (uint32_t)((N + 31) / 32), spt = (uint32_t)((KB + 1) / 2);
    const uint32_t groups = (n_rt + wpg - 1) / wpg;
    uint32_t kranges = (uint32_t)ctx->num_cu / groups;
    kranges = std::max(1u, std::min(kranges, std::max(1u, spt / 2)));
    kranges = std::min(kranges, 65535u);
    const size_t lds = ctx->lay.blob_bytes;
    if (int rc = set_lds<mfma_kernel<FMT, X2, THREADS, TOKTILES, MULTI>>(ctx, lds)) return rc;
    hipLaunchKernelGGL((mfma_kernel<FMT, X2, THREADS, TOKTILES, MULTI>), dim3(groups, kranges), dim3(THREADS), lds, st, ctx->d_blob, ctx->lay, d_idx,
                       reinterpret_cast<const uint16_t*>(d_gain), reinterpret_cast<const uint32_t*>(d_x), M, N, KB, cd, kranges, items, d_y);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? LLVQ_OK : hip_fail(ctx, e, "mfma matmul launch");
}

constexpr int kTileMaxM = 32;       // up to this many activation rows the batched-decode kernel with row tiles per workgroup is used

template <int FMT, typename X2, int TT, bool MULTI = false>
static int launch_tile(llvq_ctx* ctx, const void* d_x, int M, const void* d_idx, const void* d_gain, const Code& cd, int N, int KB, float* d_y, hipStream_t st,
                       const MatItems& items = MatItems{}) {
    // persistent workgroups, whole row tiles split evenly among them
    const int n_tiles = MULTI ? items.tile16_end[kMaxItems - 1] : (N + kTileRows - 1) / kTileRows;
    int grid = std::min(ctx->num_cu, n_tiles);
    const int per_wg = (n_tiles + grid - 1) / grid;
    grid = (n_tiles + per_wg - 1) / per_wg;
    const size_t lds = llvq::kOffInner + (size_t)(kThreads / 64) * kTilePassSlots * 256 * sizeof(float);
    if (int rc = set_lds<tile_kernel<FMT, X2, TT, MULTI>>(ctx, lds)) return rc;
    hipLaunchKernelGGL((tile_kernel<FMT, X2, TT, MULTI>), dim3(grid), dim3(kThreads), lds, st, ctx->d_blob, ctx->lay, d_idx,
                       reinterpret_cast<const uint16_t*>(d_gain), reinterpret_cast<const uint32_t*>(d_x), M, N, KB, cd, n_tiles, per_wg, items, d_y);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? LLVQ_OK : hip_fail(ctx, e, "tile matmul launch");
}

template <int FMT>
static int launch_encode(llvq_ctx* ctx, const int8_t* d_x, size_t n, void* d_idx, hipStream_t st, size_t out_stride = 1) {
    const size_t lds = ctx->enc_lay.bytes + 16;        // + the batch counter
    // the encoder's tables take 68.5 KB: two workgroups share a compute unit (64 vector registers per lane)
    const size_t wgs = (n + kThreads - 1) / kThreads;
    const int grid = (int)std::max<size_t>(1, std::min<size_t>(wgs, (size_t)2 * ctx->num_cu));
    // from about 3.5 batches of 64 vectors per wave on, the waves take their batches as they finish
    if (n >= (size_t)ctx->num_cu * 64 * 112) {
        if (int rc = set_lds<encode_kernel<FMT, true>>(ctx, lds)) return rc;
        hipLaunchKernelGGL((encode_kernel<FMT, true>), dim3(grid), dim3(kThreads), lds, st, ctx->d_enc_blob, ctx->enc_lay,
                           reinterpret_cast<const uint2*>(d_x), n, d_idx, out_stride);
    } else {
        if (int rc = set_lds<encode_kernel<FMT, false>>(ctx, lds)) return rc;
        hipLaunchKernelGGL((encode_kernel<FMT, false>), dim3(grid), dim3(kThreads), lds, st, ctx->d_enc_blob, ctx->enc_lay,
                           reinterpret_cast<const uint2*>(d_x), n, d_idx, out_stride);
    }
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? LLVQ_OK : hip_fail(ctx, e, "encode launch");
}

// nearest-direction search of n blocks whose rows start ldw floats apart
static int launch_search(llvq_ctx* ctx, int metric, const float* d_w, size_t ldw, size_t n, int8_t* d_points, float* d_score, hipStream_t st) {
    const int grid = (int)std::min<size_t>(n, (size_t)2 * ctx->num_cu);
    if (metric == LLVQ_ANGULAR)
        hipLaunchKernelGGL(search_mfma_kernel<LLVQ_ANGULAR>, dim3(grid), dim3(kMfmaSearchThreads), 0, st, ctx->d_search, ctx->search_lay,
                           ctx->d_tile_a, ctx->d_tile_scale, ctx->d_words, d_w, ldw, n, d_points, d_score);
    else
        hipLaunchKernelGGL(search_mfma_kernel<LLVQ_EUCLIDEAN>, dim3(grid), dim3(kMfmaSearchThreads), 0, st, ctx->d_search, ctx->search_lay,
                           ctx->d_tile_a, ctx->d_tile_scale, ctx->d_words, d_w, ldw, n, d_points, d_score);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? LLVQ_OK : hip_fail(ctx, e, "search launch");
}

template <int FMT>
static int launch_validate(llvq_ctx* ctx, int grid, const void* d_idx, size_t n, hipStream_t st) {
    hipLaunchKernelGGL(validate_kernel<FMT>, dim3(grid), dim3(256), 0, st, d_idx, n, ctx->index_mask, ctx->lay.npoints, ctx->d_counter);
    return 0;
}

template <int FMT>
static int launch_validate_partial(int grid, const void* d_idx, size_t n, uint64_t index_mask, uint64_t npoints, unsigned int* partial, hipStream_t st) {
    hipLaunchKernelGGL(validate_partial_kernel<FMT>, dim3(grid), dim3(kValidateStaticThreads), 0, st, d_idx, n, index_mask, npoints, partial);
    return 0;
}

template <int FMT>
static int launch_repack(const void* d_idx, const void* d_gain, size_t n, uint64_t* d_packed, hipStream_t st) {
    const unsigned grid = (unsigned)std::min<size_t>((n + 255) / 256, 65536);
    hipLaunchKernelGGL(repack_kernel<FMT>, dim3(grid), dim3(256), 0, st, d_idx, reinterpret_cast<const uint16_t*>(d_gain), n, d_packed);
    return 0;
}

template <int FMT, typename X2, int WAVES, int TT>
static int launch_prefill(llvq_ctx* ctx, const void* d_x, int M, const void* d_idx, const void* d_gain, const Code& cd, int N, int KB, float* d_y, hipStream_t st) {
    constexpr int kRows = 32 * WAVES, kTokens = 32 * TT;
    const unsigned strips = (unsigned)((N + kRows - 1) / kRows), passes = (unsigned)((M + kTokens - 1) / kTokens);
    // enough workgroups for the chip: split the block pairs of a row among up to ksplit workgroups (at least 8 steps each)
    const unsigned spt = ((unsigned)KB + 1) / 2;
    unsigned ksplit = (unsigned)ctx->num_cu / (strips * passes);
    ksplit = std::max(1u, std::min(ksplit, std::max(1u, spt / 8)));
    if (ksplit > 1) {
        const size_t ny = (size_t)M * N;
        hipLaunchKernelGGL(fill_kernel, dim3((unsigned)std::min<size_t>((ny / 4 + 256) / 256, 4096)), dim3(256), 0, st, d_y, ny, 0.0f);
    }
    const dim3 grid(strips, passes, ksplit);
    const size_t lds = ctx->lay.lds_bytes + 2 * (size_t)kTokens * kATokenPitch;
    if (int rc = set_lds<prefill_kernel<FMT, X2, WAVES, TT>>(ctx, lds)) return rc;
    hipLaunchKernelGGL((prefill_kernel<FMT, X2, WAVES, TT>), grid, dim3(64 * WAVES), lds, st, ctx->d_blob, ctx->lay, d_idx,
                       reinterpret_cast<const uint16_t*>(d_gain), reinterpret_cast<const uint32_t*>(d_x), M, N, KB, cd, (int)ksplit, d_y);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? LLVQ_OK : hip_fail(ctx, e, "prefill matmul launch");
}

// MULTI: N is not used; the strips are those of `items`
template <int FMT, typename X2, bool MULTI = false>
static int launch_panel(llvq_ctx* ctx, const void* d_x, int M, const void* d_idx, const void* d_gain, const Code& cd, int N, int KB, float* d_y, hipStream_t st,
                        const MatItems& items = MatItems{}, int n_items = 1) {
    const unsigned strips = MULTI ? (unsigned)items.strip_end[kMaxItems - 1] : (unsigned)((N + kPanelRows - 1) / kPanelRows);
    const unsigned passes = (unsigned)((M + kPanelTokens - 1) / kPanelTokens);
    // enough workgroups for the chip: split the block pairs of a row among up to ksplit workgroups (at least 16 steps each)
    const unsigned spt = ((unsigned)KB + 1) / 2;
    unsigned ksplit = (unsigned)ctx->num_cu / (strips * passes);
    ksplit = std::max(1u, std::min(ksplit, std::max(1u, spt / 16)));
    if (ksplit > 1) {
        if (MULTI) {
            int widest = 0;
            for (int i = 0; i < n_items; i++) widest = std::max(widest, items.row_end[i] - (i ? items.row_end[i - 1] : 0));
            const size_t ny = (size_t)M * (size_t)widest;
            hipLaunchKernelGGL(fill_multi_kernel, dim3((unsigned)std::min<size_t>((ny / 4 + 256) / 256, 2048), (unsigned)n_items), dim3(256), 0, st, items, M, 0.0f);
        } else {
            const size_t ny = (size_t)M * N;
            hipLaunchKernelGGL(fill_kernel, dim3((unsigned)std::min<size_t>((ny / 4 + 256) / 256, 4096)), dim3(256), 0, st, d_y, ny, 0.0f);
        }
    }
    const dim3 grid(strips, passes, ksplit);
    constexpr int kTerms = Mma<X2>::kTerms;
    const size_t lds = ctx->lay.lds_bytes + (size_t)(kTerms == 1 ? 2 : 1) * (4 * 3 * 1024 * kTerms) + (size_t)kPanelWaves * 7 * 1024;
    if (int rc = set_lds<panel_kernel<FMT, X2, MULTI>>(ctx, lds)) return rc;
    hipLaunchKernelGGL((panel_kernel<FMT, X2, MULTI>), grid, dim3(64 * kPanelWaves), lds, st, ctx->d_blob, ctx->lay, d_idx,
                       reinterpret_cast<const uint16_t*>(d_gain), reinterpret_cast<const uint32_t*>(d_x), M, N, KB, cd, (int)ksplit, items, d_y);
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? LLVQ_OK : hip_fail(ctx, e, "panel matmul launch");
}

// whether a product with this many strips of 128 rows takes the panel kernel: from kPanelMinM tokens on, when there are
// panels for at least a sixteenth of the chip (the rest comes from splitting the rows' block pairs, at least 16 steps
// per part; measured on Llama-3-8B shapes: 4096 rows at M = 512 take 72 us against 92 us in the strip kernel, 1024 rows
// are level at M = 1024 and slower below); activation offsets inside the kernel are 32-bit byte offsets
static bool panel_fits(const llvq_ctx* ctx, int M, uint64_t strips, int KB) {
    return M >= kPanelMinM && (uint64_t)M * (uint64_t)KB * 48u < (1ull << 32) &&
           strips * (uint64_t)((M + kPanelTokens - 1) / kPanelTokens) * 16u >= (uint64_t)ctx->num_cu;
}

template <int FMT, typename X2>
static int launch_any_matmul(llvq_ctx* ctx, const void* d_x, int M, const void* d_idx, const void* d_gain, const Code& cd, int N, int KB, float* d_y, hipStream_t st) {
    if (M < kMfmaMinM) return launch_matmul<FMT, X2>(ctx, d_x, M, d_idx, d_gain, cd, N, KB, d_y, st);
    if (panel_fits(ctx, M, (uint64_t)((N + kPanelRows - 1) / kPanelRows), KB))
        return launch_panel<FMT, X2>(ctx, d_x, M, d_idx, d_gain, cd, N, KB, d_y, st);
    if (M > 64) return launch_prefill<FMT, X2, 8, 8>(ctx, d_x, M, d_idx, d_gain, cd, N, KB, d_y, st);
    if (M <= 16) return launch_tile<FMT, X2, 1>(ctx, d_x, M, d_idx, d_gain, cd, N, KB, d_y, st);
    if (M <= kTileMaxM) return launch_tile<FMT, X2, 2>(ctx, d_x, M, d_idx, d_gain, cd, N, KB, d_y, st);
    const size_t ny = (size_t)M * N;
    hipLaunchKernelGGL(fill_kernel, dim3((unsigned)std::min<size_t>((ny / 4 + 256) / 256, 4096)), dim3(256), 0, st, d_y, ny, 0.0f);
    return launch_mfma_cfg<FMT, X2, 1024, 2>(ctx, d_x, M, d_idx, d_gain, cd, N, KB, d_y, st);
}

// evaluates EXPR with the constant F set to the storage format `fmt` (which check_idx has accepted)
#define LLVQ_BY_FMT(fmt, EXPR)                                                                 \
    ((fmt) == LLVQ_IDX_U48   ? [&] { constexpr int F = LLVQ_IDX_U48; return (EXPR); }()       \
     : (fmt) == LLVQ_IDX_U64 ? [&] { constexpr int F = LLVQ_IDX_U64; return (EXPR); }()       \
                             : [&] { constexpr int F = LLVQ_IDX_U24; return (EXPR); }())

namespace {

int word_bits(int fmt) { return fmt == LLVQ_IDX_U24 ? 24 : 48; }

// the stored word is the index itself, gains come from the per-block array
Code plain_code(int fmt) {
    Code cd;
    cd.base = 0;
    cd.mask = (1ull << word_bits(fmt)) - 1;
    cd.lut = nullptr;
    cd.shape_bits = (uint32_t)word_bits(fmt);
    cd.lut_last = 0;
    cd.gain_in_word = 0;
    return cd;
}

// layout of a coded word (see llvq_*_coded in llvq.h); checks the arguments
int make_code(int fmt, int shape_bits, uint64_t base_index, const void* d_gain_lut, Code& cd) {
    if (fmt != LLVQ_IDX_U48 && fmt != LLVQ_IDX_U64 && fmt != LLVQ_IDX_U24) return LLVQ_EINVAL;
    const int wb = word_bits(fmt);
    if (shape_bits < 1 || shape_bits > wb || base_index >= (1ull << 48)) return LLVQ_EINVAL;
    if (d_gain_lut && wb - shape_bits > 12) return LLVQ_EINVAL;
    if (d_gain_lut && !aligned(d_gain_lut, 2)) return LLVQ_EALIGN;
    cd.base = base_index;
    cd.mask = (1ull << shape_bits) - 1;
    cd.lut = reinterpret_cast<const uint16_t*>(d_gain_lut);
    cd.shape_bits = (uint32_t)shape_bits;
    cd.lut_last = (1u << (wb - shape_bits)) - 1;
    cd.gain_in_word = 0;
    return LLVQ_OK;
}

int decode_i8_impl(llvq_ctx* ctx, const void* d_idx, int fmt, const Code& cd, size_t n_blocks, int8_t* d_out, void* stream) {
    if (n_blocks == 0) return LLVQ_OK;                                   // nothing to read or write
    if (!d_out) return LLVQ_EINVAL;
    if (int rc = check_idx(d_idx, fmt)) return rc;
    if (!aligned(d_out, 8)) return LLVQ_EALIGN;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    return LLVQ_BY_FMT(fmt, launch_decode_i8<F>(ctx, d_idx, cd, n_blocks, d_out, st));
}

int decode_impl(llvq_ctx* ctx, const void* d_idx, int fmt, const void* d_gain, const Code& cd, size_t n_blocks, void* d_out,
                int out_dtype, void* stream) {
    if (out_dtype != LLVQ_F16 && out_dtype != LLVQ_BF16 && out_dtype != LLVQ_F32) return LLVQ_EINVAL;
    if (n_blocks == 0) return LLVQ_OK;
    if (!d_out || (!d_gain && cd.gain_array())) return LLVQ_EINVAL;
    if (int rc = check_idx(d_idx, fmt)) return rc;
    if (!aligned(d_out, 16) || !aligned(d_gain, 2)) return LLVQ_EALIGN;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    return LLVQ_BY_FMT(fmt, launch_dequant<F>(ctx, d_idx, d_gain, cd, n_blocks, d_out, out_dtype, st));
}

int matmul_impl(llvq_ctx* ctx, const void* d_x, int x_dtype, int M, const void* d_idx, int fmt, const void* d_gain, const Code& cd,
                int N, int KB, float* d_y, void* stream) {
    if (!d_x || (!d_gain && cd.gain_array()) || !d_y) return LLVQ_EINVAL;
    if (M < 1 || M > 1024 || N < 1 || KB < 1 || KB >= (1 << 24)) return LLVQ_EINVAL;
    if (x_dtype != LLVQ_F16 && x_dtype != LLVQ_BF16) return LLVQ_EINVAL;
    if ((size_t)N * (size_t)KB >= (1ull << 32)) return LLVQ_EINVAL;
    if (int rc = check_idx(d_idx, fmt)) return rc;
    if (!aligned(d_x, 16) || !aligned(d_gain, 2) || !aligned(d_y, 4)) return LLVQ_EALIGN;
    if (M >= kMfmaMinM && ((size_t)((N + 31) / 32) * (size_t)((KB + 1) / 2) >= (1ull << 32) || (size_t)M * (size_t)N >= (1ull << 32) ||
                           (size_t)M * (size_t)KB * 12 >= (1ull << 32)))
        return LLVQ_EINVAL;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (x_dtype == LLVQ_F16) return LLVQ_BY_FMT(fmt, (launch_any_matmul<F, half2_t>(ctx, d_x, M, d_idx, d_gain, cd, N, KB, d_y, st)));
    return LLVQ_BY_FMT(fmt, (launch_any_matmul<F, bf16x2_t>(ctx, d_x, M, d_idx, d_gain, cd, N, KB, d_y, st)));
}

int matmul_multi_impl(llvq_ctx* ctx, const void* d_x, int x_dtype, int M, int n_items, const void* const* d_idx, int fmt,
                      const void* const* d_gain, const int* N, int KB, float* const* d_y, void* stream) {
    if (!d_x || !d_idx || !d_gain || !N || !d_y) return LLVQ_EINVAL;
    if (n_items < 1 || n_items > kMaxItems || M < 1 || M > 1024 || KB < 1 || KB >= (1 << 24)) return LLVQ_EINVAL;
    if (x_dtype != LLVQ_F16 && x_dtype != LLVQ_BF16) return LLVQ_EINVAL;
    if (!aligned(d_x, 16)) return LLVQ_EALIGN;
    const Code cd = plain_code(fmt);
    size_t total = 0;
    for (int i = 0; i < n_items; i++) {
        if (!d_gain[i] || !d_y[i] || N[i] < 1) return LLVQ_EINVAL;
        if (int rc = check_idx(d_idx[i], fmt)) return rc;
        if (!aligned(d_gain[i], 2) || !aligned(d_y[i], 4)) return LLVQ_EALIGN;
        total += (size_t)N[i];
    }
    if (total * (size_t)KB >= (1ull << 32)) return LLVQ_EINVAL;
    if (M >= kMfmaMinM) {
        size_t tiles = 0;
        for (int i = 0; i < n_items; i++) {
            if ((size_t)M * (size_t)N[i] >= (1ull << 32)) return LLVQ_EINVAL;
            tiles += (size_t)((N[i] + 31) / 32);
        }
        if (tiles * (size_t)((KB + 1) / 2) >= (1ull << 32) || (size_t)M * (size_t)KB * 12 >= (1ull << 32)) return LLVQ_EINVAL;
    }
    MatItems items;
    int rows = 0, tiles = 0, tiles16 = 0, strips = 0;
    for (int i = 0; i < kMaxItems; i++) {
        const int k = i < n_items ? i : n_items - 1;
        if (i < n_items) { rows += N[i]; tiles += (N[i] + 31) / 32; tiles16 += (N[i] + kTileRows - 1) / kTileRows; strips += (N[i] + kPanelRows - 1) / kPanelRows; }
        items.tile16_end[i] = tiles16;
        items.strip_end[i] = strips;
        items.idx[i] = d_idx[k];
        items.gain[i] = reinterpret_cast<const uint16_t*>(d_gain[k]);
        items.y[i] = d_y[k];
        items.row_end[i] = rows;
        items.tile_end[i] = tiles;
    }
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    // prefill: the 128-row strips of all matrices in one launch when at least one of them has panels for less than half
    // of the chip (small matrices such as k and v then run at the rate of the large ones; matrices that fill the chip
    // on their own gain nothing from sharing a launch and lose to the uneven last round)
    bool small_item = false;
    for (int i = 0; i < n_items; i++)
        small_item = small_item || (uint64_t)((N[i] + kPanelRows - 1) / kPanelRows) * (uint64_t)((M + kPanelTokens - 1) / kPanelTokens) * 2u < (uint64_t)ctx->num_cu;
    if (n_items > 1 && small_item && panel_fits(ctx, M, (uint64_t)strips, KB)) {
        if (x_dtype == LLVQ_F16)
            return LLVQ_BY_FMT(fmt, (launch_panel<F, half2_t, true>(ctx, d_x, M, d_idx[0], d_gain[0], cd, rows, KB, d_y[0], st, items, n_items)));
        return LLVQ_BY_FMT(fmt, (launch_panel<F, bf16x2_t, true>(ctx, d_x, M, d_idx[0], d_gain[0], cd, rows, KB, d_y[0], st, items, n_items)));
    }
    if (n_items == 1 || M > 64) {
        // one matrix, or a batch that takes the strip kernel: one product after the other
        for (int i = 0; i < n_items; i++)
            if (int rc = matmul_impl(ctx, d_x, x_dtype, M, d_idx[i], fmt, d_gain[i], cd, N[i], KB, d_y[i], stream)) return rc;
        return LLVQ_OK;
    }
    if (M >= kMfmaMinM && M <= kTileMaxM) {
        // row tiles of all matrices in one launch, each tile reduced inside its workgroup
        if (x_dtype == LLVQ_F16) {
            if (M <= 16) return LLVQ_BY_FMT(fmt, (launch_tile<F, half2_t, 1, true>(ctx, d_x, M, d_idx[0], d_gain[0], cd, rows, KB, d_y[0], st, items)));
            return LLVQ_BY_FMT(fmt, (launch_tile<F, half2_t, 2, true>(ctx, d_x, M, d_idx[0], d_gain[0], cd, rows, KB, d_y[0], st, items)));
        }
        if (M <= 16) return LLVQ_BY_FMT(fmt, (launch_tile<F, bf16x2_t, 1, true>(ctx, d_x, M, d_idx[0], d_gain[0], cd, rows, KB, d_y[0], st, items)));
        return LLVQ_BY_FMT(fmt, (launch_tile<F, bf16x2_t, 2, true>(ctx, d_x, M, d_idx[0], d_gain[0], cd, rows, KB, d_y[0], st, items)));
    }
    if (M >= kMfmaMinM) {
        // the batched-decode kernel over the row tiles of all matrices; the outputs are cleared by one launch as well
        int widest = 0;
        for (int i = 0; i < n_items; i++) widest = std::max(widest, N[i]);
        const size_t ny = (size_t)M * (size_t)widest;
        hipLaunchKernelGGL(fill_multi_kernel, dim3((unsigned)std::min<size_t>((ny / 4 + 256) / 256, 2048), (unsigned)n_items), dim3(256), 0, st, items, M, 0.0f);
        if (x_dtype == LLVQ_F16)
            return LLVQ_BY_FMT(fmt, (launch_mfma_cfg<F, half2_t, 1024, 2, true>(ctx, d_x, M, d_idx[0], d_gain[0], cd, rows, KB, d_y[0], st, items)));
        return LLVQ_BY_FMT(fmt, (launch_mfma_cfg<F, bf16x2_t, 1024, 2, true>(ctx, d_x, M, d_idx[0], d_gain[0], cd, rows, KB, d_y[0], st, items)));
    }
    if (x_dtype == LLVQ_F16)
        return LLVQ_BY_FMT(fmt, (launch_matmul<F, half2_t, true>(ctx, d_x, M, d_idx[0], d_gain[0], cd, rows, KB, d_y[0], st, items)));
    return LLVQ_BY_FMT(fmt, (launch_matmul<F, bf16x2_t, true>(ctx, d_x, M, d_idx[0], d_gain[0], cd, rows, KB, d_y[0], st, items)));
}

bool plain_fmt(int fmt) { return fmt == LLVQ_IDX_U48 || fmt == LLVQ_IDX_U64 || fmt == LLVQ_IDX_U24; }

}  // namespace

namespace {

int wide_grid(const llvq_ctx* ctx, size_t n) { return (int)std::max<size_t>(1, std::min<size_t>((n + 255) / 256, (size_t)ctx->num_cu * 16)); }

template <int FMT>
int wide_launch_decode_i8(llvq_ctx* ctx, const void* d_idx, size_t n, int8_t* d_out, hipStream_t st) {
    hipLaunchKernelGGL(wide_decode_i8_kernel<FMT>, dim3(wide_grid(ctx, n)), dim3(256), 0, st, ctx->wide_ptrs(), d_idx, n, reinterpret_cast<uint2*>(d_out));
    return 0;
}

template <int FMT>
int wide_launch_dequant(llvq_ctx* ctx, const void* d_idx, const void* d_gain, size_t n, void* d_out, int out_dtype, hipStream_t st) {
    const uint16_t* g = reinterpret_cast<const uint16_t*>(d_gain);
    const dim3 grid(wide_grid(ctx, n));
    if (out_dtype == LLVQ_F16) hipLaunchKernelGGL((wide_dequant_kernel<FMT, LLVQ_F16>), grid, dim3(256), 0, st, ctx->wide_ptrs(), d_idx, g, n, d_out);
    else if (out_dtype == LLVQ_BF16) hipLaunchKernelGGL((wide_dequant_kernel<FMT, LLVQ_BF16>), grid, dim3(256), 0, st, ctx->wide_ptrs(), d_idx, g, n, d_out);
    else hipLaunchKernelGGL((wide_dequant_kernel<FMT, LLVQ_F32>), grid, dim3(256), 0, st, ctx->wide_ptrs(), d_idx, g, n, d_out);
    return 0;
}

template <int FMT>
int wide_launch_matmul(llvq_ctx* ctx, const void* d_x, int x_dtype, int M, const void* d_idx, const void* d_gain, int N, int KB, float* d_y, hipStream_t st) {
    const size_t ny = (size_t)M * N, n = (size_t)N * KB;
    hipLaunchKernelGGL(fill_kernel, dim3((unsigned)std::min<size_t>((ny / 4 + 256) / 256, 4096)), dim3(256), 0, st, d_y, ny, 0.0f);
    const uint16_t* x = reinterpret_cast<const uint16_t*>(d_x);
    const uint16_t* g = reinterpret_cast<const uint16_t*>(d_gain);
    if (x_dtype == LLVQ_BF16) hipLaunchKernelGGL((wide_matmul_kernel<FMT, true>), dim3(wide_grid(ctx, n)), dim3(256), 0, st, ctx->wide_ptrs(), x, M, d_idx, g, N, KB, d_y);
    else hipLaunchKernelGGL((wide_matmul_kernel<FMT, false>), dim3(wide_grid(ctx, n)), dim3(256), 0, st, ctx->wide_ptrs(), x, M, d_idx, g, N, KB, d_y);
    return 0;
}

constexpr int kWideMaxBatch = 16;      // activation rows the wide contexts' product accepts

int wide_finish(llvq_ctx* ctx, const char* what) {
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? LLVQ_OK : hip_fail(ctx, e, what);
}

}  // namespace

extern "C" {

const char* llvq_strerror(int rc) {
    switch (rc) {
        case LLVQ_OK: return "ok";
        case LLVQ_EINVAL: return "invalid argument";
        case LLVQ_EALIGN: return "misaligned pointer";
        case LLVQ_EHIP: return "HIP call failed";
        case LLVQ_ENOTIMPL: return "not implemented";
        default: return "unknown error";
    }
}

const char* llvq_last_hip_error(const llvq_ctx* ctx) { return ctx ? ctx->err : ""; }

// a context for 14 <= m_max <= 19: the tables of llvq_wide.h in global memory
static int create_wide(llvq_ctx** out, int m_max, int device) {
    llvq::WideTables tabs;
    if (!llvq::build_wide_tables(m_max, tabs)) return LLVQ_EINVAL;
    llvq_ctx* ctx = new (std::nothrow) llvq_ctx;
    if (!ctx) return LLVQ_EINVAL;
    ctx->device = device; ctx->m_max = m_max; ctx->wide = true;
    ctx->lay = llvq::TableLayout{};
    ctx->lay.ncls = tabs.lay.ncls; ctx->lay.npoints = tabs.lay.npoints;
    ctx->index_mask = kWideIndexMask;
    for (int m = 0; m < 24; m++) ctx->wide_shell_off[m] = tabs.shell_off[m];
    hipDeviceProp_t prop;
    auto upload = [&](auto** dst, const auto& v) {
        const size_t bytes = v.size() * sizeof(v[0]);
        return hipMalloc(reinterpret_cast<void**>(dst), bytes) == hipSuccess && hipMemcpy(*dst, v.data(), bytes, hipMemcpyHostToDevice) == hipSuccess;
    };
    if (hipSetDevice(device) != hipSuccess || hipGetDeviceProperties(&prop, device) != hipSuccess ||
        !upload(&ctx->d_wrecs, tabs.recs) || !upload(&ctx->d_wcls_off, tabs.cls_off) || !upload(&ctx->d_wgs, tabs.gs) ||
        !upload(&ctx->d_wbinom, tabs.binom) || hipMalloc(&ctx->d_counter, sizeof(unsigned long long)) != hipSuccess ||
        hipGetSymbolAddress(reinterpret_cast<void**>(&ctx->d_validate_scratch), HIP_SYMBOL(g_validate_scratch)) != hipSuccess) {
        llvq_destroy(ctx);
        return LLVQ_EHIP;
    }
    ctx->num_cu = prop.multiProcessorCount;
    *out = ctx;
    return LLVQ_OK;
}

int llvq_create(llvq_ctx** out, int m_max, int device) {
    if (!out || m_max < 2 || m_max > llvq::kWideMaxM || device < 0) return LLVQ_EINVAL;
    *out = nullptr;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) return LLVQ_EHIP;
    if (m_max > 13) return create_wide(out, m_max, device);
    llvq::Tables tabs;
    if (!llvq::build_tables(m_max, tabs)) return LLVQ_EINVAL;
    llvq_ctx* ctx = new (std::nothrow) llvq_ctx;
    if (!ctx) return LLVQ_EINVAL;
    ctx->device = device; ctx->m_max = m_max; ctx->lay = tabs.lay;
    for (int m = 0; m < 16; m++) ctx->shell_off[m] = tabs.shell_off[m];
    hipError_t e;
    if ((e = hipSetDevice(device)) != hipSuccess) { delete ctx; return LLVQ_EHIP; }
    hipDeviceProp_t prop;
    if ((e = hipGetDeviceProperties(&prop, device)) != hipSuccess) { delete ctx; return LLVQ_EHIP; }
    ctx->num_cu = prop.multiProcessorCount;
    constexpr size_t kScratch = (size_t)kRowsPerPass * kMaxMChunk * sizeof(float) + 16;    // the largest kernel scratch beside the tables (row sums + batch counter)
    if (tabs.lay.blob_bytes + kScratch > prop.sharedMemPerBlock && tabs.lay.blob_bytes + kScratch > (size_t)prop.sharedMemPerBlockOptin) { delete ctx; return LLVQ_ENOTIMPL; }
    if ((e = hipMalloc(&ctx->d_blob, tabs.blob.size())) != hipSuccess) { delete ctx; return LLVQ_EHIP; }
    if ((e = hipMalloc(&ctx->d_counter, sizeof(unsigned long long))) != hipSuccess) { (void)hipFree(ctx->d_blob); delete ctx; return LLVQ_EHIP; }
    if ((e = hipMemcpy(ctx->d_blob, tabs.blob.data(), tabs.blob.size(), hipMemcpyHostToDevice)) != hipSuccess) {
        (void)hipFree(ctx->d_blob); (void)hipFree(ctx->d_counter); delete ctx; return LLVQ_EHIP;
    }
    // this device's copy of the library's own scratch array (llvq_validate_static)
    if ((e = hipGetSymbolAddress(reinterpret_cast<void**>(&ctx->d_validate_scratch), HIP_SYMBOL(g_validate_scratch))) != hipSuccess) {
        (void)hipFree(ctx->d_blob); (void)hipFree(ctx->d_counter); delete ctx; return LLVQ_EHIP;
    }
    ctx->enc_lay = tabs.enc_lay;
    if ((e = hipMalloc(&ctx->d_enc_blob, tabs.enc_blob.size())) != hipSuccess ||
        (e = hipMemcpy(ctx->d_enc_blob, tabs.enc_blob.data(), tabs.enc_blob.size(), hipMemcpyHostToDevice)) != hipSuccess) {
        if (ctx->d_enc_blob) (void)hipFree(ctx->d_enc_blob);
        (void)hipFree(ctx->d_blob); (void)hipFree(ctx->d_counter); delete ctx; return LLVQ_EHIP;
    }
    ctx->search_lay = tabs.search_lay;
    const size_t sbytes = tabs.search_recs.size() * sizeof(llvq::SearchRec), wbytes = tabs.golay_sorted.size() * sizeof(uint32_t);
    if ((e = hipMalloc(&ctx->d_search, sbytes)) != hipSuccess || (e = hipMalloc(&ctx->d_words, wbytes)) != hipSuccess ||
        (e = hipMemcpy(ctx->d_search, tabs.search_recs.data(), sbytes, hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(ctx->d_words, tabs.golay_sorted.data(), wbytes, hipMemcpyHostToDevice)) != hipSuccess) {
        llvq_destroy(ctx);
        return LLVQ_EHIP;
    }
    const size_t abytes = tabs.search_tile_a.size() * sizeof(uint16_t), scbytes = tabs.search_tile_scale.size() * sizeof(float);
    if ((e = hipMalloc(&ctx->d_tile_a, abytes)) != hipSuccess || (e = hipMalloc(&ctx->d_tile_scale, scbytes)) != hipSuccess ||
        (e = hipMemcpy(ctx->d_tile_a, tabs.search_tile_a.data(), abytes, hipMemcpyHostToDevice)) != hipSuccess ||
        (e = hipMemcpy(ctx->d_tile_scale, tabs.search_tile_scale.data(), scbytes, hipMemcpyHostToDevice)) != hipSuccess) {
        llvq_destroy(ctx);
        return LLVQ_EHIP;
    }
    *out = ctx;
    return LLVQ_OK;
}

void llvq_destroy(llvq_ctx* ctx) {
    if (!ctx) return;
    (void)hipSetDevice(ctx->device);
    if (ctx->d_blob) (void)hipFree(ctx->d_blob);
    if (ctx->d_counter) (void)hipFree(ctx->d_counter);
    if (ctx->d_enc_blob) (void)hipFree(ctx->d_enc_blob);
    if (ctx->d_search) (void)hipFree(ctx->d_search);
    if (ctx->d_words) (void)hipFree(ctx->d_words);
    if (ctx->d_tile_a) (void)hipFree(ctx->d_tile_a);
    if (ctx->d_tile_scale) (void)hipFree(ctx->d_tile_scale);
    if (ctx->blas) (void)rocblas_destroy_handle(ctx->blas);
    if (ctx->d_wrecs) (void)hipFree(ctx->d_wrecs);
    if (ctx->d_wcls_off) (void)hipFree(ctx->d_wcls_off);
    if (ctx->d_wgs) (void)hipFree(ctx->d_wgs);
    if (ctx->d_wbinom) (void)hipFree(ctx->d_wbinom);
    delete ctx;
}

uint64_t llvq_num_points(const llvq_ctx* ctx) { return ctx ? ctx->lay.npoints : 0; }
int llvq_num_classes(const llvq_ctx* ctx) { return ctx ? (int)ctx->lay.ncls : 0; }

uint64_t llvq_shell_offset(const llvq_ctx* ctx, int m) {
    if (!ctx || m < 2) return 0;
    if (m > ctx->m_max) return ctx->lay.npoints;
    return ctx->wide ? ctx->wide_shell_off[m] : ctx->shell_off[m];
}


int llvq_decode_i8(llvq_ctx* ctx, const void* d_idx, int fmt, size_t n_blocks, int8_t* d_out, void* stream) {
    if (!ctx || !plain_fmt(fmt)) return LLVQ_EINVAL;
    if (ctx->wide) {
        if (n_blocks == 0) return LLVQ_OK;
        if (!d_out) return LLVQ_EINVAL;
        if (int rc = check_idx(d_idx, fmt)) return rc;
        if (!aligned(d_out, 8)) return LLVQ_EALIGN;
        LLVQ_BY_FMT(fmt, wide_launch_decode_i8<F>(ctx, d_idx, n_blocks, d_out, reinterpret_cast<hipStream_t>(stream)));
        return wide_finish(ctx, "decode_i8 launch");
    }
    return decode_i8_impl(ctx, d_idx, fmt, plain_code(fmt), n_blocks, d_out, stream);
}

int llvq_decode(llvq_ctx* ctx, const void* d_idx, int fmt, const void* d_gain, size_t n_blocks, void* d_out, int out_dtype, void* stream) {
    if (!ctx || !plain_fmt(fmt)) return LLVQ_EINVAL;
    if (n_blocks && !d_gain) return LLVQ_EINVAL;
    if (ctx->wide) {
        if (out_dtype != LLVQ_F16 && out_dtype != LLVQ_BF16 && out_dtype != LLVQ_F32) return LLVQ_EINVAL;
        if (n_blocks == 0) return LLVQ_OK;
        if (!d_out) return LLVQ_EINVAL;
        if (int rc = check_idx(d_idx, fmt)) return rc;
        if (!aligned(d_out, 16) || !aligned(d_gain, 2)) return LLVQ_EALIGN;
        LLVQ_BY_FMT(fmt, wide_launch_dequant<F>(ctx, d_idx, d_gain, n_blocks, d_out, out_dtype, reinterpret_cast<hipStream_t>(stream)));
        return wide_finish(ctx, "dequant launch");
    }
    return decode_impl(ctx, d_idx, fmt, d_gain, plain_code(fmt), n_blocks, d_out, out_dtype, stream);
}

int llvq_matmul(llvq_ctx* ctx, const void* d_x, int x_dtype, int M, const void* d_idx, int fmt, const void* d_gain,
                int N, int KB, float* d_y, void* stream) {
    if (!ctx || !d_gain || !plain_fmt(fmt)) return LLVQ_EINVAL;
    if (ctx->wide) {
        if (!d_x || !d_y || M < 1 || N < 1 || KB < 1 || KB >= (1 << 24)) return LLVQ_EINVAL;
        if (x_dtype != LLVQ_F16 && x_dtype != LLVQ_BF16) return LLVQ_EINVAL;
        if (M > kWideMaxBatch) return LLVQ_ENOTIMPL;
        if (int rc = check_idx(d_idx, fmt)) return rc;
        if (!aligned(d_x, 16) || !aligned(d_gain, 2) || !aligned(d_y, 4)) return LLVQ_EALIGN;
        LLVQ_BY_FMT(fmt, wide_launch_matmul<F>(ctx, d_x, x_dtype, M, d_idx, d_gain, N, KB, d_y, reinterpret_cast<hipStream_t>(stream)));
        return wide_finish(ctx, "matmul launch");
    }
    return matmul_impl(ctx, d_x, x_dtype, M, d_idx, fmt, d_gain, plain_code(fmt), N, KB, d_y, stream);
}

int llvq_matmul_multi(llvq_ctx* ctx, const void* d_x, int x_dtype, int M, int n_items, const void* const* d_idx, int fmt,
                      const void* const* d_gain, const int* N, int KB, float* const* d_y, void* stream) {
    if (!ctx) return LLVQ_EINVAL;
    if (ctx->wide) return LLVQ_ENOTIMPL;
    if (!plain_fmt(fmt)) return LLVQ_EINVAL;
    return matmul_multi_impl(ctx, d_x, x_dtype, M, n_items, d_idx, fmt, d_gain, N, KB, d_y, stream);
}

int llvq_decode_i8_coded(llvq_ctx* ctx, const void* d_idx, int fmt, int shape_bits, uint64_t base_index, size_t n_blocks,
                         int8_t* d_out, void* stream) {
    if (!ctx) return LLVQ_EINVAL;
    if (ctx->wide) return LLVQ_ENOTIMPL;
    Code cd;
    if (int rc = make_code(fmt, shape_bits, base_index, nullptr, cd)) return rc;
    return decode_i8_impl(ctx, d_idx, fmt, cd, n_blocks, d_out, stream);
}

int llvq_decode_coded(llvq_ctx* ctx, const void* d_idx, int fmt, int shape_bits, uint64_t base_index, const void* d_gain_lut,
                      const void* d_gain, size_t n_blocks, void* d_out, int out_dtype, void* stream) {
    if (!ctx) return LLVQ_EINVAL;
    if (ctx->wide) return LLVQ_ENOTIMPL;
    Code cd;
    if (int rc = make_code(fmt, shape_bits, base_index, d_gain_lut, cd)) return rc;
    cd.gain_in_word = !d_gain_lut && !d_gain && fmt == LLVQ_IDX_U64 && shape_bits == 48;     // the layout llvq_repack writes
    return decode_impl(ctx, d_idx, fmt, d_gain, cd, n_blocks, d_out, out_dtype, stream);
}

int llvq_matmul_coded(llvq_ctx* ctx, const void* d_x, int x_dtype, int M, const void* d_idx, int fmt, int shape_bits,
                      uint64_t base_index, const void* d_gain_lut, const void* d_gain, int N, int KB, float* d_y, void* stream) {
    if (!ctx) return LLVQ_EINVAL;
    if (ctx->wide) return LLVQ_ENOTIMPL;
    Code cd;
    if (int rc = make_code(fmt, shape_bits, base_index, d_gain_lut, cd)) return rc;
    cd.gain_in_word = !d_gain_lut && !d_gain && fmt == LLVQ_IDX_U64 && shape_bits == 48;     // the layout llvq_repack writes
    return matmul_impl(ctx, d_x, x_dtype, M, d_idx, fmt, d_gain, cd, N, KB, d_y, stream);
}

int llvq_repack(llvq_ctx* ctx, const void* d_idx, int fmt, const void* d_gain, size_t n_blocks, uint64_t* d_packed, void* stream) {
    if (!ctx || (fmt != LLVQ_IDX_U48 && fmt != LLVQ_IDX_U64)) return LLVQ_EINVAL;
    if (ctx->wide) return LLVQ_ENOTIMPL;
    if (n_blocks == 0) return LLVQ_OK;
    if (!d_gain || !d_packed) return LLVQ_EINVAL;
    if (int rc = check_idx(d_idx, fmt)) return rc;
    if (!aligned(d_gain, 2) || !aligned(d_packed, 8)) return LLVQ_EALIGN;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    LLVQ_BY_FMT(fmt, launch_repack<F>(d_idx, d_gain, n_blocks, d_packed, st));
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? LLVQ_OK : hip_fail(ctx, e, "repack launch");
}

int llvq_encode(llvq_ctx* ctx, const int8_t* d_x, size_t n_blocks, void* d_idx, int fmt, void* stream) {
    if (!ctx || (fmt != LLVQ_IDX_U48 && fmt != LLVQ_IDX_U64)) return LLVQ_EINVAL;
    if (ctx->wide) return LLVQ_ENOTIMPL;
    if (n_blocks == 0) return LLVQ_OK;
    if (!d_x) return LLVQ_EINVAL;
    if (int rc = check_idx(d_idx, fmt)) return rc;
    if (!aligned(d_x, 8)) return LLVQ_EALIGN;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    return fmt == LLVQ_IDX_U48 ? launch_encode<LLVQ_IDX_U48>(ctx, d_x, n_blocks, d_idx, st) : launch_encode<LLVQ_IDX_U64>(ctx, d_x, n_blocks, d_idx, st);
}

int llvq_quantize(llvq_ctx* ctx, const float* d_w, size_t n_blocks, int metric, int8_t* d_points, void* d_idx, int fmt,
                  float* d_score, void* stream) {
    if (!ctx || (metric != LLVQ_ANGULAR && metric != LLVQ_EUCLIDEAN)) return LLVQ_EINVAL;
    if (ctx->wide) return LLVQ_ENOTIMPL;
    if (d_idx && fmt != LLVQ_IDX_U48 && fmt != LLVQ_IDX_U64) return LLVQ_EINVAL;
    if (n_blocks == 0) return LLVQ_OK;
    if (!d_w || !d_points) return LLVQ_EINVAL;
    if (!aligned(d_w, 4) || !aligned(d_points, 8) || !aligned(d_score, 4)) return LLVQ_EALIGN;
    if (d_idx) { if (int rc = check_idx(d_idx, fmt)) return rc; }
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (int rc = launch_search(ctx, metric, d_w, 24, n_blocks, d_points, d_score, st)) return rc;
    return d_idx ? llvq_encode(ctx, d_points, n_blocks, d_idx, fmt, stream) : LLVQ_OK;
}

size_t llvq_gptq_workspace_bytes(int N) { return N < 1 ? 0 : (size_t)N * (24 * sizeof(float) + 24) + 256; }

int llvq_gptq_quantize(llvq_ctx* ctx, float* d_W, int N, int KB, size_t ldw, const float* d_U, void* d_idx, int fmt,
                       void* d_gain, void* d_ws, size_t ws_bytes, void* stream) {
    return llvq_gptq_quantize_levels(ctx, d_W, N, KB, ldw, d_U, d_idx, fmt, d_gain, nullptr, 0, d_ws, ws_bytes, stream);
}

int llvq_gptq_quantize_levels(llvq_ctx* ctx, float* d_W, int N, int KB, size_t ldw, const float* d_U, void* d_idx, int fmt,
                              void* d_gain, const void* d_gain_levels, int n_levels, void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx || !d_W || !d_U || !d_gain || !d_ws || N < 1 || KB < 1 || ldw < (size_t)24 * KB) return LLVQ_EINVAL;
    if (ctx->wide) return LLVQ_ENOTIMPL;
    if (d_gain_levels && (n_levels < 1 || n_levels > 4096)) return LLVQ_EINVAL;
    if (!aligned(d_gain_levels, 2)) return LLVQ_EALIGN;
    if (fmt != LLVQ_IDX_U48 && fmt != LLVQ_IDX_U64) return LLVQ_EINVAL;
    if (ws_bytes < llvq_gptq_workspace_bytes(N)) return LLVQ_EINVAL;
    if (int rc = check_idx(d_idx, fmt)) return rc;
    if (!aligned(d_W, 4) || !aligned(d_U, 4) || !aligned(d_gain, 2) || !aligned(d_ws, 16)) return LLVQ_EALIGN;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!ctx->blas && rocblas_create_handle(&ctx->blas) != rocblas_status_success) { ctx->set_error("rocblas_create_handle failed"); return LLVQ_EHIP; }
    if (rocblas_set_stream(ctx->blas, st) != rocblas_status_success) { ctx->set_error("rocblas_set_stream failed"); return LLVQ_EHIP; }
    float* d_E = reinterpret_cast<float*>(d_ws);                                             // [N][24]
    int8_t* d_pts = reinterpret_cast<int8_t*>(d_ws) + (((size_t)N * 24 * sizeof(float) + 255) & ~(size_t)255);   // [N][24]
    const size_t K = (size_t)24 * KB;
    const size_t isz = fmt == LLVQ_IDX_U48 ? 6 : 8;
    const float one = 1.0f, minus_one = -1.0f;
    for (int t = 0; t < KB; t++) {
        float* Wq = d_W + (size_t)24 * t;
        // directions of this block column, their indices (strided into the [N][KB] array), gain reset and error
        if (int rc = launch_search(ctx, LLVQ_ANGULAR, Wq, ldw, (size_t)N, d_pts, nullptr, st)) return rc;
        void* idx_t = reinterpret_cast<unsigned char*>(d_idx) + isz * (size_t)t;
        const int rc = fmt == LLVQ_IDX_U48 ? launch_encode<LLVQ_IDX_U48>(ctx, d_pts, (size_t)N, idx_t, st, (size_t)KB)
                                           : launch_encode<LLVQ_IDX_U64>(ctx, d_pts, (size_t)N, idx_t, st, (size_t)KB);
        if (rc) return rc;
        hipLaunchKernelGGL(retract_kernel, dim3((N + 255) / 256), dim3(256), 0, st, Wq, ldw, d_pts, N, d_E,
                           reinterpret_cast<uint16_t*>(d_gain) + t, (size_t)KB, reinterpret_cast<const uint16_t*>(d_gain_levels), n_levels);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(ctx, e, "gptq step launch");
        const size_t r0 = (size_t)24 * (t + 1);
        if (r0 >= K) break;
        // W[:, R] -= (E U_QQ^-1) U_QR.  Row-major arrays seen column-major: E^T (24 x N), U^T (lower triangular)
        const float* Uqq = d_U + (size_t)24 * t * K + (size_t)24 * t;
        rocblas_status bs = rocblas_strsm(ctx->blas, rocblas_side_left, rocblas_fill_lower, rocblas_operation_none,
                                          rocblas_diagonal_non_unit, 24, N, &one, Uqq, (rocblas_int)K, d_E, 24);
        if (bs == rocblas_status_success)
            bs = rocblas_sgemm(ctx->blas, rocblas_operation_none, rocblas_operation_none, (rocblas_int)(K - r0), N, 24, &minus_one,
                               d_U + (size_t)24 * t * K + r0, (rocblas_int)K, d_E, 24, &one, d_W + r0, (rocblas_int)ldw);
        if (bs != rocblas_status_success) { ctx->set_error(std::string("rocblas: ") + rocblas_status_to_string(bs)); return LLVQ_EHIP; }
    }
    return LLVQ_OK;
}

// rows of a chunk of llvq_gptq_group_scales (one KB x KB system per row is held in the workspace)
static int group_chunk_rows(int N) { return N < 128 ? N : 128; }

size_t llvq_gptq_group_scales_workspace_bytes(int N, int KB) {
    if (N < 1 || KB < 1) return 0;
    const size_t K = (size_t)24 * KB, C = (size_t)group_chunk_rows(N);
    return sizeof(float) * ((size_t)N * K + C * K + C * KB * KB + (size_t)N * KB) + 1024;
}

int llvq_gptq_group_scales(llvq_ctx* ctx, float* d_Wq, const float* d_W0, int N, int KB, size_t ldw, const float* d_H, float lambda,
                           void* d_gain, float* d_s, void* d_ws, size_t ws_bytes, void* stream) {
    if (!ctx || !d_Wq || !d_W0 || !d_H || !d_gain || !d_ws || N < 1 || KB < 1 || KB > 1024 || ldw < (size_t)24 * KB) return LLVQ_EINVAL;
    if (ctx->wide) return LLVQ_ENOTIMPL;
    if (!(lambda >= 0.0f)) return LLVQ_EINVAL;
    if (ws_bytes < llvq_gptq_group_scales_workspace_bytes(N, KB)) return LLVQ_EINVAL;
    if (!aligned(d_Wq, 4) || !aligned(d_W0, 4) || !aligned(d_H, 4) || !aligned(d_gain, 2) || !aligned(d_s, 4) || !aligned(d_ws, 16)) return LLVQ_EALIGN;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!ctx->blas && rocblas_create_handle(&ctx->blas) != rocblas_status_success) { ctx->set_error("rocblas_create_handle failed"); return LLVQ_EHIP; }
    if (rocblas_set_stream(ctx->blas, st) != rocblas_status_success) { ctx->set_error("rocblas_set_stream failed"); return LLVQ_EHIP; }
    const size_t K = (size_t)24 * KB;
    const int C = group_chunk_rows(N);
    auto up = [](size_t v) { return (v + 63) & ~(size_t)63; };
    float* d_T = reinterpret_cast<float*>(d_ws);                       // [N][K]  = W0 H
    float* d_Z = d_T + up((size_t)N * K);                              // [C][K]  = Wq[rows, block p] H[block p, :]
    float* d_M = d_Z + up((size_t)C * K);                              // [C][KB][KB]
    float* d_r = d_M + up((size_t)C * KB * KB);                        // [N][KB]
    const float one = 1.0f, zero = 0.0f;
    // T = W0 H.  Row-major arrays seen column-major: T^T (K x N) = H (K x K, symmetric) * W0^T (K x N, leading dimension ldw)
    rocblas_status bs = rocblas_sgemm(ctx->blas, rocblas_operation_none, rocblas_operation_none, (rocblas_int)K, N, (rocblas_int)K, &one,
                                      d_H, (rocblas_int)K, d_W0, (rocblas_int)ldw, &zero, d_T, (rocblas_int)K);
    if (bs != rocblas_status_success) { ctx->set_error(std::string("rocblas: ") + rocblas_status_to_string(bs)); return LLVQ_EHIP; }
    {
        const size_t n = (size_t)N * KB;
        hipLaunchKernelGGL(group_rhs_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, d_Wq, ldw, d_T, K, N, KB, d_r);
    }
    for (int row0 = 0; row0 < N; row0 += C) {
        const int c = std::min(C, N - row0);
        for (int p = 0; p < KB; p++) {
            // Z^T (K x c) = H[block p, :]^T (K x 24) * Wq[rows, block p]^T (24 x c)
            bs = rocblas_sgemm(ctx->blas, rocblas_operation_none, rocblas_operation_none, (rocblas_int)K, c, 24, &one,
                               d_H + (size_t)24 * p * K, (rocblas_int)K, d_Wq + (size_t)row0 * ldw + (size_t)24 * p, (rocblas_int)ldw, &zero,
                               d_Z, (rocblas_int)K);
            if (bs != rocblas_status_success) { ctx->set_error(std::string("rocblas: ") + rocblas_status_to_string(bs)); return LLVQ_EHIP; }
            const size_t n = (size_t)c * KB;
            hipLaunchKernelGGL(group_gram_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, d_Wq, ldw, d_Z, K, row0, c, KB, p, d_M);
        }
        hipLaunchKernelGGL(group_solve_kernel, dim3(c), dim3(kGroupSolveThreads), 0, st, d_M, d_r, lambda, row0, c, KB, d_Wq, ldw,
                           reinterpret_cast<uint16_t*>(d_gain), d_s);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(ctx, e, "group scales launch");
    }
    return LLVQ_OK;
}

int llvq_matmul_ws(llvq_ctx* ctx, const void* d_x, int x_dtype, int M, const void* d_idx, int fmt, const void* d_gain,
                   int N, int KB, float* d_y, void* d_ws, size_t ws_bytes, void* stream) {
    if (ctx && ctx->wide) return llvq_matmul(ctx, d_x, x_dtype, M, d_idx, fmt, d_gain, N, KB, d_y, stream);
    const size_t need = (size_t)N * (size_t)KB * 24 * 2;
    if (!ctx || !d_ws || ws_bytes < need || M < kGemmMinM)
        return llvq_matmul(ctx, d_x, x_dtype, M, d_idx, fmt, d_gain, N, KB, d_y, stream);
    if (!d_x || !d_gain || !d_y || M > 1024 || N < 1 || KB < 1) return LLVQ_EINVAL;
    if (x_dtype != LLVQ_F16 && x_dtype != LLVQ_BF16) return LLVQ_EINVAL;
    if (!aligned(d_x, 16) || !aligned(d_ws, 16) || !aligned(d_y, 4)) return LLVQ_EALIGN;
    // step 1: shape-gain reconstruction of the whole matrix into the workspace, in the activation type
    if (int rc = llvq_decode(ctx, d_idx, fmt, d_gain, (size_t)N * KB, d_ws, x_dtype, stream)) return rc;
    // step 2: plain dense GEMM y[M][N] = x[M][K] * W[N][K]^T on the matrix cores (library routine), fp32 accumulate
    if (!ctx->blas && rocblas_create_handle(&ctx->blas) != rocblas_status_success) { ctx->set_error("rocblas_create_handle failed"); return LLVQ_EHIP; }
    if (rocblas_set_stream(ctx->blas, reinterpret_cast<hipStream_t>(stream)) != rocblas_status_success) { ctx->set_error("rocblas_set_stream failed"); return LLVQ_EHIP; }
    const float alpha = 1.0f, beta = 0.0f;
    const int K = 24 * KB;
    const rocblas_datatype ab = x_dtype == LLVQ_F16 ? rocblas_datatype_f16_r : rocblas_datatype_bf16_r;
    // column-major view: y^T (N x M, ld N) = W^T-as-stored (K x N, ld K) transposed  x  x^T-as-stored (K x M, ld K)
    const rocblas_status st = rocblas_gemm_ex(ctx->blas, rocblas_operation_transpose, rocblas_operation_none, N, M, K, &alpha,
                                              d_ws, ab, K, d_x, ab, K, &beta, d_y, rocblas_datatype_f32_r, N,
                                              d_y, rocblas_datatype_f32_r, N, rocblas_datatype_f32_r, rocblas_gemm_algo_standard, 0, 0);
    if (st != rocblas_status_success) { ctx->set_error(std::string("rocblas_gemm_ex: ") + rocblas_status_to_string(st)); return LLVQ_EHIP; }
    return LLVQ_OK;
}

int llvq_validate(llvq_ctx* ctx, const void* d_idx, int fmt, size_t n_blocks, uint64_t* h_bad, void* stream) {
    if (!ctx || !h_bad || !plain_fmt(fmt)) return LLVQ_EINVAL;
    if (n_blocks) { if (int rc = check_idx(d_idx, fmt)) return rc; }
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    hipError_t e;
    unsigned long long zero = 0;
    if ((e = hipMemcpyAsync(ctx->d_counter, &zero, sizeof zero, hipMemcpyHostToDevice, st)) != hipSuccess) return hip_fail(ctx, e, "validate reset");
    if (n_blocks) {
        const int grid = grid_for(ctx, n_blocks);
        LLVQ_BY_FMT(fmt, launch_validate<F>(ctx, grid, d_idx, n_blocks, st));
        if ((e = hipGetLastError()) != hipSuccess) return hip_fail(ctx, e, "validate launch");
    }
    unsigned long long got = 0;
    if ((e = hipMemcpyAsync(&got, ctx->d_counter, sizeof got, hipMemcpyDeviceToHost, st)) != hipSuccess) return hip_fail(ctx, e, "validate read");
    if ((e = hipStreamSynchronize(st)) != hipSuccess) return hip_fail(ctx, e, "validate sync");
    *h_bad = got;
    return LLVQ_OK;
}

int llvq_validate_static(llvq_ctx* ctx, const void* d_idx, int fmt, size_t n_blocks, uint64_t* d_bad, void* stream) {
    if (!ctx || !d_bad || !plain_fmt(fmt)) return LLVQ_EINVAL;
    if (n_blocks > LLVQ_VALIDATE_STATIC_MAX_BLOCKS) {
        ctx->set_error("llvq_validate_static: n_blocks exceeds LLVQ_VALIDATE_STATIC_MAX_BLOCKS");
        return LLVQ_EINVAL;
    }
    if (!aligned(d_bad, 8)) return LLVQ_EALIGN;
    if (n_blocks) { if (int rc = check_idx(d_idx, fmt)) return rc; }
    if (!ctx->d_validate_scratch) return LLVQ_EHIP;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    int grid = 0;
    if (n_blocks) {
        const size_t wgs = (n_blocks + kValidateStaticThreads - 1) / kValidateStaticThreads;
        grid = (int)std::min<size_t>(wgs, (size_t)std::min(kValidateStaticMaxWg, 4 * ctx->num_cu));
        LLVQ_BY_FMT(fmt, launch_validate_partial<F>(grid, d_idx, n_blocks, ctx->index_mask, ctx->lay.npoints, ctx->d_validate_scratch, st));
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return hip_fail(ctx, e, "validate_static launch");
    }
    hipLaunchKernelGGL(validate_sum_kernel, dim3(1), dim3(kValidateStaticThreads), 0, st, ctx->d_validate_scratch, grid,
                       reinterpret_cast<unsigned long long*>(d_bad));
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? LLVQ_OK : hip_fail(ctx, e, "validate_static sum launch");
}

}  // extern "C"
