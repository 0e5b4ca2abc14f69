// Test-only harness: runs the library's table builder and its index -> block reconstruction on the host CPU
// so that the host logic (tables, digit extraction, ranking) can be compared with the oracle without a GPU.
// It is not part of the library and nothing in the product links to it.
#include <cstdint>
#include <cstring>

#include "../../paper_2603_11021_amd/csrc/llvq_decode_core.h"
#include "../../paper_2603_11021_amd/csrc/llvq_encode_core.h"
#include "../../paper_2603_11021_amd/csrc/llvq_tables.h"
#include "../../paper_2603_11021_amd/csrc/llvq_wide.h"

static llvq::Tables g_tabs;
static bool g_ok = false;

extern "C" {

int emul_init(int m_max) {
    g_ok = llvq::build_tables(m_max, g_tabs);
    return g_ok ? 0 : -1;
}

uint32_t emul_lds_bytes() { return g_tabs.lay.blob_bytes; }     // the most any kernel copies into LDS
uint32_t emul_num_classes() { return g_tabs.lay.ncls; }
uint64_t emul_num_points() { return g_tabs.lay.npoints; }
uint32_t emul_inner_entries() { return g_tabs.lay.inner_entries; }

// returns the number of out-of-range indices (decoded to zero)
uint64_t emul_decode_i8(const uint64_t* idx, uint64_t n, int8_t* out) {
    const llvq::TabPtrs T = llvq::make_tab_ptrs(g_tabs.blob.data(), g_tabs.blob.data(), g_tabs.lay);
    uint64_t bad = 0;
    for (uint64_t k = 0; k < n; k++) {
        if (idx[k] >= T.npoints) { bad++; std::memset(out + 24 * k, 0, 24); continue; }
        uint32_t w[4], o[6];
        const llvq::BlockInfo bi = llvq::decode_block(T, idx[k], w);
        llvq::nibbles_to_i8(w, bi.vti_lo, bi.vti_hi, o);
        std::memcpy(out + 24 * k, o, 24);
    }
    return bad;
}

uint32_t emul_enc_bytes() { return g_tabs.enc_lay.bytes; }

// pts: n x 24 int8; idx receives the index or all ones; returns the number of vectors that are not points
uint64_t emul_encode(const int8_t* pts, uint64_t n, uint64_t* idx) {
    const llvq::EncPtrs T = llvq::make_enc_ptrs(g_tabs.enc_blob.data(), g_tabs.enc_lay);
    uint64_t bad = 0;
    for (uint64_t k = 0; k < n; k++) {
        uint32_t x[6];
        std::memcpy(x, pts + 24 * k, 24);
        idx[k] = llvq::encode_block(T, x);
        bad += idx[k] == llvq::kInvalidIndex;
    }
    return bad;
}

// ---- the decoder of the larger unions (m_max up to 19) ------------------------------------------------------
static llvq::WideTables g_wide;

int emul_wide_init(int m_max) { return llvq::build_wide_tables(m_max, g_wide) ? 0 : -1; }
uint32_t emul_wide_num_classes() { return g_wide.lay.ncls; }
uint64_t emul_wide_num_points() { return g_wide.lay.npoints; }
uint64_t emul_wide_shell_offset(int m) { return (m >= 0 && m < 24) ? g_wide.shell_off[m] : 0; }

uint64_t emul_wide_decode_i8(const uint64_t* idx, uint64_t n, int8_t* out) {
    llvq::WidePtrs T = {g_wide.recs.data(), g_wide.cls_off.data(), g_wide.gs.data(), g_wide.binom.data(), g_wide.lay.ncls, g_wide.lay.npoints};
    uint64_t bad = 0;
    for (uint64_t k = 0; k < n; k++) {
        if (idx[k] >= T.npoints) { bad++; std::memset(out + 24 * k, 0, 24); continue; }
        uint32_t o[6];
        float rnorm;
        llvq::wide_decode(T, idx[k], o, rnorm);
        std::memcpy(out + 24 * k, o, 24);
    }
    return bad;
}

}  // extern "C"
