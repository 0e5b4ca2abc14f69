// Nearest point of the ball cut Lambda_24(m_max) for a real vector of 24 coordinates (paper Sec. 3, Sec. 3.1):
// the search over leaders (classes) and Golay words, scored by cosine (angular, for shape-gain) or by Euclidean
// distance (spherical shaping).  Included by llvq_kernels.hip.
//
// Given a class and a Golay word the best arrangement follows from sorting (rearrangement inequality):
//   odd class : x_i = 1 + 2 c_i (mod 4) fixes every sign, so <w, x> = sum coef_k * y_(k) with y_i = +-w_i by c_i
//               sorted descending and coef = +a (a = 1 mod 4) / -a (a = 3 mod 4) sorted descending;
//   even class: the 2-mod-4 values on supp(c), the 0-mod-4 values outside, each list descending onto the positions
//               by descending |w_i|, signs those of w_i; if the number of negative signs on supp(c) has the wrong
//               parity for condition (iii) of Sec. 2.3, the position of supp(c) with the smallest |w_i| (it holds
//               the smallest value) changes sign, which costs 2 * a_min * |w|_min.
// One workgroup handles one input vector at a time: a thread takes one Golay word and sorts once for the odd classes
// and once for the even classes of the word's weight; the scores of all classes against the sorted inputs are a
// dense contraction and run on the matrix cores (see below).  The workgroup's best candidate is then turned back
// into coordinates by the first 24 lanes.
#pragma once

namespace {

// Batcher's merge-exchange network for any n, largest element first; all indices are compile-time constants
template <int N, typename T, typename CE>
__device__ __forceinline__ void sort_network(T (&v)[N], CE ce) {
#pragma unroll
    for (int p = 1; p < N; p <<= 1) {
#pragma unroll
        for (int k = p; k >= 1; k >>= 1) {
#pragma unroll
            for (int j = k % p; j + k < N; j += 2 * k) {
#pragma unroll
                for (int i = 0; i < k; i++) {
                    if (i + j + k < N && (i + j) / (2 * p) == (i + j + k) / (2 * p)) ce(v[i + j], v[i + j + k]);
                }
            }
        }
    }
}

struct ScoredId {
    float score;
    uint32_t id;     // record index | word index << 9
};

__device__ __forceinline__ ScoredId better(ScoredId a, ScoredId b) {
    return (b.score > a.score || (b.score == a.score && b.id < a.id)) ? b : a;
}

// ---- the class scores on the matrix cores -------------------------------------------------------------------
// Scoring all classes against all Golay words is a dense contraction: scores[class][word] = sum_k C[class][k] Z[k][word],
// Z the sorted inputs of a word.  The class values are small integers, exact in bf16; the inputs are split exactly
// into three bf16 terms (8 + 8 + 8 mantissa bits), so three bf16 MFMA passes accumulate in fp32 what an fp32
// product would.  A wave takes 64 words (one per lane): each lane sorts for its word, the operands of the two
// 32-word column tiles are formed by swapping registers between the lane halves (v_permlane32_swap), and every
// tile of 32 classes costs six v_mfma_f32_32x32x16_bf16 per column tile.  Only the best score per lane and the
// tile it came from are tracked; the class inside the winning tile is found afterwards by scoring that one tile
// for the winning word in fp32 on the vector ALUs, which also yields the reported score.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kMfmaSearchThreads = 512;

// the 24 sorted inputs of the odd classes for word c
__device__ __forceinline__ void arrange_odd(const float (&wv)[24], uint32_t c, float (&y)[24]) {
#pragma unroll
    for (int i = 0; i < 24; i++) y[i] = __uint_as_float(__float_as_uint(wv[i]) ^ (((c >> i) & 1u) << 31));
    sort_network<24>(y, [](float& a, float& b) { const float hi = fmaxf(a, b), lo = fminf(a, b); a = hi; b = lo; });
}

// the 24 sorted magnitudes of the even classes for word c (support first), and the two parity-repair costs
__device__ __forceinline__ void arrange_even(const float (&wv)[24], uint32_t negmask, uint32_t c, float (&e)[24], float& pen_k0,
                                             float& pen_k1, int& grp) {
    uint32_t key[24];
#pragma unroll
    for (int i = 0; i < 24; i++) key[i] = (__float_as_uint(wv[i]) & 0x7FFFFFFFu) | (((c >> i) & 1u) << 31);
    sort_network<24>(key, [](uint32_t& a, uint32_t& b) { const uint32_t hi = max(a, b), lo = min(a, b); a = hi; b = lo; });
#pragma unroll
    for (int i = 0; i < 24; i++) e[i] = __uint_as_float(key[i] & 0x7FFFFFFFu);
    const uint32_t wt = (uint32_t)__popc(c);
    grp = wt == 0 ? 0 : (wt == 8 ? 1 : (wt == 12 ? 2 : (wt == 16 ? 3 : 4)));
    const float xmin1 = wt == 0 ? 0.0f : (wt == 8 ? e[7] : (wt == 12 ? e[11] : (wt == 16 ? e[15] : e[23])));
    const uint32_t negpar = (uint32_t)__popc(c & negmask) & 1u;
    pen_k0 = negpar ? xmin1 : 0.0f;      // cost when the class wants an even number of negative signs on the support
    pen_k1 = negpar ? 0.0f : xmin1;      // ... an odd number
}

// exact three-way split of fp32 values into bf16 terms, packed two per dword: out[t][d] holds elements 2d, 2d+1 of term t
template <int NPAIR>
__device__ __forceinline__ void split_bf16(const float* v, uint32_t (&out)[3][NPAIR]) {
#pragma unroll
    for (int d = 0; d < NPAIR; d++) {
        float a = v[2 * d], b = v[2 * d + 1];
#pragma unroll
        for (int t = 0; t < 3; t++) {
            // the upper halves of a and b side by side (a in the low half): one byte permute, which also truncates
            out[t][d] = __builtin_amdgcn_perm(__float_as_uint(b), __float_as_uint(a), 0x07060302u);
            if (t < 2) {
                a -= __uint_as_float(__float_as_uint(a) & 0xFFFF0000u);
                b -= __uint_as_float(__float_as_uint(b) & 0xFFFF0000u);
            }
        }
    }
}

struct ColumnOperands {      // B operands of one 32-word column tile: [term][k block] as four dwords
    uint4 b[3][2];
};

// v[0..23] (+ two extra values at k = 24, 25) of this lane's word -> operands of the column tiles of the lower and upper lane half
__device__ __forceinline__ void make_operands(const float (&v)[24], float x24, float x25, ColumnOperands& lo, ColumnOperands& hi) {
    uint32_t p[3][12], q[3][1];
    split_bf16<12>(v, p);
    const float extra[2] = {x24, x25};
    split_bf16<1>(extra, q);
#pragma unroll
    for (int t = 0; t < 3; t++) {
        uint32_t x[4], z[4], x2[4], z2[4];
#pragma unroll
        for (int d = 0; d < 4; d++) {
            // k block 0: k 0..7 from the lower half, 8..15 from the upper half; k block 1: 16..23 and 24..31
            const auto s0 = __builtin_amdgcn_permlane32_swap(p[t][d], p[t][4 + d], false, false);
            const auto s1 = __builtin_amdgcn_permlane32_swap(p[t][8 + d], d == 0 ? q[t][0] : 0u, false, false);
            x[d] = s0[0]; z[d] = s0[1]; x2[d] = s1[0]; z2[d] = s1[1];
        }
        lo.b[t][0] = make_uint4(x[0], x[1], x[2], x[3]);
        lo.b[t][1] = make_uint4(x2[0], x2[1], x2[2], x2[3]);
        hi.b[t][0] = make_uint4(z[0], z[1], z[2], z[3]);
        hi.b[t][1] = make_uint4(z2[0], z2[1], z2[2], z2[3]);
    }
}

// best score of one class tile against one column tile, per lane (the lane's 16 accumulator rows).  Angular metric:
// score = product x factor of the class.  Euclidean metric: score = product + offset of the class, and the offsets
// are what the accumulators start from, so the products need no further instruction.
template <int METRIC>
__device__ __forceinline__ float tile_best(const uint4 (&A)[2], const ColumnOperands& B, const float (&scale)[16]) {
    f32x16_t acc;
#pragma unroll
    for (int r = 0; r < 16; r++) acc[r] = METRIC == 0 ? 0.0f : scale[r];
#pragma unroll
    for (int t = 0; t < 3; t++) {
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, A[kb]), __builtin_bit_cast(bf16x8_t, B.b[t][kb]), acc, 0, 0, 0);
    }
    float x[16];
#pragma unroll
    for (int r = 0; r < 16; r++) x[r] = METRIC == 0 ? acc[r] * scale[r] : acc[r];
    float best = fmaxf(x[0], x[1]);
#pragma unroll
    for (int r = 2; r < 16; r += 2) best = fmaxf(fmaxf(x[r], x[r + 1]), best);       // compiles to v_max3_f32
    return best;
}

template <int METRIC>
__global__ void __launch_bounds__(kMfmaSearchThreads, 4) search_mfma_kernel(const llvq::SearchRec* __restrict__ recs, llvq::SearchLayout lay,
                                                                          const uint4* __restrict__ tile_a, const float* __restrict__ tile_scale,
                                                                          const uint32_t* __restrict__ words, const float* __restrict__ w_in,
                                                                          size_t ldw, size_t n, int8_t* __restrict__ pts,
                                                                          float* __restrict__ score_out) {
    constexpr int kWavesHere = kMfmaSearchThreads / 64;
    __shared__ uint4 s_a[llvq::kMaxSearchTiles * 2 * 64];
    __shared__ float s_scale[llvq::kMaxSearchTiles * 32];          // [tile][half][16] of this metric
    __shared__ float s_score[kWavesHere];
    __shared__ uint32_t s_id[kWavesHere];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
    for (uint32_t i = threadIdx.x; i < lay.n_tiles * 128u; i += kMfmaSearchThreads) s_a[i] = tile_a[i];
    for (uint32_t i = threadIdx.x; i < lay.n_tiles * 32u; i += kMfmaSearchThreads)
        s_scale[i] = tile_scale[(i >> 5) * llvq::kSearchTileScaleFloats + METRIC * 32 + (i & 31u)];
    __syncthreads();

    for (size_t v = blockIdx.x; v < n; v += gridDim.x) {
        float wv[24];
        uint32_t negmask = 0;
#pragma unroll
        for (int i = 0; i < 24; i++) {
            wv[i] = w_in[ldw * v + i];
            negmask |= (wv[i] < 0.0f ? 1u : 0u) << i;
        }
        ScoredId best = {-INFINITY, 0u};          // id = tile << 16 | word index
        for (int r = 0; r < 4096 / kMfmaSearchThreads; r++) {
            const uint32_t ubase = (uint32_t)(kMfmaSearchThreads * r + 64 * wave);
            const uint32_t c = words[ubase + lane];
            // word index of this lane's column in the two column tiles
            const uint32_t u_lo = ubase + (lane & 31), u_hi = u_lo + 32;
            auto score_tiles = [&](const ColumnOperands& lo, const ColumnOperands& hi, uint32_t t0, uint32_t t1, bool ok_lo, bool ok_hi) {
                for (uint32_t ct = t0; ct < t1; ct++) {
                    uint4 A[2];
                    A[0] = s_a[(ct * 2 + 0) * 64 + lane];
                    A[1] = s_a[(ct * 2 + 1) * 64 + lane];
                    float scale[16];
#pragma unroll
                    for (int k = 0; k < 16; k++) scale[k] = s_scale[ct * 32 + half * 16 + k];
                    const float b_lo = tile_best<METRIC>(A, lo, scale), b_hi = tile_best<METRIC>(A, hi, scale);
                    if (ok_lo && b_lo > best.score) best = {b_lo, (ct << 16) | u_lo};
                    if (ok_hi && b_hi > best.score) best = {b_hi, (ct << 16) | u_hi};
                }
            };
            {
                float y[24];
                arrange_odd(wv, c, y);
                ColumnOperands lo, hi;
                make_operands(y, 0.0f, 0.0f, lo, hi);
                score_tiles(lo, hi, lay.grp_tile_first[0], lay.grp_tile_first[0] + lay.grp_tile_count[0], true, true);
            }
            {
                float e[24], pen_k0, pen_k1;
                int grp;
                arrange_even(wv, negmask, c, e, pen_k0, pen_k1, grp);
                ColumnOperands lo, hi;
                make_operands(e, pen_k0, pen_k1, lo, hi);
                // weight group of the words of the two column tiles, as seen from this lane
                const auto gs = __builtin_amdgcn_permlane32_swap((uint32_t)grp, (uint32_t)grp, false, false);
                const int g_lo = (int)gs[0], g_hi = (int)gs[1];
                for (int g = 0; g < 5; g++) {
                    if (!__builtin_amdgcn_ballot_w64(grp == g)) continue;
                    score_tiles(lo, hi, lay.grp_tile_first[1 + g], lay.grp_tile_first[1 + g] + lay.grp_tile_count[1 + g], g_lo == g, g_hi == g);
                }
            }
        }
        // ---- best of the workgroup: (score, tile, word) -------------------------------------------------------
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            ScoredId o;
            o.score = __shfl_xor(best.score, off);
            o.id = __shfl_xor(best.id, off);
            best = better(best, o);
        }
        if (lane == 0) { s_score[wave] = best.score; s_id[wave] = best.id; }
        __syncthreads();
        if (wave == 0) {
            ScoredId b = {lane < kWavesHere ? s_score[lane] : -INFINITY, lane < kWavesHere ? s_id[lane] : 0xFFFFFFFFu};
#pragma unroll
            for (int off = 4; off > 0; off >>= 1) {
                ScoredId o;
                o.score = __shfl_xor(b.score, off);
                o.id = __shfl_xor(b.id, off);
                b = better(b, o);
            }
            const uint32_t win = __shfl(b.id, 0);
            const uint32_t ct = win >> 16, u = win & 0xFFFFu;
            const uint32_t c = words[u];
            // ---- the class inside the winning tile: lane = row of the tile, fp32 on the vector ALUs ----------
            const bool odd_tile = ct < lay.grp_tile_first[1];
            float z[24], pen_k0 = 0.0f, pen_k1 = 0.0f;
            int grp = 0;
            if (odd_tile) arrange_odd(wv, c, z);
            else arrange_even(wv, negmask, c, z, pen_k0, pen_k1, grp);
            const uint32_t row = lane & 31;
            const bool valid = row < lay.tile_rows[ct];
            const uint32_t j = lay.tile_first_rec[ct] + (valid ? row : 0u);
            const llvq::SearchRec& S = recs[j];
            float acc = 0.0f;
#pragma unroll
            for (int k = 0; k < 24; k++) acc = fmaf(S.coef[k], z[k], acc);
            acc = fmaf(-S.amin2, S.kappa ? pen_k1 : pen_k0, acc);
            ScoredId cand = {valid ? fmaf(acc, S.mul[METRIC], S.bias[METRIC]) : -INFINITY, j};
#pragma unroll
            for (int off = 16; off > 0; off >>= 1) {
                ScoredId o;
                o.score = __shfl_xor(cand.score, off);
                o.id = __shfl_xor(cand.id, off);
                cand = better(cand, o);
            }
            cand.score = __shfl(cand.score, 0);
            cand.id = __shfl(cand.id, 0);
            // ---- the winner's coordinates: lane i = position i ------------------------------------------------
            const llvq::SearchRec& R = recs[cand.id];
            const int i = lane < 24 ? lane : 23;
            const float wi = w_in[ldw * v + i];
            const uint32_t ci = (c >> i) & 1u;
            int x;
            if (odd_tile) {
                const float yi = __uint_as_float(__float_as_uint(wi) ^ (ci << 31));
                int rank = 0;
                for (int k = 0; k < 24; k++) {
                    const float yk = __shfl(yi, k);
                    rank += (yk > yi || (yk == yi && k < i)) ? 1 : 0;
                }
                const int a = (int)R.coef[rank];
                x = ci ? -a : a;
            } else {
                const uint32_t keyi = (__float_as_uint(wi) & 0x7FFFFFFFu) | (ci << 31);
                int rank = 0;
                for (int k = 0; k < 24; k++) {
                    const uint32_t kk = __shfl(keyi, k);
                    rank += (kk > keyi || (kk == keyi && k < i)) ? 1 : 0;
                }
                const int a = (int)R.coef[rank];
                x = wi < 0.0f ? -a : a;
                const uint32_t wt = (uint32_t)__popc(c);
                const uint32_t negpar = (uint32_t)__popc(c & negmask) & 1u;
                if (wt > 0 && negpar != R.kappa && rank == (int)wt - 1) x = -x;
            }
            if (lane < 24) pts[24 * v + lane] = (int8_t)x;
            if (lane == 0 && score_out) score_out[v] = cand.score;
        }
        __syncthreads();
    }
}

// One step of the block-wise loop of paper App. B (Alg. 1): for every row the block v = W[row][0..23] has been
// given its nearest direction x (pts); the block is replaced by g * x / ||x|| with g = ||v|| rounded to fp16 (the
// norm-preserving "gain reset" of paper Sec. 3.3), and the error E = v - g x/||x|| is kept for the propagation.
// levels != nullptr: the optional scalar gain quantiser of App. B Alg. 1 -- g is the nearest of n_levels fp16
// reconstruction levels (ascending; ties go to the lower level) instead of the rounded norm.
__global__ void retract_kernel(float* __restrict__ W, size_t ldw, const int8_t* __restrict__ pts, int N,
                               float* __restrict__ E, uint16_t* __restrict__ gain, size_t gain_stride,
                               const uint16_t* __restrict__ levels, int n_levels) {
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= N) return;
    float v[24], x[24], n2 = 0.0f, x2 = 0.0f;
#pragma unroll
    for (int i = 0; i < 24; i++) {
        v[i] = W[(size_t)row * ldw + i];
        x[i] = (float)pts[(size_t)row * 24 + i];
        n2 = fmaf(v[i], v[i], n2);
        x2 = fmaf(x[i], x[i], x2);
    }
    const float norm = sqrtf(n2);
    __half gh = __float2half_rn(norm);
    if (levels) {
        float best = INFINITY;
        for (int k = 0; k < n_levels; k++) {
            const __half lv = __ushort_as_half(levels[k]);
            const float d = fabsf(norm - __half2float(lv));
            if (d < best) { best = d; gh = lv; }
        }
    }
    const float scale = __half2float(gh) / sqrtf(x2);
#pragma unroll
    for (int i = 0; i < 24; i++) {
        const float q = scale * x[i];
        W[(size_t)row * ldw + i] = q;
        E[(size_t)row * 24 + i] = v[i] - q;
    }
    gain[(size_t)row * gain_stride] = __half_as_ushort(gh);
}

// ---- closed-form group scales (paper App. J): per row, the Hessian-weighted least-squares gains of the fixed blocks ----
// r[i][p] = sum over the channels a of block p of Wq[i][a] * T[i][a], T = W0 H
__global__ void group_rhs_kernel(const float* __restrict__ Wq, size_t ldw, const float* __restrict__ T, size_t ldt, int N, int KB,
                                 float* __restrict__ r) {
    const size_t u = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= (size_t)N * KB) return;
    const size_t i = u / KB, p = u - i * KB;
    const float* a = Wq + i * ldw + 24 * p;
    const float* t = T + i * ldt + 24 * p;
    float acc = 0.0f;
#pragma unroll
    for (int k = 0; k < 24; k++) acc = fmaf(a[k], t[k], acc);
    r[u] = acc;
}

// M[c][p][q] = sum over the channels b of block q of Z[c][b] * Wq[row0 + c][b], Z = Wq[rows, block p] H[block p, :]
__global__ void group_gram_kernel(const float* __restrict__ Wq, size_t ldw, const float* __restrict__ Z, size_t ldz, int row0, int C, int KB,
                                  int p, float* __restrict__ Mm) {
    const size_t u = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= (size_t)C * KB) return;
    const size_t c = u / KB, q = u - c * KB;
    const float* a = Wq + (size_t)(row0 + c) * ldw + 24 * q;
    const float* z = Z + c * ldz + 24 * q;
    float acc = 0.0f;
#pragma unroll
    for (int k = 0; k < 24; k++) acc = fmaf(z[k], a[k], acc);
    Mm[(c * KB + (size_t)p) * KB + q] = acc;
}

// One workgroup per row: solves (M + lambda I) s = r by a Cholesky factorisation in place (lower triangle), then
// rescales the row's blocks and gains.  A matrix that is not positive definite in fp32 leaves the row as it is (s = 1).
constexpr int kGroupSolveThreads = 256;
__global__ void __launch_bounds__(kGroupSolveThreads) group_solve_kernel(float* __restrict__ Mm, const float* __restrict__ r, float lambda,
                                                                        int row0, int C, int KB, float* __restrict__ Wq, size_t ldw,
                                                                        uint16_t* __restrict__ gain, float* __restrict__ s_out) {
    const int c = blockIdx.x;
    if (c >= C) return;
    float* A = Mm + (size_t)c * KB * KB;
    const float* b = r + (size_t)(row0 + c) * KB;
    __shared__ float sol[1024];            // KB <= 1024 is checked by the host
    __shared__ int failed;
    const int tid = threadIdx.x;
    if (tid == 0) failed = 0;
    for (int i = tid; i < KB; i += kGroupSolveThreads) A[(size_t)i * KB + i] += lambda;
    __syncthreads();
    for (int j = 0; j < KB; j++) {
        const float d = A[(size_t)j * KB + j];
        if (!(d > 0.0f)) { if (tid == 0) failed = 1; break; }       // every thread reads the same value: uniform exit
        const float inv = 1.0f / sqrtf(d);
        __syncthreads();
        for (int i = j + tid; i < KB; i += kGroupSolveThreads) A[(size_t)i * KB + j] *= inv;       // column j of L (diagonal: sqrt d)
        __syncthreads();
        // trailing update of the lower triangle: A[i][k] -= L[i][j] L[k][j], j < k <= i
        const int n = KB - j - 1;
        for (int u = tid; u < n * n; u += kGroupSolveThreads) {
            const int i = j + 1 + u / n, k = j + 1 + u % n;
            if (k <= i) A[(size_t)i * KB + k] -= A[(size_t)i * KB + j] * A[(size_t)k * KB + j];
        }
        __syncthreads();
    }
    __syncthreads();
    if (!failed) {
        // L z = b, then L^T s = z: short dependent chains, one thread
        if (tid == 0) {
            for (int i = 0; i < KB; i++) {
                float acc = b[i];
                for (int k = 0; k < i; k++) acc -= A[(size_t)i * KB + k] * sol[k];
                sol[i] = acc / A[(size_t)i * KB + i];
            }
            for (int i = KB - 1; i >= 0; i--) {
                float acc = sol[i];
                for (int k = i + 1; k < KB; k++) acc -= A[(size_t)k * KB + i] * sol[k];
                sol[i] = acc / A[(size_t)i * KB + i];
            }
        }
    } else {
        for (int i = tid; i < KB; i += kGroupSolveThreads) sol[i] = 1.0f;
    }
    __syncthreads();
    // new gain = old gain * s rounded to fp16; the block is rescaled by the ratio of the two fp16 gains
    const size_t row = (size_t)(row0 + c);
    for (int u = tid; u < KB * 24; u += kGroupSolveThreads) {
        const int p = u / 24;
        const float g_old = __half2float(__ushort_as_half(gain[row * KB + p]));
        const float g_new = __half2float(__float2half_rn(g_old * sol[p]));
        const float ratio = g_old != 0.0f ? g_new / g_old : 0.0f;
        Wq[row * ldw + u] *= ratio;
    }
    __syncthreads();
    for (int p = tid; p < KB; p += kGroupSolveThreads) {
        const float g_old = __half2float(__ushort_as_half(gain[row * KB + p]));
        gain[row * KB + p] = __half_as_ushort(__float2half_rn(g_old * sol[p]));
        if (s_out) s_out[row * KB + p] = sol[p];
    }
}

}  // namespace
