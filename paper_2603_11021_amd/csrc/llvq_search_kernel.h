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
// One workgroup handles one input vector at a time: a thread takes one Golay word, sorts once for the odd classes
// and once for the even classes of the word's weight, and then every class costs 24 multiply-adds whose class
// coefficients arrive in scalar registers (wave-uniform loads).  The workgroup's best (score, class, word) is
// then turned back into coordinates by the first 24 lanes.
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

constexpr int kSearchThreads = 1024;

template <int METRIC>
__global__ void __launch_bounds__(kSearchThreads) search_kernel(const llvq::SearchRec* __restrict__ recs, llvq::SearchLayout lay,
                                                                 const uint32_t* __restrict__ words, const float* __restrict__ w_in,
                                                                 size_t ldw, size_t n, int8_t* __restrict__ pts,
                                                                 float* __restrict__ score_out) {
    __shared__ float s_score[kSearchThreads / 64];
    __shared__ uint32_t s_id[kSearchThreads / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    for (size_t v = blockIdx.x; v < n; v += gridDim.x) {
        // the input vector is the same for every thread: it lives in scalar registers
        float wv[24];
        uint32_t negmask = 0;
#pragma unroll
        for (int i = 0; i < 24; i++) {
            wv[i] = w_in[ldw * v + i];
            negmask |= (wv[i] < 0.0f ? 1u : 0u) << i;
        }
        ScoredId best = {-INFINITY, 0u};
        for (int r = 0; r < 4096 / kSearchThreads; r++) {
            const uint32_t u = threadIdx.x + kSearchThreads * r;
            const uint32_t c = words[u];
            // ---- odd classes: every Golay word ------------------------------------------------------------
            {
                float y[24];
#pragma unroll
                for (int i = 0; i < 24; i++) y[i] = __uint_as_float(__float_as_uint(wv[i]) ^ (((c >> i) & 1u) << 31));
                sort_network<24>(y, [](float& a, float& b) { const float hi = fmaxf(a, b), lo = fminf(a, b); a = hi; b = lo; });
                // the record of the next class is requested (scalar loads) before the current one is multiplied
                llvq::SearchRec nxt = recs[0];
                for (uint32_t j = 0; j < lay.n_odd; j++) {
                    const llvq::SearchRec R = nxt;
                    nxt = recs[min(j + 1, lay.n_odd - 1)];
                    float acc = 0.0f;
#pragma unroll
                    for (int k = 0; k < 24; k++) acc = fmaf(R.coef[k], y[k], acc);
                    const ScoredId cand = {fmaf(acc, R.mul[METRIC], R.bias[METRIC]), j | (u << 9)};
                    if (cand.score > best.score) best = cand;
                }
            }
            // ---- even classes of the word's weight ----------------------------------------------------------
            {
                uint32_t key[24];
#pragma unroll
                for (int i = 0; i < 24; i++) key[i] = (__float_as_uint(wv[i]) & 0x7FFFFFFFu) | (((c >> i) & 1u) << 31);
                // as unsigned integers: positions of the word first, each part by descending |w|
                sort_network<24>(key, [](uint32_t& a, uint32_t& b) { const uint32_t hi = max(a, b), lo = min(a, b); a = hi; b = lo; });
                float e[24];
#pragma unroll
                for (int i = 0; i < 24; i++) e[i] = __uint_as_float(key[i] & 0x7FFFFFFFu);
                const uint32_t wt = (uint32_t)__popc(c);
                const int grp = wt == 0 ? 0 : (wt == 8 ? 1 : (wt == 12 ? 2 : (wt == 16 ? 3 : 4)));
                const float xmin1 = wt == 0 ? 0.0f : (wt == 8 ? e[7] : (wt == 12 ? e[11] : (wt == 16 ? e[15] : e[23])));
                const uint32_t negpar = (uint32_t)__popc(c & negmask) & 1u;
                // the repair applies when negpar != kappa: two per-thread values, the class picks one
                const float pen_k0 = negpar ? xmin1 : 0.0f, pen_k1 = negpar ? 0.0f : xmin1;
                for (int g = 0; g < 5; g++) {
                    if (!__builtin_amdgcn_ballot_w64(grp == g)) continue;            // no lane of this wave has that weight
                    const uint32_t j0 = lay.even_first[g], j1 = j0 + lay.even_count[g];
                    if (j0 == j1) continue;
                    llvq::SearchRec nxt = recs[j0];
                    for (uint32_t j = j0; j < j1; j++) {
                        const llvq::SearchRec R = nxt;
                        nxt = recs[min(j + 1, j1 - 1)];
                        float acc = 0.0f;
#pragma unroll
                        for (int k = 0; k < 24; k++) acc = fmaf(R.coef[k], e[k], acc);
                        acc = fmaf(-R.amin2, R.kappa ? pen_k1 : pen_k0, acc);
                        const ScoredId cand = {fmaf(acc, R.mul[METRIC], R.bias[METRIC]), j | (u << 9)};
                        if (grp == g && cand.score > best.score) best = cand;
                    }
                }
            }
        }
        // ---- best of the workgroup ---------------------------------------------------------------------------
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
            ScoredId b = {lane < kSearchThreads / 64 ? s_score[lane] : -INFINITY, lane < kSearchThreads / 64 ? s_id[lane] : 0xFFFFFFFFu};
#pragma unroll
            for (int off = 8; off > 0; off >>= 1) {
                ScoredId o;
                o.score = __shfl_xor(b.score, off);
                o.id = __shfl_xor(b.id, off);
                b = better(b, o);
            }
            b.score = __shfl(b.score, 0);
            b.id = __shfl(b.id, 0);
            // ---- the winner's coordinates: lane i = position i ------------------------------------------------
            const uint32_t j = b.id & 511u, u = b.id >> 9;
            const uint32_t c = words[u];
            const llvq::SearchRec& R = recs[j];
            const int i = lane < 24 ? lane : 23;
            const float wi = w_in[ldw * v + i];
            const uint32_t ci = (c >> i) & 1u;
            int x;
            if (j < lay.n_odd) {
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
            if (lane == 0 && score_out) score_out[v] = b.score;
        }
        __syncthreads();
    }
}

// One step of the block-wise loop of paper App. B (Alg. 1): for every row the block v = W[row][0..23] has been
// given its nearest direction x (pts); the block is replaced by g * x / ||x|| with g = ||v|| rounded to fp16 (the
// norm-preserving "gain reset" of paper Sec. 3.3), and the error E = v - g x/||x|| is kept for the propagation.
__global__ void retract_kernel(float* __restrict__ W, size_t ldw, const int8_t* __restrict__ pts, int N,
                               float* __restrict__ E, uint16_t* __restrict__ gain, size_t gain_stride) {
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
    const __half gh = __float2half_rn(sqrtf(n2));
    const float scale = __half2float(gh) / sqrtf(x2);
#pragma unroll
    for (int i = 0; i < 24; i++) {
        const float q = scale * x[i];
        W[(size_t)row * ldw + i] = q;
        E[(size_t)row * 24 + i] = v[i] - q;
    }
    gain[(size_t)row * gain_stride] = __half_as_ushort(gh);
}

}  // namespace
