// Device-side building blocks shared by the k-means kernels (gfx950, wave64).
//
// The assignment step of k-means (paper Sec. 3.3 / Algorithm 1, "K-means.run") is done in
// two stages so that labels equal those of a plain double-precision evaluation:
//   1. fp32 screen:  score(c) = |mu'_c|^2 - 2 x'.mu'_c  (x', mu' centred by an integer
//      offset per knob), best and second-best tracked per row;
//   2. every row whose best/second gap is inside the proven fp32 error bound is re-evaluated
//      by the whole wave in double, one centroid per lane, as sum_j ((double)x_j - mu_j)^2
//      with j ascending and no fused multiply-add, ties to the lowest cluster index.
// The library is compiled with -ffp-contract=off; fused operations are written explicitly.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cham {

constexpr int kWave = 64;
constexpr int kRowsPerThread = 4;          // byte knobs: one 32-bit load holds knob j of 4 consecutive rows

// LDS-resident description of the k centroids of one clustering.
struct CentroidView {
    const double *mu64T;   // [DP][kp]   exact centroids, transposed (lane c reads column c)
    const float  *wf;      // [k][DP+4]  fp32 screen: w_j = -2*mu'_j (j < DP), then b = |mu'|^2
    const float  *ojf;     // [DP]       centring offsets as floats (0 for padded knobs)
    float         m2;      // upper bound of max_c |mu'_c|^2
    int           kp;      // column stride of mu64T
    int           k;
};

__device__ __forceinline__ float readlane_f(float v, int lane)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// Butterfly arg-min over the wave on (value, index) pairs, lowest index on equal values.
// Every lane returns the same pair.
__device__ __forceinline__ void wave_argmin(double &s, int &c)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        double s2 = __shfl_xor(s, off, kWave);
        int c2 = __shfl_xor(c, off, kWave);
        bool take = (s2 < s) || (s2 == s && c2 < c);
        s = take ? s2 : s;
        c = take ? c2 : c;
    }
}

// Fixed-order sum of one double per lane; every lane returns the total.
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = v + __shfl_xor(v, off, kWave);
    return v;
}

// Relative size of the fp32 screening error: for DP fused multiply-adds on top of a rounded
// bias and rounded weights, |score_fp32 - score_exact| <= (DP + 2.1) * 2^-24 * (|x'|^2 + 2|mu'|^2).
// A decision is trusted when the best/second gap exceeds twice that; the factor 2.5 leaves
// 25 % headroom for the rounding of the bound itself.
template <int DP>
__device__ __forceinline__ float screen_bound(float x2, float m2)
{
    constexpr float kE = 2.5f * (float)(DP + 3) * 5.9604644775390625e-8f;
    return kE * (x2 + 2.0f * m2);
}

// Load knob values of R consecutive rows (rows g..g+R-1, g % R == 0) and centre them.  XT is the
// storage type of a knob value (one or two bytes); one load of R * sizeof(XT) bytes holds knob j
// of the R rows.  Padded knobs (j >= d) and rows of a group that is out of range read as zero.
template <typename XT, int DP, int R>
__device__ __forceinline__ void load_rows(const XT *__restrict__ X, int64_t ld, int d, int64_t g,
                                          bool in_range, const float *ojf, float (&xf)[R][DP],
                                          float (&x2)[R])
{
    constexpr int kBits = 8 * (int)sizeof(XT);
    constexpr int kWords = R * (int)sizeof(XT) / 4;      // 32-bit words per load: 1 or 2
    static_assert(kWords == 1 || kWords == 2, "a load is 4 or 8 bytes");
#pragma unroll
    for (int p = 0; p < R; ++p) x2[p] = 0.0f;
#pragma unroll
    for (int j = 0; j < DP; ++j) {
        uint32_t w[2] = {0u, 0u};
        float o = 0.0f;
        if (j < d) {
            o = ojf[j];
            if (in_range) {
                if constexpr (kWords == 1) {
                    w[0] = *reinterpret_cast<const uint32_t *>(X + (int64_t)j * ld + g);
                } else {
                    const uint2 v = *reinterpret_cast<const uint2 *>(X + (int64_t)j * ld + g);
                    w[0] = v.x;
                    w[1] = v.y;
                }
            }
        }
#pragma unroll
        for (int p = 0; p < R; ++p) {
            constexpr int kPerWord = 32 / kBits;
            const uint32_t raw = (w[p / kPerWord] >> (kBits * (p % kPerWord))) & ((1u << kBits) - 1u);
            float v = (float)raw - o;
            xf[p][j] = v;
            x2[p] = __builtin_fmaf(v, v, x2[p]);
        }
    }
}
template <int DP>
__device__ __forceinline__ void load_rows(const uint8_t *__restrict__ X, int64_t ld, int d, int64_t g,
                                          bool in_range, const float *ojf, float (&xf)[4][DP],
                                          float (&x2)[4])
{
    load_rows<uint8_t, DP, 4>(X, ld, d, g, in_range, ojf, xf, x2);
}

// Exact squared distance of this lane's row p to centroid c (the oracle's operation order).
template <int DP>
__device__ __forceinline__ double exact_dist(const float (&x)[DP], const CentroidView &L, int c)
{
    double s = 0.0;
    const double *col = L.mu64T + c;
#pragma unroll
    for (int j = 0; j < DP; ++j) {
        double t = (double)(x[j] + L.ojf[j]) - col[(size_t)j * L.kp];
        s = s + t * t;
    }
    return s;
}

// Nearest centroid of R rows per lane.  rowmask bit p = row p takes part.
// Returns labels; dist[p] is the exact distance to the assigned centroid when want_dist.
template <int DP, int R = 4>
__device__ __forceinline__ void assign_rows(const float (&xf)[R][DP], const float (&x2)[R],
                                            uint32_t rowmask, const CentroidView &L, bool force_exact,
                                            bool want_dist, int (&lab)[R], double (&dist)[R])
{
    const int lane = threadIdx.x & (kWave - 1);
    const int k = L.k;
    bool flag[R];
    if (!force_exact) {
        float best[R], second[R];
#pragma unroll
        for (int p = 0; p < R; ++p) {
            best[p] = __builtin_inff();
            second[p] = __builtin_inff();
            lab[p] = 0;
        }
        for (int c = 0; c < k; ++c) {
            const float4 *wrow = reinterpret_cast<const float4 *>(L.wf + (size_t)c * (DP + 4));
            float acc[R];
            const float b = wrow[DP / 4].x;
#pragma unroll
            for (int p = 0; p < R; ++p) acc[p] = b;
#pragma unroll
            for (int q = 0; q < DP / 4; ++q) {
                const float4 w = wrow[q];
#pragma unroll
                for (int p = 0; p < R; ++p) {
                    acc[p] = __builtin_fmaf(xf[p][4 * q + 0], w.x, acc[p]);
                    acc[p] = __builtin_fmaf(xf[p][4 * q + 1], w.y, acc[p]);
                    acc[p] = __builtin_fmaf(xf[p][4 * q + 2], w.z, acc[p]);
                    acc[p] = __builtin_fmaf(xf[p][4 * q + 3], w.w, acc[p]);
                }
            }
#pragma unroll
            for (int p = 0; p < R; ++p) {
                second[p] = __builtin_amdgcn_fmed3f(best[p], second[p], acc[p]);
                lab[p] = acc[p] < best[p] ? c : lab[p];
                best[p] = fminf(best[p], acc[p]);
            }
        }
#pragma unroll
        for (int p = 0; p < R; ++p) {
            const float e = screen_bound<DP>(x2[p], L.m2);
            flag[p] = ((rowmask >> p) & 1u) && !((second[p] - best[p]) > e);
        }
    } else {
#pragma unroll
        for (int p = 0; p < R; ++p) {
            flag[p] = (rowmask >> p) & 1u;
            lab[p] = 0;
        }
    }

    // wave-cooperative exact re-evaluation of the flagged rows
#pragma unroll
    for (int p = 0; p < R; ++p) {
        uint64_t m = __ballot(flag[p]);
        while (m) {
            const int l = __ffsll((unsigned long long)m) - 1;
            m &= m - 1;
            double bs = __builtin_inf();
            int bc = 0x7fffffff;
            for (int c0 = 0; c0 < k; c0 += kWave) {
                int c = c0 + lane;
                const int cc = c < k ? c : k - 1;
                const double *col = L.mu64T + cc;
                double s = 0.0;
#pragma unroll
                for (int j = 0; j < DP; ++j) {
                    const float xj = readlane_f(xf[p][j], l) + L.ojf[j];
                    double t = (double)xj - col[(size_t)j * L.kp];
                    s = s + t * t;
                }
                if (c >= k) {
                    s = __builtin_inf();
                    c = 0x7fffffff;
                }
                wave_argmin(s, c);
                if (s < bs) {
                    bs = s;
                    bc = c;
                }
            }
            if (lane == l) {
                lab[p] = bc < k ? bc : 0;      // bc stays unset only if every distance is NaN
                dist[p] = bs;
            }
        }
    }

    if (want_dist) {
#pragma unroll
        for (int p = 0; p < R; ++p)
            if (((rowmask >> p) & 1u) && !flag[p]) dist[p] = exact_dist<DP>(xf[p], L, lab[p]);
    }
}

// 64-bit FNV-1a over d knob values (one step per value) with the salted offset basis.
__device__ __forceinline__ uint64_t fnv_begin(uint64_t salt)
{
    return 0xCBF29CE484222325ULL ^ (salt * 0x9E3779B97F4A7C15ULL);
}
__device__ __forceinline__ uint64_t fnv_step(uint64_t h, uint32_t byte)
{
    return (h ^ (uint64_t)byte) * 0x100000001B3ULL;
}

}  // namespace cham
