// Matrix-core variant of the resident Lloyd kernel: one workgroup runs the whole iteration of
// one (task, k) unit (paper Algorithm 1, K-means.run(s_Theta, k); Sec. 3.3), with the
// -2 x.mu term of the squared distance evaluated by v_mfma_f32_32x32x16_f16.
//
// Screen:  score(c, i) = |mu'_c|^2 - 2 x'_i . mu'_c   (x', mu' centred by an integer offset)
//   A (32 centroids x K) = [ hi(w) | lo(w) ],  w = fl32(-2 mu'),  hi = f16(w), lo = f16(w - hi)
//   B (K x 32 rows)      = [ x' ; x' ]        (x' is a small integer: exact in f16)
//   C                    = |mu'_c|^2 broadcast along the rows of a centroid
// so every product is exact and only the fp32 accumulation and the 22-bit split of w round.
// Each lane then holds the scores of 16 centroids for one row; the epilogue takes the minimum
// (v_min3), and marks every centroid within the error bound of it (one subtract and one
// v_alignbit per score).  A row with a single mark is decided; the others are queued per wave
// and their marked centroids are re-evaluated in double in the oracle's operation order.
// Rows (as f16 B fragments), previous labels and the row norms stay in registers for all
// passes; centroids, integer sums and counts stay in LDS.
#include "cham_device.h"
#include "cham_internal.h"

namespace cham {

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int kRecCap = 64;          // flagged rows a wave can queue before it resolves them
constexpr float kPadBias = 1.0e30f;  // score of a padding centroid row: never the minimum

// Error bound of the matrix-core screen relative to (|x'|^2 + 2 max|mu'|^2), in units of 2^-24.
// Inputs: w = fl32(-2mu') and the bias are rounded once (1 each), hi + lo keeps 22 bits of w (4).
// Accumulation: each instruction adds 16 exact products to the running value; the hardware aligns
// the 17 addends to the largest and rounds once, which is modelled very generously as 18 units
// per instruction.  NS2 = number of chained instructions.
template <int NS2>
__device__ __forceinline__ float mfma_bound(float x2, float m2)
{
    constexpr float kE = 2.5f * (float)(18 * NS2 + 6) * 5.9604644775390625e-8f;
    return kE * (x2 + 2.0f * m2);
}

// LDS carve-up.  DK = padded knob count (16 or 32), KP = padded centroid count (32 or 64).
template <int DK>
struct MfmaLds {
    double *mu64T;      // [DK][KP]
    double *red;        // [16]
    half8 *afrag;       // [KP/32][2*DK/16][64]
    float *bias;        // [KP]
    int *S;             // [KP][DK]
    int *n;             // [KP]
    float *ojf;         // [DK]
    unsigned *m2bits;   // [1] (+pad)
    unsigned char *wave_base;   // per-wave regions follow
    static constexpr size_t kWaveBytes = ((size_t)kRecCap * DK * 2 + 512 * 8 + 512 * 2 + 512 + 512 * 4 + 15) / 16 * 16;
    __host__ __device__ static size_t bytes(int KP, int nwaves)
    {
        size_t b = sizeof(double) * DK * KP + sizeof(double) * 16;
        b += 16 * (size_t)(KP / 32) * (2 * DK / 16) * 64;
        b += sizeof(float) * KP + sizeof(int) * (size_t)KP * DK + sizeof(int) * KP + sizeof(float) * DK + 64;
        b = (b + 15) & ~(size_t)15;
        return b + kWaveBytes * nwaves;
    }
    __device__ MfmaLds(unsigned char *p, int KP)
    {
        mu64T = reinterpret_cast<double *>(p);  p += sizeof(double) * DK * KP;
        red = reinterpret_cast<double *>(p);    p += sizeof(double) * 16;
        afrag = reinterpret_cast<half8 *>(p);   p += 16 * (size_t)(KP / 32) * (2 * DK / 16) * 64;
        bias = reinterpret_cast<float *>(p);    p += sizeof(float) * KP;
        S = reinterpret_cast<int *>(p);         p += sizeof(int) * (size_t)KP * DK;
        n = reinterpret_cast<int *>(p);         p += sizeof(int) * KP;
        ojf = reinterpret_cast<float *>(p);     p += sizeof(float) * DK;
        m2bits = reinterpret_cast<unsigned *>(p);  p += 64;
        wave_base = reinterpret_cast<unsigned char *>((reinterpret_cast<uintptr_t>(p) + 15) & ~(uintptr_t)15);
    }
};

// Fragment position of (centroid c, part p in {hi, lo}, knob j): [mt][step][lane] half8, element i.
template <int DK>
__device__ __forceinline__ int afrag_index(int c, int part, int j, int &elem)
{
    constexpr int NS = DK / 16;
    const int mt = c >> 5, m = c & 31;
    const int step = part * NS + (j >> 4);
    const int h = (j & 15) >> 3;
    elem = j & 7;
    return (mt * (2 * NS) + step) * 64 + 32 * h + m;
}

// From the exact centroids build the A fragments, the bias column and the bound m2.
template <int DK>
__device__ __forceinline__ void derive_fragments(const MfmaLds<DK> &U, int k, int KP)
{
    for (int c = threadIdx.x; c < k; c += blockDim.x) {
        double b = 0.0;
#pragma unroll 4
        for (int j = 0; j < DK; ++j) {
            const double m = U.mu64T[(size_t)j * KP + c] - (double)U.ojf[j];
            b = __builtin_fma(m, m, b);
            const float w = (float)(-2.0 * m);
            const _Float16 hi = (_Float16)w;
            const _Float16 lo = (_Float16)(w - (float)hi);
            int e;
            int idx = afrag_index<DK>(c, 0, j, e);
            reinterpret_cast<_Float16 *>(U.afrag + idx)[e] = hi;
            idx = afrag_index<DK>(c, 1, j, e);
            reinterpret_cast<_Float16 *>(U.afrag + idx)[e] = lo;
        }
        U.bias[c] = (float)b;
        atomicMax(U.m2bits, __float_as_uint(__double2float_ru(b) * 1.0000005f));
    }
}

__device__ __forceinline__ float min3f(float a, float b, float c)
{
    return __builtin_fminf(__builtin_fminf(a, b), c);
}

// centroid index of score q (processing order: m-tile, then accumulator register) in half hh
__device__ __forceinline__ int centroid_of(int q, int hh)
{
    return 32 * (q >> 4) + 8 * ((q & 15) >> 2) + 4 * hh + (q & 3);
}


// Per-wave queue of flagged rows.  Every row of the wave can be queued (index + candidate masks
// of both lane halves); the first kRecCap queued rows also carry their knob values (f16,
// centred) in LDS, later ones are re-read from the packed row copy in global memory.
template <int DK>
struct WaveQueue {
    static constexpr int kRows = 512;                       // rows a wave owns at most
    static constexpr size_t kOffMask = (size_t)kRecCap * DK * 2;
    static constexpr size_t kOffPid = kOffMask + (size_t)kRows * 8;
    static constexpr size_t kOffLab = kOffPid + (size_t)kRows * 2;
    static constexpr size_t kOffX2 = kOffLab + (size_t)kRows;
    static constexpr size_t kBytes = (kOffX2 + (size_t)kRows * 4 + 15) / 16 * 16;
    unsigned char *base;
    __device__ explicit WaveQueue(unsigned char *wb) : base(wb) {}
    __device__ _Float16 *rec_x() const { return reinterpret_cast<_Float16 *>(base); }                    // [kRecCap][DK]
    __device__ unsigned *rec_mask() const { return reinterpret_cast<unsigned *>(base + kOffMask); }      // [kRows][2]
    __device__ unsigned short *rec_pid() const { return reinterpret_cast<unsigned short *>(base + kOffPid); }
    __device__ unsigned char *lab_res() const { return base + kOffLab; }                                  // [kRows]
    __device__ float *x2() const { return reinterpret_cast<float *>(base + kOffX2); }                     // [kRows]
};

// Resolve the queued rows of this wave: one row per lane, exact double distances to its marked
// centroids (four at a time, knobs ascending, no fused multiply-add), lowest index on ties.
// xh_wave points at the packed f16 copy of the wave's first row (uncentred values).
template <int DK>
__device__ __forceinline__ void resolve_queue(const WaveQueue<DK> &Q, int nrec, const double *mu64T,
                                              const float *ojf, int KP, int k, int d,
                                              const _Float16 *xh_wave)
{
    const int lane = threadIdx.x & 63;
    __builtin_amdgcn_wave_barrier();
    for (int r = lane; r < nrec; r += 64) {
        unsigned rem0 = Q.rec_mask()[r * 2 + 0], rem1 = Q.rec_mask()[r * 2 + 1];
        const int pid = Q.rec_pid()[r];
        double bs = __builtin_inf();
        int bc = 0x7fffffff;
        while (rem0 | rem1) {
            int cc[4];
            double ss[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                cc[q] = -1;
                ss[q] = 0.0;
                if (rem0) {
                    const int b = __clz((int)rem0);
                    rem0 &= ~(0x80000000u >> b);
                    cc[q] = centroid_of(b, 0);
                } else if (rem1) {
                    const int b = __clz((int)rem1);
                    rem1 &= ~(0x80000000u >> b);
                    cc[q] = centroid_of(b, 1);
                }
            }
            for (int j = 0; j < d; ++j) {
                float xf;
                if (r < kRecCap) xf = (float)Q.rec_x()[(size_t)r * DK + j] + ojf[j];
                else xf = (float)xh_wave[(size_t)pid * DK + j];
                const double xv = (double)xf;
                const double *row = mu64T + (size_t)j * KP;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const double tq = xv - row[cc[q] < 0 ? 0 : cc[q]];
                    ss[q] = ss[q] + tq * tq;
                }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (cc[q] >= 0 && (ss[q] < bs || (ss[q] == bs && cc[q] < bc))) {
                    bs = ss[q];
                    bc = cc[q];
                }
            }
        }
        Q.lab_res()[pid] = (unsigned char)(bc < k ? bc : 0);
    }
    __builtin_amdgcn_wave_barrier();
}

// Row-major f16 copy of X (one row = DK halfs, padded knobs zero): a lane fetches the eight knobs
// of a B fragment with one 16-byte load.
template <int DK>
__global__ void pack_rows_kernel(const uint8_t *__restrict__ X, int64_t ld, int d, int64_t n_rows,
                                 _Float16 *__restrict__ xh)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_rows) return;
#pragma unroll
    for (int g = 0; g < DK / 8; ++g) {
        half8 v;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int j = 8 * g + i;
            v[i] = j < d ? (_Float16)(float)X[(int64_t)j * ld + r] : (_Float16)0.0f;
        }
        *reinterpret_cast<half8 *>(xh + r * DK + 8 * g) = v;
    }
}

template <int DK, int NTW>
__global__ __launch_bounds__(512) void resident_mfma_kernel(const SweepArgs a)
{
    constexpr int NS = DK / 16;          // distinct B fragments per row
    constexpr int NS2 = 2 * NS;          // chained instructions per 32x32 tile
    extern __shared__ __align__(16) unsigned char smem[];
    const int KP = a.kmax > 32 ? 64 : 32;
    MfmaLds<DK> U(smem, KP);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int nwaves = blockDim.x >> 6;
    const int n32 = lane & 31;           // row within a 32-row tile
    const int h = lane >> 5;             // which half of the knob slots / centroid rows this lane holds

    const int u = blockIdx.x;
    const int ki = a.n_k - 1 - u / a.T;
    const int t = u % a.T;
    const int k = a.ks[ki];
    const int d = a.d;
    const int64_t r0 = a.task_off[t], r1 = a.task_off[t + 1];
    const int nrows = (int)(r1 - r0);
    const int64_t slot = (int64_t)t * a.n_k + ki;
    const int64_t crow = (int64_t)t * a.Ksum + a.koff[ki];
    uint8_t *labrow = a.labbuf + (int64_t)ki * a.ld;
    const bool two = k > 32;

    if (a.init_mode == 0 && a.ndist[t] < k) {
        for (int e = tid; e < k * d; e += blockDim.x) a.centroids[crow * d + e] = 0.0;
        for (int c = tid; c < k; c += blockDim.x) a.counts[crow + c] = 0;
        for (int64_t r = r0 + tid; r < r1; r += blockDim.x) labrow[r] = 0;
        if (tid == 0) {
            a.status[slot] = 1;
            a.inertia[slot] = 0.0;
        }
        if (a.trace)
            for (int e = tid; e <= a.n_iter; e += blockDim.x) a.trace[slot * (a.n_iter + 1) + e] = 0.0;
        return;
    }

    // per-wave queue of flagged rows
    WaveQueue<DK> Q(U.wave_base + MfmaLds<DK>::kWaveBytes * wave);

    // ---- set-up
    for (int e = tid; e < DK * KP; e += blockDim.x) U.mu64T[e] = 0.0;
    for (int e = tid; e < KP * DK; e += blockDim.x) U.S[e] = 0;
    for (int c = tid; c < KP; c += blockDim.x) {
        U.n[c] = 0;
        U.bias[c] = kPadBias;
    }
    {
        half8 z;
#pragma unroll
        for (int i = 0; i < 8; ++i) z[i] = (_Float16)0.0f;
        for (int e = tid; e < (KP / 32) * NS2 * 64; e += blockDim.x) U.afrag[e] = z;
    }
    if (tid == 0) *U.m2bits = 0u;
    __syncthreads();
    for (int e = tid; e < k * d; e += blockDim.x) {
        const int c = e / d, j = e % d;
        double v;
        if (a.init_mode == 0) {
            const int row = a.init_rows[(int64_t)t * a.kmax + c];
            v = (double)a.X[(int64_t)j * a.ld + r0 + row];
        } else {
            v = a.init_centroids[(crow + c) * d + j];
        }
        U.mu64T[(size_t)j * KP + c] = v;
    }
    __syncthreads();
    if (tid < DK) {
        float o = 0.0f;
        if (tid < d) {
            double s = 0.0;
            for (int c = 0; c < k; ++c) s += U.mu64T[(size_t)tid * KP + c];
            double m = rint(s / (double)k);
            m = m < 0.0 ? 0.0 : (m > 255.0 ? 255.0 : m);
            o = (float)m;
        }
        U.ojf[tid] = o;
    }
    __syncthreads();
    derive_fragments<DK>(U, k, KP);

    // ---- this lane's rows as B fragments (kept in registers for every pass)
    const _Float16 *xh_wave = reinterpret_cast<const _Float16 *>(a.xh) + (r0 + (int64_t)wave * NTW * 32) * DK;
    half8 B[NTW][NS];
    uint32_t prevpack[(NTW + 3) / 4];
#pragma unroll
    for (int q = 0; q < (NTW + 3) / 4; ++q) prevpack[q] = 0;
    half8 off8[NS];
#pragma unroll
    for (int f = 0; f < NS; ++f)
#pragma unroll
        for (int i = 0; i < 8; ++i) off8[f][i] = (_Float16)U.ojf[16 * f + 8 * h + i];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
        const int pid = (wave * NTW + nt) * 32 + n32;
        const bool live = pid < nrows;
        const int64_t prow = live ? (int64_t)(nt * 32 + n32) : 0;       // a valid row of the wave or row 0
#pragma unroll
        for (int f = 0; f < NS; ++f) {
            half8 v = *reinterpret_cast<const half8 *>(xh_wave + prow * DK + 16 * f + 8 * h);
            if ((wave * NTW) * 32 >= nrows) v = off8[f];                // wave owns no row at all
            v = v - off8[f];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if (!live || 16 * f + 8 * h + i >= d) v[i] = (_Float16)0.0f;
            }
            B[nt][f] = v;
        }
    }
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
        float part = 0.0f;
#pragma unroll
        for (int f = 0; f < NS; ++f)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float v = (float)B[nt][f][i];
                part = __builtin_fmaf(v, v, part);
            }
        part = part + __shfl_xor(part, 32, 64);
        if (h == 0) Q.x2()[nt * 32 + n32] = part;
    }
    __syncthreads();

    double loss = 0.0;
    for (int it = 0; it <= a.n_iter; ++it) {
        const bool final_pass = (it == a.n_iter);
        const bool want_dist = final_pass || (a.trace != nullptr);
        const float m2 = __uint_as_float(*U.m2bits);

        // A fragments of this pass
        half8 A0[NS2], A1[NS2];
#pragma unroll
        for (int s = 0; s < NS2; ++s) {
            A0[s] = U.afrag[s * 64 + lane];
            A1[s] = two ? U.afrag[(NS2 + s) * 64 + lane] : A0[s];
        }

        uint32_t newpack[(NTW + 3) / 4];
#pragma unroll
        for (int q = 0; q < (NTW + 3) / 4; ++q) newpack[q] = 0;
        uint32_t flagged_tiles = 0;
        int nrec = 0;

#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            const int tile_first = (wave * NTW + nt) * 32;
            if (tile_first >= nrows) continue;            // wave-uniform
            float16v acc0, acc1;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 b0 = *reinterpret_cast<const float4 *>(U.bias + 8 * g + 4 * h);
                acc0[4 * g + 0] = b0.x; acc0[4 * g + 1] = b0.y; acc0[4 * g + 2] = b0.z; acc0[4 * g + 3] = b0.w;
            }
#pragma unroll
            for (int s = 0; s < NS2; ++s)
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A0[s], B[nt][s % NS], acc0, 0, 0, 0);
            float best = min3f(acc0[0], acc0[1], acc0[2]);
#pragma unroll
            for (int i = 3; i < 15; i += 2) best = min3f(best, acc0[i], acc0[i + 1]);
            best = __builtin_fminf(best, acc0[15]);
            if (two) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 b1 = *reinterpret_cast<const float4 *>(U.bias + 32 + 8 * g + 4 * h);
                    acc1[4 * g + 0] = b1.x; acc1[4 * g + 1] = b1.y; acc1[4 * g + 2] = b1.z; acc1[4 * g + 3] = b1.w;
                }
#pragma unroll
                for (int s = 0; s < NS2; ++s)
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A1[s], B[nt][s % NS], acc1, 0, 0, 0);
#pragma unroll
                for (int i = 0; i < 16; i += 2) best = min3f(best, acc1[i], acc1[i + 1]);
            }
            best = __builtin_fminf(best, __shfl_xor(best, 32, 64));
            const float thr = best + mfma_bound<NS2>(Q.x2()[nt * 32 + n32], m2);

            // bit (31 - q) of `far` is set when score q is above the threshold
            uint32_t far = 0;
#pragma unroll
            for (int i = 0; i < 16; ++i)
                far = __builtin_amdgcn_alignbit(far, __float_as_uint(thr - acc0[i]), 31);
            if (two) {
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    far = __builtin_amdgcn_alignbit(far, __float_as_uint(thr - acc1[i]), 31);
            } else {
                far = (far << 16) | 0xFFFFu;
            }
            const uint32_t cand = ~far;
            const uint32_t cand_o = (uint32_t)__shfl_xor((int)cand, 32, 64);
            const int total = __popc(cand) + __popc(cand_o);
            const bool live = (tile_first + n32) < nrows;
            const bool flagged = live && total != 1;
            const int hh = cand ? h : 1 - h;
            const int q = __clz((int)(cand ? cand : cand_o));
            const int lab = centroid_of(q & 31, hh);
            newpack[nt >> 2] |= (uint32_t)(flagged ? 0 : lab) << (8 * (nt & 3));

            const uint64_t fm = __ballot(flagged) & 0xFFFFFFFFull;
            if (fm) {
                flagged_tiles |= flagged ? (1u << nt) : 0u;
                if (flagged) {
                    const int rs = nrec + __popcll(fm & ((1ull << n32) - 1ull));
                    if (rs < kRecCap) {
#pragma unroll
                        for (int f = 0; f < NS; ++f)
                            *reinterpret_cast<half8 *>(Q.rec_x() + (size_t)rs * DK + 16 * f + 8 * h) = B[nt][f];
                    }
                    Q.rec_mask()[rs * 2 + h] = cand;
                    if (h == 0) Q.rec_pid()[rs] = (unsigned short)(nt * 32 + n32);
                }
                nrec += __popcll(fm);
            }
            __builtin_amdgcn_sched_barrier(0);   // keep one tile's accumulators live at a time
        }
        if (nrec) resolve_queue<DK>(Q, nrec, U.mu64T, U.ojf, KP, k, d, xh_wave);

        // label changes -> integer sums and counts (only rows whose label changed touch LDS)
        double part = 0.0;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            const int pid = (wave * NTW + nt) * 32 + n32;
            if (pid >= nrows) continue;
            int cur = (newpack[nt >> 2] >> (8 * (nt & 3))) & 0xFF;
            if ((flagged_tiles >> nt) & 1u) cur = Q.lab_res()[nt * 32 + n32];
            const int prev = (prevpack[nt >> 2] >> (8 * (nt & 3))) & 0xFF;
            if (it == 0 || cur != prev) {
#pragma unroll
                for (int f = 0; f < NS; ++f) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int j = 16 * f + 8 * h + i;
                        if (j < d) {
                            const int xi = (int)((float)B[nt][f][i] + U.ojf[j]);
                            atomicAdd(&U.S[cur * DK + j], xi);
                            if (it > 0) atomicSub(&U.S[prev * DK + j], xi);
                        }
                    }
                }
                if (h == 0) {
                    atomicAdd(&U.n[cur], 1);
                    if (it > 0) atomicSub(&U.n[prev], 1);
                }
                prevpack[nt >> 2] = (prevpack[nt >> 2] & ~(0xFFu << (8 * (nt & 3)))) | ((uint32_t)cur << (8 * (nt & 3)));
            }
            if (want_dist && h == 0) labrow[r0 + pid] = (uint8_t)cur;
        }
        __syncthreads();

        if (want_dist) {
            // exact loss of this pass: every row against its centroid, double, knobs ascending
            const int64_t g0 = r0 & ~(int64_t)3;
            for (int64_t g = g0 + (int64_t)tid * 4; g < r1; g += (int64_t)blockDim.x * 4) {
                const uint32_t lw = *reinterpret_cast<const uint32_t *>(labrow + g);
                double s4[4] = {0.0, 0.0, 0.0, 0.0};
                for (int j = 0; j < d; ++j) {
                    const uint32_t w = *reinterpret_cast<const uint32_t *>(a.X + (int64_t)j * a.ld + g);
                    const double *row = U.mu64T + (size_t)j * KP;
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const int c = (lw >> (8 * p)) & 0xFF;
                        const double tq = (double)((w >> (8 * p)) & 0xFFu) - row[c < k ? c : 0];
                        s4[p] = s4[p] + tq * tq;
                    }
                }
#pragma unroll
                for (int p = 0; p < 4; ++p)
                    if (g + p >= r0 && g + p < r1) part = part + s4[p];
            }
            const double ws = wave_sum(part);
            if (lane == 0) U.red[wave] = ws;
            __syncthreads();
            if (tid == 0) {
                double s = 0.0;
                for (int w = 0; w < nwaves; ++w) s = s + U.red[w];
                loss = s;
                if (a.trace) a.trace[slot * (a.n_iter + 1) + it] = s;
            }
        }

        if (!final_pass) {
            if (tid == 0) *U.m2bits = 0u;
            for (int e = tid; e < k * d; e += blockDim.x) {
                const int c = e / d, j = e % d;
                const int cnt = U.n[c];
                if (cnt > 0) U.mu64T[(size_t)j * KP + c] = (double)U.S[c * DK + j] / (double)cnt;
            }
            __syncthreads();
            derive_fragments<DK>(U, k, KP);
            __syncthreads();
        }
    }

    for (int e = tid; e < k * d; e += blockDim.x) {
        const int c = e / d, j = e % d;
        a.centroids[(crow + c) * d + j] = U.mu64T[(size_t)j * KP + c];
    }
    for (int c = tid; c < k; c += blockDim.x) a.counts[crow + c] = U.n[c];
    if (tid == 0) {
        a.status[slot] = 0;
        a.inertia[slot] = loss;
    }
}

template <int DK, int NTW>
hipError_t launch_mfma_t(const SweepArgs &a, int nwaves, hipStream_t s)
{
    const int KP = a.kmax > 32 ? 64 : 32;
    const size_t lds = MfmaLds<DK>::bytes(KP, nwaves);
    auto kern = resident_mfma_kernel<DK, NTW>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const unsigned units = (unsigned)a.T * (unsigned)a.n_k;
    hipLaunchKernelGGL(kern, dim3(units), dim3(nwaves * 64), lds, s, a);
    return hipGetLastError();
}

}  // namespace

bool mfma_path_fits(int d, int kmax, int64_t n_max)
{
    return d >= 1 && d <= 32 && kmax <= 64 && n_max <= 4096;
}

hipError_t launch_mfma_sweep(const SweepArgs &a, int64_t n_max, int64_t n_total, hipStream_t s)
{
    const int ntw = n_max <= 1024 ? 4 : 16;
    int nwaves = (int)((n_max + 32 * ntw - 1) / (32 * ntw));
    if (nwaves < 1) nwaves = 1;
    if (nwaves > 8) nwaves = 8;
    const unsigned pb = (unsigned)((n_total + 255) / 256);
    if (a.d <= 16) {
        if (pb) hipLaunchKernelGGL(pack_rows_kernel<16>, dim3(pb), dim3(256), 0, s, a.X, a.ld, a.d, n_total,
                                   reinterpret_cast<_Float16 *>(a.xh));
        return ntw == 4 ? launch_mfma_t<16, 4>(a, nwaves, s) : launch_mfma_t<16, 16>(a, nwaves, s);
    }
    if (pb) hipLaunchKernelGGL(pack_rows_kernel<32>, dim3(pb), dim3(256), 0, s, a.X, a.ld, a.d, n_total,
                               reinterpret_cast<_Float16 *>(a.xh));
    return ntw == 4 ? launch_mfma_t<32, 4>(a, nwaves, s) : launch_mfma_t<32, 16>(a, nwaves, s);
}

}  // namespace cham
