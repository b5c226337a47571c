// Matrix-core variant of the resident Lloyd kernel: one workgroup runs the whole iteration of
// one (task, k) unit (paper Algorithm 1, K-means.run(s_Theta, k); Sec. 3.3), with the squared
// distance screened by v_mfma_f32_32x32x16_f16.
//
// Screen:  score(c, i) = |mu'_c|^2 - 2 x'_i . mu'_c   (x', mu' centred by an integer offset)
//   A (32 centroids x K) = [ hi(w) | lo(w) ],  w = fl32(-2 mu'),  hi = f16(w), lo = f16(w - hi)
//   B (K x 32 rows)      = [ x' ; x' ]        (x' is a small integer: exact in f16)
//   the last knob slot (always unused: d < DK) carries the bias: B = 256, A = hi/lo of |mu'_c|^2 / 256
// so every product is exact and only the fp32 accumulation and the 22-bit splits round.
// Each lane then holds the scores of 16 centroids for one row; the epilogue takes the minimum
// (v_min3) and marks every centroid within the error bound of it (one subtract and one
// v_alignbit per score).  A row with a single mark is decided; the others are queued per wave
// and their marked centroids are re-evaluated in double in the oracle's operation order.
// The matrix instructions of the next 32-row tile are issued between the epilogue pieces of the
// current one.  Rows (as f16 B fragments) and previous labels stay in registers for all passes;
// centroids, integer sums and counts stay in LDS; a row touches the sums only when its label
// changes (exact: the sums are integers), through a dense per-wave queue.
#include "cham_device.h"
#include "cham_internal.h"
#include "mfma_common.h"

namespace cham {

namespace {

#ifdef CHAM_KERNEL_TIMING
// Development aid (not built into the library): per-section cycle counts summed over waves.
__device__ unsigned long long g_timing[16];
__device__ unsigned long long g_pass[64 * 16];   // per pass index: tiles, resolve, sums, barrier, update, count-mode, waves
#define CHAM_T(var) const unsigned long long var = __builtin_readcyclecounter()
#define CHAM_TADD(slot, t0, t1) tacc[slot] += (t1) - (t0)
#define CHAM_TCOUNT(slot, v) tacc[slot] += (unsigned long long)(v)
#else
#define CHAM_T(var)
#define CHAM_TADD(slot, t0, t1)
#define CHAM_TCOUNT(slot, v)
#endif


// Cross-lane exchanges done in the vector ALU (DPP), no LDS round trip.
// xor_lanes<1|2|4>: the value held by lane ^ 1, 2 or 4.
template <int XOR>
__device__ __forceinline__ int dpp_xor_i32(int v)
{
    if (XOR == 1) return __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, false);      // quad_perm [1,0,3,2]
    if (XOR == 2) return __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, false);      // quad_perm [2,3,0,1]
    // lane ^ 4 = mirror within each group of eight lanes, then reverse within each quad
    const int m = __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, false);            // row_half_mirror
    return __builtin_amdgcn_update_dpp(0, m, 0x1B, 0xF, 0xF, false);                    // quad_perm [3,2,1,0]
}
template <int XOR>
__device__ __forceinline__ double dpp_xor_f64(double v)
{
    const long long b = __double_as_longlong(v);
    const int lo = dpp_xor_i32<XOR>((int)(b & 0xFFFFFFFFll));
    const int hi = dpp_xor_i32<XOR>((int)(b >> 32));
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
// maximum of a non-negative float over the wave: rotations within the 16-lane rows, then the four
// row results through scalar registers
__device__ __forceinline__ float wave_max_nonneg(float v)
{
    int b = __float_as_int(v);          // non-negative floats order like integers
    int o = __builtin_amdgcn_update_dpp(0, b, 0x128, 0xF, 0xF, false);    // row_ror:8
    b = b > o ? b : o;
    o = __builtin_amdgcn_update_dpp(0, b, 0x124, 0xF, 0xF, false);        // row_ror:4
    b = b > o ? b : o;
    o = __builtin_amdgcn_update_dpp(0, b, 0x122, 0xF, 0xF, false);        // row_ror:2
    b = b > o ? b : o;
    o = __builtin_amdgcn_update_dpp(0, b, 0x121, 0xF, 0xF, false);        // row_ror:1
    b = b > o ? b : o;
    const int r0 = __builtin_amdgcn_readlane(b, 0), r1 = __builtin_amdgcn_readlane(b, 16);
    const int r2 = __builtin_amdgcn_readlane(b, 32), r3 = __builtin_amdgcn_readlane(b, 48);
    const int m01 = r0 > r1 ? r0 : r1, m23 = r2 > r3 ? r2 : r3;
    return __int_as_float(m01 > m23 ? m01 : m23);
}

// LDS carve-up.  DK = padded knob count (16 or 32), KP = padded centroid count (32 or 64).
template <int DK>
struct MfmaLds {
    double *mu64T;      // [DK][KP]   exact centroids, transposed
    double *red;        // [16]       per-wave partial sums of the loss
    float *bias;        // [KP]       upper bound of |mu - o|^2 per centroid (0 for padding rows)
    half8 *afrag;       // [KP/32][2*DK/16][64]  A fragments: hi parts then lo parts
    int *S;             // [KP][DK+1] integer cluster sums (row stride DK + 1: rows of different clusters fall into different banks)
    int *n;             // [KP]       cluster sizes
    int *dirty;         // [KP]       pass in which the cluster last changed
    float *ojf;         // [DK]       centring offsets
    int *upd_stamp;     // [3]        1 + pass whose update last rewrote a centroid; last pass that changed a sum; broken-invariant flag
    unsigned char *wave_base;   // per-wave regions follow
    static constexpr size_t kWaveBytes =
        ((size_t)kRecCap * DK * 2 + 512 * 8 + 512 * 2 + 512 + 512 * 4 + 512 * 4 + 15) / 16 * 16;
    __host__ __device__ static size_t bytes(int KP, int nwaves)
    {
        size_t b = sizeof(double) * DK * KP + sizeof(double) * 16 + sizeof(float) * KP;
        b += 16 * (size_t)(KP / 32) * (2 * DK / 16) * 64;
        b += sizeof(int) * (size_t)KP * (DK + 1) + sizeof(int) * KP * 2 + sizeof(float) * DK + 16;
        b = (b + 15) & ~(size_t)15;
        return b + kWaveBytes * nwaves;
    }
    __device__ MfmaLds(unsigned char *base, int KP)
    {
        // plain offset arithmetic from the LDS base keeps every pointer provably in LDS
        size_t o = 0;
        mu64T = reinterpret_cast<double *>(base + o);  o += sizeof(double) * DK * KP;
        red = reinterpret_cast<double *>(base + o);    o += sizeof(double) * 16;
        bias = reinterpret_cast<float *>(base + o);    o += sizeof(float) * KP;
        afrag = reinterpret_cast<half8 *>(base + o);   o += 16 * (size_t)(KP / 32) * (2 * DK / 16) * 64;
        S = reinterpret_cast<int *>(base + o);         o += sizeof(int) * (size_t)KP * (DK + 1);
        n = reinterpret_cast<int *>(base + o);         o += sizeof(int) * KP;
        dirty = reinterpret_cast<int *>(base + o);     o += sizeof(int) * KP;
        ojf = reinterpret_cast<float *>(base + o);     o += sizeof(float) * DK;
        upd_stamp = reinterpret_cast<int *>(base + o); o += 16;
        o = (o + 15) & ~(size_t)15;
        wave_base = base + o;
    }
};

// Per-wave LDS region.  Every row of the wave can be queued (index + candidate masks of both lane
// halves); the first kRecCap queued rows also carry their knob values (f16, centred), later ones
// are re-read from the packed row copy in global memory.  The same storage then queues the label
// changes of the pass.
template <int DK>
struct WaveQueue {
    static constexpr int kRows = 512;                       // rows a wave owns at most
    static constexpr size_t kOffMask = (size_t)kRecCap * DK * 2;
    static constexpr size_t kOffPid = kOffMask + (size_t)kRows * 8;
    static constexpr size_t kOffLab = kOffPid + (size_t)kRows * 2;
    static constexpr size_t kOffX2 = kOffLab + (size_t)kRows;
    unsigned char *base;
    __device__ explicit WaveQueue(unsigned char *wb) : base(wb) {}
    __device__ _Float16 *rec_x() const { return reinterpret_cast<_Float16 *>(base); }                    // [kRecCap][DK]
    __device__ unsigned *rec_mask() const { return reinterpret_cast<unsigned *>(base + kOffMask); }      // [kRows][2]
    __device__ unsigned short *rec_pid() const { return reinterpret_cast<unsigned short *>(base + kOffPid); }
    __device__ unsigned char *lab_res() const { return base + kOffLab; }                                  // [kRows]
    __device__ float *x2() const { return reinterpret_cast<float *>(base + kOffX2); }                     // [kRows] bound scale: at least |x'|^2 + |tau|
    __device__ float *best() const { return reinterpret_cast<float *>(base + kOffX2 + (size_t)kRows * 4); }     // [kRows] smallest score of the measuring pass
};

// Resolve the queued rows of this wave: four lanes per row, each lane takes every fourth marked
// centroid of its row and evaluates the exact double distance (knobs ascending, no fused
// multiply-add); the four lanes then agree on the smallest distance, lowest index on ties.
// xh_wave points at the packed f16 copy of the wave's first row (uncentred values).
template <int DK, bool kAllInLds>
__device__ __forceinline__ void resolve_rows(const WaveQueue<DK> &Q, int nrec, const double *mu64T,
                                             const float *ojf, int KP, int k, int d,
                                             const _Float16 *xh_wave)
{
    const int lane = threadIdx.x & 63;
    const int q = lane & 3;
    __builtin_amdgcn_wave_barrier();
    for (int r0 = 0; r0 < nrec; r0 += 16) {
        const int r = r0 + (lane >> 2);
        const bool have = r < nrec;
        const int rr = have ? r : 0;
        unsigned rem0 = 0, rem1 = 0;
        if (have) {
            rem0 = Q.rec_mask()[r * 2 + 0];
            rem1 = Q.rec_mask()[r * 2 + 1];
        }
        const int pid = Q.rec_pid()[rr];
        // next marked centroid of the row, -1 when none is left
        auto pop = [&]() -> int {
            int c = -1;
            if (rem0) {
                const int b = __clz((int)rem0);
                rem0 &= ~(0x80000000u >> b);
                c = centroid_of(b, 0);
            } else if (rem1) {
                const int b = __clz((int)rem1);
                rem1 &= ~(0x80000000u >> b);
                c = centroid_of(b, 1);
            }
            return c;
        };
        for (int i = 0; i < q; ++i) pop();
        double bs = __builtin_inf();
        int bc = 0x7fffffff;
        while (__ballot((rem0 | rem1) != 0u)) {
            const int cc = pop();
            const int ci = cc < 0 ? 0 : cc;
            double ss = 0.0;
            // knobs in groups of 8; the loads of a group are independent and overlap
            for (int j0 = 0; j0 < d; j0 += 8) {
                half8 xq;
                if (kAllInLds || rr < kRecCap) {
                    xq = *reinterpret_cast<const half8 *>(Q.rec_x() + (size_t)rr * DK + j0);
                } else {
                    xq = *reinterpret_cast<const half8 *>(xh_wave + (size_t)pid * DK + j0);
                }
                const float4 oa = *reinterpret_cast<const float4 *>(ojf + j0);
                const float4 ob = *reinterpret_cast<const float4 *>(ojf + j0 + 4);
                const float of[8] = {oa.x, oa.y, oa.z, oa.w, ob.x, ob.y, ob.z, ob.w};
                double mu[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) mu[i] = mu64T[(size_t)(j0 + i) * KP + ci];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    // queued copies are centred; padded knobs are skipped (one of them carries the bias)
                    float xf = (kAllInLds || rr < kRecCap) ? (float)xq[i] + of[i] : (float)xq[i];
                    if (j0 + i >= d) xf = 0.0f;
                    const double tq = (double)xf - mu[i];
                    ss = ss + tq * tq;
                }
            }
            if (cc >= 0 && cc < k && (ss < bs || (ss == bs && cc < bc))) {
                bs = ss;
                bc = cc;
            }
            pop();
            pop();
            pop();
        }
        {
            const double os = dpp_xor_f64<1>(bs);
            const int oc = dpp_xor_i32<1>(bc);
            if (os < bs || (os == bs && oc < bc)) {
                bs = os;
                bc = oc;
            }
        }
        {
            const double os = dpp_xor_f64<2>(bs);
            const int oc = dpp_xor_i32<2>(bc);
            if (os < bs || (os == bs && oc < bc)) {
                bs = os;
                bc = oc;
            }
        }
        if (have && q == 0) Q.lab_res()[pid] = (unsigned char)(bc < k ? bc : 0);
    }
    __builtin_amdgcn_wave_barrier();
}

// A few queued rows (the usual case): two rows at a time, two marked centroids per row at a time,
// sixteen lanes per (row, centroid): every lane squares the differences of its one or two knobs,
// then one lane adds the d squares up in knob order (the only part that has to be serial) and the
// lanes of a row agree on the smallest distance, lowest index on ties.
template <int DK>
__device__ __forceinline__ void resolve_few(const WaveQueue<DK> &Q, int nrec, const double *mu64T,
                                            const float *ojf, int KP, int k, int d)
{
    const int lane = threadIdx.x & 63;
    const int slot = lane >> 4, jl = lane & 15;
    // [4][32] squares of one (row, centroid), in the upper half of the mask array (unused by <= 8 queued rows)
    double *sc = reinterpret_cast<double *>(Q.rec_mask() + 512) + slot * 32;
    __builtin_amdgcn_wave_barrier();
    for (int r0 = 0; r0 < nrec; r0 += 2) {
        const int r = r0 + (slot >> 1);
        const bool have = r < nrec;
        const int rr = have ? r : 0;
        unsigned rem0 = 0, rem1 = 0;
        if (have) {
            rem0 = Q.rec_mask()[r * 2 + 0];
            rem1 = Q.rec_mask()[r * 2 + 1];
        }
        const int pid = Q.rec_pid()[rr];
        // this lane's knobs of the row (the queued copy is centred; reserved and padded slots count as zero)
        float xa = 0.0f, xb = 0.0f;
        if (jl < d) xa = (float)Q.rec_x()[(size_t)rr * DK + jl] + ojf[jl];
        if (DK == 32 && jl + 16 < d) xb = (float)Q.rec_x()[(size_t)rr * DK + jl + 16] + ojf[jl + 16];
        auto pop = [&]() -> int {
            int c = -1;
            if (rem0) {
                const int b = __clz((int)rem0);
                rem0 &= ~(0x80000000u >> b);
                c = centroid_of(b, 0);
            } else if (rem1) {
                const int b = __clz((int)rem1);
                rem1 &= ~(0x80000000u >> b);
                c = centroid_of(b, 1);
            }
            return c;
        };
        if (slot & 1) pop();
        double bs = __builtin_inf();
        int bc = 0x7fffffff;
        while (__ballot((rem0 | rem1) != 0u)) {
            const int cc = pop();
            const int ci = cc < 0 ? 0 : cc;
            const double ta = (double)xa - mu64T[(size_t)jl * KP + ci];
            sc[jl] = ta * ta;
            if (DK == 32) {
                const double tb = (double)xb - mu64T[(size_t)(jl + 16) * KP + ci];
                sc[jl + 16] = tb * tb;
            }
            __builtin_amdgcn_wave_barrier();
            if (jl == 0) {
                // eight loads in flight at a time; slots from d on hold exact zeros
                double ss = 0.0;
                for (int j0 = 0; j0 < d; j0 += 8) {
                    double v[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[i] = sc[j0 + i];
#pragma unroll
                    for (int i = 0; i < 8; ++i) ss = ss + v[i];
                }
                if (cc >= 0 && cc < k && (ss < bs || (ss == bs && cc < bc))) {
                    bs = ss;
                    bc = cc;
                }
            }
            __builtin_amdgcn_wave_barrier();
            pop();
        }
        const double os = __shfl_xor(bs, 16, 64);
        const int oc = __shfl_xor(bc, 16, 64);
        if (os < bs || (os == bs && oc < bc)) {
            bs = os;
            bc = oc;
        }
        if (have && (lane & 31) == 0) Q.lab_res()[pid] = (unsigned char)(bc < k ? bc : 0);
    }
    __builtin_amdgcn_wave_barrier();
}

// The usual case (every queued row has its LDS copy) never touches global memory.
template <int DK>
__device__ __forceinline__ void resolve_queue(const WaveQueue<DK> &Q, int nrec, const double *mu64T,
                                              const float *ojf, int KP, int k, int d,
                                              const _Float16 *xh_wave)
{
    if (nrec <= 8) {
        resolve_few<DK>(Q, nrec, mu64T, ojf, KP, k, d);
    } else if (nrec <= kRecCap) {
        resolve_rows<DK, true>(Q, nrec, mu64T, ojf, KP, k, d, xh_wave);
    } else {
        resolve_rows<DK, false>(Q, nrec, mu64T, ojf, KP, k, d, xh_wave);
    }
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

// Apply queued label changes of this wave to the integer sums and counts: 256 / DK queued rows
// per step, one lane per (row, group of 4 knobs).  Entry word: cur | prev << 8, prev = 0xFF for a
// row that had no label yet.
template <int DK>
__device__ __forceinline__ void apply_changes(const WaveQueue<DK> &Q, int cnt, int *S, int *n, int *dirty,
                                              int *pass_dirty, const float *ojf, int d, int stamp)
{
    constexpr int LPR = DK / 4;              // lanes per row
    constexpr int EPI = 64 / LPR;            // rows per step
    const int lane = threadIdx.x & 63;
    const int j0 = 4 * (lane % LPR);
    const float4 o4 = *reinterpret_cast<const float4 *>(ojf + j0);
    const float of[4] = {o4.x, o4.y, o4.z, o4.w};
    if (lane == 0) *pass_dirty = stamp;          // this pass changes a sum: the centroids need their update
    __builtin_amdgcn_wave_barrier();
#pragma unroll 2
    for (int e0 = 0; e0 < cnt; e0 += EPI) {
        const int e = e0 + lane / LPR;
        if (e < cnt && j0 < d) {
            const unsigned w = Q.rec_mask()[e];
            typedef _Float16 half4 __attribute__((ext_vector_type(4)));
            const half4 xq = *reinterpret_cast<const half4 *>(Q.rec_x() + (size_t)e * DK + j0);
            const int cur = w & 0xFF, prev = (w >> 8) & 0xFF;
            const bool first = prev == 0xFF;
            int *sc = S + cur * (DK + 1) + j0;
            int *sp = S + (first ? cur : prev) * (DK + 1) + j0;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (j0 + i < d) {
                    const int xi = (int)((float)xq[i] + of[i]);
                    atomicAdd(sc + i, xi);
                    if (!first) atomicSub(sp + i, xi);
                }
            }
            if (j0 == 0) {
                atomicAdd(&n[cur], 1);
                dirty[cur] = stamp;
                if (!first) {
                    atomicSub(&n[prev], 1);
                    dirty[prev] = stamp;
                }
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// Centroid update for the clusters touched in this pass, all threads: item (c, q) owns knobs
// 4q..4q+3 of centroid c: mean = (double)S / (double)n, then the f16 hi/lo fragments of
// w = -2 (mu - o) (one 8-byte store each).  The DK/4 items of a centroid sit in adjacent lanes and
// add up |mu - o|^2 among themselves; the last of them owns the bias slot (knob slot DK - 3) and
// stores the sum / 256 there as hi/lo, and its rounded-up value for the error bound.  The two
// threshold slots (DK - 2, DK - 1) hold the constant 256.  A rewritten centroid is recorded in
// upd_stamp.
template <int DK>
__device__ __forceinline__ void update_centroids(const MfmaLds<DK> &U, int k, int KP, int d, int stamp, bool all)
{
    constexpr int NS = DK / 16, NS2 = 2 * NS, QN = DK / 4;
    typedef _Float16 half4 __attribute__((ext_vector_type(4)));
    const int items = k * QN;
    for (int base = 0; base < items; base += blockDim.x) {      // uniform trip count: every lane shuffles
        const int item = base + (int)threadIdx.x;
        const int c = item / QN, q = item % QN;
        bool act = item < items;
        int cnt = 0;
        if (act) {
            cnt = U.n[c];
            if (!all && (U.dirty[c] != stamp || cnt == 0)) act = false;   // an empty cluster keeps its centroid
        }
        half4 hi4 = {(_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f};
        half4 lo4 = hi4;
        double b = 0.0;
        if (act && 4 * q < d) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int j = 4 * q + i;
                double mu = U.mu64T[(size_t)j * KP + c];
                if (!all && j < d) {
                    mu = (double)U.S[c * (DK + 1) + j] / (double)cnt;
                    U.mu64T[(size_t)j * KP + c] = mu;
                }
                const double m = j < d ? mu - (double)U.ojf[j] : 0.0;
                b = __builtin_fma(m, m, b);
                const float w = (float)(-2.0 * m);
                const _Float16 hi = (_Float16)w;
                hi4[i] = hi;
                lo4[i] = (_Float16)(w - (float)hi);
            }
        }
        b = b + dpp_xor_f64<1>(b);
        b = b + dpp_xor_f64<2>(b);
        if (QN == 8) b = b + dpp_xor_f64<4>(b);
        if (act && (4 * q < d || q == QN - 1)) {
            if (q == QN - 1) {
                const float bs = (float)b * (1.0f / kBiasScale);
                const _Float16 bhi = (_Float16)bs;
                hi4[1] = bhi;
                lo4[1] = (_Float16)(bs - (float)bhi);
                hi4[2] = hi4[3] = (_Float16)kBiasScale;      // the two threshold slots
                lo4[2] = lo4[3] = (_Float16)0.0f;
                U.bias[c] = __double2float_ru(b) * 1.0000005f;
                if (!all) *U.upd_stamp = stamp + 1;
            }
            const int mt = c >> 5, m32 = c & 31;
            const int g = q >> 1, hh = g & 1, fstep = g >> 1, sub = q & 1;
            half4 *fh = reinterpret_cast<half4 *>(U.afrag + (mt * NS2 + fstep) * 64 + 32 * hh + m32) + sub;
            half4 *fl = reinterpret_cast<half4 *>(U.afrag + (mt * NS2 + NS + fstep) * 64 + 32 * hh + m32) + sub;
            *fh = hi4;
            *fl = lo4;
        }
    }
}

// Everything one workgroup does for its unit.  Units with more than 32 centroids use two 32-row
// m-tiles per row tile; otherwise the two accumulators alternate between row tiles.
template <int DK, int NTW>
__device__ __forceinline__ void run_unit(const SweepArgs &a, unsigned char *smem, int ki, int t, int k)
{
    const bool two = k > 32;
    constexpr int NS = DK / 16;          // distinct B fragments per row
    constexpr int NS2 = 2 * NS;          // chained instructions per 32x32 tile
    constexpr int CH = 16 / NS2;         // scores handled between two matrix instructions
    const int KP = a.kmax > 32 ? 64 : 32;
    MfmaLds<DK> U(smem, KP);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int nwaves = blockDim.x >> 6;
    const int n32 = lane & 31;           // row within a 32-row tile
    const int h = lane >> 5;             // which half of the knob slots / centroid rows this lane holds

    const int d = a.d;
    const int64_t r0 = a.task_off[t], r1 = a.task_off[t + 1];
    const int nrows = (int)(r1 - r0);
    const int64_t slot = (int64_t)t * a.n_k + ki;
    const int64_t crow = (int64_t)t * a.Ksum + a.koff[ki];
    uint8_t *labrow = a.labbuf + (int64_t)ki * a.ld;

    WaveQueue<DK> Q(U.wave_base + MfmaLds<DK>::kWaveBytes * wave);
    const int wave_row0 = wave * NTW * 32;                 // first row (task-relative) of this wave
    const bool wave_live = wave_row0 < nrows;              // the wave owns at least one row

    // The last three knob slots of the fragments are reserved (d <= DK - 3): slot DK - 3 carries the
    // bias (256 in B, |mu'|^2 / 256 as hi/lo in A), slots DK - 2 and DK - 1 a per-row threshold
    // (-tau / 256 as hi/lo in B, 256 in A), so that the scores come out as score - tau.
    constexpr int bstep = NS - 1, bhalf = 1, belem = 5;

    // ---- set-up
    for (int e = tid; e < DK * KP; e += blockDim.x) U.mu64T[e] = 0.0;
    for (int e = tid; e < KP * (DK + 1); e += blockDim.x) U.S[e] = 0;
    for (int c = tid; c < KP; c += blockDim.x) {
        U.n[c] = 0;
        U.dirty[c] = -1;
    }
    for (int c = tid; c < KP; c += blockDim.x) U.bias[c] = 0.0f;
    {
        half8 z;
#pragma unroll
        for (int i = 0; i < 8; ++i) z[i] = (_Float16)0.0f;
        for (int e = tid; e < (KP / 32) * NS2 * 64; e += blockDim.x) U.afrag[e] = z;
    }
    __syncthreads();
    // padding centroid rows (beyond k) carry a huge bias so that they never win
    for (int c = k + tid; c < KP; c += blockDim.x) {
        _Float16 *slot = reinterpret_cast<_Float16 *>(U.afrag + ((c >> 5) * NS2 + bstep) * 64 + 32 * bhalf + (c & 31)) + belem;
        slot[0] = (_Float16)kPadBiasHi;
        slot[1] = slot[2] = (_Float16)kBiasScale;
    }
    if (tid == 0) {
        U.upd_stamp[0] = -1;
        U.upd_stamp[1] = -1;      // last pass that changed a sum
        U.upd_stamp[2] = 0;       // set if a pass that must not change a label did
    }
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
    update_centroids<DK>(U, k, KP, d, 0, true);

    // ---- this lane's rows as B fragments (kept in registers for every pass)
    const _Float16 *xh_wave = reinterpret_cast<const _Float16 *>(a.xh) + (r0 + (wave_live ? wave_row0 : 0)) * DK;
    half8 B[NTW][NS];
    uint32_t prevpack[(NTW + 3) / 4];
#pragma unroll
    for (int q = 0; q < (NTW + 3) / 4; ++q) prevpack[q] = 0xFFFFFFFFu;   // 0xFF = row has no label yet
    {
        half8 off8[NS];
#pragma unroll
        for (int f = 0; f < NS; ++f)
#pragma unroll
            for (int i = 0; i < 8; ++i) off8[f][i] = (_Float16)U.ojf[16 * f + 8 * h + i];
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            const bool live = wave_live && (wave_row0 + nt * 32 + n32) < nrows;
            const int64_t prow = live ? (int64_t)(nt * 32 + n32) : 0;     // always a row of this task
#pragma unroll
            for (int f = 0; f < NS; ++f) {
                half8 v = off8[f];
                if (nrows > 0) v = *reinterpret_cast<const half8 *>(xh_wave + prow * DK + 16 * f + 8 * h);
                v = v - off8[f];
#pragma unroll
                for (int i = 0; i < 8; ++i)
                    if (!live || 16 * f + 8 * h + i >= d) v[i] = (_Float16)0.0f;
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
            // the bias slot: a constant for every live row (after the norm, which excludes it)
            const bool live = wave_live && (wave_row0 + nt * 32 + n32) < nrows;
            if (live && h == bhalf) {
#pragma unroll
                for (int f = 0; f < NS; ++f)
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        if (f == bstep && i == belem) B[nt][f][i] = (_Float16)kBiasScale;
            }
        }
    }
    __syncthreads();

    double loss = 0.0;
    const int rows_left = nrows - wave_row0 - n32;      // this lane's row of tile nt is in the task iff 32 nt < rows_left
    bool have_tau = false;      // the rows' threshold slots are valid for the current centroids
#ifdef CHAM_KERNEL_TIMING
    unsigned long long tacc[16] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#endif
    for (int it = 0; it <= a.n_iter; ++it) {
        const bool final_pass = (it == a.n_iter);
        const bool want_dist = final_pass || (a.trace != nullptr);
        CHAM_T(t_a);

        uint32_t newpack[(NTW + 3) / 4];
#pragma unroll
        for (int q = 0; q < (NTW + 3) / 4; ++q) newpack[q] = 0;
        uint32_t flagged_tiles = 0;
        int nrec = 0;

        // How this pass decides its rows (the same for every wave of the workgroup):
        //   kScreen   best score, threshold best + bound, one mark per score (always valid); the
        //             best score of every row is kept for a later measurement;
        //   kCount    no centroid has changed since the rows' thresholds tau were measured: a row
        //             keeps its label iff exactly one score lies below its tau (one sign bit per
        //             score); a row with several is queued with exactly those centroids.
        // The thresholds are measured at the start of the first pass that finds the centroids of
        // the pass before unchanged, from the best scores of that pass.
        enum { kScreen = 0, kCount = 2 };
        const bool changed_prev = it == 0 || __builtin_amdgcn_readfirstlane(*U.upd_stamp) == it;
        const int mode = changed_prev ? kScreen : kCount;
        const bool measure_now = !changed_prev && !have_tau;
        have_tau = !changed_prev;

        CHAM_TCOUNT(14, mode == kCount ? 1 : 0);
        if (wave_live) {
            // A fragments of this pass (the bias slot included) and the bound m2
            half8 A0[NS2], A1[NS2];
#pragma unroll
            for (int s = 0; s < NS2; ++s) {
                A0[s] = U.afrag[s * 64 + lane];
                A1[s] = two ? U.afrag[(NS2 + s) * 64 + lane] : A0[s];
            }
            float m2 = 0.0f;
            if (mode != kCount || measure_now) {
                m2 = wave_max_nonneg(lane < KP ? U.bias[lane] : 0.0f);
            }

            if (measure_now) {
                // Every row's threshold for the passes to come.  best = smallest computed
                // score - tau_old of the pass before (same centroids), bnd = the bound it was screened
                // with.  The new tau exceeds the true score of the row's centroid by more than the
                // screen errors of that pass and of the passes that use it, and a centroid that is
                // not counted later is farther than the row's centroid by more than those errors.
                // Lanes of the upper half own the slots.
#pragma unroll
                for (int nt = 0; nt < NTW; ++nt) {
                    const float best = Q.best()[nt * 32 + n32];
                    const float xs = Q.x2()[nt * 32 + n32];
                    const float bnd = mfma_bound<NS2>(xs, m2);
                    const float b6 = (float)B[nt][NS - 1][6], b7 = (float)B[nt][NS - 1][7];
                    const float tq = best - kBiasScale * (b6 + b7);                    // score with tau_old taken out
                    const float bnd2 = mfma_bound<NS2>(xs + 2.0f * __builtin_fabsf(tq) + 4.0f * bnd + 2.0f, m2) + 1.0e-4f;
                    // one screen error is at most 0.4 of a bound (mfma_bound = 2 errors x 1.25): tau lies above
                    // the measured best by this pass's error, the later passes' error and a quarter more
                    const float tau = tq + 0.5f * bnd + 0.5f * bnd2 + __builtin_fabsf(tq) * 9.5367431640625e-7f;
                    const float u = -tau * (1.0f / kBiasScale);
                    const _Float16 h6 = (_Float16)u;
                    const _Float16 h7 = (_Float16)(u - (float)h6);
                    if (h == bhalf) {
                        B[nt][NS - 1][6] = h6;
                        B[nt][NS - 1][7] = h7;
                        Q.x2()[nt * 32 + n32] = xs + __builtin_fabsf(tau) * 1.000001f + 1.0f;
                    }
                }
            }

            CHAM_T(t_a2);
            CHAM_TADD(10, t_a, t_a2);   // pass prologue (inside "tiles")
            float16v accA, accB;
            const float16v zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

            // one matrix instruction of the chain of a 32x32 tile
            auto mma = [&](float16v &acc, const half8 (&Af)[NS2], const half8 (&Bt)[NS], int s) {
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(Af[s], Bt[s % NS], s == 0 ? zero16 : acc, 0, 0, 0);
            };
            // mark scores [i0, i0 + CH): bit set = above the threshold (or padding)
            auto mark = [&](uint32_t &far, const float16v &acc, float thr, int i0) {
#pragma unroll
                for (int i = 0; i < CH; ++i)
                    far = __builtin_amdgcn_alignbit(far, __float_as_uint(thr - acc[i0 + i]), 31);
            };
            // sign bits of scores [i0, i0 + CH): bit set = score - tau below zero
            auto signs = [&](uint32_t &neg, const float16v &acc, int i0) {
#pragma unroll
                for (int i = 0; i < CH; ++i) neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(acc[i0 + i]), 31);
            };
            auto min16 = [&](const float16v &acc) {
                float b = __builtin_fminf(min3f(acc[0], acc[1], acc[2]), acc[3]);
                b = min3f(min3f(b, acc[4], acc[5]), acc[6], acc[7]);
                b = min3f(min3f(b, acc[8], acc[9]), acc[10], acc[11]);
                b = min3f(min3f(b, acc[12], acc[13]), acc[14], acc[15]);
                return b;
            };
            // decide or queue the rows of tile nt from the candidate mask of this lane half
            auto decide = [&](uint32_t far, int nt, bool keep) {
                const uint32_t cand = ~far;
                uint32_t cand_lo, cand_hi;
                both_halves(cand, cand_lo, cand_hi);
                const int total = __popc(cand_lo) + __popc(cand_hi);
                // compared afresh in every tile: sixteen hoisted lane masks cost more than sixteen compares
                int rl = rows_left;
                asm volatile("" : "+v"(rl));
                const bool live = nt * 32 < rl;
                const bool flagged = live && total != 1;
                if (keep) {
                    // the single candidate is the row's centroid of the pass before (rows outside the
                    // task carry 0xFF there already)
                    const uint32_t prev = prevpack[nt >> 2] & (0xFFu << (8 * (nt & 3)));
                    newpack[nt >> 2] |= flagged ? (0xFEu << (8 * (nt & 3))) : prev;
                } else {
                    const int hh = cand_lo ? 0 : 1;
                    const int q = __clz((int)(cand_lo ? cand_lo : cand_hi));
                    const int lab = centroid_of(q & 31, hh);
                    newpack[nt >> 2] |= (uint32_t)(!live ? 0xFF : (flagged ? 0xFE : lab)) << (8 * (nt & 3));
                }
                // the label is packed here and now: left to itself the compiler defers all of this to
                // the end of the pass and keeps both candidate masks of every tile live until then
                asm volatile("" : "+v"(newpack[nt >> 2]));
                const uint64_t fm = __ballot(flagged) & 0xFFFFFFFFull;
                if (fm) {
                    flagged_tiles |= flagged ? (1u << nt) : 0u;
                    if (flagged) {
                        const int rs = nrec + __popcll(fm & ((1ull << n32) - 1ull));
                        if (rs < kRecCap) {
#pragma unroll
                            for (int f = 0; f < NS; ++f) {
                                *reinterpret_cast<half8 *>(Q.rec_x() + (size_t)rs * DK + 16 * f + 8 * h) = B[nt][f];
                            }
                        }
                        // no candidate at all cannot happen with valid thresholds; if it does, every centroid is one
                        Q.rec_mask()[rs * 2 + h] = total ? cand : (two ? 0xFFFFFFFFu : 0xFFFF0000u);
                        if (h == 0) Q.rec_pid()[rs] = (unsigned short)(nt * 32 + n32);
                    }
                    nrec += __popcll(fm);
                }
            };
            if (mode == kCount) {
                // The scores come out as score - tau.  A row whose only negative score is its
                // centroid's keeps its label; a row with several is queued with exactly those
                // centroids as candidates (the nearest centroid is always among them).
                if (two) {
#pragma unroll
                    for (int s = 0; s < NS2; ++s) mma(accA, A0, B[0], s);
#pragma unroll
                    for (int s = 0; s < NS2; ++s) mma(accB, A1, B[0], s);
#pragma unroll
                    for (int nt = 0; nt < NTW; ++nt) {
                        constexpr int kLast = NTW - 1;
                        const int nx = nt < kLast ? nt + 1 : nt;
                        uint32_t neg = 0;
#pragma unroll
                        for (int s = 0; s < NS2; ++s) signs(neg, accA, s * CH);
                        // accA is consumed: its next chain runs under the sign collection of accB
#pragma unroll
                        for (int s = 0; s < NS2; ++s) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (nt < kLast) mma(accA, A0, B[nx], s);
                            __builtin_amdgcn_sched_barrier(0);
                            signs(neg, accB, s * CH);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        if (nt < kLast) {
#pragma unroll
                            for (int s = 0; s < NS2; ++s) mma(accB, A1, B[nx], s);
                        }
                        decide(~neg, nt, true);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else {
#pragma unroll
                    for (int s = 0; s < NS2; ++s) mma(accA, A0, B[0], s);
#pragma unroll
                    for (int nt = 0; nt < NTW; ++nt) {
                        constexpr int kLast = NTW - 1;
                        const int nx = nt < kLast ? nt + 1 : nt;
                        float16v &cur = (nt & 1) ? accB : accA;
                        float16v &nxt = (nt & 1) ? accA : accB;
                        uint32_t neg = 0;
#pragma unroll
                        for (int s = 0; s < NS2; ++s) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (nt < kLast) mma(nxt, A0, B[nx], s);
                            __builtin_amdgcn_sched_barrier(0);
                            signs(neg, cur, s * CH);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        decide((~neg << 16) | 0xFFFFu, nt, true);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            } else {
                float x2cur = Q.x2()[n32];
                if (two) {
                    // accA = centroids 0..31, accB = centroids 32..63 of the current tile
#pragma unroll
                    for (int s = 0; s < NS2; ++s) mma(accA, A0, B[0], s);
#pragma unroll
                    for (int s = 0; s < NS2; ++s) mma(accB, A1, B[0], s);
#pragma unroll
                    for (int nt = 0; nt < NTW; ++nt) {
                        constexpr int kLast = NTW - 1;
                        const int nx = nt < kLast ? nt + 1 : nt;
                        float best = min_halves(__builtin_fminf(min16(accA), min16(accB)));
                        const float thr = best + mfma_bound<NS2>(x2cur, m2);
                        if (nt < kLast) x2cur = Q.x2()[nx * 32 + n32];
                        uint32_t far = 0;
#pragma unroll
                        for (int s = 0; s < NS2; ++s) mark(far, accA, thr, s * CH);
                        // accA is consumed: its next chain runs under the marking of accB
#pragma unroll
                        for (int s = 0; s < NS2; ++s) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (nt < kLast) mma(accA, A0, B[nx], s);
                            __builtin_amdgcn_sched_barrier(0);
                            mark(far, accB, thr, s * CH);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        if (nt < kLast) {
#pragma unroll
                            for (int s = 0; s < NS2; ++s) mma(accB, A1, B[nx], s);
                        }
                        decide(far, nt, false);
                        if (h == 0) Q.best()[nt * 32 + n32] = best;
                        __builtin_amdgcn_sched_barrier(0);   // labels of this tile are packed before the next tile
                    }
                } else {
                    // one m-tile: the accumulators alternate, the next tile's chain runs under this epilogue
#pragma unroll
                    for (int s = 0; s < NS2; ++s) mma(accA, A0, B[0], s);
#pragma unroll
                    for (int nt = 0; nt < NTW; ++nt) {
                        constexpr int kLast = NTW - 1;
                        const int nx = nt < kLast ? nt + 1 : nt;
                        float16v &cur = (nt & 1) ? accB : accA;
                        float16v &nxt = (nt & 1) ? accA : accB;
                        float best = min_halves(min16(cur));
                        const float thr = best + mfma_bound<NS2>(x2cur, m2);
                        if (nt < kLast) x2cur = Q.x2()[nx * 32 + n32];
                        uint32_t far = 0;
#pragma unroll
                        for (int s = 0; s < NS2; ++s) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (nt < kLast) mma(nxt, A0, B[nx], s);
                            __builtin_amdgcn_sched_barrier(0);
                            mark(far, cur, thr, s * CH);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        far = (far << 16) | 0xFFFFu;
                        decide(far, nt, false);
                        if (h == 0) Q.best()[nt * 32 + n32] = best;
                        __builtin_amdgcn_sched_barrier(0);   // labels of this tile are packed before the next tile
                    }
                }
            }
        }
        CHAM_T(t_b);
        CHAM_TCOUNT(8, nrec);
        if (nrec) resolve_queue<DK>(Q, nrec, U.mu64T, U.ojf, KP, k, d, xh_wave);
        CHAM_TCOUNT(11, nrec ? 1 : 0);
        CHAM_T(t_c);

        // Labels of the rows that went through the queue replace their placeholders.
        if (wave_live && __ballot(flagged_tiles != 0u)) {
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt) {
                if ((flagged_tiles >> nt) & 1u) {
                    const uint32_t lab = Q.lab_res()[nt * 32 + n32];
                    newpack[nt >> 2] = (newpack[nt >> 2] & ~(0xFFu << (8 * (nt & 3)))) | (lab << (8 * (nt & 3)));
                }
            }
        }
        if (wave_live && want_dist) {
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt) {
                const int pid = wave_row0 + nt * 32 + n32;
                if (pid < nrows && h == 0) labrow[r0 + pid] = (uint8_t)((newpack[nt >> 2] >> (8 * (nt & 3))) & 0xFF);
            }
        }
        // Label changes -> queue of (previous, new, knob values) -> integer sums.  A row without a
        // label yet has previous = 0xFF; rows outside the task keep 0xFF and never change.  The
        // queue holds kRecCap rows; if a pass changes more (the first passes do), the tiles are
        // walked again from the first tile that did not fit.
        CHAM_T(t_c1);
        if (wave_live) {
            uint32_t diff[(NTW + 3) / 4];
            uint32_t any = 0;
#pragma unroll
            for (int q = 0; q < (NTW + 3) / 4; ++q) {
                diff[q] = newpack[q] ^ prevpack[q];
                any |= diff[q];
            }
            int start = __ballot(any != 0u) ? 0 : NTW;
            while (start < NTW) {
                int cnt = 0;
                int next_start = NTW;
#pragma unroll
                for (int nt = 0; nt < NTW; ++nt) {
                    if (nt < start || next_start != NTW) continue;
                    const bool changed = ((diff[nt >> 2] >> (8 * (nt & 3))) & 0xFFu) != 0u;
                    const uint64_t cm = __ballot(changed) & 0xFFFFFFFFull;
                    if (cm) {
                        if (cnt + 32 > kRecCap) {
                            next_start = nt;
                            continue;
                        }
                        if (changed) {
                            const int rs = cnt + __popcll(cm & ((1ull << n32) - 1ull));
#pragma unroll
                            for (int f = 0; f < NS; ++f)
                                *reinterpret_cast<half8 *>(Q.rec_x() + (size_t)rs * DK + 16 * f + 8 * h) = B[nt][f];
                            const uint32_t cur = (newpack[nt >> 2] >> (8 * (nt & 3))) & 0xFFu;
                            const uint32_t prev = (prevpack[nt >> 2] >> (8 * (nt & 3))) & 0xFFu;
                            if (h == 0) Q.rec_mask()[rs] = cur | (prev << 8);
                        }
                        cnt += __popcll(cm);
                    }
                }
                CHAM_TCOUNT(7, cnt);
                CHAM_T(t_p0);
                if (cnt) apply_changes<DK>(Q, cnt, U.S, U.n, U.dirty, U.upd_stamp + 1, U.ojf, d, it);
                if (cnt && mode == kCount && lane == 0) U.upd_stamp[2] = 1;
                CHAM_T(t_p1);
                CHAM_TADD(12, t_p0, t_p1);   // apply (inside "sums")
                start = next_start;
            }
#pragma unroll
            for (int q = 0; q < (NTW + 3) / 4; ++q) prevpack[q] = newpack[q];
        }
        if (want_dist) {
            // Exact loss of this pass from the rows in registers: (x - mu)^2 in double over the knobs
            // a lane holds (x = centred value + offset, exact), the two lanes of a row and all rows
            // added up afterwards.  Reserved slots are left out; padded slots are zero on both sides.
            double part = 0.0;
            if (wave_live) {
                float of[NS][8];
#pragma unroll
                for (int f = 0; f < NS; ++f)
#pragma unroll
                    for (int i = 0; i < 8; ++i) of[f][i] = U.ojf[16 * f + 8 * h + i];
#pragma unroll
                for (int nt = 0; nt < NTW; ++nt) {
                    const uint32_t lab = (newpack[nt >> 2] >> (8 * (nt & 3))) & 0xFFu;
                    const bool live = lab != 0xFFu;
                    const double *mc = U.mu64T + (live ? lab : 0u) + (size_t)(8 * h) * KP;
                    double s = 0.0;
#pragma unroll
                    for (int f = 0; f < NS; ++f)
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            float xf = (float)B[nt][f][i] + of[f][i];
                            if (f == NS - 1 && i >= belem) xf = h == bhalf ? 0.0f : xf;
                            const double tq = (double)xf - mc[(size_t)(16 * f + i) * KP];
                            s = s + tq * tq;
                        }
                    part = part + (live ? s : 0.0);
                }
            }
            const double ws = wave_sum(part);
            if (lane == 0) U.red[(it & 1) * 8 + wave] = ws;
        }
        // Once the centroids have stopped changing, a pass reads shared state only (fragments,
        // centroids) and writes nothing that another wave reads: identical inputs give identical
        // labels, so no sum can change and the waves need not meet until a pass that reports the
        // loss.  A label change in such a pass would mean the invariant is broken; it is recorded
        // and reported as status 2.
        const bool free_run = mode == kCount && !want_dist;
        CHAM_T(t_d);
        if (!free_run) __syncthreads();
        CHAM_T(t_e);

        if (want_dist && tid == 0) {
            double s = 0.0;
            for (int w = 0; w < nwaves; ++w) s = s + U.red[(it & 1) * 8 + w];
            loss = s;
            if (a.trace) a.trace[slot * (a.n_iter + 1) + it] = s;
        }

        CHAM_T(t_e2);
        CHAM_TADD(13, t_e, t_e2);    // exact loss (inside "loss/update")
        // A pass that moved no row leaves every sum as it was: no update, and no second barrier
        // (the flag is read after the barrier above; a wave that runs ahead can only overwrite it
        // with a later pass number, which reads the same).
        if (!free_run && !final_pass && __builtin_amdgcn_readfirstlane(U.upd_stamp[1]) == it) {
            update_centroids<DK>(U, k, KP, d, it, false);
            __syncthreads();
        }
        CHAM_T(t_f);
        CHAM_TADD(0, t_a, t_b);   // tiles
        if (mode == kCount) { CHAM_TADD(5, t_a, t_b); CHAM_TADD(6, t_a, t_f); }
        CHAM_TADD(1, t_b, t_c);   // resolve
        CHAM_TADD(2, t_c, t_d);   // sums
        CHAM_TADD(3, t_d, t_e);   // barrier wait
        CHAM_TADD(4, t_e, t_f);   // loss / update
        CHAM_TCOUNT(9, 1);
#ifdef CHAM_KERNEL_TIMING
        if (lane == 0 && it < 64) {
            atomicAdd(&g_pass[it * 16 + 0], t_b - t_a);
            atomicAdd(&g_pass[it * 16 + 1], t_c - t_b);
            atomicAdd(&g_pass[it * 16 + 2], t_d - t_c);
            atomicAdd(&g_pass[it * 16 + 3], t_e - t_d);
            atomicAdd(&g_pass[it * 16 + 4], t_f - t_e);
            atomicAdd(&g_pass[it * 16 + 5], (unsigned long long)(mode == kCount ? 1 : 0));
            atomicAdd(&g_pass[it * 16 + 6], 1ull);
            atomicAdd(&g_pass[it * 16 + 7], (unsigned long long)nrec);
            atomicAdd(&g_pass[it * 16 + 8], (unsigned long long)__popc(flagged_tiles));
        }
#endif
    }

#ifdef CHAM_KERNEL_TIMING
    if (lane == 0)
        for (int q = 0; q < 16; ++q) atomicAdd(&g_timing[q], tacc[q]);
#endif
    for (int e = tid; e < k * d; e += blockDim.x) {
        const int c = e / d, j = e % d;
        a.centroids[(crow + c) * d + j] = U.mu64T[(size_t)j * KP + c];
    }
    for (int c = tid; c < k; c += blockDim.x) a.counts[crow + c] = U.n[c];
    if (tid == 0) {
        a.status[slot] = U.upd_stamp[2] ? 2 : 0;
        a.inertia[slot] = loss;
    }
}

template <int DK, int NTW>
__global__ __launch_bounds__(512) void resident_mfma_kernel(const SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;

    // units in descending-k order so that the longest ones start first
    const int u = blockIdx.x;
    const int ki = a.ki_end - 1 - u / a.T;
    const int t = u % a.T;
    const int k = a.ks[ki];
    const bool skipped = a.done && a.done[t];     // the task's sweep stopped at a smaller k

    if (skipped || (a.init_mode == 0 && a.ndist[t] < k)) {
        // fewer than k distinct rows, or not needed any more: all outputs zero, status says which
        const int d = a.d;
        const int64_t r0 = a.task_off[t], r1 = a.task_off[t + 1];
        const int64_t slot = (int64_t)t * a.n_k + ki;
        const int64_t crow = (int64_t)t * a.Ksum + a.koff[ki];
        uint8_t *labrow = a.labbuf + (int64_t)ki * a.ld;
        for (int e = tid; e < k * d; e += blockDim.x) a.centroids[crow * d + e] = 0.0;
        for (int c = tid; c < k; c += blockDim.x) a.counts[crow + c] = 0;
        for (int64_t r = r0 + tid; r < r1; r += blockDim.x) labrow[r] = 0;
        if (tid == 0) {
            a.status[slot] = skipped ? 3 : 1;
            a.passes[slot] = 0;
            a.inertia[slot] = 0.0;
        }
        if (a.trace)
            for (int e = tid; e <= a.n_iter; e += blockDim.x) a.trace[slot * (a.n_iter + 1) + e] = 0.0;
        return;
    }
    run_unit<DK, NTW>(a, smem, ki, t, k);
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
    const unsigned units = (unsigned)a.T * (unsigned)(a.ki_end - a.ki_begin);
    hipLaunchKernelGGL(kern, dim3(units), dim3(nwaves * 64), lds, s, a);
    return hipGetLastError();
}

}  // namespace

#ifdef CHAM_KERNEL_TIMING
extern "C" int cham_dev_pass_timing(unsigned long long *host512, int reset)
{
    static unsigned long long z[64 * 16] = {0};
    if (reset) return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_pass), z, sizeof(z));
    return (int)hipMemcpyFromSymbol(host512, HIP_SYMBOL(g_pass), sizeof(z));
}
extern "C" int cham_dev_timing(unsigned long long *host16, int reset)
{
    unsigned long long z[16] = {0};
    if (reset) return (int)hipMemcpyToSymbol(HIP_SYMBOL(g_timing), z, sizeof(z));
    return (int)hipMemcpyFromSymbol(host16, HIP_SYMBOL(g_timing), sizeof(z));
}
#endif

// Three knob slots stay free for the bias and the per-row threshold, so d <= 29.
bool mfma_path_fits(int d, int kmax, int64_t n_max)
{
    return d >= 1 && d <= 29 && kmax <= 64 && n_max <= 4096;
}

// The packed row copy is made by the launch that starts at the first k (chunked sweeps reuse it).
hipError_t launch_mfma_sweep(const SweepArgs &a, int64_t n_max, int64_t n_total, hipStream_t s)
{
    const int ntw = n_max <= 1024 ? 4 : 16;
    int nwaves = (int)((n_max + 32 * ntw - 1) / (32 * ntw));
    if (nwaves < 1) nwaves = 1;
    if (nwaves > 8) nwaves = 8;
    const unsigned pb = (unsigned)((n_total + 255) / 256);
    if (a.d <= 13) {
        if (pb && a.ki_begin == 0) hipLaunchKernelGGL(pack_rows_kernel<16>, dim3(pb), dim3(256), 0, s, a.X, a.ld, a.d, n_total,
                                   reinterpret_cast<_Float16 *>(a.xh));
        return ntw == 4 ? launch_mfma_t<16, 4>(a, nwaves, s) : launch_mfma_t<16, 16>(a, nwaves, s);
    }
    if (pb && a.ki_begin == 0) hipLaunchKernelGGL(pack_rows_kernel<32>, dim3(pb), dim3(256), 0, s, a.X, a.ld, a.d, n_total,
                               reinterpret_cast<_Float16 *>(a.xh));
    return ntw == 4 ? launch_mfma_t<32, 4>(a, nwaves, s) : launch_mfma_t<32, 16>(a, nwaves, s);
}

}  // namespace cham
