// Matrix-core variant of the resident Lloyd kernel: one workgroup runs the whole iteration of
// one (task, k) unit (paper Algorithm 1, K-means.run(s_Theta, k); Sec. 3.3), with the squared
// distance screened by v_mfma_f32_32x32x16_f16.
//
// Screen:  score(c, i) = |mu'_c|^2 - 2 x'_i . mu'_c   (x', mu' centred by an integer offset)
//   A (32 centroids x K) = [ hi(w) | lo(w) ],  w = fl32(-2 mu'),  hi = f16(w), lo = f16(w - hi)
//   B (K x 32 rows)      = [ x' ; x' ]        (x' is a small integer: exact in f16)
//   the last knob slot (always unused: d < DK) carries the bias: B = 256, A = hi/lo of |mu'_c|^2 / 256
// so every product is exact and only the fp32 accumulation and the 22-bit splits round.
//
// Centroid c sits in fragment row 8 (i / 4) + 4 (c & 1) + (i & 3), i = (c & 31) / 2, of m-tile c / 32,
// so that accumulator register i of lane half hh holds centroid 2 i + hh: a unit with k centroids
// has live scores in its first ceil(k / 2) registers only, and the epilogue walks live groups of
// four registers, not all sixteen.  Per 32-row tile: minimum over the live registers (v_min3),
// threshold = minimum + error bound of the row (a constant of the row for the whole unit: the
// bound uses the largest squared norm that a centroid can have, that of the farthest row), one
// subtract and one v_alignbit per score for the mask of centroids beyond the threshold.  If every
// row's mask equals the mask it had when the tile was last decided (and none of its rows was
// undecided then), every row keeps its label and nothing else happens for the tile.  Otherwise a
// row with a single centroid inside the threshold takes it; the others are queued per wave and
// their marked centroids are re-evaluated in double in the oracle's operation order.
// The matrix instructions of the next tile are issued between the epilogue pieces of the current
// one.  Rows (as f16 B fragments) and labels stay in registers for all passes; centroids, integer
// sums and counts stay in LDS; a row touches the sums only when its label changes (exact: the
// sums are integers), through a dense per-wave queue.
//
// A pass that changes no label leaves the sums, hence the centroids, hence every later pass as
// they are: the iteration stops there and reports the state it has, which is what the remaining
// passes of the fixed-length iteration would reproduce.  The number of passes run is recorded.
#include <type_traits>

#include "cham_device.h"
#include "cham_internal.h"
#include "mfma_common.h"

namespace cham {

namespace {

// Cross-lane exchanges done in the vector ALU (DPP), no LDS round trip.
// xor_lanes<1|2|4|8>: the value held by lane ^ 1, 2, 4 or 8.
template <int XOR>
__device__ __forceinline__ int dpp_xor_i32(int v)
{
    if (XOR == 8) return __builtin_amdgcn_update_dpp(0, v, 0x128, 0xF, 0xF, false);     // row_ror:8 = lane ^ 8 within a row of 16
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

// Minimum of two / three scores.  This file is compiled with -fno-honor-nans (every score is a finite
// sum of finite products), which spares the instruction that would otherwise quiet a possible NaN in
// each operand coming out of a matrix instruction.  (Not inline assembly: the compiler has to see
// these reads to keep the wait states between a matrix instruction and the use of its result.)
__device__ __forceinline__ float vmin(float a, float b) { return __builtin_fminf(a, b); }
__device__ __forceinline__ float vmin3(float a, float b, float c) { return __builtin_fminf(__builtin_fminf(a, b), c); }

// Score position -> centroid.  Position q = 16 * m-tile + accumulator register (the order in which
// the mask bits are collected, most significant first), hh = lane half.
__device__ __forceinline__ int slot_centroid(int q, int hh) { return 2 * q + hh; }
// Row of the 32-row A fragment that holds centroid c of its m-tile.
__device__ __forceinline__ int frag_row(int c)
{
    const int i = (c & 31) >> 1;
    return 8 * (i >> 2) + 4 * (c & 1) + (i & 3);
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
    unsigned long long *acc64;  // [2]  sum over the task's rows of |x|^2; sum over the clusters of floor(|S|^2 / n)
    int *stamp;         // [4]        [1] float bits of the largest squared row norm, [2], [3] rows that changed in an even / odd pass
    unsigned char *wave_base;   // per-wave regions follow
    __host__ __device__ static size_t wave_bytes(int ntw)
    {
        return ((size_t)kRecCap * DK * 2 + kRecCap * 8 + kRecCap * 2 + 4 * 32 * 8 + 512 + 512 + 512 * 4 + (size_t)ntw * 64 * 4 + 15) / 16 * 16;
    }
    __host__ __device__ static size_t bytes(int KP, int nwaves, int ntw)
    {
        size_t b = sizeof(double) * DK * KP + sizeof(double) * 16 + sizeof(float) * KP;
        b += 16 * (size_t)(KP / 32) * (2 * DK / 16) * 64;
        b += sizeof(int) * (size_t)KP * (DK + 1) + sizeof(int) * KP * 2 + sizeof(float) * DK + 32;
        b = (b + 15) & ~(size_t)15;
        return b + wave_bytes(ntw) * nwaves;
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
        stamp = reinterpret_cast<int *>(base + o);     o += 16;
        acc64 = reinterpret_cast<unsigned long long *>(base + o);  o += 16;
        o = (o + 15) & ~(size_t)15;
        wave_base = base + o;
    }
};

// Per-wave LDS region.  A queue of at most kRecCap rows (their centred knob values as f16, the
// candidate masks of both lane halves, the row index), used first for the rows the screen could
// not decide and then for the label changes of the pass, in batches; behind it the current label of
// every row, the labels the pass arrives at, the error bound of every row and, per (tile, lane),
// the mask the lane had when its tile was last decided.
template <int DK>
struct WaveQueue {
    static constexpr int kRows = 512;                       // rows a wave owns at most
    static constexpr size_t kOffMask = (size_t)kRecCap * DK * 2;
    static constexpr size_t kOffPid = kOffMask + (size_t)kRecCap * 8;
    static constexpr size_t kOffFew = kOffPid + (size_t)kRecCap * 2;
    static constexpr size_t kOffLab = kOffFew + 4 * 32 * 8;
    static constexpr size_t kOffNew = kOffLab + (size_t)kRows;
    static constexpr size_t kOffEb = kOffNew + (size_t)kRows;
    static constexpr size_t kOffSeen = kOffEb + (size_t)kRows * 4;
    __host__ __device__ static constexpr size_t bytes(int ntw) { return (kOffSeen + (size_t)ntw * 64 * 4 + 15) / 16 * 16; }
    unsigned char *base;
    __device__ explicit WaveQueue(unsigned char *wb) : base(wb) {}
    __device__ _Float16 *rec_x() const { return reinterpret_cast<_Float16 *>(base); }                    // [kRecCap][DK]
    __device__ unsigned *rec_mask() const { return reinterpret_cast<unsigned *>(base + kOffMask); }      // [kRecCap][2]
    __device__ unsigned short *rec_pid() const { return reinterpret_cast<unsigned short *>(base + kOffPid); }
    __device__ double *few() const { return reinterpret_cast<double *>(base + kOffFew); }                 // [4][32] squares of one (row, centroid)
    __device__ unsigned char *lab() const { return base + kOffLab; }                                      // [kRows] current labels (0xFF: none)
    __device__ unsigned char *lab_new() const { return base + kOffNew; }                                  // [kRows] labels of the pass under way
    __device__ float *eb() const { return reinterpret_cast<float *>(base + kOffEb); }                     // [kRows] screen bound of the row
    __device__ unsigned *seen() const { return reinterpret_cast<unsigned *>(base + kOffSeen); }           // [tiles][64] mask at the last decision
};

// Resolve the queued rows of this wave: four lanes per row, each lane takes every fourth marked
// centroid of its row and evaluates the exact double distance (knobs ascending, no fused
// multiply-add); the four lanes then agree on the smallest distance, lowest index on ties.  The
// result goes to the row's entry of the labels of the pass under way.
template <int DK>
__device__ __forceinline__ void resolve_rows(const WaveQueue<DK> &Q, int nrec, const double *mu64T,
                                             const float *ojf, int KP, int k, int d)
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
                c = slot_centroid(b, 0);
            } else if (rem1) {
                const int b = __clz((int)rem1);
                rem1 &= ~(0x80000000u >> b);
                c = slot_centroid(b, 1);
            }
            return c;
        };
        for (int i = 0; i < q; ++i) pop();
        double bs = __builtin_inf();
        int bc = 0x7fffffff;
        while (__ballot((rem0 | rem1) != 0u)) {
            const int cc = pop();
            const int ci = (cc < 0 || cc >= k) ? 0 : cc;
            double ss = 0.0;
            // knobs in groups of 8; the loads of a group are independent and overlap
            for (int j0 = 0; j0 < d; j0 += 8) {
                const half8 xq = *reinterpret_cast<const half8 *>(Q.rec_x() + (size_t)rr * DK + j0);
                const float4 oa = *reinterpret_cast<const float4 *>(ojf + j0);
                const float4 ob = *reinterpret_cast<const float4 *>(ojf + j0 + 4);
                const float of[8] = {oa.x, oa.y, oa.z, oa.w, ob.x, ob.y, ob.z, ob.w};
                double mu[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) mu[i] = mu64T[(size_t)(j0 + i) * KP + ci];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    // queued copies are centred; padded knobs are skipped (the last one carries the bias)
                    float xf = (float)xq[i] + of[i];
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
        if (have && q == 0) Q.lab_new()[pid] = (unsigned char)(bc < k ? bc : 0);
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
    double *sc = Q.few() + slot * 32;      // squares of one (row, centroid)
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
        // this lane's knobs of the row (the queued copy is centred; the bias slot and padded slots count as zero)
        float xa = 0.0f, xb = 0.0f;
        if (jl < d) xa = (float)Q.rec_x()[(size_t)rr * DK + jl] + ojf[jl];
        if (DK == 32 && jl + 16 < d) xb = (float)Q.rec_x()[(size_t)rr * DK + jl + 16] + ojf[jl + 16];
        auto pop = [&]() -> int {
            int c = -1;
            if (rem0) {
                const int b = __clz((int)rem0);
                rem0 &= ~(0x80000000u >> b);
                c = slot_centroid(b, 0);
            } else if (rem1) {
                const int b = __clz((int)rem1);
                rem1 &= ~(0x80000000u >> b);
                c = slot_centroid(b, 1);
            }
            return c;
        };
        if (slot & 1) pop();
        double bs = __builtin_inf();
        int bc = 0x7fffffff;
        while (__ballot((rem0 | rem1) != 0u)) {
            const int cc = pop();
            const int ci = (cc < 0 || cc >= k) ? 0 : cc;
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
        if (have && (lane & 31) == 0) Q.lab_new()[pid] = (unsigned char)(bc < k ? bc : 0);
    }
    __builtin_amdgcn_wave_barrier();
}

template <int DK>
__device__ __forceinline__ void resolve_queue(const WaveQueue<DK> &Q, int nrec, const double *mu64T,
                                              const float *ojf, int KP, int k, int d)
{
    if constexpr (DK <= 32) {
        if (nrec <= 8) {
            resolve_few<DK>(Q, nrec, mu64T, ojf, KP, k, d);
            return;
        }
    }
    resolve_rows<DK>(Q, nrec, mu64T, ojf, KP, k, d);
}

// Row-major f16 copy of X (one row = DK halfs, padded knobs zero): a lane fetches the eight knobs
// of a B fragment with one 16-byte load.
// Two-byte knobs take this path only when every value is below 2048 (integers up to 2048 are
// exact in f16): a larger value sets *too_large, which makes the sweep kernel report status 4.
template <int DK, typename XT>
__global__ void pack_rows_kernel(const XT *__restrict__ X, int64_t ld, int d, int64_t n_rows,
                                 _Float16 *__restrict__ xh, int *too_large)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_rows) return;
    unsigned top = 0;
#pragma unroll
    for (int g = 0; g < DK / 8; ++g) {
        half8 v;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int j = 8 * g + i;
            const unsigned xv = j < d ? (unsigned)X[(int64_t)j * ld + r] : 0u;
            top = xv > top ? xv : top;
            v[i] = (_Float16)(float)xv;
        }
        *reinterpret_cast<half8 *>(xh + r * DK + 8 * g) = v;
    }
    if (sizeof(XT) == 2 && top >= 2048u) *too_large = 1;
}

// Apply queued label changes of this wave to the integer sums and counts: 256 / DK queued rows
// per step, one lane per (row, group of 4 knobs).  Entry word: cur | prev << 8, prev = 0xFF for a
// row that had no label yet.
template <int DK>
__device__ __forceinline__ void apply_changes(const WaveQueue<DK> &Q, int cnt, int *S, int *n, int *dirty,
                                              const float *ojf, int d, int stamp)
{
    constexpr int LPR = DK / 4;              // lanes per row
    constexpr int EPI = 64 / LPR;            // rows per step
    const int lane = threadIdx.x & 63;
    const int j0 = 4 * (lane % LPR);
    const float4 o4 = *reinterpret_cast<const float4 *>(ojf + j0);
    const float of[4] = {o4.x, o4.y, o4.z, o4.w};
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

// Sums and sizes of every cluster over this wave's rows, from the current labels, on the matrix
// cores: S^T (knob x centroid) = X^T (knob x row) * onehot (row x centroid), sixteen rows per
// instruction.  Lane (m, kh) of the A fragment holds knob m of eight consecutive rows, read straight
// from the knob-major byte matrix (32 consecutive rows = 32 bytes per lane and group of 64 rows; the
// same row order is used for the labels, so any order would do).  A byte b becomes the f16 value
// 1024 + b by byte placement alone (0x6400 | b); the knob rows therefore sum to S + 1024 n, and the
// rows of absent knobs (all bytes zero) to 1024 n, of which row 31 serves as the cluster size.  The
// one-hot operand is clamp(1025 - (1024 + (label ^ centroid)), 0, 1).  Every product and partial sum
// is an integer below 2^24, so the fp32 accumulation is exact.  The results are added to the sums
// of the workgroup (still raised by 1024 n: the centroid update takes that off) and to the sizes.
// Needs 16-byte aligned rows (xw, ld) and reads whole groups of 64 rows: the caller makes sure
// that the last group of the task still lies inside the matrix (rows of other tasks or padding
// read there meet the label 0xFF, which matches no centroid).  NG = groups of 64 rows a wave owns
// at most; the loads of four groups are under way at any time.
template <int DK, int NG>
__device__ __forceinline__ void full_sums(const WaveQueue<DK> &Q, int *S, int *n, const uint8_t *xw, int64_t ld,
                                          int d, int k, int rows_here, int lane)
{
    typedef unsigned uint4v __attribute__((ext_vector_type(4)));
    typedef _Float16 half2v __attribute__((ext_vector_type(2)));
    constexpr int kDepth = NG < 4 ? NG : 4;
    const int m32 = lane & 31, kh = lane >> 5;
    const bool two = k > 32;
    const bool knob = m32 < d;
    const uint8_t *xp = xw + (int64_t)(knob ? m32 : 0) * ld + 32 * kh;
    const unsigned char *lp = Q.lab() + 32 * kh;
    const unsigned c4a = (unsigned)m32 * 0x01010101u, c4b = c4a + 0x20202020u;
    const float16v zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float16v acc0 = zero16, acc1 = zero16;
    const int ngroups = (rows_here + 63) >> 6;

    // this lane's 32 bytes of group g (zero where the knob or the group does not exist)
    auto fetch = [&](int g, uint4v &w0, uint4v &w1) {
        w0 = uint4v{0u, 0u, 0u, 0u};
        w1 = w0;
        if (knob && g < ngroups) {
            w0 = *reinterpret_cast<const uint4v *>(xp + 64 * g);
            w1 = *reinterpret_cast<const uint4v *>(xp + 64 * g + 16);
        }
    };
    // eight bytes -> eight f16 values 1024 + byte
    auto widen = [](unsigned lo4, unsigned hi4) {
        uint4v r;
        r[0] = __builtin_amdgcn_perm(0x64646464u, lo4, 0x04010400u);
        r[1] = __builtin_amdgcn_perm(0x64646464u, lo4, 0x04030402u);
        r[2] = __builtin_amdgcn_perm(0x64646464u, hi4, 0x04010400u);
        r[3] = __builtin_amdgcn_perm(0x64646464u, hi4, 0x04030402u);
        return r;
    };
    // eight (label ^ centroid) bytes -> eight f16 values: 1 where the byte is zero, else 0
    auto onehot = [&](unsigned lo4, unsigned hi4) {
        const uint4v r = widen(lo4, hi4);
        uint4v o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const unsigned re = r[e];           // (a scalar copy: a bit cast of the vector element itself reads element 0)
            half2v v = __builtin_bit_cast(half2v, re);
            v = half2v{(_Float16)1025.0f, (_Float16)1025.0f} - v;
            v = __builtin_elementwise_min(__builtin_elementwise_max(v, half2v{(_Float16)0.0f, (_Float16)0.0f}),
                                          half2v{(_Float16)1.0f, (_Float16)1.0f});
            o[e] = __builtin_bit_cast(unsigned, v);
        }
        return __builtin_bit_cast(half8, o);
    };

    uint4v w0[kDepth], w1[kDepth];
#pragma unroll
    for (int g = 0; g < kDepth; ++g) fetch(g, w0[g], w1[g]);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
        if (g < ngroups) {
            const uint4v c0 = w0[g % kDepth], c1 = w1[g % kDepth];
            const uint4v l0 = *reinterpret_cast<const uint4v *>(lp + 64 * g);
            const uint4v l1 = *reinterpret_cast<const uint4v *>(lp + 64 * g + 16);
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const unsigned xa = t < 2 ? c0[(2 * t) & 3] : c1[(2 * t) & 3];
                const unsigned xb = t < 2 ? c0[(2 * t + 1) & 3] : c1[(2 * t + 1) & 3];
                const unsigned la = t < 2 ? l0[(2 * t) & 3] : l1[(2 * t) & 3];
                const unsigned lb = t < 2 ? l0[(2 * t + 1) & 3] : l1[(2 * t + 1) & 3];
                const half8 A = __builtin_bit_cast(half8, widen(xa, xb));
                acc0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A, onehot(la ^ c4a, lb ^ c4a), acc0, 0, 0, 0);
                if (two) acc1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(A, onehot(la ^ c4b, lb ^ c4b), acc1, 0, 0, 0);
            }
            if (g + kDepth < NG) fetch(g + kDepth, w0[g % kDepth], w1[g % kDepth]);
        }
    }
    // accumulator register i of lane (c, kh) = knob (i & 3) + 8 (i >> 2) + 4 kh of centroid c (or 32 + c)
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int m = (i & 3) + 8 * (i >> 2) + 4 * kh;
        if (m < d) {
            if (m32 < k) atomicAdd(&S[m32 * (DK + 1) + m], (int)acc0[i]);
            if (two && m32 + 32 < k) atomicAdd(&S[(m32 + 32) * (DK + 1) + m], (int)acc1[i]);
        }
        if (i == 15 && kh == 1) {                              // knob row 31: 1024 per row of the cluster
            if (m32 < k) atomicAdd(&n[m32], (int)acc0[i] >> 10);
            if (two && m32 + 32 < k) atomicAdd(&n[m32 + 32], (int)acc1[i] >> 10);
        }
    }
}

// Centroid update for the clusters touched in this pass, all threads: item (c, q) owns knobs
// 4q..4q+3 of centroid c: mean = (double)S / (double)n, then the f16 hi/lo fragments of
// w = -2 (mu - o) (one 8-byte store each).  The DK/4 items of a centroid sit in adjacent lanes and
// add up |mu - o|^2 among themselves; the last of them owns the bias slot (knob slot DK - 1) and
// stores the sum / 256 there as hi/lo, and its rounded-up value for the error bound.
// all: fragments from the centroids as they are (no sums yet).  raw: the sums were rebuilt by
// full_sums for every cluster (each still raised by 1024 n): every cluster is updated, and the sums
// are left either corrected (the next pass applies label changes to them) or, with zero_after,
// cleared together with the sizes (the next pass rebuilds them).
template <int DK, bool BYTE_KNOBS = true>
__device__ __forceinline__ void update_centroids(const MfmaLds<DK> &U, int k, int KP, int d, int stamp, bool all,
                                                 bool raw = false, bool zero_after = false)
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
            if (!all && ((!raw && U.dirty[c] != stamp) || cnt == 0)) act = false;   // an empty cluster keeps its centroid
        }
        half4 hi4 = {(_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f, (_Float16)0.0f};
        half4 lo4 = hi4;
        double b = 0.0;
        // The mean S / n with one division per item instead of one per knob: r = fl(1 / n), then
        // q0 = fl(S r), rem = S - q0 n (exact in one fused operation), fl(q0 + rem r).  That this
        // equals the correctly rounded quotient fl(S / n) for every count 1 <= n <= 4096 and every
        // integer sum 0 <= S <= 255 n (the whole domain of this kernel: byte knobs, tasks of at most
        // 4096 rows) is checked exhaustively on the CPU (quotient_check.c, run by the test suite).
        const double dn = (double)(cnt > 0 ? cnt : 1);
        const double rn = 1.0 / dn;
        if (act && 4 * q < d) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int j = 4 * q + i;
                double mu = U.mu64T[(size_t)j * KP + c];
                if (!all && j < d) {
                    int sv = U.S[c * (DK + 1) + j];
                    if (raw) {
                        sv -= 1024 * cnt;
                        U.S[c * (DK + 1) + j] = sv;
                    }
                    const double sd = (double)sv;
                    if (BYTE_KNOBS) {
                        const double q0 = sd * rn;
                        const double rem = __builtin_fma(-q0, dn, sd);
                        mu = __builtin_fma(rem, rn, q0);
                    } else {
                        mu = sd / dn;             // (sums of two-byte knobs lie outside the checked domain)
                    }
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
        if (QN >= 8) b = b + dpp_xor_f64<4>(b);
        if (QN == 16) b = b + dpp_xor_f64<8>(b);
        if (act && (4 * q < d || q == QN - 1)) {
            if (q == QN - 1) {
                const float bs = (float)b * (1.0f / kBiasScale);
                const _Float16 bhi = (_Float16)bs;
                hi4[3] = bhi;
                lo4[3] = (_Float16)(bs - (float)bhi);
                U.bias[c] = __double2float_ru(b) * 1.0000005f;
            }
            const int mt = c >> 5, m32 = frag_row(c);
            const int g = q >> 1, kh = g & 1, fstep = g >> 1, sub = q & 1;
            half4 *fh = reinterpret_cast<half4 *>(U.afrag + (mt * NS2 + fstep) * 64 + 32 * kh + m32) + sub;
            half4 *fl = reinterpret_cast<half4 *>(U.afrag + (mt * NS2 + NS + fstep) * 64 + 32 * kh + m32) + sub;
            *fh = hi4;
            *fl = lo4;
        }
        if (zero_after && item < items) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (4 * q + i < d) U.S[c * (DK + 1) + 4 * q + i] = 0;
            // every item of a cluster sits in this wave and has read the size by now
            __builtin_amdgcn_wave_barrier();
            if (q == 0) U.n[c] = 0;
        }
    }
}

// Everything one workgroup does for its unit.  Units with more than 32 centroids use two 32-row
// m-tiles per row tile; otherwise the two accumulators alternate between row tiles.
template <int DK, int NTW, typename XT>
__device__ __forceinline__ void run_unit(const SweepArgs &a, unsigned char *smem, int ki, int t, int k)
{
    constexpr bool kByteKnobs = sizeof(XT) == 1;
    constexpr double kMaxValue = kByteKnobs ? 255.0 : 2047.0;
    constexpr bool kAllowTwo = DK <= 32;     // 64-wide rows leave no registers for a second m-tile: k <= 32 there
    const XT *X = reinterpret_cast<const XT *>(a.X);
    const bool two = kAllowTwo && k > 32;
    constexpr int NS = DK / 16;          // distinct B fragments per row
    constexpr int NS2 = 2 * NS;          // chained instructions per 32x32 tile
    constexpr int CH = 16 / NS2;         // scores handled between two matrix instructions
    const int KP = a.kmax > 32 ? 64 : 32;
    MfmaLds<DK> U(smem, KP);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int nwaves = blockDim.x >> 6;
    const int n32 = lane & 31;           // row within a 32-row tile
    const int h = lane >> 5;             // which half of the knob slots / centroid rows this lane holds
    // The phases of a pass take the lane index through this: values derived from it (addresses into
    // the wave's tables) are then computed where they are used instead of living, or being spilled,
    // across the whole iteration next to the 128 registers of rows.
    const int lane_id = lane;
    auto opaque = [](int v) {
        asm volatile("" : "+v"(v));
        return v;
    };

    const int d = a.d;
    const int64_t r0 = a.task_off[t], r1 = a.task_off[t + 1];
    const int nrows = (int)(r1 - r0);
    const int64_t slot = (int64_t)t * a.n_k + ki;
    const int64_t crow = (int64_t)t * a.Ksum + a.koff[ki];
    uint8_t *labrow = a.labbuf + (int64_t)ki * a.ld;

    WaveQueue<DK> Q(U.wave_base + MfmaLds<DK>::wave_bytes(NTW) * wave);
    const int wave_row0 = wave * NTW * 32;                 // first row (task-relative) of this wave
    const bool wave_live = wave_row0 < nrows;              // the wave owns at least one row

    // Live accumulator registers: centroids 2 i + hh sit in register i, so a tile of kk centroids has
    // scores in its first ceil(kk / 2) registers; they are walked in groups of four.
    const int kk_last = two ? k - 32 : k;                  // centroids in the last (or only) m-tile
    const int lregs = ((kk_last + 1) / 2 + 3) & ~3;        // 4, 8, 12 or 16

    // The last knob slot of the fragments is reserved (d <= DK - 1): it carries the bias (256 in B,
    // |mu'|^2 / 256 as hi/lo in A).
    constexpr int bstep = NS - 1, bhalf = 1, belem = 7;
    constexpr int kFullDivisor = 8;

    // ---- this lane's rows as B fragments (kept in registers for every pass).  The loads are issued
    // first (raw knob values; they are centred once the offsets are known) so that they are under way
    // during the set-up of the unit's state.
    const _Float16 *xh_wave = reinterpret_cast<const _Float16 *>(a.xh) + (r0 + (wave_live ? wave_row0 : 0)) * DK;
    half8 B[NTW][NS];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
        const bool live = wave_live && (wave_row0 + nt * 32 + n32) < nrows;
        const int64_t prow = live ? (int64_t)(nt * 32 + n32) : 0;         // always a row of this task
#pragma unroll
        for (int f = 0; f < NS; ++f) {
            half8 v;
#pragma unroll
            for (int i = 0; i < 8; ++i) v[i] = (_Float16)0.0f;
            if (nrows > 0) v = *reinterpret_cast<const half8 *>(xh_wave + prow * DK + 16 * f + 8 * h);
            B[nt][f] = v;
        }
    }

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
        _Float16 *bslot = reinterpret_cast<_Float16 *>(U.afrag + ((c >> 5) * NS2 + bstep) * 64 + 32 * bhalf + frag_row(c)) + belem;
        bslot[0] = (_Float16)kPadBiasHi;
    }
    if (tid == 0) {
        U.stamp[0] = 0;           // (unused)
        U.stamp[1] = 0;           // float bits of the largest squared norm of a centred row
        U.stamp[2] = 0;           // rows that changed their label in an even pass
        U.stamp[3] = 0;           // ... in an odd pass
        U.acc64[0] = 0ull;
        U.acc64[1] = 0ull;
    }
    for (int e = tid; e < k * d; e += blockDim.x) {
        const int c = e / d, j = e % d;
        double v;
        if (a.init_mode == 0) {
            const int row = a.init_rows[(int64_t)t * a.kmax + c];
            v = (double)X[(int64_t)j * a.ld + r0 + row];
        } else {
            v = a.init_centroids[(crow + c) * d + j];
        }
        U.mu64T[(size_t)j * KP + c] = v;
    }
    __syncthreads();
    {
        // centring offset of knob j: the rounded mean of the starting centroids (any integer would do:
        // it only keeps the centred magnitudes small); eight lanes per knob
        const int part = tid & 7;
        for (int j = tid >> 3; j < DK; j += blockDim.x >> 3) {       // (uniform within a wave: every lane shuffles)
            double s = 0.0;
            if (j < d)
                for (int c = part; c < k; c += 8) s += U.mu64T[(size_t)j * KP + c];
            s = s + dpp_xor_f64<1>(s);
            s = s + dpp_xor_f64<2>(s);
            s = s + dpp_xor_f64<4>(s);
            if (part == 0) {
                float o = 0.0f;
                if (j < d) {
                    double m = rint(s / (double)k);
                    m = m < 0.0 ? 0.0 : (m > kMaxValue ? kMaxValue : m);
                    o = (float)m;
                }
                U.ojf[j] = o;
            }
        }
    }
    __syncthreads();
    update_centroids<DK, kByteKnobs>(U, k, KP, d, 0, true);

    // ---- centre the rows; on the way, the sum of |x|^2 over the task's rows as an integer (for the loss
    // at a fixed point, see the end) and the squared norm of every centred row (for the error bound).
    // Squares are summed two at a time into fp32 (v_dot2): the raw values are integers below 256, so
    // a lane's sum per tile stays below 16 * 255^2 < 2^24 and is exact.
    {
        typedef _Float16 half2v __attribute__((ext_vector_type(2)));
        typedef unsigned uint4v __attribute__((ext_vector_type(4)));
        auto sumsq = [](const half8 &v, float acc) {
            const uint4v w = __builtin_bit_cast(uint4v, v);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const unsigned we = w[e];
                const half2v p = __builtin_bit_cast(half2v, we);
                acc = __builtin_amdgcn_fdot2(p, p, acc, false);
            }
            return acc;
        };
        float x2row[NTW];                // squared norm of this lane's centred row of every tile
        half8 off8[NS];
        uint4v keep[NS];                 // all ones in the halves of the knobs that exist
#pragma unroll
        for (int f = 0; f < NS; ++f) {
#pragma unroll
            for (int i = 0; i < 8; ++i) off8[f][i] = (_Float16)U.ojf[16 * f + 8 * h + i];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int j = 16 * f + 8 * h + 2 * e;
                keep[f][e] = (j < d ? 0x0000FFFFu : 0u) | (j + 1 < d ? 0xFFFF0000u : 0u);
            }
        }
        unsigned q2 = 0;
        float xmax = 0.0f;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            const bool live = wave_live && (wave_row0 + nt * 32 + n32) < nrows;
            float raw = 0.0f, part = 0.0f;
#pragma unroll
            for (int f = 0; f < NS; ++f) {
                if (kByteKnobs) raw = sumsq(B[nt][f], raw);
                const half8 c8 = B[nt][f] - off8[f];
                uint4v w = __builtin_bit_cast(uint4v, c8) & keep[f];
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = live ? w[e] : 0u;
                half8 cv = __builtin_bit_cast(half8, w);
                part = sumsq(cv, part);
                // the bias slot: a constant for every live row (after the norm, which excludes it)
                if (f == bstep && live && h == bhalf) cv[belem] = (_Float16)kBiasScale;
                B[nt][f] = cv;
            }
            if (kByteKnobs) q2 += live ? (unsigned)raw : 0u;
            part = part + __shfl_xor(part, 32, 64);
            x2row[nt] = part;
            xmax = __builtin_fmaxf(xmax, part);
        }
        // the wave's sum of |x|^2 (at most 512 rows * 31 * 255^2 < 2^31) -> the unit's 64-bit sum
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) q2 += (unsigned)__shfl_xor((int)q2, off, 64);
        if (lane_id == 0 && q2) atomicAdd(&U.acc64[0], (unsigned long long)q2);
        xmax = wave_max_nonneg(xmax);
        if (lane == 0) atomicMax(&U.stamp[1], __float_as_int(xmax));     // non-negative floats order like integers
        __syncthreads();
        // Largest squared norm a centred centroid can take during the iteration: every later centroid
        // is a mean of rows (inside their convex hull) or stays where it started.
        float m2 = wave_max_nonneg(lane < k ? U.bias[lane] : 0.0f);
        m2 = __builtin_fmaxf(m2, __int_as_float(U.stamp[1])) * 1.000001f;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt)
            if (h == 0) Q.eb()[nt * 32 + n32] = mfma_bound<NS2>(x2row[nt], m2);
    }
    __builtin_amdgcn_wave_barrier();

    // no row has a label yet
    for (int e = lane; e < WaveQueue<DK>::kRows; e += 64) Q.lab()[e] = 0xFF;
    __builtin_amdgcn_wave_barrier();

    const int rows_wave = __builtin_amdgcn_readfirstlane(nrows - wave_row0);   // rows from this wave's first row to the task's end
    uint32_t force_tiles = 0xFFFFFFFFu;  // tiles to decide whatever their masks say: all at first, later those with undecided rows
    int passes_run = 0;
    bool at_fixed_point = false;         // the last pass run moved no row: every centroid is the mean of its cluster
    // A pass after one that moved many rows rebuilds the sums from the labels on the matrix cores
    // instead of applying the changes one by one; the first pass (every row is new) always does.
    const uint8_t *xw = a.X + r0 + (wave_live ? wave_row0 : 0);
    const bool x_aligned = kByteKnobs &&                              // (the rebuild reads the byte matrix)
                           ((reinterpret_cast<uintptr_t>(a.X) | (uintptr_t)a.ld | (uintptr_t)r0) & 15) == 0 &&
                           r0 + ((nrows + 63) & ~63) <= a.ld;       // ... and its last group of 64 rows lies inside the matrix
    bool full_mode = x_aligned;
    const int full_above = nrows / kFullDivisor;      // changed rows of a pass above which the next one rebuilds
    bool traced_last = false;

    // lanes of tile nt (as a 32-bit mask over the row index within the tile) whose row belongs to the task
    auto live_rows = [&](int nt) -> uint32_t {
        int left = rows_wave - 32 * nt;
        left = left < 0 ? 0 : (left > 32 ? 32 : left);
        return left == 32 ? 0xFFFFFFFFu : ((1u << left) - 1u);
    };
    // This lane's B fragments of tile nt, nt known at run time only (the same for the whole wave): one
    // branch per tile around a register copy, so that the code that follows exists once, not per tile.
    auto rows_of_tile = [&](int nt, half8 (&bt)[NS]) {
#pragma unroll
        for (int n = 0; n < NTW; ++n) {
            if (nt == n) {
#pragma unroll
                for (int f = 0; f < NS; ++f) {
                    bt[f] = B[n][f];
                    asm volatile("" : "+v"(bt[f]));      // keeps the copy under its branch
                }
            }
        }
    };

    // Exact loss of the current labels from the rows in registers: (x - mu)^2 in double over the knobs
    // a lane holds (x = centred value + offset, exact), the two lanes of a row and all rows added up
    // afterwards; the per-wave sums land in U.red[slot8 .. slot8 + nwaves).
    auto wave_loss = [&](int slot8) {
        double part = 0.0;
        const int lane = opaque(lane_id), n32 = lane & 31, h = lane >> 5;
        if (wave_live) {
            float of[NS][8];
#pragma unroll
            for (int f = 0; f < NS; ++f)
#pragma unroll
                for (int i = 0; i < 8; ++i) of[f][i] = U.ojf[16 * f + 8 * h + i];
            // (unrolled over the tiles: runs once per unit, and the loads of several tiles overlap)
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt) {
                const half8 (&bt)[NS] = B[nt];
                const uint32_t lab = Q.lab()[nt * 32 + n32];
                const bool live = lab != 0xFFu;
                const double *mc = U.mu64T + (live ? lab : 0u) + (size_t)(8 * h) * KP;
                // the centroid's knobs first, all loads under way together, then the sum in knob order
                double mu[NS][8];
#pragma unroll
                for (int f = 0; f < NS; ++f)
#pragma unroll
                    for (int i = 0; i < 8; ++i) mu[f][i] = mc[(size_t)(16 * f + i) * KP];
                double s = 0.0;
#pragma unroll
                for (int f = 0; f < NS; ++f)
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        float xf = (float)bt[f][i] + of[f][i];
                        if (f == bstep && i == belem) xf = h == bhalf ? 0.0f : xf;     // the bias slot is no knob
                        const double tq = (double)xf - mu[f][i];
                        s = s + tq * tq;
                    }
                part = part + (live ? s : 0.0);
            }
        }
        // the wave's total in the fixed order lane ^ 32, 16, ..., 1 (partner indices from the local lane index)
        double ws = part;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const long long b = __double_as_longlong(ws);
            const int plo = __builtin_amdgcn_ds_bpermute((lane ^ off) << 2, (int)(b & 0xFFFFFFFFll));
            const int phi = __builtin_amdgcn_ds_bpermute((lane ^ off) << 2, (int)(b >> 32));
            ws = ws + __longlong_as_double(((long long)phi << 32) | (unsigned int)plo);
        }
        if (lane == 0) U.red[slot8 + wave] = ws;
    };

    for (int it = 0; it <= a.n_iter; ++it) {
        const bool last_pass = (it == a.n_iter);
        passes_run = it + 1;
        uint32_t flagged_tiles = 0;      // tiles with rows that the screen could not decide
        uint32_t changed_tiles = 0;      // tiles in which a label may differ from the current one

        // The tile loop, compiled once per number of live registers of the last m-tile (4, 8, 12 or 16),
        // so that the epilogue has no branches.
        auto tile_pass = [&](auto live_tag) {
            constexpr int LREGS = decltype(live_tag)::value;
            const int lane = opaque(lane_id), n32 = lane & 31;
            // A fragments of this pass (the bias slot included)
            half8 A0[NS2], A1[NS2];
#pragma unroll
            for (int s = 0; s < NS2; ++s) {
                A0[s] = U.afrag[s * 64 + lane];
                A1[s] = two ? U.afrag[(NS2 + s) * 64 + lane] : A0[s];
            }

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
            // minimum over the first nreg registers (nreg = 4, 8, 12 or 16)
            auto min_live = [&](const float16v &acc, auto nreg_tag) {
                constexpr int nreg = decltype(nreg_tag)::value;
                float b = vmin(vmin3(acc[0], acc[1], acc[2]), acc[3]);
                if (nreg > 4) b = vmin3(vmin3(b, acc[4], acc[5]), acc[6], acc[7]);
                if (nreg > 8) b = vmin3(vmin3(b, acc[8], acc[9]), acc[10], acc[11]);
                if (nreg > 12) b = vmin3(vmin3(b, acc[12], acc[13]), acc[14], acc[15]);
                return b;
            };
            // both lane halves' minima of a row -> the row's minimum
            auto row_min = [&](float v) {
                unsigned lo, hi;
                both_halves(__float_as_uint(v), lo, hi);
                return vmin(__uint_as_float(lo), __uint_as_float(hi));
            };
            // After the masks of tile nt: if any row's mask differs from the remembered one (or the tile is
            // forced), remember the new masks and decide the tile's rows: a row with exactly one
            // candidate takes it, any other row is left to the exact evaluation after the tile loop
            // (label 0xFE until then).  Tiles with such rows and tiles in which a label differs from
            // the current one are listed.  (The matrix instructions of the next tile are under way
            // meanwhile.)
            auto settle = [&](uint32_t far, uint32_t seen, int nt) {
                const uint64_t diff = __ballot(far != seen);
                const uint32_t live32 = live_rows(nt);
                uint32_t dirty32 = ((uint32_t)diff | (uint32_t)(diff >> 32)) & live32;
                if ((force_tiles >> nt) & 1u) dirty32 = live32;
                if (dirty32) {
                    Q.seen()[nt * 64 + lane] = far;
                    const uint32_t prev = Q.lab()[nt * 32 + n32];
                    const uint32_t cand = ~far;                          // bit 31 = position 0
                    uint32_t cand_lo, cand_hi;
                    both_halves(cand, cand_lo, cand_hi);
                    const int total = __popc(cand_lo) + __popc(cand_hi);
                    const bool live = (live32 >> n32) & 1u;
                    const bool flagged = live && total != 1;
                    const int hh = cand_lo ? 0 : 1;
                    const int q = __clz((int)(cand_lo ? cand_lo : cand_hi));
                    const uint32_t lab = (uint32_t)slot_centroid(q & 31, hh);
                    const uint32_t now = !live ? 0xFFu : (flagged ? 0xFEu : lab);
                    if (__ballot(flagged)) flagged_tiles |= 1u << nt;
                    if (__ballot(now != prev)) {
                        changed_tiles |= 1u << nt;
                        if (lane < 32) Q.lab_new()[nt * 32 + n32] = (unsigned char)now;
                    }
                }
            };

            // bound and remembered mask of the tile under way; those of the next tile are fetched a tile ahead
            float eb_cur = Q.eb()[n32];
            uint32_t seen_cur = Q.seen()[lane];
            if (kAllowTwo && two) {
                // accA = centroids 0..31 (all sixteen registers live), accB = centroids 32..k-1 of the current tile
#pragma unroll
                for (int s = 0; s < NS2; ++s) mma(accA, A0, B[0], s);
#pragma unroll
                for (int s = 0; s < NS2; ++s) mma(accB, A1, B[0], s);
#pragma unroll
                for (int nt = 0; nt < NTW; ++nt) {
                    constexpr int kLast = NTW - 1;
                    const int nx = nt < kLast ? nt + 1 : nt;
                    const float eb_nxt = Q.eb()[nx * 32 + n32];
                    const uint32_t seen_nxt = Q.seen()[nx * 64 + lane];
                    const float best = row_min(vmin(min_live(accA, std::integral_constant<int, 16>{}), min_live(accB, live_tag)));
                    const float thr = best + eb_cur;
                    uint32_t far = 0;
#pragma unroll
                    for (int s = 0; s < NS2; ++s) mark(far, accA, thr, s * CH);
                    // accA is consumed: its next chain runs under the marking of accB
#pragma unroll
                    for (int s = 0; s < NS2; ++s) {
                        __builtin_amdgcn_sched_barrier(0);
                        if (nt < kLast) mma(accA, A0, B[nx], s);
                        __builtin_amdgcn_sched_barrier(0);
                        if (s * CH < LREGS) mark(far, accB, thr, s * CH);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    if (nt < kLast) {
#pragma unroll
                        for (int s = 0; s < NS2; ++s) mma(accB, A1, B[nx], s);
                    }
                    // registers of accB that were not walked hold padding only: far
                    constexpr int live_marks = CH * ((LREGS + CH - 1) / CH);
                    far = (far << (16 - live_marks)) | ((1u << (16 - live_marks)) - 1u);
                    settle(far, seen_cur, nt);
                    eb_cur = eb_nxt;
                    seen_cur = seen_nxt;
                    __builtin_amdgcn_sched_barrier(0);
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
                    const float eb_nxt = Q.eb()[nx * 32 + n32];
                    const uint32_t seen_nxt = Q.seen()[nx * 64 + lane];
                    const float best = row_min(min_live(cur, live_tag));
                    const float thr = best + eb_cur;
                    uint32_t far = 0;
#pragma unroll
                    for (int s = 0; s < NS2; ++s) {
                        __builtin_amdgcn_sched_barrier(0);
                        if (nt < kLast) mma(nxt, A0, B[nx], s);
                        __builtin_amdgcn_sched_barrier(0);
                        if (s * CH < LREGS) mark(far, cur, thr, s * CH);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    constexpr int live_marks = CH * ((LREGS + CH - 1) / CH);
                    far = (far << (32 - live_marks)) | (0xFFFFFFFFu >> live_marks);
                    settle(far, seen_cur, nt);
                    eb_cur = eb_nxt;
                    seen_cur = seen_nxt;
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        if (wave_live) {
            switch (lregs) {
            case 4: tile_pass(std::integral_constant<int, 4>{}); break;
            case 8: tile_pass(std::integral_constant<int, 8>{}); break;
            case 12: tile_pass(std::integral_constant<int, 12>{}); break;
            default: tile_pass(std::integral_constant<int, 16>{}); break;
            }
        }

        // ---- the undecided rows: exact evaluation, through the queue (this code exists once; the tile
        // index is a run-time value)
        int nrec = 0;
        {
            const int lane = opaque(lane_id), n32 = lane & 31, h = lane >> 5;
            uint32_t todo = flagged_tiles;
            while (todo) {
                const int nt = __builtin_ctz(todo);
                todo &= todo - 1;
                // a batch of queued rows that may not fit one more tile is resolved first
                if (nrec + 32 > kRecCap) {
                    resolve_queue<DK>(Q, nrec, U.mu64T, U.ojf, KP, k, d);
                    nrec = 0;
                }
                const uint32_t live32 = live_rows(nt);
                const uint32_t cand = ~Q.seen()[nt * 64 + lane];       // bit 31 = position 0
                uint32_t cand_lo, cand_hi;
                both_halves(cand, cand_lo, cand_hi);
                const int total = __popc(cand_lo) + __popc(cand_hi);
                const bool live = (live32 >> n32) & 1u;
                const bool flagged = live && total != 1;
                const uint64_t fm = __ballot(flagged) & 0xFFFFFFFFull;
                if (fm) {
                    half8 bt[NS];
                    rows_of_tile(nt, bt);
                    if (flagged) {
                        const int rs = nrec + __popcll(fm & ((1ull << n32) - 1ull));
#pragma unroll
                        for (int f = 0; f < NS; ++f)
                            *reinterpret_cast<half8 *>(Q.rec_x() + (size_t)rs * DK + 16 * f + 8 * h) = bt[f];
                        // no candidate at all cannot happen (the smallest score is always one); if it does, every centroid is one
                        Q.rec_mask()[rs * 2 + h] = total ? cand : 0xFFFFFFFFu;
                        if (h == 0) Q.rec_pid()[rs] = (unsigned short)(nt * 32 + n32);
                    }
                    nrec += __popcll(fm);
                }
            }
            if (nrec) resolve_queue<DK>(Q, nrec, U.mu64T, U.ojf, KP, k, d);
        }
        force_tiles = flagged_tiles;

        // ---- label changes of the decided tiles -> integer sums and counts.
        // A row without a label yet has previous = 0xFF; rows outside the task keep 0xFF and never change.
        int wave_changed = 0;
        if (full_mode) {
            // the new labels become the current ones; the sums are rebuilt from all of them
            const int lane = opaque(lane_id), n32 = lane & 31, h = lane >> 5;
            uint32_t todo = changed_tiles;
            while (todo) {
                const int nt = __builtin_ctz(todo);
                todo &= todo - 1;
                const uint32_t cur = Q.lab_new()[nt * 32 + n32];
                const uint32_t prev = Q.lab()[nt * 32 + n32];
                const bool changed = cur != prev;
                wave_changed += __popcll(__ballot(changed) & 0xFFFFFFFFull);
                if (changed && h == 0) Q.lab()[nt * 32 + n32] = (unsigned char)cur;
            }
            __builtin_amdgcn_wave_barrier();
            if (wave_live) {
                const int left = nrows - wave_row0;
                full_sums<DK, NTW / 2>(Q, U.S, U.n, xw, a.ld, d, k, left < NTW * 32 ? left : NTW * 32, lane);
            }
        } else {
            // a dense queue of (previous, new, knob values), applied with one lane per (row, group of four
            // knobs), in batches of at most kRecCap rows
            const int lane = opaque(lane_id), n32 = lane & 31, h = lane >> 5;
            (void)lane;
            uint32_t todo = changed_tiles;
            int cnt = 0;
            while (todo) {
                const int nt = __builtin_ctz(todo);
                todo &= todo - 1;
                const uint32_t cur = Q.lab_new()[nt * 32 + n32];
                const uint32_t prev = Q.lab()[nt * 32 + n32];
                const bool changed = cur != prev;
                const uint64_t cm = __ballot(changed) & 0xFFFFFFFFull;
                if (cm) {
                    if (cnt + 32 > kRecCap) {
                        apply_changes<DK>(Q, cnt, U.S, U.n, U.dirty, U.ojf, d, it);
                        cnt = 0;
                    }
                    half8 bt[NS];
                    rows_of_tile(nt, bt);
                    if (changed) {
                        const int rs = cnt + __popcll(cm & ((1ull << n32) - 1ull));
#pragma unroll
                        for (int f = 0; f < NS; ++f)
                            *reinterpret_cast<half8 *>(Q.rec_x() + (size_t)rs * DK + 16 * f + 8 * h) = bt[f];
                        if (h == 0) {
                            Q.rec_mask()[rs] = cur | (prev << 8);
                            Q.lab()[nt * 32 + n32] = (unsigned char)cur;
                        }
                    }
                    cnt += __popcll(cm);
                    wave_changed += __popcll(cm);
                }
            }
            if (cnt) apply_changes<DK>(Q, cnt, U.S, U.n, U.dirty, U.ojf, d, it);
        }
        if (wave_changed && lane_id == 0) atomicAdd(&U.stamp[2 + (it & 1)], wave_changed);
        traced_last = false;
        if (a.trace) {
            wave_loss((it & 1) * 8);
            traced_last = true;
        }
        __syncthreads();
        if (a.trace && tid == 0) {
            double s = 0.0;
            for (int w = 0; w < nwaves; ++w) s = s + U.red[(it & 1) * 8 + w];
            a.trace[slot * (a.n_iter + 1) + it] = s;
        }
        // A pass that moved no row leaves every sum, hence every centroid, as it was: the labels are
        // final.  (The count is read between this pass's two barriers, or after its only one when the
        // loop ends here; no wave adds to it in between.)
        const int rows_changed = __builtin_amdgcn_readfirstlane(U.stamp[2 + (it & 1)]);
        at_fixed_point = rows_changed == 0;
        if (last_pass || rows_changed == 0) break;
        if (tid == 0) U.stamp[2 + ((it + 1) & 1)] = 0;      // the next pass counts from zero (nobody adds before the barrier below)
        const bool full_next = x_aligned && rows_changed > full_above;
        update_centroids<DK, kByteKnobs>(U, k, KP, d, it, false, full_mode, full_next);
        full_mode = full_next;
        __syncthreads();
    }

    // ---- results: labels, loss, centroids, counts
    if (wave_live) {
        for (int e = lane; e < NTW * 32; e += 64) {
            const int pid = wave_row0 + e;
            if (pid < nrows) labrow[r0 + pid] = Q.lab()[e];
        }
    }
    // the loss of the final labels: the per-wave sums of the last traced pass are still in place
    int loss_slot = ((passes_run - 1) & 1) * 8;
    double loss = 0.0;
    if (kByteKnobs && !traced_last && at_fixed_point) {
        // At a fixed point every non-empty centroid is the mean S / n of its cluster, so the loss is
        // sum_rows |x|^2 - sum_c |S_c|^2 / n_c, all integers but the last division: with
        // |S_c|^2 = q_c n_c + r_c it is the integer (sum |x|^2 - sum q_c) minus the sum of the fractions
        // r_c / n_c, which is exact up to the rounding of those k fractions and of the final
        // subtraction (and exactly zero when every cluster's rows coincide).  The sums left by a
        // pass that rebuilt them on the matrix cores are still raised by 1024 n.
        double *frac0 = WaveQueue<DK>(U.wave_base).few();     // the queues are idle: [k] doubles of the first wave's region
        for (int c = tid; c < k; c += blockDim.x) {
            const int nc = U.n[c];
            double fr = 0.0;
            if (nc > 0) {
                unsigned long long ss = 0;
                for (int j = 0; j < d; ++j) {
                    const long long sv = (long long)U.S[c * (DK + 1) + j] - (full_mode ? 1024ll * nc : 0ll);
                    ss += (unsigned long long)(sv * sv);
                }
                const unsigned long long qc = ss / (unsigned long long)nc;
                const unsigned long long rc = ss - qc * (unsigned long long)nc;
                atomicAdd(&U.acc64[1], qc);
                fr = (double)rc / (double)nc;
            }
            frac0[c] = fr;
        }
        __syncthreads();
        if (tid == 0) {
            double fsum = 0.0;
            for (int c = 0; c < k; ++c) fsum = fsum + frac0[c];
            loss = (double)(U.acc64[0] - U.acc64[1]) - fsum;
        }
    } else {
        if (!traced_last) {
            loss_slot = 0;
            wave_loss(0);
            __syncthreads();
        }
        if (tid == 0)
            for (int w = 0; w < nwaves; ++w) loss = loss + U.red[loss_slot + w];
    }
    if (a.trace && tid == 0) {
        // the passes that were not run would have seen the same labels and centroids
        for (int it = passes_run; it <= a.n_iter; ++it) a.trace[slot * (a.n_iter + 1) + it] = loss;
    }
    for (int e = tid; e < k * d; e += blockDim.x) {
        const int c = e / d, j = e % d;
        a.centroids[(crow + c) * d + j] = U.mu64T[(size_t)j * KP + c];
    }
    for (int c = tid; c < k; c += blockDim.x) a.counts[crow + c] = U.n[c];
    if (tid == 0) {
        a.status[slot] = 0;
        a.inertia[slot] = loss;
        a.passes[slot] = passes_run;
    }
}

// Persistent workgroups (one per compute unit) take units from a counter until none is left: the
// next unit starts as soon as the last one ends, without a new dispatch of a workgroup of this size.
// Units are handed out in descending-k order so that the longest ones start first.
template <int DK, int NTW, typename XT>
__global__ __launch_bounds__(512) void resident_mfma_kernel(const SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    __shared__ int next_unit;
    const int tid = threadIdx.x;
    const int n_units = a.T * (a.ki_end - a.ki_begin);

    if (tid == 0) next_unit = atomicAdd(a.unit_counter, 1);
    for (;;) {
        __syncthreads();
        const int u = __builtin_amdgcn_readfirstlane(next_unit);     // uniform: what derives from it lives in scalar registers
        __syncthreads();                           // everyone has read it before it is written again
        if (u >= n_units) break;
        // the unit after this one is asked for now; the answer is needed when this one is done
        int after = 0;
        if (tid == 0) after = atomicAdd(a.unit_counter, 1);
        const int ki = a.ki_end - 1 - u / a.T;
        const int t = u % a.T;
        const int k = a.ks[ki];
        const bool skipped = a.done && a.done[t];     // the task's sweep stopped at a smaller k
        const bool too_large = a.too_large && *a.too_large != 0;     // a two-byte value the f16 rows cannot hold

        if (skipped || too_large || (a.init_mode == 0 && a.ndist[t] < k)) {
            // fewer than k distinct rows, not needed any more, or unusable input: all outputs zero, status says which
            const int d = a.d;
            const int64_t r0 = a.task_off[t], r1 = a.task_off[t + 1];
            const int64_t slot = (int64_t)t * a.n_k + ki;
            const int64_t crow = (int64_t)t * a.Ksum + a.koff[ki];
            uint8_t *labrow = a.labbuf + (int64_t)ki * a.ld;
            for (int e = tid; e < k * d; e += blockDim.x) a.centroids[crow * d + e] = 0.0;
            for (int c = tid; c < k; c += blockDim.x) a.counts[crow + c] = 0;
            for (int64_t r = r0 + tid; r < r1; r += blockDim.x) labrow[r] = 0;
            if (tid == 0) {
                a.status[slot] = too_large ? 4 : (skipped ? 3 : 1);
                a.passes[slot] = 0;
                a.inertia[slot] = 0.0;
            }
            if (a.trace)
                for (int e = tid; e <= a.n_iter; e += blockDim.x) a.trace[slot * (a.n_iter + 1) + e] = 0.0;
        } else {
            run_unit<DK, NTW, XT>(a, smem, ki, t, k);
        }
        if (tid == 0) next_unit = after;            // (read by everyone after the barrier at the loop's head)
    }
}

template <int DK, int NTW, typename XT>
hipError_t launch_mfma_t(const SweepArgs &a, int nwaves, int64_t n_total, hipStream_t s)
{
    const unsigned pb = (unsigned)((n_total + 255) / 256);
    if (pb && a.ki_begin == 0)
        hipLaunchKernelGGL((pack_rows_kernel<DK, XT>), dim3(pb), dim3(256), 0, s, reinterpret_cast<const XT *>(a.X), a.ld, a.d,
                           n_total, reinterpret_cast<_Float16 *>(a.xh), a.too_large);
    const int KP = a.kmax > 32 ? 64 : 32;
    const size_t lds = MfmaLds<DK>::bytes(KP, nwaves, NTW);
    auto kern = resident_mfma_kernel<DK, NTW, XT>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    // as many workgroups as can be resident at once
    int dev = 0, cus = 0, per_cu = 0;
    e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return e;
    e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, nwaves * 64, lds);
    if (e != hipSuccess) return e;
    if (per_cu < 1) per_cu = 1;
    const unsigned units = (unsigned)a.T * (unsigned)(a.ki_end - a.ki_begin);
    unsigned grid = (unsigned)cus * (unsigned)per_cu;
    if (grid > units) grid = units;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(nwaves * 64), lds, s, a);
    return hipGetLastError();
}

}  // namespace

// One knob slot stays free for the bias.  Byte knobs: d <= 31, k <= 64, tasks of at most 4096 rows.
bool mfma_path_fits(int d, int kmax, int64_t n_max)
{
    return d >= 1 && d <= 31 && kmax <= 64 && n_max <= 4096;
}

// Two-byte knobs whose values the caller promises to be below 2048: the same limits up to 31 knobs;
// up to 63 knobs in 64-wide rows, which leave registers for 2048 rows and one tile of 32 centroids.
bool mfma_path_fits_u16(int d, int kmax, int64_t n_max)
{
    if (mfma_path_fits(d, kmax, n_max)) return true;
    return d >= 1 && d <= 63 && kmax <= 32 && n_max <= 2048;
}

template <typename XT>
static hipError_t launch_mfma_sweep_t(const SweepArgs &a, int64_t n_max, int64_t n_total, hipStream_t s)
{
    const int DK = a.d <= 15 ? 16 : (a.d <= 31 ? 32 : 64);
    const int ntw = n_max <= 1024 ? 4 : (DK == 64 ? 8 : 16);
    int nwaves = (int)((n_max + 32 * ntw - 1) / (32 * ntw));
    if (nwaves < 1) nwaves = 1;
    if (nwaves > 8) nwaves = 8;
    if (DK == 16) return ntw == 4 ? launch_mfma_t<16, 4, XT>(a, nwaves, n_total, s) : launch_mfma_t<16, 16, XT>(a, nwaves, n_total, s);
    if (DK == 32) return ntw == 4 ? launch_mfma_t<32, 4, XT>(a, nwaves, n_total, s) : launch_mfma_t<32, 16, XT>(a, nwaves, n_total, s);
    if (sizeof(XT) == 1) return hipErrorInvalidValue;        // (byte knobs never come with more than 32 knobs)
    return ntw == 4 ? launch_mfma_t<64, 4, uint16_t>(a, nwaves, n_total, s) : launch_mfma_t<64, 8, uint16_t>(a, nwaves, n_total, s);
}

hipError_t launch_mfma_sweep(const SweepArgs &a, int64_t n_max, int64_t n_total, hipStream_t s)
{
    if (a.xbytes == 2) return launch_mfma_sweep_t<uint16_t>(a, n_max, n_total, s);
    return launch_mfma_sweep_t<uint8_t>(a, n_max, n_total, s);
}

}  // namespace cham
