// Streaming variant of the sweep for tasks too large to stay on one compute unit
// (paper Algorithm 1, K-means.run(s_Theta, k); Sec. 3.3): every Lloyd pass is one launch of
// stream_assign_kernel over (unit, row chunk) workgroups followed by one launch of
// stream_update_kernel over units.  Labels, integer sums and counts live in global memory and are
// updated incrementally (a row touches the sums only when its label changes: exact, integers).
//
// The screen is an f16 hi/lo matrix-core screen as in the resident kernel, for up to 256
// centroids, with every knob slot of the fragments holding a knob (d <= 16 takes one 16-wide
// step per part): |mu'|^2 enters as the initial value of the accumulator, in fp32.  Centroids
// are taken in chunks of 64 (two 32-row m-tiles); one sweep over the chunks leaves, per chunk, the
// minimum score of every row and the scores within the error bound of that minimum, and the chunks
// whose minimum lies within the bound of the overall minimum contribute their marks.  A row with
// exactly one marked score is decided; any other row is re-evaluated in double against its marked
// centroids (one lane per (row, centroid) pair; knobs ascending, no fused multiply-add, lowest
// index on ties), or against all k centroids when the pairs do not fit.
#include "cham_device.h"
#include "cham_internal.h"
#include "mfma_common.h"

namespace cham {

namespace {

constexpr int kMaxTiles = 8;         // 32-row tiles a wave handles per step, at most
constexpr int kStepRows = kMaxTiles * 32;
constexpr int kStreamRec = 32;       // queued rows whose knob values are kept in LDS
constexpr int kWavesPerWg = 4;
constexpr int kPairCap = 128;        // (queued row, candidate centroid) pairs evaluated per step and wave
constexpr float kPadScore = 1.0e30f; // score of a padding centroid row (real scores stay below 4 * 32 * 255^2)

// Per-unit state in global memory.  KPM = kmax rounded up to 32.
struct UnitState {
    int *S;            // [KPM][32]      integer sums
    int *n;            // [KPM]          counts
    double *mu;        // [32][KPM]      exact centroids, transposed
    half8 *afrag;      // [KPM/32][4][64] A fragments (hi steps then lo steps; NS2 <= 4)
    float *bias;       // [KPM]          |mu'|^2 (fp32), huge for padding rows: initial accumulator values
};

__device__ __forceinline__ UnitState unit_state(const StreamArgs &a, int u)
{
    UnitState s;
    const size_t kpm = (size_t)a.kpm;
    s.S = a.Sg + (size_t)u * kpm * 32;
    s.n = a.ng + (size_t)u * kpm;
    s.mu = a.mu + (size_t)u * 32 * kpm;
    s.afrag = reinterpret_cast<half8 *>(a.afrag) + (size_t)u * (kpm / 32) * 4 * 64;
    s.bias = a.biasf + (size_t)u * kpm;
    return s;
}

// Centring offsets per task: rounded mean of the starting centroids of the largest k.
__global__ void stream_offsets_kernel(const StreamArgs a)
{
    const int t = blockIdx.x;
    const int j = threadIdx.x;
    if (j >= 32) return;
    float o = 0.0f;
    if (j < a.d) {
        double s = 0.0;
        int cnt = 0;
        if (a.init_mode == 0) {
            cnt = a.ndist[t] < a.kmax ? a.ndist[t] : a.kmax;
            const int64_t r0 = a.task_off[t];
            for (int c = 0; c < cnt; ++c) s += (double)a.X[(int64_t)j * a.ld + r0 + a.init_rows[(int64_t)t * a.kmax + c]];
        } else {
            cnt = a.kmax;
            const int64_t crow = (int64_t)t * a.Ksum + a.koff[a.n_k - 1];
            for (int c = 0; c < cnt; ++c) s += a.init_centroids[(crow + c) * a.d + j];
        }
        double m = cnt > 0 ? rint(s / (double)cnt) : 0.0;
        m = m < 0.0 ? 0.0 : (m > 255.0 ? 255.0 : m);
        o = (float)m;
    }
    a.ojf[t * 32 + j] = o;
}

// Centred f16 copy of the rows (row-major, DK halfs per row, absent knobs zero) and the squared
// norm of every centred row.
template <int DK>
__global__ void stream_pack_kernel(const StreamArgs a, int64_t n_rows)
{
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_rows) return;
    int lo = 0, hi = a.T;                      // task of row r: last t with task_off[t] <= r
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.task_off[mid] <= r) lo = mid; else hi = mid;
    }
    const float *o = a.ojf + lo * 32;
    float x2 = 0.0f;
    _Float16 *dst = reinterpret_cast<_Float16 *>(a.xh) + r * DK;
#pragma unroll
    for (int g = 0; g < DK / 8; ++g) {
        half8 v;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int j = 8 * g + i;
            float f = 0.0f;
            if (j < a.d) f = (float)a.X[(int64_t)j * a.ld + r] - o[j];
            x2 = __builtin_fmaf(f, f, x2);
            v[i] = (_Float16)f;
        }
        *reinterpret_cast<half8 *>(dst + 8 * g) = v;
    }
    a.x2[r] = x2;
}

// mode 0: start of the sweep (centroids from the first distinct rows or from the caller);
// mode 1: centroid update after pass a.it; mode 2: outputs after the final pass.
// Grid: (unit, tile of 32 centroids); a thread per (centroid of the tile, group of 8 knobs).  The
// bound on max |mu'|^2 is kept per tile: m2[unit][tile], tile 0 negative = unit unusable.
constexpr int kM2Tiles = 8;            // k <= 256
template <int DK>
__global__ __launch_bounds__(32 * (DK / 8)) void stream_update_kernel(const StreamArgs a, int mode)
{
    constexpr int NS = DK / 16, G = DK / 8;
    __shared__ float red[32 * G / 64 + 1];
    const int ul = blockIdx.x;                 // unit within this launch
    const int mt = blockIdx.y;                 // tile of 32 centroids
    const int u = a.u_begin + ul;
    const int ki = a.n_k - 1 - u / a.T;
    const int t = u % a.T;
    const int k = a.ks[ki];
    const int d = a.d;
    const int tid = threadIdx.x;
    const int64_t slot = (int64_t)t * a.n_k + ki;
    const int64_t crow = (int64_t)t * a.Ksum + a.koff[ki];
    const int64_t r0 = a.task_off[t], r1 = a.task_off[t + 1];
    const UnitState st = unit_state(a, u);
    const int kpm = a.kpm;
    const bool skipped = a.done && a.done[t];  // the task's sweep stopped at a smaller k
    const bool unusable = skipped || (a.init_mode == 0 && a.ndist[t] < k);

    if (unusable) {
        if (mt != 0) return;
        if (mode == 0 && tid == 0) a.m2[u * kM2Tiles] = -1.0f;
        if (mode == 2) {
            for (int e = tid; e < k * d; e += blockDim.x) a.centroids[crow * d + e] = 0.0;
            for (int c = tid; c < k; c += blockDim.x) a.counts[crow + c] = 0;
            uint8_t *labrow = a.labbuf + (int64_t)ki * a.ld;
            for (int64_t r = r0 + tid; r < r1; r += blockDim.x) labrow[r] = 0;
            if (tid == 0) {
                a.status[slot] = skipped ? 3 : 1;
            a.passes[slot] = 0;
                a.inertia[slot] = 0.0;
            }
            if (a.trace)
                for (int e = tid; e <= a.n_iter; e += blockDim.x) a.trace[slot * (a.n_iter + 1) + e] = 0.0;
        }
        return;
    }

    // loss of the pass that just ran: workgroup partials in workgroup order
    if (mt == 0 && mode != 0 && tid == 0 && (mode == 2 || a.trace)) {
        const int nwg = a.wg_off[ul + 1] - a.wg_off[ul];
        double s = 0.0;
        for (int w = 0; w < nwg; ++w) s = s + a.loss_part[(size_t)a.wg_off[ul] + w];
        if (a.trace) a.trace[slot * (a.n_iter + 1) + a.it] = s;
        if (mode == 2) {
            a.inertia[slot] = s;
            a.status[slot] = 0;
        }
    }
    const int kpu = (k + 31) & ~31;
    if (mt * 32 >= kpu) return;                // no such tile in this unit
    if (mode == 2) {
        for (int e = tid; e < 32 * d; e += blockDim.x) {
            const int c = mt * 32 + e / d, j = e % d;
            if (c < k) a.centroids[(crow + c) * d + j] = st.mu[(size_t)j * kpm + c];
        }
        for (int c = mt * 32 + tid; c < k && c < mt * 32 + 32; c += blockDim.x) a.counts[crow + c] = st.n[c];
        return;
    }

    const float *o = a.ojf + t * 32;
    const int m32 = tid / G, g = tid % G;
    const int c = mt * 32 + m32;
    if (mode == 0) {
        if (g == 0) st.n[c] = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) st.S[c * 32 + 8 * g + i] = 0;
        if (DK == 16) {
#pragma unroll
            for (int i = 0; i < 8; ++i) st.S[c * 32 + 16 + 8 * g + i] = 0;
        }
    }
    const int cnt = (mode == 1 && c < k) ? st.n[c] : 0;
    double b = 0.0;
    half8 hi8, lo8;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int j = 8 * g + i;
        double m = 0.0;
        if (c < k && j < d) {
            double mu;
            if (mode == 0) {
                if (a.init_mode == 0) mu = (double)a.X[(int64_t)j * a.ld + r0 + a.init_rows[(int64_t)t * a.kmax + c]];
                else mu = a.init_centroids[(crow + c) * d + j];
                st.mu[(size_t)j * kpm + c] = mu;
            } else if (cnt > 0) {
                mu = (double)st.S[c * 32 + j] / (double)cnt;      // an empty cluster keeps its centroid
                st.mu[(size_t)j * kpm + c] = mu;
            } else {
                mu = st.mu[(size_t)j * kpm + c];
            }
            m = mu - (double)o[j];
        } else if (mode == 0 && c < k) {
            st.mu[(size_t)j * kpm + c] = 0.0;
        }
        b = __builtin_fma(m, m, b);
        const float w = (float)(-2.0 * m);
        const _Float16 hi = (_Float16)w;
        hi8[i] = hi;
        lo8[i] = (_Float16)(w - (float)hi);
    }
    // |mu'|^2 over all knob groups of the centroid (the G lanes of a centroid are neighbours)
#pragma unroll
    for (int off = G / 2; off >= 1; off >>= 1) b = b + __shfl_xor(b, off, 64);
    // |mu'|^2 starts the accumulator; padding centroid rows get a score above all others
    if (g == G - 1) st.bias[c] = c < k ? (float)b : kPadScore;
    const int hh = g & 1, fstep = g >> 1;
    st.afrag[(mt * 4 + fstep) * 64 + 32 * hh + m32] = hi8;
    st.afrag[(mt * 4 + NS + fstep) * 64 + 32 * hh + m32] = lo8;

    float bmax = c < k ? __double2float_ru(b) * 1.0000005f : 0.0f;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) bmax = __builtin_fmaxf(bmax, __shfl_xor(bmax, off, 64));
    if ((tid & 63) == 0) red[tid >> 6] = bmax;
    __syncthreads();
    if (tid == 0) {
        float m = 0.0f;
        for (int i = 0; i < (int)(blockDim.x + 63) / 64; ++i) m = __builtin_fmaxf(m, red[i]);
        a.m2[u * kM2Tiles + mt] = m;
    }
}

template <int DK>
struct StreamLds {
    half8 *afrag;        // [KPM/32][4][64]
    int *S;              // [KPM][DK] changes of the sums made by this workgroup
    int *n;              // [KPM]
    float *ojf;          // [DK]
    float *bias;         // [KPM]
    double *red;         // [8]
    unsigned char *wave_base;
    // per wave: knob values of queued rows, their row slots, resolved labels, labels of the step
    // ... and for the exact evaluation of queued rows: (record, centroid) pairs, per record the
    // smallest distance (bits) and the lowest centroid attaining it, the pair counter
    static constexpr size_t kWaveBytes = (size_t)kStreamRec * DK * 2 + kStepRows * 2 + kStepRows + kStepRows +
                                         kStreamRec * 4 + kPairCap * 2 + kStepRows * 8 + kStepRows * 4 + 16;
    __host__ __device__ static size_t bytes(int kpm)
    {
        size_t b = 16 * (size_t)(kpm / 32) * 4 * 64 + sizeof(int) * (size_t)kpm * DK + sizeof(int) * kpm +
                   sizeof(float) * DK + sizeof(float) * kpm + sizeof(double) * 8 + 16;
        b = (b + 15) & ~(size_t)15;
        return b + ((kWaveBytes + 15) & ~(size_t)15) * kWavesPerWg;
    }
    __device__ StreamLds(unsigned char *base, int kpm)
    {
        size_t o = 0;
        afrag = reinterpret_cast<half8 *>(base + o);  o += 16 * (size_t)(kpm / 32) * 4 * 64;
        red = reinterpret_cast<double *>(base + o);   o += sizeof(double) * 8;
        S = reinterpret_cast<int *>(base + o);        o += sizeof(int) * (size_t)kpm * DK;
        n = reinterpret_cast<int *>(base + o);        o += sizeof(int) * kpm;
        ojf = reinterpret_cast<float *>(base + o);    o += sizeof(float) * DK;
        o = (o + 15) & ~(size_t)15;
        bias = reinterpret_cast<float *>(base + o);   o += sizeof(float) * kpm;
        o = (o + 15) & ~(size_t)15;
        wave_base = base + o;
    }
};

// One (unit, row chunk) workgroup of the assignment.  NCH = chunks of 64 centroids of the unit
// (compiled for 1, 2 or 4), TILES = 32-row tiles a wave handles per step: the more rows a step
// holds, the fewer chains of dependent short phases (decision, exact evaluation, label changes) a
// workgroup goes through, within what the registers hold beside the per-chunk marks.
template <int DK, int NCH, int TILES>
__device__ __forceinline__ void assign_unit(const StreamArgs &a, int unit_idx)
{
    constexpr int NS = DK / 16, NS2 = 2 * NS;
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int n32 = lane & 31;
    const int h = lane >> 5;
    const int wgi = blockIdx.x - a.wg_off[unit_idx];
    const int u = a.u_begin + unit_idx;
    const int ki = a.n_k - 1 - u / a.T;
    const int t = u % a.T;
    const int k = a.ks[ki];
    const int d = a.d;
    const int kpm = a.kpm;
    const int kpu = (k + 31) & ~31;
    float m2 = a.m2[u * kM2Tiles];
    if (m2 < 0.0f) return;                     // unusable unit (fewer than k distinct rows)
    for (int i = 1; i < kpu / 32; ++i) m2 = __builtin_fmaxf(m2, a.m2[u * kM2Tiles + i]);
    const UnitState st = unit_state(a, u);
    StreamLds<DK> L(smem, kpm);

    const int64_t t0 = a.task_off[t], t1 = a.task_off[t + 1];
    const int64_t rpw = stream_rows_per_wg(k);
    const int64_t r0 = t0 + (int64_t)wgi * rpw;
    const int64_t r1 = (r0 + rpw < t1) ? r0 + rpw : t1;
    uint8_t *labrow = a.labbuf + (int64_t)ki * a.ld;
    const bool first = a.it == 0;
    const bool want_dist = a.final_pass || (a.trace != nullptr);
    unsigned char *wb = L.wave_base + ((StreamLds<DK>::kWaveBytes + 15) & ~(size_t)15) * wave;
    _Float16 *rec_x = reinterpret_cast<_Float16 *>(wb);                                          // [kStreamRec][DK]
    unsigned short *rec_slot = reinterpret_cast<unsigned short *>(wb + (size_t)kStreamRec * DK * 2);   // [kStepRows]
    unsigned char *lab_res = wb + (size_t)kStreamRec * DK * 2 + kStepRows * 2;                    // [kStepRows]
    unsigned char *lab_new = lab_res + kStepRows;                                                  // [kStepRows]
    unsigned *chg = reinterpret_cast<unsigned *>(lab_new + kStepRows);                             // [kStreamRec] cur | prev << 8 | first << 16
    unsigned short *pairs = reinterpret_cast<unsigned short *>(chg + kStreamRec);                  // [kPairCap] record << 8 | centroid
    unsigned long long *best_bits = reinterpret_cast<unsigned long long *>(pairs + kPairCap);      // [kStepRows]
    int *best_c = reinterpret_cast<int *>(best_bits + kStepRows);                                  // [kStepRows]
    unsigned *npairs = reinterpret_cast<unsigned *>(best_c + kStepRows);

    const _Float16 *xh = reinterpret_cast<const _Float16 *>(a.xh);
    const int nch = (k + 63) >> 6;
    double part = 0.0;

    const int64_t step_rows = (int64_t)kWavesPerWg * TILES * 32;

    // rows of one step of this wave: B fragments, squared norms, previous labels
    struct StepRows {
        half8 B[TILES][NS];
        float x2[TILES];
        int prev[TILES];
    };
    auto load_step = [&](int64_t wrow0, StepRows &R) {
#pragma unroll
        for (int tt = 0; tt < TILES; ++tt) {
            const int64_t row = wrow0 + tt * 32 + n32;
            const bool lv = row < r1;
            const int64_t rr = lv ? row : (wrow0 < r1 ? wrow0 : r0);     // a valid row either way
#pragma unroll
            for (int f = 0; f < NS; ++f) {
                half8 v = *reinterpret_cast<const half8 *>(xh + rr * DK + 16 * f + 8 * h);
                if (!lv) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) v[i] = (_Float16)0.0f;
                }
                R.B[tt][f] = v;
            }
            R.x2[tt] = a.x2[rr];
            R.prev[tt] = first ? 0 : (int)labrow[rr];
        }
    };

    StepRows nxt;
    if (r0 < r1) load_step(r0 + (int64_t)wave * TILES * 32, nxt);    // under way during the set-up below

    for (int e = tid; e < (kpu / 32) * NS2 * 64; e += blockDim.x) {      // the NS2 slots in use of every m-tile
        const int src = (e / (NS2 * 64)) * 4 * 64 + e % (NS2 * 64);
        L.afrag[src] = st.afrag[src];
    }
    for (int e = tid; e < kpu; e += blockDim.x) L.bias[e] = st.bias[e];
    for (int e = tid; e < k * DK; e += blockDim.x) L.S[e] = 0;
    for (int c = tid; c < k; c += blockDim.x) L.n[c] = 0;
    if (tid < DK) L.ojf[tid] = tid < 32 ? a.ojf[t * 32 + tid] : 0.0f;
    __syncthreads();

    for (int64_t base = r0; base < r1; base += step_rows) {
        const int64_t wrow0 = base + (int64_t)wave * TILES * 32;      // first row of this wave's step
        const StepRows cur = nxt;
        if (base + step_rows < r1) load_step(wrow0 + step_rows, nxt);  // next step's rows load under this step
        if (wrow0 >= r1) continue;                                      // wave-uniform
        bool live[TILES];
#pragma unroll
        for (int tt = 0; tt < TILES; ++tt) live[tt] = (wrow0 + tt * 32 + n32) < r1;

        constexpr int kMaxCh = NCH;                  // chunks of 64 centroids
        int cnt[TILES], candq[TILES];
        uint32_t cmask[TILES][kMaxCh];             // candidate centroids of this lane half, per chunk
#pragma unroll
        for (int tt = 0; tt < TILES; ++tt) {
            cnt[tt] = 0;
            candq[tt] = 0;
#pragma unroll
            for (int ch = 0; ch < kMaxCh; ++ch) cmask[tt][ch] = 0u;
        }
        if (lane == 0) *npairs = 0u;
        // fragments of the two m-tiles of chunk ch and the initial accumulator values (|mu'|^2 of the
        // centroid rows this lane's registers belong to: rows 8 g + 4 h + (0..3) for registers 4 g + (0..3))
        auto load_a = [&](int ch, bool has1, half8 (&A0)[NS2], half8 (&A1)[NS2], float16v &c0, float16v &c1) {
#pragma unroll
            for (int s = 0; s < NS2; ++s) {
                A0[s] = L.afrag[((2 * ch) * 4 + s) * 64 + lane];        // slots 0..NS-1 hi parts, NS..2NS-1 lo parts
                A1[s] = has1 ? L.afrag[((2 * ch + 1) * 4 + s) * 64 + lane] : A0[s];
            }
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float4 b0 = *reinterpret_cast<const float4 *>(L.bias + (2 * ch) * 32 + 8 * g + 4 * h);
                const float4 b1 = has1 ? *reinterpret_cast<const float4 *>(L.bias + (2 * ch + 1) * 32 + 8 * g + 4 * h) : b0;
                c0[4 * g + 0] = b0.x; c0[4 * g + 1] = b0.y; c0[4 * g + 2] = b0.z; c0[4 * g + 3] = b0.w;
                c1[4 * g + 0] = b1.x; c1[4 * g + 1] = b1.y; c1[4 * g + 2] = b1.z; c1[4 * g + 3] = b1.w;
            }
        };
        // one matrix instruction of the chain of a 32x32 tile
        auto mma = [&](float16v &acc, const half8 (&Af)[NS2], const half8 (&Bt)[NS], const float16v &cinit, int s) {
            acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(Af[s], Bt[s % NS], s == 0 ? cinit : acc, 0, 0, 0);
        };
        auto min16 = [&](const float16v &acc) {
            float m = min3f(acc[0], acc[1], acc[2]);
#pragma unroll
            for (int i = 3; i < 15; i += 2) m = min3f(m, acc[i], acc[i + 1]);
            return __builtin_fminf(m, acc[15]);
        };
        // mark scores [i0, i0 + CH): bit set = above the threshold
        constexpr int CH = 16 / NS2;
        auto mark = [&](uint32_t &far, const float16v &acc, float thr, int i0) {
#pragma unroll
            for (int i = 0; i < CH; ++i)
                far = __builtin_amdgcn_alignbit(far, __float_as_uint(thr - acc[i0 + i]), 31);
        };

        // One sweep over the chunks of 64 centroids.  Every chunk leaves its own minimum (over both
        // lane halves) and the marks within the bound of that minimum; afterwards a chunk's marks
        // count iff its minimum lies within the bound of the overall minimum.  The centroids
        // within the bound of the overall minimum are all among them (their chunk's minimum is
        // no larger than their score), at worst joined by some up to two bounds away, which
        // only sends a few more rows to the exact evaluation.  Within a chunk the tiles are
        // pipelined: the chain of the next tile is issued under the marking of the current one.
        float bch[TILES][kMaxCh];
        float bnd[TILES];
#pragma unroll
        for (int tt = 0; tt < TILES; ++tt) bnd[tt] = mfma_bound<NS2>(cur.x2[tt], m2);
#pragma unroll
        for (int ch = 0; ch < kMaxCh; ++ch) {
            if (ch < nch) {
                const bool has1 = (2 * ch + 1) * 32 < kpu;
                half8 A0[NS2], A1[NS2];
                float16v cin0, cin1;
                load_a(ch, has1, A0, A1, cin0, cin1);
                float16v accA, accB;
                constexpr int kLast = TILES - 1;
                if (has1) {
                    // accA = centroids 0..31, accB = centroids 32..63 of the chunk
#pragma unroll
                    for (int s = 0; s < NS2; ++s) mma(accA, A0, cur.B[0], cin0, s);
#pragma unroll
                    for (int s = 0; s < NS2; ++s) mma(accB, A1, cur.B[0], cin1, s);
#pragma unroll
                    for (int tt = 0; tt < TILES; ++tt) {
                        const int nx = tt < kLast ? tt + 1 : tt;
                        const float m = min_halves(__builtin_fminf(min16(accA), min16(accB)));
                        const float thr = m + bnd[tt];
                        uint32_t far = 0;
#pragma unroll
                        for (int s = 0; s < NS2; ++s) mark(far, accA, thr, s * CH);
                        // accA is consumed: its next chain runs under the marking of accB
#pragma unroll
                        for (int s = 0; s < NS2; ++s) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (tt < kLast) mma(accA, A0, cur.B[nx], cin0, s);
                            __builtin_amdgcn_sched_barrier(0);
                            mark(far, accB, thr, s * CH);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        if (tt < kLast) {
#pragma unroll
                            for (int s = 0; s < NS2; ++s) mma(accB, A1, cur.B[nx], cin1, s);
                        }
                        bch[tt][ch] = m;
                        cmask[tt][ch] = ~far;
                        __builtin_amdgcn_sched_barrier(0);
                    }
                } else {
                    // one block of 32 centroids: the accumulators alternate
#pragma unroll
                    for (int s = 0; s < NS2; ++s) mma(accA, A0, cur.B[0], cin0, s);
#pragma unroll
                    for (int tt = 0; tt < TILES; ++tt) {
                        const int nx = tt < kLast ? tt + 1 : tt;
                        float16v &now = (tt & 1) ? accB : accA;
                        float16v &nxt2 = (tt & 1) ? accA : accB;
                        const float m = min_halves(min16(now));
                        const float thr = m + bnd[tt];
                        uint32_t far = 0;
#pragma unroll
                        for (int s = 0; s < NS2; ++s) {
                            __builtin_amdgcn_sched_barrier(0);
                            if (tt < kLast) mma(nxt2, A0, cur.B[nx], cin0, s);
                            __builtin_amdgcn_sched_barrier(0);
                            mark(far, now, thr, s * CH);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                        bch[tt][ch] = m;
                        cmask[tt][ch] = ~((far << 16) | 0xFFFFu);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            } else {
#pragma unroll
                for (int tt = 0; tt < TILES; ++tt) bch[tt][ch] = __builtin_inff();
            }
        }
#pragma unroll
        for (int tt = 0; tt < TILES; ++tt) {
            float best = bch[tt][0];
#pragma unroll
            for (int ch = 1; ch < kMaxCh; ++ch) best = __builtin_fminf(best, bch[tt][ch]);
            const float lim = best + bnd[tt];
#pragma unroll
            for (int ch = 0; ch < kMaxCh; ++ch) {
                const uint32_t cand = bch[tt][ch] <= lim ? cmask[tt][ch] : 0u;
                cnt[tt] += __popc(cand);
                candq[tt] = cand ? (ch * 32 + __clz((int)cand)) : candq[tt];
                cmask[tt][ch] = cand;
            }
        }
        // decide, or queue for the exact evaluation
        int lab[TILES];
        uint32_t flagged_mask = 0;
        int nrec = 0;
        bool no_candidate = false;          // a queued row without any candidate (cannot happen with a valid bound)
        __builtin_amdgcn_wave_barrier();    // the pair counter is zero
#pragma unroll
        for (int tt = 0; tt < TILES; ++tt) {
            unsigned c_lo, c_hi, q_lo, q_hi;
            both_halves((unsigned)cnt[tt], c_lo, c_hi);
            both_halves((unsigned)candq[tt], q_lo, q_hi);
            const int total = (int)(c_lo + c_hi);
            const int hh = c_lo ? 0 : 1;
            const int qg = (int)(c_lo ? q_lo : q_hi);
            lab[tt] = 64 * (qg >> 5) + centroid_of(qg & 31, hh);
            const bool flagged = live[tt] && total != 1;
            const uint64_t fm = __ballot(flagged) & 0xFFFFFFFFull;
            if (fm) {
                if (flagged) {
                    flagged_mask |= 1u << tt;
                    const int rs = nrec + __popcll(fm & ((1ull << n32) - 1ull));
                    if (rs < kStreamRec) {
#pragma unroll
                        for (int f = 0; f < NS; ++f)
                            *reinterpret_cast<half8 *>(rec_x + (size_t)rs * DK + 16 * f + 8 * h) = cur.B[tt][f];
                    }
                    if (h == 0) rec_slot[rs] = (unsigned short)(tt * 32 + n32);
                    // this lane half's candidates of the row join the list of (record, centroid) pairs
                    unsigned pos = atomicAdd(npairs, (unsigned)cnt[tt]);
#pragma unroll
                    for (int ch = 0; ch < kMaxCh; ++ch) {
                        uint32_t m = cmask[tt][ch];
                        while (m) {
                            const int q = __clz((int)m);
                            m &= ~(0x80000000u >> q);
                            if (pos < (unsigned)kPairCap)
                                pairs[pos] = (unsigned short)((rs << 8) | (64 * ch + centroid_of(q, h)));
                            ++pos;
                        }
                    }
                }
                no_candidate = no_candidate || (flagged && total == 0);
                nrec += __popcll(fm);
            }
        }
        __builtin_amdgcn_wave_barrier();
        const unsigned np = nrec ? *npairs : 0u;
        const bool full_eval = nrec && (np > (unsigned)kPairCap || __ballot(no_candidate) != 0ull);
        if (nrec && !full_eval) {
            // Exact evaluation of the queued rows against their candidates only: one lane per
            // (row, centroid) pair, the distance as sum_j ((double)x_j - mu_j)^2 with j ascending;
            // per row the smallest distance, then the lowest centroid attaining it.
            for (int r = lane; r < nrec; r += 64) {
                best_bits[r] = ~0ull;
                best_c[r] = 0x7fffffff;
            }
            __builtin_amdgcn_wave_barrier();
            unsigned long long mine[kPairCap / 64];
            int mine_rc[kPairCap / 64];
#pragma unroll
            for (int rd = 0; rd < kPairCap / 64; ++rd) {
                const unsigned p = rd * 64 + lane;
                mine[rd] = ~0ull;
                mine_rc[rd] = -1;
                if (p < np) {
                    const int pr = pairs[p];
                    const int r = pr >> 8, c = pr & 0xFF;
                    const int sl = rec_slot[r];
                    double sd = 0.0;
                    for (int j0 = 0; j0 < d; j0 += 8) {
                        double mu[8];
                        half8 xq;
                        if (r < kStreamRec) xq = *reinterpret_cast<const half8 *>(rec_x + (size_t)r * DK + j0);
                        else xq = *reinterpret_cast<const half8 *>(xh + (wrow0 + sl) * DK + j0);
#pragma unroll
                        for (int i = 0; i < 8; ++i) mu[i] = (j0 + i < d) ? st.mu[(size_t)(j0 + i) * kpm + c] : 0.0;
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            if (j0 + i < d) {
                                const double tq = (double)((float)xq[i] + L.ojf[j0 + i]) - mu[i];
                                sd = sd + tq * tq;
                            }
                        }
                    }
                    mine[rd] = (unsigned long long)__double_as_longlong(sd);
                    mine_rc[rd] = pr;
                    atomicMin(&best_bits[r], mine[rd]);
                }
            }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int rd = 0; rd < kPairCap / 64; ++rd) {
                if (mine_rc[rd] >= 0 && best_bits[mine_rc[rd] >> 8] == mine[rd])
                    atomicMin(&best_c[mine_rc[rd] >> 8], mine_rc[rd] & 0xFF);
            }
            __builtin_amdgcn_wave_barrier();
            for (int r = lane; r < nrec; r += 64) {
                const int bc = best_c[r];
                lab_res[rec_slot[r]] = (unsigned char)(bc < k ? bc : 0);
            }
            __builtin_amdgcn_wave_barrier();
        }
        if (nrec && full_eval) {
            // exact evaluation of the queued rows against all k centroids, one centroid per lane;
            // the centroid loads of 8 knobs are issued together
            __builtin_amdgcn_wave_barrier();
            for (int r = 0; r < nrec; ++r) {
                const int sl = rec_slot[r];
                double bs = __builtin_inf();
                int bc = 0x7fffffff;
                for (int c0 = 0; c0 < k; c0 += 64) {
                    int c = c0 + lane;
                    const int cc = c < k ? c : k - 1;
                    double s = 0.0;
                    for (int j0 = 0; j0 < d; j0 += 8) {
                        double mu[8];
                        half8 xq;
                        if (r < kStreamRec) xq = *reinterpret_cast<const half8 *>(rec_x + (size_t)r * DK + j0);
                        else xq = *reinterpret_cast<const half8 *>(xh + (wrow0 + sl) * DK + j0);
#pragma unroll
                        for (int i = 0; i < 8; ++i) mu[i] = (j0 + i < d) ? st.mu[(size_t)(j0 + i) * kpm + cc] : 0.0;
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            if (j0 + i < d) {
                                const double tq = (double)((float)xq[i] + L.ojf[j0 + i]) - mu[i];
                                s = s + tq * tq;
                            }
                        }
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
                if (lane == 0) lab_res[sl] = (unsigned char)(bc < k ? bc : 0);
            }
            __builtin_amdgcn_wave_barrier();
        }
        // Label changes -> sums of this workgroup (LDS).  The rows of the step whose label changed
        // are listed with their knob values (kStreamRec of them at most, then the list is applied
        // and starts again) and applied together, one lane per (row, group of 4 knobs): one chain
        // of dependent LDS accesses per step when few rows move, however many tiles hold one.
        auto apply_changes = [&](int count) {
            __builtin_amdgcn_wave_barrier();
            constexpr int LPR = DK / 4, EPI = 64 / LPR;
            const int j0 = 4 * (lane % LPR);
            for (int e0 = 0; e0 < count; e0 += EPI) {
                const int e = e0 + lane / LPR;
                if (e < count && j0 < d) {
                    const unsigned w = chg[e];
                    const int cc = w & 0xFF, pp = (w >> 8) & 0xFF;
                    const bool had = ((w >> 16) & 1u) == 0u;     // the row had a label before
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        if (j0 + i < d) {
                            const int xi = (int)((float)rec_x[(size_t)e * DK + j0 + i] + L.ojf[j0 + i]);
                            atomicAdd(&L.S[cc * DK + j0 + i], xi);
                            if (had) atomicSub(&L.S[pp * DK + j0 + i], xi);
                        }
                    }
                    if (j0 == 0) {
                        atomicAdd(&L.n[cc], 1);
                        if (had) atomicSub(&L.n[pp], 1);
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        };
        int nchg = 0;
#pragma unroll
        for (int tt = 0; tt < TILES; ++tt) {
            const int64_t row = wrow0 + tt * 32 + n32;
            int cl = lab[tt];
            if ((flagged_mask >> tt) & 1u) cl = lab_res[tt * 32 + n32];
            const int prev = cur.prev[tt];
            const bool changed = live[tt] && (first || cl != prev);
            if (want_dist && h == 0) lab_new[tt * 32 + n32] = (unsigned char)(live[tt] ? cl : 0);
            const uint64_t cm = __ballot(changed) & 0xFFFFFFFFull;
            if (cm) {
                const int c = __popcll(cm);
                if (nchg + c > kStreamRec) {                       // wave-uniform
                    apply_changes(nchg);
                    nchg = 0;
                }
                if (changed) {
                    const int rs = nchg + __popcll(cm & ((1ull << n32) - 1ull));
#pragma unroll
                    for (int f = 0; f < NS; ++f)
                        *reinterpret_cast<half8 *>(rec_x + (size_t)rs * DK + 16 * f + 8 * h) = cur.B[tt][f];
                    if (h == 0) {
                        chg[rs] = (unsigned)cl | ((unsigned)prev << 8) | (first ? 0x10000u : 0u);
                        labrow[row] = (uint8_t)cl;
                    }
                }
                nchg += c;
            }
        }
        if (nchg) apply_changes(nchg);
        if (want_dist) {
            // exact loss terms of the rows of this step: one row per lane, knobs ascending
            __builtin_amdgcn_wave_barrier();
            for (int s0 = 0; s0 < TILES * 32; s0 += 64) {
                const int sl = s0 + lane;
                const int64_t row = wrow0 + sl;
                if (row < r1) {
                    const int c = lab_new[sl];
                    // all loads of the row first (they are independent), then the sum in knob order
                    double mu[DK];
                    uint8_t xv[DK];
#pragma unroll
                    for (int j = 0; j < DK; ++j) {
                        const int jj = j < d ? j : 0;
                        xv[j] = a.X[(int64_t)jj * a.ld + row];
                        mu[j] = st.mu[(size_t)jj * kpm + c];
                    }
                    double s = 0.0;
#pragma unroll
                    for (int j = 0; j < DK; ++j) {
                        if (j < d) {
                            const double tq = (double)xv[j] - mu[j];
                            s = s + tq * tq;
                        }
                    }
                    part = part + s;
                }
            }
        }
    }

    if (want_dist) {
        const double ws = wave_sum(part);
        if (lane == 0) L.red[wave] = ws;
    }
    __syncthreads();
    // changes of this workgroup -> the unit's sums
    for (int e = tid; e < k * DK; e += blockDim.x) {
        const int v = L.S[e];
        if (v != 0) atomicAdd(&st.S[(e / DK) * 32 + (e % DK)], v);
    }
    for (int c = tid; c < k; c += blockDim.x) {
        const int v = L.n[c];
        if (v != 0) atomicAdd(&st.n[c], v);
    }
    if (want_dist && tid == 0) {
        double s = 0.0;
        for (int w = 0; w < kWavesPerWg; ++w) s = s + (w < (int)(blockDim.x >> 6) ? L.red[w] : 0.0);
        a.loss_part[blockIdx.x] = s;
    }
}

template <int DK>
__global__ __launch_bounds__(kWavesPerWg * 64, 2) void stream_assign_kernel(const StreamArgs a)
{
    __shared__ int unit_sh;
    const int tid = threadIdx.x;
    if (tid < 64) {
        // last unit with wg_off[unit] <= blockIdx.x: a 64-way search by the first wave (one or two
        // rounds of independent loads instead of a chain of dependent ones)
        int lo = 0, hi = a.n_units;
        while (hi - lo > 1) {
            const int span = hi - lo;
            const int stride = (span + 63) / 64;
            const int probe = lo + tid * stride;
            const bool le = probe < hi && a.wg_off[probe] <= (int)blockIdx.x;     // true for a prefix of the lanes
            const int cntle = __popcll(__ballot(le));                              // >= 1: wg_off[lo] <= blockIdx.x
            const int nlo = lo + (cntle - 1) * stride;
            const int nhi = nlo + stride < hi ? nlo + stride : hi;
            lo = nlo;
            hi = nhi;
        }
        if (tid == 0) unit_sh = lo;
    }
    __syncthreads();
    const int unit_idx = __builtin_amdgcn_readfirstlane(unit_sh);
    const int u = a.u_begin + unit_idx;
    const int k = a.ks[a.n_k - 1 - u / a.T];
    // the unit index goes through an opaque copy per variant: what a variant derives from it stays inside
    // its branch instead of being computed for all three ahead of the branch (scalar registers)
    int ui = unit_idx;
    if (k <= 64) {
        asm volatile("" : "+s"(ui));
        assign_unit<DK, 1, (DK == 16 ? 8 : 4)>(a, ui);
    } else if (k <= 128) {
        asm volatile("" : "+s"(ui));
        assign_unit<DK, 2, 4>(a, ui);
    } else {
        asm volatile("" : "+s"(ui));
        assign_unit<DK, 4, 4>(a, ui);
    }
}

template <int DK>
hipError_t run_stream(StreamArgs a, int64_t n_total, int total_wgs, hipStream_t s)
{
    const size_t lds = StreamLds<DK>::bytes(a.kpm);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(stream_assign_kernel<DK>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    if (a.prepare) {
        hipLaunchKernelGGL(stream_offsets_kernel, dim3(a.T), dim3(64), 0, s, a);
        const unsigned pb = (unsigned)((n_total + 255) / 256);
        if (pb) hipLaunchKernelGGL(stream_pack_kernel<DK>, dim3(pb), dim3(256), 0, s, a, n_total);
    }
    a.it = 0;
    a.final_pass = 0;
    const dim3 ugrid(a.n_units, a.kpm / 32), ublock(32 * (DK / 8));
    hipLaunchKernelGGL(stream_update_kernel<DK>, ugrid, ublock, 0, s, a, 0);
    for (int it = 0; it <= a.n_iter; ++it) {
        a.it = it;
        a.final_pass = it == a.n_iter ? 1 : 0;
        hipLaunchKernelGGL(stream_assign_kernel<DK>, dim3(total_wgs), dim3(kWavesPerWg * 64), lds, s, a);
        hipLaunchKernelGGL(stream_update_kernel<DK>, ugrid, ublock, 0, s, a, a.final_pass ? 2 : 1);
    }
    return hipGetLastError();
}

}  // namespace

int64_t stream_lds_bytes(int d, int kpm)
{
    return d <= 16 ? (int64_t)StreamLds<16>::bytes(kpm) : (int64_t)StreamLds<32>::bytes(kpm);
}

hipError_t launch_stream_sweep(const StreamArgs &a, int64_t n_total, int total_wgs, hipStream_t s)
{
    if (a.d <= 16) return run_stream<16>(a, n_total, total_wgs, s);
    return run_stream<32>(a, n_total, total_wgs, s);
}

}  // namespace cham
