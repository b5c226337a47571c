// One workgroup runs the whole Lloyd iteration of one (task, k) unit of the sweep
// (paper Algorithm 1: K-means.run(s_Theta, k) for one k; Sec. 3.3).
//
// Centroids, integer cluster sums and counts live in LDS for the whole unit; the task's rows
// are read from global memory (L2-resident after the first pass) four rows per lane and pass.
// Cluster sums are kept incrementally: a row touches the sums only when its label changes,
// which is exact because the sums are integers.
#include <type_traits>

#include "cham_device.h"
#include "cham_internal.h"

namespace cham {

namespace {

// SumT: type of the integer cluster sums.  32 bits hold the sums of byte knobs (at most 2^23 rows of
// values below 256); two-byte knobs need 64.
template <int DP, typename SumT>
struct UnitLds {
    double *mu64T;
    float *wf;
    SumT *S;
    int *n;
    float *ojf;
    double *red;
    unsigned *m2bits;
    __device__ UnitLds(unsigned char *base, int kmax)
    {
        mu64T = reinterpret_cast<double *>(base);
        base += sizeof(double) * (size_t)DP * kmax;
        red = reinterpret_cast<double *>(base);
        base += sizeof(double) * 16;
        if (sizeof(SumT) == 8) {            // 8-byte items first
            S = reinterpret_cast<SumT *>(base);
            base += sizeof(SumT) * (size_t)kmax * DP;
        }
        wf = reinterpret_cast<float *>(base);
        base += sizeof(float) * (size_t)kmax * (DP + 4);
        if (sizeof(SumT) == 4) {
            S = reinterpret_cast<SumT *>(base);
            base += sizeof(SumT) * (size_t)kmax * DP;
        }
        n = reinterpret_cast<int *>(base);
        base += sizeof(int) * (size_t)kmax;
        ojf = reinterpret_cast<float *>(base);
        base += sizeof(float) * (size_t)DP;
        m2bits = reinterpret_cast<unsigned *>(base);
    }
};

// From the exact centroids build the fp32 screening form: w = -2*(mu - o), b = |mu - o|^2,
// and the bound m2 >= max_c b.  Caller synchronises before and after.
__device__ __forceinline__ void lds_add(int *p, int v) { atomicAdd(p, v); }
__device__ __forceinline__ void lds_add(long long *p, int v)
{
    atomicAdd(reinterpret_cast<unsigned long long *>(p), (unsigned long long)(long long)v);
}

template <int DP, typename SumT>
__device__ __forceinline__ void derive_screen(const UnitLds<DP, SumT> &U, int k, int kp)
{
    // eight lanes per centroid, each taking every eighth knob
    constexpr int kGroup = 8;
    const int sub = threadIdx.x % kGroup;
    for (int c = threadIdx.x / kGroup; c < k; c += blockDim.x / kGroup) {
        double b = 0.0;
        float *w = U.wf + (size_t)c * (DP + 4);
        for (int j = sub; j < DP; j += kGroup) {
            const double m = U.mu64T[(size_t)j * kp + c] - (double)U.ojf[j];
            b = __builtin_fma(m, m, b);
            w[j] = (float)(-2.0 * m);
        }
#pragma unroll
        for (int off = kGroup / 2; off >= 1; off >>= 1) b = b + __shfl_xor(b, off, kWave);
        if (sub == 0) {
            w[DP] = (float)b;
            w[DP + 1] = 0.0f;
            w[DP + 2] = 0.0f;
            w[DP + 3] = 0.0f;
            const float bu = __double2float_ru(b) * 1.0000005f;
            atomicMax(U.m2bits, __float_as_uint(bu));
        }
    }
}

// XT: storage type of a knob value (uint8_t or uint16_t); R: rows per lane and pass (one load of
// R * sizeof(XT) bytes holds knob j of R consecutive rows).
template <typename XT, int DP, int R, int MAXNT>
__global__ __launch_bounds__(MAXNT) void resident_sweep_kernel(const SweepArgs a)
{
    using SumT = typename std::conditional<sizeof(XT) == 1, int, long long>::type;
    constexpr double kMaxValue = sizeof(XT) == 1 ? 255.0 : 65535.0;
    extern __shared__ __align__(16) unsigned char smem[];
    // per wave: the rows of one step that changed their label (row within the task; new | previous << 8),
    // behind the unit's state when the LDS has room for them
    const bool use_queue = a.queue_lds_off != 0;
    int *q_row = reinterpret_cast<int *>(smem + a.queue_lds_off) + (threadIdx.x / kWave) * 2 * kWave;
    int *q_lab = q_row + kWave;
    constexpr int LPR = DP <= 8 ? 8 : (DP <= 16 ? 16 : (DP <= 32 ? 32 : 64));     // lanes per queued row
    UnitLds<DP, SumT> U(smem, a.kmax);
    const XT *X = reinterpret_cast<const XT *>(a.X);

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int nwaves = blockDim.x / kWave;

    // units in descending-k order so that the longest ones start first
    const int u = blockIdx.x;
    const int ki = a.ki_end - 1 - u / a.T;
    const int t = u % a.T;
    const int k = a.ks[ki];
    const int kp = k;
    const bool skipped = a.done && a.done[t];     // the task's sweep stopped at a smaller k
    const int d = a.d;
    const int64_t r0 = a.task_off[t], r1 = a.task_off[t + 1];
    const int64_t slot = (int64_t)t * a.n_k + ki;
    const int64_t crow = (int64_t)t * a.Ksum + a.koff[ki];
    uint8_t *labrow = a.labbuf + (int64_t)ki * a.ld;
    const int64_t g0 = r0 & ~(int64_t)(R - 1);
    const int tile_rows = blockDim.x * R;
    const bool force_exact = (a.flags & 1) != 0;

    if (skipped || (a.init_mode == 0 && a.ndist[t] < k)) {
        // fewer than k distinct rows, or not needed any more: all outputs zero, status says which
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

    // ---- set-up: zero state, stage the starting centroids, choose centring offsets
    for (int e = tid; e < DP * kp; e += blockDim.x) U.mu64T[e] = 0.0;
    for (int e = tid; e < k * DP; e += blockDim.x) U.S[e] = 0;
    for (int c = tid; c < k; c += blockDim.x) U.n[c] = 0;
    if (tid == 0) *U.m2bits = 0u;
    __syncthreads();
    for (int e = tid; e < k * d; e += blockDim.x) {
        const int c = e / d, j = e % d;
        double v;
        if (a.init_mode == 0) {
            const int row = a.init_rows[(int64_t)t * a.kmax + c];
            v = (double)X[(int64_t)j * a.ld + r0 + row];
        } else {
            v = a.init_centroids[(crow + c) * d + j];
        }
        U.mu64T[(size_t)j * kp + c] = v;
    }
    __syncthreads();
    if (tid < DP) {
        float o = 0.0f;
        if (tid < d) {
            double s = 0.0;
            for (int c = 0; c < k; ++c) s += U.mu64T[(size_t)tid * kp + c];
            double m = rint(s / (double)k);
            m = m < 0.0 ? 0.0 : (m > kMaxValue ? kMaxValue : m);
            o = (float)m;
        }
        U.ojf[tid] = o;
    }
    __syncthreads();
    derive_screen<DP>(U, k, kp);
    __syncthreads();

    const int64_t span = r1 - g0;
    const int ntiles = (int)((span + tile_rows - 1) / tile_rows);
    double loss = 0.0;
    int passes_run = 0;

    for (int it = 0; it <= a.n_iter; ++it) {
        const bool final_pass = (it == a.n_iter);
        const bool want_dist = final_pass || (a.trace != nullptr);
        bool moved = false;              // this thread changed a label in this pass
        ++passes_run;
        CentroidView L;
        L.mu64T = U.mu64T;
        L.wf = U.wf;
        L.ojf = U.ojf;
        L.m2 = __uint_as_float(*U.m2bits);
        L.kp = kp;
        L.k = k;
        double part = 0.0;

        for (int tile = 0; tile < ntiles; ++tile) {
            const int64_t g = g0 + (int64_t)tile * tile_rows + (int64_t)tid * R;
            const bool in_range = g < r1;
            uint32_t rowmask = 0;
#pragma unroll
            for (int p = 0; p < R; ++p)
                if (g + p >= r0 && g + p < r1) rowmask |= 1u << p;

            float xf[R][DP];
            float x2[R];
            load_rows<XT, DP, R>(X, a.ld, d, g, in_range, U.ojf, xf, x2);

            int lab[R];
            double dist[R];
#pragma unroll
            for (int p = 0; p < R; ++p) dist[p] = 0.0;
            assign_rows<DP, R>(xf, x2, rowmask, L, force_exact, want_dist, lab, dist);

            uint32_t prevpack = 0;
            if (it > 0 && in_range) {
                if (R == 4) prevpack = *reinterpret_cast<const uint32_t *>(labrow + g);
                else prevpack = *reinterpret_cast<const uint16_t *>(labrow + g);
            }
            uint32_t newpack = 0;
            bool changed = false;
#pragma unroll
            for (int p = 0; p < R; ++p) {
                const int prev = (prevpack >> (8 * p)) & 0xFF;
                const bool on = (rowmask >> p) & 1u;
                const int cur = on ? lab[p] : prev;
                newpack |= (uint32_t)cur << (8 * p);
                const bool ch = on && (it == 0 || cur != prev);
                changed = changed || ch;
                if (it == 0 || !use_queue) {
                    // every row is new (or there is no room for the queue): each lane adds its own
                    // row from its registers
                    if (ch) {
                        // fully unrolled: a run-time index into xf would move the rows out of registers
#pragma unroll
                        for (int j = 0; j < DP; ++j) {
                            if (j < d) {
                                const int xi = (int)(xf[p][j] + U.ojf[j]);
                                lds_add(&U.S[cur * DP + j], xi);
                                if (it > 0) lds_add(&U.S[prev * DP + j], -xi);
                            }
                        }
                        atomicAdd(&U.n[cur], 1);
                        if (it > 0) atomicSub(&U.n[prev], 1);
                    }
                } else {
                    // Later passes move few rows: they are queued (row, new and previous label) and
                    // the wave applies the queue with one lane per (row, knob), the knob value read
                    // again from the matrix, so that the cost follows the number of moved rows
                    // instead of every wave walking all knobs whenever one of its lanes moved.
                    const uint64_t cm = __ballot(ch);
                    if (cm) {
                        if (ch) {
                            const int pos = __popcll(cm & ((1ull << lane) - 1ull));
                            q_row[pos] = (int)(g + p - r0);
                            q_lab[pos] = cur | (prev << 8);
                        }
                        __builtin_amdgcn_wave_barrier();
                        const int qn = __popcll(cm);
                        const int sub = lane / LPR, j = lane % LPR;
                        for (int e0 = 0; e0 < qn; e0 += 64 / LPR) {
                            const int e = e0 + sub;
                            if (e < qn && j < d) {
                                const int w = q_lab[e];
                                const int xi = (int)X[(int64_t)j * a.ld + r0 + q_row[e]];
                                lds_add(&U.S[(w & 0xFF) * DP + j], xi);
                                lds_add(&U.S[(w >> 8) * DP + j], -xi);
                                if (j == 0) {
                                    atomicAdd(&U.n[w & 0xFF], 1);
                                    atomicSub(&U.n[w >> 8], 1);
                                }
                            }
                        }
                        __builtin_amdgcn_wave_barrier();
                    }
                }
                if (on && want_dist) part = part + dist[p];
            }
            moved = moved || changed;
            if (changed) {
                if (rowmask == (1u << R) - 1u) {
                    if (R == 4) *reinterpret_cast<uint32_t *>(labrow + g) = newpack;
                    else *reinterpret_cast<uint16_t *>(labrow + g) = (uint16_t)newpack;
                } else {
#pragma unroll
                    for (int p = 0; p < R; ++p)
                        if ((rowmask >> p) & 1u) labrow[g + p] = (uint8_t)lab[p];
                }
            }
        }

        if (want_dist) {
            // fixed-order reduction: lanes (butterfly), then waves in order
            const double ws = wave_sum(part);
            if (lane == 0) U.red[wave] = ws;
        }
        const bool any_moved = __syncthreads_or(moved ? 1 : 0) != 0;
        if (want_dist && tid == 0) {
            double s = 0.0;
            for (int w = 0; w < nwaves; ++w) s = s + U.red[w];
            loss = s;
            if (a.trace) a.trace[slot * (a.n_iter + 1) + it] = s;
        }

        // A pass that moved no row leaves the sums, hence the centroids, hence every later pass as
        // they are: the remaining passes would repeat this one.  With the loss at hand (a traced
        // run) the iteration ends here; otherwise the final pass, which computes it, runs next.
        if (!final_pass && !any_moved) {
            if (want_dist) {
                if (tid == 0)
                    for (int r = it + 1; r <= a.n_iter; ++r) a.trace[slot * (a.n_iter + 1) + r] = loss;
                break;
            }
            it = a.n_iter - 1;
            continue;
        }

        if (!final_pass) {
            // centroid update: mean of the members, an empty cluster keeps its centroid
            if (tid == 0) *U.m2bits = 0u;
            for (int e = tid; e < k * d; e += blockDim.x) {
                const int c = e / d, j = e % d;
                const int cnt = U.n[c];
                if (cnt > 0) U.mu64T[(size_t)j * kp + c] = (double)U.S[c * DP + j] / (double)cnt;
            }
            __syncthreads();
            derive_screen<DP>(U, k, kp);
            __syncthreads();
        }
    }

    for (int e = tid; e < k * d; e += blockDim.x) {
        const int c = e / d, j = e % d;
        a.centroids[(crow + c) * d + j] = U.mu64T[(size_t)j * kp + c];
    }
    for (int c = tid; c < k; c += blockDim.x) a.counts[crow + c] = U.n[c];
    if (tid == 0) {
        a.status[slot] = 0;
        a.inertia[slot] = loss;
        a.passes[slot] = passes_run;
    }
}

// First kmax distinct rows of each task, in row order: one wave per task walks the rows 64 at a
// time; a row is taken unless it equals a row taken before it.
template <typename XT>
__global__ __launch_bounds__(64) void first_distinct_kernel(const SweepArgs a, int *init_rows, int *ndist)
{
    const XT *X = reinterpret_cast<const XT *>(a.X);
    __shared__ uint64_t taken_hash[256];
    __shared__ int taken_row[256];
    const int t = blockIdx.x;
    const int lane = threadIdx.x;
    const int d = a.d;
    const int64_t r0 = a.task_off[t], r1 = a.task_off[t + 1];
    const int kmax = a.kmax;
    int found = 0;
    for (int64_t base = r0; base < r1 && found < kmax; base += kWave) {
        const int64_t r = base + lane;
        const bool live = r < r1;
        uint64_t h = fnv_begin(0);
        if (live)
            for (int j = 0; j < d; ++j) h = fnv_step(h, X[(int64_t)j * a.ld + r]);
        bool fresh = live;
        // against rows already taken
        for (int q = 0; q < found && fresh; ++q) {
            if (taken_hash[q] != h) continue;
            bool same = true;
            const int64_t rq = r0 + taken_row[q];
            for (int j = 0; j < d && same; ++j)
                same = X[(int64_t)j * a.ld + rq] == X[(int64_t)j * a.ld + r];
            if (same) fresh = false;
        }
        // against earlier rows of this batch of 64
        for (int q = 0; q < kWave; ++q) {
            const uint64_t hq = __shfl(h, q, kWave);
            if (q < lane && fresh && hq == h && base + q < r1) {
                bool same = true;
                for (int j = 0; j < d && same; ++j)
                    same = X[(int64_t)j * a.ld + base + q] == X[(int64_t)j * a.ld + r];
                if (same) fresh = false;
            }
        }
        const uint64_t m = __ballot(fresh);
        const int pos = found + __popcll(m & ((1ull << lane) - 1ull));
        if (fresh && pos < kmax) {
            taken_hash[pos] = h;
            taken_row[pos] = (int)(r - r0);
            init_rows[(int64_t)t * kmax + pos] = (int)(r - r0);
        }
        found += __popcll(m);
        if (found > kmax) found = kmax;
        __syncthreads();
    }
    if (lane == 0) ndist[t] = found;
}

template <typename XT, int DP, int R, int MAXNT>
hipError_t launch_dp(const SweepArgs &a, int nt, hipStream_t s)
{
    size_t lds = (resident_lds_bytes(DP, a.kmax, sizeof(XT) == 1 ? 4 : 8) + 15) & ~(size_t)15;
    SweepArgs b = a;
    if (nt > MAXNT) nt = MAXNT;
    const size_t queue = (size_t)((nt + kWave - 1) / kWave) * 2 * kWave * sizeof(int);    // per-wave queues of moved rows
    b.queue_lds_off = 0;
    if (lds + queue <= 160 * 1024) {
        b.queue_lds_off = (int)lds;
        lds += queue;
    }
    auto kern = resident_sweep_kernel<XT, DP, R, MAXNT>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    const unsigned units = (unsigned)a.T * (unsigned)(a.ki_end - a.ki_begin);
    hipLaunchKernelGGL(kern, dim3(units), dim3(nt), lds, s, b);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_first_distinct(const SweepArgs &a, int *init_rows, int *ndist, hipStream_t s)
{
    if (a.xbytes == 2)
        hipLaunchKernelGGL(first_distinct_kernel<uint16_t>, dim3(a.T), dim3(64), 0, s, a, init_rows, ndist);
    else
        hipLaunchKernelGGL(first_distinct_kernel<uint8_t>, dim3(a.T), dim3(64), 0, s, a, init_rows, ndist);
    return hipGetLastError();
}

// Padded knob count of the two-byte instantiations.
int resident_dp16(int d) { return (d + 7) / 8 * 8; }

hipError_t launch_resident_sweep(const SweepArgs &a, int nt, hipStream_t s)
{
    const int d = a.d;
    if (a.xbytes == 2) {
        if (d <= 8) return launch_dp<uint16_t, 8, 4, 512>(a, nt, s);
        if (d <= 16) return launch_dp<uint16_t, 16, 4, 512>(a, nt, s);
        if (d <= 24) return launch_dp<uint16_t, 24, 4, 512>(a, nt, s);
        if (d <= 32) return launch_dp<uint16_t, 32, 4, 512>(a, nt, s);
        if (d <= 40) return launch_dp<uint16_t, 40, 2, 512>(a, nt, s);
        if (d <= 48) return launch_dp<uint16_t, 48, 2, 512>(a, nt, s);
        if (d <= 56) return launch_dp<uint16_t, 56, 2, 512>(a, nt, s);
        return launch_dp<uint16_t, 64, 2, 512>(a, nt, s);
    }
    if (d <= 4) return launch_dp<uint8_t, 4, 4, 1024>(a, nt, s);
    if (d <= 8) return launch_dp<uint8_t, 8, 4, 1024>(a, nt, s);
    if (d <= 12) return launch_dp<uint8_t, 12, 4, 1024>(a, nt, s);
    if (d <= 16) return launch_dp<uint8_t, 16, 4, 512>(a, nt, s);
    if (d <= 20) return launch_dp<uint8_t, 20, 4, 512>(a, nt, s);
    if (d <= 24) return launch_dp<uint8_t, 24, 4, 512>(a, nt, s);
    if (d <= 28) return launch_dp<uint8_t, 28, 4, 512>(a, nt, s);
    return launch_dp<uint8_t, 32, 4, 512>(a, nt, s);
}

}  // namespace cham
