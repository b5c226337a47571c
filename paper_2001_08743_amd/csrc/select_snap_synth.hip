// Knee selection, centroid snap, Sample Synthesis and dedupe kernels
// (paper Algorithm 1: threshold exit of the sweep, and the replacement loop; Sec. 3.3).
#include "cham_device.h"
#include "cham_internal.h"

namespace cham {

namespace {

// ---------------------------------------------------------------------------------------------
// Knee: one thread per task walks its loss curve (Algorithm 1: previous_loss starts at
// infinity; the first k with threshold * loss >= previous_loss is returned, else the last k).
__global__ void select_k_kernel(const double *inertia, const int *status, int T, int n_k,
                                double threshold, int *chosen)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const double *L = inertia + (int64_t)t * n_k;
    const int *st = status + (int64_t)t * n_k;
    bool have_prev = false;
    double prev = 0.0;
    int last = -1, pick = -1;
    for (int i = 0; i < n_k; ++i) {
        if (st[i] != 0) continue;
        if (have_prev && threshold * L[i] >= prev) {
            pick = i;
            break;
        }
        prev = L[i];
        have_prev = true;
        last = i;
    }
    chosen[t] = pick >= 0 ? pick : last;
}

// Between two chunks of a sweep that stops at the knee (Algorithm 1 breaks out of its loop over k at
// the first k with threshold * loss >= previous_loss): tasks whose curve has reached that k are
// marked done; the remaining chunks skip them.
__global__ void knee_update_kernel(const double *inertia, const int *status, int T, int n_k, int ki_end,
                                   double threshold, int *done)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T || done[t]) return;
    const double *L = inertia + (int64_t)t * n_k;
    const int *st = status + (int64_t)t * n_k;
    bool have_prev = false;
    double prev = 0.0;
    for (int i = 0; i < ki_end; ++i) {
        if (st[i] != 0) continue;
        if (have_prev && threshold * L[i] >= prev) {
            done[t] = 1;
            return;
        }
        prev = L[i];
        have_prev = true;
    }
}

__global__ void fill_i32_kernel(int *dst, int64_t n, int value)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = value;
}

// ---------------------------------------------------------------------------------------------
// Snap: one workgroup per task.  Labels under the chosen centroids (same two-stage exact
// assignment as the sweep), then per cluster the member with the smallest exact distance,
// lowest row on ties: a 64-bit minimum on the distance bits followed by a minimum on the row
// among the members that attain it.
template <int DP>
struct SnapLds {
    double *mu64T;
    double *red;
    float *wf;
    unsigned long long *best;   // [k] distance bits
    int *brow;                  // [k]
    float *ojf;
    unsigned *m2bits;
    __device__ SnapLds(unsigned char *base, int kmax)
    {
        mu64T = reinterpret_cast<double *>(base);
        base += sizeof(double) * (size_t)DP * kmax;
        red = reinterpret_cast<double *>(base);
        base += sizeof(double) * 16;
        wf = reinterpret_cast<float *>(base);
        base += sizeof(float) * (size_t)kmax * (DP + 4);
        best = reinterpret_cast<unsigned long long *>(base);
        brow = reinterpret_cast<int *>(base + sizeof(unsigned long long) * (size_t)kmax);
        base += sizeof(int) * (size_t)kmax * DP;     // same footprint as the sweep's sums (DP >= 4)
        base += sizeof(int) * (size_t)kmax;
        ojf = reinterpret_cast<float *>(base);
        base += sizeof(float) * (size_t)DP;
        m2bits = reinterpret_cast<unsigned *>(base);
    }
};

// XT: storage type of a knob value; R: rows per lane and pass (as in the sweep kernel).
template <typename XT, int DP, int R, int MAXNT>
__global__ __launch_bounds__(MAXNT) void snap_kernel(const SnapArgs a)
{
    constexpr double kMaxValue = sizeof(XT) == 1 ? 255.0 : 65535.0;
    const XT *X = reinterpret_cast<const XT *>(a.X);
    XT *pick_cfg = reinterpret_cast<XT *>(a.pick_cfg);
    extern __shared__ __align__(16) unsigned char smem[];
    SnapLds<DP> U(smem, a.kmax);
    const int tid = threadIdx.x;
    const int t = blockIdx.x;
    const int d = a.d;
    const int64_t r0 = a.task_off[t], r1 = a.task_off[t + 1];
    const int ci = a.chosen[t];
    const int tile_rows = blockDim.x * R;

    for (int c = tid; c < a.kmax; c += blockDim.x) a.pick_row[(int64_t)t * a.kmax + c] = -1;
    for (int e = tid; e < a.kmax * d; e += blockDim.x) pick_cfg[(int64_t)t * a.kmax * d + e] = 0;
    if (ci < 0 || ci >= a.n_k) return;
    const int k = a.ks[ci];
    const int kp = k;
    const int64_t crow = (int64_t)t * a.Ksum + a.koff[ci];

    for (int e = tid; e < DP * kp; e += blockDim.x) U.mu64T[e] = 0.0;
    for (int c = tid; c < k; c += blockDim.x) {
        U.best[c] = ~0ull;
        U.brow[c] = 0x7fffffff;
    }
    if (tid == 0) *U.m2bits = 0u;
    __syncthreads();
    for (int e = tid; e < k * d; e += blockDim.x) {
        const int c = e / d, j = e % d;
        U.mu64T[(size_t)j * kp + c] = a.centroids[(crow + c) * d + j];
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
    for (int c = tid; c < k; c += blockDim.x) {
        double b = 0.0;
        float *w = U.wf + (size_t)c * (DP + 4);
#pragma unroll
        for (int j = 0; j < DP; ++j) {
            const double m = U.mu64T[(size_t)j * kp + c] - (double)U.ojf[j];
            b = __builtin_fma(m, m, b);
            w[j] = (float)(-2.0 * m);
        }
        w[DP] = (float)b;
        w[DP + 1] = w[DP + 2] = w[DP + 3] = 0.0f;
        atomicMax(U.m2bits, __float_as_uint(__double2float_ru(b) * 1.0000005f));
    }
    __syncthreads();

    CentroidView L;
    L.mu64T = U.mu64T;
    L.wf = U.wf;
    L.ojf = U.ojf;
    L.m2 = __uint_as_float(*U.m2bits);
    L.kp = kp;
    L.k = k;
    const bool force_exact = (a.flags & 1) != 0;
    const int64_t g0 = r0 & ~(int64_t)(R - 1);
    const int ntiles = (int)((r1 - g0 + tile_rows - 1) / tile_rows);

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
        assign_rows<DP, R>(xf, x2, rowmask, L, force_exact, true, lab, dist);
#pragma unroll
        for (int p = 0; p < R; ++p) {
            if (!((rowmask >> p) & 1u)) continue;
            a.labels_sel[g + p] = (uint8_t)lab[p];
            a.dist_ws[g + p] = dist[p];
            atomicMin(&U.best[lab[p]], (unsigned long long)__double_as_longlong(dist[p]));
        }
    }
    __syncthreads();
    for (int64_t r = r0 + tid; r < r1; r += blockDim.x) {
        const int c = a.labels_sel[r];
        if ((unsigned long long)__double_as_longlong(a.dist_ws[r]) == U.best[c])
            atomicMin(&U.brow[c], (int)(r - r0));
    }
    __syncthreads();
    for (int c = tid; c < k; c += blockDim.x) {
        const int row = U.brow[c];
        if (row != 0x7fffffff) a.pick_row[(int64_t)t * a.kmax + c] = row;
    }
    for (int e = tid; e < k * d; e += blockDim.x) {
        const int c = e / d, j = e % d;
        const int row = U.brow[c];
        if (row != 0x7fffffff)
            pick_cfg[((int64_t)t * a.kmax + c) * d + j] = X[(int64_t)j * a.ld + r0 + row];
    }
}

// ---------------------------------------------------------------------------------------------
// Membership in the visited set.  n >= 0: v is a sorted array of n hashes (binary search).
// n < 0: v is an open-addressing table of -n slots (a power of two, linear probing, empty slots
// hold all ones; the one hash that equals the empty mark is stored as the value below it).
constexpr uint64_t kEmptySlot = ~0ull;
__device__ __forceinline__ uint64_t table_key(uint64_t h) { return h == kEmptySlot ? h - 1 : h; }

__device__ __forceinline__ bool visited_has(const uint64_t *v, int64_t n, uint64_t key)
{
    if (n < 0) {
        const uint64_t mask = (uint64_t)(-n) - 1;
        const uint64_t k = table_key(key);
        uint64_t pos = k & mask;
        for (uint64_t probes = 0; probes <= mask; ++probes) {       // a full table ends the walk
            const uint64_t cur = v[pos];
            if (cur == k) return true;
            if (cur == kEmptySlot) return false;
            pos = (pos + 1) & mask;
        }
        return false;
    }
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = lo + ((hi - lo) >> 1);
        if (v[mid] < key) lo = mid + 1; else hi = mid;
    }
    return lo < n && v[lo] == key;
}

// Insert one hash: 1 = newly inserted, 2 = was there already, 0 = the table is full.
__device__ __forceinline__ int table_insert_new(uint64_t *v, uint64_t mask, uint64_t h)
{
    const uint64_t k = table_key(h);
    uint64_t pos = k & mask;
    for (uint64_t probes = 0; probes <= mask; ++probes) {
        const unsigned long long seen = atomicCAS(reinterpret_cast<unsigned long long *>(v + pos),
                                                  (unsigned long long)kEmptySlot, (unsigned long long)k);
        if (seen == kEmptySlot) return 1;
        if (seen == k) return 2;
        pos = (pos + 1) & mask;
    }
    return 0;
}
__device__ __forceinline__ bool table_insert(uint64_t *v, uint64_t mask, uint64_t h)
{
    return table_insert_new(v, mask, h) != 0;
}

// Configuration updater of the exploration step (Sec. 3.2: the agent emits increment / decrement /
// stay per knob and the updater applies it): theta <- clip(theta + a, 0, card - 1) per knob, n_steps
// times.  One workgroup carries one configuration, a chunk of steps at a time, in three phases: all
// threads stage the chunk's actions in LDS; one lane per knob walks the chunk (the knobs of a
// configuration move independently of each other, the steps of a knob do not) and leaves every
// configuration reached in LDS; then one thread per step hashes its configuration and enters it
// into the table of configurations seen, all steps of the chunk at once, so the latency of the
// table's compare-and-swap is paid once per chunk instead of once per step.  The thread that
// enters a configuration first also appends it to the list of distinct configurations (the set
// S_Theta that the sampling step receives; order unspecified); a wave reserves its list slots with
// one atomic add.
constexpr int kUpdChunk = 512;
constexpr int kUpdThreads = 256;

__global__ void __launch_bounds__(kUpdThreads)
update_configs_kernel(uint8_t *theta, const int8_t *actions, int64_t B, int d, int n_steps,
                      const uint16_t *cards, uint64_t salt, uint64_t *seen, int64_t slots,
                      uint8_t *unique_rows, int64_t cap, int *n_unique, int *overflow)
{
    __shared__ int8_t act[kUpdChunk * 32];
    __shared__ uint8_t cfg[kUpdChunk * 32];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    for (int64_t b = blockIdx.x; b < B; b += gridDim.x) {
        int cur = 0, hi = 0;
        if (tid < d) {
            cur = theta[b * d + tid];
            hi = (int)cards[tid] - 1;
        }
        for (int t0 = 0; t0 < n_steps; t0 += kUpdChunk) {
            const int nt = min(kUpdChunk, n_steps - t0);
            for (int e = tid; e < nt * d; e += kUpdThreads) {
                const int t = e / d;
                act[e] = actions[((int64_t)(t0 + t) * B + b) * d + (e - t * d)];
            }
            __syncthreads();
            if (tid < d) {
#pragma unroll 8
                for (int t = 0; t < nt; ++t) {
                    int v = cur + (int)act[t * d + tid];
                    v = v < 0 ? 0 : (v > hi ? hi : v);
                    cur = v;
                    cfg[t * d + tid] = (uint8_t)v;
                }
            }
            __syncthreads();
            if (seen) {
                for (int base = 0; base < nt; base += kUpdThreads) {
                    const int t = base + tid;
                    bool is_new = false;
                    if (t < nt) {
                        uint64_t h = fnv_begin(salt);
                        for (int j = 0; j < d; ++j) h = fnv_step(h, cfg[t * d + j]);
                        const int r = table_insert_new(seen, (uint64_t)slots - 1, h);
                        if (r == 0 && overflow) *overflow = 1;
                        is_new = r == 1;
                    }
                    const uint64_t m = __ballot(is_new);
                    if (m != 0) {                                  // wave-uniform
                        const int leader = __ffsll((unsigned long long)m) - 1;
                        int first = 0;
                        if (lane == leader) first = atomicAdd(n_unique, __popcll(m));
                        first = __shfl(first, leader);
                        if (is_new) {
                            const int64_t idx = (int64_t)first + __popcll(m & ((1ull << lane) - 1ull));
                            if (idx < cap) {
                                for (int j = 0; j < d; ++j) unique_rows[idx * d + j] = cfg[t * d + j];
                            } else if (overflow) {
                                *overflow = 1;
                            }
                        }
                    }
                }
            }
            __syncthreads();                                       // the next chunk overwrites act and cfg
        }
        if (tid < d) theta[b * d + tid] = (uint8_t)cur;
    }
}

__global__ void table_clear_kernel(uint64_t *v, int64_t slots)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < slots) v[i] = kEmptySlot;
}

__global__ void table_insert_hashes_kernel(uint64_t *v, int64_t slots, const uint64_t *hashes, int64_t n,
                                           int *overflow)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if (!table_insert(v, (uint64_t)slots - 1, hashes[i]) && overflow) *overflow = 1;
}

// Hash and insert configurations: row i of cfgs [n][d] is inserted iff flags is null or flags[i] is
// KEPT (1) or SYNTH (2); its salt is salts[i / rows_per_salt] (salts null: i / rows_per_salt itself).
template <typename XT>
__global__ void table_insert_configs_kernel(uint64_t *v, int64_t slots, const XT *cfgs, int64_t n, int d,
                                            const uint8_t *flags, const uint64_t *salts, int64_t rows_per_salt,
                                            int *overflow)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if (flags && flags[i] != 1 && flags[i] != 2) return;
    const uint64_t g = (uint64_t)(i / rows_per_salt);
    uint64_t h = fnv_begin(salts ? salts[g] : g);
    for (int j = 0; j < d; ++j) h = fnv_step(h, cfgs[i * d + j]);
    if (!table_insert(v, (uint64_t)slots - 1, h) && overflow) *overflow = 1;
}

// Synthesis: one workgroup per task.
//  A. flag picks (invalid row, or hash in the visited set); unflagged picks are KEPT.
//  B. histograms value counts per (flagged cluster, knob) over the cluster's valid members, a
//     chunk of clusters at a time (as many as fit the LDS histogram), and takes the mode.
//  C. one wave walks the flagged clusters in ascending order and accepts or drops each mode.
template <typename XT>
__global__ __launch_bounds__(1024) void synth_kernel(const SynthArgs a)
{
    const XT *X = reinterpret_cast<const XT *>(a.X);
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int t = blockIdx.x;
    const int d = a.d;
    const int kmax = a.kmax;
    const int64_t r0 = a.task_off[t], r1 = a.task_off[t + 1];
    const int ci = a.chosen[t];
    XT *ocfg = reinterpret_cast<XT *>(a.out_cfg) + (int64_t)t * kmax * d;
    uint8_t *oflag = a.out_flag + (int64_t)t * kmax;

    // LDS carve
    unsigned *hist = reinterpret_cast<unsigned *>(smem);                       // [hist_words]
    unsigned char *p8 = smem + sizeof(unsigned) * (size_t)a.hist_words;
    int *slot_of = reinterpret_cast<int *>(p8);           p8 += sizeof(int) * (size_t)kmax;      // [kmax]
    int *flagged = reinterpret_cast<int *>(p8);           p8 += sizeof(int) * (size_t)kmax;      // compact list
    int *misc = reinterpret_cast<int *>(p8);              p8 += sizeof(int) * 8;
    XT *cfg = reinterpret_cast<XT *>(p8);                 p8 += sizeof(XT) * (size_t)kmax * d;   // [kmax][d] kept / accepted
    XT *mode = reinterpret_cast<XT *>(p8);                p8 += sizeof(XT) * (size_t)kmax * d;   // [kmax][d] candidate modes
    uint8_t *fl = p8;                                     p8 += (size_t)kmax;                    // [kmax] flags
    uint8_t *hasv = p8;                                                                           // [kmax] cluster has a valid member

    for (int c = tid; c < kmax; c += blockDim.x) {
        fl[c] = 0;          // CHAM_OUT_EMPTY
        hasv[c] = 0;
        slot_of[c] = -1;
    }
    for (int e = tid; e < kmax * d; e += blockDim.x) cfg[e] = 0;
    __syncthreads();
    const int k = (ci >= 0 && ci < a.n_k) ? a.ks[ci] : 0;
    const uint64_t salt = a.salts[t];
    const uint16_t *card = a.cards + (int64_t)t * d;

    // A. flag picks
    for (int c = tid; c < k; c += blockDim.x) {
        const int row = a.pick_row[(int64_t)t * kmax + c];
        if (row < 0) continue;
        const XT *pc = reinterpret_cast<const XT *>(a.pick_cfg) + ((int64_t)t * kmax + c) * d;
        uint64_t h = fnv_begin(salt);
        for (int j = 0; j < d; ++j) h = fnv_step(h, pc[j]);
        const bool invalid = a.valid && a.valid[r0 + row] == 0;
        const bool bad = invalid || visited_has(a.visited, a.n_visited, h);
        if (bad) {
            fl[c] = 3;      // CHAM_OUT_DROPPED until a replacement is accepted
        } else {
            fl[c] = 1;      // CHAM_OUT_KEPT
            for (int j = 0; j < d; ++j) cfg[c * d + j] = pc[j];
        }
    }
    __syncthreads();
    if (tid == 0) {
        int nf = 0;
        for (int c = 0; c < k; ++c)
            if (fl[c] == 3) flagged[nf++] = c;
        misc[0] = nf;
    }
    __syncthreads();
    const int nf = misc[0];

    // B. modes, a window of knobs and a chunk of flagged clusters at a time (all knobs at once when
    // the histogram of a whole cluster fits)
    int cmax = 1;
    for (int j = 0; j < d; ++j) cmax = card[j] > cmax ? card[j] : cmax;
    int jn = a.hist_words / cmax;                       // >= 1 by construction on the host
    jn = jn > d ? d : jn;
    const int per_cluster = jn * cmax;
    const int chunk = a.hist_words / per_cluster;
    for (int j0 = 0; j0 < d; j0 += jn) {
        const int jw = (d - j0) < jn ? (d - j0) : jn;
        for (int f0 = 0; f0 < nf; f0 += chunk) {
            const int fn = (nf - f0) < chunk ? (nf - f0) : chunk;
            for (int e = tid; e < fn * per_cluster; e += blockDim.x) hist[e] = 0u;
            for (int q = tid; q < fn; q += blockDim.x) slot_of[flagged[f0 + q]] = q;
            __syncthreads();
            for (int64_t r = r0 + tid; r < r1; r += blockDim.x) {
                const int s = slot_of[a.labels_sel[r]];
                if (s < 0) continue;
                if (a.valid && a.valid[r] == 0) continue;
                unsigned *hrow = hist + (size_t)s * per_cluster;
                for (int j = 0; j < jw; ++j) {
                    const unsigned v = X[(int64_t)(j0 + j) * a.ld + r];
                    if (v < (unsigned)cmax) atomicAdd(&hrow[j * cmax + v], 1u);
                }
            }
            __syncthreads();
            for (int e = tid; e < fn * jw; e += blockDim.x) {
                const int q = e / jw, j = e % jw;
                const unsigned *hv = hist + (size_t)q * per_cluster + (size_t)j * cmax;
                int bv = 0;
                unsigned bc = hv[0];
                unsigned total = hv[0];
                for (int v = 1; v < cmax; ++v) {
                    total += hv[v];
                    if (v < card[j0 + j] && hv[v] > bc) {
                        bc = hv[v];
                        bv = v;
                    }
                }
                const int c = flagged[f0 + q];
                mode[c * d + j0 + j] = (XT)bv;
                if (j0 + j == 0) hasv[c] = total > 0 ? 1 : 0;
            }
            __syncthreads();
            for (int q = tid; q < fn; q += blockDim.x) slot_of[flagged[f0 + q]] = -1;
            __syncthreads();
        }
    }

    // C. accept or drop, in ascending cluster order, by the first wave
    if (tid < kWave) {
        const int lane = tid;
        for (int f = 0; f < nf; ++f) {
            const int c = flagged[f];
            if (!hasv[c]) continue;
            const XT *m = mode + c * d;
            bool dup = false;
            for (int q = lane; q < k; q += kWave) {
                const int fq = fl[q];
                if (fq == 1 || (fq == 2 && q < c)) {
                    bool same = true;
                    for (int j = 0; j < d && same; ++j) same = cfg[q * d + j] == m[j];
                    dup = dup || same;
                }
            }
            uint64_t h = fnv_begin(salt);
            for (int j = 0; j < d; ++j) h = fnv_step(h, m[j]);
            const bool vis = visited_has(a.visited, a.n_visited, h);
            const bool any_dup = __ballot(dup) != 0ull;
            if (!vis && !any_dup) {
                if (lane == 0) fl[c] = 2;       // CHAM_OUT_SYNTH
                for (int j = lane; j < d; j += kWave) cfg[c * d + j] = m[j];
            }
            __builtin_amdgcn_wave_barrier();
            __threadfence_block();
        }
    }
    __syncthreads();
    for (int e = tid; e < kmax * d; e += blockDim.x) ocfg[e] = cfg[e];
    for (int c = tid; c < kmax; c += blockDim.x) oflag[c] = fl[c];
    if (tid == 0) {
        int cnt = 0;
        for (int c = 0; c < k; ++c) cnt += (fl[c] == 1 || fl[c] == 2) ? 1 : 0;
        a.out_count[t] = cnt;
    }
}

template <typename XT>
__global__ void hash_rows_kernel(const XT *rows, int64_t n, int d, const uint64_t *salts,
                                 uint64_t salt_all, uint64_t *out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    uint64_t h = fnv_begin(salts ? salts[i] : salt_all);
    for (int j = 0; j < d; ++j) h = fnv_step(h, rows[i * d + j]);
    out[i] = h;
}


// ---------------------------------------------------------------------------------------------
// Wide variants for tasks too large for one workgroup: the same steps, split over 4096-row chunks
// with per-cluster minima and value histograms combined through global atomics.

constexpr int kWideRows = 4096;

__device__ __forceinline__ void wide_locate(const int *wg_off, int T, int &t, int &chunk)
{
    int lo = 0, hi = T;                        // last task with wg_off[task] <= blockIdx.x
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (wg_off[mid] <= (int)blockIdx.x) lo = mid; else hi = mid;
    }
    t = lo;
    chunk = (int)blockIdx.x - wg_off[lo];
}

__global__ void snap_wide_init_kernel(const SnapArgs a)
{
    const int t = blockIdx.x;
    for (int c = threadIdx.x; c < a.kmax; c += blockDim.x) {
        a.pick_row[(int64_t)t * a.kmax + c] = -1;
        a.wide_best[(int64_t)t * a.kmax + c] = ~0ull;
        a.wide_row[(int64_t)t * a.kmax + c] = 0x7fffffff;
    }
    for (int e = threadIdx.x; e < a.kmax * a.d; e += blockDim.x) a.pick_cfg[(int64_t)t * a.kmax * a.d + e] = 0;
}

template <int DP, int MAXNT>
__global__ __launch_bounds__(MAXNT) void snap_wide_assign_kernel(const SnapArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    SnapLds<DP> U(smem, a.kmax);
    __shared__ int loc[2];
    const int tid = threadIdx.x;
    if (tid == 0) wide_locate(a.wg_off, a.T, loc[0], loc[1]);
    __syncthreads();
    const int t = loc[0];
    const int d = a.d;
    const int ci = a.chosen[t];
    if (ci < 0 || ci >= a.n_k) return;
    const int64_t t0 = a.task_off[t], t1 = a.task_off[t + 1];
    const int64_t r0 = t0 + (int64_t)loc[1] * kWideRows;
    const int64_t r1 = r0 + kWideRows < t1 ? r0 + kWideRows : t1;
    const int k = a.ks[ci];
    const int kp = k;
    const int64_t crow = (int64_t)t * a.Ksum + a.koff[ci];
    const int tile_rows = blockDim.x * kRowsPerThread;

    for (int e = tid; e < DP * kp; e += blockDim.x) U.mu64T[e] = 0.0;
    for (int c = tid; c < k; c += blockDim.x) U.best[c] = ~0ull;
    if (tid == 0) *U.m2bits = 0u;
    __syncthreads();
    for (int e = tid; e < k * d; e += blockDim.x) {
        const int c = e / d, j = e % d;
        U.mu64T[(size_t)j * kp + c] = a.centroids[(crow + c) * d + j];
    }
    __syncthreads();
    if (tid < DP) {
        float o = 0.0f;
        if (tid < d) {
            double s = 0.0;
            for (int c = 0; c < k; ++c) s += U.mu64T[(size_t)tid * kp + c];
            double m = rint(s / (double)k);
            m = m < 0.0 ? 0.0 : (m > 255.0 ? 255.0 : m);
            o = (float)m;
        }
        U.ojf[tid] = o;
    }
    __syncthreads();
    for (int c = tid; c < k; c += blockDim.x) {
        double b = 0.0;
        float *w = U.wf + (size_t)c * (DP + 4);
#pragma unroll
        for (int j = 0; j < DP; ++j) {
            const double m = U.mu64T[(size_t)j * kp + c] - (double)U.ojf[j];
            b = __builtin_fma(m, m, b);
            w[j] = (float)(-2.0 * m);
        }
        w[DP] = (float)b;
        w[DP + 1] = w[DP + 2] = w[DP + 3] = 0.0f;
        atomicMax(U.m2bits, __float_as_uint(__double2float_ru(b) * 1.0000005f));
    }
    __syncthreads();

    CentroidView L;
    L.mu64T = U.mu64T;
    L.wf = U.wf;
    L.ojf = U.ojf;
    L.m2 = __uint_as_float(*U.m2bits);
    L.kp = kp;
    L.k = k;
    const bool force_exact = (a.flags & 1) != 0;
    const int64_t g0 = r0 & ~(int64_t)3;
    const int ntiles = (int)((r1 - g0 + tile_rows - 1) / tile_rows);
    for (int tile = 0; tile < ntiles; ++tile) {
        const int64_t g = g0 + (int64_t)tile * tile_rows + (int64_t)tid * kRowsPerThread;
        const bool in_range = g < r1;
        uint32_t rowmask = 0;
#pragma unroll
        for (int p = 0; p < 4; ++p)
            if (g + p >= r0 && g + p < r1) rowmask |= 1u << p;
        float xf[4][DP];
        float x2[4];
        load_rows<DP>(a.X, a.ld, d, g, in_range, U.ojf, xf, x2);
        int lab[4];
        double dist[4] = {0.0, 0.0, 0.0, 0.0};
        assign_rows<DP>(xf, x2, rowmask, L, force_exact, true, lab, dist);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            if (!((rowmask >> p) & 1u)) continue;
            a.labels_sel[g + p] = (uint8_t)lab[p];
            a.dist_ws[g + p] = dist[p];
            atomicMin(&U.best[lab[p]], (unsigned long long)__double_as_longlong(dist[p]));
        }
    }
    __syncthreads();
    for (int c = tid; c < k; c += blockDim.x)
        if (U.best[c] != ~0ull) atomicMin(&a.wide_best[(int64_t)t * a.kmax + c], U.best[c]);
}

__global__ void snap_wide_pick_kernel(const SnapArgs a)
{
    __shared__ int loc[2];
    __shared__ int brow[256];
    const int tid = threadIdx.x;
    if (tid == 0) wide_locate(a.wg_off, a.T, loc[0], loc[1]);
    for (int c = tid; c < 256; c += blockDim.x) brow[c] = 0x7fffffff;
    __syncthreads();
    const int t = loc[0];
    const int ci = a.chosen[t];
    if (ci < 0 || ci >= a.n_k) return;
    const int k = a.ks[ci];
    const int64_t t0 = a.task_off[t], t1 = a.task_off[t + 1];
    const int64_t r0 = t0 + (int64_t)loc[1] * kWideRows;
    const int64_t r1 = r0 + kWideRows < t1 ? r0 + kWideRows : t1;
    for (int64_t r = r0 + tid; r < r1; r += blockDim.x) {
        const int c = a.labels_sel[r];
        if ((unsigned long long)__double_as_longlong(a.dist_ws[r]) == a.wide_best[(int64_t)t * a.kmax + c])
            atomicMin(&brow[c], (int)(r - t0));
    }
    __syncthreads();
    for (int c = tid; c < k; c += blockDim.x)
        if (brow[c] != 0x7fffffff) atomicMin(&a.wide_row[(int64_t)t * a.kmax + c], brow[c]);
}

__global__ void snap_wide_finish_kernel(const SnapArgs a)
{
    const int t = blockIdx.x;
    const int ci = a.chosen[t];
    if (ci < 0 || ci >= a.n_k) return;
    const int k = a.ks[ci];
    const int d = a.d;
    const int64_t t0 = a.task_off[t];
    for (int e = threadIdx.x; e < k * d; e += blockDim.x) {
        const int c = e / d, j = e % d;
        const int row = a.wide_row[(int64_t)t * a.kmax + c];
        if (row != 0x7fffffff) {
            a.pick_cfg[((int64_t)t * a.kmax + c) * d + j] = a.X[(int64_t)j * a.ld + t0 + row];
            if (j == 0) a.pick_row[(int64_t)t * a.kmax + c] = row;
        }
    }
}

// Synthesis, wide: flag picks (one workgroup per task), value histograms of the flagged clusters
// over row chunks, then modes and the ordered accept / drop per task.
__global__ __launch_bounds__(256) void synth_wide_flag_kernel(const SynthArgs a)
{
    __shared__ int nf_sh;
    const int tid = threadIdx.x;
    const int t = blockIdx.x;
    const int d = a.d, kmax = a.kmax;
    const int64_t r0 = a.task_off[t];
    const int ci = a.chosen[t];
    const int k = (ci >= 0 && ci < a.n_k) ? a.ks[ci] : 0;
    const uint64_t salt = a.salts[t];
    uint8_t *ocfg = a.out_cfg + (int64_t)t * kmax * d;
    uint8_t *oflag = a.out_flag + (int64_t)t * kmax;
    int *slot_of = a.wide_slot + (int64_t)t * kmax;
    for (int e = tid; e < kmax * d; e += blockDim.x) ocfg[e] = 0;
    for (int c = tid; c < kmax; c += blockDim.x) {
        int f = 0;
        slot_of[c] = -1;
        if (c < k) {
            const int row = a.pick_row[(int64_t)t * kmax + c];
            if (row >= 0) {
                const uint8_t *pc = a.pick_cfg + ((int64_t)t * kmax + c) * d;
                uint64_t h = fnv_begin(salt);
                for (int j = 0; j < d; ++j) h = fnv_step(h, pc[j]);
                const bool invalid = a.valid && a.valid[r0 + row] == 0;
                f = (invalid || visited_has(a.visited, a.n_visited, h)) ? 3 : 1;
            }
        }
        oflag[c] = (uint8_t)f;
    }
    __syncthreads();
    for (int c = tid; c < k; c += blockDim.x) {
        if (oflag[c] == 1) {
            const uint8_t *pc = a.pick_cfg + ((int64_t)t * kmax + c) * d;
            for (int j = 0; j < d; ++j) ocfg[c * d + j] = pc[j];
        }
    }
    if (tid == 0) {
        int nf = 0;
        for (int c = 0; c < k; ++c)
            if (oflag[c] == 3) {
                a.wide_list[(int64_t)t * kmax + nf] = c;
                slot_of[c] = nf++;
            }
        a.wide_nf[t] = nf;
        nf_sh = nf;
    }
    __syncthreads();
    const int64_t words = (int64_t)nf_sh * d * a.wide_cmax;
    unsigned *hist = a.wide_hist + (int64_t)t * kmax * d * a.wide_cmax;
    for (int64_t e = tid; e < words; e += blockDim.x) hist[e] = 0u;
}

__global__ __launch_bounds__(1024) void synth_wide_hist_kernel(const SynthArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned *lh = reinterpret_cast<unsigned *>(smem);
    __shared__ int loc[2];
    const int tid = threadIdx.x;
    if (tid == 0) wide_locate(a.wg_off, a.T, loc[0], loc[1]);
    __syncthreads();
    const int t = loc[0];
    const int nf = a.wide_nf[t];
    if (nf == 0) return;
    const int d = a.d, kmax = a.kmax, cmax = a.wide_cmax;
    const int64_t t0 = a.task_off[t], t1 = a.task_off[t + 1];
    const int64_t r0 = t0 + (int64_t)loc[1] * kWideRows;
    const int64_t r1 = r0 + kWideRows < t1 ? r0 + kWideRows : t1;
    const int *slot_of = a.wide_slot + (int64_t)t * kmax;
    unsigned *hist = a.wide_hist + (int64_t)t * kmax * d * cmax;
    const uint16_t *card = a.cards + (int64_t)t * d;
    int tcmax = 1;                             // values at or above the task's largest cardinality are not counted
    for (int j = 0; j < d; ++j) tcmax = card[j] > tcmax ? card[j] : tcmax;
    const int per_cluster = d * cmax;
    const int chunk = a.hist_words / per_cluster;
    for (int f0 = 0; f0 < nf; f0 += chunk) {
        const int fn = (nf - f0) < chunk ? (nf - f0) : chunk;
        for (int e = tid; e < fn * per_cluster; e += blockDim.x) lh[e] = 0u;
        __syncthreads();
        for (int64_t r = r0 + tid; r < r1; r += blockDim.x) {
            const int s = slot_of[a.labels_sel[r]] - f0;
            if (s < 0 || s >= fn) continue;
            if (a.valid && a.valid[r] == 0) continue;
            unsigned *hrow = lh + (size_t)s * per_cluster;
            for (int j = 0; j < d; ++j) {
                const unsigned v = a.X[(int64_t)j * a.ld + r];
                if (v < (unsigned)tcmax) atomicAdd(&hrow[j * cmax + v], 1u);
            }
        }
        __syncthreads();
        for (int e = tid; e < fn * per_cluster; e += blockDim.x) {
            const unsigned v = lh[e];
            if (v) atomicAdd(&hist[(size_t)f0 * per_cluster + e], v);
        }
        __syncthreads();
    }
}

__global__ __launch_bounds__(256) void synth_wide_finish_kernel(const SynthArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    const int t = blockIdx.x;
    const int d = a.d, kmax = a.kmax, cmax = a.wide_cmax;
    const int ci = a.chosen[t];
    const int k = (ci >= 0 && ci < a.n_k) ? a.ks[ci] : 0;
    const int nf = a.wide_nf[t];
    const uint64_t salt = a.salts[t];
    const uint16_t *card = a.cards + (int64_t)t * d;
    uint8_t *ocfg = a.out_cfg + (int64_t)t * kmax * d;
    uint8_t *oflag = a.out_flag + (int64_t)t * kmax;
    const int *flagged = a.wide_list + (int64_t)t * kmax;
    const unsigned *hist = a.wide_hist + (int64_t)t * kmax * d * cmax;
    uint8_t *cfg = smem;                       // [kmax][d]
    uint8_t *mode = cfg + (size_t)kmax * d;    // [kmax][d]
    uint8_t *fl = mode + (size_t)kmax * d;     // [kmax]
    uint8_t *hasv = fl + kmax;                 // [kmax]
    for (int e = tid; e < kmax * d; e += blockDim.x) cfg[e] = ocfg[e];
    for (int c = tid; c < kmax; c += blockDim.x) {
        fl[c] = oflag[c];
        hasv[c] = 0;
    }
    __syncthreads();
    int tcmax = 1;
    for (int j = 0; j < d; ++j) tcmax = card[j] > tcmax ? card[j] : tcmax;
    for (int e = tid; e < nf * d; e += blockDim.x) {
        const int q = e / d, j = e % d;
        const unsigned *hv = hist + ((size_t)q * d + j) * cmax;
        int bv = 0;
        unsigned bc = hv[0], total = hv[0];
        for (int v = 1; v < tcmax; ++v) {
            total += hv[v];
            if (v < card[j] && hv[v] > bc) {
                bc = hv[v];
                bv = v;
            }
        }
        const int c = flagged[q];
        mode[c * d + j] = (uint8_t)bv;
        if (j == 0) hasv[c] = total > 0 ? 1 : 0;
    }
    __syncthreads();
    if (tid < kWave) {
        const int lane = tid;
        for (int f = 0; f < nf; ++f) {
            const int c = flagged[f];
            if (!hasv[c]) continue;
            const uint8_t *m = mode + c * d;
            bool dup = false;
            for (int q = lane; q < k; q += kWave) {
                const int fq = fl[q];
                if (fq == 1 || (fq == 2 && q < c)) {
                    bool same = true;
                    for (int j = 0; j < d && same; ++j) same = cfg[q * d + j] == m[j];
                    dup = dup || same;
                }
            }
            uint64_t h = fnv_begin(salt);
            for (int j = 0; j < d; ++j) h = fnv_step(h, m[j]);
            const bool vis = visited_has(a.visited, a.n_visited, h);
            const bool any_dup = __ballot(dup) != 0ull;
            if (!vis && !any_dup) {
                if (lane == 0) fl[c] = 2;
                for (int j = lane; j < d; j += kWave) cfg[c * d + j] = m[j];
            }
            __builtin_amdgcn_wave_barrier();
            __threadfence_block();
        }
    }
    __syncthreads();
    for (int e = tid; e < kmax * d; e += blockDim.x) ocfg[e] = cfg[e];
    for (int c = tid; c < kmax; c += blockDim.x) oflag[c] = fl[c];
    if (tid == 0) {
        int cnt = 0;
        for (int c = 0; c < k; ++c) cnt += (fl[c] == 1 || fl[c] == 2) ? 1 : 0;
        a.out_count[t] = cnt;
    }
}

template <int DP, int MAXNT>
hipError_t launch_snap_wide_dp(const SnapArgs &a, int total_wgs, hipStream_t s)
{
    const size_t lds = resident_lds_bytes(DP, a.kmax);
    auto kern = snap_wide_assign_kernel<DP, MAXNT>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(snap_wide_init_kernel, dim3(a.T), dim3(256), 0, s, a);
    hipLaunchKernelGGL(kern, dim3(total_wgs), dim3(MAXNT), lds, s, a);
    hipLaunchKernelGGL(snap_wide_pick_kernel, dim3(total_wgs), dim3(1024), 0, s, a);
    hipLaunchKernelGGL(snap_wide_finish_kernel, dim3(a.T), dim3(256), 0, s, a);
    return hipGetLastError();
}

template <typename XT, int DP, int R, int MAXNT>
hipError_t launch_snap_dp(const SnapArgs &a, int nt, hipStream_t s)
{
    const size_t lds = resident_lds_bytes(DP, a.kmax);
    auto kern = snap_kernel<XT, DP, R, MAXNT>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    if (nt > MAXNT) nt = MAXNT;
    hipLaunchKernelGGL(kern, dim3(a.T), dim3(nt), lds, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_knee_update(const double *inertia, const int *status, int T, int n_k, int ki_end, double thr,
                              int *done, hipStream_t s)
{
    hipLaunchKernelGGL(knee_update_kernel, dim3((T + 127) / 128), dim3(128), 0, s, inertia, status, T, n_k, ki_end, thr,
                       done);
    return hipGetLastError();
}

hipError_t launch_fill_i32(int *dst, int64_t n, int value, hipStream_t s)
{
    if (n > 0) hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, dst, n, value);
    return hipGetLastError();
}

hipError_t launch_select_k(const double *inertia, const int *status, int T, int n_k, double thr,
                           int *chosen, hipStream_t s)
{
    hipLaunchKernelGGL(select_k_kernel, dim3((T + 127) / 128), dim3(128), 0, s, inertia, status, T, n_k,
                       thr, chosen);
    return hipGetLastError();
}

hipError_t launch_snap(const SnapArgs &a, int nt, hipStream_t s)
{
    const int d = a.d;
    if (a.xbytes == 2) {
        if (d <= 8) return launch_snap_dp<uint16_t, 8, 4, 512>(a, nt, s);
        if (d <= 16) return launch_snap_dp<uint16_t, 16, 4, 512>(a, nt, s);
        if (d <= 24) return launch_snap_dp<uint16_t, 24, 4, 512>(a, nt, s);
        if (d <= 32) return launch_snap_dp<uint16_t, 32, 4, 512>(a, nt, s);
        if (d <= 40) return launch_snap_dp<uint16_t, 40, 2, 512>(a, nt, s);
        if (d <= 48) return launch_snap_dp<uint16_t, 48, 2, 512>(a, nt, s);
        if (d <= 56) return launch_snap_dp<uint16_t, 56, 2, 512>(a, nt, s);
        return launch_snap_dp<uint16_t, 64, 2, 512>(a, nt, s);
    }
    if (d <= 4) return launch_snap_dp<uint8_t, 4, 4, 1024>(a, nt, s);
    if (d <= 8) return launch_snap_dp<uint8_t, 8, 4, 1024>(a, nt, s);
    if (d <= 12) return launch_snap_dp<uint8_t, 12, 4, 1024>(a, nt, s);
    if (d <= 16) return launch_snap_dp<uint8_t, 16, 4, 512>(a, nt, s);
    if (d <= 20) return launch_snap_dp<uint8_t, 20, 4, 512>(a, nt, s);
    if (d <= 24) return launch_snap_dp<uint8_t, 24, 4, 512>(a, nt, s);
    if (d <= 28) return launch_snap_dp<uint8_t, 28, 4, 512>(a, nt, s);
    return launch_snap_dp<uint8_t, 32, 4, 512>(a, nt, s);
}

hipError_t launch_snap_wide(const SnapArgs &a, int total_wgs, hipStream_t s)
{
    const int d = a.d;
    if (d <= 4) return launch_snap_wide_dp<4, 1024>(a, total_wgs, s);
    if (d <= 8) return launch_snap_wide_dp<8, 1024>(a, total_wgs, s);
    if (d <= 12) return launch_snap_wide_dp<12, 1024>(a, total_wgs, s);
    if (d <= 16) return launch_snap_wide_dp<16, 512>(a, total_wgs, s);
    if (d <= 20) return launch_snap_wide_dp<20, 512>(a, total_wgs, s);
    if (d <= 24) return launch_snap_wide_dp<24, 512>(a, total_wgs, s);
    if (d <= 28) return launch_snap_wide_dp<28, 512>(a, total_wgs, s);
    return launch_snap_wide_dp<32, 512>(a, total_wgs, s);
}

hipError_t launch_synth_wide(const SynthArgs &a, int total_wgs, hipStream_t s)
{
    const size_t lds_hist = sizeof(unsigned) * (size_t)a.hist_words;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(synth_wide_hist_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_hist);
    if (e != hipSuccess) return e;
    const size_t lds_fin = (size_t)a.kmax * a.d * 2 + (size_t)a.kmax * 2 + 16;
    hipLaunchKernelGGL(synth_wide_flag_kernel, dim3(a.T), dim3(256), 0, s, a);
    hipLaunchKernelGGL(synth_wide_hist_kernel, dim3(total_wgs), dim3(1024), lds_hist, s, a);
    hipLaunchKernelGGL(synth_wide_finish_kernel, dim3(a.T), dim3(256), lds_fin, s, a);
    return hipGetLastError();
}

size_t synth_lds_bytes(int d, int kmax, int hist_words, int xbytes)
{
    size_t b = sizeof(unsigned) * (size_t)hist_words;
    b += sizeof(int) * (size_t)kmax * 2 + sizeof(int) * 8;
    b += (size_t)xbytes * kmax * d * 2 + (size_t)kmax * 2;
    return (b + 15) & ~(size_t)15;
}

hipError_t launch_synth(const SynthArgs &a, int nt, hipStream_t s)
{
    const size_t lds = synth_lds_bytes(a.d, a.kmax, a.hist_words, a.xbytes);
    auto kern = a.xbytes == 2 ? synth_kernel<uint16_t> : synth_kernel<uint8_t>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(a.T), dim3(nt), lds, s, a);
    return hipGetLastError();
}

hipError_t launch_table_clear(uint64_t *v, int64_t slots, hipStream_t s)
{
    hipLaunchKernelGGL(table_clear_kernel, dim3((unsigned)((slots + 255) / 256)), dim3(256), 0, s, v, slots);
    return hipGetLastError();
}

hipError_t launch_table_insert_hashes(uint64_t *v, int64_t slots, const uint64_t *hashes, int64_t n, int *overflow,
                                      hipStream_t s)
{
    if (n > 0)
        hipLaunchKernelGGL(table_insert_hashes_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, v, slots,
                           hashes, n, overflow);
    return hipGetLastError();
}

hipError_t launch_table_insert_configs(uint64_t *v, int64_t slots, const void *cfgs, int xbytes, int64_t n, int d,
                                       const uint8_t *flags, const uint64_t *salts, int64_t rows_per_salt,
                                       int *overflow, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const dim3 grid((unsigned)((n + 255) / 256));
    if (xbytes == 2)
        hipLaunchKernelGGL(table_insert_configs_kernel<uint16_t>, grid, dim3(256), 0, s, v, slots,
                           static_cast<const uint16_t *>(cfgs), n, d, flags, salts, rows_per_salt, overflow);
    else
        hipLaunchKernelGGL(table_insert_configs_kernel<uint8_t>, grid, dim3(256), 0, s, v, slots,
                           static_cast<const uint8_t *>(cfgs), n, d, flags, salts, rows_per_salt, overflow);
    return hipGetLastError();
}

hipError_t launch_update_configs(uint8_t *theta, const int8_t *actions, int64_t B, int d, int n_steps,
                                 const uint16_t *cards, uint64_t salt, uint64_t *seen, int64_t slots,
                                 uint8_t *unique_rows, int64_t cap, int *n_unique, int *overflow, hipStream_t s)
{
    if (B > 0)
        hipLaunchKernelGGL(update_configs_kernel, dim3((unsigned)(B < (1 << 20) ? B : (1 << 20))), dim3(kUpdThreads), 0, s,
                           theta, actions, B, d, n_steps, cards, salt, seen, slots, unique_rows, cap, n_unique, overflow);
    return hipGetLastError();
}

hipError_t launch_hash_rows(const void *rows, int xbytes, int64_t n, int d, const uint64_t *salts,
                            uint64_t salt_all, uint64_t *out, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const dim3 grid((unsigned)((n + 255) / 256));
    if (xbytes == 2)
        hipLaunchKernelGGL(hash_rows_kernel<uint16_t>, grid, dim3(256), 0, s, static_cast<const uint16_t *>(rows), n, d,
                           salts, salt_all, out);
    else
        hipLaunchKernelGGL(hash_rows_kernel<uint8_t>, grid, dim3(256), 0, s, static_cast<const uint8_t *>(rows), n, d,
                           salts, salt_all, out);
    return hipGetLastError();
}

}  // namespace cham
