// C ABI of libcham: argument checks, workspace carving, staging of the small host arrays and
// kernel launches for the Adaptive Sampling path (paper Sec. 3.3, Algorithm 1).
#include "../../include/cham.h"

#include <stdlib.h>
#include <string.h>

#include "cham_internal.h"

namespace cham {

namespace {

thread_local int32_t g_last_hip = 0;

int32_t hip_fail(hipError_t e)
{
    g_last_hip = (int32_t)e;
    return CHAM_E_HIP;
}

constexpr int64_t kAlign = 256;
inline int64_t up(int64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// Growable array of 64-bit words for the small host-side tables.  The first kInline words live
// inside the object; beyond that it takes heap memory with malloc and reports failure through its
// return value (nothing in the library throws).  With heap use forbidden (the entry point that must
// not allocate) a request beyond the inline part fails the same way.
class Words {
public:
    static constexpr size_t kInline = 1024;
    Words() = default;
    Words(const Words &) = delete;
    Words &operator=(const Words &) = delete;
    ~Words() { free(heap_); }
    void forbid_heap() { heap_ok_ = false; }
    // n zero words, previous content dropped
    bool assign(size_t n)
    {
        n_ = 0;
        return resize(n);
    }
    // n words, the first min(n, size) kept, the rest zero
    bool resize(size_t n)
    {
        if (n > cap_) {
            if (!heap_ok_) return false;
            size_t cap = cap_ * 2 > n ? cap_ * 2 : n;
            uint64_t *h = static_cast<uint64_t *>(malloc(cap * sizeof(uint64_t)));
            if (!h) return false;
            memcpy(h, data(), n_ * sizeof(uint64_t));
            free(heap_);
            heap_ = h;
            cap_ = cap;
        }
        if (n > n_) memset(data() + n_, 0, (n - n_) * sizeof(uint64_t));
        n_ = n;
        return true;
    }
    uint64_t *data() { return heap_ ? heap_ : inl_; }
    const uint64_t *data() const { return heap_ ? heap_ : inl_; }
    size_t size() const { return n_; }
    uint64_t &operator[](size_t i) { return data()[i]; }
    const uint64_t &operator[](size_t i) const { return data()[i]; }

private:
    uint64_t inl_[kInline];
    uint64_t *heap_ = nullptr;
    size_t n_ = 0, cap_ = kInline;
    bool heap_ok_ = true;
};

// Small host arrays travel to the device inside kernel arguments (copied at launch time), so
// no host buffer has to outlive the call and no device memory is allocated.
constexpr int kPokeWords = 496;           // with the two fields below just under the 4 KiB of kernel arguments
constexpr int kPokeThreads = 512;
struct PokeArgs {
    uint64_t v[kPokeWords];
    uint64_t *dst;
    int n;
};
static_assert(sizeof(PokeArgs) <= 4096 && kPokeWords <= kPokeThreads, "one thread per word, arguments within 4 KiB");
__global__ void poke_kernel(const PokeArgs p)
{
    const int i = threadIdx.x;
    if (i < p.n) p.dst[i] = p.v[i];
}

hipError_t stage_words(const Words &blob, uint64_t *dst, hipStream_t s)
{
    for (size_t o = 0; o < blob.size(); o += kPokeWords) {
        PokeArgs p;
        p.n = (int)((blob.size() - o) < (size_t)kPokeWords ? (blob.size() - o) : (size_t)kPokeWords);
        for (int i = 0; i < p.n; ++i) p.v[i] = blob[o + i];
        p.dst = dst + o;
        hipLaunchKernelGGL(poke_kernel, dim3(1), dim3(kPokeThreads), 0, s, p);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// Host blob: [task_off (T+1) x i64][ks n_k x i32][koff (n_k+1) x i32][extra ...], 8-byte units.
struct Plan {
    int T = 0, n_k = 0, Ksum = 0, kmax = 0, DP = 0, nt = 0;
    int64_t n_total = 0, n_max = 0;
    Words blob;
    int64_t off_task = 0, off_ks = 0, off_koff = 0, off_extra = 0;   // byte offsets in the blob
};

// xbytes: bytes per knob value (1, or 2 for the *_u16 entry points).
int32_t check_common(const void *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                     const int32_t *ks, int32_t n_k, bool need_x, Plan &pl, int xbytes = 1)
{
    if ((need_x && !X) || !task_off || !ks) return CHAM_E_NULL;
    if (d < 1 || d > (xbytes == 1 ? 32 : 64) || T < 1 || ld < 0 || (ld % 4) != 0) return CHAM_E_BAD_DIM;
    if (need_x && (reinterpret_cast<uintptr_t>(X) % (4 * xbytes)) != 0) return CHAM_E_BAD_DIM;
    if (n_k < 1 || n_k > 256) return CHAM_E_BAD_K;
    int64_t ksum = 0;
    for (int i = 0; i < n_k; ++i) {
        if (ks[i] < 1 || ks[i] > 256) return CHAM_E_BAD_K;
        if (i > 0 && ks[i] <= ks[i - 1]) return CHAM_E_BAD_K;
        ksum += ks[i];
    }
    if (task_off[0] < 0) return CHAM_E_BAD_OFFSETS;
    int64_t nmax = 0;
    for (int t = 0; t < T; ++t) {
        const int64_t n = task_off[t + 1] - task_off[t];
        if (n < 0 || n > ((int64_t)1 << 23)) return CHAM_E_BAD_OFFSETS;
        if (n > nmax) nmax = n;
    }
    if (task_off[T] > ld) return CHAM_E_BAD_DIM;
    pl.T = T;
    pl.n_k = n_k;
    pl.Ksum = (int)ksum;
    pl.kmax = ks[n_k - 1];
    pl.DP = xbytes == 1 ? (d + 3) / 4 * 4 : resident_dp16(d);
    pl.n_total = task_off[T];
    pl.n_max = nmax;
    const int maxnt = (xbytes == 1 && pl.DP <= 12) ? 1024 : 512;
    const int rpt = (xbytes == 2 && pl.DP > 32) ? 2 : 4;           // rows per lane and pass
    int64_t nt = ((nmax + 2 * (rpt - 1)) / rpt + 63) / 64 * 64;
    if (nt < 64) nt = 64;
    if (nt > maxnt) nt = maxnt;
    pl.nt = (int)nt;

    // blob
    const size_t w_task = (size_t)T + 1;
    const size_t w_ks = ((size_t)n_k + 1) / 2;
    const size_t w_koff = ((size_t)n_k + 2) / 2;
    if (!pl.blob.assign(w_task + w_ks + w_koff)) return CHAM_E_NOMEM;
    for (int t = 0; t <= T; ++t) pl.blob[t] = (uint64_t)task_off[t];
    int32_t *pk = reinterpret_cast<int32_t *>(pl.blob.data() + w_task);
    for (int i = 0; i < n_k; ++i) pk[i] = ks[i];
    int32_t *po = reinterpret_cast<int32_t *>(pl.blob.data() + w_task + w_ks);
    int acc = 0;
    for (int i = 0; i < n_k; ++i) {
        po[i] = acc;
        acc += ks[i];
    }
    po[n_k] = acc;
    pl.off_task = 0;
    pl.off_ks = (int64_t)w_task * 8;
    pl.off_koff = (int64_t)(w_task + w_ks) * 8;
    pl.off_extra = (int64_t)(w_task + w_ks + w_koff) * 8;
    return CHAM_OK;
}

constexpr int kStreamRowsPerWg = 4096;      // the smallest value of stream_rows_per_wg: bounds the workgroup count

constexpr int kSweepFlags = CHAM_F_FORCE_EXACT | CHAM_F_STREAMING | CHAM_F_RESIDENT | CHAM_F_NO_MFMA | CHAM_F_VALUES_BELOW_2048;

// Which kernel family runs the sweep.
enum class SweepPath { kMfmaResident, kVectorResident, kStream };

SweepPath choose_path(const Plan &pl, int d, int flags, int xbytes = 1)
{
    const bool exact = (flags & CHAM_F_FORCE_EXACT) != 0;
    const bool no_mfma = (flags & CHAM_F_NO_MFMA) != 0;
    if (xbytes == 2) {
        // two-byte knobs: the f16 rows of the matrix-core kernel hold integers below 2048 only, which the
        // caller has to promise (the kernel checks); there is no streaming variant for them
        const bool promised = (flags & CHAM_F_VALUES_BELOW_2048) != 0;
        if (promised && !exact && !no_mfma && mfma_path_fits_u16(d, pl.kmax, pl.n_max)) return SweepPath::kMfmaResident;
        return SweepPath::kVectorResident;
    }
    if (exact || no_mfma || d > 31) return SweepPath::kVectorResident;
    if (flags & CHAM_F_STREAMING) return SweepPath::kStream;
    if (mfma_path_fits(d, pl.kmax, pl.n_max)) return SweepPath::kMfmaResident;
    if (flags & CHAM_F_RESIDENT) return SweepPath::kVectorResident;
    return SweepPath::kStream;
}

struct SweepWs {
    int64_t blob = 0, init_rows = 0, ndist = 0, passes = 0, counters = 0, xh = 0, labbuf = 0, total = 0;
    // streaming path
    int64_t x2 = 0, ojf = 0, Sg = 0, ng = 0, mu = 0, afrag = 0, biasf = 0, m2 = 0, wg_off = 0, loss = 0;
    int kpm = 0, n_units = 0, total_wgs = 0;
};

// xh_halfs: f16 values per row of the packed copy of the rows (0: the path needs none).
SweepWs sweep_ws(const Plan &pl, int64_t ld, bool own_labels, bool stream, const int64_t *task_off,
                 int xh_halfs = 32)
{
    SweepWs w;
    int64_t o = 0;
    w.blob = o;
    o += up((int64_t)pl.blob.size() * 8);
    w.init_rows = o;
    o += up((int64_t)pl.T * pl.kmax * 4);
    w.ndist = o;
    o += up((int64_t)pl.T * 4);
    w.passes = o;
    o += up((int64_t)pl.T * pl.n_k * 4);
    w.counters = o;                                   // one work counter per launch of a chunked sweep
    o += up(((int64_t)pl.n_k + 1) * 4);               // (+ the flag of a two-byte value too large for the f16 rows)
    w.xh = o;
    o += up(ld * xh_halfs * 2);
    w.labbuf = o;
    if (own_labels) o += up((int64_t)pl.n_k * ld);
    if (stream) {
        w.kpm = (pl.kmax + 31) / 32 * 32;
        w.n_units = pl.T * pl.n_k;
        int64_t wgs_per_sweep_of_tasks = 0;
        for (int t = 0; t < pl.T; ++t)
            wgs_per_sweep_of_tasks += (task_off[t + 1] - task_off[t] + kStreamRowsPerWg - 1) / kStreamRowsPerWg;
        w.total_wgs = (int)(wgs_per_sweep_of_tasks * pl.n_k);
        const int64_t u = w.n_units, kpm = w.kpm;
        w.x2 = o;      o += up(ld * 4);
        w.ojf = o;     o += up((int64_t)pl.T * 32 * 4);
        w.Sg = o;      o += up(u * kpm * 32 * 4);
        w.ng = o;      o += up(u * kpm * 4);
        w.mu = o;      o += up(u * 32 * kpm * 8);
        w.afrag = o;   o += up(u * (kpm / 32) * 4 * 64 * 16);
        w.biasf = o;   o += up(u * kpm * 4);
        w.m2 = o;      o += up(u * 8 * 4);
        w.wg_off = o;  o += up((u + 2) * 4);
        w.loss = o;    o += up(((int64_t)w.total_wgs + 1) * 8);
    }
    w.total = o;
    return w;
}

}  // namespace

}  // namespace cham

using namespace cham;

extern "C" {

int32_t cham_version(void) { return 100; }

int32_t cham_last_hip_error(void) { return g_last_hip; }

const char *cham_strerror(int32_t code)
{
    switch (code) {
    case CHAM_OK: return "ok";
    case CHAM_E_NULL: return "a required pointer is NULL";
    case CHAM_E_BAD_DIM: return "bad dimension (d outside [1,32], or [1,64] for two-byte knobs; ld < rows or not a multiple of 4; misaligned X; n_iter < 0; T < 1)";
    case CHAM_E_BAD_K: return "bad k list (empty, not strictly increasing, outside [1,256], or too large for the knob count of two-byte knobs)";
    case CHAM_E_BAD_OFFSETS: return "bad task offsets (negative, decreasing, or a task above 2^23 rows)";
    case CHAM_E_CARD: return "bad cardinality (0, above 256, or above 16384 for two-byte knobs)";
    case CHAM_E_WORKSPACE: return "workspace missing or too small";
    case CHAM_E_HIP: return "HIP runtime error (see cham_last_hip_error)";
    case CHAM_E_BAD_FLAG: return "unknown flag bits or init mode";
    case CHAM_E_NOMEM: return "out of host memory for the call's small tables";
    case CHAM_E_TOO_LARGE: return "input needs more scratch memory than the library's static buffer holds (use the entry point that takes a workspace)";
    default: return "unknown error code";
    }
}

// Two-byte knobs always run the vector resident kernel; its LDS need bounds k * padded knob count.
static bool u16_fits(const Plan &pl) { return resident_lds_bytes(pl.DP, pl.kmax, 8) <= 160 * 1024; }

static int64_t sweep_ws_bytes(int xbytes, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                              const int32_t *ks, int32_t n_k, int32_t flags, bool no_heap = false)
{
    Plan pl;
    if (no_heap) pl.blob.forbid_heap();
    const int32_t rc = check_common(nullptr, ld, d, task_off, T, ks, n_k, false, pl, xbytes);
    if (rc != CHAM_OK) return rc;
    if (xbytes == 2) {
        if (choose_path(pl, d, flags, 2) == SweepPath::kMfmaResident)
            return sweep_ws(pl, ld, true, false, task_off, d <= 31 ? 32 : 64).total;
        return u16_fits(pl) ? sweep_ws(pl, ld, true, false, task_off, 0).total : CHAM_E_BAD_K;
    }
    return sweep_ws(pl, ld, true, choose_path(pl, d, flags) == SweepPath::kStream, task_off).total;
}

int64_t cham_sweep_workspace_bytes(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                   const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t flags)
{
    (void)n_iter;
    return sweep_ws_bytes(1, ld, d, task_off, T, ks, n_k, flags);
}

int64_t cham_sweep_workspace_bytes_u16(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                       const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t flags)
{
    (void)n_iter;
    return sweep_ws_bytes(2, ld, d, task_off, T, ks, n_k, flags);
}

// The sweep, whole (chunk <= 0) or in chunks of `chunk` values of k with the knee test between them:
// tasks whose loss curve has reached the knee are marked done and the later chunks skip them.
static int32_t sweep_impl(const void *Xv, int xbytes, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                          const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t init_mode,
                          const double *init_centroids, double *centroids, int32_t *counts,
                          double *inertia, int32_t *status, uint8_t *labels, double *inertia_trace,
                          void *workspace, int64_t workspace_bytes, int32_t flags, void *stream,
                          int32_t chunk, double threshold, int32_t *chosen_idx, bool no_heap = false)
{
    const uint8_t *X = static_cast<const uint8_t *>(Xv);
    Plan pl;
    if (no_heap) pl.blob.forbid_heap();
    int32_t rc = check_common(X, ld, d, task_off, T, ks, n_k, true, pl, xbytes);
    if (rc != CHAM_OK) return rc;
    if (!centroids || !counts || !inertia || !status) return CHAM_E_NULL;
    if (n_iter < 0) return CHAM_E_BAD_DIM;
    if (init_mode != 0 && init_mode != 1) return CHAM_E_BAD_FLAG;
    if (init_mode == 1 && !init_centroids) return CHAM_E_NULL;
    if (flags & ~kSweepFlags) return CHAM_E_BAD_FLAG;
    if (xbytes == 2 && (flags & CHAM_F_STREAMING)) return CHAM_E_BAD_FLAG;
    const SweepPath path = choose_path(pl, d, flags, xbytes);
    if (xbytes == 2 && path == SweepPath::kVectorResident && !u16_fits(pl)) return CHAM_E_BAD_K;
    const int xh_halfs = xbytes == 1 ? 32 : (path == SweepPath::kMfmaResident ? (d <= 31 ? 32 : 64) : 0);
    const SweepWs w = sweep_ws(pl, ld, labels == nullptr, path == SweepPath::kStream, task_off, xh_halfs);
    const bool chunked = chunk > 0;
    const int64_t done_bytes = chunked ? up((int64_t)T * 4) : 0;
    if (!workspace || workspace_bytes < w.total + done_bytes) return CHAM_E_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return CHAM_E_WORKSPACE;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    unsigned char *ws = static_cast<unsigned char *>(workspace);

    hipError_t e = stage_words(pl.blob, reinterpret_cast<uint64_t *>(ws + w.blob), s);
    if (e != hipSuccess) return hip_fail(e);

    SweepArgs a;
    a.X = X;
    a.xbytes = xbytes;
    a.ld = ld;
    a.d = d;
    a.T = T;
    a.n_k = n_k;
    a.Ksum = pl.Ksum;
    a.kmax = pl.kmax;
    a.n_iter = n_iter;
    a.init_mode = init_mode;
    a.flags = flags;
    a.task_off = reinterpret_cast<const int64_t *>(ws + w.blob + pl.off_task);
    a.ks = reinterpret_cast<const int *>(ws + w.blob + pl.off_ks);
    a.koff = reinterpret_cast<const int *>(ws + w.blob + pl.off_koff);
    a.init_centroids = init_centroids;
    a.init_rows = reinterpret_cast<const int *>(ws + w.init_rows);
    a.ndist = reinterpret_cast<const int *>(ws + w.ndist);
    a.centroids = centroids;
    a.counts = counts;
    a.inertia = inertia;
    a.status = status;
    a.labbuf = labels ? labels : ws + w.labbuf;
    a.trace = inertia_trace;
    a.xh = reinterpret_cast<uint16_t *>(ws + w.xh);
    a.passes = reinterpret_cast<int *>(ws + w.passes);
    a.queue_lds_off = 0;
    a.too_large = (xbytes == 2 && path == SweepPath::kMfmaResident) ? reinterpret_cast<int *>(ws + w.counters) + n_k : nullptr;
    a.ki_begin = 0;
    a.ki_end = n_k;
    a.done = nullptr;
    int *done = chunked ? reinterpret_cast<int *>(ws + w.total) : nullptr;
    if (chunked) {
        e = launch_fill_i32(done, T, 0, s);
        if (e != hipSuccess) return hip_fail(e);
    }

    // labelling passes per (task, k): n_iter + 1 unless the kernel records that it stopped earlier
    e = launch_fill_i32(a.passes, (int64_t)T * n_k, n_iter + 1, s);
    if (e != hipSuccess) return hip_fail(e);
    // work counters of the launches (the matrix-core resident kernel hands out its units through one)
    e = launch_fill_i32(reinterpret_cast<int *>(ws + w.counters), n_k + 1, 0, s);
    if (e != hipSuccess) return hip_fail(e);
    if (init_mode == 0) {
        e = launch_first_distinct(a, reinterpret_cast<int *>(ws + w.init_rows),
                                  reinterpret_cast<int *>(ws + w.ndist), s);
        if (e != hipSuccess) return hip_fail(e);
    }
    const int step = chunked ? chunk : n_k;
    for (int ki_begin = 0; ki_begin < n_k; ki_begin += step) {
        const int ki_end = ki_begin + step < n_k ? ki_begin + step : n_k;
        a.ki_begin = ki_begin;
        a.ki_end = ki_end;
        a.unit_counter = reinterpret_cast<int *>(ws + w.counters) + ki_begin;
        a.done = ki_begin > 0 ? done : nullptr;
        if (path == SweepPath::kStream) {
            // first workgroup of every unit, in launch order (largest k first)
            const int n_units = (ki_end - ki_begin) * T;        // units of this chunk, largest k first
            Words wo;
            if (no_heap) wo.forbid_heap();
            if (!wo.assign(((size_t)n_units + 2) / 2)) return CHAM_E_NOMEM;
            int32_t *po = reinterpret_cast<int32_t *>(wo.data());
            int acc = 0;
            for (int u = 0; u < n_units; ++u) {
                const int t = u % T;
                const int rpw = stream_rows_per_wg(ks[ki_end - 1 - u / T]);
                po[u] = acc;
                acc += (int)((task_off[t + 1] - task_off[t] + rpw - 1) / rpw);
            }
            po[n_units] = acc;
            e = stage_words(wo, reinterpret_cast<uint64_t *>(ws + w.wg_off), s);
            if (e != hipSuccess) return hip_fail(e);
            StreamArgs sa;
            sa.X = X;
            sa.ld = ld;
            sa.d = d;
            sa.T = T;
            sa.n_k = n_k;
            sa.Ksum = pl.Ksum;
            sa.kmax = pl.kmax;
            sa.kpm = w.kpm;
            sa.n_iter = n_iter;
            sa.init_mode = init_mode;
            sa.n_units = n_units;
            sa.u_begin = (n_k - ki_end) * T;
            sa.prepare = ki_begin == 0 ? 1 : 0;
            sa.done = a.done;
            sa.it = 0;
            sa.final_pass = 0;
            sa.task_off = a.task_off;
            sa.ks = a.ks;
            sa.koff = a.koff;
            sa.init_centroids = init_centroids;
            sa.init_rows = a.init_rows;
            sa.ndist = a.ndist;
            sa.wg_off = reinterpret_cast<const int *>(ws + w.wg_off);
            sa.centroids = centroids;
            sa.counts = counts;
            sa.inertia = inertia;
            sa.status = status;
            sa.labbuf = a.labbuf;
            sa.trace = inertia_trace;
            sa.xh = a.xh;
            sa.x2 = reinterpret_cast<float *>(ws + w.x2);
            sa.ojf = reinterpret_cast<float *>(ws + w.ojf);
            sa.Sg = reinterpret_cast<int *>(ws + w.Sg);
            sa.ng = reinterpret_cast<int *>(ws + w.ng);
            sa.mu = reinterpret_cast<double *>(ws + w.mu);
            sa.afrag = ws + w.afrag;
            sa.biasf = reinterpret_cast<float *>(ws + w.biasf);
            sa.m2 = reinterpret_cast<float *>(ws + w.m2);
            sa.loss_part = reinterpret_cast<double *>(ws + w.loss);
            sa.passes = a.passes;
            if (stream_lds_bytes(d, w.kpm) > 160 * 1024) return CHAM_E_BAD_K;
            e = acc > 0 ? launch_stream_sweep(sa, pl.n_total, acc, s) : hipSuccess;
            if (acc == 0) e = launch_resident_sweep(a, pl.nt, s);   // all tasks empty: trivial path
        } else if (path == SweepPath::kMfmaResident) {
            e = launch_mfma_sweep(a, pl.n_max, pl.n_total, s);
        } else {
            e = launch_resident_sweep(a, pl.nt, s);
        }
        if (e != hipSuccess) return hip_fail(e);
        if (chunked && ki_end < n_k) {
            e = launch_knee_update(inertia, status, T, n_k, ki_end, threshold, done, s);
            if (e != hipSuccess) return hip_fail(e);
        }
    }
    if (chunked) {
        e = launch_select_k(inertia, status, T, n_k, threshold, chosen_idx, s);
        if (e != hipSuccess) return hip_fail(e);
    }
    return CHAM_OK;
}

int32_t cham_kmeans_sweep(const uint8_t *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                          const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t init_mode,
                          const double *init_centroids, double *centroids, int32_t *counts,
                          double *inertia, int32_t *status, uint8_t *labels, double *inertia_trace,
                          void *workspace, int64_t workspace_bytes, int32_t flags, void *stream)
{
    return sweep_impl(X, 1, ld, d, task_off, T, ks, n_k, n_iter, init_mode, init_centroids, centroids, counts, inertia,
                      status, labels, inertia_trace, workspace, workspace_bytes, flags, stream, 0, 0.0, nullptr);
}

// Scratch memory of cham_kmeans_sweep_static, the entry point for callers that cannot allocate:
// one array per GPU, inside the loaded code object, kept until the process ends.  The name below
// is only a host-side handle of the symbol; the array's device address is looked up once per
// device and every use in host code goes through that address.
constexpr int64_t kStaticScratchBytes = (int64_t)CHAM_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
static void *g_scratch_addr[kMaxDevices];       // device address of `scratch` on each GPU, null until looked up

static int32_t static_scratch_address(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e);
    if (dev < 0 || dev >= kMaxDevices) return CHAM_E_BAD_DIM;
    void *p = __atomic_load_n(&g_scratch_addr[dev], __ATOMIC_ACQUIRE);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_fail(e);
        if (!p) return hip_fail(hipErrorInvalidSymbol);
        __atomic_store_n(&g_scratch_addr[dev], p, __ATOMIC_RELEASE);
    }
    *out = p;
    return CHAM_OK;
}

int32_t cham_static_init(void)
{
    void *p = nullptr;
    return static_scratch_address(&p);
}

int32_t cham_kmeans_sweep_static(const uint8_t *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                 const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t init_mode,
                                 const double *init_centroids, double *centroids, int32_t *counts,
                                 double *inertia, int32_t *status, uint8_t *labels, double *inertia_trace,
                                 int32_t flags, void *stream)
{
    // argument errors come out of the size query exactly as they would out of the sweep
    const int64_t need = sweep_ws_bytes(1, ld, d, task_off, T, ks, n_k, flags, true);
    if (need == CHAM_E_NOMEM) return CHAM_E_TOO_LARGE;      // tables beyond the part kept on the stack
    if (need < 0) return (int32_t)need;
    if (flags & ~kSweepFlags) return CHAM_E_BAD_FLAG;
    if (need > kStaticScratchBytes) return CHAM_E_TOO_LARGE;
    void *ws = nullptr;
    int32_t rc = static_scratch_address(&ws);
    if (rc != CHAM_OK) return rc;
    rc = sweep_impl(X, 1, ld, d, task_off, T, ks, n_k, n_iter, init_mode, init_centroids, centroids, counts, inertia,
                    status, labels, inertia_trace, ws, kStaticScratchBytes, flags, stream, 0, 0.0, nullptr, true);
    // the host-side tables of this entry point live on the stack only
    return rc == CHAM_E_NOMEM ? CHAM_E_TOO_LARGE : rc;
}

int32_t cham_kmeans_sweep_u16(const uint16_t *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                              const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t init_mode,
                              const double *init_centroids, double *centroids, int32_t *counts,
                              double *inertia, int32_t *status, uint8_t *labels, double *inertia_trace,
                              void *workspace, int64_t workspace_bytes, int32_t flags, void *stream)
{
    return sweep_impl(X, 2, ld, d, task_off, T, ks, n_k, n_iter, init_mode, init_centroids, centroids, counts, inertia,
                      status, labels, inertia_trace, workspace, workspace_bytes, flags, stream, 0, 0.0, nullptr);
}

static int32_t sweep_path_impl(int xbytes, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                              const int32_t *ks, int32_t n_k, int32_t flags)
{
    Plan pl;
    const int32_t rc = check_common(nullptr, ld, d, task_off, T, ks, n_k, false, pl, xbytes);
    if (rc != CHAM_OK) return rc;
    if (flags & ~kSweepFlags) return CHAM_E_BAD_FLAG;
    if (xbytes == 2 && (flags & CHAM_F_STREAMING)) return CHAM_E_BAD_FLAG;
    switch (choose_path(pl, d, flags, xbytes)) {
    case SweepPath::kMfmaResident: return CHAM_PATH_RESIDENT_MFMA;
    case SweepPath::kStream: return CHAM_PATH_STREAM_MFMA;
    default: return (xbytes == 2 && !u16_fits(pl)) ? CHAM_E_BAD_K : CHAM_PATH_RESIDENT_VECTOR;
    }
}

int32_t cham_sweep_path(int64_t ld, int32_t d, const int64_t *task_off, int32_t T, const int32_t *ks, int32_t n_k,
                        int32_t flags)
{
    return sweep_path_impl(1, ld, d, task_off, T, ks, n_k, flags);
}

int32_t cham_sweep_path_u16(int64_t ld, int32_t d, const int64_t *task_off, int32_t T, const int32_t *ks,
                            int32_t n_k, int32_t flags)
{
    return sweep_path_impl(2, ld, d, task_off, T, ks, n_k, flags);
}

const char *cham_sweep_path_kernel(int32_t path)
{
    switch (path) {
    case CHAM_PATH_RESIDENT_MFMA: return "resident_mfma_kernel";
    case CHAM_PATH_STREAM_MFMA: return "stream_assign_kernel";
    case CHAM_PATH_RESIDENT_VECTOR: return "resident_sweep_kernel";
    default: return "unknown";
    }
}

int32_t cham_sweep_passes(const void *workspace, int64_t workspace_bytes, int64_t ld, int32_t d,
                          const int64_t *task_off, int32_t T, const int32_t *ks, int32_t n_k, int32_t flags,
                          int32_t *passes, void *stream)
{
    Plan pl;
    const int32_t rc = check_common(nullptr, ld, d, task_off, T, ks, n_k, false, pl, d > 32 ? 2 : 1);
    if (rc != CHAM_OK) return rc;
    if (!passes) return CHAM_E_NULL;
    // the region sits before every part of the workspace whose size depends on the path or the knob width
    const SweepWs w = sweep_ws(pl, ld, false, false, task_off, 0);
    if (!workspace || workspace_bytes < w.passes + (int64_t)T * n_k * 4) return CHAM_E_WORKSPACE;
    (void)flags;
    hipError_t e = hipMemcpyAsync(passes, static_cast<const unsigned char *>(workspace) + w.passes,
                                  (size_t)T * n_k * 4, hipMemcpyDeviceToDevice, reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return CHAM_OK;
}

int64_t cham_sweep_knee_workspace_bytes(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                        const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t flags)
{
    const int64_t base = cham_sweep_workspace_bytes(ld, d, task_off, T, ks, n_k, n_iter, flags);
    if (base < 0) return base;
    return base + up((int64_t)T * 4);
}

int32_t cham_kmeans_sweep_knee(const uint8_t *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                               const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t init_mode,
                               const double *init_centroids, double threshold, int32_t chunk,
                               double *centroids, int32_t *counts, double *inertia, int32_t *status,
                               int32_t *chosen_idx, uint8_t *labels, double *inertia_trace,
                               void *workspace, int64_t workspace_bytes, int32_t flags, void *stream)
{
    if (!chosen_idx) return CHAM_E_NULL;
    if (chunk < 1) return CHAM_E_BAD_K;
    if (chunk > n_k) chunk = n_k;
    return sweep_impl(X, 1, ld, d, task_off, T, ks, n_k, n_iter, init_mode, init_centroids, centroids, counts, inertia,
                      status, labels, inertia_trace, workspace, workspace_bytes, flags, stream, chunk, threshold,
                      chosen_idx);
}

int64_t cham_sweep_knee_workspace_bytes_u16(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                            const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t flags)
{
    const int64_t base = cham_sweep_workspace_bytes_u16(ld, d, task_off, T, ks, n_k, n_iter, flags);
    if (base < 0) return base;
    return base + up((int64_t)T * 4);
}

int32_t cham_kmeans_sweep_knee_u16(const uint16_t *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                   const int32_t *ks, int32_t n_k, int32_t n_iter, int32_t init_mode,
                                   const double *init_centroids, double threshold, int32_t chunk,
                                   double *centroids, int32_t *counts, double *inertia, int32_t *status,
                                   int32_t *chosen_idx, uint8_t *labels, double *inertia_trace,
                                   void *workspace, int64_t workspace_bytes, int32_t flags, void *stream)
{
    if (!chosen_idx) return CHAM_E_NULL;
    if (chunk < 1) return CHAM_E_BAD_K;
    if (chunk > n_k) chunk = n_k;
    return sweep_impl(X, 2, ld, d, task_off, T, ks, n_k, n_iter, init_mode, init_centroids, centroids, counts, inertia,
                      status, labels, inertia_trace, workspace, workspace_bytes, flags, stream, chunk, threshold,
                      chosen_idx);
}

int32_t cham_select_k_host(const double *curve, const int32_t *status, int32_t n_k, double threshold)
{
    if (!curve || n_k < 1) return -1;
    bool have_prev = false;
    double prev = 0.0;
    int32_t last = -1;
    for (int32_t i = 0; i < n_k; ++i) {
        if (status && status[i] != 0) continue;
        if (have_prev && threshold * curve[i] >= prev) return i;
        prev = curve[i];
        have_prev = true;
        last = i;
    }
    return last;
}

int32_t cham_select_k(const double *inertia, const int32_t *status, int32_t T, int32_t n_k,
                      double threshold, int32_t *chosen_idx, void *stream)
{
    if (!inertia || !status || !chosen_idx) return CHAM_E_NULL;
    if (T < 1) return CHAM_E_BAD_DIM;
    if (n_k < 1 || n_k > 256) return CHAM_E_BAD_K;
    hipError_t e = launch_select_k(inertia, status, T, n_k, threshold, chosen_idx,
                                   reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return CHAM_OK;
}

// Tasks above this many rows are split over 4096-row chunks in the snap and synthesis steps.
constexpr int64_t kWideTaskRows = 16384;
constexpr int64_t kWideChunkRows = 4096;

static bool wide_tasks(const Plan &pl) { return pl.n_max > kWideTaskRows; }

// first workgroup of every task when each task is cut into 4096-row chunks; returns the total
static int wide_offsets(const int64_t *task_off, int T, Words &words)
{
    if (!words.assign((size_t)(T + 2) / 2 + 1)) return -1;
    int *w = reinterpret_cast<int *>(words.data());
    int acc = 0;
    for (int t = 0; t < T; ++t) {
        w[t] = acc;
        acc += (int)((task_off[t + 1] - task_off[t] + kWideChunkRows - 1) / kWideChunkRows);
    }
    w[T] = acc;
    return acc;
}

static int64_t wide_snap_bytes(const Plan &pl)
{
    if (!wide_tasks(pl)) return 0;
    return up((int64_t)(pl.T + 4) * 4) + up((int64_t)pl.T * pl.kmax * 8) + up((int64_t)pl.T * pl.kmax * 4);
}

static int64_t wide_synth_bytes(const Plan &pl, int d)
{
    if (!wide_tasks(pl)) return 0;
    return up((int64_t)(pl.T + 4) * 4) + 2 * up((int64_t)pl.T * pl.kmax * 4) + up((int64_t)pl.T * 4) +
           up((int64_t)pl.T * pl.kmax * d * 256 * 4);
}

static int64_t snap_ws_bytes(int xbytes, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                             const int32_t *ks, int32_t n_k)
{
    Plan pl;
    const int32_t rc = check_common(nullptr, ld, d, task_off, T, ks, n_k, false, pl, xbytes);
    if (rc != CHAM_OK) return rc;
    return up((int64_t)pl.blob.size() * 8) + up(ld * 8) + (xbytes == 1 ? wide_snap_bytes(pl) : 0);
}

int64_t cham_snap_workspace_bytes(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                  const int32_t *ks, int32_t n_k)
{
    return snap_ws_bytes(1, ld, d, task_off, T, ks, n_k);
}

int64_t cham_snap_workspace_bytes_u16(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                      const int32_t *ks, int32_t n_k)
{
    return snap_ws_bytes(2, ld, d, task_off, T, ks, n_k);
}

static int32_t snap_impl(const void *Xv, int xbytes, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                         const int32_t *ks, int32_t n_k, const int32_t *chosen_idx,
                         const double *centroids, uint8_t *labels_sel, int32_t *pick_row,
                         void *pick_cfg, void *workspace, int64_t workspace_bytes, int32_t flags,
                         void *stream)
{
    const uint8_t *X = static_cast<const uint8_t *>(Xv);
    Plan pl;
    int32_t rc = check_common(X, ld, d, task_off, T, ks, n_k, true, pl, xbytes);
    if (rc != CHAM_OK) return rc;
    if (!chosen_idx || !centroids || !labels_sel || !pick_row || !pick_cfg) return CHAM_E_NULL;
    if (flags & ~kSweepFlags) return CHAM_E_BAD_FLAG;
    if (xbytes == 2 && resident_lds_bytes(pl.DP, pl.kmax) > 160 * 1024) return CHAM_E_BAD_K;
    const bool wide = xbytes == 1 && wide_tasks(pl);
    const int64_t blob_bytes = up((int64_t)pl.blob.size() * 8);
    if (!workspace || workspace_bytes < blob_bytes + up(ld * 8) + (wide ? wide_snap_bytes(pl) : 0)) return CHAM_E_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return CHAM_E_WORKSPACE;
    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    hipError_t e = stage_words(pl.blob, reinterpret_cast<uint64_t *>(ws), s);
    if (e != hipSuccess) return hip_fail(e);
    SnapArgs a;
    a.X = X;
    a.xbytes = xbytes;
    a.ld = ld;
    a.d = d;
    a.T = T;
    a.n_k = n_k;
    a.Ksum = pl.Ksum;
    a.kmax = pl.kmax;
    a.flags = flags;
    a.task_off = reinterpret_cast<const int64_t *>(ws + pl.off_task);
    a.ks = reinterpret_cast<const int *>(ws + pl.off_ks);
    a.koff = reinterpret_cast<const int *>(ws + pl.off_koff);
    a.chosen = chosen_idx;
    a.centroids = centroids;
    a.labels_sel = labels_sel;
    a.pick_row = pick_row;
    a.pick_cfg = static_cast<uint8_t *>(pick_cfg);
    a.dist_ws = reinterpret_cast<double *>(ws + blob_bytes);
    a.wg_off = nullptr;
    a.wide_best = nullptr;
    a.wide_row = nullptr;
    if (wide) {
        unsigned char *p = ws + blob_bytes + up(ld * 8);
        Words wo;
        const int total = wide_offsets(task_off, T, wo);
        if (total < 0) return CHAM_E_NOMEM;
        e = stage_words(wo, reinterpret_cast<uint64_t *>(p), s);
        if (e != hipSuccess) return hip_fail(e);
        a.wg_off = reinterpret_cast<const int *>(p);
        p += up((int64_t)(T + 4) * 4);
        a.wide_best = reinterpret_cast<unsigned long long *>(p);
        p += up((int64_t)T * pl.kmax * 8);
        a.wide_row = reinterpret_cast<int *>(p);
        e = launch_snap_wide(a, total, s);
    } else {
        e = launch_snap(a, pl.nt, s);
    }
    if (e != hipSuccess) return hip_fail(e);
    return CHAM_OK;
}

int32_t cham_snap_centroids(const uint8_t *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                            const int32_t *ks, int32_t n_k, const int32_t *chosen_idx,
                            const double *centroids, uint8_t *labels_sel, int32_t *pick_row,
                            uint8_t *pick_cfg, void *workspace, int64_t workspace_bytes, int32_t flags,
                            void *stream)
{
    return snap_impl(X, 1, ld, d, task_off, T, ks, n_k, chosen_idx, centroids, labels_sel, pick_row, pick_cfg,
                     workspace, workspace_bytes, flags, stream);
}

int32_t cham_snap_centroids_u16(const uint16_t *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                const int32_t *ks, int32_t n_k, const int32_t *chosen_idx,
                                const double *centroids, uint8_t *labels_sel, int32_t *pick_row,
                                uint16_t *pick_cfg, void *workspace, int64_t workspace_bytes, int32_t flags,
                                void *stream)
{
    return snap_impl(X, 2, ld, d, task_off, T, ks, n_k, chosen_idx, centroids, labels_sel, pick_row, pick_cfg,
                     workspace, workspace_bytes, flags, stream);
}

static int64_t synth_blob_extra_words(int32_t T, int32_t d)
{
    return (int64_t)T + ((int64_t)T * d + 3) / 4;      // salts (u64) + cards (u16)
}

static int64_t synth_ws_bytes(int xbytes, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                              const int32_t *ks, int32_t n_k)
{
    Plan pl;
    const int32_t rc = check_common(nullptr, ld, d, task_off, T, ks, n_k, false, pl, xbytes);
    if (rc != CHAM_OK) return rc;
    return up(((int64_t)pl.blob.size() + synth_blob_extra_words(T, d)) * 8) + (xbytes == 1 ? wide_synth_bytes(pl, d) : 0);
}

int64_t cham_synth_workspace_bytes(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                   const int32_t *ks, int32_t n_k)
{
    return synth_ws_bytes(1, ld, d, task_off, T, ks, n_k);
}

int64_t cham_synth_workspace_bytes_u16(int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                       const int32_t *ks, int32_t n_k)
{
    return synth_ws_bytes(2, ld, d, task_off, T, ks, n_k);
}

// Largest cardinality of a two-byte knob: the value histogram of one knob has to fit in LDS.
constexpr int kMaxCard16 = 16384;

// n_visited >= 0: sorted array of that many hashes; n_visited < 0: table of -n_visited slots.
static int32_t synth_impl(const void *Xv, int xbytes, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                          const uint16_t *cards, const uint8_t *valid, const int32_t *ks, int32_t n_k,
                          const int32_t *chosen_idx, const uint8_t *labels_sel, const int32_t *pick_row,
                          const void *pick_cfg, const uint64_t *visited, int64_t n_visited,
                          const uint64_t *task_salt, void *out_cfg, uint8_t *out_flag,
                          int32_t *out_count, void *workspace, int64_t workspace_bytes, void *stream)
{
    const uint8_t *X = static_cast<const uint8_t *>(Xv);
    Plan pl;
    int32_t rc = check_common(X, ld, d, task_off, T, ks, n_k, true, pl, xbytes);
    if (rc != CHAM_OK) return rc;
    if (!cards || !chosen_idx || !labels_sel || !pick_row || !pick_cfg || !out_cfg || !out_flag || !out_count)
        return CHAM_E_NULL;
    if (n_visited != 0 && !visited) return CHAM_E_NULL;
    int cmax = 1;
    for (int64_t i = 0; i < (int64_t)T * d; ++i) {
        if (cards[i] < 1 || cards[i] > (xbytes == 1 ? 256 : kMaxCard16)) return CHAM_E_CARD;
        if (cards[i] > cmax) cmax = cards[i];
    }
    const int64_t base_words = (int64_t)pl.blob.size();
    const int64_t need = up((base_words + synth_blob_extra_words(T, d)) * 8);
    const bool wide = xbytes == 1 && wide_tasks(pl);
    if (!workspace || workspace_bytes < need + (wide ? wide_synth_bytes(pl, d) : 0)) return CHAM_E_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return CHAM_E_WORKSPACE;
    // extend the blob: salts then cards
    if (!pl.blob.resize((size_t)(base_words + synth_blob_extra_words(T, d)))) return CHAM_E_NOMEM;
    for (int t = 0; t < T; ++t) pl.blob[(size_t)base_words + t] = task_salt ? task_salt[t] : (uint64_t)t;
    uint16_t *pc = reinterpret_cast<uint16_t *>(pl.blob.data() + base_words + T);
    for (int64_t i = 0; i < (int64_t)T * d; ++i) pc[i] = cards[i];

    hipStream_t s = reinterpret_cast<hipStream_t>(stream);
    unsigned char *ws = static_cast<unsigned char *>(workspace);
    hipError_t e = stage_words(pl.blob, reinterpret_cast<uint64_t *>(ws), s);
    if (e != hipSuccess) return hip_fail(e);

    SynthArgs a;
    a.X = X;
    a.xbytes = xbytes;
    a.ld = ld;
    a.d = d;
    a.T = T;
    a.n_k = n_k;
    a.kmax = pl.kmax;
    // LDS histogram: room for every cluster if that fits in 96 KiB and beside the kernel's other
    // arrays; byte knobs: never less than one cluster (all knobs, which always fits); two-byte
    // knobs: never less than one knob of one cluster
    int64_t words = (int64_t)pl.kmax * d * cmax;
    if (words > 24576) words = 24576;
    const int64_t avail = (160 * 1024 - (int64_t)synth_lds_bytes(d, pl.kmax, 0, xbytes)) / 4;
    if (words > avail) words = avail;
    if (xbytes == 1 && words < (int64_t)d * cmax) words = (int64_t)d * cmax;
    if (words < cmax) return CHAM_E_CARD;
    a.hist_words = (int)words;
    a.task_off = reinterpret_cast<const int64_t *>(ws + pl.off_task);
    a.ks = reinterpret_cast<const int *>(ws + pl.off_ks);
    a.salts = reinterpret_cast<const uint64_t *>(ws + base_words * 8);
    a.cards = reinterpret_cast<const uint16_t *>(ws + (base_words + T) * 8);
    a.valid = valid;
    a.chosen = chosen_idx;
    a.labels_sel = labels_sel;
    a.pick_row = pick_row;
    a.pick_cfg = static_cast<const uint8_t *>(pick_cfg);
    a.visited = visited;
    a.n_visited = n_visited;
    a.out_cfg = static_cast<uint8_t *>(out_cfg);
    a.out_flag = out_flag;
    a.out_count = out_count;
    a.wg_off = nullptr;
    a.wide_cmax = cmax;
    a.wide_slot = a.wide_list = a.wide_nf = nullptr;
    a.wide_hist = nullptr;
    if (wide) {
        unsigned char *p = ws + need;
        Words wo;
        const int total = wide_offsets(task_off, T, wo);
        if (total < 0) return CHAM_E_NOMEM;
        e = stage_words(wo, reinterpret_cast<uint64_t *>(p), s);
        if (e != hipSuccess) return hip_fail(e);
        a.wg_off = reinterpret_cast<const int *>(p);
        p += up((int64_t)(T + 4) * 4);
        a.wide_slot = reinterpret_cast<int *>(p);
        p += up((int64_t)T * pl.kmax * 4);
        a.wide_list = reinterpret_cast<int *>(p);
        p += up((int64_t)T * pl.kmax * 4);
        a.wide_nf = reinterpret_cast<int *>(p);
        p += up((int64_t)T * 4);
        a.wide_hist = reinterpret_cast<unsigned *>(p);
        e = launch_synth_wide(a, total, s);
    } else {
        int nt = pl.nt < 256 ? 256 : pl.nt;
        if (nt > 1024) nt = 1024;
        e = launch_synth(a, nt, s);
    }
    if (e != hipSuccess) return hip_fail(e);
    return CHAM_OK;
}

int32_t cham_synthesize(const uint8_t *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                        const uint16_t *cards, const uint8_t *valid, const int32_t *ks, int32_t n_k,
                        const int32_t *chosen_idx, const uint8_t *labels_sel, const int32_t *pick_row,
                        const uint8_t *pick_cfg, const uint64_t *visited, int64_t n_visited,
                        const uint64_t *task_salt, uint8_t *out_cfg, uint8_t *out_flag,
                        int32_t *out_count, void *workspace, int64_t workspace_bytes, void *stream)
{
    if (n_visited < 0) return CHAM_E_NULL;
    return synth_impl(X, 1, ld, d, task_off, T, cards, valid, ks, n_k, chosen_idx, labels_sel, pick_row, pick_cfg,
                      visited, n_visited, task_salt, out_cfg, out_flag, out_count, workspace, workspace_bytes, stream);
}

static bool table_ok(const void *table, int64_t slots)
{
    return table && slots >= 2 && (slots & (slots - 1)) == 0 && reinterpret_cast<uintptr_t>(table) % 8 == 0;
}

int32_t cham_synthesize_table(const uint8_t *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                              const uint16_t *cards, const uint8_t *valid, const int32_t *ks, int32_t n_k,
                              const int32_t *chosen_idx, const uint8_t *labels_sel, const int32_t *pick_row,
                              const uint8_t *pick_cfg, const uint64_t *table, int64_t slots,
                              const uint64_t *task_salt, uint8_t *out_cfg, uint8_t *out_flag,
                              int32_t *out_count, void *workspace, int64_t workspace_bytes, void *stream)
{
    if (!table_ok(table, slots)) return table ? CHAM_E_BAD_DIM : CHAM_E_NULL;
    return synth_impl(X, 1, ld, d, task_off, T, cards, valid, ks, n_k, chosen_idx, labels_sel, pick_row, pick_cfg,
                      table, -slots, task_salt, out_cfg, out_flag, out_count, workspace, workspace_bytes, stream);
}

int32_t cham_synthesize_u16(const uint16_t *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                            const uint16_t *cards, const uint8_t *valid, const int32_t *ks, int32_t n_k,
                            const int32_t *chosen_idx, const uint8_t *labels_sel, const int32_t *pick_row,
                            const uint16_t *pick_cfg, const uint64_t *visited, int64_t n_visited,
                            const uint64_t *task_salt, uint16_t *out_cfg, uint8_t *out_flag,
                            int32_t *out_count, void *workspace, int64_t workspace_bytes, void *stream)
{
    if (n_visited < 0) return CHAM_E_NULL;
    return synth_impl(X, 2, ld, d, task_off, T, cards, valid, ks, n_k, chosen_idx, labels_sel, pick_row, pick_cfg,
                      visited, n_visited, task_salt, out_cfg, out_flag, out_count, workspace, workspace_bytes, stream);
}

int32_t cham_synthesize_table_u16(const uint16_t *X, int64_t ld, int32_t d, const int64_t *task_off, int32_t T,
                                  const uint16_t *cards, const uint8_t *valid, const int32_t *ks, int32_t n_k,
                                  const int32_t *chosen_idx, const uint8_t *labels_sel, const int32_t *pick_row,
                                  const uint16_t *pick_cfg, const uint64_t *table, int64_t slots,
                                  const uint64_t *task_salt, uint16_t *out_cfg, uint8_t *out_flag,
                                  int32_t *out_count, void *workspace, int64_t workspace_bytes, void *stream)
{
    if (!table_ok(table, slots)) return table ? CHAM_E_BAD_DIM : CHAM_E_NULL;
    return synth_impl(X, 2, ld, d, task_off, T, cards, valid, ks, n_k, chosen_idx, labels_sel, pick_row, pick_cfg,
                      table, -slots, task_salt, out_cfg, out_flag, out_count, workspace, workspace_bytes, stream);
}

int32_t cham_visited_table_clear(uint64_t *table, int64_t slots, void *stream)
{
    if (!table_ok(table, slots)) return table ? CHAM_E_BAD_DIM : CHAM_E_NULL;
    hipError_t e = launch_table_clear(table, slots, reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHAM_OK : hip_fail(e);
}

int32_t cham_visited_table_insert_hashes(uint64_t *table, int64_t slots, const uint64_t *hashes, int64_t n,
                                         int32_t *overflow, void *stream)
{
    if (!table_ok(table, slots)) return table ? CHAM_E_BAD_DIM : CHAM_E_NULL;
    if (n < 0) return CHAM_E_BAD_DIM;
    if (n > 0 && !hashes) return CHAM_E_NULL;
    hipError_t e = launch_table_insert_hashes(table, slots, hashes, n, overflow, reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHAM_OK : hip_fail(e);
}

int32_t cham_visited_table_insert_configs(uint64_t *table, int64_t slots, const uint8_t *cfgs, int64_t n, int32_t d,
                                          const uint8_t *flags, const uint64_t *salts, int64_t rows_per_salt,
                                          int32_t *overflow, void *stream)
{
    if (!table_ok(table, slots)) return table ? CHAM_E_BAD_DIM : CHAM_E_NULL;
    if (n < 0 || d < 1 || d > 32 || rows_per_salt < 1) return CHAM_E_BAD_DIM;
    if (n > 0 && !cfgs) return CHAM_E_NULL;
    hipError_t e = launch_table_insert_configs(table, slots, cfgs, 1, n, d, flags, salts, rows_per_salt, overflow,
                                               reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHAM_OK : hip_fail(e);
}

int32_t cham_visited_table_insert_configs_u16(uint64_t *table, int64_t slots, const uint16_t *cfgs, int64_t n,
                                              int32_t d, const uint8_t *flags, const uint64_t *salts,
                                              int64_t rows_per_salt, int32_t *overflow, void *stream)
{
    if (!table_ok(table, slots)) return table ? CHAM_E_BAD_DIM : CHAM_E_NULL;
    if (n < 0 || d < 1 || d > 64 || rows_per_salt < 1) return CHAM_E_BAD_DIM;
    if (n > 0 && !cfgs) return CHAM_E_NULL;
    hipError_t e = launch_table_insert_configs(table, slots, cfgs, 2, n, d, flags, salts, rows_per_salt, overflow,
                                               reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHAM_OK : hip_fail(e);
}

int32_t cham_update_configs(uint8_t *theta, const int8_t *actions, int64_t B, int32_t d, int32_t n_steps,
                            const uint16_t *cards, uint64_t salt, uint64_t *seen_table, int64_t slots,
                            uint8_t *unique_rows, int64_t capacity, int32_t *n_unique, int32_t *overflow,
                            void *stream)
{
    if (!theta || !actions || !cards) return CHAM_E_NULL;
    if (B < 0 || d < 1 || d > 32 || n_steps < 0) return CHAM_E_BAD_DIM;
    if (seen_table) {
        if (!table_ok(seen_table, slots)) return CHAM_E_BAD_DIM;
        if (!unique_rows || !n_unique || capacity < 0) return CHAM_E_NULL;
    }
    hipError_t e = launch_update_configs(theta, actions, B, d, n_steps, cards, salt, seen_table, slots, unique_rows,
                                         capacity, n_unique, overflow, reinterpret_cast<hipStream_t>(stream));
    return e == hipSuccess ? CHAM_OK : hip_fail(e);
}

uint64_t cham_hash_config(const uint8_t *cfg, int32_t d, uint64_t salt)
{
    uint64_t h = 0xCBF29CE484222325ULL ^ (salt * 0x9E3779B97F4A7C15ULL);
    if (!cfg) return h;
    for (int32_t j = 0; j < d; ++j) h = (h ^ (uint64_t)cfg[j]) * 0x100000001B3ULL;
    return h;
}

int32_t cham_hash_rows(const uint8_t *rows, int64_t n, int32_t d, const uint64_t *salts,
                       uint64_t salt_all, uint64_t *out, void *stream)
{
    if (n < 0 || d < 0) return CHAM_E_BAD_DIM;
    if (n == 0) return CHAM_OK;
    if (!rows || !out) return CHAM_E_NULL;
    hipError_t e = launch_hash_rows(rows, 1, n, d, salts, salt_all, out, reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return CHAM_OK;
}

uint64_t cham_hash_config_u16(const uint16_t *cfg, int32_t d, uint64_t salt)
{
    uint64_t h = 0xCBF29CE484222325ULL ^ (salt * 0x9E3779B97F4A7C15ULL);
    if (!cfg) return h;
    for (int32_t j = 0; j < d; ++j) h = (h ^ (uint64_t)cfg[j]) * 0x100000001B3ULL;
    return h;
}

int32_t cham_hash_rows_u16(const uint16_t *rows, int64_t n, int32_t d, const uint64_t *salts,
                           uint64_t salt_all, uint64_t *out, void *stream)
{
    if (n < 0 || d < 0) return CHAM_E_BAD_DIM;
    if (n == 0) return CHAM_OK;
    if (!rows || !out) return CHAM_E_NULL;
    hipError_t e = launch_hash_rows(rows, 2, n, d, salts, salt_all, out, reinterpret_cast<hipStream_t>(stream));
    if (e != hipSuccess) return hip_fail(e);
    return CHAM_OK;
}

}  // extern "C"
