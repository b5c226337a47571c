// Host/device shared declarations internal to libcham (not part of the public ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cham {

// Arguments of the sweep kernels.  Pointers are device pointers.
struct SweepArgs {
    const uint8_t *X;              // knob values, [d][ld] items of xbytes bytes each
    int xbytes;                    // 1: byte knobs; 2: two-byte knobs (vector resident kernel only)
    int64_t ld;
    int d;
    int T;
    int n_k;
    int Ksum;
    int kmax;
    int n_iter;
    int init_mode;
    int flags;
    const int64_t *task_off;       // [T+1]
    const int *ks;                 // [n_k]
    const int *koff;               // [n_k+1]
    const double *init_centroids;  // [T][Ksum][d] or null
    const int *init_rows;          // [T][kmax] first distinct rows (task-relative)
    const int *ndist;              // [T] how many distinct rows were found (<= kmax)
    double *centroids;             // [T][Ksum][d]
    int *counts;                   // [T][Ksum]
    double *inertia;               // [T][n_k]
    int *status;                   // [T][n_k]
    uint8_t *labbuf;               // [n_k][ld] working / final labels
    double *trace;                 // [T][n_k][n_iter+1] or null
    uint16_t *xh;                  // [ld][16 or 32] f16 row-major copy of X (matrix-core path)
    int *passes;                   // [T][n_k] labelling passes actually run (preset to n_iter + 1 by the host code)
    int *too_large;                // matrix-core kernels, two-byte knobs: set by the packing kernel when a value is 2048 or more (null: byte knobs)
    int queue_lds_off;             // vector kernel: LDS offset of the per-wave queues of moved rows, 0 = no room for them
    int *unit_counter;             // zeroed before the launch: next unit to hand out (matrix-core resident kernel)
    int ki_begin, ki_end;          // this launch runs ks[ki_begin .. ki_end) (the whole list by default)
    const int *done;               // [T] or null: tasks whose sweep has already stopped; their units are skipped (status 3)
};

// LDS bytes the resident kernel needs for padded knob count DP and largest k.
inline size_t resident_lds_bytes(int DP, int kmax, int sum_bytes = 4)
{
    size_t b = 0;
    b += sizeof(double) * (size_t)DP * kmax;          // mu64T
    b += sizeof(float) * (size_t)kmax * (DP + 4);     // wf
    b += (size_t)sum_bytes * (size_t)kmax * DP;       // S
    b += sizeof(int) * (size_t)kmax;                  // n
    b += sizeof(float) * (size_t)DP;                  // ojf
    b += sizeof(double) * 16;                         // per-wave partials
    b += 64;                                          // m2 bits and padding
    return b;
}

// Rows one workgroup of the streaming assignment kernel walks, by the unit's k.  (Measured on the
// large single-task workload: 2048 or 16384 rows for k <= 64 are both slower than 4096.)
__host__ __device__ inline int stream_rows_per_wg(int /*k*/) { return 4096; }

// Arguments of the streaming sweep kernels (tasks too large for one workgroup).
struct StreamArgs {
    const uint8_t *X;
    int64_t ld;
    int d;
    int T;
    int n_k;
    int Ksum;
    int kmax;
    int kpm;                       // kmax rounded up to a multiple of 32
    int n_iter;
    int init_mode;
    int n_units;                   // units of this launch; unit u = u_begin + local index = (ki = n_k - 1 - u / T, t = u % T)
    int u_begin;                   // first unit of this launch
    int prepare;                   // 1: this launch also computes the centring offsets and the packed rows
    const int *done;               // [T] or null: tasks whose sweep has already stopped (their units report status 3)
    int it;                        // pass being run
    int final_pass;
    const int64_t *task_off;
    const int *ks;
    const int *koff;
    const double *init_centroids;
    const int *init_rows;
    const int *ndist;
    const int *wg_off;             // [n_units + 1] first workgroup of every unit
    double *centroids;
    int *counts;
    double *inertia;
    int *status;
    uint8_t *labbuf;
    double *trace;
    uint16_t *xh;                  // [ld][16 or 32] centred f16 rows (absent knobs zero)
    float *x2;                     // [ld] squared norm of the centred rows
    float *ojf;                    // [T][32] centring offsets
    int *Sg;                       // [n_units][kpm][32] integer sums
    int *ng;                       // [n_units][kpm] counts
    double *mu;                    // [n_units][32][kpm] exact centroids, transposed
    void *afrag;                   // [n_units][kpm/32][4][64] 16-byte A fragments
    float *biasf;                  // [n_units][kpm] |mu'|^2 per centroid row (huge for padding rows)
    float *m2;                     // [n_units][8] bound on max |mu'|^2 per tile of 32 centroids; tile 0 negative = unit unusable
    double *loss_part;             // [total workgroups] loss partials of the last pass
    int *passes;                   // [T][n_k] labelling passes actually run (preset to n_iter + 1 by the host code)
};

// Arguments of the snap kernel.
struct SnapArgs {
    const uint8_t *X;           // knob values, [d][ld] items of xbytes bytes each
    int xbytes;                 // 1 or 2; pick_cfg holds items of the same size
    int64_t ld;
    int d;
    int T;
    int n_k;
    int Ksum;
    int kmax;
    int flags;
    const int64_t *task_off;
    const int *ks;
    const int *koff;
    const int *chosen;          // [T]
    const double *centroids;    // [T][Ksum][d]
    uint8_t *labels_sel;        // [ld]
    int *pick_row;              // [T][kmax]
    uint8_t *pick_cfg;          // [T][kmax][d]
    double *dist_ws;            // [ld] exact distance of every row to its centroid
    // wide variant (tasks split over row chunks)
    const int *wg_off;                  // [T+1] first workgroup of every task
    unsigned long long *wide_best;      // [T][kmax] smallest distance bits per cluster
    int *wide_row;                      // [T][kmax] lowest row attaining it
};

// Arguments of the synthesis kernel.
struct SynthArgs {
    const uint8_t *X;           // knob values, [d][ld] items of xbytes bytes each
    int xbytes;                 // 1 or 2; pick_cfg and out_cfg hold items of the same size
    int64_t ld;
    int d;
    int T;
    int n_k;
    int kmax;
    int hist_words;             // LDS words available for value histograms
    const int64_t *task_off;
    const int *ks;
    const uint16_t *cards;      // [T][d]
    const uint64_t *salts;      // [T]
    const uint8_t *valid;       // [ld] or null
    const int *chosen;          // [T]
    const uint8_t *labels_sel;  // [ld]
    const int *pick_row;        // [T][kmax]
    const uint8_t *pick_cfg;    // [T][kmax][d]
    const uint64_t *visited;    // sorted array of n_visited hashes, or (n_visited < 0) a table of -n_visited slots
    int64_t n_visited;
    uint8_t *out_cfg;           // [T][kmax][d]
    uint8_t *out_flag;          // [T][kmax]
    int *out_count;             // [T]
    // wide variant (tasks split over row chunks)
    const int *wg_off;          // [T+1] first workgroup of every task
    int wide_cmax;              // largest cardinality of the batch
    int *wide_slot;             // [T][kmax] slot of a flagged cluster, -1 otherwise
    int *wide_list;             // [T][kmax] flagged clusters in ascending order
    int *wide_nf;               // [T] how many
    unsigned *wide_hist;        // [T][kmax][d][wide_cmax] value counts of flagged clusters (by slot)
};

hipError_t launch_first_distinct(const SweepArgs &a, int *init_rows, int *ndist, hipStream_t s);
hipError_t launch_resident_sweep(const SweepArgs &a, int nt, hipStream_t s);
int resident_dp16(int d);      // padded knob count the two-byte kernels use for d knobs
// Matrix-core resident kernel: usable when every task has at most 4096 rows and k <= 64.
bool mfma_path_fits(int d, int kmax, int64_t n_max);
bool mfma_path_fits_u16(int d, int kmax, int64_t n_max);
hipError_t launch_mfma_sweep(const SweepArgs &a, int64_t n_max, int64_t n_total, hipStream_t s);
int64_t stream_lds_bytes(int d, int kpm);
hipError_t launch_stream_sweep(const StreamArgs &a, int64_t n_total, int total_wgs, hipStream_t s);
hipError_t launch_knee_update(const double *inertia, const int *status, int T, int n_k, int ki_end, double thr,
                              int *done, hipStream_t s);
hipError_t launch_fill_i32(int *dst, int64_t n, int value, hipStream_t s);
hipError_t launch_select_k(const double *inertia, const int *status, int T, int n_k, double thr,
                           int *chosen, hipStream_t s);
hipError_t launch_snap(const SnapArgs &a, int nt, hipStream_t s);
hipError_t launch_snap_wide(const SnapArgs &a, int total_wgs, hipStream_t s);
hipError_t launch_synth_wide(const SynthArgs &a, int total_wgs, hipStream_t s);
size_t synth_lds_bytes(int d, int kmax, int hist_words, int xbytes);
hipError_t launch_synth(const SynthArgs &a, int nt, hipStream_t s);
hipError_t launch_table_clear(uint64_t *v, int64_t slots, hipStream_t s);
hipError_t launch_table_insert_hashes(uint64_t *v, int64_t slots, const uint64_t *hashes, int64_t n, int *overflow,
                                      hipStream_t s);
hipError_t launch_table_insert_configs(uint64_t *v, int64_t slots, const void *cfgs, int xbytes, int64_t n, int d,
                                       const uint8_t *flags, const uint64_t *salts, int64_t rows_per_salt,
                                       int *overflow, hipStream_t s);
hipError_t launch_update_configs(uint8_t *theta, const int8_t *actions, int64_t B, int d, int n_steps,
                                 const uint16_t *cards, uint64_t salt, uint64_t *seen, int64_t slots,
                                 uint8_t *unique_rows, int64_t cap, int *n_unique, int *overflow, hipStream_t s);
hipError_t launch_hash_rows(const void *rows, int xbytes, int64_t n, int d, const uint64_t *salts,
                            uint64_t salt_all, uint64_t *out, hipStream_t s);

}  // namespace cham
