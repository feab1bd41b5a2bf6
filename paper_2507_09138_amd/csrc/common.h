// Shared declarations of the gfx950 IVF search library (internal; the public ABI is hr_ivf.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hr_ivf.h"

namespace hr {

constexpr int kWave = 64;
// internal storage code next to HR_F32 / HR_F16 / HR_BF16: float32 rows already split into a
// binary16 hi table and a 2^11-scaled binary16 lo table (the centroid table, split at load)
constexpr int HR_F16X2 = 3;
constexpr int kBlockRows = 16;             // rows per MFMA block (M of 16x16x32)
constexpr int kRowPad = 32;                // bytes of LDS padding per staged row: measured conflict-free
                                           // for the 16-rows x 16-byte MFMA fragment reads (16 is 2-way)
constexpr int kAppendMax = 16;             // most candidates one column can gain per block
constexpr int kMinSegRows = 256;           // smallest rows-per-work-item
constexpr int kItemTarget = 4096;          // aimed number of scan work items per batch
constexpr int kHistBins = 64;              // per-query histogram of candidate keys (one bin per lane)

// columns (queries) per 16-column MFMA set: 16 when the query operand is one binary16 row, 8
// when it is a (hi, lo) pair occupying two MFMA columns.
__host__ __device__ constexpr int cols_per_set(int dtype) { return dtype == HR_F16 ? 16 : 8; }

// Workgroup shapes of the scan kernel: waves x column sets per wave.  A work item covers
// shape_sets(shape) * cols_per_set(dtype) queries of a bucket.
enum { SCAN_NARROW = 0 /* 4 waves, one per SIMD */, SCAN_WIDE = 1 /* 8 waves, two per SIMD */ };
__host__ __device__ constexpr int shape_waves(int shape) { return shape == SCAN_WIDE ? 8 : 4; }
__host__ __device__ constexpr int shape_ncs(int) { return 1; }                         // column sets per wave
__host__ __device__ constexpr int shape_sets(int shape) { return shape_waves(shape) * shape_ncs(shape); }

// k-steps (of 32 elements) whose row fragments a wave fetches from LDS together
__host__ __device__ constexpr int scan_group(int dtype, int ksteps, int nw)
{
    if (ksteps < 8) return ksteps < 4 ? ksteps : 4;
    if (nw == 8 && dtype == HR_F32 && ksteps >= 24) return 2;       // (leaves registers for a second row block in flight)
    if (nw == 8) return ((dtype == HR_F32 || dtype == HR_F16X2) && ksteps >= 32) ? 2 : 4;   // (256 registers per lane)
    return 8;
}
// row blocks a wave keeps in flight in registers ahead of the one being staged: what the
// register budget (512 per lane with one wave per SIMD, 256 with two) leaves after the query
// operand, two groups of row fragments and working registers; at most 4
__host__ __device__ constexpr int scan_prefetch(int dtype, int ksteps, int ncs, int nw)
{
    const int planes = dtype == HR_F32 ? 2 : 1;
    const int rowb = ksteps * 32 * (dtype == HR_F32 ? 4 : 2);
    const int chunks = kBlockRows * rowb / 16;
    const int nld = (chunks + nw * 64 - 1) / (nw * 64);
    const int left = (nw == 8 ? 256 : 512) - ncs * ksteps * 4 - 2 * planes * scan_group(dtype, ksteps, nw) * 4 - (nw == 8 ? 67 : 96);
    const int fit = left / (nld * 4 + 1);
    return fit < 1 ? 1 : (fit > 4 ? 4 : fit);
}

// selection buffer capacity per column for a given k: room for k kept entries plus a batch of
// new ones between two prunes (a prune costs about the same for any fill up to 64 entries per
// lane slot, so bigger batches make each candidate cheaper), bounded by LDS
__host__ __device__ constexpr int sel_cap(int k)
{
    int c = k <= 24 ? 64 : (k <= 64 ? 128 : 192);
    if (c < k + kAppendMax + 4) c = k + kAppendMax + 4;
    return c;
}

// order-preserving map float -> uint32 (larger float = larger unsigned), and back
__host__ __device__ inline uint32_t enc_key(float f)
{
    uint32_t b = __builtin_bit_cast(uint32_t, f);
    return b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
}
__host__ __device__ inline float dec_key(uint32_t u)
{
    uint32_t b = (u >> 31) ? (u ^ 0x80000000u) : ~u;
    return __builtin_bit_cast(float, b);
}
constexpr uint32_t kKeyNegInf = 0x007fffffu;   // enc_key(-inf)

// One candidate: key (enc_key of the score, larger is better) and row number.
struct Cand { uint32_t key; uint32_t row; };

// Arguments of the scan kernel (both uses: centroid table with all queries as one dense
// bucket, and the inverted lists with the per-list buckets).
struct ScanArgs {
    const void* rows;           // [nrows, d] storage (HR_F16X2: the hi table)
    const void* rows_lo;        // HR_F16X2: the lo table
    const float* row_norm;      // [nrows] squared norms (used when l2 != 0)
    const int64_t* row_ids;     // [nrows] labels, or nullptr: label = row number
    const void* qop;            // query operand rows (layout depends on dtype)
    uint32_t* thr;              // [nq] running per-query lower bound of the k-th key (enc_key)
    int* slot_cnt;              // [slots]: one slot per (list segment, query of the list's bucket)
    Cand* slot_ent;             // [slots * slot_stride]
    int slot_stride;            // entries per slot: k, or cap where that is small (no cut at the end of an item)
    int* work_counter;          // zeroed before launch
    // bucket mode
    const int* list_off;        // [nlist+1] row offsets
    const int* bucket_off;      // [nlist+1]
    const int* bucket_q;        // [pairs] query index per bucket entry
    const int* dyn;             // device scalars: [0] = items, [1] = rows per segment
    const int4* xq_rec;         // [8][xq_stride][2] the items queued per XCD, each a record of two int4:
                                // (first row, rows, first entry of the list's bucket, width of the bucket),
                                // (query tile, first result slot of the item, list, segment)
    const int* xq_count;        // [8] queue lengths
    int* xq_head;               // [8] next position to pop (zeroed before launch)
    int xq_stride;
    // dense mode (dense != 0): one list = all rows, bucket = all queries
    int dense, dense_items, dense_nqt, dense_seg_rows, dense_nrows;
    int nq, k, cap, l2;
    int nbuf;                   // staging buffers in LDS (16-bit storage; float32 always uses 2)
    int gsel;                   // selection buffers = the item's slots in global memory (slot_stride = cap), none in LDS
    float* key_out;             // dense mode: [nq, dense_nrows] every key is written here and nothing is selected
    int* hist;                  // [nq][kHistBins] keys found so far per query, by key range (or nullptr)
    const float* hpar;          // [nq][2] lower edge of bin 0 and bin width (width 0: query has no histogram)
};

struct SeedArgs {
    const void* rows;           // [nrows, d] storage
    const float* row_norm;      // [nrows]
    const void* qop;            // query operand rows
    const int* probe;           // [nq, nprobe]; the first resident list among the first 64 places is the one used
    const int* list_off;        // [nlist+1]
    const int* resident;        // [nlist] 1 = the list's vectors are in place
    uint32_t* thr;              // [nq]
    float* hpar;                // [nq][2] histogram parameters of the scan (see ScanArgs)
    int nq, nprobe, nlist, k, seed_rows, l2;
};

// Device scalars written by the bucketing kernels (ints in workspace)
enum { DYN_ITEMS = 0, DYN_SEG_ROWS = 1, DYN_ROWS_LO = 2, DYN_ROWS_HI = 3, DYN_PAIRS = 4, DYN_SLOTS = 5, DYN_ROUNDS = 6, DYN_COUNT = 8 };
constexpr int kRounds = 64;                // most rounds of a work queue (see the bucketing kernels)

struct MergeArgs {
    const int* slot_cnt;
    const Cand* slot_ent;
    int slot_stride;
    const int64_t* row_ids;     // nullptr: label = row number
    const float* qnorm;         // [nq] squared norm of the query operand (L2 only)
    const int* probe;           // [nq, nprobe]
    const int* pair_entry;      // [nq, nprobe] position of the pair inside its list's bucket
    const int* list_off;        // [nlist+1]
    const int* bucket_off;      // [nlist+1]
    const int* slot_base;       // [nlist+1] first result slot of every list
    const int* dyn;
    int nq, nprobe, nlist, k, l2;
    int carried;                // out_ids / out_scores hold a previous result on entry: merged in (ids < 0: empty places)
    int64_t* out_ids;           // [nq, k] or nullptr
    float* out_scores;          // [nq, k] or nullptr
    int32_t* io_rows;           // [nq, k] or nullptr: row numbers of the entries, carried along with them (-1: empty place)
};

// launchers implemented in the .hip files
hipError_t launch_scan(int dtype, int d, const ScanArgs& a, int shape, int grid, size_t lds_bytes, hipStream_t s);
size_t scan_lds_bytes(int dtype, int d, int cap, int shape, int nbuf);
hipError_t launch_merge(const MergeArgs& a, hipStream_t s);
hipError_t launch_topk_rows(const float* keys, const float* qnorm, int32_t* out_ids, float* out_scores,
                            int64_t nq, int n, int k, int l2, hipStream_t s);
hipError_t launch_seed(int dtype, int d, const SeedArgs& a, hipStream_t s);
hipError_t launch_row_norms(const void* rows, int dtype, int64_t nrows, int d, float* out, hipStream_t s);
hipError_t launch_prep_queries(const float* q, int64_t nq, int d, int dtype, void* qop_coarse,
                               float* qnorm_coarse, void* qop_scan, float* qnorm_scan,
                               int* zero, int64_t n_zero, int* neg, int64_t n_neg, int neg_value, hipStream_t s);
hipError_t launch_fill_i32(int* p, int64_t n, int v, hipStream_t s);
hipError_t launch_hot_lists(const unsigned long long* hits, int nlist, int gc, int32_t* out, hipStream_t s);
hipError_t launch_read_hits(unsigned long long* hits, int64_t n, int64_t* out, int reset, hipStream_t s);
hipError_t launch_state_thr(const int64_t* ids, const float* scores, const float* qnorm, int64_t nq, int k, int l2,
                            uint32_t* thr, hipStream_t s);
hipError_t launch_lists_of_rows(const int32_t* rows, int64_t n, const int* list_off, int nlist, int32_t* out, hipStream_t s);
hipError_t launch_reorder_probes(const int32_t* probe, int np, const int32_t* prev, int pp, const int32_t* hot, int nh,
                                 int64_t nq, int32_t* out, hipStream_t s);
hipError_t launch_rescore(const float* q, int64_t nq, int d, int dtype, const void* rows, const float* row_norm,
                          const int64_t* row_ids, int64_t nrows, const int32_t* cand, int m, int k, int l2,
                          int64_t* out_ids, float* out_scores, int32_t* out_rows, hipStream_t s);
hipError_t launch_bf16_to_f16(const void* x, int64_t n, void* out, int* overflow, hipStream_t s);
hipError_t launch_split_f32(const float* x, int64_t n, void* hi, void* lo, hipStream_t s);
hipError_t launch_set_resident(int* resident, int nlist, const int32_t* lists, int64_t n, int value, hipStream_t s);
hipError_t launch_split_probes(const int32_t* probe, int64_t nq, int np, const int* resident, int nlist, unsigned long long* hits,
                               int32_t* out_resident, int32_t* out_missing, hipStream_t s);
hipError_t launch_check_labels(const int64_t* ids, int64_t n, int* negative, hipStream_t s);

struct BucketArgs {
    const int* probe;           // [nq*nprobe]
    int nq, nprobe, nlist, cw;
    const int* list_off;        // [nlist+1]
    int* list_w;                // [nlist]   (zeroed by the first kernel's launch sequence)
    int* pair_entry;            // [nq*nprobe]
    int* bucket_off;            // [nlist+1]
    int* bucket_q;              // [nq*nprobe]
    int* item_base;             // [nlist+1]
    int* slot_base;             // [nlist+1] first result slot of every list
    int* dyn;                   // device scalars
    int4* xq_rec;               // [8][item_cap][2] per-XCD queues of item records (see ScanArgs)
    int* xq_count;              // [8] queue lengths
    int* round_cnt;             // [8][64] items per queue and round, then where each round starts (zeroed before launch)
    int* round_cur;             // [8][64] items placed so far per queue and round (zeroed before launch)
    int item_cap;
    int slot_cap;               // result slots the workspace holds
    int item_target;            // aimed number of work items (rows per segment follow from it)
    unsigned long long* hits;   // [nlist] probes per list since load or the last reset (index-owned), or nullptr
    const int* resident;        // [nlist] 1 = the list's vectors are in place; probes of the other lists are dropped
};
hipError_t launch_bucketing(const BucketArgs& a, hipStream_t s);

}  // namespace hr
