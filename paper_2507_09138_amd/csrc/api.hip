// Host side of the C ABI declared in hr_ivf.h: argument checks, workspace layout, launch
// sequence.  Nothing here synchronises the caller's stream except hr_ivf_load and hr_ivf_stats.
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "common.h"

// Scratch memory of hr_ivf_search_static, the entry point for callers that cannot allocate: a
// fixed array in the library's device image, one copy per GPU, held until the process ends.  In
// host code the array's name only stands for the symbol; its address on a device is asked for
// once per device (with that device current) and kept, and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[HR_STATIC_SCRATCH_BYTES];
static constexpr int kMaxDevices = 64;
static void* g_scratch[kMaxDevices];           // device address of `scratch` per device, null until asked for
static std::mutex g_scratch_mu;

// address of the scratch array on device `dev`, which must be the current device.  (Not a static function: the
// compiler gives a file-scope static device variable a symbol that the runtime can look up only when a host
// function with external linkage names it.)
namespace hr {
hipError_t static_scratch_address(int dev, void** out);
}
hipError_t hr::static_scratch_address(int dev, void** out)
{
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (g_scratch[dev] == nullptr) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (p == nullptr) return hipErrorInvalidSymbol;
        g_scratch[dev] = p;
    }
    *out = g_scratch[dev];
    return hipSuccess;
}

namespace hr {
hipError_t launch_scan_f32(int d, const ScanArgs& a, int shape, int grid, size_t lds, hipStream_t s);
hipError_t launch_scan_f16(int d, const ScanArgs& a, int shape, int grid, size_t lds, hipStream_t s);
hipError_t launch_scan_bf16(int d, const ScanArgs& a, int shape, int grid, size_t lds, hipStream_t s);
hipError_t launch_scan_f16x2(int d, const ScanArgs& a, int shape, int grid, size_t lds, hipStream_t s);

hipError_t launch_seed_f32(int d, const SeedArgs& a, hipStream_t s);
hipError_t launch_seed_f16(int d, const SeedArgs& a, hipStream_t s);
hipError_t launch_seed_bf16(int d, const SeedArgs& a, hipStream_t s);

hipError_t launch_seed(int dtype, int d, const SeedArgs& a, hipStream_t s)
{
    switch (dtype) {
    case HR_F32: return launch_seed_f32(d, a, s);
    case HR_F16: return launch_seed_f16(d, a, s);
    case HR_BF16: return launch_seed_bf16(d, a, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_scan(int dtype, int d, const ScanArgs& a, int shape, int grid, size_t lds, hipStream_t s)
{
    switch (dtype) {
    case HR_F32: return launch_scan_f32(d, a, shape, grid, lds, s);
    case HR_F16: return launch_scan_f16(d, a, shape, grid, lds, s);
    case HR_BF16: return launch_scan_bf16(d, a, shape, grid, lds, s);
    case HR_F16X2: return launch_scan_f16x2(d, a, shape, grid, lds, s);
    default: return hipErrorInvalidValue;
    }
}

// LDS bytes of one workgroup of the given shape with nbuf staging buffers and selection
// buffers of cap entries per query column (must match the carve-up at the top of k_scan and
// ScanShape::buf_bytes)
size_t scan_lds_bytes(int dtype, int d, int cap, int shape, int nbuf)
{
    const int nw = shape_waves(shape);
    size_t buf;
    if (dtype == HR_F32) {
        buf = (size_t)kBlockRows * (d * 2 + kRowPad) * 2;
    } else if (dtype == HR_F16X2) {
        const int chunks = kBlockRows * d * 2 / 16, threads = nw * 64;
        buf = (size_t)((chunks + threads - 1) / threads) * threads * 16 * 2;
    } else {
        const int chunks = kBlockRows * d * 2 / 16, threads = nw * 64;
        buf = (size_t)((chunks + threads - 1) / threads) * threads * 16;
    }
    const size_t cw = (size_t)cols_per_set(dtype) * shape_sets(shape);
    return nbuf * buf + cw * cap * sizeof(Cand) + (size_t)nbuf * kBlockRows * sizeof(float) + 32;
}
}  // namespace hr

static constexpr int kLdsLimit = 160 * 1024;      // LDS per workgroup on gfx950

// Workgroup shape, number of staging buffers and selection buffers of a list scan.
// Rows that go straight from HBM to LDS (16-bit storage, and float32 lists split into two
// binary16 tables at load): 8 waves, the selection buffers in global memory (they are the
// item's result slots; a wave alone uses those of its columns and candidates are few), and
// LDS left to as many 16-row buffers as fit: 6 or 4 (blocks in pairs, one barrier per pair),
// else 3 or 2.  More rows on their way is what counts when few queries share a list and the
// scan is bound by HBM (measured with the buffers in LDS and 4 row buffers instead: C4 +2 %,
// the 38 M x 1024 index +2.5 %, C3 +1 %).
// float32 rows split on the fly are staged through registers into 2 padded buffers: selection
// buffers in LDS for small k when they fit (8 waves, else 4 with half the columns), in global
// memory for large k.  shape -1 = no fit.
struct ScanPick { int shape, nbuf, cap, gsel; };
static ScanPick pick_shape(int dtype, int d, int k)
{
    const int cap = hr::sel_cap(k);
    if (dtype != HR_F32) {
        for (int nbuf : {6, 4, 3, 2})
            if (hr::scan_lds_bytes(dtype, d, 0, hr::SCAN_WIDE, nbuf) <= (size_t)kLdsLimit) return {hr::SCAN_WIDE, nbuf, cap, 1};
        return {-1, 0, 0, 0};
    }
    if (cap > 64) {
        if (hr::scan_lds_bytes(dtype, d, 0, hr::SCAN_WIDE, 2) <= (size_t)kLdsLimit) return {hr::SCAN_WIDE, 2, cap, 1};
        return {-1, 0, 0, 0};
    }
    for (int shape : {hr::SCAN_WIDE, hr::SCAN_NARROW})
        if (hr::scan_lds_bytes(dtype, d, cap, shape, 2) <= (size_t)kLdsLimit) return {shape, 2, cap, 0};
    return {-1, 0, 0, 0};
}

using namespace hr;

static thread_local char g_err[512] = "";

static int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

#define HR_HIP(call)                                                                      \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) return fail(HR_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

static constexpr uint64_t kMagic = 0x4852495646313031ULL;   // "HRIVF101"

struct hr_ivf_index {
    uint64_t magic;
    const float* centroids;
    const void* vectors;
    const int64_t* ids;
    int64_t nlist, N;
    int d, dtype;
    int* d_list_off;       // [nlist+1] int32
    float* d_row_norm;     // [N]
    float* d_cent_norm;    // [nlist]
    void* d_cent_hi;       // [nlist, d] binary16: centroids rounded
    void* d_cent_lo;       // [nlist, d] binary16: (centroid - hi) * 2^11
    void* d_vec_hi;        // float32 lists only, when memory allows: [N, d] binary16 hi and scaled lo tables of the
    void* d_vec_lo;        // rows (the split the scan would otherwise redo for every block it stages); else null
    void* d_vec16;         // bfloat16 lists only, when memory and the value range allow: [N, d] the rows as binary16
    int* d_flag;           // two device ints: [0] a bfloat16 value did not fit binary16, [1] a negative label
    unsigned long long* d_hits;   // [nlist] probes per list since load / last reset
    int* d_resident;       // [nlist] 1 = the list's vectors are in place (all lists, until the caller says otherwise)
    int num_cus;
    int lds_limit;
    int device;            // the device the index lives on
    void* scratch;         // address of the library's static scratch array on that device
    // optional kernel timing (hr_ivf_profile_begin/end)
    hipEvent_t* prof_ev;   // 2 * prof_cap events
    int prof_cap, prof_n;
};

// storage type the list scan runs on
static int scan_dtype(const hr_ivf_index* ix) { return ix->d_vec_hi ? (int)HR_F16X2 : (ix->d_vec16 ? (int)HR_F16 : ix->dtype); }
// form of the query operand the list scan multiplies (what k_prep_queries is asked for)
static int operand_dtype(const hr_ivf_index* ix) { const int s = scan_dtype(ix); return s == HR_F16X2 ? (int)HR_F32 : s; }
// rows and their type for the kernels that read single rows (threshold seeding, rescoring)
static int row_dtype(const hr_ivf_index* ix) { return ix->d_vec16 ? (int)HR_F16 : ix->dtype; }
static const void* row_table(const hr_ivf_index* ix) { return ix->d_vec16 ? ix->d_vec16 : ix->vectors; }

static bool dim_supported(int d)
{
    return d == 64 || d == 128 || d == 256 || d == 512 || d == 768 || d == 1024;
}

static size_t align_up(size_t v) { return (v + HR_WORKSPACE_ALIGN - 1) & ~(size_t)(HR_WORKSPACE_ALIGN - 1); }

// Layout of the caller's workspace for one batch shape.  Offsets in bytes.
struct Plan {
    // coarse step: centroid table scanned with all queries as one dense bucket
    int shape_c /* workgroup shape, -1 = no fit */, nbuf_c, cap_c, cw_c, nqt_c, seg_c, nseg_c, items_c;
    // list scan
    int shape_s, nbuf_s, cap_s, gsel_s, cw_s, item_cap, item_target;
    int slot_stride;                // entries per result slot of the list scan
    int slot_cap;                   // result slots: one per (list segment, query of the list's bucket)
    size_t o_zero, n_zero;          // ints cleared per call: list_w[nlist], dyn[DYN_COUNT], counters[8], ..., then
    size_t zoff_round, zoff_hist, zoff_hpar;   // (in ints from o_zero) round counters of the queues, per-query key histograms and their parameters
    size_t o_thr;                   // 2*nq ints set to "-inf"
    size_t o_qop_c, o_qnorm_c, o_qop_s, o_qnorm_s;
    size_t o_probe;
    size_t o_pair_entry, o_bucket_off, o_bucket_q, o_item_base, o_slot_base, o_xq;
    size_t o_ckeys;                 // coarse step: [cchunk, nlist] keys of one chunk of queries
    int64_t cchunk;                 // queries per coarse chunk
    size_t o_slot_cnt, o_slot_ent;
    size_t total;
    // the regions above in order of their offsets (for hr_ivf_workspace_layout); a guard gap of
    // HR_WORKSPACE_ALIGN bytes that nothing writes lies behind every one
    int nreg;
    size_t reg_off[24], reg_len[24];
};

// What bounds the size of a plan: the aimed number of work items of the list scan (segments are sized so that
// about that many items result: fewer, larger items need fewer result slots) and the bytes of the coarse key table
// (queries are scored in chunks that fit it).
struct PlanLimits { int item_target; size_t ckeys_bytes; };
static constexpr PlanLimits kDefaultLimits = {kItemTarget, (size_t)512 << 20};

static Plan make_plan(const hr_ivf_index* ix, int64_t nq, int nprobe, int k, const PlanLimits& lim = kDefaultLimits)
{
    Plan p{};
    const int64_t nlist = ix->nlist;
    // coarse step: dense scoring (no selection buffers in LDS) in the widest shape that fits
    const ScanPick ps = pick_shape(scan_dtype(ix), ix->d, k);
    p.shape_c = -1; p.nbuf_c = 0; p.cap_c = 0;
    for (int nbuf = 3; nbuf >= 2 && p.shape_c < 0; nbuf--)
        if (scan_lds_bytes(HR_F16X2, ix->d, 0, SCAN_WIDE, nbuf) <= (size_t)kLdsLimit) { p.shape_c = SCAN_WIDE; p.nbuf_c = nbuf; }
    p.shape_s = ps.shape; p.nbuf_s = ps.nbuf; p.cap_s = ps.cap; p.gsel_s = ps.gsel;
    p.cw_c = cols_per_set(HR_F32) * shape_sets(p.shape_c < 0 ? 0 : p.shape_c);
    // queries per coarse chunk: the [chunk, nlist] key table stays within its limit, 512 MiB by default (the more
    // queries per launch the better both kernels fill the device: 16384 lists, four chunks of 2048 queries 1.88 ms,
    // one of 8192 1.45 ms)
    p.cchunk = (int64_t)lim.ckeys_bytes / (nlist * 4) / p.cw_c * p.cw_c;
    if (p.cchunk < p.cw_c) p.cchunk = p.cw_c;
    if (p.cchunk > nq) p.cchunk = nq > 0 ? nq : 1;
    p.nqt_c = (int)((p.cchunk + p.cw_c - 1) / p.cw_c);
    int64_t seg = (nlist * (int64_t)p.nqt_c + 511) / 512;
    seg = (seg + 15) & ~15LL;
    if (seg < 32) seg = 32;
    if (seg > 1024) seg = 1024;
    p.seg_c = (int)seg;
    p.nseg_c = (int)((nlist + seg - 1) / seg);
    p.items_c = p.nseg_c * p.nqt_c;
    p.cw_s = cols_per_set(scan_dtype(ix)) * shape_sets(p.shape_s < 0 ? 0 : p.shape_s);
    const int64_t pairs = nq * nprobe;
    // Work items: sum over probed lists of segments x query tiles.  Segments have at least C / item_target rows, C =
    // sum of rows x tiles, so there are at most item_target items plus one per (list, tile) for the ragged ends.
    // Result slots: sum of segments x bucket width <= cw x item_target, plus one per pair for the ragged ends.
    p.item_target = lim.item_target;
    p.item_cap = (int)(lim.item_target + pairs / p.cw_s + (pairs < nlist ? pairs : nlist) + 8);
    p.slot_cap = (int)((int64_t)p.cw_s * lim.item_target + pairs);

    size_t o = 0;
    auto take = [&](size_t bytes) {
        size_t at = o;
        p.reg_off[p.nreg] = at; p.reg_len[p.nreg] = bytes; p.nreg++;
        o = align_up(o + bytes) + HR_WORKSPACE_ALIGN;
        return at;
    };
    p.zoff_round = (size_t)nlist + DYN_COUNT + 24;  // + 8 counters, 8 queue lengths, 8 queue heads
    p.zoff_hist = p.zoff_round + 2 * 8 * 64;
    p.zoff_hpar = p.zoff_hist + (size_t)nq * kHistBins;
    p.n_zero = p.zoff_hpar + (size_t)nq * 2;
    p.o_zero = take(p.n_zero * 4);
    p.o_thr = take((size_t)nq * 2 * 4);
    p.o_qop_c = take((size_t)nq * 2 * ix->d * 2);
    p.o_qnorm_c = take((size_t)nq * 4);
    p.o_qop_s = operand_dtype(ix) == HR_F32 ? p.o_qop_c
                                            : take((size_t)nq * (operand_dtype(ix) == HR_BF16 ? 2 : 1) * ix->d * 2);
    p.o_qnorm_s = take((size_t)nq * 4);
    p.o_probe = take((size_t)pairs * 4);
    p.o_pair_entry = take((size_t)pairs * 4);
    p.o_bucket_off = take((size_t)(nlist + 1) * 4);
    p.o_bucket_q = take((size_t)pairs * 4);
    p.o_item_base = take((size_t)(nlist + 1) * 4);
    p.o_slot_base = take((size_t)(nlist + 1) * 4);
    p.o_xq = take((size_t)p.item_cap * 8 * 2 * sizeof(int4));
    p.o_ckeys = take((size_t)p.cchunk * nlist * 4);
    const size_t slots = (size_t)p.slot_cap;
    p.o_slot_cnt = take(slots * 4);
    p.slot_stride = p.gsel_s || (p.cap_s <= 64 && p.cap_s > k) ? p.cap_s : k;   // whole selection buffers, nothing to cut (else: k)
    p.o_slot_ent = take(slots * (size_t)p.slot_stride * sizeof(Cand));
    p.total = o;
    return p;
}

static int check_index(const hr_ivf_index* ix)
{
    if (!ix || ix->magic != kMagic) return fail(HR_ERR_HANDLE, "index handle is null, freed or corrupt");
    return HR_OK;
}

static int check_batch(const hr_ivf_index* ix, int64_t nq, int nprobe, int k, int metric, bool need_k)
{
    if (nq < 0 || nq > (1 << 24)) return fail(HR_ERR_ARG, "nq=%lld out of range", (long long)nq);
    if (nprobe < 1 || nprobe > ix->nlist || nprobe > HR_NPROBE_MAX)
        return fail(HR_ERR_ARG, "nprobe=%d must be in 1..min(nlist=%lld, %d)", nprobe, (long long)ix->nlist, HR_NPROBE_MAX);
    if (need_k && (k < 1 || k > HR_K_MAX)) return fail(HR_ERR_ARG, "k=%d must be in 1..%d", k, HR_K_MAX);
    if (metric != HR_METRIC_IP && metric != HR_METRIC_L2) return fail(HR_ERR_ARG, "unknown metric %d", metric);
    if (nq * (int64_t)nprobe >= (1LL << 30)) return fail(HR_ERR_UNSUPPORTED, "nq*nprobe too large");
    return HR_OK;
}

static int check_ws(const Plan& p, const void* ws, size_t bytes)
{
    if (!ws) return fail(HR_ERR_WORKSPACE, "workspace is null");
    if (((uintptr_t)ws) % HR_WORKSPACE_ALIGN) return fail(HR_ERR_WORKSPACE, "workspace not %d-byte aligned", HR_WORKSPACE_ALIGN);
    if (bytes < p.total) return fail(HR_ERR_WORKSPACE, "workspace has %zu bytes, need %zu", bytes, p.total);
    return HR_OK;
}

extern "C" {

const char* hr_last_error(void) { return g_err; }
const char* hr_version(void) { return "hr_ivf 0.1 gfx950"; }

int hr_ivf_load(const float* centroids, const int64_t* list_offsets, const void* list_vectors,
                const int64_t* list_ids, int64_t nlist, int64_t N, int32_t d, int32_t dtype,
                void* stream, hr_ivf_index** out)
{
    if (!out) return fail(HR_ERR_ARG, "out is null");
    *out = nullptr;
    if (!centroids || !list_offsets) return fail(HR_ERR_ARG, "centroids / list_offsets is null");
    if (nlist < 1 || nlist >= (1LL << 24)) return fail(HR_ERR_ARG, "nlist=%lld out of range", (long long)nlist);
    if (N < 0 || N >= (1LL << 31)) return fail(HR_ERR_ARG, "N=%lld out of range (< 2^31)", (long long)N);
    if (N > 0 && (!list_vectors || !list_ids)) return fail(HR_ERR_ARG, "list_vectors / list_ids is null");
    const bool row_tables = (dtype & HR_LOAD_ROW_TABLES) != 0;
    dtype &= ~HR_LOAD_ROW_TABLES;
    if (dtype != HR_F32 && dtype != HR_F16 && dtype != HR_BF16) return fail(HR_ERR_ARG, "unknown dtype %d", dtype);
    if (d < 1) return fail(HR_ERR_ARG, "d=%d", d);
    if (!dim_supported(d)) return fail(HR_ERR_UNSUPPORTED, "d=%d not one of 64,128,256,512,768,1024", d);
    if (list_offsets[0] != 0 || list_offsets[nlist] != N) return fail(HR_ERR_ARG, "list_offsets must start at 0 and end at N");
    for (int64_t l = 0; l < nlist; l++)
        if (list_offsets[l + 1] < list_offsets[l]) return fail(HR_ERR_ARG, "list_offsets decreases at list %lld", (long long)l);

    hipStream_t s = (hipStream_t)stream;
    int dev = 0;
    HR_HIP(hipGetDevice(&dev));
    hr_ivf_index* ix = new (std::nothrow) hr_ivf_index();
    if (!ix) return fail(HR_ERR_HIP, "out of host memory");
    ix->centroids = centroids; ix->vectors = list_vectors; ix->ids = list_ids;
    ix->nlist = nlist; ix->N = N; ix->d = d; ix->dtype = dtype;
    int* h_off = new (std::nothrow) int[nlist + 1];
    if (!h_off) { delete ix; return fail(HR_ERR_HIP, "out of host memory"); }
    for (int64_t l = 0; l <= nlist; l++) h_off[l] = (int)list_offsets[l];
    ix->device = dev;
    hipError_t e = hipDeviceGetAttribute(&ix->num_cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess) e = hr::static_scratch_address(dev, &ix->scratch);
    ix->lds_limit = 160 * 1024;     // LDS per workgroup on gfx950
    if (e == hipSuccess) {
        hipDeviceProp_t prop;
        e = hipGetDeviceProperties(&prop, dev);
        if (e == hipSuccess && strncmp(prop.gcnArchName, "gfx950", 6) != 0) {
            delete[] h_off;
            delete ix;
            return fail(HR_ERR_UNSUPPORTED, "device is %s; this library is built for gfx950 only", prop.gcnArchName);
        }
    }
    if (e == hipSuccess) e = hipMalloc(&ix->d_list_off, (size_t)(nlist + 1) * 4);
    if (e == hipSuccess) e = hipMalloc(&ix->d_row_norm, (size_t)(N > 0 ? N : 1) * 4);
    if (e == hipSuccess) e = hipMalloc(&ix->d_cent_norm, (size_t)nlist * 4);
    if (e == hipSuccess) e = hipMalloc(&ix->d_cent_hi, (size_t)nlist * d * 2);
    if (e == hipSuccess) e = hipMalloc(&ix->d_cent_lo, (size_t)nlist * d * 2);
    if (e == hipSuccess) e = hipMalloc(&ix->d_hits, (size_t)nlist * 8);
    if (e == hipSuccess) e = hipMalloc(&ix->d_flag, 2 * sizeof(int));
    if (e == hipSuccess) e = hipMalloc(&ix->d_resident, (size_t)nlist * sizeof(int));
    if (e == hipSuccess) e = launch_set_resident(ix->d_resident, (int)nlist, nullptr, nlist, 1, s);
    if (e == hipSuccess) e = hipMemsetAsync(ix->d_hits, 0, (size_t)nlist * 8, s);
    if (e == hipSuccess) e = hipMemsetAsync(ix->d_flag, 0, 2 * sizeof(int), s);
    if (e == hipSuccess) e = launch_check_labels(list_ids, N, ix->d_flag + 1, s);
    if (e == hipSuccess) e = hipMemcpyAsync(ix->d_list_off, h_off, (size_t)(nlist + 1) * 4, hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = launch_row_norms(list_vectors, dtype, N, d, ix->d_row_norm, s);
    if (e == hipSuccess) e = launch_row_norms(centroids, HR_F32, nlist, d, ix->d_cent_norm, s);
    if (e == hipSuccess) e = launch_split_f32(centroids, nlist * d, ix->d_cent_hi, ix->d_cent_lo, s);
    if (e == hipSuccess && dtype == HR_F32 && N > 0 && row_tables) {
        // float32 lists, when the caller asks for row tables: the scan multiplies binary16 hi and lo parts
        // of the rows.  Made once here (same bytes again: 2 + 2 per element) they go straight from HBM to
        // LDS like 16-bit lists; made on the fly they pass through registers for every block.  Only when
        // that leaves at least half of the free device memory; otherwise the scan splits on the fly.
        const size_t bytes = (size_t)N * d * 2;
        size_t free_b = 0, total_b = 0;
        if (hipMemGetInfo(&free_b, &total_b) == hipSuccess && 2 * bytes <= free_b / 2) {
            if (hipMalloc(&ix->d_vec_hi, bytes) != hipSuccess) ix->d_vec_hi = nullptr;
            if (ix->d_vec_hi && hipMalloc(&ix->d_vec_lo, bytes) != hipSuccess) { (void)hipFree(ix->d_vec_hi); ix->d_vec_hi = nullptr; ix->d_vec_lo = nullptr; }
            if (!ix->d_vec_hi) (void)hipGetLastError();          // (not an error of the load: the other path is taken)
            else e = launch_split_f32((const float*)list_vectors, N * d, ix->d_vec_hi, ix->d_vec_lo, s);
        }
    }
    if (e == hipSuccess && dtype == HR_BF16 && N > 0 && row_tables) {
        // bfloat16 lists, when the caller asks for row tables: as binary16 (same bytes again) every value
        // keeps its 8 significant bits, and the scan can multiply them with the query rounded to binary16
        // in one MFMA column per query instead of two (bfloat16 hi and lo parts): twice the queries per
        // work item.  Only when that leaves at least half of the free device memory and no value overflows.
        const size_t bytes = (size_t)N * d * 2;
        size_t free_b = 0, total_b = 0;
        if (hipMemGetInfo(&free_b, &total_b) == hipSuccess && bytes <= free_b / 2) {
            if (hipMalloc(&ix->d_vec16, bytes) != hipSuccess) ix->d_vec16 = nullptr;
            if (!ix->d_vec16) (void)hipGetLastError();
            else e = launch_bf16_to_f16(list_vectors, N * d, ix->d_vec16, ix->d_flag, s);
        }
    }
    if (e == hipSuccess) e = hipStreamSynchronize(s);
    int flags[2] = {0, 0};                      // [0] a bfloat16 value beyond binary16, [1] a negative label
    if (e == hipSuccess) e = hipMemcpy(flags, ix->d_flag, sizeof flags, hipMemcpyDeviceToHost);
    if (e == hipSuccess && ix->d_vec16 && flags[0]) {      // the lists are scanned as bfloat16
        (void)hipFree(ix->d_vec16);
        ix->d_vec16 = nullptr;
    }
    delete[] h_off;
    if (e != hipSuccess || flags[1]) {
        if (ix->d_list_off) (void)hipFree(ix->d_list_off);
        if (ix->d_row_norm) (void)hipFree(ix->d_row_norm);
        if (ix->d_cent_norm) (void)hipFree(ix->d_cent_norm);
        if (ix->d_cent_hi) (void)hipFree(ix->d_cent_hi);
        if (ix->d_cent_lo) (void)hipFree(ix->d_cent_lo);
        if (ix->d_hits) (void)hipFree(ix->d_hits);
        if (ix->d_resident) (void)hipFree(ix->d_resident);
        if (ix->d_vec_hi) (void)hipFree(ix->d_vec_hi);
        if (ix->d_vec_lo) (void)hipFree(ix->d_vec_lo);
        if (ix->d_vec16) (void)hipFree(ix->d_vec16);
        if (ix->d_flag) (void)hipFree(ix->d_flag);
        delete ix;
        if (e == hipSuccess) return fail(HR_ERR_ARG, "list_ids holds a negative label (labels must be >= 0: -1 marks an empty place in results)");
        return fail(HR_ERR_HIP, "hr_ivf_load: %s", hipGetErrorString(e));
    }
    ix->magic = kMagic;
    *out = ix;
    return HR_OK;
}

static void drop_events(hr_ivf_index* ix)
{
    if (!ix->prof_ev) return;
    for (int i = 0; i < 2 * ix->prof_cap; i++)
        if (ix->prof_ev[i]) (void)hipEventDestroy(ix->prof_ev[i]);
    delete[] ix->prof_ev;
    ix->prof_ev = nullptr;
    ix->prof_cap = ix->prof_n = 0;
}

int hr_ivf_profile_begin(hr_ivf_index* ix, int32_t max_calls)
{
    if (int rc = check_index(ix)) return rc;
    if (max_calls < 1 || max_calls > 65536) return fail(HR_ERR_ARG, "max_calls=%d", max_calls);
    drop_events(ix);
    ix->prof_ev = new (std::nothrow) hipEvent_t[2 * (size_t)max_calls]();
    if (!ix->prof_ev) return fail(HR_ERR_HIP, "out of host memory");
    ix->prof_cap = max_calls;
    for (int i = 0; i < 2 * max_calls; i++) {
        hipError_t e = hipEventCreate(&ix->prof_ev[i]);
        if (e != hipSuccess) { drop_events(ix); return fail(HR_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e)); }
    }
    return HR_OK;
}

int hr_ivf_profile_end(hr_ivf_index* ix, int32_t* n, double* scan_ms_avg)
{
    if (int rc = check_index(ix)) return rc;
    if (!n || !scan_ms_avg) return fail(HR_ERR_ARG, "n / scan_ms_avg is null");
    double sum = 0.0;
    int cnt = 0;
    for (int i = 0; i < ix->prof_n; i++) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(ix->prof_ev[2 * i + 1]);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ix->prof_ev[2 * i], ix->prof_ev[2 * i + 1]);
        if (e != hipSuccess) { drop_events(ix); return fail(HR_ERR_HIP, "event timing: %s", hipGetErrorString(e)); }
        sum += ms;
        cnt++;
    }
    *n = cnt;
    *scan_ms_avg = cnt ? sum / cnt : 0.0;
    drop_events(ix);
    return HR_OK;
}

int hr_ivf_free(hr_ivf_index* ix)
{
    if (int rc = check_index(ix)) return rc;
    drop_events(ix);
    ix->magic = 0;
    (void)hipFree(ix->d_list_off);
    (void)hipFree(ix->d_row_norm);
    (void)hipFree(ix->d_cent_norm);
    (void)hipFree(ix->d_cent_hi);
    (void)hipFree(ix->d_cent_lo);
    (void)hipFree(ix->d_hits);
    (void)hipFree(ix->d_resident);
    if (ix->d_vec_hi) (void)hipFree(ix->d_vec_hi);
    if (ix->d_vec_lo) (void)hipFree(ix->d_vec_lo);
    if (ix->d_vec16) (void)hipFree(ix->d_vec16);
    if (ix->d_flag) (void)hipFree(ix->d_flag);
    delete ix;
    return HR_OK;
}

size_t hr_ivf_workspace_bytes(const hr_ivf_index* ix, int64_t nq, int32_t nprobe, int32_t k)
{
    if (check_index(ix)) return 0;
    // (hr_ivf_scan and its step-wise forms take rows of up to HR_NPROBE_MAX places whatever the number of lists)
    if (nprobe < 1 || nprobe > HR_NPROBE_MAX) { fail(HR_ERR_ARG, "nprobe=%d must be in 1..%d", nprobe, HR_NPROBE_MAX); return 0; }
    if (check_batch(ix, nq, nprobe > ix->nlist ? (int)ix->nlist : nprobe, k, HR_METRIC_IP, true)) return 0;
    return make_plan(ix, nq, nprobe, k).total;
}

}  // extern "C"

// ---------------------------------------------------------------------------------------
// persistent workgroups: one per CU (8-wave shape), or two where LDS lets two 4-wave ones share a CU
static int scan_grid(const hr_ivf_index* ix, size_t lds, int shape)
{
    int occ = (int)((size_t)kLdsLimit / lds);
    if (occ < 1) occ = 1;
    const int most = shape == SCAN_WIDE ? 1 : 2;
    if (occ > most) occ = most;
    return ix->num_cus * occ;
}

// query operands for the coarse step (coarse) and / or the list scan (scan), and, in the same launch, what the
// call needs cleared in its workspace
static int enqueue_prep(const hr_ivf_index* ix, const Plan& p, char* ws, const float* queries, int64_t nq, bool coarse,
                        bool scan, hipStream_t s)
{
    const int od = operand_dtype(ix);
    const bool f32 = od == HR_F32;             // the scan multiplies the operand of the coarse step
    HR_HIP(launch_prep_queries(queries, nq, ix->d, scan ? od : (int)HR_F32, (coarse || (scan && f32)) ? ws + p.o_qop_c : nullptr,
                               coarse ? (float*)(ws + p.o_qnorm_c) : nullptr, (scan && !f32) ? ws + p.o_qop_s : nullptr,
                               scan ? (float*)(ws + p.o_qnorm_s) : nullptr, (int*)(ws + p.o_zero), (int64_t)p.n_zero,
                               (int*)(ws + p.o_thr), nq * 2, (int)kKeyNegInf, s));
    return HR_OK;
}

// coarse scoring + top-nprobe: the scan kernel over the centroid table writes every key of a
// chunk of queries, then one wave per query picks the nprobe best
static int enqueue_coarse(const hr_ivf_index* ix, const Plan& p, char* ws, int64_t nq, int nprobe,
                          int metric, int32_t* out_probe, float* out_scores, hipStream_t s)
{
    if (p.shape_c < 0)
        return fail(HR_ERR_UNSUPPORTED, "coarse step does not fit in LDS (d=%d)", ix->d);
    const size_t lds = scan_lds_bytes(HR_F16X2, ix->d, 0, p.shape_c, p.nbuf_c);
    int* zero = (int*)(ws + p.o_zero);
    float* ckeys = (float*)(ws + p.o_ckeys);
    for (int64_t q0 = 0; q0 < nq; q0 += p.cchunk) {
        const int64_t n = nq - q0 < p.cchunk ? nq - q0 : p.cchunk;
        const int nqt = (int)((n + p.cw_c - 1) / p.cw_c);
        ScanArgs a{};
        a.rows = ix->d_cent_hi;
        a.rows_lo = ix->d_cent_lo;
        a.row_norm = ix->d_cent_norm;
        a.qop = ws + p.o_qop_c + (size_t)q0 * 2 * ix->d * 2;
        a.thr = (uint32_t*)(ws + p.o_thr);
        a.work_counter = zero + ix->nlist + DYN_COUNT;
        a.dense = 1;
        a.dense_items = p.nseg_c * nqt;
        a.dense_nqt = nqt;
        a.dense_seg_rows = p.seg_c;
        a.dense_nrows = (int)ix->nlist;
        a.key_out = ckeys;
        a.nq = (int)n; a.k = nprobe; a.cap = 0; a.l2 = metric == HR_METRIC_L2;
        a.nbuf = p.nbuf_c;
        if (q0 > 0) HR_HIP(launch_fill_i32(a.work_counter, 1, 0, s));
        int grid = scan_grid(ix, lds, p.shape_c);
        if (grid > a.dense_items) grid = a.dense_items;
        HR_HIP(launch_scan(HR_F16X2, ix->d, a, p.shape_c, grid, lds, s));
        HR_HIP(launch_topk_rows(ckeys, (const float*)(ws + p.o_qnorm_c) + q0, out_probe + q0 * nprobe,
                                out_scores ? out_scores + q0 * nprobe : nullptr, n, (int)ix->nlist, nprobe,
                                a.l2, s));
    }
    return HR_OK;
}

// grouping by list + cluster-major scan + per-query merge
static int enqueue_scan(const hr_ivf_index* ix, const Plan& p, char* ws, int64_t nq, const int32_t* probe,
                        int nprobe, int k, int metric, int64_t* out_ids, float* out_scores, hipStream_t s,
                        bool carried = false, int32_t* io_rows = nullptr)
{
    if (p.shape_s < 0)
        return fail(HR_ERR_UNSUPPORTED, "list scan does not fit in LDS (d=%d, k=%d)", ix->d, k);
    const size_t lds = scan_lds_bytes(scan_dtype(ix), ix->d, p.gsel_s ? 0 : p.cap_s, p.shape_s, p.nbuf_s);
    int* zero = (int*)(ws + p.o_zero);
    BucketArgs b{};
    b.probe = probe; b.nq = (int)nq; b.nprobe = nprobe; b.nlist = (int)ix->nlist; b.cw = p.cw_s;
    b.list_off = ix->d_list_off;
    b.list_w = zero;
    b.hits = ix->d_hits;
    b.resident = ix->d_resident;
    b.pair_entry = (int*)(ws + p.o_pair_entry);
    b.bucket_off = (int*)(ws + p.o_bucket_off);
    b.bucket_q = (int*)(ws + p.o_bucket_q);
    b.item_base = (int*)(ws + p.o_item_base);
    b.slot_base = (int*)(ws + p.o_slot_base);
    b.slot_cap = p.slot_cap;
    b.item_target = p.item_target;
    b.dyn = zero + ix->nlist;
    b.xq_rec = (int4*)(ws + p.o_xq);
    b.xq_count = zero + ix->nlist + DYN_COUNT + 8;
    b.round_cnt = zero + p.zoff_round;
    b.round_cur = zero + p.zoff_round + 8 * 64;
    b.item_cap = p.item_cap;
    HR_HIP(launch_bucketing(b, s));

    // starting lower bounds: from a carried result, and from the first rows of every query's best-ranked list
    if (carried)
        HR_HIP(launch_state_thr(out_ids, out_scores, (const float*)(ws + p.o_qnorm_s), nq, k, metric == HR_METRIC_L2,
                                (uint32_t*)(ws + p.o_thr) + nq, s));
    SeedArgs sd{};
    sd.rows = row_table(ix); sd.row_norm = ix->d_row_norm; sd.qop = ws + p.o_qop_s;
    sd.probe = probe; sd.list_off = ix->d_list_off; sd.resident = ix->d_resident;
    sd.thr = (uint32_t*)(ws + p.o_thr) + nq;
    sd.hpar = (float*)(zero + p.zoff_hpar);
    sd.nq = (int)nq; sd.nprobe = nprobe; sd.nlist = (int)ix->nlist; sd.k = k;
    sd.seed_rows = k + 28 < 64 ? 64 : ((k + 28 + 15) & ~15);
    if (sd.seed_rows > 192) sd.seed_rows = 192;
    sd.l2 = metric == HR_METRIC_L2;
    HR_HIP(launch_seed(row_dtype(ix), ix->d, sd, s));

    ScanArgs a{};
    a.rows = ix->d_vec_hi ? ix->d_vec_hi : row_table(ix);
    a.rows_lo = ix->d_vec_lo;
    a.row_norm = ix->d_row_norm;
    a.row_ids = ix->ids;
    a.qop = ws + p.o_qop_s;
    a.thr = (uint32_t*)(ws + p.o_thr) + nq;
    a.slot_cnt = (int*)(ws + p.o_slot_cnt);
    a.slot_ent = (Cand*)(ws + p.o_slot_ent);
    a.slot_stride = p.slot_stride;
    a.work_counter = zero + ix->nlist + DYN_COUNT + 1;
    a.list_off = ix->d_list_off;
    a.bucket_off = b.bucket_off;
    a.bucket_q = b.bucket_q;
    a.dyn = b.dyn;
    a.xq_rec = b.xq_rec;
    a.xq_count = b.xq_count;
    a.xq_head = zero + ix->nlist + DYN_COUNT + 16;
    a.xq_stride = p.item_cap;
    a.dense = 0;
    a.nq = (int)nq; a.k = k; a.cap = p.cap_s; a.l2 = metric == HR_METRIC_L2;
    a.nbuf = p.nbuf_s;
    a.gsel = p.gsel_s;
    a.hist = zero + p.zoff_hist;
    a.hpar = (const float*)(zero + p.zoff_hpar);
    hr_ivf_index* mix = const_cast<hr_ivf_index*>(ix);
    const bool timed = mix->prof_ev && mix->prof_n < mix->prof_cap;
    if (timed) HR_HIP(hipEventRecord(mix->prof_ev[2 * mix->prof_n], s));
    HR_HIP(launch_scan(scan_dtype(ix), ix->d, a, p.shape_s, scan_grid(ix, lds, p.shape_s), lds, s));
    if (timed) {
        HR_HIP(hipEventRecord(mix->prof_ev[2 * mix->prof_n + 1], s));
        mix->prof_n++;
    }

    MergeArgs m{};
    m.slot_cnt = a.slot_cnt; m.slot_ent = a.slot_ent; m.slot_stride = p.slot_stride;
    m.row_ids = ix->ids;
    m.qnorm = (const float*)(ws + p.o_qnorm_s);
    m.probe = probe; m.pair_entry = b.pair_entry;
    m.list_off = ix->d_list_off; m.bucket_off = b.bucket_off; m.slot_base = b.slot_base; m.dyn = b.dyn;
    m.nq = (int)nq; m.nprobe = nprobe; m.nlist = (int)ix->nlist; m.k = k; m.l2 = a.l2;
    m.out_ids = out_ids; m.out_scores = out_scores;
    m.carried = carried ? 1 : 0;
    m.io_rows = io_rows;
    HR_HIP(launch_merge(m, s));
    return HR_OK;
}

extern "C" {

int hr_ivf_search(const hr_ivf_index* ix, const float* queries, int64_t nq, int32_t nprobe, int32_t k,
                  int32_t metric, int64_t* out_ids, float* out_scores, void* workspace,
                  size_t workspace_bytes, void* stream)
{
    if (int rc = check_index(ix)) return rc;
    if (int rc = check_batch(ix, nq, nprobe, k, metric, true)) return rc;
    if (nq == 0) return HR_OK;
    if (!queries || !out_ids || !out_scores) return fail(HR_ERR_ARG, "queries / out_ids / out_scores is null");
    const Plan p = make_plan(ix, nq, nprobe, k);
    if (int rc = check_ws(p, workspace, workspace_bytes)) return rc;
    char* ws = (char*)workspace;
    hipStream_t s = (hipStream_t)stream;
    if (int rc = enqueue_prep(ix, p, ws, queries, nq, true, true, s)) return rc;
    int32_t* probe = (int32_t*)(ws + p.o_probe);
    if (int rc = enqueue_coarse(ix, p, ws, nq, nprobe, metric, probe, nullptr, s)) return rc;
    return enqueue_scan(ix, p, ws, nq, probe, nprobe, k, metric, out_ids, out_scores, s);
}

// Limits of a plan that has to fit the static scratch array: few, large work items (result slots are
// what takes the room) and a small coarse key table.
static constexpr PlanLimits kStaticLimits = {256, (size_t)4 << 20};

int hr_ivf_search_static(const hr_ivf_index* ix, const float* queries, int64_t nq, int32_t nprobe, int32_t k,
                         int32_t metric, int64_t* out_ids, float* out_scores, void* stream)
{
    if (int rc = check_index(ix)) return rc;
    if (int rc = check_batch(ix, nq, nprobe, k, metric, true)) return rc;
    if (nq == 0) return HR_OK;
    if (!queries || !out_ids || !out_scores) return fail(HR_ERR_ARG, "queries / out_ids / out_scores is null");
    int dev = -1;
    HR_HIP(hipGetDevice(&dev));
    if (dev != ix->device) return fail(HR_ERR_ARG, "current device is %d, the index lives on device %d", dev, ix->device);
    const Plan p = make_plan(ix, nq, nprobe, k, kStaticLimits);
    if (p.total > (size_t)HR_STATIC_SCRATCH_BYTES)
        return fail(HR_ERR_WORKSPACE, "this batch (nq=%lld, nprobe=%d, k=%d) needs %zu bytes of scratch, the static array has %zu: "
                                      "use hr_ivf_search with a workspace", (long long)nq, nprobe, k, p.total, (size_t)HR_STATIC_SCRATCH_BYTES);
    char* ws = (char*)ix->scratch;
    hipStream_t s = (hipStream_t)stream;
    if (int rc = enqueue_prep(ix, p, ws, queries, nq, true, true, s)) return rc;
    int32_t* probe = (int32_t*)(ws + p.o_probe);
    if (int rc = enqueue_coarse(ix, p, ws, nq, nprobe, metric, probe, nullptr, s)) return rc;
    return enqueue_scan(ix, p, ws, nq, probe, nprobe, k, metric, out_ids, out_scores, s);
}

int hr_ivf_coarse(const hr_ivf_index* ix, const float* queries, int64_t nq, int32_t nprobe, int32_t metric,
                  int32_t* out_probe_ids, float* out_probe_scores, void* workspace, size_t workspace_bytes,
                  void* stream)
{
    if (int rc = check_index(ix)) return rc;
    if (int rc = check_batch(ix, nq, nprobe, 1, metric, false)) return rc;
    if (nq == 0) return HR_OK;
    if (!queries || !out_probe_ids) return fail(HR_ERR_ARG, "queries / out_probe_ids is null");
    const Plan p = make_plan(ix, nq, nprobe, 1);
    if (int rc = check_ws(p, workspace, workspace_bytes)) return rc;
    char* ws = (char*)workspace;
    hipStream_t s = (hipStream_t)stream;
    if (int rc = enqueue_prep(ix, p, ws, queries, nq, true, false, s)) return rc;
    return enqueue_coarse(ix, p, ws, nq, nprobe, metric, out_probe_ids, out_probe_scores, s);
}

int hr_ivf_scan(const hr_ivf_index* ix, const float* queries, int64_t nq, const int32_t* probe_ids,
                int32_t nprobe, int32_t k, int32_t metric, int64_t* out_ids, float* out_scores,
                void* workspace, size_t workspace_bytes, void* stream)
{
    if (int rc = check_index(ix)) return rc;
    if (nprobe < 1 || nprobe > HR_NPROBE_MAX) return fail(HR_ERR_ARG, "nprobe=%d must be in 1..%d", nprobe, HR_NPROBE_MAX);
    int np_plan = nprobe > ix->nlist ? (int)ix->nlist : nprobe;
    if (int rc = check_batch(ix, nq, np_plan, k, metric, true)) return rc;
    if (nq == 0) return HR_OK;
    if (!queries || !probe_ids || !out_ids || !out_scores) return fail(HR_ERR_ARG, "queries / probe_ids / outputs null");
    const Plan p = make_plan(ix, nq, nprobe, k);
    if (int rc = check_ws(p, workspace, workspace_bytes)) return rc;
    char* ws = (char*)workspace;
    hipStream_t s = (hipStream_t)stream;
    if (int rc = enqueue_prep(ix, p, ws, queries, nq, false, true, s)) return rc;
    return enqueue_scan(ix, p, ws, nq, probe_ids, nprobe, k, metric, out_ids, out_scores, s);
}

static int scan_step(const hr_ivf_index* ix, const float* queries, int64_t nq, const int32_t* probe_ids,
                     int32_t nprobe, int32_t k, int32_t metric, int64_t* io_ids, float* io_scores, int32_t* io_rows,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    if (int rc = check_index(ix)) return rc;
    if (nprobe < 1 || nprobe > HR_NPROBE_MAX) return fail(HR_ERR_ARG, "nprobe=%d must be in 1..%d", nprobe, HR_NPROBE_MAX);
    int np_plan = nprobe > ix->nlist ? (int)ix->nlist : nprobe;
    if (int rc = check_batch(ix, nq, np_plan, k, metric, true)) return rc;
    if (nq == 0) return HR_OK;
    if (!queries || !probe_ids || !io_ids || !io_scores) return fail(HR_ERR_ARG, "queries / probe_ids / state null");
    const Plan p = make_plan(ix, nq, nprobe, k);
    if (int rc = check_ws(p, workspace, workspace_bytes)) return rc;
    char* ws = (char*)workspace;
    hipStream_t s = (hipStream_t)stream;
    if (int rc = enqueue_prep(ix, p, ws, queries, nq, false, true, s)) return rc;
    return enqueue_scan(ix, p, ws, nq, probe_ids, nprobe, k, metric, io_ids, io_scores, s, true, io_rows);
}

int hr_ivf_scan_step(const hr_ivf_index* ix, const float* queries, int64_t nq, const int32_t* probe_ids,
                     int32_t nprobe, int32_t k, int32_t metric, int64_t* io_ids, float* io_scores,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    return scan_step(ix, queries, nq, probe_ids, nprobe, k, metric, io_ids, io_scores, nullptr, workspace, workspace_bytes, stream);
}

int hr_ivf_scan_step_rows(const hr_ivf_index* ix, const float* queries, int64_t nq, const int32_t* probe_ids,
                          int32_t nprobe, int32_t k, int32_t metric, int64_t* io_ids, float* io_scores,
                          int32_t* io_rows, void* workspace, size_t workspace_bytes, void* stream)
{
    if (int rc = check_index(ix)) return rc;
    if (nq > 0 && !io_rows) return fail(HR_ERR_ARG, "io_rows is null");
    return scan_step(ix, queries, nq, probe_ids, nprobe, k, metric, io_ids, io_scores, io_rows, workspace, workspace_bytes, stream);
}

int hr_ivf_rescore(const hr_ivf_index* ix, const float* queries, int64_t nq, const int32_t* rows, int32_t m,
                   int32_t k, int32_t metric, int64_t* out_ids, float* out_scores, int32_t* out_rows, void* stream)
{
    if (int rc = check_index(ix)) return rc;
    if (nq < 0 || nq > (1 << 24)) return fail(HR_ERR_ARG, "nq=%lld out of range", (long long)nq);
    if (m < 1 || m > HR_K_MAX) return fail(HR_ERR_ARG, "m=%d must be in 1..%d", m, HR_K_MAX);
    if (k < 1 || k > HR_K_MAX) return fail(HR_ERR_ARG, "k=%d must be in 1..%d", k, HR_K_MAX);
    if (metric != HR_METRIC_IP && metric != HR_METRIC_L2) return fail(HR_ERR_ARG, "unknown metric %d", metric);
    if (nq == 0) return HR_OK;
    if (!queries || !rows || !out_ids || !out_scores || !out_rows) return fail(HR_ERR_ARG, "queries / rows / outputs null");
    HR_HIP(launch_rescore(queries, nq, ix->d, row_dtype(ix), row_table(ix), ix->d_row_norm, ix->ids, ix->N, rows, m, k,
                          metric == HR_METRIC_L2, out_ids, out_scores, out_rows, (hipStream_t)stream));
    return HR_OK;
}

int hr_ivf_lists_of_rows(const hr_ivf_index* ix, const int32_t* rows, int64_t n, int32_t* out_lists, void* stream)
{
    if (int rc = check_index(ix)) return rc;
    if (n < 0) return fail(HR_ERR_ARG, "n=%lld is negative", (long long)n);
    if (n == 0) return HR_OK;
    if (!rows || !out_lists) return fail(HR_ERR_ARG, "rows / out_lists null");
    HR_HIP(launch_lists_of_rows(rows, n, ix->d_list_off, (int)ix->nlist, out_lists, (hipStream_t)stream));
    return HR_OK;
}

int hr_ivf_reorder_probes(const int32_t* probe, int64_t nq, int32_t nprobe, const int32_t* prev, int32_t nprev,
                          const int32_t* hot, int32_t nhot, int32_t* out_probe, void* stream)
{
    if (nq < 0 || nq > (1 << 24)) return fail(HR_ERR_ARG, "nq=%lld out of range", (long long)nq);
    if (nprobe < 1 || nprobe > HR_NPROBE_MAX) return fail(HR_ERR_ARG, "nprobe=%d must be in 1..%d", nprobe, HR_NPROBE_MAX);
    if (nprev < 0 || nprev > HR_NPROBE_MAX) return fail(HR_ERR_ARG, "nprev=%d must be in 0..%d", nprev, HR_NPROBE_MAX);
    if (nhot < 0 || nhot > HR_K_MAX) return fail(HR_ERR_ARG, "nhot=%d must be in 0..%d", nhot, HR_K_MAX);
    if (nq == 0) return HR_OK;
    if (!probe || !out_probe) return fail(HR_ERR_ARG, "probe / out_probe null");
    if (probe == out_probe) return fail(HR_ERR_ARG, "out_probe must not be probe");
    HR_HIP(launch_reorder_probes(probe, nprobe, nprev > 0 ? prev : nullptr, nprev, nhot > 0 ? hot : nullptr, nhot, nq,
                                 out_probe, (hipStream_t)stream));
    return HR_OK;
}

int hr_ivf_list_hits(const hr_ivf_index* ix, int64_t* out_hits, int32_t reset, void* stream)
{
    if (int rc = check_index(ix)) return rc;
    if (!out_hits) return fail(HR_ERR_ARG, "out_hits is null");
    HR_HIP(launch_read_hits(ix->d_hits, ix->nlist, out_hits, reset != 0, (hipStream_t)stream));
    return HR_OK;
}

int hr_ivf_hot_lists(const hr_ivf_index* ix, int32_t gc, int32_t* out_lists, void* stream)
{
    if (int rc = check_index(ix)) return rc;
    if (gc < 1 || gc > ix->nlist) return fail(HR_ERR_ARG, "gc=%d must be in 1..nlist=%lld", gc, (long long)ix->nlist);
    if (ix->nlist > 65536) return fail(HR_ERR_UNSUPPORTED, "hr_ivf_hot_lists ranks by counting: nlist=%lld > 65536", (long long)ix->nlist);
    if (!out_lists) return fail(HR_ERR_ARG, "out_lists is null");
    HR_HIP(launch_hot_lists(ix->d_hits, (int)ix->nlist, gc, out_lists, (hipStream_t)stream));
    return HR_OK;
}

int hr_ivf_set_resident(hr_ivf_index* ix, const int32_t* lists, int64_t n, int32_t resident, void* stream)
{
    if (int rc = check_index(ix)) return rc;
    if (n < 0) return fail(HR_ERR_ARG, "n=%lld is negative", (long long)n);
    if (lists == nullptr) n = ix->nlist;                     // all lists
    HR_HIP(launch_set_resident(ix->d_resident, (int)ix->nlist, lists, n, resident != 0 ? 1 : 0, (hipStream_t)stream));
    return HR_OK;
}

int hr_ivf_split_probes(const hr_ivf_index* ix, const int32_t* probe_ids, int64_t nq, int32_t nprobe,
                        int32_t* out_resident, int32_t* out_missing, void* stream)
{
    if (int rc = check_index(ix)) return rc;
    if (nq < 0 || nq > (1 << 24)) return fail(HR_ERR_ARG, "nq=%lld out of range", (long long)nq);
    if (nprobe < 1 || nprobe > HR_NPROBE_MAX) return fail(HR_ERR_ARG, "nprobe=%d must be in 1..%d", nprobe, HR_NPROBE_MAX);
    if (nq == 0) return HR_OK;
    if (!probe_ids || !out_resident || !out_missing) return fail(HR_ERR_ARG, "probe_ids / outputs null");
    if (probe_ids == out_resident || probe_ids == out_missing || out_resident == out_missing)
        return fail(HR_ERR_ARG, "the three arrays must be distinct");
    HR_HIP(launch_split_probes(probe_ids, nq, nprobe, ix->d_resident, (int)ix->nlist, ix->d_hits, out_resident, out_missing,
                               (hipStream_t)stream));
    return HR_OK;
}

int hr_ivf_refresh_rows(hr_ivf_index* ix, int64_t row_begin, int64_t row_end, void* stream)
{
    if (int rc = check_index(ix)) return rc;
    if (row_begin < 0 || row_end < row_begin || row_end > ix->N)
        return fail(HR_ERR_ARG, "rows %lld..%lld outside 0..N=%lld", (long long)row_begin, (long long)row_end, (long long)ix->N);
    const int64_t n = row_end - row_begin;
    if (n == 0) return HR_OK;
    hipStream_t s = (hipStream_t)stream;
    const size_t esize = ix->dtype == HR_F32 ? 4 : 2;
    const char* rows = (const char*)ix->vectors + (size_t)row_begin * ix->d * esize;
    HR_HIP(launch_row_norms(rows, ix->dtype, n, ix->d, ix->d_row_norm + row_begin, s));
    if (ix->d_vec16) {
        // (the only case in which this call waits for the stream: a new value beyond binary16 cannot go into the
        // table, and a later search must not read an infinity there)
        HR_HIP(launch_bf16_to_f16(rows, n * ix->d, (char*)ix->d_vec16 + (size_t)row_begin * ix->d * 2, ix->d_flag, s));
        int over = 0;
        HR_HIP(hipMemcpyAsync(&over, ix->d_flag, sizeof(int), hipMemcpyDeviceToHost, s));
        HR_HIP(hipStreamSynchronize(s));
        if (over) {
            HR_HIP(hipMemsetAsync(ix->d_flag, 0, sizeof(int), s));
            return fail(HR_ERR_UNSUPPORTED, "a refreshed bfloat16 value exceeds 65504 and does not fit the binary16 row table: "
                                            "replace the rows again, or load the index without HR_LOAD_ROW_TABLES");
        }
    }
    if (ix->d_vec_hi)
        HR_HIP(launch_split_f32((const float*)rows, n * ix->d, (char*)ix->d_vec_hi + (size_t)row_begin * ix->d * 2,
                                (char*)ix->d_vec_lo + (size_t)row_begin * ix->d * 2, s));
    return HR_OK;
}

int hr_ivf_workspace_layout(const hr_ivf_index* ix, int64_t nq, int32_t nprobe, int32_t k, int64_t* out, int32_t cap,
                            int32_t* n)
{
    if (int rc = check_index(ix)) return rc;
    if (!out || !n || cap < 0) return fail(HR_ERR_ARG, "out / n is null");
    if (nprobe < 1 || nprobe > HR_NPROBE_MAX) return fail(HR_ERR_ARG, "nprobe=%d must be in 1..%d", nprobe, HR_NPROBE_MAX);
    if (int rc = check_batch(ix, nq, nprobe > ix->nlist ? (int)ix->nlist : nprobe, k, HR_METRIC_IP, true)) return rc;
    const Plan p = make_plan(ix, nq, nprobe, k);
    *n = p.nreg;
    for (int i = 0; i < p.nreg && i < cap; i++) { out[2 * i] = (int64_t)p.reg_off[i]; out[2 * i + 1] = (int64_t)p.reg_len[i]; }
    return HR_OK;
}

int hr_ivf_stats(const hr_ivf_index* ix, const void* workspace, size_t workspace_bytes, int64_t nq,
                 int32_t nprobe, int32_t k, int64_t out[4])
{
    if (int rc = check_index(ix)) return rc;
    if (!out) return fail(HR_ERR_ARG, "out is null");
    if (int rc = check_batch(ix, nq, nprobe > ix->nlist ? (int)ix->nlist : nprobe, k, HR_METRIC_IP, true)) return rc;
    const Plan p = make_plan(ix, nq, nprobe, k);
    if (int rc = check_ws(p, workspace, workspace_bytes)) return rc;
    int dyn[DYN_COUNT];
    HR_HIP(hipMemcpy(dyn, (const char*)workspace + p.o_zero + (size_t)ix->nlist * 4, sizeof dyn, hipMemcpyDeviceToHost));
    out[0] = dyn[DYN_ITEMS];
    out[1] = dyn[DYN_SEG_ROWS];
    out[2] = ((int64_t)(uint32_t)dyn[DYN_ROWS_HI] << 32) | (uint32_t)dyn[DYN_ROWS_LO];
    out[3] = dyn[DYN_PAIRS];
    return HR_OK;
}

}  // extern "C"
