// Small kernels around the list scan: query operand preparation, row norms, grouping of
// (query, list) probes by list, and the per-query merge of the scan's partial results.
#include <algorithm>
#include <type_traits>

#include "scan_kernel.h"

namespace hr {

// ------------------------------------------------------------------------------------------
__global__ void k_fill_i32(int* p, int64_t n, int v)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

hipError_t launch_fill_i32(int* p, int64_t n, int v, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_i32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n, v);
    return hipGetLastError();
}

// float32 -> binary16 hi + 2^11-scaled binary16 lo (the split the scan applies to float32 rows)
__global__ void k_split_f32(const float* x, int64_t n, _Float16* hi, _Float16* lo)
{
    // (grid-stride: a launch may not have 2^32 threads or more)
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const float v = x[i];
        const _Float16 h = (_Float16)v;
        hi[i] = h;
        lo[i] = (_Float16)((v - (float)h) * 2048.0f);
    }
}

// bfloat16 -> binary16 (exact for magnitudes from 2^-14 to 65504: 8 significant bits fit in 11;
// below that the result is rounded to a multiple of 2^-24; above, the flag is raised)
__global__ void k_bf16_to_f16(const uint16_t* x, int64_t n, _Float16* out, int* overflow)
{
    bool over = false;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
        const float v = __builtin_bit_cast(float, ((uint32_t)x[i]) << 16);
        over |= !(fabsf(v) <= 65504.0f);                       // (also for NaN)
        out[i] = (_Float16)v;
    }
    if (over) atomicOr(overflow, 1);
}

hipError_t launch_bf16_to_f16(const void* x, int64_t n, void* out, int* overflow, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_bf16_to_f16, dim3((unsigned)std::min<int64_t>((n + 255) / 256, 1 << 20)), dim3(256), 0, s, (const uint16_t*)x, n, (_Float16*)out, overflow);
    return hipGetLastError();
}

// Labels must be non-negative: a negative id marks an empty place in results and carried results.
__global__ void k_check_labels(const int64_t* ids, int64_t n, int* negative)
{
    bool neg = false;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) neg |= ids[i] < 0;
    if (neg) atomicOr(negative, 1);
}

hipError_t launch_check_labels(const int64_t* ids, int64_t n, int* negative, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_check_labels, dim3((unsigned)std::min<int64_t>((n + 255) / 256, 1 << 16)), dim3(256), 0, s, ids, n, negative);
    return hipGetLastError();
}

hipError_t launch_split_f32(const float* x, int64_t n, void* hi, void* lo, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_split_f32, dim3((unsigned)std::min<int64_t>((n + 255) / 256, 1 << 20)), dim3(256), 0, s, x, n, (_Float16*)hi, (_Float16*)lo);
    return hipGetLastError();
}

// Per-list access counters (how often each list was probed: the frequency a cache of hot
// clusters is driven by, Section 4.4 of the paper): copy out, optionally start again from zero.
__global__ void k_read_hits(unsigned long long* hits, int64_t n, int64_t* out, int reset)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    out[i] = (int64_t)(reset ? atomicExch(&hits[i], 0ull) : hits[i]);
}

hipError_t launch_read_hits(unsigned long long* hits, int64_t n, int64_t* out, int reset, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_read_hits, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, hits, n, out, reset);
    return hipGetLastError();
}

// Partial residency (Section 4.4 of the paper: only the most frequently accessed clusters are kept in GPU memory, the
// searches of the others are served elsewhere and the partial results merged).  A flag per list says whether its
// vectors are in place; the grouping of probes drops the probes of the other lists.
__global__ void k_set_resident(int* resident, int nlist, const int32_t* lists, int64_t n, int value)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    if (lists == nullptr) { resident[i] = value; return; }
    const int l = lists[i];
    if (l >= 0 && l < nlist) resident[l] = value;
}

hipError_t launch_set_resident(int* resident, int nlist, const int32_t* lists, int64_t n, int value, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_set_resident, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, resident, nlist, lists, n, value);
    return hipGetLastError();
}

// Every query's probe list split into the lists whose vectors are in place and the others, each part in the given
// order, the rest of both rows filled with -1 (entries outside 0..nlist-1 go to neither).  The lists of the second
// part are counted as accessed here: no scan will see them.  One wave per query.
__global__ __launch_bounds__(256) void k_split_probes(const int32_t* probe, int64_t nq, int np, const int* resident, int nlist,
                                                      unsigned long long* hits, int32_t* out_res, int32_t* out_mis)
{
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t q = (int64_t)blockIdx.x * 4 + wave;
    if (q >= nq) return;
    int nres = 0, nmis = 0;
    for (int i0 = 0; i0 < np; i0 += 64) {
        const int i = i0 + lane;
        const int l = i < np ? probe[q * np + i] : -1;
        const bool valid = l >= 0 && l < nlist;
        const bool here = valid && resident[l] != 0;
        const unsigned long long mr = __builtin_amdgcn_ballot_w64(here), mm = __builtin_amdgcn_ballot_w64(valid && !here);
        if (here) out_res[q * np + nres + lanes_below(mr)] = l;
        if (valid && !here) {
            out_mis[q * np + nmis + lanes_below(mm)] = l;
            if (hits != nullptr) atomicAdd(&hits[l], 1ull);
        }
        nres += __builtin_popcountll(mr);
        nmis += __builtin_popcountll(mm);
    }
    for (int i = nres + lane; i < np; i += 64) out_res[q * np + i] = -1;
    for (int i = nmis + lane; i < np; i += 64) out_mis[q * np + i] = -1;
}

hipError_t launch_split_probes(const int32_t* probe, int64_t nq, int np, const int* resident, int nlist, unsigned long long* hits,
                               int32_t* out_resident, int32_t* out_missing, hipStream_t s)
{
    if (nq <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_split_probes, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, s, probe, nq, np, resident, nlist, hits,
                       out_resident, out_missing);
    return hipGetLastError();
}

// The gc most frequently probed lists, most frequent first, equal counts by list number: the
// lists a cache of hot clusters would keep (Section 4.4).  Every list counts the lists that
// come before it (tiles of the counters pass through LDS); its rank is its place in the output.
__global__ __launch_bounds__(256) void k_hot_lists(const unsigned long long* hits, int nlist, int gc, int32_t* out)
{
    __shared__ unsigned long long s_h[256];
    const int l = blockIdx.x * 256 + threadIdx.x;
    const unsigned long long mine = l < nlist ? hits[l] : 0ull;
    int rank = 0;
    for (int j0 = 0; j0 < nlist; j0 += 256) {
        __syncthreads();
        s_h[threadIdx.x] = j0 + (int)threadIdx.x < nlist ? hits[j0 + threadIdx.x] : 0ull;
        __syncthreads();
        const int n = min(256, nlist - j0);
        for (int t = 0; t < n; t++) {
            const unsigned long long h = s_h[t];
            rank += (h > mine || (h == mine && j0 + t < l)) ? 1 : 0;
        }
    }
    if (l < nlist && rank < gc) out[rank] = l;
}

hipError_t launch_hot_lists(const unsigned long long* hits, int nlist, int gc, int32_t* out, hipStream_t s)
{
    hipLaunchKernelGGL(k_hot_lists, dim3((unsigned)((nlist + 255) / 256)), dim3(256), 0, s, hits, nlist, gc, out);
    return hipGetLastError();
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__device__ __forceinline__ uint16_t bf16_rne(float f)
{
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b)
{
    return __builtin_bit_cast(float, ((uint32_t)b) << 16);
}

// Squared norm of every stored row, float32 accumulation of the exact stored values; used by
// the squared-L2 metric in its expanded form |q|^2 + |x|^2 - 2 q.x.  One wave per row.
__global__ __launch_bounds__(256) void k_row_norms(const void* rows, int dtype, int64_t nrows, int d, float* out)
{
    int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= nrows) return;
    int lane = threadIdx.x & 63;
    float acc = 0.f;
    if (dtype == HR_F32) {
        const float* p = (const float*)rows + row * d;
        for (int i = lane; i < d; i += 64) acc += p[i] * p[i];
    } else if (dtype == HR_F16) {
        const _Float16* p = (const _Float16*)rows + row * d;
        for (int i = lane; i < d; i += 64) { float x = (float)p[i]; acc += x * x; }
    } else {
        const uint16_t* p = (const uint16_t*)rows + row * d;
        for (int i = lane; i < d; i += 64) { float x = bf16_to_f32(p[i]); acc += x * x; }
    }
    acc = wave_sum(acc);
    if (lane == 0) out[row] = acc;
}

hipError_t launch_row_norms(const void* rows, int dtype, int64_t nrows, int d, float* out, hipStream_t s)
{
    if (nrows <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_row_norms, dim3((unsigned)((nrows + 3) / 4)), dim3(256), 0, s, rows, dtype, nrows, d, out);
    return hipGetLastError();
}

// Query operands.  Coarse step and float32 storage: binary16 hi row and 2^11-scaled binary16
// lo row per query.  binary16 storage: the query rounded to binary16.  bfloat16 storage:
// bfloat16 hi and lo rows.  The squared norms are those of the operand actually multiplied,
// so that the expanded L2 form cancels consistently.  One wave per query.
// The same launch clears what a call needs cleared in its workspace (counters, histograms: zero; the per-query
// lower bounds: the key of -inf): one small launch less in front of every search.
__global__ __launch_bounds__(256) void k_prep_queries(const float* q, int64_t nq, int d, int dtype,
                                                      _Float16* qc, float* qnorm_c, void* qs, float* qnorm_s,
                                                      int* zero, int64_t n_zero, int* neg, int64_t n_neg, int neg_value)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_zero; i += (int64_t)gridDim.x * blockDim.x) zero[i] = 0;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_neg; i += (int64_t)gridDim.x * blockDim.x) neg[i] = neg_value;
    int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= nq) return;
    int lane = threadIdx.x & 63;
    const float* p = q + row * d;
    float n32 = 0.f, ns = 0.f;
    for (int i = lane; i < d; i += 64) {
        float x = p[i];
        n32 += x * x;
        if (qc) {
            _Float16 h = (_Float16)x;
            qc[(row * 2) * d + i] = h;
            qc[(row * 2 + 1) * d + i] = (_Float16)((x - (float)h) * 2048.0f);
        }
        if (qs) {
            if (dtype == HR_F16) {
                _Float16 h = (_Float16)x;
                ((_Float16*)qs)[row * d + i] = h;
                ns += (float)h * (float)h;
            } else if (dtype == HR_BF16) {
                uint16_t hi = bf16_rne(x);
                uint16_t lo = bf16_rne(x - bf16_to_f32(hi));
                ((uint16_t*)qs)[(row * 2) * d + i] = hi;
                ((uint16_t*)qs)[(row * 2 + 1) * d + i] = lo;
                float e = bf16_to_f32(hi) + bf16_to_f32(lo);
                ns += e * e;
            }
        }
    }
    n32 = wave_sum(n32);
    ns = wave_sum(ns);
    if (lane == 0) {
        if (qnorm_c) qnorm_c[row] = n32;
        if (qnorm_s) qnorm_s[row] = (dtype == HR_F32) ? n32 : ns;
    }
}

hipError_t launch_prep_queries(const float* q, int64_t nq, int d, int dtype, void* qop_coarse,
                               float* qnorm_coarse, void* qop_scan, float* qnorm_scan,
                               int* zero, int64_t n_zero, int* neg, int64_t n_neg, int neg_value, hipStream_t s)
{
    if (nq <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_prep_queries, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, s, q, nq, d, dtype,
                       (_Float16*)qop_coarse, qnorm_coarse, qop_scan, qnorm_scan, zero, n_zero, neg, n_neg, neg_value);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Grouping of the nq*nprobe (query, list) pairs by list (the cross-request grouping behind
// the variable-length cluster search interface, Section 5 of the paper).

// pair -> its position inside the list's bucket (order of arrival; results do not depend on it)
__global__ void k_bucket_count(BucketArgs a)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)a.nq * a.nprobe) return;
    int l = a.probe[i];
    const bool valid = l >= 0 && l < a.nlist;
    const bool here = valid && a.resident[l] != 0;
    // (a list whose vectors are not in place is not scanned; the probe still counts as an access)
    if (valid && !here && a.hits != nullptr) atomicAdd(&a.hits[l], 1ull);
    a.pair_entry[i] = here ? atomicAdd(&a.list_w[l], 1) : -1;
}

// Exclusive prefix sum over the 1024 threads of a workgroup (16 waves); total returned to all.
__device__ __forceinline__ int block_scan_1024(int v, int* s_wave /* [17] */, int& total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int incl = wave_prefix_sum(v);
    __syncthreads();                                   // (s_wave may still be read from the last call)
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int i = 0; i < 16; i++) { int x = s_wave[i]; s_wave[i] = run; run += x; }
        s_wave[16] = run;
    }
    __syncthreads();
    total = s_wave[16];
    return s_wave[wave] + incl - v;
}

__device__ __forceinline__ long long block_sum_1024(long long v, long long* s_wave /* [16] */)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) s_wave[threadIdx.x >> 6] = v;
    __syncthreads();
    long long t = 0;
    for (int i = 0; i < 16; i++) t += s_wave[i];
    return t;
}

// Work items and their order of execution.  Items are numbered list-major (segment-major,
// query tile minor inside a list).  The order of execution is given by eight queues, one per
// XCD: all query tiles of one (list, segment) go to the same queue, next to each other, so the
// workgroups that re-read that segment run on one XCD at about the same time and share it
// through that XCD's L2.  Inside a queue the segments are ordered in rounds.  The longest list
// has eight segments per round, in order: its segments are spread over the whole run, and the
// later ones start from the lower bounds that the earlier ones have published.  The segments
// of a shorter list are spread evenly over the same rounds from a start that depends on the
// list (a list of one segment lands in a round of its own choosing).  So every stretch of a
// queue holds the same mix of items that many queries share (long lists of popular clusters:
// bound by the matrix pipes) and items of a few queries (bound by the row stream from HBM), and
// the two kinds run side by side on the compute units of an XCD for the whole run; with all
// short lists in the first round the device streams rows with idle matrix pipes first and
// multiplies with an idle HBM afterwards.  (Within a round the order is that of arrival;
// results do not depend on the order.)
// (kRounds, the most rounds a queue has, is declared with the device scalars in common.h)

// segment s of the nseg segments of list l: queue and round (R rounds in use)
__device__ __forceinline__ int queue_of(int l, int s) { return (l + s) & 7; }
__device__ __forceinline__ int round_of(int l, int s, int nseg, int R)
{
    const unsigned u = ((unsigned)l * 2654435761u) >> 16;            // start of the list inside its first stretch, in 65536ths
    return (int)((((long long)s << 16) + u) * R / ((long long)nseg << 16));
}

// One workgroup: bucket offsets, rows per segment for this batch, first work item and first
// result slot of every list, and where every round of every queue starts.
// (PER > 0: every thread owns at most PER lists and reads their widths and lengths once, all loads in flight
// together, into registers; the passes below then run without touching memory again.  PER == 0: any number of
// lists per thread, read from memory in every pass.)
template <int PER>
__global__ __launch_bounds__(1024) void k_bucket_scan(BucketArgs a)
{
    __shared__ int s_wave[17];
    __shared__ long long s_lwave[16];
    __shared__ int s_maxseg;
    const int t = threadIdx.x;
    if (t == 0) s_maxseg = 0;
    const int per = (a.nlist + 1023) / 1024;
    const int l0 = min(a.nlist, t * per), l1 = min(a.nlist, l0 + per);
    constexpr int NR = PER > 0 ? PER : 1;
    constexpr int UN = NR;                              // loops over a thread's lists: unrolled when they sit in registers
    int wv[NR], lv[NR];
    if constexpr (PER > 0) {
#pragma unroll
        for (int i = 0; i < PER; i++) {
            const int l = min(l0 + i, a.nlist - 1);
            wv[i] = a.list_w[l];
            lv[i] = a.list_off[l + 1] - a.list_off[l];
        }
    }
    auto width = [&](int l) __attribute__((always_inline)) -> int {
        if constexpr (PER > 0) {
            int r = 0;
#pragma unroll
            for (int i = 0; i < PER; i++) r = (l - l0 == i) ? wv[i] : r;
            return r;
        } else {
            return a.list_w[l];
        }
    };
    auto length = [&](int l) __attribute__((always_inline)) -> int {
        if constexpr (PER > 0) {
            int r = 0;
#pragma unroll
            for (int i = 0; i < PER; i++) r = (l - l0 == i) ? lv[i] : r;
            return r;
        } else {
            return a.list_off[l + 1] - a.list_off[l];
        }
    };

    // pass 1: bucket offsets, cost = sum rows * query tiles, rows streamed, pairs
    int w_sum = 0;
    long long cost = 0, rows = 0;
#pragma unroll UN
    for (int i = 0; i < (PER > 0 ? PER : per); i++) {
        const int l = l0 + i;
        if (l >= l1) break;
        int w = width(l);
        long long len = length(l);
        if (a.hits != nullptr && w > 0) atomicAdd(&a.hits[l], (unsigned long long)w);     // access frequency of the list
        w_sum += w;
        cost += len * ((w + a.cw - 1) / a.cw);
        if (w > 0) rows += len;
    }
    int total;
    {
        int run = block_scan_1024(w_sum, s_wave, total);
#pragma unroll UN
        for (int i = 0; i < (PER > 0 ? PER : per); i++) {
            const int l = l0 + i;
            if (l >= l1) break;
            a.bucket_off[l] = run; run += width(l);
        }
        if (t == 0) { a.bucket_off[a.nlist] = total; a.dyn[DYN_PAIRS] = total; }
    }
    const long long c = block_sum_1024(cost, s_lwave);
    // rows per segment: about item_target items at most; and, since every item costs some ten
    // microseconds whatever its size, segments of up to 1024 rows as long as that leaves 1024 items
    // (one million rows in 1024 lists: 1024 items of 1024 rows, 0.60 ms; 4096 items of 256 rows, 0.65 ms)
    long long segll = (c + a.item_target - 1) / a.item_target;
    const long long fewer = c / 1024 < 1024 ? c / 1024 : 1024;
    if (segll < fewer) segll = fewer;
    segll = (segll + 15) & ~15LL;
    if (segll < kMinSegRows) segll = kMinSegRows;
    if (segll > 0x7ffffff0LL) segll = 0x7ffffff0LL;          // (a list has fewer than 2^31 rows: one segment then)
    const int seg = (int)segll;
    const long long r = block_sum_1024(rows, s_lwave);
    if (t == 0) {
        a.dyn[DYN_SEG_ROWS] = seg;
        a.dyn[DYN_ROWS_LO] = (int)(r & 0xffffffffLL);
        a.dyn[DYN_ROWS_HI] = (int)(r >> 32);
    }

    // pass 2: work items per list = segments * query tiles; result slots per list = segments * bucket width
    // (one slot per (segment, query of the bucket): slot of entry e of segment s = slot_base[l] + s * w + e)
    auto list_items = [&](int l, int& nseg, int& nqt) __attribute__((always_inline)) {
        const int w = width(l);
        const int len = length(l);
        nseg = (w > 0 && len > 0) ? (len + seg - 1) / seg : 0;
        nqt = (w + a.cw - 1) / a.cw;
    };
    int items = 0, slots = 0, maxseg = 0;
#pragma unroll UN
    for (int i = 0; i < (PER > 0 ? PER : per); i++) {
        const int l = l0 + i;
        if (l >= l1) break;
        int nseg, nqt; list_items(l, nseg, nqt);
        items += nseg * nqt; slots += nseg * width(l); maxseg = max(maxseg, nseg);
    }
    if (maxseg > 0) atomicMax(&s_maxseg, maxseg);
    {
        int run = block_scan_1024(items, s_wave, total);
#pragma unroll UN
        for (int i = 0; i < (PER > 0 ? PER : per); i++) {
            const int l = l0 + i;
            if (l >= l1) break;
            a.item_base[l] = run;
            int nseg, nqt; list_items(l, nseg, nqt);
            run += nseg * nqt;
        }
        if (t == 0) {
            a.item_base[a.nlist] = total;
            // never more than the table holds (cannot happen: the host sizes it from the same bound)
            a.dyn[DYN_ITEMS] = min(total, a.item_cap);
        }
    }
    {
        int run = block_scan_1024(slots, s_wave, total);
#pragma unroll UN
        for (int i = 0; i < (PER > 0 ? PER : per); i++) {
            const int l = l0 + i;
            if (l >= l1) break;
            a.slot_base[l] = run;
            int nseg, nqt; list_items(l, nseg, nqt);
            run += nseg * width(l);
        }
        if (t == 0) {
            a.slot_base[a.nlist] = total;
            a.dyn[DYN_SLOTS] = total;
        }
    }
    // rounds of the queues: the longest list has eight segments per round
    if (t == 0) a.dyn[DYN_ROUNDS] = max(1, min(kRounds, (s_maxseg + 7) / 8));
}

__global__ void k_bucket_scatter(BucketArgs a)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)a.nq * a.nprobe) return;
    int e = a.pair_entry[i];
    if (e < 0) return;
    int l = a.probe[i];
    a.bucket_q[a.bucket_off[l] + e] = (int)(i / a.nprobe);
}

// items per queue and round (one wave per list, its segments over the lanes)
__global__ __launch_bounds__(256) void k_round_count(BucketArgs a)
{
    int l = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (l >= a.nlist) return;
    int lane = threadIdx.x & 63;
    int w = a.list_w[l];
    int len = a.list_off[l + 1] - a.list_off[l];
    if (w <= 0 || len <= 0) return;
    int seg = a.dyn[DYN_SEG_ROWS];
    int nqt = (w + a.cw - 1) / a.cw;
    int nseg = (len + seg - 1) / seg;
    const int R = a.dyn[DYN_ROUNDS];
    for (int s = lane; s < nseg; s += 64) atomicAdd(&a.round_cnt[queue_of(l, s) * kRounds + round_of(l, s, nseg, R)], nqt);
}

// (every workgroup turns the 8 x kRounds counts into where every round starts in its queue, for itself; the
// first one also writes the queue lengths)
__global__ __launch_bounds__(256) void k_item_expand(BucketArgs a)
{
    __shared__ int s_start[8 * kRounds];
    for (int i = threadIdx.x; i < 8 * kRounds; i += 256) s_start[i] = a.round_cnt[i];
    __syncthreads();
    if (threadIdx.x < 8) {
        int run = 0;
        for (int r = 0; r < kRounds; r++) { const int c = s_start[threadIdx.x * kRounds + r]; s_start[threadIdx.x * kRounds + r] = run; run += c; }
        if (blockIdx.x == 0) a.xq_count[threadIdx.x] = min(run, a.item_cap);
    }
    __syncthreads();
    int l = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (l >= a.nlist) return;
    int lane = threadIdx.x & 63;
    int w = a.list_w[l];
    int len = a.list_off[l + 1] - a.list_off[l];
    if (w <= 0 || len <= 0) return;
    int seg = a.dyn[DYN_SEG_ROWS];
    int nqt = (w + a.cw - 1) / a.cw;
    int nseg = (len + seg - 1) / seg;
    long long base = a.item_base[l];
    const long long sbase = a.slot_base[l];
    const int R = a.dyn[DYN_ROUNDS];
    const int row_first = a.list_off[l], boff = a.bucket_off[l];
    for (int s = lane; s < nseg; s += 64) {
        const int x = queue_of(l, s), slot = x * kRounds + round_of(l, s, nseg, R);
        const int pos = s_start[slot] + atomicAdd(&a.round_cur[slot], nqt);
        const int row0 = row_first + s * seg;
        const int nrows = min(len - s * seg, seg);
        for (int t = 0; t < nqt; t++) {
            long long idx = base + (long long)s * nqt + t;
            // first result slot of the item: entries t*cw .. of segment s (the last tile of a bucket has fewer
            // than cw entries; what lies behind them belongs to the next segment and is never touched)
            const long long first = sbase + (long long)s * w + (long long)t * a.cw;
            // (the guards cannot fail: the host sizes the tables from the same bounds)
            if (idx < a.item_cap && pos + t < a.item_cap && first + min(a.cw, w - t * a.cw) <= a.slot_cap) {
                int4* rec = a.xq_rec + ((size_t)x * a.item_cap + pos + t) * 2;
                rec[0] = make_int4(row0, nrows, boff, w);
                rec[1] = make_int4(t, (int)first, l, s);
            }
        }
    }
}

hipError_t launch_bucketing(const BucketArgs& a, hipStream_t s)
{
    int64_t pairs = (int64_t)a.nq * a.nprobe;
    unsigned gp = (unsigned)((pairs + 255) / 256);
    hipLaunchKernelGGL(k_bucket_count, dim3(gp), dim3(256), 0, s, a);
    const int per = (a.nlist + 1023) / 1024;
    if (per <= 4) hipLaunchKernelGGL(k_bucket_scan<4>, dim3(1), dim3(1024), 0, s, a);
    else if (per <= 16) hipLaunchKernelGGL(k_bucket_scan<16>, dim3(1), dim3(1024), 0, s, a);
    else hipLaunchKernelGGL(k_bucket_scan<0>, dim3(1), dim3(1024), 0, s, a);
    hipLaunchKernelGGL(k_bucket_scatter, dim3(gp), dim3(256), 0, s, a);
    hipLaunchKernelGGL(k_round_count, dim3((unsigned)((a.nlist + 3) / 4)), dim3(256), 0, s, a);
    hipLaunchKernelGGL(k_item_expand, dim3((unsigned)((a.nlist + 3) / 4)), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Per-query merge of the scan's partial results (the reduction step of the cluster search of
// Section 5 and the per-request merge of Section 4.4): one wave per query walks the slots that hold its
// candidates, keeps the k best in an LDS buffer pruned as in the scan, then orders the
// survivors by (key, label) and writes the output row.
// Key (larger is better) of an entry of a carried result, from its reported score: the score
// itself for the inner product; |q|^2 - distance for squared L2 (the inverse of what the merge
// reports, up to rounding).
__device__ __forceinline__ float key_of_score(float score, float qn, int l2) { return l2 ? qn - score : score; }

// Carried results as starting lower bounds: a query whose carried result is full starts the
// scan at the key of its worst entry (minus a margin for the rounding of the line above).
__global__ void k_state_thr(const int64_t* ids, const float* scores, const float* qnorm, int64_t nq, int k, int l2,
                            uint32_t* thr)
{
    int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= nq) return;
    if (ids[q * k + k - 1] < 0) return;                      // (best first, empty places last)
    const float sc = scores[q * k + k - 1];
    const float qn = l2 ? qnorm[q] : 0.f;
    const float key = key_of_score(sc, qn, l2);
    const float margin = l2 ? 4.0e-7f * fmaxf(fabsf(qn), fabsf(sc)) : 0.f;
    atomicMax(&thr[q], enc_key(key - margin));
}

hipError_t launch_state_thr(const int64_t* ids, const float* scores, const float* qnorm, int64_t nq, int k, int l2,
                            uint32_t* thr, hipStream_t s)
{
    if (nq <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_state_thr, dim3((unsigned)((nq + 255) / 256)), dim3(256), 0, s, ids, scores, qnorm, nq, k, l2, thr);
    return hipGetLastError();
}

constexpr int kMergeCap = 256;     // candidates buffered per query (k <= 128, up to 64 appended per step)

__global__ __launch_bounds__(256) void k_merge(MergeArgs a)
{
    __shared__ Cand s_buf[4][kMergeCap];
    __shared__ int64_t s_tie[4][HR_K_MAX];
    __shared__ int s_pref[4][HR_NPROBE_MAX + 1];
    __shared__ int s_cnt[4];
    __shared__ int s_first[4][64];
    __shared__ size_t s_slot[4][64];
    __shared__ int64_t s_ext_id[4][HR_K_MAX];
    __shared__ float s_ext_score[4][HR_K_MAX];
    __shared__ int s_ext_row[4][HR_K_MAX];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t q = (int64_t)blockIdx.x * 4 + wave;
    if (q >= a.nq) return;                       // whole wave leaves; no block barrier below
    int64_t* ext_id = s_ext_id[wave];
    int* ext_row = s_ext_row[wave];              // rows of the carried entries (-1: empty place or rows not carried)
    float* ext_score = s_ext_score[wave];
    Cand* buf = s_buf[wave];
    int64_t* tie = s_tie[wave];
    int* pref = s_pref[wave];
    int* first = s_first[wave];
    size_t* slot_of = s_slot[wave];
    const int k = a.k;
    const int seg_rows = a.dyn[DYN_SEG_ROWS];

    // ---- how many segments (= slots) does each probed list contribute
    int total;
    {
        int run = 0;
        for (int p0 = 0; p0 < a.nprobe; p0 += 64) {
            int p = p0 + lane;
            int ns = 0;
            if (p < a.nprobe) {
                int l = a.probe[q * a.nprobe + p];
                if (l >= 0 && l < a.nlist && a.pair_entry[q * a.nprobe + p] >= 0) {
                    int len = a.list_off[l + 1] - a.list_off[l];
                    ns = (len + seg_rows - 1) / seg_rows;
                }
            }
            int inc = ns;                         // inclusive scan over the wave
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                int v = __shfl_up(inc, o);
                if (lane >= o) inc += v;
            }
            if (p < a.nprobe) pref[p + 1] = run + inc;
            run += __shfl(inc, 63);
        }
        if (lane == 0) pref[0] = 0;
        total = run;
    }
    if (lane == 0) s_cnt[wave] = 0;
    wave_sync();
    // ---- a carried result joins as one more partial result (read whole before anything of
    // this query is written: the same arrays take the merged result)
    const float qn0 = (a.l2 && a.qnorm) ? a.qnorm[q] : 0.f;
    if (a.carried) {
        for (int j0 = 0; j0 < k; j0 += 64) {
            const int j = j0 + lane;
            const int64_t id = j < k ? a.out_ids[(size_t)q * k + j] : -1;
            const bool have = id >= 0;
            const unsigned long long m = __builtin_amdgcn_ballot_w64(have);
            if (j < k) ext_row[j] = (have && a.io_rows) ? a.io_rows[(size_t)q * k + j] : -1;
            if (have) {
                const float sc = a.out_scores[(size_t)q * k + j];
                ext_id[j] = id;
                ext_score[j] = sc;
                buf[s_cnt[wave] + lanes_below(m)] = Cand{enc_key(key_of_score(sc, qn0, a.l2)), kCarried | (uint32_t)j};
            }
            wave_sync();
            if (lane == 0) s_cnt[wave] += __builtin_popcountll(m);
            wave_sync();
        }
    }

    uint32_t thr = 0;                              // below every encoded key
    for (int f0 = 0; f0 < total; f0 += 64) {
        const int f = f0 + lane;
        int c = 0;
        size_t slot = 0;
        if (f < total) {
            {
                int lo = 0, hi = a.nprobe;        // largest p with pref[p] <= f
                while (hi - lo > 1) {
                    int mid = (lo + hi) >> 1;
                    if (pref[mid] <= f) lo = mid; else hi = mid;
                }
                int p = lo;
                int s = f - pref[p];
                int l = a.probe[q * a.nprobe + p];
                int e = a.pair_entry[q * a.nprobe + p];
                int w = a.bucket_off[l + 1] - a.bucket_off[l];
                slot = (size_t)a.slot_base[l] + (size_t)s * w + (size_t)e;
            }
            c = a.slot_cnt[slot];
        }
        // the entries of these 64 slots, 64 at a time whichever slot they sit in (a loop over the fullest slot's
        // entries would be one round trip to memory per entry: the slot of a query's own cluster holds up to k)
        int inc = c;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            int v = __shfl_up(inc, o);
            if (lane >= o) inc += v;
        }
        const int tot = __shfl(inc, 63);
        first[lane] = inc - c;
        slot_of[lane] = slot;
        wave_sync();
        for (int e0 = 0; e0 < tot; e0 += 64) {
            const int e = e0 + lane;
            if (e < tot) {
                int lo = 0, hi = 64;                  // largest lane o with first[o] <= e: the slot that holds entry e
                while (hi - lo > 1) {
                    int mid = (lo + hi) >> 1;
                    if (first[mid] <= e) lo = mid; else hi = mid;
                }
                Cand cd = a.slot_ent[slot_of[lo] * a.slot_stride + (e - first[lo])];
                bool take = cd.key >= thr;
                // a row the carried result already holds (it came from a cache of earlier results
                // and its list is scanned now) is not taken a second time
                if (take && a.io_rows && a.carried)
                    for (int t = 0; t < k; t++) take = take && ext_row[t] != (int)cd.row;
                if (take) {
                    int pos = atomicAdd(&s_cnt[wave], 1);
                    buf[pos] = cd;
                }
            }
            wave_sync();
            int n = __builtin_amdgcn_readfirstlane(s_cnt[wave]);
            if (n > kMergeCap - 64) {
                uint32_t kth = wave_select<4>(buf, n, k, a.row_ids, ext_id);
                thr = kth > thr ? kth : thr;
                if (lane == 0) s_cnt[wave] = k;
                wave_sync();
            }
        }
        wave_sync();
    }
    wave_sync();
    int n = __builtin_amdgcn_readfirstlane(s_cnt[wave]);
    if (n > k) {
        wave_select<4>(buf, n, k, a.row_ids, ext_id);
        n = k;
    }
    wave_sync();

    // ---- final order by (key descending, label ascending); n <= k <= 128: two entries per lane
    Cand e[2];
    int64_t id[2];
#pragma unroll
    for (int m = 0; m < 2; m++) {
        int idx = lane + 64 * m;
        e[m] = (idx < n) ? buf[idx] : Cand{0u, 0u};
        id[m] = (idx < n) ? label_of(e[m].row, a.row_ids, ext_id) : INT64_MAX;
        if (idx < n) tie[idx] = id[m];
    }
    wave_sync();
    int pos[2] = {0, 0};
    for (int i = 0; i < n; i++) {
        uint32_t so = buf[i].key;
        int64_t oid = tie[i];
#pragma unroll
        for (int m = 0; m < 2; m++)
            pos[m] += (so > e[m].key || (so == e[m].key && oid < id[m])) ? 1 : 0;
    }
    const float qn = (a.l2 && a.qnorm) ? a.qnorm[q] : 0.f;
#pragma unroll
    for (int m = 0; m < 2; m++) {
        int idx = lane + 64 * m;
        if (idx < n) {
            float key = dec_key(e[m].key);
            float score = a.l2 ? fmaxf(qn - key, 0.f) : key;
            if (e[m].row & kCarried) score = ext_score[e[m].row & ~kCarried];     // (as it was reported)
            size_t o = (size_t)q * k + pos[m];
            if (a.out_ids) a.out_ids[o] = id[m];
            if (a.out_scores) a.out_scores[o] = score;
            if (a.io_rows) a.io_rows[o] = (e[m].row & kCarried) ? ext_row[e[m].row & ~kCarried] : (int)e[m].row;
        }
    }
    for (int idx = n + lane; idx < k; idx += 64) {     // fewer than k candidates: pad
        size_t o = (size_t)q * k + idx;
        if (a.out_ids) a.out_ids[o] = -1;
        if (a.out_scores) a.out_scores[o] = a.l2 ? __builtin_inff() : -__builtin_inff();
        if (a.io_rows) a.io_rows[o] = -1;
    }
}

// ------------------------------------------------------------------------------------------
// Top-k of one row of keys per wave (coarse step: the nprobe best centroids of a query out of
// the nlist keys the dense scan wrote; Section 2.2: the closest clusters are the ones probed).
// Exact: radix select on the order-preserving 32-bit image of the key, one 8-bit digit per pass
// with a 256-bin histogram in LDS, then the entries above the k-th key and, of those equal to
// it, the ones with the lowest index, ordered best first (equal keys: lower index first).
struct TopkArgs {
    const float* keys;          // [nq, n] larger is better
    const float* qnorm;         // [nq] squared query norms (L2 only)
    int32_t* out_ids;           // [nq, k]
    float* out_scores;          // [nq, k] or nullptr
    int nq, n, k, l2;
};

__global__ __launch_bounds__(256) void k_topk_rows(TopkArgs a)
{
    constexpr int kCollect = 1024;                  // entries one wave can collect in LDS (>= HR_NPROBE_MAX)
    __shared__ int s_hist[4][256];
    __shared__ Cand s_ent[4][kCollect];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int64_t q = (int64_t)blockIdx.x * 4 + wave;
    if (q >= a.nq) return;
    const float* row = a.keys + (size_t)q * a.n;
    int* hist = s_hist[wave];
    Cand* ent = s_ent[wave];
    const int k = min(a.k, a.n);

    // ---- the quick way, one pass over the row: a lower bound t0 from 512 keys spread over the
    // row (their m-th largest, m chosen so that about 3k keys of the row are expected above
    // it), every key >= t0 collected in LDS, the k best of those selected there.  It is exact
    // whenever at least k and at most kCollect keys were collected (all keys >= the k-th best
    // are then among them); otherwise the radix passes below do the work.
    bool done = false;
    {
        uint32_t t0 = 0;                            // (below every encoded key: short rows are collected whole)
        if (a.n > kCollect) {
            constexpr int S = 512;
            uint32_t sv[S / 64];
#pragma unroll
            for (int j = 0; j < S / 64; j++) sv[j] = enc_key(row[(int)(((long long)(j * 64 + lane) * a.n) / S)]);
            int want = (int)((3LL * k * S + a.n - 1) / a.n);
            want = max(2, min(S, want));
            unsigned long long alive[S / 64];
#pragma unroll
            for (int j = 0; j < S / 64; j++) alive[j] = ~0ull;
            for (int b = 31; b >= 0; b--) {
                unsigned long long ones[S / 64];
                int c1 = 0;
#pragma unroll
                for (int j = 0; j < S / 64; j++) {
                    ones[j] = alive[j] & __builtin_amdgcn_ballot_w64((sv[j] >> b) & 1u);
                    c1 += __builtin_popcountll(ones[j]);
                }
                if (c1 >= want) {
                    t0 |= 1u << b;
#pragma unroll
                    for (int j = 0; j < S / 64; j++) alive[j] = ones[j];
                } else {
                    want -= c1;
#pragma unroll
                    for (int j = 0; j < S / 64; j++) alive[j] &= ~ones[j];
                }
            }
        }
        int cnt = 0;
        auto collect = [&](float key, int i, bool valid) __attribute__((always_inline)) {
            const uint32_t u = enc_key(key);
            const bool take = valid && u >= t0;
            const unsigned long long m = __builtin_amdgcn_ballot_w64(take);
            if (m == 0) return;
            const int pos = cnt + lanes_below(m);
            if (take && pos < kCollect) ent[pos] = Cand{u, (uint32_t)i};
            cnt += __builtin_popcountll(m);
        };
        // (what hides the latency of the loads is how many are in flight: 8 of 16 bytes per
        // lane when the rows allow it; the order of collection does not matter)
        if ((a.n & 3) == 0) {
            const float4* row4 = (const float4*)row;
            const int n4 = a.n >> 2;
            for (int i0 = 0; i0 < n4; i0 += 64 * 8) {
                float4 v[8];
#pragma unroll
                for (int j = 0; j < 8; j++) v[j] = row4[min(i0 + j * 64 + lane, n4 - 1)];
#pragma unroll
                for (int j = 0; j < 8; j++) {
                    const int i4 = i0 + j * 64 + lane;
                    collect(v[j].x, i4 * 4, i4 < n4);
                    collect(v[j].y, i4 * 4 + 1, i4 < n4);
                    collect(v[j].z, i4 * 4 + 2, i4 < n4);
                    collect(v[j].w, i4 * 4 + 3, i4 < n4);
                }
            }
        } else {
            for (int i0 = 0; i0 < a.n; i0 += 64 * 8) {
                float v[8];
#pragma unroll
                for (int j = 0; j < 8; j++) { const int i = i0 + j * 64 + lane; v[j] = row[min(i, a.n - 1)]; }
#pragma unroll
                for (int j = 0; j < 8; j++) collect(v[j], i0 + j * 64 + lane, i0 + j * 64 + lane < a.n);
            }
        }
        wave_sync();
        if (cnt >= k && cnt <= kCollect) {
            // (equal keys: lower index first; the select walks as many 64-entry chunks as were collected, not
            // as many as the buffer holds)
            if (cnt > k) {
                if (cnt <= 256) wave_select<4>(ent, cnt, k, nullptr);
                else if (cnt <= 512) wave_select<8>(ent, cnt, k, nullptr);
                else wave_select<kCollect / 64>(ent, cnt, k, nullptr);
            }
            done = true;
        }
    }

    uint32_t prefix = 0, mask = 0;
    int need = k;                                   // entries still to take among those matching the prefix
    for (int shift = 24; shift >= 0 && !done; shift -= 8) {
#pragma unroll
        for (int j = 0; j < 4; j++) hist[lane * 4 + j] = 0;
        wave_sync();
        // (8 loads in flight per lane: the row is read once per pass and nothing else hides
        // the latency of a load)
        for (int i0 = 0; i0 < a.n; i0 += 64 * 8) {
            float v[8];
#pragma unroll
            for (int j = 0; j < 8; j++) { const int i = i0 + j * 64 + lane; v[j] = row[min(i, a.n - 1)]; }
#pragma unroll
            for (int j = 0; j < 8; j++) {
                const uint32_t u = enc_key(v[j]);
                const bool in = i0 + j * 64 + lane < a.n && (u & mask) == prefix;
                const int dg = (u >> shift) & 255;
                // keys of one row mostly share their leading digits: the lanes whose digit is
                // that of the first counted lane are added in one go, only the others one by
                // one (64 atomic additions to one LDS word would go one after the other)
                const unsigned long long min_ = __builtin_amdgcn_ballot_w64(in);
                if (min_ == 0) continue;
                const int d0 = __builtin_amdgcn_readlane(dg, __builtin_ctzll(min_));
                const unsigned long long same = __builtin_amdgcn_ballot_w64(in && dg == d0);
                if (lane == 0) atomicAdd(&hist[d0], (int)__builtin_popcountll(same));
                if (in && dg != d0) atomicAdd(&hist[dg], 1);
            }
        }
        wave_sync();
        // lane L holds digits 255-4L .. 252-4L: the prefix sum over lanes counts from the top digit down
        int c[4], tot = 0;
#pragma unroll
        for (int j = 0; j < 4; j++) { c[j] = hist[255 - (lane * 4 + j)]; tot += c[j]; }
        const int incl = wave_prefix_sum(tot);
        const unsigned long long reach = __builtin_amdgcn_ballot_w64(incl >= need);
        const int L = __builtin_ctzll(reach);       // (need <= number of matching entries, so some lane reaches it)
        int digit = 0, above = 0;
        if (lane == L) {
            int run = incl - tot;
#pragma unroll
            for (int j = 0; j < 4; j++) {
                if (run < need && run + c[j] >= need) { digit = 255 - (lane * 4 + j); above = run; }
                run += c[j];
            }
        }
        digit = __builtin_amdgcn_readlane(digit, L);
        above = __builtin_amdgcn_readlane(above, L);
        need -= above;
        prefix |= (uint32_t)digit << shift;
        mask |= 255u << shift;
        wave_sync();
    }
    // prefix = k-th best key; `need` of the entries equal to it are taken, lowest index first
    int n_gt = 0, n_eq = 0;
    for (int i0 = 0; i0 < a.n && !done; i0 += 64 * 8) {
        float v[8];
#pragma unroll
        for (int j = 0; j < 8; j++) { const int i = i0 + j * 64 + lane; v[j] = row[min(i, a.n - 1)]; }
#pragma unroll
        for (int j = 0; j < 8; j++) {
            const int i = i0 + j * 64 + lane;
            const uint32_t u = enc_key(v[j]);
            const bool gt = i < a.n && u > prefix;
            const bool eq = i < a.n && u == prefix;
            const unsigned long long mg = __builtin_amdgcn_ballot_w64(gt), me = __builtin_amdgcn_ballot_w64(eq);
            if (gt) ent[n_gt + lanes_below(mg)] = Cand{u, (uint32_t)i};
            n_gt += __builtin_popcountll(mg);
            // the equal ones go to the far end, in index order, until enough are taken
            const int r = n_eq + lanes_below(me);
            if (eq && r < need) ent[k - 1 - r] = Cand{u, (uint32_t)i};
            n_eq += __builtin_popcountll(me);
        }
    }
    wave_sync();
    // order: key descending, index ascending (rank of every entry = entries ahead of it)
    const float qn = (a.l2 && a.qnorm) ? a.qnorm[q] : 0.f;
    auto emit = [&](auto per) __attribute__((always_inline)) {
        constexpr int PER = decltype(per)::value;       // entries per lane
        Cand e[PER];
        int pos[PER];
#pragma unroll
        for (int m = 0; m < PER; m++) { e[m] = lane + 64 * m < k ? ent[lane + 64 * m] : Cand{0u, 0u}; pos[m] = 0; }
        for (int i = 0; i < k; i++) {
            const Cand o = ent[i];
#pragma unroll
            for (int m = 0; m < PER; m++) pos[m] += (o.key > e[m].key || (o.key == e[m].key && o.row < e[m].row)) ? 1 : 0;
        }
#pragma unroll
        for (int m = 0; m < PER; m++) {
            if (lane + 64 * m < k) {
                const float key = dec_key(e[m].key);
                const size_t o = (size_t)q * a.k + pos[m];
                a.out_ids[o] = (int32_t)e[m].row;
                if (a.out_scores) a.out_scores[o] = a.l2 ? fmaxf(qn - key, 0.f) : key;
            }
        }
    };
    if (k <= 64) emit(std::integral_constant<int, 1>{});
    else if (k <= 128) emit(std::integral_constant<int, 2>{});
    else if (k <= 256) emit(std::integral_constant<int, 4>{});
    else emit(std::integral_constant<int, HR_NPROBE_MAX / 64>{});
    for (int idx = k + lane; idx < a.k; idx += 64) {       // fewer than k rows: pad
        const size_t o = (size_t)q * a.k + idx;
        a.out_ids[o] = -1;
        if (a.out_scores) a.out_scores[o] = a.l2 ? __builtin_inff() : -__builtin_inff();
    }
}

hipError_t launch_topk_rows(const float* keys, const float* qnorm, int32_t* out_ids, float* out_scores,
                            int64_t nq, int n, int k, int l2, hipStream_t s)
{
    if (nq <= 0) return hipSuccess;
    TopkArgs a{keys, qnorm, out_ids, out_scores, (int)nq, n, k, l2};
    hipLaunchKernelGGL(k_topk_rows, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------
// Reuse of the previous retrieval of a request (Section 4.3 of the paper: consecutive queries
// v, v' of a request are close, so the results of v' tend to lie among a larger top-k of v, in
// the clusters H_v that held v's results, and in clusters probed both times).

// List of every given row (binary search in the row offsets); -1 for rows outside the index.
__global__ void k_lists_of_rows(const int32_t* rows, int64_t n, const int* list_off, int nlist, int32_t* out)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int r = rows[i];
    int res = -1;
    if (r >= 0 && r < list_off[nlist]) {
        int lo = 0, hi = nlist;                 // largest l with list_off[l] <= r (lists may be empty)
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (list_off[mid] <= r) lo = mid; else hi = mid;
        }
        res = lo;
    }
    out[i] = res;
}

hipError_t launch_lists_of_rows(const int32_t* rows, int64_t n, const int* list_off, int nlist, int32_t* out, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_lists_of_rows, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, rows, n, list_off, nlist, out);
    return hipGetLastError();
}

// Search order of the new probe lists C' of every query: first those in H_v, then those of
// the previous probe lists C that are not in H_v, then the rest, each group in its given
// (rank) order; absent entries (-1) last.  One wave per query.
struct ReorderArgs {
    const int32_t* probe;       // [nq, np]
    const int32_t* prev;        // [nq, pp] or nullptr
    const int32_t* hot;         // [nq, nh] or nullptr
    int32_t* out;               // [nq, np]
    int nq, np, pp, nh;
};

__global__ __launch_bounds__(256) void k_reorder_probes(ReorderArgs a)
{
    __shared__ int s_prev[4][HR_NPROBE_MAX];
    __shared__ int s_hot[4][HR_K_MAX];
    __shared__ unsigned char s_cls[4][HR_NPROBE_MAX];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t q = (int64_t)blockIdx.x * 4 + wave;
    if (q >= a.nq) return;
    int* prev = s_prev[wave];
    int* hot = s_hot[wave];
    unsigned char* cls = s_cls[wave];
    for (int i = lane; i < a.pp; i += 64) prev[i] = a.prev[q * a.pp + i];
    for (int i = lane; i < a.nh; i += 64) hot[i] = a.hot[q * a.nh + i];
    wave_sync();
    int count[4] = {0, 0, 0, 0};                // entries per group (whole wave holds the same values)
    for (int i0 = 0; i0 < a.np; i0 += 64) {
        const int i = i0 + lane;
        int c = 4;                              // (past the end)
        if (i < a.np) {
            const int l = a.probe[q * a.np + i];
            c = 3;
            if (l >= 0) {
                c = 2;
                for (int t = 0; t < a.pp; t++) if (prev[t] == l) { c = 1; break; }
                for (int t = 0; t < a.nh; t++) if (hot[t] == l) { c = 0; break; }
            }
            cls[i] = (unsigned char)c;
        }
#pragma unroll
        for (int g = 0; g < 4; g++) count[g] += __builtin_popcountll(__builtin_amdgcn_ballot_w64(c == g));
    }
    wave_sync();
    int base[4] = {0, count[0], count[0] + count[1], count[0] + count[1] + count[2]};
    for (int i0 = 0; i0 < a.np; i0 += 64) {
        const int i = i0 + lane;
        const int c = i < a.np ? cls[i] : 4;
#pragma unroll
        for (int g = 0; g < 4; g++) {
            const unsigned long long m = __builtin_amdgcn_ballot_w64(c == g);
            if (c == g) a.out[q * a.np + base[g] + lanes_below(m)] = a.probe[q * a.np + i];
            base[g] += __builtin_popcountll(m);
        }
    }
}

hipError_t launch_reorder_probes(const int32_t* probe, int np, const int32_t* prev, int pp, const int32_t* hot, int nh,
                                 int64_t nq, int32_t* out, hipStream_t s)
{
    if (nq <= 0) return hipSuccess;
    ReorderArgs a{probe, prev, hot, out, (int)nq, np, prev ? pp : 0, hot ? nh : 0};
    hipLaunchKernelGGL(k_reorder_probes, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, s, a);
    return hipGetLastError();
}

// The local cache of a request: the rows a previous retrieval returned (a larger top-k of v)
// are scored against the new query v' and the k best become the starting result of v's
// successor.  One wave per query, 16 lanes per row (four rows at a time); the query is rounded
// as the scan's operand is (binary16 for binary16 lists, bfloat16 hi + lo for bfloat16 lists),
// products and sums in float32.  Rows listed twice count once; -1 = no row.
struct RescoreArgs {
    const float* q;             // [nq, d]
    const void* rows;           // stored rows
    const float* row_norm;      // [N]
    const int64_t* row_ids;     // labels or nullptr
    const int32_t* cand;        // [nq, m] row numbers
    int64_t* out_ids;           // [nq, k]
    float* out_scores;          // [nq, k]
    int32_t* out_rows;          // [nq, k]
    int64_t nrows;
    int nq, m, k, d, dtype, l2;
};

__device__ __forceinline__ float rounded_like_operand(float x, int dtype)
{
    if (dtype == HR_F16) return (float)(_Float16)x;
    if (dtype == HR_BF16) {
        const uint16_t hi = bf16_rne(x);
        return bf16_to_f32(hi) + bf16_to_f32(bf16_rne(x - bf16_to_f32(hi)));
    }
    return x;
}

__global__ __launch_bounds__(256) void k_rescore(RescoreArgs a)
{
    __shared__ float s_key[4][HR_K_MAX];
    __shared__ int s_row[4][HR_K_MAX];
    __shared__ int64_t s_lab[4][HR_K_MAX];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t q = (int64_t)blockIdx.x * 4 + wave;
    if (q >= a.nq) return;
    float* key = s_key[wave];
    int* row = s_row[wave];
    int64_t* lab = s_lab[wave];
    const float* qp = a.q + q * a.d;
    const int sub = lane & 15, grp = lane >> 4;
    float qn = 0.f;
    for (int i = lane; i < a.d; i += 64) { const float x = rounded_like_operand(qp[i], a.dtype); qn += x * x; }
    qn = wave_sum(qn);
    for (int j0 = 0; j0 < a.m; j0 += 4) {
        const int j = j0 + grp;
        int r = j < a.m ? a.cand[q * a.m + j] : -1;
        if (r < 0 || r >= a.nrows) r = -1;
        float dot = 0.f;
        if (r >= 0) {
            // 8 elements per lane and step, the 16 lanes of a group side by side
            for (int e = sub * 8; e < a.d; e += 128) {
                float x[8];
                if (a.dtype == HR_F32) {
                    const float4* p = (const float4*)((const float*)a.rows + (size_t)r * a.d + e);
                    const float4 u = p[0], v = p[1];
                    x[0] = u.x; x[1] = u.y; x[2] = u.z; x[3] = u.w; x[4] = v.x; x[5] = v.y; x[6] = v.z; x[7] = v.w;
                } else {
                    const uint4 u = *(const uint4*)((const uint16_t*)a.rows + (size_t)r * a.d + e);
                    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
                    for (int t = 0; t < 4; t++) {
                        if (a.dtype == HR_F16) {
                            x[2 * t] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[t] & 0xffffu));
                            x[2 * t + 1] = (float)__builtin_bit_cast(_Float16, (uint16_t)(w[t] >> 16));
                        } else {
                            x[2 * t] = bf16_to_f32((uint16_t)(w[t] & 0xffffu));
                            x[2 * t + 1] = bf16_to_f32((uint16_t)(w[t] >> 16));
                        }
                    }
                }
#pragma unroll
                for (int t = 0; t < 8; t++) dot = __builtin_fmaf(x[t], rounded_like_operand(qp[e + t], a.dtype), dot);
            }
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
        if (sub == 0 && j < a.m) {
            row[j] = r;
            key[j] = r < 0 ? 0.f : (a.l2 ? 2.0f * dot - a.row_norm[r] : dot);
            lab[j] = r < 0 ? INT64_MAX : (a.row_ids ? a.row_ids[r] : (int64_t)r);
        }
    }
    wave_sync();
    // rows listed twice: the first copy counts, the others become "no row"
    {
        bool dup[(HR_K_MAX + 63) / 64];
#pragma unroll
        for (int c = 0; c < (HR_K_MAX + 63) / 64; c++) {
            const int j = c * 64 + lane;
            dup[c] = false;
            if (j < a.m && row[j] >= 0)
                for (int u = 0; u < j; u++) if (row[u] == row[j]) { dup[c] = true; break; }
        }
        wave_sync();
#pragma unroll
        for (int c = 0; c < (HR_K_MAX + 63) / 64; c++)
            if (dup[c]) row[c * 64 + lane] = -1;
        wave_sync();
    }
    // rank among the valid rows: better key first, equal keys by label
    int nvalid = 0;
    for (int j0 = 0; j0 < a.m; j0 += 64) {
        const int j = j0 + lane;
        const bool valid = j < a.m && row[j] >= 0;
        nvalid += __builtin_popcountll(__builtin_amdgcn_ballot_w64(valid));
        if (!valid) continue;
        int rank = 0;
        for (int t = 0; t < a.m; t++)
            if (row[t] >= 0 && (key[t] > key[j] || (key[t] == key[j] && lab[t] < lab[j]))) rank++;
        if (rank < a.k) {
            const size_t o = (size_t)q * a.k + rank;
            a.out_ids[o] = lab[j];
            a.out_scores[o] = a.l2 ? fmaxf(qn - key[j], 0.f) : key[j];
            a.out_rows[o] = row[j];
        }
    }
    for (int i = nvalid + lane; i < a.k; i += 64) {      // fewer than k rows: the other places stay empty
        const size_t o = (size_t)q * a.k + i;
        a.out_ids[o] = -1;
        a.out_scores[o] = a.l2 ? __builtin_inff() : -__builtin_inff();
        a.out_rows[o] = -1;
    }
}

hipError_t launch_rescore(const float* q, int64_t nq, int d, int dtype, const void* rows, const float* row_norm,
                          const int64_t* row_ids, int64_t nrows, const int32_t* cand, int m, int k, int l2,
                          int64_t* out_ids, float* out_scores, int32_t* out_rows, hipStream_t s)
{
    if (nq <= 0) return hipSuccess;
    RescoreArgs a{q, rows, row_norm, row_ids, cand, out_ids, out_scores, out_rows, nrows, (int)nq, m, k, d, dtype, l2};
    hipLaunchKernelGGL(k_rescore, dim3((unsigned)((nq + 3) / 4)), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_merge(const MergeArgs& a, hipStream_t s)
{
    if (a.nq <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_merge, dim3((unsigned)((a.nq + 3) / 4)), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace hr
