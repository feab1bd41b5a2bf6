// Cluster-major list scan with in-kernel top-k selection (gfx950, wave64, MFMA 16x16x32).
//
// One work item = (a segment of consecutive rows of one inverted list) x (a tile of the
// queries bucketed to that list).  The rows are streamed once through LDS in blocks of 16
// and every wave multiplies each block with the query operand it keeps in registers, so a
// staged block is reused by all queries of the tile (the cross-request sharing of one pass
// over a probed cluster: Sections 4.4 and 5 of the paper; the per-pair similarity is the
// one of Section 2.2).  Each wave owns a fixed set of query columns and keeps, per column,
// a small candidate buffer in LDS that is pruned to the k best whenever it fills up; what
// is left at the end of the item goes to the item's slots for the per-query merge.
//
// Storage types:
//   HR_F16   rows are binary16; the query is rounded to binary16; one MFMA per k-step.
//   HR_BF16  rows are bfloat16; the query is split into bfloat16 hi + lo parts that take two
//            MFMA columns (lanes j and j+8 of each 16-lane row), summed after the MFMA.
//   HR_F32   rows are float32, split on the fly into binary16 hi + 2^11-scaled lo planes; the
//            query likewise; the four partial products are recombined with their scales,
//            which keeps about 22 bits of each factor with float32 accumulation.
#pragma once
#include "common.h"

namespace hr {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Keep the k best of the n (> k) candidates in buf[0..n), sorted best-first in buf[0..k).
// Order: key descending, then label ascending (label = row number when ids == nullptr; rows
// of one buffer come from one list segment, labels are only fetched when equal keys straddle
// the k-th place).  Called by a whole converged wave with wave-uniform arguments.
// tie_scratch: per-wave LDS array of cap int64.  Returns the k-th key.
template <int CAPE>   // entries held per lane: CAPE * 64 >= n
__device__ __forceinline__ float wave_prune(Cand* buf, int n, int k, const int64_t* ids,
                                            int64_t* tie_scratch)
{
    const int lane = lane_id();
    Cand e[CAPE];
    int rank[CAPE];
#pragma unroll
    for (int m = 0; m < CAPE; m++) {
        int idx = lane + 64 * m;
        e[m] = (idx < n) ? buf[idx] : Cand{0u, 0xffffffffu};
        rank[m] = 0;
    }
    for (int i = 0; i < n; i++) {
        Cand o = buf[i];
        float so = __builtin_bit_cast(float, o.key);
#pragma unroll
        for (int m = 0; m < CAPE; m++) {
            float sm = __builtin_bit_cast(float, e[m].key);
            rank[m] += (so > sm || (so == sm && o.row < e[m].row)) ? 1 : 0;
        }
    }
    wave_sync();
#pragma unroll
    for (int m = 0; m < CAPE; m++)
        if (lane + 64 * m < n && rank[m] < k) buf[rank[m]] = e[m];
    wave_sync();
    const float kth = __builtin_bit_cast(float, buf[k - 1].key);
    if (ids != nullptr) {
        bool dropped_tie = false;
#pragma unroll
        for (int m = 0; m < CAPE; m++)
            dropped_tie |= (lane + 64 * m < n && rank[m] >= k &&
                            __builtin_bit_cast(float, e[m].key) == kth);
        if (__builtin_amdgcn_ballot_w64(dropped_tie) != 0) {
            // equal keys on both sides of the k-th place: order that group by label
            int greater = 0;
            int64_t my_id[CAPE];
#pragma unroll
            for (int m = 0; m < CAPE; m++) {
                int idx = lane + 64 * m;
                float sm = __builtin_bit_cast(float, e[m].key);
                bool in = idx < n;
                greater += __builtin_popcountll(__builtin_amdgcn_ballot_w64(in && sm > kth));
                bool tied = in && sm == kth;
                my_id[m] = tied ? ids[e[m].row] : INT64_MAX;
                if (in) tie_scratch[idx] = my_id[m];
            }
            wave_sync();
            int pos[CAPE];
#pragma unroll
            for (int m = 0; m < CAPE; m++) pos[m] = 0;
            for (int i = 0; i < n; i++) {
                int64_t oid = tie_scratch[i];
#pragma unroll
                for (int m = 0; m < CAPE; m++) pos[m] += (oid < my_id[m]) ? 1 : 0;
            }
#pragma unroll
            for (int m = 0; m < CAPE; m++)
                if (my_id[m] != INT64_MAX && greater + pos[m] < k) buf[greater + pos[m]] = e[m];
            wave_sync();
        }
    }
    return kth;
}

template <int DT> struct StoreTraits;
template <> struct StoreTraits<HR_F32>  { static constexpr int esize = 4, planes = 2, nc = 8;  };
template <> struct StoreTraits<HR_F16>  { static constexpr int esize = 2, planes = 1, nc = 16; };
template <> struct StoreTraits<HR_BF16> { static constexpr int esize = 2, planes = 1, nc = 8;  };

template <int DT, int KSTEPS>
struct ScanShape {
    static constexpr int d = KSTEPS * 32;
    static constexpr int rowb = d * StoreTraits<DT>::esize;        // bytes of one stored row
    static constexpr int rowp = d * 2 + kRowPad;                   // bytes of one staged row (one plane)
    static constexpr int plane_bytes = kBlockRows * rowp;
    static constexpr int buf_bytes = plane_bytes * StoreTraits<DT>::planes;
    static constexpr int chunks = kBlockRows * rowb / 16;          // 16-byte chunks per block
    static constexpr int nld = (chunks + kScanThreads - 1) / kScanThreads;
    static constexpr int cw = StoreTraits<DT>::nc * 4;             // query columns per item
};

template <int DT, int KSTEPS>
__device__ __forceinline__ void load_block(const char* src, int valid_chunks, uint4 (&regs)[ScanShape<DT, KSTEPS>::nld])
{
    using S = ScanShape<DT, KSTEPS>;
#pragma unroll
    for (int m = 0; m < S::nld; m++) {
        int c = threadIdx.x + kScanThreads * m;
        regs[m] = (c < valid_chunks) ? *(const uint4*)(src + (size_t)c * 16) : uint4{0, 0, 0, 0};
    }
}

template <int DT, int KSTEPS>
__device__ __forceinline__ void stage_block(char* buf, const uint4 (&regs)[ScanShape<DT, KSTEPS>::nld])
{
    using S = ScanShape<DT, KSTEPS>;
#pragma unroll
    for (int m = 0; m < S::nld; m++) {
        int c = threadIdx.x + kScanThreads * m;
        if (S::chunks % kScanThreads != 0 && c >= S::chunks) continue;
        constexpr int cpr = S::rowb / 16;              // chunks per row
        int r = c / cpr, p = c % cpr;
        if constexpr (DT == HR_F32) {
            float x[4] = {__builtin_bit_cast(float, regs[m].x), __builtin_bit_cast(float, regs[m].y),
                          __builtin_bit_cast(float, regs[m].z), __builtin_bit_cast(float, regs[m].w)};
            half4 hi, lo;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                _Float16 h = (_Float16)x[i];
                hi[i] = h;
                lo[i] = (_Float16)((x[i] - (float)h) * 2048.0f);
            }
            *(half4*)(buf + r * S::rowp + p * 8) = hi;
            *(half4*)(buf + S::plane_bytes + r * S::rowp + p * 8) = lo;
        } else {
            *(uint4*)(buf + r * S::rowp + p * 16) = regs[m];
        }
    }
}

template <int DT, int KSTEPS>
__global__ __launch_bounds__(kScanThreads) void k_scan(ScanArgs a)
{
    using S = ScanShape<DT, KSTEPS>;
    using T = StoreTraits<DT>;
    constexpr int NC = T::nc;
    constexpr int CAPE = 3;
    extern __shared__ __align__(16) char smem[];
    // LDS: [2 staging buffers][selection buffers CW*cap][tie scratch 4*cap int64][cnt CW][item]
    char* stage = smem;
    Cand* sel = (Cand*)(smem + 2 * S::buf_bytes);
    int64_t* tie = (int64_t*)(sel + S::cw * a.cap);
    int* cnt = (int*)(tie + 4 * a.cap);
    int* s_item = cnt + S::cw;

    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int g = lane >> 4;                       // k-group / output row group
    const int jcol = lane & (NC - 1);              // column inside the wave
    const int part = (NC == 8) ? ((lane >> 3) & 1) : 0;   // 0 = hi, 1 = lo operand column
    const bool owner = (NC == 16) || part == 0;    // lane whose accumulator holds the full dot
    Cand* mysel = sel + (wave * NC) * a.cap;
    int* mycnt = cnt + wave * NC;
    int64_t* mytie = tie + wave * a.cap;
    const int total_items = a.dense ? a.dense_items : a.dyn[DYN_ITEMS];
    const int seg_rows = a.dense ? a.dense_seg_rows : a.dyn[DYN_SEG_ROWS];

    for (;;) {
        if (threadIdx.x == 0) *s_item = atomicAdd(a.work_counter, 1);
        __syncthreads();
        const int item = *s_item;
        if (item >= total_items) break;

        // ---- decode the work item
        int list, seg, qt, row0, row_end, w, boff;
        if (a.dense) {
            seg = item / a.dense_nqt;
            qt = item - seg * a.dense_nqt;
            list = 0;
            row0 = seg * seg_rows;
            row_end = min(a.dense_nrows, row0 + seg_rows);
            w = a.nq;
            boff = 0;
        } else {
            int4 it = a.item_tab[item];
            list = it.x; seg = it.y; qt = it.z;
            int l0 = a.list_off[list], l1 = a.list_off[list + 1];
            row0 = l0 + seg * seg_rows;
            row_end = min(l1, row0 + seg_rows);
            boff = a.bucket_off[list];
            w = a.bucket_off[list + 1] - boff;
        }
        const int nrows = row_end - row0;
        const int nblk = (nrows + kBlockRows - 1) / kBlockRows;

        // ---- query operand of this lane's column into registers (B fragments)
        const int ecol = qt * S::cw + wave * NC + jcol;      // entry inside the bucket
        const bool col_ok = ecol < w;
        int q = 0;
        if (col_ok) q = a.dense ? ecol : a.bucket_q[boff + ecol];
        uint4 bfrag[KSTEPS];
        {
            const size_t qrow = (NC == 8) ? ((size_t)q * 2 + part) : (size_t)q;
            const char* qp = (const char*)a.qop + qrow * (size_t)(S::d * 2) + g * 16;
#pragma unroll
            for (int t = 0; t < KSTEPS; t++)
                bfrag[t] = col_ok ? *(const uint4*)(qp + t * 64) : uint4{0, 0, 0, 0};
        }
        float thr = col_ok ? dec_order(a.thr[q]) : __builtin_inff();
        if (lane < NC) mycnt[lane] = 0;

        // ---- stream the rows
        const char* src = (const char*)a.rows + (size_t)row0 * S::rowb;
        uint4 regs[S::nld];
        load_block<DT, KSTEPS>(src, min(nrows, kBlockRows) * (S::rowb / 16), regs);
        stage_block<DT, KSTEPS>(stage, regs);
        __syncthreads();

        for (int blk = 0; blk < nblk; blk++) {
            char* cur = stage + (blk & 1) * S::buf_bytes;
            const bool more = blk + 1 < nblk;
            if (more) {
                int left = nrows - (blk + 1) * kBlockRows;
                load_block<DT, KSTEPS>(src + (size_t)(blk + 1) * kBlockRows * S::rowb,
                                       min(left, kBlockRows) * (S::rowb / 16), regs);
            }
            const int rbase = row0 + blk * kBlockRows + g * 4;   // first of this lane's 4 rows
            float nrm[4] = {0.f, 0.f, 0.f, 0.f};
            if (a.l2) {
#pragma unroll
                for (int r = 0; r < 4; r++)
                    if (rbase + r < row_end) nrm[r] = a.row_norm[rbase + r];
            }

            // ---- 16 rows x NC*? columns x d : MFMA over the k-steps
            floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
            const char* ap = cur + (lane & 15) * S::rowp + g * 16;
#pragma unroll
            for (int t = 0; t < KSTEPS; t++) {
                if constexpr (DT == HR_F32) {
                    half8 ahi = *(const half8*)(ap + t * 64);
                    half8 alo = *(const half8*)(ap + S::plane_bytes + t * 64);
                    half8 b = __builtin_bit_cast(half8, bfrag[t]);
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(ahi, b, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(alo, b, acc1, 0, 0, 0);
                } else if constexpr (DT == HR_F16) {
                    half8 av = *(const half8*)(ap + t * 64);
                    half8 b = __builtin_bit_cast(half8, bfrag[t]);
                    if (t & 1) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, b, acc1, 0, 0, 0);
                    else       acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, b, acc0, 0, 0, 0);
                } else {
                    bf16x8 av = *(const bf16x8*)(ap + t * 64);
                    bf16x8 b = __builtin_bit_cast(bf16x8, bfrag[t]);
                    if (t & 1) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, b, acc1, 0, 0, 0);
                    else       acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, b, acc0, 0, 0, 0);
                }
            }

            // ---- keys of this lane's 4 (row, column) pairs
            float key[4];
#pragma unroll
            for (int r = 0; r < 4; r++) {
                float dot;
                if constexpr (DT == HR_F32) {
                    float t0 = __shfl_xor(acc0[r], 8);       // hi rows x lo query
                    float t1 = __shfl_xor(acc1[r], 8);       // lo rows x lo query
                    dot = acc0[r] + (t0 + acc1[r]) * (1.0f / 2048.0f) + t1 * (1.0f / 4194304.0f);
                } else if constexpr (DT == HR_BF16) {
                    float s = acc0[r] + acc1[r];
                    dot = s + __shfl_xor(s, 8);
                } else {
                    dot = acc0[r] + acc1[r];
                }
                key[r] = a.l2 ? (2.0f * dot - nrm[r]) : dot;
            }

            // ---- append what reaches the column's threshold
            bool any = false;
            bool pass[4];
#pragma unroll
            for (int r = 0; r < 4; r++) {
                pass[r] = owner && col_ok && (rbase + r < row_end) && key[r] >= thr;
                any |= pass[r];
            }
            if (__builtin_amdgcn_ballot_w64(any) != 0) {
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    if (pass[r]) {
                        int pos = atomicAdd(&mycnt[jcol], 1);
                        mysel[jcol * a.cap + pos] = Cand{__builtin_bit_cast(uint32_t, key[r]), (uint32_t)(rbase + r)};
                    }
                }
                wave_sync();
                int c = (lane < NC) ? mycnt[lane] : 0;
                unsigned long long full = __builtin_amdgcn_ballot_w64(c > a.cap - kAppendMax);
                while (full) {
                    int col = __builtin_ctzll(full);
                    full &= full - 1;
                    int n = __builtin_amdgcn_readlane(c, col);
                    float kth = wave_prune<CAPE>(mysel + col * a.cap, n, a.k, a.row_ids, mytie);
                    float nt = kth;
                    if (lane == col) {
                        mycnt[col] = a.k;
                        int old = atomicMax(&a.thr[q], enc_order(kth));
                        nt = fmaxf(kth, dec_order(old));
                    }
                    nt = __shfl(nt, col);
                    if (jcol == col) thr = fmaxf(thr, nt);
                }
                wave_sync();
            }

            if (more) stage_block<DT, KSTEPS>(stage + ((blk + 1) & 1) * S::buf_bytes, regs);
            __syncthreads();
        }

        // ---- hand what is left to the item's slots
        wave_sync();
        const unsigned long long okmask = __builtin_amdgcn_ballot_w64(col_ok && lane < NC);
        for (int col = 0; col < NC; col++) {
            if (!((okmask >> col) & 1)) continue;
            int n = mycnt[col];
            n = __builtin_amdgcn_readfirstlane(n);
            Cand* cb = mysel + col * a.cap;
            if (n > a.k) {
                float kth = wave_prune<CAPE>(cb, n, a.k, a.row_ids, mytie);
                n = a.k;
                int qq = __builtin_amdgcn_readlane(q, col);
                if (lane == 0) atomicMax(&a.thr[qq], enc_order(kth));
            }
            size_t slot = (size_t)item * S::cw + wave * NC + col;
            if (lane == 0) a.slot_cnt[slot] = n;
            for (int i = lane; i < n; i += 64) a.slot_ent[slot * a.k + i] = cb[i];
        }
        __syncthreads();
    }
}

template <int DT>
inline hipError_t launch_scan_dtype(int d, const ScanArgs& a, int grid, size_t lds, hipStream_t s)
{
#define HR_SCAN_CASE(KS)                                                                           \
    case KS * 32: {                                                                                \
        auto kern = k_scan<DT, KS>;                                                                \
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e != hipSuccess) return e;                                                             \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kScanThreads), lds, s, a);                       \
        return hipGetLastError();                                                                  \
    }
    switch (d) {
        HR_SCAN_CASE(2)
        HR_SCAN_CASE(4)
        HR_SCAN_CASE(8)
        HR_SCAN_CASE(16)
        HR_SCAN_CASE(24)
        HR_SCAN_CASE(32)
    default: return hipErrorInvalidValue;
    }
#undef HR_SCAN_CASE
}

}  // namespace hr
