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
#include <utility>

#include "common.h"

namespace hr {

// compile-time loop: f(std::integral_constant<int, 0>) ... f(std::integral_constant<int, N-1>)
template <typename F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
// 16 bytes as a register vector (a struct such as HIP's uint4 is copied with memcpy semantics,
// which can pin a local array of them to scratch memory)
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ int lanes_below(unsigned long long mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// Keep the k best of the n (> k) candidates in buf[0..n): afterwards buf[0..k) holds them, in
// no particular order.  Order: key descending, then label ascending (label = row number when
// ids == nullptr; labels are only fetched when equal keys straddle the k-th place).
// Binary radix select on the 32 key bits: the cost does not depend on n.  Called by a whole
// converged wave with wave-uniform arguments.  Returns the k-th best key.
template <int CAPE>   // entries held per lane: CAPE * 64 >= n
__device__ __forceinline__ uint32_t wave_select(Cand* buf, int n, int k, const int64_t* ids)
{
    const int lane = lane_id();
    Cand e[CAPE];
    unsigned long long alive[CAPE], kept[CAPE];
#pragma unroll
    for (int m = 0; m < CAPE; m++) {
        const int idx = lane + 64 * m;
        const bool valid = idx < n;
        e[m] = valid ? buf[idx] : Cand{0u, 0u};
        alive[m] = __builtin_amdgcn_ballot_w64(valid);
        kept[m] = 0;
    }
    int need = k;              // how many of the entries still alive belong to the k best
    uint32_t T = 0;            // k-th best key, built from the top bit down
    for (int b = 31; b >= 0; b--) {
        const uint32_t bit = 1u << b;
        unsigned long long ones[CAPE];
        int c1 = 0;
#pragma unroll
        for (int m = 0; m < CAPE; m++) {
            ones[m] = alive[m] & __builtin_amdgcn_ballot_w64((e[m].key & bit) != 0);
            c1 += __builtin_popcountll(ones[m]);
        }
        if (c1 >= need) {
            T |= bit;
#pragma unroll
            for (int m = 0; m < CAPE; m++) alive[m] = ones[m];
        } else {
            need -= c1;
#pragma unroll
            for (int m = 0; m < CAPE; m++) { kept[m] |= ones[m]; alive[m] &= ~ones[m]; }
        }
    }
    // alive = entries whose key equals T; `need` of them complete the k best
    int n_eq = 0;
#pragma unroll
    for (int m = 0; m < CAPE; m++) n_eq += __builtin_popcountll(alive[m]);
    if (n_eq > need) {
        // equal keys on both sides of the k-th place: take the lowest labels
        int64_t label[CAPE];
        int rank[CAPE];
#pragma unroll
        for (int m = 0; m < CAPE; m++) {
            const bool mine = (alive[m] >> lane) & 1;
            label[m] = mine ? (ids ? ids[e[m].row] : (int64_t)e[m].row) : INT64_MAX;
            rank[m] = 0;
        }
#pragma unroll
        for (int m2 = 0; m2 < CAPE; m2++) {
            unsigned long long mask = alive[m2];
            while (mask) {
                const int L = __builtin_ctzll(mask);
                mask &= mask - 1;
                const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)label[m2], L);
                const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)((uint64_t)label[m2] >> 32), L);
                const int64_t other = (int64_t)(((uint64_t)hi << 32) | lo);
#pragma unroll
                for (int m = 0; m < CAPE; m++) rank[m] += (other < label[m]) ? 1 : 0;
            }
        }
#pragma unroll
        for (int m = 0; m < CAPE; m++)
            alive[m] &= __builtin_amdgcn_ballot_w64(rank[m] < need);
    }
    wave_sync();
    int base = 0;
#pragma unroll
    for (int m = 0; m < CAPE; m++) {
        const unsigned long long both = kept[m] | alive[m];
        if ((both >> lane) & 1) buf[base + lanes_below(both)] = e[m];
        base += __builtin_popcountll(both);
    }
    wave_sync();
    return T;
}

template <int DT> struct StoreTraits;
template <> struct StoreTraits<HR_F32>  { static constexpr int esize = 4, planes = 2, nc = 8;  };
template <> struct StoreTraits<HR_F16>  { static constexpr int esize = 2, planes = 1, nc = 16; };
template <> struct StoreTraits<HR_BF16> { static constexpr int esize = 2, planes = 1, nc = 8;  };

constexpr int kScanWaves = 4;                 // one wave per SIMD: each may use all 512 registers

// NCS = 16-column MFMA sets per wave (1 or 2).  Every wave owns NCS * nc query columns, so a
// work item covers 4 * NCS * nc queries of a bucket; all waves share the staged rows.
template <int DT, int KSTEPS, int NCS>
struct ScanShape {
    static constexpr int threads = kScanWaves * 64;
    static constexpr int d = KSTEPS * 32;
    static constexpr int rowb = d * StoreTraits<DT>::esize;        // bytes of one stored row
    static constexpr int rowp = d * 2 + kRowPad;                   // bytes of one staged row (one plane)
    static constexpr int plane_bytes = kBlockRows * rowp;
    static constexpr int buf_bytes = plane_bytes * StoreTraits<DT>::planes;
    static constexpr int chunks = kBlockRows * rowb / 16;          // 16-byte chunks per block
    static constexpr int nld = (chunks + threads - 1) / threads;   // chunks per thread per block
    // row blocks kept in flight in registers ahead of the one being staged
    static constexpr int pf = 24 / nld < 1 ? 1 : (24 / nld > 4 ? 4 : 24 / nld);
    static constexpr int wcols = StoreTraits<DT>::nc * NCS;        // query columns per wave
    static constexpr int cw = wcols * kScanWaves;                  // query columns per item
};

#ifdef HR_SCAN_TIMING
#define HR_TIC(var) long long var = clock64()
#define HR_TOC(acc, var) do { long long n_ = clock64(); acc += n_ - var; var = n_; } while (0)
#else
#define HR_TIC(var)
#define HR_TOC(acc, var)
#endif

// Every thread always loads (chunks past the end of the segment re-read its last chunk; the
// rows they would belong to are masked out of the selection): an unconditional load keeps the
// ring registers free of the zero-fill writes that would otherwise have to wait for the
// loads still in flight.
template <typename S>
__device__ __forceinline__ void load_block(const char* src, int valid_chunks, u32x4 (&regs)[S::nld])
{
#pragma unroll
    for (int m = 0; m < S::nld; m++) {
        int c = min((int)threadIdx.x + S::threads * m, valid_chunks - 1);
        regs[m] = *(const u32x4*)(src + (size_t)c * 16);
    }
}

template <int DT, typename S>
__device__ __forceinline__ void stage_block(char* buf, const u32x4 (&regs)[S::nld])
{
#pragma unroll
    for (int m = 0; m < S::nld; m++) {
        int c = threadIdx.x + S::threads * m;
        if (S::chunks % S::threads != 0 && c >= S::chunks) continue;
        constexpr int cpr = S::rowb / 16;              // chunks per row
        int r = c / cpr, p = c % cpr;
        if constexpr (DT == HR_F32) {
            const floatx4 xv = __builtin_bit_cast(floatx4, regs[m]);
            const float x[4] = {xv[0], xv[1], xv[2], xv[3]};
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
            *(u32x4*)(buf + r * S::rowp + p * 16) = regs[m];
        }
    }
}

// 16 staged rows x NA column sets x d: the MFMA chain of one block.  acc[s][0..1] are the two
// partial accumulators of set s (for HR_F32: hi-row and lo-row products).  The row fragments
// are fetched from LDS a group of k-steps ahead of the MFMAs that use them (the scheduling
// barriers keep the compiler from sinking each read next to its use, which would expose the
// LDS latency 24 times per block).
template <int DT, int KSTEPS, int NCS, int NA, typename S>
__device__ __forceinline__ void mfma_block(const char* ap, const u32x4 (&bfrag)[NCS][KSTEPS], floatx4 (&acc)[NCS][2])
{
    constexpr int G = KSTEPS < 8 ? KSTEPS : 8;       // k-steps per group
    constexpr int NG = KSTEPS / G;
    constexpr int P = StoreTraits<DT>::planes;
    static_assert(KSTEPS % G == 0, "k-steps must split into whole groups");
#pragma unroll
    for (int s = 0; s < NA; s++) { acc[s][0] = floatx4{0.f, 0.f, 0.f, 0.f}; acc[s][1] = floatx4{0.f, 0.f, 0.f, 0.f}; }
    u32x4 af[2][P][G];
#pragma unroll
    for (int i = 0; i < G; i++)
#pragma unroll
        for (int pl = 0; pl < P; pl++) af[0][pl][i] = *(const u32x4*)(ap + pl * S::plane_bytes + i * 64);
#pragma unroll
    for (int gi = 0; gi < NG; gi++) {
        if (gi + 1 < NG) {
#pragma unroll
            for (int i = 0; i < G; i++)
#pragma unroll
                for (int pl = 0; pl < P; pl++)
                    af[(gi + 1) & 1][pl][i] = *(const u32x4*)(ap + pl * S::plane_bytes + ((gi + 1) * G + i) * 64);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < G; i++) {
            const int t = gi * G + i;
#pragma unroll
            for (int s = 0; s < NA; s++) {
                if constexpr (DT == HR_F32) {
                    half8 b = __builtin_bit_cast(half8, bfrag[s][t]);
                    acc[s][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, af[gi & 1][0][i]), b, acc[s][0], 0, 0, 0);
                    acc[s][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, af[gi & 1][1][i]), b, acc[s][1], 0, 0, 0);
                } else if constexpr (DT == HR_F16) {
                    half8 b = __builtin_bit_cast(half8, bfrag[s][t]);
                    acc[s][t & 1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, af[gi & 1][0][i]), b, acc[s][t & 1], 0, 0, 0);
                } else {
                    bf16x8 b = __builtin_bit_cast(bf16x8, bfrag[s][t]);
                    acc[s][t & 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[gi & 1][0][i]), b, acc[s][t & 1], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// prune with as few register slots per lane as the buffer capacity needs
__device__ __forceinline__ uint32_t select_k(Cand* buf, int n, int k, int cap, const int64_t* ids)
{
    if (cap <= 64) return wave_select<1>(buf, n, k, ids);
    if (cap <= 128) return wave_select<2>(buf, n, k, ids);
    return wave_select<3>(buf, n, k, ids);
}

template <int DT, int KSTEPS, int NCS>
__global__ __launch_bounds__(kScanWaves * 64, 1) void k_scan(ScanArgs a)
{
    using S = ScanShape<DT, KSTEPS, NCS>;
    using T = StoreTraits<DT>;
    constexpr int NC = T::nc;
    constexpr int WC = S::wcols;
    constexpr int PF = S::pf;
    extern __shared__ __align__(16) char smem[];
    // LDS: [2 staging buffers][selection buffers cw*cap][cnt cw][2 x 16 row norms][item]
    char* stage = smem;
    Cand* sel = (Cand*)(smem + 2 * S::buf_bytes);
    int* cnt = (int*)(sel + S::cw * a.cap);
    float* nstage = (float*)(cnt + S::cw);
    int* s_item = (int*)(nstage + 2 * kBlockRows);

    const int lane = lane_id();
    const int wave = threadIdx.x >> 6;
    const int g = lane >> 4;                       // k-group / output row group
    const int jcol = lane & (NC - 1);              // column inside a set
    const int part = (NC == 8) ? ((lane >> 3) & 1) : 0;   // 0 = hi, 1 = lo operand column
    const bool owner = (NC == 16) || part == 0;    // lane whose accumulator holds the full dot
    Cand* mysel = sel + (wave * WC) * a.cap;
    int* mycnt = cnt + wave * WC;
    const int seg_rows = a.dense ? a.dense_seg_rows : a.dyn[DYN_SEG_ROWS];
    const int myx = blockIdx.x & 7;                // workgroups are dealt round-robin to the 8 XCDs
    int drained = 0;                               // thread 0: queues found empty
#ifdef HR_SCAN_TIMING
    long long t_pop = 0, t_setup = 0, t_mfma = 0, t_sel = 0, t_stage = 0, t_bar = 0, t_emit = 0;
    int n_items = 0, n_blocks = 0, n_cand_blocks = 0, n_prunes = 0;
#endif
    HR_TIC(tk);

    for (;;) {
        if (threadIdx.x == 0) {
            int item = -1;
            if (a.dense) {
                int i = atomicAdd(a.work_counter, 1);
                if (i < a.dense_items) item = i;
            } else {
                // own XCD's queue first (its items share list segments through this XCD's L2),
                // then the others' leftovers
                for (int t = 0; t < 8 && item < 0; t++) {
                    int x = (myx + t) & 7;
                    if (drained & (1 << x)) continue;
                    int pos = atomicAdd(&a.xq_head[x], 1);
                    if (pos < a.xq_count[x]) item = a.xq[(size_t)x * a.xq_stride + pos];
                    else drained |= 1 << x;
                }
            }
            *s_item = item;
        }
        __syncthreads();
        const int item = *s_item;
        if (item < 0) break;
        HR_TOC(t_pop, tk);

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
        const char* src = (const char*)a.rows + (size_t)row0 * S::rowb;
        // Loads for a block past the end of the segment re-read its last block: every path then
        // issues the same number of loads per iteration, which is what lets the staging code
        // wait for "all but the newest PF-1 blocks" with a fixed counter value instead of
        // draining the whole prefetch ring.
        auto block_chunks = [&](int blk) __attribute__((always_inline)) { return min(nrows - min(blk, nblk - 1) * kBlockRows, kBlockRows) * (S::rowb / 16); };
        auto block_src = [&](int blk) __attribute__((always_inline)) { return src + (size_t)min(blk, nblk - 1) * kBlockRows * S::rowb; };

        // ---- first row blocks on their way before anything else
        // (the squared row norms of a block travel with it: a separate load inside the block
        // loop would make every block wait for all the prefetches issued before it)
        u32x4 ring[PF][S::nld];
        float nring[PF];
        auto load_norm = [&](int blk) __attribute__((always_inline)) {
            const int r = min(row0 + min(blk, nblk - 1) * kBlockRows + (int)(threadIdx.x & (kBlockRows - 1)), row_end - 1);
            return a.row_norm[r];
        };
        load_block<S>(block_src(0), block_chunks(0), ring[0]);
        nring[0] = load_norm(0);

        // ---- query operands of this lane's columns into registers (B fragments)
        const int ecol0 = qt * S::cw + wave * WC + jcol;     // entry inside the bucket, set 0
        bool col_ok[NCS];
        int q[NCS];
        float thr[NCS];
        u32x4 bfrag[NCS][KSTEPS];
#pragma unroll
        for (int s = 0; s < NCS; s++) {
            const int ecol = ecol0 + s * NC;
            col_ok[s] = ecol < w;
            q[s] = 0;
            if (col_ok[s]) q[s] = a.dense ? ecol : a.bucket_q[boff + ecol];
        }
#pragma unroll
        for (int s = 0; s < NCS; s++) {
            const size_t qrow = (NC == 8) ? ((size_t)q[s] * 2 + part) : (size_t)q[s];
            const char* qp = (const char*)a.qop + qrow * (size_t)(S::d * 2) + g * 16;
#pragma unroll
            for (int t = 0; t < KSTEPS; t++)
                bfrag[s][t] = col_ok[s] ? *(const u32x4*)(qp + t * 64) : u32x4{0, 0, 0, 0};
            thr[s] = (col_ok[s] && !(a.dbg_flags & 1)) ? dec_key(a.thr[q[s]]) : __builtin_inff();
        }
        // candidates buffered per column: kept in a register by every lane of the column (the
        // lanes of a column see the same ballots, so they stay in step without LDS traffic)
        int ccnt[NCS];
#pragma unroll
        for (int s = 0; s < NCS; s++) ccnt[s] = 0;
        const unsigned long long colmask = 0x0001000100010001ULL << jcol;   // owner lanes of my column
        const unsigned long long below = (1ULL << lane) - 1;
        // column sets of this wave that hold at least one query (sets fill in order); a wave
        // with none only helps to stage rows
        int nact = 0;
#pragma unroll
        for (int s = 0; s < NCS; s++) nact += __builtin_amdgcn_ballot_w64(col_ok[s]) != 0 ? 1 : 0;
        if (a.dbg_flags & 2) nact = 0;

        // Everything loaded so far (query operands, thresholds, first row block) is waited for
        // here, once, and only then are the next PF blocks requested, oldest ring slot first.
        // The loop is thus entered with exactly the loads in flight, in exactly the order, that
        // every later iteration sees; the compiler's wait-count analysis (which merges the two
        // ways into the loop) can then let the staging of a block wait for that block alone,
        // with the PF-1 younger blocks still in flight, instead of draining the ring.
        __builtin_amdgcn_s_waitcnt(0x0F70);     // vmcnt(0) only
        stage_block<DT, S>(stage, ring[0]);
        nstage[threadIdx.x & (kBlockRows - 1)] = nring[0];      // (same value from 16 threads each)
        static_for<PF>([&](auto pc) __attribute__((always_inline)) {
            constexpr int slot = (decltype(pc)::value + 1) % PF;
            load_block<S>(block_src(decltype(pc)::value + 1), block_chunks(decltype(pc)::value + 1), ring[slot]);
            nring[slot] = load_norm(decltype(pc)::value + 1);
        });
        __syncthreads();
        HR_TOC(t_setup, tk);

        for (int b0 = 0; b0 < nblk; b0 += PF) {
            static_for<PF>([&](auto pc) __attribute__((always_inline)) {
                constexpr int p = decltype(pc)::value;
                const int blk = b0 + p;
                if (blk >= nblk) return;
                char* cur = stage + (blk & 1) * S::buf_bytes;
                const int rbase = row0 + blk * kBlockRows + g * 4;   // first of this lane's 4 rows

#ifdef HR_SCAN_TIMING
                n_blocks++;
#endif
                if (nact > 0) {
                    const floatx4 nrm = *(const floatx4*)(nstage + (blk & 1) * kBlockRows + g * 4);
                    floatx4 acc[NCS][2];
                    const char* ap = cur + (lane & 15) * S::rowp + g * 16;
                    if (NCS == 2 && nact == 2) mfma_block<DT, KSTEPS, NCS, NCS, S>(ap, bfrag, acc);
                    else                       mfma_block<DT, KSTEPS, NCS, 1, S>(ap, bfrag, acc);
                    HR_TOC(t_mfma, tk);

#pragma unroll
                    for (int s = 0; s < NCS; s++) {
                        if (s >= nact) break;
                        // ---- keys of this lane's 4 (row, column) pairs of set s
                        float key[4];
                        bool pass[4];
                        bool any = false;
#pragma unroll
                        for (int r = 0; r < 4; r++) {
                            float dot;
                            if constexpr (DT == HR_F32) {
                                float t0 = __shfl_xor(acc[s][0][r], 8);       // hi rows x lo query
                                float t1 = __shfl_xor(acc[s][1][r], 8);       // lo rows x lo query
                                dot = acc[s][0][r] + (t0 + acc[s][1][r]) * (1.0f / 2048.0f) + t1 * (1.0f / 4194304.0f);
                            } else if constexpr (DT == HR_BF16) {
                                float v = acc[s][0][r] + acc[s][1][r];
                                dot = v + __shfl_xor(v, 8);
                            } else {
                                dot = acc[s][0][r] + acc[s][1][r];
                            }
                            key[r] = a.l2 ? (2.0f * dot - nrm[r]) : dot;
                            pass[r] = owner && col_ok[s] && (rbase + r < row_end) && key[r] >= thr[s];
                            any |= pass[r];
                        }
                        // ---- append what reaches the column's threshold
                        if (__builtin_amdgcn_ballot_w64(any) != 0) {
#ifdef HR_SCAN_TIMING
                            n_cand_blocks++;
#endif
                            Cand* ssel = mysel + (s * NC) * a.cap;
                            // slot of each new candidate = column count + candidates of the same
                            // column in earlier row slots and in lower lanes of this row slot
                            int add = 0;
#pragma unroll
                            for (int r = 0; r < 4; r++) {
                                const unsigned long long mine = __builtin_amdgcn_ballot_w64(pass[r]) & colmask;
                                if (pass[r]) {
                                    const int pos = ccnt[s] + add + __builtin_popcountll(mine & below);
                                    ssel[jcol * a.cap + pos] = Cand{enc_key(key[r]), (uint32_t)(rbase + r)};
                                }
                                add += __builtin_popcountll(mine);
                            }
                            ccnt[s] += add;
                            unsigned long long full = __builtin_amdgcn_ballot_w64(lane < NC && ccnt[s] > a.cap - kAppendMax);
                            if (full) wave_sync();
                            while (full) {
                                int col = __builtin_ctzll(full);
                                full &= full - 1;
                                int n = __builtin_amdgcn_readlane(ccnt[s], col);
                                uint32_t kth = select_k(ssel + col * a.cap, n, a.k, a.cap, a.row_ids);
#ifdef HR_SCAN_TIMING
                                n_prunes++;
#endif
                                float nt = 0.f;
                                if (lane == col) {
                                    uint32_t old = atomicMax(&a.thr[q[s]], kth);
                                    nt = dec_key(kth > old ? kth : old);
                                }
                                nt = __shfl(nt, col);
                                if (jcol == col) { thr[s] = fmaxf(thr[s], nt); ccnt[s] = a.k; }
                            }
                        }
                    }
                    HR_TOC(t_sel, tk);
                }

                // ---- next block: registers -> LDS, and refill the ring slot it leaves
                {
                    constexpr int pn = (p + 1) % PF;
                    stage_block<DT, S>(stage + ((blk + 1) & 1) * S::buf_bytes, ring[pn]);
                    nstage[((blk + 1) & 1) * kBlockRows + (threadIdx.x & (kBlockRows - 1))] = nring[pn];
                    load_block<S>(block_src(blk + 1 + PF), block_chunks(blk + 1 + PF), ring[pn]);
                    nring[pn] = load_norm(blk + 1 + PF);
                }
                HR_TOC(t_stage, tk);
                __syncthreads();
                HR_TOC(t_bar, tk);
            });
        }

        // ---- hand what is left to the item's slots: columns still over k are cut down first
        // (one at a time, whole wave), then every lane copies one column's entries
        wave_sync();
        {
            int c = 0;
#pragma unroll
            for (int s = 0; s < NCS; s++) {
                const int v = __shfl(ccnt[s], (lane - s * NC) & 63);
                if (lane >= s * NC && lane < (s + 1) * NC) c = v;
            }
            unsigned long long over = __builtin_amdgcn_ballot_w64(c > a.k);
            while (over) {
                const int wc = __builtin_ctzll(over);
                over &= over - 1;
                const int n = __builtin_amdgcn_readlane(c, wc);
                uint32_t kth = select_k(mysel + wc * a.cap, n, a.k, a.cap, a.row_ids);
                // column wc = set wc / NC, lane wc % NC of that set holds its query
                int qq = 0;
#pragma unroll
                for (int s = 0; s < NCS; s++) {
                    int v = __builtin_amdgcn_readlane(q[s], wc % NC);
                    if (s == wc / NC) qq = v;
                }
                if (lane == 0) atomicMax(&a.thr[qq], kth);
            }
            wave_sync();
            bool ok = false;
#pragma unroll
            for (int s = 0; s < NCS; s++) {
                // is column `lane` of this wave (set s, lane - s*NC) a real query?
                bool v = __shfl(col_ok[s] ? 1 : 0, (lane - s * NC) & 63) != 0;
                if (lane >= s * NC && lane < (s + 1) * NC) ok = v;
            }
            if (lane < WC && ok) {
                const int n = min(c, a.k);
                const size_t slot = (size_t)item * S::cw + wave * WC + lane;
                a.slot_cnt[slot] = n;
                const Cand* cb = mysel + lane * a.cap;
                Cand* out = a.slot_ent + slot * a.k;
                for (int i = 0; i < n; i++) out[i] = cb[i];
            }
        }
        __syncthreads();
        HR_TOC(t_emit, tk);
#ifdef HR_SCAN_TIMING
        n_items++;
#endif
    }
#ifdef HR_SCAN_TIMING
    if (a.dbg && threadIdx.x == 0) {
        long long* o = a.dbg + blockIdx.x * 8;
        o[0] = t_pop; o[1] = t_setup; o[2] = t_mfma; o[3] = t_sel; o[4] = t_stage; o[5] = t_bar; o[6] = t_emit; o[7] = n_items;
        long long* o2 = a.dbg + 4096 + blockIdx.x * 4;
        o2[0] = n_blocks; o2[1] = n_cand_blocks; o2[2] = n_prunes;
    }
#endif
}

template <int DT, int NCS>
inline hipError_t launch_scan_ncs(int d, const ScanArgs& a, int grid, size_t lds, hipStream_t s)
{
#define HR_SCAN_CASE(KS)                                                                           \
    case KS * 32: {                                                                                \
        auto kern = k_scan<DT, KS, NCS>;                                                           \
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e != hipSuccess) return e;                                                             \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(kScanWaves * 64), lds, s, a);                    \
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

template <int DT>
inline hipError_t launch_scan_dtype(int d, const ScanArgs& a, int ncs, int grid, size_t lds, hipStream_t s)
{
    return ncs == 2 ? launch_scan_ncs<DT, 2>(d, a, grid, lds, s) : launch_scan_ncs<DT, 1>(d, a, grid, lds, s);
}

// ------------------------------------------------------------------------------------------
// Threshold seeding.  One wave per query scores the first rows of the query's best-ranked
// list (with the very MFMA sequence of k_scan, so the keys are the ones the scan will compute
// for these rows) and publishes the k-th best of them as the query's starting lower bound.
// On clustered data that bound already excludes nearly every row of the other probed lists,
// which then cost the scan one compare per score instead of a candidate insertion.  Any k
// real candidates give a valid bound, so the result of the search does not depend on this.
constexpr int kSeedRowsMax = 192;

template <int DT, int KSTEPS>
__global__ __launch_bounds__(256) void k_seed(SeedArgs a)
{
    using T = StoreTraits<DT>;
    constexpr int NC = T::nc;
    constexpr int d = KSTEPS * 32;
    constexpr int rowb = d * T::esize;
    __shared__ uint32_t s_keys[4][kSeedRowsMax];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int64_t q = (int64_t)blockIdx.x * 4 + wave;
    if (q >= a.nq) return;
    const int l = a.probe[q * a.nprobe];
    if (l < 0 || l >= a.nlist) return;
    const int row0 = a.list_off[l];
    const int nrows = min(a.list_off[l + 1] - row0, a.seed_rows);
    if (nrows < a.k) return;
    const int g = lane >> 4;
    const int part = (NC == 8) ? ((lane >> 3) & 1) : 0;
    const bool bcol = (lane & (NC - 1)) == 0;          // MFMA column 0 (and its lo twin)
    u32x4 bfrag[KSTEPS];
    {
        const size_t qrow = (NC == 8) ? ((size_t)q * 2 + part) : (size_t)q;
        const char* qp = (const char*)a.qop + qrow * (size_t)(d * 2) + g * 16;
#pragma unroll
        for (int t = 0; t < KSTEPS; t++) bfrag[t] = bcol ? *(const u32x4*)(qp + t * 64) : u32x4{0, 0, 0, 0};
    }
    uint32_t* keys = s_keys[wave];
    const int nblk = (nrows + 15) / 16;
    for (int blk = 0; blk < nblk; blk++) {
        const int r = row0 + blk * 16 + (lane & 15);
        const bool rv = r < row0 + nrows;
        const char* rp = (const char*)a.rows + (size_t)r * rowb;
        floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < KSTEPS; t++) {
            if constexpr (DT == HR_F32) {
                float x[8];
                u32x4 v0 = rv ? *(const u32x4*)(rp + t * 128 + g * 32) : u32x4{0, 0, 0, 0};
                u32x4 v1 = rv ? *(const u32x4*)(rp + t * 128 + g * 32 + 16) : u32x4{0, 0, 0, 0};
                const floatx4 f0 = __builtin_bit_cast(floatx4, v0), f1 = __builtin_bit_cast(floatx4, v1);
#pragma unroll
                for (int i = 0; i < 4; i++) { x[i] = f0[i]; x[4 + i] = f1[i]; }
                half8 hi, lo;
#pragma unroll
                for (int i = 0; i < 8; i++) {
                    _Float16 h = (_Float16)x[i];
                    hi[i] = h;
                    lo[i] = (_Float16)((x[i] - (float)h) * 2048.0f);
                }
                half8 b = __builtin_bit_cast(half8, bfrag[t]);
                acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(hi, b, acc0, 0, 0, 0);
                acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(lo, b, acc1, 0, 0, 0);
            } else {
                u32x4 v = rv ? *(const u32x4*)(rp + t * 64 + g * 16) : u32x4{0, 0, 0, 0};
                if constexpr (DT == HR_F16) {
                    half8 b = __builtin_bit_cast(half8, bfrag[t]);
                    if (t & 1) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, v), b, acc1, 0, 0, 0);
                    else       acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, v), b, acc0, 0, 0, 0);
                } else {
                    bf16x8 b = __builtin_bit_cast(bf16x8, bfrag[t]);
                    if (t & 1) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v), b, acc1, 0, 0, 0);
                    else       acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, v), b, acc0, 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++) {
            float dot;
            if constexpr (DT == HR_F32) {
                float t0 = __shfl_xor(acc0[r4], 8);
                float t1 = __shfl_xor(acc1[r4], 8);
                dot = acc0[r4] + (t0 + acc1[r4]) * (1.0f / 2048.0f) + t1 * (1.0f / 4194304.0f);
            } else if constexpr (DT == HR_BF16) {
                float v = acc0[r4] + acc1[r4];
                dot = v + __shfl_xor(v, 8);
            } else {
                dot = acc0[r4] + acc1[r4];
            }
            const int row = row0 + blk * 16 + g * 4 + r4;
            if ((lane & 15) == 0 && row < row0 + nrows) {
                float key = a.l2 ? (2.0f * dot - a.row_norm[row]) : dot;
                keys[blk * 16 + g * 4 + r4] = enc_key(key);
            }
        }
    }
    wave_sync();
    // k-th largest of the nrows keys (binary radix select, as in wave_select)
    uint32_t e[3];
    unsigned long long alive[3];
#pragma unroll
    for (int m = 0; m < 3; m++) {
        const int idx = lane + 64 * m;
        e[m] = idx < nrows ? keys[idx] : 0u;
        alive[m] = __builtin_amdgcn_ballot_w64(idx < nrows);
    }
    int need = a.k;
    uint32_t kth = 0;
    for (int b = 31; b >= 0; b--) {
        const uint32_t bit = 1u << b;
        unsigned long long ones[3];
        int c1 = 0;
#pragma unroll
        for (int m = 0; m < 3; m++) {
            ones[m] = alive[m] & __builtin_amdgcn_ballot_w64((e[m] & bit) != 0);
            c1 += __builtin_popcountll(ones[m]);
        }
        if (c1 >= need) {
            kth |= bit;
#pragma unroll
            for (int m = 0; m < 3; m++) alive[m] = ones[m];
        } else {
            need -= c1;
#pragma unroll
            for (int m = 0; m < 3; m++) alive[m] &= ~ones[m];
        }
    }
    // a few units in the last place lower, in case a later pass rounds a sum differently
    if (lane == 0) atomicMax(&a.thr[q], kth > 8u ? kth - 8u : 0u);
}

template <int DT>
inline hipError_t launch_seed_dtype(int d, const SeedArgs& a, hipStream_t s)
{
    if (a.nq <= 0) return hipSuccess;
    const dim3 grid((unsigned)((a.nq + 3) / 4));
#define HR_SEED_CASE(KS) case KS * 32: hipLaunchKernelGGL((k_seed<DT, KS>), grid, dim3(256), 0, s, a); return hipGetLastError();
    switch (d) {
        HR_SEED_CASE(2)
        HR_SEED_CASE(4)
        HR_SEED_CASE(8)
        HR_SEED_CASE(16)
        HR_SEED_CASE(24)
        HR_SEED_CASE(32)
    default: return hipErrorInvalidValue;
    }
#undef HR_SEED_CASE
}

}  // namespace hr
