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
//   HR_F16X2 (internal) the same arithmetic on rows that were split into hi and lo tables
//            beforehand (the centroid table: the coarse step of Section 2.2 runs this kernel
//            in "dense" mode, all queries against all rows, and writes every key out).
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

// value of lane ^ 8 (the other half of a row of 16 lanes: rotation by 8 inside the row, a
// data-parallel-primitive operand modifier, no LDS round trip)
__device__ __forceinline__ float lane_xor8(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128 /* row_ror:8 */, 0xf, 0xf, false));
}

__device__ __forceinline__ int lanes_below(unsigned long long mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// ---- global memory -> LDS without passing through registers (global_load_lds).  Every lane
// gives a byte offset from a wave-uniform base address; the 64 chunks of a wave land next to
// each other from the wave-uniform LDS address on (lane * 16 or lane * 4 bytes in).
// Written as inline assembly on purpose: when the compiler knows of such a load it makes every
// later LDS read wait for all of them, which would undo the prefetching.  The loads complete
// in order and are counted by vmcnt, so "all but the n youngest have landed" is wait_vmcnt<n>;
// loads the compiler issues itself in between only make that wait longer, never shorter.
// (m0 is reserved: the compiler sets it immediately before each of its own uses.  The s_nop is
// the wait state between a scalar write of m0 and a memory instruction that reads it; inside
// inline assembly nobody else would insert it.)
__device__ __forceinline__ uint32_t lds_addr(const void* p)
{
    return (uint32_t)(size_t)(__attribute__((address_space(3))) const char*)p;
}
__device__ __forceinline__ void lds_dma16(const void* base, uint32_t byte_off, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" :: "s"(lds), "v"(byte_off), "s"(base) : "memory");
}
// the same marked non-temporal: rows that nobody else will ask for (a list scanned by one work item) should not
// push the rows that several work items share out of the L2
__device__ __forceinline__ void lds_dma16_nt(const void* base, uint32_t byte_off, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt" :: "s"(lds), "v"(byte_off), "s"(base) : "memory");
}
__device__ __forceinline__ void lds_dma4(const void* base, uint32_t byte_off, uint32_t lds)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" :: "s"(lds), "v"(byte_off), "s"(base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// inclusive prefix sum over the 64 lanes of a wave (row shifts inside each group of 16 lanes,
// then the last lane of rows 0..2 added to the rows after it)
__device__ __forceinline__ int wave_prefix_sum(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return v;
}

// Lower edge of histogram bin b of a query whose bin 0 starts at base and whose bins are w
// wide; one expression, used wherever a key is binned or a bound is derived, so that a key
// counted in bin b is never below the edge that later readers compute for b.
__device__ __forceinline__ float hist_edge(float base, float w, int b) { return __builtin_fmaf((float)b, w, base); }

// Keep the k best of the n (> k) candidates in buf[0..n): afterwards buf[0..k) holds them, in
// no particular order.  Order: key descending, then label ascending (label = row number when
// ids == nullptr; labels are only fetched when equal keys straddle the k-th place).
// Binary radix select on the 32 key bits: the cost does not depend on n.  Called by a whole
// converged wave with wave-uniform arguments.  Returns the k-th best key.
// Label of a candidate for tie-breaking and output: rows with the top bit set are entries of
// a carried result (index into ext), the others stored rows.
constexpr uint32_t kCarried = 0x80000000u;
__device__ __forceinline__ int64_t label_of(uint32_t row, const int64_t* ids, const int64_t* ext)
{
    if (row & kCarried) return ext[row & ~kCarried];
    return ids ? ids[row] : (int64_t)row;
}

template <int CAPE>   // entries held per lane: CAPE * 64 >= n
__device__ __forceinline__ uint32_t wave_select(Cand* buf, int n, int k, const int64_t* ids, const int64_t* ext = nullptr)
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
            label[m] = mine ? label_of(e[m].row, ids, ext) : INT64_MAX;
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
template <> struct StoreTraits<HR_F16X2> { static constexpr int esize = 2, planes = 2, nc = 8; };

// NW = waves per workgroup (4: one per SIMD, each may use all 512 registers; 8: two per SIMD
// with 256 registers each, so that one wave's MFMAs run while the other selects or waits).
// NCS = 16-column MFMA sets per wave (1 or 2).  Every wave owns NCS * nc query columns, so a
// work item covers NW * NCS * nc queries of a bucket; all waves share the staged rows.
//
// Two ways of staging a block of 16 rows in LDS:
//   direct (16-bit storage): global_load_lds moves 16-byte chunks from HBM straight into LDS,
//     no registers and no LDS store instructions in between.  Such a load writes the 64 chunks
//     of a wave next to each other, so rows cannot be padded; instead chunk c of row r sits at
//     position c ^ (r & 15) of its row, which spreads the 16 rows of an MFMA fragment read over
//     all banks.  Up to four blocks are in flight or waiting in LDS ahead of the one in use.
//   through registers (float32 storage): rows are split into binary16 hi and lo planes on the
//     way, from a ring of prefetch registers into two padded buffers.
constexpr int kAcc = 2;                       // accumulators per column set (independent MFMA chains)
constexpr int kMaxAhead = 4;                  // most blocks staged ahead of the one in use (direct)

template <int DT, int KSTEPS, int NCS, int NW>
struct ScanShape {
    static constexpr int nw = NW;
    static constexpr int threads = NW * 64;
    static constexpr int d = KSTEPS * 32;
    static constexpr int planes = StoreTraits<DT>::planes;
    static constexpr bool direct = DT != HR_F32;                   // (HR_F16X2: two planes, both moved directly)
    static constexpr int rowb = d * StoreTraits<DT>::esize;        // bytes of one stored row
    static constexpr int cpr = rowb / 16;                          // 16-byte chunks per stored row
    static constexpr int swz = (cpr < 16 ? cpr : 16) - 1;          // row bits xor-ed into the chunk position
    static constexpr int rowp = direct ? rowb : d * 2 + kRowPad;   // bytes of one staged row (one plane)
    static constexpr int plane_bytes_padded = kBlockRows * rowp;
    static constexpr int chunks = kBlockRows * cpr;                // 16-byte chunks per block
    static constexpr int nfw = NW;                                 // waves that move rows: all
    static constexpr int nld = (chunks + nfw * 64 - 1) / (nfw * 64);   // chunks per thread per block
    // (direct: every wave always issues nld loads, so a buffer is a whole number of them)
    static constexpr int plane_bytes = direct ? nld * nfw * 1024 : plane_bytes_padded;
    static constexpr int buf_bytes = plane_bytes * planes;
    static constexpr int lpf = planes * nld + 1;                   // direct: loads per wave per block (chunks + norms)
    // k-steps whose row fragments are fetched from LDS together, ahead of their MFMAs
    static constexpr int grp = scan_group(DT, KSTEPS, NW);
    // register path: row blocks kept in flight in registers ahead of the one being staged
    static constexpr int pf = scan_prefetch(DT, KSTEPS, NCS, NW);
    static constexpr int wcols = StoreTraits<DT>::nc * NCS;        // query columns per wave
    static constexpr int cw = wcols * NW;                          // query columns per item
};

// s_waitcnt immediate that waits for all but n vector-memory operations (n <= 63) and for
// nothing else
__host__ __device__ constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }


// Every thread always loads (chunks past the end of the segment re-read its last chunk; the
// rows they would belong to are masked out of the selection): an unconditional load keeps the
// ring registers free of the zero-fill writes that would otherwise have to wait for the
// loads still in flight.
template <typename S>
__device__ __forceinline__ void load_block(const char* src, int valid_chunks, u32x4 (&regs)[S::nld], bool once)
{
    // (once: nobody else reads these rows: non-temporal loads, so that they do not displace shared rows in the L2)
    if (once) {
#pragma unroll
        for (int m = 0; m < S::nld; m++) {
            int c = min((int)threadIdx.x + S::threads * m, valid_chunks - 1);
            regs[m] = __builtin_nontemporal_load((const u32x4*)(src + (size_t)c * 16));
        }
    } else {
#pragma unroll
        for (int m = 0; m < S::nld; m++) {
            int c = min((int)threadIdx.x + S::threads * m, valid_chunks - 1);
            regs[m] = *(const u32x4*)(src + (size_t)c * 16);
        }
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

// 16 staged rows x NA column sets x d: the MFMA chain of one block.  acc[s][*] are the partial
// accumulators of set s (for HR_F32: [0] hi-row and [1] lo-row products; else summed at the end).  The row fragments
// are fetched from LDS a group of k-steps ahead of the MFMAs that use them (the scheduling
// barriers keep the compiler from sinking each read next to its use, which would expose the
// LDS latency 24 times per block).  The fragment of k-step t is at ap[t & 3] + (t >> 2) * 256:
// with padded rows the four bases are 64 bytes apart, with the xor-ed chunk positions of the
// direct staging they are permuted per lane.
template <int DT, int KSTEPS, int NCS, int NA, typename S>
__device__ __forceinline__ void mfma_block(const char* const (&ap)[4], const u32x4 (&bfrag)[NCS][KSTEPS], floatx4 (&acc)[NCS][kAcc])
{
    constexpr int G = S::grp;                        // k-steps per group
    constexpr int NG = KSTEPS / G;
    constexpr int AM = (NA == 1 ? kAcc : 2) - 1;     // a lone set spreads over all accumulators
    constexpr int P = StoreTraits<DT>::planes;
    static_assert(KSTEPS % G == 0, "k-steps must split into whole groups");
#pragma unroll
    for (int s = 0; s < NA; s++)
#pragma unroll
        for (int i = 0; i < kAcc; i++) acc[s][i] = floatx4{0.f, 0.f, 0.f, 0.f};
    u32x4 af[2][P][G];
#pragma unroll
    for (int i = 0; i < G; i++)
#pragma unroll
        for (int pl = 0; pl < P; pl++) af[0][pl][i] = *(const u32x4*)(ap[i & 3] + pl * S::plane_bytes + (i >> 2) * 256);
#pragma unroll
    for (int gi = 0; gi < NG; gi++) {
        if (gi + 1 < NG) {
#pragma unroll
            for (int i = 0; i < G; i++)
#pragma unroll
                for (int pl = 0; pl < P; pl++)
                    af[(gi + 1) & 1][pl][i] = *(const u32x4*)(ap[((gi + 1) * G + i) & 3] + pl * S::plane_bytes + (((gi + 1) * G + i) >> 2) * 256);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < G; i++) {
            const int t = gi * G + i;
#pragma unroll
            for (int s = 0; s < NA; s++) {
                if constexpr (StoreTraits<DT>::planes == 2) {
                    half8 b = __builtin_bit_cast(half8, bfrag[s][t]);
                    acc[s][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, af[gi & 1][0][i]), b, acc[s][0], 0, 0, 0);
                    acc[s][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, af[gi & 1][1][i]), b, acc[s][1], 0, 0, 0);
                } else if constexpr (DT == HR_F16) {
                    half8 b = __builtin_bit_cast(half8, bfrag[s][t]);
                    acc[s][t & AM] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, af[gi & 1][0][i]), b, acc[s][t & AM], 0, 0, 0);
                } else {
                    bf16x8 b = __builtin_bit_cast(bf16x8, bfrag[s][t]);
                    acc[s][t & AM] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[gi & 1][0][i]), b, acc[s][t & AM], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Two blocks that lie ready in LDS, multiplied back to back as one chain of 2 * KSTEPS k-steps: the first
// fragments of the second block are fetched while the last MFMAs of the first are issued (a block started on
// its own begins with a round trip to LDS during which the wave has nothing to issue), and `between` (the
// filter of the first block) runs after the first MFMAs of the second block have been handed to the matrix pipe.
template <int DT, int KSTEPS, int NCS, int NA, typename S, typename F>
__device__ __forceinline__ void mfma_pair(const char* const (&ap0)[4], const char* const (&ap1)[4], const u32x4 (&bfrag)[NCS][KSTEPS],
                                          floatx4 (&acc0)[NCS][kAcc], floatx4 (&acc1)[NCS][kAcc], F&& between)
{
    constexpr int G = S::grp;
    constexpr int NG = KSTEPS / G;
    constexpr int AM = (NA == 1 ? kAcc : 2) - 1;
    constexpr int P = StoreTraits<DT>::planes;
    static_assert(KSTEPS % G == 0, "k-steps must split into whole groups");
    static_assert(NG % 2 == 0, "the fragment buffers alternate: an even number of groups per block");
#pragma unroll
    for (int s = 0; s < NA; s++)
#pragma unroll
        for (int i = 0; i < kAcc; i++) { acc0[s][i] = floatx4{0.f, 0.f, 0.f, 0.f}; acc1[s][i] = floatx4{0.f, 0.f, 0.f, 0.f}; }
    u32x4 af[2][P][G];
    // (every index below is a compile-time constant: the loop over the groups is unrolled by the type system,
    // so that the operand and accumulator arrays stay in registers)
    auto fetch = [&](auto gc) __attribute__((always_inline)) {       // group gg of the 2 * NG groups of the pair
        constexpr int gg = decltype(gc)::value;
        constexpr int g0 = (gg < NG ? gg : gg - NG) * G;
#pragma unroll
        for (int i = 0; i < G; i++)
#pragma unroll
            for (int pl = 0; pl < P; pl++) {
                if constexpr (gg < NG) af[gg & 1][pl][i] = *(const u32x4*)(ap0[(g0 + i) & 3] + pl * S::plane_bytes + ((g0 + i) >> 2) * 256);
                else                   af[gg & 1][pl][i] = *(const u32x4*)(ap1[(g0 + i) & 3] + pl * S::plane_bytes + ((g0 + i) >> 2) * 256);
            }
    };
    auto group = [&](auto gc, floatx4 (&acc)[NCS][kAcc]) __attribute__((always_inline)) {
        constexpr int gg = decltype(gc)::value;
#pragma unroll
        for (int i = 0; i < G; i++) {
            const int t = (gg < NG ? gg : gg - NG) * G + i;
#pragma unroll
            for (int s = 0; s < NA; s++) {
                if constexpr (StoreTraits<DT>::planes == 2) {
                    half8 b = __builtin_bit_cast(half8, bfrag[s][t]);
                    acc[s][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, af[gg & 1][0][i]), b, acc[s][0], 0, 0, 0);
                    acc[s][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, af[gg & 1][1][i]), b, acc[s][1], 0, 0, 0);
                } else if constexpr (DT == HR_F16) {
                    half8 b = __builtin_bit_cast(half8, bfrag[s][t]);
                    acc[s][t & AM] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, af[gg & 1][0][i]), b, acc[s][t & AM], 0, 0, 0);
                } else {
                    bf16x8 b = __builtin_bit_cast(bf16x8, bfrag[s][t]);
                    acc[s][t & AM] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, af[gg & 1][0][i]), b, acc[s][t & AM], 0, 0, 0);
                }
            }
        }
    };
    fetch(std::integral_constant<int, 0>{});
    static_for<2 * NG>([&](auto gc) __attribute__((always_inline)) {
        constexpr int gg = decltype(gc)::value;
        if constexpr (gg + 1 < 2 * NG) fetch(std::integral_constant<int, gg + 1>{});
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (gg < NG) group(gc, acc0); else group(gc, acc1);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (gg == NG) between();
    });
}

// prune with as few register slots per lane as the buffer capacity needs
__device__ __forceinline__ uint32_t select_k(Cand* buf, int n, int k, int cap, const int64_t* ids)
{
    if (cap <= 64) return wave_select<1>(buf, n, k, ids);
    if (cap <= 128) return wave_select<2>(buf, n, k, ids);
    return wave_select<3>(buf, n, k, ids);
}

template <int DT, int KSTEPS, int NCS, int NW, bool GS>   // GS = a.gsel
__global__ __launch_bounds__(NW * 64, 1) void k_scan(ScanArgs a)
{
    using S = ScanShape<DT, KSTEPS, NCS, NW>;
    using T = StoreTraits<DT>;
    constexpr int NC = T::nc;
    constexpr int WC = S::wcols;
    constexpr int PF = S::pf;
    constexpr int NLD = S::nld;
    extern __shared__ __align__(16) char smem[];
    // staging buffers in LDS: a.nbuf of them (direct) or 2 (through registers); block blk of an
    // item uses buffer blk % NB, and the blocks up to blk + NB - 1 are on their way meanwhile
    // With 4 or 6 buffers (direct) the blocks go in pairs: one barrier per two blocks, the next pair
    // on its way meanwhile.  A barrier per block keeps the two waves of a SIMD in step (both
    // want the matrix pipeline, then both the vector ALU); between the barriers of a pair they
    // drift apart and overlap.
    const int NB = S::direct ? a.nbuf : 2;
    const bool pairs = S::direct && (NB == 4 || NB == 6);
    const int D = pairs ? NB - 2 : NB - 1;         // blocks requested ahead of the one in use
    // LDS: [NB staging buffers][selection buffers cw*cap][row norms NB x 16][item]
    // (GS: the selection buffers are the item's result slots in global memory instead: a
    // wave alone writes and reads the buffers of its columns, candidates are few, and LDS is
    // left to the row buffers)
    char* stage = smem;
    Cand* sel = (Cand*)(smem + NB * S::buf_bytes);
    float* nstage = (float*)(sel + (GS ? 0 : S::cw * a.cap));
    int* s_item = (int*)(nstage + NB * kBlockRows);

    const int lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4;                       // k-group / output row group
    const int jcol = lane & (NC - 1);              // column inside a set
    const int part = (NC == 8) ? ((lane >> 3) & 1) : 0;   // 0 = hi, 1 = lo operand column
    const bool owner = (NC == 16) || part == 0;    // lane whose accumulator holds the full dot
    Cand* mysel = sel + (wave * WC) * a.cap;
    const int seg_rows = a.dense_seg_rows;                   // (dense mode only: the items of the lists carry their rows)
    const int myx = blockIdx.x & 7;                // workgroups are dealt round-robin to the 8 XCDs
    int drained = 0;                               // thread 0: queues found empty

    // ---- per-lane constants of the staging layout
    // row fragment of k-step t of this lane: abase[t & 3] + (t >> 2) * 256 inside a buffer
    int abase[4];
    // direct: byte offset inside a stored block of the chunk that load m of this lane moves
    uint32_t goff[NLD];
    {
        const int i = lane & 15;
        if constexpr (S::direct) {
            const int hi = (i & S::swz) >> 2, lo = i & 3;
#pragma unroll
            for (int j = 0; j < 4; j++) abase[j] = i * S::rowp + 64 * (j ^ hi) + 16 * (g ^ lo);
#pragma unroll
            for (int m = 0; m < NLD; m++) {
                const int L = (m * S::nfw + wave) * 64 + lane;  // chunk position inside the buffer
                const int r = L / S::cpr, pos = L % S::cpr;
                goff[m] = (uint32_t)(min(r, kBlockRows - 1) * S::cpr + (pos ^ (r & S::swz))) * 16u;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; j++) abase[j] = i * S::rowp + g * 16 + j * 64;
#pragma unroll
            for (int m = 0; m < NLD; m++) goff[m] = 0;
        }
    }

    for (;;) {
        if (threadIdx.x == 0) {
            int item = -1;
            if (a.dense) {
                int i = atomicAdd(a.work_counter, 1);
                if (i < a.dense_items) item = i;
            } else {
                // own XCD's queue first (its items share list segments through this XCD's L2),
                // then the others' leftovers.  A queue entry is the whole record of the item.
                for (int t = 0; t < 8 && item < 0; t++) {
                    int x = (myx + t) & 7;
                    if (drained & (1 << x)) continue;
                    int pos = atomicAdd(&a.xq_head[x], 1);
                    if (pos < a.xq_count[x]) {
                        const int4* rec = a.xq_rec + ((size_t)x * a.xq_stride + pos) * 2;
                        const int4 r0 = rec[0], r1 = rec[1];
                        s_item[1] = r0.x; s_item[2] = r0.y; s_item[3] = r0.z; s_item[4] = r0.w;
                        s_item[5] = r1.x; s_item[6] = r1.y;
                        item = 0;
                    } else {
                        drained |= 1 << x;
                    }
                }
            }
            s_item[0] = item;
        }
        __syncthreads();
        const int item = __builtin_amdgcn_readfirstlane(s_item[0]);
        if (item < 0) break;

        // ---- decode the work item
        int qt, row0, row_end, w, boff, slot0 = 0;
        if (a.dense) {
            const int seg = item / a.dense_nqt;
            qt = item - seg * a.dense_nqt;
            row0 = seg * seg_rows;
            row_end = min(a.dense_nrows, row0 + seg_rows);
            w = a.nq;
            boff = 0;
        } else {
            row0 = __builtin_amdgcn_readfirstlane(s_item[1]);
            row_end = row0 + __builtin_amdgcn_readfirstlane(s_item[2]);
            boff = __builtin_amdgcn_readfirstlane(s_item[3]);
            w = __builtin_amdgcn_readfirstlane(s_item[4]);
            qt = __builtin_amdgcn_readfirstlane(s_item[5]);
            slot0 = __builtin_amdgcn_readfirstlane(s_item[6]);
        }
        const int nrows = row_end - row0;
        const int nblk = (nrows + kBlockRows - 1) / kBlockRows;
        Cand* const gsel = a.slot_ent + ((size_t)slot0 + wave * WC) * (size_t)a.slot_stride;   // (GS: slot_stride = cap)
        const char* src = (const char*)a.rows + (size_t)row0 * S::rowb;
        const char* src_lo = S::planes == 2 ? (const char*)a.rows_lo + (size_t)row0 * S::rowb : src;

        // ---- staging.  Requests for a block past the end of the segment fetch its last block
        // again (nobody reads the copy): every wave then has the same, fixed number of loads
        // in flight at every point of the loop, which is what the wait counts below rely on.
        //
        // direct: block blk -> buffer buf, straight from HBM; the squared norms of its rows go
        // to a place of this wave's own (each wave fetches its own copy: 64 bytes)
        const bool stream_once = !a.dense && w <= S::cw;   // the only work item that reads these rows
        auto fill_direct = [&](int blk, int buf) __attribute__((always_inline)) {
            const int bl = min(blk, nblk - 1);
            const int valid = min(nrows - bl * kBlockRows, kBlockRows);
#pragma unroll
            for (int pl = 0; pl < S::planes; pl++) {
                const char* bsrc = (pl == 0 ? src : src_lo) + (size_t)bl * kBlockRows * S::rowb;
                const uint32_t dst = lds_addr(stage) + buf * S::buf_bytes + pl * S::plane_bytes + wave * 1024;
                if (valid == kBlockRows) {
                    if (stream_once) {
#pragma unroll
                        for (int m = 0; m < NLD; m++) lds_dma16_nt(bsrc, goff[m], dst + m * S::nfw * 1024);
                    } else {
#pragma unroll
                        for (int m = 0; m < NLD; m++) lds_dma16(bsrc, goff[m], dst + m * S::nfw * 1024);
                    }
                } else {
                    // ragged last block: rows past the end repeat the last valid one (their scores
                    // are masked out of the selection)
#pragma unroll
                    for (int m = 0; m < NLD; m++) {
                        const int L = (m * S::nfw + wave) * 64 + lane;
                        const int r = L / S::cpr, pos = L % S::cpr;
                        const uint32_t o = (uint32_t)(min(r, valid - 1) * S::cpr + (pos ^ (r & S::swz))) * 16u;
                        lds_dma16(bsrc, o, dst + m * S::nfw * 1024);
                    }
                }
            }
            // (every wave writes the same 16 norms: the same number of loads per wave; the inner
            // product needs none)
            if (a.l2 && lane < kBlockRows)
                lds_dma4(a.row_norm + row0 + bl * kBlockRows, (uint32_t)min(lane, valid - 1) * 4u,
                         lds_addr(nstage) + buf * (kBlockRows * 4));
        };
        // through registers: a ring of PF blocks in flight
        u32x4 ring[S::direct ? 1 : PF][NLD];
        float nring[S::direct ? 1 : PF];
        auto block_chunks = [&](int blk) __attribute__((always_inline)) { return min(nrows - min(blk, nblk - 1) * kBlockRows, kBlockRows) * S::cpr; };
        auto block_src = [&](int blk) __attribute__((always_inline)) { return src + (size_t)min(blk, nblk - 1) * kBlockRows * S::rowb; };
        auto load_norm = [&](int blk) __attribute__((always_inline)) {
            const int r = min(row0 + min(blk, nblk - 1) * kBlockRows + (int)(threadIdx.x & (kBlockRows - 1)), row_end - 1);
            return a.row_norm[r];
        };

        // ---- first row blocks on their way before anything else
        if constexpr (S::direct) {
            for (int i = 0; i < D; i++) fill_direct(i, i);
        } else {
            load_block<S>(block_src(0), block_chunks(0), ring[0], stream_once);
            nring[0] = load_norm(0);
        }

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
            thr[s] = (owner && col_ok[s]) ? dec_key(a.thr[q[s]]) : __builtin_inff();
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

        if constexpr (!S::direct) {
            // Everything loaded so far (query operands, thresholds, first row block) is waited
            // for here, once, and only then are the next PF blocks requested, oldest ring slot
            // first.  The loop is thus entered with exactly the loads in flight, in exactly the
            // order, that every later iteration sees; the compiler's wait-count analysis can
            // then let the staging of a block wait for that block alone, with the PF-1 younger
            // blocks still in flight, instead of draining the ring.
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
            stage_block<DT, S>(stage, ring[0]);
            nstage[threadIdx.x & (kBlockRows - 1)] = nring[0];      // (same value from several threads)
            static_for<PF>([&](auto pc) __attribute__((always_inline)) {
                constexpr int slot = (decltype(pc)::value + 1) % PF;
                load_block<S>(block_src(decltype(pc)::value + 1), block_chunks(decltype(pc)::value + 1), ring[slot], stream_once);
                nring[slot] = load_norm(decltype(pc)::value + 1);
            });
        } else {
            // The query operands and thresholds are waited for here, once (the first blocks
            // with them): if the compiler still counted them as in flight inside the loop it
            // would wait for "everything" at their first use in every iteration, and that
            // includes the blocks on their way to LDS.
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
        }

        // ---- the blocks of the segment.  Per block (direct staging): (1) this wave's part of
        // the block has landed, (2) barrier: so has everybody's, and nobody reads the previous
        // block any more, (3) request block blk + D into the buffer the previous block leaves,
        // (4) multiply, (5) select.
        //
        // ---- dense scoring: the keys of a block are written out at the start of the next
        // step, right after the barrier.  Stores count in vmcnt like the requests for blocks,
        // and may complete in any order relative to them, so the wait at the top of a step has
        // to assume they are still outstanding; issued here they have a whole step to complete.
        floatx4 held[NCS];
        int held_rbase = -1;
        auto flush_keys = [&]() __attribute__((always_inline)) {
            if (held_rbase < 0) return;
#pragma unroll
            for (int s = 0; s < NCS; s++) {
                if (s < nact && owner && col_ok[s]) {
                    float* out = a.key_out + (size_t)q[s] * a.dense_nrows + held_rbase;
                    if (held_rbase + 3 < row_end && (a.dense_nrows & 3) == 0) {
                        *(floatx4*)out = held[s];
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; r++)
                            if (held_rbase + r < row_end) out[r] = held[s][r];
                    }
                }
            }
            held_rbase = -1;
        };

        // ---- selection over the scores of one block: acc = accumulators of the block, nrm =
        // squared norms of this lane's 4 rows, rbase = first of those rows
        auto select_block = [&](const floatx4 (&acc)[NCS][kAcc], const floatx4 nrm, const int rbase) __attribute__((always_inline)) {
#pragma unroll
            for (int s = 0; s < NCS; s++) {
                if (s >= nact) break;
                // ---- keys of this lane's 4 (row, column) pairs of set s.  The common case is
                // that none reaches the column's threshold: that is decided with one compare
                // of the largest of the four (thr is +inf in lanes that own no query column).
                float key[4];
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    float dot;
                    if constexpr (T::planes == 2) {
                        float t0 = lane_xor8(acc[s][0][r]);      // hi rows x lo query
                        float t1 = lane_xor8(acc[s][1][r]);      // lo rows x lo query
                        dot = acc[s][0][r] + (t0 + acc[s][1][r]) * (1.0f / 2048.0f) + t1 * (1.0f / 4194304.0f);
                    } else if constexpr (DT == HR_BF16) {
                        float v = acc[s][0][r] + acc[s][1][r];
                        dot = v + lane_xor8(v);
                    } else {
                        dot = acc[s][0][r] + acc[s][1][r];
                    }
                    key[r] = dot;
                }
                if (a.l2) {
#pragma unroll
                    for (int r = 0; r < 4; r++) key[r] = 2.0f * key[r] - nrm[r];
                }
                if (a.key_out != nullptr) {
                    // dense scoring only: every key goes to its place in the [query, row] table,
                    // one block late (see flush_keys)
                    held[s] = floatx4{key[0], key[1], key[2], key[3]};
                    held_rbase = rbase;
                    continue;
                }
                const float best = fmaxf(fmaxf(key[0], key[1]), fmaxf(key[2], key[3]));
                // ---- append what reaches the column's threshold
                if (__builtin_amdgcn_ballot_w64(best >= thr[s]) != 0) {
                    bool pass[4];
#pragma unroll
                    for (int r = 0; r < 4; r++) pass[r] = key[r] >= thr[s] && (rbase + r < row_end);
                    Cand* ssel = mysel + (s * NC) * a.cap;
                    Cand* gs = gsel + (s * NC) * a.cap;
                    // slot of each new candidate = column count + candidates of the same
                    // column in earlier row slots and in lower lanes of this row slot
                    int add = 0;
#pragma unroll
                    for (int r = 0; r < 4; r++) {
                        const unsigned long long mine = __builtin_amdgcn_ballot_w64(pass[r]) & colmask;
                        if (pass[r]) {
                            const int pos = ccnt[s] + add + __builtin_popcountll(mine & below);
                            const Cand cd{enc_key(key[r]), (uint32_t)(rbase + r)};
                            if (GS) gs[jcol * a.cap + pos] = cd;
                            else ssel[jcol * a.cap + pos] = cd;
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
                        uint32_t kth = GS ? select_k(gs + col * a.cap, n, a.k, a.cap, a.row_ids)
                                              : select_k(ssel + col * a.cap, n, a.k, a.cap, a.row_ids);
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
        };

        int bi = 0;                                              // blk % NB
        floatx4 accs[2][NCS][kAcc];
        floatx4 nrms[2] = {floatx4{0.f, 0.f, 0.f, 0.f}, floatx4{0.f, 0.f, 0.f, 0.f}};
        // direct staging: (1) this wave's part of block blk has landed, (2) barrier: so has
        // everybody's, and nobody reads block blk-1 any more, (3) request block blk+D into the
        // buffer that one leaves, (4) multiply, (5) select
        auto step_direct = [&](int blk) __attribute__((always_inline)) {
            // all but the D-1 youngest requests of this wave (S::lpf loads each) are done
            if (a.l2) {
                switch (D) {
                case 1: wait_vmcnt<0>(); break;
                case 2: wait_vmcnt<S::lpf>(); break;
                case 3: wait_vmcnt<2 * S::lpf>(); break;
                default: wait_vmcnt<3 * S::lpf>(); break;
                }
            } else {
                switch (D) {
                case 1: wait_vmcnt<0>(); break;
                case 2: wait_vmcnt<S::lpf - 1>(); break;
                case 3: wait_vmcnt<2 * (S::lpf - 1)>(); break;
                default: wait_vmcnt<3 * (S::lpf - 1)>(); break;
                }
            }
            __builtin_amdgcn_s_barrier();
            if (a.key_out != nullptr) flush_keys();
            fill_direct(blk + D, bi == 0 ? NB - 1 : bi - 1);
            if (nact > 0) {
                const char* cur = stage + bi * S::buf_bytes;
                if (a.l2) nrms[0] = *(const floatx4*)(nstage + bi * kBlockRows + g * 4);
                const char* const ap[4] = {cur + abase[0], cur + abase[1], cur + abase[2], cur + abase[3]};
                if (NCS == 2 && nact == 2) mfma_block<DT, KSTEPS, NCS, NCS, S>(ap, bfrag, accs[0]);
                else                       mfma_block<DT, KSTEPS, NCS, 1, S>(ap, bfrag, accs[0]);
                select_block(accs[0], nrms[0], row0 + blk * kBlockRows + g * 4);
            }
            bi = bi + 1 == NB ? 0 : bi + 1;
        };
        // direct staging, 4 buffers: blocks blk and blk+1 between two barriers, blocks blk+2 and
        // blk+3 requested into the two buffers the previous pair leaves
        auto pair_direct = [&](int blk) __attribute__((always_inline)) {
            // (6 buffers: the requests of the pair after the next one may still be on their way)
            if (NB != 6) wait_vmcnt<0>();
            else if (a.l2) wait_vmcnt<2 * S::lpf>();
            else wait_vmcnt<2 * (S::lpf - 1)>();
            __builtin_amdgcn_s_barrier();
            // (the requests of all waves at once keep the address unit busy for a while, and a
            // wave cannot go on before its own are accepted: half of the waves send theirs
            // now, the other half after their first block, when the first half multiplies)
            const bool early = NW != 8 || wave < 4 || nact == 0;
            auto requests = [&]() __attribute__((always_inline)) {
                const int fb = bi + D >= NB ? bi + D - NB : bi + D;     // the buffers the pair before this one used
                fill_direct(blk + D, fb);
                fill_direct(blk + D + 1, fb + 1);
            };
            if (early) requests();
            if (NCS == 1 && S::grp * 2 <= KSTEPS && (KSTEPS / S::grp) % 2 == 0 && nact > 0 && blk + 1 < nblk) {
                // both blocks of the pair as one chain (see mfma_pair); the late requests go out with the
                // filter of the first block
                const char* c0 = stage + bi * S::buf_bytes;
                const char* c1 = c0 + S::buf_bytes;
                if (a.l2) {
                    nrms[0] = *(const floatx4*)(nstage + bi * kBlockRows + g * 4);
                    nrms[1] = *(const floatx4*)(nstage + (bi + 1) * kBlockRows + g * 4);
                }
                const char* const ap0[4] = {c0 + abase[0], c0 + abase[1], c0 + abase[2], c0 + abase[3]};
                const char* const ap1[4] = {c1 + abase[0], c1 + abase[1], c1 + abase[2], c1 + abase[3]};
                if constexpr (NCS == 1 && (KSTEPS / S::grp) % 2 == 0 && S::grp * 2 <= KSTEPS) {
                    mfma_pair<DT, KSTEPS, NCS, 1, S>(ap0, ap1, bfrag, accs[0], accs[1], [&]() __attribute__((always_inline)) {
                        if (!early) requests();
                        select_block(accs[0], nrms[0], row0 + blk * kBlockRows + g * 4);
                    });
                }
                select_block(accs[1], nrms[1], row0 + (blk + 1) * kBlockRows + g * 4);
            } else {
#pragma unroll
                for (int h = 0; h < 2; h++) {
                    if (nact > 0 && blk + h < nblk) {
                        const char* cur = stage + (bi + h) * S::buf_bytes;
                        if (a.l2) nrms[0] = *(const floatx4*)(nstage + (bi + h) * kBlockRows + g * 4);
                        const char* const ap[4] = {cur + abase[0], cur + abase[1], cur + abase[2], cur + abase[3]};
                        if (NCS == 2 && nact == 2) mfma_block<DT, KSTEPS, NCS, NCS, S>(ap, bfrag, accs[0]);
                        else                       mfma_block<DT, KSTEPS, NCS, 1, S>(ap, bfrag, accs[0]);
                        select_block(accs[0], nrms[0], row0 + (blk + h) * kBlockRows + g * 4);
                    }
                    if (h == 0 && !early) requests();
                }
            }
            bi = bi + 2 == NB ? 0 : bi + 2;
        };
        // through registers: (1) barrier: block blk is complete in LDS and nobody reads block
        // blk-1 any more, (2) block blk+1 from the ring into the buffer that one leaves, and
        // its ring slot refilled, (3) multiply, (4) select
        auto step_regs = [&](int blk, auto pc) __attribute__((always_inline)) {
            constexpr int p = decltype(pc)::value;               // ring position
            const bool live = blk < nblk;
            __syncthreads();
            constexpr int pn = (p + 1) % PF;
            stage_block<DT, S>(stage + (bi ^ 1) * S::buf_bytes, ring[pn]);
            nstage[(bi ^ 1) * kBlockRows + (threadIdx.x & (kBlockRows - 1))] = nring[pn];
            load_block<S>(block_src(blk + 1 + PF), block_chunks(blk + 1 + PF), ring[pn], stream_once);
            nring[pn] = load_norm(blk + 1 + PF);
            if (live && nact > 0) {
                const char* cur = stage + bi * S::buf_bytes;
                nrms[0] = *(const floatx4*)(nstage + bi * kBlockRows + g * 4);
                const char* const ap[4] = {cur + abase[0], cur + abase[1], cur + abase[2], cur + abase[3]};
                if (NCS == 2 && nact == 2) mfma_block<DT, KSTEPS, NCS, NCS, S>(ap, bfrag, accs[0]);
                else                       mfma_block<DT, KSTEPS, NCS, 1, S>(ap, bfrag, accs[0]);
                select_block(accs[0], nrms[0], row0 + blk * kBlockRows + g * 4);
            }
            bi ^= 1;
        };
        if constexpr (S::direct) {
            if (pairs) {
                for (int blk = 0; blk < nblk; blk += 2) pair_direct(blk);
            } else {
                for (int blk = 0; blk < nblk; blk++) step_direct(blk);
            }
        } else {
            // (iterations past the last block of a ragged round still stage and load: an early
            // exit would be a path with fewer loads in flight, and the compiler would size
            // every wait in the loop for that path)
            for (int b0 = 0; b0 < nblk; b0 += PF)
                static_for<PF>([&](auto pc) __attribute__((always_inline)) { step_regs(b0 + decltype(pc)::value, pc); });
        }

        if (a.key_out != nullptr) flush_keys();
        // ---- hand what is left to the item's slots: columns with more entries than a slot holds
        // (slot_stride: k, or the whole buffer for small k, when nothing has to be cut) are cut
        // down to the k best first (one at a time, whole wave), then every lane copies one
        // column's entries
        wave_sync();
        if (a.key_out == nullptr) {
            int c = 0;
#pragma unroll
            for (int s = 0; s < NCS; s++) {
                const int v = __shfl(ccnt[s], (lane - s * NC) & 63);
                if (lane >= s * NC && lane < (s + 1) * NC) c = v;
            }
            unsigned long long over = __builtin_amdgcn_ballot_w64(!GS && c > a.slot_stride);
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
            const int n = c > a.slot_stride ? a.k : c;
            if (lane < WC && ok) {
                const size_t slot = (size_t)slot0 + wave * WC + lane;
                a.slot_cnt[slot] = n;
                if (!GS) {
                    const Cand* cb = mysel + lane * a.cap;
                    Cand* out = a.slot_ent + slot * a.slot_stride;
                    for (int i = 0; i < n; i++) out[i] = cb[i];
                }
            }
            // ---- what this item found tightens the lower bounds of its queries for the items
            // still to come.  Every query has a histogram of the keys reported so far over
            // fixed key ranges above its seed; each reported key is a distinct row (an item
            // owns its rows), so "k keys in the bins from b up" proves that the k-th best of
            // the query is at least the lower edge of bin b.  Counts only grow, so a reader
            // that misses concurrent additions merely gets a weaker bound.
            if (a.hist != nullptr) {
                int qcol = 0;
#pragma unroll
                for (int s = 0; s < NCS; s++) {
                    const int v = __shfl(q[s], (lane - s * NC) & 63);
                    if (lane >= s * NC && lane < (s + 1) * NC) qcol = v;
                }
                const bool have = lane < WC && ok && n > 0;
                float base = 0.f, wd = 0.f;
                uint32_t now = 0;
                if (have) {
                    base = a.hpar[2 * (size_t)qcol];
                    wd = a.hpar[2 * (size_t)qcol + 1];
                    // keys under the bound other items have reached meanwhile cannot raise it
                    now = __hip_atomic_load(&a.thr[qcol], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                int added = 0;
                if (GS) {
                    // the entries of all columns of this wave side by side over the lanes (entry e of the
                    // wave = entry e - start[c] of column c): one load and one addition per entry, all
                    // of a pass in flight together
                    const int cnt = (have && wd > 0.f) ? n : 0;
                    const int incl = wave_prefix_sum(cnt);
                    const int total = __builtin_amdgcn_readlane(incl, 63);
                    unsigned long long gained = 0;                   // columns whose histogram got an addition
                    for (int e0 = 0; e0 < total; e0 += 64) {
                        const int e = e0 + lane;
                        const bool live = e < total;
                        int c = 0;                                   // column of entry e: columns that end at or before e
#pragma unroll
                        for (int cl = 0; cl < WC; cl++) c += (__builtin_amdgcn_readlane(incl, cl) <= e) ? 1 : 0;
                        c = live ? c : 0;
                        const int start = __shfl(incl - cnt, c);
                        const float cbase = __shfl(base, c), cwd = __shfl(wd, c);
                        const uint32_t cnow = (uint32_t)__shfl((int)now, c);
                        const int qc = __shfl(qcol, c);
                        bool did = false;
                        if (live) {
                            const uint32_t ek = gsel[c * a.cap + (e - start)].key;
                            if (ek >= cnow) {
                                const float key = dec_key(ek);
                                int b = (int)fminf(fmaxf((key - cbase) * (1.0f / cwd), 0.f), (float)(kHistBins - 1));
                                if (hist_edge(cbase, cwd, b) > key) b--;
                                else if (b < kHistBins - 1 && hist_edge(cbase, cwd, b + 1) <= key) b++;
                                // (the returned value is used so that the additions have been performed
                                // before the counts are read back below)
                                if (b >= 0) did = atomicAdd(&a.hist[(size_t)qc * kHistBins + b], 1) >= 0;
                            }
                        }
#pragma unroll
                        for (int cl = 0; cl < WC; cl++)
                            if (__builtin_amdgcn_ballot_w64(did && c == cl) != 0) gained |= 1ull << cl;
                    }
                    if (lane < WC && ((gained >> lane) & 1)) added = 1;
                } else if (have && wd > 0.f) {
                    const Cand* cb = mysel + lane * a.cap;
                    const float inv = 1.0f / wd;
                    for (int i = 0; i < n; i++) {
                        if (cb[i].key < now) continue;
                        const float key = dec_key(cb[i].key);
                        int b = (int)fminf(fmaxf((key - base) * inv, 0.f), (float)(kHistBins - 1));
                        if (hist_edge(base, wd, b) > key) b--;
                        else if (b < kHistBins - 1 && hist_edge(base, wd, b + 1) <= key) b++;
                        // (the returned value is used so that the additions have been performed
                        // before the counts are read back below)
                        if (b >= 0) added += atomicAdd(&a.hist[(size_t)qcol * kHistBins + b], 1) >= 0 ? 1 : 0;
                    }
                }
                const unsigned long long todo = __builtin_amdgcn_ballot_w64(added > 0);
                // lane i looks at bin 63 - i: the prefix sum over lanes then counts the keys
                // from the top bin down (all columns' loads go out before the first is used)
                int h[WC];
#pragma unroll
                for (int cl = 0; cl < WC; cl++) {
                    const int qc = __builtin_amdgcn_readlane(qcol, cl);
                    h[cl] = 0;
                    if ((todo >> cl) & 1)
                        h[cl] = __hip_atomic_load(&a.hist[(size_t)qc * kHistBins + (kHistBins - 1 - lane)], __ATOMIC_RELAXED,
                                                  __HIP_MEMORY_SCOPE_AGENT);
                }
#pragma unroll
                for (int cl = 0; cl < WC; cl++) {
                    if (!((todo >> cl) & 1)) continue;
                    const unsigned long long reach = __builtin_amdgcn_ballot_w64(wave_prefix_sum(h[cl]) >= a.k);
                    if (reach) {
                        const int b = kHistBins - 1 - __builtin_ctzll(reach);
                        const int qc = __builtin_amdgcn_readlane(qcol, cl);
                        const float cb0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, base), cl));
                        const float cw0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wd), cl));
                        if (b > 0 && lane == 0) atomicMax(&a.thr[qc], enc_key(hist_edge(cb0, cw0, b)));
                    }
                }
            }
        }
        __syncthreads();
    }
}

template <int DT, int NCS, int NW, bool GS>
inline hipError_t launch_scan_shape(int d, const ScanArgs& a, int grid, size_t lds, hipStream_t s)
{
#define HR_SCAN_CASE(KS)                                                                           \
    case KS * 32: {                                                                                \
        auto kern = k_scan<DT, KS, NCS, NW, GS>;                                                      \
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); \
        if (e != hipSuccess) return e;                                                             \
        hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 64), lds, s, a);                            \
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
inline hipError_t launch_scan_dtype(int d, const ScanArgs& a, int shape, int grid, size_t lds, hipStream_t s)
{
    if constexpr (DT == HR_F16X2) {
        // (the centroid table in the coarse step, and float32 lists split at load)
        return a.gsel ? launch_scan_shape<DT, 1, 8, true>(d, a, grid, lds, s) : launch_scan_shape<DT, 1, 8, false>(d, a, grid, lds, s);
    } else {
        if (a.gsel) return shape == SCAN_WIDE ? launch_scan_shape<DT, 1, 8, true>(d, a, grid, lds, s) : hipErrorInvalidValue;
        if constexpr (DT == HR_F32) {
            return shape == SCAN_WIDE ? launch_scan_shape<DT, 1, 8, false>(d, a, grid, lds, s)
                                      : launch_scan_shape<DT, 1, 4, false>(d, a, grid, lds, s);
        } else {
            return hipErrorInvalidValue;       // (16-bit lists always keep their selection buffers in global memory)
        }
    }
}

// ------------------------------------------------------------------------------------------
// Threshold seeding.  One workgroup per query scores the first rows of the query's best-ranked
// list (with the very MFMA sequence of k_scan, so the keys are the ones the scan will compute
// for these rows) and publishes the k-th best of them as the query's starting lower bound.
// On clustered data that bound already excludes nearly every row of the other probed lists,
// which then cost the scan one compare per score instead of a candidate insertion.  Any k
// real candidates give a valid bound, so the result of the search does not depend on this.
// The kernel is a chain of round trips to memory (probe row, list offsets, rows), so what
// matters is how few there are one after the other: each wave takes every fourth 16-row
// block and asks for the whole block at once (the query operand waits in LDS meanwhile,
// not in registers), wave 0 then picks the k-th key.
constexpr int kSeedRowsMax = 192;

template <int DT, int KSTEPS>
__global__ __launch_bounds__(256) void k_seed(SeedArgs a)
{
    using T = StoreTraits<DT>;
    constexpr int NC = T::nc;
    constexpr int d = KSTEPS * 32;
    constexpr int rowb = d * T::esize;
    constexpr int QP = (NC == 8) ? 2 : 1;               // operand rows per query (bfloat16: hi and lo)
    __shared__ uint32_t s_keys[kSeedRowsMax];
    __shared__ u32x4 s_q[QP * KSTEPS * 4];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    const int64_t q = blockIdx.x;
    // the best-ranked list of the query whose vectors are in place (among the first 64 places of its row);
    // every wave finds it for itself (same loads, same answer: what follows is uniform over the workgroup)
    int l = -1;
    {
        const int c = lane < a.nprobe ? a.probe[q * a.nprobe + lane] : -1;
        const unsigned long long ok = __builtin_amdgcn_ballot_w64(c >= 0 && c < a.nlist && a.resident[c] != 0);
        if (ok == 0) return;
        l = __builtin_amdgcn_readlane(c, __builtin_ctzll(ok));
    }
    const int row0 = a.list_off[l];
    const int nrows = min(a.list_off[l + 1] - row0, a.seed_rows);
    if (nrows < a.k) return;
    for (int i = threadIdx.x; i < QP * KSTEPS * 4; i += 256)
        s_q[i] = ((const u32x4*)((const char*)a.qop + (size_t)q * QP * (size_t)(d * 2)))[i];
    const int g = lane >> 4;
    const int part = (NC == 8) ? ((lane >> 3) & 1) : 0;
    const bool bcol = (lane & (NC - 1)) == 0;          // MFMA column 0 (and its lo twin)
    const u32x4* qfrag = s_q + part * (KSTEPS * 4) + g;
    __syncthreads();
    const int nblk = (nrows + 15) / 16;
    for (int blk = wave; blk < nblk; blk += 4) {
        const int r = row0 + blk * 16 + (lane & 15);
        const bool rv = r < row0 + nrows;
        const char* rp = (const char*)a.rows + (size_t)(rv ? r : row0) * rowb;
        floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
        if constexpr (DT == HR_F32) {
            constexpr int H = KSTEPS / 2;               // half a row at a time: 8 registers per k-step
#pragma unroll
            for (int h = 0; h < 2; h++) {
                u32x4 v0[H], v1[H];
#pragma unroll
                for (int t = 0; t < H; t++) {
                    v0[t] = *(const u32x4*)(rp + (h * H + t) * 128 + g * 32);
                    v1[t] = *(const u32x4*)(rp + (h * H + t) * 128 + g * 32 + 16);
                }
#pragma unroll
                for (int t = 0; t < H; t++) {
                    const floatx4 f0 = __builtin_bit_cast(floatx4, v0[t]), f1 = __builtin_bit_cast(floatx4, v1[t]);
                    float x[8];
#pragma unroll
                    for (int i = 0; i < 4; i++) { x[i] = rv ? f0[i] : 0.f; x[4 + i] = rv ? f1[i] : 0.f; }
                    half8 hi, lo;
#pragma unroll
                    for (int i = 0; i < 8; i++) {
                        _Float16 hh = (_Float16)x[i];
                        hi[i] = hh;
                        lo[i] = (_Float16)((x[i] - (float)hh) * 2048.0f);
                    }
                    const half8 b = __builtin_bit_cast(half8, bcol ? qfrag[(h * H + t) * 4] : u32x4{0, 0, 0, 0});
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(hi, b, acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(lo, b, acc1, 0, 0, 0);
                }
            }
        } else {
            u32x4 v[KSTEPS];
#pragma unroll
            for (int t = 0; t < KSTEPS; t++) v[t] = *(const u32x4*)(rp + t * 64 + g * 16);
#pragma unroll
            for (int t = 0; t < KSTEPS; t++) {
                const u32x4 x = rv ? v[t] : u32x4{0, 0, 0, 0};
                const u32x4 bq = bcol ? qfrag[t * 4] : u32x4{0, 0, 0, 0};
                if constexpr (DT == HR_F16) {
                    const half8 b = __builtin_bit_cast(half8, bq);
                    if (t & 1) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, x), b, acc1, 0, 0, 0);
                    else       acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8, x), b, acc0, 0, 0, 0);
                } else {
                    const bf16x8 b = __builtin_bit_cast(bf16x8, bq);
                    if (t & 1) acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x), b, acc1, 0, 0, 0);
                    else       acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, x), b, acc0, 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int r4 = 0; r4 < 4; r4++) {
            float dot;
            if constexpr (DT == HR_F32) {
                float t0 = lane_xor8(acc0[r4]);
                float t1 = lane_xor8(acc1[r4]);
                dot = acc0[r4] + (t0 + acc1[r4]) * (1.0f / 2048.0f) + t1 * (1.0f / 4194304.0f);
            } else if constexpr (DT == HR_BF16) {
                float v2 = acc0[r4] + acc1[r4];
                dot = v2 + lane_xor8(v2);
            } else {
                dot = acc0[r4] + acc1[r4];
            }
            const int row = row0 + blk * 16 + g * 4 + r4;
            if ((lane & 15) == 0 && row < row0 + nrows) {
                float key = a.l2 ? (2.0f * dot - a.row_norm[row]) : dot;
                s_keys[blk * 16 + g * 4 + r4] = enc_key(key);
            }
        }
    }
    __syncthreads();
    if (wave != 0) return;
    const uint32_t* keys = s_keys;
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
    const uint32_t pub = kth > 8u ? kth - 8u : 0u;
    if (lane == 0) atomicMax(&a.thr[q], pub);
    // key ranges of the query's histogram in the scan: from the seed upwards, an eighth of
    // the distance between the seed and the best key of the sample per bin
    if (a.hpar != nullptr) {
        uint32_t mx = 0;
#pragma unroll
        for (int m = 0; m < 3; m++) mx = max(mx, e[m]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) mx = max(mx, (uint32_t)__shfl_xor((int)mx, o));
        if (lane == 0) {
            const float base = dec_key(pub);
            const float wd = (dec_key(mx) - base) * 0.125f;
            const bool fine = wd > 0.f && wd < 3.0e38f && base > -3.0e38f;
            a.hpar[2 * q] = fine ? base : 0.f;
            a.hpar[2 * q + 1] = fine ? wd : 0.f;
        }
    }
}

template <int DT>
inline hipError_t launch_seed_dtype(int d, const SeedArgs& a, hipStream_t s)
{
    if (a.nq <= 0) return hipSuccess;
    const dim3 grid((unsigned)a.nq);
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
