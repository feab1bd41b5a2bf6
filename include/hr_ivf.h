/*
 * hr_ivf.h — C ABI of the MI355X (gfx950) batched IVF-Flat top-k search.
 *
 * The operation is the retrieval stage of the paper (Section 2.2): similarity
 * (inner product on caller-normalised vectors, or squared L2 distance) between
 * each query and the stored vectors, restricted to the nprobe clusters whose
 * centroids are closest to the query, top-k nearest returned.  A call handles a
 * whole batch of queries; queries that probe the same inverted list share one
 * pass over it (the cross-request, variable-length cluster search of Section 5,
 * with the per-request merge of Section 4.4).
 *
 * Pointers marked DEV are device (HBM) addresses on the current HIP device;
 * HOST are ordinary host addresses.  No call takes ownership of caller memory.
 * Every function returns HR_OK (0) or a negative error code; nothing is thrown
 * and nothing aborts.  On any error other than HR_ERR_HIP nothing was enqueued
 * and outputs are untouched.  hr_last_error() gives a message for the last
 * failing call on the calling thread.
 *
 * Result convention: row q of the outputs is sorted best-first (inner product
 * descending, L2 ascending; equal scores by ascending id).  If fewer than k
 * candidates exist, ids are padded with -1 and scores with -inf (IP) / +inf (L2).
 * Same inputs give bit-identical outputs on every run.
 */
#ifndef HR_IVF_H
#define HR_IVF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hr_ivf_index hr_ivf_index; /* opaque */

enum { HR_METRIC_IP = 0, HR_METRIC_L2 = 1 };      /* L2 = squared distance, smaller is better */
enum { HR_F32 = 0, HR_F16 = 1, HR_BF16 = 2 };     /* storage type of list_vectors only */
enum {
    HR_OK = 0,
    HR_ERR_ARG = -1,          /* null pointer, size or enum out of range, offsets not monotone */
    HR_ERR_HANDLE = -2,       /* index handle null, freed or corrupt */
    HR_ERR_WORKSPACE = -3,    /* workspace null, misaligned or smaller than hr_ivf_workspace_bytes */
    HR_ERR_HIP = -4,          /* a HIP runtime call failed (message in hr_last_error) */
    HR_ERR_UNSUPPORTED = -5   /* valid request outside what the kernels are built for */
};

#define HR_K_MAX 128          /* largest k */
#define HR_NPROBE_MAX 512     /* largest nprobe (the paper probes 128 to 512 clusters: Section 6.1) */
#define HR_WORKSPACE_ALIGN 256
#define HR_LOAD_ROW_TABLES 0x100      /* or-ed into hr_ivf_load's dtype: see there */
#define HR_STATIC_SCRATCH_BYTES (64u << 20)   /* scratch of hr_ivf_search_static: 64 MiB per GPU */

/*
 * hr_ivf_load — wrap an IVF-Flat index that already lives in HBM (Section 2.2: vectors
 * partitioned into clusters, each represented by a centroid).
 *   centroids     DEV  [nlist, d] float32, row-major.
 *   list_offsets  HOST [nlist+1] int64; list l holds rows list_offsets[l] .. list_offsets[l+1]-1;
 *                 list_offsets[0] = 0, list_offsets[nlist] = N, non-decreasing (empty lists allowed).
 *                 Copied during the call.
 *   list_vectors  DEV  [N, d] row-major in `dtype` (HR_F32 / HR_F16 / HR_BF16), list-major.
 *   list_ids      DEV  [N] int64 >= 0, the label reported for each row (ties between equal scores
 *                 are broken by ascending label; a negative id marks an empty place in results and
 *                 carried results, so a negative label is refused: HR_ERR_ARG).
 *   d             supported: 64, 128, 256, 512, 768, 1024 (else HR_ERR_UNSUPPORTED).
 *   N < 2^31.  Values must be finite and, for HR_F32 storage and for centroids/queries, of
 *   magnitude below 65504 (they pass through binary16 pairs inside the kernels).
 *   stream        hipStream_t (as void*) on which the derived tables are computed.
 * centroids, list_vectors and list_ids are BORROWED: they must stay valid and unchanged until
 * hr_ivf_free.  The library allocates (hipMalloc) derived tables: device copies of the offsets,
 * 4 bytes per row / per centroid of squared norms, the centroids as two binary16 tables, 8 bytes
 * per list of access counters.  Nothing the size of list_vectors, unless the caller asks for it:
 * with dtype = HR_F32 | HR_LOAD_ROW_TABLES the rows are also kept as two binary16 tables (hi and
 * scaled lo part: N*d*4 bytes, as much as list_vectors itself) which the scan then reads instead of
 * splitting every row block on the fly: same products in the same order, the same bits, faster.
 * With HR_BF16 | HR_LOAD_ROW_TABLES the rows are also kept as one binary16 table (N*d*2 bytes; every
 * bfloat16 value of magnitude 2^-14 .. 65504 is a binary16 value, smaller ones are rounded to a
 * multiple of 2^-24): the lists are then multiplied with the query rounded to binary16 (as HR_F16
 * lists are) and twice as many queries share one pass over a list; without the table the query goes
 * in as bfloat16 hi + lo parts; the two ways agree within the tolerance of 16-bit storage, not bit
 * for bit.  The tables are made only when they take at most half of the device memory free at the
 * time and, for bfloat16, no value exceeds 65504; otherwise the flag has no effect.  HR_F16 ignores
 * it.  The call synchronises `stream` before returning.
 */
int hr_ivf_load(const float* centroids, const int64_t* list_offsets, const void* list_vectors,
                const int64_t* list_ids, int64_t nlist, int64_t N, int32_t d, int32_t dtype,
                void* stream, hr_ivf_index** out);

/* Releases the derived tables.  The handle is invalid afterwards (HR_ERR_HANDLE if reused). */
int hr_ivf_free(hr_ivf_index* index);

/*
 * Bytes of DEV scratch that hr_ivf_search / hr_ivf_coarse / hr_ivf_scan and the step-wise calls
 * need for this batch shape; 0 on invalid arguments (nprobe 1 .. HR_NPROBE_MAX: hr_ivf_scan takes
 * rows of that many places whatever the number of lists).  Depends only on (index, nq, nprobe, k),
 * never on the data.
 */
size_t hr_ivf_workspace_bytes(const hr_ivf_index* index, int64_t nq, int32_t nprobe, int32_t k);

/*
 * hr_ivf_search — the whole hot path for one batch: coarse scoring of queries against the
 * centroids, top-nprobe selection, grouping of (query, list) probes by list, cluster-major
 * scan with per-query top-k merge (Sections 2.2, 5 and 4.4 of the paper).
 *   queries     DEV  [nq, d] float32 row-major.   nq >= 0 (0 is a no-op).
 *   nprobe      1 .. min(nlist, HR_NPROBE_MAX);   k  1 .. HR_K_MAX.
 *   metric      HR_METRIC_IP or HR_METRIC_L2; the coarse step uses the same metric.
 *   out_ids     DEV  [nq, k] int64;   out_scores  DEV [nq, k] float32.
 *   workspace   DEV, HR_WORKSPACE_ALIGN-aligned, >= hr_ivf_workspace_bytes(...) bytes; contents
 *               are scratch.  Two calls that overlap in time must not share a workspace.
 *   stream      hipStream_t (as void*).  The call only enqueues kernels on it: no allocation,
 *               no host synchronisation; outputs are valid once the stream reaches that point.
 *               (Kernels only, no memset or copy nodes: the call can be captured in a HIP
 *               graph and replayed with new contents in the same buffers.)
 */
int hr_ivf_search(const hr_ivf_index* index, const float* queries, int64_t nq, int32_t nprobe,
                  int32_t k, int32_t metric, int64_t* out_ids, float* out_scores,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * hr_ivf_search_static — hr_ivf_search for callers that cannot allocate device memory or have no
 * workspace to pass: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments without the workspace; the scratch memory is an array of
 * HR_STATIC_SCRATCH_BYTES (64 MiB) inside the library's device image, which every GPU the
 * library runs on holds until the process ends.  The call allocates nothing and frees nothing,
 * it only enqueues kernels on `stream`; the index's device must be the current one.
 * To fit the array, the list scan is cut into about 256 work items instead of about 4096 and the
 * coarse keys of at most 4 MiB of queries x lists are scored at a time; results are the same bits
 * as hr_ivf_search's.  A batch shape that needs more scratch is refused with HR_ERR_WORKSPACE and
 * a message that gives the bytes needed (what fits: e.g. 512 queries x nprobe 32, k 10 on 4096
 * lists of 768 dimensions takes about 31 MiB; the bulk are the 128 x 256 + nq x nprobe result
 * slots of 512 bytes each for k <= 24, 1024 up to k = 64, 1536 beyond).
 * All calls on one GPU share that GPU's array: two calls that overlap in time (different
 * streams, or threads) race; put them on one stream or give one of them hr_ivf_search with a
 * workspace of its own.  The array keeps what the last call left; every call clears what it
 * needs cleared.
 */
int hr_ivf_search_static(const hr_ivf_index* index, const float* queries, int64_t nq, int32_t nprobe,
                         int32_t k, int32_t metric, int64_t* out_ids, float* out_scores, void* stream);

/*
 * hr_ivf_coarse — first half only: the choice of the clusters a query is searched in (Section 2.2).
 *   out_probe_ids     DEV [nq, nprobe] int32, best-first (ties: lower list number first).
 *   out_probe_scores  DEV [nq, nprobe] float32 or NULL.
 */
int hr_ivf_coarse(const hr_ivf_index* index, const float* queries, int64_t nq, int32_t nprobe,
                  int32_t metric, int32_t* out_probe_ids, float* out_probe_scores,
                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * hr_ivf_scan — second half only, with the probe lists given by the caller: the step-wise,
 * variable-length cluster search of Section 5 (a scheduler hands each query the clusters it
 * wants searched in this step).
 *   probe_ids  DEV [nq, nprobe] int32.  An entry < 0 or >= nlist means "no list here", which
 *              gives queries probe lists of different lengths.  A list must not appear twice
 *              in one query's row (its vectors would be reported twice).
 */
int hr_ivf_scan(const hr_ivf_index* index, const float* queries, int64_t nq,
                const int32_t* probe_ids, int32_t nprobe, int32_t k, int32_t metric,
                int64_t* out_ids, float* out_scores, void* workspace, size_t workspace_bytes,
                void* stream);

/*
 * hr_ivf_scan_step — hr_ivf_scan with a carried result: one sub-stage of a retrieval that a
 * scheduler splits into several (Section 4.2: clusters are added to a request's sub-stage until
 * the time budget is reached; Section 5: the variable-length cluster search interface).
 *   io_ids     DEV [nq, k] int64   } on entry the result of the earlier steps of these queries, best
 *   io_scores  DEV [nq, k] float32 } first, empty places last with id -1 (all -1: nothing yet; the
 *                                    scores of empty places are ignored); on return the k best of
 *                                    that result and of the lists probed in this step, in the same
 *                                    form.  Updated in place.
 *   A full carried result also gives the scan its starting lower bound: rows that cannot enter
 *   the result cost one compare.  Entries are ordered by (score, id) like everywhere else; a
 *   carried entry keeps the score it was reported with.  A list must not be probed in two steps
 *   of the same query (its vectors would be reported twice).  Other arguments as hr_ivf_scan.
 */
int hr_ivf_scan_step(const hr_ivf_index* index, const float* queries, int64_t nq,
                     const int32_t* probe_ids, int32_t nprobe, int32_t k, int32_t metric,
                     int64_t* io_ids, float* io_scores, void* workspace, size_t workspace_bytes,
                     void* stream);

/*
 * hr_ivf_hot_lists — the gc most frequently probed lists by the counters of hr_ivf_list_hits,
 * most frequent first, equal counts by ascending list number: the clusters a partial index
 * cache keeps resident (Section 4.4).   out_lists DEV [gc] int32, 1 <= gc <= nlist.
 * Ranks by counting (nlist^2 compares): nlist <= 65536, else HR_ERR_UNSUPPORTED.  Meant to be
 * called now and then (the paper updates its cache every 50 sub-stages), not per search.
 */
int hr_ivf_hot_lists(const hr_ivf_index* index, int32_t gc, int32_t* out_lists, void* stream);

/*
 * Partial residency (Section 4.4: only the most frequently accessed clusters are kept in GPU memory and updated
 * from time to time; searches of the other clusters are served elsewhere, and the partial results of a request
 * are merged).  The index keeps a flag per list: are its vectors in place?  All lists are, after hr_ivf_load.
 *
 * hr_ivf_set_resident — set the flag of the given lists.
 *   lists     DEV [n] int32 list numbers (entries outside 0..nlist-1 are ignored), or NULL: all lists.
 *   resident  0: the lists' rows may be overwritten by the caller from now on; no search reads them: their
 *             probes are dropped by hr_ivf_search / hr_ivf_scan / the step-wise calls (and still counted by
 *             hr_ivf_list_hits).  1: the rows are in place again (after the caller's copy and
 *             hr_ivf_refresh_rows on the same stream, or behind them).
 * Enqueues one small kernel; searches enqueued later on the same stream see the new flags.
 *
 * hr_ivf_split_probes — which of a batch's probes can be served here.
 *   probe_ids     DEV [nq, nprobe] int32 (as hr_ivf_coarse writes them, or any rows hr_ivf_scan would take)
 *   out_resident  DEV [nq, nprobe] int32: the lists of each row whose vectors are in place, in the given order,
 *                 then -1: what to hand to hr_ivf_scan / hr_ivf_scan_step
 *   out_missing   DEV [nq, nprobe] int32: the other lists of the row, in the given order, then -1: what the
 *                 caller has to search elsewhere (their partial results can be merged in by the caller, or
 *                 the lists scanned here in a later step once they are resident).  These probes are counted
 *                 as accesses here, since no scan will see them.
 * The three arrays must be distinct.  Entries outside 0..nlist-1 appear in neither output.
 */
int hr_ivf_set_resident(hr_ivf_index* index, const int32_t* lists, int64_t n, int32_t resident, void* stream);
int hr_ivf_split_probes(const hr_ivf_index* index, const int32_t* probe_ids, int64_t nq, int32_t nprobe,
                        int32_t* out_resident, int32_t* out_missing, void* stream);

/*
 * hr_ivf_refresh_rows — after the caller has replaced the vectors of rows row_begin ..
 * row_end-1 in list_vectors (a cluster loaded asynchronously into the place of another one of
 * the same length: the index loading interface of Section 5), recompute what the library
 * derives from them (squared norms; the binary16 row tables of HR_LOAD_ROW_TABLES).  Enqueued on
 * `stream`: put it behind the copy, and the next search behind it.  list_ids is read at search time
 * and needs no refresh; list_offsets cannot change.  Only with a binary16 table of bfloat16 rows the
 * call also waits for the stream, to learn whether a new value exceeds 65504: HR_ERR_UNSUPPORTED
 * then (the table holds an infinity there until the rows are replaced again).
 */
int hr_ivf_refresh_rows(hr_ivf_index* index, int64_t row_begin, int64_t row_end, void* stream);

/*
 * Reuse of a request's previous retrieval (Section 4.3: consecutive queries v, v' of a request are
 * close; the results of v' tend to lie among a larger top-k of v, in the clusters H_v that held
 * v's results, and in clusters probed for both).  Four calls; each only enqueues kernels.
 *
 * hr_ivf_scan_step_rows — hr_ivf_scan_step whose carried result also holds the row number of
 * every entry:
 *   io_rows  DEV [nq, k] int32: position of the entry's vector in list_vectors, -1 for an empty
 *            place; updated in place with the ids and scores.
 * Rows tell where a result lies (hr_ivf_lists_of_rows) and let it be scored again for another
 * query (hr_ivf_rescore).  A vector of a probed list whose row the carried result already
 * holds is not taken again, so a carried result may come from hr_ivf_rescore and its rows'
 * lists may be probed afterwards.  (A list probed in two steps is still the caller's error.)
 */
int hr_ivf_scan_step_rows(const hr_ivf_index* index, const float* queries, int64_t nq,
                          const int32_t* probe_ids, int32_t nprobe, int32_t k, int32_t metric,
                          int64_t* io_ids, float* io_scores, int32_t* io_rows, void* workspace,
                          size_t workspace_bytes, void* stream);

/*
 * hr_ivf_rescore — the local cache: the m rows a request kept from its previous retrieval (the
 * paper keeps the 20 best) are scored for its new query and the k best of them become the
 * starting result of the new retrieval.
 *   rows        DEV [nq, m] int32 row numbers, 1 <= m <= HR_K_MAX; < 0 or >= N: no row; a row
 *               listed twice counts once.
 *   out_ids, out_scores, out_rows   DEV [nq, k]: the k best by (score, id), best first, empty
 *               places last (-1, +-inf, -1): the form hr_ivf_scan_step_rows carries.
 * Scores as in the search (query rounded as the list scan rounds it, float32 sums).
 */
int hr_ivf_rescore(const hr_ivf_index* index, const float* queries, int64_t nq, const int32_t* rows,
                   int32_t m, int32_t k, int32_t metric, int64_t* out_ids, float* out_scores,
                   int32_t* out_rows, void* stream);

/*
 * hr_ivf_lists_of_rows — the list every row belongs to (for H_v: the clusters that held the
 * results of v).   rows DEV [n] int32;  out_lists DEV [n] int32, -1 for rows < 0 or >= N.
 */
int hr_ivf_lists_of_rows(const hr_ivf_index* index, const int32_t* rows, int64_t n, int32_t* out_lists,
                         void* stream);

/*
 * hr_ivf_reorder_probes — search order of the new probe lists C' of every query: first the
 * lists that are in hot (H_v), then those in prev (C, the lists probed for v) that are not in
 * hot, then the others; inside each group the given order is kept; entries < 0 go last.
 *   probe      DEV [nq, nprobe] int32, 1 <= nprobe <= HR_NPROBE_MAX
 *   prev       DEV [nq, nprev] int32 or NULL, nprev <= HR_NPROBE_MAX   (entries < 0 ignored)
 *   hot        DEV [nq, nhot] int32 or NULL, nhot <= HR_K_MAX          (entries < 0 ignored)
 *   out_probe  DEV [nq, nprobe] int32, must not overlap probe
 * Needs no index: list numbers are only compared.
 */
int hr_ivf_reorder_probes(const int32_t* probe, int64_t nq, int32_t nprobe, const int32_t* prev,
                          int32_t nprev, const int32_t* hot, int32_t nhot, int32_t* out_probe,
                          void* stream);

/*
 * hr_ivf_list_hits — how often every list has been probed by hr_ivf_search / hr_ivf_scan /
 * hr_ivf_scan_step calls on this index since it was loaded or since the last reset: the
 * per-cluster access frequency that a cache of hot clusters is driven by (Section 4.4: the
 * clusters accessed most often are the ones kept resident).  A by-product of the grouping of
 * probes by list; counted on the device, in the order of the stream.
 *   out_hits  DEV [nlist] int64.   reset != 0: the counters start again from zero.
 * Enqueues one small kernel on the stream; calls that run concurrently on other streams are
 * counted, but a reset concurrent with them may miss or keep some of their probes.
 */
int hr_ivf_list_hits(const hr_ivf_index* index, int64_t* out_hits, int32_t reset, void* stream);

/*
 * hr_ivf_stats — host-side facts about the last hr_ivf_search / hr_ivf_scan enqueued with this
 * workspace, read back AFTER the caller has synchronised the stream (this call does a small
 * blocking device-to-host copy).  out[0] = work items of the list scan, out[1] = rows per
 * segment chosen for this batch, out[2] = sum over probed lists of their row counts (rows
 * streamed once each), out[3] = number of (query, list) pairs.  For benchmarks and tests.
 */
int hr_ivf_stats(const hr_ivf_index* index, const void* workspace, size_t workspace_bytes,
                 int64_t nq, int32_t nprobe, int32_t k, int64_t out[4]);

/*
 * hr_ivf_workspace_layout — how the library divides a workspace of hr_ivf_workspace_bytes(index, nq, nprobe, k)
 * bytes: for every region it uses, its offset and its length in bytes (out[2i], out[2i+1], HOST, in order of
 * offset; *n = number of regions, of which at most cap are written).  Behind every region lie at least
 * HR_WORKSPACE_ALIGN bytes that no kernel writes: a test can fill the workspace with a pattern, run a search and
 * verify that the pattern survives everywhere outside the regions (an overrun of a region that is sized on the
 * host and indexed on the device would show there).  For tests; the layout may change between versions.
 */
int hr_ivf_workspace_layout(const hr_ivf_index* index, int64_t nq, int32_t nprobe, int32_t k, int64_t* out,
                            int32_t cap, int32_t* n);

/*
 * Kernel timing for benchmarks.  hr_ivf_profile_begin creates max_calls pairs of HIP events
 * (no device memory); from then on every hr_ivf_search / hr_ivf_scan records one pair on its
 * stream immediately before and after the list-scan kernel (the dominant kernel), until
 * max_calls pairs are used.  hr_ivf_profile_end waits for the recorded events, returns the
 * number of timed launches in *n and their average duration in milliseconds in *scan_ms_avg
 * (0 if none), destroys the events and switches timing off.  Not thread-safe with concurrent
 * searches on the same index.
 */
int hr_ivf_profile_begin(hr_ivf_index* index, int32_t max_calls);
int hr_ivf_profile_end(hr_ivf_index* index, int32_t* n, double* scan_ms_avg);

/* Message for the last error on this thread (static storage, never NULL). */
const char* hr_last_error(void);

/* Library version string, e.g. "hr_ivf 0.1 gfx950". */
const char* hr_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HR_IVF_H */
