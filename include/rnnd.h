/*
 * rnnd.h -- C ABI of librnnd: graph construction by Relative NN-Descent
 * (arXiv 2310.20419) on one AMD MI355X (gfx950).
 *
 * Everything behind these calls runs in hand-written HIP kernels.  There is no
 * CPU fallback: without a usable GPU every compute call returns RNND_ERR_HIP.
 *
 * Conventions
 *   - "device" pointers are HIP device memory owned by the caller; the library
 *     never keeps a caller's pointer after a call returns.  Its own workspace is one
 *     block per device that it keeps between calls (see rnnd_workspace_bytes).
 *   - X is row-major N x d, contiguous: uint8, float32, or (RNND_F16, RNND_BF16) IEEE binary16 or
 *     bfloat16 as a storage format for float data -- every coordinate stands for the float32 value it
 *     converts to exactly, all arithmetic is that of float data, and the graph is the one
 *     rnnd_build gives for that float32 matrix; it halves the bytes the rounds gather.
 *   - vertex ids are 0-based (the paper's V = {1..n}, Sec. 2.2, shifted by one).
 *   - delta(u,v) is the squared Euclidean distance of x_u and x_v (Eq. 3 with
 *     dist = squared L2; every comparison of Alg. 3-5 is monotone in it).
 *     uint8 data: exact int32.  float data: accumulated in double, rounded once
 *     to float, bit-identical for delta(u,v) and delta(v,u).
 *   - every call enqueues its work on `stream` (a hipStream_t, may be NULL for
 *     the default stream) and returns after that work has completed, so the
 *     status reflects kernel errors too.
 *   - return value: RNND_OK (0) or a negative rnnd_status; outputs are
 *     unspecified after an error.  No call aborts or throws.
 *
 * Graph state ("snapshot") used by the step-wise entry points
 *   keys : device uint64 [N * R], row u = neighbour list of u, deg[u] valid entries in
 *          ascending order, each  (dist_bits << 32) | (id << 1) | is_new
 *          where dist_bits is the int32 distance (uint8 data) or the IEEE bit pattern of
 *          the float distance (float data; non-negative, so the unsigned order is the
 *          numeric order) and is_new is the paper's "new"/"old" flag of Alg. 4.
 *          Ascending key order is ascending (delta, id).  Entries past deg[u] are unspecified.
 *   deg  : device int32 [N].
 */
#ifndef RNND_H
#define RNND_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define RNND_MAX_R 128          /* largest supported degree cap R */
#define RNND_MAX_ROUNDS 256     /* per-round statistics are kept for the first 256 rounds */
#define RNND_STATIC_SCRATCH_BYTES (64u << 20)   /* size of the static device array rnnd_build_static works in */

typedef enum { RNND_U8 = 0, RNND_F32 = 1, RNND_F16 = 2, RNND_BF16 = 3 } rnnd_dtype;
typedef enum { RNND_L2SQ = 0 } rnnd_metric;

typedef enum {
    RNND_OK = 0,
    RNND_ERR_NULL = -1,         /* a required pointer is NULL */
    RNND_ERR_BAD_SHAPE = -2,    /* N < 2, N > 2^31-2, N * (slots per row) > 2^31-256, d < 1, or uint8 d > 33025 (int32 overflow) */
    RNND_ERR_BAD_PARAM = -3,    /* S < 1, S > R, S > N-1, R < 1, R > RNND_MAX_R, T1 < 1, T2 < 1, T1*T2 (x runs per pass) > 131072 */
    RNND_ERR_UNSUPPORTED = -4,  /* unknown dtype or metric */
    RNND_ERR_OOM = -5,          /* workspace allocation failed (also: a workspace of more than 1 TiB, which no
                                   device holds, is refused before any device is touched) */
    RNND_ERR_HIP = -6,          /* a HIP call or kernel failed (no GPU, launch error, ...) */
    RNND_ERR_SCRATCH = -7       /* rnnd_build_static: the workspace for these sizes exceeds RNND_STATIC_SCRATCH_BYTES */
} rnnd_status;

/* Counters of one build, filled on the host.  "algo" evaluations are the delta(v,w)
 * evaluations the prune test of Alg. 4 performs (with its old/old skip and its break at the
 * first failure); "exec" are the distances the kernels actually computed. */
typedef struct {
    int32_t rounds;                         /* UpdateNeighbors rounds run (T1*T2) */
    int32_t reverse_calls;                  /* AddReverseEdges calls run (T1-1) */
    int32_t kernel_variant;                 /* UpdateNeighbors scan kernel used: 1 generic, 2 int8 MFMA, 3 float MFMA (fp32, then f64) */
    int32_t reserved;
    float total_ms, init_ms;                /* GPU time of the whole call / of RandomGraph (HIP events) */
    float round_ms[RNND_MAX_ROUNDS];        /* GPU time of each UpdateNeighbors round (see rnnd_set_event_timing) */
    float scan_ms[RNND_MAX_ROUNDS];         /* of which: the scan kernels (Alg. 4's loop body) */
    float reverse_ms[RNND_MAX_ROUNDS];      /* GPU time of each AddReverseEdges call */
    int64_t init_evals;                     /* N*S */
    int64_t active[RNND_MAX_ROUNDS];        /* vertices with at least one "new" entry */
    int64_t proposals[RNND_MAX_ROUNDS];     /* redirected edges emitted (Alg. 4's edge update) */
    int64_t algo_evals[RNND_MAX_ROUNDS];
    int64_t exec_evals[RNND_MAX_ROUNDS];
    int64_t gathered_rows[RNND_MAX_ROUNDS]; /* rows of X the round kernel fetched */
    int64_t dropped[RNND_MAX_ROUNDS];       /* list entries the round's merges dropped because a list was full (rows
                                               are R, or M, slots wide; the paper's UpdateNeighbors never drops one:
                                               where this is 0 in every round of rnnd_build_wide, its graph is the
                                               one unbounded lists give).  A hub that receives more than 128 edges in
                                               one round may count an edge twice. */
} rnnd_stats;

/* Alg. 6, RNN-Descent(S, R, T1, T2), with synchronous rounds:
 *   G <- RandomGraph(S), all flags new; T1 x { T2 x UpdateNeighbors; AddReverseEdges unless last }.
 * Each UpdateNeighbors round scans every vertex against the same snapshot (the body of Alg. 4's vertex loop)
 * and then rebuilds every list as the first R entries, in (delta, id) order and without
 * duplicates, of its kept entries plus the edges redirected to it (the edge update: v enters w's list).
 *   X          device, N x d
 *   graph_out  device int32 [N * R]: row u = neighbour ids of u, ascending (delta, id), -1 padded
 *   degree_out device int32 [N]
 *   seed       seeds RandomGraph's counter-based generator; same seed, same graph, bit for bit
 */
int rnnd_build(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S, int32_t R,
               int32_t T1, int32_t T2, uint64_t seed, int32_t *graph_out, int32_t *degree_out,
               void *stream);

/* Same build; additionally returns the final snapshot (keys_out: device uint64 [N*R], may be
 * NULL) and the counters (stats: host, may be NULL). */
int rnnd_build_ex(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S, int32_t R,
                  int32_t T1, int32_t T2, uint64_t seed, int32_t *graph_out, int32_t *degree_out,
                  uint64_t *keys_out, rnnd_stats *stats, void *stream);

/* Alg. 6 with synchronous rounds whose merges cut a list to M >= R entries instead of R: in the
 * paper UpdateNeighbors never drops an edge for lack of room and only AddReverseEdges bounds the
 * degrees by R (Sec. 5.3 reports out-degrees above R in the finished graphs), whereas rnnd_build
 * keeps rows of fixed width R throughout.  Here rows are M slots wide, 1 <= R <= M <= RNND_MAX_R:
 * between two AddReverseEdges calls, and in the result, a list may hold up to M entries.
 *   graph_out  device int32 [N * M], keys_out device uint64 [N * M] or NULL
 * M = R gives the graph of rnnd_build.  Other arguments, ownership and errors as for rnnd_build_ex. */
int rnnd_build_wide(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S, int32_t R,
                    int32_t M, int32_t T1, int32_t T2, uint64_t seed, int32_t *graph_out,
                    int32_t *degree_out, uint64_t *keys_out, rnnd_stats *stats, void *stream);

/* Alg. 6 with block-sequential passes: a variant between the synchronous round and the in-place
 * vertex loop of Alg. 4 (it visits the vertices one after the other and its edge update changes the
 * edge set at once, so a vertex visited later in the same pass already sees the edges redirected
 * to it).  The vertices are cut into runs of ceil(N / blocks) consecutive ids; the runs take their
 * turn in id order; every vertex of a run is scanned against the graph as it stands when the run
 * starts, and the run's redirected edges are merged into their targets' lists (any vertex; first R
 * entries as in rnnd_build) before the next run starts.  blocks = 1 gives the graph of rnnd_build;
 * blocks = N visits the vertices in Alg. 4's own order.  Every value of blocks defines one graph
 * per seed, bit for bit.
 *   blocks     1 <= blocks <= N, and T1 * T2 * (runs per pass) <= 131072 (one small counter block each)
 *   keys_out   device uint64 [N*R] or NULL; stats: host or NULL (per-pass sums; scan_ms is not measured)
 * Other arguments, ownership and errors as for rnnd_build_ex. */
int rnnd_build_blocks(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S, int32_t R,
                      int32_t T1, int32_t T2, uint64_t seed, int64_t blocks, int32_t *graph_out,
                      int32_t *degree_out, uint64_t *keys_out, rnnd_stats *stats, void *stream);

/* n_passes block-sequential UpdateNeighbors passes (see rnnd_build_blocks) applied in place to a
 * snapshot.  stats (host, may be NULL) receives the per-pass counters. */
int rnnd_update_neighbors_blocks(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t R,
                                 uint64_t *keys, int32_t *deg, int32_t n_passes, int64_t blocks,
                                 rnnd_stats *stats, void *stream);

/* Bytes of device workspace a build of `rounds` = T1 * T2 UpdateNeighbors rounds (times the runs per pass for
 * rnnd_build_blocks; at most 131072) needs for these sizes (an upper bound; for rnnd_build_wide pass M as R).
 * The library allocates it at the first call that needs it and keeps it, per device, for later calls (a
 * larger request replaces it); rnnd_release_workspace hands it back. */
int rnnd_workspace_bytes(int64_t N, int32_t d, int dtype, int32_t R, int64_t rounds, size_t *bytes);

/* Frees the workspace block the library keeps on the current device between calls (no-op if there is none
 * or a call is using it). */
int rnnd_release_workspace(void);

/* rnnd_build for callers that cannot allocate device memory (code that runs under HIP graph capture
 * elsewhere in the process, tight serving loops, harnesses that forbid hipMalloc): the same build with the
 * workspace in a static device array of RNND_STATIC_SCRATCH_BYTES that the library's code object carries
 * (every device the library runs on holds its copy until the process ends).  The call performs no
 * hipMalloc, hipFree, event creation or any other allocating call, on the device or through a library.
 *   limit   rnnd_workspace_bytes(N, d, dtype, R, T1*T2) <= RNND_STATIC_SCRATCH_BYTES, else RNND_ERR_SCRATCH
 *           (e.g. N = 5,000 x d = 32 uint8 with R = 32 needs 8 MB; N = 17,000 x 128 with R = 96 just fits)
 *   sharing every call on a device works in that device's one array, which keeps the previous call's
 *           contents (what must start at zero is cleared by a kernel on `stream`): calls that overlap in
 *           time on one device race and give undefined graphs -- serialise them.
 * Arguments, result, ownership and the other errors as for rnnd_build; same graph, bit for bit. */
int rnnd_build_static(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S, int32_t R,
                      int32_t T1, int32_t T2, uint64_t seed, int32_t *graph_out, int32_t *degree_out,
                      void *stream);

/* Testing aid: with on != 0 every workspace (kept block, fresh allocation or static array) is filled with
 * 0xA5 bytes before a call clears what it needs cleared, so that a kernel that relies on memory the library
 * never initialised shows up as a wrong result instead of passing on zeroed pages.  Process-wide. */
int rnnd_set_workspace_poison(int on);

/* Where the per-round times of rnnd_stats (round_ms, scan_ms, reverse_ms) come from.  Process-wide.
 *   0 (default)  the device's constant-rate clock, read by the kernels themselves (the first workgroup of a round's
 *                first scan launch, of its scatter launch, ...): costs nothing, so a build with statistics takes as
 *                long as one without; a scan's time then includes the dispatch of the kernel that follows it
 *   1            HIP events attached to the launches (hipExtLaunchKernelGGL): each holds the queue for 4-7
 *                microseconds after its kernel, three per round
 * Block-sequential builds always use events (one per pass).  Returns RNND_OK. */
int rnnd_set_event_timing(int on);

/* RandomGraph(S) (first step of Alg. 6): row u <- S distinct ids != u drawn from a counter-based
 * generator (draw j of vertex u = mix64(mix64(seed + G*(u+1)) + G*(j+1)), mix64 = splitmix64's
 * output function, G = 0x9E3779B97F4A7C15; id = c + (c >= u) with c = ((draw >> 32) * (N-1)) >> 32;
 * repeats are skipped), with delta(u, id), flag new, sorted.  Writes keys [N*R] and deg [N]. */
int rnnd_random_graph(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t S,
                      int32_t R, uint64_t seed, uint64_t *keys, int32_t *deg, void *stream);

/* n_rounds synchronous UpdateNeighbors rounds (Alg. 4) applied in place to a snapshot.
 * stats (host, may be NULL) receives the per-round counters, round_ms and scan_ms (device clock). */
int rnnd_update_neighbors(const void *X, int64_t N, int32_t d, int dtype, int metric, int32_t R,
                          uint64_t *keys, int32_t *deg, int32_t n_rounds, rnnd_stats *stats,
                          void *stream);

/* AddReverseEdges(G, R) (Alg. 5) applied in place to a snapshot: union with the reversed edges
 * (flag new, existing entries keep theirs), then every out-list is cut to its R shortest, then
 * every in-list is cut to its R shortest by (delta, source id). */
int rnnd_add_reverse_edges(int64_t N, int32_t R, uint64_t *keys, int32_t *deg, void *stream);

/* The same on a snapshot whose rows are M >= R slots wide and may hold up to M entries on entry (the state
 * rnnd_build_wide is in between two calls): afterwards every out-list and every in-list holds at most R.
 * keys: device uint64 [N * M].  M = R is rnnd_add_reverse_edges. */
int rnnd_add_reverse_edges_wide(int64_t N, int32_t R, int32_t M, uint64_t *keys, int32_t *deg, void *stream);

/* Snapshot -> output format of rnnd_build (ids, -1 padded; degrees). */
int rnnd_export_graph(int64_t N, int32_t R, const uint64_t *keys, const int32_t *deg,
                      int32_t *graph_out, int32_t *degree_out, void *stream);

/* Search (Alg. 1) on a built graph, with the out-degree cap K of Eq. 4 (Sec. 4.4; studied in Sec. 5.4): for each of nq
 * queries, the candidate list C of at most L points starts from min(L, N) distinct seeded random
 * vertices (InitializeCandidates is not specified by the paper; the generator is the one RandomGraph
 * uses, keyed by seed + 0x9E3779B97F4A7C15 * query index), the nearest unvisited member of C is
 * expanded through its first min(degree, K) neighbours until C holds no unvisited point, and the k
 * nearest members of C are written, nearest first, ties by id.
 *   X          device, N x d row-major, as for rnnd_build; graph / degree: device, the output format of
 *              rnnd_build (row u = neighbour ids nearest-first, degree[u] valid entries), rows
 *              row_stride ints apart; entries that are not vertex ids are ignored.
 *   Q          device, nq x d row-major, same dtype as X.
 *   L, K, k    1 <= k <= L <= 128, K >= 1 (K >= row_stride: no cap).
 *   out_ids    device, nq x k; -1 where C has fewer than k members.
 *   out_dist_bits  device, nq x k, or NULL: delta(q, id) as for the build's keys (the int32 value for
 *              uint8 data, the float's bit pattern for float32); 0xFFFFFFFF where out_ids is -1.
 *   dist_evals host, or NULL: number of delta(q, .) evaluations over all queries.
 * Work is enqueued on `stream` and the call returns after it has completed; a bitmap of N bits per
 * wavefront in flight (at most 1 GiB in all) lives in the workspace block the library keeps between calls
 * (see rnnd_workspace_bytes).  Caller keeps ownership of every buffer.  Errors as for rnnd_build (RNND_ERR_BAD_PARAM for L, K, k, row_stride). */
int rnnd_search(const void *X, int64_t N, int32_t d, int dtype, int metric, const int32_t *graph,
                const int32_t *degree, int32_t row_stride, const void *Q, int64_t nq, int32_t L,
                int32_t K, int32_t k, uint64_t seed, int32_t *out_ids, uint32_t *out_dist_bits,
                int64_t *dist_evals, void *stream);

/* Measurement aid, not a step of the method: the rate at which this GPU delivers random whole rows
 * when a kernel does nothing but gather them with the scan kernels' access pattern (16 bytes per
 * lane, up to 8 lanes per row, row numbers from the counter generator), i.e. the ceiling that the
 * gather-bound UpdateNeighbors scan is compared with besides the HBM peak.
 *   X           device, n_rows rows of row_bytes bytes (a multiple of 16, at most 1 MiB), 16-byte aligned
 *   n_gather    rows to read in the timed pass (rounded up to a whole number of wavefront trips)
 *   gbytes_per_s  host: rows read x row_bytes / time of the second of two passes, in GB/s
 * Returns after the work has completed; allocates and frees a few MB of device memory. */
int rnnd_probe_gather(const void *X, int64_t n_rows, int64_t row_bytes, int64_t n_gather, uint64_t seed,
                      double *gbytes_per_s, void *stream);

/* A second probe with the lane -> address map as its only variable: lanes_per_row = 1, 2, 4 or 8 lanes read
 * one row together, each its share of the row's 16-byte pieces (lanes_per_row pieces apart), so that one load
 * instruction of a wavefront touches 64 / lanes_per_row rows with 16 x lanes_per_row contiguous bytes of each
 * (2 is the operand layout of the 32x32x32 int8 matrix instruction that the uint8 scan gathers into, 4 that
 * of the 16x16x64 one, 8 whole 128-byte lines).  Every lane keeps 8 loads of 16 bytes in flight whatever the
 * map.  row_bytes / 16 / lanes_per_row must be 1, 2, 4 or 8 (else RNND_ERR_BAD_PARAM).  Everything else as for
 * rnnd_probe_gather.  For deciding whether a different operand layout could gather faster, without writing
 * the kernel first. */
int rnnd_probe_gather_map(const void *X, int64_t n_rows, int64_t row_bytes, int64_t n_gather, int lanes_per_row,
                          uint64_t seed, double *gbytes_per_s, void *stream);

/* Selects the UpdateNeighbors scan kernel: 0 = automatic (default), 1 = generic pair-at-a-time
 * kernel for every input, 2 = automatic, but the float matrix-core scan works in double precision
 * throughout.  Automatic uses the dense Gram-block kernels on the matrix cores where they apply
 * and the generic kernel otherwise:
 *   uint8 rows with d = 32, 64 or 128: int8 MFMA;
 *   float32 rows with d a multiple of 16, 16-bit rows with d a multiple of 32: a single-precision
 *   Gram block first (fp32 MFMA on float32 rows; f16 / bf16 MFMA on 16-bit rows as stored), every
 *   pair whose outcome lies within that block's error bound decided by the exact distance, and
 *   vertices with very many such pairs redone on the f64 MFMA.
 * All give identical graphs; this exists for testing and profiling.  Process-wide, not thread-safe. */
int rnnd_set_kernel_variant(int variant);

/* Selects how AddReverseEdges transposes the edge set (every edge (u, v) must reach v's list): 0 = by size
 * (default: N >= 262,144 and N <= 2^25 binned, else atomics), 1 = one arrival-number atomic per edge,
 * 2 = binned by target range (blocks count their edges per range of 2,048 targets, a prefix over the counts
 * places them in one array ordered by range, one workgroup per range then numbers the arrivals in LDS; needs
 * N <= 2^25, else falls back to 1).  Both give identical graphs; this exists for testing and profiling.
 * Process-wide, not thread-safe. */
int rnnd_set_transpose_path(int path);

/* Selects how the uint8 matrix-core scan of a round is launched: 0 = by size (default: N <= 524,288 as 2, N <=
 * 2,097,152 as 3, else as 1), 1 = one launch for the three short-list classes and one per longer class (each with the occupancy that
 * suits it), 2 = one launch in which the blocks are divided among all classes in proportion to their work (the
 * classes share one start-up and one tail; pays when no class alone fills the chip), 3 = the short-list launch
 * and one launch shared by all longer classes.  All give identical graphs and counters; this exists for testing
 * and profiling.  No effect on other inputs or where R <= 32 (short lists only); 3 is 1 where R <= 64 (one
 * longer class).  Process-wide, not thread-safe. */
int rnnd_set_scan_launches(int mode);

const char *rnnd_strerror(int status);
int rnnd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RNND_H */
