/*
 * ginex.h - C ABI of the MI355X (gfx950) hot path of the Ginex inspector-executor
 * pipeline (arXiv 2208.09151): superbatch sample -> changeset precomputation ->
 * feature cache initialization -> per-iteration gather + cache update.
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer unless its comment says "host".  The structs
 *    themselves live in host memory; the pointers inside them follow the same rule.
 *  - The caller owns every buffer, including the workspace `ws`; the library allocates
 *    nothing.  Workspace sizes come from the matching *_workspace_bytes query called
 *    with the same shape arguments.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All kernels
 *    of a call are enqueued on it.  The executor calls (ginex_cache_init*, ginex_gather,
 *    ginex_cache_update) only enqueue; ginex_sample_superbatch, ginex_changeset*,
 *    and ginex_neighbor_cache_build also wait for the stream before they return, because
 *    they hand counts back to the host.
 *  - Every function returns 0 (GINEX_OK) or a negative GINEX_ERR_* code; the message of
 *    the last failure on the calling thread is returned by ginex_last_error().
 *    Arguments are validated on the host before anything is launched.  On
 *    GINEX_ERR_CAPACITY the required element counts are written to the host size
 *    outputs and the contents of the output arrays are unspecified.
 *  - Node ids are int32 in [0, num_nodes); CSR offsets are int32 or int64.
 *  - Environment switches, read at every call; none changes a result, only the way to it:
 *      GINEX_VALIDATE=1       check the documented preconditions on the device first
 *      GINEX_TRACE=1          ginex_changeset_resume reports on stderr which way it went
 *      GINEX_SAMPLER_LDS=0    seeds and first hop through the tables in HBM like the later hops
 *      GINEX_SAMPLER_TILES=n  at most n tiles of a batch per workgroup column of the sampler
 *      GINEX_DEAD_SCATTER=0/1 evictions among dead rows from a pass over the lines / from the id bitmap
 *      GINEX_LIVE_SELECT=1    no shortcut that relies on the cache holding the whole superbatch
 *      GINEX_STATIC_THRESHOLDS=0  Belady thresholds from histograms of the cache state, iteration by
 *                             iteration, instead of from the trace alone in front of the loop
 *      GINEX_PLANNED=0/2      a carried cache that holds the whole superbatch: still the general
 *                             loop / the three-launch steps also where the replay would do
 */
#ifndef GINEX_H
#define GINEX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GINEX_OK 0
#define GINEX_ERR_ARG (-1)        /* null pointer, negative size, unsupported shape   */
#define GINEX_ERR_CAPACITY (-2)   /* an output array is too small                     */
#define GINEX_ERR_WORKSPACE (-3)  /* ws_bytes below the *_workspace_bytes figure      */
#define GINEX_ERR_INPUT (-4)      /* the data violates a documented precondition      */
#define GINEX_ERR_HIP (-5)        /* a HIP runtime call failed                        */

#define GINEX_MAX_FANOUT 64
#define GINEX_MAX_HOPS 8

/* Message of the last error on this thread ("" if none). Owned by the library. */
const char* ginex_last_error(void);
/* Library version: major*10000 + minor*100 + patch. */
int32_t ginex_version(void);

/* Graph in CSR form.  Row v lists the nodes that may be sampled for v (the paper stores
 * in-neighbours, Section 2.2); multi-edges are allowed. */
typedef struct ginex_csr {
  int64_t num_nodes;
  int64_t num_edges;
  const void* offsets;     /* [num_nodes+1], int32 if offsets_64 == 0, else int64 */
  int32_t offsets_64;
  const int32_t* indices;  /* [num_edges] */
  /* Optional neighbour cache (Section 3.2), both NULL or both set: built by
   * ginex_neighbor_cache_build over this same graph.  The sampler then serves the rows of
   * cached nodes from nc_cache_array (HBM) and only the others from offsets/indices, which
   * may then live in host-pinned memory.  The sampled result does not depend on it. */
  const int64_t* nc_address_table; /* device [num_nodes] */
  const int32_t* nc_cache_array;   /* device */
} ginex_csr_t;

/* ---------------------------------------------------------------------------------
 * Superbatch sample (Section 3.1 "Superbatch Sample"; sampling rule of Section 2.1
 * "Neighborhood Sampling"): samples S batches at once and returns, per batch, `ids`
 * (the 1-D list of all sampled node ids) and `adj` (the connectivity among them).
 *
 * Batch b (global index first_batch_index+b) starts from seeds[seed_offsets[b] ..
 * seed_offsets[b+1]).  At hop h every node in the batch's list at the start of the hop
 * draws min(degree, fanout[h]) distinct positions of its CSR row, uniformly, from a
 * Philox4x32-10 stream keyed by rng_seed with counter (node, global batch, hop, draw);
 * unseen neighbours are appended to the list in the order frontier node by frontier
 * node, pick by ascending row position.  The result for a batch depends only on its
 * seeds, its global index and rng_seed.
 *
 * Outputs
 *   ids[ids_offsets[b] .. ids_offsets[b+1])   the list of batch b (seeds first, a seed
 *                                              repeated within a batch is kept once)
 *   ids_offsets (host, [S+1]), hop_sizes (host, [S*(H+1)]): hop_sizes[b*(H+1)+h] is the
 *                                              list length after the seeds (h=0) and
 *                                              after hop h-1 (h>=1)
 *   adj: segment g = h*S + b (hop-major) describes hop h of batch b as a CSR over the
 *   frontier: adj_rowptr[adj_row_offsets[g] + r], r = 0..frontier, starts at 0, and
 *   adj_col[adj_col_offsets[g] + e] is the position inside the batch's ids of pick e;
 *   row r belongs to ids[r].  adj_row_offsets/adj_col_offsets (host) have S*H+1 entries.
 *   Pass adj_rowptr = adj_col = NULL to skip adj (offset arrays are still filled).
 *   totals (host, [3]): number of ids, of rowptr entries and of col entries (= sampled
 *   edges) produced, or required on GINEX_ERR_CAPACITY.
 * Limits: 1 <= H <= GINEX_MAX_HOPS, 1 <= fanout[h] <= GINEX_MAX_FANOUT, and a batch's
 * list must stay below 2^30 entries.  Seeds must lie in [0, num_nodes) and the CSR must be
 * well formed (offsets from 0 to num_edges without a decrease, indices in range): unchecked
 * by default, checked on the device first (GINEX_ERR_INPUT) when GINEX_VALIDATE=1 is set in
 * the environment.
 * ------------------------------------------------------------------------------- */
size_t ginex_sample_workspace_bytes(int64_t num_nodes, int32_t S, int64_t max_batch,
                                    const int32_t* fanout /*host [H]*/, int32_t H);

int32_t ginex_sample_superbatch(
    const ginex_csr_t* g /*host struct*/,
    const int32_t* seeds, const int64_t* seed_offsets /*host [S+1]*/, int32_t S,
    const int32_t* fanout /*host [H]*/, int32_t H,
    uint64_t rng_seed, uint32_t first_batch_index,
    int32_t* ids, int64_t ids_capacity, int64_t* ids_offsets /*host [S+1]*/,
    int64_t* hop_sizes /*host [S*(H+1)]*/,
    int64_t* adj_rowptr, int64_t rowptr_capacity, int32_t* adj_col, int64_t col_capacity,
    int64_t* adj_row_offsets /*host [S*H+1]*/, int64_t* adj_col_offsets /*host [S*H+1]*/,
    int64_t* totals /*host [3]*/,
    void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------
 * Neighbour cache construction (Section 3.2 "Neighbor Cache Policy" and "Neighbor Cache
 * Structure").  Ranks the nodes by out-degree / in-degree, larger first (in-degree = length
 * of the node's CSR row, out-degree = number of times the node occurs in `indices`; the
 * ratio is compared as the integer floor(out * 2^32 / in), ties go to the smaller id, nodes
 * with an empty row are never cached) and stores the rows of the best-ranked nodes back to
 * back from index 0 of cache_array, each as a record (neighbour count, neighbour ids),
 * stopping at the first node whose record does not fit into `budget` entries.
 *   address_table (device, [num_nodes]): index of the node's record in cache_array, or -1
 *   cache_array   (device, [budget])
 *   cached_nodes, used_entries (host): number of records and of cache_array entries used
 * g->offsets and g->indices may be device or host-pinned memory; g's nc_* fields are
 * ignored.  An entry of indices outside [0, num_nodes) returns GINEX_ERR_INPUT (offsets are
 * trusted).  The call waits for the stream before it returns.
 * ------------------------------------------------------------------------------- */
size_t ginex_neighbor_cache_workspace_bytes(int64_t num_nodes);

int32_t ginex_neighbor_cache_build(const ginex_csr_t* g /*host struct*/, int64_t budget,
                                   int64_t* address_table, int32_t* cache_array,
                                   int64_t* cached_nodes /*host*/, int64_t* used_entries /*host*/,
                                   void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------
 * Changeset precomputation (Section 3.4; lists of Section 3.3 "Feature Cache Update").
 * Given the access trace ids_0 .. ids_{S-1} of a superbatch (ids within one iteration
 * distinct) and a cache of `cap` rows, computes
 *   C_0       the cap rows accessed earliest (ties: smaller id), row of rank r in line r;
 *   C_{i+1}   the cap elements of union(C_i, ids_i) whose next accessed iteration is
 *             smallest (ties: a resident row before an incoming one, then smaller id);
 *   per iteration i: in_ids = C_{i+1}\C_i ordered by position in ids_i, in_positions =
 *   those positions, out_ids = C_i\C_{i+1} ordered by cache line; in_ids[j] takes the
 *   line of out_ids[j].  Records of iteration i occupy [cs_offsets[i], cs_offsets[i+1]).
 *   miss_count[i] = |ids_i \ C_i|.
 *   src_line (device, [ids_offsets[S]], may be NULL): for every access p of iteration i, the
 *   cache line that holds ids[p] in C_i, or -1 if the row is not resident then.  It is what
 *   the address table of Section 3.3 would return at gather time, resolved ahead of time, so
 *   that the executor's gather (ginex_gather_lines) reads it sequentially instead of probing
 *   the table; it holds for an executor that loads C_0 line by line and applies every
 *   changeset in order.
 * init_count and total_changes are host outputs.  cs_capacity >= total_changes is
 * required (ids_offsets[S] always suffices).
 * init_ready (host, [S], may be NULL): init_ready[i] = number of rows of C_0 first accessed
 * in iterations 0..i.  C_0 is ordered by first access, so iteration i only reads cache
 * lines below init_ready[i]: an executor may load C_0 in pieces (ginex_cache_init_part)
 * and start iteration i as soon as that prefix is in place, provided no changeset has been
 * applied yet (a changeset may evict a row that was not loaded yet).
 * Preconditions (ids in range, ids distinct inside an iteration) are the caller's duty and
 * unchecked by default; with GINEX_VALIDATE=1 in the environment they are checked on the
 * device first and a violation returns GINEX_ERR_INPUT before anything else runs.
 * Limits: 1 <= S <= 8191, total ids < 2^31.
 * ------------------------------------------------------------------------------- */
size_t ginex_changeset_workspace_bytes(int64_t num_nodes, int64_t total_ids, int32_t S,
                                       int64_t cap);

int32_t ginex_changeset(
    int64_t num_nodes, const int32_t* ids, const int64_t* ids_offsets /*host [S+1]*/,
    int32_t S, int64_t cap,
    int32_t* init_ids /*[cap]*/, int64_t* init_count /*host*/,
    int32_t* in_ids, int32_t* out_ids, int32_t* in_positions, int64_t cs_capacity,
    int64_t* cs_offsets /*[S+1]*/, int64_t* miss_count /*[S]*/,
    int32_t* src_line /*[total ids] or NULL*/,
    int64_t* total_changes /*host*/, int64_t* init_ready /*host [S] or NULL*/,
    void* ws, size_t ws_bytes, void* stream);

/* The same precomputation for the LRU policy (Section 2.3 and Figure 2: the policy that
 * Belady's is compared with), so that both run through the same executor and their miss
 * counts can be compared on one trace.  Arguments, outputs, workspace and limits are those
 * of ginex_changeset.  C_0 is the same prefetch as above, its rows counting as not used yet;
 * C_{i+1} keeps the cap elements of union(C_i, ids_i) used most recently (ties: a resident
 * row before an incoming one, then smaller id), so the rows of ids_i outrank every other. */
int32_t ginex_changeset_lru(
    int64_t num_nodes, const int32_t* ids, const int64_t* ids_offsets /*host [S+1]*/,
    int32_t S, int64_t cap,
    int32_t* init_ids /*[cap]*/, int64_t* init_count /*host*/,
    int32_t* in_ids, int32_t* out_ids, int32_t* in_positions, int64_t cs_capacity,
    int64_t* cs_offsets /*[S+1]*/, int64_t* miss_count /*[S]*/,
    int32_t* src_line /*[total ids] or NULL*/,
    int64_t* total_changes /*host*/, int64_t* init_ready /*host [S] or NULL*/,
    void* ws, size_t ws_bytes, void* stream);

/* ginex_changeset for callers that cannot allocate device memory or hand over a workspace
 * (code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc): the same arguments, outputs, order and limits, without `ws`.  The scratch
 * memory is an array of GINEX_NOALLOC_SCRATCH_BYTES built into the library, one copy per GPU,
 * held until the process ends; the call allocates nothing on the device and frees nothing.
 * A shape whose ginex_changeset_workspace_bytes figure exceeds that size is rejected with
 * GINEX_ERR_WORKSPACE before anything is launched.  All calls on one GPU share the array:
 * calls that overlap in time on the same GPU (other streams, other threads) race; one after
 * the other they are independent, the array needs no clearing by the caller. */
#define GINEX_NOALLOC_SCRATCH_BYTES (64ll << 20)

int32_t ginex_changeset_noalloc(
    int64_t num_nodes, const int32_t* ids, const int64_t* ids_offsets /*host [S+1]*/,
    int32_t S, int64_t cap,
    int32_t* init_ids /*[cap]*/, int64_t* init_count /*host*/,
    int32_t* in_ids, int32_t* out_ids, int32_t* in_positions, int64_t cs_capacity,
    int64_t* cs_offsets /*[S+1]*/, int64_t* miss_count /*[S]*/,
    int32_t* src_line /*[total ids] or NULL*/,
    int64_t* total_changes /*host*/, int64_t* init_ready /*host [S] or NULL*/,
    void* stream);

/* Belady changesets of a superbatch that starts from the cache the previous superbatch left
 * behind (an extension: the paper prefetches a fresh C_0 for every superbatch, Section 3.1,
 * which costs one slow-tier read per distinct row per superbatch; carried over, only rows
 * that are not resident any more are read, as ordinary misses).  C_0 is given: cache line r
 * holds start_ids[r] (device, [cap], all distinct and in range: checked, GINEX_ERR_INPUT).
 * The cache must be full, 1 <= cap.  A resident row that the superbatch never accesses has
 * next accessed iteration "never" and is evicted first (larger id first).  The recurrence,
 * the lists and their order are those of ginex_changeset.  final_ids (device, [cap], may be
 * NULL) receives the row of every line after the last iteration: the start_ids of the next
 * superbatch.  No cache initialization is needed between the two superbatches.
 * When the cache also has a line for every distinct row of the superbatch, no iteration
 * evicts a row that is still needed: hits, misses and insertions are known up front and only
 * the choice of the evicted rows follows the iterations, replayed by one workgroup or, for
 * more candidates or evictions than that holds, in three small launches per iteration
 * (same result; GINEX_PLANNED=0 in the environment keeps the general loop, 2 takes the
 * three-launch way also where the replay would do, GINEX_TRACE=1 reports on stderr which way
 * a call went). */
int32_t ginex_changeset_resume(
    int64_t num_nodes, const int32_t* ids, const int64_t* ids_offsets /*host [S+1]*/,
    int32_t S, int64_t cap, const int32_t* start_ids /*[cap]*/, int32_t* final_ids /*[cap]*/,
    int32_t* in_ids, int32_t* out_ids, int32_t* in_positions, int64_t cs_capacity,
    int64_t* cs_offsets /*[S+1]*/, int64_t* miss_count /*[S]*/,
    int32_t* src_line /*[total ids] or NULL*/,
    int64_t* total_changes /*host*/,
    void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------
 * Feature cache (Section 3.3 "Feature Cache Structure"): a 2-D array of `cap` rows in
 * HBM plus an address table with one entry per node (cache line, or -1).  `slow` is the
 * full feature table [num_nodes x row_bytes] in memory the GPU can read: host-pinned
 * memory standing in for the SSD tier, or device memory.  row_bytes % 16 == 0 and every
 * base pointer 16-byte aligned.
 * ------------------------------------------------------------------------------- */
typedef struct ginex_cache {
  void* rows;
  int64_t cap;
  int64_t row_bytes;
  int32_t* addr;
  int64_t num_nodes;
  const void* slow;
} ginex_cache_t;

/* Feature cache initialization (Section 3.1): addr[*] = -1, then row init_ids[r] is
 * loaded into line r and addr[init_ids[r]] = r.  init_count <= cap. */
int32_t ginex_cache_init(const ginex_cache_t* c /*host struct*/, const int32_t* init_ids,
                         int64_t init_count, void* stream);

/* The same initialization in pieces (Section 3.1; the paper runs the initialization as one
 * stage in front of the main loop, here the main loop may start under it): loads rows
 * init_ids[begin .. end) into lines begin .. end-1.  The piece with begin == 0 resets the
 * address table first, so pieces are issued in ascending order on one stream.
 * 0 <= begin <= end <= cap. */
int32_t ginex_cache_init_part(const ginex_cache_t* c /*host struct*/, const int32_t* init_ids,
                              int64_t begin, int64_t end, void* stream);

/* Initialization of the next superbatch's cache with the previous one still in HBM (the
 * paper reloads every row from storage, Section 3.1; here a row of the new C_0 that `prev`
 * still holds is copied from prev's line, HBM to HBM, and only the others cross the host
 * link).  Same pieces and the same resulting cache content as ginex_cache_init_part.  `c`
 * and `prev` front the same slow tier with the same row size and share no array; `prev` is
 * only read. */
int32_t ginex_cache_init_warm(const ginex_cache_t* c /*host struct*/,
                              const ginex_cache_t* prev /*host struct*/,
                              const int32_t* init_ids, int64_t begin, int64_t end, void* stream);

/* One executor iteration (Section 3.1 "Main Loop", Section 3.3 worked example):
 * gather   out[p,:] = addr[ids[p]] >= 0 ? rows[addr[ids[p]],:] : slow[ids[p],:]
 * then the cache update  line = addr[out_ids[j]]; rows[line,:] = out[in_positions[j],:];
 *                        addr[out_ids[j]] = -1; addr[in_ids[j]] = line.
 * `out` is [n x row_bytes] in HBM.  n_change may be 0 (then the three lists may be
 * NULL). */
int32_t ginex_gather(const ginex_cache_t* c /*host struct*/, const int32_t* ids, int64_t n,
                     void* out, const int32_t* in_ids, const int32_t* out_ids,
                     const int32_t* in_positions, int64_t n_change, void* stream);

/* The same iteration with the address-table lookups resolved ahead of time: src_line[p]
 * (device, [n]) is the cache line of ids[p], or -1 for a row to be read from the slow tier
 * (the src_line output of ginex_changeset* for this iteration).  The gather reads src_line
 * and ids sequentially and never probes the address table; the update is the one of
 * ginex_gather and keeps the address table current, so the two calls may be mixed.  The
 * gathered bytes equal those of ginex_gather provided src_line describes the cache as it
 * stands (checked by the caller's bookkeeping, not by the kernel).
 * n_slow: how many entries of src_line are -1 (miss_count[i] of the changeset call), or -1 if
 * not known.  Only a hint for the launch shape: an iteration with many slow-tier rows is bound
 * by the host link, which a smaller grid uses better; the result does not depend on it. */
int32_t ginex_gather_lines(const ginex_cache_t* c /*host struct*/, const int32_t* ids,
                           const int32_t* src_line, int64_t n, int64_t n_slow, void* out,
                           const int32_t* in_ids, const int32_t* out_ids,
                           const int32_t* in_positions, int64_t n_change, void* stream);

/* The cache update of one iteration on its own (Section 3.1 "Main Loop": the step between
 * gather and transfer; Section 3.3 "Feature Cache Update"): exactly the second half of
 * ginex_gather, for callers that gather with n_change = 0 and update separately.  `out`
 * is the batch input that the gather of the same iteration produced. */
int32_t ginex_cache_update(const ginex_cache_t* c /*host struct*/, const void* out,
                           const int32_t* in_ids, const int32_t* out_ids,
                           const int32_t* in_positions, int64_t n_change, void* stream);

/* ---------------------------------------------------------------------------------
 * Static cache policy (Section 2.3 "Challenge 1": the policy the paper compares Belady's
 * with keeps the nodes of highest out-degree in memory and never replaces them; Figure
 * "miss ratio over cache size").  With CSR rows holding in-neighbours, a node's out-degree
 * is the number of times it occurs in g->indices (device or host-pinned memory; g->offsets
 * and the nc_* fields are not read).  static_ids[r] (device, [min(cap, num_nodes)]) receives
 * the node of rank r: larger out-degree first, smaller id first among equal out-degrees.
 * count (host) receives min(cap, num_nodes).  An entry of indices outside [0, num_nodes)
 * returns GINEX_ERR_INPUT.  The call waits for the stream before it returns.
 * A static run is ginex_cache_init(static_ids) followed by ginex_gather calls with
 * n_change = 0.
 * ------------------------------------------------------------------------------- */
size_t ginex_static_select_workspace_bytes(int64_t num_nodes);

int32_t ginex_static_select(const ginex_csr_t* g /*host struct*/, int64_t cap,
                            int32_t* static_ids, int64_t* count /*host*/,
                            void* ws, size_t ws_bytes, void* stream);

/* Misses of one iteration against the cache as it stands (Section 3.3: an id whose
 * address-table entry is -1 is read from the slow tier): adds |{p : addr[ids[p]] < 0}| to
 * *misses (device, 8-byte aligned; the caller zeroes it).  For policies whose changesets do
 * not carry miss counts (the static cache).  Only enqueues. */
int32_t ginex_cache_count_misses(const ginex_cache_t* c /*host struct*/, const int32_t* ids,
                                 int64_t n, int64_t* misses, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* GINEX_H */
