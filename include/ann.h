/*
 * ann.h - C ABI of the MI355X (gfx950) batched graph-ANN search library.
 *
 * The library implements the data-parallel hot path of the VSAG search method
 * (arXiv 2503.17911): best-first search over a fixed-degree proximity graph
 * with scalar-quantized traversal distances, an exact fp32 rerank, and an
 * exhaustive exact top-k used as ground truth for recall.
 *
 * Conventions that hold for every call
 *   - All array arguments are DEVICE pointers unless a comment says "host".
 *     The caller owns every input and output buffer; the library owns only the
 *     packed index it builds in ann_upload_index and the workspaces for folded
 *     queries it keeps with that index (one per stream, see below).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return without waiting, except where noted.
 *   - Ids are uint32_t < 2^31.  ANN_PAD_ID marks "no entry"; result lists
 *     shorter than requested are padded with ANN_PAD_ID and +infinity.
 *   - A "distance" is smaller-is-better: squared L2, or the NEGATED inner
 *     product for ANN_IP.
 *   - Every function returns an ann_status.  Argument errors are detected on
 *     the host before anything is launched; ann_last_error() then returns a
 *     message (thread-local, valid until the next call on that thread).
 *   - No C++ exception crosses this boundary.
 *   - Several batches in flight on one index: calls that fold queries for an
 *     index (ann_search_batch, ann_entry_scan, ann_query_prep, ann_rescore)
 *     use a workspace the index keeps per stream, so batches issued on
 *     different streams may run at the same time, and batches on one stream
 *     follow each other as stream order says.  An index keeps up to 8 such
 *     workspaces; a 9th stream takes over the least recently used one after a
 *     device-wide wait.  A workspace grows (hipMalloc, device-wide wait) when a
 *     batch is larger than any before it on that stream; ann_reserve_workspace
 *     sizes it ahead of time, after which no call on that stream allocates for
 *     batches up to the reserved size.  Calls for one index may come from
 *     several host threads as long as no two of them use the same stream at once.
 */
#ifndef ANN_H_
#define ANN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ANN_PAD_ID 0xFFFFFFFFu
#define ANN_MAX_LEVELS 2
#define ANN_MAX_EF 512u
#define ANN_MAX_DEGREE 64u
#define ANN_MAX_ENTRIES 64u
#define ANN_STATIC_SCRATCH_BYTES (8u << 20) /* see ann_search_batch_static */

typedef struct ann_index ann_index; /* opaque; device memory owned by the library */

typedef enum {
  ANN_OK = 0,
  ANN_EINVAL = 1,       /* bad argument; nothing was launched                 */
  ANN_ENOMEM = 2,       /* device or host allocation failed                   */
  ANN_EDEVICE = 3,      /* a HIP call failed (message has the HIP error)      */
  ANN_EUNSUPPORTED = 4, /* valid request outside the built kernel variants    */
  ANN_ECAPACITY = 5     /* a size exceeds a documented maximum                */
} ann_status;

typedef enum { ANN_L2 = 0, ANN_IP = 1 } ann_metric;

/* ann_index_desc.flags */
#define ANN_DESC_HOST_POINTERS 1u /* every array in the descriptor is in HOST memory */
/*
 * For ANN_IP indexes whose base vectors have unit norm (an improvement of the
 * low-precision distance in the sense of the paper's Appendix G): traversal,
 * entry-scan and rescore keys take the Euclidean form of Section 5.2,
 * ||x^||^2 - 2 q.x^ with x^ the decoded vector, instead of -(q.x^).  On exact
 * unit vectors both orders are the same; on decoded vectors the Euclidean form
 * is the squared distance to x^ (minus ||q||^2), in which the part of the
 * quantization error that lies along q - x, short for near neighbours, counts,
 * where -(q.x^) carries the error along q at full length.  Needs norm_term
 * for every level.  ann_rerank and ann_bruteforce_topk are not affected:
 * returned distances stay -<q, x>.
 */
#define ANN_DESC_UNIT_NORM_L2_KEYS 2u
/*
 * Fold queries to 15 bits instead of 8 (a finer low-precision distance in the
 * sense of Appendix G): t_j = rint(a_j * 16256 / max|a|) in [-16256, 16256],
 * s = max|a| / 16256; the value is kept as two signed bytes (t = 128 hi + lo,
 * lo in [-64, 63]) and every code row is multiplied by both (two passes of the
 * packed int8 dot product); the two int32 sums are joined in 64 bits,
 * converted to fp32 with one rounding, and enter the same key formula.  The
 * query's rounding error in q.x^ shrinks by 128; every distance evaluation
 * costs twice the integer work and the folded query twice the bytes.  Applies
 * to every call that folds queries for this index (search, entry scan,
 * rescore, ann_query_prep, whose t output then is int16_t [nq][d]).  out_idot
 * of ann_search_batch must be NULL (the products exceed 32 bits) and
 * ann_rescore writes zeros there.
 */
#define ANN_DESC_QUERY_15BIT 4u

/*
 * One scalar-quantization level (paper Appendix G, SQ-b with b = bits).
 *   codes     [n][row_bytes], row_bytes = d (bits 8) or d/2 (bits 4, d even;
 *             dimension 2i in the low nibble of byte i, 2i+1 in the high one);
 *             code c of dimension j decodes to lo[j] + delta[j] * c.
 *   lo, delta [d] per-dimension minimum and step.
 *   norm_term [n] squared norm of the decoded vector: the one extra fp32 per
 *             base vector of the paper's distance decomposition (Section 5.2).
 *             May be NULL for ANN_IP.
 */
typedef struct {
  uint32_t bits;
  const uint8_t *codes;
  const float *lo;
  const float *delta;
  const float *norm_term;
} ann_sq_level;

/*
 * Everything ann_upload_index needs (the G, D and I of Algorithm 1).
 *   vectors   [n][d] fp32 base vectors for the rerank; NULL disables ann_rerank.
 *   level[0]  codes used during traversal; level[1] (optional) a finer level
 *             for ann_rescore.
 *   adjacency fixed-degree form (csr_offsets == NULL): [n][degree], unused
 *             slots ANN_PAD_ID.  CSR form: csr_offsets is [n+1] and adjacency
 *             holds csr_offsets[n] neighbour ids; rows longer than `degree` are
 *             an error.  degree <= ANN_MAX_DEGREE.
 *   entry_point  default initial node of every search.
 *   edge_labels  optional [n][degree] (same shape as the fixed-degree adjacency,
 *             or [csr_offsets[n]] in CSR form): the label L of every edge
 *             (paper Section 4.3: the smallest pruning rate under which the edge
 *             exists).  NULL: no labels.
 *   A row must not name the same neighbour twice (ANN_EINVAL).
 */
typedef struct {
  uint64_t n;
  uint32_t d;
  uint32_t degree;
  uint32_t metric; /* ann_metric */
  uint32_t n_levels;
  const float *vectors;
  ann_sq_level level[ANN_MAX_LEVELS];
  const uint32_t *adjacency;
  const uint64_t *csr_offsets;
  uint32_t entry_point;
  uint32_t flags;
  const float *edge_labels;
} ann_index_desc;

/*
 * Search parameters (k and ef_s of Algorithm 1 plus launch knobs that change
 * speed only).
 *   ef            pool size, k <= ef <= ANN_MAX_EF.
 *   mode          0: one expansion per step, results identical to a sequential
 *                    execution of Algorithm 1 with (key, id) tie-breaking;
 *                 1: several expansions per step (faster, approximate order of
 *                    expansion; same pool/visited semantics).
 *   expansions_per_step   mode 1 only, 1..8 (0 = library default, see
 *                 ann_default_expansions_per_step): the closest
 *                 un-expanded entries expanded together in one step.  More of
 *                 them shorten a query's chain of dependent steps and evaluate
 *                 more nodes: 8 is faster than 4 where the batch is too small
 *                 to fill the GPU (measured on 1,000 queries with 480-byte code
 *                 rows), slower where it does.
 *   visited_kind, visited_slots   how the visited set V is kept in LDS
 *                 (visited_slots a power of two <= 8192, 0 = library default).
 *                 ANN_VISITED_CACHE: a two-way set-associative cache of node
 *                 ids (least recently entered way replaced); a node pushed out
 *                 of its set is forgotten and may be evaluated again.  A slot
 *                 holds one set of two 16-bit tags while (n - 1) / visited_slots
 *                 stays below 65534 (set and tag together still name exactly
 *                 one node), else a slot holds one node id and a set is two
 *                 slots; ANN_VISITED_CACHE_WIDE asks for the second form
 *                 whatever n is.  ANN_VISITED_TABLE: an
 *                 open-addressing table that holds every evaluated node while it
 *                 fits and is rebuilt from the current pool when 3/4 full.
 *                 Forgetting a node costs a repeated distance evaluation, never
 *                 a different pool: a forgotten node outside the pool is
 *                 rejected again by a pool maximum that only decreases, one
 *                 inside the pool is recognised when it is merged.  The
 *                 exception is the cap m_s, whose choice of neighbours depends
 *                 on V itself: with m_s below the degree the table is used and
 *                 the result is the sequential one only for queries that report
 *                 0 rebuilds in out_counts.  ANN_VISITED_AUTO: the cache, or the
 *                 table (8192 slots by default) when m_s is active.
 *   alpha_s, m_s  the search-time edge filter of Algorithm 1 (Section 4.3): an
 *                 edge is followed only if its label <= alpha_s, and at most
 *                 m_s unvisited neighbours are taken per expansion, in stored
 *                 order.  alpha_s = 0 (labels are >= 1): no label test; needs an
 *                 index uploaded with edge_labels otherwise.  m_s = 0: no cap.
 *   ef_per_query  NULL: every query uses ef.  Otherwise [nq] on the device: query
 *                 i runs Algorithm 1 with pool size min(max(ef_per_query[i], 1),
 *                 ef) - the hook for query-level parameters (Section 4.2, where
 *                 a classifier picks ef_s per query).  Output rows keep the
 *                 stride ef; slots past a query's own pool size are padding.
 *   query_order   NULL: workgroup b searches query b.  Otherwise a permutation of
 *                 0..nq-1 on the device: workgroup b searches query
 *                 query_order[b] (outputs stay at the query's own index).  A
 *                 speed knob: results do not depend on it.
 *   reuse_folded_queries   non-zero: the last folding launched for this index
 *                 on this stream (by ann_entry_scan, ann_query_prep for level 0
 *                 or ann_search_batch) was of this same q and
 *                 nq and q has not changed since; the search skips its own
 *                 folding pass.  ANN_EINVAL if q or nq differ from that call's.
 *   layout        0: neighbour code rows are gathered from the code table;
 *                 1: they are read from the redundant copy made by
 *                    ann_build_prs (same results; not with alpha_s / m_s);
 *                 2: code rows are gathered, and a neighbour's norm term is
 *                    read with the adjacency row (ann_build_row_norms) instead
 *                    of from the per-node array (same results).
 */
typedef enum {
  ANN_VISITED_AUTO = 0,
  ANN_VISITED_CACHE = 1,
  ANN_VISITED_TABLE = 2,
  ANN_VISITED_CACHE_WIDE = 3
} ann_visited_kind;

typedef struct {
  uint32_t k;
  uint32_t ef;
  uint32_t mode;
  uint32_t expansions_per_step;
  uint32_t visited_slots;
  float alpha_s;
  uint32_t m_s;
  uint32_t layout;
  uint32_t visited_kind; /* ann_visited_kind */
  const uint32_t *query_order; /* device, [nq], or NULL: see ann_schedule_queries */
  uint32_t reuse_folded_queries;
  const uint32_t *ef_per_query; /* device, [nq], or NULL */
} ann_search_params;

/*
 * Scalar-quantization codebook and encoder (paper Appendix G; per-dimension
 * range reading).  ann_sq_train writes lo[j] = min_i x[i][j] and delta[j] =
 * (max - min) / (2^bits - 1) (1 if the range is empty).  ann_sq_encode writes
 * codes = clamp(floor((x - lo) / delta + 0.5), 0, 2^bits - 1) in the layout of
 * ann_sq_level and, if norm_term != NULL, the squared norms of the decoded rows
 * (fp64 accumulation in dimension order, rounded once).
 *   x [n][d] fp32; bits 8 or 4 (d even for 4).  Both calls allocate a small
 *   temporary and synchronise the stream before returning.
 */
ann_status ann_sq_train(const float *x, uint64_t n, uint32_t d, uint32_t bits, float *lo, float *delta,
                        void *stream);
/*
 * Truncated scalar quantization (paper Appendix G: the range comes from
 * percentile statistics rather than the extremes).  With a column sorted
 * ascending, lo[j] is its element of rank k = floor((1 - coverage) * (n - 1))
 * and the upper end its element of rank n - 1 - k (exact order statistics);
 * coverage in (0.5, 1], 0.99 being the paper's choice, 1 the same as
 * ann_sq_train.  ann_sq_encode clamps values outside the range.
 */
ann_status ann_sq_train_truncated(const float *x, uint64_t n, uint32_t d, uint32_t bits, double coverage,
                                  float *lo, float *delta, void *stream);
ann_status ann_sq_encode(const float *x, uint64_t n, uint32_t d, uint32_t bits, const float *lo,
                         const float *delta, uint8_t *codes, float *norm_term, void *stream);

/*
 * Build the device index: copy (or upload) the arrays of `desc`, repack codes
 * into 16-byte aligned rows and the adjacency into [n][degree].  Synchronous;
 * the descriptor's arrays may be released afterwards.  *out receives the index.
 * Errors: ANN_EINVAL (NULL arrays, n == 0 or n >= 2^31, degree == 0, bits not
 * 4/8, odd d with 4 bits, entry_point >= n, neighbour id >= n, repeated neighbour
 * in a row), ANN_ECAPACITY
 * (degree > ANN_MAX_DEGREE, d > 2048), ANN_ENOMEM, ANN_EDEVICE.
 */
ann_status ann_upload_index(const ann_index_desc *desc, void *stream, ann_index **out);
ann_status ann_free_index(ann_index *index); /* synchronises the device; NULL is a no-op */

/*
 * Size the folded-query workspaces of `stream` (every code level of the index)
 * for batches of up to max_nq queries, so that the calls that fold queries
 * (ann_search_batch, ann_entry_scan, ann_query_prep, ann_rescore) never
 * allocate on that stream for nq <= max_nq: Algorithm 1's per-query state is
 * then set up without touching the allocator.  May allocate and wait for the
 * device; call it once after ann_upload_index, per stream that will be used.
 * Errors: ANN_EINVAL (NULL index, max_nq == 0), ANN_ENOMEM, ANN_EDEVICE.
 */
ann_status ann_reserve_workspace(ann_index *index, uint32_t max_nq, void *stream);

/*
 * Query folding for one code level (the query side of the low-precision
 * distance; paper Section 5.2 precomputes the query terms before the search):
 * a_j = delta_j * q_j, s = max|a| / 127, t_j = rint(a_j * 127 / max|a|) as
 * int8, qlo = sum_j q_j * lo_j.  Outputs (any may be NULL): t [nq][d] int8,
 * s [nq], qlo [nq].  ann_search_batch does this internally; the entry point
 * exists so the folded query can be inspected.
 */
ann_status ann_query_prep(ann_index *index, uint32_t level, const float *q, uint32_t nq, int8_t *t, float *s,
                          float *qlo, void *stream);

/*
 * Redundant vector storage (the paper's PRS layout, Section 3.3, redundancy
 * ratio 1): stores, for every node, the level-0 code rows and norm terms of its
 * neighbours next to each other in slot order, so that an expansion reads them
 * in one sequential sweep together with the id row.  Costs n * degree *
 * row_stride bytes of device memory.  Synchronous; a second call is a no-op.
 * Errors: ANN_EINVAL, ANN_ENOMEM.
 */
ann_status ann_build_prs(ann_index *index, void *stream);
/*
 * Redundant storage of the norm terms alone (the light end of the paper's
 * redundant layout, Section 3.3; the norm term is the extra fp32 per vector of
 * Section 5.2's decomposition): every adjacency row is stored followed by the
 * level-0 norm terms of its neighbours in slot order, so that a distance
 * evaluation needs the neighbour's code row only, not a second scattered read
 * for four bytes.  Used by searches with layout = 2.  Costs n * degree * 8
 * bytes of device memory beside the plain adjacency.  Synchronous; a second
 * call is a no-op.  Errors: ANN_EINVAL (NULL index; keys of the index use no
 * norm term: inner-product keys), ANN_ENOMEM.
 */
ann_status ann_build_row_norms(ann_index *index, void *stream);
/*
 * The same with a redundancy ratio below 1 (the paper's delta, Section 3.3):
 * only the first ceil(ratio * degree) slots of every adjacency row get their
 * neighbours' code rows stored with the node; an expansion reads those in one
 * sweep and gathers the unvisited neighbours of the remaining slots from the
 * code table.  Results are the same for every ratio; memory is n *
 * ceil(ratio * degree) * row_stride bytes.  ratio in (0, 1]; a call with
 * another ratio replaces the earlier copy (device-wide wait).  Synchronous.
 */
ann_status ann_build_prs_ratio(ann_index *index, float ratio, void *stream);

/*
 * Entry-point stage: per-query initial nodes I for Algorithm 1 (which takes
 * "initial nodes I" as an input).  ann_build_entry_table samples n_pivots base
 * vectors, node floor(i * n / n_pivots) for i = 0..n_pivots-1, and keeps a
 * compact copy of their level-0 codes in the index (synchronous; replaces an
 * earlier table).  ann_entry_scan evaluates the traversal distance tau_l of
 * every pivot for every query and writes the n_entry (<= 4) closest pivots'
 * node ids, in ascending (key, id) order, to out_entry_ids [nq][n_entry]
 * (padded with ANN_PAD_ID if n_pivots < n_entry) - ready to be passed to
 * ann_search_batch as entry_ids.  Errors: ANN_EINVAL (NULL arguments, n_pivots
 * outside [1, n], no table built), ANN_ECAPACITY (n_entry > 4), ANN_ENOMEM.
 */
ann_status ann_build_entry_table(ann_index *index, uint32_t n_pivots, void *stream);
ann_status ann_entry_scan(ann_index *index, const float *q, uint32_t nq, uint32_t n_entry,
                          uint32_t *out_entry_ids, void *stream);

/*
 * Processing order for a batch (a speed knob, for callers that search many
 * queries at once): queries with equal or close keys are placed so that they
 * run at the same time on the same accelerator die and share its L2 cache.
 *   keys       [nq] device: one value per query, equal or close for queries
 *              that will visit the same part of the graph - e.g. the node id
 *              of the closest scanned pivot as written by ann_entry_scan with
 *              n_entry = 1 (then key_range = n).  Keys >= key_range count as
 *              key_range - 1.
 *   out_order  [nq] device: a permutation of 0..nq-1 for
 *              ann_search_params.query_order.
 * One small kernel on the stream; no allocation.  Errors: ANN_EINVAL.
 */
ann_status ann_schedule_queries(const uint32_t *keys, uint32_t nq, uint32_t key_range, uint32_t *out_order,
                                void *stream);

/*
 * Algorithm 1 ("Deterministic Access Greedy Search") for a batch of queries,
 * up to but excluding the final rerank: returns the whole final pool.
 *   q          [nq][d] fp32.
 *   entry_ids  NULL: every query starts from the index entry point; otherwise
 *              [nq][n_entry] initial nodes per query (ANN_PAD_ID and duplicates
 *              are skipped), n_entry <= ANN_MAX_ENTRIES.
 *   out_ids    [nq][ef] pool ids in ascending (key, id) order.
 *   out_keys   [nq][ef] traversal keys (NULL allowed).  L2: ||x^||^2 - 2 q.x^
 *              (the squared distance to the decoded vector minus ||q||^2);
 *              IP: -(q.x^); both with the query folded to int8.
 *   out_idot   [nq][ef] the int32 code/query dot products (NULL allowed; asking
 *              for them costs one more pass over the pool's code rows).
 *   out_counts [nq][4] (NULL allowed): expansions, distance evaluations,
 *              pool size, visited-table rebuilds.
 * Errors: ANN_EINVAL (NULL q/out_ids/params, nq == 0, k == 0, ef < k, unknown
 * mode, layout or visited_kind, visited_slots not a power of two or too small
 * for ef, ANN_VISITED_CACHE together with m_s below the degree),
 * ANN_ECAPACITY (ef > ANN_MAX_EF, n_entry > ANN_MAX_ENTRIES), ANN_ENOMEM when
 * the per-index workspace has to grow for a larger nq (the only allocation on
 * this path; none after ann_reserve_workspace), ANN_EDEVICE.
 */
ann_status ann_search_batch(ann_index *index, const float *q, uint32_t nq, const ann_search_params *params,
                            const uint32_t *entry_ids, uint32_t n_entry, uint32_t *out_ids, float *out_keys,
                            int32_t *out_idot, uint32_t *out_counts, void *stream);

/*
 * ann_search_batch for callers that cannot allocate device memory: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same kernels, same results; the folded queries go into a
 * buffer of ANN_STATIC_SCRATCH_BYTES (8 MiB) that is part of the library's
 * device image (each GPU the library runs on holds it until the process ends)
 * instead of the index's workspace.  The call makes no hipMalloc / hipFree and
 * no allocating library call.
 *   Limit: 256-byte rounded nq * folded_row + 4 * (4 * nq) bytes must fit, where
 *   folded_row is 16 bytes (8-bit codes) or 32 bytes (4-bit codes) per 16-byte
 *   chunk of a code row, for at least the chunks the search kernel's lanes
 *   cover (twice that with ANN_DESC_QUERY_15BIT): 128 bytes for d = 128 at 8
 *   bits (about 58,000 queries), 1,024 bytes for d = 960 at 4 bits (about
 *   8,000).  Beyond it: ANN_ECAPACITY,
 *   nothing launched.
 *   reuse_folded_queries is refused (ANN_EINVAL): the buffer belongs to no index.
 *   Every call on a GPU shares that GPU's buffer and overwrites what the last
 *   call left (each call writes all the bytes it reads, so nothing needs
 *   clearing): calls whose execution may overlap on one GPU - on different
 *   streams, or from different threads - race.  Calls on one stream are safe.
 * Other errors as ann_search_batch.
 */
ann_status ann_search_batch_static(ann_index *index, const float *q, uint32_t nq, const ann_search_params *params,
                                   const uint32_t *entry_ids, uint32_t n_entry, uint32_t *out_ids, float *out_keys,
                                   int32_t *out_idot, uint32_t *out_counts, void *stream);

/*
 * Re-evaluate candidates with code level `level` and sort them by (key, id):
 * the middle stage of a low -> higher -> full precision cascade.
 *   cand_ids [nq][cand_stride], the first n_cand of each row are used
 *   (ANN_PAD_ID skipped); outputs [nq][n_cand].  n_cand <= 4096.
 */
ann_status ann_rescore(ann_index *index, uint32_t level, const float *q, uint32_t nq, const uint32_t *cand_ids,
                       uint32_t n_cand, uint32_t cand_stride, uint32_t *out_ids, float *out_keys,
                       int32_t *out_idot, void *stream);

/*
 * Final line of Algorithm 1 with a fixed-length prefix in place of the
 * paper's selective rerank: exact distance tau_h on the fp32 base vectors for
 * the first n_cand candidates of each row of cand_ids [nq][cand_stride], sorted
 * by (distance, id); the best k go to out_ids / out_dist [nq][k].
 * Distances are accumulated in fp64 and rounded once to fp32.
 * n_cand <= 4096, k <= n_cand.  ANN_EINVAL if the index holds no fp32 vectors.
 */
ann_status ann_rerank(ann_index *index, const float *q, uint32_t nq, const uint32_t *cand_ids, uint32_t n_cand,
                      uint32_t cand_stride, uint32_t k, uint32_t *out_ids, float *out_dist, void *stream);

/*
 * Rerank of a per-query prefix: a stand-in for the paper's selective re-rank
 * (Section 5.3 keeps the exact-distance work to the candidates that can still
 * enter the result; its rule is given only in a cited work).  The rule here:
 * with the candidates in ascending order of their low-precision keys
 * cand_keys [nq][cand_stride] (as ann_search_batch and ann_rescore return
 * them), query i re-evaluates the candidates whose key is not above
 *     key[k-1] + gamma * (key[k-1] - key[0])        (fp32: one subtraction, one fma),
 * at least n_min and at most n_max of them (all n_max when key[k-1] is not
 * finite, i.e. the list is shorter than k): a candidate far behind the k-th
 * in the low-precision order, measured by the spread of the first k keys,
 * is taken not to be among the true k nearest.  Then as ann_rerank.
 *   out_n [nq] (NULL allowed): the number of candidates re-evaluated per query.
 * k <= n_min <= n_max <= cand_stride, n_max <= 4096, gamma >= 0.
 */
ann_status ann_rerank_adaptive(ann_index *index, const float *q, uint32_t nq, const uint32_t *cand_ids,
                               const float *cand_keys, uint32_t n_min, uint32_t n_max, uint32_t cand_stride,
                               float gamma, uint32_t k, uint32_t *out_ids, float *out_dist, uint32_t *out_n,
                               void *stream);

/*
 * Exact k nearest neighbours NN_k of every query by exhaustive search (the
 * ground truth of the paper's recall, Section 6.1): a dense Q.X^T contraction
 * on the matrix cores selects k + margin candidates per query, which are then
 * re-evaluated directly in fp64 and sorted by (distance, id).
 *   x [n][d], q [nq][d] fp32; out_ids/out_dist [nq][k]; k <= 256, d <= 2048,
 *   n < 2^31.  The fastest path needs d to be a multiple of 4, 16-byte aligned
 *   x and q, and k <= 16; any d and k within the limits work.
 * Allocates temporaries and synchronises the stream before returning.
 */
ann_status ann_bruteforce_topk(const float *x, uint64_t n, uint32_t d, const float *q, uint32_t nq, uint32_t k,
                               uint32_t metric, uint32_t *out_ids, float *out_dist, void *stream);

/*
 * The number of expansions per step that mode 1 uses when
 * ann_search_params.expansions_per_step is 0, for a pool of ef entries on a
 * graph of the given degree (the multi-expansion mode is this library's own,
 * not the paper's; Algorithm 1 is mode 0): 4, or 8 for pools of more than
 * 128 entries where the kernels built for eight serve the degree without the
 * run-time switches (degree <= 32, or ef > 256).  Measured: with a larger pool
 * a step's merge costs more and fewer, wider steps win (1M x 128, ef = 256:
 * 0.88 against 0.97 ms per 10,000 queries); with ef <= 128 four evaluate fewer
 * nodes for the same time.  Host-only, no error state.
 */
uint32_t ann_default_expansions_per_step(uint32_t ef, uint32_t degree);

const char *ann_last_error(void);
const char *ann_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ANN_H_ */
