/*
 * attncache.h -- C ABI of the MI355X (gfx950) AttnCache hot path.
 *
 * The library implements, on one GPU, the data-parallel part of AttnCache
 * (arXiv 2510.25979): similarity search over the feature-vector database,
 * reuse of a cached attention map (O = A_cached . V) and the exact causal
 * attention that serves queries without a hit.
 *
 * General rules
 *   - Plain C.  Every pointer argument says whether it is DEVICE memory
 *     (hipMalloc'd, e.g. a torch CUDA tensor's data_ptr()) or HOST memory.
 *   - Every function returns an int32_t status: AC_OK (0) or a negative
 *     AC_ERR_* code.  Nothing throws, aborts or prints.
 *   - The memory space of every pointer of a call is checked before anything
 *     is launched (AC_ERR_MEMSPACE: a host pointer never reaches a kernel and
 *     a device pointer is never dereferenced on the host).  The check is one
 *     driver query per pointer; it is skipped while `stream` is being
 *     captured into a graph, and attncache_set_pointer_checks(0) switches it
 *     off for loops that have validated their buffers once.
 *   - All GPU work is enqueued asynchronously on the caller's stream
 *     (`stream` is a hipStream_t passed as void*; NULL = the default
 *     stream).  A status covers argument validation and launch errors only.
 *   - The library never allocates or frees device memory.  Inputs, outputs,
 *     workspace and staging memory are owned by the caller; a database
 *     handle borrows the pointers it is given and the caller keeps that
 *     memory alive until attncache_destroy_db() and does not modify it
 *     behind the library's back (attncache_insert is the library's own
 *     way of writing it).
 *   - Tensors are dense, row-major, innermost index last, no padding.
 *     Every tensor base pointer must be 16-byte aligned.
 *   - Notation: B queries, N database feature vectors of dimension E,
 *     M map entries, L layers, Hq query heads, Hkv key/value heads
 *     (g = Hq / Hkv, query head h uses value head h / g), sequence length S,
 *     head dimension D.
 */
#ifndef ATTNCACHE_H
#define ATTNCACHE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- status codes ------------------------------------------------------ */
#define AC_OK 0
#define AC_ERR_NULL -1      /* a required pointer is NULL                      */
#define AC_ERR_SHAPE -2     /* a size is non-positive or unsupported           */
#define AC_ERR_DTYPE -3     /* unknown / unsupported element type or metric    */
#define AC_ERR_ALIGN -4     /* pointer not 16-byte aligned                     */
#define AC_ERR_K_RANGE -5   /* k outside 1..min(AC_MAX_K, N)                   */
#define AC_ERR_WORKSPACE -6 /* workspace / staging buffer too small            */
#define AC_ERR_INDEX -7     /* a hit index is outside [-1, M)                  */
#define AC_ERR_HIP -8       /* a HIP call failed, see attncache_last_hip_error */
#define AC_ERR_MEMSPACE -9  /* pointer is not in the memory space it must be   */
#define AC_ERR_NOMEM -10    /* a host-side allocation of the library failed     */

/* ---- element types, metrics ------------------------------------------- */
#define AC_F32 0
#define AC_F16 1  /* IEEE binary16 (feature vectors)                         */
#define AC_BF16 2 /* bfloat16 (maps, Q, K, V, O)                             */

#define AC_IP 0 /* similarity = inner product                               */
#define AC_L2 1 /* score = -||q - e||^2, similarity = 1 - ||q - e||          */

#define AC_LAYOUT_DENSE 0  /* each map is a row-major [S][S] matrix              */
#define AC_LAYOUT_PACKED 1 /* block-packed, see attncache_pack_maps (bf16 only)   */

#define AC_MAX_K 64

/* Size of the built-in search workspace of attncache_search_static. */
#define AC_STATIC_SCRATCH_BYTES (4u << 20)

/* ---- database ---------------------------------------------------------- */

/*
 * Description of the two stores of the paper's "Databases" paragraph
 * (Sec. 3.1): the feature-vector store that is searched and the
 * attention-map store that is fetched from.  Both share one index; when
 * several feature vectors refer to one map entry the optional table map_of
 * gives the entry of each vector.
 *
 * Supported: emb_dtype AC_F16 with emb_dim % 8 == 0 (16-byte rows) and either
 * metric: metric AC_IP with emb_dim % 16 == 0 and emb_dim <= 512 runs on the
 * matrix cores, every other fp16 shape on the vector ALUs; emb_dtype AC_F32
 * with either metric and any emb_dim (vector ALUs).  map_dtype AC_BF16 with seq_len % 32 == 0 and head_dim
 * 64 or 128 (matrix-core path, either layout), or map_dtype AC_F32 with any
 * seq_len and head_dim <= 256 (vector-ALU path, dense layout only).
 * n_q_heads % n_kv_heads == 0.
 */
typedef struct {
  int32_t n_emb;        /* N: feature vectors                                */
  int32_t emb_dim;      /* E                                                  */
  int32_t emb_dtype;    /* AC_F16 | AC_F32                                    */
  int32_t metric;       /* AC_IP | AC_L2                                      */
  int32_t n_entries;    /* M: map entries                                     */
  int32_t n_layers;     /* L                                                  */
  int32_t n_q_heads;    /* Hq                                                 */
  int32_t n_kv_heads;   /* Hkv                                                */
  int32_t head_dim;     /* D                                                  */
  int32_t seq_len;      /* S                                                  */
  int32_t map_dtype;    /* AC_BF16 | AC_F32                                   */
  int32_t causal;       /* 1: every map is exactly 0 above the diagonal and
                           those blocks are never read; 0: dense maps        */
  int32_t maps_on_host; /* 0: maps is DEVICE memory; 1: pinned HOST memory   */
  int32_t map_layout;   /* AC_LAYOUT_DENSE | AC_LAYOUT_PACKED                 */
} attncache_db_desc;

typedef struct attncache_db attncache_db; /* opaque, host-side */

/*
 * Bytes of DEVICE workspace attncache_search needs for up to max_batch
 * queries and top-k.  Written to *out.
 */
int32_t attncache_workspace_bytes(const attncache_db_desc *desc,
                                  int32_t max_batch, int32_t k, size_t *out);

/*
 * Bytes of one map entry (all layers and heads of one database item) in the
 * layout desc->map_layout.  Dense: L*Hq*S*S elements.  Packed causal:
 * L*Hq*(S/32)*(S/32+1)*512 elements (20 KiB instead of 32 KiB per head at
 * S = 128); packed non-causal: the same count as dense.
 */
int32_t attncache_map_entry_bytes(const attncache_db_desc *desc, size_t *out);

/*
 * Storage format conversion of the store step (Fig. 3, step 3): rewrite
 * n_entries dense maps into the packed layout the reuse kernel reads fastest.
 *
 *   dense   DEVICE [n_entries][L][Hq][S][S] bf16.
 *   packed  DEVICE, n_entries * attncache_map_entry_bytes(packed desc) bytes.
 *
 * Packed layout of one [S][S] map: rows are cut into blocks of 16, columns
 * into blocks of 32.  Row block r keeps its first nc(r) column blocks, nc(r) =
 * ceil((r+1)/2) for causal maps (everything above is zero by definition and is
 * dropped), S/32 otherwise.  Blocks are stored row-block-major; inside a block
 * (16 x 32 = 512 elements) element (i, 8q + e), q in 0..3, e in 0..7, sits at
 * offset (16q + i)*8 + e, which is the operand order of the 16x16x32 matrix
 * instruction.  desc->map_layout is ignored here (the result IS packed);
 * desc->map_dtype must be AC_BF16.  Entries can be converted in slices, so
 * the dense form never has to exist as a whole.
 */
int32_t attncache_pack_maps(const attncache_db_desc *desc, const void *dense,
                            int32_t n_entries, void *packed, void *stream);

/*
 * Store step of database building (Fig. 3, step 3): bind finished feature
 * vectors and attention maps into one searchable handle.
 *
 *   emb       DEVICE [N][E] of emb_dtype.
 *   map_of    DEVICE [N] int32 with values in [0, M), or NULL for the
 *             identity (requires N == M): map entry of each feature vector.
 *   maps      M entries of attncache_map_entry_bytes() each, of map_dtype, in
 *             the layout desc->map_layout (dense: [M][L][Hq][S][S]); DEVICE,
 *             or pinned HOST memory (hipHostMalloc) when desc->maps_on_host.
 *             Each row of each map sums to 1; with desc->causal the part
 *             above the diagonal is 0.  One entry is one contiguous block (all
 *             layers of one item lie together, as the paper's layer-adjacent
 *             layout).
 *   staging   DEVICE buffer of staging_bytes, used only when maps_on_host;
 *             must hold at least two entries.  NULL / 0 otherwise.  It is
 *             managed as a cache of whole entries (floor(staging_bytes /
 *             entry bytes) slots, least recently used slot replaced first;
 *             per call the entries that are already cached are served
 *             before the others, ascending entry number inside each class):
 *             an entry that an earlier attncache_apply left there is reused
 *             without a new copy, so spare HBM given here absorbs the popular
 *             entries of a skewed request stream (Sec. 3.1, locality of the
 *             stored maps).  The host maps must not change while the handle
 *             lives, or attncache_cache_reset() must be called.
 *   side_stream  hipStream_t on which host-to-device map copies are issued;
 *             used only when maps_on_host (must differ from the stream
 *             later passed to attncache_apply).
 *   out       receives the handle (host malloc; free with destroy).
 *
 * Validates sizes, types, alignment and the memory space of each pointer
 * (so a host pointer can never reach a kernel).  Copies nothing.
 */
int32_t attncache_build_db(const attncache_db_desc *desc, const void *emb,
                           const int32_t *map_of, const void *maps,
                           void *staging, size_t staging_bytes,
                           void *side_stream, attncache_db **out);

/* Releases the handle (and the events of the host-resident path).  The
 * caller must have synchronised the streams the handle was used on. */
int32_t attncache_destroy_db(attncache_db *db);

/*
 * Algorithm 1, search and threshold steps: exact top-k of the similarity
 * between each query and every database feature vector, then hit / miss
 * routing.
 *
 *   q         DEVICE [B][E] of the database's emb_dtype.
 *   k         1..min(AC_MAX_K, N).
 *   threshold theta: a query is a hit when the similarity of its best match
 *             is >= theta (compared in fp32).
 *   idx       DEVICE [B][k] int32 out: database rows, best first; equal
 *             scores are ordered by ascending row index.
 *   score     DEVICE [B][k] float out: fp32 scores (see AC_IP / AC_L2).
 *   hit       DEVICE [B] int32 out: map entry (map_of[idx[b][0]]) for a hit,
 *             -1 for a miss.
 *   ws        DEVICE workspace of ws_bytes >= attncache_workspace_bytes().
 *
 * B == 0 is a no-op.  Scores are accumulated in fp32; the order of the
 * additions depends on the kernel that serves the shape, so two rows whose
 * exact scores differ by less than about 1e-6 relative may come out in
 * either order (rows with bit-identical feature vectors never do: the lower
 * index wins).  A query with a NaN component has no ordered scores: it is a
 * miss (hit -1), and its idx entries are -1 (score -inf) or name rows whose
 * score is NaN, depending on the kernel; nothing is read out of bounds.
 */
int32_t attncache_search(const attncache_db *db, const void *q, int32_t B,
                         int32_t k, float threshold, int32_t *idx,
                         float *score, int32_t *hit, void *ws, size_t ws_bytes,
                         void *stream);

/*
 * attncache_search for callers that cannot allocate or bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, same kernels and bit-identical results, but
 * the workspace is a fixed array of AC_STATIC_SCRATCH_BYTES (4 MiB) inside
 * the library's code object: every GPU the library runs on holds one copy
 * until the process ends.  The call allocates and frees nothing.
 *
 * Limit: shapes whose attncache_workspace_bytes() exceeds
 * AC_STATIC_SCRATCH_BYTES return AC_ERR_WORKSPACE (k = 1 fits up to about
 * 1,000 queries on a million-row index; large k on a large index does not).
 * All calls on one GPU share the one array: calls that overlap in time on
 * the same GPU (two streams, two threads, two handles) race and give wrong
 * results -- order them.  Nothing in it has to start at zero (every word
 * that is read was written by the same call before).  The array's device
 * address is looked up once per GPU, at attncache_build_db or at the first
 * call with that GPU current; when the first call of a process is to be
 * captured into a graph, build the handle beforehand (that is the norm).
 */
int32_t attncache_search_static(const attncache_db *db, const void *q,
                                int32_t B, int32_t k, float threshold,
                                int32_t *idx, float *score, int32_t *hit,
                                void *stream);

/*
 * Algorithm 2, reuse branch: O[b][l][h] = A[hit[b]][layer_begin+l][h] . V[b][l][h/g]
 * for l in [0, layer_count).  The maps are read in place from the database
 * (no gather copy) when they live in device memory.
 *
 *   hit       [B] int32 entry per query, -1 = miss.  DEVICE memory when the
 *             maps are in device memory; HOST memory when maps_on_host (the
 *             host schedules one copy per distinct entry and the indices
 *             are range-checked, AC_ERR_INDEX).
 *   V         DEVICE [B][layer_count][Hkv][S][D], element type = map_dtype.
 *   O         DEVICE [B][layer_count][Hq][S][D], element type = map_dtype.
 *             Rows of misses (hit[b] == -1) are not written.
 *
 * Device-resident maps: hit values outside [-1, M) are treated as misses by
 * the kernel (never dereferenced).  Host-resident maps: entries not yet in
 * the staging cache are copied on the side stream (one copy per distinct
 * entry, shared by all queries that hit it) and overlapped with the products
 * on `stream`; on return all work is enqueued, nothing is waited for.  Calls
 * on one handle must be issued in order (one stream, or ordered by the
 * caller): a slot remembers only its latest reader.
 * fp32 accumulation; bf16 results are rounded once (nearest even).
 */
int32_t attncache_apply(const attncache_db *db, const int32_t *hit,
                        const void *V, void *O, int32_t B, int32_t layer_begin,
                        int32_t layer_count, void *stream);

/*
 * Algorithm 2, recompute branch with the map of Sec. 4:
 * O = softmax(scale * Q K^T) V per (batch item, head); with causal != 0 keys
 * j > i are excluded.  Flash-style: the S x S map is never written.
 *
 *   Q         DEVICE [B][Hq][S][D]; K, V DEVICE [B][Hkv][S][D]; O DEVICE
 *             [B][Hq][S][D]; all of element type dtype (AC_BF16: S % 32 == 0,
 *             D 64 or 128; AC_F32: any S, D <= 256).  Q and K are taken as
 *             given (position encoding already applied).
 *   row_sel   NULL, or DEVICE [B] int32: items with row_sel[b] >= 0 are
 *             skipped and their O rows not written -- pass the hit array of
 *             attncache_search to compute only the misses.
 *   key_len   NULL, or DEVICE [B] int32: number of real tokens of sentence b
 *             in a batch padded on the right to S (values are clamped to
 *             [1, S]).  Keys j >= key_len[b] are hidden from every row (the
 *             attention mask of a padded batch, needed for non-causal
 *             models; with causal != 0 the rows inside the sentence never see
 *             the padding anyway) and chunks of keys that lie wholly in the
 *             padding are not read.  Rows i >= key_len[b] are padding
 *             themselves; they are computed by the same rule.
 *   scale     0 selects 1/sqrt(D).
 *
 * Softmax statistics and accumulators are fp32.
 */
int32_t attention_exact(const void *Q, const void *K, const void *V, void *O,
                        const int32_t *row_sel, const int32_t *key_len,
                        int32_t B, int32_t Hq,
                        int32_t Hkv, int32_t S, int32_t D, int32_t dtype,
                        int32_t causal, float scale, void *stream);

/*
 * Database building on the device (Fig. 3, steps 2 and 3: the attention maps
 * an input produced are stored under the input's feature vector): the
 * recompute branch for items that are to be remembered.  For every item b
 * with row_sel[b] < 0 (or row_sel == NULL)
 *
 *   O[b][l][h]                            = softmax(scale * Q K^T) V   (as attention_exact)
 *   maps[slot[b]][layer_begin + l][h]     = softmax(scale * Q K^T), rounded
 *                                           once to bf16, in the database's
 *                                           map layout (dense causal maps get
 *                                           their zeros above the diagonal)
 *   emb[slot[b]]                          = feat[b]
 *
 * for l in [0, layer_count), so that a later attncache_search hit on the slot
 * makes attncache_apply reproduce O from the stored map.  O is formed from
 * the ROUNDED map (what the reuse branch will read), fp32 accumulation.
 *
 *   db        map_dtype AC_BF16, maps in DEVICE memory (AC_ERR_DTYPE /
 *             AC_ERR_MEMSPACE otherwise).  This is the one entry point that
 *             WRITES the memory the handle borrows (feature rows and map
 *             entries of the named slots); the caller orders it against
 *             searches and reuses of the same slots (same stream, or events).
 *   feat      DEVICE [B][E] of emb_dtype, or NULL to store maps only (a
 *             layer-by-layer caller passes it once).  Requires map_of == NULL
 *             and N == M (one index for both stores) and E * sizeof(element)
 *             a multiple of 16.
 *   slot      DEVICE [B] int32: entry to overwrite, values outside [0, M)
 *             (e.g. -1) store nothing for that item.  NULL: nothing is stored
 *             at all.  Slots of one call must be distinct (equal slots race).
 *   row_sel   NULL or DEVICE [B] int32: items with row_sel[b] >= 0 are skipped
 *             entirely (pass the hit array to handle only the misses).
 *   key_len   NULL or DEVICE [B] int32: real tokens of sentence b in a batch
 *             padded on the right to S, as for attention_exact (clamped to
 *             [1, S]); keys in the padding get weight zero, and those zeros
 *             are what the stored map holds in their columns.
 *   Q         DEVICE [B][layer_count][Hq][S][D] bf16; K, V DEVICE
 *             [B][layer_count][Hkv][S][D]; O DEVICE like Q.
 *   scale     0 selects 1/sqrt(D).
 *
 * Two passes over the keys (row statistics first, then the normalised
 * weights), so it costs about twice the first product of attention_exact.
 */
int32_t attncache_insert(attncache_db *db, const void *feat,
                         const int32_t *slot, const int32_t *row_sel,
                         const int32_t *key_len, const void *Q, const void *K,
                         const void *V, void *O,
                         int32_t B, int32_t layer_begin, int32_t layer_count,
                         float scale, void *stream);

/*
 * Counters of the entry cache of a host-resident database since build /
 * reset: lookups = distinct entries requested, summed over attncache_apply
 * calls; copies = host-to-device entry copies issued.  HOST pointers.
 */
int32_t attncache_cache_stats(const attncache_db *db, uint64_t *lookups,
                              uint64_t *copies);

/* Forget every cached entry (after the host maps were modified) and zero the
 * counters.  The caller must have synchronised the streams the handle was
 * used on. */
int32_t attncache_cache_reset(attncache_db *db);

/*
 * Feature projector (Algorithm 1: f = feature_projector(h); Sec. 3.1
 * "Feature Projector": two MLP layers that map the input embedding to a
 * feature vector of lower dimension).  The step in front of
 * attncache_search: its output is a query block, or, for database building,
 * the `feat` argument of attncache_insert.  The paper fixes the two layers;
 * the pooling over tokens, the activation and the normalisation are this
 * library's reading:
 *
 *   x[b]    = mean of h[b][t] over the sentence's tokens t < seq_len[b]
 *   u[b]    = max(0, W1 x[b] + b1)
 *   f[b]    = W2 u[b] + b2,   divided by its Euclidean norm when `normalize`
 *             (a zero vector stays zero)
 *
 * All arithmetic is binary32 (fp32 matrix cores for the two layers).
 *
 *   h          DEVICE [B][S][model_dim], h_dtype AC_BF16 or AC_F32.
 *   seq_len    NULL (every sentence has S tokens) or DEVICE [B] int32; values
 *              are clamped to [1, S].  Tokens at and after seq_len[b] are not
 *              read.
 *   W1, b1     DEVICE fp32 [hidden_dim][model_dim] and [hidden_dim]
 *              (row j holds the weights of hidden unit j); b1 may be NULL.
 *   W2, b2     DEVICE fp32 [emb_dim][hidden_dim] and [emb_dim]; b2 may be NULL.
 *   feat       DEVICE [B][emb_dim], feat_dtype AC_F16 or AC_F32 (rounded to
 *              nearest even once, after normalisation).
 *   model_dim, hidden_dim, emb_dim   multiples of 8; emb_dim <= 2048;
 *              B <= 65535 (AC_ERR_SHAPE otherwise).  B == 0 is a no-op.
 *   workspace  DEVICE, at least attncache_project_workspace_bytes(...) bytes
 *              (0 is returned for non-positive sizes), 16-byte aligned;
 *              contents are scratch.  AC_ERR_WORKSPACE if too small.
 *
 * Four launches on `stream`; deterministic (partial sums are added in a fixed
 * order).  Weights and inputs are only read.
 */
size_t attncache_project_workspace_bytes(int32_t B, int32_t model_dim,
                                         int32_t hidden_dim, int32_t emb_dim);
int32_t attncache_project(const void *h, const int32_t *seq_len,
                          const float *W1, const float *b1, const float *W2,
                          const float *b2, void *feat, int32_t B, int32_t S,
                          int32_t model_dim, int32_t hidden_dim,
                          int32_t emb_dim, int32_t h_dtype, int32_t feat_dtype,
                          int32_t normalize, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * Switches the per-call memory-space checks of pointers on (non-zero, the
 * default) or off for the whole process; returns the previous setting.
 * attncache_build_db always checks.
 */
int32_t attncache_set_pointer_checks(int32_t on);

/* Short constant description of a status code. */
const char *attncache_status_string(int32_t status);

/* hipError_t (as int) of the last failed HIP call on this thread, 0 if none. */
int32_t attncache_last_hip_error(void);

/* Library version, major * 1000 + minor. */
int32_t attncache_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ATTNCACHE_H */
