/*
 * pqt.h -- C ABI of the Product Quantization Tree (PQT) query library for AMD MI355X (gfx950).
 *
 * The library answers the nearest-neighbour problem of Eq. 1 of the paper,
 *     N(y) = argmin_{x in X} ||y - x||^2 ,
 * approximately, with the online phase of Sec. 3.2 / 3.3: tree traversal (level-1
 * distances, Eq. 6; level-2 refinement of the w best clusters), bin proposal, vector
 * proposal from the inverted lists of Sec. 4, re-ranking by line quantisation
 * (Eq. 8-9) and a final sort.  Every query-dependent step runs inside
 * pqt_query_batch on the GPU (Sec. 1: all query-dependent work belongs to the online phase).
 *
 * Conventions
 *   - plain C, no exceptions cross this boundary; every function that can fail returns
 *     0 (PQT_OK) or a negative PQT_E* code and leaves a message for pqt_last_error();
 *   - "device" pointers are HIP device addresses on the index's GPU, "host" pointers are
 *     ordinary process memory; the library never takes ownership of caller memory;
 *   - all distances are squared Euclidean distances (Sec. 1: d(.) := ||.||^2);
 *   - symbols: D dimension, P tree parts, k1/k2 level-1/level-2 centroids per part,
 *     M re-rank sub-parts = code bytes per vector ("P_line", Sec. 3.3), H bin slots,
 *     T bin tuples examined per query, C candidate budget per query, w clusters refined
 *     per part, k results per query, R = w*k2.
 */
#ifndef PQT_H
#define PQT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PQT_OK            0
#define PQT_EINVAL       (-1)  /* null pointer, size or parameter out of range               */
#define PQT_EIO          (-2)  /* file missing or unreadable                                 */
#define PQT_EFORMAT      (-3)  /* bad magic/version, truncated file, inconsistent arrays     */
#define PQT_ENOMEM       (-4)  /* host or device allocation failed                           */
#define PQT_EHIP         (-5)  /* a HIP runtime call or kernel launch failed                 */
#define PQT_EUNSUPPORTED (-6)  /* valid request outside the implemented limits               */

/* Limits of the kernels (requests beyond them return PQT_EUNSUPPORTED or PQT_EINVAL). */
#define PQT_MAX_K1      256    /* code table stores centroid numbers in one byte             */
#define PQT_MAX_R      1024    /* w*k2 level-2 entries per part                              */
#define PQT_MAX_T      8192
#define PQT_MAX_C     16384
#define PQT_MAX_K      1024

typedef struct pqt_index pqt_index;   /* opaque; owns all device and host memory of one index */

/*
 * Re-rank code formats (Sec. 3.3, Eq. 7: a vector is the tuple of (lambda, i, j) of its sub-parts).
 *   PQT_CODES_TABLE        one byte per sub-part: the number of an (i, j, lambda) entry in a table of
 *                          256 per sub-part (tbl_i, tbl_j, tbl_lambda); M bytes per vector.
 *   PQT_CODES_PAIR_LAMBDA  the tuple stored directly in "1+1 bytes" per sub-part (Sec. 3.3): byte 2m is
 *                          the number of the centroid pair i < j in lexicographic order
 *                          (i (2 k1 - i - 1) / 2 + j - i - 1; needs k1 (k1 - 1) / 2 <= 256), byte 2m+1 the
 *                          level of lambda = (level - 96) / 16, i.e. -6 .. 9.94 in steps of 1/16;
 *                          2M bytes per vector.  The score is Eq. 9
 *                          evaluated per candidate; the line table is not used and may be NULL.
 */
#define PQT_CODES_TABLE        0
#define PQT_CODES_PAIR_LAMBDA  1

typedef struct pqt_info {
    uint64_t N, H;
    uint32_t D, P, k1, k2, M;
    uint32_t T, C;               /* current budgets (defaults come from the index file)      */
    int32_t  device;
    uint64_t bytes_index;        /* device bytes held by the index arrays                    */
    uint64_t bytes_workspace;    /* device bytes held by the per-batch workspace             */
    uint32_t code_format;        /* PQT_CODES_*                                              */
    uint32_t code_bytes;         /* bytes per vector in the codes array                      */
} pqt_info;

/*
 * pqt_index_load -- read an index file (host path) and place it in the memory of GPU
 * `device`.  The file holds what the offline phase produces (Sec. 3.1, 3.3, 4): the
 * two-level codebooks, the line-code table (i, j, lambda) per code byte value (Eq. 7),
 * the centroid-pair distance table of Sec. 3.3, the pointer array over the H hashed bin
 * slots, the ids sorted by slot, and the codes stored in the same order as the ids.
 * Layout: 256-byte header  "PQTIDX1\0", u32 version=1, D, P, k1, k2, M, u64 N, u64 H,
 * u32 T, u32 C, u32 offset_bits=32, u32 code_format; then, each at the next multiple of 256 bytes:
 * C1 f32[P][k1][D/P], C2 f32[P][k1][k2][D/P], tbl_i u8[M][256], tbl_j u8[M][256],
 * tbl_lambda f32[M][256], cc f32[M][k1][k1], offsets u32[H+1], ids u32[N], codes u8[N][M]
 * (u8[N][2M] for PQT_CODES_PAIR_LAMBDA, whose table sections are present but unused).
 * On success *out is a handle the caller releases with pqt_index_free.
 * Errors: PQT_EINVAL (null), PQT_EIO, PQT_EFORMAT (also: offsets not monotone,
 * offsets[H] != N, table entries >= k1, a pair byte >= k1 (k1 - 1) / 2), PQT_EUNSUPPORTED (P not in
 * {1,2,4}, sizes beyond the limits above, more than 256 centroid pairs for PQT_CODES_PAIR_LAMBDA),
 * PQT_ENOMEM, PQT_EHIP.
 */
int pqt_index_load(const char* path, int device, pqt_index** out);

/*
 * pqt_index_from_arrays -- the same index from arrays already in memory (what the offline
 * phase of Sec. 3.1 / 3.3 / 4 produces, with the shapes listed for the file above).
 * C1, C2, tbl_i, tbl_j, tbl_lambda and cc are always host pointers (they are small and the
 * library derives its own tables from them).  offsets (H+1), ids (N) and codes (N x M) are
 * host pointers when location == PQT_HOST and device pointers on GPU `device` when
 * location == PQT_DEVICE (an index built on the GPU never has to leave it).  Everything is
 * copied: the caller keeps ownership of all arrays and may release them after the call.
 * T and C are the default budgets.  Errors as for pqt_index_load (no PQT_EIO).
 */
#define PQT_HOST   0
#define PQT_DEVICE 1
typedef struct pqt_index_arrays {
    uint64_t N, H;
    uint32_t D, P, k1, k2, M, T, C;
    const float*    C1;          /* [P][k1][D/P]        host */
    const float*    C2;          /* [P][k1][k2][D/P]    host */
    const uint8_t*  tbl_i;       /* [M][256]            host */
    const uint8_t*  tbl_j;       /* [M][256]            host */
    const float*    tbl_lambda;  /* [M][256]            host */
    const float*    cc;          /* [M][k1][k1]         host */
    const uint32_t* offsets;     /* [H+1]               host or device */
    const uint32_t* ids;         /* [N]                 host or device */
    const uint8_t*  codes;       /* [N][M] or [N][2M]   host or device */
    uint32_t        code_format; /* PQT_CODES_TABLE (0) or PQT_CODES_PAIR_LAMBDA; with the latter
                                    tbl_i, tbl_j, tbl_lambda may be NULL */
} pqt_index_arrays;
int pqt_index_from_arrays(const pqt_index_arrays* arrays, int location, int device, pqt_index** out);

/*
 * pqt_train -- everything that is learned from a sample (Sec. 3.1 "Training the codebook", Sec. 3.3
 * "Offline computation"), on GPU `device`:
 *   C1   level-1 product quantiser: per tree part, k1 centroids by `iters` Lloyd iterations (Sec. 2.1)
 *        on the part's slice of the n training vectors.  Start: k1 vectors at evenly spaced places of
 *        the sample; ties in the assignment go to the smaller centroid number; an empty cell is
 *        re-seeded with the vector farthest from its centroid.
 *   C2   level-2 quantisers: inside each level-1 cell, k2 centroids trained the same way on the
 *        sub-vectors assigned to the cell (the sub-vectors themselves, not residuals).  A cell with
 *        at most k2 members keeps them as centroids, the remaining centroids repeat their mean (the
 *        cell's own centroid when it is empty).
 *   cc   ||[c_s]_m - [c_t]_m||^2 for every re-rank sub-part m and pair of level-1 centroids (Sec. 3.3).
 *   tbl_i, tbl_j, tbl_lambda   the 256 line code points of every sub-part (PQT_CODES_TABLE): each of
 *        the first n_table training sub-vectors votes for the line through two level-1 centroids
 *        that it is nearest to (projection error from its own level-1 distances, fp32); lines get
 *        code points in proportion to their votes (largest-remainder rounding), placed at the
 *        (t + 1/2) / count quantiles of the projection parameters seen on the line; entries ordered
 *        by (i, j, lambda).  n_table = 0 (or k1 = 1) leaves the table at zeros and the three pointers
 *        may be NULL ((pair, lambda) codes need no table).
 * vectors: device, n x D row-major fp32 (unchanged).  The six outputs are HOST buffers of the shapes
 * listed for pqt_index_from_arrays, owned by the caller.  Synchronous: returns when they are filled.
 * The same inputs give the same bytes.  Errors: PQT_EINVAL (null, n = 0, n_table > n, inconsistent
 * sizes), PQT_EUNSUPPORTED (sizes beyond the kernel limits), PQT_ENOMEM, PQT_EHIP.
 */
typedef struct pqt_train_params {
    uint32_t D, P, k1, k2, M;
    uint32_t iters;      /* Lloyd iterations per quantiser                       */
    uint64_t n;          /* training vectors                                     */
    uint64_t n_table;    /* the first n_table of them vote for the line table    */
} pqt_train_params;
int pqt_train(const pqt_train_params* params, const float* vectors, int device, float* C1, float* C2,
              uint8_t* tbl_i, uint8_t* tbl_j, float* tbl_lambda, float* cc, void* hip_stream);

/*
 * Streaming index construction on the GPU -- the per-vector part of the offline phase
 * (Sec. 3.1: every database vector is sorted into its bin by the tree; Sec. 3.3 "Offline
 * computation": its line-quantisation code; Sec. 4: ids sorted by bin, pointer array from a
 * histogram and a prefix sum).  The codebooks and the line-code table (pqt_train, or the
 * caller's own) are passed in `params`, whose N is the number
 * of vectors that will be added and whose offsets / ids / codes are ignored.
 *   pqt_builder_create  copies the codebooks to GPU `device`.
 *   pqt_builder_add     takes n more vectors (device, n x D row-major fp32; they get the next
 *                       n ids), sorts them into bins with the query path's own traversal
 *                       kernel and encodes them; asynchronous on hip_stream.  Any number of
 *                       calls; the total must be N.
 *   pqt_builder_finish  orders the ids by (slot, id), builds the pointer array, permutes the
 *                       codes, and returns the finished index (released with
 *                       pqt_index_free); the builder is then empty and only needs
 *                       pqt_builder_free.  Synchronises the device.
 * A code byte is the nearest of the 256 code points of its sub-part, with distances from
 * Eq. 9 on the vector's own level-1 distances (fp32); ties go to the smaller code value.
 * With params->code_format == PQT_CODES_PAIR_LAMBDA a sub-part's code is the nearest of the
 * points (pair, level) stand for: per centroid pair the level nearest to the projection's
 * lambda (clamped to 0..255), then the pair whose point is nearest by Eq. 9 on the same
 * level-1 distances and the pair distance table (ties: smaller pair number; pairs of
 * coinciding centroids never win).
 * Errors: PQT_EINVAL (null, N = 0, more or fewer than N vectors), PQT_EFORMAT /
 * PQT_EUNSUPPORTED as for pqt_index_from_arrays, PQT_ENOMEM, PQT_EHIP.
 */
typedef struct pqt_builder pqt_builder;
int  pqt_builder_create(const pqt_index_arrays* params, int device, pqt_builder** out);
int  pqt_builder_add(pqt_builder* builder, const float* vectors, int64_t n, void* hip_stream);
int  pqt_builder_finish(pqt_builder* builder, pqt_index** out);
void pqt_builder_free(pqt_builder* builder);

/*
 * pqt_index_export -- copy the index arrays out.  dst names caller-owned buffers of the sizes
 * pqt_index_info reports (shapes as for pqt_index_from_arrays; the scalar fields of dst are
 * ignored); a NULL pointer skips that array.  C1 .. cc are host buffers; offsets, ids and
 * codes are host buffers when location == PQT_HOST, device buffers on the index's GPU when
 * location == PQT_DEVICE.  Synchronous.  Errors: PQT_EINVAL, PQT_EHIP.
 */
int pqt_index_export(const pqt_index* index, const pqt_index_arrays* dst, int location);

/*
 * pqt_index_save -- write the index to a file in the format pqt_index_load reads (the
 * device arrays are copied back through host memory).  Errors: PQT_EINVAL, PQT_EIO,
 * PQT_ENOMEM, PQT_EHIP.
 */
int pqt_index_save(const pqt_index* index, const char* path);

/* Releases the index, its device arrays and its workspace.  NULL is allowed. */
void pqt_index_free(pqt_index* index);

/* Fills *out.  PQT_EINVAL on null arguments. */
int pqt_index_info(const pqt_index* index, pqt_info* out);

/*
 * pqt_set_budget -- how far the bin proposal goes (Sec. 3.2 "until a sufficient number
 * of vectors ... is generated"; Table 1: the first 2^12 proposed vectors are used):
 * T_bins rank tuples are examined per query (empty and repeated slots count), and the
 * candidate list is cut after C_candidates vectors.  1 <= T <= PQT_MAX_T,
 * 1 <= C <= PQT_MAX_C, else PQT_EINVAL.
 */
int pqt_set_budget(pqt_index* index, uint32_t T_bins, uint32_t C_candidates);

/*
 * pqt_set_bin_order -- the sequence in which neighbouring bins are proposed (Sec. 3.2 "Bin
 * Proposal Heuristic").
 *   PQT_ORDER_SUMMED_DISTANCE (default)  rank tuples by their summed level-2 distance: the
 *       sequence the paper calls optimal (the priority-queue order of its reference [4]).
 *   PQT_ORDER_STATIC_SLOPES  the paper's fixed anisotropic heuristic: ten pre-computed orders
 *       of the rank pairs, one per slope 1.08^k, k = -5..4, nothing sorted per query.  The paper
 *       prints neither the weighted norm nor how a query picks its slope; here the order for
 *       slope s ranks pairs (v1, v2), counted from 1, by v1^2 + (s v2)^2 (ties by (v1, v2)), and
 *       a query takes slope index #{ j in 1..9 : g2 > 1.08^(j-5.5) g1 } (fp32), where
 *       g_p = L_p[min(w*k2 - 1, 8)] - L_p[0] is the rise of its sorted level-2 list of part p.
 *       Two tree parts and H = (k1*k2)^2 only (PQT_EUNSUPPORTED otherwise).  The tables are
 *       rebuilt inside the next query call whenever w*k2 or T changed.
 * PQT_EINVAL for a null index or an unknown order.
 */
#define PQT_ORDER_SUMMED_DISTANCE 0
#define PQT_ORDER_STATIC_SLOPES   1
int pqt_set_bin_order(pqt_index* index, int order);

/*
 * pqt_query_batch -- the online phase for nq queries.
 *   queries   device, nq x D row-major fp32
 *   k         results per query, 1 <= k <= min(C, PQT_MAX_K)
 *   w         level-1 clusters refined per part, 1 <= w <= k1, w*k2 <= PQT_MAX_R
 *   out_ids   device, nq x k int64: database ids ascending by (distance, id); when fewer
 *             than k candidates exist the tail is -1
 *   out_dists device, nq x k fp32: the Eq. 8-9 approximation of ||y-x||^2 for each id
 *             (i.e. the exact squared distance to the line-quantised vector); tail +inf
 *   hip_stream  a hipStream_t (NULL = the default stream).  The call only enqueues work:
 *             it returns before the results exist and never synchronises the device,
 *             except when the library's workspace has to grow (a larger nq, w * k2 or T than
 *             any call before: it is freed and allocated anew, which waits for the device).
 *             Same inputs give the same bytes.
 * Calls on one index must not overlap (they share the workspace).
 * Errors: PQT_EINVAL (null pointers with nq > 0, nq < 0, k or w out of range),
 * PQT_EUNSUPPORTED (LDS budget exceeded for this D/M/k1/R/T/C), PQT_ENOMEM, PQT_EHIP.
 */
int pqt_query_batch(pqt_index* index, const float* queries, int64_t nq, int k, int w,
                    int64_t* out_ids, float* out_dists, void* hip_stream);

/*
 * pqt_query_batch_noalloc -- pqt_query_batch for callers that cannot allocate device memory: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same results (bit for bit) as pqt_query_batch.  The per-batch workspace (level-1 distances, the
 * sorted level-2 lists, run lists and counters of every query) is not the index's grown-on-demand
 * allocation but a static array of pqt_noalloc_workspace_bytes() = 32 MiB of device memory that
 * every GPU the library runs on holds until the process ends; the call allocates and frees nothing
 * (no hipMalloc, hipFree, event or stream creation) and records no stage times.
 *   - The workspace of one call is nq * (4 M k1 + 8 P w k2 + 8 T + 12) bytes plus rounding of each
 *     of its seven arrays to 256 bytes; a call that needs more than the array holds returns
 *     PQT_EINVAL and does nothing: send fewer queries per call (about 3,400 at M k1 = 128,
 *     P w k2 = 128, T = 1024).
 *   - With PQT_ORDER_STATIC_SLOPES the order tables for the current w * k2 and T must exist already
 *     (any earlier pqt_query_batch with this w builds them), else PQT_EUNSUPPORTED.
 *   - All calls on one GPU share the array, whichever index they use: calls that overlap in time
 *     on one GPU (different streams or threads) race.  Nothing in it has to survive between calls;
 *     what must start at zero is cleared by the first kernel of each call.
 * Other errors as for pqt_query_batch.
 */
int pqt_query_batch_noalloc(pqt_index* index, const float* queries, int64_t nq, int k, int w,
                            int64_t* out_ids, float* out_dists, void* hip_stream);
size_t pqt_noalloc_workspace_bytes(void);

/*
 * Exact re-ranking of a short list -- step (3) of the pipelines named in Sec. 1 of the paper
 * ("re-ranking the vectors on a short-list by their exact distance"), the variant PQT_2 of
 * Table 1.
 *
 * pqt_index_set_vectors attaches the raw database vectors, N x D row-major in id order, as
 * 4-byte floats (elem_bytes = 4) or 1-byte unsigned integers (elem_bytes = 1, for integer-valued
 * data such as SIFT descriptors; 10^9 x 128 bytes fit one GPU).  location == PQT_HOST: the
 * array is copied to the GPU and the library owns the copy.  location == PQT_DEVICE: the
 * array is used in place, NOT copied: the caller keeps it alive and unchanged until the index
 * is freed or other vectors are attached.  vectors == NULL detaches.  Synchronises the
 * device.  Errors: PQT_EINVAL, PQT_EUNSUPPORTED (a row is not a whole number of 16-byte pieces:
 * D not a multiple of 4 for floats, of 16 for bytes), PQT_ENOMEM, PQT_EHIP.
 *
 * pqt_query_batch_exact runs pqt_query_batch with k_short results per query (held in the
 * library's workspace), computes ||y - x||^2 exactly (fp32) for each of them and returns
 * the k best by (distance, id): out_ids / out_dists as for pqt_query_batch, but out_dists
 * are exact squared distances.  1 <= k <= k_short <= min(C, PQT_MAX_K).  Errors as for
 * pqt_query_batch; PQT_EINVAL also when no vectors are attached.
 */
int pqt_index_set_vectors(pqt_index* index, const void* vectors, int elem_bytes, int location);
int pqt_query_batch_exact(pqt_index* index, const float* queries, int64_t nq, int k_short, int k, int w,
                          int64_t* out_ids, float* out_dists, void* hip_stream);

/*
 * pqt_brute_force -- Eq. 1 itself: the k exact nearest database vectors of every query, by
 * brute force over the attached vectors (pqt_index_set_vectors); the paper's "strong baseline"
 * (Table 1) and the ground truth for recall.  Distances are ||q||^2 + ||x||^2 - 2 q.x in fp32
 * (exact for integer-valued data with norms below 2^24); results ascend by (distance, id).
 *   queries device nq x D fp32; out_ids device nq x k int64; out_dists device nq x k fp32;
 *   1 <= k <= min(N, 256).  Asynchronous on hip_stream except for workspace growth.
 * Errors: PQT_EINVAL (no vectors attached, k or nq out of range, null), PQT_ENOMEM, PQT_EHIP.
 */
int pqt_brute_force(pqt_index* index, const float* queries, int64_t nq, int k,
                    int64_t* out_ids, float* out_dists, void* hip_stream);

/*
 * Optional device buffers that receive every intermediate of the path, for checking it
 * stage by stage.  Any pointer may be NULL (that tap is skipped).  Shapes are per batch:
 *   a          nq x M x k1   fp32   level-1 sub-part distances (Eq. 6 per sub-part)
 *   sel        nq x P x w    int32  kept level-1 clusters, closest first
 *   L_d, L_id  nq x P x R    fp32 / uint32  sorted level-2 lists (distance, leaf id i*k2+j)
 *   n_tuples   nq            uint32 rank tuples examined (min(T, R^P))
 *   tuples     nq x T x 4    uint16 examined rank tuples in bin order (unused parts 0)
 *   tuple_keys nq x T        fp32   their summed level-2 distances
 *   n_slots    nq            uint32 proposed (non-empty, first-seen, before the C cut) slots
 *   slots      nq x T        uint64 those slots in visit order
 *   n_cand     nq            uint32 candidates gathered (<= C)
 *   cand_ids   nq x C        int64  candidate ids in visit order
 *   scores     nq x C        fp32   their Eq. 8-9 scores
 *   lut        nq x M x 256  fp32   per-query table of Eq. 9 summands (PQT_CODES_TABLE only: PQT_EINVAL otherwise)
 */
typedef struct pqt_debug_taps {
    float*    a;
    int32_t*  sel;
    float*    L_d;
    uint32_t* L_id;
    uint32_t* n_tuples;
    uint16_t* tuples;
    float*    tuple_keys;
    uint32_t* n_slots;
    uint64_t* slots;
    uint32_t* n_cand;
    int64_t*  cand_ids;
    float*    scores;
    float*    lut;
} pqt_debug_taps;

/* pqt_query_batch plus the taps above (taps may be NULL: then identical to pqt_query_batch). */
int pqt_query_batch_debug(pqt_index* index, const float* queries, int64_t nq, int k, int w,
                          int64_t* out_ids, float* out_dists, void* hip_stream,
                          const pqt_debug_taps* taps);

/*
 * Per-stage device timing.  With profiling enabled every pqt_query_batch records HIP events
 * on its stream around its three kernels: [0] traversal (level-1 + level-2 distances and
 * sorts), [1] bin ranking head pass (all of the bin ranking for four tree parts), [2] gather +
 * re-rank + top-k (with the full bin ranking of the queries the head pass left over), [3] exact
 * re-ranking of the short list (pqt_query_batch_exact only, else 0).
 * pqt_stage_times synchronises on the recorded events, adds up the elapsed milliseconds of
 * all profiled calls since the last pqt_stage_times into ms[4], stores their number in *calls, and
 * resets.  At most 4096 calls are profiled between two reads; later ones run unprofiled, and a
 * call that fails is not counted.  PQT_EINVAL on null arguments.
 */
int pqt_set_profiling(pqt_index* index, int enabled);
int pqt_stage_times(pqt_index* index, float ms[4], int* calls);

/*
 * pqt_measure_peaks -- what GPU `device` delivers, measured: the read bandwidth of a 4 GiB
 * streaming read (GB/s) and the rate of a loop of independent fp32 matrix-core instructions
 * (TFLOP/s).  The benchmark prices the query kernels against these as well as against the
 * published peaks.  Takes about a second; allocates and frees 4 GiB.  Errors: PQT_EINVAL,
 * PQT_ENOMEM, PQT_EHIP.
 */
int pqt_measure_peaks(int device, double* hbm_read_gb_per_s, double* mfma_f32_tflop_per_s);

/* Message of the last failing call on this thread ("" if none).  Static storage. */
const char* pqt_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PQT_H */
