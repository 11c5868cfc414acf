/*
 * gbnn.h -- C ABI of the MI355X (gfx950) library for batched retrieval in the Gripon-Berrou
 * clustered associative memory, after Yao, Gripon, Rabbat, "A Massively Parallel Associative
 * Memory Based on Sparse Neural Networks" (arXiv 1303.7032).
 *
 * Model (Section II-A): C clusters of L binary neurons, n = C*L; neuron (c,l) has flat index
 * i = c*L + l (Section IV-B, 0-based here).  A message is C symbols in [0,L); it activates one
 * neuron per cluster.  W is the n x n binary, symmetric adjacency with no edge inside a cluster.
 *
 * Conventions common to all calls
 *   - Every pointer is a DEVICE pointer owned by the caller (e.g. a torch tensor's data_ptr()).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *     work on that stream and return; they never allocate, free or synchronise, and the library
 *     keeps no state between calls (the one exception, for tests, is gbnn_set_kernel_choice).
 *   - Return value: GBNN_OK (0) or a negative gbnn_status.  All argument checks happen on the
 *     host before anything is enqueued; nothing is launched when an error is returned.
 *   - W layout ("canonical"): uint32_t[n][nw], nw = ceil(n/32), row-major; bit (j % 32) of word
 *     (j / 32) of row i is w_ij, least significant bit first; padding bits of the last word of
 *     a row are zero.  W must be symmetric with all-zero intra-cluster blocks (what gbnn_store
 *     produces); results for any other W are unspecified but memory-safe.
 *   - Activity layout: uint8_t[K][n], probe k contiguous (column k of the paper's matrix V,
 *     Section IV-B "Batch Retrieval"); each byte must be 0 or 1 (any other value gives an
 *     unspecified, memory-safe result).
 *   - Limits: 2 <= C <= GBNN_MAX_C, L >= 1, n <= GBNN_MAX_N, 0 <= gamma <= GBNN_MAX_GAMMA,
 *     max_iters >= 1, 0 <= K <= GBNN_MAX_K, M >= 0.
 */
#ifndef GBNN_H
#define GBNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GBNN_MAX_C 64
#define GBNN_MAX_N 16384
#define GBNN_MAX_GAMMA 32767
#define GBNN_MAX_K 2147483647 /* probes per call */

/* Retrieval rules. */
typedef enum {
    GBNN_SUM_OF_SUM = 0, /* Eq. (3)-(5), Algorithm 1 */
    GBNN_SUM_OF_MAX = 1, /* Eq. (6)-(7) in its bail-out-early form (Section IV-D, Theorem 1) */
    GBNN_HYBRID = 2      /* the joint scheme, Algorithm 2 */
} gbnn_rule;

typedef enum {
    GBNN_OK = 0,
    GBNN_ERR_NULL = -1,      /* a required pointer is NULL */
    GBNN_ERR_SHAPE = -2,     /* C, L, n, K or M outside the limits above */
    GBNN_ERR_RULE = -3,      /* rule is not a gbnn_rule */
    GBNN_ERR_GAMMA = -4,     /* gamma outside [0, GBNN_MAX_GAMMA] */
    GBNN_ERR_ITERS = -5,     /* max_iters < 1 */
    GBNN_ERR_WORKSPACE = -6, /* workspace NULL, misaligned (needs 256 bytes) or too small */
    GBNN_ERR_DEVICE = -7,    /* the HIP runtime refused a launch */
    GBNN_ERR_TOO_LARGE = -8  /* gbnn_retrieve_static: the network exceeds GBNN_STATIC_MAX_N neurons */
} gbnn_status;

/* Words per row of W: ceil(C*L/32).  0 if the shape is outside the limits. */
size_t gbnn_w_row_words(int C, int L);
/* Bytes of W: n * gbnn_w_row_words * 4.  0 if the shape is outside the limits. */
size_t gbnn_w_bytes(int C, int L);
/* Bytes of the device workspace that gbnn_prepare fills and gbnn_retrieve reads for this shape,
 * batch and rule (a multiple of 256, never 0 for a valid shape; about the size of W, of W with its
 * clusters padded to the next power of two of at least 32 neurons where L is not one).  0 if an
 * argument is outside the limits. */
size_t gbnn_workspace_bytes(int C, int L, int64_t K, int rule);

/*
 * Storing (Section II-A): for every message, connect all pairs of its C active neurons, i.e.
 * set w_ab = w_ba = 1 for a = c*L + m_c, b = c'*L + m_c', c != c'.  Bits are OR-ed into W, so
 * W must be zeroed by the caller for an empty network and a later call adds more messages;
 * the result does not depend on message order or repetition.
 *   W      device, uint32_t[n][nw], read-modify-write
 *   msgs   device, int32_t[M][C], 0-based symbols
 *   status device int32_t or NULL; bit 0 is OR-ed in if some message had a symbol outside
 *          [0,L); such a message is skipped entirely.  Zero it before the call.
 * Calls that store into the same W must not overlap in time (order them on one stream): rows of W
 * are updated with plain loads and stores.
 */
int gbnn_store(uint32_t *W, int C, int L, const int32_t *msgs, int64_t M, int32_t *status, void *stream);

/*
 * Derives from W the read-only tables the retrieval kernels use and writes them to `workspace`:
 * a copy of W whose intra-cluster blocks are all ones (so that "OR of the rows of the active
 * neurons of cluster c', or the neuron is itself in c'" -- the bail-out-early test of Section
 * IV-D -- is a plain OR of rows), and one summary row per cluster, the OR of its L rows (what a
 * fully active cluster, i.e. an erased cluster at the start of sum-of-max, contributes), with a
 * flag per cluster telling whether that row is all ones (it then changes nothing and is skipped).
 * Call it after W changes (gbnn_store) and before gbnn_retrieve; the workspace then serves any
 * number of gbnn_retrieve calls on that W, of any rule and batch size up to the K it was sized
 * for.  It depends only on W, C and L.
 *   workspace  device, 256-byte aligned, at least gbnn_workspace_bytes(C, L, K, rule) bytes.
 */
int gbnn_prepare(const uint32_t *W, int C, int L, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Storing a few more messages (Section II-A) into W and into a workspace that gbnn_prepare has
 * filled for W as it was: afterwards W and the workspace are what gbnn_store followed by
 * gbnn_prepare would have produced, without the pass over all of W.  Meant for storing and
 * retrieving in turn, one message or a handful at a time (the one-after-another use that
 * Section VII-C sets against batches); its cost grows with M, one atomic update per bit.
 *   W, msgs, M, status   as for gbnn_store
 *   workspace  device, as for gbnn_prepare; read and written.  Retrievals that read it must not
 *          overlap this call in time.
 */
int gbnn_store_update(uint32_t *W, int C, int L, const int32_t *msgs, int64_t M, int32_t *status, void *workspace,
                      size_t workspace_bytes, void *stream);

/*
 * Retrieval of K probes, each independently, iterated until its activity vector is reproduced
 * by a pass or max_iters passes have been made.
 *   V0     device, uint8_t[K][n]; an erased cluster is all-zero for EVERY rule, the library
 *          applies the rule's own initialisation: sum-of-sum and hybrid leave erased clusters
 *          off (Section III-A, Algorithm 2 line 1), sum-of-max turns them all on (Section III-C).
 *   V_out  device, uint8_t[K][n], the last activity vector computed; may be the same pointer as
 *          V0 (in place), must not overlap it otherwise.
 *   rule   GBNN_SUM_OF_SUM: s_i = gamma*v_i + sum_j w_ji v_j, then per cluster every neuron
 *            reaching the cluster maximum stays on (ties and an all-zero maximum included).
 *          GBNN_SUM_OF_MAX: v_i stays on iff it is on and every other cluster holds an active
 *            neighbour of i (score gamma + C - 1 with gamma = 1; `gamma` is ignored).
 *          GBNN_HYBRID: pass 1 keeps, in the clusters that are all-zero in the probe (e of
 *            them), the neurons whose sum-of-sum score is exactly C - e; later passes apply the
 *            sum-of-max update to those clusters only; `gamma` is ignored.
 *   max_iters  cap on the number of passes (the hybrid's first pass counts).
 *   iters_out  device int32_t[K] or NULL: +p if pass p reproduced its input (the confirming
 *          pass counts; for the hybrid the test is made from pass 2 on), -max_iters if the cap
 *          was reached first.
 *   workspace  the workspace filled by gbnn_prepare for this W; only read here, so calls that
 *          overlap in time may share it.
 */
int gbnn_retrieve(const uint32_t *W, int C, int L, const uint8_t *V0, uint8_t *V_out, int64_t K, int rule,
                  int gamma, int max_iters, int32_t *iters_out, void *workspace, size_t workspace_bytes,
                  void *stream);

/*
 * gbnn_retrieve for callers that cannot allocate device memory and so have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The table that
 * gbnn_prepare derives from W is built, on every call, in a device array that is part of the library
 * itself (about 8.6 MiB on every GPU the library runs on, held until the process ends), and the
 * retrieval then reads it there: gbnn_prepare followed by gbnn_retrieve, enqueued on `stream`, same
 * arguments, same results, and no allocation anywhere.
 *   Limit: n = C*L <= GBNN_STATIC_MAX_N, and, where L is not a power of two of at least 32, also
 *   C*L' <= GBNN_STATIC_MAX_N for the next such number L' (the table is laid out for padded clusters);
 *   else GBNN_ERR_TOO_LARGE (nothing is enqueued).
 *   All calls on one GPU share that one array: calls that overlap in time on one GPU (different
 *   streams or threads) race; order them on one stream.  The array keeps what the last call wrote;
 *   every word a call reads is rewritten by that call first.
 *   Because the table is rebuilt per call (a pass over W: 18 us at C=8, L=256), callers that can
 *   hold a workspace should use gbnn_prepare once and gbnn_retrieve.
 */
#define GBNN_STATIC_MAX_N 8192
int gbnn_retrieve_static(const uint32_t *W, int C, int L, const uint8_t *V0, uint8_t *V_out, int64_t K, int rule,
                         int gamma, int max_iters, int32_t *iters_out, void *stream);

/*
 * The same retrieval with messages at the boundary (Section II-A: a message is C symbols, a probe is
 * a message with some symbols erased): 4*C bytes in per probe instead of n, and the result as packed
 * bits and / or symbols instead of n bytes.  Probe k is the activity vector with neuron
 * c*L + probes[k][c] active for every cluster c whose entry lies in [0, L) and no active neuron in
 * the other clusters (-1, by convention, marks an erased cluster); rule, gamma, max_iters,
 * iters_out, workspace and errors are those of gbnn_retrieve, and so is the final activity vector.
 *   probes       device, int32_t[K][C]
 *   bits_out     device uint32_t[K][nw] or NULL: the final activity vector, neuron i = bit (i % 32)
 *                of word (i / 32), least significant bit first, padding bits zero
 *   symbols_out  device int32_t[K][C] or NULL: per cluster, the index of its active neuron if it
 *                holds exactly one, GBNN_SYM_NONE if none, GBNN_SYM_AMBIGUOUS if several (more than
 *                one clique survived, Section V-B)
 */
#define GBNN_SYM_NONE (-1)
#define GBNN_SYM_AMBIGUOUS (-2)
int gbnn_retrieve_symbols(const uint32_t *W, int C, int L, const int32_t *probes, int64_t K, int rule, int gamma,
                          int max_iters, uint32_t *bits_out, int32_t *symbols_out, int32_t *iters_out,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Sparse form W' of W (Section IV-B, "Sparsification": only the nonzero elements and their
 * coordinates are kept) and sum-of-max retrieval from W' alone.  W' is one caller-owned device
 * buffer, 256-byte aligned: uint32_t offsets[n+1], then, each at the next multiple of 256 bytes, the
 * C cluster summary rows of gbnn_prepare with their flags (256 bytes) and uint16_t cols[] to the end
 * of the buffer; the neighbours of neuron i are cols[offsets[i] .. offsets[i+1]), ascending neuron
 * numbers.  A list is shorter than a packed row below a density of 1/16 (2 bytes per edge against
 * n/8 per row); it is the faster form only for shapes that gbnn_retrieve_path reports as "generic".
 * Shapes: L a multiple of 32.
 *
 * gbnn_sparse_count   *nnz_out (device) = number of nonzero elements of W, i.e. the entries cols
 *                     needs.  Read it back, then size W' with gbnn_sparse_bytes.
 * gbnn_sparse_bytes   bytes of a W' with room for nnz entries; 0 for arguments outside the limits
 *                     (nnz < 2^32).
 * gbnn_sparsify       fills W' from W.  status: device int32_t or NULL; bit 0 is OR-ed in if the
 *                     buffer is too small for all entries -- W' must then not be used for
 *                     retrieval (the call itself stays within the buffer).  Zero it before.
 * gbnn_retrieve_sparse  gbnn_retrieve_symbols with rule GBNN_SUM_OF_MAX (Eq. 6-7) reading W'
 *                     instead of W and a workspace: same probes, outputs, pass counts and results.
 */
size_t gbnn_sparse_bytes(int C, int L, int64_t nnz);
int gbnn_sparse_count(const uint32_t *W, int C, int L, uint64_t *nnz_out, void *stream);
int gbnn_sparsify(const uint32_t *W, int C, int L, void *Wp, size_t Wp_bytes, int32_t *status, void *stream);
int gbnn_retrieve_sparse(const void *Wp, size_t Wp_bytes, int C, int L, const int32_t *probes, int64_t K,
                         int max_iters, uint32_t *bits_out, int32_t *symbols_out, int32_t *iters_out, void *stream);

/* Static description of a status code (never NULL). */
const char *gbnn_strerror(int code);

/* Name of the kernel family gbnn_retrieve would run for this shape and rule
 * ("half1" = two probes per wavefront, one packed word per lane, networks of up to 1024 neurons;
 * "wave1", "wave2", "wave4", "wave8" = one wavefront per probe with 1, 2, 4 or 8 packed words per lane;
 * "generic" = any shape), or NULL for invalid arguments.  gbnn_retrieve_symbols runs the same family.
 * Host only; for tests and reports.
 * The register-resident families hold a cluster in 2^k >= 32 neurons' worth of lanes; a cluster size L that
 * is not such a number is padded to the next one inside the library (W, activity vectors and results keep
 * their layout, results and pass counts are the same; the workspace grows accordingly).  They serve every
 * shape whose padded network has clusters of at most 2048 and at most GBNN_MAX_N neurons in all, with V0
 * and V_out at any alignment; the any-shape kernel, several times slower, serves the rest. */
const char *gbnn_retrieve_path(int C, int L, int rule, const void *V0, const void *V_out);

/*
 * For tests and A/B timing only: which kernel serves the calls that follow, in place of the library's own
 * choice.  Process-wide and not synchronised with calls running on other threads; both start as
 * "the library chooses".  Results are identical whatever is chosen: the kernels differ in speed only.
 *   retrieve_family  GBNN_FAMILY_AUTO; GBNN_FAMILY_GENERIC = the any-shape kernel for every shape;
 *                    GBNN_FAMILY_WAVE = one wavefront per probe also where two probes per wavefront
 *                    would be chosen (shapes no register kernel serves still take the any-shape kernel)
 *   store_kernel     GBNN_STORE_AUTO; GBNN_STORE_ATOMIC = one atomic OR per bit; GBNN_STORE_ROWS = rows
 *                    built in LDS
 * Returns GBNN_ERR_RULE for a value outside these enumerations (nothing is changed then).
 * gbnn_retrieve_path reports the choice in force.
 */
enum { GBNN_FAMILY_AUTO = 0, GBNN_FAMILY_GENERIC = 1, GBNN_FAMILY_WAVE = 2 };
enum { GBNN_STORE_AUTO = 0, GBNN_STORE_ATOMIC = 1, GBNN_STORE_ROWS = 2 };
int gbnn_set_kernel_choice(int retrieve_family, int store_kernel);

/*
 * For measurement only, not part of the method: a plain copy of `bytes` bytes from src to dst (both device
 * pointers, 16-byte aligned; bytes a multiple of 16; the ranges must not overlap), moved the way the retrieval
 * kernels move activity: one wavefront per 2 KiB, 16 bytes per lane and instruction.  streaming != 0 reads and
 * writes with non-temporal hints.  The benchmark times it beside the retrieval kernels, as what the memory
 * system delivers for one read stream and one write stream of a batch's size.  Enqueues on `stream` and
 * returns; GBNN_ERR_NULL for a null pointer with bytes > 0, GBNN_ERR_SHAPE for a size or pointer that is not
 * a multiple of 16.
 */
int gbnn_reference_copy(void *dst, const void *src, size_t bytes, int streaming, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GBNN_H */
