/*
 * libvnm -- V:N:M sparse linear layers on AMD MI355X (gfx950), C ABI.
 *
 * The pattern (paper, abstract and Section 3 "Pruning of V:N:M sparsity"): a weight matrix
 * W [out x in] is cut into V x M blocks (V rows, M consecutive input columns).  Each block keeps
 * the 4 columns of largest column L1 norm of the importance score, and every row keeps the 2
 * largest scores among those 4, so the density is 2/M and M = 4 is plain 2:4.  N is always 2
 * (Section 4.1).  W is treated as zero-extended so that out is a multiple of V and in a multiple
 * of M (Section 3 "Acceleration of V:N:M sparsity"); callers never pad anything themselves.
 * Ties in both selections go to the lower index, which makes the mask unique.
 *
 * Compressed form (Appendix A), all row-major, all caller-allocated device memory:
 *   values  fp16  [out_pad x 2*col_blocks]        A_n : the two kept values of block b of a row at
 *                                                       columns 2b, 2b+1, ascending position
 *   meta    u8    [out_pad x ceil(col_blocks/2)]  A_i2: one nibble p0 | p1 << 2 per (row, block),
 *                                                       p0 < p1 the positions (0..3) of the kept
 *                                                       values among the block's 4 kept columns;
 *                                                       byte j = block 2j (low), 2j+1 (high nibble)
 *   colidx  u8    [row_blocks x col_blocks x 4]   A_i1: in-block indices (0..M-1) of the 4 kept
 *                                                       columns, ascending
 *   packed  opaque, packed_bytes                  the same information re-ordered for the matrix
 *                                                 cores; produced by vnm_prune_compress / vnm_pack,
 *                                                 consumed by vnm_spmm; not a storage format
 *
 * Conventions: every function returns a vnm_status (0 = success) and never throws.  Pointers named
 * in capitals or marked "dev" are device pointers; everything else is host.  The library never
 * allocates or frees device memory and keeps no reference to any buffer after the enqueued work
 * has run.  Device work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 * stream) and is asynchronous to the host.  Inputs are never written; outputs are fully
 * overwritten, including the pad rows of values / meta (value +0.0, positions (0,1)).
 * Argument errors are detected on the host before anything touches the device.
 */
#ifndef VNM_H
#define VNM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VNM_FORMAT_VERSION 1

typedef enum vnm_status {
  VNM_OK = 0,
  VNM_ERR_NULL = 1,        /* a required pointer is NULL */
  VNM_ERR_SHAPE = 2,       /* out <= 0, in <= 0, T < 0, or a leading dimension below the row width */
  VNM_ERR_UNSUPPORTED = 3, /* N != 2, M < 4 or M > 255, V not in {16, 32, 64, 128}, bad enum value */
  VNM_ERR_ALIGN = 4,       /* a pointer violates the stated alignment */
  VNM_ERR_WORKSPACE = 5,   /* workspace smaller than vnm_sizes.workspace_bytes */
  VNM_ERR_HIP = 6          /* a HIP call or kernel launch failed; see vnm_last_hip_error() */
} vnm_status;

/* Sizes of everything the caller allocates for one layer (Section 3 padding; Appendix A triple). */
typedef struct vnm_sizes {
  int64_t out_pad;         /* ceil(out / V) * V */
  int64_t in_pad;          /* ceil(in / M) * M */
  int64_t row_blocks;      /* out_pad / V */
  int64_t col_blocks;      /* in_pad / M */
  int64_t kc;              /* compacted K = 4 * col_blocks */
  int64_t values_elems;    /* out_pad * 2 * col_blocks  fp16 elements */
  int64_t meta_bytes;      /* out_pad * ceil(col_blocks / 2) */
  int64_t colidx_bytes;    /* row_blocks * col_blocks * 4 */
  int64_t packed_bytes;    /* size of the opaque matrix-core copy (0 if this V, M has none) */
  int64_t workspace_bytes; /* scratch of vnm_prune_compress (currently 0); vnm_spmm's depends on the
                              token count, see vnm_spmm_workspace_bytes */
} vnm_sizes;

/* Which kernel vnm_spmm uses. */
typedef enum vnm_spmm_path {
  VNM_PATH_AUTO = 0,       /* sparse matrix-core kernel when `packed` is given and the shape allows, else generic */
  VNM_PATH_GENERIC = 1,    /* scalar kernel on the canonical triple; any V, M, alignment */
  VNM_PATH_SMFMAC = 2      /* 2:4 sparse MFMA kernel on `packed`; fails with UNSUPPORTED if not applicable */
} vnm_spmm_path;

/* Host only.  Fills *s for a layer of `out` x `in` at V:N:M. */
int vnm_query_sizes(int64_t out, int64_t in, int V, int N, int M, vnm_sizes* s);

/*
 * Section 3, steps 1-3 with the ABS score, followed by the conversion of Appendix A.
 *   W        dev, fp16 [out x in], row-major with leading dimension ldw >= in (elements); 2-byte aligned
 *   values, meta, colidx   dev outputs, sizes from vnm_query_sizes
 *   mask     dev u8 [out x in] (dense, leading dimension in) or NULL: the 0-1 mask of Section 3
 *   packed   dev, packed_bytes, 256-byte aligned, or NULL
 * Column norms are accumulated exactly (integer fixed point, or fp64 where every partial sum is
 * representable), so the result does not depend on any summation order.  Non-finite weights are not supported (result unspecified, no fault).
 */
int vnm_prune_compress(const void* W, int64_t out, int64_t in, int64_t ldw, int V, int N, int M,
                       void* values, void* meta, void* colidx, void* mask, void* packed,
                       void* workspace, int64_t workspace_bytes, void* stream);

/*
 * Section 3, step 1 with the RIA criterion (Eq. 1): fp32 scores
 *   S[i, j] = (|W[i,j]| / sum_i' |W[i',j]| + |W[i,j]| / sum_j' |W[i,j']|) * act[j],
 * act[j] = (L2 norm of the activations of input channel j)^a supplied by the caller (dev fp32 [in]).
 * The two sums are exact; each score is five single IEEE fp64 operations (convert, divide, divide,
 * add, multiply) and one rounding to fp32, so the result is reproducible bit for bit.  A term whose
 * sum is zero counts as zero.
 *   S          dev fp32 [out x in], leading dimension lds >= in
 *   workspace  dev, 8-byte aligned, (out + in) * 8 bytes; contents are scratch
 */
int vnm_ria_scores(const void* W, int64_t out, int64_t in, int64_t ldw, const void* act,
                   void* S, int64_t lds, void* workspace, int64_t workspace_bytes, void* stream);

/*
 * vnm_prune_compress with the importance scores handed in (Section 3, steps 2-3 on any score):
 * S, dev fp32 [out x in] (leading dimension lds), finite and non-negative, zero-padded like W.
 * Column L1 norms of the scores are added in fp64 in row order (row 0 of the block first), which
 * fixes the selection where the order of addition would matter; step 3 compares the scores
 * themselves; ties go to the lower index in both steps; the kept values are W's.  Outputs as
 * for vnm_prune_compress (`colidx` 4-byte aligned).  Other scores: result unspecified, no fault.
 */
int vnm_prune_compress_scored(const void* W, const void* S, int64_t out, int64_t in,
                              int64_t ldw, int64_t lds, int V, int N, int M,
                              void* values, void* meta, void* colidx, void* mask, void* packed,
                              void* stream);

/*
 * Merge of the low-rank LoRA matrices into the dense weight (Section 4.3, Eq. 10: W' = (W + B A) (.) M;
 * in the stage with dynamic masks the mask update merges B A into W before scores are computed and
 * the pattern is pruned):  W_merged = fp16(W + scale * B A).
 *   W, W_merged  dev fp16 [out x in], leading dimensions ldw, ldm >= in (W_merged may be W)
 *   B            dev fp32 [out x r], leading dimension ldb >= r;   A  dev fp32 [r x in], lda >= in
 *   scale        the LoRA scaling alpha / r (2 in the paper's runs); r = 0 copies W
 * The paper fixes neither precision nor order; since the merged weights decide a mask, the merge is
 * defined to the bit: fp32, one rounding per operation, no fused multiply-add, k ascending:
 * acc = acc + (B[o,k] * A[k,i]), then (scale * acc) + W[o,i], then one rounding to fp16.
 * A mask refresh is this call followed by vnm_prune_compress, or by vnm_ria_scores and
 * vnm_prune_compress_scored, on W_merged.
 */
int vnm_lora_merge(const void* W, int64_t out, int64_t in, int64_t ldw, const void* B, int64_t ldb,
                   const void* A, int64_t lda, int r, float scale, void* W_merged, int64_t ldm,
                   void* stream);

/* Builds `packed` from an existing canonical triple (e.g. one loaded from storage). */
int vnm_pack(const void* values, const void* meta, const void* colidx,
             int64_t out, int64_t in, int V, int N, int M, void* packed, void* stream);

/*
 * Y = X . W'^T on the compressed weight (Section 3 "Acceleration"; Appendix A describes the kernel's
 * job: fetch the kept weights and the matching input columns so that the layout is that of a 2:4
 * product, then use the sparse matrix cores):
 *   Y[t, o] = sum_b sum_{j<2} values[o, 2b+j] * X[t, b*M + colidx[o / V, b, pos_j(o, b)]],
 * fp16 operands, fp32 accumulation; X counts as 0 at padded columns and is never read there.
 *   X        dev fp16 [T x in], leading dimension ldx >= in
 *   Y        dev [T x out], leading dimension ldy >= out; y_dtype 0 = fp16, 1 = fp32
 *   packed   dev or NULL (NULL forces the generic kernel under VNM_PATH_AUTO)
 *   path     a vnm_spmm_path
 *   workspace  dev, 256-byte aligned, vnm_spmm_workspace_bytes(T, ...) bytes: the matrix-core
 *            kernel first re-lays X there (token tiles x K steps, column-major inside, the order
 *            it streams through LDS; vnm_stage_x_bytes bytes, the required minimum); the rest
 *            (vnm_spmm_scratch_bytes, optional) holds fp32 partial products when, for few tokens,
 *            the K dimension is split over workgroups; contents are scratch, nothing persists
 * The matrix-core kernel needs V in {32, 64, 128}, M <= 16, in % 8 == 0, ldx % 8 == 0 and X 16-byte
 * aligned; otherwise (or when `packed` is NULL) AUTO uses the generic kernel, which needs no
 * workspace.  For T <= 32 the matrix-core path is a single kernel that reads X directly and needs no
 * workspace (if one is given, its scratch part may hold split-K partial products).  For larger T, when the
 * matrix-core kernel applies but the workspace is missing or too small the call fails with VNM_ERR_WORKSPACE
 * instead of silently taking the slow kernel (also where, up to 256 tokens, the few-token kernels end up
 * serving the call and use at most the scratch part).
 * T == 0 is a successful no-op (X and Y may then be NULL).
 */
int vnm_spmm(const void* X, int64_t T, int64_t ldx,
             const void* values, const void* meta, const void* colidx, const void* packed,
             int64_t out, int64_t in, int V, int N, int M,
             void* Y, int64_t ldy, int y_dtype, int path,
             void* workspace, int64_t workspace_bytes, void* stream);

/*
 * vnm_spmm for callers that cannot hand over or allocate a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and errors as
 * vnm_spmm without `workspace`: the re-laid activations and the split-K partial products go to a
 * device array of VNM_NOALLOC_SCRATCH_BYTES that is part of the library image (every GPU the library
 * runs on holds its own copy until the process ends).  The call allocates and frees nothing, on the
 * host side of HIP or the device.  A shape whose staged activations (vnm_stage_x_bytes(T, in, M),
 * rounded up to 256) exceed the array fails with VNM_ERR_WORKSPACE and vnm_last_hip_error() says how
 * much was needed; what the activations leave free serves as split-K scratch (less of it may mean a
 * different split and so a different, equally valid, rounding than vnm_spmm with a full workspace).
 * All calls on one GPU share the one array: calls that overlap in time on the same GPU (different
 * streams or threads) race; calls on one stream are ordered and safe.  Nothing in the array has to
 * start at zero: every byte a product reads is written by the same call first, apart from slack
 * that is fetched and never used.
 */
#define VNM_NOALLOC_SCRATCH_BYTES (32ll << 20)
int vnm_spmm_noalloc(const void* X, int64_t T, int64_t ldx,
                     const void* values, const void* meta, const void* colidx, const void* packed,
                     int64_t out, int64_t in, int V, int N, int M,
                     void* Y, int64_t ldy, int y_dtype, int path, void* stream);

/*
 * vnm_spmm with the steps that Section 4.2 says can be merged into the layer at inference (Eq. 6:
 * Y = P_o^T W_p P_i^T X, W_p = P_o W P_i the channel-permuted weight that was pruned) and the layer's
 * bias:
 *   Y[t, perm_out[o]] = bias[o] + sum_i W'_p[o, i] * X[t, perm_in[i]]
 * where W'_p is the compressed weight handed in.  Each of the three is optional (NULL):
 *   bias      dev fp16 [out], in the row order of the compressed weight (a bias travels with its
 *             row: bias[o] is the layer's bias of output channel perm_out[o]); added in fp32
 *             before the result is rounded
 *   perm_in   dev int32 [in], 16-byte aligned: column i of the compressed weight multiplies input
 *             channel perm_in[i] (P_i[perm_in[i], i] = 1); applied while X is re-laid, X itself is
 *             not modified
 *   perm_out  dev int32 [out], 4-byte aligned: row o of the compressed weight produces output
 *             channel perm_out[o] (P_o[o, perm_out[o]] = 1); applied when Y is stored
 * Both must be permutations of 0..n-1; the device arrays are not checked, but an entry outside the
 * range never faults: such an input channel reads as zero, such an output channel is not stored
 * (if perm_out is not a permutation, the contents of columns of Y that no row maps to are
 * unspecified).
 * With perm_in the matrix-core path needs the workspace for every T (for T <= 32 it holds a permuted
 * copy of X).  vnm_spmm_fused_workspace_bytes (host only) is vnm_spmm_workspace_bytes plus, with
 * perm_in, room for a permuted copy of X; with only vnm_spmm_workspace_bytes the call still works,
 * the permutation then costs more time.  The cheapest permutation is none: leave Y in the weight's
 * row order and fold P_o into the next layer's input permutation (vnm_fold_permutations).
 * Everything else as vnm_spmm.
 */
int vnm_spmm_fused(const void* X, int64_t T, int64_t ldx,
                   const void* values, const void* meta, const void* colidx, const void* packed,
                   int64_t out, int64_t in, int V, int N, int M,
                   const void* bias, const void* perm_in, const void* perm_out,
                   void* Y, int64_t ldy, int y_dtype, int path,
                   void* workspace, int64_t workspace_bytes, void* stream);
int vnm_spmm_fused_workspace_bytes(int64_t T, int64_t out, int64_t in, int V, int N, int M,
                                   int with_perm_in, int64_t* bytes);

/*
 * Host only (host pointers, int32 [n] each).  Merges the output permutation of one layer into the
 * input permutation of the layer that consumes its output (Section 4.2: the permutations can be
 * fused with the preceding layer): if the first layer is run without perm_out, its output Z holds
 * Z[:, o] = Y[:, perm_out_prev[o]], and the next layer must read
 *   folded[i] = inverse(perm_out_prev)[perm_in_next[i]]
 * instead of perm_in_next[i].  VNM_ERR_SHAPE if either input is not a permutation of 0..n-1.
 */
int vnm_fold_permutations(const void* perm_out_prev, const void* perm_in_next, int64_t n, void* folded);

/*
 * The two halves of vnm_spmm's matrix-core path as separate calls, for callers that feed the same
 * activations to several layers (the q/k/v projections or the gate/up projections of a block share
 * their input): re-lay X once, multiply many times.  Same arguments and errors as vnm_spmm;
 * `staged` (vnm_stage_x_bytes(T, in, M) bytes, 256-byte aligned) holds the re-laid activations and
 * depends only on T, in and M, not on the layer's weights; vnm_spmm_staged takes its size too and
 * fails with VNM_ERR_WORKSPACE if it is below vnm_stage_x_bytes(T, in, M): that size includes three
 * images of slack behind the last token tile, which the product kernel's look-ahead copies read (and
 * never use), so a buffer sized for the tiles alone would be read out of bounds.
 * `scratch` (vnm_spmm_scratch_bytes(T, out)
 * bytes, 256-byte aligned, or NULL) is the optional split-K scratch: without it, or with less than
 * asked for, the product is still correct, only slower for small T.  vnm_spmm_staged fails with
 * VNM_ERR_UNSUPPORTED where vnm_spmm would have used the generic kernel.
 */
int vnm_stage_x(const void* X, int64_t T, int64_t ldx, int64_t in, int M,
                void* staged, int64_t staged_bytes, void* stream);
int vnm_spmm_staged(const void* staged, int64_t staged_bytes, int64_t T, const void* packed,
                    int64_t out, int64_t in, int V, int N, int M,
                    void* Y, int64_t ldy, int y_dtype,
                    void* scratch, int64_t scratch_bytes, void* stream);
/* Host only.  Sizes of the two buffers above. */
int vnm_stage_x_bytes(int64_t T, int64_t in, int M, int64_t* bytes);
int vnm_spmm_scratch_bytes(int64_t T, int64_t out, int64_t* bytes);

/*
 * Host only.  Which kernel vnm_spmm (VNM_PATH_AUTO, `packed` given, X aligned as the matrix-core
 * kernels need it, no input permutation) runs for T tokens with a workspace of the given size:
 *   VNM_KERNEL_GENERIC     scalar kernel (no matrix-core copy for this V, M, or in % 8 != 0)
 *   VNM_KERNEL_FEW_TOKENS  no staging pass, X token-major in LDS (one to four tokens: a stream through the vector
 *                          ALUs): T <= 32 always; up to 256 tokens where one workgroup per (row blocks, group of 16
 *                          or 32 tokens, piece of K) fits the compute units at once (with the workspace that
 *                          vnm_spmm_workspace_bytes asks for; fp32 partial products + a reduction kernel if K is split)
 *   VNM_KERNEL_RESIDENT    one kernel without a staging pass: the workgroup's slice of X is turned
 *                          around into LDS by the kernel itself (a K range that fits LDS; or at most
 *                          1024 output channels and at least 8192 tokens, K streaming through LDS)
 *   VNM_KERNEL_STAGED      staging pass + streaming matrix-core kernel (vnm_stage_x + vnm_spmm_staged)
 * For measurement and tests; results never depend on the choice beyond rounding.
 */
typedef enum vnm_kernel_choice {
  VNM_KERNEL_GENERIC = 0, VNM_KERNEL_FEW_TOKENS = 1, VNM_KERNEL_RESIDENT = 2, VNM_KERNEL_STAGED = 3
} vnm_kernel_choice;
int vnm_spmm_kernel_choice(int64_t T, int64_t out, int64_t in, int V, int N, int M,
                           int64_t workspace_bytes, int* choice);

/* Host only.  Bytes of workspace vnm_spmm wants for T tokens of this layer: staged activations
 * (rounded up to 256) + split-K scratch (0 if the matrix-core kernel does not exist for this V, M). */
int vnm_spmm_workspace_bytes(int64_t T, int64_t out, int64_t in, int V, int N, int M, int64_t* bytes);

/* Inverse of the conversion of Appendix A: dense fp16 W' [out x in] (leading dimension ldw),
 * kept values as bit copies, +0.0 everywhere else. */
int vnm_decompress(const void* values, const void* meta, const void* colidx,
                   int64_t out, int64_t in, int V, int N, int M,
                   void* W_out, int64_t ldw, void* stream);

/*
 * V and M selection (Section 4.1, Eq. 4-5 and Appendix B).  Host only.
 * vnm_mask_diversity_log: ln K(V, M) = (ln C(M,4) + V ln C(4,N)) / (V M), the per-weight logarithm
 * of the mask diversity; for one network a larger K means a larger mask diversity whatever the
 * layer shapes.  N must be 2, 4 <= M <= 255.
 * vnm_select_vm: the two-phase sifting.  Candidates i = 0..n-1 are (V[i], M[i]) with measured
 * speedup[i] over the dense model; those with speedup >= threshold qualify; for every V only its
 * smallest qualifying M stays; of the rest the one of largest K is selected (ties: higher speedup,
 * then smaller V, then lower i).  *selected = its index, or -1 if none qualifies.  M = 4 stands for
 * plain 2:4 (K does not depend on V then).
 */
int vnm_mask_diversity_log(int V, int N, int M, double* ln_k);
int vnm_select_vm(const int* V, const int* M, const double* speedup, int n, double threshold,
                  int* selected);

/*
 * Search for the channel permutations (Section 4.2, Eqs. 7-9): alternating optimisation of the input
 * and the output permutation, both starting as the identity, `iterations` times (the paper uses 2),
 * maximising the importance that V:N:M pruning retains on the permuted score matrix (Eq. 7).
 *   S        dev fp32 [out x in], leading dimension lds >= in: importance scores (RIA, Eq. 1, in the
 *            paper), finite and non-negative
 *   scale    > 0: scores are quantised once to integers, rint(S * scale) in fp64 clipped to
 *            [0, 2^32 - 1]; all sums are exact 64-bit integers, so results do not depend on any
 *            order of summation (choose scale so that the largest score lands near 2^30)
 *   perm_out host int32 [out], perm_in host int32 [in] (outputs): row o / column i of the permuted
 *            matrix is row perm_out[o] / column perm_in[i] of S -- the arrays vnm_spmm_fused takes
 *   history  host int64 [1 + 2 * iterations] (output): the objective at the identity, then after
 *            every half-step (input first); never decreasing
 *   workspace dev, 256-byte aligned, vnm_permutation_search_workspace_bytes bytes
 * The paper models each half-step as a linear sum assignment problem without printing the model.
 * The one used: the half-step visits the in-block positions in turn; for position q the channel at
 * position q of every full block is lifted out, gain[b][k] is the retained importance of block k
 * with the channel lifted from block b put into the free position, and the assignment of maximal
 * total gain (vnm_lsa_max) is applied.  Channels of a ragged last block (in % M, out % V) stay in
 * place.  The call is synchronous (it alternates device kernels and the host solver) and uses
 * `stream` for its device work.  V in {16, 32, 64, 128}, 4 <= M <= 32, out / V <= 8192.
 *
 * vnm_permutation_gain: one gain matrix of that search, for inspection and tests: which = 0 input
 * half-step (gain int64 [B x B], B = in / M), 1 output half-step ([R x R], R = out / V), for position
 * `slot`, at the given permutations (host int32 arrays, NULL = identity); gain is a host array.
 * vnm_retained_score: the objective (Eq. 7) at the given permutations.
 */
int vnm_permutation_search_workspace_bytes(int64_t out, int64_t in, int V, int N, int M, int64_t* bytes);
int vnm_permutation_search(const void* S, int64_t out, int64_t in, int64_t lds, int V, int N, int M,
                           double scale, int iterations, void* perm_out, void* perm_in,
                           int64_t* history, void* workspace, int64_t workspace_bytes, void* stream);
int vnm_permutation_gain(const void* S, int64_t out, int64_t in, int64_t lds, int V, int N, int M,
                         double scale, int which, int slot, const void* perm_out, const void* perm_in,
                         void* gain, void* workspace, int64_t workspace_bytes, void* stream);
int vnm_retained_score(const void* S, int64_t out, int64_t in, int64_t lds, int V, int N, int M,
                       double scale, const void* perm_out, const void* perm_in, int64_t* total,
                       void* workspace, int64_t workspace_bytes, void* stream);

/*
 * Host only.  Linear sum assignment (Section 4.2: every half-step of the permutation search is
 * modelled as one and solved exactly; the paper names the Hungarian algorithm): assign[i] = the
 * column given to row i such that sum_i gain[i, assign[i]] is maximal; *total = that sum.  gain:
 * int64 [n x n], row-major, entries in [0, 2^60]; assign: int32 [n].  Exact integer arithmetic.
 * Among equally good assignments which one is returned is unspecified (and differs between the
 * methods).  vnm_lsa_max = vnm_lsa_max_method with VNM_LSA_AUTO: an auction with epsilon scaling,
 * and the Hungarian method (O(n^3)) where the auction gives up (values beyond about 2^60 / n, or a
 * bid budget of 2000 n spent).  VNM_LSA_HUNGARIAN and VNM_LSA_AUCTION force one of them; the
 * auction alone returns VNM_ERR_UNSUPPORTED where it gives up.  VNM_LSA_AUCTION_SCALAR is the
 * auction without its AVX-512 row scan (same bids, same result; for checking one against the other).
 */
enum vnm_lsa_method { VNM_LSA_AUTO = 0, VNM_LSA_HUNGARIAN = 1, VNM_LSA_AUCTION = 2, VNM_LSA_AUCTION_SCALAR = 3 };
int vnm_lsa_max(const void* gain, int n, void* assign, int64_t* total);
int vnm_lsa_max_method(const void* gain, int n, int method, void* assign, int64_t* total);

const char* vnm_status_string(int status);
/* Text of the last HIP error seen by the calling thread ("" if none). */
const char* vnm_last_hip_error(void);
int vnm_format_version(void);
/* Hex SHA-256 of the sources and compiler flags this library was built from; the Python binding
 * compares it with the sources in the tree and rebuilds a stale library before using it. */
const char* vnm_source_hash(void);

#ifdef __cplusplus
}
#endif
#endif /* VNM_H */
