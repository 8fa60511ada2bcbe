/*
 * fsd.h -- C ABI of the MI355X (gfx950) candidate-verification library for
 * Fuzzy Speculative Decoding (FSD).
 *
 * One call verifies, for a batch of sequences, every candidate position a
 * draft model proposed: it turns the target-model and draft-model logits of
 * each position into next-token distributions, measures the divergence
 * between them, accepts the position when the divergence is within the
 * threshold T, finds the accepted prefix (or accepted tree path) and draws the
 * one extra token from the target distribution.
 *
 * Conventions shared by all entry points
 *   - Every tensor pointer is a DEVICE pointer owned by the caller; the
 *     library never allocates, frees or keeps it.  Tensors are dense and
 *     row-major.  Logits are binary32 (FSD_F32) or bfloat16 (FSD_BF16).
 *     Rows that start on 16-byte boundaries (V * element size a multiple of
 *     16 and aligned base pointers) take the 128-bit load path; anything else
 *     is still correct through an element-wise path.
 *   - -inf logits are legal (masked vocabulary entries).  A NaN or +inf logit,
 *     or a row that is -inf everywhere, in a row the method reads is reported
 *     per sequence in row_status (FSD_ROW_NONFINITE): that sequence gets
 *     accept_len / path_len 0, all its output tokens -1 and NaN divergences
 *     for the affected positions.
 *   - Calls are asynchronous on `hip_stream` (a hipStream_t, NULL = the null
 *     stream), do no host synchronisation and no host<->device copy.
 *   - `workspace` is device memory of at least fsd_workspace_bytes(...) bytes,
 *     256-byte aligned, private to the call while it runs; its contents need
 *     no initialisation and mean nothing afterwards.
 *   - The return value is an fsd_status.  Argument errors are found before
 *     anything is launched and leave all outputs untouched.
 *   - The vocabulary-reduction kernel is persistent: the wavefronts that share a
 *     row pair wait for each other's partial results, so its grid is sized to
 *     what an otherwise idle device holds at once.  If other work occupies the
 *     GPU while a call runs (another stream, another process), some of its
 *     workgroups may start late; every wait is bounded (see
 *     fsd_debug_set_spin_limit), and a wait that expires ends the call with
 *     FSD_ROW_INTERNAL in row_status for every sequence (lengths 0, tokens -1)
 *     instead of hanging.  Run verify calls on a GPU that is theirs while they
 *     run, and treat FSD_ROW_INTERNAL as "call again".
 *   - Random numbers: Philox4x32-10 keyed by `seed`; `offset` selects the
 *     decode step (counter words 2,3), the sequence index is counter word 1 and
 *     the vocabulary (or position) index picks counter word 0 and the lane.
 *     Equal (seed, offset, inputs) give equal outputs on every launch.
 */
#ifndef FSD_H_
#define FSD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FSD_OK = 0,
    FSD_ERR_NULL = -1,      /* a required pointer is NULL */
    FSD_ERR_SHAPE = -2,     /* B, K, N, V, max_depth out of range, or T is NaN */
    FSD_ERR_DTYPE = -3,     /* dtype is not an fsd_dtype */
    FSD_ERR_DIV = -4,       /* div is not an fsd_div */
    FSD_ERR_WORKSPACE = -5, /* workspace NULL, misaligned or too small */
    FSD_ERR_MODE = -6,      /* mode is not an fsd_mode */
    FSD_ERR_LAUNCH = -7,    /* the HIP runtime refused a launch */
    FSD_ERR_TOO_LARGE = -8  /* fsd_verify_chain_static: sizes beyond its fixed scratch buffer */
} fsd_status;

typedef enum { FSD_F32 = 0, FSD_BF16 = 1 } fsd_dtype;

/* Divergence between the target distribution p and the draft distribution q
 * (paper App. C): KL is KL(p || q) (C.1), JS the Jensen-Shannon divergence
 * with the even mixture (C.2), TV the total-variation distance (C.3).
 * Natural logarithm. */
typedef enum { FSD_DIV_KL = 0, FSD_DIV_JS = 1, FSD_DIV_TV = 2 } fsd_div;

/* How the extra token is drawn from the target row (paper Sec. 4, "whatever
 * sampling method the user sets", and Sec. 6.3): an exact categorical draw
 * from softmax(logits) by Gumbel-max, or the argmax (lowest index on ties). */
typedef enum { FSD_SAMPLE = 0, FSD_GREEDY = 1 } fsd_mode;

/* bits of row_status[b] */
enum {
    FSD_ROW_NONFINITE = 1,  /* NaN / +inf / all -inf row among the rows read */
    FSD_ROW_BAD_PARENT = 2, /* tree: parent[j] outside [-1, j) */
    FSD_ROW_TOO_DEEP = 4,   /* tree: a node deeper than max_depth */
    FSD_ROW_BAD_TOKEN = 8,  /* strict SD: candidate token id outside [0, V) */
    FSD_ROW_INTERNAL = 16   /* a bounded device-side wait expired (never expected) */
};

/* Limits: 1 <= V <= fsd_max_vocab(dtype) (524288 for both dtypes); 1 <= K, N,
 * max_depth <= 2048; 1 <= B <= 65535; B*K (B*N) < 2^24. */
int64_t fsd_max_vocab(int dtype);

/* Bytes of workspace a call with these sizes needs (rows_per_seq = K or N).
 * Returns 0 for arguments no call would accept. */
size_t fsd_workspace_bytes(int B, int rows_per_seq, int V, int dtype);

const char* fsd_status_string(int status);

/*
 * FSD verification of linear candidate sequences (paper Sec. 4, eq. 4).
 *
 *   target_logits [B, K+1, V]  row i < K: target model's logits for position i;
 *                              row K: the position after the last candidate
 *   draft_logits  [B, K, V]    draft model's logits for position i
 *   cand_tokens   [B, K]       the K candidate token ids (copied to the output;
 *                              the FSD decision does not depend on them)
 *   div, T                     accept position i iff div(p_i, q_i) <= T
 *                              (T may be +-inf; NaN is rejected)
 *   accept_len    [B]   out    n_b = number of leading accepted positions
 *   out_tokens    [B, K+1] out cand[b, :n_b], then the token drawn from
 *                              softmax(target[b, n_b]), then -1 padding
 *   divergences   [B, K] out   optional (NULL to skip), the chosen divergence.
 *                              p and q are evaluated in binary32: the value is
 *                              within 1e-5 (binary32 logits) or 2e-3 (bfloat16)
 *                              relative of the exact one from 2e-2 (binary32)
 *                              or 1e-4 (bfloat16) upwards; below that (nearly
 *                              equal rows) its ABSOLUTE error stays under
 *                              2.5e-7, measured on rows that differ by noise of
 *                              0.001 to 0.3, and bit-identical rows give 0
 *   row_status    [B]   out    optional (NULL to skip), see FSD_ROW_*
 *
 * A call only enqueues kernels on hip_stream (what it needs clear in the
 * workspace is cleared by its kernels, never by a memset), so it may be
 * recorded into a HIP graph; seed and offset are then part of the recording.
 */
int fsd_verify_chain(const void* target_logits, const void* draft_logits, const int32_t* cand_tokens,
                     int B, int K, int V, int dtype, int div, float T, int mode, uint64_t seed,
                     uint64_t offset, int32_t* accept_len, int32_t* out_tokens, float* divergences,
                     int32_t* row_status, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * fsd_verify_chain for callers that cannot allocate device memory or pass a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same inputs, outputs, kernels and results as
 * fsd_verify_chain; the workspace is a buffer of FSD_STATIC_SCRATCH_BYTES bytes
 * that is part of the loaded library (one copy per GPU, held until the process
 * ends).  The call allocates and frees nothing.
 *
 *   - Sizes whose fsd_workspace_bytes(B, K, V, dtype) exceeds
 *     FSD_STATIC_SCRATCH_BYTES are refused with FSD_ERR_TOO_LARGE before
 *     anything is launched (B=64, K=8, V=128256 bfloat16 needs 2.1 MiB).
 *   - Every call on a GPU uses that GPU's one buffer, which keeps the last
 *     call's contents; the call clears what it needs cleared itself.  Calls that
 *     overlap in time on one GPU (different streams, or threads) race on it:
 *     keep them on one stream or serialise them.
 */
#define FSD_STATIC_SCRATCH_BYTES (4u << 20)
int fsd_verify_chain_static(const void* target_logits, const void* draft_logits, const int32_t* cand_tokens,
                            int B, int K, int V, int dtype, int div, float T, int mode, uint64_t seed,
                            uint64_t offset, int32_t* accept_len, int32_t* out_tokens, float* divergences,
                            int32_t* row_status, void* hip_stream);

/*
 * FSD verification of a token tree (paper Sec. 6.4: FSD on top of a
 * tree-drafting method; the rule below is this library's statement of it).
 *
 *   target_logits [B, N+1, V]  row 0: target logits at the root context;
 *                              row j+1: at the context that ends with node j
 *   draft_logits  [B, N, V]    row j: the draft logits node j was proposed from
 *   node_tokens   [B, N]       token id of node j
 *   parent        [B, N]       parent node of j, -1 for children of the root;
 *                              parent[j] < j (checked on the device)
 *   max_depth                  longest path the outputs can hold
 *
 * Node j is accepted iff div(softmax(target[parent[j]+1]), softmax(draft[j])) <= T
 * and its parent is accepted.  The deepest accepted node wins (lowest index on
 * ties); the extra token is drawn from the target row of the winner's context
 * (row 0 when no node is accepted).
 *
 *   path_len   [B]              out  depth of the winner (0 = none)
 *   path_nodes [B, max_depth]   out  node indices root-to-winner, -1 padded
 *   out_tokens [B, max_depth+1] out  tokens of the path, the drawn token, -1 padding
 *   divergences [B, N] out optional; row_status [B] out optional
 */
int fsd_verify_tree(const void* target_logits, const void* draft_logits, const int32_t* node_tokens,
                    const int32_t* parent, int B, int N, int max_depth, int V, int dtype, int div,
                    float T, int mode, uint64_t seed, uint64_t offset, int32_t* path_len,
                    int32_t* path_nodes, int32_t* out_tokens, float* divergences, int32_t* row_status,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Strict speculative decoding on the same tensors (paper Sec. 3, eq. 1-3), the
 * baseline FSD generalises: position i is accepted iff min(1, p_i(x_i)/q_i(x_i)) > y_i
 * with y_i uniform in (0,1) from the Philox stream; at the first rejection the
 * token is drawn from the normalised positive part of p - q, and from the row
 * after the last candidate when everything is accepted.
 *
 *   log_ratio [B, K] out  optional, ln p_i(x_i) - ln q_i(x_i)
 */
int sd_verify_chain(const void* target_logits, const void* draft_logits, const int32_t* cand_tokens,
                    int B, int K, int V, int dtype, int mode, uint64_t seed, uint64_t offset,
                    int32_t* accept_len, int32_t* out_tokens, float* log_ratio, int32_t* row_status,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Strict speculative decoding over a token tree: the tree analogue of
 * sd_verify_chain, for the tree-structured proposals of the methods the paper's
 * Sec. 2 cites (item 1) and Sec. 6.4 builds on.  The paper gives no procedure
 * of its own; this is the multi-round rejection rule of that family on the
 * tensors of fsd_verify_tree.  At the current context, with target
 * distribution p, the children are tried in index order: child j is accepted
 * iff min(1, p(x_j)/q_j(x_j)) > y_j (Sec. 3, eq. 1-2; y_j the uniform number
 * of index j) and the walk moves to the context after node j; after a
 * rejection p becomes the normalised positive part of p - q_j (Sec. 3, eq. 3)
 * before the next child is tried.  When no child is accepted the token is
 * drawn from the p in force: the target row itself at a node without
 * children, otherwise the residual of the last rejection.  Every emitted
 * token then follows the target distribution of its context.  With one child
 * per node the outputs are sd_verify_chain's.
 *
 *   inputs and path_len / path_nodes / out_tokens / row_status as in fsd_verify_tree
 *   log_ratio [B, N] out  optional: ln p(x_j) - ln q_j(x_j) with the p in
 *                         force when node j was tried, NaN for nodes never tried
 */
int sd_verify_tree(const void* target_logits, const void* draft_logits, const int32_t* node_tokens,
                   const int32_t* parent, int B, int N, int max_depth, int V, int dtype, int mode,
                   uint64_t seed, uint64_t offset, int32_t* path_len, int32_t* path_nodes,
                   int32_t* out_tokens, float* log_ratio, int32_t* row_status, void* workspace,
                   size_t workspace_bytes, void* hip_stream);

/*
 * fsd_verify_chain with the usual sampling-method warpers applied where the
 * token is drawn (paper Sec. 4: "whatever sampling method the user sets"), in
 * this order, on the target row the token comes from:
 *   temperature  s_v = z_v * binary32(1 / temperature), 1e-3 <= temperature <= 1e3;
 *   top_k        keep the entries with s_v >= the top_k-th largest s (ties at it
 *                are all kept); 0 or >= V switches it off;
 *   top_p        with q = softmax of the kept s, keep s_v >= t, t the largest
 *                value with sum_{s_v >= t} q_v >= top_p (ties kept); 1 = off;
 * then the Gumbel-max draw of fsd_verify_chain over the kept entries, on
 * s_v + G_v with the same random stream.  FSD_GREEDY ignores the warpers (the
 * argmax is always kept).  Acceptance does not depend on them.  With
 * temperature 1, top_k 0 and top_p 1 the call is fsd_verify_chain.
 */
int fsd_verify_chain_warped(const void* target_logits, const void* draft_logits, const int32_t* cand_tokens,
                            int B, int K, int V, int dtype, int div, float T, int mode, uint64_t seed,
                            uint64_t offset, float temperature, int top_k, float top_p, int32_t* accept_len,
                            int32_t* out_tokens, float* divergences, int32_t* row_status, void* workspace,
                            size_t workspace_bytes, void* hip_stream);

/*
 * fsd_verify_tree with the same warpers, applied to the target row after the
 * last node of the accepted path.  Arguments as in fsd_verify_tree and
 * fsd_verify_chain_warped.
 */
int fsd_verify_tree_warped(const void* target_logits, const void* draft_logits, const int32_t* node_tokens,
                           const int32_t* parent, int B, int N, int max_depth, int V, int dtype, int div,
                           float T, int mode, uint64_t seed, uint64_t offset, float temperature, int top_k,
                           float top_p, int32_t* path_len, int32_t* path_nodes, int32_t* out_tokens,
                           float* divergences, int32_t* row_status, void* workspace, size_t workspace_bytes,
                           void* hip_stream);

/*
 * Reducible FSD (paper Sec. 4.3, "Reducing FSD to standard SD"): position i is
 * accepted iff div(p_i, q_i) <= T (the rule of fsd_verify_chain) OR the strict
 * SD test of sd_verify_chain accepts the candidate token, with the same uniform
 * numbers; at the first rejection the token is drawn from the normalised
 * positive part of p - q, otherwise from the row after the last candidate.
 * With T <= 0 and no bit-identical rows the outputs equal sd_verify_chain's.
 * Tensors and outputs as in fsd_verify_chain, plus
 *
 *   log_ratio [B, K] out  optional, ln p_i(x_i) - ln q_i(x_i)
 */
int rfsd_verify_chain(const void* target_logits, const void* draft_logits, const int32_t* cand_tokens,
                      int B, int K, int V, int dtype, int div, float T, int mode, uint64_t seed,
                      uint64_t offset, int32_t* accept_len, int32_t* out_tokens, float* divergences,
                      float* log_ratio, int32_t* row_status, void* workspace, size_t workspace_bytes,
                      void* hip_stream);

/*
 * Threshold tuning on a dev set (paper Sec. 6.2 "Selecting T", paragraph "Tuning T on small dev set";
 * App. A: the threshold that accepts about the same share of candidate tokens
 * as strict SD).  From the divergences of a batch of candidate sequences (the
 * `divergences` output of fsd_verify_chain, any T) it finds the smallest
 * threshold, among the values that occur, at which the chain rule accepts at
 * least `target_fraction` of all B*K candidate positions; +inf if no threshold
 * does (NaN divergences are never accepted).  Exact: the result is one of the
 * input values.
 *
 *   divergences  [B, K] device, binary32, >= 0 or NaN
 *   target_fraction      0 < f <= 1 (e.g. sum(accept_len of strict SD) / (B*K))
 *   T_out        [1] device out   the threshold
 *   fraction_out [1] device out   optional, the share accepted at T_out
 *   workspace    device, 256-byte aligned, fsd_calibrate_workspace_bytes(B, K)
 *
 * Asynchronous on hip_stream like the verify calls; limits as there.
 */
size_t fsd_calibrate_workspace_bytes(int B, int K);
int fsd_calibrate_threshold(const float* divergences, int B, int K, float target_fraction, float* T_out,
                            float* fraction_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---------------------------------------------------------------------------
 * Everything below is for tests, tuning and benchmarks, not for serving code.
 * These calls set or read PROCESS-WIDE state inside the library (the only such
 * state it has; the verify calls themselves keep none between calls, apart from
 * per-device constants looked up once).  They are not thread-safe: use them from
 * one thread while no verify call is in flight on another.
 * ------------------------------------------------------------------------- */

/*
 * Timing of the vocabulary-reduction kernel, for benchmarks.  After
 * fsd_profile_enable(1) every verify call launches that kernel with a pair of
 * events that take the start and the end of its dispatch on the call's stream
 * (what a kernel trace shows; up to 4096 pairs are kept; later calls are
 * not recorded).  fsd_profile_collect waits for the recorded events, returns
 * the number of pairs and their mean / minimum duration in milliseconds, and
 * forgets them.  Not thread-safe; meant for a single benchmarking thread.
 */
int fsd_profile_enable(int on);
int fsd_profile_collect(float* mean_ms, float* min_ms);

/* Test hook: number of polls a wavefront spends waiting for the words of the
 * other wavefronts that share its row pair before it gives up and the call
 * flags FSD_ROW_INTERNAL (default 1<<22).  Returns the previous value. */
unsigned fsd_debug_set_spin_limit(unsigned polls);

/* Test hooks of the bfloat16 Jensen-Shannon reduction.  It evaluates App. C.2 in
 * entropy form (one logarithm per entry), whose absolute error (about 1e-7
 * for small results) does not shrink with the result; results below a floor (default 1e-3 nats)
 * are evaluated again in the pointwise form, whose error does.
 * fsd_debug_set_js_floor sets that floor (0: never again; +inf: always) and
 * returns the previous one; fsd_debug_set_exact_js(1) makes every bfloat16 JS
 * call use the pointwise form only and returns the previous setting. */
float fsd_debug_set_js_floor(float floor_nats);
int fsd_debug_set_exact_js(int on);

/* Test hook: the verify calls launch no kernel of their own to clear the
 * workspace's exchange words: the reduction kernel's wavefronts clear them and
 * wait for their team to have done so (calls with more than 4 MB of such words
 * apart).  0 makes every call launch the clearing kernel again; returns the
 * previous setting. */
int fsd_debug_set_self_clear(int on);

/* Tuning hook: shape of the vocabulary-reduction kernel.  `wavefronts` per
 * workgroup must be 4 (or 0 = default); `slots_per_thread` is the number of
 * 16-byte slots of each row a lane holds: 2, 4 or 8 (bfloat16: 2, 4 or 5), 0 =
 * the library's own choice (32 vocabulary entries per lane and row; 48 for the
 * bfloat16 JS and TV kernels).  A shape
 * that would need more than 256 wavefronts per row pair is ignored.  Results
 * do not depend on the shape beyond the rounding order of the partial sums. */
int fsd_debug_set_shape(int wavefronts, int slots_per_thread);

/* Test hook: grid size (workgroups) of the last vocabulary-reduction launch and
 * the number of its workgroups the device can hold at once, which caps it. */
void fsd_debug_last_launch(int* grid, int* resident);

/* Test hook: byte offset, inside a workspace of fsd_workspace_bytes(B,
 * rows_per_seq, V, dtype), of the B binary32 values fsd_verify_chain_warped
 * leaves there: per sequence the smallest scaled logit its warpers kept on the
 * row the token was drawn from (-inf when nothing is cut).  0 for bad shapes. */
size_t fsd_debug_warp_threshold_offset(int B, int rows_per_seq, int V, int dtype);

#ifdef __cplusplus
}
#endif
#endif /* FSD_H_ */
