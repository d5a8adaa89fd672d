/*
 * mlda — collapsed Gibbs sampling for LDA on one AMD MI355X (gfx950).
 *
 * C ABI of libmlda.so.  The problem statement follows the paper's Section 2.1:
 * a corpus of D documents over a vocabulary of V words, K topics and the
 * hyper-parameters alpha and beta go in; the topic assignment of every token,
 * the document-topic counts theta, the topic-word counts phi and a
 * log-likelihood come out, one sampling pass ("iteration") at a time.
 *
 * What one iteration computes (Sections 2.1 and 6):
 *   every token (document d, word v, current topic o) draws a new topic from
 *       p(k) ~ (theta_dk + alpha)(phi_kv + beta) / (n_k + beta V)          (Eq. 1)
 *   evaluated as p = p1 + p2 with p1 = theta_dk p*(k), p2 = alpha p*(k),
 *   p*(k) = (phi_kv + beta)/(n_k + beta V), S = sum p1, Q = sum p2       (Eq. 6-8),
 *   one uniform choosing the bucket and the smallest k whose prefix sum
 *   exceeds the draw (Section 6.1.1, Algorithm 2);
 *   then phi and theta are rebuilt from the new assignments (Section 6.2).
 * Fixed by this library where the paper leaves a choice:
 *   - all tokens of an iteration see the counts as they stood when the
 *     iteration began, each with the token's own assignment removed;
 *   - p*(k) is the fp64 quotient rounded once to fp32, products and sums are fp64;
 *   - the uniform of token t in iteration i is the top 53 bits of the first two
 *     words of Philox4x32-10 with counter (t lo, t hi, i, 0) and key
 *     (seed lo, seed hi), where t is the token's index in the caller's
 *     document-major word_ids array; x = u (S+Q); x < S takes the p1 bucket
 *     (topics ascending) at position x, otherwise the p2 bucket at x - S;
 *   - iteration 0 of the same generator gives the initial topics, floor(u K).
 *
 * Conventions
 *   - Every function returns MLDA_OK (0) or a negative code; mlda_last_error()
 *     gives the message of the calling thread's most recent failure.
 *   - "host" pointers are ordinary CPU memory owned by the caller and only read
 *     or written during the call.  The device workspace and the HIP stream are
 *     the caller's too (e.g. a torch uint8 CUDA tensor and
 *     torch.cuda.current_stream().cuda_stream); the library allocates no device
 *     memory, keeps the workspace until mlda_destroy, and launches all kernels on
 *     that stream (a context made by mlda_create_streamed also owns pinned host
 *     memory and two copy streams).  Getters synchronise the stream.
 *   - A context is not thread-safe.  Token order at the boundary is always the
 *     caller's document-major order; the word-major order used on the device is
 *     internal.
 */
#ifndef MLDA_H
#define MLDA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MLDA_OK        0
#define MLDA_EINVAL   -1   /* bad argument (null pointer, K outside [1,65535], alpha or beta <= 0,
                              word id outside [0,V), doc_ptr not starting at 0 or decreasing,
                              2^31 or more tokens, topic >= K) */
#define MLDA_ENOMEM   -2   /* device workspace smaller than mlda_workspace_bytes, or host malloc failed */
#define MLDA_EHIP     -3   /* a HIP call failed; the message names it */
#define MLDA_ENOTSUP  -4   /* the device allows a workgroup less LDS than a kernel needs for this K (not on
                              MI355X, whose 160 KB serve every K up to 65,535, the range of the 16-bit topic
                              index of Section 6.1.3: up to about 30,900 the sampler keeps the word's column
                              of p* (Eq. 8) in LDS, beyond that in device memory, several times slower; the
                              paper's own range is 1,000 to 10,000, Section 2.1); also theta rows beyond
                              64 GiB in one chunk, and a device index beyond the library's table */

#define MLDA_STEP_LOGLIK 1u /* mlda_step flag: also evaluate the log-likelihood after each iteration */

typedef struct mlda_ctx mlda_ctx;   /* opaque */

/* Bytes of device workspace mlda_create needs for a corpus of D documents and T
 * tokens (an upper bound that depends on the sizes only).  bytes: host, out. */
int mlda_workspace_bytes(int64_t D, int64_t T, int32_t V, int32_t K, size_t* bytes);

/*
 * Build a context (Section 2.1: the corpus; Section 6.1.2: tokens are put in
 * word-first order, on the host; Section 6.2: a document->token map, which the paper
 * builds on the CPU, is derived on the device).
 *   doc_ptr   host, D+1 entries, doc_ptr[0] = 0, non-decreasing; document d owns
 *             tokens doc_ptr[d] .. doc_ptr[d+1]-1.  T = doc_ptr[D] < 2^31.
 *   word_ids  host, T entries, each in [0,V).
 *   dev_workspace  DEVICE pointer, 256-byte aligned, workspace_bytes long.
 *   hip_stream     a hipStream_t (0 = the default stream).
 * The corpus is copied; the host arrays may be released after the call.  No
 * topics are assigned yet: call mlda_init_random or mlda_set_assignments next.
 * K: 1 .. 65,535 (MLDA_EINVAL outside).  A K whose column of p* does not fit the 160 KB of LDS
 * of a workgroup (beyond about 30,900) is sampled with p* in device memory: same results, several
 * times slower per token; the workspace then holds 512 such columns more.
 * Environment, read here: MLDA_WIDE_SLOT_OFFSETS=1 makes the sampler address theta rows with 64-bit
 * offsets, the form it otherwise takes only when the rows of a chunk fill more than 4 GiB (for
 * tests; same results, a few per cent slower).
 */
int mlda_create(mlda_ctx** out, const int64_t* doc_ptr, const int32_t* word_ids,
                int64_t D, int32_t V, int32_t K, double alpha, double beta, uint64_t seed,
                void* dev_workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The same with the corpus cut by document into n_chunks chunks of about equal token
 * counts that take turns on the GPU (Section 4: partition by document; Algorithm 1,
 * WorkSchedule2: with more than one chunk per GPU the chunks are transferred every
 * iteration, phi stays on the device).  For corpora whose tokens and theta rows do not fit
 * the device beside phi.  The preprocessed chunks and all assignments are kept in pinned
 * host memory that the library allocates; per iteration every chunk is uploaded (on a stream
 * of default priority that the library creates, overlapping the kernels of the chunk
 * before), its theta rows are rebuilt from its assignments, it is sampled against the phi of
 * the iteration's start, its counts are added to the next phi, and its new assignments go
 * back to the host (on a second such stream).  Results are identical, bit for bit, to those of mlda_create: the counts
 * of an iteration are frozen and the uniforms are keyed by the caller's token index.
 * The workspace (mlda_workspace_bytes_streamed: two copies of phi and two chunk buffers) and
 * the other arguments are as for mlda_create; doc_ptr is read by the sizing call too.
 * Differences in use: the rows of mlda_get_timing and mlda_get_sampler_bytes are sums over the
 * chunk visits of an iteration (kernel time on the context's stream: waiting for a transfer is
 * not in them), and the third column of mlda_get_timing also holds the two changes of token
 * order a visit needs; the theta getters and mlda_get_loglik (when the last step did not
 * evaluate it) revisit every chunk.
 */
int mlda_workspace_bytes_streamed(const int64_t* doc_ptr, int64_t D, int32_t V, int32_t K,
                                  int32_t n_chunks, size_t* bytes);
int mlda_create_streamed(mlda_ctx** out, const int64_t* doc_ptr, const int32_t* word_ids,
                         int64_t D, int32_t V, int32_t K, double alpha, double beta, uint64_t seed,
                         int32_t n_chunks, void* dev_workspace, size_t workspace_bytes,
                         void* hip_stream);

/*
 * mlda_create for callers that cannot allocate device memory (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc) and so have no workspace to hand over:
 * the context works in a static device array of MLDA_STATIC_WORKSPACE_BYTES that belongs to
 * the library (each GPU the library is used on holds its own copy until the process ends).
 * The call, and every later call on the context, allocates no device memory.  Everything else
 * is as for mlda_create, with the same kernels and bit-identical results.
 *   - A corpus whose mlda_workspace_bytes exceeds MLDA_STATIC_WORKSPACE_BYTES is refused with
 *     MLDA_ENOMEM (the message names both sizes): use mlda_create for it.
 *   - The array is shared by all such contexts of the process on one GPU, so only one of them
 *     may be alive per GPU at a time: a second call on the same device before mlda_destroy of
 *     the first returns MLDA_EINVAL (two contexts working in the one array would race).  The
 *     device that is current at the call is the one whose array is used; hip_stream must be
 *     a stream of that device.
 *   - The array keeps what the previous context left there; the library initialises
 *     every part it reads, as it does for a caller's uninitialised workspace.
 */
#define MLDA_STATIC_WORKSPACE_BYTES (64u << 20)
int mlda_create_static(mlda_ctx** out, const int64_t* doc_ptr, const int32_t* word_ids,
                       int64_t D, int32_t V, int32_t K, double alpha, double beta, uint64_t seed,
                       void* hip_stream);

/* Random initial topics (Section 2.1), z[t] = floor(u(seed, 0, t) K); rebuilds all
 * counts; the iteration counter becomes 0. */
int mlda_init_random(mlda_ctx* ctx);

/* Install assignments (host, T entries, document-major, each < K), rebuild all counts,
 * and set the number of iterations already done (the next pass uses iter+1 in the
 * generator's counter): resumes a run from a saved state. */
int mlda_set_assignments(mlda_ctx* ctx, const uint16_t* z, int32_t iter);

/* Run n_iters iterations: sample every token (Section 6.1), rebuild phi and n_k, then
 * theta (Section 6.2); with MLDA_STEP_LOGLIK also the log-likelihood of each new state.
 * Asynchronous on the context's stream. */
int mlda_step(mlda_ctx* ctx, int32_t n_iters, uint32_t flags);

/* Number of iterations done so far. iter: host, out. */
int mlda_iteration(const mlda_ctx* ctx, int32_t* iter);

/* Current assignments, document-major.  z: host, T entries, out. */
int mlda_get_assignments(mlda_ctx* ctx, uint16_t* z);

/* phi as a word-major matrix: n_wk[v*K + k] = tokens of word v with topic k, exact (on the
 * device 16-bit cells, int32 for words with 2^16 tokens or more; widened here on the host,
 * which takes V*K*2 bytes of temporary host memory).  n_wk: host, V*K entries, out. */
int mlda_get_word_topic(mlda_ctx* ctx, int32_t* n_wk);

/* n_k[k] = sum_v phi_kv, the denominator term of Eq. 1.  n_k: host, K entries, out. */
int mlda_get_topic_totals(mlda_ctx* ctx, int32_t* n_k);

/* Number of non-zero entries of theta. nnz: host, out. */
int mlda_get_doc_topic_nnz(mlda_ctx* ctx, int64_t* nnz);

/* theta in CSR form (Sections 3.1 and 6.1.3: 16-bit column indices): row_ptr host D+1
 * entries; topics / counts host, mlda_get_doc_topic_nnz entries each; within a row the
 * topics ascend and every count is positive. */
int mlda_get_doc_topic_csr(mlda_ctx* ctx, int64_t* row_ptr, uint16_t* topics, int32_t* counts);

/* Joint collapsed log-likelihood log p(w, z | alpha, beta) of the current state
 * (the "log-likelihood per token" of Section 7.2 is this value divided by T).
 * ll: host, out. */
int mlda_get_loglik(mlda_ctx* ctx, double* ll);

/*
 * Kernel times of the iterations of the most recent mlda_step, from HIP events on
 * the context's stream.  ms: host, capacity_iters rows of 4 doubles (sampling, rebuild
 * phi and n_k, rebuild theta, log-likelihood), out; n_iters: host, out, rows filled
 * (the last min(n, capacity_iters, 1024) iterations of that step).
 */
int mlda_get_timing(mlda_ctx* ctx, double* ms, int32_t capacity_iters, int32_t* n_iters);

/*
 * Algorithmic bytes each sampling launch of the most recent mlda_step had to move
 * (Section 3.1's accounting, with p* shared per word tile): per token 16 bytes (slot of
 * its theta row, token id, old and new topic, row length) plus the entries of its theta row
 * (Section 6.1.3's compression taken further: 2 bytes per entry when K < 1024, ten bits of
 * topic and four of count, else 4 bytes, sixteen bits of topic and fourteen of count; a count
 * beyond its field takes several entries), plus the word's row of phi per tile: 2 K bytes
 * (Section 6.1.3: short integers), 4 K for a word with 2^16 tokens or more, whose counts the
 * library keeps as int32.  With K > 2048 the words of at most 1024 tokens are sampled in runs
 * of 16 by one workgroup, which derives every following word's p* from the one before: such
 * a word then counts, instead of a row of phi, 6 bytes per token (the topics of the word
 * before it, and topic and cell of phi of its own tokens).  bytes: host, capacity_iters
 * doubles, out; rows as in mlda_get_timing.
 */
int mlda_get_sampler_bytes(mlda_ctx* ctx, double* bytes, int32_t capacity_iters, int32_t* n_iters);

/* Releases the context (host memory, events, its copy streams if any); the workspace stays
 * the caller's. */
void mlda_destroy(mlda_ctx* ctx);

/* n uniforms of iteration iter for tokens token0 .. token0+n-1 into DEVICE memory
 * (out_dev: device, n doubles), on hip_stream: exposes the generator for checking. */
int mlda_philox_uniform(uint64_t seed, uint32_t iter, uint64_t token0, int64_t n,
                        double* out_dev, void* hip_stream);

const char* mlda_strerror(int code);
const char* mlda_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MLDA_H */
