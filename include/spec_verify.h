/*
 * libspecverify — the target-side verification step of hybrid ordinary-parallel
 * speculative serving, as hand-written HIP kernels for gfx950 (MI355X).
 *
 * One decoding round on the target server (paper, Appendix "Implementation
 * Details", "Target side"): the batch Y_n = {y^(i)} of verification candidates
 * y^(i) = [b, d_1 .. d_gamma_i] is scored in one pass, the accepted length L
 * is computed per request, and the verified tokens are committed.  The four
 * calls below are that pass for one attention layer plus the LM head:
 *
 *   spec_verify_attn  attention of every candidate position over the paged KV
 *   spec_lm_head      one logits row per candidate position
 *   spec_accept       greedy prefix match or rejection sampling -> L, bonus
 *   spec_kv_commit    Commit on the KV side: new length, rejected pages freed
 *
 * Conventions for every call
 *   - All pointers are DEVICE pointers into caller-owned memory unless the
 *     comment says "host".  The library never allocates, frees or keeps them.
 *   - Every call only enqueues kernels on `stream` (a hipStream_t passed as
 *     void*); it never synchronises with the host.  `workspace` is scratch
 *     with no state carried between calls; it must be 256-byte aligned.
 *   - Return value: SPEC_OK (0) or a negative code; spec_last_error_string()
 *     gives the reason for the calling thread's last failure.  A failing call
 *     has enqueued nothing.
 *   - Data errors only the device can see (a page id out of range, a length
 *     beyond the stated bound, a non-finite logits row, a token id outside the
 *     vocabulary) never fault: the offending request is skipped or produces
 *     the documented neutral output and a bit is OR-ed into *status_flags
 *     (nullable, int32, device).
 *   - Request i has c_i = seq_lens[i] committed tokens and n_i =
 *     qo_indptr[i+1] - qo_indptr[i] = gamma_i + 1 >= 1 candidate rows; row
 *     qo_indptr[i] + j is candidate position j.  gamma_i = 0 is ordinary
 *     one-token decoding (the padded parallel-mode candidate of eq.
 *     parallel_rollback_pad / the "Fallback" paragraph).
 *   - bf16 = IEEE bfloat16 bit patterns (uint16_t storage).
 */
#ifndef SPEC_VERIFY_H
#define SPEC_VERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SPEC_OK 0
#define SPEC_EINVAL (-1)      /* NULL pointer, negative size, misaligned workspace */
#define SPEC_ESHAPE (-2)      /* shape outside what the kernels are built for */
#define SPEC_EWORKSPACE (-3)  /* workspace smaller than the *_workspace_bytes() answer */
#define SPEC_EHIP (-4)        /* the HIP runtime refused a launch */

/* bits of *status_flags */
#define SPEC_FLAG_BAD_PAGE 1      /* page id < 0 or >= num_pages met inside a visible range */
#define SPEC_FLAG_BAD_LENGTH 2    /* c_i + n_i > max_kv_len, n_i < 1 or n_i > max_q_len */
#define SPEC_FLAG_BAD_LOGITS 4    /* NaN in a logits row or a row maximum that is not finite */
#define SPEC_FLAG_BAD_TOKEN 8     /* draft token id outside [0, V) */
#define SPEC_FLAG_FREE_OVERFLOW 16 /* free list capacity exceeded in spec_kv_commit */
#define SPEC_FLAG_NO_SEED 32      /* temperature > 0 but seeds == NULL */
#define SPEC_FLAG_BAD_TREE 64     /* parent[] of a request is not a tree in topological order */

/* Text of the calling thread's last error ("" if none). host. */
const char* spec_last_error_string(void);

/* Library version, major * 1000 + minor. host. */
int spec_version(void);

/* Benchmark hook (host).  Overrides a launch heuristic; never changes results beyond fp32 summation order.
 * The settings are PROCESS-WIDE (one value per key for all threads and devices).  Each is a single word that is
 * written and read atomically, so a call racing with a launch on another thread is safe, but which of the two
 * values that launch sees is unspecified: set the keys before the serving threads start, as a benchmark does.
 * The verification calls themselves keep no other mutable state.  Keys:
 *   "attn_chunk"       keys per kv split of spec_verify_attn; 0 = automatic.
 *   "attn_plan"        device-built balanced work list of spec_verify_attn: 0 = automatic, 1 = always
 *                      (B <= 1024), 2 = never.
 *   "attn_plan_waves"  work items per CU that list aims at; 0 = automatic.
 *   "attn_nr3_waves"   waves per workgroup of spec_verify_attn when a request has 33..48 query rows per kv
 *                      head: 8 (default) or 4.
 *   "attn_rows"        the row-split kernel of spec_verify_attn (one 16-row tile per wave, K/V staged once per
 *                      workgroup): 0 = automatic (49..128 query rows per kv head), 1 = never, 2 = also for
 *                      17..48 rows.
 *   "attn_rows_ring"   K/V stages (32 keys each) a workgroup of that kernel keeps in LDS: 2 (default) or 4.
 *   "accept_filter"    how spec_accept normalises the rows of sampled requests: 0 = automatic and 1 = fp32 sums over
 *                      every row, an interval test, and fp64 sums only on the row a bonus token is drawn from and on
 *                      rows whose test the interval leaves open; 2 = fp64 sums over every row; 3 = as 1 with an
 *                      interval so wide that most tests take the fp64 path (a test hook).  Same integers in all.
 *   "lm_kernel"       kernel used by spec_lm_head: 0 = automatic (weight-streaming kernel for M <= 160,
 *                      MFMA-bound kernel above), 1 = weight-streaming, 2 = MFMA-bound with direct global->LDS
 *                      loads, 3 = plain tiled, 4..7 = weight-streaming variants (wave count / register-ring
 *                      depth), 8 = MFMA-bound with register staging.
 *   "lm_big_waves"     waves per workgroup of the MFMA-bound kernels of spec_lm_head: 4 or 8 (default).
 *   "lm_packed_waves"  waves per workgroup of the weight-streaming kernel of spec_lm_head_packed: 4 or 8 (default).
 *   "lm_packed_wide"   that kernel with passes of 512 vocabulary entries over row groups of at most 80 rows:
 *                      0 = automatic (off), 1 = always, 2 = never.
 *   "lm_packed_tile"   which kernel spec_lm_head_packed runs for M > 160: 0 = automatic (the large-tile MFMA-bound
 *                      kernel), 1 = the weight-streaming kernel over row groups of at most 160 rows.
 *   "lm_mfma_rows"     rows per row group of that large-tile kernel at most, 144..256; 0 = automatic.
 *   "lm_mfma_nt"       its logits stores nontemporal: 0 = automatic (one or two row groups), 1 = always, 2 = never.
 * A forced kernel that cannot take the shape falls back to the plain tiled one.  Unknown key: SPEC_EINVAL. */
int spec_set_tuning(const char* key, int value);

/* ---------------------------------------------------------------------------
 * spec_verify_attn — ragged multi-query paged attention over the candidates
 * (the target model's pass over Y_n, Method "Execution in ordinary/parallel
 * mode": the target performs the verification pass on the merged batch).
 *
 * For request i, candidate position j, query head h:
 *   out[row, h, :] = softmax_t( scale * <q[row, h, :], K_t> ) . V_t   over key
 *   positions t = 0 .. c_i + j   (causal inside the candidate block),
 * where position t of request i is slot t % page_size of physical page
 * page_table[i * max_pages_per_seq + t / page_size], and query head h reads
 * kv head h / (Hq / Hkv).  The K/V of the n_i candidate tokens must already be
 * in the cache at positions c_i .. c_i + gamma_i.
 *
 *   q        [M, Hq, D] bf16          out  [M, Hq, D] bf16
 *   k_cache  [num_pages, Hkv, page_size, D] bf16 (same for v_cache)
 *   page_table [B, max_pages_per_seq] int32     seq_lens [B] int32 (c_i)
 *   qo_indptr  [B+1] int32                      lse [M, Hq] fp32 or NULL:
 *                                                natural-log sum-exp of the scaled scores
 * Host bounds the launch is sized from: max_kv_len >= max_i(c_i + n_i),
 * max_q_len >= max_i n_i.  Built for D = 128, page_size = 16, Hq % Hkv == 0,
 * (Hq / Hkv) * max_q_len <= 128 query rows per kv head; anything else is SPEC_ESHAPE.  fp32 accumulation.
 * Requests that break a bound are skipped (rows left untouched) and flagged.
 * ------------------------------------------------------------------------- */
size_t spec_verify_attn_workspace_bytes(int B, int M, int Hq, int Hkv, int D, int max_kv_len, int max_q_len);

int spec_verify_attn(const void* q, const void* k_cache, const void* v_cache,
                     const int32_t* page_table, int max_pages_per_seq, int num_pages,
                     const int32_t* seq_lens, const int32_t* qo_indptr,
                     void* out, float* lse,
                     int B, int M, int Hq, int Hkv, int D, int page_size,
                     int max_kv_len, int max_q_len, float scale,
                     int32_t* status_flags,
                     void* workspace, size_t workspace_bytes, void* stream);

/* spec_verify_attn for tree-structured candidates (Appendix "Target side", "Unified verification interface": the
 * remote tokens become a verification tree; one remote sequence is the chain that spec_verify_attn handles).
 * parent [M] int32 (device): for every candidate row the row-local index of its parent inside its request,
 * -1 for the root (row 0), parent < own index; NULL = chains, identical to spec_verify_attn.  Row j attends to the
 * committed prefix and to the candidate rows on its own path to the root, itself included; the K/V of row j sits at
 * cache position c_i + j as before.  At most 64 rows per request (SPEC_ESHAPE beyond); a request whose parent[]
 * is not such a tree is skipped and SPEC_FLAG_BAD_TREE is raised.  Everything else as spec_verify_attn. */
int spec_verify_attn_tree(const void* q, const void* k_cache, const void* v_cache,
                          const int32_t* page_table, int max_pages_per_seq, int num_pages,
                          const int32_t* seq_lens, const int32_t* qo_indptr, const int32_t* parent,
                          void* out, float* lse,
                          int B, int M, int Hq, int Hkv, int D, int page_size,
                          int max_kv_len, int max_q_len, float scale,
                          int32_t* status_flags,
                          void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * spec_lm_head — logits of every candidate position (each position of Y_n is
 * scored so the accepted length can be computed; Appendix "Target side").
 *   logits[r, v] = sum_k hidden[r, k] * W[v, k]
 *   hidden [M, H] bf16, W [V, H] bf16 (one vocabulary entry per row),
 *   logits [M, V] fp32.  bf16 MFMA, fp32 accumulation.  H % 64 == 0 required
 *   (SPEC_ESHAPE otherwise); M and V are arbitrary (ragged tiles are handled).
 * ------------------------------------------------------------------------- */
int spec_lm_head(const void* hidden, const void* W, float* logits, int M, int H, int V, void* stream);

/* ---------------------------------------------------------------------------
 * spec_lm_head_stats — spec_lm_head that also leaves, for every row, the
 * maximum of each vocabulary block it computed and that maximum's lowest
 * index, so that greedy acceptance (temperature 0, the paper's default
 * setting: Experiments, "greedy decoding") need not read the logits again.
 * Same operation and passage as spec_lm_head; the statistics are what
 * spec_accept_stats consumes.
 *   blocks = spec_lm_head_stats_blocks(M, H, V) (host): blocks per row, 0 when
 *     the shape is not served by the fused kernel (then this call is exactly
 *     spec_lm_head, blk_max/blk_arg are not touched and may be NULL).
 *   blk_max [M, blocks] fp32, blk_arg [M, blocks] int32 (device, caller-owned):
 *     blocks cover increasing vocabulary ranges; a block that holds a NaN has
 *     blk_max = NaN; a block without entries has -inf and INT32_MAX.
 * Errors as spec_lm_head.
 * ------------------------------------------------------------------------- */
int spec_lm_head_stats_blocks(int M, int H, int V);

int spec_lm_head_stats(const void* hidden, const void* W, float* logits, int M, int H, int V,
                       float* blk_max, int32_t* blk_arg, void* stream);

/* ---------------------------------------------------------------------------
 * spec_lm_head_pack / spec_lm_head_packed — spec_lm_head (same operation, same
 * passage, same logits up to fp32 summation order) with the vocabulary matrix
 * re-laid once, when the model is loaded, into the order the matrix cores read
 * it, so that the weight stream of a verify batch is a linear read.
 *   Wp (device, caller-owned, spec_lm_head_packed_bytes(V, H) bytes, 16-byte
 *   aligned): panels of 16 vocabulary entries; for panel p, k-tile t (32
 *   consecutive k), lane l in [0, 64), element j in [0, 8):
 *     Wp[((p * (H/32) + t) * 64 + l) * 8 + j] = W[16 p + l % 16][32 t + 8 (l / 16) + j]
 *   and 0 where 16 p + l % 16 >= V; ceil(V / 16) panels.
 *   spec_lm_head_packed_bytes: host arithmetic; 0 for V <= 0 or H <= 0.
 *   spec_lm_head_pack: W [V, H] bf16 row-major -> Wp; H % 32 == 0 (SPEC_ESHAPE).
 *   spec_lm_head_packed: hidden [M, H] bf16, logits [M, V] fp32; H % 256 == 0
 *   (SPEC_ESHAPE otherwise); any M (above 160 rows the batch is cut into
 *   row groups of at most 256 rows that stream the same panels at the same
 *   time on one XCD, so that HBM still sees Wp once) and any V.
 * Both are asynchronous on the stream and allocate nothing.
 * ------------------------------------------------------------------------- */
size_t spec_lm_head_packed_bytes(int V, int H);

int spec_lm_head_pack(const void* W, void* Wp, int V, int H, void* stream);

int spec_lm_head_packed(const void* hidden, const void* Wp, float* logits, int M, int H, int V, void* stream);

/* spec_lm_head_packed that also leaves the block statistics described at spec_lm_head_stats (same meaning, same
 * consumer: spec_accept_stats), one block per row for every pass of a workgroup (256 vocabulary entries or fewer).
 *   blocks = spec_lm_head_packed_stats_blocks(M, H, V) (host): blocks per row; 0 when spec_lm_head_packed does
 *   not take the shape.  blk_max [M, blocks] fp32, blk_arg [M, blocks] int32 (device, caller-owned, required).
 * Errors as spec_lm_head_packed. */
int spec_lm_head_packed_stats_blocks(int M, int H, int V);

int spec_lm_head_packed_stats(const void* hidden, const void* Wp, float* logits, int M, int H, int V,
                              float* blk_max, int32_t* blk_arg, void* stream);

/* spec_lm_head_packed_summary — spec_lm_head_packed for more than 160 rows that also leaves what acceptance needs
 * from each row of logits, so that no row has to be read again (same operation and passage as spec_lm_head; the
 * consumer is spec_accept_summary).  A block is a run of at most 64 consecutive vocabulary entries; blocks cover
 * increasing ranges.
 *   blocks = spec_lm_head_packed_summary_blocks(M, H, V) (host): blocks per row; 0 when this call does not take the
 *     shape (M <= 160, H not a multiple of 256, or V not a multiple of 4) - use spec_lm_head_packed then.
 *   temperature [B] fp32, qo_indptr [B + 1] int32 (device): as for spec_accept; they say which rows are sampled.
 *   blk_max  [M, blocks] fp32: the block's maximum; NaN if the block holds a NaN.
 *   blk_sum  [M, blocks] fp32: for the rows of requests with temperature T > 0 the sum over the block of
 *     2^((l - blk_max) * log2(e) / T) (fp32 arithmetic, relative error < 2^-16), else 0.
 *   blk_span [blocks, 2] int32: first entry and number of entries of every block (0 entries: the slot is unused and
 *     its blk_max / blk_sum are not written).
 *   All four are device memory owned by the caller.  Logits as spec_lm_head_packed, bit for bit.  Errors as there;
 *   SPEC_ESHAPE for a shape with blocks == 0. */
int spec_lm_head_packed_summary_blocks(int M, int H, int V);

int spec_lm_head_packed_summary(const void* hidden, const void* Wp, float* logits, int M, int H, int V,
                                const float* temperature, const int32_t* qo_indptr, int B,
                                float* blk_max, float* blk_sum, int32_t* blk_span, void* stream);

/* ---------------------------------------------------------------------------
 * spec_accept — accepted length and bonus token per request (Method,
 * "Rollback-Based Mode Selection": after the verification pass the target
 * performs rejection sampling and identifies the rollback set).
 *
 * temperature[i] == 0: greedy.  g_j = argmax_v logits[row j] (lowest index on
 *   ties); drafts are accepted while tokens[row j] == g_{j-1}; bonus = g_a.
 * temperature[i]  > 0: rejection sampling with p_j = softmax(logits[row j]/T):
 *   draft d_j = tokens[row j] (j >= 1) is accepted iff u_j * q_j(d_j) < p_{j-1}(d_j);
 *   at the first rejection j* the bonus is drawn from norm(max(0, p_{j*-1} - q_{j*}));
 *   if every draft is accepted it is drawn from p_gamma.  q_j is row
 *   qo_indptr[i] - i + (j-1) of draft_probs; draft_probs == NULL means a
 *   deterministic drafter (q_j one-hot at d_j).  Uniforms come from
 *   Philox4x32-10 with key = seeds[i] (low, high word) and counter
 *   (0, j, tag, round): tag 0 for the accept test of draft j, tag 1 for the
 *   bonus draw at j* (or gamma_i + 1 when nothing is rejected); the first
 *   output word's top 24 bits give u in [0, 1).  Probabilities, sums and
 *   products are formed in fp64 and rounded to fp32 before they are compared.
 *   (A test whose outcome is the same at both ends of the error interval of an
 *   fp32 estimate of the normaliser is settled from that estimate; any other,
 *   and every bonus draw, uses the fp64 sum.  The integers returned are those of
 *   the fp64 definition; "accept_filter" of spec_set_tuning turns the estimate off.)
 *
 *   logits [M, V] fp32; tokens [M] int32 (row 0 of a request = its last
 *   committed token, unused here); draft_probs [M - B, V] fp32 or NULL;
 *   temperature [B] fp32; seeds [B] uint64 (NULL allowed if all greedy).
 * Outputs: accept_len [B] int32 (a_i in [0, gamma_i]); out_tokens
 *   [B, gamma_max + 1] int32 = a_i accepted drafts, the bonus, then -1;
 *   rollback [B] uint8 or NULL = (a_i < gamma_i); stats [4] int32 or NULL =
 *   {number of rollback requests |R_n|, sum of emitted tokens, B, 0} for the
 *   mode rule r_hat = |R_n| / B (eq. mode_switch_batch).
 * A request with a bad row or token gets a_i = 0, bonus -1, and a flag.
 * ------------------------------------------------------------------------- */
size_t spec_accept_workspace_bytes(int B, int M, int V, int gamma_max);

int spec_accept(const float* logits, const int32_t* tokens, const float* draft_probs,
                const float* temperature, const uint64_t* seeds, uint32_t round,
                const int32_t* qo_indptr,
                int32_t* accept_len, int32_t* out_tokens, uint8_t* rollback, int32_t* stats,
                int B, int M, int V, int gamma_max,
                int32_t* status_flags,
                void* workspace, size_t workspace_bytes, void* stream);

/* spec_accept_static — spec_accept for callers that cannot allocate device memory or hand in a workspace: code
 * recorded into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (without
 * workspace), same kernels, same outputs, flags and errors as spec_accept; the scratch is a 4 MiB array inside
 * the library image, one copy per GPU, held until the process ends.  Allocates nothing.
 *   Limit: spec_accept_workspace_bytes(B, M, V, gamma_max) <= 4 MiB (e.g. M = 1206 rows x V = 151936 needs 1.1 MiB);
 *   beyond it SPEC_EWORKSPACE with the sizes in the error text, and nothing is enqueued.
 *   All calls on one GPU share that GPU's array, which keeps the previous call's contents (no part of it has to
 *   be cleared: each call overwrites what it reads): calls that overlap in time on one GPU, on different
 *   streams, race and must be ordered by the caller.  The first call on each device resolves the array's device
 *   address (one hipGetSymbolAddress, no allocation); make it outside stream capture. */
int spec_accept_static(const float* logits, const int32_t* tokens, const float* draft_probs,
                       const float* temperature, const uint64_t* seeds, uint32_t round,
                       const int32_t* qo_indptr,
                       int32_t* accept_len, int32_t* out_tokens, uint8_t* rollback, int32_t* stats,
                       int B, int M, int V, int gamma_max,
                       int32_t* status_flags, void* stream);

/* spec_accept with the block summaries of spec_lm_head_packed_summary (blocks == 0: identical to spec_accept).  No
 * row of logits is scanned: a greedy row finds its argmax inside the one block that holds the row maximum (64 logits
 * are read), a sampled row takes the estimate of its normaliser from the block sums, which the interval test of
 * spec_accept then uses (the "accept_filter" key cannot turn that off here); the one row per sampled request that
 * the bonus is drawn from is still summed in fp64 from the logits.  Same outputs, flags and errors as spec_accept. */
int spec_accept_summary(const float* logits, const int32_t* tokens, const float* draft_probs,
                        const float* temperature, const uint64_t* seeds, uint32_t round,
                        const int32_t* qo_indptr,
                        int32_t* accept_len, int32_t* out_tokens, uint8_t* rollback, int32_t* stats,
                        int B, int M, int V, int gamma_max,
                        const float* blk_max, const float* blk_sum, const int32_t* blk_span, int blocks,
                        int32_t* status_flags,
                        void* workspace, size_t workspace_bytes, void* stream);

/* spec_accept with the block statistics of spec_lm_head_stats (blk_max, blk_arg, blocks as described there;
 * blocks == 0: identical to spec_accept).  Requests with temperature 0 take their row maxima from the
 * statistics; the logits of their rows are not read.  Sampled requests are handled as in spec_accept.  With
 * seeds == NULL (all requests greedy) no logits are read at all.  Same outputs, flags and errors. */
int spec_accept_stats(const float* logits, const int32_t* tokens, const float* draft_probs,
                      const float* temperature, const uint64_t* seeds, uint32_t round,
                      const int32_t* qo_indptr,
                      int32_t* accept_len, int32_t* out_tokens, uint8_t* rollback, int32_t* stats,
                      int B, int M, int V, int gamma_max,
                      const float* blk_max, const int32_t* blk_arg, int blocks,
                      int32_t* status_flags,
                      void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * spec_next_mode — execution mode of round n+1 (Method, "Rollback-Based Mode
 * Selection", eq. mode_switch_batch) from the observed rollback ratio
 * r_hat = |R_n| / B and the critical ratio (Section "Throughput-Guided Hybrid
 * Coordination", eq. r_threshold)
 *   r* = (gamma - 1) L t_draft / ((t_target + (gamma - 1) t_draft) (L - 1)),
 * L = emitted tokens / B.  PARALLEL iff r_hat <= r*.  With L <= 1 (the
 * derivation assumes L > 1) r* is +infinity: a round then yields one token
 * per request in either mode and the ordinary round is the longer one.
 *   stats_host: HOST copy of the stats[4] written by spec_accept.
 *   gamma: speculative tokens per verification in the paper's counting, i.e.
 *     candidate rows per request (drafts + the bonus position); t_draft,
 *     t_target: latency of one draft step / one target verification, same unit.
 *   r_hat, r_star: optional outputs (host).
 * Pure host arithmetic; launches nothing.  Returns SPEC_MODE_PARALLEL or
 * SPEC_MODE_ORDINARY, or SPEC_EINVAL (< 0) on NULL / inconsistent arguments.
 * ------------------------------------------------------------------------- */
#define SPEC_MODE_ORDINARY 0
#define SPEC_MODE_PARALLEL 1
int spec_next_mode(const int32_t* stats_host, double gamma, double t_draft, double t_target,
                   double* r_hat, double* r_star);

/* ---------------------------------------------------------------------------
 * spec_kv_commit — Commit(p_n, y_n, L_n) on the KV cache (Appendix "Target
 * side"; rollback frees the KV of the rejected suffix, Appendix "Draft side").
 *   new_len_i = c_i + a_i + 1; pages ceil(new_len_i / P) .. ceil((c_i + n_i) / P) - 1
 *   of request i are unmapped (-1) and appended to free_list in request order,
 *   then logical-page order; seq_lens[i] <- new_len_i; *free_count grows.
 *   accept_len values outside [0, gamma_i] are clamped.  No KV data moves: the
 *   accepted tokens of a chain are a prefix of the candidate.
 *   page_table [B, max_pages_per_seq] int32 in/out; seq_lens [B] in/out;
 *   free_list [free_capacity] int32 in/out; free_count [1] int32 in/out.
 *   If the list would overflow, the excess pages are still unmapped, are not
 *   recorded, and SPEC_FLAG_FREE_OVERFLOW is raised.
 * ------------------------------------------------------------------------- */
int spec_kv_commit(int32_t* page_table, int max_pages_per_seq, int32_t* seq_lens,
                   const int32_t* qo_indptr, const int32_t* accept_len,
                   int32_t* free_list, int32_t free_capacity, int32_t* free_count,
                   int B, int page_size, int32_t* status_flags, void* stream);

/* ---------------------------------------------------------------------------
 * spec_assemble_next — the candidates y_{n+1} of the next verification round,
 * on the device, from the outputs of spec_accept (Method, "Execution in
 * ordinary mode" and "Execution in parallel mode": eqs. ordinary_rollback_seq,
 * ordinary_stable_seq, parallel_stable_seq, parallel_rollback_pad; Appendix
 * "Target side", eq. target_suffix_reuse).  Per request, with a accepted
 * drafts, bonus b = out_tokens[i][a] and gamma_i verified drafts:
 *   stable  <=>  a == gamma_i and the continuation the drafter prepared
 *     meanwhile starts with b (cont_len[i] >= 1 and cont[i][0] == b; the
 *     reading taken for Consistent()).  Candidate [b, cont[i][1 .. 1+g)],
 *     g = min(cont_len[i] - 1, gamma_next).
 *   otherwise the request is in the rollback set (Method, "Rollback-Based Mode Selection": a request
 *     belongs to it when the verified drafts were not all accepted, or when the continuation the drafter
 *     prepared in the meantime no longer fits what verification produced):
 *     mode SPEC_MODE_ORDINARY with repair != NULL: [b, repair[i][0 .. g)],
 *       g = min(repair_len[i], gamma_next) (the continuation regenerated from b);
 *     mode SPEC_MODE_PARALLEL: [b] (the padded candidate, ragged: gamma = 0).
 *   A request spec_accept could not decide (bonus -1) gets the row [-1].
 * Inputs (device): accept_len [B], out_tokens [B, gamma_max+1], qo_indptr [B+1]
 *   of the round just verified; cont [B, cont_stride] / cont_len [B] and repair
 *   [B, repair_stride] / repair_len [B] int32, each pair NULL if absent.
 * Outputs (device, caller-owned): next_tokens [B * (gamma_next + 1)] (rows of all
 *   requests in request order, first row of a request = b), next_qo_indptr
 *   [B+1], rollback [B] uint8 or NULL (the rollback set as defined above),
 *   stats [4] int32 or NULL = {|R_n|, sum (a_i + 1), B, rows of round n+1},
 *   the input of spec_next_mode.  Deterministic layout.  Asynchronous on stream;
 *   SPEC_EINVAL on NULL / negative arguments or an unknown mode.
 * ------------------------------------------------------------------------- */
int spec_assemble_next(const int32_t* accept_len, const int32_t* out_tokens, int gamma_max,
                       const int32_t* qo_indptr, int B,
                       const int32_t* cont, int cont_stride, const int32_t* cont_len,
                       const int32_t* repair, int repair_stride, const int32_t* repair_len,
                       int mode, int gamma_next,
                       int32_t* next_tokens, int32_t* next_qo_indptr, uint8_t* rollback,
                       int32_t* stats, void* stream);

/* ---------------------------------------------------------------------------
 * Draft-side primitives (Appendix "Draft side"; Method, "Draft-side context
 * compression").  Integer-only, ragged, asynchronous on stream; device pointers.
 *
 * spec_divergence — "Message handling and update": delta_i = min{ t :
 *   p_i[t] != h_i[t] } between the verified prefix p_i and the draft's own
 *   decoded tokens h_i (rows p_indptr[i] .. p_indptr[i+1] of p_tokens, likewise
 *   h); when one is a prefix of the other, the shorter length.  delta [B] int32.
 *
 * spec_kv_truncate — "State recovery", Rollback(S, delta): request i keeps
 *   min(seq_lens[i], max(keep_len[i], 0)) tokens; the pages beyond
 *   ceil(new_len / page_size) are set to -1 in page_table and appended to
 *   free_list (requests ascending, logical pages ascending), seq_lens and
 *   *free_count are updated.  Arguments, flags and errors as spec_kv_commit.
 *
 * spec_compress_prompts — eq. token_eviction: E(x_{1:S}) = [x_{:k}, x_{S-k+1:}],
 *   k = floor(p S / 2): the first k and the last k tokens, with the retained
 *   ratio p = p_num / p_den given as a fraction (k = p_num * S / (2 p_den) in
 *   integers; the paper's p = 0.1 is 1 / 10).  A prompt with 2k >= S is kept
 *   whole.  tokens / indptr [B+1] in; out_tokens (capacity: the input's token
 *   count), out_indptr [B+1], kept_index (or NULL: the position inside its
 *   prompt of every kept token) out.
 * SPEC_EINVAL on NULL / negative arguments; nothing is launched for B == 0
 * except that out_indptr[0] is set.
 * ------------------------------------------------------------------------- */
int spec_divergence(const int32_t* p_tokens, const int32_t* p_indptr, const int32_t* h_tokens,
                    const int32_t* h_indptr, int32_t* delta, int B, void* stream);

int spec_kv_truncate(int32_t* page_table, int max_pages_per_seq, int32_t* seq_lens, const int32_t* keep_len,
                     int32_t* free_list, int32_t free_capacity, int32_t* free_count,
                     int B, int page_size, int32_t* status_flags, void* stream);

int spec_compress_prompts(const int32_t* tokens, const int32_t* indptr, int B, int p_num, int p_den,
                          int32_t* out_tokens, int32_t* out_indptr, int32_t* kept_index, void* stream);

/* ---------------------------------------------------------------------------
 * Tree-structured verification, acceptance and commit (Appendix "Target side",
 * "Unified verification interface").  Attention: spec_verify_attn_tree above.
 *
 * spec_accept_tree — greedy (temperature 0) acceptance on candidate trees: from
 *   the root, at node u the target's token is the argmax of logits row u (lowest
 *   index on ties); the walk moves to the child of u that carries this token
 *   (the lowest row among equal children) and ends where there is none.
 *   tokens [M], parent [M] (as for spec_verify_attn_tree), logits [M, V] fp32.
 *   Outputs: accept_len [B] = drafts accepted, out_tokens [B, gamma_max+1] =
 *   their tokens, the bonus (argmax at the last node), then -1; path
 *   [B, gamma_max+1] = row-local indices of the visited nodes (path[0] = 0),
 *   then -1; rollback [B] or NULL = the last node still had children; stats [4]
 *   or NULL as for spec_accept.  Bad rows / tokens / trees: a = 0, tokens -1,
 *   path {0}, and SPEC_FLAG_BAD_LOGITS / _BAD_TOKEN / _BAD_TREE.  Workspace:
 *   spec_accept_workspace_bytes.  Sampling on trees is not built.
 *
 * spec_kv_commit_tree — the K/V of the accepted nodes (cache positions
 *   c_i + path[k]) are moved to c_i + k, k = 1 .. a_i, then lengths, page table
 *   and free list are updated exactly as by spec_kv_commit.  k_cache / v_cache
 *   [num_pages, Hkv, page_size, D] bf16 are modified in place.  A path that is
 *   not increasing with path[k] >= k raises SPEC_FLAG_BAD_TREE and moves nothing
 *   further for that request.
 * ------------------------------------------------------------------------- */
int spec_accept_tree(const float* logits, const int32_t* tokens, const int32_t* parent,
                     const int32_t* qo_indptr, int32_t* accept_len, int32_t* out_tokens, int32_t* path,
                     uint8_t* rollback, int32_t* stats, int B, int M, int V, int gamma_max,
                     int32_t* status_flags, void* workspace, size_t workspace_bytes, void* stream);

int spec_kv_commit_tree(void* k_cache, void* v_cache, int32_t* page_table, int max_pages_per_seq, int num_pages,
                        int32_t* seq_lens, const int32_t* qo_indptr, const int32_t* accept_len,
                        const int32_t* path, int gamma_max,
                        int32_t* free_list, int32_t free_capacity, int32_t* free_count,
                        int B, int Hkv, int D, int page_size, int32_t* status_flags, void* stream);

/* ---------------------------------------------------------------------------
 * Measurement probes (not part of the verification path; no passage of the paper defines them).  They give the
 * ceilings this particular chip reaches, for reports that quote a kernel against the measured roof as well as
 * against the datasheet.  Asynchronous on stream; time them with events on that stream.
 *   spec_probe_read: reads `bytes` bytes at src (device, 16-byte aligned, bytes % 16 == 0) exactly once, linearly;
 *     sink (device, >= 4 bytes) is practically never written.  SPEC_EINVAL on misuse.
 *   spec_probe_read_pages: reads the n_pages pages of 4096 bytes listed in pages[] (device int32, page p = bytes
 *     4096 p .. 4096 p + 4095 of src), each once, in list order: the access pattern of a paged K/V cache.
 *   spec_probe_mfma: one workgroup of 8 waves per compute unit, each wave `iters` x 16 independent
 *     v_mfma_f32_16x16x32_bf16 on register operands (random bit patterns, or all equal when bit 0 of
 *     constant_operands is set: the chip's power limit makes the two differ; bit 1 set: the same flops as `iters` x 8
 *     v_mfma_f32_32x32x16_bf16).  Returns the floating-point operations of the launch as a
 *     double (> 0), or -1 on misuse.  sink: device, >= 4 bytes, practically never written.
 * ------------------------------------------------------------------------- */
int spec_probe_read(const void* src, size_t bytes, void* sink, void* stream);

int spec_probe_read_pages(const void* src, const int32_t* pages, int n_pages, void* sink, void* stream);

double spec_probe_mfma(int iters, int constant_operands, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SPEC_VERIFY_H */
