/*
 * tli.h -- C ABI of the MI355X (gfx950) Token-Level Intersection draft-and-verify library.
 *
 * One iteration of speculative decoding for heterogeneous vocabularies by token-level intersection:
 * the drafter distribution q over vocabulary D is restricted to the tokens it shares with the target
 * vocabulary T and renormalised (q'), K draft tokens are drawn from q', and the target's K+1
 * distributions p verify them with the lossless rejection rule of standard speculative decoding.
 * (Paper: section "Speculative Decoding for Heterogeneous Vocabularies with Token-Level Verification",
 * the intersection algorithm; appendix "Standard Speculative Decoding".)
 *
 * Conventions shared by every entry point
 *   - "dev" pointers are device pointers on the device that was current when the map was built;
 *     "host" pointers are ordinary host memory.  The library never takes ownership of a buffer the
 *     caller passes; it owns only the tli_map object.
 *   - Logits stand for distributions: p = softmax(logits_t / temp_t) over T, q = softmax(logits_d /
 *     temp_d) over D.  Logit storage is fp32 or bf16 (tli_dtype); all arithmetic is fp32 with fp64
 *     combination of partial sums and fp64 scalar decisions.
 *   - Logit base pointers must be 16-byte aligned and every row must start on a 16-byte boundary
 *     (row strides are multiples of 4 fp32 / 8 bf16 elements).  -inf logits are legal (probability 0).
 *   - Randomness is supplied by the caller as fp32 uniforms in [0,1).
 *   - Inverse-CDF sampling walks ids in ascending order and returns the first id whose running sum
 *     exceeds u * total (strict), so zero-probability ids are never returned.
 *   - The hot calls (tli_draft_sample, tli_verify) only enqueue kernels on the given HIP stream: no
 *     allocation, no synchronisation.  On a non-zero return nothing was enqueued.
 *   - Data-dependent trouble is reported per row / per sequence as TLI_FLAG_* bits, never by aborting.
 *   - Sizes: 1 <= K <= 64 draft positions per sequence; row counts (R, B*K, B*(m+1)) up to 2^31/64;
 *     vocabularies up to 2^30 ids.  Offsets into the logit buffers are 64-bit: a buffer may hold more
 *     than 2^31 elements.  Anything outside these limits returns TLI_ERR_INVALID_ARG (workspace queries: 0).
 */
#ifndef TLI_H
#define TLI_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tli_map tli_map; /* opaque, device-resident vocabulary intersection */

typedef enum { TLI_F32 = 0, TLI_BF16 = 1 } tli_dtype;

typedef enum {
    TLI_OK = 0,
    TLI_ERR_INVALID_ARG = -1,        /* null pointer, non-positive size or temperature, bad alignment */
    TLI_ERR_OUT_OF_RANGE = -2,       /* a d2t entry is neither -1 nor in [0, Vt)                       */
    TLI_ERR_NOT_INJECTIVE = -3,      /* two drafter ids map to the same target id                      */
    TLI_ERR_EMPTY_INTERSECTION = -4, /* no shared token: q' would be 0/0 and nothing can be accepted   */
    TLI_ERR_ALLOC = -5,              /* device allocation failed, or the workspace is too small        */
    TLI_ERR_HIP = -6,                /* a HIP runtime call failed                                      */
    TLI_ERR_INTERNAL = -7,           /* the library's own tables failed their consistency check        */
    TLI_ERR_TOO_LARGE = -8           /* tli_verify_static: the problem needs more than the fixed scratch */
} tli_status;

/* bits of row_status / seq_status */
enum {
    TLI_FLAG_NONFINITE = 1,  /* a logit that takes part in the computation is NaN or +inf           */
    TLI_FLAG_ZERO_MASS = 2,  /* the shared ids of a drafter row carry no mass (all -inf)            */
    TLI_FLAG_BAD_DRAFT = 4,  /* a draft id given to tli_verify is not a shared drafter id (or -1)   */
    TLI_FLAG_DEGENERATE = 8  /* rejected, but the residual is identically zero; extra token from p  */
};

/*
 * Vocabulary intersection T∩D (section "Preliminaries", the notation paragraph: a vocabulary is a set of
 * strings, so two tokens are shared iff their strings are equal, which the caller resolves into d2t; the
 * intersection algorithm needs nothing else of the two vocabularies).
 *   d2t_host [Vd] host : target id of drafter id x, or -1 if x is not in T.  Must be injective on
 *                        the ids it maps.
 *   out_map            : receives the new map (tables live on the current HIP device).
 *   out_num_shared     : receives |T∩D| (may be NULL).
 * All argument checks run before the first HIP call, so every TLI_ERR_* except ALLOC/HIP can be
 * returned on a machine without a GPU.  Synchronous.  Free with tli_free_map.
 */
int tli_build_map(const int32_t* d2t_host, int32_t Vd, int32_t Vt, tli_map** out_map, int32_t* out_num_shared);
void tli_free_map(tli_map* map);
/* Vd, Vt and |T∩D| of a map (any pointer may be NULL). */
int tli_map_info(const tli_map* map, int32_t* Vd, int32_t* Vt, int32_t* num_shared);
/*
 * Host-only convenience (notation paragraph: a vocabulary is a set of strings, so two tokens are shared iff their
 * strings are equal): d2t from the two vocabularies' token strings by exact byte equality.  Token x of a vocabulary
 * is the bytes [offs[x], offs[x+1]) of its byte array (any bytes, no terminator).
 *   bytes_d, offs_d [Vd+1] host : the drafter's tokens;  bytes_t, offs_t [Vt+1] host : the target's
 *   d2t_out [Vd] host           : receives the target id of every drafter id, or -1
 *   out_num_shared              : receives |T∩D| (may be NULL)
 * TLI_ERR_NOT_INJECTIVE if a string occurs twice in one vocabulary (a set has no duplicates),
 * TLI_ERR_OUT_OF_RANGE if offsets do not ascend.  Touches no device.
 */
int tli_d2t_from_strings(const char* bytes_d, const int64_t* offs_d, int32_t Vd, const char* bytes_t, const int64_t* offs_t,
                         int32_t Vt, int32_t* d2t_out, int32_t* out_num_shared);
/*
 * Host-only rehearsal of tli_build_map (intersection algorithm: everything it needs to know about T∩D): runs the
 * same argument checks and builds the same tables, touches no device, and then replays on the host what the
 * residual-scan kernel does with them, for both storage types and both drafter-row layouts: every index the kernel
 * would form must stay inside the tables and the LDS area it addresses, every staged slot must be written exactly
 * once, and every shared pair (target id, drafter id) must be visited exactly once with both sides matching d2t.
 *   out_num_shared   : receives |T∩D| (may be NULL)
 *   out_nparts [2]   : receives the number of parts the target chunks are cut into, per tli_dtype (may be NULL)
 *   out_failed_check : receives 0, or a number naming the check that failed (may be NULL)
 * Returns what tli_build_map would return for these arguments short of ALLOC/HIP, or TLI_ERR_INTERNAL if a
 * consistency check fails (a defect of the library, never of the input).
 */
int tli_map_dry_run(const int32_t* d2t_host, int32_t Vd, int32_t Vt, int32_t* out_num_shared, int32_t* out_nparts,
                    int32_t* out_failed_check);

/*
 * Bytes of device scratch that tli_draft_sample (with R <= B*K rows) and tli_verify (with these B, K)
 * need for vocabularies of these sizes.  The caller allocates it (256-byte aligned) and may reuse it
 * across calls on one stream.  Returns 0 on invalid arguments.
 */
size_t tli_workspace_bytes(int32_t B, int32_t K, int32_t Vt, int32_t Vd, tli_dtype dtype);

/*
 * Draft step of the intersection algorithm: for each of R independent drafter rows build
 * q'(x) = q(x) / sum_{t in T∩D} q(t) on shared ids (0 elsewhere) and draw one token from it.
 *   logits_d   dev [R rows, row_stride_elems apart, Vd valid entries each]
 *   u_draft    dev [R] fp32 in [0,1)
 *   tok_d      dev [R] int32  sampled drafter id            (-1 if the row is flagged)
 *   tok_t      dev [R] int32  the same token's target id    (-1 if the row is flagged)
 *   q_tok      dev [R] fp64   q'(tok_d)                      (may be NULL)
 *   lse_q      dev [R] fp64   log sum_{x shared} exp(logits_d[x]/temp_d): log q'(x) = logit/temp - lse_q
 *   row_status dev [R] int32  TLI_FLAG_NONFINITE / TLI_FLAG_ZERO_MASS, else 0
 *   io_stride  >= 1 : row r's entry of u_draft and of every output array is at index r * io_stride.
 *                     1 = packed arrays.  With io_stride = K and every pointer advanced by k, a call on
 *                     the B rows logits_d[:, k, :] (row_stride_elems = K*Vd) of a [B,K,Vd] tensor reads
 *                     and fills column k of [B,K] arrays: the shape of the drafting loop, one call after
 *                     each drafter forward, whose results tli_verify then takes as they are.
 * Unshared drafter logits are never inspected.
 * The draw is the ascending inverse CDF, min{x : C_x > u * C_last}, with the weights of a row's ids formed in fp32
 * relative to the row's largest: an id whose weight lies more than 2^120 below it is not drawn (u = 0 returns the
 * first id above that floor; together the ids below it hold less than 2^-100 of the row).
 */
int tli_draft_sample(const tli_map* map, const void* logits_d, tli_dtype dtype, int64_t row_stride_elems,
                     int32_t R, float temp_d, const float* u_draft, int32_t* tok_d, int32_t* tok_t,
                     double* q_tok, double* lse_q, int32_t* row_status, int64_t io_stride, void* workspace,
                     size_t workspace_bytes, void* hip_stream);

/*
 * Verification step (standard speculative decoding run with p and q'): every position k tests its
 * draft d_k with "accept iff u_acc * q'_k(d_k) < p_k(d_k)" (probability min(1, p/q')); n_accepted is
 * the length of the all-accept prefix; the extra token comes from the residual
 * norm(max(0, p_j - q'_j)) of the first rejected position j, or from p_{K+1} if nothing was rejected.
 *   logits_t   dev [B, K+1, Vt] dense      logits_d dev [B, K, Vd] dense
 *   tok_d      dev [B,K] int32 draft ids in DRAFTER id space (as returned by tli_draft_sample)
 *   lse_q      dev [B,K] fp64  as returned by tli_draft_sample for the same rows, or NULL: the library
 *                              then recomputes it with one extra scan of the drafter rows (K*Vd more
 *                              logits read per sequence)
 *   u_acc      dev [B,K] fp32, u_fin dev [B] fp32
 *   n_accepted dev [B]     int32
 *   out_tok    dev [B,K+1] int32 : n_accepted target ids, then the extra token, then -1 padding
 *   accept     dev [B,K]   uint8 : outcome of each position's own test (may be NULL)
 *   p_tok,q_tok dev [B,K]  fp64  : p_k(d_k), q'_k(d_k)                    (may be NULL)
 *   lse_p      dev [B,K+1] fp64  : log-normalisers of the target rows; entry K is NaN unless the
 *                                  bonus row was used (may be NULL)
 *   seq_status dev [B]     int32 : TLI_FLAG_* bits.  A draft id that is -1, out of range or unshared is
 *                                  rejected with q' = 0 (BAD_DRAFT): the extra token is then drawn from
 *                                  p_j itself.  NONFINITE sequences return n_accepted 0, out_tok -1.
 */
int tli_verify(const tli_map* map, const void* logits_t, const void* logits_d, tli_dtype dtype, int32_t B,
               int32_t K, float temp_t, float temp_d, const int32_t* tok_d, const double* lse_q,
               const float* u_acc, const float* u_fin, int32_t* n_accepted, int32_t* out_tok,
               uint8_t* accept, double* p_tok, double* q_tok, double* lse_p, int32_t* seq_status,
               void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * tli_verify for callers that cannot allocate device memory or pass a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs and kernels as tli_verify, without
 * the workspace: the scratch is a fixed array inside the library's device code, tli_verify_static_max_bytes() =
 * 8 MiB on every GPU the library runs on, held until the process ends.  The call allocates nothing and only
 * enqueues kernels on the stream (the array's device address is looked up when a map is built on the device).
 *   TLI_ERR_TOO_LARGE   : tli_workspace_bytes(B, K, Vt, Vd, dtype) exceeds the fixed scratch; nothing was enqueued
 *                         (the large-vocabulary batch B=256, K=8, Vt=256000, Vd=128256 in bf16 needs 3.6 MB)
 *   TLI_ERR_INVALID_ARG : also when the current device is not the one the map was built on
 * All calls on one GPU share that GPU's array: two calls whose kernels may overlap (different streams, or a graph
 * replayed beside an eager call) race on it; calls on one stream are ordered and safe.  Nothing in the scratch has
 * to start at zero, so the previous call's contents do no harm.
 */
size_t tli_verify_static_max_bytes(void);
int tli_verify_static(const tli_map* map, const void* logits_t, const void* logits_d, tli_dtype dtype, int32_t B,
                      int32_t K, float temp_t, float temp_d, const int32_t* tok_d, const double* lse_q,
                      const float* u_acc, const float* u_fin, int32_t* n_accepted, int32_t* out_tok,
                      uint8_t* accept, double* p_tok, double* q_tok, double* lse_p, int32_t* seq_status,
                      void* hip_stream);

/*
 * Compact drafter layout, for a drafter whose output head is pruned to the shared tokens (the intersection
 * algorithm only ever needs q on T∩D): a row holds |T∩D| logits, entry r = the logit of the shared token of
 * rank r, ranks ascending with the drafter id.  Same semantics and outputs as tli_draft_sample / tli_verify
 * (tok_d stays a DRAFTER id); no mask is read and no gather is needed to stage a row.
 *   logits_c dev [rows, row stride apart (a multiple of 4 fp32 / 8 bf16, >= |T∩D|), |T∩D| valid entries]
 *            tli_verify_compact: rows of sequence b, position k at (b*K + k) * c_row_stride_elems.
 */
int tli_draft_sample_compact(const tli_map* map, const void* logits_c, tli_dtype dtype, int64_t row_stride_elems,
                             int32_t R, float temp_d, const float* u_draft, int32_t* tok_d, int32_t* tok_t,
                             double* q_tok, double* lse_q, int32_t* row_status, int64_t io_stride, void* workspace,
                             size_t workspace_bytes, void* hip_stream);
int tli_verify_compact(const tli_map* map, const void* logits_t, const void* logits_c, int64_t c_row_stride_elems,
                       tli_dtype dtype, int32_t B, int32_t K, float temp_t, float temp_d, const int32_t* tok_d,
                       const double* lse_q, const float* u_acc, const float* u_fin, int32_t* n_accepted,
                       int32_t* out_tok, uint8_t* accept, double* p_tok, double* q_tok, double* lse_p,
                       int32_t* seq_status, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * ---- The neighbouring token-level steps of the paper, on the same rows -------------------------------
 *
 * The "union" algorithm (section "Motivating Examples", the simple union strategy: p and q are extended by
 * zeros to T ∪ D and standard speculative decoding runs unchanged).  Same arguments and outputs as
 * tli_draft_sample / tli_verify, with these differences: drafts are drawn from q = softmax over ALL of D;
 * tok_t is -1 for a token outside T; lse_q is the normaliser over all of D (NULL in the verify call: one
 * unmasked scan recomputes it); a draft outside T is a legal draft that the target rejects for every u
 * (p = 0), and the residual after it still subtracts q on the shared ids; BAD_DRAFT only marks ids outside
 * [0, Vd); every drafter logit takes part, so NaN/+inf anywhere in a drafter row flags it.
 */
int tli_union_draft_sample(const tli_map* map, const void* logits_d, tli_dtype dtype, int64_t row_stride_elems,
                           int32_t R, float temp_d, const float* u_draft, int32_t* tok_d, int32_t* tok_t,
                           double* q_tok, double* lse_q, int32_t* row_status, int64_t io_stride, void* workspace,
                           size_t workspace_bytes, void* hip_stream);
int tli_union_verify(const tli_map* map, const void* logits_t, const void* logits_d, tli_dtype dtype, int32_t B,
                     int32_t K, float temp_t, float temp_d, const int32_t* tok_d, const double* lse_q,
                     const float* u_acc, const float* u_fin, int32_t* n_accepted, int32_t* out_tok,
                     uint8_t* accept, double* p_tok, double* q_tok, double* lse_p, int32_t* seq_status,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Expected acceptance rate of one draft token at every position (the paper's table of expected acceptance
 * rates; the theorem on the intersection algorithm states alpha_union <= alpha_tli):
 *   alpha_union[b,k] = sum_{t in T∩D} min{p_k(t), q_k(t)}
 *   alpha_tli[b,k]   = sum_{t in T∩D} min{p_k(t), q_k(t) / sum_{x in T∩D} q_k(x)}
 *   logits_t dev [B,K+1,Vt] (row K of a sequence is not used), logits_d dev [B,K,Vd], both dense
 *   alpha_tli, alpha_union dev [B,K] fp64; pos_status dev [B,K] int32: NONFINITE (a target logit or ANY drafter
 *   logit of the position is NaN/+inf: both rates NaN) or ZERO_MASS (no drafter mass on the shared ids: both 0).
 * Both rates are good to 1e-5 relative at any size an fp64 number holds: positions whose rates come out below 2^-24
 * from the fp32 terms are summed a second time with fp64 exponent arguments and exactly scaled terms.
 * Scratch: tli_acceptance_rates_workspace_bytes (it depends on the map).
 */
size_t tli_acceptance_rates_workspace_bytes(const tli_map* map, int32_t B, int32_t K, tli_dtype dtype);
int tli_acceptance_rates(const tli_map* map, const void* logits_t, const void* logits_d, tli_dtype dtype, int32_t B,
                         int32_t K, float temp_t, float temp_d, double* alpha_tli, double* alpha_union,
                         int32_t* pos_status, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * One token from each of R rows of any vocabulary (no map): tok[r] ~ softmax(logits_r / temp) by the ascending
 * inverse CDF with u[r]; temp == 0 takes the argmax instead (largest logit, lowest id among equal ones; u may
 * then be NULL) -- the paper runs its exact-matching method at temperature zero.
 *   logits dev [R rows, row_stride_elems apart, V valid entries], u dev fp32, tok dev int32 (-1 if flagged),
 *   p_tok dev fp64 probability of the returned token (1 at temp 0; may be NULL), lse dev fp64 log-normaliser
 *   (NaN at temp 0; may be NULL), row_status dev int32 (NONFINITE / ZERO_MASS), io_stride as in tli_draft_sample.
 * Scratch: tli_sample_rows_workspace_bytes(R, V, dtype).
 */
size_t tli_sample_rows_workspace_bytes(int32_t R, int32_t V, tli_dtype dtype);
int tli_sample_rows(const void* logits, tli_dtype dtype, int64_t row_stride_elems, int32_t R, int32_t V, float temp,
                    const float* u, int32_t* tok, double* p_tok, double* lse, int32_t* row_status, int64_t io_stride,
                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Draft step of TLI at temperature zero: tok_d[r] = argmax of drafter row r over the SHARED ids (lowest id on
 * ties), tok_t = its target id; rows whose shared logits hold NaN/+inf or are all -inf are flagged and return -1.
 * Scratch: tli_workspace_bytes covers R <= B*K rows.
 */
int tli_greedy_draft(const tli_map* map, const void* logits_d, tli_dtype dtype, int64_t row_stride_elems, int32_t R,
                     int32_t* tok_d, int32_t* tok_t, int32_t* row_status, int64_t io_stride, void* workspace,
                     size_t workspace_bytes, void* hip_stream);

/*
 * Data-parallel tail of string-level exact matching (section "String-Level Exact Match", the steps after the
 * target forward): one token t'_j is drawn from each of the m+1 target rows (temp_t == 0: argmax), j* is the
 * first position where it differs from the re-tokenised draft, and draft_1..draft_{j*-1}, t'_{j*} are returned.
 *   logits_t dev [B, m+1, Vt] dense; draft_t dev [B, m] int32 target ids (negative = no draft token there);
 *   u dev [B, m+1] fp32 (may be NULL at temp_t == 0); n_accepted dev [B] = j* - 1; out_tok dev [B, m+1] (-1
 *   padded); tgt_tok dev [B, m+1] every t'_j; seq_status dev [B]: NONFINITE / ZERO_MASS if any of the m+1 rows is
 *   flagged (then n_accepted = 0 and out_tok = -1).  1 <= m < 64.
 * With temp_t == 0 and draft_t = the tok_t of tli_greedy_draft this is TLI's verification at temperature zero:
 * a draft is accepted iff it is the target's argmax, the extra token is the argmax of the first rejected row.
 * Scratch: tli_exact_match_workspace_bytes.
 */
size_t tli_exact_match_workspace_bytes(int32_t B, int32_t m, int32_t Vt, tli_dtype dtype);
int tli_exact_match_verify(const void* logits_t, tli_dtype dtype, int32_t B, int32_t m, int32_t Vt, float temp_t,
                           const int32_t* draft_t, const float* u, int32_t* n_accepted, int32_t* out_tok,
                           int32_t* tgt_tok, int32_t* seq_status, void* workspace, size_t workspace_bytes,
                           void* hip_stream);

/*
 * Logit warpers ahead of the softmax (the standard serving knobs; the paper itself samples at plain temperature
 * or temperature zero).  Both are thresholds on the logit VALUE, so equal logits are kept or dropped together:
 *   top_k > 0 : keep the logits >= the k-th largest competing logit (more than k survive on ties);
 *   top_p < 1 : on what survived top-k (renormalised at `temp`), keep x iff the probability mass of the strictly
 *               larger logits is < top_p (the smallest top set reaching top_p; the largest logit always survives).
 * logits_out receives the rows with every dropped logit set to -inf (same dtype; it may alias `logits`), so every
 * other entry point runs unchanged on warped rows.  logits_out = NULL (then kept must be NULL and thr must not):
 * no rewrite, only the thresholds -- thr is then the lowest value kept (-inf if no warper is active for the row) --
 * for tli_sample_rows_warped / tli_draft_sample_warped, which read the rows as they are.  With a map only the shared drafter ids compete (V must be Vd)
 * and unshared ids are dropped: the warped adjusted drafter of the intersection algorithm.
 *   logits dev [R rows, row_stride_elems apart, V valid], logits_out dev [R rows, out_stride_elems apart]
 *   thr dev [R] fp32: the threshold (-inf if nothing was dropped, NaN if the row is flagged); may be NULL
 *   kept dev [R] int32: number of surviving ids; may be NULL.  row_status dev [R]: NONFINITE / ZERO_MASS (such rows
 *   come out all -inf).
 * One workgroup per row; top-k 50 + top-p 0.9 on two-digit (bf16) keys takes two sweeps of the rows and the
 * rewrite: built for batches, not tuned for few rows.
 */
size_t tli_warp_workspace_bytes(int32_t R, int32_t V, tli_dtype dtype);
int tli_warp_rows(const tli_map* map, const void* logits, tli_dtype dtype, int64_t row_stride_elems, int32_t R,
                  int32_t V, float temp, int32_t top_k, float top_p, void* logits_out, int64_t out_stride_elems,
                  float* thr, int32_t* kept, int32_t* row_status, void* workspace, size_t workspace_bytes,
                  void* hip_stream);

/*
 * The same draws on rows that are warped by threshold instead of rewritten: only the logits >= thr[row] take part
 * (thr from tli_warp_rows with logits_out = NULL, on the same rows, at the same temperature; -inf = the row as it
 * is).  tli_sample_rows_warped is tli_sample_rows (temp > 0), tli_draft_sample_warped is tli_draft_sample (the
 * warped adjusted drafter: thr from tli_warp_rows with the map); p_tok / q_tok and lse are those of the warped,
 * renormalised distribution.  A row whose thr is NaN was flagged by the warp and is flagged here again.
 *   thr dev [R] fp32, entry of row r at index r * io_stride like the other per-row arrays.
 * Everything else as in the plain calls, the scratch included.
 */
int tli_sample_rows_warped(const void* logits, tli_dtype dtype, int64_t row_stride_elems, int32_t R, int32_t V, float temp,
                           const float* thr, const float* u, int32_t* tok, double* p_tok, double* lse,
                           int32_t* row_status, int64_t io_stride, void* workspace, size_t workspace_bytes,
                           void* hip_stream);
int tli_draft_sample_warped(const tli_map* map, const void* logits_d, tli_dtype dtype, int64_t row_stride_elems,
                            int32_t R, float temp_d, const float* thr, const float* u_draft, int32_t* tok_d,
                            int32_t* tok_t, double* q_tok, double* lse_q, int32_t* row_status, int64_t io_stride,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/* Human-readable name of a tli_status value. */
const char* tli_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* TLI_H */
