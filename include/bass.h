/*
 * bass.h -- C ABI of the BASS verification step for AMD MI355X (gfx950).
 *
 * BASS = batched speculative sampling: B sequences are verified at once by the main
 * model; every sequence brings its own number of draft query tokens and its own,
 * differently long KV cache (ragged K, V, P tensors), then per-sequence
 * speculative-sampling acceptance decides how many drafts are kept.
 *
 * Conventions for every call
 *   - Pointers are DEVICE pointers unless a parameter says "host".  They are borrowed:
 *     the library never frees or retains them.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work; they never synchronise and never allocate.
 *   - Return value: BASS_OK (0) or a negative error found on the host BEFORE anything is
 *     enqueued (see the enum).  Errors that depend on device data (a length out of range,
 *     a token id >= V) cannot be seen by the host: the kernels clamp to a safe range and
 *     OR a BASS_STATUS_* bit into `*dev_status` (int32 on the device, optional, may be
 *     NULL; the caller zeroes it).
 *   - One GPU; calls on the same stream are ordered; calls on different streams must not
 *     share a workspace.
 */
#ifndef BASS_H
#define BASS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  BASS_OK = 0,
  BASS_ERR_INVALID_ARG = -1,        /* null pointer, non-positive size, Hq % Hkv != 0 ...      */
  BASS_ERR_UNSUPPORTED = -2,        /* head size / dtype / row count outside what is compiled  */
  BASS_ERR_WORKSPACE_TOO_SMALL = -3,
  BASS_ERR_HIP = -4                 /* a launch failed; hipGetLastError() still holds the code */
};

enum {
  BASS_STATUS_LEN_CLAMPED = 1,      /* a ctx_len / draft_len / n_new / n_draft was out of range */
  BASS_STATUS_TOKEN_CLAMPED = 2,    /* a draft token id was outside [0, V)                      */
  BASS_STATUS_ZERO_MASS = 4,        /* a probability row had no mass to sample from             */
  BASS_STATUS_PLAN_MISMATCH = 8     /* the plan handed to an attention launch was made for another
                                       shape, work spread or kind of launch; nothing was computed */
};

/* BASS_DTYPE_INT8KV: Q, K_new, V_new are bf16; the caches hold INT8 codes with one fp32 scale per
 * token and kv head (the paper's appendix: dynamic per-head and per-token quantization of keys,
 * queries and values, the granularity of the inner-product dimension, so that the score product runs
 * in integer arithmetic).  Symmetric: amax = max_d |x_d|, code_d = rint(x_d * (127 / amax)) (one fp32
 * division, one fp32 product, round half to even), scale = amax / 127; a row of zeros has scale 0.
 * The attention kernels quantize every query row (one token, one query head) the same way on the fly;
 * the scores are the exact integer products of query and key codes times both scales, and the whole
 * attention is the one over the represented values code * scale of queries, keys and values. */
enum { BASS_DTYPE_BF16 = 0, BASS_DTYPE_FP32 = 1, BASS_DTYPE_INT8KV = 2 };

/* Shape of one attention layer's verification call. */
typedef struct bass_attn_desc {
  int32_t B;      /* sequences in the batch                                                     */
  int32_t kmax;   /* query-token slots per sequence (tensors are padded to kmax)                */
  int32_t Hq;     /* query heads                                                                */
  int32_t Hkv;    /* key/value heads, Hq % Hkv == 0 (query head h uses kv head h / (Hq/Hkv))     */
  int32_t D;      /* head size: 64 or 128 for bf16 / int8 caches; a multiple of 4 up to 256 for fp32 */
  int32_t Lcap;   /* cache capacity in tokens per sequence                                      */
  int32_t dtype;  /* BASS_DTYPE_*: element type of Q, K_new, V_new and of the caches; O is fp32  */
  float scale;    /* the 1/c of P = softmax(Q^T K / c) (Section 3.2); callers pass 1/sqrt(D)     */
} bass_attn_desc;

int bass_version(void);
const char* bass_status_string(int code); /* static string, host */

/* Bytes of ONE cache (K or V) for this shape.  The cache layout is owned by the library
 * (bf16 caches are stored in matrix-core fragment order); a cache is written only through
 * bass_kv_append and read back only through bass_kv_gather.  Returns 0 for a bad shape. */
size_t bass_kv_cache_bytes(const bass_attn_desc* desc);

/* Scratch bytes bass_verify_attention needs for this shape (split-context partial results
 * and one arrival counter per (sequence, kv head)).  Returns 0 for a bad shape.
 * The caller ZEROES the workspace once after allocating it; every successful call leaves
 * the counters at zero again, so the same workspace serves any number of calls (also of
 * other shapes that fit).  After a failed launch, zero it again. */
size_t bass_verify_attention_workspace_bytes(const bass_attn_desc* desc);

/*
 * Append this step's key/value rows to the per-sequence caches (Section 2.1: keys and
 * values of processed tokens are cached; Section 3.2: every sequence proceeds at its own
 * pace, so each has its own write offset; rows of rejected drafts are simply overwritten
 * by the next step).
 *   K_new, V_new [B, kmax, Hkv, D]  rows of the new tokens (desc->dtype)
 *   ctx_len      [B] int32          write offset (tokens already valid) of each sequence
 *   n_new        [B] int32          rows to write, 0..kmax
 * Row i < n_new[b] of sequence b becomes cache token ctx_len[b] + i.  Rows that would fall
 * outside [0, Lcap) are dropped and BASS_STATUS_LEN_CLAMPED is raised.  Also used to fill a
 * cache with a whole prompt (kmax = prompt length, ctx_len = 0).
 */
int bass_kv_append(const bass_attn_desc* desc, void* Kcache, void* Vcache, const void* K_new,
                   const void* V_new, const int32_t* ctx_len, const int32_t* n_new,
                   int32_t* dev_status, void* stream);

/*
 * INT8 caches only (desc->dtype == BASS_DTYPE_INT8KV): read the codes and scales of tokens
 * start[b] .. start[b]+n[b]-1 back in token-major order.
 *   K_codes, V_codes   [B, kmax, Hkv, D] int8 out
 *   K_scales, V_scales [B, kmax, Hkv] fp32 out
 * Rows beyond n[b] are left untouched.
 */
int bass_kv_gather_int8(const bass_attn_desc* desc, const void* Kcache, const void* Vcache,
                        int8_t* K_codes, int8_t* V_codes, float* K_scales, float* V_scales,
                        const int32_t* start, const int32_t* n, int32_t* dev_status, void* stream);

/*
 * Read cache rows back in token-major order (inverse of bass_kv_append; for tests and for
 * moving a sequence; bf16 and fp32 caches): K_out, V_out [B, kmax, Hkv, D] receive tokens
 * start[b] .. start[b]+n[b]-1 of sequence b; other rows are left untouched.
 */
int bass_kv_gather(const bass_attn_desc* desc, const void* Kcache, const void* Vcache, void* K_out,
                   void* V_out, const int32_t* start, const int32_t* n, int32_t* dev_status,
                   void* stream);

/*
 * Ragged verify attention (Section 3.2, attention flow: scores of the current tokens'
 * queries against the keys of all tokens processed so far, P = softmax(Q^T K / c), then
 * P times V; Section 2.2: the draft tokens are processed as incremental context encoding).
 *   Q         [B, kmax, Hq, D]   queries of the current tokens (desc->dtype)
 *   ctx_len   [B] int32          tokens cached BEFORE this step
 *   draft_len [B] int32          query tokens of this step, 0..kmax (0 = inactive sequence)
 *   O         [B, kmax, Hq, D]   fp32 output
 *   lse       [B, kmax, Hq]      fp32 natural-log softmax denominator (max included);
 *                                optional, may be NULL
 * Query i of sequence b attends to cache tokens j <= ctx_len[b] + i: all of the sequence's
 * own cache and, causally, the step's own tokens, whose K/V must already have been appended
 * at [ctx_len[b], ctx_len[b] + draft_len[b]).  Every other position -- another sequence's
 * tokens, padding, stale rows beyond the valid range -- has probability exactly zero, as
 * padded positions have in BASS-PAD; no work is spent on them, as in BASS-SPLIT.  Rows
 * i >= draft_len[b] of O and lse are written as 0.  ctx_len[b] = 0 is legal.
 * Lengths outside the cache are clamped (BASS_STATUS_LEN_CLAMPED).
 * bf16: kmax * (Hq/Hkv) <= 64.  `workspace` must hold at least
 * bass_verify_attention_workspace_bytes(desc) bytes, be 16-byte aligned and have been zeroed
 * once (see above).  One launch when a kv head has at most 16 query rows (kmax * Hq/Hkv <= 16): the
 * split-context reduction runs inside the same kernel; with more rows a second, chip-wide launch
 * merges the partial results.
 */
int bass_verify_attention(const bass_attn_desc* desc, const void* Q, const void* Kcache,
                          const void* Vcache, const int32_t* ctx_len, const int32_t* draft_len,
                          float* O, float* lse, void* workspace, size_t workspace_bytes,
                          int32_t* dev_status, void* stream);

/*
 * The paper's two ways of batching ragged attention (Section 3.2), as launch variants of the
 * same kernel, for comparison with bass_verify_attention; arguments and results as there.
 *
 * bass_verify_attention_pad (BASS-PAD): one launch in which every active sequence is
 * processed over max(padded_len, ctx_len[b] + draft_len[b]) cache positions (at most Lcap):
 * K, V and P are treated as padded to a common length, the padded positions are read, take
 * part in the products and get probability exactly zero.  With padded_len = the longest
 * sequence of the batch this is the paper's scheme; padded_len = 0 is bass_verify_attention.
 * (fp32 caches: padded positions are skipped, not read.)
 *
 * bass_verify_attention_split (BASS-SPLIT): one launch per sequence, each over that sequence's
 * own length; no wasted work, B launches.  The workspace of the whole batch is passed and shared.
 */
int bass_verify_attention_pad(const bass_attn_desc* desc, const void* Q, const void* Kcache,
                              const void* Vcache, const int32_t* ctx_len, const int32_t* draft_len,
                              int32_t padded_len, float* O, float* lse, void* workspace,
                              size_t workspace_bytes, int32_t* dev_status, void* stream);
int bass_verify_attention_split(const bass_attn_desc* desc, const void* Q, const void* Kcache,
                                const void* Vcache, const int32_t* ctx_len,
                                const int32_t* draft_len, float* O, float* lse, void* workspace,
                                size_t workspace_bytes, int32_t* dev_status, void* stream);

/*
 * bass_kv_append and bass_verify_attention in ONE call: appends rows i < draft_len[b] of K_new,
 * V_new [B, kmax, Hkv, D] at cache tokens ctx_len[b] + i, exactly as
 * bass_kv_append(desc, Kcache, Vcache, K_new, V_new, ctx_len, draft_len, ...) would, and computes
 * bass_verify_attention over the updated caches.  The valid tokens of the caches are identical to
 * those after the two separate calls (stale rows beyond a sequence's new length may differ); O and
 * lse agree with them up to rounding (the fused launch cuts the context at other points).  Rows of
 * sequences whose lengths had to be clamped are appended at the clamped positions.  Arguments as
 * in those calls.  bf16 and INT8 caches with kmax * D <= 2048 and fp32 caches append inside the
 * attention launch (INT8: the rows are quantized on the way, with the quantizer of bass_kv_append);
 * longer drafts run the append as a launch of its own inside this call.
 */
int bass_append_verify_attention(const bass_attn_desc* desc, const void* Q, const void* K_new,
                                 const void* V_new, void* Kcache, void* Vcache,
                                 const int32_t* ctx_len, const int32_t* draft_len, float* O,
                                 float* lse, void* workspace, size_t workspace_bytes,
                                 int32_t* dev_status, void* stream);

/*
 * A verification step runs the same ragged attention once per layer of the main model, and all layers
 * see the same lengths (Section 3.2: a sequence's length changes between steps, when its accepted
 * drafts are known, not inside one).  The division of the ragged work over the GPU is therefore made
 * once per step -- bass_attention_plan, one small launch -- and every layer's call takes the plan:
 * bass_verify_attention_planned starts streaming the caches a microsecond earlier than
 * bass_verify_attention / bass_append_verify_attention, which make a plan of their own inside the call.
 *
 * bass_attention_plan_bytes: size of a plan buffer for this shape (0 for a bad shape).
 * bass_attention_plan: writes the plan for ctx_len / draft_len [B] (device, read when the launch runs)
 *   into `plan` (device, 16-byte aligned, at least bass_attention_plan_bytes(desc) bytes; no need to clear
 *   it).  flags: BASS_PLAN_APPEND if the attention calls will bring K_new / V_new (the step's rows are then
 *   appended as in bass_append_verify_attention), 0 if they will not.  padded_len: as in
 *   bass_verify_attention_pad (0 = none; not together with BASS_PLAN_APPEND).  Lengths outside the cache
 *   are clamped as everywhere (BASS_STATUS_LEN_CLAMPED); the plan holds the clamped values.
 * bass_attention_plan_host: the same plan, byte for byte in every part a launch reads, computed on the
 *   HOST from HOST arrays into HOST memory (for callers that keep the lengths on the host and copy the
 *   plan up themselves, and for checking the planner without a GPU); host_status (optional) receives
 *   BASS_STATUS_LEN_CLAMPED.
 * bass_verify_attention_planned: the attention of one layer with the step's plan; arguments and results
 *   as in bass_verify_attention (K_new = V_new = NULL) or bass_append_verify_attention (both given), the
 *   lengths being those the plan was made from.  The plan must come from bass_attention_plan with the
 *   same descriptor, the matching flags and the same bass_set_attention_waves setting; a launch that
 *   finds anything else in `plan` computes nothing and raises BASS_STATUS_PLAN_MISMATCH.  A plan may be
 *   used by any number of calls; it is read only.
 */
enum { BASS_PLAN_APPEND = 1 };
size_t bass_attention_plan_bytes(const bass_attn_desc* desc);
int bass_attention_plan(const bass_attn_desc* desc, const int32_t* ctx_len, const int32_t* draft_len,
                        int32_t flags, int32_t padded_len, void* plan, size_t plan_bytes,
                        int32_t* dev_status, void* stream);
int bass_attention_plan_host(const bass_attn_desc* desc, const int32_t* ctx_len_host,
                             const int32_t* draft_len_host, int32_t flags, int32_t padded_len,
                             void* plan_host, size_t plan_bytes, int32_t* host_status);
int bass_verify_attention_planned(const bass_attn_desc* desc, const void* Q, const void* K_new,
                                  const void* V_new, void* Kcache, void* Vcache, const void* plan,
                                  float* O, float* lse, void* workspace, size_t workspace_bytes,
                                  int32_t* dev_status, void* stream);

/*
 * Speculative-sampling acceptance for the batch (Section 2.2: the number of accepted
 * drafts is decided from the main- and draft-model probabilities; on rejection a corrected
 * token is sampled from the main model's outputs; the procedure is equivalent to sampling
 * from the main model).
 *   p          [B, kmax+1, V] fp32  main-model probabilities; row i judges draft i, row
 *                                   n_draft[b] is the bonus row
 *   q          [B, kmax,   V] fp32  draft-model probabilities
 *   draft_tok  [B, kmax] int32      drafted token ids
 *   n_draft    [B] int32            drafts of each sequence, 0..kmax
 *   u          [B, kmax+1] fp32     uniforms in [0,1): u[b,i] judges draft i, u[b,kmax]
 *                                   drives the corrected / bonus draw
 *   n_accept   [B] int32 out        length of the accepted prefix
 *   next_token [B] int32 out        corrected token (after a rejection) or bonus token
 *   ctx_len    [B] int32 in/out     optional (may be NULL): += n_accept + 1
 * Rule, per sequence: draft i with token x is accepted iff u_i * q_i(x) < p_i(x), evaluated
 * exactly (fp64 product of fp32 values); the prefix stops at the first rejection.  The new
 * token is drawn by inverse CDF from max(p_n - q_n, 0) (one fp32 subtraction per entry) after
 * a rejection at position n, or from p_k after k acceptances, or from p_n if the residual has
 * no mass.  Weights are floor(min(w,1) * 2^44) as integers, T = (floor(u * 2^32) * sum) >> 32,
 * and the token is the first whose cumulative weight exceeds T, so the result does not
 * depend on summation order.  V <= 2^19.
 */
int bass_spec_accept(int32_t B, int32_t kmax, int32_t V, const float* p, const float* q,
                     const int32_t* draft_tok, const int32_t* n_draft, const float* u,
                     int32_t* n_accept, int32_t* next_token, int32_t* ctx_len,
                     int32_t* dev_status, void* stream);

/*
 * Logits front end: temperature, nucleus (top-p) filter and softmax, producing the probability
 * rows p and q that bass_spec_accept consumes (the paper's experiments use temperature 0.2 and
 * nucleus top-p 0.95: captions of the result tables in Section 4).
 *   logits [R, V] fp32 (device)   R rows, e.g. B * (kmax + 1) main-model or B * kmax draft-model rows
 *   probs  [R, V] fp32 (device)   out; may not alias logits
 * Per row: e_i = 2^((z_i - max z) * log2(e) / temperature); the tokens are ordered by decreasing
 * e_i, equal values by increasing token id; the shortest prefix whose mass reaches top_p of the
 * total is kept (the token that crosses top_p included; top_p >= 1 keeps every token); probs is
 * e_i / (kept mass) on kept tokens and 0 elsewhere.  Masses are compared as the integers
 * floor(e_i * 2^40) against ceil(top_p * their sum), so the kept set and the normaliser do not
 * depend on summation order and repeated calls give identical bits.  NaN logits get probability 0;
 * a row without any finite logit is written as zeros and raises BASS_STATUS_ZERO_MASS.
 * temperature > 0, top_p > 0, V <= 2^19; otherwise BASS_ERR_INVALID_ARG / BASS_ERR_UNSUPPORTED.
 */
int bass_warp_probs(int32_t R, int32_t V, const float* logits, float temperature, float top_p,
                    float* probs, int32_t* dev_status, void* stream);

/*
 * Logits front end and acceptance in one call: the result of bass_warp_probs on the main- and the
 * draft-model logits followed by bass_spec_accept on the rows it made (Section 2.2; temperature and
 * top-p as in the captions of Section 4's tables), without storing any probability row.  n_accept,
 * next_token, ctx_len and the status bits are identical, bit for bit, to those of the two calls.
 *   logits_main  [B, kmax+1, V] fp32 (device)  main-model logits; row i judges draft i
 *   logits_draft [B, kmax,   V] fp32 (device)  draft-model logits (may be NULL if kmax = 0)
 *   temperature, top_p                         as in bass_warp_probs
 *   draft_tok, n_draft, u, n_accept, next_token, ctx_len   as in bass_spec_accept
 *   workspace    device scratch of at least bass_warp_accept_workspace_bytes(B, kmax, V) bytes,
 *                256-byte aligned, contents irrelevant on entry (per-row summaries of the warp,
 *                partial sums of the draw); calls that share one workspace must not overlap
 * Two launches: one workgroup per row of logits, then several workgroups per sequence for the
 * accept tests and the draw.  temperature > 0, top_p > 0, V <= 2^19, B <= 65535; otherwise
 * BASS_ERR_INVALID_ARG / BASS_ERR_UNSUPPORTED.  bass_warp_accept_workspace_bytes returns 0 for
 * arguments the call would refuse.
 */
size_t bass_warp_accept_workspace_bytes(int32_t B, int32_t kmax, int32_t V);
int bass_warp_accept(int32_t B, int32_t kmax, int32_t V, const float* logits_main,
                     const float* logits_draft, float temperature, float top_p,
                     const int32_t* draft_tok, const int32_t* n_draft, const float* u,
                     int32_t* n_accept, int32_t* next_token, int32_t* ctx_len, void* workspace,
                     size_t workspace_bytes, int32_t* dev_status, void* stream);

/*
 * Draft-length heuristic (Algorithm 1 of the paper; HOST code, HOST pointers): picks the
 * uniform draft length of the next speculative step from the numbers of drafts the sequences
 * accepted in the last one.  If some sequence accepted all l_draft drafts the length grows by
 * l_incre (up to l_limit) and s is cleared; otherwise it shrinks by ceil(l_draft / l_mod) + s,
 * but not below 1 nor below the largest accepted count, and s is set to 1 (a consecutive
 * shrink is one larger).  The paper's constants: l0 = 7, l_incre = 2, l_mod = 10, l_limit = 32.
 *   state     in/out; initialise with bass_draft_len_init (l0 <= 0 selects the paper's 7)
 *   n_accept  [B] host array: accepted drafts per sequence (bass_spec_accept's n_accept)
 *   l_incre, l_mod, l_limit  <= 0 selects the paper's value
 * Returns the new draft length (also stored in state), or a negative BASS_ERR_* code.
 */
typedef struct bass_draft_len_state {
  int32_t l_draft; /* current draft length */
  int32_t s;       /* 1 after a step that shrank the length, else 0 */
} bass_draft_len_state;

void bass_draft_len_init(bass_draft_len_state* state, int32_t l0);
int32_t bass_next_draft_len(bass_draft_len_state* state, const int32_t* n_accept, int32_t B,
                            int32_t l_incre, int32_t l_mod, int32_t l_limit);

/*
 * Tuning knob (host state, process wide): number of wavefronts the attention kernels spread the
 * flattened (sequence, kv-head, context-block) work over.  Values are clamped to [64, 8192]; 0 restores
 * the defaults, which depend on the call: 768 with up to 16 query rows per kv head; with more, 1024 for
 * INT8 caches and 256 workgroups of four wavefronts for bf16 caches (a setting W gives W / 2 workgroups
 * there).  Returns the value in effect for the first of these cases.  (A launch of 768 wavefronts runs as 256 workgroups of three, one per compute
 * unit; every other count as workgroups of four.)
 */
int bass_set_attention_waves(int waves);

/*
 * bass_verify_attention for callers that cannot allocate device memory or keep a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Arguments and results as in
 * bass_verify_attention, without the workspace: the arrival counters, the plan and the partial results
 * live in a static device array of BASS_NOALLOC_SCRATCH_BYTES = 16 MiB inside the library (held
 * by every GPU the library runs on until the process ends).  The call allocates nothing and frees nothing.
 * Shapes whose scratch need -- 256-byte padded B*Hkv counters + the plan + (shares + B*Hkv) * kmax*(Hq/Hkv)
 * * (D+2) * 4 bytes of partial results, shares being the work spread in effect -- exceeds the array are
 * refused with BASS_ERR_WORKSPACE_TOO_SMALL before anything is enqueued (the benchmark configurations need
 * 3.5 to 10 MiB).  All calls on one GPU share that GPU's array, which keeps the last call's contents (every
 * call clears what must start at zero): calls that overlap in time on one GPU -- different streams,
 * different host threads -- race and must not be made; calls on one stream are ordered and safe.
 */
#define BASS_NOALLOC_SCRATCH_BYTES ((size_t)16 << 20)
int bass_verify_attention_noalloc(const bass_attn_desc* desc, const void* Q, const void* Kcache,
                                  const void* Vcache, const int32_t* ctx_len, const int32_t* draft_len,
                                  float* O, float* lse, int32_t* dev_status, void* stream);

/*
 * Measurement aid (not part of the verification step): a plain streaming read of the first
 * floor(bytes_each / 8192) * 8192 bytes of K and of V with the access pattern of the attention kernel
 * (`waves` wavefronts, each a contiguous share of 8 KiB K blocks and 8 KiB V blocks, 1 KiB per
 * wavefront load instruction, non-temporal, two blocks in flight, the workgroup shape of an attention
 * launch of as many wavefronts) and no arithmetic: the time the memory
 * system needs for the bytes of an attention launch, which is what Section 3.2 says the step is bound by.
 * K, V: device, 16-byte aligned; waves: a multiple of 4 in [4, 8192]; sink: device, >= waves words, or
 * NULL.  Returns the bytes read per launch (K and V together), or a negative BASS_ERR_* code.
 */
int64_t bass_bench_stream_read(const void* K, const void* V, size_t bytes_each, int32_t waves,
                               uint32_t* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BASS_H */
