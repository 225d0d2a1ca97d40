/*
 * mtp_draft.h - C ABI of the MI355X (gfx950) FastMTP draft library.
 *
 * The library runs the drafting phase of FastMTP (arXiv 2509.18362, Sec. 2.3): K recursive
 * applications of ONE multi-token-prediction head whose weights are shared by all draft depths
 * (Sec. 2.1 "Architecture Design"), with the compressed output head of Sec. 2.2 / Eq. (3), followed
 * by sequential greedy acceptance against the target model's tokens (Sec. 2.3 "Verification phase").
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the current device, owned by the caller; "host"
 *     pointers are ordinary host memory.  The library allocates no device memory of its own: all
 *     scratch lives in the caller's workspace.
 *   - bf16 tensors are 16-bit brain-float bit patterns; matrices are row-major [out][in].
 *   - Every device pointer must be 16-byte aligned.
 *   - Work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = default stream) and the
 *     calls return without waiting for it, except where stated.
 *   - Every function returning int32_t returns MTP_OK (0) or a negative mtp_status; on a host-detected
 *     error nothing is enqueued and no output is written.
 *   - One handle must not be used from two streams at the same time: calls share its workspace.
 */
#ifndef MTP_DRAFT_H
#define MTP_DRAFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MTP_OK = 0,
    MTP_ERR_NULL = -1,         /* a required pointer is NULL                                  */
    MTP_ERR_ALIGN = -2,        /* a device pointer is not 16-byte aligned                     */
    MTP_ERR_CONFIG = -3,       /* unsupported or inconsistent mtp_config                      */
    MTP_ERR_BATCH = -4,        /* B outside [1, max_batch]                                    */
    MTP_ERR_STEPS = -5,        /* K outside [1, max_draft_steps]                              */
    MTP_ERR_SUBSET = -6,       /* subset_index out of range, or an invalid id list at init    */
    MTP_ERR_WORKSPACE = -7,    /* workspace too small                                         */
    MTP_ERR_HIP = -8,          /* a HIP runtime call failed                                   */
    MTP_ERR_KV_OVERFLOW = -9,  /* device saw kv_len[b] + K > kv_capacity (from mtp_poll_error)*/
    MTP_ERR_TOKEN_RANGE = -10, /* device saw an input token id outside [0, vocab_size)        */
    MTP_ERR_MODE = -11,        /* unknown rollback_mode / launch mode / timing mode           */
    MTP_ERR_TIMEOUT = -12      /* device: a grid barrier of the single-launch path timed out   */
} mtp_status;

/* Shape of the head (Sec. 3.1 "Model Configuration" for the 7B case) and limits of this handle. Host POD. */
typedef struct {
    int32_t d_model;         /* d; multiple of 32, 256..8192                                   */
    int32_t n_q_heads;       /* Hq                                                             */
    int32_t n_kv_heads;      /* Hkv; Hq / Hkv must be 1, 2, 4 or 8                             */
    int32_t head_dim;        /* hd; 64 or 128                                                  */
    int32_t d_ffn;           /* F, SwiGLU width; multiple of 8, at least 256; Hq*hd >= 256 too */
    int32_t vocab_size;      /* |V|                                                            */
    float rms_eps;           /* added to the mean square inside every RMSNorm                  */
    float rope_theta;        /* rotary base; pairs are (j, j + hd/2), the full head is rotated */
    int32_t max_batch;       /* largest B a call may pass; rows of the KV cache                */
    int32_t kv_capacity;     /* cache slots per (sequence, KV head)                            */
    int32_t max_draft_steps; /* largest K a call may pass                                      */
} mtp_config;

/* Device pointers to the head's tensors, all bf16.  The embedding table and the output head are the main
 * model's (Sec. 2.1: only the head is fine-tuned; Sec. 2.2: W is the main model's output head). */
typedef struct {
    const void *embed;   /* [V][d]                                                            */
    const void *lm_head; /* [V][d]  W of Eq. (3)                                              */
    const void *g_hnorm, *g_enorm, *g_attn_norm, *g_mlp_norm, *g_final_norm; /* RMSNorm gains, [d] each */
    const void *w_proj;  /* [d][2d]; columns 0..d-1 multiply the normalised hidden state,
                            columns d..2d-1 the normalised token embedding                    */
    const void *w_q;     /* [Hq*hd][d]                                                        */
    const void *w_k;     /* [Hkv*hd][d]                                                       */
    const void *w_v;     /* [Hkv*hd][d]                                                       */
    const void *b_q, *b_k, *b_v; /* [Hq*hd], [Hkv*hd], [Hkv*hd]; each may be NULL (no bias)  */
    const void *w_o;     /* [d][Hq*hd]                                                        */
    const void *w_gate;  /* [F][d]                                                            */
    const void *w_up;    /* [F][d]                                                            */
    const void *w_down;  /* [d][F]                                                            */
} mtp_weights;

typedef struct mtp_handle mtp_handle; /* host object: configuration, pointers, launch plan */

/* Text for a status code (static storage). */
const char *mtp_status_string(int32_t status);

/* Bytes of device workspace a handle with this configuration needs.  Host-only, touches no device.
 * Returns 0 if the configuration is not supported. */
size_t mtp_workspace_bytes(const mtp_config *cfg);

/*
 * Create a handle (Sec. 2.2: one id list V_high^(l) per language l; the caller picks one per call).
 *   n_subsets    number of compressed vocabularies (may be 0)
 *   subset_ids   host array of n_subsets device pointers; list s holds subset_sizes[s] int32 ids, strictly
 *                ascending, each in [0, vocab_size).  Row i of the compressed head is W[subset_ids[s][i], :].
 *   subset_sizes host array of n_subsets sizes, each in [1, vocab_size]
 *   workspace    device memory of at least mtp_workspace_bytes(cfg) bytes; the library keeps using it until
 *                mtp_draft_destroy and it must not be shared between handles that run concurrently
 * The id lists are copied to the host once and validated here (this call synchronises the device); the
 * device copies stay owned by the caller and must outlive the handle.  The workspace is zeroed.
 */
int32_t mtp_draft_init(mtp_handle **out, const mtp_config *cfg, const mtp_weights *weights, int32_t n_subsets,
                       const int32_t *const *subset_ids, const int32_t *subset_sizes, void *workspace,
                       size_t workspace_bytes);

/*
 * K recursive draft steps for B sequences (Sec. 2.3 "Drafting phase"), enqueued without any host wait.
 * Step k = 1..K for sequence b, at cache position p = kv_len[b] + k - 1:
 *   c   = [ RMSNorm(h; g_hnorm) ; RMSNorm(embed[x_k]; g_enorm) ]      h = hidden_in[b] at k = 1, else the
 *                                                                     previous step's output hidden state;
 *                                                                     x_1 = token_in[b], x_k = draft d_{k-1}
 *   x   = w_proj c
 *   y   = RMSNorm(x; g_attn_norm); q,k,v = w_q y + b_q, ...; rotary at position p on q and k;
 *         k and v are rounded to bf16 into cache slot p; attention of the Hq query heads over slots 0..p
 *   x1  = x + w_o attn;  x2 = x1 + w_down( silu(w_gate y2) * (w_up y2) ), y2 = RMSNorm(x1; g_mlp_norm)
 *   hh  = RMSNorm(x2; g_final_norm)                                   the step's output hidden state
 *   z_i = lm_head[ids[i], :] . hh  for i < n (Eq. (3));  d_k = ids[argmax_i z_i], lowest i on ties
 * All arithmetic is float32 on bf16 weights; activations entering a matrix product are carried as the sum of
 * two bf16 numbers (relative error below 2^-16).
 *
 *   subset_index  which id list to use; -1 = the full vocabulary (ids[i] = i, n = vocab_size)
 *   hidden_in     device [B][d] bf16: the target model's last hidden state per sequence
 *   token_in      device [B] int32: the verified token whose embedding pairs with hidden_in
 *   k_cache, v_cache  device [max_batch][Hkv][kv_capacity][hd] bf16; keys are stored after the rotary
 *                 embedding.  Slots kv_len[b] .. kv_len[b]+K-1 of sequence b are overwritten; others are only read
 *   kv_len        device [B] int32: valid entries per sequence before the call; not modified
 *   forced_tokens device [B][K-1] int32 or NULL: if given, x_k = forced_tokens[b][k-2] for k >= 2 instead of
 *                 the previous draft (teacher forcing as in Sec. 2.1 "Training Mechanism"; a test hook)
 *   draft_out     device [B][K] int32: drafted full-vocabulary ids
 *   logits_out    device [B][K][n] float32 or NULL
 *   hidden_out    device [B][K][d] float32 or NULL: hh of every step
 * Host-detected errors: NULL/misaligned pointers, B, K, subset_index.  Device-detected conditions set a sticky
 * error word read by mtp_poll_error: a sequence with kv_len[b] < 0 or kv_len[b] + K > kv_capacity writes draft id -1
 * at every step and its cache is left untouched; an input or forced token id outside [0, vocab_size) is replaced by
 * id 0 (so that every access stays in bounds) and the sequence goes on drafting and appending from that embedding.
 */
int32_t mtp_draft_steps(mtp_handle *h, int32_t B, int32_t K, int32_t subset_index, const void *hidden_in,
                        const int32_t *token_in, void *k_cache, void *v_cache, const int32_t *kv_len,
                        const int32_t *forced_tokens, int32_t *draft_out, float *logits_out, float *hidden_out,
                        void *hip_stream);

/*
 * Sequential greedy acceptance (Sec. 2.3 "Verification phase": accept until the first position where the draft
 * differs from the target model's token; Sec. 3.1: strict criteria, greedy decoding) and draft-cache bookkeeping.
 *   draft      device [B][K] int32   d_1..d_K (from mtp_draft_steps)
 *   target     device [B][K+1] int32 g_1..g_{K+1}: the target model's greedy tokens at the same positions,
 *              full-vocabulary ids (verification is not compressed, Sec. 2.2 last sentence)
 *   rollback_mode 0 = keep confirmed entries: cache slot kv_len+j-1 was built from input token x_j (x_1 verified,
 *                     x_j = d_{j-1}), so min(a+1, K) slots stay;  pending = 1 iff a == K (no entry for d_K yet)
 *                 1 = discard every slot written while drafting (kv_len unchanged), pending = 0
 *   kv_len     device [B] int32, in: length before drafting; out: length after rollback.  No cache bytes move.
 *   accept_len device [B] int32: a in [0, K]
 *   out_tokens device [B][K+1] int32: d_1..d_a, g_{a+1}, then -1
 *   pending    device [B] int32
 */
int32_t mtp_accept(mtp_handle *h, int32_t B, int32_t K, const int32_t *draft, const int32_t *target,
                   int32_t rollback_mode, int32_t *kv_len, int32_t *accept_len, int32_t *out_tokens,
                   int32_t *pending, void *hip_stream);

/*
 * The first draft step over a block of new positions (Sec. 2.3 "Drafting phase": step 1 runs over the shifted
 * prefix): the head is applied to every new position of every sequence with the TARGET model's hidden state of that
 * position and the token that follows it.  Position j of sequence b is written to cache slot kv_len[b] + j and attends
 * slots 0 .. kv_len[b] + j (causal inside the block).  The last position of a sequence yields its first draft token;
 * the others fill the head's KV cache, e.g. with the a + 1 tokens a verification has just confirmed, or a prompt.
 * Every weight is read once for all B * m_max (position, sequence) rows, and one attention launch serves all rows.
 *
 *   B, m_max     sequences and positions per sequence; B * m_max <= max_batch of mtp_draft_init (else
 *                MTP_ERR_BATCH)
 *   hidden_in    device [m_max][B][d] bf16     target hidden states, position-major
 *   tokens       device [m_max][B] int32       token paired with each hidden state
 *   ext_len      device [B] int32              new positions of each sequence, 0 .. m_max
 *   k_cache, v_cache  as for mtp_draft_steps; slots kv_len[b] .. kv_len[b] + ext_len[b] - 1 are written
 *   kv_len       device [B] int32              read, then advanced by ext_len[b] (on the stream, after the block)
 *   draft_out    device [m_max][B] int32       greedy token of every position; -1 at positions >= ext_len[b]
 *   logits_out   device [m_max][B][n] float or NULL;  hidden_out device [m_max][B][d] float or NULL (rows of
 *                positions >= ext_len[b] are unspecified)
 * A sequence whose block does not fit its cache (kv_len[b] + ext_len[b] > kv_capacity), or with a negative kv_len
 * or an ext_len outside 0 .. m_max, is left alone: drafts -1, cache and kv_len untouched, MTP_ERR_KV_OVERFLOW from
 * mtp_poll_error.  Always one launch per phase, whatever the launch mode.
 */
int32_t mtp_draft_extend(mtp_handle *h, int32_t B, int32_t m_max, int32_t subset_index, const void *hidden_in,
                         const int32_t *tokens, const int32_t *ext_len, void *k_cache, void *v_cache, int32_t *kv_len,
                         int32_t *draft_out, float *logits_out, float *hidden_out, void *hip_stream);

/*
 * mtp_draft_steps with one id list per sequence: several languages in one batch (Sec. 2.2: which language's list a
 * sequence uses follows from its context).  Every phase but the output head runs once for the whole batch; the output
 * head runs once per list, over the sequences that use it.
 *   seq_subset   HOST [B] int32   index of each sequence's list (-1 = full vocabulary).  Sequences that share a list
 *                                 must be adjacent (sort the batch by language); at most 16 different lists per call;
 *                                 otherwise MTP_ERR_SUBSET.  Read before the call returns.
 *   logits_out   device [B][K][n_max] float or NULL, n_max = the largest list of the call; a sequence with a shorter
 *                list fills its first n entries of every row.
 * Everything else as for mtp_draft_steps.  Always one launch per phase, whatever the launch mode.
 */
int32_t mtp_draft_steps_lists(mtp_handle *h, int32_t B, int32_t K, const int32_t *seq_subset, const void *hidden_in,
                              const int32_t *token_in, void *k_cache, void *v_cache, const int32_t *kv_len,
                              const int32_t *forced_tokens, int32_t *draft_out, float *logits_out, float *hidden_out,
                              void *hip_stream);

/*
 * Draft steps that start from the head's OWN output instead of the target model's hidden state (Sec. 2.3: from the
 * second step on the head consumes its own output hidden state and the previously drafted token).  After
 * mtp_draft_extend has produced the first draft token d_1 and the hidden state of a sequence's last new position,
 * this call drafts d_2 .. d_{K+1}: identical to mtp_draft_steps except that the first step reads
 *   own_hidden   device [B][d] float     the head's output (mtp_draft_extend's hidden_out row of the last live
 *                                        position of each sequence; copied into the workspace on the stream)
 * in place of hidden_in, and token_in [B] is the token drafted from it.  Everything else (cache slots kv_len[b] ..
 * kv_len[b] + K - 1, outputs, errors, launch modes) as for mtp_draft_steps.
 */
int32_t mtp_draft_continue(mtp_handle *h, int32_t B, int32_t K, int32_t subset_index, const float *own_hidden,
                           const int32_t *token_in, void *k_cache, void *v_cache, const int32_t *kv_len,
                           const int32_t *forced_tokens, int32_t *draft_out, float *logits_out, float *hidden_out,
                           void *hip_stream);

/*
 * Teacher-forced K-step forward of the shared head over all positions of one sequence and its weighted cross-entropy
 * (Sec. 2.1 "Training Mechanism" and "Training Objective", Eq. (1) and (2)); forward only, full vocabulary.
 * Step k at position i consumes (h^{k-1}_i, embedding of t_{i+k}) and is scored against t_{i+k+1}; h^0 is the main
 * model's hidden state, h^k the head's own output of step k.  Inside a step a position attends the step's own keys of
 * positions <= i.  CE_k = mean over the positions of logsumexp(z) - z[label]; loss = sum_k alpha_k CE_k with
 * alpha_k = beta^(k-1) / sum_j beta^(j-1).  Each step is the block-of-positions pipeline of mtp_draft_extend from an
 * empty cache (every weight read once per 64 positions), followed by a cross-entropy kernel.
 *   n_pos        positions i = 1 .. n_pos (= T - K of the paper); n_pos <= max_batch and <= kv_capacity of
 *                mtp_draft_init (else MTP_ERR_BATCH);  K: 1 .. 16;  beta > 0
 *   hidden_in    device [n_pos][d] bf16          the main model's hidden states
 *   tokens       device [n_pos + K + 1] int32    t_1 .. t_{n_pos+K+1}
 *   k_cache, v_cache  device, ONE sequence's cache [n_kv_heads][kv_capacity][head_dim] bf16: scratch, overwritten
 *   scratch      device, mtp_train_workspace_bytes(cfg, n_pos) bytes.  Its first n_pos * vocab_size floats hold the
 *                logits of a step, [n_pos][vocab_size]: after the call, those of step K
 *   loss_out     device [K + 1] float            CE_1 .. CE_K, then the weighted loss
 * A token id outside the vocabulary is reported by mtp_poll_error (MTP_ERR_TOKEN_RANGE) and treated as id 0.
 */
size_t mtp_train_workspace_bytes(const mtp_config *cfg, int32_t n_pos);
int32_t mtp_train_loss(mtp_handle *h, int32_t n_pos, int32_t K, float beta, const void *hidden_in,
                       const int32_t *tokens, void *k_cache, void *v_cache, void *scratch, size_t scratch_bytes,
                       float *loss_out, void *hip_stream);

/* Waits for `hip_stream`, then returns and clears the sticky device error word:
 * MTP_OK, MTP_ERR_KV_OVERFLOW or MTP_ERR_TOKEN_RANGE (or MTP_ERR_HIP). */
int32_t mtp_poll_error(mtp_handle *h, void *hip_stream);

/*
 * Timing of the most recent mtp_draft_steps call with HIP events recorded on that call's stream.
 *   mtp_set_timing(h, 0)      no events (default)
 *   mtp_set_timing(h, 1)      one event pair around everything the call enqueues
 *   mtp_set_timing(h, 2 + f)  one pair around each launch of phase f (0 proj, 1 qkv, 2 attn, 3 oproj, 4 gateup,
 *                             5 down, 6 lmhead); such calls use one launch per phase whatever the launch mode
 * mtp_last_draft_ms waits for the last event and returns milliseconds (mode 1: the call; mode 2 + f: the mean over
 * the call's K launches of phase f), or a negative value if nothing was recorded.
 */
int32_t mtp_set_timing(mtp_handle *h, int32_t mode);
float mtp_last_draft_ms(mtp_handle *h);

/*
 * How mtp_draft_steps enqueues its work.
 *   2 (default) automatic: mode 1 where it applies, mode 0 otherwise (also when the single launch is refused).
 *   0           one launch per phase.  One sequence: the row-streaming kernels, 7 launches per step plus one to publish
 *               the last draft id.  Two or more (also the rows of a block of positions): the batched kernels (every
 *               weight read once per pass of up to 64 sequences), one preparation launch per step, and one epilogue
 *               launch after each matrix phase whose reduction is split over workgroups (above 16 sequences).
 *               Matrices of 2 GiB or more: as mode 3.
 *   1           one sequence whose reduction lengths (d_model, n_q_heads * head_dim, d_ffn) are all at least 512: one
 *               launch of one workgroup per compute unit runs all phases of all K steps; its workgroups hand their
 *               results over element by element (every element carries a tag naming the call, step and phase that
 *               produced it, consumers poll for it), there are no grid barriers.  The workgroups wait for one another,
 *               so the launch needs every compute unit of the device to itself: do not overlap it with other kernels
 *               (other streams, other processes); a wait that does not end within ~2 s gives up and sets
 *               MTP_ERR_TIMEOUT.  Every other call: as mode 0.
 *   3           as mode 0, with the row-streaming kernels for up to four sequences (slower from the second
 *               sequence on; the form the library itself falls back to for matrices of 2 GiB or more).
 * Other values return MTP_ERR_MODE.  HIP-graph capture: mtp_draft_steps, mtp_draft_steps_lists, mtp_draft_extend,
 * mtp_draft_continue and mtp_accept only enqueue kernels (no memset or copy nodes except mtp_draft_continue's one
 * device-to-device copy, no synchronisation, no allocation) and may be captured on a non-default stream with timing
 * off; a captured call always takes one launch per phase (the single-launch kernel's tags count calls on the host,
 * which replays do not).  Results agree between the modes to rounding (one sequence: bit for bit between
 * modes 0 and 3; the single-launch kernel adds the two halves of the projection separately).
 */
int32_t mtp_set_launch_mode(mtp_handle *h, int32_t mode);

/*
 * Measurement aid: reads the first bytes / 16384 * 16384 bytes of buffer (device, 16-byte aligned, at least 16 KiB) once,
 * with the access pattern of the draft kernels' weight stream (one workgroup per compute unit, 1 KiB per wave and load,
 * sixteen loads in flight, non-temporal) and nothing else; out8 (device, 8 bytes) may receive a checksum.  Timed by the
 * caller (events on hip_stream), bytes / time is the streaming-read rate this device sustains: the ceiling the
 * kernels' own rates are to be read against.  Stateless; nothing waits.
 */
int32_t mtp_stream_probe(const void *buffer, size_t bytes, void *out8, void *hip_stream);

/*
 * Diagnostics for the single-launch kernel of one sequence: device_buffer (device, int64, mtp_phase_trace_bytes(cfg)
 * bytes, or NULL to stop) receives 100 MHz wall-clock stamps of EVERY workgroup, laid out
 * [step][section 0..7][point 0..3][workgroup 0..W-1] with W = the device's compute-unit count: sections are the phases
 * of a draft step in order (0 projection, 1 q/k/v, 2 attention, 3 output projection, 4 gate/up, 5 down, 6 output head,
 * 7 unused); points: 0 the section's first weights have been requested, 1 its input is available (the hand-over from
 * the phase before has completed), 2 the input is staged in LDS, 3 its results are stored.
 */
size_t mtp_phase_trace_bytes(const mtp_config *cfg);
int32_t mtp_set_phase_trace(mtp_handle *h, void *device_buffer);

/*
 * The high-frequency id list of one language from a token stream (Sec. 2.2: the subsets come from token statistics
 * over a corpus of that language; Eq. (3) gathers the output head's rows with them): occurrence counts per id, the n ids
 * with the largest counts (equal counts: the lower id first), written in ascending id order - the format
 * mtp_draft_init takes.  Stateless: no handle; everything is enqueued on hip_stream and nothing waits.
 *   tokens       device [n_tokens] int32     ids; values outside [0, vocab_size) are skipped and counted (may be
 *                                            NULL when n_tokens is 0)
 *   n_tokens     0 .. 2^31 - 1;  n: 0 .. vocab_size (else MTP_ERR_CONFIG)
 *   workspace    device, mtp_subset_workspace_bytes(vocab_size) bytes, owned by the caller; holds the counts, the
 *                selection state and one 160 KB copy of the counting kernel's bins per workgroup (41 MB in all)
 *   ids_out      device [n] int32            the list, ascending
 *   counts_out   device [vocab_size] int32 or NULL;  invalid_out device [1] int32 or NULL (skipped ids)
 * All device pointers 16-byte aligned.
 */
size_t mtp_subset_workspace_bytes(int32_t vocab_size);
int32_t mtp_subset_build(const int32_t *tokens, int64_t n_tokens, int32_t vocab_size, int32_t n, void *workspace,
                         size_t workspace_bytes, int32_t *ids_out, int32_t *counts_out, int32_t *invalid_out,
                         void *hip_stream);

/*
 * mtp_subset_build for callers that cannot allocate device memory and have no workspace to hand over (code under
 * HIP-graph capture, tight serving loops, harnesses that forbid hipMalloc): the counts and the selection state live in
 * an array built into the library's device image instead of a caller's workspace.  Same arguments (minus the
 * workspace), same results.  Calls no hipMalloc/hipFree and no allocating routine.
 *   vocab_size   at most mtp_subset_static_max_vocab() (262144 ids: the array is 1 MiB + 26 KB per GPU, held until
 *                the process ends); larger vocabularies return MTP_ERR_WORKSPACE with a message on stderr
 * The array has no room for the per-workgroup copies of the bins, so the counting kernel adds its bins to the counts
 * with atomics instead: about twice the time of mtp_subset_build on a stream of 2^26 tokens.
 * Every call on a GPU uses that GPU's one array (its contents are cleared at the start of each call): calls that
 * overlap on one GPU - different streams, or graphs replayed concurrently - race and must be serialised by the
 * caller.  The first call on a device looks the array's address up (a host-side query, no allocation).
 */
int32_t mtp_subset_static_max_vocab(void);
int32_t mtp_subset_build_static(const int32_t *tokens, int64_t n_tokens, int32_t vocab_size, int32_t n,
                                int32_t *ids_out, int32_t *counts_out, int32_t *invalid_out, void *hip_stream);

/* Frees the host object.  Device memory stays with the caller. */
void mtp_draft_destroy(mtp_handle *h);

#ifdef __cplusplus
}
#endif
#endif /* MTP_DRAFT_H */
