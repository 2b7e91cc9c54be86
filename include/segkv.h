/*
 * libsegkv -- fused decode-step scaled-dot-product attention over a segment
 * KV cache, for AMD MI355X (gfx950).  C ABI.
 *
 * Method: arxiv 2401.05391.  The KV cache of a batch of B requests decoded
 * with beam width W is kept in two segments (Section 3.2):
 *   prompt   K and V  [B, Lp, Hkv, D]        fp16, batch first, one copy per
 *                                            request shared by its W beams;
 *   response K and V  [Tcap, B*W, Hkv, D]    fp16, sequence first,
 *                                            pre-allocated, rows 0..T-1 valid.
 * One decode step of one layer (Section 3.1, decoding phase; Section 3.3)
 * writes the step's K/V into response row T-1 and computes, for each of the
 * B*W beam rows and Hq query heads, softmax attention of the single query
 * token over the Lp prompt keys of its request and over the T response rows on
 * its own beam lineage (the "index select" of Section 3.3, fused).
 *
 * Conventions common to all entry points
 *   - Every tensor pointer is a DEVICE pointer to memory owned by the caller,
 *     dense, row-major in the shape given, 16-byte aligned.  The library never
 *     allocates, frees or retains caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls enqueue work on it and return without synchronising.
 *   - `segkv_dims*` is a HOST pointer, read during the call only.
 *   - Return value: SEGKV_OK (0), or a negative segkv_status; on error nothing
 *     has been enqueued.  Faults raised later by the device (for example from
 *     parent entries outside [0, beam)) are not reported by the call.
 *   - Beam rows of request b are rows b*beam .. b*beam+beam-1.  Query head hq
 *     reads KV head hq / (Hq/Hkv).
 */
#ifndef SEGKV_H
#define SEGKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t B;     /* requests, >= 1                                            */
    int32_t beam;  /* beam width W, 1..8                                        */
    int32_t Hq;    /* query heads, multiple of Hkv                              */
    int32_t Hkv;   /* key/value heads                                           */
    int32_t D;     /* head dimension: 64, 128 or 256                            */
    int32_t Lp;    /* prompt length, >= 0 (0: response segment only)            */
    int32_t T;     /* valid response rows INCLUDING the current step, 1..Tcap   */
    int32_t Tcap;  /* allocated rows of resp_k / resp_v                         */
} segkv_dims;

typedef enum {
    SEGKV_OK = 0,
    SEGKV_INVALID_ARG = -1,         /* null required pointer, bad dimension, t out of range,
                                       only one of k_new / v_new given                        */
    SEGKV_UNSUPPORTED = -2,         /* D or beam outside the compiled variants                */
    SEGKV_MISALIGNED = -3,          /* a tensor base is not 16-byte aligned                   */
    SEGKV_WORKSPACE_TOO_SMALL = -4, /* workspace_bytes < segkv_workspace_bytes(d)             */
    SEGKV_HIP_ERROR = -5,           /* a launch was rejected by the HIP runtime               */
    SEGKV_STATIC_SCRATCH_EXCEEDED = -6 /* segkv_sdpa_decode_static_scratch only: the dimensions
                                       need more than SEGKV_STATIC_SCRATCH_BYTES of scratch   */
} segkv_status;

/*
 * Append (Section 3.1: the step's Key_t / Value_t are kept in their row of the
 * pre-allocated sequence-first response buffers, replacing the concatenation).
 * Copies k_new, v_new [B*beam, Hkv, D] into row t of resp_k, resp_v
 * [Tcap, B*beam, Hkv, D].  0 <= t < Tcap.  d->T, d->Lp and d->Hq are not used.
 */
int segkv_append_kv(void* resp_k, void* resp_v,
                    const void* k_new, const void* v_new,
                    int32_t t, const segkv_dims* d, void* stream);

/*
 * Producer step of a decode step (Section 3.1: RoPE follows the QKV projection
 * and is fused to a single kernel; the step's Key_t / Value_t are kept in their
 * row of the response buffers).  One launch that
 *   - rotates q [B*beam, Hq, D] IN PLACE,
 *   - writes the rotated k_new [B*beam, Hkv, D] to row t of resp_k,
 *   - copies v_new [B*beam, Hkv, D] to row t of resp_v,
 * after which segkv_sdpa_decode is called with T = t + 1 and k_new = v_new = NULL.
 * Rotary embedding as published (RoFormer): theta_i = rope_base^(-2i/rotary_dim),
 * i < rotary_dim/2; the pair (a, b) at position pos becomes
 * (a cos(pos theta_i) - b sin(pos theta_i), b cos(pos theta_i) + a sin(pos theta_i)).
 * The pair is elements (i, i + rotary_dim/2) of a head vector when interleaved
 * == 0 (Llama2) and (2i, 2i+1) otherwise (GPT-J); elements >= rotary_dim pass
 * through.  rotary_dim <= min(D, 256), a multiple of 16 (of 8 when interleaved);
 * 0 makes this a plain append.
 *   positions   NULL: every row sits at position d->Lp + t (prompt token i at i,
 *               response step s at Lp + s, as for the ALiBi bias); else [B] int32
 *               device array with the position of each request's current token.
 * Angles are evaluated in double precision, the rotation in fp32, results are
 * rounded to fp16 (round to nearest even).  Uses d->B, beam, Hq, Hkv, D, Lp,
 * Tcap; 0 <= t < Tcap.
 */
int segkv_rope_append(void* q, const void* k_new, const void* v_new,
                      void* resp_k, void* resp_v, const int32_t* positions,
                      int32_t t, float rope_base, int32_t rotary_dim, int32_t interleaved,
                      const segkv_dims* d, void* stream);

/*
 * Fused decode-step attention (Section 3.3).
 *   out           [B*beam, Hq, D] fp16, written.
 *   q             [B*beam, Hq, D] fp16.
 *   prompt_k/v    [B, Lp, Hkv, D] fp16 (may be NULL when Lp == 0).
 *   resp_k/v      [Tcap, B*beam, Hkv, D] fp16.  Rows >= T are never read.
 *   parent        [T, B*beam] int32 beam-search back pointers, request-local:
 *                 parent[s][b*beam+j] in [0, beam) is the slot at step s-1 of the
 *                 hypothesis that slot j extends at step s.  Row 0 (which points
 *                 into the shared prompt) is ignored.  The library resolves the
 *                 lineage itself: slot_at[T-1] = j, slot_at[s-1] =
 *                 parent[s][b*beam + slot_at[s]].  May be NULL when beam == 1.
 *                 Entries are not range-checked on the device.
 *   k_new, v_new  both NULL, or both [B*beam, Hkv, D] fp16: the current step's
 *                 K/V.  If given they are written to row T-1 of resp_k/resp_v
 *                 by this call and used as that row; the previous content of
 *                 row T-1 is never read.  Result and final buffer contents equal
 *                 segkv_append_kv(..., t = T-1) followed by this call with NULLs.
 *   alibi_slopes  NULL, or [Hq] fp32: slope[hq] * key_position is added to the
 *                 scaled logit (prompt key i has position i, response step s has
 *                 position Lp+s).  Not multiplied by `scale`.
 *   anc_out       NULL, or [T, B*beam] int32, written with the resolved slot of
 *                 every (step, beam row) exactly as the kernel used it.
 *   workspace     device scratch of at least segkv_workspace_bytes(d) bytes,
 *                 need not be initialised; contents undefined afterwards.
 *   scale         logit scale, normally 1/sqrt(D).
 * The single query token sits at position Lp+T-1 and attends to all Lp+T keys.
 * Arithmetic: fp16 inputs, fp32 logits, softmax statistics and accumulation,
 * output rounded to fp16 (round to nearest even).
 * Concurrent calls must not share `workspace`, nor write the tensors read here.
 */
int segkv_sdpa_decode(void* out, const void* q,
                      const void* prompt_k, const void* prompt_v,
                      void* resp_k, void* resp_v,
                      const int32_t* parent,
                      const void* k_new, const void* v_new,
                      const float* alibi_slopes,
                      int32_t* anc_out,
                      void* workspace, size_t workspace_bytes,
                      float scale, const segkv_dims* d, void* stream);

/*
 * The same step for a padded static batch whose requests have prompts of
 * different lengths (Section 2.2: requests of a batch are padded to one
 * length).  prompt_lens: NULL (identical to segkv_sdpa_decode), or [B] int32 on
 * the device: request b owns rows 0 .. prompt_lens[b]-1 of prompt_k[b] /
 * prompt_v[b] (0 <= prompt_lens[b] <= Lp; values outside are clamped); the
 * padding rows behind them are never read.  Positions follow the request's own
 * length: its response step s sits at prompt_lens[b] + s, its query at
 * prompt_lens[b] + T - 1.  Everything else as in segkv_sdpa_decode; the
 * workspace size is the same.
 */
int segkv_sdpa_decode_ragged(void* out, const void* q,
                             const void* prompt_k, const void* prompt_v,
                             void* resp_k, void* resp_v,
                             const int32_t* parent,
                             const void* k_new, const void* v_new,
                             const float* alibi_slopes,
                             const int32_t* prompt_lens,
                             int32_t* anc_out,
                             void* workspace, size_t workspace_bytes,
                             float scale, const segkv_dims* d, void* stream);

/*
 * The same step with the prompt segment stored sequence first, prompt_k /
 * prompt_v = [Lp, B, Hkv, D] (the response buffers' own layout): the second
 * arm of the prompt-layout comparison of Section 4.1, which the paper decides
 * in favour of the batch-first layout that segkv_sdpa_decode takes.  Here for
 * that comparison and for callers whose prefill writes sequence-first tensors;
 * every other argument, the arithmetic, the workspace size and the status
 * codes are those of segkv_sdpa_decode_ragged.  SEGKV_UNSUPPORTED when
 * B * Hkv * D exceeds 2^25 elements (rows of a tile are addressed with 32-bit
 * offsets).
 */
int segkv_sdpa_decode_seq_first_prompt(void* out, const void* q,
                                       const void* prompt_k, const void* prompt_v,
                                       void* resp_k, void* resp_v,
                                       const int32_t* parent,
                                       const void* k_new, const void* v_new,
                                       const float* alibi_slopes,
                                       const int32_t* prompt_lens,
                                       int32_t* anc_out,
                                       void* workspace, size_t workspace_bytes,
                                       float scale, const segkv_dims* d, void* stream);

/*
 * The lineage list: the index tensor of Section 3.3 (which response row every
 * beam reads at every past step; the paper obtains it once per generated token,
 * as FasterTransformer does) kept with equal rows merged.  Per request one
 * entry (step << 16) | (slot << 8) | mask for every distinct (step, slot) row
 * that some beam of the request still descends from; mask bit j = beam j reads
 * it; ordered by step, and by slot within a step.  With it the attention call
 * of every layer reads the list instead of re-deriving it from the parent table
 * (which costs one wave 3.5-5 us per 256 steps in every work-group: nothing next
 * to a long prompt, a third of the time when the response is the longer part).
 *
 *   lineage            device buffer of segkv_lineage_bytes(d, lineage_capacity)
 *                      bytes, 16-byte aligned, owned by the caller, opaque
 *                      (per request a 4-word header, then the entries).  No
 *                      initialisation is needed: the call with t == 0 starts
 *                      every request's list.
 *   lineage_capacity   entries per request: a multiple of 4, at least beam times
 *                      the number of steps the list will ever hold.
 *
 * segkv_lineage_update   one generated token, all requests, one small launch:
 *   must be called for t = 0, 1, 2, ... in order, once per step (NOT per layer).
 *   parent_row = row t of the parent table ([B*beam] int32, as in
 *   segkv_sdpa_decode: parent_row[b*beam+j] is the slot at step t-1 of the
 *   hypothesis that slot j extends at step t); ignored, and may be NULL, for
 *   t == 0 and for beam == 1.  Old entries keep the beams whose parent was among
 *   their readers and are dropped when none was; step t adds one row per beam.
 *   Uses d->B and d->beam; 0 <= t < 65536.
 *
 * segkv_sdpa_decode_lineage   segkv_sdpa_decode_ragged with the list in place of
 *   the parent table (prompt_lens may be NULL).  The list must have been updated
 *   through step d->T - 1.  Same tiles and arithmetic as the call with the raw
 *   table: bit-identical output for T <= 256; beyond that the fp32 partial sums
 *   of the waves are combined in a different order (the wave that prepares the
 *   list is free earlier), so outputs agree to rounding.  No anc_out.  The
 *   workspace is that of segkv_sdpa_decode.
 */
size_t segkv_lineage_bytes(const segkv_dims* d, int32_t lineage_capacity);
int segkv_lineage_update(void* lineage, int32_t lineage_capacity, const int32_t* parent_row,
                         int32_t t, const segkv_dims* d, void* stream);
int segkv_sdpa_decode_lineage(void* out, const void* q,
                              const void* prompt_k, const void* prompt_v,
                              void* resp_k, void* resp_v,
                              const void* lineage, int32_t lineage_capacity,
                              const void* k_new, const void* v_new,
                              const float* alibi_slopes,
                              const int32_t* prompt_lens,
                              void* workspace, size_t workspace_bytes,
                              float scale, const segkv_dims* d, void* stream);

/*
 * segkv_sdpa_decode for callers that cannot allocate device memory and have no
 * workspace to pass: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, kernels, arithmetic and results as
 * segkv_sdpa_decode, without `workspace`: the split-KV partial results go to a
 * buffer of SEGKV_STATIC_SCRATCH_BYTES that is part of the library's device
 * image (one copy on every GPU the library runs on, held until the process
 * ends).  The call allocates and frees nothing, on the host side of the HIP
 * runtime or through it.
 *   - Dimensions whose segkv_workspace_bytes(d) exceeds SEGKV_STATIC_SCRATCH_BYTES
 *     are rejected with SEGKV_STATIC_SCRATCH_EXCEEDED before anything is enqueued
 *     (the check is host arithmetic and needs no device).
 *   - The buffer's address is looked up once per device, on the first call made
 *     with that device current that needs scratch; make that call outside graph
 *     capture.  SEGKV_HIP_ERROR if the lookup fails.
 *   - Every call on a GPU uses that GPU's one buffer, which keeps the previous
 *     call's contents (none of them is read before it is overwritten).  Calls
 *     that overlap in time on one GPU -- different streams, or graphs replayed
 *     concurrently -- race on it: serialise them, or use segkv_sdpa_decode with
 *     a workspace per stream.
 */
#define SEGKV_STATIC_SCRATCH_BYTES (16u << 20)
int segkv_sdpa_decode_static_scratch(void* out, const void* q,
                                     const void* prompt_k, const void* prompt_v,
                                     void* resp_k, void* resp_v,
                                     const int32_t* parent,
                                     const void* k_new, const void* v_new,
                                     const float* alibi_slopes,
                                     int32_t* anc_out,
                                     float scale, const segkv_dims* d, void* stream);

/* Bytes of device scratch segkv_sdpa_decode needs for these dimensions (the
 * split-KV partial results of Section 3.3's accumulate step).  0 on invalid
 * dimensions. */
size_t segkv_workspace_bytes(const segkv_dims* d);

/*
 * Placement hint for the caller's allocator (Section 3.2 leaves the relative
 * placement of the K and V buffers open).  Returns the number of bytes by which
 * the base addresses of prompt_v / resp_v should differ from those of prompt_k /
 * resp_k modulo 8192 for the kernel these dimensions select (for example: K
 * buffers 8192-byte aligned, V buffers at an 8192-byte aligned address plus this
 * value).  Two things were measured on MI355X.  One in four 256-byte address
 * classes is served more slowly; when every work-group streams a single 256-byte
 * column of K and of V, an offset of 256 modulo 1024 keeps any KV head from
 * drawing both from the slow class (3-5 % on the Llama2-7B and 70B shapes).  And a
 * wave asks for row i of K and row i of V at the same moment; when the bytes of
 * one token's keys are a power of two, a further 4096 puts the two in different
 * places of the memory system (1.4 % on the Llama2-7B shape, 0.6 % on the 70B
 * shape, nothing where a token's keys are not a power of two bytes).  Purely a
 * performance hint: results never depend on it, and 0 is returned where it does
 * not help (heads of 512 bytes).  Host-only.
 */
size_t segkv_value_stagger_bytes(const segkv_dims* d);

/* Human-readable text for a status code.  Static strings, except for
 * SEGKV_HIP_ERROR, whose text ends with the HIP runtime's own description of
 * the error that the calling thread's most recent rejected launch returned
 * (hipGetErrorString); that one is kept per thread and stays valid until the
 * thread's next segkv_status_string(SEGKV_HIP_ERROR). */
const char* segkv_status_string(int status);

/*
 * TEST-ONLY.  The launch planner can be overridden through environment
 * variables so that tests and A/B measurements reach every kernel and plan on
 * small inputs: SEGKV_PATH (alu | mfma), SEGKV_TARGET_GROUPS, SEGKV_MIN_PCHUNK,
 * SEGKV_MFMA_WAVES (4 | 8), SEGKV_HEADS_PER_WAVE (1 | 2 | 4), SEGKV_PAIR_HEADS
 * (0 | 1), SEGKV_XCD_HEAD_ORDER (0), SEGKV_PREFILL (regs).  They are read ONCE, on the library's first
 * use in the process, so that the workspace size a caller asked for and the
 * launch that follows always agree; this call reads them again.  Not for use
 * while other threads are inside the library.  Results never depend on the
 * overrides beyond rounding order; production callers set none of them.
 */
void segkv_reload_tuning(void);

/*
 * MEASUREMENT ONLY (no attention arithmetic; nothing else in the library calls it).
 * Runs a register-resident chain of the fp16 32x32x16 matrix instruction, the one the
 * attention kernels use: n_groups work-groups of 4 waves, `iters` iterations of 16
 * instructions per wave = n_groups * 4 * iters * 16 * 32768 flop in all.  The caller times
 * the call (stream order) to get the rate the part sustains for the operands it supplied --
 * constant ones run near the published clock, random ones under the power limit -- which is
 * the practical ceiling for the prefill kernel's TFLOP/s.
 *   operands  device, 16 * 256 * 16 bytes of fp16: 8 A then 8 B operands, 16 bytes per lane
 *             of a 256-thread group (every group reads the same ones); 16-byte aligned
 *   out       device, n_groups * 256 fp32 (sums of the accumulators, written so that the work
 *             cannot be dropped)
 *   clocks    device, n_groups * 2 uint64: shader cycles and 100 MHz ticks each group ran
 *             (their ratio x 100 = its clock in MHz)
 * Buffers stay the caller's; nothing is allocated.  Returns SEGKV_OK, SEGKV_INVALID_ARG (a
 * null pointer, n_groups or iters <= 0, n_groups > 2^20), SEGKV_MISALIGNED or SEGKV_HIP_ERROR.
 */
int segkv_probe_mfma_rate(const void* operands, void* out, void* clocks, int32_t n_groups, int32_t iters,
                          void* stream);

/*
 * Prefill-phase attention (Section 3.1, prefill phase; Section 3.3: the special
 * case of the decode kernel that uses only the query and the prompt key/value).
 * Batch-first tensors in and out, no transposes:
 *   out, q   [B, Lp, Hq, D]  fp16        k, v   [B, Lp, Hkv, D]  fp16
 * k and v are the prompt segment itself: after this call they are what
 * segkv_sdpa_decode takes as prompt_k / prompt_v.  Token i of a request attends
 * to keys 0..i of the same request (causal); beams are not expanded yet.
 * alibi_slopes (NULL or [Hq] fp32) and scale as in segkv_sdpa_decode; key j has
 * position j.  Uses d->B, Hq, Hkv, D and d->Lp (>= 1); beam, T, Tcap are ignored.
 * Arithmetic: fp16 operands on the matrix cores, fp32 softmax and accumulation,
 * softmax weights rounded to fp16 for the PV product, fp16 output (RNE).
 */
int segkv_sdpa_prefill(void* out, const void* q, const void* k, const void* v,
                       const float* alibi_slopes, float scale, const segkv_dims* d, void* stream);

/*
 * Segment-cache bookkeeping (Section 3.2).  Host-only arithmetic, no device.
 *
 * segkv_cache_token_bytes      Eq. (1): bytes of K and V of one token over all
 *                              layers = 2 * L * H * D * elem_bytes.
 * segkv_cache_standard_bytes   Eq. (2): contiguous per-beam cache
 *                              BS * BW * (N_prompt + N_response) * token bytes.
 * segkv_cache_segment_bytes    Eq. (3): prompt once per request plus the
 *                              response buffer at its grown capacity,
 *                              BS * (N_prompt + BW * capacity(N_response)) * token bytes.
 * segkv_response_capacity      rows allocated for n_response valid rows: the
 *                              response buffer grows in steps of 16 rows
 *                              (capacity = ceil(n/16) * 16; 0 for n <= 0).
 * All sizes are exact 64-bit integers; arguments <= 0 give 0.
 */
uint64_t segkv_cache_token_bytes(int32_t L, int32_t H, int32_t D, int32_t elem_bytes);
uint64_t segkv_cache_standard_bytes(int32_t BS, int32_t BW, int32_t n_prompt, int32_t n_response,
                                    uint64_t token_bytes);
uint64_t segkv_cache_segment_bytes(int32_t BS, int32_t BW, int32_t n_prompt, int32_t n_response,
                                   uint64_t token_bytes);
int32_t segkv_response_capacity(int32_t n_response);

/*
 * Growth of the response buffers (Section 3.2: when the step count passes the
 * capacity, a buffer 16 rows longer is allocated, the old rows are copied over
 * and the old buffer is released).  The caller allocates and frees; this call
 * copies rows 0..T-1 of old_k / old_v [Tcap_old, B*beam, Hkv, D] into new_k /
 * new_v [Tcap_new, B*beam, Hkv, D] -- one contiguous block each, because the
 * layout is sequence first.  Uses d->B, beam, Hkv, D and d->T (rows to copy,
 * 0 <= T <= d->Tcap = Tcap_old); tcap_new >= d->Tcap.  Rows >= T of the new
 * buffers are left untouched.  Device pointers, 16-byte aligned; asynchronous
 * on `stream`.
 */
int segkv_grow_response(void* new_k, void* new_v, const void* old_k, const void* old_v,
                        int32_t tcap_new, const segkv_dims* d, void* stream);

/*
 * Measurement helper: reads `bytes` bytes (multiple of 16) from `src` with
 * 128-bit loads spread over the whole device and writes one checksum word per
 * work-group to `sink` (>= 4096 * 4 bytes).  Gives the practical streaming-read
 * ceiling of the device next to which attention timings are quoted.
 */
int segkv_stream_read_probe(const void* src, size_t bytes, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SEGKV_H */
