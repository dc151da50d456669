/*
 * libmixkvq: decode-time attention over a mixed-precision quantized KV cache
 * (MixKVQ) for AMD MI355X (gfx950).  C ABI; no C++ or torch types cross it.
 *
 * Conventions for every call
 *   - Returns MIXKVQ_OK (0) or a negative MIXKVQ_E* code; nothing throws or aborts
 *     across this boundary.  On an error return the cache is unchanged.
 *   - Pointers marked DEVICE are HIP device pointers owned by the caller (for
 *     example torch allocations); pointers marked HOST are ordinary host memory.
 *     The library allocates only the small host-side handle.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  All
 *     device work is enqueued asynchronously on it; no call synchronises or reads
 *     device memory back.  Token counts depend only on the sequence of n_new
 *     values, so the host-side state is exact without a read-back.
 *   - The batch calls advance all sequences together.  Sequences may still differ in length: the *_seq calls
 *     work on one sequence of the batch (prefill of a new request into a free slot, reset of a finished one); after
 *     them every batch call appends to / attends over each sequence from its own state.
 *   - Grouped-query mapping: query heads [j*g, (j+1)*g) use KV head j, g = Hq/Hkv.
 *   - "fp16" tensors below are IEEE binary16, or bfloat16 when cfg.in_dtype == 1 (same shapes and strides, in
 *     elements); Inf/NaN inputs are outside the contract.
 *   - Precision of mixkvq_decode_attention / mixkvq_decode_step: fp16 operands, binary32 sums.  Against exact
 *     arithmetic on the same dequantized cache, |out - exact| <= 2e-3 + 1e-2 |exact| per element as long as the
 *     dequantized values stay within +-512; beyond, the absolute term is 2^-18 of the largest |value| (Eq. 3 is
 *     evaluated as sum (p s) c + sum p z, two binary32 sums that cancel where a group's zero-point is far from its
 *     values).  Scaled logits are binary32 numbers: a query/key pair that drives them beyond ~2^13 loses the
 *     differences between tokens that binary32 cannot hold at that magnitude.
 *   - Calls on one cache must be issued from one host thread at a time.
 */
#ifndef MIXKVQ_H
#define MIXKVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MIXKVQ_OK          0
#define MIXKVQ_EINVAL    (-1)  /* bad shape, alignment, NULL pointer or unsupported configuration */
#define MIXKVQ_ECAPACITY (-2)  /* the append would exceed T_max quantized tokens */
#define MIXKVQ_EHIP      (-3)  /* a HIP call failed; mixkvq_strerror gives the HIP message */
#define MIXKVQ_ENOMEM    (-4)  /* host allocation of the handle failed */
#define MIXKVQ_EEMPTY    (-5)  /* decode attention on a cache that holds no token */
#define MIXKVQ_ESCRATCH  (-7)  /* mixkvq_decode_attention_noalloc: the launch needs more than the built-in scratch buffer */
#define MIXKVQ_ERAGGED   (-6)  /* mixkvq_cache_state on a batch whose sequences differ: use mixkvq_cache_state_seq */

typedef struct mixkvq_cache mixkvq_cache; /* opaque HOST handle: counts + the caller's device pointers */

/* Caller-filled plain data.  Symbols follow the paper: R = residual length
 * (Appendix D.1), G = group size (Section 5, "Settings"). */
typedef struct {
  int32_t B, Hq, Hkv;   /* batch, query heads, KV heads; Hq % Hkv == 0, Hq/Hkv <= 8 */
  int32_t D;            /* head dimension; must be 128 */
  int32_t T_max;        /* capacity of the quantized part in tokens; multiple of R */
  int32_t Gk;           /* key group: Gk consecutive tokens of one channel; Rr % Gk == 0 (Rr below), Gk % 16 == 0 */
  int32_t Gv;           /* value group: Gv consecutive channels of one token; D % Gv == 0, Gv % 16 == 0 */
  int32_t R;            /* residual window length == flush unit; a multiple of 16 up to 128, or 256.  A block of R tokens
                           is scored as a whole and stored as R / Rr records of Rr tokens with one channel list: Rr = R,
                           except Rr = 128 for R = 256 and Rr = 32 for R = 96 with Gk = 16 or 32 */
  int32_t k4, k16;      /* salient key channels kept at 4 bit / as fp16; k4 % 8 == 0, k16 % 4 == 0, k4+k16 < D */
  int32_t flush_mode;   /* 0 deferred: the newest <= R tokens stay fp16; 1 eager: flush as soon as R are buffered */
  int32_t score_mode;   /* 0: A_d = I_d * S_d (Eq. 8); 1: A_d = S_d (error-only ablation) */
  int32_t qacc_reset_on_flush; /* 0: |q| accumulator runs since sequence start; 1: cleared by every call that flushes */
  int32_t policy;       /* 0: the k16 + k4 channels with the highest score; 1: the thresholds of Section 4.2 (below) */
  double tau16, tau4;   /* policy 1: A_d > tau16 -> fp16 tier; tau4 < A_d <= tau16 -> 4-bit tier; otherwise 2 bit.
                         * A_d = I_d * S_d in real units: I_d the mean |q| (Eq. 6), S_d = range / 3 (Eq. 7 for the two-bit
                         * quantizer), or S_d alone with score_mode 1.  Both >= 0 (infinity allowed), not NaN.  k16 and k4
                         * are then the record's capacity per block: if more channels pass a threshold, the best by (score,
                         * lower index) keep the tier and the others fall to the next tier down. */
  int32_t sink;         /* the first `sink` tokens of every sequence stay in fp16 for good (the sink length of Appendix E);
                         * 0, 32, 64, 96 or 128.  They are attended like the residual window and never quantized. */
  int32_t in_dtype;     /* element type of every q, k, v tensor the caller passes and of `out`: 0 binary16, 1 bfloat16.
                         * bfloat16 inputs enter the cache as the nearest binary16 (ties to even, saturated at +-65504:
                         * exact wherever binary16 has the range); everything stored and computed is as for binary16. */
} mixkvq_config;

#define MIXKVQ_NO_CHANNEL 255  /* unused entry of a channel list (policy 1) */

/* Bytes of each caller-owned device buffer. */
typedef struct {
  uint64_t blocks;     /* [B*Hkv][T_max/Rr] block records (Rr tokens each, see R above), see mixkvq_block_layout */
  uint64_t res_k;      /* [B*Hkv][sink + R][D] fp16 keys: per pair the sink rows, then the residual window */
  uint64_t res_v;      /* [B*Hkv][sink + R][D] fp16 values likewise */
  uint64_t qacc;       /* [B*Hkv][D] u64 sums of |q| in units of 2^-24, then [B*Hkv] u64 counts */
  uint64_t workspace;  /* split-K partials and selection scratch */
} mixkvq_sizes;

typedef struct {
  void *blocks, *res_k, *res_v, *qacc, *workspace; /* DEVICE, 256-byte aligned */
} mixkvq_buffers;

/* Byte offsets of the planes inside one block record (Rr tokens of one (batch, KV head) pair, see mixkvq_config.R;
 * R below stands for Rr).  Every plane starts on a 16-byte boundary, padding is 0.
 *   idx    u8  [k16+k4]      fp16-tier channels ascending, then 4-bit-tier channels ascending; under policy 1 each
 *                            tier is filled up to its capacity with MIXKVQ_NO_CHANNEL and the unused entries of
 *                            every plane of that tier are 0
 *   kmax   f16 [NG + 1]      [g < NG]: largest stored scale among group g's 2-bit and 4-bit key channels; [NG]: largest
 *                            stored value scale of the block (derived metadata: lets a reader pick exponents without a scan)
 *   klo_s  f16 [NG][NLp]     scales of the 2-bit key channels (the non-salient channels, ascending)
 *   klo_z  f16 [NG][NLp]     zero-points (group minima, Eq. 2)
 *   k4_s   f16 [NG][k4]      4-bit tier scales, tier order;  k4_z likewise
 *   klo    u32 [R][Wlo]      16 two-bit codes per word along channels; even codes fill the low half-word, odd
 *                            codes the high one: code i in bits [16(i&1) + 2(i>>1), +2)
 *   k4     u32 [R][k4/8]     8 four-bit codes per word, code i in bits [16(i&1) + 4(i>>1), +4)
 *   k16    f16 [R][k16]      raw values of the fp16 tier
 *   v      u32 [R/16][D]     16 two-bit codes per word along TOKENS for one channel, same bit order as klo.  Code i of
 *                            word tg belongs to token 16 tg + i; with v_interleave (set when Gk == 32 and R % 64 == 0)
 *                            to token 64 (tg/4) + 8 (tg%4) + (i%8) + 32 (i/8): word j of a 64-token span holds the
 *                            j-th 8 tokens of each of the span's two key groups
 *   v_s    f16 [R][D/Gv]     value scales per (token, channel group);  v_z likewise
 * NL = D-k4-k16 (policy 1: NL = D, room for every channel; the 2-bit channels of a block fill the first
 * D-n16-n4 places), Wlo = ceil(NL/16), NLp = 16*Wlo, NG = R/Gk, NVG = D/Gv, W4 = k4/8. */
typedef struct {
  int32_t NL, Wlo, NLp, NG, NVG, W4;
  int32_t off_idx, off_kmax, off_klo_s, off_klo_z, off_k4_s, off_k4_z, off_klo, off_k4, off_k16, off_v, off_v_s, off_v_z;
  int32_t rec_bytes;
  int32_t v_interleave;
} mixkvq_block_layout_t;

/* Validates cfg and fills the record layout.  HOST pointers.  EINVAL on a bad configuration. */
int mixkvq_block_layout(const mixkvq_config* cfg, mixkvq_block_layout_t* out);

/* Sizes of the five device buffers for cfg.  HOST pointers. */
int mixkvq_cache_sizes(const mixkvq_config* cfg, mixkvq_sizes* out);

/* Creates the host handle over caller-owned device buffers (each at least as large as
 * mixkvq_cache_sizes says, 256-byte aligned).  The cache starts empty; call
 * mixkvq_cache_reset once before first use to clear the |q| accumulator. */
int mixkvq_cache_create(const mixkvq_config* cfg, const mixkvq_buffers* bufs, mixkvq_cache** out);
void mixkvq_cache_destroy(mixkvq_cache* c);

/* Paged storage of the block records.  table: DEVICE int32 [B][T_max/Rr], owned by the caller; record i of sequence b
 * (for its Hkv heads, one after the other) then lives in slot table[b][i] of a pool, and bufs->blocks is that pool:
 * slots * Hkv * rec_bytes bytes for as many slots as the caller's allocator hands out, instead of the size
 * mixkvq_cache_sizes reports.  The kernels read the table when a call runs: an entry must be set before the call that
 * flushes or reads its block, and must not change while the block is in use.  NULL returns to the contiguous layout.
 * EINVAL while any sequence holds quantized blocks. */
int mixkvq_cache_set_block_table(mixkvq_cache* c, const int32_t* table);

/* Empties the cache (token counts to 0) and zeroes the |q| accumulator on `stream`. */
int mixkvq_cache_reset(mixkvq_cache* c, void* stream);

/* Host-only: quantized, residual-window and sink token counts.  Any out pointer may be NULL.
 * ERAGGED if the sequences differ (then ask per sequence). */
int mixkvq_cache_state(const mixkvq_cache* c, int64_t* n_quantized, int32_t* n_residual, int32_t* n_sink);
int mixkvq_cache_state_seq(const mixkvq_cache* c, int32_t b, int64_t* n_quantized, int32_t* n_residual, int32_t* n_sink);

/* Resuming from a snapshot.  Everything a cache holds is in its five device buffers plus these token counts, so a
 * snapshot is a copy of the buffers and of what mixkvq_cache_state(_seq) reports; to resume, copy the buffers back
 * (into the same or another cache of the same configuration, with the same block table if one is in use) and set the
 * counts here.  Host-only.  EINVAL for counts that no sequence of appends produces (n_quantized a multiple of R up to
 * T_max; n_residual 1..R with the deferred flush once anything was flushed, 0..R-1 with the eager one; the window
 * empty until the sink is full).  Appendix D.1 describes the cache as exactly this state. */
int mixkvq_cache_set_state(mixkvq_cache* c, int64_t n_quantized, int32_t n_residual, int32_t n_sink);
int mixkvq_cache_set_state_seq(mixkvq_cache* c, int32_t b, int64_t n_quantized, int32_t n_residual, int32_t n_sink);

/* Empties sequence b only (its token counts and its rows of the |q| accumulator).  The per-sequence calls
 * (mixkvq_cache_reset_seq, mixkvq_quantize_append_seq) are for batches of at most 256 sequences: EINVAL beyond. */
int mixkvq_cache_reset_seq(mixkvq_cache* c, int32_t b, void* stream);

/* Channel selection (Section 4.2, Eq. 6-8; top-k channel budget or thresholds, see mixkvq_config.policy).
 *   q  DEVICE fp16 [B][Hq][Lq][D] after rotary embedding, element strides q_strides = {batch, head, token},
 *      channel stride 1; may be NULL with Lq = 0 (use the running accumulator only).
 *   k  DEVICE fp16 [B][Hkv][L][D] after rotary embedding, strides k_strides likewise; L >= 1.
 * Adds sum|q| over the Lq tokens and over the g query heads of each KV head into the cache's accumulator
 * (Eq. 6; Appendix D), takes max-min of every key channel over the L tokens (Eq. 7), scores
 * A_d = sum|q|_d * range_d (Eq. 8 up to constants shared by the head), and writes the k16+k4 best
 * channels per (b, KV head) to sel DEVICE u8 [B][Hkv][k16+k4]: first the k16 best, ascending, then the
 * next k4, ascending.  Ties go to the lower channel index.  Under policy 1 the two lists hold the channels
 * that pass the thresholds, each filled up with MIXKVQ_NO_CHANNEL.  The token counts are unchanged. */
int mixkvq_select_channels(mixkvq_cache* c, const void* q, int32_t Lq, const int64_t q_strides[3],
                           const void* k, int32_t L, const int64_t k_strides[3],
                           uint8_t* sel, void* stream);

/* mixkvq_select_channels for sequence b alone: q DEVICE [Hq][Lq][D] with element strides {head, token}, k DEVICE
 * [Hkv][L][D] likewise, sel DEVICE u8 [Hkv][k16+k4].  Same rules otherwise. */
int mixkvq_select_channels_seq(mixkvq_cache* c, int32_t b, const void* q, int32_t Lq, const int64_t q_strides[2],
                               const void* k, int32_t L, const int64_t k_strides[2], uint8_t* sel, void* stream);

/* Prefill (n_new = prompt length) and per-step (n_new = 1) append (Appendix D.1).
 *   k_new, v_new  DEVICE fp16 [B][Hkv][n_new][D], element strides kv_strides = {batch, head, token}.
 *   sel           DEVICE u8 [B][Hkv][k16+k4] or NULL.
 * The first cfg.sink tokens of a sequence go to the sink and stay there.  Later tokens enter the fp16 residual window;
 * whole R-token blocks leave it per flush_mode and are quantized
 * (Eq. 2: keys per channel in groups of Gk tokens, 2 bit, the selected channels at 4 bit or fp16; values per
 * token in groups of Gv channels, 2 bit) into block records.  With sel != NULL every block flushed by this
 * call uses that selection; with sel == NULL each block is scored from the accumulator and its own R tokens.
 * ECAPACITY if the quantized part would exceed T_max. */
int mixkvq_quantize_append(mixkvq_cache* c, const void* k_new, const void* v_new, int32_t n_new,
                           const int64_t kv_strides[3], const uint8_t* sel, void* stream);

/* A prompt in one call: the same selection, records and cache state as
 *   mixkvq_select_channels(c, q, Lq, q_strides, k, L, kv_strides, sel, stream) followed by
 *   mixkvq_quantize_append(c, k, v, L, kv_strides, sel, stream),
 * with the same argument rules and errors, all of them checked before anything is enqueued: a prompt that does not
 * fit (ECAPACITY) leaves the |q| accumulator untouched as well (Section 4.2 scores the prompt, Appendix D.1 stores
 * it).  sel: DEVICE u8 [B][Hkv][k16+k4], written. */
int mixkvq_prefill(mixkvq_cache* c, const void* q, int32_t Lq, const int64_t q_strides[3], const void* k, const void* v,
                   int32_t L, const int64_t kv_strides[3], uint8_t* sel, void* stream);

/* mixkvq_quantize_append for sequence b alone: k_new, v_new DEVICE [Hkv][n_new][D] with element strides
 * {head, token}, sel DEVICE u8 [Hkv][k16+k4] or NULL.  The other sequences are untouched. */
int mixkvq_quantize_append_seq(mixkvq_cache* c, int32_t b, const void* k_new, const void* v_new, int32_t n_new,
                               const int64_t kv_strides[2], const uint8_t* sel, void* stream);

/* One query token per sequence (Section 3.1, Eq. 1, over keys/values dequantized by Eq. 3).
 *   q    DEVICE fp16 [B][Hq][D] contiguous;  out DEVICE fp16 [B][Hq][D];  lse DEVICE fp32 [B][Hq] or NULL
 *        (natural-log sum of exp of the scaled logits).
 *   scale <= 0 means 1/sqrt(D).  accumulate_q != 0 also adds |q| to the accumulator (Appendix D.2).
 * EEMPTY if the cache holds no token.  When the sequences differ in length each attends over its own tokens (at most
 * 256 sequences then, else EINVAL); a sequence without tokens gets out = 0 and lse = -inf and its |q| is not accumulated. */
int mixkvq_decode_attention(mixkvq_cache* c, const void* q, void* out, float* lse,
                            float scale, int32_t accumulate_q, void* stream);

/* mixkvq_decode_attention for callers that cannot allocate device memory and hand over no workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid allocation.  Same arguments, results and errors; the
 * split-K partials go to a buffer built into the library (MIXKVQ_NOALLOC_SCRATCH_BYTES of device memory on every GPU
 * the library runs on, held until the process ends) instead of the cache's workspace, and the call allocates nothing
 * on the host or the device.  ESCRATCH if the launch would need more: pairs x splits x (Hq/Hkv) x 130 floats (any
 * configuration of up to 512 (batch, KV head) pairs fits).  The buffer is shared by every call on a GPU and needs no
 * clearing (a launch writes every partial it reads); calls that overlap on one GPU (two streams, two threads) race. */
#define MIXKVQ_NOALLOC_SCRATCH_BYTES (8u << 20)
int mixkvq_decode_attention_noalloc(mixkvq_cache* c, const void* q, void* out, float* lse,
                                    float scale, int32_t accumulate_q, void* stream);

/* One decode step in the fewest launches: the same result and cache state as
 * mixkvq_quantize_append(c, k_new, v_new, 1, kv_strides, NULL, stream) followed by
 * mixkvq_decode_attention(c, q, out, lse, scale, accumulate_q, stream), with the same argument rules and
 * errors (Appendix D.1: the new key/value enter the residual buffer; Eq. 1 over the cache).  When the append
 * flushes no block, the attention launch moves the new rows into the window itself. */
int mixkvq_decode_step(mixkvq_cache* c, const void* k_new, const void* v_new, const int64_t kv_strides[3],
                       const void* q, void* out, float* lse, float scale, int32_t accumulate_q, void* stream);

/* Profiling aid.  With a pair of hipEvent_t handles (HOST, created by the caller with timing enabled), every
 * following mixkvq_decode_attention / mixkvq_decode_step on this cache makes start_event and stop_event take the start
 * and the end time of its split-K attention kernel (the kernel's own time stamps, as a profiler reports them; with the
 * vector-ALU fallback kernel the events are recorded in the stream just before and after it).  Pass NULL, NULL to
 * switch it off. */
int mixkvq_set_timing_events(mixkvq_cache* c, void* start_event, void* stop_event);

/* Profiling aid: which kernel the last mixkvq_decode_attention / mixkvq_decode_step on this cache launched.
 * MIXKVQ_PATH_NONE (no attention call yet), MIXKVQ_PATH_MATRIX (the matrix-core kernel) or MIXKVQ_PATH_VECTOR (the
 * vector-ALU kernel, which covers the configurations the matrix-core kernel has no variant for and is many times
 * slower).  Host-only, no synchronisation; negative on a NULL handle. */
#define MIXKVQ_PATH_NONE 0
#define MIXKVQ_PATH_MATRIX 1
#define MIXKVQ_PATH_VECTOR 2
int mixkvq_decode_path(const mixkvq_cache* c);

/* Message for a return code (for EHIP: the last HIP error string seen by this thread). */
const char* mixkvq_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* MIXKVQ_H */
