/*
 * hqmq.h - C ABI of the MI355X (gfx950) HQMQ KV-cache encode / decode library.
 *
 * HQMQ (Hurwitz Quaternion Multiplicative Quantization) splits every K or V head vector
 * into 4-element chunks read as quaternions x, stores the norm r = |x| with a uniform
 * b_r-bit quantiser against a per-token scale, and the direction u = x / r as the index of
 * the nearest product q_p * q_s, q_p in the 24-element Hurwitz group 2T, q_s in a seeded
 * per-(layer, head, role) codebook of S unit quaternions (paper Sec. 3, Eq. 1, Alg. 1).
 * Chunks whose norm exceeds C times the batch median norm of their (layer, head, role) are
 * kept verbatim in fp16 next to a one-bit flag (Sec. 3 "Median-multiplier outlier
 * extraction").
 *
 * Conventions common to every entry point
 *   - extern "C", plain pointers and sizes.  "HOST" / "DEVICE" says where a pointer lives.
 *   - The caller owns every buffer.  The library allocates nothing, keeps no global state
 *     besides the last HIP error code of each thread and a set-up flag per device (see hqmq_init),
 *     and only enqueues work on the given HIP stream
 *     (hipStream_t passed as void*; NULL = the default stream).  Calls return as soon as the
 *     work is enqueued; results are valid once the stream has been synchronised.
 *   - Return value: HQMQ_OK or a negative HQMQ_ERR_* code.  Nothing is enqueued when an
 *     argument error is returned.  Data-dependent conditions are reported through the
 *     device-side status word (see hqmq_encoded.status).
 *   - One call handles one (layer, role) tensor X, fp16 [B, H, T, D] addressed through
 *     element strides (D contiguous): "the current batch" of Alg. 1.  A row is one (b, h, t)
 *     vector, linear row index R = (b*H + h)*T + t; chunk c of a row is elements 4c..4c+3,
 *     element 0 being the real part; linear chunk index = R*n_c + c, n_c = ceil(D/4).
 *   - Head dimensions 1 <= D <= 128 (the paper's models have 64, 96 and 128): a row has
 *     n_c <= 32 chunks, one flag word and ceil(n_c*w/32) code words (exactly w at D = 128).  A
 *     D that is not a multiple of 4 is handled as the paper's padding wrapper does (App.
 *     "Padding wrapper for d_h not divisible by 4"): the last chunk is completed with zeros on
 *     encode and the surplus elements are not written on decode; nothing past D is touched.
 *     D = 128 is the tuned path and wants strides that are multiples of 8; other D take any
 *     strides (multiples of 4 and a D that is one keep every chunk one aligned 8-byte access).
 *     hqmq_attend takes D = 64, 96 and 128 (the head dimensions of the paper's models).
 */
#ifndef HQMQ_H
#define HQMQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Largest secondary codebook every entry point takes: a joint index k = p S + s < 24 S has to fit 16 bits.
 * The paper sweeps S = 24 .. 192.  Up to 512 entries the search keeps a head's codebook and its matrix operands
 * in a CU's LDS; beyond that every chunk scores all S secondaries in fp32 on the vector ALUs: the same result
 * (the decision is taken on fp32 scores either way), several times slower per codeword. */
#define HQMQ_MAX_S 2730

#define HQMQ_OK 0
#define HQMQ_ERR_INVALID_ARG (-1)      /* null pointer, non-positive size, misaligned pointer or stride */
#define HQMQ_ERR_UNSUPPORTED (-2)      /* D > 128 (hqmq_attend: D not 64, 96 or 128), S outside 1..2730, b_r outside 1..8, C not a positive finite number */
#define HQMQ_ERR_BUFFER_TOO_SMALL (-3) /* workspace smaller than hqmq_sizes() asks for */
#define HQMQ_ERR_HIP (-4)              /* a HIP call failed; see hqmq_last_hip_error() */

/* hqmq_params.flags */
#define HQMQ_FLAG_NO_OUTLIERS 1u /* skip the median and the extraction: no chunk is flagged */
#define HQMQ_FLAG_CHECK_FINITE 2u /* encode: report an input that holds an infinity or a NaN in the status word \
                                     (the encoded result of such a tensor is undefined, but every access stays  \
                                     in bounds and every index inside the codebook) */

#define HQMQ_FLAG_ATTEND_TABLES 4u /* hqmq_attend*: read the reconstruction from per-head tables of codeword      \
                                      directions in LDS whenever they fit (S <= 256 or so), not only for long     \
                                      caches, where the library does so by itself; same results up to the last     \
                                      fp32 bit before the fp16 rounding of an element; ask                         \
                                      hqmq_attend_workspace_bytes with the same flags; the other entry points      \
                                      ignore it */

/* bits of the device-side status word */
#define HQMQ_STATUS_OUTLIER_OVERFLOW 1u /* more outliers than outlier_capacity: payload truncated */
#define HQMQ_STATUS_NONFINITE 2u        /* HQMQ_FLAG_CHECK_FINITE was set and x holds an infinity or a NaN */

typedef struct hqmq_params {
    int32_t B, H, T, D;                   /* X is fp16 [B, H, T, D], D contiguous                  */
    int64_t stride_b, stride_h, stride_t; /* element strides of b, h, t; multiples of 8 at D = 128 */
    int32_t S;                            /* secondary codebook size per (layer, head, role)       */
    int32_t b_r;                          /* radius bits (paper: 3, 4 or 6)                        */
    float C;                              /* outlier multiplier (paper: 3)                         */
    uint32_t flags;                       /* HQMQ_FLAG_*                                           */
} hqmq_params;

/* Buffer sizes for a given hqmq_params, in bytes unless said otherwise. */
typedef struct hqmq_size_info {
    uint64_t n_rows;               /* B*H*T                                                        */
    uint32_t index_bits;           /* w_idx = ceil(log2(24 S)) (Sec. 3: index width)               */
    uint32_t code_bits;            /* w = w_idx + b_r: bits per chunk                              */
    uint64_t code_bytes;           /* n_rows * code_words_per_row * 4                              */
    uint64_t sigma_bytes;          /* n_rows * 2                                                   */
    uint64_t flag_bytes;           /* n_rows * 4                                                   */
    uint64_t row_off_bytes;        /* (n_rows + 1) * 4                                             */
    uint64_t n_outliers_bytes;     /* (H + 1) * 4                                                  */
    uint64_t status_bytes;         /* 4                                                            */
    uint64_t outlier_capacity_max; /* chunks: no input can flag more than this                     */
    uint64_t outlier_bytes_max;    /* outlier_capacity_max * 8                                     */
    uint64_t workspace_bytes;      /* scratch hqmq_encode needs                                    */
    uint32_t chunks_per_row;       /* n_c = ceil(D / 4)                                            */
    uint32_t code_words_per_row;   /* ceil(n_c * w / 32): w at D = 128                             */
} hqmq_size_info;

/* The encoded form of one tensor: a HOST struct of DEVICE pointers, all caller-owned.
 *   codes      uint32 [n_rows][code_words_per_row]
 *                                   chunk code = (r_q << w_idx) | k, k = p*S + s (p-major),
 *                                   flagged chunks 0; the n_c codes of a row concatenated
 *                                   LSB first: chunk c at bits [c*w, (c+1)*w) of the row's
 *                                   little-endian words, unused high bits of the last word 0
 *                                                                             (Alg. 1 "store")
 *   sigma      fp16   [n_rows]      per-token scale: largest norm among the row's unflagged
 *                                   chunks, rounded to nearest even, saturating (Sec. 3
 *                                   "Radius quantization")
 *   flags      uint32 [n_rows]      bit c set = chunk c of the row is an outlier
 *   row_off    uint32 [n_rows + 1]  number of outliers in all earlier rows (exclusive prefix);
 *                                   last entry = total
 *   outliers   fp16   [cap][4]      the flagged chunks verbatim, ascending linear chunk index
 *                                   (may be NULL when the capacity passed is 0)
 *   n_outliers uint32 [H + 1]       outliers per head, then the total (true counts even on
 *                                   overflow)
 *   status     uint32 [1]           HQMQ_STATUS_* bits, written by hqmq_encode             */
typedef struct hqmq_encoded {
    uint32_t *codes;
    uint16_t *sigma;
    uint32_t *flags;
    uint32_t *row_off;
    uint16_t *outliers;
    uint32_t *n_outliers;
    uint32_t *status;
} hqmq_encoded;

/* Per-device set-up for the CURRENT device (hipSetDevice): raises the dynamic-LDS limit of the search and
 * attention kernels and looks up the device address of the workspace of hqmq_encode_static.  Thread-safe
 * and idempotent.  Every encode and attention entry point runs it by itself on its first call on a device,
 * so calling it is optional - except before a stream capture: the set-up is not stream work and must not
 * happen while a capture is open, so call hqmq_init() (or run one eager encode) on the device first.
 * Errors: HIP. */
int32_t hqmq_init(void);

/* Secondary codebooks (App. D "Secondary codebook initialization"): for every (layer, role,
 * head) S i.i.d. standard-normal 4-vectors, normalised to unit length, drawn from a
 * counter-based generator so that entry (layer, role, head, s) depends only on the seed and
 * its linear index ((layer*2 + role)*n_kv_heads + head)*S + s.  role 0 = K, 1 = V.
 *   sec_host  HOST, out, fp32 [n_layers][2][n_kv_heads][S][4], caller-owned.
 * Pure host function (no GPU work).  Errors: INVALID_ARG (null pointer, non-positive size),
 * UNSUPPORTED (S > HQMQ_MAX_S: the limit of hqmq_encode and hqmq_decode). */
int32_t hqmq_build_codebooks(uint64_t seed, int32_t n_layers, int32_t n_kv_heads, int32_t S,
                             float *sec_host);

/* Sizes of the encoded buffers and of the encode workspace for `params` (HOST pointers).
 * Errors: INVALID_ARG, UNSUPPORTED (same checks as hqmq_encode). */
int32_t hqmq_sizes(const hqmq_params *params, hqmq_size_info *out);

/* Encode one tensor (Alg. 1 "Encode" + "Outlier extraction", App. D "Encode", "Outlier
 * extraction").  Steps, all on the GPU: squared chunk norms in fp64; exact lower median per
 * head over the batch (radix select); flag r^2 > C^2 * median (strict); ordered compaction
 * of the flagged chunks; per-row fp16 scale over the unflagged chunks; nearest joint codeword
 * by exhaustive search over all S secondaries (24 primaries each, lowest index on ties);
 * radius code r_q = clamp(rint(r * (2^b_r - 1) / sigma), 0, 2^b_r - 1); bit packing.
 *   params            HOST.
 *   x_dev             DEVICE, in, fp16, 16-byte aligned, addressed with params strides; finite (the
 *                     paper does not define the encode of an infinity or a NaN; with HQMQ_FLAG_CHECK_FINITE
 *                     status gets HQMQ_STATUS_NONFINITE for such an input).
 *   sec_dev           DEVICE, in, fp32 [H][S][4]: the codebooks of THIS (layer, role); unit
 *                     quaternions (what hqmq_build_codebooks makes).  Components must stay below
 *                     32 in magnitude (they pass through fp16 parts scaled by 2^10).
 *   enc               HOST struct of DEVICE pointers (see hqmq_encoded), sized per hqmq_sizes.
 *   outlier_capacity  entries (chunks) available in enc->outliers; outlier_capacity_max always
 *                     suffices.  If fewer, surplus outliers are dropped, status gets
 *                     HQMQ_STATUS_OUTLIER_OVERFLOW and n_outliers / row_off still hold the true
 *                     counts so the caller can retry.
 *   workspace_dev     DEVICE scratch, 256-byte aligned, at least workspace_bytes; contents
 *                     need not be preserved or initialised.
 *   stream            hipStream_t.
 * Two calls may run concurrently only with distinct workspaces and outputs. */
int32_t hqmq_encode(const hqmq_params *params, const void *x_dev, const float *sec_dev,
                    const hqmq_encoded *enc, uint64_t outlier_capacity, void *workspace_dev,
                    uint64_t workspace_bytes, void *stream);

/* hqmq_encode for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Identical to hqmq_encode in arguments,
 * results and errors, except that the workspace is an array of HQMQ_STATIC_SCRATCH_BYTES inside the
 * library's own device image (every GPU the library runs on holds one copy of it until the process ends);
 * the call allocates and frees nothing.
 *   - Shapes whose hqmq_sizes().workspace_bytes exceeds HQMQ_STATIC_SCRATCH_BYTES are rejected with
 *     HQMQ_ERR_BUFFER_TOO_SMALL and nothing is enqueued (16 MiB covers H <= 48 kv heads at S = 256; the
 *     need grows with H, S and the number of row blocks B*H*T/64).
 *   - Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (different streams or
 *     threads) race on it and give undefined results; calls ordered on one stream are fine.  What must
 *     start at zero is cleared by the call's first kernel, so the previous call's contents do not matter.
 *   - hqmq_thresholds cannot read this workspace; use hqmq_encode when the thresholds are wanted.
 *   - The array's address is looked up by the per-device set-up (hqmq_init): before a stream capture,
 *     call hqmq_init() on the device once. */
#define HQMQ_STATIC_SCRATCH_BYTES (16u << 20)
int32_t hqmq_encode_static(const hqmq_params *params, const void *x_dev, const float *sec_dev,
                           const hqmq_encoded *enc, uint64_t outlier_capacity, void *stream);

/* hqmq_encode with measurement marks: an entry point of this library's own, for callers who want the
 * encode's time split by phase (the paper reports no encode timing at all; its latency tables, App. E /
 * Sec. 4.10, are per call of a whole kernel).
 * phase_events: HOST array of 4 caller-created hipEvent_t (any entry, or the array, may be
 * NULL), recorded on `stream`: [0] before the first kernel, [1] after the median select,
 * [2] after the search kernel (flags, scales, codes), [3] after the outlier list (scan and
 * payload gather).  Otherwise identical to hqmq_encode. */
int32_t hqmq_encode_timed(const hqmq_params *params, const void *x_dev, const float *sec_dev,
                          const hqmq_encoded *enc, uint64_t outlier_capacity, void *workspace_dev,
                          uint64_t workspace_bytes, void *stream, void *const *phase_events);

/* Decode one tensor (Alg. 1 "Decode", App. D "Decode"): x_hat = r_hat * (q_p * q_s) with
 * r_hat = r_q * sigma / (2^b_r - 1) and the Hamilton product taken at decode time, rounded to
 * fp16; flagged chunks are restored from the outlier list.
 *   params   HOST; B, H, T, D, S, b_r and the strides (of out_dev) are used.
 *   enc      HOST struct of DEVICE pointers as produced by hqmq_encode (n_outliers and status
 *            are not read).  Codes must hold k < 24*S.
 *   outlier_capacity  entries available in enc->outliers; a flagged chunk whose list position
 *            lies beyond it (an encode that overflowed) decodes to zeros.
 *   sec_dev  DEVICE, fp32 [H][S][4], the same codebooks used to encode.
 *   out_dev  DEVICE, out, fp16, 16-byte aligned, addressed with params strides.
 *   stream   hipStream_t. */
int32_t hqmq_decode(const hqmq_params *params, const hqmq_encoded *enc, uint64_t outlier_capacity,
                    const float *sec_dev, void *out_dev, void *stream);

/* Incremental encode: as hqmq_encode, for the few token rows a generation step appends, with the
 * outlier thresholds SUPPLIED by the caller instead of taken from the call's own median (the
 * median over the 32 B T chunks of a one-token tensor means nothing; Sec. 3 "Median-multiplier
 * outlier extraction" leaves a running estimate for short contexts to the implementation).
 *   thr_dev  DEVICE, fp64 [H]: a chunk of head h is flagged iff its squared norm r^2 > thr_dev[h]
 *            (for the paper's rule with a running median estimate r_med: thr = (C r_med)^2; to
 *            freeze the prefill's thresholds pass what hqmq_thresholds returned).  params->C is
 *            not used; HQMQ_FLAG_NO_OUTLIERS is rejected (INVALID_ARG).
 * Everything else (buffers, sizes from hqmq_sizes for THIS small shape, ordering of the outlier
 * list, errors) is as in hqmq_encode; the encoded rows form a tensor of their own.  One bound of
 * hqmq_sizes does not carry over: with arbitrary thresholds every chunk may be flagged, so a list
 * that can never overflow needs n_rows * chunks_per_row entries (an overflow is reported in status as usual). */
int32_t hqmq_encode_given_thresholds(const hqmq_params *params, const void *x_dev, const float *sec_dev,
                                     const double *thr_dev, const hqmq_encoded *enc,
                                     uint64_t outlier_capacity, void *workspace_dev,
                                     uint64_t workspace_bytes, void *stream);

/* hqmq_encode_given_thresholds for n_tensors tensors of one shape in one call (e.g. the new K and
 * V rows of every layer of a generation step): up to 32 tensors per kernel launch, arguments as in
 * hqmq_encode_batch plus thr_dev, a HOST array of n_tensors DEVICE pointers to fp64 [H]. */
int32_t hqmq_encode_batch_given_thresholds(const hqmq_params *params, int32_t n_tensors,
                                           const void *const *x_dev, const float *const *sec_dev,
                                           const double *const *thr_dev, const hqmq_encoded *enc,
                                           const uint64_t *outlier_capacity, void *workspace_dev,
                                           uint64_t workspace_bytes, void *stream);

/* The thresholds on squared chunk norms, fp64 [H], that the last encode using this workspace
 * applied (fl(fl(C C) median(r^2)) per head, Sec. 3; +infinity with HQMQ_FLAG_NO_OUTLIERS): a
 * stream-ordered device-to-device copy of H doubles, e.g. to seed or update a caller's running
 * estimate.  slice: 0 for hqmq_encode; for hqmq_encode_batch the index of the tensor within its
 * launch group of 32.  workspace_bytes: the size of the caller's workspace, as passed to the encode.
 * Errors: INVALID_ARG (null / misaligned pointer, slice outside 0..31), UNSUPPORTED (params),
 * BUFFER_TOO_SMALL (the slice does not lie inside workspace_bytes), HIP. */
int32_t hqmq_thresholds(const hqmq_params *params, const void *workspace_dev, uint64_t workspace_bytes,
                        int32_t slice, double *thr_out_dev, void *stream);

/* The median of a cache whose TOKEN axis is split over several shards (context-parallel serving:
 * each GPU holds a slice of T of the same (layer, role) tensor).  Sec. 3 "Median-multiplier outlier
 * extraction" takes the median per (layer, head, role) over the whole batch, so the shards must agree
 * on it; everything else of the encode is local to a shard.  The select is a radix select that
 * exchanges nothing but histograms:
 *     for pass = 0 .. 5:   every shard calls hqmq_shard_median_pass(pass) on its slice; the caller then
 *                          SUMS the region hqmq_shard_median_region(pass) names (uint32 counters inside
 *                          the shard's workspace) over all shards and writes the sums back into every
 *                          shard's workspace (one all-reduce of 32 KiB * H for pass 0, 4 KiB * H after)
 *     pass = 6:            every shard calls hqmq_shard_median_pass(6): the thresholds
 *                          fl(fl(C*C) * median) are now in its workspace, the same on every shard;
 *                          read them with hqmq_thresholds(params, workspace, 0, ...) and encode the slice
 *                          with hqmq_encode_given_thresholds.
 * Pass 0 counts bits 62..50 of the squared norms' bit patterns, passes 1..5 the next 10 bits each of
 * the keys under the prefix fixed so far; the result is the exact lower median of all shards' chunks,
 * whatever the values (no candidate lists that could overflow).
 *   params                 HOST; THIS shard's shape and strides (B, H, D, S, b_r equal on all shards; T may
 *                          differ); C is used by pass 6; HQMQ_FLAG_NO_OUTLIERS is rejected (INVALID_ARG).
 *   total_chunks_per_head  B * ceil(D/4) * (sum of T over all shards): the same number on every shard
 *                          and in every pass; < 2^32 (else UNSUPPORTED), >= this shard's own count.
 *   pass                   0..5 a counting pass, 6 the finish.  Passes must run in order; the summed
 *                          histogram of pass p must be in place before pass p + 1 is enqueued.
 *   x_dev                  DEVICE, this shard's slice, as for hqmq_encode (not read by pass 6, where it
 *                          may be NULL).
 *   workspace_dev          DEVICE, 256-byte aligned, >= hqmq_sizes(params).workspace_bytes; holds the
 *                          select's state between the calls, so nothing else may use it meanwhile.
 * hqmq_shard_median_region: HOST function; byte offset inside the workspace and number of uint32
 * counters of the histogram that pass 0..5 leaves behind. */
int32_t hqmq_shard_median_pass(const hqmq_params *params, uint64_t total_chunks_per_head, int32_t pass,
                               const void *x_dev, void *workspace_dev, uint64_t workspace_bytes, void *stream);
int32_t hqmq_shard_median_region(const hqmq_params *params, int32_t pass, uint64_t *offset_bytes,
                                 uint64_t *n_counters);

/* Encode n_tensors tensors of ONE shape (the same params: e.g. the K and V of every layer of the
 * current batch, Alg. 1 applied per (layer, role)) with as few launches as possible: up to 32
 * tensors share each kernel launch, which removes the launch gaps and small-kernel tails of the
 * per-tensor sequence.  Semantics per tensor are exactly hqmq_encode's.
 *   x_dev, sec_dev, enc, outlier_capacity   HOST arrays of n_tensors entries (device pointers /
 *            structs of device pointers); the tensors must not overlap.
 *   workspace_dev   DEVICE scratch, 256-byte aligned, min(n_tensors, 32) * workspace_bytes(of
 *            hqmq_sizes) bytes: one slice per tensor of a launch group.
 *   phase_events    NULL, or 4 hipEvent_t as in hqmq_encode_timed (entries may be NULL): [0] is
 *            recorded before the first launch, [1..3] after the select / search / outlier-list
 *            phase of EVERY group of 32 tensors, so with more than 32 tensors they hold the times
 *            of the last group; time groups of at most 32 with one call each.
 * Errors: as hqmq_encode; INVALID_ARG also for n_tensors <= 0 or a null array. */
int32_t hqmq_encode_batch(const hqmq_params *params, int32_t n_tensors, const void *const *x_dev,
                          const float *const *sec_dev, const hqmq_encoded *enc,
                          const uint64_t *outlier_capacity, void *workspace_dev,
                          uint64_t workspace_bytes, void *stream, void *const *phase_events);

/* Decode n_tensors tensors of ONE shape (the same params: e.g. the K and V caches of every layer)
 * with as few launches as possible: up to 32 tensors share a launch, which keeps the GPU streaming
 * across tensor boundaries (the paper's deployment setting decodes the whole cache, Sec. 4.10
 * "Memory and latency").  Semantics per tensor are exactly hqmq_decode's.
 *   enc, outlier_capacity, sec_dev, out_dev   HOST arrays of n_tensors entries; sec_dev[i] and
 *            out_dev[i] are DEVICE pointers, enc[i] a struct of DEVICE pointers.
 * Errors: as hqmq_decode; INVALID_ARG also for n_tensors <= 0 or a null array. */
int32_t hqmq_decode_batch(const hqmq_params *params, int32_t n_tensors, const hqmq_encoded *enc,
                          const uint64_t *outlier_capacity, const float *const *sec_dev,
                          void *const *out_dev, void *stream);

/* Single-query attention read straight from a packed K cache and a packed V cache (the paper's
 * fused attention kernel, App. F: O = softmax(Q K^T * scale) V with K and V reconstructed inside
 * the attention loop and never materialised), for ONE query token per sequence (the generation
 * step).  Query head hq attends to kv head hq / (n_q_heads / H) (grouped-query attention); all T
 * cached tokens are visible.  K_hat and V_hat are exactly the fp16 tensors hqmq_decode would
 * return; their products with Q and with the softmax weights are accumulated in fp32 (the
 * weights enter with about 22 significant bits), the softmax subtracts the running maximum
 * (online form), and the result is rounded once to fp16.
 *   params     HOST; B, H, T, D, S, b_r describe BOTH caches (strides are ignored).
 *   n_q_heads  a multiple of H, at most 16 * H.  Several query tokens that all see the whole cache
 *              (a few speculative or chunked decode positions) can ride along as extra query
 *              heads of their kv head: lay q out as [B][H][tokens * heads_per_kv][D] and pass
 *              n_q_heads = H * tokens * heads_per_kv <= 16 * H.
 *   q_dev      DEVICE, fp16 [B][n_q_heads][D] contiguous, 16-byte aligned.
 *   scale      softmax scale (usually 1/sqrt(D)); finite.
 *   enc_k, enc_v, cap_k, cap_v, sec_k_dev, sec_v_dev   as enc / outlier_capacity / sec_dev of
 *              hqmq_decode, for the key and the value cache.
 *   out_dev    DEVICE, out, fp16 [B][n_q_heads][D] contiguous, 16-byte aligned.
 *   workspace_dev  DEVICE scratch, 256-byte aligned, hqmq_attend_workspace_bytes() bytes; owned
 *              by the caller, contents undefined afterwards; concurrent calls need their own.
 *   stream     hipStream_t; two kernels are enqueued, nothing is synchronised or allocated.
 * Errors: INVALID_ARG (null / misaligned pointer, bad n_q_heads, non-finite scale), UNSUPPORTED
 * (params the decode rejects, D other than 64, 96, 128, more than 16 query heads per kv head),
 * BUFFER_TOO_SMALL, HIP. */
int32_t hqmq_attend(const hqmq_params *params, int32_t n_q_heads, const void *q_dev, float scale,
                    const hqmq_encoded *enc_k, uint64_t cap_k, const float *sec_k_dev,
                    const hqmq_encoded *enc_v, uint64_t cap_v, const float *sec_v_dev, void *out_dev,
                    void *workspace_dev, uint64_t workspace_bytes, void *stream);

/* hqmq_attend that also returns, per query head, the natural logarithm of the softmax denominator,
 * lse = ln(sum_t exp(scale * <q, K_hat_t>)): what is needed to combine attention results over
 * several token ranges exactly (a cache kept as a prefill tensor plus tensors of appended tokens, or
 * a recent-token tail the caller holds in fp16): with parts (o_i, lse_i) the whole is
 * o = sum_i exp(lse_i - L) o_i, L = ln(sum_i exp(lse_i)).
 *   lse_dev    DEVICE, out, fp32 [B][n_q_heads], 4-byte aligned.
 * Everything else, and the errors, as hqmq_attend (INVALID_ARG also for a null or misaligned lse_dev). */
int32_t hqmq_attend_lse(const hqmq_params *params, int32_t n_q_heads, const void *q_dev, float scale,
                        const hqmq_encoded *enc_k, uint64_t cap_k, const float *sec_k_dev,
                        const hqmq_encoded *enc_v, uint64_t cap_v, const float *sec_v_dev, void *out_dev,
                        float *lse_dev, void *workspace_dev, uint64_t workspace_bytes, void *stream);

/* hqmq_attend with a causal limit per query head, for steps that carry several query tokens (a few
 * speculative or chunked positions riding along as extra query heads, see n_q_heads): query head hq
 * sees only the first visible_dev[b][hq] cached tokens, t < visible (the paper's fused kernel applies
 * the causal mask, App. F; with one query token per sequence the mask is empty).  Values above T mean
 * T; a head that may see nothing gets zeros and lse = -infinity.
 *   visible_dev  DEVICE, in, int32 [B][n_q_heads], 4-byte aligned, values >= 0.
 *   lse_dev      DEVICE, out, fp32 [B][n_q_heads] as in hqmq_attend_lse, or NULL.
 * Everything else, and the errors, as hqmq_attend (INVALID_ARG also for a null or misaligned
 * visible_dev). */
int32_t hqmq_attend_masked(const hqmq_params *params, int32_t n_q_heads, const void *q_dev, float scale,
                           const hqmq_encoded *enc_k, uint64_t cap_k, const float *sec_k_dev,
                           const hqmq_encoded *enc_v, uint64_t cap_v, const float *sec_v_dev,
                           const int32_t *visible_dev, void *out_dev, float *lse_dev, void *workspace_dev,
                           uint64_t workspace_bytes, void *stream);

/* Workspace hqmq_attend needs for these params and n_q_heads, in bytes (0 if they are invalid). */
uint64_t hqmq_attend_workspace_bytes(const hqmq_params *params, int32_t n_q_heads);

/* hipError_t value of the last failed HIP call made by this library on the calling thread
 * (0 if none). */
int32_t hqmq_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* HQMQ_H */
