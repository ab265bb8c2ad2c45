/*
 * aqsgd.h -- C ABI of the MI355X stage-boundary codec of AQ-SGD
 * ("Fine-tuning Language Models over Slow Networks using Activation
 * Quantization with Guarantees", NeurIPS 2022).
 *
 * Between two pipeline stages the method does not quantise the activation a(xi)
 * of training sample xi itself, but its change against m(xi), the message the
 * two stages exchanged the last time they saw xi, which both keep (Algorithm 1;
 * Algorithm 2 is the two-machine view):
 *
 *     sender:    Delta m = Q(a(xi) - m(xi));  m(xi) <- m(xi) + Delta m;  send Delta m
 *     receiver:  m(xi) <- m(xi) + Delta m;    the next stage consumes m(xi)
 *     backward:  receiver sends Q(gradient w.r.t. the activation), directly
 *
 * Q (Section 4.1) normalises a group of G consecutive elements by its max-abs s
 * and maps each onto one of 2^b equally spaced levels on [-s, s]; rounding is to
 * nearest (ties upwards) or stochastic (unbiased, as Theorem 3.1 requires).
 *
 * General rules for every entry point
 *   - Every data pointer is DEVICE memory on the current HIP device, owned by the
 *     caller before, during and after the call.  The codec calls allocate no device
 *     memory, keep no state between calls and may be made from several host threads
 *     at once.  Descriptors and job lists are HOST memory and are read before the
 *     call returns.  Three things are stateful, and say so where they are declared:
 *     the launch-shape knobs (process-wide atomics, aqsgd_set_launch_shape), the
 *     request to time the next launch (per host thread, aqsgd_profile_next_launch)
 *     and the host-memory tier (an object that owns events, a worker thread and
 *     host bookkeeping, aqsgd_tier_*).
 *   - Calls only enqueue work on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream) and return; results are valid once the stream reaches
 *     that point.  Ordering between a sender's and a receiver's stream is the
 *     caller's business (events).
 *   - Tensors are dense, row-major.  act/grad/out are [batch, n_per]; m_buf is
 *     [n_samples, n_per]; all in `dtype`.  Groups tile the flattened call tensor:
 *     group g covers elements [g*group, (g+1)*group); n_per must be a multiple of
 *     `group`, so a group never spans two samples.  "Per-row" scaling is
 *     group == hidden size.
 *   - codes: the b-bit level index of flat element j occupies bits [j*b, j*b+b) of
 *     the byte stream, bit k of the stream being bit (k mod 8) of byte k/8.
 *     aqsgd_codes_bytes() bytes.  scales: one binary32 max-abs per group,
 *     aqsgd_scales_count() floats; a scale of 0 means "group unchanged".
 *   - Alignment: act, grad, out, m_buf and codes 16 bytes, scales 4, ids 8.
 *   - Return value: AQSGD_OK or a negative aqsgd_status.  Everything the host can
 *     check is checked before any work is enqueued; on error nothing is enqueued.
 *     NOT checked: sample ids outside [0, n_samples) (out-of-bounds accesses),
 *     duplicate ids within one call (two rows of the call race on one row of
 *     m_buf: undefined results, all accesses in bounds), non-finite inputs
 *     (undefined results), buffers smaller than the descriptor says.
 *     aqsgd_check_ids() checks the first two on the device.  AQSGD_ERR_LAUNCH
 *     reports the status of the call's own launch.
 *   - Arithmetic is IEEE binary32 with one rounding per operation and no fused
 *     multiply-add; stores to float16/bfloat16 round to nearest-even.  Results are
 *     bit-identical for any launch configuration.
 */
#ifndef AQSGD_H
#define AQSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { AQSGD_F32 = 0, AQSGD_F16 = 1, AQSGD_BF16 = 2 } aqsgd_dtype;
typedef enum { AQSGD_ROUND_NEAREST = 0, AQSGD_ROUND_STOCHASTIC = 1 } aqsgd_round;

typedef enum {
    AQSGD_OK = 0,
    AQSGD_ERR_NULL = -1,      /* a required pointer is NULL                         */
    AQSGD_ERR_BITS = -2,      /* bits not in {2, 3, 4, 6, 8}                        */
    AQSGD_ERR_GROUP = -3,     /* group <= 0, n_per % group != 0, (group*bits) % 8   */
    AQSGD_ERR_DTYPE = -4,     /* unknown dtype or rounding mode                     */
    AQSGD_ERR_SHAPE = -5,     /* negative or overflowing batch / n_per / n_samples  */
    AQSGD_ERR_ALIGN = -6,     /* a pointer misses its alignment                     */
    AQSGD_ERR_LAUNCH = -7,    /* the HIP runtime refused the launch                 */
    AQSGD_ERR_IO = -8         /* file tier: open / read / write failed              */
} aqsgd_status;

/* Shape and settings of one call (host memory). */
typedef struct {
    int64_t batch;        /* B: samples in this call (0 is allowed: nothing happens) */
    int64_t n_per;        /* elements per sample (sequence length * hidden size)     */
    int64_t n_samples;    /* N: rows of m_buf; ignored by the two grad calls         */
    int32_t bits;         /* b in {2, 3, 4, 6, 8}                                    */
    int32_t group;        /* G: elements per scale                                   */
    int32_t dtype;        /* aqsgd_dtype of act / grad / m_buf / out                 */
    int32_t rounding;     /* aqsgd_round; decode and grad_dequant ignore it          */
    uint64_t rng_seed;    /* key of the stochastic rounding; use a fresh one per     */
                          /* message.  Ignored for AQSGD_ROUND_NEAREST               */
} aqsgd_desc;

/* Bytes of `codes` and number of `scales` for a call of this shape (0 on a bad desc). */
size_t aqsgd_codes_bytes(const aqsgd_desc* desc);
size_t aqsgd_scales_count(const aqsgd_desc* desc);

/*
 * Sender side of the forward message (Algorithm 2, the block for network a;
 * Algorithm 1's update of m).  For each sample i of the call, with row = sample_ids[i]:
 *     delta = act[i] - m_buf[row]                     (binary32)
 *     codes, scales <- Q(delta)                       (Section 4.1)
 *     m_buf[row] <- dtype(m_buf[row] + Q(delta))      (in place)
 * m_buf starts as all zeros (Algorithm 1's initialisation), which makes the first
 * visit of a sample a direct quantisation of its activation.
 *   act         in   [batch, n_per]
 *   sample_ids  in   int64[batch], distinct, each in [0, n_samples)
 *   m_buf       i/o  [n_samples, n_per], the sender's copy
 *   codes       out  aqsgd_codes_bytes() bytes
 *   scales      out  aqsgd_scales_count() floats
 */
int aqsgd_encode(const aqsgd_desc* desc, const void* act, const int64_t* sample_ids,
                 void* m_buf, uint8_t* codes, float* scales, void* stream);

/*
 * Receiver side (Algorithm 2, the block for network b): applies the same update to the
 * receiver's copy of m and hands m(xi) on as the activation of the next stage.
 *     m_buf[row] <- dtype(m_buf[row] + Q^-1(codes, scales));  out[i] <- m_buf[row]
 * After matching encode/decode calls the two copies of m_buf are bit-identical.
 *   codes, scales  in   as produced by aqsgd_encode with the same desc
 *   m_buf          i/o  [n_samples, n_per], the receiver's copy
 *   out            out  [batch, n_per]
 */
int aqsgd_decode(const aqsgd_desc* desc, const uint8_t* codes, const float* scales,
                 const int64_t* sample_ids, void* m_buf, void* out, void* stream);

/*
 * Backward message (Algorithm 1, the step in which machine b returns the quantised
 * gradient): direct quantisation of the activation-gradient, no buffer.
 *   grad  in  [batch, n_per];  codes, scales out as above.
 */
int aqsgd_grad_quant(const aqsgd_desc* desc, const void* grad, uint8_t* codes,
                     float* scales, void* stream);

/* Reconstruction of the backward message on the sender: out <- dtype(Q^-1(codes, scales)). */
int aqsgd_grad_dequant(const aqsgd_desc* desc, const uint8_t* codes, const float* scales,
                       void* out, void* stream);

/*
 * Several independent messages in as few launches as possible.
 *
 * The two stages of a boundary each have two kinds of message to handle at about the
 * same time (Algorithm 2: network a sends the activation change and reconstructs the
 * returned gradient, network b reconstructs the activation and sends the gradient), a
 * stage in the middle of a pipeline has two boundaries, and Appendix A.1's K machines
 * are K-1 independent instances.  A launch of a few tens of MB spends a good part of its
 * time filling and draining the GPU, so messages that are ready together should share a
 * grid.  Each job is exactly one of the four calls above (or one of the two first-visit
 * variants of encode and decode), with the same arguments, meaning, alignment and
 * preconditions:
 *   AQSGD_JOB_ENCODE        src = act,  sample_ids, m_buf (i/o), codes and scales (out)
 *   AQSGD_JOB_DECODE        codes and scales (in), sample_ids, m_buf (i/o), out
 *   AQSGD_JOB_GRAD_QUANT    src = grad, codes and scales (out)
 *   AQSGD_JOB_GRAD_DEQUANT  codes and scales (in), out
 * Unused pointers of a job are ignored.  The jobs of one call must be independent: none
 * reads what another writes, and no two touch the same row of the same m_buf; they run
 * concurrently, in no particular order.  Results are bit-identical to the single calls.
 * How jobs share launches: quantising jobs (ENCODE, GRAD_QUANT) with the same dtype,
 * rounding and group-size class share one grid whatever their bit widths, and the
 * dequantising jobs of that dtype join it; dequantising jobs without such a host share a grid of their own; up to
 * 8 + 8 jobs per grid, more are split; jobs whose group is not a multiple of 8 or larger
 * than 32768 run on their own.  The typical stage-side call (one ENCODE and one
 * GRAD_DEQUANT, or one DECODE and one GRAD_QUANT) is one launch.
 * Every job is checked first; on an error (the first bad job's status, or
 * AQSGD_ERR_SHAPE for an unknown kind or a negative count) nothing is enqueued.
 */
typedef enum {
    AQSGD_JOB_ENCODE = 0, AQSGD_JOB_DECODE = 1, AQSGD_JOB_GRAD_QUANT = 2, AQSGD_JOB_GRAD_DEQUANT = 3,
    /* the two calls of Algorithm 1 with its first-visit branch (declared further down),
     * same arguments and rules as aqsgd_encode_seen / aqsgd_decode_seen: */
    AQSGD_JOB_ENCODE_SEEN = 4,    /* ENCODE's pointers + seen (i/o), stamp, first (out)      */
    AQSGD_JOB_DECODE_SEEN = 5     /* DECODE's pointers + full (in), seen (i/o), stamp        */
} aqsgd_job_kind;

typedef struct {
    int32_t kind;                 /* aqsgd_job_kind                                   */
    aqsgd_desc desc;
    const void* src;              /* act (ENCODE) or grad (GRAD_QUANT)                */
    const int64_t* sample_ids;    /* ENCODE, DECODE                                   */
    void* m_buf;                  /* ENCODE, DECODE                                   */
    uint8_t* codes;               /* written by the quantising, read by the other jobs */
    float* scales;
    void* out;                    /* DECODE, GRAD_DEQUANT                             */
    uint32_t* seen;               /* the *_SEEN kinds: one word per sample of m_buf   */
    int32_t* first;               /* ENCODE_SEEN: [batch], 1 where the sample was new */
    const void* full;             /* DECODE_SEEN: uncompressed rows of the new samples */
    uint32_t stamp;               /* the *_SEEN kinds: this call's stamp, non-zero    */
    uint32_t reserved;            /* 0                                                */
} aqsgd_job;

int aqsgd_run_jobs(const aqsgd_job* jobs, int32_t n_jobs, void* stream);

/*
 * Uncompressed first visit (Algorithm 1's branch for a sample without a previous
 * message; Appendix D runs a whole warm-up epoch this way): the message is the
 * activation itself, at full precision, and both stages store it as m(xi).
 *     m_buf[sample_ids[i]] <- act[i]        for every sample i of the call
 * The sender calls it with its activation, the receiver with the activation it
 * received, which keeps the two copies identical.  A later aqsgd_encode of the same
 * activation finds a zero change.  Only batch, n_per, n_samples and dtype of the
 * descriptor are used; bits, group and rounding are ignored (but must be valid).
 *   act         in   [batch, n_per]
 *   sample_ids  in   int64[batch], distinct, each in [0, n_samples)
 *   m_buf       i/o  [n_samples, n_per]
 */
int aqsgd_seed(const aqsgd_desc* desc, const void* act, const int64_t* sample_ids,
               void* m_buf, void* stream);

/*
 * Algorithm 1 with its first-visit branch (a sample without a previous message: the
 * activation is sent in full precision and m(xi) <- a(xi); otherwise the quantised
 * change is sent).  One launch per call.
 * `seen` holds one 32-bit word per sample of m_buf, zero-initialised by the caller:
 * 0 = no previous message yet, otherwise the stamp of the call that first visited the
 * sample.  Every call carries a `stamp` of the caller's choosing that is not 0 and
 * that no earlier call on this buffer has used (a running call counter does); a sample
 * is new to a call if its word is 0.  Both stages keep their own `seen`; they stay
 * identical (as zero / non-zero patterns) because both see the same sample ids.  The
 * stamps of the two stages need not agree.  Reusing a stamp makes the samples first
 * visited under it count as new once more (they are sent in full again: wasteful, but
 * both stages still agree as long as they reuse alike).
 *   aqsgd_encode_seen   new samples: m_buf[id] <- act[i], first[i] = 1, their slices of
 *                       codes / scales are NOT written (row i of act is the message);
 *                       other samples: exactly aqsgd_encode, first[i] = 0
 *   aqsgd_decode_seen   new samples: m_buf[id] <- full[i], out[i] <- full[i];
 *                       other samples: exactly aqsgd_decode (their rows of full are not read)
 * Both store the call's stamp in the words of the new samples.
 *   seen    i/o  uint32[n_samples], device, 4-byte aligned
 *   stamp   in   non-zero (else AQSGD_ERR_SHAPE)
 *   first   out  int32[batch], device, 4-byte aligned
 *   full    in   [batch, n_per] of desc.dtype, 16-byte aligned: the uncompressed rows
 * Everything else (arguments, alignment, preconditions, status codes) as in
 * aqsgd_encode / aqsgd_decode.
 */
int aqsgd_encode_seen(const aqsgd_desc* desc, const void* act, const int64_t* sample_ids,
                      void* m_buf, uint32_t* seen, uint32_t stamp, int32_t* first, uint8_t* codes,
                      float* scales, void* stream);
int aqsgd_decode_seen(const aqsgd_desc* desc, const uint8_t* codes, const float* scales,
                      const void* full, const int64_t* sample_ids, void* m_buf, uint32_t* seen,
                      uint32_t stamp, void* out, void* stream);

/*
 * Previous messages kept at low precision ("m z", Appendix H.5: z bits for the
 * previous messages; the appendix reports z = 8 and z = 2).  m(xi) is stored as z-bit
 * levels plus one binary32 scale per group, produced by the same Q with nearest
 * rounding; the group is the descriptor's.  Both stages work from the stored value
 * m^ = Q_z^-1(stored):
 *     sender:    Delta m = Q_b(act - m^)  -> codes, scales;   v = m^ + Delta m;  store Q_z(v)
 *     receiver:  v = m^ + Q_b^-1(codes, scales);  out = dtype(v);                store Q_z(v)
 * All-zero storage decodes to m^ = 0, so a first visit is direct quantisation.  After
 * matching calls the two stages' storage is bit-identical.
 *   m_bits    2 or 8 (else AQSGD_ERR_BITS)
 *   m_codes   i/o  uint8 [n_samples, aqsgd_lowbit_row_bytes()], level e of a row at bits
 *                  [e*z, e*z+z) of the row's byte stream
 *   m_scales  i/o  float [n_samples, n_per / group]
 *   group must be a multiple of 8 and at most 16384 here (else AQSGD_ERR_GROUP).
 * Everything else as in aqsgd_encode / aqsgd_decode.
 */
size_t aqsgd_lowbit_row_bytes(const aqsgd_desc* desc, int32_t m_bits);
int aqsgd_encode_lowbit(const aqsgd_desc* desc, int32_t m_bits, const void* act,
                        const int64_t* sample_ids, uint8_t* m_codes, float* m_scales,
                        uint8_t* codes, float* scales, void* stream);
int aqsgd_decode_lowbit(const aqsgd_desc* desc, int32_t m_bits, const uint8_t* codes,
                        const float* scales, const int64_t* sample_ids, uint8_t* m_codes,
                        float* m_scales, void* out, void* stream);

/*
 * Sparsified backward message ("bw8[0.2]", Appendix H.6: only the largest fifth of
 * the gradient entries is sent, at 8 bits).  The appendix gives no format; here, per
 * group of `group` consecutive entries, the `keep` entries of largest magnitude are
 * sent (equal magnitudes: the lower index first) as levels of the same Q with the
 * group's max-abs scale; every other entry reconstructs as +0.
 *   desc     bits must be 8 (else AQSGD_ERR_BITS); group a multiple of 8, at most 2048
 *            (else AQSGD_ERR_GROUP); batch * n_per entries; n_samples unused
 *   keep     1 .. group (else AQSGD_ERR_SHAPE)
 *   grad     in   [batch, n_per] of desc.dtype, 16-byte aligned, no NaN
 *   bitmap   out/in  uint8[batch * n_per / 8]: entry j kept <=> bit j % 8 of byte j / 8
 *   codes    out/in  uint8[n_groups * keep]: a group's levels in ascending entry order;
 *            16-byte aligned when keep is a multiple of 16
 *   scales   out/in  float[n_groups], n_groups = batch * n_per / group
 *   out      out  [batch, n_per] of desc.dtype
 * A receiver handed a bitmap with more than `keep` bits in a group returns unspecified
 * values for that group (no access leaves the buffers).  All pointers are DEVICE
 * pointers owned by the caller; the calls enqueue on `stream` and return.
 */
size_t aqsgd_topk_bitmap_bytes(const aqsgd_desc* desc);
size_t aqsgd_topk_codes_bytes(const aqsgd_desc* desc, int32_t keep);
int aqsgd_grad_topk_quant(const aqsgd_desc* desc, int32_t keep, const void* grad, uint8_t* bitmap,
                          uint8_t* codes, float* scales, void* stream);
int aqsgd_grad_topk_dequant(const aqsgd_desc* desc, int32_t keep, const uint8_t* bitmap,
                            const uint8_t* codes, const float* scales, void* out, void* stream);

/*
 * Tiers below HBM for the previous messages (the implementation notes of Section 3.3
 * and Appendix G: m(xi) lives in host memory or on an SSD, is brought to the GPU before
 * the forward pass of its sample and goes back after the update, both behind the
 * computation of other samples).
 *
 * HBM holds `slots` windows of `batch` rows.  A micro-batch's rows are brought into a
 * window ahead of time (prefetch), the codec runs on the window with the window's row
 * numbers as its sample ids (acquire), and the updated rows go back afterwards (release).
 * The tier object is the stateful part of this library: it owns HIP events, which samples
 * each window holds and, for the file tier, a file descriptor and a worker thread.  It
 * never owns data memory: dev_rows [slots*batch, row_bytes] and dev_row_ids int64
 * [slots*batch] are the caller's device memory, the host memory below the caller's pinned
 * host memory (hipHostMalloc / a pinned tensor).  Calls on one tier must come from one host
 * thread, and every call that takes a copy stream must name the same one (the order of
 * its copies keeps a write-back ahead of a later prefetch of the same window or sample;
 * another stream is refused with AQSGD_ERR_SHAPE).
 *
 *   aqsgd_tier_create       host tier: host_rows [n_samples, row_bytes] pinned holds every row
 *   aqsgd_tier_create_file  file tier: the rows live in the file `path` (created or extended to
 *                           n_samples * row_bytes; bytes never written read as zeros, Algorithm
 *                           1's initial m); staging_rows [slots*batch, row_bytes] pinned is the
 *                           only host memory.  A worker thread reads a window's rows into the
 *                           staging rows and issues their copy to the device (read-ahead: up to
 *                           `slots` windows ahead of the compute), and writes released rows back
 *                           once they have arrived from the device (write-behind).  direct_io != 0
 *                           opens the file unbuffered (O_DIRECT), which needs row_bytes to be a
 *                           multiple of 4096 (else AQSGD_ERR_ALIGN); the tier then also owns one
 *                           window of ordinary host memory, through which the file transfers
 *                           pass (the kernel cannot do unbuffered I/O on pinned GPU-visible pages).
 *   both fill dev_row_ids with 0 .. slots*batch-1 (synchronously) and create the events
 *   prefetch  window <- rows of host_ids (HOST int64[batch], distinct), on copy_stream;
 *             a window must be released before it is prefetched again, and a sample that
 *             sits in an unreleased window cannot be prefetched (its newest row is in that
 *             window, not below): both are refused with AQSGD_ERR_SHAPE.  If a copy cannot
 *             be issued the window stays empty
 *   acquire   makes compute_stream wait for the window's rows (file tier: first blocks the
 *             host until the worker has read them from the file); returns the sample_ids
 *             pointer (device, batch entries) to pass to the codec with m_buf = dev_rows,
 *             n_samples = slots*batch
 *   release   after the codec calls queued so far on compute_stream, sends the window's
 *             rows back on copy_stream (file tier: and from the staging rows to the file)
 *   drain     blocks until every copy and file transfer issued so far has finished
 *   destroy   drains, stops the worker, closes the file, destroys the events
 * Return: AQSGD_OK, AQSGD_ERR_NULL / _SHAPE / _ALIGN for bad arguments, AQSGD_ERR_LAUNCH if
 * the HIP runtime fails, AQSGD_ERR_IO if the file cannot be opened, sized, read or written
 * (a failure inside the worker is reported by the next acquire, release, prefetch or drain).
 */
typedef struct aqsgd_tier aqsgd_tier;
int aqsgd_tier_create(aqsgd_tier** tier, void* host_rows, void* dev_rows, int64_t* dev_row_ids,
                      int64_t n_samples, int64_t row_bytes, int32_t slots, int32_t batch);
int aqsgd_tier_create_file(aqsgd_tier** tier, const char* path, int32_t direct_io, void* staging_rows,
                           void* dev_rows, int64_t* dev_row_ids, int64_t n_samples,
                           int64_t row_bytes, int32_t slots, int32_t batch);
int aqsgd_tier_prefetch(aqsgd_tier* tier, int32_t slot, const int64_t* host_ids, void* copy_stream);
int aqsgd_tier_acquire(aqsgd_tier* tier, int32_t slot, void* compute_stream,
                       const int64_t** sample_ids);
int aqsgd_tier_release(aqsgd_tier* tier, int32_t slot, void* compute_stream, void* copy_stream);
int aqsgd_tier_drain(aqsgd_tier* tier);
void aqsgd_tier_destroy(aqsgd_tier* tier);

/*
 * Debug helper: checks on the device that sample_ids are distinct and in range.
 * `flag` is one device int32 the caller has zeroed; the kernel sets bit 0 if an id
 * is out of range and bit 1 if two ids are equal.  O(batch^2) comparisons.
 */
int aqsgd_check_ids(const int64_t* sample_ids, int64_t batch, int64_t n_samples,
                    int32_t* flag, void* stream);

/*
 * Tuning helper (process-wide state): how launches are cut into workgroups.  It never
 * changes a result bit.  max_blocks bounds the workgroups of one job (kernels loop
 * when it is smaller than the work), dequant_unroll (1, 2 or 4) is the number of chunks a
 * lane takes per step in a launch that holds dequantising jobs only; 0 restores the value
 * from the environment (AQSGD_MAX_BLOCKS, AQSGD_DEQUANT_UNROLL) or the built-in default.
 * The two settings are atomics, read once per call: a change made while another host
 * thread is inside a codec call applies to that thread's next call.  AQSGD_ERR_SHAPE for
 * values out of range.  A third setting of the same kind has no setter and exists for
 * measurements only: AQSGD_LAUNCH_BLOCKS in the environment (read once per process) bounds
 * the workgroups of a whole launch, shared by its jobs in proportion to their sizes; unset,
 * the library bounds only launches of small groups (fewer than 512 elements), at 2048.
 */
int aqsgd_set_launch_shape(int64_t max_blocks, int32_t dequant_unroll);

/*
 * Measurement helper (per-thread state): the next codec launch made by the calling host thread
 * stamps `start_event` and `stop_event` (hipEvent_t created with timing enabled,
 * passed as void*; either may be NULL) with the kernel's own begin and end, so
 * hipEventElapsedTime(start, stop) is that launch's duration on the device.  The
 * request applies to one launch and is then cleared.  Such a launch cannot be
 * recorded into a HIP graph.
 */
int aqsgd_profile_next_launch(void* start_event, void* stop_event);

/* Human-readable text for a status code (static storage). */
const char* aqsgd_strerror(int status);

/* Library version, "major.minor.patch". */
const char* aqsgd_version(void);

#ifdef __cplusplus
}
#endif
#endif /* AQSGD_H */
