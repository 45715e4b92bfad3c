/*
 * sbc.h - C ABI of libsbc: Sparse Binary Compression (arXiv 1805.08768) on one
 * AMD MI355X (gfx950).
 *
 * The library implements the client lines of the paper's Alg. 1 between
 * "dW_i <- R_i + SGD_n(W_i) - W_i" and "msg_i <- encode(dW_i*)" for a list of
 * fp32 weight tensors (residual accumulation, Alg. 2 sparse binarization per
 * tensor, residual update, Alg. 3 Golomb position encoding), and the matching
 * server lines (Alg. 4 decoding followed by the scaled accumulation of
 * Alg. 1's averaging step).
 *
 * Conventions
 *   - Every function returns SBC_OK (0) or a negative sbc_status; nothing
 *     throws.  sbc_strerror() names a code.
 *   - "device" pointers are HIP device addresses valid on the context's GPU;
 *     "host" pointers are ordinary process memory.  The arrays of tensor
 *     pointers (dW[], residual[], out[]) and numel[] are HOST arrays whose
 *     ELEMENTS are device pointers / sizes.
 *   - The caller owns every buffer it passes.  The library reads or writes
 *     them only during the call (between sbc_compress_begin and
 *     sbc_compress_end, and until the stream has passed a deferred decode
 *     call, where those are used) and keeps no reference afterwards.  All
 *     scratch memory is owned by the sbc_ctx and allocated in sbc_create();
 *     sbc_compress() and sbc_decompress_accumulate() allocate nothing.
 *   - Work is enqueued on the caller's HIP stream (a hipStream_t passed as
 *     void*; NULL is the default stream).  sbc_compress and (unless its status
 *     is deferred) sbc_decompress_accumulate synchronise that stream once
 *     before returning, so results and the status are final.
 *   - A context must not be used from two threads at once.
 *   - Tensor sizes: 1 <= numel < 2^32.  Sparsity: 0 < p < 1.
 *
 * Message layout (little endian), produced by sbc_compress and consumed by
 * sbc_decompress_accumulate.  The paper transmits, per tensor, the Golomb bit
 * string of the gaps between kept positions and one mean value; tensor shapes
 * and b* are known to both sides ("Optimal Position Encoding"; supplement,
 * "Golomb Position Decoding").  The container around those is this library's:
 *     header   { u32 magic 'SBC1', u32 version = 1, u32 n_tensors, u32 bstar,
 *                u64 payload_words, u64 reserved = 0 }                 32 bytes
 *     table    n_tensors x { f32 mu_signed, u32 nnz, u64 bit_len,
 *                            u64 word_offset }                    24 bytes each
 *     payload  payload_words x u32; tensor t's stream occupies words
 *              [word_offset, word_offset + ceil(bit_len/32)); stream bit i is
 *              bit (31 - i%32) of word i/32; padding bits are zero.
 * mu_signed is +mu^+ when the positive side was kept and -mu^- otherwise
 * (Alg. 2).  Each kept position contributes q ones, one zero and b* remainder
 * bits, most significant first, with q, r = divmod(skipped entries since the
 * previous kept position, 2^b*) (Alg. 3).
 */
#ifndef SBC_H
#define SBC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sbc_status {
    SBC_OK = 0,
    SBC_EINVAL = -1,     /* null/misaligned pointer, p outside (0,1), numel out of range,
                            n_tensors <= 0, dW aliasing residual */
    SBC_ECAPACITY = -2,  /* message buffer below sbc_msg_bound(), or sizes beyond what the
                            context was created for */
    SBC_EHIP = -3,       /* a HIP runtime call failed */
    SBC_ECORRUPT = -4,   /* decode: bad magic/version, tensor count or b* mismatch, nnz or
                            bit_len inconsistent with the stream, position >= numel */
    SBC_ENONFINITE = -5, /* compress: an accumulated entry R + dW was NaN or +-Inf */
    SBC_EINTERNAL = -6   /* an internal invariant failed on the device (a bug) */
} sbc_status;

typedef struct sbc_ctx sbc_ctx;

/* Scratch memory for problems of up to max_total_elems entries in up to max_tensors
 * tensors per call, on HIP device `device`.  Device memory taken: about
 * 17 bytes per entry of max_total_elems plus 50 KiB per tensor, and 2.4 MiB whatever
 * the sizes.  The context also owns a few HIP events.  *out receives the
 * context.  SBC_EINVAL for non-positive sizes or a bad device, SBC_EHIP if an
 * allocation fails (nothing is leaked). */
int sbc_create(sbc_ctx** out, int device, int64_t max_total_elems, int max_tensors);

/* The same with candidate lists that hold a quarter of a tensor's entries per side instead of all
 * of them (Alg. 2's top_p% only ever needs the entries near the k-th; "Sparse Binarization"):
 * about 5 bytes per entry of max_total_elems instead of 17.  What it costs:
 *   - a list holds max(n/4, 4 k + 1024) entries (k as sbc_num_kept gives it for the call's p,
 *     never more than n); a call whose lists do not fit half an entry per entry of
 *     max_total_elems in all (plus 2048 per tensor) returns SBC_ECAPACITY before anything is
 *     enqueued (p above about 0.06 on a context sized for the model);
 *   - a tensor whose filter lets more candidates pass than its lists hold is redone through the
 *     histogram route, like one whose filter lets too few pass; if even that route's candidates
 *     (the entries of the histogram bins at and beyond the k-th entry's) do not fit, as happens
 *     when more than a quarter of the tensor's entries are about equal to the k-th (a constant
 *     tensor), sbc_compress returns
 *     SBC_ECAPACITY after the fact: no message was produced, and residual and msg contents are
 *     unspecified as after the other late errors (the tensors that completed have had their kept
 *     entries taken out of the residual).  Data like that needs a context from sbc_create.
 * Results are the same as on a context from sbc_create whenever the call succeeds. */
int sbc_create_compact(sbc_ctx** out, int device, int64_t max_total_elems, int max_tensors);

/* Frees the context's scratch memory.  NULL is allowed.  The caller must have
 * no work of this context in flight. */
void sbc_destroy(sbc_ctx* ctx);

/* b* of Alg. 3 / "Optimal Position Encoding":
 * max(0, 1 + floor(log2(log(phi-1)/log(1-p)))), phi the golden ratio, in fp64.
 * Returns SBC_EINVAL (negative) unless 0 < p < 1. */
int sbc_golomb_bstar(double p);

/* Entries kept per tensor and sign side ("fraction p", Alg. 2):
 * max(1, floor(p*numel)) with the product in fp64, at most numel.
 * Returns SBC_EINVAL (negative) on bad arguments. */
int64_t sbc_num_kept(int64_t numel, double p);

/* Worst-case size in bytes of the message for these tensor sizes: header, table and,
 * per tensor, ceil((k*(1+b*) + floor((numel-k)/2^b*)) / 32) words.  0 on bad arguments.
 * numel is a host array. */
size_t sbc_msg_bound(const int64_t* numel, int n_tensors, double p);

/* Same for a context with SBC_OPT_SAMPLED_THRESHOLD set, where a tensor sends up to
 * min(numel, 2k + 64) positions. */
size_t sbc_msg_bound_sampled(const int64_t* numel, int n_tensors, double p);

/* Client step (Alg. 1 client lines, Alg. 2, Alg. 3) for n_tensors tensors:
 *     A_t   = residual_t + dW_t                     (fp32, one rounding)
 *     dW*_t = SBC(A_t, p)                           (exactly k_t kept entries on one side;
 *                                                    equal values resolved to the lowest index;
 *                                                    see SBC_OPT_SAMPLED_THRESHOLD for the
 *                                                    variant with a noisy count)
 *     residual_t <- A_t - dW*_t                     (in place)
 *     msg   <- container of { mu_signed_t, Golomb(kept positions of t) }
 * dW[t]        device, read only, numel[t] floats, 4-byte aligned (16 is faster)
 * residual[t]  device, read/write, numel[t] floats, must not overlap dW[t]
 * numel        host array
 * msg          device, 8-byte aligned, msg_capacity >= sbc_msg_bound(...) bytes; bytes past
 *              *msg_bytes are not written
 * msg_bytes    host, receives the message size in bytes
 * Errors: SBC_EINVAL, SBC_ECAPACITY (nothing was enqueued; on a context from sbc_create_compact
 * see there), SBC_EHIP, SBC_ENONFINITE and SBC_EINTERNAL (residual and msg contents are then
 * unspecified).
 * Completion: the call returns as soon as the step's last kernel has reported the message size
 * (it writes status and size to pinned host memory, where the call looks for them), which may be
 * a few microseconds before hip_stream is idle.  msg and residual are complete for everything
 * enqueued on hip_stream afterwards; whoever reads them outside that order (another stream, a
 * blocking copy while hip_stream is a non-blocking stream) synchronises with hip_stream first. */
int sbc_compress(sbc_ctx* ctx, void* hip_stream,
                 const float* const* dW, float* const* residual,
                 const int64_t* numel, int n_tensors, double p,
                 void* msg, size_t msg_capacity, size_t* msg_bytes);

/* The same step in two calls, for callers that keep several independent client steps in flight
 * (one context, one stream and one set of buffers per client): sbc_compress_begin checks its
 * arguments (same meaning and errors as above) and enqueues the step on hip_stream without
 * waiting; sbc_compress_end waits until that step has reported its result (not for work the
 * caller has enqueued behind it on the stream; see "Completion" above for what may be read
 * when), completes the rare tensors that need a second pass, and returns the status
 * and the message size.  Between the two calls the context accepts
 * sbc_decompress_accumulate and nothing else (SBC_EINVAL), dW, residual and msg must not be
 * touched, and the host arrays passed to begin are no longer needed.  sbc_compress_end without
 * a pending step returns SBC_EINVAL.  sbc_compress is begin followed by end. */
int sbc_compress_begin(sbc_ctx* ctx, void* hip_stream,
                       const float* const* dW, float* const* residual,
                       const int64_t* numel, int n_tensors, double p,
                       void* msg, size_t msg_capacity);
int sbc_compress_end(sbc_ctx* ctx, size_t* msg_bytes);

/* Server step for one client message (Alg. 4, then the summand of Alg. 1's average):
 *     out_t[j] += scale * mu_signed_t   for every decoded position j of every tensor t
 * (fp32: the addend fl32(scale*mu) is formed once).  Call once per client with
 * scale = 1/|I_t| on zero-initialised accumulators to obtain the averaged update; calls on
 * one stream apply in call order.
 * msg          device, 8-byte aligned, msg_bytes valid bytes
 * numel        host array; n_tensors and p must match what the sender used
 * out[t]       device, read/write, numel[t] floats
 * Errors: SBC_EINVAL, SBC_ECAPACITY, SBC_EHIP; SBC_ECORRUPT if the message fails
 * validation: no write outside out_t[0..numel_t) ever happens, but accumulators may have
 * received part of the message.
 * Completion: as for sbc_compress, the call returns when the status is known; out is complete
 * for everything enqueued on hip_stream afterwards. */
int sbc_decompress_accumulate(sbc_ctx* ctx, void* hip_stream,
                              const void* msg, size_t msg_bytes,
                              const int64_t* numel, int n_tensors, double p,
                              float scale, float* const* out);

/* The server step for callers that cannot allocate: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same operation as sbc_decompress_accumulate on the
 * kernel that decodes one stream per workgroup, without a context: the tables that kernel reads
 * live in a device array that is part of the loaded library (about 9 KiB on every GPU the library
 * runs on, held until the process ends), and the call neither allocates, frees, copies to or from
 * the host nor waits: it enqueues three kernels on hip_stream and returns.
 *   device       HIP device the stream and all buffers belong to (SBC_EINVAL if there is no such device)
 *   msg, out, numel, n_tensors, p, scale   as for sbc_decompress_accumulate
 *   status       device, 4-byte aligned: receives SBC_OK, SBC_ECORRUPT or SBC_EINTERNAL once the
 *                stream has passed the call (validation is done on the device)
 * At most SBC_NOALLOC_MAX_TENSORS tensors per call (SBC_ECAPACITY beyond, nothing enqueued); other
 * argument errors as for sbc_decompress_accumulate.  All calls on one GPU share the one array,
 * which keeps the previous call's contents (every call rewrites what it reads): calls on one GPU
 * must not overlap, i.e. use one stream, or order the streams. */
#define SBC_NOALLOC_MAX_TENSORS 192
int sbc_decompress_accumulate_noalloc(int device, void* hip_stream,
                                      const void* msg, size_t msg_bytes,
                                      const int64_t* numel, int n_tensors, double p,
                                      float scale, float* const* out, int32_t* status);

/* Options of a context.  Except for SBC_OPT_SAMPLED_THRESHOLD none of them changes a result:
 * sbc_compress is exact on every route.  It finds each tensor's top-k candidates with a filter key per sign side and, for a tensor
 * whose filter turns out to have kept fewer than k entries, falls back to an exact histogram
 * of a second read of that tensor.
 *   SBC_OPT_FORCE_EXACT_PATH   (0/1, default 0)  1 makes every tensor take the histogram route
 *       (to exercise and to time it).
 *   SBC_OPT_CARRY_FILTER_KEYS  (0/1, default 1)  1 lets a call start from filter keys that the
 *       previous successful call on this context left behind, when tensor sizes and p are
 *       unchanged (successive rounds of one training run), and skips the sampling kernel: per
 *       tensor and side the key of that call's entry of rank 9/8 k to 2 k (more while its
 *       update moves many entries across the key).  Only a filter: a tensor for which it keeps
 *       fewer than k entries (the data shrank, the residual was cleared) is redone exactly
 *       through the histogram route, and the next call samples; so do the calls after one that
 *       saw many times k candidates (the data grew), until a call's sample says that the keys
 *       of the call before it would have held.  0 estimates the keys from a sample of the new
 *       data in every call.
 *   SBC_OPT_WIDE_MIN_KEPT      (default 0 = 8192)  a tensor that keeps at least this many entries
 *       per side is selected by grid-wide kernels instead of one workgroup, and its stream is
 *       decoded tile by tile by many workgroups instead of one (a 1.5e9-entry tensor at
 *       p = 0.001 keeps 1.5e6); tests lower it to send small tensors that way, or raise it (one
 *       workgroup selects and encodes up to 16384 kept entries by itself).
 *   SBC_OPT_SAMPLED_THRESHOLD  (0/1, default 0)  1 selects the subsampled variant of
 *       "Sparse Binarization" (the threshold is estimated from a random subsample, which makes
 *       the amount of sparsity noisy).  Per tensor t of the call a stratified sample of at most
 *       16384 entries of A_t is drawn: the whole tensor if it is no larger, else 256 aligned runs
 *       of 64 consecutive entries, run r at slot floor(r*S/256) + floor(h*w/2^32) of the S =
 *       floor(numel/64) slots, w the width of stratum r and h = mix32(r*0x9E3779B9 +
 *       t*0x85EBCA6B + 1 mod 2^32), mix32(x): x ^= x>>16; x *= 0x7FEB352D; x ^= x>>15;
 *       x *= 0x846CA68B; x ^= x>>16.  With m sampled entries and r = max(1, floor(p*m)) a
 *       side's threshold is its r-th most extreme sampled value; the side keeps every entry at or
 *       beyond it, at most min(numel, 2k + 64) of them (the most extreme, equal values to the
 *       lowest index); mu+ and mu- are means over each side's own count.  The message buffer
 *       must hold sbc_msg_bound_sampled() bytes; set the option on a decoding context as well,
 *       so that it reserves for the longer streams.  The options FORCE_EXACT_PATH and
 *       CARRY_FILTER_KEYS are ignored while it is set.
 *   SBC_OPT_FUSED_STEP         (0/1, default 0)  1 lets the streaming kernel finish, by itself, every
 *       tensor that keeps few enough entries for one workgroup (Alg. 2 and Alg. 3 run in the last
 *       workgroup of the tensor to finish streaming, beside the streaming of the other tensors)
 *       instead of leaving all of them to the selection kernel that follows.  Same results.
 *   SBC_OPT_DEFER_DECODE_STATUS (0/1, default 0)  1 makes sbc_decompress_accumulate return as
 *       soon as its kernels are enqueued (SBC_OK unless an argument is bad), so that a server can
 *       decode the messages of all clients back to back without waiting for each; validation
 *       failures of those calls are collected on the device and reported by sbc_decode_status().
 *       Every message buffer must stay unchanged until the stream has passed its call.  The
 *       option cannot be changed while a status is outstanding (SBC_EINVAL). */
enum { SBC_OPT_FORCE_EXACT_PATH = 1, SBC_OPT_CARRY_FILTER_KEYS = 2, SBC_OPT_WIDE_MIN_KEPT = 3,
       SBC_OPT_SAMPLED_THRESHOLD = 4, SBC_OPT_DEFER_DECODE_STATUS = 5, SBC_OPT_FUSED_STEP = 6 };
int sbc_set_option(sbc_ctx* ctx, int option, int value);

/* With SBC_OPT_DEFER_DECODE_STATUS: waits for hip_stream (the stream the deferred
 * sbc_decompress_accumulate calls were enqueued on) and returns SBC_OK if every such call since
 * the previous sbc_decode_status passed validation, else the error (SBC_ECORRUPT, SBC_EHIP); the
 * collected status starts afresh.  SBC_OK at once if nothing is outstanding. */
int sbc_decode_status(sbc_ctx* ctx, void* hip_stream);

/* Which routes the most recent successful sbc_compress() took: a bit set of
 * SBC_ROUTE_CARRIED_KEYS (filter keys came from the previous call, no sampling) and
 * SBC_ROUTE_HISTOGRAM (the histogram route ran for at least one tensor), SBC_ROUTE_WIDE (the
 * grid-wide selection kernels completed at least one tensor); SBC_EINVAL (negative) without a
 * successful call. */
enum { SBC_ROUTE_CARRIED_KEYS = 1, SBC_ROUTE_HISTOGRAM = 2, SBC_ROUTE_WIDE = 4,
       SBC_ROUTE_LOOSE_KEYS = 8,    /* some filter key let so many entries pass that the next call samples afresh */
       SBC_ROUTE_TAKEN_OVER = 16 }; /* a tensor the streaming kernel could not finish was completed by the
                                       one-workgroup selection kernel in a second pass */
int sbc_last_route(sbc_ctx* ctx);

/* Inspection of the most recent sbc_compress() on this context, for tests and reports
 * (Alg. 2 intermediates).  All out pointers are host memory and may be NULL.
 *   mu_pos, mu_neg : mean(val+), mean(val-) in fp64
 *   side           : +1 or -1
 *   nnz            : kept entries (= k)
 *   bit_len        : length of the tensor's Golomb stream in bits */
int sbc_last_tensor_stats(sbc_ctx* ctx, int tensor, double* mu_pos, double* mu_neg,
                          int* side, int64_t* nnz, int64_t* bit_len);

/* Candidates per sign side that the filter of the most recent sbc_compress() let pass for a
 * tensor that the streaming kernel finished itself (0 for the others: one-chunk tensors, which
 * need no filter, and tensors selected by the other kernels).  Out pointers are host memory and
 * may be NULL.  The ratio to the kept count is what a filter key costs ("Sparse Binarization":
 * the selection works on these instead of the whole tensor). */
int sbc_last_candidates(sbc_ctx* ctx, int tensor, int64_t* positive, int64_t* negative);

/* Copies the kept-position bitmap of tensor `tensor` from the most recent sbc_compress()
 * into host memory: entry j is bit (j%32) of mask_words[j/32]; n_words must be
 * ceil(numel/32). */
int sbc_last_mask(sbc_ctx* ctx, int tensor, uint32_t* mask_words, size_t n_words);

/* Measurement support: per-kernel durations of sbc_compress().  A profiled launch carries a
 * start and a stop event on the caller's stream that take the begin and end time stamps of that
 * dispatch, so the figure is the kernel's own duration.
 *   level 0  off (default; no events are recorded)
 *   level 1  only the residual-accumulation kernel (the pass that carries the method's
 *            mandatory 12 bytes per entry) and the kernel launched before it are timed (with
 *            events on its predecessor too, its own start stamp is not taken while that one
 *            still drains)
 *   level 2  every kernel is timed
 * sbc_profile_enable sets the level and clears the accumulated totals; sbc_profile_level only
 * sets the level (a caller may time every n-th call and keep adding up). */
int sbc_profile_enable(sbc_ctx* ctx, int level);
int sbc_profile_level(sbc_ctx* ctx, int level);

/* Accumulated time of stage `stage` (0 .. n-1 in launch order; SBC_EINVAL past the end):
 * *name gets a static string (the kernel's name), *total_ms the summed duration over
 * *calls bracketed launches.  Out pointers are host memory and may be NULL. */
int sbc_profile_read(sbc_ctx* ctx, int stage, const char** name, double* total_ms, int64_t* calls);

/* Measurement support: enqueues a plain device-to-device streaming copy kernel of `bytes`
 * bytes (a multiple of 16; both pointers 16-byte aligned) on the stream and returns without
 * synchronising.  It is the yardstick for achievable HBM bandwidth and for scaling hardware
 * counters; it is not part of the method. */
int sbc_copy_baseline(void* hip_stream, void* dst, const void* src, size_t bytes);

/* Static string for a status code. */
const char* sbc_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* SBC_H */
