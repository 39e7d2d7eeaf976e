/* libmqgrad -- the data-parallel hot path of MQGrad (arXiv 1804.08066) for AMD MI355X (gfx950).
 *
 * The paper trains on a parameter server.  Every iteration each worker quantizes its gradient to
 * K bits and pushes it; the server de-quantizes all workers' gradients, averages them and updates
 * the parameters (Section 3.2; Algorithm 1, WorkerIterate and ReceiveQGThenSendQG).  K is chosen
 * by a small MDP agent on the server from the recent loss values (Section 3.3; Algorithm 2).
 *
 * This library is that path for one GPU:
 *   mqg_quantize          worker side: per-bucket range, stochastic rounding to the 2^K-level
 *                         grid, dense bit packing            (the paper's Quantize(g, K))
 *   mqg_aggregate_update  server side: unpack, de-quantize, mean over W workers, SGD update
 *                         (the paper's De-quantize + average + w <- w - eta g)
 *   mqg_mdp_*             the host-side agent that picks K  (the paper's MQGrad-SARSA)
 * and, further down: the server's re-quantizing step of the printed Algorithm 1 with the worker's
 * de-quantizing update, several layer tensors per launch, the footnote's deterministic [min, max]
 * encoder (per bucket or per tensor), and the Adaptive baseline's bit rule.
 *
 * Conventions
 *   - Plain C ABI.  No function throws, aborts or allocates device memory.
 *   - "device pointer" = memory the current HIP device can read/write.  The library neither
 *     retains nor frees any pointer it is given.
 *   - GPU calls are asynchronous: they enqueue work on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and return.  A returned MQG_OK means "enqueued".
 *   - Every error is reported through the return code; nothing is enqueued when it is not MQG_OK.
 *
 * The quantizer (the paper gives only "range-linear encode/decode to K bits"; the rest is this
 * library's reading of it):
 *   bucket k covers elements [k*bucket, min((k+1)*bucket, n));  s_k = max |g_i| over the bucket
 *   (stored as 0 when below 2^-96);  L = 2^bits - 1;  the 2^bits levels are s_k*(2c - L)/L for
 *   code c = 0..L (top bit of c = sign, low bits = magnitude level).  Element i is placed at
 *   u = clamp(fma(g_i, (L/2)/s_k, L/2), 0, L) and rounded down or up at random so that the
 *   expectation is u: c = floor(u) + [r < u - floor(u)], r = (h + 1/2) / 65536, where h is the
 *   16-bit uniform that Philox4x32-10 (Salmon et al., SC'11) yields for key = seed and counter =
 *   (group lo, group hi, iteration, worker), group = (elem_base + i) >> 3, 16-bit slot
 *   (elem_base + i) & 7 of the 128-bit output.  Code i occupies bits [i*bits, (i+1)*bits) of a
 *   little-endian stream of 32-bit words; unused bits of the last word are 0.
 */
#ifndef MQGRAD_H
#define MQGRAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MQG_OK = 0,
    MQG_EINVAL = -1,  /* an argument is out of its documented range, or a required pointer is NULL */
    MQG_EALIGN = -2,  /* a pointer is not aligned as its argument requires (4 bytes unless stated) */
    MQG_ELAUNCH = -3  /* the HIP runtime refused the launch (hipGetLastError was consumed) */
} mqg_status;

typedef enum {
    MQG_SCALE_MAXABS = 0, /* s_k = max |g_i|  (order independent, bit exact) */
    MQG_SCALE_L2 = 1      /* s_k = ||bucket||_2 (>= max |g_i|), same grid */
} mqg_scale_mode;

#define MQG_MAX_WORKERS 64u
#define MQG_MIN_BUCKET 32u
#define MQG_MAX_BUCKET 16384u

/* Human-readable name of a status code (static storage, never NULL). */
const char* mqg_status_string(mqg_status st);

/* Number of buckets, ceil(n / bucket), and of 32-bit words in the packed stream,
 * ceil(n * bits / 32).  Pure host arithmetic; bucket and bits must be non-zero. */
size_t mqg_num_buckets(uint64_t n, uint32_t bucket);
size_t mqg_packed_words(uint64_t n, uint32_t bits);

/* Worker side: Quantize(g, K) of Algorithm 1 (WorkerIterate), Section 3.2 footnote.
 *
 *   grad        device, n floats, read only.  Values must be finite (non-finite values never
 *               fault but give unspecified codes for their bucket).
 *   n           element count; 0 is a no-op.
 *   bits        K, 1..8.
 *   bucket      elements per scale; a multiple of 32 in [32, 16384].  bucket >= n gives the
 *               paper's one-range-per-tensor quantizer.
 *   seed, iteration, worker, elem_base
 *               select the random stream (see top of file).  elem_base must be a multiple of 8;
 *               it offsets the element index so that several tensors of one model draw from
 *               disjoint parts of one stream.
 *   packed_out  device, mqg_packed_words(n, bits) words, fully overwritten.
 *   scales_out  device, mqg_num_buckets(n, bucket) floats, fully overwritten.
 *   stream      hipStream_t.
 * Pointers need 4-byte alignment only (128-bit accesses are used at any dword address).
 * Errors: MQG_EINVAL (bits, bucket, elem_base out of range; NULL pointer with n > 0),
 *         MQG_EALIGN, MQG_ELAUNCH. */
mqg_status mqg_quantize(const float* grad, uint64_t n, uint32_t bits, uint32_t bucket,
                        uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                        uint32_t* packed_out, float* scales_out, void* stream);

/* mqg_quantize with a statement about what happens to the code words next.  Results are identical; only
 * the cache policy of the stores differs.  MQG_CODES_KEEP_CACHED (what mqg_quantize does): stores with
 * agent scope -- written through to memory at once, the lines stay in the last-level cache, where a
 * server step that follows on this GPU finds them (8 workers, 100 M elements, 4 bits: the update takes
 * 181 us instead of 196, and the quantizer itself is 1-3 us faster).  MQG_CODES_TO_MEMORY: streaming
 * stores, for streams that leave this GPU or that, together with the other workers' streams, exceed its
 * caches before they are read (16 workers, 3 bits: the update takes 243 us instead of 276).
 * MQG_EINVAL for any other value of `dest`; other arguments and errors as for mqg_quantize. */
typedef enum {
    MQG_CODES_KEEP_CACHED = 0,
    MQG_CODES_TO_MEMORY = 1
} mqg_codes_destination;
mqg_status mqg_quantize_to(const float* grad, uint64_t n, uint32_t bits, uint32_t bucket,
                           uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                           uint32_t* packed_out, float* scales_out, mqg_codes_destination dest, void* stream);

/* Same, with the bucket range taken as the L2 norm of the bucket when mode == MQG_SCALE_L2
 * (the norm scaling of the QSGD family the paper cites in Section 2).  mode == MQG_SCALE_MAXABS
 * is exactly mqg_quantize.  The sum of squares is accumulated in a fixed order (groups of four squares
 * in fp32, everything above in fp64), so the scale is reproducible, but only close (about 1e-7
 * relative) to a scale summed in another order; it is raised to max |g_i| if rounding left it below. */
mqg_status mqg_quantize_mode(const float* grad, uint64_t n, uint32_t bits, uint32_t bucket,
                             mqg_scale_mode mode,
                             uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                             uint32_t* packed_out, float* scales_out, void* stream);

/* Same as mqg_quantize, but the bucket scales are READ from scales_in (device,
 * mqg_num_buckets(n, bucket) floats) instead of being computed; they are copied to scales_out
 * (scales_out may equal scales_in).  Elements larger than their scale clamp to the end levels.
 * Lets a caller fix the range across workers, or inject scales computed elsewhere. */
mqg_status mqg_quantize_with_scales(const float* grad, uint64_t n, uint32_t bits, uint32_t bucket,
                                    uint64_t seed, uint32_t iteration, uint32_t worker,
                                    uint64_t elem_base, const float* scales_in,
                                    uint32_t* packed_out, float* scales_out, void* stream);

/* Server side: De-quantize each worker's gradient, average over the W workers, update the
 * parameters (Algorithm 1, ReceiveQGThenSendQG: mean over P workers; WorkerIterate: w <- w - eta g).
 *
 *   params[i] <- fma(-(lr / W), sum_{w=0}^{W-1} (2 c_{w,i} - L) * (s_{w,k} / L), params[i])
 *
 * with the sum taken in worker order, one fused multiply-add per worker, all in fp32.
 *
 *   packed, scales  HOST arrays of W device pointers (read during the call only): worker w's
 *                   packed stream and bucket scales as written by mqg_quantize with the same
 *                   n, bits and bucket (the paper broadcasts one K to all workers).
 *   W               1..MQG_MAX_WORKERS.
 *   lr              learning rate eta.
 *   params          device, n floats, updated in place.
 * Errors as for mqg_quantize; additionally MQG_EINVAL for W out of range or a NULL entry. */
mqg_status mqg_aggregate_update(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                                uint64_t n, uint32_t bits, uint32_t bucket,
                                float lr, float* params, void* stream);

/* The same step with a statement about where the code words are.  Results are identical; only the cache
 * policy of the code loads differs.  MQG_CODES_MAY_BE_CACHED (what mqg_aggregate_update assumes) suits
 * streams that this GPU wrote itself just before, as in a one-GPU step: up to 3 bits they are read with
 * ordinary loads.  MQG_CODES_FROM_MEMORY suits a parameter server whose W streams arrive over the
 * network (Section 3.2: workers push, the server aggregates): every width is read with streaming loads,
 * which is 5-9 % faster at 2 and 3 bits when no code word is in the caches and 3-8 % slower when they are.
 * MQG_EINVAL for any other value of `origin`. */
typedef enum {
    MQG_CODES_MAY_BE_CACHED = 0,
    MQG_CODES_FROM_MEMORY = 1
} mqg_codes_origin;
mqg_status mqg_aggregate_update_from(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                                     uint64_t n, uint32_t bits, uint32_t bucket,
                                     float lr, float* params, mqg_codes_origin origin, void* stream);

/* The server's mean gradient itself, for callers whose optimizer is not the plain SGD step of the
 * paper: mean_out[i] <- (sum over workers, in worker order, of the de-quantized values -- the chain of
 * mqg_aggregate_update) / W, one IEEE fp32 division per element.  With W = 1 this is De-quantize.
 *   mean_out  device, n floats, fully overwritten.  Other arguments and errors as for
 *   mqg_aggregate_update. */
mqg_status mqg_aggregate_mean(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                              uint64_t n, uint32_t bits, uint32_t bucket,
                              float* mean_out, void* stream);

/* ---- the paper's full exchange (Algorithm 1): the server sends the quantized mean back ---------
 *
 * ReceiveQGThenSendQG:  g^m <- sum_p De-quantize(gbar_p) / P;  gbar^m <- Quantize(g^m, K);  send.
 * WorkerIterate:        g^m <- De-quantize(gbar^m);  w <- w - eta g^m.
 *
 * mqg_aggregate_requantize is the server's half, fused: the W streams are unpacked, de-quantized and
 * summed in worker order (the same fp32 fma chain as mqg_aggregate_update), and the sum is quantized
 * with the same `bits` and `bucket` exactly as mqg_quantize would quantize it (max-abs range S per
 * bucket, stochastic rounding with the stream selected by seed / iteration / worker / elem_base --
 * give the server a `worker` id of its own, e.g. W).  The division by W is applied to the stored
 * range: scales_out holds S / W, so that De-quantize(packed_out, scales_out) is the mean.  No fp32
 * copy of the sum or the mean is ever written to memory.
 *   packed, scales  HOST arrays of W device pointers, as for mqg_aggregate_update.
 *   packed_out      device, mqg_packed_words(n, bits) words;  scales_out: mqg_num_buckets(n, bucket) floats.
 * Errors as for mqg_quantize and mqg_aggregate_update. */
mqg_status mqg_aggregate_requantize(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                                    uint64_t n, uint32_t bits, uint32_t bucket,
                                    uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                                    uint32_t* packed_out, float* scales_out, void* stream);
/* The same with the bucket range of mqg_quantize_mode: MQG_SCALE_L2 takes S = the L2 norm of the sum's
 * bucket (raised to max |sum| if rounding left it below), and stores S / W. */
mqg_status mqg_aggregate_requantize_mode(const uint32_t* const* packed, const float* const* scales, uint32_t W,
                                         uint64_t n, uint32_t bits, uint32_t bucket, mqg_scale_mode mode,
                                         uint64_t seed, uint32_t iteration, uint32_t worker, uint64_t elem_base,
                                         uint32_t* packed_out, float* scales_out, void* stream);

/* The worker's half: params[i] <- fma(-lr, (2 c_i - L) * (s_k / L), params[i]), i.e. w <- w - eta *
 * De-quantize(gbar).  Same as mqg_aggregate_update with one worker. */
mqg_status mqg_dequantize_update(const uint32_t* packed, const float* scales, uint64_t n, uint32_t bits,
                                 uint32_t bucket, float lr, float* params, void* stream);

/* ---- several layer tensors per launch, and layers that are sent uncompressed -----------------
 *
 * A model is a list of layer tensors; the paper quantizes only its two large fully connected layers
 * and communicates the other parameters without compression (Section 4.1).  Small layers are bound
 * by launch overhead when handled one call at a time, so these entry points take up to
 * MQG_MAX_TENSORS layers in ONE launch.  Results are bit-identical to the per-tensor calls. */

#define MQG_MAX_TENSORS 32u
#define MQG_MAX_TENSOR_POINTERS 256u  /* sum over layers of (quantized ? 2 * W : W) */

typedef struct {
    const float* grad;     /* device, n floats */
    uint64_t n;            /* 0 is allowed (the layer is skipped) */
    uint64_t elem_base;    /* multiple of 8: the layer's offset in the model's random stream */
    uint32_t* packed_out;  /* device, mqg_packed_words(n, bits) words */
    float* scales_out;     /* device, mqg_num_buckets(n, bucket) floats */
    const float* scales_in; /* NULL: the layer's scales are computed; else device, mqg_num_buckets(n, bucket)
                               floats that are read instead (and copied to scales_out), as in
                               mqg_quantize_with_scales */
} mqg_quantize_item;

/* mqg_quantize for `count` layers of one worker.  `items` is a HOST array, read during the call.
 * mqg_quantize_tensors_mode: the same with the bucket range of mqg_quantize_mode (MQG_SCALE_L2: the
 * bucket's L2 norm) for the layers whose scales are computed.  Results are bit-identical to the
 * per-layer calls mqg_quantize / mqg_quantize_mode / mqg_quantize_with_scales. */
mqg_status mqg_quantize_tensors(const mqg_quantize_item* items, uint32_t count, uint32_t bits, uint32_t bucket,
                                uint64_t seed, uint32_t iteration, uint32_t worker, void* stream);
mqg_status mqg_quantize_tensors_mode(const mqg_quantize_item* items, uint32_t count, uint32_t bits, uint32_t bucket,
                                     mqg_scale_mode mode, uint64_t seed, uint32_t iteration, uint32_t worker,
                                     void* stream);

typedef struct {
    uint64_t n;
    float* params;                   /* device, n floats, updated in place */
    const uint32_t* const* packed;   /* HOST array of W device pointers; NULL for an uncompressed layer */
    const float* const* scales;      /* HOST array of W device pointers; NULL for an uncompressed layer */
    const float* const* raw;         /* uncompressed layer: HOST array of W device pointers to fp32 gradients */
} mqg_update_item;

/* mqg_aggregate_update for `count` layers.  A layer with packed == NULL is uncompressed:
 *   params[i] <- fma(-(lr / W), sum_{w} raw[w][i], params[i])   (fp32 sum in worker order).
 * Errors: MQG_EINVAL also for count > MQG_MAX_TENSORS or more than MQG_MAX_TENSOR_POINTERS pointers. */
mqg_status mqg_aggregate_update_tensors(const mqg_update_item* items, uint32_t count, uint32_t W,
                                        uint32_t bits, uint32_t bucket, float lr, void* stream);

/* ---- the Section 3.2 footnote read literally: deterministic range-linear encode over [min, max] ----
 *
 * The footnote defines Quantize / De-quantize as a range-linear Encode / Decode: the tensor's range
 * [min, max] is cut into 2^K - 1 equal steps, a value is stored as the index of the nearest level and
 * restored as min + index * step.  No random numbers are drawn.  The range is taken per bucket of
 * `bucket` consecutive elements (bucket >= n: one range per tensor, as in the paper).
 *
 *   mn, mx   min and max of the bucket (a zero bound is stored as +0)
 *   a        fl(L / fl(mx - mn)), L = 2^bits - 1;  0 when the range is below 2^-96 (one level)
 *   c        clamp(rint(fl(fl(g - mn) * a)), 0, L), ties to the even index
 *   value    fma((float)c, fl(fl(mx - mn) / L), mn)
 *
 *   ranges_out   device, 2 * mqg_num_buckets(n, bucket) floats, 8-byte aligned: (mn, mx) of bucket k
 *                at [2k], [2k+1].  packed_out as for mqg_quantize (same dense little-endian stream).
 * Errors as for mqg_quantize (MQG_EALIGN also when ranges_out is not 8-byte aligned). */
mqg_status mqg_quantize_minmax(const float* grad, uint64_t n, uint32_t bits, uint32_t bucket,
                               uint32_t* packed_out, float* ranges_out, void* stream);

/* Server step for that encoding (Algorithm 1, ReceiveQGThenSendQG + the update of WorkerIterate):
 * acc = sum over workers, in worker order, of value_w;  params[i] <- fma(-fl(lr / W), acc, params[i]).
 *   packed, ranges  HOST arrays of W device pointers (streams and (mn, mx) pairs of the workers, the
 *                   range arrays 8-byte aligned); the arrays may be freed on return.
 * Errors as for mqg_aggregate_update. */
mqg_status mqg_aggregate_update_minmax(const uint32_t* const* packed, const float* const* ranges, uint32_t W,
                                       uint64_t n, uint32_t bits, uint32_t bucket,
                                       float lr, float* params, void* stream);

/* The paper's full exchange with that encoding.  Server (ReceiveQGThenSendQG): the W streams are
 * de-quantized and added in worker order (the chain of mqg_aggregate_update_minmax), the sum is encoded
 * over its own per-bucket [mn, mx] exactly as mqg_quantize_minmax would encode it, and the stored range
 * is (mn / W, mx / W): a range-linear grid is equivariant under positive scaling, so what the worker
 * de-quantizes is the mean.  No fp32 copy of the sum or the mean is written to memory.
 *   packed, ranges          HOST arrays of W device pointers, as for mqg_aggregate_update_minmax.
 *   packed_out, ranges_out  device, as for mqg_quantize_minmax.
 * The worker's half, w <- w - eta De-quantize(gbar), is mqg_aggregate_update_minmax with W = 1. */
mqg_status mqg_aggregate_requantize_minmax(const uint32_t* const* packed, const float* const* ranges, uint32_t W,
                                           uint64_t n, uint32_t bits, uint32_t bucket,
                                           uint32_t* packed_out, float* ranges_out, void* stream);

/* One range for the whole tensor, as the paper encodes (any n; the bucketed calls above stop at buckets
 * of MQG_MAX_BUCKET elements).
 *
 * mqg_tensor_range: range_out[0] = min, range_out[1] = max of grad[0..n) (a zero bound as +0).
 *   range_out  device, 2 floats, 8-byte aligned.  n = 0 leaves it untouched.
 * mqg_quantize_minmax_tensor: mqg_tensor_range followed by the encode of mqg_quantize_minmax with that
 *   one (mn, mx) for every element -- two passes over the gradient, on the same stream.
 * mqg_aggregate_update_minmax_tensor: the server step with one (mn, mx) pair per worker.
 *   ranges  HOST array of W device pointers, each to 2 floats (8-byte aligned).
 * Arithmetic, packed layout and errors as for the bucketed calls.
 * mqg_aggregate_requantize_minmax_tensor: the server's re-encoding step of Algorithm 1 as printed
 *   (ReceiveQGThenSendQG with the footnote's encoder): the W streams are de-quantized and added in worker
 *   order, the sum is encoded over its own whole-tensor [mn, mx], and range_out receives (mn / W, mx / W),
 *   so that what a worker de-quantizes (mqg_aggregate_update_minmax_tensor with W = 1) is the mean.  The
 *   range of the sum is known only after every element has been decoded, so the W streams are read twice
 *   ((2 W + 1) * bits / 8 bytes per element; no fp32 copy of the sum is written).  Five launches on the stream.
 *   ranges      HOST array of W device pointers, each to 2 floats (8-byte aligned).
 *   packed_out  device, mqg_packed_words(n, bits) words;  range_out: device, 2 floats, 8-byte aligned.
 */
mqg_status mqg_tensor_range(const float* grad, uint64_t n, float* range_out, void* stream);
mqg_status mqg_quantize_minmax_tensor(const float* grad, uint64_t n, uint32_t bits,
                                      uint32_t* packed_out, float* range_out, void* stream);
mqg_status mqg_aggregate_update_minmax_tensor(const uint32_t* const* packed, const float* const* ranges,
                                              uint32_t W, uint64_t n, uint32_t bits,
                                              float lr, float* params, void* stream);
mqg_status mqg_aggregate_requantize_minmax_tensor(const uint32_t* const* packed, const float* const* ranges,
                                                  uint32_t W, uint64_t n, uint32_t bits,
                                                  uint32_t* packed_out, float* range_out, void* stream);

/* Several layer tensors per launch with this encoding (Section 4.1: the two large fully connected layers
 * are encoded, each over its own range, and the other layers travel as fp32) -- the [min, max] forms of
 * mqg_quantize_tensors and mqg_aggregate_update_tensors, with the same limits (MQG_MAX_TENSORS,
 * MQG_MAX_TENSOR_POINTERS).  Results are bit-identical to the per-layer calls.
 *
 * mqg_quantize_minmax_tensors: `items` is a HOST array, read during the call.
 *   bucket > 0   mqg_quantize_minmax for every layer in ONE launch; items[i].scales_out receives the
 *                layer's 2 * mqg_num_buckets(n, bucket) floats.
 *   bucket == 0  one range per layer, as the paper encodes: mqg_quantize_minmax_tensor for every layer --
 *                a batched range reduction, then a batched encode (four launches for any number of
 *                layers); items[i].scales_out receives the layer's 2 floats.
 *   items[i].scales_out must be 8-byte aligned; items[i].scales_in must be NULL (MQG_EINVAL otherwise);
 *   items[i].elem_base is not read (no random numbers are drawn).
 * mqg_aggregate_update_minmax_tensors: mqg_aggregate_update_minmax (bucket > 0) or
 *   mqg_aggregate_update_minmax_tensor (bucket == 0) for `count` layers in one launch; items[i].scales[w]
 *   is worker w's range array of layer i (8-byte aligned); a layer with packed == NULL is uncompressed
 *   and updated as in mqg_aggregate_update_tensors. */
mqg_status mqg_quantize_minmax_tensors(const mqg_quantize_item* items, uint32_t count, uint32_t bits, uint32_t bucket,
                                       void* stream);
mqg_status mqg_aggregate_update_minmax_tensors(const mqg_update_item* items, uint32_t count, uint32_t W,
                                               uint32_t bits, uint32_t bucket, float lr, void* stream);

/* ---- the "Adaptive" baseline's bit rule (Section 4.1; idea in Section 2: the larger the gradient's
 * norm, the more bits) ------------------------------------------------------------------------------
 *
 * mqg_sum_squares: *sumsq_out <- sum_i grad[i]^2, accumulated in fp64 (squares of fp32 values are
 * exact in fp64; the order of the partial sums is not fixed, so the result is reproducible to about
 * 1e-15 relative, not to the bit).  sumsq_out: device, one double, 8-byte aligned, overwritten.
 * n = 0 stores 0. */
mqg_status mqg_sum_squares(const float* grad, uint64_t n, double* sumsq_out, void* stream);

/* The same sum for up to MQG_MAX_SUMSQ_TENSORS tensors in one call -- the W workers' gradients of an
 * iteration, or a model's layers (the Adaptive rule takes the norm of every worker's gradient, Section
 * 4.1) -- and reproducible to the bit: every workgroup stores one partial sum and a finishing kernel adds
 * the partial sums of a tensor in a fixed order, so sumsq_out[k] depends on (items[k].n, the values) only.
 *   items       HOST array of `count` tensors (read during the call only); n = 0 gives 0.
 *   workspace   device, mqg_sum_squares_workspace_bytes(count) bytes of scratch memory, 8-byte aligned;
 *               contents on entry are of no interest, contents on return are unspecified.  Calls that
 *               share a workspace must not overlap.
 *   sumsq_out   device, `count` doubles, 8-byte aligned, overwritten.
 * Errors: MQG_EINVAL (count > MQG_MAX_SUMSQ_TENSORS, NULL pointer), MQG_EALIGN, MQG_ELAUNCH. */
#define MQG_MAX_SUMSQ_TENSORS 64u
typedef struct {
    const float* grad;   /* device, n floats */
    uint64_t n;
} mqg_sumsq_item;
size_t mqg_sum_squares_workspace_bytes(uint32_t count);
mqg_status mqg_sum_squares_batch(const mqg_sumsq_item* items, uint32_t count, void* workspace, double* sumsq_out,
                                 void* stream);

/* mqg_sum_squares_batch for callers that cannot allocate device memory -- code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc: no workspace argument; the partial sums live in
 * a device array that the library itself holds (256 KB on every GPU it runs on, until the process ends).
 * The call allocates and frees nothing.  Results are bit-identical to mqg_sum_squares_batch.
 *   count   at most MQG_MAX_SUMSQ_TENSORS (the array's size); more is MQG_EINVAL.
 * Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (different streams,
 * different threads) race and must be serialised by the caller.  Nothing has to be cleared between
 * calls (every partial sum is written before it is read).  Other arguments and errors as above. */
mqg_status mqg_sum_squares_batch_static(const mqg_sumsq_item* items, uint32_t count, double* sumsq_out, void* stream);

typedef struct {
    uint32_t base_bits;     /* 2: this build's reading (the published Section 4.1 names the baseline, not its rule) */
    double norm_per_bit;    /* 0.0005: this build's reading, as above */
    uint32_t bits_min;      /* paper's range of widths: 2 */
    uint32_t bits_max;      /* paper's range of widths: 8 */
} mqg_adaptive_config;

void mqg_adaptive_default_config(mqg_adaptive_config* cfg);

/* Host only.  K = base_bits + floor(Z / norm_per_bit), kept inside [bits_min, bits_max], where Z is
 * the mean over the W workers of their gradients' L2 norms (worker_norms[w] = sqrt of the sum of
 * squares of worker w's gradient).  An infinite Z gives bits_max.  MQG_EINVAL for NULL arguments,
 * W = 0, a negative or NaN norm, norm_per_bit <= 0 or bits_min > bits_max or bits outside 1..8. */
mqg_status mqg_adaptive_bits(const double* worker_norms, uint32_t W, const mqg_adaptive_config* cfg,
                             uint32_t* bits_out);

/* ---- host-side agent that chooses K (Section 3.3, Algorithm 2).  No GPU involved. ---------- */

typedef struct mqg_mdp mqg_mdp;

typedef struct {
    uint64_t seed;          /* seeds the Q-network initialisation and the epsilon-greedy draws */
    uint32_t bits_min;      /* paper: 2 */
    uint32_t bits_max;      /* paper: 8 */
    uint32_t window;        /* T, losses per MDP state; paper: 5 */
    uint32_t decide_every;  /* training iterations between decisions; paper: T = 5 */
    uint32_t hidden;        /* hidden units of the Q network; paper: 10 */
    double alpha;           /* moving-average weight of Eq. (1); paper: 0.01 */
    double epsilon;         /* exploration rate; paper: 0.1 */
    double eta;             /* SARSA step size; paper: 0.1 */
    double reward_scale;    /* gamma of the reward equation; paper: 300 */
    double discount;        /* gamma of the SARSA update; the paper gives no value */
    uint32_t follow_taken_action;  /* 0 (paper): the state's width n_t moves by the greedy action (Transition);
                                      1: by the action that was taken, so the announced width never drops back */
} mqg_mdp_config;

/* Fill cfg with the paper's values (Section 4.1), discount = 0.9 and follow_taken_action = 0. */
void mqg_mdp_default_config(mqg_mdp_config* cfg);

/* Create / destroy an agent.  Returns NULL for an invalid configuration
 * (bits_min < 1, bits_max > 8, bits_min > bits_max, window < 2, decide_every < 1, hidden < 1). */
mqg_mdp* mqg_mdp_create(const mqg_mdp_config* cfg);
void mqg_mdp_destroy(mqg_mdp* agent);

/* Feed the global loss of training iteration m = 0, 1, 2, ... and the wall time (ms) that the
 * previous iteration took; returns the number of bits K = n_t + a_t to use for iteration m.  K
 * changes only when m is a multiple of decide_every.  The state's width n_t never decreases; an
 * exploratory "one more bit" (a_t = 1 against the greedy choice) lasts for one period, as the
 * paper's transition function moves n_t by the greedy action only.  Returns 0 if agent is NULL. */
uint32_t mqg_mdp_step(mqg_mdp* agent, double loss, double elapsed_ms);

/* The same from the workers' local losses: the server restores the global loss as their mean over the
 * P workers (Algorithm 1, ReceiveLossThenSendbits), summed in worker order, and steps the agent with it.
 * Returns 0 if agent or worker_losses is NULL or P is 0. */
uint32_t mqg_mdp_step_workers(mqg_mdp* agent, const double* worker_losses, uint32_t P, double elapsed_ms);

/* Introspection for tests: current n_t, the smoothed-loss window (writes `window` doubles,
 * oldest first), the last reward, and the number of decisions taken so far. */
uint32_t mqg_mdp_current_bits(const mqg_mdp* agent);
void mqg_mdp_smoothed_losses(const mqg_mdp* agent, double* out);
double mqg_mdp_last_reward(const mqg_mdp* agent);
uint64_t mqg_mdp_decisions(const mqg_mdp* agent);

/* The parameter vector v of the Q network (Section 3.3, Q function), for checkpointing an agent and for
 * tests of the SARSA update (Algorithm 2): mqg_mdp_num_weights doubles laid out as
 * [W1: hidden x window, row by row | b1: hidden | W2: (bits_max - bits_min + 1) x hidden | b2].
 * mqg_mdp_q_values evaluates the network as it stands: `input` holds `window` values (the smoothed
 * losses divided by the first loss), `out` receives one value per bit width; Q(s, a) is
 * out[n - bits_min + a].  NULL arguments are ignored. */
uint32_t mqg_mdp_num_weights(const mqg_mdp* agent);
void mqg_mdp_get_weights(const mqg_mdp* agent, double* out);
void mqg_mdp_set_weights(mqg_mdp* agent, const double* in);
void mqg_mdp_q_values(const mqg_mdp* agent, const double* input, double* out);

#ifdef __cplusplus
}
#endif
#endif /* MQGRAD_H */
