/*
 * fastsgd.h -- C ABI of the MI355X (gfx950) FastSGD gradient codec.
 *
 * The codec is the encoder/decoder pair of FastSGD (arXiv 2112.04291, Section 3):
 *   encoder  = Algorithm 1 (GV-Encoder: sum of |v|, early-stop threshold sum/b^tau, reciprocal
 *              mapper Eq. 2, logarithm quantization Eq. 3, threshold filter, sign) followed by
 *              Algorithm 2 (GK-Encoder: delta keys Eq. 4, maximal length M, l-bit length flag,
 *              bit-level binary encoding) on the keys of the surviving values;
 *   decoder  = phases 1-4 of Section 3.1 (split by flags, prefix-sum deltas, scale integers back
 *              up, divide sum by them).
 *
 * Conventions for every entry point
 *   - Pointers named d_* are DEVICE pointers (readable/writable by kernels on the current
 *     device); everything else is host memory read during the call only.
 *   - The caller owns every buffer.  The library allocates no device memory and keeps no state
 *     between calls; two calls may run concurrently if they use different workspaces.
 *     (include/fastsgd_profile.h declares two measurement aids that do not follow these rules.)
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = default
 *     stream).  No entry point synchronises with the host.  Values only the device knows are
 *     reported through the d_* result words, valid once the stream has been synchronised.
 *   - The return value covers what the host can see (bad arguments, workspace too small, launch
 *     failure).  Conditions detected on the device set *d_status to a fastsgd_status value and
 *     the reported length (bytes / pairs) to 0; nothing is ever written past a stated capacity.
 *   - Where several device-detected conditions hold at once the encoder reports, in this order, a
 *     non-finite value, keys out of order, an output buffer too small.  (A sequential encoder would
 *     report whichever of the last two it meets first; both verdicts describe the same refused input.)
 *     The decoders check the header and the pair capacity before anything else (a header that is
 *     corrupt, then a capacity that is too small); the decoders that update dense arrays meet keys
 *     beyond those arrays while they decode, and report a corrupt stream in preference to such a key.
 *   - Keys are uint32 and strictly increasing within one gradient (the first may be 0);
 *     values are IEEE binary32.  n <= 2^32 - 1024 per gradient.
 *
 * Stream layout (little-endian): 64-byte header {"FSGD", version u8, l u8, tau u16,
 * block_keys u32, n_blocks u32, b f64, sum f64, n u64, d u64, total_bytes u64, 0 u64}; value
 * plane of d tokens of 1 + ceil(log2 tau) bits (Section 3.2; low bits code-1, top bit sign; token j
 * at bit j * width, LSB first; one byte each for tau in 65..128, nine bits for tau in 129..256)
 * zero-padded to 8 bytes; block
 * directory of n_blocks x {off8 u32, preKey u32, M u32, payload_bits u32}; key blocks back to
 * back, each a flags plane
 * (cnt*l bits) and a payload plane (payload_bits bits), LSB first, zero-padded to 64-bit words.
 */
#ifndef FASTSGD_H
#define FASTSGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Hyper-parameters of Section 4.2 ("effect of the hyper-parameters"): base b of the logarithm
 * quantization, threshold tau of the filter, size l of the length flag; block_keys is how many
 * surviving keys share one M (Algorithm 2 is applied per block, preKey carried across). */
typedef struct {
    double   base;       /* b: 1 + 2^-20 <= b <= 16 (paper: about 1.1); <= 4 when tau > 128,
                            so that b^tau stays finite                             */
    uint32_t tau;        /* 1..256 (paper: 128, so a code fits one byte with sign;
                            smaller tau gives narrower codes, larger tau nine-bit
                            ones, see the stream layout)                            */
    uint32_t flag_bits;  /* l: 1..5 (paper: 2)                                     */
    uint32_t block_keys; /* power of two, 256..4096 (default 1024)                 */
    uint32_t reserved;   /* must be 0                                              */
} fastsgd_params;

typedef enum {
    FASTSGD_OK = 0,
    FASTSGD_ERR_INVALID_ARG = 1,
    FASTSGD_ERR_BUFFER_TOO_SMALL = 2, /* output / pair capacity or workspace too small      */
    FASTSGD_ERR_NONFINITE = 3,        /* a NaN or infinity among the values                  */
    FASTSGD_ERR_UNSORTED_KEYS = 4,    /* surviving keys not strictly increasing             */
    FASTSGD_ERR_CORRUPT_STREAM = 5,   /* decoder: header, directory or planes inconsistent  */
    FASTSGD_ERR_DEVICE = 6            /* HIP launch failure                                  */
} fastsgd_status;

/* Host-only, pure.  Worst-case stream size in bytes for a gradient of n elements (all survive,
 * every key token takes l + 32 bits); Section 3.4 gives the expected size, this is the bound an
 * output buffer must have.  Returns 0 if *p is invalid. */
size_t fastsgd_compressed_size(uint64_t n, const fastsgd_params* p);

/* Host-only, pure.  Bytes of device workspace fastsgd_compress (n_segments = 1) or
 * fastsgd_compress_segmented needs for total_n elements in n_segments gradients whose smallest
 * block_keys is min_block_keys (about 6 bytes per element: the scratch keys and codes of the
 * survivors, whose number is not known beforehand).  Returns 0 on invalid arguments. */
size_t fastsgd_workspace_size(uint64_t total_n, uint32_t n_segments, uint32_t min_block_keys);

/* The same for a caller that knows the largest threshold tau it will pass: up to 128 a code takes
 * one byte of scratch instead of two (about 5 bytes per element instead of 6).  A call whose tau
 * needs more than its workspace has returns FASTSGD_ERR_BUFFER_TOO_SMALL.  Returns 0 on invalid
 * arguments (max_tau 1..256). */
size_t fastsgd_workspace_size_tau(uint64_t total_n, uint32_t n_segments, uint32_t min_block_keys,
                                  uint32_t max_tau);

/* Host-only, pure.  Bytes of device workspace the decoders need for n_segments streams.
 * The first 4096 bytes of a decoder workspace hold control words that must be ZERO before the workspace's
 * first use (clear them once after allocating it); every decoder call leaves them zero again, so the
 * workspace can be reused call after call without further clearing.  The rest needs no initialisation. */
size_t fastsgd_decompress_workspace_size(uint32_t n_segments);

/* Encoder (Algorithms 1 and 2) for one worker's gradient {(k_j, v_j)}, j = 1..n.
 *   d_keys, d_values   device, read-only, n entries each (4-byte aligned); d_keys may be NULL
 *                      for a dense gradient, whose keys are then 0..n-1 (the stream is the one
 *                      the explicit keys 0..n-1 give; the key array is never read)
 *   p                  host
 *   d_out              device, out_capacity bytes, 8-byte aligned; receives the stream
 *   d_out_bytes        device u64: stream length, or 0 if *d_status != FASTSGD_OK
 *   d_status           device u32: fastsgd_status detected on the device
 *   d_workspace        device, >= fastsgd_workspace_size(n, 1, p->block_keys) bytes, 256-byte aligned;
 *                      contents need no initialisation and are garbage afterwards */
fastsgd_status fastsgd_compress(const uint32_t* d_keys, const float* d_values, uint64_t n,
                                const fastsgd_params* p,
                                void* d_out, size_t out_capacity,
                                uint64_t* d_out_bytes, uint32_t* d_status,
                                void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* fastsgd_compress for callers that cannot allocate or hand over a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same stream byte for
 * byte, but the workspace is a fixed array of FASTSGD_STATIC_SCRATCH_BYTES inside the library (one per
 * GPU, held until the process ends).  The call allocates nothing on host or device.
 *   n                  at most FASTSGD_STATIC_MAX_ELEMS, else FASTSGD_ERR_BUFFER_TOO_SMALL is returned
 *                      and nothing is enqueued
 * Every call on one GPU shares that GPU's array: calls that overlap in time on one GPU (different streams,
 * or graph launches in flight together) race and give undefined streams; calls on one stream, or otherwise
 * ordered, are fine -- each call clears the control words it relies on.  The first call on a device looks
 * the array's address up (no stream work); make it outside any graph capture.
 * Returns FASTSGD_ERR_DEVICE if that lookup fails. */
#define FASTSGD_STATIC_MAX_ELEMS 1048576ull
#define FASTSGD_STATIC_SCRATCH_BYTES (8u << 20)
fastsgd_status fastsgd_compress_static(const uint32_t* d_keys, const float* d_values, uint64_t n,
                                       const fastsgd_params* p,
                                       void* d_out, size_t out_capacity,
                                       uint64_t* d_out_bytes, uint32_t* d_status, void* hip_stream);

/* Decoder (Section 3.1, phases 1-4) of one stream.
 *   d_stream           device, stream_bytes bytes, 8-byte aligned
 *   d_keys_out, d_values_out   device, `capacity` entries each; receive the d surviving pairs
 *   d_count            device u64: d, or 0 if *d_status != FASTSGD_OK
 *   d_workspace        device, >= fastsgd_decompress_workspace_size(1) bytes, 256-byte aligned, control
 *                      words zero (see fastsgd_decompress_workspace_size)
 * One kernel launch: the header is checked and the table of decoded magnitudes rebuilt inside it.  A stream
 * in which a key repeats its predecessor (a delta of 0 anywhere but at the first key) is corrupt. */
fastsgd_status fastsgd_decompress(const void* d_stream, size_t stream_bytes,
                                  uint32_t* d_keys_out, float* d_values_out, uint64_t capacity,
                                  uint64_t* d_count, uint32_t* d_status,
                                  void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Encoder for a batch of independent gradients (e.g. one per layer) in one call: gradient s is
 * elements [seg_offsets[s], seg_offsets[s+1]) of d_keys / d_values and is encoded exactly as
 * fastsgd_compress would encode it alone (d_keys NULL: every gradient has the keys 0..n_s-1).
 * Streams are written back to back into d_out (each a
 * multiple of 8 bytes, each decodable on its own).
 *   seg_offsets        host, n_segments + 1 non-decreasing element offsets
 *   params             host; params_stride = 0: one entry shared by all segments,
 *                      params_stride = 1: n_segments entries
 *   d_out_seg_offsets  device u64[n_segments + 1]: byte offset of each stream in d_out, last
 *                      entry = total bytes; all 0 if *d_status != FASTSGD_OK
 *   n_segments         1..65536 */
fastsgd_status fastsgd_compress_segmented(const uint32_t* d_keys, const float* d_values,
                                          const uint64_t* seg_offsets, uint32_t n_segments,
                                          const fastsgd_params* params, uint32_t params_stride,
                                          void* d_out, size_t out_capacity,
                                          uint64_t* d_out_seg_offsets, uint32_t* d_status,
                                          void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Decoder for such a batch.
 *   d_streams, total_bytes   device, the concatenated streams
 *   d_stream_offsets   device u64[n_segments + 1] as written by fastsgd_compress_segmented
 *   d_keys_out, d_values_out   device, `capacity` pairs; pairs of segment s start at
 *                      d_pair_offsets[s]
 *   d_pair_offsets     device u64[n_segments + 1]; all 0 if *d_status != FASTSGD_OK */
fastsgd_status fastsgd_decompress_segmented(const void* d_streams, size_t total_bytes,
                                            const uint64_t* d_stream_offsets, uint32_t n_segments,
                                            uint32_t* d_keys_out, float* d_values_out, uint64_t capacity,
                                            uint64_t* d_pair_offsets, uint32_t* d_status,
                                            void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Decoder followed by the aggregation the decoded gradients are for (Section 2.1, Fig. 1: the
 * workers' gradients are decoded and added up before the model update): for every pair (k, v)
 * of every stream, d_dense[k] += v, a binary32 addition.  At every key the streams are added in
 * the given order and keys are unique inside a stream, so the result does not depend on how the
 * work is spread over the GPU: sparse streams are added by one decode launch per stream, dense
 * ones (from about one kept entry in two hundred on, if d_dense is 16-byte aligned) in one pass
 * over d_dense per group of eight streams, with the same sums.
 * If several streams fail, or one fails in several ways, *d_status holds the gravest failure:
 * a corrupt stream outranks a key beyond the dense vector.
 *   d_streams, total_bytes   device, the concatenated streams of the workers, 8-byte aligned
 *   d_stream_offsets   device u64[n_streams + 1]: byte offset of each stream, each a multiple of 8
 *   d_dense, dense_len device float[dense_len], updated in place; a decoded key >= dense_len
 *                      sets *d_status = FASTSGD_ERR_BUFFER_TOO_SMALL
 *   d_count            device u64: pairs added, or 0 if *d_status != FASTSGD_OK (d_dense then
 *                      holds an unspecified partial sum)
 *   d_workspace        device, >= fastsgd_decompress_workspace_size(n_streams) bytes, 256-aligned
 *   n_streams          1..65536 */
fastsgd_status fastsgd_decompress_accumulate(const void* d_streams, size_t total_bytes,
                                             const uint64_t* d_stream_offsets, uint32_t n_streams,
                                             float* d_dense, uint64_t dense_len,
                                             uint64_t* d_count, uint32_t* d_status,
                                             void* d_workspace, size_t workspace_bytes, void* hip_stream);

/* Hyper-parameters of the Adam SGD update of Section 4.1 (paper: beta1 = 0.9, beta2 = 0.999,
 * eps = 1e-8, eta tuned by grid search). */
typedef struct {
    double eta;    /* learning rate                 */
    double beta1;  /* 0..1                          */
    double beta2;  /* 0..1                          */
    double eps;    /* >= 0, added under the root    */
} fastsgd_adam;

/* Decoder followed by the model update of Section 4.1 at the decoded keys: for every pair (k, g)
 * of the stream,  m[k] = beta1 m[k] + (1 - beta1) g,  v[k] = beta2 v[k] + (1 - beta2) g^2,
 * theta[k] -= eta m[k] / sqrt(v[k] + eps)  (the two equations as printed: eps under the root, no
 * bias correction), in binary32.  Coordinates that are not in the stream are not touched.
 *   d_stream, stream_bytes   device, 8-byte aligned: one stream (e.g. the re-encoded aggregate,
 *                      or one worker's gradient)
 *   d_theta, d_m, d_v  device float[dim], updated in place; a decoded key >= dim sets
 *                      *d_status = FASTSGD_ERR_BUFFER_TOO_SMALL
 *   h                  host
 *   d_count            device u64: pairs applied, or 0 if *d_status != FASTSGD_OK (the arrays then
 *                      hold an unspecified partial update)
 *   d_workspace        device, >= fastsgd_decompress_workspace_size(1) bytes, 256-byte aligned */
fastsgd_status fastsgd_decompress_adam(const void* d_stream, size_t stream_bytes,
                                       float* d_theta, float* d_m, float* d_v, uint64_t dim,
                                       const fastsgd_adam* h,
                                       uint64_t* d_count, uint32_t* d_status,
                                       void* d_workspace, size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FASTSGD_H */
