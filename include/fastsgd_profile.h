/*
 * fastsgd_profile.h -- measurement aids of the MI355X (gfx950) FastSGD codec.
 *
 * NOT part of the production interface of fastsgd.h and exempt from its conventions: the two profiling
 * calls create and destroy HIP events (which allocates), and they WAIT for the stream before returning.  They
 * exist so that a benchmark can split the encoder's and the decoder's time per kernel (Section 4.2 of the
 * paper, "time breakdown", reports encoder and decoder time separately; these split each further).
 *
 * Same arguments and results as fastsgd_compress / fastsgd_decompress, run `iterations` (1..4096) times
 * back to back with a HIP event recorded on hip_stream before the first and after every kernel; the
 * average milliseconds per kernel are stored in kernel_ms (host).  Kernel order, compress: abs-sum,
 * tables, encode-values, measure-keys (with the scan of the chunk counts in front of it), pack-keys;
 * decompress: decode (its only kernel).
 */
#ifndef FASTSGD_PROFILE_H
#define FASTSGD_PROFILE_H

#include "fastsgd.h"

#ifdef __cplusplus
extern "C" {
#endif

#define FASTSGD_PROFILE_COMPRESS_KERNELS 5
#define FASTSGD_PROFILE_DECOMPRESS_KERNELS 1
fastsgd_status fastsgd_profile_compress(const uint32_t* d_keys, const float* d_values, uint64_t n,
                                        const fastsgd_params* p,
                                        void* d_out, size_t out_capacity,
                                        uint64_t* d_out_bytes, uint32_t* d_status,
                                        void* d_workspace, size_t workspace_bytes, void* hip_stream,
                                        uint32_t iterations, float* kernel_ms);
fastsgd_status fastsgd_profile_decompress(const void* d_stream, size_t stream_bytes,
                                          uint32_t* d_keys_out, float* d_values_out, uint64_t capacity,
                                          uint64_t* d_count, uint32_t* d_status,
                                          void* d_workspace, size_t workspace_bytes, void* hip_stream,
                                          uint32_t iterations, float* kernel_ms);

/* Plain streaming read of `bytes` bytes at d_src (16-byte aligned) on hip_stream: every byte is loaded
 * once with the access pattern of the codec's first value pass (16 bytes per lane, neighbouring workgroups
 * on neighbouring tiles) and nothing else is done with it.  Timed by the caller, it gives the read
 * bandwidth this GPU actually sustains, the practical ceiling next to the published peak.  Enqueues one
 * kernel, allocates nothing, does not wait.  d_sink: device u64, written only if the data hashes to one
 * particular value (it keeps the loads alive). */
fastsgd_status fastsgd_probe_read(const void* d_src, size_t bytes, uint64_t* d_sink, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* FASTSGD_PROFILE_H */
