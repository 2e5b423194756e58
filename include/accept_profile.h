/*
 * accept_profile.h -- measurement entry points of libaccept: per-kernel durations of a call.
 * Not part of the compression interface (accept.h): these functions create HIP events,
 * wait for the device and exist for benchmarks and profiles only.
 */
#ifndef ACCEPT_PROFILE_H
#define ACCEPT_PROFILE_H

#include "accept.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Measurement variants: same work as accept_compress / accept_decompress, but every
 * kernel the call launches is bracketed by HIP events on the given stream; the call then
 * WAITS for the last event and writes each stage's duration in milliseconds to the host
 * array stage_ms[0..*n_stages) (capacity ACCEPT_MAX_STAGES).  Stage order:
 *   UNIFORM compress: range, [range finalize], quantize+pack;   MBQ compress: encode+sums, finalize;
 *   decompress: the one kernel.
 * For benchmarks only; creates and destroys its events on every call.
 */
enum { ACCEPT_MAX_STAGES = 8 };
accept_status accept_compress_timed(const accept_desc* desc, const void* x_dev, const float* alpha_prev_dev,
                                    void* header_dev, void* payload_dev, void* workspace_dev, void* hip_stream,
                                    float* stage_ms, int* n_stages);
accept_status accept_decompress_timed(const accept_desc* desc, const void* header_dev, const void* payload_dev,
                                      void* xhat_dev, void* hip_stream, float* stage_ms, int* n_stages);

/* Name of stage i of the call accept_*_timed would make for this descriptor
 * (is_decompress = 0/1); null when i is out of range.  Host-only. */
const char* accept_stage_name(const accept_desc* desc, int is_decompress, int i);

#ifdef __cplusplus
}
#endif
#endif /* ACCEPT_PROFILE_H */
