/*
 * nz_trace.h -- benchmark aid of libnz.so, kept apart from the product interface in nz.h (it is not part of the
 * paper's path and it is the only thing in the library that keeps state: a pointer per host thread while armed).
 *
 * While armed for the calling thread, every nz_* entry point records events[0] on its stream before its first
 * kernel and events[i] after its i-th kernel, up to `count` events (hipEvent_t handles created by the caller, in a
 * host array that must stay alive while armed).  nz_trace_recorded() returns how many events the last call
 * recorded.  nz_trace_events(NULL, 0) disarms.  Kernel order:
 *   nz_compress       statistics, codebook + selector, encode
 *   nz_decompress     decode, finish (result record, zero-fill of rejected frames)
 *   nz_reduce_frames  init, stage A, decode B + add, fix (late RAW frames), codebook + selector, encode
 *   nz_reduce_k       init, stage operand 0, one interval per accumulated operand (add + fix), decode the last + add, fix,
 *                     codebook + selector, encode
 *   nz_reduce_local   init, decode + quantize local + add, fix, codebook + selector, encode
 *   nz_compress_rea   encode (every workgroup profiles the frame's sample first), finish
 *   nz_reduce_local_rea   init, decode + quantize local + add, fix, encode (profiles the staged sums first), finish
 * (nz_compress_sr, nz_compress_static: as nz_compress; the *_step forms as their namesakes.  With the delta
 * predictor the reduces run one more kernel, the statistics of the staged sums, inside the "codebook" interval.)
 */
#ifndef NZ_TRACE_H
#define NZ_TRACE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

void   nz_trace_events(void** events, size_t count);
size_t nz_trace_recorded(void);

#ifdef __cplusplus
}
#endif
#endif /* NZ_TRACE_H */
