/*
 * nz.h -- C ABI of the MI355X (gfx950) per-rank compression path.
 *
 * The path is the per-rank pipeline that sits in front of and behind a
 * collective's transport: interface quantizer (Sec. IV-A/IV-B of the paper),
 * device-side runtime entropy arbitration among RAW / FIXEDLEN / HUFFMAN
 * (Sec. IV-C, Eq. 1-2, Algorithm 1), self-describing frames (Sec. IV-D "Batch
 * Framing"), receiver-side validate + decode (Algorithm 2, receiver side) and
 * the compute part of the fused receive-decode-reduce-encode-send step
 * (Sec. IV-D "In-Primitive Overlap").
 *
 * Conventions for every entry point
 *   - Pointers named d_* are DEVICE pointers (hipMalloc'd or PyTorch-owned),
 *     16-byte aligned; `opts` is a HOST pointer (may be NULL = defaults).
 *   - The caller owns every buffer.  The library allocates nothing, keeps no
 *     state between calls, enqueues its kernels on `stream` (a hipStream_t
 *     passed as void*) and never synchronises it.  Two calls may run
 *     concurrently only if they use different workspaces and outputs.
 *     (The optional benchmark aid in nz_trace.h is the one exception: it
 *     keeps a per-host-thread pointer while armed.)
 *   - The return value reports what the host can check before launching
 *     (NZ_ERR_INVALID arguments, a workspace or output too small to hold even
 *     the stream header, a failed launch = NZ_ERR_HIP).  Everything detected
 *     on the device is written to d_res->status once the stream has run; when
 *     several conditions hold the numerically largest code is reported.
 *   - No kernel reads or writes outside [d_out, d_out+out_cap), the given
 *     input lengths, or the workspace, whatever the input bytes are.
 *   - `eb` is an ABSOLUTE error bound: finite, 2^-100 <= eb <= 2^100.  A
 *     range-relative bound (the paper's REL, Sec. V-B) is converted by the
 *     caller: eb = REL * (max - min).
 */
#ifndef NZ_H
#define NZ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NZ_OK           = 0,
    NZ_ERR_INVALID  = 1,   /* bad argument (n = 0, eb out of range, misaligned pointer, bad opts)        */
    NZ_ERR_CAPACITY = 2,   /* output does not fit out_cap: nothing is published (Algorithm 1 returns 0) */
    NZ_ERR_CORRUPT  = 3,   /* a stream or frame failed validation (Algorithm 2, ValidateHeader)         */
    NZ_ERR_MISMATCH = 4,   /* n, frame size, alphabet, predictor or quantization step differ from the stream's */
    NZ_ERR_HIP      = 5    /* a HIP launch failed (host return value only)                              */
} nz_status;

typedef enum { NZ_CODEC_RAW = 0, NZ_CODEC_FIXEDLEN = 1, NZ_CODEC_HUFFMAN = 2 } nz_codec;

/* Options; zero in a size field selects the default. */
typedef struct {
    uint32_t chunk_elems;      /* fp32 elements per frame, 1..2^20 (the paper's frame is one 4 MiB channel
                                  buffer, Sec. IV-D "8-slot batching"); default 262144 (1 MiB)              */
    uint32_t seg_syms;         /* symbols per independently decodable Huffman segment.  The stream format
                                  allows 32..1024; these kernels encode and decode one segment per wavefront
                                  pass (64 lanes x 4 symbols), so only 256 (or 0 = default) is accepted and
                                  any other value is NZ_ERR_INVALID from every entry point                  */
    uint32_t alphabet;         /* Huffman alphabet K (escape + K-1 symbols), power of two 2..1024;
                                  default 256 (the paper's selector profiles a 256-bin histogram, Sec. IV-C) */
    int32_t  force_codec;      /* -1 = arbitrate; 0/1/2 pin RAW/FIXEDLEN/HUFFMAN as the paper does for its
                                  ratio study (Sec. V-B)                                                    */
    uint32_t min_gain_permil;  /* minimum-gain threshold of Algorithm 1 (minGainPermil), 0..1000            */
    uint32_t huff_min_bytes;   /* Huffman size threshold T_huff of Algorithm 1 on the frame's raw bytes     */
    uint32_t predictor;        /* 0 = none (the paper's path).  1 = delta, an extension in front of the entropy
                                  stage (the prediction stage of the SZ-style pipeline of Sec. II-B): what is
                                  coded for element i of a frame is q[i] - q[i-1] modulo 2^32, q[i] itself at
                                  the start of every 256-symbol segment; lossless and linear, so streams still
                                  reduce exactly.  A stream records its predictor; decompress and reduce must
                                  be called with the same value (else NZ_ERR_MISMATCH).  nz_compress_rea and
                                  nz_compress_sr accept 0 only.                                              */
    uint32_t reserved;         /* 0                                                                        */
} nz_opts;

/* Result record, lives in DEVICE memory, valid once the stream has executed the call. */
typedef struct {
    uint64_t bytes;            /* compress/reduce: stream bytes written (0 on any error);
                                  decompress: total_bytes field of the stream header                        */
    uint32_t status;           /* nz_status                                                                 */
    uint32_t n_frames;
    uint32_t n_raw, n_fixed, n_huff;   /* frames per chosen (compress/reduce) or found (decompress) codec   */
    uint32_t reserved;
} nz_result;

/* Host, pure.  Capacity that always suffices (the payload budget of Algorithm 1, lines 1-4: a frame is
 * committed only if it fits, and RAW must fit for the safe fallback to exist): every frame RAW.  A pinned
 * HUFFMAN can exceed RAW and is bounded at 60 bits per symbol (a 28-bit code plus the 32 bits of an escaped
 * value).  0 when n = 0 or opts are invalid. */
size_t nz_compress_bound(size_t n, const nz_opts* opts);

/* Host, pure.  Workspace bytes nz_compress / nz_decompress need for n elements (0 on invalid opts). */
size_t nz_workspace_bytes(size_t n, const nz_opts* opts);

/* Host, pure.  Workspace bytes nz_reduce_frames needs: about 12 bytes per element (operand A between the two
 * decode passes, and the sums handed to the encoder, each staged as 16-bit codes with a 32-bit spill array). */
size_t nz_reduce_workspace_bytes(size_t n, const nz_opts* opts);

/*
 * Quantize d_in[0..n) with bin width fl32(eb*63/32) and write an NZ stream:
 * per frame of chunk_elems elements the exact sizes of the three codecs are
 * computed from the frame's full statistics and the smallest admissible one is
 * materialised (Eq. 2 with transmitted size as the cost; Algorithm 1's gates
 * are min_gain_permil, huff_min_bytes, force_codec and out_cap).  A frame with
 * a value that cannot be quantized within eb (NaN, Inf, |x| > 32767 bins) is
 * RAW and carries the fp32 input unchanged.
 *   d_out/out_cap  device output and its capacity in bytes; a stream larger
 *                  than out_cap sets NZ_ERR_CAPACITY and bytes = 0.
 *   d_ws/ws_bytes  device scratch of at least nz_workspace_bytes(n, opts).
 */
nz_status nz_compress(const float* d_in, size_t n, float eb, void* d_out, size_t out_cap, nz_result* d_res,
                      const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream);

/*
 * Sampled runtime entropy arbitration: Algorithm 1 taken literally (Sec. IV-C).
 *
 * nz_context_build makes the "pre-initialized Huffman context" / "cached codebook" of Sec. IV-C: one canonical
 * code over the K symbols of the alphabet, built from a calibration message d_sample[0..n_sample) (n_sample <=
 * 2^20, quantized with eb like any message): symbol counts plus one each (every symbol, the escape included, owns
 * a code), optimal lengths, canonical codes.  d_ctx: device memory of nz_context_bytes() bytes, 16-byte aligned,
 * reusable for any number of messages; d_ws: at least 4096 bytes of device scratch.
 *
 * nz_compress_rea: per frame, ProfileSample reads a prefix of at most sample_bytes (64 KiB) of the frame;
 * ArbitratePlan predicts FIXEDLEN from the width of the sample's largest code and HUFFMAN from the sample's
 * expected code length under the context, applies the gates (SmallBatchFastPath, T_huff = huff_min_bytes, context
 * valid for this alphabet, minimum gain, payload capacity) and takes the candidate of least predicted cost (Eq. 2;
 * the cost is Eq. 1 under the caller's transport hint, or the transmitted size without one; force_codec pins the plan); EncodePlan runs only the planned codec over the frame,
 * in one pass over the input; AcceptRealized checks the realized payload (materialised, fits, minimum gain) and
 * CommitRawOrFail stores the frame RAW otherwise.  d_ctx may be NULL (no Huffman).
 * Output: an NZ stream that nz_decompress / nz_reduce_* read like any other, except that frame k starts at the
 * fixed offset 64 + pad16(8*n_frames) + k * pad16(32 + 4*chunk_elems): every frame is materialised in a slot that
 * can hold its RAW form (the paper's staging bank) and carries its byte-accurate length in its header; the bytes
 * between a frame's end and the next slot are not written.  out_cap must hold every slot (nz_compress_bound with
 * force_codec = -1), else NZ_ERR_CAPACITY (return value and d_res->status) and nothing is written.
 *   d_ws/ws_bytes  device scratch of at least nz_rea_workspace_bytes(n, opts).
 */
typedef struct {
    uint32_t sample_bytes;       /* SampleWindow: bytes of the frame's prefix that are profiled; 0 = 65536       */
    uint32_t small_batch_bytes;  /* SmallBatchFastPath: frames with fewer raw bytes are RAW unprofiled; default 0 */
    /* Cost model of Eq. 1, T_c = alpha_c + lambda_enc*E_c + P_c/beta_eff(pi) + lambda_dec*D_c, in integers.  The
     * caller supplies what TransportHint and its calibration would: link_ps_per_byte = 1/beta_eff in picoseconds per
     * byte (8 TB/s = 0.125, 25 GB/s = 40; 0 = no hint: the cost is the predicted transmitted size alone), and for
     * each entropy codec the fixed cost alpha_c in nanoseconds and the exposed codec time lambda_enc*E_c +
     * lambda_dec*D_c in picoseconds per raw byte.  ArbitratePlan takes the admissible candidate with the least
     * T_c = 1000*alpha_c + codec_ps_c*rawBytes + link_ps*predictedTotal_c (RAW: link_ps*total_RAW), ties to the
     * lower codec id: on a fast link RAW is the planned outcome, not a fallback (Sec. IV-C). */
    uint32_t link_ps_per_byte;
    uint32_t fixed_alpha_ns, fixed_ps_per_byte;
    uint32_t huff_alpha_ns, huff_ps_per_byte;
    uint32_t reserved;           /* 0 */
} nz_rea_opts;

typedef struct {                 /* lives in DEVICE memory, 16-byte aligned */
    uint64_t span_bytes;         /* extent of the slotted stream: what nz_decompress is handed (0 on error)      */
    uint64_t wire_bytes;         /* stream header + offsets table + realized frames: what a transport sends      */
    uint32_t status;             /* nz_status                                                                     */
    uint32_t n_frames;
    uint32_t n_raw, n_fixed, n_huff;   /* frames per committed codec                                              */
    uint32_t n_fallback;         /* frames planned FIXEDLEN / HUFFMAN whose realized output was rejected (now RAW) */
} nz_rea_result;

size_t    nz_context_bytes(void);
nz_status nz_context_build(const float* d_sample, size_t n_sample, float eb, const nz_opts* opts, void* d_ctx, void* d_ws,
                           size_t ws_bytes, void* stream);
size_t    nz_rea_workspace_bytes(size_t n, const nz_opts* opts);
nz_status nz_compress_rea(const float* d_in, size_t n, float eb, const void* d_ctx, void* d_out, size_t out_cap,
                          nz_rea_result* d_res, const nz_opts* opts, const nz_rea_opts* ropts, void* d_ws, size_t ws_bytes,
                          void* stream);

/*
 * The ring step with the sampled arbitration on the way out: nz_reduce_local whose output frames are committed by
 * Algorithm 1 instead of the exact selector, as in the paper's receive-reduce-send pipeline (Sec. IV-D with Sec. IV-C
 * in front of the send).  The incoming stream is decoded and the rank's own data quantized and added as in
 * nz_reduce_local; every frame of integer sums is then planned from a prefix sample of its sums and the cached
 * context, only the planned codec is materialised, the realized size validated, and the frame stored RAW otherwise.
 * A RAW frame of integer sums (planned so, or fallen back) holds fl32(fl32(qa*step) + fl32(qb*step)); a frame that
 * has no integer sums (incoming frame RAW, local value that cannot be quantized, a sum beyond 2^30) is RAW with the
 * fp32 sums of nz_reduce_local and counts neither as planned nor as fallback.  Output: the slotted stream of
 * nz_compress_rea; d_res as there (status carries an error of the incoming stream; then nothing is published).
 *   d_ws/ws_bytes  device scratch of at least nz_reduce_rea_workspace_bytes(n, opts).  opts.predictor must be 0.
 */
size_t    nz_reduce_rea_workspace_bytes(size_t n, const nz_opts* opts);
nz_status nz_reduce_local_rea(const void* d_in, size_t in_bytes, const float* d_local, size_t n, float eb, const void* d_ctx,
                              void* d_out, size_t out_cap, nz_rea_result* d_res, const nz_opts* opts, const nz_rea_opts* ropts,
                              void* d_ws, size_t ws_bytes, void* stream);

/*
 * Stochastic interface quantizer (QSGD, Sec. II-B "Quantization", Sec. IV-B): nz_compress_sr is nz_compress with
 * randomized rounding in the place of round-to-nearest.  Values are rounded to multiples of `step` (finite,
 * 2^-100 <= step <= 2^101): with a = |x| / step the level is floor(a) + 1 with probability a - floor(a), else
 * floor(a), so E[xhat] = x; |x - xhat| <= step * (1 + 2^-6); a value with a > 32767 or NaN makes its frame RAW.
 * Element i of the message draws from a counter-based generator keyed by (seed, i) -- the 32-bit finalizer of
 * MurmurHash3, top 24 bits -- so the result does not depend on how the work is scheduled.  Statistics, selector
 * and frames are those of nz_compress; the stream records `step`, and its receivers are the *_step forms below
 * (nz_decompress / nz_reduce_frames / nz_reduce_k derive the width from an error bound, which such a stream does
 * not have).
 * nz_qsgd_step writes QSGD's width for `levels` levels per sign, ||x||_2 / levels (at least 2^-100; NaN if the
 * message is not finite), to the device float *d_step; d_ws: at least 8192 bytes of device scratch.  Ranks that
 * reduce their streams must agree on one width (e.g. the largest).
 */
nz_status nz_qsgd_step(const float* d_in, size_t n, uint32_t levels, float* d_step, void* d_ws, size_t ws_bytes, void* stream);
nz_status nz_compress_sr(const float* d_in, size_t n, float step, uint32_t seed, void* d_out, size_t out_cap, nz_result* d_res,
                         const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream);
nz_status nz_decompress_step(const void* d_stream, size_t stream_bytes, float* d_out, size_t n, float step,
                             nz_result* d_res, const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream);
nz_status nz_reduce_frames_step(const void* d_a, size_t a_bytes, const void* d_b, size_t b_bytes, void* d_out,
                                size_t out_cap, size_t n, float step, nz_result* d_res, const nz_opts* opts,
                                void* d_ws, size_t ws_bytes, void* stream);
nz_status nz_reduce_k_step(const void* const* d_streams, const size_t* stream_bytes, uint32_t k, void* d_out, size_t out_cap,
                           size_t n, float step, nz_result* d_res, const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream);
/* The ring step of such a collective (Sec. IV-D, receive-reduce-send): nz_reduce_local with the stochastic quantizer
 * on the rank's own data, element i drawing from (seed, i); byte-identical to
 * nz_reduce_frames_step(d_in, nz_compress_sr(d_local, step, seed)).  opts.predictor must be 0. */
nz_status nz_reduce_local_sr(const void* d_in, size_t in_bytes, const float* d_local, void* d_out, size_t out_cap,
                             size_t n, float step, uint32_t seed, nz_result* d_res, const nz_opts* opts, void* d_ws,
                             size_t ws_bytes, void* stream);

/*
 * nz_compress for callers that cannot allocate or hand over scratch memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same result, byte for byte, as nz_compress; the
 * workspace is an array that lives inside the library on every GPU (nz_static_scratch_bytes() bytes, 8 MiB,
 * resident until the process ends) and the call allocates nothing.  The message must be small enough for
 * it: nz_workspace_bytes(n, opts) <= nz_static_scratch_bytes() (about 96 Mi elements in 1 MiB frames, 14 Mi
 * elements in 64 KiB frames), otherwise NZ_ERR_INVALID and nothing is launched.  NZ_ERR_HIP if the array's
 * address cannot be obtained on the current device.  All calls on one GPU share that GPU's array: calls that
 * overlap in time on the same GPU (different streams or threads) race and must be serialised by the caller.
 */
size_t    nz_static_scratch_bytes(void);
nz_status nz_compress_static(const float* d_in, size_t n, float eb, void* d_out, size_t out_cap, nz_result* d_res,
                             const nz_opts* opts, void* stream);

/*
 * Receiver side of Algorithm 2 (ParseHeader, ValidateHeader, DecodeOrMemcpy):
 * validate and decode an NZ stream into d_out[0..n): xhat = fl32(float(q) *
 * step); RAW frames are copied through.  n, eb and opts (chunk_elems,
 * alphabet) must be the ones the stream was produced with, otherwise
 * NZ_ERR_MISMATCH and nothing is written.  A stream header that fails
 * validation sets NZ_ERR_CORRUPT and nothing is written.  A frame that fails
 * validation -- at its header, or because a segment does not use exactly its
 * recorded bits -- sets NZ_ERR_CORRUPT, is not counted in n_raw/n_fixed/n_huff
 * and its whole output range is filled with zeros (the paper's receiver copies
 * rawBytes from an invalid frame; this format never hands bytes of an
 * untrusted frame to the caller); the other frames are decoded normally.
 *   d_ws/ws_bytes  device scratch of at least nz_workspace_bytes(n, opts).
 */
nz_status nz_decompress(const void* d_stream, size_t stream_bytes, float* d_out, size_t n, float eb,
                        nz_result* d_res, const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream);

/*
 * Fused decode(A), decode(B), integer add, re-arbitrate, re-encode, frame by
 * frame: the output decodes to qa+qb exactly, so no lossy step is repeated
 * (Sec. III "Error propagation").  A and B must have been produced with the
 * same n, eb and opts.  If either input frame is RAW the output frame is RAW
 * and holds the fp32 sum (NaN sums stored as 0x7FC00000).  A frame in which a
 * sum exceeds 2^30 in magnitude can no longer be carried as integer codes: it
 * is committed as RAW (the selector's safe fallback, Sec. IV-C) and holds
 * fl32(fl32(qa*step) + fl32(qb*step)); so does a frame of integer sums that
 * the selector commits RAW all the same (codec pinned to RAW, no entropy
 * candidate passes the gates): a RAW frame of a reduce always carries what the
 * receiver would have computed from the two operands.
 *   d_ws/ws_bytes  device scratch of at least nz_reduce_workspace_bytes(n, opts).
 */
nz_status nz_reduce_frames(const void* d_a, size_t a_bytes, const void* d_b, size_t b_bytes, void* d_out,
                           size_t out_cap, size_t n, float eb, nz_result* d_res, const nz_opts* opts,
                           void* d_ws, size_t ws_bytes, void* stream);

/*
 * k-ary reduce (the reduction of Sec. IV-D "In-Primitive Overlap" over all the
 * contributions a rank holds at once, e.g. the chunks of a direct or
 * tree-shaped reduce-scatter): out = s_0 (+) s_1 (+) ... (+) s_{k-1}, every
 * operand decoded once and the sum encoded once.  The operands are folded in
 * the order given with the rule of nz_reduce_frames, frame by frame: codes are
 * added exactly while the running value and the operand's frame are both coded;
 * at the operand where a partial sum passes 2^30 in magnitude, or whose frame
 * is RAW, the running value becomes fp32 (fl32(v + v_p), v and v_p dequantized
 * or raw) and stays fp32.  Byte-identical to the chain nz_reduce_frames(...
 * nz_reduce_frames(s_0, s_1) ..., s_{k-1}) as long as the chain's intermediate
 * streams keep integer sums as codes; opts that turn such frames RAW (pinned
 * RAW, gates) apply to the final stream only.  k = 2 is nz_reduce_frames.
 *   d_streams / stream_bytes  HOST arrays of k device pointers (16-byte aligned
 *                  NZ streams made with the same n, eb and opts) and their sizes;
 *                  read during the call only.  2 <= k <= 64, else NZ_ERR_INVALID.
 *   d_ws/ws_bytes  device scratch of at least nz_reduce_workspace_bytes(n, opts).
 * Errors as for nz_reduce_frames (a stream-level or frame-level error in any
 * operand fails the call: status set, bytes = 0).
 */
nz_status nz_reduce_k(const void* const* d_streams, const size_t* stream_bytes, uint32_t k, void* d_out, size_t out_cap,
                      size_t n, float eb, nz_result* d_res, const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream);

/*
 * Ring-step reduce (the receive-reduce-send step of Sec. IV-D "In-Primitive
 * Overlap"): out = incoming stream (+) the rank's own fp32 data d_local[0..n).
 * The local data is quantized exactly as nz_compress would quantize it (Sec.
 * IV-B) but is never entropy coded; the result is byte-identical to
 * nz_reduce_frames(d_in, nz_compress(d_local)).  A local frame holding an
 * element that cannot be quantized counts as RAW: the output frame is RAW and
 * holds incoming value + original local value.  d_in is an NZ stream made with
 * the same n, eb and opts; d_local is device memory, 16-byte aligned; the
 * workspace is that of nz_reduce_frames (nz_reduce_workspace_bytes).  Errors as
 * for nz_reduce_frames.
 */
nz_status nz_reduce_local(const void* d_in, size_t in_bytes, const float* d_local, void* d_out, size_t out_cap,
                          size_t n, float eb, nz_result* d_res, const nz_opts* opts, void* d_ws, size_t ws_bytes,
                          void* stream);

/* Library version (format version in the high 16 bits, build in the low 16). */
uint32_t nz_version(void);

#ifdef __cplusplus
}
#endif
#endif /* NZ_H */
