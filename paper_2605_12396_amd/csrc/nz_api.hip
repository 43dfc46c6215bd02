// nz_api.hip -- extern "C" boundary: argument checks, workspace carve-up and kernel launches.
// Host code only validates and launches; every step of the path runs in the kernels.
#include "../../include/nz.h"
#include "../../include/nz_trace.h"
#include "nz_common.hpp"
#include <mutex>

using namespace nz;

namespace {

struct Opts { uint32_t chunk, seg, K; int32_t force; uint32_t gain, huff_min, pred; };

bool resolve(const nz_opts* in, Opts& o) {
    o.chunk = 262144u; o.seg = kSeg; o.K = 256u; o.force = -1; o.gain = 0; o.huff_min = 0; o.pred = 0;
    if (in) {
        if (in->chunk_elems) o.chunk = in->chunk_elems;
        if (in->seg_syms) o.seg = in->seg_syms;
        if (in->alphabet) o.K = in->alphabet;
        o.force = in->force_codec; o.gain = in->min_gain_permil; o.huff_min = in->huff_min_bytes;
        o.pred = in->predictor;
        if (in->reserved) return false;
    }
    if (o.pred > 1u) return false;
    if (o.chunk > kMaxChunk) return false;
    if (o.seg != kSeg) return false;                                   // the kernels decode 256-symbol segments
    if (o.K < 2u || o.K > kMaxK || (o.K & (o.K - 1u))) return false;
    if (o.force < -1 || o.force > 2) return false;
    if (o.gain > 1000u) return false;
    return true;
}

// step = fl32(eb * 63/32), inv_step = fl32(1/step); each operation rounded once to fp32.
bool step_constants(float eb, float& step, float& inv) {
    if (!(eb >= 0x1p-100f && eb <= 0x1p100f)) return false;
    volatile float s = eb * 1.96875f;
    volatile float r = 1.0f / s;
    step = s; inv = r;
    return true;
}

uint32_t bits_of(float f) { uint32_t u; __builtin_memcpy(&u, &f, 4); return u; }
uint64_t pad16h(uint64_t v) { return (v + 15u) & ~(uint64_t)15u; }
uint64_t pad4h(uint64_t v) { return (v + 3u) & ~(uint64_t)3u; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

uint64_t frame_bound(uint64_t nf, const Opts& o) {
    uint64_t pay = 4ull * nf;
    if (o.force == NZ_CODEC_HUFFMAN) {
        const uint64_t nseg = (nf + o.seg - 1) / o.seg;
        const uint64_t h = pad4h(o.K) + pad4h(2ull * nseg) + 4ull * ((nf * 60ull + 31u) / 32u);
        if (h > pay) pay = h;
    }
    return pad16h(kHdrBytes + pay);
}

// Optional per-kernel event trace (benchmark aid), per host thread.
thread_local void** t_events = nullptr;
thread_local size_t t_event_cap = 0, t_event_n = 0;

inline void trace_reset() { t_event_n = 0; }
inline void trace_mark(hipStream_t st) {
    if (t_events && t_event_n < t_event_cap) {
        (void)hipEventRecord(reinterpret_cast<hipEvent_t>(t_events[t_event_n]), st);
        t_event_n++;
    }
}

// Scratch of the entry point that allocates nothing: one array per GPU, resident until the process ends.
constexpr size_t kStaticScratchBytes = 8u << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};          // device address of `scratch` on each GPU, looked up on first use

// The array's name is a host-side handle, not a device address: ask the runtime for the address on the current
// device (every GPU holds its own copy at its own address) and use only that pointer from host code.
void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

constexpr uint64_t kMaxElems = 1ull << 38;      // keeps every grid below 2^31 workgroups for frames >= 8192 elements

bool geometry_ok(size_t n, const Opts& o) {
    if (n == 0 || n > kMaxElems) return false;
    const uint64_t nfr = (n + o.chunk - 1) / o.chunk;
    const uint64_t ebpf = (o.chunk + kEncBlock - 1) / kEncBlock;
    return nfr * ebpf < (1ull << 31) && nfr < (1ull << 31);
}

}  // namespace

extern "C" {

uint32_t nz_version(void) { return (1u << 16) | 1u; }

void nz_trace_events(void** events, size_t count) { t_events = events; t_event_cap = events ? count : 0; t_event_n = 0; }
size_t nz_trace_recorded(void) { return t_event_n; }

size_t nz_compress_bound(size_t n, const nz_opts* opts) {
    Opts o;
    if (!resolve(opts, o) || !geometry_ok(n, o)) return 0;
    const uint64_t nfr = (n + o.chunk - 1) / o.chunk;
    const uint64_t last = n - (nfr - 1) * o.chunk;
    return (size_t)(kStreamHdr + pad16h(8ull * nfr) + (nfr - 1) * frame_bound(o.chunk, o) + frame_bound(last, o));
}

size_t nz_workspace_bytes(size_t n, const nz_opts* opts) {
    Opts o;
    if (!resolve(opts, o) || !geometry_ok(n, o)) return 0;
    return ws_layout(n, o.chunk, kStatBlock, false).total;
}

size_t nz_reduce_workspace_bytes(size_t n, const nz_opts* opts) {
    Opts o;
    if (!resolve(opts, o) || !geometry_ok(n, o)) return 0;
    return ws_layout(n, o.chunk, kDecBlock, true).total;
}

// Bin width given directly (stochastic quantizer; receivers of its streams): same range as step_constants produces.
static bool step_given(float step, float& inv) {
    if (!(step >= 0x1p-100f && step <= 0x1p101f)) return false;
    volatile float r = 1.0f / step;
    inv = r;
    return true;
}

static nz_status compress_impl(const float* d_in, size_t n, float eb, float step, float inv, bool stochastic, uint32_t seed,
                               void* d_out, size_t out_cap, nz_result* d_res, const nz_opts* opts, void* d_ws,
                               size_t ws_bytes, void* stream) {
    Opts o;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!d_in || !d_out || !d_res || !d_ws || !resolve(opts, o) || !geometry_ok(n, o))
        return NZ_ERR_INVALID;
    if (!aligned16(d_in) || !aligned16(d_out) || !aligned16(d_ws) || !aligned16(d_res)) return NZ_ERR_INVALID;
    const WsLayout L = ws_layout(n, o.chunk, kStatBlock, false);
    if (ws_bytes < L.total) return NZ_ERR_INVALID;
    const uint32_t nfr = (uint32_t)((n + o.chunk - 1) / o.chunk);
    uint8_t* ws = reinterpret_cast<uint8_t*>(d_ws);
    if (out_cap < kStreamHdr + pad16h(8ull * nfr)) {        // not even the frame table fits: publish nothing
        if (launch_init(ws, 0, d_res, nfr, NZ_ERR_CAPACITY, st) != hipSuccess) return NZ_ERR_HIP;
        return NZ_ERR_CAPACITY;
    }
    CompressArgs A;
    A.in = d_in; A.n = n; A.chunk = o.chunk; A.n_frames = nfr; A.K = o.K;
    A.stat_block = kStatBlock; A.sbpf = (o.chunk + kStatBlock - 1) / kStatBlock;
    A.force_codec = o.force; A.min_gain_permil = o.gain; A.huff_min_bytes = o.huff_min;
    A.eb = eb; A.step = step; A.inv_step = inv; A.step_bits = bits_of(step); A.seed = seed; A.pred = o.pred;
    A.red_local = nullptr; A.red_sr = 0;
    A.out = reinterpret_cast<uint8_t*>(d_out); A.out_cap = out_cap; A.ws = ws; A.L = L; A.res = d_res;
    A.rea_ctx = nullptr; A.rea_tmp = nullptr; A.rea_gbits = nullptr; A.rea_fail = nullptr;
    if (stochastic && o.pred) return NZ_ERR_INVALID;              // (the stochastic quantizer is not built with the predictor)
    trace_reset(); trace_mark(st);
    if (launch_stats(A, stochastic, st) != hipSuccess) return NZ_ERR_HIP;     // also clears the control block and the result record
    trace_mark(st);
    if (launch_codebook(A, st) != hipSuccess) return NZ_ERR_HIP;
    trace_mark(st);
    if (launch_encode(A, false, stochastic, st) != hipSuccess) return NZ_ERR_HIP;
    trace_mark(st);
    return NZ_OK;
}

nz_status nz_compress(const float* d_in, size_t n, float eb, void* d_out, size_t out_cap, nz_result* d_res,
                      const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream) {
    float step, inv;
    if (!step_constants(eb, step, inv)) return NZ_ERR_INVALID;
    return compress_impl(d_in, n, eb, step, inv, false, 0u, d_out, out_cap, d_res, opts, d_ws, ws_bytes, stream);
}

nz_status nz_compress_sr(const float* d_in, size_t n, float step, uint32_t seed, void* d_out, size_t out_cap, nz_result* d_res,
                         const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream) {
    float inv;
    if (!step_given(step, inv)) return NZ_ERR_INVALID;
    return compress_impl(d_in, n, 0.0f, step, inv, true, seed, d_out, out_cap, d_res, opts, d_ws, ws_bytes, stream);
}

nz_status nz_qsgd_step(const float* d_in, size_t n, uint32_t levels, float* d_step, void* d_ws, size_t ws_bytes, void* stream) {
    if (!d_in || !d_step || !d_ws || n == 0 || levels == 0 || levels > (uint32_t)kQMax) return NZ_ERR_INVALID;
    if (!aligned16(d_in) || !aligned16(d_ws) || (reinterpret_cast<uintptr_t>(d_step) & 3u) || ws_bytes < 8192) return NZ_ERR_INVALID;
    if (launch_qsgd_step(d_in, n, levels, d_step, reinterpret_cast<double*>(d_ws), reinterpret_cast<hipStream_t>(stream)) != hipSuccess)
        return NZ_ERR_HIP;
    return NZ_OK;
}

size_t nz_static_scratch_bytes(void) { return kStaticScratchBytes; }

nz_status nz_compress_static(const float* d_in, size_t n, float eb, void* d_out, size_t out_cap, nz_result* d_res,
                             const nz_opts* opts, void* stream) {
    Opts o;
    if (!resolve(opts, o) || !geometry_ok(n, o)) return NZ_ERR_INVALID;
    if (ws_layout(n, o.chunk, kStatBlock, false).total > kStaticScratchBytes) return NZ_ERR_INVALID;   // message too large for the resident scratch
    void* ws = static_scratch();
    if (!ws) return NZ_ERR_HIP;
    return nz_compress(d_in, n, eb, d_out, out_cap, d_res, opts, ws, kStaticScratchBytes, stream);
}

size_t nz_context_bytes(void) { return sizeof(DevContext); }

nz_status nz_context_build(const float* d_sample, size_t n_sample, float eb, const nz_opts* opts, void* d_ctx, void* d_ws,
                           size_t ws_bytes, void* stream) {
    Opts o; float step, inv;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!d_sample || !d_ctx || !d_ws || n_sample == 0 || n_sample > kMaxChunk || !resolve(opts, o) || !step_constants(eb, step, inv))
        return NZ_ERR_INVALID;
    if (!aligned16(d_sample) || !aligned16(d_ctx) || !aligned16(d_ws) || ws_bytes < 4u * kMaxK) return NZ_ERR_INVALID;
    if (launch_context(d_sample, n_sample, eb, step, inv, o.K, reinterpret_cast<uint32_t*>(d_ws),
                       reinterpret_cast<DevContext*>(d_ctx), st) != hipSuccess) return NZ_ERR_HIP;
    return NZ_OK;
}

size_t nz_rea_workspace_bytes(size_t n, const nz_opts* opts) {
    Opts o;
    if (!resolve(opts, o) || !geometry_ok(n, o)) return 0;
    return rea_layout(n, o.chunk).total;
}

nz_status nz_compress_rea(const float* d_in, size_t n, float eb, const void* d_ctx, void* d_out, size_t out_cap,
                          nz_rea_result* d_res, const nz_opts* opts, const nz_rea_opts* ropts, void* d_ws, size_t ws_bytes,
                          void* stream) {
    Opts o; float step, inv;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!d_in || !d_out || !d_res || !d_ws || !resolve(opts, o) || !geometry_ok(n, o) || !step_constants(eb, step, inv))
        return NZ_ERR_INVALID;
    if (!aligned16(d_in) || !aligned16(d_out) || !aligned16(d_ws) || !aligned16(d_res) || !aligned16(d_ctx)) return NZ_ERR_INVALID;
    if (o.pred) return NZ_ERR_INVALID;                            // the sampled path codes the codes themselves
    const ReaLayout L = rea_layout(n, o.chunk);
    if (ws_bytes < L.total) return NZ_ERR_INVALID;
    const uint32_t nfr = (uint32_t)((n + o.chunk - 1) / o.chunk);
    const uint64_t slot = pad16h(kHdrBytes + 4ull * o.chunk);
    const uint64_t last = n - (uint64_t)(nfr - 1) * o.chunk;
    const uint64_t need = kStreamHdr + pad16h(8ull * nfr) + (uint64_t)(nfr - 1) * slot + pad16h(kHdrBytes + 4ull * last);
    if (out_cap < need) {                                          // every frame needs its RAW-sized slot: publish nothing
        if (launch_rea_status(d_res, nfr, NZ_ERR_CAPACITY, st) != hipSuccess) return NZ_ERR_HIP;
        return NZ_ERR_CAPACITY;
    }
    ReaArgs A;
    A.in = d_in; A.n = n; A.chunk = o.chunk; A.n_frames = nfr; A.K = o.K;
    A.gpf = (o.chunk + kEncGroup - 1) / kEncGroup;
    A.force_codec = o.force; A.min_gain_permil = o.gain; A.huff_min_bytes = o.huff_min;
    uint32_t sample_bytes = 65536u, small = 0u;
    A.link_ps = 0; A.fixed_alpha_ns = 0; A.fixed_ps = 0; A.huff_alpha_ns = 0; A.huff_ps = 0;
    if (ropts) {
        if (ropts->reserved) return NZ_ERR_INVALID;
        if (ropts->sample_bytes) sample_bytes = ropts->sample_bytes;
        small = ropts->small_batch_bytes;
        A.link_ps = ropts->link_ps_per_byte;
        A.fixed_alpha_ns = ropts->fixed_alpha_ns; A.fixed_ps = ropts->fixed_ps_per_byte;
        A.huff_alpha_ns = ropts->huff_alpha_ns; A.huff_ps = ropts->huff_ps_per_byte;
    }
    A.sample_elems = sample_bytes / 4u; A.small_batch_bytes = small;
    A.eb = eb; A.step = step; A.inv_step = inv; A.step_bits = bits_of(step);
    A.ctx = reinterpret_cast<const DevContext*>(d_ctx);
    A.out = reinterpret_cast<uint8_t*>(d_out); A.slot = slot;
    A.ws = reinterpret_cast<uint8_t*>(d_ws); A.L = L; A.res = d_res;
    A.tmp_base = reinterpret_cast<uint32_t*>(A.ws + L.tmp);
    trace_reset(); trace_mark(st);
    if (launch_rea(A, st, trace_mark) != hipSuccess) return NZ_ERR_HIP;
    return NZ_OK;
}

static nz_status decompress_impl(const void* d_stream, size_t stream_bytes, float* d_out, size_t n, float step,
                                 nz_result* d_res, const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream) {
    Opts o;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!d_stream || !d_out || !d_res || !d_ws || !resolve(opts, o) || !geometry_ok(n, o))
        return NZ_ERR_INVALID;
    if (!aligned16(d_stream) || !aligned16(d_out) || !aligned16(d_res) || !aligned16(d_ws)) return NZ_ERR_INVALID;
    const WsLayout L = ws_layout(n, o.chunk, kStatBlock, false);     // one verdict word per decode workgroup
    if (ws_bytes < L.total) return NZ_ERR_INVALID;
    const uint32_t nfr = (uint32_t)((n + o.chunk - 1) / o.chunk);
    DecodeArgs A;
    A.a = reinterpret_cast<const uint8_t*>(d_stream); A.a_bytes = stream_bytes; A.b = nullptr; A.b_bytes = 0;
    A.out = d_out; A.local = nullptr; A.eb = 0.0f; A.inv_step = 0.0f; A.sr = 0; A.seed = 0; A.set_in = 0; A.n = n; A.chunk = o.chunk; A.n_frames = nfr; A.K = o.K;
    A.dbpf = (o.chunk + kDecBlock - 1) / kDecBlock; A.pred = o.pred;
    A.step = step; A.step_bits = bits_of(step); A.ws = reinterpret_cast<uint8_t*>(d_ws); A.L = L; A.res = d_res;
    static_assert(kDecBlock == kStatBlock, "the verdict words reuse the per-statistics-block slots of the workspace");
    trace_reset(); trace_mark(st);
    if (launch_decode(A, 0, st) != hipSuccess) return NZ_ERR_HIP;
    trace_mark(st);
    if (launch_decode_finish(A, st) != hipSuccess) return NZ_ERR_HIP;   // result record; rejected frames zero-filled
    trace_mark(st);
    return NZ_OK;
}

nz_status nz_decompress(const void* d_stream, size_t stream_bytes, float* d_out, size_t n, float eb,
                        nz_result* d_res, const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream) {
    float step, inv;
    if (!step_constants(eb, step, inv)) return NZ_ERR_INVALID;
    return decompress_impl(d_stream, stream_bytes, d_out, n, step, d_res, opts, d_ws, ws_bytes, stream);
}

nz_status nz_decompress_step(const void* d_stream, size_t stream_bytes, float* d_out, size_t n, float step,
                             nz_result* d_res, const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream) {
    float inv;
    if (!step_given(step, inv)) return NZ_ERR_INVALID;
    return decompress_impl(d_stream, stream_bytes, d_out, n, step, d_res, opts, d_ws, ws_bytes, stream);
}

// The two reduce entry points differ only in the second operand: a stream (d_b) or the rank's own fp32 data (d_local).
constexpr uint32_t kMaxOperands = 64;         // operand streams of one k-ary reduce

// The reduce entry points: k operand streams (k >= 2), or one incoming stream and the rank's own fp32 message.
// k > 2: the running value lives in one of two staging sets of the workspace; every operand between the first and
// the last is added by an accumulating pass that reads one set and writes the other (the set of the first pass is
// chosen so that the last accumulating pass leaves the running value where the statistics pass expects operand A).
static nz_status reduce_impl(const void* const* d_ops, const size_t* op_bytes, uint32_t k, const float* d_local,
                             void* d_out, size_t out_cap, size_t n, float eb, float step, float inv, nz_result* d_res,
                             const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream, bool stochastic = false,
                             uint32_t seed = 0) {
    Opts o;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!d_ops || !op_bytes || k < 1 || k > kMaxOperands || (!d_local && k < 2) || (d_local && k != 1)) return NZ_ERR_INVALID;
    for (uint32_t p = 0; p < k; p++) if (!d_ops[p] || !aligned16(d_ops[p])) return NZ_ERR_INVALID;
    if (!d_out || !d_res || !d_ws || !resolve(opts, o) || !geometry_ok(n, o))
        return NZ_ERR_INVALID;
    if (stochastic && o.pred) return NZ_ERR_INVALID;               // (the stochastic quantizer is not built with the predictor)
    if ((d_local && !aligned16(d_local)) || !aligned16(d_out) || !aligned16(d_ws) || !aligned16(d_res))
        return NZ_ERR_INVALID;
    const WsLayout L = ws_layout(n, o.chunk, kDecBlock, true);
    if (ws_bytes < L.total) return NZ_ERR_INVALID;
    const uint32_t nfr = (uint32_t)((n + o.chunk - 1) / o.chunk);
    uint8_t* ws = reinterpret_cast<uint8_t*>(d_ws);
    if (out_cap < kStreamHdr + pad16h(8ull * nfr)) {
        if (launch_init(ws, 0, d_res, nfr, NZ_ERR_CAPACITY, st) != hipSuccess) return NZ_ERR_HIP;
        return NZ_ERR_CAPACITY;
    }
    DecodeArgs D;
    D.a = reinterpret_cast<const uint8_t*>(d_ops[0]); D.a_bytes = op_bytes[0];
    D.b = k > 1 ? reinterpret_cast<const uint8_t*>(d_ops[1]) : nullptr; D.b_bytes = k > 1 ? op_bytes[1] : 0;
    D.out = nullptr; D.local = d_local; D.eb = eb; D.inv_step = inv; D.sr = stochastic ? 1u : 0u; D.seed = seed;
    D.set_in = 0;
    D.n = n; D.chunk = o.chunk; D.n_frames = nfr; D.K = o.K;
    D.dbpf = (o.chunk + kDecBlock - 1) / kDecBlock; D.pred = o.pred;
    D.step = step; D.step_bits = bits_of(step); D.ws = ws; D.L = L; D.res = d_res;
    CompressArgs A;
    A.in = nullptr; A.n = n; A.chunk = o.chunk; A.n_frames = nfr; A.K = o.K;
    A.stat_block = kDecBlock; A.sbpf = D.dbpf;
    A.force_codec = o.force; A.min_gain_permil = o.gain; A.huff_min_bytes = o.huff_min;
    A.eb = eb; A.step = step; A.inv_step = inv; A.step_bits = bits_of(step); A.seed = seed; A.pred = o.pred;
    A.red_local = d_local; A.red_sr = stochastic ? 1u : 0u;
    A.out = reinterpret_cast<uint8_t*>(d_out); A.out_cap = out_cap; A.ws = ws; A.L = L; A.res = d_res;
    A.rea_ctx = nullptr; A.rea_tmp = nullptr; A.rea_gbits = nullptr; A.rea_fail = nullptr;
    trace_reset(); trace_mark(st);
    if (launch_init(ws + L.ctrl, L.zero_end - L.ctrl, d_res, nfr, NZ_OK, st) != hipSuccess) return NZ_ERR_HIP;
    trace_mark(st);
    if (d_local) {
        if (launch_decode(D, stochastic ? 4 : 3, st) != hipSuccess) return NZ_ERR_HIP;   // decode incoming + quantize local + add
        trace_mark(st);
    } else {
        D.set_in = (k - 2u) & 1u;                                           // where the first pass stages operand 0
        if (launch_decode(D, 1, st) != hipSuccess) return NZ_ERR_HIP;       // stage operand 0
        trace_mark(st);
        for (uint32_t p = 1; p + 1 < k; p++) {                              // operands 1 .. k-2: running value += operand
            D.b = reinterpret_cast<const uint8_t*>(d_ops[p]); D.b_bytes = op_bytes[p];
            if (launch_decode(D, 6, st) != hipSuccess) return NZ_ERR_HIP;
            if (launch_fix_acc(D, st) != hipSuccess) return NZ_ERR_HIP;     // frames whose partial sums left the range
            trace_mark(st);
            D.set_in ^= 1u;
        }
        D.b = reinterpret_cast<const uint8_t*>(d_ops[k - 1]); D.b_bytes = op_bytes[k - 1];
        if (launch_decode(D, 2, st) != hipSuccess) return NZ_ERR_HIP;       // decode the last operand + add + statistics
        trace_mark(st);
    }
    if (launch_fix(D, st) != hipSuccess) return NZ_ERR_HIP;                 // frames that turn RAW late (local data, sums past 2^30)
    trace_mark(st);
    // with the delta predictor the encoder codes differences of the sums: their statistics come from a pass over the
    // staged sums (the adding pass counted the sums themselves)
    if (o.pred && launch_stats_codes(A, st) != hipSuccess) return NZ_ERR_HIP;
    if (launch_codebook(A, st) != hipSuccess) return NZ_ERR_HIP;
    trace_mark(st);
    if (launch_encode(A, true, false, st) != hipSuccess) return NZ_ERR_HIP;
    trace_mark(st);
    return NZ_OK;
}

nz_status nz_reduce_frames(const void* d_a, size_t a_bytes, const void* d_b, size_t b_bytes, void* d_out,
                           size_t out_cap, size_t n, float eb, nz_result* d_res, const nz_opts* opts,
                           void* d_ws, size_t ws_bytes, void* stream) {
    float step, inv;
    if (!step_constants(eb, step, inv)) return NZ_ERR_INVALID;
    const void* ops[2] = { d_a, d_b }; const size_t lens[2] = { a_bytes, b_bytes };
    return reduce_impl(ops, lens, 2, nullptr, d_out, out_cap, n, eb, step, inv, d_res, opts, d_ws, ws_bytes, stream);
}

nz_status nz_reduce_frames_step(const void* d_a, size_t a_bytes, const void* d_b, size_t b_bytes, void* d_out,
                                size_t out_cap, size_t n, float step, nz_result* d_res, const nz_opts* opts,
                                void* d_ws, size_t ws_bytes, void* stream) {
    float inv;
    if (!step_given(step, inv)) return NZ_ERR_INVALID;
    const void* ops[2] = { d_a, d_b }; const size_t lens[2] = { a_bytes, b_bytes };
    return reduce_impl(ops, lens, 2, nullptr, d_out, out_cap, n, 0.0f, step, inv, d_res, opts, d_ws, ws_bytes, stream);
}

nz_status nz_reduce_k(const void* const* d_streams, const size_t* stream_bytes, uint32_t k, void* d_out, size_t out_cap,
                      size_t n, float eb, nz_result* d_res, const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream) {
    float step, inv;
    if (k < 2 || !step_constants(eb, step, inv)) return NZ_ERR_INVALID;
    return reduce_impl(d_streams, stream_bytes, k, nullptr, d_out, out_cap, n, eb, step, inv, d_res, opts, d_ws, ws_bytes, stream);
}

nz_status nz_reduce_k_step(const void* const* d_streams, const size_t* stream_bytes, uint32_t k, void* d_out, size_t out_cap,
                           size_t n, float step, nz_result* d_res, const nz_opts* opts, void* d_ws, size_t ws_bytes, void* stream) {
    float inv;
    if (k < 2 || !step_given(step, inv)) return NZ_ERR_INVALID;
    return reduce_impl(d_streams, stream_bytes, k, nullptr, d_out, out_cap, n, 0.0f, step, inv, d_res, opts, d_ws, ws_bytes, stream);
}

nz_status nz_reduce_local(const void* d_in, size_t in_bytes, const float* d_local, void* d_out, size_t out_cap,
                          size_t n, float eb, nz_result* d_res, const nz_opts* opts, void* d_ws, size_t ws_bytes,
                          void* stream) {
    float step, inv;
    if (!d_local || !step_constants(eb, step, inv)) return NZ_ERR_INVALID;
    return reduce_impl(&d_in, &in_bytes, 1, d_local, d_out, out_cap, n, eb, step, inv, d_res, opts, d_ws, ws_bytes, stream);
}

// Workspace of the sampled ring step: the adding pass's workspace, a result record of its own for that pass, and
// the sampled path's part (plans are kept in the first, realized sizes, flags and group scratch in the last).
struct RedReaLayout { WsLayout R; size_t add_res; size_t rea; ReaLayout E; size_t total; };
static RedReaLayout red_rea_layout(size_t n, uint32_t chunk) {
    RedReaLayout L;
    L.R = ws_layout(n, chunk, kDecBlock, true);
    L.add_res = (L.R.total + 255u) & ~(size_t)255u;
    L.rea = L.add_res + 256u;
    L.E = rea_layout(n, chunk);
    L.total = L.rea + L.E.total;
    return L;
}

size_t nz_reduce_rea_workspace_bytes(size_t n, const nz_opts* opts) {
    Opts o;
    if (!resolve(opts, o) || !geometry_ok(n, o)) return 0;
    return red_rea_layout(n, o.chunk).total;
}

nz_status nz_reduce_local_rea(const void* d_in, size_t in_bytes, const float* d_local, size_t n, float eb, const void* d_ctx,
                              void* d_out, size_t out_cap, nz_rea_result* d_res, const nz_opts* opts, const nz_rea_opts* ropts,
                              void* d_ws, size_t ws_bytes, void* stream) {
    Opts o; float step, inv;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (!d_in || !d_local || !d_out || !d_res || !d_ws || !resolve(opts, o) || !geometry_ok(n, o) || !step_constants(eb, step, inv))
        return NZ_ERR_INVALID;
    if (!aligned16(d_in) || !aligned16(d_local) || !aligned16(d_out) || !aligned16(d_ws) || !aligned16(d_res) ||
        (d_ctx && !aligned16(d_ctx))) return NZ_ERR_INVALID;
    if (o.pred) return NZ_ERR_INVALID;                            // the sampled path codes the codes themselves
    if (ropts && ropts->reserved) return NZ_ERR_INVALID;
    const RedReaLayout L = red_rea_layout(n, o.chunk);
    if (ws_bytes < L.total) return NZ_ERR_INVALID;
    const uint32_t nfr = (uint32_t)((n + o.chunk - 1) / o.chunk);
    const uint64_t slot = pad16h(kHdrBytes + 4ull * o.chunk);
    const uint64_t last = n - (uint64_t)(nfr - 1) * o.chunk;
    const uint64_t need = kStreamHdr + pad16h(8ull * nfr) + (uint64_t)(nfr - 1) * slot + pad16h(kHdrBytes + 4ull * last);
    if (out_cap < need) {                                          // every frame needs its RAW-sized slot: publish nothing
        if (launch_rea_status(d_res, nfr, NZ_ERR_CAPACITY, st) != hipSuccess) return NZ_ERR_HIP;
        return NZ_ERR_CAPACITY;
    }
    uint8_t* ws = reinterpret_cast<uint8_t*>(d_ws);
    DecodeArgs D;
    D.a = reinterpret_cast<const uint8_t*>(d_in); D.a_bytes = in_bytes; D.b = nullptr; D.b_bytes = 0;
    D.out = nullptr; D.local = d_local; D.eb = eb; D.inv_step = inv; D.sr = 0; D.seed = 0; D.set_in = 0;
    D.n = n; D.chunk = o.chunk; D.n_frames = nfr; D.K = o.K;
    D.dbpf = (o.chunk + kDecBlock - 1) / kDecBlock; D.pred = 0;
    D.step = step; D.step_bits = bits_of(step); D.ws = ws; D.L = L.R; D.res = ws + L.add_res;
    ReaArgs A;
    A.in = nullptr; A.n = n; A.chunk = o.chunk; A.n_frames = nfr; A.K = o.K;
    A.gpf = (o.chunk + kEncGroup - 1) / kEncGroup;
    A.force_codec = o.force; A.min_gain_permil = o.gain; A.huff_min_bytes = o.huff_min;
    uint32_t sample_bytes = 65536u, small = 0u;
    A.link_ps = 0; A.fixed_alpha_ns = 0; A.fixed_ps = 0; A.huff_alpha_ns = 0; A.huff_ps = 0;
    if (ropts) {
        if (ropts->sample_bytes) sample_bytes = ropts->sample_bytes;
        small = ropts->small_batch_bytes;
        A.link_ps = ropts->link_ps_per_byte;
        A.fixed_alpha_ns = ropts->fixed_alpha_ns; A.fixed_ps = ropts->fixed_ps_per_byte;
        A.huff_alpha_ns = ropts->huff_alpha_ns; A.huff_ps = ropts->huff_ps_per_byte;
    }
    A.sample_elems = sample_bytes / 4u; A.small_batch_bytes = small;
    A.eb = eb; A.step = step; A.inv_step = inv; A.step_bits = bits_of(step);
    A.ctx = reinterpret_cast<const DevContext*>(d_ctx);
    A.out = reinterpret_cast<uint8_t*>(d_out); A.slot = slot;
    A.ws = ws + L.rea; A.L = L.E; A.res = d_res;
    A.tmp_base = reinterpret_cast<uint32_t*>(A.ws + L.E.tmp);
    A.red_ws = ws; A.RL = L.R; A.local = d_local; A.add_res = ws + L.add_res;
    trace_reset(); trace_mark(st);
    if (launch_init(ws + L.R.ctrl, L.R.zero_end - L.R.ctrl, ws + L.add_res, nfr, NZ_OK, st) != hipSuccess) return NZ_ERR_HIP;
    trace_mark(st);
    if (launch_decode(D, 5, st) != hipSuccess) return NZ_ERR_HIP;        // decode incoming + quantize local + add (no statistics)
    trace_mark(st);
    if (launch_fix(D, st) != hipSuccess) return NZ_ERR_HIP;              // frames without integer sums: fp32 sums
    trace_mark(st);
    if (launch_rea(A, st, trace_mark) != hipSuccess) return NZ_ERR_HIP;  // plan + encode, then accept / pack / header
    return NZ_OK;
}

nz_status nz_reduce_local_sr(const void* d_in, size_t in_bytes, const float* d_local, void* d_out, size_t out_cap,
                             size_t n, float step, uint32_t seed, nz_result* d_res, const nz_opts* opts, void* d_ws,
                             size_t ws_bytes, void* stream) {
    float inv;
    if (!d_local || !step_given(step, inv)) return NZ_ERR_INVALID;
    return reduce_impl(&d_in, &in_bytes, 1, d_local, d_out, out_cap, n, 0.0f, step, inv, d_res, opts, d_ws, ws_bytes, stream,
                       true, seed);
}

}  // extern "C"
