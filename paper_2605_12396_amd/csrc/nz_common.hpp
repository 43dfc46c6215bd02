// nz_common.hpp -- constants, workspace layout and wave/LDS helpers shared by the gfx950 kernels.
// (Device-side only; the CPU oracle has its own, separate definitions.)
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nz {

// ---- stream format v1 constants (the paper leaves header layout open, Sec. IV-D "Batch Framing") ----
constexpr uint32_t kHdrBytes      = 32;          // frame header: 8 little-endian u32
constexpr uint32_t kStreamHdr     = 64;          // stream header bytes
constexpr uint32_t kMagicFrame    = 0x31465A4Eu; // 'N','Z','F','1'
constexpr uint32_t kMagicStream   = 0x31535A4Eu; // 'N','Z','S','1'
constexpr uint32_t kCheckXor      = 0x5A5A5A5Au;
constexpr uint32_t kCanonNaN      = 0x7FC00000u;
constexpr int      kQMax          = 32767;       // largest quantization code magnitude
constexpr int      kQSumMax       = 1 << 30;     // largest magnitude a reduced code may take
constexpr uint32_t kMaxChunk      = 1u << 20;
constexpr uint32_t kMaxK          = 1024;
constexpr uint32_t kSeg           = 256;         // symbols per Huffman segment (one wave pass of 4 symbols/lane)
constexpr uint32_t kMaxLen        = 28;          // deepest optimal code for <= 2^20 symbols (Fibonacci bound)

enum : uint32_t { ST_OK = 0, ST_INVALID = 1, ST_CAPACITY = 2, ST_CORRUPT = 3, ST_MISMATCH = 4 };
enum : uint32_t { CODEC_RAW = 0, CODEC_FIXED = 1, CODEC_HUFF = 2 };

// ---- launch geometry ----
constexpr uint32_t kStatThreads   = 512;
constexpr uint32_t kStatBlock     = 65536;       // symbols per statistics workgroup (compress)
constexpr uint32_t kEncThreads    = 256;
constexpr uint32_t kEncBlock      = 4096;        // symbols per encode sub-block = 16 segments
constexpr uint32_t kEncIters      = kEncBlock / (kEncThreads * 4);   // passes of 1024 symbols
constexpr uint32_t kEncSegs       = kEncBlock / kSeg;                // segments per encode sub-block
constexpr uint32_t kEncGroup      = 65536;       // symbols per encode workgroup: a whole number of statistics blocks
constexpr uint32_t kDecThreads    = 256;
constexpr uint32_t kDecBlock      = kDecThreads * kSeg;              // 65536 symbols per decode workgroup
constexpr uint32_t kBookThreads   = 1024;

// ---- per-frame record written by the codebook/selector kernel, read by the encoder ----
struct FrameMeta {
    uint64_t offset;      // byte offset of the frame in the stream
    uint32_t total;       // padded frame bytes
    uint32_t payload;     // payload bytes
    uint32_t codec;
    uint32_t w;           // FIXEDLEN width
    uint32_t nsym;        // HUFFMAN: 1 + largest used symbol
    uint32_t fits;        // 1 when offset+total <= out_cap (the encoder writes nothing otherwise)
    uint32_t segt_off;    // byte offset of the segment table inside the frame
    uint32_t bits_off;    // byte offset of the bitstream inside the frame
    uint32_t bits_words;  // bitstream length in 32-bit words
    uint32_t pad_;        // reduce: 1 = the frame has no integer sums (its fp32 sums are staged); else 0
    uint64_t huff_bits;
    uint64_t pad2_;
};
static_assert(sizeof(FrameMeta) == 64, "FrameMeta is 64 bytes");

// ---- control block at the start of the workspace (zeroed at the start of every call) ----
struct Ctrl {
    uint32_t ticket_book;   // frame ids handed to codebook workgroups in start order: the frame look-back only waits on smaller ones
    uint32_t pad[15];
};
static_assert(sizeof(Ctrl) == 64, "Ctrl is 64 bytes");

// Workspace carve-up; computed identically on host for sizing and launch.
struct WsLayout {
    size_t ctrl, frame_desc, zero_end;      // [ctrl, zero_end) is cleared per call
    size_t meta, book_code, book_len, phist, pmeta, grp_start, codes, c16, cwide, a16, a32, akind, awide, akind1, awide1, total;
};

__host__ __device__ inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

__host__ inline WsLayout ws_layout(size_t n, uint32_t chunk, uint32_t stat_block, bool with_codes) {
    WsLayout L;
    const size_t n_frames = (n + chunk - 1) / chunk;
    const size_t sbpf = (chunk + stat_block - 1) / stat_block;      // statistics blocks per frame
    size_t o = 0;
    L.ctrl = o;        o += sizeof(Ctrl);
    L.frame_desc = o;  o += align_up(8 * n_frames, 256);
    L.zero_end = o;
    L.meta = o;        o += align_up(sizeof(FrameMeta) * n_frames, 256);
    L.book_code = o;   o += align_up(4 * (size_t)kMaxK * n_frames, 256);
    L.book_len = o;    o += align_up((size_t)kMaxK * n_frames, 256);
    L.phist = o;       o += align_up(4 * (size_t)kMaxK * n_frames * sbpf, 256);
    L.pmeta = o;       o += align_up(8 * n_frames * sbpf, 256);
    L.grp_start = o;   o += align_up(4 * n_frames * sbpf, 256);
    L.codes = o;       if (with_codes) o += align_up(4 * n, 256);      // reduce: sums that need 32 bits, fp32 sums of RAW frames
    L.c16 = o;         if (with_codes) o += align_up(2 * n, 256);      // reduce: the sums as 16-bit codes
    L.cwide = o;       if (with_codes) o += align_up(4 * n_frames * sbpf, 256);
    L.a16 = o;         if (with_codes) o += align_up(2 * n, 256);      // reduce: operand A, 16-bit codes
    L.a32 = o;         if (with_codes) o += align_up(4 * n, 256);      // reduce: operand A, wide codes and RAW words
    L.akind = o;       if (with_codes) o += align_up(4 * n_frames, 256);
    L.awide = o;       if (with_codes) o += align_up(4 * n_frames * sbpf, 256);
    L.akind1 = o;      if (with_codes) o += align_up(4 * n_frames, 256);           // k-ary reduce: flags of the second staging set
    L.awide1 = o;      if (with_codes) o += align_up(4 * n_frames * sbpf, 256);
    L.total = o;
    return L;
}

// ---- agent-scope relaxed atomics: the only inter-workgroup traffic inside a kernel ----
__device__ inline uint64_t ld_agent(const uint64_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_agent(uint64_t* p, uint64_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline uint32_t ld_agent(const uint32_t* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_agent(uint32_t* p, uint32_t v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// ---- wave64 helpers ----
__device__ inline uint32_t lane_id() { return __lane_id(); }

// Inclusive wave scan on the DPP network (no LDS traffic): Kogge-Stone inside each row of 16 lanes, then the
// last lane of row 0 / 2 is added to row 1 / 3 and the last lane of the lower half to the upper half.
__device__ inline uint32_t wave_incl_scan_dpp(uint32_t v) {
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xF, 0xF, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xF, 0xF, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xF, 0xF, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xF, 0xF, true);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xA, 0xF, false);  // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xC, 0xF, false);  // row_bcast:31 into rows 2 and 3
    return v;
}
__device__ inline uint64_t wave_sum64(uint64_t v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}
__device__ inline uint32_t wave_max(uint32_t v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) { uint32_t t = __shfl_xor(v, d, 64); v = t > v ? t : v; }
    return v;
}

__device__ inline uint32_t zigzag(int32_t q) { return ((uint32_t)q << 1) ^ (uint32_t)(q >> 31); }
__device__ inline int32_t unzigzag(uint32_t z) { return (int32_t)(z >> 1) ^ -(int32_t)(z & 1u); }
// Symbol of a zigzag code: z + 1 for z <= K-2, else the escape symbol 0.  Histogram bin while counting: min(z, K-1),
// one instruction; bin b < K-1 counts symbol b + 1 and bin K-1 counts the escape symbol (bin_symbol maps back when
// the counts are written out).  The encoder's codebook is indexed the same way.
__device__ inline uint32_t bin_of(uint32_t z, uint32_t K) { return z < K - 1u ? z : K - 1u; }
__device__ inline uint32_t bin_symbol(uint32_t b, uint32_t K) { return b == K - 1u ? 0u : b + 1u; }

// Quantize one value (interface quantizer, Sec. IV-B): u = fl(x*inv_step), q = rne(u), accepted when
// |u| <= 32767 and fl(|x - fl(q*step)|) <= eb.  Every product is rounded on its own.
// The second test is implied by the first and is not evaluated here: with step = fl(eb*63/32), inv_step = fl(1/step)
// and |u| <= 32767 the roundings of inv_step, u and q*step move x - xhat by at most 32767*(2^-23 + 2^-24) bins beyond
// the half bin of the rounding to q, so |x - xhat| <= 0.50586*step < 0.50794*step <= eb, also after the fp32 rounding
// of the difference; NaN and Inf fail the first test.  (A CPU test holds the reference quantizer, which evaluates both
// tests, to this on rounding boundaries, range ends, denormals and random values over the whole range of eb.)
// (r = rne(u) is an integer-valued float, so float(q) = r whenever |u| <= 32767.)
__device__ inline bool quantize_ok(float x, float eb, float step, float inv_step, float& r) {
#pragma clang fp contract(off)
    (void)eb; (void)step;
    const float u = x * inv_step;
    r = __builtin_rintf(u);                    // ties to even
    return fabsf(u) <= 32767.0f;               // false for NaN
}
__device__ inline bool quantize1(float x, float eb, float step, float inv_step, int32_t& q) {
    float r;
    const bool ok = quantize_ok(x, eb, step, inv_step, r);
    q = ok ? (int32_t)r : 0;
    return ok;
}
// ---- stochastic interface quantizer (QSGD, Sec. II-B "Quantization", Sec. IV-B) ----
// Counter-based draw of message element i under a seed: the 32-bit finalizer of MurmurHash3, keyed by the seed and
// the high half of the index; the top 24 bits are the draw (so every pass over the data sees the same bits).
__device__ inline uint32_t fmix32(uint32_t h) {
    h ^= h >> 16; h *= 0x85EBCA6Bu;
    h ^= h >> 13; h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}
__device__ inline uint32_t sr_key(uint32_t seed, uint64_t i) { return fmix32(seed + 0x9E3779B9u * (uint32_t)(i >> 32)); }
__device__ inline uint32_t sr_draw(uint32_t key, uint32_t i_lo) { return fmix32(i_lo ^ key) >> 8; }
// Draws for the elements base + off, off < 2^32, of a piece of work: the key changes where the low half of the index
// wraps, so two keys cover the piece.
struct SrKeys {
    uint32_t base_lo, key0, key1;
    __device__ inline void init(uint32_t seed, uint64_t base) {
        base_lo = (uint32_t)base; key0 = sr_key(seed, base); key1 = sr_key(seed, base + (1ull << 32));
    }
    __device__ inline uint32_t draw(uint32_t off) const {
        const uint32_t lo = base_lo + off;
        return sr_draw(lo < base_lo ? key1 : key0, lo);
    }
};
// a = fl(|x|*inv_step), l = floor(a), level l + 1 with probability a - l (draw * 2^-24 < a - l), sign of x;
// accepted when a <= 32767 and fl(|x - fl(q*step)|) <= fl(step * (1 + 2^-6)).
__device__ inline bool sr_quantize1(float x, float step, float inv_step, uint32_t draw24, int32_t& q) {
#pragma clang fp contract(off)
    const float a = fabsf(x) * inv_step;
    const bool ok1 = a <= 32767.0f;                       // false for NaN
    const float l = __builtin_floorf(a);
    const float f = a - l;
    const float u = (float)draw24 * 0x1p-24f;
    float m = l + ((u < f) ? 1.0f : 0.0f);                // exact: integers below 2^24
    m = (x < 0.0f) ? -m : m;
    const float xh = m * step;
    const float d = x - xh;
    const float lim = step * 1.015625f;
    const bool ok = ok1 && (fabsf(d) <= lim);
    q = ok ? (int32_t)m : 0;
    return ok;
}

__device__ inline float dequantize1(int32_t q, float step) {
#pragma clang fp contract(off)
    return (float)q * step;
}

// ---- sampled arbitration (REA): cached Huffman context and per-call arguments ----
// Device-resident context record: one canonical code over the K symbols, every symbol coded (Sec. IV-C "cached codebook").
struct DevContext {
    uint32_t valid, K, pad_[2];
    uint8_t  len[kMaxK];        // by symbol (0 = escape): code length, 1..28
    uint64_t book[kMaxK];       // by min(z, K-1): bit-reversed code | length << 32 (entry K-1 = escape)
};
// A group of kEncGroup symbols never needs more bitstream words than this (28-bit code + 32 escaped bits per symbol).
constexpr uint32_t kReaTmpWords = kEncGroup * 60u / 32u;

struct ReaLayout { size_t fail, meta, gbits, tmp, total; };
__host__ inline ReaLayout rea_layout(size_t n, uint32_t chunk) {
    ReaLayout L;
    const size_t n_frames = (n + chunk - 1) / chunk;
    const size_t gpf = (chunk + kEncGroup - 1) / kEncGroup;
    size_t o = 0;
    L.fail = o;  o += align_up(4 * n_frames * gpf, 256);          // one failure flag per encoder group
    L.meta = o;  o += align_up(sizeof(FrameMeta) * n_frames, 256);
    L.gbits = o; o += align_up(4 * n_frames * gpf, 256);
    L.tmp = o;   o += gpf > 1 ? align_up(4 * (size_t)kReaTmpWords * n_frames * gpf, 256) : 0;   // (a one-group frame is coded in place)
    L.total = o;
    return L;
}

struct ReaResultRec { uint64_t span_bytes, wire_bytes; uint32_t status, n_frames, n_raw, n_fixed, n_huff, n_fallback; };

struct ReaArgs {
    const float* in; uint64_t n;
    uint32_t chunk, n_frames, K, gpf;           // encoder workgroups (groups of kEncGroup symbols) per frame
    int32_t force_codec; uint32_t min_gain_permil, huff_min_bytes;
    uint32_t sample_elems, small_batch_bytes;
    uint32_t link_ps, fixed_alpha_ns, fixed_ps, huff_alpha_ns, huff_ps;   // cost model of Eq. 1 (link_ps 0: size only)
    float eb, step, inv_step; uint32_t step_bits;
    const DevContext* ctx;
    uint8_t* out; uint64_t slot;               // bytes between frame starts
    uint8_t* ws; ReaLayout L;                  // the sampled path's part of the workspace (ws + L.*)
    uint32_t* tmp_base;                        // scratch regions of kReaTmpWords words per (frame, group)
    void* res;                                 // nz_rea_result* (device)
    // ring step only (in == nullptr): the adding pass's workspace with the staged sums, the rank's own data, and
    // the adding pass's own result record (its status is carried over)
    uint8_t* red_ws; WsLayout RL; const float* local; const void* add_res;
};

// Launchers (one per translation unit).
hipError_t launch_context(const float* sample, uint64_t n, float eb, float step, float inv_step, uint32_t K, uint32_t* ghist,
                          DevContext* ctx, hipStream_t st);
hipError_t launch_rea(const ReaArgs& A, hipStream_t st, void (*mark)(hipStream_t));   // A.in: compress; else the ring step's encode + finish
hipError_t launch_rea_status(void* res, uint32_t n_frames, uint32_t status, hipStream_t st);
// ---- staging of the reduce (workspace) ----
constexpr uint32_t kTile16R = 32;                    // symbols a decoding thread produces between two output phases
constexpr int32_t kWideMarker = -32768;              // "this code does not fit 16 bits"
constexpr uint32_t kHalf = 65536;                    // statistics granularity of the reduce (one encoder group)

// Staging of operand A between the two reduce passes (workspace): a16 holds one 16-bit code per element,
// kWideMarker where the code needs 32 bits, which then sits in a32; a RAW frame keeps its fp32 words in a32.
// a32 is indexed by the element's position in the message.  a16 is too, except that inside every full half
// (kHalf elements = 256 segments) the order is phase-major -- [phase of 32 symbols][segment][32] -- so that
// what a wave stores or loads in one phase (8 segments x 32 codes) is 512 contiguous bytes, not eight half lines.
struct StageA {
    int16_t* a16; uint32_t* a32;
    // position in a16 of frame element i (frame starts at message element f0 and has nf elements)
    __device__ static inline uint64_t at16(uint64_t f0, uint32_t nf, uint32_t i) {
        const uint32_t base = i & ~(kHalf - 1u), j = i & (kHalf - 1u);
        const bool full = base + kHalf <= nf;
        return f0 + base + (full ? ((j & (kSeg - 1u)) >> 5) * (kHalf / 8u) + (j >> 8) * kTile16R + (j & 31u) : j);
    }
    __device__ inline void put_code(uint64_t f0, uint32_t nf, uint32_t i, int32_t q, uint32_t& wide_seen) const {
        if (q > 32767 || q <= kWideMarker) { a16[at16(f0, nf, i)] = (int16_t)kWideMarker; a32[f0 + i] = (uint32_t)q; wide_seen = 1; }
        else a16[at16(f0, nf, i)] = (int16_t)q;
    }
    __device__ inline uint32_t get(uint64_t f0, uint32_t nf, uint32_t i, bool a_raw) const {   // fp32 bits (RAW) or the code
        if (a_raw) return a32[f0 + i];
        const int32_t q = a16[at16(f0, nf, i)];
        return (q == kWideMarker) ? a32[f0 + i] : (uint32_t)q;
    }
};
static_assert(kTile16R == 32 && kSeg == 256, "at16 assumes 8 phases of 32 symbols per segment");

struct CompressArgs {
    const float* in;          // fp32 input (compress) or nullptr (reduce: the sums staged in the workspace are encoded)
    uint64_t n;
    uint32_t chunk, n_frames, K, sbpf, stat_block;
    int32_t force_codec;
    uint32_t min_gain_permil, huff_min_bytes;
    float eb, step, inv_step;
    uint32_t step_bits;
    uint32_t seed;            // stochastic quantizer only (kernels built with QM = 1; reduce: the ring step's local quantizer)
    const float* red_local;   // reduce only: the rank's own fp32 message of a ring step (nullptr: two coded operands)
    uint32_t red_sr;          // reduce only: the ring step quantizes its local data stochastically
    uint32_t pred;            // predictor of the stream: 0 none, 1 delta on the codes (kernels built with DELTA = 1)
    uint8_t* out; uint64_t out_cap;
    uint8_t* ws; WsLayout L;
    void* res;                // nz_result* (device)
    // sampled arbitration only (encoder source 2): the cached code, where each group's bitstream is materialised
    // before the frame's groups are packed together, the groups' realized bit counts and the frames' failure flags
    const DevContext* rea_ctx; uint32_t* rea_tmp; uint32_t* rea_gbits; uint32_t* rea_fail;
    uint32_t rea_sample_elems, rea_small_batch_bytes;   // SampleWindow in elements, SmallBatchFastPath threshold
    uint32_t rea_link_ps, rea_fixed_alpha_ns, rea_fixed_ps, rea_huff_alpha_ns, rea_huff_ps;   // cost model of Eq. 1
    uint64_t rea_slot;        // bytes between frame starts of the slotted stream
};

// Result record as laid out by nz_result in the public header.
struct ResultRec { uint64_t bytes; uint32_t status, n_frames, n_raw, n_fixed, n_huff, reserved; };

struct DecodeArgs {
    const uint8_t* a; uint64_t a_bytes;
    const uint8_t* b; uint64_t b_bytes;       // second operand (reduce only)
    float* out;                               // decompress only
    const float* local;                       // ring-step reduce only: the rank's own fp32 message
    float eb, inv_step;                       // ring-step reduce only: the quantizer's bound and 1/step
    uint32_t sr, seed;                        // ring-step reduce only: local data quantized stochastically, with this seed
    uint32_t set_in;                          // k-ary reduce: the staging set that holds the running value (see k_decode)
    uint64_t n;
    uint32_t chunk, n_frames, K, dbpf, pred;
    float step; uint32_t step_bits;
    uint8_t* ws; WsLayout L;                  // reduce only: staged codes, partial histograms
    void* res;
};

hipError_t launch_init(void* zero_base, size_t zero_bytes, void* res, uint32_t n_frames, uint32_t status, hipStream_t st);
hipError_t launch_stats(const CompressArgs& A, bool stochastic, hipStream_t st);
hipError_t launch_stats_codes(const CompressArgs& A, hipStream_t st);   // reduce with the delta predictor: statistics of the staged sums
hipError_t launch_codebook(const CompressArgs& A, hipStream_t st);
hipError_t launch_encode(const CompressArgs& A, bool from_codes, bool stochastic, hipStream_t st);
hipError_t launch_qsgd_step(const float* in, uint64_t n, uint32_t levels, float* step_out, double* partials, hipStream_t st);
hipError_t launch_decode(const DecodeArgs& A, int pass, hipStream_t st);   // 0 decompress, 1 / 2 reduce passes, 3-5 ring-step adds, 6 accumulate
hipError_t launch_fix(const DecodeArgs& A, hipStream_t st);
hipError_t launch_fix_acc(const DecodeArgs& A, hipStream_t st);   // k-ary reduce: after an accumulating pass
hipError_t launch_decode_finish(const DecodeArgs& A, hipStream_t st);

}  // namespace nz
