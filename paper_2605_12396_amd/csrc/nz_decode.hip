// nz_decode.hip -- gfx950 kernels of the receiver side: validate stream and frame headers, rebuild the
// canonical decode table from the code lengths carried in the frame, decode one 256-symbol segment per
// thread from its recorded bit offset, then either dequantize (decompress) or add the codes of two
// streams and gather the statistics of the sum (front end of the fused reduce).
//
// Paper mapping: receiver side of Algorithm 2 (ParseHeader, ValidateHeader, DecodeOrMemcpy) and the
// decode + reduce part of the fused receive-decode-reduce-encode-send step (Sec. IV-D).
#include "nz_common.hpp"
#include "nz_scan.hpp"

namespace nz {

constexpr uint32_t kPrimaryBits = 11;         // first-level decode table: 2048 entries of zigzag code | len<<10 (+flags)
enum : uint32_t { KIND_RAW = 0, KIND_FIXED = 1, KIND_HUFF = 2, KIND_ZERO = 3 };

__device__ inline uint64_t pad4d(uint64_t v) { return (v + 3u) & ~(uint64_t)3u; }
__device__ inline uint64_t pad16d(uint64_t v) { return (v + 15u) & ~(uint64_t)15u; }

// Stream header checks (format violations first, then disagreement with the caller's n / step / options).
__device__ inline uint32_t check_stream(const uint8_t* s, uint64_t bytes, const DecodeArgs& A, uint64_t& total) {
    total = 0;
    if (bytes < kStreamHdr) return ST_CORRUPT;
    const uint32_t* h = reinterpret_cast<const uint32_t*>(s);
    if (h[0] != kMagicStream || h[1] != 1u) return ST_CORRUPT;
    const uint64_t n = (uint64_t)h[2] | ((uint64_t)h[3] << 32);
    const uint32_t chunk = h[4], nfr = h[5], stepb = h[6], seg = h[7], K = h[8];
    total = (uint64_t)h[10] | ((uint64_t)h[11] << 32);
    if (n == 0 || chunk == 0 || chunk > kMaxChunk) return ST_CORRUPT;
    if (seg < 32u || seg > 1024u) return ST_CORRUPT;
    if (K < 2u || K > kMaxK || (K & (K - 1u))) return ST_CORRUPT;
    if ((n + chunk - 1) / chunk != (uint64_t)nfr) return ST_CORRUPT;
    if (total > bytes || total < kStreamHdr + pad16d(8ull * nfr)) return ST_CORRUPT;
    if (n != A.n || stepb != A.step_bits) return ST_MISMATCH;
    if (chunk != A.chunk || K != A.K || seg != kSeg) return ST_MISMATCH;
    return ST_OK;
}

// Shared memory of one operand's decoder.
constexpr uint32_t kRun = 8;                   // symbols per run: window reloads happen at run starts only
constexpr uint32_t kWinFreshBits = 193;        // bits a freshly loaded window offers before a lane must reload
constexpr uint32_t kSubBits = 6;               // second-level tables resolve codes of 12..17 bits
constexpr uint32_t kMaxSub = 32;               // at most this many second-level tables (the rest: canonical search)

struct DecTables {
    uint16_t tab[1u << kPrimaryBits];
    uint16_t tab2[kMaxSub << kSubBits];
    uint16_t sorted[kMaxK];
    uint16_t sub_prefix[kMaxSub];
    uint32_t cnt[32], first[32], idx0[32];
    uint32_t nsub;
};

struct FrameView {
    uint32_t status;          // ST_OK or the reason the frame was rejected
    uint32_t kind;            // KIND_*
    uint32_t w;               // FIXEDLEN width
    const uint32_t* words;    // RAW: payload words; FIXEDLEN/HUFFMAN: bitstream words
    uint32_t nwords;
    const uint16_t* segt;
    uint64_t seg_prefix;      // bits before this workgroup's first segment
    uint32_t cadence;         // HUFFMAN: runs of 8 symbols between two scheduled window reloads
};

// Build-time scratch shared by both operands.
struct BuildScratch {
    __align__(4) uint8_t len[kMaxK];
    uint16_t rank[kMaxK];
    uint32_t wcnt[16 * 32];
    uint64_t red[2][kDecThreads / 64];
};

// Sums of two 64-bit values over the workgroup, one barrier pair for both.
template <int NT>
__device__ inline void block_sum64x2(uint64_t& a, uint64_t& b, uint64_t (*s_red)[kDecThreads / 64]) {
    a = wave_sum64(a); b = wave_sum64(b);
    __syncthreads();
    if (lane_id() == 0) { s_red[0][threadIdx.x >> 6] = a; s_red[1][threadIdx.x >> 6] = b; }
    __syncthreads();
    a = 0; b = 0;
    for (int i = 0; i < NT / 64; i++) { a += s_red[0][i]; b += s_red[1][i]; }
}

// Validate one frame and prepare its decoder (all threads of the workgroup call this together).
template <int NT>
__device__ inline void open_frame(const uint8_t* s, uint64_t total, uint32_t frame, uint32_t nf, uint32_t first_seg,
                                  const DecodeArgs& A, DecTables* T, BuildScratch* B, FrameView& V) {
    const uint32_t tid = threadIdx.x;
    V.status = ST_CORRUPT; V.kind = KIND_ZERO; V.w = 0; V.words = nullptr; V.nwords = 0; V.segt = nullptr; V.seg_prefix = 0;
    V.cadence = 1;
    const uint64_t off = *reinterpret_cast<const uint64_t*>(s + kStreamHdr + 8ull * frame);
    if ((off & 15u) || off < kStreamHdr + pad16d(8ull * A.n_frames) || off + kHdrBytes > total) return;
    const uint8_t* fr = s + off;
    const uint4 h0 = reinterpret_cast<const uint4*>(fr)[0], h1 = reinterpret_cast<const uint4*>(fr)[1];
    const uint32_t x = kCheckXor ^ h0.x ^ h0.y ^ h0.z ^ h0.w ^ h1.x ^ h1.y ^ h1.z;
    if (h0.x != kMagicFrame || h1.w != x) return;
    const uint32_t codec = h0.y, raw_bytes = h0.z, payload = h0.w, p0 = h1.x, p1 = h1.y;
    if (codec > 2u || raw_bytes != 4u * nf) return;
    if (off + kHdrBytes + (uint64_t)payload > total) return;
    if (h1.z != A.step_bits) { V.status = ST_MISMATCH; return; }
    const uint8_t* pay = fr + kHdrBytes;
    if (codec == CODEC_RAW) {
        if (payload != 4u * nf || p0 || p1) return;
        V.status = ST_OK; V.kind = KIND_RAW; V.words = reinterpret_cast<const uint32_t*>(pay); V.nwords = nf;
        return;
    }
    if (codec == CODEC_FIXED) {
        if (p0 > 32u || p1) return;
        const uint64_t need = 4ull * (((uint64_t)nf * p0 + 31u) / 32u);
        if (payload != need) return;
        V.status = ST_OK; V.kind = KIND_FIXED; V.w = p0;
        V.words = reinterpret_cast<const uint32_t*>(pay); V.nwords = payload / 4;
        return;
    }
    // HUFFMAN
    const uint32_t nsym = p0, seg = p1 & 0xFFFFu, K = p1 >> 16;
    if (seg != kSeg || K != A.K || nsym == 0 || nsym > K) return;
    const uint32_t nseg = (nf + kSeg - 1) / kSeg;
    const uint64_t tables = pad4d(nsym) + pad4d(2ull * nseg);
    if (payload < tables || (payload & 3u)) return;
    const uint8_t* lens = pay;
    const uint16_t* segt = reinterpret_cast<const uint16_t*>(pay + pad4d(nsym));
    // code lengths (4 per thread): <= 28, padding zero, at least one used, Kraft sum <= 1
    static_assert(NT * 4 >= kMaxK, "one pass over the code lengths");
    uint32_t bad = 0;
    uint64_t kraft = 0;
    {
        const uint32_t lw = (4u * tid < (uint32_t)pad4d(nsym)) ? reinterpret_cast<const uint32_t*>(lens)[tid] : 0u;
        uint32_t clean = 0;
#pragma unroll
        for (uint32_t j = 0; j < 4; j++) {
            const uint32_t L = (lw >> (8 * j)) & 0xFFu, t = 4u * tid + j;
            if (L > kMaxLen || (t >= nsym && L)) bad = 1;
            else if (L) { kraft += 1ull << (kMaxLen - L); clean |= L << (8 * j); }
        }
        if (4u * tid < kMaxK) reinterpret_cast<uint32_t*>(B->len)[tid] = clean;
    }
    // segment table (two entries per load): bits before this workgroup's first segment, and in the whole frame
    uint32_t pre = 0, all = 0;
    {
        const uint32_t* segt32 = reinterpret_cast<const uint32_t*>(segt);
        const uint32_t npairs = (nseg + 1u) / 2u;
        for (uint32_t p2 = tid; p2 < npairs; p2 += NT) {
            const uint32_t v = segt32[p2], g = 2u * p2, v0 = v & 0xFFFFu, v1 = v >> 16;
            all += v0; if (g < first_seg) pre += v0;
            if (g + 1u < nseg) { all += v1; if (g + 1u < first_seg) pre += v1; }
            else if (v1) bad = 1;                                      // padding entry of an odd table
        }
    }
    uint64_t r0 = kraft + ((uint64_t)bad << 48), r1 = (uint64_t)pre | ((uint64_t)all << 32);
    block_sum64x2<NT>(r0, r1, B->red);
    kraft = r0 & ((1ull << 48) - 1ull);
    const uint64_t pre_bits = r1 & 0xFFFFFFFFull, all_bits = r1 >> 32;
    if ((r0 >> 48) || kraft == 0 || kraft > (1ull << kMaxLen)) return;
    const uint64_t avail = 8ull * (payload - tables);
    if (all_bits > avail || 4ull * ((all_bits + 31u) / 32u) != payload - tables) return;
    // canonical tables and the first-level lookup
    uint32_t* s_cnt = T->cnt; uint32_t* s_first = T->first; uint32_t* s_idx0 = T->idx0;
    canonical_tables<NT>(B->len, K, B->wcnt, s_cnt, s_first, s_idx0, B->rank);
    for (uint32_t sy = tid; sy < K; sy += NT) {
        const uint32_t L = B->len[sy];
        if (L) T->sorted[s_idx0[L] + B->rank[sy]] = (uint16_t)sy;
    }
    if (tid == 0) T->nsub = 0;
    __syncthreads();
    // Entry formats (16 bits).  First level, indexed by the next 11 stream bits:
    //   (q & 1023) | L<<10   symbol with quantization code q (10-bit two's complement) and an L <= 11 bit code
    //   0x8000 | L<<10       escape symbol with an L-bit code (32 raw bits follow)
    //   0xC000 | id          no code of <= 11 bits starts here; id < kMaxSub: second-level table, else search
    // Second level, indexed by stream bits 11..16: same with L-11 in place of L; 0xC000 = longer still.
    // Canonical codes left-justified to a common width are ordered by length, so the length of the code that
    // starts an entry's bits is found by comparing against the end of every length's range (no table walk).
    {
        uint32_t lim[kPrimaryBits + 1];                                // end of the codes of length <= l, 11-bit scale
#pragma unroll
        for (uint32_t l = 1; l <= kPrimaryBits; l++) lim[l] = (s_first[l] + s_cnt[l]) << (kPrimaryBits - l);
#pragma unroll
        for (uint32_t i = tid; i < (1u << kPrimaryBits); i += NT) {
            const uint32_t v = __brev(i) >> (32 - kPrimaryBits);       // stream order: first bit is the code's MSB
            uint32_t L = 1;
#pragma unroll
            for (uint32_t l = 1; l < kPrimaryBits; l++) L += (v >= lim[l]) ? 1u : 0u;
            uint32_t e = 0xC000u;
            if (v < lim[kPrimaryBits]) {
                const uint32_t sy = T->sorted[s_idx0[L] + (v >> (kPrimaryBits - L)) - s_first[L]];
                e = sy ? (((uint32_t)unzigzag(sy - 1u) & 1023u) | (L << 10)) : (0x8000u | (L << 10));
            } else {
                const uint32_t id = atomicAdd(&T->nsub, 1u);
                if (id < kMaxSub) { e |= id; T->sub_prefix[id] = (uint16_t)i; } else e |= 0x3FFu;
            }
            T->tab[i] = (uint16_t)e;
        }
    }
    __syncthreads();
    {
        constexpr uint32_t W2 = kPrimaryBits + kSubBits;
        const uint32_t nsub = T->nsub < kMaxSub ? T->nsub : kMaxSub;
        uint32_t lim[kSubBits + 1];                                    // end of the codes of length <= 11 + l, 17-bit scale
#pragma unroll
        for (uint32_t l = 1; l <= kSubBits; l++) lim[l] = (s_first[kPrimaryBits + l] + s_cnt[kPrimaryBits + l]) << (kSubBits - l);
#pragma unroll 1
        for (uint32_t idx = tid; idx < (nsub << kSubBits); idx += NT) {
            const uint32_t hi11 = __brev((uint32_t)T->sub_prefix[idx >> kSubBits]) >> (32 - kPrimaryBits);
            const uint32_t v = (hi11 << kSubBits) | (__brev(idx & ((1u << kSubBits) - 1u)) >> (32 - kSubBits));
            uint32_t L = kPrimaryBits + 1;
#pragma unroll
            for (uint32_t l = 1; l < kSubBits; l++) L += (v >= lim[l]) ? 1u : 0u;
            uint32_t e = 0xC000u;
            if (v < lim[kSubBits]) {
                const uint32_t sy = T->sorted[s_idx0[L] + (v >> (W2 - L)) - s_first[L]];
                e = sy ? (((uint32_t)unzigzag(sy - 1u) & 1023u) | ((L - kPrimaryBits) << 10)) : (0x8000u | ((L - kPrimaryBits) << 10));
            }
            T->tab2[idx] = (uint16_t)e;
        }
    }
    __syncthreads();
    {   // schedule reloads so that an average lane (with a 25 % margin) never needs one of its own
        const uint32_t run_bits = (uint32_t)((all_bits * kRun) / nf) + 1u;
        const uint32_t c = kWinFreshBits / (run_bits + run_bits / 4u);
        V.cadence = c < 1u ? 1u : (c > 16u ? 16u : c);
    }
    V.status = ST_OK; V.kind = KIND_HUFF; V.segt = segt; V.seg_prefix = pre_bits;
    V.words = reinterpret_cast<const uint32_t*>(pay + tables); V.nwords = (uint32_t)((payload - tables) / 4);
}

// Per-thread sequential reader of one HUFFMAN segment.  Every lane owns a small window (kWinWords words) in
// LDS, filled from global memory with dword-aligned 16-byte loads starting at the word the lane is in.  Reloads
// happen at the start of a run of 8 symbols, a point that is uniform over the wave: on a schedule derived from
// the frame's average code length (so that the global-load stall is paid once for all lanes and few fetched
// bytes go unused), and for a single lane when it is kWinRunLimit or more bits into its window; a lane also
// reloads at once when a long code or an escape leaves it kWinSlowLimit or more bits into the window.
// Window words k and k+1 of the current position live in registers (lo, hi), so the next 32 stream bits are a
// funnel shift away and the only LDS access on a symbol's critical path is the table lookup; words k+2 and k+3
// are re-read from the window after every symbol and are back long before a later symbol shifts them in.
// Budget: 8 first-level symbols use at most 88 bits, a long code 28, an escape 60, so lo and hi always come
// from inside the window (k + 1 < kWinWords); the two prefetched words may lie up to two rows past it, inside
// the shared-memory block that follows the windows, and are never shifted in before a reload replaces them.
// Near the end of the bitstream words are fetched one by one with the index clamped to the last word, so any
// input stays in bounds (a valid stream never consumes a clamped word).
constexpr uint32_t kWinWords = 12;
constexpr uint32_t kWinBits = 32 * kWinWords;
// A read of words k, k+1 at position p needs p < kWinBits - 32.  After a long code or an escape a lane reloads
// unless p < kWinSlowLimit; up to 7 first-level symbols (77 bits) and the code of an escape (28 bits) may follow
// before the next check, and the escape's raw word is read there: kWinSlowLimit + 77 + 28 < kWinBits - 32.
constexpr uint32_t kWinSlowLimit = kWinBits - 32 - 77 - 28 - 7;      // 240 for 12 words
constexpr uint32_t kWinRunLimit = kWinSlowLimit - 16;                // reload at a run start when this far in
static_assert(kWinRunLimit - 31 == kWinFreshBits, "cadence constant out of step with the window size");
constexpr uint32_t kWinOverRows = 2;                                 // rows a prefetch may reach past the window

struct HuffReader {
    uint64_t bits_addr;                  // byte address of bitstream word 0
    uint32_t nwords;                     // words in the bitstream (at least 1)
    uint32_t* win;                       // this lane's window in LDS (word j at win[j * kDecThreads])
    int32_t win_bit0;                    // bit index (relative to bitstream bit 0) of window word 0
    uint32_t k, sh;                      // current position: bit sh (0..31) of window word k
    uint32_t lo, hi, n1, n2;             // window words k .. k+3
    uint32_t start_bit, bad;
    const DecTables* T;

    __device__ inline void init(const FrameView& V, const DecTables* tables, uint32_t bitpos, const void* safe16,
                                uint32_t* lane_window) {
        T = tables; bad = 0; win = lane_window; start_bit = bitpos;
        if (V.nwords == 0 || V.kind != KIND_HUFF) {                      // nothing to read: point at valid memory
            bits_addr = reinterpret_cast<uint64_t>(safe16); nwords = 1;
        } else {
            bits_addr = reinterpret_cast<uint64_t>(V.words); nwords = V.nwords;
        }
        win_bit0 = (int32_t)bitpos; k = 0; sh = 0; lo = hi = n1 = n2 = 0;
    }
    __device__ inline uint32_t pos() const { return 32u * k + sh; }
    __device__ inline void reload() {
        const uint32_t cur = (uint32_t)(win_bit0 + (int32_t)pos());
        const uint32_t wi = cur >> 5;
        // the window is stored word-major (word j of every lane side by side): conflict-free for equal j
        if (__builtin_expect(wi + kWinWords <= nwords, 1)) {
            // dword-aligned 16-byte loads straight from the lane's position (no alignment waste)
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            typedef u32x4 u32x4_a4 __attribute__((aligned(4)));
            typedef const u32x4_a4 __attribute__((address_space(1))) * gptr;  // plain global loads, not flat ones
            gptr p = reinterpret_cast<gptr>(bits_addr + 4ull * wi);
            u32x4 x[kWinWords / 4];
#pragma unroll
            for (uint32_t c = 0; c < kWinWords / 4; c++) x[c] = p[c];
#pragma unroll
            for (uint32_t c = 0; c < kWinWords / 4; c++) {
                win[(4 * c + 0) * kDecThreads] = x[c].x; win[(4 * c + 1) * kDecThreads] = x[c].y;
                win[(4 * c + 2) * kDecThreads] = x[c].z; win[(4 * c + 3) * kDecThreads] = x[c].w;
            }
            lo = x[0].x; hi = x[0].y; n1 = x[0].z; n2 = x[0].w;
        } else {
            // near the end of the bitstream: word by word, indices clamped to the last word
            typedef const uint32_t __attribute__((address_space(1))) * wptr;
            wptr w = reinterpret_cast<wptr>(bits_addr);
            const uint32_t last = nwords - 1u;
#pragma unroll 1
            for (uint32_t j = 0; j < kWinWords; j++) win[j * kDecThreads] = w[wi + j < last ? wi + j : last];
            lo = win[0]; hi = win[kDecThreads]; n1 = win[2 * kDecThreads]; n2 = win[3 * kDecThreads];
        }
        win_bit0 = (int32_t)(cur & ~31u);
        k = 0; sh = cur & 31u;
    }
    __device__ inline uint32_t consumed() const { return (uint32_t)(win_bit0 + (int32_t)pos()) - start_bit; }
    // Decode one symbol in two halves, so that a caller with two readers can issue both table lookups before
    // either result is needed: lookup() returns the table entry for the next stream bits (w32), finish() turns
    // it into the symbol's quantization code and advances.  on_escape(z) maps the zigzag value carried by an
    // escaped symbol to the returned code.
    __device__ inline uint32_t lookup(uint32_t& w32) const {
        w32 = __builtin_amdgcn_alignbit(hi, lo, sh);                     // the next 32 stream bits
        return T->tab[w32 & ((1u << kPrimaryBits) - 1u)];
    }
    template <typename F>
    __device__ inline int32_t finish(uint32_t e, uint32_t w32, F&& on_escape) {
        int32_t q;
        if (__builtin_expect(e < 0x8000u, 1)) { sh += e >> 10; q = (int32_t)(e << 22) >> 22; }
        else q = next_slow(e, w32, on_escape);
        const bool c = sh >= 32u;                                        // at most one word is used up per symbol here
        lo = c ? hi : lo; hi = c ? n1 : hi; k += c ? 1u : 0u; sh &= 31u;
        const uint32_t* p = win + k * kDecThreads;
        n1 = p[2 * kDecThreads]; n2 = p[3 * kDecThreads];
        return q;
    }
    template <typename F>
    __device__ inline int32_t next(F&& on_escape) {
        uint32_t w32;
        const uint32_t e = lookup(w32);
        return finish(e, w32, on_escape);
    }
    template <typename F>
    __device__ inline int32_t next_slow(uint32_t e, uint32_t w32, F&& on_escape) {
        uint32_t L = (e >> 10) & 15u, esc = (e < 0xC000u);
        int32_t q = 0;
        if (e >= 0xC000u) {
            uint32_t e2 = 0xC000u;
            const uint32_t id = e & 0x3FFu;
            if (id < kMaxSub) e2 = T->tab2[(id << kSubBits) + ((w32 >> kPrimaryBits) & ((1u << kSubBits) - 1u))];
            if (e2 < 0xC000u) {
                L = kPrimaryBits + ((e2 >> 10) & 7u); q = (int32_t)(e2 << 22) >> 22; esc = (e2 >= 0x8000u);
            } else {                                                     // longer than 17 bits or unassigned: search
                uint32_t code = 0, sy = 1;
                L = 0;
#pragma unroll 1
                for (uint32_t l = 1; l <= kMaxLen; l++) {
                    uint32_t li = l;
                    asm volatile("" : "+v"(li));                         // keeps the table reads inside this rare loop
                    code = (code << 1) | ((w32 >> (l - 1)) & 1u);
                    const uint32_t d = code - T->first[li];
                    if (d < T->cnt[li]) { sy = T->sorted[T->idx0[li] + d]; L = l; break; }
                }
                if (L == 0) { bad = 1; L = 1; sy = 1; }
                q = unzigzag(sy - 1u); esc = (sy == 0);
            }
        }
        sh += L;                                                         // < 64
        if (esc) {                                                       // escape: the 32 raw bits of z follow
            if (sh >= 32u) { lo = hi; hi = n1; n1 = n2; k++; sh -= 32u; }
            q = on_escape(__builtin_amdgcn_alignbit(hi, lo, sh));
            lo = hi; hi = n1; k++;
        }
        if (32u * k + sh >= kWinSlowLimit) reload_normalised();
        return q;
    }
    // reload from a position whose sh may still be >= 32 (the caller's word shift has not happened yet)
    __device__ inline void reload_normalised() { k += sh >> 5; sh &= 31u; reload(); }
};

// Position-addressed fetch of element e of a RAW / FIXEDLEN (or rejected = all-zero) frame.
struct DirectFetch {
    const uint32_t* words; uint32_t last, w, mask, kind;
    __device__ inline void init(const FrameView& V, const uint32_t* safe_word) {
        words = V.words; kind = V.kind; w = V.w;
        uint32_t nwords = V.nwords;
        if (kind == KIND_ZERO) { nwords = 0; w = 0; kind = KIND_FIXED; }
        if (nwords == 0) { words = safe_word; nwords = 1; }
        last = nwords - 1;
        mask = (w >= 32u) ? 0xFFFFFFFFu : ((1u << w) - 1u);
    }
    // zigzag code (FIXEDLEN) or fp32 bit pattern (RAW)
    __device__ inline uint32_t get(uint32_t e) const {
        if (kind == KIND_RAW) return words[e < last ? e : last];
        const uint64_t bp = (uint64_t)e * w;
        const uint32_t i = (uint32_t)(bp >> 5), sh = (uint32_t)(bp & 31u);
        const uint32_t lo = words[i < last ? i : last], hi = words[i + 1 < last ? i + 1 : last];
        return __builtin_amdgcn_alignbit(hi, lo, sh) & mask;
    }
};

constexpr uint32_t kTileR = 16;                      // symbols per thread between two coalesced output phases
constexpr uint32_t kTileStride = kTileR + 1;         // odd row stride: conflict-free column writes

// Shared memory of one decode workgroup.  The windows come first and the tile follows them directly: a
// reader's prefetch may touch up to kWinOverRows rows past its window, which then fall into the next window or
// the tile (valid shared memory, values never used).
template <int NOPS>
struct __align__(16) DecShared {
    uint32_t win[NOPS][kDecThreads * kWinWords];
    union { uint32_t tile[kDecThreads * kTileStride]; BuildScratch build; } u;
    uint64_t wsum[4];
    uint32_t zmax, flags;
};
static_assert(kDecThreads * kTileStride >= kWinOverRows * kDecThreads, "prefetch rows must stay inside the tile");

struct SegCtx {
    uint32_t tid, lane, first_seg, nf, cntseg, e0;
    uint64_t f0;
    bool vec_ok;
};

// Combine one element of A and one of B (reduce): raw operands give the canonical fp32 sum, coded operands
// the exact integer sum (wrapped to 32 bits; a sum beyond 2^30 raises the overflow flag).  ta / tb are fp32 bit
// patterns for a RAW operand and quantization codes otherwise.
template <bool ANY_RAW>
__device__ inline uint32_t combine(uint32_t ta, bool a_raw, uint32_t tb, bool b_raw, float step, uint32_t& overflow) {
    if (ANY_RAW) {
#pragma clang fp contract(off)
        const float fa = a_raw ? __uint_as_float(ta) : dequantize1((int32_t)ta, step);
        const float fb = b_raw ? __uint_as_float(tb) : dequantize1((int32_t)tb, step);
        const float sum = fa + fb;
        return (sum != sum) ? kCanonNaN : __float_as_uint(sum);
    }
    const int32_t qa = (int32_t)ta, qb = (int32_t)tb;
    // only when an operand is 2^29 or more in magnitude can |qa+qb| pass 2^30
    if (__builtin_expect((((uint32_t)qa + (1u << 29)) | ((uint32_t)qb + (1u << 29))) >> 30, 0)) {
        const int64_t Q = (int64_t)qa + (int64_t)qb;
        if (Q > (int64_t)kQSumMax || Q < -(int64_t)kQSumMax) overflow = 1;
    }
    return (uint32_t)qa + (uint32_t)qb;
}

// Coalesced consumer of 4 consecutive elements starting at frame element e (m of them valid).
// MODE 0: dequantize (or pass RAW bits through) and store fp32.  MODE 1: histogram + zmax of the sums
// (coded output) and stage the 32-bit values.
template <int MODE>
__device__ inline void emit4(const DecodeArgs& A, const SegCtx& C, uint32_t e, uint32_t m, const uint32_t t[4], bool raw_vals,
                             uint32_t* s_h, uint32_t ncs, uint32_t copy, uint32_t& zmax) {
    if (MODE == 0) {
        float v[4];
#pragma unroll
        for (uint32_t j = 0; j < 4; j++) v[j] = raw_vals ? __uint_as_float(t[j]) : dequantize1(unzigzag(t[j]), A.step);
        float* dst = A.out + C.f0 + e;
        if (C.vec_ok && m == 4) *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
        else for (uint32_t j = 0; j < m; j++) dst[j] = v[j];
    } else {
        if (!raw_vals) {
#pragma unroll
            for (uint32_t j = 0; j < 4; j++) {
                if (j < m) {
                    const uint32_t z = zigzag((int32_t)t[j]);
                    zmax = z > zmax ? z : zmax;
                    atomicAdd(&s_h[(sym_of(z, A.K) << ncs) + copy], 1u);
                }
            }
        }
        uint32_t* dst = reinterpret_cast<uint32_t*>(A.ws + A.L.codes) + C.f0 + e;
        if (C.vec_ok && m == 4) *reinterpret_cast<uint4*>(dst) = make_uint4(t[0], t[1], t[2], t[3]);
        else for (uint32_t j = 0; j < m; j++) dst[j] = t[j];
    }
}

// One 256-symbol segment per thread, kTileR symbols at a time into an LDS tile, then the workgroup writes the
// tile out with 16-byte stores (kTileR/4 lanes cover one thread's run, so every store instruction fills whole
// 64-byte runs).  KA / KB say which operands are HUFFMAN (sequential reader) and which are addressed directly.
template <int MODE, int KA, int KB, typename SH>
__device__ inline void run_segments(const DecodeArgs& A, const SegCtx& C, HuffReader& ra, HuffReader& rb,
                                    const DirectFetch& da, const DirectFetch& db, SH* S,
                                    uint32_t* s_h, uint32_t ncs, uint32_t ca, uint32_t cb, uint32_t& overflow) {
    const uint32_t tid = C.tid;
    const uint32_t copy = C.lane & ((1u << ncs) - 1u);
    uint32_t* tile = S->u.tile;
    uint32_t zmax = 0;
    constexpr uint32_t LPR = kTileR / 4;             // lanes per row in the output phase
    constexpr bool ANY_RAW = (MODE == 1) && (KA == KIND_RAW || KB == KIND_RAW);
    uint32_t e = C.e0;                               // next element of my segment (frame index)
    auto produce = [&]() -> uint32_t {
        auto code_of = [](uint32_t z) -> int32_t { return unzigzag(z); };
        // both table lookups are issued before either symbol is finished (two independent dependency chains)
        uint32_t wa = 0, wb = 0, ea = 0, eb = 0;
        if (KA == KIND_HUFF) ea = ra.lookup(wa);
        if (KB == KIND_HUFF) eb = rb.lookup(wb);
        uint32_t ta, tb;
        if (KA == KIND_HUFF) ta = (uint32_t)ra.finish(ea, wa, code_of);
        else { ta = da.get(e); if (KA == KIND_FIXED) ta = (uint32_t)unzigzag(ta); }
        if (KB == KIND_HUFF) tb = (uint32_t)rb.finish(eb, wb, code_of);
        else { tb = db.get(e); if (KB == KIND_FIXED) tb = (uint32_t)unzigzag(tb); }
        e++;
        return combine<ANY_RAW>(ta, KA == KIND_RAW, tb, KB == KIND_RAW, A.step, overflow);
    };
    uint32_t due_a = 1, due_b = 1;                                       // runs left until the next scheduled reload
    auto start_run = [&]() {
        if (KA == KIND_HUFF) {
            const bool sched = (--due_a == 0);                           // uniform over the workgroup
            if (sched) due_a = ca;
            if (sched || ra.pos() >= kWinRunLimit) ra.reload();
        }
        if (MODE == 1 && KB == KIND_HUFF) {
            const bool sched = (--due_b == 0);
            if (sched) due_b = cb;
            if (sched || rb.pos() >= kWinRunLimit) rb.reload();
        }
    };
    for (uint32_t r0 = 0; r0 < kSeg; r0 += kTileR) {
        uint32_t* row = tile + tid * kTileStride;
        if (r0 + kTileR <= C.cntseg) {                                   // full run: static tile offsets
#pragma unroll
            for (uint32_t h = 0; h < kTileR; h += kRun) {
                start_run();
#pragma unroll
                for (uint32_t r = 0; r < kRun; r++) row[h + r] = produce();
            }
        } else if (r0 < C.cntseg) {
            const uint32_t nr = C.cntseg - r0;
            for (uint32_t r = 0; r < nr; r++) {
                if ((r % kRun) == 0) start_run();
                row[r] = produce();
            }
        }
        __syncthreads();
#pragma unroll
        for (uint32_t k = 0; k < LPR; k++) {
            const uint32_t g = tid + kDecThreads * k;
            const uint32_t rw = g / LPR, c = (g % LPR) * 4;
            const uint32_t eo = (C.first_seg + rw) * kSeg + r0 + c;             // element index in the frame
            if (eo < C.nf) {
                const uint32_t m = (C.nf - eo < 4) ? (C.nf - eo) : 4u;
                uint32_t t[4];
#pragma unroll
                for (uint32_t j = 0; j < 4; j++) t[j] = tile[rw * kTileStride + c + j];
                emit4<MODE>(A, C, eo, m, t, MODE == 0 ? false : ANY_RAW, s_h, ncs, copy, zmax);
            }
        }
        __syncthreads();
    }
    if (MODE == 1) {
        zmax = wave_max(zmax);
        if (C.lane == 0) atomicMax(&S->zmax, zmax);
    }
}

// Decompress of a HUFFMAN frame.  Same scheme as run_segments, but the tile holds 16-bit quantization codes,
// 32 per thread between two output phases, so that eight lanes write one thread's run as a full 128-byte line.
// A code that does not fit 16 bits (an escape with a large value) is stored straight to global memory by the
// decoding lane, which leaves the marker -32768 in the tile and raises a workgroup flag; only then does the
// output phase look for markers and write around them.
constexpr uint32_t kTile16R = 32;
constexpr uint32_t kTile16Stride = kTile16R + 2;     // halfwords per row: 17 words, an odd word stride
constexpr int32_t kWideMarker = -32768;

template <typename SH>
__device__ inline void run_decompress_huff(const DecodeArgs& A, const SegCtx& C, HuffReader& ra, SH* S, uint32_t ca) {
    static_assert(kDecThreads * kTile16Stride * 2 <= sizeof(S->u.tile), "16-bit tile must fit the tile storage");
    const uint32_t tid = C.tid;
    uint16_t* tile = reinterpret_cast<uint16_t*>(S->u.tile);
    uint32_t* row32 = reinterpret_cast<uint32_t*>(tile + tid * kTile16Stride);
    float* seg_out = A.out + C.f0 + C.e0;
    uint32_t e = 0;                                   // symbols of my segment decoded so far
    uint32_t due = 1;
    auto start_run = [&]() {
        const bool sched = (--due == 0);              // uniform over the workgroup
        if (sched) due = ca;
        if (sched || ra.pos() >= kWinRunLimit) ra.reload();
    };
    auto wide = [&](uint32_t z) -> int32_t {          // only an escape can carry a code of 16 bits or more
        int32_t q = unzigzag(z);
        if (z >= 0xFFFFu) { seg_out[e] = dequantize1(q, A.step); q = kWideMarker; S->flags = 1u; }
        return q;
    };
    auto next16 = [&]() -> uint32_t { const int32_t q = ra.next(wide); e++; return (uint32_t)q; };
    constexpr uint32_t LPR = kTile16R / 4;            // 8 lanes write one row
    // output phase: thread (row rw0 + 32 k, columns c .. c+3) for k = 0..7
    const uint32_t rw0 = tid / LPR, c = (tid % LPR) * 4;
    const uint32_t* src0 = reinterpret_cast<const uint32_t*>(tile + rw0 * kTile16Stride + c);
    const uint32_t eo0 = (C.first_seg + rw0) * kSeg + c;
    const bool whole = C.vec_ok && (C.first_seg + kDecThreads) * kSeg <= C.nf;   // every store is a full, aligned float4
    for (uint32_t r0 = 0; r0 < kSeg; r0 += kTile16R) {
        if (r0 + kTile16R <= C.cntseg) {
#pragma unroll
            for (uint32_t h = 0; h < kTile16R; h += kRun) {
                start_run();
#pragma unroll
                for (uint32_t r = 0; r < kRun; r += 2) {
                    const uint32_t q0 = next16(), q1 = next16();
                    row32[(h + r) / 2] = (q0 & 0xFFFFu) | (q1 << 16);
                }
            }
        } else if (r0 < C.cntseg) {
            const uint32_t nr = C.cntseg - r0;
            uint16_t* row = tile + tid * kTile16Stride;
            for (uint32_t r = 0; r < nr; r++) {
                if ((r % kRun) == 0) start_run();
                row[r] = (uint16_t)next16();
            }
        }
        __syncthreads();
        if (__builtin_expect(whole && S->flags == 0, 1)) {
            float* dst = A.out + C.f0 + eo0 + r0;
#pragma unroll
            for (uint32_t k = 0; k < LPR; k++) {
                const uint32_t* src = src0 + k * (kDecThreads / LPR) * (kTile16Stride / 2);
                const uint32_t p0 = src[0], p1 = src[1];
                float4 v;
                v.x = dequantize1((int32_t)(int16_t)(p0 & 0xFFFFu), A.step); v.y = dequantize1((int32_t)p0 >> 16, A.step);
                v.z = dequantize1((int32_t)(int16_t)(p1 & 0xFFFFu), A.step); v.w = dequantize1((int32_t)p1 >> 16, A.step);
                // streaming store: the output is not read again here and should not displace the bitstream in L2
                typedef float f32x4 __attribute__((ext_vector_type(4)));
                f32x4 vv; vv.x = v.x; vv.y = v.y; vv.z = v.z; vv.w = v.w;
                __builtin_nontemporal_store(vv, reinterpret_cast<f32x4*>(dst + (size_t)k * (kDecThreads / LPR) * kSeg));
            }
        } else {
#pragma unroll 1
            for (uint32_t k = 0; k < LPR; k++) {
                const uint32_t eo = eo0 + k * (kDecThreads / LPR) * kSeg + r0;      // element index in the frame
                if (eo < C.nf) {
                    const uint32_t m = (C.nf - eo < 4) ? (C.nf - eo) : 4u;
                    const uint32_t* src = src0 + k * (kDecThreads / LPR) * (kTile16Stride / 2);
                    const uint32_t p0 = src[0], p1 = src[1];
                    const int32_t q[4] = { (int32_t)(int16_t)(p0 & 0xFFFFu), (int32_t)p0 >> 16,
                                           (int32_t)(int16_t)(p1 & 0xFFFFu), (int32_t)p1 >> 16 };
                    float* dst = A.out + C.f0 + eo;
                    for (uint32_t j = 0; j < m; j++) if (q[j] != kWideMarker) dst[j] = dequantize1(q[j], A.step);
                }
            }
        }
        __syncthreads();
    }
}

// Frames without a HUFFMAN operand: element-parallel and coalesced on both sides.
template <int MODE, typename SH>
__device__ inline void run_elementwise(const DecodeArgs& A, const SegCtx& C, uint32_t blk0, const DirectFetch& da,
                                       const DirectFetch& db, SH* S, uint32_t* s_h, uint32_t ncs, uint32_t& overflow) {
    const uint32_t cnt = (C.nf - blk0 < kDecBlock) ? (C.nf - blk0) : kDecBlock;
    const uint32_t copy = C.lane & ((1u << ncs) - 1u);
    const bool a_raw = da.kind == KIND_RAW, b_raw = (MODE == 1) && db.kind == KIND_RAW;
    uint32_t zmax = 0;
    for (uint32_t i = C.tid * 4; i < cnt; i += kDecThreads * 4) {
        const uint32_t e = blk0 + i;
        const uint32_t m = (cnt - i < 4) ? (cnt - i) : 4u;
        uint32_t t[4] = { 0, 0, 0, 0 };
        for (uint32_t j = 0; j < m; j++) {
            uint32_t ta = da.get(e + j);
            if (MODE == 0) t[j] = ta;
            else {
                uint32_t tb = db.get(e + j);
                if (!a_raw) ta = (uint32_t)unzigzag(ta);
                if (!b_raw) tb = (uint32_t)unzigzag(tb);
                t[j] = (a_raw || b_raw) ? combine<true>(ta, a_raw, tb, b_raw, A.step, overflow)
                                        : combine<false>(ta, false, tb, false, A.step, overflow);
            }
        }
        emit4<MODE>(A, C, e, m, t, MODE == 0 ? a_raw : (a_raw || b_raw), s_h, ncs, copy, zmax);
    }
    if (MODE == 1) {
        zmax = wave_max(zmax);
        if (C.lane == 0) atomicMax(&S->zmax, zmax);
    }
}

// MODE 0: decompress A into fp32.  MODE 1: reduce front end, Q = qa + qb into the workspace + statistics.
template <int MODE>
__global__ __launch_bounds__(kDecThreads) void k_decode(DecodeArgs A) {
    __shared__ DecTables s_t[MODE == 1 ? 2 : 1];
    __shared__ DecShared<(MODE == 1 ? 2 : 1)> S;
    __shared__ uint32_t s_h[MODE == 1 ? 2048 : 1];

    const uint32_t tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const uint32_t frame = blockIdx.x / A.dbpf, db = blockIdx.x % A.dbpf;
    const uint64_t f0 = (uint64_t)frame * A.chunk;
    const uint32_t nf = (uint32_t)((A.n - f0 < A.chunk) ? (A.n - f0) : A.chunk);
    const uint32_t blk0 = db * kDecBlock;
    if (blk0 >= nf) return;
    ResultRec* res = reinterpret_cast<ResultRec*>(A.res);
    const uint32_t first_seg = db * kDecThreads;
    const uint32_t nseg = (nf + kSeg - 1) / kSeg;
    const uint32_t gseg = first_seg + tid;
    const bool seg_valid = gseg < nseg;
    const uint32_t e0 = gseg * kSeg;                                    // first element of my segment in the frame
    const uint32_t cntseg = seg_valid ? ((nf - e0 < kSeg) ? (nf - e0) : kSeg) : 0u;

    uint64_t total_a = 0, total_b = 0;
    const uint32_t st_a = check_stream(A.a, A.a_bytes, A, total_a);
    uint32_t st_b = ST_OK;
    if (MODE == 1) st_b = check_stream(A.b, A.b_bytes, A, total_b);
    if (blockIdx.x == 0 && tid == 0) {
        if (st_a) atomicMax(&res->status, st_a);
        if (st_b) atomicMax(&res->status, st_b);
        if (MODE == 0 && st_a == ST_OK) res->bytes = total_a;
    }
    if (MODE == 0 && st_a) return;                                      // nothing is written on a stream-level error

    FrameView va, vb;
    va.status = ST_OK; va.kind = KIND_ZERO; va.w = 0; va.words = nullptr; va.nwords = 0; va.segt = nullptr; va.seg_prefix = 0;
    va.cadence = 1;
    vb = va;
    if (st_a == ST_OK && (MODE == 0 || st_b == ST_OK)) {
        open_frame<kDecThreads>(A.a, total_a, frame, nf, first_seg, A, &s_t[0], &S.u.build, va);
        if (MODE == 1) open_frame<kDecThreads>(A.b, total_b, frame, nf, first_seg, A, &s_t[MODE == 1 ? 1 : 0], &S.u.build, vb);
        if (tid == 0) {
            if (va.status) atomicMax(&res->status, va.status);
            if (MODE == 1 && vb.status) atomicMax(&res->status, vb.status);
            if (MODE == 0 && db == 0 && va.status == ST_OK)
                atomicAdd(va.kind == KIND_RAW ? &res->n_raw : (va.kind == KIND_FIXED ? &res->n_fixed : &res->n_huff), 1u);
        }
        if (MODE == 1 && (va.status || vb.status)) { va.kind = KIND_ZERO; vb.kind = KIND_ZERO; }
    }
    if (MODE == 0 && va.status) return;                                 // rejected frame: its output range is left alone

    // bit offset of my segment inside a HUFFMAN bitstream: prefix of the segment table
    uint32_t bit_a = 0, bit_b = 0, seglen_a = 0, seglen_b = 0;
    {
        const uint32_t la = (va.kind == KIND_HUFF && seg_valid) ? va.segt[gseg] : 0u;
        const uint32_t lb = (MODE == 1 && vb.kind == KIND_HUFF && seg_valid) ? vb.segt[gseg] : 0u;
        seglen_a = la; seglen_b = lb;
        // both lengths are < 2^16: scan them packed in one 64-bit lane value (sums stay below 2^32 each)
        const uint64_t v = (uint64_t)la | ((uint64_t)lb << 32);
        uint64_t incl = v;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) { uint64_t t = __shfl_up(incl, d, 64); if ((int)lane >= d) incl += t; }
        if (lane == 63) S.wsum[wave] = incl;
        if (tid == 0) { S.zmax = 0; S.flags = 0; }
        __syncthreads();
        uint64_t excl = incl - v;
        for (uint32_t w = 0; w < wave; w++) excl += S.wsum[w];
        bit_a = (uint32_t)va.seg_prefix + (uint32_t)(excl & 0xFFFFFFFFull);
        bit_b = (uint32_t)vb.seg_prefix + (uint32_t)(excl >> 32);
    }
    const uint32_t* safe = reinterpret_cast<const uint32_t*>(A.res);
    HuffReader ra, rb;
    DirectFetch da, dbf;
    ra.init(va, &s_t[0], bit_a, safe, &S.win[0][tid]);
    rb.init(vb, &s_t[MODE == 1 ? 1 : 0], bit_b, safe, &S.win[MODE == 1 ? 1 : 0][tid]);
    da.init(va, safe);
    dbf.init(vb, safe);
    SegCtx C;
    C.tid = tid; C.lane = lane; C.first_seg = first_seg; C.nf = nf; C.cntseg = cntseg; C.e0 = e0; C.f0 = f0;
    C.vec_ok = ((f0 & 3u) == 0);
    uint32_t overflow = 0;

    if (MODE == 0) {
        if (va.kind == KIND_HUFF) {
            run_decompress_huff(A, C, ra, &S, va.cadence);
            if (seg_valid && (ra.bad || ra.consumed() != seglen_a)) atomicMax(&res->status, (uint32_t)ST_CORRUPT);
        } else {
            run_elementwise<0>(A, C, blk0, da, dbf, &S, s_h, 0, overflow);
        }
        return;
    }

    // ---- MODE 1: sum of codes, statistics of the sum ----
    const uint32_t K = A.K;
    uint32_t ncs = 0;
    while ((K << (ncs + 1)) <= 2048u && ncs < 5) ncs++;
    for (uint32_t i = tid; i < (K << ncs); i += kDecThreads) s_h[i] = 0;
    __syncthreads();
    const bool out_raw = (va.kind == KIND_RAW) || (vb.kind == KIND_RAW);      // uniform over the frame
    const bool ha = va.kind == KIND_HUFF, hb = vb.kind == KIND_HUFF;
    if (!ha && !hb) run_elementwise<1>(A, C, blk0, da, dbf, &S, s_h, ncs, overflow);
    else if (ha && hb) run_segments<1, KIND_HUFF, KIND_HUFF>(A, C, ra, rb, da, dbf, &S, s_h, ncs, va.cadence, vb.cadence, overflow);
    else if (ha && vb.kind == KIND_RAW) run_segments<1, KIND_HUFF, KIND_RAW>(A, C, ra, rb, da, dbf, &S, s_h, ncs, va.cadence, vb.cadence, overflow);
    else if (ha) run_segments<1, KIND_HUFF, KIND_FIXED>(A, C, ra, rb, da, dbf, &S, s_h, ncs, va.cadence, vb.cadence, overflow);
    else if (va.kind == KIND_RAW) run_segments<1, KIND_RAW, KIND_HUFF>(A, C, ra, rb, da, dbf, &S, s_h, ncs, va.cadence, vb.cadence, overflow);
    else run_segments<1, KIND_FIXED, KIND_HUFF>(A, C, ra, rb, da, dbf, &S, s_h, ncs, va.cadence, vb.cadence, overflow);
    if (seg_valid) {
        if (ha && (ra.bad || ra.consumed() != seglen_a)) atomicMax(&res->status, (uint32_t)ST_CORRUPT);
        if (hb && (rb.bad || rb.consumed() != seglen_b)) atomicMax(&res->status, (uint32_t)ST_CORRUPT);
    }
    if (overflow) atomicMax(&res->status, (uint32_t)ST_RANGE);
    __syncthreads();
    uint32_t* ph = reinterpret_cast<uint32_t*>(A.ws + A.L.phist) + (size_t)blockIdx.x * kMaxK;
    for (uint32_t sy = tid; sy < K; sy += kDecThreads) {
        uint32_t t = 0;
        for (uint32_t c = 0; c < (1u << ncs); c++) t += s_h[(sy << ncs) + c];
        ph[sy] = t;
    }
    if (tid == 0) reinterpret_cast<uint2*>(A.ws + A.L.pmeta)[blockIdx.x] = make_uint2(S.zmax, out_raw ? 1u : 0u);
}

hipError_t launch_decode(const DecodeArgs& A, bool reduce, hipStream_t st) {
    if (reduce) hipLaunchKernelGGL(k_decode<1>, dim3(A.n_frames * A.dbpf), dim3(kDecThreads), 0, st, A);
    else hipLaunchKernelGGL(k_decode<0>, dim3(A.n_frames * A.dbpf), dim3(kDecThreads), 0, st, A);
    return hipGetLastError();
}

}  // namespace nz
