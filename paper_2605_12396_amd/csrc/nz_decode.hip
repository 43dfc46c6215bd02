// nz_decode.hip -- gfx950 kernels of the receiver side: validate stream and frame headers, rebuild the
// canonical decode table from the code lengths carried in the frame, decode one 256-symbol segment per
// thread from its recorded bit offset, then dequantize (decompress), or -- front end of the fused reduce --
// stage the codes of operand A (first pass) and add operand B to them while gathering the statistics of the
// sum (second pass).  One operand per pass keeps the per-workgroup shared memory small enough for four
// waves per SIMD in every pass.
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
    const uint32_t chunk = h[4], nfr = h[5], stepb = h[6], seg = h[7], K = h[8], pred = h[9];
    total = (uint64_t)h[10] | ((uint64_t)h[11] << 32);
    if (n == 0 || chunk == 0 || chunk > kMaxChunk) return ST_CORRUPT;
    if (seg < 32u || seg > 1024u) return ST_CORRUPT;
    if (K < 2u || K > kMaxK || (K & (K - 1u))) return ST_CORRUPT;
    if (pred > 1u) return ST_CORRUPT;
    if ((n + chunk - 1) / chunk != (uint64_t)nfr) return ST_CORRUPT;
    if (total > bytes || total < kStreamHdr + pad16d(8ull * nfr)) return ST_CORRUPT;
    if (n != A.n || stepb != A.step_bits) return ST_MISMATCH;
    if (chunk != A.chunk || K != A.K || seg != kSeg || pred != A.pred) return ST_MISMATCH;
    return ST_OK;
}

// Shared memory of one operand's decoder.
constexpr uint32_t kRun = 8;                   // symbols per run: window reloads happen at run starts only
constexpr uint32_t kSubBits = 6;               // second-level tables resolve codes of 12..17 bits
constexpr uint32_t kMaxSub = 32;               // at most this many second-level tables (the rest: canonical search)

struct DecTables {
    uint16_t tab[1u << kPrimaryBits];
    uint16_t tab2[kMaxSub << kSubBits];
    uint16_t sorted[kMaxK];
    uint16_t sub_prefix[kMaxSub];
    uint32_t cnt[32], first[32], idx0[32];
    __align__(16) uint32_t lim[32];            // lim[l]: end of the codes of length <= l, left-justified to 28 bits
    int32_t base[32];                          // base[l] = idx0[l] - first[l]: sorted index = (code of length l) + base[l]
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
    bool dense;               // HUFFMAN: 6 or more bits per symbol on average (the window is renewed every run, not every phase)
    bool hot_esc;             // escapes are frequent in this frame (short escape code / codes wider than the alphabet)
};

// Build-time scratch shared by both operands.
struct BuildScratch {
    __align__(4) uint8_t len[kMaxK];
    uint16_t rank[kMaxK];
    uint32_t wcnt[16 * 32];
    uint32_t red[5][8];
};

// Sums over the workgroup of five 32-bit values (the caller keeps every total below 2^32): wave totals over the DPP
// network (no shared-memory crossbar), one barrier pair for all of them.
template <int NT>
__device__ inline void block_sum32x5(uint32_t (&v)[5], uint32_t (*s_red)[8]) {
    static_assert(NT / 64 <= 8, "one slot per wavefront");
#pragma unroll
    for (int k = 0; k < 5; k++) v[k] = wave_incl_scan_dpp(v[k]);          // lane 63: the wave's total
    __syncthreads();
    if (lane_id() == 63) {
#pragma unroll
        for (int k = 0; k < 5; k++) s_red[k][threadIdx.x >> 6] = v[k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 5; k++) { v[k] = 0; for (int i = 0; i < NT / 64; i++) v[k] += s_red[k][i]; }
}

// Validate one frame and prepare its decoder (all threads of the workgroup call this together).
template <int NT>
__device__ inline void open_frame(const uint8_t* s, uint64_t total, uint64_t off, uint64_t bytes, uint32_t nf, uint32_t first_seg,
                                  const DecodeArgs& A, DecTables* T, BuildScratch* B, FrameView& V) {
    // off: the frame's entry of the offsets table, read by the caller at kernel start; bytes: size of the stream buffer
    // (total <= bytes was checked with the stream header), the bound of the early read of the code lengths below
    const uint32_t tid = threadIdx.x;
    V.status = ST_CORRUPT; V.kind = KIND_ZERO; V.w = 0; V.words = nullptr; V.nwords = 0; V.segt = nullptr; V.seg_prefix = 0; V.dense = false;
    V.hot_esc = false;
    if ((off & 15u) || off < kStreamHdr + pad16d(8ull * A.n_frames) || off + kHdrBytes > total) return;
    const uint8_t* fr = s + off;
    const uint4 h0 = reinterpret_cast<const uint4*>(fr)[0], h1 = reinterpret_cast<const uint4*>(fr)[1];
    // the code-length table of a HUFFMAN frame starts right behind the header: its words are requested together with
    // the header (inside the stream buffer; used only once the header has shown that they belong to the table)
    const uint32_t lens_word = (off + kHdrBytes + 4ull * tid + 4ull <= bytes) ? reinterpret_cast<const uint32_t*>(fr + kHdrBytes)[tid] : 0u;
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
        if (p0 > 32u || (p1 & 0x7FFFFFFFu) || (p1 >> 31) != A.pred) return;   // (the stream's predictor is the caller's: checked before)
        const uint64_t need = 4ull * (((uint64_t)nf * p0 + 31u) / 32u);
        if (payload != need) return;
        V.status = ST_OK; V.kind = KIND_FIXED; V.w = p0; V.hot_esc = (p0 >= 32u) || ((1u << p0) > A.K);
        V.words = reinterpret_cast<const uint32_t*>(pay); V.nwords = payload / 4;
        return;
    }
    // HUFFMAN
    const uint32_t nsym = p0, seg = p1 & 0xFFFFu, K = (p1 >> 16) & 0x7FFFu;
    if ((p1 >> 31) != A.pred) return;
    if (seg != kSeg || K != A.K || nsym == 0 || nsym > K) return;
    const uint32_t nseg = (nf + kSeg - 1) / kSeg;
    const uint64_t tables = pad4d(nsym) + pad4d(2ull * nseg);
    if (payload < tables || (payload & 3u)) return;
    const uint16_t* segt = reinterpret_cast<const uint16_t*>(pay + pad4d(nsym));
    // code lengths (4 per thread): <= 28, padding zero, at least one used, Kraft sum <= 1
    static_assert(NT * 4 >= kMaxK, "one pass over the code lengths");
    uint32_t bad = 0;
    uint64_t kraft = 0;
    {
        const uint32_t lw = (4u * tid < (uint32_t)pad4d(nsym)) ? lens_word : 0u;
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
    // workgroup sums: the Kraft sum in two halves (a thread adds at most 4 x 2^27: the low 16 bits and the rest each
    // sum to less than 2^32 over the workgroup), the bits of the whole frame and those before this workgroup (a segment
    // has at most 65535 bits, a frame at most 4096 segments), and the number of threads that saw something illegal
    uint32_t sums[5] = { (uint32_t)(kraft & 0xFFFFu), (uint32_t)(kraft >> 16), all, pre, bad };
    block_sum32x5<NT>(sums, B->red);
    kraft = (uint64_t)sums[0] + ((uint64_t)sums[1] << 16);
    const uint64_t pre_bits = sums[3], all_bits = sums[2];
    if (sums[4] || kraft == 0 || kraft > (1ull << kMaxLen)) return;
    const uint64_t avail = 8ull * (payload - tables);
    if (all_bits > avail || 4ull * ((all_bits + 31u) / 32u) != payload - tables) return;
    if (all_bits < nf) return;            // every symbol costs at least one bit (so the bitstream is never empty here)
    // canonical tables and the first-level lookup
    uint32_t* s_cnt = T->cnt; uint32_t* s_first = T->first; uint32_t* s_idx0 = T->idx0;
    canonical_tables<NT>(B->len, K, B->wcnt, s_cnt, s_first, s_idx0, B->rank);
    for (uint32_t sy = tid; sy < K; sy += NT) {
        const uint32_t L = B->len[sy];
        if (L) T->sorted[s_idx0[L] + B->rank[sy]] = (uint16_t)sy;
    }
    if (tid == 0) T->nsub = 0;
    if (tid < 32) {
        T->lim[tid] = (tid >= 1 && tid <= kMaxLen) ? ((s_first[tid] + s_cnt[tid]) << (kMaxLen - tid)) : 0u;
        T->base[tid] = (int32_t)s_idx0[tid] - (int32_t)s_first[tid];
    }
    __syncthreads();
    // Entry formats (16 bits).  First level, indexed by the next 11 stream bits:
    //   (q & 1023) | L<<10   symbol with quantization code q (10-bit two's complement) and an L <= 11 bit code
    //   0x8000 | L<<10       escape symbol with an L-bit code (32 raw bits follow)
    //   0xC000 | id          no code of <= 11 bits starts here; id < kMaxSub: second-level table, else range compare
    // Second level, indexed by stream bits 11..16: same with L-11 in place of L; 0xC000 = longer still.
    // Canonical codes left-justified to a common width are ordered by length, so the length of the code that
    // starts an entry's bits is found by comparing against the end of every length's range (no table walk).
    {
        uint32_t lim[kPrimaryBits + 1];                                // end of the codes of length <= l, 11-bit scale
#pragma unroll
        for (uint32_t l = 1; l <= kPrimaryBits; l++) lim[l] = (s_first[l] + s_cnt[l]) << (kPrimaryBits - l);
        // a thread's entries in three sweeps (lengths and sorted positions, symbols, entries), so that the shared-memory
        // reads of all of them are in flight together
        constexpr uint32_t EPT = (1u << kPrimaryBits) / NT;
        uint32_t LL[EPT], pos[EPT], sym[EPT];
        bool has[EPT];
        // A thread's entries i = tid + k NT differ in their top bits only, so their prefixes v = reversed(i) share all but
        // the lowest log2(EPT) bits: the limits of the short lengths are multiples of EPT and compare alike for all of
        // them (counted once), only the last lengths are compared entry by entry.
        constexpr uint32_t kLowBits = (EPT == 8) ? 3u : ((EPT == 4) ? 2u : 0u);     // log2(EPT) for the workgroup sizes in use
        static_assert(EPT == 8 || EPT == 4, "entries per thread");
        const uint32_t vhigh = __brev(tid) >> (32 - kPrimaryBits);                  // prefix of entry k = 0 (low bits zero)
        uint32_t Lshared = 1;
#pragma unroll
        for (uint32_t l = 1; l + kLowBits <= kPrimaryBits; l++) Lshared += (vhigh >= lim[l]) ? 1u : 0u;   // lim[l] is a multiple of 2^(11-l)
#pragma unroll
        for (uint32_t k = 0; k < EPT; k++) {
            const uint32_t i = tid + k * NT;
            const uint32_t v = __brev(i) >> (32 - kPrimaryBits);       // stream order: first bit is the code's MSB
            uint32_t L = Lshared;
#pragma unroll
            for (uint32_t l = kPrimaryBits - kLowBits + 1; l < kPrimaryBits; l++) L += (v >= lim[l]) ? 1u : 0u;
            LL[k] = L; has[k] = v < lim[kPrimaryBits];
            pos[k] = has[k] ? (uint32_t)((int32_t)(v >> (kPrimaryBits - L)) + T->base[L]) : 0u;
        }
#pragma unroll
        for (uint32_t k = 0; k < EPT; k++) sym[k] = T->sorted[pos[k]];
#pragma unroll
        for (uint32_t k = 0; k < EPT; k++) {
            const uint32_t i = tid + k * NT, L = LL[k], sy = sym[k];
            uint32_t e = 0xC000u;
            if (has[k]) e = sy ? (((uint32_t)unzigzag(sy - 1u) & 1023u) | (L << 10)) : (0x8000u | (L << 10));
            else {
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
    V.status = ST_OK; V.kind = KIND_HUFF; V.segt = segt; V.seg_prefix = pre_bits;
    V.dense = all_bits >= 6ull * nf;
    V.hot_esc = B->len[0] != 0 && B->len[0] <= 6u;                   // the escape symbol has a probability of a percent or more
    V.words = reinterpret_cast<const uint32_t*>(pay + tables); V.nwords = (uint32_t)((payload - tables) / 4);
}

// Per-thread sequential reader of one HUFFMAN segment.  Every lane owns a small window (kWinWords words) in
// LDS, filled from global memory with dword-aligned 16-byte loads starting at the word the lane is in.  The
// window is renewed at the start of every phase of 32 symbols (requested before the workgroup's output phase,
// installed after it), and by a single lane at the start of a run of 8 symbols when it is kWinRunLimit or more
// bits into its window; a lane also reloads at once when a long code or an escape leaves it kWinSlowLimit or
// more bits into the window.
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

template <int NT>
struct HuffReader {
    uint64_t bits_addr;                  // byte address of bitstream word 0
    uint32_t nwords;                     // words in the bitstream (at least 1)
    uint32_t* win;                       // this lane's window in LDS (word j at win[j * NT])
    int32_t win_bit0;                    // bit index (relative to bitstream bit 0) of window word 0
    uint32_t k, sh;                      // current position: bit sh (0..31) of window word k
    uint32_t lo, hi, n1, n2;             // window words k .. k+3
    uint32_t start_bit, bad;
    const DecTables* T;

    __device__ inline void init(const FrameView& V, const DecTables* tables, uint32_t bitpos, const void* safe16,
                                uint32_t* lane_window) {
        T = tables; bad = 0; win = lane_window; start_bit = bitpos;
        if (V.nwords == 0 || V.kind != KIND_HUFF) {                      // not a HUFFMAN frame: the reader is never used
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
                win[(4 * c + 0) * NT] = x[c].x; win[(4 * c + 1) * NT] = x[c].y;
                win[(4 * c + 2) * NT] = x[c].z; win[(4 * c + 3) * NT] = x[c].w;
            }
            lo = x[0].x; hi = x[0].y; n1 = x[0].z; n2 = x[0].w;
        } else {
            // near the end of the bitstream: word by word, indices clamped to the last word
            typedef const uint32_t __attribute__((address_space(1))) * wptr;
            wptr w = reinterpret_cast<wptr>(bits_addr);
            const uint32_t last = nwords - 1u;
#pragma unroll 1
            for (uint32_t j = 0; j < kWinWords; j++) win[j * NT] = w[wi + j < last ? wi + j : last];
            lo = win[0]; hi = win[NT]; n1 = win[2 * NT]; n2 = win[3 * NT];
        }
        win_bit0 = (int32_t)(cur & ~31u);
        k = 0; sh = cur & 31u;
    }
    // Scheduled refill in two halves, so that the global-load latency passes while the workgroup does something
    // else (its output phase): request() issues the loads for the window at the current position, install()
    // makes it the lane's window.  A lane too close to the end of the bitstream for 16-byte loads reads a
    // harmless 48 bytes in front of the bitstream instead and refills the slow way at install time.  Only readers
    // of an accepted HUFFMAN frame request windows; its bitstream (at least one word) is preceded by the 32-byte
    // frame header, at least 8 bytes of tables and the stream header, so those 48 bytes lie inside the stream.
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    struct Pending { u32x4 x[kWinWords / 4]; uint32_t cur; bool ok; };
    __device__ inline void request(Pending& P) const {
        typedef u32x4 u32x4_a4 __attribute__((aligned(4)));
        typedef const u32x4_a4 __attribute__((address_space(1))) * gptr;
        P.cur = (uint32_t)(win_bit0 + (int32_t)pos());
        const uint32_t wi = P.cur >> 5;
        P.ok = wi + kWinWords <= nwords;
        gptr p = reinterpret_cast<gptr>(P.ok ? bits_addr + 4ull * wi : bits_addr - 4ull * kWinWords);
#pragma unroll
        for (uint32_t c = 0; c < kWinWords / 4; c++) P.x[c] = p[c];
    }
    __device__ inline void install(const Pending& P) {
        if (__builtin_expect(P.ok, 1)) {
#pragma unroll
            for (uint32_t c = 0; c < kWinWords / 4; c++) {
                win[(4 * c + 0) * NT] = P.x[c].x; win[(4 * c + 1) * NT] = P.x[c].y;
                win[(4 * c + 2) * NT] = P.x[c].z; win[(4 * c + 3) * NT] = P.x[c].w;
            }
            lo = P.x[0].x; hi = P.x[0].y; n1 = P.x[0].z; n2 = P.x[0].w;
            win_bit0 = (int32_t)(P.cur & ~31u);
            k = 0; sh = P.cur & 31u;
        } else reload();
    }
    // install() for a window that was requested one run of symbols ago: the lane has moved on since, so its
    // position is re-expressed inside the new window and the four words at it are read back from the window.  A
    // lane that has outrun what the window can still serve refills on its own instead.
    __device__ inline void install_at(const Pending& P) {
        const uint32_t abs_pos = (uint32_t)(win_bit0 + (int32_t)pos());
        const uint32_t rel = abs_pos - (P.cur & ~31u);                   // P.cur <= abs_pos: positions only grow
        if (__builtin_expect(P.ok && rel < kWinRunLimit, 1)) {
#pragma unroll
            for (uint32_t c = 0; c < kWinWords / 4; c++) {
                win[(4 * c + 0) * NT] = P.x[c].x; win[(4 * c + 1) * NT] = P.x[c].y;
                win[(4 * c + 2) * NT] = P.x[c].z; win[(4 * c + 3) * NT] = P.x[c].w;
            }
            win_bit0 = (int32_t)(P.cur & ~31u);
            k = rel >> 5; sh = rel & 31u;
            const uint32_t* p = win + k * NT;
            lo = p[0]; hi = p[NT]; n1 = p[2 * NT]; n2 = p[3 * NT];
        } else reload();
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
        const uint32_t* p = win + k * NT;
        n1 = p[2 * NT]; n2 = p[3 * NT];
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
            } else {
                // Longer than 17 bits, unassigned, or no second-level table left: v = the next 28 stream bits as a
                // number, first bit most significant.  Canonical codes left-justified to 28 bits are ordered by
                // length, so the length is 12 + the number of lengths 12..27 whose range ends at or below v; the
                // symbol follows from the canonical order.  All limits are read at once (no dependent loop).
                uint32_t li = 0;
                asm volatile("" : "+v"(li));                             // keeps the limit reads inside this rare path
                const uint4* lp = reinterpret_cast<const uint4*>(T->lim + li);
                const uint4 l3 = lp[3], l4 = lp[4], l5 = lp[5], l6 = lp[6], l7 = lp[7];     // lim[12..31]
                const uint32_t v = __brev(w32) >> 4;
                static_assert(kPrimaryBits == 11 && kMaxLen == 28, "limits 12..27 are compared below");
                L = 12u + (v >= l3.x) + (v >= l3.y) + (v >= l3.z) + (v >= l3.w) + (v >= l4.x) + (v >= l4.y) + (v >= l4.z) + (v >= l4.w) +
                    (v >= l5.x) + (v >= l5.y) + (v >= l5.z) + (v >= l5.w) + (v >= l6.x) + (v >= l6.y) + (v >= l6.z) + (v >= l6.w);
                uint32_t sy = 1;
                if (v >= l7.x) { bad = 1; L = 1; }                       // no code starts with these bits
                else sy = T->sorted[(uint32_t)((int32_t)(v >> (kMaxLen - L)) + T->base[L])];
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

// The tile: 16-bit quantization codes, 32 per thread between two output phases, so that eight lanes write
// one thread's run of 32 consecutive elements together (a full 128-byte line of fp32 or int32 output).
constexpr uint32_t kTile16Stride = kTile16R + 2;     // halfwords per row: 17 words, an odd word stride

enum : int { MODE_DECOMPRESS = 0, MODE_STAGE_A = 1, MODE_ADD_B = 2, MODE_ADD_LOCAL = 3, MODE_ADD_LOCAL_SR = 4,
             MODE_ADD_LOCAL_PLAIN = 5, MODE_ACC = 6 };
// the adding passes: ADD_B adds the staged codes of operand A, ADD_LOCAL the rank's own fp32 data, quantized on the fly
// (ADD_LOCAL_SR: by the stochastic quantizer; ADD_LOCAL_PLAIN: without the statistics of the sums, for the sampled
// arbitration, which profiles a prefix of the staged sums instead)
#define NZ_LOCAL(M) ((M) == MODE_ADD_LOCAL || (M) == MODE_ADD_LOCAL_SR || (M) == MODE_ADD_LOCAL_PLAIN)
#define NZ_STATS(M) ((M) == MODE_ADD_B || (M) == MODE_ADD_LOCAL || (M) == MODE_ADD_LOCAL_SR)
#define NZ_ADDS(M) ((M) == MODE_ADD_B || (M) == MODE_ACC || NZ_LOCAL(M))
// the passes whose other operand is the staged running value (operand A of the two-stream reduce); ACC, the
// accumulating pass of the k-ary reduce, stages its sums in operand A's format again, without statistics
#define NZ_STAGED(M) ((M) == MODE_ADD_B || (M) == MODE_ACC)

// Shared memory of one decode workgroup.  The window comes first and the tile follows it directly: a reader's
// prefetch may touch up to two rows past its window, which then fall into the tile (valid shared
// memory, values never used).
template <int NT>
struct __align__(16) DecShared {
    uint32_t win[NT * kWinWords];
    union { uint16_t tile[NT * kTile16Stride]; BuildScratch build; } u;
    uint64_t wsum[NT / 64];
    uint32_t zmax[2], flags, cwide[2], lunq[2], ovf;
};

struct SegCtx {
    uint32_t tid, lane, first_seg, nf, cntseg, e0, blk0;
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


// Second reduce pass, one element the general way: fetch A, combine, stage the sum, count its symbol.
// The sums are staged for the encoder as 16-bit codes in c16 (message order), kWideMarker where a sum needs 32
// bits, which then sits in codes; a frame with a RAW operand keeps its fp32 sums in codes.  wide[h] is raised when
// half h of the workgroup's block holds a marker.
// In the ring-step pass the other operand is the rank's own fp32 message (`local`), quantized here; an element
// that cannot be quantized counts as code 0 and raises lunq[h]: its frame becomes RAW and is redone by k_fix_local.
struct AddCtx {
    StageA sa; uint32_t* codes; int16_t* c16; uint32_t* s_h; uint32_t* s_cwide; uint32_t* s_lunq;
    StageA so; bool acc;       // accumulating pass of the k-ary reduce: the sums go to this staging set, in operand A's format
    const float* local; float eb, inv;
    bool sr; SrKeys keys;      // stochastic local quantizer: draws by element offset from the workgroup's block
    bool stats;                // the pass gathers the statistics of the sums
    uint32_t ncs, copy, K; float step; bool a_raw, b_raw;
    __device__ inline void finish(const SegCtx& C, uint32_t i, uint32_t tb, uint32_t (&zmax)[2], uint32_t& overflow) const {
        const uint64_t g = C.f0 + i;
        const uint32_t h = (i - C.blk0) >> 16;
        uint32_t ta;
        if (local) {
            int32_t q;
            const bool okq = sr ? sr_quantize1(local[g], step, inv, keys.draw(i - C.blk0), q) : quantize1(local[g], eb, step, inv, q);
            if (!okq) s_lunq[h] = 1u;
            ta = (uint32_t)q;
        } else ta = sa.get(C.f0, C.nf, i, a_raw);
        if (acc) {
            if (a_raw || b_raw) { so.a32[g] = combine<true>(ta, a_raw, tb, b_raw, step, overflow); return; }
            uint32_t wide_seen = 0;
            so.put_code(C.f0, C.nf, i, (int32_t)combine<false>(ta, false, tb, false, step, overflow), wide_seen);
            if (wide_seen) s_cwide[h] = 1u;
            return;
        }
        if (a_raw || b_raw) { codes[g] = combine<true>(ta, a_raw, tb, b_raw, step, overflow); return; }
        const uint32_t t = combine<false>(ta, false, tb, false, step, overflow);
        const int32_t Q = (int32_t)t;
        if (Q > 32767 || Q <= kWideMarker) { c16[g] = (int16_t)kWideMarker; codes[g] = t; s_cwide[h] = 1u; }
        else c16[g] = (int16_t)Q;
        if (!stats) return;
        const uint32_t z = zigzag(Q);
        zmax[h] = z > zmax[h] ? z : zmax[h];
        atomicAdd(&s_h[h * 1024u + (bin_of(z, K) << ncs) + copy], 1u);
    }
};

// HUFFMAN frame: every thread decodes its 256-symbol segment 32 symbols at a time into its tile row; after a
// barrier the workgroup consumes the tile with coalesced accesses (eight lanes per row).
//   MODE_DECOMPRESS  dequantize and store fp32
//   MODE_STAGE_A     store the 16-bit codes
//   MODE_ADD_B       add the staged codes of A, store the sums as 16-bit codes, count their symbols per half of
//                    kHalf elements
//   MODE_ADD_LOCAL   the same with the rank's own fp32 data, quantized here, in the place of A
// A code that does not fit 16 bits (an escape with a large value) is finished by the decoding lane itself,
// which leaves kWideMarker in the tile and raises a workgroup flag; only then does the consumer look for
// markers.
// DELTA: the stream carries differences; the thread keeps the running sum of its segment (modulo 2^32) and a sum
// that does not fit 16 bits is finished by the decoding lane like a wide escape.
template <int MODE, int NT, int DELTA>
__device__ inline void run_huff(const DecodeArgs& A, const SegCtx& C, HuffReader<NT>& ra, DecShared<NT>* S, bool dense,
                                bool hot_esc, const AddCtx& X, bool a_wide, uint32_t (&zmax)[2], uint32_t& overflow) {
    const uint32_t tid = C.tid;
    uint16_t* tile = S->u.tile;
    uint32_t* row32 = reinterpret_cast<uint32_t*>(tile + tid * kTile16Stride);
    uint32_t e = 0;                                   // symbols of my segment decoded so far
    // Every phase starts with a fresh window: its loads are requested at the end of the phase before and
    // installed after the output phase in between, so their latency is not waited for.  Inside a phase a lane
    // refills on its own at a run start when it is too far into its window.
    typename HuffReader<NT>::Pending pend;
    ra.request(pend);
    auto start_run = [&]() { if (ra.pos() >= kWinRunLimit) ra.reload(); };
    auto wide_code = [&](int32_t q) -> int32_t {      // a code outside the tile's 16 bits: finished here, marked there
        if (MODE == MODE_DECOMPRESS) A.out[C.f0 + C.e0 + e] = dequantize1(q, A.step);
        else if (MODE == MODE_STAGE_A) X.sa.a32[C.f0 + C.e0 + e] = (uint32_t)q;
        else X.finish(C, C.e0 + e, (uint32_t)q, zmax, overflow);
        S->flags = 1u;
        return kWideMarker;
    };
    auto wide = [&](uint32_t z) -> int32_t {          // without a predictor only an escape can carry a code of 16 bits or more
        const int32_t q = unzigzag(z);
        if (DELTA) return q;
        return (z >= 0xFFFFu) ? wide_code(q) : q;
    };
    uint32_t acc = 0;                                 // DELTA: the code before this one (0 at the segment start)
    auto next16 = [&]() -> uint32_t {
        int32_t q = ra.next(wide);
        if (DELTA) {
            acc += (uint32_t)q; q = (int32_t)acc;
            if (__builtin_expect(q > 32767 || q <= kWideMarker, 0)) q = wide_code(q);
        }
        e++;
        return (uint32_t)q;
    };
    constexpr uint32_t LPR = kTile16R / 4;            // 8 lanes consume one row
    constexpr uint32_t RPK = NT / LPR;                // rows covered by one step k of the consumer
    // consumer: thread (row rw0 + RPK k, columns c .. c+3) for k = 0..7
    const uint32_t rw0 = tid / LPR, c = (tid % LPR) * 4;
    const uint32_t* src0 = reinterpret_cast<const uint32_t*>(tile + rw0 * kTile16Stride + c);
    const uint32_t eo0 = (C.first_seg + rw0) * kSeg + c;
    const bool whole = C.vec_ok && (C.first_seg + NT) * kSeg <= C.nf;   // every access is a full, aligned group of 4
    const bool fast_add = NZ_ADDS(MODE) && whole && !a_wide && !X.a_raw;
    for (uint32_t r0 = 0; r0 < kSeg; r0 += kTile16R) {
        // Instruction issue favours the wavefronts that were started first, so the workgroups that share a compute unit
        // would finish one after the other and leave it half empty towards the end of the kernel (there is nothing left
        // to start in their place).  A wavefront's priority falls as it gets through its segment, which lets the ones
        // that are behind catch up: the workgroups of a compute unit finish closer together.
        // (the levels get shorter towards the end -- phases 0-3, 4-5, 6, 7 -- so that the workgroups draw level at every
        // boundary and can only drift apart again inside the last phase)
        switch (r0 / kTile16R) {
            case 0: case 1: case 2: case 3: __builtin_amdgcn_s_setprio(3); break;
            case 4: case 5: __builtin_amdgcn_s_setprio(2); break;
            case 6: __builtin_amdgcn_s_setprio(1); break;
            default: __builtin_amdgcn_s_setprio(0); break;
        }
        ra.install(pend);
        uint2 pa[LPR];                                // MODE_ADD_B: the staged codes of A this thread will add
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        f32x4 pl[NZ_LOCAL(MODE) ? LPR : 1];           // ring step: the rank's own values this thread will add
        if (r0 + kTile16R <= C.cntseg) {
#pragma unroll
            for (uint32_t h = 0; h < kTile16R; h += kRun) {
                // dense frames (uniform over the workgroup): a phase uses up most of a window, so every run starts
                // with a window requested at the start of the run before it; the others only watch their margin
                if (dense && h > 0) ra.install_at(pend);
                start_run();
                if (dense && h + kRun < kTile16R) ra.request(pend);
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
        ra.request(pend);                             // (after the last phase: requested and dropped)
        __syncthreads();
        const bool plain = whole && S->flags == 0;    // no markers in the tile, no bounds to watch
        if (MODE == MODE_DECOMPRESS && __builtin_expect(plain, 1)) {
            float* dst = A.out + C.f0 + eo0 + r0;
#pragma unroll
            for (uint32_t k = 0; k < LPR; k++) {
                const uint32_t* src = src0 + k * RPK * (kTile16Stride / 2);
                const uint32_t p0 = src[0], p1 = src[1];
                // streaming store: the output is not read again here and should not displace the bitstream in L2
                typedef float f32x4 __attribute__((ext_vector_type(4)));
                f32x4 v;
                v.x = dequantize1((int32_t)(int16_t)(p0 & 0xFFFFu), A.step); v.y = dequantize1((int32_t)p0 >> 16, A.step);
                v.z = dequantize1((int32_t)(int16_t)(p1 & 0xFFFFu), A.step); v.w = dequantize1((int32_t)p1 >> 16, A.step);
                __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(dst + (size_t)k * RPK * kSeg));
            }
        } else if (MODE == MODE_STAGE_A && __builtin_expect(whole, 1)) {
            int16_t* dst = X.sa.a16 + C.f0 + C.blk0 + (r0 / kTile16R) * (kHalf / 8u) + rw0 * kTile16R + c;   // markers are staged as they are
#pragma unroll
            for (uint32_t k = 0; k < LPR; k++) {
                const uint32_t* src = src0 + k * RPK * (kTile16Stride / 2);
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                u32x2 v; v.x = src[0]; v.y = src[1];
                __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(dst + (size_t)k * RPK * kTile16R));   // streaming, as above
            }
        } else if (NZ_ADDS(MODE) && __builtin_expect(fast_add && plain, 1)) {
            int16_t* dst = X.c16 + C.f0 + eo0 + r0;
            // the other operand is requested here rather than across the decode phase (no registers held, no spills);
            // the other workgroup of the CU covers the wait
            if (NZ_STAGED(MODE)) {
                // row rw0 + RPK k of this block, phase r0 / 32 (both halves are full here)
                const int16_t* ap = X.sa.a16 + C.f0 + C.blk0 + (r0 / kTile16R) * (kHalf / 8u) + c;
#pragma unroll
                for (uint32_t k = 0; k < LPR; k++) {
                    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                    const uint32_t rw = rw0 + k * RPK;
                    const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(
                        ap + (size_t)(rw / kSeg) * kHalf + (rw % kSeg) * kTile16R));
                    pa[k] = make_uint2(v.x, v.y);
                }
            }
            if (NZ_LOCAL(MODE)) {
                const float* lp = X.local + C.f0 + eo0 + r0;
#pragma unroll
                for (uint32_t k = 0; k < LPR; k++)
                    pl[k] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(lp + (size_t)k * RPK * kSeg));
            }
#pragma unroll
            for (uint32_t k = 0; k < LPR; k++) {
                const uint32_t* src = src0 + k * RPK * (kTile16Stride / 2);
                const uint32_t p0 = src[0], p1 = src[1];
                const uint32_t h = (k * RPK >= kHalf / kSeg) ? 1u : 0u;       // which half of the block this row is in
                int32_t Q[4];
                if (NZ_LOCAL(MODE)) {
                    // quantize the rank's own values; one that cannot be quantized counts as 0 and flags its half
                    int32_t ql[4];
                    const float xl[4] = { pl[k].x, pl[k].y, pl[k].z, pl[k].w };
                    bool ok = true;
                    const uint32_t off = eo0 + r0 + k * RPK * kSeg - C.blk0;      // element offset inside the workgroup's block
#pragma unroll
                    for (uint32_t j = 0; j < 4; j++)
                        ok = (MODE == MODE_ADD_LOCAL_SR ? sr_quantize1(xl[j], X.step, X.inv, X.keys.draw(off + j), ql[j])
                                                        : quantize1(xl[j], X.eb, X.step, X.inv, ql[j])) && ok;
                    if (!ok) X.s_lunq[h] = 1u;
                    Q[0] = (int32_t)(int16_t)(p0 & 0xFFFFu) + ql[0]; Q[1] = ((int32_t)p0 >> 16) + ql[1];
                    Q[2] = (int32_t)(int16_t)(p1 & 0xFFFFu) + ql[2]; Q[3] = ((int32_t)p1 >> 16) + ql[3];
                } else {
                Q[0] = (int32_t)(int16_t)(p0 & 0xFFFFu) + (int32_t)(int16_t)(pa[k].x & 0xFFFFu);
                Q[1] = ((int32_t)p0 >> 16) + ((int32_t)pa[k].x >> 16);
                Q[2] = (int32_t)(int16_t)(p1 & 0xFFFFu) + (int32_t)(int16_t)(pa[k].y & 0xFFFFu);
                Q[3] = ((int32_t)p1 >> 16) + ((int32_t)pa[k].y >> 16);
                }
                if (!NZ_STATS(MODE)) {
                    // (no statistics in this pass)
                } else if (hot_esc) {
                    // Where escapes are frequent (sums of many peers: most codes leave the alphabet) they all hit one
                    // bin, whose few copies serialise the wave.  They are counted per wavefront and added once; the
                    // whole wave is here and h is the same for all of it.  (Uniform branch: the incoming frame's kind.)
                    uint32_t wave_esc = 0;
#pragma unroll
                    for (uint32_t j = 0; j < 4; j++) {
                        const uint32_t z = zigzag(Q[j]);
                        zmax[h] = z > zmax[h] ? z : zmax[h];
                        const bool esc = z >= X.K - 1u;
                        wave_esc += (uint32_t)__builtin_popcountll(__ballot(esc));
                        if (!esc) atomicAdd(&X.s_h[h * 1024u + (z << X.ncs) + X.copy], 1u);
                    }
                    if (C.lane == 0 && wave_esc) atomicAdd(&X.s_h[h * 1024u + ((X.K - 1u) << X.ncs)], wave_esc);
                } else {
#pragma unroll
                    for (uint32_t j = 0; j < 4; j++) {
                        const uint32_t z = zigzag(Q[j]);
                        zmax[h] = z > zmax[h] ? z : zmax[h];
                        atomicAdd(&X.s_h[h * 1024u + (bin_of(z, X.K) << X.ncs) + X.copy], 1u);
                    }
                }
                // operands of 16 bits (|q| <= 32767 from the quantizer too): |Q| <= 65534; a sum outside the 16-bit codes
                // is rare and goes to the 32-bit array
                const int32_t qhi = max(max(Q[0], Q[1]), max(Q[2], Q[3])), qlo = min(min(Q[0], Q[1]), min(Q[2], Q[3]));
                uint32_t w0 = ((uint32_t)Q[0] & 0xFFFFu) | ((uint32_t)Q[1] << 16), w1 = ((uint32_t)Q[2] & 0xFFFFu) | ((uint32_t)Q[3] << 16);
                if (__builtin_expect(qhi > 32767 || qlo <= kWideMarker, 0)) {
                    uint32_t* c32 = (MODE == MODE_ACC ? X.so.a32 : X.codes) + C.f0 + eo0 + r0 + (size_t)k * RPK * kSeg;
                    uint32_t hw[4];
#pragma unroll
                    for (uint32_t j = 0; j < 4; j++) {
                        const bool wd = Q[j] > 32767 || Q[j] <= kWideMarker;
                        if (wd) c32[j] = (uint32_t)Q[j];
                        hw[j] = wd ? (uint32_t)(uint16_t)kWideMarker : ((uint32_t)Q[j] & 0xFFFFu);
                    }
                    w0 = hw[0] | (hw[1] << 16); w1 = hw[2] | (hw[3] << 16);
                    X.s_cwide[h] = 1u;
                }
                typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
                u32x2 v; v.x = w0; v.y = w1;
                if (MODE == MODE_ACC) {
                    // the running value keeps operand A's phase-major layout: the position the codes of A came from
                    const uint32_t rw = rw0 + k * RPK;
                    int16_t* ad = X.so.a16 + C.f0 + C.blk0 + (r0 / kTile16R) * (kHalf / 8u) + c + (size_t)(rw / kSeg) * kHalf + (rw % kSeg) * kTile16R;
                    *reinterpret_cast<u32x2*>(ad) = v;
                } else
                __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(dst + (size_t)k * RPK * kSeg));   // streaming, as above
            }
        } else {
            // ragged block, markers in the tile, wide or raw codes of A: element by element
#pragma unroll 1
            for (uint32_t k = 0; k < LPR; k++) {
                const uint32_t eo = eo0 + k * RPK * kSeg + r0;                    // element index in the frame
                const uint16_t* src = tile + (rw0 + k * RPK) * kTile16Stride + c;
                for (uint32_t j = 0; j < 4; j++) {
                    if (eo + j >= C.nf) break;
                    const int32_t q = (int16_t)src[j];
                    if (MODE == MODE_STAGE_A) X.sa.a16[StageA::at16(C.f0, C.nf, eo + j)] = (int16_t)q;
                    else if (q != kWideMarker) {
                        if (MODE == MODE_DECOMPRESS) A.out[C.f0 + eo + j] = dequantize1(q, A.step);
                        else X.finish(C, eo + j, (uint32_t)q, zmax, overflow);
                    }
                }
            }
        }
        __syncthreads();
    }
}

// RAW frames and rejected frames (= all zero): element-parallel.
template <int MODE, int NT>
__device__ inline void run_elementwise(const DecodeArgs& A, const SegCtx& C, const DirectFetch& da, DecShared<NT>* S,
                                       const AddCtx& X, uint32_t (&zmax)[2], uint32_t& overflow) {
    const uint32_t cnt = (C.nf - C.blk0 < NT * kSeg) ? (C.nf - C.blk0) : NT * kSeg;
    const bool raw = da.kind == KIND_RAW;
    uint32_t wide_seen = 0;
    for (uint32_t i = C.tid * 4; i < cnt; i += NT * 4) {
        const uint32_t m = (cnt - i < 4) ? (cnt - i) : 4u;
        if (MODE == MODE_DECOMPRESS && raw && m == 4u && C.vec_ok) {      // a RAW frame is a copy (payload and output 16-byte aligned)
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(da.words + C.blk0 + i));
            __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(A.out + C.f0 + C.blk0 + i));
            continue;
        }
        for (uint32_t j = 0; j < m; j++) {
            const uint32_t e = C.blk0 + i + j;
            uint32_t t = da.get(e);                                               // fp32 bits (RAW) or zero
            if (!raw) t = (uint32_t)unzigzag(t);
            if (MODE == MODE_DECOMPRESS) A.out[C.f0 + e] = raw ? __uint_as_float(t) : dequantize1((int32_t)t, A.step);
            else if (MODE == MODE_STAGE_A) { if (raw) X.sa.a32[C.f0 + e] = t; else X.sa.put_code(C.f0, C.nf, e, (int32_t)t, wide_seen); }
            else X.finish(C, e, t, zmax, overflow);
        }
    }
    if (MODE == MODE_STAGE_A && wide_seen) S->flags = 1u;
}

// FIXEDLEN frames, the streaming way: a pass of NT * 4 elements is NT * w / 8 whole words of the payload (at a 16-byte
// boundary), which the workgroup copies into shared memory with 16-byte loads (the next pass's words are requested
// before this pass is worked on); every thread then cuts its four consecutive codes out of the copy.  Two copies
// alternate (they live in the window area, which only HUFFMAN frames use), so one barrier per pass is enough.
// DELTA: the running sums of a segment are a scan over the wavefront that holds it.
template <int MODE, int NT, int DELTA>
__device__ inline void run_fixed(const DecodeArgs& A, const SegCtx& C, const FrameView& V, DecShared<NT>* S,
                                 const AddCtx& X, uint32_t (&zmax)[2], uint32_t& overflow) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    constexpr uint32_t kPass = NT * 4;                                   // elements per pass
    static_assert(2 * (kPass + 8) <= NT * kWinWords, "two pass copies fit the window area");
    const uint32_t cnt = (C.nf - C.blk0 < NT * kSeg) ? (C.nf - C.blk0) : NT * kSeg;
    const uint32_t w = V.w, tid = C.tid;
    const uint32_t mask = (w >= 32u) ? 0xFFFFFFFFu : ((1u << w) - 1u);
    const uint32_t pass_words = (kPass / 32u) * w;                       // words of a whole pass (at most kPass)
    uint32_t wide_seen = 0;
    // words [4 tid, 4 tid + 4) of the pass that starts at element `base` of the block (zero where the payload ends)
    auto fetch = [&](uint32_t base) -> u32x4 {
        u32x4 x = { 0u, 0u, 0u, 0u };
        if (base >= cnt) return x;
        const uint32_t g0 = ((C.blk0 + base) >> 5) * w + 4u * tid;        // first of my words in the payload
        if (4u * tid >= pass_words || g0 >= V.nwords) return x;
        if (g0 + 4u <= V.nwords) return *reinterpret_cast<const u32x4*>(V.words + g0);
        x.x = V.words[g0];
        if (g0 + 1u < V.nwords) x.y = V.words[g0 + 1u];
        if (g0 + 2u < V.nwords) x.z = V.words[g0 + 2u];
        return x;
    };
    u32x4 nxt = fetch(0);
    uint32_t it = 0;
    for (uint32_t base = 0; base < cnt; base += kPass, it++) {
        uint32_t* buf = S->win + (it & 1u) * (kPass + 8u);
        *reinterpret_cast<u32x4*>(buf + 4u * tid) = nxt;
        nxt = fetch(base + kPass);
        __syncthreads();
        const uint32_t i = base + tid * 4u;
        const uint32_t m = (i < cnt) ? ((cnt - i < 4u) ? (cnt - i) : 4u) : 0u;
        uint32_t tv[4];
        uint32_t pos = tid * 4u * w;
#pragma unroll
        for (uint32_t j = 0; j < 4; j++) {
            const uint32_t k = pos >> 5;                                  // (k + 1 <= kPass + 3: inside the copy's slack)
            tv[j] = (uint32_t)unzigzag(__builtin_amdgcn_alignbit(buf[k + 1u], buf[k], pos & 31u) & mask);
            pos += w;
        }
        if (DELTA) {
#pragma unroll
            for (uint32_t j = 0; j < 4; j++) if (j >= m) tv[j] = 0;       // (elements past the end add nothing)
            tv[1] += tv[0]; tv[2] += tv[1]; tv[3] += tv[2];
            const uint32_t before = wave_incl_scan_dpp(tv[3]) - tv[3];
            tv[0] += before; tv[1] += before; tv[2] += before; tv[3] += before;
        }
        if (MODE == MODE_DECOMPRESS && m == 4u && C.vec_ok) {
            f32x4 v;
            v.x = dequantize1((int32_t)tv[0], A.step); v.y = dequantize1((int32_t)tv[1], A.step);
            v.z = dequantize1((int32_t)tv[2], A.step); v.w = dequantize1((int32_t)tv[3], A.step);
            __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(A.out + C.f0 + C.blk0 + i));
        } else {
            for (uint32_t j = 0; j < m; j++) {
                const uint32_t e = C.blk0 + i + j;
                if (MODE == MODE_DECOMPRESS) A.out[C.f0 + e] = dequantize1((int32_t)tv[j], A.step);
                else if (MODE == MODE_STAGE_A) X.sa.put_code(C.f0, C.nf, e, (int32_t)tv[j], wide_seen);
                else X.finish(C, e, tv[j], zmax, overflow);
            }
        }
    }
    if (MODE == MODE_STAGE_A && wide_seen) S->flags = 1u;
}

// One workgroup per NT segments of one frame.
template <int MODE, int NT, int DELTA>
__global__ __launch_bounds__(NT) __attribute__((amdgpu_waves_per_eu(4))) void k_decode(DecodeArgs A) {
    __shared__ DecTables s_t;
    __shared__ DecShared<NT> S;
    __shared__ uint32_t s_h[NZ_STATS(MODE) ? 2048 : 1];

    const uint32_t tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const uint32_t frame = blockIdx.x / A.dbpf, db = blockIdx.x % A.dbpf;
    const uint64_t f0 = (uint64_t)frame * A.chunk;
    const uint32_t nf = (uint32_t)((A.n - f0 < A.chunk) ? (A.n - f0) : A.chunk);
    const uint32_t blk0 = db * NT * kSeg;
    if (blk0 >= nf) return;
    ResultRec* res = reinterpret_cast<ResultRec*>(A.res);
    const uint32_t first_seg = db * NT;
    const uint32_t nseg = (nf + kSeg - 1) / kSeg;
    const uint32_t gseg = first_seg + tid;
    const bool seg_valid = gseg < nseg;
    const uint32_t e0 = gseg * kSeg;                                    // first element of my segment in the frame
    const uint32_t cntseg = seg_valid ? ((nf - e0 < kSeg) ? (nf - e0) : kSeg) : 0u;
    const uint32_t hpf = (A.chunk + kHalf - 1) / kHalf;                 // halves (statistics blocks) per frame

    // the frame's entry of the offsets table is requested before the stream header is looked at (its place does not
    // depend on the header; the entry is only believed once the header is)
    uint64_t frame_off = 0;
    {
        const uint8_t* sp = NZ_STAGED(MODE) ? A.b : A.a;
        const uint64_t sb = NZ_STAGED(MODE) ? A.b_bytes : A.a_bytes;
        if (kStreamHdr + 8ull * frame + 8ull <= sb) frame_off = *reinterpret_cast<const uint64_t*>(sp + kStreamHdr + 8ull * frame);
    }
    // stream headers: the reduce passes look at both operands, so that neither goes on after a stream-level error
    uint64_t total_a = 0, total_b = 0;
    const uint32_t st_a = check_stream(A.a, A.a_bytes, A, total_a);
    uint32_t st_b = ST_OK;
    if (MODE == MODE_STAGE_A || NZ_STAGED(MODE)) st_b = check_stream(A.b, A.b_bytes, A, total_b);
    // decompress: one verdict word per workgroup (status | kind << 8), summed up by k_decode_finish; nothing here
    // touches the result record.  The reduce passes report through the (pre-cleared) record with atomics.
    uint32_t* verdict = reinterpret_cast<uint32_t*>(A.ws + A.L.pmeta);
    if (MODE != MODE_DECOMPRESS && blockIdx.x == 0 && tid == 0) {
        if (st_a) atomicMax(&res->status, st_a);
        if (st_b) atomicMax(&res->status, st_b);
    }
    if (MODE == MODE_DECOMPRESS && st_a) {                              // nothing is written on a stream-level error
        if (tid == 0) verdict[blockIdx.x] = st_a;
        return;
    }

    FrameView V;
    V.status = ST_OK; V.kind = KIND_ZERO; V.w = 0; V.words = nullptr; V.nwords = 0; V.segt = nullptr; V.seg_prefix = 0; V.dense = false;
    V.hot_esc = false;
    if (st_a == ST_OK && st_b == ST_OK) {
        open_frame<NT>(NZ_STAGED(MODE) ? A.b : A.a, NZ_STAGED(MODE) ? total_b : total_a, frame_off,
                       NZ_STAGED(MODE) ? A.b_bytes : A.a_bytes, nf, first_seg, A, &s_t, &S.u.build, V);
        if (MODE != MODE_DECOMPRESS && tid == 0 && V.status) atomicMax(&res->status, V.status);
    }
    const uint32_t found_kind = V.kind;
    if (V.status) V.kind = KIND_ZERO;                                   // a rejected frame counts as zeros (and decodes to zeros)

    // bit offset of my segment inside a HUFFMAN bitstream: prefix of the segment table
    uint32_t bit0 = 0, seglen = 0;
    {
        seglen = (V.kind == KIND_HUFF && seg_valid) ? V.segt[gseg] : 0u;
        const uint32_t incl = wave_incl_scan_dpp(seglen);
        if (lane == 63) S.wsum[wave] = incl;
        if (tid == 0) { S.zmax[0] = 0; S.zmax[1] = 0; S.flags = 0; S.cwide[0] = 0; S.cwide[1] = 0; S.lunq[0] = 0; S.lunq[1] = 0; S.ovf = 0; }
        __syncthreads();
        uint32_t excl = incl - seglen;
        for (uint32_t w = 0; w < wave; w++) excl += (uint32_t)S.wsum[w];
        bit0 = (uint32_t)V.seg_prefix + excl;
    }
    const uint32_t* safe = reinterpret_cast<const uint32_t*>(A.res);
    HuffReader<NT> ra;
    DirectFetch da;
    ra.init(V, &s_t, bit0, safe, &S.win[tid]);
    da.init(V, safe);
    SegCtx C;
    C.tid = tid; C.lane = lane; C.first_seg = first_seg; C.nf = nf; C.cntseg = cntseg; C.e0 = e0; C.f0 = f0; C.blk0 = blk0;
    C.vec_ok = ((f0 & 3u) == 0);
    uint32_t overflow = 0;
    uint32_t zmax[2] = { 0, 0 };

    // Two staging sets in operand A's format: set 0 = (a16, a32, akind, awide), set 1 = the arrays of the sums (c16,
    // codes) with flag arrays of its own.  The two-stream reduce only knows set 0.  In the k-ary reduce the running
    // value alternates: the staging pass writes set A.set_in, an accumulating pass reads set A.set_in and writes the
    // other one, and the last accumulating pass ends in set 0, where the statistics pass (ADD_B) reads operand A
    // while it writes the sums in their own format to c16 / codes.
    const uint32_t si = (MODE == MODE_STAGE_A || MODE == MODE_ACC) ? (A.set_in & 1u) : 0u;
    AddCtx X;
    X.sa.a16 = reinterpret_cast<int16_t*>(A.ws + (si ? A.L.c16 : A.L.a16)); X.sa.a32 = reinterpret_cast<uint32_t*>(A.ws + (si ? A.L.codes : A.L.a32));
    X.so.a16 = reinterpret_cast<int16_t*>(A.ws + (si ? A.L.a16 : A.L.c16)); X.so.a32 = reinterpret_cast<uint32_t*>(A.ws + (si ? A.L.a32 : A.L.codes));
    X.acc = (MODE == MODE_ACC);
    X.codes = reinterpret_cast<uint32_t*>(A.ws + A.L.codes); X.c16 = reinterpret_cast<int16_t*>(A.ws + A.L.c16);
    X.s_cwide = S.cwide; X.s_lunq = S.lunq;
    X.local = NZ_LOCAL(MODE) ? A.local : nullptr; X.eb = A.eb; X.inv = A.inv_step;
    X.sr = (MODE == MODE_ADD_LOCAL_SR); X.stats = NZ_STATS(MODE);
    if (MODE == MODE_ADD_LOCAL_SR) X.keys.init(A.seed, f0 + blk0); else { X.keys.base_lo = 0; X.keys.key0 = 0; X.keys.key1 = 0; }
    X.s_h = s_h; X.K = A.K; X.step = A.step; X.ncs = 0; X.copy = 0; X.a_raw = false; X.b_raw = false;
    uint32_t* akind = reinterpret_cast<uint32_t*>(A.ws + (si ? A.L.akind1 : A.L.akind));   // per frame: operand A is RAW
    uint32_t* awide = reinterpret_cast<uint32_t*>(A.ws + (si ? A.L.awide1 : A.L.awide));   // per half: some code of A needs 32 bits
    uint32_t* akind_out = reinterpret_cast<uint32_t*>(A.ws + (si ? A.L.akind : A.L.akind1));   // (accumulating pass: the set it writes)
    uint32_t* awide_out = reinterpret_cast<uint32_t*>(A.ws + (si ? A.L.awide : A.L.awide1));
    bool a_wide = false;
    if (NZ_ADDS(MODE)) {
        while ((A.K << (X.ncs + 1)) <= 1024u && X.ncs < 5) X.ncs++;
        X.copy = lane & ((1u << X.ncs) - 1u);
        if (NZ_STATS(MODE)) for (uint32_t i = tid; i < 2048u; i += NT) s_h[i] = 0;
        X.b_raw = V.kind == KIND_RAW;
        if (NZ_STAGED(MODE)) {
            X.a_raw = akind[frame] != 0;
            for (uint32_t h = 0; h < NT * kSeg / kHalf; h++)
                if (blk0 + h * kHalf < nf) a_wide = a_wide || (awide[(size_t)frame * hpf + blk0 / kHalf + h] != 0);
        } else if (db == 0 && tid == 0) akind[frame] = X.b_raw ? 1u : 0u;   // ring step: "the incoming frame is RAW", for k_fix_local
        __syncthreads();
    }

    bool late = false;                                                  // a segment that did not use exactly its recorded bits
    if (V.kind == KIND_HUFF) {
        run_huff<MODE, NT, DELTA>(A, C, ra, &S, V.dense, V.hot_esc, X, a_wide, zmax, overflow);
        late = seg_valid && (ra.bad || ra.consumed() != seglen);
        if (MODE != MODE_DECOMPRESS && late) atomicMax(&res->status, (uint32_t)ST_CORRUPT);
    } else if (V.kind == KIND_FIXED) {
        run_fixed<MODE, NT, DELTA>(A, C, V, &S, X, zmax, overflow);
    } else {
        run_elementwise<MODE, NT>(A, C, da, &S, X, zmax, overflow);
    }
    if (MODE == MODE_DECOMPRESS) {
        // a frame found corrupt only now has been written already: k_decode_finish clears it again
        if (late) S.ovf = 1u;                                           // (cleared before the first barrier; otherwise unused here)
        __syncthreads();
        const uint32_t any_late = S.ovf;
        if (tid == 0) verdict[blockIdx.x] = (V.status ? V.status : (any_late ? (uint32_t)ST_CORRUPT : (uint32_t)ST_OK)) | (found_kind << 8);
        return;
    }

    if (MODE == MODE_STAGE_A) {
        static_assert(MODE != MODE_STAGE_A || NT * kSeg == kHalf, "the first reduce pass works in halves");
        __syncthreads();
        if (tid == 0) {
            awide[(size_t)frame * hpf + db] = S.flags;
            if (db == 0) akind[frame] = (V.kind == KIND_RAW) ? 1u : 0u;
        }
        return;
    }
    // ---- adding passes: statistics of the sum, per half ----
    // (a sum beyond 2^30 turns the whole frame RAW, which only k_fix can do once every workgroup of the frame is
    // done; the flag travels with the half's statistics)
    if (overflow) S.ovf = 1u;
#pragma unroll
    for (uint32_t h = 0; h < 2; h++) {
        const uint32_t zm = wave_max(zmax[h]);
        if (lane == 0 && zm) atomicMax(&S.zmax[h], zm);
    }
    __syncthreads();
    const bool out_raw = X.a_raw || X.b_raw;                            // uniform over the frame
    if (MODE == MODE_ACC) {
        // the running value's flags, in the set just written; the range flag goes where k_fix_acc looks for it
        if (tid == 0) {
            for (uint32_t h = 0; h < NT * kSeg / kHalf; h++) {
                if (blk0 + h * kHalf >= nf) break;
                const size_t hb = (size_t)frame * hpf + blk0 / kHalf + h;
                awide_out[hb] = S.cwide[h] ? 1u : 0u;
                reinterpret_cast<uint2*>(A.ws + A.L.pmeta)[hb] = make_uint2(0u, out_raw ? 1u : 0u);
                reinterpret_cast<uint32_t*>(A.ws + A.L.cwide)[hb] = S.ovf ? 2u : 0u;
            }
            if (db == 0) akind_out[frame] = out_raw ? 1u : 0u;
        }
        return;
    }
    for (uint32_t h = 0; h < NT * kSeg / kHalf; h++) {
        if (blk0 + h * kHalf >= nf) break;
        const size_t hb = (size_t)frame * hpf + blk0 / kHalf + h;
        uint32_t* ph = reinterpret_cast<uint32_t*>(A.ws + A.L.phist) + hb * kMaxK;
        if (NZ_STATS(MODE)) for (uint32_t sy = tid; sy < A.K; sy += NT) {
            uint32_t t = 0;
            for (uint32_t cc = 0; cc < (1u << X.ncs); cc++) t += s_h[h * 1024u + (sy << X.ncs) + cc];
            ph[bin_symbol(sy, A.K)] = t;
        }
        if (tid == 0) {
            // flag word: bit 0 = an operand frame is RAW, bit 1 = the local data of this half cannot be quantized
            reinterpret_cast<uint2*>(A.ws + A.L.pmeta)[hb] = make_uint2(S.zmax[h], (out_raw ? 1u : 0u) | (S.lunq[h] ? 2u : 0u));
            // bit 0 = the half holds sums that need 32 bits, bit 1 = a sum of this workgroup is out of range
            reinterpret_cast<uint32_t*>(A.ws + A.L.cwide)[hb] = (S.cwide[h] ? 1u : 0u) | (S.ovf ? 2u : 0u);
        }
    }
}

// After an adding pass: frames that turn RAW late.  (1) Ring step: a frame whose local data holds an element that
// cannot be quantized is RAW (as the interface quantizer would have made it), so its payload is the fp32 sum of the
// incoming values and the ORIGINAL local values.  (2) Either reduce: a frame in which some integer sum exceeds 2^30
// in magnitude cannot be carried as codes any further; it is committed as RAW and holds the fp32 sum of the two
// dequantized operands (RAW is the safe fallback of the selector, Sec. IV-C / Algorithm 1).  Both are rare; one
// workgroup per half looks at the frame's flags and returns at once otherwise.  The operand codes are recovered
// exactly from the staged sums: incoming = Q - q_local (q_local = 0 where the element was not quantizable), or
// B = Q - A with the staged codes of A; a RAW incoming frame is read from the stream again.
__global__ __launch_bounds__(256) void k_fix(DecodeArgs A) {
    const uint32_t tid = threadIdx.x;
    const uint32_t hpf = (A.chunk + kHalf - 1) / kHalf;
    const uint32_t frame = blockIdx.x / hpf, h = blockIdx.x % hpf;
    const uint64_t f0 = (uint64_t)frame * A.chunk;
    const uint32_t nf = (uint32_t)((A.n - f0 < A.chunk) ? (A.n - f0) : A.chunk);
    const uint32_t h0 = h * kHalf;
    if (h0 >= nf) return;
    const uint32_t cnt = (nf - h0 < kHalf) ? (nf - h0) : kHalf;
    const uint2* pm = reinterpret_cast<const uint2*>(A.ws + A.L.pmeta) + (size_t)frame * hpf;
    const uint32_t* cw = reinterpret_cast<const uint32_t*>(A.ws + A.L.cwide) + (size_t)frame * hpf;
    uint32_t lunq = 0, ovf = 0, raw = 0;
    for (uint32_t j = 0; j < hpf && j * kHalf < nf; j++) { raw |= pm[j].y & 1u; lunq |= pm[j].y & 2u; ovf |= cw[j] & 2u; }
    // an operand frame that is RAW already has fp32 sums staged (no integer sums, no range question); only the ring
    // step's local data can still change what those sums must be
    if (!lunq && (raw || !ovf)) return;
    uint32_t* codes = reinterpret_cast<uint32_t*>(A.ws + A.L.codes) + f0 + h0;
    const int16_t* c16 = reinterpret_cast<const int16_t*>(A.ws + A.L.c16) + f0 + h0;
    StageA sa;
    sa.a16 = reinterpret_cast<int16_t*>(A.ws + A.L.a16); sa.a32 = reinterpret_cast<uint32_t*>(A.ws + A.L.a32);
    const uint32_t* raw_in = nullptr;
    if (raw) {          // ring step, incoming frame RAW: header and extent were validated by the adding pass
        const uint64_t off = *reinterpret_cast<const uint64_t*>(A.a + kStreamHdr + 8ull * frame);
        raw_in = reinterpret_cast<const uint32_t*>(A.a + off + kHdrBytes) + h0;
    }
    uint32_t dummy = 0;
    for (uint32_t i = tid; i < cnt; i += 256) {
        uint32_t ta, tb; bool b_is_raw = false;
        if (raw) { ta = raw_in[i]; tb = __float_as_uint(A.local[f0 + h0 + i]); b_is_raw = true; }
        else {
            const int32_t s16 = c16[i];
            const uint32_t Q = (s16 == kWideMarker) ? codes[i] : (uint32_t)s16;
            if (A.local) {
                const float x = A.local[f0 + h0 + i];
                int32_t q;
                const uint64_t g = f0 + h0 + i;
                if (A.sr) sr_quantize1(x, A.step, A.inv_step, sr_draw(sr_key(A.seed, g), (uint32_t)g), q);
                else quantize1(x, A.eb, A.step, A.inv_step, q);
                ta = Q - (uint32_t)q;                                   // the incoming code
                if (lunq) { tb = __float_as_uint(x); b_is_raw = true; } else tb = (uint32_t)q;
            } else {
                ta = sa.get(f0, nf, h0 + i, false);
                tb = Q - ta;
            }
        }
        codes[i] = combine<true>(ta, raw != 0, tb, b_is_raw, A.step, dummy);
    }
}

// After an accumulating pass of the k-ary reduce: a frame in which a partial sum passed 2^30 in magnitude leaves the
// integer domain at this operand.  Its running value becomes fp32 -- fl(fl(v*step) + fl(q*step)) with v the running
// code before this operand (still in the set the pass read) and q the operand's code, recovered as the staged sum
// minus v -- and the frame counts as RAW for the operands that follow.  One workgroup per half; rare.
__global__ __launch_bounds__(256) void k_fix_acc(DecodeArgs A) {
    const uint32_t tid = threadIdx.x;
    const uint32_t hpf = (A.chunk + kHalf - 1) / kHalf;
    const uint32_t frame = blockIdx.x / hpf, h = blockIdx.x % hpf;
    const uint64_t f0 = (uint64_t)frame * A.chunk;
    const uint32_t nf = (uint32_t)((A.n - f0 < A.chunk) ? (A.n - f0) : A.chunk);
    const uint32_t h0 = h * kHalf;
    if (h0 >= nf) return;
    const uint32_t cnt = (nf - h0 < kHalf) ? (nf - h0) : kHalf;
    const uint2* pm = reinterpret_cast<const uint2*>(A.ws + A.L.pmeta) + (size_t)frame * hpf;
    const uint32_t* cw = reinterpret_cast<const uint32_t*>(A.ws + A.L.cwide) + (size_t)frame * hpf;
    uint32_t ovf = 0, raw = 0;
    for (uint32_t j = 0; j < hpf && j * kHalf < nf; j++) { raw |= pm[j].y & 1u; ovf |= cw[j] & 2u; }
    if (raw || !ovf) return;                  // (a frame that was fp32 already has no integer sums to go out of range)
    const uint32_t si = A.set_in & 1u;
    StageA sa, so;
    sa.a16 = reinterpret_cast<int16_t*>(A.ws + (si ? A.L.c16 : A.L.a16)); sa.a32 = reinterpret_cast<uint32_t*>(A.ws + (si ? A.L.codes : A.L.a32));
    so.a16 = reinterpret_cast<int16_t*>(A.ws + (si ? A.L.a16 : A.L.c16)); so.a32 = reinterpret_cast<uint32_t*>(A.ws + (si ? A.L.a32 : A.L.codes));
    uint32_t dummy = 0;
    for (uint32_t i = tid; i < cnt; i += 256) {
        const uint32_t ta = sa.get(f0, nf, h0 + i, false);
        const uint32_t tb = so.get(f0, nf, h0 + i, false) - ta;
        so.a32[f0 + h0 + i] = combine<true>(ta, false, tb, false, A.step, dummy);
    }
    if (h == 0 && tid == 0) reinterpret_cast<uint32_t*>(A.ws + (si ? A.L.akind : A.L.akind1))[frame] = 1u;
}

hipError_t launch_fix_acc(const DecodeArgs& A, hipStream_t st) {
    const uint32_t hpf = (A.chunk + kHalf - 1) / kHalf;
    hipLaunchKernelGGL(k_fix_acc, dim3(A.n_frames * hpf), dim3(256), 0, st, A);
    return hipGetLastError();
}

hipError_t launch_fix(const DecodeArgs& A, hipStream_t st) {
    const uint32_t hpf = (A.chunk + kHalf - 1) / kHalf;
    hipLaunchKernelGGL(k_fix, dim3(A.n_frames * hpf), dim3(256), 0, st, A);
    return hipGetLastError();
}

// Decompress, second kernel: sums the workgroups' verdicts up into the result record (plain stores: the record needs
// no clearing beforehand) and zero-fills every rejected frame -- the ones rejected at the header decode to zeros
// anyway, the ones found corrupt while decoding (a segment that did not use exactly its recorded bits) were written
// before the verdict was known.  A rejected frame never hands untrusted bytes to the caller (the paper's receiver
// copies rawBytes from an invalid frame, Algorithm 2; this format reports the frame and fills it with zeros).
__global__ __launch_bounds__(256) void k_decode_finish(DecodeArgs A) {
    __shared__ uint32_t s_status, s_cnt[3];
    const uint32_t tid = threadIdx.x;
    const uint32_t* verdict = reinterpret_cast<const uint32_t*>(A.ws + A.L.pmeta);
    uint64_t total = 0;
    const uint32_t st_a = check_stream(A.a, A.a_bytes, A, total);
    auto frame_verdict = [&](uint32_t frame, uint32_t& kind) -> uint32_t {
        const uint64_t f0 = (uint64_t)frame * A.chunk;
        const uint32_t nf = (uint32_t)((A.n - f0 < A.chunk) ? (A.n - f0) : A.chunk);
        uint32_t st = 0;
        for (uint32_t db = 0; db < A.dbpf && db * kDecBlock < nf; db++) {
            const uint32_t v = verdict[(size_t)frame * A.dbpf + db];
            st = (v & 0xFFu) > st ? (v & 0xFFu) : st;
            if (db == 0) kind = v >> 8;
        }
        return st;
    };
    if (st_a == ST_OK) {
        for (uint32_t frame = blockIdx.x; frame < A.n_frames; frame += gridDim.x) {
            uint32_t kind;
            if (frame_verdict(frame, kind) == ST_OK) continue;
            const uint64_t f0 = (uint64_t)frame * A.chunk;
            const uint32_t nf = (uint32_t)((A.n - f0 < A.chunk) ? (A.n - f0) : A.chunk);
            for (uint32_t i = tid; i < nf; i += 256) A.out[f0 + i] = 0.0f;
        }
    }
    if (blockIdx.x != 0) return;
    if (tid == 0) { s_status = st_a; s_cnt[0] = 0; s_cnt[1] = 0; s_cnt[2] = 0; }
    __syncthreads();
    if (st_a == ST_OK) {
        uint32_t worst = 0, c[3] = { 0, 0, 0 };
        for (uint32_t frame = tid; frame < A.n_frames; frame += 256) {
            uint32_t kind = KIND_ZERO;
            const uint32_t st = frame_verdict(frame, kind);
            worst = st > worst ? st : worst;
            if (st == ST_OK && kind < 3u) c[kind]++;
        }
        if (worst) atomicMax(&s_status, worst);
        for (int k = 0; k < 3; k++) if (c[k]) atomicAdd(&s_cnt[k], c[k]);
    }
    __syncthreads();
    if (tid == 0) {
        ResultRec* res = reinterpret_cast<ResultRec*>(A.res);
        res->bytes = (st_a == ST_OK) ? total : 0ull;
        res->status = s_status; res->n_frames = A.n_frames;
        res->n_raw = s_cnt[KIND_RAW]; res->n_fixed = s_cnt[KIND_FIXED]; res->n_huff = s_cnt[KIND_HUFF]; res->reserved = 0;
    }
}

hipError_t launch_decode_finish(const DecodeArgs& A, hipStream_t st) {
    DecodeArgs D = A;
    D.dbpf = (A.chunk + kDecBlock - 1) / kDecBlock;
    const uint32_t grid = A.n_frames < 1024u ? A.n_frames : 1024u;
    hipLaunchKernelGGL(k_decode_finish, dim3(grid), dim3(256), 0, st, D);
    return hipGetLastError();
}

constexpr int kAddThreads = 512;        // second reduce pass: two halves per workgroup, four waves per SIMD at 2 workgroups per CU

template <int DELTA>
static void launch_decode_t(DecodeArgs& D, const DecodeArgs& A, int pass, hipStream_t st) {
    if (pass == 0) {
        D.dbpf = (A.chunk + kDecBlock - 1) / kDecBlock;
        hipLaunchKernelGGL((k_decode<MODE_DECOMPRESS, kDecThreads, DELTA>), dim3(D.n_frames * D.dbpf), dim3(kDecThreads), 0, st, D);
    } else if (pass == 1) {
        D.dbpf = (A.chunk + kDecBlock - 1) / kDecBlock;
        hipLaunchKernelGGL((k_decode<MODE_STAGE_A, kDecThreads, DELTA>), dim3(D.n_frames * D.dbpf), dim3(kDecThreads), 0, st, D);
    } else if (pass == 2) {
        D.dbpf = (A.chunk + kAddThreads * kSeg - 1) / (kAddThreads * kSeg);
        hipLaunchKernelGGL((k_decode<MODE_ADD_B, kAddThreads, DELTA>), dim3(D.n_frames * D.dbpf), dim3(kAddThreads), 0, st, D);
    } else if (pass == 3) {
        D.dbpf = (A.chunk + kAddThreads * kSeg - 1) / (kAddThreads * kSeg);
        hipLaunchKernelGGL((k_decode<MODE_ADD_LOCAL, kAddThreads, DELTA>), dim3(D.n_frames * D.dbpf), dim3(kAddThreads), 0, st, D);
    } else if (pass == 6) {
        D.dbpf = (A.chunk + kAddThreads * kSeg - 1) / (kAddThreads * kSeg);
        hipLaunchKernelGGL((k_decode<MODE_ACC, kAddThreads, DELTA>), dim3(D.n_frames * D.dbpf), dim3(kAddThreads), 0, st, D);
    } else if constexpr (DELTA == 0) {          // (the stochastic and the sampled ring step are not built with the predictor)
        D.dbpf = (A.chunk + kAddThreads * kSeg - 1) / (kAddThreads * kSeg);
        if (pass == 4) hipLaunchKernelGGL((k_decode<MODE_ADD_LOCAL_SR, kAddThreads, 0>), dim3(D.n_frames * D.dbpf), dim3(kAddThreads), 0, st, D);
        else hipLaunchKernelGGL((k_decode<MODE_ADD_LOCAL_PLAIN, kAddThreads, 0>), dim3(D.n_frames * D.dbpf), dim3(kAddThreads), 0, st, D);
    }
}

hipError_t launch_decode(const DecodeArgs& A, int pass, hipStream_t st) {
    DecodeArgs D = A;
    if (A.pred) launch_decode_t<1>(D, A, pass, st); else launch_decode_t<0>(D, A, pass, st);
    return hipGetLastError();
}

}  // namespace nz
