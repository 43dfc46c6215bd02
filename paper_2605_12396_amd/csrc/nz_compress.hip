// nz_compress.hip -- gfx950 kernels of the sender side: frame statistics (quantize + zmax + histogram),
// per-frame codebook + exact-size selector + frame-offset look-back, and the bit-packing encoder.
//
// Paper mapping: interface quantizer (Sec. IV-B), runtime entropy arbitration with transmitted size as
// the cost (Sec. IV-C, Eq. 1-2, Algorithm 1), frame = header + payload (Sec. IV-D "Batch Framing").
// Unlike the paper's sampled estimate by one control thread, the statistics here cover the whole frame,
// so predicted and realized sizes coincide and Algorithm 1's post-validation never fires.
#include "nz_common.hpp"
#include "nz_scan.hpp"

namespace nz {

// ------------------------------------------------------------------------------------------------
// K0: clear the control block / look-back descriptors and initialise the result record
// ------------------------------------------------------------------------------------------------
__global__ void k_init(uint32_t* zero_base, size_t zero_words, ResultRec* res, uint32_t n_frames, uint32_t status) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < zero_words) zero_base[i] = 0;
    if (i == 0 && res) {
        res->bytes = 0; res->status = status; res->n_frames = n_frames;
        res->n_raw = 0; res->n_fixed = 0; res->n_huff = 0; res->reserved = 0;
    }
}

// ------------------------------------------------------------------------------------------------
// K1: frame statistics.  One workgroup per kStatBlock symbols of one frame: coalesced 16-byte loads,
// quantize, zigzag, lane-replicated LDS histogram, zmax and the "cannot be quantized" flag.
// The partial histogram goes to the workspace with plain stores; the codebook kernel adds the partials.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kStatThreads) void k_stats(CompressArgs A) {
    __shared__ uint32_t s_h[8192];
    __shared__ uint32_t s_zmax, s_unq;
    const uint32_t tid = threadIdx.x, lane = lane_id();
    const uint32_t frame = blockIdx.x / A.sbpf, sb = blockIdx.x % A.sbpf;
    const uint64_t f0 = (uint64_t)frame * A.chunk;
    const uint32_t nf = (uint32_t)((A.n - f0 < A.chunk) ? (A.n - f0) : A.chunk);
    const uint32_t b0 = sb * kStatBlock;
    if (b0 >= nf) return;
    const uint32_t cnt = (nf - b0 < kStatBlock) ? (nf - b0) : kStatBlock;
    const uint32_t K = A.K;
    // replicate the histogram over lanes: 8192/K copies (at most 32) so hot bins do not serialise
    uint32_t ncs = 0;
    while ((K << (ncs + 1)) <= 8192u && ncs < 5) ncs++;
    const uint32_t copy = lane & ((1u << ncs) - 1u);
    for (uint32_t i = tid; i < (K << ncs); i += kStatThreads) s_h[i] = 0;
    if (tid == 0) { s_zmax = 0; s_unq = 0; }
    __syncthreads();

    const float* src = A.in + f0 + b0;
    const bool vec_ok = (((f0 + b0) & 3u) == 0);
    uint32_t zmax = 0, unq = 0;
    for (uint32_t i = tid * 4; i < cnt; i += kStatThreads * 4) {
        float v[4];
        const uint32_t m = (cnt - i < 4) ? (cnt - i) : 4;
        if (vec_ok && m == 4) {
            const float4 t = *reinterpret_cast<const float4*>(src + i);
            v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
        } else {
            for (uint32_t j = 0; j < 4; j++) v[j] = (j < m) ? src[i + j] : 0.0f;
        }
#pragma unroll
        for (uint32_t j = 0; j < 4; j++) {
            if (j < m) {
                int32_t q;
                if (!quantize1(v[j], A.eb, A.step, A.inv_step, q)) unq = 1;
                const uint32_t z = zigzag(q);
                zmax = z > zmax ? z : zmax;
                atomicAdd(&s_h[(sym_of(z, K) << ncs) + copy], 1u);
            }
        }
    }
    zmax = wave_max(zmax);
    unq = wave_max(unq);
    if (lane == 0) { atomicMax(&s_zmax, zmax); atomicMax(&s_unq, unq); }
    __syncthreads();
    uint32_t* ph = reinterpret_cast<uint32_t*>(A.ws + A.L.phist) + (size_t)blockIdx.x * kMaxK;
    for (uint32_t s = tid; s < K; s += kStatThreads) {
        uint32_t t = 0;
        for (uint32_t c = 0; c < (1u << ncs); c++) t += s_h[(s << ncs) + c];
        ph[s] = t;
    }
    if (tid == 0) {
        uint2* pm = reinterpret_cast<uint2*>(A.ws + A.L.pmeta) + blockIdx.x;
        *pm = make_uint2(s_zmax, s_unq);
    }
}

// ------------------------------------------------------------------------------------------------
// K2: one workgroup per frame.  Sum the partial histograms, build optimal prefix-code lengths with the
// two-queue construction (leaves sorted by (count, symbol), a leaf wins a weight tie against an internal
// node), assign canonical codes, compute the exact size of each codec, arbitrate, place the frame with a
// decoupled look-back over frame sizes, and write header, code-length table and the encoder's codebook.
// ------------------------------------------------------------------------------------------------
__device__ inline uint64_t pad4u(uint64_t v) { return (v + 3u) & ~(uint64_t)3u; }
__device__ inline uint64_t pad16u(uint64_t v) { return (v + 15u) & ~(uint64_t)15u; }

__global__ __launch_bounds__(kBookThreads) void k_codebook(CompressArgs A) {
    __shared__ uint32_t s_f[kMaxK];
    __shared__ __align__(16) uint32_t s_key[kMaxK];
    __shared__ uint32_t s_sorted[kMaxK];
    __shared__ uint32_t s_w[2 * kMaxK];
    __shared__ uint16_t s_par[2 * kMaxK];
    __shared__ __align__(4) uint8_t s_len[kMaxK];
    __shared__ uint16_t s_rank[kMaxK];
    __shared__ uint32_t s_wcnt[16 * 32], s_cnt[32], s_first[32], s_idx0[32];
    __shared__ uint64_t s_part[16];
    __shared__ uint32_t s_fid, s_m, s_nsym, s_zmax, s_unq, s_codec, s_payload, s_total, s_w_fixed;
    __shared__ uint64_t s_bits, s_off;

    const uint32_t tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const uint32_t K = A.K;
    Ctrl* ctrl = reinterpret_cast<Ctrl*>(A.ws + A.L.ctrl);
    if (tid == 0) { s_fid = atomicAdd(&ctrl->ticket_book, 1u); s_m = 0; s_nsym = 0; s_zmax = 0; s_unq = 0; }
    __syncthreads();
    const uint32_t fid = s_fid;
    const uint64_t f0 = (uint64_t)fid * A.chunk;
    const uint32_t nf = (uint32_t)((A.n - f0 < A.chunk) ? (A.n - f0) : A.chunk);
    const uint32_t sbc = (nf + A.stat_block - 1) / A.stat_block;

    // (1) frame histogram, zmax, quantizable flag
    uint32_t f = 0;
    if (tid < K) {
        const uint32_t* ph = reinterpret_cast<const uint32_t*>(A.ws + A.L.phist) + (size_t)fid * A.sbpf * kMaxK + tid;
        for (uint32_t b = 0; b < sbc; b++) f += ph[(size_t)b * kMaxK];
    }
    s_f[tid] = f;
    s_len[tid] = 0;
    if (tid < sbc) {
        const uint2 pm = reinterpret_cast<const uint2*>(A.ws + A.L.pmeta)[(size_t)fid * A.sbpf + tid];
        atomicMax(&s_zmax, pm.x);
        atomicMax(&s_unq, pm.y);
    }
    const bool used = f > 0;
    {
        const uint64_t um = __ballot(used);
        if (lane == 0 && um) { atomicAdd(&s_m, (uint32_t)__popcll(um)); atomicMax(&s_nsym, wave * 64 + 64 - (uint32_t)__clzll(um)); }
    }
    // (2) sort used symbols ascending by (count, symbol): rank = number of smaller keys
    const uint32_t key = used ? ((f << 10) | tid) : 0xFFFFFFFFu;
    s_key[tid] = key;
    __syncthreads();
    const uint32_t m = s_m, nsym = s_nsym;
    if (used) {
        uint32_t rank = 0;
        const uint4* k4 = reinterpret_cast<const uint4*>(s_key);
        for (uint32_t j = 0; j < K / 4 || j < 1; j++) {
            const uint4 t = k4[j];
            rank += (t.x < key) + (t.y < key) + (t.z < key) + (t.w < key);
        }
        s_sorted[rank] = key;
    }
    __syncthreads();
    if (tid < m) s_w[tid] = s_sorted[tid] >> 10;
    __syncthreads();

    // (3) two-queue merge, one lane; queue heads cached in registers
    if (tid == 0 && m >= 2) {
        const uint32_t INF = 0xFFFFFFFFu;
        uint32_t ia = 0, ib = m, nb = m;
        uint32_t a0 = s_w[0], a1 = (m > 1) ? s_w[1] : INF, b0 = INF, b1 = INF;
        for (uint32_t step = 0; step + 1 < m; step++) {
            uint32_t p0, p1, w;
            if (a0 <= b0) {                       // first pick: leaf (a leaf wins ties)
                if (a1 <= b0) {                   // second pick: leaf
                    p0 = ia; p1 = ia + 1; w = a0 + a1; ia += 2;
                    a0 = (ia < m) ? s_w[ia] : INF; a1 = (ia + 1 < m) ? s_w[ia + 1] : INF;
                } else {                          // second pick: internal node
                    p0 = ia; p1 = ib; w = a0 + b0; ia += 1; ib += 1;
                    a0 = a1; a1 = (ia + 1 < m) ? s_w[ia + 1] : INF;
                    b0 = b1; b1 = (ib + 1 < nb) ? s_w[ib + 1] : INF;
                }
            } else {                              // first pick: internal node
                if (a0 <= b1) {                   // second pick: leaf
                    p0 = ib; p1 = ia; w = b0 + a0; ia += 1; ib += 1;
                    a0 = a1; a1 = (ia + 1 < m) ? s_w[ia + 1] : INF;
                    b0 = b1; b1 = (ib + 1 < nb) ? s_w[ib + 1] : INF;
                } else {                          // second pick: internal node
                    p0 = ib; p1 = ib + 1; w = b0 + b1; ib += 2;
                    b0 = (ib < nb) ? s_w[ib] : INF; b1 = (ib + 1 < nb) ? s_w[ib + 1] : INF;
                }
            }
            s_w[nb] = w; s_par[p0] = (uint16_t)nb; s_par[p1] = (uint16_t)nb;
            if (ib == nb) b0 = w; else if (ib + 1 == nb) b1 = w;   // the new node may be a queue head
            nb++;
        }
    }
    __syncthreads();
    // (4) code length = depth of the leaf
    if (tid < m) {
        uint32_t d = 1;
        if (m >= 2) {
            const uint32_t root = 2 * m - 2;
            d = 0;
            for (uint32_t x = tid; x != root; x = s_par[x]) d++;
        }
        s_len[s_sorted[tid] & 1023u] = (uint8_t)d;
    }
    __syncthreads();
    // (5) canonical codes
    canonical_tables<kBookThreads>(s_len, K, s_wcnt, s_cnt, s_first, s_idx0, s_rank);
    const uint32_t L = s_len[tid];
    const uint32_t code = L ? (s_first[L] + s_rank[tid]) : 0u;
    // (6) exact Huffman bitstream length: sum f*len, an escape carries 32 more bits
    {
        uint64_t b = (uint64_t)f * L + (tid == 0 ? 32ull * f : 0ull);
        b = wave_sum64(b);
        if (lane == 0) s_part[wave] = b;
    }
    __syncthreads();
    // (7) sizes and arbitration (Eq. 2: argmin of frame bytes over RAW + admissible codecs, ties to the lower id)
    if (tid == 0) {
        uint64_t bits = 0;
        for (int i = 0; i < 16; i++) bits += s_part[i];
        const uint32_t zmax = s_zmax;
        const uint32_t w = zmax ? (32u - (uint32_t)__clz(zmax)) : 0u;
        const uint32_t nseg = (nf + kSeg - 1) / kSeg;
        uint64_t pay[3], tot[3];
        pay[CODEC_RAW] = 4ull * nf;
        pay[CODEC_FIXED] = 4ull * (((uint64_t)nf * w + 31u) / 32u);
        pay[CODEC_HUFF] = pad4u(nsym) + pad4u(2ull * nseg) + 4ull * ((bits + 31u) / 32u);
        for (int c = 0; c < 3; c++) tot[c] = pad16u(kHdrBytes + pay[c]);
        uint32_t best = CODEC_RAW;
        if (!s_unq) {
            if (A.force_codec >= 0) best = (uint32_t)A.force_codec;
            else {
                for (uint32_t c = CODEC_FIXED; c <= CODEC_HUFF; c++) {
                    if (c == CODEC_HUFF && pay[CODEC_RAW] < A.huff_min_bytes) continue;
                    if (pay[c] > pay[CODEC_RAW]) continue;
                    if ((pay[CODEC_RAW] - pay[c]) * 1000ull < (uint64_t)A.min_gain_permil * pay[CODEC_RAW]) continue;
                    if (tot[c] < tot[best]) best = c;
                }
            }
        }
        s_codec = best; s_payload = (uint32_t)pay[best]; s_total = (uint32_t)tot[best];
        s_w_fixed = w; s_bits = bits;
    }
    __syncthreads();
    // (8) place the frame: decoupled look-back over padded frame sizes
    uint64_t* fdesc = reinterpret_cast<uint64_t*>(A.ws + A.L.frame_desc);
    if (wave == 0) {
        const uint64_t mine = s_total;
        if (lane == 0) st_agent(fdesc + fid, kDescA | mine);
        const uint64_t base = kStreamHdr + pad16u(8ull * A.n_frames);
        const uint64_t excl = lookback_exclusive(fdesc, 0, (int64_t)fid, base);
        if (lane == 0) { st_agent(fdesc + fid, kDescP | (excl + mine)); s_off = excl; }
    }
    __syncthreads();
    // (9) publish: offsets table, header, code-length table, encoder codebook, counters
    const uint64_t off = s_off;
    const uint32_t codec = s_codec, payload = s_payload, total = s_total;
    const bool fits = off + total <= A.out_cap;
    const uint32_t nseg = (nf + kSeg - 1) / kSeg;
    uint8_t* fr = A.out + off;
    if (tid == 0) {
        *reinterpret_cast<uint64_t*>(A.out + kStreamHdr + 8ull * fid) = off;
        if (fid == A.n_frames - 1 && (A.n_frames & 1u))
            *reinterpret_cast<uint64_t*>(A.out + kStreamHdr + 8ull * A.n_frames) = 0;      // pad16 of the table
        FrameMeta M;
        M.offset = off; M.total = total; M.payload = payload; M.codec = codec; M.w = s_w_fixed; M.nsym = nsym;
        M.fits = fits ? 1u : 0u;
        M.segt_off = kHdrBytes + (uint32_t)pad4u(nsym);
        M.bits_off = (codec == CODEC_HUFF) ? (M.segt_off + (uint32_t)pad4u(2ull * nseg)) : kHdrBytes;
        M.bits_words = (codec == CODEC_HUFF) ? (uint32_t)((s_bits + 31u) / 32u)
                                             : (uint32_t)(((uint64_t)nf * s_w_fixed + 31u) / 32u);
        M.pad_ = 0; M.huff_bits = s_bits; M.pad2_ = 0;
        reinterpret_cast<FrameMeta*>(A.ws + A.L.meta)[fid] = M;
        if (fits) {
            uint32_t h[8];
            h[0] = kMagicFrame; h[1] = codec; h[2] = 4u * nf; h[3] = payload;
            h[4] = (codec == CODEC_FIXED) ? s_w_fixed : (codec == CODEC_HUFF ? nsym : 0u);
            h[5] = (codec == CODEC_HUFF) ? (kSeg | (K << 16)) : 0u;
            h[6] = A.step_bits;
            uint32_t x = kCheckXor;
            for (int i = 0; i < 7; i++) x ^= h[i];
            h[7] = x;
            uint4* dst = reinterpret_cast<uint4*>(fr);
            dst[0] = make_uint4(h[0], h[1], h[2], h[3]);
            dst[1] = make_uint4(h[4], h[5], h[6], h[7]);
        }
        ResultRec* res = reinterpret_cast<ResultRec*>(A.res);
        atomicAdd(codec == CODEC_RAW ? &res->n_raw : (codec == CODEC_FIXED ? &res->n_fixed : &res->n_huff), 1u);
        if (fid == A.n_frames - 1) {
            const uint64_t stream_total = off + total;
            if (stream_total > A.out_cap) atomicMax(&res->status, (uint32_t)ST_CAPACITY);
            uint32_t* sh = reinterpret_cast<uint32_t*>(A.out);
            sh[0] = kMagicStream; sh[1] = 1u;
            sh[2] = (uint32_t)A.n; sh[3] = (uint32_t)(A.n >> 32);
            sh[4] = A.chunk; sh[5] = A.n_frames; sh[6] = A.step_bits; sh[7] = kSeg; sh[8] = K; sh[9] = 0;
            sh[10] = (uint32_t)stream_total; sh[11] = (uint32_t)(stream_total >> 32);
            sh[12] = 0; sh[13] = 0; sh[14] = 0; sh[15] = 0;
            const uint32_t st = atomicMax(&res->status, 0u);
            res->bytes = (st == ST_OK && stream_total <= A.out_cap) ? stream_total : 0ull;
        }
    }
    if (codec == CODEC_HUFF) {
        // Exact bitstream position of every statistics block (= one encoder workgroup): its bit count is
        // sum over symbols of (block count) x (code length), an escape carrying 32 more bits.  The encoder
        // therefore needs no scan of its own.  The word in which two blocks meet is written by both with an
        // atomic OR, so it is cleared here.
        const uint32_t* ph = reinterpret_cast<const uint32_t*>(A.ws + A.L.phist) + (size_t)fid * A.sbpf * kMaxK;
        for (uint32_t b = wave; b < sbc; b += kBookThreads / 64) {
            uint64_t t = 0;
            for (uint32_t sy = lane; sy < K; sy += 64) {
                const uint32_t c = ph[(size_t)b * kMaxK + sy];
                t += (uint64_t)c * (s_len[sy] + (sy == 0 ? 32u : 0u));
            }
            t = wave_sum64(t);
            if (lane == 0) s_w[b] = (uint32_t)t;                          // s_w is free again: block bit counts
        }
        __syncthreads();
        if (tid == 0) {
            uint32_t* gs = reinterpret_cast<uint32_t*>(A.ws + A.L.grp_start) + (size_t)fid * A.sbpf;
            uint32_t run = 0;
            const uint32_t segt_off = kHdrBytes + (uint32_t)pad4u(nsym);
            uint32_t* bitsw = reinterpret_cast<uint32_t*>(fr + segt_off + (uint32_t)pad4u(2ull * nseg));
            for (uint32_t b = 0; b < sbc; b++) {
                gs[b] = run;
                if (fits && b > 0) bitsw[run >> 5] = 0;
                run += s_w[b];
            }
        }
        if (fits) {   // code lengths, one byte per symbol, zero padded to 4
            const uint32_t words = (uint32_t)(pad4u(nsym) / 4);
            if (tid < words) reinterpret_cast<uint32_t*>(fr + kHdrBytes)[tid] = reinterpret_cast<const uint32_t*>(s_len)[tid];
        }
        // encoder codebook: code bits reversed so that emitting them LSB-first sends the code MSB-first
        if (tid < K) {
            reinterpret_cast<uint32_t*>(A.ws + A.L.book_code)[(size_t)fid * kMaxK + tid] = L ? (__brev(code) >> (32u - L)) : 0u;
            (A.ws + A.L.book_len)[(size_t)fid * kMaxK + tid] = (uint8_t)L;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// K4: encoder.  One workgroup per statistics block of one frame (32768 symbols for compress, 65536 for
// the reduce), worked through in sub-blocks of kEncBlock symbols; the next sub-block's source words are
// loaded while the current one is packed.
//   RAW      copy the words.
//   FIXEDLEN w bits per zigzag code at closed-form positions (a pass of 1024 codes is 32*w whole words).
//   HUFFMAN  the workgroup's first bit in the frame's bitstream comes from the codebook kernel, so there is
//            no scan and no waiting between workgroups.  Per sub-block: phase 1 looks every symbol up once,
//            packs the 4 symbols of a thread (codes, and the 32 raw bits of an escape) into 64 bits and scans
//            the bit counts on the DPP network (segment table entries fall out of the scan); phase 2 ORs the
//            packed strings into an LDS stage at their final bit positions and flushes whole words
//            coalesced.  The word in which two workgroups meet was cleared by the codebook kernel and
//            receives both parts by atomic OR; every other word has a single writer.
// SRC = 0: symbols are quantized from the fp32 input; SRC = 1: symbols are the int32 codes staged in the
// workspace by the reduce front end (RAW frames hold fp32 bit patterns there).
// ------------------------------------------------------------------------------------------------
template <int SRC>
__global__ __launch_bounds__(kEncThreads) void k_encode(CompressArgs A) {
    constexpr uint32_t kStageWords = 2048;
    __shared__ uint64_t s_book[kMaxK];            // reversed code | length << 32
    __shared__ uint32_t s_stage[kStageWords];
    __shared__ uint32_t s_wtot[kEncSegs];         // bit count of each of the sub-block's segments
    __shared__ uint32_t s_pbase[kEncIters + 1];   // bit offset of every pass inside the sub-block

    const uint32_t tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const uint32_t frame = blockIdx.x / A.sbpf, gb = blockIdx.x % A.sbpf;
    const uint64_t f0 = (uint64_t)frame * A.chunk;
    const uint32_t nf = (uint32_t)((A.n - f0 < A.chunk) ? (A.n - f0) : A.chunk);
    const uint32_t g0 = gb * A.stat_block;                               // first symbol of this workgroup in the frame
    if (g0 >= nf) return;
    const uint32_t gcnt = (nf - g0 < A.stat_block) ? (nf - g0) : A.stat_block;
    const bool last_grp = (g0 + gcnt == nf);
    const uint32_t nsub = (gcnt + kEncBlock - 1) / kEncBlock;
    const uint32_t K = A.K;
    // source words: fp32 input (SRC 0) or the staged codes / fp32 sums of the reduce (SRC 1)
    const uint32_t* gsrc = (SRC == 0 ? reinterpret_cast<const uint32_t*>(A.in) : reinterpret_cast<const uint32_t*>(A.ws + A.L.codes)) + f0 + g0;
    const bool vec_ok = (((f0 + g0) & 3u) == 0);                         // kEncBlock is a multiple of 4

    // loads of one sub-block: pass `it` covers its symbols it*1024 + tid*4 .. +3
    auto load_sub = [&](uint32_t sb, uint32_t (&raw)[kEncIters][4]) {
        const uint32_t* src = gsrc + sb * kEncBlock;
        const uint32_t cnt = (sb < nsub) ? ((gcnt - sb * kEncBlock < kEncBlock) ? (gcnt - sb * kEncBlock) : kEncBlock) : 0u;
#pragma unroll
        for (uint32_t it = 0; it < kEncIters; it++) {
            const uint32_t i = it * 1024 + tid * 4;
            const uint32_t mvalid = (i < cnt) ? ((cnt - i < 4) ? (cnt - i) : 4u) : 0u;
            if (vec_ok && mvalid == 4) {
                const uint4 t = *reinterpret_cast<const uint4*>(src + i);
                raw[it][0] = t.x; raw[it][1] = t.y; raw[it][2] = t.z; raw[it][3] = t.w;
            } else {
#pragma unroll
                for (uint32_t j = 0; j < 4; j++) raw[it][j] = (j < mvalid) ? src[i + j] : 0u;
            }
        }
    };
    uint32_t raw[kEncIters][4], nxt[kEncIters][4];
    load_sub(0, raw);
    const FrameMeta M = reinterpret_cast<const FrameMeta*>(A.ws + A.L.meta)[frame];
    if (!M.fits) return;
    uint8_t* fr = A.out + M.offset;
    // zigzag code of a source word
    auto zz = [&](uint32_t w) -> uint32_t {
        if (SRC == 0) { int32_t t; quantize1(__uint_as_float(w), A.eb, A.step, A.inv_step, t); return zigzag(t); }
        return zigzag((int32_t)w);
    };
    auto pad_frame = [&]() {     // the frame's last workgroup zero-fills the padding after the payload
        if (last_grp) {
            const uint32_t w0 = (kHdrBytes + M.payload) / 4, w1 = M.total / 4;
            if (tid < w1 - w0) reinterpret_cast<uint32_t*>(fr)[w0 + tid] = 0;
        }
    };

    // ---- RAW: copy the words ----
    if (M.codec == CODEC_RAW) {
        uint32_t* dst = reinterpret_cast<uint32_t*>(fr + kHdrBytes) + g0;
        for (uint32_t i = tid * 4; i < gcnt; i += kEncThreads * 4) {
            if (vec_ok && i + 4 <= gcnt) *reinterpret_cast<uint4*>(dst + i) = *reinterpret_cast<const uint4*>(gsrc + i);
            else for (uint32_t j = 0; j < 4; j++) if (i + j < gcnt) dst[i + j] = gsrc[i + j];
        }
        pad_frame();
        return;
    }
    uint32_t* bits = reinterpret_cast<uint32_t*>(fr + M.bits_off);

    // ---- FIXEDLEN ----
    if (M.codec == CODEC_FIXED) {
        const uint32_t w = M.w;
        for (uint32_t sb = 0; sb < nsub; sb++) {
            const uint32_t cnt = (gcnt - sb * kEncBlock < kEncBlock) ? (gcnt - sb * kEncBlock) : kEncBlock;
            load_sub(sb + 1, nxt);
            const uint32_t wblk = ((g0 + sb * kEncBlock) / 32u) * w;     // first bitstream word of this sub-block
#pragma unroll
            for (uint32_t it = 0; it < kEncIters; it++) {
                if (it * 1024 < cnt) {
                    const uint32_t i = it * 1024 + tid * 4;
                    const uint32_t pass_syms = (cnt - it * 1024 < 1024u) ? (cnt - it * 1024) : 1024u;
                    const uint32_t pass_words = (pass_syms * w + 31u) / 32u;
                    for (uint32_t k = tid; k < pass_words; k += kEncThreads) s_stage[k] = 0;
                    __syncthreads();
                    uint32_t pos = tid * 4 * w;
#pragma unroll
                    for (uint32_t j = 0; j < 4; j++) {
                        if (i + j < cnt && w) {
                            const uint32_t z = zz(raw[it][j]);
                            const uint32_t sh = pos & 31u, wi = pos >> 5;
                            atomicOr(&s_stage[wi], z << sh);
                            if (sh + w > 32u) atomicOr(&s_stage[wi + 1], z >> (32u - sh));
                            pos += w;
                        }
                    }
                    __syncthreads();
                    uint32_t* dst = bits + wblk + it * 32u * w;
                    for (uint32_t k = tid; k < pass_words; k += kEncThreads) dst[k] = s_stage[k];
                    __syncthreads();
                }
            }
#pragma unroll
            for (uint32_t it = 0; it < kEncIters; it++)
#pragma unroll
                for (uint32_t j = 0; j < 4; j++) raw[it][j] = nxt[it][j];
        }
        pad_frame();
        return;
    }

    // ---- HUFFMAN ----
    for (uint32_t s = tid; s < K; s += kEncThreads) {
        const uint32_t c = reinterpret_cast<const uint32_t*>(A.ws + A.L.book_code)[(size_t)frame * kMaxK + s];
        const uint32_t l = (A.ws + A.L.book_len)[(size_t)frame * kMaxK + s];
        s_book[s] = (uint64_t)c | ((uint64_t)l << 32);
    }
    for (uint32_t i = tid; i < kStageWords; i += kEncThreads) s_stage[i] = 0;
    const uint32_t start_bit = reinterpret_cast<const uint32_t*>(A.ws + A.L.grp_start)[blockIdx.x];
    const uint32_t c0 = start_bit & 31u;          // bits of the first word that belong to the previous workgroup
    const uint32_t w_first = start_bit >> 5;
    uint16_t* segt = reinterpret_cast<uint16_t*>(fr + M.segt_off);
    const uint32_t nseg = (nf + kSeg - 1) / kSeg;
    uint32_t run_bits = c0;                       // bits in front of the current sub-block, from stage origin
    uint32_t flushed = 0;                         // stage-origin words already written out
    __syncthreads();

    for (uint32_t sb = 0; sb < nsub; sb++) {
        const uint32_t cnt = (gcnt - sb * kEncBlock < kEncBlock) ? (gcnt - sb * kEncBlock) : kEncBlock;
        load_sub(sb + 1, nxt);
        uint64_t pk[kEncIters];                   // the thread's 4 symbols of a pass packed LSB-first
        uint32_t ln[kEncIters];                   // exclusive bit offset of the thread inside its pass
        uint32_t wide = 0;                        // pass mask: the 4 symbols need more than 64 bits
        // phase 1
#pragma unroll
        for (uint32_t it = 0; it < kEncIters; it++) {
            const uint32_t i = it * 1024 + tid * 4;
            uint64_t acc = 0;
            uint32_t tl = 0;
#pragma unroll
            for (uint32_t j = 0; j < 4; j++) {
                if (i + j < cnt) {
                    const uint32_t z = zz(raw[it][j]);
                    const uint32_t sy = sym_of(z, K);
                    const uint64_t b = s_book[sy];
                    if (tl < 64u) acc |= (uint64_t)(uint32_t)b << tl;
                    tl += (uint32_t)(b >> 32);
                    if (sy == 0) { if (tl < 64u) acc |= (uint64_t)z << tl; tl += 32u; }
                }
            }
            pk[it] = acc;
            wide |= (tl > 64u ? 1u : 0u) << it;
            const uint32_t incl = wave_incl_scan_dpp(tl);
            ln[it] = incl - tl;                                       // exclusive inside the wave's segment
            if (lane == 63) s_wtot[it * 4 + wave] = incl;             // bits of segment it*4 + wave
        }
        __syncthreads();
        uint32_t block_bits = 0;
#pragma unroll
        for (uint32_t it = 0; it < kEncIters; it++) {
            if (tid == 0) s_pbase[it] = block_bits;
#pragma unroll
            for (uint32_t w = 0; w < 4; w++) {
                const uint32_t t = s_wtot[it * 4 + w];
                if (w < wave) ln[it] += t;                                // now exclusive inside the pass
                block_bits += t;
            }
        }
        if (tid == 0) s_pbase[kEncIters] = block_bits;
        if (tid < kEncSegs) {
            const uint32_t gseg = (g0 + sb * kEncBlock) / kSeg + tid;
            if (gseg < nseg) segt[gseg] = (uint16_t)s_wtot[tid];
            if (gseg == nseg - 1 && (nseg & 1u)) segt[nseg] = 0;          // pad4 of the table
        }
        __syncthreads();

        // phase 2: as many passes at a time as fit the stage
        uint32_t it0 = 0;
        while (it0 < kEncIters && it0 * 1024 < cnt) {
            uint32_t it1 = it0 + 1;
            while (it1 < kEncIters && run_bits + s_pbase[it1 + 1] - 32u * flushed <= 32u * (kStageWords - 2)) it1++;
#pragma unroll
            for (uint32_t it = 0; it < kEncIters; it++) {
                if (it >= it0 && it < it1) {
                    const uint32_t i = it * 1024 + tid * 4;
                    uint32_t pos = run_bits + s_pbase[it] + ln[it] - 32u * flushed;
                    if (!((wide >> it) & 1u)) {
                        const uint64_t a = pk[it];
                        if (a) {
                            const uint32_t sh = pos & 31u, wi = pos >> 5;
                            const uint64_t t = a << sh;
                            atomicOr(&s_stage[wi], (uint32_t)t);
                            if ((uint32_t)(t >> 32)) atomicOr(&s_stage[wi + 1], (uint32_t)(t >> 32));
                            if (sh) { const uint32_t hi = (uint32_t)(a >> (64u - sh)); if (hi) atomicOr(&s_stage[wi + 2], hi); }
                        }
                    } else {
                        // the pass needs more than 64 bits (rare): emit symbol by symbol
#pragma unroll
                        for (uint32_t j = 0; j < 4; j++) {
                            if (i + j < cnt) {
                                const uint32_t z = zz(raw[it][j]);
                                const uint32_t sy = sym_of(z, K);
                                const uint64_t b = s_book[sy];
                                const uint32_t val = (uint32_t)b, len = (uint32_t)(b >> 32);
                                if (len) {
                                    const uint32_t sh = pos & 31u, wi = pos >> 5;
                                    atomicOr(&s_stage[wi], val << sh);
                                    if (sh + len > 32u) atomicOr(&s_stage[wi + 1], val >> (32u - sh));
                                    pos += len;
                                }
                                if (sy == 0) {
                                    const uint32_t sh = pos & 31u, wi = pos >> 5;
                                    atomicOr(&s_stage[wi], z << sh);
                                    if (sh) atomicOr(&s_stage[wi + 1], z >> (32u - sh));
                                    pos += 32u;
                                }
                            }
                        }
                    }
                }
            }
            __syncthreads();
            const uint32_t nbits = run_bits + s_pbase[it1] - 32u * flushed;  // bits now in the stage
            const uint32_t nw = nbits >> 5;
            const uint32_t wpos = w_first + flushed;
            for (uint32_t k = tid; k < nw; k += kEncThreads) {
                const uint32_t wv = s_stage[k];
                if (gb > 0 && flushed == 0 && k == 0) atomicOr(bits + wpos, wv);   // word shared with the previous workgroup
                else bits[wpos + k] = wv;
            }
            const uint32_t partial = s_stage[nw];
            __syncthreads();
            for (uint32_t k = tid; k <= nw + 2 && k < kStageWords; k += kEncThreads) s_stage[k] = (k == 0) ? partial : 0u;
            flushed += nw;
            it0 = it1;
            __syncthreads();
        }
        run_bits += block_bits;
#pragma unroll
        for (uint32_t it = 0; it < kEncIters; it++)
#pragma unroll
            for (uint32_t j = 0; j < 4; j++) raw[it][j] = nxt[it][j];
    }
    // the last, partial word: shared with the next workgroup, or the frame's last bitstream word
    if (tid == 0 && (run_bits & 31u)) {
        const uint32_t partial = s_stage[0];
        const uint32_t wpos = w_first + flushed;
        if (!last_grp || (gb > 0 && flushed == 0)) atomicOr(bits + wpos, partial);
        else bits[wpos] = partial;
    }
    pad_frame();
}

// ------------------------------------------------------------------------------------------------
// host launchers
// ------------------------------------------------------------------------------------------------
hipError_t launch_init(void* zero_base, size_t zero_bytes, void* res, uint32_t n_frames, uint32_t status,
                       hipStream_t st) {
    const size_t words = zero_bytes / 4;
    const uint32_t blocks = (uint32_t)((words + 255) / 256);
    hipLaunchKernelGGL(k_init, dim3(blocks ? blocks : 1), dim3(256), 0, st, reinterpret_cast<uint32_t*>(zero_base), words,
                       reinterpret_cast<ResultRec*>(res), n_frames, status);
    return hipGetLastError();
}

hipError_t launch_stats(const CompressArgs& A, hipStream_t st) {
    hipLaunchKernelGGL(k_stats, dim3(A.n_frames * A.sbpf), dim3(kStatThreads), 0, st, A);
    return hipGetLastError();
}

hipError_t launch_codebook(const CompressArgs& A, hipStream_t st) {
    hipLaunchKernelGGL(k_codebook, dim3(A.n_frames), dim3(kBookThreads), 0, st, A);
    return hipGetLastError();
}

hipError_t launch_encode(const CompressArgs& A, bool from_codes, hipStream_t st) {
    if (from_codes) hipLaunchKernelGGL(k_encode<1>, dim3(A.n_frames * A.sbpf), dim3(kEncThreads), 0, st, A);
    else hipLaunchKernelGGL(k_encode<0>, dim3(A.n_frames * A.sbpf), dim3(kEncThreads), 0, st, A);
    return hipGetLastError();
}

}  // namespace nz
