// nz_compress.hip -- gfx950 kernels of the sender side: frame statistics (quantize + zmax + histogram),
// per-frame codebook + exact-size selector + frame-offset look-back, and the bit-packing encoder.
//
// Paper mapping: interface quantizer (Sec. IV-B), runtime entropy arbitration with transmitted size as
// the cost (Sec. IV-C, Eq. 1-2, Algorithm 1), frame = header + payload (Sec. IV-D "Batch Framing").
// Unlike the paper's sampled estimate by one control thread, the statistics here cover the whole frame,
// so predicted and realized sizes coincide and Algorithm 1's post-validation never fires.
#include <type_traits>
#include "nz_common.hpp"
#include "nz_scan.hpp"

namespace nz {

// ------------------------------------------------------------------------------------------------
// K0: clear the control block / look-back descriptors and initialise the result record (decompress and reduce;
// nz_compress does this inside its statistics kernel)
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
// QM 0: deterministic error-bounded quantizer; 1: stochastic rounding to multiples of step.
// DELTA 1: the statistics are those of the differences q[i] - q[i-1] (modulo 2^32; q[i] itself at the start of every
// segment), which is what the entropy stage codes under the delta predictor.  A wavefront always covers exactly one
// segment (64 lanes x 4 consecutive values), so a thread gets its predecessor's last code from the lane below.
// SRC 0: fp32 input.  SRC 1 (reduce with the delta predictor): the integer sums staged by the adding pass.
template <int QM, int DELTA, int SRC>
__global__ __launch_bounds__(kStatThreads) void k_stats(CompressArgs A) {
    __shared__ uint32_t s_h[8192];
    __shared__ uint32_t s_zmax, s_unq;
    const uint32_t tid = threadIdx.x, lane = lane_id();
    if (SRC == 0 && blockIdx.x == 0) {
        // The control block, the frame descriptors and the result record are first used by the next kernel, so
        // this kernel clears them on the side (no separate launch): nothing here reads or writes them.
        uint32_t* z = reinterpret_cast<uint32_t*>(A.ws + A.L.ctrl);
        const uint32_t words = (uint32_t)((A.L.zero_end - A.L.ctrl) / 4);
        for (uint32_t i = tid; i < words; i += kStatThreads) z[i] = 0;
        if (tid == 0) {
            ResultRec* res = reinterpret_cast<ResultRec*>(A.res);
            res->bytes = 0; res->status = ST_OK; res->n_frames = A.n_frames;
            res->n_raw = 0; res->n_fixed = 0; res->n_huff = 0; res->reserved = 0;
        }
    }
    const uint32_t frame = blockIdx.x / A.sbpf, sb = blockIdx.x % A.sbpf;
    const uint64_t f0 = (uint64_t)frame * A.chunk;
    const uint32_t nf = (uint32_t)((A.n - f0 < A.chunk) ? (A.n - f0) : A.chunk);
    const uint32_t b0 = sb * kStatBlock;
    if (b0 >= nf) return;
    const uint32_t cnt = (nf - b0 < kStatBlock) ? (nf - b0) : kStatBlock;
    const uint32_t K = A.K;
    uint2* pm = reinterpret_cast<uint2*>(A.ws + A.L.pmeta) + blockIdx.x;
    if (SRC == 1 && (pm->y & 3u)) return;      // a frame with fp32 sums (RAW operand, local data not quantizable) has no codes
    // replicate the histogram over lanes: 8192/K copies (at most 32) so hot bins do not serialise
    uint32_t ncs = 0;
    while ((K << (ncs + 1)) <= 8192u && ncs < 5) ncs++;
    const uint32_t copy = lane & ((1u << ncs) - 1u);
    for (uint32_t i = tid; i < (K << ncs); i += kStatThreads) s_h[i] = 0;
    if (tid == 0) { s_zmax = 0; s_unq = 0; }
    __syncthreads();

    const float* src = A.in + f0 + b0;
    const int16_t* c16 = reinterpret_cast<const int16_t*>(A.ws + A.L.c16) + f0 + b0;         // SRC 1
    const uint32_t* c32 = reinterpret_cast<const uint32_t*>(A.ws + A.L.codes) + f0 + b0;
    const bool vec_ok = (((f0 + b0) & 3u) == 0);
    uint32_t zmax = 0, unq = 0;
    SrKeys keys;
    if (QM == 1) keys.init(A.seed, f0 + b0);
    // four consecutive codes of the block starting at position off (m of them exist); every lane of the wave calls this
    auto count4 = [&](const int32_t (&q)[4], uint32_t m) {
        uint32_t v[4] = { (uint32_t)q[0], (uint32_t)q[1], (uint32_t)q[2], (uint32_t)q[3] };
        if (DELTA) {
            const uint32_t below = (uint32_t)__shfl_up(q[3], 1, 64);
            const uint32_t prev = lane ? below : 0u;                  // lane 0 starts a segment
            v[3] -= v[2]; v[2] -= v[1]; v[1] -= v[0]; v[0] -= prev;
        }
#pragma unroll
        for (uint32_t j = 0; j < 4; j++) {
            if (j < m) {
                const uint32_t z = zigzag((int32_t)v[j]);
                zmax = z > zmax ? z : zmax;
                atomicAdd(&s_h[(bin_of(z, K) << ncs) + copy], 1u);
            }
        }
    };
    auto quant4 = [&](const float (&x)[4], uint32_t m, uint32_t off, int32_t (&q)[4]) {
#pragma unroll
        for (uint32_t j = 0; j < 4; j++) {
            q[j] = 0;
            if (j < m) {
                const bool okq = (QM == 1) ? sr_quantize1(x[j], A.step, A.inv_step, keys.draw(off + j), q[j])
                                           : quantize1(x[j], A.eb, A.step, A.inv_step, q[j]);
                if (!okq) unq = 1;
            }
        }
    };
    if (SRC == 0 && vec_ok && cnt == kStatBlock) {
        // whole block: eight 16-byte loads in flight per thread, no bounds checks
        constexpr uint32_t kIters = kStatBlock / (kStatThreads * 4), kDepth = 8;
        static_assert(kIters % kDepth == 0, "statistics block must be a whole number of load groups");
        const float4* src4 = reinterpret_cast<const float4*>(src) + tid;
#pragma unroll 1
        for (uint32_t g = 0; g < kIters; g += kDepth) {
            float4 t[kDepth];
#pragma unroll
            for (uint32_t u = 0; u < kDepth; u++) t[u] = src4[(g + u) * kStatThreads];
#pragma unroll
            for (uint32_t u = 0; u < kDepth; u++) {
                const float x[4] = { t[u].x, t[u].y, t[u].z, t[u].w };
                int32_t q[4];
                quant4(x, 4, ((g + u) * kStatThreads + tid) * 4u, q);
                count4(q, 4);
            }
        }
    } else {
        for (uint32_t base = 0; base < cnt; base += kStatThreads * 4) {      // (uniform trip count: count4 shuffles)
            const uint32_t i = base + tid * 4;
            const uint32_t m = (i < cnt) ? ((cnt - i < 4) ? (cnt - i) : 4u) : 0u;
            int32_t q[4];
            if (SRC == 0) {
                float x[4];
                for (uint32_t j = 0; j < 4; j++) x[j] = (j < m) ? src[i + j] : 0.0f;
                quant4(x, m, i, q);
            } else {
                for (uint32_t j = 0; j < 4; j++) {
                    q[j] = 0;
                    if (j < m) { const int32_t h = c16[i + j]; q[j] = (h == -32768) ? (int32_t)c32[i + j] : h; }
                }
            }
            count4(q, m);
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
        ph[bin_symbol(s, K)] = t;
    }
    if (tid == 0) {
        if (SRC == 1) pm->x = s_zmax;          // (the flags of the adding pass stay)
        else *pm = make_uint2(s_zmax, s_unq);
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

// Shared memory of the code construction (one workgroup of kBookThreads threads, thread = symbol).
struct BookShared {
    __align__(16) uint32_t key[kMaxK];
    uint32_t sorted[kMaxK];
    uint32_t w[2 * (kMaxK + 128)];    // leaves [0, m) + sentinels; internal nodes from kMaxK + 128, then sentinels
    uint16_t par[2 * kMaxK];
    __align__(4) uint8_t len[kMaxK];
    uint16_t rank[kMaxK];
    uint32_t wcnt[16 * 32], cnt[32], first[32], idx0[32];
    uint32_t m, nsym;
};

// Value of lane (lane ^ d), d a power of two (compile-time after unrolling); up = (lane & d) != 0.  Distances inside a row
// of 16 lanes go over the DPP network (quad permutes, or the row shifted both ways), the others through the LDS crossbar.
__device__ inline uint32_t lane_xor(uint32_t v, uint32_t d, bool up) {
    if (d == 1) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
    if (d == 2) return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
    if (d == 4) {
        const uint32_t below = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xF, 0xF, true);   // row_shr:4 = lane - 4
        const uint32_t above = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x104, 0xF, 0xF, true);   // row_shl:4 = lane + 4
        return up ? below : above;
    }
    if (d == 8) {
        const uint32_t below = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xF, 0xF, true);
        const uint32_t above = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x108, 0xF, 0xF, true);
        return up ? below : above;
    }
    return (uint32_t)__shfl_xor((int)v, (int)d, 64);
}

// Optimal prefix-code lengths and canonical codes for the counts f (one per thread = symbol; 0 = unused) of an
// alphabet of K symbols.  Called by all kBookThreads threads of the workgroup.  On return B.len[] holds the lengths,
// B.nsym = 1 + largest used symbol, and (L, code) are the calling thread's symbol's length and canonical code.
__device__ inline void book_build(BookShared& B, uint32_t f, uint32_t K, uint32_t& L_out, uint32_t& code_out) {
    const uint32_t tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    if (tid == 0) { B.m = 0; B.nsym = 0; }
    B.len[tid] = 0;
    __syncthreads();
    const bool used = f > 0;
    {
        const uint64_t um = __ballot(used);
        if (lane == 0 && um) { atomicAdd(&B.m, (uint32_t)__popcll(um)); atomicMax(&B.nsym, wave * 64 + 64 - (uint32_t)__clzll(um)); }
    }
    // (2) sort used symbols ascending by (count, symbol).  Every wavefront sorts its 64 keys with a bitonic network over
    // its lanes (unused symbols carry the largest key and end up last); a key's rank is then its place in its own run
    // plus, found by binary search, the number of smaller keys in every other run (keys are distinct).
    const uint32_t key = used ? ((f << 10) | tid) : 0xFFFFFFFFu;
    const uint32_t runs = K >= 64u ? K / 64u : 1u;            // K is a power of two; symbols past K do not exist
    uint32_t v = key;
    if (wave < runs) {
#pragma unroll
        for (uint32_t k = 2; k <= 64; k <<= 1) {
#pragma unroll
            for (uint32_t j = k >> 1; j >= 1; j >>= 1) {
                const bool up = (lane & j) != 0;
                const uint32_t vp = lane_xor(v, j, up);
                const bool asc = k == 64u || (lane & k) == 0;      // direction of this lane's block of k
                v = (up != asc) ? (v < vp ? v : vp) : (v > vp ? v : vp);
            }
        }
        B.key[tid] = v;                                       // run `wave`, place `lane`
    }
    __syncthreads();
    const uint32_t m = B.m;
    if (wave < runs && v != 0xFFFFFFFFu) {
        uint32_t rank = lane;
#pragma unroll 4
        for (uint32_t r = 0; r < runs; r++) {
            if (r == wave) continue;                          // (uniform over the wavefront)
            const uint32_t* run = B.key + r * 64u;
            uint32_t pos = 0;                                 // number of keys of the run below v
#pragma unroll
            for (uint32_t st = 32; st >= 1; st >>= 1) pos += (run[pos + st - 1u] < v) ? st : 0u;
            pos += (run[pos] < v) ? 1u : 0u;                  // (pos <= 63 before this probe)
            rank += pos;
        }
        B.sorted[rank] = v;
    }
    __syncthreads();
    // leaves in order, followed by sentinels; the internal-node queue starts out all sentinels
    constexpr uint32_t INF = 0xFFFFFFFFu;
    uint32_t* s_w = B.w;
    uint32_t* s_int = B.w + kMaxK + 128;
    uint16_t* s_par = B.par;
    if (tid < m) s_w[tid] = B.sorted[tid] >> 10;
    if (tid < 128) { s_w[m + tid] = INF; s_int[kMaxK + tid] = INF; }
    s_int[tid] = INF;
    __syncthreads();

    // (3) two-queue merge by wave 0, many steps per round.  The sequential construction picks, step after step, the two
    // smallest items of the leaf queue and the node queue (a leaf wins a weight tie against a node, nodes leave in the
    // order they were made) and appends their sum to the node queue.  New nodes never weigh less than older ones, so the
    // picks of the steps to come are simply the merged order of the remaining leaves and the nodes that exist now, up to
    // the point where the first node made in this round (weight T = the sum of the first pair) would be picked: that is,
    // all existing nodes and all leaves of weight <= T.  A round therefore merges a window of 64 leaves and 64 nodes --
    // packed keys weight << 11 | kind << 10 | index order exactly like the picks; an item counts only if no item
    // outside the window could precede it -- with a bitonic network over the wavefront, pairs consecutive items, and
    // lets lane j make node j of the round.  The first pair always qualifies, so every round makes progress; the result
    // is the sequential construction step for step, in a number of rounds that grows with the logarithm of the weight
    // range instead of the number of alternations between the queues.
    if (wave == 0 && m >= 2) {
        uint32_t ia = 0, ib = 0, nint = 0;                    // heads: leaf ia, internal node ib; nodes created
        while (nint + 1 < m) {
            const uint32_t left = m - 1 - nint;               // nodes still to be made
            const uint32_t lw = s_w[ia + lane], nwr = s_int[ib + 63u - lane];   // the windows (INF: no such leaf / node yet); nodes reversed
            const uint32_t lbeyond = s_w[ia + 64], nbeyond = s_int[ib + 64];    // first items outside the windows
            const uint32_t a0 = (uint32_t)__builtin_amdgcn_readlane((int)lw, 0), a1 = (uint32_t)__builtin_amdgcn_readlane((int)lw, 1);
            const uint32_t b0 = (uint32_t)__builtin_amdgcn_readlane((int)nwr, 63), b1 = (uint32_t)__builtin_amdgcn_readlane((int)nwr, 62);
            uint32_t T;                                       // weight of the first node of this round
            if (a0 <= b0) T = a0 + (a1 <= b0 ? a1 : b0); else T = b0 + (a0 <= b1 ? a0 : b1);
            const bool lv = lw <= T && lw <= nbeyond;         // (an equal node outside the window comes after the leaf)
            const bool nv = nwr != INF && nwr < lbeyond;      // (an equal leaf outside the window comes before the node)
            const uint32_t kl = lv ? ((lw << 11) | lane) : INF;
            const uint32_t knr = nv ? ((nwr << 11) | (1u << 10) | (63u - lane)) : INF;
            const uint32_t items = (uint32_t)__popcll(__ballot(lv)) + (uint32_t)__popcll(__ballot(nv));
            uint32_t P = items / 2u;                          // pairs of this round (at least 1)
            P = P < left ? P : left;
            // bitonic merge of the ascending leaf keys and the descending node keys
            uint32_t lo = kl < knr ? kl : knr, hi = kl < knr ? knr : kl;
#pragma unroll
            for (uint32_t d = 32; d >= 1; d >>= 1) {
                const bool up = (lane & d) != 0;
                const uint32_t plo = lane_xor(lo, d, up), phi = lane_xor(hi, d, up);
                lo = up ? (lo > plo ? lo : plo) : (lo < plo ? lo : plo);
                hi = up ? (hi > phi ? hi : phi) : (hi < phi ? hi : phi);
            }
            // merged item p sits in lo of lane p (p < 64) or hi of lane p - 64; items 2j and 2j + 1 make node j of the
            // round: the even lane of a pair writes the node, every lane the parent of its own item
            {
                const uint32_t qlo = lane_xor(lo, 1, (lane & 1u) != 0), qhi = lane_xor(hi, 1, (lane & 1u) != 0);
                const uint32_t jlo = lane >> 1, jhi = 32u + (lane >> 1);
                if (jlo < P) {
                    if (!(lane & 1u)) s_int[nint + jlo] = (lo >> 11) + (qlo >> 11);
                    s_par[((lo >> 10) & 1u) ? (m + ib + (lo & 1023u)) : (ia + (lo & 1023u))] = (uint16_t)(m + nint + jlo);   // (bits 0..9: index in its window)
                }
                if (jhi < P) {
                    if (!(lane & 1u)) s_int[nint + jhi] = (hi >> 11) + (qhi >> 11);
                    s_par[((hi >> 10) & 1u) ? (m + ib + (hi & 1023u)) : (ia + (hi & 1023u))] = (uint16_t)(m + nint + jhi);
                }
            }
            // heads: leaves and nodes among the first 2 P merged items
            const uint32_t cl = (uint32_t)__popcll(__ballot(lane < 2u * P && !((lo >> 10) & 1u))) +
                                (uint32_t)__popcll(__ballot(lane + 64u < 2u * P && !((hi >> 10) & 1u)));
            ia += cl; ib += 2u * P - cl; nint += P;
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
        B.len[B.sorted[tid] & 1023u] = (uint8_t)d;
    }
    __syncthreads();
    // (5) canonical codes
    canonical_tables<kBookThreads>(B.len, K, B.wcnt, B.cnt, B.first, B.idx0, B.rank);
    L_out = B.len[tid];
    code_out = L_out ? (B.first[L_out] + B.rank[tid]) : 0u;
}

__global__ __launch_bounds__(kBookThreads) void k_codebook(CompressArgs A) {
    __shared__ uint32_t s_f[kMaxK];
    __shared__ BookShared s_b;
    __shared__ uint64_t s_part[16];
    __shared__ uint32_t s_fid, s_zmax, s_unq, s_codec, s_payload, s_total, s_w_fixed, s_skip;
    __shared__ uint64_t s_bits, s_off;
    uint32_t* const s_w = s_b.w;
    uint8_t* const s_len = s_b.len;

    const uint32_t tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const uint32_t K = A.K;
    Ctrl* ctrl = reinterpret_cast<Ctrl*>(A.ws + A.L.ctrl);
    if (tid == 0) { s_fid = atomicAdd(&ctrl->ticket_book, 1u); s_zmax = 0; s_unq = 0; }
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
    if (tid < sbc) {
        const uint2 pm = reinterpret_cast<const uint2*>(A.ws + A.L.pmeta)[(size_t)fid * A.sbpf + tid];
        atomicMax(&s_zmax, pm.x);
        atomicMax(&s_unq, pm.y);
        // reduce: a sum beyond 2^30 somewhere in the frame has turned it RAW (its fp32 sums were staged by k_fix)
        if (!A.in) atomicMax(&s_unq, reinterpret_cast<const uint32_t*>(A.ws + A.L.cwide)[(size_t)fid * A.sbpf + tid] & 2u);
    }
    __syncthreads();
    // Frames that cannot end up HUFFMAN skip the code construction (most of this kernel's latency): a frame that is
    // RAW anyway, a pinned RAW / FIXEDLEN, and a frame whose HUFFMAN bitstream is bound to be at least as long as
    // FIXEDLEN's -- every symbol costs a bit and every escape 32 more, so bits >= n_f + 32 * escapes; if that reaches
    // n_f * w, HUFFMAN's payload (tables on top) exceeds FIXEDLEN's and FIXEDLEN, the lower codec id, wins any tie,
    // while a gate that rejects FIXEDLEN's payload rejects the larger one too.
    if (tid == 0) {
        const uint32_t zmax = s_zmax;
        const uint64_t w = zmax ? (32u - (uint32_t)__clz(zmax)) : 0u;
        bool skip = s_unq != 0;
        if (A.force_codec >= 0) skip = skip || A.force_codec != (int32_t)CODEC_HUFF;
        else skip = skip || ((uint64_t)nf + 32ull * s_f[0] >= (uint64_t)nf * w);
        s_skip = skip ? 1u : 0u;
    }
    __syncthreads();
    const bool skip = s_skip != 0;
    // (2)-(5) code lengths and canonical codes
    uint32_t L = 0, code = 0, nsym = 0;
    if (!skip) {
        book_build(s_b, f, K, L, code);
        nsym = s_b.nsym;
        // (6) exact Huffman bitstream length: sum f*len, an escape carries 32 more bits
        uint64_t b = (uint64_t)f * L + (tid == 0 ? 32ull * f : 0ull);
        b = wave_sum64(b);
        if (lane == 0) s_part[wave] = b;
    }
    __syncthreads();
    // (7) sizes and arbitration (Eq. 2: argmin of frame bytes over RAW + admissible codecs, ties to the lower id)
    if (tid == 0) {
        uint64_t bits = skip ? (1ull << 40) : 0ull;               // (skipped: larger than any RAW payload, never admissible)
        if (!skip) for (int i = 0; i < 16; i++) bits += s_part[i];
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
        M.pad_ = (!A.in && s_unq) ? 1u : 0u;      // reduce: the frame's fp32 sums are staged, there are no integer sums
        M.huff_bits = s_bits; M.pad2_ = 0;
        reinterpret_cast<FrameMeta*>(A.ws + A.L.meta)[fid] = M;
        if (fits) {
            uint32_t h[8];
            h[0] = kMagicFrame; h[1] = codec; h[2] = 4u * nf; h[3] = payload;
            h[4] = (codec == CODEC_FIXED) ? s_w_fixed : (codec == CODEC_HUFF ? nsym : 0u);
            h[5] = (codec == CODEC_HUFF) ? (kSeg | (K << 16) | (A.pred << 31)) : (codec == CODEC_FIXED ? (A.pred << 31) : 0u);
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
            sh[4] = A.chunk; sh[5] = A.n_frames; sh[6] = A.step_bits; sh[7] = kSeg; sh[8] = K; sh[9] = A.pred;
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
// K4: encoder.  One workgroup per group of kEncGroup symbols of one frame (a whole number of statistics
// blocks), worked through in sub-blocks of kEncBlock symbols.
//   RAW      copy the words.
//   FIXEDLEN w bits per zigzag code at closed-form positions (a pass of 1024 codes is 32*w whole words).
//   HUFFMAN  the group's first bit in the frame's bitstream comes from the codebook kernel, so there is no
//            scan and no waiting between workgroups.  Per sub-block: phase 1 looks every symbol up once,
//            packs the 4 symbols of a thread (codes, and the 32 raw bits of an escape) into 64 bits and scans
//            the bit counts on the DPP network (segment table entries fall out of the scan); the source words
//            of the next sub-block are requested as soon as phase 1 has used the current ones; phase 2 ORs
//            the packed strings into an LDS stage at their final bit positions; whole words are then flushed
//            coalesced while the partial last word moves on to the other of two stages, which makes two
//            barriers per sub-block enough.  The word in which two groups meet was cleared by the codebook
//            kernel and receives both parts by atomic OR; every other word has a single writer.
// SRC = 0: symbols are quantized from the fp32 input; SRC = 1: symbols are the int32 codes staged in the
// workspace by the reduce front end (RAW frames hold fp32 bit patterns there).
// ------------------------------------------------------------------------------------------------
constexpr uint32_t kStageWords = 2048;        // one stage holds a sub-block of up to ~16 bits per symbol at once

struct EncShared {
    uint64_t book[kMaxK];                      // by min(z, K-1): reversed code | length << 32; entry K-1 = escape
    uint32_t stage[2][kStageWords + 4];
    __align__(16) uint32_t wtot[kEncSegs];     // bit count of each of the sub-block's segments
};

// zigzag code of a source word.  Sources 0 and 1: only coded (FIXEDLEN / HUFFMAN) frames come here, and a frame is
// coded only if the statistics pass found every element quantizable, so the acceptance tests of the quantizer are
// known to pass and q is simply rne(x * inv_step).  Source 2 (sampled arbitration): nothing has looked at the values
// before, so the quantizer runs with its tests; a value that fails them counts as code 0 and clears *ok.
// QM = 1 (source 0 only): the stochastic quantizer, with the draw of the element (its tests are known to pass too).
// Sources 1 and 3 take their symbols from the sums a reduce staged; sources 2 and 3 are the sampled arbitration (the
// context's code, every group materialised from bit 0, realized sizes reported to the finishing kernel).
constexpr bool src_codes(int SRC) { return SRC == 1 || SRC == 3; }
constexpr bool src_rea(int SRC) { return SRC == 2 || SRC == 3; }

template <int SRC, int QM = 0>
__device__ inline int32_t enc_q(uint32_t w, const CompressArgs& A, bool* ok = nullptr, uint32_t draw24 = 0) {
    if (SRC == 0 && QM == 1) {
        int32_t q;
        sr_quantize1(__uint_as_float(w), A.step, A.inv_step, draw24, q);
        return q;
    }
    if (SRC == 0) {
#pragma clang fp contract(off)
        const float u = __uint_as_float(w) * A.inv_step;
        return (int32_t)__builtin_rintf(u);
    }
    if (SRC == 2) {
        int32_t q;
        const bool good = quantize1(__uint_as_float(w), A.eb, A.step, A.inv_step, q);
        if (ok && !good) *ok = false;
        return q;
    }
    return (int32_t)w;
}
template <int SRC, int QM = 0>
__device__ inline uint32_t enc_zz(uint32_t w, const CompressArgs& A, bool* ok = nullptr, uint32_t draw24 = 0) {
    return zigzag(enc_q<SRC, QM>(w, A, ok, draw24));
}
// Delta predictor: four consecutive codes of one thread become differences to their predecessors (modulo 2^32).
// A wavefront's 64 x 4 values are exactly one segment, so the predecessor of a thread's first code is the last code
// of the lane below, and lane 0 starts the segment with the code itself.  Every lane of the wave must call this.
__device__ inline void delta4(int32_t (&q)[4]) {
    const uint32_t below = (uint32_t)__shfl_up(q[3], 1, 64);
    const uint32_t prev = lane_id() ? below : 0u;
    const uint32_t v0 = (uint32_t)q[0], v1 = (uint32_t)q[1], v2 = (uint32_t)q[2], v3 = (uint32_t)q[3];
    q[0] = (int32_t)(v0 - prev); q[1] = (int32_t)(v1 - v0); q[2] = (int32_t)(v2 - v1); q[3] = (int32_t)(v3 - v2);
}
// Geometry of one encode workgroup.
struct EncGroup {
    const uint32_t* src;      // first 32-bit source word of the group (fp32 input; reduce: wide sums, fp32 sums of RAW frames)
    const int16_t* src16;     // reduce: the group's sums as 16-bit codes, -32768 = "needs 32 bits, look in src"
    uint32_t g0, gcnt, nf, nsub, gb;
    bool vec_ok, last_grp, wide16;   // wide16: the group's 16-bit codes contain markers
};

// Source word i of the group: fp32 bits (SRC 0) or the summed code (SRC 1, coded frames).
template <int SRC>
__device__ inline uint32_t enc_word(const EncGroup& G, uint32_t i) {
    if (!src_codes(SRC)) return G.src[i];
    const int32_t q = G.src16[i];
    return (q == -32768) ? G.src[i] : (uint32_t)q;
}

// The coded value of group element i, the slow way (the element and, under the delta predictor, the one before it).
template <int SRC, int QM, int DELTA>
__device__ inline uint32_t enc_zz_at(const EncGroup& G, const CompressArgs& A, const SrKeys& keys, uint32_t i) {
    int32_t q = enc_q<SRC, QM>(enc_word<SRC>(G, i), A, nullptr, QM ? keys.draw(i) : 0u);
    if (DELTA && (i & (kSeg - 1u))) q = (int32_t)((uint32_t)q - (uint32_t)enc_q<SRC, QM>(enc_word<SRC>(G, i - 1u), A, nullptr, 0u));
    return zigzag(q);
}

// Source words of sub-block sb: pass `it` covers its symbols it*1024 + tid*4 .. +3 (zero past the end).
template <int SRC>
__device__ inline void enc_load(const EncGroup& G, uint32_t sb, uint32_t (&raw)[kEncIters][4]) {
    const uint32_t tid = threadIdx.x;
    const uint32_t* src = G.src + sb * kEncBlock;
    const uint32_t cnt = (sb < G.nsub) ? ((G.gcnt - sb * kEncBlock < kEncBlock) ? (G.gcnt - sb * kEncBlock) : kEncBlock) : 0u;
    if (G.vec_ok && cnt == kEncBlock && (!src_codes(SRC) || !G.wide16)) {       // uniform: the common, branch-free case
#pragma unroll
        for (uint32_t it = 0; it < kEncIters; it++) {
            if (!src_codes(SRC)) {
                const uint4 t = *reinterpret_cast<const uint4*>(src + it * 1024 + tid * 4);
                raw[it][0] = t.x; raw[it][1] = t.y; raw[it][2] = t.z; raw[it][3] = t.w;
            } else {
                const uint2 t = *reinterpret_cast<const uint2*>(G.src16 + sb * kEncBlock + it * 1024 + tid * 4);
                raw[it][0] = (uint32_t)(int32_t)(int16_t)(t.x & 0xFFFFu); raw[it][1] = (uint32_t)((int32_t)t.x >> 16);
                raw[it][2] = (uint32_t)(int32_t)(int16_t)(t.y & 0xFFFFu); raw[it][3] = (uint32_t)((int32_t)t.y >> 16);
            }
        }
    } else {
#pragma unroll 1
        for (uint32_t it = 0; it < kEncIters; it++) {
            const uint32_t i = it * 1024 + tid * 4;
            uint32_t t[4];
#pragma unroll
            for (uint32_t j = 0; j < 4; j++) t[j] = (i + j < cnt) ? enc_word<SRC>(G, sb * kEncBlock + i + j) : 0u;
#pragma unroll
            for (uint32_t q = 0; q < kEncIters; q++)
                if (q == it) { raw[q][0] = t[0]; raw[q][1] = t[1]; raw[q][2] = t[2]; raw[q][3] = t[3]; }
        }
    }
}

// Reduce, a frame of integer sums that the selector commits RAW (codec pinned to RAW, no entropy candidate passes the
// gates, a width of 32 bits): like every RAW frame of a reduce it holds fl(fl(qa*step) + fl(qb*step)), the sums of the
// two dequantized operands (RAW is the fallback every frame can take, Sec. IV-C).  The operands are recovered from the
// staged sums Q: two streams -- qa from the staged codes of operand A, qb = Q - qa; ring step -- qb is the rank's own
// value quantized again (it was quantizable, or the frame would have no integer sums), qa = Q - qb.
__device__ inline void enc_raw_sums(const CompressArgs& A, const EncGroup& G, uint64_t f0, uint8_t* fr) {
#pragma clang fp contract(off)
    StageA sa;
    sa.a16 = reinterpret_cast<int16_t*>(A.ws + A.L.a16); sa.a32 = reinterpret_cast<uint32_t*>(A.ws + A.L.a32);
    uint32_t* dst = reinterpret_cast<uint32_t*>(fr + kHdrBytes) + G.g0;
    for (uint32_t i = threadIdx.x; i < G.gcnt; i += kEncThreads) {
        const int32_t Q = (int32_t)enc_word<1>(G, i);
        int32_t qa, qb;
        if (A.red_local) {
            const uint64_t g = f0 + G.g0 + i;
            const float x = A.red_local[g];
            if (A.red_sr) sr_quantize1(x, A.step, A.inv_step, sr_draw(sr_key(A.seed, g), (uint32_t)g), qb);
            else quantize1(x, A.eb, A.step, A.inv_step, qb);
            qa = (int32_t)((uint32_t)Q - (uint32_t)qb);
        } else {
            qa = (int32_t)sa.get(f0, G.nf, G.g0 + i, false);
            qb = (int32_t)((uint32_t)Q - (uint32_t)qa);
        }
        const float sum = dequantize1(qa, A.step) + dequantize1(qb, A.step);
        dst[i] = (sum != sum) ? kCanonNaN : __float_as_uint(sum);
    }
}

template <int SRC, int QM, int DELTA>
__device__ inline void enc_raw_fixed(const CompressArgs& A, const EncGroup& G, const FrameMeta& M, uint8_t* fr, uint32_t* stage,
                                     uint32_t& bad, const SrKeys& keys) {
    const uint32_t tid = threadIdx.x;
    if (M.codec == CODEC_RAW) {
        uint32_t* dst = reinterpret_cast<uint32_t*>(fr + kHdrBytes) + G.g0;
        for (uint32_t i = tid * 4; i < G.gcnt; i += kEncThreads * 4) {
            if (G.vec_ok && i + 4 <= G.gcnt) *reinterpret_cast<uint4*>(dst + i) = *reinterpret_cast<const uint4*>(G.src + i);
            else for (uint32_t j = 0; j < 4; j++) if (i + j < G.gcnt) dst[i + j] = G.src[i + j];
        }
        return;
    }
    // FIXEDLEN: a pass of 1024 codes is 32*w whole words.  The codes of up to four passes (as many as fit a stage) are
    // ORed into one of two LDS stages at their bit positions; after a barrier the words are written out coalesced and
    // cleared, while the next round already fills the other stage (a stage is used again two rounds later, behind the
    // barrier in between): one barrier per round.  The source words of the next pass are requested before the current
    // ones are worked on.
    const uint32_t w = M.w;
    uint32_t* bits = reinterpret_cast<uint32_t*>(fr + M.bits_off) + (G.g0 / 32u) * w;
    constexpr uint32_t kStage2 = kStageWords + 4;                        // the second stage follows the first
    static_assert(kStageWords == 2048, "the passes per round below are sized for stages of 2048 words");
    const uint32_t ppr = (w <= 16u) ? 4u : (w <= 21u ? 3u : 2u);          // passes per round: ppr * 32 * w <= 2048 words
    for (uint32_t k = tid; k < kStageWords + 1u; k += kEncThreads) { stage[k] = 0; stage[kStage2 + k] = 0; }
    // source words of the thread's four codes in the pass that starts at p0 (zero past the end)
    auto load4 = [&](uint32_t p0, uint32_t (&x)[4]) {
        const uint32_t i = p0 + tid * 4;
        x[0] = x[1] = x[2] = x[3] = 0;
        if (i >= G.gcnt) return;
        if (G.vec_ok && i + 4 <= G.gcnt && (!src_codes(SRC) || !G.wide16)) {
            if (!src_codes(SRC)) {
                const uint4 t = *reinterpret_cast<const uint4*>(G.src + i);
                x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
            } else {
                const uint2 t = *reinterpret_cast<const uint2*>(G.src16 + i);
                x[0] = (uint32_t)(int32_t)(int16_t)(t.x & 0xFFFFu); x[1] = (uint32_t)((int32_t)t.x >> 16);
                x[2] = (uint32_t)(int32_t)(int16_t)(t.y & 0xFFFFu); x[3] = (uint32_t)((int32_t)t.y >> 16);
            }
        } else {
            for (uint32_t j = 0; j < 4; j++) if (i + j < G.gcnt) x[j] = enc_word<SRC>(G, i + j);
        }
    };
    uint32_t cur[4], nxt[4];
    load4(0, nxt);
    __syncthreads();
    uint32_t ri = 0;
    for (uint32_t r0 = 0; r0 < G.gcnt; r0 += ppr * 1024u, ri++) {
        const uint32_t round_syms = (G.gcnt - r0 < ppr * 1024u) ? (G.gcnt - r0) : ppr * 1024u;
        const uint32_t round_words = (round_syms * w + 31u) / 32u;
        uint32_t* buf = stage + (ri & 1u) * kStage2;
        for (uint32_t u = 0; u < ppr; u++) {
            const uint32_t p0 = r0 + u * 1024u;
            if (p0 >= G.gcnt) break;
            const uint32_t pass_syms = (G.gcnt - p0 < 1024u) ? (G.gcnt - p0) : 1024u;
#pragma unroll
            for (uint32_t j = 0; j < 4; j++) cur[j] = nxt[j];
            load4(p0 + 1024u, nxt);
            int32_t q[4];
#pragma unroll
            for (uint32_t j = 0; j < 4; j++) {
                bool ok = true;
                q[j] = enc_q<SRC, QM>(cur[j], A, &ok, QM ? keys.draw(p0 + tid * 4 + j) : 0u);     // (words past the end are 0)
                if (src_rea(SRC) && tid * 4 + j < pass_syms && !ok) bad = 1;
            }
            if (DELTA) delta4(q);                     // (a pass is four whole segments, one per wave)
            uint32_t pos = (u * 1024u + tid * 4u) * w;
#pragma unroll
            for (uint32_t j = 0; j < 4; j++) {
                uint32_t z = zigzag(q[j]);
                if (tid * 4 + j < pass_syms && w) {
                    if (src_rea(SRC) && w < 32u && (z >> w)) { bad = 1; z &= (1u << w) - 1u; }   // wider than the sampled width
                    const uint32_t sh = pos & 31u, wi = pos >> 5;
                    atomicOr(&buf[wi], z << sh);
                    if (sh + w > 32u) atomicOr(&buf[wi + 1], z >> (32u - sh));
                    pos += w;
                } else if (src_rea(SRC) && tid * 4 + j < pass_syms && z) bad = 1;               // (sampled width 0, value not 0)
            }
        }
        __syncthreads();
        uint32_t* dst = bits + (r0 / 32u) * w;
        for (uint32_t k = 4u * tid; k < round_words; k += 4u * kEncThreads) {     // 16 bytes per thread and step
            if (k + 4u <= round_words) {
                const uint4 v = *reinterpret_cast<const uint4*>(buf + k);
                *reinterpret_cast<uint4*>(buf + k) = make_uint4(0u, 0u, 0u, 0u);
                *reinterpret_cast<uint4*>(dst + k) = v;
            } else {
                for (uint32_t kk = k; kk < round_words; kk++) { dst[kk] = buf[kk]; buf[kk] = 0; }
            }
        }
    }
}

// Sampled arbitration, ProfileSample + ArbitratePlan (Sec. IV-C, Algorithm 1), run by every encoder workgroup of a frame
// for itself (the sample is at most 64 KiB and hot in L2 after its first reader; a kernel of its own would cost more
// than the repeated profiling).  The sample is the frame's prefix; FIXEDLEN's width is the bit length of the sample's
// largest zigzag code, HUFFMAN's size the sample's bits under the context scaled to the frame (rounded up);
// admissibility (fits the payload capacity = RAW size, minimum gain, context valid, T_huff) and Eq. 2 with transmitted
// size as the cost, ties to the lower codec id.  Leaves the context's code in S.book when the context is valid.  The
// frame's first group also writes the plan, the frame's entry of the offsets table (slots are fixed) and, for frame 0,
// the stream header and the cleared result record, for the finishing kernel.
// Source 3 (the ring step): the frame exists as integer sums staged by the adding pass, the sample is their prefix and
// every code is codable; a frame that has no integer sums (an operand RAW, a sum out of range: flags of the adding
// pass) is RAW without arbitration and holds the fp32 sums staged for it.
template <int SRC>
__device__ inline FrameMeta rea_plan_frame(const CompressArgs& A, uint32_t frame, uint64_t f0, uint32_t nf, uint32_t gb, EncShared& S) {
    const uint32_t tid = threadIdx.x, lane = lane_id(), wave = tid >> 6, K = A.K;
    const bool ctx_ok = A.rea_ctx && A.rea_ctx->valid == 1u && A.rea_ctx->K == K;
    const uint64_t base = kStreamHdr + pad16u(8ull * A.n_frames);
    uint32_t* s_red = S.wtot;                    // [0] largest zigzag code, [1] unquantizable flag, [2..9] the waves' bit sums
    static_assert(kEncSegs >= 10 && kEncThreads == 256, "the reduction scratch of the plan fits the segment totals");
    if (tid == 0) {
        s_red[0] = 0; s_red[1] = 0;
        A.rea_fail[(size_t)frame * A.sbpf + gb] = 0;
        if (gb == 0) {
            *reinterpret_cast<uint64_t*>(A.out + kStreamHdr + 8ull * frame) = base + (uint64_t)frame * A.rea_slot;
            if (frame == A.n_frames - 1 && (A.n_frames & 1u)) *reinterpret_cast<uint64_t*>(A.out + kStreamHdr + 8ull * A.n_frames) = 0;
            if (frame == 0) {
                ReaResultRec* res = reinterpret_cast<ReaResultRec*>(A.res);
                res->span_bytes = 0; res->wire_bytes = 0; res->status = ST_OK; res->n_frames = A.n_frames;
                res->n_raw = 0; res->n_fixed = 0; res->n_huff = 0; res->n_fallback = 0;
                uint32_t* sh = reinterpret_cast<uint32_t*>(A.out);
                sh[0] = kMagicStream; sh[1] = 1u; sh[2] = (uint32_t)A.n; sh[3] = (uint32_t)(A.n >> 32);
                sh[4] = A.chunk; sh[5] = A.n_frames; sh[6] = A.step_bits; sh[7] = kSeg; sh[8] = K; sh[9] = 0;
                sh[10] = 0; sh[11] = 0; sh[12] = 0; sh[13] = 0; sh[14] = 0; sh[15] = 0;     // total_bytes: the finishing kernel
            }
        }
    }
    if (ctx_ok) for (uint32_t b = tid; b < K; b += kEncThreads) S.book[b] = A.rea_ctx->book[b];
    __syncthreads();
    const uint64_t rawb = 4ull * nf;
    const bool profiled = rawb >= A.rea_small_batch_bytes;               // SmallBatchFastPath
    const uint32_t n_s = profiled ? (A.rea_sample_elems < nf ? A.rea_sample_elems : nf) : 0u;
    uint32_t zmax = 0, bad = 0;
    uint64_t bits = 0;
    auto profile1 = [&](float x) {
        int32_t q;
        if (!quantize1(x, A.eb, A.step, A.inv_step, q)) bad = 1;
        const uint32_t z = zigzag(q);
        zmax = z > zmax ? z : zmax;
        if (ctx_ok) { const uint32_t b = bin_of(z, K); bits += (uint32_t)(S.book[b] >> 32) + (b == K - 1u ? 32u : 0u); }
    };
    if (SRC == 3) {
        const int16_t* c16 = reinterpret_cast<const int16_t*>(A.ws + A.L.c16) + f0;
        const uint32_t* c32 = reinterpret_cast<const uint32_t*>(A.ws + A.L.codes) + f0;
        const uint32_t hpf = A.sbpf, halves = (nf + kEncGroup - 1) / kEncGroup;
        if (tid < halves && tid < hpf) {          // no integer sums in this frame?
            const uint32_t y = reinterpret_cast<const uint2*>(A.ws + A.L.pmeta)[(size_t)frame * hpf + tid].y;
            const uint32_t cw = reinterpret_cast<const uint32_t*>(A.ws + A.L.cwide)[(size_t)frame * hpf + tid];
            if ((y & 3u) || (cw & 2u)) bad = 1;
        }
        auto profile_code = [&](int32_t h, uint32_t k) {
            const uint32_t z = zigzag(h == -32768 ? (int32_t)c32[k] : h);
            zmax = z > zmax ? z : zmax;
            if (ctx_ok) { const uint32_t b = bin_of(z, K); bits += (uint32_t)(S.book[b] >> 32) + (b == K - 1u ? 32u : 0u); }
        };
        uint32_t k0 = 0;
        if ((f0 & 7u) == 0) {                    // eight 16-bit codes per 16-byte load, up to eight loads in flight per thread
            constexpr uint32_t kBatch = 8 * kEncThreads * 8;
            for (; k0 < (n_s & ~7u); k0 += kBatch) {
                uint4 t[8];
#pragma unroll
                for (uint32_t u = 0; u < 8; u++) {
                    const uint32_t k = k0 + (u * kEncThreads + tid) * 8u;
                    t[u] = (k + 8u <= n_s) ? *reinterpret_cast<const uint4*>(c16 + k) : make_uint4(0u, 0u, 0u, 0u);
                }
#pragma unroll
                for (uint32_t u = 0; u < 8; u++) {
                    const uint32_t k = k0 + (u * kEncThreads + tid) * 8u;
                    if (k + 8u <= n_s) {
                        const uint32_t wds[4] = { t[u].x, t[u].y, t[u].z, t[u].w };
#pragma unroll
                        for (uint32_t j = 0; j < 4; j++) {
                            profile_code((int32_t)(int16_t)(wds[j] & 0xFFFFu), k + 2u * j);
                            profile_code((int32_t)wds[j] >> 16, k + 2u * j + 1u);
                        }
                    }
                }
            }
            k0 = n_s & ~7u;
        }
        for (uint32_t k = k0 + tid; k < n_s; k += kEncThreads) profile_code(c16[k], k);
    }
    const float* sp = A.in + f0;
    uint32_t i = (SRC == 3) ? n_s : 0u;
    if (SRC != 3 && (f0 & 3u) == 0) {            // eight 16-byte loads in flight per thread
        constexpr uint32_t kBatch = 8 * kEncThreads * 4;
        for (; i + kBatch <= n_s; i += kBatch) {
            float4 t[8];
#pragma unroll
            for (uint32_t u = 0; u < 8; u++) t[u] = reinterpret_cast<const float4*>(sp + i)[u * kEncThreads + tid];
#pragma unroll
            for (uint32_t u = 0; u < 8; u++) { profile1(t[u].x); profile1(t[u].y); profile1(t[u].z); profile1(t[u].w); }
        }
    }
    for (uint32_t k = i + tid; k < n_s; k += kEncThreads) profile1(sp[k]);
    zmax = wave_max(zmax); bad = wave_max(bad); bits = wave_sum64(bits);
    if (lane == 0) { atomicMax(&s_red[0], zmax); atomicMax(&s_red[1], bad); reinterpret_cast<uint64_t*>(s_red + 2)[wave] = bits; }
    __syncthreads();
    // every thread draws the same conclusion from the same numbers
    uint32_t plan = CODEC_RAW;
    const uint32_t zm = s_red[0];
    const uint32_t w = zm ? (32u - (uint32_t)__clz(zm)) : 0u;
    const uint32_t nseg = (nf + kSeg - 1) / kSeg;
    if (n_s && !s_red[1]) {                      // (source 3: the flag also stands for "no integer sums")
        const uint64_t* wb = reinterpret_cast<const uint64_t*>(s_red + 2);
        const uint64_t sample_bits = wb[0] + wb[1] + wb[2] + wb[3];
        const uint64_t pred_bits = (sample_bits * nf + n_s - 1) / n_s;
        uint64_t pay[3];
        pay[CODEC_RAW] = rawb;
        pay[CODEC_FIXED] = 4ull * (((uint64_t)nf * w + 31u) / 32u);
        pay[CODEC_HUFF] = pad4u(K) + pad4u(2ull * nseg) + 4ull * ((pred_bits + 31u) / 32u);
        if (A.force_codec >= 0) plan = (A.force_codec == (int32_t)CODEC_HUFF && !ctx_ok) ? (uint32_t)CODEC_RAW : (uint32_t)A.force_codec;
        else {
            // Eq. 1 in picoseconds under the caller's transport hint (no hint: the predicted total bytes)
            auto cost = [&](uint32_t c, uint64_t total) -> uint64_t {
                if (A.rea_link_ps == 0u) return total;
                uint64_t t = (uint64_t)A.rea_link_ps * total;
                if (c == CODEC_FIXED) t += 1000ull * A.rea_fixed_alpha_ns + (uint64_t)A.rea_fixed_ps * rawb;
                if (c == CODEC_HUFF) t += 1000ull * A.rea_huff_alpha_ns + (uint64_t)A.rea_huff_ps * rawb;
                return t;
            };
            uint64_t best_cost = cost(CODEC_RAW, pad16u(kHdrBytes + rawb));
            for (uint32_t c = CODEC_FIXED; c <= CODEC_HUFF; c++) {
                if (c == CODEC_HUFF && (!ctx_ok || rawb < A.huff_min_bytes)) continue;
                if (pay[c] > rawb) continue;
                if ((rawb - pay[c]) * 1000ull < (uint64_t)A.min_gain_permil * rawb) continue;
                const uint64_t t = cost(c, pad16u(kHdrBytes + pay[c]));
                if (t < best_cost) { best_cost = t; plan = c; }
            }
        }
    }
    FrameMeta M;
    M.offset = base + (uint64_t)frame * A.rea_slot; M.total = 0; M.payload = 0; M.codec = plan; M.w = w; M.nsym = K; M.fits = 1u;
    M.segt_off = kHdrBytes + (uint32_t)pad4u(K);
    M.bits_off = (plan == CODEC_HUFF) ? (M.segt_off + (uint32_t)pad4u(2ull * nseg)) : kHdrBytes;
    M.bits_words = 0; M.pad_ = (SRC == 3 && s_red[1]) ? 1u : 0u; M.huff_bits = 0; M.pad2_ = 0;
    if (gb == 0 && tid == 0) reinterpret_cast<FrameMeta*>(A.ws + A.L.meta)[frame] = M;
    __syncthreads();                             // the scratch is the encoder's again
    return M;
}

template <int SRC, int QM = 0, int DELTA = 0>
__global__ __launch_bounds__(kEncThreads) __attribute__((amdgpu_waves_per_eu(4))) void k_encode(CompressArgs A) {
    __shared__ EncShared S;
    const uint32_t tid = threadIdx.x, lane = lane_id(), wave = tid >> 6;
    const uint32_t gpf = (A.chunk + kEncGroup - 1) / kEncGroup;
    const uint32_t frame = blockIdx.x / gpf;
    EncGroup G;
    G.gb = blockIdx.x % gpf;
    const uint64_t f0 = (uint64_t)frame * A.chunk;
    G.nf = (uint32_t)((A.n - f0 < A.chunk) ? (A.n - f0) : A.chunk);
    G.g0 = G.gb * kEncGroup;                                             // first symbol of this group in the frame
    if (G.g0 >= G.nf) return;
    G.gcnt = (G.nf - G.g0 < kEncGroup) ? (G.nf - G.g0) : kEncGroup;
    G.last_grp = (G.g0 + G.gcnt == G.nf);
    G.nsub = (G.gcnt + kEncBlock - 1) / kEncBlock;
    // source words: fp32 input (SRC 0, 2) or the staged codes / fp32 sums of the reduce (SRC 1)
    G.src = (!src_codes(SRC) ? reinterpret_cast<const uint32_t*>(A.in) : reinterpret_cast<const uint32_t*>(A.ws + A.L.codes)) + f0 + G.g0;
    G.vec_ok = (((f0 + G.g0) & 3u) == 0);                                // kEncBlock is a multiple of 4
    G.src16 = reinterpret_cast<const int16_t*>(A.ws + A.L.c16) + f0 + G.g0;
    G.wide16 = false;
    if (src_codes(SRC)) G.wide16 = (reinterpret_cast<const uint32_t*>(A.ws + A.L.cwide)[(size_t)frame * A.sbpf + G.g0 / A.stat_block] & 1u) != 0;
    const uint32_t K = A.K, kesc = K - 1u;

    FrameMeta M;
    if (src_rea(SRC)) M = rea_plan_frame<SRC>(A, frame, f0, G.nf, G.gb, S);
    else M = reinterpret_cast<const FrameMeta*>(A.ws + A.L.meta)[frame];
    if (!M.fits) return;
    uint8_t* fr = A.out + M.offset;
    uint32_t bad = 0;                             // SRC 2: a value that cannot be coded as planned fails the frame
    SrKeys keys;                                  // QM 1: draws of the group's elements, by position in the group
    if (QM == 1) keys.init(A.seed, f0 + G.g0); else { keys.base_lo = 0; keys.key0 = 0; keys.key1 = 0; }
    if (SRC == 3 && M.codec == CODEC_RAW && !M.pad_) {
        // (a frame of integer sums that goes RAW holds the sums of the dequantized operands: the finishing kernel's)
    } else if (SRC == 1 && M.codec == CODEC_RAW && !M.pad_) enc_raw_sums(A, G, f0, fr);
    else if (M.codec != CODEC_HUFF) enc_raw_fixed<SRC, QM, DELTA>(A, G, M, fr, S.stage[0], bad, keys);
    else {
        uint32_t raw[kEncIters][4];
        enc_load<SRC>(G, 0, raw);
        if (src_rea(SRC)) {
            // (the plan left the context's code in S.book)
        } else {
            for (uint32_t s = tid; s < K; s += kEncThreads) {
                const uint32_t sy = (s == kesc) ? 0u : s + 1u;
                const uint32_t c = reinterpret_cast<const uint32_t*>(A.ws + A.L.book_code)[(size_t)frame * kMaxK + sy];
                const uint32_t l = (A.ws + A.L.book_len)[(size_t)frame * kMaxK + sy];
                S.book[s] = (uint64_t)c | ((uint64_t)l << 32);
            }
        }
        for (uint32_t i = tid; i < 2 * (kStageWords + 4); i += kEncThreads) (&S.stage[0][0])[i] = 0;
        // Where the group's bits go.  Sources 0, 1: the exact position in the frame's bitstream, known from the block
        // histograms.  Source 2: sizes are only known once realized, so the frame's first group is materialised in
        // place (from bit 0) and every other group from bit 0 of a scratch region of its own; the finishing kernel
        // packs them behind each other.  In place nothing is written past the payload capacity (the RAW size of the
        // frame: Algorithm 1's EncodePlan works inside payloadCap); what is dropped belongs to a frame whose realized
        // payload exceeds that size and is rejected for it.
        const uint32_t start_bit = src_rea(SRC) ? 0u
            : reinterpret_cast<const uint32_t*>(A.ws + A.L.grp_start)[(size_t)frame * A.sbpf + G.g0 / A.stat_block];
        uint32_t* bits = reinterpret_cast<uint32_t*>(fr + M.bits_off) + (start_bit >> 5);   // first word this group touches
        if (src_rea(SRC) && G.gb > 0) bits = A.rea_tmp + ((size_t)frame * gpf + G.gb) * kReaTmpWords;
        const uint32_t cap_end = kHdrBytes + 4u * G.nf;                   // SRC 2: first byte of the frame that is off limits
        const uint32_t cap_segs = src_rea(SRC) ? (M.segt_off < cap_end ? (cap_end - M.segt_off) / 2u : 0u) : 0xFFFFFFFFu;
        const uint32_t cap_words = (src_rea(SRC) && G.gb == 0) ? (M.bits_off < cap_end ? (cap_end - M.bits_off) / 4u : 0u) : 0xFFFFFFFFu;
        uint16_t* segt = reinterpret_cast<uint16_t*>(fr + M.segt_off);
        const uint32_t nseg = (G.nf + kSeg - 1) / kSeg;
        uint32_t rel = start_bit & 31u;           // bits already in the current stage (carried over)
        uint32_t flushed = 0;                     // words of the group already written out
        uint32_t cur = 0;                         // stage in use
        uint32_t carry = 0;                       // thread 0: the partial word carried into the current stage
        __syncthreads();

        // Write the whole words of stage X to the bitstream, clear them, and move the partial word to Y[0].
        auto flush = [&](uint32_t* X, uint32_t* Y, uint32_t nbits) {
            const uint32_t nw = nbits >> 5;
            uint32_t* dst = bits + flushed;
            for (uint32_t k = tid; k < nw; k += kEncThreads) {
                const uint32_t wv = X[k];
                X[k] = 0;
                if (!src_rea(SRC) && G.gb > 0 && flushed == 0 && k == 0) atomicOr(dst, wv);   // word shared with the previous group
                else if (flushed + k < cap_words) dst[k] = wv;
            }
            if (tid == 0) { carry = X[nw]; X[nw] = 0; Y[0] = carry; }
            flushed += nw;
            rel = nbits & 31u;
        };
        // One symbol's code (and the raw bits of an escape) ORed into stage X at bit position pos.
        auto put_symbol = [&](uint32_t* X, uint32_t z, uint32_t& pos) {
            const uint64_t b = S.book[z < kesc ? z : kesc];
            const uint32_t val = (uint32_t)b, len = (uint32_t)(b >> 32);
            if (len) {
                const uint32_t sh = pos & 31u, wi = pos >> 5;
                atomicOr(&X[wi], val << sh);
                if (sh + len > 32u) atomicOr(&X[wi + 1], val >> (32u - sh));
                pos += len;
            }
            if (z >= kesc) {
                const uint32_t sh = pos & 31u, wi = pos >> 5;
                atomicOr(&X[wi], z << sh);
                if (sh) atomicOr(&X[wi + 1], z >> (32u - sh));
                pos += 32u;
            }
        };

        for (uint32_t sb = 0; sb < G.nsub; sb++) {
            // (a wavefront's issue priority falls as it gets through its group: instruction issue favours the wavefronts
            // started first, and the workgroups that share a compute unit would otherwise finish one after the other)
            // the levels get shorter towards the end (1/2, 1/4, 1/8, 1/8 of the group): workgroups draw level at every
            // boundary and can only drift apart again inside the last, short one
            {
                const uint32_t togo = G.nsub - sb;                // sub-blocks left, this one included
                if (8u * togo > 4u * G.nsub) __builtin_amdgcn_s_setprio(3);
                else if (8u * togo > 2u * G.nsub) __builtin_amdgcn_s_setprio(2);
                else if (8u * togo > G.nsub) __builtin_amdgcn_s_setprio(1);
                else __builtin_amdgcn_s_setprio(0);
            }
            const uint32_t cnt = (G.gcnt - sb * kEncBlock < kEncBlock) ? (G.gcnt - sb * kEncBlock) : kEncBlock;
            uint64_t pk[kEncIters];               // the thread's 4 symbols of a pass packed LSB-first
            uint32_t ln[kEncIters];               // exclusive bit offset of the thread inside its pass
            uint32_t wide = 0;                    // pass mask: the 4 symbols need more than 64 bits
            uint32_t zs[kEncIters][4];            // zigzag codes, kept for the passes that have to be redone
            // phase 1 (compiled twice: whole sub-blocks carry no bounds logic)
            auto phase1 = [&](auto whole_tag) {
                constexpr bool WHOLE = decltype(whole_tag)::value;
#pragma unroll
                for (uint32_t it = 0; it < kEncIters; it++) {
                    const uint32_t i = it * 1024 + tid * 4;
                    uint64_t acc = 0;
                    uint32_t tl = 0;
                    int32_t q4[4];
#pragma unroll
                    for (uint32_t j = 0; j < 4; j++) {
                        const bool valid = WHOLE || i + j < cnt;
                        bool ok = true;
                        q4[j] = enc_q<SRC, QM>(raw[it][j], A, &ok, QM ? keys.draw(sb * kEncBlock + i + j) : 0u);   // (words past the end are 0)
                        if (src_rea(SRC) && valid && !ok) bad = 1;
                    }
                    if (DELTA) delta4(q4);            // (a pass is four whole segments, one per wave)
#pragma unroll
                    for (uint32_t j = 0; j < 4; j++) {
                        const bool valid = WHOLE || i + j < cnt;
                        const uint32_t z = zigzag(q4[j]);
                        zs[it][j] = z;
                        const uint64_t b = S.book[z < kesc ? z : kesc];
                        const uint32_t len = valid ? (uint32_t)(b >> 32) : 0u, code = valid ? (uint32_t)b : 0u;
                        acc |= (uint64_t)code << (tl & 63u);              // garbage once tl > 64: the pass is then redone
                        tl += len;
                        if (z >= kesc && valid) { acc |= (uint64_t)z << (tl & 63u); tl += 32u; }
                    }
                    pk[it] = acc;
                    wide |= (tl > 64u ? 1u : 0u) << it;
                    const uint32_t incl = wave_incl_scan_dpp(tl);
                    ln[it] = incl - tl;                               // exclusive inside the wave's segment
                    if (lane == 63) S.wtot[it * 4 + wave] = incl;     // bits of segment it*4 + wave
                }
            };
            if (cnt == kEncBlock) phase1(std::true_type{}); else phase1(std::false_type{});
            enc_load<SRC>(G, sb + 1, raw);             // the next sub-block's words arrive during phase 2 and the flush
            __syncthreads();
            uint32_t pbase[kEncIters + 1];        // bit offset of every pass inside the sub-block
            pbase[0] = 0;
#pragma unroll
            for (uint32_t it = 0; it < kEncIters; it++) {
                const uint4 t = reinterpret_cast<const uint4*>(S.wtot)[it];
                ln[it] += (wave > 0 ? t.x : 0u) + (wave > 1 ? t.y : 0u) + (wave > 2 ? t.z : 0u);   // exclusive inside the pass
                pbase[it + 1] = pbase[it] + t.x + t.y + t.z + t.w;
            }
            if (tid < kEncSegs) {
                const uint32_t gseg = (G.g0 + sb * kEncBlock) / kSeg + tid;
                if (gseg < nseg && gseg < cap_segs) segt[gseg] = (uint16_t)S.wtot[tid];
                if (gseg == nseg - 1 && (nseg & 1u) && nseg < cap_segs) segt[nseg] = 0;      // pad4 of the table
            }
            uint32_t* X = S.stage[cur];
            if (__builtin_expect(rel + pbase[kEncIters] <= 32u * kStageWords, 1)) {
                // phase 2: the whole sub-block into the stage
#pragma unroll
                for (uint32_t it = 0; it < kEncIters; it++) {
                    uint32_t pos = rel + pbase[it] + ln[it];
                    if (__builtin_expect(!((wide >> it) & 1u), 1)) {
                        const uint64_t a = pk[it];
                        if (a) {
                            const uint32_t sh = pos & 31u, wi = pos >> 5;
                            const uint64_t t = a << sh;
                            atomicOr(&X[wi], (uint32_t)t);
                            if ((uint32_t)(t >> 32)) atomicOr(&X[wi + 1], (uint32_t)(t >> 32));
                            if (sh) { const uint32_t hi = (uint32_t)(a >> (64u - sh)); if (hi) atomicOr(&X[wi + 2], hi); }
                        }
                    } else {
                        // the thread's 4 symbols need more than 64 bits (rare): symbol by symbol
                        const uint32_t i = it * 1024 + tid * 4;
#pragma unroll
                        for (uint32_t j = 0; j < 4; j++)
                            if (i + j < cnt) put_symbol(X, zs[it][j], pos);
                    }
                }
                __syncthreads();
                flush(X, S.stage[cur ^ 1u], rel + pbase[kEncIters]);
                cur ^= 1u;
            } else {
                // more bits than the stage holds at once (rare): pass by pass, symbol by symbol from the source
#pragma unroll 1
                for (uint32_t it = 0; it < kEncIters; it++) {
                    const uint32_t i = it * 1024 + tid * 4;
                    uint32_t lnit = 0, pbits = 0;
#pragma unroll
                    for (uint32_t q = 0; q < kEncIters; q++) if (q == it) { lnit = ln[q]; pbits = pbase[q + 1] - pbase[q]; }
                    uint32_t pos = rel + lnit;
                    for (uint32_t j = 0; j < 4; j++)
                        if (i + j < cnt) put_symbol(X, enc_zz_at<SRC, QM, DELTA>(G, A, keys, sb * kEncBlock + i + j), pos);
                    __syncthreads();
                    flush(X, X, rel + pbits);
                    __syncthreads();
                }
            }
        }
        // the last, partial word: shared with the next group, or the frame's last bitstream word
        if (tid == 0 && rel) {
            uint32_t* dst = bits + flushed;
            if (src_rea(SRC)) { if (flushed < cap_words) *dst = carry; }
            else if (!G.last_grp || (G.gb > 0 && flushed == 0)) atomicOr(dst, carry);
            else *dst = carry;
        }
        if (src_rea(SRC) && tid == 0) A.rea_gbits[(size_t)frame * gpf + G.gb] = flushed * 32u + rel;     // realized bits of the group
    }
    if (src_rea(SRC)) {          // (header, padding and the packing of the groups are the finishing kernel's)
        if (bad) atomicOr(A.rea_fail + (size_t)frame * gpf + G.gb, 1u);
        return;
    }
    if (G.last_grp) {            // the frame's last group zero-fills the padding after the payload
        const uint32_t w0 = (kHdrBytes + M.payload) / 4, w1 = M.total / 4;
        if (tid < w1 - w0) reinterpret_cast<uint32_t*>(fr)[w0 + tid] = 0;
    }
}

// ------------------------------------------------------------------------------------------------
// Sampled runtime entropy arbitration (Sec. IV-C, Eq. 1-2, Algorithm 1): a cached Huffman context, a plan per
// frame from a bounded prefix sample, one pass of the selected codec over the frame, validation of the realized
// size and RAW as the fallback.  Frames sit in RAW-sized slots (the paper's frames are materialised in a staging
// bank and publish a byte-accurate length), so no frame has to wait for the size of another.
// ------------------------------------------------------------------------------------------------

// Context, step 1: symbol counts of the calibration message (values that cannot be quantized do not count).
__global__ __launch_bounds__(256) void k_ctx_hist(const float* x, uint64_t n, float eb, float step, float inv, uint32_t K,
                                                  uint32_t* ghist) {
    __shared__ uint32_t s_h[kMaxK];
    const uint32_t tid = threadIdx.x;
    for (uint32_t i = tid; i < K; i += 256) s_h[i] = 0;
    __syncthreads();
    const uint64_t i0 = (uint64_t)blockIdx.x * 4096u;
    for (uint32_t k = tid; k < 4096u && i0 + k < n; k += 256) {
        int32_t q;
        if (quantize1(x[i0 + k], eb, step, inv, q)) {
            const uint32_t z = zigzag(q);
            atomicAdd(&s_h[z <= K - 2u ? z + 1u : 0u], 1u);
        }
    }
    __syncthreads();
    for (uint32_t i = tid; i < K; i += 256) if (s_h[i]) atomicAdd(&ghist[i], s_h[i]);
}

// Context, step 2: one more than every count (each symbol, the escape included, gets a code), optimal lengths by the
// same two-queue rule as the per-frame codebooks, canonical codes, and the encoder's table.
__global__ __launch_bounds__(kBookThreads) void k_context(const uint32_t* ghist, uint32_t K, DevContext* ctx) {
    __shared__ BookShared s_b;
    const uint32_t tid = threadIdx.x;
    const uint32_t f = tid < K ? ghist[tid] + 1u : 0u;
    uint32_t L, code;
    book_build(s_b, f, K, L, code);
    if (tid < K) {
        ctx->len[tid] = (uint8_t)L;
        ctx->book[tid == 0 ? K - 1u : tid - 1u] = (uint64_t)(__brev(code) >> (32u - L)) | ((uint64_t)L << 32);
    } else if (tid < kMaxK) { ctx->len[tid] = 0; ctx->book[tid] = 0; }
    if (tid == 0) { ctx->valid = 1u; ctx->K = K; ctx->pad_[0] = 0; ctx->pad_[1] = 0; }
}

hipError_t launch_context(const float* sample, uint64_t n, float eb, float step, float inv_step, uint32_t K, uint32_t* ghist,
                          DevContext* ctx, hipStream_t st) {
    hipLaunchKernelGGL(k_init, dim3(kMaxK / 256), dim3(256), 0, st, ghist, (size_t)kMaxK, (ResultRec*)nullptr, 0u, 0u);
    hipLaunchKernelGGL(k_ctx_hist, dim3((uint32_t)((n + 4095u) / 4096u)), dim3(256), 0, st, sample, n, eb, step, inv_step, K, ghist);
    hipLaunchKernelGGL(k_context, dim3(1), dim3(kBookThreads), 0, st, ghist, K, ctx);
    return hipGetLastError();
}

// AcceptRealized + CommitRawOrFail, and everything that needs the realized size: the groups of a HUFFMAN frame are
// packed behind each other (every group but the first was materialised from bit 0 of a scratch region), then header,
// code-length table, padding, the result record.  A rejected frame is copied again as RAW by all of its workgroups.
//
// Bits of the stream `src` (len bits, starting at bit `start` of the frame's bitstream) that fall into word w of
// the frame's bitstream; words of src at or beyond nwords are not read.
__device__ inline uint32_t rea_contrib(const uint32_t* src, uint64_t start, uint64_t len, uint64_t w) {
    const int64_t r = (int64_t)(32ull * w) - (int64_t)start;            // first bit of word w, relative to the stream
    if (r <= -32 || r >= (int64_t)len) return 0;
    const uint64_t nwords = (len + 31u) >> 5;
    uint32_t v;
    uint64_t have;                                                       // valid bits from the low end of v (before masking)
    if (r >= 0) {
        const uint64_t a = (uint64_t)r >> 5;
        const uint32_t s = (uint32_t)r & 31u;
        const uint32_t lo = src[a], hi = (s && a + 1 < nwords) ? src[a + 1] : 0u;
        v = s ? ((lo >> s) | (hi << (32u - s))) : lo;
        have = len - (uint64_t)r;
        if (have < 32u) v &= (1u << have) - 1u;
    } else {
        const uint32_t sh = (uint32_t)(-r);
        uint32_t lo = src[0];
        if (len < 32u) lo &= (1u << len) - 1u;
        v = lo << sh;
    }
    return v;
}

__global__ __launch_bounds__(256) void k_rea_finish(ReaArgs A) {
    const uint32_t tid = threadIdx.x;
    const uint32_t frame = blockIdx.x / A.gpf, wg = blockIdx.x % A.gpf;
    const uint64_t f0 = (uint64_t)frame * A.chunk;
    const uint32_t nf = (uint32_t)((A.n - f0 < A.chunk) ? (A.n - f0) : A.chunk);
    const uint32_t g0 = wg * kEncGroup;
    if (g0 >= nf) return;
    const uint32_t ngrp = (nf + kEncGroup - 1) / kEncGroup;
    const FrameMeta M = A.in ? reinterpret_cast<const FrameMeta*>(A.ws + A.L.meta)[frame]
                             : reinterpret_cast<const FrameMeta*>(A.red_ws + A.RL.meta)[frame];
    uint8_t* fr = A.out + M.offset;
    const uint32_t K = A.K, plan = M.codec;
    const uint32_t nseg = (nf + kSeg - 1) / kSeg;
    const uint32_t* gbits = reinterpret_cast<const uint32_t*>(A.ws + A.L.gbits) + (size_t)frame * A.gpf;
    const uint64_t rawb = 4ull * nf;
    uint64_t payload = rawb, bits = 0, start = 0;                       // start: first bit of this workgroup's group
    if (plan == CODEC_FIXED) payload = 4ull * (((uint64_t)nf * M.w + 31u) / 32u);
    else if (plan == CODEC_HUFF) {
        for (uint32_t g = 0; g < ngrp; g++) { if (g == wg) start = bits; bits += gbits[g]; }
        payload = pad4u(K) + pad4u(2ull * nseg) + 4ull * ((bits + 31u) / 32u);
    }
    uint32_t codec = plan;
    if (plan != CODEC_RAW) {
        uint32_t failed = 0;
        for (uint32_t g = 0; g < ngrp; g++) failed |= reinterpret_cast<const uint32_t*>(A.ws + A.L.fail)[(size_t)frame * A.gpf + g];
        if (failed || payload > rawb || (rawb - payload) * 1000ull < (uint64_t)A.min_gain_permil * rawb) codec = CODEC_RAW;
    }
    const bool fell_back = (codec == CODEC_RAW && plan != CODEC_RAW);
    if (codec == CODEC_RAW) payload = rawb;
    const uint32_t total = (uint32_t)pad16u(kHdrBytes + payload);
    if (A.in) {
        if (fell_back) {
            const uint32_t gcnt = (nf - g0 < kEncGroup) ? (nf - g0) : kEncGroup;
            const uint32_t* src = reinterpret_cast<const uint32_t*>(A.in) + f0 + g0;
            uint32_t* dst = reinterpret_cast<uint32_t*>(fr + kHdrBytes) + g0;
            for (uint32_t i = tid; i < gcnt; i += 256) dst[i] = src[i];
        }
    } else if (codec == CODEC_RAW && !M.pad_) {
        // Ring step, a frame of integer sums that ends up RAW (planned so, or its realized output was rejected): it
        // holds fl(fl(qa*step) + fl(qb*step)), the sums of the dequantized operands.  qb is the rank's own value
        // quantized again (it was quantizable, or the frame would have no integer sums), qa = Q - qb.
#pragma clang fp contract(off)
        const uint32_t gcnt = (nf - g0 < kEncGroup) ? (nf - g0) : kEncGroup;
        const int16_t* c16 = reinterpret_cast<const int16_t*>(A.red_ws + A.RL.c16) + f0 + g0;
        const uint32_t* c32 = reinterpret_cast<const uint32_t*>(A.red_ws + A.RL.codes) + f0 + g0;
        const float* loc = A.local + f0 + g0;
        float* dst = reinterpret_cast<float*>(fr + kHdrBytes) + g0;
        for (uint32_t i = tid; i < gcnt; i += 256) {
            const int32_t h = c16[i];
            const int32_t Q = (h == -32768) ? (int32_t)c32[i] : h;
            int32_t qb;
            quantize1(loc[i], A.eb, A.step, A.inv_step, qb);
            const float va = (float)(Q - qb) * A.step, vb = (float)qb * A.step;
            const float sum = va + vb;
            reinterpret_cast<uint32_t*>(dst)[i] = (sum != sum) ? 0x7FC00000u : __float_as_uint(sum);   // (one canonical NaN)
        }
    }
    if (codec == CODEC_HUFF && wg > 0) {
        // Pack this group behind the one before it.  It writes every word its bits reach, the first one together
        // with the tail of the group before (which left that word alone unless it is the frame's first group, whose
        // tail is already in place), and leaves its own last word to the next group if it is partial.
        uint32_t* bits0 = reinterpret_cast<uint32_t*>(fr + M.bits_off);
        const uint32_t* tmp = A.tmp_base + ((size_t)frame * A.gpf + wg) * kReaTmpWords;
        const uint64_t len = gbits[wg], end = start + len;
        const uint64_t W0 = start >> 5;
        const uint64_t W1 = (wg == ngrp - 1 || (end & 31u) == 0) ? ((end + 31u) >> 5) : (end >> 5);   // one past the last word written
        const uint64_t plen = gbits[wg - 1], pstart = start - plen;
        const uint32_t* ptmp = A.tmp_base + ((size_t)frame * A.gpf + wg - 1) * kReaTmpWords;
        const uint32_t sh = (uint32_t)(start & 31u), back = sh ? 1u : 0u, s = (32u - sh) & 31u;
        const uint32_t nw = (uint32_t)(W1 - W0);
        const uint32_t interior = (uint32_t)(len >> 5);                   // words w of the frame with k - back + 1 < interior need no care
        uint32_t* dst = bits0 + W0;
        // interior words (k = back + a, a + 1 < interior) are a funnel shift of two words of the group: four per thread
        // and pass, several passes in flight (16-byte accesses that are only dword aligned)
        typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
        typedef u32x4 u32x4_a4 __attribute__((aligned(4)));
        const uint32_t fast = interior ? ((interior - 1u) & ~3u) : 0u;    // a in [0, fast) goes the fast way
        constexpr uint32_t kPasses = 4;
        for (uint32_t a0 = tid * 4; a0 < fast; a0 += 256 * 4 * kPasses) {
            u32x4 x[kPasses]; uint32_t y[kPasses];
#pragma unroll
            for (uint32_t u = 0; u < kPasses; u++) {
                const uint32_t a = a0 + u * 1024;
                if (a < fast) { x[u] = *reinterpret_cast<const u32x4_a4*>(tmp + a); y[u] = tmp[a + 4]; }
            }
#pragma unroll
            for (uint32_t u = 0; u < kPasses; u++) {
                const uint32_t a = a0 + u * 1024;
                if (a < fast) {
                    u32x4 v;
                    v.x = __builtin_amdgcn_alignbit(x[u].y, x[u].x, s); v.y = __builtin_amdgcn_alignbit(x[u].z, x[u].y, s);
                    v.z = __builtin_amdgcn_alignbit(x[u].w, x[u].z, s); v.w = __builtin_amdgcn_alignbit(y[u], x[u].w, s);
                    *reinterpret_cast<u32x4_a4*>(dst + back + a) = v;
                }
            }
        }
        for (uint32_t j = tid; j < nw - fast; j += 256) {                 // the words in front of and behind the fast part
            const uint32_t k = j < back ? j : j + fast;
            uint32_t v;
            if (k >= back && k - back + 1 < interior) {
                const uint32_t a = k - back;                              // group bits [32a + s', ...) with s' = s
                v = __builtin_amdgcn_alignbit(tmp[a + 1], tmp[a], s);
            } else {
                v = rea_contrib(tmp, start, len, W0 + k);
                if (k == 0 && sh) v |= (wg == 1) ? dst[0] : rea_contrib(ptmp, pstart, plen, W0);
            }
            dst[k] = v;
        }
    }
    if (wg != 0) return;
    if (codec == CODEC_HUFF) {
        const uint32_t words = (uint32_t)(pad4u(K) / 4);                 // code lengths, one byte per symbol, zero padded
        const uint32_t* lw = reinterpret_cast<const uint32_t*>(A.ctx->len);
        for (uint32_t i = tid; i < words; i += 256) {
            uint32_t v = lw[i];
            if (4 * i + 4 > K) v &= (1u << (8 * (K - 4 * i))) - 1u;      // K = 2: two lengths, two bytes of padding
            reinterpret_cast<uint32_t*>(fr + kHdrBytes)[i] = v;
        }
    }
    {
        const uint32_t w0 = (uint32_t)((kHdrBytes + payload) / 4), w1 = total / 4;
        if (tid < w1 - w0) reinterpret_cast<uint32_t*>(fr)[w0 + tid] = 0;
    }
    if (tid == 0) {
        uint32_t h[8];
        h[0] = kMagicFrame; h[1] = codec; h[2] = 4u * nf; h[3] = (uint32_t)payload;
        h[4] = (codec == CODEC_FIXED) ? M.w : (codec == CODEC_HUFF ? K : 0u);
        h[5] = (codec == CODEC_HUFF) ? (kSeg | (K << 16)) : 0u;
        h[6] = A.step_bits;
        uint32_t x = kCheckXor;
        for (int i = 0; i < 7; i++) x ^= h[i];
        h[7] = x;
        uint4* dst = reinterpret_cast<uint4*>(fr);
        dst[0] = make_uint4(h[0], h[1], h[2], h[3]);
        dst[1] = make_uint4(h[4], h[5], h[6], h[7]);
        ReaResultRec* res = reinterpret_cast<ReaResultRec*>(A.res);
        // ring step: a stream-level or frame-level error found by the adding pass voids the output (nothing published)
        const uint32_t add_status = A.in ? (uint32_t)ST_OK : reinterpret_cast<const ResultRec*>(A.add_res)->status;
        if (add_status != ST_OK) {
            if (frame == A.n_frames - 1) res->status = add_status;
            return;
        }
        atomicAdd(codec == CODEC_RAW ? &res->n_raw : (codec == CODEC_FIXED ? &res->n_fixed : &res->n_huff), 1u);
        if (fell_back) atomicAdd(&res->n_fallback, 1u);
        uint64_t wire = total;
        if (frame == A.n_frames - 1) {
            const uint64_t end = M.offset + total;
            wire += kStreamHdr + pad16u(8ull * A.n_frames);
            res->span_bytes = end;
            uint32_t* sh = reinterpret_cast<uint32_t*>(A.out);
            sh[10] = (uint32_t)end; sh[11] = (uint32_t)(end >> 32);
        }
        atomicAdd(reinterpret_cast<unsigned long long*>(&res->wire_bytes), (unsigned long long)wire);
    }
}

__global__ void k_rea_status(ReaResultRec* res, uint32_t n_frames, uint32_t status) {
    res->span_bytes = 0; res->wire_bytes = 0; res->status = status; res->n_frames = n_frames;
    res->n_raw = 0; res->n_fixed = 0; res->n_huff = 0; res->n_fallback = 0;
}

hipError_t launch_rea_status(void* res, uint32_t n_frames, uint32_t status, hipStream_t st) {
    hipLaunchKernelGGL(k_rea_status, dim3(1), dim3(1), 0, st, reinterpret_cast<ReaResultRec*>(res), n_frames, status);
    return hipGetLastError();
}

hipError_t launch_rea(const ReaArgs& A, hipStream_t st, void (*mark)(hipStream_t)) {
    // ProfileSample, ArbitratePlan, EncodePlan: the shared encoder with the sampled-arbitration source (quantizer tests on, the context's code,
    // group bitstreams from bit 0)
    CompressArgs C = {};
    C.in = A.in; C.n = A.n; C.chunk = A.chunk; C.n_frames = A.n_frames; C.K = A.K; C.sbpf = A.gpf; C.stat_block = kEncGroup;
    C.force_codec = A.force_codec; C.min_gain_permil = A.min_gain_permil; C.huff_min_bytes = A.huff_min_bytes;
    C.eb = A.eb; C.step = A.step; C.inv_step = A.inv_step; C.step_bits = A.step_bits;
    C.out = A.out; C.out_cap = 0; C.res = A.res;
    if (A.in) { C.ws = A.ws; C.L = WsLayout(); C.L.meta = A.L.meta; }
    else { C.ws = A.red_ws; C.L = A.RL; }        // ring step: the adding pass's workspace (staged sums, flags, frame plans)
    C.rea_ctx = A.ctx; C.rea_tmp = A.tmp_base; C.rea_gbits = reinterpret_cast<uint32_t*>(A.ws + A.L.gbits);
    C.rea_fail = reinterpret_cast<uint32_t*>(A.ws + A.L.fail);
    C.rea_sample_elems = A.sample_elems; C.rea_small_batch_bytes = A.small_batch_bytes; C.rea_slot = A.slot;
    C.rea_link_ps = A.link_ps; C.rea_fixed_alpha_ns = A.fixed_alpha_ns; C.rea_fixed_ps = A.fixed_ps;
    C.rea_huff_alpha_ns = A.huff_alpha_ns; C.rea_huff_ps = A.huff_ps;
    if (A.in) hipLaunchKernelGGL((k_encode<2, 0, 0>), dim3(A.n_frames * A.gpf), dim3(kEncThreads), 0, st, C);
    else hipLaunchKernelGGL((k_encode<3, 0, 0>), dim3(A.n_frames * A.gpf), dim3(kEncThreads), 0, st, C);
    mark(st);
    hipLaunchKernelGGL(k_rea_finish, dim3(A.n_frames * A.gpf), dim3(256), 0, st, A);
    mark(st);
    return hipGetLastError();
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

hipError_t launch_stats(const CompressArgs& A, bool stochastic, hipStream_t st) {
    const dim3 grid(A.n_frames * A.sbpf);
    if (stochastic) hipLaunchKernelGGL((k_stats<1, 0, 0>), grid, dim3(kStatThreads), 0, st, A);
    else if (A.pred) hipLaunchKernelGGL((k_stats<0, 1, 0>), grid, dim3(kStatThreads), 0, st, A);
    else hipLaunchKernelGGL((k_stats<0, 0, 0>), grid, dim3(kStatThreads), 0, st, A);
    return hipGetLastError();
}

hipError_t launch_stats_codes(const CompressArgs& A, hipStream_t st) {
    static_assert(kStatBlock == kEncGroup, "the reduce's statistics blocks are the encoder's groups");
    hipLaunchKernelGGL((k_stats<0, 1, 1>), dim3(A.n_frames * A.sbpf), dim3(kStatThreads), 0, st, A);
    return hipGetLastError();
}

// Bin width of QSGD with `levels` levels per sign: ||x||_2 / levels.  Squares are summed in float64 by a fixed grid in
// a fixed order (per-thread strided partial sums, wave and workgroup trees, then the workgroups' partials in index
// order), so the result does not depend on scheduling.
constexpr uint32_t kSsqBlocks = 1024;
__global__ __launch_bounds__(256) void k_ssq(const float* x, uint64_t n, double* partials) {
    __shared__ double s_w[4];
    double acc = 0.0;
    for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (uint64_t)kSsqBlocks * 256) {
        const double v = (double)x[i];
        acc += v * v;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
    if (lane_id() == 0) s_w[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) partials[blockIdx.x] = (s_w[0] + s_w[1]) + (s_w[2] + s_w[3]);
}
__global__ void k_qsgd_step(const double* partials, uint32_t levels, float* step_out) {
    double ssq = 0.0;
    for (uint32_t b = 0; b < kSsqBlocks; b++) ssq += partials[b];
    double st = sqrt(ssq) / (double)levels;
    if (!(st <= 0x1p100)) st = __longlong_as_double(0x7FF8000000000000ll);     // non-finite input: the caller sees NaN
    else if (st < 0x1p-100) st = 0x1p-100;
    *step_out = (float)st;
}
hipError_t launch_qsgd_step(const float* in, uint64_t n, uint32_t levels, float* step_out, double* partials, hipStream_t st) {
    hipLaunchKernelGGL(k_ssq, dim3(kSsqBlocks), dim3(256), 0, st, in, n, partials);
    hipLaunchKernelGGL(k_qsgd_step, dim3(1), dim3(1), 0, st, partials, levels, step_out);
    return hipGetLastError();
}

hipError_t launch_codebook(const CompressArgs& A, hipStream_t st) {
    hipLaunchKernelGGL(k_codebook, dim3(A.n_frames), dim3(kBookThreads), 0, st, A);
    return hipGetLastError();
}

hipError_t launch_encode(const CompressArgs& A, bool from_codes, bool stochastic, hipStream_t st) {
    const dim3 grid(A.n_frames * ((A.chunk + kEncGroup - 1) / kEncGroup));
    if (from_codes && A.pred) hipLaunchKernelGGL((k_encode<1, 0, 1>), grid, dim3(kEncThreads), 0, st, A);
    else if (from_codes) hipLaunchKernelGGL((k_encode<1, 0, 0>), grid, dim3(kEncThreads), 0, st, A);
    else if (stochastic) hipLaunchKernelGGL((k_encode<0, 1, 0>), grid, dim3(kEncThreads), 0, st, A);
    else if (A.pred) hipLaunchKernelGGL((k_encode<0, 0, 1>), grid, dim3(kEncThreads), 0, st, A);
    else hipLaunchKernelGGL((k_encode<0, 0, 0>), grid, dim3(kEncThreads), 0, st, A);
    return hipGetLastError();
}

}  // namespace nz
