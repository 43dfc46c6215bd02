// nz_scan.hpp -- wave-wide decoupled look-back and canonical-code ranking, shared by the gfx950 kernels.
#pragma once
#include "nz_common.hpp"

namespace nz {

constexpr uint64_t kDescA    = 1ull << 62;          // descriptor holds this item's own amount
constexpr uint64_t kDescP    = 2ull << 62;          // descriptor holds the inclusive prefix up to this item
constexpr uint64_t kDescMask = (1ull << 62) - 1;

// Decoupled look-back, executed by one full wave.  Items lo..idx-1 precede item idx; a virtual item lo-1
// carries the inclusive prefix base0.  Every item publishes kDescA|own as soon as it knows its amount and
// kDescP|inclusive once it knows its prefix; a waiter only ever waits on items that were started before
// it (dynamic tickets), so every wait ends.  Returns the exclusive prefix of item idx.
__device__ inline uint64_t lookback_exclusive(const uint64_t* desc, int64_t lo, int64_t idx, uint64_t base0) {
    const int lane = (int)lane_id();
    uint64_t acc = 0;
    int64_t pos = idx - 1;
    for (;;) {
        const int64_t j = pos - lane;
        uint64_t v;
        int pl;
        for (;;) {
            v = (j >= lo) ? ld_agent(desc + j) : (kDescP | base0);
            const uint64_t pm = __ballot((v >> 62) == 2);
            const uint64_t zm = __ballot((v >> 62) == 0);
            pl = pm ? (__ffsll((unsigned long long)pm) - 1) : 64;
            const uint64_t need = (pl >= 64) ? ~0ull : ((2ull << pl) - 1ull);
            if ((zm & need) == 0) break;
            __builtin_amdgcn_s_sleep(2);
        }
        acc += wave_sum64(lane <= pl ? (v & kDescMask) : 0ull);
        if (pl < 64) break;
        pos -= 64;
    }
    return acc;
}

// Canonical-code bookkeeping for an alphabet of K <= 1024 symbols whose code lengths sit in s_len[0..K)
// (0 = unused).  NT threads (multiple of 64) cooperate.  On return (after the trailing barrier):
//   s_cnt[L]   number of symbols with length L (s_cnt[0] = 0), L = 0..31
//   s_first[L] first canonical code of length L:  first[L] = (first[L-1] + cnt[L-1]) << 1
//   s_idx0[L]  number of symbols with a shorter length (index of the first length-L symbol in (len,sym) order)
//   s_rank[s]  position of symbol s among the symbols of its own length, in increasing symbol order
// so code(s) = s_first[len] + s_rank[s] and sorted position = s_idx0[len] + s_rank[s].
// Scratch: s_wcnt[16*32].
template <int NT>
__device__ inline void canonical_tables(const uint8_t* s_len, uint32_t K, uint32_t* s_wcnt, uint32_t* s_cnt,
                                        uint32_t* s_first, uint32_t* s_idx0, uint16_t* s_rank) {
    const uint32_t tid = threadIdx.x, lane = lane_id();
    // rank inside each group of 64 consecutive symbols (one wavefront), and the group's count per length: one ballot per
    // possible length, no shared memory inside the loop.  Lane l of the wavefront keeps the count of length l and writes
    // it (every entry of a group that some wavefront covers has exactly one writer; the other groups are cleared here).
    const uint32_t covered = ((K + NT - 1) / NT) * (NT / 64);         // groups the loop below writes
    for (uint32_t i = covered * 32 + tid; i < 16 * 32; i += NT) s_wcnt[i] = 0;
    for (uint32_t base = 0; base < K; base += NT) {
        const uint32_t s = base + tid;
        const uint32_t L = (s < K) ? s_len[s] : 0u;
        const uint32_t grp = s >> 6;
        uint32_t rank = 0, mine = 0;
#pragma unroll
        for (uint32_t l = 1; l <= kMaxLen; l++) {
            const uint64_t mask = __ballot(L == l);
            if (L == l) rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
            if (lane == l) mine = (uint32_t)__popcll(mask);
        }
        if (lane < 32 && grp < 16) s_wcnt[grp * 32 + lane] = mine;
        if (s < K) s_rank[s] = (uint16_t)rank;
    }
    __syncthreads();
    // per length (lane = length, wave 0): exclusive prefix over the 16 groups and the total count, then
    // idx0 = exclusive scan of the counts and first[L] = sum over l < L of cnt[l] << (L - l), taken as an
    // exclusive scan of the counts left-justified to 28 bits (the Kraft sum is at most 1, so it fits).
    if (tid < 64) {
        uint32_t run = 0;
        if (tid >= 1 && tid <= kMaxLen) {
            uint32_t c[16];
#pragma unroll
            for (uint32_t g = 0; g < 16; g++) c[g] = s_wcnt[g * 32 + tid];
#pragma unroll
            for (uint32_t g = 0; g < 16; g++) { s_wcnt[g * 32 + tid] = run; run += c[g]; }
        }
        const uint32_t lj = (tid >= 1 && tid <= kMaxLen) ? (run << (kMaxLen - tid)) : 0u;
        const uint32_t incl_i = wave_incl_scan_dpp(run);
        const uint32_t incl_f = wave_incl_scan_dpp(lj);
        if (tid < 32) {
            s_cnt[tid] = run;
            s_idx0[tid] = incl_i - run;
            s_first[tid] = (tid <= kMaxLen) ? ((incl_f - lj) >> (kMaxLen - tid)) : (incl_f << (tid - kMaxLen));
        }
    }
    __syncthreads();
    for (uint32_t base = 0; base < K; base += NT) {
        const uint32_t s = base + tid;
        if (s < K) { const uint32_t L = s_len[s]; if (L) s_rank[s] = (uint16_t)(s_rank[s] + s_wcnt[(s >> 6) * 32 + L]); }
    }
    __syncthreads();
}

}  // namespace nz
