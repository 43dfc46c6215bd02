/*
 * nz_oracle.c -- plain, slow, single-threaded CPU oracle of the NZ per-rank
 * compression path (error-bounded quantizer -> per-frame selector among
 * RAW / FIXEDLEN / HUFFMAN -> self-describing frames -> decode/dequantize ->
 * frame-wise integer reduce).
 *
 * THIS IS TEST INFRASTRUCTURE.  Only the test-suite, the smoke check and the
 * benchmark's cpu_baseline leg may call it.  It shares no code, header, table
 * or helper with the HIP library; the product path never routes through it.
 *
 * What the paper fixes and where this file follows it:
 *   - one-time deterministic error-bounded quantization at the interface, the
 *     only lossy step (Sec. II-B "Quantization", Sec. IV-A, IV-B);
 *   - three lossless paths RAW / FIXEDLEN / HUFFMAN and the rule "choose the
 *     argmin over {RAW} + admissible entropy codecs, RAW when nothing is
 *     admissible" (Sec. IV-C, Eq. 1 and Eq. 2, Algorithm 1);
 *   - admissibility = fits capacity, beats the minimum-gain threshold, codec
 *     enable conditions such as the Huffman size threshold (Sec. IV-C);
 *   - self-describing frame = header {codecId, rawBytes, payloadBytes, codec
 *     parameters} + payload, validated and decoded independently by the
 *     receiver (Sec. IV-D "Batch Framing", Algorithm 2 receiver side);
 *   - reduction works on the lossless (integer) representation so that no
 *     lossy step is repeated (Sec. III "Error propagation", Sec. IV-A).
 * What the paper leaves open (quantizer formula, symbol width, header layout,
 * bit order, tie-breaks, codebook origin) is fixed by the NZ stream format v1,
 * written out next to each function below.
 *
 * Pins (tests/test_oracle_pins.py and friends): error bound in float64, worked
 * quantizer values, brute-force optimal prefix-code cost, Kraft equality,
 * closed-form code lengths, independent numpy bit-unpack, exhaustive selector,
 * header-mutation rejection, reduce == encode(qa+qb), ring-step reduce ==
 * encode(q_incoming + quantize(local)) and == reduce with the coded local message.
 * Parity unpinned: the paper prints no bitstream, no worked example and no
 * compression ratio reachable without its datasets, so nothing here is pinned
 * against a number printed in the paper.
 */
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>

#ifdef __FAST_MATH__
#error "the oracle must be compiled without -ffast-math"
#endif

/* ------------------------------------------------------------------ */
/* public types                                                         */
/* ------------------------------------------------------------------ */

/* Status codes are ordered by precedence: when several conditions hold the largest code is reported. */
enum { NZO_OK = 0, NZO_ERR_INVALID = 1, NZO_ERR_CAPACITY = 2, NZO_ERR_CORRUPT = 3, NZO_ERR_MISMATCH = 4 };

enum { NZO_RAW = 0, NZO_FIXEDLEN = 1, NZO_HUFFMAN = 2 };

typedef struct {
    uint32_t chunk_elems;     /* fp32 elements per frame, 1..2^20; 0 -> 262144        */
    uint32_t seg_syms;        /* symbols per Huffman segment, 32..1024; 0 -> 256      */
    uint32_t alphabet;        /* K, power of two in 2..1024; 0 -> 256                 */
    int32_t  force_codec;     /* -1 auto, 0/1/2 pin a codec (Sec. V-B pins codecs)    */
    uint32_t min_gain_permil; /* minimum-gain threshold of Algorithm 1, default 0     */
    uint32_t huff_min_bytes;  /* Huffman size threshold T_huff of Algorithm 1         */
    uint32_t predictor;       /* 0 none; 1 delta on the codes (section 12, an extension) */
    uint32_t reserved;        /* 0                                                    */
} nzo_opts;

typedef struct {
    uint64_t bytes;
    uint32_t status;
    uint32_t n_frames;
    uint32_t n_raw, n_fixed, n_huff;
    uint32_t reserved;
} nzo_result;

#define NZO_HDR_BYTES      32u
#define NZO_STREAM_HDR     64u
#define NZO_QMAX           32767
#define NZO_QSUM_MAX       (1 << 30)
#define NZO_MAX_CHUNK      (1u << 20)
#define NZO_MAX_K          1024u
#define NZO_MAX_OPERANDS   64u          /* operands of one k-ary reduce */
#define NZO_MAGIC_FRAME    0x31465A4Eu   /* bytes 'N','Z','F','1' */
#define NZO_MAGIC_STREAM   0x31535A4Eu   /* bytes 'N','Z','S','1' */
#define NZO_CHECK_XOR      0x5A5A5A5Au
#define NZO_CANON_NAN      0x7FC00000u

/* ------------------------------------------------------------------ */
/* little helpers                                                       */
/* ------------------------------------------------------------------ */

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

static void put_u32(uint8_t* p, uint32_t v) {
    p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); p[2] = (uint8_t)(v >> 16); p[3] = (uint8_t)(v >> 24);
}
static void put_u64(uint8_t* p, uint64_t v) { put_u32(p, (uint32_t)v); put_u32(p + 4, (uint32_t)(v >> 32)); }
static uint32_t get_u32(const uint8_t* p) {
    return (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16) | ((uint32_t)p[3] << 24);
}
static uint64_t get_u64(const uint8_t* p) { return (uint64_t)get_u32(p) | ((uint64_t)get_u32(p + 4) << 32); }

static uint64_t pad4(uint64_t v) { return (v + 3u) & ~(uint64_t)3u; }
static uint64_t pad16(uint64_t v) { return (v + 15u) & ~(uint64_t)15u; }

static int bit_length32(uint32_t v) { int n = 0; while (v) { n++; v >>= 1; } return n; }

static int is_pow2(uint32_t v) { return v && !(v & (v - 1)); }

/* Fill in defaults and check ranges.  Returns NZO_OK or NZO_ERR_INVALID. */
static int resolve_opts(const nzo_opts* in, nzo_opts* o) {
    nzo_opts d = { 0, 0, 0, -1, 0, 0, 0, 0 };
    if (in) d = *in;
    if (d.chunk_elems == 0) d.chunk_elems = 262144u;
    if (d.seg_syms == 0) d.seg_syms = 256u;
    if (d.alphabet == 0) d.alphabet = 256u;    /* the paper profiles a 256-bin histogram (Sec. IV-C) */
    if (d.chunk_elems > NZO_MAX_CHUNK) return NZO_ERR_INVALID;
    if (d.seg_syms < 32u || d.seg_syms > 1024u) return NZO_ERR_INVALID;
    if (d.alphabet < 2u || d.alphabet > NZO_MAX_K || !is_pow2(d.alphabet)) return NZO_ERR_INVALID;
    if (d.force_codec < -1 || d.force_codec > 2) return NZO_ERR_INVALID;
    if (d.min_gain_permil > 1000u) return NZO_ERR_INVALID;
    if (d.predictor > 1u || d.reserved) return NZO_ERR_INVALID;
    *o = d;
    return NZO_OK;
}

/* ------------------------------------------------------------------ */
/* 1. quantizer (the interface quantizer of Sec. IV-A / IV-B)           */
/* ------------------------------------------------------------------ */

/*
 * Step constants.  The paper asks for uniformly spaced bins set by the user's
 * error bound with strict pointwise control (Sec. II-B) and gives no formula.
 * Format v1: bin width step = fl32(eb * 63/32) (= 2*eb*63/64), reciprocal
 * inv_step = fl32(1/step).  The 63/64 leaves room for the fp32 roundings of
 * x*inv_step and q*step so that |x - xhat| <= eb is a theorem for |q| <= 32767.
 */
int nzo_step_constants(float eb, float* step, float* inv_step) {
    if (!(eb >= 0x1p-100f && eb <= 0x1p100f)) return NZO_ERR_INVALID;   /* also rejects NaN */
    volatile float s = eb * 1.96875f;
    volatile float r = 1.0f / s;
    *step = s; *inv_step = r;
    return NZO_OK;
}

/*
 * Quantize one value: u = fl32(x*inv_step); unquantizable unless |u| <= 32767;
 * q = round-half-even(u); xhat = fl32(float(q)*step); unquantizable unless
 * fl32(|x - xhat|) <= eb.  Returns 1 and stores q when quantizable, else 0.
 * volatile keeps every product and difference a separately rounded fp32
 * operation (no fused multiply-add, no excess precision).
 */
int nzo_quantize_one(float x, float eb, float step, float inv_step, int32_t* q) {
    volatile float u = x * inv_step;
    if (!(fabsf(u) <= 32767.0f)) return 0;
    volatile float r = nearbyintf(u);            /* default rounding mode: ties to even */
    int32_t qi = (int32_t)r;
    volatile float xh = (float)qi * step;
    volatile float d = x - xh;
    if (!(fabsf(d) <= eb)) return 0;
    *q = qi;
    return 1;
}

/* Dequantize: xhat = fl32(float(q) * step), float(q) rounding to nearest even. */
float nzo_dequantize_one(int32_t q, float step) {
    volatile float xh = (float)q * step;
    return xh;
}

/* Array form used by the pins: q[i] and ok[i] per element. */
int nzo_quantize(const float* x, size_t n, float eb, int32_t* q, uint8_t* ok) {
    float step, inv;
    int rc = nzo_step_constants(eb, &step, &inv);
    if (rc) return rc;
    for (size_t i = 0; i < n; i++) {
        int32_t v = 0;
        ok[i] = (uint8_t)nzo_quantize_one(x[i], eb, step, inv, &v);
        q[i] = ok[i] ? v : 0;
    }
    return NZO_OK;
}

/* Zigzag map 0,-1,1,-2,2,... -> 0,1,2,3,4,... and its inverse. */
uint32_t nzo_zigzag(int32_t q) { return ((uint32_t)q << 1) ^ (uint32_t)(q >> 31); }
int32_t nzo_unzigzag(uint32_t z) { return (int32_t)(z >> 1) ^ -(int32_t)(z & 1u); }

/* ------------------------------------------------------------------ */
/* 2. Huffman code lengths and canonical codes (Sec. II-B "Entropy      */
/*    coding": shorter codes for more frequent symbols)                 */
/* ------------------------------------------------------------------ */

typedef struct { uint32_t f; uint32_t s; } leaf_t;

static int leaf_cmp(const void* a, const void* b) {
    const leaf_t* x = (const leaf_t*)a; const leaf_t* y = (const leaf_t*)b;
    if (x->f != y->f) return x->f < y->f ? -1 : 1;
    if (x->s != y->s) return x->s < y->s ? -1 : 1;
    return 0;
}

/*
 * Optimal prefix-code lengths by the two-queue construction.  Leaves are the
 * symbols with f>0 sorted ascending by (f, symbol); internal nodes enter a
 * FIFO in creation order.  pick() takes the leaf head when the leaf queue is
 * non-empty and (the FIFO is empty or leaf weight <= node weight): a leaf wins
 * a tie.  m-1 merges; len[s] = depth of leaf s; a single used symbol gets
 * length 1; unused symbols get 0.  K <= 1024.  Returns the number of used
 * symbols.
 */
int nzo_huffman_lengths(const uint32_t* f, uint32_t K, uint8_t* len) {
    leaf_t leaves[NZO_MAX_K];
    uint64_t w[2 * NZO_MAX_K];      /* node weights: 0..m-1 leaves (sorted), m.. internal */
    int32_t parent[2 * NZO_MAX_K];
    uint32_t m = 0;
    if (K > NZO_MAX_K) return -1;
    for (uint32_t s = 0; s < K; s++) { len[s] = 0; if (f[s]) { leaves[m].f = f[s]; leaves[m].s = s; m++; } }
    if (m == 0) return 0;
    if (m == 1) { len[leaves[0].s] = 1; return 1; }
    qsort(leaves, m, sizeof(leaf_t), leaf_cmp);
    for (uint32_t i = 0; i < m; i++) { w[i] = leaves[i].f; parent[i] = -1; }
    uint32_t ia = 0;          /* head of leaf queue   */
    uint32_t ib = m;          /* head of node FIFO    */
    uint32_t nb = m;          /* tail of node FIFO    */
    for (uint32_t step = 0; step + 1 < m; step++) {
        uint32_t pick[2];
        for (int k = 0; k < 2; k++) {
            int take_leaf;
            if (ia < m && ib < nb) take_leaf = (w[ia] <= w[ib]);
            else take_leaf = (ia < m);
            pick[k] = take_leaf ? ia++ : ib++;
        }
        w[nb] = w[pick[0]] + w[pick[1]];
        parent[nb] = -1;
        parent[pick[0]] = (int32_t)nb;
        parent[pick[1]] = (int32_t)nb;
        nb++;
    }
    for (uint32_t i = 0; i < m; i++) {
        uint32_t d = 0;
        for (int32_t p = parent[i]; p >= 0; p = parent[p]) d++;
        len[leaves[i].s] = (uint8_t)d;
    }
    return (int)m;
}

/*
 * Canonical code assignment (the textbook rule, as stated publicly in
 * RFC 1951 sec. 3.2.2): count codes per length, first code of length L is
 * (first[L-1] + count[L-1]) << 1, symbols of equal length get consecutive
 * codes in increasing symbol order.
 */
void nzo_canonical_codes(const uint8_t* len, uint32_t nsym, uint32_t* code) {
    uint32_t count[33], next[33];
    memset(count, 0, sizeof count);
    for (uint32_t s = 0; s < nsym; s++) count[len[s]]++;
    count[0] = 0;
    next[0] = 0;
    uint32_t c = 0;
    for (int L = 1; L <= 32; L++) { c = (c + count[L - 1]) << 1; next[L] = c; }
    for (uint32_t s = 0; s < nsym; s++) code[s] = len[s] ? next[len[s]]++ : 0;
}

/* ------------------------------------------------------------------ */
/* 3. bit writer / reader: LSB-first into little-endian 32-bit words   */
/* ------------------------------------------------------------------ */

typedef struct { uint8_t* p; uint64_t nbits; } bitw_t;   /* p must be zero-filled */

static void bw_put1(bitw_t* b, uint32_t bit) {
    if (bit & 1u) b->p[b->nbits >> 3] |= (uint8_t)(1u << (b->nbits & 7u));
    b->nbits++;
}
/* value's bit 0 first */
static void bw_put_lsb(bitw_t* b, uint32_t v, int n) { for (int i = 0; i < n; i++) bw_put1(b, v >> i); }
/* value's bit n-1 first (prefix-code orientation) */
static void bw_put_msb(bitw_t* b, uint32_t v, int n) { for (int i = n - 1; i >= 0; i--) bw_put1(b, v >> i); }

typedef struct { const uint8_t* p; uint64_t pos, end; int overrun; } bitr_t;

static uint32_t br_get1(bitr_t* b) {
    if (b->pos >= b->end) { b->overrun = 1; return 0; }
    uint32_t bit = (b->p[b->pos >> 3] >> (b->pos & 7u)) & 1u;
    b->pos++;
    return bit;
}
static uint32_t br_get_lsb(bitr_t* b, int n) {
    uint32_t v = 0;
    for (int i = 0; i < n; i++) v |= br_get1(b) << i;
    return v;
}

/* ------------------------------------------------------------------ */
/* 4. frame statistics, exact sizes, selector (Sec. IV-C, Eq. 2, Alg. 1)*/
/* ------------------------------------------------------------------ */

typedef struct {
    uint32_t zmax;                 /* max zigzag code                         */
    uint32_t w;                    /* FIXEDLEN width = bit_length(zmax)        */
    uint32_t f[NZO_MAX_K];         /* histogram over symbols, 0 = ESC          */
    uint32_t nsym;                 /* 1 + largest used symbol                  */
    uint8_t  len[NZO_MAX_K];
    uint32_t code[NZO_MAX_K];
    uint64_t huff_bits;            /* exact bitstream length                   */
    uint32_t nseg;
    uint64_t payload[3];           /* exact payload bytes per codec            */
    uint64_t total[3];             /* pad16(header + payload)                  */
} frame_plan;

/* symbol of a zigzag code under alphabet K: z+1 when z <= K-2, else ESC = 0 */
static uint32_t sym_of(uint32_t z, uint32_t K) { return z <= K - 2u ? z + 1u : 0u; }

/*
 * 12. Prediction before the entropy stage (the first stage of the SZ-style pipeline that Sec. II-B lists:
 * prediction, quantization, entropy coding).  The paper's own path has no predictor; this is an extension,
 * lossless and linear, so the integer reduce still holds.  predictor = 1 (delta): what the entropy stage codes
 * for element i of a frame is v_i = q_i - q_{i-1}, taken modulo 2^32, except at the start of every segment of
 * seg_syms elements, where v_i = q_i (segments stay independently decodable).  The receiver adds up again:
 * q_i = q_{i-1} + v_i modulo 2^32.  FIXEDLEN and HUFFMAN work on zigzag(v); the selector sizes them on v.
 */
static int32_t coded_value(const int32_t* q, uint32_t i, const nzo_opts* o) {
    if (o->predictor == 1u && (i % o->seg_syms) != 0u) return (int32_t)((uint32_t)q[i] - (uint32_t)q[i - 1]);
    return q[i];
}

static void plan_frame(const int32_t* q, uint32_t nf, const nzo_opts* o, frame_plan* P) {
    memset(P, 0, sizeof *P);
    const uint32_t K = o->alphabet;
    for (uint32_t i = 0; i < nf; i++) {
        uint32_t z = nzo_zigzag(coded_value(q, i, o));
        if (z > P->zmax) P->zmax = z;
        P->f[sym_of(z, K)]++;
    }
    P->w = (uint32_t)bit_length32(P->zmax);
    for (uint32_t s = 0; s < K; s++) if (P->f[s]) P->nsym = s + 1;
    nzo_huffman_lengths(P->f, K, P->len);
    nzo_canonical_codes(P->len, P->nsym, P->code);
    P->huff_bits = (uint64_t)P->f[0] * (P->len[0] + 32u);
    for (uint32_t s = 1; s < K; s++) P->huff_bits += (uint64_t)P->f[s] * P->len[s];
    P->nseg = (nf + o->seg_syms - 1) / o->seg_syms;
    P->payload[NZO_RAW] = 4ull * nf;
    P->payload[NZO_FIXEDLEN] = 4ull * (((uint64_t)nf * P->w + 31u) / 32u);
    P->payload[NZO_HUFFMAN] = pad4(P->nsym) + pad4(2ull * P->nseg) + 4ull * ((P->huff_bits + 31u) / 32u);
    for (int c = 0; c < 3; c++) P->total[c] = pad16(NZO_HDR_BYTES + P->payload[c]);
}

/*
 * Selector.  With encode/decode fully overlapped and no fixed cost, Eq. 1
 * reduces to transmitted size, so Eq. 2 is argmin of total frame bytes over
 * {RAW} + admissible codecs.  Admissible: frame quantizable; Huffman needs
 * rawBytes >= huff_min_bytes; gain (RAW - payload)*1000 >= min_gain_permil*RAW.
 * Ties go to the lower codec id (the cheaper codec).  A pinned codec overrides
 * the choice but an unquantizable frame is always RAW.  Sizes are exact, so
 * Algorithm 1's post-validation of the realized size cannot fail.
 */
static int select_codec(const frame_plan* P, int quantizable, const nzo_opts* o) {
    if (!quantizable) return NZO_RAW;
    if (o->force_codec >= 0) return o->force_codec;
    int best = NZO_RAW;
    const uint64_t rawb = P->payload[NZO_RAW];
    for (int c = NZO_FIXEDLEN; c <= NZO_HUFFMAN; c++) {
        if (c == NZO_HUFFMAN && rawb < o->huff_min_bytes) continue;
        if (P->payload[c] > rawb) continue;
        if ((rawb - P->payload[c]) * 1000ull < (uint64_t)o->min_gain_permil * rawb) continue;
        if (P->total[c] < P->total[best]) best = c;
    }
    return best;
}

/* ------------------------------------------------------------------ */
/* 5. frame writer                                                      */
/* ------------------------------------------------------------------ */

static void write_header(uint8_t* dst, uint32_t codec, uint32_t raw_bytes, uint32_t payload_bytes,
                         uint32_t p0, uint32_t p1, uint32_t step_bits) {
    uint32_t h[8] = { NZO_MAGIC_FRAME, codec, raw_bytes, payload_bytes, p0, p1, step_bits, 0 };
    uint32_t x = NZO_CHECK_XOR;
    for (int i = 0; i < 7; i++) x ^= h[i];
    h[7] = x;
    for (int i = 0; i < 8; i++) put_u32(dst + 4 * i, h[i]);
}

/*
 * Write one frame (header + payload, zero padded to 16 bytes) with the given
 * codec.  q = integer codes (coded frames); rawbits = the fp32 bit patterns a
 * RAW frame carries.  dst has room for P->total[codec] bytes.
 *   RAW:      payload = the nf fp32 words.
 *   FIXEDLEN: each zigzag code in w bits, bit 0 first; p0 = w.
 *   HUFFMAN:  len[0..nsym) as bytes (pad4) | u16 bit length of every segment
 *             of seg_syms symbols (pad4) | bitstream: per symbol its canonical
 *             code most-significant bit first, an ESC code followed by the 32
 *             bits of z bit 0 first; segments back to back, no padding between
 *             them.  p0 = nsym, p1 = seg_syms | K<<16 (both are <= 1024, so each
 *             fits its 16-bit half) | predictor<<31; FIXEDLEN: p1 = predictor<<31.
 */
static void write_frame(uint8_t* dst, int codec, const int32_t* q, const uint32_t* rawbits, uint32_t nf,
                        const frame_plan* P, const nzo_opts* o, uint32_t step_bits) {
    memset(dst, 0, (size_t)P->total[codec]);
    uint8_t* pay = dst + NZO_HDR_BYTES;
    if (codec == NZO_RAW) {
        write_header(dst, NZO_RAW, 4u * nf, (uint32_t)P->payload[NZO_RAW], 0, 0, step_bits);
        for (uint32_t i = 0; i < nf; i++) put_u32(pay + 4ull * i, rawbits[i]);
    } else if (codec == NZO_FIXEDLEN) {
        write_header(dst, NZO_FIXEDLEN, 4u * nf, (uint32_t)P->payload[NZO_FIXEDLEN], P->w, o->predictor << 31, step_bits);
        bitw_t b = { pay, 0 };
        for (uint32_t i = 0; i < nf; i++) bw_put_lsb(&b, nzo_zigzag(coded_value(q, i, o)), (int)P->w);
    } else {
        write_header(dst, NZO_HUFFMAN, 4u * nf, (uint32_t)P->payload[NZO_HUFFMAN], P->nsym,
                     o->seg_syms | (o->alphabet << 16) | (o->predictor << 31), step_bits);
        uint8_t* lens = pay;
        uint8_t* segt = pay + pad4(P->nsym);
        uint8_t* bits = segt + pad4(2ull * P->nseg);
        for (uint32_t s = 0; s < P->nsym; s++) lens[s] = P->len[s];
        bitw_t b = { bits, 0 };
        for (uint32_t g = 0; g < P->nseg; g++) {
            uint64_t start = b.nbits;
            uint32_t i0 = g * o->seg_syms, i1 = i0 + o->seg_syms;
            if (i1 > nf) i1 = nf;
            for (uint32_t i = i0; i < i1; i++) {
                uint32_t z = nzo_zigzag(coded_value(q, i, o));
                uint32_t s = sym_of(z, o->alphabet);
                bw_put_msb(&b, P->code[s], P->len[s]);
                if (s == 0) bw_put_lsb(&b, z, 32);
            }
            uint32_t sl = (uint32_t)(b.nbits - start);
            segt[2 * g] = (uint8_t)sl; segt[2 * g + 1] = (uint8_t)(sl >> 8);
        }
    }
}

/* Stream layout: 64-byte header | u64 offsets[n_frames] (pad16) | frames. */
static uint64_t frames_base(uint32_t n_frames) { return NZO_STREAM_HDR + pad16(8ull * n_frames); }

static void write_stream_header(uint8_t* out, uint64_t n, const nzo_opts* o, uint32_t n_frames,
                                uint32_t step_bits, uint64_t total) {
    memset(out, 0, NZO_STREAM_HDR);
    put_u32(out + 0, NZO_MAGIC_STREAM);
    put_u32(out + 4, 1u);
    put_u64(out + 8, n);
    put_u32(out + 16, o->chunk_elems);
    put_u32(out + 20, n_frames);
    put_u32(out + 24, step_bits);
    put_u32(out + 28, o->seg_syms);
    put_u32(out + 32, o->alphabet);
    put_u32(out + 36, o->predictor);
    put_u64(out + 40, total);
}

/* Worst-case bytes of one frame of nf symbols: RAW (FIXEDLEN never exceeds it, the selector never picks a
 * larger HUFFMAN), except when HUFFMAN is pinned: then every symbol may cost a 28-bit code plus 32 escape bits. */
static uint64_t frame_bound(uint64_t nf, const nzo_opts* o) {
    uint64_t pay = 4ull * nf;
    if (o->force_codec == NZO_HUFFMAN) {
        uint64_t nseg = (nf + o->seg_syms - 1) / o->seg_syms;
        uint64_t h = pad4(o->alphabet) + pad4(2ull * nseg) + 4ull * ((nf * 60ull + 31u) / 32u);
        if (h > pay) pay = h;
    }
    return pad16(NZO_HDR_BYTES + pay);
}

size_t nzo_compress_bound(size_t n, const nzo_opts* opts) {
    nzo_opts o;
    if (resolve_opts(opts, &o) || n == 0) return 0;
    uint64_t nfr = (n + o.chunk_elems - 1) / o.chunk_elems;
    uint64_t last = n - (nfr - 1) * o.chunk_elems;
    return (size_t)(NZO_STREAM_HDR + pad16(8ull * nfr) + (nfr - 1) * frame_bound(o.chunk_elems, &o) +
                    frame_bound(last, &o));
}

/*
 * Shared back end of compress and reduce: given per-frame integer codes (or
 * raw fp32 bits for frames that must be RAW) select, size and write all
 * frames.  get_frame() fills q / rawbits for one frame and says whether the
 * frame may be entropy coded.
 */
typedef int (*frame_src_fn)(void* ctx, uint32_t k, uint64_t i0, uint32_t nf, int32_t* q, uint32_t* rawbits);

static int emit_stream(frame_src_fn src, void* ctx, uint64_t n, const nzo_opts* o, uint32_t step_bits,
                       uint8_t* out, size_t cap, nzo_result* res) {
    const uint64_t nfr64 = (n + o->chunk_elems - 1) / o->chunk_elems;
    if (nfr64 > 0xFFFFFFFFull) return NZO_ERR_INVALID;
    const uint32_t nfr = (uint32_t)nfr64;
    memset(res, 0, sizeof *res);
    res->n_frames = nfr;
    uint64_t off = frames_base(nfr);
    if (off > cap) { res->status = NZO_ERR_CAPACITY; return NZO_ERR_CAPACITY; }
    int32_t* q = (int32_t*)malloc(sizeof(int32_t) * o->chunk_elems);
    uint32_t* rb = (uint32_t*)malloc(sizeof(uint32_t) * o->chunk_elems);
    frame_plan* P = (frame_plan*)malloc(sizeof(frame_plan));
    if (!q || !rb || !P) { free(q); free(rb); free(P); return NZO_ERR_INVALID; }
    memset(out + NZO_STREAM_HDR, 0, (size_t)(off - NZO_STREAM_HDR));
    int rc = NZO_OK;
    for (uint32_t k = 0; k < nfr; k++) {
        uint64_t i0 = (uint64_t)k * o->chunk_elems;
        uint32_t nf = (uint32_t)((n - i0 < o->chunk_elems) ? (n - i0) : o->chunk_elems);
        int quantizable = src(ctx, k, i0, nf, q, rb);
        if (quantizable) plan_frame(q, nf, o, P);
        else { memset(P, 0, sizeof *P); P->payload[NZO_RAW] = 4ull * nf; P->total[NZO_RAW] = pad16(NZO_HDR_BYTES + 4ull * nf); }
        int c = select_codec(P, quantizable, o);
        if (off + P->total[c] > cap) { rc = NZO_ERR_CAPACITY; break; }
        write_frame(out + off, c, q, rb, nf, P, o, step_bits);
        put_u64(out + NZO_STREAM_HDR + 8ull * k, off);
        off += P->total[c];
        if (c == NZO_RAW) res->n_raw++; else if (c == NZO_FIXEDLEN) res->n_fixed++; else res->n_huff++;
    }
    free(q); free(rb); free(P);
    if (rc) { res->status = (uint32_t)rc; res->bytes = 0; res->n_raw = res->n_fixed = res->n_huff = 0; return rc; }
    write_stream_header(out, n, o, nfr, step_bits, off);
    res->bytes = off;
    res->status = NZO_OK;
    return NZO_OK;
}

/* ------------------------------------------------------------------ */
/* 6. compress                                                          */
/* ------------------------------------------------------------------ */

typedef struct { const float* x; float eb, step, inv; } quant_ctx;

static int quant_src(void* vctx, uint32_t k, uint64_t i0, uint32_t nf, int32_t* q, uint32_t* rb) {
    (void)k;
    quant_ctx* c = (quant_ctx*)vctx;
    int all_ok = 1;
    for (uint32_t i = 0; i < nf; i++) {
        float x = c->x[i0 + i];
        rb[i] = f32_bits(x);
        int32_t v = 0;
        if (!nzo_quantize_one(x, c->eb, c->step, c->inv, &v)) all_ok = 0;
        q[i] = v;
    }
    return all_ok;          /* one unquantizable element makes the whole frame RAW */
}

int nzo_compress(const float* x, size_t n, float eb, const nzo_opts* opts, uint8_t* out, size_t cap,
                 nzo_result* res) {
    nzo_opts o; quant_ctx c;
    nzo_result dummy;
    if (!res) res = &dummy;
    memset(res, 0, sizeof *res);
    if (n == 0 || !x || !out) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    if (resolve_opts(opts, &o) || nzo_step_constants(eb, &c.step, &c.inv)) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    c.x = x; c.eb = eb;
    return emit_stream(quant_src, &c, n, &o, f32_bits(c.step), out, cap, res);
}

/* ------------------------------------------------------------------ */
/* 7. decode (receiver side of Algorithm 2: parse, validate, decode)    */
/* ------------------------------------------------------------------ */

typedef struct {
    uint64_t n; uint32_t chunk, n_frames, step_bits, seg_syms, K, predictor; uint64_t total;
} stream_hdr;

static int parse_stream(const uint8_t* s, size_t bytes, stream_hdr* h) {
    if (bytes < NZO_STREAM_HDR) return NZO_ERR_CORRUPT;
    if (get_u32(s) != NZO_MAGIC_STREAM || get_u32(s + 4) != 1u) return NZO_ERR_CORRUPT;
    h->n = get_u64(s + 8); h->chunk = get_u32(s + 16); h->n_frames = get_u32(s + 20);
    h->step_bits = get_u32(s + 24); h->seg_syms = get_u32(s + 28); h->K = get_u32(s + 32);
    h->predictor = get_u32(s + 36);
    h->total = get_u64(s + 40);
    if (h->predictor > 1u) return NZO_ERR_CORRUPT;
    if (h->n == 0 || h->chunk == 0 || h->chunk > NZO_MAX_CHUNK) return NZO_ERR_CORRUPT;
    if (h->seg_syms < 32u || h->seg_syms > 1024u) return NZO_ERR_CORRUPT;
    if (h->K < 2u || h->K > NZO_MAX_K || !is_pow2(h->K)) return NZO_ERR_CORRUPT;
    if ((h->n + h->chunk - 1) / h->chunk != h->n_frames) return NZO_ERR_CORRUPT;
    if (h->total > bytes || h->total < frames_base(h->n_frames)) return NZO_ERR_CORRUPT;
    return NZO_OK;
}

/* Receiver side of the delta predictor: running sums modulo 2^32, restarted at every segment. */
static void undo_prediction(int32_t* q, uint32_t nf, const stream_hdr* sh) {
    if (sh->predictor != 1u) return;
    for (uint32_t i = 0; i < nf; i++)
        if ((i % sh->seg_syms) != 0u) q[i] = (int32_t)((uint32_t)q[i] + (uint32_t)q[i - 1]);
}

/*
 * Validate and decode one frame to integer codes (coded frame) or raw fp32
 * bits (RAW frame).  Returns NZO_OK / NZO_ERR_CORRUPT / NZO_ERR_MISMATCH;
 * *is_raw tells which output array was filled.
 * Validation: magic, check word, codecId <= 2, rawBytes == 4*nf, payload
 * inside the stream and equal to the size the parameters imply or larger than
 * the minimum they imply, w <= 32, nsym <= K, Kraft sum <= 1, every segment
 * consumes exactly its recorded bit length.
 */
static int decode_frame(const uint8_t* s, uint64_t total, uint64_t off, uint32_t nf, const stream_hdr* sh,
                        int32_t* q, uint32_t* rawbits, int* is_raw) {
    *is_raw = 0;
    if ((off & 15u) || off < frames_base(sh->n_frames) || off + NZO_HDR_BYTES > total) return NZO_ERR_CORRUPT;
    const uint8_t* fr = s + off;
    uint32_t h[8], x = NZO_CHECK_XOR;
    for (int i = 0; i < 8; i++) h[i] = get_u32(fr + 4 * i);
    for (int i = 0; i < 7; i++) x ^= h[i];
    if (h[0] != NZO_MAGIC_FRAME || h[7] != x) return NZO_ERR_CORRUPT;
    const uint32_t codec = h[1], raw_bytes = h[2], payload = h[3], p0 = h[4], p1 = h[5];
    if (codec > 2u || raw_bytes != 4u * nf) return NZO_ERR_CORRUPT;
    if (off + NZO_HDR_BYTES + (uint64_t)payload > total) return NZO_ERR_CORRUPT;
    if (h[6] != sh->step_bits) return NZO_ERR_MISMATCH;
    const uint8_t* pay = fr + NZO_HDR_BYTES;
    if (codec == NZO_RAW) {
        if (payload != 4u * nf || p0 || p1) return NZO_ERR_CORRUPT;
        for (uint32_t i = 0; i < nf; i++) rawbits[i] = get_u32(pay + 4ull * i);
        *is_raw = 1;
        return NZO_OK;
    }
    if (codec == NZO_FIXEDLEN) {
        if (p0 > 32u || (p1 & 0x7FFFFFFFu) || (p1 >> 31) != sh->predictor) return NZO_ERR_CORRUPT;
        if (payload != 4ull * (((uint64_t)nf * p0 + 31u) / 32u)) return NZO_ERR_CORRUPT;
        bitr_t b = { pay, 0, 8ull * payload, 0 };
        for (uint32_t i = 0; i < nf; i++) q[i] = nzo_unzigzag(br_get_lsb(&b, (int)p0));
        if (b.overrun) return NZO_ERR_CORRUPT;
        undo_prediction(q, nf, sh);
        return NZO_OK;
    }
    /* HUFFMAN */
    const uint32_t nsym = p0, seg = p1 & 0xFFFFu, K = (p1 >> 16) & 0x7FFFu;
    if ((p1 >> 31) != sh->predictor) return NZO_ERR_CORRUPT;
    if (seg != sh->seg_syms || K != sh->K || nsym == 0 || nsym > K) return NZO_ERR_CORRUPT;
    const uint32_t nseg = (nf + seg - 1) / seg;
    const uint64_t tables = pad4(nsym) + pad4(2ull * nseg);
    if (payload < tables || (payload & 3u)) return NZO_ERR_CORRUPT;
    const uint8_t* lens = pay;
    const uint8_t* segt = pay + pad4(nsym);
    const uint8_t* bits = pay + tables;
    const uint64_t avail = 8ull * (payload - tables);
    /* code lengths: <= 28, Kraft sum <= 1, at least one used symbol */
    uint32_t count[33]; memset(count, 0, sizeof count);
    uint64_t kraft = 0; uint32_t used = 0;
    for (uint32_t t = 0; t < nsym; t++) {
        if (lens[t] > 28u) return NZO_ERR_CORRUPT;
        if (lens[t]) { count[lens[t]]++; kraft += 1ull << (28u - lens[t]); used++; }
    }
    for (uint64_t t = nsym; t < pad4(nsym); t++) if (lens[t]) return NZO_ERR_CORRUPT;
    if (used == 0 || kraft > (1ull << 28)) return NZO_ERR_CORRUPT;
    /* canonical decode tables: first code and first index per length */
    uint32_t first[33], index0[33], sorted[NZO_MAX_K];
    {
        uint32_t c = 0, idx = 0;
        count[0] = 0;
        for (int L = 1; L <= 32; L++) { c = (c + count[L - 1]) << 1; first[L] = c; index0[L] = idx; idx += count[L]; }
        uint32_t fill[33]; memcpy(fill, index0, sizeof fill);
        for (uint32_t t = 0; t < nsym; t++) if (lens[t]) sorted[fill[lens[t]]++] = t;
    }
    uint64_t sum_bits = 0;
    for (uint32_t g = 0; g < nseg; g++) sum_bits += (uint32_t)segt[2 * g] | ((uint32_t)segt[2 * g + 1] << 8);
    if ((nseg & 1u) && (segt[2 * nseg] || segt[2 * nseg + 1])) return NZO_ERR_CORRUPT;
    if (sum_bits > avail || 4ull * ((sum_bits + 31u) / 32u) != payload - tables) return NZO_ERR_CORRUPT;
    uint64_t pos = 0;
    for (uint32_t g = 0; g < nseg; g++) {
        uint32_t sl = (uint32_t)segt[2 * g] | ((uint32_t)segt[2 * g + 1] << 8);
        bitr_t b = { bits, pos, pos + sl, 0 };
        uint32_t i0 = g * seg, i1 = i0 + seg;
        if (i1 > nf) i1 = nf;
        for (uint32_t i = i0; i < i1; i++) {
            uint32_t code = 0, sym = 0; int found = 0;
            for (int L = 1; L <= 28 && !found; L++) {
                code = (code << 1) | br_get1(&b);
                if (b.overrun) return NZO_ERR_CORRUPT;
                if (count[L] && code >= first[L] && code - first[L] < count[L]) { sym = sorted[index0[L] + code - first[L]]; found = 1; }
            }
            if (!found) return NZO_ERR_CORRUPT;
            uint32_t z = sym ? sym - 1u : br_get_lsb(&b, 32);
            if (b.overrun) return NZO_ERR_CORRUPT;
            q[i] = nzo_unzigzag(z);
        }
        if (b.pos != b.end) return NZO_ERR_CORRUPT;
        pos += sl;
    }
    undo_prediction(q, nf, sh);
    return NZO_OK;
}

/*
 * Decode a whole stream to integer codes / raw bits.  frame_raw[k] = 1 when
 * frame k was RAW (then rawbits holds its elements, q is 0 there), 0 when
 * coded (q valid), 2 when the frame was rejected (both zero-filled).
 */
static int step_ok(float step) { return step >= 0x1p-100f && step <= 0x1p101f; }   /* also rejects NaN */

/* The receiver needs the bin width only; the *_step forms take it directly (a stream made by the stochastic
 * quantizer of section 11 has a width that is not derived from an error bound), the others derive it from eb. */
int nzo_decode_codes_step(const uint8_t* s, size_t bytes, size_t n, float step, int32_t* q, uint32_t* rawbits,
                          uint8_t* frame_raw, nzo_result* res) {
    stream_hdr sh;
    nzo_result dummy;
    if (!res) res = &dummy;
    memset(res, 0, sizeof *res);
    if (n == 0 || !s || !step_ok(step)) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    int rc = parse_stream(s, bytes, &sh);
    if (rc) { res->status = (uint32_t)rc; return rc; }
    if (sh.n != n || sh.step_bits != f32_bits(step)) { res->status = NZO_ERR_MISMATCH; return NZO_ERR_MISMATCH; }
    res->n_frames = sh.n_frames;
    res->bytes = sh.total;
    int worst = NZO_OK;
    for (uint32_t k = 0; k < sh.n_frames; k++) {
        uint64_t i0 = (uint64_t)k * sh.chunk;
        uint32_t nf = (uint32_t)((n - i0 < sh.chunk) ? (n - i0) : sh.chunk);
        uint64_t off = get_u64(s + NZO_STREAM_HDR + 8ull * k);
        int is_raw = 0;
        memset(q + i0, 0, 4ull * nf); memset(rawbits + i0, 0, 4ull * nf);
        int frc = decode_frame(s, sh.total, off, nf, &sh, q + i0, rawbits + i0, &is_raw);
        if (frc) {
            memset(q + i0, 0, 4ull * nf); memset(rawbits + i0, 0, 4ull * nf);
            if (frame_raw) frame_raw[k] = 2;
            if (frc > worst) worst = frc;      /* status = largest code over frames (order-free) */
            continue;
        }
        if (frame_raw) frame_raw[k] = (uint8_t)is_raw;
        if (is_raw) res->n_raw++;
        else if (get_u32(s + off + 4) == NZO_FIXEDLEN) res->n_fixed++;
        else res->n_huff++;
    }
    res->status = (uint32_t)worst;
    return worst;
}

int nzo_decode_codes(const uint8_t* s, size_t bytes, size_t n, float eb, int32_t* q, uint32_t* rawbits,
                     uint8_t* frame_raw, nzo_result* res) {
    float step, inv;
    if (nzo_step_constants(eb, &step, &inv)) { if (res) { memset(res, 0, sizeof *res); res->status = NZO_ERR_INVALID; } return NZO_ERR_INVALID; }
    return nzo_decode_codes_step(s, bytes, n, step, q, rawbits, frame_raw, res);
}

/* Decompress: decode then xhat = fl32(float(q)*step); RAW frames pass through.
 * A stream-level error (bad stream header, n or step mismatch) writes nothing;
 * a rejected frame is zero-filled and reported in the status. */
int nzo_decompress_step(const uint8_t* s, size_t bytes, float* out, size_t n, float step, nzo_result* res) {
    stream_hdr sh;
    nzo_result dummy;
    if (!res) res = &dummy;
    memset(res, 0, sizeof *res);
    if (n == 0 || !out || !s || !step_ok(step)) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    int rc = parse_stream(s, bytes, &sh);
    if (rc) { res->status = (uint32_t)rc; return rc; }
    if (sh.n != n || sh.step_bits != f32_bits(step)) { res->status = NZO_ERR_MISMATCH; return NZO_ERR_MISMATCH; }
    int32_t* q = (int32_t*)malloc(4ull * n);
    uint32_t* rb = (uint32_t*)malloc(4ull * n);
    uint8_t* fr = (uint8_t*)calloc(sh.n_frames, 1);
    if (!q || !rb || !fr) { free(q); free(rb); free(fr); return NZO_ERR_INVALID; }
    rc = nzo_decode_codes_step(s, bytes, n, step, q, rb, fr, res);
    for (uint32_t k = 0; k < sh.n_frames; k++) {
        uint64_t i0 = (uint64_t)k * sh.chunk;
        uint32_t nf = (uint32_t)((n - i0 < sh.chunk) ? (n - i0) : sh.chunk);
        for (uint32_t i = 0; i < nf; i++) {
            if (fr[k] == 1) out[i0 + i] = bits_f32(rb[i0 + i]);
            else if (fr[k] == 0) out[i0 + i] = nzo_dequantize_one(q[i0 + i], step);
            else out[i0 + i] = 0.0f;
        }
    }
    free(q); free(rb); free(fr);
    return rc;
}

int nzo_decompress(const uint8_t* s, size_t bytes, float* out, size_t n, float eb, nzo_result* res) {
    float step, inv;
    if (nzo_step_constants(eb, &step, &inv)) { if (res) { memset(res, 0, sizeof *res); res->status = NZO_ERR_INVALID; } return NZO_ERR_INVALID; }
    return nzo_decompress_step(s, bytes, out, n, step, res);
}

/* ------------------------------------------------------------------ */
/* 8. frame-wise reduce (compute part of the fused recv-reduce-send     */
/*    step of Sec. IV-D "In-Primitive Overlap")                         */
/* ------------------------------------------------------------------ */

typedef struct {
    const int32_t* qa; const int32_t* qb; const uint32_t* ra; const uint32_t* rb;
    const uint8_t* fa; const uint8_t* fb; float step;
} reduce_ctx;

static uint32_t canon_sum_bits(float a, float b) {
    volatile float s = a + b;
    float t = s;
    if (t != t) return NZO_CANON_NAN;      /* NaN sums are stored as one canonical NaN */
    return f32_bits(t);
}

/*
 * Frame k of the output: both inputs coded -> Q = qa + qb exactly (64-bit), re-planned and re-selected on
 * Q.  A frame in which some |Q| > 2^30 cannot be carried further as integer codes; like every frame the
 * entropy paths cannot take, it is committed as RAW (the safe fallback of Sec. IV-C / Algorithm 1,
 * CommitRawOrFail) and holds fl32(fl32(qa*step) + fl32(qb*step)) for every element.
 * Either input RAW -> RAW frame holding the fp32 sum of the two (dequantized or raw) values.
 * A frame of integer sums that the selector commits RAW all the same (codec pinned to RAW, no entropy candidate
 * passes the gates, or RAW wins the size tie at a width of 32 bits) holds the same fp32 sums of the dequantized
 * operands: a RAW frame always carries what the receiver would have computed from the two operands.
 */
static int reduce_src(void* vctx, uint32_t k, uint64_t i0, uint32_t nf, int32_t* q, uint32_t* rbits) {
    reduce_ctx* c = (reduce_ctx*)vctx;
    const int a_raw = c->fa[k] == 1, b_raw = c->fb[k] == 1;
    int coded = !a_raw && !b_raw;
    if (coded) {
        for (uint32_t i = 0; i < nf; i++) {
            int64_t Q = (int64_t)c->qa[i0 + i] + (int64_t)c->qb[i0 + i];
            if (Q > NZO_QSUM_MAX || Q < -(int64_t)NZO_QSUM_MAX) { coded = 0; break; }
            q[i] = (int32_t)Q;
        }
        if (coded) {
            /* the selector may still commit the frame RAW (pinned RAW, minimum gain, a width of 32 bits): like every
             * RAW frame of a reduce it then holds the fp32 sums of the two dequantized operands */
            for (uint32_t i = 0; i < nf; i++)
                rbits[i] = canon_sum_bits(nzo_dequantize_one(c->qa[i0 + i], c->step), nzo_dequantize_one(c->qb[i0 + i], c->step));
            return 1;
        }
    }
    for (uint32_t i = 0; i < nf; i++) {
        float va = a_raw ? bits_f32(c->ra[i0 + i]) : nzo_dequantize_one(c->qa[i0 + i], c->step);
        float vb = b_raw ? bits_f32(c->rb[i0 + i]) : nzo_dequantize_one(c->qb[i0 + i], c->step);
        rbits[i] = canon_sum_bits(va, vb);
        q[i] = 0;
    }
    return 0;
}

int nzo_reduce_frames_step(const uint8_t* a, size_t a_bytes, const uint8_t* b, size_t b_bytes, uint8_t* out, size_t cap,
                           size_t n, float step, const nzo_opts* opts, nzo_result* res) {
    nzo_opts o; stream_hdr ha, hb;
    nzo_result dummy;
    if (!res) res = &dummy;
    memset(res, 0, sizeof *res);
    if (n == 0 || !a || !b || !out) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    if (resolve_opts(opts, &o) || !step_ok(step)) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    int rc = parse_stream(a, a_bytes, &ha);
    if (!rc) rc = parse_stream(b, b_bytes, &hb);
    if (rc) { res->status = (uint32_t)rc; return rc; }
    /* both operands and the output agree on n, frame size and step */
    if (ha.n != n || hb.n != n || ha.chunk != hb.chunk || ha.chunk != o.chunk_elems ||
        ha.step_bits != hb.step_bits || ha.step_bits != f32_bits(step) ||
        ha.predictor != o.predictor || hb.predictor != o.predictor) { res->status = NZO_ERR_MISMATCH; return NZO_ERR_MISMATCH; }
    int32_t* qa = (int32_t*)malloc(4ull * n); int32_t* qb = (int32_t*)malloc(4ull * n);
    uint32_t* ra = (uint32_t*)malloc(4ull * n); uint32_t* rb = (uint32_t*)malloc(4ull * n);
    uint8_t* fa = (uint8_t*)calloc(ha.n_frames, 1); uint8_t* fb = (uint8_t*)calloc(ha.n_frames, 1);
    if (!qa || !qb || !ra || !rb || !fa || !fb) rc = NZO_ERR_INVALID;
    if (!rc) rc = nzo_decode_codes_step(a, a_bytes, n, step, qa, ra, fa, NULL);
    if (!rc) rc = nzo_decode_codes_step(b, b_bytes, n, step, qb, rb, fb, NULL);
    if (!rc) {
        reduce_ctx c = { qa, qb, ra, rb, fa, fb, step };
        rc = emit_stream(reduce_src, &c, n, &o, f32_bits(step), out, cap, res);
    } else {
        res->status = (uint32_t)rc;
    }
    free(qa); free(qb); free(ra); free(rb); free(fa); free(fb);
    return rc;
}

int nzo_reduce_frames(const uint8_t* a, size_t a_bytes, const uint8_t* b, size_t b_bytes, uint8_t* out, size_t cap,
                      size_t n, float eb, const nzo_opts* opts, nzo_result* res) {
    float step, inv;
    if (nzo_step_constants(eb, &step, &inv)) { if (res) { memset(res, 0, sizeof *res); res->status = NZO_ERR_INVALID; } return NZO_ERR_INVALID; }
    return nzo_reduce_frames_step(a, a_bytes, b, b_bytes, out, cap, n, step, opts, res);
}

/* ------------------------------------------------------------------ */
/* 8b. ring-step reduce: incoming frames + the rank's own fp32 data     */
/*     (the receive-reduce-send step of Sec. IV-D "In-Primitive         */
/*     Overlap": the local contribution is quantized at the interface,  */
/*     Sec. IV-B, and never entropy coded before it is added)           */
/* ------------------------------------------------------------------ */

/*
 * out = incoming (+) local.  The local message is quantized frame by frame exactly as nzo_compress would
 * quantize it (one unquantizable element makes its frame "raw": the original fp32 words stand for it), and
 * then takes the place of operand B of nzo_reduce_frames: both coded -> exact integer sum of the codes,
 * re-planned and re-selected; incoming frame RAW or local frame raw -> RAW frame of fp32 sums of the
 * (dequantized or raw) values.  |Q| > 2^30 in a coded frame -> that frame is RAW and holds the fp32 sums of
 * the two dequantized values (as in nzo_reduce_frames).
 */
int nzo_reduce_local(const uint8_t* in, size_t in_bytes, const float* local, uint8_t* out, size_t cap,
                     size_t n, float eb, const nzo_opts* opts, nzo_result* res) {
    nzo_opts o; stream_hdr hi; float step, inv;
    nzo_result dummy;
    if (!res) res = &dummy;
    memset(res, 0, sizeof *res);
    if (n == 0 || !in || !local || !out) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    if (resolve_opts(opts, &o) || nzo_step_constants(eb, &step, &inv)) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    int rc = parse_stream(in, in_bytes, &hi);
    if (rc) { res->status = (uint32_t)rc; return rc; }
    if (hi.n != n || hi.chunk != o.chunk_elems || hi.step_bits != f32_bits(step) || hi.predictor != o.predictor) {
        res->status = NZO_ERR_MISMATCH; return NZO_ERR_MISMATCH;
    }
    int32_t* qa = (int32_t*)malloc(4ull * n); int32_t* qb = (int32_t*)malloc(4ull * n);
    uint32_t* ra = (uint32_t*)malloc(4ull * n); uint32_t* rb = (uint32_t*)malloc(4ull * n);
    uint8_t* fa = (uint8_t*)calloc(hi.n_frames, 1); uint8_t* fb = (uint8_t*)calloc(hi.n_frames, 1);
    if (!qa || !qb || !ra || !rb || !fa || !fb) rc = NZO_ERR_INVALID;
    if (!rc) rc = nzo_decode_codes(in, in_bytes, n, eb, qa, ra, fa, NULL);
    if (!rc) {
        /* the local message, frame by frame: codes, original words, and the per-frame "raw" flag */
        for (uint32_t k = 0; k < hi.n_frames; k++) {
            const uint64_t i0 = (uint64_t)k * o.chunk_elems;
            const uint64_t i1 = (i0 + o.chunk_elems < n) ? i0 + o.chunk_elems : n;
            int all_ok = 1;
            for (uint64_t i = i0; i < i1; i++) {
                int32_t v = 0;
                if (!nzo_quantize_one(local[i], eb, step, inv, &v)) all_ok = 0;
                qb[i] = v; rb[i] = f32_bits(local[i]);
            }
            fb[k] = all_ok ? 0 : 1;
        }
        reduce_ctx c = { qa, qb, ra, rb, fa, fb, step };
        rc = emit_stream(reduce_src, &c, n, &o, f32_bits(step), out, cap, res);
    } else {
        res->status = (uint32_t)rc;
    }
    free(qa); free(qb); free(ra); free(rb); free(fa); free(fb);
    return rc;
}

/* ------------------------------------------------------------------ */
/* 8c. k-ary reduce: one output stream from k operand streams           */
/*     (the reduction of Sec. IV-D "In-Primitive Overlap" taken over    */
/*     all the contributions a rank holds at once, e.g. the k chunks    */
/*     that arrive in a direct or tree-shaped reduce-scatter)           */
/* ------------------------------------------------------------------ */

typedef struct { const int32_t* q; const uint32_t* r; const uint8_t* f; } acc_ctx;

static int acc_src(void* vctx, uint32_t k, uint64_t i0, uint32_t nf, int32_t* q, uint32_t* rbits) {
    acc_ctx* c = (acc_ctx*)vctx;
    memcpy(q, c->q + i0, 4ull * nf);
    memcpy(rbits, c->r + i0, 4ull * nf);
    return c->f[k] == 0;
}

/*
 * out = s_0 (+) s_1 (+) ... (+) s_{k-1}, the operands taken in the order given: a left fold of the two-operand rule
 * of nzo_reduce_frames, frame by frame, without the intermediate streams.  A frame's running value is either integer
 * codes or fp32 words.  Adding operand p: while the running value and the operand's frame are both coded, the codes
 * are added exactly; if some partial sum passes 2^30 in magnitude at this operand, or the operand's frame is RAW,
 * the running value becomes fp32 -- fl32(v + v_p) element by element with v the running value (dequantized if it
 * was coded) and v_p the operand's value (dequantized or raw) -- and stays fp32 for the operands that follow.
 * Frames that end coded are re-planned and re-selected on the sums (one that the selector commits RAW holds the fp32
 * form of the last step, as in nzo_reduce_frames); the others are RAW.  Since a frame of codes (or of fp32 words)
 * survives being written and read back unchanged, the result is, byte for byte, what the chain
 * nzo_reduce_frames(... nzo_reduce_frames(nzo_reduce_frames(s_0, s_1), s_2) ..., s_{k-1}) gives as long as the
 * chain's intermediate streams keep integer sums as codes (no pinned RAW, no gate that turns such a frame RAW on the
 * way: those options then apply to the final stream only).
 */
int nzo_reduce_k_step(const uint8_t* const* streams, const size_t* bytes, uint32_t k, uint8_t* out, size_t cap,
                      size_t n, float step, const nzo_opts* opts, nzo_result* res) {
    nzo_opts o;
    nzo_result dummy;
    if (!res) res = &dummy;
    memset(res, 0, sizeof *res);
    if (n == 0 || !streams || !bytes || !out || k < 2 || k > NZO_MAX_OPERANDS) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    for (uint32_t p = 0; p < k; p++) if (!streams[p]) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    if (resolve_opts(opts, &o) || !step_ok(step)) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    int rc = NZO_OK;
    uint32_t n_frames = 0;
    for (uint32_t p = 0; p < k && !rc; p++) {
        stream_hdr h;
        rc = parse_stream(streams[p], bytes[p], &h);
        if (!rc && (h.n != n || h.chunk != o.chunk_elems || h.step_bits != f32_bits(step) || h.predictor != o.predictor))
            rc = NZO_ERR_MISMATCH;
        n_frames = h.n_frames;
    }
    if (rc) { res->status = (uint32_t)rc; return rc; }
    int32_t* qs = (int32_t*)malloc(4ull * n); int32_t* qp = (int32_t*)malloc(4ull * n);
    uint32_t* rs = (uint32_t*)malloc(4ull * n); uint32_t* rp = (uint32_t*)malloc(4ull * n);
    uint8_t* fs = (uint8_t*)calloc(n_frames, 1); uint8_t* fp = (uint8_t*)calloc(n_frames, 1);
    if (!qs || !qp || !rs || !rp || !fs || !fp) rc = NZO_ERR_INVALID;
    if (!rc) rc = nzo_decode_codes_step(streams[0], bytes[0], n, step, qs, rs, fs, NULL);   /* the running value starts as s_0 */
    for (uint32_t p = 1; p < k && !rc; p++) {
        rc = nzo_decode_codes_step(streams[p], bytes[p], n, step, qp, rp, fp, NULL);
        if (rc) break;
        for (uint32_t f = 0; f < n_frames; f++) {
            const uint64_t i0 = (uint64_t)f * o.chunk_elems;
            const uint64_t i1 = (i0 + o.chunk_elems < n) ? i0 + o.chunk_elems : n;
            int coded = fs[f] == 0 && fp[f] == 0;
            if (coded)
                for (uint64_t i = i0; i < i1; i++) {
                    const int64_t Q = (int64_t)qs[i] + (int64_t)qp[i];
                    if (Q > NZO_QSUM_MAX || Q < -(int64_t)NZO_QSUM_MAX) { coded = 0; break; }
                }
            if (coded) {
                /* (the fp32 form of this step is kept beside the codes: if it is the last one and the selector commits
                 * the frame RAW, that is what the frame holds, as in nzo_reduce_frames) */
                for (uint64_t i = i0; i < i1; i++) {
                    rs[i] = canon_sum_bits(nzo_dequantize_one(qs[i], step), nzo_dequantize_one(qp[i], step));
                    qs[i] += qp[i];
                }
                continue;
            }
            for (uint64_t i = i0; i < i1; i++) {
                const float v = fs[f] ? bits_f32(rs[i]) : nzo_dequantize_one(qs[i], step);
                const float vp = fp[f] ? bits_f32(rp[i]) : nzo_dequantize_one(qp[i], step);
                rs[i] = canon_sum_bits(v, vp);
                qs[i] = 0;
            }
            fs[f] = 1;
        }
    }
    if (!rc) {
        acc_ctx c = { qs, rs, fs };
        rc = emit_stream(acc_src, &c, n, &o, f32_bits(step), out, cap, res);
    } else {
        res->status = (uint32_t)rc;
    }
    free(qs); free(qp); free(rs); free(rp); free(fs); free(fp);
    return rc;
}

int nzo_reduce_k(const uint8_t* const* streams, const size_t* bytes, uint32_t k, uint8_t* out, size_t cap,
                 size_t n, float eb, const nzo_opts* opts, nzo_result* res) {
    float step, inv;
    if (nzo_step_constants(eb, &step, &inv)) { if (res) { memset(res, 0, sizeof *res); res->status = NZO_ERR_INVALID; } return NZO_ERR_INVALID; }
    return nzo_reduce_k_step(streams, bytes, k, out, cap, n, step, opts, res);
}

/* ------------------------------------------------------------------ */
/* 9. single-frame entry points used by the pins                        */
/* ------------------------------------------------------------------ */

/*
 * Plan one frame of integer codes: fills sizes[3] (total bytes per codec),
 * payloads[3], w, nsym, huff_bits, len[K], code[K] and returns the selector's
 * choice.
 */
int nzo_frame_plan(const int32_t* q, uint32_t nf, int quantizable, const nzo_opts* opts, uint64_t* totals,
                   uint64_t* payloads, uint32_t* w, uint32_t* nsym, uint64_t* huff_bits, uint8_t* len,
                   uint32_t* code) {
    nzo_opts o;
    if (resolve_opts(opts, &o) || nf == 0 || nf > o.chunk_elems) return -1;
    frame_plan* P = (frame_plan*)malloc(sizeof *P);
    plan_frame(q, nf, &o, P);
    for (int c = 0; c < 3; c++) { totals[c] = P->total[c]; payloads[c] = P->payload[c]; }
    *w = P->w; *nsym = P->nsym; *huff_bits = P->huff_bits;
    memcpy(len, P->len, o.alphabet); memcpy(code, P->code, 4u * o.alphabet);
    int c = select_codec(P, quantizable, &o);
    free(P);
    return c;
}

/* Write one frame of integer codes with a pinned codec; returns its bytes. */
int64_t nzo_frame_encode(const int32_t* q, const uint32_t* rawbits, uint32_t nf, int codec, const nzo_opts* opts,
                         uint32_t step_bits, uint8_t* dst, size_t cap) {
    nzo_opts o;
    if (resolve_opts(opts, &o) || nf == 0 || nf > o.chunk_elems || codec < 0 || codec > 2) return -1;
    frame_plan* P = (frame_plan*)malloc(sizeof *P);
    plan_frame(q, nf, &o, P);
    int64_t t = (int64_t)P->total[codec];
    if ((uint64_t)t > cap) { free(P); return -2; }
    write_frame(dst, codec, q, rawbits, nf, P, &o, step_bits);
    free(P);
    return t;
}

/* ------------------------------------------------------------------ */
/* 10. sampled runtime entropy arbitration (REA), Sec. IV-C, Eq. 1-2,   */
/*     Algorithm 1 taken literally: the plan is made from a bounded      */
/*     sample and a cached Huffman context, only the selected codec      */
/*     touches the full frame, the realized size is validated and RAW    */
/*     is the fallback.                                                  */
/* ------------------------------------------------------------------ */

/*
 * The Huffman context ("pre-initialized Huffman context huffCtx", "cached codebook", Sec. IV-C): one
 * canonical prefix code over the K symbols of the alphabet, built ahead of time and shared by all frames.
 * The paper does not say how it is initialised.  Format v1: from a calibration message of at most 2^20
 * values (same quantizer), count the symbols, add one to every count (so that every symbol, the escape
 * included, owns a code and any frame can be coded), build the optimal lengths with the two-queue rule of
 * section 2 and assign canonical codes.  With at most 2^20 + K <= Fib(31) counted symbols no length exceeds 28.
 */
typedef struct {
    uint32_t valid;                /* 1 once built; REA's "context validity" gate */
    uint32_t K;                    /* alphabet the code was built for             */
    uint8_t  len[NZO_MAX_K];
    uint32_t code[NZO_MAX_K];
} nzo_context;

int nzo_context_build(const float* sample, size_t n_s, float eb, const nzo_opts* opts, nzo_context* ctx) {
    nzo_opts o; float step, inv;
    memset(ctx, 0, sizeof *ctx);
    if (!sample || n_s == 0 || n_s > NZO_MAX_CHUNK) return NZO_ERR_INVALID;
    if (resolve_opts(opts, &o) || nzo_step_constants(eb, &step, &inv)) return NZO_ERR_INVALID;
    uint32_t f[NZO_MAX_K];
    for (uint32_t s = 0; s < o.alphabet; s++) f[s] = 1;
    for (size_t i = 0; i < n_s; i++) {
        int32_t q = 0;
        if (!nzo_quantize_one(sample[i], eb, step, inv, &q)) continue;    /* values that cannot be coded do not count */
        f[sym_of(nzo_zigzag(q), o.alphabet)]++;
    }
    nzo_huffman_lengths(f, o.alphabet, ctx->len);
    nzo_canonical_codes(ctx->len, o.alphabet, ctx->code);
    ctx->K = o.alphabet;
    ctx->valid = 1;
    return NZO_OK;
}

typedef struct {
    uint32_t sample_bytes;         /* SampleWindow: at most this many bytes of the frame's prefix; 0 -> 65536 (Sec. IV-C) */
    uint32_t small_batch_bytes;    /* SmallBatchFastPath: frames with fewer raw bytes go RAW unprofiled; default 0        */
    /* Cost model of Eq. 1, T_c = alpha_c + lambda_enc*E_c + P_c/beta_eff(pi) + lambda_dec*D_c, in integers.  The
     * caller supplies what TransportHint and calibration would: link_ps_per_byte = 1/beta_eff in picoseconds per
     * byte (0 = no hint: the cost is the transmitted size alone), and per entropy codec the fixed cost alpha_c in
     * nanoseconds and the exposed codec time lambda_enc*E_c + lambda_dec*D_c as picoseconds per raw byte.  RAW has
     * no codec cost (Sec. IV-C). */
    uint32_t link_ps_per_byte;
    uint32_t fixed_alpha_ns, fixed_ps_per_byte;
    uint32_t huff_alpha_ns, huff_ps_per_byte;
    uint32_t reserved;             /* 0 */
} nzo_rea_opts;

typedef struct {
    uint64_t span_bytes;           /* extent of the slotted stream (what a decoder is handed)                 */
    uint64_t wire_bytes;           /* stream header + offsets table + the realized frames: what is transmitted */
    uint32_t status, n_frames, n_raw, n_fixed, n_huff;
    uint32_t n_fallback;           /* frames planned as FIXEDLEN / HUFFMAN whose realized output was rejected  */
} nzo_rea_result;

/* One frame's plan (ProfileSample + ArbitratePlan), exposed for the pins. */
typedef struct {
    uint32_t n_s;                  /* sampled elements                                  */
    uint32_t sample_ok;            /* every sampled element quantizable                 */
    uint32_t w_s;                  /* width implied by the sample's largest zigzag code */
    uint64_t sample_bits;          /* Huffman bits of the sample under the context      */
    uint64_t pred_payload[3];      /* predicted payload bytes per codec                 */
    int      plan;                 /* planned codec                                     */
} nzo_rea_plan;

/*
 * ProfileSample + ArbitratePlan for one frame of nf elements starting at x (Algorithm 1, "Arbitration
 * overhead"): the sample is the prefix of min(nf, sample_bytes/4) elements; FIXEDLEN's width is the bit
 * length of the sample's largest zigzag code (the max-|x| scan); HUFFMAN's size follows the sample's
 * K-bin histogram and the context's code lengths (expected code length), scaled from the sample to the
 * frame with integer arithmetic, rounded up: bits = ceil(sample_bits * nf / n_s).  Predicted payloads
 * include the codec's tables.  A candidate is admissible if its predicted payload fits the payload
 * capacity (the RAW size: a frame's slot holds a RAW frame), meets the minimum gain, and -- HUFFMAN --
 * the context is valid for this alphabet and rawBytes >= T_huff.  Eq. 2: the candidate of least predicted
 * cost, ties to the lower codec id; a pinned codec replaces the choice.  The cost is Eq. 1 evaluated in
 * picoseconds with the caller's transport hint and codec costs, T_c = 1000*alpha_c + codec_ps_c*rawBytes +
 * link_ps*total_c (RAW: link_ps*total_RAW), or the predicted total bytes when there is no hint.
 */
static uint64_t rea_cost(const nzo_rea_opts* ro, int codec, uint64_t rawb, uint64_t total) {
    if (ro->link_ps_per_byte == 0u) return total;
    uint64_t t = (uint64_t)ro->link_ps_per_byte * total;
    if (codec == NZO_FIXEDLEN) t += 1000ull * ro->fixed_alpha_ns + (uint64_t)ro->fixed_ps_per_byte * rawb;
    if (codec == NZO_HUFFMAN) t += 1000ull * ro->huff_alpha_ns + (uint64_t)ro->huff_ps_per_byte * rawb;
    return t;
}

/* ArbitratePlan on a profiled sample (P->n_s, P->sample_ok, P->w_s, P->sample_bits filled in). */
static void rea_arbitrate(uint32_t nf, const nzo_opts* o, const nzo_rea_opts* ro, int ctx_ok, nzo_rea_plan* P) {
    const uint32_t K = o->alphabet;
    const uint64_t rawb = 4ull * nf;
    const uint64_t nseg = (nf + o->seg_syms - 1) / o->seg_syms;
    const uint64_t pred_bits = (P->sample_bits * nf + P->n_s - 1) / P->n_s;
    P->pred_payload[NZO_FIXEDLEN] = 4ull * (((uint64_t)nf * P->w_s + 31u) / 32u);
    P->pred_payload[NZO_HUFFMAN] = pad4(K) + pad4(2ull * nseg) + 4ull * ((pred_bits + 31u) / 32u);
    if (o->force_codec >= 0) {
        P->plan = (o->force_codec == NZO_HUFFMAN && !ctx_ok) ? NZO_RAW : o->force_codec;
        return;
    }
    uint64_t best_cost = rea_cost(ro, NZO_RAW, rawb, pad16(NZO_HDR_BYTES + rawb));
    for (int c = NZO_FIXEDLEN; c <= NZO_HUFFMAN; c++) {
        if (c == NZO_HUFFMAN && (!ctx_ok || rawb < o->huff_min_bytes)) continue;
        const uint64_t p = P->pred_payload[c];
        if (p > rawb) continue;                                  /* predicted payload must fit the payload capacity */
        if ((rawb - p) * 1000ull < (uint64_t)o->min_gain_permil * rawb) continue;
        const uint64_t t = rea_cost(ro, c, rawb, pad16(NZO_HDR_BYTES + p));
        if (t < best_cost) { best_cost = t; P->plan = c; }
    }
}

static void rea_plan_frame(const float* x, uint32_t nf, float eb, float step, float inv, const nzo_opts* o,
                           const nzo_rea_opts* ro, const nzo_context* ctx, nzo_rea_plan* P) {
    memset(P, 0, sizeof *P);
    const uint32_t K = o->alphabet;
    const uint64_t rawb = 4ull * nf;
    (void)step;
    P->pred_payload[NZO_RAW] = rawb;
    P->plan = NZO_RAW;
    if (rawb < ro->small_batch_bytes) return;                    /* SmallBatchFastPath */
    P->n_s = ro->sample_bytes / 4u < nf ? ro->sample_bytes / 4u : nf;
    if (P->n_s == 0) return;
    const int ctx_ok = ctx && ctx->valid && ctx->K == K;
    uint32_t zmax = 0;
    P->sample_ok = 1;
    for (uint32_t i = 0; i < P->n_s; i++) {
        int32_t q = 0;
        if (!nzo_quantize_one(x[i], eb, step, inv, &q)) { P->sample_ok = 0; break; }
        uint32_t z = nzo_zigzag(q);
        if (z > zmax) zmax = z;
        if (ctx_ok) { uint32_t s = sym_of(z, K); P->sample_bits += ctx->len[s] + (s == 0 ? 32u : 0u); }
    }
    if (!P->sample_ok) return;                                   /* the sample already shows the frame cannot be coded */
    P->w_s = (uint32_t)bit_length32(zmax);
    rea_arbitrate(nf, o, ro, ctx_ok, P);
}

/* The same for a frame that exists as integer codes already (the sums of a reduce step): the sample is the prefix
 * of the codes, every code is codable. */
static void rea_plan_codes(const int32_t* q, uint32_t nf, const nzo_opts* o, const nzo_rea_opts* ro,
                           const nzo_context* ctx, nzo_rea_plan* P) {
    memset(P, 0, sizeof *P);
    const uint32_t K = o->alphabet;
    const uint64_t rawb = 4ull * nf;
    P->pred_payload[NZO_RAW] = rawb;
    P->plan = NZO_RAW;
    if (rawb < ro->small_batch_bytes) return;
    P->n_s = ro->sample_bytes / 4u < nf ? ro->sample_bytes / 4u : nf;
    if (P->n_s == 0) return;
    const int ctx_ok = ctx && ctx->valid && ctx->K == K;
    uint32_t zmax = 0;
    P->sample_ok = 1;
    for (uint32_t i = 0; i < P->n_s; i++) {
        uint32_t z = nzo_zigzag(q[i]);
        if (z > zmax) zmax = z;
        if (ctx_ok) { uint32_t s = sym_of(z, K); P->sample_bits += ctx->len[s] + (s == 0 ? 32u : 0u); }
    }
    P->w_s = (uint32_t)bit_length32(zmax);
    rea_arbitrate(nf, o, ro, ctx_ok, P);
}

int nzo_rea_plan_frame(const float* x, uint32_t nf, float eb, const nzo_opts* opts, const nzo_rea_opts* ropts,
                       const nzo_context* ctx, nzo_rea_plan* P) {
    nzo_opts o; float step, inv;
    nzo_rea_opts ro = { 65536u, 0u, 0u, 0u, 0u, 0u, 0u, 0u };
    if (ropts) { ro = *ropts; if (ro.sample_bytes == 0) ro.sample_bytes = 65536u; }
    if (ro.reserved) return NZO_ERR_INVALID;
    if (resolve_opts(opts, &o) || nzo_step_constants(eb, &step, &inv) || nf == 0 || nf > o.chunk_elems) return NZO_ERR_INVALID;
    rea_plan_frame(x, nf, eb, step, inv, &o, &ro, ctx, P);
    return NZO_OK;
}

/*
 * EncodePlan + AcceptRealized + CommitRawOrFail for one frame, written at dst (a slot that holds a RAW
 * frame).  FIXEDLEN is materialised with the sampled width, HUFFMAN with the context's code; either fails
 * if an element cannot be quantized, FIXEDLEN also if a zigzag code needs more than w_s bits.  The
 * realized payload P is accepted if the materialisation succeeded, P <= payload capacity (= rawBytes)
 * and the minimum gain holds for P; otherwise the frame is committed as RAW with the original values.
 * Returns the codec committed; *total = the frame's padded bytes; *fell_back = 1 if a non-RAW plan was
 * rejected.
 */
static int rea_commit_codes(uint8_t* dst, const int32_t* q, const uint32_t* rb, int ok, uint32_t nf, const nzo_opts* o,
                            const nzo_context* ctx, const nzo_rea_plan* P, uint32_t step_bits, frame_plan* FP,
                            uint64_t* total, int* fell_back) {
    const uint64_t rawb = 4ull * nf;
    *fell_back = 0;
    memset(FP, 0, sizeof *FP);
    FP->payload[NZO_RAW] = rawb; FP->total[NZO_RAW] = pad16(NZO_HDR_BYTES + rawb);
    int codec = NZO_RAW;
    if (P->plan == NZO_FIXEDLEN && ok) {
        const uint32_t w = P->w_s;
        for (uint32_t i = 0; i < nf && ok; i++) if (w < 32u && (nzo_zigzag(q[i]) >> w) != 0u) ok = 0;
        FP->w = w;
        FP->payload[NZO_FIXEDLEN] = 4ull * (((uint64_t)nf * w + 31u) / 32u);
        codec = NZO_FIXEDLEN;
    } else if (P->plan == NZO_HUFFMAN && ok) {
        const uint32_t K = o->alphabet;
        FP->nsym = K;
        memcpy(FP->len, ctx->len, K); memcpy(FP->code, ctx->code, 4u * K);
        FP->nseg = (nf + o->seg_syms - 1) / o->seg_syms;
        for (uint32_t i = 0; i < nf; i++) { uint32_t s = sym_of(nzo_zigzag(q[i]), K); FP->huff_bits += FP->len[s] + (s == 0 ? 32u : 0u); }
        FP->payload[NZO_HUFFMAN] = pad4(K) + pad4(2ull * FP->nseg) + 4ull * ((FP->huff_bits + 31u) / 32u);
        codec = NZO_HUFFMAN;
    }
    if (codec != NZO_RAW) {
        const uint64_t p = FP->payload[codec];
        if (!ok || p > rawb || (rawb - p) * 1000ull < (uint64_t)o->min_gain_permil * rawb) codec = NZO_RAW;   /* AcceptRealized */
    }
    if (codec == NZO_RAW && P->plan != NZO_RAW) *fell_back = 1;
    FP->total[codec] = pad16(NZO_HDR_BYTES + FP->payload[codec]);
    write_frame(dst, codec, q, rb, nf, FP, o, step_bits);
    *total = FP->total[codec];
    return codec;
}

static int rea_commit_frame(uint8_t* dst, const float* x, uint32_t nf, float eb, float step, float inv,
                            const nzo_opts* o, const nzo_context* ctx, const nzo_rea_plan* P, uint32_t step_bits,
                            int32_t* q, uint32_t* rb, frame_plan* FP, uint64_t* total, int* fell_back) {
    int ok = 1;
    for (uint32_t i = 0; i < nf; i++) {
        rb[i] = f32_bits(x[i]);
        q[i] = 0;
        if (P->plan != NZO_RAW && !nzo_quantize_one(x[i], eb, step, inv, &q[i])) ok = 0;
    }
    return rea_commit_codes(dst, q, rb, ok, nf, o, ctx, P, step_bits, FP, total, fell_back);
}

/*
 * Whole message.  Stream layout ("slotted"): the same container as nzo_compress, but frame k sits at the
 * fixed offset base + k * slot, slot = pad16(32 + 4*chunk_elems) -- each frame is materialised in a slot
 * that can hold its RAW form, as the paper's frames are materialised in a staging bank, and its
 * byte-accurate length (header: payloadBytes) is what a transport would send (Sec. IV-D).  The bytes
 * between a frame's end and the next slot are not part of the stream (zero here).  total_bytes in the
 * stream header = end of the last frame.  cap must hold every slot (nzo_compress_bound), else
 * NZO_ERR_CAPACITY and nothing is published.  The stream decodes with nzo_decompress unchanged.
 */
int nzo_compress_rea(const float* x, size_t n, float eb, const nzo_opts* opts, const nzo_rea_opts* ropts,
                     const nzo_context* ctx, uint8_t* out, size_t cap, nzo_rea_result* res, uint8_t* plans) {
    nzo_opts o; float step, inv;
    nzo_rea_opts ro = { 65536u, 0u, 0u, 0u, 0u, 0u, 0u, 0u };
    nzo_rea_result dummy;
    if (!res) res = &dummy;
    memset(res, 0, sizeof *res);
    if (ropts) { ro = *ropts; if (ro.sample_bytes == 0) ro.sample_bytes = 65536u; }
    if (n == 0 || !x || !out || ro.reserved) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    if (resolve_opts(opts, &o) || nzo_step_constants(eb, &step, &inv)) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    if (o.predictor) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }     /* the sampled path codes the codes themselves */
    const uint64_t nfr64 = (n + o.chunk_elems - 1) / o.chunk_elems;
    if (nfr64 > 0xFFFFFFFFull) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    const uint32_t nfr = (uint32_t)nfr64;
    res->n_frames = nfr;
    const uint64_t base = frames_base(nfr), slot = pad16(NZO_HDR_BYTES + 4ull * o.chunk_elems);
    const uint32_t last_nf = (uint32_t)(n - (uint64_t)(nfr - 1) * o.chunk_elems);
    const uint64_t need = base + (uint64_t)(nfr - 1) * slot + pad16(NZO_HDR_BYTES + 4ull * last_nf);
    if (need > cap) { res->status = NZO_ERR_CAPACITY; return NZO_ERR_CAPACITY; }
    int32_t* q = (int32_t*)malloc(4ull * o.chunk_elems);
    uint32_t* rb = (uint32_t*)malloc(4ull * o.chunk_elems);
    frame_plan* FP = (frame_plan*)malloc(sizeof *FP);
    if (!q || !rb || !FP) { free(q); free(rb); free(FP); res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    memset(out, 0, (size_t)need);
    const uint32_t step_bits = f32_bits(step);
    uint64_t wire = base, end = base;
    for (uint32_t k = 0; k < nfr; k++) {
        const uint64_t i0 = (uint64_t)k * o.chunk_elems;
        const uint32_t nf = (uint32_t)((n - i0 < o.chunk_elems) ? (n - i0) : o.chunk_elems);
        const uint64_t off = base + (uint64_t)k * slot;
        nzo_rea_plan P;
        uint64_t total = 0; int fb = 0;
        rea_plan_frame(x + i0, nf, eb, step, inv, &o, &ro, ctx, &P);
        int c = rea_commit_frame(out + off, x + i0, nf, eb, step, inv, &o, ctx, &P, step_bits, q, rb, FP, &total, &fb);
        put_u64(out + NZO_STREAM_HDR + 8ull * k, off);
        if (plans) plans[k] = (uint8_t)P.plan;
        wire += total; end = off + total;
        res->n_fallback += (uint32_t)fb;
        if (c == NZO_RAW) res->n_raw++; else if (c == NZO_FIXEDLEN) res->n_fixed++; else res->n_huff++;
    }
    free(q); free(rb); free(FP);
    write_stream_header(out, n, &o, nfr, step_bits, end);
    res->span_bytes = end; res->wire_bytes = wire; res->status = NZO_OK;
    return NZO_OK;
}


/*
 * Ring-step reduce with the sampled arbitration on the way out (the receive-reduce-send step of Sec. IV-D with the
 * selector of Sec. IV-C / Algorithm 1 in front of the send, as the paper's pipeline has it): the incoming stream is
 * decoded, the rank's own data quantized and added exactly as in nzo_reduce_local; every output frame is then
 * committed by Algorithm 1 on its integer sums -- plan from a prefix sample of the sums and the cached context, only
 * the planned codec materialised, realized size validated, RAW otherwise -- into the slotted stream of
 * nzo_compress_rea.  A frame that has no integer sums (incoming frame RAW, local element that cannot be quantized, a
 * sum beyond 2^30) is RAW with the fp32 sums of nzo_reduce_local and counts neither as planned nor as fallback.  The
 * RAW form of a coded frame whose realized output is rejected holds the sums of the dequantized operands,
 * fl32(fl32(qa*step) + fl32(qb*step)), like any frame whose codes cannot be carried on.
 */
int nzo_reduce_local_rea(const uint8_t* in, size_t in_bytes, const float* local, size_t n, float eb, const nzo_opts* opts,
                         const nzo_rea_opts* ropts, const nzo_context* ctx, uint8_t* out, size_t cap, nzo_rea_result* res,
                         uint8_t* plans) {
    nzo_opts o; stream_hdr hi; float step, inv;
    nzo_rea_opts ro = { 65536u, 0u, 0u, 0u, 0u, 0u, 0u, 0u };
    nzo_rea_result dummy;
    if (!res) res = &dummy;
    memset(res, 0, sizeof *res);
    if (ropts) { ro = *ropts; if (ro.sample_bytes == 0) ro.sample_bytes = 65536u; }
    if (n == 0 || !in || !local || !out || ro.reserved) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    if (resolve_opts(opts, &o) || nzo_step_constants(eb, &step, &inv) || o.predictor) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    int rc = parse_stream(in, in_bytes, &hi);
    if (rc) { res->status = (uint32_t)rc; return rc; }
    if (hi.n != n || hi.chunk != o.chunk_elems || hi.step_bits != f32_bits(step) || hi.predictor != 0u) {
        res->status = NZO_ERR_MISMATCH; return NZO_ERR_MISMATCH;
    }
    const uint32_t nfr = hi.n_frames;
    res->n_frames = nfr;
    const uint64_t base = frames_base(nfr), slot = pad16(NZO_HDR_BYTES + 4ull * o.chunk_elems);
    const uint32_t last_nf = (uint32_t)(n - (uint64_t)(nfr - 1) * o.chunk_elems);
    const uint64_t need = base + (uint64_t)(nfr - 1) * slot + pad16(NZO_HDR_BYTES + 4ull * last_nf);
    if (need > cap) { res->status = NZO_ERR_CAPACITY; return NZO_ERR_CAPACITY; }
    int32_t* qa = (int32_t*)malloc(4ull * n); int32_t* qb = (int32_t*)malloc(4ull * n);
    uint32_t* ra = (uint32_t*)malloc(4ull * n); uint32_t* rb = (uint32_t*)malloc(4ull * n);
    uint8_t* fa = (uint8_t*)calloc(nfr, 1); uint8_t* fb = (uint8_t*)calloc(nfr, 1);
    int32_t* q = (int32_t*)malloc(4ull * o.chunk_elems);
    uint32_t* rw = (uint32_t*)malloc(4ull * o.chunk_elems);
    frame_plan* FP = (frame_plan*)malloc(sizeof *FP);
    if (!qa || !qb || !ra || !rb || !fa || !fb || !q || !rw || !FP) rc = NZO_ERR_INVALID;
    if (!rc) rc = nzo_decode_codes(in, in_bytes, n, eb, qa, ra, fa, NULL);
    if (!rc) {
        for (uint32_t k = 0; k < nfr; k++) {
            const uint64_t i0 = (uint64_t)k * o.chunk_elems;
            const uint64_t i1 = (i0 + o.chunk_elems < n) ? i0 + o.chunk_elems : n;
            int all_ok = 1;
            for (uint64_t i = i0; i < i1; i++) {
                int32_t v = 0;
                if (!nzo_quantize_one(local[i], eb, step, inv, &v)) all_ok = 0;
                qb[i] = v; rb[i] = f32_bits(local[i]);
            }
            fb[k] = all_ok ? 0 : 1;
        }
        memset(out, 0, (size_t)need);
        const uint32_t step_bits = f32_bits(step);
        reduce_ctx c = { qa, qb, ra, rb, fa, fb, step };
        uint64_t wire = base, end = base;
        for (uint32_t k = 0; k < nfr; k++) {
            const uint64_t i0 = (uint64_t)k * o.chunk_elems;
            const uint32_t nf = (uint32_t)((n - i0 < o.chunk_elems) ? (n - i0) : o.chunk_elems);
            const uint64_t off = base + (uint64_t)k * slot;
            nzo_rea_plan P;
            uint64_t total = 0; int fell = 0;
            const int coded = reduce_src(&c, k, i0, nf, q, rw);          /* integer sums, or the fp32 sums of a frame without them */
            if (coded) {
                for (uint32_t i = 0; i < nf; i++)                        /* what the frame holds should it end up RAW */
                    rw[i] = canon_sum_bits(nzo_dequantize_one(qa[i0 + i], step), nzo_dequantize_one(qb[i0 + i], step));
                rea_plan_codes(q, nf, &o, &ro, ctx, &P);
            } else {
                memset(&P, 0, sizeof P);
                P.plan = NZO_RAW;
            }
            int cdc = rea_commit_codes(out + off, q, rw, 1, nf, &o, ctx, &P, step_bits, FP, &total, &fell);
            put_u64(out + NZO_STREAM_HDR + 8ull * k, off);
            if (plans) plans[k] = (uint8_t)P.plan;
            wire += total; end = off + total;
            res->n_fallback += (uint32_t)fell;
            if (cdc == NZO_RAW) res->n_raw++; else if (cdc == NZO_FIXEDLEN) res->n_fixed++; else res->n_huff++;
        }
        write_stream_header(out, n, &o, nfr, step_bits, end);
        res->span_bytes = end; res->wire_bytes = wire; res->status = NZO_OK;
    } else {
        res->status = (uint32_t)rc;
    }
    free(qa); free(qb); free(ra); free(rb); free(fa); free(fb); free(q); free(rw); free(FP);
    return rc;
}

/* ------------------------------------------------------------------ */
/* 11. stochastic interface quantizer (QSGD, Sec. II-B "Quantization",  */
/*     Sec. IV-B): randomized rounding to a neighbouring level with      */
/*     probability proportional to the distance, unbiased                */
/* ------------------------------------------------------------------ */

/*
 * The random draw of element i under a 32-bit seed: a counter-based generator, so that every implementation
 * draws the same bits whatever order it visits the elements in.  Format v1: the 32-bit finalizer of the
 * public-domain MurmurHash3 (two multiply / xor-shift rounds), keyed with the seed and the high half of the
 * index; the top 24 bits are the draw.
 */
static uint32_t fmix32(uint32_t h) {
    h ^= h >> 16; h *= 0x85EBCA6Bu;
    h ^= h >> 13; h *= 0xC2B2AE35u;
    h ^= h >> 16;
    return h;
}
uint32_t nzo_sr_draw(uint32_t seed, uint64_t i) {
    uint32_t key = fmix32(seed + 0x9E3779B9u * (uint32_t)(i >> 32));
    return fmix32((uint32_t)i ^ key) >> 8;
}

/*
 * Quantize one value with bin width step (inv_step = fl32(1/step)) and a 24-bit draw: a = fl32(|x|*inv_step),
 * unquantizable unless a <= 32767 (catches NaN); l = floor(a), f = a - l (exact in fp32); the level is l + 1
 * with probability f -- draw * 2^-24 < f -- else l (QSGD: probability proportional to the distance from the
 * lower level, so E[q] = a); q takes the sign of x.  Belt and braces as for the deterministic quantizer:
 * unquantizable unless fl32(|x - fl32(q*step)|) <= fl32(step * (1 + 2^-6)).
 */
int nzo_sr_quantize_one(float x, float step, float inv_step, uint32_t draw24, int32_t* q) {
    volatile float a = fabsf(x) * inv_step;
    if (!(a <= 32767.0f)) return 0;
    float l = floorf(a);
    volatile float f = a - l;
    volatile float u = (float)draw24 * 0x1p-24f;
    int32_t qi = (int32_t)l + (u < f ? 1 : 0);
    if (x < 0.0f) qi = -qi;
    volatile float xh = (float)qi * step;
    volatile float d = x - xh;
    volatile float lim = step * 1.015625f;
    if (!(fabsf(d) <= lim)) return 0;
    *q = qi;
    return 1;
}

/* Bin width of QSGD with `levels` levels per sign: step = ||x||_2 / levels (sum of squares in float64, in index
 * order), at least 2^-100 (an all-zero message quantizes to zeros under any width). */
int nzo_qsgd_step(const float* x, size_t n, uint32_t levels, float* step) {
    if (!x || n == 0 || levels == 0 || levels > (uint32_t)NZO_QMAX) return NZO_ERR_INVALID;
    double ssq = 0.0;
    for (size_t i = 0; i < n; i++) ssq += (double)x[i] * (double)x[i];
    double st = sqrt(ssq) / (double)levels;
    if (!(st <= 0x1p100)) return NZO_ERR_INVALID;                /* non-finite input */
    if (st < 0x1p-100) st = 0x1p-100;
    *step = (float)st;
    return NZO_OK;
}

int nzo_sr_quantize(const float* x, size_t n, float step, uint32_t seed, uint64_t first_index, int32_t* q, uint8_t* ok) {
    if (!step_ok(step)) return NZO_ERR_INVALID;
    volatile float inv = 1.0f / step;
    for (size_t i = 0; i < n; i++) {
        int32_t v = 0;
        ok[i] = (uint8_t)nzo_sr_quantize_one(x[i], step, inv, nzo_sr_draw(seed, first_index + i), &v);
        q[i] = ok[i] ? v : 0;
    }
    return NZO_OK;
}

typedef struct { const float* x; float step, inv; uint32_t seed; } sr_ctx;

static int sr_src(void* vctx, uint32_t k, uint64_t i0, uint32_t nf, int32_t* q, uint32_t* rb) {
    (void)k;
    sr_ctx* c = (sr_ctx*)vctx;
    int all_ok = 1;
    for (uint32_t i = 0; i < nf; i++) {
        float x = c->x[i0 + i];
        rb[i] = f32_bits(x);
        int32_t v = 0;
        if (!nzo_sr_quantize_one(x, c->step, c->inv, nzo_sr_draw(c->seed, i0 + i), &v)) all_ok = 0;
        q[i] = v;
    }
    return all_ok;
}

/* Compress with the stochastic quantizer in the place of the deterministic one: same statistics, selector and
 * frames; the stream records step, and element i of the message uses draw (seed, i). */
int nzo_compress_sr(const float* x, size_t n, float step, uint32_t seed, const nzo_opts* opts, uint8_t* out, size_t cap,
                    nzo_result* res) {
    nzo_opts o; sr_ctx c;
    nzo_result dummy;
    if (!res) res = &dummy;
    memset(res, 0, sizeof *res);
    if (n == 0 || !x || !out || !step_ok(step) || resolve_opts(opts, &o) || o.predictor) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    volatile float inv = 1.0f / step;
    c.x = x; c.step = step; c.inv = inv; c.seed = seed;
    return emit_stream(sr_src, &c, n, &o, f32_bits(step), out, cap, res);
}

/*
 * Ring-step reduce with the stochastic interface quantizer (the receive-reduce-send step of Sec. IV-D for a QSGD
 * collective): out = incoming (+) local, where the local message is quantized as nzo_compress_sr would quantize it
 * (element i draws (seed, i)) and never entropy coded.  Frame rules as in nzo_reduce_local: both coded -> exact
 * integer sum, re-planned and re-selected; incoming frame RAW, or a local element that cannot be quantized -> RAW
 * frame of fp32 sums; |Q| > 2^30 -> RAW frame of the dequantized sums.  The stream must have been made with `step`.
 */
int nzo_reduce_local_sr(const uint8_t* in, size_t in_bytes, const float* local, uint8_t* out, size_t cap, size_t n,
                        float step, uint32_t seed, const nzo_opts* opts, nzo_result* res) {
    nzo_opts o; stream_hdr hi;
    nzo_result dummy;
    if (!res) res = &dummy;
    memset(res, 0, sizeof *res);
    if (n == 0 || !in || !local || !out) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    if (resolve_opts(opts, &o) || !step_ok(step) || o.predictor) { res->status = NZO_ERR_INVALID; return NZO_ERR_INVALID; }
    int rc = parse_stream(in, in_bytes, &hi);
    if (rc) { res->status = (uint32_t)rc; return rc; }
    if (hi.n != n || hi.chunk != o.chunk_elems || hi.step_bits != f32_bits(step) || hi.predictor != 0u) {
        res->status = NZO_ERR_MISMATCH; return NZO_ERR_MISMATCH;
    }
    volatile float inv = 1.0f / step;
    int32_t* qa = (int32_t*)malloc(4ull * n); int32_t* qb = (int32_t*)malloc(4ull * n);
    uint32_t* ra = (uint32_t*)malloc(4ull * n); uint32_t* rb = (uint32_t*)malloc(4ull * n);
    uint8_t* fa = (uint8_t*)calloc(hi.n_frames, 1); uint8_t* fb = (uint8_t*)calloc(hi.n_frames, 1);
    if (!qa || !qb || !ra || !rb || !fa || !fb) rc = NZO_ERR_INVALID;
    if (!rc) rc = nzo_decode_codes_step(in, in_bytes, n, step, qa, ra, fa, NULL);
    if (!rc) {
        for (uint32_t k = 0; k < hi.n_frames; k++) {
            const uint64_t i0 = (uint64_t)k * o.chunk_elems;
            const uint64_t i1 = (i0 + o.chunk_elems < n) ? i0 + o.chunk_elems : n;
            int all_ok = 1;
            for (uint64_t i = i0; i < i1; i++) {
                int32_t v = 0;
                if (!nzo_sr_quantize_one(local[i], step, inv, nzo_sr_draw(seed, i), &v)) all_ok = 0;
                qb[i] = v; rb[i] = f32_bits(local[i]);
            }
            fb[k] = all_ok ? 0 : 1;
        }
        reduce_ctx c = { qa, qb, ra, rb, fa, fb, step };
        rc = emit_stream(reduce_src, &c, n, &o, f32_bits(step), out, cap, res);
    } else {
        res->status = (uint32_t)rc;
    }
    free(qa); free(qb); free(ra); free(rb); free(fa); free(fb);
    return rc;
}
