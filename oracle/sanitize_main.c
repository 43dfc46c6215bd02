/*
 * sanitize_main.c -- driver that runs the CPU oracle under AddressSanitizer / UndefinedBehaviorSanitizer.
 * TEST INFRASTRUCTURE (built and run by tests/test_oracle_sanitize.py only).  It includes the oracle's source
 * directly, so every function is instrumented, and pushes valid, ragged, unquantizable and corrupted inputs
 * through compress / decompress / reduce / ring-step reduce.  Exit status 0 = no finding (a sanitizer report
 * aborts with a non-zero status).
 */
#include "nz_oracle.c"
#include <stdio.h>

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint32_t rnd(void) { rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(rng_state >> 33); }
static float laplace_like(float b) {
    float u = ((float)(rnd() % 2000001u) - 1000000.0f) / 1000001.0f;       /* (-1, 1) */
    float a = u < 0 ? -u : u;
    float v = -b * logf(1.0f - a);
    return u < 0 ? -v : v;
}

static int run_case(size_t n, uint32_t chunk, uint32_t K, uint32_t seg, int force, float eb, int poison) {
    nzo_opts o = { chunk, seg, K, force, 0, 0, 0, 0 };
    float* x = (float*)malloc(4 * n); float* y = (float*)malloc(4 * n); float* z = (float*)malloc(4 * n);
    for (size_t i = 0; i < n; i++) { x[i] = laplace_like(1e-3f); y[i] = laplace_like(3e-2f); }
    if (poison && n > 3) { x[n / 2] = NAN; y[n - 1] = INFINITY; x[1] = 1e30f; }
    size_t cap = nzo_compress_bound(n, &o);
    if (!cap) return 1;
    uint8_t* sa = (uint8_t*)malloc(cap); uint8_t* sb = (uint8_t*)malloc(cap); uint8_t* sc = (uint8_t*)malloc(cap);
    nzo_result ra, rb, rc;
    if (nzo_compress(x, n, eb, &o, sa, cap, &ra) || nzo_compress(y, n, eb, &o, sb, cap, &rb)) return 2;
    if (nzo_decompress(sa, ra.bytes, z, n, eb, &rc)) return 3;
    for (size_t i = 0; i < n; i++) if (isfinite(x[i]) && fabs((double)x[i] - (double)z[i]) > (double)eb) return 4;
    nzo_opts od = o; od.force_codec = -1;
    if (nzo_reduce_frames(sa, ra.bytes, sb, rb.bytes, sc, cap, n, eb, &od, &rc)) return 5;
    if (nzo_reduce_local(sa, ra.bytes, y, sc, cap, n, eb, &od, &rc)) return 6;
    {
        const uint8_t* ops[3] = { sa, sb, sa }; const size_t lens[3] = { ra.bytes, rb.bytes, ra.bytes };
        if (nzo_reduce_k(ops, lens, 3, sc, cap, n, eb, &od, &rc)) return 7;
    }
    /* sampled arbitration with a cached context: valid, pinned, without context, capacity one slot short */
    {
        nzo_context ctx; nzo_rea_result rr; nzo_rea_opts ro = { 4096u, 0u, 0u, 0u, 0u, 0u, 0u, 0u };
        size_t cal = n < 5000 ? n : 5000;
        if (nzo_context_build(y, cal, eb, &od, &ctx)) return 8;
        size_t rcap = nzo_compress_bound(n, &od);
        uint8_t* sr = (uint8_t*)malloc(rcap);
        if (nzo_compress_rea(x, n, eb, &od, NULL, &ctx, sr, rcap, &rr, NULL)) return 9;
        if (nzo_decompress(sr, rr.span_bytes, z, n, eb, &rc)) return 10;
        for (size_t i = 0; i < n; i++) if (isfinite(x[i]) && fabs((double)x[i] - (double)z[i]) > (double)eb) return 11;
        if (nzo_compress_rea(y, n, eb, &o, &ro, &ctx, sr, rcap, &rr, NULL)) return 12;
        if (nzo_decompress(sr, rr.span_bytes, z, n, eb, &rc)) return 13;
        if (nzo_compress_rea(y, n, eb, &od, &ro, NULL, sr, rcap, &rr, NULL)) return 14;
        if (rcap > 16 && nzo_compress_rea(y, n, eb, &od, &ro, &ctx, sr, rcap - 16, &rr, NULL) != NZO_ERR_CAPACITY) return 15;
        /* the ring step with the sampled arbitration on the way out */
        if (nzo_reduce_local_rea(sa, ra.bytes, y, n, eb, &od, &ro, &ctx, sr, rcap, &rr, NULL)) return 16;
        if (nzo_decompress(sr, rr.span_bytes, z, n, eb, &rc)) return 17;
        if (nzo_reduce_local_rea(sa, ra.bytes, y, n, eb, &od, NULL, NULL, sr, rcap, &rr, NULL)) return 18;
        free(sr);
    }
    /* delta predictor: compress, decode, reduce */
    {
        nzo_opts op = od; op.predictor = 1u;
        nzo_result r1, r2;
        size_t pcap = nzo_compress_bound(n, &op);
        uint8_t* s1 = (uint8_t*)malloc(pcap); uint8_t* s2 = (uint8_t*)malloc(pcap); uint8_t* s3 = (uint8_t*)malloc(pcap);
        if (nzo_compress(x, n, eb, &op, s1, pcap, &r1) || nzo_compress(y, n, eb, &op, s2, pcap, &r2)) return 20;
        if (nzo_decompress(s1, r1.bytes, z, n, eb, &rc)) return 21;
        for (size_t i = 0; i < n; i++) if (isfinite(x[i]) && fabs((double)x[i] - (double)z[i]) > (double)eb) return 22;
        if (nzo_reduce_frames(s1, r1.bytes, s2, r2.bytes, s3, pcap, n, eb, &op, &rc)) return 23;
        if (nzo_reduce_local(s1, r1.bytes, y, s3, pcap, n, eb, &op, &rc)) return 24;
        for (int t = 0; t < 20; t++) { s1[rnd() % r1.bytes] ^= (uint8_t)(1u + rnd() % 255u); (void)nzo_decompress(s1, r1.bytes, z, n, eb, &rc); }
        free(s1); free(s2); free(s3);
    }
    /* stochastic quantizer: compress, decode with the recorded width, reduce */
    {
        float st; nzo_result r1, r2;
        if (nzo_qsgd_step(y, n, 64, &st) && !poison) return 16;
        if (poison) st = 1e-3f;
        size_t scap = nzo_compress_bound(n, &od);
        uint8_t* s1 = (uint8_t*)malloc(scap); uint8_t* s2 = (uint8_t*)malloc(scap); uint8_t* s3 = (uint8_t*)malloc(scap);
        if (nzo_compress_sr(y, n, st, 7u, &od, s1, scap, &r1) || nzo_compress_sr(x, n, st, 8u, &od, s2, scap, &r2)) return 17;
        if (nzo_decompress_step(s1, r1.bytes, z, n, st, &rc)) return 18;
        if (nzo_reduce_frames_step(s1, r1.bytes, s2, r2.bytes, s3, scap, n, st, &od, &rc)) return 19;
        if (nzo_reduce_local_sr(s1, r1.bytes, x, s3, scap, n, st, 8u, &od, &rc)) return 24;
        free(s1); free(s2); free(s3);
    }
    /* too small an output: capacity error, nothing written past cap */
    uint8_t* small = (uint8_t*)malloc(ra.bytes > 16 ? ra.bytes - 16 : 1);
    if (nzo_compress(x, n, eb, &o, small, ra.bytes > 16 ? ra.bytes - 16 : 1, &rc) != NZO_ERR_CAPACITY) return 7;
    free(small);
    /* corrupted streams: byte flips anywhere, truncation; any verdict is fine, memory errors are not */
    const int flips = n < 20000 ? 150 : (n < 100000 ? 30 : 4);
    for (int t = 0; t < flips; t++) {
        uint8_t* m = (uint8_t*)malloc(ra.bytes);
        memcpy(m, sa, ra.bytes);
        size_t pos = rnd() % ra.bytes;
        m[pos] ^= (uint8_t)(1u + rnd() % 255u);
        size_t len = (t % 10 == 0) ? (size_t)(rnd() % (ra.bytes + 1)) : (size_t)ra.bytes;
        (void)nzo_decompress(m, len, z, n, eb, &rc);
        (void)nzo_reduce_frames(m, len, sb, rb.bytes, sc, cap, n, eb, &od, &rc);
        (void)nzo_reduce_local(m, len, y, sc, cap, n, eb, &od, &rc);
        {
            const uint8_t* ops[3] = { sb, m, sb }; const size_t lens[3] = { rb.bytes, len, rb.bytes };
            (void)nzo_reduce_k(ops, lens, 3, sc, cap, n, eb, &od, &rc);
        }
        free(m);
    }
    free(x); free(y); free(z); free(sa); free(sb); free(sc);
    return 0;
}

int main(void) {
    static const struct { size_t n; uint32_t chunk, K, seg; int force; float eb; int poison; } cases[] = {
        { 1, 0, 0, 0, -1, 1e-4f, 0 },       { 37, 16, 0, 0, -1, 1e-4f, 0 },     { 70001, 20000, 0, 0, -1, 1e-4f, 0 },
        { 30011, 10003, 1024, 0, -1, 1e-5f, 1 }, { 5000, 1000, 2, 32, 2, 1e-3f, 0 }, { 40000, 16384, 16, 1024, 2, 1e-4f, 0 },
        { 50000, 16384, 0, 0, 1, 1e-4f, 0 }, { 50000, 16384, 0, 0, 0, 1e-4f, 1 },  { (1u << 20) + 77, 1u << 20, 64, 100, -1, 3e-4f, 0 },
    };
    for (size_t c = 0; c < sizeof cases / sizeof cases[0]; c++) {
        int rc = run_case(cases[c].n, cases[c].chunk, cases[c].K, cases[c].seg, cases[c].force, cases[c].eb, cases[c].poison);
        if (rc) { printf("case %zu failed at step %d\n", c, rc); return 10 + rc; }
    }
    printf("sanitize ok\n");
    return 0;
}
