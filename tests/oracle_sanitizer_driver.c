/*
 * Runs the float64 oracle (oracle/hta_oracle.c, compiled into this program with AddressSanitizer and
 * UndefinedBehaviorSanitizer) on one case read from a file and writes its results to another file.
 * TEST INFRASTRUCTURE: tests/test_oracle_sanitizers.py builds and runs it and compares the results with those of the
 * ordinary oracle library; any out-of-bounds access, use of uninitialised heap, leak or undefined behaviour inside the
 * oracle ends the program with a report on stderr and a non-zero exit status.
 *
 * Input file (native endianness):
 *   int32  layer, batch, Hq, Hkv, d, has_rt;  int64 total_q, total_kv;  float64 scale, norm
 *   int32  q_start[batch+1], kv_start[batch+1], hist_len[batch], n_targets[batch]
 *   int32  rt_len[batch], timestamps[total_kv]                         (only if has_rt)
 *   float64 q[total_q*Hq*d], k[total_kv*Hkv*d], v[total_kv*Hkv*d], dout[total_q*Hq*d]
 * Output file: float64 out, lse, dq, dk, dv (softmax reading), then out, dq, dk, dv (pointwise reading), then the
 * probabilities of (user 0, head Hq-1) as [rows][N].
 */
#include "../oracle/hta_oracle.c"

#include <stdio.h>

static void* xmalloc(size_t n) {
    void* p = malloc(n ? n : 1);
    if (!p) { fprintf(stderr, "out of memory\n"); exit(3); }
    return p;
}
static void rd(FILE* f, void* dst, size_t bytes) {
    if (bytes && fread(dst, 1, bytes, f) != bytes) { fprintf(stderr, "short read\n"); exit(3); }
}
static void wr(FILE* f, const void* src, size_t bytes) {
    if (bytes && fwrite(src, 1, bytes, f) != bytes) { fprintf(stderr, "short write\n"); exit(3); }
}

int main(int argc, char** argv) {
    if (argc != 3) { fprintf(stderr, "usage: %s case.bin results.bin\n", argv[0]); return 2; }
    FILE* f = fopen(argv[1], "rb");
    if (!f) { perror(argv[1]); return 2; }
    int32_t hdr[6];
    int64_t tot[2];
    double sc[2];
    rd(f, hdr, sizeof hdr); rd(f, tot, sizeof tot); rd(f, sc, sizeof sc);
    const int32_t layer = hdr[0], B = hdr[1], Hq = hdr[2], Hkv = hdr[3], d = hdr[4], has_rt = hdr[5];
    const int64_t tq = tot[0], tkv = tot[1];
    /* every array is allocated at its exact size, so that an access past its end lands in a red zone */
    int32_t* q_start = xmalloc((size_t)(B + 1) * 4); int32_t* kv_start = xmalloc((size_t)(B + 1) * 4);
    int32_t* hist = xmalloc((size_t)B * 4); int32_t* tgts = xmalloc((size_t)B * 4);
    int32_t *rt = NULL, *ts = NULL;
    rd(f, q_start, (size_t)(B + 1) * 4); rd(f, kv_start, (size_t)(B + 1) * 4); rd(f, hist, (size_t)B * 4); rd(f, tgts, (size_t)B * 4);
    if (has_rt) {
        rt = xmalloc((size_t)B * 4); ts = xmalloc((size_t)tkv * 4);
        rd(f, rt, (size_t)B * 4); rd(f, ts, (size_t)tkv * 4);
    }
    const size_t nq = (size_t)tq * Hq * d, nkv = (size_t)tkv * Hkv * d, nl = (size_t)tq * Hq;
    double *q = xmalloc(nq * 8), *k = xmalloc(nkv * 8), *v = xmalloc(nkv * 8), *dout = xmalloc(nq * 8);
    rd(f, q, nq * 8); rd(f, k, nkv * 8); rd(f, v, nkv * 8); rd(f, dout, nq * 8);
    fclose(f);
    double *out = xmalloc(nq * 8), *lse = xmalloc(nl * 8), *dq = xmalloc(nq * 8), *dk = xmalloc(nkv * 8), *dv = xmalloc(nkv * 8);
    FILE* g = fopen(argv[2], "wb");
    if (!g) { perror(argv[2]); return 2; }
    if (hta_oracle_fwd_rt(q, k, v, out, lse, q_start, kv_start, hist, rt, tgts, ts, B, tq, Hq, Hkv, d, sc[0], layer)) return 4;
    if (hta_oracle_bwd_rt(dout, q, k, v, out, lse, dq, dk, dv, q_start, kv_start, hist, rt, tgts, ts, B, tq, Hq, Hkv, d, sc[0], layer)) return 4;
    wr(g, out, nq * 8); wr(g, lse, nl * 8); wr(g, dq, nq * 8); wr(g, dk, nkv * 8); wr(g, dv, nkv * 8);
    if (hta_oracle_pw_fwd_rt(q, k, v, out, q_start, kv_start, hist, rt, tgts, ts, B, Hq, Hkv, d, sc[0], sc[1], layer)) return 4;
    if (hta_oracle_pw_bwd_rt(dout, q, k, v, dq, dk, dv, q_start, kv_start, hist, rt, tgts, ts, B, Hq, Hkv, d, sc[0], sc[1], layer)) return 4;
    wr(g, out, nq * 8); wr(g, dq, nq * 8); wr(g, dk, nkv * 8); wr(g, dv, nkv * 8);
    if (B > 0) {
        const int64_t R = rt ? rt[0] : 0, N = (int64_t)hist[0] + R + tgts[0], rows = layer == 0 ? N : tgts[0];
        double* pr = xmalloc((size_t)(rows * N) * 8);
        if (hta_oracle_probs_rt(q, k, pr, q_start[0], kv_start[0], hist[0], (int32_t)R, tgts[0], ts, Hq - 1, Hq, Hkv, d, sc[0], layer)) return 4;
        wr(g, pr, (size_t)(rows * N) * 8);
        free(pr);
    }
    fclose(g);
    free(q_start); free(kv_start); free(hist); free(tgts); free(rt); free(ts);
    free(q); free(k); free(v); free(dout); free(out); free(lse); free(dq); free(dk); free(dv);
    return 0;
}
