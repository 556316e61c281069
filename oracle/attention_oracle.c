/*
 * TEST INFRASTRUCTURE, not product code: a plain, slow, fp64 CPU statement of
 * what prefix-tree decode attention must return.  Only tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it; the library never does.
 *
 * What it computes (paper Sec. 2.2, Eq. 1-2; prefix path and logical
 * concatenation of node KV, Sec. 4.1 "Formal model and notation"): for every
 * request r and query head hq, the request's context is the concatenation,
 * root to leaf, of the K and V rows of the nodes on its prefix path; the
 * output is softmax(scale * q . K^T) V over that whole context, with the
 * maximum subtracted before exponentiation (Eq. 2).  No tree sharing, no
 * chunking, no partial merging: each (request, head) is evaluated from the
 * definition on its own, in double precision, on the exact values the 16-bit
 * inputs hold.
 *
 * Visibility (Sec. 4.1, "Streaming softmax across nodes": a position (n, j)
 * that is not visible to r gets the score -inf and contributes 0).  Here a
 * request may carry a visibility mask over the tokens of the LAST node of its
 * path (the drafted tokens of a multi-token decoding step, of which a query
 * sees its ancestors and itself); every token of the other nodes on the path is
 * visible.  An invisible token is left out of the request's context: that is
 * what a score of -inf amounts to in Eq. 2.
 *
 * Readings the paper leaves open: query head hq uses KV head hq / (h_q / h_kv)
 * (consecutive query heads share a KV head); without a mask every token of the
 * path is visible to the decode query; each node owns whole pages and fills
 * them in order, so logical token t of a node lives in the node's page
 * t / page_size at slot t % page_size.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double fp16_bits_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int expo = (h >> 10) & 0x1f;
    int frac = h & 0x3ff;
    double v;
    if (expo == 0)
        v = ldexp((double)frac, -24);                 /* subnormal: frac * 2^-10 * 2^-14 */
    else if (expo == 31)
        v = frac ? NAN : INFINITY;
    else
        v = ldexp(1.0 + (double)frac / 1024.0, expo - 15);
    return sign ? -v : v;
}

static double bf16_bits_to_double(uint16_t b)
{
    uint32_t u = ((uint32_t)b) << 16;                 /* bf16 is the top half of an fp32 */
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

static inline double load16(const uint16_t *p, int dtype)
{
    return dtype == 0 ? fp16_bits_to_double(*p) : bf16_bits_to_double(*p);
}

/* exported so that tests can pin the 16-bit decoding on its own */
double codec_oracle_decode16(uint16_t bits, int32_t dtype)
{
    return load16(&bits, dtype);
}

/*
 * Returns 0 on success, -1 on a malformed forest (bad parent index or a cycle),
 * -2 on allocation failure.
 *
 * sel_req / sel_head: n_sel (request, query head) pairs to evaluate, or NULL
 * to evaluate all B*h_q pairs in (request-major, head-minor) order.
 * out: [n][d] doubles, lse: [n] doubles (natural-log sum-exp of the scaled
 * scores), n = n_sel or B*h_q.  Strides are in elements.
 *
 * req_mask_off / req_mask: NULL, or per request r the 32-bit words
 * req_mask[req_mask_off[r] .. req_mask_off[r+1]): none = everything visible,
 * else bit (t % 32) of word t / 32 says whether token t of node req_node[r]
 * is visible to r (there must be a word for every 32 tokens of that node).
 * Returns -3 if a request with a mask sees no token at all.
 */
int codec_oracle_decode_attention(
    int32_t num_nodes, const int32_t *parent, const int32_t *node_len,
    int32_t num_requests, const int32_t *req_node,
    const int32_t *node_page_off, const int32_t *page_ids, int32_t page_size,
    int32_t h_q, int32_t h_kv, int32_t d, int32_t dtype, double scale,
    const uint16_t *q,
    const uint16_t *k_pool, const uint16_t *v_pool,
    int64_t page_stride, int64_t token_stride, int64_t head_stride,
    int64_t n_sel, const int32_t *sel_req, const int32_t *sel_head,
    const int32_t *req_mask_off, const uint32_t *req_mask,
    double *out, double *lse, int32_t nthreads)
{
    const int64_t total = sel_req ? n_sel : (int64_t)num_requests * h_q;
    const int group = h_q / h_kv;
    int status = 0;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t idx = 0; idx < total; ++idx) {
        const int r = sel_req ? sel_req[idx] : (int)(idx / h_q);
        const int hq = sel_req ? sel_head[idx] : (int)(idx % h_q);
        const int kvh = hq / group;

        /* prefix path of r, leaf to root, then walked backwards */
        int *path = (int *)malloc(sizeof(int) * (size_t)(num_nodes > 0 ? num_nodes : 1));
        if (!path) {
#pragma omp atomic write
            status = -2;
            continue;
        }
        int depth = 0, bad = 0;
        int64_t ctx = 0;
        for (int n = req_node[r]; n != -1; n = parent[n]) {
            if (n < 0 || n >= num_nodes || depth >= num_nodes) { bad = 1; break; }
            path[depth++] = n;
            ctx += node_len[n];
        }
        if (bad) {
#pragma omp atomic write
            status = -1;
            free(path);
            continue;
        }

        double *score = (double *)malloc(sizeof(double) * (size_t)(ctx > 0 ? ctx : 1));
        double *qv = (double *)malloc(sizeof(double) * (size_t)d);
        if (!score || !qv) {
#pragma omp atomic write
            status = -2;
            free(path); free(score); free(qv);
            continue;
        }
        for (int c = 0; c < d; ++c)
            qv[c] = load16(q + ((int64_t)r * h_q + hq) * d + c, dtype);

        /* the request's mask over its last node, if it has one */
        const uint32_t *mask = NULL;
        if (req_mask_off && req_mask_off[r + 1] > req_mask_off[r]) mask = req_mask + req_mask_off[r];

        /* scores over the concatenated visible context, root first */
        int64_t pos = 0;
        double mx = -INFINITY;
        for (int lvl = depth - 1; lvl >= 0; --lvl) {
            const int n = path[lvl];
            for (int t = 0; t < node_len[n]; ++t) {
                if (lvl == 0 && mask && !((mask[t / 32] >> (t % 32)) & 1u)) continue;
                const int64_t page = page_ids[node_page_off[n] + t / page_size];
                const uint16_t *krow = k_pool + page * page_stride
                                       + (int64_t)(t % page_size) * token_stride
                                       + (int64_t)kvh * head_stride;
                double dot = 0.0;
                for (int c = 0; c < d; ++c)
                    dot += qv[c] * load16(krow + c, dtype);
                const double s = scale * dot;
                score[pos++] = s;
                if (s > mx) mx = s;
            }
        }
        const int64_t seen = pos;
        if (seen == 0) {
#pragma omp atomic write
            status = -3;
            free(path); free(score); free(qv);
            continue;
        }
        /* softmax with the maximum subtracted (Eq. 2) */
        double sum = 0.0;
        for (int64_t i = 0; i < seen; ++i) {
            score[i] = exp(score[i] - mx);
            sum += score[i];
        }
        double *o = out + idx * d;
        for (int c = 0; c < d; ++c) o[c] = 0.0;
        pos = 0;
        for (int lvl = depth - 1; lvl >= 0; --lvl) {
            const int n = path[lvl];
            for (int t = 0; t < node_len[n]; ++t) {
                if (lvl == 0 && mask && !((mask[t / 32] >> (t % 32)) & 1u)) continue;
                const int64_t page = page_ids[node_page_off[n] + t / page_size];
                const uint16_t *vrow = v_pool + page * page_stride
                                       + (int64_t)(t % page_size) * token_stride
                                       + (int64_t)kvh * head_stride;
                const double p = score[pos++] / sum;
                for (int c = 0; c < d; ++c)
                    o[c] += p * load16(vrow + c, dtype);
            }
        }
        if (lse) lse[idx] = mx + log(sum);
        free(path); free(score); free(qv);
    }
    return status;
}

int32_t codec_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
