/* Driver for the scalar C twin of the oracle, built with -fsanitize=address,undefined by
 * tests/test_host_sanitizers.py.  argv[1]: input file (a header of 12 int64, then the arrays, every one in a
 * heap block of exactly its size so that an access past its end is caught); argv[2]: output file of doubles. */
#include <stdio.h>
#include <stdlib.h>

#include "../oracle/brute_attn.c"

static void *read_block(FILE *f, size_t bytes)
{
    void *p = malloc(bytes ? bytes : 1);
    if (!p || (bytes && fread(p, 1, bytes, f) != bytes)) exit(3);
    return p;
}

int main(int argc, char **argv)
{
    if (argc != 3) return 2;
    FILE *f = fopen(argv[1], "rb");
    if (!f) return 2;
    int64_t h[12];
    if (fread(h, sizeof(int64_t), 12, f) != 12) return 3;
    /* rows, batch, hq, hkv, d, page_size, max_pages, num_pages, q_dtype, kv_dtype, has_qlens, has_scales */
    const int64_t rows = h[0], batch = h[1], hq = h[2], hkv = h[3], d = h[4], ps = h[5], max_pages = h[6], num_pages = h[7];
    const int qd = (int)h[8], kvd = (int)h[9];
    const size_t qb = qd == 0 ? 4 : 2, kvb = kvd == 0 ? 4 : (kvd == 1 ? 2 : 1);
    float scale;
    if (fread(&scale, 4, 1, f) != 1) return 3;
    void *q = read_block(f, (size_t)(rows * hq * d) * qb);
    int32_t *q_lens = h[10] ? read_block(f, (size_t)batch * 4) : NULL;
    void *kp = read_block(f, (size_t)(num_pages * hkv * ps * d) * kvb);
    void *vp = read_block(f, (size_t)(num_pages * hkv * ps * d) * kvb);
    float *ks = h[11] ? read_block(f, (size_t)num_pages * 4) : NULL;
    float *vs = h[11] ? read_block(f, (size_t)num_pages * 4) : NULL;
    int32_t *table = read_block(f, (size_t)(batch * max_pages) * 4);
    int32_t *ctx = read_block(f, (size_t)batch * 4);
    fclose(f);
    double *out = malloc((size_t)(rows * hq * d) * sizeof(double) + 1);
    const int rc = brute_paged_attention(q, qd, q_lens, kp, vp, kvd, ks, vs, table, ctx, (int)batch, (int)hq, (int)hkv, (int)d,
                                         (int)ps, max_pages, num_pages, scale, out);
    if (rc) return 4;
    f = fopen(argv[2], "wb");
    if (!f || fwrite(out, sizeof(double), (size_t)(rows * hq * d), f) != (size_t)(rows * hq * d)) return 5;
    fclose(f);
    free(q); free(q_lens); free(kp); free(vp); free(ks); free(vs); free(table); free(ctx); free(out);
    return 0;
}
