/* Brute-force twin of the float64 oracle: scalar loops, one token at a time.
 *
 * TEST INFRASTRUCTURE ONLY.  Independent of the numpy oracle (it decodes storage
 * formats arithmetically, walks the page table itself and exponentiates term by
 * term) and of the HIP library (no shared code).  Used on tiny inputs to pin the
 * numpy oracle: the engine's decode / prefill step over a paged KV cache (Section
 * 6.1, inference worker loop; Section 3.1, the two phases), written as the textbook
 * softmax-attention sum.
 *
 * dtype codes: 0 = float32, 1 = bfloat16 bits, 2 = OCP FP8 E4M3 code (times a
 * float32 scale per physical page).
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static double load_elem(const void *base, int64_t idx, int dtype)
{
    if (dtype == 0) {
        float f;
        memcpy(&f, (const char *)base + 4 * idx, 4);
        return (double)f;
    }
    if (dtype == 1) {
        uint16_t h;
        memcpy(&h, (const char *)base + 2 * idx, 2);
        int sign = h >> 15, e = (h >> 7) & 0xFF, m = h & 0x7F;
        double mag;
        if (e == 0xFF)
            mag = m ? NAN : INFINITY;
        else if (e == 0)
            mag = ldexp((double)m, -126 - 7);
        else
            mag = ldexp((double)(128 + m), e - 127 - 7);
        return sign ? -mag : mag;
    }
    {
        uint8_t c = ((const uint8_t *)base)[idx];
        int sign = c >> 7, e = (c >> 3) & 0xF, m = c & 7;
        double mag;
        if (e == 15 && m == 7)
            mag = NAN;
        else if (e == 0)
            mag = ldexp((double)m, -6 - 3);
        else
            mag = ldexp((double)(8 + m), e - 7 - 3);
        return sign ? -mag : mag;
    }
}

/* One output row: query row `qrow` (index into the packed q array), head h of
 * trajectory b, attending tokens 0..pos.  Returns 0, or -1 if a page id is bad. */
static int one_row(const void *q, int q_dtype, int64_t qrow, int h, int b, int64_t pos,
                   const void *k_pages, const void *v_pages, int kv_dtype,
                   const float *k_scale, const float *v_scale,
                   const int32_t *page_table, int64_t max_pages, int64_t num_pages,
                   int hq, int hkv, int d, int page_size, double sm_scale, double *out)
{
    int g = h / (hq / hkv);
    double zmax = -INFINITY;
    /* pass 1: largest score */
    for (int64_t t = 0; t <= pos; ++t) {
        int64_t p = page_table[(int64_t)b * max_pages + t / page_size];
        if (p < 0 || p >= num_pages)
            return -1;
        int64_t base = ((p * hkv + g) * page_size + t % page_size) * d;
        double ks = (kv_dtype == 2) ? (double)k_scale[p] : 1.0;
        double z = 0.0;
        for (int j = 0; j < d; ++j)
            z += load_elem(q, (qrow * hq + h) * d + j, q_dtype) * (load_elem(k_pages, base + j, kv_dtype) * ks);
        z *= sm_scale;
        if (z > zmax)
            zmax = z;
    }
    /* pass 2: weights and weighted values */
    double denom = 0.0;
    for (int j = 0; j < d; ++j)
        out[j] = 0.0;
    for (int64_t t = 0; t <= pos; ++t) {
        int64_t p = page_table[(int64_t)b * max_pages + t / page_size];
        int64_t base = ((p * hkv + g) * page_size + t % page_size) * d;
        double ks = (kv_dtype == 2) ? (double)k_scale[p] : 1.0;
        double vs = (kv_dtype == 2) ? (double)v_scale[p] : 1.0;
        double z = 0.0;
        for (int j = 0; j < d; ++j)
            z += load_elem(q, (qrow * hq + h) * d + j, q_dtype) * (load_elem(k_pages, base + j, kv_dtype) * ks);
        double w = exp(z * sm_scale - zmax);
        denom += w;
        for (int j = 0; j < d; ++j)
            out[j] += w * (load_elem(v_pages, base + j, kv_dtype) * vs);
    }
    for (int j = 0; j < d; ++j)
        out[j] /= denom;
    return 0;
}

/* q_lens == NULL means decode (one row per trajectory).  out is [total rows, hq, d]
 * float64, zero-filled rows where the context is empty. */
int brute_paged_attention(const void *q, int q_dtype, const int32_t *q_lens,
                          const void *k_pages, const void *v_pages, int kv_dtype,
                          const float *k_scale, const float *v_scale,
                          const int32_t *page_table, const int32_t *ctx_lens,
                          int batch, int hq, int hkv, int d, int page_size,
                          int64_t max_pages, int64_t num_pages, float sm_scale, double *out)
{
    int64_t row = 0;
    for (int b = 0; b < batch; ++b) {
        int64_t n = q_lens ? q_lens[b] : 1;
        int64_t len = ctx_lens[b];
        for (int64_t i = 0; i < n; ++i, ++row) {
            int64_t pos = len - n + i;
            for (int h = 0; h < hq; ++h) {
                double *o = out + (row * hq + h) * d;
                if (pos < 0) {
                    for (int j = 0; j < d; ++j)
                        o[j] = 0.0;
                    continue;
                }
                int rc = one_row(q, q_dtype, row, h, b, pos, k_pages, v_pages, kv_dtype, k_scale,
                                 v_scale, page_table, max_pages, num_pages, hq, hkv, d, page_size,
                                 (double)sm_scale, o);
                if (rc)
                    return rc;
            }
        }
    }
    return 0;
}
