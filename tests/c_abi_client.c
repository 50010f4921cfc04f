/*
 * A caller of librollattn written in plain C: no torch, only the HIP runtime for device memory and the entry
 * points declared in rollattn.h, resolved with dlopen.  The GPU test next to it writes a small batch to files,
 * has this code run on them and compares what it writes back with the oracle, which shows that the boundary
 * really is plain pointers and sizes.  Built as a shared object whose c_abi_client_run() the test calls in its own
 * process, and usable as a program of its own through main().
 *
 * usage: c_abi_client <librollattn.so> <dir> <decode|append> B Hq Hkv D q_dtype kv_dtype max_pages num_pages
 *                     total_q max_q_len sm_scale
 * reads  <dir>/{q,k_pages,v_pages,page_table,ctx_lens,q_lens,q_offsets,k_scale,v_scale}.bin (raw arrays)
 * writes <dir>/out.bin (same element type and shape as q)
 */
#define __HIP_PLATFORM_AMD__ 1
#include <dlfcn.h>
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "rollattn.h"

typedef int (*decode_fn)(const rollattn_desc *, const void *, const void *, const void *, const int32_t *,
                         const int32_t *, void *, void *, size_t, void *);
typedef int (*append_fn)(const rollattn_desc *, const void *, const int32_t *, const int32_t *, int32_t, int32_t,
                         const void *, const void *, const int32_t *, const int32_t *, void *, void *, size_t, void *);
typedef size_t (*ws_fn)(const rollattn_desc *, int32_t);
typedef const char *(*str_fn)(int);

static char g_error[512];
const char *c_abi_client_error(void) { return g_error; }

static int fail(const char *what) {
  snprintf(g_error, sizeof g_error, "c_abi_client: %s", what);
  return 1;
}

#define DIE(what) return fail(what)
#define HIP_OK(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) return fail(hipGetErrorString(e_)); } while (0)

/* Reads a whole file into device memory (*dev stays NULL for a missing or empty file); *bytes gets its size. */
static int to_device(const char *dir, const char *name, void **dev, size_t *bytes) {
  char path[4096];
  snprintf(path, sizeof path, "%s/%s.bin", dir, name);
  FILE *f = fopen(path, "rb");
  *bytes = 0;
  *dev = NULL;
  if (!f) return 0;
  fseek(f, 0, SEEK_END);
  long n = ftell(f);
  fseek(f, 0, SEEK_SET);
  if (n > 0) {
    void *host = malloc((size_t)n);
    if (!host || fread(host, 1, (size_t)n, f) != (size_t)n) DIE("short read");
    HIP_OK(hipMalloc(dev, (size_t)n));
    HIP_OK(hipMemcpy(*dev, host, (size_t)n, hipMemcpyHostToDevice));
    free(host);
    *bytes = (size_t)n;
  }
  fclose(f);
  return 0;
}

int c_abi_client_run(int argc, char **argv) {
  if (argc != 15) DIE("expected 14 arguments");
  const char *dir = argv[2];
  const int append = strcmp(argv[3], "append") == 0;
  rollattn_desc d;
  memset(&d, 0, sizeof d);
  d.batch = atoi(argv[4]);
  d.num_q_heads = atoi(argv[5]);
  d.num_kv_heads = atoi(argv[6]);
  d.head_dim = atoi(argv[7]);
  d.page_size = 16;
  d.q_dtype = atoi(argv[8]);
  d.kv_dtype = atoi(argv[9]);
  d.max_pages_per_seq = atoi(argv[10]);
  d.num_pages = atoll(argv[11]);
  const int32_t total_q = atoi(argv[12]), max_q_len = atoi(argv[13]);
  d.sm_scale = (float)atof(argv[14]);

  void *lib = dlopen(argv[1], RTLD_NOW);
  if (!lib) DIE(dlerror());
  decode_fn attn_decode_p = (decode_fn)dlsym(lib, "attn_decode");
  append_fn attn_append_p = (append_fn)dlsym(lib, "attn_append");
  ws_fn ws_bytes_p = (ws_fn)dlsym(lib, "rollattn_workspace_bytes");
  str_fn status_p = (str_fn)dlsym(lib, "rollattn_status_string");
  if (!attn_decode_p || !attn_append_p || !ws_bytes_p || !status_p) DIE("a declared symbol is missing");

  size_t nb, q_bytes;
  void *q, *k_pages, *v_pages, *page_table, *ctx_lens, *q_lens, *q_offsets, *k_scale, *v_scale;
  if (to_device(dir, "q", &q, &q_bytes) || to_device(dir, "k_pages", &k_pages, &nb) ||
      to_device(dir, "v_pages", &v_pages, &nb) || to_device(dir, "page_table", &page_table, &nb) ||
      to_device(dir, "ctx_lens", &ctx_lens, &nb) || to_device(dir, "q_lens", &q_lens, &nb) ||
      to_device(dir, "q_offsets", &q_offsets, &nb) || to_device(dir, "k_scale", &k_scale, &nb) ||
      to_device(dir, "v_scale", &v_scale, &nb))
    return 1;
  d.k_scale = (const float *)k_scale;
  d.v_scale = (const float *)v_scale;

  const size_t ws_bytes = ws_bytes_p(&d, total_q);
  if (!ws_bytes) DIE("rollattn_workspace_bytes rejected the descriptor");
  void *workspace = NULL, *out = NULL;
  HIP_OK(hipMalloc(&workspace, ws_bytes));
  HIP_OK(hipMalloc(&out, q_bytes));
  hipStream_t stream;
  HIP_OK(hipStreamCreate(&stream));

  const int rc = append
      ? attn_append_p(&d, q, (const int32_t *)q_lens, (const int32_t *)q_offsets, total_q, max_q_len, k_pages, v_pages,
                      (const int32_t *)page_table, (const int32_t *)ctx_lens, out, workspace, ws_bytes, stream)
      : attn_decode_p(&d, q, k_pages, v_pages, (const int32_t *)page_table, (const int32_t *)ctx_lens, out, workspace,
                      ws_bytes, stream);
  if (rc) DIE(status_p(rc));
  HIP_OK(hipStreamSynchronize(stream));

  void *host = malloc(q_bytes);
  if (!host) DIE("out of memory");
  HIP_OK(hipMemcpy(host, out, q_bytes, hipMemcpyDeviceToHost));
  char path[4096];
  snprintf(path, sizeof path, "%s/out.bin", dir);
  FILE *f = fopen(path, "wb");
  if (!f || fwrite(host, 1, q_bytes, f) != q_bytes) DIE("cannot write out.bin");
  fclose(f);
  free(host);
  void *bufs[] = {q, k_pages, v_pages, page_table, ctx_lens, q_lens, q_offsets, k_scale, v_scale, workspace, out};
  for (size_t i = 0; i < sizeof bufs / sizeof bufs[0]; ++i)
    if (bufs[i]) HIP_OK(hipFree(bufs[i]));
  HIP_OK(hipStreamDestroy(stream));
  return 0;
}

int main(int argc, char **argv) {
  const int rc = c_abi_client_run(argc, argv);
  if (rc) fprintf(stderr, "%s\n", c_abi_client_error());
  return rc;
}
