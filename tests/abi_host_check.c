/* Host-side walk through the C ABI for the sanitizer leg of the CPU test suite: every call here is
 * answered by the library's host code alone (argument checks, the buffer planner, the host-side
 * Philox and dropout-mask functions); nothing is launched and no device is needed.  The test
 * builds the library's host side and this file with -fsanitize=address,undefined and runs it: any
 * out-of-bounds access, overflow or leak in that code ends the run with a report. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "elmo_head.h"

static int failures = 0;
#define CHECK(cond)                                                              \
  do {                                                                           \
    if (!(cond)) {                                                               \
      ++failures;                                                                \
      fprintf(stderr, "line %d: %s (last error: %s)\n", __LINE__, #cond, elmo_last_error()); \
    }                                                                            \
  } while (0)

int main(void) {
  /* Philox4x32-10, published known-answer vectors (Salmon et al., SC'11) */
  {
    uint32_t c[4] = {0, 0, 0, 0}, k[2] = {0, 0}, o[4];
    elmo_philox4x32_10(c, k, o);
    CHECK(o[0] == 0x6627E8D5u && o[1] == 0xE169C58Du && o[2] == 0xBC57AC4Cu && o[3] == 0x9B00DBD8u);
    uint32_t c2[4] = {0x243F6A88u, 0x85A308D3u, 0x13198A2Eu, 0x03707344u}, k2[2] = {0xA4093822u, 0x299F31D0u};
    elmo_philox4x32_10(c2, k2, o);
    CHECK(o[0] == 0xD16CFE09u && o[1] == 0x94FDCCEBu && o[2] == 0x5001E420u && o[3] == 0x24126EA1u);
  }
  /* dropout mask: threshold 0 keeps everything, the kept share falls with the threshold */
  {
    CHECK(elmo_dropout_keep16(1, 2, 3, 0) == 0xFFFFu);
    long kept = 0;
    for (uint64_t blk = 0; blk < 4096; ++blk) kept += __builtin_popcount(elmo_dropout_keep16(7, 9, blk + ((uint64_t)1 << 40), 64));
    CHECK(kept > 4096 * 16 * 0.72 && kept < 4096 * 16 * 0.78);
    (void)elmo_dropout_keep16(~0ull, ~0ull, ~0ull, 255);
    (void)elmo_dropout_keep16(0, 0, 0, 1000); /* only the low 8 bits of the threshold count */
  }
  /* the planner over the corners of its argument ranges: an answer or an error text, never undefined behaviour */
  {
    const int64_t Ls[] = {-1, 0, 1, 127, 128, 129, 8192, 670091, 3000000, ((int64_t)1 << 31), ((int64_t)1 << 31) + 1, INT64_MAX};
    const int32_t ds[] = {-128, 0, 100, 128, 256, 768, 65536, 65536 + 256, 1 << 20, (1 << 20) + 128, INT32_MAX};
    const int64_t chunks[] = {-1, 0, 1, 100, 128, 131072, (int64_t)1 << 30, ((int64_t)1 << 30) + 1, INT64_MAX};
    const int32_t Bs[] = {-1, 0, 1, 64, 128, 129, 1024, 65536, 65537, INT32_MAX};
    const int64_t nnzs[] = {-1, 0, 1, 65536, (int64_t)1 << 30, ((int64_t)1 << 30) + 1};
    int ok = 0, bad = 0;
    for (size_t a = 0; a < sizeof Ls / sizeof *Ls; ++a)
      for (size_t b = 0; b < sizeof ds / sizeof *ds; ++b)
        for (size_t c = 0; c < sizeof chunks / sizeof *chunks; ++c)
          for (size_t e = 0; e < sizeof Bs / sizeof *Bs; ++e)
            for (size_t f = 0; f < sizeof nnzs / sizeof *nnzs; ++f)
              for (int fmt = -1; fmt <= 3; ++fmt)
                for (uint32_t flags = 0; flags <= 8; ++flags) {
                  size_t w = 0, cp = 0, ws = 0;
                  const int64_t kr = (flags & ELMO_KAHAN) && Ls[a] > 256 ? 128 : 0;
                  const int rc = elmo_head_sizes(Ls[a], ds[b], fmt, chunks[c], Bs[e], nnzs[f], flags, kr, &w, &cp, &ws);
                  if (rc == 0) {
                    ++ok;
                    CHECK(w == (size_t)Ls[a] * (size_t)ds[b] * (fmt == ELMO_FP8_E4M3 ? 1 : 2));
                    CHECK(cp == ((flags & ELMO_KAHAN) ? (size_t)(kr ? kr : Ls[a]) * (size_t)ds[b] * 2 : 0));
                    CHECK(ws >= elmo_logit_buffer_bytes(Bs[e], chunks[c] < Ls[a] ? chunks[c] : Ls[a]));
                  } else {
                    ++bad;
                    CHECK(rc == -1 || rc == -2);
                    CHECK(strlen(elmo_last_error()) > 10);
                  }
                }
    CHECK(ok > 1000 && bad > 1000);
    CHECK(elmo_head_sizes(1000, 256, ELMO_BF16, 512, 8, 64, 0, 0, NULL, NULL, NULL) == 0); /* outputs are optional */
    CHECK(elmo_head_sizes(1000, 256, ELMO_BF16, 512, 8, 64, ELMO_KAHAN, 100, NULL, NULL, NULL) == -1);
    CHECK(elmo_logit_buffer_bytes(-1, 5) == 0 && elmo_logit_buffer_bytes(128, 2812281) == (size_t)128 * 2812281 * 2);
  }
  /* create / destroy: rejected before anything touches a device */
  {
    elmo_head_t* h = NULL;
    elmo_head_opts o;
    memset(&o, 0, sizeof o);
    CHECK(elmo_head_create(1000, 256, ELMO_BF16, 512, NULL, &h) == -1);
    CHECK(elmo_head_create(1000, 256, ELMO_BF16, 512, &o, NULL) == -1);
    o.max_B = 8;
    o.max_nnz = 64;
    CHECK(elmo_head_create(1000, 256, ELMO_BF16, 512, &o, &h) == -1 && h == NULL); /* no buffers */
    size_t w = 0, cp = 0, ws = 0;
    CHECK(elmo_head_sizes(1000, 256, ELMO_FP8_E4M3, 512, 8, 64, ELMO_KAHAN | ELMO_SR, 0, &w, &cp, &ws) == 0);
    o.flags = ELMO_KAHAN | ELMO_SR;
    /* pointers are only compared and stored by create: fake 256-byte aligned addresses, never dereferenced */
    o.W = (void*)(uintptr_t)0x10000; o.W_bytes = w;
    o.comp = (void*)(uintptr_t)0x20000; o.comp_bytes = cp - 1;
    o.workspace = (void*)(uintptr_t)0x30000; o.workspace_bytes = ws;
    CHECK(elmo_head_create(1000, 256, ELMO_FP8_E4M3, 512, &o, &h) == -1); /* compensation one byte short */
    o.comp_bytes = cp;
    o.W = (void*)(uintptr_t)0x10010;
    CHECK(elmo_head_create(1000, 256, ELMO_FP8_E4M3, 512, &o, &h) == -1); /* misaligned */
    o.W = (void*)(uintptr_t)0x10000;
    o.dropout_p = 2.0f;
    CHECK(elmo_head_create(1000, 256, ELMO_FP8_E4M3, 512, &o, &h) == -1);
    o.dropout_p = 0.25f;
    o.weight_decay = -1.0f;
    CHECK(elmo_head_create(1000, 256, ELMO_FP8_E4M3, 512, &o, &h) == -1);
    o.weight_decay = 1e-4f;
    for (int i = 0; i < 3; ++i) {                     /* a head is host memory only: create and destroy leak nothing */
      CHECK(elmo_head_create(1000, 256, ELMO_FP8_E4M3, 512, &o, &h) == 0 && h != NULL);
      CHECK(elmo_head_profile(h, 1) == 0 && elmo_head_profile(h, 0) == 0);
      /* argument checks of the calls that would launch: refused before any launch */
      CHECK(elmo_head_step(h, NULL, 4, NULL, NULL, 0, 0.05f, 0, 0, NULL, NULL, NULL) == -1);
      CHECK(elmo_head_step(h, (void*)(uintptr_t)0x40000, 9, (int32_t*)(uintptr_t)0x50000, NULL, 0, 0.05f, 0, 0, NULL, NULL, NULL) == -1);
      CHECK(elmo_head_step(h, (void*)(uintptr_t)0x40000, 4, (int32_t*)(uintptr_t)0x50000, NULL, 65, 0.05f, 0, 0, NULL, NULL, NULL) == -1);
      CHECK(elmo_head_step(h, (void*)(uintptr_t)0x40000, 4, (int32_t*)(uintptr_t)0x50000, NULL, 5, 0.05f, 0, 0, NULL, NULL, NULL) == -1);
      CHECK(elmo_head_step(h, (void*)(uintptr_t)0x40000, 4, (int32_t*)(uintptr_t)0x50000, (int32_t*)(uintptr_t)0x60000, 5, 0.05f, 0,
                           (uint64_t)1 << 63, NULL, NULL, NULL) == -1);
      CHECK(elmo_head_topk(h, NULL, 4, 5, NULL, NULL, NULL) == -1);
      CHECK(elmo_head_topk(h, (void*)(uintptr_t)0x40000, 0, 5, NULL, NULL, NULL) == -1);
      CHECK(elmo_head_topk(h, (void*)(uintptr_t)0x40000, 4, 0, NULL, NULL, NULL) == -1);
      CHECK(elmo_head_topk(h, (void*)(uintptr_t)0x40000, 4, 1001, NULL, NULL, NULL) == -1);
      CHECK(elmo_head_destroy(h) == 0);
      h = NULL;
    }
    CHECK(elmo_head_destroy(NULL) == -1);
    CHECK(elmo_head_step(NULL, NULL, 1, NULL, NULL, 0, 0.0f, 0, 0, NULL, NULL, NULL) == -1);
    double ms[6];
    int64_t n[6];
    CHECK(elmo_head_profile_read(NULL, ms, n) == -1);
  }
  /* the stand-alone calls */
  {
    CHECK(elmo_quantize(NULL, 10, ELMO_BF16, 0, 0, 0, 0, NULL, NULL) == -1);
    CHECK(elmo_quantize(NULL, 0, ELMO_BF16, 0, 0, 0, 0, NULL, NULL) == 0);
    CHECK(elmo_quantize((float*)(uintptr_t)0x1000, 10, 5, 0, 0, 0, 0, (void*)(uintptr_t)0x2000, NULL) == -2);
    CHECK(elmo_quantize((float*)(uintptr_t)0x1000, 10, ELMO_BF16, 2, 0, 0, 0, (void*)(uintptr_t)0x2000, NULL) == -1);
    CHECK(elmo_quantize_em((float*)(uintptr_t)0x1000, 10, 9, 3, 0, 0, 0, 0, (float*)(uintptr_t)0x2000, NULL) == -2);
    CHECK(elmo_quantize_em((float*)(uintptr_t)0x1000, 10, 4, 23, 0, 0, 0, 0, (float*)(uintptr_t)0x2000, NULL) == -2);
    CHECK(elmo_quantize_em(NULL, 0, 4, 3, 1, 0, 0, 0, NULL, NULL) == 0);
    CHECK(elmo_precision_hits(NULL, 4, 5, NULL, NULL, NULL, NULL) == -1);
    CHECK(elmo_precision_hits((int32_t*)(uintptr_t)0x1000, 1 << 20, 1 << 12, (int32_t*)(uintptr_t)0x1000, NULL, (int64_t*)(uintptr_t)0x1000, NULL) == -1);
    CHECK(elmo_kahan_adamw(NULL, NULL, NULL, NULL, NULL, 8, ELMO_BF16, 1e-3f, 0.9, 0.999, 1e-8f, 0.0f, 1, NULL) == -1);
    CHECK(elmo_kahan_adamw(NULL, NULL, NULL, NULL, NULL, 0, ELMO_BF16, 1e-3f, 0.9, 0.999, 1e-8f, 0.0f, 1, NULL) == 0);
    CHECK(elmo_topk_static(NULL, 10, 256, ELMO_BF16, NULL, 1, 1, NULL, NULL, NULL) == -1);
    CHECK(elmo_topk_static((void*)(uintptr_t)0x1000, 1000, 256, ELMO_BF16, (void*)(uintptr_t)0x2000, 129, 5, NULL, NULL, NULL) == -1);
    CHECK(elmo_topk_static((void*)(uintptr_t)0x1000, 1000, 8192, ELMO_BF16, (void*)(uintptr_t)0x2000, 8, 5, NULL, NULL, NULL) == -1);
    CHECK(elmo_topk_static((void*)(uintptr_t)0x1000, 1000, 256, 7, (void*)(uintptr_t)0x2000, 8, 5, NULL, NULL, NULL) == -2);
    CHECK(elmo_topk_static((void*)(uintptr_t)0x1000, 1000, 256, ELMO_BF16, (void*)(uintptr_t)0x2000, 8, 1001, NULL, NULL, NULL) == -1);
  }
  if (failures) {
    fprintf(stderr, "%d host-side ABI checks failed\n", failures);
    return 1;
  }
  puts("host-side ABI checks passed");
  return 0;
}
