/* Host-side sweep of the library's planning code (workspace sizing, slab fitting, option and argument
 * checks) over shapes from 1 to the largest sizes the ABI accepts and over every flag combination that
 * changes a layout.  Nothing here reaches the GPU: every call either is pure host arithmetic or is refused
 * before the first HIP call.  tests/test_abi.py builds the library's host code with the address and
 * undefined-behaviour sanitizers and runs this program against it. */
#include <stdio.h>
#include <string.h>

#include "cce.h"

static int fail(const char* what, long long n, long long d, long long v, unsigned flags) {
  printf("FAILED %s at N=%lld D=%lld V=%lld flags=%u\n", what, n, d, v, flags);
  return 1;
}

int main(void) {
  static const long long Ns[] = {1, 7, 255, 256, 257, 1024, 8192, 65536, 131072, 131073, 1 << 24, 0x7fff0000LL};
  static const long long Ds[] = {8, 64, 72, 2304, 5120, 1 << 22};
  static const long long Vs[] = {1, 2, 255, 256, 257, 32064, 256000, 1 << 24, 0x7fff0000LL};
  static const unsigned flag_sets[] = {0u, CCE_FILTER_DE | CCE_FILTER_DC, CCE_VOCAB_SORT, CCE_SKIP_TILES,
                                       CCE_COMPACT_IGNORED, CCE_PLAIN_KERNELS, CCE_ACCUM_KAHAN,
                                       CCE_VOCAB_SORT | CCE_COMPACT_IGNORED | CCE_SKIP_TILES | CCE_ACCUM_BF16};
  static char host_buffer[8192];
  char* p = (char*)(((size_t)host_buffer + 255) / 256 * 256);
  unsigned long long calls = 0;
  for (int dt = 0; dt < 2; ++dt)
    for (size_t fi = 0; fi < sizeof(flag_sets) / sizeof(flag_sets[0]); ++fi)
      for (size_t ni = 0; ni < sizeof(Ns) / sizeof(Ns[0]); ++ni)
        for (size_t di = 0; di < sizeof(Ds) / sizeof(Ds[0]); ++di)
          for (size_t vi = 0; vi < sizeof(Vs) / sizeof(Vs[0]); ++vi) {
            const long long N = Ns[ni], D = Ds[di], V = Vs[vi];
            cce_opts o;
            cce_default_opts(dt ? CCE_F32 : CCE_BF16, &o);
            o.flags = flag_sets[fi];
            const size_t f = cce_workspace_bytes(CCE_OP_FORWARD, N, D, V, &o);
            const size_t mn = cce_workspace_bytes(CCE_OP_BACKWARD_MIN, N, D, V, &o);
            const size_t rec = cce_workspace_bytes(CCE_OP_BACKWARD, N, D, V, &o);
            const size_t wide = cce_workspace_bytes(CCE_OP_BACKWARD_WIDE, N, D, V, &o);
            if (f == 0 || mn == 0) return fail("zero size", N, D, V, o.flags);
            if (!(mn <= rec && rec <= wide)) return fail("min <= recommended <= wide", N, D, V, o.flags);
            if (f % 256 || mn % 256 || rec % 256 || wide % 256) return fail("sizes are multiples of 256", N, D, V, o.flags);
            if (cce_block_max_bytes(N, V) == 0) return fail("block_max size", N, D, V, o.flags);
            int br = 0, bc = 0;
            cce_filter_block(N, D, V, &o, &br, &bc);
            if (br <= 0 || bc <= 0) return fail("filter block", N, D, V, o.flags);
            /* a workspace that is too small is refused before anything touches the device */
            o.workspace = p;
            o.workspace_bytes = 256;
            o.filter_eps = 0x1p-12f;
            int st = cce_forward_ex(p, p, (const int64_t*)p, N, D, V, 0.0f, -100, (float*)p, (float*)p, &o);
            if (st != CCE_EWORKSPACE && st != CCE_EUNSUPPORTED && st != CCE_EINVAL) return fail("forward refusal", N, D, V, o.flags);
            st = cce_backward_ex(p, p, (const int64_t*)p, N, D, V, 30.0f, -100, (const float*)p, (const float*)p, p, p, &o);
            if (st != CCE_EWORKSPACE && st != CCE_EUNSUPPORTED && st != CCE_EINVAL) return fail("backward refusal", N, D, V, o.flags);
            calls += 8;
          }
  /* sizes beyond the ABI's limits and other bad arguments */
  cce_opts o;
  cce_default_opts(CCE_BF16, &o);
  if (cce_workspace_bytes(CCE_OP_FORWARD, 0, 64, 64, &o) != 0 || cce_workspace_bytes(7, 8, 64, 64, &o) != 0) return 2;
  if (cce_workspace_bytes(CCE_OP_FORWARD, 8, 64, 64, NULL) != 0) return 3;
  o.workspace = p;
  o.workspace_bytes = 4096;
  if (cce_forward_ex(p, p, (const int64_t*)p, 0x7fff0001LL, 64, 64, 0.0f, -100, (float*)p, (float*)p, &o) != CCE_EINVAL) return 4;
  if (cce_forward_ex(p, p, (const int64_t*)p, 8, (1 << 22) + 8, 64, 0.0f, -100, (float*)p, (float*)p, &o) != CCE_EINVAL) return 5;
  if (cce_forward_noalloc(p, p, (const int64_t*)p, 1 << 22, 64, 64, 0.0f, -100, (float*)p, (float*)p, &o) != CCE_ESCRATCH) return 6;
  if (strstr(cce_strerror(CCE_ESCRATCH), "8388608") == NULL) return 7;
  if (cce_set_workspace(p + 8, 1024) != CCE_EINVAL || cce_set_workspace(NULL, 16) != CCE_EINVAL) return 8;
  if (cce_noalloc_scratch_bytes() != (size_t)8 << 20) return 9;
  for (int s = 1; s >= -7; --s)
    if (strlen(cce_strerror(s)) == 0) return 10;
  printf("host sweep ok: %llu calls\n", calls);
  return 0;
}
