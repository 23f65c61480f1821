// Host-side sanitizer run of libchunkkv's argument checks and workspace plans (check_problem, make_plan,
// decode_plan, the hybrid and quality plans): built with -fsanitize=address,undefined on the host pass only and
// run on a machine without a GPU.  Every call below either only computes a size or fails its checks before the
// first launch (the last check is the workspace size, which is passed as 0), so nothing touches a device.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "chunkkv.h"

static int failures = 0;
#define EXPECT(cond)                                                    \
  do {                                                                  \
    if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
  } while (0)

struct Case {
  std::vector<int32_t> seqlen, n_keep;
  std::vector<int64_t> kv_base, out_base;
  chunkkv_problem p;
};

static void make(Case &c, int batch, int hq, int hkv, int d, int w, int chunk, int dtype, int L0, int pct) {
  c.seqlen.resize(batch); c.n_keep.resize(batch); c.kv_base.resize(batch); c.out_base.resize(batch);
  int64_t kv = 0, out = 0;
  int sel_cap = 1, score_cap = 1;
  for (int b = 0; b < batch; ++b) {
    const int L = L0 + 37 * b;
    c.seqlen[b] = L;
    c.n_keep[b] = (int)((int64_t)(L - w) * pct / 100);
    c.kv_base[b] = kv; kv += (int64_t)hkv * L * d;
    c.out_base[b] = out; out += (int64_t)hkv * (c.n_keep[b] + w) * d;
    const int sc = (c.n_keep[b] + chunk - 1) / chunk + 1, cc = (L - w + chunk - 1) / chunk;
    sel_cap = sc > sel_cap ? sc : sel_cap;
    score_cap = cc > score_cap ? cc : score_cap;
  }
  std::memset(&c.p, 0, sizeof(c.p));
  c.p.batch = batch; c.p.n_q_heads = hq; c.p.n_kv_heads = hkv; c.p.head_dim = d; c.p.window = w; c.p.chunk = chunk;
  c.p.dtype = dtype; c.p.softmax_scale = 0.f;
  c.p.seqlen = c.seqlen.data(); c.p.n_keep = c.n_keep.data(); c.p.kv_base = c.kv_base.data();
  c.p.kv_stride_head = 0; c.p.kv_stride_tok = (int64_t)hkv * d;   // [L][Hkv][d] per sequence
  c.p.kv_stride_head = d;
  c.p.out_base = c.out_base.data(); c.p.out_stride_head = d; c.p.out_stride_tok = (int64_t)hkv * d;
  c.p.sel_cap = sel_cap; c.p.score_cap = score_cap; c.p.flags = 0;
}

int main() {
  void *fake = (void *)0x1000;   // never dereferenced
  const int dtypes[3] = {CHUNKKV_F32, CHUNKKV_BF16, CHUNKKV_F16};
  const int chunks[6] = {1, 3, 5, 10, 20, 33};
  int n_cases = 0, n_refused = 0;
  for (int dt = 0; dt < 3; ++dt)
    for (int ci = 0; ci < 6; ++ci)
      for (int batch : {1, 3, 19})
        for (int w : {8, 32, 64})
          for (int d : {64, 128}) {
            const int hkv = 2 + (ci % 3), g = 1 + (batch + ci) % 7, hq = hkv * g;
            if (g * w > 512) continue;
            Case c;
            make(c, batch, hq, hkv, d, w, chunks[ci], dtypes[dt], 97 + 4000 * (ci % 3) + w, 10 + 15 * (ci % 4));
            ++n_cases;
            if (chunkkv_workspace_bytes(&c.p, 1, 1) == 0) {
              // the only shapes of this sweep the library does not support: fp32 rows of 128 elements with more
              // than 256 window rows per kv-head; every entry point says so
              EXPECT(dtypes[dt] == CHUNKKV_F32 && d == 128 && g * w > 256);
              EXPECT(chunkkv_score(&c.p, fake, fake, (float *)fake, nullptr, fake, 1 << 30, nullptr) == CHUNKKV_ERR_UNSUPPORTED);
              ++n_refused;
              continue;
            }
            for (int n_layers : {1, 5, 33})
              for (int reuse : {1, 2, 7}) {
                const size_t ws = chunkkv_workspace_bytes(&c.p, n_layers, reuse);
                EXPECT(ws > 0);
                std::vector<const void *> tab(n_layers, fake);
                std::vector<void *> otab(n_layers, fake);
                // passes every check up to the workspace size
                EXPECT(chunkkv_compress_stack(&c.p, n_layers, reuse, tab.data(), tab.data(), tab.data(), otab.data(),
                                              otab.data(), (int32_t *)fake, (int32_t *)fake, (int32_t *)fake, fake, ws - 1,
                                              nullptr) == CHUNKKV_ERR_WORKSPACE);
                std::vector<int32_t> table((n_layers + reuse - 1) / reuse);
                for (size_t i = 0; i < table.size(); ++i) table[i] = chunks[ci] + (int)(i % 3) * chunks[ci];   // >= chunk
                const size_t wh = chunkkv_workspace_bytes_hybrid(&c.p, n_layers, reuse, table.data());
                EXPECT(wh >= ws);
                EXPECT(chunkkv_compress_stack_hybrid(&c.p, n_layers, reuse, table.data(), tab.data(), tab.data(),
                                                     tab.data(), nullptr, otab.data(), otab.data(), (int32_t *)fake,
                                                     (int32_t *)fake, (int32_t *)fake, fake, wh - 1, nullptr) ==
                       CHUNKKV_ERR_WORKSPACE);
              }
            for (int layer : {0, 1, 6}) {
              const size_t ws1 = chunkkv_workspace_bytes(&c.p, 1, 1);
              EXPECT(chunkkv_compress_layer(&c.p, layer, 2, fake, nullptr, fake, fake, fake, fake, (int32_t *)fake,
                                            (int32_t *)fake, (int32_t *)fake, fake, ws1 - 1, nullptr) == CHUNKKV_ERR_WORKSPACE);
            }
            EXPECT(chunkkv_score(&c.p, fake, fake, (float *)fake, nullptr, fake, 0, nullptr) == CHUNKKV_ERR_WORKSPACE);
            EXPECT(chunkkv_score_lse(&c.p, fake, fake, (const float *)fake, (float *)fake, nullptr, fake, 0, nullptr) ==
                   CHUNKKV_ERR_WORKSPACE);
            for (int compacted : {0, 1}) {
              const size_t wd = chunkkv_decode_workspace_bytes(&c.p, compacted);
              EXPECT(wd > 0);
              EXPECT(chunkkv_decode_attention(&c.p, compacted, nullptr, fake, fake, fake, (float *)fake, nullptr, fake,
                                              wd - 1, nullptr) == CHUNKKV_ERR_WORKSPACE);
            }
            const size_t wq = chunkkv_quality_workspace_bytes(&c.p);
            EXPECT(wq >= chunkkv_decode_workspace_bytes(&c.p, 0));
            EXPECT(chunkkv_quality_metrics(&c.p, nullptr, fake, fake, fake, fake, fake, (float *)fake, (float *)fake, fake,
                                           wq - 1, nullptr) == CHUNKKV_ERR_WORKSPACE);
            // a problem too large for the device-resident scratch array is refused before anything else happens
            if (chunkkv_decode_workspace_bytes(&c.p, 0) > CHUNKKV_STATIC_SCRATCH_BYTES)
              EXPECT(chunkkv_decode_attention_static(&c.p, 0, nullptr, fake, fake, fake, (float *)fake, nullptr, nullptr) ==
                     CHUNKKV_ERR_WORKSPACE);
            // broken problems
            chunkkv_problem bad = c.p;
            bad.n_keep = nullptr;
            EXPECT(chunkkv_workspace_bytes(&bad, 1, 1) == 0);
            bad = c.p; bad.chunk = 0;
            EXPECT(chunkkv_workspace_bytes(&bad, 1, 1) == 0);
            bad = c.p; bad.flags = 0x80;
            EXPECT(chunkkv_score(&bad, fake, fake, (float *)fake, nullptr, fake, 1 << 30, nullptr) == CHUNKKV_ERR_UNSUPPORTED);
            bad = c.p; bad.sel_cap = 0;
            EXPECT(chunkkv_workspace_bytes(&bad, 1, 1) == 0);
          }
  // the 128K headline problem and a long ragged batch
  Case big;
  make(big, 1, 32, 8, 128, 64, 10, CHUNKKV_BF16, 131072, 10);
  EXPECT(chunkkv_workspace_bytes(&big.p, 32, 2) > (size_t)1 << 28);
  EXPECT(chunkkv_workspace_bytes(&big.p, 32, 2) < chunkkv_workspace_bytes(&big.p, 32, 1));
  EXPECT(chunkkv_decode_workspace_bytes(&big.p, 0) <= CHUNKKV_STATIC_SCRATCH_BYTES);
  EXPECT(chunkkv_workspace_bytes(nullptr, 1, 1) == 0);
  EXPECT(std::strcmp(chunkkv_status_string(CHUNKKV_OK), "ok") == 0);
  std::printf("%d problem shapes checked (%d refused as unsupported), %d failures\n", n_cases, n_refused, failures);
  if (failures == 0) std::printf("HOST SANITIZER RUN OK\n");
  return failures ? 1 : 0;
}
