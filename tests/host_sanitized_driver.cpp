// Host-side driver for the sanitizer build of the library's plan code (tests/test_host_sanitized.py links it with
// csrc/mdbf_api.hip compiled under AddressSanitizer and UndefinedBehaviorSanitizer on the host side).  It calls
// only host functions of the C ABI, over placeholder device pointers: plan building touches no device memory.
// Every plan buffer is a heap block of exactly the size the library asked for, so that a write past the plan
// or the tables inside it lands in a red zone.  Prints one line per case; exit status 0 when every call
// returned what the case expects.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "mdbf.h"

static void* const FAKE = (void*)(uintptr_t)0x10000000;
static int g_fail = 0;

static mdbf_layer_t layer(int m, int n, int k, int l, int T, int env_dt = MDBF_F16, uint32_t flags = 0) {
  mdbf_layer_t L;
  memset(&L, 0, sizeof(L));
  L.desc.m = m; L.desc.n = n; L.desc.k = k; L.desc.l = l;
  L.desc.x_dtype = MDBF_F16; L.desc.env_dtype = env_dt; L.desc.y_dtype = MDBF_F16; L.desc.flags = flags;
  L.SA_packed_dev = FAKE; L.SB_packed_dev = FAKE;
  L.env.A_dev = FAKE; L.env.Q_dev = FAKE; L.env.G_dev = FAKE; L.env.B_dev = FAKE;
  L.X_dev = FAKE; L.ldx = n; L.Y_dev = FAKE; L.ldy = m; L.T = T;
  return L;
}

// builds the plan into an exact-size heap block; expect: the status both calls must return
static void plan_case(const char* name, const std::vector<mdbf_layer_t>& layers, int expect = MDBF_OK) {
  size_t pb = 0, wb = 0;
  int st = mdbf_batch_plan_bytes((int)layers.size(), layers.data(), &pb, &wb);
  const char* k1 = "";
  const char* k2 = "";
  if (st == MDBF_OK) {
    unsigned char* buf = (unsigned char*)malloc(pb);
    st = mdbf_batch_plan_build((int)layers.size(), layers.data(), FAKE, wb, buf, pb);
    if (st == MDBF_OK) {
      k1 = mdbf_batch_plan_kernel(buf, pb, 1);
      k2 = mdbf_batch_plan_kernel(buf, pb, 2);
      // a second build into an unaligned block of the same size (the header says: any alignment)
      unsigned char* odd = (unsigned char*)malloc(pb + 1);
      if (mdbf_batch_plan_build((int)layers.size(), layers.data(), FAKE, wb, odd + 1, pb) != MDBF_OK) st = -100;
      else if (memcmp(odd + 1, buf, pb) != 0) st = -101;
      free(odd);
      // too small a plan buffer or workspace must be refused, not written
      if (pb > 16 && mdbf_batch_plan_build((int)layers.size(), layers.data(), FAKE, wb, buf, pb - 16) == MDBF_OK) st = -102;
      if (wb > 0 && mdbf_batch_plan_build((int)layers.size(), layers.data(), FAKE, wb - 1, buf, pb) == MDBF_OK) st = -103;
    }
    free(buf);
  }
  printf("%-28s layers %6zu plan %9zu B workspace %11zu B status %d kernels %s %s\n", name, layers.size(), pb, wb, st,
         k1, k2);
  if (st != expect) {
    printf("  FAILED: expected status %d\n", expect);
    g_fail = 1;
  }
}

int main() {
  uint64_t rng = 0x9E3779B97F4A7C15ull;
  auto next = [&](int lo, int hi) {
    rng = rng * 6364136223846793005ull + 1442695040888963407ull;
    return lo + (int)((rng >> 33) % (uint64_t)(hi - lo + 1));
  };
  plan_case("attn 336", std::vector<mdbf_layer_t>(336, layer(4096, 4096, 2656, 16, 1)));
  plan_case("attn 256 (whole rounds)", std::vector<mdbf_layer_t>(256, layer(4096, 4096, 2656, 16, 1)));
  plan_case("attn 337 (odd tail)", std::vector<mdbf_layer_t>(337, layer(4096, 4096, 2656, 16, 1)));
  plan_case("one layer", std::vector<mdbf_layer_t>(1, layer(4096, 4096, 2656, 16, 1)));
  plan_case("rank 8", std::vector<mdbf_layer_t>(400, layer(4096, 4096, 1856, 8, 1)));
  {
    std::vector<mdbf_layer_t> v;
    for (int i = 0; i < 32; ++i) {
      for (int j = 0; j < 4; ++j) v.push_back(layer(4096, 4096, 2656, 16, 1));
      v.push_back(layer(11008, 4096, 4096, 16, 1));
      v.push_back(layer(11008, 4096, 4096, 16, 1));
      v.push_back(layer(4096, 11008, 4096, 16, 1));
    }
    plan_case("stack 1.5 bpw T=1", v);
    for (auto& L : v) L.T = 8;
    plan_case("stack 1.5 bpw T=8", v);
    for (size_t i = 0; i < v.size(); ++i) v[i].T = 1 + (int)(i % 16);
    plan_case("stack, tokens 1..16", v);
  }
  {
    std::vector<mdbf_layer_t> v;
    for (int i = 0; i < 300; ++i) v.push_back(layer(next(1, 3000), next(1, 3000), next(1, 3000), 16, next(1, 3)));
    plan_case("300 random shapes l=16", v);
    v.clear();
    for (int i = 0; i < 500; ++i)
      v.push_back(layer(next(1, 700), next(1, 700), next(1, 700), next(1, 16), next(1, 17), i % 3 == 0 ? MDBF_F32 : MDBF_F16));
    plan_case("500 random, any rank/dtype", v);
    v.clear();
    for (int i = 0; i < 200; ++i) v.push_back(layer(next(2000, 6000), next(129, 6000), next(129, 6000), 16, 1, MDBF_F16,
                                                     i % 2 ? MDBF_FLAG_BLOCK_SCALED : 0));
    plan_case("200 large, half forced mx", v);
    v.clear();
    for (int i = 0; i < 64; ++i) v.push_back(layer(4096, 4096, 2656, 16, 1, MDBF_F16, MDBF_FLAG_FP16_STAGED));
    plan_case("64 fp16-staged", v);
    v.clear();
    for (int i = 0; i < 40; ++i) v.push_back(layer(512, 512, 256, 4, 1, MDBF_F32, MDBF_FLAG_PRECISE));
    plan_case("40 precise", v);
  }
  // more work items than a table can index: refused
  plan_case("70000 tiny layers", std::vector<mdbf_layer_t>(70000, layer(16, 16, 16, 4, 1)), MDBF_EUNSUPPORTED);
  plan_case("no layers", std::vector<mdbf_layer_t>(), MDBF_EINVAL);

  // workspace sizes of single calls and of the projection, over a range of shapes (host arithmetic only)
  size_t total = 0;
  for (int i = 0; i < 2000; ++i) {
    mdbf_desc_t d = layer(next(1, 12000), next(1, 12000), next(1, 6000), next(1, 16), 1, i % 2 ? MDBF_F16 : MDBF_BF16).desc;
    size_t b = 0;
    if (mdbf_workspace_bytes(&d, next(1, 40), &b) != MDBF_OK) g_fail = 1;
    total += b;
    size_t mb = 0;
    const int st = mdbf_msvid_workspace_bytes(d.m, d.k, d.l, &mb);
    if (st != MDBF_OK && st != MDBF_EUNSUPPORTED) g_fail = 1;
  }
  printf("workspace sizes: 2000 shapes, %zu bytes in total\n", total);
  printf(g_fail ? "FAILED\n" : "ok\n");
  return g_fail;
}
