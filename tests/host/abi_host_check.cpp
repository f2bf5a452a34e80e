// Drives the C ABI of libvq on the host only: every entry point with valid and invalid
// arguments, and many random descriptors, against launcher stand-ins that check the launch
// parameters (launcher_stubs.cpp).  Built with AddressSanitizer and UBSan on the host side by
// tests/test_host_sanitizers.py; the "device" pointers are addresses inside one host buffer that
// nothing dereferences.  Exit status 0 and a last line "host check ok" mean that no sanitizer
// report, no violated launch assumption and no unexpected status occurred.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../../include/vq.h"

#include "../../paper_2402_15319_amd/csrc/vq_internal.h"

namespace vq { long long stub_launch_count(); }

namespace {

int g_failures = 0;
#define EXPECT(cond)                                                           \
  do {                                                                         \
    if (!(cond)) {                                                             \
      std::fprintf(stderr, "%s:%d: expectation failed: %s\n", __FILE__, __LINE__, #cond); \
      ++g_failures;                                                            \
    }                                                                          \
  } while (0)

uint64_t g_state = 0x9E3779B97F4A7C15ull;
uint32_t rnd() {   // splitmix64, upper half
  uint64_t z = (g_state += 0x9E3779B97F4A7C15ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return (uint32_t)((z ^ (z >> 31)) >> 32);
}
int pick(std::initializer_list<int> v) { return *(v.begin() + rnd() % v.size()); }

vq_desc make(int out, int in, int gr, int d, int k, int bits, int dtype) {
  vq_desc s;
  std::memset(&s, 0, sizeof s);
  s.out_features = out; s.in_features = in; s.group_rows = gr; s.group_cols = 256;
  s.d = d; s.k = k; s.index_bits = bits; s.codebook_dtype = dtype;
  return s;
}

// The representations the decode path accepts (format, group heights).
std::vector<vq_desc> supported(int out_mult, int n_cb) {
  std::vector<vq_desc> v;
  const int in = 256 * n_cb;
  v.push_back(make(8 * out_mult, in, 8, 2, 16, 4, VQ_F16));
  v.push_back(make(8 * out_mult, in, 8, 2, 256, 8, VQ_F16));
  v.push_back(make(8 * out_mult, in, 8, 2, 16, 4, VQ_I8));
  v.push_back(make(8 * out_mult, in, 4, 2, 16, 4, VQ_I8));
  v.push_back(make(8 * out_mult, in, 8, 2, 32, 5, VQ_I8));
  for (int gr : {8, 16, 32}) v.push_back(make(gr * out_mult, in, gr, 2, 64, 6, VQ_I8));
  for (int gr : {8, 16, 32}) v.push_back(make(gr * out_mult, in, gr, 2, 64, 6, VQ_I8_BN));
  v.push_back(make(8 * out_mult, in, 8, 2, 16, 4, VQ_I8_BN));
  for (int gr : {64, 128, 256}) v.push_back(make(gr * out_mult, in, gr, 2, 256, 8, VQ_I8));
  v.push_back(make(8 * out_mult, in, 8, 1, 16, 4, VQ_F16));
  for (int gr : {8, 16, 32}) v.push_back(make(gr * out_mult, in, gr, 1, 8, 3, VQ_I8));
  for (int gr : {8, 16, 32}) v.push_back(make(gr * out_mult, in, gr, 1, 8, 3, VQ_I8_BN));
  v.push_back(make(8 * out_mult, in, 1, 1, 4, 2, VQ_I8));
  for (int gr : {64, 128, 256}) v.push_back(make(gr * out_mult, in, gr, 4, 256, 8, VQ_I8));
  for (int gr : {64, 128, 256}) v.push_back(make(gr * out_mult, in, gr, 4, 256, 8, VQ_F16));
  for (int gr : {64, 128, 256}) v.push_back(make(gr * out_mult, in, gr, 4, 256, 8, VQ_I8_BN));
  for (int gr : {64, 128, 256}) v.push_back(make(gr * out_mult, in, gr, 2, 256, 8, VQ_I8_BN));
  return v;
}

}  // namespace

int main(int argc, char** argv) {
  // Planted mistakes, to show that the checks are live (the test expects both to die):
  if (argc > 1 && !std::strcmp(argv[1], "--plant-overflow")) {
    std::vector<int> v(8);
    volatile int* p = v.data();
    std::printf("%d\n", p[8 + (argc > 5)]);            // one past the end of a heap buffer
    return 0;
  }
  if (argc > 1 && !std::strcmp(argv[1], "--plant-launch")) {
    static vq::GemvBatch b;                              // a split-K launch whose grid misses a workgroup
    b.count = 1; b.total_wgs = 4; b.total_cost = 64;
    b.p[0].idx = (const uint8_t*)argv; b.p[0].cb = (const uint32_t*)argv; b.p[0].x = (const uint16_t*)argv; b.p[0].y = argv;
    b.p[0].n_rb = 16; b.p[0].n_cb = 4; b.p[0].splits = 1; b.p[0].rb_per_cb = 1;
    return vq::launch_gemv(16, b, 2, 3, 4, nullptr, 4) == hipSuccess ? 0 : 1;
  }
  // one host buffer; "device" pointers are 16-byte aligned addresses inside it
  std::vector<unsigned char> arena(1 << 16);
  unsigned char* base = arena.data() + (16 - (reinterpret_cast<uintptr_t>(arena.data()) & 15)) % 16;
  void* idx = base; void* cb = base + 4096; void* x = base + 8192; void* y = base + 12288;
  void* A = base + 16384; void* Bm = base + 20480; void* ws = base + 24576;

  EXPECT(vq_version() >= 1);
  for (int st = -10; st <= 1; ++st) EXPECT(vq_status_string(st) != nullptr);

  // ---- every supported representation, several shapes: sizes, pack, decode, gemv, gemm
  long long ok_calls = 0;
  for (int out_mult : {1, 3, 8, 43, 172, 512, 1376, 4100}) {
    for (int n_cb : {1, 2, 3, 4, 5, 8, 16, 17, 43, 96, 97, 130}) {
      for (const vq_desc& d : supported(out_mult, n_cb)) {
        size_t a = 0, b = 0, c = 0, e = 0;
        EXPECT(vq_canonical_bytes(&d, &a, &b) == VQ_OK && a > 0 && b > 0);
        const int st = vq_layout_bytes(&d, &c, &e);
        if (st != VQ_OK) continue;     // e.g. out_features not a multiple of 64 for the 64-row kernels
        EXPECT(c >= a && e > 0);
        EXPECT(vq_pack_layout(&d, idx, cb, y, x, nullptr) == VQ_OK);
        EXPECT(vq_decode_dense(&d, idx, cb, y, nullptr) == VQ_OK);
        for (int dt : {VQ_F16, VQ_F32}) {
          EXPECT(vq_gemv(&d, idx, cb, x, y, dt, nullptr) == VQ_OK);
          for (int B : {1, 7, 16, 17, 32, 100, 256, 1000, 2048, 5000}) {
            const int ld = (B + 7) / 8 * 8;
            EXPECT(vq_gemm_batched(&d, idx, cb, x, B, ld, y, ld, dt, nullptr) == VQ_OK);
          }
        }
        ++ok_calls;
      }
    }
  }
  EXPECT(ok_calls > 500);

  // ---- several matrices per launch, with and without adapters: random mixes of shapes
  for (int trial = 0; trial < 400; ++trial) {
    const int fmt_pick = rnd() % 16;
    const int count = 1 + rnd() % (trial % 7 == 0 ? 600 : 12);
    std::vector<vq_desc> descs;
    std::vector<const void*> idxs, cbs, xs;
    std::vector<void*> ys;
    std::vector<vq_lora_desc> lora;
    for (int i = 0; i < count; ++i) {
      const int n_cb = pick({1, 2, 3, 4, 8, 16, 43, 96, 100});
      const int m = pick({1, 2, 5, 64, 172, 512, 1376, 4096});
      vq_desc d;
      switch (fmt_pick) {
        case 0: d = make(8 * m, 256 * n_cb, 8, 2, 16, 4, VQ_F16); break;
        case 1: d = make(8 * m, 256 * n_cb, 8, 2, 256, 8, VQ_F16); break;
        case 2: d = make(32 * m, 256 * n_cb, pick({8, 16, 32}), 2, 64, 6, VQ_I8); break;
        case 3: d = make(8 * m, 256 * n_cb, 8, 2, 16, 4, VQ_I8); break;
        case 4: d = make(32 * m, 256 * n_cb, pick({8, 16, 32}), 2, 64, 6, VQ_I8_BN); break;
        case 5: d = make(8 * m, 256 * n_cb, 8, 1, 16, 4, VQ_F16); break;
        case 6: d = make(32 * m, 256 * n_cb, pick({8, 16, 32}), 1, 8, 3, VQ_I8); break;
        case 7: d = make(8 * m, 256 * n_cb, 1, 1, 4, 2, VQ_I8); break;
        case 8: d = make(256 * m, 256 * n_cb, pick({64, 128, 256}), 4, 256, 8, VQ_I8); break;
        case 9: d = make(8 * m, 256 * n_cb, 8, 2, 16, 4, VQ_I8_BN); break;
        case 10: d = make(32 * m, 256 * n_cb, pick({8, 16, 32}), 1, 8, 3, VQ_I8_BN); break;
        case 11: d = make(256 * m, 256 * n_cb, pick({64, 128, 256}), 4, 256, 8, VQ_I8_BN); break;
        case 12: d = make(256 * m, 256 * n_cb, pick({64, 128, 256}), 2, 256, 8, VQ_I8_BN); break;
        case 13: d = make(8 * m, 256 * n_cb, 4, 2, 16, 4, VQ_I8); break;
        case 14: d = make(8 * m, 256 * n_cb, 8, 2, 32, 5, VQ_I8); break;
        default: d = make(256 * m, 256 * n_cb, pick({64, 128, 256}), 2, 256, 8, VQ_I8); break;
      }
      descs.push_back(d);
      idxs.push_back(idx); cbs.push_back(cb); xs.push_back(x); ys.push_back(y);
      vq_lora_desc l;
      std::memset(&l, 0, sizeof l);
      l.rank = 8 * (rnd() % 9);
      l.A_f16 = l.rank ? A : nullptr;
      l.B_f16 = l.rank ? Bm : nullptr;
      lora.push_back(l);
    }
    const int dt = rnd() % 2 ? VQ_F16 : VQ_F32;
    EXPECT(vq_gemv_multi(count, descs.data(), idxs.data(), cbs.data(), xs.data(), ys.data(), dt, nullptr) == VQ_OK);
    size_t need = 0;
    EXPECT(vq_lora_workspace_bytes(count, &need) == VQ_OK && need >= (size_t)count * 4 * 64);
    EXPECT(vq_gemv_lora_multi(count, descs.data(), idxs.data(), cbs.data(), xs.data(), lora.data(), ws, need,
                              ys.data(), dt, nullptr) == VQ_OK);
    EXPECT(vq_gemv_lora_multi(count, descs.data(), idxs.data(), cbs.data(), xs.data(), lora.data(), ws, need - 1,
                              ys.data(), dt, nullptr) == VQ_ERR_BAD_ARG);
    // the variant without a workspace needs a GPU for the address of its static array: with one
    // it succeeds, without one it reports the runtime error; more than 256 products are refused
    const int st = vq_gemv_lora_multi_static(count, descs.data(), idxs.data(), cbs.data(), xs.data(), lora.data(),
                                             ys.data(), dt, nullptr);
    EXPECT(count > 256 ? st == VQ_ERR_BAD_ARG : (st == VQ_OK || st == VQ_ERR_HIP));
  }

  // ---- quantiser steps: every group shape of the decode formats
  for (int d : {1, 2, 4})
    for (int k : {4, 8, 16, 32, 64, 256})
      for (int gr : {1, 4, 8, 16, 32, 64, 128, 256}) {
        int bits = 0;
        while ((1 << bits) < k) ++bits;
        const vq_desc s = make((gr < 8 ? 8 : gr) * 3, 512, gr, d, k, bits, VQ_F16);
        const int st = vq_em_assign(&s, idx, cb, x, y, nullptr);
        EXPECT(st == VQ_OK || st == VQ_ERR_UNSUPPORTED);
        EXPECT(vq_em_update(&s, idx, cb, x, y, nullptr) == st);
      }

  // ---- arguments that must be refused before any launch
  {
    const long long before = vq::stub_launch_count();
    vq_desc d = make(64, 512, 8, 2, 16, 4, VQ_F16);
    size_t a, b;
    EXPECT(vq_layout_bytes(nullptr, &a, &b) == VQ_ERR_NULL);
    EXPECT(vq_gemv(&d, nullptr, cb, x, y, VQ_F16, nullptr) == VQ_ERR_NULL);
    EXPECT(vq_gemv(&d, idx, cb, x, x, VQ_F16, nullptr) == VQ_ERR_BAD_ARG);
    EXPECT(vq_gemv(&d, idx, cb, x, y, 7, nullptr) == VQ_ERR_BAD_ARG);
    EXPECT(vq_gemv(&d, (char*)idx + 4, cb, x, y, VQ_F16, nullptr) == VQ_ERR_ALIGN);
    EXPECT(vq_gemm_batched(&d, idx, cb, x, 0, 8, y, 8, VQ_F16, nullptr) == VQ_ERR_BAD_ARG);
    EXPECT(vq_gemm_batched(&d, idx, cb, x, 16, 8, y, 16, VQ_F16, nullptr) == VQ_ERR_BAD_ARG);
    EXPECT(vq_gemm_batched(&d, idx, cb, x, 4, 12, y, 16, VQ_F16, nullptr) == VQ_ERR_ALIGN);
    for (int trial = 0; trial < 20000; ++trial) {   // random descriptors: any status but a crash
      vq_desc r = make((int)(rnd() % 70000) - 100, (int)(rnd() % 40000) - 100, pick({0, 1, 4, 8, 16, 32, 64, 128, 256, 512, -8}),
                       pick({0, 1, 2, 3, 4, 8}), pick({0, 2, 4, 8, 16, 32, 64, 128, 256, 512, 65536}),
                       pick({0, 1, 2, 3, 4, 5, 6, 8, 16, 31, 40}), pick({VQ_F16, VQ_I8, VQ_I8_BN, 9}));
      if (rnd() % 4 == 0) r.group_cols = pick({0, 32, 128, 512, -256});
      size_t c = 0, e = 0;
      const int s1 = vq_canonical_bytes(&r, &c, &e);
      const int s2 = vq_layout_bytes(&r, &c, &e);
      EXPECT(s1 <= 0 && s2 <= 0);
      if (s2 != VQ_OK) {   // what the size query refuses, the compute calls refuse too
        EXPECT(vq_gemv(&r, idx, cb, x, y, VQ_F16, nullptr) != VQ_OK);
        EXPECT(vq_decode_dense(&r, idx, cb, y, nullptr) != VQ_OK);
        EXPECT(vq_gemm_batched(&r, idx, cb, x, 8, 8, y, 8, VQ_F16, nullptr) != VQ_OK);
      }
    }
    (void)before;
  }

  std::printf("launches checked: %lld\n", vq::stub_launch_count());
  if (g_failures) {
    std::printf("host check FAILED: %d expectations\n", g_failures);
    return 1;
  }
  std::printf("host check ok\n");
  return 0;
}
