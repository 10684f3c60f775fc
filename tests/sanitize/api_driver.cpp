// Drives the host side of the C ABI (argument validation, size helpers, descriptor marshalling) with the kernel
// launchers replaced by stubs that only record that they were reached.  Built by tests/test_sanitizers.py from
// csrc/akvq_api.hip with AddressSanitizer and UndefinedBehaviorSanitizer on the host code; no GPU is touched and no
// pointer is dereferenced (the "device pointers" are fake, aligned addresses).  Prints "ok <launches>".
#include <cstdint>
#include <cstdio>
#include <cstdlib>

#include "../../include/akvq.h"
#include "../../paper_2501_15021_amd/csrc/akvq_kernels.h"

static int g_launches = 0;
namespace akvq {
hipError_t launch_quantize_append(const QuantArgs &a, int B, int G, hipStream_t) {
  if (a.n_blk <= 0 || a.first_blk < 0 || B <= 0 || (G != 64 && G != 128)) abort();
  ++g_launches; return hipSuccess;
}
hipError_t launch_decode_attention(const DecodeArgs &a, int G, hipStream_t) {
  if (a.n_split <= 0 || a.t_win < 0 || a.t_win > a.T_len || (G != 64 && G != 128)) abort();
  ++g_launches; return hipSuccess;
}
hipError_t decode_static_scratch(void **ptr) { *ptr = reinterpret_cast<void *>(0x7F0000100000ull); return hipSuccess; }
hipError_t launch_select_tsa(const SelectArgs &, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_select_psa(const SelectArgs &a, hipStream_t) { if (a.n_chunk <= 0) abort(); ++g_launches; return hipSuccess; }
hipError_t launch_select_massive(const SelectArgs &, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_fold_hadamard(const uint16_t *, uint16_t *, int, int, int, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_stream_read(const void *, size_t, uint32_t *, int, hipStream_t) { ++g_launches; return hipSuccess; }
}  // namespace akvq

#define EXPECT(call, want) do { int got_ = (call); if (got_ != (want)) { std::printf("line %d: got %d, want %d\n", __LINE__, got_, (want)); return 1; } } while (0)

int main() {
  void *P = reinterpret_cast<void *>(0x7F0000001000ull);
  uint32_t *P32 = static_cast<uint32_t *>(P); uint16_t *P16 = static_cast<uint16_t *>(P); int32_t *PI = static_cast<int32_t *>(P);
  auto cache = [&](int B, int Hkv, int G, int T_cap, int S_cap, int T_len) {
    akvq_cache c{B, Hkv, G, T_cap, S_cap, T_len, P32, P32, P32, P32, P16, P16, PI, PI};
    return c;
  };
  size_t sizes[8];
  // size helpers over a sweep of shapes, up to the largest the descriptor can express
  for (int B : {1, 3, 64, 2047}) for (int Hkv : {1, 4, 32}) for (int G : {64, 128}) for (int T_cap : {64, 4096, 1 << 20, 2147483584}) {
    akvq_cache c = cache(B, Hkv, G, T_cap, 64, 0);
    EXPECT(akvq_cache_bytes(&c, sizes), AKVQ_OK);
    if (sizes[0] != (size_t)B * Hkv * (size_t)(T_cap / 32) * 1024) return 2;
    (void)akvq_select_workspace_bytes(B, Hkv * 7, Hkv, T_cap, 64);
    (void)akvq_massive_workspace_bytes(B, T_cap);
    (void)akvq_decode_default_splits(B, Hkv, T_cap);
    for (int ns : {1, 5, 1024}) (void)akvq_decode_workspace_bytes(B, Hkv * 8, ns);
  }
  int b = 0, e = 0;
  for (int n_tiles = 0; n_tiles < 300; ++n_tiles) for (int ns = 1; ns < 40; ++ns) for (int s = 0; s < ns; ++s)
    if (akvq_decode_split_range(n_tiles, ns, s, &b, &e) < 0 || b > e || e > n_tiles) return 3;
  EXPECT(akvq_decode_split_range(2147483647, 1024, 1023, &b, &e) >= 0 ? 0 : 1, 0);
  for (int st = -7; st <= 1; ++st) if (!akvq_strerror(st)) return 4;
  (void)akvq_last_hip_error(); (void)akvq_version(); (void)akvq_decode_static_scratch_bytes();

  // every entry point once with well-formed arguments (reaches the stub), and the rejections around it
  akvq_cache c = cache(2, 2, 128, 256, 64, 100);
  akvq_window win{P16, P16, 64};
  akvq_rope rope{P16, P16, 64};
  const size_t big = (size_t)1 << 40;
  EXPECT(akvq_select_salient(&c, AKVQ_MODE_TSA, static_cast<const uint8_t *>(P), nullptr, 2, nullptr, 200, 0, 0, 0.f, nullptr, nullptr, 0, nullptr), AKVQ_OK);
  EXPECT(akvq_select_salient(&c, AKVQ_MODE_PSA, nullptr, P, 4, P, 200, 64, 16, 0.1f, nullptr, P, big, nullptr), AKVQ_OK);
  EXPECT(akvq_select_salient(&c, AKVQ_MODE_PSA_SHARED, nullptr, P, 4, P, 200, 16, 64, 0.1f, static_cast<float *>(P), P, big, nullptr), AKVQ_OK);
  EXPECT(akvq_select_salient(&c, AKVQ_MODE_PSA, nullptr, P, 4, P, 200, 64, 16, 0.1f, nullptr, P, 100, nullptr), AKVQ_ERR_WORKSPACE);
  EXPECT(akvq_select_massive(&c, P, 200, 1024, 15, 100.f, nullptr, P, big, nullptr), AKVQ_OK);
  EXPECT(akvq_fold_hadamard(P, static_cast<char *>(P) + 4096, 256, 128, 0, nullptr), AKVQ_OK);
  EXPECT(akvq_fold_hadamard(P, P, 256, 128, 1, nullptr), AKVQ_OK);
  EXPECT(akvq_quantize_append(&c, P, P, 156, 0.8f, 0, nullptr), AKVQ_OK);
  EXPECT(akvq_quantize_append(&c, P, P, 157, 0.8f, 0, nullptr), AKVQ_ERR_CAPACITY);
  EXPECT(akvq_quantize_append_tiered(&c, P, P, 50, PI, static_cast<const uint8_t *>(P), 60, 0.8f, 1.0f, P32, &win, AKVQ_V_PREROTATED, nullptr), AKVQ_OK);
  EXPECT(akvq_quantize_append_rope(&c, P, P, 50, nullptr, nullptr, 50, 0.8f, 1.0f, nullptr, nullptr, &rope, 0, nullptr), AKVQ_OK);
  EXPECT(akvq_quantize_append_rope(&c, P, P, 50, nullptr, nullptr, 51, 0.8f, 1.0f, nullptr, nullptr, &rope, 0, nullptr), AKVQ_ERR_INVALID_ARG);
  for (uint32_t flags : {0u, (uint32_t)AKVQ_OUT_ROTATED, (uint32_t)(AKVQ_OUT_FP16 | AKVQ_Q_PREROTATED)}) for (int ns : {0, 1, 7}) {
    EXPECT(akvq_decode_attention(&c, P, 14, 0.1f, P, static_cast<float *>(P), ns, P, big, flags, nullptr), AKVQ_OK);
    EXPECT(akvq_decode_attention_tiered(&c, P32, &win, P, 2, 0.1f, P, nullptr, ns, P, big, flags, nullptr), AKVQ_OK);
    EXPECT(akvq_decode_attention_static(&c, P, 2, 0.1f, P, nullptr, ns, flags, nullptr), AKVQ_OK);
  }
  EXPECT(akvq_decode_attention_rope(&c, nullptr, nullptr, P, &rope, 2, 0.1f, P, nullptr, 1, P, big, 0, nullptr), AKVQ_OK);
  EXPECT(akvq_decode_attention_static(&c, P, 16, 0.1f, P, nullptr, 1024, 0, nullptr), AKVQ_ERR_WORKSPACE);
  EXPECT(akvq_decode_step(&c, nullptr, &win, P, P, P, &rope, 4, 0.8f, 0.1f, P, nullptr, 3, P, big, 0, nullptr), AKVQ_OK);
  akvq_cache full = cache(2, 2, 128, 256, 64, 256);
  EXPECT(akvq_decode_step(&full, nullptr, nullptr, P, P, P, nullptr, 2, 0.8f, 0.1f, P, nullptr, 1, P, big, 0, nullptr), AKVQ_ERR_CAPACITY);
  EXPECT(akvq_stream_read(P, 1 << 20, P32, 1, nullptr), AKVQ_OK);
  akvq_cache huge = cache(2048, 32, 128, 64, 64, 1);
  EXPECT(akvq_decode_attention(&huge, P, 2048 * 32, 0.1f, P, nullptr, 1, P, big, 0, nullptr), AKVQ_ERR_UNSUPPORTED);
  std::printf("ok %d\n", g_launches);
  return 0;
}
