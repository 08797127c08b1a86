// Driver for an AddressSanitizer + UndefinedBehaviorSanitizer build of the library's HOST code
// (argument checks, plan and workspace arithmetic, the host side of the hand-off).  Every
// sampling call below is rejected on the host before anything is enqueued -- the pointers that
// stand for device memory are never dereferenced and no kernel is launched -- so this runs
// without a GPU.  Exit code 0 and no sanitizer report is the test
// (tests/test_sanitizers_cpu.py builds and runs it).
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <thread>

#include "sip.h"
#include "sip_diag.h"

static int fails = 0;
#define EXPECT(cond)                                                     \
  do {                                                                   \
    if (!(cond)) { std::fprintf(stderr, "line %d: %s\n", __LINE__, #cond); ++fails; } \
  } while (0)

int main() {
  EXPECT(sip_version() > 0);
  for (int s = -2; s < 12; ++s) EXPECT(sip_status_string((sip_status)s) != nullptr);

  // sizes: every shape gives 0 or a multiple of 256; the arithmetic must not overflow
  const int32_t Bs[] = {-1, 0, 1, 3, 4, 64, 255, 256, 257, 600, 1024, 2048, 65536, INT32_MAX};
  const int32_t Vs[] = {-5, 0, 1, 1000, 16383, 16384, 32000, 70001, 129280, 152064, 262144, 262145, 1 << 20, INT32_MAX};
  const int64_t Ns[] = {-1, 0, 1, 100000, (int64_t)1 << 31, (int64_t)1 << 40};
  for (int32_t B : Bs)
    for (int32_t V : Vs)
      for (int dt = -1; dt <= 2; ++dt) {
        for (int64_t n : Ns)
          for (int32_t k : {-2, -1, 0, 20, 1 << 20}) {
            const size_t w = sip_workspace_bytes(B, V, (sip_dtype)dt, n, k);
            EXPECT(w % 256 == 0);
          }
        for (int32_t t = -1; t <= 9; ++t) {
          (void)sip_workspace_bytes_sharded(B, V, t, (sip_dtype)dt, 1000, 5);
          const int32_t S = sip_plan_chunks(B, V, (sip_dtype)dt, t);
          EXPECT(S >= -1 && S <= 16);
        }
      }
  for (int32_t slots : {-1, 0, 1, 256, 1 << 20, INT32_MAX})
    for (int32_t L : {-1, 0, 1, 1280, 1 << 20, INT32_MAX}) (void)sip_state_bytes(slots, L);
  EXPECT(sip_noalloc_scratch_bytes() > 0);

  // calls that the host rejects; 0x100000 stands for "some aligned device pointer"
  void* dev = reinterpret_cast<void*>(0x100000);
  int32_t* di = reinterpret_cast<int32_t*>(0x200000);
  float* df = reinterpret_cast<float*>(0x300000);
  const int64_t* dl = reinterpret_cast<const int64_t*>(0x400000);
  const size_t need = sip_workspace_bytes(8, 32000, SIP_F32, 0, 0);
  EXPECT(need > 0);
  EXPECT(sip_sample(nullptr, 8, 32000, 32000, SIP_F32, nullptr, nullptr, nullptr, 0, 1, 0, di, di, df, 0, dev, need, nullptr) == SIP_ERR_INVALID_ARG);
  EXPECT(sip_sample(dev, 0, 32000, 32000, SIP_F32, nullptr, nullptr, nullptr, 0, 1, 0, di, di, df, 0, dev, need, nullptr) == SIP_ERR_INVALID_ARG);
  EXPECT(sip_sample(dev, 8, 32000, 31999, SIP_F32, nullptr, nullptr, nullptr, 0, 1, 0, di, di, df, 0, dev, need, nullptr) == SIP_ERR_INVALID_ARG);
  EXPECT(sip_sample(dev, 8, 32000, 32000, (sip_dtype)7, nullptr, nullptr, nullptr, 0, 1, 0, di, di, df, 0, dev, need, nullptr) == SIP_ERR_INVALID_ARG);
  EXPECT(sip_sample(dev, 8, 32000, 32000, SIP_F32, nullptr, nullptr, nullptr, 5, 1, 0, di, di, df, 0, dev, need, nullptr) == SIP_ERR_INVALID_ARG);
  EXPECT(sip_sample(dev, 8, 32000, 32000, SIP_F32, nullptr, nullptr, nullptr, 0, 1, 0, nullptr, di, df, 0, dev, need, nullptr) == SIP_ERR_INVALID_ARG);
  EXPECT(sip_sample(dev, 8, 32000, 32000, SIP_F32, nullptr, nullptr, nullptr, 0, 1, 0, di, nullptr, df, 0, dev, need, nullptr) == SIP_ERR_INVALID_ARG);
  EXPECT(sip_sample(dev, 8, 32000, 32000, SIP_F32, nullptr, nullptr, nullptr, 0, 1, 0, di, di, df, 0, nullptr, need, nullptr) == SIP_ERR_WORKSPACE);
  EXPECT(sip_sample(dev, 8, 32000, 32000, SIP_F32, nullptr, nullptr, nullptr, 0, 1, 0, di, di, df, 0, dev, need - 1, nullptr) == SIP_ERR_WORKSPACE);
  EXPECT(sip_sample(dev, 8, 32000, 32000, SIP_F32, nullptr, nullptr, nullptr, 0, 1, 0, di, di, df, 0,
                    reinterpret_cast<void*>(0x100010), need, nullptr) == SIP_ERR_WORKSPACE);
  EXPECT(sip_sample(dev, 8, 1 << 24, 1 << 24, SIP_F32, nullptr, nullptr, nullptr, 0, 1, 0, di, di, df, 0, dev, (size_t)1 << 40, nullptr) == SIP_ERR_UNSUPPORTED);
  EXPECT(sip_sample_noalloc(nullptr, 8, 32000, 32000, SIP_F32, nullptr, nullptr, nullptr, 0, 1, 0, di, di, df, 0, nullptr) == SIP_ERR_INVALID_ARG);

  const void* pieces[9] = {dev, dev, dev, dev, dev, dev, dev, dev, dev};
  EXPECT(sip_sample_sharded(pieces, 9, 8, 16384, 16384, SIP_F32, nullptr, nullptr, nullptr, 0, 1, 0, di, di, df, 0, dev, (size_t)1 << 30, nullptr) != SIP_OK);
  EXPECT(sip_sample_sharded(nullptr, 2, 8, 16384, 16384, SIP_F32, nullptr, nullptr, nullptr, 0, 1, 0, di, di, df, 0, dev, (size_t)1 << 30, nullptr) == SIP_ERR_INVALID_ARG);
  EXPECT(sip_sample_sharded(pieces, 2, 8, 16383, 16383, SIP_BF16, nullptr, nullptr, nullptr, 0, 1, 0, di, di, df, 0, dev, (size_t)1 << 30, nullptr) == SIP_ERR_INVALID_ARG);

  EXPECT(sip_state_init(nullptr, 1 << 20, 4, 16, nullptr) != SIP_OK);
  EXPECT(sip_state_init(dev, 16, 4, 16, nullptr) != SIP_OK);
  EXPECT(sip_state_assign(dev, 16, 4, 16, 1, di, dl, di, 0, nullptr) != SIP_OK);
  EXPECT(sip_sample_state(dev, 8, 32000, 32000, SIP_F32, nullptr, dev, 16, 4, 16, di, 1, 0, di, di, df, 0, dev, need, nullptr) != SIP_OK);

  sip_call c;
  std::memset(&c, 0, sizeof c);
  EXPECT(sip_sample_call(nullptr) == SIP_ERR_INVALID_ARG);
  EXPECT(sip_call_workspace_bytes(nullptr) == 0);
  EXPECT(sip_sample_call(&c) != SIP_OK);
  c.logits = dev; c.row_stride = 32000; c.V = 32000; c.B = 8; c.dtype = SIP_F32; c.out_ids = di; c.k_logprobs = -1;
  c.workspace = dev;
  c.prompt_nnz = -3;
  EXPECT(sip_sample_call(&c) == SIP_ERR_INVALID_ARG);
  c.prompt_nnz = 10;                       // prompt arrays missing
  EXPECT(sip_sample_call(&c) == SIP_ERR_INVALID_ARG);
  c.prompt_indptr = dl; c.prompt_tokens = di;
  EXPECT(sip_call_workspace_bytes(&c) >= sip_workspace_bytes(8, 32000, SIP_F32, 10, -1));
  c.workspace_bytes = 16;
  EXPECT(sip_sample_call(&c) == SIP_ERR_WORKSPACE);
  c.host_ids = di;                         // a flag without... one of the two hand-off pointers
  EXPECT(sip_sample_call(&c) != SIP_OK);

  // the host side of the hand-off
  uint64_t flag = 7;
  EXPECT(sip_wait_ids(&flag, 7, 0) == SIP_OK);
  EXPECT(sip_wait_ids(&flag, 3, 0) == SIP_OK);
  EXPECT(sip_wait_ids(&flag, 8, 2000000) == SIP_ERR_TIMEOUT);
  EXPECT(sip_wait_ids(nullptr, 8, 1000) == SIP_ERR_INVALID_ARG);
  std::thread setter([&] {
    std::this_thread::sleep_for(std::chrono::milliseconds(5));
    __atomic_store_n(&flag, (uint64_t)9, __ATOMIC_RELEASE);
  });
  EXPECT(sip_wait_ids(&flag, 9, 2000000000ull) == SIP_OK);
  setter.join();
  EXPECT(sip_publish_ids(nullptr, 8, di, &flag, 1, nullptr) == SIP_ERR_INVALID_ARG);
  EXPECT(sip_probe_read(nullptr, 0, 0, nullptr, 0, nullptr, nullptr, nullptr) != SIP_OK);

  if (fails) { std::fprintf(stderr, "%d expectation(s) failed\n", fails); return 1; }
  std::puts("ok");
  return 0;
}
