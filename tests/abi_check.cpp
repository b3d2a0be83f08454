// The C ABI used the way a C or C++ program uses it: no Python, no torch; device memory from the HIP runtime.
// Checks are against plain definitions (received == sent, sums of small integers), on purpose independent of
// everything else in the repository.  Exit status 0 = all checks passed.  Run by tests/test_gpu_abi_program.py.
#include <hip/hip_runtime_api.h>

#include <chrono>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../include/mw.h"

#define CHECK(cond)                                                              \
  do {                                                                           \
    if (!(cond)) {                                                               \
      std::fprintf(stderr, "abi_check: line %d: %s\n", __LINE__, #cond);         \
      std::fflush(stderr);                                                       \
      return 1;                                                                  \
    }                                                                            \
  } while (0)

static int wait_for(mw_handle h) {  // poll with a deadline; never blocks inside the library
  const auto t0 = std::chrono::steady_clock::now();
  for (;;) {
    int st = mw_poll(h);
    if (st != MW_PENDING) return st;
    if (std::chrono::steady_clock::now() - t0 > std::chrono::seconds(30)) return -1000;
  }
}

int main() {
  CHECK(hipSetDevice(0) == hipSuccess);
  CHECK(mw_poll(1) == MW_ENOTINIT);
  CHECK(mw_init(0, 4) == MW_OK);
  const int a[2] = {0, 1}, b[2] = {0, 2}, c[3] = {1, 2, 3};
  CHECK(mw_world_create(10, a, 2) == MW_OK);
  CHECK(mw_world_create(11, b, 2) == MW_OK);
  CHECK(mw_world_create(12, c, 3) == MW_OK);
  CHECK(mw_world_create(10, a, 2) == MW_EEXIST);

  // send / recv of 1 MiB + 6 bytes of bf16, unaligned by 2 bytes
  const size_t nbytes = (1u << 20) + 6;
  std::vector<uint8_t> host(nbytes), back(nbytes);
  uint32_t x = 12345;
  for (auto& v : host) v = (uint8_t)((x = x * 1664525u + 1013904223u) >> 24);
  uint8_t *src = nullptr, *dst = nullptr;
  CHECK(hipMalloc(reinterpret_cast<void**>(&src), nbytes + 2) == hipSuccess);
  CHECK(hipMalloc(reinterpret_cast<void**>(&dst), nbytes + 2) == hipSuccess);
  CHECK(hipMemcpy(src + 2, host.data(), nbytes, hipMemcpyHostToDevice) == hipSuccess);
  CHECK(hipMemset(dst, 0, nbytes + 2) == hipSuccess);
  CHECK(hipDeviceSynchronize() == hipSuccess);
  mw_handle hs = 0, hr = 0, lonely = 0;
  CHECK(mw_recv(11, 1, 0, dst, 4, MW_F32, MW_STREAM_NONE, &lonely) == MW_OK);  // its sender never arrives
  CHECK(mw_send(10, 1, 0, src + 2, nbytes / 2, MW_BF16, MW_STREAM_NONE, &hs) == MW_OK);
  CHECK(mw_poll(hs) == MW_PENDING);  // rendezvous: no receiver yet
  CHECK(mw_recv(10, 1, 0, dst + 2, nbytes / 2, MW_BF16, MW_STREAM_NONE, &hr) == MW_OK);
  CHECK(wait_for(hr) == MW_DONE && wait_for(hs) == MW_DONE);
  CHECK(mw_poll(lonely) == MW_PENDING);
  CHECK(hipMemcpy(back.data(), dst + 2, nbytes, hipMemcpyDeviceToHost) == hipSuccess);
  CHECK(std::memcmp(back.data(), host.data(), nbytes) == 0);

  // sum all-reduce among three ranks, integer-valued fp32: the sum is exact
  const size_t n = 100003;
  std::vector<float> in[3], out(n);
  float* dev[3];
  for (int r = 0; r < 3; ++r) {
    in[r].resize(n);
    for (size_t i = 0; i < n; ++i) in[r][i] = (float)((int)((i * 7 + r * 13) % 19) - 9);
    CHECK(hipMalloc(reinterpret_cast<void**>(&dev[r]), n * 4) == hipSuccess);
    CHECK(hipMemcpy(dev[r], in[r].data(), n * 4, hipMemcpyHostToDevice) == hipSuccess);
  }
  CHECK(hipDeviceSynchronize() == hipSuccess);
  mw_handle hc[3];
  for (int r = 2; r >= 0; --r) CHECK(mw_allreduce_sum(12, r, dev[r], n, MW_F32, MW_STREAM_NONE, &hc[r]) == MW_OK);
  for (int r = 0; r < 3; ++r) CHECK(wait_for(hc[r]) == MW_DONE);
  for (int r = 0; r < 3; ++r) {
    CHECK(hipMemcpy(out.data(), dev[r], n * 4, hipMemcpyDeviceToHost) == hipSuccess);
    for (size_t i = 0; i < n; ++i) CHECK(out[i] == in[0][i] + in[1][i] + in[2][i]);
  }

  // worker 2 fails: worlds 11 and 12 break, world 10 goes on
  CHECK(mw_worker_abort(2) == MW_OK);
  CHECK(mw_poll(lonely) == MW_BROKEN);
  CHECK(mw_world_state(11) == MW_BROKEN && mw_world_state(12) == MW_BROKEN && mw_world_state(10) == MW_ALIVE);
  CHECK(mw_send(11, 1, 0, src, 4, MW_F32, MW_STREAM_NONE, &hs) == MW_EBROKEN);
  CHECK(hipMemset(dst, 0, nbytes + 2) == hipSuccess);
  CHECK(hipDeviceSynchronize() == hipSuccess);
  CHECK(mw_send(10, 1, 0, src + 2, nbytes / 2, MW_BF16, MW_STREAM_NONE, &hs) == MW_OK);
  CHECK(mw_recv(10, 1, 0, dst + 2, nbytes / 2, MW_BF16, MW_STREAM_NONE, &hr) == MW_OK);
  CHECK(wait_for(hr) == MW_DONE);
  CHECK(hipMemcpy(back.data(), dst + 2, nbytes, hipMemcpyDeviceToHost) == hipSuccess);
  CHECK(std::memcmp(back.data(), host.data(), nbytes) == 0);

  CHECK(mw_shutdown() == MW_OK);
  for (int r = 0; r < 3; ++r) (void)hipFree(dev[r]);
  (void)hipFree(src);
  (void)hipFree(dst);
  std::printf("abi_check ok\n");
  return 0;
}
