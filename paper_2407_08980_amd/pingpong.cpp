// Post-to-done time of one message through the C ABI, without an interpreter in the loop: post the send and the
// recv, flush, poll the recv until it reports done (arXiv 2407.08980 Sec. 3.2: non-blocking operations whose status
// the worker polls; Sec. 4.3 measures small messages, where this time is the whole cost).
//
//   pingpong.bin [--iters N] [--sizes BYTES,BYTES,...] [--gap-us T]
//
// --gap-us leaves T microseconds between one message's completion and the next post (default 0: back to back); with a
// gap beyond the resident kernel's idle time every message finds it closed and has to start it.
//
// For every size, with small flushes served by the resident mailbox kernel and with every flush launched, it prints
// one JSON line: medians (and the 10th / 90th percentile of the total) of the three phases in microseconds.
// The payload is checked once per size.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../include/mw.h"

static double now() { return std::chrono::duration<double>(std::chrono::steady_clock::now().time_since_epoch()).count(); }

#define MW_CK(x)                                                        \
  do {                                                                  \
    int rc_ = (x);                                                      \
    if (rc_ < 0) {                                                      \
      std::fprintf(stderr, "%s: %s\n", #x, mw_strerror(rc_));           \
      return 1;                                                         \
    }                                                                   \
  } while (0)
#define HIP_CK(x)                                                       \
  do {                                                                  \
    hipError_t e_ = (x);                                                \
    if (e_ != hipSuccess) {                                             \
      std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));      \
      return 1;                                                         \
    }                                                                   \
  } while (0)

int main(int argc, char** argv) {
  int iters = 2000;
  double gap_us = 0.0;
  std::vector<size_t> sizes = {4096, 32768, 262144};
  for (int i = 1; i < argc; ++i) {
    if (!std::strcmp(argv[i], "--iters") && i + 1 < argc) {
      iters = std::max(10, std::atoi(argv[++i]));
    } else if (!std::strcmp(argv[i], "--gap-us") && i + 1 < argc) {
      gap_us = std::min(1e6, std::max(0.0, std::atof(argv[++i])));
    } else if (!std::strcmp(argv[i], "--sizes") && i + 1 < argc) {
      sizes.clear();
      std::string s = argv[++i];
      for (size_t at = 0; at < s.size();) {
        size_t end = s.find(',', at);
        if (end == std::string::npos) end = s.size();
        const long v = std::atol(s.substr(at, end - at).c_str());
        if (v < 4 || v % 4 != 0 || v > (1l << 30)) {
          std::fprintf(stderr, "sizes are multiples of 4 bytes up to 1 GiB\n");
          return 2;
        }
        sizes.push_back((size_t)v);
        at = end + 1;
      }
    } else {
      std::fprintf(stderr, "usage: %s [--iters N] [--sizes BYTES,BYTES,...] [--gap-us T]\n", argv[0]);
      return 2;
    }
  }
  size_t max_bytes = 0;
  for (size_t b : sizes) max_bytes = std::max(max_bytes, b);
  void *src = nullptr, *dst = nullptr;
  HIP_CK(hipSetDevice(0));
  HIP_CK(hipMalloc(&src, max_bytes));
  HIP_CK(hipMalloc(&dst, max_bytes));
  std::vector<unsigned char> pattern(max_bytes), back(max_bytes);
  for (size_t i = 0; i < max_bytes; ++i) pattern[i] = (unsigned char)(i * 131u + (i >> 8) * 17u + 5u);
  HIP_CK(hipMemcpy(src, pattern.data(), max_bytes, hipMemcpyHostToDevice));

  for (long mailbox = 1; mailbox >= 0; --mailbox) {
    MW_CK(mw_config_set("mailbox", mailbox));
    MW_CK(mw_init(0, 2));
    const int ids[2] = {0, 1};
    MW_CK(mw_world_create(0, ids, 2));
    for (size_t bytes : sizes) {
      HIP_CK(hipMemset(dst, 0, bytes));
      HIP_CK(hipDeviceSynchronize());
      std::vector<double> post((size_t)iters), flush((size_t)iters), wait((size_t)iters), total((size_t)iters);
      for (int k = -200; k < iters; ++k) {  // 200 untimed round trips first
        mw_handle hs = 0, hr = 0;
        const double t0 = now();
        MW_CK(mw_send(0, 0, 1, src, bytes / 4, MW_F32, MW_STREAM_NONE, &hs));
        MW_CK(mw_recv(0, 0, 1, dst, bytes / 4, MW_F32, MW_STREAM_NONE, &hr));
        const double t1 = now();
        MW_CK(mw_flush());
        const double t2 = now();
        int st;
        while ((st = mw_poll(hr)) == MW_PENDING) {
          if (now() - t2 > 10.0) {
            std::fprintf(stderr, "a message did not complete within 10 s\n");
            return 3;
          }
        }
        const double t3 = now();
        if (st != MW_DONE || mw_poll(hs) != MW_DONE) {
          std::fprintf(stderr, "a message ended as %s\n", mw_strerror(st));
          return 3;
        }
        if (k >= 0) post[(size_t)k] = t1 - t0, flush[(size_t)k] = t2 - t1, wait[(size_t)k] = t3 - t2, total[(size_t)k] = t3 - t0;
        if (gap_us > 0.0)
          while (now() - t3 < gap_us * 1e-6) {
          }
      }
      HIP_CK(hipMemcpy(back.data(), dst, bytes, hipMemcpyDeviceToHost));
      if (std::memcmp(back.data(), pattern.data(), bytes) != 0) {
        std::fprintf(stderr, "payload differs after %zu-byte messages\n", bytes);
        return 4;
      }
      auto pct = [](std::vector<double> v, double q) {
        std::sort(v.begin(), v.end());
        return v[(size_t)(q * (double)(v.size() - 1))] * 1e6;
      };
      std::printf("{\"bytes\": %zu, \"mailbox\": %ld, \"iters\": %d, \"gap_us\": %.0f, \"post_us\": %.2f, \"flush_us\": %.2f, \"wait_us\": %.2f, "
                  "\"total_us\": {\"median\": %.2f, \"p10\": %.2f, \"p90\": %.2f}}\n",
                  bytes, mailbox, iters, gap_us, pct(post, 0.5), pct(flush, 0.5), pct(wait, 0.5), pct(total, 0.5), pct(total, 0.1), pct(total, 0.9));
      std::fflush(stdout);
    }
    MW_CK(mw_shutdown());
  }
  (void)hipFree(src);
  (void)hipFree(dst);
  return 0;
}
