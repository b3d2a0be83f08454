// Post-to-done time of one message through the C ABI, without an interpreter in the loop: post the send and the
// recv, flush, poll the recv until it reports done (arXiv 2407.08980 Sec. 3.2: non-blocking operations whose status
// the worker polls; Sec. 4.3 measures small messages, where this time is the whole cost).
//
//   pingpong.bin [--iters N] [--sizes BYTES,BYTES,...] [--gap-us T]
//   pingpong.bin --tp [--iters N]
//   pingpong.bin --windows [--iters N]
//
// --gap-us leaves T microseconds between one message's completion and the next post (default 0: back to back); with a
// gap beyond the resident kernel's idle time every message finds it closed and has to start it.
//
// For every size, with small flushes served by the resident mailbox kernel and with every flush launched, it prints
// one JSON line: medians (and the 10th / 90th percentile of the total) of the three phases in microseconds.
// The payload is checked once per size.
//
// --tp runs the tensor-parallel partial-sum loop instead (Sec. 3.1's tensor-parallel stages; 4 worlds x 4 ranks, per
// iteration every world all-reduces fp32 [16,4096] and [16,14336], inputs U(-1,1)): 1 to 4 iterations in flight, both
// forms, one JSON line each with the microseconds per iteration.  Results are not checked here (the parity tests do).
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

// The tensor-parallel loop: `depth` iterations in flight, each on input buffers of its own (4 sets).
static int tensor_parallel_loop(int iters) {
  const int n_worlds = 4, n_ranks = 4, n_sets = 4;
  const size_t counts[2] = {16 * 4096, 16 * 14336};
  std::vector<float> host(counts[1]);
  unsigned long long x = 88172645463325252ull;  // xorshift64: inputs in (-1, 1)
  std::vector<std::vector<mw_post_desc>> posts((size_t)n_sets);
  std::vector<void*> bufs;
  HIP_CK(hipSetDevice(0));
  for (int k = 0; k < n_sets; ++k)
    for (int j = 0; j < 2; ++j)
      for (int w = 0; w < n_worlds; ++w)
        for (int r = 0; r < n_ranks; ++r) {
          for (size_t i = 0; i < counts[j]; ++i) {
            x ^= x << 13, x ^= x >> 7, x ^= x << 17;
            host[i] = (float)((double)(x >> 11) / 4503599627370496.0 - 1.0);
          }
          void* p = nullptr;
          HIP_CK(hipMalloc(&p, counts[j] * 4));
          HIP_CK(hipMemcpy(p, host.data(), counts[j] * 4, hipMemcpyHostToDevice));
          bufs.push_back(p);
          mw_post_desc d{};
          d.kind = MW_POST_ALLREDUCE_SUM, d.world_id = w, d.a = r, d.buf = p, d.count = counts[j], d.dtype = MW_F32, d.hip_stream = MW_STREAM_NONE;
          posts[(size_t)k].push_back(d);
        }
  HIP_CK(hipDeviceSynchronize());
  const int n_posts = (int)posts[0].size();
  for (long mailbox = 1; mailbox >= 0; --mailbox) {
    MW_CK(mw_config_set("mailbox", mailbox));
    MW_CK(mw_init(0, n_worlds * n_ranks));
    for (int w = 0; w < n_worlds; ++w) {
      int ids[4];
      for (int r = 0; r < n_ranks; ++r) ids[r] = w * n_ranks + r;
      MW_CK(mw_world_create(w, ids, n_ranks));
    }
    std::vector<std::vector<mw_handle>> h((size_t)n_sets, std::vector<mw_handle>((size_t)n_posts));
    std::vector<int> res((size_t)n_posts), st((size_t)n_posts);
    for (int depth = 1; depth <= n_sets; ++depth) {
      double us = 0.0;
      for (int pass = 0; pass < 2; ++pass) {  // the first pass is the warm-up
        const int n = pass == 0 ? 200 : iters;
        const double t0 = now();
        for (int it = 0; it < n; ++it) {
          const size_t k = (size_t)(it % n_sets);
          if (it >= depth) {  // the iteration that used this depth's slot must be done (it is the one whose buffers come up next)
            const size_t o = (size_t)((it - depth) % n_sets);
            int pending;
            while ((pending = mw_poll_many(h[o].data(), n_posts, st.data())) > 0) {
              if (now() - t0 > 30.0) {
                std::fprintf(stderr, "the loop did not make progress\n");
                return 3;
              }
            }
            MW_CK(pending);
          }
          MW_CK(mw_post_many(posts[k].data(), n_posts, h[k].data(), res.data()));
          MW_CK(mw_flush());
        }
        for (size_t o = 0; o < (size_t)n_sets; ++o)
          while (mw_poll_many(h[o].data(), n_posts, st.data()) > 0) {
            if (now() - t0 > 30.0) return 3;
          }
        us = (now() - t0) / n * 1e6;
      }
      std::printf("{\"workload\": \"tp\", \"mailbox\": %ld, \"iterations_in_flight\": %d, \"iters\": %d, \"us_per_iteration\": %.2f}\n", mailbox, depth, iters, us);
      std::fflush(stdout);
    }
    MW_CK(mw_shutdown());
  }
  for (void* p : bufs) (void)hipFree(p);
  return 0;
}

// Windows of 16 messages of 32 KiB, alternating between two worlds that share worker 0.
static int window_loop(int iters) {
  const int window = 16, n_sets = 2;
  const size_t bytes = 32768;
  std::vector<unsigned char> pattern(bytes), back(bytes);
  for (size_t i = 0; i < bytes; ++i) pattern[i] = (unsigned char)(i * 29u + (i >> 7) * 13u + 3u);
  HIP_CK(hipSetDevice(0));
  std::vector<std::vector<mw_post_desc>> posts((size_t)n_sets);
  std::vector<void*> bufs, dsts;
  for (int k = 0; k < n_sets; ++k)
    for (int m = 0; m < window; ++m) {
      void *src = nullptr, *dst = nullptr;
      HIP_CK(hipMalloc(&src, bytes));
      HIP_CK(hipMalloc(&dst, bytes));
      HIP_CK(hipMemcpy(src, pattern.data(), bytes, hipMemcpyHostToDevice));
      HIP_CK(hipMemset(dst, 0, bytes));
      bufs.push_back(src), bufs.push_back(dst), dsts.push_back(dst);
      mw_post_desc d{};
      d.world_id = m % 2, d.a = 1, d.b = 0, d.count = bytes / 4, d.dtype = MW_F32, d.hip_stream = MW_STREAM_NONE;
      d.kind = MW_POST_SEND, d.buf = src;
      posts[(size_t)k].push_back(d);
      d.kind = MW_POST_RECV, d.buf = dst;
      posts[(size_t)k].push_back(d);
    }
  HIP_CK(hipDeviceSynchronize());
  const int n_posts = 2 * window;
  for (long mailbox = 1; mailbox >= 0; --mailbox) {
    MW_CK(mw_config_set("mailbox", mailbox));
    MW_CK(mw_init(0, 3));
    const int a[2] = {0, 1}, b[2] = {0, 2};
    MW_CK(mw_world_create(0, a, 2));
    MW_CK(mw_world_create(1, b, 2));
    std::vector<std::vector<mw_handle>> h((size_t)n_sets, std::vector<mw_handle>((size_t)n_posts));
    std::vector<int> res((size_t)n_posts), st((size_t)n_posts);
    for (int depth = 1; depth <= n_sets; ++depth) {
      double us = 0.0;
      for (int pass = 0; pass < 2; ++pass) {  // the first pass is the warm-up
        const int n = pass == 0 ? 200 : iters;
        const double t0 = now();
        for (int it = 0; it < n; ++it) {
          const size_t k = (size_t)(it % n_sets);
          if (it >= depth) {
            const size_t o = (size_t)((it - depth) % n_sets);
            while (mw_poll_many(h[o].data(), n_posts, st.data()) > 0) {
              if (now() - t0 > 30.0) {
                std::fprintf(stderr, "the loop did not make progress\n");
                return 3;
              }
            }
          }
          MW_CK(mw_post_many(posts[k].data(), n_posts, h[k].data(), res.data()));
          MW_CK(mw_flush());
        }
        for (size_t o = 0; o < (size_t)n_sets; ++o)
          while (mw_poll_many(h[o].data(), n_posts, st.data()) > 0) {
            if (now() - t0 > 30.0) return 3;
          }
        us = (now() - t0) / n / window * 1e6;
      }
      std::printf("{\"workload\": \"windows\", \"mailbox\": %ld, \"windows_in_flight\": %d, \"window\": %d, \"iters\": %d, \"us_per_message\": %.3f}\n",
                  mailbox, depth, window, iters, us);
      std::fflush(stdout);
    }
    MW_CK(mw_shutdown());
  }
  for (void* d : dsts) {
    HIP_CK(hipMemcpy(back.data(), d, bytes, hipMemcpyDeviceToHost));
    if (std::memcmp(back.data(), pattern.data(), bytes) != 0) {
      std::fprintf(stderr, "payload differs\n");
      return 4;
    }
  }
  for (void* p : bufs) (void)hipFree(p);
  return 0;
}

int main(int argc, char** argv) {
  int iters = 2000;
  bool tp = false, windows = false;
  double gap_us = 0.0;
  std::vector<size_t> sizes = {4096, 32768, 262144};
  for (int i = 1; i < argc; ++i) {
    if (!std::strcmp(argv[i], "--tp")) {
      tp = true;
    } else if (!std::strcmp(argv[i], "--windows")) {
      windows = true;
    } else if (!std::strcmp(argv[i], "--iters") && i + 1 < argc) {
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
      std::fprintf(stderr, "usage: %s [--iters N] [--sizes BYTES,BYTES,...] [--gap-us T] | --tp [--iters N] | --windows [--iters N]\n", argv[0]);
      return 2;
    }
  }
  if (tp) return tensor_parallel_loop(iters);
  if (windows) return window_loop(iters);
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
