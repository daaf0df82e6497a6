// Host-side exerciser for libdfa's C ABI, built with AddressSanitizer + UndefinedBehaviorSanitizer on
// the HOST code only (tests/test_host_sanitizers.py compiles and runs it; no GPU is needed: every
// call here either is a pure host function or fails validation before anything is launched).
// Buffers are heap blocks of exactly the size a call may touch, so a write past the end is caught.
#include <climits>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "dfa.h"

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

static dfa_shape base_shape() {
  dfa_shape sh;
  std::memset(&sh, 0, sizeof(sh));
  sh.h_q = 2; sh.h_kv = 2; sh.s_q = 64; sh.s_k = 64; sh.d = 64; sh.dtype = DFA_F32; sh.o_dtype = DFA_F32;
  sh.causal = 0; sh.scale = 0.125f; sh.reserved = 0;
  sh.q_stride_h = 64 * 64; sh.q_stride_s = 64; sh.kv_stride_h = 64 * 64; sh.kv_stride_s = 64;
  sh.o_stride_h = 64 * 64; sh.o_stride_s = 64; sh.lse_stride_h = 64;
  sh.dq_stride_h = 64 * 64; sh.dq_stride_s = 64; sh.dkv_stride_h = 64 * 64; sh.dkv_stride_s = 64;
  return sh;
}

int main() {
  // ---- schedules: exact-size and truncated output buffers, every worker, P = 1..64
  for (int P = 1; P <= 64; ++P) {
    for (int w = 0; w < P; ++w) {
      for (int mode = 0; mode < 2; ++mode) {
        const int n = dfa_schedule_mode(mode, P, w, nullptr, 0);
        EXPECT(n == (mode == DFA_SCHED_BALANCED ? 1 + P / 2 : P));
        for (int cap : {n, n - 1, 1}) {
          if (cap < 1) continue;
          dfa_step* buf = static_cast<dfa_step*>(std::malloc(sizeof(dfa_step) * cap));
          EXPECT(dfa_schedule_mode(mode, P, w, buf, cap) == n);
          EXPECT(buf[0].kind == DFA_STEP_DIAG && buf[0].q_chunk == w && buf[0].kv_chunk == w);
          for (int t = 0; t < cap && t < n; ++t) {
            EXPECT(buf[t].t == t);
            EXPECT(buf[t].q_chunk >= -1 && buf[t].q_chunk < P && buf[t].kv_chunk >= -1 && buf[t].kv_chunk < P);
            EXPECT(buf[t].kv_chunk <= buf[t].q_chunk);
          }
          std::free(buf);
        }
      }
      for (int W : {0, 1, P - 1, P + 3}) {
        const int n = dfa_schedule_window(P, w, W, nullptr, 0);
        EXPECT(n == 1 + (W < P - 1 ? W : P - 1));
        dfa_step* buf = static_cast<dfa_step*>(std::malloc(sizeof(dfa_step) * n));
        EXPECT(dfa_schedule_window(P, w, W, buf, n) == n);
        std::free(buf);
      }
    }
  }
  EXPECT(dfa_schedule(0, 0, nullptr, 0) == DFA_ERR_ARG);
  EXPECT(dfa_schedule(INT32_MAX, INT32_MAX - 1, nullptr, 0) == 1 + INT32_MAX / 2);
  EXPECT(dfa_schedule_mode(DFA_SCHED_RING, INT32_MAX, 0, nullptr, 0) == INT32_MAX);
  EXPECT(dfa_schedule_window(INT32_MAX, 5, INT32_MAX, nullptr, 0) == INT32_MAX);
  EXPECT(dfa_schedule(4, 1, nullptr, 3) == DFA_ERR_NULL);
  EXPECT(dfa_schedule(4, 1, nullptr, -1) == DFA_ERR_ARG);

  // ---- argument validation: nothing is launched, the fake pointers are never dereferenced
  void* fake = reinterpret_cast<void*>(uintptr_t{4096});
  float* ffake = static_cast<float*>(fake);
  {
    dfa_shape sh = base_shape();
    // extreme strides and sizes must be refused by comparison, not by overflowing arithmetic
    for (int64_t big : {int64_t{1} << 29, int64_t{1} << 40, (int64_t{1} << 62), INT64_MAX - 7, INT64_MAX}) {
      dfa_shape s2 = sh; s2.q_stride_s = big;
      EXPECT(dfa_chunk_fwd(&s2, fake, fake, fake, fake, ffake, nullptr) == DFA_ERR_SHAPE);
      s2 = sh; s2.kv_stride_h = big;
      const int rc = dfa_chunk_fwd(&s2, fake, fake, fake, fake, ffake, nullptr);
      EXPECT(rc == DFA_ERR_SHAPE || (big % 8 == 0 && rc != DFA_OK) || rc == DFA_ERR_SHAPE);
      s2 = sh; s2.s_q = INT32_MAX; s2.lse_stride_h = INT64_MAX; s2.q_stride_s = big;
      EXPECT(dfa_chunk_bwd(&s2, fake, fake, fake, ffake, ffake, fake, ffake, ffake, ffake, 0, nullptr) == DFA_ERR_SHAPE);
      s2 = sh; s2.s_k = INT32_MAX; s2.dkv_stride_s = big;
      EXPECT(dfa_chunk_bwd(&s2, fake, fake, fake, ffake, ffake, fake, ffake, ffake, ffake, 0, nullptr) == DFA_ERR_SHAPE);
      dfa_merge_desc md;
      std::memset(&md, 0, sizeof(md));
      md.heads = 2; md.rows = INT32_MAX; md.d = 128; md.o_dtype = DFA_F32;
      md.a_stride_h = big; md.a_stride_s = big; md.lse_a_stride_h = INT64_MAX;
      md.b_stride_h = big; md.b_stride_s = big; md.lse_b_stride_h = INT64_MAX;
      EXPECT(dfa_merge(&md, fake, ffake, reinterpret_cast<void*>(uintptr_t{8192}),
                       reinterpret_cast<float*>(uintptr_t{8192}), nullptr) == DFA_ERR_SHAPE);
    }
    dfa_shape s3 = sh; s3.scale = std::nanf("");
    EXPECT(dfa_chunk_fwd(&s3, fake, fake, fake, fake, ffake, nullptr) == DFA_ERR_ARG);
    s3 = sh; s3.scale = -1.f;
    EXPECT(dfa_chunk_fwd_acc(&s3, fake, fake, fake, fake, ffake, nullptr) == DFA_ERR_ARG);
    s3 = sh; s3.h_q = INT32_MAX; s3.h_kv = 1;
    EXPECT(dfa_chunk_fwd(&s3, fake, fake, fake, fake, ffake, nullptr) == DFA_ERR_SHAPE);
    s3 = sh; s3.s_q = 0; s3.lse_stride_h = 0;
    EXPECT(dfa_chunk_fwd(&s3, fake, fake, fake, fake, ffake, nullptr) == DFA_OK);       // empty query chunk: no-op
    EXPECT(dfa_delta(&s3, fake, fake, ffake, nullptr) == DFA_OK);
    EXPECT(dfa_delta(&sh, fake, nullptr, ffake, nullptr) == DFA_ERR_NULL);
    EXPECT(dfa_chunk_fwd(nullptr, fake, fake, fake, fake, ffake, nullptr) == DFA_ERR_NULL);
  }
  {
    double flop = -1.0;
    EXPECT(dfa_mfma_probe(nullptr, 1 << 20, 10, &flop, nullptr) == DFA_ERR_NULL);
    EXPECT(dfa_mfma_probe(ffake, 1 << 20, INT32_MIN, &flop, nullptr) == DFA_ERR_ARG);
    EXPECT(dfa_mfma_probe_data(fake, INT64_MAX, ffake, 10, 10, &flop, nullptr) == DFA_ERR_ARG);
    EXPECT(dfa_mfma_probe_data(fake, -1, ffake, 1 << 20, 10, &flop, nullptr) == DFA_ERR_ARG);
    EXPECT(flop == -1.0);
  }
  for (int s = -8; s <= 1; ++s) EXPECT(dfa_status_str(s) != nullptr && std::strlen(dfa_status_str(s)) > 0);
  EXPECT(dfa_version() >= 100);
  std::printf(failures ? "host sanitizer driver: %d check(s) FAILED\n" : "host sanitizer driver: ok\n", failures);
  return failures ? 1 : 0;
}
