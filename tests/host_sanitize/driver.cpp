// Exercises the host side of every C-ABI entry point (validation, overlap checks, workspace layout, dispatch) with
// the kernel launchers stubbed out (stubs.cpp), for a build with -fsanitize=address,undefined.  Pointers are fake
// addresses: nothing dereferences them on the host.  Exit status 0 = every expectation held; the sanitizers abort
// the process on their own findings.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>

#include "../../include/tvmattn.h"

extern int g_stub_launches;
static int fails = 0;
#define EXPECT(cond)                                             \
  do {                                                           \
    if (!(cond)) {                                               \
      ++fails;                                                   \
      std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); \
    }                                                            \
  } while (0)

static void* P(uint64_t a) { return reinterpret_cast<void*>(a); }

static tvmattn_desc mk(int B, int H, int N, int D, int dtype = TVMATTN_BF16, int M = 0) {
  tvmattn_desc d{};
  d.B = B; d.H = H; d.N = N; d.D = D; d.dtype = dtype; d.M = M;
  return d;
}

int main() {
  const uint64_t G = 0x100000000ull;  // 4 GiB between fake buffers
  // ---- forward
  tvmattn_desc d = mk(2, 3, 100, 72);
  EXPECT(tvmattn_jvp_fwd(&d, P(G), P(2 * G), P(3 * G), P(4 * G), P(5 * G), P(6 * G), P(7 * G), P(8 * G), (float*)P(9 * G),
                         (float*)P(10 * G), nullptr) == TVMATTN_OK);
  EXPECT(g_stub_launches == 1);
  EXPECT(tvmattn_jvp_fwd(&d, P(G), P(2 * G), P(3 * G), P(4 * G), P(5 * G), P(6 * G), P(G + 64), P(8 * G), (float*)P(9 * G),
                         (float*)P(10 * G), nullptr) == TVMATTN_INVALID_ARG);
  EXPECT(tvmattn_jvp_fwd(nullptr, P(G), P(2 * G), P(3 * G), P(4 * G), P(5 * G), P(6 * G), P(7 * G), P(8 * G), nullptr, nullptr,
                         nullptr) == TVMATTN_INVALID_ARG);
  // extreme descriptors: nothing may overflow on the way to the verdict
  for (int B : {1, 65535, INT32_MAX})
    for (int N : {1, 4096, INT32_MAX})
      for (int D : {1, 8, 256, 257, INT32_MAX})
        for (int64_t st : {(int64_t)0, (int64_t)8, (int64_t)1 << 40, INT64_MAX / 4}) {
          tvmattn_desc e = mk(B, 16, N, D);
          e.stride_b = st; e.stride_h = st; e.stride_n = st;
          e.M = N / 2;
          (void)tvmattn_jvp_bwd_workspace_bytes(&e);
          (void)tvmattn_jvp_fwd(&e, P(G), P(2 * G), P(3 * G), P(4 * G), P(5 * G), P(6 * G), P(7 * G), P(8 * G), (float*)P(9 * G),
                                (float*)P(10 * G), nullptr);
        }
  // ---- norm + forward in one call: a valid call is two launches; the same extreme descriptors
  {
    const int before = g_stub_launches;
    EXPECT(tvmattn_jvp_fwd_qknorm(&d, P(G), P(2 * G), P(3 * G), P(4 * G), (const float*)P(5 * G), (const float*)P(6 * G), 1e-6f,
                                  P(7 * G), P(8 * G), P(9 * G), P(10 * G), P(11 * G), P(12 * G), P(13 * G), P(14 * G),
                                  (float*)P(15 * G), (float*)P(16 * G), nullptr) == TVMATTN_OK);
    EXPECT(g_stub_launches == before + 2);
    EXPECT(tvmattn_jvp_fwd_qknorm(&d, P(G), P(2 * G), P(3 * G), P(4 * G), (const float*)P(5 * G), (const float*)P(6 * G), 1e-6f,
                                  P(7 * G), P(8 * G), P(9 * G), P(10 * G), P(11 * G), P(3 * G + 32), P(13 * G), P(14 * G),
                                  (float*)P(15 * G), (float*)P(16 * G), nullptr) == TVMATTN_INVALID_ARG);  // tkn inside k
    for (int B : {1, 65535, INT32_MAX})
      for (int N : {1, 4096, INT32_MAX})
        for (int D : {8, 128, 136, INT32_MAX})
          for (int64_t st : {(int64_t)0, (int64_t)8, (int64_t)1 << 40, INT64_MAX / 4}) {
            tvmattn_desc e = mk(B, 16, N, D);
            e.stride_b = st; e.stride_h = st; e.stride_n = st;
            e.M = N / 2;
            (void)tvmattn_jvp_fwd_qknorm(&e, P(G), P(2 * G), P(3 * G), P(4 * G), (const float*)P(5 * G), (const float*)P(6 * G),
                                         1e-6f, P(7 * G), P(8 * G), P(9 * G), P(10 * G), P(11 * G), P(12 * G), P(13 * G),
                                         P(14 * G), (float*)P(15 * G), (float*)P(16 * G), nullptr);
          }
  }
  // ---- backward: workspace contract, one-sided calls, the timed variant
  const size_t need = tvmattn_jvp_bwd_workspace_bytes(&d);
  EXPECT(need >= 3u * 2 * 3 * 100 * 4 && need % 256 == 0);
  auto bwd = [&](const void* gO, const void* gTO, void* ws, size_t wsb, void* dk) {
    return tvmattn_jvp_bwd(&d, P(G), P(2 * G), P(3 * G), P(4 * G), P(5 * G), P(6 * G), P(7 * G), P(8 * G), (float*)P(9 * G),
                           (float*)P(10 * G), gO, gTO, P(13 * G), dk, P(15 * G), P(16 * G), P(17 * G), P(18 * G), ws, wsb,
                           nullptr);
  };
  int before = g_stub_launches;
  EXPECT(bwd(P(11 * G), P(12 * G), P(19 * G), need, P(14 * G)) == TVMATTN_OK);
  EXPECT(g_stub_launches == before + 2);
  EXPECT(bwd(P(11 * G), P(12 * G), P(19 * G), need - 1, P(14 * G)) == TVMATTN_WORKSPACE_TOO_SMALL);
  EXPECT(bwd(nullptr, nullptr, P(19 * G), need, P(14 * G)) == TVMATTN_INVALID_ARG);
  EXPECT(bwd(P(11 * G), nullptr, P(19 * G), need, P(14 * G)) == TVMATTN_OK);
  EXPECT(bwd(nullptr, P(12 * G), P(19 * G), need, P(14 * G)) == TVMATTN_OK);
  EXPECT(bwd(P(11 * G), P(12 * G), nullptr, need, P(14 * G)) == TVMATTN_INVALID_ARG);
  EXPECT(bwd(P(11 * G), P(12 * G), P(19 * G), need, P(13 * G + 1024)) == TVMATTN_INVALID_ARG);  // dk inside dq
  EXPECT(bwd(P(11 * G), P(12 * G), P(14 * G + 256), need, P(14 * G)) == TVMATTN_INVALID_ARG);   // workspace inside dk
  void* ev[4] = {nullptr, nullptr, nullptr, nullptr};
  EXPECT(tvmattn_jvp_bwd_timed(&d, P(G), P(2 * G), P(3 * G), P(4 * G), P(5 * G), P(6 * G), P(7 * G), P(8 * G), (float*)P(9 * G),
                               (float*)P(10 * G), P(11 * G), P(12 * G), P(13 * G), P(14 * G), P(15 * G), P(16 * G), P(17 * G),
                               P(18 * G), P(19 * G), need, ev, nullptr) == TVMATTN_OK);
  d.flags = TVMATTN_FLAG_PLAIN_ALU;
  before = g_stub_launches;
  EXPECT(bwd(P(11 * G), P(12 * G), P(19 * G), need, P(14 * G)) == TVMATTN_OK);
  EXPECT(g_stub_launches == before + 3);  // the plain-ALU path has a separate row-scalar launch
  d.flags = 4;
  EXPECT(bwd(P(11 * G), P(12 * G), P(19 * G), need, P(14 * G)) == TVMATTN_INVALID_ARG);
  d.flags = 0;
  // ---- static-scratch backward: size limit first; without a GPU the device query fails cleanly
  tvmattn_desc big = mk(16, 16, 4097, 64);
  EXPECT(tvmattn_jvp_bwd_static(&big, P(G), P(2 * G), P(3 * G), P(4 * G), P(5 * G), P(6 * G), P(7 * G), P(8 * G),
                                (float*)P(9 * G), (float*)P(10 * G), P(11 * G), P(12 * G), P(13 * G), P(14 * G), P(15 * G),
                                P(16 * G), P(17 * G), P(18 * G), nullptr) == TVMATTN_SCRATCH_TOO_SMALL);
  const int rs = tvmattn_jvp_bwd_static(&d, P(G), P(2 * G), P(3 * G), P(4 * G), P(5 * G), P(6 * G), P(7 * G), P(8 * G),
                                        (float*)P(9 * G), (float*)P(10 * G), P(11 * G), P(12 * G), P(13 * G), P(14 * G),
                                        P(15 * G), P(16 * G), P(17 * G), P(18 * G), nullptr);
  EXPECT(rs == TVMATTN_OK || rs == TVMATTN_LAUNCH_FAILED);
  // ---- the overlap check on random strided layouts: two tensors of one layout share an element exactly when a
  // brute-force walk over their elements says so
  std::mt19937 rng(2511);
  for (int it = 0; it < 400; ++it) {
    const int B = 1 + rng() % 2, H = 1 + rng() % 3, N = 1 + rng() % 5, D = 8 * (1 + rng() % 2);
    // a [B,N,3,H,D] fused buffer viewed as [B,H,N,D], or a dense [B,H,N,D] tensor
    const bool fused = rng() % 2;
    tvmattn_desc e = mk(B, H, N, D);
    if (fused) { e.stride_n = 3 * H * D; e.stride_h = D; e.stride_b = (int64_t)N * 3 * H * D; }
    const int64_t sn = fused ? 3 * H * D : D, sh = fused ? D : (int64_t)N * D, sb = fused ? (int64_t)N * 3 * H * D : (int64_t)H * N * D;
    const int64_t delta_el = 8 * (int64_t)(rng() % (3 * B * H * N * D / 8 + 4));  // dq..dk distance in elements, 16-byte steps
    bool hit = false;
    for (int b = 0; b < B && !hit; ++b) for (int h = 0; h < H && !hit; ++h) for (int n = 0; n < N && !hit; ++n)
      for (int b2 = 0; b2 < B && !hit; ++b2) for (int h2 = 0; h2 < H && !hit; ++h2) for (int n2 = 0; n2 < N && !hit; ++n2) {
        const int64_t a0 = b * sb + h * sh + n * sn, b0 = delta_el + b2 * sb + h2 * sh + n2 * sn;
        if (a0 < b0 + D && b0 < a0 + D) hit = true;
      }
    const size_t nd = tvmattn_jvp_bwd_workspace_bytes(&e);
    const int rc = tvmattn_jvp_bwd(&e, P(G), P(2 * G), P(3 * G), P(4 * G), P(5 * G), P(6 * G), P(7 * G), P(8 * G),
                                   (float*)P(9 * G), (float*)P(10 * G), P(11 * G), P(12 * G), P(13 * G),
                                   P(13 * G + 2 * delta_el), P(15 * G), P(16 * G), P(17 * G), P(18 * G), P(19 * G), nd - 1,
                                   nullptr);
    EXPECT(rc == (hit ? TVMATTN_INVALID_ARG : TVMATTN_WORKSPACE_TOO_SMALL));
  }
  // ---- QK-norm, fused backward, AdaLN, gate, activation: one valid call each and a few bad ones
  float* gq = (float*)P(20 * G); float* gk = (float*)P(21 * G);
  EXPECT(tvmattn_qknorm_jvp_fwd(&d, P(G), P(2 * G), P(3 * G), P(4 * G), gq, gk, 1e-6f, P(5 * G), P(6 * G), P(7 * G), P(8 * G),
                                nullptr) == TVMATTN_OK);
  EXPECT(tvmattn_qknorm_jvp_fwd(&d, P(G), P(2 * G), P(3 * G), P(4 * G), gq, gk, -1.f, P(5 * G), P(6 * G), P(7 * G), P(8 * G),
                                nullptr) == TVMATTN_INVALID_ARG);
  const size_t nq = tvmattn_qknorm_jvp_bwd_workspace_bytes(&d);
  EXPECT(tvmattn_qknorm_jvp_bwd(&d, P(G), P(2 * G), P(3 * G), P(4 * G), gq, gk, 1e-6f, P(5 * G), P(6 * G), P(7 * G), P(8 * G),
                                P(9 * G), P(10 * G), P(11 * G), P(12 * G), (float*)P(13 * G), (float*)P(14 * G), P(15 * G), nq,
                                nullptr) == TVMATTN_OK);
  EXPECT(tvmattn_qknorm_jvp_bwd(&d, P(G), P(2 * G), P(3 * G), P(4 * G), gq, gk, 1e-6f, P(5 * G), P(6 * G), P(7 * G), P(8 * G),
                                P(9 * G), P(10 * G), P(11 * G), P(12 * G), (float*)P(13 * G), (float*)P(13 * G + 16), P(15 * G),
                                nq, nullptr) == TVMATTN_INVALID_ARG);  // the two gain gradients overlap
  const size_t nf = tvmattn_jvp_bwd_qknorm_workspace_bytes(&d);
  EXPECT(nf > need);
  EXPECT(tvmattn_jvp_bwd_qknorm(&d, P(G), P(2 * G), P(3 * G), P(4 * G), gq, gk, 1e-6f, P(5 * G), P(6 * G), P(7 * G), P(8 * G),
                                P(9 * G), P(10 * G), P(11 * G), P(12 * G), (float*)P(13 * G), (float*)P(14 * G), P(15 * G),
                                P(16 * G), P(17 * G), P(18 * G), P(19 * G), P(22 * G), P(23 * G), P(24 * G), (float*)P(25 * G),
                                (float*)P(26 * G), P(27 * G), nf, nullptr) == TVMATTN_OK);
  tvmattn_desc wide = mk(1, 1, 64, 128);
  EXPECT(tvmattn_jvp_bwd_qknorm_workspace_bytes(&wide) == 0);
  const int B = 4, T = 100, C = 1152;
  EXPECT(tvmattn_adaln_jvp_fwd(B, T, C, 1, P(G), P(2 * G), (float*)P(3 * G), (float*)P(4 * G), (float*)P(5 * G), (float*)P(6 * G),
                               1e-6f, P(7 * G), P(8 * G), nullptr) == TVMATTN_OK);
  EXPECT(tvmattn_adaln_jvp_fwd(B, T, C, 1, P(G), P(2 * G), (float*)P(3 * G), (float*)P(4 * G), (float*)P(5 * G), (float*)P(6 * G),
                               1e-6f, P(7 * G), P(G + 4096), nullptr) == TVMATTN_INVALID_ARG);
  const size_t na = tvmattn_adaln_jvp_bwd_workspace_bytes(B, T, C, 1);
  EXPECT(tvmattn_adaln_jvp_bwd(B, T, C, 1, P(G), P(2 * G), (float*)P(3 * G), (float*)P(4 * G), (float*)P(5 * G), (float*)P(6 * G),
                               1e-6f, P(7 * G), P(8 * G), P(9 * G), P(10 * G), (float*)P(11 * G), (float*)P(12 * G),
                               (float*)P(13 * G), (float*)P(14 * G), P(15 * G), na, nullptr) == TVMATTN_OK);
  EXPECT(tvmattn_adaln_jvp_bwd_residual(B, T, C, 1, P(G), P(2 * G), (float*)P(3 * G), (float*)P(4 * G), (float*)P(5 * G),
                                        (float*)P(6 * G), 1e-6f, P(7 * G), P(8 * G), P(16 * G), nullptr, P(9 * G), P(10 * G),
                                        (float*)P(11 * G), (float*)P(12 * G), (float*)P(13 * G), (float*)P(14 * G), P(15 * G), na,
                                        nullptr) == TVMATTN_INVALID_ARG);
  EXPECT(tvmattn_gate_jvp_fwd(B, T, C, 1, P(G), P(2 * G), P(3 * G), P(4 * G), (float*)P(5 * G), (float*)P(6 * G), 1e-6f, P(G),
                              P(2 * G), nullptr) == TVMATTN_OK);  // the stream updated in place
  EXPECT(tvmattn_gate_jvp_fwd(B, T, C, 1, P(G), P(2 * G), P(3 * G), P(4 * G), (float*)P(5 * G), (float*)P(6 * G), 1e-6f,
                              P(G + 16), P(2 * G), nullptr) == TVMATTN_INVALID_ARG);  // ... but not shifted
  const size_t ng = tvmattn_gate_jvp_bwd_workspace_bytes(B, T, C, 1);
  EXPECT(tvmattn_gate_jvp_bwd(B, T, C, 1, P(G), P(2 * G), (float*)P(3 * G), (float*)P(4 * G), 1e-6f, P(5 * G), P(6 * G), P(7 * G),
                              P(8 * G), (float*)P(9 * G), (float*)P(10 * G), P(11 * G), ng, nullptr) == TVMATTN_OK);
  EXPECT(tvmattn_gelu_jvp_fwd(1 << 20, 1, P(G), P(2 * G), P(3 * G), P(4 * G), nullptr) == TVMATTN_OK);
  EXPECT(tvmattn_gelu_jvp_fwd(1 << 20, 1, P(G), P(2 * G), P(3 * G), P(3 * G + (2 << 20) - 16), nullptr) == TVMATTN_INVALID_ARG);
  EXPECT(tvmattn_gelu_jvp_bwd(1ll << 41, 1, P(G), P(2 * G), P(3 * G), P(4 * G), P(5 * G), P(6 * G), nullptr) ==
         TVMATTN_UNSUPPORTED);
  for (int code = -7; code <= 0; ++code) EXPECT(tvmattn_strerror(code) != nullptr);
  std::printf("%s (%d stub launches)\n", fails ? "FAILED" : "host checks ok", g_stub_launches);
  return fails ? 1 : 0;
}
