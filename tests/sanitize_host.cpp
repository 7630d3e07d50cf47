// Host-code driver for the sanitizer build (tests/test_host_sanitizers.py): compiled together with the
// constructor, the operator entry points' host side and the C oracle under -fsanitize=address,undefined and
// run on the CPU.  It walks the host paths that never launch a kernel: construction for every operator
// kind and layout, single-walk traces, the cost model over every compiled instance, workspace sizing,
// argument refusals of the operators (which return before any launch), and the oracle's loop nests on
// exact-size buffers (any out-of-bounds index there is a sanitizer report).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../include/gensor.h"

extern "C" {
int oracle_gemm(int dtype, int transA, int transB, int64_t M, int64_t N, int64_t K, double alpha, const void* A, int64_t lda,
                const void* B, int64_t ldb, double beta, double* C, int64_t ldc);
int oracle_conv2d(int dtype, int64_t N, int64_t C, int64_t H, int64_t W, int64_t K, int64_t R, int64_t S, int64_t stride,
                  int64_t pad, const void* I, const void* Wt, double* O);
int oracle_gemv(int dtype, int64_t M, int64_t N, double alpha, const void* A, int64_t lda, const void* x, double beta, double* y);
int oracle_avgpool2d(int dtype, int64_t N, int64_t C, int64_t H, int64_t W, int64_t F, int64_t S, const void* I, double* O);
}

static int failures = 0;
#define CHECK(cond) do { if (!(cond)) { std::printf("CHECK failed line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)

static gensor_problem gemm(int dt, int64_t M, int64_t N, int64_t K, int ta, int tb, int64_t batch = 1, int out = GENSOR_F32) {
  gensor_problem p;
  std::memset(&p, 0, sizeof(p));
  p.op = batch > 1 ? GENSOR_OP_BMM : GENSOR_OP_GEMM;
  p.in_dtype = dt; p.out_dtype = out; p.transA = ta; p.transB = tb; p.batch = batch; p.M = M; p.N = N; p.K = K;
  return p;
}
static gensor_problem conv(int dt, int64_t n, int64_t c, int64_t h, int64_t w, int64_t k, int64_t r, int64_t s, int64_t stride, int64_t pad) {
  gensor_problem p;
  std::memset(&p, 0, sizeof(p));
  p.op = GENSOR_OP_CONV2D; p.in_dtype = dt; p.out_dtype = GENSOR_F32;
  p.n = n; p.c = c; p.h = h; p.w = w; p.k = k; p.r = r; p.s = s; p.stride = stride; p.pad = pad;
  return p;
}

int main() {
  std::vector<gensor_problem> ps = {
      gemm(GENSOR_F16, 4096, 4096, 4096, 0, 1), gemm(GENSOR_F32, 512, 512, 512, 0, 0), gemm(GENSOR_F16, 8192, 3072, 768, 0, 0),
      gemm(GENSOR_BF16, 1024, 1024, 64, 0, 1, 96), gemm(GENSOR_F16, 65536, 1024, 4, 0, 0), gemm(GENSOR_F16, 77, 53, 41, 0, 0, 1, GENSOR_F16),
      gemm(GENSOR_F16, 2048, 1024, 512, 1, 0), gemm(GENSOR_F32, 200, 136, 72, 1, 1), gemm(GENSOR_F16, 1, 1, 1, 0, 0),
      gemm(GENSOR_F16, 512, 512, 32768, 0, 1),
      conv(GENSOR_F16, 32, 64, 56, 56, 64, 3, 3, 1, 1), conv(GENSOR_F16, 32, 256, 56, 56, 512, 1, 1, 2, 0),
      conv(GENSOR_F16, 8, 64, 27, 27, 128, 1, 1, 2, 0), conv(GENSOR_F32, 4, 24, 13, 11, 40, 3, 2, 2, 1), conv(GENSOR_BF16, 1, 8, 5, 5, 8, 5, 5, 1, 2)};
  const int n_inst = gensor_num_instances();
  CHECK(n_inst > 100);
  for (size_t i = 0; i < ps.size(); ++i) {
    gensor_schedule s;
    for (uint64_t seed : {0ull, 7ull}) {
      gensor_construct_opts o;
      std::memset(&o, 0, sizeof(o));
      o.chains = 512;
      CHECK(gensor_construct(&ps[i], nullptr, &o, seed, &s) == GENSOR_OK);
      CHECK(s.kernel_id >= 0 && s.kernel_id < n_inst && s.predicted_us > 0);
      o.no_vthread = 1; o.keep_policy = 1; o.tiling_benefit = 1;
      gensor_status st = gensor_construct(&ps[i], nullptr, &o, seed, &s);
      CHECK(st == GENSOR_OK || st == GENSOR_ERR_NO_SCHEDULE);
      o.greedy = 1; o.chains = 1;
      st = gensor_construct(&ps[i], nullptr, &o, seed, &s);
      CHECK(st == GENSOR_OK || st == GENSOR_ERR_NO_SCHEDULE);
    }
    int32_t steps = 0;
    std::vector<int32_t> actions(128), dims(128), states(128 * 12);
    CHECK(gensor_construct_trace(&ps[i], nullptr, nullptr, 3, 128, &steps, actions.data(), dims.data(), states.data()) == GENSOR_OK);
    CHECK(steps > 0 && steps <= 100);
    CHECK(gensor_construct_trace(&ps[i], nullptr, nullptr, 3, 5, &steps, actions.data(), dims.data(), states.data()) == GENSOR_OK);   // a short buffer
    CHECK(steps <= 5);
    int served = 0;
    for (int id = 0; id < n_inst; ++id) {
      gensor_schedule t;
      if (gensor_instance_schedule(id, &ps[i], &t) != GENSOR_OK) continue;
      ++served;
      for (int split : {1, 2, 16}) {
        t.split_k = split;
        (void)gensor_predict_us(&t, &ps[i], nullptr);
        (void)gensor_workspace_bytes(&t, &ps[i]);
      }
    }
    CHECK(served > 0);
    (void)gensor_workspace_bytes(nullptr, &ps[i]);
  }
  // refusals: each returns before anything is launched
  {
    gensor_problem p = gemm(GENSOR_F16, 64, 64, 64, 0, 1);
    alignas(16) static char buf[64];
    CHECK(gensor_gemm(nullptr, &p, 1.f, nullptr, 64, buf, 64, 0.f, buf, 64, nullptr, 0, nullptr) == GENSOR_ERR_INVALID_ARG);
    CHECK(gensor_gemm(nullptr, &p, 1.f, buf, 8, buf, 64, 0.f, buf, 64, nullptr, 0, nullptr) == GENSOR_ERR_INVALID_ARG);
    gensor_problem bad = gemm(GENSOR_F16, 0, 64, 64, 0, 1);
    CHECK(gensor_gemm(nullptr, &bad, 1.f, buf, 64, buf, 64, 0.f, buf, 64, nullptr, 0, nullptr) == GENSOR_ERR_INVALID_ARG);
    gensor_problem odd = gemm(GENSOR_F16, 64, 64, 64, 0, 1, 1, GENSOR_BF16);
    CHECK(gensor_gemm(nullptr, &odd, 1.f, buf, 64, buf, 64, 0.f, buf, 64, nullptr, 0, nullptr) == GENSOR_ERR_UNSUPPORTED);
    gensor_problem c = conv(GENSOR_F16, 1, 4, 2, 2, 4, 3, 3, 1, 0);
    CHECK(gensor_conv2d(nullptr, &c, buf, buf, buf, nullptr, 0, nullptr) == GENSOR_ERR_INVALID_ARG);
    CHECK(gensor_gemv(GENSOR_F16, 4, 4, 1.f, nullptr, 4, buf, 0.f, (float*)buf, nullptr) == GENSOR_ERR_INVALID_ARG);
    CHECK(gensor_avgpool2d(GENSOR_F16, GENSOR_F32, 1, 1, 2, 2, 3, 1, buf, buf, nullptr) == GENSOR_ERR_INVALID_ARG);
    gensor_schedule s;
    CHECK(gensor_construct(&bad, nullptr, nullptr, 0, &s) == GENSOR_ERR_INVALID_ARG);
    CHECK(gensor_predict_us(nullptr, &p, nullptr) < 0);
    CHECK(std::strlen(gensor_status_string(GENSOR_ERR_WORKSPACE)) > 0);
    CHECK(gensor_hw_mi355x()->compute_units == 256);
  }
  // the oracle on exact-size heap buffers
  {
    const int64_t M = 5, N = 7, K = 3;
    for (int dt = 0; dt < 3; ++dt)
      for (int ta = 0; ta < 2; ++ta)
        for (int tb = 0; tb < 2; ++tb) {
          const size_t es = dt == 0 ? 4 : 2;
          std::vector<char> A(M * K * es, 0), B(K * N * es, 0);
          std::vector<double> C(M * N, 1.0);
          CHECK(oracle_gemm(dt, ta, tb, M, N, K, 2.0, A.data(), ta ? M : K, B.data(), tb ? K : N, 0.5, C.data(), N) == 0);
          CHECK(C[0] == 0.5 && C[M * N - 1] == 0.5);
        }
    std::vector<char> I(2 * 3 * 6 * 5 * 2, 0), W(4 * 3 * 3 * 2 * 2, 0);
    std::vector<double> O(2 * 4 * 3 * 3, -1.0);              // P = (6 + 2 - 3)/2 + 1 = 3, Q = (5 + 2 - 2)/2 + 1 = 3
    CHECK(oracle_conv2d(1, 2, 3, 6, 5, 4, 3, 2, 2, 1, I.data(), W.data(), O.data()) == 0);
    CHECK(O[0] == 0.0 && O.back() == 0.0);
    std::vector<char> Av(4 * 9 * 2, 0), xv(9 * 2, 0);
    std::vector<double> y(4, 3.0);
    CHECK(oracle_gemv(1, 4, 9, 1.0, Av.data(), 9, xv.data(), 1.0, y.data()) == 0);
    CHECK(y[3] == 3.0);
    std::vector<char> Ip(1 * 2 * 7 * 5 * 2, 0);
    std::vector<double> Op(1 * 2 * 3 * 2, -1.0);              // F = 3, S = 2: P = (7-3)/2+1 = 3, Q = (5-3)/2+1 = 2
    CHECK(oracle_avgpool2d(1, 1, 2, 7, 5, 3, 2, Ip.data(), Op.data()) == 0);
    CHECK(Op.back() == 0.0);
  }
  std::printf("%s: %d failure(s)\n", failures ? "FAILED" : "sanitized host paths ok", failures);
  return failures ? 1 : 0;
}
