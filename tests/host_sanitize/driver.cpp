// driver.cpp — host-only program run under AddressSanitizer + UBSan (tests/test_host_sanitizers.py):
//  * the layer-spec planner on the five workload specs and on hostile specs (huge dimensions, empty tokens,
//    nine-digit channel counts, shapes that do not fit together): every bad spec must come back as a negative
//    status, never as undefined behaviour;
//  * the CPU oracle's C interface on a small network (forward, activations, backward), the noise generator
//    across the 2^32 sample boundary, the message bits and the error counter.
// Prints "sanitize-ok" and exits 0 when everything ran; a sanitizer report aborts the process instead.
#include <stdint.h>
#include <stdio.h>
#include <string.h>

#include <string>
#include <vector>

#include "ae_internal.h"

extern "C" {
void* oracle_create(const char* spec, int batch, int bn_mode, int store_bf16);
void oracle_destroy(void* h);
int64_t oracle_param_count(void* h);
int oracle_num_ops(void* h);
int oracle_forward(void* h, const float* params, const float* x, float snr_db, uint64_t seed, uint64_t first_sample, double* y);
int64_t oracle_get_activation(void* h, int i, double* out);
int oracle_backward(void* h, const float* params, const double* dy, double* grads, double* dx);
void oracle_noise(uint64_t seed, uint64_t first_sample, int64_t batch, int64_t n, float* out);
void oracle_gen_bits(uint64_t seed, uint64_t first_sample, int64_t batch, int k, float* x_pm1);
void oracle_count_errors(const double* y, const float* x_pm1, int64_t batch, int k, uint64_t* bit_err, uint64_t* blk_err);
double oracle_loss_mse(const double* y, const double* t, int64_t n, double* dy);
}

static int g_fail = 0;
#define EXPECT(cond)                                                   \
  do {                                                                 \
    if (!(cond)) { printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); ++g_fail; } \
  } while (0)

static int plan_rc(const char* spec, int batch, int dtype, int bn_mode = 0) {
  ae::Plan p;
  return ae::build_plan(spec, batch, dtype, bn_mode, &p);
}

int main(int argc, char** argv) {
  // ---- planner: the five workloads parse and size up
  const char* good[] = {
      "in:1x28x28,conv3:16,bn,relu,pool2,conv3:32,bn,relu,pool2,flatten,fc:64,pnorm,awgn,fc:1568,reshape:32x7x7,up2,conv3:16,relu,up2,conv3:1,sigmoid",
      "in:3x32x32,conv3:64,bn,relu,pool2,conv3:128,bn,relu,pool2,conv3:256,bn,relu,pool2,flatten,fc:512,pnorm,awgn,fc:4096,reshape:256x4x4,up2,conv3:128,relu,up2,conv3:64,relu,up2,conv3:3,sigmoid",
      "in:64x1x1,fc:512,relu,fc:512,relu,fc:128,pnorm,awgn,fc:512,relu,fc:512,relu,fc:64,sigmoid",
      "in:3x256x256,conv3:64,bn,relu,pool2,conv3:128,bn,relu,pool2,conv3:256,bn,relu,pool2,conv3:512,bn,relu,pool2,conv3:512,bn,relu,pool2,conv1:64,pnorm,awgn,conv1:512,up2,conv3:512,relu,up2,conv3:256,relu,up2,conv3:128,relu,up2,conv3:64,relu,up2,conv3:3,sigmoid",
  };
  const int batches[] = {64, 256, 65536, 32};
  for (int i = 0; i < 4; ++i)
    for (int dtype = 0; dtype < 2; ++dtype) {
      ae::Plan p;
      EXPECT(ae::build_plan(good[i], batches[i], dtype, 0, &p) == AE_OK);
      EXPECT(p.ws_bytes > 0 && p.n_params > 0 && !p.steps.empty());
      for (const ae::Step& st : p.steps) EXPECT(st.off_out >= 0 && st.off_out < p.ws_bytes);
    }
  // ---- planner: hostile specs
  struct Bad { const char* spec; int batch; int rc; };
  const Bad bad[] = {
      {"in:1x65536x65536,flatten,fc:8", 1, AE_ESHAPE},             // 2^32 pixels
      {"in:3x100000x100000,conv3:8", 2, AE_ESHAPE},
      {"in:1x1x1,fc:8,reshape:65536x65536x1", 1, AE_ESHAPE},       // overflowing reshape
      {"in:4x4x4,conv3:999999999", 1, AE_ESHAPE},                  // nine-digit channel count
      {"in:4x4x4,conv3:9999999999", 1, AE_ESPEC},                  // ten digits do not parse
      {"in:999999999x999999999x999999999,conv3:4", 1, AE_ESHAPE},
      {"in:8x2x2,up2,conv3:536870912", 1, AE_ESHAPE},
      {"in:3x8x8,,conv3:4", 1, AE_ESPEC},                          // empty token
      {"", 1, AE_ESPEC},
      {",", 1, AE_ESPEC},
      {"in:3x8x8,", 1, AE_ESPEC},
      {"in:3x8x8", 1, AE_ESPEC},                                   // no layers
      {"in:3x8", 1, AE_ESPEC},
      {"in:3x8x8x8,conv3:4", 1, AE_ESPEC},
      {"in:-3x8x8,conv3:4", 1, AE_ESPEC},
      {"in:0x8x8,conv3:4", 1, AE_ESPEC},
      {"in:3x8x8,conv3:", 1, AE_ESPEC},
      {"in:3x8x8,conv3:4x", 1, AE_ESPEC},
      {"in:3x8x8,conv5:4", 1, AE_ESPEC},
      {"in:3x8x8,relu", 1, AE_ESPEC},
      {"in:3x8x8,up2,relu", 1, AE_ESPEC},
      {"in:3x8x8,up2", 1, AE_ESPEC},
      {"in:3x5x5,conv3:4,pool2", 1, AE_ESHAPE},
      {"in:3x8x8,fc:4", 1, AE_ESHAPE},
      {"in:12x1x1,reshape:3x2x3", 1, AE_ESHAPE},
      {"in:3x8x8,reshape:3x8x8", 1, AE_ESPEC},
      {"in:3x8x8,conv3:4", 0, AE_EINVAL},
      {"in:3x8x8,conv3:4", -5, AE_EINVAL},
      {"in:3x2048x2048,conv3:64", 2147483647, AE_ESHAPE},
      {"in:1x1x1,fc:1", 2147483647, AE_ESHAPE},
  };
  for (const Bad& b : bad) {
    const int rc = plan_rc(b.spec, b.batch, 0);
    if (rc != b.rc) { printf("FAILED spec '%s' batch %d: rc %d, expected %d (%s)\n", b.spec, b.batch, rc, b.rc, ae::last_error()); ++g_fail; }
  }
  EXPECT(plan_rc(nullptr, 1, 0) == AE_EINVAL);
  EXPECT(plan_rc("in:3x8x8,conv3:4", 1, 7) == AE_EINVAL);
  EXPECT(plan_rc("in:3x8x8,conv3:4", 1, 0, 3) == AE_EINVAL);
  {  // a long chain of tokens and a very long token
    std::string s = "in:4x8x8";
    for (int i = 0; i < 200; ++i) s += ",conv3:4,relu";
    EXPECT(plan_rc(s.c_str(), 2, 1) == AE_OK);
    std::string t = "in:4x8x8,conv3:" + std::string(4000, '7');
    EXPECT(plan_rc(t.c_str(), 2, 1) == AE_ESPEC);
    std::string u = "in:4x8x8," + std::string(5000, 'z');
    EXPECT(plan_rc(u.c_str(), 2, 1) == AE_ESPEC);   // the error text is cut to the message buffer
  }

  // ---- oracle: a small network end to end
  {
    const char* spec = "in:2x8x12,conv3:5,bn,relu,pool2,conv1:3,pnorm,awgn,conv1:4,up2,conv3:2,sigmoid";
    const int B = 3;
    for (int store = 0; store < 2; ++store)
      for (int bn_mode = 0; bn_mode < 2; ++bn_mode) {
        void* h = oracle_create(spec, B, bn_mode, store);
        EXPECT(h != nullptr);
        if (!h) continue;
        const int64_t np = oracle_param_count(h);
        std::vector<float> prm((size_t)np), x((size_t)B * 2 * 8 * 12);
        uint32_t r = 12345u;
        auto rnd = [&]() { r = r * 1664525u + 1013904223u; return (float)((r >> 8) & 0xFFFF) / 65536.0f - 0.5f; };
        for (float& v : prm) v = rnd();
        if (bn_mode == 1) for (float& v : prm) v = v * v + 0.3f;    // stored variances must be positive
        for (float& v : x) v = rnd() + 0.5f;
        std::vector<double> y((size_t)B * 2 * 8 * 12), dy(y.size()), g((size_t)np), dx(x.size());
        EXPECT(oracle_backward(h, prm.data(), dy.data(), g.data(), dx.data()) != 0);   // backward before forward
        EXPECT(oracle_forward(h, prm.data(), x.data(), 7.0f, 99, ((uint64_t)1 << 32) - 2, y.data()) == 0);
        for (int i = -1; i < oracle_num_ops(h); ++i) {
          const int64_t n = oracle_get_activation(h, i, nullptr);
          EXPECT(n > 0);
          std::vector<double> a((size_t)n);
          EXPECT(oracle_get_activation(h, i, a.data()) == n);
        }
        EXPECT(oracle_get_activation(h, oracle_num_ops(h), nullptr) < 0);
        std::vector<double> t(y.size(), 0.25);
        EXPECT(oracle_loss_mse(y.data(), t.data(), (int64_t)y.size(), dy.data()) >= 0.0);
        EXPECT(oracle_backward(h, prm.data(), dy.data(), g.data(), dx.data()) == 0);
        oracle_destroy(h);
      }
    EXPECT(oracle_create("in:3x5x5,conv3:4,pool2", 2, 0, 0) == nullptr);
    EXPECT(oracle_create("in:3x8x8,bogus", 2, 0, 0) == nullptr);
    EXPECT(oracle_create("in:3x8x8,conv3:4", 0, 0, 0) == nullptr);
  }
  {  // generator, message bits, counters
    std::vector<float> nz(7 * 37);
    oracle_noise(5, ((uint64_t)1 << 32) - 3, 7, 37, nz.data());
    std::vector<float> bits(5 * 200);
    oracle_gen_bits(3, 0xFFFFFFFFFFFFFFF0ull, 5, 200, bits.data());
    std::vector<double> y(bits.size());
    for (size_t i = 0; i < y.size(); ++i) y[i] = (i % 7 == 0) ? 0.2 : (bits[i] > 0 ? 0.9 : 0.1);
    uint64_t be = 0, ke = 0;
    oracle_count_errors(y.data(), bits.data(), 5, 200, &be, &ke);
    EXPECT(ke <= 5 && be <= 1000);
  }
  if (g_fail) { printf("%d check(s) failed\n", g_fail); return 1; }
  printf("sanitize-ok\n");
  return 0;
}
