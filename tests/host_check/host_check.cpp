// Host-side code of the library run under AddressSanitizer and UndefinedBehaviorSanitizer: argument
// validation of every entry point (each call here must be rejected before any GPU work), the
// Gram-Schmidt orthonormalisation of demo_set_basis, and the builders of the kernels' fragment
// tables, called directly on exactly sized buffers.  No GPU is touched.  Exit status 0 = all checks
// passed; a sanitizer report aborts the program.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <limits>
#include <vector>

#include "demo.h"
#include "demo_debug.h"
#include "demo_internal.h"

static int failures = 0;
#define EXPECT(cond)                                                     \
  do {                                                                   \
    if (!(cond)) {                                                       \
      std::fprintf(stderr, "host_check: line %d: %s\n", __LINE__, #cond); \
      ++failures;                                                        \
    }                                                                    \
  } while (0)

static demo_tensor tensor(int64_t rows, int64_t cols) {
  demo_tensor t;
  std::memset(&t, 0, sizeof t);
  // never dereferenced: every call below fails validation first
  t.grad = reinterpret_cast<const void*>(0x1000);
  t.mom = reinterpret_cast<float*>(0x2000);
  t.param = reinterpret_cast<void*>(0x3000);
  t.idx = reinterpret_cast<int32_t*>(0x4000);
  t.val = reinterpret_cast<float*>(0x5000);
  t.rows = rows;
  t.cols = cols;
  t.grad_dtype = DEMO_F32;
  t.param_dtype = DEMO_F32;
  return t;
}

// orthonormal DCT-II of size n in double (Sec. 2.1 "Blockwise Linear Projection")
static std::vector<double> dct(int n) {
  std::vector<double> P((size_t)n * n);
  const double pi = std::acos(-1.0);
  for (int u = 0; u < n; ++u)
    for (int j = 0; j < n; ++j)
      P[(size_t)u * n + j] = std::sqrt((u == 0 ? 1.0 : 2.0) / n) * std::cos(pi * (2 * j + 1) * u / (2.0 * n));
  return P;
}

static bool all_finite(const std::vector<float>& v) {
  for (float x : v)
    if (!std::isfinite(x)) return false;
  return true;
}

int main() {
  demo_ctx* ctx = nullptr;
  EXPECT(demo_create(nullptr) == DEMO_ERR_ARG);
  EXPECT(demo_create(&ctx) == DEMO_OK && ctx != nullptr);
  EXPECT(demo_destroy(nullptr) == DEMO_ERR_ARG);

  // payload sizes and shape checks over a grid of arguments
  for (int s : {16, 32, 48, 64, 128, 256})
    for (int64_t rows : {(int64_t)-64, (int64_t)0, (int64_t)64, (int64_t)100, (int64_t)1024, (int64_t)1 << 40})
      for (int64_t cols : {(int64_t)0, (int64_t)96, (int64_t)128, (int64_t)1 << 40})
        for (int k : {-1, 0, 1, 32, 64, 65, 256, 257, 1 << 20}) {
          int64_t out = -1;
          const int rc = demo_payload_elems(rows, cols, s, k, &out);
          if (rc == DEMO_OK) {
            const int64_t nch = cols == 0 ? rows / s : (rows / s) * (cols / s);
            EXPECT(out == nch * k);
          } else {
            EXPECT(rc == DEMO_ERR_ARG || rc == DEMO_ERR_SHAPE || rc == DEMO_ERR_UNSUPPORTED);
          }
        }
  EXPECT(demo_payload_elems(64, 64, 64, 1, nullptr) == DEMO_ERR_ARG);

  // status texts
  for (int code = -8; code <= 1; ++code) EXPECT(demo_strerror(code) != nullptr && std::strlen(demo_strerror(code)) > 0);
  EXPECT(demo_last_hip_error(ctx) != nullptr);

  // calls that must be rejected on the host
  demo_tensor good = tensor(128, 128);
  EXPECT(demo_encode(nullptr, &good, 1, 0.9f, 64, 8, nullptr) == DEMO_ERR_ARG);
  EXPECT(demo_encode(ctx, nullptr, 1, 0.9f, 64, 8, nullptr) == DEMO_ERR_ARG);
  EXPECT(demo_encode(ctx, &good, -1, 0.9f, 64, 8, nullptr) == DEMO_ERR_ARG);
  EXPECT(demo_encode(ctx, &good, 0, 0.9f, 64, 8, nullptr) == DEMO_OK);   // empty list: nothing to do
  EXPECT(demo_encode(ctx, &good, 1, 0.9f, 48, 8, nullptr) == DEMO_ERR_UNSUPPORTED);
  EXPECT(demo_encode(ctx, &good, 1, 0.9f, 64, 0, nullptr) == DEMO_ERR_ARG);
  EXPECT(demo_encode(ctx, &good, 1, 0.9f, 64, 4097, nullptr) == DEMO_ERR_ARG);
  EXPECT(demo_encode(ctx, &good, 1, 0.9f, 64, DEMO_MAX_K + 1, nullptr) == DEMO_ERR_UNSUPPORTED);
  EXPECT(demo_encode(ctx, &good, 1, std::numeric_limits<float>::quiet_NaN(), 64, 8, nullptr) == DEMO_ERR_ARG);
  EXPECT(demo_decode(ctx, &good, 1, 0, 1e-3f, 0.f, 64, 8, nullptr) == DEMO_ERR_ARG);
  EXPECT(demo_decode(ctx, &good, 1, 1, std::numeric_limits<float>::infinity(), 0.f, 64, 8, nullptr) == DEMO_ERR_ARG);
  {
    demo_tensor t = tensor(100, 128);
    EXPECT(demo_encode(ctx, &t, 1, 0.9f, 64, 8, nullptr) == DEMO_ERR_SHAPE);
    t = tensor(128, 100);
    EXPECT(demo_step(ctx, &t, 1, 0.9f, 1e-3f, 0.f, 64, 8, nullptr) == DEMO_ERR_SHAPE);
    t = tensor(128, 0);
    EXPECT(demo_encode(ctx, &t, 1, 0.9f, 64, 65, nullptr) == DEMO_ERR_ARG);   // k > M = s for an order-1 tensor
    t = tensor(128, 128);
    t.grad_dtype = 7;
    EXPECT(demo_encode(ctx, &t, 1, 0.9f, 64, 8, nullptr) == DEMO_ERR_UNSUPPORTED);
    t = tensor(128, 128);
    t.param_dtype = -1;
    EXPECT(demo_decode(ctx, &t, 1, 1, 1e-3f, 0.f, 64, 8, nullptr) == DEMO_ERR_UNSUPPORTED);
    t = tensor(128, 128);
    t.mom = nullptr;
    EXPECT(demo_encode(ctx, &t, 1, 0.9f, 64, 8, nullptr) == DEMO_ERR_ARG);
    t = tensor(128, 128);
    t.param = nullptr;
    EXPECT(demo_decode(ctx, &t, 1, 1, 1e-3f, 0.f, 64, 8, nullptr) == DEMO_ERR_ARG);
    t = tensor(128, 128);
    t.idx = nullptr;
    EXPECT(demo_step(ctx, &t, 1, 0.9f, 1e-3f, 0.f, 64, 8, nullptr) == DEMO_ERR_ARG);
    // the bad tensor is the last of a longer list
    std::vector<demo_tensor> list(40, tensor(256, 128));
    list.back().rows = 255;
    EXPECT(demo_encode(ctx, list.data(), (int)list.size(), 0.9f, 64, 8, nullptr) == DEMO_ERR_SHAPE);
  }

  // hyper-parameter block
  demo_hparams hp;
  EXPECT(demo_hparams_default(nullptr, 0.9f, 1e-3f, 0.f) == DEMO_ERR_ARG);
  EXPECT(demo_hparams_default(&hp, 0.9f, 1e-3f, 0.1f) == DEMO_OK);
  EXPECT(hp.grad_scale == 1.f && hp.alpha == 1.f && hp.phi == DEMO_PHI_SIGN && hp.aggregate == DEMO_AGG_SUM && hp.reserved == 0);
  EXPECT(demo_encode_ex(ctx, &good, 1, nullptr, 64, 8, nullptr) == DEMO_ERR_ARG);
  {
    demo_hparams bad = hp;
    bad.reserved = 1;
    EXPECT(demo_encode_ex(ctx, &good, 1, &bad, 64, 8, nullptr) == DEMO_ERR_ARG);
    bad = hp;
    bad.alpha = std::numeric_limits<float>::quiet_NaN();
    EXPECT(demo_step_ex(ctx, &good, 1, &bad, 64, 8, nullptr) == DEMO_ERR_ARG);
    bad = hp;
    bad.phi = 2;
    EXPECT(demo_decode_ex(ctx, &good, 1, 1, &bad, 64, 8, nullptr) == DEMO_ERR_ARG);
    bad = hp;
    bad.aggregate = 3;
    EXPECT(demo_decode_ex(ctx, &good, 1, 1, &bad, 64, 8, nullptr) == DEMO_ERR_ARG);
    bad = hp;
    bad.aggregate = DEMO_AGG_COUNT;
    EXPECT(demo_decode_ex(ctx, &good, 1, 256, &bad, 64, 8, nullptr) == DEMO_ERR_ARG);
  }

  // projection matrices: everything rejected before the device is bound
  EXPECT(demo_set_basis(nullptr, 64, DEMO_BASIS_DCT, nullptr) == DEMO_ERR_ARG);
  EXPECT(demo_set_basis(ctx, 48, DEMO_BASIS_DCT, nullptr) == DEMO_ERR_UNSUPPORTED);
  EXPECT(demo_set_basis(ctx, 64, 9, nullptr) == DEMO_ERR_ARG);
  EXPECT(demo_set_basis(ctx, 64, DEMO_BASIS_GRAM_SCHMIDT, nullptr) == DEMO_ERR_ARG);
  for (int s : {32, 64, 128}) {
    std::vector<float> a((size_t)s * s);
    for (size_t i = 0; i < a.size(); ++i) a[i] = std::sin(0.37 * (double)i) + 0.01 * (double)(i % 7);
    for (int c = 0; c < s; ++c) a[(size_t)(s - 1) * s + c] = 2.f * a[(size_t)3 * s + c];   // last row depends on row 3
    EXPECT(demo_set_basis(ctx, s, DEMO_BASIS_GRAM_SCHMIDT, a.data()) == DEMO_ERR_ARG);
    a[5] = std::numeric_limits<float>::infinity();
    EXPECT(demo_set_basis(ctx, s, DEMO_BASIS_GRAM_SCHMIDT, a.data()) == DEMO_ERR_ARG);
  }

  // other host-only entry points
  EXPECT(demo_set_timing(nullptr, 1) == DEMO_ERR_ARG);
  EXPECT(demo_set_timing(ctx, 1) == DEMO_OK);
  float ms = 0.f;
  EXPECT(demo_last_kernel_ms(ctx, 0, &ms) == DEMO_ERR_ARG);    // nothing recorded
  EXPECT(demo_last_kernel_ms(ctx, 9, &ms) == DEMO_ERR_ARG);
  EXPECT(demo_last_kernel_ms(ctx, 0, nullptr) == DEMO_ERR_ARG);
  EXPECT(demo_set_timing(ctx, 0) == DEMO_OK);
  EXPECT(demo_set_variant(ctx, 7) == DEMO_ERR_ARG);
  EXPECT(demo_set_variant(ctx, 0) == DEMO_OK && demo_set_variant(ctx, 1) == DEMO_OK);
  EXPECT(demo_copy_probe(ctx, nullptr, nullptr, 1024, nullptr) == DEMO_ERR_ARG);
  EXPECT(demo_copy_probe(ctx, reinterpret_cast<void*>(0x1000), reinterpret_cast<const void*>(0x2000), 1000, nullptr) == DEMO_ERR_ARG);
  EXPECT(demo_copy_probe(ctx, reinterpret_cast<void*>(0x1008), reinterpret_cast<const void*>(0x2000), 1024, nullptr) == DEMO_ERR_ARG);

  // fragment tables of the wavefront kernels, into buffers of exactly the declared sizes
  {
    const std::vector<double> P64 = dct(64), P32 = dct(32);
    std::vector<double> B64((size_t)64 * 64, 0.0);   // diag(P32, P32)
    for (int h = 0; h < 2; ++h)
      for (int u = 0; u < 32; ++u)
        for (int j = 0; j < 32; ++j) B64[(size_t)(32 * h + u) * 64 + 32 * h + j] = P32[(size_t)u * 32 + j];
    std::vector<float> e64(demo::kEnc64TableFloats), d64(demo::kDec64TableFloats), e32(demo::kEnc64dTableFloats),
        d32(demo::kDec32TableFloats);
    demo::build_enc64_tables(P64.data(), e64.data());
    demo::build_dec64_tables(P64.data(), d64.data());
    demo::build_enc64d_tables(B64.data(), e32.data());
    demo::build_dec32_tables(P32.data(), d32.data());
    EXPECT(all_finite(e64) && all_finite(d64) && all_finite(e32) && all_finite(d32));
    double energy = 0.0;
    for (float x : e64) energy += (double)x * x;
    EXPECT(energy > 1.0);   // the tables hold entries of an orthonormal matrix
  }

  // pre-split float16 fragment tables (the matrix entries times 2^4 as hi + lo halves): exactly sized buffers, and
  // every entry of the s = 128 decode and encode tables and of the full-product s = 64 decode table decoded again:
  // hi + lo must give 16 P to 2^-21 of the entry (two float16 parts hold 22 significant bits) or 2^-25 absolute
  // (the spacing of the float16 subnormals, halved)
  {
    auto half = [](uint32_t h) {   // float16 code -> value
      const int e = (int)((h >> 10) & 31u);
      const double m = (double)(h & 1023u);
      const double mag = e == 0 ? std::ldexp(m, -24) : std::ldexp(m + 1024.0, e - 25);
      return (h & 0x8000u) ? -mag : mag;
    };
    // block `blk` (512 words: [hi | lo][64 lanes][4 words]) of a table, lane, slot j -> hi + lo
    auto entry = [&](const std::vector<float>& tab, int blk, int lane, int j) {
      uint32_t wh, wl;
      std::memcpy(&wh, &tab[(size_t)blk * 512 + (0 * 64 + lane) * 4 + (j >> 1)], 4);
      std::memcpy(&wl, &tab[(size_t)blk * 512 + (1 * 64 + lane) * 4 + (j >> 1)], 4);
      return half((j & 1) ? wh >> 16 : wh & 0xffffu) + half((j & 1) ? wl >> 16 : wl & 0xffffu);
    };
    auto close = [](double got, double want) { return std::fabs(got - want) <= std::fabs(want) * std::ldexp(1.0, -21) + std::ldexp(1.0, -25); };
    const std::vector<double> P64 = dct(64), P128 = dct(128);
    std::vector<float> d64g(demo::kDec64DenseTableFloats), e64g(demo::kEnc64DenseTableFloats), d128(demo::kDec128TableFloats),
        e128(demo::kEnc128TableFloats);
    demo::build_dec64_dense_tables(P64.data(), d64g.data());
    demo::build_enc64_dense_tables(P64.data(), e64g.data());
    demo::build_dec128_tables(P128.data(), d128.data());
    demo::build_enc128_tables(P128.data(), e128.data());
    EXPECT(all_finite(e64g));
    int bad = 0;
    for (int t = 0; t < 4; ++t)
      for (int h = 0; h < 2; ++h)
        for (int lane = 0; lane < 64; ++lane)
          for (int j = 0; j < 8; ++j) {
            const int g = lane >> 4, c = lane & 15;
            const int kk = 16 * (2 * h + (j >> 2)) + 4 * g + (j & 3);   // contraction index of slot j
            // full-product s = 64 decode: P[kk][16 t + c]
            if (!close(entry(d64g, 2 * t + h, lane, j), 16.0 * P64[(size_t)kk * 64 + 16 * t + c])) ++bad;
            for (int m = 0; m < 2; ++m) {
              // s = 128 decode: rows 2 kk + m of P, columns 16 t + c; encode: the transposed fragments
              if (!close(entry(d128, 8 * m + 2 * t + h, lane, j), 16.0 * P128[(size_t)(2 * kk + m) * 128 + 16 * t + c])) ++bad;
              if (!close(entry(e128, 8 * m + 2 * t + h, lane, j), 16.0 * P128[(size_t)(2 * (16 * t + c) + m) * 128 + kk])) ++bad;
            }
          }
    EXPECT(bad == 0);
  }

  EXPECT(demo_destroy(ctx) == DEMO_OK);
  if (failures == 0) std::printf("host_check OK\n");
  return failures == 0 ? 0 : 1;
}
