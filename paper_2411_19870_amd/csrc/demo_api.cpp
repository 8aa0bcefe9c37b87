// Host side of the C ABI declared in include/demo.h: argument validation,
// context (DCT basis tables, cached device descriptor tables), dispatch.
#include "demo.h"
#include "demo_debug.h"
#include "demo_internal.h"

#include <cmath>
#include <cstring>
#include <new>
#include <string>
#include <vector>

static_assert(DEMO_MAX_K == DEMO_MAXK_INTERNAL, "public and internal k limits must agree");
static_assert(sizeof(demo_tensor) == 64, "demo_tensor layout is part of the ABI");
static_assert(DEMO_NOALLOC_MAX_TENSORS == demo::kNoallocMaxTensors && DEMO_NOALLOC_MAX_CHUNKS == demo::kNoallocMaxChunks &&
                  DEMO_NOALLOC_SCRATCH_BYTES == demo::kNoallocScratchBytes,
              "public and internal limits of the allocation-free entry point must agree");


namespace {

using demo::TableView;
using demo::TensorDev;

struct BasisTable {
  int s = 0;
  float* dev = nullptr;      // P, s x s
  float* enc64 = nullptr;    // tables of the s = 64 wavefront-per-chunk kernels
  float* dec64 = nullptr;
  float* dec64h = nullptr;   // DCT fragments for the full-product s = 64 decode kernel (float16 matrix pipe)
  float* enc32 = nullptr;    // dense-basis tile tables for s = 32
  float* dec32 = nullptr;    // fragment table of the s = 32 tile decode kernel
  float* dec128 = nullptr;   // fragment tables of the s = 128 kernels
  float* enc128 = nullptr;
  float* custom = nullptr;   // s x s matrix set with demo_set_basis (identity / Gram-Schmidt), allocated on first use
  float* custom_enc64 = nullptr;   // s = 64: tables of the full-product wavefront kernels for `custom`
  float* custom_dec64 = nullptr;
  bool use_custom = false;   // later calls project with `custom` (s = 64: full-product wavefront kernels, else generic)
};

// The order-2 tensors of a list that share gradient and parameter dtype: they go out in one launch per
// side (the wavefront kernels are instances per dtype; a list of mixed dtypes takes one launch per group
// instead of falling back to the kernels that read the dtype per tensor).
struct TableGroup {
  TableView tv2{};
  TableView tv2t{};           // the same tensors counted in 64 x 64 tiles (s = 32, all dimensions multiples of 64), else n = 0
  demo::Worklist wl{};        // queue of this group's chunks for the exact fallback kernel
};

// One cached descriptor upload: the host bytes it was built from and the device copy.
struct TableCache {
  std::vector<char> key;      // raw demo_tensor bytes + s (empty: the slot holds nothing valid)
  hipStream_t last_stream = nullptr;   // stream of the last call that used the tables
  bool many_streams = false;  // ... and whether calls on several streams have used them
  bool pinned = false;        // used under stream capture: a graph holds the table's address, never evicted
  void* dev = nullptr;        // per group [TensorDev x n][int32 x (n+1)][queue][tile tables], then the order-1 tables
  size_t dev_bytes = 0;
  std::vector<TableGroup> groups;   // order-2 tensors by (gradient dtype, parameter dtype, tileable at s = 32)
  TableView tv1{};
  uint64_t last_use = 0;
};

constexpr int kMaxCachedTables = 8;
constexpr int kNumTimers = 4;
constexpr int kMaxTimedLaunches = 256;

}  // namespace

struct demo_ctx {
  int device = -1;            // bound at first GPU use
  int num_cus = 0;
  std::vector<BasisTable> bases;
  std::vector<TableCache> tables;
  uint64_t use_counter = 0;
  bool timing = false;
  std::vector<hipEvent_t> ev[kNumTimers][2];   // event pairs, one per recorded launch
  int ev_count[kNumTimers] = {};               // launches recorded since timing was enabled
  hipError_t last_hip = hipSuccess;
  int variant = 1;            // 0 = generic kernels only
  int enc_stage = 0;          // 1..3: cut-down copies of the s = 64 encode kernel (time attribution)
  int dec_stage = 0;          // 1, 2: cut-down runs of the s = 64 decode kernel
};

namespace {

int fail_hip(demo_ctx* ctx, hipError_t e) {
  ctx->last_hip = e;
  return DEMO_ERR_HIP;
}

bool s_supported(int s) { return s == 32 || s == 64 || s == 128; }

// Shape / s / k checks shared by every entry point.  Order of checks is part of
// the documented behaviour: unsupported s first, then k < 1, then shape, then
// k against the chunk size, then the k limit.
int check_shape(int64_t rows, int64_t cols, int s, int k) {
  if (!s_supported(s)) return DEMO_ERR_UNSUPPORTED;
  if (k < 1) return DEMO_ERR_ARG;
  if (rows <= 0 || cols < 0) return DEMO_ERR_SHAPE;
  if (rows % s != 0 || cols % s != 0) return DEMO_ERR_SHAPE;
  if (cols >= DEMO_MAX_COLS) return DEMO_ERR_UNSUPPORTED;   // 32-bit row offsets inside a chunk
  const int64_t M = cols == 0 ? (int64_t)s : (int64_t)s * s;
  if (k > M) return DEMO_ERR_ARG;
  if (k > DEMO_MAX_K) return DEMO_ERR_UNSUPPORTED;
  // chunks are numbered with 32 bits (and the products below must not overflow)
  const int64_t r = rows / s, c = cols / s;
  if (r > INT32_MAX || (c > 0 && r > INT32_MAX / c)) return DEMO_ERR_UNSUPPORTED;
  return DEMO_OK;
}

enum Need { NEED_ENCODE = 1, NEED_DECODE = 2 };

int validate(const demo_ctx* ctx, const demo_tensor* t, int n, int s, int k, int need) {
  if (ctx == nullptr || n < 0 || (n > 0 && t == nullptr)) return DEMO_ERR_ARG;
  if (!s_supported(s)) return DEMO_ERR_UNSUPPORTED;
  if (k < 1) return DEMO_ERR_ARG;
  int64_t total2 = 0, total1 = 0;
  for (int i = 0; i < n; ++i) {
    const int rc = check_shape(t[i].rows, t[i].cols, s, k);
    if (rc != DEMO_OK) return rc;
    if ((need & NEED_ENCODE) && (t[i].grad_dtype != DEMO_F32 && t[i].grad_dtype != DEMO_BF16))
      return DEMO_ERR_UNSUPPORTED;
    if ((need & NEED_DECODE) && (t[i].param_dtype != DEMO_F32 && t[i].param_dtype != DEMO_BF16))
      return DEMO_ERR_UNSUPPORTED;
    if (t[i].idx == nullptr || t[i].val == nullptr) return DEMO_ERR_ARG;
    if ((need & NEED_ENCODE) && (t[i].grad == nullptr || t[i].mom == nullptr)) return DEMO_ERR_ARG;
    if ((need & NEED_DECODE) && t[i].param == nullptr) return DEMO_ERR_ARG;
    // the kernels move tensor rows with 16-byte accesses; payload arrays only need their natural alignment
    auto misaligned = [](const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; };
    if ((need & NEED_ENCODE) && (misaligned(t[i].grad, 16) || misaligned(t[i].mom, 16))) return DEMO_ERR_ARG;
    if ((need & NEED_DECODE) && misaligned(t[i].param, 16)) return DEMO_ERR_ARG;
    if (misaligned(t[i].idx, 4) || misaligned(t[i].val, 4)) return DEMO_ERR_ARG;
    if (t[i].cols == 0) total1 += t[i].rows / s;
    else total2 += (t[i].rows / s) * (t[i].cols / s);
    if (total1 > INT32_MAX || total2 > INT32_MAX) return DEMO_ERR_UNSUPPORTED;
  }
  return DEMO_OK;
}

int bind_device(demo_ctx* ctx) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(ctx, e);
  if (ctx->device < 0) {
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess) return fail_hip(ctx, e);
    ctx->device = dev;
    ctx->num_cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
  } else if (ctx->device != dev) {
    return DEMO_ERR_ARG;  // a context stays on the device it first ran on
  }
  return DEMO_OK;
}

// One device allocation filled from the host (Sec. 2.1 "Blockwise Linear Projection": the matrices are
// precomputed once and shared by all tensors).
int upload(demo_ctx* ctx, const std::vector<float>& host, float** dev) {
  hipError_t e = hipMalloc(reinterpret_cast<void**>(dev), host.size() * sizeof(float));
  if (e != hipSuccess) return fail_hip(ctx, e);
  e = hipMemcpy(*dev, host.data(), host.size() * sizeof(float), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(*dev);
    *dev = nullptr;
    return fail_hip(ctx, e);
  }
  return DEMO_OK;
}

// Host copies of the tables of one chunk size: the orthonormal DCT-II matrix P[u][n] = c_u cos(pi (2n+1) u / (2s))
// evaluated in double precision and rounded once to float32, and the fragment tables the wavefront kernels read.
struct HostBasis {
  std::vector<float> P, enc64, dec64, dec64h, enc32, dec32, dec128, enc128;
};

void build_host_basis(int s, HostBasis* hb) {
  std::vector<double> P((size_t)s * s);
  const double pi = 3.14159265358979323846;
  for (int u = 0; u < s; ++u) {
    const double cu = u == 0 ? std::sqrt(1.0 / s) : std::sqrt(2.0 / s);
    for (int n = 0; n < s; ++n) P[(size_t)u * s + n] = cu * std::cos(pi * (2.0 * n + 1.0) * u / (2.0 * s));
  }
  hb->P.assign(P.begin(), P.end());   // one rounding to float32
  if (s == 64) {
    hb->enc64.resize(demo::kEnc64TableFloats);
    hb->dec64.resize(demo::kDec64TableFloats);
    demo::build_enc64_tables(P.data(), hb->enc64.data());
    demo::build_dec64_tables(P.data(), hb->dec64.data());
    hb->dec64h.resize(demo::kDec64DenseTableFloats);
    demo::build_dec64_dense_tables(P.data(), hb->dec64h.data());
  }
  if (s == 32) {
    // 64 x 64 block-diagonal basis diag(P32, P32): a wavefront tile holds 2 x 2 chunks
    std::vector<double> B2(64 * 64, 0.0);
    for (int blk = 0; blk < 2; ++blk)
      for (int u = 0; u < 32; ++u)
        for (int i = 0; i < 32; ++i) B2[(size_t)(32 * blk + u) * 64 + 32 * blk + i] = P[(size_t)u * 32 + i];
    hb->enc32.resize(demo::kEnc64dTableFloats);
    demo::build_enc64d_tables(B2.data(), hb->enc32.data());
    hb->dec32.resize(demo::kDec32TableFloats);
    demo::build_dec32_tables(P.data(), hb->dec32.data());
  }
  if (s == 128) {
    hb->dec128.resize(demo::kDec128TableFloats);
    demo::build_dec128_tables(P.data(), hb->dec128.data());
    hb->enc128.resize(demo::kEnc128TableFloats);
    demo::build_enc128_tables(P.data(), hb->enc128.data());
  }
}

int get_basis(demo_ctx* ctx, int s, demo::BasisTables* out) {
  for (const BasisTable& b : ctx->bases)
    if (b.s == s) {
      // the wavefront kernels are built on the symmetries of the DCT: any other matrix runs on the
      // kernels that read the matrix itself
      *out = b.use_custom ? demo::BasisTables{b.custom, nullptr, nullptr, nullptr, nullptr, false, b.custom_enc64, b.custom_dec64}
                          : demo::BasisTables{b.dev, b.enc64, b.dec64, b.enc32, b.dec32, true};
      if (!b.use_custom) { out->dec128 = b.dec128; out->enc128 = b.enc128; out->dec64g = b.dec64h; }
      return DEMO_OK;
    }
  HostBasis hb;
  build_host_basis(s, &hb);
  BasisTable b;
  b.s = s;
  int rc = upload(ctx, hb.P, &b.dev);
  if (rc != DEMO_OK) return rc;
  auto drop = [&]() {
    (void)hipFree(b.dev);
    if (b.enc64) (void)hipFree(b.enc64);
    if (b.dec64) (void)hipFree(b.dec64);
    if (b.dec64h) (void)hipFree(b.dec64h);
    if (b.enc32) (void)hipFree(b.enc32);
    if (b.dec32) (void)hipFree(b.dec32);
    if (b.dec128) (void)hipFree(b.dec128);
    if (b.enc128) (void)hipFree(b.enc128);
  };
  if (!hb.enc64.empty() && (rc = upload(ctx, hb.enc64, &b.enc64)) != DEMO_OK) { drop(); return rc; }
  if (!hb.dec64.empty() && (rc = upload(ctx, hb.dec64, &b.dec64)) != DEMO_OK) { drop(); return rc; }
  if (!hb.dec64h.empty() && (rc = upload(ctx, hb.dec64h, &b.dec64h)) != DEMO_OK) { drop(); return rc; }
  if (!hb.enc32.empty() && (rc = upload(ctx, hb.enc32, &b.enc32)) != DEMO_OK) { drop(); return rc; }
  if (!hb.dec32.empty() && (rc = upload(ctx, hb.dec32, &b.dec32)) != DEMO_OK) { drop(); return rc; }
  if (!hb.dec128.empty() && (rc = upload(ctx, hb.dec128, &b.dec128)) != DEMO_OK) { drop(); return rc; }
  if (!hb.enc128.empty() && (rc = upload(ctx, hb.enc128, &b.enc128)) != DEMO_OK) { drop(); return rc; }
  ctx->bases.push_back(b);
  *out = demo::BasisTables{b.dev, b.enc64, b.dec64, b.enc32, b.dec32, true};
  out->dec128 = b.dec128;
  out->enc128 = b.enc128;
  out->dec64g = b.dec64h;
  return DEMO_OK;
}

// Host image of the device tables of one tensor list.  `head` holds everything the kernels read before they
// write: per group of order-2 tensors [TensorDev x n][int32 prefix x (n+1)][queue header: count, ticket, 0, 0]
// [TensorDev x n in 64 x 64 tiles][int32 prefix], then the order-1 tables.  The queue lists (one int32 per order-2
// chunk) follow the head on the device and need no initial contents.
struct TableImage {
  struct Group {
    size_t o_d2 = 0, o_p2 = 0, o_wl = 0, o_d2t = 0, o_p2t = 0, o_list = 0;
    int32_t n = 0, total = 0, n_t = 0, total_t = 0;
    uint32_t mix = 0;
  };
  std::vector<char> head;
  std::vector<Group> groups;
  size_t o_d1 = 0, o_p1 = 0;
  int32_t n1 = 0, total1 = 0;
  uint32_t mix1 = 0;
  size_t total_bytes = 0;      // head + queue lists
  int64_t chunks2 = 0;         // order-2 chunks of the whole list
};

void build_image(const demo_tensor* t, int n, int s, TableImage* img) {
  struct HostGroup {
    uint32_t dt = 0;   // (gradient is bf16) | (parameter is bf16) << 1 | (s = 32 and not made of 64 x 64 tiles) << 2
    std::vector<TensorDev> d2, d2t;
    std::vector<int32_t> p2{0}, p2t{0};
    bool tiles_ok = true;
    uint32_t mix = 0;
  };
  std::vector<HostGroup> hg;
  std::vector<TensorDev> d1;
  std::vector<int32_t> p1(1, 0);
  uint32_t mix1 = 0;
  for (int i = 0; i < n; ++i) {
    const bool al16 = ((reinterpret_cast<uintptr_t>(t[i].idx) | reinterpret_cast<uintptr_t>(t[i].val)) & 15u) == 0;
    const uint32_t mix = (t[i].grad_dtype == DEMO_BF16 ? 1u : 2u) | (t[i].param_dtype == DEMO_BF16 ? 4u : 8u) | (al16 ? 0u : 16u);
    TensorDev d{};
    d.grad = t[i].grad;
    d.mom = t[i].mom;
    d.param = t[i].param;
    d.idx = t[i].idx;
    d.val = t[i].val;
    d.rows = t[i].rows;
    d.cols = t[i].cols;
    d.grad_bf16 = t[i].grad_dtype == DEMO_BF16;
    d.param_bf16 = t[i].param_dtype == DEMO_BF16;
    if (t[i].cols == 0) {
      mix1 |= mix;
      d.cchunks = 1;
      d.nchunks = (int32_t)(t[i].rows / s);
      d1.push_back(d);
      p1.push_back(p1.back() + d.nchunks);
    } else {
      // s = 32: tensors that the 64 x 64 tile kernels cannot take (a dimension not a multiple of 64) form groups
      // of their own, so that they do not pull the others onto the generic kernels
      const bool odd_tiles = s == 32 && (t[i].rows % 64 != 0 || t[i].cols % 64 != 0);
      const uint32_t dt = (d.grad_bf16 ? 1u : 0u) | (d.param_bf16 ? 2u : 0u) | (odd_tiles ? 4u : 0u);
      HostGroup* g = nullptr;
      for (HostGroup& x : hg)
        if (x.dt == dt) g = &x;
      if (g == nullptr) {
        hg.emplace_back();
        g = &hg.back();
        g->dt = dt;
        g->tiles_ok = s == 32;
      }
      g->mix |= mix;
      d.cchunks = (int32_t)(t[i].cols / s);
      d.nchunks = (int32_t)((t[i].rows / s) * (t[i].cols / s));
      g->d2.push_back(d);
      g->p2.push_back(g->p2.back() + d.nchunks);
      if (t[i].rows % 64 != 0 || t[i].cols % 64 != 0) g->tiles_ok = false;
      TensorDev dt64 = d;
      dt64.cchunks = (int32_t)(t[i].cols / 64);
      dt64.nchunks = (int32_t)((t[i].rows / 64) * (t[i].cols / 64));
      g->d2t.push_back(dt64);
      g->p2t.push_back(g->p2t.back() + dt64.nchunks);
    }
  }
  auto align16 = [](size_t x) { return (x + 15) & ~(size_t)15; };
  img->groups.clear();
  size_t off = 0;
  for (HostGroup& g : hg) {
    if (!g.tiles_ok) { g.d2t.clear(); g.p2t.assign(1, 0); }
    TableImage::Group ig;
    ig.o_d2 = off;
    ig.o_p2 = align16(ig.o_d2 + g.d2.size() * sizeof(TensorDev));
    ig.o_wl = align16(ig.o_p2 + g.p2.size() * sizeof(int32_t));   // count, ticket, pad, pad
    ig.o_d2t = align16(ig.o_wl + 4 * sizeof(int32_t));
    ig.o_p2t = align16(ig.o_d2t + g.d2t.size() * sizeof(TensorDev));
    off = align16(ig.o_p2t + g.p2t.size() * sizeof(int32_t));
    ig.n = (int32_t)g.d2.size();
    ig.total = g.p2.back();
    ig.n_t = (int32_t)g.d2t.size();
    ig.total_t = g.p2t.back();
    ig.mix = g.mix;
    img->groups.push_back(ig);
  }
  img->o_d1 = off;
  img->o_p1 = align16(img->o_d1 + d1.size() * sizeof(TensorDev));
  const size_t head_bytes = align16(img->o_p1 + p1.size() * sizeof(int32_t));
  img->n1 = (int32_t)d1.size();
  img->total1 = p1.back();
  img->mix1 = mix1;
  img->head.assign(head_bytes, 0);   // the queue headers start out zero
  img->chunks2 = 0;
  off = head_bytes;
  for (size_t gi = 0; gi < hg.size(); ++gi) {
    const HostGroup& g = hg[gi];
    TableImage::Group& ig = img->groups[gi];
    std::memcpy(img->head.data() + ig.o_d2, g.d2.data(), g.d2.size() * sizeof(TensorDev));
    std::memcpy(img->head.data() + ig.o_p2, g.p2.data(), g.p2.size() * sizeof(int32_t));
    if (!g.d2t.empty()) std::memcpy(img->head.data() + ig.o_d2t, g.d2t.data(), g.d2t.size() * sizeof(TensorDev));
    std::memcpy(img->head.data() + ig.o_p2t, g.p2t.data(), g.p2t.size() * sizeof(int32_t));
    ig.o_list = off;
    off = align16(off + (size_t)ig.total * sizeof(int32_t));
    img->chunks2 += ig.total;
  }
  if (!d1.empty()) std::memcpy(img->head.data() + img->o_d1, d1.data(), d1.size() * sizeof(TensorDev));
  std::memcpy(img->head.data() + img->o_p1, p1.data(), p1.size() * sizeof(int32_t));
  img->total_bytes = off;
}

// Views of an image that lives at `base` on the device.
void bind_image(const TableImage& img, char* base, std::vector<TableGroup>* groups, TableView* tv1) {
  groups->clear();
  for (const TableImage::Group& g : img.groups) {
    TableGroup tg;
    tg.tv2.descs = reinterpret_cast<const TensorDev*>(base + g.o_d2);
    tg.tv2.prefix = reinterpret_cast<const int32_t*>(base + g.o_p2);
    tg.tv2.n = g.n;
    tg.tv2.total_chunks = g.total;
    tg.tv2.dtypes = g.mix;
    tg.tv2t.descs = reinterpret_cast<const TensorDev*>(base + g.o_d2t);
    tg.tv2t.prefix = reinterpret_cast<const int32_t*>(base + g.o_p2t);
    tg.tv2t.n = g.n_t;
    tg.tv2t.total_chunks = g.total_t;
    tg.tv2t.dtypes = g.mix;
    int32_t* wl = reinterpret_cast<int32_t*>(base + g.o_wl);
    tg.wl = demo::Worklist{wl, wl + 1, reinterpret_cast<int32_t*>(base + g.o_list)};
    groups->push_back(tg);
  }
  tv1->descs = reinterpret_cast<const TensorDev*>(base + img.o_d1);
  tv1->prefix = reinterpret_cast<const int32_t*>(base + img.o_p1);
  tv1->n = img.n1;
  tv1->total_chunks = img.total1;
  tv1->dtypes = img.mix1;
}

// Find or build the device descriptor tables of a tensor list.  A table, once written, is never changed while its
// list stays cached (a captured graph may hold its address): a list seen before costs nothing; a new list takes a
// free or the least recently used slot.  While slots are free that is one allocation and one blocking copy; once
// all are in use the evicted slot's memory is reused when it is large enough, and the new table is then written
// by a small kernel on the call's stream, with no allocation and no host synchronisation (a caller whose buffers
// move every step ends up here).  Slots used under stream capture are never evicted.
int get_tables(demo_ctx* ctx, const demo_tensor* t, int n, int s, hipStream_t st, TableCache** out) {
  const size_t raw = sizeof(demo_tensor) * (size_t)n;
  std::vector<char> key(raw + sizeof(int));
  std::memcpy(key.data(), t, raw);
  std::memcpy(key.data() + raw, &s, sizeof(int));
  hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &cap) != hipSuccess) cap = hipStreamCaptureStatusNone;
  const bool capturing = cap == hipStreamCaptureStatusActive;
  for (TableCache& tc : ctx->tables) {
    if (tc.key.size() == key.size() && std::memcmp(tc.key.data(), key.data(), key.size()) == 0) {
      tc.last_use = ++ctx->use_counter;
      tc.many_streams = tc.many_streams || tc.last_stream != st;
      tc.last_stream = st;
      tc.pinned = tc.pinned || capturing;
      *out = &tc;
      return DEMO_OK;
    }
  }
  TableImage img;
  build_image(t, n, s, &img);
  TableCache* slot = nullptr;
  int unpinned = 0;
  for (const TableCache& tc : ctx->tables) unpinned += tc.pinned ? 0 : 1;
  if (unpinned < kMaxCachedTables) {
    ctx->tables.emplace_back();
    slot = &ctx->tables.back();
  } else {
    for (TableCache& tc : ctx->tables)
      if (!tc.pinned && (slot == nullptr || tc.last_use < slot->last_use)) slot = &tc;
    // kernels of the evicted list's last call may still read its table: later work on the same stream is ordered
    // behind them, any other stream is not
    if (slot->last_stream != st || slot->many_streams || slot->dev_bytes < img.total_bytes) {
      hipError_t e = hipDeviceSynchronize();
      if (e != hipSuccess) return fail_hip(ctx, e);
    }
  }
  slot->key.clear();
  if (slot->dev_bytes >= img.total_bytes) {
    hipError_t e = demo::device_write(slot->dev, img.head.data(), img.head.size(), st);
    if (e != hipSuccess) return fail_hip(ctx, e);
  } else {
    if (slot->dev) (void)hipFree(slot->dev);
    slot->dev = nullptr;
    slot->dev_bytes = 0;
    hipError_t e = hipMalloc(&slot->dev, img.total_bytes);
    if (e != hipSuccess) return fail_hip(ctx, e);
    slot->dev_bytes = img.total_bytes;
    // blocking copy: the table is complete before any launch on any stream reads it
    e = hipMemcpy(slot->dev, img.head.data(), img.head.size(), hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail_hip(ctx, e);
  }
  bind_image(img, static_cast<char*>(slot->dev), &slot->groups, &slot->tv1);
  slot->key.swap(key);
  slot->last_stream = st;
  slot->many_streams = false;
  slot->pinned = capturing;
  slot->last_use = ++ctx->use_counter;
  *out = slot;
  return DEMO_OK;
}

int timer_begin(demo_ctx* ctx, int which, hipStream_t st) {
  if (!ctx->timing) return DEMO_OK;
  const int slot = ctx->ev_count[which] % kMaxTimedLaunches;
  while ((int)ctx->ev[which][0].size() <= slot) {
    for (int j = 0; j < 2; ++j) {
      hipEvent_t e;
      hipError_t rc = hipEventCreate(&e);
      if (rc != hipSuccess) return fail_hip(ctx, rc);
      ctx->ev[which][j].push_back(e);
    }
  }
  hipError_t e = hipEventRecord(ctx->ev[which][0][slot], st);
  return e == hipSuccess ? DEMO_OK : fail_hip(ctx, e);
}

int timer_end(demo_ctx* ctx, int which, hipStream_t st) {
  if (!ctx->timing) return DEMO_OK;
  const int slot = ctx->ev_count[which] % kMaxTimedLaunches;
  hipError_t e = hipEventRecord(ctx->ev[which][1][slot], st);
  if (e != hipSuccess) return fail_hip(ctx, e);
  ctx->ev_count[which]++;
  return DEMO_OK;
}

int run_encode(demo_ctx* ctx, const std::vector<TableGroup>& groups, const TableView& tv1,
               const demo::BasisTables& basis, const demo_hparams& hp, int s, int k, hipStream_t st) {
  demo::EncodeArgs a{hp.beta, hp.grad_scale, hp.alpha, k, basis.dct ? 1 : 0, ctx->enc_stage};
  if (ctx->enc_stage != 0) {
    // the cut-down kernels exist for the s = 64 DCT kernel with bfloat16 gradients only
    if (s != 64 || !basis.dct || ctx->variant != 1 || k > demo::kFast64MaxK) return DEMO_ERR_UNSUPPORTED;
    for (const TableGroup& g : groups)
      if (g.tv2.dtypes & 2u) return DEMO_ERR_UNSUPPORTED;
  }
  int rc;
  if (!groups.empty()) {   // the timer brackets the launches of all groups
    if ((rc = timer_begin(ctx, 0, st)) != DEMO_OK) return rc;
    for (const TableGroup& g : groups) {
      hipError_t e = demo::launch_encode2d(g.tv2, g.tv2t.n > 0 ? &g.tv2t : nullptr, basis, s, a, g.wl, ctx->num_cus,
                                           ctx->variant, st);
      if (e != hipSuccess) return fail_hip(ctx, e);
    }
    if ((rc = timer_end(ctx, 0, st)) != DEMO_OK) return rc;
  }
  if (tv1.total_chunks > 0) {
    if ((rc = timer_begin(ctx, 1, st)) != DEMO_OK) return rc;
    hipError_t e = demo::launch_encode1d(tv1, basis.basis, s, a, st);
    if (e != hipSuccess) return fail_hip(ctx, e);
    if ((rc = timer_end(ctx, 1, st)) != DEMO_OK) return rc;
  }
  return DEMO_OK;
}

int run_decode(demo_ctx* ctx, TableCache* tc, const demo::BasisTables& basis, int W, const demo_hparams& hp, int s,
               int k, hipStream_t st) {
  const float scale = hp.aggregate == DEMO_AGG_MEAN ? 1.0f / (float)W : 1.0f;
  demo::DecodeArgs a{hp.lr, hp.weight_decay, scale, k, W, hp.phi, hp.aggregate, basis.dct ? 1 : 0, ctx->dec_stage};
  if (ctx->dec_stage != 0 && (s != 64 || ctx->variant != 1 || (int64_t)W * k <= 64 || (int64_t)W * k > 2048 || hp.aggregate == DEMO_AGG_COUNT))
    return DEMO_ERR_UNSUPPORTED;   // the cut-down runs exist in the s = 64 wavefront kernel with the payload in registers
  int rc;
  if (!tc->groups.empty()) {
    if ((rc = timer_begin(ctx, 2, st)) != DEMO_OK) return rc;
    for (const TableGroup& g : tc->groups) {
      hipError_t e = demo::launch_decode2d(g.tv2, g.tv2t.n > 0 ? &g.tv2t : nullptr, basis, s, a, ctx->num_cus,
                                           ctx->variant, st);
      if (e != hipSuccess) return fail_hip(ctx, e);
    }
    if ((rc = timer_end(ctx, 2, st)) != DEMO_OK) return rc;
  }
  if (tc->tv1.total_chunks > 0) {
    if ((rc = timer_begin(ctx, 3, st)) != DEMO_OK) return rc;
    hipError_t e = demo::launch_decode1d(tc->tv1, basis.basis, s, a, st);
    if (e != hipSuccess) return fail_hip(ctx, e);
    if ((rc = timer_end(ctx, 3, st)) != DEMO_OK) return rc;
  }
  return DEMO_OK;
}

// Scalars and modes of the _ex calls; `need` says which side's fields are used.
int check_hparams(const demo_hparams* hp, int need, int W) {
  if (hp == nullptr || hp->reserved != 0) return DEMO_ERR_ARG;
  if (need & NEED_ENCODE) {
    if (!std::isfinite(hp->beta) || !std::isfinite(hp->grad_scale) || !std::isfinite(hp->alpha)) return DEMO_ERR_ARG;
  }
  if (need & NEED_DECODE) {
    if (!std::isfinite(hp->lr) || !std::isfinite(hp->weight_decay)) return DEMO_ERR_ARG;
    if (hp->phi != DEMO_PHI_SIGN && hp->phi != DEMO_PHI_IDENTITY) return DEMO_ERR_ARG;
    if (hp->aggregate != DEMO_AGG_SUM && hp->aggregate != DEMO_AGG_MEAN && hp->aggregate != DEMO_AGG_COUNT)
      return DEMO_ERR_ARG;
    if (hp->aggregate == DEMO_AGG_COUNT && W > 255) return DEMO_ERR_ARG;
    // the aggregate is summed in block fixed point with 30 - ceil(log2 W) fractional bits: beyond this many workers
    // its rounding would show in the real-valued update of phi = identity (the sign update does not see it)
    if (hp->phi == DEMO_PHI_IDENTITY && W > DEMO_MAX_W_IDENTITY) return DEMO_ERR_UNSUPPORTED;
  }
  return DEMO_OK;
}

int prepare(demo_ctx* ctx, const demo_tensor* t, int n, int s, hipStream_t st, demo::BasisTables* basis,
            TableCache** tc) {
  int rc = bind_device(ctx);
  if (rc != DEMO_OK) return rc;
  if ((rc = get_basis(ctx, s, basis)) != DEMO_OK) return rc;
  return get_tables(ctx, t, n, s, st, tc);
}

}  // namespace

extern "C" {

int demo_create(demo_ctx** out) {
  if (out == nullptr) return DEMO_ERR_ARG;
  demo_ctx* c = new (std::nothrow) demo_ctx();
  if (c == nullptr) return DEMO_ERR_NOMEM;
  *out = c;
  return DEMO_OK;
}

int demo_destroy(demo_ctx* ctx) {
  if (ctx == nullptr) return DEMO_ERR_ARG;
  if (ctx->device >= 0) {
    (void)hipDeviceSynchronize();
    for (BasisTable& b : ctx->bases) {
      (void)hipFree(b.dev);
      if (b.enc64) (void)hipFree(b.enc64);
      if (b.dec64) (void)hipFree(b.dec64);
      if (b.dec64h) (void)hipFree(b.dec64h);
      if (b.enc32) (void)hipFree(b.enc32);
      if (b.dec32) (void)hipFree(b.dec32);
      if (b.dec128) (void)hipFree(b.dec128);
      if (b.enc128) (void)hipFree(b.enc128);
      if (b.custom) (void)hipFree(b.custom);
      if (b.custom_enc64) (void)hipFree(b.custom_enc64);
      if (b.custom_dec64) (void)hipFree(b.custom_dec64);
    }
    for (TableCache& tc : ctx->tables)
      if (tc.dev) (void)hipFree(tc.dev);
    for (int i = 0; i < kNumTimers; ++i)
      for (int j = 0; j < 2; ++j)
        for (hipEvent_t e : ctx->ev[i][j]) (void)hipEventDestroy(e);
  }
  delete ctx;
  return DEMO_OK;
}

int demo_payload_elems(int64_t rows, int64_t cols, int s, int k, int64_t* out) {
  if (out == nullptr) return DEMO_ERR_ARG;
  const int rc = check_shape(rows, cols, s, k);
  if (rc != DEMO_OK) return rc;
  const int64_t nchunks = cols == 0 ? rows / s : (rows / s) * (cols / s);
  *out = nchunks * k;
  return DEMO_OK;
}

int demo_hparams_default(demo_hparams* hp, float beta, float lr, float weight_decay) {
  if (hp == nullptr) return DEMO_ERR_ARG;
  hp->beta = beta;
  hp->grad_scale = 1.0f;
  hp->alpha = 1.0f;
  hp->lr = lr;
  hp->weight_decay = weight_decay;
  hp->phi = DEMO_PHI_SIGN;
  hp->aggregate = DEMO_AGG_SUM;
  hp->reserved = 0;
  return DEMO_OK;
}

int demo_encode_ex(demo_ctx* ctx, const demo_tensor* tensors, int n, const demo_hparams* hp, int s, int k,
                   void* hip_stream) {
  int rc = validate(ctx, tensors, n, s, k, NEED_ENCODE);
  if (rc != DEMO_OK) return rc;
  if ((rc = check_hparams(hp, NEED_ENCODE, 1)) != DEMO_OK || n == 0) return rc;
  demo::BasisTables basis{};
  TableCache* tc = nullptr;
  if ((rc = prepare(ctx, tensors, n, s, static_cast<hipStream_t>(hip_stream), &basis, &tc)) != DEMO_OK) return rc;
  return run_encode(ctx, tc->groups, tc->tv1, basis, *hp, s, k, static_cast<hipStream_t>(hip_stream));
}

int demo_decode_ex(demo_ctx* ctx, const demo_tensor* tensors, int n, int W, const demo_hparams* hp, int s, int k,
                   void* hip_stream) {
  int rc = validate(ctx, tensors, n, s, k, NEED_DECODE);
  if (rc != DEMO_OK) return rc;
  if (W < 1) return DEMO_ERR_ARG;
  if ((rc = check_hparams(hp, NEED_DECODE, W)) != DEMO_OK || n == 0) return rc;
  demo::BasisTables basis{};
  TableCache* tc = nullptr;
  if ((rc = prepare(ctx, tensors, n, s, static_cast<hipStream_t>(hip_stream), &basis, &tc)) != DEMO_OK) return rc;
  return run_decode(ctx, tc, basis, W, *hp, s, k, static_cast<hipStream_t>(hip_stream));
}

int demo_step_ex(demo_ctx* ctx, const demo_tensor* tensors, int n, const demo_hparams* hp, int s, int k,
                 void* hip_stream) {
  int rc = validate(ctx, tensors, n, s, k, NEED_ENCODE | NEED_DECODE);
  if (rc != DEMO_OK) return rc;
  if ((rc = check_hparams(hp, NEED_ENCODE | NEED_DECODE, 1)) != DEMO_OK || n == 0) return rc;
  demo::BasisTables basis{};
  TableCache* tc = nullptr;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if ((rc = prepare(ctx, tensors, n, s, st, &basis, &tc)) != DEMO_OK) return rc;
  if ((rc = run_encode(ctx, tc->groups, tc->tv1, basis, *hp, s, k, st)) != DEMO_OK) return rc;
  return run_decode(ctx, tc, basis, 1, *hp, s, k, st);
}

int demo_encode(demo_ctx* ctx, const demo_tensor* tensors, int n, float beta, int s, int k, void* hip_stream) {
  demo_hparams hp;
  demo_hparams_default(&hp, beta, 0.0f, 0.0f);
  return demo_encode_ex(ctx, tensors, n, &hp, s, k, hip_stream);
}

int demo_decode(demo_ctx* ctx, const demo_tensor* tensors, int n, int W, float lr, float weight_decay, int s,
                int k, void* hip_stream) {
  demo_hparams hp;
  demo_hparams_default(&hp, 0.0f, lr, weight_decay);
  return demo_decode_ex(ctx, tensors, n, W, &hp, s, k, hip_stream);
}

int demo_step(demo_ctx* ctx, const demo_tensor* tensors, int n, float beta, float lr, float weight_decay, int s,
              int k, void* hip_stream) {
  demo_hparams hp;
  demo_hparams_default(&hp, beta, lr, weight_decay);
  return demo_step_ex(ctx, tensors, n, &hp, s, k, hip_stream);
}

int demo_encode_noalloc(demo_ctx* ctx, const demo_tensor* tensors, int n, float beta, int s, int k,
                        void* hip_stream) {
  int rc = validate(ctx, tensors, n, s, k, NEED_ENCODE);
  if (rc != DEMO_OK) return rc;
  demo_hparams hp;
  demo_hparams_default(&hp, beta, 0.0f, 0.0f);
  if ((rc = check_hparams(&hp, NEED_ENCODE, 1)) != DEMO_OK || n == 0) return rc;
  // capacity of the static scratch array
  if (n > demo::kNoallocMaxTensors) return DEMO_ERR_LIMIT;
  int64_t chunks2 = 0;
  for (int i = 0; i < n; ++i)
    if (tensors[i].cols != 0) chunks2 += (tensors[i].rows / s) * (tensors[i].cols / s);
  if (chunks2 > demo::kNoallocMaxChunks) return DEMO_ERR_LIMIT;
  for (const BasisTable& b : ctx->bases)
    if (b.s == s && b.use_custom) return DEMO_ERR_UNSUPPORTED;   // the scratch array holds the DCT tables only
  if ((rc = bind_device(ctx)) != DEMO_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  void* base = nullptr;
  hipError_t e = demo::noalloc_scratch(ctx->device, &base);
  if (e != hipSuccess) return fail_hip(ctx, e);
  char* sc = static_cast<char*>(base);

  // basis tables of this chunk size: written once, kept until a call with another chunk size replaces them
  auto align256 = [](size_t x) { return (x + 255) & ~(size_t)255; };
  const size_t o_enc = align256((size_t)s * s * sizeof(float));
  if (demo::noalloc_basis_resident(ctx->device) != s) {
    HostBasis hb;
    build_host_basis(s, &hb);
    const std::vector<float>& enc = s == 64 ? hb.enc64 : s == 32 ? hb.enc32 : hb.enc128;
    if (o_enc + enc.size() * sizeof(float) > demo::kNoallocBasisBytes) return DEMO_ERR_LIMIT;
    demo::noalloc_set_basis_resident(ctx->device, 0);
    if ((e = demo::device_write(sc, hb.P.data(), hb.P.size() * sizeof(float), st)) != hipSuccess) return fail_hip(ctx, e);
    if (!enc.empty() && (e = demo::device_write(sc + o_enc, enc.data(), enc.size() * sizeof(float), st)) != hipSuccess)
      return fail_hip(ctx, e);
    demo::noalloc_set_basis_resident(ctx->device, s);
  }
  const float* P = reinterpret_cast<const float*>(sc);
  const float* enc = reinterpret_cast<const float*>(sc + o_enc);
  demo::BasisTables basis{P, s == 64 ? enc : nullptr, nullptr, s == 32 ? enc : nullptr, nullptr, true};
  if (s == 128) basis.enc128 = enc;

  // descriptor tables and queue headers of this call (the headers are zero in the image: the queue starts empty
  // whatever the last call left); the queue lists behind them need no initial contents
  TableImage img;
  build_image(tensors, n, s, &img);
  if (img.total_bytes > demo::kNoallocScratchBytes - demo::kNoallocBasisBytes) return DEMO_ERR_LIMIT;
  char* tb = sc + demo::kNoallocBasisBytes;
  if ((e = demo::device_write(tb, img.head.data(), img.head.size(), st)) != hipSuccess) return fail_hip(ctx, e);
  std::vector<TableGroup> groups;
  TableView tv1{};
  bind_image(img, tb, &groups, &tv1);
  const bool timing = ctx->timing;
  ctx->timing = false;   // timers create events on first use
  rc = run_encode(ctx, groups, tv1, basis, hp, s, k, st);
  ctx->timing = timing;
  return rc;
}

int demo_set_timing(demo_ctx* ctx, int enabled) {
  if (ctx == nullptr) return DEMO_ERR_ARG;
  ctx->timing = enabled != 0;
  for (int i = 0; i < kNumTimers; ++i) ctx->ev_count[i] = 0;   // a new measurement window starts
  return DEMO_OK;
}

int demo_last_kernel_ms(demo_ctx* ctx, int which, float* ms) {
  if (ctx == nullptr || ms == nullptr || which < 0 || which >= kNumTimers) return DEMO_ERR_ARG;
  const int n = ctx->ev_count[which] < kMaxTimedLaunches ? ctx->ev_count[which] : kMaxTimedLaunches;
  if (n == 0) return DEMO_ERR_ARG;
  double sum = 0.0;
  for (int i = 0; i < n; ++i) {
    hipError_t e = hipEventSynchronize(ctx->ev[which][1][i]);
    if (e != hipSuccess) return fail_hip(ctx, e);
    float one = 0.f;
    e = hipEventElapsedTime(&one, ctx->ev[which][0][i], ctx->ev[which][1][i]);
    if (e != hipSuccess) return fail_hip(ctx, e);
    sum += one;
  }
  *ms = (float)(sum / n);
  return DEMO_OK;
}

int demo_copy_probe(demo_ctx* ctx, void* dst, const void* src, int64_t nbytes, void* hip_stream) {
  if (ctx == nullptr || dst == nullptr || src == nullptr || nbytes < 0 || (nbytes & 15) != 0) return DEMO_ERR_ARG;
  if (((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15u) != 0) return DEMO_ERR_ARG;
  if (nbytes == 0) return DEMO_OK;
  int rc = bind_device(ctx);
  if (rc != DEMO_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  // timed like an encode order-1 launch would be: slot 1 of the timing window is reused for the probe
  if ((rc = timer_begin(ctx, 1, st)) != DEMO_OK) return rc;
  hipError_t e = demo::launch_copy_probe(src, dst, (size_t)nbytes, ctx->num_cus, st);
  if (e != hipSuccess) return fail_hip(ctx, e);
  return timer_end(ctx, 1, st);
}

int demo_stream_probe(demo_ctx* ctx, void* dst, const void* src, int64_t nbytes, int mode, void* hip_stream) {
  if (ctx == nullptr || dst == nullptr || src == nullptr || nbytes < 0 || (nbytes & 15) != 0) return DEMO_ERR_ARG;
  if (((reinterpret_cast<uintptr_t>(dst) | reinterpret_cast<uintptr_t>(src)) & 15u) != 0) return DEMO_ERR_ARG;
  if (mode < 0 || mode > 4) return DEMO_ERR_ARG;
  if (nbytes == 0) return DEMO_OK;
  int rc = bind_device(ctx);
  if (rc != DEMO_OK) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  if ((rc = timer_begin(ctx, 1, st)) != DEMO_OK) return rc;
  hipError_t e = demo::launch_stream_probe(src, dst, (size_t)nbytes, mode, ctx->num_cus, st);
  if (e != hipSuccess) return fail_hip(ctx, e);
  return timer_end(ctx, 1, st);
}

int demo_debug_set_encode_stage(demo_ctx* ctx, int stage) {
  if (ctx == nullptr || stage < 0 || stage > 3) return DEMO_ERR_ARG;
  ctx->enc_stage = stage;
  return DEMO_OK;
}

int demo_debug_set_decode_stage(demo_ctx* ctx, int stage) {
  if (ctx == nullptr || stage < 0 || stage > 2) return DEMO_ERR_ARG;
  ctx->dec_stage = stage;
  return DEMO_OK;
}

int demo_set_basis(demo_ctx* ctx, int s, int kind, const float* a_host) {
  if (ctx == nullptr) return DEMO_ERR_ARG;
  if (s != 32 && s != 64 && s != 128) return DEMO_ERR_UNSUPPORTED;
  if (kind != DEMO_BASIS_DCT && kind != DEMO_BASIS_IDENTITY && kind != DEMO_BASIS_GRAM_SCHMIDT) return DEMO_ERR_ARG;
  if (kind == DEMO_BASIS_GRAM_SCHMIDT && a_host == nullptr) return DEMO_ERR_ARG;
  std::vector<double> P;
  if (kind == DEMO_BASIS_IDENTITY) {
    P.assign((size_t)s * s, 0.0);
    for (int i = 0; i < s; ++i) P[(size_t)i * s + i] = 1.0;
  } else if (kind == DEMO_BASIS_GRAM_SCHMIDT) {
    // rows orthonormalised in order, in double: each row loses its components along the finished
    // rows one after the other, then is normalised
    P.assign(a_host, a_host + (size_t)s * s);
    for (int i = 0; i < s; ++i) {
      double* v = &P[(size_t)i * s];
      double n0 = 0.0;
      for (int c = 0; c < s; ++c) n0 += v[c] * v[c];
      if (!std::isfinite(n0)) return DEMO_ERR_ARG;
      for (int j = 0; j < i; ++j) {
        const double* q = &P[(size_t)j * s];
        double dot = 0.0;
        for (int c = 0; c < s; ++c) dot += q[c] * v[c];
        for (int c = 0; c < s; ++c) v[c] -= dot * q[c];
      }
      double n1 = 0.0;
      for (int c = 0; c < s; ++c) n1 += v[c] * v[c];
      if (!(n1 > 1e-20 * n0) || n0 == 0.0) return DEMO_ERR_ARG;   // rows (numerically) dependent
      const double inv = 1.0 / std::sqrt(n1);
      for (int c = 0; c < s; ++c) v[c] *= inv;
    }
  }
  int rc = bind_device(ctx);
  if (rc != DEMO_OK) return rc;
  demo::BasisTables unused{};
  if ((rc = get_basis(ctx, s, &unused)) != DEMO_OK) return rc;   // makes sure the entry of this s exists
  for (BasisTable& b : ctx->bases) {
    if (b.s != s) continue;
    if (kind == DEMO_BASIS_DCT) {
      b.use_custom = false;
      return DEMO_OK;
    }
    // kernels enqueued earlier may still read the matrix this call replaces
    hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) return fail_hip(ctx, e);
    const std::vector<float> host(P.begin(), P.end());   // one rounding to float32
    auto put = [&](const std::vector<float>& h, float** dev) -> int {
      if (*dev == nullptr) return upload(ctx, h, dev);
      hipError_t ee = hipMemcpy(*dev, h.data(), h.size() * sizeof(float), hipMemcpyHostToDevice);
      return ee == hipSuccess ? DEMO_OK : fail_hip(ctx, ee);
    };
    b.use_custom = false;
    if ((rc = put(host, &b.custom)) != DEMO_OK) return rc;
    if (s == 64) {
      // tables of the wavefront kernels' full-product instances, from the float32 matrix the other kernels read
      std::vector<double> Pr(host.begin(), host.end());
      std::vector<float> et(demo::kEnc64DenseTableFloats), dt(demo::kDec64DenseTableFloats);
      demo::build_enc64_dense_tables(Pr.data(), et.data());
      demo::build_dec64_dense_tables(Pr.data(), dt.data());
      if ((rc = put(et, &b.custom_enc64)) != DEMO_OK) return rc;
      if ((rc = put(dt, &b.custom_dec64)) != DEMO_OK) return rc;
    }
    b.use_custom = true;
    return DEMO_OK;
  }
  return DEMO_ERR_ARG;
}

int demo_set_variant(demo_ctx* ctx, int variant) {
  if (ctx == nullptr || variant < 0 || variant > 2) return DEMO_ERR_ARG;
  ctx->variant = variant;
  return DEMO_OK;
}

const char* demo_strerror(int status) {
  switch (status) {
    case DEMO_OK: return "ok";
    case DEMO_ERR_ARG: return "invalid argument (null pointer, n < 0, W < 1, k < 1 or k > chunk elements)";
    case DEMO_ERR_SHAPE: return "tensor shape is not a positive multiple of the chunk size";
    case DEMO_ERR_UNSUPPORTED: return "unsupported chunk size, dtype or k above DEMO_MAX_K";
    case DEMO_ERR_HIP: return "HIP runtime error";
    case DEMO_ERR_NOMEM: return "out of memory";
    case DEMO_ERR_LIMIT: return "tensor list beyond the fixed capacity of the allocation-free entry point";
  }
  return "unknown status";
}

const char* demo_last_hip_error(demo_ctx* ctx) {
  if (ctx == nullptr) return "no context";
  return hipGetErrorString(ctx->last_hip);
}

}  // extern "C"
