// Internal interface between the C-ABI host layer and the HIP kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

// Largest sparsity budget per chunk the kernels accept (equals DEMO_MAX_K of the public header).
#define DEMO_MAXK_INTERNAL 256

namespace demo {

// Device-side tensor descriptor (one per tensor of a call; order-2 and order-1
// tensors are kept in two separate tables).
struct TensorDev {
  const void* grad;
  float* mom;
  void* param;
  int32_t* idx;
  float* val;
  int64_t rows;
  int64_t cols;       // 0 for order-1
  int32_t cchunks;    // chunks along dimension 1 (order-2 only)
  int32_t nchunks;    // chunks of this tensor
  int32_t grad_bf16;
  int32_t param_bf16;
};

// A table on the device: `n` descriptors followed by n+1 int32 chunk prefix sums.
struct TableView {
  const TensorDev* descs;
  const int32_t* prefix;   // prefix[t] = first global chunk id of tensor t; prefix[n] = total
  int32_t n;
  int32_t total_chunks;
  uint32_t dtypes;         // bit 0: some gradient is bf16, 1: some is f32, 2: some parameter is bf16, 3: some is f32,
                           // bit 4: some payload pointer is not 16-byte aligned
};

// Chunks a fast kernel hands over to the exact generic kernel (device memory owned by the
// context, one per cached tensor list).  `count` and `ticket` are zero between calls.
struct Worklist {
  int32_t* count;
  int32_t* ticket;
  int32_t* list;     // capacity: total order-2 chunks of the tensor list
};

struct EncodeArgs {
  float beta;
  float grad_scale;   // m <- beta*m + grad_scale*g
  float alpha;        // m <- m - alpha*IDCT(kept)
  int k;
  int mirror;         // the projection matrix is the DCT (mirror-folded products allowed); set by the launch wrappers
  int stage;          // 0 = encode; 1..3 = cut-down copies of the s = 64 kernel for time attribution (debug interface)
};

struct DecodeArgs {
  float lr;
  float weight_decay;
  float scale;        // factor on the aggregate when phi is the identity: 1 (sum, count) or 1/W (mean)
  int k;
  int W;
  int phi;            // demo_phi
  int agg;            // demo_aggregate
  int mirror;         // as in EncodeArgs
  int stage;          // 0 = decode; 1, 2 = cut-down runs of the s = 64 wavefront kernel for time attribution (debug interface)
};
// The fast decode kernels aggregate by the plain sum (the mean is the sum times `scale`) and apply phi = sgn or
// the identity in their epilogues.  The count-normalised aggregate runs in them while a chunk's whole payload
// fits their registers (it is counted before it is summed), else on the generic kernels.
inline bool decode_is_sign_of_sum(const DecodeArgs& a) { return a.agg != 2; }
constexpr int kFast64CountMaxPairs = 2048;

// Device tables of one chunk size.
struct BasisTables {
  const float* basis;    // s x s orthonormal DCT-II matrix P, row-major float32
  const float* enc64;    // fragment tables of the wavefront-per-chunk encode kernel (s = 64 only, else null)
  const float* dec64;    // tables of the wavefront-per-chunk decode kernel (s = 64 only, else null)
  const float* enc32;    // dense-basis tile tables for diag(P32, P32) (s = 32 only, else null)
  const float* dec32;    // fragment table of the wavefront-per-tile decode kernel (s = 32 only, else null)
  bool dct;              // `basis` is the orthonormal DCT-II (false: a matrix set by the caller)
  const float* enc64g = nullptr;   // s = 64, matrix set by the caller: tables of the full-product wavefront kernels
  const float* dec64g = nullptr;
  const float* dec128 = nullptr;   // tables of the s = 128 decode kernel (DCT only, else null)
  const float* enc128 = nullptr;   // tables of the s = 128 encode kernel (DCT only, else null)
};

// Launch wrappers (demo_kernels.hip).  `variant` selects the kernel family:
// 0 = generic LDS-staged kernels, 1 = fastest available for this s and k.
// `tiles` (may be null): the same order-2 tensors counted in 64 x 64 tiles, present when s = 32 and
// every order-2 dimension is a multiple of 64.
hipError_t launch_encode2d(const TableView& tv, const TableView* tiles, const BasisTables& bt, int s,
                           const EncodeArgs& a, const Worklist& wl, int num_cus, int variant, hipStream_t stream);
hipError_t launch_encode1d(const TableView& tv, const float* basis, int s, const EncodeArgs& a,
                           hipStream_t stream);
hipError_t launch_decode2d(const TableView& tv, const TableView* tiles, const BasisTables& bt, int s,
                           const DecodeArgs& a, int num_cus, int variant, hipStream_t stream);
hipError_t launch_decode1d(const TableView& tv, const float* basis, int s, const DecodeArgs& a,
                           hipStream_t stream);

// demo_noalloc.hip: stream-ordered host-to-device write through kernel arguments, and the static scratch array
// of the entry point that allocates nothing.  Scratch layout: [basis tables of one chunk size][descriptor tables
// and queue headers][fallback queue, one int32 per order-2 chunk].
constexpr size_t kNoallocBasisBytes = 128 * 1024;
constexpr int kNoallocMaxTensors = 1024;
constexpr int kNoallocMaxChunks = 1 << 20;          // order-2 chunks per call
constexpr size_t kNoallocHeadBytes = 256 * 1024;    // descriptors of kNoallocMaxTensors tensors fit
constexpr size_t kNoallocScratchBytes = kNoallocBasisBytes + kNoallocHeadBytes + 4 * (size_t)kNoallocMaxChunks + 4096;
hipError_t device_write(void* dst, const void* host, size_t nbytes, hipStream_t stream);
hipError_t noalloc_scratch(int device, void** ptr);
int noalloc_basis_resident(int device);
void noalloc_set_basis_resident(int device, int s);

hipError_t launch_copy_probe(const void* src, void* dst, size_t nbytes, int num_cus, hipStream_t stream);
hipError_t launch_stream_probe(const void* src, void* dst, size_t nbytes, int mode, int num_cus, hipStream_t stream);

// s = 64 wavefront-per-chunk kernels (demo_enc64.hip, demo_dec64.hip).
constexpr int kEnc64TableFloats = 3072 + 4096 + 2048;
constexpr int kDec64TableFloats = 4096 + 1536 + 2048;
constexpr int kFast64MaxK = 64;
void build_enc64_tables(const double* P, float* out /* kEnc64TableFloats */);
void build_dec64_tables(const double* P, float* out /* kDec64TableFloats */);
// ... and their instances for a projection matrix without mirror symmetry: full products, other tables
constexpr int kEnc64DenseTableFloats = 16 * 512 + 2 * 4096;   // 16 pre-split float16 fragment blocks + the reconstruction's float32 rows
void build_enc64_dense_tables(const double* P, float* out /* kEnc64DenseTableFloats */);
hipError_t launch_encode2d_wave64(const TableView& tv, const float* tables, const EncodeArgs& a, const Worklist& wl,
                                  bool grad_bf16, bool dense, int num_cus, hipStream_t stream);
// dense-basis tile kernel (demo_enc64d.hip)
constexpr int kEnc64dTableFloats = 1024 + 4096 + 512;
void build_enc64d_tables(const double* B64, float* out /* kEnc64dTableFloats */);
hipError_t launch_encode2d_tile32(const TableView& tiles, const int32_t* prefix32, const float* tables,
                                  const EncodeArgs& a, const Worklist& wl, bool grad_bf16, int num_cus,
                                  hipStream_t stream);
// The decode kernel keeps all W workers' pairs of a chunk in registers: W <= 64 when k <= 32, W <= 32 above.
// s = 32 decode, one wavefront per 64 x 64 tile (2 x 2 chunks): the registers hold W*k <= 512 pairs per chunk
constexpr int kDec32TableFloats = 512;
constexpr int kFast32MaxPairs = 512;
// ... and streams larger payloads (k a multiple of 4, 16-byte aligned arrays, at most 65536 pairs per chunk)
inline bool fast32_decode_supports(int W, int k, bool payload_aligned16) {
  if (W < 1 || k < 1) return false;
  if ((int64_t)W * k <= kFast32MaxPairs) return true;
  return payload_aligned16 && k % 4 == 0 && (int64_t)W * k <= 65536;
}
void build_dec32_tables(const double* P32, float* out /* kDec32TableFloats */);
hipError_t launch_decode2d_tile32(const TableView& tiles, const float* tables, const DecodeArgs& a, bool param_bf16,
                                  int num_cus, hipStream_t stream);

// s = 128 kernels, one workgroup per chunk (demo_wg128.hip); they need the DCT (mirror-folded products).  The encode
// kernel reads the plain 128 x 128 basis, the decode kernel its own tables.
constexpr int kFast128MaxK = 64;
constexpr int kEnc128TableFloats = 2 * 8 * 512;   // pre-split float16 fragment blocks of the transposed even and odd rows of P
void build_enc128_tables(const double* P128, float* out /* kEnc128TableFloats */);
hipError_t launch_encode2d_wg128(const TableView& tv, const float* basis, const float* tables, const EncodeArgs& a,
                                 const Worklist& wl, bool grad_bf16, int num_cus, hipStream_t stream);
// decode keeps the W*k pairs of a chunk in eight registers per lane of its 512 threads
constexpr int kFast128MaxPairs = 4096;
constexpr int kDec128TableFloats = 2 * 8 * 512;   // pre-split float16 fragment blocks of the even and the odd rows of P
void build_dec128_tables(const double* P128, float* out /* kDec128TableFloats */);
// ... and streams larger payloads (k a multiple of 4, 16-byte aligned arrays, at most 65536 pairs per chunk)
inline bool fast128_decode_supports(int W, int k, bool payload_aligned16) {
  if (W < 1 || k < 1) return false;
  if ((int64_t)W * k <= kFast128MaxPairs) return true;
  return payload_aligned16 && k % 4 == 0 && (int64_t)W * k <= 65536;
}
hipError_t launch_decode2d_wg128(const TableView& tv, const float* basis, const float* tables, const DecodeArgs& a,
                                 bool param_bf16, int num_cus, hipStream_t stream);

// ... and streams larger payloads (k a multiple of 4, 16-byte aligned arrays, at most 65536 pairs per chunk).
inline bool fast64_decode_supports(int W, int k, bool payload_aligned16) {
  if (k > kFast64MaxK) return false;
  if ((int64_t)W * k <= 2048) return true;
  return payload_aligned16 && k % 4 == 0 && (int64_t)W * k <= 65536;
}
hipError_t launch_decode2d_wave64(const TableView& tv, const float* tables, const DecodeArgs& a, bool param_bf16,
                                  bool payload_aligned16, int num_cus, hipStream_t stream);
// ... and its instances for a projection matrix without mirror symmetry
constexpr int kDec64DenseTableFloats = 8 * 512;   // 8 pre-split float16 fragment blocks
void build_dec64_dense_tables(const double* P, float* out /* kDec64DenseTableFloats */);
bool dense64_decode_supports(const DecodeArgs& a);
hipError_t launch_decode2d_dense64(const TableView& tv, const float* tables, const DecodeArgs& a, bool param_bf16,
                                   bool payload_aligned16, int num_cus, hipStream_t stream);

}  // namespace demo
