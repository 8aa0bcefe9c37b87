// Device-side helpers shared by the kernel files.
#pragma once
#include "demo_internal.h"

namespace demo {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// Pointers read from a descriptor table are generic; these casts tell the compiler they
// are global memory so that it emits global_* rather than flat_* accesses.
#define DEMO_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ DEMO_GLOBAL T* as_global(T* p) {
  return (DEMO_GLOBAL T*)(p);
}
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ f32x4 gload_f4(const float* p) { return *(const DEMO_GLOBAL f32x4*)(p); }
__device__ __forceinline__ u32x2 gload_u2(const void* p) { return *(const DEMO_GLOBAL u32x2*)(p); }
// Payload loads of the decode kernels.  The payload is read once, so rows of a full 128-byte line or more
// (k >= 32) are fetched non-temporally; shorter rows share their lines with the neighbouring chunks that other
// wavefronts read at about the same time, and must stay in the cache for them (measured on the 1B-like set, W = 64:
// s = 32, k = 8 2.96 -> 2.05 ms and s = 64, k = 2 1.41 -> 1.22 ms with plain loads; k = 32 1 to 3 % the other way).
template <bool NT, class T>
__device__ __forceinline__ T payload_load(const DEMO_GLOBAL T* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
// Stores whose data registers stay untouched for two wait states behind them (see bstore_f4 below for why).
template <class T>
__device__ __forceinline__ void store_guarded(DEMO_GLOBAL T* p, T v) {
  *p = v;
#ifndef DEMO_NO_STORE_GUARD
  asm volatile("s_nop 1" ::"v"(v));
#endif
}
template <class T>
__device__ __forceinline__ void store_guarded(T* p, T v) {
  *p = v;
#ifndef DEMO_NO_STORE_GUARD
  asm volatile("s_nop 1" ::"v"(v));
#endif
}
__device__ __forceinline__ void gstore_f4(float* p, f32x4 v) { store_guarded((DEMO_GLOBAL f32x4*)(p), v); }
__device__ __forceinline__ void gstore_u2(void* p, u32x2 v) { store_guarded((DEMO_GLOBAL u32x2*)(p), v); }

// ---------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------
__device__ __forceinline__ int find_tensor(const int32_t* __restrict__ prefix, int n, int chunk) {
  int lo = 0, hi = n;  // invariant: prefix[lo] <= chunk < prefix[hi]
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (prefix[mid] <= chunk) lo = mid; else hi = mid;
  }
  return lo;
}

// Work item (chunk or tile) at which a wavefront of an 8-wavefront workgroup starts; it then advances by the
// number of wavefronts of the grid.  The workgroup takes 8 / RUN runs of RUN consecutive items that lie
// gridDim runs apart (RUN = 8: eight consecutive items).  Measured on the 1B-like set (same box, alternating
// runs): decode 1.60 / 1.49 / 1.41 / 1.44 ms and encode 1.95 / 1.89 / 1.89 / 1.90 ms for RUN = 1 / 2 / 4 / 8.
// Consecutive workgroups run on different XCDs (the dispatcher hands them out round robin), so neighbouring runs
// are streamed by different XCDs; giving each XCD a contiguous range of runs instead was measured and is slower
// (memory-stream-only copies of the kernels: encode 1.65 -> 1.68 ms, decode 1.37 -> 1.43 ms).
#ifndef DEMO_RUN
#define DEMO_RUN 4
#endif
template <int RUN>
__device__ __forceinline__ int first_work_item(int wave) {
  return RUN * ((int)blockIdx.x + (wave / RUN) * (int)gridDim.x) + (wave % RUN);
}

// The wavefront-per-chunk kernels walk the descriptor table with wavefront-uniform indices.  Reading
// the entries through the first active lane keeps them (and every address derived from them, e.g. a
// buffer resource descriptor) in scalar registers; without it the compiler must assume a divergent
// descriptor and wraps each buffer access in a loop over the distinct values.
//
// The walk from one tensor to the next (prefix sums, descriptors; `t` wavefront-uniform) reads the table through
// the constant address space, i.e. with scalar loads: the table is written before the launch and never during it.
// Read with vector loads, the walk's waits count in the same counter as the tensor loads and stores, and the
// point where the walk's rarely taken loop rejoins the chunk loop became a wait for everything outstanding.
typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr;
typedef const __attribute__((address_space(4))) uint32_t* const_u32_ptr;
__device__ __forceinline__ int uniform_i32(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ __forceinline__ int uniform_prefix(const TableView& tv, int t) {
  return (int)((const_i32_ptr)(uintptr_t)tv.prefix)[t];
}
__device__ __forceinline__ int find_tensor_uniform(const TableView& tv, int chunk) {
  return __builtin_amdgcn_readfirstlane(find_tensor(tv.prefix, tv.n, chunk));
}
__device__ __forceinline__ TensorDev load_desc_uniform(const TableView& tv, int t) {
  static_assert(sizeof(TensorDev) % 4 == 0, "descriptor is a whole number of dwords");
  constexpr int NW = sizeof(TensorDev) / 4;
  struct Words { uint32_t w[NW]; };
  const_u32_ptr p = (const_u32_ptr)(uintptr_t)(tv.descs + t);
  Words u;
#pragma unroll
  for (int i = 0; i < NW; ++i) u.w[i] = p[i];
  return __builtin_bit_cast(TensorDev, u);
}

__device__ __forceinline__ float bf16_to_f32(uint32_t h) { return __uint_as_float(h << 16); }

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t b = __float_as_uint(f);
  if ((b & 0x7fffffffu) > 0x7f800000u) return (b >> 16) | 0x40u;  // NaN stays NaN
  return (b + 0x7fffu + ((b >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ float4 load4(const void* __restrict__ base, int64_t off, int is_bf16) {
  if (is_bf16) {
    uint2 r = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(base) + off);
    return make_float4(bf16_to_f32(r.x & 0xffffu), bf16_to_f32(r.x >> 16), bf16_to_f32(r.y & 0xffffu),
                       bf16_to_f32(r.y >> 16));
  }
  return *reinterpret_cast<const float4*>(static_cast<const float*>(base) + off);
}

__device__ __forceinline__ void store4(void* __restrict__ base, int64_t off, int is_bf16, float4 v) {
  if (is_bf16) {
    u32x2 r;
    r[0] = f32_to_bf16_rne(v.x) | (f32_to_bf16_rne(v.y) << 16);
    r[1] = f32_to_bf16_rne(v.z) | (f32_to_bf16_rne(v.w) << 16);
    store_guarded(reinterpret_cast<u32x2*>(static_cast<uint16_t*>(base) + off), r);
  } else {
    store_guarded(reinterpret_cast<f32x4*>(static_cast<float*>(base) + off), (f32x4){v.x, v.y, v.z, v.w});
  }
}

// sgn(r) in {-1, 0, +1}: copy the sign bit onto 1.0, then zero it for r == +-0.
__device__ __forceinline__ float sgnf(float r) {
  const float s = __uint_as_float((__float_as_uint(r) & 0x80000000u) | 0x3f800000u);
  return r == 0.0f ? 0.0f : s;
}

// Two floats to packed bfloat16 (round to nearest even, hardware conversion on gfx950).
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// x' = x - lr*(sgn + wd*x) with two float32 fused multiply-adds (update line of Algorithm 1).
__device__ __forceinline__ float sign_update(float x, float sg, float lr, float wd) {
  float t = __fmaf_rn(wd, x, sg);
  return __fmaf_rn(-lr, t, x);
}

// Register layout shared by the s = 64 wavefront-per-chunk kernels.  Lane l = 16 g + c holds, for
// q = 4 s + w, the four consecutive elements (row rho(q, g), columns 4 chi(c) .. 4 chi(c) + 3), so
// that mirror quadruples {i, 31-i, 32+i, 63-i} of rows sit in one lane and those of columns in one
// aligned group of four lanes.  freq(t, m) is the frequency held by row / column m of coefficient
// tile t (tiles group frequencies by residue: 0 mod 4, 2 mod 4, odd).
__host__ __device__ constexpr int rho(int q, int g) {
  return (q & 3) == 0   ? 4 * (q >> 2) + g
         : (q & 3) == 1 ? 31 - (4 * (q >> 2) + g)
         : (q & 3) == 2 ? 32 + 4 * (q >> 2) + g
                        : 63 - (4 * (q >> 2) + g);
}
// rho(q, g) = rho_base(q) + (q even ? g : 3 - g)
__host__ __device__ constexpr int rho_base(int q) {
  return (q & 3) == 0 ? 4 * (q >> 2) : (q & 3) == 1 ? 28 - 4 * (q >> 2) : (q & 3) == 2 ? 32 + 4 * (q >> 2) : 60 - 4 * (q >> 2);
}
__host__ __device__ constexpr int chi(int c) {
  return (c & 3) == 0 ? (c >> 2) : (c & 3) == 1 ? 7 - (c >> 2) : (c & 3) == 2 ? 8 + (c >> 2) : 15 - (c >> 2);
}
__host__ __device__ constexpr int freq(int t, int m) {
  return t == 0 ? 4 * m : t == 1 ? 4 * m + 2 : t == 2 ? 2 * m + 1 : 2 * m + 33;
}

// Cache policy of the streaming tensor accesses (aux operand of the raw buffer intrinsics on gfx94x/95x:
// bit 0 = sc0, bit 1 = nt, bit 4 = sc1).  Every tensor element is touched once per call, so the accesses are
// marked non-temporal: measured +5 % on both s = 64 kernels against the default policy.
#ifndef DEMO_LOAD_AUX
#define DEMO_LOAD_AUX 3
#endif
#ifndef DEMO_STORE_AUX
#define DEMO_STORE_AUX 3
#endif

// Raw buffer access: a uniform base (resource descriptor in SGPRs) plus a 32-bit per-lane byte
// offset and a uniform byte offset.  Keeps per-lane addressing to one VGPR per access pattern.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7fffffff, 0x00020000);
}
// A buffer of zero records: every load from it returns zero and every store to it is dropped by the range check.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc_empty(const void* base) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0, 0x00020000);
}
__device__ __forceinline__ f32x4 bload_f4(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
  return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, DEMO_LOAD_AUX));
}
__device__ __forceinline__ u32x2 bload_u2(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff) {
  return __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(r, (int)voff, (int)soff, DEMO_LOAD_AUX));
}
// The data registers of a buffer store have to survive the instructions right behind it.  The compiler knows of
// no hazard there when the store has a scalar offset, yet on this part a VALU write to the first data register in
// the slot after the store has been seen to reach memory in its place (lanes 12-15 of every row of 16, now and
// then, in the first launches of a process).  The empty-operand asm keeps the registers live past two wait states.
__device__ __forceinline__ void bstore_f4(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff, f32x4 v) {
  const u32x4 u = __builtin_bit_cast(u32x4, v);
  __builtin_amdgcn_raw_buffer_store_b128(u, r, (int)voff, (int)soff, DEMO_STORE_AUX);
#ifndef DEMO_NO_STORE_GUARD
  asm volatile("s_nop 1" ::"v"(u));
#endif
}
__device__ __forceinline__ void bstore_u2(__amdgpu_buffer_rsrc_t r, uint32_t voff, uint32_t soff, u32x2 v) {
  __builtin_amdgcn_raw_buffer_store_b64(v, r, (int)voff, (int)soff, DEMO_STORE_AUX);
#ifndef DEMO_NO_STORE_GUARD
  asm volatile("s_nop 1" ::"v"(v));
#endif
}

__device__ __forceinline__ f32x4 mfma4(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// ---- float32 products on the float16 matrix pipe ------------------------------------------------------------------
// A float32 x whose magnitude is bounded is, to 2^-22 |x|, the sum of two float16 values: hi = rne16(x),
// lo = rne16(x - hi) (the remainder is exact in float32), as long as x's lowest bit is not below 2^-24, the spacing of
// the float16 subnormals, which conversion and matrix pipe both keep (checked on the device).  Three products
// hi hi + hi lo + lo hi on v_mfma_f32_16x16x32_f16 (16 cycles for 32 contraction indices, where v_mfma_f32_16x16x4_f32
// needs 32 cycles for 4) drop lo lo, 2^-22 of the product: float32 accumulation and a typical relative error of
// 2^-23 per term, that of a float32 multiply, at 3/16 of the float32 instructions' time.  (Three bfloat16 parts are
// exact for any float32 but need six products and five more vector instructions per element to form.)
// The callers scale so that nothing reaches 65504: basis entries (|P| <= 1) by 2^kSplitHBasisLog2, the data to below
// 2^8 (the decode's block fixed-point sums by construction, the encode's tile by a power of two taken from its
// largest magnitude), hence a first product below 2^4 sqrt(128) 2^8 < 2^15.6; the results carry these powers of two
// and are unscaled exactly.
// Operand layout: lane 16 g + c holds row (A) or column (B) c and eight contraction indices of group g, two per
// register; both operands number their eight indices alike, so any fixed assignment of indices to the eight
// slots serves as long as A and B share it.
typedef _Float16 h16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 h16x2 __attribute__((ext_vector_type(2)));
struct SplitH8 {
  u32x4 hi, lo;
};
constexpr int kSplitHBasisLog2 = 4;
// -1.0 in a scalar register that the compiler cannot see through: with it the remainder x - hi is written as
// fma(hi, -1, x), which the mixed-precision v_fma_mix_f32 takes straight from the packed float16 (one instruction
// instead of a conversion and a subtraction; the result is the same exact difference).  Formed once per kernel.
__device__ __forceinline__ float opaque_minus_one() {
  float m1;
  asm volatile("s_mov_b32 %0, 0xbf800000" : "=s"(m1));
  return m1;
}
__device__ __forceinline__ void split_pair_h(float x0, float x1, float m1, uint32_t& h, uint32_t& l) {
  const h16x2 hh = __builtin_convertvector((f32x2){x0, x1}, h16x2);
  const float r0 = __builtin_fmaf((float)hh[0], m1, x0), r1 = __builtin_fmaf((float)hh[1], m1, x1);
  const h16x2 ll = __builtin_convertvector((f32x2){r0, r1}, h16x2);
  h = __builtin_bit_cast(uint32_t, hh);
  l = __builtin_bit_cast(uint32_t, ll);
}
// `m1` = opaque_minus_one()
__device__ __forceinline__ SplitH8 split8h(float m1, float x0, float x1, float x2, float x3, float x4, float x5, float x6, float x7) {
  uint32_t h[4], l[4];
  split_pair_h(x0, x1, m1, h[0], l[0]);
  split_pair_h(x2, x3, m1, h[1], l[1]);
  split_pair_h(x4, x5, m1, h[2], l[2]);
  split_pair_h(x6, x7, m1, h[3], l[3]);
  return SplitH8{(u32x4){h[0], h[1], h[2], h[3]}, (u32x4){l[0], l[1], l[2], l[3]}};
}
__device__ __forceinline__ f32x4 mfma_f16(u32x4 a, u32x4 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h16x8, a), __builtin_bit_cast(h16x8, b), c, 0, 0, 0);
}
// c += a b from the split operands (smallest terms first)
__device__ __forceinline__ f32x4 mfma_split_h(const SplitH8& a, const SplitH8& b, f32x4 c) {
  c = mfma_f16(a.lo, b.hi, c);
  c = mfma_f16(a.hi, b.lo, c);
  return mfma_f16(a.hi, b.hi, c);
}
// pre-split fragment table: [part (hi, lo)][64 lanes] 16-byte entries
__device__ __forceinline__ SplitH8 load_split8h(const float* frag, int lane) {
  SplitH8 s;
  s.hi = *reinterpret_cast<const u32x4*>(frag + (0 * 64 + lane) * 4);
  s.lo = *reinterpret_cast<const u32x4*>(frag + (1 * 64 + lane) * 4);
  return s;
}
// Host: float16 code of a float32 (|f| < 65520), round to nearest even, subnormals kept.
inline uint16_t host_f16_rne(float f) {
  uint32_t b;
  __builtin_memcpy(&b, &f, 4);
  const uint16_t sign = (uint16_t)((b >> 16) & 0x8000u);
  const uint32_t a = b & 0x7fffffffu;
  if (a < 0x33000001u) return sign;                      // |f| <= 2^-25: rounds to zero
  if (a < 0x38800000u) {                                 // below 2^-14: subnormal, units of 2^-24
    const uint32_t man = (a & 0x7fffffu) | 0x800000u;    // 24-bit significand, value man * 2^(e - 150)
    const int shift = 126 - (int)(a >> 23);              // man >> shift counts units of 2^-24 (shift 14 .. 24)
    const uint32_t q = man >> shift, rem = man & ((1u << shift) - 1u), half = 1u << (shift - 1);
    return (uint16_t)(sign | (q + ((rem > half || (rem == half && (q & 1u))) ? 1u : 0u)));
  }
  const uint32_t r = a + 0xfffu + ((a >> 13) & 1u);      // round the 13 dropped bits, ties to even
  return (uint16_t)(sign | ((r - 0x38000000u) >> 13));
}
inline float host_f16_widen(uint16_t h) {
  const uint32_t e = (h >> 10) & 0x1fu, m = h & 0x3ffu;
  float mag = e == 0 ? (float)m * 0x1p-24f : __builtin_ldexpf((float)(m | 0x400u), (int)e - 25);
  return (h & 0x8000u) ? -mag : mag;
}
// Host: writes the pre-split fragment of one lane, eight values (already scaled), into a [part][64 lanes][4 words] block.
inline void host_store_split8h(float* frag, int lane, const float v[8]) {
  uint32_t* w = reinterpret_cast<uint32_t*>(frag);
  for (int j = 0; j < 8; ++j) {
    uint16_t p[2];
    p[0] = host_f16_rne(v[j]);
    p[1] = host_f16_rne(v[j] - host_f16_widen(p[0]));
    for (int part = 0; part < 2; ++part) {
      uint32_t& word = w[(part * 64 + lane) * 4 + (j >> 1)];
      word = (j & 1) ? (word & 0x0000ffffu) | ((uint32_t)p[part] << 16) : (word & 0xffff0000u) | p[part];
    }
  }
}
constexpr int kSplitHFragFloats = 2 * 64 * 4;   // words of one pre-split float16 fragment block

// LDS operations of one wavefront execute in order; this only stops the compiler from moving
// LDS accesses across the point.
__device__ __forceinline__ void wave_lds_sync() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// LDS accessed through a 32-bit byte address
typedef __attribute__((address_space(3))) uint32_t lds_u32;
__device__ __forceinline__ lds_u32* lds_u32_at(uint32_t byte_address) { return (lds_u32*)(uintptr_t)byte_address; }

// The lane id formed on the spot (two VALU instructions, nothing kept alive for it).  For per-lane constants that are
// needed late in a long loop body: derived from threadIdx they stay live across the whole body, and where the body
// is short of registers they are spilled, which costs a wait for every load in flight at each reload.
__device__ __forceinline__ int fresh_lane_id() {
  int x;
  asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(x));
  return x;
}

// number of lanes below this one whose bit is set in mask
__device__ __forceinline__ int lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// Optional per-phase cycle accounting (profiling builds only: -DDEMO_PHASE_CLOCKS).  A kernel
// marks phase boundaries with DEMO_PHASE(i); lane 0 of every wavefront adds its totals to
// demo_phase_clocks[] when the kernel ends.
#ifdef DEMO_PHASE_CLOCKS
static __device__ unsigned long long demo_phase_clocks[16];   // one copy per translation unit
#define DEMO_PHASE_GETTER(name)                                                                              \
  extern "C" int name(unsigned long long* out16, int reset) {                                               \
    hipError_t e = hipMemcpyFromSymbol(out16, HIP_SYMBOL(demo::demo_phase_clocks), 16 * sizeof(unsigned long long)); \
    if (e == hipSuccess && reset) {                                                                         \
      unsigned long long z[16] = {};                                                                        \
      e = hipMemcpyToSymbol(HIP_SYMBOL(demo::demo_phase_clocks), z, sizeof(z));                             \
    }                                                                                                       \
    return e == hipSuccess ? 0 : -4;                                                                        \
  }
#define DEMO_PHASE_DECL unsigned long long ph_acc[8] = {0, 0, 0, 0, 0, 0, 0, 0}; unsigned long long ph_t = __builtin_readcyclecounter();
#define DEMO_PHASE(i)                                             \
  do {                                                            \
    __builtin_amdgcn_sched_barrier(0);                            \
    const unsigned long long ph_now = __builtin_readcyclecounter(); \
    ph_acc[i] += ph_now - ph_t;                                   \
    ph_t = ph_now;                                                \
    __builtin_amdgcn_sched_barrier(0);                            \
  } while (0)
#define DEMO_PHASE_FLUSH(off)                                                              \
  do {                                                                                     \
    if ((threadIdx.x & 63) == 0)                                                           \
      for (int ph_i = 0; ph_i < 8; ++ph_i) atomicAdd(&demo_phase_clocks[(off) + ph_i], ph_acc[ph_i]); \
  } while (0)
#elif defined(DEMO_PHASE_MARKS)
// -DDEMO_PHASE_MARKS: the phase boundaries only leave a comment in the generated assembly (for counting the
// instructions of each phase in a -save-temps listing); the code is the ordinary build's up to scheduling
#define DEMO_PHASE_GETTER(name)
#define DEMO_PHASE_DECL
#define DEMO_PHASE(i) asm volatile("; PHASE_MARK " #i)
#define DEMO_PHASE_FLUSH(off)
#else
#define DEMO_PHASE_GETTER(name)
#define DEMO_PHASE_DECL
#define DEMO_PHASE(i)
#define DEMO_PHASE_FLUSH(off)
#endif

}  // namespace demo
