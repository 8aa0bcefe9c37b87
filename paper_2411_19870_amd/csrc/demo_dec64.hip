// s = 64 decode kernel: one wavefront per 64 x 64 chunk.
//
// R = P^T S P for the coefficient sums S of the W payloads, with both basis products reduced to 3/8
// of their dense size by the mirror symmetries of the DCT-II basis:
//   rows u = 0 mod 4 of P are even under i -> 63-i and under i -> 31-i,
//   rows u = 2 mod 4 are even under i -> 63-i and odd under i -> 31-i,
//   odd rows are odd under i -> 63-i,
// so for a mirror quadruple {i0, 31-i0, 32+i0, 63-i0} (i0 < 16) only four partial sums are needed
// (ee: u = 0 mod 4 at i0; eo: u = 2 mod 4 at i0; o0, o1: odd u at i0 and at 31-i0):
//   out[i0] = ee+eo+o0, out[31-i0] = ee-eo+o1, out[32+i0] = ee-eo-o1, out[63-i0] = ee+eo-o0.
// The same holds for the columns.  Both products therefore keep the four members of a quadruple
// in one lane: lane l = 16 g + c ends up with the elements
//   rows    member(w, 4 s + g)        s, w  = 0..3   (16 rows)
//   columns member(w', kappa(c))      w'    = 0..3   ( 4 columns).
// Accessing the parameters in that layout would take 2- or 4-byte accesses, and the address path of
// the CU (one wavefront instruction per 16 cycles whatever its width) then limits the kernel, so R
// is passed once through the LDS tile of S (dead by then) into the layout of the encode kernel
// (demo_device.h: rows rho(q, g), columns 4 chi(c) .. +3), where every load and store instruction
// covers whole 128- or 256-byte rows, and the sign update is fused there.
//
// S is accumulated in a private LDS tile in block fixed point with integer atomics (see `scatter`
// below); its rows and columns are stored grouped by residue mod 4 (physical index
// 16 (u % 4) + u / 4), which is what the partial sums contract over.  The products run as chains of
// v_mfma_f32_16x16x4_f32:
//   product a   per row tile t (rows u = 4 m + t):  ee/eo/o0/o1[u][j0] = sum over one residue class
//               of v of S[u][v] P[v][.]; A = S from LDS, B = basis fragments G; then the four
//               column members Y[u][member(w', j0)] by in-lane adds.
//   product b   per w':  Cee/Ceo/Co0/Co1[i0][j] += G (as A) * Y tile (accumulators as B operand),
//               row tile t feeding the class t belongs to; the four row members by in-lane adds.
// Both products use the same fragment table G (6 groups x 64 lanes x 4 floats).
#include "demo_device.h"

namespace demo {

namespace {
constexpr int D64_WAVES = 8;                       // 8 private tiles + the fragment table fill the LDS
constexpr int D64_THREADS = D64_WAVES * 64;
constexpr int D64_LDT = 68;                        // tile row stride (floats); columns 64..67 are pad slots
constexpr int D64_TILE_FLOATS = 64 * D64_LDT;
constexpr int D64_PCOL = 0;                        // pcol[v*64 + 4c + e] = P[v][4 chi(c) + e]       (sparse kernel)
constexpr int D64_G = 4096;                        // fragment table G of the dense kernel
constexpr int D64_G_FLOATS = 1536;
constexpr int D64_PK = 4096 + 1536;                // pk[u*16 + c]  = P[u][kappa(c)]       (sparse kernel: quadruple bases)
constexpr int D64_PK2 = 4096 + 1536 + 1024;        // pk2[u*16 + c] = P[u][31 - kappa(c)]  (odd u: the second member)
constexpr int D64_ALL_TABLE_FLOATS = 4096 + 1536 + 2048;
constexpr int D64_LDS_BYTES = 4 * (D64_G_FLOATS + D64_WAVES * D64_TILE_FLOATS);
// Instances for a projection matrix without mirror symmetry (DENSE).  Both products run on the float16 matrix pipe
// with every float32 operand split into two parts (demo_device.h), and one table of pre-split basis fragments (scaled
// by 2^kSplitHBasisLog2) serves both: block 2 t + h (kSplitHFragFloats words), slot j of contraction group g holds
//   P[16 (2 h + j / 4) + 4 g + j % 4][16 t + c]
// (product a: B operand, contracts v = 16 a + 4 g + b with (a, b) = (2 h + j / 4, j % 4), output columns
// j = 16 t + c; product b: A operand, contracts u = 16 a + 4 g + b, output rows i = 16 t + c).
constexpr int D64G_FLOATS = 8 * kSplitHFragFloats;
static_assert(D64G_FLOATS == kDec64DenseTableFloats, "table size");
template <bool DENSE>
constexpr int d64_table_floats() { return DENSE ? D64G_FLOATS : D64_G_FLOATS; }
template <bool DENSE>
constexpr int d64_lds_bytes() { return 4 * (d64_table_floats<DENSE>() + D64_WAVES * D64_TILE_FLOATS); }
static_assert(d64_lds_bytes<true>() <= 160 * 1024, "LDS budget");
static_assert(D64_ALL_TABLE_FLOATS == kDec64TableFloats, "table size");
static_assert(D64_LDS_BYTES <= 160 * 1024, "LDS budget");

// column (and product-b output row) base index served by lane c of a 16-lane group
__host__ __device__ constexpr int kappa(int c) { return 4 * (c & 3) + (c >> 2); }
// member w of the mirror quadruple with base i0 < 16
__host__ __device__ constexpr int member(int w, int i0) {
  return w == 0 ? i0 : w == 1 ? 31 - i0 : w == 2 ? 32 + i0 : 63 - i0;
}
}  // namespace

void build_dec64_dense_tables(const double* P, float* out) {
  for (int t = 0; t < 4; ++t)
    for (int h = 0; h < 2; ++h)
      for (int lane = 0; lane < 64; ++lane) {
        float v[8];
        for (int j = 0; j < 8; ++j)
          v[j] = (float)__builtin_ldexp(P[(16 * (2 * h + (j >> 2)) + 4 * (lane >> 4) + (j & 3)) * 64 + 16 * t + (lane & 15)],
                                        kSplitHBasisLog2);
        host_store_split8h(out + (2 * t + h) * kSplitHFragFloats, lane, v);
      }
}

// Host: tables of the decode kernels from the 64 x 64 basis P (double, row-major).
void build_dec64_tables(const double* P, float* out) {
  auto Pm = [&](int u, int i) { return (float)P[u * 64 + i]; };
  for (int v = 0; v < 64; ++v)
    for (int cc = 0; cc < 16; ++cc)
      for (int e = 0; e < 4; ++e) out[D64_PCOL + v * 64 + 4 * cc + e] = Pm(v, 4 * chi(cc) + e);
  for (int u = 0; u < 64; ++u)
    for (int cc = 0; cc < 16; ++cc) {
      out[D64_PK + u * 16 + cc] = Pm(u, kappa(cc));
      out[D64_PK2 + u * 16 + cc] = Pm(u, 31 - kappa(cc));
    }
  // G: lane (g, c), component r.  The contraction index of k-slot g at step r is 4 (4 g + r) + class,
  // the other index is kappa(c) (groups 0..3) or 31 - kappa(c) (groups 4, 5: odd classes only).
  for (int lane = 0; lane < 64; ++lane) {
    const int g = lane >> 4, c = lane & 15, kap = kappa(c);
    for (int r = 0; r < 4; ++r) {
      const int u4 = 4 * (4 * g + r);
      out[D64_G + (0 * 64 + lane) * 4 + r] = Pm(u4 + 0, kap);
      out[D64_G + (1 * 64 + lane) * 4 + r] = Pm(u4 + 2, kap);
      out[D64_G + (2 * 64 + lane) * 4 + r] = Pm(u4 + 1, kap);
      out[D64_G + (3 * 64 + lane) * 4 + r] = Pm(u4 + 3, kap);
      out[D64_G + (4 * 64 + lane) * 4 + r] = Pm(u4 + 1, 31 - kap);
      out[D64_G + (5 * 64 + lane) * 4 + r] = Pm(u4 + 3, 31 - kap);
    }
  }
}

// PBF16: parameter dtype of every tensor in the table.  MODE 1: k == 32 and W == 64, the payload of a chunk is
// read with eight fully populated 16-byte loads per array (eight workers each).  MODE 2: k == 32 and W a smaller
// multiple of 8: the first W / 8 of those loads.  MODE 3 / 4: k a multiple of 4 / 2, any W: a lane fetches 4 / 2
// consecutive pairs of one worker per load (unit 64 j + lane of the chunk's W k pairs in worker-major order).
// MODE 0: any k <= 64, W * k <= 2048, one pair per load (unit-wise like modes 3 and 4).  MODE 5: k a multiple of 4 and more than 2048 pairs per
// chunk (up to 65536): the payload is streamed once, in rounds of 2048 pairs, the sums being shifted down whenever a
// round raises the block exponent; the first round of the next chunk is fetched during the products.
// Modes 1 to 5 need 16-byte aligned payload arrays.
// IDENT: phi is the identity on the aggregate instead of sgn (its own instance, so that the sign kernels carry
// nothing for it).  COUNT: the count-normalised aggregate of the appendix algorithm "Sparse Top-k Averaging" (every
// coefficient's sum divided by the number of pairs that name it), modes 0, 3 and 4 only.  NT: the 16- and 8-byte
// payload loads of modes 3 to 5 are non-temporal (the launch wrapper asks for that when a row of k pairs fills a
// 128-byte line; shorter rows share lines with neighbouring chunks and stay cached).
// DENSE: any orthonormal 64 x 64 matrix (table of build_dec64_dense_tables): the tile holds S in its natural order,
// both products are full (on the float16 matrix pipe, float32 operands split into two parts: 96
// v_mfma_f32_16x16x32_f16 each), R goes through the tile in its natural order.
template <bool PBF16, int MODE, bool IDENT, bool COUNT = false, bool NT = true, bool DENSE = false>
__global__ __launch_bounds__(D64_THREADS) void decode2d_wave64(TableView tv, const float* __restrict__ tables,
                                                               DecodeArgs args) {
  extern __shared__ float lds[];
  const float* sG = lds;
  constexpr int G_FLOATS = d64_table_floats<DENSE>();
  constexpr bool DENSE_LATE_X = false;   // (the full-product instances once had no registers for the parameters before their products)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, c = lane & 15;
  float* tile = lds + G_FLOATS + wave * D64_TILE_FLOATS;
  int* itile = reinterpret_cast<int*>(tile);
  constexpr bool FULL = MODE == 1;          // every payload register is in use
  constexpr bool WIDE = MODE == 1 || MODE == 2;   // 16-byte payload loads, eight workers per load
  constexpr int VW = (MODE == 3 || MODE == 5) ? 4 : MODE == 4 ? 2 : 1;   // pairs per load of the unit-wise modes
  constexpr bool UNITS = MODE >= 3 || MODE == 0;   // unit 64 j + lane of the chunk's pairs, VW pairs per unit
  constexpr bool STREAM = MODE == 5;        // more pairs than the registers hold: rounds of 2048
  const int k = WIDE ? 32 : args.k, W = args.W;
  [[maybe_unused]] const float m1h = opaque_minus_one();

  for (int e = tid; e < G_FLOATS / 4; e += D64_THREADS)
    reinterpret_cast<float4*>(lds)[e] = reinterpret_cast<const float4*>(tables + (DENSE ? 0 : D64_G))[e];
  __syncthreads();

  const int nwaves = gridDim.x * D64_WAVES;
  const int wid = first_work_item<DEMO_RUN>(wave);
  const int total = tv.total_chunks;
  int chunk = wid;   // wavefront w takes chunks w, w + nwaves, ... (see the encode kernel)
  if (chunk >= total) return;

  // ---- payload access ---------------------------------------------------------------------------------
  // 32 (index, value) pairs per lane hold the whole payload of a chunk (W * k <= 2048 pairs).
  //   WIDE:  load j (0..7) fetches pairs 4(l%8) .. +3 of worker 8j + l/8 as one 16-byte load;
  //   else:  load j fetches unit 64 j + l of the chunk's W k / VW units in worker-major order (VW pairs each).
  constexpr int NP = 32;
  int32_t pi[NP];
  float pv[NP];
#pragma unroll
  for (int j = 0; j < NP; ++j) {   // registers past the W workers are never loaded and stay empty
    pi[j] = -1;
    pv[j] = 0.f;
  }
  const int nunits = (W * k) / VW;                                   // UNITS: loads per array and chunk
  const int nloads = STREAM ? NP / VW : (nunits + 63) >> 6;          // ... per lane (STREAM: per round)
  const int nrounds = (nunits + 64 * (NP / VW) - 1) / (64 * (NP / VW));
  const float rk = 1.0f / (float)k;
  const int nact = FULL ? NP : WIDE ? W / 2 : VW * nloads;   // payload registers in use (uniform)
  const int sub = lane >> 3, pt = 4 * (lane & 7);              // WIDE: worker within the load, first pair
  // `round` matters in STREAM mode only: units 512 round + 64 j + lane
  auto load_payload = [&](const TensorDev& dd, int ccc, int round = 0) {
    const int64_t wstride = (int64_t)dd.nchunks * k;
    const uint32_t lane_off = (uint32_t)(sub * (int)wstride + pt);
    const DEMO_GLOBAL int32_t* ip = as_global(dd.idx) + (int64_t)ccc * k;
    const DEMO_GLOBAL float* vp = as_global(dd.val) + (int64_t)ccc * k;
    if constexpr (UNITS) {
      // worker and position of a unit are formed anew at every call (kept across the chunk loop they would be
      // spilled, and the reload of a spilled value waits for every load in flight)
      int lanev = lane;
      asm volatile("" : "+v"(lanev));
      {
#pragma unroll
        for (int j = 0; j < NP / VW; ++j) {
          if (j < nloads) {   // uniform
            const int unit = (STREAM ? 64 * (NP / VW) * round : 0) + 64 * j + lanev;
            const int p = VW * unit;
            // worker p / k and position p % k; (p + 1/2) / k is never within 1/(2k) of an integer, far more than
            // the rounding error of the float product for p < 65536
            const int w = (int)(((float)p + 0.5f) * rk);
            const int pos = p - w * k;
            const bool ok = unit < nunits;
            const uint32_t off = ok ? (uint32_t)(w * (int)wstride + pos) : 0u;
            // The loads are unconditional (a unit past the end reads the chunk's first pairs) and what they bring
            // is taken as it is: mask_payload discards the units past the end where the pairs are consumed.  A
            // select right behind a load makes the wavefront wait for that load before it issues the next one.
            if constexpr (VW == 4) {
              const f32x4 b = payload_load<NT>(reinterpret_cast<const DEMO_GLOBAL f32x4*>(vp + off));
#pragma unroll
              for (int x = 0; x < 4; ++x) pv[4 * j + x] = b[x];
              const u32x4 a = payload_load<NT>(reinterpret_cast<const DEMO_GLOBAL u32x4*>(ip + off));
#pragma unroll
              for (int x = 0; x < 4; ++x) pi[4 * j + x] = (int32_t)a[x];
            } else if constexpr (VW == 2) {
              const u32x2 a = payload_load<NT>(reinterpret_cast<const DEMO_GLOBAL u32x2*>(ip + off));
              const f32x2 b = payload_load<NT>(reinterpret_cast<const DEMO_GLOBAL f32x2*>(vp + off));
#pragma unroll
              for (int x = 0; x < 2; ++x) {
                pi[2 * j + x] = (int32_t)a[x];
                pv[2 * j + x] = b[x];
              }
            } else {   // one pair per load: any k, arrays with their natural alignment only
              pi[j] = ip[off];
              pv[j] = vp[off];
              // the 32 offsets are formed eight at a time (all at once they would not fit the registers)
              if ((j & 7) == 7) __builtin_amdgcn_sched_barrier(0);
            }
          }
        }
      }
    } else if (WIDE) {
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        if (FULL || 4 * j < nact) {
          const u32x4 a = payload_load<true>(reinterpret_cast<const DEMO_GLOBAL u32x4*>(ip + lane_off));
          const f32x4 b = payload_load<true>(reinterpret_cast<const DEMO_GLOBAL f32x4*>(vp + lane_off));
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            pi[4 * j + x] = (int32_t)a[x];
            pv[4 * j + x] = b[x];
          }
          ip += 8 * wstride;
          vp += 8 * wstride;
        }
      }
    }
  };

  // Units past the end of the chunk's payload (the last load of a lane may reach beyond W k pairs) become
  // (no index, 0); called where the pairs are consumed.
  auto mask_payload = [&](int round = 0) {
    if constexpr (UNITS) {
      int lanev = lane;
      asm volatile("" : "+v"(lanev));
#pragma unroll
      for (int j = 0; j < NP / VW; ++j) {
        if (j < nloads) {   // uniform
          const bool ok = (STREAM ? 64 * (NP / VW) * round : 0) + 64 * j + lanev < nunits;
#pragma unroll
          for (int x = 0; x < VW; ++x) {
            pi[VW * j + x] = ok ? pi[VW * j + x] : -1;
            pv[VW * j + x] = ok ? pv[VW * j + x] : 0.f;
          }
        }
      }
    }
  };

  // S[idx] += val in block fixed point.  LDS float atomics are an order of magnitude slower than
  // integer ones on this part, and an integer sum does not depend on the order of arrival, so the
  // coefficients are scaled by a power of two taken from the largest magnitude of the chunk's
  // payload (exact), rounded to integers of `vbits` bits and added with ds_add_u32; W such values
  // cannot overflow 31 bits.  Only sgn(IDCT(S)) is used, so the scale is never undone.  Lanes with
  // nothing to add (inactive pair, index out of range) add zero-weight garbage into their pad slot.
  // Coefficient (u, v) lives at tile[(16 (u%4) + u/4) * LDT + 16 (v%4) + v/4].
  const uint32_t dummy = (uint32_t)(lane * D64_LDT + 64);
  int vbits = 30;
  for (int w = 1; w < W; w <<= 1) --vbits;                // 30 - ceil(log2 W)
  auto lane_max = [&](float mx) {
#pragma unroll
    for (int j = 0; j < NP; ++j)
      if (FULL || j < nact) mx = fmaxf(mx, fabsf(pv[j]));
    return mx;
  };
  // shift of the block fixed point from the lanes' largest magnitudes
  auto shift_of = [&](float mx) {
    uint32_t mb = __float_as_uint(mx);
    mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
    mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
    mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x141, 0xf, 0xf, false));  // row_half_mirror
    mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x140, 0xf, 0xf, false));  // row_mirror
    const uint32_t m01 = max((uint32_t)__builtin_amdgcn_readlane((int)mb, 0), (uint32_t)__builtin_amdgcn_readlane((int)mb, 16));
    const uint32_t m23 = max((uint32_t)__builtin_amdgcn_readlane((int)mb, 32), (uint32_t)__builtin_amdgcn_readlane((int)mb, 48));
    int ex = (int)(max(m01, m23) >> 23);                  // biased exponent of the largest magnitude
    ex = ex < 1 ? 1 : ex;
    return vbits + 126 - ex;                              // max |val| * 2^sh < 2^vbits
  };
  auto slot_of = [&](int j) {
    const uint32_t u = (uint32_t)pi[j];
    // 12-bit index [u5..u0 v5..v0] -> [u1 u0 u5..u2 | v1 v0 v5..v2], then row stride 64 -> LDT
    const uint32_t x = DENSE ? u : ((u & 0xC3u) << 4) | ((u >> 2) & 0x3CFu);
    return u < 4096u ? x + ((x >> 6) << 2) : dummy;
  };
  auto add_pairs = [&](int sh) {
#pragma unroll
    for (int j = 0; j < NP; ++j)
      if (FULL || j < nact) atomicAdd(&itile[slot_of(j)], __float2int_rn(ldexpf(pv[j], sh)));
  };
  auto scatter = [&]() {
    if constexpr (COUNT) {
      static_assert(!COUNT || !STREAM, "the count pass needs the whole payload in registers");
      // every pair adds one to its coefficient's slot, reads the total back and is divided by it; the slots are
      // cleared again before the sums go in.  Sum of val/n over the n pairs of a slot = (sum of val) / n.
#pragma unroll
      for (int j = 0; j < NP; ++j)
        if (j < nact) atomicAdd(&itile[slot_of(j)], 1);
      wave_lds_sync();
#pragma unroll
      for (int j = 0; j < NP; ++j)
        if (j < nact) pv[j] = pv[j] / (float)itile[slot_of(j)];
      wave_lds_sync();
#pragma unroll
      for (int j = 0; j < NP; ++j)
        if (j < nact) itile[slot_of(j)] = 0;
      wave_lds_sync();
    }
    const int sh = shift_of(lane_max(0.f));
    add_pairs(sh);
    return sh;
  };

  int t = find_tensor_uniform(tv, chunk);
  int t_first = uniform_prefix(tv, t), t_next = uniform_prefix(tv, t + 1);
  TensorDev d = load_desc_uniform(tv, t);
  load_payload(d, chunk - t_first, 0);
  // The first payload is waited for here, outside the loop.  Inside, the wait before the scatter then only has the
  // back edge to serve, where the next chunk's payload loads have this chunk's stores and parameter loads behind
  // them: the compiler can let those stay in flight.  With the first payload still pending at the loop's entry it
  // had to wait for the count of the entry path, and thereby for the acknowledgement of every store of the
  // chunk before.
#pragma unroll
  for (int j = 0; j < NP; ++j) asm volatile("" : "+v"(pi[j]), "+v"(pv[j]));
  const int kap = kappa(c), col4 = 4 * chi(c);
  // tile offsets (floats) of the transposition of R: row parts for members w even / odd, column parts
  // for members w' even / odd (w' >= 2 adds 32 columns)
  const int row_up = 4 * g * D64_LDT, row_dn = 4 * (3 - g) * D64_LDT;
  const int wr_col_up = kap, wr_col_dn = 31 - kap;
  DEMO_PHASE_DECL

  for (; chunk < total; chunk += nwaves) {
    const int cc = chunk - t_first;
    const int k0 = cc / d.cchunks, k1 = cc - k0 * d.cchunks;
    const int64_t origin = (int64_t)k0 * 64 * d.cols + (int64_t)k1 * 64;   // uniform
    const uint32_t ucols = (uint32_t)d.cols;
    // parameters: lane (g, c) reads / writes rows rho(q, g), columns 4 chi(c) .. +3 (whole rows per instruction)
    const uint32_t vo_up = (uint32_t)g * ucols + (uint32_t)col4;           // elements
    const uint32_t vo_dn = (uint32_t)(3 - g) * ucols + (uint32_t)col4;
    const __amdgpu_buffer_rsrc_t xres = PBF16 ? make_rsrc(static_cast<const uint16_t*>(d.param) + origin)
                                              : make_rsrc(static_cast<const float*>(d.param) + origin);
    u32x2 Xh[16];   // bf16 parameters, raw: requested before the scatter, used after the products (the
                    // full-product instances have no registers for them until the products are done)
    auto fetch_x = [&]() __attribute__((always_inline)) {
#pragma unroll
      for (int q = 0; q < 16; ++q) Xh[q] = bload_u2(xres, ((q & 1) ? vo_dn : vo_up) * 2, (uint32_t)rho_base(q) * ucols * 2);
    };
    if (PBF16 && !DENSE_LATE_X) fetch_x();
    DEMO_PHASE(0);
    mask_payload(0);

    // ---- S = sum over workers ---------------------------------------------------------------------------
    int sh_chunk = 0;   // shift of this chunk's fixed point (undone when phi is the identity)
    if (args.stage == 1) {
      // time attribution (debug interface): the memory stream only -- the payload registers are merely kept alive
#pragma unroll
      for (int j = 0; j < NP; ++j) asm volatile("" ::"v"(pi[j]), "v"(pv[j]));
    } else {
#pragma unroll
    for (int i = 0; i < 17; ++i) *reinterpret_cast<float4*>(&tile[(i * 64 + lane) * 4]) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_sync();
    if constexpr (STREAM) {
      // one pass: the registers hold round 0; every round is added with the block exponent of the largest
      // magnitude seen so far, and when a round raises that exponent the sums in the tile are first shifted
      // down to the new scale (round to nearest, ties to even; every later shift at least halves the error of an earlier one,
      // so the shifts together cost at most one unit of the final scale per coefficient)
      sh_chunk = shift_of(lane_max(0.f));
      add_pairs(sh_chunk);
      for (int r = 1; r < nrounds; ++r) {
        load_payload(d, cc, r);
        mask_payload(r);
        const int sh_r = shift_of(lane_max(0.f));
        if (sh_r < sh_chunk) {   // uniform
          const int dsh = min(sh_chunk - sh_r, 31);
          const int half = (1 << (dsh - 1)) - 1;   // + the kept part's lowest bit: ties go to even (a bias would add up over the slots)
          wave_lds_sync();
#pragma unroll
          for (int i = 0; i < 17; ++i) {
            int4 v = *reinterpret_cast<int4*>(&itile[(i * 64 + lane) * 4]);
            v.x = (v.x + half + ((v.x >> dsh) & 1)) >> dsh;
            v.y = (v.y + half + ((v.y >> dsh) & 1)) >> dsh;
            v.z = (v.z + half + ((v.z >> dsh) & 1)) >> dsh;
            v.w = (v.w + half + ((v.w >> dsh) & 1)) >> dsh;
            *reinterpret_cast<int4*>(&itile[(i * 64 + lane) * 4]) = v;
          }
          wave_lds_sync();
          sh_chunk = sh_r;
        }
        add_pairs(sh_chunk);
      }
    } else {
      sh_chunk = scatter();   // the launch wrapper guarantees that one set of NP pairs per lane holds all W workers
    }
    }   // stage != 1
    DEMO_PHASE(1);
    // ---- payload of the next chunk, in flight during the products (after the last chunk the same
    //      chunk is requested again: an unconditional fetch keeps the old registers dead) -----------------
    if (chunk + nwaves < total) {
      while (chunk + nwaves >= t_next) {
        ++t;
        t_first = t_next;
        t_next = uniform_prefix(tv, t + 1);
        d = load_desc_uniform(tv, t);
      }
      load_payload(d, chunk + nwaves - t_first, 0);
    } else {
      load_payload(d, cc, 0);
    }
    wave_lds_sync();
    DEMO_PHASE(2);

    // ---- products ---------------------------------------------------------------------------------------
    auto comp = [](const float4& v, int r) { return r == 0 ? v.x : r == 1 ? v.y : r == 2 ? v.z : v.w; };
    if (args.stage != 0) {
      // time attribution: no products, the epilogue reads whatever the tile holds
      if constexpr (DENSE_LATE_X) {
        if (PBF16) fetch_x();
      }
    } else if constexpr (DENSE) {
      // product a per row tile ut: Y[u = 16 ut + 4g + r][j = 16 jt + c] = sum_v S[u][v] P[v][j], A = S from the tile
      // (row 16 ut + c; the eight v of a slot group are two 16-byte reads), B = fragments.  The accumulators of two
      // row tiles are, as they lie, the eight contraction slots of product b,
      // R[i = 16 it + 4g + r'][j] += sum_u P[u][i] Y[u][j], A = the same fragments.
      f32x4 R[4][4];   // [it][jt]
#pragma unroll
      for (int it = 0; it < 4; ++it)
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) R[it][jt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int hp = 0; hp < 2; ++hp) {
        f32x4 Y[2][4];   // [ut - 2 hp][jt]
#pragma unroll
        for (int uu = 0; uu < 2; ++uu)
#pragma unroll
          for (int jt = 0; jt < 4; ++jt) Y[uu][jt] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          SplitH8 A[2];   // [ut - 2 hp]: S as float32 below 2^8 (the tile holds fixed-point sums below 2^30), split
#pragma unroll
          for (int uu = 0; uu < 2; ++uu) {
            const float* arow = &tile[(16 * (2 * hp + uu) + c) * D64_LDT + 4 * g + 32 * h];
            const float4 a0 = *reinterpret_cast<const float4*>(arow);
            const float4 a1 = *reinterpret_cast<const float4*>(arow + 16);
            constexpr float sc = 0x1p-22f;
            A[uu] = split8h(m1h, (float)__float_as_int(a0.x) * sc, (float)__float_as_int(a0.y) * sc, (float)__float_as_int(a0.z) * sc,
                            (float)__float_as_int(a0.w) * sc, (float)__float_as_int(a1.x) * sc, (float)__float_as_int(a1.y) * sc,
                            (float)__float_as_int(a1.z) * sc, (float)__float_as_int(a1.w) * sc);
          }
#pragma unroll
          for (int jt = 0; jt < 4; ++jt) {
            const SplitH8 Bq = load_split8h(sG + (2 * jt + h) * kSplitHFragFloats, lane);
#pragma unroll
            for (int uu = 0; uu < 2; ++uu) Y[uu][jt] = mfma_f16(A[uu].lo, Bq.hi, Y[uu][jt]);
#pragma unroll
            for (int uu = 0; uu < 2; ++uu) Y[uu][jt] = mfma_f16(A[uu].hi, Bq.lo, Y[uu][jt]);
#pragma unroll
            for (int uu = 0; uu < 2; ++uu) Y[uu][jt] = mfma_f16(A[uu].hi, Bq.hi, Y[uu][jt]);
          }
          __builtin_amdgcn_sched_barrier(0);
        }
        SplitH8 Bt[4];
#pragma unroll
        for (int jt = 0; jt < 4; ++jt)
          Bt[jt] = split8h(m1h, Y[0][jt][0], Y[0][jt][1], Y[0][jt][2], Y[0][jt][3], Y[1][jt][0], Y[1][jt][1], Y[1][jt][2], Y[1][jt][3]);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const SplitH8 Ap = load_split8h(sG + (2 * it + hp) * kSplitHFragFloats, lane);
#pragma unroll
          for (int jt = 0; jt < 4; ++jt) R[it][jt] = mfma_f16(Ap.lo, Bt[jt].hi, R[it][jt]);
#pragma unroll
          for (int jt = 0; jt < 4; ++jt) R[it][jt] = mfma_f16(Ap.hi, Bt[jt].lo, R[it][jt]);
#pragma unroll
          for (int jt = 0; jt < 4; ++jt) R[it][jt] = mfma_f16(Ap.hi, Bt[jt].hi, R[it][jt]);
        }
      }
      DEMO_PHASE(3);
      // R through the tile (dead by now) in its natural order: a store instruction covers four rows 4 * 68 words
      // apart, i.e. 16 banks apart, and the sixteen columns fill the gaps
#pragma unroll
      for (int it = 0; it < 4; ++it)
#pragma unroll
        for (int jt = 0; jt < 4; ++jt)
#pragma unroll
          for (int r = 0; r < 4; ++r) tile[(16 * it + 4 * g + r) * D64_LDT + 16 * jt + c] = R[it][jt][r];
      if (PBF16 && DENSE_LATE_X) fetch_x();
    } else {
    float4 G[6];
#pragma unroll
    for (int i = 0; i < 6; ++i) G[i] = *reinterpret_cast<const float4*>(&sG[(i * 64 + lane) * 4]);
    f32x4 Cee[4], Ceo[4], Co0[4], Co1[4];   // [w'], component s: quadruple base i0 = 4s + g
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      Cee[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
      Ceo[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
      Co0[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
      Co1[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int rt = 0; rt < 4; ++rt) {
      // product a for rows u = 4 m + rt (physical rows 16 rt + m); column class of k-block kg is kg
      const float* arow = &tile[(16 * rt + c) * D64_LDT + 4 * g];
      float4 a[4];
#pragma unroll
      for (int kg = 0; kg < 4; ++kg) a[kg] = *reinterpret_cast<const float4*>(arow + 16 * kg);
      f32x4 ee = {0.f, 0.f, 0.f, 0.f}, eo = ee, o0 = ee, o1 = ee;
#pragma unroll
      for (int kr = 0; kr < 4; ++kr) {
        // the tile holds fixed-point sums
        const float a0 = (float)__float_as_int(comp(a[0], kr)), a1 = (float)__float_as_int(comp(a[1], kr));
        const float a2 = (float)__float_as_int(comp(a[2], kr)), a3 = (float)__float_as_int(comp(a[3], kr));
        ee = mfma4(a0, comp(G[0], kr), ee);
        o0 = mfma4(a1, comp(G[2], kr), o0);
        o1 = mfma4(a1, comp(G[4], kr), o1);
        eo = mfma4(a2, comp(G[1], kr), eo);
        o0 = mfma4(a3, comp(G[3], kr), o0);
        o1 = mfma4(a3, comp(G[5], kr), o1);
      }
      // columns member(w', kappa(c)) of Y, rows u = 4 (4g + r) + rt
      const f32x4 t1 = ee + eo, t2 = ee - eo;
      const f32x4 Y[4] = {t1 + o0, t2 + o1, t2 - o1, t1 - o0};
      // product b: this row tile feeds the accumulators of its class
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          if (rt == 0) Cee[e] = mfma4(comp(G[0], r), Y[e][r], Cee[e]);
          if (rt == 2) Ceo[e] = mfma4(comp(G[1], r), Y[e][r], Ceo[e]);
          if (rt == 1) {
            Co0[e] = mfma4(comp(G[2], r), Y[e][r], Co0[e]);
            Co1[e] = mfma4(comp(G[4], r), Y[e][r], Co1[e]);
          }
          if (rt == 3) {
            Co0[e] = mfma4(comp(G[3], r), Y[e][r], Co0[e]);
            Co1[e] = mfma4(comp(G[5], r), Y[e][r], Co1[e]);
          }
        }
    }
    DEMO_PHASE(3);

    // ---- R (quadruple identities) goes through the tile, which is dead by now, into the layout of the
    //      parameters.  Row i is kept at tile row rperm(i) = 16 (i / 16) + 4 (i % 4) + (i / 4) % 4: the four
    //      rows written by one instruction are then 16 banks apart and the sixteen columns fill the gaps.
    //      For i = member(w, 4s + g):  rperm = 16 w + 4 g + s (w even),  16 w + 4 (3 - g) + (3 - s) (w odd).
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float* wcol = tile + ((e & 1) ? wr_col_dn : wr_col_up) + (e >= 2 ? 32 : 0);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const float t1 = Cee[e][s] + Ceo[e][s], t2 = Cee[e][s] - Ceo[e][s];
        const float rr[4] = {t1 + Co0[e][s], t2 + Co1[e][s], t2 - Co1[e][s], t1 - Co0[e][s]};
#pragma unroll
        for (int w = 0; w < 4; ++w)
          wcol[((w & 1) ? row_dn : row_up) + (16 * w + ((w & 1) ? 3 - s : s)) * D64_LDT] = rr[w];
      }
    }
    }   // !DENSE
    wave_lds_sync();
    DEMO_PHASE(4);

    // ---- x <- x - lr*(phi(R) + wd*x): phi = sgn (the scale of the fixed point does not matter), or the identity
    //      on the aggregate itself (the sum of the tile is R * 2^sh; `scale` is 1 or 1/W) ------------------------------
    // (full-product instances: the sums went in as 2^-22 of their integers and both products carry 2^kSplitHBasisLog2)
    const float factor = IDENT ? ldexpf(args.scale, (DENSE ? 22 - 2 * kSplitHBasisLog2 : 0) - sh_chunk) : 0.f;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      f32x4 xin[4];   // fp32 parameters of the four rows of this quadruple
      if (!PBF16) {
#pragma unroll
        for (int w = 0; w < 4; ++w)
          xin[w] = bload_f4(xres, ((w & 1) ? vo_dn : vo_up) * 4, (uint32_t)rho_base(4 * s + w) * ucols * 4);
      }
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int q = 4 * s + w;
        const float4 rv = *reinterpret_cast<const float4*>(
            DENSE ? &tile[(rho_base(q) + ((q & 1) ? 3 - g : g)) * D64_LDT + col4]
                  : &tile[((w & 1) ? row_dn : row_up) + (16 * w + ((w & 1) ? 3 - s : s)) * D64_LDT + col4]);
        const float rr[4] = {rv.x, rv.y, rv.z, rv.w};
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float x;
          if (PBF16) {
            const uint32_t raw = Xh[q][e >> 1];
            x = __uint_as_float((e & 1) ? (raw & 0xffff0000u) : (raw << 16));
          } else {
            x = xin[w][e];
          }
          o[e] = sign_update(x, IDENT ? rr[e] * factor : sgnf(rr[e]), args.lr, args.weight_decay);
        }
        const uint32_t vo = (q & 1) ? vo_dn : vo_up, so = (uint32_t)rho_base(q) * ucols;
        if (PBF16) {
          const u32x2 pk = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
          bstore_u2(xres, vo * 2, so * 2, pk);
        } else {
          const f32x4 ov = {o[0], o[1], o[2], o[3]};
          bstore_f4(xres, vo * 4, so * 4, ov);
        }
      }
    }
    wave_lds_sync();
    DEMO_PHASE(5);
  }
  DEMO_PHASE_FLUSH(8);
}

// ---------------------------------------------------------------------------
// Few pairs per chunk (W * k <= 64, e.g. a worker decoding its own payload): no coefficient tile.
// R = sum_p val_p P[u_p]^T P[v_p] is accumulated by MFMA chains whose operands are gathered rows of P, as in the
// reconstruction of the encode kernel: the pairs are filed by the class of u (0 mod 4, 2 mod 4, odd), each class
// accumulates one 16-row tile per column tile on the quadruple bases (two for odd u), and the four members of a
// quadruple follow from in-lane adds.  Pairs of different workers that hit the same coefficient simply add up.
// ---------------------------------------------------------------------------
namespace {
constexpr int D64S_WAVES = 4;                     // three workgroups per CU (3 wavefronts per SIMD)
constexpr int D64S_THREADS = D64S_WAVES * 64;
constexpr int D64S_TABLE_FLOATS = 4096 + 2048;    // pcol, pk, pk2
constexpr int D64S_LDS_BYTES = 4 * (D64S_TABLE_FLOATS + D64S_WAVES * 3 * 2 * 64);   // + three class lists per wavefront
}  // namespace

template <bool PBF16>
__global__ __launch_bounds__(D64S_THREADS, 3) void decode2d_sparse64(TableView tv, const float* __restrict__ tables,
                                                                     DecodeArgs args) {
  extern __shared__ float lds[];
  const float* sPcol = lds;
  const float* sPk = lds + 4096;
  const float* sPk2 = lds + 4096 + 1024;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, c = lane & 15;
  uint2* sel = reinterpret_cast<uint2*>(lds + D64S_TABLE_FLOATS) + wave * 3 * 64;   // [3][64] {flat index, value bits}
  const int k = args.k, W = args.W;
  const int npairs = W * k;

  for (int e = tid; e < 4096 / 4; e += D64S_THREADS)
    reinterpret_cast<float4*>(lds)[e] = reinterpret_cast<const float4*>(tables + D64_PCOL)[e];
  for (int e = tid; e < 2048 / 4; e += D64S_THREADS)
    reinterpret_cast<float4*>(lds + 4096)[e] = reinterpret_cast<const float4*>(tables + D64_PK)[e];
  __syncthreads();

  const int nwaves = gridDim.x * D64S_WAVES;
  const int wid = blockIdx.x * D64S_WAVES + wave;
  const int total = tv.total_chunks;
  int chunk = wid;   // wavefront w takes chunks w, w + nwaves, ... (see the encode kernel)
  if (chunk >= total) return;

  // pair `lane` of a chunk: worker lane / k, position lane % k
  const int pw = lane / k, pt = lane - pw * k;
  int32_t pi = -1;
  float pv = 0.f;
  auto load_pair = [&](const TensorDev& dd, int ccc) {
    const int64_t off = ((int64_t)pw * dd.nchunks + ccc) * k + pt;
    pi = lane < npairs ? as_global(dd.idx)[off] : -1;
    pv = lane < npairs ? as_global(dd.val)[off] : 0.f;
  };

  int t = find_tensor_uniform(tv, chunk);
  int t_first = uniform_prefix(tv, t), t_next = uniform_prefix(tv, t + 1);
  TensorDev d = load_desc_uniform(tv, t);
  load_pair(d, chunk - t_first);
  const int col4 = 4 * chi(c);

  for (; chunk < total; chunk += nwaves) {
    const int cc = chunk - t_first;
    const int k0 = cc / d.cchunks, k1 = cc - k0 * d.cchunks;
    const int64_t origin = (int64_t)k0 * 64 * d.cols + (int64_t)k1 * 64;   // uniform
    const uint32_t ucols = (uint32_t)d.cols;
    const uint32_t vo_up = (uint32_t)g * ucols + (uint32_t)col4;           // elements
    const uint32_t vo_dn = (uint32_t)(3 - g) * ucols + (uint32_t)col4;
    const __amdgpu_buffer_rsrc_t xres = PBF16 ? make_rsrc(static_cast<const uint16_t*>(d.param) + origin)
                                              : make_rsrc(static_cast<const float*>(d.param) + origin);
    // parameters of this chunk
    u32x2 Xh[16];
    f32x4 Xf[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      if (PBF16) Xh[q] = bload_u2(xres, ((q & 1) ? vo_dn : vo_up) * 2, (uint32_t)rho_base(q) * ucols * 2);
      else Xf[q] = bload_f4(xres, ((q & 1) ? vo_dn : vo_up) * 4, (uint32_t)rho_base(q) * ucols * 4);
    }
    // pairs of this chunk -> class lists in LDS (out-of-range indices contribute nothing), padded with zero-valued
    // entries to a multiple of four
    int ncls[3];
    {
      const bool ok = (uint32_t)pi < 4096u;
      const uint32_t u = ((uint32_t)pi >> 6) & 63u;
      const int cls = (u & 1u) ? 2 : (int)((u >> 1) & 1u);
#pragma unroll
      for (int q = 0; q < 3; ++q) {
        const uint64_t m = __ballot(ok && cls == q);
        ncls[q] = __popcll(m);
        if (ok && cls == q) sel[q * 64 + lanes_below(m)] = make_uint2((uint32_t)pi, __float_as_uint(pv));
        if (lane < ((4 - (ncls[q] & 3)) & 3)) sel[q * 64 + ncls[q] + lane] = make_uint2(0u, 0u);
      }
    }
    wave_lds_sync();
    // pair of the next chunk (after the last chunk the same one again: keeps the old registers dead)
    if (chunk + nwaves < total) {
      while (chunk + nwaves >= t_next) {
        ++t;
        t_first = t_next;
        t_next = uniform_prefix(tv, t + 1);
        d = load_desc_uniform(tv, t);
      }
      load_pair(d, chunk + nwaves - t_first);
    } else {
      load_pair(d, cc);
    }

    // compact accumulators: component s of tile e is the quadruple base i0 = 4s + g, column 4 chi(c) + e
    f32x4 Ree[4], Reo[4], Ro0[4], Ro1[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      Ree[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
      Reo[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
      Ro0[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
      Ro1[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
    for (int ks = 0; ks < (ncls[0] + 3) / 4; ++ks) {
      const uint2 sv = sel[0 * 64 + 4 * ks + g];
      const float a = __uint_as_float(sv.y) * sPk[((sv.x >> 6) & 63u) * 16 + c];
      const float4 pb = *reinterpret_cast<const float4*>(&sPcol[(sv.x & 63u) * 64 + 4 * c]);
      const float bf[4] = {pb.x, pb.y, pb.z, pb.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) Ree[e] = mfma4(a, bf[e], Ree[e]);
    }
    for (int ks = 0; ks < (ncls[1] + 3) / 4; ++ks) {
      const uint2 sv = sel[1 * 64 + 4 * ks + g];
      const float a = __uint_as_float(sv.y) * sPk[((sv.x >> 6) & 63u) * 16 + c];
      const float4 pb = *reinterpret_cast<const float4*>(&sPcol[(sv.x & 63u) * 64 + 4 * c]);
      const float bf[4] = {pb.x, pb.y, pb.z, pb.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) Reo[e] = mfma4(a, bf[e], Reo[e]);
    }
    for (int ks = 0; ks < (ncls[2] + 3) / 4; ++ks) {
      const uint2 sv = sel[2 * 64 + 4 * ks + g];
      const uint32_t ur = ((sv.x >> 6) & 63u) * 16 + c;
      const float a0 = __uint_as_float(sv.y) * sPk[ur], a1 = __uint_as_float(sv.y) * sPk2[ur];
      const float4 pb = *reinterpret_cast<const float4*>(&sPcol[(sv.x & 63u) * 64 + 4 * c]);
      const float bf[4] = {pb.x, pb.y, pb.z, pb.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        Ro0[e] = mfma4(a0, bf[e], Ro0[e]);
        Ro1[e] = mfma4(a1, bf[e], Ro1[e]);
      }
    }

    // x <- x - lr*(phi(R) + wd*x); members of the quadruple with base 4s + g: rows rho(4s + w, g).  phi = sgn, or the
    // identity on the aggregate (times `scale`: 1 or 1/W), chosen per element: this kernel has registers for one copy
    // of the loop only
    const bool ident = args.phi != 0;
#pragma unroll
    for (int sq = 0; sq < 4; ++sq) {
      float o[4][4];   // [w][e]
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float t1 = Ree[e][sq] + Reo[e][sq], t2 = Ree[e][sq] - Reo[e][sq];
        const float rr[4] = {t1 + Ro0[e][sq], t2 + Ro1[e][sq], t2 - Ro1[e][sq], t1 - Ro0[e][sq]};
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const int q = 4 * sq + w;
          float x;
          if (PBF16) {
            const uint32_t raw = Xh[q][e >> 1];
            x = __uint_as_float((e & 1) ? (raw & 0xffff0000u) : (raw << 16));
          } else {
            x = Xf[q][e];
          }
          o[w][e] = sign_update(x, ident ? rr[w] * args.scale : sgnf(rr[w]), args.lr, args.weight_decay);
        }
      }
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int q = 4 * sq + w;
        const uint32_t vo = (q & 1) ? vo_dn : vo_up, so = (uint32_t)rho_base(q) * ucols;
        if (PBF16) {
          const u32x2 pk = {pack_bf16x2(o[w][0], o[w][1]), pack_bf16x2(o[w][2], o[w][3])};
          bstore_u2(xres, vo * 2, so * 2, pk);
        } else {
          const f32x4 ov = {o[w][0], o[w][1], o[w][2], o[w][3]};
          bstore_f4(xres, vo * 4, so * 4, ov);
        }
      }
    }
    wave_lds_sync();
  }
}

template <bool PBF16>
static hipError_t launch_dec_sparse64(const TableView& tv, const float* tables, const DecodeArgs& a, int num_cus,
                                      hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode2d_sparse64<PBF16>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, D64S_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  int64_t grid = (int64_t)num_cus * (PBF16 ? 4 : 3);   // workgroups per CU the registers allow
  const int64_t max_grid = ((int64_t)tv.total_chunks + D64S_WAVES - 1) / D64S_WAVES;
  if (grid > max_grid) grid = max_grid;
  hipLaunchKernelGGL(decode2d_sparse64<PBF16>, dim3((unsigned)grid), dim3(D64S_THREADS), D64S_LDS_BYTES, stream, tv,
                     tables, a);
  return hipGetLastError();
}

template <bool PBF16, int MODE, bool IDENT, bool COUNT = false, bool NT = true, bool DENSE = false>
static hipError_t launch_dec_wave64_phi(const TableView& tv, const float* tables, const DecodeArgs& a, int64_t grid,
                                        hipStream_t stream) {
  static bool attr_set = false;
  constexpr int lds_bytes = d64_lds_bytes<DENSE>();
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode2d_wave64<PBF16, MODE, IDENT, COUNT, NT, DENSE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((decode2d_wave64<PBF16, MODE, IDENT, COUNT, NT, DENSE>), dim3((unsigned)grid), dim3(D64_THREADS),
                     lds_bytes, stream, tv, tables, a);
  return hipGetLastError();
}
template <bool PBF16, int MODE, bool NT>
static hipError_t launch_dec_wave64_nt(const TableView& tv, const float* tables, const DecodeArgs& a, int64_t grid,
                                       hipStream_t stream) {
  if constexpr (MODE == 0 || MODE == 3 || MODE == 4) {
    if (a.agg == 2)
      return a.phi != 0 ? launch_dec_wave64_phi<PBF16, MODE, true, true, NT>(tv, tables, a, grid, stream)
                        : launch_dec_wave64_phi<PBF16, MODE, false, true, NT>(tv, tables, a, grid, stream);
  }
  return a.phi != 0 ? launch_dec_wave64_phi<PBF16, MODE, true, false, NT>(tv, tables, a, grid, stream)
                    : launch_dec_wave64_phi<PBF16, MODE, false, false, NT>(tv, tables, a, grid, stream);
}
template <bool PBF16, int MODE>
static hipError_t launch_dec_wave64(const TableView& tv, const float* tables, const DecodeArgs& a, int64_t grid,
                                    hipStream_t stream) {
  // rows of k pairs shorter than a 128-byte line: plain loads (mode 4 has such rows but for k = 34 ... 62)
  if constexpr (MODE == 3 || MODE == 5) {
    if (a.k < 32) return launch_dec_wave64_nt<PBF16, MODE, false>(tv, tables, a, grid, stream);
  }
  if constexpr (MODE == 4) return launch_dec_wave64_nt<PBF16, MODE, false>(tv, tables, a, grid, stream);
  return launch_dec_wave64_nt<PBF16, MODE, true>(tv, tables, a, grid, stream);
}

// Full-product instances (any orthonormal matrix; `tables` of build_dec64_dense_tables): the whole payload of a chunk in
// registers (W * k <= 2048), plain sum or mean, four pairs per load when k is a multiple of 4 and the arrays are
// 16-byte aligned, else one.
bool dense64_decode_supports(const DecodeArgs& a) { return a.k <= kFast64MaxK && (int64_t)a.W * a.k <= 2048 && a.agg != 2; }
hipError_t launch_decode2d_dense64(const TableView& tv, const float* tables, const DecodeArgs& a, bool param_bf16,
                                   bool payload_aligned16, int num_cus, hipStream_t stream) {
  if (!dense64_decode_supports(a)) return hipErrorInvalidValue;
  int64_t grid = num_cus;
  const int64_t max_grid = ((int64_t)tv.total_chunks + DEMO_RUN - 1) / DEMO_RUN;
  if (grid > max_grid) grid = max_grid;
  const bool vec = payload_aligned16 && a.k % 4 == 0, ident = a.phi != 0;
  const bool nt = a.k >= 32;   // rows of k pairs shorter than a 128-byte line: plain loads (as in launch_dec_wave64)
  if (param_bf16) {
    if (vec && nt) return ident ? launch_dec_wave64_phi<true, 3, true, false, true, true>(tv, tables, a, grid, stream)
                                : launch_dec_wave64_phi<true, 3, false, false, true, true>(tv, tables, a, grid, stream);
    if (vec) return ident ? launch_dec_wave64_phi<true, 3, true, false, false, true>(tv, tables, a, grid, stream)
                          : launch_dec_wave64_phi<true, 3, false, false, false, true>(tv, tables, a, grid, stream);
    return ident ? launch_dec_wave64_phi<true, 0, true, false, true, true>(tv, tables, a, grid, stream)
                 : launch_dec_wave64_phi<true, 0, false, false, true, true>(tv, tables, a, grid, stream);
  }
  if (vec && nt) return ident ? launch_dec_wave64_phi<false, 3, true, false, true, true>(tv, tables, a, grid, stream)
                              : launch_dec_wave64_phi<false, 3, false, false, true, true>(tv, tables, a, grid, stream);
  if (vec) return ident ? launch_dec_wave64_phi<false, 3, true, false, false, true>(tv, tables, a, grid, stream)
                        : launch_dec_wave64_phi<false, 3, false, false, false, true>(tv, tables, a, grid, stream);
  return ident ? launch_dec_wave64_phi<false, 0, true, false, true, true>(tv, tables, a, grid, stream)
               : launch_dec_wave64_phi<false, 0, false, false, true, true>(tv, tables, a, grid, stream);
}

hipError_t launch_decode2d_wave64(const TableView& tv, const float* tables, const DecodeArgs& a, bool param_bf16,
                                  bool payload_aligned16, int num_cus, hipStream_t stream) {
  if (!fast64_decode_supports(a.W, a.k, payload_aligned16)) return hipErrorInvalidValue;
  const bool by_count = a.agg == 2;   // needs the coefficient tile and the whole payload in registers
  if (by_count && a.W * a.k > 2048) return hipErrorInvalidValue;
  if (a.W * a.k <= 64 && !by_count)
    return param_bf16 ? launch_dec_sparse64<true>(tv, tables, a, num_cus, stream)
                      : launch_dec_sparse64<false>(tv, tables, a, num_cus, stream);
  int64_t grid = num_cus;
  const int64_t max_grid = ((int64_t)tv.total_chunks + DEMO_RUN - 1) / DEMO_RUN;   // few items: one run per workgroup, spread over the CUs
  if (grid > max_grid) grid = max_grid;
  const int mode = !payload_aligned16 ? 0
                   : a.W * a.k > 2048 ? 5
                   : (a.k == 32 && a.W % 8 == 0 && a.W <= 64 && !by_count) ? (a.W == 64 ? 1 : 2)
                   : a.k % 4 == 0 ? 3 : a.k % 2 == 0 ? 4 : 0;
  if (param_bf16) {
    switch (mode) {
      case 1: return launch_dec_wave64<true, 1>(tv, tables, a, grid, stream);
      case 2: return launch_dec_wave64<true, 2>(tv, tables, a, grid, stream);
      case 3: return launch_dec_wave64<true, 3>(tv, tables, a, grid, stream);
      case 4: return launch_dec_wave64<true, 4>(tv, tables, a, grid, stream);
      case 5: return launch_dec_wave64<true, 5>(tv, tables, a, grid, stream);
      default: return launch_dec_wave64<true, 0>(tv, tables, a, grid, stream);
    }
  }
  switch (mode) {
    case 1: return launch_dec_wave64<false, 1>(tv, tables, a, grid, stream);
    case 2: return launch_dec_wave64<false, 2>(tv, tables, a, grid, stream);
    case 3: return launch_dec_wave64<false, 3>(tv, tables, a, grid, stream);
    case 4: return launch_dec_wave64<false, 4>(tv, tables, a, grid, stream);
    case 5: return launch_dec_wave64<false, 5>(tv, tables, a, grid, stream);
    default: return launch_dec_wave64<false, 0>(tv, tables, a, grid, stream);
  }
}

}  // namespace demo

DEMO_PHASE_GETTER(demo_debug_phase_clocks_dec)
