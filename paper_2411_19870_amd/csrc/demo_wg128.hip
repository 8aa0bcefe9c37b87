// s = 128 kernels: one 512-thread workgroup (8 wavefronts) per 128 x 128 chunk, one workgroup per CU.
//
// A chunk is too large for one wavefront's registers.  Row u of the 128-point orthonormal DCT-II is even (u even)
// or odd (u odd) under i -> 127-i, so the coefficients of parities (u % 2, v % 2) are four independent 64 x 64
// two-sided transforms of the chunk folded along both mirrors (encode), or give the chunk's update by sums and
// differences of four such transforms (decode): a quarter of the multiplications of the full products.  Each
// quadrant is computed in registers by two wavefronts, on the float16 matrix pipe with float32 operands split into
// two parts (demo_device.h); LDS holds the four quadrant tiles, the pre-split basis fragments and, for the encode,
// the float32 basis rows its reconstruction gathers (class-major: row u at position pos3(u)).
#include <type_traits>

#include "demo_device.h"

namespace demo {

namespace {
constexpr int W128_LDP = 68;                           // row stride of the class-major float32 basis tile P[u][i], i < 64
constexpr int W128_P_FLOATS = 128 * W128_LDP;
constexpr int W128_CAP = 512;                          // candidate list of the top-k
constexpr int W128_SEL = 68;                           // entries per class list of selected coefficients (k <= 64, padded)

// Workgroup barrier that orders LDS accesses only: global loads and stores stay in flight across it.
__device__ __forceinline__ void wg_lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// class-major position of frequency u: u = 0 mod 4 first, then u = 2 mod 4, then odd u
__device__ __forceinline__ int pos3(uint32_t u) { return (int)((u & 1u) ? 64u + (u >> 1) : ((u & 2u) << 4) + (u >> 2)); }

}  // namespace

// ---------------------------------------------------------------------------
// encode:  m <- beta m + g ;  Q = P B P^T ;  k largest |Q| ;  m <- m - alpha P^T Q^ P      (Algorithm 1, worker side)
// ---------------------------------------------------------------------------
// With A[u'][i] = P[2u'][i], O[u'][i] = P[2u'+1][i] (i < 64; row u of the DCT is even or odd under i -> 127 - i) the
// coefficients of parities (a, b) = (u % 2, v % 2) are one 64 x 64 two-sided product each,
//   Q[2u'+a][2v'+b] = (M_a B_ab M_b^T)[u'][v'],   M_0 = A, M_1 = O,
//   B_ab[i][j] = D[i][j] + (-1)^b D[i][127-j] + (-1)^a D[127-i][j] + (-1)^(a+b) D[127-i][127-j]      (i, j < 64),
// a quarter of the multiplications of the full products.  Thread t owns, for p < 2, position (i, j0..j0+3) =
// ((t + 512 p) / 16, 4 ((t + 512 p) % 16)) of the quadrants, i.e. the four row segments (i, j0..), (i, 124 - j0..),
// (127 - i, j0..), (127 - i, 124 - j0..) of the chunk: it loads them, forms D = beta m + g and the four folded values,
// keeps D for the final m <- D - alpha R, and unfolds the reconstruction from the same four quadrant values.
// The products run on the float16 matrix pipe, operands split into two parts (demo_device.h): the folded tile is
// scaled by a power of two taken from the chunk's largest |D| to below 2^8, the basis fragments by 2^4, so that the
// first product stays below 2^15; two wavefronts per quadrant, each with half of the columns, and the accumulators of
// the first product are, as they lie, operands of the second (as in the decode kernel below).  The coefficients are
// ranked at that scale and unscaled (exactly) where they leave for the payload and the reconstruction.
// Top-k: bound of the k-th magnitude from 128 group maxima (groups of 4 lanes), candidate list, ranks by slices of
// the list; reconstruction: class lists in rank order, float32 MFMA gathers on the class-major basis tile.  A chunk
// whose candidate list overflows (many equal magnitudes at the threshold) is left untouched and queued for the exact
// generic kernel that runs next.
namespace {
constexpr int E128_WAVES = 8;
constexpr int E128_THREADS = 64 * E128_WAVES;
constexpr int E128_LDT = 68;                                    // quadrant row stride (floats)
constexpr int E128_TILE_FLOATS = 64 * E128_LDT;
constexpr int E128_TILES_FLOATS = 4 * E128_TILE_FLOATS;
constexpr int E128_FRAGS = 8 * kSplitHFragFloats;               // fragment table of one 64 x 64 matrix
constexpr int E128_TABLE_FLOATS = 2 * E128_FRAGS;               // A^T, then O^T
constexpr int E128_LDS_BYTES = 4 * (E128_TABLE_FLOATS + W128_P_FLOATS + E128_TILES_FLOATS + 128 + 16 + 16 + W128_CAP) +
                               8 * (W128_CAP + 2 + 4 * W128_SEL);
static_assert(E128_TABLE_FLOATS == kEnc128TableFloats, "table size");
static_assert(E128_LDS_BYTES <= 160 * 1024, "LDS budget");
static_assert(W128_CAP == E128_THREADS, "one candidate per thread in the selection step");
}  // namespace

// Host: pre-split float16 fragment tables of A^T and O^T (scaled by 2^kSplitHBasisLog2) from the 128 x 128 DCT matrix
// P: per matrix M block 2 t + h, slot j of contraction group g holds M[16 t + c][16 (2 h + j / 4) + 4 g + j % 4]
// (first product: B operand, contracts j, output columns v' = 16 t + c; second: A operand, contracts i, output rows
// u' = 16 t + c).
void build_enc128_tables(const double* P, float* out) {
  for (int m = 0; m < 2; ++m)
    for (int t = 0; t < 4; ++t)
      for (int h = 0; h < 2; ++h)
        for (int lane = 0; lane < 64; ++lane) {
          float v[8];
          for (int j = 0; j < 8; ++j) {
            const int kk = 16 * (2 * h + (j >> 2)) + 4 * (lane >> 4) + (j & 3);
            v[j] = (float)__builtin_ldexp(P[(2 * (16 * t + (lane & 15)) + m) * 128 + kk], kSplitHBasisLog2);
          }
          host_store_split8h(out + m * E128_FRAGS + (2 * t + h) * kSplitHFragFloats, lane, v);
        }
}

template <bool GBF16>
__global__ __launch_bounds__(E128_THREADS) void encode2d_quad128(TableView tv, const float* __restrict__ basis,
                                                                  const float* __restrict__ tables, EncodeArgs args,
                                                                  Worklist wl) {
  extern __shared__ float lds[];
  const float* sT = lds;
  float* sP = lds + E128_TABLE_FLOATS;
  float* tiles = sP + W128_P_FLOATS;
  uint32_t* gmax = reinterpret_cast<uint32_t*>(tiles + E128_TILES_FLOATS);   // [128] maxima of groups of 4 lanes
  int* ctl = reinterpret_cast<int*>(gmax + 128);                      // [0] candidate cursor, [1] threshold, [2] all-zero flag, [4..7] class counts
  uint32_t* wmax = reinterpret_cast<uint32_t*>(ctl + 16);             // [8] per-wavefront largest |D|
  uint32_t* rk = wmax + 16;                                           // [CAP] rank | class rank << 16 of a candidate
  uint2* cand = reinterpret_cast<uint2*>(rk + W128_CAP);              // [CAP + 2] {coefficient bits (scaled), flat index}
  uint2* sel = cand + W128_CAP + 2;                                   // [4][SEL]  {basis row offsets, coefficient bits}
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int k = args.k;
  const int total = tv.total_chunks;
  int chunk = blockIdx.x;
  if (chunk >= total) return;

  const float m1h = opaque_minus_one();
  for (int e = tid; e < E128_TABLE_FLOATS / 4; e += E128_THREADS)
    reinterpret_cast<f32x4*>(lds)[e] = gload_f4(tables + 4 * e);
  for (int e = tid; e < 128 * 16; e += E128_THREADS) {
    const int u = e >> 4, c4 = (e & 15) * 4;
    *reinterpret_cast<f32x4*>(&sP[pos3((uint32_t)u) * W128_LDP + c4]) = gload_f4(basis + u * 128 + c4);
  }

  using GT = typename std::conditional<GBF16, u32x2, f32x4>::type;
  f32x4 mv[2][4];
  GT gv[2][4];
  __amdgpu_buffer_rsrc_t mres_in, gres_in;
  uint32_t ucols_in = 0;
  auto set_source = [&](const TensorDev& dd, int cc) {
    const int k0 = cc / dd.cchunks, k1 = cc - k0 * dd.cchunks;
    const int64_t origin = (int64_t)k0 * 128 * dd.cols + (int64_t)k1 * 128;
    ucols_in = (uint32_t)dd.cols;
    mres_in = make_rsrc(dd.mom + origin);
    gres_in = GBF16 ? make_rsrc(static_cast<const uint16_t*>(dd.grad) + origin)
                    : make_rsrc(static_cast<const float*>(dd.grad) + origin);
  };
  // element offset of segment sg of position block p in a chunk whose rows are `uc` elements apart
  auto seg_offset = [](uint32_t t, int p, int sg, uint32_t uc) {
    const uint32_t pb = t + E128_THREADS * p, ir = pb >> 4, j0 = (pb & 15u) * 4u;
    return ((sg & 2) ? 127u - ir : ir) * uc + ((sg & 1) ? 124u - j0 : j0);
  };
  // quarter q < 4 of the rows: position block q / 2, segments 2 (q % 2) and 2 (q % 2) + 1
  auto issue_rows_part = [&](uint32_t t, int q) __attribute__((always_inline)) {
#pragma unroll
    for (int sg = 2 * (q & 1); sg < 2 * (q & 1) + 2; ++sg) {
      const uint32_t eo = seg_offset(t, q >> 1, sg, ucols_in);
      mv[q >> 1][sg] = bload_f4(mres_in, eo * 4, 0u);
      if constexpr (GBF16) gv[q >> 1][sg] = bload_u2(gres_in, eo * 2, 0u);
      else gv[q >> 1][sg] = bload_f4(gres_in, eo * 4, 0u);
    }
  };
  auto issue_rows = [&](uint32_t t) {
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_rows_part(t, q);
  };

  int t = find_tensor_uniform(tv, chunk);
  int t_first = uniform_prefix(tv, t), t_next = uniform_prefix(tv, t + 1);
  TensorDev d = load_desc_uniform(tv, t);
  set_source(d, chunk - t_first);
  issue_rows((uint32_t)tid);
  // the first chunk's rows are waited for here, outside the loop: with loads pending at the loop's entry and the
  // momentum stores pending on its back edge, the loop's first wait would be for everything outstanding
#pragma unroll
  for (int p = 0; p < 2; ++p)
#pragma unroll
    for (int sg = 0; sg < 4; ++sg) asm volatile("" : "+v"(mv[p][sg]), "+v"(gv[p][sg]));

  // products: quadrant of this wavefront, its half of the columns, the two fragment tables
  const int quad = wave >> 1, jh = wave & 1;
  const float* tq = tiles + quad * E128_TILE_FLOATS;
  const float* TB = sT + (quad & 1) * E128_FRAGS;              // first product: M_b^T, the column parity
  const float* TA = sT + (quad >> 1) * E128_FRAGS;             // second product: M_a, the row parity

  DEMO_PHASE_DECL
  for (;;) {
    int tidv = tid;
    asm volatile("" : "+v"(tidv));   // addresses below are recomputed per chunk rather than kept (and spilled) across it
    const int lanev = tidv & 63;
    const uint32_t zero = (uint32_t)(tidv >> 31);                            // 0, formed per chunk like the addresses
    if (tidv < 4 * W128_SEL) sel[tidv] = make_uint2(zero, zero);             // zero-valued padding of the class lists
    cand[tidv] = make_uint2(zero, ~zero);                                     // entries that precede nothing
    if (tidv < 2) cand[W128_CAP + tidv] = make_uint2(zero, ~zero);
    rk[tidv] = zero;
    if (tidv < 8) ctl[tidv] = (int)zero;
    // where this chunk's results go
    const int cc = chunk - t_first;
    const uint32_t ucols = (uint32_t)d.cols;
    float* const mom_out = d.mom + ((int64_t)(cc / d.cchunks) * 128 * d.cols + (int64_t)(cc % d.cchunks) * 128);
    DEMO_GLOBAL int32_t* const out_idx = as_global(d.idx) + (int64_t)cc * k;
    DEMO_GLOBAL float* const out_val = as_global(d.val) + (int64_t)cc * k;

    // ---- D = beta m + g from the rows in the registers, and its largest magnitude -------------------------------
    f32x4 D[2][4];
    float mx = 0.f;
#pragma unroll
    for (int p = 0; p < 2; ++p)
#pragma unroll
      for (int sg = 0; sg < 4; ++sg) {
        f32x4 gf;
        if constexpr (GBF16) {
          gf = (f32x4){bf16_to_f32(gv[p][sg][0] & 0xffffu), bf16_to_f32(gv[p][sg][0] >> 16),
                       bf16_to_f32(gv[p][sg][1] & 0xffffu), bf16_to_f32(gv[p][sg][1] >> 16)};
        } else {
          gf = gv[p][sg];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          D[p][sg][e] = __fmaf_rn(args.beta, mv[p][sg][e], args.grad_scale * gf[e]);
          mx = fmaxf(mx, fabsf(D[p][sg][e]));
        }
      }
    {
      uint32_t mb = __float_as_uint(mx);
      mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
      mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
      mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x141, 0xf, 0xf, false));  // row_half_mirror
      mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x140, 0xf, 0xf, false));  // row_mirror
      const uint32_t m01 = max((uint32_t)__builtin_amdgcn_readlane((int)mb, 0), (uint32_t)__builtin_amdgcn_readlane((int)mb, 16));
      const uint32_t m23 = max((uint32_t)__builtin_amdgcn_readlane((int)mb, 32), (uint32_t)__builtin_amdgcn_readlane((int)mb, 48));
      if (lane == 0) wmax[wave] = max(m01, m23);
    }
    const int nxt = chunk + (int)gridDim.x;
    const bool has_next = nxt < total;
    wg_lds_barrier();
    // ---- scale 2^sexp: |D| < 2^(e+1), so the folded values stay below 2^(e+3) and 2^(5-e) brings them below 2^8 ------
    int sexp;
    {
      uint32_t mall = wmax[lanev & 7];
      mall = max(mall, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mall, 0xB1, 0xf, 0xf, false));
      mall = max(mall, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mall, 0x4E, 0xf, 0xf, false));
      mall = max(mall, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mall, 0x141, 0xf, 0xf, false));
      const int ex = (int)((uint32_t)__builtin_amdgcn_readfirstlane((int)mall) >> 23);   // biased exponent of the largest |D|
      int se = 259 - ex;                                       // biased exponent of 2^(5 - (ex - 127))
      se = se < 1 ? 1 : se > 254 ? 254 : se;                   // (chunks below 2^-121 keep fewer bits)
      sexp = se - 127;
    }
    const float scale = __uint_as_float((uint32_t)(sexp + 127) << 23);
    // ---- folded and scaled values into the quadrant tiles -----------------------------------------------------------
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const uint32_t pb = (uint32_t)tidv + E128_THREADS * p, ir = pb >> 4, j0 = (pb & 15u) * 4u;
      f32x4 b00, b01, b10, b11;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float d0 = D[p][0][e], d1 = D[p][1][3 - e], d2 = D[p][2][e], d3 = D[p][3][3 - e];
        const float s0 = d0 + d1, t0 = d0 - d1, s1 = d2 + d3, t1 = d2 - d3;
        b00[e] = (s0 + s1) * scale;
        b01[e] = (t0 + t1) * scale;
        b10[e] = (s0 - s1) * scale;
        b11[e] = (t0 - t1) * scale;
      }
      float* wq = tiles + ir * E128_LDT + j0;
      *reinterpret_cast<f32x4*>(wq) = b00;
      *reinterpret_cast<f32x4*>(wq + E128_TILE_FLOATS) = b01;
      *reinterpret_cast<f32x4*>(wq + 2 * E128_TILE_FLOATS) = b10;
      *reinterpret_cast<f32x4*>(wq + 3 * E128_TILE_FLOATS) = b11;
    }
    wg_lds_barrier();
    DEMO_PHASE(0);

    // ---- the rows of the next chunk: requested a quarter per step of the products (sixteen requests per lane issued
    //      at one point queue up in the memory pipeline and hold the wavefront there), in flight until the top of the
    //      next turn -----------------------------------------------------------------------------------------------
    if (has_next) {
      while (nxt >= t_next) {
        ++t;
        t_first = t_next;
        t_next = uniform_prefix(tv, t + 1);
        d = load_desc_uniform(tv, t);
      }
      set_source(d, nxt - t_first);
    }
    // ---- the two products of this wavefront's quadrant, columns v' = 32 jh .. 32 jh + 31 ---------------------------
    // first: Z[i][v'] = sum_j B_ab[i][j] M_b[v'][j], A = B_ab from the tile (row 16 it + c; the eight j of a slot group
    // are two 16-byte reads), B = fragments.  The accumulators of two row tiles are, as they lie, the eight contraction
    // slots of the second, Q[u'][v'] += sum_i M_a[u'][i] Z[i][v'], A = fragments.
    f32x4 Q[4][2];   // [ut][vt - 2 jh]: coefficient (2 (16 ut + 4 g + r) + a, 2 (16 vt + c) + b), scaled
    {
      const int g = lanev >> 4, c = lanev & 15;
#pragma unroll
      for (int ut = 0; ut < 4; ++ut)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) Q[ut][jj] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int hp = 0; hp < 2; ++hp) {
        f32x4 Z[2][2];   // [it - 2 hp][vt - 2 jh]
#pragma unroll
        for (int uu = 0; uu < 2; ++uu)
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) Z[uu][jj] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          SplitH8 A[2];
#pragma unroll
          for (int uu = 0; uu < 2; ++uu) {
            const float* arow = &tq[(16 * (2 * hp + uu) + c) * E128_LDT + 4 * g + 32 * h];
            const float4 a0 = *reinterpret_cast<const float4*>(arow);
            const float4 a1 = *reinterpret_cast<const float4*>(arow + 16);
            A[uu] = split8h(m1h, a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w);
          }
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) {
            const SplitH8 Bq = load_split8h(TB + (2 * (2 * jh + jj) + h) * kSplitHFragFloats, lanev);
#pragma unroll
            for (int uu = 0; uu < 2; ++uu) Z[uu][jj] = mfma_f16(A[uu].lo, Bq.hi, Z[uu][jj]);
#pragma unroll
            for (int uu = 0; uu < 2; ++uu) Z[uu][jj] = mfma_f16(A[uu].hi, Bq.lo, Z[uu][jj]);
#pragma unroll
            for (int uu = 0; uu < 2; ++uu) Z[uu][jj] = mfma_f16(A[uu].hi, Bq.hi, Z[uu][jj]);
          }
          if (has_next) issue_rows_part((uint32_t)tidv, 2 * hp + h);
        }
        SplitH8 Bt[2];
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
          Bt[jj] = split8h(m1h, Z[0][jj][0], Z[0][jj][1], Z[0][jj][2], Z[0][jj][3], Z[1][jj][0], Z[1][jj][1], Z[1][jj][2], Z[1][jj][3]);
#pragma unroll
        for (int ut = 0; ut < 4; ++ut) {
          const SplitH8 Ap = load_split8h(TA + (2 * ut + hp) * kSplitHFragFloats, lanev);
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) Q[ut][jj] = mfma_f16(Ap.lo, Bt[jj].hi, Q[ut][jj]);
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) Q[ut][jj] = mfma_f16(Ap.hi, Bt[jj].lo, Q[ut][jj]);
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) Q[ut][jj] = mfma_f16(Ap.hi, Bt[jj].hi, Q[ut][jj]);
        }
      }
    }
    DEMO_PHASE(1);

    // ---- top-k over the 16384 coefficients -----------------------------------------------------------------
    // (1) lower bound of the k-th largest magnitude: the k-th largest of the 128 maxima of groups of 4 lanes
    //     (each a coefficient of its own), resolved to its upper 16 bits
    float gm[4][2];   // largest magnitude of each accumulator
    float lmf = 0.f;
#pragma unroll
    for (int ut = 0; ut < 4; ++ut)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        gm[ut][jj] = fmaxf(fmaxf(fabsf(Q[ut][jj][0]), fabsf(Q[ut][jj][1])), fmaxf(fabsf(Q[ut][jj][2]), fabsf(Q[ut][jj][3])));
        lmf = fmaxf(lmf, gm[ut][jj]);
      }
    uint32_t lm = __float_as_uint(lmf);
    lm = max(lm, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lm, 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
    lm = max(lm, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lm, 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
    if ((lanev & 3) == 0) gmax[16 * wave + (lanev >> 2)] = lm;
    wg_lds_barrier();
    if (wave == 0) {
      // one wavefront bisects (eight doing the same would only queue at the scalar unit)
      const uint32_t g0 = gmax[lanev], g1 = gmax[lanev + 64];
      uint32_t t0 = 0;
      for (int bit = 30; bit >= 16; --bit) {
        const uint32_t cnd = t0 | (1u << bit);
        if (__popcll(__ballot(g0 >= cnd)) + __popcll(__ballot(g1 >= cnd)) >= k) t0 = cnd;
      }
      const bool none = __ballot((g0 | g1) != 0u) == 0;
      if (lane == 0) {
        ctl[1] = (int)t0;
        ctl[2] = none ? 1 : 0;
      }
    }
    wg_lds_barrier();
    DEMO_PHASE(2);
    const float thr_f = __uint_as_float((uint32_t)__builtin_amdgcn_readfirstlane(ctl[1]));
    // (2) candidates |q| >= thr: a wavefront reserves its range of the list with one atomic.  Accumulators whose
    //     largest magnitude is below the threshold in every lane are passed over as a whole.
    {
      // lane part of the flat index 128 u + v = 4096 ut + 1024 g + 256 r + 128 a + 64 jh + 32 jj + 2 c + b
      const uint32_t fl = (uint32_t)(1024 * (lanev >> 4) + 2 * (lanev & 15) + 128 * (quad >> 1) + 64 * jh + (quad & 1));
      int cnt = 0;
#pragma unroll
      for (int ut = 0; ut < 4; ++ut)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
          if (__ballot(gm[ut][jj] >= thr_f) != 0) {
#pragma unroll
            for (int r = 0; r < 4; ++r) cnt += __popcll(__ballot(fabsf(Q[ut][jj][r]) >= thr_f));
          }
      int base = 0;
      if (lane == 0 && cnt != 0) base = atomicAdd(&ctl[0], cnt);
      base = __builtin_amdgcn_readfirstlane(base);
#pragma unroll
      for (int ut = 0; ut < 4; ++ut)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
          if (__ballot(gm[ut][jj] >= thr_f) != 0) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const bool is = fabsf(Q[ut][jj][r]) >= thr_f;
              const uint64_t mask = __ballot(is);
              if (mask != 0) {
                const int pos = base + lanes_below(mask);
                if (is && pos < W128_CAP) cand[pos] = make_uint2(__float_as_uint(Q[ut][jj][r]), fl + (uint32_t)(4096 * ut + 256 * r + 32 * jj));
                base += __popcll(mask);
              }
            }
          }
    }
    wg_lds_barrier();
    DEMO_PHASE(3);
    const int ncand = __builtin_amdgcn_readfirstlane(ctl[0]);
    const bool overflow = ncand > W128_CAP;
    const bool all_zero = overflow && __builtin_amdgcn_readfirstlane(ctl[2]) != 0;
    const bool skip = overflow && !all_zero;
    if (skip && tid == 0) store_guarded(&wl.list[atomicAdd(wl.count, 1)], chunk);
    if (all_zero && tid < k) {
      // every coefficient is zero: the k lowest flat indices with zero values; m = D is stored below
      store_guarded(out_idx + tid, (int32_t)tid);
      store_guarded(out_val + tid, 0.f);
    }
    // (3) rank the candidates (magnitude descending, flat index ascending).  Wavefront w counts, for every
    //     candidate, the entries of its slice of the list that precede it, and those among them of the same class
    //     2 (u % 2) + v % 2; the eight partial counts meet in rk[].
    if (!overflow) {
      const int slice = 2 * ((ncand + 15) >> 4);
      const int j0 = wave * slice;
      if (j0 < ncand) {
        for (int ib = 0; 64 * ib < ncand; ++ib) {
          const int i = 64 * ib + lane;
          const uint2 me = cand[i < ncand ? i : W128_CAP];
          const uint32_t mag = me.x & 0x7fffffffu;
          uint32_t part = 0;
          for (int j = j0; j < j0 + slice; j += 2) {
            const uint4 o = *reinterpret_cast<const uint4*>(&cand[j]);
            const uint32_t m0 = o.x & 0x7fffffffu, m1 = o.z & 0x7fffffffu;
            const bool p0 = m0 > mag || (m0 == mag && o.y < me.y), p1 = m1 > mag || (m1 == mag && o.w < me.y);
            part += (p0 ? (((o.y ^ me.y) & 0x81u) == 0 ? 0x10001u : 1u) : 0u) +
                    (p1 ? (((o.w ^ me.y) & 0x81u) == 0 ? 0x10001u : 1u) : 0u);
          }
          if (i < ncand && part != 0) atomicAdd(&rk[i], part);
        }
      }
    }
    wg_lds_barrier();
    // ranks < k are the payload; a selected coefficient also goes to the list of its class, at the number of
    // class members ahead of it (a deterministic order of summation for the reconstruction)
    if (!overflow && tidv < ncand) {
      const uint2 me = cand[tidv];
      const uint32_t r2 = rk[tidv];
      const int rank = (int)(r2 & 0xffffu), rcls = (int)(r2 >> 16);
      if (rank < k) {
        const float val = ldexpf(__uint_as_float(me.x), -sexp - 2 * kSplitHBasisLog2);   // exact
        store_guarded(out_idx + rank, (int32_t)me.y);
        store_guarded(out_val + rank, val);
        const int cls = (int)(((me.y >> 6) & 2u) | (me.y & 1u));
        // byte offsets of rows pos3(u) and pos3(v) of the basis tile, and the value
        const uint32_t offs = (uint32_t)(pos3(me.y >> 7) * (W128_LDP * 4)) | ((uint32_t)(pos3(me.y & 127u) * (W128_LDP * 4)) << 16);
        sel[cls * W128_SEL + rcls] = make_uint2(offs, __float_as_uint(val));
        atomicAdd(&ctl[4 + cls], 1);
      }
    }
    wg_lds_barrier();
    DEMO_PHASE(4);

    // ---- reconstruction on the quadrant i, j < 64, one partial sum per class (a, b) = (u % 2, v % 2), written to
    //      the quadrant tiles (the folded values are dead): row tile mt, column tiles nt0 and nt0 + 1 ---------------
    {
      const int mt = wave >> 1, nt0 = 2 * (wave & 1);
      const int lqv = lanev >> 4, l16v = lanev & 15;
      f32x4 rc[2][4];
#pragma unroll
      for (int n = 0; n < 2; ++n)
#pragma unroll
        for (int c = 0; c < 4; ++c) rc[n][c] = (f32x4){0.f, 0.f, 0.f, 0.f};
      // the lists are zero-padded, so every class runs to the length of the longest
      const int4 nc = *reinterpret_cast<const int4*>(&ctl[4]);
      const int nmax = __builtin_amdgcn_readfirstlane(max(max(nc.x, nc.y), max(nc.z, nc.w)));
      const float* pa = sP + 16 * mt + l16v;
      const float* pb = sP + 16 * nt0 + l16v;
      uint2 en[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) en[c] = sel[c * W128_SEL + lqv];
      for (int st = 0; 4 * st < nmax; ++st) {
        uint2 e[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) e[c] = en[c];
        float a[4], b0[4], b1[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          a[c] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(pa) + (e[c].x & 0xffffu));
          b0[c] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(pb) + (e[c].x >> 16));
          b1[c] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(pb + 16) + (e[c].x >> 16));
        }
        // entries of the next step (the lists are 68 long and zero past their ends: step 16 reads padding)
#pragma unroll
        for (int c = 0; c < 4; ++c) en[c] = sel[c * W128_SEL + 4 * (st + 1) + lqv];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          // the column factor as A operand, the row factor as B: component r of the result is column
          // 16 nt + 4 lq + r of row 16 mt + l16, four consecutive columns per lane
          const float va = __uint_as_float(e[c].y) * a[c];
          rc[0][c] = mfma4(b0[c], va, rc[0][c]);
          rc[1][c] = mfma4(b1[c], va, rc[1][c]);
        }
      }
#pragma unroll
      for (int n = 0; n < 2; ++n)
#pragma unroll
        for (int c = 0; c < 4; ++c)
          *reinterpret_cast<f32x4*>(&tiles[c * E128_TILE_FLOATS + (16 * mt + l16v) * E128_LDT + 16 * (nt0 + n) + 4 * lqv]) = rc[n][c];
    }
    wg_lds_barrier();
    DEMO_PHASE(5);

    // The stores are unconditional (a queued chunk's go to a buffer of zero records, where the range check drops
    // them): behind conditional stores the wait for the next chunk's rows would be a wait for everything outstanding.
    const __amdgpu_buffer_rsrc_t mres_out = skip ? make_rsrc_empty(mom_out) : make_rsrc(mom_out);
    // ---- m <- D - alpha R, R unfolded from the four class sums:  R[i][j] = sum s_ab,  R[i][127-j] = sum (-1)^b s_ab,
    //      R[127-i][j] = sum (-1)^a s_ab,  R[127-i][127-j] = sum (-1)^(a+b) s_ab -----------------------------------------
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const uint32_t pb = (uint32_t)tidv + E128_THREADS * p, ir = pb >> 4, j0 = (pb & 15u) * 4u;
      const float* rq = tiles + ir * E128_LDT + j0;
      const f32x4 q00 = *reinterpret_cast<const f32x4*>(rq), q01 = *reinterpret_cast<const f32x4*>(rq + E128_TILE_FLOATS);
      const f32x4 q10 = *reinterpret_cast<const f32x4*>(rq + 2 * E128_TILE_FLOATS);
      const f32x4 q11 = *reinterpret_cast<const f32x4*>(rq + 3 * E128_TILE_FLOATS);
      const f32x4 ea = q00 + q01, eb = q00 - q01, oa = q10 + q11, ob = q10 - q11;
      f32x4 rr[4];
      rr[0] = ea + oa;
      rr[2] = ea - oa;
      const f32x4 m1 = eb + ob, m3 = eb - ob;   // columns 127 - j0 - e: reversed within the segment
      rr[1] = (f32x4){m1[3], m1[2], m1[1], m1[0]};
      rr[3] = (f32x4){m3[3], m3[2], m3[1], m3[0]};
#pragma unroll
      for (int sg = 0; sg < 4; ++sg) {
        f32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = __fmaf_rn(-args.alpha, rr[sg][e], D[p][sg][e]);
        bstore_f4(mres_out, seg_offset((uint32_t)tidv, p, sg, ucols) * 4, 0u, o);
      }
    }
    DEMO_PHASE(6);
    if (!has_next) break;
    chunk = nxt;
  }
  DEMO_PHASE_FLUSH(0);
}

template <bool GBF16>
static hipError_t launch_enc_wg128(const TableView& tv, const float* basis, const float* tables, const EncodeArgs& a,
                                   const Worklist& wl, int64_t grid, hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&encode2d_quad128<GBF16>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, E128_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(encode2d_quad128<GBF16>, dim3((unsigned)grid), dim3(E128_THREADS), E128_LDS_BYTES, stream, tv,
                     basis, tables, a, wl);
  return hipGetLastError();
}

hipError_t launch_encode2d_wg128(const TableView& tv, const float* basis, const float* tables, const EncodeArgs& a,
                                 const Worklist& wl, bool grad_bf16, int num_cus, hipStream_t stream) {
  if (a.k < 1 || a.k > kFast128MaxK || wl.list == nullptr || tables == nullptr) return hipErrorInvalidValue;
  int64_t grid = num_cus;
  if (grid > tv.total_chunks) grid = tv.total_chunks;
  return grad_bf16 ? launch_enc_wg128<true>(tv, basis, tables, a, wl, grid, stream)
                   : launch_enc_wg128<false>(tv, basis, tables, a, wl, grid, stream);
}

// ---------------------------------------------------------------------------
// decode:  S = sum over workers of the payloads ;  R = P^T S P ;  x <- x - lr (sgn(R) + wd x)     (Algorithm 1, update)
// ---------------------------------------------------------------------------
// One 512-thread workgroup (8 wavefronts) per chunk.  Row u of the 128-point DCT-II is even (u even) or odd (u odd)
// under i -> 127 - i, so with A[u'][i] = P[2u'][i], O[u'][i] = P[2u'+1][i] (i < 64) and the coefficients sorted by the
// parities (a, b) of (u, v) into four 64 x 64 quadrants S_ab[u'][v'] = S[2u'+a][2v'+b], the four two-sided products
//   R_ab = M_a^T S_ab M_b,   M_0 = A, M_1 = O      (64 x 64 x 64 each)
// give, for i, j < 64,
//   R[i][j] = R_00 + R_01 + R_10 + R_11,  R[i][127-j] = R_00 - R_01 + R_10 - R_11,
//   R[127-i][j] = R_00 + R_01 - R_10 - R_11,  R[127-i][127-j] = R_00 - R_01 - R_10 + R_11:
// a quarter of the multiplications of the full products.  The quadrant products run on the float16 matrix pipe with
// both operands split into two parts (demo_device.h; 3 instructions of 16 cycles per 32 contraction indices where the
// float32 instruction needs 8 of 32 cycles), two wavefronts per quadrant, each with half of the rows i of R_ab: the
// chain is run transposed, R_ab^T = M_b^T (S_ab^T M_a), in which rows i are independent through both products, the
// accumulators of the first are, as they lie, operands of the second (as in the full-product instance of
// demo_dec64.hip) and those of the second hold four consecutive columns of a row; nothing but S and the four R_ab
// passes through LDS.
// The W k <= 4096 pairs of a chunk sit in at most eight registers per lane (pair 512 j + tid belongs to worker p / k,
// position p % k) and are fetched for the next chunk while the products of this one run.  S is accumulated in block
// fixed point with integer LDS atomics (one scale per chunk: the sum is exact and independent of the order of arrival).
// Thread t owns, for p < 2, row i = (t + 512 p) / 16 and columns j0 = 4 ((t + 512 p) % 16) .. j0 + 3 of the quadrants,
// i.e. the parameters (i, j0..), (i, 124 - j0..), (127 - i, j0..), (127 - i, 124 - j0..): sixteen lanes cover a whole
// 128-element row segment of the chunk with either pair of accesses.
namespace {
constexpr int Q128_WAVES = 8;
constexpr int Q128_THREADS = 64 * Q128_WAVES;
constexpr int Q128_LDT = 68;                                    // quadrant row stride (floats); columns 64..67 are pad slots
constexpr int Q128_TILE_FLOATS = 64 * Q128_LDT;
constexpr int Q128_TILES_FLOATS = 4 * Q128_TILE_FLOATS;
constexpr int Q128_FRAGS = 8 * kSplitHFragFloats;               // fragment table of one 64 x 64 matrix
constexpr int Q128_TABLE_FLOATS = 2 * Q128_FRAGS;               // A, then O
constexpr int Q128_SLOTS = 8;
constexpr int Q128_LDS_BYTES = 4 * (Q128_TABLE_FLOATS + Q128_TILES_FLOATS + 32);
static_assert(kFast128MaxPairs == Q128_SLOTS * Q128_THREADS, "pairs per chunk held in registers");
static_assert(Q128_TABLE_FLOATS == kDec128TableFloats, "table size");
static_assert(Q128_LDS_BYTES <= 160 * 1024, "LDS budget");
}  // namespace

// Host: pre-split float16 fragment tables of A and O (scaled by 2^kSplitHBasisLog2) from the 128 x 128 DCT matrix P
// (double, row-major).  Per matrix M the layout of the full-product s = 64 decode kernel: block 2 t + h, slot j of
// contraction group g holds M[16 (2 h + j / 4) + 4 g + j % 4][16 t + c].
void build_dec128_tables(const double* P, float* out) {
  for (int m = 0; m < 2; ++m)
    for (int t = 0; t < 4; ++t)
      for (int h = 0; h < 2; ++h)
        for (int lane = 0; lane < 64; ++lane) {
          float v[8];
          for (int j = 0; j < 8; ++j) {
            const int row = 16 * (2 * h + (j >> 2)) + 4 * (lane >> 4) + (j & 3);
            v[j] = (float)__builtin_ldexp(P[(2 * row + m) * 128 + 16 * t + (lane & 15)], kSplitHBasisLog2);
          }
          host_store_split8h(out + m * Q128_FRAGS + (2 * t + h) * kSplitHFragFloats, lane, v);
        }
}

// STREAM false: W k <= 4096, one pair per load (consecutive threads read consecutive pairs).  STREAM true: more than
// 4096 pairs per chunk (up to 65536), k a multiple of four and 16-byte aligned payload arrays: one pass in rounds of
// 4096 pairs, a thread fetching four consecutive pairs of one worker per load; the sums are shifted down whenever a
// round raises the block exponent.
// IDENT: phi is the identity on the aggregate instead of sgn (its own instance).  COUNT: the count-normalised
// aggregate of the appendix algorithm "Sparse Top-k Averaging" (every coefficient's sum divided by the number of pairs
// that name it), without STREAM only.
template <bool PBF16, bool STREAM, bool IDENT, bool COUNT = false>
__global__ __launch_bounds__(Q128_THREADS) void decode2d_quad128(TableView tv, const float* __restrict__ tables,
                                                                  DecodeArgs args) {
  constexpr bool VEC4 = STREAM;
  extern __shared__ float lds[];
  const float* sT = lds;
  float* tiles = lds + Q128_TABLE_FLOATS;
  int* itiles = reinterpret_cast<int*>(tiles);
  uint32_t* wmax = reinterpret_cast<uint32_t*>(tiles + Q128_TILES_FLOATS);   // [2][16] per-wavefront largest |val| (two buffers: consecutive rounds of a streamed payload alternate)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, c = lane & 15;
  const int k = args.k, W = args.W;
  const int npairs = W * k;
  const int nunits = npairs >> 2;                                  // VEC4: 16-byte units per chunk
  const int nslots = VEC4 ? Q128_SLOTS : (npairs + Q128_THREADS - 1) / Q128_THREADS;   // payload registers in use (uniform)
  const int nrounds = STREAM ? (nunits + 2 * Q128_THREADS - 1) / (2 * Q128_THREADS) : 1;
  const int total = tv.total_chunks;
  int chunk = blockIdx.x;
  if (chunk >= total) return;

  const float m1h = opaque_minus_one();
  for (int e = tid; e < Q128_TABLE_FLOATS / 4; e += Q128_THREADS)
    reinterpret_cast<f32x4*>(lds)[e] = gload_f4(tables + 4 * e);

  int32_t pi[Q128_SLOTS];
  float pv[Q128_SLOTS];
#pragma unroll
  for (int j = 0; j < Q128_SLOTS; ++j) {
    pi[j] = -1;
    pv[j] = 0.f;
  }
  const float rk = 1.0f / (float)k;
  // Payload requests in two steps: prep_payload forms every offset (units 1024 round + 512 jj + tid in STREAM mode,
  // pairs 512 j + tid otherwise), issue_payload_part(q), q < 4, requests a quarter of the registers.  Every offset
  // before the first load, and the loads unconditional (a slot past the end reads the chunk's first pair; mask_payload
  // discards it where the pairs are consumed): address arithmetic between the loads can pick up a register of a load
  // in flight as the unused high half of a 64-bit operand, and the wave then waits out that load before it issues
  // the next.
  const DEMO_GLOBAL int32_t* pl_ip = nullptr;
  const DEMO_GLOBAL float* pl_vp = nullptr;
  uint32_t pl_off[Q128_SLOTS];
#pragma unroll
  for (int j = 0; j < Q128_SLOTS; ++j) pl_off[j] = 0u;
  auto prep_payload = [&](const TensorDev& dd, int cc, int round) {
    pl_ip = as_global(dd.idx) + (int64_t)cc * k;
    pl_vp = as_global(dd.val) + (int64_t)cc * k;
    const int wstride = dd.nchunks * k;                        // pairs of one worker for this tensor
    if constexpr (VEC4) {
      static_assert(Q128_SLOTS == 8, "two 16-byte loads per array fill the payload registers");
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) {
        const int unit = (STREAM ? 2 * Q128_THREADS * round : 0) + Q128_THREADS * jj + tid;
        const int p = 4 * unit;
        const int w = (int)(((float)p + 0.5f) * rk);           // as below (p < 65536)
        const int pos = p - w * k;
        pl_off[jj] = unit < nunits ? (uint32_t)(w * wstride + pos) : 0u;
      }
    } else {
#pragma unroll
      for (int j = 0; j < Q128_SLOTS; ++j) {
        const int p = Q128_THREADS * j + tid;
        // worker p / k and position p % k; (p + 1/2) / k is never within 1/(2k) of an integer, far more than
        // the rounding error of the float product for p < 4096
        const int w = (int)(((float)p + 0.5f) * rk);
        const int pos = p - w * k;
        pl_off[j] = p < npairs ? (uint32_t)w * (uint32_t)wstride + (uint32_t)pos : 0u;
      }
    }
  };
  auto issue_payload_part = [&](int q) {
    if constexpr (VEC4) {
      if (q < 2) {
        const f32x4 vv = payload_load<true>(reinterpret_cast<const DEMO_GLOBAL f32x4*>(pl_vp + pl_off[q]));
#pragma unroll
        for (int e = 0; e < 4; ++e) pv[4 * q + e] = vv[e];
        const u32x4 iv = payload_load<true>(reinterpret_cast<const DEMO_GLOBAL u32x4*>(pl_ip + pl_off[q]));
#pragma unroll
        for (int e = 0; e < 4; ++e) pi[4 * q + e] = (int32_t)iv[e];
      }
    } else {
#pragma unroll
      for (int j = 2 * q; j < 2 * q + 2; ++j) {
        if (j < nslots) {                                      // uniform
          pi[j] = payload_load<true>(pl_ip + pl_off[j]);
          pv[j] = payload_load<true>(pl_vp + pl_off[j]);
        }
      }
    }
  };
  auto load_payload = [&](const TensorDev& dd, int cc, int round = 0) {
    prep_payload(dd, cc, round);
#pragma unroll
    for (int q = 0; q < 4; ++q) issue_payload_part(q);
  };
  // Slots past the end of the chunk's payload become (no index, 0).  Applied where the pairs are consumed, not where
  // they are requested: a select behind the load would make the prefetch wait for its own data.
  auto mask_payload = [&](int round = 0) {
#pragma unroll
    for (int j = 0; j < Q128_SLOTS; ++j) {
      const bool ok = VEC4 ? (STREAM ? 2 * Q128_THREADS * round : 0) + Q128_THREADS * (j >> 2) + tid < nunits
                           : Q128_THREADS * j + tid < npairs;
      pi[j] = ok ? pi[j] : -1;
      pv[j] = ok ? pv[j] : 0.f;
    }
  };
  // coefficient (u, v) lives in quadrant 2 (u % 2) + v % 2, transposed, at (v / 2, u / 2): the products below form
  // R_ab^T = M_b^T S_ab^T M_a, whose accumulators hold four consecutive columns j of a row i of R_ab per lane (16-byte
  // stores into the quadrant).  Lanes with nothing to add use a pad slot.
  const uint32_t dummy = (uint32_t)((tid & 63) * Q128_LDT + 64 + ((tid >> 6) & 3));
  auto slot_of = [&](int j) {
    const uint32_t fi = (uint32_t)pi[j];
    const uint32_t a = (((fi >> 6) & 2u) | (fi & 1u)) * (uint32_t)Q128_TILE_FLOATS + ((fi & 127u) >> 1) * (uint32_t)Q128_LDT + (fi >> 8);
    return fi < 16384u ? a : dummy;
  };

  int t = find_tensor_uniform(tv, chunk);
  int t_first = uniform_prefix(tv, t), t_next = uniform_prefix(tv, t + 1);
  TensorDev d = load_desc_uniform(tv, t);
  load_payload(d, chunk - t_first, 0);
  // the first chunk's pairs are waited for here, outside the loop: with loads pending at the loop's entry and
  // the parameter stores pending on its back edge, the loop's first wait would be for everything outstanding,
  // i.e. every chunk would begin by waiting for the acknowledgements of the previous chunk's stores
#pragma unroll
  for (int j = 0; j < Q128_SLOTS; ++j) asm volatile("" : "+v"(pi[j]), "+v"(pv[j]));

  int vbits = 30;
  for (int w = 1; w < W; w <<= 1) --vbits;                     // 30 - ceil(log2 W)
  // products: quadrant of this wavefront, its half of the rows i, the two fragment tables
  const int quad = wave >> 1, jh = wave & 1;
  const float* tq = tiles + quad * Q128_TILE_FLOATS;
  const float* TB = sT + (quad >> 1) * Q128_FRAGS;             // first product: M_a, the row class
  const float* TA = sT + (quad & 1) * Q128_FRAGS;              // second product: M_b, the column class

  // per-wavefront largest magnitude (as bits) of the payload registers into wmax buffer `buf`
  auto post_wave_max = [&](int buf) {
    float mx = 0.f;
#pragma unroll
    for (int j = 0; j < Q128_SLOTS; ++j)
      if (j < nslots) mx = fmaxf(mx, fabsf(pv[j]));
    uint32_t mb = __float_as_uint(mx);
    mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
    mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
    mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x141, 0xf, 0xf, false));  // row_half_mirror
    mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x140, 0xf, 0xf, false));  // row_mirror
    const uint32_t m01 = max((uint32_t)__builtin_amdgcn_readlane((int)mb, 0), (uint32_t)__builtin_amdgcn_readlane((int)mb, 16));
    const uint32_t m23 = max((uint32_t)__builtin_amdgcn_readlane((int)mb, 32), (uint32_t)__builtin_amdgcn_readlane((int)mb, 48));
    if (lane == 0) wmax[16 * buf + wave] = max(m01, m23);
  };
  // shift of the block fixed point from the eight posted maxima (after a barrier)
  auto shift_from = [&](int buf) {
    uint32_t mall = wmax[16 * buf + (lane & 7)];
    mall = max(mall, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mall, 0xB1, 0xf, 0xf, false));
    mall = max(mall, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mall, 0x4E, 0xf, 0xf, false));
    mall = max(mall, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mall, 0x141, 0xf, 0xf, false));
    mall = max(mall, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mall, 0x140, 0xf, 0xf, false));
    int ex = (int)((uint32_t)__builtin_amdgcn_readfirstlane((int)mall) >> 23);   // biased exponent of the largest magnitude
    ex = ex < 1 ? 1 : ex;
    return vbits + 126 - ex;                                 // max |val| * 2^sh < 2^vbits
  };
  auto add_pairs = [&](int sh) {
#pragma unroll
    for (int j = 0; j < Q128_SLOTS; ++j)
      if (j < nslots) atomicAdd(&itiles[slot_of(j)], __float2int_rn(ldexpf(pv[j], sh)));
  };
  // first chunk: pairs masked, maxima posted, tiles zero (for the others the epilogue of the chunk before does this)
  mask_payload(0);
  post_wave_max(0);
  for (int e = tid; e < Q128_TILES_FLOATS / 4; e += Q128_THREADS)
    *reinterpret_cast<f32x4*>(&tiles[4 * e]) = (f32x4){0.f, 0.f, 0.f, 0.f};
  wg_lds_barrier();

  DEMO_PHASE_DECL
  for (;;) {
    const int cc = chunk - t_first;
    const uint32_t ucols = (uint32_t)d.cols;
    const int64_t origin = (int64_t)(cc / d.cchunks) * 128 * d.cols + (int64_t)(cc % d.cchunks) * 128;
    const __amdgpu_buffer_rsrc_t xres = PBF16 ? make_rsrc(static_cast<const uint16_t*>(d.param) + origin)
                                              : make_rsrc(static_cast<const float*>(d.param) + origin);

    if constexpr (COUNT) {
      static_assert(!COUNT || !STREAM, "the count pass needs the whole payload in registers");
      // every pair adds one to its coefficient's slot, reads the total back and is divided by it (sum of val/n over
      // the n pairs of a slot = (sum of val) / n); the tiles are zero on entry and zeroed again below before the sums
      // go in
#pragma unroll
      for (int j = 0; j < Q128_SLOTS; ++j)
        if (j < nslots) atomicAdd(&itiles[slot_of(j)], 1);
      wg_lds_barrier();
#pragma unroll
      for (int j = 0; j < Q128_SLOTS; ++j)
        if (j < nslots) pv[j] = pv[j] / (float)itiles[slot_of(j)];
      wg_lds_barrier();
    }
    if constexpr (COUNT) {
      // (the count pass used the tiles and the registers changed: clear and post again)
      post_wave_max(0);
      for (int e = tid; e < Q128_TILES_FLOATS / 4; e += Q128_THREADS)
        *reinterpret_cast<f32x4*>(&tiles[4 * e]) = (f32x4){0.f, 0.f, 0.f, 0.f};
      wg_lds_barrier();
    }

    // ---- S[idx] += val in fixed point (the tiles are zero and the maxima posted: before the loop for the first
    //      chunk, by the epilogue of the chunk before for the others) ---------------------------------------------
    int sh_chunk = shift_from(0);   // shift of this chunk's fixed point (undone when phi is the identity)
    add_pairs(sh_chunk);
    if constexpr (STREAM) {
      // one pass over the payload: the registers held round 0; every further round is added with the block
      // exponent of the largest magnitude seen so far, and when a round raises that exponent the sums in the tiles
      // are first shifted down to the new scale (round to nearest, ties to even; every later shift at least halves the error of
      // an earlier one, so the shifts together cost at most one unit of the final scale per coefficient)
      for (int r = 1; r < nrounds; ++r) {
        load_payload(d, cc, r);
        mask_payload(r);
        post_wave_max(r & 1);
        wg_lds_barrier();   // maxima posted; the previous round's additions have landed
        const int sh_r = shift_from(r & 1);
        if (sh_r < sh_chunk) {   // uniform over the workgroup
          const int dsh = min(sh_chunk - sh_r, 31);
          const int half = (1 << (dsh - 1)) - 1;   // + the kept part's lowest bit: ties go to even (a bias would add up over the slots)
          for (int e = tid; e < Q128_TILES_FLOATS / 4; e += Q128_THREADS) {
            int4 v = *reinterpret_cast<int4*>(&itiles[4 * e]);
            v.x = (v.x + half + ((v.x >> dsh) & 1)) >> dsh;
            v.y = (v.y + half + ((v.y >> dsh) & 1)) >> dsh;
            v.z = (v.z + half + ((v.z >> dsh) & 1)) >> dsh;
            v.w = (v.w + half + ((v.w >> dsh) & 1)) >> dsh;
            *reinterpret_cast<int4*>(&itiles[4 * e]) = v;
          }
          wg_lds_barrier();
          sh_chunk = sh_r;
        }
        add_pairs(sh_chunk);
      }
    }
    // ---- payload of the next chunk and the parameters of this one: requested a quarter per step of the products
    //      (sixteen requests per lane issued at one point queue up in the memory pipeline and hold the wavefront there),
    //      in flight until the epilogue / the next turn ----------------------------------------------------------------
    const int nxt = chunk + (int)gridDim.x;
    const bool has_next = nxt < total;
    if (has_next) {
      while (nxt >= t_next) {
        ++t;
        t_first = t_next;
        t_next = uniform_prefix(tv, t + 1);
        d = load_desc_uniform(tv, t);
      }
      prep_payload(d, nxt - t_first, 0);
    }
    using XT = typename std::conditional<PBF16, u32x2, f32x4>::type;
    constexpr uint32_t XB = PBF16 ? 2u : 4u;                   // bytes per parameter
    XT xin[2][4];
    uint32_t xo[2][4];                                         // byte offsets of the four segments of position block p
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const uint32_t pb = (uint32_t)tid + Q128_THREADS * p, ir = pb >> 4, j0 = (pb & 15u) * 4u;
      xo[p][0] = (ir * ucols + j0) * XB;
      xo[p][1] = (ir * ucols + 124u - j0) * XB;
      xo[p][2] = ((127u - ir) * ucols + j0) * XB;
      xo[p][3] = ((127u - ir) * ucols + 124u - j0) * XB;
    }
    auto issue_step = [&](int q) __attribute__((always_inline)) {
      if (has_next) issue_payload_part(q);
#pragma unroll
      for (int sg = 2 * (q & 1); sg < 2 * (q & 1) + 2; ++sg) {
        if constexpr (PBF16) xin[q >> 1][sg] = bload_u2(xres, xo[q >> 1][sg], 0u);
        else xin[q >> 1][sg] = bload_f4(xres, xo[q >> 1][sg], 0u);
      }
    };
    wg_lds_barrier();
    DEMO_PHASE(0);

    // ---- the two products of this wavefront's quadrant, rows i = 32 jh .. 32 jh + 31 of R_ab ---------------------------
    // first: Y[v][i] = sum_u S_ab[u][v] M_a[u][i], A = S^T from the tile (row 16 vt + c; the eight u of a slot group
    // are two 16-byte reads), B = fragments.  The accumulators of two row tiles are, as they lie, the eight
    // contraction slots of the second, R_ab[i][j] += sum_v M_b[v][j] Y[v][i], A = fragments: component r of
    // R[jt][it - 2 jh] is R_ab[16 it + c][16 jt + 4 g + r].
    f32x4 R[4][2];   // [jt][it - 2 jh]
#pragma unroll
    for (int it = 0; it < 4; ++it)
#pragma unroll
      for (int jj = 0; jj < 2; ++jj) R[it][jj] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int hp = 0; hp < 2; ++hp) {
      f32x4 Y[2][2];   // [ut - 2 hp][jt - 2 jh]
#pragma unroll
      for (int uu = 0; uu < 2; ++uu)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) Y[uu][jj] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        SplitH8 A[2];   // the sums as float32 below 2^8 (integers below 2^30 in the tile), split
#pragma unroll
        for (int uu = 0; uu < 2; ++uu) {
          const float* arow = &tq[(16 * (2 * hp + uu) + c) * Q128_LDT + 4 * g + 32 * h];
          const float4 a0 = *reinterpret_cast<const float4*>(arow);
          const float4 a1 = *reinterpret_cast<const float4*>(arow + 16);
          constexpr float sc = 0x1p-22f;
          A[uu] = split8h(m1h, (float)__float_as_int(a0.x) * sc, (float)__float_as_int(a0.y) * sc, (float)__float_as_int(a0.z) * sc,
                          (float)__float_as_int(a0.w) * sc, (float)__float_as_int(a1.x) * sc, (float)__float_as_int(a1.y) * sc,
                          (float)__float_as_int(a1.z) * sc, (float)__float_as_int(a1.w) * sc);
        }
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
          const SplitH8 Bq = load_split8h(TB + (2 * (2 * jh + jj) + h) * kSplitHFragFloats, lane);
#pragma unroll
          for (int uu = 0; uu < 2; ++uu) Y[uu][jj] = mfma_f16(A[uu].lo, Bq.hi, Y[uu][jj]);
#pragma unroll
          for (int uu = 0; uu < 2; ++uu) Y[uu][jj] = mfma_f16(A[uu].hi, Bq.lo, Y[uu][jj]);
#pragma unroll
          for (int uu = 0; uu < 2; ++uu) Y[uu][jj] = mfma_f16(A[uu].hi, Bq.hi, Y[uu][jj]);
        }
        issue_step(2 * hp + h);
      }
      SplitH8 Bt[2];
#pragma unroll
      for (int jj = 0; jj < 2; ++jj)
        Bt[jj] = split8h(m1h, Y[0][jj][0], Y[0][jj][1], Y[0][jj][2], Y[0][jj][3], Y[1][jj][0], Y[1][jj][1], Y[1][jj][2], Y[1][jj][3]);
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const SplitH8 Ap = load_split8h(TA + (2 * it + hp) * kSplitHFragFloats, lane);
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) R[it][jj] = mfma_f16(Ap.lo, Bt[jj].hi, R[it][jj]);
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) R[it][jj] = mfma_f16(Ap.hi, Bt[jj].lo, R[it][jj]);
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) R[it][jj] = mfma_f16(Ap.hi, Bt[jj].hi, R[it][jj]);
      }
    }
    DEMO_PHASE(1);
    wg_lds_barrier();   // every read of S is done: the R_ab replace it
    {
      float* wq = tiles + quad * Q128_TILE_FLOATS;
#pragma unroll
      for (int it = 0; it < 4; ++it)
#pragma unroll
        for (int jj = 0; jj < 2; ++jj)
          *reinterpret_cast<f32x4*>(&wq[(16 * (2 * jh + jj) + c) * Q128_LDT + 16 * it + 4 * g]) = R[it][jj];
    }
    wg_lds_barrier();
    DEMO_PHASE(2);

    // ---- x <- x - lr (phi(R) + wd x): phi = sgn, or the identity on the aggregate (the quadrants hold R times
    //      2^sh 2^-22 2^(2 kSplitHBasisLog2); `scale` is 1 or 1/W) --------------------------------------------------
    const float factor = IDENT ? ldexpf(args.scale, 22 - 2 * kSplitHBasisLog2 - sh_chunk) : 0.f;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const uint32_t pb = (uint32_t)tid + Q128_THREADS * p, ir = pb >> 4, j0 = (pb & 15u) * 4u;
      const float* rq = tiles + ir * Q128_LDT + j0;
      const f32x4 q00 = *reinterpret_cast<const f32x4*>(rq), q01 = *reinterpret_cast<const f32x4*>(rq + Q128_TILE_FLOATS);
      const f32x4 q10 = *reinterpret_cast<const f32x4*>(rq + 2 * Q128_TILE_FLOATS);
      const f32x4 q11 = *reinterpret_cast<const f32x4*>(rq + 3 * Q128_TILE_FLOATS);
      // every element of the quadrants is read here and nowhere else: the reader leaves it zero for the next chunk
      {
        float* zq = tiles + ir * Q128_LDT + j0;
        const f32x4 z4 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int qd = 0; qd < 4; ++qd) *reinterpret_cast<f32x4*>(zq + qd * Q128_TILE_FLOATS) = z4;
      }
      const f32x4 ea = q00 + q01, eb = q00 - q01, oa = q10 + q11, ob = q10 - q11;
      f32x4 rr[4];   // segments (i, j0..), (i, 124 - j0..), (127 - i, j0..), (127 - i, 124 - j0..)
      rr[0] = ea + oa;
      rr[2] = ea - oa;
      const f32x4 m1 = eb + ob, m3 = eb - ob;   // columns 127 - j0 - e: reversed within the segment
      rr[1] = (f32x4){m1[3], m1[2], m1[1], m1[0]};
      rr[3] = (f32x4){m3[3], m3[2], m3[1], m3[0]};
#pragma unroll
      for (int sg = 0; sg < 4; ++sg) {
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float x;
          if constexpr (PBF16) {
            const uint32_t raw = xin[p][sg][e >> 1];
            x = __uint_as_float((e & 1) ? (raw & 0xffff0000u) : (raw << 16));
          } else {
            x = xin[p][sg][e];
          }
          o[e] = sign_update(x, IDENT ? rr[sg][e] * factor : sgnf(rr[sg][e]), args.lr, args.weight_decay);
        }
        if constexpr (PBF16) {
          const u32x2 pk = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
          bstore_u2(xres, xo[p][sg], 0u, pk);
        } else {
          const f32x4 ov = {o[0], o[1], o[2], o[3]};
          bstore_f4(xres, xo[p][sg], 0u, ov);
        }
      }
    }
    DEMO_PHASE(3);
    if (!has_next) break;
    chunk = nxt;
    mask_payload(0);
    post_wave_max(0);
    wg_lds_barrier();   // tiles zero, maxima posted
  }
  DEMO_PHASE_FLUSH(8);
}

// ---------------------------------------------------------------------------
// Few pairs per chunk (W k <= 64, e.g. a worker decoding its own payload): no coefficient tile and no products.
// R = sum_p val_p P[u_p]^T P[v_p] is accumulated per parity class by float32 MFMA chains whose operands are gathered
// rows of P, exactly as the encode kernel reconstructs its selection: wavefront 0 files the pairs by class
// 2 (u % 2) + v % 2 in the order of arrival (a deterministic order of summation; pairs of different workers that name
// the same coefficient simply add up), eight wavefronts accumulate the four class sums on the quadrant i, j < 64, and
// the epilogue of the tile kernel above unfolds them.  Sum and mean only (the count-normalised aggregate takes the
// tile kernel).
// ---------------------------------------------------------------------------
namespace {
constexpr int S128_THREADS = 512;
constexpr int S128_LDS_BYTES = 4 * (W128_P_FLOATS + Q128_TILES_FLOATS + 16) + 8 * (4 * W128_SEL);
}  // namespace

template <bool PBF16, bool IDENT>
__global__ __launch_bounds__(S128_THREADS) void decode2d_sparse128(TableView tv, const float* __restrict__ basis,
                                                                    DecodeArgs args) {
  extern __shared__ float lds[];
  float* sP = lds;
  float* tiles = sP + W128_P_FLOATS;
  int* ctl = reinterpret_cast<int*>(tiles + Q128_TILES_FLOATS);       // [0..3] class counts
  uint2* sel = reinterpret_cast<uint2*>(ctl + 16);                    // [4][SEL] {basis row offsets, value bits}
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int k = args.k, W = args.W;
  const int npairs = W * k;                                           // <= 64: one pair per lane of wavefront 0
  const int total = tv.total_chunks;
  int chunk = blockIdx.x;
  if (chunk >= total) return;

  for (int e = tid; e < 128 * 16; e += S128_THREADS) {
    const int u = e >> 4, c4 = (e & 15) * 4;
    *reinterpret_cast<f32x4*>(&sP[pos3((uint32_t)u) * W128_LDP + c4]) = gload_f4(basis + u * 128 + c4);
  }
  if (tid < 4 * W128_SEL) sel[tid] = make_uint2(0u, 0u);

  // pair `tid` of a chunk: worker tid / k, position tid % k
  const int pw = tid / k, pt = tid - pw * k;
  int32_t pi = -1;
  float pv = 0.f;
  auto load_pair = [&](const TensorDev& dd, int cc) {
    if (tid < npairs) {
      const int64_t off = ((int64_t)pw * dd.nchunks + cc) * k + pt;
      pi = payload_load<true>(as_global(dd.idx) + off);
      pv = payload_load<true>(as_global(dd.val) + off);
    }
  };
  int t = find_tensor_uniform(tv, chunk);
  int t_first = uniform_prefix(tv, t), t_next = uniform_prefix(tv, t + 1);
  TensorDev d = load_desc_uniform(tv, t);
  load_pair(d, chunk - t_first);
  asm volatile("" : "+v"(pi), "+v"(pv));   // waited for outside the loop (see the tile kernel)
  __syncthreads();

  for (;;) {
    const int cc = chunk - t_first;
    const uint32_t ucols = (uint32_t)d.cols;
    const int64_t origin = (int64_t)(cc / d.cchunks) * 128 * d.cols + (int64_t)(cc % d.cchunks) * 128;
    const __amdgpu_buffer_rsrc_t xres = PBF16 ? make_rsrc(static_cast<const uint16_t*>(d.param) + origin)
                                              : make_rsrc(static_cast<const float*>(d.param) + origin);
    // ---- the parameters of this chunk: requested now, used in the epilogue -------------------------------------
    using XT = typename std::conditional<PBF16, u32x2, f32x4>::type;
    constexpr uint32_t XB = PBF16 ? 2u : 4u;
    XT xin[2][4];
    uint32_t xo[2][4];
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const uint32_t pb = (uint32_t)tid + S128_THREADS * p, ir = pb >> 4, j0 = (pb & 15u) * 4u;
      xo[p][0] = (ir * ucols + j0) * XB;
      xo[p][1] = (ir * ucols + 124u - j0) * XB;
      xo[p][2] = ((127u - ir) * ucols + j0) * XB;
      xo[p][3] = ((127u - ir) * ucols + 124u - j0) * XB;
#pragma unroll
      for (int sg = 0; sg < 4; ++sg) {
        if constexpr (PBF16) xin[p][sg] = bload_u2(xres, xo[p][sg], 0u);
        else xin[p][sg] = bload_f4(xres, xo[p][sg], 0u);
      }
    }
    // ---- wavefront 0 files the pairs (the lists are zero: cleared before the loop / by the epilogue before) -------
    if (wave == 0) {
      const uint32_t fi = (uint32_t)pi;
      const bool valid = lane < npairs && fi < 16384u;
      const int cls = (int)(((fi >> 6) & 2u) | (fi & 1u));
      int rcls = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint64_t m = __ballot(valid && cls == c);
        if (cls == c) rcls = lanes_below(m);
        if (lane == 0) ctl[c] = __popcll(m);
      }
      if (valid) {
        const uint32_t offs = (uint32_t)(pos3(fi >> 7) * (W128_LDP * 4)) | ((uint32_t)(pos3(fi & 127u) * (W128_LDP * 4)) << 16);
        sel[cls * W128_SEL + rcls] = make_uint2(offs, __float_as_uint(pv));
      }
    }
    // ---- the pair of the next chunk ------------------------------------------------------------------------------
    const int nxt = chunk + (int)gridDim.x;
    const bool has_next = nxt < total;
    if (has_next) {
      while (nxt >= t_next) {
        ++t;
        t_first = t_next;
        t_next = uniform_prefix(tv, t + 1);
        d = load_desc_uniform(tv, t);
      }
      load_pair(d, nxt - t_first);
    }
    wg_lds_barrier();

    // ---- class sums on the quadrant i, j < 64: row tile mt, column tiles nt0 and nt0 + 1 ---------------------------
    {
      const int mt = wave >> 1, nt0 = 2 * (wave & 1);
      const int lq = lane >> 4, l16 = lane & 15;
      f32x4 rc[2][4];
#pragma unroll
      for (int n = 0; n < 2; ++n)
#pragma unroll
        for (int c = 0; c < 4; ++c) rc[n][c] = (f32x4){0.f, 0.f, 0.f, 0.f};
      // the lists are zero-padded, so every class runs to the length of the longest
      const int4 nc = *reinterpret_cast<const int4*>(&ctl[0]);
      const int nmax = __builtin_amdgcn_readfirstlane(max(max(nc.x, nc.y), max(nc.z, nc.w)));
      const float* pa = sP + 16 * mt + l16;
      const float* pb = sP + 16 * nt0 + l16;
      uint2 en[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) en[c] = sel[c * W128_SEL + lq];
      for (int st = 0; 4 * st < nmax; ++st) {
        uint2 e[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) e[c] = en[c];
        float a[4], b0[4], b1[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          a[c] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(pa) + (e[c].x & 0xffffu));
          b0[c] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(pb) + (e[c].x >> 16));
          b1[c] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(pb + 16) + (e[c].x >> 16));
        }
        // entries of the next step (the lists are 68 long and zero past their ends: step 16 reads padding)
#pragma unroll
        for (int c = 0; c < 4; ++c) en[c] = sel[c * W128_SEL + 4 * (st + 1) + lq];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          // the column factor as A operand, the row factor as B: four consecutive columns of a row per lane
          const float va = __uint_as_float(e[c].y) * a[c];
          rc[0][c] = mfma4(b0[c], va, rc[0][c]);
          rc[1][c] = mfma4(b1[c], va, rc[1][c]);
        }
      }
#pragma unroll
      for (int n = 0; n < 2; ++n)
#pragma unroll
        for (int c = 0; c < 4; ++c)
          *reinterpret_cast<f32x4*>(&tiles[c * Q128_TILE_FLOATS + (16 * mt + l16) * Q128_LDT + 16 * (nt0 + n) + 4 * lq]) = rc[n][c];
    }
    wg_lds_barrier();
    // the lists are read: cleared for the next chunk (entries in use only)
    if (tid < 4 * W128_SEL) sel[tid] = make_uint2(0u, 0u);

    // ---- x <- x - lr (phi(R) + wd x) ----------------------------------------------------------------------------------
    const float factor = IDENT ? args.scale : 0.f;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      const uint32_t pb = (uint32_t)tid + S128_THREADS * p, ir = pb >> 4, j0 = (pb & 15u) * 4u;
      const float* rq = tiles + ir * Q128_LDT + j0;
      const f32x4 q00 = *reinterpret_cast<const f32x4*>(rq), q01 = *reinterpret_cast<const f32x4*>(rq + Q128_TILE_FLOATS);
      const f32x4 q10 = *reinterpret_cast<const f32x4*>(rq + 2 * Q128_TILE_FLOATS);
      const f32x4 q11 = *reinterpret_cast<const f32x4*>(rq + 3 * Q128_TILE_FLOATS);
      const f32x4 ea = q00 + q01, eb = q00 - q01, oa = q10 + q11, ob = q10 - q11;
      f32x4 rr[4];   // segments (i, j0..), (i, 124 - j0..), (127 - i, j0..), (127 - i, 124 - j0..)
      rr[0] = ea + oa;
      rr[2] = ea - oa;
      const f32x4 m1 = eb + ob, m3 = eb - ob;   // columns 127 - j0 - e: reversed within the segment
      rr[1] = (f32x4){m1[3], m1[2], m1[1], m1[0]};
      rr[3] = (f32x4){m3[3], m3[2], m3[1], m3[0]};
#pragma unroll
      for (int sg = 0; sg < 4; ++sg) {
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float x;
          if constexpr (PBF16) {
            const uint32_t raw = xin[p][sg][e >> 1];
            x = __uint_as_float((e & 1) ? (raw & 0xffff0000u) : (raw << 16));
          } else {
            x = xin[p][sg][e];
          }
          o[e] = sign_update(x, IDENT ? rr[sg][e] * factor : sgnf(rr[sg][e]), args.lr, args.weight_decay);
        }
        if constexpr (PBF16) {
          const u32x2 pk = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
          bstore_u2(xres, xo[p][sg], 0u, pk);
        } else {
          const f32x4 ov = {o[0], o[1], o[2], o[3]};
          bstore_f4(xres, xo[p][sg], 0u, ov);
        }
      }
    }
    if (!has_next) break;
    chunk = nxt;
    wg_lds_barrier();   // lists cleared, quadrants read
  }
}

template <bool PBF16, bool IDENT>
static hipError_t launch_dec_sparse128(const TableView& tv, const float* basis, const DecodeArgs& a, int64_t grid,
                                       hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode2d_sparse128<PBF16, IDENT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, S128_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((decode2d_sparse128<PBF16, IDENT>), dim3((unsigned)grid), dim3(S128_THREADS), S128_LDS_BYTES, stream,
                     tv, basis, a);
  return hipGetLastError();
}

template <bool PBF16, bool STREAM, bool IDENT, bool COUNT = false>
static hipError_t launch_dec_wg128_phi(const TableView& tv, const float* basis, const DecodeArgs& a, int64_t grid,
                                       hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode2d_quad128<PBF16, STREAM, IDENT, COUNT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, Q128_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((decode2d_quad128<PBF16, STREAM, IDENT, COUNT>), dim3((unsigned)grid), dim3(Q128_THREADS),
                     Q128_LDS_BYTES, stream, tv, basis, a);
  return hipGetLastError();
}
template <bool PBF16, bool STREAM>
static hipError_t launch_dec_wg128(const TableView& tv, const float* basis, const DecodeArgs& a, int64_t grid,
                                   hipStream_t stream) {
  if constexpr (!STREAM) {
    if (a.agg == 2)
      return a.phi != 0 ? launch_dec_wg128_phi<PBF16, STREAM, true, true>(tv, basis, a, grid, stream)
                        : launch_dec_wg128_phi<PBF16, STREAM, false, true>(tv, basis, a, grid, stream);
  }
  return a.phi != 0 ? launch_dec_wg128_phi<PBF16, STREAM, true>(tv, basis, a, grid, stream)
                    : launch_dec_wg128_phi<PBF16, STREAM, false>(tv, basis, a, grid, stream);
}

hipError_t launch_decode2d_wg128(const TableView& tv, const float* basis, const float* tables, const DecodeArgs& a,
                                 bool param_bf16, int num_cus, hipStream_t stream) {
  if (!fast128_decode_supports(a.W, a.k, (tv.dtypes & 16u) == 0) || tables == nullptr) return hipErrorInvalidValue;
  if (a.agg == 2 && (int64_t)a.W * a.k > kFast128MaxPairs) return hipErrorInvalidValue;   // counted from registers
  int64_t grid = num_cus;
  if (grid > tv.total_chunks) grid = tv.total_chunks;
  if ((int64_t)a.W * a.k <= 64 && a.agg != 2) {
    if (a.phi != 0)
      return param_bf16 ? launch_dec_sparse128<true, true>(tv, basis, a, grid, stream)
                        : launch_dec_sparse128<false, true>(tv, basis, a, grid, stream);
    return param_bf16 ? launch_dec_sparse128<true, false>(tv, basis, a, grid, stream)
                      : launch_dec_sparse128<false, false>(tv, basis, a, grid, stream);
  }
  if ((int64_t)a.W * a.k > kFast128MaxPairs)
    return param_bf16 ? launch_dec_wg128<true, true>(tv, tables, a, grid, stream)
                      : launch_dec_wg128<false, true>(tv, tables, a, grid, stream);
  return param_bf16 ? launch_dec_wg128<true, false>(tv, tables, a, grid, stream)
                    : launch_dec_wg128<false, false>(tv, tables, a, grid, stream);
}

}  // namespace demo

DEMO_PHASE_GETTER(demo_debug_phase_clocks_wg128)
