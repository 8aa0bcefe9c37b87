// s = 64 encode kernel: one wavefront per 64 x 64 chunk, everything register resident.
//
// Register layout.  Lane l = 16 g + c.  For q = 4 s + w (s, w in 0..3) the lane loads the four
// consecutive floats  D[q][e] = B[rho(q,g)][4 chi(c) + e],  e = 0..3, where
//     rho(4s+w, g) = { i0, 31-i0, 32+i0, 63-i0 }[w],  i0 = 4s + g          (rows)
//     chi(4a+b)    = { a, 7-a, 8+a, 15-a }[b]                              (16-byte column groups)
// so 16 lanes still cover one 256-byte row per load instruction, and every lane holds, for each
// of its columns, complete mirror quadruples {i, 31-i, 32+i, 63-i} of rows.
//
// Transform.  Row u of the orthonormal DCT-II matrix P is even or odd under i -> 63-i according
// to the parity of u, and rows u = 0 mod 4 / 2 mod 4 are even / odd under i -> 31-i as well.  Two
// in-lane butterfly levels on each quadruple therefore split the 64-point transform into a
// 16 x 16 product (u = 4b), another 16 x 16 (u = 4b+2) and a 32 x 32 one (u odd): 3/8 of the
// multiply-adds of the dense product.  Q = P B P^T is computed as two chains of
// v_mfma_f32_16x16x4_f32 whose data operands never leave the register file:
//     product 1   T^T[j][u] = sum_i B[i][j] P[u][i]     A = butterflies of D,  B = basis fragments
//     product 2   Q^T[v][u] = sum_j P[v][j] T^T[j][u]   A = basis fragments,   B = butterflies of the
//                                                       product-1 accumulators
// (an accumulator tile holds rows 4g + r in lane group g, the k-slot layout of a B operand; the
// column-group map chi makes the mirror quadruples of j land in one lane as well).  Coefficient
// tiles come out in the order u = {4c, 4c+2, 2c+1, 2c+33}, v likewise with c -> 4g + r.
//
// Top-k runs inside the wavefront on the 64 coefficients each lane holds; the reconstruction
// m - P^T Q^ P is one more MFMA chain of contraction length k that accumulates straight into D,
// which is then stored with the load pattern.  LDS holds the basis fragment tables and a small
// candidate list per wavefront.
#include <type_traits>

#include "demo_device.h"

namespace demo {


namespace {

constexpr int E64_WAVES = 8;                      // wavefronts per workgroup (2 per SIMD)
constexpr int E64_THREADS = E64_WAVES * 64;
constexpr int E64_CAP = 128;                      // candidate list capacity per wavefront
constexpr int E64_T1 = 0;                         // product-1 fragments: 6 groups x 64 lanes x 4
constexpr int E64_T2 = 1536;                      // product-2 fragments
constexpr int E64_PCOL = 3072;                    // pcol[v*64 + 4c + e]  = P[v][4 chi(c) + e]
constexpr int E64_PK = 3072 + 4096;               // pk[u*16 + c]  = P[u][kappa(c)]       (reconstruction, quadruple bases)
constexpr int E64_PK2 = 3072 + 4096 + 1024;       // pk2[u*16 + c] = P[u][31 - kappa(c)]  (odd u: the second member)
constexpr int E64_TABLE_FLOATS = 3072 + 4096 + 2048;
// per-wavefront scratch: candidate value bits [LIST], candidate flat indices [LIST] (one gather step appends up to
// 64 entries to a list of at most CAP), 64-bit sort keys [64], selected {flat, value bits} by class [3][64]
constexpr int E64_LIST = E64_CAP + 64 + 2;
constexpr int E64_SCRATCH_WORDS = 2 * E64_LIST + 2 * 64 + 3 * 2 * 64;
static_assert(E64_LIST % 4 == 2 && (2 * E64_LIST) % 4 == 0 && E64_SCRATCH_WORDS % 4 == 0, "16-byte aligned key and list arrays");
__host__ __device__ constexpr int kappa64(int c) { return 4 * (c & 3) + (c >> 2); }
static_assert(E64_TABLE_FLOATS == kEnc64TableFloats, "table size");

// Tables of the instances for a projection matrix without mirror symmetry (DENSE).  The two products run on the
// float16 matrix pipe with every float32 operand split into two parts (demo_device.h): their basis fragments, scaled by
// 2^kSplitHBasisLog2, are stored pre-split, one block of kSplitHFragFloats words per (tile, half h of the contraction
// range); slot j of contraction group g stands for step 8 h + j of the sixteen steps the float32 instruction form
// would take.
constexpr int E64G_T1 = 0;                        // block 2 t + h, slot j:  P[16 t + c][rho(8 h + j, g)]              (product 1, B operand)
constexpr int E64G_T2 = 8 * kSplitHFragFloats;    // block 2 vt + h, slot j: P[16 vt + c][4 chi(4g + r) + e], 4 e + r = 8 h + j  (product 2, A operand)
constexpr int E64G_PCOL = 16 * kSplitHFragFloats; // pcol[v*64 + 4c + e]          = P[v][4 chi(c) + e]                (reconstruction, B operand)
constexpr int E64G_PROW = E64G_PCOL + 4096;       // prow[u*64 + 16 w + c]        = P[u][rho(4 (c%4) + w, c/4)]       (reconstruction, A operand)
constexpr int E64G_TABLE_FLOATS = E64G_PROW + 4096;
static_assert(E64G_TABLE_FLOATS == kEnc64DenseTableFloats, "table size");
template <bool DENSE>
constexpr int e64_table_floats() { return DENSE ? E64G_TABLE_FLOATS : E64_TABLE_FLOATS; }
template <bool DENSE>
constexpr int e64_lds_bytes() { return 4 * (e64_table_floats<DENSE>() + E64_WAVES * E64_SCRATCH_WORDS); }

}  // namespace

void build_enc64_dense_tables(const double* P, float* out) {
  auto Pm = [&](int u, int i) { return (float)P[u * 64 + i]; };
  for (int lane = 0; lane < 64; ++lane) {
    const int g = lane >> 4, c = lane & 15;
    for (int t = 0; t < 4; ++t)
      for (int h = 0; h < 2; ++h) {
        float v1[8], v2[8];
        for (int j = 0; j < 8; ++j) {
          const int q = 8 * h + j;   // product 1: step q; product 2: (e, r) = (q / 4, q % 4)
          v1[j] = (float)__builtin_ldexp(P[(16 * t + c) * 64 + rho(q, g)], kSplitHBasisLog2);
          v2[j] = (float)__builtin_ldexp(P[(16 * t + c) * 64 + 4 * chi(4 * g + (q & 3)) + (q >> 2)], kSplitHBasisLog2);
        }
        host_store_split8h(out + E64G_T1 + (2 * t + h) * kSplitHFragFloats, lane, v1);
        host_store_split8h(out + E64G_T2 + (2 * t + h) * kSplitHFragFloats, lane, v2);
      }
  }
  for (int u = 0; u < 64; ++u)
    for (int cc = 0; cc < 16; ++cc) {
      for (int x = 0; x < 4; ++x) out[E64G_PCOL + u * 64 + 4 * cc + x] = Pm(u, 4 * chi(cc) + x);
      for (int w = 0; w < 4; ++w) out[E64G_PROW + u * 64 + 16 * w + cc] = Pm(u, rho(4 * (cc & 3) + w, cc >> 2));
    }
}

void build_enc64_tables(const double* P, float* out) {
  auto Pm = [&](int u, int i) { return (float)P[u * 64 + i]; };
  for (int lane = 0; lane < 64; ++lane) {
    const int g = lane >> 4, c = lane & 15;
    for (int s = 0; s < 4; ++s) {
      // product 1: k-slot g of step s contracts row index i0 = 4s + g (or its mirror 31 - i0)
      const int i0 = 4 * s + g;
      out[E64_T1 + (0 * 64 + lane) * 4 + s] = Pm(4 * c, i0);
      out[E64_T1 + (1 * 64 + lane) * 4 + s] = Pm(4 * c + 2, i0);
      for (int w = 0; w < 2; ++w)
        for (int nt = 0; nt < 2; ++nt)
          out[E64_T1 + ((2 + s) * 64 + lane) * 4 + 2 * w + nt] = Pm(2 * (16 * nt + c) + 1, w ? 31 - i0 : i0);
      // product 2: k-slot g of step s contracts column index j0 = 4g + s (or 31 - j0); A rows = v
      const int j0 = 4 * g + s;
      out[E64_T2 + (0 * 64 + lane) * 4 + s] = Pm(4 * c, j0);
      out[E64_T2 + (1 * 64 + lane) * 4 + s] = Pm(4 * c + 2, j0);
      for (int w = 0; w < 2; ++w)
        for (int mt = 0; mt < 2; ++mt)
          out[E64_T2 + ((2 + s) * 64 + lane) * 4 + 2 * w + mt] = Pm(2 * (16 * mt + c) + 1, w ? 31 - j0 : j0);
    }
  }
  for (int u = 0; u < 64; ++u)
    for (int cc = 0; cc < 16; ++cc) {
      for (int x = 0; x < 4; ++x) out[E64_PCOL + u * 64 + 4 * cc + x] = Pm(u, 4 * chi(cc) + x);
      out[E64_PK + u * 16 + cc] = Pm(u, kappa64(cc));
      out[E64_PK2 + u * 16 + cc] = Pm(u, 31 - kappa64(cc));
    }
}

// the six values two butterfly levels make of a mirror quadruple (x[i], x[31-i], x[32+i], x[63-i])
struct Bfly {
  float ee, eo, o0, o1;
};
__device__ __forceinline__ Bfly butterfly(float x0, float x1, float x2, float x3) {
  const float e0 = x0 + x3, e1 = x1 + x2;
  return Bfly{e0 + e1, e0 - e1, x0 - x3, x1 - x2};
}

// STAGE 0 is the kernel.  STAGE 1..3 are cut-down copies for time attribution (they do not encode): 1 = the
// memory stream only (loads of g and m with the prefetch, momentum update, store of m, k payload pairs per chunk),
// 2 = stage 1 plus the two products, 3 = stage 2 plus top-k and the payload (everything but the reconstruction).
// DENSE: the projection matrix is any orthonormal 64 x 64 matrix (tables of build_enc64_dense_tables): the same
// register layout and the same top-k, with the full products (on the bfloat16 matrix pipe, float32 operands split
// into three parts: 192 v_mfma_f32_16x16x32_bf16 each, 3/8 of the time of 256 float32 instructions) and a reconstruction
// over all 64 rows (16 MFMAs per four selected coefficients); coefficient tiles hold u = 16 t + c, v = 16 vt + 4g + r.
template <bool GBF16, int STAGE, bool DENSE = false>   // gradient dtype of every tensor in the table
__global__ __launch_bounds__(E64_THREADS) void encode2d_wave64(TableView tv, const float* __restrict__ tables,
                                                               EncodeArgs args, Worklist wl) {
  extern __shared__ float lds[];
  constexpr int TABLE_FLOATS = e64_table_floats<DENSE>();
  const float* sT1 = lds + (DENSE ? E64G_T1 : E64_T1);
  const float* sT2 = lds + (DENSE ? E64G_T2 : E64_T2);
  const float* sPcol = lds + (DENSE ? E64G_PCOL : E64_PCOL);
  const float* sPk = lds + E64_PK;
  const float* sPk2 = lds + E64_PK2;
  const float* sProw = lds + E64G_PROW;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, c = lane & 15;
  uint32_t* scratch = reinterpret_cast<uint32_t*>(lds + TABLE_FLOATS) + wave * E64_SCRATCH_WORDS;
  uint32_t* cand_v = scratch;                                            // value bits of the candidates
  uint32_t* cand_f = scratch + E64_LIST;                                 // their flat indices
  uint2* keys = reinterpret_cast<uint2*>(scratch + 2 * E64_LIST);        // {~flat index, magnitude bits}
  uint2* sel = reinterpret_cast<uint2*>(scratch + 2 * E64_LIST + 128);   // [3][64] {flat index, value bits} by class of u
  const int k = args.k;
  [[maybe_unused]] const float m1h = opaque_minus_one();
  // LDS byte address of cand_v[0] as a scalar the compiler cannot take apart (it would otherwise re-add the
  // constant part of the address on every access)
  uint32_t list_base = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)(lds_u32*)cand_v);
  asm volatile("" : "+s"(list_base));

  for (int e = tid; e < TABLE_FLOATS / 4; e += E64_THREADS)
    reinterpret_cast<float4*>(lds)[e] = reinterpret_cast<const float4*>(tables)[e];
  __syncthreads();

  // wavefront w takes chunks w, w + nwaves, ...: at any time the wavefronts of the grid work on one
  // narrow band of memory, which the HBM channels serve faster than a far-apart range per wavefront
  const int nwaves = gridDim.x * E64_WAVES;
  const int wid = first_work_item<DEMO_RUN>(wave);
  const int total = tv.total_chunks;
  int chunk = wid;
  if (chunk >= total) return;
  int t = find_tensor_uniform(tv, chunk);
  int t_first = uniform_prefix(tv, t), t_next = uniform_prefix(tv, t + 1);
  TensorDev d = load_desc_uniform(tv, t);

  // lane constants: column offset, and flat-index bases u(t,c)*64 + v(vt,4g) of the coefficient tiles
  const int col4 = 4 * chi(c);
  uint32_t fb_a = DENSE ? (uint32_t)(64 * c + 4 * g) : (uint32_t)(256 * c + 16 * g), fb_b = (uint32_t)(256 * c + 8 * g);
  uint32_t fb_c = (uint32_t)(128 * c + 16 * g), fb_d = (uint32_t)(128 * c + 8 * g);

  // Where a chunk lives: row rho(4s+w, g) = rbase(q) + (w even ? g : 3 - g), i.e. a uniform part
  // (scalar offset of the buffer access) plus one of two per-lane offsets.
  struct Place {
    __amdgpu_buffer_rsrc_t mres, gres;
    uint32_t ucols, vo_up, vo_dn;   // elements
    int cc;
    int32_t* idx;
    float* val;
  };
  auto place = [&](const TensorDev& dd, int ccc) {
    const int k0 = ccc / dd.cchunks, k1 = ccc - k0 * dd.cchunks;
    const int64_t origin = (int64_t)k0 * 64 * dd.cols + (int64_t)k1 * 64;   // uniform
    Place p;
    p.ucols = (uint32_t)dd.cols;
    p.vo_up = (uint32_t)g * p.ucols + (uint32_t)col4;
    p.vo_dn = (uint32_t)(3 - g) * p.ucols + (uint32_t)col4;
    p.mres = make_rsrc(dd.mom + origin);
    p.gres = GBF16 ? make_rsrc(static_cast<const uint16_t*>(dd.grad) + origin)
                   : make_rsrc(static_cast<const float*>(dd.grad) + origin);
    p.cc = ccc;
    p.idx = dd.idx;
    p.val = dd.val;
    return p;
  };
  auto rbase = [](int q) { return rho_base(q); };

  // Raw inputs of the chunk being prefetched: its momentum rows are requested as soon as the
  // product-1 accumulators of the current chunk are dead, its gradient rows once top-k is done.
  f32x4 nm[16];
  u32x2 ng[16];    // bf16 gradients
  f32x4 ngf[16];   // fp32 gradients
  auto fetch_m = [&](const Place& p) {
#pragma unroll
    for (int q = 0; q < 16; ++q)
      nm[q] = bload_f4(p.mres, ((q & 1) ? p.vo_dn : p.vo_up) * 4, (uint32_t)rbase(q) * p.ucols * 4);
  };
  auto fetch_g = [&](const Place& p) {
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      if (GBF16)
        ng[q] = bload_u2(p.gres, ((q & 1) ? p.vo_dn : p.vo_up) * 2, (uint32_t)rbase(q) * p.ucols * 2);
      else
        ngf[q] = bload_f4(p.gres, ((q & 1) ? p.vo_dn : p.vo_up) * 4, (uint32_t)rbase(q) * p.ucols * 4);
    }
  };

  Place cur = place(d, chunk - t_first);
  fetch_m(cur);
  fetch_g(cur);

  // ---- momentum update: D[s][e][w] = element (row rho(4s+w, g), col 4 chi(c) + e), from the rows fetched last ----
  f32x4 D[4][4];
  // gs: coefficient of g; the multiplication is left out when it is 1 (the algorithm boxes' form)
  auto momentum = [&](auto unit_scale) {
    constexpr bool UNIT = decltype(unit_scale)::value;
    const float gs = args.grad_scale;
    if (GBF16) {
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const float g0 = __uint_as_float(ng[q][0] << 16), g1 = __uint_as_float(ng[q][0] & 0xffff0000u);
        const float g2 = __uint_as_float(ng[q][1] << 16), g3 = __uint_as_float(ng[q][1] & 0xffff0000u);
        D[q >> 2][0][q & 3] = __fmaf_rn(args.beta, nm[q][0], UNIT ? g0 : gs * g0);
        D[q >> 2][1][q & 3] = __fmaf_rn(args.beta, nm[q][1], UNIT ? g1 : gs * g1);
        D[q >> 2][2][q & 3] = __fmaf_rn(args.beta, nm[q][2], UNIT ? g2 : gs * g2);
        D[q >> 2][3][q & 3] = __fmaf_rn(args.beta, nm[q][3], UNIT ? g3 : gs * g3);
      }
    } else {
#pragma unroll
      for (int q = 0; q < 16; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) D[q >> 2][e][q & 3] = __fmaf_rn(args.beta, nm[q][e], UNIT ? ngf[q][e] : gs * ngf[q][e]);
    }
  };
  const bool unit_grad_scale = args.grad_scale == 1.0f;
  if (unit_grad_scale) momentum(std::true_type{}); else momentum(std::false_type{});

  // The loop carries D: the rows of the next chunk are requested while this chunk is worked on and turned into the
  // next D at the END of the body, behind this chunk's stores.  With the wait for those rows at the top of the body
  // instead, the two ways into it (first entry: nothing behind the loads; back edge: the stores behind them) would
  // leave the compiler only a wait for everything outstanding, i.e. for the stores' acknowledgements as well.
  DEMO_PHASE_DECL
  for (;;) {
    const int cc = cur.cc;
    const uint32_t ucols = cur.ucols, vo_up = cur.vo_up, vo_dn = cur.vo_dn;
    const __amdgpu_buffer_rsrc_t mres = cur.mres;
    // the chunk after this one (if any)
    const bool has_next = chunk + nwaves < total;
    Place nxt = cur;
    if (has_next) {
      while (chunk + nwaves >= t_next) {
        ++t;
        t_first = t_next;
        t_next = uniform_prefix(tv, t + 1);
        d = load_desc_uniform(tv, t);
      }
      nxt = place(d, chunk + nwaves - t_first);
    }
    __builtin_amdgcn_sched_barrier(0);

    DEMO_PHASE(0);
    bool skip = false;
    if constexpr (STAGE == 1) {
      fetch_m(nxt);
      if (GBF16) fetch_g(nxt);
      if (lane < k) {
        const int64_t po = (int64_t)cc * k + lane;
        store_guarded(as_global(cur.idx) + po, (int32_t)lane);
        store_guarded(as_global(cur.val) + po, D[0][0][0]);
      }
    } else {
    // ---- product 1: C1[e][t] rows j = 4 chi(4g+r) + e, cols u = freq(t, c) ------------------------
    f32x4 C1[4][4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) C1[e][tt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    [[maybe_unused]] int dense_unscale = 0;   // DENSE: the coefficients come out as Q 2^-dense_unscale
    if constexpr (DENSE) {
      // scale of the chunk: |D| < 2^(e+1) for the largest magnitude's exponent e, and 2^(7-e) brings the tile below
      // 2^8, the first product below 2^4 8 2^8 = 2^15 (float16 ends at 65504)
      float mx = 0.f;
#pragma unroll
      for (int s4 = 0; s4 < 4; ++s4)
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int w = 0; w < 4; ++w) mx = fmaxf(mx, fabsf(D[s4][e][w]));
      uint32_t mb = __float_as_uint(mx);
      mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
      mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
      mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x141, 0xf, 0xf, false));  // row_half_mirror
      mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x140, 0xf, 0xf, false));  // row_mirror
      const uint32_t m01 = max((uint32_t)__builtin_amdgcn_readlane((int)mb, 0), (uint32_t)__builtin_amdgcn_readlane((int)mb, 16));
      const uint32_t m23 = max((uint32_t)__builtin_amdgcn_readlane((int)mb, 32), (uint32_t)__builtin_amdgcn_readlane((int)mb, 48));
      int se = 261 - (int)(max(m01, m23) >> 23);               // biased exponent of 2^(7 - (ex - 127))
      se = se < 1 ? 1 : se > 254 ? 254 : se;                   // (chunks below 2^-119 keep fewer bits)
      const float sc = __uint_as_float((uint32_t)se << 23);
      dense_unscale = se - 127 + 2 * kSplitHBasisLog2;
      // contraction over the rows in two halves of 32: slot j of group g is row rho(8 h + j, g); the data are split
      // into float16 pairs once per half and serve the four tiles of u
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        SplitH8 A[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
          A[e] = split8h(m1h, D[2 * h][e][0] * sc, D[2 * h][e][1] * sc, D[2 * h][e][2] * sc, D[2 * h][e][3] * sc,
                         D[2 * h + 1][e][0] * sc, D[2 * h + 1][e][1] * sc, D[2 * h + 1][e][2] * sc, D[2 * h + 1][e][3] * sc);
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const SplitH8 Bq = load_split8h(sT1 + (2 * tt + h) * kSplitHFragFloats, lane);
#pragma unroll
          for (int e = 0; e < 4; ++e) C1[e][tt] = mfma_f16(A[e].lo, Bq.hi, C1[e][tt]);
#pragma unroll
          for (int e = 0; e < 4; ++e) C1[e][tt] = mfma_f16(A[e].hi, Bq.lo, C1[e][tt]);
#pragma unroll
          for (int e = 0; e < 4; ++e) C1[e][tt] = mfma_f16(A[e].hi, Bq.hi, C1[e][tt]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
      const float4 pee4 = *reinterpret_cast<const float4*>(&sT1[(0 * 64 + lane) * 4]);
      const float4 peo4 = *reinterpret_cast<const float4*>(&sT1[(1 * 64 + lane) * 4]);
      const float pee[4] = {pee4.x, pee4.y, pee4.z, pee4.w}, peo[4] = {peo4.x, peo4.y, peo4.z, peo4.w};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const float4 po4 = *reinterpret_cast<const float4*>(&sT1[((2 + s) * 64 + lane) * 4]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const Bfly b = butterfly(D[s][e][0], D[s][e][1], D[s][e][2], D[s][e][3]);
          C1[e][0] = mfma4(b.ee, pee[s], C1[e][0]);
          C1[e][1] = mfma4(b.eo, peo[s], C1[e][1]);
          C1[e][2] = mfma4(b.o0, po4.x, C1[e][2]);
          C1[e][3] = mfma4(b.o0, po4.y, C1[e][3]);
          C1[e][2] = mfma4(b.o1, po4.z, C1[e][2]);
          C1[e][3] = mfma4(b.o1, po4.w, C1[e][3]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    DEMO_PHASE(1);
    // ---- product 2: C2[vt][t] rows v = freq(vt, 4g+r), cols u = freq(t, c): Q[u][v] ----------------
    f32x4 C2[4][4];
#pragma unroll
    for (int vt = 0; vt < 4; ++vt)
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) C2[vt][tt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    if constexpr (DENSE) {
      // contraction over the columns j = 4 chi(4g + r) + e in two halves: slot j' of group g is (e, r) with
      // 4 e + r = 8 h + j'; the accumulators of product 1 are split as they lie and serve the four tiles of v
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        SplitH8 Bt[4];
#pragma unroll
        for (int tt = 0; tt < 4; ++tt)
          Bt[tt] = split8h(m1h, C1[2 * h][tt][0], C1[2 * h][tt][1], C1[2 * h][tt][2], C1[2 * h][tt][3],
                           C1[2 * h + 1][tt][0], C1[2 * h + 1][tt][1], C1[2 * h + 1][tt][2], C1[2 * h + 1][tt][3]);
#pragma unroll
        for (int vt = 0; vt < 4; ++vt) {
          const SplitH8 Ap = load_split8h(sT2 + (2 * vt + h) * kSplitHFragFloats, lane);
#pragma unroll
          for (int tt = 0; tt < 4; ++tt) C2[vt][tt] = mfma_f16(Ap.lo, Bt[tt].hi, C2[vt][tt]);
#pragma unroll
          for (int tt = 0; tt < 4; ++tt) C2[vt][tt] = mfma_f16(Ap.hi, Bt[tt].lo, C2[vt][tt]);
#pragma unroll
          for (int tt = 0; tt < 4; ++tt) C2[vt][tt] = mfma_f16(Ap.hi, Bt[tt].hi, C2[vt][tt]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      // back to the scale of the data (exact: a power of two)
#pragma unroll
      for (int vt = 0; vt < 4; ++vt)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt)
#pragma unroll
          for (int r = 0; r < 4; ++r) C2[vt][tt][r] = ldexpf(C2[vt][tt][r], -dense_unscale);
    } else {
      const float4 pee4 = *reinterpret_cast<const float4*>(&sT2[(0 * 64 + lane) * 4]);
      const float4 peo4 = *reinterpret_cast<const float4*>(&sT2[(1 * 64 + lane) * 4]);
      const float pee[4] = {pee4.x, pee4.y, pee4.z, pee4.w}, peo[4] = {peo4.x, peo4.y, peo4.z, peo4.w};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const float4 po4 = *reinterpret_cast<const float4*>(&sT2[((2 + s) * 64 + lane) * 4]);
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          // mirror quadruple of j0 = 4g + s: registers (e, r) = (s,0), (3-s,1), (s,2), (3-s,3)
          const Bfly b = butterfly(C1[s][tt][0], C1[3 - s][tt][1], C1[s][tt][2], C1[3 - s][tt][3]);
          C2[0][tt] = mfma4(pee[s], b.ee, C2[0][tt]);
          C2[1][tt] = mfma4(peo[s], b.eo, C2[1][tt]);
          C2[2][tt] = mfma4(po4.x, b.o0, C2[2][tt]);
          C2[3][tt] = mfma4(po4.y, b.o0, C2[3][tt]);
          C2[2][tt] = mfma4(po4.z, b.o1, C2[2][tt]);
          C2[3][tt] = mfma4(po4.w, b.o1, C2[3][tt]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    // lands while top-k, reconstruction and store of this chunk run (after the last chunk the same
    // chunk is simply requested again: an unconditional fetch keeps the old registers dead).  The full-product
    // instances are bound by their MFMAs and short of registers: they request the rows behind the reconstruction
    if (!DENSE) fetch_m(nxt);
    __builtin_amdgcn_sched_barrier(0);

    DEMO_PHASE(2);
    if constexpr (STAGE == 2) {
#pragma unroll
      for (int vt = 0; vt < 4; ++vt)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) asm volatile("" ::"v"(C2[vt][tt]));
      if (GBF16) fetch_g(nxt);
      if (lane < k) {
        const int64_t po = (int64_t)cc * k + lane;
        store_guarded(as_global(cur.idx) + po, (int32_t)lane);
        store_guarded(as_global(cur.val) + po, C2[0][0][0]);
      }
    } else {
    // ---- top-k inside the wavefront ------------------------------------------------------------
    // (1) a lower bound of the k-th largest magnitude: the k-th largest of the 64 per-lane maxima,
    //     resolved to its upper 16 bits.  For k > 32 the bound comes from 128 maxima instead, two per lane (of the
    //     lane's first and second 32 coefficients): among 64 maxima the k-th largest sinks towards the smallest
    //     one as k approaches 64, the candidate list (about 44 entries at k = 32) then overflows for every chunk,
    //     and every chunk would go to the exact kernel.  With 128 maxima k = 64 gives about 90 candidates.
    float lmax0 = 0.f, lmax1 = 0.f;
#pragma unroll
    for (int vt = 0; vt < 2; ++vt)
#pragma unroll
      for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          lmax0 = fmaxf(lmax0, fabsf(C2[vt][tt][r]));
          lmax1 = fmaxf(lmax1, fabsf(C2[vt + 2][tt][r]));
        }
    const uint32_t lm0 = __float_as_uint(lmax0), lm1 = __float_as_uint(lmax1);
    const uint32_t lm = max(lm0, lm1);
    uint32_t thr = 0;
    if (k <= 32) {
      for (int bit = 30; bit >= 16; --bit) {
        const uint32_t cnd = thr | (1u << bit);
        if (__popcll(__ballot(lm >= cnd)) >= k) thr = cnd;
      }
    } else {
      for (int bit = 30; bit >= 16; --bit) {
        const uint32_t cnd = thr | (1u << bit);
        if (__popcll(__ballot(lm0 >= cnd)) + __popcll(__ballot(lm1 >= cnd)) >= k) thr = cnd;
      }
    }
    DEMO_PHASE(3);
    // (2) gather candidates |q| >= thr: one compare and one scalar branch per coefficient.  The LDS byte address of
    //     the list's end is kept as a scalar, so a lane's slot costs its count of hits below plus one shift-add
    int ncand = 0;
    uint32_t list_end = list_base;
    // (keeps the 64 per-register flat indices from being precomputed outside the chunk loop)
    asm volatile("" : "+v"(fb_a), "+v"(fb_b), "+v"(fb_c), "+v"(fb_d));
    {
      const float thr_f = __uint_as_float(thr);
#pragma unroll
      for (int vt = 0; vt < 4; ++vt)
#pragma unroll
        for (int tt = 0; tt < 4; ++tt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float q = C2[vt][tt][r];
            const bool is = fabsf(q) >= thr_f;
            const uint64_t mask = __ballot(is);
            if (mask != 0) {
              if (is && ncand <= E64_CAP) {   // a full list takes no more: slot < CAP + 64 without a per-lane clamp
                lds_u32* slot = lds_u32_at(list_end + 4u * (uint32_t)lanes_below(mask));
                const uint32_t fbase = DENSE ? fb_a : tt < 2 ? (vt < 2 ? fb_a : fb_b) : (vt < 2 ? fb_c : fb_d);
                const uint32_t fconst = DENSE ? (uint32_t)(1024 * tt + 16 * vt + r) : (uint32_t)(64 * freq(tt, 0) + freq(vt, r));
                slot[0] = __float_as_uint(q);
                slot[E64_LIST] = fbase + fconst;
              }
              const int hits = __popcll(mask);
              ncand += hits;
              list_end += 4u * (uint32_t)hits;
            }
          }
    }
    const bool overflow = ncand > E64_CAP;   // many (near-)equal magnitudes at the threshold
    const bool all_zero = overflow && __ballot(lm != 0u) == 0;
    skip = overflow && !all_zero;
    if (skip) {
      // leave the chunk untouched and queue it for the exact workgroup kernel that runs next
      if (lane == 0) store_guarded(&wl.list[atomicAdd(wl.count, 1)], chunk);
    }
    if (all_zero) {
      // every coefficient is zero: the k lowest flat indices with zero values; D (all zero) is stored below
      if (lane < k) {
        const int64_t po = (int64_t)cc * k + lane;
        store_guarded(as_global(cur.idx) + po, (int32_t)lane);
        store_guarded(as_global(cur.val) + po, 0.f);
      }
      ncand = 0;
    }
    DEMO_PHASE(4);
    wave_lds_sync();
    // (3) rank candidates (magnitude descending, flat index ascending); ranks < k are the payload.  The selected
    //     coefficients are also listed by the class of their row frequency u (0: u = 0 mod 4, 1: u = 2 mod 4,
    //     2: u odd) for the reconstruction; ncls[] counts them (uniform).
    int ncls[3] = {0, 0, 0};
    auto file_selected = [&](bool selected, uint32_t flat, uint32_t vbits) {
      const uint32_t u = flat >> 6;
      const int cls = DENSE ? 0 : (u & 1u) ? 2 : (int)((u >> 1) & 1u);   // DENSE: one list (at most 64 long, as k <= 64)
#pragma unroll
      for (int q = 0; q < 3; ++q) {
        const uint64_t m = __ballot(selected && cls == q);
        if (selected && cls == q) sel[q * 64 + ncls[q] + lanes_below(m)] = make_uint2(flat, vbits);
        ncls[q] += __popcll(m);
      }
    };
    if (all_zero || skip) {
    } else if (ncand <= 64) {
      // one candidate per lane, ordered by the 64-bit key {magnitude, ~flat index}.  The lanes put their keys into
      // LDS and every lane reads all of them back, two per 16-byte read at a wavefront-uniform address (lanes past
      // the list carry key 0, which precedes nothing)
      const uint32_t me_v = cand_v[lane < ncand ? lane : 0], me_f = cand_f[lane < ncand ? lane : 0];
      const uint32_t mag = lane < ncand ? (me_v & 0x7fffffffu) : 0u, nfl = lane < ncand ? ~me_f : 0u;
      const uint64_t key = ((uint64_t)mag << 32) | nfl;
      keys[lane] = make_uint2(nfl, mag);
      wave_lds_sync();
      int rank = 0;
      // sixteen keys per turn, all eight reads issued before the first comparison: one LDS round trip per turn
      // (all 64 keys exist: lanes past the list wrote zeros)
      for (int j = 0; j < ncand; j += 16) {
        uint4 kk[8];
#pragma unroll
        for (int x = 0; x < 8; ++x) kk[x] = *reinterpret_cast<const uint4*>(&keys[j + 2 * x]);
#pragma unroll
        for (int x = 0; x < 8; ++x)
          rank += ((((uint64_t)kk[x].y << 32) | kk[x].x) > key ? 1 : 0) + ((((uint64_t)kk[x].w << 32) | kk[x].z) > key ? 1 : 0);
      }
      const bool selected = lane < ncand && rank < k;
      if (selected) {
        const int64_t po = (int64_t)cc * k + rank;
        store_guarded(as_global(cur.idx) + po, (int32_t)me_f);
        store_guarded(as_global(cur.val) + po, __uint_as_float(me_v));
      }
      file_selected(selected, me_f, me_v);
    } else {
      // more candidates than lanes (k > 32, or many magnitudes near the bound): the list is padded to a multiple of
      // eight with entries that precede nothing, and every lane ranks its candidate of each block of 64 against
      // the whole list, eight entries per turn with all reads issued before the first comparison
      if (lane < ((8 - (ncand & 7)) & 7)) {
        cand_v[ncand + lane] = 0u;
        cand_f[ncand + lane] = 0xffffffffu;
      }
      wave_lds_sync();
      for (int base = 0; base < ncand; base += 64) {   // uniform trip count: the ballots below need every lane
        const int i = base + lane;
        const bool valid = i < ncand;
        const uint32_t me_v = cand_v[valid ? i : 0], me_f = cand_f[valid ? i : 0];
        const uint32_t mag = me_v & 0x7fffffffu;
        int rank = 0;
        for (int j = 0; j < ncand; j += 8) {
          uint2 ov[4], of[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            ov[x] = *reinterpret_cast<const uint2*>(&cand_v[j + 2 * x]);
            of[x] = *reinterpret_cast<const uint2*>(&cand_f[j + 2 * x]);
          }
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            const uint32_t m0 = ov[x].x & 0x7fffffffu, m1 = ov[x].y & 0x7fffffffu;
            rank += (m0 > mag || (m0 == mag && of[x].x < me_f)) ? 1 : 0;
            rank += (m1 > mag || (m1 == mag && of[x].y < me_f)) ? 1 : 0;
          }
        }
        const bool selected = valid && rank < k;
        if (selected) {
          const int64_t po = (int64_t)cc * k + rank;
          store_guarded(as_global(cur.idx) + po, (int32_t)me_f);
          store_guarded(as_global(cur.val) + po, __uint_as_float(me_v));
        }
        file_selected(selected, me_f, me_v);
      }
    }
    // each class list is padded with zero-valued entries to a multiple of four (one MFMA step holds four)
#pragma unroll
    for (int q = 0; q < 3; ++q)
      if (lane < ((4 - (ncls[q] & 3)) & 3)) sel[q * 64 + ncls[q] + lane] = make_uint2(0u, 0u);
    wave_lds_sync();
    if (GBF16 && !DENSE) fetch_g(nxt);   // the coefficient registers are dead now (fp32 gradients: twice the registers, see below)
    __builtin_amdgcn_sched_barrier(0);

    DEMO_PHASE(5);
    // ---- reconstruction  D -= alpha * sum_t val_t P[u_t][i] P[v_t][j]  on the quadruple bases only: by the
    //      mirror symmetries of the rows of P (see demo_dec64.hip) the four rows {i0, 31-i0, 32+i0, 63-i0} of a
    //      term differ by signs fixed by the class of u_t, so each class accumulates one 16-row tile per column
    //      tile (two for odd u: i0 and 31-i0) instead of four, and the members follow from in-lane adds:
    //        D[i0] += ee+eo+o0, D[31-i0] += ee-eo+o1, D[32+i0] += ee-eo-o1, D[63-i0] += ee+eo-o0.
    //      MFMA row m = 4g + r of a compact tile is the base i0 = kappa(m) = 4r + g, i.e. component s = r of D.
    //      The classes are done one after the other so that at most two compact accumulators are alive.
    if constexpr (DENSE) {
      if (!skip && STAGE == 0) {
        // D[r][e][w] -= alpha sum_t val_t P[u_t][rho(4r + w, g)] P[v_t][4 chi(c) + e]: MFMA row m = 4g + r of the
        // tile of member w is row rho(4r + w, g); one member per pass over the list keeps the accumulators at 16 registers
        // A step's operands hang on two LDS reads in a row (the list entry, then the two basis rows it names): the
        // loop runs two steps per turn on alternating registers, the entry fetched two steps and the rows one step
        // ahead, with scheduling fences around the MFMAs (without them the compiler sinks every read to its use and a
        // step of four MFMAs waits out two LDS round trips)
        const int n = __builtin_amdgcn_readfirstlane((ncls[0] + 3) >> 2);
        const int lane_now = fresh_lane_id();
        const int gl = lane_now >> 4, cl = lane_now & 15;
        struct Rows {
          float val, pr;
          float4 pb;
        };
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          f32x4 Ra[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) Ra[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
          if (n > 0) {
            auto entry = [&](int step) { return sel[4 * min(step, n - 1) + gl]; };
            auto rows_of = [&](const uint2& sv) {
              return Rows{__uint_as_float(sv.y), sProw[((sv.x >> 6) & 63u) * 64 + cl + 16 * w],
                          *reinterpret_cast<const float4*>(&sPcol[(sv.x & 63u) * 64 + 4 * cl])};
            };
            auto accumulate = [&](const Rows& r) {
              const float a0 = -(args.alpha * r.val) * r.pr;
              Ra[0] = mfma4(a0, r.pb.x, Ra[0]);
              Ra[1] = mfma4(a0, r.pb.y, Ra[1]);
              Ra[2] = mfma4(a0, r.pb.z, Ra[2]);
              Ra[3] = mfma4(a0, r.pb.w, Ra[3]);
            };
            uint2 sv = entry(0);
            Rows ra = rows_of(sv), rb;
            sv = entry(1);
            for (int ks = 0; ks < n; ks += 2) {
              rb = rows_of(sv);       // step ks + 1 (past the end: the last step again, unused)
              sv = entry(ks + 2);
              __builtin_amdgcn_sched_barrier(0);
              accumulate(ra);
              __builtin_amdgcn_sched_barrier(0);
              if (ks + 1 < n) {       // uniform
                ra = rows_of(sv);     // step ks + 2
                sv = entry(ks + 3);
                __builtin_amdgcn_sched_barrier(0);
                accumulate(rb);
                __builtin_amdgcn_sched_barrier(0);
              }
            }
          }
#pragma unroll
          for (int sq = 0; sq < 4; ++sq)
#pragma unroll
            for (int e = 0; e < 4; ++e) D[sq][e][w] += Ra[e][sq];
        }
      }
    } else if (!skip && STAGE == 0) {
      {
        f32x4 Ree[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) Ree[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
        for (int ks = 0; ks < (ncls[0] + 3) / 4; ++ks) {
          const uint2 sv = sel[0 * 64 + 4 * ks + g];
          const float nv = -(args.alpha * __uint_as_float(sv.y));
          const float a = nv * sPk[((sv.x >> 6) & 63u) * 16 + c];
          const float4 pb = *reinterpret_cast<const float4*>(&sPcol[(sv.x & 63u) * 64 + 4 * c]);
          const float bf[4] = {pb.x, pb.y, pb.z, pb.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) Ree[e] = mfma4(a, bf[e], Ree[e]);
        }
#pragma unroll
        for (int sq = 0; sq < 4; ++sq)
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int w = 0; w < 4; ++w) D[sq][e][w] += Ree[e][sq];
      }
      {
        f32x4 Reo[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) Reo[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
        for (int ks = 0; ks < (ncls[1] + 3) / 4; ++ks) {
          const uint2 sv = sel[1 * 64 + 4 * ks + g];
          const float nv = -(args.alpha * __uint_as_float(sv.y));
          const float a = nv * sPk[((sv.x >> 6) & 63u) * 16 + c];
          const float4 pb = *reinterpret_cast<const float4*>(&sPcol[(sv.x & 63u) * 64 + 4 * c]);
          const float bf[4] = {pb.x, pb.y, pb.z, pb.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) Reo[e] = mfma4(a, bf[e], Reo[e]);
        }
#pragma unroll
        for (int sq = 0; sq < 4; ++sq)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            D[sq][e][0] += Reo[e][sq];
            D[sq][e][1] -= Reo[e][sq];
            D[sq][e][2] -= Reo[e][sq];
            D[sq][e][3] += Reo[e][sq];
          }
      }
      {
        f32x4 Ro0[4], Ro1[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          Ro0[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
          Ro1[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
        for (int ks = 0; ks < (ncls[2] + 3) / 4; ++ks) {
          const uint2 sv = sel[2 * 64 + 4 * ks + g];
          const float nv = -(args.alpha * __uint_as_float(sv.y));
          const uint32_t ur = ((sv.x >> 6) & 63u) * 16 + c;
          const float a0 = nv * sPk[ur], a1 = nv * sPk2[ur];
          const float4 pb = *reinterpret_cast<const float4*>(&sPcol[(sv.x & 63u) * 64 + 4 * c]);
          const float bf[4] = {pb.x, pb.y, pb.z, pb.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            Ro0[e] = mfma4(a0, bf[e], Ro0[e]);
            Ro1[e] = mfma4(a1, bf[e], Ro1[e]);
          }
        }
#pragma unroll
        for (int sq = 0; sq < 4; ++sq)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            D[sq][e][0] += Ro0[e][sq];
            D[sq][e][1] += Ro1[e][sq];
            D[sq][e][2] -= Ro1[e][sq];
            D[sq][e][3] -= Ro0[e][sq];
          }
      }
    }

    }   // STAGE != 2
    }   // STAGE != 1
    if (DENSE) fetch_m(nxt);
    if (GBF16 ? DENSE : !DENSE) fetch_g(nxt);   // 64 registers: requested once the compact accumulators are dead
    DEMO_PHASE(6);
    // ---- store the residual momentum: always issued, so that the number of stores behind the prefetched rows
    //      is fixed; a chunk left to the exact kernel stores through a buffer of zero records, which drops them
    {
      const __amdgpu_buffer_rsrc_t sres = skip ? make_rsrc_empty(nullptr) : mres;
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const f32x4 o = {D[q >> 2][0][q & 3], D[q >> 2][1][q & 3], D[q >> 2][2][q & 3], D[q >> 2][3][q & 3]};
        bstore_f4(sres, ((q & 1) ? vo_dn : vo_up) * 4, (uint32_t)rbase(q) * ucols * 4, o);
      }
    }
    if (DENSE && !GBF16) fetch_g(nxt);   // float32 gradients of the full-product instances: no registers before the stores
    wave_lds_sync();   // the lists are rewritten by the next chunk
    DEMO_PHASE(7);
    if (!has_next) break;
    chunk += nwaves;
    if (unit_grad_scale) momentum(std::true_type{}); else momentum(std::false_type{});
    cur = nxt;
  }
  DEMO_PHASE_FLUSH(0);
}

template <bool GBF16, int STAGE, bool DENSE = false>
static hipError_t launch_enc_wave64(const TableView& tv, const float* tables, const EncodeArgs& a, const Worklist& wl,
                                    int64_t grid, hipStream_t stream) {
  static bool attr_set = false;
  constexpr int lds_bytes = e64_lds_bytes<DENSE>();
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&encode2d_wave64<GBF16, STAGE, DENSE>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((encode2d_wave64<GBF16, STAGE, DENSE>), dim3((unsigned)grid), dim3(E64_THREADS), lds_bytes, stream, tv,
                     tables, a, wl);
  return hipGetLastError();
}

hipError_t launch_encode2d_wave64(const TableView& tv, const float* tables, const EncodeArgs& a, const Worklist& wl,
                                  bool grad_bf16, bool dense, int num_cus, hipStream_t stream) {
  int64_t grid = num_cus;
  const int64_t max_grid = ((int64_t)tv.total_chunks + DEMO_RUN - 1) / DEMO_RUN;   // few items: one run per workgroup, spread over the CUs
  if (grid > max_grid) grid = max_grid;
  if (dense) {   // `tables` are those of build_enc64_dense_tables
    if (a.stage != 0) return hipErrorInvalidValue;
    return grad_bf16 ? launch_enc_wave64<true, 0, true>(tv, tables, a, wl, grid, stream)
                     : launch_enc_wave64<false, 0, true>(tv, tables, a, wl, grid, stream);
  }
  if (a.stage != 0) {   // time attribution only (bfloat16 gradients)
    if (!grad_bf16) return hipErrorInvalidValue;
    switch (a.stage) {
      case 1: return launch_enc_wave64<true, 1>(tv, tables, a, wl, grid, stream);
      case 2: return launch_enc_wave64<true, 2>(tv, tables, a, wl, grid, stream);
      case 3: return launch_enc_wave64<true, 3>(tv, tables, a, wl, grid, stream);
      default: return hipErrorInvalidValue;
    }
  }
  return grad_bf16 ? launch_enc_wave64<true, 0>(tv, tables, a, wl, grid, stream)
                   : launch_enc_wave64<false, 0>(tv, tables, a, wl, grid, stream);
}

}  // namespace demo

DEMO_PHASE_GETTER(demo_debug_phase_clocks_enc)
