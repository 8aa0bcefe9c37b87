// s = 32 decode kernel: one wavefront per 64 x 64 tile = 2 x 2 chunks.
//
// The tile is transformed with the block-diagonal matrix diag(P32, P32), so chunk (a, b) of the tile is
// R_ab = P32^T S_ab P32 and the four chunks never mix.  The structure is that of the s = 64 kernel
// (demo_dec64.hip) with the mirror symmetry of the 32-point DCT in place of the two nested ones of the
// 64-point DCT: even rows of P32 are even under i -> 31-i, odd rows odd, so for the quadruple
// {i0, 31-i0, 32+i0, 63-i0} (i0 < 16: one mirror pair in each block) four partial sums
//   E_a = sum over even u of block a,  O_a = sum over odd u of block a      (16 frequencies each)
// give  out[i0] = E_0+O_0, out[31-i0] = E_0-O_0, out[32+i0] = E_1+O_1, out[63-i0] = E_1-O_1.
// Both products therefore cost 64 MFMAs per tile (a quarter of the dense 64 x 64 products), the tile of
// coefficient sums is stored with rows and columns grouped by class (block, parity), lane l = 16 g + c ends
// up with rows member(w, 4s + g) and columns member(w', kappa(c)), and R goes once through the LDS tile
// into the row layout in which the parameters are read and written (see demo_dec64.hip).
//
// Payload: the W*k <= 512 pairs of each of the four chunks sit in 8 registers per lane and chunk (pair
// p = 64 j + lane of the chunk belongs to worker p / k, position p % k) and are fetched for the next tile
// while the products of this one run.  Each chunk has its own fixed-point scale.
#include "demo_device.h"

namespace demo {

namespace {
constexpr int D32_WAVES = 8;
constexpr int D32_THREADS = D32_WAVES * 64;
constexpr int D32_LDT = 68;                        // tile row stride (floats); columns 64..67 are pad slots
constexpr int D32_TILE_FLOATS = 64 * D32_LDT;
constexpr int D32_G_FLOATS = 512;                  // fragment table: 2 parities x 64 lanes x 4
constexpr int D32_LDS_BYTES = 4 * (D32_G_FLOATS + D32_WAVES * D32_TILE_FLOATS);
constexpr int D32_SLOTS = 8;                       // payload registers per lane and chunk
static_assert(D32_G_FLOATS == kDec32TableFloats, "table size");
static_assert(D32_LDS_BYTES <= 160 * 1024, "LDS budget");
static_assert(kFast32MaxPairs == 64 * D32_SLOTS, "pairs per chunk held in registers (per round when streaming)");

__host__ __device__ constexpr int kappa32(int c) { return 4 * (c & 3) + (c >> 2); }
}  // namespace

// Host: fragment table from the 32 x 32 basis P32 (double, row-major).  Lane (g, c), component r of
// group p holds P32[2 (4g + r) + p][kappa(c)]: the contraction index of k-slot g at step r is the
// (4g + r)-th frequency of parity p, the other index the quadruple base kappa(c).
void build_dec32_tables(const double* P32, float* out) {
  for (int p = 0; p < 2; ++p)
    for (int lane = 0; lane < 64; ++lane) {
      const int g = lane >> 4, c = lane & 15;
      for (int r = 0; r < 4; ++r) out[(p * 64 + lane) * 4 + r] = (float)P32[(2 * (4 * g + r) + p) * 32 + kappa32(c)];
    }
}

// The table `tv` lists the order-2 tensors in units of 64 x 64 tiles (cchunks = cols / 64, nchunks =
// tiles); payload arrays are addressed per 32 x 32 chunk (4 * nchunks chunks per tensor).
// MODE 1, 2 (VEC4): k is a multiple of four and every payload pointer is 16-byte aligned; a lane then fetches four
// consecutive pairs of one worker with one 16-byte load per array (slot 8 q + 4 jj + e holds pair 4 (64 jj + lane) + e
// of chunk q).  MODE 2 (STREAM): more than 512 pairs per chunk (up to 65536), streamed once in rounds of 512 per
// chunk, a chunk's sums being shifted down whenever a round raises its block exponent.  MODE 0: one pair per load.
// IDENT: phi is the identity on the aggregate instead of sgn (its own instance, so that the sign kernels carry
// nothing for it).  COUNT: the count-normalised aggregate of the appendix algorithm "Sparse Top-k Averaging" (every
// coefficient's sum divided by the number of pairs that name it), modes 0 and 1 only.  NT: the 16-byte payload loads
// are non-temporal (asked for when a row of k pairs fills a 128-byte line; shorter rows share lines with the
// neighbouring chunks and stay cached).
template <bool PBF16, int MODE, bool IDENT, bool COUNT = false, bool NT = true>
__global__ __launch_bounds__(D32_THREADS) void decode2d_tile32(TableView tv, const float* __restrict__ tables,
                                                               DecodeArgs args) {
  constexpr bool VEC4 = MODE >= 1, STREAM = MODE == 2;
  extern __shared__ float lds[];
  const float* sG = lds;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, c = lane & 15;
  float* tile = lds + D32_G_FLOATS + wave * D32_TILE_FLOATS;
  int* itile = reinterpret_cast<int*>(tile);
  const int k = args.k, W = args.W;
  const int npairs = W * k;                                   // per chunk (<= 512 unless STREAM)
  const int nunits = VEC4 ? (npairs >> 2) : npairs;           // loads per array and chunk
  const int nloads = STREAM ? D32_SLOTS / 4 : (nunits + 63) >> 6;   // ... per lane (uniform; STREAM: per round)
  const int nslots = VEC4 ? 4 * nloads : nloads;              // payload registers in use per chunk (uniform)
  const int nrounds = (nunits + 16 * D32_SLOTS - 1) / (16 * D32_SLOTS);   // STREAM: rounds of 64 * SLOTS / 4 units

  for (int e = tid; e < D32_G_FLOATS / 4; e += D32_THREADS)
    reinterpret_cast<float4*>(lds)[e] = reinterpret_cast<const float4*>(tables)[e];
  __syncthreads();

  const int nwaves = gridDim.x * D32_WAVES;
  const int total = tv.total_chunks;
  int tileno = first_work_item<DEMO_RUN>(wave);                         // then tiles + nwaves, ...
  if (tileno >= total) return;

  // ---- payload: slot 8 q + j holds pair 64 j + lane of chunk q = 2 bu + bv of the tile -------------------
  int32_t pi[4 * D32_SLOTS];
  float pv[4 * D32_SLOTS];
#pragma unroll
  for (int j = 0; j < 4 * D32_SLOTS; ++j) {
    pi[j] = -1;
    pv[j] = 0.f;
  }
  const float rk = 1.0f / (float)k;
  // `round` matters in STREAM mode only: units 128 round + 64 jj + lane
  auto load_payload = [&](const TensorDev& dd, int tt, int round = 0) {
    const int K0 = tt / dd.cchunks, K1 = tt - K0 * dd.cchunks;
    const int cch32 = 2 * dd.cchunks;
    const int64_t wstride = (int64_t)dd.nchunks * 4 * k;      // pairs of one worker for this tensor
    // the per-slot (worker, position) are formed anew at every call: kept across the tile loop as 64-bit offsets
    // they are spilled, and every reload of a spilled value waits for all loads in flight
    int lanev = lane;
    asm volatile("" : "+v"(lanev));
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c32 = (2 * K0 + (q >> 1)) * cch32 + 2 * K1 + (q & 1);
      const DEMO_GLOBAL int32_t* ip = as_global(dd.idx) + (int64_t)c32 * k;
      const DEMO_GLOBAL float* vp = as_global(dd.val) + (int64_t)c32 * k;
      if constexpr (VEC4) {
        {
#pragma unroll
          for (int jj = 0; jj < D32_SLOTS / 4; ++jj) {
            if (jj < nloads) {                                  // uniform
              const int unit = (STREAM ? 16 * D32_SLOTS * round : 0) + 64 * jj + lanev;
              const int p = 4 * unit;
              const int w = (int)(((float)p + 0.5f) * rk);      // as below (p < 65536)
              const int pos = p - w * k;
              const bool ok = unit < nunits;
              const uint32_t off = ok ? (uint32_t)(w * (int)wstride + pos) : 0u;
              // unconditional, and taken as it comes: mask_payload discards the units past the end where the pairs
              // are consumed (a select right behind a load makes the wavefront wait for it before the next load)
              const f32x4 vv = payload_load<NT>(reinterpret_cast<const DEMO_GLOBAL f32x4*>(vp + off));
#pragma unroll
              for (int e = 0; e < 4; ++e) pv[D32_SLOTS * q + 4 * jj + e] = vv[e];
              const u32x4 iv = payload_load<NT>(reinterpret_cast<const DEMO_GLOBAL u32x4*>(ip + off));
#pragma unroll
              for (int e = 0; e < 4; ++e) pi[D32_SLOTS * q + 4 * jj + e] = (int32_t)iv[e];
            }
          }
        }
        continue;
      }
#pragma unroll
      for (int j = 0; j < D32_SLOTS; ++j) {
        if (j < nslots) {                                     // uniform
          const int p = 64 * j + lanev;
          // worker p / k and position p % k; (p + 1/2) / k is never within 1/(2k) of an integer, far
          // more than the rounding error of the float product for p < 512
          const int w = (int)(((float)p + 0.5f) * rk);
          const int pos = p - w * k;
          const bool ok = p < npairs;
          const uint32_t off = ok ? (uint32_t)(w * (int)wstride + pos) : 0u;
          pi[D32_SLOTS * q + j] = ip[off];
          pv[D32_SLOTS * q + j] = vp[off];
        }
      }
    }
  };
  // Slots past the end of a chunk's payload become (no index, 0); called where the pairs are consumed.
  auto mask_payload = [&](int round = 0) {
    int lanev = lane;
    asm volatile("" : "+v"(lanev));
#pragma unroll
    for (int j = 0; j < D32_SLOTS; ++j) {
      if (j < nslots) {   // uniform
        const bool ok = VEC4 ? (STREAM ? 16 * D32_SLOTS * round : 0) + 64 * (j >> 2) + lanev < nunits : 64 * j + lanev < npairs;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          pi[D32_SLOTS * q + j] = ok ? pi[D32_SLOTS * q + j] : -1;
          pv[D32_SLOTS * q + j] = ok ? pv[D32_SLOTS * q + j] : 0.f;
        }
      }
    }
  };

  // S[idx] += val in block fixed point with integer LDS atomics, one scale per chunk (see demo_dec64.hip).
  // Coefficient (u, v) of chunk (a, b) lives at tile row 32 a + 16 (u % 2) + u / 2, column
  // 32 b + 16 (v % 2) + v / 2.  Lanes with nothing to add put a zero-weight value into their pad slot.
  const uint32_t dummy = (uint32_t)(lane * D32_LDT + 64);
  int vbits = 30;
  for (int w = 1; w < W; w <<= 1) --vbits;                    // 30 - ceil(log2 W)
  auto lane_max = [&](int q, float mx) {
#pragma unroll
    for (int j = 0; j < D32_SLOTS; ++j)
      if (j < nslots) mx = fmaxf(mx, fabsf(pv[D32_SLOTS * q + j]));
    return mx;
  };
  // shift of a chunk's block fixed point from the lanes' largest magnitudes
  auto shift_of = [&](float mx) {
      uint32_t mb = __float_as_uint(mx);
      mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
      mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
      mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x141, 0xf, 0xf, false));  // row_half_mirror
      mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x140, 0xf, 0xf, false));  // row_mirror
      const uint32_t m01 = max((uint32_t)__builtin_amdgcn_readlane((int)mb, 0), (uint32_t)__builtin_amdgcn_readlane((int)mb, 16));
      const uint32_t m23 = max((uint32_t)__builtin_amdgcn_readlane((int)mb, 32), (uint32_t)__builtin_amdgcn_readlane((int)mb, 48));
      int ex = (int)(max(m01, m23) >> 23);                    // biased exponent of the chunk's largest magnitude
      ex = ex < 1 ? 1 : ex;
      return vbits + 126 - ex;                                // max |val| * 2^sh < 2^vbits
  };
  auto slot_of = [&](int q, int j) {
      const uint32_t quad = (uint32_t)(((q >> 1) << 11) | ((q & 1) << 5));
      const uint32_t u = (uint32_t)pi[D32_SLOTS * q + j];
      // 10-bit index [u4..u0 v4..v0] -> 12-bit [a u0 u4..u1 | b v0 v4..v1], then row stride 64 -> LDT
      const uint32_t x = quad | (u & 0x3C0u) | ((u & 0x20u) << 5) | ((u & 1u) << 4) | ((u >> 1) & 0xFu);
      return u < 1024u ? x + ((x >> 6) << 2) : dummy;
  };
  auto add_pairs = [&](int q, int sh) {
#pragma unroll
      for (int j = 0; j < D32_SLOTS; ++j)
        if (j < nslots) atomicAdd(&itile[slot_of(q, j)], __float2int_rn(ldexpf(pv[D32_SLOTS * q + j], sh)));
  };
  int sh[4];   // shifts of the four chunks' fixed points (undone when phi is the identity)
  auto scatter = [&]() {
    if constexpr (COUNT) {
      static_assert(!COUNT || !STREAM, "the count pass needs the whole payload in registers");
      // every pair adds one to its coefficient's slot, reads the total back and is divided by it; the slots are
      // cleared again before the sums go in.  Sum of val/n over the n pairs of a slot = (sum of val) / n.
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int j = 0; j < D32_SLOTS; ++j)
          if (j < nslots) atomicAdd(&itile[slot_of(q, j)], 1);
      wave_lds_sync();
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int j = 0; j < D32_SLOTS; ++j)
          if (j < nslots) pv[D32_SLOTS * q + j] = pv[D32_SLOTS * q + j] / (float)itile[slot_of(q, j)];
      wave_lds_sync();
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int j = 0; j < D32_SLOTS; ++j)
          if (j < nslots) itile[slot_of(q, j)] = 0;
      wave_lds_sync();
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      sh[q] = shift_of(lane_max(q, 0.f));
      add_pairs(q, sh[q]);
    }
  };

  int t = find_tensor_uniform(tv, tileno);
  int t_first = uniform_prefix(tv, t), t_next = uniform_prefix(tv, t + 1);
  TensorDev d = load_desc_uniform(tv, t);
  load_payload(d, tileno - t_first, 0);
  // the first tile's pairs are waited for here, outside the loop (see demo_dec64.hip: with loads pending at the
  // loop's entry its first wait would also be for the acknowledgements of the previous tile's stores)
#pragma unroll
  for (int j = 0; j < 4 * D32_SLOTS; ++j) asm volatile("" : "+v"(pi[j]), "+v"(pv[j]));
  const int kap = kappa32(c), col4 = 4 * chi(c);
  // tile offsets (floats) of the transposition of R: row parts for members w even / odd, column parts
  // for members w' even / odd (w' >= 2 adds 32 columns)
  const int row_up = 4 * g * D32_LDT, row_dn = 4 * (3 - g) * D32_LDT;
  const int wr_col_up = kap, wr_col_dn = 31 - kap;

  for (; tileno < total; tileno += nwaves) {
    const int tt = tileno - t_first;
    const int k0 = tt / d.cchunks, k1 = tt - k0 * d.cchunks;
    const int64_t origin = (int64_t)k0 * 64 * d.cols + (int64_t)k1 * 64;   // uniform
    const uint32_t ucols = (uint32_t)d.cols;
    // parameters: lane (g, c) reads / writes rows rho(q, g), columns 4 chi(c) .. +3 (whole rows per instruction)
    const uint32_t vo_up = (uint32_t)g * ucols + (uint32_t)col4;           // elements
    const uint32_t vo_dn = (uint32_t)(3 - g) * ucols + (uint32_t)col4;
    const __amdgpu_buffer_rsrc_t xres = PBF16 ? make_rsrc(static_cast<const uint16_t*>(d.param) + origin)
                                              : make_rsrc(static_cast<const float*>(d.param) + origin);
    // bf16 parameters, raw: requested before the scatter (with 16-byte payload loads; the 4-byte path has too many
    // addresses live for that and requests them after the payload of the next tile), used after the products
    u32x2 Xh[16];
    auto request_x = [&]() {
#pragma unroll
      for (int q = 0; q < 16; ++q) Xh[q] = bload_u2(xres, ((q & 1) ? vo_dn : vo_up) * 2, (uint32_t)rho_base(q) * ucols * 2);
    };
    if (PBF16 && VEC4) request_x();
    mask_payload(0);

    // ---- S = sum over workers, four chunks ----------------------------------------------------------------
#pragma unroll
    for (int i = 0; i < 17; ++i) *reinterpret_cast<float4*>(&tile[(i * 64 + lane) * 4]) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_sync();
    if constexpr (STREAM) {
      // one pass: the registers hold round 0; every round is added with the block exponents of the largest
      // magnitudes seen so far, and when a round raises a chunk's exponent that chunk's sums are first shifted
      // down to the new scale (round to nearest, ties to even; every later shift at least halves the error of an earlier one,
      // so the shifts together cost at most one unit of the final scale per coefficient)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        sh[q] = shift_of(lane_max(q, 0.f));
        add_pairs(q, sh[q]);
      }
      for (int r = 1; r < nrounds; ++r) {
        load_payload(d, tt, r);
        mask_payload(r);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int sh_r = shift_of(lane_max(q, 0.f));
          if (sh_r < sh[q]) {   // uniform
            const int dsh = min(sh[q] - sh_r, 31);
            const int half = (1 << (dsh - 1)) - 1;   // + the kept part's lowest bit: ties go to even (a bias would add up over the slots)
            wave_lds_sync();
            // quadrant q of the tile: rows 32 (q / 2) .. +31, columns 32 (q % 2) .. +31
            int* quad = itile + (32 * (q >> 1) + (lane >> 3)) * D32_LDT + 32 * (q & 1) + 4 * (lane & 7);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              int4 v = *reinterpret_cast<int4*>(quad + 8 * i * D32_LDT);
              v.x = (v.x + half + ((v.x >> dsh) & 1)) >> dsh;
              v.y = (v.y + half + ((v.y >> dsh) & 1)) >> dsh;
              v.z = (v.z + half + ((v.z >> dsh) & 1)) >> dsh;
              v.w = (v.w + half + ((v.w >> dsh) & 1)) >> dsh;
              *reinterpret_cast<int4*>(quad + 8 * i * D32_LDT) = v;
            }
            wave_lds_sync();
            sh[q] = sh_r;
          }
          add_pairs(q, sh[q]);
        }
      }
    } else {
      scatter();
    }
    // ---- payload of the next tile, in flight during the products (after the last tile the same tile is
    //      requested again: an unconditional fetch keeps the old registers dead) -----------------------------
    if (tileno + nwaves < total) {
      while (tileno + nwaves >= t_next) {
        ++t;
        t_first = t_next;
        t_next = uniform_prefix(tv, t + 1);
        d = load_desc_uniform(tv, t);
      }
      load_payload(d, tileno + nwaves - t_first, 0);
    } else {
      load_payload(d, tt, 0);
    }
    if (PBF16 && !VEC4) request_x();
    wave_lds_sync();

    // ---- products -----------------------------------------------------------------------------------------
    float4 G[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) G[i] = *reinterpret_cast<const float4*>(&sG[(i * 64 + lane) * 4]);
    auto comp = [](const float4& v, int r) { return r == 0 ? v.x : r == 1 ? v.y : r == 2 ? v.z : v.w; };
    f32x4 C[4][4];   // [row class 2a + parity][w'], component s: quadruple base i0 = 4s + g
#pragma unroll
    for (int rt = 0; rt < 4; ++rt)
#pragma unroll
      for (int e = 0; e < 4; ++e) C[rt][e] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int rt = 0; rt < 4; ++rt) {
      // product a for the 16 rows of class rt (physical rows 16 rt + m); k-block kg is column class kg
      const float* arow = &tile[(16 * rt + c) * D32_LDT + 4 * g];
      float4 a[4];
#pragma unroll
      for (int kg = 0; kg < 4; ++kg) a[kg] = *reinterpret_cast<const float4*>(arow + 16 * kg);
      f32x4 P[4];   // E_0, O_0, E_1, O_1
#pragma unroll
      for (int kg = 0; kg < 4; ++kg) P[kg] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int kr = 0; kr < 4; ++kr)
#pragma unroll
        for (int kg = 0; kg < 4; ++kg)   // the tile holds fixed-point sums
          P[kg] = mfma4((float)__float_as_int(comp(a[kg], kr)), comp(G[kg & 1], kr), P[kg]);
      // columns member(w', kappa(c)) of Y
      const f32x4 Y[4] = {P[0] + P[1], P[0] - P[1], P[2] + P[3], P[2] - P[3]};
      // product b: this row class feeds its own partial sum
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int e = 0; e < 4; ++e) C[rt][e] = mfma4(comp(G[rt & 1], r), Y[e][r], C[rt][e]);
    }

    // ---- R (pair identities) goes through the tile, which is dead by now, into the layout of the
    //      parameters.  Row i is kept at tile row rperm(i) = 16 (i / 16) + 4 (i % 4) + (i / 4) % 4.
    //      For i = member(w, 4s + g):  rperm = 16 w + 4 g + s (w even),  16 w + 4 (3 - g) + (3 - s) (w odd).
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float* wcol = tile + ((e & 1) ? wr_col_dn : wr_col_up) + (e >= 2 ? 32 : 0);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const float rr[4] = {C[0][e][s] + C[1][e][s], C[0][e][s] - C[1][e][s], C[2][e][s] + C[3][e][s],
                             C[2][e][s] - C[3][e][s]};
#pragma unroll
        for (int w = 0; w < 4; ++w)
          wcol[((w & 1) ? row_dn : row_up) + (16 * w + ((w & 1) ? 3 - s : s)) * D32_LDT] = rr[w];
      }
    }
    wave_lds_sync();

    // ---- x <- x - lr*(phi(R) + wd*x): phi = sgn, or the identity on the aggregate (the sums of chunk q carry the
    //      factor 2^sh[q]; rows of members w < 2 lie in the upper chunks, this lane's columns in the left or right
    //      ones) ---------------------------------------------------------------------------------------------------
    const bool right = (c & 3) >= 2;
    const float f_up = IDENT ? ldexpf(args.scale, -(right ? sh[1] : sh[0])) : 0.f;
    const float f_dn = IDENT ? ldexpf(args.scale, -(right ? sh[3] : sh[2])) : 0.f;
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
            &tile[((w & 1) ? row_dn : row_up) + (16 * w + ((w & 1) ? 3 - s : s)) * D32_LDT + col4]);
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
          o[e] = sign_update(x, IDENT ? rr[e] * (w < 2 ? f_up : f_dn) : sgnf(rr[e]), args.lr, args.weight_decay);
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
  }
}

template <bool PBF16, int MODE, bool IDENT, bool COUNT = false, bool NT = true>
static hipError_t launch_dec_tile32_phi(const TableView& tiles, const float* tables, const DecodeArgs& a, int64_t grid,
                                        hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode2d_tile32<PBF16, MODE, IDENT, COUNT, NT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, D32_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((decode2d_tile32<PBF16, MODE, IDENT, COUNT, NT>), dim3((unsigned)grid), dim3(D32_THREADS),
                     D32_LDS_BYTES, stream, tiles, tables, a);
  return hipGetLastError();
}
template <bool PBF16, int MODE, bool NT>
static hipError_t launch_dec_tile32_nt(const TableView& tiles, const float* tables, const DecodeArgs& a, int64_t grid,
                                       hipStream_t stream) {
  if constexpr (MODE != 2) {
    if (a.agg == 2)
      return a.phi != 0 ? launch_dec_tile32_phi<PBF16, MODE, true, true, NT>(tiles, tables, a, grid, stream)
                        : launch_dec_tile32_phi<PBF16, MODE, false, true, NT>(tiles, tables, a, grid, stream);
  }
  return a.phi != 0 ? launch_dec_tile32_phi<PBF16, MODE, true, false, NT>(tiles, tables, a, grid, stream)
                    : launch_dec_tile32_phi<PBF16, MODE, false, false, NT>(tiles, tables, a, grid, stream);
}
template <bool PBF16, int MODE>
static hipError_t launch_dec_tile32(const TableView& tiles, const float* tables, const DecodeArgs& a, int64_t grid,
                                    hipStream_t stream) {
  if constexpr (MODE != 0) {   // rows of k pairs shorter than a 128-byte line: plain loads
    if (a.k < 32) return launch_dec_tile32_nt<PBF16, MODE, false>(tiles, tables, a, grid, stream);
  }
  return launch_dec_tile32_nt<PBF16, MODE, true>(tiles, tables, a, grid, stream);
}

hipError_t launch_decode2d_tile32(const TableView& tiles, const float* tables, const DecodeArgs& a, bool param_bf16,
                                  int num_cus, hipStream_t stream) {
  const bool aligned16 = (tiles.dtypes & 16u) == 0;
  if (!fast32_decode_supports(a.W, a.k, aligned16)) return hipErrorInvalidValue;
  if (a.agg == 2 && (int64_t)a.W * a.k > kFast32MaxPairs) return hipErrorInvalidValue;   // counted from registers
  int64_t grid = num_cus;
  const int64_t max_grid = ((int64_t)tiles.total_chunks + DEMO_RUN - 1) / DEMO_RUN;   // few items: one run per workgroup, spread over the CUs
  if (grid > max_grid) grid = max_grid;
  const int mode = (int64_t)a.W * a.k > kFast32MaxPairs ? 2 : ((a.k & 3) == 0 && aligned16) ? 1 : 0;
  if (param_bf16) {
    switch (mode) {
      case 2: return launch_dec_tile32<true, 2>(tiles, tables, a, grid, stream);
      case 1: return launch_dec_tile32<true, 1>(tiles, tables, a, grid, stream);
      default: return launch_dec_tile32<true, 0>(tiles, tables, a, grid, stream);
    }
  }
  switch (mode) {
    case 2: return launch_dec_tile32<false, 2>(tiles, tables, a, grid, stream);
    case 1: return launch_dec_tile32<false, 1>(tiles, tables, a, grid, stream);
    default: return launch_dec_tile32<false, 0>(tiles, tables, a, grid, stream);
  }
}

}  // namespace demo
