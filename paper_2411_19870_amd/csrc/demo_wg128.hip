// s = 128 kernels: one 1024-thread workgroup (16 wavefronts) per 128 x 128 chunk, one workgroup per CU.
//
// A chunk is too large for one wavefront's registers, so it lives in an LDS tile and the products read their
// operands from LDS; sixteen wavefronts (four per SIMD) hide the operand reads behind one another's MFMAs, and
// the rows of the next chunk are fetched into registers (24 - 32 per lane) while this one is transformed.
//
// Mirror folds: row u of the 128-point orthonormal DCT-II is even (u even) or odd (u odd) under i -> 127-i, and
// the even rows are in turn even (u = 0 mod 4) or odd (u = 2 mod 4) under i -> 63-i.  A product that contracts
// over i needs i < 64 of x[i] - x[127-i] for the odd rows and i < 32 of (x[i] + x[127-i]) +- (x[63-i] + x[64+i])
// for the two even classes; a product whose output index is i needs the matching partial sums, the mirror
// outputs being their sums and differences.  Either way 768 instead of 2048 MFMAs (16x16x4) per product.  The
// basis sits in LDS as P[u][i], i < 64, rows grouped by class: row u at position pos3(u) (u = 0 mod 4, then
// u = 2 mod 4, then odd); coefficient rows and columns are held in the same class-major order and translated
// when the payload is written.
//
// The contraction index of k-slot g at step s of group kg is 16 kg + 4 g + s, so that operands whose
// contraction index runs along an LDS row come in one 16-byte read per four MFMAs.  The encode kernel contracts the
// columns first (Z = X P^T, rows of X read along j) and writes Z transposed, four consecutive i per 16-byte store
// as they lie in an accumulator, so that the second product (Q = P Z) reads Z along i as well: no operand is read
// across rows.
#include <type_traits>

#include "demo_device.h"

namespace demo {

namespace {
constexpr int W128_WAVES = 16;
constexpr int W128_THREADS = 64 * W128_WAVES;
constexpr int W128_LDX = 132;                          // data tile row stride (floats)
constexpr int W128_LDP = 68;                           // folded basis row stride
constexpr int W128_P_FLOATS = 128 * W128_LDP;
constexpr int W128_X_FLOATS = 128 * W128_LDX;
constexpr int W128_CAP = 512;                          // candidate list of the top-k
constexpr int W128_SEL = 68;                           // entries per class list of selected coefficients (k <= 64, padded)
constexpr int W128_ENC_LDS_BYTES = 4 * (W128_P_FLOATS + W128_X_FLOATS + 128 + 16 + W128_CAP) + 8 * (W128_CAP + 2 + 4 * W128_SEL);
static_assert(W128_ENC_LDS_BYTES <= 160 * 1024, "LDS budget");

// Workgroup barrier that orders LDS accesses only: global loads and stores stay in flight across it.
__device__ __forceinline__ void wg_lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// class-major position of frequency u: u = 0 mod 4 first, then u = 2 mod 4, then odd u
__device__ __forceinline__ int pos3(uint32_t u) { return (int)((u & 1u) ? 64u + (u >> 1) : ((u & 2u) << 4) + (u >> 2)); }

// folded basis into LDS: P[u][i], i < 64, at row pos3(u)
__device__ __forceinline__ void stage_folded_basis(float* sP, const float* __restrict__ basis, int tid) {
  for (int e = tid; e < 128 * 16; e += W128_THREADS) {
    const int u = e >> 4, c4 = (e & 15) * 4;
    *reinterpret_cast<f32x4*>(&sP[pos3((uint32_t)u) * W128_LDP + c4]) = gload_f4(basis + u * 128 + c4);
  }
}
}  // namespace

// ---------------------------------------------------------------------------
// encode:  m <- beta m + g ;  Q = P B P^T ;  k largest |Q| ;  m <- m - alpha P^T Q^ P      (Algorithm 1, worker side)
// ---------------------------------------------------------------------------
// Thread t owns elements (rows t/32 + 32 p, columns 4 (t%32) .. +3), p < 4, of the chunk: loads, momentum
// update and the final store happen in this layout (a wavefront touches two 512-byte row segments per access).
// A chunk whose candidate list overflows (many equal magnitudes at the threshold) is left untouched and queued
// for the exact generic kernel that runs next.
template <bool GBF16>
__global__ __launch_bounds__(W128_THREADS) void encode2d_wg128(TableView tv, const float* __restrict__ basis,
                                                                EncodeArgs args, Worklist wl) {
  extern __shared__ float lds[];
  float* sP = lds;
  float* sX = sP + W128_P_FLOATS;
  uint32_t* gmax = reinterpret_cast<uint32_t*>(sX + W128_X_FLOATS);   // [128] maxima of groups of 8 lanes
  int* ctl = reinterpret_cast<int*>(gmax + 128);                      // [0] candidate cursor, [1] threshold, [2] all-zero flag, [4..7] class counts
  uint32_t* rk = reinterpret_cast<uint32_t*>(ctl + 16);               // [CAP] rank | class rank << 16 of a candidate
  uint2* cand = reinterpret_cast<uint2*>(rk + W128_CAP);              // [CAP + 2] {coefficient bits, flat index}
  uint2* sel = cand + W128_CAP + 2;                                   // [4][SEL]  {basis row offsets, coefficient bits}
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, lq = lane >> 4;
  const int k = args.k;
  const int total = tv.total_chunks;
  int chunk = blockIdx.x;
  if (chunk >= total) return;

  stage_folded_basis(sP, basis, tid);

  using GT = typename std::conditional<GBF16, u32x2, f32x4>::type;
  const int lrow = tid >> 5, lcol = (tid & 31) * 4;
  f32x4 mv[4];
  GT gv[4];
  // rows 32 p + lrow of the chunk `cc` of tensor `dd`: one quarter of the chunk per call (p < 4)
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
  auto issue_quarter = [&](int p) {
    const uint32_t vo = (uint32_t)lrow * ucols_in + (uint32_t)lcol;
    mv[p] = bload_f4(mres_in, vo * 4, 32u * p * ucols_in * 4);
    if constexpr (GBF16) gv[p] = bload_u2(gres_in, vo * 2, 32u * p * ucols_in * 2);
    else gv[p] = bload_f4(gres_in, vo * 4, 32u * p * ucols_in * 4);
  };

  int t = find_tensor_uniform(tv, chunk);
  int t_first = uniform_prefix(tv, t), t_next = uniform_prefix(tv, t + 1);
  TensorDev d = load_desc_uniform(tv, t);
  set_source(d, chunk - t_first);
#pragma unroll
  for (int p = 0; p < 4; ++p) issue_quarter(p);

  // flat index 128 u + v of coefficient acc[a][r] of the second product (column tile vt = wave / 2, half h = wave % 2):
  // column position 16 vt + l16, i.e. v = vb + sv l16 with sv = 4 (even classes) or 2 (odd columns); row position
  // 32 h + 16 a + 4 lq + r of an even class (a < 2): u = 4 (16 a + 4 lq + r) + 2 h, or 64 + 32 h + 16 (a - 2) + 4 lq + r
  // of the odd class: u = 2 (32 h + 16 (a - 2) + 4 lq + r) + 1
  const int q_vt = wave >> 1, q_h = wave & 1;
  const int q_sv = q_vt < 4 ? 4 : 2;
  const int q_vb = q_vt < 2 ? 64 * q_vt : q_vt < 4 ? 64 * (q_vt - 2) + 2 : 32 * (q_vt - 4) + 1;

  // momentum update of the chunk whose rows are in the registers, staged into the tile
  f32x4 D[4];
  auto update_and_stage = [&]() {
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      f32x4 gf;
      if constexpr (GBF16) {
        gf = (f32x4){bf16_to_f32(gv[p][0] & 0xffffu), bf16_to_f32(gv[p][0] >> 16), bf16_to_f32(gv[p][1] & 0xffffu),
                     bf16_to_f32(gv[p][1] >> 16)};
      } else {
        gf = gv[p];
      }
#pragma unroll
      for (int e = 0; e < 4; ++e) D[p][e] = __fmaf_rn(args.beta, mv[p][e], args.grad_scale * gf[e]);
      *reinterpret_cast<f32x4*>(&sX[(lrow + 32 * p) * W128_LDX + lcol]) = D[p];
    }
  };
  update_and_stage();

  DEMO_PHASE_DECL
  for (;;) {
    // ---- the tile holds D = beta m + g of this chunk; the registers take the rows of the next one -----------
    int tidv = tid;
    asm volatile("" : "+v"(tidv));   // addresses below are recomputed per chunk rather than kept (and spilled) across it
    const uint32_t zero = (uint32_t)(tidv >> 31);                            // 0, formed per chunk like the addresses
    if (tidv < 4 * W128_SEL) sel[tidv] = make_uint2(zero, zero);             // zero-valued padding of the class lists
    if (tidv < W128_CAP + 2) cand[tidv] = make_uint2(zero, ~zero);            // entries that precede nothing
    if (tidv < W128_CAP) rk[tidv] = zero;
    if (tidv < 8) ctl[tidv] = (int)zero;
    // where this chunk's results go
    const int cc = chunk - t_first;
    const uint32_t ucols = (uint32_t)d.cols;
    const __amdgpu_buffer_rsrc_t mres_out =
        make_rsrc(d.mom + ((int64_t)(cc / d.cchunks) * 128 * d.cols + (int64_t)(cc % d.cchunks) * 128));
    DEMO_GLOBAL int32_t* const out_idx = as_global(d.idx) + (int64_t)cc * k;
    DEMO_GLOBAL float* const out_val = as_global(d.val) + (int64_t)cc * k;
    const int nxt = chunk + (int)gridDim.x;
    const bool has_next = nxt < total;
    if (has_next) {
      while (nxt >= t_next) {
        ++t;
        t_first = t_next;
        t_next = uniform_prefix(tv, t + 1);
        d = load_desc_uniform(tv, t);
      }
      set_source(d, nxt - t_first);
    }
    wg_lds_barrier();
    DEMO_PHASE(0);

    // ---- product 1: Z[i][v] = sum_j X[i][j] P[v][j] on the folded columns of X; the wavefront owns row tile
    //      it = wave / 2, two column tiles of the even class h = wave % 2 (v = 0 / 2 mod 4) and the odd column
    //      tiles 2 h, 2 h + 1 -------------------------------------------------------------------------------------
    f32x4 acc[4];
    {
      const int it = wave >> 1, h = wave & 1;
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
      const float* pc = sP + (32 * h + l16) * W128_LDP + 4 * lq;
      const float* po = sP + (64 + 32 * h + l16) * W128_LDP + 4 * lq;
      const float* xr = sX + (16 * it + l16) * W128_LDX;
#pragma unroll
      for (int kg = 0; kg < 4; ++kg) {
        // columns j = 16 kg + 4 lq + s and 127 - j
        const f32x4 t0 = *reinterpret_cast<const f32x4*>(xr + 16 * kg + 4 * lq);
        const f32x4 t1 = *reinterpret_cast<const f32x4*>(xr + 124 - 16 * kg - 4 * lq);
        if (kg < 2) {
          // and 63 - j, 64 + j
          const f32x4 t2 = *reinterpret_cast<const f32x4*>(xr + 60 - 16 * kg - 4 * lq);
          const f32x4 t3 = *reinterpret_cast<const f32x4*>(xr + 64 + 16 * kg + 4 * lq);
          float ac[4];
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            const float e0 = t0[s] + t1[3 - s], e1 = t2[3 - s] + t3[s];
            ac[s] = h ? e0 - e1 : e0 + e1;
          }
#pragma unroll
          for (int c2 = 0; c2 < 2; ++c2) {
            const f32x4 b = *reinterpret_cast<const f32x4*>(pc + 16 * c2 * W128_LDP + 16 * kg);
#pragma unroll
            for (int s = 0; s < 4; ++s) acc[c2] = mfma4(ac[s], b[s], acc[c2]);
          }
        }
#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2) {
          const f32x4 b = *reinterpret_cast<const f32x4*>(po + 16 * c2 * W128_LDP + 16 * kg);
#pragma unroll
          for (int s = 0; s < 4; ++s) acc[2 + c2] = mfma4(t0[s] - t1[3 - s], b[s], acc[2 + c2]);
        }
        // the next chunk's rows, a quarter per other step of the two products: the requests of the sixteen
        // wavefronts trickle into the memory pipeline instead of queueing at a barrier
        if (has_next && (kg & 1) == 0) issue_quarter(kg >> 1);
        __builtin_amdgcn_sched_barrier(0);
      }
      wg_lds_barrier();   // every read of X is done: Z^T replaces it, row = column position of v, four i per store
#pragma unroll
      for (int c2 = 0; c2 < 2; ++c2) {
        *reinterpret_cast<f32x4*>(&sX[(32 * h + 16 * c2 + l16) * W128_LDX + 16 * it + 4 * lq]) = acc[c2];
        *reinterpret_cast<f32x4*>(&sX[(64 + 32 * h + 16 * c2 + l16) * W128_LDX + 16 * it + 4 * lq]) = acc[2 + c2];
      }
    }
    wg_lds_barrier();
    DEMO_PHASE(1);

    // ---- product 2: Q[u][v] = sum_i P[u][i] Z[i][v] on the folded rows of Z (read along i from Z^T); the wavefront
    //      owns column tile vt = wave / 2 (positions 16 vt ..), two row tiles of the even class h = wave % 2 and the odd
    //      row tiles 2 h, 2 h + 1 -------------------------------------------------------------------------------------
    {
      const int vt = wave >> 1, h = wave & 1;
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
      const float* pc = sP + (32 * h + l16) * W128_LDP + 4 * lq;
      const float* po = sP + (64 + 32 * h + l16) * W128_LDP + 4 * lq;
      const float* zr = sX + (16 * vt + l16) * W128_LDX;
#pragma unroll
      for (int kg = 0; kg < 4; ++kg) {
        // rows i = 16 kg + 4 lq + s and 127 - i
        const f32x4 t0 = *reinterpret_cast<const f32x4*>(zr + 16 * kg + 4 * lq);
        const f32x4 t1 = *reinterpret_cast<const f32x4*>(zr + 124 - 16 * kg - 4 * lq);
        if (kg < 2) {
          // and 63 - i, 64 + i
          const f32x4 t2 = *reinterpret_cast<const f32x4*>(zr + 60 - 16 * kg - 4 * lq);
          const f32x4 t3 = *reinterpret_cast<const f32x4*>(zr + 64 + 16 * kg + 4 * lq);
          float bc[4];
#pragma unroll
          for (int s = 0; s < 4; ++s) {
            const float e0 = t0[s] + t1[3 - s], e1 = t2[3 - s] + t3[s];
            bc[s] = h ? e0 - e1 : e0 + e1;
          }
#pragma unroll
          for (int c2 = 0; c2 < 2; ++c2) {
            const f32x4 a = *reinterpret_cast<const f32x4*>(pc + 16 * c2 * W128_LDP + 16 * kg);
#pragma unroll
            for (int s = 0; s < 4; ++s) acc[c2] = mfma4(a[s], bc[s], acc[c2]);
          }
        }
#pragma unroll
        for (int c2 = 0; c2 < 2; ++c2) {
          const f32x4 a = *reinterpret_cast<const f32x4*>(po + 16 * c2 * W128_LDP + 16 * kg);
#pragma unroll
          for (int s = 0; s < 4; ++s) acc[2 + c2] = mfma4(a[s], t0[s] - t1[3 - s], acc[2 + c2]);
        }
        if (has_next && (kg & 1) == 0) issue_quarter(2 + (kg >> 1));
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    DEMO_PHASE(2);

    // ---- top-k over the 16384 coefficients -----------------------------------------------------------------
    // (1) lower bound of the k-th largest magnitude: the k-th largest of the 128 maxima of groups of 8 lanes
    //     (each a coefficient of its own), resolved to its upper 16 bits
    float gm[4];   // largest magnitude of each accumulator
#pragma unroll
    for (int i = 0; i < 4; ++i)
      gm[i] = fmaxf(fmaxf(fabsf(acc[i][0]), fabsf(acc[i][1])), fmaxf(fabsf(acc[i][2]), fabsf(acc[i][3])));
    uint32_t lm = __float_as_uint(fmaxf(fmaxf(gm[0], gm[1]), fmaxf(gm[2], gm[3])));
    lm = max(lm, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lm, 0xB1, 0xf, 0xf, false));    // quad_perm [1,0,3,2]
    lm = max(lm, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lm, 0x4E, 0xf, 0xf, false));    // quad_perm [2,3,0,1]
    lm = max(lm, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)lm, 0x141, 0xf, 0xf, false));   // row_half_mirror
    const int lanev = tidv & 63;
    if ((lanev & 7) == 0) gmax[8 * wave + (lanev >> 3)] = lm;
    wg_lds_barrier();
    if (wave == 0) {
      // one wavefront bisects (sixteen doing the same would only queue at the scalar unit)
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
    const float thr_f = __uint_as_float((uint32_t)__builtin_amdgcn_readfirstlane(ctl[1]));
    // (2) candidates |q| >= thr: a wavefront reserves its range of the list with one atomic.  Accumulators whose
    //     largest magnitude is below the threshold in every lane are passed over as a whole.
    {
      // lane parts of the flat indices, formed per chunk from the opaque lane id (kept across the chunk, these
      // and the 16 per-register indices derived from them would be spilled)
      const uint32_t fv = (uint32_t)(q_vb + q_sv * (lanev & 15));
      const uint32_t fc = (uint32_t)(2048 * (lanev >> 4) + 256 * q_h) + fv;
      const uint32_t fo = (uint32_t)(8192 * q_h + 1024 * (lanev >> 4) + 128) + fv;
      int cnt = 0;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (__ballot(gm[i] >= thr_f) != 0) {
#pragma unroll
          for (int r = 0; r < 4; ++r) cnt += __popcll(__ballot(fabsf(acc[i][r]) >= thr_f));
        }
      int base = 0;
      if (lane == 0 && cnt != 0) base = atomicAdd(&ctl[0], cnt);
      base = __builtin_amdgcn_readfirstlane(base);
#pragma unroll
      for (int i = 0; i < 4; ++i)
        if (__ballot(gm[i] >= thr_f) != 0) {
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const bool is = fabsf(acc[i][r]) >= thr_f;
            const uint64_t mask = __ballot(is);
            if (mask != 0) {
              const int pos = base + lanes_below(mask);
              if (is && pos < W128_CAP) cand[pos] = make_uint2(__float_as_uint(acc[i][r]), i < 2 ? fc + (uint32_t)(8192 * i + 512 * r) : fo + (uint32_t)(4096 * (i - 2) + 256 * r));
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
    //     2 (u % 2) + v % 2; the sixteen partial counts meet in rk[].
    if (!overflow) {
      const int slice = 2 * ((ncand + 31) >> 5);
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
        store_guarded(out_idx + rank, (int32_t)me.y);
        store_guarded(out_val + rank, __uint_as_float(me.x));
        const int cls = (int)(((me.y >> 6) & 2u) | (me.y & 1u));
        // byte offsets of rows pos3(u) and pos3(v) of the basis tile, and the value
        const uint32_t offs = (uint32_t)(pos3(me.y >> 7) * (W128_LDP * 4)) | ((uint32_t)(pos3(me.y & 127u) * (W128_LDP * 4)) << 16);
        sel[cls * W128_SEL + rcls] = make_uint2(offs, me.x);
        atomicAdd(&ctl[4 + cls], 1);
      }
    }
    wg_lds_barrier();
    DEMO_PHASE(4);

    // ---- reconstruction on the quadrant i, j < 64, one partial sum per class (a, b) = (u % 2, v % 2):
    //      R[i][j] = sum s_ab,  R[127-i][j] = sum (-1)^a s_ab,  R[i][127-j] = sum (-1)^b s_ab ---------------------
    {
      const int mt = wave >> 2, nt = wave & 3;
      f32x4 rc[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) rc[c] = (f32x4){0.f, 0.f, 0.f, 0.f};
      // the lists are zero-padded, so every class runs to the length of the longest
      const int4 nc = *reinterpret_cast<const int4*>(&ctl[4]);
      const int nmax = __builtin_amdgcn_readfirstlane(max(max(nc.x, nc.y), max(nc.z, nc.w)));
      const float* pa = sP + 16 * mt + l16;
      const float* pb = sP + 16 * nt + l16;
      uint2 en[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) en[c] = sel[c * W128_SEL + (lanev >> 4)];
      for (int st = 0; 4 * st < nmax; ++st) {
        uint2 e[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) e[c] = en[c];
        float a[4], b[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          a[c] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(pa) + (e[c].x & 0xffffu));
          b[c] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(pb) + (e[c].x >> 16));
        }
        // entries of the next step (the lists are 68 long and zero past their ends: step 16 reads padding)
#pragma unroll
        for (int c = 0; c < 4; ++c) en[c] = sel[c * W128_SEL + 4 * (st + 1) + (lanev >> 4)];
#pragma unroll
        for (int c = 0; c < 4; ++c) rc[c] = mfma4(__uint_as_float(e[c].y) * a[c], b[c], rc[c]);
      }
      // four base addresses formed per chunk (kept across the chunk they would be spilled), rows at immediate offsets
      const int lqv = lanev >> 4, l16v = lanev & 15;
      float* w00 = sX + (16 * mt + 4 * lqv) * W128_LDX + 16 * nt + l16v;            // (i0, j0), r = 0
      float* w01 = sX + (16 * mt + 4 * lqv) * W128_LDX + 127 - 16 * nt - l16v;      // (i0, 127 - j0)
      float* w10 = sX + (124 - 16 * mt - 4 * lqv) * W128_LDX + 16 * nt + l16v;      // (127 - i0, j0), r = 3
      float* w11 = sX + (124 - 16 * mt - 4 * lqv) * W128_LDX + 127 - 16 * nt - l16v;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float pe = rc[0][r] + rc[1][r], po = rc[2][r] + rc[3][r];
        const float me = rc[0][r] - rc[1][r], mo = rc[2][r] - rc[3][r];
        w00[r * W128_LDX] = pe + po;
        w01[r * W128_LDX] = me + mo;
        w10[(3 - r) * W128_LDX] = pe - po;
        w11[(3 - r) * W128_LDX] = me - mo;
      }
    }
    wg_lds_barrier();
    DEMO_PHASE(5);

    // ---- m <- D - alpha R.  The rows of the next chunk are consumed (into D and the tile) before the stores are
    //      issued, so that waiting for those rows never waits for these stores ---------------------------------
    {
      f32x4 o[4];
#pragma unroll
      for (int p = 0; p < 4; ++p) {
        const f32x4 rv = *reinterpret_cast<const f32x4*>(&sX[(lrow + 32 * p) * W128_LDX + lcol]);
#pragma unroll
        for (int e = 0; e < 4; ++e) o[p][e] = __fmaf_rn(-args.alpha, rv[e], D[p][e]);
      }
      DEMO_PHASE(6);
      if (has_next) update_and_stage();
      DEMO_PHASE(7);
      if (!skip) {
        const uint32_t vo = (uint32_t)lrow * ucols + (uint32_t)lcol;
#pragma unroll
        for (int p = 0; p < 4; ++p) bstore_f4(mres_out, vo * 4, 32u * p * ucols * 4, o[p]);
      }
    }
    DEMO_PHASE(0);
    if (!has_next) break;
    chunk = nxt;
  }
  DEMO_PHASE_FLUSH(0);
}

template <bool GBF16>
static hipError_t launch_enc_wg128(const TableView& tv, const float* basis, const EncodeArgs& a, const Worklist& wl,
                                   int64_t grid, hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&encode2d_wg128<GBF16>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, W128_ENC_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(encode2d_wg128<GBF16>, dim3((unsigned)grid), dim3(W128_THREADS), W128_ENC_LDS_BYTES, stream, tv,
                     basis, a, wl);
  return hipGetLastError();
}

hipError_t launch_encode2d_wg128(const TableView& tv, const float* basis, const EncodeArgs& a, const Worklist& wl,
                                 bool grad_bf16, int num_cus, hipStream_t stream) {
  if (a.k < 1 || a.k > kFast128MaxK || wl.list == nullptr) return hipErrorInvalidValue;
  int64_t grid = num_cus;
  if (grid > tv.total_chunks) grid = tv.total_chunks;
  return grad_bf16 ? launch_enc_wg128<true>(tv, basis, a, wl, grid, stream)
                   : launch_enc_wg128<false>(tv, basis, a, wl, grid, stream);
}

// ---------------------------------------------------------------------------
// decode:  S = sum over workers of the payloads ;  R = P^T S P ;  x <- x - lr (sgn(R) + wd x)     (Algorithm 1, update)
// ---------------------------------------------------------------------------
// Sign descent on the plain sum only (the other operating points run on the generic kernel).  The W k <= 4096
// pairs of a chunk sit in at most four registers per lane (pair 1024 j + tid belongs to worker p / k, position
// p % k) and are fetched for the next chunk while the products of this one run.  S is accumulated in block
// fixed point with integer LDS atomics (one scale per chunk: the sum is exact and independent of the order of
// arrival).  Two mirror folds: rows u = 0 mod 4 of P are even under i -> 63-i and i -> 127-i, rows u = 2 mod 4
// odd / even, odd rows odd under i -> 127-i.  For the quadruple {i, 63-i, 64+i, 127-i}, i < 32, four partial sums
//   E0 = sum over u = 0 mod 4,  E2 = sum over u = 2 mod 4  (32 frequencies each),
//   Oa = sum over odd u of P[u][i] ..,  Ob = sum over odd u of P[u][63-i] ..  (64 frequencies each)
// give out[i] = E0+E2+Oa, out[127-i] = E0+E2-Oa, out[63-i] = E0-E2+Ob, out[64+i] = E0-E2-Ob: 768 MFMAs per
// product instead of 2048.  S is held with rows and columns in class-major order pos3(); basis in LDS:
// PT[i][pos3(u)] = P[u][i], i < 64, so that both products read it along the contraction index.
namespace {
constexpr int W128_DEC_SLOTS = 4;
constexpr int W128_PT_FLOATS = 64 * W128_LDX;
constexpr int W128_DEC_LDS_BYTES = 4 * (W128_PT_FLOATS + W128_X_FLOATS + 32);
static_assert(kFast128MaxPairs == W128_DEC_SLOTS * W128_THREADS, "pairs per chunk held in registers");
}  // namespace

// STREAM false: W k <= 4096, one pair per load (consecutive threads read consecutive pairs, and the pairs are spread
// evenly over the sixteen wavefronts; 16-byte loads would leave half of them without work at W k = 2048 and measured
// slower).  STREAM true: more than 4096 pairs per chunk (up to 65536), k a multiple of four and 16-byte aligned payload
// arrays: one pass in rounds of 4096 pairs, a thread fetching four consecutive pairs of one worker per load; the sums
// are shifted down whenever a round raises the block exponent.
// IDENT: phi is the identity on the aggregate instead of sgn (its own instance).  COUNT: the count-normalised
// aggregate of the appendix algorithm "Sparse Top-k Averaging" (every coefficient's sum divided by the number of pairs
// that name it), without STREAM only.
template <bool PBF16, bool STREAM, bool IDENT, bool COUNT = false>
__global__ __launch_bounds__(W128_THREADS) void decode2d_wg128(TableView tv, const float* __restrict__ basis,
                                                                DecodeArgs args) {
  constexpr bool VEC4 = STREAM;
  extern __shared__ float lds[];
  float* sPT = lds;
  float* tile = sPT + W128_PT_FLOATS;
  int* itile = reinterpret_cast<int*>(tile);
  uint32_t* wmax = reinterpret_cast<uint32_t*>(tile + W128_X_FLOATS);   // [2][16] per-wavefront largest |val| (two buffers: consecutive rounds of a streamed payload alternate)
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l16 = lane & 15, lq = lane >> 4;
  const int k = args.k, W = args.W;
  const int npairs = W * k;
  const int nunits = npairs >> 2;                                  // VEC4: 16-byte units per chunk
  const int nslots = VEC4 ? W128_DEC_SLOTS : (npairs + W128_THREADS - 1) / W128_THREADS;   // payload registers in use (uniform)
  const int nrounds = STREAM ? (nunits + W128_THREADS - 1) / W128_THREADS : 1;
  const int total = tv.total_chunks;
  int chunk = blockIdx.x;
  if (chunk >= total) return;

  // PT[i][pos3(u)] = P[u][i]: thread reads P[u][4c..4c+3] and writes four rows of the transposed tile
  for (int e = tid; e < 128 * 16; e += W128_THREADS) {
    const int u = e >> 4, c4 = (e & 15) * 4;
    const f32x4 v = gload_f4(basis + u * 128 + c4);
#pragma unroll
    for (int x = 0; x < 4; ++x) sPT[(c4 + x) * W128_LDX + pos3((uint32_t)u)] = v[x];
  }

  int32_t pi[W128_DEC_SLOTS];
  float pv[W128_DEC_SLOTS];
#pragma unroll
  for (int j = 0; j < W128_DEC_SLOTS; ++j) {
    pi[j] = -1;
    pv[j] = 0.f;
  }
  const float rk = 1.0f / (float)k;
  // `round` matters in STREAM mode only: units 1024 round + tid
  auto load_payload = [&](const TensorDev& dd, int cc, int round = 0) {
    const DEMO_GLOBAL int32_t* ip = as_global(dd.idx) + (int64_t)cc * k;
    const DEMO_GLOBAL float* vp = as_global(dd.val) + (int64_t)cc * k;
    const int wstride = dd.nchunks * k;                        // pairs of one worker for this tensor
    if constexpr (VEC4) {
      static_assert(W128_DEC_SLOTS == 4, "one 16-byte load per array fills the payload registers");
      const int unit = (STREAM ? W128_THREADS * round : 0) + tid;
      const int p = 4 * unit;
      const int w = (int)(((float)p + 0.5f) * rk);             // as below (p < 65536)
      const int pos = p - w * k;
      const bool ok = unit < nunits;
      const uint32_t off = ok ? (uint32_t)(w * wstride + pos) : 0u;
      const f32x4 vv = payload_load<true>(reinterpret_cast<const DEMO_GLOBAL f32x4*>(vp + off));
#pragma unroll
      for (int e = 0; e < 4; ++e) pv[e] = vv[e];
      const u32x4 iv = payload_load<true>(reinterpret_cast<const DEMO_GLOBAL u32x4*>(ip + off));
#pragma unroll
      for (int e = 0; e < 4; ++e) pi[e] = (int32_t)iv[e];
      return;
    }
    // every offset before the first load, and the loads unconditional (a slot past the end reads the chunk's first
    // pair; mask_payload discards it where the pairs are consumed): address arithmetic between the loads picked up a
    // register of a load in flight as the unused high half of a 64-bit operand, and the wave then waited out that
    // load before it issued the next (two memory round trips per chunk)
    uint32_t off[W128_DEC_SLOTS];
#pragma unroll
    for (int j = 0; j < W128_DEC_SLOTS; ++j) {
      const int p = W128_THREADS * j + tid;
      // worker p / k and position p % k; (p + 1/2) / k is never within 1/(2k) of an integer, far more than
      // the rounding error of the float product for p < 4096
      const int w = (int)(((float)p + 0.5f) * rk);
      const int pos = p - w * k;
      off[j] = p < npairs ? (uint32_t)w * (uint32_t)wstride + (uint32_t)pos : 0u;
    }
#pragma unroll
    for (int j = 0; j < W128_DEC_SLOTS; ++j) {
      if (j < nslots) {                                        // uniform
        pi[j] = payload_load<true>(ip + off[j]);
        pv[j] = payload_load<true>(vp + off[j]);
      }
    }
  };
  // Slots past the end of the chunk's payload become (no index, 0).  Applied where the pairs are consumed, not where
  // they are requested: a select behind the load would make the prefetch wait for its own data.
  auto mask_payload = [&](int round = 0) {
#pragma unroll
    for (int j = 0; j < W128_DEC_SLOTS; ++j) {
      const bool ok = VEC4 ? (STREAM ? W128_THREADS * round : 0) + tid < nunits : W128_THREADS * j + tid < npairs;
      pi[j] = ok ? pi[j] : -1;
      pv[j] = ok ? pv[j] : 0.f;
    }
  };

  int t = find_tensor_uniform(tv, chunk);
  int t_first = uniform_prefix(tv, t), t_next = uniform_prefix(tv, t + 1);
  TensorDev d = load_desc_uniform(tv, t);
  load_payload(d, chunk - t_first, 0);
  // the first chunk's pairs are waited for here, outside the loop: with loads pending at the loop's entry and
  // the parameter stores pending on its back edge, the loop's first wait would be for everything outstanding,
  // i.e. every chunk would begin by waiting for the acknowledgements of the previous chunk's stores
#pragma unroll
  for (int j = 0; j < W128_DEC_SLOTS; ++j) asm volatile("" : "+v"(pi[j]), "+v"(pv[j]));

  int vbits = 30;
  for (int w = 1; w < W; w <<= 1) --vbits;                     // 30 - ceil(log2 W)
  const int lrow = tid >> 5, lcol = (tid & 31) * 4;
  const uint32_t dummy = (uint32_t)((tid & 127) * W128_LDX + 128 + ((tid >> 7) & 3));   // pad slot of this thread

  for (;;) {
    mask_payload(0);
    const int cc = chunk - t_first;
    const uint32_t ucols = (uint32_t)d.cols;
    const int64_t origin = (int64_t)(cc / d.cchunks) * 128 * d.cols + (int64_t)(cc % d.cchunks) * 128;
    const __amdgpu_buffer_rsrc_t xres = PBF16 ? make_rsrc(static_cast<const uint16_t*>(d.param) + origin)
                                              : make_rsrc(static_cast<const float*>(d.param) + origin);
    const uint32_t vo = (uint32_t)lrow * ucols + (uint32_t)lcol;

    if constexpr (COUNT) {
      static_assert(!COUNT || !STREAM, "the count pass needs the whole payload in registers");
      // every pair adds one to its coefficient's slot, reads the total back and is divided by it (sum of val/n over
      // the n pairs of a slot = (sum of val) / n); the tile is zeroed again below before the sums go in
      auto slot_of = [&](int j) {
        const uint32_t fi = (uint32_t)pi[j];
        return fi < 16384u ? (uint32_t)(pos3(fi >> 7) * W128_LDX + pos3(fi & 127u)) : dummy;
      };
      for (int e = tid; e < W128_X_FLOATS / 4; e += W128_THREADS)
        *reinterpret_cast<f32x4*>(&tile[4 * e]) = (f32x4){0.f, 0.f, 0.f, 0.f};
      wg_lds_barrier();
#pragma unroll
      for (int j = 0; j < W128_DEC_SLOTS; ++j)
        if (j < nslots) atomicAdd(&itile[slot_of(j)], 1);
      wg_lds_barrier();
#pragma unroll
      for (int j = 0; j < W128_DEC_SLOTS; ++j)
        if (j < nslots) pv[j] = pv[j] / (float)itile[slot_of(j)];
      wg_lds_barrier();
    }
    // ---- largest |val| of the payload registers, zero tile ----------------------------------------------------
    // per-wavefront largest magnitude (as bits) of the payload registers into wmax buffer `buf`
    auto post_wave_max = [&](int buf) {
      float mx = 0.f;
#pragma unroll
      for (int j = 0; j < W128_DEC_SLOTS; ++j)
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
    // shift of the block fixed point from the sixteen posted maxima (after a barrier)
    auto shift_from = [&](int buf) {
      uint32_t mall = wmax[16 * buf + (lane & 15)];
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
      for (int j = 0; j < W128_DEC_SLOTS; ++j) {
        if (j < nslots) {
          const uint32_t fi = (uint32_t)pi[j];
          const uint32_t a = fi < 16384u ? (uint32_t)(pos3(fi >> 7) * W128_LDX + pos3(fi & 127u)) : dummy;
          atomicAdd(&itile[a], __float2int_rn(ldexpf(pv[j], sh)));
        }
      }
    };
    post_wave_max(0);
    for (int e = tid; e < W128_X_FLOATS / 4; e += W128_THREADS)
      *reinterpret_cast<f32x4*>(&tile[4 * e]) = (f32x4){0.f, 0.f, 0.f, 0.f};
    wg_lds_barrier();

    // ---- S[idx] += val in fixed point ------------------------------------------------------------------------
    int sh_chunk = shift_from(0);   // shift of this chunk's fixed point (undone when phi is the identity)
    add_pairs(sh_chunk);
    if constexpr (STREAM) {
      // one pass over the payload: the registers held round 0; every further round is added with the block
      // exponent of the largest magnitude seen so far, and when a round raises that exponent the sums in the tile
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
          for (int e = tid; e < W128_X_FLOATS / 4; e += W128_THREADS) {
            int4 v = *reinterpret_cast<int4*>(&itile[4 * e]);
            v.x = (v.x + half + ((v.x >> dsh) & 1)) >> dsh;
            v.y = (v.y + half + ((v.y >> dsh) & 1)) >> dsh;
            v.z = (v.z + half + ((v.z >> dsh) & 1)) >> dsh;
            v.w = (v.w + half + ((v.w >> dsh) & 1)) >> dsh;
            *reinterpret_cast<int4*>(&itile[4 * e]) = v;
          }
          wg_lds_barrier();
          sh_chunk = sh_r;
        }
        add_pairs(sh_chunk);
      }
    }
    // ---- payload of the next chunk, in flight during the products ----------------------------------------------
    const int nxt = chunk + (int)gridDim.x;
    if (nxt < total) {
      while (nxt >= t_next) {
        ++t;
        t_first = t_next;
        t_next = uniform_prefix(tv, t + 1);
        d = load_desc_uniform(tv, t);
      }
      load_payload(d, nxt - t_first, 0);
    }
    wg_lds_barrier();

    // ---- product a: Y[i][v] = sum_u P[u][i] S[u][v]; the wavefront owns column tile nt = wave % 8 and the
    //      quadruple bases i = 16 h + m, h = wave / 8; accumulators E0, E2, Oa, Ob ---------------------------------
    f32x4 acc[4];
    {
      const int nt = wave & 7, h = wave >> 3;
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
      const float* pa = sPT + (16 * h + l16) * W128_LDX + 4 * lq;           // P[u][i]
      const float* pm = sPT + (63 - 16 * h - l16) * W128_LDX + 4 * lq;      // P[u][63 - i]
      const int* sb = itile + 4 * lq * W128_LDX + 16 * nt + l16;
#pragma unroll
      for (int kg = 0; kg < 4; ++kg) {   // kg = 0, 1: u = 0 mod 4;  kg = 2, 3: u = 2 mod 4
        float b[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) b[s] = (float)sb[(16 * kg + s) * W128_LDX];
        const f32x4 a = *reinterpret_cast<const f32x4*>(pa + 16 * kg);
#pragma unroll
        for (int s = 0; s < 4; ++s) acc[kg >> 1] = mfma4(a[s], b[s], acc[kg >> 1]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kg = 0; kg < 4; ++kg) {   // odd u
        float b[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) b[s] = (float)sb[(64 + 16 * kg + s) * W128_LDX];
        const f32x4 a = *reinterpret_cast<const f32x4*>(pa + 64 + 16 * kg);
        const f32x4 am = *reinterpret_cast<const f32x4*>(pm + 64 + 16 * kg);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          acc[2] = mfma4(a[s], b[s], acc[2]);
          acc[3] = mfma4(am[s], b[s], acc[3]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      wg_lds_barrier();   // every read of S is done: Y replaces it (rows in natural order, columns as they were)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int i = 16 * h + 4 * lq + r;
        const float ep = acc[0][r] + acc[1][r], em = acc[0][r] - acc[1][r];
        float* col = tile + 16 * nt + l16;
        col[i * W128_LDX] = ep + acc[2][r];
        col[(127 - i) * W128_LDX] = ep - acc[2][r];
        col[(63 - i) * W128_LDX] = em + acc[3][r];
        col[(64 + i) * W128_LDX] = em - acc[3][r];
      }
    }
    wg_lds_barrier();

    // ---- the parameters of this chunk: requested now, used after product b -----------------------------------
    using XT = typename std::conditional<PBF16, u32x2, f32x4>::type;
    XT xin[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      if constexpr (PBF16) xin[p] = bload_u2(xres, vo * 2, 32u * p * ucols * 2);
      else xin[p] = bload_f4(xres, vo * 4, 32u * p * ucols * 4);
    }

    // ---- product b: R[i][j] = sum_v Y[i][v] P[v][j]; the wavefront owns row tile it = wave / 2 and the quadruple
    //      bases j = 16 h + n, h = wave % 2; accumulators E0, E2, Oa, Ob ----------------------------------------------
    {
      const int it = wave >> 1, h = wave & 1;
#pragma unroll
      for (int i = 0; i < 4; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
      const float* ya = tile + (16 * it + l16) * W128_LDX + 4 * lq;
      const float* pb = sPT + (16 * h + l16) * W128_LDX + 4 * lq;            // P[v][j]
      const float* pm = sPT + (63 - 16 * h - l16) * W128_LDX + 4 * lq;       // P[v][63 - j]
#pragma unroll
      for (int kg = 0; kg < 4; ++kg) {   // kg = 0, 1: v = 0 mod 4;  kg = 2, 3: v = 2 mod 4
        const f32x4 a = *reinterpret_cast<const f32x4*>(ya + 16 * kg);
        const f32x4 b = *reinterpret_cast<const f32x4*>(pb + 16 * kg);
#pragma unroll
        for (int s = 0; s < 4; ++s) acc[kg >> 1] = mfma4(a[s], b[s], acc[kg >> 1]);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int kg = 0; kg < 4; ++kg) {   // odd v
        const f32x4 a = *reinterpret_cast<const f32x4*>(ya + 64 + 16 * kg);
        const f32x4 b = *reinterpret_cast<const f32x4*>(pb + 64 + 16 * kg);
        const f32x4 bm = *reinterpret_cast<const f32x4*>(pm + 64 + 16 * kg);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          acc[2] = mfma4(a[s], b[s], acc[2]);
          acc[3] = mfma4(a[s], bm[s], acc[3]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      wg_lds_barrier();   // every read of Y is done: R replaces it
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int j = 16 * h + l16;
        float* row = tile + (16 * it + 4 * lq + r) * W128_LDX;
        const float ep = acc[0][r] + acc[1][r], em = acc[0][r] - acc[1][r];
        row[j] = ep + acc[2][r];
        row[127 - j] = ep - acc[2][r];
        row[63 - j] = em + acc[3][r];
        row[64 + j] = em - acc[3][r];
      }
    }
    wg_lds_barrier();

    // ---- x <- x - lr (phi(R) + wd x): phi = sgn, or the identity on the aggregate (the tile holds R * 2^sh; `scale`
    //      is 1 or 1/W) -----------------------------------------------------------------------------------------------
    const float factor = IDENT ? ldexpf(args.scale, -sh_chunk) : 0.f;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
      const f32x4 rv = *reinterpret_cast<const f32x4*>(&tile[(lrow + 32 * p) * W128_LDX + lcol]);
      float o[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        float x;
        if constexpr (PBF16) {
          const uint32_t raw = xin[p][e >> 1];
          x = __uint_as_float((e & 1) ? (raw & 0xffff0000u) : (raw << 16));
        } else {
          x = xin[p][e];
        }
        o[e] = sign_update(x, IDENT ? rv[e] * factor : sgnf(rv[e]), args.lr, args.weight_decay);
      }
      if constexpr (PBF16) {
        const u32x2 pk = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
        bstore_u2(xres, vo * 2, 32u * p * ucols * 2, pk);
      } else {
        const f32x4 ov = {o[0], o[1], o[2], o[3]};
        bstore_f4(xres, vo * 4, 32u * p * ucols * 4, ov);
      }
    }
    if (nxt >= total) break;
    chunk = nxt;
    wg_lds_barrier();   // the tile is zeroed next
  }
}

template <bool PBF16, bool STREAM, bool IDENT, bool COUNT = false>
static hipError_t launch_dec_wg128_phi(const TableView& tv, const float* basis, const DecodeArgs& a, int64_t grid,
                                       hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode2d_wg128<PBF16, STREAM, IDENT, COUNT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, W128_DEC_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((decode2d_wg128<PBF16, STREAM, IDENT, COUNT>), dim3((unsigned)grid), dim3(W128_THREADS),
                     W128_DEC_LDS_BYTES, stream, tv, basis, a);
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

hipError_t launch_decode2d_wg128(const TableView& tv, const float* basis, const DecodeArgs& a, bool param_bf16,
                                 int num_cus, hipStream_t stream) {
  if (!fast128_decode_supports(a.W, a.k, (tv.dtypes & 16u) == 0)) return hipErrorInvalidValue;
  if (a.agg == 2 && (int64_t)a.W * a.k > kFast128MaxPairs) return hipErrorInvalidValue;   // counted from registers
  int64_t grid = num_cus;
  if (grid > tv.total_chunks) grid = tv.total_chunks;
  if ((int64_t)a.W * a.k > kFast128MaxPairs)
    return param_bf16 ? launch_dec_wg128<true, true>(tv, basis, a, grid, stream)
                      : launch_dec_wg128<false, true>(tv, basis, a, grid, stream);
  return param_bf16 ? launch_dec_wg128<true, false>(tv, basis, a, grid, stream)
                    : launch_dec_wg128<false, false>(tv, basis, a, grid, stream);
}

}  // namespace demo

DEMO_PHASE_GETTER(demo_debug_phase_clocks_wg128)
