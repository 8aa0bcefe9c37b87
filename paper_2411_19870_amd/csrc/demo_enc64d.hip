// s = 32 encode kernel: one wavefront per 64 x 64 tile = 2 x 2 chunks.
//
// Same ownership, register layout, prefetch and in-wavefront top-k as demo_enc64.hip.  The tile is transformed
// with the block-diagonal matrix diag(P32, P32), and the mirror symmetry of the 32-point DCT (even rows even,
// odd rows odd under i -> 31-i) halves both products once more: a mirror quadruple {i0, 31-i0, 32+i0, 63-i0}
// holds one pair of each block, the in-lane sums and differences of the pairs feed four MFMA chains -- one per
// class (block, parity) of 16 frequencies -- of contraction length 16 (64 MFMAs per product).  Top-k runs once
// per chunk on the 16 coefficients each lane holds of it, and the reconstruction accumulates, per class of the
// row frequency, the rows of the quadruple bases only (see demo_enc64.hip).
#include "demo_device.h"

namespace demo {

namespace {
constexpr int ED_WAVES = 8;
constexpr int ED_THREADS = ED_WAVES * 64;
constexpr int ED_CAP = 128;                       // candidate list capacity per wavefront
constexpr int ED_T1 = 0;                          // t1[(par*64 + lane)*4 + s] = P32[2c + par][4s + g]  (product 1, B operand)
constexpr int ED_T2 = 512;                        // t2[(par*64 + lane)*4 + s] = P32[2c + par][4g + s]  (product 2, A operand)
constexpr int ED_PCOL = 1024;                     // pcol[v*64 + 4c + e] = B[v][4 chi(c) + e]
constexpr int ED_PK = 1024 + 4096;                // pk[u*16 + c] = B[u][kappa(c)], u < 32 (= P32[u][kappa(c)]: reconstruction)
constexpr int ED_TABLE_FLOATS = 1024 + 4096 + 512;
constexpr int ED_SELCLS = 2 * 64;                 // selected coefficients per class (row block, parity of u): 2 chunks x k <= 64
constexpr int ED_SELMAX = 4 * ED_SELCLS;
// per-wavefront scratch: candidate value bits [LIST], candidate flat indices [LIST] (one gather step appends up to 64
// entries to a list of at most CAP), 64-bit sort keys [64], selected {position in tile, value bits} [SELMAX]
constexpr int ED_LIST = ED_CAP + 64 + 2;
constexpr int ED_SCRATCH_WORDS = 2 * ED_LIST + 2 * 64 + 2 * ED_SELMAX;
static_assert((2 * ED_LIST) % 4 == 0 && ED_SCRATCH_WORDS % 4 == 0 && ED_TABLE_FLOATS % 4 == 0, "16-byte aligned key array");
constexpr int ED_LDS_BYTES = 4 * (ED_TABLE_FLOATS + ED_WAVES * ED_SCRATCH_WORDS);
static_assert(ED_TABLE_FLOATS == kEnc64dTableFloats, "table size");
}  // namespace

// Host: fragment tables from a 64 x 64 basis B (double, row-major, rows = frequencies).
void build_enc64d_tables(const double* Bm, float* out) {
  auto Bf = [&](int u, int i) { return (float)Bm[u * 64 + i]; };
  for (int par = 0; par < 2; ++par)
    for (int lane = 0; lane < 64; ++lane) {
      const int g = lane >> 4, c = lane & 15;
      for (int s = 0; s < 4; ++s) {
        out[ED_T1 + (par * 64 + lane) * 4 + s] = Bf(2 * c + par, 4 * s + g);
        out[ED_T2 + (par * 64 + lane) * 4 + s] = Bf(2 * c + par, 4 * g + s);
      }
    }
  for (int u = 0; u < 64; ++u)
    for (int cc = 0; cc < 16; ++cc)
      for (int x = 0; x < 4; ++x) out[ED_PCOL + u * 64 + 4 * cc + x] = Bf(u, 4 * chi(cc) + x);
  for (int u = 0; u < 32; ++u)
    for (int cc = 0; cc < 16; ++cc) out[ED_PK + u * 16 + cc] = Bf(u, 4 * (cc & 3) + (cc >> 2));
}

// The table `tv` lists the order-2 tensors in units of 64 x 64 tiles (cchunks = cols / 64,
// nchunks = tiles); payload arrays are addressed per 32 x 32 chunk.
template <bool GBF16>
__global__ __launch_bounds__(ED_THREADS) void encode2d_tile32(TableView tv, const int32_t* __restrict__ prefix32,
                                                              const float* __restrict__ tables, EncodeArgs args,
                                                              Worklist wl) {
  extern __shared__ float lds[];
  const float* sT1 = lds + ED_T1;
  const float* sT2 = lds + ED_T2;
  const float* sPcol = lds + ED_PCOL;
  const float* sPk = lds + ED_PK;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, c = lane & 15;
  uint32_t* scratch = reinterpret_cast<uint32_t*>(lds + ED_TABLE_FLOATS) + wave * ED_SCRATCH_WORDS;
  uint32_t* cand_v = scratch;                                           // value bits of the candidates
  uint32_t* cand_f = scratch + ED_LIST;                                 // their flat indices in the chunk
  uint2* keys = reinterpret_cast<uint2*>(scratch + 2 * ED_LIST);        // {~flat index, magnitude bits}
  uint2* sel = reinterpret_cast<uint2*>(scratch + 2 * ED_LIST + 128);   // [4][SELCLS] {u*64 + tile column frequency, value bits} by class
  // LDS byte address of cand_v[0] as a scalar the compiler cannot take apart
  uint32_t list_base = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(uintptr_t)(lds_u32*)cand_v);
  asm volatile("" : "+s"(list_base));
  const int k = args.k;

  for (int e = tid; e < ED_TABLE_FLOATS / 4; e += ED_THREADS)
    reinterpret_cast<float4*>(lds)[e] = reinterpret_cast<const float4*>(tables)[e];
  __syncthreads();

  const int nwaves = gridDim.x * ED_WAVES;
  const int wid = first_work_item<DEMO_RUN>(wave);
  const int total = tv.total_chunks;
  int tileno = wid;   // wavefront w takes tiles w, w + nwaves, ...
  if (tileno >= total) return;
  int t = find_tensor_uniform(tv, tileno);
  int t_first = uniform_prefix(tv, t), t_next = uniform_prefix(tv, t + 1);
  TensorDev d = load_desc_uniform(tv, t);

  const int col4 = 4 * chi(c);

  struct Place {
    __amdgpu_buffer_rsrc_t mres, gres;
    uint32_t ucols, vo_up, vo_dn;   // elements
    int K0, K1, cch32;              // tile position, chunks per tensor row (32-grid)
    int tix;                        // tensor number
    int32_t* idx;
    float* val;
  };
  // (g, col4: the lane's row within a group of four and first column, passed in so that the tile loop can form them
  // on the spot instead of keeping them alive across its whole body)
  auto place = [&](const TensorDev& dd, int tt, int g, int col4) {
    const int k0 = tt / dd.cchunks, k1 = tt - k0 * dd.cchunks;
    const int64_t origin = (int64_t)k0 * 64 * dd.cols + (int64_t)k1 * 64;   // uniform
    Place p;
    p.ucols = (uint32_t)dd.cols;
    p.vo_up = (uint32_t)g * p.ucols + (uint32_t)col4;
    p.vo_dn = (uint32_t)(3 - g) * p.ucols + (uint32_t)col4;
    p.mres = make_rsrc(dd.mom + origin);
    p.gres = GBF16 ? make_rsrc(static_cast<const uint16_t*>(dd.grad) + origin)
                   : make_rsrc(static_cast<const float*>(dd.grad) + origin);
    p.K0 = k0;
    p.K1 = k1;
    p.cch32 = 2 * dd.cchunks;
    p.tix = t;
    p.idx = dd.idx;
    p.val = dd.val;
    return p;
  };

  f32x4 nm[16];
  u32x2 ng[16];    // bf16 gradients
  f32x4 ngf[16];   // fp32 gradients
  auto fetch_m = [&](const Place& p) {
#pragma unroll
    for (int q = 0; q < 16; ++q)
      nm[q] = bload_f4(p.mres, ((q & 1) ? p.vo_dn : p.vo_up) * 4, (uint32_t)rho_base(q) * p.ucols * 4);
  };
  auto fetch_g = [&](const Place& p) {
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      if (GBF16)
        ng[q] = bload_u2(p.gres, ((q & 1) ? p.vo_dn : p.vo_up) * 2, (uint32_t)rho_base(q) * p.ucols * 2);
      else
        ngf[q] = bload_f4(p.gres, ((q & 1) ? p.vo_dn : p.vo_up) * 4, (uint32_t)rho_base(q) * p.ucols * 4);
    }
  };

  Place cur = place(d, tileno - t_first, g, col4);
  fetch_m(cur);
  fetch_g(cur);
  // The first tile's rows are waited for here, outside the loop: the wait at the top of the body then only has
  // the back edge to serve, where the rows have the stores of the tile before behind them, and the compiler can
  // leave those stores in flight instead of waiting for their acknowledgement.
#pragma unroll
  for (int q = 0; q < 16; ++q) {
    asm volatile("" : "+v"(nm[q]));
    if (GBF16) asm volatile("" : "+v"(ng[q]));
    else asm volatile("" : "+v"(ngf[q]));
  }

  for (; tileno < total; tileno += nwaves) {
    const uint32_t ucols = cur.ucols, vo_up = cur.vo_up, vo_dn = cur.vo_dn;
    const __amdgpu_buffer_rsrc_t mres = cur.mres;
    Place nxt = cur;
    if (tileno + nwaves < total) {
      while (tileno + nwaves >= t_next) {
        ++t;
        t_first = t_next;
        t_next = uniform_prefix(tv, t + 1);
        d = load_desc_uniform(tv, t);
      }
      const int ln = fresh_lane_id();
      nxt = place(d, tileno + nwaves - t_first, ln >> 4, 4 * chi(ln & 15));
    }

    // ---- momentum update: D[s][e][w] = element (row rho(4s+w, g), col 4 chi(c) + e) ------------------
    f32x4 D[4][4];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      if (GBF16) {
        D[q >> 2][0][q & 3] = __fmaf_rn(args.beta, nm[q][0], args.grad_scale * __uint_as_float(ng[q][0] << 16));
        D[q >> 2][1][q & 3] = __fmaf_rn(args.beta, nm[q][1], args.grad_scale * __uint_as_float(ng[q][0] & 0xffff0000u));
        D[q >> 2][2][q & 3] = __fmaf_rn(args.beta, nm[q][2], args.grad_scale * __uint_as_float(ng[q][1] << 16));
        D[q >> 2][3][q & 3] = __fmaf_rn(args.beta, nm[q][3], args.grad_scale * __uint_as_float(ng[q][1] & 0xffff0000u));
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) D[q >> 2][e][q & 3] = __fmaf_rn(args.beta, nm[q][e], args.grad_scale * ngf[q][e]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- product 1: C1[e][tt] rows j = 4 chi(4g+r) + e, cols: frequency u = 2c + tt%2 of row block tt/2.
    //      k-slot g of step s contracts the pair base i0 = 4s + g: sums feed the even, differences the odd class.
    f32x4 C1[4][4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) C1[e][tt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    {
      const int ln = fresh_lane_id();
      const float4 pe4 = *reinterpret_cast<const float4*>(&sT1[(0 * 64 + ln) * 4]);
      const float4 po4 = *reinterpret_cast<const float4*>(&sT1[(1 * 64 + ln) * 4]);
      const float pe[4] = {pe4.x, pe4.y, pe4.z, pe4.w}, po[4] = {po4.x, po4.y, po4.z, po4.w};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float x0 = D[s][e][0], x1 = D[s][e][1], x2 = D[s][e][2], x3 = D[s][e][3];
          C1[e][0] = mfma4(x0 + x1, pe[s], C1[e][0]);
          C1[e][1] = mfma4(x0 - x1, po[s], C1[e][1]);
          C1[e][2] = mfma4(x2 + x3, pe[s], C1[e][2]);
          C1[e][3] = mfma4(x2 - x3, po[s], C1[e][3]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    // ---- product 2: C2[vt][tt] rows: frequency v = 2(4g + r) + vt%2 of column block vt/2, cols as above.
    //      The pair base j0 = 4g + s of the columns sits in registers (e, r) = (s,0), (3-s,1) | (s,2), (3-s,3).
    f32x4 C2[4][4];
#pragma unroll
    for (int vt = 0; vt < 4; ++vt)
#pragma unroll
      for (int tt = 0; tt < 4; ++tt) C2[vt][tt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    {
      const int ln = fresh_lane_id();
      const float4 pe4 = *reinterpret_cast<const float4*>(&sT2[(0 * 64 + ln) * 4]);
      const float4 po4 = *reinterpret_cast<const float4*>(&sT2[(1 * 64 + ln) * 4]);
      const float pe[4] = {pe4.x, pe4.y, pe4.z, pe4.w}, po[4] = {po4.x, po4.y, po4.z, po4.w};
#pragma unroll
      for (int s = 0; s < 4; ++s) {
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
          const float y0 = C1[s][tt][0], y1 = C1[3 - s][tt][1], y2 = C1[s][tt][2], y3 = C1[3 - s][tt][3];
          C2[0][tt] = mfma4(pe[s], y0 + y1, C2[0][tt]);
          C2[1][tt] = mfma4(po[s], y0 - y1, C2[1][tt]);
          C2[2][tt] = mfma4(pe[s], y2 + y3, C2[2][tt]);
          C2[3][tt] = mfma4(po[s], y2 - y3, C2[3][tt]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    // the next tile's momentum rows land while top-k, reconstruction and store of this one run
    fetch_m(nxt);
    __builtin_amdgcn_sched_barrier(0);

    // ---- top-k, once per chunk (bu, bv): coefficients C2[2bv + mh][2bu + nh][r] ---------------------------
    // the lane's number and the flat-index base of its coefficients, formed here for the four selections (flat index
    // inside a chunk of coefficient C2[vt][tt][r]: u*32 + v with u = 2c + tt%2, v = 2(4g + r) + vt%2)
    const int lt = fresh_lane_id();
    const uint32_t fbt = (uint32_t)(64 * (lt & 15) + 8 * (lt >> 4));
    bool skip = false;
    int ncls[4] = {0, 0, 0, 0};   // selected coefficients per class 2 bu + (u % 2) (uniform)
#pragma unroll
    for (int sub = 0; sub < 4; ++sub) {
      const int bu = sub >> 1, bv = sub & 1;
      // lower bound of the chunk's k-th largest magnitude: the k-th largest of the 64 per-lane maxima; for k > 32
      // of 128 maxima, two per lane (see demo_enc64.hip: with 64 maxima the list overflows for every chunk as k
      // approaches 64)
      float lmax0 = 0.f, lmax1 = 0.f;
#pragma unroll
      for (int nh = 0; nh < 2; ++nh)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          lmax0 = fmaxf(lmax0, fabsf(C2[2 * bv + 0][2 * bu + nh][r]));
          lmax1 = fmaxf(lmax1, fabsf(C2[2 * bv + 1][2 * bu + nh][r]));
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
      int ncand = 0;
      uint32_t list_end = list_base;   // scalar LDS byte address of the list's end
      {
        const float thr_f = __uint_as_float(thr);
#pragma unroll
        for (int mh = 0; mh < 2; ++mh)
#pragma unroll
          for (int nh = 0; nh < 2; ++nh)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const float q = C2[2 * bv + mh][2 * bu + nh][r];
              const bool is = fabsf(q) >= thr_f;
              const uint64_t mask = __ballot(is);
              if (mask != 0) {
                if (is && ncand <= ED_CAP) {   // a full list takes no more: slot < CAP + 64 without a per-lane clamp
                  lds_u32* slot = lds_u32_at(list_end + 4u * (uint32_t)lanes_below(mask));
                  slot[0] = __float_as_uint(q);
                  slot[ED_LIST] = fbt + (uint32_t)(32 * nh + mh + 2 * r);
                }
                const int hits = __popcll(mask);
                ncand += hits;
                list_end += 4u * (uint32_t)hits;
              }
            }
      }
      const bool overflow = ncand > ED_CAP;
      const bool all_zero = overflow && __ballot(lm != 0u) == 0;
      if (overflow && !all_zero) skip = true;   // near-ties en masse: the whole tile goes to the exact kernel
      const int c32 = (2 * cur.K0 + bu) * cur.cch32 + 2 * cur.K1 + bv;   // chunk number in the tensor
      wave_lds_sync();
      if (all_zero) {
        if (lt < k) {
          const int64_t po = (int64_t)c32 * k + lt;
          store_guarded(as_global(cur.idx) + po, (int32_t)lt);
          store_guarded(as_global(cur.val) + po, 0.f);
        }
      } else if (!overflow) {
        if (ncand > 64 && lt < ((8 - (ncand & 7)) & 7)) {   // padding for the eight-entry turns below
          cand_v[ncand + lt] = 0u;
          cand_f[ncand + lt] = 0xffffffffu;
        }
        if (ncand > 64) wave_lds_sync();
        // rank the candidates (magnitude descending, flat index ascending); ranks < k are the payload
        for (int i0 = 0; i0 < ncand; i0 += 64) {
          const int i = i0 + lt;
          const uint2 me = make_uint2(cand_v[i < ncand ? i : 0], cand_f[i < ncand ? i : 0]);
          const uint32_t mag = me.x & 0x7fffffffu;
          int rank = 0;
          if (ncand <= 64) {
            // the lanes put their 64-bit keys {magnitude, ~flat index} into LDS and every lane reads all of them back,
            // two per 16-byte read at a wavefront-uniform address (lanes past the list carry key 0, which precedes nothing)
            const uint32_t magl = i < ncand ? mag : 0u, nfl = i < ncand ? ~me.y : 0u;
            const uint64_t key = ((uint64_t)magl << 32) | nfl;
            keys[lt] = make_uint2(nfl, magl);
            wave_lds_sync();
            // sixteen keys per turn, all eight reads issued before the first comparison: a turn costs one LDS round
            // trip, and with four selections per tile the round trips of a four-key loop added up to a fifth of the
            // kernel's time at k = 32 (all 64 keys exist: lanes past the list wrote zeros)
            for (int j = 0; j < ncand; j += 16) {
              uint4 kk[8];
#pragma unroll
              for (int x = 0; x < 8; ++x) kk[x] = *reinterpret_cast<const uint4*>(&keys[j + 2 * x]);
#pragma unroll
              for (int x = 0; x < 8; ++x)
                rank += ((((uint64_t)kk[x].y << 32) | kk[x].x) > key ? 1 : 0) + ((((uint64_t)kk[x].w << 32) | kk[x].z) > key ? 1 : 0);
            }
          } else {
            // more candidates than lanes: against the whole list (padded below to a multiple of eight with entries
            // that precede nothing), eight entries per turn with all reads issued before the first comparison
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
                rank += (m0 > mag || (m0 == mag && of[x].x < me.y)) ? 1 : 0;
                rank += (m1 > mag || (m1 == mag && of[x].y < me.y)) ? 1 : 0;
              }
            }
          }
          const bool selected = i < ncand && rank < k;
          if (selected) {
            const int64_t po = (int64_t)c32 * k + rank;
            store_guarded(as_global(cur.idx) + po, (int32_t)me.y);
            store_guarded(as_global(cur.val) + po, __uint_as_float(me.x));
          }
          // filed for the reconstruction by class: {local row frequency u, column frequency 32 bv + v of the tile}
          const uint32_t u = me.y >> 5, v = me.y & 31u;
#pragma unroll
          for (int par = 0; par < 2; ++par) {
            const int q = 2 * bu + par;
            const uint64_t m = __ballot(selected && (int)(u & 1u) == par);
            if (selected && (int)(u & 1u) == par)
              sel[q * ED_SELCLS + ncls[q] + lanes_below(m)] = make_uint2(u * 64 + 32 * bv + v, me.x);
            ncls[q] += __popcll(m);
          }
        }
      }
      wave_lds_sync();
    }
    if (skip) {
      // leave the tile untouched (its payload entries are overwritten too) and queue its four chunks
      if (lt < 4) {
        const int c32 = (2 * cur.K0 + (lt >> 1)) * cur.cch32 + 2 * cur.K1 + (lt & 1);
        store_guarded(&wl.list[atomicAdd(wl.count, 1)], prefix32[cur.tix] + c32);   // chunk number in the 32-grid table
      }
    }
    if (GBF16) fetch_g(nxt);   // the coefficient registers are dead now (fp32 gradients: after the reconstruction)
    __builtin_amdgcn_sched_barrier(0);

    // ---- reconstruction on the quadruple bases: a term of chunk (bu, bv) with local row frequency u touches the
    //      rows of block bu only, and P32[u][31-i0] = +-P32[u][i0] by the parity of u, so each class (bu, parity)
    //      accumulates one 16-row tile per column tile (rows i0 = kappa(m)) and the two members of block bu follow:
    //        D[32 bu + i0] += R,  D[32 bu + 31 - i0] += R (u even) or -= R (u odd).
    //      The column side is the block-diagonal matrix as before (rows of B vanish outside their block).
#pragma unroll
    for (int q = 0; q < 4; ++q)   // pad every class list with zero-valued entries to a multiple of four
      if (lt < ((4 - (ncls[q] & 3)) & 3)) sel[q * ED_SELCLS + ncls[q] + lt] = make_uint2(0u, 0u);
    wave_lds_sync();
    if (!skip) {
      // the lane's place in the class lists is formed anew for every tile: kept across the tile loop the four list
      // addresses are spilled, and the reload of a spilled value waits for every load in flight, i.e. for the
      // rows of the next tile
      const int lane_now = fresh_lane_id();
      const int gl = lane_now >> 4, cl = lane_now & 15;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        f32x4 R[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) R[e] = (f32x4){0.f, 0.f, 0.f, 0.f};
        // A step's operands hang on two LDS reads in a row (the list entry, then the two basis rows it names).  The
        // loop runs two steps per turn on alternating registers, with the entry fetched two steps and the rows one
        // step ahead and scheduling fences around the MFMAs, so that no step waits for its own reads (at k = 32 a tile
        // has about 32 steps, and this kernel is bound by its own instructions; without the fences the compiler
        // sinks every read to its use)
        const int n = (ncls[q] + 3) >> 2;   // uniform
        if (n > 0) {
          struct Rows {
            float val, pk;
            float4 pb;
          };
          auto entry = [&](int step) { return sel[q * ED_SELCLS + 4 * min(step, n - 1) + gl]; };
          auto rows_of = [&](const uint2& sv) {
            return Rows{__uint_as_float(sv.y), sPk[((sv.x >> 6) & 31u) * 16 + cl],
                        *reinterpret_cast<const float4*>(&sPcol[(sv.x & 63u) * 64 + 4 * cl])};
          };
          auto accumulate = [&](const Rows& r) {
            const float a = -(args.alpha * r.val) * r.pk;
            R[0] = mfma4(a, r.pb.x, R[0]);
            R[1] = mfma4(a, r.pb.y, R[1]);
            R[2] = mfma4(a, r.pb.z, R[2]);
            R[3] = mfma4(a, r.pb.w, R[3]);
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
        const int w0 = 2 * (q >> 1);
#pragma unroll
        for (int sq = 0; sq < 4; ++sq)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            D[sq][e][w0] += R[e][sq];
            if (q & 1) D[sq][e][w0 + 1] -= R[e][sq];
            else D[sq][e][w0 + 1] += R[e][sq];
          }
      }
    }
    if (!GBF16) fetch_g(nxt);
    {
      // always issued, so that the number of stores behind the prefetched rows is fixed; a tile left to the exact
      // kernel stores through a buffer of zero records, which drops them
      const __amdgpu_buffer_rsrc_t sres = skip ? make_rsrc_empty(nullptr) : mres;
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const f32x4 o = {D[q >> 2][0][q & 3], D[q >> 2][1][q & 3], D[q >> 2][2][q & 3], D[q >> 2][3][q & 3]};
        bstore_f4(sres, ((q & 1) ? vo_dn : vo_up) * 4, (uint32_t)rho_base(q) * ucols * 4, o);
      }
    }
    wave_lds_sync();
    cur = nxt;
  }
}

template <bool GBF16>
static hipError_t launch_tile32(const TableView& tiles, const int32_t* prefix32, const float* tables,
                                const EncodeArgs& a, const Worklist& wl, int64_t grid, hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&encode2d_tile32<GBF16>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, ED_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(encode2d_tile32<GBF16>, dim3((unsigned)grid), dim3(ED_THREADS), ED_LDS_BYTES, stream, tiles,
                     prefix32, tables, a, wl);
  return hipGetLastError();
}

hipError_t launch_encode2d_tile32(const TableView& tiles, const int32_t* prefix32, const float* tables,
                                  const EncodeArgs& a, const Worklist& wl, bool grad_bf16, int num_cus,
                                  hipStream_t stream) {
  int64_t grid = num_cus;
  const int64_t max_grid = ((int64_t)tiles.total_chunks + DEMO_RUN - 1) / DEMO_RUN;   // few items: one run per workgroup, spread over the CUs
  if (grid > max_grid) grid = max_grid;
  return grad_bf16 ? launch_tile32<true>(tiles, prefix32, tables, a, wl, grid, stream)
                   : launch_tile32<false>(tiles, prefix32, tables, a, wl, grid, stream);
}

}  // namespace demo
