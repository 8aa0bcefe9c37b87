// s = 64 decode kernel: one wavefront per 64 x 64 chunk.
//
// Lane l = 16 g + c owns, for q = 0..15, the four consecutive parameters X[4q + g][4c .. 4c+3]
// (16 lanes cover one row of the chunk).  The coefficient sums S of the W payloads live in a
// private LDS tile; R = P^T (S P) runs as two chains of v_mfma_f32_16x16x4_f32 and lands in the
// register layout the parameters are loaded and stored with, so the sign update is fused.
#include "demo_device.h"

namespace demo {

// Host: basis tables of the decode kernel from the 64 x 64 basis P (double, row-major):
//   [0, 4096)     rows of P:                 plain[v*64 + j]      = P[v][j]
//   [4096, 8192)  rows of P, permuted:       perm[u*64 + 4c + m]  = P[u][16m + 4(c%4) + c/4]
void build_dec64_tables(const double* P, float* out) {
  for (int u = 0; u < 64; ++u)
    for (int j = 0; j < 64; ++j) out[u * 64 + j] = (float)P[u * 64 + j];
  for (int u = 0; u < 64; ++u)
    for (int cc = 0; cc < 16; ++cc)
      for (int mt = 0; mt < 4; ++mt)
        out[4096 + u * 64 + 4 * cc + mt] = (float)P[u * 64 + 16 * mt + 4 * (cc & 3) + (cc >> 2)];
}

// ---------------------------------------------------------------------------
// decode
// ---------------------------------------------------------------------------
// One wavefront per chunk.  The coefficient sums S live in a private LDS tile (row stride
// 68 floats); R = P^T (S P) runs as two MFMA chains:
//   product a   Y[u][j] = sum_v S[u][v] P[v][j]     A = S from LDS, B = rows of P
//   product b   R[i][j] = sum_u P[u][i] Y[u][j]     A = permuted rows of P, B = product-a accumulators
// and lands in the same register layout the parameters are loaded and stored with.
namespace {
constexpr int F64D_WAVES = 7;                       // 7 private tiles + the two basis tables fill the LDS
constexpr int F64D_THREADS = F64D_WAVES * 64;
constexpr int F64D_LDT = 68;
constexpr int F64D_TILE_FLOATS = 64 * F64D_LDT;
constexpr int F64D_LDS_BYTES = 4 * (2 * 4096 + F64D_WAVES * F64D_TILE_FLOATS);
}  // namespace

// PBF16: parameter dtype of every tensor in the table.  FULL: k == 32 and W a multiple of 64, so
// every payload load instruction is fully populated (two workers x 32 pairs) and needs no predicate.
template <bool PBF16, bool FULL>
__global__ __launch_bounds__(F64D_THREADS) void decode2d_wave64(TableView tv, const float* __restrict__ tables,
                                                                DecodeArgs args) {
  extern __shared__ float lds[];
  const float* sPplain = lds;
  const float* sPperm = lds + 4096;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, c = lane & 15;
  float* tile = lds + 2 * 4096 + wave * F64D_TILE_FLOATS;
  const int k = FULL ? 32 : args.k, W = args.W;

  for (int e = tid; e < 2 * 4096 / 4; e += F64D_THREADS)
    reinterpret_cast<float4*>(lds)[e] = reinterpret_cast<const float4*>(tables)[e];
  __syncthreads();

  const int nwaves = gridDim.x * F64D_WAVES;
  const int wid = blockIdx.x * F64D_WAVES + wave;
  const int total = tv.total_chunks;
  const int per = total / nwaves, rem = total - per * nwaves;
  int chunk = wid * per + (wid < rem ? wid : rem);
  const int chunk_end = chunk + per + (wid < rem ? 1 : 0);
  if (chunk >= chunk_end) return;

  // payload lanes: with k <= 32 one load instruction fetches the pairs of two workers
  const int wpi = (FULL || k <= 32) ? 2 : 1;             // workers per load instruction
  const int sub = wpi == 2 ? (lane >> 5) : 0;            // which of them this lane serves
  const int pt = wpi == 2 ? (lane & 31) : lane;          // pair index inside the chunk
  const bool pact = FULL || pt < k;
  const uint32_t dummy = (uint32_t)(lane * F64D_LDT + 64);   // a pad slot of this lane: absorbs masked-off additions
  constexpr int NLI = 32;                                // load instructions per group of workers
  int32_t pi[NLI];
  float pv[NLI];
  auto load_payload = [&](const TensorDev& dd, int ccc, int wbase) {
    // uniform 64-bit base per load instruction + one 32-bit per-lane offset
    const int64_t wstride = (int64_t)dd.nchunks * k;
    const uint32_t lane_off = (uint32_t)(sub * (int)wstride + pt);
    const DEMO_GLOBAL int32_t* ip = as_global(dd.idx) + (int64_t)ccc * k + (int64_t)wbase * wstride;
    const DEMO_GLOBAL float* vp = as_global(dd.val) + (int64_t)ccc * k + (int64_t)wbase * wstride;
#pragma unroll
    for (int j = 0; j < NLI; ++j) {
      if (FULL) {
        pi[j] = ip[lane_off];
        pv[j] = vp[lane_off];
      } else {
        const bool ok = pact && wbase + j * wpi + sub < W;
        pi[j] = ok ? ip[lane_off] : -1;
        pv[j] = ok ? vp[lane_off] : 0.f;
      }
      ip += wpi * wstride;
      vp += wpi * wstride;
    }
  };
  // S[idx] += val in block fixed point.  LDS float atomics are an order of magnitude slower than
  // integer ones on this part, and an integer sum does not depend on the order of arrival, so the
  // coefficients are scaled by a power of two taken from the largest magnitude of the chunk's
  // payload (exact), rounded to integers of `vbits` bits and added with ds_add_u32; W such
  // values cannot overflow 31 bits.  Only sgn(IDCT(S)) is used, so the scale is never undone.
  // Lanes with nothing to add (inactive pair, index out of range) add zero into their pad slot.
  int* itile = reinterpret_cast<int*>(tile);
  int vbits = 30;
  for (int w = 1; w < W; w <<= 1) --vbits;                // 30 - ceil(log2 W)
  auto scatter = [&]() {
    float mx = 0.f;
#pragma unroll
    for (int j = 0; j < NLI; ++j) mx = fmaxf(mx, fabsf(pv[j]));
    uint32_t mb = __float_as_uint(mx);
    mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0xB1, 0xf, 0xf, false));   // quad_perm [1,0,3,2]
    mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x4E, 0xf, 0xf, false));   // quad_perm [2,3,0,1]
    mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x141, 0xf, 0xf, false));  // row_half_mirror
    mb = max(mb, (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mb, 0x140, 0xf, 0xf, false));  // row_mirror
    const uint32_t m01 = max((uint32_t)__builtin_amdgcn_readlane((int)mb, 0), (uint32_t)__builtin_amdgcn_readlane((int)mb, 16));
    const uint32_t m23 = max((uint32_t)__builtin_amdgcn_readlane((int)mb, 32), (uint32_t)__builtin_amdgcn_readlane((int)mb, 48));
    int ex = (int)(max(m01, m23) >> 23);                  // biased exponent of the largest magnitude
    ex = ex < 1 ? 1 : ex;
    const int sh = vbits + 126 - ex;                      // max |val| * 2^sh < 2^vbits
#pragma unroll
    for (int j = 0; j < NLI; ++j) {
      const uint32_t u = (uint32_t)pi[j];
      const uint32_t a = u < 4096u ? u + ((u >> 6) << 2) : dummy;   // (u / 64) * 68 + u % 64
      const int q = __float2int_rn(ldexpf(pv[j], sh));
      atomicAdd(&itile[a], q);
    }
  };

  int t = find_tensor(tv.prefix, tv.n, chunk);
  int t_first = tv.prefix[t], t_next = tv.prefix[t + 1];
  TensorDev d = tv.descs[t];
  load_payload(d, chunk - t_first, 0);
  DEMO_PHASE_DECL

  for (; chunk < chunk_end; ++chunk) {
    const int cc = chunk - t_first;
    const int k0 = cc / d.cchunks, k1 = cc - k0 * d.cchunks;
    const int64_t base = (int64_t)k0 * 64 * d.cols + (int64_t)k1 * 64 + (int64_t)g * d.cols + 4 * c;
    const TensorDev dcur = d;
    DEMO_PHASE(0);

    // ---- S = sum over workers ---------------------------------------------------------------------------
#pragma unroll
    for (int i = 0; i < 17; ++i) *reinterpret_cast<float4*>(&tile[(i * 64 + lane) * 4]) = make_float4(0.f, 0.f, 0.f, 0.f);
    wave_lds_sync();
    scatter();   // the launch wrapper guarantees that one group of NLI load instructions holds all W workers
    DEMO_PHASE(1);
    // ---- payload of the next chunk, in flight during the products -----------------------------------------
    if (chunk + 1 < chunk_end) {
      while (chunk + 1 >= t_next) {
        ++t;
        t_first = t_next;
        t_next = tv.prefix[t + 1];
        d = tv.descs[t];
      }
      load_payload(d, chunk + 1 - t_first, 0);
    }
    wave_lds_sync();

    DEMO_PHASE(2);
    // ---- product a: Ya[mt][e] (rows u = 16mt+4g+r, cols j = 4c+e) --------------------------------------
    // k-step 4kg + kr contracts v = 16kg + 4g + kr: four k-steps per 16-byte LDS read of S.
    // Operands of the next k-step are read while the MFMAs of the current one run.
    f32x4 Ya[4][4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int e = 0; e < 4; ++e) Ya[mt][e] = (f32x4){0.f, 0.f, 0.f, 0.f};
    {
      float4 sa[4], sn[4];
#pragma unroll
      for (int mt = 0; mt < 4; ++mt) sn[mt] = *reinterpret_cast<const float4*>(&tile[(16 * mt + c) * F64D_LDT + 4 * g]);
      float4 pn = *reinterpret_cast<const float4*>(&sPplain[(4 * g) * 64 + 4 * c]);
#pragma unroll
      for (int ks = 0; ks < 16; ++ks) {
        const int kg = ks >> 2, kr = ks & 3;
        if (kr == 0) {
#pragma unroll
          for (int mt = 0; mt < 4; ++mt) sa[mt] = sn[mt];
          if (kg + 1 < 4) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
              sn[mt] = *reinterpret_cast<const float4*>(&tile[(16 * mt + c) * F64D_LDT + 16 * (kg + 1) + 4 * g]);
          }
        }
        const float bf[4] = {pn.x, pn.y, pn.z, pn.w};
        if (ks + 1 < 16) {
          const int kg2 = (ks + 1) >> 2, kr2 = (ks + 1) & 3;
          pn = *reinterpret_cast<const float4*>(&sPplain[(16 * kg2 + 4 * g + kr2) * 64 + 4 * c]);
        }
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          const float ai = kr == 0 ? sa[mt].x : kr == 1 ? sa[mt].y : kr == 2 ? sa[mt].z : sa[mt].w;
          const float a = (float)__float_as_int(ai);      // the tile holds fixed-point sums
#pragma unroll
          for (int e = 0; e < 4; ++e) Ya[mt][e] = mfma4(a, bf[e], Ya[mt][e]);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    DEMO_PHASE(3);
    // ---- product b: R[mt'][e] component r' = element (row 4(4mt'+r')+g, col 4c+e) --------------------------
    f32x4 R[4][4];
    u32x2 Xh[16];   // bf16 parameters, raw
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int e = 0; e < 4; ++e) R[mt][e] = (f32x4){0.f, 0.f, 0.f, 0.f};
    {
      float4 pn = *reinterpret_cast<const float4*>(&sPperm[(4 * g) * 64 + 4 * c]);
#pragma unroll
      for (int mr = 0; mr < 16; ++mr) {
        const int mt = mr >> 2, r = mr & 3;
        const float af[4] = {pn.x, pn.y, pn.z, pn.w};
        if (mr + 1 < 16) {
          const int mt2 = (mr + 1) >> 2, r2 = (mr + 1) & 3;
          pn = *reinterpret_cast<const float4*>(&sPperm[(16 * mt2 + 4 * g + r2) * 64 + 4 * c]);
        }
#pragma unroll
        for (int m2 = 0; m2 < 4; ++m2)
#pragma unroll
          for (int e = 0; e < 4; ++e) R[m2][e] = mfma4(af[m2], Ya[mt][e][r], R[m2][e]);
        if (PBF16 && r == 3) {
          // a quarter of the product-a accumulators is dead: use the registers for the parameters
          const uint16_t* xp = static_cast<const uint16_t*>(dcur.param) + base;
#pragma unroll
          for (int q = 4 * mt; q < 4 * mt + 4; ++q) Xh[q] = gload_u2(xp + (int64_t)(4 * q) * dcur.cols);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    DEMO_PHASE(4);
    // ---- x <- x - lr*(sgn(R) + wd*x) ---------------------------------------------------------------------
    if (PBF16) {
      uint16_t* xp = static_cast<uint16_t*>(dcur.param) + base;
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const float x[4] = {__uint_as_float(Xh[q][0] << 16), __uint_as_float(Xh[q][0] & 0xffff0000u),
                            __uint_as_float(Xh[q][1] << 16), __uint_as_float(Xh[q][1] & 0xffff0000u)};
        float o[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = sign_update(x[e], sgnf(R[q >> 2][e][q & 3]), args.lr, args.weight_decay);
        const u32x2 pk = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3])};
        gstore_u2(xp + (int64_t)(4 * q) * dcur.cols, pk);
      }
    } else {
      // fp32 parameters are read here, four rows at a time, to stay inside the register budget
      float* xp = static_cast<float*>(dcur.param) + base;
#pragma unroll
      for (int qb = 0; qb < 16; qb += 4) {
        f32x4 xin[4];
#pragma unroll
        for (int q = qb; q < qb + 4; ++q) xin[q - qb] = gload_f4(xp + (int64_t)(4 * q) * dcur.cols);
#pragma unroll
        for (int q = qb; q < qb + 4; ++q) {
          f32x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e)
            o[e] = sign_update(xin[q - qb][e], sgnf(R[q >> 2][e][q & 3]), args.lr, args.weight_decay);
          gstore_f4(xp + (int64_t)(4 * q) * dcur.cols, o);
        }
      }
    }
    wave_lds_sync();
    DEMO_PHASE(5);
  }
  DEMO_PHASE_FLUSH(8);
}

template <bool PBF16, bool FULL>
static hipError_t launch_dec_wave64(const TableView& tv, const float* tables, const DecodeArgs& a, int64_t grid,
                                    hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode2d_wave64<PBF16, FULL>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, F64D_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((decode2d_wave64<PBF16, FULL>), dim3((unsigned)grid), dim3(F64D_THREADS), F64D_LDS_BYTES, stream,
                     tv, tables, a);
  return hipGetLastError();
}

hipError_t launch_decode2d_wave64(const TableView& tv, const float* tables, const DecodeArgs& a, bool param_bf16,
                                  int num_cus, hipStream_t stream) {
  int64_t grid = num_cus;
  const int64_t max_grid = ((int64_t)tv.total_chunks + F64D_WAVES - 1) / F64D_WAVES;
  if (grid > max_grid) grid = max_grid;
  const bool full = a.k == 32 && a.W == 64;
  if (param_bf16)
    return full ? launch_dec_wave64<true, true>(tv, tables, a, grid, stream)
                : launch_dec_wave64<true, false>(tv, tables, a, grid, stream);
  return full ? launch_dec_wave64<false, true>(tv, tables, a, grid, stream)
              : launch_dec_wave64<false, false>(tv, tables, a, grid, stream);
}

}  // namespace demo

DEMO_PHASE_GETTER(demo_debug_phase_clocks_dec)
