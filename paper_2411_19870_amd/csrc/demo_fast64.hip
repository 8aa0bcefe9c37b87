// s = 64 kernels with one wavefront per 64 x 64 chunk, everything register resident.
//
// A wavefront owns a whole chunk: lane l = 16 g + c loads, for q = 0..15, the four
// consecutive floats B[4q + g][4c .. 4c+3] (16 lanes cover one 256-byte row), so a lane
// holds 64 elements D[q][e].  The 2-D DCT  Q = P B P^T  runs as two chains of
// v_mfma_f32_16x16x4_f32 whose data operands never leave the register file:
//
//   product 1   T^T[j][u] = sum_i B[i][j] P[u][i]      A = D (as loaded), B = basis fragments
//   product 2   Q^T[v][u] = sum_j P[v][j] T^T[j][u]    A = basis fragments, B = product-1 accumulators
//
// (an accumulator tile holds rows 4g + r in lane group g, which is exactly the k-slot
// layout of a B operand, so the accumulators of product 1 feed product 2 directly; the
// permutation of the summation index this implies is baked into the basis fragment
// tables).  Top-k runs inside the wavefront on the 64 coefficients each lane holds, and
// the reconstruction  m - P^T Q^ P  is one more MFMA chain of contraction length k that
// accumulates straight into D, which is then stored with the same coalesced pattern.
// LDS only holds the basis fragment tables and a small per-wavefront candidate list.
#include "demo_device.h"

namespace demo {

#ifdef DEMO_PHASE_CLOCKS
__device__ unsigned long long demo_phase_clocks[16];
extern "C" int demo_debug_phase_clocks(unsigned long long* out16, int reset) {
  hipError_t e = hipMemcpyFromSymbol(out16, HIP_SYMBOL(demo_phase_clocks), 16 * sizeof(unsigned long long));
  if (e == hipSuccess && reset) {
    unsigned long long z[16] = {};
    e = hipMemcpyToSymbol(HIP_SYMBOL(demo_phase_clocks), z, sizeof(z));
  }
  return e == hipSuccess ? 0 : -4;
}
#endif

namespace {

constexpr int F64_WAVES = 8;                      // wavefronts per workgroup (2 per SIMD)
constexpr int F64_THREADS = F64_WAVES * 64;
constexpr int F64_CAP = 128;                      // candidate list capacity per wavefront
constexpr int F64_TABLE_FLOATS = 4 * 4096;        // T1 | T2 | Pplain | Pperm
// per-wavefront scratch: candidates {mag, flat} as uint2 [CAP], values [CAP], selected {flat, val} [64]
constexpr int F64_SCRATCH_WORDS = 2 * F64_CAP + F64_CAP + 2 * 64;
constexpr int F64_LDS_BYTES = 4 * (F64_TABLE_FLOATS + F64_WAVES * F64_SCRATCH_WORDS);

__device__ __forceinline__ f32x4 mfma4(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ void wave_lds_sync() {
  // LDS operations of one wavefront execute in order; this only stops the compiler
  // from moving LDS accesses across the point.
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// number of lanes below this one whose bit is set in mask
__device__ __forceinline__ int lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

}  // namespace

// Host: fragment tables for the kernels below from the 64 x 64 basis P (double, row-major).
void build_fast64_tables(const double* P, float* out) {
  float* t1 = out;
  float* t2 = out + 4096;
  float* pplain = out + 2 * 4096;
  float* pperm = out + 3 * 4096;
  for (int lane = 0; lane < 64; ++lane) {
    const int g = lane >> 4, c = lane & 15;
    for (int q = 0; q < 16; ++q)
      for (int nt = 0; nt < 4; ++nt) t1[(q * 64 + lane) * 4 + nt] = (float)P[(16 * nt + c) * 64 + 4 * q + g];
    for (int e = 0; e < 4; ++e)
      for (int r = 0; r < 4; ++r)
        for (int mt = 0; mt < 4; ++mt)
          t2[((e * 4 + r) * 64 + lane) * 4 + mt] = (float)P[(16 * mt + c) * 64 + 4 * (4 * g + r) + e];
  }
  for (int u = 0; u < 64; ++u)
    for (int j = 0; j < 64; ++j) pplain[u * 64 + j] = (float)P[u * 64 + j];
  for (int u = 0; u < 64; ++u)
    for (int cc = 0; cc < 16; ++cc)
      for (int mt = 0; mt < 4; ++mt) pperm[u * 64 + 4 * cc + mt] = (float)P[u * 64 + 16 * mt + 4 * (cc & 3) + (cc >> 2)];
}

// ---------------------------------------------------------------------------
// encode
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(F64_THREADS) void encode2d_wave64(TableView tv, const float* __restrict__ tables,
                                                               EncodeArgs args, Worklist wl) {
  extern __shared__ float lds[];
  const float* sT1 = lds;
  const float* sT2 = lds + 4096;
  const float* sPplain = lds + 2 * 4096;
  const float* sPperm = lds + 3 * 4096;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, c = lane & 15;
  uint32_t* scratch = reinterpret_cast<uint32_t*>(lds + F64_TABLE_FLOATS) + wave * F64_SCRATCH_WORDS;
  uint2* cand_key = reinterpret_cast<uint2*>(scratch);                  // {magnitude bits, flat index}
  float* cand_val = reinterpret_cast<float*>(scratch + 2 * F64_CAP);
  uint2* sel = reinterpret_cast<uint2*>(scratch + 3 * F64_CAP);         // {flat index, value bits}, rank order
  const int k = args.k;
  const int kpad = (k + 3) & ~3;

  for (int e = tid; e < F64_TABLE_FLOATS / 4; e += F64_THREADS)
    reinterpret_cast<float4*>(lds)[e] = reinterpret_cast<const float4*>(tables)[e];
  __syncthreads();

  // contiguous range of chunks for this wavefront
  const int nwaves = gridDim.x * F64_WAVES;
  const int wid = blockIdx.x * F64_WAVES + wave;
  const int total = tv.total_chunks;
  const int per = total / nwaves, rem = total - per * nwaves;
  int chunk = wid * per + (wid < rem ? wid : rem);
  const int chunk_end = chunk + per + (wid < rem ? 1 : 0);
  if (chunk >= chunk_end) return;
  int t = find_tensor(tv.prefix, tv.n, chunk);
  int t_first = tv.prefix[t], t_next = tv.prefix[t + 1];
  TensorDev d = tv.descs[t];

  DEMO_PHASE_DECL
  for (; chunk < chunk_end; ++chunk) {
    while (chunk >= t_next) {
      ++t;
      t_first = t_next;
      t_next = tv.prefix[t + 1];
      d = tv.descs[t];
    }
    const int cc = chunk - t_first;
    const int k0 = cc / d.cchunks, k1 = cc - k0 * d.cchunks;
    const int64_t base = (int64_t)k0 * 64 * d.cols + (int64_t)k1 * 64 + (int64_t)g * d.cols + 4 * c;

    // ---- load and momentum update: D[mt][e][r] = element (row 4(4mt+r)+g, col 4c+e) -----------
    f32x4 D[4][4];
    if (d.grad_bf16) {
      const uint16_t* gp = static_cast<const uint16_t*>(d.grad) + base;
      const float* mp = d.mom + base;
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int64_t ro = (int64_t)(4 * q) * d.cols;
        const u32x2 gr = gload_u2(gp + ro);
        const f32x4 mo = gload_f4(mp + ro);
        D[q >> 2][0][q & 3] = __fmaf_rn(args.beta, mo[0], bf16_to_f32(gr[0] & 0xffffu));
        D[q >> 2][1][q & 3] = __fmaf_rn(args.beta, mo[1], bf16_to_f32(gr[0] >> 16));
        D[q >> 2][2][q & 3] = __fmaf_rn(args.beta, mo[2], bf16_to_f32(gr[1] & 0xffffu));
        D[q >> 2][3][q & 3] = __fmaf_rn(args.beta, mo[3], bf16_to_f32(gr[1] >> 16));
      }
    } else {
      const float* gp = static_cast<const float*>(d.grad) + base;
      const float* mp = d.mom + base;
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const int64_t ro = (int64_t)(4 * q) * d.cols;
        const f32x4 gr = gload_f4(gp + ro);
        const f32x4 mo = gload_f4(mp + ro);
#pragma unroll
        for (int e = 0; e < 4; ++e) D[q >> 2][e][q & 3] = __fmaf_rn(args.beta, mo[e], gr[e]);
      }
    }
    __builtin_amdgcn_sched_barrier(0);

    DEMO_PHASE(0);
    // ---- product 1: C1[e][nt] (rows j = 4(4g+r)+e, cols u = 16nt+c) ---------------------------
    f32x4 C1[4][4];
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) C1[e][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    {
      float4 pn = *reinterpret_cast<const float4*>(&sT1[lane * 4]);
#pragma unroll
      for (int q = 0; q < 16; ++q) {
        const float pf[4] = {pn.x, pn.y, pn.z, pn.w};
        if (q + 1 < 16) pn = *reinterpret_cast<const float4*>(&sT1[((q + 1) * 64 + lane) * 4]);
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
          for (int nt = 0; nt < 4; ++nt) C1[e][nt] = mfma4(D[q >> 2][e][q & 3], pf[nt], C1[e][nt]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    DEMO_PHASE(1);
    // ---- product 2: C2[mt][nt] (rows v = 16mt+4g+r, cols u = 16nt+c) = Q[u][v] -----------------
    f32x4 C2[4][4];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) C2[mt][nt] = (f32x4){0.f, 0.f, 0.f, 0.f};
    {
      float4 pn = *reinterpret_cast<const float4*>(&sT2[lane * 4]);
#pragma unroll
      for (int er = 0; er < 16; ++er) {
        const int e = er >> 2, r = er & 3;
        const float pf[4] = {pn.x, pn.y, pn.z, pn.w};
        if (er + 1 < 16) pn = *reinterpret_cast<const float4*>(&sT2[((er + 1) * 64 + lane) * 4]);
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
          for (int nt = 0; nt < 4; ++nt) C2[mt][nt] = mfma4(pf[mt], C1[e][nt][r], C2[mt][nt]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }

    DEMO_PHASE(2);
    // ---- top-k inside the wavefront ------------------------------------------------------------
    // flat index of C2[mt][nt][r] in this lane: u*64 + v = (16nt+c)*64 + 16mt + 4g + r
    uint32_t flat0 = (uint32_t)(c * 64 + 4 * g);
    asm volatile("" : "+v"(flat0));   // keeps the 64 per-register indices from being hoisted out of the chunk loop
    // (1) k-th largest of the 64 per-lane maxima: a lower bound of the k-th largest overall
    float lmax = 0.f;
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int r = 0; r < 4; ++r) lmax = fmaxf(lmax, fabsf(C2[mt][nt][r]));
    const uint32_t lm = __float_as_uint(lmax);
    uint32_t thr = 0;
    for (int bit = 30; bit >= 0; --bit) {
      const uint32_t cand = thr | (1u << bit);
      if (__popcll(__ballot(lm >= cand)) >= k) thr = cand;
    }
    DEMO_PHASE(3);
    // (2) gather candidates |q| >= thr (one compare and one scalar branch per coefficient)
    int ncand = 0;
    {
      const float thr_f = __uint_as_float(thr);
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 4; ++nt)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const float q = C2[mt][nt][r];
            const bool is = fabsf(q) >= thr_f;
            const uint64_t mask = __ballot(is);
            if (mask != 0) {
              const int pos = ncand + lanes_below(mask);
              if (is && pos < F64_CAP) {
                cand_key[pos] = make_uint2(__float_as_uint(q) & 0x7fffffffu, flat0 + (uint32_t)(1024 * nt + 16 * mt + r));
                cand_val[pos] = q;
              }
              ncand += __popcll(mask);
            }
          }
    }
    if (ncand > F64_CAP) {
      // Many (near-)equal magnitudes at the threshold (an all-zero chunk is the common case).
      if (__ballot(lm != 0u) == 0) {
        // every coefficient is zero: the k lowest flat indices, zero values, momentum stays zero
        if (lane < k) {
          const int64_t po = (int64_t)cc * k + lane;
          as_global(d.idx)[po] = lane;
          as_global(d.val)[po] = 0.f;
        }
#pragma unroll
        for (int q = 0; q < 16; ++q) {
          const f32x4 o = {D[q >> 2][0][q & 3], D[q >> 2][1][q & 3], D[q >> 2][2][q & 3], D[q >> 2][3][q & 3]};
          gstore_f4(d.mom + base + (int64_t)(4 * q) * d.cols, o);
        }
      } else {
        // leave the chunk untouched and queue it for the exact generic kernel that runs next
        if (lane == 0) wl.list[atomicAdd(wl.count, 1)] = chunk;
      }
      continue;
    }
    DEMO_PHASE(4);
    // pad the list to an even count for the paired reads below
    if (lane == 0 && (ncand & 1)) cand_key[ncand] = make_uint2(0u, 0xffffffffu);
    wave_lds_sync();
    // (4) rank candidates (magnitude descending, flat index ascending); ranks < k are the payload
    for (int i = lane; i < ncand; i += 64) {
      const uint2 me = cand_key[i];
      int rank = 0;
      for (int j = 0; j < ncand; j += 2) {
        const uint4 o = *reinterpret_cast<const uint4*>(&cand_key[j]);
        rank += (o.x > me.x || (o.x == me.x && o.y < me.y)) ? 1 : 0;
        rank += (o.z > me.x || (o.z == me.x && o.w < me.y)) ? 1 : 0;
      }
      if (rank < k) {
        const float v = cand_val[i];
        const int64_t po = (int64_t)cc * k + rank;
        as_global(d.idx)[po] = (int32_t)me.y;
        as_global(d.val)[po] = v;
        sel[rank] = make_uint2(me.y, __float_as_uint(v));
      }
    }
    if (lane >= k && lane < kpad) sel[lane] = make_uint2(0u, 0u);
    wave_lds_sync();

    DEMO_PHASE(5);
    // ---- reconstruction accumulated into D: D -= sum_t val_t P[u_t][i] P[v_t][j] ----------------
    for (int ks = 0; ks < kpad / 4; ++ks) {
      const uint2 s = sel[4 * ks + g];
      const int u = (int)((s.x >> 6) & 63u), v = (int)(s.x & 63u);
      const float nv = -__uint_as_float(s.y);
      const float4 pa = *reinterpret_cast<const float4*>(&sPperm[u * 64 + 4 * c]);
      const float4 pb = *reinterpret_cast<const float4*>(&sPplain[v * 64 + 4 * c]);
      const float af[4] = {nv * pa.x, nv * pa.y, nv * pa.z, nv * pa.w};
      const float bf[4] = {pb.x, pb.y, pb.z, pb.w};
#pragma unroll
      for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int e = 0; e < 4; ++e) D[mt][e] = mfma4(af[mt], bf[e], D[mt][e]);
    }

    DEMO_PHASE(6);
    // ---- store the residual momentum -------------------------------------------------------------
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const f32x4 o = {D[q >> 2][0][q & 3], D[q >> 2][1][q & 3], D[q >> 2][2][q & 3], D[q >> 2][3][q & 3]};
      gstore_f4(d.mom + base + (int64_t)(4 * q) * d.cols, o);
    }
    wave_lds_sync();   // the lists are rewritten by the next chunk
    DEMO_PHASE(7);
  }
  DEMO_PHASE_FLUSH(0);
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
    reinterpret_cast<float4*>(lds)[e] = reinterpret_cast<const float4*>(tables + 2 * 4096)[e];
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

hipError_t launch_encode2d_wave64(const TableView& tv, const float* tables, const EncodeArgs& a, const Worklist& wl,
                                  int num_cus, hipStream_t stream) {
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&encode2d_wave64),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, F64_LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  int64_t grid = num_cus;
  const int64_t max_grid = ((int64_t)tv.total_chunks + F64_WAVES - 1) / F64_WAVES;
  if (grid > max_grid) grid = max_grid;
  hipLaunchKernelGGL(encode2d_wave64, dim3((unsigned)grid), dim3(F64_THREADS), F64_LDS_BYTES, stream, tv, tables, a, wl);
  return hipGetLastError();
}

}  // namespace demo
