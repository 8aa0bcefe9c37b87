// HIP kernels (gfx950) for DeMo's per-step compression path.
//
// encode (worker side of Algorithm 1 / appendix CompressChunks), per chunk:
//     m <- beta*m + g ; Q = P B P^T ; keep the k largest |Q| ; m <- m - P^T Q^ P
// decode (server side / appendix Decompress&Aggregate + update line), per chunk:
//     S = sum_w payload_w ; R = P^T S P ; x <- x - lr*(sgn(R) + wd*x)
//
// This file holds the generic kernel family: one 256-thread workgroup per s x s
// chunk (s in {32,64,128}), tiles staged in LDS, all contractions on the fp32
// matrix cores (v_mfma_f32_16x16x4_f32), and one wavefront per order-1 chunk.
#include "demo_internal.h"
#include "demo_device.h"

namespace demo {

// ---------------------------------------------------------------------------
// Geometry of the generic order-2 kernels
// ---------------------------------------------------------------------------
constexpr int GEN_CAND_CAP = 512;   // candidate list of the generic encode kernel's top-k

template <int S>
struct Geo {
  static constexpr int NT = 256;                     // threads per workgroup (4 wavefronts)
  static constexpr int LD = S + 4;                   // LDS row stride in floats
  static constexpr int F4_PER_ROW = S / 4;
  static constexpr int ROWS_PER_PASS = NT / F4_PER_ROW;
  static constexpr int PASSES = S / ROWS_PER_PASS;   // float4 per thread
  static constexpr int TN = S / 16;                  // 16x16 tiles per dimension
  static constexpr int TPW = TN * TN / 4;            // tiles per wavefront
  static constexpr int CW = (TN >= 4) ? TN / 4 : 1;  // column tiles per wavefront (column strips when S >= 64)
  static constexpr bool INPLACE = (S >= 64);         // first product may overwrite its data operand
  static constexpr int M = S * S;
  static constexpr int TILE_FLOATS = S * LD;
  // LDS: basis, data tile, (second tile when not in place), selection scratch
  static constexpr int LDS_FLOATS = TILE_FLOATS * (INPLACE ? 2 : 3) + 3 * DEMO_MAXK_INTERNAL + 32 + 3 * GEN_CAND_CAP + 16;
};

// tile i of wavefront w -> (mt, nt)
template <int S>
__device__ __forceinline__ void tile_of(int w, int i, int& mt, int& nt) {
  using G = Geo<S>;
  if (G::TN >= 4) {
    nt = w * G::CW + (i % G::CW);
    mt = i / G::CW;
  } else {
    mt = w >> 1;
    nt = w & 1;
  }
}

// acc[i] (+)= A(rows of tile) * B(cols of tile), K = S, operands read from LDS.
//   a_at(m, kk) and b_at(kk, n) give the LDS float offsets of A[m][kk] and B[kk][n].
template <int S, class FA, class FB>
__device__ __forceinline__ void gemm_lds(f32x4* acc, int wave, int lane, const float* lds, FA a_at, FB b_at) {
  using G = Geo<S>;
  const int l16 = lane & 15, lq = lane >> 4;
#pragma unroll
  for (int i = 0; i < G::TPW; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
  for (int ks = 0; ks < S / 4; ++ks) {
    const int kk = 4 * ks + lq;
#pragma unroll
    for (int i = 0; i < G::TPW; ++i) {
      int mt, nt;
      tile_of<S>(wave, i, mt, nt);
      float a = lds[a_at(16 * mt + l16, kk)];
      float b = lds[b_at(kk, 16 * nt + l16)];
      acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[i], 0, 0, 0);
    }
  }
}

// Write a wavefront's accumulators (C layout: row 16mt + 4*(lane/16) + r, col 16nt + lane%16)
// to an LDS tile with row stride LD.
template <int S>
__device__ __forceinline__ void store_acc(const f32x4* acc, int wave, int lane, float* tile) {
  using G = Geo<S>;
  const int l16 = lane & 15, lq = lane >> 4;
#pragma unroll
  for (int i = 0; i < G::TPW; ++i) {
    int mt, nt;
    tile_of<S>(wave, i, mt, nt);
#pragma unroll
    for (int r = 0; r < 4; ++r) tile[(16 * mt + 4 * lq + r) * G::LD + 16 * nt + l16] = acc[i][r];
  }
}

// ---------------------------------------------------------------------------
// Mirror-folded products for the DCT (S >= 64).  Row u of the orthonormal DCT-II matrix is even (u even)
// or odd (u odd) under i -> S-1-i, so a product that contracts over i needs only i < S/2 on the folded
// operand x[i] +- x[S-1-i], and a product whose output index is i needs only i < S/2 of two partial
// sums (even u, odd u), the mirror outputs being their sum and difference: half the MFMAs either way.
// In these paths the basis tile in LDS holds the rows of P class-major: row u at position
// prow(u) = (u % 2) * S/2 + u / 2, so that the 16 rows of an operand tile are adjacent.
// ---------------------------------------------------------------------------
template <int S>
__device__ __forceinline__ int fold_pos(int u) { return (u & 1) * (S / 2) + (u >> 1); }   // row u -> class-major position
template <int S>
__device__ __forceinline__ int fold_idx(int p) { return 2 * (p & (S / 2 - 1)) + (p >= S / 2 ? 1 : 0); }   // inverse

// encode, first product: T[u][j] = sum_{i < S/2} P[u][i] (X[i][j] +- X[S-1-i][j]); tile (mt, nt) of the
// wavefront holds rows u = fold_idx(16 mt + m) (m-tiles below TN/2 are the even rows), columns 16 nt + n.
template <int S>
__device__ __forceinline__ void gemm_fold_enc1(f32x4* acc, int wave, int lane, const float* sP, const float* sX) {
  using G = Geo<S>;
  static_assert(G::TN >= 4, "folded products need S >= 64");
  const int l16 = lane & 15, lq = lane >> 4;
#pragma unroll
  for (int i = 0; i < G::TPW; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
  for (int ks = 0; ks < S / 8; ++ks) {
    const int kk = 4 * ks + lq;
    float be[G::CW], bo[G::CW];
#pragma unroll
    for (int j = 0; j < G::CW; ++j) {
      const int col = 16 * (wave * G::CW + j) + l16;
      const float x0 = sX[kk * G::LD + col], x1 = sX[(S - 1 - kk) * G::LD + col];
      be[j] = x0 + x1;
      bo[j] = x0 - x1;
    }
#pragma unroll
    for (int mt = 0; mt < G::TN; ++mt) {
      const float a = sP[(16 * mt + l16) * G::LD + kk];
#pragma unroll
      for (int j = 0; j < G::CW; ++j)
        acc[mt * G::CW + j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, mt >= G::TN / 2 ? bo[j] : be[j], acc[mt * G::CW + j], 0, 0, 0);
    }
  }
}
// rows of the accumulators above go to their natural places
template <int S>
__device__ __forceinline__ void store_fold_rows(const f32x4* acc, int wave, int lane, float* tile) {
  using G = Geo<S>;
  const int l16 = lane & 15, lq = lane >> 4;
#pragma unroll
  for (int i = 0; i < G::TPW; ++i) {
    int mt, nt;
    tile_of<S>(wave, i, mt, nt);
#pragma unroll
    for (int r = 0; r < 4; ++r) tile[fold_idx<S>(16 * mt + 4 * lq + r) * G::LD + 16 * nt + l16] = acc[i][r];
  }
}
// encode, second product: Q[u][v] = sum_{j < S/2} (T[u][j] +- T[u][S-1-j]) P[v][j]; tile (mt, nt) holds rows
// 16 mt + m and columns v = fold_idx(16 nt + n) (all n-tiles of a wavefront are of one class).
template <int S>
__device__ __forceinline__ void gemm_fold_enc2(f32x4* acc, int wave, int lane, const float* sP, const float* sT) {
  using G = Geo<S>;
  static_assert(G::TN >= 4, "folded products need S >= 64");
  const int l16 = lane & 15, lq = lane >> 4;
  const bool odd = wave * G::CW >= G::TN / 2;   // class of this wavefront's column tiles (uniform)
#pragma unroll
  for (int i = 0; i < G::TPW; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
  for (int ks = 0; ks < S / 8; ++ks) {
    const int kk = 4 * ks + lq;
    float b[G::CW];
#pragma unroll
    for (int j = 0; j < G::CW; ++j) b[j] = sP[(16 * (wave * G::CW + j) + l16) * G::LD + kk];
#pragma unroll
    for (int mt = 0; mt < G::TN; ++mt) {
      const float t0 = sT[(16 * mt + l16) * G::LD + kk], t1 = sT[(16 * mt + l16) * G::LD + S - 1 - kk];
      const float a = odd ? t0 - t1 : t0 + t1;
#pragma unroll
      for (int j = 0; j < G::CW; ++j)
        acc[mt * G::CW + j] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b[j], acc[mt * G::CW + j], 0, 0, 0);
    }
  }
}

// decode, first product: Y[i][v] for i < S/2 as two partial sums over even / odd u; the wavefront owns the
// column tiles of its strip (as tile_of), accumulator (2 mh + cls) * CW + j is rows 16 mh + m, class cls.
// Writes Y[i] = e + o and Y[S-1-i] = e - o (in place is safe: a wavefront reads only its own columns).
template <int S>
__device__ __forceinline__ void gemm_fold_dec1(f32x4* acc, int wave, int lane, const float* sP, const float* sS, float* sY) {
  using G = Geo<S>;
  static_assert(G::TN >= 4, "folded decode products need S >= 64");
  const int l16 = lane & 15, lq = lane >> 4;
#pragma unroll
  for (int i = 0; i < G::TPW; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
  for (int ks = 0; ks < S / 8; ++ks) {
    const int kk = 4 * ks + lq;
#pragma unroll
    for (int mh = 0; mh < G::TN / 2; ++mh)
#pragma unroll
      for (int cls = 0; cls < 2; ++cls)
#pragma unroll
        for (int j = 0; j < G::CW; ++j) {
          const int nt = wave * G::CW + j;
          const float a = sP[(cls * (S / 2) + kk) * G::LD + 16 * mh + l16];
          const float b = sS[(2 * kk + cls) * G::LD + 16 * nt + l16];
          f32x4& c = acc[(2 * mh + cls) * G::CW + j];
          c = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
        }
  }
#pragma unroll
  for (int mh = 0; mh < G::TN / 2; ++mh)
#pragma unroll
    for (int j = 0; j < G::CW; ++j) {
      const int nt = wave * G::CW + j;
      const f32x4 e = acc[(2 * mh) * G::CW + j], o = acc[(2 * mh + 1) * G::CW + j];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int i = 16 * mh + 4 * lq + r;
        sY[i * G::LD + 16 * nt + l16] = e[r] + o[r];
        sY[(S - 1 - i) * G::LD + 16 * nt + l16] = e[r] - o[r];
      }
    }
}
// decode, second product: R[i][j] for j < S/2 as two partial sums over even / odd v.  Folded column tile nh
// and the m-tiles of a wavefront: S = 128: nh = wave, all 8 m-tiles; S = 64: nh = wave % 2, m-tiles
// 2 (wave / 2) + {0, 1}.  Accumulator 2 ml + cls.  emit_fold_dec2 hands R[i][j] and R[i][S-1-j] to
// `emit(row, col, value)` (called after the barrier that ends the reads of Y).
template <int S>
__device__ __forceinline__ void gemm_fold_dec2(f32x4* acc, int wave, int lane, const float* sP, const float* sY) {
  using G = Geo<S>;
  static_assert(G::TN >= 4, "folded decode products need S >= 64");
  constexpr int NM = G::TPW / 2;                         // m-tiles per wavefront
  const int nh = S == 128 ? wave : (wave & 1);
  const int m0 = S == 128 ? 0 : 2 * (wave >> 1);
  const int l16 = lane & 15, lq = lane >> 4;
#pragma unroll
  for (int i = 0; i < G::TPW; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
  for (int ks = 0; ks < S / 8; ++ks) {
    const int kk = 4 * ks + lq;
#pragma unroll
    for (int ml = 0; ml < NM; ++ml)
#pragma unroll
      for (int cls = 0; cls < 2; ++cls) {
        const float a = sY[(16 * (m0 + ml) + l16) * G::LD + 2 * kk + cls];
        const float b = sP[(cls * (S / 2) + kk) * G::LD + 16 * nh + l16];
        acc[2 * ml + cls] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[2 * ml + cls], 0, 0, 0);
      }
  }
}
template <int S, class F>
__device__ __forceinline__ void emit_fold_dec2(const f32x4* acc, int wave, int lane, F emit) {
  using G = Geo<S>;
  constexpr int NM = G::TPW / 2;
  const int nh = S == 128 ? wave : (wave & 1);
  const int m0 = S == 128 ? 0 : 2 * (wave >> 1);
  const int l16 = lane & 15, lq = lane >> 4;
#pragma unroll
  for (int ml = 0; ml < NM; ++ml)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int i = 16 * (m0 + ml) + 4 * lq + r, j = 16 * nh + l16;
      emit(i, j, acc[2 * ml][r] + acc[2 * ml + 1][r]);
      emit(i, S - 1 - j, acc[2 * ml][r] - acc[2 * ml + 1][r]);
    }
}

// Tensor of a chunk for a workgroup that walks the chunks in ascending order: a step from the tensor
// of the previous chunk instead of a binary search (a chain of dependent loads) per chunk.  `st` holds
// {tensor, its first chunk, the next tensor's first chunk}; st.t < 0 before the first call.
struct TensorCursor {
  int t = -1, first = 0, next = 0;
};
__device__ __forceinline__ int tensor_of_chunk(const TableView& tv, int chunk, TensorCursor& st) {
  if (st.t < 0 || chunk < st.first) {
    st.t = find_tensor(tv.prefix, tv.n, chunk);
    st.first = tv.prefix[st.t];
    st.next = tv.prefix[st.t + 1];
  } else {
    while (chunk >= st.next) {
      ++st.t;
      st.first = st.next;
      st.next = tv.prefix[st.t + 1];
    }
  }
  return st.t;
}

// Workgroup-wide sum of a per-wavefront count (4 wavefronts).  `slot` must
// alternate between consecutive calls; one barrier per call.
__device__ __forceinline__ int block_sum4(int wave_count, int wave, int lane, int* s_cnt, int slot) {
  if (lane == 0) s_cnt[slot * 4 + wave] = wave_count;
  __syncthreads();
  return s_cnt[slot * 4 + 0] + s_cnt[slot * 4 + 1] + s_cnt[slot * 4 + 2] + s_cnt[slot * 4 + 3];
}

// ---------------------------------------------------------------------------
// encode, order-2 tensors, generic
// ---------------------------------------------------------------------------
// With a worklist (wl.list != nullptr) only the chunks queued there are processed, and the
// last workgroup to finish clears the queue for the next call.
// MIR: the projection matrix is the DCT and the two products are mirror-folded (instantiated for S = 128, where
// dense fp32 MFMA work is the bound; at S = 64 the extra registers cost more than the saved MFMAs).
template <int S, bool MIR>
__global__ __launch_bounds__(256) void encode2d_generic(TableView tv, const float* __restrict__ basis,
                                                        EncodeArgs args, Worklist wl) {
  using G = Geo<S>;
  extern __shared__ float lds[];
  float* sP = lds;                                     // basis P[u][n], stride LD
  float* sX = sP + G::TILE_FLOATS;                     // data tile / first product / reconstruction
  float* sT = G::INPLACE ? sX : sX + G::TILE_FLOATS;   // first product when not in place
  float* scratch = sX + G::TILE_FLOATS * (G::INPLACE ? 1 : 2);
  uint32_t* sel_mag = reinterpret_cast<uint32_t*>(scratch);            // [MAXK]
  int32_t* sel_idx = reinterpret_cast<int32_t*>(scratch + DEMO_MAXK_INTERNAL);
  float* sel_val = scratch + 2 * DEMO_MAXK_INTERNAL;
  int* s_cnt = reinterpret_cast<int*>(scratch + 3 * DEMO_MAXK_INTERNAL);  // [8] counters + [1] list cursor
  int* s_cursor = s_cnt + 8;
  uint2* cand_key = reinterpret_cast<uint2*>(scratch + 3 * DEMO_MAXK_INTERNAL + 32);   // [GEN_CAND_CAP + 8], 16-byte aligned
  float* cand_val = reinterpret_cast<float*>(cand_key + GEN_CAND_CAP + 8);              // [GEN_CAND_CAP]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l16 = lane & 15, lq = lane >> 4;
  const int k = args.k;
  const int kpad = (k + 3) & ~3;

  constexpr bool mir = MIR;
  const int nwork = wl.list != nullptr ? *wl.count : tv.total_chunks;
  if (nwork > 0)
    for (int e = tid; e < S * S; e += G::NT) sP[(mir ? fold_pos<S>(e / S) : e / S) * G::LD + (e % S)] = basis[e];

  DEMO_PHASE_DECL
  TensorCursor cur;
  for (int wi = blockIdx.x; wi < nwork; wi += gridDim.x) {
    const int chunk = wl.list != nullptr ? wl.list[wi] : wi;
    const int t = tensor_of_chunk(tv, chunk, cur);
    const TensorDev d = tv.descs[t];
    const int c = chunk - cur.first;
    const int k0 = c / d.cchunks, k1 = c - k0 * d.cchunks;
    const int64_t base = (int64_t)k0 * S * d.cols + (int64_t)k1 * S;

    // ---- load, momentum update, stage -------------------------------------------------
    float4 mid[G::PASSES];
    const int lrow = tid / G::F4_PER_ROW, lcol = (tid % G::F4_PER_ROW) * 4;
    __syncthreads();  // previous chunk's readers of sX are done
    // all loads of the chunk are issued before the first use (one dtype branch per chunk, not per load)
    {
      float4 mv[G::PASSES], gv[G::PASSES];
#pragma unroll
      for (int p = 0; p < G::PASSES; ++p)
        mv[p] = *reinterpret_cast<const float4*>(d.mom + base + (int64_t)(p * G::ROWS_PER_PASS + lrow) * d.cols + lcol);
      if (d.grad_bf16) {
        uint2 gh[G::PASSES];
#pragma unroll
        for (int p = 0; p < G::PASSES; ++p)
          gh[p] = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(d.grad) + base +
                                                  (int64_t)(p * G::ROWS_PER_PASS + lrow) * d.cols + lcol);
#pragma unroll
        for (int p = 0; p < G::PASSES; ++p)
          gv[p] = make_float4(bf16_to_f32(gh[p].x & 0xffffu), bf16_to_f32(gh[p].x >> 16), bf16_to_f32(gh[p].y & 0xffffu),
                              bf16_to_f32(gh[p].y >> 16));
      } else {
#pragma unroll
        for (int p = 0; p < G::PASSES; ++p)
          gv[p] = *reinterpret_cast<const float4*>(static_cast<const float*>(d.grad) + base +
                                                   (int64_t)(p * G::ROWS_PER_PASS + lrow) * d.cols + lcol);
      }
#pragma unroll
      for (int p = 0; p < G::PASSES; ++p) {
        const int row = p * G::ROWS_PER_PASS + lrow;
        float4 v;
        v.x = __fmaf_rn(args.beta, mv[p].x, args.grad_scale * gv[p].x);
        v.y = __fmaf_rn(args.beta, mv[p].y, args.grad_scale * gv[p].y);
        v.z = __fmaf_rn(args.beta, mv[p].z, args.grad_scale * gv[p].z);
        v.w = __fmaf_rn(args.beta, mv[p].w, args.grad_scale * gv[p].w);
        mid[p] = v;
        *reinterpret_cast<float4*>(&sX[row * G::LD + lcol]) = v;
      }
    }
    if (tid == 0) *s_cursor = 0;
    __syncthreads();
    DEMO_PHASE(0);

    // ---- T = P * X -----------------------------------------------------------------------
    f32x4 acc[G::TPW];
    if constexpr (MIR) {
      gemm_fold_enc1<S>(acc, wave, lane, sP, sX);
      store_fold_rows<S>(acc, wave, lane, sX);   // own column strip only: in place is safe
    } else {
      gemm_lds<S>(acc, wave, lane, lds,
                  [&](int m, int kk) { return m * G::LD + kk; },                              // P[u][i]
                  [&](int kk, int n) { return G::TILE_FLOATS + kk * G::LD + n; });           // X[i][j]
      // every read of this wavefront's column strip is its own: overwrite in place (S >= 64)
      store_acc<S>(acc, wave, lane, G::INPLACE ? sX : sT);
    }
    __syncthreads();

    DEMO_PHASE(1);
    // ---- Q = T * P^T ---------------------------------------------------------------------
    const int t_off = (int)(sT - lds);
    if constexpr (MIR) {
      gemm_fold_enc2<S>(acc, wave, lane, sP, sT);
    } else {
      gemm_lds<S>(acc, wave, lane, lds,
                  [&](int m, int kk) { return t_off + m * G::LD + kk; },                     // T[u][j]
                  [&](int kk, int n) { return n * G::LD + kk; });                             // P[v][j]
    }
    // column of coefficient tile nt held by this lane
    auto qcol = [&](int nt) { return mir ? fold_idx<S>(16 * nt + l16) : 16 * nt + l16; };

    DEMO_PHASE(2);
    // ---- exact top-k over the chunk (magnitude bits are order preserving as unsigned) ------
    uint32_t mag[G::TPW * 4];
#pragma unroll
    for (int i = 0; i < G::TPW; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) mag[i * 4 + r] = __float_as_uint(acc[i][r]) & 0x7fffffffu;

    // (1) a lower bound of the k-th largest magnitude: the k-th largest of the 256 per-thread maxima
    //     (each is a coefficient of its own), resolved to its upper 16 bits.  Every wavefront reads all
    //     256 maxima and bisects on its own, so this costs one barrier.
    {
      uint32_t tmax = 0;
#pragma unroll
      for (int e = 0; e < G::TPW * 4; ++e) tmax = max(tmax, mag[e]);
      sel_mag[tid] = tmax;
    }
    __syncthreads();
    uint32_t thr_lo = 0;
    {
      const uint32_t m0 = sel_mag[lane], m1 = sel_mag[lane + 64], m2 = sel_mag[lane + 128], m3 = sel_mag[lane + 192];
      for (int bit = 30; bit >= 16; --bit) {
        const uint32_t cnd = thr_lo | (1u << bit);
        const int cnt = __popcll(__ballot(m0 >= cnd)) + __popcll(__ballot(m1 >= cnd)) +
                        __popcll(__ballot(m2 >= cnd)) + __popcll(__ballot(m3 >= cnd));
        if (cnt >= k) thr_lo = cnd;
      }
    }
    // (2) candidates |q| >= thr_lo go to a list in LDS (arrival order); key = {~flat index, magnitude} so
    //     that a larger 64-bit key precedes (magnitude descending, then index ascending)
#pragma unroll
    for (int i = 0; i < G::TPW; ++i) {
      int mt, nt;
      tile_of<S>(wave, i, mt, nt);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (mag[i * 4 + r] >= thr_lo) {
          const int pos = atomicAdd(s_cursor, 1);
          if (pos < GEN_CAND_CAP) {
            cand_key[pos] = make_uint2(~(uint32_t)((16 * mt + 4 * lq + r) * S + qcol(nt)), mag[i * 4 + r]);
            cand_val[pos] = acc[i][r];
          }
        }
      }
    }
    __syncthreads();
    const int ncand = *s_cursor;   // uniform
    int my_rank = -1, my_idx = 0;
    float my_val = 0.f;
    if (ncand <= GEN_CAND_CAP) {
      // (3) rank the candidates; ranks below k are the payload.  The list is padded with zero keys (which
      //     precede nothing) to a multiple of 8 so that the reads of a trip are issued together.
      const int npad = (ncand + 7) & ~7;
      if (tid < npad - ncand) cand_key[ncand + tid] = make_uint2(0u, 0u);
      __syncthreads();
      for (int i = tid; i < ncand; i += G::NT) {
        const uint2 me = cand_key[i];
        const uint64_t key = ((uint64_t)me.y << 32) | me.x;
        int rk = 0;
        for (int j = 0; j < npad; j += 8) {
          uint4 o[4];
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) o[jj] = *reinterpret_cast<const uint4*>(&cand_key[j + 2 * jj]);
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            rk += ((((uint64_t)o[jj].y << 32) | o[jj].x) > key) ? 1 : 0;
            rk += ((((uint64_t)o[jj].w << 32) | o[jj].z) > key) ? 1 : 0;
          }
        }
        if (rk < k) {
          const float fv = cand_val[i];
          const int fi = (int)~me.x;
          const int64_t po = (int64_t)c * k + rk;
          store_guarded(d.idx + po, (int32_t)fi);
          store_guarded(d.val + po, fv);
          sel_idx[rk] = fi;
          sel_val[rk] = fv;
        }
      }
      if (tid >= k && tid < kpad) {
        sel_idx[tid] = 0;
        sel_val[tid] = 0.f;
      }
      __syncthreads();
    } else {
      // many (near-)equal magnitudes at the threshold: exact selection by bisection over the whole chunk
      if (tid == 0) *s_cursor = 0;
      __syncthreads();
      int slot = 0;
      uint32_t thr = 0;  // becomes the k-th largest magnitude
      for (int bit = 30; bit >= 0; --bit) {
        const uint32_t cand = thr | (1u << bit);
        int cw = 0;
#pragma unroll
        for (int e = 0; e < G::TPW * 4; ++e) cw += __popcll(__ballot(mag[e] >= cand));
        const int tot = block_sum4(cw, wave, lane, s_cnt, slot);
        slot ^= 1;
        if (tot >= k) thr = cand;
      }
      int cw_gt = 0, cw_ge = 0;
#pragma unroll
      for (int e = 0; e < G::TPW * 4; ++e) {
        cw_gt += __popcll(__ballot(mag[e] > thr));
        cw_ge += __popcll(__ballot(mag[e] >= thr));
      }
      const int n_gt = block_sum4(cw_gt, wave, lane, s_cnt, slot);
      slot ^= 1;
      const int n_ge = block_sum4(cw_ge, wave, lane, s_cnt, slot);
      slot ^= 1;
      const int need = k - n_gt;          // ties to take, >= 1
      uint32_t tie_last = 0xffffffffu;    // largest flat index among the ties taken
      if (n_ge - n_gt != need) {
        // more equal magnitudes than places: take the `need` lowest flat indices
        uint32_t lo = 0;
        for (int bit = 31 - __builtin_clz(G::M - 1); bit >= 0; --bit) {
          const uint32_t cand = lo | (1u << bit);
          int cw = 0;
#pragma unroll
          for (int i = 0; i < G::TPW; ++i) {
            int mt, nt;
            tile_of<S>(wave, i, mt, nt);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              const uint32_t flat = (16 * mt + 4 * lq + r) * S + qcol(nt);
              cw += __popcll(__ballot(mag[i * 4 + r] == thr && flat < cand));
            }
          }
          const int tot = block_sum4(cw, wave, lane, s_cnt, slot);
          slot ^= 1;
          if (tot < need) lo = cand;
        }
        tie_last = lo;
      }
      // gather the k selected coefficients (arrival order), then rank them
#pragma unroll
      for (int i = 0; i < G::TPW; ++i) {
        int mt, nt;
        tile_of<S>(wave, i, mt, nt);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t flat = (16 * mt + 4 * lq + r) * S + qcol(nt);
          const uint32_t mg = mag[i * 4 + r];
          if (mg > thr || (mg == thr && flat <= tie_last)) {
            const int pos = atomicAdd(s_cursor, 1);
            if (pos < DEMO_MAXK_INTERNAL) {
              sel_mag[pos] = mg;
              sel_idx[pos] = (int32_t)flat;
              sel_val[pos] = acc[i][r];
            }
          }
        }
      }
      __syncthreads();
      // rank = number of selected entries that precede this one (magnitude desc, index asc)
      if (tid < k) {
        const uint32_t mg = sel_mag[tid];
        my_idx = sel_idx[tid];
        my_val = sel_val[tid];
        int rk = 0;
        for (int j = 0; j < k; ++j) {
          const uint32_t mj = sel_mag[j];
          rk += (mj > mg || (mj == mg && sel_idx[j] < my_idx)) ? 1 : 0;
        }
        my_rank = rk;
        const int64_t po = (int64_t)c * k + rk;
        store_guarded(d.idx + po, (int32_t)my_idx);
        store_guarded(d.val + po, my_val);
      }
      __syncthreads();
      // sorted list for the reconstruction (deterministic summation order); padded to a multiple of 4
      if (tid < k) {
        sel_idx[my_rank] = my_idx;
        sel_val[my_rank] = my_val;
      } else if (tid < kpad) {
        sel_idx[tid] = 0;
        sel_val[tid] = 0.f;
      }
      __syncthreads();
    }

    DEMO_PHASE(3);
    // ---- R = P^T Q^ P = sum_t val_t * P[u_t][:]^T P[v_t][:]  (contraction length k) ----------
#pragma unroll
    for (int i = 0; i < G::TPW; ++i) acc[i] = (f32x4){0.f, 0.f, 0.f, 0.f};
    for (int ks = 0; ks < kpad / 4; ++ks) {
      const int tt = 4 * ks + lq;
      const int fi = sel_idx[tt];
      const float fv = sel_val[tt];
      const int u = fi / S, v = fi - u * S;
      const int pu = mir ? fold_pos<S>(u) : u, pv = mir ? fold_pos<S>(v) : v;   // rows of P in the LDS tile
#pragma unroll
      for (int i = 0; i < G::TPW; ++i) {
        int mt, nt;
        tile_of<S>(wave, i, mt, nt);
        const float a = fv * sP[pu * G::LD + 16 * mt + l16];
        const float b = sP[pv * G::LD + 16 * nt + l16];
        acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[i], 0, 0, 0);
      }
    }
    store_acc<S>(acc, wave, lane, sX);   // sX (and sT) are dead since the barriers above
    __syncthreads();

    DEMO_PHASE(4);
    // ---- m <- m - R ----------------------------------------------------------------------
#pragma unroll
    for (int p = 0; p < G::PASSES; ++p) {
      const int row = p * G::ROWS_PER_PASS + lrow;
      const int64_t off = base + (int64_t)row * d.cols + lcol;
      const float4 r = *reinterpret_cast<const float4*>(&sX[row * G::LD + lcol]);
      float4 o;
      o.x = __fmaf_rn(-args.alpha, r.x, mid[p].x);
      o.y = __fmaf_rn(-args.alpha, r.y, mid[p].y);
      o.z = __fmaf_rn(-args.alpha, r.z, mid[p].z);
      o.w = __fmaf_rn(-args.alpha, r.w, mid[p].w);
      store_guarded(reinterpret_cast<f32x4*>(d.mom + off), (f32x4){o.x, o.y, o.z, o.w});
    }
    DEMO_PHASE(5);
  }
  DEMO_PHASE_FLUSH(0);
  if (wl.list != nullptr) {
    __syncthreads();   // every thread has read *wl.count
    if (tid == 0) {
      __threadfence();
      if (atomicAdd(wl.ticket, 1) == (int)gridDim.x - 1) {
        store_guarded(wl.count, 0);
        store_guarded(wl.ticket, 0);
      }
    }
  }
}

// ---------------------------------------------------------------------------
// decode, order-2 tensors, generic
// ---------------------------------------------------------------------------
template <int S, bool MIR>
__global__ __launch_bounds__(256) void decode2d_generic(TableView tv, const float* __restrict__ basis,
                                                        DecodeArgs args) {
  using G = Geo<S>;
  extern __shared__ float lds[];
  float* sP = lds;
  float* sX = sP + G::TILE_FLOATS;                     // coefficient sums / first product / signs
  float* sT = G::INPLACE ? sX : sX + G::TILE_FLOATS;
  uint32_t* s_red = reinterpret_cast<uint32_t*>(sX + G::TILE_FLOATS * (G::INPLACE ? 1 : 2));   // [4]
  uint32_t* s_cnt = s_red + 4;   // [TILE_FLOATS / 4] senders per coefficient, one byte each (count aggregate)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int k = args.k, W = args.W;
  const bool by_count = args.agg == 2, plain_sign = args.phi == 0 && !by_count;

  constexpr bool mir = MIR;
  for (int e = tid; e < S * S; e += G::NT) sP[(mir ? fold_pos<S>(e / S) : e / S) * G::LD + (e % S)] = basis[e];

  TensorCursor cur;
  for (int chunk = blockIdx.x; chunk < tv.total_chunks; chunk += gridDim.x) {
    const int t = tensor_of_chunk(tv, chunk, cur);
    const TensorDev d = tv.descs[t];
    const int c = chunk - cur.first;
    const int k0 = c / d.cchunks, k1 = c - k0 * d.cchunks;
    const int64_t base = (int64_t)k0 * S * d.cols + (int64_t)k1 * S;
    const int lrow = tid / G::F4_PER_ROW, lcol = (tid % G::F4_PER_ROW) * 4;

    // parameters of the chunk: requested now, used after the products (one dtype branch per chunk)
    float4 xv[G::PASSES];
    if (d.param_bf16) {
      uint2 xh[G::PASSES];
#pragma unroll
      for (int p = 0; p < G::PASSES; ++p)
        xh[p] = *reinterpret_cast<const uint2*>(static_cast<const uint16_t*>(d.param) + base +
                                                (int64_t)(p * G::ROWS_PER_PASS + lrow) * d.cols + lcol);
#pragma unroll
      for (int p = 0; p < G::PASSES; ++p)
        xv[p] = make_float4(bf16_to_f32(xh[p].x & 0xffffu), bf16_to_f32(xh[p].x >> 16), bf16_to_f32(xh[p].y & 0xffffu),
                            bf16_to_f32(xh[p].y >> 16));
    } else {
#pragma unroll
      for (int p = 0; p < G::PASSES; ++p)
        xv[p] = *reinterpret_cast<const float4*>(static_cast<const float*>(d.param) + base +
                                                 (int64_t)(p * G::ROWS_PER_PASS + lrow) * d.cols + lcol);
    }
    __syncthreads();
    for (int e = tid; e < S * G::LD; e += G::NT) sX[e] = 0.f;
    if (by_count)
      for (int e = tid; e < G::TILE_FLOATS / 4; e += G::NT) s_cnt[e] = 0u;
    __syncthreads();

    // ---- S[idx] += val in block fixed point: the values are scaled by a power of two taken from
    //      the largest magnitude of the chunk's payload (exact), rounded to integers and added with
    //      integer LDS atomics (an order of magnitude faster than float ones on this part, and the
    //      sum does not depend on the order of arrival); W values of `vbits` bits cannot overflow.
    //      Only sgn(IDCT(S)) is used afterwards, so the scale is never undone. ---------------------
    {
      const int64_t wstride = (int64_t)d.nchunks * k;
      const int npairs = W * k;
      // pair p = tid, tid + 256, ...: worker p / k, position p % k, advanced without dividing; loads in batches
      // of four so that several are in flight per thread (S = 32 runs many workgroups per CU instead and keeps
      // its registers: batches of one)
      constexpr int NB = S == 32 ? 1 : 4;
      const int dq = G::NT / k, dr = G::NT - dq * k;
      const int w0 = tid / k, t0 = tid - w0 * k;
      const float* vbase = d.val + (int64_t)c * k;
      const int32_t* ibase = d.idx + (int64_t)c * k;
      auto advance = [&](int& w, int& tt) {
        w += dq;
        tt += dr;
        if (tt >= k) {
          tt -= k;
          ++w;
        }
      };
      float mx = 0.f;
      {
        int w = w0, tt = t0;
        for (int p = tid; p < npairs; p += NB * G::NT) {
          float v[NB];
#pragma unroll
          for (int q = 0; q < NB; ++q) {
            v[q] = p + q * G::NT < npairs ? vbase[(int64_t)w * wstride + tt] : 0.f;
            advance(w, tt);
          }
#pragma unroll
          for (int q = 0; q < NB; ++q) mx = fmaxf(mx, fabsf(v[q]));
        }
      }
      uint32_t mb = __float_as_uint(mx);
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) mb = max(mb, (uint32_t)__shfl_xor((int)mb, off));
      if (lane == 0) s_red[wave] = mb;
      __syncthreads();
      mb = max(max(s_red[0], s_red[1]), max(s_red[2], s_red[3]));
      int ex = (int)(mb >> 23);
      ex = ex < 1 ? 1 : ex;
      int vbits = 30;
      for (int w = 1; w < W; w <<= 1) --vbits;
      const int sh = vbits + 126 - ex;
      int* iX = reinterpret_cast<int*>(sX);
      {
        int w = w0, tt = t0;
        for (int p = tid; p < npairs; p += NB * G::NT) {
          int fi[NB];
          float fv[NB];
#pragma unroll
          for (int q = 0; q < NB; ++q) {
            const bool ok = p + q * G::NT < npairs;
            const int64_t po = (int64_t)w * wstride + tt;
            fi[q] = ok ? ibase[po] : -1;
            fv[q] = ok ? vbase[po] : 0.f;
            advance(w, tt);
          }
#pragma unroll
          for (int q = 0; q < NB; ++q) {
            if (fi[q] >= 0 && fi[q] < G::M) {
              const int u = fi[q] / S, v = fi[q] - u * S;
              const int a = u * G::LD + v;
              atomicAdd(&iX[a], __float2int_rn(ldexpf(fv[q], sh)));
              if (by_count) atomicAdd(&s_cnt[a >> 2], 1u << (8 * (a & 3)));   // W <= 255: no carry between bytes
            }
          }
        }
      }
      __syncthreads();
      if (plain_sign) {
        // only sgn(IDCT(S)) is used: the scale is never undone
        for (int e = tid; e < S * G::LD; e += G::NT) sX[e] = (float)iX[e];
      } else {
        for (int e = tid; e < S * G::LD; e += G::NT) {
          float v = ldexpf((float)iX[e], -sh) * args.scale;
          if (by_count) {
            const uint32_t n = (s_cnt[e >> 2] >> (8 * (e & 3))) & 255u;
            v = n != 0u ? v / (float)n : 0.f;                              // S (/) n, 0/0 = 0
          }
          sX[e] = v;
        }
      }
    }
    __syncthreads();

    // ---- Y = P^T * S, R = Y * P, phi(R) into sX ---------------------------------------------
    f32x4 acc[G::TPW];
    if constexpr (MIR) {
      gemm_fold_dec1<S>(acc, wave, lane, sP, sX, sT);   // in place: a wavefront touches only its own columns
      __syncthreads();
      gemm_fold_dec2<S>(acc, wave, lane, sP, sT);
      __syncthreads();                                   // all reads of Y are done
      emit_fold_dec2<S>(acc, wave, lane, [&](int i, int j, float r) {
        sX[i * G::LD + j] = args.phi == 0 ? sgnf(r) : r;                                     // phi(m)
      });
      __syncthreads();
    } else {
      gemm_lds<S>(acc, wave, lane, lds,
                  [&](int m, int kk) { return kk * G::LD + m; },                              // P[u][i]
                  [&](int kk, int n) { return G::TILE_FLOATS + kk * G::LD + n; });           // S[u][v]
      store_acc<S>(acc, wave, lane, sT);
      __syncthreads();
      const int t_off = (int)(sT - lds);
      gemm_lds<S>(acc, wave, lane, lds,
                  [&](int m, int kk) { return t_off + m * G::LD + kk; },                     // Y[i][v]
                  [&](int kk, int n) { return kk * G::LD + n; });                             // P[v][j]
#pragma unroll
      for (int i = 0; i < G::TPW; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[i][r] = args.phi == 0 ? sgnf(acc[i][r]) : acc[i][r];   // phi(m)
      __syncthreads();                       // all reads of Y are done
      store_acc<S>(acc, wave, lane, sX);
      __syncthreads();
    }

    // ---- x <- x - lr*(phi(m) + wd*x) --------------------------------------------------------
#pragma unroll
    for (int p = 0; p < G::PASSES; ++p) {
      const int row = p * G::ROWS_PER_PASS + lrow;
      const float4 sg = *reinterpret_cast<const float4*>(&sX[row * G::LD + lcol]);
      xv[p].x = sign_update(xv[p].x, sg.x, args.lr, args.weight_decay);
      xv[p].y = sign_update(xv[p].y, sg.y, args.lr, args.weight_decay);
      xv[p].z = sign_update(xv[p].z, sg.z, args.lr, args.weight_decay);
      xv[p].w = sign_update(xv[p].w, sg.w, args.lr, args.weight_decay);
    }
    if (d.param_bf16) {
#pragma unroll
      for (int p = 0; p < G::PASSES; ++p)
        store4(d.param, base + (int64_t)(p * G::ROWS_PER_PASS + lrow) * d.cols + lcol, 1, xv[p]);
    } else {
#pragma unroll
      for (int p = 0; p < G::PASSES; ++p)
        store4(d.param, base + (int64_t)(p * G::ROWS_PER_PASS + lrow) * d.cols + lcol, 0, xv[p]);
    }
  }
}

// ---------------------------------------------------------------------------
// order-1 tensors: one wavefront per chunk of S elements
// ---------------------------------------------------------------------------
template <int S>
__global__ __launch_bounds__(64) void encode1d_wave(TableView tv, const float* __restrict__ basis,
                                                    EncodeArgs args) {
  constexpr int EPL = (S + 63) / 64;
  __shared__ float s_b[S];
  __shared__ float s_q[S];
  __shared__ int32_t s_sel_idx[S];
  __shared__ float s_sel_val[S];
  const int lane = threadIdx.x;
  const int k = args.k;
  const int chunk = blockIdx.x;
  const int t = find_tensor(tv.prefix, tv.n, chunk);
  const TensorDev d = tv.descs[t];
  const int c = chunk - tv.prefix[t];
  const int64_t base = (int64_t)c * S;

  float b[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    const int n = lane + 64 * e;
    b[e] = 0.f;
    if (n < S) {
      const float g = d.grad_bf16 ? bf16_to_f32(static_cast<const uint16_t*>(d.grad)[base + n])
                                  : static_cast<const float*>(d.grad)[base + n];
      b[e] = __fmaf_rn(args.beta, d.mom[base + n], args.grad_scale * g);
      s_b[n] = b[e];
    }
  }
  __syncthreads();
  float q[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    const int u = lane + 64 * e;
    q[e] = 0.f;
    if (u < S) {
      float a = 0.f;
      for (int n = 0; n < S; ++n) a = __fmaf_rn(basis[u * S + n], s_b[n], a);   // q = P b
      q[e] = a;
      s_q[u] = a;
    }
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    const int u = lane + 64 * e;
    if (u < S) {
      const uint32_t mg = __float_as_uint(q[e]) & 0x7fffffffu;
      int rk = 0;
      for (int j = 0; j < S; ++j) {
        const uint32_t mj = __float_as_uint(s_q[j]) & 0x7fffffffu;
        rk += (mj > mg || (mj == mg && j < u)) ? 1 : 0;
      }
      if (rk < k) {
        store_guarded(d.idx + ((int64_t)c * k + rk), (int32_t)u);
        store_guarded(d.val + ((int64_t)c * k + rk), q[e]);
        s_sel_idx[rk] = u;
        s_sel_val[rk] = q[e];
      }
    }
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    const int n = lane + 64 * e;
    if (n < S) {
      float r = 0.f;
      for (int j = 0; j < k; ++j) r = __fmaf_rn(s_sel_val[j], basis[s_sel_idx[j] * S + n], r);   // P^T q^
      store_guarded(d.mom + (base + n), __fmaf_rn(-args.alpha, r, b[e]));
    }
  }
}

// VEC: k a multiple of four, 16-byte aligned payload arrays and at most 2048 pairs per chunk: the pairs are fetched
// once, four consecutive pairs of one worker per 16-byte load (unit 64 j + lane of the W k pairs in worker-major
// order), and kept in registers for both the maximum and the sums.
template <int S, bool VEC>
__global__ __launch_bounds__(64) void decode1d_wave(TableView tv, const float* __restrict__ basis,
                                                    DecodeArgs args) {
  constexpr int EPL = (S + 63) / 64;
  __shared__ float s_acc[S];
  const int lane = threadIdx.x;
  const int k = args.k, W = args.W;
  const int chunk = blockIdx.x;
  const int t = find_tensor(tv.prefix, tv.n, chunk);
  const TensorDev d = tv.descs[t];
  const int c = chunk - tv.prefix[t];
  const int64_t base = (int64_t)c * S;
  __shared__ int s_cnt1[S];
  int* i_acc = reinterpret_cast<int*>(s_acc);
  const bool by_count = args.agg == 2, plain_sign = args.phi == 0 && !by_count;
  for (int n = lane; n < S; n += 64) {
    i_acc[n] = 0;
    s_cnt1[n] = 0;
  }
  // sum of the W payloads in block fixed point (as in the order-2 kernels): pass 1 finds the largest
  // magnitude of the chunk's W*k values, pass 2 adds them as integers, independent of the order
  const int64_t wstride = (int64_t)d.nchunks * k;
  const DEMO_GLOBAL int32_t* ip = as_global(d.idx) + (int64_t)c * k;
  const DEMO_GLOBAL float* vp = as_global(d.val) + (int64_t)c * k;
  const int npairs = W * k;
  float mx = 0.f;
  constexpr int NPV = 32;   // VEC: payload registers per lane
  int32_t pi[NPV];
  float pv[NPV];
  const int nunits = npairs >> 2, nloads = (nunits + 63) >> 6;
  if constexpr (VEC) {
    const float rk = 1.0f / (float)k;
#pragma unroll
    for (int j = 0; j < NPV / 4; ++j) {
      if (j < nloads) {   // uniform
        const int unit = 64 * j + lane;
        const int p = 4 * unit;
        const int w = (int)(((float)p + 0.5f) * rk);   // p / k, exact for p < 65536 (see the order-2 kernels)
        const int tt = p - w * k;
        const bool ok = unit < nunits;
        const int64_t off = ok ? (int64_t)w * wstride + tt : 0;
        const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const DEMO_GLOBAL u32x4*>(ip + off));
        const f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const DEMO_GLOBAL f32x4*>(vp + off));
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          pi[4 * j + x] = ok ? (int32_t)a[x] : -1;
          pv[4 * j + x] = ok ? b[x] : 0.f;
          mx = fmaxf(mx, fabsf(pv[4 * j + x]));
        }
      }
    }
  } else {
#pragma unroll 4
    for (int p = lane; p < npairs; p += 64) {
      const int w = p / k, tt = p - w * k;
      mx = fmaxf(mx, fabsf(vp[(int64_t)w * wstride + tt]));
    }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
  int ex = (int)(__float_as_uint(mx) >> 23);
  ex = ex < 1 ? 1 : ex;
  int vbits = 30;
  for (int w = 1; w < W; w <<= 1) --vbits;
  const int sh = vbits + 126 - ex;
  __syncthreads();
  if constexpr (VEC) {
#pragma unroll
    for (int j = 0; j < NPV; ++j) {
      if (j < 4 * nloads) {   // uniform
        const int fi = pi[j];
        if (fi >= 0 && fi < S) {
          atomicAdd(&i_acc[fi], __float2int_rn(ldexpf(pv[j], sh)));
          if (by_count) atomicAdd(&s_cnt1[fi], 1);
        }
      }
    }
  } else {
#pragma unroll 4
    for (int p = lane; p < npairs; p += 64) {
      const int w = p / k, tt = p - w * k;
      const int fi = ip[(int64_t)w * wstride + tt];
      const float fv = vp[(int64_t)w * wstride + tt];
      if (fi >= 0 && fi < S) {
        atomicAdd(&i_acc[fi], __float2int_rn(ldexpf(fv, sh)));
        if (by_count) atomicAdd(&s_cnt1[fi], 1);
      }
    }
  }
  __syncthreads();
  for (int n = lane; n < S; n += 64) {
    float v = (float)i_acc[n];
    if (!plain_sign) {
      v = ldexpf(v, -sh) * args.scale;
      if (by_count) v = s_cnt1[n] != 0 ? v / (float)s_cnt1[n] : 0.f;
    }
    s_acc[n] = v;
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < EPL; ++e) {
    const int n = lane + 64 * e;
    if (n < S) {
      float r = 0.f;
      for (int u = 0; u < S; ++u) r = __fmaf_rn(s_acc[u], basis[u * S + n], r);   // P^T s
      const float sg = args.phi == 0 ? sgnf(r) : r;   // phi(m)
      if (d.param_bf16) {
        uint16_t* xp = static_cast<uint16_t*>(d.param) + base + n;
        *xp = (uint16_t)f32_to_bf16_rne(sign_update(bf16_to_f32(*xp), sg, args.lr, args.weight_decay));
      } else {
        float* xp = static_cast<float*>(d.param) + base + n;
        store_guarded(xp, sign_update(*xp, sg, args.lr, args.weight_decay));
      }
    }
  }
}

// ---------------------------------------------------------------------------
// plain streaming copy (bandwidth probe / calibration of the HBM traffic counters)
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void copy_probe_kernel(const float4* __restrict__ src, float4* __restrict__ dst,
                                                         size_t n16) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x)
    dst[i] = src[i];
}

hipError_t launch_copy_probe(const void* src, void* dst, size_t nbytes, int num_cus, hipStream_t stream) {
  const size_t n16 = nbytes / 16;
  if (n16 == 0) return hipSuccess;
  size_t grid = (size_t)num_cus * 16;
  if (grid > (n16 + 255) / 256) grid = (n16 + 255) / 256;
  hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)grid), dim3(256), 0, stream, static_cast<const float4*>(src),
                     static_cast<float4*>(dst), n16);
  return hipGetLastError();
}

// Streaming probe in the launch shape of the wavefront kernels: one 512-thread workgroup per compute unit, every
// lane moves 16 bytes per access with eight accesses in flight; a workgroup's accesses of one round are contiguous
// (8 KiB per access slot) and the workgroups advance together through memory.
// MODE 0: copy, default cache policy; 1: copy, non-temporal; 2: read only, non-temporal; 3: write only,
// non-temporal; 4: write only, default cache policy.
template <int MODE>
__global__ __launch_bounds__(512) void stream_probe_kernel(const f32x4* __restrict__ src, f32x4* __restrict__ dst, size_t n16) {
  constexpr int UNROLL = 8;
  const size_t per_round = (size_t)gridDim.x * 512 * UNROLL;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (size_t base = (size_t)blockIdx.x * 512 * UNROLL; base < n16; base += per_round) {
    f32x4 v[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const size_t i = base + (size_t)u * 512 + threadIdx.x;
      if (MODE >= 3) v[u] = (f32x4){(float)i, 1.f, 2.f, 3.f};
      else if (i < n16) v[u] = MODE == 0 ? as_global(src)[i] : __builtin_nontemporal_load(as_global(src) + i);
      else v[u] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const size_t i = base + (size_t)u * 512 + threadIdx.x;
      if (MODE == 2) {
        acc += v[u];
      } else if (i < n16) {
        if (MODE == 0 || MODE == 4) as_global(dst)[i] = v[u];
        else __builtin_nontemporal_store(v[u], as_global(dst) + i);
      }
    }
  }
  if (MODE == 2) {   // one 16-byte store per wavefront keeps the reads alive
    f32x4 r = acc;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
#pragma unroll
      for (int e = 0; e < 4; ++e) r[e] += __shfl_xor(r[e], off);
    if ((threadIdx.x & 63) == 0) as_global(dst)[blockIdx.x * 8 + (threadIdx.x >> 6)] = r;
  }
}

hipError_t launch_stream_probe(const void* src, void* dst, size_t nbytes, int mode, int num_cus, hipStream_t stream) {
  const size_t n16 = nbytes / 16;
  if (n16 == 0) return hipSuccess;
  size_t grid = (size_t)num_cus;
  if (grid > (n16 + 4095) / 4096) grid = (n16 + 4095) / 4096;
  if (grid > 512) grid = 512;   // mode 2 writes 128 bytes per workgroup into at least 64 KiB
  const f32x4* s4 = static_cast<const f32x4*>(src);
  f32x4* d4 = static_cast<f32x4*>(dst);
  switch (mode) {
    case 0: hipLaunchKernelGGL(stream_probe_kernel<0>, dim3((unsigned)grid), dim3(512), 0, stream, s4, d4, n16); break;
    case 1: hipLaunchKernelGGL(stream_probe_kernel<1>, dim3((unsigned)grid), dim3(512), 0, stream, s4, d4, n16); break;
    case 2: hipLaunchKernelGGL(stream_probe_kernel<2>, dim3((unsigned)grid), dim3(512), 0, stream, s4, d4, n16); break;
    case 3: hipLaunchKernelGGL(stream_probe_kernel<3>, dim3((unsigned)grid), dim3(512), 0, stream, s4, d4, n16); break;
    case 4: hipLaunchKernelGGL(stream_probe_kernel<4>, dim3((unsigned)grid), dim3(512), 0, stream, s4, d4, n16); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// launch wrappers
// ---------------------------------------------------------------------------
template <int S>
static hipError_t launch_enc2d_generic(const TableView& tv, const float* basis, const EncodeArgs& a,
                                       const Worklist& wl, int num_cus, hipStream_t stream) {
  using G = Geo<S>;
  const size_t lds_bytes = sizeof(float) * G::LDS_FLOATS;
  constexpr bool CAN_FOLD = S == 128;
  const bool fold = CAN_FOLD && a.mirror != 0;
  const void* kern = fold ? reinterpret_cast<const void*>(&encode2d_generic<S, CAN_FOLD>)
                          : reinterpret_cast<const void*>(&encode2d_generic<S, false>);
  hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (e != hipSuccess) return e;
  const int per_cu = (int)((160 * 1024) / lds_bytes) < 1 ? 1 : (int)((160 * 1024) / lds_bytes);
  int64_t grid = (int64_t)num_cus * (per_cu > 8 ? 8 : per_cu);
  if (grid > tv.total_chunks) grid = tv.total_chunks;
  if (wl.list != nullptr && grid > 64) grid = 64;   // the queue is short; an empty one costs one launch
  if (fold)
    hipLaunchKernelGGL((encode2d_generic<S, CAN_FOLD>), dim3((unsigned)grid), dim3(256), lds_bytes, stream, tv, basis, a, wl);
  else
    hipLaunchKernelGGL((encode2d_generic<S, false>), dim3((unsigned)grid), dim3(256), lds_bytes, stream, tv, basis, a, wl);
  return hipGetLastError();
}

template <int S>
static hipError_t launch_dec2d_generic(const TableView& tv, const float* basis, const DecodeArgs& a, int num_cus,
                                       hipStream_t stream) {
  using G = Geo<S>;
  const size_t lds_bytes = sizeof(float) * (G::TILE_FLOATS * (G::INPLACE ? 2 : 3) + 4 + G::TILE_FLOATS / 4);
  constexpr bool CAN_FOLD = S == 128;
  const bool fold = CAN_FOLD && a.mirror != 0;
  const void* kern = fold ? reinterpret_cast<const void*>(&decode2d_generic<S, CAN_FOLD>)
                          : reinterpret_cast<const void*>(&decode2d_generic<S, false>);
  hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
  if (e != hipSuccess) return e;
  const int per_cu = (int)((160 * 1024) / lds_bytes) < 1 ? 1 : (int)((160 * 1024) / lds_bytes);
  int64_t grid = (int64_t)num_cus * (per_cu > 8 ? 8 : per_cu);
  if (grid > tv.total_chunks) grid = tv.total_chunks;
  if (fold)
    hipLaunchKernelGGL((decode2d_generic<S, CAN_FOLD>), dim3((unsigned)grid), dim3(256), lds_bytes, stream, tv, basis, a);
  else
    hipLaunchKernelGGL((decode2d_generic<S, false>), dim3((unsigned)grid), dim3(256), lds_bytes, stream, tv, basis, a);
  return hipGetLastError();
}

hipError_t launch_encode2d(const TableView& tv, const TableView* tiles, const BasisTables& bt, int s,
                           const EncodeArgs& a, const Worklist& wl, int num_cus, int variant, hipStream_t stream) {
  if (tv.total_chunks == 0) return hipSuccess;
  const float* basis = bt.basis;
  const uint32_t gmix = tv.dtypes & 3u;   // gradient dtypes present: the wavefront kernels want one
  if (variant >= 1 && s == 32 && a.k <= kFast64MaxK && bt.enc32 != nullptr && tiles != nullptr &&
      wl.list != nullptr && (gmix == 1u || gmix == 2u)) {
    // wavefront-per-tile kernel (2 x 2 chunks), then the exact generic kernel over whatever it queued
    hipError_t e = launch_encode2d_tile32(*tiles, tv.prefix, bt.enc32, a, wl, gmix == 1u, num_cus, stream);
    if (e != hipSuccess) return e;
    return launch_enc2d_generic<32>(tv, basis, a, wl, num_cus, stream);
  }
  if (variant >= 1 && s == 64 && a.k <= kFast64MaxK && bt.enc64 != nullptr && wl.list != nullptr &&
      (gmix == 1u || gmix == 2u)) {
    // wavefront-per-chunk kernel, then the exact generic kernel over whatever it queued
    hipError_t e = launch_encode2d_wave64(tv, bt.enc64, a, wl, gmix == 1u, false, num_cus, stream);
    if (e != hipSuccess) return e;
    return launch_enc2d_generic<64>(tv, basis, a, wl, num_cus, stream);
  }
  if (variant >= 1 && s == 64 && a.k <= kFast64MaxK && bt.enc64g != nullptr && !bt.dct && a.stage == 0 &&
      wl.list != nullptr && (gmix == 1u || gmix == 2u)) {
    // any orthonormal matrix: the same wavefront-per-chunk kernel with the full products
    hipError_t e = launch_encode2d_wave64(tv, bt.enc64g, a, wl, gmix == 1u, true, num_cus, stream);
    if (e != hipSuccess) return e;
    return launch_enc2d_generic<64>(tv, basis, a, wl, num_cus, stream);
  }
  if (variant >= 1 && s == 128 && a.mirror != 0 && a.k <= kFast128MaxK && wl.list != nullptr && bt.enc128 != nullptr &&
      (gmix == 1u || gmix == 2u)) {
    // workgroup-per-chunk kernel with the next chunk in flight, then the exact generic kernel over its queue
    hipError_t e = launch_encode2d_wg128(tv, basis, bt.enc128, a, wl, gmix == 1u, num_cus, stream);
    if (e != hipSuccess) return e;
    return launch_enc2d_generic<128>(tv, basis, a, wl, num_cus, stream);
  }
  const Worklist none{nullptr, nullptr, nullptr};
  switch (s) {
    case 32: return launch_enc2d_generic<32>(tv, basis, a, none, num_cus, stream);
    case 64: return launch_enc2d_generic<64>(tv, basis, a, none, num_cus, stream);
    case 128: return launch_enc2d_generic<128>(tv, basis, a, none, num_cus, stream);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_decode2d(const TableView& tv, const TableView* tiles, const BasisTables& bt, int s,
                           const DecodeArgs& a, int num_cus, int variant, hipStream_t stream) {
  if (tv.total_chunks == 0) return hipSuccess;
  const uint32_t pmix = (tv.dtypes >> 2) & 3u;   // parameter dtypes present: the wavefront kernel wants one
  // the wavefront kernels address a tensor's payload with 32-bit offsets (worker * pairs-per-worker + position)
  const bool payload_fits32 = (int64_t)tv.total_chunks * a.k * a.W < (int64_t)1 << 31;
  if (variant >= 1 && s == 32 && (decode_is_sign_of_sum(a) || a.W * a.k <= kFast32MaxPairs) && tiles != nullptr &&
      fast32_decode_supports(a.W, a.k, (tiles->dtypes & 16u) == 0) && payload_fits32 && bt.dec32 != nullptr &&
      (pmix == 1u || pmix == 2u))
    return launch_decode2d_tile32(*tiles, bt.dec32, a, pmix == 1u, num_cus, stream);
  // The full-product instance on the float16 matrix pipe (any matrix, the DCT included) has overtaken the mirror-folded
  // float32 instances wherever it applies: more than 64 and at most 2048 pairs per chunk, sum or mean.  The DCT keeps
  // its own kernels for fewer pairs (no coefficient tile), for streamed payloads and for the count-normalised aggregate.
  if (variant >= 1 && s == 64 && bt.dec64g != nullptr && dense64_decode_supports(a) && payload_fits32 &&
      (!bt.dct || (a.W * a.k > 64 && variant != 2)) && (pmix == 1u || pmix == 2u))
    return launch_decode2d_dense64(tv, bt.dec64g, a, pmix == 1u, (tv.dtypes & 16u) == 0, num_cus, stream);
  if (variant >= 1 && s == 64 && bt.dct && (decode_is_sign_of_sum(a) || a.W * a.k <= kFast64CountMaxPairs) &&
      fast64_decode_supports(a.W, a.k, (tv.dtypes & 16u) == 0) && payload_fits32 &&
      bt.dec64 != nullptr && (pmix == 1u || pmix == 2u))
    return launch_decode2d_wave64(tv, bt.dec64, a, pmix == 1u, (tv.dtypes & 16u) == 0, num_cus, stream);
  if (variant >= 1 && s == 128 && a.mirror != 0 && (decode_is_sign_of_sum(a) || a.W * a.k <= kFast128MaxPairs) &&
      fast128_decode_supports(a.W, a.k, (tv.dtypes & 16u) == 0) && payload_fits32 && bt.dec128 != nullptr &&
      (pmix == 1u || pmix == 2u))
    return launch_decode2d_wg128(tv, bt.basis, bt.dec128, a, pmix == 1u, num_cus, stream);
  const float* basis = bt.basis;
  switch (s) {
    case 32: return launch_dec2d_generic<32>(tv, basis, a, num_cus, stream);
    case 64: return launch_dec2d_generic<64>(tv, basis, a, num_cus, stream);
    case 128: return launch_dec2d_generic<128>(tv, basis, a, num_cus, stream);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_encode1d(const TableView& tv, const float* basis, int s, const EncodeArgs& a,
                           hipStream_t stream) {
  if (tv.total_chunks == 0) return hipSuccess;
  const dim3 grid((unsigned)tv.total_chunks), block(64);
  switch (s) {
    case 32: hipLaunchKernelGGL(encode1d_wave<32>, grid, block, 0, stream, tv, basis, a); break;
    case 64: hipLaunchKernelGGL(encode1d_wave<64>, grid, block, 0, stream, tv, basis, a); break;
    case 128: hipLaunchKernelGGL(encode1d_wave<128>, grid, block, 0, stream, tv, basis, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_decode1d(const TableView& tv, const float* basis, int s, const DecodeArgs& a,
                           hipStream_t stream) {
  if (tv.total_chunks == 0) return hipSuccess;
  const dim3 grid((unsigned)tv.total_chunks), block(64);
  const bool vec = (tv.dtypes & 16u) == 0 && (a.k & 3) == 0 && (int64_t)a.W * a.k <= 2048;
  switch (s) {
    case 32:
      if (vec) hipLaunchKernelGGL((decode1d_wave<32, true>), grid, block, 0, stream, tv, basis, a);
      else hipLaunchKernelGGL((decode1d_wave<32, false>), grid, block, 0, stream, tv, basis, a);
      break;
    case 64:
      if (vec) hipLaunchKernelGGL((decode1d_wave<64, true>), grid, block, 0, stream, tv, basis, a);
      else hipLaunchKernelGGL((decode1d_wave<64, false>), grid, block, 0, stream, tv, basis, a);
      break;
    case 128:
      if (vec) hipLaunchKernelGGL((decode1d_wave<128, true>), grid, block, 0, stream, tv, basis, a);
      else hipLaunchKernelGGL((decode1d_wave<128, false>), grid, block, 0, stream, tv, basis, a);
      break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace demo

DEMO_PHASE_GETTER(demo_debug_phase_clocks_gen)
