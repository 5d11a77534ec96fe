// Dense contractions of the layer (paper sec. 2.1: "GEMM"), hand written for gfx950.
//   C[M,N] = act(A[M,K] . B[N,K]^T + bias[N]),  A and B both K-contiguous, fp32 accumulation.
// fp16: MFMA v_mfma_f32_32x32x16_f16 on LDS-staged tiles.  fp32: a plain LDS-tiled FMA kernel
// (only the small fp32 configuration uses it).  Bias, ReLU and the output scatter (Q to the
// activation buffer, K and V straight into the caches) are fused into the epilogue.
#include <unordered_map>

#include "lsq_internal.h"

namespace lsq {

template <typename T>
__device__ __forceinline__ void store_one(const GemmOut& o, int m, int n, float v, long tp) {
  int s = n / o.seg_n;
  reinterpret_cast<T*>(o.ptr[s])[(long)m * o.ld[s] + tp * o.tmul[s] + (n - s * o.seg_n)] = (T)v;
}

// Epilogue activation: 0 none, 1 ReLU, 2 tanh-GELU 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))).
__device__ __forceinline__ float activate(float v, int act) {
  if (act == 1) return fmaxf(v, 0.f);
  if (act == 2) return 0.5f * v * (1.0f + tanhf(0.7978845608028654f * (v + 0.044715f * v * v * v)));
  return v;
}

// four floats that are only 4-byte aligned: still one store instruction (the target allows dword-aligned
// multi-dword accesses to global memory, and the compiler uses them for this type)
struct __attribute__((packed, aligned(4))) float4_dword_aligned { float a, b, c, d; };

// Stores four consecutive outputs (m, n..n+3) of a tile: split-K slab, vector, or element-wise
// fallback for ragged / unaligned rows.  vec_ok: 1 = the four lie in one segment and are aligned to their size;
// 2 = float output of a single segment whose rows are not 16-byte aligned (an odd vocabulary size).
template <typename OutT, bool SPLIT>
__device__ __forceinline__ void store4(const GemmOut& out, int m, int n, const float (&v)[4], int M, int N,
                                       int vec_ok, int slab, long tp) {
  if constexpr (SPLIT) {
    float* dst = reinterpret_cast<float*>(out.ptr[0]) + ((size_t)slab * M + m) * N + n;
    if (vec_ok == 1 && n + 3 < N) {
      floatx4 f = {v[0], v[1], v[2], v[3]};
      *reinterpret_cast<floatx4*>(dst) = f;
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e)
        if (n + e < N) dst[e] = v[e];
    }
  } else if (vec_ok == 2 && n + 3 < N && sizeof(OutT) == 4) {
    float* dst = reinterpret_cast<float*>(out.ptr[0]) + (long)m * out.ld[0] + tp * out.tmul[0] + n;
    const float4_dword_aligned f = {v[0], v[1], v[2], v[3]};
    *reinterpret_cast<float4_dword_aligned*>(dst) = f;
  } else if (vec_ok == 1 && n + 3 < N) {
    int s = n / out.seg_n;
    OutT* dst = reinterpret_cast<OutT*>(out.ptr[s]) + (long)m * out.ld[s] + tp * out.tmul[s] + (n - s * out.seg_n);
    if constexpr (sizeof(OutT) == 2) {
      half4_t h = {(half_t)v[0], (half_t)v[1], (half_t)v[2], (half_t)v[3]};
      *reinterpret_cast<half4_t*>(dst) = h;
    } else {
      floatx4 f = {v[0], v[1], v[2], v[3]};
      *reinterpret_cast<floatx4*>(dst) = f;
    }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e)
      if (n + e < N) store_one<OutT>(out, m, n + e, v[e], tp);
  }
}

// ---------------------------------------------------------------------------------------------
// fp32, plain vector arithmetic: 64x64 tile, BK = 16, 256 threads, 4x4 outputs per thread.  Only
// for shapes the matrix-core kernel further down does not take (K not a multiple of 8, operands
// not 16-byte aligned).
__global__ void __launch_bounds__(256) gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                       int M, int N, int K, const int32_t* __restrict__ tpos,
                                                       const float* __restrict__ bias, int act, GemmOut out) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int tid = threadIdx.x;
  const long tp = tpos ? *tpos : 0;   // the counter's address is among the first arguments: requested at once, awaited by the epilogue
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tx = tid & 15, ty = tid >> 4;
  float acc[4][4] = {};
  const int lr = tid >> 2, lk = (tid & 3) * 4;   // this thread stages row lr, k-columns lk..lk+3
  for (int k0 = 0; k0 < K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int k = k0 + lk + i;
      int m = m0 + lr, n = n0 + lr;
      As[lk + i][lr] = (m < M && k < K) ? A[(size_t)m * K + k] : 0.f;
      Bs[lk + i][lr] = (n < N && k < K) ? B[(size_t)n * K + k] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      float v = acc[i][j] + (bias ? bias[n] : 0.f);
      v = activate(v, act);
      store_one<float>(out, m, n, v, tp);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// fp16 MFMA.  Block tile BM x BN x BK, four wavefronts each owning a WM x WN sub-tile made of
// 32x32 MFMA blocks.
//
// Latency hiding: at these sizes (M = batch*beam <= a few hundred rows) a k-iteration's MFMA work
// is far shorter than a trip to HBM, so the loads of the next D k-tiles are kept in flight in
// registers (D "stages", statically indexed by unrolling the k-loop D times) while the current
// tile is multiplied out of LDS.  LDS is double buffered, one barrier per k-iteration: tile kt is
// written to buffer kt&1 before the barrier and read after it; the buffer it overwrites was last
// read two iterations ago, which every wavefront has left behind by then.
// LDS rows are padded by 8 halves so the 16-byte fragment reads of consecutive rows hit distinct
// banks.  The MFMA is issued as D = Bfrag x Afrag, i.e. D[n][m]: a lane then owns four
// consecutive n of one m, which makes the epilogue store an aligned 8- or 16-byte vector.
// Parameter order (all product kernels): the operands and the shape come first, so that they are
// among the arguments that arrive in scalar registers with the wavefront and the first tile can be
// requested at once; the output description, needed only by the epilogue, is fetched meanwhile.
// Workgroup ids are dealt round-robin to the 8 XCDs (each with its own L2), so the id is remapped
// to give every XCD a contiguous run of tiles, m fastest: the tiles that share a weight tile then
// share an L2.
template <int BM, int BN, int BK, int WM, int WN, int D, bool KTAIL, bool SPLIT, typename OutT, int KG = 1>
__global__ void __launch_bounds__(64 * (BM / WM) * (BN / WN) * KG) gemm_f16_kernel(const half_t* __restrict__ A, const half_t* __restrict__ B,
                                                       int M, int N, int K, int splits,
                                                       const int32_t* __restrict__ tpos,
                                                       const half_t* __restrict__ bias, int act, int vec_ok,
                                                       GemmOut out) {
  constexpr int LDK = BK + 8;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int WAVES_N = BN / WN;
  constexpr int VPR = BK / 8;   // 16-byte vectors per tile row
  // KG = 2: two wavefronts per wave tile, each multiplying one half of every k-tile (all of them load
  // the tile); their accumulators are added through LDS at the end
  constexpr int NT = 64 * (BM / WM) * (BN / WN) * KG;   // threads
  static_assert(KG == 1 || (KG == 2 && WM == 32 && WN == 32 && BK % 32 == 0), "k-groups: 32x32 wave tiles only");
  static_assert(NT == 256 || NT == 512, "four or eight wavefronts");
  constexpr int AV = BM * VPR / NT, BV = BN * VPR / NT;   // vectors per thread
  static_assert(AV >= 1 && BV >= 1, "tile too small");
  // LDS comes from the launch (dynamic), so that tiles above the 64 KB static limit can be used
  extern __shared__ __attribute__((aligned(16))) half_t lds_tiles[];
  half_t(*As)[BM * LDK] = reinterpret_cast<half_t(*)[BM * LDK]>(lds_tiles);
  half_t(*Bs)[BN * LDK] = reinterpret_cast<half_t(*)[BN * LDK]>(lds_tiles + 2 * BM * LDK);

  const int tid = threadIdx.x, lane = tid & 63;
  constexpr int TILE_WAVES = (BM / WM) * (BN / WN);
  const int wave = (tid >> 6) % TILE_WAVES, kgrp = (tid >> 6) / TILE_WAVES;   // wave tile, k-group
  const long tp = tpos ? *tpos : 0;   // the counter's address is among the first arguments: requested at once, awaited by the epilogue
  const int mt = (M + BM - 1) / BM, nt = (N + BN - 1) / BN, total = mt * nt;
  int id = blockIdx.x;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
  const int m0 = (id % mt) * BM, n0 = (id / mt) * BN;
  const int wm = (wave / WAVES_N) * WM, wn = (wave % WAVES_N) * WN;

  // Loads are unconditional (rows clamped to the last valid one, k-tile index clamped by the
  // caller) so that the k-loop body is straight-line code and the compiler can wait for just the
  // oldest stage (vmcnt = loads of the younger stages) instead of draining all of them.
  half8_t ra[D][AV], rb[D][BV];
  auto gload = [&](half8_t(&a)[AV], half8_t(&b)[BV], int k0) {
#pragma unroll
    for (int i = 0; i < AV; ++i) {
      int v = tid + i * NT, row = v / VPR, kc = (v % VPR) * 8;
      int m = min(m0 + row, M - 1);
      int kk = KTAIL ? min(k0 + kc, K - 8) : k0 + kc;
      a[i] = *reinterpret_cast<const half8_t*>(A + (size_t)m * K + kk);
    }
#pragma unroll
    for (int i = 0; i < BV; ++i) {
      int v = tid + i * NT, row = v / VPR, kc = (v % VPR) * 8;
      int n = min(n0 + row, N - 1);
      int kk = KTAIL ? min(k0 + kc, K - 8) : k0 + kc;
      b[i] = *reinterpret_cast<const half8_t*>(B + (size_t)n * K + kk);
    }
  };
  auto sstore = [&](const half8_t(&a)[AV], const half8_t(&b)[BV], int buf, int k0) {
    const half8_t zero = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < AV; ++i) {
      int v = tid + i * NT, row = v / VPR, kc = (v % VPR) * 8;
      *reinterpret_cast<half8_t*>(&As[buf][row * LDK + kc]) = (KTAIL && k0 + kc >= K) ? zero : a[i];
    }
#pragma unroll
    for (int i = 0; i < BV; ++i) {
      int v = tid + i * NT, row = v / VPR, kc = (v % VPR) * 8;
      *reinterpret_cast<half8_t*>(&Bs[buf][row * LDK + kc]) = (KTAIL && k0 + kc >= K) ? zero : b[i];
    }
  };

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // this lane's bias values: requested behind the first tiles (whose arrival the loop waits for
  // first), four consecutive columns per 8-byte load where the row allows it
  float bv[TN][4][4];
  auto load_bias = [&]() {
    const bool bias_vec = (reinterpret_cast<uintptr_t>(bias) & 7) == 0;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int n4 = n0 + wn + j * 32 + vg * 8 + (lane >> 5) * 4;
        if (SPLIT || !bias) {
#pragma unroll
          for (int e = 0; e < 4; ++e) bv[j][vg][e] = 0.f;
        } else if (bias_vec && n4 + 3 < N) {
          const half4_t b4 = *reinterpret_cast<const half4_t*>(bias + n4);
#pragma unroll
          for (int e = 0; e < 4; ++e) bv[j][vg][e] = (float)b4[e];
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) bv[j][vg][e] = (float)bias[min(n4 + e, N - 1)];
        }
      }
  };

  // Split-K: gridDim.y workgroups share an output tile; each multiplies an equal share of the
  // k-tiles and writes its fp32 partial sums (no bias) to its own [M,N] slab; the consumer adds
  // the slabs in a fixed order, so the result does not depend on scheduling.
  const int nk_all = (K + BK - 1) / BK;
  const int nk = SPLIT ? nk_all / splits : nk_all;   // splits = gridDim.y, as an argument: no trip for it
  if constexpr (SPLIT) {
    A += (size_t)blockIdx.y * nk * BK;
    B += (size_t)blockIdx.y * nk * BK;
  }
  static_assert(D % 2 == 0, "tile kt always uses LDS buffer kt & 1 = stage & 1");
  constexpr int KS = BK / 16 / KG;                   // MFMA k-steps per tile and k-group
  const int kg0 = kgrp * (BK / KG);                  // this k-group's first column of a tile
  constexpr bool kSingle = (TM * TN == 1);           // one output block per wave: use two accumulators
  floatx16 acc2;                                     // so consecutive MFMAs do not wait on each other
  if constexpr (kSingle)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc2[e] = 0.f;
  const int fr = lane & 31, fk = (lane >> 5) * 8;
  auto compute = [&](int buf) {
    if constexpr (kSingle) {
      half8_t af[KS], bf[KS];
#pragma unroll
      for (int i = 0; i < KS; ++i) {
        af[i] = *reinterpret_cast<const half8_t*>(&As[buf][(wm + fr) * LDK + kg0 + i * 16 + fk]);
        bf[i] = *reinterpret_cast<const half8_t*>(&Bs[buf][(wn + fr) * LDK + kg0 + i * 16 + fk]);
      }
#pragma unroll
      for (int i = 0; i < KS; ++i) {
        if (i & 1) acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[i], af[i], acc2, 0, 0, 0);
        else acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[i], af[i], acc[0][0], 0, 0, 0);
      }
    } else {
      // fragments of k-step i+1 are fetched from LDS while the MFMAs of k-step i run
      half8_t af[2][TM], bf[2][TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[0][i] = *reinterpret_cast<const half8_t*>(&As[buf][(wm + i * 32 + fr) * LDK + fk]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bf[0][j] = *reinterpret_cast<const half8_t*>(&Bs[buf][(wn + j * 32 + fr) * LDK + fk]);
#pragma unroll
      for (int s = 0; s < KS; ++s) {
        const int cur = s & 1, nxt = cur ^ 1;
        if (s + 1 < KS) {
#pragma unroll
          for (int i = 0; i < TM; ++i)
            af[nxt][i] = *reinterpret_cast<const half8_t*>(&As[buf][(wm + i * 32 + fr) * LDK + (s + 1) * 16 + fk]);
#pragma unroll
          for (int j = 0; j < TN; ++j)
            bf[nxt][j] = *reinterpret_cast<const half8_t*>(&Bs[buf][(wn + j * 32 + fr) * LDK + (s + 1) * 16 + fk]);
        }
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[cur][j], af[cur][i], acc[i][j], 0, 0, 0);
      }
    }
  };
  // Register slot s holds tile s (mod D).  Per iteration: the NEXT tile goes from its slot to the
  // other LDS buffer and the slot is refilled D tiles ahead, then the current tile is multiplied,
  // then one barrier: it orders this iteration's LDS writes before the next iteration's reads and
  // this iteration's reads before the writes of the iteration after.
#pragma unroll
  for (int s = 0; s < D; ++s) gload(ra[s], rb[s], min(s, nk - 1) * BK);
  load_bias();
  sstore(ra[0], rb[0], 0, 0);
  gload(ra[0], rb[0], min(D, nk - 1) * BK);
  __syncthreads();
  int it = 0;
  for (; it + D < nk; it += D) {
#pragma unroll
    for (int s = 0; s < D; ++s) {
      const int kt = it + s;
      const int sn = (s + 1) % D;
      sstore(ra[sn], rb[sn], (s + 1) & 1, (kt + 1) * BK);
      gload(ra[sn], rb[sn], min(kt + 1 + D, nk - 1) * BK);   // past the end: a redundant load, never used
      compute(s & 1);
      __syncthreads();
    }
  }
#pragma unroll
  for (int s = 0; s < D; ++s) {   // the last 1..D tiles: already in registers or in LDS
    const int kt = it + s;
    if (kt < nk) {
      const int sn = (s + 1) % D;
      if (kt + 1 < nk) sstore(ra[sn], rb[sn], (s + 1) & 1, (kt + 1) * BK);
      compute(s & 1);
      __syncthreads();
    }
  }
  if constexpr (kSingle)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[0][0][e] += acc2[e];
  if constexpr (KG == 2) {
    // the last loop iteration ended with a barrier: the tile buffers are free
    float* red = reinterpret_cast<float*>(lds_tiles);   // [TILE_WAVES][16][64]
    if (kgrp == 1) {
#pragma unroll
      for (int e = 0; e < 16; ++e) red[(wave * 16 + e) * 64 + lane] = acc[0][0][e];
    }
    __syncthreads();
    if (kgrp == 1) return;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[0][0][e] += red[(wave * 16 + e) * 64 + lane];
  }

  // epilogue: lane owns m = .. + (lane & 31) and, per group vg, n = .. + vg*8 + (lane>>5)*4 + 0..3
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm + i * 32 + (lane & 31);
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int n = n0 + wn + j * 32 + vg * 8 + (lane >> 5) * 4;
        if (n >= N) continue;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          v[e] = activate(acc[i][j][vg * 4 + e] + bv[j][vg][e], act);
        }
        store4<OutT, SPLIT>(out, m, n, v, M, N, vec_ok, (int)blockIdx.y, tp);
      }
    }
  }
  if constexpr (std::is_same<OutT, float>::value && !SPLIT) {
    // (largest, sum of exponentials) of every (row, 32-column group), as in the large-tile kernel below: a 32x32
    // block holds a group's 32 columns of a row in the two lanes (m, half 0) and (m, half 1)
    if (out.stats) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm + i * 32 + (lane & 31);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int nb = n0 + wn + j * 32;
          if (nb >= N) continue;   // the same in every lane
          float x[16], mx = -INFINITY;
#pragma unroll
          for (int vg = 0; vg < 4; ++vg)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int n = nb + vg * 8 + (lane >> 5) * 4 + e;
              x[vg * 4 + e] = n < N ? activate(acc[i][j][vg * 4 + e] + bv[j][vg][e], act) : -INFINITY;
              mx = fmaxf(mx, x[vg * 4 + e]);
            }
          mx = max_lane_xor<32>(mx);   // finite: column nb exists
          float z = 0.f;
#pragma unroll
          for (int q = 0; q < 16; ++q) z += __expf(x[q] - mx);
          z = add_lane_xor<32>(z);
          if (lane < 32 && m < M) {
            float* st = out.stats + ((size_t)m * out.stats_groups + nb / 32) * 2;
            st[0] = mx;
            st[1] = z;
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// The same product with the tiles loaded straight into LDS (global_load_lds_dwordx4: no staging registers, no
// LDS write instructions), ST k-tiles deep.  A load instruction of a wavefront fills one contiguous KB of LDS,
// lane l at byte 16 l: eight tile rows of 128 B (BK = 64).  Which 16 bytes of its row a lane fetches is free, so the
// row's eight chunks are stored permuted, chunk c of tile row r in slot c ^ ((r >> 1) & 7): the 16 lanes of a fragment
// read that are served together (16 consecutive rows, one chunk) then fall on 16 distinct groups of four banks
// without any padding.  Tile kt lives in stage kt % ST; loads complete in order, so a wavefront knows its share of a
// tile has landed from the number of younger requests that may still be in flight, and one barrier per k-tile makes
// the shares of all wavefronts visible.  32 x 32 wave tiles, two accumulators taking turns; K a multiple of 64.
// Measured against the register-staged kernel the gain is small (0.6 us of 12.9): either way a CU takes in its
// tiles at about 31 B per clock, which is what bounds these products at 512 rows.
template <int BM, int BN, bool SPLIT, typename OutT, int ST>
__global__ void __launch_bounds__(64 * (BM / 32) * (BN / 32)) gemm_f16_direct_kernel(const half_t* __restrict__ A, const half_t* __restrict__ B,
                                                       int M, int N, int K, int splits,
                                                       const int32_t* __restrict__ tpos,
                                                       const half_t* __restrict__ bias, int act, int vec_ok,
                                                       GemmOut out) {
  constexpr int BK = 64;
  constexpr int NW = (BM / 32) * (BN / 32);    // wavefronts
  constexpr int ROWS = BM + BN;                // tile rows of a stage: A's, then B's
  constexpr int STAGE = ROWS * BK * 2;         // bytes
  constexpr int LPW = ROWS / 8 / NW;           // load instructions per wavefront and k-tile
  static_assert(ROWS % (8 * NW) == 0 && BM % 16 == 0 && ST >= 4 && ST <= 6, "tile shape");
  extern __shared__ __attribute__((aligned(16))) half_t lds_tiles[];
  char* lds = reinterpret_cast<char*>(lds_tiles);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const long tp = tpos ? *tpos : 0;
  const int mt = (M + BM - 1) / BM, nt = (N + BN - 1) / BN, total = mt * nt;
  int id = blockIdx.x;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
  const int m0 = (id % mt) * BM, n0 = (id / mt) * BN;
  constexpr int WAVES_N = BN / 32;
  const int wm = (wave / WAVES_N) * 32, wn = (wave % WAVES_N) * 32;
  const int nk_all = K / BK;
  const int nk = SPLIT ? nk_all / splits : nk_all;
  if constexpr (SPLIT) {
    A += (size_t)blockIdx.y * nk * BK;
    B += (size_t)blockIdx.y * nk * BK;
  }
  // this lane's source of every load instruction of a k-tile (rows past the matrix: the last row, never stored)
  const half_t* src[LPW];
#pragma unroll
  for (int j = 0; j < LPW; ++j) {
    const int r = (wave * LPW + j) * 8 + (lane >> 3);            // tile row
    const int c = (lane & 7) ^ ((r >> 1) & 7);                   // the chunk that belongs in this lane's slot
    src[j] = (r < BM ? A + (size_t)min(m0 + r, M - 1) * K : B + (size_t)min(n0 + r - BM, N - 1) * K) + c * 8;
  }
  auto request = [&](int kt) {
    char* stage = lds + (kt % ST) * STAGE + wave * LPW * 1024;
#pragma unroll
    for (int j = 0; j < LPW; ++j)
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[j] + (size_t)kt * BK),
                                       (__attribute__((address_space(3))) void*)(stage + j * 1024), 16, 0, 0);
  };
  float bv[4][4];
  {
    const bool bias_vec = (reinterpret_cast<uintptr_t>(bias) & 7) == 0;
#pragma unroll
    for (int vg = 0; vg < 4; ++vg) {
      const int n4 = n0 + wn + vg * 8 + (lane >> 5) * 4;
      if (SPLIT || !bias) {
#pragma unroll
        for (int e = 0; e < 4; ++e) bv[vg][e] = 0.f;
      } else if (bias_vec && n4 + 3 < N) {
        const half4_t b4 = *reinterpret_cast<const half4_t*>(bias + n4);
#pragma unroll
        for (int e = 0; e < 4; ++e) bv[vg][e] = (float)b4[e];
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) bv[vg][e] = (float)bias[min(n4 + e, N - 1)];
      }
    }
  }
  // the bias values are older than every tile, so waiting for a tile also waits for them
#pragma unroll
  for (int s = 0; s < ST - 1; ++s)
    if (s < nk) request(s);
  floatx16 acc, acc2;
#pragma unroll
  for (int e = 0; e < 16; ++e) { acc[e] = 0.f; acc2[e] = 0.f; }
  const int fr = lane & 31, hf = lane >> 5;
  const int ra = wm + fr, rb = BM + wn + fr;                      // tile rows of this lane's fragments
  const int a_off = ra * 128, a_key = (ra >> 1) & 7, b_off = rb * 128, b_key = (rb >> 1) & 7;
  // vmcnt(n) alone: the other counters at their maxima (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
#define LSQ_WAIT_VM(n_) __builtin_amdgcn_s_waitcnt(((n_) & 15) | (((n_) >> 4) << 14) | (7 << 4) | (15 << 8))
  // until at most `tiles` of this wavefront's tile requests are still in flight (loads complete in order)
  auto wait_tiles = [&](int tiles) {
    if (tiles >= 3) LSQ_WAIT_VM(3 * LPW);
    else if (tiles == 2) LSQ_WAIT_VM(2 * LPW);
    else if (tiles == 1) LSQ_WAIT_VM(LPW);
    else LSQ_WAIT_VM(0);
  };
  half8_t af[2][4], bf[2][4];
  auto fragments = [&](int kt, half8_t (&a)[4], half8_t (&b)[4]) {
    const char* stage = lds + (kt % ST) * STAGE;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = i * 2 + hf;
      a[i] = *reinterpret_cast<const half8_t*>(stage + a_off + ((c ^ a_key) << 4));
      b[i] = *reinterpret_cast<const half8_t*>(stage + b_off + ((c ^ b_key) << 4));
    }
  };
  auto multiply = [&](const half8_t (&a)[4], const half8_t (&b)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i & 1) acc2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(b[i], a[i], acc2, 0, 0, 0);
      else acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(b[i], a[i], acc, 0, 0, 0);
    }
  };
  // Fragments of tile kt + 1 are read while tile kt is multiplied: the barrier aligns the wavefronts, and with
  // "read, then multiply" inside one iteration the LDS and the matrix cores would take turns for the whole CU.
  // Iteration kt: tile kt + 1 has landed (wait, barrier), which also means every wavefront has multiplied tile
  // kt - 1, so its stage takes tile kt + ST - 1; then the reads of tile kt + 1 and the multiplies of tile kt.
  wait_tiles(min(ST - 2, nk - 1));
  __builtin_amdgcn_s_barrier();
  fragments(0, af[0], bf[0]);
  auto iteration = [&](int kt, int cur) {
    const bool more = kt + 1 < nk;
    if (more) wait_tiles(min(ST - 3, nk - 2 - kt));
    __builtin_amdgcn_s_barrier();
    if (kt + ST - 1 < nk) request(kt + ST - 1);
    if (more) fragments(kt + 1, af[cur ^ 1], bf[cur ^ 1]);
    multiply(af[cur], bf[cur]);
  };
  int kt = 0;
  for (; kt + 1 < nk; kt += 2) {
    iteration(kt, 0);
    iteration(kt + 1, 1);
  }
  if (kt < nk) iteration(kt, 0);
#undef LSQ_WAIT_VM
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] += acc2[e];
  const int m = m0 + wm + (lane & 31);
  if (m >= M) return;
#pragma unroll
  for (int vg = 0; vg < 4; ++vg) {
    const int n = n0 + wn + vg * 8 + (lane >> 5) * 4;
    if (n >= N) continue;
    float v[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) v[e] = activate(acc[vg * 4 + e] + bv[vg][e], act);
    store4<OutT, SPLIT>(out, m, n, v, M, N, vec_ok, (int)blockIdx.y, tp);
  }
}

// ---------------------------------------------------------------------------------------------
// Large products (vocabulary logits from 65 rows up, encoder and prefill layers): the same scheme with
// 64x32 .. 128x64 wave tiles and the k-loop ordered for overlap -- a k-tile's first fragments are read and
// its first matrix-core step issued BEFORE the next tile's LDS writes, and the global loads of the tile
// after that follow the second step, so that the LDS pipe works on writes while the matrix cores run
// (written in front of the multiplies, as in the kernel above, the writes of eight wavefronts queue ahead
// of every wavefront's first fragment read: 613 -> 690 TFLOP/s at 4096^3 with 128x128 tiles, and with
// 256x256 tiles of eight 128x64 wave tiles -- 96 B of LDS reads per clock and CU at full matrix-core rate
// instead of 192 -- 870-920).  K a multiple of BK; D register stages of global loads.
template <int BM, int BN, int BK, int WM, int WN, int D, typename OutT>
__global__ void __launch_bounds__(64 * (BM / WM) * (BN / WN)) gemm_f16_large_kernel(const half_t* __restrict__ A, const half_t* __restrict__ B,
                                                       int M, int N, int K, const int32_t* __restrict__ tpos,
                                                       const half_t* __restrict__ bias, int act, int vec_ok,
                                                       GemmOut out) {
  constexpr int LDK = BK + 8;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int WAVES_N = BN / WN;
  constexpr int VPR = BK / 8;
  constexpr int NT = 64 * (BM / WM) * (BN / WN);
  constexpr int AV = BM * VPR / NT, BV = BN * VPR / NT;
  constexpr int KS = BK / 16;
  static_assert(D == 2 && KS >= 2 && AV >= 1 && BV >= 1, "two register stages, two LDS buffers");
  extern __shared__ __attribute__((aligned(16))) half_t lds_tiles[];
  half_t(*As)[BM * LDK] = reinterpret_cast<half_t(*)[BM * LDK]>(lds_tiles);
  half_t(*Bs)[BN * LDK] = reinterpret_cast<half_t(*)[BN * LDK]>(lds_tiles + 2 * BM * LDK);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long tp = tpos ? *tpos : 0;
  const int mt = (M + BM - 1) / BM, nt = (N + BN - 1) / BN, total = mt * nt;
  int id = blockIdx.x;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
  const int m0 = (id % mt) * BM, n0 = (id / mt) * BN;
  const int wm = (wave / WAVES_N) * WM, wn = (wave % WAVES_N) * WN;
  const int nk = K / BK;
  half8_t ra[D][AV], rb[D][BV];
  auto gload = [&](half8_t(&a)[AV], half8_t(&b)[BV], int k0) {
#pragma unroll
    for (int i = 0; i < AV; ++i) {
      int v = tid + i * NT, row = v / VPR, kc = (v % VPR) * 8;
      a[i] = *reinterpret_cast<const half8_t*>(A + (size_t)min(m0 + row, M - 1) * K + k0 + kc);
    }
#pragma unroll
    for (int i = 0; i < BV; ++i) {
      int v = tid + i * NT, row = v / VPR, kc = (v % VPR) * 8;
      b[i] = *reinterpret_cast<const half8_t*>(B + (size_t)min(n0 + row, N - 1) * K + k0 + kc);
    }
  };
  auto sstore = [&](const half8_t(&a)[AV], const half8_t(&b)[BV], int buf) {
#pragma unroll
    for (int i = 0; i < AV; ++i) {
      int v = tid + i * NT, row = v / VPR, kc = (v % VPR) * 8;
      *reinterpret_cast<half8_t*>(&As[buf][row * LDK + kc]) = a[i];
    }
#pragma unroll
    for (int i = 0; i < BV; ++i) {
      int v = tid + i * NT, row = v / VPR, kc = (v % VPR) * 8;
      *reinterpret_cast<half8_t*>(&Bs[buf][row * LDK + kc]) = b[i];
    }
  };
  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  const int fr = lane & 31, fk = (lane >> 5) * 8;
  half8_t af[2][TM], bf[2][TN];
  auto frags = [&](int buf, int s, int slot) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
      af[slot][i] = *reinterpret_cast<const half8_t*>(&As[buf][(wm + i * 32 + fr) * LDK + s * 16 + fk]);
#pragma unroll
    for (int j = 0; j < TN; ++j)
      bf[slot][j] = *reinterpret_cast<const half8_t*>(&Bs[buf][(wn + j * 32 + fr) * LDK + s * 16 + fk]);
  };
  auto mfmas = [&](int slot) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[slot][j], af[slot][i], acc[i][j], 0, 0, 0);
  };
#pragma unroll
  for (int s = 0; s < D; ++s) gload(ra[s], rb[s], min(s, nk - 1) * BK);
  // this lane's bias values: requested behind the first tiles, or (eight accumulator tiles, which with them
  // would not fit the 256 registers of two wavefronts per SIMD) after the k-loop
  constexpr bool BIAS_LATE = TM * TN >= 8;
  float bv[TN][4][4];
  auto load_bias = [&]() {
    const bool bias_vec = (reinterpret_cast<uintptr_t>(bias) & 7) == 0;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int n4 = n0 + wn + j * 32 + vg * 8 + (lane >> 5) * 4;
        if (!bias) {
#pragma unroll
          for (int e = 0; e < 4; ++e) bv[j][vg][e] = 0.f;
        } else if (bias_vec && n4 + 3 < N) {
          const half4_t b4 = *reinterpret_cast<const half4_t*>(bias + n4);
#pragma unroll
          for (int e = 0; e < 4; ++e) bv[j][vg][e] = (float)b4[e];
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) bv[j][vg][e] = (float)bias[min(n4 + e, N - 1)];
        }
      }
  };
  if (!BIAS_LATE) load_bias();
  sstore(ra[0], rb[0], 0);
  gload(ra[0], rb[0], min(D, nk - 1) * BK);
  __syncthreads();
  // iteration kt: tile kt is in LDS buffer kt & 1, register slot (kt + 1) % D holds tile kt + 1
  for (int it = 0; it < nk; it += D) {
#pragma unroll
    for (int s = 0; s < D; ++s) {
      const int kt = it + s;
      if (kt >= nk) break;
      const int buf = s & 1, sn = (s + 1) % D;
      const bool more = kt + 1 < nk;
      frags(buf, 0, 0);
#pragma unroll
      for (int q = 0; q < KS; ++q) {
        if (q + 1 < KS) frags(buf, q + 1, (q + 1) & 1);
        mfmas(q & 1);
        if (q == 0 && more) sstore(ra[sn], rb[sn], buf ^ 1);
        if (q == 1 && more) gload(ra[sn], rb[sn], min(kt + 1 + D, nk - 1) * BK);   // past the end: redundant, never used
      }
      __syncthreads();
    }
  }
  if (BIAS_LATE) load_bias();
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm + i * 32 + (lane & 31);
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int vg = 0; vg < 4; ++vg) {
        const int n = n0 + wn + j * 32 + vg * 8 + (lane >> 5) * 4;
        if (n >= N) continue;
        float v[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = activate(acc[i][j][vg * 4 + e] + bv[j][vg][e], act);
        store4<OutT, false>(out, m, n, v, M, N, vec_ok, 0, tp);
      }
    }
  }
  if constexpr (std::is_same<OutT, float>::value) {
    // (largest, sum of exponentials) of every (row, 32-column group): a wave tile holds a group's 32 columns of a
    // row in the two lanes (m, half 0) and (m, half 1)
    if (out.stats) {
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm + i * 32 + (lane & 31);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int nb = n0 + wn + j * 32;
          if (nb >= N) continue;   // the same in every lane
          float x[16], mx = -INFINITY;
#pragma unroll
          for (int vg = 0; vg < 4; ++vg)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int n = nb + vg * 8 + (lane >> 5) * 4 + e;
              x[vg * 4 + e] = n < N ? activate(acc[i][j][vg * 4 + e] + bv[j][vg][e], act) : -INFINITY;
              mx = fmaxf(mx, x[vg * 4 + e]);
            }
          mx = max_lane_xor<32>(mx);   // finite: column nb exists
          float z = 0.f;
#pragma unroll
          for (int q = 0; q < 16; ++q) z += __expf(x[q] - mx);
          z = add_lane_xor<32>(z);
          if (lane < 32 && m < M) {
            float* st = out.stats + ((size_t)m * out.stats_groups + nb / 32) * 2;
            st[0] = mx;
            st[1] = z;
          }
        }
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Weights in fragment order, for the skinny kernels below.  Read from row-major rows, an MFMA
// weight fragment is 16 bytes from each of 32 rows: 32 cache lines per load instruction, of which
// the texture path retires few per clock.  Stored as [column block of 32][k-step of 16][lane][8]
// the same fragment is one contiguous KB, and a skinny product is 1.2-1.5 us shorter (6.4 -> 5.0 us
// for 4 rows x 3072 x 1024, 20.0 -> 15.6 us for 32 rows of the 32000 x 1024 vocabulary product).
// The model's matrices are packed once at load time next to their row-major copies (which the
// tiled kernels and the embedding lookup keep using) and found here by the row-major pointer.
namespace {
struct PackedEntry { const half_t* packed; int N, K; };
std::unordered_map<const void*, PackedEntry> g_packed;

const half_t* packed_of(const void* plain, int N, int K) {
  auto it = g_packed.find(plain);
  return (it != g_packed.end() && it->second.N == N && it->second.K == K) ? it->second.packed : nullptr;
}

__global__ void __launch_bounds__(256) pack_weights_kernel(const half_t* __restrict__ src, half_t* __restrict__ dst,
                                                           int N, int K, size_t chunks) {
  const size_t c = (size_t)blockIdx.x * 256 + threadIdx.x;   // one 16-byte piece of the packed matrix
  if (c >= chunks) return;
  const int ksteps = K / 16;
  const int lane = (int)(c & 63);
  const size_t frag = c >> 6;
  const int ks = (int)(frag % ksteps), nb = (int)(frag / ksteps);
  const int row = nb * 32 + (lane & 31), k = ks * 16 + (lane >> 5) * 8;
  half8_t v = {0, 0, 0, 0, 0, 0, 0, 0};
  if (row < N) v = *reinterpret_cast<const half8_t*>(src + (size_t)row * K + k);
  *reinterpret_cast<half8_t*>(dst + c * 8) = v;
}
}  // namespace

size_t gemm_packed_bytes(int N, int K) { return K % 16 == 0 ? (size_t)((N + 31) / 32) * 32 * K * sizeof(half_t) : 0; }

hipError_t launch_pack_weights(const void* plain, void* packed, int N, int K, hipStream_t s) {
  if (N <= 0 || K <= 0 || K % 16 != 0) return hipErrorInvalidValue;
  const size_t chunks = gemm_packed_bytes(N, K) / 16;
  pack_weights_kernel<<<(unsigned)((chunks + 255) / 256), 256, 0, s>>>((const half_t*)plain, (half_t*)packed, N, K, chunks);
  return hipGetLastError();
}

void gemm_register_packed(const void* plain, const void* packed, int N, int K) {
  g_packed[plain] = PackedEntry{(const half_t*)packed, N, K};
}

const void* gemm_packed_weights(const void* plain, int N, int K) { return packed_of(plain, N, K); }

void gemm_clear_packed() { g_packed.clear(); }

// ---------------------------------------------------------------------------------------------
// Skinny fp16 GEMM for M <= 32*TM rows (few hypotheses alive, or small batches): the product is
// a stream of weights, so the job is to keep many weight bytes in flight from many CUs.
// A workgroup owns 32 output columns and all rows; its four wavefronts take every fourth 16-wide
// k-step, load their MFMA fragments straight from global memory (16 bytes per lane, no LDS and no
// barrier in the loop, U k-steps in flight per wavefront: the launcher picks U so that a
// wavefront's share of K is covered in as few passes, with as few padded loads, as possible),
// and their four partial tiles are added through LDS at the end.  gridDim.y > 1 additionally splits K across workgroups (SPLIT, fp32
// slabs for the LayerNorm consumer).
template <int TM, int U, bool SPLIT, typename OutT>
__global__ void __launch_bounds__(256) gemm_f16_skinny_kernel(const half_t* __restrict__ A,
                                                              const half_t* __restrict__ B,
                                                              const half_t* __restrict__ Bp, int M, int N,
                                                              int K, int splits, const int32_t* __restrict__ tpos,
                                                              const half_t* __restrict__ bias, int act,
                                                              int vec_ok, GemmOut out) {
  __shared__ float red[4][TM][16][64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long tp = tpos ? *tpos : 0;   // the counter's address is among the first arguments: requested at once, awaited by the epilogue
  const int n0 = blockIdx.x * 32;
  const int fr = lane & 31, fk = (lane >> 5) * 8;
  const int ksteps_all = K / 16;                      // K % 16 == 0 is checked by the launcher
  const int ksteps = SPLIT ? ksteps_all / splits : ksteps_all;   // splits = gridDim.y
  const int ks0 = SPLIT ? (int)blockIdx.y * ksteps : 0;
  // weights: row-major rows (32 cache lines per fragment load), or, when the caller has them in
  // fragment order (Bp), one contiguous KB per fragment: 512 halves per (column block, k-step)
  const half_t* bp = Bp ? Bp + (size_t)blockIdx.x * ksteps_all * 512 + lane * 8 : B + (size_t)min(n0 + fr, N - 1) * K + fk;
  const size_t bstep = Bp ? 512 : 16;
  const half_t* ap[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) ap[i] = A + (size_t)min(i * 32 + fr, M - 1) * K + fk;
  floatx16 acc[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  const int ks_end = ks0 + ksteps;
  // Every pass requests U k-steps before using any.  A k-step past the end of this wavefront's
  // share re-reads the last valid one (no branch around the loads, so all U stay in flight) and
  // its weight fragment is replaced by zeros.
  for (int ks = ks0 + wave; ks < ks_end; ks += 4 * U) {
    half8_t bf[U], af[U][TM];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kc = min(ks + 4 * u, ks_end - 1);
      bf[u] = *reinterpret_cast<const half8_t*>(bp + (size_t)kc * bstep);
#pragma unroll
      for (int i = 0; i < TM; ++i) af[u][i] = *reinterpret_cast<const half8_t*>(ap[i] + (size_t)kc * 16);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (ks + 4 * u >= ks_end) {
#pragma unroll
        for (int e = 0; e < 8; ++e) bf[u][e] = (half_t)0.f;
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[u], af[u][i], acc[i], 0, 0, 0);
    }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) red[wave][i][e][lane] = acc[i][e];
  __syncthreads();
  // thread (vg = wave, lane) finishes the four outputs m = i*32 + (lane & 31), n = n0 + vg*8 + (lane>>5)*4 + 0..3
  const int vg = wave;
  const int n = n0 + vg * 8 + (lane >> 5) * 4;
  constexpr bool kStats = !SPLIT && std::is_same<OutT, float>::value;
  __shared__ float st_m[kStats ? 4 : 1][TM][32], st_z[kStats ? 4 : 1][TM][32];
  const bool stats = kStats && out.stats != nullptr;   // the same in every thread
  if (n >= N && !stats) return;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = i * 32 + (lane & 31);
    float v[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int r = vg * 4 + e;
      v[e] = (red[0][i][r][lane] + red[1][i][r][lane]) + (red[2][i][r][lane] + red[3][i][r][lane]);
      if (!SPLIT && bias) v[e] += (float)bias[min(n + e, N - 1)];
      v[e] = activate(v[e], act);
    }
    if (m < M && n < N) store4<OutT, SPLIT>(out, m, n, v, M, N, vec_ok, (int)blockIdx.y, tp);
    if constexpr (kStats) {
      if (stats) {
        // (largest, sum of exponentials) of the workgroup's 32 columns, row by row: this thread's four
        // columns, the other half of the lanes, then (through LDS) the four wavefronts
        float mx = -INFINITY, z = 0.f;
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n + e < N) mx = fmaxf(mx, v[e]);
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (n + e < N) z += __expf(v[e] - mx);
        const float m2 = lane_xor<32>(mx), z2 = lane_xor<32>(z);
        merge_stat(mx, z, m2, z2);
        if (lane < 32) { st_m[wave][i][lane] = mx; st_z[wave][i][lane] = z; }
      }
    }
  }
  if constexpr (kStats) {
    if (stats) {
      __syncthreads();   // every thread of the workgroup gets here (no early return on this path)
      if (wave == 0 && lane < 32) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const int m = i * 32 + lane;
          if (m >= M) continue;
          float mx = st_m[0][i][lane], z = st_z[0][i][lane];
#pragma unroll
          for (int w = 1; w < 4; ++w) merge_stat(mx, z, st_m[w][i][lane], st_z[w][i][lane]);
          float* st = out.stats + ((size_t)m * out.stats_groups + blockIdx.x) * 2;
          st[0] = mx;
          st[1] = z;
        }
      }
    }
  }
}

constexpr int kSkinnyRows = 64;   // above this the LDS-tiled kernel is faster

// Products with an epilogue (bias, activation, cache append, statistics): between 33 and 64 rows the skinny kernel's
// two row blocks re-read the input rows in every 32-column workgroup, which from k = 768 on costs more than the
// tiled kernels' LDS staging (per launch at 64 rows, skinny vs tiled: QKV of d = 1024 9.4 vs 8.0 us, of d = 768 8.4 vs
// 7.4; FFN1 of d = 1024 9.4 vs 8.1; vocabulary 32000 x 1024 31.2 vs 23.0, 50257 x 768 53.0 vs 35.1; but FFN1 of
// d = 512 6.5 vs 7.1, vocabulary 32000 x 512 16.7 vs 17.9).  Split-K partial products stay skinny up to 64 rows
// (d x d: 4.5 vs 5.1-5.3 us).
static bool skinny_rows(int M, int K) { return M <= 32 || (M <= kSkinnyRows && K < 768); }

// k-steps requested per pass for a wavefront that owns `per_wave` of them: at most `cap`
// (registers), and among the sizes built, the one that pads the last pass least.
static int skinny_unroll(int per_wave, int cap) {
  static const int sizes[] = {16, 12, 8, 6, 4, 2};
  int best = 2, best_cost = 1 << 30;
  for (int u : sizes) {
    if (u > cap) continue;
    const int passes = (per_wave + u - 1) / u;
    const int cost = passes * 64 + (passes * u - per_wave);   // passes first, then padding
    if (cost < best_cost) { best = u; best_cost = cost; }
  }
  return best;
}

template <bool SPLIT, typename OutT>
static void run_skinny(const half_t* A, const half_t* B, const half_t* Bp, const half_t* bias, const GemmOut& out,
                       int M, int N, int K, int act, int vec_ok, int splits, hipStream_t s) {
  dim3 grid((N + 31) / 32, splits), blk(256);
  const int per_wave = (K / 16 / splits + 3) / 4;
#define LSQ_SKINNY(TM_, U_) \
  gemm_f16_skinny_kernel<TM_, U_, SPLIT, OutT><<<grid, blk, 0, s>>>(A, B, Bp, M, N, K, splits, out.tpos, bias, act, vec_ok, out)
  if (M <= 32) {
    switch (skinny_unroll(per_wave, 16)) {
      case 16: LSQ_SKINNY(1, 16); break;
      case 12: LSQ_SKINNY(1, 12); break;
      case 8: LSQ_SKINNY(1, 8); break;
      case 6: LSQ_SKINNY(1, 6); break;
      case 4: LSQ_SKINNY(1, 4); break;
      default: LSQ_SKINNY(1, 2); break;
    }
  } else {
    switch (skinny_unroll(per_wave, 8)) {
      case 8: LSQ_SKINNY(2, 8); break;
      case 6: LSQ_SKINNY(2, 6); break;
      case 4: LSQ_SKINNY(2, 4); break;
      default: LSQ_SKINNY(2, 2); break;
    }
  }
#undef LSQ_SKINNY
}

// ---------------------------------------------------------------------------------------------
// fp32 models: the same streaming scheme on the fp32 matrix cores (v_mfma_f32_32x32x2_f32).  A
// workgroup owns 32 output columns and a block of 32*TM rows (blockIdx.z), its four wavefronts take
// every fourth 8-wide k-step; a lane loads four consecutive k of its row (16 bytes), lanes 0-31 the
// first half of the step and lanes 32-63 the second, so MFMA i of a step multiplies k = 8s+i and
// 8s+4+i -- any pairing of k does, as long as both operands use the same one.  U steps in flight.
template <int TM, int U>
__global__ void __launch_bounds__(256) gemm_f32_stream_kernel(const float* __restrict__ A, const float* __restrict__ B,
                                                              int M, int N, int K, const int32_t* __restrict__ tpos,
                                                              const float* __restrict__ bias, int act, int vec_ok,
                                                              GemmOut out) {
  __shared__ float red[4][TM][16][64];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long tp = tpos ? *tpos : 0;   // the counter's address is among the first arguments: requested at once, awaited by the epilogue
  const int n0 = blockIdx.x * 32, mb = blockIdx.z * 32 * TM;
  const int fr = lane & 31, fk = (lane >> 5) * 4;
  const int ksteps = K / 8;                      // K % 8 == 0 is checked by the launcher
  const float* bp = B + (size_t)min(n0 + fr, N - 1) * K + fk;
  const float* ap[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) ap[i] = A + (size_t)min(mb + i * 32 + fr, M - 1) * K + fk;
  floatx16 acc[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
  for (int ks = wave; ks < ksteps; ks += 4 * U) {
    floatx4 bf[U], af[U][TM];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int kc = min(ks + 4 * u, ksteps - 1);
      bf[u] = *reinterpret_cast<const floatx4*>(bp + (size_t)kc * 8);
#pragma unroll
      for (int i = 0; i < TM; ++i) af[u][i] = *reinterpret_cast<const floatx4*>(ap[i] + (size_t)kc * 8);
    }
    // all U steps are requested before the first multiply: without this fence the instruction
    // scheduler sinks each load next to its use and waits for it there, one at a time
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (ks + 4 * u >= ksteps) bf[u] = floatx4{0.f, 0.f, 0.f, 0.f};   // a step past the end: multiplies by zero
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < TM; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(bf[u][q], af[u][i][q], acc[i], 0, 0, 0);
    }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) red[wave][i][e][lane] = acc[i][e];
  __syncthreads();
  const int vg = wave;
  const int n = n0 + vg * 8 + (lane >> 5) * 4;
  if (n >= N) return;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = mb + i * 32 + (lane & 31);
    if (m >= M) continue;
    float v[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const int r = vg * 4 + e;
      v[e] = (red[0][i][r][lane] + red[1][i][r][lane]) + (red[2][i][r][lane] + red[3][i][r][lane]);
      if (bias) v[e] += bias[min(n + e, N - 1)];
      v[e] = activate(v[e], act);
    }
    store4<float, false>(out, m, n, v, M, N, vec_ok, 0, tp);
  }
}

// ---------------------------------------------------------------------------------------------
// Skinny product whose input rows are made on the spot: A = LayerNorm(residual + split-K partial
// sums of the previous product + its bias), for the very few rows left near the end of a batch
// (M <= kLnFusedRows), where the step is nothing but launch latencies and a separate LayerNorm
// kernel costs as much as a product.  Every workgroup requests its weight fragments first, then
// its four wavefronts normalise the M rows (the same arithmetic, in the same order, as the
// stand-alone kernel) into LDS while those fragments travel, and the multiply reads A from LDS.
// Workgroup 0 also writes the normalised rows to x_new -- a different buffer from x_old, which the
// other workgroups are still reading -- for the next residual connection.
template <int U, typename OutT>
__global__ void __launch_bounds__(256) gemm_f16_skinny_ln_kernel(const half_t* __restrict__ Bp,
                                                                 const half_t* __restrict__ B, int M, int N, int K,
                                                                 const int32_t* __restrict__ tpos, LnInput ln,
                                                                 const half_t* __restrict__ bias, int act,
                                                                 int vec_ok, GemmOut out) {
  constexpr int NV = 2;   // K <= 1024: a lane owns at most two 8-element pieces of a row
  extern __shared__ __attribute__((aligned(16))) half_t a_rows[];   // [M][K + 8]
  __shared__ float red[4][16][64];
  const int LDA = K + 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const long tp = tpos ? *tpos : 0;   // the counter's address is among the first arguments: requested at once, awaited by the epilogue
  const int n0 = blockIdx.x * 32;
  const int fr = lane & 31, fk = (lane >> 5) * 8;
  const int ksteps = K / 16;
  const half_t* bp = Bp ? Bp + (size_t)blockIdx.x * ksteps * 512 + lane * 8 : B + (size_t)min(n0 + fr, N - 1) * K + fk;
  const size_t bstep = Bp ? 512 : 16;   // weights in fragment order: see gemm_f16_skinny_kernel
  half8_t bf[U];
#pragma unroll
  for (int u = 0; u < U; ++u) bf[u] = *reinterpret_cast<const half8_t*>(bp + (size_t)min(wave + 4 * u, ksteps - 1) * bstep);

  const size_t slab = (size_t)M * K;
  for (int r = wave; r < M; r += 4) {
    float v[NV][8], gv[NV][8], bv[NV][8];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int c = (j * 64 + lane) * 8;
      if (c < K) {
        float t[8], part[4][8];
#pragma unroll
        for (int sp = 0; sp < 4; ++sp)
          if (sp < ln.splits) Vec8<float>::load(ln.P + sp * slab + (size_t)r * K + c, part[sp]);
        Vec8<half_t>::load(ln.bias + c, t);
        Vec8<half_t>::load(ln.x_old + (size_t)r * K + c, v[j]);
        Vec8<half_t>::load(ln.g + c, gv[j]);
        Vec8<half_t>::load(ln.b + c, bv[j]);
        add_partials<4>(v[j], part, ln.splits, t);
      } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) { v[j][i] = 0.f; gv[j][i] = 0.f; bv[j][i] = 0.f; }
      }
    }
    float o[NV][8];
    layernorm_row<NV>(v, gv, bv, K, ln.eps, lane, o);
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int c = (j * 64 + lane) * 8;
      if (c < K) {
        Vec8<half_t>::store(&a_rows[r * LDA + c], o[j]);
        if (blockIdx.x == 0) Vec8<half_t>::store(ln.x_new + (size_t)r * K + c, o[j]);
      }
    }
  }
  __syncthreads();

  floatx16 acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  const half_t* ar = a_rows + min(fr, M - 1) * LDA + fk;
  for (int ks = wave; ks < ksteps; ks += 4 * U) {
    if (ks != wave) {   // K beyond one pass: later fragments are fetched here
#pragma unroll
      for (int u = 0; u < U; ++u) bf[u] = *reinterpret_cast<const half8_t*>(bp + (size_t)min(ks + 4 * u, ksteps - 1) * bstep);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const half8_t af = *reinterpret_cast<const half8_t*>(ar + min(ks + 4 * u, ksteps - 1) * 16);
      if (ks + 4 * u >= ksteps) {
#pragma unroll
        for (int e = 0; e < 8; ++e) bf[u][e] = (half_t)0.f;
      }
      acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf[u], af, acc, 0, 0, 0);
    }
  }
#pragma unroll
  for (int e = 0; e < 16; ++e) red[wave][e][lane] = acc[e];
  __syncthreads();
  const int vg = wave;
  const int n = n0 + vg * 8 + (lane >> 5) * 4;
  const int m = lane & 31;
  if (n >= N || m >= M) return;
  float v4[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int r = vg * 4 + e;
    v4[e] = (red[0][r][lane] + red[1][r][lane]) + (red[2][r][lane] + red[3][r][lane]);
    if (bias) v4[e] += (float)bias[min(n + e, N - 1)];
    v4[e] = activate(v4[e], act);
  }
  store4<OutT, false>(out, m, n, v4, M, N, vec_ok, 0, tp);
}

constexpr int kLnFusedRows = 8;

bool gemm_ln_supported(int dtype, int M, int K) {
  return dtype == DT_F16 && M >= 1 && M <= kLnFusedRows && K >= 16 && K <= 1024 && K % 16 == 0;
}

hipError_t launch_gemm_ln(const LnInput& ln, const void* B, const void* bias, const GemmOut& out, int M, int N,
                          int K, int act, hipStream_t s) {
  if (N <= 0) return hipSuccess;
  if (!gemm_ln_supported(DT_F16, M, K) || ln.splits < 1 || ln.splits > 4 || ln.x_old == ln.x_new) return hipErrorInvalidValue;
  int nseg = (N + out.seg_n - 1) / out.seg_n;
  if (nseg > 3) return hipErrorInvalidValue;
  int vec_ok = (out.seg_n % 4 == 0);
  for (int i = 0; i < nseg; ++i)
    if (out.ld[i] % 4 != 0 || out.tmul[i] % 4 != 0 || (reinterpret_cast<uintptr_t>(out.ptr[i]) & (out.f32_out ? 15 : 7)) != 0) vec_ok = 0;
  dim3 grid((N + 31) / 32), blk(256);
  const size_t lds = (size_t)M * (K + 8) * sizeof(half_t);
  const int per_wave = (K / 16 + 3) / 4;
  const half_t* b = (const half_t*)B;
  const half_t* bpk = packed_of(B, N, K);
  const half_t* bi = (const half_t*)bias;
#define LSQ_SKINNY_LN(U_)                                                                                          \
  do {                                                                                                             \
    if (out.f32_out) gemm_f16_skinny_ln_kernel<U_, float><<<grid, blk, lds, s>>>(bpk, b, M, N, K, out.tpos, ln, bi, act, vec_ok, out); \
    else gemm_f16_skinny_ln_kernel<U_, half_t><<<grid, blk, lds, s>>>(bpk, b, M, N, K, out.tpos, ln, bi, act, vec_ok, out);      \
  } while (0)
  switch (skinny_unroll(per_wave, 16)) {
    case 16: LSQ_SKINNY_LN(16); break;
    case 12: LSQ_SKINNY_LN(12); break;
    case 8: LSQ_SKINNY_LN(8); break;
    case 6: LSQ_SKINNY_LN(6); break;
    case 4: LSQ_SKINNY_LN(4); break;
    default: LSQ_SKINNY_LN(2); break;
  }
#undef LSQ_SKINNY_LN
  return hipGetLastError();
}

template <int BM, int BN, int BK>
constexpr size_t gemm_lds_bytes() { return (size_t)2 * (BM + BN) * (BK + 8) * sizeof(half_t); }

// Launch with the tile's LDS size; sizes above the default 64 KB limit are opted into once per kernel.
template <typename Kern>
static void launch_tiles(Kern kern, size_t lds, dim3 grid, int threads, hipStream_t s, const half_t* A, const half_t* B,
                         const half_t* bias, const GemmOut& out, int M, int N, int K, int act, int vec_ok) {
  if (lds > 64 * 1024) {
    static bool raised = false;   // one flag per instantiation of this template, i.e. per kernel
    if (!raised) {
      (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      raised = true;
    }
  }
  kern<<<grid, dim3(threads), lds, s>>>(A, B, M, N, K, (int)grid.y, out.tpos, bias, act, vec_ok, out);
}

template <int BM, int BN, int BK, int WM, int WN>
static void run_f16_large(const half_t* A, const half_t* B, const half_t* bias, const GemmOut& out, int M, int N,
                          int K, int act, int vec_ok, hipStream_t s) {
  dim3 grid(((N + BN - 1) / BN) * ((M + BM - 1) / BM));
  constexpr size_t lds = gemm_lds_bytes<BM, BN, BK>();
  constexpr int NT = 64 * (BM / WM) * (BN / WN);
  // LDS above the default 64 KB limit is opted into once per kernel
  if (out.f32_out) {
    auto kern = gemm_f16_large_kernel<BM, BN, BK, WM, WN, 2, float>;
    static bool raised = false;
    if (!raised) { (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); raised = true; }
    kern<<<grid, dim3(NT), lds, s>>>(A, B, M, N, K, out.tpos, bias, act, vec_ok, out);
  } else {
    auto kern = gemm_f16_large_kernel<BM, BN, BK, WM, WN, 2, half_t>;
    static bool raised = false;
    if (!raised) { (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); raised = true; }
    kern<<<grid, dim3(NT), lds, s>>>(A, B, M, N, K, out.tpos, bias, act, vec_ok, out);
  }
}

template <int BM, int BN, int BK, int WM, int WN, int D, int KG = 1>
static void run_f16(const half_t* A, const half_t* B, const half_t* bias, const GemmOut& out, int M, int N,
                    int K, int act, int vec_ok, hipStream_t s) {
  dim3 grid(((N + BN - 1) / BN) * ((M + BM - 1) / BM));
  constexpr size_t lds = gemm_lds_bytes<BM, BN, BK>();
  constexpr int NT = 64 * (BM / WM) * (BN / WN) * KG;
  const bool tail = (K % BK) != 0;
  if (out.f32_out) {
    if (tail) launch_tiles(gemm_f16_kernel<BM, BN, BK, WM, WN, D, true, false, float, KG>, lds, grid, NT, s, A, B, bias, out, M, N, K, act, vec_ok);
    else launch_tiles(gemm_f16_kernel<BM, BN, BK, WM, WN, D, false, false, float, KG>, lds, grid, NT, s, A, B, bias, out, M, N, K, act, vec_ok);
  } else {
    if (tail) launch_tiles(gemm_f16_kernel<BM, BN, BK, WM, WN, D, true, false, half_t, KG>, lds, grid, NT, s, A, B, bias, out, M, N, K, act, vec_ok);
    else launch_tiles(gemm_f16_kernel<BM, BN, BK, WM, WN, D, false, false, half_t, KG>, lds, grid, NT, s, A, B, bias, out, M, N, K, act, vec_ok);
  }
}

template <int BM, int BN, bool SPLIT, int ST>
static void run_f16_direct(const half_t* A, const half_t* B, const half_t* bias, const GemmOut& out, int M, int N,
                           int K, int act, int vec_ok, int splits, hipStream_t s) {
  dim3 grid(((N + BN - 1) / BN) * ((M + BM - 1) / BM), splits);
  constexpr size_t lds = (size_t)ST * (BM + BN) * 128;
  constexpr int NT = 64 * (BM / 32) * (BN / 32);
  if (out.f32_out) launch_tiles(gemm_f16_direct_kernel<BM, BN, SPLIT, float, ST>, lds, grid, NT, s, A, B, bias, out, M, N, K, act, vec_ok);
  else launch_tiles(gemm_f16_direct_kernel<BM, BN, SPLIT, half_t, ST>, lds, grid, NT, s, A, B, bias, out, M, N, K, act, vec_ok);
}

// How many ways the k-range of an [M,N,K] product is split when its consumer can add partial
// sums (the residual + LayerNorm kernel).  More slabs put more workgroups (and more wavefronts per
// CU) on a product whose output has too few tiles to fill 256 CUs, but every slab is M*N floats
// written and read again, and a workgroup's fixed cost is only worth paying for four k-tiles or
// more.  Tiled kernel: the most slabs that keep the launch within one workgroup per CU (measured
// at d = 512 and 1024, K = d and 4d, 65..512 rows: beyond 256 workgroups every step up is slower).
// Skinny kernel (32 columns per workgroup): up to 512 workgroups.
int gemm_partial_splits(int dtype, int M, int N, int K) {
  if (dtype != DT_F16 || K % 64 != 0) return 1;
  const int nk = K / 64;
  const bool skinny = M <= kSkinnyRows;
  const long tiles = skinny ? (N + 31) / 32 : (long)((M + 63) / 64) * ((N + 63) / 64);
  const long most = skinny ? 512 : 256;
  const int least = skinny ? 2 : 4;   // k-tiles per workgroup
  int S = 1;
  const int cap = 8;
  while (S < cap && nk % (S * 2) == 0 && nk / (S * 2) >= least && tiles * S * 2 <= most) S *= 2;
  return S;
}

// P[s][M][N] (fp32) = A[:, k-share s] . B[:, k-share s]^T for s < splits; no bias, no activation.
hipError_t launch_gemm_partials(int dtype, const void* A, const void* B, float* P, int M, int N, int K,
                                int splits, hipStream_t s) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (K <= 0 || splits < 1) return hipErrorInvalidValue;
  GemmOut out = plain_out(P, N);
  out.f32_out = 1;
  if (dtype == DT_F32 || splits == 1) return launch_gemm(dtype, A, B, nullptr, out, M, N, K, false, s);
  if (K % (64 * splits) != 0) return hipErrorInvalidValue;
  const int vec_ok = (N % 4 == 0) && (reinterpret_cast<uintptr_t>(P) & 15) == 0;
  if (M <= kSkinnyRows) {
    run_skinny<true, float>((const half_t*)A, (const half_t*)B, packed_of(B, N, K), nullptr, out, M, N, K, 0, vec_ok, splits, s);
    return hipGetLastError();
  }
  dim3 grid(((N + 63) / 64) * ((M + 63) / 64), splits), blk(256);
  gemm_f16_kernel<64, 64, 64, 32, 32, 4, false, true, float><<<grid, blk, gemm_lds_bytes<64, 64, 64>(), s>>>(
      (const half_t*)A, (const half_t*)B, M, N, K, splits, out.tpos, nullptr, 0, vec_ok, out);
  return hipGetLastError();
}

// every float16 product kernel launch_gemm chooses for a float32 output can fill GemmOut::stats
bool gemm_writes_stats(int dtype, int M, int N, int K) {
  return dtype == DT_F16 && M > 0 && N > 0 && K > 0 && K % 8 == 0;
}

hipError_t launch_gemm(int dtype, const void* A, const void* B, const void* bias, const GemmOut& out, int M,
                       int N, int K, int act /* activation: 0 none, 1 ReLU, 2 tanh-GELU */, hipStream_t s,
                       bool b_packed) {
  if (M <= 0 || N <= 0) return hipSuccess;
  if (K <= 0) return hipErrorInvalidValue;
  if (b_packed && !(dtype == DT_F16 && M <= kSkinnyRows && K % 16 == 0)) return hipErrorInvalidValue;
  if (out.stats && !(out.f32_out && gemm_writes_stats(dtype, M, N, K) && out.stats_groups >= (N + 31) / 32))
    return hipErrorInvalidValue;
  if (dtype == DT_F32) {
    if (K % 8 == 0 && ((reinterpret_cast<uintptr_t>(A) | reinterpret_cast<uintptr_t>(B)) & 15) == 0) {
      int nseg = (N + out.seg_n - 1) / out.seg_n;
      if (nseg > 3) return hipErrorInvalidValue;
      int vec_ok = (out.seg_n % 4 == 0);
      for (int i = 0; i < nseg; ++i)
        if (out.ld[i] % 4 != 0 || out.tmul[i] % 4 != 0 || (reinterpret_cast<uintptr_t>(out.ptr[i]) & 15) != 0) vec_ok = 0;
      const float* a = (const float*)A;
      const float* b = (const float*)B;
      const float* bi = (const float*)bias;
      const int per_wave = (K / 8 + 3) / 4;
      if (M <= 32) {
        dim3 grid((N + 31) / 32, 1, 1), blk(256);
        if (per_wave <= 8) gemm_f32_stream_kernel<1, 8><<<grid, blk, 0, s>>>(a, b, M, N, K, out.tpos, bi, act, vec_ok, out);
        else gemm_f32_stream_kernel<1, 16><<<grid, blk, 0, s>>>(a, b, M, N, K, out.tpos, bi, act, vec_ok, out);
      } else {
        dim3 grid((N + 31) / 32, 1, (M + 63) / 64), blk(256);
        gemm_f32_stream_kernel<2, 8><<<grid, blk, 0, s>>>(a, b, M, N, K, out.tpos, bi, act, vec_ok, out);
      }
      return hipGetLastError();
    }
    dim3 grid((N + 63) / 64, (M + 63) / 64), blk(256);   // odd K or unaligned operands: the plain tile kernel
    gemm_f32_kernel<<<grid, blk, 0, s>>>((const float*)A, (const float*)B, M, N, K, out.tpos, (const float*)bias, act, out);
    return hipGetLastError();
  }
  if (K % 8 != 0) return hipErrorInvalidValue;
  int nseg = (N + out.seg_n - 1) / out.seg_n;
  if (nseg > 3) return hipErrorInvalidValue;
  int vec_ok = (out.seg_n % 4 == 0);
  for (int i = 0; i < nseg; ++i)
    if (out.ld[i] % 4 != 0 || out.tmul[i] % 4 != 0 || (reinterpret_cast<uintptr_t>(out.ptr[i]) & (out.f32_out ? 15 : 7)) != 0) vec_ok = 0;
  // float rows of one segment that are not 16-byte aligned (an odd vocabulary size): dword-aligned vector stores
  if (!vec_ok && out.f32_out && nseg == 1 && (reinterpret_cast<uintptr_t>(out.ptr[0]) & 3) == 0) vec_ok = 2;
  const half_t* a = (const half_t*)A;
  const half_t* b = (const half_t*)B;
  const half_t* bi = (const half_t*)bias;
  long tiles128 = (long)((M + 127) / 128) * ((N + 127) / 128);
  // A vocabulary-sized product (125 or more tiles of 128 columns) of 33 to 64 rows runs the tiled kernel on 64x128
  // tiles: whole translations of 16 sentences of the big model 39.5 -> 39.0 ms, level for d = 512 and 768.  Up to 32
  // rows the skinny kernel stays: alone and with its weights coming from memory the tiled kernel is far ahead there
  // (32 rows of 32000 x 1024: 22.6 -> 14.4 us, of 50257 x 768: 31.9 -> 19.5 us), but inside a step, where much of the
  // embedding is still in the memory-side cache, it is level or behind (32 rows of 32000 x 512: 9.6 -> 12.0 us in the
  // step; translations of Transformer-base 25.1 -> 25.6 ms, of the GPT-2-small shape 57.1 -> 56.8 ms).
  // Fragment-ordered weights are read by the skinny kernel only.
  const bool wide = (N + 127) / 128 >= 125 && M > 32;
  if ((b_packed || (skinny_rows(M, K) && !wide)) && K % 16 == 0) {
    const half_t* bpk = b_packed ? b : packed_of(B, N, K);
    if (out.f32_out) run_skinny<false, float>(a, b, bpk, bi, out, M, N, K, act, vec_ok, 1, s);
    else run_skinny<false, half_t>(a, b, bpk, bi, out, M, N, K, act, vec_ok, 1, s);
  } else if (M <= 32)
    run_f16<32, 128, 64, 32, 32, 4>(a, b, bi, out, M, N, K, act, vec_ok, s);
  else if (M <= 64 && wide)
    run_f16<64, 128, 64, 32, 32, 4>(a, b, bi, out, M, N, K, act, vec_ok, s);
  else if (tiles128 >= 200 && K % 64 == 0) {
    // enough 128x128 tiles to fill the chip (vocabulary product from 65 rows up, encoder and prefill
    // layers).  256x256 tiles (144 KB of LDS, eight wavefronts of 128x64) once there are about as many of
    // those as CUs and more: half the LDS reads per FLOP (vocabulary product at 512 rows 54 -> 48 us,
    // 4096^3 613 -> 870 TFLOP/s); otherwise 128x128 tiles (72 KB, two workgroups per CU, eight wavefronts
    // of 64x32)
    const long tiles256 = (long)((M + 255) / 256) * ((N + 255) / 256);
    if (tiles256 >= 256) run_f16_large<256, 256, 64, 128, 64>(a, b, bi, out, M, N, K, act, vec_ok, s);
    else run_f16_large<128, 128, 64, 64, 32>(a, b, bi, out, M, N, K, act, vec_ok, s);
  } else if (tiles128 >= 200)
    run_f16<128, 128, 64, 64, 32, 2>(a, b, bi, out, M, N, K, act, vec_ok, s);   // ragged k
  else if ((long)((M + 63) / 64) * ((N + 63) / 64) > 256) {
    // more 64x64 tiles than CUs: eight wavefronts on a 64x128 tile move fewer operand bytes per FLOP
    // into the CU and keep its LDS pipe as busy as two four-wave workgroups would.  With k a multiple of 64 the
    // tiles go straight into LDS, five deep (in the step at 512 rows: QKV 12.9 -> 12.3 us, FFN1 13.2 -> 12.6 us;
    // the split-K products on 64x64 tiles lost 0.5 us with it and keep the register-staged kernel)
    if (K % 64 == 0 && !out.stats) run_f16_direct<64, 128, false, 5>(a, b, bi, out, M, N, K, act, vec_ok, 1, s);
    else run_f16<64, 128, 64, 32, 32, 4>(a, b, bi, out, M, N, K, act, vec_ok, s);
  }
  else if ((long)((M + 63) / 64) * ((N + 63) / 64) <= 128)
    // 64x64 tiles would leave half of the CUs or more without one: 32x64 tiles reach twice as many, and
    // each workgroup takes in 12 instead of 16 KB per k-tile (two wave tiles, two k-groups each);
    // measured on whole steps: 0.480 -> 0.460 ms at 128 rows of the big model, 0.491 -> 0.486 on big128
    // (32x32 tiles with four k-groups were no better)
    run_f16<32, 64, 64, 32, 32, 4, 2>(a, b, bi, out, M, N, K, act, vec_ok, s);
  else
    // at most one 64x64 tile per CU: a second set of four wavefronts multiplies the other half of
    // every k-tile (0.5-0.7 us off a 1024-deep product)
    run_f16<64, 64, 64, 32, 32, 4, 2>(a, b, bi, out, M, N, K, act, vec_ok, s);
  return hipGetLastError();
}

}  // namespace lsq
