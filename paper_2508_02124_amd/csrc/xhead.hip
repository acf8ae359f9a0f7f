// Content scores with the paper's full sampling tensor (Eq. 3, Delta in R^{n_h x d_h x n_h}; Listing 1
// flattens the values of all heads of a token before the projection), and their chain rule:
//   x[h, j] = sum_{g, c} v_{g, j, c} Delta[h, g, c],   z = exp(A_h softplus(x)),
//   dx = dz z A_h sigmoid(x),  dA_h = sum_j dz z softplus(x),
//   dDelta[h, g, c] = sum_j dx[h, j] v_{g, j, c},   dVz[j, g, c] = sum_h dx[h, j] Delta[h, g, c].
// Delta is [H_q, H_kv * d] row-major (the weight of a linear layer from the flattened values to the
// heads).  A [T x H_kv d] x [H_kv d x H_q] contraction with H_q <= 32 output columns and fp32
// weights.  bf16 values run on the matrix cores (the *_mfma_kernel pair below: the weights split into
// three bf16 terms, exact); fp32 values, the debug dtype, use fp32 vector FMAs from LDS tiles.
#include "common.h"

namespace dma {

constexpr int XT = 64;  // tokens per tile

template <int D> struct XTile {
  static constexpr int VS = D + 4;  // row stride of the fp32 V tile (floats): 16-byte row reads by 64 different rows
};

// V[t0 .. t0 + 64, g, :] -> vs (fp32, zero rows past T); a row is loaded by D / 8 lanes, 8 channels each
template <typename TV, int D>
__device__ __forceinline__ void stage_v_tile(const TV* __restrict__ V, float* vs, int t0, int g, int T, int H_kv) {
  constexpr int LPR = D / 8, RPP = 256 / LPR, NP = XT / RPP, VS = XTile<D>::VS;
  const int tid = threadIdx.x, sub = tid % LPR, rl = tid / LPR;
#pragma unroll
  for (int pass = 0; pass < NP; pass++) {
    const int r = pass * RPP + rl, t = t0 + r;
    float v[8];
#pragma unroll
    for (int e = 0; e < 8; e++) v[e] = 0.f;
    if (t < T) {
      const size_t roff = ((size_t)t * H_kv + g) * D + 8 * sub;
      if constexpr (sizeof(TV) == 2) {
        const uint4 raw = *reinterpret_cast<const uint4*>(V + roff);
        const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int e = 0; e < 4; e++) {
          v[2 * e] = __uint_as_float(u[e] << 16);
          v[2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
        }
      } else {
        const float4 x0 = *reinterpret_cast<const float4*>(V + roff);
        const float4 x1 = *reinterpret_cast<const float4*>(V + roff + 4);
        v[0] = x0.x; v[1] = x0.y; v[2] = x0.z; v[3] = x0.w;
        v[4] = x1.x; v[5] = x1.y; v[6] = x1.z; v[7] = x1.w;
      }
    }
    float* dst = vs + r * VS + 8 * sub;
    *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(dst + 4) = make_float4(v[4], v[5], v[6], v[7]);
  }
}

// Delta[h, g, :] for the HP (padded) heads -> ds[h][D]; rows past H_q are zero
template <int D>
__device__ __forceinline__ void stage_delta(const float* __restrict__ Delta, float* ds, int g, int H_q, int H_kv, int HP) {
  for (int idx = threadIdx.x; idx < HP * D; idx += 256) {
    const int h = idx / D, c = idx % D;
    ds[idx] = h < H_q ? Delta[((size_t)h * H_kv + g) * D + c] : 0.f;
  }
}

// x[r][hq * HPT + i], i < HPT, of the thread's token r = tid % 64 and head quarter hq = tid / 64, summed
// over all kv-heads.  hq is uniform in a wave, so the wave's Delta rows are read through the scalar
// path (no LDS traffic for them) and enter the FMAs as scalar operands; only the V tile goes
// through LDS.  Barriers inside: every thread of the workgroup calls it.
template <typename TV, int D, int HPT>
__device__ __forceinline__ void xhead_x(const TV* __restrict__ V, const float* __restrict__ Delta, float* vs,
                                        int t0, int T, int H_q, int H_kv, float (&x)[HPT]) {
  constexpr int VS = XTile<D>::VS;
  const int r = threadIdx.x & 63, hq = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // rows of Delta of this wave's heads (heads past H_q read the last head: their x is never used)
  const float* drow[HPT];
#pragma unroll
  for (int i = 0; i < HPT; i++) {
    const int h = hq * HPT + i < H_q ? hq * HPT + i : H_q - 1;
    drow[i] = Delta + (size_t)h * H_kv * D;
  }
#pragma unroll
  for (int i = 0; i < HPT; i++) x[i] = 0.f;
  for (int g = 0; g < H_kv; g++) {
    __syncthreads();  // the readers of the previous contents of vs are done
    stage_v_tile<TV, D>(V, vs, t0, g, T, H_kv);
    __syncthreads();
    const float* vr = vs + r * VS;
#pragma unroll 2
    for (int c = 0; c < D; c += 8) {
      const float4 v0 = *reinterpret_cast<const float4*>(vr + c);
      const float4 v1 = *reinterpret_cast<const float4*>(vr + c + 4);
#pragma unroll
      for (int i = 0; i < HPT; i++) {
        const float* w = drow[i] + g * D + c;  // wave-uniform address: scalar loads
        x[i] = fmaf(v0.x, w[0], x[i]);
        x[i] = fmaf(v0.y, w[1], x[i]);
        x[i] = fmaf(v0.z, w[2], x[i]);
        x[i] = fmaf(v0.w, w[3], x[i]);
        x[i] = fmaf(v1.x, w[4], x[i]);
        x[i] = fmaf(v1.y, w[5], x[i]);
        x[i] = fmaf(v1.z, w[6], x[i]);
        x[i] = fmaf(v1.w, w[7], x[i]);
      }
    }
  }
}

__device__ __forceinline__ float softplus_f(float x) { return fmaxf(x, 0.f) + log1pf(expf(-fabsf(x))); }

template <typename TV, int D, int HPT>
__global__ __launch_bounds__(256) void xhead_scores_kernel(const TV* __restrict__ V, const float* __restrict__ Delta,
                                                           const float* __restrict__ A, float* __restrict__ z, int T,
                                                           int H_q, int H_kv) {
  extern __shared__ float sm[];
  float* vs = sm;
  const int t0 = blockIdx.x * XT;
  float x[HPT];
  xhead_x<TV, D, HPT>(V, Delta, vs, t0, T, H_q, H_kv, x);
  const int r = threadIdx.x & 63, hq = threadIdx.x >> 6, t = t0 + r;
  if (t >= T) return;
#pragma unroll
  for (int i = 0; i < HPT; i++) {
    const int h = hq * HPT + i;
    if (h < H_q) z[(size_t)h * T + t] = expf(A[h] * softplus_f(x[i]));
  }
}

// Delta[:, g, :] -> three swizzled bf16 planes [32 heads][D] (hi, mid, lo: truncated 8-bit pieces of the
// fp32 mantissa, hi + mid + lo == the value exactly); heads past H_q are zero rows.  In two halves, so
// that a kernel can have the loads of the next kv-head in flight while it works on the current one:
// request() reads the thread's 8-channel chunks into registers, commit() splits and stores them.
template <int D, int NTHREADS>
struct DeltaChunks {
  static constexpr int CPR = D / 8, N = 32 * CPR / NTHREADS;
  static_assert(N * NTHREADS == 32 * CPR, "chunks must divide evenly over the threads");
  float w[N][8];
  __device__ __forceinline__ void request(const float* __restrict__ Delta, int g, int H_q, int H_kv) {
#pragma unroll
    for (int j = 0; j < N; j++) {
      const int ch = threadIdx.x + j * NTHREADS, h = ch / CPR, c = ch % CPR;
      if (h < H_q) {
        const float* src = Delta + ((size_t)h * H_kv + g) * D + 8 * c;
        const float4 a = *reinterpret_cast<const float4*>(src), b = *reinterpret_cast<const float4*>(src + 4);
        w[j][0] = a.x; w[j][1] = a.y; w[j][2] = a.z; w[j][3] = a.w;
        w[j][4] = b.x; w[j][5] = b.y; w[j][6] = b.z; w[j][7] = b.w;
      } else {
#pragma unroll
        for (int e = 0; e < 8; e++) w[j][e] = 0.f;
      }
    }
  }
  __device__ __forceinline__ void commit(uint16_t* planes) const {
    constexpr int PLANE = 32 * D;
#pragma unroll
    for (int j = 0; j < N; j++) {
      const int ch = threadIdx.x + j * NTHREADS, h = ch / CPR, c = ch % CPR;
      uint32_t pk[3][4];
#pragma unroll
      for (int e = 0; e < 8; e++) {
        float r = w[j][e];
#pragma unroll
        for (int q = 0; q < 3; q++) {
          const uint32_t top = __float_as_uint(r) & 0xffff0000u;  // the leading 8 mantissa bits, truncated
          r -= __uint_as_float(top);                              // exact
          if (e & 1) pk[q][e >> 1] |= top;
          else pk[q][e >> 1] = top >> 16;
        }
      }
      const int off = TileLayout<D>::off(h, c);
#pragma unroll
      for (int q = 0; q < 3; q++)
        *reinterpret_cast<uint4*>(&planes[q * PLANE + off]) = make_uint4(pk[q][0], pk[q][1], pk[q][2], pk[q][3]);
    }
  }
};

// ---- bf16 values: the contraction on the matrix cores.  V is exact in bf16; the fp32 weights are
// split into three bf16 terms by truncation (8 + 8 + 8 mantissa bits: hi + mid + lo == the fp32 value
// exactly), so x = V (hi + mid + lo) is three bf16 MFMA chains with fp32 accumulation and matches the
// fp32 dot product to accumulation rounding.  One wave per 32-token tile, NW tiles per workgroup;
// per kv-head the workgroup splits Delta[:, g, :] once into three swizzled LDS planes,
// each wave reads its V fragments straight from global memory (lane = token, 16 bytes per step).
// Orientation D[head][token] = Delta_g[head][c] V[token][c]: lane (n, hh) ends up with the scores of
// token n for heads 8 (v / 4) + 4 hh + v % 4, so consecutive lanes write consecutive tokens of z.
template <int D, int NW>
__global__ __launch_bounds__(64 * NW) void xhead_scores_mfma_kernel(const uint16_t* __restrict__ V,
                                                                const float* __restrict__ Delta,
                                                                const float* __restrict__ A, float* __restrict__ z,
                                                                int T, int H_q, int H_kv) {
  constexpr int KS = D / 16, PLANE = 32 * D;
  __shared__ __align__(16) uint16_t planes[3 * PLANE];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, n = l & 31, hh = l >> 5;
  const int t = blockIdx.x * (32 * NW) + w * 32 + n;
  const int tl = t < T ? t : T - 1;  // rows past the end re-read the last row; their scores are not written
  FragOffsets<D> fo;
  fo.init(l);
  f32x16 acc[3];
#pragma unroll
  for (int q = 0; q < 3; q++)
#pragma unroll
    for (int v = 0; v < 16; v++) acc[q][v] = 0.f;
  // the loads of kv-head g + 1 (this lane's V fragments, the thread's Delta chunks) are in flight
  // while kv-head g is split into the planes and multiplied
  DeltaChunks<D, 64 * NW> dc;
  bf16x8 vf[KS];
  auto load_v = [&](int g, bf16x8 (&f)[KS]) {
    const uint16_t* vrow = V + ((size_t)tl * H_kv + g) * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) f[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(vrow + 16 * ks));
  };
  // one kv-head: `cd`, `cv` were requested one step earlier; `nd`, `nv` receive the next kv-head's loads
  // (two register sets used alternately, so that nothing is moved and nothing waits for them here; the
  // barriers order LDS traffic only -- a full __syncthreads() would also wait for the loads in flight)
  auto step = [&](int g, DeltaChunks<D, 64 * NW>& cd, bf16x8 (&cv)[KS], DeltaChunks<D, 64 * NW>& nd, bf16x8 (&nv)[KS]) {
    lds_barrier();  // the previous kv-head's readers of the planes are done
    cd.commit(planes);
    const int gn = g + 1 < H_kv ? g + 1 : g;
    nd.request(Delta, gn, H_q, H_kv);
    load_v(gn, nv);
    lds_barrier();
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
#pragma unroll
      for (int q = 0; q < 3; q++) acc[q] = mfma32(fo.row_frag(planes + q * PLANE, 0, ks), cv[ks], acc[q]);
    }
  };
  DeltaChunks<D, 64 * NW> dc2;
  bf16x8 vf2[KS];
  dc.request(Delta, 0, H_q, H_kv);
  load_v(0, vf);
  for (int g = 0; g < H_kv; g += 2) {
    step(g, dc, vf, dc2, vf2);
    if (g + 1 < H_kv) step(g + 1, dc2, vf2, dc, vf);
  }
  if (t >= T) return;
#pragma unroll
  for (int v = 0; v < 16; v++) {
    const int h = 8 * (v / 4) + 4 * hh + (v % 4);
    if (h < H_q) {
      const float x = (acc[2][v] + acc[1][v]) + acc[0][v];
      z[(size_t)h * T + t] = expf(A[h] * softplus_f(x));
    }
  }
}

// Chain rule on the matrix cores (bf16 values).  One wave owns TPW 32-token tiles.
//   phase 1: x as in the forward kernel, but in the orientation D[token][head], so that lane (n, hh)
//     holds, for head n, the tokens 8 (v / 4) + 4 hh + v % 4: dx in that layout is the operand of the
//     dDelta contraction as it stands (hi + lo bf16 terms); a bf16 copy goes to a wave-private
//     [token][head] LDS tile for the dVz contraction; dA is reduced over the lane's tokens.
//   phase 2, per kv-head (planes staged again, workgroups starting at staggered kv-heads): each tile's
//     V rows go to a wave-private swizzled LDS tile; dDelta[head][channel] += dx^T V reads it
//     transposed; dVz[token][channel] = dx Delta_g (hi + mid planes, read transposed) is staged as fp32,
//     32 channels at a time, and leaves as 32-byte row pieces (added to dV in fp32 when accumulating:
//     one rounding).  dDelta accumulates over the wave's tiles, is summed over the four waves through LDS
//     and added to the output once per (workgroup, kv-head).
template <int D, int TPW>
__global__ __launch_bounds__(256) void xhead_bwd_mfma_kernel(const uint16_t* __restrict__ V,
                                                             const float* __restrict__ Delta,
                                                             const float* __restrict__ A, const float* __restrict__ dz,
                                                             float* dDelta, float* dA, uint16_t* dV, int accumulate,
                                                             int T, int H_q, int H_kv) {
  using TL = TileLayout<D>;
  constexpr int KS = D / 16, CB = D / 32, PLANE = 32 * D;
  constexpr int DXS = 40;  // row stride of the [token][head] dx tile (bf16 elements)
  constexpr int SST = 36;  // row stride of the fp32 staging tile [32 tokens][32 channels]
  __shared__ __align__(16) uint16_t planes[3 * PLANE];
  __shared__ __align__(16) uint16_t vtile_all[4][32 * D];
  __shared__ __align__(16) uint16_t dxt_all[4][TPW][32 * DXS];
  __shared__ __align__(16) float stage_all[4][32 * SST];
  __shared__ __align__(16) float red_all[4][CB * 16 * 64];  // per wave: its dDelta[:, g, :] partial sums
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, n = l & 31, hh = l >> 5;
  uint16_t* vt = vtile_all[w];
  float* stg = stage_all[w];
  const int tile0 = (blockIdx.x * 4 + w) * TPW;  // first 32-token tile of this wave
  FragOffsets<D> fo;
  fo.init(l);
  auto wave_fence = [] { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); };  // orders this wave's own LDS traffic
  auto load_v = [&](int tile, int g, bf16x8 (&vf)[KS]) {
    const int t = tile * 32 + n;
    const uint16_t* vrow = V + ((size_t)(t < T ? t : T - 1) * H_kv + g) * D + 8 * hh;  // rows past the end: dx is 0
#pragma unroll
    for (int ks = 0; ks < KS; ks++) vf[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(vrow + 16 * ks));
  };

  // ---- phase 1
  bf16x8 dxh[TPW][2], dxl[TPW][2];
  {
    f32x16 xacc[TPW][3];
#pragma unroll
    for (int i = 0; i < TPW; i++)
#pragma unroll
      for (int q = 0; q < 3; q++)
#pragma unroll
        for (int v = 0; v < 16; v++) xacc[i][q][v] = 0.f;
    // (the loads of kv-head g + 1 are in flight while kv-head g is split and multiplied)
    DeltaChunks<D, 256> dc;
    bf16x8 vf[TPW][KS];
    auto step = [&](int g, DeltaChunks<D, 256>& cd, bf16x8 (&cv)[TPW][KS], DeltaChunks<D, 256>& nd, bf16x8 (&nv)[TPW][KS]) {
      lds_barrier();
      cd.commit(planes);
      const int gn = g + 1 < H_kv ? g + 1 : g;
      nd.request(Delta, gn, H_q, H_kv);
#pragma unroll
      for (int i = 0; i < TPW; i++) load_v(tile0 + i, gn, nv[i]);
      lds_barrier();
#pragma unroll
      for (int ks = 0; ks < KS; ks++)
#pragma unroll
        for (int q = 0; q < 3; q++) {
          const bf16x8 df = fo.row_frag(planes + q * PLANE, 0, ks);
#pragma unroll
          for (int i = 0; i < TPW; i++) xacc[i][q] = mfma32(cv[i][ks], df, xacc[i][q]);
        }
    };
    DeltaChunks<D, 256> dc2;
    bf16x8 vf2[TPW][KS];
    dc.request(Delta, 0, H_q, H_kv);
#pragma unroll
    for (int i = 0; i < TPW; i++) load_v(tile0 + i, 0, vf[i]);
    for (int g = 0; g < H_kv; g += 2) {
      step(g, dc, vf, dc2, vf2);
      if (g + 1 < H_kv) step(g + 1, dc2, vf2, dc, vf);
    }
    const int h = n;
    const float a = h < H_q ? A[h] : 0.f;
    float da = 0.f;
#pragma unroll
    for (int i = 0; i < TPW; i++) {
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const int tok = 8 * (v / 4) + 4 * hh + (v % 4), t = (tile0 + i) * 32 + tok;
        float dx = 0.f;
        if (h < H_q && t < T) {
          const float x = (xacc[i][2][v] + xacc[i][1][v]) + xacc[i][0][v];
          const float sp = softplus_f(x);
          const float zv = expf(a * sp), sig = 1.f / (1.f + expf(-x));
          const float dzz = dz[(size_t)h * T + t] * zv;
          dx = dzz * a * sig;
          da += dzz * sp;
        }
        const __bf16 hi = (__bf16)dx;
        dxh[i][v >> 3][v & 7] = hi;
        dxl[i][v >> 3][v & 7] = (__bf16)(dx - (float)hi);
        dxt_all[w][i][tok * DXS + h] = __builtin_bit_cast(uint16_t, hi);
      }
    }
    da += __shfl_xor(da, 32);
    if (hh == 0 && h < H_q) atomicAdd(dA + h, da);
  }

  // ---- phase 2 (same software pipeline: V rows, the dV rows to add to, and the Delta chunks of the next
  // kv-head are requested before this kv-head's work)
  const int tok2 = l >> 1, half2 = l & 1;  // this lane's row piece of the staged dVz tile
  auto load_old = [&](int tile, int g, uint4 (&old)[CB][2]) {
    const int t = tile * 32 + tok2;
#pragma unroll
    for (int cb = 0; cb < CB; cb++)
#pragma unroll
      for (int q2 = 0; q2 < 2; q2++) {
        old[cb][q2] = make_uint4(0, 0, 0, 0);
        if (accumulate && t < T)
          old[cb][q2] = *reinterpret_cast<const uint4*>(dV + ((size_t)t * H_kv + g) * D + 32 * cb + 16 * half2 + 8 * q2);
      }
  };
  DeltaChunks<D, 256> dc;
  bf16x8 vf[TPW][KS];
  uint4 old[TPW][CB][2];
  {
    const int g0 = blockIdx.x % H_kv;
    dc.request(Delta, g0, H_q, H_kv);
#pragma unroll
    for (int i = 0; i < TPW; i++) {
      load_v(tile0 + i, g0, vf[i]);
      load_old(tile0 + i, g0, old[i]);
    }
  }
  auto step2 = [&](int gi, DeltaChunks<D, 256>& cd, bf16x8 (&cv)[TPW][KS], uint4 (&cold)[TPW][CB][2],
                   DeltaChunks<D, 256>& nd, bf16x8 (&nv)[TPW][KS], uint4 (&nold)[TPW][CB][2]) {
    const int g = (gi + blockIdx.x) % H_kv;
    lds_barrier();
    cd.commit(planes);
    {
      const int gn = gi + 1 < H_kv ? (gi + 1 + blockIdx.x) % H_kv : g;
      nd.request(Delta, gn, H_q, H_kv);
#pragma unroll
      for (int i = 0; i < TPW; i++) {
        load_v(tile0 + i, gn, nv[i]);
        load_old(tile0 + i, gn, nold[i]);
      }
    }
    lds_barrier();
    f32x16 dacc[CB];
#pragma unroll
    for (int cb = 0; cb < CB; cb++)
#pragma unroll
      for (int v = 0; v < 16; v++) dacc[cb][v] = 0.f;
#pragma unroll
    for (int i = 0; i < TPW; i++) {
      const int tbase = (tile0 + i) * 32;
      if (tbase >= T) continue;  // (wave-uniform; no workgroup barrier inside this loop)
      wave_fence();  // the previous tile's transposed reads of vt are done
#pragma unroll
      for (int ks = 0; ks < KS; ks++)
        *reinterpret_cast<uint4*>(&vt[TL::off(n, 2 * ks + hh)]) = __builtin_bit_cast(uint4, cv[i][ks]);
      wave_fence();
      // dDelta[head][channel] += dx^T V: k runs over tokens 16c + 4hh + e % 4 + 8 (e / 4) on both operands
#pragma unroll
      for (int c = 0; c < 2; c++)
#pragma unroll
        for (int cb = 0; cb < CB; cb++) {
          const bf16x8 vtr = fo.tr_frag(vt, 16 * c, cb);
          dacc[cb] = mfma32(dxh[i][c], vtr, dacc[cb]);
          dacc[cb] = mfma32(dxl[i][c], vtr, dacc[cb]);
        }
      // dVz[token][channel] = dx Delta_g: k runs over heads 16c + 4hh + e % 4 + 8 (e / 4)
      f32x16 vacc[CB];
#pragma unroll
      for (int cb = 0; cb < CB; cb++)
#pragma unroll
        for (int v = 0; v < 16; v++) vacc[cb][v] = 0.f;
#pragma unroll
      for (int c = 0; c < 2; c++) {
        const uint16_t* row = dxt_all[w][i] + n * DXS + 16 * c + 4 * hh;
        const s16x4 lo4 = *reinterpret_cast<const s16x4*>(row), hi4 = *reinterpret_cast<const s16x4*>(row + 8);
        const bf16x8 af = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo4, hi4, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
        for (int cb = 0; cb < CB; cb++) {
          vacc[cb] = mfma32(af, fo.tr_frag(planes, 16 * c, cb), vacc[cb]);
          vacc[cb] = mfma32(af, fo.tr_frag(planes + PLANE, 16 * c, cb), vacc[cb]);
        }
      }
      // out through the fp32 staging tile, 32 channels at a time: lane = (token l / 2, half l % 2) writes 16 channels
#pragma unroll
      for (int cb = 0; cb < CB; cb++) {
        wave_fence();  // the previous pass's reads of the staging tile are done
#pragma unroll
        for (int v = 0; v < 16; v++) stg[(8 * (v / 4) + 4 * hh + (v % 4)) * SST + n] = vacc[cb][v];
        wave_fence();
        const int t = tbase + tok2;
        float o[16];
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
          const f32x4 x4 = *reinterpret_cast<const f32x4*>(&stg[tok2 * SST + 16 * half2 + 4 * q4]);
          o[4 * q4] = x4[0]; o[4 * q4 + 1] = x4[1]; o[4 * q4 + 2] = x4[2]; o[4 * q4 + 3] = x4[3];
        }
        if (t < T) {
          uint16_t* dst = dV + ((size_t)t * H_kv + g) * D + 32 * cb + 16 * half2;
#pragma unroll
          for (int q2 = 0; q2 < 2; q2++) {
            const uint32_t u[4] = {cold[i][cb][q2].x, cold[i][cb][q2].y, cold[i][cb][q2].z, cold[i][cb][q2].w};
            bf16x8 ob;  // (the rows to add to were requested as zeros when not accumulating)
#pragma unroll
            for (int e = 0; e < 4; e++) {
              ob[2 * e] = (__bf16)(o[8 * q2 + 2 * e] + __uint_as_float(u[e] << 16));
              ob[2 * e + 1] = (__bf16)(o[8 * q2 + 2 * e + 1] + __uint_as_float(u[e] & 0xffff0000u));
            }
            *reinterpret_cast<uint4*>(dst + 8 * q2) = __builtin_bit_cast(uint4, ob);
          }
        }
      }
    }
    // lane (n, hh) holds dDelta[head 8 (v / 4) + 4 hh + v % 4][g][32 cb + n] of its own tiles.  The four waves'
    // copies are summed through LDS and each wave adds a quarter of the values to the output (the
    // atomics are the scarce resource here: one set per workgroup and kv-head instead of four);
    // consecutive lanes, consecutive channels.
    {
      constexpr int NV = CB * 16, SH = NV / 4;
      float* mine = red_all[w];
#pragma unroll
      for (int cb = 0; cb < CB; cb++)
#pragma unroll
        for (int v = 0; v < 16; v++) mine[(cb * 16 + v) * 64 + l] = dacc[cb][v];
      lds_barrier();
#pragma unroll
      for (int j = 0; j < SH; j++) {
        const int idx = w * SH + j, cb = idx / 16, v = idx % 16;
        const float sum = (red_all[0][idx * 64 + l] + red_all[1][idx * 64 + l]) +
                          (red_all[2][idx * 64 + l] + red_all[3][idx * 64 + l]);
        const int h = 8 * (v / 4) + 4 * hh + (v % 4);
        if (h < H_q) atomicAdd(dDelta + ((size_t)h * H_kv + g) * D + 32 * cb + n, sum);
      }
    }
  };
  DeltaChunks<D, 256> dc2;
  bf16x8 vf2[TPW][KS];
  uint4 old2[TPW][CB][2];
  for (int gi = 0; gi < H_kv; gi += 2) {
    step2(gi, dc, vf, old, dc2, vf2, old2);
    if (gi + 1 < H_kv) step2(gi + 1, dc2, vf2, old2, dc, vf, old);
  }
}

// One workgroup per `tpw` consecutive 64-token tiles.  Phase 1 recomputes x of each tile, turns it
// into dx (kept in LDS for all of the workgroup's tiles) and reduces the dA summands.  Phase 2 walks
// the kv-heads: with Delta_g staged once it revisits the tiles, writes their dVz rows and
// accumulates dDelta[:, g, :] in registers (thread = one channel and HP * D / 256 heads), added to
// the output with one set of fp32 atomics per (workgroup, kv-head).
template <typename TV, int D, int HPT>
__global__ __launch_bounds__(256) void xhead_bwd_kernel(const TV* __restrict__ V, const float* __restrict__ Delta,
                                                        const float* __restrict__ A, const float* __restrict__ dz,
                                                        float* dDelta, float* dA, TV* dV, int accumulate, int T,
                                                        int H_q, int H_kv, int tpw) {
  constexpr int VS = XTile<D>::VS, HP = 4 * HPT, HPC = HP * D / 256;
  constexpr int LPR = D / 8, RPP = 256 / LPR, NP = XT / RPP;
  extern __shared__ float sm[];
  float* vs = sm;
  float* ds = vs + XT * VS;
  float* dxs = ds + HP * D;  // [tpw][64][HP]
  const int tid = threadIdx.x, r = tid & 63, hq = tid >> 6;
  const int tile0 = blockIdx.x * tpw;
  // ---- phase 1
  float da[HPT];
#pragma unroll
  for (int i = 0; i < HPT; i++) da[i] = 0.f;
  for (int tl = 0; tl < tpw; tl++) {
    const int t0 = (tile0 + tl) * XT;
    if (t0 >= T) break;
    float x[HPT];
    xhead_x<TV, D, HPT>(V, Delta, vs, t0, T, H_q, H_kv, x);
    const int t = t0 + r;
#pragma unroll
    for (int i = 0; i < HPT; i++) {
      const int h = hq * HPT + i;
      float dx = 0.f;
      if (h < H_q && t < T) {
        const float a = A[h], sp = softplus_f(x[i]);
        const float zv = expf(a * sp), sig = 1.f / (1.f + expf(-x[i]));
        const float dzz = dz[(size_t)h * T + t] * zv;
        dx = dzz * a * sig;
        da[i] += dzz * sp;
      }
      dxs[(tl * XT + r) * HP + h] = dx;
    }
  }
#pragma unroll
  for (int i = 0; i < HPT; i++) {
    float s = da[i];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
    const int h = hq * HPT + i;
    if (r == 0 && h < H_q) atomicAdd(dA + h, s);
  }
  // ---- phase 2
  const int c = tid % D, hh = tid / D, sub = tid % LPR, rl = tid / LPR;
  for (int gi = 0; gi < H_kv; gi++) {
    // workgroups start at different kv-heads, so that their atomics on dDelta spread over the output
    const int g = (gi + blockIdx.x) % H_kv;
    __syncthreads();  // dxs written; the previous readers of ds are done
    stage_delta<D>(Delta, ds, g, H_q, H_kv, HP);
    float acc[HPC];
#pragma unroll
    for (int j = 0; j < HPC; j++) acc[j] = 0.f;
    for (int tl = 0; tl < tpw; tl++) {
      const int t0 = (tile0 + tl) * XT;
      if (t0 >= T) break;
      __syncthreads();  // the previous readers of vs are done (and ds is complete)
      stage_v_tile<TV, D>(V, vs, t0, g, T, H_kv);
      __syncthreads();
      const float* dxt = dxs + tl * XT * HP;
      // dVz rows: the thread's 8 channels of NP rows
      float dv[NP][8];
#pragma unroll
      for (int p = 0; p < NP; p++)
#pragma unroll
        for (int e = 0; e < 8; e++) dv[p][e] = 0.f;
      for (int h = 0; h < H_q; h++) {
        const float4 w0 = *reinterpret_cast<const float4*>(ds + h * D + 8 * sub);
        const float4 w1 = *reinterpret_cast<const float4*>(ds + h * D + 8 * sub + 4);
#pragma unroll
        for (int p = 0; p < NP; p++) {
          const float dx = dxt[(p * RPP + rl) * HP + h];
          dv[p][0] = fmaf(dx, w0.x, dv[p][0]); dv[p][1] = fmaf(dx, w0.y, dv[p][1]);
          dv[p][2] = fmaf(dx, w0.z, dv[p][2]); dv[p][3] = fmaf(dx, w0.w, dv[p][3]);
          dv[p][4] = fmaf(dx, w1.x, dv[p][4]); dv[p][5] = fmaf(dx, w1.y, dv[p][5]);
          dv[p][6] = fmaf(dx, w1.z, dv[p][6]); dv[p][7] = fmaf(dx, w1.w, dv[p][7]);
        }
      }
#pragma unroll
      for (int p = 0; p < NP; p++) {
        const int t = t0 + p * RPP + rl;
        if (t >= T) continue;
        const size_t roff = ((size_t)t * H_kv + g) * D + 8 * sub;
        if constexpr (sizeof(TV) == 2) {
          if (accumulate) {
            const uint4 raw = *reinterpret_cast<const uint4*>(dV + roff);
            const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int e = 0; e < 4; e++) {
              dv[p][2 * e] += __uint_as_float(u[e] << 16);
              dv[p][2 * e + 1] += __uint_as_float(u[e] & 0xffff0000u);
            }
          }
          bf16x8 o;
#pragma unroll
          for (int e = 0; e < 8; e++) o[e] = (__bf16)dv[p][e];
          *reinterpret_cast<uint4*>(dV + roff) = __builtin_bit_cast(uint4, o);
        } else {
          float4 o0 = make_float4(dv[p][0], dv[p][1], dv[p][2], dv[p][3]);
          float4 o1 = make_float4(dv[p][4], dv[p][5], dv[p][6], dv[p][7]);
          if (accumulate) {
            const float4 p0 = *reinterpret_cast<const float4*>(dV + roff);
            const float4 p1 = *reinterpret_cast<const float4*>(dV + roff + 4);
            o0.x += p0.x; o0.y += p0.y; o0.z += p0.z; o0.w += p0.w;
            o1.x += p1.x; o1.y += p1.y; o1.z += p1.z; o1.w += p1.w;
          }
          *reinterpret_cast<float4*>(dV + roff) = o0;
          *reinterpret_cast<float4*>(dV + roff + 4) = o1;
        }
      }
      // dDelta[hh * HPC + j, g, c] += sum_r dx[r][.] V[r][c]
#pragma unroll 4
      for (int rr = 0; rr < XT; rr++) {
        const float v = vs[rr * VS + c];
        const float* dxr = dxt + rr * HP + hh * HPC;
#pragma unroll
        for (int j = 0; j < HPC; j++) acc[j] = fmaf(dxr[j], v, acc[j]);
      }
    }
#pragma unroll
    for (int j = 0; j < HPC; j++) {
      const int h = hh * HPC + j;
      if (h < H_q) atomicAdd(dDelta + ((size_t)h * H_kv + g) * D + c, acc[j]);
    }
  }
}

__global__ void xhead_zero_kernel(float* a, size_t na, float* b, size_t nb) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < na) a[i] = 0.f;
  if (i < nb) b[i] = 0.f;
}

static int pick_hpt(int H_q) {
  const int need = (H_q + 3) / 4;
  for (int hpt = 2; hpt <= 8; hpt *= 2)
    if (hpt >= need) return hpt;
  return 0;  // more than 32 heads
}

template <typename TV, int D>
static int scores_dispatch(int hpt, dim3 grid, size_t sh, hipStream_t st, const void* V, const float* Delta, const float* A,
                           float* z, const dma_shape& s) {
  switch (hpt) {
    case 2: xhead_scores_kernel<TV, D, 2><<<grid, 256, sh, st>>>((const TV*)V, Delta, A, z, s.T, s.H_q, s.H_kv); break;
    case 4: xhead_scores_kernel<TV, D, 4><<<grid, 256, sh, st>>>((const TV*)V, Delta, A, z, s.T, s.H_q, s.H_kv); break;
    default: xhead_scores_kernel<TV, D, 8><<<grid, 256, sh, st>>>((const TV*)V, Delta, A, z, s.T, s.H_q, s.H_kv); break;
  }
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

int launch_xhead_scores(const dma_shape& s, const void* V, const float* Delta, const float* A, float* z, hipStream_t st) {
  const int hpt = pick_hpt(s.H_q);
  if (!hpt) return DMA_EUNSUPPORTED;
  if (s.dtype == DMA_BF16) {
    constexpr int NW = 4;  // waves (32-token tiles) per workgroup
    const dim3 grid((s.T + 32 * NW - 1) / (32 * NW));
    if (s.d == 128) xhead_scores_mfma_kernel<128, NW><<<grid, 64 * NW, 0, st>>>((const uint16_t*)V, Delta, A, z, s.T, s.H_q, s.H_kv);
    else xhead_scores_mfma_kernel<64, NW><<<grid, 64 * NW, 0, st>>>((const uint16_t*)V, Delta, A, z, s.T, s.H_q, s.H_kv);
    return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
  }
  const dim3 grid((s.T + XT - 1) / XT);
  const size_t sh = (size_t)XT * (s.d + 4) * sizeof(float);
  return s.d == 128 ? scores_dispatch<float, 128>(hpt, grid, sh, st, V, Delta, A, z, s)
                    : scores_dispatch<float, 64>(hpt, grid, sh, st, V, Delta, A, z, s);
}

template <typename TV, int D>
static int bwd_dispatch(int hpt, dim3 grid, size_t sh, hipStream_t st, const void* V, const float* Delta, const float* A,
                        const float* dz, float* dDelta, float* dA, void* dV, int accumulate, const dma_shape& s, int tpw) {
  switch (hpt) {
    case 2: xhead_bwd_kernel<TV, D, 2><<<grid, 256, sh, st>>>((const TV*)V, Delta, A, dz, dDelta, dA, (TV*)dV, accumulate, s.T, s.H_q, s.H_kv, tpw); break;
    case 4: xhead_bwd_kernel<TV, D, 4><<<grid, 256, sh, st>>>((const TV*)V, Delta, A, dz, dDelta, dA, (TV*)dV, accumulate, s.T, s.H_q, s.H_kv, tpw); break;
    default: xhead_bwd_kernel<TV, D, 8><<<grid, 256, sh, st>>>((const TV*)V, Delta, A, dz, dDelta, dA, (TV*)dV, accumulate, s.T, s.H_q, s.H_kv, tpw); break;
  }
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

int launch_xhead_bwd(const dma_shape& s, const void* V, const float* Delta, const float* A, const float* dz,
                     float* dDelta, float* dA, void* dV, int accumulate, hipStream_t st) {
  const int hpt = pick_hpt(s.H_q);
  if (!hpt) return DMA_EUNSUPPORTED;
  const size_t nd = (size_t)s.H_q * s.H_kv * s.d;
  xhead_zero_kernel<<<(unsigned)((nd + 255) / 256), 256, 0, st>>>(dDelta, nd, dA, (size_t)s.H_q);
  if (s.dtype == DMA_BF16) {
    constexpr int TPW = 1;  // 32-token tiles per wave (two halve the atomics but measured slower)
    const int nwaves = ((s.T + 31) / 32 + TPW - 1) / TPW;
    const dim3 grid((nwaves + 3) / 4);
    if (s.d == 128)
      xhead_bwd_mfma_kernel<128, TPW><<<grid, 256, 0, st>>>((const uint16_t*)V, Delta, A, dz, dDelta, dA, (uint16_t*)dV, accumulate, s.T, s.H_q, s.H_kv);
    else
      xhead_bwd_mfma_kernel<64, TPW><<<grid, 256, 0, st>>>((const uint16_t*)V, Delta, A, dz, dDelta, dA, (uint16_t*)dV, accumulate, s.T, s.H_q, s.H_kv);
    return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
  }
  const int ntiles = (s.T + XT - 1) / XT;
  // tiles per workgroup: about two workgroups per CU (fewer contended atomics on dDelta), within 64 KB of LDS
  const size_t fixed = ((size_t)XT * (s.d + 4) + (size_t)4 * hpt * s.d) * sizeof(float);
  const size_t per_tile = (size_t)XT * 4 * hpt * sizeof(float);
  int tpw = (ntiles + 511) / 512;
  const int tpw_max = (int)((64 * 1024 - fixed) / per_tile);
  if (tpw > tpw_max) tpw = tpw_max;
  if (tpw < 1) tpw = 1;
  const dim3 grid((ntiles + tpw - 1) / tpw);
  const size_t sh = fixed + per_tile * tpw;
  return s.d == 128 ? bwd_dispatch<float, 128>(hpt, grid, sh, st, V, Delta, A, dz, dDelta, dA, dV, accumulate, s, tpw)
                    : bwd_dispatch<float, 64>(hpt, grid, sh, st, V, Delta, A, dz, dDelta, dA, dV, accumulate, s, tpw);
}

}  // namespace dma
