// Content scores with the paper's full sampling tensor (Eq. 3, Delta in R^{n_h x d_h x n_h}; Listing 1
// flattens the values of all heads of a token before the projection), and their chain rule:
//   x[h, j] = sum_{g, c} v_{g, j, c} Delta[h, g, c],   z = exp(A_h softplus(x)),
//   dx = dz z A_h sigmoid(x),  dA_h = sum_j dz z softplus(x),
//   dDelta[h, g, c] = sum_j dx[h, j] v_{g, j, c},   dVz[j, g, c] = sum_h dx[h, j] Delta[h, g, c].
// Delta is [H_q, H_kv * d] row-major (the weight of a linear layer from the flattened values to the
// heads).  A [T x H_kv d] x [H_kv d x H_q] contraction with H_q <= 32 output columns and fp32
// weights: one pass over V, computed with fp32 vector FMAs from LDS tiles.
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
  const dim3 grid((s.T + XT - 1) / XT);
  const size_t sh = (size_t)XT * (s.d + 4) * sizeof(float);
  if (s.dtype == DMA_BF16)
    return s.d == 128 ? scores_dispatch<uint16_t, 128>(hpt, grid, sh, st, V, Delta, A, z, s)
                      : scores_dispatch<uint16_t, 64>(hpt, grid, sh, st, V, Delta, A, z, s);
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
  if (s.dtype == DMA_BF16)
    return s.d == 128 ? bwd_dispatch<uint16_t, 128>(hpt, grid, sh, st, V, Delta, A, dz, dDelta, dA, dV, accumulate, s, tpw)
                      : bwd_dispatch<uint16_t, 64>(hpt, grid, sh, st, V, Delta, A, dz, dDelta, dA, dV, accumulate, s, tpw);
  return s.d == 128 ? bwd_dispatch<float, 128>(hpt, grid, sh, st, V, Delta, A, dz, dDelta, dA, dV, accumulate, s, tpw)
                    : bwd_dispatch<float, 64>(hpt, grid, sh, st, V, Delta, A, dz, dDelta, dA, dV, accumulate, s, tpw);
}

}  // namespace dma
