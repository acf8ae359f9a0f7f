// Gradient of the content scores (chain rule of Eq. 3; Section 6: the bias is the differentiable
// path into the score parameters).  Given dz [H_q, T] from the attention backward:
//   x = w_h . v_{g(h), j},  z = exp(A_h softplus(x)),
//   dx = dz z A_h sigmoid(x),  dA_h = sum_j dz z softplus(x),  dW_h = sum_j dx v_{g(h), j},
//   dVz_{j, g} = sum_{h in g} dx_{h, j} w_h.
// HBM-bound: one pass over V (read) and dV (write, plus a read when accumulating), dz read once.
#include "common.h"

namespace dma {

// One workgroup per (TT-token tile, kv-head); TT = 64, or 32 at 256 channels (the V tile is kept in LDS).  (1) every row is held by D / 8 lanes, which reduce
// x = w_h . v for each q-head of the group; (2) one thread per (q-head, row) turns x into dx and
// the dA summand (the transcendental work, 64 different pairs per wave instruction); (3) the row's
// lanes add dx w_h into their 8 channels of the dV row; (4) dW and dA partial sums of the tile
// (from dx and the V tile kept in LDS) are added to the outputs with fp32 atomics (G * D + G per
// workgroup).
template <typename TV, int D, int TT>
__global__ __launch_bounds__(256) void mask_bwd_kernel(const TV* __restrict__ V, const float* __restrict__ W,
                                                       const float* __restrict__ A, const float* __restrict__ dz,
                                                       float* dW, float* dA, TV* dV, int accumulate, int T,
                                                       int H_q, int H_kv, int tiles_per_wg) {
  extern __shared__ float sm[];  // [TT][D] V tile, [G][D] w, [G][D] dW partial, [G][TT] x then dx, [G][TT] dA summands, [G] dA partial
  constexpr int LPR = D / 8, RPP = 256 / LPR, NP = TT / RPP;
  const int g = blockIdx.y, G = H_q / H_kv;
  float* vs = sm;
  float* ws = vs + TT * D;
  float* dws = ws + G * D;
  float* dxs = dws + G * D;
  float* das = dxs + G * TT;
  float* dap = das + G * TT;
  const int tid = threadIdx.x, sub = tid % LPR, rl = tid / LPR;
  for (int i = tid; i < G * D; i += 256) {
    ws[i] = W[(size_t)g * G * D + i];
    dws[i] = 0.f;
  }
  for (int i = tid; i < G; i += 256) dap[i] = 0.f;
  // a workgroup walks tiles_per_wg consecutive TT-token tiles, so that the contended atomics on dW / dA
  // are issued once per workgroup instead of once per tile
  for (int tile = 0; tile < tiles_per_wg; tile++) {
  const int t0 = (blockIdx.x * tiles_per_wg + tile) * TT;
  if (t0 >= T) break;
  __syncthreads();  // the previous tile's readers of vs / dxs / das are done
  float v[NP][8];
#pragma unroll
  for (int pass = 0; pass < NP; pass++) {
    const int r = pass * RPP + rl, t = t0 + r;
#pragma unroll
    for (int e = 0; e < 8; e++) v[pass][e] = 0.f;
    if (t < T) {
      const size_t roff = ((size_t)t * H_kv + g) * D + 8 * sub;
      if constexpr (sizeof(TV) == 2) {
        const uint4 raw = *reinterpret_cast<const uint4*>(V + roff);
        const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int e = 0; e < 4; e++) {
          v[pass][2 * e] = __uint_as_float(u[e] << 16);
          v[pass][2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
        }
      } else {
        const float4 x0 = *reinterpret_cast<const float4*>(V + roff);
        const float4 x1 = *reinterpret_cast<const float4*>(V + roff + 4);
        v[pass][0] = x0.x; v[pass][1] = x0.y; v[pass][2] = x0.z; v[pass][3] = x0.w;
        v[pass][4] = x1.x; v[pass][5] = x1.y; v[pass][6] = x1.z; v[pass][7] = x1.w;
      }
    }
#pragma unroll
    for (int e = 0; e < 8; e++) vs[r * D + 8 * sub + e] = v[pass][e];
  }
  __syncthreads();
  // (1) x[hh][r]
#pragma unroll
  for (int pass = 0; pass < NP; pass++) {
    const int r = pass * RPP + rl;
    for (int hh = 0; hh < G; hh++) {
      const float* w = ws + hh * D + 8 * sub;
      float x = 0.f;
#pragma unroll
      for (int e = 0; e < 8; e++) x = fmaf(v[pass][e], w[e], x);
#pragma unroll
      for (int off = LPR / 2; off > 0; off >>= 1) x += __shfl_xor(x, off);
      if (sub == 0) dxs[hh * TT + r] = x;
    }
  }
  __syncthreads();
  // (2) dx and the dA summand, one (q-head, row) pair per thread
  for (int idx = tid; idx < G * TT; idx += 256) {
    const int hh = idx / TT, r = idx % TT, t = t0 + r, h = g * G + hh;
    float dx = 0.f, da = 0.f;
    if (t < T) {
      const float x = dxs[idx], a = A[h];
      const float sp = fmaxf(x, 0.f) + log1pf(expf(-fabsf(x)));
      const float zv = expf(a * sp);
      const float sig = 1.f / (1.f + expf(-x));
      const float dzz = dz[(size_t)h * T + t] * zv;
      dx = dzz * a * sig;
      da = dzz * sp;
    }
    dxs[idx] = dx;
    das[idx] = da;
  }
  __syncthreads();
  // (3) dVz rows
#pragma unroll
  for (int pass = 0; pass < NP; pass++) {
    const int r = pass * RPP + rl, t = t0 + r;
    if (t >= T) continue;  // (no barrier inside this loop)
    float dv[8];
#pragma unroll
    for (int e = 0; e < 8; e++) dv[e] = 0.f;
    for (int hh = 0; hh < G; hh++) {
      const float dx = dxs[hh * TT + r];
      const float* w = ws + hh * D + 8 * sub;
#pragma unroll
      for (int e = 0; e < 8; e++) dv[e] = fmaf(dx, w[e], dv[e]);
    }
    const size_t roff = ((size_t)t * H_kv + g) * D + 8 * sub;
    if constexpr (sizeof(TV) == 2) {
      if (accumulate) {
        const uint4 raw = *reinterpret_cast<const uint4*>(dV + roff);
        const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int e = 0; e < 4; e++) {
          dv[2 * e] += __uint_as_float(u[e] << 16);
          dv[2 * e + 1] += __uint_as_float(u[e] & 0xffff0000u);
        }
      }
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; e++) o[e] = (__bf16)dv[e];
      *reinterpret_cast<uint4*>(dV + roff) = __builtin_bit_cast(uint4, o);
    } else {
      float4 o0 = make_float4(dv[0], dv[1], dv[2], dv[3]), o1 = make_float4(dv[4], dv[5], dv[6], dv[7]);
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
  // (4) dW[h, c] += sum_r dx[h, r] V[r, c]: thread per (hh, c); dA[h] += sum_r dz z softplus(x)
  for (int idx = tid; idx < G * D; idx += 256) {
    const int hh = idx / D, c = idx % D;
    float s = 0.f;
#pragma unroll 8
    for (int r = 0; r < TT; r++) s = fmaf(dxs[hh * TT + r], vs[r * D + c], s);
    dws[idx] += s;  // (the same thread owns idx for every tile)
  }
  for (int hh = tid; hh < G; hh += 256) {
    float s = 0.f;
    for (int r = 0; r < TT; r++) s += das[hh * TT + r];
    dap[hh] += s;
  }
  }  // tiles
  for (int idx = tid; idx < G * D; idx += 256) atomicAdd(dW + (size_t)g * G * D + idx, dws[idx]);
  for (int hh = tid; hh < G; hh += 256) atomicAdd(dA + g * G + hh, dap[hh]);
}

__global__ void fill_zero_kernel(float* a, size_t na, float* b, size_t nb) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < na) a[i] = 0.f;
  if (i < nb) b[i] = 0.f;
}

// dynamic LDS of one workgroup; beyond 64 KiB (very many q-heads per kv-head) the shape is refused
size_t mask_bwd_lds_bytes(const dma_shape& s) {
  const size_t G = (size_t)(s.H_q / s.H_kv), TT = s.d == 256 ? 32 : 64;
  return (TT * s.d + 2 * G * s.d + 2 * G * TT + G) * sizeof(float);
}

int launch_mask_bwd(const dma_shape& s, const void* V, const float* W, const float* A, const float* dz,
                    float* dW, float* dA, void* dV, int accumulate, hipStream_t st) {
  if (mask_bwd_lds_bytes(s) > 64 * 1024) return DMA_EUNSUPPORTED;  // (before the first launch)
  const size_t nw = (size_t)s.H_q * s.d;
  fill_zero_kernel<<<(unsigned)((nw + 255) / 256), 256, 0, st>>>(dW, nw, dA, (size_t)s.H_q);
  const int TT = s.d == 256 ? 32 : 64;  // tokens per tile
  const int ntiles = (s.T + TT - 1) / TT;
  // enough workgroups to fill the chip (about four per CU), as few contended atomics as possible
  int tpw = (int)(((long)ntiles * s.H_kv + 1023) / 1024);
  if (tpw < 1) tpw = 1;
  const dim3 grid((ntiles + tpw - 1) / tpw, s.H_kv);
  const size_t sh = mask_bwd_lds_bytes(s);
#define DMA_MB(TV, DD, TTT) \
  mask_bwd_kernel<TV, DD, TTT><<<grid, 256, sh, st>>>((const TV*)V, W, A, dz, dW, dA, (TV*)dV, accumulate, s.T, s.H_q, s.H_kv, tpw)
  if (s.dtype == DMA_BF16) {
    if (s.d == 256) DMA_MB(uint16_t, 256, 32);
    else if (s.d == 128) DMA_MB(uint16_t, 128, 64);
    else DMA_MB(uint16_t, 64, 64);
  } else {
    if (s.d == 256) DMA_MB(float, 256, 32);
    else if (s.d == 128) DMA_MB(float, 128, 64);
    else DMA_MB(float, 64, 64);
  }
#undef DMA_MB
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

}  // namespace dma
