// fp32 debug path of the attention forward / backward (Eq. 5-10): plain FMA arithmetic, one wave
// per query row or per key, no tiling.  It exists to check the mask plumbing and the gradient
// formulas at fp32 accuracy on small inputs; it is not a performance path.
#include "common.h"

namespace dma {

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
  return x;
}
__device__ __forceinline__ double wave_sum(double x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off));
  return x;
}

// One wave per (query row t, head h).  MODE 0: forward (O, LSE).  MODE 1: backward row pass
// (D_t = dO_t . O_t, dQ_t), with P recomputed from LSE.
template <int D, int MODE>
__global__ __launch_bounds__(64) void row_f32_kernel(const float* __restrict__ Q, const float* __restrict__ K,
                                                     const float* __restrict__ V, const float* __restrict__ zq,
                                                     const int32_t* __restrict__ expiry, const int32_t* __restrict__ cu,
                                                     int n_docs, int causal, int T, int H_q, int H_kv, const float* __restrict__ plan_scale,
                                                     float* __restrict__ O, float* __restrict__ LSE,
                                                     const float* __restrict__ dO, double* __restrict__ Dout,
                                                     float* __restrict__ dQ) {
  const int t = blockIdx.x, h = blockIdx.y, l = threadIdx.x;
  const float scale = *plan_scale;  // the plan's: the one zq was divided by
  const int g = h / (H_q / H_kv);
  const int doc = find_doc(cu, n_docs, t);
  const int a = cu[doc];
  // candidates: keys a .. jl; key j is kept by this row if its expiry lies beyond `thr`.  Causal:
  // jl = t and thr = t; otherwise every row of the document keeps the same keys (expiry > own index).
  const int jl = causal ? t : cu[doc + 1] - 1;
  __shared__ float qs[D], dos[D];
  const float* qrow = Q + ((size_t)t * H_q + h) * D;
  for (int c = l; c < D; c += 64) qs[c] = qrow[c];
  // D_i and dP_ij are both of size |dO| |v| while their difference can vanish (one kept key: exactly):
  // both are formed in fp64 so that the difference keeps fp32 accuracy
  double Dt = 0.0;
  float lse = 0.f;
  if (MODE == 1) {
    const float* dorow = dO + ((size_t)t * H_q + h) * D;
    const float* orow = O + ((size_t)t * H_q + h) * D;
    double part = 0.0;
    for (int c = l; c < D; c += 64) {
      dos[c] = dorow[c];
      part += (double)dorow[c] * (double)orow[c];
    }
    Dt = wave_sum(part);
    lse = LSE[(size_t)h * T + t];
    if (l == 0) Dout[(size_t)h * T + t] = Dt;
  }
  __syncthreads();
  float m = -INFINITY;
  if (MODE == 0) {
    for (int j0 = a; j0 <= jl; j0 += 64) {
      const int j = j0 + l;
      if (j <= jl && expiry[(size_t)h * T + j] > (causal ? t : j)) {
        const float* kr = K + ((size_t)j * H_kv + g) * D;
        float s = 0.f;
        for (int c = 0; c < D; c++) s = fmaf(qs[c], kr[c], s);
        m = fmaxf(m, (s + zq[(size_t)h * T + j]) * scale);
      }
    }
    m = wave_max(m);
  }
  float acc[D];
#pragma unroll
  for (int c = 0; c < D; c++) acc[c] = 0.f;
  float lsum = 0.f;
  for (int j0 = a; j0 <= jl; j0 += 64) {
    const int j = j0 + l;
    if (j <= jl && expiry[(size_t)h * T + j] > (causal ? t : j)) {
      const float* kr = K + ((size_t)j * H_kv + g) * D;
      const float* vr = V + ((size_t)j * H_kv + g) * D;
      float s = 0.f;
      for (int c = 0; c < D; c++) s = fmaf(qs[c], kr[c], s);
      s = (s + zq[(size_t)h * T + j]) * scale;  // zq = (z + bias) / scale, as the plan holds it
      if (MODE == 0) {
        const float pr = expf(s - m);
        lsum += pr;
#pragma unroll
        for (int c = 0; c < D; c++) acc[c] = fmaf(pr, vr[c], acc[c]);
      } else {
        const float pr = expf(s - lse);
        double dp = 0.0;
        for (int c = 0; c < D; c++) dp += (double)dos[c] * (double)vr[c];
        const float ds = pr * (float)(dp - Dt);
#pragma unroll
        for (int c = 0; c < D; c++) acc[c] = fmaf(ds, kr[c], acc[c]);
      }
    }
  }
  if (MODE == 0) {
    lsum = wave_sum(lsum);
    if (l == 0) LSE[(size_t)h * T + t] = m + logf(lsum);
  }
  const float mul = (MODE == 0) ? 1.f / lsum : scale;
  float* outrow = (MODE == 0 ? O : dQ) + ((size_t)t * H_q + h) * D;
#pragma unroll
  for (int c = 0; c < D; c++) {
    const float tot = wave_sum(acc[c]);
    if (l == (c & 63)) outrow[c] = tot * mul;
  }
}

// One wave per (key t, kv-head g): dK_t, dV_t summed over the q-heads of the group, dz per q-head.
// Lane l owns channels l, l + 64, ...; rows are walked in order, so the result is deterministic.
template <int D>
__global__ __launch_bounds__(64) void key_f32_kernel(const float* __restrict__ Q, const float* __restrict__ K,
                                                     const float* __restrict__ V, const float* __restrict__ zq,
                                                     const int32_t* __restrict__ expiry, const int32_t* __restrict__ cu,
                                                     int n_docs, int causal, int T, int H_q, int H_kv,
                                                     const float* __restrict__ plan_scale, const float* __restrict__ LSE,
                                                     const float* __restrict__ dO, const double* __restrict__ Dws,
                                                     float* __restrict__ dK, float* __restrict__ dV,
                                                     float* __restrict__ dz) {
  constexpr int CPL = D / 64;
  const int t = blockIdx.x, g = blockIdx.y, l = threadIdx.x;
  const float scale = *plan_scale;
  const int G = H_q / H_kv;
  float kc[CPL], vc[CPL];
  double dk[CPL], dv[CPL];  // sums over up to n rows: accumulated in fp64 so that their rounding stays below 1e-5
#pragma unroll
  for (int u = 0; u < CPL; u++) {
    kc[u] = K[((size_t)t * H_kv + g) * D + l + 64 * u];
    vc[u] = V[((size_t)t * H_kv + g) * D + l + 64 * u];
    dk[u] = 0.0;
    dv[u] = 0.0;
  }
  for (int hh = 0; hh < G; hh++) {
    const int h = g * G + hh;
    const int e = expiry[(size_t)h * T + t];
    const float zt = zq[(size_t)h * T + t];
    double dzacc = 0.0;
    int i0 = t, i1 = e;  // rows that keep this key: causal t .. e - 1; otherwise the whole document or none
    if (!causal) {
      const int doc = find_doc(cu, n_docs, t);
      i0 = e > t ? cu[doc] : t;
      i1 = e > t ? cu[doc + 1] : t;
    }
    for (int i = i0; i < i1; i++) {
      const float* qr = Q + ((size_t)i * H_q + h) * D;
      const float* dor = dO + ((size_t)i * H_q + h) * D;
      float qv[CPL], dov[CPL], s = 0.f;
      double dp = 0.0;
#pragma unroll
      for (int u = 0; u < CPL; u++) {
        qv[u] = qr[l + 64 * u];
        dov[u] = dor[l + 64 * u];
        s = fmaf(qv[u], kc[u], s);
        dp += (double)dov[u] * (double)vc[u];
      }
      s = wave_sum(s);
      dp = wave_sum(dp);
      const float pr = expf((s + zt) * scale - LSE[(size_t)h * T + i]);
      const float ds = pr * (float)(dp - Dws[(size_t)h * T + i]);
      dzacc += ds;
#pragma unroll
      for (int u = 0; u < CPL; u++) {
        dk[u] += (double)ds * (double)qv[u];
        dv[u] += (double)pr * (double)dov[u];
      }
    }
    if (l == 0) dz[(size_t)h * T + t] = (float)dzacc;
  }
#pragma unroll
  for (int u = 0; u < CPL; u++) {
    dK[((size_t)t * H_kv + g) * D + l + 64 * u] = (float)(dk[u] * (double)scale);
    dV[((size_t)t * H_kv + g) * D + l + 64 * u] = (float)dv[u];
  }
}

int launch_fwd_f32(const Ptrs& p, const float* Q, const float* K, const float* V, const float* z,
                   const int32_t* expiry, const int32_t* cu, float* O, float* LSE, hipStream_t st) {
  const dma_shape& s = p.s;
  (void)z;
  const float* zq = (const float*)(p.plan + p.pl.off_zq);  // the bias as the plan holds it: (z [+ caller bias]) / scale
  const float* sc = (const float*)(p.plan + p.pl.off_consts + PLAN_SCALE_OFF);  // the scale zq was written with
  dim3 grid(s.T, s.H_q);
#define DMA_ROW0(DD) \
  row_f32_kernel<DD, 0><<<grid, 64, 0, st>>>(Q, K, V, zq, expiry, cu, s.n_docs, s.causal, s.T, s.H_q, s.H_kv, sc, O, LSE, \
                                             nullptr, nullptr, nullptr)
  if (s.d == 256) DMA_ROW0(256);
  else if (s.d == 128) DMA_ROW0(128);
  else DMA_ROW0(64);
#undef DMA_ROW0
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

int launch_bwd_f32(const Ptrs& p, const float* Q, const float* K, const float* V, const float* O, const float* dO,
                   const float* LSE, const float* z, const int32_t* expiry, const int32_t* cu, float* dQ, float* dK,
                   float* dV, float* dz, char* ws, hipStream_t st) {
  const dma_shape& s = p.s;
  (void)z;
  const float* zq = (const float*)(p.plan + p.pl.off_zq);
  const float* sc = (const float*)(p.plan + p.pl.off_consts + PLAN_SCALE_OFF);
  double* Dws = (double*)ws;
  dim3 grid(s.T, s.H_q), gridk(s.T, s.H_kv);
#define DMA_BWD32(DD)                                                                                                    \
  do {                                                                                                                   \
    row_f32_kernel<DD, 1><<<grid, 64, 0, st>>>(Q, K, V, zq, expiry, cu, s.n_docs, s.causal, s.T, s.H_q, s.H_kv, sc,        \
                                               const_cast<float*>(O), const_cast<float*>(LSE), dO, Dws, dQ);             \
    key_f32_kernel<DD><<<gridk, 64, 0, st>>>(Q, K, V, zq, expiry, cu, s.n_docs, s.causal, s.T, s.H_q, s.H_kv, sc, LSE, dO, \
                                             Dws, dK, dV, dz);                                                           \
  } while (0)
  if (s.d == 256) DMA_BWD32(256);
  else if (s.d == 128) DMA_BWD32(128);
  else DMA_BWD32(64);
#undef DMA_BWD32
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

}  // namespace dma
