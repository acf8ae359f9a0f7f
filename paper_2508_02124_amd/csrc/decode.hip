// Decode: one new query row per sequence against its whole KV cache (the case with the paper's
// largest speed-ups, Section 5 "Kernel performance").  The row is the last row of its document, so
// its candidates are all n keys of the document; it keeps the min(k, n) best by (z descending,
// index ascending) (Eq. 4), and attends to them with the bias z (Eq. 5-6).  HBM-bound: z is read a
// few times for the selection, then min(k, n) rows of K and V are gathered.
#include "common.h"

namespace dma {

__device__ __forceinline__ uint32_t desc_key_u32(float z) {
  // ascending unsigned order == descending float order (-0 and +0 compare equal)
  z = z + 0.0f;
  uint32_t u = __float_as_uint(z);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ~u;
}

// Selection: one workgroup (16 waves) per (sequence, q-head).
//  (1) radix select, most significant byte first: the key value `thr` of the kk-th best score and
//      how many keys equal to it are still needed (`need_eq`, the ones with the lowest indices);
//  (2) ordered compaction of the kept indices into `kept` (ascending).
__global__ __launch_bounds__(1024) void decode_select_kernel(const float* __restrict__ z, const int32_t* __restrict__ cu,
                                                             int32_t* kept, int T, int H_q, int k) {
  const int b = blockIdx.x, h = blockIdx.y;
  const int a = cu[b], n = cu[b + 1] - a;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
  const int kcap = k < T ? k : T;
  int32_t* list = kept + ((size_t)b * H_q + h) * kcap;
  if (n <= 0) return;
  const int kk = k < n ? k : n;
  const float* zh = z + (size_t)h * T + a;
  // every digit has 32 sub-counters (one per lane pair), so that the lanes of a wave that hit the
  // same digit (scores share their leading bits) do not serialise on one LDS address
  __shared__ uint32_t hist[256 * 32];
  __shared__ uint32_t sel[2];     // selected digit, remaining count
  __shared__ uint32_t wcnt[2][16];
  uint32_t prefix = 0, remaining = (uint32_t)kk;
  if (kk < n) {
    for (int pass = 3; pass >= 0; pass--) {
      for (int i = tid; i < 256 * 32; i += 1024) hist[i] = 0;
      __syncthreads();
      const int sh = 8 * pass;
      for (int j0 = tid; j0 < n; j0 += 8 * 1024) {  // eight loads in flight per lane
        float zv[8];
#pragma unroll
        for (int u = 0; u < 8; u++) zv[u] = j0 + u * 1024 < n ? zh[j0 + u * 1024] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; u++) {
          const uint32_t key = desc_key_u32(zv[u]);
          if (j0 + u * 1024 < n && (pass == 3 || (key >> (sh + 8)) == prefix)) atomicAdd(&hist[((key >> sh) & 255u) * 32 + (l & 31)], 1u);
        }
      }
      __syncthreads();
      if (w == 0) {  // the digit at which the running count reaches `remaining`
        uint32_t c4[4], s = 0;
#pragma unroll
        for (int i = 0; i < 4; i++) {
          c4[i] = 0;
          for (int sc = 0; sc < 32; sc++) c4[i] += hist[(4 * l + i) * 32 + ((sc + l) & 31)];
          s += c4[i];
        }
        uint32_t inc = s;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const uint32_t t = __shfl_up(inc, off);
          if (l >= off) inc += t;
        }
        uint32_t run = inc - s;  // keys with a smaller digit than 4l
#pragma unroll
        for (int i = 0; i < 4; i++) {
          if (run < remaining && remaining <= run + c4[i]) {
            sel[0] = 4 * l + i;
            sel[1] = remaining - run;
          }
          run += c4[i];
        }
      }
      __syncthreads();
      prefix = (prefix << 8) | sel[0];
      remaining = sel[1];
      __syncthreads();
    }
  }
  const uint32_t thr = prefix, need_eq = remaining;
  // (2) ordered compaction: keys better than thr, and the first need_eq keys equal to thr
  if (kk == n) {
    for (int j = tid; j < n; j += 1024) list[j] = a + j;
  } else {
    // every wave owns a contiguous range of keys: count, prefix over the waves, then write in order
    const unsigned long long lt = (1ull << l) - 1ull;
    const int seg = ((n + 15) / 16 + 63) / 64 * 64;
    const int j_begin = w * seg, j_end = min(n, j_begin + seg);
    uint32_t cb = 0, ce = 0;
    for (int j0 = j_begin; j0 < j_end; j0 += 8 * 64) {
      float zv[8];
#pragma unroll
      for (int u = 0; u < 8; u++) zv[u] = j0 + u * 64 + l < j_end ? zh[j0 + u * 64 + l] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const bool in = j0 + u * 64 + l < j_end;
        const uint32_t key = desc_key_u32(zv[u]);
        cb += (uint32_t)__popcll(__ballot(in && key < thr));
        ce += (uint32_t)__popcll(__ballot(in && key == thr));
      }
    }
    if (l == 0) {
      wcnt[0][w] = cb;
      wcnt[1][w] = ce;
    }
    __syncthreads();
    uint32_t rb = 0, re = 0;  // better / equal keys before this wave's range, then before the chunk
    for (int i = 0; i < w; i++) {
      rb += wcnt[0][i];
      re += wcnt[1][i];
    }
    for (int j0 = j_begin; j0 < j_end; j0 += 8 * 64) {
      float zv[8];
#pragma unroll
      for (int u = 0; u < 8; u++) zv[u] = j0 + u * 64 + l < j_end ? zh[j0 + u * 64 + l] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; u++) {
        const int j = j0 + u * 64 + l;
        const uint32_t key = desc_key_u32(zv[u]);
        const bool better = j < j_end && key < thr, equal = j < j_end && key == thr;
        const unsigned long long bm = __ballot(better), em = __ballot(equal);
        const uint32_t eq_before = re + (uint32_t)__popcll(em & lt);  // equal keys with a lower index
        const uint32_t pos = rb + (uint32_t)__popcll(bm & lt) + min(eq_before, need_eq);
        if (better || (equal && eq_before < need_eq)) list[pos] = a + j;
        rb += (uint32_t)__popcll(bm);
        re += (uint32_t)__popcll(em);
      }
    }
  }
}

// Keys per workgroup of the attention pass.
constexpr int DEC_CHUNK = 256;

// (3) single-row attention over one chunk of DEC_CHUNK kept keys: a key row is held by D / 8
// lanes; every lane group keeps its own running (m, l, o) over the keys it visits, the groups are
// merged through LDS, and the chunk's (o, m, l) goes to `part` for decode_merge_kernel.
template <typename TV, int D>
__global__ __launch_bounds__(256) void decode_attend_kernel(const TV* __restrict__ q, const TV* __restrict__ K,
                                                            const TV* __restrict__ V, const float* __restrict__ z,
                                                            const int32_t* __restrict__ cu,
                                                            const int32_t* __restrict__ kept, float* part, int T,
                                                            int H_q, int H_kv, int k, int nsplit, float c2) {
  const int bh = blockIdx.x, b = bh / H_q, h = bh % H_q, sp = blockIdx.y;
  const int n = cu[b + 1] - cu[b];
  const int kcap = k < T ? k : T, kk = k < n ? k : n;
  const int32_t* list = kept + (size_t)bh * kcap;
  const int i0 = sp * DEC_CHUNK, i1 = min(i0 + DEC_CHUNK, kk);
  constexpr int LPR = D / 8, NG = 256 / LPR;
  const int tid = threadIdx.x, sub = tid % LPR, grp = tid / LPR;
  const int g = h / (H_q / H_kv);
  float* out = part + ((size_t)bh * nsplit + sp) * (D + 2);
  auto load8 = [&](const TV* p, float* o8) {
    if constexpr (sizeof(TV) == 2) {
      const uint4 raw = *reinterpret_cast<const uint4*>(p);
      const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
      for (int e = 0; e < 4; e++) {
        o8[2 * e] = __uint_as_float(u[e] << 16);
        o8[2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
      }
    } else {
      const float4 x0 = *reinterpret_cast<const float4*>(p);
      const float4 x1 = *reinterpret_cast<const float4*>(p + 4);
      o8[0] = x0.x; o8[1] = x0.y; o8[2] = x0.z; o8[3] = x0.w;
      o8[4] = x1.x; o8[5] = x1.y; o8[6] = x1.z; o8[7] = x1.w;
    }
  };
  float qv[8];
  load8(q + ((size_t)b * H_q + h) * D + 8 * sub, qv);
  float m = -INFINITY, lsum = 0.f, acc[8];
#pragma unroll
  for (int e = 0; e < 8; e++) acc[e] = 0.f;
  constexpr int U = 4;  // keys in flight per lane group
  for (int i = i0 + grp; i < i1; i += NG * U) {
    float kv[U][8], vv[U][8], zz[U];
    bool ok[U];
#pragma unroll
    for (int u = 0; u < U; u++) {
      const int ii = i + u * NG;
      ok[u] = ii < i1;
      const int id = ok[u] ? list[ii] : list[i];
      const size_t off = ((size_t)id * H_kv + g) * D + 8 * sub;
      load8(K + off, kv[u]);
      load8(V + off, vv[u]);
      zz[u] = z[(size_t)h * T + id];
    }
#pragma unroll
    for (int u = 0; u < U; u++) {
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < 8; e++) s = fmaf(qv[e], kv[u][e], s);
#pragma unroll
      for (int sft = LPR / 2; sft > 0; sft >>= 1) s += __shfl_xor(s, sft);
      if (ok[u]) {
        const float s2 = fmaf(s, c2, zz[u] * LOG2E);  // exp2 domain
        const float m_new = fmaxf(m, s2);
        const float alpha = fast_exp2(m - m_new), pv = fast_exp2(s2 - m_new);
        m = m_new;
        lsum = lsum * alpha + pv;
#pragma unroll
        for (int e = 0; e < 8; e++) acc[e] = fmaf(acc[e], alpha, pv * vv[u][e]);
      }
    }
  }
  __shared__ float mo[NG][D + 2];
#pragma unroll
  for (int e = 0; e < 8; e++) mo[grp][8 * sub + e] = acc[e];
  if (sub == 0) {
    mo[grp][D] = m;
    mo[grp][D + 1] = lsum;
  }
  __syncthreads();
  if (tid < D) {
    float M = -INFINITY;
    for (int gi = 0; gi < NG; gi++) M = fmaxf(M, mo[gi][D]);
    float num = 0.f, den = 0.f;
    for (int gi = 0; gi < NG; gi++) {
      const float w8 = mo[gi][D] == -INFINITY ? 0.f : fast_exp2(mo[gi][D] - M);  // a group that saw no key
      num = fmaf(mo[gi][tid], w8, num);
      den = fmaf(mo[gi][D + 1], w8, den);
    }
    out[tid] = num;  // un-normalised: sum of exp2(s2 - M) v
    if (tid == 0) {
      out[D] = M;
      out[D + 1] = den;
    }
  }
}

// (4) merge the chunks of one (sequence, head): o = sum_c o_c 2^(M_c - M) / sum_c l_c 2^(M_c - M).
template <typename TV, int D>
__global__ __launch_bounds__(D) void decode_merge_kernel(const float* __restrict__ part, const int32_t* __restrict__ cu,
                                                         TV* o, float* lse, int H_q, int k, int nsplit) {
  const int bh = blockIdx.x, b = bh / H_q, h = bh % H_q, n_docs = gridDim.x / H_q, c = threadIdx.x;
  const int n = cu[b + 1] - cu[b];
  TV* orow = o + (size_t)bh * D;
  if (n <= 0) {  // empty sequence: zero output, LSE = -inf
    orow[c] = TV(0.f);
    if (c == 0) lse[(size_t)h * n_docs + b] = -INFINITY;
    return;
  }
  const int kk = k < n ? k : n, ns = (kk + DEC_CHUNK - 1) / DEC_CHUNK;
  const float* p = part + (size_t)bh * nsplit * (D + 2);
  float M = -INFINITY;
  for (int s = 0; s < ns; s++) M = fmaxf(M, p[s * (D + 2) + D]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < ns; s++) {
    const float w8 = fast_exp2(p[s * (D + 2) + D] - M);
    num = fmaf(p[s * (D + 2) + c], w8, num);
    den = fmaf(p[s * (D + 2) + D + 1], w8, den);
  }
  orow[c] = TV(num / den);
  if (c == 0) lse[(size_t)h * n_docs + b] = (M + __builtin_amdgcn_logf(den)) * LN2;
}

// scratch after the kept lists: per (sequence, head) and chunk, D + 2 floats
size_t decode_part_floats(const dma_shape& s) {
  const size_t kcap = (size_t)(s.k < s.T ? s.k : s.T);
  return (size_t)s.n_docs * s.H_q * ((kcap + DEC_CHUNK - 1) / DEC_CHUNK) * (s.d + 2);
}

template <typename TV, int D>
static void launch_decode_t(const dma_shape& s, float c2, const void* q, const void* K, const void* V, const float* z,
                            const int32_t* cu, void* o, float* lse, int32_t* kept, float* part, int nsplit,
                            hipStream_t st) {
  const int nbh = s.n_docs * s.H_q;
  decode_attend_kernel<TV, D><<<dim3(nbh, nsplit), 256, 0, st>>>((const TV*)q, (const TV*)K, (const TV*)V, z, cu, kept,
                                                                  part, s.T, s.H_q, s.H_kv, s.k, nsplit, c2);
  decode_merge_kernel<TV, D><<<nbh, D, 0, st>>>(part, cu, (TV*)o, lse, s.H_q, s.k, nsplit);
}

int launch_decode(const dma_shape& s, float scale, const void* q, const void* K, const void* V, const float* z,
                  const int32_t* cu, void* o, float* lse, int32_t* kept, hipStream_t st) {
  const float c2 = scale * LOG2E;
  const size_t kcap = (size_t)(s.k < s.T ? s.k : s.T);
  const int nsplit = (int)((kcap + DEC_CHUNK - 1) / DEC_CHUNK);
  float* part = reinterpret_cast<float*>(reinterpret_cast<char*>(kept) +
                                         align_up((size_t)s.n_docs * s.H_q * kcap * 4, 256));
  decode_select_kernel<<<dim3(s.n_docs, s.H_q), 1024, 0, st>>>(z, cu, kept, s.T, s.H_q, s.k);
  if (s.dtype == DMA_BF16) {
    if (s.d == 128) launch_decode_t<__bf16, 128>(s, c2, q, K, V, z, cu, o, lse, kept, part, nsplit, st);
    else launch_decode_t<__bf16, 64>(s, c2, q, K, V, z, cu, o, lse, kept, part, nsplit, st);
  } else {
    if (s.d == 128) launch_decode_t<float, 128>(s, c2, q, K, V, z, cu, o, lse, kept, part, nsplit, st);
    else launch_decode_t<float, 64>(s, c2, q, K, V, z, cu, o, lse, kept, part, nsplit, st);
  }
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

}  // namespace dma
