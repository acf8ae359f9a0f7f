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

// ---- selection of the kept set, spread over nsl slices of every (sequence, q-head) so that it
// uses the whole chip: four histogram launches (radix select of the kk-th best score, most
// significant byte first, per-pass histograms accumulated in global memory), one counting launch
// and one ordered-compaction launch.  Every workgroup re-derives the digits already fixed from the
// finished histograms (256 counters per pass), so no launch has to hand state to the next one.
struct DecSel {
  const float* z;
  const int32_t* cu;
  const int32_t* lens;  // nullable: current length of each sequence inside its rows [cu[b], cu[b + 1])
  int32_t* kept;
  uint32_t* hist;  // [4][n_docs * H_q][256], zeroed before the first pass
  uint32_t* cnt;   // [n_docs * H_q][nsl][4 waves][2]: keys better than / equal to the threshold
  int T, H_q, k, nsl;
};

// Wave 0: the digit of `h256` at which the running count reaches `remaining`; updates prefix / remaining.
__device__ __forceinline__ void dec_pick(const uint32_t* h256, int l, uint32_t& prefix, uint32_t& remaining) {
  uint32_t c4[4], sum = 0;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    c4[i] = h256[4 * l + i];
    sum += c4[i];
  }
  uint32_t inc = sum;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t t = __shfl_up(inc, off);
    if (l >= off) inc += t;
  }
  uint32_t run = inc - sum, dig = 0, rem = 0;
  bool mine = false;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    if (!mine && run < remaining && remaining <= run + c4[i]) {
      mine = true;
      dig = 4 * l + i;
      rem = remaining - run;
    }
    run += c4[i];
  }
  const unsigned long long m = __ballot(mine);
  const int src = __ffsll((long long)m) - 1;  // exactly one lane finds it (remaining >= 1 and <= total)
  prefix = (prefix << 8) | (uint32_t)__shfl((int)dig, src);
  remaining = (uint32_t)__shfl((int)rem, src);
}

// length of sequence b: all of its rows, or lens[b] of them (clamped to the rows it owns)
__device__ __forceinline__ int dec_len(const int32_t* __restrict__ cu, const int32_t* __restrict__ lens, int b) {
  const int cap = cu[b + 1] - cu[b];
  return lens ? max(0, min(lens[b], cap)) : cap;
}

struct DecSlice {
  int a, n, kk, j0, j1;  // document start / length, kept count, this wave's key range [j0, j1)
};
__device__ __forceinline__ DecSlice dec_slice(const DecSel& p, int b, int sl, int w) {
  DecSlice s;
  s.a = p.cu[b];
  s.n = dec_len(p.cu, p.lens, b);
  s.kk = p.k < s.n ? p.k : s.n;
  const int slen = ((s.n + p.nsl - 1) / p.nsl + 255) / 256 * 256;
  const int wlen = slen / 4;
  s.j0 = min(s.n, sl * slen + w * wlen);
  s.j1 = min(s.n, sl * slen + (w + 1) * wlen);
  return s;
}

// Threshold state after the passes above `pass` (pass = -1: after all four).
__device__ __forceinline__ void dec_state(const DecSel& p, int bh, int nbh, int pass, int kk, int l, uint32_t* sh2) {
  if (threadIdx.x < 64) {
    uint32_t prefix = 0, remaining = (uint32_t)kk;
    for (int q = 3; q > pass; q--) dec_pick(p.hist + ((size_t)q * nbh + bh) * 256, l, prefix, remaining);
    if (l == 0) {
      sh2[0] = prefix;
      sh2[1] = remaining;
    }
  }
  __syncthreads();
}

__global__ __launch_bounds__(256) void decode_hist_kernel(DecSel p, int pass) {
  const int bh = blockIdx.x, b = bh / p.H_q, h = bh % p.H_q, sl = blockIdx.y, nbh = gridDim.x;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
  const DecSlice s = dec_slice(p, b, sl, w);
  if (s.n <= 0 || s.kk == s.n) return;  // (workgroup-uniform)
  // every digit has 32 sub-counters (one per lane pair), so that the lanes of a wave that hit the
  // same digit (scores share their leading bits) do not serialise on one LDS address
  __shared__ uint32_t hist[256 * 32];
  __shared__ uint32_t st[2];
  for (int i = tid; i < 256 * 32; i += 256) hist[i] = 0;
  dec_state(p, bh, nbh, pass, s.kk, l, st);
  const uint32_t prefix = st[0];
  const float* zh = p.z + (size_t)h * p.T + s.a;
  const int sh = 8 * pass;
  for (int j0 = s.j0; j0 < s.j1; j0 += 8 * 64) {  // eight loads in flight per lane
    float zv[8];
#pragma unroll
    for (int u = 0; u < 8; u++) zv[u] = j0 + u * 64 + l < s.j1 ? zh[j0 + u * 64 + l] : 0.f;
#pragma unroll
    for (int u = 0; u < 8; u++) {
      const uint32_t key = desc_key_u32(zv[u]);
      if (j0 + u * 64 + l < s.j1 && (pass == 3 || (key >> (sh + 8)) == prefix))
        atomicAdd(&hist[((key >> sh) & 255u) * 32 + (l & 31)], 1u);
    }
  }
  __syncthreads();
  {
    uint32_t c = 0;
    for (int sc = 0; sc < 32; sc++) c += hist[tid * 32 + ((sc + tid) & 31)];
    if (c) atomicAdd(p.hist + ((size_t)pass * nbh + bh) * 256 + tid, c);
  }
}

__global__ __launch_bounds__(256) void decode_count_kernel(DecSel p) {
  const int bh = blockIdx.x, b = bh / p.H_q, h = bh % p.H_q, sl = blockIdx.y, nbh = gridDim.x;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
  const DecSlice s = dec_slice(p, b, sl, w);
  uint32_t* out = p.cnt + (((size_t)bh * p.nsl + sl) * 4 + w) * 2;
  if (s.n <= 0 || s.kk == s.n) {  // everything is kept
    if (l == 0) {
      out[0] = (uint32_t)(s.j1 - s.j0);
      out[1] = 0;
    }
    return;
  }
  __shared__ uint32_t st[2];
  dec_state(p, bh, nbh, -1, s.kk, l, st);
  const uint32_t thr = st[0];
  const float* zh = p.z + (size_t)h * p.T + s.a;
  uint32_t cb = 0, ce = 0;
  for (int j0 = s.j0; j0 < s.j1; j0 += 8 * 64) {
    float zv[8];
#pragma unroll
    for (int u = 0; u < 8; u++) zv[u] = j0 + u * 64 + l < s.j1 ? zh[j0 + u * 64 + l] : 0.f;
#pragma unroll
    for (int u = 0; u < 8; u++) {
      const bool in = j0 + u * 64 + l < s.j1;
      const uint32_t key = desc_key_u32(zv[u]);
      cb += (uint32_t)__popcll(__ballot(in && key < thr));
      ce += (uint32_t)__popcll(__ballot(in && key == thr));
    }
  }
  if (l == 0) {
    out[0] = cb;
    out[1] = ce;
  }
}

// Ordered compaction: keys better than the threshold, and the first need_eq keys equal to it, in
// ascending index order.
__global__ __launch_bounds__(256) void decode_write_kernel(DecSel p) {
  const int bh = blockIdx.x, b = bh / p.H_q, h = bh % p.H_q, sl = blockIdx.y, nbh = gridDim.x;
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
  const DecSlice s = dec_slice(p, b, sl, w);
  if (s.n <= 0) return;
  const int kcap = p.k < p.T ? p.k : p.T;
  int32_t* list = p.kept + (size_t)bh * kcap;
  __shared__ uint32_t st[2];
  uint32_t thr = 0xffffffffu, need_eq = 0;  // kk == n: every real key is "better"
  if (s.kk < s.n) {
    dec_state(p, bh, nbh, -1, s.kk, l, st);
    thr = st[0];
    need_eq = st[1];
  }
  // better / equal keys before this wave's range: the counts of all earlier (slice, wave) pairs
  uint32_t rb = 0, re = 0;
  {
    const uint32_t* c = p.cnt + (size_t)bh * p.nsl * 8;
    const int npairs = sl * 4 + w;
    for (int i = l; i < npairs; i += 64) {
      rb += c[2 * i];
      re += c[2 * i + 1];
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
      rb += __shfl_xor(rb, off);
      re += __shfl_xor(re, off);
    }
  }
  const unsigned long long lt = (1ull << l) - 1ull;
  const float* zh = p.z + (size_t)h * p.T + s.a;
  for (int j0 = s.j0; j0 < s.j1; j0 += 8 * 64) {
    float zv[8];
#pragma unroll
    for (int u = 0; u < 8; u++) zv[u] = j0 + u * 64 + l < s.j1 ? zh[j0 + u * 64 + l] : 0.f;
#pragma unroll
    for (int u = 0; u < 8; u++) {
      const int j = j0 + u * 64 + l;
      const uint32_t key = desc_key_u32(zv[u]);
      const bool in = j < s.j1;
      const bool better = in && (s.kk == s.n || key < thr), equal = in && s.kk < s.n && key == thr;
      const unsigned long long bm = __ballot(better), em = __ballot(equal);
      const uint32_t eq_before = re + (uint32_t)__popcll(em & lt);  // equal keys with a lower index
      const uint32_t pos = rb + (uint32_t)__popcll(bm & lt) + min(eq_before, need_eq);
      if (better || (equal && eq_before < need_eq)) list[pos] = s.a + j;
      rb += (uint32_t)__popcll(bm);
      re += (uint32_t)__popcll(em);
    }
  }
}

__global__ void decode_zero_kernel(uint32_t* p, size_t n) {
  const size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// ---- the kept set carried from one decode step to the next (Eq. 4 as a one-in / one-out update):
// `kept` holds the min(k, n - 1) best of the sequence's first n - 1 keys in ascending index order; the
// new key n - 1 joins while fewer than k are kept, otherwise it replaces the worst kept key if it
// beats it (a tie goes to the lower index, and the new key has the highest).  One workgroup per
// (sequence, head); O(k) work instead of a selection over all n scores.
__global__ __launch_bounds__(256) void decode_update_kernel(const float* __restrict__ z, const int32_t* __restrict__ cu,
                                                            const int32_t* __restrict__ lens, int32_t* kept, int T,
                                                            int H_q, int k) {
  const int bh = blockIdx.x, b = bh / H_q, h = bh % H_q, tid = threadIdx.x, l = tid & 63, w = tid >> 6;
  const int n = dec_len(cu, lens, b);
  if (n <= 0) return;
  const int kcap = k < T ? k : T, kprev = min(k, n - 1), jn = cu[b] + n - 1;
  int32_t* list = kept + (size_t)bh * kcap;
  if (kprev < k) {  // still filling (kprev < kcap: kprev <= n - 1 < T)
    if (tid == 0) list[kprev] = jn;
    return;
  }
  const float* zh = z + (size_t)h * T;
  // worst kept key: largest (descending-score key, index); position kept alongside.  Lists of up to
  // 8 * 256 entries stay in registers (all loads of a thread in flight together, and the shift below
  // needs no second pass over memory).
  constexpr int UPD_R = 8;
  const bool in_regs = kprev <= UPD_R * 256;
  int ids[UPD_R];
  unsigned long long worst = 0ull;
  int wpos = -1;
  if (in_regs) {
    float zz[UPD_R];
#pragma unroll
    for (int j = 0; j < UPD_R; j++) ids[j] = tid + 256 * j < kprev ? list[tid + 256 * j] : -1;
#pragma unroll
    for (int j = 0; j < UPD_R; j++) zz[j] = ids[j] >= 0 ? zh[ids[j]] : 0.f;
#pragma unroll
    for (int j = 0; j < UPD_R; j++) {
      const unsigned long long c = ((unsigned long long)desc_key_u32(zz[j]) << 32) | (uint32_t)ids[j];
      if (ids[j] >= 0 && (wpos < 0 || c > worst)) {
        worst = c;
        wpos = tid + 256 * j;
      }
    }
  } else {
    for (int i = tid; i < kprev; i += 256) {
      const int id = list[i];
      const unsigned long long c = ((unsigned long long)desc_key_u32(zh[id]) << 32) | (uint32_t)id;
      if (wpos < 0 || c > worst) {
        worst = c;
        wpos = i;
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    const unsigned long long oc = __shfl_xor(worst, off);
    const int op = __shfl_xor(wpos, off);
    if (op >= 0 && (wpos < 0 || oc > worst)) {
      worst = oc;
      wpos = op;
    }
  }
  __shared__ unsigned long long sw[4];
  __shared__ int sp[4];
  if (l == 0) {
    sw[w] = worst;
    sp[w] = wpos;
  }
  __syncthreads();
  for (int i = 0; i < 4; i++)
    if (sp[i] >= 0 && (wpos < 0 || sw[i] > worst)) {
      worst = sw[i];
      wpos = sp[i];
    }
  const unsigned long long cn = ((unsigned long long)desc_key_u32(zh[jn]) << 32) | (uint32_t)jn;
  if (cn > worst) return;  // the new key does not make it (workgroup-uniform)
  if (in_regs) {  // every entry was read before the barrier above: entries behind wpos move one place down
#pragma unroll
    for (int j = 0; j < UPD_R; j++) {
      const int i = tid + 256 * j;
      if (i > wpos && i < kprev) list[i - 1] = ids[j];
    }
    if (tid == 0) list[kprev - 1] = jn;
    return;
  }
  // drop position wpos: entries behind it move one place down, chunk by chunk (a chunk reads before
  // any thread writes, and a later chunk only overwrites what the earlier one has already read)
  for (int i0 = wpos; i0 < kprev - 1; i0 += 256) {
    const int i = i0 + tid;
    int v = 0;
    if (i < kprev - 1) v = list[i + 1];
    __syncthreads();
    if (i < kprev - 1) list[i] = v;
    __syncthreads();
  }
  if (tid == 0) list[kprev - 1] = jn;
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
                                                            const int32_t* __restrict__ lens,
                                                            const int32_t* __restrict__ kept, float* part, int T,
                                                            int H_q, int H_kv, int k, int nsplit, float c2) {
  const int bh = blockIdx.x, b = bh / H_q, h = bh % H_q, sp = blockIdx.y;
  const int n = dec_len(cu, lens, b);
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
                                                         const int32_t* __restrict__ lens, TV* o, float* lse, int H_q,
                                                         int k, int nsplit) {
  const int bh = blockIdx.x, b = bh / H_q, h = bh % H_q, n_docs = gridDim.x / H_q, c = threadIdx.x;
  const int n = dec_len(cu, lens, b);
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

// slices per (sequence, head) of the selection: enough workgroups for the chip, slices of >= 1024 keys
int decode_nsl(const dma_shape& s) {
  const long nbh = (long)s.n_docs * s.H_q;
  const int longest = s.max_seqlen > 0 && s.max_seqlen < s.T ? s.max_seqlen : s.T;
  long nsl = (1024 + nbh - 1) / nbh;
  const long cap = (longest + 1023) / 1024;
  if (nsl > cap) nsl = cap;
  if (nsl > 64) nsl = 64;
  if (nsl < 1) nsl = 1;
  return (int)nsl;
}

// scratch after the kept lists: per (sequence, head) and chunk, D + 2 floats of partial output;
// then the selection's histograms and slice counts (as 32-bit words)
size_t decode_part_floats(const dma_shape& s) {
  const size_t kcap = (size_t)(s.k < s.T ? s.k : s.T);
  return (size_t)s.n_docs * s.H_q * ((kcap + DEC_CHUNK - 1) / DEC_CHUNK) * (s.d + 2);
}
size_t decode_sel_words(const dma_shape& s) {
  const size_t nbh = (size_t)s.n_docs * s.H_q;
  return 4 * nbh * 256 + nbh * (size_t)decode_nsl(s) * 8;
}

template <typename TV, int D>
static void launch_decode_t(const dma_shape& s, float c2, const void* q, const void* K, const void* V, const float* z,
                            const int32_t* cu, const int32_t* lens, void* o, float* lse, int32_t* kept, float* part,
                            int nsplit, hipStream_t st) {
  const int nbh = s.n_docs * s.H_q;
  decode_attend_kernel<TV, D><<<dim3(nbh, nsplit), 256, 0, st>>>((const TV*)q, (const TV*)K, (const TV*)V, z, cu, lens,
                                                                  kept, part, s.T, s.H_q, s.H_kv, s.k, nsplit, c2);
  decode_merge_kernel<TV, D><<<nbh, D, 0, st>>>(part, cu, lens, (TV*)o, lse, s.H_q, s.k, nsplit);
}

// incremental == 0: the kept sets are selected from all scores; otherwise they are carried over from
// the previous step and updated with the newest key of every sequence.
// Scratch of dma_decode_static: the per-chunk partial outputs and the selection's histograms and
// counts of one call, held in the library's own device memory (every GPU the library runs on keeps
// its copy until the process ends).  Host code never passes the array's name to a kernel: the
// device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[DMA_DECODE_STATIC_SCRATCH_BYTES];
static void* g_scratch_ptr[64] = {};

size_t decode_scratch_bytes(const dma_shape& s) {
  return align_up(decode_part_floats(s) * 4, 256) + align_up(decode_sel_words(s) * 4, 256);
}

int decode_static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return DMA_EHIP;
  void* ptr = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return DMA_EHIP;
    __atomic_store_n(&g_scratch_ptr[dev], ptr, __ATOMIC_RELEASE);  // (two first callers store the same address)
  }
  *out = ptr;
  return DMA_OK;
}

// part_and_sel: the scratch region (decode_scratch_bytes): partial outputs, then histograms and counts
int launch_decode(const dma_shape& s, float scale, const void* q, const void* K, const void* V, const float* z,
                  const int32_t* cu, const int32_t* lens, int incremental, void* o, float* lse, int32_t* kept,
                  void* part_and_sel, hipStream_t st) {
  const float c2 = scale * LOG2E;
  const size_t kcap = (size_t)(s.k < s.T ? s.k : s.T);
  const int nsplit = (int)((kcap + DEC_CHUNK - 1) / DEC_CHUNK);
  float* part = reinterpret_cast<float*>(part_and_sel);
  const int nbh = s.n_docs * s.H_q;
  DecSel ds;
  ds.z = z; ds.cu = cu; ds.lens = lens; ds.kept = kept;
  ds.hist = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(part) + align_up(decode_part_floats(s) * 4, 256));
  ds.cnt = ds.hist + 4 * (size_t)nbh * 256;
  ds.T = s.T; ds.H_q = s.H_q; ds.k = s.k; ds.nsl = decode_nsl(s);
  if (incremental) {
    decode_update_kernel<<<nbh, 256, 0, st>>>(z, cu, lens, kept, s.T, s.H_q, s.k);
  } else {
    const size_t nz = 4 * (size_t)nbh * 256;
    decode_zero_kernel<<<(unsigned)((nz + 255) / 256), 256, 0, st>>>(ds.hist, nz);
    const dim3 sgrid(nbh, ds.nsl);
    for (int pass = 3; pass >= 0; pass--) decode_hist_kernel<<<sgrid, 256, 0, st>>>(ds, pass);
    decode_count_kernel<<<sgrid, 256, 0, st>>>(ds);
    decode_write_kernel<<<sgrid, 256, 0, st>>>(ds);
  }
  if (s.dtype == DMA_BF16) {
    if (s.d == 256) launch_decode_t<__bf16, 256>(s, c2, q, K, V, z, cu, lens, o, lse, kept, part, nsplit, st);
    else if (s.d == 128) launch_decode_t<__bf16, 128>(s, c2, q, K, V, z, cu, lens, o, lse, kept, part, nsplit, st);
    else launch_decode_t<__bf16, 64>(s, c2, q, K, V, z, cu, lens, o, lse, kept, part, nsplit, st);
  } else {
    if (s.d == 256) launch_decode_t<float, 256>(s, c2, q, K, V, z, cu, lens, o, lse, kept, part, nsplit, st);
    else if (s.d == 128) launch_decode_t<float, 128>(s, c2, q, K, V, z, cu, lens, o, lse, kept, part, nsplit, st);
    else launch_decode_t<float, 64>(s, c2, q, K, V, z, cu, lens, o, lse, kept, part, nsplit, st);
  }
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

}  // namespace dma
