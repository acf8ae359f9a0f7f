// Mask generation: content scores (Eq. 3), per-row causal top-k as one expiry per key (Eq. 4),
// and the slot table / per-block partial key lists the attention kernels walk.
//
// Selection.  Row i keeps the min(k, i+1) best keys j <= i under (z descending, index ascending).
// Sort the keys of a document once under that order (stable radix sort); the keys that rank ahead
// of key j are exactly its "dominators".  Key j stops being kept at the row where the k-th
// dominator (in index order) appears, so
//     e_j = max(j, k-th smallest index among the keys ranked ahead of j)
// (never kept if that index is below j; kept to the end if fewer than k keys rank ahead).  The
// k-th smallest index in a rank prefix is a range-quantile query, answered with a wavelet matrix
// built over the rank-ordered index array.  Everything is integer work on the fp32 score bits, so
// the result is the exact kept set of the scores as stored.
//
// Slots.  While a document has more than k rows, each row admits at most one key and evicts the
// weakest resident; the newcomer inherits the evicted key's "slot".  Slot chains partition the
// kept region into k columns that are always occupied, which gives the attention kernels dense
// tiles: per query block, the resident of every slot that stays the whole block ("clean"), plus a
// short list of keys that enter or expire inside the block ("partial").
#include "common.h"

namespace dma {

// The plan's constant block: a zero K/V row for empty slots, then the -inf / 0 / -1 / +inf scalars
// the asynchronous copies point at for empty ids (words 64, 65, 66, 67), then the softmax scale that
// z / scale is written with and scale * log2(e) (words 68, 69): the attention kernels take the scale
// from here, so it cannot differ from the one in the stored scores.
__device__ __forceinline__ void plan_consts(uint32_t* consts, size_t i, float scale) {
  if (i < 128) {
    uint32_t v = 0u;
    if (i == 64) v = 0xff800000u;       // float -inf
    if (i == 66) v = 0xffffffffu;       // int -1
    if (i == 67) v = 0x7f800000u;       // float +inf
    if (i == 68) v = __float_as_uint(scale);
    if (i == 69) v = __float_as_uint(scale * LOG2E);
    consts[i] = v;
  }
}

// ------------------------------------------------------------------ block table
// blk[i] = {document, first row, end row, w}: the attention kernels take min(k, first row - w) as the
// number of resident slot columns of the block.  Causal: w = first row of the document (the keys
// before the block); otherwise every block of a document has min(k, n) columns.
__global__ void blkinfo_kernel(const int32_t* __restrict__ cu, int n_docs, int nblk_cap, int k, int causal, int4* blk,
                               int32_t* docblk, int32_t* hdr, uint32_t* consts, float scale) {
  __shared__ int s_total, s_scan[256];
  plan_consts(consts, threadIdx.x, scale);
  // docblk = exclusive prefix sum of the documents' block counts: 256 documents per round, a
  // Hillis-Steele scan in LDS inside the round, the running total carried between rounds
  const int tid = threadIdx.x;
  int base = 0;
  for (int d0 = 0; d0 < n_docs; d0 += 256) {
    const int d = d0 + tid;
    const int nb = d < n_docs ? (cu[d + 1] - cu[d] + BQ - 1) / BQ : 0;
    s_scan[tid] = nb;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
      const int v = tid >= off ? s_scan[tid - off] : 0;
      __syncthreads();
      s_scan[tid] += v;
      __syncthreads();
    }
    if (d < n_docs) docblk[d] = base + s_scan[tid] - nb;
    base += s_scan[255];
    __syncthreads();
  }
  if (tid == 0) {
    docblk[n_docs] = base;
    hdr[0] = base;
    s_total = base;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < s_total; i += blockDim.x) {  // one block per thread
    int lo = 0, hi = n_docs;  // its document: the last d with docblk[d] <= i (empty documents own no block)
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (docblk[mid] <= i) lo = mid; else hi = mid;
    }
    const int a = cu[lo], b = cu[lo + 1], r = a + (i - docblk[lo]) * BQ;
    blk[i] = make_int4(lo, r, min(r + BQ, b), causal ? a : r - min(k, b - a));
  }
  for (int i = s_total + threadIdx.x; i < nblk_cap; i += blockDim.x) blk[i] = make_int4(-1, 0, 0, 0);
}

__global__ void fill_i32_kernel(int32_t* p, size_t n, int32_t v) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  size_t st = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += st) p[i] = v;
}

// ------------------------------------------------------------------ content scores (Eq. 3)
// One workgroup per (64 tokens, kv-head): each value row is read once and scored for all q-heads
// of its group.  z = exp(A * softplus(w . v)) in fp32; z / softmax_scale is written next to it
// (the attention kernels start their Q K^T accumulators at it).  A row is held by D / 8 lanes; the
// loads of the tile's rows are all in flight before the first dot product, and a group of up to
// GMAX q-heads keeps this lane's 8 weights of every head in registers.
template <typename TV, int D, int GMAX>
__global__ __launch_bounds__(256) void z_kernel(const TV* __restrict__ V, const float* __restrict__ W,
                                                const float* __restrict__ A, float* __restrict__ z,
                                                float* __restrict__ zq, float inv_scale, int T, int H_q, int H_kv) {
  extern __shared__ float zs[];  // [G][64]
  constexpr int LPR = D / 8;     // lanes per value row (8 elements per lane)
  constexpr int RPP = 256 / LPR; // rows per pass
  constexpr int NP = 64 / RPP;
  const int g = blockIdx.y, G = H_q / H_kv, t0 = blockIdx.x * 64;
  const int tid = threadIdx.x, sub = tid % LPR, rl = tid / LPR;
  float v[NP][8];
#pragma unroll
  for (int pass = 0; pass < NP; pass++) {
    const int t = t0 + pass * RPP + rl;
#pragma unroll
    for (int e = 0; e < 8; e++) v[pass][e] = 0.f;
    if (t < T) {
      const TV* src = V + ((size_t)t * H_kv + g) * D + 8 * sub;
      if constexpr (sizeof(TV) == 2) {
        const uint4 raw = *reinterpret_cast<const uint4*>(src);
        const uint32_t u[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int e = 0; e < 4; e++) {
          v[pass][2 * e] = __uint_as_float(u[e] << 16);
          v[pass][2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
        }
      } else {
        const float4 x0 = *reinterpret_cast<const float4*>(src);
        const float4 x1 = *reinterpret_cast<const float4*>(src + 4);
        v[pass][0] = x0.x; v[pass][1] = x0.y; v[pass][2] = x0.z; v[pass][3] = x0.w;
        v[pass][4] = x1.x; v[pass][5] = x1.y; v[pass][6] = x1.z; v[pass][7] = x1.w;
      }
    }
  }
  for (int h0 = 0; h0 < G; h0 += GMAX) {  // (one trip unless the group has more than GMAX q-heads)
    float wreg[GMAX][8];
#pragma unroll
    for (int hh = 0; hh < GMAX; hh++) {
      const float4* w4 = reinterpret_cast<const float4*>(W + (size_t)(g * G + min(h0 + hh, G - 1)) * D + 8 * sub);
      const float4 a = w4[0], b = w4[1];
      wreg[hh][0] = a.x; wreg[hh][1] = a.y; wreg[hh][2] = a.z; wreg[hh][3] = a.w;
      wreg[hh][4] = b.x; wreg[hh][5] = b.y; wreg[hh][6] = b.z; wreg[hh][7] = b.w;
    }
#pragma unroll
    for (int pass = 0; pass < NP; pass++) {
      const int r = pass * RPP + rl;
#pragma unroll
      for (int hh = 0; hh < GMAX; hh++) {
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e++) acc = fmaf(v[pass][e], wreg[hh][e], acc);
#pragma unroll
        for (int off = LPR / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off);
        if (sub == 0 && h0 + hh < G) zs[(h0 + hh) * 64 + r] = acc;
      }
    }
  }
  __syncthreads();
  for (int idx = tid; idx < G * 64; idx += 256) {
    const int hh = idx / 64, r = idx % 64, t = t0 + r;
    if (t < T) {
      const float x = zs[idx];
      const float sp = fmaxf(x, 0.f) + log1pf(expf(-fabsf(x)));
      const float zv = expf(A[g * G + hh] * sp);
      const size_t o = (size_t)(g * G + hh) * T + t;
      z[o] = zv;
      zq[o] = zv * inv_scale;
    }
  }
}

// zq = z / softmax_scale for scores supplied by the caller (the attention kernels start their
// Q K^T accumulators at it, so that scale * accumulator is the biased score).
__global__ __launch_bounds__(256) void zq_kernel(const float* __restrict__ z, float* __restrict__ zq,
                                                 float inv_scale, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t st = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += st) zq[i] = z[i] * inv_scale;
}

// ------------------------------------------------------------------ sort + wavelet matrix
// Ascending unsigned order of the result == descending float order of z (-0 and +0 compare equal).
__device__ __forceinline__ uint32_t desc_key(float z) {
  z = z + 0.0f;
  uint32_t u = __float_as_uint(z);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ~u;
}

__device__ __forceinline__ int dev_ceil_log2(int n) { return n <= 1 ? 0 : 32 - __clz(n - 1); }

struct SortArgs {
  const float* z;
  const int32_t* cu;
  int32_t* expiry;
  uint32_t *sk0, *sk1, *si0, *si1;
  unsigned long long* wbits;
  uint32_t* wcnt;
  uint32_t* wzero;
  int T, n_docs, k, nbits_cap, wcap, nseg_cap, seg;
};

// Documents are handled in segments of `seg` consecutive keys (4096 or 16384, one launch-wide
// choice).  Segment p of document d (first token a) has the slot number a / seg + d + p, unique and
// increasing over the batch, and its wavelet levels start at word seg_woff of each level's row.
__device__ __forceinline__ int seg_slot(int seg, int a, int d, int p) { return a / seg + d + p; }
__device__ __forceinline__ int seg_woff(int seg, int a, int d, int p) {
  return a / 64 + 2 * (a / seg) + 5 * d + p * (seg / 64 + 2);
}

// One workgroup (16 waves) per (segment, head).  The segment's keys are sorted by (score descending,
// index ascending) -- a stable LSD radix sort on 8-bit digits, entirely in registers and LDS: every
// wave owns a contiguous run of 64-key chunks, counts its digits, and after a (digit, wave)-ordered
// scan scatters its chunks in order, ranking equal digits inside a chunk with ballots -- and a
// wavelet matrix is built over the rank-ordered local indices (most significant bit first: per 64
// positions the mask of zero bits and the number of zeros before the word; the array is stably
// partitioned, zeros first, for the next level).  A document of one segment leaves its rank order in
// si0 for expiry_kernel; the segments of a longer document leave their sorted keys and local
// indices in sk1 / si1 for merge_expiry_kernel.
template <int NB>  // chunks of 64 keys per wave: a segment is 16 waves x NB chunks = 1024 NB keys
__global__ __launch_bounds__(1024) void sort_wavelet_kernel(SortArgs p) {
  constexpr int SEG = 1024 * NB;
  const int slot = blockIdx.x, h = blockIdx.y;
  // the document whose segment range [seg_slot(a, d, 0), seg_slot(a, d, nseg)) holds this slot
  int d = 0;
  {
    int lo = 0, hi = p.n_docs;  // answer in [lo, hi): largest d with seg_slot(cu[d], d, 0) <= slot
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (seg_slot(SEG, p.cu[mid], mid, 0) <= slot) lo = mid; else hi = mid;
    }
    d = lo;
  }
  const int a = p.cu[d], b = p.cu[d + 1], ndoc = b - a;
  const int ps = slot - seg_slot(SEG, a, d, 0), nseg = (ndoc + SEG - 1) / SEG;
  if (ndoc <= 0 || ps >= nseg) return;
  const int n = min(SEG, ndoc - ps * SEG);  // keys of this segment
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
  const size_t hb = (size_t)h * p.T + a + (size_t)ps * SEG;
  if (ndoc <= p.k) {  // every causal key is kept by every later row
    for (int j = tid; j < n; j += 1024) p.expiry[hb + j] = b;
    return;
  }
  __shared__ uint32_t hist[4096];  // [digit][wave]
  __shared__ uint32_t wsum[16];
  const int nchunks = (n + 63) / 64, cpw = (nchunks + 15) / 16;
  const int c_begin = w * cpw;
  const unsigned long long lt = (1ull << l) - 1ull;
  constexpr int LDS_N = SEG;
  {
    // ---- whole segment in registers (16 elements per thread, chunk c of a wave = elements
    // 64c + lane) and LDS: every pass scatters from registers into LDS and reads its chunks back.
    __shared__ __align__(16) uint32_t lk[LDS_N];
    __shared__ __align__(16) uint32_t li[LDS_N];
    uint32_t kk[NB], ii[NB];
#pragma unroll
    for (int i = 0; i < NB; i++) {
      const int j = (c_begin + i) * 64 + l;
      const bool valid = i < cpw && j < n;
      kk[i] = valid ? desc_key(p.z[hb + j]) : 0u;
      ii[i] = (uint32_t)j;
    }
    for (int pass = 0; pass < 4; pass++) {
      const int shift = 8 * pass;
      for (int i = tid; i < 4096; i += 1024) hist[i] = 0;
      __syncthreads();
#pragma unroll
      for (int i = 0; i < NB; i++) {
        const int j = (c_begin + i) * 64 + l;
        if (i < cpw && j < n) atomicAdd(&hist[((kk[i] >> shift) & 255u) * 16 + w], 1u);
      }
      __syncthreads();
      {  // exclusive scan of hist[4096] in (digit, wave) order
        const uint32_t v0 = hist[4 * tid], v1 = hist[4 * tid + 1], v2 = hist[4 * tid + 2], v3 = hist[4 * tid + 3];
        const uint32_t sm = v0 + v1 + v2 + v3;
        uint32_t inc = sm;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
          const uint32_t t = __shfl_up(inc, off);
          if (l >= off) inc += t;
        }
        if (l == 63) wsum[w] = inc;
        __syncthreads();
        uint32_t wbase = 0;
        for (int i = 0; i < w; i++) wbase += wsum[i];
        const uint32_t ex = wbase + inc - sm;
        hist[4 * tid] = ex;
        hist[4 * tid + 1] = ex + v0;
        hist[4 * tid + 2] = ex + v0 + v1;
        hist[4 * tid + 3] = ex + v0 + v1 + v2;
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < NB; i++) {
        const int j = (c_begin + i) * 64 + l;
        const bool valid = i < cpw && j < n;
        const uint32_t dig = (kk[i] >> shift) & 255u;
        unsigned long long m = __ballot(valid);
#pragma unroll
        for (int bit = 0; bit < 8; bit++) {
          const bool one = (dig >> bit) & 1u;
          const unsigned long long bm = __ballot(one);
          m &= one ? bm : ~bm;
        }
        const uint32_t rank = __popcll(m & lt);
        const uint32_t base = hist[dig * 16 + w];
        if (valid) {
          lk[base + rank] = kk[i];
          li[base + rank] = ii[i];
          if (rank == 0) hist[dig * 16 + w] = base + (uint32_t)__popcll(m);
        }
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < NB; i++) {
        const int j = (c_begin + i) * 64 + l;
        if (i < cpw && j < n) {
          kk[i] = lk[j];
          ii[i] = li[j];
        }
      }
    }
    // sorted: kk / ii hold the keys and the local indices in rank order
    if (nseg == 1) {
#pragma unroll
      for (int i = 0; i < NB; i++) {
        const int j = (c_begin + i) * 64 + l;
        if (i < cpw && j < n) p.si0[hb + j] = ii[i];
      }
    } else {
#pragma unroll
      for (int i = 0; i < NB; i++) {
        const int j = (c_begin + i) * 64 + l;
        if (i < cpw && j < n) {
          p.sk1[hb + j] = kk[i];
          p.si1[hb + j] = ii[i];
        }
      }
    }
    // wavelet matrix over ii (see below), partitioned through LDS; the level tables are collected
    // in the (now free) key buffer and written out once at the end, so no level waits on a store
    const int nbits = dev_ceil_log2(n);
    const int woff = seg_woff(SEG, a, d, ps);
    const int lrow = nchunks + 1;  // entries per level
    unsigned long long* lwb = reinterpret_cast<unsigned long long*>(lk);  // [nbits][lrow]
    uint32_t* lwc = lk + 2 * 14 * (LDS_N / 64 + 1);                        // [nbits][lrow]
    static_assert(3 * 14 * (LDS_N / 64 + 1) <= LDS_N, "level tables must fit the key buffer");
    for (int lev = 0; lev < nbits; lev++) {
      const int sh = nbits - 1 - lev;
      unsigned long long* wb = lwb + lev * lrow;
      uint32_t* wc = lwc + lev * lrow;
      uint32_t zc = 0;
#pragma unroll
      for (int i = 0; i < NB; i++) {
        const int j = (c_begin + i) * 64 + l;
        const bool zero = i < cpw && j < n && !((ii[i] >> sh) & 1u);
        zc += (uint32_t)__popcll(__ballot(zero));
      }
      __syncthreads();  // the previous level's reads of wsum / li are done
      if (l == 0) wsum[w] = zc;
      __syncthreads();
      uint32_t run = 0, Z = 0;
      for (int i = 0; i < 16; i++) {
        const uint32_t x = wsum[i];
        if (i < w) run += x;
        Z += x;
      }
#pragma unroll
      for (int i = 0; i < NB; i++) {
        const int c = c_begin + i, j = c * 64 + l;
        const bool valid = i < cpw && j < n;
        const bool zero = valid && !((ii[i] >> sh) & 1u);
        const unsigned long long zm = __ballot(zero);
        const uint32_t zb = run + (uint32_t)__popcll(zm & lt);  // zeros before position j
        if (l == 0 && i < cpw && c < nchunks) {
          wb[c] = zm;
          wc[c] = run;
        }
        if (valid) li[zero ? zb : Z + ((uint32_t)j - zb)] = ii[i];
        run += (uint32_t)__popcll(zm);
      }
      if (tid == 0) {
        wb[nchunks] = 0ull;
        wc[nchunks] = Z;
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < NB; i++) {
        const int j = (c_begin + i) * 64 + l;
        if (i < cpw && j < n) ii[i] = li[j];
      }
    }
    for (int i = tid; i < nbits * lrow; i += 1024) {
      const int lev = i / lrow, c = i - lev * lrow;
      const size_t o = ((size_t)h * p.nbits_cap + lev) * p.wcap + woff + c;
      p.wbits[o] = lwb[i];
      p.wcnt[o] = lwc[i];
      if (c == nchunks) p.wzero[((size_t)h * p.nseg_cap + slot) * p.nbits_cap + lev] = lwc[i];
    }
  }
}

// The kk-th smallest (0-based) local index among the first `hi` rank positions of a segment:
// one range-quantile query on its wavelet matrix.
__device__ __forceinline__ uint32_t wavelet_kth(const SortArgs& p, int h, int slot, int woff, int nbits, uint32_t hi,
                                                uint32_t kk) {
  uint32_t lo = 0, val = 0;
  for (int lev = 0; lev < nbits; lev++) {
    const unsigned long long* wb = p.wbits + ((size_t)h * p.nbits_cap + lev) * p.wcap + woff;
    const uint32_t* wc = p.wcnt + ((size_t)h * p.nbits_cap + lev) * p.wcap + woff;
    const uint32_t zlo = wc[lo >> 6] + (uint32_t)__popcll(wb[lo >> 6] & ((1ull << (lo & 63)) - 1ull));
    const uint32_t zhi = wc[hi >> 6] + (uint32_t)__popcll(wb[hi >> 6] & ((1ull << (hi & 63)) - 1ull));
    const uint32_t c0 = zhi - zlo;
    if (kk < c0) {
      lo = zlo;
      hi = zhi;
    } else {
      kk -= c0;
      const uint32_t Z = p.wzero[((size_t)h * p.nseg_cap + slot) * p.nbits_cap + lev];
      lo = Z + (lo - zlo);
      hi = Z + (hi - zhi);
      val |= 1u << (nbits - 1 - lev);
    }
  }
  return val;
}

// Documents of one segment.  One thread per (head, rank position): expiry of the key at that rank,
// e_j = max(j, k-th smallest index among the keys ranked ahead of j).
__global__ __launch_bounds__(256) void expiry_kernel(SortArgs p) {
  const int t = blockIdx.x * 256 + threadIdx.x, h = blockIdx.y;
  if (t >= p.T) return;
  const int d = find_doc(p.cu, p.n_docs, t);
  const int a = p.cu[d], b = p.cu[d + 1], n = b - a;
  if (n <= p.k || n > p.seg) return;
  const int r = t - a;
  const int j = (int)p.si0[(size_t)h * p.T + t];
  int e = b;
  if (r >= p.k)
    e = a + max(j, (int)wavelet_kth(p, h, seg_slot(p.seg, a, d, 0), seg_woff(p.seg, a, d, 0), dev_ceil_log2(n), (uint32_t)r,
                                    (uint32_t)p.k - 1u));
  p.expiry[(size_t)h * p.T + a + j] = e;
}

// Longer documents.  One thread per (head, key), visited in the sorted order of its segment.  Its
// rank in the whole document is its rank in the segment plus, for every other segment, the number
// of keys there that come before it -- a binary search in that segment's sorted keys (ties go to
// the lower index, i.e. to the earlier segment).  Those same counts say how many of the keys ranked
// ahead of it lie in each segment, so the k-th smallest index among them is found by walking the
// segments in index order and asking the wavelet matrix of the one that holds it.
// RANK (no causal restriction): only the key's rank in the whole document is needed (every segment is
// searched).  Otherwise only the expiry is: the segments are searched in index order and the walk stops
// at the one that holds the k-th earlier-ranked key -- for most keys of a long document the first
// segment already holds k better keys, and an answer in an earlier segment needs no quantile query
// (every index there is below the key's own, so the key is never kept).
template <bool RANK>
__global__ __launch_bounds__(256) void merge_expiry_kernel(SortArgs p) {
  const int t = blockIdx.x * 256 + threadIdx.x, h = blockIdx.y;
  if (t >= p.T) return;
  const int d = find_doc(p.cu, p.n_docs, t);
  const int a = p.cu[d], b = p.cu[d + 1], n = b - a;
  const int SEG = p.seg;
  if (n <= p.k || n <= SEG) return;
  const int nseg = (n + SEG - 1) / SEG;
  const int ps = (t - a) / SEG, r = (t - a) - ps * SEG;
  const size_t hd = (size_t)h * p.T + a;
  const uint32_t key = p.sk1[hd + (t - a)];
  const int j = ps * SEG + (int)p.si1[hd + (t - a)];  // index in the document
  // keys of segment s that precede (key, j): all equal keys of an earlier segment do, none of a later one
  auto before = [&](int s) -> int {
    if (s == ps) return r;
    const uint32_t* ks = p.sk1 + hd + (size_t)s * SEG;
    int lo = 0, hi = min(SEG, n - s * SEG);
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      const uint32_t v = ks[mid];
      if (s < ps ? v <= key : v < key) lo = mid + 1; else hi = mid;
    }
    return lo;
  };
  if (RANK) {
    int R = 0;
    for (int s = 0; s < nseg; s++) R += before(s);
    p.si0[hd + R] = (uint32_t)j;  // rank order of the whole document
    return;
  }
  int e = b;
  uint32_t kk = (uint32_t)p.k - 1u;
  for (int s = 0; s < nseg; s++) {
    const uint32_t c = (uint32_t)before(s);
    if (kk < c) {
      e = a + j;
      if (s >= ps) {
        const int ns = min(SEG, n - s * SEG);
        const int val = (int)wavelet_kth(p, h, seg_slot(SEG, a, d, s), seg_woff(SEG, a, d, s), dev_ceil_log2(ns), c, kk);
        e = a + max(j, s * SEG + val);
      }
      break;
    }
    kk -= c;
  }
  p.expiry[hd + j] = e;
}

// ------------------------------------------------------------------ slots
// parent[i] = the key evicted when key i entered (global index, -1 if none); slotid[i] = root of
// i's eviction chain = its slot column (document-local, < k).
__global__ __launch_bounds__(1024) void slot_kernel(const int32_t* __restrict__ cu, const int32_t* __restrict__ expiry,
                                                    int32_t* parent, int32_t* slotid, int T, int k) {
  const int d = blockIdx.x, h = blockIdx.y;
  const int a = cu[d], b = cu[d + 1], n = b - a;
  if (n <= 0) return;
  const size_t hb = (size_t)h * T + a;
  int32_t* par = parent + hb;
  int32_t* sid = slotid + hb;
  const int32_t* ex = expiry + hb;
  const int tid = threadIdx.x;
  const int rounds = dev_ceil_log2(n);
  constexpr int LDS_N = 65536;  // local indices fit 16 bits up to this length
  __shared__ uint16_t ls[LDS_N];
  if (n > k && n <= LDS_N) {
    // the chain links live in LDS from the start: only parent[] and the final slot ids touch memory
    for (int j = tid; j < n; j += 1024) {
      par[j] = -1;
      ls[j] = (uint16_t)j;
    }
    __syncthreads();
    for (int j = tid; j < n; j += 1024) {
      const int e = ex[j] - a;
      if (e > j && e < n) {  // key j is evicted at row e by key e
        par[e] = a + j;
        ls[e] = (uint16_t)j;
      }
    }
    __syncthreads();
    for (int r = 0; r < rounds; r++) {  // pointer jumping towards the chain root (< k)
      // (a thread may read an entry another thread has already advanced this round: still an
      // ancestor on the same chain, so the jumping only converges faster)
      int moved = 0;
      for (int j = tid; j < n; j += 1024) {
        const int q = ls[j];
        if (q >= k && q != j) {  // (q == j: a key that never enters; nothing points at it)
          ls[j] = ls[q];
          moved = 1;
        }
      }
      if (!__syncthreads_or(moved)) break;  // every entry is a root: chains are short (about n / k links)
    }
    for (int j = tid; j < n; j += 1024) sid[j] = ls[j];
    return;
  }
  for (int j = tid; j < n; j += 1024) {
    par[j] = -1;
    sid[j] = j;
  }
  __syncthreads();
  if (n <= k) return;
  for (int j = tid; j < n; j += 1024) {
    const int e = ex[j] - a;
    if (e > j && e < n) {  // key j is evicted at row e by key e
      par[e] = a + j;
      sid[e] = j;
    }
  }
  __syncthreads();
  for (int r = 0; r < rounds; r++) {
    int moved = 0;
    for (int j = tid; j < n; j += 1024) {
      const int q = sid[j];
      if (q >= k && q != j) {
        sid[j] = sid[q];
        moved = 1;
      }
    }
    if (!__syncthreads_or(moved)) break;
  }
}

// One thread per (head, key): write the key into the slot table of every block it is clean in.
__global__ __launch_bounds__(256) void slot_table_kernel(const int32_t* __restrict__ cu, int n_docs,
                                                         const int32_t* __restrict__ expiry,
                                                         const int32_t* __restrict__ slotid,
                                                         const int32_t* __restrict__ docblk, int32_t* slot_tab,
                                                         int T, int nblk_cap, int kpad) {
  const int t = blockIdx.x * 256 + threadIdx.x, h = blockIdx.y;
  if (t >= T) return;
  const int d = find_doc(cu, n_docs, t);
  const int a = cu[d], n = cu[d + 1] - a;
  const int j = t - a;
  const int e = expiry[(size_t)h * T + t] - a;
  if (e <= j) return;
  const int slot = slotid[(size_t)h * T + t];
  const int blk0 = docblk[d];
  for (int bl = j / BQ + 1;; bl++) {
    const int i_lo = bl * BQ;
    if (i_lo >= n) break;
    const int i_hi = min(i_lo + BQ, n) - 1;
    if (e <= i_hi) break;
    slot_tab[((size_t)h * nblk_cap + blk0 + bl) * kpad + slot] = t;
  }
}

// The same table, row by row, in tiles of SLOT_TILE columns.  One workgroup per (chunk of
// consecutive blocks, head, column tile) keeps in LDS, per slot, the latest key of the slot's chain among the keys
// before the current block, with its expiry; a block's row is then one coalesced pass (the key if
// it outlives the block, else -1; nothing is left for a fill launch), after which the block's own
// keys are taken in.  The state at the chunk's first block comes from one scan of the document's
// earlier keys (exactly one key per chain is still kept at a given row; every column tile repeats
// the scan, so this kernel serves windows of up to SLOT_TILES_MAX tiles).  The scattered 4-byte
// stores of the kernel above cost a 64-byte write each; these rows are written whole.
constexpr int SLOT_TILE = 4096;
constexpr int SLOT_TILES_MAX = 4;
__global__ __launch_bounds__(512) void slot_rows_kernel(const int4* __restrict__ blk, const int32_t* __restrict__ expiry,
                                                        const int32_t* __restrict__ slotid, int32_t* slot_tab, int T,
                                                        int nblk_cap, int kpad, int blocks_per_chunk) {
  __shared__ unsigned long long cur[SLOT_TILE];  // (key + 1) << 32 | expiry; 0 = no key yet
  const int h = blockIdx.y, tid = threadIdx.x;
  const int c0 = blockIdx.z * SLOT_TILE, nc = min(SLOT_TILE, kpad - c0);  // this workgroup's columns
  const int b_begin = blockIdx.x * blocks_per_chunk, b_end = min(b_begin + blocks_per_chunk, nblk_cap);
  const int32_t* ex = expiry + (size_t)h * T;
  const int32_t* sid = slotid + (size_t)h * T;
  int doc = -1;
  for (int b = b_begin; b < b_end; b++) {
    const int4 info = blk[b];  // (the same for every thread: the branches below are uniform)
    int32_t* row = slot_tab + ((size_t)h * nblk_cap + b) * kpad + c0;
    if (info.x < 0) {
      for (int c = tid; c < nc; c += 512) row[c] = -1;
      continue;
    }
    const int lo = info.y, hi = info.z - 1, a = info.w;  // causal plan: w = first row of the document
    if (info.x != doc) {
      doc = info.x;
      __syncthreads();
      for (int c = tid; c < nc; c += 512) cur[c] = 0ull;
      __syncthreads();
      for (int j = a + tid; j < lo; j += 512) {
        const int e = ex[j];
        if (e > j && e >= lo) {
          const int c = sid[j] - c0;
          if (c >= 0 && c < nc) cur[c] = ((unsigned long long)(unsigned)(j + 1) << 32) | (unsigned)e;
        }
      }
      __syncthreads();
    }
    for (int c = tid; c < nc; c += 512) {
      const unsigned long long v = cur[c];
      row[c] = (v != 0ull && (int)(unsigned)v > hi) ? (int)(v >> 32) - 1 : -1;
    }
    __syncthreads();
    for (int j = lo + tid; j <= hi; j += 512) {
      const int e = ex[j];
      if (e > j) {
        const int c = sid[j] - c0;
        if (c >= 0 && c < nc) atomicMax(&cur[c], ((unsigned long long)(unsigned)(j + 1) << 32) | (unsigned)e);
      }
    }
    __syncthreads();
  }
}

// One workgroup (BQ threads) per (block, head): keys that enter inside the block (ascending), then
// keys that were resident at the block's first row and are evicted inside it (by ascending evictor).
__global__ __launch_bounds__(BQ) void partial_list_kernel(const int4* __restrict__ blk,
                                                          const int32_t* __restrict__ expiry,
                                                          const int32_t* __restrict__ parent, int32_t* pcnt,
                                                          int32_t* plist, int T, int nblk_cap) {
  const int bi = blockIdx.x, h = blockIdx.y;
  const int4 info = blk[bi];
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63;
  if (info.x < 0) {
    if (tid == 0) pcnt[(size_t)h * nblk_cap + bi] = 0;
    return;
  }
  const int i = info.y + tid;
  const bool ent = (i < info.z) && expiry[(size_t)h * T + i] > i;
  int m = -1;
  if (ent) m = parent[(size_t)h * T + i];
  const bool exq = ent && m >= 0 && m < info.y && i > info.y;  // evicted at the block's first row: not active here
  __shared__ int cnt[2][BQ / 64];
  const unsigned long long em = __ballot(ent), xm = __ballot(exq);
  const unsigned long long lt = (1ull << l) - 1ull;
  if (l == 0) {
    cnt[0][w] = __popcll(em);
    cnt[1][w] = __popcll(xm);
  }
  __syncthreads();
  int ebase = 0, xbase = 0, etot = 0, xtot = 0;
  for (int i2 = 0; i2 < BQ / 64; i2++) {
    if (i2 < w) { ebase += cnt[0][i2]; xbase += cnt[1][i2]; }
    etot += cnt[0][i2];
    xtot += cnt[1][i2];
  }
  int32_t* out = plist + ((size_t)h * nblk_cap + bi) * MAXPART;
  if (ent) out[ebase + __popcll(em & lt)] = i;
  if (exq) out[etot + xbase + __popcll(xm & lt)] = m;
  if (tid == 0) pcnt[(size_t)h * nblk_cap + bi] = etot + xtot;
}

// Without the causal restriction every row of a document keeps the same min(k, n) best keys.  One
// thread per (head, rank position r of the sorted order): the key at rank r < k is kept (expiry =
// end of the document) and fills slot column r of every block of the document; the others are
// never kept (expiry = own index).  Documents of at most k keys were not sorted: key j is rank j.
__global__ __launch_bounds__(256) void noncausal_plan_kernel(const int32_t* __restrict__ cu, int n_docs,
                                                             const uint32_t* __restrict__ si0,
                                                             const int32_t* __restrict__ docblk, int32_t* expiry,
                                                             int32_t* slot_tab, int T, int k, int nblk_cap, int kpad) {
  const int t = blockIdx.x * 256 + threadIdx.x, h = blockIdx.y;
  if (t >= T) return;
  const int d = find_doc(cu, n_docs, t);
  const int a = cu[d], b = cu[d + 1], n = b - a;
  const int r = t - a;
  const int j = n <= k ? r : (int)si0[(size_t)h * T + t];
  const bool kept = r < k;
  expiry[(size_t)h * T + a + j] = kept ? b : a + j;
  if (!kept) return;
  for (int bl = docblk[d]; bl < docblk[d + 1]; bl++) slot_tab[((size_t)h * nblk_cap + bl) * kpad + r] = a + j;
}

// Debug output: kept keys of every row, ascending, -1 padded.  One wave per (row, head).
__global__ __launch_bounds__(64) void topk_idx_kernel(const int32_t* __restrict__ cu, int n_docs, int causal,
                                                      const int32_t* __restrict__ expiry, int32_t* out, int T, int k) {
  const int t = blockIdx.x, h = blockIdx.y, l = threadIdx.x;
  const int d = find_doc(cu, n_docs, t);
  const int a = cu[d];
  int32_t* o = out + ((size_t)h * T + t) * k;
  const unsigned long long lt = (1ull << l) - 1ull;
  int count = 0;
  const int jl = causal ? t : cu[d + 1] - 1;
  for (int j0 = a; j0 <= jl; j0 += 64) {
    const int j = j0 + l;
    const bool keep = (j <= jl) && expiry[(size_t)h * T + j] > (causal ? t : j);
    const unsigned long long m = __ballot(keep);
    const int pos = count + __popcll(m & lt);
    if (keep && pos < k) o[pos] = j;
    count += __popcll(m);
  }
  for (int q = count + l; q < k; q += 64) o[q] = -1;
}

// ------------------------------------------------------------------ host side
// A caller-supplied attention bias, one value per key (broadcast over the query rows), is added to
// the start values of the score accumulators only: zq += bias / scale.  The selection keeps ranking z.
// bias is [bias_heads, T] (per_token) or [bias_heads, n_max] indexed by the key's position in its
// document (shared by all documents); bias_heads = H_q or 1.
__global__ __launch_bounds__(256) void bias_add_kernel(const float* __restrict__ bias, const int32_t* __restrict__ cu,
                                                       int n_docs, int bias_heads, int per_token, int n_max,
                                                       float* __restrict__ zq, float inv_scale, int T) {
  const int t = blockIdx.x * 256 + threadIdx.x, h = blockIdx.y;
  if (t >= T) return;
  const size_t row = bias_heads == 1 ? 0 : (size_t)h;
  float b;
  if (per_token) b = bias[row * T + t];
  else b = bias[row * n_max + (t - cu[find_doc(cu, n_docs, t)])];
  zq[(size_t)h * T + t] += b * inv_scale;
}

// Gradient of that bias from dz (the bias enters the score exactly like z): summed over the heads and
// the documents that share an entry.  One thread per output element, no atomics.
__global__ __launch_bounds__(256) void bias_bwd_kernel(const float* __restrict__ dz, const int32_t* __restrict__ cu,
                                                       int n_docs, int bias_heads, int per_token, int n_max, int H_q,
                                                       int T, float* __restrict__ dbias) {
  const int n_out = per_token ? T : n_max;
  const int x = blockIdx.x * 256 + threadIdx.x, bh = blockIdx.y;
  if (x >= n_out) return;
  const int h0 = bias_heads == 1 ? 0 : bh, h1 = bias_heads == 1 ? H_q : bh + 1;
  float acc = 0.f;
  if (per_token) {
    for (int h = h0; h < h1; h++) acc += dz[(size_t)h * T + x];
  } else {
    for (int d = 0; d < n_docs; d++) {
      const int a = cu[d], b = cu[d + 1];
      if (x < b - a)
        for (int h = h0; h < h1; h++) acc += dz[(size_t)h * T + a + x];
    }
  }
  dbias[(size_t)bh * n_out + x] = acc;
}

int launch_bias_add(const Ptrs& p, const float* bias, int bias_heads, int per_token, const int32_t* cu, hipStream_t st) {
  const dma_shape& s = p.s;
  float* zq = (float*)(p.plan + p.pl.off_zq);
  bias_add_kernel<<<dim3((s.T + 255) / 256, s.H_q), 256, 0, st>>>(bias, cu, s.n_docs, bias_heads, per_token, s.max_seqlen,
                                                                 zq, 1.0f / p.scale, s.T);
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

int launch_bias_bwd(const dma_shape& s, const float* dz, int bias_heads, int per_token, const int32_t* cu, float* dbias,
                    hipStream_t st) {
  const int n_out = per_token ? s.T : s.max_seqlen;
  bias_bwd_kernel<<<dim3((n_out + 255) / 256, bias_heads), 256, 0, st>>>(dz, cu, s.n_docs, bias_heads, per_token,
                                                                        s.max_seqlen, s.H_q, s.T, dbias);
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

int launch_mask_gen(const Ptrs& p, const void* V, const float* W, const float* A, const int32_t* cu,
                    float* z, int32_t* expiry, int32_t* topk_idx, hipStream_t st) {
  const dma_shape& s = p.s;
  const PlanLayout& L = p.pl;
  char* base = p.plan;
  int32_t* hdr = (int32_t*)(base + L.off_hdr);
  int4* blk = (int4*)(base + L.off_blk);
  int32_t* docblk = (int32_t*)(base + L.off_docblk);
  int32_t* slot_tab = (int32_t*)(base + L.off_slot);
  int32_t* pcnt = (int32_t*)(base + L.off_pcnt);
  int32_t* plist = (int32_t*)(base + L.off_plist);
  int32_t* parent = (int32_t*)(base + L.off_parent);
  int32_t* slotid = (int32_t*)(base + L.off_slotid);

  prof_begin(DMA_STAGE_Z, st);
  blkinfo_kernel<<<1, 256, 0, st>>>(cu, s.n_docs, L.nblk_cap, s.k, s.causal, blk, docblk, hdr,
                                   (uint32_t*)(base + L.off_consts), p.scale);
  float* zq = (float*)(base + L.off_zq);
  const float inv_scale = 1.0f / p.scale;
  if (W) {
    const int G = s.H_q / s.H_kv;
    dim3 grid((s.T + 63) / 64, s.H_kv);
    const size_t sh = (size_t)G * 64 * sizeof(float);
#define DMA_Z(TV, DD, GM) \
  z_kernel<TV, DD, GM><<<grid, 256, sh, st>>>((const TV*)V, W, A, z, zq, inv_scale, s.T, s.H_q, s.H_kv)
    if (s.dtype == DMA_BF16) {
      if (s.d == 256) { if (G <= 4) DMA_Z(uint16_t, 256, 4); else DMA_Z(uint16_t, 256, 8); }
      else if (s.d == 128) { if (G <= 4) DMA_Z(uint16_t, 128, 4); else DMA_Z(uint16_t, 128, 8); }
      else { if (G <= 4) DMA_Z(uint16_t, 64, 4); else DMA_Z(uint16_t, 64, 8); }
    } else {
      if (s.d == 256) { if (G <= 4) DMA_Z(float, 256, 4); else DMA_Z(float, 256, 8); }
      else if (s.d == 128) { if (G <= 4) DMA_Z(float, 128, 4); else DMA_Z(float, 128, 8); }
      else { if (G <= 4) DMA_Z(float, 64, 4); else DMA_Z(float, 64, 8); }
    }
#undef DMA_Z
  }
  if (!W) {  // caller-supplied scores: only z / softmax_scale is left to do
    const size_t n = (size_t)s.H_q * s.T;
    size_t grid = (n + 1023) / 1024;
    if (grid > (1u << 20)) grid = 1u << 20;
    zq_kernel<<<(unsigned)grid, 256, 0, st>>>(z, zq, inv_scale, n);
  }
  prof_end(DMA_STAGE_Z, st);
  SortArgs sa;
  sa.z = z; sa.cu = cu; sa.expiry = expiry;
  sa.sk0 = (uint32_t*)(base + L.off_sk0); sa.sk1 = (uint32_t*)(base + L.off_sk1);
  sa.si0 = (uint32_t*)(base + L.off_si0); sa.si1 = (uint32_t*)(base + L.off_si1);
  sa.wbits = (unsigned long long*)(base + L.off_wbits);
  sa.wcnt = (uint32_t*)(base + L.off_wcnt);
  sa.wzero = (uint32_t*)(base + L.off_wzero);
  sa.T = s.T; sa.n_docs = s.n_docs; sa.k = s.k; sa.nbits_cap = L.nbits_cap; sa.wcap = L.wcap;
  sa.nseg_cap = L.nseg_cap; sa.seg = L.seg;
  prof_begin(DMA_STAGE_SORT, st);
  if (L.seg == SEG_MIN) sort_wavelet_kernel<SEG_MIN / 1024><<<dim3(L.nseg_cap, s.H_q), 1024, 0, st>>>(sa);
  else sort_wavelet_kernel<SEG_MAX / 1024><<<dim3(L.nseg_cap, s.H_q), 1024, 0, st>>>(sa);
  prof_end(DMA_STAGE_SORT, st);
  const auto fill = [&](int32_t* dst, size_t n, int32_t v) {
    size_t grid = (n + 2047) / 2048;
    if (grid > (1u << 20)) grid = 1u << 20;
    if (grid < 1) grid = 1;
    fill_i32_kernel<<<(unsigned)grid, 256, 0, st>>>(dst, n, v);
  };
  if (!s.causal) {
    prof_begin(DMA_STAGE_EXPIRY, st);
    prof_end(DMA_STAGE_EXPIRY, st);
    prof_begin(DMA_STAGE_PLAN, st);
    fill(slot_tab, (size_t)s.H_q * L.nblk_cap * L.kpad, -1);
    fill(pcnt, (size_t)s.H_q * L.nblk_cap, 0);
    // (documents of several segments get their whole-document rank order from the merge kernel)
    if (s.T > L.seg) merge_expiry_kernel<true><<<dim3((s.T + 255) / 256, s.H_q), 256, 0, st>>>(sa);
    noncausal_plan_kernel<<<dim3((s.T + 255) / 256, s.H_q), 256, 0, st>>>(cu, s.n_docs, sa.si0, docblk, expiry, slot_tab,
                                                                        s.T, s.k, L.nblk_cap, L.kpad);
  } else {
    prof_begin(DMA_STAGE_EXPIRY, st);
    // (documents of one segment / of several segments; a single document is one or the other)
    if (s.n_docs > 1 || s.T <= L.seg) expiry_kernel<<<dim3((s.T + 255) / 256, s.H_q), 256, 0, st>>>(sa);
    if (s.T > L.seg) merge_expiry_kernel<false><<<dim3((s.T + 255) / 256, s.H_q), 256, 0, st>>>(sa);
    prof_end(DMA_STAGE_EXPIRY, st);
    prof_begin(DMA_STAGE_PLAN, st);
    slot_kernel<<<dim3(s.n_docs, s.H_q), 1024, 0, st>>>(cu, expiry, parent, slotid, s.T, s.k);
    if (L.kpad <= SLOT_TILES_MAX * SLOT_TILE) {
      const int per = L.nblk_cap / 16 > 4 ? L.nblk_cap / 16 : 4;  // about 16 chunks per head
      slot_rows_kernel<<<dim3((L.nblk_cap + per - 1) / per, s.H_q, (L.kpad + SLOT_TILE - 1) / SLOT_TILE), 512, 0, st>>>(blk, expiry, slotid, slot_tab, s.T,
                                                                               L.nblk_cap, L.kpad, per);
    } else {
      fill(slot_tab, (size_t)s.H_q * L.nblk_cap * L.kpad, -1);
      slot_table_kernel<<<dim3((s.T + 255) / 256, s.H_q), 256, 0, st>>>(cu, s.n_docs, expiry, slotid, docblk, slot_tab,
                                                                      s.T, L.nblk_cap, L.kpad);
    }
    partial_list_kernel<<<dim3(L.nblk_cap, s.H_q), BQ, 0, st>>>(blk, expiry, parent, pcnt, plist, s.T, L.nblk_cap);
  }
  if (topk_idx) topk_idx_kernel<<<dim3(s.T, s.H_q), 64, 0, st>>>(cu, s.n_docs, s.causal, expiry, topk_idx, s.T, s.k);
  prof_end(DMA_STAGE_PLAN, st);
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

}  // namespace dma
