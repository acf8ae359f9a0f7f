// Forward pass (Eq. 5-6; online softmax of Alg. 1, query-stationary so O, l, m stay in registers).
//
// One workgroup = one block of BQ query rows of one head; wave w owns rows 32w .. 32w+31.  The
// keys a block needs are gathered, KT at a time, into LDS: first the slot table row of the block
// (residents active for every row of the block: no mask needed, empty slots carry z = -inf), then
// the block's partial list (keys entering or expiring inside the block: masked per element with
// j <= i < e_j).
//
// Per tile the wave computes S^T = K Q^T (keys x queries) so that each lane holds one query column:
// the softmax statistics are per lane, and the exponentiated block is already laid out as the B
// operand of O^T += V^T P^T.  V^T fragments come from the row-major LDS tile through transposing
// LDS reads.
#include "common.h"

namespace dma {

struct FwdArgs {
  const uint16_t *Q, *K, *V;
  uint16_t* O;
  const float* z;
  float* LSE;
  const int32_t* expiry;
  const int4* blk;
  const int32_t* slot_tab;
  const int32_t* pcnt;
  const int32_t* plist;
  int T, H_q, H_kv, k, nblk_cap, kpad;
  float c2;  // softmax scale * log2(e)
};

template <int D>
__global__ __launch_bounds__(256, 2) void fwd_kernel(FwdArgs p) {
  using TL = TileLayout<D>;
  constexpr int LDK = TL::LD;     // LDS row stride in elements
  constexpr int KS = D / 16;      // contraction steps of K Q^T
  constexpr int CB = D / 32;      // 32-channel blocks of O^T
  constexpr int CPR = D / 8;      // 16-byte chunks per row
  constexpr int NCH = KT * CPR / 256;  // chunks per thread per tile
  __shared__ __align__(16) uint16_t smem[2 * KT * LDK];
  __shared__ __align__(16) float zs[KT];
  __shared__ __align__(16) int js[KT];
  __shared__ __align__(16) int es[KT];
  uint16_t* Ks = smem;
  uint16_t* Vs = smem + KT * LDK;

  int h, item;
  if (!xcd_map(blockIdx.x, p.H_q, p.nblk_cap, h, item)) return;
  const int bi = p.nblk_cap - 1 - item;  // long blocks first
  const int4 info = p.blk[bi];
  if (info.x < 0) return;
  const int row0 = info.y, row1 = info.z, doc0 = info.w;
  const int g = h / (p.H_q / p.H_kv);
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, n = l & 31, hh = l >> 5;
  const int ncol = min(p.k, row0 - doc0);
  const int nc = (ncol + KT - 1) / KT;
  const int np_keys = p.pcnt[(size_t)h * p.nblk_cap + bi];
  const int nt = nc + (np_keys + KT - 1) / KT;
  const int32_t* slot_row = p.slot_tab + ((size_t)h * p.nblk_cap + bi) * p.kpad;
  const int32_t* plist_row = p.plist + ((size_t)h * p.nblk_cap + bi) * MAXPART;
  const float* zh = p.z + (size_t)h * p.T;
  const int32_t* eh = p.expiry + (size_t)h * p.T;

  // query fragments (B operand of K Q^T): lane holds row qi, channels 16*ks + 8*hh .. +8
  const int qi = row0 + 32 * w + n;
  bf16x8 qreg[KS];
  {
    const uint16_t* qrow = p.Q + ((size_t)qi * p.H_q + h) * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (qi < row1) raw = *reinterpret_cast<const uint4*>(qrow + 16 * ks);
      qreg[ks] = __builtin_bit_cast(bf16x8, raw);
    }
  }

  f32x16 oacc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; cb++)
#pragma unroll
    for (int v = 0; v < 16; v++) oacc[cb][v] = 0.f;
  float m_run = -INFINITY, lsum = 0.f;

  uint4 kst[NCH], vst[NCH];
  float z_st = 0.f;
  int j_st = 0, e_st = 0;
  int idn[NCH], idz = -1;  // key ids of the tile about to be loaded (rows of this thread's chunks; row tid)
  auto tile_id = [&](int t, int r) -> int {
    if (t >= nt) return -1;
    if (t < nc) return slot_row[t * KT + r];
    const int q = (t - nc) * KT + r;
    return q < np_keys ? plist_row[q] : -1;
  };
  auto load_ids = [&](int t) {
#pragma unroll
    for (int it = 0; it < NCH; it++) idn[it] = tile_id(t, (tid + 256 * it) / CPR);
    if (tid < KT) idz = tile_id(t, tid);
  };
  auto load_tile = [&]() {  // gathers the tile whose ids are in idn / idz
#pragma unroll
    for (int it = 0; it < NCH; it++) {
      const int col = (tid + 256 * it) % CPR;
      const int id = idn[it];
      kst[it] = make_uint4(0, 0, 0, 0);
      vst[it] = make_uint4(0, 0, 0, 0);
      if (id >= 0) {
        const size_t off = ((size_t)id * p.H_kv + g) * D + 8 * col;
        kst[it] = *reinterpret_cast<const uint4*>(p.K + off);
        vst[it] = *reinterpret_cast<const uint4*>(p.V + off);
      }
    }
    if (tid < KT) {
      const int id = idz;
      z_st = id >= 0 ? zh[id] * LOG2E : -INFINITY;
      j_st = id >= 0 ? id : 0x7fffffff;
      e_st = id >= 0 ? eh[id] : 0;
    }
  };

  load_ids(0);
  load_tile();
  load_ids(1);
  for (int t = 0; t < nt; t++) {
    __syncthreads();
#pragma unroll
    for (int it = 0; it < NCH; it++) {
      const int c = tid + 256 * it, r = c / CPR, col = c % CPR;
      *reinterpret_cast<uint4*>(&Ks[TL::off(r, col)]) = kst[it];
      *reinterpret_cast<uint4*>(&Vs[TL::off(r, col)]) = vst[it];
    }
    if (tid < KT) {
      zs[tid] = z_st;
      js[tid] = j_st;
      es[tid] = e_st;
    }
    __syncthreads();
    if (t + 1 < nt) {
      load_tile();
      load_ids(t + 2);
    }
    const bool masked = t >= nc;

    // S^T = K Q^T for the two 32-key halves of the tile
    f32x16 sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; kb++) {
#pragma unroll
      for (int v = 0; v < 16; v++) sacc[kb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        const bf16x8 a = *reinterpret_cast<const bf16x8*>(&Ks[TL::off(32 * kb + n, 2 * ks + hh)]);
        sacc[kb] = mfma32(a, qreg[ks], sacc[kb]);
      }
    }
    // scores in log2 units, bias, mask, running max
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; kb++) {
#pragma unroll
      for (int gq = 0; gq < 4; gq++) {
        const int r = 32 * kb + 8 * gq + 4 * hh;
        const f32x4 zz = *reinterpret_cast<const f32x4*>(&zs[r]);
#pragma unroll
        for (int u = 0; u < 4; u++) sacc[kb][4 * gq + u] = fmaf(sacc[kb][4 * gq + u], p.c2, zz[u]);
        if (masked) {
          const int4 jj = *reinterpret_cast<const int4*>(&js[r]);
          const int4 ee = *reinterpret_cast<const int4*>(&es[r]);
          const int jv[4] = {jj.x, jj.y, jj.z, jj.w}, ev[4] = {ee.x, ee.y, ee.z, ee.w};
#pragma unroll
          for (int u = 0; u < 4; u++)
            if (!(qi >= jv[u] && qi < ev[u])) sacc[kb][4 * gq + u] = -INFINITY;
        }
#pragma unroll
        for (int u = 0; u < 4; u++) mx = fmaxf(mx, sacc[kb][4 * gq + u]);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(m_run, mx);
    const float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    const float alpha = fast_exp2(m_run - m_safe);
    m_run = m_new;
    float psum = 0.f;
    bf16x8 pb[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const float pv = fast_exp2(sacc[kb][v] - m_safe);
        psum += pv;
        pb[kb][v >> 3][v & 7] = (__bf16)pv;
      }
    lsum = lsum * alpha + psum;
    if (!__all(alpha == 1.0f)) {  // the running maximum rarely moves after the first tiles
#pragma unroll
      for (int cb = 0; cb < CB; cb++)
#pragma unroll
        for (int v = 0; v < 16; v++) oacc[cb][v] *= alpha;
    }

    // O^T += V^T P^T
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int c = 0; c < 2; c++)
#pragma unroll
        for (int cb = 0; cb < CB; cb++)
          oacc[cb] = mfma32(tr_frag<D>(Vs, 32 * kb + 16 * c, cb, l), pb[kb][c], oacc[cb]);
  }

  // epilogue: normalise, stage O through LDS for coalesced rows, write LSE
  const float ltot = lsum + __shfl_xor(lsum, 32);
  const float inv = 1.f / ltot;
  if (hh == 0 && qi < row1) p.LSE[(size_t)h * p.T + qi] = (m_run + __builtin_amdgcn_logf(ltot)) * LN2;
  __syncthreads();
  uint16_t* Os = smem;  // [BQ][LDK]
#pragma unroll
  for (int cb = 0; cb < CB; cb++)
#pragma unroll
    for (int gq = 0; gq < 4; gq++) {
      bf16x4 o4;
#pragma unroll
      for (int u = 0; u < 4; u++) o4[u] = (__bf16)(oacc[cb][4 * gq + u] * inv);
      *reinterpret_cast<bf16x4*>(&Os[TL::off(32 * w + n, 4 * cb + gq) + 4 * hh]) = o4;
    }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < BQ * CPR / 256; it++) {
    const int c = tid + 256 * it, r = c / CPR, col = c % CPR;
    if (row0 + r < row1)
      *reinterpret_cast<uint4*>(p.O + ((size_t)(row0 + r) * p.H_q + h) * D + 8 * col) =
          *reinterpret_cast<const uint4*>(&Os[TL::off(r, col)]);
  }
}

int launch_fwd(const Ptrs& p, const void* Q, const void* K, const void* V, const float* z, const int32_t* expiry,
               const int32_t* cu, void* O, float* LSE, hipStream_t st) {
  (void)cu;
  const dma_shape& s = p.s;
  const PlanLayout& L = p.pl;
  FwdArgs a;
  a.Q = (const uint16_t*)Q; a.K = (const uint16_t*)K; a.V = (const uint16_t*)V; a.O = (uint16_t*)O;
  a.z = z; a.LSE = LSE; a.expiry = expiry;
  a.blk = (const int4*)(p.plan + L.off_blk);
  a.slot_tab = (const int32_t*)(p.plan + L.off_slot);
  a.pcnt = (const int32_t*)(p.plan + L.off_pcnt);
  a.plist = (const int32_t*)(p.plan + L.off_plist);
  a.T = s.T; a.H_q = s.H_q; a.H_kv = s.H_kv; a.k = s.k; a.nblk_cap = L.nblk_cap; a.kpad = L.kpad;
  a.c2 = p.scale * LOG2E;
  const unsigned grid = xcd_grid(s.H_q, L.nblk_cap);
  prof_begin(DMA_STAGE_FWD, st);
  if (s.d == 128) fwd_kernel<128><<<grid, 256, 0, st>>>(a);
  else fwd_kernel<64><<<grid, 256, 0, st>>>(a);
  prof_end(DMA_STAGE_FWD, st);
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

}  // namespace dma
