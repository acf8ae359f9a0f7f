// Backward pass (Eq. 7-10; the tile arithmetic of Alg. 2 with D_i = rowsum(dO o O)).
//
// Two kernels share the work so that no accumulator is spread over workgroups at tile granularity:
//
//  * dq_kernel, query-stationary (the forward's structure): per block of BQ rows it recomputes
//    S^T and dP^T on the gathered key tiles, forms dS^T = P^T o (dP^T - D) and accumulates
//    dQ^T += K^T dS^T in registers.  It also produces D for the other kernel.
//
//  * dkv_kernel, key-stationary: a workgroup owns SG slot columns of one head and sweeps query
//    blocks.  A slot column always holds one resident key, so its tiles are dense and need no
//    mask; K and V fragments of the resident stay in registers together with the dK^T, dV^T and dz
//    accumulators.  When the resident of a column changes, the finished key is flushed with a
//    handful of fp32 atomics (dK and dV are shared by the q-heads of a group) and the column is
//    re-armed.  The same kernel, in "partial" mode, handles the keys that enter or expire inside a
//    block: columns come from the block's partial list, elements are masked with j <= i < e_j, and
//    the sweep is that single block.
//
// The dS/P blocks are produced in the accumulator layout of S = Q K^T (dkv) or S^T = K Q^T (dq),
// which is exactly the B-operand layout of the products that consume them; the other operand of
// those products is read from row-major LDS tiles with transposing LDS reads.
#include "common.h"

namespace dma {

struct BwdArgs {
  const uint16_t *Q, *K, *V, *O, *dO;
  uint16_t* dQ;
  const float *z, *LSE;
  float *Dws, *dK32, *dV32, *dz;
  const int32_t* expiry;
  const int4* blk;
  const int32_t* slot_tab;
  const int32_t* pcnt;
  const int32_t* plist;
  int T, H_q, H_kv, k, nblk_cap, kpad;
  int seg;  // query blocks swept by one clean-mode work item of dkv_kernel
  float scale, c2;
};

// ------------------------------------------------------------------ dQ (and D)
template <int D>
__global__ __launch_bounds__(256, 2) void dq_kernel(BwdArgs p) {
  using TL = TileLayout<D>;
  constexpr int LDK = TL::LD, KS = D / 16, CB = D / 32, CPR = D / 8, NCH = KT * CPR / 256;
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

  const int qi = row0 + 32 * w + n;
  const bool qvalid = qi < row1;
  bf16x8 qreg[KS], doreg[KS];
  float Dsum = 0.f;
  {
    const size_t off = ((size_t)qi * p.H_q + h) * D + 8 * hh;
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      uint4 rq = make_uint4(0, 0, 0, 0), rd = rq, ro = rq;
      if (qvalid) {
        rq = *reinterpret_cast<const uint4*>(p.Q + off + 16 * ks);
        rd = *reinterpret_cast<const uint4*>(p.dO + off + 16 * ks);
        ro = *reinterpret_cast<const uint4*>(p.O + off + 16 * ks);
      }
      qreg[ks] = __builtin_bit_cast(bf16x8, rq);
      doreg[ks] = __builtin_bit_cast(bf16x8, rd);
      const bf16x8 ov = __builtin_bit_cast(bf16x8, ro);
#pragma unroll
      for (int e = 0; e < 8; e++) Dsum = fmaf((float)doreg[ks][e], (float)ov[e], Dsum);
    }
  }
  Dsum += __shfl_xor(Dsum, 32);
  const float lse2 = qvalid ? p.LSE[(size_t)h * p.T + qi] * LOG2E : INFINITY;
  if (qvalid && hh == 0) p.Dws[(size_t)h * p.T + qi] = Dsum;

  f32x16 dqacc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; cb++)
#pragma unroll
    for (int v = 0; v < 16; v++) dqacc[cb][v] = 0.f;

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

#pragma unroll 1
    for (int kb = 0; kb < 2; kb++) {
      bf16x8 dsb[2];
      {
        f32x16 sacc, dpacc;
#pragma unroll
        for (int v = 0; v < 16; v++) { sacc[v] = 0.f; dpacc[v] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
          const bf16x8 ak = *reinterpret_cast<const bf16x8*>(&Ks[TL::off(32 * kb + n, 2 * ks + hh)]);
          const bf16x8 av = *reinterpret_cast<const bf16x8*>(&Vs[TL::off(32 * kb + n, 2 * ks + hh)]);
          sacc = mfma32(ak, qreg[ks], sacc);
          dpacc = mfma32(av, doreg[ks], dpacc);
        }
#pragma unroll
        for (int gq = 0; gq < 4; gq++) {
          const int r = 32 * kb + 8 * gq + 4 * hh;
          const f32x4 zz = *reinterpret_cast<const f32x4*>(&zs[r]);
          int jv[4] = {0, 0, 0, 0}, ev[4] = {0, 0, 0, 0};
          if (masked) {
            const int4 jj = *reinterpret_cast<const int4*>(&js[r]);
            const int4 ee = *reinterpret_cast<const int4*>(&es[r]);
            jv[0] = jj.x; jv[1] = jj.y; jv[2] = jj.z; jv[3] = jj.w;
            ev[0] = ee.x; ev[1] = ee.y; ev[2] = ee.z; ev[3] = ee.w;
          }
#pragma unroll
          for (int u = 0; u < 4; u++) {
            const int v = 4 * gq + u;
            float pv = fast_exp2(fmaf(sacc[v], p.c2, zz[u]) - lse2);
            if (masked && !(qi >= jv[u] && qi < ev[u])) pv = 0.f;
            const float ds = pv * (dpacc[v] - Dsum);
            dsb[v >> 3][v & 7] = (__bf16)ds;
          }
        }
      }
      // dQ^T += K^T dS^T for this half of the tile
#pragma unroll
      for (int c = 0; c < 2; c++) {
#pragma unroll
        for (int cb = 0; cb < CB; cb++)
          dqacc[cb] = mfma32(tr_frag<D>(Ks, 32 * kb + 16 * c, cb, l), dsb[c], dqacc[cb]);
      }
    }
  }

  __syncthreads();
  uint16_t* Os = smem;  // [BQ][LDK]
#pragma unroll
  for (int cb = 0; cb < CB; cb++)
#pragma unroll
    for (int gq = 0; gq < 4; gq++) {
      bf16x4 o4;
#pragma unroll
      for (int u = 0; u < 4; u++) o4[u] = (__bf16)(dqacc[cb][4 * gq + u] * p.scale);
      *reinterpret_cast<bf16x4*>(&Os[TL::off(32 * w + n, 4 * cb + gq) + 4 * hh]) = o4;
    }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < BQ * CPR / 256; it++) {
    const int c = tid + 256 * it, r = c / CPR, col = c % CPR;
    if (row0 + r < row1)
      *reinterpret_cast<uint4*>(p.dQ + ((size_t)(row0 + r) * p.H_q + h) * D + 8 * col) =
          *reinterpret_cast<const uint4*>(&Os[TL::off(r, col)]);
  }
}

// ------------------------------------------------------------------ dK, dV, dz
// Lane (n, hh) of wave w owns column 32w + n of the workgroup's SG columns; its accumulators hold
// channels 32cb + 8gq + 4hh + u of dK^T / dV^T for that column's key.
template <int D, bool PARTIAL>
__global__ __launch_bounds__(256) void dkv_kernel(BwdArgs p) {
  using TL = TileLayout<D>;
  constexpr int LDQ = TL::LD, KS = D / 16, CB = D / 32, CPR = D / 8, NCH = BQ * CPR / 256;
  __shared__ __align__(16) uint16_t Qs[BQ * LDQ];
  __shared__ __align__(16) uint16_t dOs[BQ * LDQ];
  __shared__ __align__(16) float lses[BQ];
  __shared__ __align__(16) float Dss[BQ];
  constexpr int LDS_ST = D + 4;
  __shared__ __align__(16) float stage_all[4 * 32 * LDS_ST];  // per wave: [32 columns][D] fp32, flush staging

  // item = chunk * ngrp + group: the groups of one (head, chunk) run side by side and share Q / dO
  const int ngrp = PARTIAL ? MAXPART / SG : p.kpad / SG;
  const int nchunk = PARTIAL ? p.nblk_cap : (p.nblk_cap + p.seg - 1) / p.seg;
  int h, item;
  if (!xcd_map(blockIdx.x, p.H_q, ngrp * nchunk, h, item)) return;
  const int chunk = item / ngrp, grp = item - chunk * ngrp;
  const int g = h / (p.H_q / p.H_kv);
  const int tid = threadIdx.x, w = tid >> 6, l = tid & 63, n = l & 31, hh = l >> 5;
  const int col = grp * SG + 32 * w + n;
  const float* zh = p.z + (size_t)h * p.T;

  int bi_begin, bi_end;
  if (PARTIAL) {
    bi_begin = chunk;
    bi_end = bi_begin + 1;
  } else {
    bi_begin = chunk * p.seg;
    bi_end = min(bi_begin + p.seg, p.nblk_cap);
  }

  int curid = -1, kj = 0x7fffffff, ke = 0;
  float z2 = -INFINITY;
  bf16x8 kreg[KS], vreg[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    kreg[ks] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
    vreg[ks] = kreg[ks];
  }
  f32x16 dkacc[CB], dvacc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; cb++)
#pragma unroll
    for (int v = 0; v < 16; v++) { dkacc[cb][v] = 0.f; dvacc[cb][v] = 0.f; }
  float dzacc = 0.f;

  float* stage = stage_all + w * 32 * LDS_ST;
  // Flush the columns whose lanes pass doit = true (wave-uniform call).  The accumulators are
  // transposed through the wave's LDS staging area so that each atomic instruction adds 64
  // consecutive channels of one key.
  auto flush = [&](bool doit) {
    const float dzt = dzacc + __shfl_xor(dzacc, 32);
    doit = doit && curid >= 0;
    const unsigned fm = (unsigned)(__ballot(doit) & 0xffffffffull);
    if (fm == 0) return;
    if (doit && hh == 0) atomicAdd(p.dz + (size_t)h * p.T + curid, dzt);
#pragma unroll
    for (int which = 0; which < 2; which++) {
      if (doit) {
#pragma unroll
        for (int cb = 0; cb < CB; cb++)
#pragma unroll
          for (int gq = 0; gq < 4; gq++) {
            f32x4 v4;
#pragma unroll
            for (int u = 0; u < 4; u++)
              v4[u] = which == 0 ? dkacc[cb][4 * gq + u] * p.scale : dvacc[cb][4 * gq + u];
            *reinterpret_cast<f32x4*>(&stage[n * LDS_ST + 32 * cb + 8 * gq + 4 * hh]) = v4;
          }
      }
      float* dst = which == 0 ? p.dK32 : p.dV32;
      unsigned m = fm;
      while (m) {
        const int c = __ffs(m) - 1;
        m &= m - 1;
        const int id = __shfl(curid, c);
        float* row = dst + ((size_t)id * p.H_kv + g) * D;
#pragma unroll
        for (int u = 0; u < D / 64; u++) atomicAdd(row + l + 64 * u, stage[c * LDS_ST + l + 64 * u]);
      }
    }
  };

  for (int bi = bi_begin; bi < bi_end; bi++) {
    const int4 info = p.blk[bi];
    if (info.x < 0) break;
    const int row0 = info.y, row1 = info.z;
    int newid = -1;
    if (PARTIAL) {
      const int np_keys = p.pcnt[(size_t)h * p.nblk_cap + bi];
      if (grp * SG >= np_keys) return;
      if (col < np_keys) newid = p.plist[((size_t)h * p.nblk_cap + bi) * MAXPART + col];
    } else {
      const int ncol = min(p.k, row0 - info.w);
      if (col < ncol) newid = p.slot_tab[((size_t)h * p.nblk_cap + bi) * p.kpad + col];
    }
    const bool changed = newid != curid;
    if (__any(changed)) {
      flush(changed);  // finished keys out, then re-arm the changed columns
      if (changed) {
#pragma unroll
        for (int cb = 0; cb < CB; cb++)
#pragma unroll
          for (int v = 0; v < 16; v++) { dkacc[cb][v] = 0.f; dvacc[cb][v] = 0.f; }
        dzacc = 0.f;
        curid = newid;
        if (newid >= 0) {
          const size_t off = ((size_t)newid * p.H_kv + g) * D + 8 * hh;
#pragma unroll
          for (int ks = 0; ks < KS; ks++) {
            kreg[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p.K + off + 16 * ks));
            vreg[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(p.V + off + 16 * ks));
          }
          z2 = zh[newid] * LOG2E;
          if (PARTIAL) {
            kj = newid;
            ke = p.expiry[(size_t)h * p.T + newid];
          }
        } else {
#pragma unroll
          for (int ks = 0; ks < KS; ks++) {
            kreg[ks] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
            vreg[ks] = kreg[ks];
          }
          z2 = -INFINITY;
          kj = 0x7fffffff;
          ke = 0;
        }
      }
    }
    if (!PARTIAL) {
      // nothing resident in this group's columns for this block: skip the tile (workgroup-uniform)
      if (min(p.k, row0 - info.w) <= grp * SG) continue;
    }

    __syncthreads();  // previous block's LDS reads are done
#pragma unroll
    for (int it = 0; it < NCH; it++) {
      const int c = tid + 256 * it, r = c / CPR, cc = c % CPR;
      uint4 rq = make_uint4(0, 0, 0, 0), rd = rq;
      if (row0 + r < row1) {
        const size_t off = ((size_t)(row0 + r) * p.H_q + h) * D + 8 * cc;
        rq = *reinterpret_cast<const uint4*>(p.Q + off);
        rd = *reinterpret_cast<const uint4*>(p.dO + off);
      }
      *reinterpret_cast<uint4*>(&Qs[TL::off(r, cc)]) = rq;
      *reinterpret_cast<uint4*>(&dOs[TL::off(r, cc)]) = rd;
    }
    if (tid < BQ) {
      const bool rv = row0 + tid < row1;
      lses[tid] = rv ? p.LSE[(size_t)h * p.T + row0 + tid] * LOG2E : INFINITY;
      Dss[tid] = rv ? p.Dws[(size_t)h * p.T + row0 + tid] : 0.f;
    }
    __syncthreads();

#pragma unroll 1
    for (int qs = 0; qs < BQ / 32; qs++) {
      f32x16 sacc, dpacc;
#pragma unroll
      for (int v = 0; v < 16; v++) { sacc[v] = 0.f; dpacc[v] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < KS; ks++) {
        const bf16x8 aq = *reinterpret_cast<const bf16x8*>(&Qs[TL::off(32 * qs + n, 2 * ks + hh)]);
        const bf16x8 ad = *reinterpret_cast<const bf16x8*>(&dOs[TL::off(32 * qs + n, 2 * ks + hh)]);
        sacc = mfma32(aq, kreg[ks], sacc);
        dpacc = mfma32(ad, vreg[ks], dpacc);
      }
      bf16x8 pb[2], dsb[2];
#pragma unroll
      for (int gq = 0; gq < 4; gq++) {
        const int r = 32 * qs + 8 * gq + 4 * hh;
        const f32x4 ls = *reinterpret_cast<const f32x4*>(&lses[r]);
        const f32x4 dd = *reinterpret_cast<const f32x4*>(&Dss[r]);
#pragma unroll
        for (int u = 0; u < 4; u++) {
          const int v = 4 * gq + u;
          float pv = fast_exp2(fmaf(sacc[v], p.c2, z2) - ls[u]);
          if (PARTIAL) {
            const int row = row0 + r + u;
            if (!(row >= kj && row < ke)) pv = 0.f;
          }
          const float ds = pv * (dpacc[v] - dd[u]);
          dzacc += ds;
          pb[v >> 3][v & 7] = (__bf16)pv;
          dsb[v >> 3][v & 7] = (__bf16)ds;
        }
      }
      // dV^T += dO^T P ; dK^T += Q^T dS   (contraction over the 32 query rows of this sub-block)
#pragma unroll
      for (int c = 0; c < 2; c++) {
#pragma unroll
        for (int cb = 0; cb < CB; cb++) {
          dvacc[cb] = mfma32(tr_frag<D>(dOs, 32 * qs + 16 * c, cb, l), pb[c], dvacc[cb]);
          dkacc[cb] = mfma32(tr_frag<D>(Qs, 32 * qs + 16 * c, cb, l), dsb[c], dkacc[cb]);
        }
      }
    }
  }
  flush(true);
}

__global__ void fill_f32_kernel(float* p, size_t n, float v) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t st = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += st) p[i] = v;
}

// dK, dV: fp32 accumulators -> bf16 outputs
__global__ void cvt_bf16_kernel(const float* __restrict__ a, const float* __restrict__ b, uint16_t* __restrict__ oa,
                                uint16_t* __restrict__ ob, size_t n4) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  const size_t st = (size_t)gridDim.x * blockDim.x;
  for (; i < n4; i += st) {
    const float4 x = reinterpret_cast<const float4*>(a)[i];
    const float4 y = reinterpret_cast<const float4*>(b)[i];
    bf16x4 xo, yo;
    xo[0] = (__bf16)x.x; xo[1] = (__bf16)x.y; xo[2] = (__bf16)x.z; xo[3] = (__bf16)x.w;
    yo[0] = (__bf16)y.x; yo[1] = (__bf16)y.y; yo[2] = (__bf16)y.z; yo[3] = (__bf16)y.w;
    reinterpret_cast<bf16x4*>(oa)[i] = xo;
    reinterpret_cast<bf16x4*>(ob)[i] = yo;
  }
}

static unsigned grid_for(size_t n, size_t per_block) {
  size_t g = (n + per_block - 1) / per_block;
  if (g > (1u << 20)) g = 1u << 20;
  return g < 1 ? 1u : (unsigned)g;
}

int launch_bwd(const Ptrs& p, const void* Q, const void* K, const void* V, const void* O, const void* dO,
               const float* LSE, const float* z, const int32_t* expiry, const int32_t* cu, void* dQ, void* dK,
               void* dV, float* dz, char* ws, hipStream_t st) {
  (void)cu;
  const dma_shape& s = p.s;
  const PlanLayout& L = p.pl;
  const WsLayout wl = ws_layout(s);
  BwdArgs a;
  a.Q = (const uint16_t*)Q; a.K = (const uint16_t*)K; a.V = (const uint16_t*)V;
  a.O = (const uint16_t*)O; a.dO = (const uint16_t*)dO; a.dQ = (uint16_t*)dQ;
  a.z = z; a.LSE = LSE; a.expiry = expiry;
  a.Dws = (float*)(ws + wl.off_D); a.dK32 = (float*)(ws + wl.off_dK); a.dV32 = (float*)(ws + wl.off_dV); a.dz = dz;
  a.blk = (const int4*)(p.plan + L.off_blk);
  a.slot_tab = (const int32_t*)(p.plan + L.off_slot);
  a.pcnt = (const int32_t*)(p.plan + L.off_pcnt);
  a.plist = (const int32_t*)(p.plan + L.off_plist);
  a.T = s.T; a.H_q = s.H_q; a.H_kv = s.H_kv; a.k = s.k; a.nblk_cap = L.nblk_cap; a.kpad = L.kpad;
  a.scale = p.scale; a.c2 = p.scale * LOG2E;
  {  // sweep length of a clean-mode work item: as long as possible while keeping >= 512 work items
    const long groups = (long)(L.kpad / SG) * s.H_q;
    long seg = (long)L.nblk_cap * groups / 512;
    if (seg < 4) seg = 4;
    if (seg > L.nblk_cap) seg = L.nblk_cap;
    a.seg = (int)seg;
  }

  const size_t nkv = (size_t)s.T * s.H_kv * s.d;
  prof_begin(DMA_STAGE_BWD_ZERO, st);
  fill_f32_kernel<<<grid_for(2 * nkv, 2048), 256, 0, st>>>(a.dK32, (wl.off_dV - wl.off_dK) / 4 + nkv, 0.f);
  fill_f32_kernel<<<grid_for((size_t)s.H_q * s.T, 2048), 256, 0, st>>>(dz, (size_t)s.H_q * s.T, 0.f);
  prof_end(DMA_STAGE_BWD_ZERO, st);
  const unsigned gq = xcd_grid(s.H_q, L.nblk_cap);
  const unsigned gclean = xcd_grid(s.H_q, (long)((L.nblk_cap + a.seg - 1) / a.seg) * (L.kpad / SG));
  const unsigned gpart = xcd_grid(s.H_q, (long)L.nblk_cap * (MAXPART / SG));
  prof_begin(DMA_STAGE_BWD_DQ, st);
  if (s.d == 128) dq_kernel<128><<<gq, 256, 0, st>>>(a);
  else dq_kernel<64><<<gq, 256, 0, st>>>(a);
  prof_end(DMA_STAGE_BWD_DQ, st);
  prof_begin(DMA_STAGE_BWD_DKV, st);
  if (s.d == 128) dkv_kernel<128, false><<<gclean, 256, 0, st>>>(a);
  else dkv_kernel<64, false><<<gclean, 256, 0, st>>>(a);
  prof_end(DMA_STAGE_BWD_DKV, st);
  prof_begin(DMA_STAGE_BWD_PART, st);
  if (s.d == 128) dkv_kernel<128, true><<<gpart, 256, 0, st>>>(a);
  else dkv_kernel<64, true><<<gpart, 256, 0, st>>>(a);
  prof_end(DMA_STAGE_BWD_PART, st);
  prof_begin(DMA_STAGE_BWD_CVT, st);
  cvt_bf16_kernel<<<grid_for(nkv / 4, 1024), 256, 0, st>>>(a.dK32, a.dV32, (uint16_t*)dK, (uint16_t*)dV, nkv / 4);
  prof_end(DMA_STAGE_BWD_CVT, st);
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

}  // namespace dma
