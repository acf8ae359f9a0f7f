// Backward pass (Eq. 7-10; the tile arithmetic of Alg. 2 with D_i = rowsum(dO o O)).
//
// Two kernels share the work so that no accumulator is spread over workgroups at tile granularity:
//
//  * dq_kernel, query-stationary (the forward's structure and copy ring): per block of BQ rows it
//    recomputes S^T and dP^T on the gathered key tiles, forms dS^T = P^T o (dP^T - D) and
//    accumulates dQ^T += K^T dS^T in registers.  It also produces D and LSE * log2(e) for the
//    other kernel.
//
//  * dkv_kernel, key-stationary: a workgroup owns SG slot columns of one head and sweeps query
//    blocks in steps of 32 rows, fed by a ring of asynchronous Q / dO copies.  A slot column always
//    holds one resident key, so its tiles are dense and need no mask; K and V fragments of the
//    resident stay in registers together with the dK^T, dV^T and dz accumulators.  When the
//    resident of a column changes, the finished key is flushed with a handful of fp32 atomics (dK
//    and dV are shared by the q-heads of a group) and the column is re-armed.  The same kernel, in
//    "partial" mode, handles the keys that enter or expire inside a block: columns come from the
//    blocks' partial lists, elements are masked with j <= i < e_j, and every column changes at
//    every block of the (short) sweep.
//
// The dS / P blocks are produced in the accumulator layout of S = Q K^T (dkv) or S^T = K Q^T (dq),
// which is exactly the B-operand layout of the products that consume them; the other operand of
// those products is read from row-major LDS tiles with transposing LDS reads.
#include "common.h"
#include <type_traits>

namespace dma {

struct BwdArgs {
  const uint16_t *Q, *K, *V, *O, *dO;
  uint16_t* dQ;
  const float *zq, *LSE;  // zq = z / softmax_scale
  float *Dws, *L2ws, *dK32, *dV32, *dz;
  const int32_t* expiry;
  const int4* blk;
  const int32_t* slot_tab;
  const int32_t* pcnt;
  const int32_t* plist;
  const char* consts;  // [0,256) zeros; +256: float -inf; +260: int 0; +264: int -1; +268: float +inf; +272: softmax scale, scale * log2(e)
  int T, H_q, H_kv, k, nblk_cap, kpad;
  int seg;       // query blocks swept by one clean-mode work item of dkv_kernel
  int seg_part;  // ... by one partial-mode work item
  size_t zero_n4;  // float4 elements from dK32 to the end of dV32 (cleared by dq_kernel)
  size_t dz_n;     // elements of dz (cleared by dq_kernel)
  unsigned grid_dq;  // workgroups of the dq_kernel launch
};

// ------------------------------------------------------------------ dQ (and D, LSE * log2 e)
// NW waves per workgroup: 8 (a whole 256-row block, four ring stages) or 4 (half a block, two ring
// stages, two workgroups per compute unit), as in the forward kernel.
template <int D, int NW>
__global__ __launch_bounds__(NW * 64, (NW == 8 || D == 256) ? 1 : (D == 64 ? 3 : 2)) void dq_kernel(BwdArgs p) {
  using TL = TileLayout<D>;
  constexpr int KS = D / 16, CB = D / 32, CPR = D / 8, RPL = 64 / CPR, WL = KT / RPL / NW;
  constexpr int NS = NW == 8 ? 4 : 2, TILE = KT * D, NT = NW * 64, HALVES = 8 / NW;
  __shared__ __align__(16) uint16_t ringK[NS * TILE];
  __shared__ __align__(16) uint16_t ringV[NS * TILE];
  __shared__ __align__(16) int ids_ring[2 * NS][KT];
  __shared__ __align__(16) float z_ring[NS][KT];
  __shared__ __align__(16) int e_ring[NS][KT];

  // This launch also clears what the key-stationary launches behind it accumulate into with atomics
  // (the fp32 dK / dV buffers and dz): every workgroup, also one without a block, takes its share of
  // the stores; this kernel is bound by the matrix cores, so they cost no time here.
  {
    const size_t nth = (size_t)p.grid_dq * NT, gid = (size_t)wg_id() * NT + thread_id();
    float4* acc4 = reinterpret_cast<float4*>(p.dK32);
    for (size_t i = gid; i < p.zero_n4; i += nth) acc4[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (size_t i = gid; i < p.dz_n; i += nth) p.dz[i] = 0.f;
  }
  int h, item;
  if (!xcd_map_interleaved(wg_id(), p.H_q, p.nblk_cap * HALVES, h, item)) return;
  const int bi = p.nblk_cap - 1 - item / HALVES;  // long blocks first
  const int4 info = p.blk[bi];
  if (info.x < 0) return;
  const int blk_row0 = info.y, row1 = info.z, doc0 = info.w;
  const int row0 = blk_row0 + (item % HALVES) * (NW * 32);  // first row of this workgroup's part of the block
  if (row0 >= row1) return;
  const int g = h / (p.H_q / p.H_kv);
  const int tid = thread_id(), w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63, n = l & 31, hh = l >> 5;
  const int ncol = min(p.k, blk_row0 - doc0);
  const int nc = (ncol + KT - 1) / KT;
  const int np_keys = p.pcnt[(size_t)h * p.nblk_cap + bi];
  const int nt = nc + (np_keys + KT - 1) / KT;
  const int32_t* slot_row = p.slot_tab + ((size_t)h * p.nblk_cap + bi) * p.kpad;
  const int32_t* plist_row = p.plist + ((size_t)h * p.nblk_cap + bi) * MAXPART;
  const float* zqh = p.zq + (size_t)h * p.T;
  const int32_t* eh = p.expiry + (size_t)h * p.T;
  const float* c_ninf = reinterpret_cast<const float*>(p.consts + 256);
  const int32_t* c_zero = reinterpret_cast<const int32_t*>(p.consts + 260);
  const int32_t* c_m1 = reinterpret_cast<const int32_t*>(p.consts + 264);
  const float scale = *reinterpret_cast<const float*>(p.consts + PLAN_SCALE_OFF);
  const float c2 = *reinterpret_cast<const float*>(p.consts + PLAN_C2_OFF);

  // gathered rows: wave-uniform base of the kv-head plus a 32-bit byte offset (id * row pitch + the
  // lane's chunk); an empty slot (id < 0) copies row 0, which its score of -inf keeps out of every sum
  const void* Kg = uniform_ptr(p.K + (size_t)g * D);
  const void* Vg = uniform_ptr(p.V + (size_t)g * D);
  const uint32_t row_pitch = (uint32_t)p.H_kv * D * 2;
  uint32_t lane_chunk[WL];
  int lane_row[WL];
#pragma unroll
  for (int j = 0; j < WL; j++) {
    lane_row[j] = (w * WL + j) * RPL + l / CPR;
    lane_chunk[j] = (uint32_t)(((l % CPR) ^ TL::swz(lane_row[j])) * 16);
  }
  const uint32_t ldsK = lds_addr(ringK) + (uint32_t)(w * WL * RPL * D * 2);
  const uint32_t ldsV = lds_addr(ringV) + (uint32_t)(w * WL * RPL * D * 2);
  auto issue_ids = [&](int tt) {
    if (w == 0) {
      const int32_t* src = c_m1;
      if (tt < nc) {
        src = slot_row + tt * KT + l;
      } else if (tt < nt) {
        const int q = (tt - nc) * KT + l;
        if (q < np_keys) src = plist_row + q;
      }
      dma4(src, &ids_ring[tt % (2 * NS)][0]);
    }
  };
  auto issue_kv = [&](int tt, int st) {  // st = tt % NS (a constant in the main loop)
    const int* idr = ids_ring[tt % (2 * NS)];
    int idv[WL];
#pragma unroll
    for (int j = 0; j < WL; j++) idv[j] = idr[lane_row[j]];
    int idl = 0;
    if (w == 1) idl = idr[l];
#pragma unroll
    for (int j = 0; j < WL; j++) {
      const uint32_t off = mul24((uint32_t)max(idv[j], 0), row_pitch) + lane_chunk[j];
      const uint32_t dst = (uint32_t)((st * TILE + j * RPL * D) * 2);
      dma16s_pair(Kg, Vg, off, ldsK + dst, ldsV + dst);
    }
    if (w == 1) {
      dma4(idl >= 0 ? zqh + idl : c_ninf, &z_ring[st][0]);
      dma4(idl >= 0 ? (const void*)(eh + idl) : (const void*)c_zero, &e_ring[st][0]);
    }
  };
  auto wait_tile = [&]() {
    if (w == 0) wait_vmcnt<(NS - 2) * (2 * WL + 1)>();
    else if (w == 1) wait_vmcnt<(NS - 2) * (2 * WL + 2)>();
    else wait_vmcnt<(NS - 2) * (2 * WL)>();
  };

  for (int tt = 0; tt < NS - 1; tt++) issue_ids(tt);
  wait_vmcnt<0>();
  lds_barrier();
  for (int i = 0; i < NS - 1; i++) {
    issue_ids(NS - 1 + i);
    issue_kv(i, i);
  }

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
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    settle(qreg[ks]);
    settle(doreg[ks]);
  }
  Dsum = half_swap_sum(Dsum);
  float lse2 = qvalid ? p.LSE[(size_t)h * p.T + qi] * LOG2E : INFINITY;
  settle(lse2);
  if (qvalid && hh == 0) {
    p.Dws[(size_t)h * p.T + qi] = -Dsum;  // (negated: the key-stationary kernel starts its dP accumulators at -D_i)
    p.L2ws[(size_t)h * p.T + qi] = lse2;
  }
  // fragment addresses with the ring bases folded in: inside the stage-unrolled main loop every LDS
  // read is one of these registers plus an immediate
  FragOffsets<D> fo;
  fo.init(l);
  uint32_t kfrag[KS], vfrag[KS], ktr[CB][2];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    kfrag[ks] = lds_addr(ringK) + 2 * fo.row(ks);
    vfrag[ks] = lds_addr(ringV) + 2 * fo.row(ks);
    settle(kfrag[ks]);
    settle(vfrag[ks]);
  }
#pragma unroll
  for (int cb = 0; cb < CB; cb++)
#pragma unroll
    for (int q = 0; q < 2; q++) {
      ktr[cb][q] = lds_addr(ringK) + 2 * fo.tr(cb, q);
      settle(ktr[cb][q]);
    }
  uint32_t zlane = lds_addr(&z_ring[0][4 * hh]);
  const uint32_t jlane = lds_addr(&ids_ring[0][4 * hh]), elane = lds_addr(&e_ring[0][4 * hh]);
  settle(zlane);
  f32x16 dqacc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; cb++)
#pragma unroll
    for (int v = 0; v < 16; v++) dqacc[cb][v] = 0.f;
  wait_vmcnt<0>();  // the ordinary loads and stores above; from here on only copies are in flight

  // one key tile; ST = t % NS is a compile-time constant (the loop below is unrolled over the ring)
  auto tile = [&](auto stc, const int t) {
    constexpr int ST = decltype(stc)::value;
    if (t > 0) wait_tile();
    lds_barrier();
    issue_ids(t + 2 * NS - 2);
    issue_kv(t + NS - 1, (ST + NS - 1) % NS);
    const int ist = t % (2 * NS);
    const bool masked = t >= nc;
    if (masked) {
      // partial tile: skip it if none of its keys is active on any of this wave's 32 rows
      const int jl = ids_ring[ist][l], el = e_ring[ST][l];
      const int rfirst = row0 + 32 * w;
      if (!__any((jl >= 0) & (jl <= rfirst + 31) & (el > rfirst))) return;
    }

#pragma unroll
    for (int kb = 0; kb < 2; kb++) {
      bf16x8 dsb[2];  // the two 16-key halves
      {
        // S^T starts at z / scale (so that scale * acc is the biased score) and, in a partial
        // tile, at -inf for pairs outside [j, e_j): those get P = 0 and dS = 0 exactly.
        f32x16 sacc, dpacc;
#pragma unroll
        for (int gq = 0; gq < 4; gq++) {
          const f32x4 zz = lds_load<f32x4>(zlane + 4 * (ST * KT + 32 * kb + 8 * gq));
#pragma unroll
          for (int u = 0; u < 4; u++) {
            sacc[4 * gq + u] = zz[u];
            dpacc[4 * gq + u] = 0.f;
          }
        }
        if (masked) {
#pragma unroll
          for (int gq = 0; gq < 4; gq++) {
            const i32x4 jj = lds_load<i32x4>(jlane + 4 * (ist * KT + 32 * kb + 8 * gq));
            const i32x4 ee = lds_load<i32x4>(elane + 4 * (ST * KT + 32 * kb + 8 * gq));
#pragma unroll
            for (int u = 0; u < 4; u++) {
              const bool ok = (jj[u] >= 0) & (qi >= jj[u]) & (qi < ee[u]);
              sacc[4 * gq + u] = ok ? sacc[4 * gq + u] : -INFINITY;
            }
          }
        }
#pragma unroll
        for (int ks = 0; ks < KS; ks++) {
          sacc = mfma32(lds_load<bf16x8>(kfrag[ks] + 2 * (ST * TILE + 32 * kb * D)), qreg[ks], sacc);
          dpacc = mfma32(lds_load<bf16x8>(vfrag[ks] + 2 * (ST * TILE + 32 * kb * D)), doreg[ks], dpacc);
        }
#pragma unroll
        for (int v = 0; v < 16; v++) {
          const float pv = fast_exp2(fmaf(sacc[v], c2, -lse2));
          const float ds = pv * (dpacc[v] - Dsum);
          dsb[v >> 3][v & 7] = (__bf16)ds;
        }
      }
      // dQ^T += K^T dS^T for this half of the tile
#pragma unroll
      for (int c = 0; c < 2; c++)
#pragma unroll
        for (int cb = 0; cb < CB; cb++) {
          const s16x4 lo = lds_read_tr_at(ktr[cb][0] + 2 * (ST * TILE + (32 * kb + 16 * c) * D));
          const s16x4 hi = lds_read_tr_at(ktr[cb][1] + 2 * (ST * TILE + (32 * kb + 16 * c) * D));
          const bf16x8 kf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
          dqacc[cb] = mfma32(kf, dsb[c], dqacc[cb]);
        }
    }
  };
  for (int t = 0; t < nt; t += NS) {
    tile(std::integral_constant<int, 0>{}, t);
    if (t + 1 >= nt) break;
    tile(std::integral_constant<int, 1>{}, t + 1);
    if constexpr (NS == 4) {
      if (t + 2 >= nt) break;
      tile(std::integral_constant<int, 2>{}, t + 2);
      if (t + 3 >= nt) break;
      tile(std::integral_constant<int, 3>{}, t + 3);
    }
  }
  static_assert(NS == 4 || NS == 2, "the main loop is unrolled over the ring stages");

  wait_vmcnt<0>();
  lds_barrier();
  uint16_t* Os = ringK;  // [NW * 32][D] staging with the tile swizzle
  static_assert(NS * KT >= NW * 32, "dQ staging aliases the K ring");
#pragma unroll
  for (int cb = 0; cb < CB; cb++)
#pragma unroll
    for (int gq = 0; gq < 4; gq++) {
      bf16x4 o4;
#pragma unroll
      for (int u = 0; u < 4; u++) o4[u] = (__bf16)(dqacc[cb][4 * gq + u] * scale);
      *reinterpret_cast<bf16x4*>(&Os[TL::off(32 * w + n, 4 * cb + gq) + 4 * hh]) = o4;
    }
  lds_barrier();
#pragma unroll
  for (int it = 0; it < NW * 32 * CPR / NT; it++) {
    const int c = tid + NT * it, r = c / CPR, col = c % CPR;
    if (row0 + r < row1)
      *reinterpret_cast<uint4*>(p.dQ + ((size_t)(row0 + r) * p.H_q + h) * D + 8 * col) =
          *reinterpret_cast<const uint4*>(&Os[TL::off(r, col)]);
  }
}

// ------------------------------------------------------------------ dK, dV, dz
constexpr int MAXSWEEP = 320;  // most query blocks one key-stationary work item sweeps

// Eight waves.  Wave w serves columns 32 * (w % 4) .. +31 of the workgroup's SG columns in one of two
// roles (w / 4); the two waves of a column block share a SIMD and overlap each other's MFMA and
// element-wise work, and each wave's state fits the register budget of two waves per SIMD:
//   role 0 ("P"):  S = Q K^T + z / scale, P = exp2(S c2 - LSE2) (masked in partial mode), dV^T += dO^T P;
//                  holds K fragments and dV^T; hands P (fp32) to its partner through LDS.
//   role 1 ("dS"): dP = dO V^T in the same period as role 0's S, then, one period later (so that
//                  its element-wise work overlaps role 0's MFMAs and vice versa),
//                  dS = P o (dP - D), dz += colsum(dS), dK^T += Q^T dS; holds V fragments and dK^T.
// Lane (n, hh) owns column 32 * (w % 4) + n; its accumulator holds channels 32cb + 8gq + 4hh + u.
template <int D, bool PARTIAL>
__global__ __launch_bounds__(512, 1) void dkv_kernel(BwdArgs p) {
  using TL = TileLayout<D>;
  constexpr int KS = D / 16, CB = D / 32, CPR = D / 8, RPL = 64 / CPR;
  constexpr int SUB = 32;                 // query rows per pipeline step
  constexpr int NSUB = BQ / SUB;          // steps per query block
  constexpr int NWL = 2 * (SUB / RPL);    // 16-byte wave copies per step (Q rows, then dO rows)
  constexpr int NS = D == 256 ? 3 : 5;    // ring stages (a stage of 512-byte rows is 32 KiB)
  constexpr int STILE = SUB * D;
  constexpr int LDS_ST = 32 + 4;          // staging row: the 32 channels of one flush pass, padded
  constexpr int NCH = D == 256 ? 2 : 1;   // column halves of a flush pass (LDS is short at 256 channels)
  constexpr int STC = 32 / NCH;           // columns staged at a time
  __shared__ __align__(16) uint16_t ringQ[NS * STILE];
  __shared__ __align__(16) uint16_t ringdO[NS * STILE];
  __shared__ __align__(16) float meta[NS][64];   // per stage: [0,32) LSE * log2 e, [32,64) -D
  __shared__ __align__(16) int idbuf[2][SG];     // column ids of the current / next block
  __shared__ __align__(16) int4 binfo[MAXSWEEP + 1];  // block table of this work item's sweep
  __shared__ __align__(16) float stage_all[8 * STC * LDS_ST];  // per wave: [STC columns][32 channels] fp32, flush staging
  __shared__ __align__(16) f32x4 pbuf[2][4][4][64];  // P hand-off (fp32): [step parity][column block][row group][lane]

  const int ngrp = PARTIAL ? MAXPART / SG : p.kpad / SG;
  const int nchunk = (p.nblk_cap + (PARTIAL ? p.seg_part : p.seg) - 1) / (PARTIAL ? p.seg_part : p.seg);
  int h, item;
  if (!xcd_map_interleaved(wg_id(), p.H_q, ngrp * nchunk, h, item)) return;
  // Clean mode: the groups of a chunk are neighbours.  Partial mode: group-major, because the high
  // groups of most chunks are empty and workgroups go to the shader engines in turn: with the
  // groups as the fast index all the work would land on the engines that get groups 0 and 1.
  const int chunk = PARTIAL ? item % nchunk : item / ngrp, grp = PARTIAL ? item / nchunk : item - chunk * ngrp;
  const int g = h / (p.H_q / p.H_kv);
  const int tid = thread_id(), w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63, n = l & 31, hh = l >> 5;
  const int kb4 = w & 3, role = w >> 2;
  const float* zqh = p.zq + (size_t)h * p.T;
  const float* Dh = p.Dws + (size_t)h * p.T;
  const float* L2h = p.L2ws + (size_t)h * p.T;
  const float* c_zero_f = reinterpret_cast<const float*>(p.consts + 260);
  const int32_t* c_m1 = reinterpret_cast<const int32_t*>(p.consts + 264);
  const float* c_pinf = reinterpret_cast<const float*>(p.consts + 268);
  const float scale = *reinterpret_cast<const float*>(p.consts + PLAN_SCALE_OFF);
  const float c2 = *reinterpret_cast<const float*>(p.consts + PLAN_C2_OFF);

  const int seg = PARTIAL ? p.seg_part : p.seg;
  const int bi_begin = chunk * seg, bi_end = min(bi_begin + seg, p.nblk_cap);
  // Block table of this sweep, kept in LDS so that the copy-ring loop issues no ordinary loads:
  // {block index, first row, end row, columns of this group} of every block of the chunk in which
  // the group has at least one column (clean mode: resident slots; partial mode: listed keys).
  __shared__ int nblocks_s;
  for (int i = tid; i < MAXSWEEP + 1; i += 512) binfo[i] = make_int4(-1, 0, 0, 0);
  __syncthreads();
  if (w == 0) {
    int cnt = 0;
    for (int base = bi_begin; base < bi_end; base += 64) {
      const int bi = base + l;
      int4 info = make_int4(-1, 0, 0, 0);
      int nc = 0;
      if (bi < bi_end) {
        info = p.blk[bi];
        if (info.x >= 0) {
          const int total = PARTIAL ? p.pcnt[(size_t)h * p.nblk_cap + bi] : min(p.k, info.y - info.w);
          nc = max(0, min(SG, total - grp * SG));
        }
      }
      const unsigned long long m = __ballot(nc > 0);
      if (nc > 0) binfo[cnt + __popcll(m & ((1ull << l) - 1ull))] = make_int4(bi, info.y, info.z, nc);
      cnt += __popcll(m);
    }
    if (l == 0) nblocks_s = cnt;
  }
  __syncthreads();
  const int nblocks = nblocks_s;
  if (nblocks == 0) return;
  const int nsteps = nblocks * NSUB;

  // Block cursor: the table entry of one block of the sweep, held in scalar registers and
  // refreshed only when a stream (producer or consumer) enters the next block.  Past the end of
  // the sweep it is a dummy without columns.
  struct Cursor {
    int bi, row0, row1, ncols;
  };
  auto load_cursor = [&](int bl) -> Cursor {
    const int4 info = binfo[min(bl, MAXSWEEP)];
    Cursor c;
    c.bi = __builtin_amdgcn_readfirstlane(info.x);
    c.row0 = __builtin_amdgcn_readfirstlane(info.y);
    c.row1 = __builtin_amdgcn_readfirstlane(info.z);
    c.ncols = __builtin_amdgcn_readfirstlane(info.w);
    return c;
  };

  // ---- producer: copies of step v (32 query rows of Q and dO, their LSE/D, and at a block's first
  // step the block's column ids).  Only the four role-0 waves issue copies: the role-1 waves carry
  // the longer chain of a step (they run the dS / dK^T part of the previous step before their dP),
  // while the role-0 waves have idle time at every barrier.  Every issuing wave issues the same
  // number of copies for every step.  Rows past the end of the block (or every row of a block without
  // columns) re-read a valid row: their LSE is +inf and their D is 0, so whatever Q / dO they hold
  // contributes exactly 0.
  constexpr int WLW0 = NWL / 4;   // copies per issuing wave and step: first half Q rows, second half dO rows
  constexpr int NLO = WLW0 / 2;   // distinct row positions among them
  static_assert(WLW0 == 2 * NLO && NLO >= 1, "copy layout of the key-stationary kernel");
  const uint32_t row_stride = (uint32_t)p.H_q * D * 2;  // bytes between consecutive rows of Q / dO
  int lane_r[NLO];          // tile row this lane copies (copy j takes rows (kb4 + 4 (j mod NLO)) * RPL ...)
  uint32_t lane_c[NLO];     // byte offset of its 16-byte chunk within the row
  uint32_t lane_off[NLO];   // ... from the step's first row, for a full step
#pragma unroll
  for (int u = 0; u < NLO; u++) {
    lane_r[u] = (kb4 + 4 * u) * RPL + l / CPR;
    lane_c[u] = (uint32_t)(((l % CPR) ^ TL::swz(lane_r[u])) * 16);
    lane_off[u] = (uint32_t)lane_r[u] * row_stride + lane_c[u];
    settle(lane_off[u]);
  }
  const char* Qh = (const char*)uniform_ptr(reinterpret_cast<const char*>(p.Q) + (size_t)h * D * 2);   // row 0 of this head
  const char* dOh = (const char*)uniform_ptr(reinterpret_cast<const char*>(p.dO) + (size_t)h * D * 2);
  Cursor pc = {-1, 0, 0, 0};
  int issue_st = 0;   // ring stage of the next step to issue (steps are issued in order: v mod NS without a division)
  auto issue = [&](int v) {
    if (role != 0) return;
    const int qs = v % NSUB;
    if (qs == 0) pc = load_cursor(v / NSUB);
    const int st = issue_st;
    issue_st = issue_st + 1 == NS ? 0 : issue_st + 1;
    const int rowb = pc.row0 + SUB * qs;
    const int left = pc.ncols > 0 ? pc.row1 - rowb : 0;   // rows of the block from this step on (wave-uniform)
    uint16_t* dstQ = ringQ + st * STILE;
    uint16_t* dstdO = ringdO + st * STILE;
    if (left >= SUB) {  // a full step: scalar base of the step's first row + the lane's fixed offset
      const uint32_t boff = (uint32_t)__builtin_amdgcn_readfirstlane((int)((uint32_t)rowb * row_stride));  // (below 4 GiB: checked on the host)
#pragma unroll
      for (int j = 0; j < WLW0; j++) {
        const int u = j % NLO;
        dma16s((j >= NLO ? dOh : Qh) + boff, lane_off[u], (j >= NLO ? dstdO : dstQ) + (kb4 + 4 * u) * RPL * D);
      }
      if (w == 0) dma4(hh == 0 ? L2h + rowb + n : Dh + rowb + n, &meta[st][0]);
    } else {  // the ragged last step of a block, or a block without columns: rows past the end repeat a valid one
      const int nvalid = max(left, 0);
      const uint32_t boff = (uint32_t)(nvalid > 0 ? rowb : 0) * row_stride;
#pragma unroll
      for (int j = 0; j < WLW0; j++) {
        const int u = j % NLO;
        const uint32_t off = (uint32_t)min(lane_r[u], max(nvalid - 1, 0)) * row_stride + lane_c[u];
        dma16s((j >= NLO ? dOh : Qh) + boff, off, (j >= NLO ? dstdO : dstQ) + (kb4 + 4 * u) * RPL * D);
      }
      if (w == 0) {
        const bool ok = n < nvalid;
        const float* src = hh == 0 ? (ok ? L2h + rowb + n : c_pinf) : (ok ? Dh + rowb + n : c_zero_f);
        dma4(src, &meta[st][0]);
      }
    }
    if (qs == 0 && (w == 1 || w == 2)) {
      const int bi = pc.bi;
      const int cl = (w - 1) * 64 + l;
      const int32_t* src = c_m1;
      if (cl < pc.ncols) {
        src = PARTIAL ? p.plist + ((size_t)h * p.nblk_cap + bi) * MAXPART + grp * SG + cl
                      : p.slot_tab + ((size_t)h * p.nblk_cap + bi) * p.kpad + grp * SG + cl;
      }
      dma4(src, &idbuf[(v / NSUB) & 1][(w - 1) * 64]);
    }
  };

  int curid = -1, kj = 0x7fffffff, ke = 0;
  float zq = -INFINITY;  // z / scale of this lane's key: the start value of its S accumulator
  bf16x8 breg[KS];  // B-operand fragments of this lane's key: K rows (role 0) or V rows (role 1)
#pragma unroll
  for (int ks = 0; ks < KS; ks++) breg[ks] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
  f32x16 acc[CB];   // dV^T (role 0) or dK^T (role 1) of this lane's column
#pragma unroll
  for (int cb = 0; cb < CB; cb++)
#pragma unroll
    for (int v = 0; v < 16; v++) acc[cb][v] = 0.f;
  float dzacc = 0.f;

  float* stage = stage_all + w * STC * LDS_ST;
  // Flush the columns whose lanes pass doit = true (wave-uniform call).  The accumulator is
  // transposed through the wave's LDS staging area, 32 channels at a time, so that
  // each atomic instruction adds consecutive channels of one key.
  auto flush = [&](bool doit) {
    const float dzt = dzacc + __shfl_xor(dzacc, 32);
    doit = doit && curid >= 0;
    const unsigned fm = (unsigned)(__ballot(doit) & 0xffffffffull);
    if (fm == 0) return;
    if (role == 1 && doit && hh == 0) atomicAdd(p.dz + (size_t)h * p.T + curid, dzt);
    const float mul = role == 1 ? scale : 1.f;
    float* dst = role == 1 ? p.dK32 : p.dV32;
    const bool dense = __popc(fm) > 6;  // many columns (a partial-mode block change, the end of a sweep)
    int* stage_id = reinterpret_cast<int*>(stage);
    if (NCH == 1 && dense && hh == 0) stage_id[n * LDS_ST + 32] = doit ? curid : -1;
#pragma unroll
    for (int cb = 0; cb < CB; cb++) {
#pragma unroll
      for (int ch = 0; ch < NCH; ch++) {  // columns STC * ch .. + STC - 1 of the wave's 32
        const bool mine = NCH == 1 || (n >> 4) == ch;
        const int sr = n & (STC - 1);     // staging row of this lane's column
        if (NCH > 1 && dense && hh == 0 && mine) stage_id[sr * LDS_ST + 32] = doit ? curid : -1;
        if (doit && mine) {
#pragma unroll
          for (int gq = 0; gq < 4; gq++) {
            f32x4 v4;
#pragma unroll
            for (int u = 0; u < 4; u++) v4[u] = acc[cb][4 * gq + u] * mul;
            *reinterpret_cast<f32x4*>(&stage[sr * LDS_ST + 8 * gq + 4 * hh]) = v4;
          }
        }
        if (dense) {
          // every pass handles the column pair (2i, 2i+1): the ids sit in the padding of the staging
          // rows, so the passes are independent of each other and pipeline
#pragma unroll
          for (int i = 0; i < STC / 2; i++) {
            const int c = 2 * i + hh;
            const int id = stage_id[c * LDS_ST + 32];
            if (id >= 0) atomicAdd(dst + ((size_t)id * p.H_kv + g) * D + 32 * cb + n, stage[c * LDS_ST + n]);
          }
        } else {
          unsigned m = NCH == 1 ? fm : fm & (0xffffu << (16 * ch));
          while (m) {  // two flushed columns per pass: lanes 0-31 and 32-63 take one column each
            const int c0 = __ffs(m) - 1;
            m &= m - 1;
            int c1 = c0;
            if (m) {
              c1 = __ffs(m) - 1;
              m &= m - 1;
            }
            const int c = hh == 0 ? c0 : c1;
            const int id = __shfl(curid, c);
            if (hh == 0 || c1 != c0)
              atomicAdd(dst + ((size_t)id * p.H_kv + g) * D + 32 * cb + n, stage[(c & (STC - 1)) * LDS_ST + n]);
          }
        }
      }
    }
  };

  FragOffsets<D> fo;
  fo.init(l);
  Cursor cc = {-1, 0, 0, 0};
  f32x16 sacc;        // role 0: S of the current step; role 1: dP of the step it has in flight
  bool pend = false;  // role 1: step pstep has its dP computed; dS, dz and dK^T are still due
  int pstep = 0;
#pragma unroll
  for (int vv = 0; vv < 16; vv++) sacc[vv] = 0.f;
  for (int v = 0; v < NS - 2; v++) issue(v);

  for (int it = 0; it <= nsteps; it++) {
    // copies of step `it` must have landed: at most NS-3 later steps' worth may still be in flight
    // (the occasional id copies and the flush traffic only make this wait more conservative)
    if (w == 0) wait_vmcnt<(NS - 3) * (WLW0 + 1)>();
    else wait_vmcnt<(NS - 3) * WLW0>();
    lds_barrier();
    fo.pin();
    issue(it + NS - 2);

    // role 1 first finishes the step whose dP it computed at the end of the previous period
    // (dS, dz, dK^T): its element-wise work then runs while role 0 is in its S = Q K^T MFMAs, and
    // its dK^T MFMAs while role 0 computes P.
    if (role == 1 && pend) {
      const int st = pstep % NS;
      const f32x4* ph = &pbuf[pstep & 1][kb4][0][l];  // row group gq at ph[64 * gq]
      bf16x8 bb[2];
#pragma unroll
      for (int gq = 0; gq < 4; gq++) {
        const f32x4 pq = ph[64 * gq];
#pragma unroll
        for (int u = 0; u < 4; u++) {
          const int vv = 4 * gq + u;
          const float ds = pq[u] * sacc[vv];  // sacc = dP - D (the accumulator started at -D_i)
          dzacc += ds;
          bb[vv >> 3][vv & 7] = (__bf16)ds;
        }
      }
      const uint16_t* Qs = ringQ + st * STILE;
#pragma unroll
      for (int c = 0; c < 2; c++)
#pragma unroll
        for (int cb = 0; cb < CB; cb++) acc[cb] = mfma32(fo.tr_frag(Qs, 16 * c, cb), bb[c], acc[cb]);
    }
    pend = false;

    const int v = it;
    if (v >= nsteps) continue;
    const int qs = v % NSUB;
    if (qs == 0) cc = load_cursor(v / NSUB);
    const int ncols = cc.ncols, row0 = cc.row0, row1 = cc.row1;
    if (qs == 0) {
      const int cl = 32 * kb4 + n;
      const int newid = (cl < ncols) ? idbuf[(v / NSUB) & 1][cl] : -1;
      const bool changed = newid != curid;
      if (__any(changed)) {
        // The new keys' rows are requested first and arrive while the finished keys are flushed
        // (the flush reads the accumulators and the old ids only).
        if (changed) {
          if (newid >= 0) {
            const uint16_t* src = (role == 0 ? p.K : p.V) + ((size_t)newid * p.H_kv + g) * D + 8 * hh;
#pragma unroll
            for (int ks = 0; ks < KS; ks++)
              breg[ks] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(src + 16 * ks));
            zq = zqh[newid];
            if (PARTIAL) {
              kj = newid;
              ke = p.expiry[(size_t)h * p.T + newid];
            }
          } else {
#pragma unroll
            for (int ks = 0; ks < KS; ks++) breg[ks] = __builtin_bit_cast(bf16x8, make_uint4(0, 0, 0, 0));
            zq = -INFINITY;
            kj = 0x7fffffff;
            ke = 0;
          }
        }
        flush(changed);  // finished keys out, then re-arm the changed columns
        if (changed) {
#pragma unroll
          for (int cb = 0; cb < CB; cb++)
#pragma unroll
            for (int vv = 0; vv < 16; vv++) acc[cb][vv] = 0.f;
          dzacc = 0.f;
          curid = newid;
        }
        if (PARTIAL) settle(ke);
        settle(zq);
#pragma unroll
        for (int ks = 0; ks < KS; ks++) settle(breg[ks]);
      }
    }
    if (ncols == 0 || row0 + SUB * qs >= row1) continue;  // nothing to do this step (same for both roles)
    if (PARTIAL) {
      // none of this wave's keys is active on these rows (entering keys are listed by ascending
      // first row, expiring ones by ascending end row); both roles of a column block agree
      const int rf = row0 + SUB * qs;
      if (!__any((kj < rf + SUB) & (ke > rf))) continue;
    }

    const int st = v % NS;
    const uint16_t* Qs = ringQ + st * STILE;
    const uint16_t* dOs = ringdO + st * STILE;

    // role 0: S = Q K^T ; role 1: dP = dO V^T   (this lane's key column against the step's 32 rows)
    const uint16_t* As = role == 0 ? Qs : dOs;
    if (role == 0) {  // S starts at z / scale, so that scale * S is the biased score
#pragma unroll
      for (int vv = 0; vv < 16; vv++) sacc[vv] = zq;
    } else {  // dP starts at -D_i of the accumulator's rows: the products then leave dP - D, what dS needs
      const float* Dss = meta[st] + 32;
#pragma unroll
      for (int gq = 0; gq < 4; gq++) {
        const f32x4 dd = *reinterpret_cast<const f32x4*>(&Dss[8 * gq + 4 * hh]);
#pragma unroll
        for (int u = 0; u < 4; u++) sacc[4 * gq + u] = dd[u];
      }
    }
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
      sacc = mfma32(fo.row_frag(As, 0, ks), breg[ks], sacc);
    }
    if (role == 1) {  // the rest of this step follows the next barrier
      pend = true;
      pstep = v;
      continue;
    }
    f32x4* ph = &pbuf[v & 1][kb4][0][l];
    bf16x8 bb[2];  // P: the B operand of the dV^T accumulation
    const float* lses = meta[st];
#pragma unroll
    for (int gq = 0; gq < 4; gq++) {
      const int r = 8 * gq + 4 * hh;
      const f32x4 ls = *reinterpret_cast<const f32x4*>(&lses[r]);
      f32x4 pq;
#pragma unroll
      for (int u = 0; u < 4; u++) {
        const int vv = 4 * gq + u;
        float pv = fast_exp2(fmaf(sacc[vv], c2, -ls[u]));
        if (PARTIAL) {
          const int row = row0 + SUB * qs + r + u;
          pv = ((row >= kj) & (row < ke)) ? pv : 0.f;
        }
        pq[u] = pv;
        bb[vv >> 3][vv & 7] = (__bf16)pv;
      }
      ph[64 * gq] = pq;
    }
#pragma unroll
    for (int c = 0; c < 2; c++)
#pragma unroll
      for (int cb = 0; cb < CB; cb++) acc[cb] = mfma32(fo.tr_frag(dOs, 16 * c, cb), bb[c], acc[cb]);
  }
  wait_vmcnt<0>();
  flush(true);
}

// dK, dV: fp32 accumulators -> bf16 outputs
__global__ void cvt_bf16_kernel(const float* __restrict__ a, const float* __restrict__ b, uint16_t* __restrict__ oa,
                                uint16_t* __restrict__ ob, size_t n4, unsigned nwg) {
  size_t i = wg_id() * (size_t)256 + thread_id();  // launched with 256 threads
  const size_t st = (size_t)nwg * 256;
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
  (void)z;
  const dma_shape& s = p.s;
  const PlanLayout& L = p.pl;
  const WsLayout wl = ws_layout(s);
  BwdArgs a;
  a.Q = (const uint16_t*)Q; a.K = (const uint16_t*)K; a.V = (const uint16_t*)V;
  a.O = (const uint16_t*)O; a.dO = (const uint16_t*)dO; a.dQ = (uint16_t*)dQ;
  a.zq = (const float*)(p.plan + L.off_zq); a.LSE = LSE; a.expiry = expiry;
  a.Dws = (float*)(ws + wl.off_D); a.L2ws = (float*)(ws + wl.off_L2);
  a.dK32 = (float*)(ws + wl.off_dK); a.dV32 = (float*)(ws + wl.off_dV); a.dz = dz;
  a.blk = (const int4*)(p.plan + L.off_blk);
  a.slot_tab = (const int32_t*)(p.plan + L.off_slot);
  a.pcnt = (const int32_t*)(p.plan + L.off_pcnt);
  a.plist = (const int32_t*)(p.plan + L.off_plist);
  a.consts = p.plan + L.off_consts;
  a.T = s.T; a.H_q = s.H_q; a.H_kv = s.H_kv; a.k = s.k; a.nblk_cap = L.nblk_cap; a.kpad = L.kpad;
  {  // sweep length of a clean-mode work item: as long as possible while keeping >= 512 work items
    const long groups = (long)(L.kpad / SG) * s.H_q;
    long seg = (long)L.nblk_cap * groups / 512;
    if (seg < 2) seg = 2;
    if (seg > L.nblk_cap) seg = L.nblk_cap;
    if (seg > MAXSWEEP) seg = MAXSWEEP;
    a.seg = (int)seg;
    a.seg_part = L.nblk_cap < 8 ? L.nblk_cap : 8;  // blocks per partial-mode work item: amortises the pipeline fill
  }

  const size_t nkv = (size_t)s.T * s.H_kv * s.d;
  a.zero_n4 = ((wl.off_dV - wl.off_dK) / 4 + nkv + 3) / 4;  // (the layout pads both buffers to 256 bytes)
  a.dz_n = (size_t)s.H_q * s.T;
  prof_begin(DMA_STAGE_BWD_ZERO, st);  // (an empty stage: dq_kernel clears the accumulators)
  prof_end(DMA_STAGE_BWD_ZERO, st);
  // (at 256 channels the query-stationary kernels run as half blocks: four waves with the whole register file each)
  const unsigned gq = s.d != 128 ? xcd_grid(s.H_q, 2l * L.nblk_cap) : xcd_grid(s.H_q, L.nblk_cap);
  a.grid_dq = gq;
  const unsigned gclean = xcd_grid(s.H_q, (long)((L.nblk_cap + a.seg - 1) / a.seg) * (L.kpad / SG));
  const unsigned gpart = xcd_grid(s.H_q, (long)((L.nblk_cap + a.seg_part - 1) / a.seg_part) * (MAXPART / SG));
  prof_begin(DMA_STAGE_BWD_DQ, st);
  // (the half-block variant, NW = 4, measured the same or slower at every benchmark shape)
  if (s.d == 256) dq_kernel<256, 4><<<gq, 256, 0, st>>>(a);
  else if (s.d == 128) dq_kernel<128, 8><<<gq, 512, 0, st>>>(a);
  else dq_kernel<64, 4><<<gq, 256, 0, st>>>(a);  // half blocks, three workgroups per compute unit (three waves per SIMD)
  prof_end(DMA_STAGE_BWD_DQ, st);
  prof_begin(DMA_STAGE_BWD_DKV, st);
  if (s.d == 256) dkv_kernel<256, false><<<gclean, 512, 0, st>>>(a);
  else if (s.d == 128) dkv_kernel<128, false><<<gclean, 512, 0, st>>>(a);
  else dkv_kernel<64, false><<<gclean, 512, 0, st>>>(a);
  prof_end(DMA_STAGE_BWD_DKV, st);
  prof_begin(DMA_STAGE_BWD_PART, st);
  if (s.d == 256) dkv_kernel<256, true><<<gpart, 512, 0, st>>>(a);
  else if (s.d == 128) dkv_kernel<128, true><<<gpart, 512, 0, st>>>(a);
  else dkv_kernel<64, true><<<gpart, 512, 0, st>>>(a);
  prof_end(DMA_STAGE_BWD_PART, st);
  prof_begin(DMA_STAGE_BWD_CVT, st);
  const unsigned gcvt = grid_for(nkv / 4, 1024);
  cvt_bf16_kernel<<<gcvt, 256, 0, st>>>(a.dK32, a.dV32, (uint16_t*)dK, (uint16_t*)dV, nkv / 4, gcvt);
  prof_end(DMA_STAGE_BWD_CVT, st);
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

}  // namespace dma
