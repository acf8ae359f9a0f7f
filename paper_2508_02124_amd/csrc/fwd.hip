// Forward pass (Eq. 5-6; online softmax of Alg. 1, query-stationary so O, l, m stay in registers).
//
// One workgroup (8 waves) = one block of BQ = 256 query rows of one head; wave w owns rows
// 32w .. 32w+31, and the two waves that share a SIMD overlap each other's MFMA and softmax work.
// The keys a block needs are gathered, KT at a time, into a ring of LDS stages by asynchronous
// global->LDS copies issued NS-1 tiles ahead (no staging registers): first the slot table row of
// the block (residents active for every row of the block: no mask needed, empty slots carry
// z = -inf), then the block's partial list (keys entering or expiring inside the block: pairs
// outside j <= i < e_j start their score at -inf).  The key ids of a tile are themselves copied
// into an LDS ring NS-1 tiles before the tile's K/V copies are issued, so no register ever waits
// on a load.
//
// Per tile the wave computes S^T = K Q^T (keys x queries) so that each lane holds one query column
// per block: the softmax statistics are per lane, and the exponentiated block is already laid out
// as the B operand of O^T += V^T P^T.  The bias z is not added after the product: the accumulator
// starts at z / scale, so scale * acc is the biased score and one FMA gives the exp2 argument.
#include "common.h"
#include <type_traits>

namespace dma {

struct FwdArgs {
  const uint16_t *Q, *K, *V;
  uint16_t* O;
  const float* zq;      // z / softmax_scale
  float* LSE;
  const int32_t* expiry;
  const int4* blk;
  const int32_t* slot_tab;
  const int32_t* pcnt;
  const int32_t* plist;
  const char* consts;   // [0,256) zeros; +256: float -inf; +260: int 0; +264: int -1; +272: softmax scale, scale * log2(e)
  int T, H_q, H_kv, k, nblk_cap, kpad;
};

constexpr float MSLACK = 8.f;  // log2 slack of the lazily updated softmax reference maximum

// (second launch bound = waves per SIMD: at D = 64 the kernel is held to 128 registers so that two
// workgroups share a compute unit -- four waves per SIMD hide the element-wise work, which weighs
// twice as much per MFMA there; at D = 128 the accumulators alone need more than that)
// NW waves per workgroup: 8 (one 256-row block per workgroup, four ring stages) or 4 (half a block,
// two ring stages, two workgroups per compute unit: the two waves of a SIMD then belong to different
// workgroups and do not meet at the same barriers).
template <int D, int NW>
__global__ __launch_bounds__(NW * 64, D == 64 ? 4 : ((NW == 8 || D == 256) ? 1 : 2)) void fwd_kernel(FwdArgs p) {
  using TL = TileLayout<D>;
  constexpr int KS = D / 16;          // contraction steps of K Q^T
  constexpr int CB = D / 32;          // 32-channel blocks of O^T
  constexpr int CPR = D / 8;          // 16-byte chunks per row
  constexpr int RPL = 64 / CPR;       // rows covered by one wave-wide 16-byte copy
  constexpr int WL = KT / RPL / NW;   // such copies per wave per K (or V) tile
  constexpr int NS = NW == 8 ? 4 : 2; // ring stages
  constexpr int NT = NW * 64;         // threads
  constexpr int HALVES = 8 / NW;      // workgroups per 256-row block
  constexpr int TILE = KT * D;        // elements of one K or V tile
  __shared__ __align__(16) uint16_t ringK[NS * TILE];
  __shared__ __align__(16) uint16_t ringV[NS * TILE];
  __shared__ __align__(16) int ids_ring[2 * NS][KT];
  __shared__ __align__(16) float z_ring[NS][KT];
  __shared__ __align__(16) int e_ring[NS][KT];

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
  const float c2 = *reinterpret_cast<const float*>(p.consts + PLAN_C2_OFF);  // softmax scale * log2(e)

  // ---- asynchronous producers (every wave issues the same number of copies for every tile index,
  // real or past the end, so the outstanding-copy counts below are constants).  A gathered row is
  // addressed as a wave-uniform base (the kv-head's first row) plus a 32-bit byte offset
  // id * row pitch + the lane's chunk; an empty slot (id < 0) copies row 0 instead, which its score
  // of -inf keeps out of every sum.
  const void* Kg = uniform_ptr(p.K + (size_t)g * D);
  const void* Vg = uniform_ptr(p.V + (size_t)g * D);
  const uint32_t row_pitch = (uint32_t)p.H_kv * D * 2;
  uint32_t lane_chunk[WL];  // byte offset of the lane's 16-byte chunk within its row, per copy
  int lane_row[WL];         // tile row the lane copies
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
  // copies a wave issues per tile step, and how many may still be in flight when tile t is needed
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
#pragma unroll
    for (int ks = 0; ks < KS; ks++) settle(qreg[ks]);
  }
  // The lane's fragment addresses with the ring bases folded in: inside the (stage-unrolled) main
  // loop every LDS read is one of these registers plus an immediate.
  FragOffsets<D> fo;
  fo.init(l);
  uint32_t kfrag[KS], vfrag[CB][2];
#pragma unroll
  for (int ks = 0; ks < KS; ks++) {
    kfrag[ks] = lds_addr(ringK) + 2 * fo.row(ks);
    settle(kfrag[ks]);
  }
#pragma unroll
  for (int cb = 0; cb < CB; cb++)
#pragma unroll
    for (int q = 0; q < 2; q++) {
      vfrag[cb][q] = lds_addr(ringV) + 2 * fo.tr(cb, q);
      settle(vfrag[cb][q]);
    }
  uint32_t zlane = lds_addr(&z_ring[0][4 * hh]);
  const uint32_t jlane = lds_addr(&ids_ring[0][4 * hh]), elane = lds_addr(&e_ring[0][4 * hh]);
  settle(zlane);
  f32x16 oacc[CB];
#pragma unroll
  for (int cb = 0; cb < CB; cb++)
#pragma unroll
    for (int v = 0; v < 16; v++) oacc[cb][v] = 0.f;
  float m_run = -INFINITY, lsum = 0.f;
  // the query loads above are ordinary loads issued after the prologue copies; wait for them here so
  // that the per-tile counts below only ever see copies
  wait_vmcnt<0>();

  // one key tile; ST = t % NS is a compile-time constant (the loop below is unrolled over the ring)
  auto tile = [&](auto stc, const int t) {
    constexpr int ST = decltype(stc)::value;
    if (t > 0) wait_tile();  // (t == 0: the wait above already drained everything)
    lds_barrier();
    issue_ids(t + 2 * NS - 2);
    issue_kv(t + NS - 1, (ST + NS - 1) % NS);
    const int ist = t % (2 * NS);  // stage of the tile's ids
    if (t >= nc) {
      // partial tile: skip it if none of its keys is active on any of this wave's 32 rows (the
      // lists are ordered by first / last active row, so about half of the wave-tiles drop out)
      const int jl = ids_ring[ist][l], el = e_ring[ST][l];
      const int rfirst = row0 + 32 * w;
      if (!__any((jl >= 0) & (jl <= rfirst + 31) & (el > rfirst))) return;
    }

    // The accumulator of S^T = K Q^T starts at z / scale, so that scale * acc is the biased score;
    // in a partial tile, pairs outside [j, e_j) start (and stay) at -inf.
    f32x16 sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int gq = 0; gq < 4; gq++) {
        const f32x4 zz = lds_load<f32x4>(zlane + 4 * (ST * KT + 32 * kb + 8 * gq));
#pragma unroll
        for (int u = 0; u < 4; u++) sacc[kb][4 * gq + u] = zz[u];
      }
    if (t >= nc) {
      const uint32_t js = jlane + 4 * ist * KT;
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int gq = 0; gq < 4; gq++) {
          const i32x4 jj = lds_load<i32x4>(js + 4 * (32 * kb + 8 * gq));
          const i32x4 ee = lds_load<i32x4>(elane + 4 * (ST * KT + 32 * kb + 8 * gq));
#pragma unroll
          for (int u = 0; u < 4; u++) {
            const bool ok = (jj[u] >= 0) & (qi >= jj[u]) & (qi < ee[u]);
            sacc[kb][4 * gq + u] = ok ? sacc[kb][4 * gq + u] : -INFINITY;
          }
        }
    }
    // two independent accumulation chains (the tile's two 32-key halves), interleaved
#pragma unroll
    for (int ks = 0; ks < KS; ks++)
#pragma unroll
      for (int kb = 0; kb < 2; kb++) {
        const bf16x8 kf = lds_load<bf16x8>(kfrag[ks] + 2 * (ST * TILE + 32 * kb * D));
        sacc[kb] = mfma32(kf, qreg[ks], sacc[kb]);
      }
    // Online softmax in the exp2 domain with a lazily updated reference maximum: m_run moves only
    // when the tile's maximum exceeds it by more than MSLACK, so that the rescaling of O and l is
    // rare; until then the exponentials are at most 2^MSLACK, which fp32 accumulation absorbs.
    float mx = fmaxf(sacc[0][0], sacc[1][0]);
#pragma unroll
    for (int v = 1; v < 16; v++) mx = fmaxf(fmaxf(mx, sacc[0][v]), sacc[1][v]);  // one three-input maximum each
    mx = half_swap_max(mx) * c2;
    const bool grow = mx > m_run + MSLACK;
    if (__any(grow)) {
      const float m_new = grow ? mx : m_run;
      const float alpha = grow ? fast_exp2(m_run - m_new) : 1.f;  // m_run = -inf: 0, nothing accumulated yet
      m_run = m_new;
      lsum *= alpha;
#pragma unroll
      for (int cb = 0; cb < CB; cb++)
#pragma unroll
        for (int v = 0; v < 16; v++) oacc[cb][v] *= alpha;
    }
    const float msub = (m_run == -INFINITY) ? 0.f : m_run;  // row with nothing kept so far: exp2(-inf - 0) = 0
    bf16x8 pb[4];  // the four 16-key quarters
    float ls2 = 0.f;  // (two chains: the sums stay fp32-exact in the weights, LSE feeds the backward)
#pragma unroll
    for (int kb = 0; kb < 2; kb++)
#pragma unroll
      for (int v = 0; v < 16; v++) {
        const float pv = fast_exp2(fmaf(sacc[kb][v], c2, -msub));
        if (kb == 0) lsum += pv; else ls2 += pv;
        pb[2 * kb + (v >> 3)][v & 7] = (__bf16)pv;
      }
    lsum += ls2;
    // O^T += V^T P^T
#pragma unroll
    for (int c = 0; c < 4; c++)
#pragma unroll
      for (int cb = 0; cb < CB; cb++) {
        const s16x4 lo = lds_read_tr_at(vfrag[cb][0] + 2 * (ST * TILE + 16 * c * D));
        const s16x4 hi = lds_read_tr_at(vfrag[cb][1] + 2 * (ST * TILE + 16 * c * D));
        const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        oacc[cb] = mfma32(vf, pb[c], oacc[cb]);
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

  // epilogue: drain the (dummy) copies still in flight, normalise, stage O through LDS for
  // coalesced rows, write LSE
  wait_vmcnt<0>();
  lds_barrier();
  uint16_t* Os = ringK;  // [NW * 32][D] with the tile swizzle
  static_assert(NS * KT >= NW * 32, "O staging aliases the K ring");
  {
    const float ltot = half_swap_sum(lsum);
    const float inv = 1.f / ltot;
    if (hh == 0 && qi < row1) p.LSE[(size_t)h * p.T + qi] = (m_run + __builtin_amdgcn_logf(ltot)) * LN2;
#pragma unroll
    for (int cb = 0; cb < CB; cb++)
#pragma unroll
      for (int gq = 0; gq < 4; gq++) {
        bf16x4 o4;
#pragma unroll
        for (int u = 0; u < 4; u++) o4[u] = (__bf16)(oacc[cb][4 * gq + u] * inv);
        *reinterpret_cast<bf16x4*>(&Os[TL::off(32 * w + n, 4 * cb + gq) + 4 * hh]) = o4;
      }
  }
  lds_barrier();
#pragma unroll
  for (int it = 0; it < NW * 32 * CPR / NT; it++) {
    const int c = tid + NT * it, r = c / CPR, col = c % CPR;
    if (row0 + r < row1)
      *reinterpret_cast<uint4*>(p.O + ((size_t)(row0 + r) * p.H_q + h) * D + 8 * col) =
          *reinterpret_cast<const uint4*>(&Os[TL::off(r, col)]);
  }
}

int launch_fwd(const Ptrs& p, const void* Q, const void* K, const void* V, const float* z, const int32_t* expiry,
               const int32_t* cu, void* O, float* LSE, hipStream_t st) {
  (void)cu;
  (void)z;
  const dma_shape& s = p.s;
  const PlanLayout& L = p.pl;
  FwdArgs a;
  a.Q = (const uint16_t*)Q; a.K = (const uint16_t*)K; a.V = (const uint16_t*)V; a.O = (uint16_t*)O;
  a.zq = (const float*)(p.plan + L.off_zq); a.LSE = LSE; a.expiry = expiry;
  a.blk = (const int4*)(p.plan + L.off_blk);
  a.slot_tab = (const int32_t*)(p.plan + L.off_slot);
  a.pcnt = (const int32_t*)(p.plan + L.off_pcnt);
  a.plist = (const int32_t*)(p.plan + L.off_plist);
  a.consts = p.plan + L.off_consts;
  a.T = s.T; a.H_q = s.H_q; a.H_kv = s.H_kv; a.k = s.k; a.nblk_cap = L.nblk_cap; a.kpad = L.kpad;
  prof_begin(DMA_STAGE_FWD, st);
  // Small problems (fewer than four 256-row blocks per compute unit, e.g. 2 x 4096 tokens x 16 heads) run
  // the half-block variant: twice as many, shorter work items balance better over the chip (-7 % there);
  // at the headline size the two variants measure the same and the whole-block one gathers half as much.
  const bool half_blocks = s.d == 128 && (long)s.H_q * L.nblk_cap < 1024;
  // 256 channels: half blocks of four waves, one per SIMD with the whole register file (the output
  // accumulators alone are 128 registers per wave).
  if (s.d == 256) fwd_kernel<256, 4><<<xcd_grid(s.H_q, 2l * L.nblk_cap), 256, 0, st>>>(a);
  else if (half_blocks) fwd_kernel<128, 4><<<xcd_grid(s.H_q, 2l * L.nblk_cap), 256, 0, st>>>(a);
  else if (s.d == 128) fwd_kernel<128, 8><<<xcd_grid(s.H_q, L.nblk_cap), 512, 0, st>>>(a);
  else fwd_kernel<64, 8><<<xcd_grid(s.H_q, L.nblk_cap), 512, 0, st>>>(a);
  prof_end(DMA_STAGE_FWD, st);
  return hipGetLastError() == hipSuccess ? DMA_OK : DMA_EHIP;
}

}  // namespace dma
