// Shared device/host definitions of the gfx950 Dynamic Mask Attention kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/dma.h"

namespace dma {

// ------------------------------------------------------------------ tiling constants
constexpr int BQ = 256;        // query rows per block (one workgroup of the query-stationary kernels: 8 waves x 32 rows)
constexpr int KT = 64;         // keys per tile of the query-stationary kernels
constexpr int MAXPART = 2 * BQ;  // a block has at most BQ entering + BQ expiring keys
constexpr int SG = 128;        // slot columns per workgroup of the key-stationary backward
constexpr int SEG_MIN = 4096;  // keys per segment of the selection (what one workgroup sorts in LDS): 4096 when
constexpr int SEG_MAX = 16384; // no document is longer than four such segments (more workgroups), else 16384
constexpr float LOG2E = 1.4426950408889634f;
// byte offsets in the plan's constant block of the softmax scale the stored z / scale was written with,
// and of scale * log2(e)
constexpr int PLAN_SCALE_OFF = 272, PLAN_C2_OFF = 276;
constexpr float LN2 = 0.6931471805599453f;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// ------------------------------------------------------------------ mask plan layout (host + device)
// The plan is one device buffer.  All offsets are in bytes from its start.
struct PlanLayout {
  int nblk_cap;    // upper bound on the number of query blocks: T / BQ + n_docs
  int kpad;        // slot-table row length: min(k, T) rounded up to SG
  int seg;         // segment length chosen for this shape
  int nbits_cap;   // wavelet levels of a segment (at most log2 SEG_MAX)
  int wcap;        // 64-bit words per wavelet level per head (every segment has two spare words)
  int nseg_cap;    // upper bound on the number of segments: T / seg + n_docs + 1
  size_t off_hdr;      // int32[16]: [0] number of blocks
  size_t off_consts;   // 512 B: [0,256) zeros (a dummy K/V row); then float -inf, int32 0, int32 -1, float +inf,
                       // float softmax scale, float scale * log2(e) (what zq was divided by: the attention kernels read it here)
  size_t off_zq;       // float[H_q][T]: z / softmax_scale, the bias as the start value of a Q K^T accumulator
  size_t off_blk;      // int4[nblk_cap]: {doc, row0, row1, doc_start}; doc = -1 past the end
  size_t off_docblk;   // int32[n_docs + 1]: first block of each document
  size_t off_slot;     // int32[H_q][nblk_cap][kpad]: clean resident key of each slot, or -1
  size_t off_pcnt;     // int32[H_q][nblk_cap]
  size_t off_plist;    // int32[H_q][nblk_cap][MAXPART]: keys partially active in the block
  size_t off_parent;   // int32[H_q][T]: key evicted when this key entered (global index) or -1
  size_t off_slotid;   // int32[H_q][T]: slot column of the key (local), valid if the key ever enters
  size_t off_sk0, off_sk1;   // uint32[H_q][T] x2: sort keys (ping-pong), later wavelet values
  size_t off_si0, off_si1;   // uint32[H_q][T] x2: sort payload (local key index)
  size_t off_wbits;    // uint64[H_q][nbits_cap][wcap]: zero-bit masks of each wavelet level
  size_t off_wcnt;     // uint32[H_q][nbits_cap][wcap]: zeros before each word
  size_t off_wzero;    // uint32[H_q][nseg_cap][nbits_cap]: total zeros of each level of each segment
  size_t total;
};

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

static inline int ceil_log2(int n) {
  int b = 0;
  while ((1ll << b) < n) b++;
  return b;
}

static inline PlanLayout plan_layout(const dma_shape& s) {
  PlanLayout p;
  size_t T = s.T, H = s.H_q;
  p.nblk_cap = s.T / BQ + s.n_docs;
  int kk = s.k < s.T ? s.k : s.T;
  p.kpad = (kk + SG - 1) / SG * SG;
  {
    const int longest = s.max_seqlen > 0 && s.max_seqlen < s.T ? s.max_seqlen : s.T;
    p.seg = longest <= 4 * SEG_MIN ? SEG_MIN : SEG_MAX;  // (any choice is correct; this one is a matter of speed)
  }
  p.nbits_cap = ceil_log2(s.T < 2 ? 2 : (s.T < p.seg ? s.T : p.seg));
  p.nseg_cap = s.T / p.seg + s.n_docs + 1;
  p.wcap = s.T / 64 + 2 * (s.T / p.seg) + 5 * s.n_docs + p.seg / 64 + 8;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o = align_up(o + bytes, 256); return r; };
  p.off_hdr = take(64);
  p.off_consts = take(512);
  p.off_zq = take(H * T * 4);
  p.off_blk = take((size_t)p.nblk_cap * 16);
  p.off_docblk = take((size_t)(s.n_docs + 1) * 4);
  p.off_slot = take(H * p.nblk_cap * (size_t)p.kpad * 4);
  p.off_pcnt = take(H * p.nblk_cap * 4);
  p.off_plist = take(H * p.nblk_cap * (size_t)MAXPART * 4);
  p.off_parent = take(H * T * 4);
  p.off_slotid = take(H * T * 4);
  p.off_sk0 = take(H * T * 4);
  p.off_sk1 = take(H * T * 4);
  p.off_si0 = take(H * T * 4);
  p.off_si1 = take(H * T * 4);
  p.off_wbits = take(H * p.nbits_cap * (size_t)p.wcap * 8);
  p.off_wcnt = take(H * p.nbits_cap * (size_t)p.wcap * 4);
  p.off_wzero = take(H * (size_t)p.nseg_cap * p.nbits_cap * 4);
  p.total = o;
  return p;
}

// workspace of dma_bwd: D and LSE * log2(e) [H_q][T] float, dK32 / dV32 [T][H_kv][d] float
struct WsLayout {
  size_t off_D, off_L2, off_dK, off_dV, total;
};
static inline WsLayout ws_layout(const dma_shape& s) {
  WsLayout w;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o = align_up(o + bytes, 256); return r; };
  w.off_D = take((size_t)s.H_q * s.T * 4);
  w.off_L2 = take((size_t)s.H_q * s.T * 4);
  w.off_dK = take((size_t)s.T * s.H_kv * s.d * 4);
  w.off_dV = take((size_t)s.T * s.H_kv * s.d * 4);
  w.total = o;
  return w;
}

// ------------------------------------------------------------------ launch entry points (defined in the .hip files)
struct Ptrs {  // everything the kernels need, resolved by the host API
  dma_shape s;
  PlanLayout pl;
  char* plan;
  float scale;
};

int launch_mask_gen(const Ptrs& p, const void* V, const float* W, const float* A, const int32_t* cu,
                    float* z, int32_t* expiry, int32_t* topk_idx, hipStream_t st);
int launch_bias_add(const Ptrs& p, const float* bias, int bias_heads, int per_token, const int32_t* cu, hipStream_t st);
int launch_bias_bwd(const dma_shape& s, const float* dz, int bias_heads, int per_token, const int32_t* cu, float* dbias,
                    hipStream_t st);
int launch_fwd(const Ptrs& p, const void* Q, const void* K, const void* V, const float* z,
               const int32_t* expiry, const int32_t* cu, void* O, float* LSE, hipStream_t st);
int launch_bwd(const Ptrs& p, const void* Q, const void* K, const void* V, const void* O, const void* dO,
               const float* LSE, const float* z, const int32_t* expiry, const int32_t* cu,
               void* dQ, void* dK, void* dV, float* dz, char* ws, hipStream_t st);
int launch_fwd_f32(const Ptrs& p, const float* Q, const float* K, const float* V, const float* z,
                   const int32_t* expiry, const int32_t* cu, float* O, float* LSE, hipStream_t st);
int launch_bwd_f32(const Ptrs& p, const float* Q, const float* K, const float* V, const float* O,
                   const float* dO, const float* LSE, const float* z, const int32_t* expiry,
                   const int32_t* cu, float* dQ, float* dK, float* dV, float* dz, char* ws, hipStream_t st);

int launch_mask_bwd(const dma_shape& s, const void* V, const float* W, const float* A, const float* dz,
                    float* dW, float* dA, void* dV, int accumulate, hipStream_t st);

int launch_xhead_scores(const dma_shape& s, const void* V, const float* Delta, const float* A, float* z, hipStream_t st);
int launch_xhead_bwd(const dma_shape& s, const void* V, const float* Delta, const float* A, const float* dz,
                     float* dDelta, float* dA, void* dV, int accumulate, hipStream_t st);

size_t decode_part_floats(const dma_shape& s);
size_t decode_sel_words(const dma_shape& s);
size_t decode_scratch_bytes(const dma_shape& s);   // partial outputs + selection words of one call
int decode_static_scratch(void** out);             // the current device's copy of the library-owned scratch
int launch_decode(const dma_shape& s, float scale, const void* q, const void* K, const void* V, const float* z,
                  const int32_t* cu, const int32_t* lens, int incremental, void* o, float* lse, int32_t* kept,
                  void* part_and_sel, hipStream_t st);


// stage events (see dma_profile_events): no-ops unless the caller armed them on this thread
void prof_begin(int stage, hipStream_t st);
void prof_end(int stage, hipStream_t st);

#ifdef __HIPCC__
// ------------------------------------------------------------------ device helpers
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  // D[32x32] += A[32x16] B[16x32].  Lane l holds A[l%32][8*(l/32) .. +8), B[8*(l/32) .. +8)[l%32],
  // and D[8*(v/4) + 4*(l/32) + v%4][l%32] in register v.
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Four bf16 of one column of a row-major LDS tile, taken from four consecutive rows:
// within each group of 16 lanes, lane i supplies the address of row (i/4), columns 4*(i%4)..+3 of a
// 4 x 16 patch, and receives column i of that patch (rows 0..3).
__device__ __forceinline__ s16x4 lds_read_tr(const void* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
}

// LDS layout of a row-major bf16 tile with D channels per row, addressed in 16-byte chunks: chunk c
// of row r is stored at chunk position c ^ swz(r) of that row (rows are D * 2 bytes, unpadded).
// D = 128 (256-byte rows, one pass over all LDS banks): swz(r) = 4 * (r % 4) + (r / 4) % 4.  Sixteen
// consecutive rows put the same chunk in sixteen different positions (conflict-free 16-byte row
// reads); four consecutive rows put a 64-byte channel group in four different 64-byte bank groups
// (conflict-free transposing reads).  D = 64 (128-byte rows, two per bank pass):
// swz(r) = 4 * ((r / 2) % 2) + (r / 4) % 4 gives the same two properties.
template <int D> struct TileLayout;
template <> struct TileLayout<128> {
  static __device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }
  static __device__ __forceinline__ int off(int r, int c) { return r * 128 + ((c ^ swz(r)) << 3); }
};
template <> struct TileLayout<256> {  // rows of 32 chunks: the low four chunk bits are swizzled as at 128
  static __device__ __forceinline__ int swz(int r) { return ((r & 3) << 2) | ((r >> 2) & 3); }
  static __device__ __forceinline__ int off(int r, int c) { return r * 256 + ((c ^ swz(r)) << 3); }
};
template <> struct TileLayout<64> {
  static __device__ __forceinline__ int swz(int r) { return (((r >> 1) & 1) << 2) | ((r >> 2) & 3); }
  static __device__ __forceinline__ int off(int r, int c) { return r * 64 + ((c ^ swz(r)) << 3); }
};

// ---- asynchronous global -> LDS copies.  Each lane supplies its own global address; the wave's
// 64 x 16 bytes (or 64 x 4 bytes) land contiguously at the wave-uniform LDS address.  Completion is
// tracked by the wave's vmcnt counter, in issue order; nothing else waits for them, so the kernels
// below count their outstanding copies explicitly and use a bare s_barrier (no implied vmcnt(0)).
typedef __attribute__((address_space(3))) void* lds_vptr;
typedef __attribute__((address_space(1))) const void* glb_vptr;
// They are issued from inline assembly on purpose: the compiler's own model of such a copy makes
// every later LDS read of the same array wait for ALL outstanding copies (vmcnt(0)), which would
// serialise the ring.  M0 carries the LDS base and is restored afterwards.
__device__ __forceinline__ void dma16(const void* g, void* lds_wave_base) {
  const uint32_t lds = (uint32_t)(uintptr_t)(lds_vptr)lds_wave_base;
  uint32_t keep;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(keep) : "v"(g), "s"(lds) : "memory");
}
__device__ __forceinline__ void dma4(const void* g, void* lds_wave_base) {
  const uint32_t lds = (uint32_t)(uintptr_t)(lds_vptr)lds_wave_base;
  uint32_t keep;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %1, off\n\ts_mov_b32 m0, %0"
               : "=&s"(keep) : "v"(g), "s"(lds) : "memory");
}
// Same copy with the address split into a wave-uniform 64-bit base (scalar registers) and a
// per-lane unsigned 32-bit byte offset: no 64-bit vector arithmetic per copy.
__device__ __forceinline__ void dma16s(const void* uniform_base, uint32_t lane_off, void* lds_wave_base) {
  const uint32_t lds = (uint32_t)(uintptr_t)(lds_vptr)lds_wave_base;
  const uint64_t b = (uint64_t)(uintptr_t)uniform_base;
  const uint64_t sb = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(b >> 32)) << 32) |
                      (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b);
  uint32_t keep;
  asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %3\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b32 m0, %0"
               : "=&s"(keep) : "v"(lane_off), "s"(sb), "s"(lds) : "memory");
}
// Two copies with one scalar base each and a shared per-lane 32-bit byte offset (the K and the V row
// piece of one gathered key): M0 is saved and restored once around the pair.
__device__ __forceinline__ void dma16s_pair(const void* base_a, const void* base_b, uint32_t lane_off,
                                            uint32_t lds_a, uint32_t lds_b) {
  uint32_t keep;
  asm volatile(
      "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %4\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2\n\t"
      "s_mov_b32 m0, %5\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %3\n\ts_mov_b32 m0, %0"
      : "=&s"(keep)
      : "v"(lane_off), "s"(base_a), "s"(base_b), "s"(lds_a), "s"(lds_b)
      : "memory");
}
// a * b for a, b < 2^24 (one full-rate instruction; the masks fold away)
__device__ __forceinline__ uint32_t mul24(uint32_t a, uint32_t b) { return (a & 0xffffffu) * (b & 0xffffffu); }
__device__ __forceinline__ uint32_t lds_addr(const void* p) { return (uint32_t)(uintptr_t)(lds_vptr)p; }
// Reads at a 32-bit LDS byte address (kept as an integer so that a pinned register keeps its address
// space; a constant added at the call site becomes the instruction's immediate offset).
template <typename T> __device__ __forceinline__ T lds_load(uint32_t a) {
  return *(__attribute__((address_space(3))) const T*)(uintptr_t)a;
}
__device__ __forceinline__ s16x4 lds_read_tr_at(uint32_t a) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(uintptr_t)a);
}
__device__ __forceinline__ const void* uniform_ptr(const void* p) {
  const uint64_t b = (uint64_t)(uintptr_t)p;
  return (const void*)(uintptr_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(b >> 32)) << 32) |
                                  (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)b));
}
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// Pins a freshly loaded register value: the compiler must finish the load before this point, so
// it will not place its own (full) vmcnt wait at a later first use inside a copy-ring loop.
template <typename T> __device__ __forceinline__ void settle(T& v) { asm volatile("" : "+v"(v)); }

// workgroup barrier that orders LDS traffic only (the caller has waited for the copies it needs)
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// A-operand fragment of the TRANSPOSE of a row-major LDS tile: for lane (n = l % 32, hh = l / 32),
// element e of the result is tile[rowbase + 4*hh + (e % 4) + 8*(e / 4)][32*cb + n].
template <int D>
__device__ __forceinline__ bf16x8 tr_frag(const uint16_t* tile, int rowbase, int cb, int l) {
  const int l16 = l & 15, b16 = (l >> 4) & 1, hh = l >> 5;
  const int r = rowbase + 4 * hh + (l16 >> 2);
  const int c = 4 * cb + 2 * b16 + ((l16 & 3) >> 1);
  const int sub = 4 * (l16 & 1);
  const s16x4 lo = lds_read_tr(tile + TileLayout<D>::off(r, c) + sub);
  const s16x4 hi = lds_read_tr(tile + TileLayout<D>::off(r + 8, c) + sub);
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// The lane's element offsets of the fragments it reads from a swizzled tile:
//   row(ks)    row fragment (16 bytes): tile[rowbase + n][16*ks + 8*hh .. +8), rowbase a multiple of 16
//   tr(cb, q)  the two halves (q) of tr_frag(tile, rowbase, cb), rowbase a multiple of 16
// (the swizzle only looks at the low four row bits, so rowbase adds rowbase * D elements).  The
// swizzle XORs the chunk index, and the chunk bits that ks / cb select lie above the lane's own, so
// row(ks) = row(0) ^ (16 ks) and tr(cb, q) = tr(0, q) ^ (32 cb): three registers hold all of them
// and a read costs one XOR-and-add (the key-stationary kernel has no registers to spare for more).
template <int D>
struct FragOffsets {
  int row0;
  int tr0[2];
  __device__ __forceinline__ void init(int l) {
    const int n = l & 31, hh = l >> 5, l16 = l & 15, b16 = (l >> 4) & 1;
    row0 = TileLayout<D>::off(n & 15, hh) + (n & 16) * D;
    asm volatile("" : "+v"(row0));
    const int r = 4 * hh + (l16 >> 2);
    const int c = 2 * b16 + ((l16 & 3) >> 1);
    tr0[0] = TileLayout<D>::off(r, c) + 4 * (l16 & 1);
    tr0[1] = TileLayout<D>::off(r + 8, c) + 4 * (l16 & 1);
    asm volatile("" : "+v"(tr0[0]));
    asm volatile("" : "+v"(tr0[1]));
  }
  // called inside a loop: keeps the compiler from hoisting every row(ks) / tr(cb, q) out of it again
  __device__ __forceinline__ void pin() {
    asm volatile("" : "+v"(row0), "+v"(tr0[0]), "+v"(tr0[1]));
  }
  __device__ __forceinline__ int row(int ks) const { return row0 ^ (16 * ks); }
  __device__ __forceinline__ int tr(int cb, int q) const { return tr0[q] ^ (32 * cb); }
  __device__ __forceinline__ bf16x8 row_frag(const uint16_t* tile, int rowbase, int ks) const {
    return *reinterpret_cast<const bf16x8*>(tile + row(ks) + rowbase * D);
  }
  __device__ __forceinline__ bf16x8 tr_frag(const uint16_t* tile, int rowbase, int cb) const {
    const s16x4 lo = lds_read_tr(tile + tr(cb, 0) + rowbase * D);
    const s16x4 hi = lds_read_tr(tile + tr(cb, 1) + rowbase * D);
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  }
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// max(x of lane l, x of lane l ^ 32) in every lane: the two half-waves exchange their values with
// one cross-half swap (no LDS round trip).
__device__ __forceinline__ float half_swap_max(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__builtin_bit_cast(float, (unsigned)r[0]), __builtin_bit_cast(float, (unsigned)r[1]));
}
__device__ __forceinline__ float half_swap_sum(float x) {
  const unsigned u = __builtin_bit_cast(unsigned, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return __builtin_bit_cast(float, (unsigned)r[0]) + __builtin_bit_cast(float, (unsigned)r[1]);
}


__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// Launch indices read from the hardware registers directly.  fwd.hip and bwd.hip are compiled with
// IEEE mode off (maxima need no NaN quieting there); the device library's index helpers are built
// with it on and would stay out-of-line calls in such a kernel.
__device__ __forceinline__ int wg_id() { return (int)__builtin_amdgcn_workgroup_id_x(); }
__device__ __forceinline__ int thread_id() { return (int)__builtin_amdgcn_workitem_id_x(); }

// Workgroups are dealt round-robin to the chip's 8 XCDs in launch order, and each XCD has its own
// L2.  A 1-D grid of 8 * ceil(H / 8) * items_per_head workgroups is mapped so that XCD x works on
// heads x, x + 8, ...: neighbouring query blocks of a head gather almost the same keys, and the slot
// groups of a head sweep the same Q / dO tiles, so those re-reads hit in that L2.  The heads of an
// XCD take turns item by item: with items ordered from long to short the whole XCD then works from
// long to short, and its last items are the shortest ones.
__device__ __forceinline__ bool xcd_map_interleaved(int wg, int H, int items_per_head, int& h, int& item) {
  const int x = wg & 7, idx = wg >> 3, hb = (H + 7) >> 3;
  item = idx / hb;
  h = x + 8 * (idx - item * hb);
  return h < H;
}
static inline unsigned xcd_grid(int H, long items_per_head) { return (unsigned)(8l * ((H + 7) / 8) * items_per_head); }

// document of a global row: largest d with cu[d] <= t
__device__ __forceinline__ int find_doc(const int32_t* __restrict__ cu, int n_docs, int t) {
  int lo = 0, hi = n_docs;  // answer in [lo, hi)
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (cu[mid] <= t) lo = mid; else hi = mid;
  }
  return lo;
}
#endif

}  // namespace dma
