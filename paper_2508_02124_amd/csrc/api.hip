// Host side of the C ABI: argument validation, layout computation, dispatch.  No allocation, no
// synchronisation.  State kept between calls: the caller's array of stage events while
// dma_profile_events has one set (per host thread), nothing else in this file.
#include "common.h"

using namespace dma;

namespace dma {
static thread_local void** g_stage_events = nullptr;
void prof_begin(int stage, hipStream_t st) {
  if (g_stage_events) (void)hipEventRecord((hipEvent_t)g_stage_events[2 * stage], st);
}
void prof_end(int stage, hipStream_t st) {
  if (g_stage_events) (void)hipEventRecord((hipEvent_t)g_stage_events[2 * stage + 1], st);
}
}  // namespace dma

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// max_d: 256 everywhere except the cross-head scores (128).
int check_shape(const dma_shape* s, int max_d = 128) {
  if (!s) return DMA_EINVAL;
  if (s->T <= 0 || s->n_docs <= 0 || s->k <= 0 || s->H_q <= 0 || s->H_kv <= 0) return DMA_EINVAL;
  if (s->H_q % s->H_kv != 0) return DMA_EINVAL;
  if (s->softmax_scale < 0.f || s->softmax_scale != s->softmax_scale) return DMA_EINVAL;
  if (s->d != 64 && s->d != 128 && !(s->d == 256 && max_d >= 256)) return DMA_EUNSUPPORTED;
  if (s->dtype != DMA_BF16 && s->dtype != DMA_F32) return DMA_EUNSUPPORTED;
  if (s->H_q > 65535 || s->H_kv > 65535) return DMA_EUNSUPPORTED;
  // the score kernel holds the projection vectors of one kv-head's group in LDS, 256 bytes per q-head
  if (s->H_q / s->H_kv > 256) return DMA_EUNSUPPORTED;
  return DMA_OK;
}

// The bf16 attention kernels address a gathered K / V row as a 32-bit byte offset from the kv-head's
// first row (row index below 2^24, row pitch below 2^24, K and V at most 4 GiB each).
int check_gather_limits(const dma_shape& s) {
  if (s.dtype != DMA_BF16) return DMA_OK;
  const unsigned long long pitch = (unsigned long long)s.H_kv * s.d * 2;
  if (s.T >= (1 << 24) || pitch >= (1ull << 24) || (unsigned long long)s.T * pitch > (1ull << 32)) return DMA_EUNSUPPORTED;
  // (the key-stationary backward addresses Q / dO rows the same way: at most 4 GiB each)
  if ((unsigned long long)s.T * s.H_q * s.d * 2 > (1ull << 32)) return DMA_EUNSUPPORTED;
  return DMA_OK;
}

size_t ws_bytes_for(const dma_shape& s) {
  if (s.dtype == DMA_F32) return align_up((size_t)s.H_q * s.T * 8, 256);  // D_i in fp64
  return ws_layout(s).total;
}

Ptrs make_ptrs(const dma_shape* s, const void* mask) {
  Ptrs p;
  p.s = *s;
  p.pl = plan_layout(*s);
  p.plan = const_cast<char*>(static_cast<const char*>(mask));
  p.scale = s->softmax_scale > 0.f ? s->softmax_scale : 1.0f / sqrtf((float)s->d);
  return p;
}

}  // namespace

extern "C" {

size_t dma_mask_bytes(const dma_shape* shape) {
  if (check_shape(shape, 256) != DMA_OK) return 0;
  return plan_layout(*shape).total;
}

size_t dma_workspace_bytes(const dma_shape* shape) {
  if (check_shape(shape, 256) != DMA_OK) return 0;
  return ws_bytes_for(*shape);
}

int dma_mask_describe(const dma_shape* shape, dma_mask_layout* out) {
  int rc = check_shape(shape, 256);
  if (rc != DMA_OK) return rc;
  if (!out) return DMA_EINVAL;
  const PlanLayout L = plan_layout(*shape);
  out->block_rows = BQ; out->group_cols = SG; out->max_partial = MAXPART;
  out->nblk_cap = L.nblk_cap; out->kpad = L.kpad; out->reserved = 0;
  out->off_header = L.off_hdr; out->off_zq = L.off_zq; out->off_blocks = L.off_blk;
  out->off_slot_table = L.off_slot; out->off_partial_count = L.off_pcnt; out->off_partial_list = L.off_plist;
  out->total = L.total;
  return DMA_OK;
}

int dma_mask_gen(const dma_shape* shape, const void* V, const float* W, const float* A,
                 const int32_t* cu_seqlens, float* z, int32_t* expiry, int32_t* topk_idx,
                 void* mask, void* stream) {
  int rc = check_shape(shape, 256);
  if (rc != DMA_OK) return rc;
  if (!cu_seqlens || !z || !expiry || !mask) return DMA_EINVAL;
  if (W && (!V || !A)) return DMA_EINVAL;
  if (!aligned16(V) || !aligned16(W) || !aligned16(z) || !aligned16(expiry) || !aligned16(mask)) return DMA_EINVAL;
  Ptrs p = make_ptrs(shape, mask);
  return launch_mask_gen(p, V, W, A, cu_seqlens, z, expiry, topk_idx, (hipStream_t)stream);
}

static int check_bias(const dma_shape* s, const float* bias, int bias_heads, int bias_per_token) {
  if (!bias || !aligned16(bias)) return DMA_EINVAL;
  if (bias_heads != 1 && bias_heads != s->H_q) return DMA_EINVAL;
  if (!bias_per_token && s->max_seqlen <= 0) return DMA_EINVAL;  // the shared row's length must be stated
  return DMA_OK;
}

int dma_mask_gen_bias(const dma_shape* shape, const void* V, const float* W, const float* A,
                      const int32_t* cu_seqlens, const float* bias, int32_t bias_heads, int32_t bias_per_token,
                      float* z, int32_t* expiry, int32_t* topk_idx, void* mask, void* stream) {
  int rc = check_shape(shape, 256);
  if (rc != DMA_OK) return rc;
  if ((rc = check_bias(shape, bias, bias_heads, bias_per_token)) != DMA_OK) return rc;
  if ((rc = dma_mask_gen(shape, V, W, A, cu_seqlens, z, expiry, topk_idx, mask, stream)) != DMA_OK) return rc;
  Ptrs p = make_ptrs(shape, mask);
  return launch_bias_add(p, bias, bias_heads, bias_per_token != 0, cu_seqlens, (hipStream_t)stream);
}

int dma_bias_bwd(const dma_shape* shape, const float* dz, const int32_t* cu_seqlens, int32_t bias_heads,
                 int32_t bias_per_token, float* dbias, void* stream) {
  int rc = check_shape(shape, 256);
  if (rc != DMA_OK) return rc;
  if (!dz || !cu_seqlens || !aligned16(dz)) return DMA_EINVAL;
  if ((rc = check_bias(shape, dbias, bias_heads, bias_per_token)) != DMA_OK) return rc;
  return launch_bias_bwd(*shape, dz, bias_heads, bias_per_token != 0, cu_seqlens, dbias, (hipStream_t)stream);
}

int dma_fwd(const dma_shape* shape, const void* Q, const void* K, const void* V, const float* z,
            const int32_t* expiry, const void* mask, const int32_t* cu_seqlens,
            void* O, float* LSE, void* ws, size_t ws_bytes, void* stream) {
  (void)ws;
  (void)ws_bytes;
  int rc = check_shape(shape, 256);
  if (rc != DMA_OK) return rc;
  if (!Q || !K || !V || !z || !expiry || !mask || !cu_seqlens || !O || !LSE) return DMA_EINVAL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(z) || !aligned16(LSE) ||
      !aligned16(mask))
    return DMA_EINVAL;
  if ((rc = check_gather_limits(*shape)) != DMA_OK) return rc;
  Ptrs p = make_ptrs(shape, mask);
  if (shape->dtype == DMA_F32)
    return launch_fwd_f32(p, (const float*)Q, (const float*)K, (const float*)V, z, expiry, cu_seqlens, (float*)O, LSE,
                          (hipStream_t)stream);
  return launch_fwd(p, Q, K, V, z, expiry, cu_seqlens, O, LSE, (hipStream_t)stream);
}

int dma_bwd(const dma_shape* shape, const void* Q, const void* K, const void* V, const void* O,
            const void* dO, const float* LSE, const float* z, const int32_t* expiry,
            const void* mask, const int32_t* cu_seqlens,
            void* dQ, void* dK, void* dV, float* dz, void* ws, size_t ws_bytes, void* stream) {
  int rc = check_shape(shape, 256);
  if (rc != DMA_OK) return rc;
  if (!Q || !K || !V || !O || !dO || !LSE || !z || !expiry || !mask || !cu_seqlens || !dQ || !dK || !dV || !dz)
    return DMA_EINVAL;
  if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O) || !aligned16(dO) || !aligned16(dQ) ||
      !aligned16(dK) || !aligned16(dV) || !aligned16(dz) || !aligned16(LSE) || !aligned16(z) || !aligned16(mask) ||
      !aligned16(ws))
    return DMA_EINVAL;
  if (!ws || ws_bytes < ws_bytes_for(*shape)) return DMA_EWORKSPACE;
  if ((rc = check_gather_limits(*shape)) != DMA_OK) return rc;
  Ptrs p = make_ptrs(shape, mask);
  if (shape->dtype == DMA_F32)
    return launch_bwd_f32(p, (const float*)Q, (const float*)K, (const float*)V, (const float*)O, (const float*)dO, LSE,
                          z, expiry, cu_seqlens, (float*)dQ, (float*)dK, (float*)dV, dz, (char*)ws,
                          (hipStream_t)stream);
  return launch_bwd(p, Q, K, V, O, dO, LSE, z, expiry, cu_seqlens, dQ, dK, dV, dz, (char*)ws, (hipStream_t)stream);
}

int dma_mask_bwd(const dma_shape* shape, const void* V, const float* W, const float* A, const float* dz,
                 float* dW, float* dA, void* dV, int accumulate, void* stream) {
  int rc = check_shape(shape, 256);
  if (rc != DMA_OK) return rc;
  if (!V || !W || !A || !dz || !dW || !dA || !dV) return DMA_EINVAL;
  if (!aligned16(V) || !aligned16(W) || !aligned16(dz) || !aligned16(dW) || !aligned16(dV)) return DMA_EINVAL;
  return launch_mask_bwd(*shape, V, W, A, dz, dW, dA, dV, accumulate != 0, (hipStream_t)stream);
}

int dma_scores_xhead(const dma_shape* shape, const void* V, const float* Delta, const float* A, float* z,
                     void* stream) {
  int rc = check_shape(shape);
  if (rc != DMA_OK) return rc;
  if (!V || !Delta || !A || !z) return DMA_EINVAL;
  if (!aligned16(V) || !aligned16(Delta) || !aligned16(z)) return DMA_EINVAL;
  return launch_xhead_scores(*shape, V, Delta, A, z, (hipStream_t)stream);
}

int dma_scores_xhead_bwd(const dma_shape* shape, const void* V, const float* Delta, const float* A, const float* dz,
                         float* dDelta, float* dA, void* dV, int accumulate, void* stream) {
  int rc = check_shape(shape);
  if (rc != DMA_OK) return rc;
  if (!V || !Delta || !A || !dz || !dDelta || !dA || !dV) return DMA_EINVAL;
  if (!aligned16(V) || !aligned16(Delta) || !aligned16(dz) || !aligned16(dDelta) || !aligned16(dV)) return DMA_EINVAL;
  return launch_xhead_bwd(*shape, V, Delta, A, dz, dDelta, dA, dV, accumulate != 0, (hipStream_t)stream);
}

static size_t decode_list_bytes(const dma_shape& s) {
  const size_t kcap = (size_t)(s.k < s.T ? s.k : s.T);
  return align_up((size_t)s.n_docs * s.H_q * kcap * 4, 256);
}

size_t dma_decode_kept_bytes(const dma_shape* shape) {
  if (check_shape(shape, 256) != DMA_OK) return 0;
  return decode_list_bytes(*shape) + decode_scratch_bytes(*shape);
}

int dma_decode(const dma_shape* shape, const void* q, const void* K, const void* V, const float* z,
               const int32_t* cu_seqlens, void* o, float* lse, int32_t* kept, size_t kept_bytes, void* stream) {
  int rc = check_shape(shape, 256);
  if (rc != DMA_OK) return rc;
  if (!q || !K || !V || !z || !cu_seqlens || !o || !lse) return DMA_EINVAL;
  if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(z) || !aligned16(o) || !aligned16(kept))
    return DMA_EINVAL;
  if (!kept || kept_bytes < dma_decode_kept_bytes(shape)) return DMA_EWORKSPACE;
  const float scale = shape->softmax_scale > 0.f ? shape->softmax_scale : 1.0f / sqrtf((float)shape->d);
  return launch_decode(*shape, scale, q, K, V, z, cu_seqlens, nullptr, 0, o, lse, kept,
                       reinterpret_cast<char*>(kept) + decode_list_bytes(*shape), (hipStream_t)stream);
}

size_t dma_decode_static_scratch_bytes(const dma_shape* shape) {
  if (check_shape(shape, 256) != DMA_OK) return 0;
  return decode_scratch_bytes(*shape);
}

int dma_decode_static(const dma_shape* shape, const void* q, const void* K, const void* V, const float* z,
                      const int32_t* cu_seqlens, void* o, float* lse, int32_t* kept, void* stream) {
  int rc = check_shape(shape, 256);
  if (rc != DMA_OK) return rc;
  if (!q || !K || !V || !z || !cu_seqlens || !o || !lse || !kept) return DMA_EINVAL;
  if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(z) || !aligned16(o) || !aligned16(kept))
    return DMA_EINVAL;
  if (decode_scratch_bytes(*shape) > DMA_DECODE_STATIC_SCRATCH_BYTES) return DMA_EWORKSPACE;
  void* scratch_ptr = nullptr;
  if ((rc = decode_static_scratch(&scratch_ptr)) != DMA_OK) return rc;
  const float scale = shape->softmax_scale > 0.f ? shape->softmax_scale : 1.0f / sqrtf((float)shape->d);
  return launch_decode(*shape, scale, q, K, V, z, cu_seqlens, nullptr, 0, o, lse, kept, scratch_ptr, (hipStream_t)stream);
}

int dma_decode_step(const dma_shape* shape, const void* q, const void* K, const void* V, const float* z,
                    const int32_t* cu_seqlens, const int32_t* seq_lens, int refresh, void* o, float* lse,
                    int32_t* kept, size_t kept_bytes, void* stream) {
  int rc = check_shape(shape, 256);
  if (rc != DMA_OK) return rc;
  if (!q || !K || !V || !z || !cu_seqlens || !seq_lens || !o || !lse) return DMA_EINVAL;
  if (!aligned16(q) || !aligned16(K) || !aligned16(V) || !aligned16(z) || !aligned16(o) || !aligned16(kept))
    return DMA_EINVAL;
  if (!kept || kept_bytes < dma_decode_kept_bytes(shape)) return DMA_EWORKSPACE;
  const float scale = shape->softmax_scale > 0.f ? shape->softmax_scale : 1.0f / sqrtf((float)shape->d);
  return launch_decode(*shape, scale, q, K, V, z, cu_seqlens, seq_lens, refresh == 0, o, lse, kept,
                       reinterpret_cast<char*>(kept) + decode_list_bytes(*shape), (hipStream_t)stream);
}

void dma_profile_events(void** events) { dma::g_stage_events = events; }

const char* dma_strerror(int status) {
  switch (status) {
    case DMA_OK: return "ok";
    case DMA_EINVAL: return "invalid argument (null or misaligned pointer, non-positive size, H_q % H_kv != 0)";
    case DMA_EUNSUPPORTED: return "unsupported configuration (d must be 64, 128 or 256 -- cross-head scores: 64 or 128 --, dtype bf16 or f32; cross-head scores: at most 32 q-heads; bf16 attention: Q, K, V at most 4 GiB each, fewer than 2^24 tokens)";
    case DMA_EWORKSPACE: return "workspace missing or too small (dma_workspace_bytes, dma_decode_kept_bytes), or the shape needs more than the library-owned scratch of dma_decode_static";
    case DMA_EHIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

int dma_version(void) { return 140; }

}  // extern "C"
