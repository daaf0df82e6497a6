// C-ABI layer: argument validation on the host, then dispatch to the kernel launchers.
#include "dfa_internal.h"

namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
bool mult8(int64_t x) { return (x & 7) == 0; }

int check_common(const dfa_shape* sh) {
  if (!sh) return DFA_ERR_NULL;
  if (sh->reserved != 0) return DFA_ERR_ARG;
  if (sh->dtype != DFA_BF16 && sh->dtype != DFA_F32) return DFA_ERR_DTYPE;
  if (sh->o_dtype != DFA_BF16 && sh->o_dtype != DFA_F32) return DFA_ERR_DTYPE;
  if (sh->h_q < 1 || sh->h_kv < 1 || sh->h_q % sh->h_kv != 0) return DFA_ERR_SHAPE;
  if (sh->h_q > 65535) return DFA_ERR_SHAPE;
  if (sh->s_q < 0 || sh->s_k < 0) return DFA_ERR_SHAPE;
  if (sh->d != 64 && sh->d != 128) return DFA_ERR_SHAPE;
  if (sh->dtype == DFA_BF16 && sh->d != 128) return DFA_ERR_SHAPE;
  if (sh->causal != 0 && sh->causal != 1) return DFA_ERR_ARG;
  if (sh->causal && sh->s_q != sh->s_k) return DFA_ERR_ARG;
  if (!(sh->scale == sh->scale) || sh->scale <= 0.f) return DFA_ERR_ARG;
  return DFA_OK;
}

bool stride_ok(int64_t sh_, int64_t ss, int d, int rows) {
  if (ss < d || !mult8(ss) || !mult8(sh_)) return false;
  // head offsets are formed in 64 bits from at most 65535 heads: keep them far from overflow
  if (sh_ < 0 || sh_ > (int64_t{1} << 40)) return false;
  // the kernels address one head's slice of a chunk with 32-bit byte offsets (fp32 at most):
  // rows * ss * 4 < 2^31, compared without forming a product that could overflow
  if (rows > 0 && ss > ((int64_t{1} << 29) - 1) / rows) return false;
  return true;
}

// head stride of an [heads, rows] fp32 vector (lse, D)
bool row_stride_ok(int64_t sh_, int rows) { return sh_ >= rows && sh_ <= (int64_t{1} << 40); }

}  // namespace

extern "C" const char* dfa_status_str(int s) {
  switch (s) {
    case DFA_OK: return "DFA_OK";
    case DFA_ERR_NULL: return "DFA_ERR_NULL: required pointer is NULL";
    case DFA_ERR_SHAPE: return "DFA_ERR_SHAPE: unsupported size, stride or alignment";
    case DFA_ERR_DTYPE: return "DFA_ERR_DTYPE: unsupported dtype";
    case DFA_ERR_ARG: return "DFA_ERR_ARG: inconsistent arguments";
    case DFA_ERR_HIP: return "DFA_ERR_HIP: HIP runtime error";
    default: return "unknown dfa_status";
  }
}

extern "C" int dfa_version(void) { return 100; }

namespace {
int chunk_fwd(const dfa_shape* sh, const void* q, const void* k, const void* v,
              void* o, float* lse, int accumulate, void* stream) {
  int rc = check_common(sh);
  if (rc != DFA_OK) return rc;
  const bool have_kv = sh->s_k > 0;   // an empty key/value chunk may come with NULL k, v
  if (!q || !o || !lse || (have_kv && (!k || !v))) return DFA_ERR_NULL;
  if (!aligned16(q) || !aligned16(o) || (have_kv && (!aligned16(k) || !aligned16(v)))) return DFA_ERR_SHAPE;
  if (!stride_ok(sh->q_stride_h, sh->q_stride_s, sh->d, sh->s_q) ||
      !stride_ok(sh->kv_stride_h, sh->kv_stride_s, sh->d, sh->s_k) ||
      !stride_ok(sh->o_stride_h, sh->o_stride_s, sh->d, sh->s_q))
    return DFA_ERR_SHAPE;
  if (!row_stride_ok(sh->lse_stride_h, sh->s_q)) return DFA_ERR_SHAPE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (sh->s_q == 0) return DFA_OK;
  if (sh->s_k == 0) return accumulate ? DFA_OK : dfa::launch_fill_empty_fwd(*sh, o, lse, st);
  if (sh->dtype == DFA_F32)
    return dfa::launch_fwd_f32(*sh, static_cast<const float*>(q), static_cast<const float*>(k),
                               static_cast<const float*>(v), o, lse, accumulate, st);
  return dfa::launch_fwd_bf16(*sh, q, k, v, o, lse, accumulate, st);
}
}  // namespace

extern "C" int dfa_chunk_fwd(const dfa_shape* sh, const void* q, const void* k, const void* v,
                             void* o, float* lse, void* stream) {
  return chunk_fwd(sh, q, k, v, o, lse, 0, stream);
}

extern "C" int dfa_chunk_fwd_acc(const dfa_shape* sh, const void* q, const void* k, const void* v,
                                 void* o, float* lse, void* stream) {
  return chunk_fwd(sh, q, k, v, o, lse, 1, stream);
}

extern "C" int dfa_merge(const dfa_merge_desc* md, void* o_a, float* lse_a,
                         const void* o_b, const float* lse_b, void* stream) {
  if (!md) return DFA_ERR_NULL;
  if (md->heads < 0 || md->rows < 0 || md->heads > 65535) return DFA_ERR_SHAPE;
  if (md->d != 64 && md->d != 128) return DFA_ERR_SHAPE;
  if (md->o_dtype != DFA_BF16 && md->o_dtype != DFA_F32) return DFA_ERR_DTYPE;
  if (!o_a || !lse_a || !o_b || !lse_b) return DFA_ERR_NULL;
  if (!aligned16(o_a) || !aligned16(o_b)) return DFA_ERR_SHAPE;
  if (!stride_ok(md->a_stride_h, md->a_stride_s, md->d, md->rows) ||
      !stride_ok(md->b_stride_h, md->b_stride_s, md->d, md->rows))
    return DFA_ERR_SHAPE;
  if (!row_stride_ok(md->lse_a_stride_h, md->rows) || !row_stride_ok(md->lse_b_stride_h, md->rows)) return DFA_ERR_SHAPE;
  if (o_a == o_b || lse_a == lse_b) return DFA_ERR_ARG;
  if (md->rows == 0 || md->heads == 0) return DFA_OK;
  return dfa::launch_merge(*md, o_a, lse_a, o_b, lse_b, static_cast<hipStream_t>(stream));
}

extern "C" int dfa_delta(const dfa_shape* sh, const void* o, const void* dO, float* delta, void* stream) {
  int rc = check_common(sh);
  if (rc != DFA_OK) return rc;
  if (!o || !dO || !delta) return DFA_ERR_NULL;
  if (!aligned16(o) || !aligned16(dO)) return DFA_ERR_SHAPE;
  if (!stride_ok(sh->q_stride_h, sh->q_stride_s, sh->d, sh->s_q) ||
      !stride_ok(sh->o_stride_h, sh->o_stride_s, sh->d, sh->s_q))
    return DFA_ERR_SHAPE;
  if (!row_stride_ok(sh->lse_stride_h, sh->s_q)) return DFA_ERR_SHAPE;
  if (sh->s_q == 0) return DFA_OK;
  return dfa::launch_delta(*sh, o, dO, delta, static_cast<hipStream_t>(stream));
}

extern "C" int dfa_chunk_bwd(const dfa_shape* sh, const void* q, const void* k, const void* v,
                             const float* lse, const float* delta, const void* dO,
                             float* dq, float* dk, float* dv, int accumulate, void* stream) {
  int rc = check_common(sh);
  if (rc != DFA_OK) return rc;
  if (!q || !k || !v || !lse || !delta || !dO) return DFA_ERR_NULL;
  // dq alone, (dk, dv) alone, or all three: a NULL output selects which gradients are computed
  if ((dk == nullptr) != (dv == nullptr)) return DFA_ERR_NULL;
  if (!dq && !dk) return DFA_ERR_NULL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(dO) || !aligned16(dq) ||
      !aligned16(dk) || !aligned16(dv))
    return DFA_ERR_SHAPE;
  if (!stride_ok(sh->q_stride_h, sh->q_stride_s, sh->d, sh->s_q) ||
      !stride_ok(sh->kv_stride_h, sh->kv_stride_s, sh->d, sh->s_k) ||
      !stride_ok(sh->dq_stride_h, sh->dq_stride_s, sh->d, sh->s_q) ||
      !stride_ok(sh->dkv_stride_h, sh->dkv_stride_s, sh->d, sh->s_k))
    return DFA_ERR_SHAPE;
  if (!row_stride_ok(sh->lse_stride_h, sh->s_q)) return DFA_ERR_SHAPE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  if (sh->s_q == 0 || sh->s_k == 0) {
    // nothing flows through an empty pair; honour "overwrite" semantics
    if (!accumulate) {
      if (sh->s_q > 0 && dq) { rc = dfa::launch_fill_zero_rows(dq, sh->h_q, sh->s_q, sh->d, sh->dq_stride_h, sh->dq_stride_s, st); if (rc) return rc; }
      if (sh->s_k > 0 && dk) {
        rc = dfa::launch_fill_zero_rows(dk, sh->h_kv, sh->s_k, sh->d, sh->dkv_stride_h, sh->dkv_stride_s, st); if (rc) return rc;
        rc = dfa::launch_fill_zero_rows(dv, sh->h_kv, sh->s_k, sh->d, sh->dkv_stride_h, sh->dkv_stride_s, st); if (rc) return rc;
      }
    }
    return DFA_OK;
  }
  if (sh->dtype == DFA_F32)
    return dfa::launch_bwd_f32(*sh, static_cast<const float*>(q), static_cast<const float*>(k),
                               static_cast<const float*>(v), lse, delta, static_cast<const float*>(dO),
                               dq, dk, dv, accumulate, st);
  return dfa::launch_bwd_bf16(*sh, q, k, v, lse, delta, dO, dq, dk, dv, accumulate, st);
}
