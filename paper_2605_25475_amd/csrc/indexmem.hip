// libindexmem: host side of the C ABI declared in include/indexmem.h.
// Validation happens first and touches no GPU; the rest only enqueues kernels on the caller's
// stream.  No device memory is allocated here.
#include "../../include/indexmem.h"

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "im_kernels.h"
#include "im_decode.h"

struct im_handle {
  im_config cfg;
  char* ws;
  size_t ws_bytes;
  int max_live;
  bool ws_ready;
  // workspace layout (byte offsets)
  size_t off_status, off_qy, off_alpha, off_mem, off_attn, off_dpart, off_dcand, off_dqm, off_spart, off_xk, off_hspart, total;
  int mem_split, attn_chunks, dec_splits;
  // optional kernel timing (im_profile_start / im_profile_stop)
  hipEvent_t* prof_ev;
  int prof_max, prof_n, prof_span;
  char err[256];
};

#define IM_SCORE_GROUPS 8   // query groups of a scoring launch over a short cache

// Scratch of the entry point that allocates nothing (im_decode_attn_with_readout_static): a status
// word in the first 256 bytes, then the attention partials.  Every GPU the library runs on holds
// its own copy of this array, at its own address, until the process ends.  In host code the name is
// only a handle for hipGetSymbolAddress: the per-device address it returns is what kernels, fills and
// copies are given.
#define IM_STATIC_MAX_DEVICES 64
static __device__ __align__(256) unsigned char im_static_scratch[IM_STATIC_SCRATCH_BYTES];
static void* g_static_ptr[IM_STATIC_MAX_DEVICES];
static std::mutex g_static_mu;
static thread_local char g_static_err[256] = "";

namespace {

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

int set_err(im_handle* h, int code, const char* fmt, ...) {
  if (h) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(h->err, sizeof(h->err), fmt, ap);
    va_end(ap);
  }
  return code;
}

// the calling thread's error text of a call that takes no handle (im_last_error(NULL))
int static_err(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_static_err, sizeof(g_static_err), fmt, ap);
  va_end(ap);
  return code;
}

const char* config_problem(const im_config* c, int* code) {
  *code = IM_ERR_INVALID_ARG;
  if (!c) return "config is NULL";
  if (c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1) return "batch and head counts must be >= 1";
  if (c->n_q_heads % c->n_kv_heads != 0) return "n_q_heads must be a multiple of n_kv_heads";
  if (c->capacity < 1) return "capacity must be >= 1";
  if (c->n_idx_heads < 1 || c->n_idx_heads > 16) return "n_idx_heads must be in 1..16";
  if (c->gate_in_dim < 16 || c->gate_in_dim % 16 != 0) return "gate_in_dim must be a positive multiple of 16";
  if (c->n_sink < 0 || c->n_recent < 0) return "n_sink and n_recent must be >= 0";
  if ((long long)c->n_sink + c->n_recent > c->capacity) return "n_sink + n_recent exceeds capacity";
  if (c->fold_block < 32 || c->fold_block % 32 != 0) return "fold_block must be a positive multiple of 32";
  if (c->max_queries < 1) return "max_queries must be >= 1";
  if (!(c->rms_eps >= 0.f) || !(c->mem_eps > 0.f) || !(c->softmax_scale > 0.f))
    return "rms_eps >= 0, mem_eps > 0 and softmax_scale > 0 are required";
  if ((long long)c->batch * c->n_kv_heads > 65535) return "batch * n_kv_heads must be <= 65535";
  if (c->head_shared != 0 && c->head_shared != 1) return "head_shared must be 0 or 1";
  *code = IM_ERR_UNSUPPORTED;
  if (c->head_dim != IM_D) return "head_dim must be 128";
  if (c->idx_dim != (c->head_shared ? IM_DI_SHARED : IM_DI)) return "idx_dim must be 64 (16 with head_shared = 1)";
  if (c->mem_dim != IM_DM) return "mem_dim must be 128";
  if (c->n_q_heads / c->n_kv_heads > 8) return "more than 8 query heads per KV head";
  *code = IM_OK;
  return nullptr;
}

void layout(const im_config* c, im_handle* h) {
  const size_t B = c->batch, Hi = c->n_idx_heads, units = (size_t)c->batch * c->n_kv_heads;
  h->mem_split = (c->capacity + 1023) / 1024;
  if (h->mem_split < 1) h->mem_split = 1;
  if (h->mem_split > 32) h->mem_split = 32;
  h->attn_chunks = (c->capacity + IM_ATT_CHUNK - 1) / IM_ATT_CHUNK;
  size_t off = 0;
  // status word (in a 32-word slot of its own), then one newest-position word per unit
  h->off_status = off; off = align256(off + (32 + units) * sizeof(int32_t));
  h->dec_splits = (c->capacity + DEC_KEYS - 1) / DEC_KEYS + 1;   // + the last-slot record
  h->off_qy = off;     off = align256(off + B * c->max_queries * Hi * IM_DI * sizeof(double));
  h->off_alpha = off;  off = align256(off + B * c->max_queries * Hi * sizeof(double));
  h->off_mem = off;    off = align256(off + units * h->mem_split * (IM_DM * IM_D + IM_DM) * sizeof(float));
  h->off_attn = off;   off = align256(off + B * c->n_q_heads * h->attn_chunks * IM_ATT_REC * sizeof(float));
  h->off_dpart = off;  off = align256(off + units * h->dec_splits * DEC_GMAX * DEC_REC * sizeof(float));  // upper bound: G <= 8
  h->off_dcand = off;  off = align256(off + units * h->dec_splits * DEC_CAND * sizeof(uint32_t));
  h->off_dqm = off;    off = align256(off + units * DEC_GMAX * DEC_QM * sizeof(float));
  h->off_spart = off;  off = align256(off + (size_t)IM_SCORE_GROUPS * units * c->capacity * sizeof(float));
  // head_shared: U_k X of the rows of one append, fp64
  h->off_xk = off;     off = align256(off + (c->head_shared ? B * c->capacity * IM_DI_SHARED * sizeof(double) : 0));
  h->off_hspart = off; off = align256(off + (c->head_shared ? B * HS_NSC * sizeof(uint4) : 0));
  h->total = off;
}

int launch_check(im_handle* h, const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_err(h, IM_ERR_LAUNCH, "%s: %s", what, hipGetErrorString(e));
  return IM_OK;
}

int ensure_ws(im_handle* h, hipStream_t s) {
  if (h->ws_ready) return IM_OK;
  const int n_words = 32 + h->cfg.batch * h->cfg.n_kv_heads;
  k_fill_i32<<<(n_words + 255) / 256, 256, 0, s>>>((int32_t*)(h->ws + h->off_status), n_words, 0);
  int rc = launch_check(h, "workspace clear");
  if (rc == IM_OK) h->ws_ready = true;
  return rc;
}

int32_t* status_ptr(im_handle* h) { return (int32_t*)(h->ws + h->off_status); }

bool state_ok(const im_state* st) {
  return st && st->K && st->V && st->Kidx && st->pos && st->len && st->n_projected && st->M && st->b;
}
bool params_ok(const im_params* p) { return p && p->Uq && p->G && p->Uk && p->Wtheta && p->wg; }

// KV heads per set, and the number of sets (what lengths, lists and the memory state are kept per)
int heads_per_set(const im_config& c) { return c.head_shared ? c.n_kv_heads : 1; }
int n_sets(const im_config& c) { return c.batch * c.n_kv_heads / heads_per_set(c); }

#define IM_REQUIRE(cond, msg) \
  do { if (!(cond)) return set_err(h, IM_ERR_INVALID_ARG, "%s: %s", __func__, msg); } while (0)

// the tail kernel stages CHW split records per round: the smallest variant that holds the launch's
// splits (more splits than the largest variant are merged in several rounds)
template <int G>
void launch_tail(const DecArgs& a, int units, hipStream_t s) {
  // one workgroup per (unit, head) when those fit the chip once and one staging round holds the splits
  if (units * G <= 256 && a.S <= 64) {
    if (a.S <= 8) k_dec_tail_head<G, 8><<<units * G, DEC_TT, 0, s>>>(a);
    else if (a.S <= 16) k_dec_tail_head<G, 16><<<units * G, DEC_TT, 0, s>>>(a);
    else if (a.S <= 32) k_dec_tail_head<G, 32><<<units * G, DEC_TT, 0, s>>>(a);
    else k_dec_tail_head<G, 64><<<units * G, DEC_TT, 0, s>>>(a);
    return;
  }
  if constexpr (G <= 4) {
    if (a.S <= 8) k_dec_tail<G, 8><<<units, DEC_TT, 0, s>>>(a);
    else if (a.S <= 16) k_dec_tail<G, 16><<<units, DEC_TT, 0, s>>>(a);
    else k_dec_tail<G, 24><<<units, DEC_TT, 0, s>>>(a);
  } else {
    if (a.S <= 4) k_dec_tail<G, 4><<<units, DEC_TT, 0, s>>>(a);
    else if (a.S <= 8) k_dec_tail<G, 8><<<units, DEC_TT, 0, s>>>(a);
    else k_dec_tail<G, 16><<<units, DEC_TT, 0, s>>>(a);
  }
}

// C[m][n] = sum_k A[m][k] B[n][k] in fp64: matrix cores when the contraction length allows, one
// tile per wave for small products (more waves), 2 x 2 tiles per wave for large ones (less L2 traffic)
void gemm_nt(hipStream_t s, const bf16_t* A, const bf16_t* B, double* Cm, int M, int N, int Kd) {
  if (Kd % 32 != 0) {
    k_gemm_nt_f64<<<dim3((N + 63) / 64, (M + 63) / 64), 256, 0, s>>>(A, B, Cm, M, N, Kd);
  } else if (Kd % 128 == 0 && (long long)((M + 15) / 16) * ((N + 15) / 16) <= 2048) {
    k_gemm_nt_mfma_k4<<<dim3((N + 15) / 16, (M + 15) / 16), 256, 0, s>>>(A, B, Cm, M, N, Kd);
  } else if ((long long)M * N <= (1ll << 21) || N <= 16) {
    k_gemm_nt_mfma<1, 1><<<dim3((N + 31) / 32, (M + 31) / 32), 256, 0, s>>>(A, B, Cm, M, N, Kd);
  } else {
    k_gemm_nt_mfma<2, 2><<<dim3((N + 63) / 64, (M + 63) / 64), 256, 0, s>>>(A, B, Cm, M, N, Kd);
  }
}

}  // namespace

extern "C" {

size_t im_workspace_bytes(const im_config* cfg) {
  int code;
  if (config_problem(cfg, &code)) return 0;
  im_handle tmp;
  layout(cfg, &tmp);
  return tmp.total;
}

int32_t im_create(const im_config* cfg, void* workspace, size_t workspace_bytes, im_handle** out) {
  if (!out) return IM_ERR_INVALID_ARG;
  *out = nullptr;
  int code;
  if (config_problem(cfg, &code)) return code;
  im_handle* h = (im_handle*)calloc(1, sizeof(im_handle));
  if (!h) return IM_ERR_LAUNCH;
  h->cfg = *cfg;
  layout(cfg, h);
  if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < h->total) {
    free(h);
    return IM_ERR_INVALID_ARG;
  }
  h->ws = (char*)workspace;
  h->ws_bytes = workspace_bytes;
  h->max_live = cfg->capacity;
  h->ws_ready = false;
  h->err[0] = 0;
  *out = h;
  return IM_OK;
}

static void release_profile(im_handle* h) {
  if (!h->prof_ev) return;
  for (int i = 0; i < 2 * h->prof_max; ++i) (void)hipEventDestroy(h->prof_ev[i]);
  free(h->prof_ev);
  h->prof_ev = nullptr;
  h->prof_max = h->prof_n = 0;
}

void im_destroy(im_handle* h) {
  if (!h) return;
  release_profile(h);
  free(h);
}

int32_t im_profile_start(im_handle* h, int32_t max_records, int32_t span) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(max_records >= 1 && max_records <= (1 << 20), "max_records must be in 1..2^20");
  IM_REQUIRE(span >= IM_PROFILE_MAIN && span <= IM_PROFILE_PREP_AND_MAIN, "span must be one of IM_PROFILE_*");
  release_profile(h);
  h->prof_ev = (hipEvent_t*)calloc(2 * (size_t)max_records, sizeof(hipEvent_t));
  if (!h->prof_ev) return set_err(h, IM_ERR_LAUNCH, "im_profile_start: out of host memory");
  h->prof_max = max_records;
  for (int i = 0; i < 2 * max_records; ++i) {
    hipError_t e = hipEventCreate(&h->prof_ev[i]);
    if (e != hipSuccess) {
      h->prof_max = i / 2;
      release_profile(h);
      return set_err(h, IM_ERR_LAUNCH, "hipEventCreate: %s", hipGetErrorString(e));
    }
  }
  h->prof_n = 0;
  h->prof_span = span;
  return IM_OK;
}

int32_t im_stream_read(const void* src, size_t bytes, uint32_t never, void* sink, void* stream) {
  if (!src || !sink || bytes < 16 || bytes % 16 != 0 || ((uintptr_t)src & 15) != 0)
    return static_err(IM_ERR_INVALID_ARG, "im_stream_read: src / sink is NULL, or bytes / src is not a multiple of 16");
  // 8 workgroups of 4 waves per CU: 2048 workgroups, each thread 8 x 16 bytes per round
  k_stream_read<<<2048, 256, 0, (hipStream_t)stream>>>((const uint4*)src, bytes / 16, never, (uint32_t*)sink);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return static_err(IM_ERR_LAUNCH, "im_stream_read: %s", hipGetErrorString(e));
  return IM_OK;
}

int32_t im_profile_stop(im_handle* h, float* ms_host, int32_t* n_records, void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(ms_host && n_records, "ms_host / n_records is NULL");
  IM_REQUIRE(h->prof_ev, "im_profile_start was not called");
  hipError_t e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) return set_err(h, IM_ERR_LAUNCH, "stream synchronize: %s", hipGetErrorString(e));
  for (int i = 0; i < h->prof_n; ++i) {
    e = hipEventElapsedTime(&ms_host[i], h->prof_ev[2 * i], h->prof_ev[2 * i + 1]);
    if (e != hipSuccess) return set_err(h, IM_ERR_LAUNCH, "hipEventElapsedTime: %s", hipGetErrorString(e));
  }
  *n_records = h->prof_n;
  release_profile(h);
  return IM_OK;
}

const char* im_last_error(const im_handle* h) { return h ? h->err : g_static_err; }

int32_t im_set_max_live(im_handle* h, int32_t max_live) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(max_live >= 1 && max_live <= h->cfg.capacity, "max_live must be in 1..capacity");
  h->max_live = max_live;
  return IM_OK;
}

int32_t im_query_status(im_handle* h, int32_t* status_host, void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(status_host, "status_host is NULL");
  hipStream_t s = (hipStream_t)stream;
  int rc = ensure_ws(h, s);
  if (rc) return rc;
  hipError_t e = hipMemcpyAsync(status_host, status_ptr(h), sizeof(int32_t), hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return set_err(h, IM_ERR_LAUNCH, "status copy: %s", hipGetErrorString(e));
  k_fill_i32<<<1, 64, 0, s>>>(status_ptr(h), 1, 0);
  rc = launch_check(h, "status clear");
  if (rc) return rc;
  e = hipStreamSynchronize(s);
  if (e != hipSuccess) return set_err(h, IM_ERR_LAUNCH, "stream synchronize: %s", hipGetErrorString(e));
  return IM_OK;
}

int32_t im_append_kv(im_handle* h, const im_state* st, const void* k_new, const void* v_new,
                     const int32_t* pos_new, int32_t n_new, void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(state_ok(st), "state has a NULL pointer");
  IM_REQUIRE(pos_new && ((k_new && v_new) || (!k_new && !v_new)), "pos_new is NULL, or only one of k_new / v_new is");
  IM_REQUIRE(n_new >= 1 && n_new <= h->cfg.capacity, "n_new must be in 1..capacity");
  if (h->cfg.head_shared) return set_err(h, IM_ERR_UNSUPPORTED, "im_append_kv: head_shared = 1 takes im_append_kv_hidden");
  hipStream_t s = (hipStream_t)stream;
  int rc = ensure_ws(h, s);
  if (rc) return rc;
  const im_config& c = h->cfg;
  const int units = c.batch * c.n_kv_heads;
  dim3 grid((n_new * 16 + 255) / 256, units);
  k_append_rows<<<grid, 256, 0, s>>>((bf16_t*)st->K, (bf16_t*)st->V, st->pos, st->len,
                                     (const bf16_t*)k_new, (const bf16_t*)v_new, pos_new, n_new,
                                     c.n_kv_heads, 1, c.capacity);
  k_append_len<<<(units + 255) / 256, 256, 0, s>>>(st->len, units, n_new, c.capacity, status_ptr(h));
  return launch_check(h, "im_append_kv");
}

int32_t im_append_kv_hidden(im_handle* h, const im_params* p, const im_state* st, const void* k_new,
                            const void* v_new, const void* x_new, const int32_t* pos_new,
                            int32_t n_new, void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(params_ok(p), "params has a NULL pointer");
  IM_REQUIRE(state_ok(st), "state has a NULL pointer");
  IM_REQUIRE(x_new && pos_new && ((k_new && v_new) || (!k_new && !v_new)),
             "x_new / pos_new is NULL, or only one of k_new / v_new is");
  IM_REQUIRE(n_new >= 1 && n_new <= h->cfg.capacity, "n_new must be in 1..capacity");
  if (!h->cfg.head_shared) return set_err(h, IM_ERR_UNSUPPORTED, "im_append_kv_hidden: head_shared = 0 takes im_append_kv");
  hipStream_t s = (hipStream_t)stream;
  int rc = ensure_ws(h, s);
  if (rc) return rc;
  const im_config& c = h->cfg;
  const int units = c.batch * c.n_kv_heads;
  dim3 grid((n_new * 16 + 255) / 256, units);
  k_append_rows<<<grid, 256, 0, s>>>((bf16_t*)st->K, (bf16_t*)st->V, st->pos, st->len,
                                     (const bf16_t*)k_new, (const bf16_t*)v_new, pos_new, n_new,
                                     c.n_kv_heads, c.n_kv_heads, c.capacity);
  double* xk = (double*)(h->ws + h->off_xk);
  const int M = c.batch * n_new;
  if (M <= 32)
    k_gemv_nt_f64<<<IM_DI_SHARED / 2, 256, 0, s>>>((const bf16_t*)x_new, (const bf16_t*)p->Uk, xk, M, IM_DI_SHARED,
                                                   c.gate_in_dim);
  else
    gemm_nt(s, (const bf16_t*)x_new, (const bf16_t*)p->Uk, xk, M, IM_DI_SHARED, c.gate_in_dim);
  k_store_hidden_keys<<<dim3((n_new + 15) / 16, c.batch), 256, 0, s>>>(
      xk, (bf16_t*)st->Kidx, st->len, st->n_projected, (const bf16_t*)p->norm_k_w, n_new, c.capacity, c.rms_eps);
  k_append_len<<<(c.batch + 255) / 256, 256, 0, s>>>(st->len, c.batch, n_new, c.capacity, status_ptr(h));
  return launch_check(h, "im_append_kv_hidden");
}

int32_t im_index_score(im_handle* h, const im_params* p, const im_state* st, const void* q_new,
                       const void* x_gate, const int32_t* q_pos, int32_t n_q, float* scores_out,
                       void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(params_ok(p), "params has a NULL pointer");
  IM_REQUIRE(state_ok(st), "state has a NULL pointer");
  IM_REQUIRE(q_new && x_gate && q_pos && scores_out, "q_new / x_gate / q_pos / scores_out is NULL");
  IM_REQUIRE(n_q >= 1 && n_q <= h->cfg.max_queries, "n_q must be in 1..max_queries");
  hipStream_t s = (hipStream_t)stream;
  int rc = ensure_ws(h, s);
  if (rc) return rc;
  const im_config& c = h->cfg;
  const int units = n_sets(c), di = c.idx_dim;
  double* qy = (double*)(h->ws + h->off_qy);
  double* al = (double*)(h->ws + h->off_alpha);

  const int M = c.batch * n_q, Nq = c.n_idx_heads * di, Kq = c.n_q_heads * IM_D;
  const int rows = M * c.n_idx_heads;
  const double alpha_denom = sqrt((double)(c.n_idx_heads * di));
  // fewer queries than indexer heads (a decode step): the heads of a query are the scoring product's columns
  const bool few = n_q < c.n_idx_heads && c.n_idx_heads <= 16;
  if (M <= 32) {
    // a decode-size call: the key projection of the new rows and both query-side products in one launch,
    // the QK-Norm and the gate scaling in another
    const int n_proj = c.head_shared ? 0 : units;
    k_query_side_few<<<n_proj * IM_PROJ_WGS + (Nq + 1) / 2 + (c.n_idx_heads + 1) / 2, 256, 0, s>>>(
        (const bf16_t*)q_new, (const bf16_t*)p->Uq, qy, Nq, Kq, (const bf16_t*)x_gate, (const bf16_t*)p->G, al,
        c.n_idx_heads, c.gate_in_dim, M, n_proj, (const bf16_t*)st->K, (bf16_t*)st->Kidx, st->len, st->n_projected,
        (const bf16_t*)p->Uk, (const bf16_t*)p->norm_k_w, c.capacity, h->max_live, c.rms_eps, status_ptr(h));
    k_qnorm_alpha<<<(rows + 3) / 4 + (rows + 255) / 256, 256, 0, s>>>(qy, rows, di, (const bf16_t*)p->norm_q_w,
                                                                     c.rms_eps, al, rows, alpha_denom);
  } else {
    if (!c.head_shared)
      k_project_keys<<<dim3((h->max_live + 63) / 64, units), 256, 0, s>>>(
          (const bf16_t*)st->K, (bf16_t*)st->Kidx, st->len, st->n_projected, (const bf16_t*)p->Uk,
          (const bf16_t*)p->norm_k_w, c.capacity, h->max_live, c.rms_eps, status_ptr(h));
    gemm_nt(s, (const bf16_t*)q_new, (const bf16_t*)p->Uq, qy, M, Nq, Kq);
    gemm_nt(s, (const bf16_t*)x_gate, (const bf16_t*)p->G, al, M, c.n_idx_heads, c.gate_in_dim);
    k_qnorm<<<(rows + 3) / 4, 256, 0, s>>>(qy, rows, di, (const bf16_t*)p->norm_q_w, c.rms_eps);
    k_alpha_scale<<<(rows + 255) / 256, 256, 0, s>>>(al, rows, alpha_denom);
  }
  if (few) {
    const dim3 grid((h->max_live + 63) / 64, units);
    if (c.head_shared)
      k_score_few<IM_DI_SHARED><<<grid, 256, 0, s>>>((const bf16_t*)st->Kidx, st->pos, st->len, st->n_projected, qy, al,
                                                     q_pos, n_q, c.n_kv_heads / heads_per_set(c), c.capacity,
                                                     c.n_idx_heads, h->max_live, scores_out);
    else
      k_score_few<IM_DI><<<grid, 256, 0, s>>>((const bf16_t*)st->Kidx, st->pos, st->len, st->n_projected, qy, al,
                                              q_pos, n_q, c.n_kv_heads / heads_per_set(c), c.capacity,
                                              c.n_idx_heads, h->max_live, scores_out);
    return launch_check(h, "im_index_score");
  }
  // a launch over a short cache has few (256-key tile, unit) workgroups: its queries then go in up
  // to IM_SCORE_GROUPS groups with workgroups of their own (partial maxima in the workspace,
  // folded by k_score_max); a very short one also drops to 16 keys per wave
  const long long tile_wgs = (long long)((h->max_live + 255) / 256) * units;
  const bool small = tile_wgs * IM_SCORE_GROUPS < 1024;
  int groups = 1, q_per_group = n_q;
  if (tile_wgs < 1024 && n_q >= 32) {
    // (aiming at 2048 workgroups, 8 per CU: measured against 1024 at 256 and 288 tile workgroups, the
    // scoring launch is 12 % and 6 % shorter)
    const int want = (int)((2048 + tile_wgs - 1) / tile_wgs), most = (n_q + 15) / 16;
    groups = want < most ? want : most;
    if (groups > IM_SCORE_GROUPS) groups = IM_SCORE_GROUPS;
    q_per_group = ((n_q + groups - 1) / groups + 15) & ~15;
    groups = (n_q + q_per_group - 1) / q_per_group;
  }
  float* sc_out = groups > 1 ? (float*)(h->ws + h->off_spart) : scores_out;
  // (the kernel's "units" are the sets; H_kv / H_set of them belong to one batch element)
#define IM_SCORE(TPW, DI)                                                                                    \
  k_score<TPW, DI><<<dim3((h->max_live + 64 * TPW - 1) / (64 * TPW), units, groups), 256, 0, s>>>(           \
      (const bf16_t*)st->Kidx, st->pos, st->len, st->n_projected, qy, al, q_pos, n_q,                        \
      c.n_kv_heads / heads_per_set(c), c.capacity, c.n_idx_heads, h->max_live, sc_out, q_per_group)
  if (c.head_shared) { if (small) IM_SCORE(1, IM_DI_SHARED); else IM_SCORE(4, IM_DI_SHARED); }
  else { if (small) IM_SCORE(1, IM_DI); else IM_SCORE(4, IM_DI); }
#undef IM_SCORE
  if (groups > 1)
    k_score_max<<<dim3((h->max_live + 255) / 256, units), 256, 0, s>>>(sc_out, groups, st->len, c.capacity,
                                                                      h->max_live, scores_out);
  return launch_check(h, "im_index_score");
}

int32_t im_topb_select(im_handle* h, const float* scores, const im_state* st, int32_t budget,
                       int32_t* keep_idx, int32_t* evict_idx, int32_t* n_keep, int32_t* n_evict,
                       void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(state_ok(st), "state has a NULL pointer");
  IM_REQUIRE(scores && keep_idx && evict_idx && n_keep && n_evict, "an array pointer is NULL");
  IM_REQUIRE(budget >= h->cfg.n_sink + h->cfg.n_recent, "budget is below n_sink + n_recent");
  IM_REQUIRE(budget <= h->cfg.capacity, "budget exceeds capacity");
  hipStream_t s = (hipStream_t)stream;
  int rc = ensure_ws(h, s);
  if (rc) return rc;
  const im_config& c = h->cfg;
  k_select<<<n_sets(c), 1024, 0, s>>>(scores, st->pos, st->len, c.capacity, h->max_live,
                                                  budget, c.n_sink, c.n_recent, keep_idx, evict_idx,
                                                  n_keep, n_evict, status_ptr(h));
  return launch_check(h, "im_topb_select");
}

int32_t im_memory_update(im_handle* h, const im_params* p, const im_state* st,
                         const int32_t* evict_idx, const int32_t* n_evict, float lambda, float eta,
                         void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(params_ok(p), "params has a NULL pointer");
  IM_REQUIRE(state_ok(st), "state has a NULL pointer");
  IM_REQUIRE(evict_idx && n_evict, "evict_idx / n_evict is NULL");
  IM_REQUIRE(lambda > 0.f && lambda <= 1.f, "lambda must be in (0, 1]");
  IM_REQUIRE(eta > 0.f, "eta must be > 0");
  hipStream_t s = (hipStream_t)stream;
  int rc = ensure_ws(h, s);
  if (rc) return rc;
  const im_config& c = h->cfg;
  const int units = n_sets(c);
  float* part = (float*)(h->ws + h->off_mem);
  // (the partials' buffer holds mem_split records per (batch element, KV head): a set of H_kv heads has
  // one memory, so its rows can go to H_kv times as many splits; with only `batch` sets the launch needs them)
  const int n_split = c.head_shared ? h->mem_split * c.n_kv_heads : h->mem_split;
  if (c.head_shared)
    k_mem_partial_sets<<<dim3(n_split, units), 256, 0, s>>>(
        (const bf16_t*)st->K, (const bf16_t*)st->V, evict_idx, n_evict, (const bf16_t*)p->Wtheta,
        c.capacity, c.n_kv_heads, c.fold_block, n_split, part);
  else
    k_mem_partial<<<dim3(n_split, units), 256, 0, s>>>(
        (const bf16_t*)st->K, (const bf16_t*)st->V, evict_idx, n_evict, (const bf16_t*)p->Wtheta,
        c.capacity, c.fold_block, n_split, part);
  k_mem_finalize<<<dim3((IM_DM * IM_D + IM_DM + 255) / 256, units), 256, 0, s>>>(
      st->M, st->b, n_evict, part, c.fold_block, n_split, lambda, eta, (const bf16_t*)st->K,
      (const bf16_t*)st->V, evict_idx, (const bf16_t*)p->Wtheta, c.capacity, heads_per_set(c));
  return launch_check(h, "im_memory_update");
}

int32_t im_compact_kv(im_handle* h, const im_state* st, const int32_t* keep_idx, const int32_t* n_keep,
                      const int32_t* evict_idx, const int32_t* n_evict, void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(state_ok(st), "state has a NULL pointer");
  IM_REQUIRE(keep_idx && n_keep && evict_idx && n_evict, "a list pointer is NULL");
  hipStream_t s = (hipStream_t)stream;
  int rc = ensure_ws(h, s);
  if (rc) return rc;
  const im_config& c = h->cfg;
  int gx = (h->max_live + 3) / 4;
  if (gx > 64) gx = 64;
  k_compact<<<dim3(gx, c.batch * c.n_kv_heads), 256, 0, s>>>(
      (bf16_t*)st->K, (bf16_t*)st->V, (bf16_t*)st->Kidx, st->pos, st->len, st->n_projected, keep_idx,
      n_keep, evict_idx, n_evict, c.capacity, heads_per_set(c), c.idx_dim, h->max_live, status_ptr(h));
  return launch_check(h, "im_compact_kv");
}

int32_t im_gather_kept(im_handle* h, const im_state* src, const im_state* dst, int32_t dst_capacity,
                       const int32_t* keep_idx, const int32_t* n_keep, const int32_t* evict_idx,
                       const int32_t* n_evict, void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(state_ok(src) && state_ok(dst), "a state has a NULL pointer");
  IM_REQUIRE(keep_idx && n_keep && evict_idx && n_evict, "a list pointer is NULL");
  IM_REQUIRE(dst_capacity >= 1, "dst_capacity must be >= 1");
  IM_REQUIRE(src->K != dst->K && src->V != dst->V && src->Kidx != dst->Kidx && src->pos != dst->pos &&
                 src->M != dst->M && src->b != dst->b,
             "source and destination must be different buffers (im_compact_kv works in place)");
  hipStream_t s = (hipStream_t)stream;
  int rc = ensure_ws(h, s);
  if (rc) return rc;
  const im_config& c = h->cfg;
  int gx = (h->max_live + 3) / 4;
  if (gx > 64) gx = 64;
  k_gather_kept<<<dim3(gx, c.batch * c.n_kv_heads), 256, 0, s>>>(
      (const bf16_t*)src->K, (const bf16_t*)src->V, (const bf16_t*)src->Kidx, src->pos, src->len, src->M, src->b,
      (bf16_t*)dst->K, (bf16_t*)dst->V, (bf16_t*)dst->Kidx, dst->pos, dst->len, dst->n_projected, dst->M, dst->b,
      keep_idx, n_keep, evict_idx, c.capacity, dst_capacity, heads_per_set(c), c.idx_dim, h->max_live, status_ptr(h));
  return launch_check(h, "im_gather_kept");
}

// the two launches of step a5 over `part` (attention partials, attn_chunks records per query head)
static int launch_attn(const im_config& c, int max_live, const im_params* p, const im_state* st, const void* q,
                       void* out, float* readout_dbg, float* part, int attn_chunks, int32_t* status,
                       hipStream_t s) {
  const int units = c.batch * c.n_kv_heads, G = c.n_q_heads / c.n_kv_heads;
  const int H_set = c.head_shared ? c.n_kv_heads : 1;
  const int chunks = (max_live + IM_ATT_CHUNK - 1) / IM_ATT_CHUNK;
  dim3 grid(chunks, units);
#define IM_ATT_CASE(g)                                                                          \
  case g:                                                                                       \
    k_attn_partial<g><<<grid, 256, 0, s>>>((const bf16_t*)st->K, (const bf16_t*)st->V, st->len,   \
                                           (const bf16_t*)q, c.n_q_heads, c.n_kv_heads, H_set,   \
                                           c.capacity, max_live, c.softmax_scale, part,         \
                                           attn_chunks, status);                                \
    break;
  switch (G) {
    IM_ATT_CASE(1) IM_ATT_CASE(2) IM_ATT_CASE(3) IM_ATT_CASE(4)
    IM_ATT_CASE(5) IM_ATT_CASE(6) IM_ATT_CASE(7) IM_ATT_CASE(8)
    default: return IM_ERR_UNSUPPORTED;
  }
#undef IM_ATT_CASE
  k_attn_combine<<<c.batch * c.n_q_heads, 128, 0, s>>>(
      part, attn_chunks, st->len, (const bf16_t*)q, (const bf16_t*)p->Wtheta, (const bf16_t*)p->wg,
      p->cg, st->M, st->b, c.n_q_heads, c.n_kv_heads, H_set, max_live, c.mem_eps, (bf16_t*)out,
      readout_dbg);
  return IM_OK;
}

int32_t im_decode_attn_with_readout(im_handle* h, const im_params* p, const im_state* st,
                                    const void* q, void* out, float* readout_dbg, void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(params_ok(p), "params has a NULL pointer");
  IM_REQUIRE(state_ok(st), "state has a NULL pointer");
  IM_REQUIRE(q && out, "q / out is NULL");
  hipStream_t s = (hipStream_t)stream;
  int rc = ensure_ws(h, s);
  if (rc) return rc;
  rc = launch_attn(h->cfg, h->max_live, p, st, q, out, readout_dbg, (float*)(h->ws + h->off_attn),
                   h->attn_chunks, status_ptr(h), s);
  if (rc) return set_err(h, rc, "group size %d", h->cfg.n_q_heads / h->cfg.n_kv_heads);
  return launch_check(h, "im_decode_attn_with_readout");
}

static size_t static_scratch_bytes(const im_config* cfg, int32_t max_live) {
  int code;
  if (config_problem(cfg, &code) || max_live < 1 || max_live > cfg->capacity) return 0;
  const size_t chunks = ((size_t)max_live + IM_ATT_CHUNK - 1) / IM_ATT_CHUNK;
  return 256 + (size_t)cfg->batch * cfg->n_q_heads * chunks * IM_ATT_REC * sizeof(float);
}

int32_t im_decode_attn_with_readout_static(const im_config* cfg, int32_t max_live, const im_params* p,
                                           const im_state* st, const void* q, void* out,
                                           float* readout_dbg, int32_t* status_dev, void* stream) {
  // host-only validation first: an invalid call touches no GPU
  int code;
  if (const char* why = config_problem(cfg, &code)) return static_err(code, "im_decode_attn_with_readout_static: %s", why);
  if (!params_ok(p) || !state_ok(st) || !q || !out)
    return static_err(IM_ERR_INVALID_ARG, "im_decode_attn_with_readout_static: a params / state / q / out pointer is NULL");
  if (max_live < 1 || max_live > cfg->capacity)
    return static_err(IM_ERR_INVALID_ARG, "im_decode_attn_with_readout_static: max_live must be in 1..capacity");
  const size_t need = static_scratch_bytes(cfg, max_live);
  if (need > (size_t)IM_STATIC_SCRATCH_BYTES)
    return static_err(IM_ERR_INVALID_ARG,
                      "im_decode_attn_with_readout_static: batch %d x %d query heads x %d live entries need %zu bytes of "
                      "scratch, the built-in buffer holds %zu (IM_STATIC_SCRATCH_BYTES); use im_decode_attn_with_readout "
                      "with a workspace",
                      cfg->batch, cfg->n_q_heads, max_live, need, (size_t)IM_STATIC_SCRATCH_BYTES);
  // this device's copy of the scratch array: looked up once per device, with that device current
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= IM_STATIC_MAX_DEVICES)
    return static_err(IM_ERR_LAUNCH, "im_decode_attn_with_readout_static: hipGetDevice: %s (device %d)",
                      hipGetErrorString(e), dev);
  char* scratch = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ptr[dev]) {
      void* sym = nullptr;
      e = hipGetSymbolAddress(&sym, HIP_SYMBOL(im_static_scratch));
      if (e != hipSuccess || !sym)
        return static_err(IM_ERR_LAUNCH, "im_decode_attn_with_readout_static: hipGetSymbolAddress: %s",
                          hipGetErrorString(e));
      g_static_ptr[dev] = sym;
    }
    scratch = (char*)g_static_ptr[dev];
  }
  hipStream_t s = (hipStream_t)stream;
  // the buffer keeps the last call's contents.  The partial records need no clearing (every record the
  // combine reads is written by this call's first launch); the status word does when it is the sink.
  int32_t* status = status_dev ? status_dev : (int32_t*)scratch;
  if (!status_dev) k_fill_i32<<<1, 64, 0, s>>>((int32_t*)scratch, 1, 0);
  const int chunks = (max_live + IM_ATT_CHUNK - 1) / IM_ATT_CHUNK;
  const int rc = launch_attn(*cfg, max_live, p, st, q, out, readout_dbg, (float*)(scratch + 256), chunks, status, s);
  if (rc) return static_err(rc, "im_decode_attn_with_readout_static: group size %d", cfg->n_q_heads / cfg->n_kv_heads);
  e = hipGetLastError();
  if (e != hipSuccess) return static_err(IM_ERR_LAUNCH, "im_decode_attn_with_readout_static: %s", hipGetErrorString(e));
  return IM_OK;
}

static int32_t decode_launch(im_handle* h, const im_params* p, const im_state* st, const void* q,
                             const void* x_gate, const int32_t* q_pos, const void* k_new, const void* v_new,
                             const int32_t* pos_new, int32_t budget, float lambda, float eta, void* out,
                             float* readout_dbg, int32_t* evicted_slot, float* scores_dbg, void* stream,
                             const bool no_score, const int32_t* ext_evict, const char* what) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(params_ok(p), "params has a NULL pointer");
  IM_REQUIRE(state_ok(st), "state has a NULL pointer");
  IM_REQUIRE(q && k_new && v_new && pos_new && out, "an input / output pointer is NULL");
  IM_REQUIRE(no_score || (x_gate && q_pos), "x_gate / q_pos is NULL");
  IM_REQUIRE(!h->cfg.head_shared || x_gate, "the new token's hidden state is NULL");
  IM_REQUIRE(budget >= h->cfg.n_sink + h->cfg.n_recent, "budget is below n_sink + n_recent");
  IM_REQUIRE(budget <= h->cfg.capacity, "budget exceeds capacity");
  IM_REQUIRE(lambda > 0.f && lambda <= 1.f, "lambda must be in (0, 1]");
  IM_REQUIRE(eta > 0.f, "eta must be > 0");
  const im_config& c = h->cfg;
  if (c.batch > 64) return set_err(h, IM_ERR_UNSUPPORTED, "%s: batch above 64", what);
  if (c.head_shared && h->max_live > 64 * DEC_KEYS + 1)
    return set_err(h, IM_ERR_UNSUPPORTED, "%s: head_shared = 1 needs max_live <= %d", what, 64 * DEC_KEYS + 1);
  hipStream_t s = (hipStream_t)stream;
  int rc = ensure_ws(h, s);
  if (rc) return rc;
  const int units = c.batch * c.n_kv_heads, G = c.n_q_heads / c.n_kv_heads;
  int32_t* words = (int32_t*)(h->ws + h->off_status);
  DecArgs a = {};
  a.K = (bf16_t*)st->K; a.V = (bf16_t*)st->V; a.Kidx = (bf16_t*)st->Kidx;
  a.pos = st->pos; a.len = st->len; a.nproj = st->n_projected; a.M = st->M; a.bvec = st->b;
  a.Uq = (const bf16_t*)p->Uq; a.Gw = (const bf16_t*)p->G; a.Uk = (const bf16_t*)p->Uk;
  a.nqw = (const bf16_t*)p->norm_q_w; a.nkw = (const bf16_t*)p->norm_k_w;
  a.Wt = (const bf16_t*)p->Wtheta; a.wg = (const bf16_t*)p->wg; a.cg = p->cg;
  a.q = (const bf16_t*)q; a.xg = (const bf16_t*)x_gate; a.k_new = (const bf16_t*)k_new;
  a.v_new = (const bf16_t*)v_new; a.pos_new = pos_new; a.q_pos = q_pos; a.ext_evict = ext_evict;
  a.out = (bf16_t*)out; a.readout = readout_dbg; a.scores = scores_dbg; a.evicted = evicted_slot;
  a.qy = (double*)(h->ws + h->off_qy); a.alpha = (double*)(h->ws + h->off_alpha);
  a.status = words; a.maxpos = words + 32;
  a.part = (float*)(h->ws + h->off_dpart); a.cand = (uint32_t*)(h->ws + h->off_dcand);
  a.qm = (float*)(h->ws + h->off_dqm);
  a.B = c.batch; a.H = c.n_q_heads; a.H_kv = c.n_kv_heads; a.C = c.capacity; a.H_idx = c.n_idx_heads;
  a.gate_in = c.gate_in_dim; a.n_sink = c.n_sink; a.n_recent = c.n_recent; a.budget = budget;
  // 128-key splits for the main kernel; a single key beyond a multiple of 128 (the steady state with
  // a budget that is a multiple of 128) is left to the tail kernel instead of a one-key split
  a.S = (h->max_live % DEC_KEYS == 1 && h->max_live > 1) ? h->max_live / DEC_KEYS
                                                         : (h->max_live + DEC_KEYS - 1) / DEC_KEYS;
  a.S_alloc = h->dec_splits; a.max_live = h->max_live;
  a.rms_eps = c.rms_eps; a.mem_eps = c.mem_eps; a.scale = c.softmax_scale; a.lambda = lambda; a.eta = eta;
  a.hs = c.head_shared; a.H_set = heads_per_set(c); a.di = c.idx_dim; a.xk = (double*)(h->ws + h->off_xk);
  if (c.head_shared) {
    // four launches: projections + append + readout terms; the sequence's scores and decision; the
    // attention partials with that slot named; the per-(unit, head) tail
    a.hs_part = (uint4*)(h->ws + h->off_hspart);
    a.hs_evict = words + 32;   // [units]
    a.hs_named = ext_evict;    // a follower step: one slot per sequence from the caller
    a.ext_evict = a.hs_evict;
    if (c.n_kv_heads > 16) return set_err(h, IM_ERR_UNSUPPORTED, "%s: head_shared = 1 with more than 16 KV heads", what);
    a.attend = no_score ? 1 : 0;   // attend-only: U_k alone in the prep launch, no scoring launch
    const int hs_prep_blocks = (1 + DEC_MP) * units + IM_DI_SHARED / 2 +
                               (no_score ? 0 : c.n_idx_heads * IM_DI_SHARED / 2 + (c.n_idx_heads + 1) / 2);
    const int hs_main_blocks = units * (a.S > 0 ? a.S : 1);
    const bool hprof = h->prof_ev && h->prof_n < h->prof_max;
    hipEvent_t hev0 = hprof ? h->prof_ev[2 * h->prof_n] : nullptr, hev1 = hprof ? h->prof_ev[2 * h->prof_n + 1] : nullptr;
    // an attend-only or follower step has nothing between its projections and its attention: the prep
    // roles ride in the attention launch (two launches in all)
    const bool merged = no_score;
    if (hprof && (merged || h->prof_span != IM_PROFILE_MAIN)) (void)hipEventRecord(hev0, s);
    if (!merged) {
      k_hs_prep<<<hs_prep_blocks, 256, 0, s>>>(a);
      k_hs_score<<<c.batch * HS_NSC, HS_ST, 0, s>>>(a);
      if (hprof && h->prof_span == IM_PROFILE_MAIN) (void)hipEventRecord(hev0, s);
      if (hprof && h->prof_span == IM_PROFILE_PREP) (void)hipEventRecord(hev1, s);
    }
#define IM_HS_CASE(g)                                                                  \
  case g:                                                                              \
    if (merged) k_att_merged<g><<<hs_prep_blocks + hs_main_blocks, DEC_MT / 2, 0, s>>>(a, hs_prep_blocks); \
    else k_att_main<g><<<hs_main_blocks, DEC_MT / 2, 0, s>>>(a);                       \
    if (hprof && (merged || h->prof_span != IM_PROFILE_PREP)) (void)hipEventRecord(hev1, s); \
    if (a.S <= 8) k_dec_tail_head<g, 8><<<units * g, DEC_TT, 0, s>>>(a);               \
    else if (a.S <= 16) k_dec_tail_head<g, 16><<<units * g, DEC_TT, 0, s>>>(a);        \
    else if (a.S <= 32) k_dec_tail_head<g, 32><<<units * g, DEC_TT, 0, s>>>(a);        \
    else k_dec_tail_head<g, 64><<<units * g, DEC_TT, 0, s>>>(a);                       \
    break;
    switch (G) {
      IM_HS_CASE(1) IM_HS_CASE(2) IM_HS_CASE(3) IM_HS_CASE(4)
      IM_HS_CASE(5) IM_HS_CASE(6) IM_HS_CASE(7) IM_HS_CASE(8)
      default: return set_err(h, IM_ERR_UNSUPPORTED, "group size %d", G);
    }
#undef IM_HS_CASE
    if (hprof) h->prof_n++;
    return launch_check(h, what);
  }
  // the per-unit blocks come first in the prep kernel's block order: an attend-only step launches
  // just those (no query-side indexer projections)
  const int row_pairs = c.n_idx_heads * IM_DI / 2 + (c.n_idx_heads + 1) / 2;
  // projection blocks take 4 batch rows each (a shorter chain per block) while the grid then still is
  // one generation of workgroups (4 per CU), else 8
  const int prep_rows = (row_pairs * ((c.batch + 3) / 4) + (1 + DEC_MP) * units <= 4 * 256) ? 4 : 8;
  const int prep_blocks = (no_score ? 0 : row_pairs * ((c.batch + prep_rows - 1) / prep_rows)) + (1 + DEC_MP) * units;
  const int main_blocks = units * (a.S > 0 ? a.S : 1);
  const bool prof = h->prof_ev && h->prof_n < h->prof_max;
  hipEvent_t ev0 = prof ? h->prof_ev[2 * h->prof_n] : nullptr, ev1 = prof ? h->prof_ev[2 * h->prof_n + 1] : nullptr;
  // a step that scores nothing has nothing between its prep roles and its attention: they share a
  // launch (a follower's tail then takes the moved entry's indexer key from the cache, where the
  // launch's unit block has put the new token's, instead of from the last-slot record)
  const bool merged = no_score;
  a.kidx_in_cache = (merged && ext_evict) ? 1 : 0;
  if (prof && (merged || h->prof_span != IM_PROFILE_MAIN)) (void)hipEventRecord(ev0, s);
  if (!merged) {
    if (prep_rows == 4) k_dec_prep<4><<<prep_blocks, 256, 0, s>>>(a);
    else k_dec_prep<8><<<prep_blocks, 256, 0, s>>>(a);
    if (prof && h->prof_span == IM_PROFILE_MAIN) (void)hipEventRecord(ev0, s);
    if (prof && h->prof_span == IM_PROFILE_PREP) (void)hipEventRecord(ev1, s);
  }
#define IM_DEC_CASE(g)                                              \
  case g:                                                           \
    if (merged) k_att_merged<g><<<prep_blocks + main_blocks, DEC_MT / 2, 0, s>>>(a, prep_blocks); \
    else if (no_score) k_att_main<g><<<main_blocks, DEC_MT / 2, 0, s>>>(a); \
    else k_dec_main<g><<<main_blocks, DEC_MT, 0, s>>>(a, a.qy, a.alpha); \
    if (prof && (merged || h->prof_span != IM_PROFILE_PREP)) (void)hipEventRecord(ev1, s); \
    launch_tail<g>(a, units, s);                                    \
    break;
  switch (G) {
    IM_DEC_CASE(1) IM_DEC_CASE(2) IM_DEC_CASE(3) IM_DEC_CASE(4)
    IM_DEC_CASE(5) IM_DEC_CASE(6) IM_DEC_CASE(7) IM_DEC_CASE(8)
    default: return set_err(h, IM_ERR_UNSUPPORTED, "group size %d", G);
  }
#undef IM_DEC_CASE
  if (prof) h->prof_n++;
  return launch_check(h, what);
}

int32_t im_decode_step(im_handle* h, const im_params* p, const im_state* st, const void* q,
                       const void* x_gate, const int32_t* q_pos, const void* k_new, const void* v_new,
                       const int32_t* pos_new, int32_t budget, float lambda, float eta, void* out,
                       float* readout_dbg, int32_t* evicted_slot, float* scores_dbg, void* stream) {
  return decode_launch(h, p, st, q, x_gate, q_pos, k_new, v_new, pos_new, budget, lambda, eta, out,
                       readout_dbg, evicted_slot, scores_dbg, stream, false, nullptr, "im_decode_step");
}

int32_t im_attend_step(im_handle* h, const im_params* p, const im_state* st, const void* q,
                       const void* k_new, const void* v_new, const int32_t* pos_new, void* out,
                       float* readout_dbg, void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  // budget = capacity: no unit can be above it, so nothing is evicted; lambda, eta are unused
  if (h->cfg.head_shared) return set_err(h, IM_ERR_UNSUPPORTED, "im_attend_step: head_shared = 1 takes im_attend_step_hidden");
  return decode_launch(h, p, st, q, nullptr, nullptr, k_new, v_new, pos_new, h->cfg.capacity, 1.f, 1.f, out,
                       readout_dbg, nullptr, nullptr, stream, true, nullptr, "im_attend_step");
}

int32_t im_attend_step_hidden(im_handle* h, const im_params* p, const im_state* st, const void* q,
                              const void* x_new, const void* k_new, const void* v_new,
                              const int32_t* pos_new, void* out, float* readout_dbg, void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  if (!h->cfg.head_shared) return set_err(h, IM_ERR_UNSUPPORTED, "im_attend_step_hidden: head_shared = 0 takes im_attend_step");
  return decode_launch(h, p, st, q, x_new, nullptr, k_new, v_new, pos_new, h->cfg.capacity, 1.f, 1.f, out,
                       readout_dbg, nullptr, nullptr, stream, true, nullptr, "im_attend_step_hidden");
}

int32_t im_decode_step_shared(im_handle* h, const im_params* p, const im_state* st, const void* q,
                              const void* k_new, const void* v_new, const int32_t* pos_new,
                              const int32_t* evict_slot, float lambda, float eta, void* out,
                              float* readout_dbg, void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(evict_slot, "evict_slot is NULL");
  if (h->cfg.head_shared) return set_err(h, IM_ERR_UNSUPPORTED, "im_decode_step_shared: head_shared = 1 takes im_decode_step_shared_hidden");
  return decode_launch(h, p, st, q, nullptr, nullptr, k_new, v_new, pos_new, h->cfg.capacity, lambda, eta, out,
                       readout_dbg, nullptr, nullptr, stream, true, evict_slot, "im_decode_step_shared");
}

int32_t im_decode_step_shared_hidden(im_handle* h, const im_params* p, const im_state* st, const void* q,
                                     const void* x_new, const void* k_new, const void* v_new,
                                     const int32_t* pos_new, const int32_t* evict_slot, float lambda,
                                     float eta, void* out, float* readout_dbg, void* stream) {
  if (!h) return IM_ERR_INVALID_ARG;
  IM_REQUIRE(evict_slot, "evict_slot is NULL");
  if (!h->cfg.head_shared) return set_err(h, IM_ERR_UNSUPPORTED, "im_decode_step_shared_hidden: head_shared = 0 takes im_decode_step_shared");
  return decode_launch(h, p, st, q, x_new, nullptr, k_new, v_new, pos_new, h->cfg.capacity, lambda, eta, out,
                       readout_dbg, nullptr, nullptr, stream, true, evict_slot, "im_decode_step_shared_hidden");
}

}  // extern "C"
