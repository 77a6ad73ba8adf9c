// C ABI of the pruning stage (see include/asap.h): host-side validation and dispatch only.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "asap_launch.hpp"

// Scratch of asap_score_static: one array per GPU, part of the library's code object, so that the
// call needs no allocation and no workspace from the caller.  In host code the name stands for the
// symbol only; the device address is asked for once per device (scratch_for_device) and that pointer
// is what the launches get.
static __device__ __align__(256) unsigned char scratch[ASAP_STATIC_SCRATCH_BYTES];

struct asap_ctx {
  int device;
  void* static_scratch;   // device address of `scratch` on this context's GPU; null if the query failed
  hipError_t static_scratch_err;
  char err[512];
  asap::Timer* timer;   // non-null while kernel timing is on
  hipStream_t side;     // second stream of asap_stage and its fork / join events; made on first use
  hipEvent_t ev_start, ev_fork, ev_join;
};

namespace {

using namespace asap;

asap_status fail(asap_ctx* ctx, asap_status st, const char* fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return st;
}

// Address of `scratch` on `device`, asked for once per device with that device current.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];
bool g_scratch_known[kMaxDevices];

hipError_t scratch_for_device(int device, void** out) {
  *out = nullptr;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_known[device]) {
    *out = g_scratch_ptr[device];
    return hipSuccess;
  }
  int prev = -1;
  hipError_t e = hipGetDevice(&prev);
  if (e != hipSuccess) return e;
  if (prev != device && (e = hipSetDevice(device)) != hipSuccess) return e;
  void* ptr = nullptr;
  e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
  if (prev != device) {
    hipError_t e2 = hipSetDevice(prev);
    if (e == hipSuccess) e = e2;
  }
  if (e != hipSuccess) return e;
  if (ptr == nullptr) return hipErrorInvalidSymbol;
  g_scratch_ptr[device] = ptr;
  g_scratch_known[device] = true;
  *out = ptr;
  return hipSuccess;
}

bool valid_dtype(asap_dtype t) { return t == ASAP_F32 || t == ASAP_BF16; }
int dtype_size(asap_dtype t) { return t == ASAP_BF16 ? 2 : 4; }

asap_status check_params(const asap_params* p, char* msg, size_t n) {
#define BAD(cond, text)                                  \
  if (cond) {                                            \
    if (msg && n) snprintf(msg, n, "%s", text);          \
    return ASAP_EINVAL;                                  \
  }
  BAD(p == nullptr, "params is NULL");
  BAD(p->B < 1, "B must be >= 1");
  BAD(p->H < 1 || p->Hkv < 1 || p->H % p->Hkv != 0, "H must be a positive multiple of Hkv");
  BAD(p->d != 64 && p->d != 128, "d must be 64 or 128");
  BAD((int64_t)p->Hkv * p->d > 8192, "Hkv * d must be <= 8192");
  BAD(p->D < 64 || p->D % 64 != 0 || p->D > 8192, "D must be a multiple of 64 in [64, 8192]");
  BAD(p->P < 0 || p->P > (1 << 20), "P must be in [0, 1048576]");
  BAD(p->V < 1 || p->V > 16384, "V must be in [1, 16384]");
  BAD(p->Tmax < 1 || p->Tmax > 128, "Tmax must be in [1, 128]");
  BAD(p->k < 1 || p->k > p->V, "k must be in [1, V]");
  BAD(!valid_dtype(p->qk_dtype) || !valid_dtype(p->h_dtype) || !valid_dtype(p->kv_dtype), "unknown dtype");
  BAD(!(p->lambda_max > 0.0f && p->lambda_max <= 1.0f), "lambda_max must be in (0, 1]");
  BAD(!(p->eps > 0.0f) || !isfinite(p->eps), "eps must be positive and finite");
  BAD(isnan(p->sim_threshold), "sim_threshold is NaN");
  BAD(!(p->merge_weight >= 0.0f) || !isfinite(p->merge_weight), "merge_weight must be finite and >= 0");
  BAD(p->mask_mode != ASAP_MASK_OFF && p->mask_mode != ASAP_MASK_KEYBIAS, "unknown mask_mode");
  BAD(p->route != ASAP_ROUTE_ABSORB && p->route != ASAP_ROUTE_PAPER, "unknown route");
  BAD(p->score_rows != ASAP_ROWS_ALL && p->score_rows != ASAP_ROWS_LAST, "unknown score_rows");
  BAD(p->route == ASAP_ROUTE_PAPER && 2 * (int64_t)p->k > p->V, "ASAP_ROUTE_PAPER needs k <= V / 2 (the vacated slots are refilled from the pruned tokens)");
  BAD((int64_t)p->B * p->Hkv > 65535 || (int64_t)p->B * p->H > 65535, "B * heads must be <= 65535");
#undef BAD
  if (msg && n) msg[0] = 0;
  return ASAP_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

asap_status common_checks(asap_ctx* ctx, const asap_params* p) {
  if (!ctx) return ASAP_EINVAL;
  ctx->err[0] = 0;
  char msg[128];
  asap_status st = check_params(p, msg, sizeof(msg));
  if (st != ASAP_OK) return fail(ctx, st, "invalid parameters: %s", msg);
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(ctx, ASAP_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
  if (dev != ctx->device)
    return fail(ctx, ASAP_EINVAL, "current device %d is not the context's device %d", dev, ctx->device);
  return ASAP_OK;
}

asap_status check_strides(asap_ctx* ctx, const char* name, const int64_t* s, int n, int unit) {
  if (!s) return fail(ctx, ASAP_EINVAL, "%s is NULL", name);
  for (int i = 0; i < n; ++i)
    if (s[i] < 0 || s[i] % unit != 0)
      return fail(ctx, ASAP_EINVAL, "%s[%d] = %lld must be a non-negative multiple of %d elements", name, i,
                  (long long)s[i], unit);
  return ASAP_OK;
}

// The kernels address the rows of one (image, head) block -- or of one image's hidden states --
// with 32-bit byte offsets: the block, rows * stride elements of esz bytes, must stay below 2 GiB.
asap_status check_span(asap_ctx* ctx, const char* name, int64_t rows, int64_t row_stride, int64_t esz) {
  if (rows * row_stride * esz >= ((int64_t)1 << 31))
    return fail(ctx, ASAP_EUNSUPPORTED, "%s: %lld rows at a stride of %lld elements span 2 GiB or more", name,
                (long long)rows, (long long)row_stride);
  return ASAP_OK;
}

asap_status check_workspace(asap_ctx* ctx, size_t need, const void* ws, size_t bytes) {
  if (need == 0) return ASAP_OK;
  if (!ws) return fail(ctx, ASAP_EINVAL, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(ws) & 255u) return fail(ctx, ASAP_EINVAL, "workspace is not 256-byte aligned");
  if (bytes < need)
    return fail(ctx, ASAP_EWORKSPACE, "workspace of %zu bytes is smaller than the %zu required", bytes, need);
  return ASAP_OK;
}

asap_status hip_result(asap_ctx* ctx, hipError_t e, const char* what) {
  if (e == hipSuccess) return ASAP_OK;
  return fail(ctx, ASAP_EHIP, "%s: %s", what, hipGetErrorString(e));
}

}  // namespace

extern "C" {

asap_status asap_create(asap_ctx** out_ctx, int device) {
  if (!out_ctx) return ASAP_EINVAL;
  *out_ctx = nullptr;
  int count = 0;
  if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return ASAP_EINVAL;
  hipDeviceProp_t prop;
  if (hipGetDeviceProperties(&prop, device) != hipSuccess) return ASAP_EHIP;
  if (strncmp(prop.gcnArchName, "gfx950", 6) != 0) return ASAP_EUNSUPPORTED;
  asap_ctx* c = new (std::nothrow) asap_ctx;
  if (!c) return ASAP_EHIP;
  c->device = device;
  c->static_scratch_err = scratch_for_device(device, &c->static_scratch);   // reported by asap_score_static
  c->err[0] = 0;
  c->timer = nullptr;
  c->side = nullptr;
  c->ev_start = c->ev_fork = c->ev_join = nullptr;
  *out_ctx = c;
  return ASAP_OK;
}

static void drop_timer(asap_ctx* ctx) {
  if (!ctx->timer) return;
  for (int i = 0; i < ctx->timer->n_created; ++i) {
    (void)hipEventDestroy(ctx->timer->rec[i].start);
    (void)hipEventDestroy(ctx->timer->rec[i].stop);
  }
  delete ctx->timer;
  ctx->timer = nullptr;
}

static void drop_stage_resources(asap_ctx* ctx) {
  if (ctx->ev_start) (void)hipEventDestroy(ctx->ev_start);
  if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
  if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
  if (ctx->side) (void)hipStreamDestroy(ctx->side);
  ctx->side = nullptr;
  ctx->ev_start = ctx->ev_fork = ctx->ev_join = nullptr;
}

void asap_destroy(asap_ctx* ctx) {
  if (!ctx) return;
  drop_timer(ctx);
  drop_stage_resources(ctx);
  delete ctx;
}

asap_status asap_timing_enable(asap_ctx* ctx, int32_t max_launches) {
  if (!ctx) return ASAP_EINVAL;
  drop_timer(ctx);
  if (max_launches <= 0) return ASAP_OK;
  if (max_launches > asap::Timer::kMaxRecords) max_launches = asap::Timer::kMaxRecords;
  asap::Timer* t = new (std::nothrow) asap::Timer;
  if (!t) return fail(ctx, ASAP_EHIP, "asap_timing_enable: out of host memory");
  ctx->timer = t;
  for (int i = 0; i < max_launches; ++i) {
    hipError_t e = hipEventCreate(&t->rec[i].start);
    if (e == hipSuccess) {
      e = hipEventCreate(&t->rec[i].stop);
      if (e != hipSuccess) (void)hipEventDestroy(t->rec[i].start);
    }
    if (e != hipSuccess) {
      drop_timer(ctx);
      return fail(ctx, ASAP_EHIP, "asap_timing_enable: hipEventCreate: %s", hipGetErrorString(e));
    }
    t->n_created = i + 1;
  }
  return ASAP_OK;
}

int32_t asap_timing_collect(asap_ctx* ctx, char* names, size_t names_len, double* total_ms, int32_t* launches,
                            int32_t max_kernels) {
  if (!ctx || !ctx->timer || !names || !total_ms || !launches || max_kernels < 1) return -1;
  asap::Timer* t = ctx->timer;
  const char* seen[64];
  int n_seen = 0;
  size_t used = 0;
  if (names_len) names[0] = 0;
  for (int i = 0; i < t->n_used; ++i) {
    if (hipEventSynchronize(t->rec[i].stop) != hipSuccess) return -1;
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, t->rec[i].start, t->rec[i].stop) != hipSuccess) return -1;
    int slot = -1;
    for (int j = 0; j < n_seen; ++j)
      if (seen[j] == t->rec[i].name || strcmp(seen[j], t->rec[i].name) == 0) { slot = j; break; }
    if (slot < 0) {
      if (n_seen >= max_kernels || n_seen >= 64) continue;
      size_t len = strlen(t->rec[i].name);
      if (used + len + 2 > names_len) continue;
      memcpy(names + used, t->rec[i].name, len);
      names[used + len] = '\n';
      names[used + len + 1] = 0;
      used += len + 1;
      slot = n_seen++;
      seen[slot] = t->rec[i].name;
      total_ms[slot] = 0.0;
      launches[slot] = 0;
    }
    total_ms[slot] += (double)ms;
    launches[slot] += 1;
  }
  t->n_used = 0;
  return n_seen;
}

const char* asap_last_error(const asap_ctx* ctx) { return ctx ? ctx->err : "null context"; }

asap_status asap_check_params(const asap_params* p, char* msg, size_t msg_len) {
  return check_params(p, msg, msg_len);
}

size_t asap_workspace_bytes(const asap_params* p) {
  if (check_params(p, nullptr, 0) != ASAP_OK) return 0;
  size_t a = score_workspace(*p).total, b = paper_workspace_bytes(*p) + sim_workspace_bytes(*p);
  return a > b ? a : b;
}

static asap_status score_checks(asap_ctx* ctx, const asap_params* p, const void* q_vis,
                                const int64_t q_vis_stride[3], const void* q_txt, const int64_t q_txt_stride[3],
                                const void* k_vis, const int64_t k_vis_stride[3], const int32_t* text_len,
                                float* s_raw, float* s_hat, float* score, void* workspace, size_t workspace_bytes,
                                size_t workspace_need) {
  asap_status st = common_checks(ctx, p);
  if (st != ASAP_OK) return st;
  if (!q_vis || !q_txt || !k_vis || !text_len || !s_raw || !s_hat || !score)
    return fail(ctx, ASAP_EINVAL, "asap_score: a required pointer is NULL");
  if (!aligned16(q_vis) || !aligned16(q_txt) || !aligned16(k_vis))
    return fail(ctx, ASAP_EINVAL, "asap_score: q_vis, q_txt and k_vis must be 16-byte aligned");
  if ((st = check_strides(ctx, "q_vis_stride", q_vis_stride, 3, 8)) != ASAP_OK) return st;
  if ((st = check_strides(ctx, "q_txt_stride", q_txt_stride, 3, 8)) != ASAP_OK) return st;
  if ((st = check_strides(ctx, "k_vis_stride", k_vis_stride, 3, 8)) != ASAP_OK) return st;
  if (q_vis_stride[2] < p->d || q_txt_stride[2] < p->d || k_vis_stride[2] < p->d)
    return fail(ctx, ASAP_EINVAL, "asap_score: row strides must be >= d");
  const int64_t esz = dtype_size(p->qk_dtype);
  if ((st = check_span(ctx, "q_vis", p->V, q_vis_stride[2], esz)) != ASAP_OK) return st;
  if ((st = check_span(ctx, "q_txt", p->Tmax, q_txt_stride[2], esz)) != ASAP_OK) return st;
  if ((st = check_span(ctx, "k_vis", p->V, k_vis_stride[2], esz)) != ASAP_OK) return st;
  return check_workspace(ctx, workspace_need, workspace, workspace_bytes);
}

asap_status asap_score(asap_ctx* ctx, const asap_params* p, const void* q_vis, const int64_t q_vis_stride[3],
                       const void* q_txt, const int64_t q_txt_stride[3], const void* k_vis,
                       const int64_t k_vis_stride[3], const int32_t* text_len, const float* lse_extra,
                       float* s_raw, float* s_hat, float* score, void* workspace, size_t workspace_bytes,
                       void* stream) {
  asap_status st = score_checks(ctx, p, q_vis, q_vis_stride, q_txt, q_txt_stride, k_vis, k_vis_stride, text_len,
                                s_raw, s_hat, score, workspace, workspace_bytes, asap_workspace_bytes(p));
  if (st != ASAP_OK) return st;
  Strides3 qv{q_vis_stride[0], q_vis_stride[1], q_vis_stride[2]};
  Strides3 qt{q_txt_stride[0], q_txt_stride[1], q_txt_stride[2]};
  Strides3 kv{k_vis_stride[0], k_vis_stride[1], k_vis_stride[2]};
  return hip_result(ctx,
                    launch_score(*p, q_vis, qv, q_txt, qt, k_vis, kv, text_len, lse_extra, s_raw, s_hat, score,
                                 nullptr, nullptr, nullptr, nullptr, static_cast<char*>(workspace), ~size_t(0),
                                 static_cast<hipStream_t>(stream), ctx->timer),
                    "asap_score launch");
}

size_t asap_front_end_workspace_bytes(const asap_params* p) {
  if (check_params(p, nullptr, 0) != ASAP_OK) return 0;
  return score_workspace(*p).total + front_workspace_bytes(*p);
}

asap_status asap_score_from_hidden(asap_ctx* ctx, const asap_params* p, const void* hidden,
                                   const int64_t hidden_stride[2], const void* w_q, double rope_theta,
                                   const int32_t* vis_positions, const void* q_txt, const int64_t q_txt_stride[3],
                                   const void* k_vis, const int64_t k_vis_stride[3], const int32_t* text_len,
                                   const float* lse_extra, float* s_raw, float* s_hat, float* score, void* workspace,
                                   size_t workspace_bytes, void* stream) {
  asap_status st = common_checks(ctx, p);
  if (st != ASAP_OK) return st;
  if (!hidden || !w_q || !q_txt || !k_vis || !text_len || !s_raw || !s_hat || !score)
    return fail(ctx, ASAP_EINVAL, "asap_score_from_hidden: a required pointer is NULL");
  if (!aligned16(hidden) || !aligned16(w_q) || !aligned16(q_txt) || !aligned16(k_vis))
    return fail(ctx, ASAP_EINVAL, "asap_score_from_hidden: hidden, w_q, q_txt and k_vis must be 16-byte aligned");
  if (!(rope_theta > 1.0) || !isfinite(rope_theta))
    return fail(ctx, ASAP_EINVAL, "asap_score_from_hidden: rope_theta must be finite and > 1");
  if ((st = check_strides(ctx, "hidden_stride", hidden_stride, 2, 8)) != ASAP_OK) return st;
  if ((st = check_strides(ctx, "q_txt_stride", q_txt_stride, 3, 8)) != ASAP_OK) return st;
  if ((st = check_strides(ctx, "k_vis_stride", k_vis_stride, 3, 8)) != ASAP_OK) return st;
  if (hidden_stride[1] < p->D || q_txt_stride[2] < p->d || k_vis_stride[2] < p->d)
    return fail(ctx, ASAP_EINVAL, "asap_score_from_hidden: row strides must cover a row");
  const int64_t esz = dtype_size(p->qk_dtype);
  if ((st = check_span(ctx, "q_txt", p->Tmax, q_txt_stride[2], esz)) != ASAP_OK) return st;
  if ((st = check_span(ctx, "k_vis", p->V, k_vis_stride[2], esz)) != ASAP_OK) return st;
  const size_t need = asap_front_end_workspace_bytes(p);
  if (!workspace) return fail(ctx, ASAP_EINVAL, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(workspace) & 255u) return fail(ctx, ASAP_EINVAL, "workspace is not 256-byte aligned");
  if (workspace_bytes < need)
    return fail(ctx, ASAP_EWORKSPACE, "asap_score_from_hidden: workspace of %zu bytes, %zu needed", workspace_bytes, need);
  char* ws = static_cast<char*>(workspace);
  FrontArgs fe;
  fe.hidden = hidden; fe.hsb = hidden_stride[0]; fe.hsr = hidden_stride[1]; fe.wq = w_q; fe.rope_theta = rope_theta;
  fe.vis_positions = vis_positions; fe.ws = ws + score_workspace(*p).total;
  Strides3 none{0, 0, 0};
  Strides3 qt{q_txt_stride[0], q_txt_stride[1], q_txt_stride[2]};
  Strides3 kv{k_vis_stride[0], k_vis_stride[1], k_vis_stride[2]};
  return hip_result(ctx,
                    launch_score(*p, nullptr, none, q_txt, qt, k_vis, kv, text_len, lse_extra, s_raw, s_hat, score,
                                 nullptr, nullptr, &fe, nullptr, ws, ~size_t(0), static_cast<hipStream_t>(stream),
                                 ctx->timer),
                    "asap_score_from_hidden launch");
}

asap_status asap_score_static(asap_ctx* ctx, const asap_params* p, const void* q_vis,
                              const int64_t q_vis_stride[3], const void* q_txt, const int64_t q_txt_stride[3],
                              const void* k_vis, const int64_t k_vis_stride[3], const int32_t* text_len,
                              const float* lse_extra, float* s_raw, float* s_hat, float* score, void* stream) {
  if (!ctx) return ASAP_EINVAL;
  ctx->err[0] = 0;
  char msg[128];
  asap_status st = check_params(p, msg, sizeof(msg));
  if (st != ASAP_OK) return fail(ctx, st, "invalid parameters: %s", msg);
  const size_t need = score_workspace(*p, ASAP_STATIC_SCRATCH_BYTES).total;
  if (need > (size_t)ASAP_STATIC_SCRATCH_BYTES)
    return fail(ctx, ASAP_EWORKSPACE,
                "asap_score_static: these parameters need %zu bytes of scratch, the built-in array holds %zu; "
                "use asap_score with a workspace",
                need, (size_t)ASAP_STATIC_SCRATCH_BYTES);
  if (!ctx->static_scratch)
    return fail(ctx, ASAP_EHIP, "asap_score_static: address of the built-in scratch array: %s",
                hipGetErrorString(ctx->static_scratch_err));
  st = score_checks(ctx, p, q_vis, q_vis_stride, q_txt, q_txt_stride, k_vis, k_vis_stride, text_len, s_raw, s_hat,
                    score, ctx->static_scratch, ASAP_STATIC_SCRATCH_BYTES, need);
  if (st != ASAP_OK) return st;
  Strides3 qv{q_vis_stride[0], q_vis_stride[1], q_vis_stride[2]};
  Strides3 qt{q_txt_stride[0], q_txt_stride[1], q_txt_stride[2]};
  Strides3 kv{k_vis_stride[0], k_vis_stride[1], k_vis_stride[2]};
  return hip_result(ctx,
                    launch_score(*p, q_vis, qv, q_txt, qt, k_vis, kv, text_len, lse_extra, s_raw, s_hat, score,
                                 nullptr, nullptr, nullptr, nullptr, static_cast<char*>(ctx->static_scratch),
                                 ASAP_STATIC_SCRATCH_BYTES, static_cast<hipStream_t>(stream), ctx->timer),
                    "asap_score_static launch");
}

static asap_status select_checks(asap_ctx* ctx, const asap_params* p, const float* score, int32_t* kept_idx,
                                 int32_t* pruned_idx) {
  asap_status st = common_checks(ctx, p);
  if (st != ASAP_OK) return st;
  if (!score || !kept_idx || (!pruned_idx && p->k < p->V))
    return fail(ctx, ASAP_EINVAL, "asap_select: a required pointer is NULL");
  return ASAP_OK;
}

asap_status asap_select(asap_ctx* ctx, const asap_params* p, const float* score, int32_t* kept_idx,
                        int32_t* pruned_idx, void* workspace, size_t workspace_bytes, void* stream) {
  (void)workspace;
  (void)workspace_bytes;
  asap_status st = select_checks(ctx, p, score, kept_idx, pruned_idx);
  if (st != ASAP_OK) return st;
  return hip_result(ctx, launch_select(*p, score, kept_idx, pruned_idx, static_cast<hipStream_t>(stream), ctx->timer),
                    "asap_select launch");
}

static asap_status merge_checks(asap_ctx* ctx, const asap_params* p, const void* hidden,
                                const int64_t hidden_stride[2], const float* s_raw, const float* s_hat,
                                const int32_t* text_len, const int32_t* kept_idx, const int32_t* pruned_idx,
                                void* out_hidden, int32_t* pos_out, int32_t* new_len, int32_t* assign,
                                float* best_sim, float* wsum, int32_t* final_idx, void* workspace,
                                size_t workspace_bytes) {
  asap_status st = common_checks(ctx, p);
  if (st != ASAP_OK) return st;
  const bool paper = p->route == ASAP_ROUTE_PAPER;
  if (paper && (!s_raw || !assign || !best_sim))
    return fail(ctx, ASAP_EINVAL, "asap_merge: ASAP_ROUTE_PAPER needs s_raw, assign and best_sim");
  const bool has_pruned = p->k < p->V;
  if (!hidden || !s_hat || !text_len || !kept_idx || !out_hidden || !pos_out || !new_len || !wsum ||
      !final_idx || (has_pruned && (!pruned_idx || !assign || !best_sim)))
    return fail(ctx, ASAP_EINVAL, "asap_merge: a required pointer is NULL");
  if (!aligned16(hidden) || !aligned16(out_hidden))
    return fail(ctx, ASAP_EINVAL, "asap_merge: hidden and out_hidden must be 16-byte aligned");
  if ((st = check_strides(ctx, "hidden_stride", hidden_stride, 2, 8)) != ASAP_OK) return st;
  if (hidden_stride[1] < p->D) return fail(ctx, ASAP_EINVAL, "asap_merge: hidden row stride must be >= D");
  if ((st = check_span(ctx, "hidden", (int64_t)p->P + p->V + p->Tmax, hidden_stride[1], dtype_size(p->h_dtype))) !=
      ASAP_OK)
    return st;
  {
    const int64_t esz = dtype_size(p->h_dtype);
    const char* a0 = static_cast<const char*>(hidden);
    const char* a1 = a0 + ((int64_t)(p->B - 1) * hidden_stride[0] +
                           (int64_t)(p->P + p->V + p->Tmax - 1) * hidden_stride[1] + p->D) * esz;
    const char* b0 = static_cast<const char*>(out_hidden);
    const char* b1 = b0 + (int64_t)p->B * (p->P + p->k + p->Tmax) * p->D * esz;
    if (a0 < b1 && b0 < a1) return fail(ctx, ASAP_EINVAL, "asap_merge: out_hidden overlaps hidden");
  }
  return check_workspace(ctx, asap_workspace_bytes(p), workspace, workspace_bytes);
}

asap_status asap_merge(asap_ctx* ctx, const asap_params* p, const void* hidden, const int64_t hidden_stride[2],
                       const float* s_raw, const float* s_hat, const int32_t* text_len, const int32_t* kept_idx,
                       const int32_t* pruned_idx, void* out_hidden, int32_t* pos_out, int32_t* new_len,
                       int32_t* assign, float* best_sim, float* wsum, int32_t* final_idx, void* workspace,
                       size_t workspace_bytes, void* stream) {
  asap_status st = merge_checks(ctx, p, hidden, hidden_stride, s_raw, s_hat, text_len, kept_idx, pruned_idx,
                                out_hidden, pos_out, new_len, assign, best_sim, wsum, final_idx, workspace,
                                workspace_bytes);
  if (st != ASAP_OK) return st;
  return hip_result(ctx,
                    launch_merge(*p, hidden, hidden_stride[0], hidden_stride[1], s_raw, s_hat, text_len, kept_idx,
                                 pruned_idx, out_hidden, pos_out, new_len, assign, best_sim, wsum, final_idx,
                                 static_cast<char*>(workspace), static_cast<hipStream_t>(stream), ctx->timer),
                    "asap_merge launch");
}

asap_status asap_positions(asap_ctx* ctx, const asap_params* p, const int32_t* kept_idx, const int32_t* text_len,
                           int32_t* pos_out, int32_t* new_len, void* stream) {
  asap_status st = common_checks(ctx, p);
  if (st != ASAP_OK) return st;
  if (p->route != ASAP_ROUTE_ABSORB)
    return fail(ctx, ASAP_EUNSUPPORTED, "asap_positions: the positions follow from the kept set only with ASAP_ROUTE_ABSORB");
  if (!kept_idx || !text_len || !pos_out || !new_len)
    return fail(ctx, ASAP_EINVAL, "asap_positions: a required pointer is NULL");
  return hip_result(ctx, launch_positions(*p, kept_idx, text_len, pos_out, new_len, static_cast<hipStream_t>(stream),
                                          ctx->timer),
                    "asap_positions launch");
}

// shared checks of the contiguous K/V compaction entry points
static asap_status check_kv_buffers(asap_ctx* ctx, const asap_params* p, const char* fn, int32_t n_layers,
                                    const void* const* k_src, const void* const* v_src, void* const* k_dst,
                                    void* const* v_dst) {
  if (n_layers < 1 || n_layers > 64) return fail(ctx, ASAP_EINVAL, "%s: n_layers must be in [1, 64]", fn);
  if (!k_src || !v_src || !k_dst || !v_dst) return fail(ctx, ASAP_EINVAL, "%s: a required pointer is NULL", fn);
  const int64_t esz = dtype_size(p->kv_dtype);
  const int64_t src_bytes = (int64_t)p->B * p->Hkv * (p->P + p->V + p->Tmax) * p->d * esz;
  const int64_t dst_bytes = (int64_t)p->B * p->Hkv * (p->P + p->k + p->Tmax) * p->d * esz;
  for (int l = 0; l < n_layers; ++l) {
    const void* ptrs[4] = {k_src[l], v_src[l], k_dst[l], v_dst[l]};
    for (const void* q : ptrs) {
      if (!q) return fail(ctx, ASAP_EINVAL, "%s: layer %d has a NULL pointer", fn, l);
      if (!aligned16(q)) return fail(ctx, ASAP_EINVAL, "%s: layer %d pointer not 16-byte aligned", fn, l);
    }
  }
  // no destination may overlap any source (a kernel that reads and writes one buffer would race)
  for (int l = 0; l < n_layers; ++l)
    for (int which = 0; which < 2; ++which) {
      const char* d0 = static_cast<const char*>(which ? v_dst[l] : k_dst[l]);
      const char* d1 = d0 + dst_bytes;
      for (int m = 0; m < n_layers; ++m)
        for (int w2 = 0; w2 < 2; ++w2) {
          const char* s0 = static_cast<const char*>(w2 ? v_src[m] : k_src[m]);
          if (d0 < s0 + src_bytes && s0 < d1)
            return fail(ctx, ASAP_EINVAL, "%s: destination of layer %d overlaps a source", fn, l);
        }
    }
  return ASAP_OK;
}

asap_status asap_compact_kv(asap_ctx* ctx, const asap_params* p, int32_t n_layers, const void* const* k_src,
                            const void* const* v_src, void* const* k_dst, void* const* v_dst,
                            const int32_t* pos_out, const int32_t* new_len, void* stream) {
  asap_status st = common_checks(ctx, p);
  if (st != ASAP_OK) return st;
  if ((st = check_kv_buffers(ctx, p, "asap_compact_kv", n_layers, k_src, v_src, k_dst, v_dst)) != ASAP_OK) return st;
  if (!pos_out || !new_len) return fail(ctx, ASAP_EINVAL, "asap_compact_kv: a required pointer is NULL");
  return hip_result(ctx,
                    launch_compact_kv(*p, KV_BY_POS, n_layers, k_src, v_src, k_dst, v_dst, pos_out, new_len,
                                      static_cast<hipStream_t>(stream), ctx->timer),
                    "asap_compact_kv launch");
}

asap_status asap_compact_kv_from_kept(asap_ctx* ctx, const asap_params* p, int32_t n_layers,
                                      const void* const* k_src, const void* const* v_src, void* const* k_dst,
                                      void* const* v_dst, const int32_t* final_idx, const int32_t* text_len,
                                      void* stream) {
  asap_status st = common_checks(ctx, p);
  if (st != ASAP_OK) return st;
  if ((st = check_kv_buffers(ctx, p, "asap_compact_kv_from_kept", n_layers, k_src, v_src, k_dst, v_dst)) != ASAP_OK)
    return st;
  if (!final_idx || !text_len) return fail(ctx, ASAP_EINVAL, "asap_compact_kv_from_kept: a required pointer is NULL");
  return hip_result(ctx,
                    launch_compact_kv(*p, KV_FROM_KEPT, n_layers, k_src, v_src, k_dst, v_dst, final_idx, text_len,
                                      static_cast<hipStream_t>(stream), ctx->timer),
                    "asap_compact_kv_from_kept launch");
}

// The second stream and the three events of asap_stage, made on first use.
static asap_status stage_resources(asap_ctx* ctx) {
  if (ctx->side) return ASAP_OK;
  hipError_t e = hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking);     // default priority
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_start, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming);
  if (e != hipSuccess) {
    drop_stage_resources(ctx);
    return fail(ctx, ASAP_EHIP, "asap_stage: stream / event creation: %s", hipGetErrorString(e));
  }
  return ASAP_OK;
}

asap_status asap_stage(asap_ctx* ctx, const asap_params* p, const asap_stage_io* io, int32_t two_streams,
                       void* stream) {
  if (!ctx) return ASAP_EINVAL;
  if (!io) return fail(ctx, ASAP_EINVAL, "asap_stage: io is NULL");
  if (two_streams < ASAP_STREAMS_ONE || two_streams > ASAP_STREAMS_TWO)
    return fail(ctx, ASAP_EINVAL, "asap_stage: two_streams = %d is no asap_stream_mode", (int)two_streams);
  // every check of the single calls first: a failed check launches nothing
  asap_status st = score_checks(ctx, p, io->q_vis, io->q_vis_stride, io->q_txt, io->q_txt_stride, io->k_vis,
                                io->k_vis_stride, io->text_len, io->s_raw, io->s_hat, io->score, io->workspace,
                                io->workspace_bytes, asap_workspace_bytes(p));
  if (st == ASAP_OK) st = select_checks(ctx, p, io->score, io->kept_idx, io->pruned_idx);
  if (st == ASAP_OK)
    st = merge_checks(ctx, p, io->hidden, io->hidden_stride, io->s_raw, io->s_hat, io->text_len, io->kept_idx,
                      io->pruned_idx, io->out_hidden, io->pos_out, io->new_len, io->assign, io->best_sim, io->wsum,
                      io->final_idx, io->workspace, io->workspace_bytes);
  const bool has_kv = io->n_layers != 0;
  if (st == ASAP_OK && has_kv)
    st = check_kv_buffers(ctx, p, "asap_stage", io->n_layers, io->k_src, io->v_src, io->k_dst, io->v_dst);
  if (st != ASAP_OK) return st;
  // With ASAP_ROUTE_ABSORB the kept set is final after the selection: the K/V rows can move while the merge
  // runs.  The two hand-overs between the streams cost the caller's stream about as much as copying 64 MB
  // does (measured: single images and batches of 4 ran 3 to 9 % faster on one stream), so with
  // ASAP_STREAMS_AUTO smaller compactions stay on the caller's stream.
  const int64_t kv_row_bytes = p->d * (p->kv_dtype == ASAP_BF16 ? 2 : 4);
  const int64_t kv_bytes = 4 * (int64_t)io->n_layers * p->B * p->Hkv * (p->P + p->k + p->Tmax) * kv_row_bytes;
  const bool early = has_kv && p->route == ASAP_ROUTE_ABSORB &&
                     (two_streams == ASAP_STREAMS_TWO || (two_streams == ASAP_STREAMS_AUTO && kv_bytes >= (64ll << 20)));
  if (early && (st = stage_resources(ctx)) != ASAP_OK) return st;

  hipStream_t main = static_cast<hipStream_t>(stream);
  Strides3 qv{io->q_vis_stride[0], io->q_vis_stride[1], io->q_vis_stride[2]};
  Strides3 qt{io->q_txt_stride[0], io->q_txt_stride[1], io->q_txt_stride[2]};
  Strides3 kv{io->k_vis_stride[0], io->k_vis_stride[1], io->k_vis_stride[2]};
  char* ws = static_cast<char*>(io->workspace);
  // The K/V rows that no selection can change (prefix, valid text; Fig. 3) need not wait for it.
  //  * Deep caches (the compaction moves more than four times the bytes of the hidden states, so it
  //    outlasts similarity search and merge): the second stream starts on those rows at once, beside
  //    the score kernels, and takes the kept tokens' rows after the selection.
  //  * Otherwise, for large bf16 batches: the launch that finishes the score and selects keeps B
  //    compute units busy and moves next to nothing, so further workgroups of it copy those rows.
  const int64_t hidden_bytes = (int64_t)p->B * p->V * p->D * (p->h_dtype == ASAP_BF16 ? 2 : 4);
  const bool fixed_first = early && kv_bytes > 4 * hidden_bytes;
  const bool fixed_with_selection = early && !fixed_first && score_fuses_selection(*p) && p->h_dtype == ASAP_BF16 &&
                                    io->n_layers <= KV_LAYERS_PER_LAUNCH;
  hipError_t e = hipSuccess;
  bool forked = false;
  if (fixed_first) {
    e = hipEventRecord(ctx->ev_start, main);
    if (e == hipSuccess) e = hipStreamWaitEvent(ctx->side, ctx->ev_start, 0);
    if (e == hipSuccess) {
      forked = true;
      e = launch_compact_kv(*p, KV_FIXED_ONLY, io->n_layers, io->k_src, io->v_src, io->k_dst, io->v_dst,
                            io->kept_idx /* not read in this mode */, io->text_len, ctx->side, ctx->timer);
    }
  }
  KvFixedRows fixed;
  if (fixed_with_selection) {
    fill_kv_pointers(&fixed.ptrs, io->n_layers, io->k_src, io->v_src, io->k_dst, io->v_dst);
    fixed.n_bufs = 2 * io->n_layers;
    fixed.Hkv = p->Hkv; fixed.N = p->P + p->V + p->Tmax; fixed.Nout = p->P + p->k + p->Tmax;
    fixed.row_bytes = (int)kv_row_bytes;
    fixed.P = p->P; fixed.V = p->V; fixed.k = p->k; fixed.Tmax = p->Tmax;
  }
  if (e == hipSuccess)
    e = launch_score(*p, io->q_vis, qv, io->q_txt, qt, io->k_vis, kv, io->text_len, io->lse_extra, io->s_raw,
                     io->s_hat, io->score, io->kept_idx, io->pruned_idx, nullptr,
                     fixed_with_selection ? &fixed : nullptr, ws, ~size_t(0), main, ctx->timer);
  if (e == hipSuccess && early) {
    e = hipEventRecord(ctx->ev_fork, main);
    if (e == hipSuccess) e = hipStreamWaitEvent(ctx->side, ctx->ev_fork, 0);
    if (e == hipSuccess) {
      forked = true;
      e = launch_compact_kv(*p, (fixed_first || fixed_with_selection) ? KV_KEPT_ONLY : KV_FROM_KEPT, io->n_layers,
                            io->k_src, io->v_src, io->k_dst, io->v_dst, io->kept_idx, io->text_len, ctx->side,
                            ctx->timer);
    }
  }
  if (e == hipSuccess)
    e = launch_merge(*p, io->hidden, io->hidden_stride[0], io->hidden_stride[1], io->s_raw, io->s_hat, io->text_len,
                     io->kept_idx, io->pruned_idx, io->out_hidden, io->pos_out, io->new_len, io->assign, io->best_sim,
                     io->wsum, io->final_idx, ws, main, ctx->timer);
  if (forked) {      // also after an error: the caller's stream must not run ahead of the second one
    hipError_t e2 = hipEventRecord(ctx->ev_join, ctx->side);
    if (e2 == hipSuccess) e2 = hipStreamWaitEvent(main, ctx->ev_join, 0);
    if (e == hipSuccess) e = e2;
  } else if (e == hipSuccess && has_kv) {
    e = launch_compact_kv(*p, KV_FROM_KEPT, io->n_layers, io->k_src, io->v_src, io->k_dst, io->v_dst, io->final_idx,
                          io->text_len, main, ctx->timer);
  }
  return hip_result(ctx, e, "asap_stage launch");
}

asap_status asap_compact_kv_paged(asap_ctx* ctx, const asap_params* p, int32_t n_layers,
                                  const void* const* k_src_pool, const void* const* v_src_pool,
                                  void* const* k_dst_pool, void* const* v_dst_pool, int32_t page_size,
                                  const int32_t* src_table, int32_t src_table_stride, const int32_t* dst_table,
                                  int32_t dst_table_stride, const int32_t* pos_out, const int32_t* new_len,
                                  void* stream) {
  asap_status st = common_checks(ctx, p);
  if (st != ASAP_OK) return st;
  if (n_layers < 1 || n_layers > 64)
    return fail(ctx, ASAP_EINVAL, "asap_compact_kv_paged: n_layers must be in [1, 64]");
  if (!k_src_pool || !v_src_pool || !k_dst_pool || !v_dst_pool || !src_table || !dst_table || !pos_out || !new_len)
    return fail(ctx, ASAP_EINVAL, "asap_compact_kv_paged: a required pointer is NULL");
  if (page_size < 1) return fail(ctx, ASAP_EINVAL, "asap_compact_kv_paged: page_size must be >= 1");
  const int64_t n_in = (int64_t)p->P + p->V + p->Tmax, n_out = (int64_t)p->P + p->k + p->Tmax;
  if (src_table_stride < (n_in + page_size - 1) / page_size)
    return fail(ctx, ASAP_EINVAL, "asap_compact_kv_paged: src_table_stride %d below the %lld pages of a sequence",
                src_table_stride, (long long)((n_in + page_size - 1) / page_size));
  if (dst_table_stride < (n_out + page_size - 1) / page_size)
    return fail(ctx, ASAP_EINVAL, "asap_compact_kv_paged: dst_table_stride %d below the %lld pages of a sequence",
                dst_table_stride, (long long)((n_out + page_size - 1) / page_size));
  for (int l = 0; l < n_layers; ++l) {
    const void* ptrs[4] = {k_src_pool[l], v_src_pool[l], k_dst_pool[l], v_dst_pool[l]};
    for (const void* q : ptrs) {
      if (!q) return fail(ctx, ASAP_EINVAL, "asap_compact_kv_paged: layer %d has a NULL pointer", l);
      if (!aligned16(q))
        return fail(ctx, ASAP_EINVAL, "asap_compact_kv_paged: layer %d pointer not 16-byte aligned", l);
    }
  }
  return hip_result(ctx,
                    launch_compact_kv_paged(*p, n_layers, k_src_pool, v_src_pool, k_dst_pool, v_dst_pool, page_size,
                                            src_table, src_table_stride, dst_table, dst_table_stride, pos_out,
                                            new_len, static_cast<hipStream_t>(stream), ctx->timer),
                    "asap_compact_kv_paged launch");
}

size_t asap_attention_workspace_bytes(const asap_params* p) {
  if (check_params(p, nullptr, 0) != ASAP_OK) return 0;
  return attention_workspace_bytes(*p);
}

asap_status asap_attention(asap_ctx* ctx, const asap_params* p, const void* q, const int64_t q_stride[3],
                           const void* k, const int64_t k_stride[3], const void* v, const int64_t v_stride[3],
                           const float* s_hat, void* out, void* workspace, size_t workspace_bytes, void* stream) {
  asap_status st = common_checks(ctx, p);
  if (st != ASAP_OK) return st;
  if (!q || !k || !v || !out || (p->mask_mode == ASAP_MASK_KEYBIAS && !s_hat))
    return fail(ctx, ASAP_EINVAL, "asap_attention: a required pointer is NULL");
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out))
    return fail(ctx, ASAP_EINVAL, "asap_attention: q, k, v and out must be 16-byte aligned");
  if ((st = check_strides(ctx, "q_stride", q_stride, 3, 8)) != ASAP_OK) return st;
  if ((st = check_strides(ctx, "k_stride", k_stride, 3, 8)) != ASAP_OK) return st;
  if ((st = check_strides(ctx, "v_stride", v_stride, 3, 8)) != ASAP_OK) return st;
  if (q_stride[2] < p->d || k_stride[2] < p->d || v_stride[2] < p->d)
    return fail(ctx, ASAP_EINVAL, "asap_attention: row strides must be >= d");
  {
    const int64_t n = (int64_t)p->P + p->V + p->Tmax, esz = dtype_size(p->qk_dtype);
    if ((st = check_span(ctx, "q", n, q_stride[2], esz)) != ASAP_OK) return st;
    if ((st = check_span(ctx, "k", n, k_stride[2], esz)) != ASAP_OK) return st;
    if ((st = check_span(ctx, "v", n, v_stride[2], esz)) != ASAP_OK) return st;
  }
  const size_t need = attention_workspace_bytes(*p);
  if (!workspace) return fail(ctx, ASAP_EINVAL, "workspace is NULL");
  if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
    return fail(ctx, ASAP_EINVAL, "workspace must be 256-byte aligned");
  if (workspace_bytes < need)
    return fail(ctx, ASAP_EWORKSPACE, "asap_attention: workspace of %zu bytes, %zu needed", workspace_bytes, need);
  Strides3 sq{q_stride[0], q_stride[1], q_stride[2]};
  Strides3 sk{k_stride[0], k_stride[1], k_stride[2]};
  Strides3 sv{v_stride[0], v_stride[1], v_stride[2]};
  return hip_result(ctx,
                    launch_attention(*p, q, sq, k, sk, v, sv, s_hat, out, static_cast<char*>(workspace),
                                     static_cast<hipStream_t>(stream), ctx->timer),
                    "asap_attention launch");
}

// Eq. 7 / Eq. 8: host-side arithmetic only
static double layer_cost(double v, double d, double m) { return 4.0 * v * d * d + 2.0 * v * v * d + 3.0 * v * d * m; }

asap_status asap_theoretical_flops(const int32_t* layers, const int32_t* tokens, int32_t n_stages, int32_t d,
                                   int32_t m, double* flops) {
  if (!layers || !tokens || !flops || n_stages < 1 || d < 1 || m < 1) return ASAP_EINVAL;
  double total = 0.0;
  for (int n = 0; n < n_stages; ++n) {
    if (layers[n] < 0 || tokens[n] < 0) return ASAP_EINVAL;
    total += (double)layers[n] * layer_cost(tokens[n], d, m);
  }
  *flops = total;
  return ASAP_OK;
}

asap_status asap_flops_ratio(const int32_t* layers, const int32_t* tokens, int32_t n_stages, int32_t v0,
                             int32_t d, int32_t m, double* ratio) {
  if (!ratio || v0 < 1) return ASAP_EINVAL;
  double pruned = 0.0;
  asap_status st = asap_theoretical_flops(layers, tokens, n_stages, d, m, &pruned);
  if (st != ASAP_OK) return st;
  long total_layers = 0;
  for (int n = 0; n < n_stages; ++n) total_layers += layers[n];
  if (total_layers < 1) return ASAP_EINVAL;
  *ratio = pruned / ((double)total_layers * layer_cost(v0, d, m));
  return ASAP_OK;
}

}  // extern "C"
