// Context, error reporting, workspace and per-kernel event timing of libslim.
#include <mutex>
#include <set>

#include "slim_internal.h"

slim_status slim_fail(slim_ctx* ctx, slim_status code, const char* fmt, ...) {
  if (ctx) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(ctx->err, sizeof(ctx->err), fmt, ap);
    va_end(ap);
  }
  return code;
}

slim_status slim_ws_reserve(slim_ctx* ctx, size_t bytes) {
  ctx->ws_off = 0;
  ctx->sba_prep.valid = false;    // whoever reserves is about to overwrite what a prepare call left
  if (bytes <= ctx->ws_bytes) return SLIM_OK;
  if (ctx->ws_external)
    return slim_fail(ctx, SLIM_ERR_ALLOC, "the workspace given to slim_create holds %zu bytes, this call needs %zu "
                     "(slim_workspace_query gives the size for a shape)", ctx->ws_bytes, bytes);
  // the old buffer may still be in use by work enqueued earlier
  SLIM_HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
  if (ctx->ws) {
    SLIM_HIP_TRY(ctx, hipFree(ctx->ws));
    ctx->ws = nullptr;
    ctx->ws_bytes = 0;
  }
  void* p = nullptr;
  hipError_t e = hipMalloc(&p, bytes);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return slim_fail(ctx, SLIM_ERR_ALLOC, "cannot allocate %zu bytes of device workspace: %s", bytes,
                     hipGetErrorString(e));
  }
  ctx->ws = static_cast<char*>(p);
  ctx->ws_bytes = bytes;
  return SLIM_OK;
}

void* slim_ws_alloc(slim_ctx* ctx, size_t bytes) {
  size_t need = slim_ws_round(bytes);
  if (ctx->ws_off + need > ctx->ws_bytes) return nullptr;  // callers reserve the exact total first
  void* p = ctx->ws + ctx->ws_off;
  ctx->ws_off += need;
  return p;
}

slim_status slim_ensure_side(slim_ctx* ctx) {
  if (ctx->side) return SLIM_OK;
  SLIM_HIP_TRY(ctx, hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking));
  SLIM_HIP_TRY(ctx, hipStreamCreateWithFlags(&ctx->side2, hipStreamNonBlocking));
  SLIM_HIP_TRY(ctx, hipStreamCreateWithFlags(&ctx->side3, hipStreamNonBlocking));
  for (hipEvent_t& e : ctx->ev) SLIM_HIP_TRY(ctx, hipEventCreateWithFlags(&e, hipEventDisableTiming));
  return SLIM_OK;
}

// "<name>#side": a launch on one of the context's side streams, beside the work on its main stream
static const char* side_name(const char* name) {
  static std::mutex mu;
  static std::set<std::string> names;
  std::lock_guard<std::mutex> lock(mu);
  return names.insert(std::string(name) + "#side").first->c_str();
}

const char* slim_prof_name(const char* step, const char* kernel_function) {
  static std::mutex mu;
  static std::set<std::string> names;   // node-based: the strings never move
  std::lock_guard<std::mutex> lock(mu);
  return names.insert(std::string(step) + "@" + kernel_function).first->c_str();
}

void slim_prof_begin(slim_ctx* ctx, const char* name) {
  slim_prof_pending p;
  p.name = ctx->on_side ? side_name(name) : name;
  for (hipEvent_t* ev : {&p.start, &p.stop}) {
    if (!ctx->free_events.empty()) {
      *ev = ctx->free_events.back();
      ctx->free_events.pop_back();
    } else if (hipEventCreate(ev) != hipSuccess) {
      *ev = nullptr;
    }
  }
  if (p.start) (void)hipEventRecord(p.start, ctx->stream);
  ctx->pending.push_back(p);
}

void slim_prof_end(slim_ctx* ctx) {
  slim_prof_pending& p = ctx->pending.back();
  if (p.stop) (void)hipEventRecord(p.stop, ctx->stream);
}

extern "C" {

void slim_default_params(slim_params* p) {
  if (p) memset(p, 0, sizeof(*p));
}

int slim_default_tau(double* tau_host, int cap) {
  const double lambda = 0.1;
  const int n = 50;
  if (tau_host) {
    for (int c = 0; c < 2 * n && c < cap; ++c) tau_host[c] = (1.0 - lambda) + static_cast<double>(c) * (lambda / n);
  }
  return 2 * n;
}

slim_status slim_create(slim_ctx** out, void* hip_stream, void* workspace, size_t workspace_bytes) {
  if (!out) return SLIM_ERR_INVALID_ARG;
  *out = nullptr;
  if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return SLIM_ERR_INVALID_ARG;
  slim_ctx* ctx = new (std::nothrow) slim_ctx();
  if (!ctx) return SLIM_ERR_ALLOC;
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  if (workspace) {
    ctx->ws = static_cast<char*>(workspace);
    ctx->ws_bytes = workspace_bytes;
    ctx->ws_external = true;
  }
  auto bail = [&](hipError_t e, const char* what) {
    fprintf(stderr, "slim_create: %s failed: %s\n", what, hipGetErrorString(e));
    if (ctx->tau_default) (void)hipFree(ctx->tau_default);
    if (ctx->dflags) (void)hipFree(ctx->dflags);
    if (ctx->hpin) (void)hipHostFree(ctx->hpin);
    delete ctx;
    return SLIM_ERR_HIP;
  };
  hipError_t e = hipGetDevice(&ctx->device);
  if (e != hipSuccess) return bail(e, "hipGetDevice");
  e = hipDeviceGetAttribute(&ctx->num_cus, hipDeviceAttributeMultiprocessorCount, ctx->device);
  if (e != hipSuccess) return bail(e, "hipDeviceGetAttribute");
  e = hipMalloc(reinterpret_cast<void**>(&ctx->tau_default), SLIM_MAX_CAND * sizeof(double));
  if (e != hipSuccess) return bail(e, "hipMalloc(tau)");
  e = hipMalloc(reinterpret_cast<void**>(&ctx->dflags), 64 * sizeof(int));
  if (e != hipSuccess) return bail(e, "hipMalloc(flags)");
  e = hipHostMalloc(reinterpret_cast<void**>(&ctx->hpin), SLIM_HPIN_BYTES, hipHostMallocDefault);
  if (e != hipSuccess) return bail(e, "hipHostMalloc");
  double* tau_h = reinterpret_cast<double*>(ctx->hpin);
  ctx->ncand_default = slim_default_tau(tau_h, SLIM_MAX_CAND);
  e = hipMemcpyAsync(ctx->tau_default, tau_h, ctx->ncand_default * sizeof(double), hipMemcpyHostToDevice,
                     ctx->stream);
  if (e != hipSuccess) return bail(e, "hipMemcpyAsync(tau)");
  e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return bail(e, "hipStreamSynchronize");
  if (slim_dq_scratch_resolve(ctx) != SLIM_OK) {
    fprintf(stderr, "slim_create: %s\n", ctx->err);
    return bail(hipErrorUnknown, "looking up the fixed buffer");
  }
  *out = ctx;
  return SLIM_OK;
}

slim_status slim_destroy(slim_ctx* ctx) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  (void)hipStreamSynchronize(ctx->stream);
  for (auto& p : ctx->pending) {
    if (p.start) (void)hipEventDestroy(p.start);
    if (p.stop) (void)hipEventDestroy(p.stop);
  }
  for (hipEvent_t ev : ctx->free_events) (void)hipEventDestroy(ev);
  if (ctx->side) {
    (void)hipStreamSynchronize(ctx->side);
    for (hipEvent_t e : ctx->ev)
      if (e) (void)hipEventDestroy(e);
    (void)hipStreamDestroy(ctx->side);
    for (hipStream_t st : {ctx->side2, ctx->side3})
      if (st) {
        (void)hipStreamSynchronize(st);
        (void)hipStreamDestroy(st);
      }
  }
  if (ctx->ws && !ctx->ws_external) (void)hipFree(ctx->ws);
  if (ctx->tau_default) (void)hipFree(ctx->tau_default);
  if (ctx->dflags) (void)hipFree(ctx->dflags);
  if (ctx->hpin) (void)hipHostFree(ctx->hpin);
  delete ctx;
  return SLIM_OK;
}

const char* slim_last_error(const slim_ctx* ctx) { return ctx ? ctx->err : "null context"; }

size_t slim_workspace_bytes(const slim_ctx* ctx) { return ctx ? ctx->ws_bytes : 0; }

size_t slim_workspace_query(const slim_shape* s, int num_cus) {
  if (!s || s->m <= 0) return 0;
  const int ncu = num_cus > 0 ? num_cus : 256;
  size_t need = 0;
  if (s->t_c > 0) need = std::max(need, slim_ws_need_gram(s->m, s->t_c, ncu));
  need = std::max(need, slim_ws_need_inverse(s->m));
  if (s->n > 0) {
    need = std::max(need, slim_ws_need_salience(s->n, s->m));
    need = std::max(need, slim_ws_need_sqc(s->n));
    need = std::max(need, slim_ws_need_gptq(s->n, s->m));
    if (s->beta > 0 && s->t_s > 0) need = std::max(need, slim_ws_need_sba(s->n, s->m, s->beta, s->t_s));
    if (s->beta > 0 && s->t_x > 0)     // (with room for the unpacked zero points of slim_dequant_matmul_zp)
      need = std::max(need, slim_ws_need_dequant(s->n, s->m, s->beta, s->t_x, ncu) +
                                slim_ws_round(sizeof(double) * (size_t)s->n * (s->m / s->beta)));
    if (s->beta > 0 && s->lwc_steps > 0) need = std::max(need, slim_ws_need_lwc(s->n, s->m, s->beta, s->lwc_steps));
  }
  return need;
}

slim_status slim_profile_enable(slim_ctx* ctx, int on) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  ctx->prof = on != 0;
  return SLIM_OK;
}

int slim_profile_collect(slim_ctx* ctx) {
  if (!ctx) return 0;
  (void)hipStreamSynchronize(ctx->stream);
  for (auto& p : ctx->pending) {
    float ms = 0.f;
    if (p.start && p.stop && hipEventElapsedTime(&ms, p.start, p.stop) == hipSuccess) {
      slim_prof_entry* hit = nullptr;
      for (auto& en : ctx->entries)
        if (en.name == p.name) hit = &en;
      if (!hit) {
        ctx->entries.emplace_back();
        hit = &ctx->entries.back();
        hit->name = p.name;
      }
      hit->total_ms += ms;
      hit->launches += 1;
    }
    if (p.start) ctx->free_events.push_back(p.start);
    if (p.stop) ctx->free_events.push_back(p.stop);
  }
  ctx->pending.clear();
  return static_cast<int>(ctx->entries.size());
}

slim_status slim_profile_entry(const slim_ctx* ctx, int i, const char** name, double* total_ms, int* launches) {
  if (!ctx || i < 0 || i >= static_cast<int>(ctx->entries.size())) return SLIM_ERR_INVALID_ARG;
  if (name) *name = ctx->entries[i].name.c_str();
  if (total_ms) *total_ms = ctx->entries[i].total_ms;
  if (launches) *launches = ctx->entries[i].launches;
  return SLIM_OK;
}

slim_status slim_profile_reset(slim_ctx* ctx) {
  if (!ctx) return SLIM_ERR_INVALID_ARG;
  slim_profile_collect(ctx);
  ctx->entries.clear();
  return SLIM_OK;
}

}  // extern "C"
