// C-ABI entry points (include/br.h): argument checks, workspace layout, kernel launches.
// Host code only; every step of the path runs in the kernels.
#include <hip/hip_runtime.h>

#include <new>
#include <vector>

#include "br.h"
#include "br_device.h"
#include "br_launch.h"
#include "br_subset_dp.h"

namespace {

struct EvPair {
  hipEvent_t a, b;
  int kid;
};

uint64_t align_up(uint64_t x) { return (x + 255u) & ~(uint64_t)255u; }

int pred_width(const br_config &c) {
  if (c.H == 0) return 0;
  return c.pred_mode == 2 ? 3 : (c.pred_mode == 3 ? 2 : (c.pred_mode == 1 ? 1 : c.H));
}

int queue_pred_width(const br_config &c) { return c.pred_mode == 2 ? 0 : pred_width(c); }

bool config_ok(const br_config *c) {
  if (!c) return false;
  if (c->n_inst < 1 || c->G < 1 || c->G > BR_MAX_G || c->B < 1 || c->B > BR_MAX_B) return false;
  if (c->max_wait < 1 || c->max_wait > BR_MAX_WAIT || c->H < 0 || c->H > BR_MAX_H) return false;
  if (c->R_max < 1 || c->R_max > BR_MAX_RMAX || c->S_greedy < 0) return false;
  if (c->token_watermark < 0 || c->token_cap < 0) return false;
  if (c->pred_mode < 0 || c->pred_mode > 3) return false;
  if (c->H > BR_HP && c->pred_mode == 0) return false;  // a hazard per offset is carried for short horizons only
  if (c->H > BR_HP && c->R_max > 16) return false;      // the search by reachable sums serves the register-horizon kernels
  if (c->pred_mode == 2) {
    if (c->H == 0 || !c->hist || !c->hist_sum || c->hist_n < 1 || c->hist_n > (1 << 20) || c->refresh_period < 1)
      return false;
  }
  if (c->H > 0) {
    if (!(c->alpha > 0.0f) || !(c->beta >= 0.0f) || !(c->gamma > 0.0f) || !(c->gamma <= 1.0f)) return false;
  }
  return true;
}

// `dl`: byte offset of the discount table that horizons beyond BR_HP keep in the workspace (after the
// arrays of the public layout), or 0
void make_layout(const br_config &c, br_layout *l, uint64_t *dl = nullptr, uint64_t *score_scratch = nullptr,
                 uint64_t *pol = nullptr, uint64_t *dp = nullptr) {
  const uint64_t N = (uint64_t)c.n_inst, G = (uint64_t)c.G, Q = (uint64_t)c.max_wait, H1 = (uint64_t)c.H + 1;
  const uint64_t P = (uint64_t)pred_width(c), Pq = (uint64_t)queue_pred_width(c);
  const uint64_t Bs = ((uint64_t)c.B + 3u) & ~(uint64_t)3u;
  uint64_t off = 0;
  auto take = [&](uint64_t words) {
    const uint64_t at = off;
    off = align_up(off + words * 4u);
    return at;
  };
  l->L = take(N * G);
  l->n = take(N * G);
  l->kv = take(N * G * Bs);
  l->rem = take(N * G * Bs);
  l->pred = take(N * G * Bs * P);
  l->qlen = take(N);
  l->qs = take(N * Q);
  l->qo = take(N * Q);
  l->qid = take(N * Q);
  l->qpred = take(N * Q * Pq);
  l->Lh = take(N * G * H1);
  l->Mh = take(N * H1);
  l->mh = take(N * G * H1);
  l->minm = take(N * G);
  const uint64_t dl_at = c.H > BR_HP ? take((uint64_t)BR_HS(c.H)) : 0;
  if (dl) *dl = dl_at;
  const uint64_t ss_bytes = br_score_scratch_bytes(c.n_inst, c.max_wait, c.G);
  const uint64_t ss_at = ss_bytes ? take(ss_bytes / 4) : 0;  // partial results of the tiled score path (private)
  if (score_scratch) *score_scratch = ss_at;
  const uint64_t pol_at = take(2 * N);  // comparison policies: round-robin cursor and draw count per cluster (private)
  if (pol) *pol = pol_at;
  // windows beyond 16 requests: bit rows and first-request table of the subset search, per cluster (private)
  const uint64_t dp_at = c.R_max > 16 ? take(N * (uint64_t)br_dp_cluster_words(c.B < c.R_max ? c.B : c.R_max)) : 0;
  if (dp) *dp = dp_at;
  l->total_bytes = off;
  l->B_stride = (int32_t)Bs;
  l->P = (int32_t)P;
  l->Pq = (int32_t)Pq;
  l->pad = 0;
}

}  // namespace

struct br_ctx {
  br_config cfg;
  br_layout lay;
  BrParams p;
  int *score_scratch;
  int *pol;                // [N][2] state of the comparison policies
  int *static_scratch;     // the library's fixed scratch array on this context's device (br_route_step_static), or null
  int32_t static_hip;      // why it is null: the hipError_t of the failed look-up
  hipStream_t st;
  int32_t last_hip;
  bool prof;
  std::vector<EvPair> pending, spare;
  double ms[BR_NKERNELS];
  int64_t launches[BR_NKERNELS];
};

namespace {

int32_t fail_hip(br_ctx *ctx, hipError_t e) {
  ctx->last_hip = (int32_t)e;
  return BR_EHIP;
}

// Enqueue one kernel; with profiling on, bracket it with an event pair on the same stream.
template <class Fn>
int32_t enqueue(br_ctx *ctx, int kid, Fn &&fn, bool bracket = true) {
  EvPair ev{};
  const bool prof = ctx->prof && bracket;
  if (prof) {
    if (!ctx->spare.empty()) {
      ev = ctx->spare.back();
      ctx->spare.pop_back();
    } else {
      hipError_t e = hipEventCreate(&ev.a);
      if (e != hipSuccess) return fail_hip(ctx, e);
      e = hipEventCreate(&ev.b);
      if (e != hipSuccess) {
        (void)hipEventDestroy(ev.a);
        return fail_hip(ctx, e);
      }
    }
    ev.kid = kid;
    hipError_t e = hipEventRecord(ev.a, ctx->st);
    if (e != hipSuccess) {
      ctx->spare.push_back(ev);
      return fail_hip(ctx, e);
    }
  }
  // an error left behind by an earlier, unrelated HIP call of this thread is not this launch's: clear it first,
  // so that what is read after the launch is the launch's own result
  (void)hipGetLastError();
  fn();
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    if (prof) ctx->spare.push_back(ev);
    return fail_hip(ctx, e);
  }
  if (prof) {
    e = hipEventRecord(ev.b, ctx->st);
    if (e != hipSuccess) {
      ctx->spare.push_back(ev);
      return fail_hip(ctx, e);
    }
    ctx->pending.push_back(ev);
  }
  return BR_OK;
}

}  // namespace

extern "C" {

uint64_t br_workspace_bytes(const br_config *cfg) {
  if (!config_ok(cfg)) return 0;
  br_layout l;
  make_layout(*cfg, &l);
  return l.total_bytes;
}

int32_t br_init(const br_config *cfg, const br_init_state *init, br_ctx **out) {
  if (!out || !config_ok(cfg) || !cfg->workspace) return BR_EINVAL;
  if (((uintptr_t)cfg->workspace & 255u) != 0) return BR_EINVAL;
  br_layout l;
  uint64_t dl_at = 0, ss_at = 0, pol_at = 0, dp_at = 0;
  make_layout(*cfg, &l, &dl_at, &ss_at, &pol_at, &dp_at);
  if (cfg->workspace_bytes < l.total_bytes) return BR_ENOMEM;
  const int P = pred_width(*cfg);
  if (init && (!init->n || !init->kv || !init->rem || (P > 0 && !init->pred))) return BR_EINVAL;

  br_ctx *ctx = new (std::nothrow) br_ctx();
  if (!ctx) return BR_ENOMEM;
  ctx->cfg = *cfg;
  ctx->lay = l;
  ctx->st = (hipStream_t)cfg->stream;
  ctx->last_hip = 0;
  ctx->prof = false;
  for (int k = 0; k < BR_NKERNELS; ++k) {
    ctx->ms[k] = 0.0;
    ctx->launches[k] = 0;
  }

  BrParams &p = ctx->p;
  p.N = cfg->n_inst;
  p.G = cfg->G;
  p.B = cfg->B;
  p.Bs = l.B_stride;
  p.Q = cfg->max_wait;
  p.H = cfg->H;
  p.P = P;
  p.Pq = queue_pred_width(*cfg);
  p.hist_n = cfg->pred_mode == 2 ? cfg->hist_n : 0;
  p.refresh = cfg->pred_mode == 2 ? cfg->refresh_period : 1;
  p.adv_t = 0;
  p.hist = cfg->pred_mode == 2 ? cfg->hist : nullptr;
  p.hsum = cfg->pred_mode == 2 ? (const long long *)cfg->hist_sum : nullptr;
  p.R_max = cfg->R_max;
  p.S_greedy = cfg->S_greedy;
  p.W = cfg->token_watermark;
  p.C = cfg->token_cap;
  p.pred_mode = cfg->pred_mode;
  p.gate = cfg->gate_pfin;
  // discount vector d = (1, gamma, ..., gamma^H) by repeated product, D = 1^T d summed upwards
  // (Sec. 4.1); fp32 throughout so the device sees the same constants a float reference does
  for (int h = 0; h <= BR_HP; ++h) p.d[h] = 0.0f;
  volatile float acc = 0.0f, dh = 1.0f;
  for (int h = 0; h <= cfg->H; ++h) {
    if (h > 0) dh = dh * cfg->gamma;
    if (h <= BR_HP) p.d[h] = dh;
    acc = acc + dh;
  }
  volatile float aD = cfg->alpha * acc;
  p.aD = cfg->H > 0 ? (float)aD : 1.0f;
  p.beta = cfg->H > 0 ? cfg->beta : (float)cfg->G;

  char *base = (char *)cfg->workspace;
  p.L = (int32_t *)(base + l.L);
  p.n = (int32_t *)(base + l.n);
  p.kv = (int32_t *)(base + l.kv);
  p.rem = (int32_t *)(base + l.rem);
  p.pred = (float *)(base + l.pred);
  p.qlen = (int32_t *)(base + l.qlen);
  p.qs = (int32_t *)(base + l.qs);
  p.qo = (int32_t *)(base + l.qo);
  p.qid = (int32_t *)(base + l.qid);
  p.qpred = (float *)(base + l.qpred);
  p.Lh = (int32_t *)(base + l.Lh);
  p.Mh = (int32_t *)(base + l.Mh);
  p.mh = (int32_t *)(base + l.mh);
  p.minm = (int32_t *)(base + l.minm);
  p.dl = dl_at ? (const float *)(base + dl_at) : nullptr;
  p.dp = dp_at ? (int32_t *)(base + dp_at) : nullptr;
  ctx->score_scratch = ss_at ? (int *)(base + ss_at) : nullptr;
  ctx->pol = (int *)(base + pol_at);
  // set-up of the allocation-free entry point: the device address of the fixed scratch array, looked up once per
  // device with the context's device current (the caller's, as for every launch on its stream)
  ctx->static_scratch = nullptr;
  ctx->static_hip = (int32_t)br_static_scratch_resolve(&ctx->static_scratch);

  int32_t rc = enqueue(ctx, BR_K_INIT, [&] { br_launch_clear(p, ctx->pol, ctx->st); });
  if (rc == BR_OK && p.dl) rc = enqueue(ctx, BR_K_INIT, [&] { br_launch_discounts(p, cfg->gamma, ctx->st); });
  if (rc == BR_OK && init)
    rc = enqueue(ctx, BR_K_INIT, [&] { br_launch_load_init(p, init->n, init->kv, init->rem, init->pred, ctx->st); });
  if (rc != BR_OK) {
    delete ctx;
    return rc;
  }
  *out = ctx;
  return BR_OK;
}

// one round, optionally followed inside the assignment kernel by `adv_t` decode steps
// fixed_scratch: the tiled score path keeps its partial results in the library's fixed device array instead of
// the workspace, and no launch is bracketed by profiling events (creating one allocates)
static int32_t route(br_ctx *ctx, const br_arrivals *in, const br_step_out *out, int32_t adv_t, bool fixed_scratch = false) {
  if (!ctx || adv_t < 0) return BR_EINVAL;
  const bool br = !fixed_scratch;
  int *partials = ctx->score_scratch;
  if (fixed_scratch) {
    if ((uint64_t)br_score_scratch_bytes(ctx->p.N, ctx->p.Q, ctx->p.G) > (uint64_t)br_static_scratch_bytes() ||
        ctx->p.N > BR_STATIC_MAX_INST)
      return BR_ELIMIT;
    if (!ctx->static_scratch) {
      ctx->last_hip = ctx->static_hip;
      return BR_EHIP;
    }
    partials = ctx->static_scratch;
  }
  BrArr a{};
  if (in && in->arr_cap < 0) return BR_EINVAL;
  if (in && in->count && in->arr_cap > 0) {
    if (!in->s || !in->o || (ctx->p.Pq > 0 && !in->pred)) return BR_EINVAL;
    a.count = in->count;
    a.s = in->s;
    a.o = in->o;
    a.id = in->id;
    a.pred = in->pred;
    a.arr_cap = in->arr_cap;
  }
  BrOut o{};
  if (out) {
    o.assign = out->assign;
    o.assign_id = out->assign_id;
    o.stats = (long long *)out->stats;
    o.F = out->F;
    o.best_g = out->best_g;
    o.best_i = out->best_i;
  }
  BrParams p = ctx->p;
  // windows beyond 8 requests and long-horizon rounds shared by several waves have no fused instantiation: the
  // decode steps follow as their own launch
  const bool split_adv = adv_t > 0 && (p.R_max > 8 || (p.H > BR_HP && br_long_waves(p) > 1));
  p.adv_t = split_adv ? 0 : adv_t;
  int32_t rc = BR_OK;
  if (p.H > 0) rc = enqueue(ctx, BR_K_PROJECT, [&] { br_launch_project(p, ctx->st); }, br);
  // large batches of clusters with short queues: the reductions ride along in the assignment launch
  const bool together = (o.best_g || o.best_i) && !o.F && p.N >= BR_SCORE_WAVE_MIN_N && p.R_max <= 8 &&
                        (p.H == 0 ? p.Q <= 256 : (p.H <= BR_HP && p.Q <= 512));
  // BR-0 with decode steps: round and decode steps on two waves per cluster; the reductions ride on the helper wave
  // unless the matrix is asked for (then the score kernel writes all three outputs)
  const bool split = br_split_serves(p);
  if (split) {
    BrOut o2 = o;
    if (o.F) {
      rc = enqueue(ctx, BR_K_SCORE, [&] { br_launch_score(p, a, o, partials, ctx->st); }, br);
      o2.F = nullptr, o2.best_g = nullptr, o2.best_i = nullptr;
    }
    if (rc == BR_OK) rc = enqueue(ctx, BR_K_ASSIGN, [&] { br_launch_route_split(p, a, o2, ctx->st); }, br);
    return rc;
  }
  if (rc == BR_OK && !together && (o.F || o.best_g || o.best_i))
    rc = enqueue(ctx, BR_K_SCORE, [&] { br_launch_score(p, a, o, partials, ctx->st); }, br);
  if (rc == BR_OK) {
    if (together && p.H > 0)
      rc = enqueue(ctx, BR_K_ASSIGN, [&] { br_launch_route_h(p, a, o, ctx->st); }, br);
    else if (together)
      rc = enqueue(ctx, BR_K_ASSIGN, [&] { br_launch_route4(p, a, o, ctx->st); }, br);
    else
      rc = enqueue(ctx, BR_K_ASSIGN, [&] { br_launch_assign(p, a, o, ctx->st); }, br);
  }
  if (rc == BR_OK && split_adv) rc = enqueue(ctx, BR_K_ADVANCE, [&] { br_launch_advance(p, adv_t, ctx->st); }, br);
  return rc;
}

int32_t br_route_step(br_ctx *ctx, const br_arrivals *in, const br_step_out *out) { return route(ctx, in, out, 0); }

int32_t br_route_advance(br_ctx *ctx, const br_arrivals *in, const br_step_out *out, int32_t n_steps) {
  return route(ctx, in, out, n_steps);
}

int32_t br_route_step_static(br_ctx *ctx, const br_arrivals *in, const br_step_out *out) {
  return route(ctx, in, out, 0, true);
}

int32_t br_route_bypass(br_ctx *ctx, const br_arrivals *in, const br_step_out *out) {
  if (!ctx || ctx->p.H != 0) return BR_EINVAL;
  if (in && in->arr_cap < 0) return BR_EINVAL;
  if (!in || !in->count || in->arr_cap == 0) return BR_OK;  // nothing to place
  if (in->arr_cap > BR_MAX_WAIT || !in->s || !in->o) return BR_EINVAL;
  BrArr a{};
  a.count = in->count;
  a.s = in->s;
  a.o = in->o;
  a.id = in->id;
  a.pred = nullptr;
  a.arr_cap = in->arr_cap;
  BrOut o{};
  if (out) {
    o.assign = out->assign;
    o.stats = (long long *)out->stats;
  }
  return enqueue(ctx, BR_K_BYPASS, [&] { br_launch_bypass(ctx->p, a, o, ctx->st); });
}

int32_t br_route_baseline(br_ctx *ctx, const br_arrivals *in, const br_step_out *out, int32_t policy, uint64_t seed) {
  if (!ctx || ctx->p.H != 0 || policy < BR_POLICY_RANDOM || policy > BR_POLICY_JSQ) return BR_EINVAL;
  if (in && in->arr_cap < 0) return BR_EINVAL;
  BrArr a{};
  if (in && in->count && in->arr_cap > 0) {
    if (!in->s || !in->o) return BR_EINVAL;
    a.count = in->count;
    a.s = in->s;
    a.o = in->o;
    a.id = in->id;
    a.arr_cap = in->arr_cap;
  }
  BrOut o{};
  if (out) {
    o.assign = out->assign;
    o.assign_id = out->assign_id;
    o.stats = (long long *)out->stats;
  }
  return enqueue(ctx, BR_K_BASELINE, [&] { br_launch_baseline(ctx->p, a, o, ctx->pol, policy, (unsigned long long)seed, ctx->st); });
}

int32_t br_advance_decode(br_ctx *ctx, int32_t n_steps) {
  if (!ctx || n_steps < 0) return BR_EINVAL;
  if (n_steps == 0) return BR_OK;
  return enqueue(ctx, BR_K_ADVANCE, [&] { br_launch_advance(ctx->p, n_steps, ctx->st); });
}

void br_free(br_ctx *ctx) {
  if (!ctx) return;
  for (auto &v : {&ctx->pending, &ctx->spare})
    for (EvPair &e : *v) {
      (void)hipEventDestroy(e.a);
      (void)hipEventDestroy(e.b);
    }
  delete ctx;
}

int32_t br_last_hip_error(const br_ctx *ctx) { return ctx ? ctx->last_hip : 0; }

int32_t br_get_layout(const br_ctx *ctx, br_layout *out) {
  if (!ctx || !out) return BR_EINVAL;
  *out = ctx->lay;
  return BR_OK;
}

int32_t br_profile_enable(br_ctx *ctx, int32_t on) {
  if (!ctx) return BR_EINVAL;
  ctx->prof = on != 0;
  return BR_OK;
}

int32_t br_profile_read(br_ctx *ctx, double *ms, int64_t *launches) {
  if (!ctx || !ms || !launches) return BR_EINVAL;
  for (EvPair &e : ctx->pending) {
    hipError_t r = hipEventSynchronize(e.b);
    if (r != hipSuccess) return fail_hip(ctx, r);
    float t = 0.0f;
    r = hipEventElapsedTime(&t, e.a, e.b);
    if (r != hipSuccess) return fail_hip(ctx, r);
    ctx->ms[e.kid] += (double)t;
    ctx->launches[e.kid] += 1;
    ctx->spare.push_back(e);
  }
  ctx->pending.clear();
  for (int k = 0; k < BR_NKERNELS; ++k) {
    ms[k] = ctx->ms[k];
    launches[k] = ctx->launches[k];
    ctx->ms[k] = 0.0;
    ctx->launches[k] = 0;
  }
  return BR_OK;
}

}  // extern "C"
