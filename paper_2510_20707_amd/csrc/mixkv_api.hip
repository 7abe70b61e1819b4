// Host side of libmixkv: argument validation, workspace carve-up and the launch sequence.
#include <cmath>
#include <cstring>
#include <mutex>

#include "mixkv_internal.h"

namespace mixkv {

int stream_chunk_keys(int dtype, int D);
int max_adaptive_heads();
bool mixsel_supported(const Shape &s);
hipError_t launch_topsel(const Shape &s, const LayerOutTable &out, char *ws, const Workspace &w, int64_t unit0, int nunits,
                         int cand_m, const int32_t *budgets, hipStream_t st);
hipError_t launch_mixsel(const Shape &s, bool select, const LayerOutTable &out, char *ws, const Workspace &w,
                         int64_t unit0, int nunits, const LayerInTable &in, int gather_eb, int cand_m,
                         const int32_t *budgets, hipStream_t st);

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

mixkv_status make_shape(const mixkv_params *p, Shape *s) {
  if (!p || !s) return MIXKV_ERR_INVALID_ARG;
  if (p->dtype != MIXKV_F32 && p->dtype != MIXKV_BF16) return MIXKV_ERR_INVALID_ARG;
  if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1) return MIXKV_ERR_INVALID_ARG;
  if (p->n_q_heads % p->n_kv_heads != 0) return MIXKV_ERR_INVALID_ARG;
  if (p->head_dim != 64 && p->head_dim != 128) return MIXKV_ERR_UNSUPPORTED;
  if (p->seq_len < 2) return MIXKV_ERR_INVALID_ARG;
  if (p->window < 1 || p->window >= p->seq_len) return MIXKV_ERR_INVALID_ARG;
  if (p->window > MIXKV_MAX_WINDOW) return MIXKV_ERR_UNSUPPORTED;
  if (p->budget < p->window || p->budget > p->seq_len) return MIXKV_ERR_INVALID_ARG;
  if (p->pool != MIXKV_POOL_NONE && p->pool != MIXKV_POOL_AVG && p->pool != MIXKV_POOL_MAX) return MIXKV_ERR_INVALID_ARG;
  if (p->pool != MIXKV_POOL_NONE && (p->pool_kernel < 1 || p->pool_kernel > 63 || p->pool_kernel % 2 == 0))
    return MIXKV_ERR_INVALID_ARG;
  if (p->causal_window != 0 && p->causal_window != 1) return MIXKV_ERR_INVALID_ARG;
  if (!(p->softmax_scale > 0.f) || !std::isfinite(p->softmax_scale)) return MIXKV_ERR_INVALID_ARG;
  if (!(p->eps > 0.f) || !std::isfinite(p->eps)) return MIXKV_ERR_INVALID_ARG;
  if (p->intrinsic != MIXKV_INTRINSIC_NONE && p->intrinsic != MIXKV_INTRINSIC_VNORM &&
      p->intrinsic != MIXKV_INTRINSIC_KNORM)
    return MIXKV_ERR_INVALID_ARG;
  if ((int)p->mix < MIXKV_MIX_HEAD_ADAPTIVE || (int)p->mix > MIXKV_MIX_GIVEN_R) return MIXKV_ERR_INVALID_ARG;
  if (p->budget_mode != MIXKV_BUDGET_FIXED && p->budget_mode != MIXKV_BUDGET_HEAD_ADAPTIVE &&
      p->budget_mode != MIXKV_BUDGET_PER_HEAD)
    return MIXKV_ERR_INVALID_ARG;
  const int G = p->n_q_heads / p->n_kv_heads;
  if ((int64_t)G * p->window > MIXKV_MAX_GROUP_ROWS) return MIXKV_ERR_UNSUPPORTED;
  if (p->budget_mode == MIXKV_BUDGET_HEAD_ADAPTIVE) {
    if (p->budget_floor < 0 || p->budget_floor > p->budget - p->window) return MIXKV_ERR_INVALID_ARG;
    if (p->n_kv_heads > max_adaptive_heads()) return MIXKV_ERR_UNSUPPORTED;
    if ((int64_t)p->n_kv_heads * (p->seq_len - p->window) > INT32_MAX) return MIXKV_ERR_UNSUPPORTED;
  }
  if ((int64_t)p->batch * kLayersPerLaunch > 65535) return MIXKV_ERR_UNSUPPORTED;
  if ((int64_t)p->batch * p->n_kv_heads * p->seq_len > INT32_MAX) return MIXKV_ERR_UNSUPPORTED;

  s->batch = p->batch; s->hq = p->n_q_heads; s->hkv = p->n_kv_heads; s->G = G; s->D = p->head_dim;
  s->N = p->seq_len; s->W = p->window; s->Nc = s->N - s->W; s->B = p->budget; s->Bp = s->B - s->W;
  s->GW = G * s->W;
  s->QT = (s->GW + 31) / 32;
  s->chunk = stream_chunk_keys(p->dtype, p->head_dim);
  s->nchunks = (s->N + s->chunk - 1) / s->chunk;
  s->Npad = s->nchunks * s->chunk;
  s->units_per_layer = s->batch * s->hkv;
  s->nb_rows = (s->QT * 32 + 255) / 256 * 256;
  s->pool = p->pool; s->pool_k = p->pool == MIXKV_POOL_NONE ? 1 : p->pool_kernel;
  s->causal = p->causal_window; s->intrinsic = p->intrinsic; s->mix = p->mix;
  s->adaptive = p->budget_mode == MIXKV_BUDGET_HEAD_ADAPTIVE; s->floor_ = s->adaptive ? p->budget_floor : 0;
  s->per_head = p->budget_mode == MIXKV_BUDGET_PER_HEAD;
  s->scale_log2e = (float)((double)p->softmax_scale * 1.4426950408889634);
  s->eps = p->eps;
  s->kstats = 1;                                    // run() clears it when nothing reads the key statistics
  return MIXKV_OK;
}

// `select_only`: the layout of a call that only selects on the caller's scores (the budget table and
// the candidate lists; nothing of the scoring passes).
void carve_workspace(const Shape &s, int64_t units, Workspace *w, bool select_only) {
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + (select_only ? 0 : bytes), 256); return o; };
  auto take_sel = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
  const size_t QTR = (size_t)s.QT * 32;
  // one slot per run of the streaming kernels: each launch group owns kMaxStreamGrid + its units
  const size_t per_group = (size_t)kMaxStreamGrid + (size_t)kLayersPerLaunch * s.units_per_layer;
  const size_t groups = ((size_t)(units / s.units_per_layer) + kLayersPerLaunch - 1) / kLayersPerLaunch;
  w->budgets = take_sel(s.per_head ? (size_t)(units / s.units_per_layer) * s.hkv * 4 : 0);
  w->part_ml = take(groups * per_group * QTR * 8);
  w->part_ksum = take(groups * per_group * s.D * 4);
  w->rbar = take((size_t)units * 4);
  w->nb = take((size_t)units * s.nb_rows * 4);
  w->kbarp = take((size_t)units * 64 * 16);
  // per-key rows; the slack lets 16-byte vector loads of a row's tail run past the last row
  w->invnorm = take((size_t)units * s.Npad * 4 + 256);
  w->vnorm = take((size_t)units * s.Npad * 4 + 256);
  w->araw = take((size_t)units * s.Npad * 4 + 256);
  w->sdiv = take((size_t)units * s.Npad * 4 + 256);
  w->cand_idx = take_sel(s.adaptive ? (size_t)units * kMaxCandPerHead * 4 : 0);
  w->cand_key = take_sel(s.adaptive ? (size_t)units * kMaxCandPerHead * 4 : 0);
  w->scores = take((size_t)units * s.N * 4);
  w->total = off;
}

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

enum Stage { kScore = 1, kSelect = 2, kGather = 4 };

// Compute units of the current device (0 on failure); asked of the runtime once per device.
static int compute_units() {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static int cus[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
  std::lock_guard<std::mutex> lock(mu);
  if (cus[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) return 0;
    cus[dev] = n;
  }
  return cus[dev];
}

// Optional per-kernel timing: each launch is bracketed by a pair of events on the call's stream.
struct StageTimer {
  hipStream_t stream;
  float *ms;                                   // host [MIXKV_N_STAGES], may be null (no timing)
  hipEvent_t ev[2 * MIXKV_N_STAGES * (MIXKV_MAX_LAYERS / kLayersPerLaunch + 1)];
  int stage_of[MIXKV_N_STAGES * (MIXKV_MAX_LAYERS / kLayersPerLaunch + 1)];
  int n = 0;
  bool failed = false;
  template <class F> hipError_t operator()(int stage, F launch) {
    if (!ms) return launch();
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { failed = true; return launch(); }
    (void)hipEventRecord(a, stream);
    hipError_t e = launch();
    (void)hipEventRecord(b, stream);
    ev[2 * n] = a; ev[2 * n + 1] = b; stage_of[n] = stage; ++n;
    return e;
  }
  mixkv_status finish() {
    if (!ms) return MIXKV_OK;
    for (int i = 0; i < MIXKV_N_STAGES; ++i) ms[i] = 0.f;
    hipError_t e = hipStreamSynchronize(stream);
    for (int i = 0; i < n; ++i) {
      float t = 0.f;
      if (e == hipSuccess && hipEventElapsedTime(&t, ev[2 * i], ev[2 * i + 1]) == hipSuccess) ms[stage_of[i]] += t;
      (void)hipEventDestroy(ev[2 * i]);
      (void)hipEventDestroy(ev[2 * i + 1]);
    }
    return (e == hipSuccess && !failed) ? MIXKV_OK : MIXKV_ERR_HIP;
  }
};

static mixkv_status run(const mixkv_params *params, const mixkv_layer_in *in, mixkv_layer_out *out, int32_t n_layers,
                        void *workspace, size_t workspace_bytes, void *hip_stream, int stages,
                        float *stage_ms = nullptr) {
  Shape s;
  mixkv_status st = make_shape(params, &s);
  if (st != MIXKV_OK) return st;
  if (n_layers < 1 || n_layers > MIXKV_MAX_LAYERS || !out) return MIXKV_ERR_INVALID_ARG;
  if ((stages & (kScore | kGather)) && !in) return MIXKV_ERR_INVALID_ARG;
  const int eb = params->dtype == MIXKV_BF16 ? 2 : 4;
  const int64_t units = (int64_t)n_layers * s.units_per_layer;
  Workspace w;
  const bool select_only = stages == kSelect;
  carve_workspace(s, units, &w, select_only);
  // Selection on caller-provided scores needs no workspace, except for the per-head budget table.
  // Head-adaptive mode uses one for the heads' candidate lists if the caller brings it (one workgroup
  // per head, then a small split); without it one workgroup per batch item ranks all heads' scores.
  const bool stage_budgets = s.per_head && (stages & kSelect);
  if ((stages & kScore) || stage_budgets) {
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return MIXKV_ERR_INVALID_ARG;
    if (workspace_bytes < w.total) return MIXKV_ERR_WORKSPACE_TOO_SMALL;
  }
  const bool lists_fit = workspace && !(reinterpret_cast<uintptr_t>(workspace) & 255u) && workspace_bytes >= w.total;
  if (stage_budgets) {
    if (!params->head_budgets) return MIXKV_ERR_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l) {
      int64_t sum = 0;
      for (int h = 0; h < s.hkv; ++h) {
        const int32_t b = params->head_budgets[(size_t)l * s.hkv + h];
        if (b < s.W || b > s.N) return MIXKV_ERR_INVALID_ARG;
        sum += b;
      }
      if (sum > (int64_t)s.hkv * s.B) return MIXKV_ERR_INVALID_ARG;
    }
  }

  for (int l = 0; l < n_layers; ++l) {
    if (stages & (kScore | kGather)) {
      const mixkv_layer_in &li = in[l];
      if (!li.K || !li.V || !aligned16(li.K) || !aligned16(li.V)) return MIXKV_ERR_INVALID_ARG;
      if (li.kv_stride_n < s.D || li.kv_stride_h < 0 || li.kv_stride_b < 0) return MIXKV_ERR_INVALID_ARG;
      if ((li.kv_stride_n * eb) % 16 || (li.kv_stride_h * eb) % 16 || (li.kv_stride_b * eb) % 16) return MIXKV_ERR_INVALID_ARG;
      if ((stages & kScore) && (!li.Qwin || !aligned16(li.Qwin))) return MIXKV_ERR_INVALID_ARG;
      if ((stages & kScore) && s.mix == MIXKV_MIX_GIVEN_R && !li.r_given) return MIXKV_ERR_INVALID_ARG;
      if ((stages & kScore) && ((li.window_lse != nullptr) != (in[0].window_lse != nullptr))) return MIXKV_ERR_INVALID_ARG;
    }
    const mixkv_layer_out &lo = out[l];
    if (stages == kScore && !lo.scores) return MIXKV_ERR_INVALID_ARG;
    if (stages == kSelect && !lo.scores) return MIXKV_ERR_INVALID_ARG;
    if (stages & kSelect) {
      if (!lo.indices || !lo.counts) return MIXKV_ERR_INVALID_ARG;
      if ((s.adaptive || s.per_head) && !lo.offsets) return MIXKV_ERR_INVALID_ARG;
    }
    if (stages & kGather) {
      if (!lo.K_out || !lo.V_out || !aligned16(lo.K_out) || !aligned16(lo.V_out)) return MIXKV_ERR_INVALID_ARG;
    }
  }

  // The key statistics (1 / |K_i|, the mean normalised key, r) feed the diversity score, the head weight of
  // Eq. 5, the key-norm intrinsic score and the redundancy output.  The importance-only score of the
  // ablation (Table 4; the SnapKV-style base of Sec. 4.1) reads none of them unless the caller asks for r.
  if (stages & kScore) {
    bool wants_r = false;
    for (int l = 0; l < n_layers; ++l) wants_r = wants_r || out[l].redundancy != nullptr;
    s.kstats = (s.mix != MIXKV_MIX_IMP_ONLY || s.intrinsic == MIXKV_INTRINSIC_KNORM || wants_r) ? 1 : 0;
  }
  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  char *ws = reinterpret_cast<char *>(workspace);
  int num_cus = 0;
  if ((stages & kScore) && (num_cus = compute_units()) < 1) return MIXKV_ERR_HIP;
  const int32_t *budgets_dev = nullptr;
  if (stage_budgets) {
    int32_t *dst = reinterpret_cast<int32_t *>(ws + w.budgets);
    if (upload_ints(params->head_budgets, n_layers * s.hkv, dst, stream) != hipSuccess) return MIXKV_ERR_HIP;
    budgets_dev = dst;
  }
  StageTimer timed;
  timed.stream = stream;
  timed.ms = stage_ms;
  mixkv_status result = MIXKV_OK;
  auto ok = [&](hipError_t e) { if (e != hipSuccess) result = MIXKV_ERR_HIP; return e == hipSuccess; };
  for (int l0 = 0; l0 < n_layers; l0 += kLayersPerLaunch) {
    const int nl = (n_layers - l0 < kLayersPerLaunch) ? n_layers - l0 : kLayersPerLaunch;
    LayerInTable ti;
    LayerOutTable to;
    LseTable tl;
    std::memset(&ti, 0, sizeof(ti));
    std::memset(&to, 0, sizeof(to));
    std::memset(&tl, 0, sizeof(tl));
    const int64_t unit0 = (int64_t)l0 * s.units_per_layer;
    // One fused kernel mixes the scores and, in fixed-budget mode, selects; scores reach memory
    // only if somebody reads them (the caller, or the separate selection kernels).
    const bool fused = (stages & kScore) && mixsel_supported(s);
    const bool fused_select = fused && (stages & kSelect) && !s.adaptive;
    const bool fused_gather = fused_select && (stages & kGather);   // the selecting workgroup also copies its rows
    // head-adaptive mode: the fused kernel hands every head's best candidates to a small split kernel
    // selection alone: the same selection code on the caller's scores, one workgroup per head
    const bool topsel = select_only && mixsel_supported(s) && (!s.adaptive || (lists_fit && adaptive_candidates(s) > 0));
    const int cand_m = ((fused || topsel) && (stages & kSelect) && s.adaptive) ? adaptive_candidates(s) : 0;
    for (int l = 0; l < nl; ++l) {
      if (in) {
        const mixkv_layer_in &li = in[l0 + l];
        ti.l[l] = LayerIn{li.K, li.V, li.Qwin, li.kv_stride_b, li.kv_stride_h, li.kv_stride_n,
                          s.mix == MIXKV_MIX_GIVEN_R ? li.r_given : nullptr};
        tl.l[l] = li.window_lse;
      }
      const mixkv_layer_out &lo = out[l0 + l];
      float *scores = lo.scores;
      if (!scores && !fused_select && cand_m == 0)
        scores = reinterpret_cast<float *>(ws + w.scores) + (unit0 + (int64_t)l * s.units_per_layer) * s.N;
      to.l[l] = LayerOut{scores, lo.redundancy, lo.indices, lo.counts, lo.offsets, lo.K_out, lo.V_out};
    }
    const int nunits = nl * s.units_per_layer;
    const int32_t *budgets_l0 = budgets_dev ? budgets_dev + (size_t)l0 * s.hkv : nullptr;
    if (result == MIXKV_OK && (stages & kScore)) {
      const int grid = stream_grid(s, nunits, num_cus);
      const int64_t slot0 = (int64_t)(l0 / kLayersPerLaunch) * (kMaxStreamGrid + kLayersPerLaunch * s.units_per_layer);
      const bool given_lse = in[0].window_lse != nullptr;
      ok(timed(0, [&] { return launch_stats(s, params->dtype, ti, ws, w, unit0, nunits, grid, slot0, given_lse, stream); })) &&
          ok(timed(1, [&] {
            hipError_t e = launch_fold(s, params->dtype, to, tl, ws, w, unit0, nunits, grid, s.nchunks, slot0, stream);
            if (e != hipSuccess) return e;
            return launch_attn(s, params->dtype, ti, to, tl, ws, w, unit0, nunits, grid, slot0, stream);
          })) &&
          ok(timed(2, [&] {
            return fused ? launch_mixsel(s, fused_select || cand_m > 0, to, ws, w, unit0, nunits, ti,
                                         fused_gather ? eb : 0, cand_m, budgets_l0, stream)
                         : launch_mix(s, ti, to, ws, w, unit0, nunits, stream);
          }));
    }
    if (result == MIXKV_OK && topsel)
      ok(timed(3, [&] { return launch_topsel(s, to, ws, w, unit0, nunits, cand_m, budgets_l0, stream); }));
    if (result == MIXKV_OK && (stages & kSelect) && !fused_select && !(topsel && !s.adaptive))
      ok(timed(3, [&] {
        return cand_m > 0 ? launch_select_candidates(s, to, ws, w, unit0, nl, cand_m, stream) : launch_select(s, to, nl, budgets_l0, stream);
      }));
    if (result == MIXKV_OK && (stages & kGather) && !fused_gather)
      ok(timed(4, [&] { return launch_gather(s, params->dtype, ti, to, nl, stream); }));
    if (result != MIXKV_OK) break;
  }
  mixkv_status fin = timed.finish();
  return result != MIXKV_OK ? result : fin;
}

// The workspace of mixkv_compress_static: one array per GPU the library runs on, in the code object's
// own data, so it exists from the moment the library is loaded until the process ends.  In host code
// the array's name is only a handle for the symbol lookup: the device address is asked for once per
// device (with that device current) and everything else uses the address.
static __device__ __align__(256) unsigned char scratch[MIXKV_STATIC_SCRATCH_BYTES];

static mixkv_status static_scratch(void **ptr) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void *addr[kMaxDevices] = {};
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MIXKV_ERR_HIP;
  std::lock_guard<std::mutex> lock(mu);
  if (!addr[dev]) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MIXKV_ERR_HIP;
    if (reinterpret_cast<uintptr_t>(p) & 255u) return MIXKV_ERR_HIP;
    addr[dev] = p;
  }
  *ptr = addr[dev];
  return MIXKV_OK;
}

}  // namespace mixkv

extern "C" {

mixkv_status mixkv_workspace_size(const mixkv_params *params, int32_t n_layers, size_t *bytes) {
  mixkv::Shape s;
  mixkv_status st = mixkv::make_shape(params, &s);
  if (st != MIXKV_OK) return st;
  if (!bytes || n_layers < 1 || n_layers > MIXKV_MAX_LAYERS) return MIXKV_ERR_INVALID_ARG;
  mixkv::Workspace w;
  mixkv::carve_workspace(s, (int64_t)n_layers * s.units_per_layer, &w);
  *bytes = w.total;
  return MIXKV_OK;
}

mixkv_status mixkv_score(const mixkv_params *params, const mixkv_layer_in *in, mixkv_layer_out *out, int32_t n_layers,
                         void *workspace, size_t workspace_bytes, void *hip_stream) {
  return mixkv::run(params, in, out, n_layers, workspace, workspace_bytes, hip_stream, mixkv::kScore);
}

mixkv_status mixkv_select(const mixkv_params *params, mixkv_layer_out *out, int32_t n_layers, void *workspace,
                          size_t workspace_bytes, void *hip_stream) {
  return mixkv::run(params, nullptr, out, n_layers, workspace, workspace_bytes, hip_stream, mixkv::kSelect);
}

mixkv_status mixkv_compress(const mixkv_params *params, const mixkv_layer_in *in, mixkv_layer_out *out,
                            int32_t n_layers, void *workspace, size_t workspace_bytes, void *hip_stream) {
  return mixkv::run(params, in, out, n_layers, workspace, workspace_bytes, hip_stream,
                    mixkv::kScore | mixkv::kSelect | mixkv::kGather);
}

mixkv_status mixkv_compress_profiled(const mixkv_params *params, const mixkv_layer_in *in, mixkv_layer_out *out,
                                     int32_t n_layers, void *workspace, size_t workspace_bytes, void *hip_stream,
                                     float *stage_ms) {
  if (!stage_ms) return MIXKV_ERR_INVALID_ARG;
  return mixkv::run(params, in, out, n_layers, workspace, workspace_bytes, hip_stream,
                    mixkv::kScore | mixkv::kSelect | mixkv::kGather, stage_ms);
}

mixkv_status mixkv_compress_static(const mixkv_params *params, const mixkv_layer_in *in, mixkv_layer_out *out,
                                   int32_t n_layers, void *hip_stream) {
  mixkv::Shape s;
  mixkv_status st = mixkv::make_shape(params, &s);
  if (st != MIXKV_OK) return st;
  if (n_layers < 1 || n_layers > MIXKV_MAX_LAYERS) return MIXKV_ERR_INVALID_ARG;
  mixkv::Workspace w;
  mixkv::carve_workspace(s, (int64_t)n_layers * s.units_per_layer, &w);
  if (w.total > (size_t)MIXKV_STATIC_SCRATCH_BYTES) return MIXKV_ERR_WORKSPACE_TOO_SMALL;
  void *ws = nullptr;
  st = mixkv::static_scratch(&ws);
  if (st != MIXKV_OK) return st;
  return mixkv::run(params, in, out, n_layers, ws, MIXKV_STATIC_SCRATCH_BYTES, hip_stream,
                    mixkv::kScore | mixkv::kSelect | mixkv::kGather);
}

const char *mixkv_stage_name(int32_t stage) {
  static const char *names[MIXKV_N_STAGES] = {"stats", "attn", "mix", "select", "gather"};
  return (stage >= 0 && stage < MIXKV_N_STAGES) ? names[stage] : "";
}

const char *mixkv_status_string(mixkv_status status) {
  switch (status) {
    case MIXKV_OK: return "ok";
    case MIXKV_ERR_INVALID_ARG: return "invalid argument";
    case MIXKV_ERR_UNSUPPORTED: return "unsupported configuration";
    case MIXKV_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case MIXKV_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

int32_t mixkv_version(void) { return MIXKV_VERSION; }

}  // extern "C"
