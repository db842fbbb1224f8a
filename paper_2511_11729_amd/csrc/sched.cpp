// Latency predictor, allocation choice and compute-unit partitions (Harli Sec. 5, Sec. 6.2, Sec. 7).
// Host code only.  The two regressions are ordinary least squares solved by Householder QR in double precision.
#include <hip/hip_runtime.h>

#include <cmath>
#include <map>
#include <mutex>
#include <vector>

#include "common.h"
#include "harli_sched.h"

using namespace harli;

namespace {

struct SoloSample {
  double bs, seqlen, lat;
};
struct ColoSample {
  double sm_i, sm_f, colo, solo;
};

// min ||X beta - y||_2 for an n x m design (row-major), m <= 3; false when rank deficient
bool lstsq(std::vector<double> X, std::vector<double> y, int n, int m, double* beta) {
  double col_scale = 0.0;
  for (double v : X) col_scale = std::fmax(col_scale, std::fabs(v));
  for (int k = 0; k < m; ++k) {
    double norm = 0.0;
    for (int i = k; i < n; ++i) norm += X[i * m + k] * X[i * m + k];
    norm = std::sqrt(norm);
    if (!(norm > 1e-13 * col_scale * std::sqrt((double)n))) return false;
    const double alpha = X[k * m + k] > 0 ? -norm : norm;
    std::vector<double> v(n - k);
    for (int i = k; i < n; ++i) v[i - k] = X[i * m + k];
    v[0] -= alpha;
    double vv = 0.0;
    for (double t : v) vv += t * t;
    if (vv > 0.0) {
      for (int j = k; j < m; ++j) {
        double dot = 0.0;
        for (int i = k; i < n; ++i) dot += v[i - k] * X[i * m + j];
        const double f = 2.0 * dot / vv;
        for (int i = k; i < n; ++i) X[i * m + j] -= f * v[i - k];
      }
      double dot = 0.0;
      for (int i = k; i < n; ++i) dot += v[i - k] * y[i];
      const double f = 2.0 * dot / vv;
      for (int i = k; i < n; ++i) y[i] -= f * v[i - k];
    }
  }
  for (int k = m - 1; k >= 0; --k) {
    double s = y[k];
    for (int j = k + 1; j < m; ++j) s -= X[k * m + j] * beta[j];
    beta[k] = s / X[k * m + k];
  }
  return true;
}

}  // namespace

struct harli_predictor {
  int n_levels = 0;
  std::vector<std::vector<SoloSample>> solo;  // per level (index level-1)
  std::vector<ColoSample> colo;
  std::vector<double> coef;       // 3 per level
  std::vector<double> coef_hi;    // 3 per level: the line for batches from bs_split on (equal to coef without a split)
  int bs_split = 0;               // 0: one line per level (Eq. 1 as printed)
  std::vector<char> fitted;       // per level
  std::vector<double> scale;      // per level: calibration factor on Eq. 1's prediction (1 unless the caller sets it)
  std::vector<char> observed;     // per level: a measured step has been folded into `scale` (harli_pred_observe)
  double b1 = 0, k1 = 0;
  bool colo_fitted = false;
  bool colo_floor = true;         // Eq. 2's factor floored at 1 (this library's reading); false: Eq. 2 as printed
};

namespace {
constexpr double kScaleMin = 0.6, kScaleMax = 2.5;  // one measured step moves a prediction by no more than this
bool level_ok(const harli_predictor* p, int level) { return level >= 1 && level <= p->n_levels; }
double eval_solo(const harli_predictor* p, int level, double bs, double seqlen) {
  const std::vector<double>& all = (p->bs_split > 0 && bs >= p->bs_split) ? p->coef_hi : p->coef;
  const double* c = &all[(size_t)(level - 1) * 3];
  return p->scale[level - 1] * (bs * c[0] + c[1] + bs * c[2] * seqlen);
}
// Eq. 2, with the slowdown factor floored at 1: the paper derives the factor as (f_infer + f_ft) / B for the
// contended case f_infer + f_ft > B only; without contention the co-located latency is the solo latency.
double eval_colo(const harli_predictor* p, int il, int fl, double solo) {
  const double factor = (double)il / p->n_levels * p->b1 + (double)fl / p->n_levels * p->k1;
  return (p->colo_floor && factor < 1.0 ? 1.0 : factor) * solo;
}
}  // namespace

extern "C" harli_status harli_pred_create(int32_t n_levels, harli_predictor** out) {
  if (!out || n_levels < 2 || n_levels > 64) return fail(HARLI_ERR_INVALID, "pred_create: n_levels %d outside 2..64", n_levels);
  harli_predictor* p = new harli_predictor;
  p->n_levels = n_levels;
  p->solo.resize(n_levels);
  p->coef.assign((size_t)n_levels * 3, 0.0);
  p->coef_hi.assign((size_t)n_levels * 3, 0.0);
  p->fitted.assign(n_levels, 0);
  p->scale.assign(n_levels, 1.0);
  p->observed.assign(n_levels, 0);
  *out = p;
  return HARLI_OK;
}

extern "C" void harli_pred_destroy(harli_predictor* p) { delete p; }

extern "C" harli_status harli_pred_add_solo(harli_predictor* p, int32_t level, int32_t bs, int32_t seqlen, double latency) {
  if (!p || !level_ok(p, level) || bs < 1 || seqlen < 0 || !(latency > 0.0) || !std::isfinite(latency))
    return fail(HARLI_ERR_INVALID, "pred_add_solo: bad sample (level %d bs %d seqlen %d)", level, bs, seqlen);
  p->solo[level - 1].push_back(SoloSample{(double)bs, (double)seqlen, latency});
  return HARLI_OK;
}

extern "C" harli_status harli_pred_add_colo(harli_predictor* p, int32_t infer_level, int32_t ft_level, double latency_colo,
                                            double latency_solo) {
  if (!p || !level_ok(p, infer_level) || ft_level < 1 || infer_level + ft_level > p->n_levels || !(latency_colo > 0.0) ||
      !(latency_solo > 0.0) || !std::isfinite(latency_colo) || !std::isfinite(latency_solo))
    return fail(HARLI_ERR_INVALID, "pred_add_colo: bad sample (levels %d + %d)", infer_level, ft_level);
  p->colo.push_back(ColoSample{(double)infer_level / p->n_levels, (double)ft_level / p->n_levels, latency_colo, latency_solo});
  return HARLI_OK;
}

extern "C" harli_status harli_pred_fit(harli_predictor* p) {
  if (!p) return fail(HARLI_ERR_INVALID, "pred_fit: null predictor");
  for (int l = 0; l < p->n_levels; ++l) {
    const std::vector<SoloSample>& s = p->solo[l];
    if (s.empty()) continue;
    const int n = (int)s.size();
    if (n < 3) return fail(HARLI_ERR_STATE, "pred_fit: level %d has %d samples, Eq. 1 needs 3", l + 1, n);
    // one least-squares line per batch family (a single family without a split)
    auto fit_family = [&](bool upper, double* beta) -> bool {
      std::vector<double> X, y;
      for (const SoloSample& q : s) {
        if (p->bs_split > 0 && (q.bs >= p->bs_split) != upper) continue;
        X.push_back(q.bs);
        X.push_back(1.0);
        X.push_back(q.bs * q.seqlen);
        y.push_back(q.lat);
      }
      const int m = (int)y.size();
      return m >= 3 && lstsq(X, y, m, 3, beta);
    };
    double lo[3], hi[3];
    const bool ok_lo = fit_family(false, lo), ok_hi = p->bs_split > 0 && fit_family(true, hi);
    if (!ok_lo && !ok_hi)
      return fail(HARLI_ERR_STATE, "pred_fit: level %d samples do not determine Eq. 1 (vary batch size and sequence length)", l + 1);
    // a family the samples do not determine takes the other family's line
    for (int i = 0; i < 3; ++i) {
      p->coef[(size_t)l * 3 + i] = ok_lo ? lo[i] : hi[i];
      p->coef_hi[(size_t)l * 3 + i] = ok_hi ? hi[i] : lo[i];
    }
    p->fitted[l] = 1;
  }
  if (!p->colo.empty()) {
    const int n = (int)p->colo.size();
    if (n < 2) return fail(HARLI_ERR_STATE, "pred_fit: Eq. 2 needs at least 2 co-located samples");
    std::vector<double> X((size_t)n * 2), y(n);
    for (int i = 0; i < n; ++i) {
      X[i * 2 + 0] = p->colo[i].sm_i * p->colo[i].solo;
      X[i * 2 + 1] = p->colo[i].sm_f * p->colo[i].solo;
      y[i] = p->colo[i].colo;
    }
    double b[2];
    if (!lstsq(X, y, n, 2, b)) return fail(HARLI_ERR_STATE, "pred_fit: co-located samples do not determine Eq. 2");
    // Prediction floors the factor at 1, so a sample whose fitted factor is below 1 says nothing about b1, k1:
    // repeat the fit over the samples the floor does not cover until that set is stable.
    std::vector<char> active(n, 1), now(n);
    for (int round = 0; p->colo_floor && round < 32; ++round) {
      int cnt = 0;
      bool same = true;
      for (int i = 0; i < n; ++i) {
        now[i] = p->colo[i].sm_i * b[0] + p->colo[i].sm_f * b[1] >= 1.0;
        cnt += now[i];
        same = same && now[i] == active[i];
      }
      if (same || cnt < 2) break;
      std::vector<double> Xa, ya;
      for (int i = 0; i < n; ++i)
        if (now[i]) {
          Xa.push_back(X[i * 2 + 0]);
          Xa.push_back(X[i * 2 + 1]);
          ya.push_back(y[i]);
        }
      double nb[2];
      if (!lstsq(Xa, ya, cnt, 2, nb)) break;
      active = now;
      b[0] = nb[0];
      b[1] = nb[1];
    }
    p->b1 = b[0];
    p->k1 = b[1];
    p->colo_fitted = true;
  }
  return HARLI_OK;
}

extern "C" harli_status harli_pred_set_colo_floor(harli_predictor* p, int32_t enabled) {
  if (!p) return fail(HARLI_ERR_INVALID, "pred_set_colo_floor: null predictor");
  p->colo_floor = enabled != 0;
  p->colo_fitted = false;  // the fit depends on the reading: fit again
  return HARLI_OK;
}

extern "C" harli_status harli_pred_set_scale(harli_predictor* p, int32_t level, double scale) {
  if (!p || !level_ok(p, level) || !(scale > 0.0) || !std::isfinite(scale))
    return fail(HARLI_ERR_INVALID, "pred_set_scale: bad argument (level %d, scale %g)", level, scale);
  p->scale[level - 1] = scale;
  p->observed[level - 1] = 0;  // a factor set by hand is a prior: the first measured step replaces it
  return HARLI_OK;
}

extern "C" harli_status harli_pred_get_scale(const harli_predictor* p, int32_t level, double* scale) {
  if (!p || !scale || !level_ok(p, level)) return fail(HARLI_ERR_INVALID, "pred_get_scale: bad argument");
  *scale = p->scale[level - 1];
  return HARLI_OK;
}

extern "C" harli_status harli_pred_observe(harli_predictor* p, int32_t level, double predicted_ms, double measured_ms,
                                           double weight) {
  if (!p || !level_ok(p, level) || !(predicted_ms > 0.0) || !std::isfinite(predicted_ms) || !(measured_ms > 0.0) ||
      !std::isfinite(measured_ms) || !(weight > 0.0) || !(weight <= 1.0))
    return fail(HARLI_ERR_INVALID, "pred_observe: bad argument (level %d, predicted %g, measured %g, weight %g)", level,
                predicted_ms, measured_ms, weight);
  double r = measured_ms / predicted_ms;
  r = r < kScaleMin ? kScaleMin : r > kScaleMax ? kScaleMax : r;
  double& s = p->scale[level - 1];
  if (p->observed[level - 1]) s += weight * (r - s);
  else s = r;  // the first measurement of a level is taken whole
  p->observed[level - 1] = 1;
  for (int l = 0; l < p->n_levels; ++l)  // levels never measured borrow from the one measured last
    if (!p->observed[l]) p->scale[l] = s;
  return HARLI_OK;
}

extern "C" harli_status harli_pred_solo_coef(const harli_predictor* p, int32_t level, double* solo) {
  if (!p || !solo || !level_ok(p, level)) return fail(HARLI_ERR_INVALID, "pred_solo_coef: bad argument");
  if (!p->fitted[level - 1]) return fail(HARLI_ERR_STATE, "pred_solo_coef: level %d is not fitted", level);
  for (int i = 0; i < 3; ++i) solo[i] = p->coef[(size_t)(level - 1) * 3 + i];
  return HARLI_OK;
}

extern "C" harli_status harli_pred_solo_coef_upper(const harli_predictor* p, int32_t level, double* solo) {
  if (!p || !solo || !level_ok(p, level)) return fail(HARLI_ERR_INVALID, "pred_solo_coef_upper: bad argument");
  if (!p->fitted[level - 1]) return fail(HARLI_ERR_STATE, "pred_solo_coef_upper: level %d is not fitted", level);
  for (int i = 0; i < 3; ++i) solo[i] = p->coef_hi[(size_t)(level - 1) * 3 + i];
  return HARLI_OK;
}

extern "C" harli_status harli_pred_set_batch_split(harli_predictor* p, int32_t bs_split) {
  if (!p || bs_split < 0) return fail(HARLI_ERR_INVALID, "pred_set_batch_split: bad argument");
  if (bs_split != p->bs_split) {
    p->bs_split = bs_split;
    std::fill(p->fitted.begin(), p->fitted.end(), 0);  // the lines were fitted for the other reading
  }
  return HARLI_OK;
}

extern "C" harli_status harli_pred_colo_coef(const harli_predictor* p, double* colo) {
  if (!p || !colo) return fail(HARLI_ERR_INVALID, "pred_colo_coef: bad argument");
  if (!p->colo_fitted) return fail(HARLI_ERR_STATE, "pred_colo_coef: Eq. 2 is not fitted");
  colo[0] = p->b1;
  colo[1] = p->k1;
  return HARLI_OK;
}

extern "C" harli_status harli_pred_solo(const harli_predictor* p, int32_t level, int32_t bs, int32_t seqlen, double* latency) {
  if (!p || !latency || !level_ok(p, level) || bs < 1 || seqlen < 0) return fail(HARLI_ERR_INVALID, "pred_solo: bad argument");
  if (!p->fitted[level - 1]) return fail(HARLI_ERR_STATE, "pred_solo: level %d is not fitted", level);
  *latency = eval_solo(p, level, bs, seqlen);
  return HARLI_OK;
}

extern "C" harli_status harli_pred_colo(const harli_predictor* p, int32_t infer_level, int32_t ft_level, int32_t bs,
                                        int32_t seqlen, double* latency) {
  if (!p || !latency || !level_ok(p, infer_level) || ft_level < 1 || infer_level + ft_level > p->n_levels || bs < 1 || seqlen < 0)
    return fail(HARLI_ERR_INVALID, "pred_colo: bad argument");
  if (!p->fitted[infer_level - 1] || !p->colo_fitted) return fail(HARLI_ERR_STATE, "pred_colo: models are not fitted");
  *latency = eval_colo(p, infer_level, ft_level, eval_solo(p, infer_level, bs, seqlen));
  return HARLI_OK;
}

extern "C" harli_status harli_sched_pick(const harli_predictor* p, int32_t bs, int32_t seqlen, double slo, int32_t* infer_level,
                                         int32_t* ft_level, double* predicted) {
  if (!p || !infer_level || !ft_level || !predicted || bs < 1 || seqlen < 0 || !(slo > 0.0))
    return fail(HARLI_ERR_INVALID, "sched_pick: bad argument");
  if (!p->colo_fitted) return fail(HARLI_ERR_STATE, "sched_pick: Eq. 2 is not fitted");
  for (int l = 0; l < p->n_levels; ++l)
    if (!p->fitted[l]) return fail(HARLI_ERR_STATE, "sched_pick: level %d is not fitted", l + 1);
  bool have = false;
  int bi = 0, bf = 0;
  double bl = 0.0;
  for (int i = 1; i < p->n_levels; ++i)
    for (int f = 1; i + f <= p->n_levels; ++f) {
      const double lat = eval_colo(p, i, f, eval_solo(p, i, bs, seqlen));
      if (!(lat <= slo)) continue;
      const bool better = !have || lat > bl || (lat == bl && (f > bf || (f == bf && i < bi)));
      if (better) {
        have = true;
        bi = i;
        bf = f;
        bl = lat;
      }
    }
  if (!have) {
    bi = p->n_levels;
    bf = 0;
    bl = eval_solo(p, p->n_levels, bs, seqlen);
  }
  *infer_level = bi;
  *ft_level = bf;
  *predicted = bl;
  return HARLI_OK;
}

struct harli_scheduler {
  const harli_predictor* p;
  double slo;
  int refresh;
  bool have;  // a plan is in force
  int i, f, age;
};

extern "C" harli_status harli_sched_create(const harli_predictor* p, double slo, int32_t refresh_phases, harli_scheduler** out) {
  if (!p || !out || !(slo > 0.0) || refresh_phases < 0) return fail(HARLI_ERR_INVALID, "sched_create: bad argument");
  if (!p->colo_fitted) return fail(HARLI_ERR_STATE, "sched_create: Eq. 2 is not fitted");
  for (int l = 0; l < p->n_levels; ++l)
    if (!p->fitted[l]) return fail(HARLI_ERR_STATE, "sched_create: level %d is not fitted", l + 1);
  *out = new harli_scheduler{p, slo, refresh_phases, false, 0, 0, 0};
  return HARLI_OK;
}

extern "C" void harli_sched_destroy(harli_scheduler* s) { delete s; }

static harli_status sched_replan(harli_scheduler* s, int bs, int seqlen, harli_sched_decision* out) {
  int32_t i = 0, f = 0;
  double lat = 0.0;
  harli_status rc = harli_sched_pick(s->p, bs, seqlen, s->slo, &i, &f, &lat);
  if (rc != HARLI_OK) return rc;
  s->age = 0;
  s->have = f > 0;
  s->i = i;
  s->f = f;
  *out = harli_sched_decision{i, f, f > 0 ? HARLI_SCHED_REPLAN : HARLI_SCHED_PAUSED, lat};
  return HARLI_OK;
}

extern "C" harli_status harli_sched_step(harli_scheduler* s, int32_t bs, int32_t seqlen, int32_t ft_ready, harli_sched_decision* out) {
  if (!s || !out || bs < 1 || seqlen < 0) return fail(HARLI_ERR_INVALID, "sched_step: bad argument");
  const harli_predictor* p = s->p;
  if (!ft_ready) {
    s->have = false;
    s->age = 0;
    *out = harli_sched_decision{p->n_levels, 0, HARLI_SCHED_STARVED, eval_solo(p, p->n_levels, bs, seqlen)};
    return HARLI_OK;
  }
  if (!s->have) return sched_replan(s, bs, seqlen, out);
  const double lat = eval_colo(p, s->i, s->f, eval_solo(p, s->i, bs, seqlen));
  if (lat > s->slo) return sched_replan(s, bs, seqlen, out);
  s->age += 1;
  if (s->refresh > 0 && s->age >= s->refresh) {
    const int oi = s->i, of = s->f;
    harli_status rc = sched_replan(s, bs, seqlen, out);
    if (rc == HARLI_OK && out->action == HARLI_SCHED_REPLAN && out->infer_level == oi && out->ft_level == of) out->action = HARLI_SCHED_KEEP;
    return rc;
  }
  *out = harli_sched_decision{s->i, s->f, HARLI_SCHED_KEEP, lat};
  return HARLI_OK;
}

// streams made here and the number of compute units each may use: the weight GEMM sizes its last round of tiles for it
namespace {
std::mutex g_cu_mu;
std::map<void*, int> g_cu_streams;
}  // namespace
namespace harli {
int cu_stream_count(void* hip_stream) {
  std::lock_guard<std::mutex> lk(g_cu_mu);
  auto it = g_cu_streams.find(hip_stream);
  return it == g_cu_streams.end() ? 0 : it->second;
}
}  // namespace harli

extern "C" harli_status harli_cu_stream_create(int32_t cu_first, int32_t cu_count, void** hip_stream) {
  if (!hip_stream) return fail(HARLI_ERR_INVALID, "cu_stream_create: null out pointer");
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess)
    return fail(HARLI_ERR_HIP, "cu_stream_create: no HIP device available");
  const int n_cu = prop.multiProcessorCount;
  if (cu_first < 0 || cu_count < 1 || cu_first + cu_count > n_cu)
    return fail(HARLI_ERR_INVALID, "cu_stream_create: range [%d, %d) outside the device's %d compute units", cu_first,
                cu_first + cu_count, n_cu);
  std::vector<uint32_t> mask((n_cu + 31) / 32, 0u);
  for (int c = cu_first; c < cu_first + cu_count; ++c) mask[c >> 5] |= 1u << (c & 31);
  hipStream_t st = nullptr;
  hipError_t e = hipExtStreamCreateWithCUMask(&st, (uint32_t)mask.size(), mask.data());
  if (e != hipSuccess) return fail(HARLI_ERR_HIP, "cu_stream_create: %s", hipGetErrorString(e));
  {
    std::lock_guard<std::mutex> lk(g_cu_mu);
    g_cu_streams[st] = cu_count;
  }
  *hip_stream = st;
  return HARLI_OK;
}

extern "C" harli_status harli_cu_stream_destroy(void* hip_stream) {
  if (!hip_stream) return fail(HARLI_ERR_INVALID, "cu_stream_destroy: null stream");
  {
    std::lock_guard<std::mutex> lk(g_cu_mu);
    g_cu_streams.erase(hip_stream);
  }
  hipError_t e = hipStreamDestroy(static_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail(HARLI_ERR_HIP, "cu_stream_destroy: %s", hipGetErrorString(e));
  return HARLI_OK;
}
