/*
 * harli_sched.h -- latency predictor, allocation choice and compute-unit partitions of the
 * co-location scheduler (Harli Sec. 5 and Sec. 6.2).  Host-side arithmetic in double precision, plus two
 * calls that create / destroy HIP streams restricted to a range of compute units (the MI355X counterpart of
 * the paper's per-stream SM partitions, Sec. 7).
 */
#ifndef HARLI_SCHED_H
#define HARLI_SCHED_H

#include "harli.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct harli_predictor harli_predictor;

/* A predictor over n_levels compute-unit ratios 1/n_levels, 2/n_levels, ..., 1 (the paper uses ten, Sec. 5.1).
 * n_levels in 2..64.  Level indices below are 1-based: level i means ratio i / n_levels. */
harli_status harli_pred_create(int32_t n_levels, harli_predictor** out);
void harli_pred_destroy(harli_predictor* p);

/* One profiled solo decode step at compute-unit level `level`: batch size, sequence length, measured latency
 * (any unit, used consistently).  Samples accumulate until harli_pred_fit. */
harli_status harli_pred_add_solo(harli_predictor* p, int32_t level, int32_t bs, int32_t seqlen, double latency);
/* One profiled co-located decode step: inference at `infer_level`, finetune at `ft_level`
 * (infer_level + ft_level <= n_levels), measured co-located latency and the solo latency of the same
 * (bs, seqlen) at infer_level. */
harli_status harli_pred_add_colo(harli_predictor* p, int32_t infer_level, int32_t ft_level, double latency_colo,
                                 double latency_solo);

/* Ordinary least squares (Householder QR) of
 *   Eq. 1 per level:  latency = bs*b0 + c0 + bs*k0*seqlen           (needs >= 3 samples at that level)
 *   Eq. 2 overall:    latency_colo = (SM_infer*b1 + SM_ft*k1) * latency_solo   (needs >= 2 samples; optional)
 *                     Predictions floor the factor at 1 (see harli_pred_colo), and a sample whose fitted factor is
 *                     below 1 is then predicted by the floor whatever b1 and k1 are: after the pass over all samples
 *                     the fit is repeated over the samples whose current factor is at least 1 until that set is
 *                     stable.  With every sample in the contended regime this is the plain least-squares fit.
 * Levels without samples stay unfitted; HARLI_ERR_STATE if a sampled level has fewer than 3 samples or a
 * rank-deficient design (e.g. one batch size only). */
harli_status harli_pred_fit(harli_predictor* p);

/* Which reading of Eq. 2 (Sec. 5.2.1) the fit and the co-located predictions use.  enabled != 0 (the state after
 * create): the factor SM_infer*b1 + SM_ft*k1 is floored at 1 and the fit leaves out the samples the floor covers, as
 * described at harli_pred_fit.  enabled == 0: Eq. 2 exactly as printed -- one ordinary least-squares fit over every
 * sample, predictions without a floor -- so that the paper's accuracy figure for this model (Sec. 8.4) can be
 * evaluated as written.  Changing the reading discards the co-located fit (the samples stay): call harli_pred_fit
 * again before the next co-located prediction. */
harli_status harli_pred_set_colo_floor(harli_predictor* p, int32_t enabled);

/* Calibration (an addition to the paper's predictor): every prediction at `level` -- alone, co-located, in
 * harli_sched_pick and in the runtime scheduler -- is Eq. 1's value times `scale` (> 0; 1 after create).  A caller that
 * times its decode steps at run time folds the ratio measured / predicted back in here; the fitted coefficients
 * (harli_pred_solo_coef) are not changed.  HARLI_ERR_INVALID for a level outside 1..n_levels or a scale that is not a
 * positive finite number. */
harli_status harli_pred_set_scale(harli_predictor* p, int32_t level, double scale);
harli_status harli_pred_get_scale(const harli_predictor* p, int32_t level, double* scale /* host out */);
/* Run-time feedback into that factor: one finished decode step at `level` took measured_ms where Eq. 1 (and Eq. 2 when a
 * finetune task ran beside it) WITHOUT the calibration factor gave predicted_ms -- a caller that planned with a calibrated
 * prediction divides it by the factor harli_pred_get_scale returned at planning time.  With r = measured / predicted
 * clipped to [0.6, 2.5]: the first observation of a level sets its factor to r, later ones move it by weight * (r -
 * factor) (0 < weight <= 1); every level that has not been observed yet takes the observed level's new factor, so a plan
 * that moves to a fresh partition starts from the latest evidence.  harli_pred_set_scale puts a level back to "not
 * observed".  HARLI_ERR_INVALID for a level outside 1..n_levels, times that are not positive finite numbers, or a weight
 * outside (0, 1]. */
harli_status harli_pred_observe(harli_predictor* p, int32_t level, double predicted_ms, double measured_ms, double weight);

/* Coefficients after a fit (host out-pointers): solo[3] = b0, c0, k0 of `level`; colo[2] = b1, k1.
 * HARLI_ERR_STATE when that model has not been fitted. */
harli_status harli_pred_solo_coef(const harli_predictor* p, int32_t level, double* solo);
harli_status harli_pred_colo_coef(const harli_predictor* p, double* colo);

/* Eq. 1 per kernel family.  Eq. 1 is one line in the batch size; the decode step of this library runs two kernel
 * families, each linear with a slope of its own (weight-streaming GEMMs, and from harli_decode_tiled_min_batch()
 * sequences on tiled GEMMs), and one line through both is off by up to 25 % at the switch.  bs_split > 0: samples and
 * predictions with bs >= bs_split use a second set of Eq. 1 coefficients per level (harli_pred_solo_coef_upper); a
 * family whose samples of a level do not determine a line (fewer than three, one batch size, one sequence length)
 * takes the other family's line.  0, the default: one line per level, Eq. 1 as printed.  A change discards the solo
 * fits (call harli_pred_fit again); calibration factors and the co-located fit stay. */
harli_status harli_pred_set_batch_split(harli_predictor* p, int32_t bs_split);
harli_status harli_pred_solo_coef_upper(const harli_predictor* p, int32_t level, double* solo);

/* Predictions (host out-pointer).  Co-located: max(1, SM_infer*b1 + SM_ft*k1) * solo(infer_level): Eq. 2's slowdown
 * factor is derived (Sec. 5.2.2) for the contended case only, where it is at least 1; below that the two tasks do not
 * contend and the prediction is the solo latency. */
harli_status harli_pred_solo(const harli_predictor* p, int32_t level, int32_t bs, int32_t seqlen, double* latency);
harli_status harli_pred_colo(const harli_predictor* p, int32_t infer_level, int32_t ft_level, int32_t bs, int32_t seqlen,
                             double* latency);

/* Allocation for the next decode phase (Sec. 5.2, 6.2): over all pairs (infer_level, ft_level) with
 * infer_level + ft_level <= n_levels, both >= 1, whose predicted co-located latency is <= slo, the pair with the
 * largest predicted latency (closest to the target without exceeding it); ties go to the larger ft_level, then
 * to the smaller infer_level.  When no pair qualifies: infer_level = n_levels, ft_level = 0 (finetune paused,
 * every compute unit to inference) and the solo prediction at the full level.  Every level must be fitted. */
harli_status harli_sched_pick(const harli_predictor* p, int32_t bs, int32_t seqlen, double slo, int32_t* infer_level,
                              int32_t* ft_level, double* predicted);

/* Runtime scheduling (Sec. 6.2): one decision at the beginning of every decode phase. */
typedef struct harli_scheduler harli_scheduler;

enum {
  HARLI_SCHED_KEEP = 0,    /* the plan in force still meets the target: both tasks continue */
  HARLI_SCHED_REPLAN = 1,  /* new plan: pause the finetune task (let its unit in flight finish) before switching */
  HARLI_SCHED_PAUSED = 2,  /* no plan meets the target: finetune stays paused, inference gets every compute unit */
  HARLI_SCHED_STARVED = 3  /* the finetune task has no ready work: inference gets every compute unit this phase */
};

typedef struct harli_sched_decision {
  int32_t infer_level; /* 1..n_levels */
  int32_t ft_level;    /* 0 = finetune does not run in this phase */
  int32_t action;      /* HARLI_SCHED_* */
  double predicted;    /* predicted decode latency of this phase under the decision */
} harli_sched_decision;

/* `p` must be fully fitted and outlive the scheduler.  slo > 0 in the predictor's latency unit.  refresh_phases >= 0:
 * after that many consecutive phases under one plan the choice is recomputed even though the plan still meets the
 * target (0 = never; the paper reports adjustments about every 100 ms, Sec. 8.6, without giving the rule). */
harli_status harli_sched_create(const harli_predictor* p, double slo, int32_t refresh_phases, harli_scheduler** out);
void harli_sched_destroy(harli_scheduler* s);

/* Decision for the decode phase that is about to start: batch size bs >= 1, sequence length seqlen >= 0, ft_ready
 * non-zero when the finetune task has a unit ready to run.  Rules, in this order: not ready -> STARVED (all compute
 * units to inference, plan dropped); no plan in force -> harli_sched_pick (REPLAN, or PAUSED when no pair meets the
 * target); plan in force and its predicted co-located latency above the target -> harli_sched_pick likewise;
 * otherwise KEEP, except that a plan older than refresh_phases is recomputed (REPLAN only if the pair changes).
 * *out is a host pointer. */
harli_status harli_sched_step(harli_scheduler* s, int32_t bs, int32_t seqlen, int32_t ft_ready, harli_sched_decision* out);

/* A HIP stream (default priority) whose kernels run only on compute units [cu_first, cu_first + cu_count) of the
 * current device's compute-unit mask order; the runtime spreads consecutive mask bits round-robin over the XCDs,
 * so a contiguous range is an equal share of every XCD.  *hip_stream receives a hipStream_t.  Ranges outside
 * 0..multiProcessorCount or empty ranges give HARLI_ERR_INVALID.  Only contiguous ranges are offered. */
harli_status harli_cu_stream_create(int32_t cu_first, int32_t cu_count, void** hip_stream);
harli_status harli_cu_stream_destroy(void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* HARLI_SCHED_H */
