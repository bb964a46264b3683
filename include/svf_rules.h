/*
 * libsvf - the two per-token rules beside the sparse verification kernels, on AMD MI355X:
 * expert skipping of the sparse mixture of experts (Sec. 3.5, Eq. 15-16) and the acceptance /
 * resampling of the draft tokens (Sec. 2.1, Eq. 2-3).
 *
 * Conventions as in svf.h: every pointer is a DEVICE pointer owned by the caller unless said
 * otherwise; work is enqueued on `stream` and the call returns immediately; 0 on success, a
 * negative SVF_ERR_* code (svf.h) otherwise, checked before any launch; inputs must be finite.
 */
#ifndef SVF_RULES_H_
#define SVF_RULES_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Expert skipping (Eq. 16).  w: fp32 [T][k], the routing weights of the k experts each of T tokens
 * was routed to (any order, positive); beta: fp32 [k-1], the layer's threshold map; m: the skipping
 * budget, 1 <= m < k <= 32.  With the weights of a token in ascending order (equal weights: the
 * expert listed first is the lower one) and r_i = (w_1 + .. + w_i) / (w_1 + .. + w_k), the share of
 * the routing mass the i lowest experts carry, the token skips its i lowest experts for the
 * largest i <= m with r_i < beta[i-1], none if there is no such i.  (Eq. 15-16 print the sum over
 * the first k - i weights; this is the reading under which the skipped experts are the lowest
 * ones and, for k = 2, the rule is the two-expert rule the section generalises.)
 *   n_skip     int32 [T]   experts skipped
 *   keep_mask  uint32 [T]  bit j set = the token's j-th listed expert is computed
 */
int svf_moe_skip(const float* w, int32_t T, int32_t k, int32_t m, const float* beta, int32_t* n_skip,
                 uint32_t* keep_mask, void* stream);

/* Bytes of device workspace svf_moe_calibrate needs (multiple of 256; 0 if T < 1 or k outside 2..32). */
size_t svf_moe_calibrate_workspace_bytes(int32_t T, int32_t k);

/*
 * Threshold map of one layer (Sec. 3.5, Eq. 15): beta[i-1] = median over the T calibration tokens
 * of r_i, i = 1 .. k-1 (the mean of the two middle values when T is even).  w_cal: fp32 [T][k].
 */
int svf_moe_calibrate(const float* w_cal, int32_t T, int32_t k, float* beta, void* ws, size_t ws_bytes,
                      void* stream);

/*
 * Acceptance and resampling of a linear draft (Eq. 2-3), per sequence b:
 *   alpha_j = min(1, p_target[b][j][x_j] / p_draft[b][j][x_j]),  x_j = draft_tokens[b][j];
 *   draft token j is accepted iff u_accept[b][j] < alpha_j; n_accepted[b] = number accepted before the
 *   first rejection (everything behind it is dropped);
 *   if position j = n_accepted[b] < gamma was rejected, resampled[b] = the first token v whose
 *   cumulative residual  sum_{v' <= v} max(0, p_target[b][j][v'] - p_draft[b][j][v'])  exceeds
 *   u_resample[b] times the total residual (the residual is p_target itself if it is zero
 *   everywhere); otherwise resampled[b] = -1.
 * p_target, p_draft: fp32 [B][gamma][V] probabilities; draft_tokens int32 [B][gamma] in [0, V);
 * u_accept fp32 [B][gamma], u_resample fp32 [B], uniform numbers in [0, 1) supplied by the caller.
 * 1 <= gamma <= 64, 1 <= V <= 524288.  Sums are fp32 in a fixed order (same bits on every call).
 */
int svf_accept_resample(const float* p_target, const float* p_draft, const int32_t* draft_tokens,
                        const float* u_accept, const float* u_resample, int32_t B, int32_t gamma, int32_t V,
                        int32_t* n_accepted, int32_t* resampled, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* SVF_RULES_H_ */
