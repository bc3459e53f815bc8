/* taw_sched.h -- host-side model of the weight-pipeline schedule the layer kernels serve
 * (TawPipe, arXiv 2511.09741, Methodology).  Pure host code: no GPU, no allocation, no I/O.
 *
 * P devices in D topology-aware groups of P/D devices (group g_k = devices k*P/D .. (k+1)*P/D - 1),
 * L layers with L mod P = 0, N micro-batches.
 *
 * Device-Bound Storage + the interleaved assignment of "Group-Based Weight Pipeline Scheduler":
 * inside group g_k, device number i of the group holds weight shard W_((D*i + k) mod P); a model with
 * L > P layers repeats the pattern, layer j living where shard j mod P lives.
 *
 * Step table (same section; forward steps 0..5 and backward steps 6..11 of the six-device example):
 * group g_k applies layer j to its micro-batches at step j + k (the groups are staggered by one
 * step), and back-propagates through layer j at step L + (L-1-j) + k.  While a group computes at step
 * t its staging device prefetches the shard of step t+1 when that shard lives in another group
 * ("Communication-Computation Overlap"); the shard is fetched from its owner (the paper gives the
 * two-group exchange only; fetching from the owner is the reading adopted for D > 2).  After the
 * backward of layer j the group reduces its gradients onto the device that sits at the owner's
 * position inside the group, which passes them to the owner; the owner of layer j can update once
 * the last group has delivered, at step L + (L-1-j) + D-1.
 *
 * Every function returns TAW_SCHED_OK or TAW_SCHED_ERR (bad arguments: NULL, P % D != 0,
 * L % P != 0, index out of range). */
#ifndef TAW_SCHED_H
#define TAW_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { TAW_SCHED_OK = 0, TAW_SCHED_ERR = -1 };
enum { TAW_PHASE_IDLE = 0, TAW_PHASE_FWD = 1, TAW_PHASE_BWD = 2 };

typedef struct {
  int32_t P; /* devices */
  int32_t D; /* groups (nodes); P % D == 0 */
  int32_t L; /* layers; L % P == 0 */
  int32_t N; /* micro-batches per iteration (used by the bubble ratios only) */
} taw_sched_desc;

/* device that owns layer `layer` (weights, gradient shard, optimizer state), and its group */
int taw_sched_owner(const taw_sched_desc* s, int32_t layer, int32_t* device, int32_t* group);

/* what group `group` does at step t of one forward+backward sweep (steps 0 .. 2L + D - 2):
 *   *phase    TAW_PHASE_FWD / _BWD / _IDLE (the stagger leaves k idle steps at the start, D-1-k at the end)
 *   *layer    layer computed (undefined when idle)
 *   *master   device of this group that distributes the layer's shard inside the group: the owner
 *             when it is a member, else the group's device at the owner's position, which prefetched it
 *   *prefetch_from  device the next step's shard is fetched from during this step, or -1 when that
 *             shard is already in the group (or there is no next step) */
int taw_sched_step(const taw_sched_desc* s, int32_t group, int32_t t, int32_t* phase, int32_t* layer,
                   int32_t* master, int32_t* prefetch_from);

/* step at which the owner of `layer` has received every group's gradients and can update */
int taw_sched_update_step(const taw_sched_desc* s, int32_t layer, int32_t* t);

/* bubble ratios of "Theoretical Analysis": ((D-1) P + N) / ((3N + D-1) P + N) for this schedule,
 * (P-1) / (N + P-1) for 1F1B and for ring-based weight passing */
int taw_sched_bubble_ratio(const taw_sched_desc* s, double* tawpipe, double* one_f_one_b);

/* elements received per device per step, same section, for a layer of 12 H^2 parameters and
 * activations of B*S*H: 24 H^2 (one shard + its gradients) here, 36 H^2 for the ring-based scheme,
 * 2 P B S H for activation passing */
int taw_sched_comm_elems(int32_t P, int32_t B, int32_t S, int32_t H, double* tawpipe, double* weipipe,
                         double* one_f_one_b);

#ifdef __cplusplus
}
#endif
#endif /* TAW_SCHED_H */
