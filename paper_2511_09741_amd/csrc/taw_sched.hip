// Host-side model of the weight-pipeline schedule (mapping, step table, bubble ratio, communication
// volume).  No device code; it lives in the library so that a runtime driving the layer calls can
// ask it which shard to stage next and from where.
#include "../../include/taw_sched.h"

static bool valid(const taw_sched_desc* s) {
  return s && s->P > 0 && s->D > 0 && s->L > 0 && s->P % s->D == 0 && s->L % s->P == 0;
}

// shard index sigma = layer mod P sits in group sigma mod D at position sigma / D
static void place(const taw_sched_desc* s, int layer, int* group, int* pos) {
  const int sigma = layer % s->P;
  *group = sigma % s->D;
  *pos = sigma / s->D;
}

extern "C" int taw_sched_owner(const taw_sched_desc* s, int32_t layer, int32_t* device, int32_t* group) {
  if (!valid(s) || !device || layer < 0 || layer >= s->L) return TAW_SCHED_ERR;
  int g, pos;
  place(s, layer, &g, &pos);
  *device = g * (s->P / s->D) + pos;
  if (group) *group = g;
  return TAW_SCHED_OK;
}

// layer the group works on at step t, or -1
static int layer_at(const taw_sched_desc* s, int group, int t, int* phase) {
  const int u = t - group;                 // the group's own clock
  if (u >= 0 && u < s->L) { *phase = TAW_PHASE_FWD; return u; }
  if (u >= s->L && u < 2 * s->L) { *phase = TAW_PHASE_BWD; return 2 * s->L - 1 - u; }
  *phase = TAW_PHASE_IDLE;
  return -1;
}

extern "C" int taw_sched_step(const taw_sched_desc* s, int32_t group, int32_t t, int32_t* phase, int32_t* layer, int32_t* master,
                              int32_t* prefetch_from) {
  if (!valid(s) || !phase || !layer || !master || !prefetch_from) return TAW_SCHED_ERR;
  if (group < 0 || group >= s->D || t < 0 || t > 2 * s->L + s->D - 2) return TAW_SCHED_ERR;
  int ph;
  const int j = layer_at(s, group, t, &ph);
  *phase = ph;
  *layer = j;
  *master = -1;
  *prefetch_from = -1;
  const int per = s->P / s->D;
  if (j >= 0) {
    int g, pos;
    place(s, j, &g, &pos);
    *master = group * per + pos;           // the owner itself when g == group
  }
  int ph2;
  const int jn = layer_at(s, group, t + 1, &ph2);
  if (jn >= 0 && jn != j) {
    int g, pos;
    place(s, jn, &g, &pos);
    if (g != group) *prefetch_from = g * per + pos;
  }
  return TAW_SCHED_OK;
}

extern "C" int taw_sched_update_step(const taw_sched_desc* s, int32_t layer, int32_t* t) {
  if (!valid(s) || !t || layer < 0 || layer >= s->L) return TAW_SCHED_ERR;
  *t = s->L + (s->L - 1 - layer) + (s->D - 1);
  return TAW_SCHED_OK;
}

extern "C" int taw_sched_bubble_ratio(const taw_sched_desc* s, double* tawpipe, double* one_f_one_b) {
  if (!valid(s) || s->N <= 0 || !tawpipe || !one_f_one_b) return TAW_SCHED_ERR;
  const double P = s->P, D = s->D, N = s->N;
  *tawpipe = ((D - 1) * P + N) / ((3 * N + D - 1) * P + N);
  *one_f_one_b = (P - 1) / (N + P - 1);
  return TAW_SCHED_OK;
}

extern "C" int taw_sched_comm_elems(int32_t P, int32_t B, int32_t S, int32_t H, double* tawpipe, double* weipipe, double* one_f_one_b) {
  if (P <= 0 || B <= 0 || S <= 0 || H <= 0 || !tawpipe || !weipipe || !one_f_one_b) return TAW_SCHED_ERR;
  const double h2 = (double)H * H;
  *tawpipe = 24.0 * h2;
  *weipipe = 36.0 * h2;
  *one_f_one_b = 2.0 * P * (double)B * S * H;
  return TAW_SCHED_OK;
}
