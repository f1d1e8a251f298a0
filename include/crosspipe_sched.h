/*
 * crosspipe_sched.h -- host-side schedule generation and performance model for
 * a unidirectional pipeline whose stages run F / D / W blocks (D is the
 * input-gradient block, called B by stage.h; same numeric code 1).
 *
 * crosspipe_greedy follows the paper's Algorithm 1 ("Greedy Generation for
 * CrossUDSub Schedule") and its scheduling loop (section 4.2.2: stage
 * selection, operation selection by phase priority, operation scheduling), with
 * the range-based bandwidth occupancy model of section 4.2.3 and the alpha-beta
 * communication model of section 2.2.  crosspipe_simulate is the performance
 * model of section 3.5: the start of a block is the later of the end of the
 * previous block on its stage and the end of the block it depends on plus the
 * communication delay.  Both are pure host code: no GPU, no allocation visible
 * to the caller; all pointers are HOST memory owned by the caller.
 *
 * The per-stage ordered list a generator emits ("per-stage schedule S_d") is
 * what stage_run_subschedule consumes: crosspipe_stage_ops extracts it.
 *
 * Model: n_pp stages = devices, one model chunk each.  F(s,m) depends on
 * F(s-1,m); D(s,m) on D(s+1,m), on F(s,m) at the last stage; W(s,m) on D(s,m).
 * Every block is n_sub equal sub-blocks; a dependent block becomes schedulable
 * when the last sub-block of its predecessor has been scheduled.  Starting an F
 * block adds m_f to the stage's memory, finishing a D block adds m_d, finishing
 * a W block adds m_w; an F block may start only while memory + m_f <= m_limit.
 * A message leaves when its producing block ends, takes the earliest free
 * window of beta[src][dst] * msg_bytes on the directed link, and arrives
 * alpha[src][dst] after the window closes.
 *
 * Return: 0, or CROSSPIPE_E_INVAL (null pointer, non-positive sizes, capacity
 * too small, malformed list), CROSSPIPE_E_DEADLOCK (crosspipe_simulate only:
 * the given per-stage orders can never complete).
 */
#ifndef PAPER_2507_00217_CROSSPIPE_SCHED_H
#define PAPER_2507_00217_CROSSPIPE_SCHED_H

#include <stdint.h>

#include "stage.h"

#ifdef __cplusplus
extern "C" {
#endif

enum { CROSSPIPE_F = 0, CROSSPIPE_D = 1, CROSSPIPE_W = 2 };
enum { CROSSPIPE_OK = 0, CROSSPIPE_E_INVAL = -1, CROSSPIPE_E_DEADLOCK = -5 };

typedef struct {
  int32_t n_pp, n_mb, n_sub;
  const double* t_f;      /* [n_pp] duration of a full F block on each stage (T_F) */
  const double* t_d;      /* [n_pp] T_D */
  const double* t_w;      /* [n_pp] T_W */
  double m_f, m_d, m_w;   /* net memory change of a full F / D / W block (M_F, M_D, M_W) */
  double m_limit;         /* per-stage memory limit M_L */
  const double* alpha;    /* [n_pp * n_pp] latency from device i to device j at [i * n_pp + j]; NULL = 0 */
  const double* beta;     /* [n_pp * n_pp] inverse bandwidth (time per byte); NULL = 0 */
  double msg_bytes;       /* size of one activation / gradient message */
} crosspipe_params_t;

/* one scheduled sub-block; sub is the layer-group index (D walks them from n_sub-1 down to 0) */
typedef struct { int32_t stage, kind, mb, sub; double t_start, t_end; } crosspipe_slot_t;

/* Greedy CrossUDSub generation.  out receives the 3 * n_mb * n_sub * n_pp sub-blocks in the order the main
 * loop scheduled them (one per iteration); *n_out their number; *makespan the latest t_end. */
int crosspipe_greedy(const crosspipe_params_t* p, crosspipe_slot_t* out, int capacity, int* n_out, double* makespan);

/* Performance model.  The per-stage execution orders are read from `sched` (entries of one stage in list order;
 * their times are ignored); out_timed receives the same sub-blocks with recomputed times, in start-time order. */
int crosspipe_simulate(const crosspipe_params_t* p, const crosspipe_slot_t* sched, int n, crosspipe_slot_t* out_timed,
                       double* makespan);

/* The ordered (kind, mb, sub) list of one stage, ready for stage_run_subschedule / stage_validate_subschedule. */
int crosspipe_stage_ops(const crosspipe_slot_t* sched, int n, int stage, stage_subop_t* out, int capacity, int* n_out);

#ifdef __cplusplus
}
#endif
#endif
