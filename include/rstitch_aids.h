/*
 * rstitch_aids.h - measurement and test aids of librstitch.so.  Not part of the
 * method: nothing here computes anything of the stitched-decoding path.  Kept
 * apart from rstitch.h so that the method's ABI stays the calls the paper's
 * procedure needs (Algorithm 1; Eq. 1-2).
 */
#ifndef RSTITCH_AIDS_H
#define RSTITCH_AIDS_H

#include "rstitch.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Test aid: the single-kernel decode step separates its phases with grid-wide
 * waits that give up after `polls` polls (default 2^22, about a second) instead
 * of hanging; a tiny value forces that error path from the host.  0 restores the
 * default.  After a wait has given up the model is unusable (RS_FLAG_ABORTED on
 * every record) until it is created again. */
rs_status rs_set_spin_limit(rs_model *model, uint32_t polls);

/* Measurement aid (not part of the method): while armed, every forward call on
 * this model records `start_event` immediately before and `stop_event`
 * immediately after the launch of ONE kernel on the call's stream: the kernel of
 * phase `phase` (RS_PHASE_*) in layer `layer` (layer is ignored for
 * RS_PHASE_LMHEAD).  Both are caller-owned hipEvent_t handles passed as void*;
 * the caller reads them with hipEventElapsedTime after synchronising.
 * phase < 0 disarms.  While armed, calls run as plain launches (no launch-graph
 * replay, no single-kernel step), so that there is a kernel to bracket.
 * Errors: RS_EINVAL (null model/event, layer out of range). */
#define RS_PHASE_QKV     0
#define RS_PHASE_OPROJ   1
#define RS_PHASE_GATEUP  2
#define RS_PHASE_DOWN    3
#define RS_PHASE_LMHEAD  4
#define RS_PHASE_ATTN    5
rs_status rs_set_phase_timer(rs_model *model, int32_t phase, int32_t layer,
                             void *start_event, void *stop_event);

#ifdef __cplusplus
}
#endif
#endif /* RSTITCH_AIDS_H */
