// Argument of the kernel that arms the event tensors of a step on the launch stream (host and device side).
#pragma once
#include <stdint.h>

namespace etc {

// Null pointers / zero counts leave a part out.
struct ArmArgs {
    int32_t *ev_cur;            // [n_events] <- ev_init: the event tensor the next launch drains
    const int32_t *ev_init;
    int32_t *disp_cur;          // [n_events] <- ev_init: dispatch counters of the dynamic scheduler
    int n_events;
    int32_t *pending;           // [n_pending] <- 0: per-task counters of the dynamic scheduler
    int n_pending;
    int32_t *exp_event;         // [n_exp] <- 0: run-time armed expert events
    int n_exp;
    int32_t *qctrl;             // [8] <- 0: ready-queue control words
    int32_t *exec_count;        // [n_exec] <- 0: execution counts (debug)
    int n_exec;
};

}  // namespace etc
