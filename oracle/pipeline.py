"""Double-buffered staging stated plainly (test infrastructure only).

Paper Sec. 4.1 says that double-buffered staging regions overlap communication
with compute; it gives no further detail.  What that leaves to be stated:

 * There are two staging sets (layout arrays + receive buffers).  Step i uses
   set i mod 2.  The dispatch side D(i) of a step (routing, layout, pack) fills
   its set; the combine side C(i) (expert stage, combine) reads it.  D(i+1) may
   run while C(i) runs, because they touch different sets.
 * Overlap changes no result: every step computes what it computes alone, under
   the tables (placement, mask) that were in force when its D was issued
   (Sec. 3.1: reconfiguration happens between forward passes; the routing of a
   step is decided in its dispatch).
 * Hazards.  A set is refilled only after the step it holds has been combined.
   A membership update only affects later D's.  A placement update changes what
   the slots hold, which the expert stage of a step reads; so it is allowed only
   when no dispatched step is still waiting for its combine side.

`validate` checks a sequence of issue events against these rules; `run` gives the
expected outputs of a valid sequence by running every step alone.
"""

D, C, SET_MEMBERSHIP, UPDATE_PLACEMENT = "D", "C", "membership", "placement"


class ScheduleError(ValueError):
    pass


def two_batch_overlap(n_steps):
    """Issue order of a pass over n_steps steps with two staging sets:
    D(0); then for every i: D(i+1) beside C(i).  Drained at both ends."""
    ev = [(D, 0)] if n_steps else []
    for i in range(n_steps):
        if i + 1 < n_steps:
            ev.append((D, i + 1))
        ev.append((C, i))
    return ev


def validate(events, n_sets=2):
    """events: (D, step) | (C, step) | (SET_MEMBERSHIP, mask) | (UPDATE_PLACEMENT, p2l), in
    the order the host issues them.  Raises ScheduleError on a hazard."""
    holds = [None] * n_sets          # step whose rows a set holds, dispatched and not yet combined
    for what, arg in events:
        if what == D:
            s = arg % n_sets
            if holds[s] is not None:
                raise ScheduleError(f"D({arg}): set {s} still holds step {holds[s]}")
            holds[s] = arg
        elif what == C:
            s = arg % n_sets
            if holds[s] != arg:
                raise ScheduleError(f"C({arg}): set {s} does not hold that step")
            holds[s] = None
        elif what == UPDATE_PLACEMENT:
            if any(h is not None for h in holds):
                raise ScheduleError("placement update while a dispatched step awaits its combine")
        elif what != SET_MEMBERSHIP:
            raise ScheduleError(f"unknown event {what}")
    if any(h is not None for h in holds):
        raise ScheduleError("pass ends with a step that was never combined")


def run(events, step_alone, p2l, active):
    """Expected results of a valid event sequence.  step_alone(step, p2l, active) is the
    oracle's single step.  Returns {step: result}: each step alone, under the tables in
    force when its D was issued."""
    validate(events)
    out = {}
    for what, arg in events:
        if what == SET_MEMBERSHIP:
            active = arg
        elif what == UPDATE_PLACEMENT:
            p2l = arg
        elif what == D:
            out[arg] = step_alone(arg, p2l, active)
    return out
