"""Helpers of the replay comparisons (no method arithmetic)."""


def take_over_stop_decision(check_mask, threshold, call, cont):
    """Parameters under which a replay takes the stop test after draft call `call` (Eq. 1) as decided elsewhere:
    a forced "continue" removes the call from the check set S, a forced "stop" makes it the only member of S and
    puts the threshold above every possible P (P <= 1), so the test fails there.  Calls before `call` must already
    have been decided the same way by both sides: their tests came out "continue", so dropping them from S changes
    nothing."""
    if cont:
        return check_mask & ~(1 << call), threshold
    return 1 << call, 2.0
