"""Oracle for the per-request lifecycle and the call-duration forecast.  TEST INFRASTRUCTURE ONLY.

Lifecycle (paper Sec. 6.2: every request is in one of five states - running, pending-offload,
offloaded, pending-upload, uploaded - driven by the call_start / call_finish endpoints and the
scheduling loop; Sec. 4.1: if the KV is already uploaded when the tool returns the agent resumes
at once, if the tool returns earlier than predicted an immediate upload is triggered).

Forecast (Sec. 4.1, Eq. 1): per function type; without history the user's estimate, else a
system-wide constant; from the first observation on an exponentially weighted moving average;
with both a user estimate and history, t = alpha * t_user + (1 - alpha) * t_history.

Readings (the paper gives no transition table and no constants): a request whose offload was never
issued stays pending-offload and simply resumes at call_finish; a call_finish that arrives while a
copy is in flight is remembered and acted on when the copy completes; the moving average is
h <- gamma * observed + (1 - gamma) * h with the first observation taken as is; alpha, gamma and the
system constant are parameters.
"""
RUNNING, PENDING_OFFLOAD, OFFLOADED, PENDING_UPLOAD, UPLOADED = range(5)
CALL_START, OFFLOAD_ISSUED, OFFLOAD_DONE, UPLOAD_ISSUED, UPLOAD_DONE, CALL_FINISH = range(6)
NONE, RESUME, UPLOAD_NOW, WAIT = range(4)


class Invalid(Exception):
    pass


def step(req, event):
    """req = (state, finish_seen, copy_in_flight) -> (new req, action); raises Invalid."""
    state, finished, in_flight = req
    if event == CALL_START:
        if state == RUNNING and not finished and not in_flight:
            return (PENDING_OFFLOAD, False, False), NONE
    elif event == OFFLOAD_ISSUED:
        if state == PENDING_OFFLOAD and not in_flight and not finished:
            return (PENDING_OFFLOAD, False, True), NONE
    elif event == OFFLOAD_DONE:
        if state == PENDING_OFFLOAD and in_flight:
            # the tool may have returned while the copy ran: bring the KV straight back
            return (OFFLOADED, finished, False), (UPLOAD_NOW if finished else NONE)
    elif event == UPLOAD_ISSUED:
        if state == OFFLOADED:
            return (PENDING_UPLOAD, finished, True), NONE
    elif event == UPLOAD_DONE:
        if state == PENDING_UPLOAD and in_flight:
            if finished:
                return (RUNNING, False, False), RESUME
            return (UPLOADED, False, False), NONE
    elif event == CALL_FINISH:
        if finished:
            raise Invalid("call_finish twice")
        if state == UPLOADED:
            return (RUNNING, False, False), RESUME          # already back: resume immediately
        if state == OFFLOADED:
            return (OFFLOADED, True, False), UPLOAD_NOW     # returned early: immediate upload
        if state == PENDING_UPLOAD:
            return (PENDING_UPLOAD, True, in_flight), WAIT
        if state == PENDING_OFFLOAD:
            if in_flight:
                return (PENDING_OFFLOAD, True, True), WAIT
            return (RUNNING, False, False), RESUME          # never left the GPU
    raise Invalid(f"event {event} in state {req}")


class Forecaster:
    def __init__(self, alpha, gamma, default_ms):
        self.alpha, self.gamma, self.default_ms = alpha, gamma, default_ms
        self.history = {}

    def observe(self, fn_type, elapsed_ms):
        if fn_type in self.history:
            self.history[fn_type] = self.gamma * elapsed_ms + (1 - self.gamma) * self.history[fn_type]
        else:
            self.history[fn_type] = elapsed_ms

    def estimate(self, fn_type, t_user_ms=None):
        h = self.history.get(fn_type)
        if h is None:
            return t_user_ms if t_user_ms is not None else self.default_ms
        if t_user_ms is None:
            return h
        return self.alpha * t_user_ms + (1 - self.alpha) * h      # Eq. 1
