"""Algorithm 2's outer loop (Sec. 3.2) around the step library: iterate until the scale-invariant
clock reaches T_SI.  Holds no arithmetic of the method; gradients come from a caller-supplied
function and everything else happens inside adascale_step."""
from __future__ import annotations

import json
from typing import Callable, List, Optional

from .binding import AdaScale, State


def run_until_done(ada: AdaScale, w: List, mom: List, make_grads: Callable[[int], List[List]],
                   max_steps: int, poll_every: int = 1, on_step: Optional[Callable[[int, State], None]] = None,
                   stream=None, log_path: Optional[str] = None) -> int:
    """Step until tau >= T_SI (the length of the lr table) or max_steps.  `make_grads(t)` returns
    the S gradient lists of iteration t (computed from the current w).  The state is polled every
    `poll_every` steps (polling synchronises the stream); with poll_every = 1 the loop stops at
    exactly the iteration Algorithm 2 would.  `log_path`: append one JSON line per poll with the
    iteration and the state record (r_t, eta_t, tau, the estimates: the quantities the paper's
    training curves plot).  Returns the number of iterations performed."""
    t = 0
    log = open(log_path, "a") if log_path else None
    try:
        while t < max_steps:
            ada.step(w, mom, make_grads(t), stream=stream)
            t += 1
            if t % poll_every == 0 or t == max_steps:
                st = ada.get_state(stream)
                if log is not None:
                    log.write(json.dumps({"iteration": t, **st.as_dict()}) + "\n")
                if on_step is not None:
                    on_step(t, st)
                if st.done:
                    break
    finally:
        if log is not None:
            log.close()
    return t
