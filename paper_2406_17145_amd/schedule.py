"""Host-side micro-batch schedules for one stage: which HIP stream each fw_j / bw_j call is
enqueued on, and the events between them.  No arithmetic: the calls are the C ABI's.

The paper's per-stage order condition C4 (paper section 3) asks for fw_k before fw_{k+1},
bw_k before bw_{k+1} and fw_k before bw_k, nothing more, and weights change only between
mini-batches (paper section 6: synchronous schedules).  So fw_{k+1} may run WHILE bw_k
runs: the stage then holds two in-flight micro-batches (two stash slots), exactly the
"in-flight" activations of paper section 2.  On one GPU this fills compute units that a
few-row micro-batch leaves idle.  Weight gradients still accumulate in micro-batch order
(all backward calls share one stream), so results are bit-identical to the serial order.
"""
from __future__ import annotations


class SerialSchedule:
    """fw_0 bw_0 fw_1 bw_1 ... on the current stream, one slot."""

    def __init__(self, stage):
        self.st = stage

    def minibatch(self, batches, outputs=None, grad_outputs=None, grad_inputs=None, losses=None):
        st = self.st
        st.grad_reset()
        for k, mb in enumerate(batches):
            st.forward(0, mb, outputs=outputs, loss=None if losses is None else losses[k % len(losses)])
            st.backward(0, grad_outputs=grad_outputs, grad_inputs=grad_inputs)


class OverlapSchedule:
    """1F1B with two in-flight slots on two streams: forward calls on one, backward calls (and the
    gradient reset) on the other.  The stage must have been created with at least two slots."""

    def __init__(self, stage):
        torch = stage.torch
        if stage.slots < 2:
            raise ValueError("OverlapSchedule needs a stage with in_flight_slots >= 2")
        self.st = stage
        self.s_f = torch.cuda.Stream(device=stage.dev)   # default priority on both
        self.s_b = torch.cuda.Stream(device=stage.dev)
        self.ev_f = [torch.cuda.Event() for _ in range(2)]
        self.ev_b = [torch.cuda.Event() for _ in range(2)]
        self.ev_start = torch.cuda.Event()

    def minibatch(self, batches, outputs=None, grad_outputs=None, grad_inputs=None, losses=None):
        """outputs: None or [per-slot list of output tensors] x 2; losses: None or one loss tensor per micro-batch
        (or per slot); grad_outputs / grad_inputs are shared by all backward calls (they run in order)."""
        st, torch = self.st, self.st.torch
        main = torch.cuda.current_stream(st.dev)
        self.ev_start.record(main)
        self.s_f.wait_event(self.ev_start)
        self.s_b.wait_event(self.ev_start)
        with torch.cuda.stream(self.s_b):
            st.grad_reset()
        for k, mb in enumerate(batches):
            slot = k & 1
            with torch.cuda.stream(self.s_f):
                if k >= 2:
                    self.s_f.wait_event(self.ev_b[slot])      # the slot's previous micro-batch has been consumed
                st.forward(slot, mb, outputs=None if outputs is None else outputs[slot],
                           loss=None if losses is None else losses[k % len(losses)])
                self.ev_f[slot].record(self.s_f)
            with torch.cuda.stream(self.s_b):
                self.s_b.wait_event(self.ev_f[slot])
                st.backward(slot, grad_outputs=grad_outputs, grad_inputs=grad_inputs)
                self.ev_b[slot].record(self.s_b)
        main.wait_stream(self.s_f)
        main.wait_stream(self.s_b)
