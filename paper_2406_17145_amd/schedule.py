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
            if st.grouped_dw:
                st.backward_weights()      # groups of one


class OverlapSchedule:
    """Forward calls on one stream, backward calls (and the gradient reset) on another; micro-batch k
    uses stash slot k % slots, and fw_k waits for bw_{k - slots} (the slot's previous micro-batch).
    The stage must have at least two slots.  With as many slots as micro-batches no forward call ever
    waits for a backward call; that is the only form GraphedMinibatch accepts for capture into a HIP
    graph (it refuses fewer slots than micro-batches and says why)."""

    def __init__(self, stage):
        torch = stage.torch
        if stage.slots < 2:
            raise ValueError("OverlapSchedule needs a stage with in_flight_slots >= 2")
        self.st = stage
        self.s_f = torch.cuda.Stream(device=stage.dev)   # default priority on both
        self.s_b = torch.cuda.Stream(device=stage.dev)
        self.ev_f, self.ev_b = [], []      # one event per micro-batch and direction (an event is recorded once per mini-batch)
        self.ev_start = torch.cuda.Event()

    def minibatch(self, batches, outputs=None, grad_outputs=None, grad_inputs=None, losses=None):
        """outputs: None or one list of output tensors per slot; losses: None or one loss tensor per micro-batch
        (or per slot); grad_outputs / grad_inputs are shared by all backward calls (they run in order)."""
        st, torch = self.st, self.st.torch
        while len(self.ev_f) < len(batches):
            self.ev_f.append(torch.cuda.Event())
            self.ev_b.append(torch.cuda.Event())
        main = torch.cuda.current_stream(st.dev)
        self.ev_start.record(main)
        self.s_f.wait_event(self.ev_start)
        self.s_b.wait_event(self.ev_start)
        with torch.cuda.stream(self.s_b):
            st.grad_reset()
        slots = st.slots
        for k, mb in enumerate(batches):
            slot = k % slots
            with torch.cuda.stream(self.s_f):
                if k >= slots:
                    self.s_f.wait_event(self.ev_b[k - slots])   # the slot's previous micro-batch has been consumed
                st.forward(slot, mb, outputs=None if outputs is None else outputs[slot],
                           loss=None if losses is None else losses[k % len(losses)])
                self.ev_f[k].record(self.s_f)
            with torch.cuda.stream(self.s_b):
                self.s_b.wait_event(self.ev_f[k])
                st.backward(slot, grad_outputs=grad_outputs, grad_inputs=grad_inputs)
                if st.grouped_dw:
                    st.backward_weights()  # groups of one
                self.ev_b[k].record(self.s_b)
        main.wait_stream(self.s_f)
        main.wait_stream(self.s_b)


class TaskSchedule:
    """The kFkB order of paper section 6 for one stage, from the library's ScheduleTask for the configuration
    c = (i, k, b) (in-flight samples, group size, micro-batch size), run by the library's executor: warm-up of
    i / b forward passes, then k backward and k forward passes in turn, cool-down.  The stage must have been
    created with at least i / b stash slots.  With two_streams the forward passes go to one stream and the
    backward passes to another (C4 allows them to overlap); otherwise everything runs in task order on the
    current stream.  lanes = (forward streams, backward streams): passes of neighbouring micro-batches go to
    different streams (gpp_stage_run_schedule_lanes; the stage must allow it, see gpp_stage_lanes); with
    shared_lanes the backward passes use the forward streams (fw_j and bw_j of a micro-batch then follow each
    other on ONE stream: no event between them, one chain of launches per micro-batch)."""

    def __init__(self, stage, in_flight_samples, k, two_streams=True, lanes=(1, 1), shared_lanes=False, same_stream=False):
        from . import binding as B
        torch = stage.torch
        self.B, self.st = B, stage
        self.i, self.k = int(in_flight_samples), int(k)
        cap = max(1, self.i // stage.b)
        if stage.slots < cap:
            raise ValueError(f"{cap} micro-batches in flight need a stage with in_flight_slots >= {cap}")
        self.two = bool(two_streams)
        self.lanes = (int(lanes[0]), int(lanes[1]))
        # same_stream: the lanes' calls (and their group launches) all on the current stream, for timing passes
        self.same_stream = bool(same_stream) and self.lanes != (1, 1)
        if self.lanes != (1, 1) and not self.two and not self.same_stream:
            raise ValueError("lanes need two_streams")
        if self.two:                                         # default priority on all
            self.fw_streams = [torch.cuda.Stream(device=stage.dev) for _ in range(self.lanes[0])]
            if shared_lanes:
                if self.lanes[0] != self.lanes[1]:
                    raise ValueError("shared lanes: as many backward as forward streams")
                self.bw_streams = self.fw_streams
            else:
                self.bw_streams = [torch.cuda.Stream(device=stage.dev) for _ in range(self.lanes[1])]
            self.s_f, self.s_b = self.fw_streams[0], self.bw_streams[0]
        self._keep = None

    def tasks(self, n_micro):
        return self.B.gpp_schedule_tasks(n_micro, self.i, self.k, self.st.b)

    def minibatch(self, batches, outputs=None, grad_outputs=None, grad_inputs=None, losses=None):
        """batches: one list of device tensors (Stage.stage_inputs) per micro-batch.  outputs: one list of output
        tensors per slot or per micro-batch (micro-batch j writes outputs[j % len(outputs)]); losses likewise.
        grad_outputs / grad_inputs: one list of tensors shared by all backward passes (they run in order), or one
        list per micro-batch."""
        st, torch, B = self.st, self.st.torch, self.B
        if outputs is None:
            outputs = self._outs = getattr(self, "_outs", None) or [st.alloc_outputs() for _ in range(st.slots)]
        if grad_inputs is None:     # one set per backward stream: passes on different streams may overlap
            grouped = (B.gpp_stage_info(st.handle)[2] >> 8) & 15     # group launches: a set per micro-batch in flight
            sets = st.slots if grouped else self.lanes[1]
            grad_inputs = self._gin = getattr(self, "_gin", None) or (
                st.alloc_grad_inputs() if sets == 1 else [st.alloc_grad_inputs() for _ in range(sets)])
        if losses is None:
            losses = [st.loss]

        def per_microbatch(x, j):
            if not x:
                return None
            row = x[j % len(x)] if isinstance(x[0], (list, tuple)) else x
            return [t.data_ptr() if t is not None else None for t in row]
        io = []
        for j, mb in enumerate(batches):
            io.append(([t.data_ptr() for t in mb], [t.data_ptr() for t in outputs[j % len(outputs)]],
                       losses[j % len(losses)].data_ptr(), per_microbatch(grad_outputs, j), per_microbatch(grad_inputs, j)))
        tasks = self.tasks(len(batches))
        main = torch.cuda.current_stream(st.dev)
        if self.two:
            every = list(dict.fromkeys(self.fw_streams + self.bw_streams))
            for s in every:
                s.wait_stream(main)
            if self.lanes == (1, 1):
                keep = B.gpp_stage_run_schedule(st.handle, tasks, io, self.s_f.cuda_stream, self.s_b.cuda_stream)
            else:
                keep = B.gpp_stage_run_schedule_lanes(st.handle, tasks, io, [s.cuda_stream for s in self.fw_streams],
                                                      [s.cuda_stream for s in self.bw_streams])
            for s in every:
                main.wait_stream(s)
        elif self.same_stream:
            keep = B.gpp_stage_run_schedule_lanes(st.handle, tasks, io, [main.cuda_stream] * self.lanes[0], [main.cuda_stream] * self.lanes[1])
        else:
            keep = B.gpp_stage_run_schedule(st.handle, tasks, io, main.cuda_stream, main.cuda_stream)
        self._keep = (keep, batches, outputs, grad_outputs, grad_inputs, losses)
        return tasks


class StagePipeline:
    """Several stages of one stage graph on one GPU (paper section 3: G_S; section 2: stages without a path
    between them run concurrently): the library's pipeline executor over stages created by the binding.  Every
    stage gets its own pair of streams (they stand in for its devices), its schedule configuration (i, k) comes
    from the library's reverse traversal of the stage graph (gpp_assign_schedules) unless given, and the
    edges carry tensors forward and gradients backward through buffers of the pipeline's workspace.

    edges: (from_stage, from_output, to_stage, to_input); (x, -1, y, -1) orders y after x without data (a
    linearised pipeline chains independent stages this way).  A stage must have been created with at least
    i / b stash slots (see in_flight_microbatches for the counts a stage graph needs)."""

    @staticmethod
    def in_flight_microbatches(n_stages, edges, micro_batch, k_candidates=None):
        from . import binding as B
        i, k = B.gpp_assign_schedules(n_stages, [(e[0], e[2]) for e in edges], [micro_batch] * n_stages,
                                      k_candidates or [[1]] * n_stages)
        return [v // micro_batch for v in i], k

    def __init__(self, stages, edges, in_flight=None, k=None, streams_per_stage=2):
        from . import binding as B
        self.B, self.stages, self.edges = B, stages, list(edges)
        torch = stages[0].torch
        b = stages[0].b
        if in_flight is None:
            caps, k = self.in_flight_microbatches(len(stages), self.edges, b)
            in_flight = [c * b for c in caps]
        self.in_flight, self.k = list(in_flight), list(k or [1] * len(stages))
        hs = [st.handle for st in stages]
        self.ws_bytes = B.gpp_pipeline_workspace_bytes(hs, self.edges, self.in_flight, self.k)
        self.ws = torch.empty(self.ws_bytes + 256, dtype=torch.uint8, device=stages[0].dev)
        base = (self.ws.data_ptr() + 255) // 256 * 256
        self.handle = B.gpp_pipeline_create(hs, self.edges, self.in_flight, self.k, base, self.ws_bytes)
        dev = stages[0].dev
        self.s_f = [torch.cuda.Stream(device=dev) for _ in stages]      # default priority on all
        self.s_b = [torch.cuda.Stream(device=dev) for _ in stages] if streams_per_stage == 2 else self.s_f
        self._keep = None

    def minibatch(self, io):
        """io[s][j] = (inputs, outputs, loss, grad_outputs, grad_inputs): lists of device tensors (None entries
        where an edge carries the tensor), a loss tensor or None.  Kept alive until the next call."""
        torch = self.stages[0].torch
        self.check_not_capturing_slot_reuse(io, torch.cuda.is_current_stream_capturing())
        main = torch.cuda.current_stream(self.stages[0].dev)
        for s in set(self.s_f + self.s_b):
            s.wait_stream(main)

        def ptrs(x):
            return None if x is None else [t.data_ptr() if t is not None else None for t in x]
        raw = [[(ptrs(i), ptrs(o), None if l is None else l.data_ptr(), ptrs(go), ptrs(gi)) for (i, o, l, go, gi) in rows]
               for rows in io]
        self._keep = (self.B.gpp_pipeline_run(self.handle, raw, [s.cuda_stream for s in self.s_f],
                                              [s.cuda_stream for s in self.s_b]), io)
        for s in set(self.s_f + self.s_b):
            main.wait_stream(s)

    def check_not_capturing_slot_reuse(self, io, capturing):
        """A pipeline step under stream capture is refused when a stage would reuse a stash slot inside the
        step: the slot-reuse wait (a forward stream waiting for a backward stream's event) is the form whose
        capture has crashed the runtime (see GraphedMinibatch)."""
        if capturing and any(st.slots < len(rows) for st, rows in zip(self.stages, io)):
            raise ValueError("capture refused: a stage of the pipeline has fewer stash slots than micro-batches")

    def stash_bytes(self):
        """Per stage: bytes its in-flight micro-batches pin (slots it uses x bytes of a slot)."""
        b = self.stages[0].b
        return [max(1, i // b) * self.B.gpp_stage_memory(st.handle)[0] for i, st in zip(self.in_flight, self.stages)]

    def close(self):
        if self.handle is not None:
            self.B.gpp_pipeline_destroy(self.handle)
            self.handle = None


class GraphedMinibatch:
    """One whole mini-batch of a schedule (gradient reset, every fw_j and bw_j, the events between
    the streams) captured once into a HIP graph and replayed: the stage's calls only enqueue kernels
    on the streams they are given, so nothing in them needs the host again, and a step of a dozen
    few-microsecond launches per micro-batch is no longer paced by the host.

    The captured launches carry their arguments: a replay runs the SAME device buffers (inputs,
    outputs, losses, gradient inputs), so new data is copied into those buffers before a replay, and
    every replay is one complete mini-batch starting with the gradient reset -- which is also what
    keeps the stage's host-side state (overwrite-on-first-backward, slots) consistent with the
    recorded launches.  Capture after at least one eager mini-batch (the first one may clear whole
    embedding-gradient tables, later ones only the touched rows).

    Refused (ValueError, before anything touches the GPU): a schedule on more than one stream whose
    stage has fewer stash slots than the mini-batch has micro-batches.  Such a schedule makes fw_k
    wait for the event of bw_{k - slots} (the slot's previous micro-batch); the capture of that
    forward-stream wait on a backward-stream event has ended in a host-side segmentation fault
    inside the runtime's end-of-capture call (three micro-batches on two slots), and its cause is
    not known.  With a slot per micro-batch no such wait is recorded.
    """

    @staticmethod
    def check_capturable(schedule, n_micro):
        """Raises ValueError for the schedule / slot combinations described above."""
        one_stream = isinstance(schedule, SerialSchedule) or (isinstance(schedule, TaskSchedule) and not schedule.two)
        if not one_stream and schedule.st.slots < n_micro:
            raise ValueError(f"capture refused: {n_micro} micro-batches on {schedule.st.slots} stash slots would record a "
                             "forward-stream wait on a backward-stream event (slot reuse); give the stage a slot per "
                             "micro-batch or run the schedule eagerly")

    def __init__(self, schedule, batches, outputs=None, grad_outputs=None, grad_inputs=None, losses=None):
        self.check_capturable(schedule, len(batches))
        torch = schedule.st.torch
        self.schedule = schedule
        self.keep = (batches, outputs, grad_outputs, grad_inputs, losses)
        self.graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize(schedule.st.dev)
        with torch.cuda.graph(self.graph):
            schedule.minibatch(batches, outputs=outputs, grad_outputs=grad_outputs, grad_inputs=grad_inputs, losses=losses)

    def replay(self):
        self.graph.replay()
