"""GPU timing helpers shared by ``bench.py`` and the pooling auto-tuner (measurement support, not the hot path)."""
from __future__ import annotations

class TimingEvents:
    """HIP events made for timing: created with hipEventDisableSystemFence, which drops the system-scope
    fence (and the cache write-back that comes with it) that a default event performs when it completes.
    HIP documents the flag for events that only measure time.  Measured on MI355X with a 46 us copy kernel:
    an event after every launch adds 2.8 us per launch with default events (torch.cuda.Event) and 1.0 us
    with these.  They are recorded on torch's current stream, the stream the library launches on."""

    DISABLE_SYSTEM_FENCE = 0x20000000

    def __init__(self, torch):
        import ctypes
        self._ct = ctypes
        path = None
        with open("/proc/self/maps") as f:                      # the HIP runtime this process already uses
            for line in f:
                if "libamdhip64.so" in line:
                    path = line.split()[-1]
                    break
        if path is None:
            raise RuntimeError("the HIP runtime is not loaded in this process")
        self._hip = ctypes.CDLL(path)
        self._hip.hipEventCreateWithFlags.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint]
        self._hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        self._hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self._hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self._torch = torch
        self._made = []

    def _check(self, status, what):
        if status != 0:
            raise RuntimeError(f"{what} failed with HIP status {status}")

    def create(self, n):
        out = []
        for _ in range(n):
            ev = self._ct.c_void_p()
            self._check(self._hip.hipEventCreateWithFlags(self._ct.byref(ev), self.DISABLE_SYSTEM_FENCE),
                        "hipEventCreateWithFlags")
            out.append(ev)
        self._made += out
        return out

    def record(self, ev):
        stream = self._ct.c_void_p(self._torch.cuda.current_stream().cuda_stream)
        self._check(self._hip.hipEventRecord(ev, stream), "hipEventRecord")

    def elapsed_ms(self, a, b):
        ms = self._ct.c_float()
        self._check(self._hip.hipEventElapsedTime(self._ct.byref(ms), a, b), "hipEventElapsedTime")
        return ms.value

    def destroy_all(self):
        for ev in self._made:
            self._hip.hipEventDestroy(ev)
        self._made = []



def graph_train_ms(torch, tev: TimingEvents, launch, nsets: int, iters: int = 20, replays: int = 3) -> float:
    """Milliseconds per launch of ``launch(set_index)``: ``iters`` launches on rotating buffer sets are captured
    into one HIP graph, and the best of ``replays`` replays between one pair of events is divided by ``iters``.
    A launch of a few microseconds is shorter than the host needs to issue it from Python and than an event
    costs, so neither may sit between the launches that are timed."""
    for i in range(3):
        if launch(i % nsets) != 0:
            raise RuntimeError("launch failed")
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for i in range(iters):
            launch(i % nsets)
    graph.replay()
    best = None
    for _ in range(replays):
        a, b = tev.create(2)
        torch.cuda.synchronize()
        tev.record(a)
        graph.replay()
        tev.record(b)
        torch.cuda.synchronize()
        ms = tev.elapsed_ms(a, b) / iters
        best = ms if best is None or ms < best else best
    tev.destroy_all()
    del graph
    return best
