"""Two batches in flight on one GPU: the sequential block of batch i+1 beside the Jacobi blocks of batch i.

The sequential inverse of the first block is a chain of T-1 dependent steps whose time is set by
latencies, not by the number of CUs it runs on (configuration C2: 24.5 ms on 256 CUs, 30.8 ms on
128); the Jacobi blocks are throughput work.  Run one after the other, each leaves most of the chip
idle or waiting for half of the time.  Here the two kinds of work run on two streams restricted to
disjoint sets of CUs (a CU mask with the same number of CUs on every XCD), on two flows that hold
the same weights, driven by two host threads; a batch still goes through exactly the cascade of
``Flow.sample`` (block 0 sequential, blocks 1..K-1 Jacobi) and gives the same bits.

Argument marshalling and stream plumbing only: every step runs in the library's kernels.
"""
import ctypes as C
import queue
import threading
import time
from typing import List, Optional

from . import Flow, JacobiOpts, DTYPE_F16

_hip = None


def _hip_runtime():
    global _hip
    if _hip is None:
        _hip = C.CDLL("libamdhip64.so")
        _hip.hipExtStreamCreateWithCUMask.argtypes = [C.POINTER(C.c_void_p), C.c_uint32, C.POINTER(C.c_uint32)]
        _hip.hipStreamDestroy.argtypes = [C.c_void_p]
    return _hip


def masked_stream(first_cu: int, last_cu: int, n_cus_device: int):
    """A stream whose kernels run on CU-mask bits first_cu .. last_cu-1 only.  Bit i of the mask is CU
    i // 8 of XCD i % 8 on this part, so a contiguous range of bits whose ends are multiples of 32
    takes the same number of CUs from every XCD and from every shader engine of an XCD (a workgroup
    that needs a whole CU is not placed otherwise: the dispatcher deals workgroups to the engines in
    turn).  Returns (torch ExternalStream, raw handle)."""
    import torch
    if first_cu % 32 or last_cu % 32 or not 0 <= first_cu < last_cu <= n_cus_device:
        raise ValueError("CU ranges must start and end at multiples of 32 inside the device")
    words = (C.c_uint32 * ((n_cus_device + 31) // 32))()
    for i in range(first_cu, last_cu):
        words[i // 32] |= 1 << (i % 32)
    handle = C.c_void_p()
    rc = _hip_runtime().hipExtStreamCreateWithCUMask(C.byref(handle), len(words), words)
    if rc != 0:
        raise RuntimeError(f"hipExtStreamCreateWithCUMask failed with HIP error {rc}")
    return torch.cuda.ExternalStream(handle.value), handle


class PipelinedSampler:
    """Samples a list of latent batches with the sequential block of one batch overlapped with the
    Jacobi blocks of the previous one.  ``n_seq_cus`` CUs (a multiple of 32) carry the sequential
    kernel, the rest the whole-sequence passes."""

    def __init__(self, cfg, weights_blob, n_seq_cus: int = 128, n_cus_device: int = 0, dtype: int = DTYPE_F16):
        if cfg.n_blocks < 2:
            raise ValueError("needs at least one Jacobi block after the sequential one")
        self.cfg = cfg
        self.n_seq_cus = n_seq_cus
        self.flows: List[Flow] = []
        self.last_timing = None
        for _ in range(2):
            f = Flow(cfg, dtype=dtype)
            f.load_weights(weights_blob)
            f.set_sequential_path(3)             # ordinary launch: the stream's CU mask decides where it runs
            f.set_sequential_cus(n_seq_cus)
            self.flows.append(f)
        if n_cus_device <= 0:       # the device's own CU count
            import torch
            n_cus_device = torch.cuda.get_device_properties(torch.cuda.current_device()).multi_processor_count
        self.seq_stream, self._seq_handle = masked_stream(0, n_seq_cus, n_cus_device)
        self.jac_stream, self._jac_handle = masked_stream(n_seq_cus, n_cus_device, n_cus_device)

    def close(self):
        import torch
        torch.cuda.synchronize()
        for f in self.flows:
            f.close()
        self.flows = []
        for h in (self._seq_handle, self._jac_handle):
            if h is not None:
                _hip_runtime().hipStreamDestroy(h)
        self._seq_handle = self._jac_handle = None

    def run(self, latents, opts: Optional[JacobiOpts] = None):
        """latents: list of device tensors [B, T, D].  Returns (outputs, per-batch list of per-block pass counts)."""
        import torch
        opts = opts or JacobiOpts()
        K = self.cfg.n_blocks
        n = len(latents)
        outs = [None] * n
        passes = [None] * n
        handover: "queue.Queue" = queue.Queue()
        free = [threading.Semaphore(1), threading.Semaphore(1)]   # a flow's workspace: one batch at a time
        errors = []
        seq_ms, jac_ms = [], []          # host-side duration of every sequential block / Jacobi cascade

        def seq_worker():
            try:
                with torch.cuda.stream(self.seq_stream):
                    for i in range(n):
                        free[i & 1].acquire()
                        t0 = time.perf_counter()
                        x0 = self.flows[i & 1].sequential_inverse_block(0, latents[i])   # returns when the block is done
                        seq_ms.append((time.perf_counter() - t0) * 1e3)
                        handover.put((i, x0))
            except BaseException as e:   # noqa: BLE001 - reported to the caller below
                errors.append(e)
            finally:
                handover.put(None)

        def jac_worker():
            try:
                with torch.cuda.stream(self.jac_stream):
                    while True:
                        item = handover.get()
                        if item is None:
                            break
                        i, x = item
                        t0 = time.perf_counter()
                        counts = [self.cfg.seq_len - 1]
                        for j in range(1, K):
                            x, _, launched, _ = self.flows[i & 1].jacobi_inverse_block(j, x, opts)
                            counts.append(launched)
                        outs[i], passes[i] = x, counts
                        jac_ms.append((time.perf_counter() - t0) * 1e3)
                        free[i & 1].release()
            except BaseException as e:   # noqa: BLE001
                errors.append(e)
                for s in free:
                    s.release()

        threads = [threading.Thread(target=seq_worker), threading.Thread(target=jac_worker)]
        for t in threads:
            t.start()
        for t in threads:
            t.join()
        if errors:
            raise errors[0]
        torch.cuda.synchronize()
        self.last_timing = {"sequential_ms": seq_ms, "jacobi_ms": jac_ms}
        return outs, passes
