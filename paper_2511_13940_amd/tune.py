"""Search for the compute-unit split between communicator and compute workgroups (the paper's section 3.1.3, "SM
partitioning": the best split depends on the problem size and is found by running the candidates).

Host-side orchestration only: for every candidate it creates a partition (pk_partition_create), lets the caller's
function launch one live iteration on the two streams, times it with events, and destroys the partition."""
import torch

from . import pk


def search_comm_cus(launch, candidates=(8, 16, 32, 64), iters=5, warmup=2):
    """launch(compute_stream, comm_stream, comm_cus) must enqueue one complete iteration: the communicator side on
    comm_stream, the op (called with the same comm_cus) on compute_stream, and make compute_stream wait for
    comm_stream at the end.  Both streams are torch.cuda.ExternalStream objects.

    Returns (best_comm_cus, {comm_cus: milliseconds per iteration})."""
    times = {}
    for cc in candidates:
        h_comp, h_comm = pk.pk_partition_create(cc)
        comp, comm = torch.cuda.ExternalStream(h_comp), torch.cuda.ExternalStream(h_comm)
        try:
            torch.cuda.synchronize()
            for _ in range(warmup):
                launch(comp, comm, cc)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(comp)
            for _ in range(iters):
                launch(comp, comm, cc)
            b.record(comp)
            torch.cuda.synchronize()
            times[cc] = a.elapsed_time(b) / iters
        finally:
            torch.cuda.synchronize()
            pk.pk_partition_destroy(h_comp, h_comm)
    best = min(times, key=times.get)
    return best, times
