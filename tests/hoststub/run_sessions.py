"""Run seeded random streamed sessions (tests/session_cases.py) on the host code of libsaga built against the CPU
stand-in of the HIP runtime. Meant to be started as a child process with the AddressSanitizer runtime preloaded:

  python tests/hoststub/run_sessions.py <library> <mode> <first seed> <count> <new_edge_data 0|1>

mode: 0 operations run when enqueued, 1 as late as the API allows, 2 at seeded random points. Exits non-zero on the
first failed comparison with the oracle; a memory error ends the process through the sanitizer."""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
TESTS = os.path.dirname(HERE)
sys.path[:0] = [os.path.dirname(TESTS), TESTS, HERE]

import numpy as np
import torch

from paper_1810_08403_amd import binding as B
from session_cases import streamed_session
from stub_binding import StubContext, dev
from test_gpu_random_cases import _case


class StubBackend:
    error = B.SagaError

    def __init__(self, lib_path, mode):
        self.lib_path, self.mode, self.ctxs = lib_path, mode, 0

    def context(self, budget):
        c = StubContext(self.lib_path, hbm_budget_bytes=budget)
        c.set_mode(self.mode, 77 + self.ctxs)
        self.ctxs += 1
        self.last = c
        return c

    def dev(self, t):
        return dev(t)

    def host(self, a):
        return torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32).clone()

    def host_full(self, shape, value):
        return torch.full(shape, value)

    def dev_full(self, shape, value):
        return dev(torch.full(shape, value))

    def numpy(self, t):
        return t.t.numpy()


def main():
    lib, mode, first, count, new_edge_data = sys.argv[1], int(sys.argv[2]), int(sys.argv[3]), int(sys.argv[4]), int(sys.argv[5])
    be = StubBackend(lib, mode)
    for seed in range(first, first + count):
        # the CPU kernels are stand-ins: the bar only has to tell a right schedule from one that read stale or foreign rows
        streamed_session(be, seed, bool(new_edge_data), _case, log=lambda s: print(s, flush=True) if os.environ.get("SAGA_STUB_VERBOSE") else None,
                         tol=1e-4)
        live = be.last.live_counts()
        assert live["allocations"] == 0 and live["streams"] == 0 and live["events"] == 0, f"seed {seed}: left behind {live}"
    print(f"ok: {count} sessions from seed {first}, mode {mode}, new_edge_data {new_edge_data}", flush=True)


if __name__ == "__main__":
    main()
