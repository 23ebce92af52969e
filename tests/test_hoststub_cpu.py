"""The host code of the streamed path (context, tilings, chunk schedule, streamed backward passes; Section 3.1 of the
paper) built with g++ against a CPU stand-in of the HIP runtime and run under AddressSanitizer and UBSan, in child
processes that preload the sanitizer runtime. The stand-in defers every stream operation and executes the queues in
three legal orders (at once, as late as the API allows, at seeded random points), treats device memory as out of
bounds for host code, and aborts on a destroyed stream or event handed back to it. Every call is checked against the
oracle. No GPU is involved."""
import os
import subprocess
import sys

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.join(HERE, "hoststub"))
import build as hoststub_build  # noqa: E402


@pytest.fixture(scope="module")
def stub_lib():
    return hoststub_build.build(sanitize=True)


def _run(script, *args, timeout=900):
    env = dict(os.environ)
    env["LD_PRELOAD"] = (hoststub_build.asan_runtime() + " " + env.get("LD_PRELOAD", "")).strip()
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=0"
    env["OMP_NUM_THREADS"] = "2"
    r = subprocess.run([sys.executable, os.path.join(HERE, "hoststub", script), *map(str, args)], env=env, capture_output=True, text=True,
                       timeout=timeout)
    assert r.returncode == 0, f"{script} {args}: exit {r.returncode}\n{r.stdout[-3000:]}\n{r.stderr[-6000:]}"
    assert "ok:" in r.stdout, r.stdout[-2000:]


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_recorded_session_with_new_edge_data(stub_lib, mode):
    """The session whose GPU run once ended in a host-side segmentation fault (seed 479: grid 3 x 4, 200 vertices,
    widths 40 / 40 / 16 / 3 / 8, backward calls after the third and fourth forward call, edge data attached again before
    the fourth and fifth), replayed call for call."""
    _run("run_sessions.py", stub_lib, mode, 479, 1, 1)


@pytest.mark.parametrize("new_edge_data", [0, 1])
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_random_sessions(stub_lib, mode, new_edge_data):
    _run("run_sessions.py", stub_lib, mode, 1000 + 100 * mode, 25, new_edge_data)


def test_sessions_under_thread_sanitizer():
    """The same host code built with ThreadSanitizer (tilings are built on several threads): the recorded session and its
    neighbours, operations executed at seeded random points. The oracle runs on one thread here: its OpenMP runtime is
    not instrumented and would be reported for races it does not have."""
    lib = hoststub_build.build(sanitize="thread")
    env = dict(os.environ)
    env["LD_PRELOAD"] = (hoststub_build.tsan_runtime() + " " + env.get("LD_PRELOAD", "")).strip()
    env["TSAN_OPTIONS"] = "halt_on_error=0:report_signal_unsafe=0:history_size=4"
    env["OMP_NUM_THREADS"] = "1"
    r = subprocess.run([sys.executable, os.path.join(HERE, "hoststub", "run_sessions.py"), lib, "2", "474", "8", "1"], env=env,
                       capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, f"exit {r.returncode}\n{r.stdout[-3000:]}\n{r.stderr[-6000:]}"
    assert "ok:" in r.stdout and "ThreadSanitizer" not in r.stderr and "ThreadSanitizer" not in r.stdout, r.stderr[-6000:]


def test_failed_allocations_come_back_as_errors(stub_lib):
    _run("run_alloc_failures.py", stub_lib)


def test_no_alloc_entry_point_reaches_no_allocator(stub_lib):
    _run("run_no_alloc.py", stub_lib)


def test_dense_block_plan_and_schedule(stub_lib):
    """The dense-block form of a resident graph (ranks, 64 x 32 blocks as edge lists or finished operands, chunks, the
    partial-row slots shared with the sparse remainder's work list, weight packing) against the oracle."""
    _run("run_hybrid.py", stub_lib)


def test_max_over_gated_messages_from_host_memory(stub_lib):
    """The streamed forward call keeps its Gather output (accum_out in host memory) and the streamed backward call of max
    over gated messages carries those maxima through both chunk schedules as a third row per vertex."""
    _run("run_gated_max.py", stub_lib)


def test_products_over_endpoint_lists(stub_lib):
    """Gated and pooled layers on a directed graph with many vertices without in- or out-edges: the per-vertex products
    go over the graph's lists of edge endpoints (forward, backward, the call that must not allocate)."""
    _run("run_endpoints.py", stub_lib)
