"""Host logic of the streaming and file-tier pipelines, without a GPU.

The library's host sources (ABI, host-resident step, file tier) are compiled with g++ against
a small stand-in for the HIP runtime (tests/hipmock: streams are real concurrent queues, events
order them, copies are memcpy) and run under ThreadSanitizer.  The step kernel is replaced by a
trivial element-wise stand-in, so this checks plumbing only: every element is staged, updated
exactly once and written back to its host address or file offset; file-tier failures come back
as GS_ERR_IO, and HIP calls that the stand-in makes fail in the middle of a layer (a copy, a launch,
an event record or wait, a host-function enqueue) come back as GS_ERR_HIP without a hang or a leak.
The mutants show that the harness notices a dropped event wait, a dropped slot hand-over, a wrong
file offset, a lost failure status.
"""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2512_17570_amd", "csrc")
MOCK = os.path.join(ROOT, "tests", "hipmock")
HOST_SOURCES = ["gs_api.hip", "gs_stream.hip", "gs_tier.hip", "gs_defer.hip"]


def _build(src_dir: str, out: str, tsan: bool, sanitize: str = "thread") -> None:
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-Wall", "-I", MOCK, "-I", os.path.join(ROOT, "include"), "-I", src_dir]
    if tsan:
        cmd += [f"-fsanitize={sanitize}", "-fno-omit-frame-pointer"]
    for s in HOST_SOURCES:
        cmd += ["-x", "c++", os.path.join(src_dir, s)]
    cmd += [os.path.join(MOCK, "hipmock.cpp"), os.path.join(MOCK, "pipeline_harness.cpp"), "-o", out, "-lpthread"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)


def _run(exe: str, scratch: str):
    os.makedirs(scratch, exist_ok=True)
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=0 exitcode=66", ASAN_OPTIONS="detect_leaks=1 exitcode=67",
               UBSAN_OPTIONS="print_stacktrace=1 halt_on_error=1 exitcode=68")
    return subprocess.run([exe, scratch], capture_output=True, text=True, timeout=30, env=env)


@pytest.fixture(scope="module")
def tsan_ok(tmp_path_factory):
    """ThreadSanitizer cannot start under some address-space layouts; then the harness still runs,
    unsanitized, and only its own result checks count."""
    d = tmp_path_factory.mktemp("tsan_probe")
    src = d / "t.cpp"
    src.write_text("int main(){return 0;}\n")
    r = subprocess.run(["g++", "-fsanitize=thread", str(src), "-o", str(d / "t")], capture_output=True, text=True)
    if r.returncode != 0:
        return False
    return subprocess.run([str(d / "t")], capture_output=True, text=True).returncode == 0


def test_pipelines_move_every_element_once_and_are_race_free(tmp_path, tsan_ok):
    exe = str(tmp_path / "harness")
    _build(CSRC, exe, tsan_ok)
    r = _run(exe, str(tmp_path / "scratch"))
    assert "PIPELINE OK" in r.stdout and r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "ThreadSanitizer" not in r.stderr, r.stderr[-3000:]


def test_pipelines_under_address_and_undefined_behaviour_sanitizers(tmp_path, tsan_ok):
    """The same harness under AddressSanitizer (with leak detection: every context that is created
    is destroyed, failure paths included) and UndefinedBehaviorSanitizer."""
    if not tsan_ok:
        pytest.skip("sanitizer runtimes do not start in this environment")
    exe = str(tmp_path / "harness_asan")
    _build(CSRC, exe, True, "address,undefined")
    r = _run(exe, str(tmp_path / "scratch"))
    assert "PIPELINE OK" in r.stdout and r.returncode == 0, r.stdout[-3000:] + r.stderr[-3000:]
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-3000:]


def _build_c_sequence(out_dir: str, tsan: bool) -> str:
    """tests/c_abi/step_demo.c (the plain-C program over the C ABI) built against the HIP stand-in:
    gcc for the C file and the C oracle, g++ for the library's host sources, the stand-in and the
    scalar stand-ins for the kernel launchers."""
    san = ["-fsanitize=thread", "-fno-omit-frame-pointer"] if tsan else []
    inc = ["-I", MOCK, "-I", os.path.join(ROOT, "include")]
    demo_o, oracle_o = os.path.join(out_dir, "demo.o"), os.path.join(out_dir, "oracle.o")
    subprocess.run(["gcc", "-std=c99", "-O1", "-g", "-ffp-contract=off", *san, *inc, "-c",
                    os.path.join(ROOT, "tests", "c_abi", "step_demo.c"), "-o", demo_o], check=True, capture_output=True, text=True)
    subprocess.run(["gcc", "-std=c99", "-O2", "-ffp-contract=off", "-c", os.path.join(ROOT, "oracle", "gs_oracle.c"),
                    "-o", oracle_o], check=True, capture_output=True, text=True)
    exe = os.path.join(out_dir, "c_sequence")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-ffp-contract=off", *san, *inc, "-I", CSRC]
    for s in HOST_SOURCES:
        cmd += ["-x", "c++", os.path.join(CSRC, s)]
    cmd += ["-x", "none", os.path.join(MOCK, "hipmock.cpp"), os.path.join(MOCK, "scalar_kernels.cpp"), demo_o, oracle_o,
            "-o", exe, "-lpthread", "-lm"]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    return exe


@pytest.mark.parametrize("legacy_null_stream", [False, True])
def test_c_program_sequence_completes_under_null_stream_orderings(tmp_path, tsan_ok, legacy_null_stream):
    """The whole plain-C sequence -- resident norm and split step on the null stream, then the
    host-resident step in place on a CU-masked (blocking) stream and staged on three non-blocking
    streams, null stream as the producer -- against the stand-in, with the null stream run in place
    and with HIP's legacy ordering between the null stream and blocking streams: it has to finish
    (no wait cycle in the library's event logic) and match the oracle bit for bit."""
    exe = _build_c_sequence(str(tmp_path), tsan_ok)
    env = dict(os.environ, TSAN_OPTIONS="halt_on_error=0 exitcode=66")
    env.pop("HIPMOCK_LEGACY_NULL", None)
    if legacy_null_stream:
        env["HIPMOCK_LEGACY_NULL"] = "1"
    for argv in ([exe], [exe, "--host-resident"]):
        r = subprocess.run(argv, capture_output=True, text=True, timeout=60, env=env)
        assert r.returncode == 0 and "C ABI OK" in r.stdout, r.stdout[-3000:] + r.stderr[-3000:]
        assert "ThreadSanitizer" not in r.stderr, r.stderr[-3000:]
    assert "host-resident staged: compare" in r.stdout and "host-resident in place: compare" in r.stdout


MUTANTS = [
    ("stream_check_never_swaps_the_colliding_stream", "gs_stream.hip",
     "            if (verdict == 1 || attempt == 9) break;\n", "            break;\n"),
    ("stream_check_leaks_rejected_streams", "gs_stream.hip",
     "        for (hipStream_t r : rejected) (void)hipStreamDestroy(r);\n", ""),
    ("deferred_deadline_not_waited_for", "gs_defer.hip",
     '    hipError_t e = hipStreamWaitEvent(static_cast<hipStream_t>(consumer_stream), c->done[layer], 0);\n',
     '    hipError_t e = hipSuccess;\n'),
    ("deferred_step_ignores_producer", "gs_defer.hip",
     '    if ((e = hipStreamWaitEvent(c->stream, c->ev_producer, 0)) != hipSuccess)\n        return hip_fail(e, "hipStreamWaitEvent(producer)");\n', ""),
    ("deferred_layer_event_on_wrong_layer", "gs_defer.hip",
     'hipEventRecord(c->done[layer], c->stream)', 'hipEventRecord(c->done[0], c->stream)'),
    ("kernel_ignores_producer", "gs_stream.hip",
     '    GS_TRY(hipStreamWaitEvent(c->s_comp, c->ev_producer, 0), "hipStreamWaitEvent(producer)");\n', ""),
    ("staged_upload_ignores_pending_download", "gs_stream.hip",
     '    if (c->used[slot]) GS_TRY(hipStreamWaitEvent(c->s_h2d, c->ev_d2h[slot], 0), "hipStreamWaitEvent(slot free)");\n', ""),
    ("staged_kernel_ignores_upload", "gs_stream.hip",
     '    GS_TRY(hipStreamWaitEvent(c->s_comp, c->ev_h2d[slot], 0), "hipStreamWaitEvent(h2d)");\n', ""),
    ("staged_download_ignores_kernel", "gs_stream.hip",
     '    GS_TRY(hipStreamWaitEvent(c->s_d2h, c->ev_comp[slot], 0), "hipStreamWaitEvent(compute)");\n', ""),
    ("staged_chunk_lands_at_wrong_slot_offset", "gs_stream.hip",
     "    const intptr_t shift = (intptr_t)(pad - b) * (intptr_t)sizeof(float);", "    const intptr_t shift = (intptr_t)(-b) * (intptr_t)sizeof(float);"),
    ("notification_ignores_kernel", "gs_tier.hip",
     "            if (he == hipSuccess) he = hipStreamWaitEvent(c->s_note, t->ev_done[slot], 0);\n", ""),
    ("read_into_slot_still_being_written", "gs_tier.hip",
     "            t->cv.wait(lk, [&] { return !t->busy[slot]; });\n", ""),
    ("writer_ignores_notification", "gs_tier.hip",
     "            t->cv.wait(lk, [&] { return t->finished[j.slot] != 0; });\n", ""),
    ("file_offset_from_layer_start", "gs_tier.hip",
     "off[a] = base[a] + (b - L->n_host) * (int64_t)sizeof(float);", "off[a] = base[a] + b * (int64_t)sizeof(float);"),
    ("host_chunk_index_off_by_one", "gs_tier.hip",
     "            const int64_t b = h_lo + hi * t->chunk;", "            const int64_t b = h_lo + (hi ? hi - 1 : 0) * t->chunk;"),
    ("file_part_of_a_range_starts_at_the_host_boundary", "gs_tier.hip",
     "const int64_t f_lo = begin > L->n_host ? begin : L->n_host, f_hi = end;", "const int64_t f_lo = L->n_host, f_hi = end;"),
    ("bounce_offset_forgotten_on_write_back", "gs_tier.hip",
     "        j.pad = (int)pad;", "        j.pad = 0;"),
    ("failed_chunk_still_queued_for_write_back", "gs_tier.hip",
     '            t->fail_hip(st, "enqueue of a file chunk failed");\n            return;\n',
     '            t->fail_hip(st, "enqueue of a file chunk failed");\n'),
    ("failure_on_the_context_threads_dropped", "gs_tier.hip",
     "            err = st;\n", "            (void)st;\n"),
    ("tier_call_waits_for_the_reader", "gs_tier.hip",
     "        t->layers.push_back(job);\n    }\n    t->cv.notify_all();\n    return GS_OK;\n",
     "        t->layers.push_back(job);\n    }\n    t->cv.notify_all();\n"
     "    {\n        std::unique_lock<std::mutex> lk(t->mu);\n"
     "        t->cv.wait(lk, [&] { return t->layers.empty() && !t->reader_active; });\n    }\n    return GS_OK;\n"),
    ("tier_kernel_ignores_producer", "gs_tier.hip",
     "    hipError_t we = hipStreamWaitEvent(c->s_comp, job.ev_producer, 0);", "    hipError_t we = hipSuccess;"),
    ("tier_sync_ignores_queued_layers", "gs_tier.hip",
     "return t->layers.empty() && !t->reader_active && t->jobs.empty()", "return t->jobs.empty()"),
    ("tier_sync_ignores_layer_being_read", "gs_tier.hip",
     "return t->layers.empty() && !t->reader_active && t->jobs.empty()", "return t->layers.empty() && t->jobs.empty()"),
]


def test_mutation_sites_exist_once():
    for name, fn, old, _ in MUTANTS:
        assert open(os.path.join(CSRC, fn)).read().count(old) == 1, name


def _judge_mutant(work, tsan, name, fn, old, new):
    """Builds the harness from a copy of the host sources with one planted mistake and runs it.
    Returns True if the harness noticed (wrong result, sanitizer report, or a hang)."""
    d = os.path.join(work, name)
    src = os.path.join(d, "src")
    os.makedirs(src, exist_ok=True)
    for f in os.listdir(CSRC):
        if f.endswith((".hip", ".h")):
            shutil.copy(os.path.join(CSRC, f), os.path.join(src, f))
    path = os.path.join(src, fn)
    text = open(path).read()
    assert text.count(old) == 1
    with open(path, "w") as f:
        f.write(text.replace(old, new))
    exe = os.path.join(d, "harness")
    _build(src, exe, tsan)
    try:
        r = _run(exe, os.path.join(d, "scratch"))
    except subprocess.TimeoutExpired:
        return True      # a hang is a failure of the mutant too
    return r.returncode != 0 or "ThreadSanitizer" in r.stderr


@pytest.fixture(scope="module")
def mutant_verdicts(tmp_path_factory, tsan_ok):
    """All mutants are built and run once, a few at a time; under pytest-xdist each test judges its
    own mutant instead (the run is already spread over processes)."""
    from concurrent.futures import ThreadPoolExecutor
    work = str(tmp_path_factory.mktemp("pipeline_mutants"))
    table = {m[0]: m for m in MUTANTS}
    if os.environ.get("PYTEST_XDIST_WORKER"):
        class OnDemand(dict):
            def __missing__(self, name):
                self[name] = _judge_mutant(work, tsan_ok, *table[name])
                return self[name]
        return OnDemand()
    workers = max(1, min(6, (os.cpu_count() or 2) - 1))
    with ThreadPoolExecutor(workers) as ex:
        futs = {name: ex.submit(_judge_mutant, work, tsan_ok, *m) for name, m in table.items()}
        return {name: f.result() for name, f in futs.items()}


@pytest.mark.parametrize("name", [m[0] for m in MUTANTS])
def test_harness_notices_planted_pipeline_mistake(mutant_verdicts, tsan_ok, name):
    if not tsan_ok and name in ("kernel_ignores_producer", "read_into_slot_still_being_written",
                                "staged_upload_ignores_pending_download", "tier_kernel_ignores_producer"):
        pytest.skip("without ThreadSanitizer this ordering mistake only shows by chance")
    assert mutant_verdicts[name], f"mutant {name} went unnoticed"
