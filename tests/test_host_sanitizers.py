"""Host code under AddressSanitizer / UndefinedBehaviorSanitizer (CPU only): the plan, the schedule
and the engine's state machine are compiled with g++ -fsanitize=address,undefined together with a
randomised driver (tests/host_fuzz/plan_fuzz.cpp); the device entry points that the engine calls
are replaced by stand-ins that do nothing."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2501_18512_amd", "csrc")
FLAGS = ["-std=c++17", "-g", "-O1", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
         "-fno-omit-frame-pointer", "-I", os.path.join(ROOT, "include")]

TYPED_STANDINS = r'''
#include "sdl.h"
extern "C" {
int sdl_plan_message_bytes(const sdl_plan_t* plan, uint32_t p, sdl_format_t fmt, size_t* c, size_t* s)
{
    const sdl_span_t* r; uint32_t n;
    int rc = sdl_plan_fragment_runs(plan, p, &r, &n);
    if (rc) return rc;
    if ((int)fmt < 0 || (int)fmt > 7) return -1;
    if (c) *c = 0;
    if (s) *s = 0;
    return 0;
}
uint64_t sdl_plan_staged_numel(const sdl_plan_t* plan, uint32_t p)
{
    const sdl_span_t* r; uint32_t n;
    if (sdl_plan_fragment_runs(plan, p, &r, &n)) return 0;
    uint64_t t = 0;
    for (uint32_t i = 0; i < n; ++i) t += (r[i].numel + 511) / 512 * 512;
    return t;
}
}
'''


def _run(cmd, **kw):
    return subprocess.run(cmd, check=True, capture_output=True, text=True, **kw)


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("nm") is None, reason="needs g++ and nm")
def test_plan_and_engine_host_logic_under_sanitizers(tmp_path):
    objs = []
    for name, src in (("plan", os.path.join(CSRC, "sdl_plan.cpp")), ("engine", os.path.join(CSRC, "sdl_engine.cpp")),
                      ("fuzz", os.path.join(ROOT, "tests", "host_fuzz", "plan_fuzz.cpp"))):
        obj = str(tmp_path / f"{name}.o")
        _run(["g++", *FLAGS, "-c", src, "-o", obj])
        objs.append(obj)
    # whatever the host code references and does not define is a device entry point: stand-ins
    undefined = {l.split()[-1] for o in objs for l in _run(["nm", "-u", o]).stdout.splitlines() if " U sdl_" in l}
    defined = {l.split()[-1] for o in objs for l in _run(["nm", "--defined-only", o]).stdout.splitlines()
               if " T sdl_" in l}
    typed = {"sdl_plan_message_bytes", "sdl_plan_staged_numel"}
    rest = sorted(undefined - defined - typed)
    assert "sdl_fragment_outer_step_plan_ex" in rest and "sdl_receive_outer_step_plan" in rest
    (tmp_path / "typed.cpp").write_text(TYPED_STANDINS)
    (tmp_path / "rest.c").write_text("".join(f"int {n}() {{ return 0; }}\n" for n in rest))
    _run(["g++", *FLAGS, "-c", str(tmp_path / "typed.cpp"), "-o", str(tmp_path / "typed.o")])
    _run(["gcc", "-g", "-c", str(tmp_path / "rest.c"), "-o", str(tmp_path / "rest.o")])
    exe = str(tmp_path / "plan_fuzz")
    _run(["g++", "-fsanitize=address,undefined", *objs, str(tmp_path / "typed.o"), str(tmp_path / "rest.o"), "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert "engines walked" in res.stdout and "ERROR" not in res.stderr
    walked = int(res.stdout.split("engines walked")[1].split()[0])
    assert walked > 500


@pytest.mark.skipif(shutil.which("g++") is None or shutil.which("nm") is None, reason="needs g++ and nm")
def test_offloaded_engine_data_path_under_sanitizers(tmp_path):
    """The schedule driver with the outer state in host memory, end to end on the CPU: csrc/sdl_offload.cpp against a
    stand-in HIP runtime whose copies are memcpy, staged device calls that count, random plans / delays / pool sizes /
    look-aheads (tests/host_fuzz/offload_fuzz.cpp).  A pool that is too small must be refused when it is bound, every
    other walk must finish without running out of slots and leave the right counts in the host arrays."""
    fake = os.path.join(ROOT, "tests", "host_fuzz", "fake_hip")
    objs = []
    for name, src, inc in (("plan", os.path.join(CSRC, "sdl_plan.cpp"), []), ("engine", os.path.join(CSRC, "sdl_engine.cpp"), []),
                           ("offload", os.path.join(CSRC, "sdl_offload.cpp"), ["-I", fake]),
                           ("fuzz", os.path.join(ROOT, "tests", "host_fuzz", "offload_fuzz.cpp"), [])):
        obj = str(tmp_path / f"{name}.o")
        _run(["g++", *FLAGS, *inc, "-c", src, "-o", obj])
        objs.append(obj)
    undefined = {l.split()[-1] for o in objs for l in _run(["nm", "-u", o]).stdout.splitlines() if " U sdl_" in l}
    defined = {l.split()[-1] for o in objs for l in _run(["nm", "--defined-only", o]).stdout.splitlines()
               if " T sdl_" in l}
    rest = sorted(undefined - defined)
    assert "sdl_receive_outer_step_staged" in defined and "sdl_offload_acquire" in defined
    # what is left are the calls on flat device arrays, which an engine with offloaded state never makes
    (tmp_path / "rest.c").write_text("#include <stdlib.h>\n" + "".join(f"int {n}() {{ abort(); }}\n" for n in rest))
    _run(["gcc", "-g", "-c", str(tmp_path / "rest.c"), "-o", str(tmp_path / "rest.o")])
    exe = str(tmp_path / "offload_fuzz")
    _run(["g++", "-fsanitize=address,undefined", *objs, str(tmp_path / "rest.o"), "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=900)
    assert res.returncode == 0, res.stdout[-2000:] + res.stderr[-4000:]
    assert "offload engines walked" in res.stdout and "ERROR" not in res.stderr
    walked = int(res.stdout.split("offload engines walked")[1].split()[0])
    refused = int(res.stdout.split("refused")[1].split()[0])
    assert walked > 1000 and refused > 20
