"""The host-side planning of the library under AddressSanitizer and UndefinedBehaviorSanitizer
(CPU only; GPU sanitizers are not available here).  csrc/emb_bag_plan.cpp - argument checks,
kernel choice, grid layout, table lists in fixed arrays, fusing - is plain C++: it is rebuilt here
with g++ and both sanitizers, linked with the kernel objects of the regular build (they supply the
kernel pickers the planner consults), and driven by tests/sanitize/plan_driver.c through
emb_bag_plan_forward* (which needs no GPU) over table counts around 1024 and 65535, every row
class, element type, mode and tuning key."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]


def test_host_planning_under_asan_and_ubsan(tmp_path):
    build_dir = os.path.join(ROOT, "_build")
    # every object of the regular build except the planner itself and the entry points that launch
    kernels = sorted(os.path.join(build_dir, f) for f in os.listdir(build_dir)
                     if f.endswith(".o") and f.startswith("emb_bag_")
                     and not f.startswith(("emb_bag_plan.", "emb_bag_hot_rows.")))
    assert len(kernels) >= 20, "the regular build's objects are needed (run __graft_entry__.build())"
    obj = str(tmp_path / "emb_bag_plan_san.o")
    exe = str(tmp_path / "plan_driver")
    inc = ["-I", os.path.join(ROOT, "include")]
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fPIC"] + SAN + inc + ["-c", "-o", obj,
                   os.path.join(ROOT, "paper_2410_22249_amd", "csrc", "emb_bag_plan.cpp")], check=True)
    drv = str(tmp_path / "plan_driver.o")
    subprocess.run(["gcc", "-std=c99", "-O1", "-g"] + SAN + inc + ["-c", "-o", drv,
                   os.path.join(ROOT, "tests", "sanitize", "plan_driver.c")], check=True)
    subprocess.run(["g++"] + SAN + ["-o", exe, drv, obj] + kernels +
                   ["-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:halt_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=900)
    assert r.returncode == 0, f"status {r.returncode}\n{r.stdout[-2000:]}\n{r.stderr[-6000:]}"
    assert "sanitized planning:" in r.stdout
    print(r.stdout.strip())
