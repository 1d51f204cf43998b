"""Builds libcoop.so (HIP, gfx950) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcoop.so")
SOURCES = ["runtime.hip", "sample.hip", "labor.hip", "ns.hip", "rw.hip", "unique.hip", "gather.hip", "owner.hip", "cache.hip", "selftest.hip"]

# -ffp-contract=off: the variate kit spells every fused multiply-add out; nothing may be contracted behind its back.
# packed-fp32-ops off: keep the compiler from forming packed fp32 instructions.
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-ffp-contract=off", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wall", "-Wno-unused-function",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


# Host-side sanitizers (the device code is compiled as usual; GPU sanitizers are not available): every -fsanitize= option
# directly after -Xarch_host.
SAN_FLAGS = ["-O1", "-g", "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
             "-fno-omit-frame-pointer", "-Xarch_host", "-shared-libsan"]
SAN_DIR = os.path.join(ROOT, "_build", "sanitize")


def build(verbose=False, sanitize=False):
    """Compiles every HIP source for gfx950 and links libcoop.so in-tree.  sanitize=True builds a second library,
    _build/sanitize/libcoop_san.so, whose host code runs under AddressSanitizer and UndefinedBehaviorSanitizer (see
    sanitize_check)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in FLAGS if f != "-O3"] + SAN_FLAGS if sanitize else FLAGS
    flags = flags + os.environ.get("COOP_EXTRA_FLAGS", "").split()   # (experiments: -D switches of the kernels)
    obj_dir = SAN_DIR if sanitize else CSRC
    lib = os.path.join(SAN_DIR, "libcoop_san.so") if sanitize else os.environ.get("COOP_BUILD_LIB", LIB)
    if os.environ.get("COOP_BUILD_LIB"):
        obj_dir = os.environ["COOP_BUILD_LIB"] + ".objs"
    os.makedirs(obj_dir, exist_ok=True)
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(obj_dir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc] + flags + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if verbose and out.strip():
            print(out)
    link = [hipcc, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", lib] + objs
    if sanitize:
        link += ["-fsanitize=address", "-fsanitize=undefined", "-shared-libsan"]
    subprocess.check_call(link)
    return lib


def sanitize_check(verbose=True):
    """CPU-only sanitizer pass over the host code on both sides of the parity tests:
      - the oracle (oracle/coopref.c, gcc -fsanitize=address,undefined) under its pins, tests/test_oracle_pins.py;
      - the library's host code (argument checks, arena, profiling table; hipcc with the host sanitizers) under the
        C-ABI checks that need no GPU, tests/test_abi.py.
    Each runs in a pytest process of its own with that compiler's sanitizer runtime preloaded.  Raises on any report."""
    import sys
    os.makedirs(SAN_DIR, exist_ok=True)
    oracle_san = os.path.join(SAN_DIR, "libcoopref_san.so")
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fsanitize=address,undefined", "-fno-omit-frame-pointer",
                           "-Wall", "-Wextra", "-fPIC", "-shared", os.path.join(ROOT, "oracle", "coopref.c"), "-o", oracle_san, "-lm"])
    lib_san = build(verbose=False, sanitize=True)
    gcc_asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    clang_asan = subprocess.check_output([hipcc, "-print-file-name=libclang_rt.asan-x86_64.so"], text=True).strip()
    common = {"ASAN_OPTIONS": "detect_leaks=0", "UBSAN_OPTIONS": "print_stacktrace=1:halt_on_error=1"}
    runs = [("oracle", {"COOPREF_LIBRARY_PATH": oracle_san, "LD_PRELOAD": gcc_asan}, "tests/test_oracle_pins.py"),
            ("library host code", {"COOP_LIBRARY_PATH": lib_san, "LD_PRELOAD": clang_asan}, "tests/test_abi.py")]
    for what, extra, test in runs:
        env = dict(os.environ)
        if env.get("LD_PRELOAD"):
            extra = dict(extra, LD_PRELOAD=extra["LD_PRELOAD"] + ":" + env["LD_PRELOAD"])
        env.update(common)
        env.update(extra)
        if verbose:
            print("sanitize_check: %s under %s" % (what, test), flush=True)
        subprocess.check_call([sys.executable, "-m", "pytest", test, "-x", "-q", "-m", "not gpu"], cwd=ROOT, env=env)
    return True


if __name__ == "__main__":
    import sys
    if "--sanitize" in sys.argv:
        print(sanitize_check())
    else:
        print(build(verbose=True))
