"""Build libhidet_mi355x.so: every (tile configuration, input type) instance object plus the C ABI.

    python -m paper_2210_09603_amd.build            # incremental
    python -m paper_2210_09603_amd.build --force    # recompile everything
    HIDET_CONFIGS=0,3,14 python -m paper_2210_09603_amd.build   # development subset of the schedule space

hipcc cross-compiles for gfx950 without a GPU.  Objects live in _build/ (not committed); the shared
library is written next to this file so that it travels with the source tree.
"""
import concurrent.futures
import hashlib
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhidet_mi355x.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def schedule_space():
    """[(index, is_f32)] parsed from configs.def."""
    out = []
    with open(os.path.join(CSRC, "configs.def")) as fh:
        for line in fh:
            m = re.match(r"\s*X(16|32)\((\d+),", line)
            if m:
                out.append((int(m.group(2)), m.group(1) == "32"))
    return out


def _sources_digest():
    h = hashlib.sha256()
    for name in sorted(os.listdir(CSRC)):
        with open(os.path.join(CSRC, name), "rb") as fh:
            h.update(name.encode())
            h.update(fh.read())
    with open(os.path.join(HERE, "..", "include", "hidet_mi355x.h"), "rb") as fh:
        h.update(fh.read())
    h.update(" ".join(FLAGS).encode())
    return h.hexdigest()


def _compile(args):
    src, obj, defines = args
    cmd = [HIPCC] + FLAGS + defines + ["-c", src, "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # hipcc's host pass does not know the packed-fp32 feature and says so on every file; drop that line
    log = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    return r.returncode, obj, log


def build(force=False, jobs=None, verbose=True):
    os.makedirs(BUILD, exist_ok=True)
    digest = _sources_digest()
    subset = os.environ.get("HIDET_CONFIGS")
    chosen = None if not subset else {int(x) for x in subset.split(",") if x.strip()}
    stamp = os.path.join(BUILD, "digest.txt")
    if force or not os.path.exists(stamp) or open(stamp).read() != digest:
        for f in os.listdir(BUILD):
            if f.endswith(".o"):
                os.remove(os.path.join(BUILD, f))
    tasks, objs = [], []
    for idx, is_f32 in schedule_space():
        if chosen is not None and idx not in chosen:
            continue
        for t in ([0] if is_f32 else [1, 2]):
            obj = os.path.join(BUILD, "inst_%d_%d.o" % (idx, t))
            objs.append(obj)
            if not os.path.exists(obj):
                tasks.append((os.path.join(CSRC, "instances.hip"), obj, ["-DHIDET_TU=%d" % idx, "-DHIDET_TYPE=%d" % t]))
    for name in ("api", "probe", "reduce"):
        obj = os.path.join(BUILD, name + ".o")
        objs.append(obj)
        if not os.path.exists(obj):
            tasks.append((os.path.join(CSRC, name + ".hip"), obj, []))
    jobs = jobs or min(8, os.cpu_count() or 1)
    failed = False
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as ex:
        for rc, obj, log in ex.map(_compile, tasks):
            if verbose:
                print("[build] %s rc=%d" % (os.path.basename(obj), rc), flush=True)
            if log.strip() and (rc != 0 or verbose):
                print(log)
            if rc != 0:
                failed = True
                if os.path.exists(obj):
                    os.remove(obj)
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = LIB + ".tmp.%d" % os.getpid()
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs, check=True)
    os.replace(tmp, LIB)
    with open(stamp, "w") as fh:
        fh.write(digest)
    return LIB


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))
