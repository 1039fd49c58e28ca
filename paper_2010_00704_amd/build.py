"""Builds libbcnn.so (HIP, gfx950) next to this file with hipcc."""
import glob
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
LIB_PATH = os.path.join(_HERE, "libbcnn.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # packed-fp32 instruction forms are kept out of all device code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # a*b + c is fused only where the source says fma: float results are part of the interface
    "-ffp-contract=off",
    "-Wall", "-Wno-unused-command-line-argument",
]


def sources():
    return sorted(glob.glob(os.path.join(_HERE, "csrc", "*.hip")))


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # hipcc's host pass does not know the packed-fp32 feature name and says so; harmless
    log = "\n".join(l for l in proc.stdout.splitlines() if "packed-fp32-ops" not in l)
    return proc.returncode, log


def build_library(verbose=False):
    """Compile every .hip file under csrc/ (one hipcc process per file, in
    parallel) and link them into libbcnn.so.  Always compiles."""
    import shutil
    import tempfile
    from concurrent.futures import ThreadPoolExecutor

    srcs = sources()
    tmpdir = tempfile.mkdtemp(prefix="bcnn_build_")
    try:
        common = [f for f in FLAGS if f != "-shared"] + ["-I", os.path.join(_ROOT, "include"),
                                                         "-I", os.path.join(_HERE, "csrc")]
        objs = [os.path.join(tmpdir, os.path.basename(src) + ".o") for src in srcs]
        jobs = min(len(srcs), max(1, min(8, os.cpu_count() or 1)))
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            results = list(pool.map(lambda so: _run([HIPCC] + common + ["-c", so[0], "-o", so[1]]), zip(srcs, objs)))
        logs = []
        for src, (rc, log) in zip(srcs, results):
            if rc != 0:
                raise RuntimeError("hipcc failed on %s:\n%s" % (os.path.basename(src), log))
            if log.strip():
                logs.append(log)
        tmp = LIB_PATH + ".tmp.%d" % os.getpid()
        rc, log = _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs)
        if rc != 0:
            if os.path.exists(tmp):
                os.remove(tmp)
            raise RuntimeError("link failed:\n" + log)
        if verbose and (logs or log.strip()):
            print("\n".join(logs + [log]))
        os.replace(tmp, LIB_PATH)
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)
    return LIB_PATH


def resource_usage(jobs=None):
    """Device-only compile of every source with the compiler's per-kernel
    resource remarks switched on.  Returns {kernel symbol: {"scratch": bytes
    per lane, "vgpr_spills": n, "sgpr_spills": n, "vgprs": n, "agprs": n,
    "occupancy": waves per SIMD}}; nothing is linked or written."""
    import re
    import shutil
    import tempfile
    from concurrent.futures import ThreadPoolExecutor

    srcs = sources()
    tmpdir = tempfile.mkdtemp(prefix="bcnn_usage_")
    common = [f for f in FLAGS if f not in ("-shared", "-fPIC")] + [
        "--cuda-device-only", "-Rpass-analysis=kernel-resource-usage",
        "-I", os.path.join(_ROOT, "include"), "-I", os.path.join(_HERE, "csrc")]
    fields = {"ScratchSize [bytes/lane]": "scratch", "VGPRs Spill": "vgpr_spills", "SGPRs Spill": "sgpr_spills",
              "VGPRs": "vgprs", "AGPRs": "agprs", "Occupancy [waves/SIMD]": "occupancy"}
    out = {}
    try:
        jobs = jobs or min(len(srcs), max(1, min(8, os.cpu_count() or 1)))
        with ThreadPoolExecutor(max_workers=jobs) as pool:
            results = list(pool.map(
                lambda src: _run([HIPCC] + common + ["-c", src, "-o", os.path.join(tmpdir, os.path.basename(src) + ".o")]),
                srcs))
        for src, (rc, log) in zip(srcs, results):
            if rc != 0:
                raise RuntimeError("hipcc failed on %s:\n%s" % (os.path.basename(src), log))
            cur = None
            for line in log.splitlines():
                m = re.search(r"remark:\s+(.*?):\s+(\S+) \[-Rpass-analysis", line)
                if not m:
                    continue
                key, val = m.group(1).strip(), m.group(2)
                if key == "Function Name":
                    cur = out.setdefault(val, {"source": os.path.basename(src)})
                elif cur is not None and key in fields:
                    cur[fields[key]] = int(val)
    finally:
        shutil.rmtree(tmpdir, ignore_errors=True)
    return out


if __name__ == "__main__":
    print(build_library(verbose=True))
