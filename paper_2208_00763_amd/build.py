"""Build libhikonv.so for gfx950 with hipcc (cross-compiles without a GPU)."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhikonv.so")

SOURCES = [
    "hikonv_plan.cpp",
    "hikonv_api.hip",
    "hikonv_conv1d.hip",
    "hikonv_conv1d_fast.hip",
    "hikonv_conv1d_window.hip",
    "hikonv_conv1d_window_t1.hip",
    "hikonv_conv1d_window_t2.hip",
    "hikonv_conv1d_window_t3.hip",
    "hikonv_conv1d_window_t4.hip",
    "hikonv_conv1d_window_t5.hip",
    "hikonv_conv1d_window_t6.hip",
    "hikonv_conv1d_window_t7.hip",
    "hikonv_conv1d_requant.hip",
    "hikonv_conv1d_requant_aligned.hip",
    "hikonv_conv2d.hip",
    "hikonv_conv2d_fused.hip",
    "hikonv_conv2d_wide.hip",
    "hikonv_conv2d_narrow.hip",
    "hikonv_conv2d_sreg_unsigned.hip",
    "hikonv_conv2d_sreg_signed.hip",
    "hikonv_misc.hip",
]

# packed-FP32 VALU forms are switched off for every HIP translation unit
HIP_FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-x", "hip",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-command-line-argument", "-Wno-option-ignored"]


# Kernels whose hand-written load/wait pipeline keeps loaded values in registers across
# separate inline-assembly statements: a register spill between a load and its wait would make
# them read stale data, so the build fails if the compiler reports any for them.
NO_SPILL_SOURCES = ("hikonv_conv2d_sreg_unsigned.hip", "hikonv_conv2d_sreg_signed.hip")


def check_no_spills(src: str, remarks: str) -> None:
    """Parse -Rpass-analysis=kernel-resource-usage remarks; raise if a k_conv2d_sreg kernel spills."""
    kernel, seen = None, 0
    for line in remarks.splitlines():
        if "Function Name:" in line:
            kernel = line.split("Function Name:")[1].strip()
        for key in ("SGPRs Spill:", "VGPRs Spill:", "ScratchSize [bytes/lane]:"):
            if key in line and kernel and "k_conv2d_sreg" in kernel:
                seen += 1
                value = int(line.split(key)[1].split()[0])
                if value != 0:
                    raise RuntimeError("%s: %s spills registers (%s %d); its load/wait pipeline needs all values "
                                       "in registers" % (src, kernel, key, value))
    if seen == 0:
        raise RuntimeError("%s: no resource-usage remarks for k_conv2d_sreg found; the spill check did not run" % src)


def _hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _deps_mtime() -> float:
    files = [os.path.join(CSRC, f) for f in os.listdir(CSRC)]
    files.append(os.path.join(os.path.dirname(HERE), "include", "hikonv.h"))
    return max(os.path.getmtime(f) for f in files)


def is_fresh() -> bool:
    return os.path.exists(LIB) and os.path.getmtime(LIB) >= _deps_mtime()


def build(force: bool = True, jobs: int = 8, extra_flags=(), out: str = LIB, obj_dir: str = OBJ_DIR) -> str:
    """Compile every translation unit and link paper_2208_00763_amd/libhikonv.so.

    extra_flags/out/obj_dir build a tuning variant next to the default library."""
    if not force and out == LIB and is_fresh():
        return LIB
    os.makedirs(obj_dir, exist_ok=True)
    hipcc = _hipcc()

    def compile_one(src: str) -> str:
        obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc] + HIP_FLAGS + list(extra_flags) + ["-c", os.path.join(CSRC, src), "-o", obj]
        if src in NO_SPILL_SOURCES:
            cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s" % (src, res.stderr[-4000:]))
        if src in NO_SPILL_SOURCES:
            check_no_spills(src, res.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + objs
    res = subprocess.run(link, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("link failed:\n%s" % res.stderr[-4000:])
    return out


if __name__ == "__main__":
    print(build(force=True))
