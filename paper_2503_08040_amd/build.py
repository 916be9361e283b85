"""Compile the HIP sources into paper_2503_08040_amd/libfq.so (gfx950 only)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfq.so")
SOURCES = ["fq_api.hip", "fq_quantize.hip", "fq_gemm.hip", "fq_group.hip", "fq_ctx.hip"]
HEADERS = ["fq_device.h", "fq_kernels.h", os.path.join("..", "..", "include", "fq.h")]

# Packed FP32 VALU instructions are switched off for the device pass (the host
# pass prints a harmless "not a recognized feature" note).
# -amdgpu-atomic-optimizer-strategy=None: the compiler otherwise turns an atomic issued by one
# thread into its wavefront-aggregated form, whose result is broadcast (and therefore waited for)
# right behind the instruction; the quantizer issues its atomics early precisely so that their
# round trip passes behind the arithmetic that follows.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
               "-Wall", "-Wno-unused-command-line-argument"]


TOOLS = ["mfma_ceiling", "pipeline_probe"]
TOOL_BIN = os.path.join(HERE, "mfma_ceiling")


def build_tools() -> list:
    """Register-only throughput probes (measurement support for the benchmark's roofline
    context): one executable per source under csrc/tools, placed next to the library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = []
    for name in TOOLS:
        exe = os.path.join(HERE, name)
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature",
               "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument", "-o", exe,
               os.path.join(CSRC, "tools", name + ".hip")]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed:\n{r.stderr}")
        out.append(exe)
    return out


# Ablation builds of the GEMM kernel (measurement support, see the switches at the top of
# csrc/fq_gemm.hip): whole libraries, libfq_ablate_<name>.so, loaded instead of libfq.so when the
# environment variable FQ_LIBRARY names one.  They compute wrong products on purpose.
ABLATIONS = {
    "no_dma": ["-DFQ_ABLATE_NO_DMA"],
    "no_multiply": ["-DFQ_ABLATE_NO_MULTIPLY"],
    "no_dequant": ["-DFQ_ABLATE_NO_DEQUANT"],
    "extra_salu_40": ["-DFQ_ABLATE_EXTRA_SALU=40"],
    "extra_salu_120": ["-DFQ_ABLATE_EXTRA_SALU=120"],
    "dma_hot": ["-DFQ_ABLATE_DMA_HOT"],
    "one_stager": ["-DFQ_ABLATE_ONE_STAGER"],
    "team_skew": ["-DFQ_ABLATE_TEAM_SKEW"],
    "team_skew_no_dma": ["-DFQ_ABLATE_TEAM_SKEW", "-DFQ_ABLATE_NO_DMA"],
}


def ablation_lib(name: str) -> str:
    return os.path.join(HERE, f"libfq_ablate_{name}.so")


def build_ablations(names=None, jobs: int = 6) -> list:
    """Compile the ablation libraries (in parallel: each is a full build of the library)."""
    from concurrent.futures import ThreadPoolExecutor
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    names = list(ABLATIONS) if names is None else list(names)

    def one(name):
        cmd = [hipcc] + HIPCC_FLAGS + ["-Wno-unused-but-set-variable", "-Wno-unused-variable"] + \
              ABLATIONS[name] + ["-o", ablation_lib(name)] + [os.path.join(CSRC, f) for f in SOURCES]
        r = subprocess.run(cmd, capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed ({name}):\n{r.stderr}")
        return ablation_lib(name)

    with ThreadPoolExecutor(max_workers=max(1, jobs)) as ex:
        return list(ex.map(one, names))


def stale() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS]
    return any(os.path.getmtime(d) > t for d in deps)


def build(force: bool = True, extra_flags=()) -> str:
    if not force and not stale():
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + list(extra_flags) + ["-o", LIB] + \
          [os.path.join(CSRC, f) for f in SOURCES]
    r = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(ln for ln in r.stderr.splitlines() if noise not in ln)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed:\n{err}")
    if err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build())
    print(build_tools())
    print(build_ablations())
