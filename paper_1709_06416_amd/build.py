"""Build libweldhip.so (host runtime + ahead-of-time gfx950 kernels) in-tree.

    python -m paper_1709_06416_amd.build            # library + precompiled fused kernels
    python -m paper_1709_06416_amd.build --lib-only

hipcc cross-compiles for gfx950 without a GPU.  The device-side prelude of the
run-time compiled kernels is embedded into the library as a string.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
ROOT = os.path.dirname(HERE)
INCLUDE = os.path.join(ROOT, "include")
BUILD = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libweldhip.so")
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HOST_SOURCES = ["validate.cpp", "codegen.cpp", "jit.cpp", "pool.cpp", "runtime.cpp", "unfused.cpp", "lazy.cpp", "nested.cpp", "tuner.cpp"]
HIP_SOURCES = ["aot_kernels.hip", "spill_kernels.hip", "static_entry.hip"]
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")
HIPCC = os.path.join(ROCM, "bin", "hipcc")

COMMON = ["-O2", "-fPIC", "-std=c++17", "-I" + INCLUDE, "-I" + CSRC, "-I" + os.path.join(ROCM, "include"),
          "-D__HIP_PLATFORM_AMD__", "-Wall", "-Werror=format", "-Wno-unused-function"]
DEVICE = ["--offload-arch=gfx950", "-ffp-contract=off",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        sys.stderr.write(" ".join(cmd) + "\n" + r.stdout + "\n")
        raise RuntimeError("build step failed: " + cmd[-1])
    return r.stdout


def _embed_prelude():
    src = open(os.path.join(CSRC, "fused_prelude.hip.h")).read()
    from paper_1709_06416_amd import erf_table, logexp_table
    assert src.count("@W_ERF_TABLE@") == 1
    src = src.replace("@W_ERF_TABLE@", erf_table.c_initialiser())
    for mark, text in (("@W_LOG_TABLE@", logexp_table.log_initialiser()), ("@W_EXP_TABLE@", logexp_table.exp_initialiser()),
                       ("@W_LOGEXP_CONSTS@", logexp_table.constant_defines())):
        assert src.count(mark) == 1
        src = src.replace(mark, text)
    assert ')WELDPRE"' not in src
    out = os.path.join(BUILD, "prelude_embed.cpp")
    # split into chunks: string literals have a length limit in some compilers
    chunks = [src[i:i + 8000] for i in range(0, len(src), 8000)]
    body = "\n".join('R"WELDPRE(' + c + ')WELDPRE"' for c in chunks)
    text = ("// generated from fused_prelude.hip.h\nnamespace weld {\n"
            "extern const char* const kPreludeSource;\n"
            "const char* const kPreludeSource =\n" + body + ";\n}\n")
    if not os.path.exists(out) or open(out).read() != text:
        open(out, "w").write(text)
    return out


def build_library(verbose=False):
    os.makedirs(BUILD, exist_ok=True)
    objs = []
    embed = _embed_prelude()
    jobs = [(os.path.join(CSRC, s), False) for s in HOST_SOURCES] + [(embed, False)]
    jobs += [(os.path.join(CSRC, s), True) for s in HIP_SOURCES if os.path.exists(os.path.join(CSRC, s))]
    procs = []
    for path, is_hip in jobs:
        obj = os.path.join(BUILD, os.path.basename(path) + ".o")
        objs.append(obj)
        cmd = [HIPCC] + COMMON
        if is_hip:
            cmd += DEVICE + ["-x", "hip"]
        else:
            cmd += ["-x", "c++"]
        cmd += ["-c", path, "-o", obj]
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for cmd, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            sys.stderr.write(" ".join(cmd) + "\n" + out + "\n")
            failed = True
        elif verbose and out.strip():
            sys.stderr.write(out)
    if failed:
        raise RuntimeError("compilation of libweldhip failed")
    link = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs + \
           ["-L" + os.path.join(ROCM, "lib"), "-lhiprtc", "-lamdhip64", "-ldl", "-lpthread"]
    _run(link)
    return LIB


def precompile_standard_kernels():
    """Compile the fused kernels of the benchmark loops into the in-tree cache (the probe side of the
    join takes its dictionary's types from a result handle and is compiled on first use)."""
    sys.path.insert(0, ROOT)
    from paper_1709_06416_amd import binding
    from workloads import configs
    names = []
    for name, make in configs.PROGRAMS.items():
        binding.precompile(make())
        names.append(name)
    for name, make in configs.EXAMPLES.items():
        binding.precompile(make())
        names.append(name)
    from workloads import graphs
    binding.precompile(graphs.program_contrib())
    binding.nested_precompile(graphs.program_pagerank(graphs.PAGERANK_VERTICES))
    binding.nested_precompile(graphs.program_spmv())
    names += ["pagerank", "spmv"]
    from workloads import joins
    binding.precompile(configs.program_group_by_zip())
    binding.precompile(joins.program_build(joins.ORDERS))
    names += ["group_by_zip", "join_build"]
    return names


def main(argv):
    lib = build_library(verbose="-v" in argv)
    print("built", lib)
    if "--lib-only" not in argv:
        print("precompiled", precompile_standard_kernels())


if __name__ == "__main__":
    main(sys.argv[1:])
