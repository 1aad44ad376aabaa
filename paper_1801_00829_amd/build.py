"""Build libfuse.so (host C++ + the statically compiled probe kernels) with hipcc for gfx950."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfuse.so")
ARCH = "gfx950"

HOST_SOURCES = ["libfuse.cpp", "expr.cpp", "runtime.cpp"]
DEVICE_SOURCES = ["probe.hip", "check.hip", "transpose.hip", "noalloc.hip"]
TEXT_DEPS = ["fuse_args.h", "skel_common.inc", "skel_cell.inc", "skel_row_dense.inc", "skel_row_csr.inc", "skel_row_csr_stream.inc", "skel_row_mfma.inc", "skel_row_mfma_wave.inc",
             "skel_outer.inc", "expr.h", "runtime.h"]


def _gen_args_text():
    """The kernel-argument header is also compiled by hipRTC: wrap its text as a raw string."""
    with open(os.path.join(CSRC, "fuse_args.h")) as f:
        text = f.read()
    out = os.path.join(CSRC, "gen_args_text.inc")
    body = 'R"FUSESKEL(\n' + text + ')FUSESKEL"\n'
    if not os.path.exists(out) or open(out).read() != body:
        with open(out, "w") as f:
            f.write(body)
    return out


def needs_build() -> bool:
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    srcs = HOST_SOURCES + DEVICE_SOURCES + TEXT_DEPS
    paths = [os.path.join(CSRC, s) for s in srcs] + [os.path.join(HERE, "..", "include", "fuse.h")]
    return any(os.path.getmtime(p) > t for p in paths)


def build(force: bool = True, verbose: bool = False) -> str:
    """Compile everything; returns the path of libfuse.so."""
    if not force and not needs_build():
        return LIB
    _gen_args_text()
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    common = ["-O2", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-result", "--offload-arch=" + ARCH]
    objs = []
    for s in HOST_SOURCES + DEVICE_SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(s)[0] + ".o")
        if s.endswith(".hip"):
            # never let the compiler form packed-fp32 instructions (device code only)
            cmd = [hipcc] + common + ["-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                                      "-c", os.path.join(CSRC, s), "-o", obj]
        else:
            # host-only translation units (no kernels inside); built as HIP for the runtime headers
            cmd = [hipcc] + common + ["-x", "hip", "-c", os.path.join(CSRC, s), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True)
        objs.append(obj)
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [hipcc, "-shared", "-fPIC", "--offload-arch=" + ARCH, "-o", tmp] + objs + \
          ["-L/opt/rocm/lib", "-lhiprtc", "-Wl,-rpath,/opt/rocm/lib"]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose="-v" in sys.argv))
