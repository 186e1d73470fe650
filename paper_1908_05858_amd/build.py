"""Builds libdabnn.so from the HIP sources with hipcc for gfx950 (in-tree, next to this file)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_PATH = os.path.join(HERE, "libdabnn.so")
SOURCES = (["dabnn_api.hip", "bitpack.hip", "bconv.hip", "bconv_areg.hip", "bconv_zeropad.hip", "bgemm.hip", "bconv_mfma.hip", "bconv_mfma_bits.hip"] +
           [f"bconv_areg_cw{cw}_s{st}.hip" for cw in (8, 7, 6, 5, 4, 3, 2, 1) for st in (1, 2)] +
           [f"bconv_areg_split_cw{cw}.hip" for cw in (4, 3, 2, 1)])
AREG_UNITS = [s for s in SOURCES if s.startswith("bconv_areg_") and "_cw" in s]
# -packed-fp32-ops is switched off for every HIP translation unit of this project.
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wextra",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# bitpack.hip holds the one kernel with float arithmetic (the fused BN + shortcut + sign layer),
# whose operations must round separately: no contraction into fused multiply-adds in that file.
EXTRA_FLAGS = {"bitpack.hip": ["-ffp-contract=off"]}
# ... and so does the BN + shortcut epilogue of the activation-stationary convolution kernels.
EXTRA_FLAGS.update({src: ["-ffp-contract=off"] for src in AREG_UNITS})


def build_library(verbose=False, incremental=False):
    """Compiles every translation unit and links the library.  `incremental` (a development
    convenience) skips units whose object file is newer than the unit and every header."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    headers = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    headers.append(os.path.join(os.path.dirname(HERE), "include", "dabnn.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    objs = []
    build_dir = os.path.join(HERE, "_build")
    os.makedirs(build_dir, exist_ok=True)
    procs = []
    for src in SOURCES:
        obj = os.path.join(build_dir, src.replace(".hip", ".o"))
        objs.append(obj)
        if incremental and os.path.exists(obj) and \
                os.path.getmtime(obj) > max(newest_header, os.path.getmtime(os.path.join(CSRC, src))):
            continue
        cmd = [hipcc] + HIPCC_FLAGS + EXTRA_FLAGS.get(src, []) + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stderr=subprocess.PIPE, text=True)))
    for cmd, p in procs:
        _, err = p.communicate()
        # hipcc's host pass does not know the device-only feature switch above and says so once
        # per translation unit; everything else it prints is shown
        err = "".join(l for l in err.splitlines(True) if "'-packed-fp32-ops' is not a recognized feature" not in l)
        if err.strip():
            print(err, end="", flush=True)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB_PATH]
    if verbose:
        print(" ".join(link), flush=True)
    subprocess.run(link, check=True)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
