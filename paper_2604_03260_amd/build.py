"""Builds libfocus.so (HIP, gfx950) in-tree next to this file."""
import os
import re
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfocus.so")
SOURCES = ["focus_api.hip", "focus_assign.hip", "focus_attn_simple.hip", "focus_attn_mfma.hip",
           "focus_route.hip", "focus_decode.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=on", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-result", "-Wno-unused-command-line-argument"]


def source_id():
    """Hash of everything the library is compiled from (sources, internal headers, the public header, the
    flags).  The build stores it in the library (focus_build_id); the binding compares it on load."""
    import hashlib
    h = hashlib.sha256()
    names = sorted(os.listdir(CSRC))
    for name in names:
        path = os.path.join(CSRC, name)
        if os.path.isfile(path) and name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(path, "rb").read())
    h.update(open(os.path.join(os.path.dirname(HERE), "include", "focus.h"), "rb").read())
    h.update(" ".join(FLAGS).encode())
    return h.hexdigest()[:16]


# The attention kernel reads its LDS operands with inline ds_read whose completion the compiler does not track
# (one s_waitcnt before the matrix products).  A register spilled between such a read and its wait would be
# stored before the data has arrived, so a build in which any instantiation of that kernel spills is refused.
NO_SPILL_SOURCE = "focus_attn_mfma.hip"
NO_SPILL_KERNEL = "attn_mfma_kernel"


def check_no_spills(remarks):
    """remarks: the compiler's -Rpass-analysis=kernel-resource-usage output.  Returns the number of kernels seen."""
    seen = 0
    for block in remarks.split("Function Name:")[1:]:
        name = block.split()[0]
        if NO_SPILL_KERNEL not in name:
            continue
        seen += 1
        m = re.search(r"VGPRs Spill:\s*(\d+)", block)
        s = re.search(r"ScratchSize \[bytes/lane\]:\s*(\d+)", block)
        if m is None or int(m.group(1)) != 0 or (s is not None and int(s.group(1)) != 0):
            raise RuntimeError("%s spills registers (%s): its untracked LDS reads are unsafe, see build.py"
                               % (name, m.group(0) if m else "no report"))
    if seen == 0:
        raise RuntimeError("no resource report for %s: cannot check for spills" % NO_SPILL_KERNEL)
    return seen


def build_library(verbose=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for s in SOURCES:
        o = os.path.join(HERE, "_build", s.replace(".hip", ".o"))
        cmd = [hipcc] + [f for f in FLAGS if f != "-shared"] + ["-c", os.path.join(CSRC, s), "-o", o]
        if s == "focus_api.hip":
            cmd.insert(1, '-DFOCUS_BUILD_ID="%s"' % source_id())
        err = None
        if s == NO_SPILL_SOURCE:
            cmd.insert(1, "-Rpass-analysis=kernel-resource-usage")
            err = open(os.path.join(HERE, "_build", "resource_usage.txt"), "w")
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((subprocess.Popen(cmd, stderr=err), cmd, err))
        objs.append(o)
    for p, cmd, err in procs:
        rc = p.wait()
        if err is not None:
            err.close()
            remarks = open(err.name).read()
            if rc != 0:
                sys.stderr.write(remarks[-4000:])
            else:
                n = check_no_spills(remarks)
                if verbose:
                    print("%d instantiations of %s, none spills" % (n, NO_SPILL_KERNEL), flush=True)
        if rc != 0:
            raise RuntimeError("compile failed: " + " ".join(cmd))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def build_ablation(bits, verbose=False):
    """_build/libfocus_ablate_<bits>.so: the library with the attention kernel compiled with -DFOCUS_ABLATE=<bits>
    (one ingredient of its key-tile loop taken out, see focus_attn_mfma.hip).  For timing only (profiles/
    attn_loop_ablation.txt): its results are meaningless.  Needs the objects of a normal build."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    bdir = os.path.join(HERE, "_build")
    o = os.path.join(bdir, "focus_attn_mfma_ablate_%d.o" % bits)
    cmd = [hipcc, "-DFOCUS_ABLATE=%d" % bits] + [f for f in FLAGS if f != "-shared"] + \
          ["-c", os.path.join(CSRC, NO_SPILL_SOURCE), "-o", o]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
    objs = [o] + [os.path.join(bdir, s.replace(".hip", ".o")) for s in SOURCES if s != NO_SPILL_SOURCE]
    out = os.path.join(bdir, "libfocus_ablate_%d.so" % bits)
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + objs)
    return out


def build_probes(verbose=False):
    """The stand-alone MFMA-rate program under csrc/probes that bench.py runs as a child process (not part of the library)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = os.path.join(HERE, "_build", "mfma_peak")
    os.makedirs(os.path.dirname(out), exist_ok=True)
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-w", "-o", out, os.path.join(CSRC, "probes", "mfma_peak.hip")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return out


if __name__ == "__main__":
    if "--ablate" in sys.argv:                      # python build.py --ablate 1 2 4 8
        for b in sys.argv[sys.argv.index("--ablate") + 1:]:
            print(build_ablation(int(b), verbose=True))
        sys.exit(0)
    print(build_library(verbose=True))
    print(build_probes(verbose=True))
