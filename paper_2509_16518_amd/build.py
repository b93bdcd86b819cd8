"""In-tree builds: the HIP C-ABI library (hipcc, gfx950) and the input-generator library (gcc)."""
import os
import subprocess

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
REPO_DIR = os.path.dirname(PKG_DIR)
CSRC = os.path.join(PKG_DIR, "csrc")
LIBFGATTN = os.path.join(PKG_DIR, "libfgattn.so")
LIBFGW = os.path.join(PKG_DIR, "workloads", "libfgw.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-fno-honor-nans",
]


def _run(cmd):
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("build failed: %s\n%s" % (" ".join(cmd), r.stdout))
    return r.stdout


def build_workloads(force=True):
    src = os.path.join(PKG_DIR, "workloads", "fgw_gen.c")
    if force or not os.path.exists(LIBFGW):
        _run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", src, "-o", LIBFGW, "-lm"])
    return LIBFGW


def check_m0_writes(asm_path):
    """The gathers of the forward kernel set the LDS-DMA base register M0 in one inline-assembly statement and rely
    on it in the following ones; nothing the compiler emits in between may write M0.  Every mention of M0 in the
    device assembly must therefore be one of the kernel's own marked `s_mov_b32 m0` lines."""
    import re
    tok = re.compile(r"\bm0\b")
    with open(asm_path) as f:
        for n, line in enumerate(f, 1):
            code = line.split(";", 1)[0]
            if tok.search(code) and "fg_m0" not in line:
                raise RuntimeError("%s:%d: M0 is touched outside the kernel's own gather statements: %s" %
                                   (asm_path, n, line.strip()))


def build_hip(force=True, extra_flags=()):
    """Compile every .hip translation unit for gfx950 (in parallel) and link libfgattn.so in-tree."""
    from concurrent.futures import ThreadPoolExecutor
    srcs = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith(".hip")]
    if not force and os.path.exists(LIBFGATTN):
        return LIBFGATTN
    objdir = os.path.join(PKG_DIR, "_build")
    os.makedirs(objdir, exist_ok=True)
    common = [f for f in HIP_FLAGS if f != "-shared"] + list(extra_flags) + \
        ["-save-temps=obj", "-I", os.path.join(REPO_DIR, "include"), "-I", CSRC]
    objs = [os.path.join(objdir, os.path.basename(s)[:-4] + ".o") for s in srcs]
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        list(ex.map(lambda so: _run([HIPCC] + common + ["-c", so[0], "-o", so[1]]), zip(srcs, objs)))
    for f in sorted(os.listdir(objdir)):
        if f.endswith("-gfx950.s"):
            check_m0_writes(os.path.join(objdir, f))
        elif not f.endswith(".o"):
            os.remove(os.path.join(objdir, f))   # other intermediates of -save-temps
    _run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIBFGATTN])
    return LIBFGATTN


def source_id():
    """What a measurement script prints so that its table can be tied to a tree: the git commit if this is a
    checkout (with '+' if tracked files differ from it), and a digest of the kernel and generator sources, which can
    be recomputed from any copy of the files."""
    import hashlib
    head = "unknown"
    try:
        r = subprocess.run(["git", "-C", REPO_DIR, "rev-parse", "--short=12", "HEAD"], stdout=subprocess.PIPE,
                           stderr=subprocess.DEVNULL, text=True)
        if r.returncode == 0 and r.stdout.strip():
            head = r.stdout.strip()
            d = subprocess.run(["git", "-C", REPO_DIR, "status", "--porcelain", "--untracked-files=no"],
                               stdout=subprocess.PIPE, stderr=subprocess.DEVNULL, text=True)
            if d.returncode == 0 and d.stdout.strip():
                head += "+"
    except OSError:
        pass
    h = hashlib.sha256()
    files = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC)) if f.endswith((".hip", ".hpp"))]
    files += [os.path.join(REPO_DIR, "include", "fgattn.h"), os.path.join(PKG_DIR, "workloads", "fgw_gen.c")]
    for path in files:
        with open(path, "rb") as f:
            h.update(os.path.basename(path).encode() + b"\0" + f.read())
    return {"git_head": head, "source_sha256": h.hexdigest()[:16]}
