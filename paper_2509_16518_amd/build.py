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


def check_inline_asm_hazards(asm_path):
    """Vector-memory instructions written as inline assembly (the LDS-DMA gathers, the untracked id loads) get none of
    the wait states the compiler inserts for hardware hazards.  The one that could apply to them: a vector-ALU
    instruction that writes a scalar register (v_readfirstlane, v_readlane, a compare with a scalar destination) must be
    five wait states ahead of a vector-memory instruction that reads that register as its base.  The kernels keep such
    bases in scalar registers from the start, so no such write should be anywhere near; this scan fails the build if
    one ever is."""
    import re
    sreg = re.compile(r"\bs\[(\d+):(\d+)\]|\bs(\d+)\b")
    window = []   # (wait states this instruction contributes, scalar registers a vector-ALU instruction writes)
    with open(asm_path) as f:
        for n, line in enumerate(f, 1):
            code = line.split(";", 1)[0].strip()
            if not code or code.startswith(".") or code.endswith(":"):
                continue
            op = code.split()[0]
            if op.startswith("global_load") or op.startswith("global_store"):
                m = sreg.search(code.split(None, 1)[1]) if " " in code else None
                if m:
                    lo, hi = (int(m.group(1)), int(m.group(2))) if m.group(1) else (int(m.group(3)), int(m.group(3)))
                    states = 0
                    for w, written in reversed(window):
                        if states >= 5:
                            break
                        if any(lo <= r <= hi for r in written):
                            raise RuntimeError("%s:%d: a vector-ALU write of s%s is only %d wait states ahead of %s" %
                                               (asm_path, n, sorted(written), states, code))
                        states += w
            written = set()
            if op.startswith("v_"):
                first = code.split(None, 1)[1].split(",")[0] if " " in code else ""
                m = sreg.fullmatch(first.strip())
                if m:
                    written = set(range(int(m.group(1)), int(m.group(2)) + 1)) if m.group(1) else {int(m.group(3))}
            states = 1
            if op == "s_nop":
                states = int(code.split()[1], 0) + 1
            window.append((states, written))
            if len(window) > 8:
                window.pop(0)


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
            check_inline_asm_hazards(os.path.join(objdir, f))
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
