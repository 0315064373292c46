"""Build libvideoscan.so (HIP, gfx950 only) in-tree with hipcc."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libvideoscan.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I" + os.path.join(ROOT, "include"), "-I" + CSRC,
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def generate() -> None:
    """Write the generated instruction sequences that vs_prefill_mfma.hip includes."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("gen_prefill_asm", os.path.join(CSRC, "gen_prefill_asm.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    mod.main(os.path.join(CSRC, "vs_prefill_asm.inc"))


def check_prefill_listing(listing: str) -> None:
    """The prefill kernel keeps state in fixed registers that the compiler does not know about
    (accumulators and query fragments in a0..a191 for the whole kernel; scores, fragments and
    temporaries and packed probabilities in v128..v247 while the pipeline runs).  `listing` is the
    device assembly of vs_prefill_mfma.hip as written by the very compile that produced the library:
    make sure that no compiler-generated instruction touches a0..a191, or writes v128..v247 between the
    first matrix block and the marker that ends the pipeline, and that the kernels and the marker
    are there to be checked at all."""
    import re
    lines = listing.split("\n")
    kernels_seen, markers_seen = 0, 0
    kern, in_asm, live, body, bad, label_line = None, False, False, [], [], 0
    stores = ("global_store", "ds_write", "scratch_store", "buffer_store", "s_", "v_cmp", "v_readlane",
              "v_readfirstlane")
    for ln, raw in enumerate(lines, 1):
        t = raw.strip()
        m = re.match(r"^(_Z\w*prefill_mfma_kernel\w*):", t)
        if m:
            kern, live = m.group(1), False
            kernels_seen += 1
        if t.startswith(";;#ASMSTART"):
            in_asm, body = True, []
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            if any("v_mfma" in x for x in body):
                live = True
            if any("pipeline registers free" in x for x in body):
                markers_seen += 1
                live = False  # the marker's own basic block already belongs to the epilogue
                bad = [x for x in bad if x[0] < label_line or x[2]]
            continue
        if in_asm:
            body.append(t)
            continue
        if t.startswith(".LBB"):
            label_line = ln
        if kern is None or not t or t[0] in ";.":
            continue
        if t.startswith("s_endpgm"):
            kern = None
            continue
        for m in re.finditer(r"\ba(\d+)\b|\ba\[(\d+):(\d+)\]", t):
            if int(m.group(1) or m.group(2)) < 192:
                bad.append((ln, t, True))
        parts = t.split(None, 1)
        if live and len(parts) == 2 and not parts[0].startswith(stores):
            d = re.match(r"v(\d+)$|v\[(\d+):(\d+)\]$", parts[1].split(",")[0].strip())
            if d:
                lo = int(d.group(1) or d.group(2))
                hi = int(d.group(3) or lo)
                # (the exact redo of a sub-block rebuilds its packed probabilities in their fixed
                # registers v216..v247: those conversions are the one intended compiler write)
                rebuild = lo >= 216 and parts[0] == "v_cvt_pk_bf16_f32"
                if hi >= 128 and lo <= 247 and not rebuild:
                    bad.append((ln, t, False))
    if kernels_seen < 2 or markers_seen < kernels_seen:
        raise RuntimeError(f"prefill kernel: the listing shows {kernels_seen} kernels and {markers_seen} end-of-pipeline "
                           "markers; nothing was checked")
    if bad:
        raise RuntimeError("prefill kernel: the compiler touches registers reserved for the hand-scheduled "
                           "blocks:\n" + "\n".join(f"  line {ln}: {t}" for ln, t, _ in bad[:20]))


def build(verbose: bool = False) -> str:
    """Compiles the library and checks the prefill kernel's listing from that same compile (the
    compiler keeps its intermediate files, in a scratch directory); the library is put in place only
    if the check passes."""
    import glob as _glob
    import shutil
    import tempfile
    generate()
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "libvideoscan.so")
        cmd = [HIPCC] + FLAGS + ["-save-temps=cwd", "-o", out] + sources()
        if verbose:
            print(" ".join(cmd))
        subprocess.run(cmd, check=True, cwd=tmp)
        found = _glob.glob(os.path.join(tmp, "vs_prefill_mfma*gfx950*.s"))
        if len(found) != 1:
            raise RuntimeError(f"prefill kernel: expected one device listing of vs_prefill_mfma.hip, found {found}")
        check_prefill_listing(open(found[0]).read())
        shutil.copyfile(out, LIB)
        os.chmod(LIB, 0o755)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
