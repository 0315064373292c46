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


def check_prefill_listing() -> None:
    """The prefill kernel keeps state in fixed registers that the compiler does not know about
    (accumulators and query fragments in a0..a191 for the whole kernel; scores, fragments and
    temporaries and packed probabilities in v128..v247 while the pipeline runs).  Compile it to a listing and make sure
    that no compiler-generated instruction touches a0..a191, or writes v128..v247 between the
    first matrix block and the marker that ends the pipeline."""
    import re
    import tempfile
    src = os.path.join(CSRC, "vs_prefill_mfma.hip")
    with tempfile.TemporaryDirectory() as tmp:
        lst = os.path.join(tmp, "prefill.s")
        flags = [f for f in FLAGS if f not in ("-shared", "-fPIC")]
        subprocess.run([HIPCC] + flags + ["-S", "--cuda-device-only", "-o", lst, src], check=True,
                       stderr=subprocess.DEVNULL)
        lines = open(lst).read().split("\n")
    kern, in_asm, live, body, bad, label_line = None, False, False, [], [], 0
    stores = ("global_store", "ds_write", "scratch_store", "buffer_store", "s_", "v_cmp", "v_readlane",
              "v_readfirstlane")
    for ln, raw in enumerate(lines, 1):
        t = raw.strip()
        m = re.match(r"^(_Z\w*prefill_mfma_kernel\w*):", t)
        if m:
            kern, live = m.group(1), False
        if t.startswith(";;#ASMSTART"):
            in_asm, body = True, []
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            if any("v_mfma" in x for x in body):
                live = True
            if any("pipeline registers free" in x for x in body):
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
    if bad:
        raise RuntimeError("prefill kernel: the compiler touches registers reserved for the hand-scheduled "
                           "blocks:\n" + "\n".join(f"  line {ln}: {t}" for ln, t, _ in bad[:20]))


def build(verbose: bool = False) -> str:
    generate()
    check_prefill_listing()
    cmd = [HIPCC] + FLAGS + ["-o", LIB] + sources()
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
