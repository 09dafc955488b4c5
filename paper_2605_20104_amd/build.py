"""Builds libgraft.so (the C-ABI library) from the HIP sources with hipcc for gfx950."""
from __future__ import annotations

import os
import re
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
INCLUDE = os.path.join(ROOT, "include")
OBJ_DIR = os.path.join(PKG, "_build")
LIB = os.path.join(PKG, "libgraft.so")
LIB_TIMING = os.path.join(PKG, "libgraft_timing.so")     # the same library with the attention kernel's time stamps
SOURCES = ["api.hip", "retrieve.hip", "tree_mask.hip", "tree_attn.hip", "accept.hip", "matrix.hip", "kv_compact.hip", "prune.hip"]

# packed-fp32 code generation is switched off for every device compile; VGPR spills must not
# land in AccVGPRs (the attention kernel manages those by hand)
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", INCLUDE, "-I", CSRC,
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-mllvm", "-amdgpu-spill-vgpr-to-agpr=0",
               "-Wno-unused-command-line-argument"]


def _hipcc() -> str:
    for c in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if c and (os.path.isabs(c) and os.path.exists(c) or not os.path.isabs(c)):
            return c
    return "hipcc"


ATTN_ASM = os.path.join(OBJ_DIR, "tree_attn-hip-amdgcn-amd-amdhsa-gfx950.s")


def _compile(src: str, extra):
    obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
    return _compile_to(src, extra, obj)


def _compile_to(src: str, extra, obj: str):
    keep = ["-save-temps=obj"] if src == "tree_attn.hip" else []    # keeps the device assembly for the check below
    cmd = [_hipcc(), *HIPCC_FLAGS, *extra, *keep, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed for %s:\n%s" % (src, r.stdout))
    warn = [l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l and l.strip()]
    return obj, "\n".join(warn)


def _reg_span(tok: str):
    """'v12' -> ('v', 12, 12); 'a[4:7]' -> ('a', 4, 7); 'a[0xf0]' -> ('a', 240, 240); else None."""
    m = re.fullmatch(r"([va])(\d+|0x[0-9a-f]+)", tok)
    if m:
        n = int(m.group(2), 0)
        return m.group(1), n, n
    m = re.fullmatch(r"([va])\[(\d+|0x[0-9a-f]+):(\d+|0x[0-9a-f]+)\]", tok)
    if m:
        return m.group(1), int(m.group(2), 0), int(m.group(3), 0)
    m = re.fullmatch(r"([va])\[(\d+|0x[0-9a-f]+)\]", tok)
    if m:
        n = int(m.group(2), 0)
        return m.group(1), n, n
    return None


# Wait states between an MFMA and the first other instruction that may read its result: the
# passes of the widest MFMA used here (8) plus 3, as for the compiler's own MFMAs, plus one.
MFMA_RESULT_WAIT = 12


def check_attention_asm(asm_text: str):
    """Checks the generated device assembly of the MFMA attention kernels against the rules
    their hand-placed registers and inline-assembly MFMAs rely on.  Returns a list of
    violations (empty = fine):
      * no scratch memory (register spills) in any of the kernels;
      * outside the inline-assembly blocks no instruction names an AccVGPR below
        48 * MB + 4 * min(MB, 4) (the accumulators, the Q operand and the row sums live there
        and the compiler must not touch them);
      * no MFMA has a vector ALU instruction writing one of its VGPR sources within the two
        preceding wait states (an s_nop k counts k + 1): the hardware needs them and the
        compiler does not know that the asm statement is an MFMA.  The same holds for a
        v_accvgpr_write of an AccVGPR source;
      * no instruction other than an MFMA reads a register that an MFMA wrote within the
        MFMA_RESULT_WAIT preceding wait states, in program order across labels (the result of a
        16x16x32 MFMA is written at the end of its passes, and nothing interlocks a vector ALU,
        LDS or memory instruction, or a v_accvgpr_read, that comes earlier).
    """
    problems = []
    lines = asm_text.split("\n")
    kernel, mb, in_asm, desc = None, 0, False, ""
    history = []          # (wait states, destination span or None) of the preceding instructions
    results = []          # [wait states since, span] of MFMA results still inside MFMA_RESULT_WAIT

    def age(states):
        for r in results:
            r[0] += states
        while results and results[0][0] >= MFMA_RESULT_WAIT:
            del results[0]

    for ln, raw in enumerate(lines, 1):
        text = raw.split(";")[0].strip() if not raw.lstrip().startswith(";") else ""
        m = re.match(r"^(_ZN5graft21tree_attn_mfma_kernelILi(\d+)E\w*):", raw)
        if m:
            kernel, mb, history, results = m.group(1), int(m.group(2)), [(1, ("v", 0, 1 << 20))], []
            continue
        if kernel and raw.startswith(".Lfunc_end"):
            kernel = None
            continue
        if "ASMSTART" in raw:
            in_asm = True
            continue
        if "ASMEND" in raw:
            in_asm = False
            continue
        m = re.match(r"\s*\.amdhsa_kernel\s+(\S+)", raw)
        if m:
            desc = m.group(1)
            continue
        m = re.match(r"\s*\.amdhsa_private_segment_fixed_size\s+(\d+)", raw)
        if m:
            if "tree_attn_mfma_kernel" in desc and int(m.group(1)) != 0:
                problems.append("%s uses %s bytes of scratch memory (spills)" % (desc, m.group(1)))
            continue
        if not kernel:
            continue
        if raw.startswith(".LBB") or raw.startswith(".Ltmp"):
            if raw.startswith(".LBB"):
                # another block may jump here: assume that its last instruction wrote every VGPR
                history = [(1, ("v", 0, 1 << 20))]
            continue
        if not text or text.startswith("."):
            continue
        parts = text.replace(",", " ").split()
        op, args = parts[0], parts[1:]
        if not in_asm:
            for a in args:
                sp = _reg_span(a)
                if sp and sp[0] == "a" and sp[1] < 48 * mb + 4 * min(mb, 4):
                    problems.append("line %d (%s): compiler-generated use of a hand-managed AccVGPR: %s"
                                    % (ln, kernel, text))
        if op.startswith("v_mfma"):
            srcs = [sp for sp in map(_reg_span, args[1:]) if sp]
            states = 0
            for w, dst in reversed(history):
                if states >= 2:
                    break
                if dst is not None and any(dst[0] == s_[0] and dst[1] <= s_[2] and s_[1] <= dst[2] for s_ in srcs):
                    problems.append("line %d (%s): vector ALU write of an MFMA source %d wait state(s) before: %s"
                                    % (ln, kernel, states, text))
                    break
                states += w
            history.append((1, None))
            age(1)
            d = _reg_span(args[0]) if args else None
            if d:
                results.append([0, d])
            continue
        if op == "s_nop":
            history.append((int(args[0], 0) + 1, None))
            age(int(args[0], 0) + 1)
            continue
        # any other instruction: it must not read what an MFMA has just written (stores and LDS
        # writes have no destination: all their operands are read)
        reads = args if op.startswith(("global_store", "buffer_store", "flat_store", "ds_write", "ds_store",
                                       "global_atomic", "v_cmp")) else args[1:]
        for a in reads:
            sp = _reg_span(a)
            hit = sp and next((r for r in results if r[1][0] == sp[0] and r[1][1] <= sp[2] and sp[1] <= r[1][2]), None)
            if hit:
                problems.append("line %d (%s): read of an MFMA result %d wait state(s) after the MFMA: %s"
                                % (ln, kernel, hit[0], text))
                break
        dst = None
        if op.startswith("v_") and not op.startswith(("v_cmp", "v_readlane", "v_readfirstlane")) and args:
            sp = _reg_span(args[0])
            if sp and (sp[0] == "v" or op.startswith("v_accvgpr_write")):
                dst = sp
        history.append((1, dst))
        age(1)
        if len(history) > 8:
            del history[0]
    return problems


def _check_and_clean(asm_path: str, what: str):
    with open(asm_path) as f:
        problems = check_attention_asm(f.read())
    for name in os.listdir(OBJ_DIR):             # the other intermediate files are not needed
        if name.startswith("tree_attn") and not name.endswith((".o", "gfx950.s")) or name.endswith(".hipfb"):
            os.remove(os.path.join(OBJ_DIR, name))
    if problems:
        raise RuntimeError("%s: the generated assembly breaks a rule of the hand-scheduled kernel:\n  "
                           % what + "\n  ".join(problems[:20]))


def _link(objects, lib: str) -> str:
    tmp = lib + ".tmp%d" % os.getpid()
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *objects, "-o", tmp]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    os.replace(tmp, lib)
    return lib


def build(verbose: bool = False, extra_flags=()) -> str:
    """Compile every HIP source and link libgraft.so next to the package. Always recompiles."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(lambda s: _compile(s, list(extra_flags)), SOURCES))
    if verbose:
        for _, w in results:
            if w:
                print(w)
    _check_and_clean(ATTN_ASM, "tree_attn.hip")
    return _link([o for o, _ in results], LIB)


def build_timing(verbose: bool = False) -> str:
    """libgraft_timing.so: the library with the attention kernel compiled with -DGRAFT_ATTN_STAMPS
    (time stamps per workgroup, read by `python -m paper_2605_20104_amd.timing`).  The other
    objects are those of the last build(); the stamped kernels pass the same assembly check."""
    others = [os.path.join(OBJ_DIR, os.path.splitext(s)[0] + ".o") for s in SOURCES if s != "tree_attn.hip"]
    if not all(os.path.exists(o) for o in others):
        build(verbose)
    src_dir = os.path.join(OBJ_DIR, "timing")
    os.makedirs(src_dir, exist_ok=True)
    obj = os.path.join(src_dir, "tree_attn.o")
    _, warn = _compile_to("tree_attn.hip", ["-DGRAFT_ATTN_STAMPS"], obj)
    if verbose and warn:
        print(warn)
    asm = os.path.join(src_dir, "tree_attn-hip-amdgcn-amd-amdhsa-gfx950.s")
    with open(asm) as f:
        problems = check_attention_asm(f.read())
    for name in os.listdir(src_dir):
        if not name.endswith((".o", "gfx950.s")):
            os.remove(os.path.join(src_dir, name))
    if problems:
        raise RuntimeError("tree_attn.hip (timing build): the generated assembly breaks a rule of the "
                           "hand-scheduled kernel:\n  " + "\n  ".join(problems[:20]))
    return _link([obj, *others], LIB_TIMING)


if __name__ == "__main__":
    flags = [a for a in sys.argv[1:] if a != "--timing"]
    print(build(verbose=True, extra_flags=flags))
    if "--timing" in sys.argv[1:]:
        print(build_timing(verbose=True))
