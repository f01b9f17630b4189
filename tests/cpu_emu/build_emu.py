"""Builds the library's HIP sources for the host CPU (g++), for tests only: the sources are copied
with four textual changes (dynamic LDS declarations, the one inline-assembly barrier, `__shared__`, the
place of a file-scope array's alignment)
and compiled against the stand-in header in this folder."""
import os
import re
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
CSRC = os.path.join(ROOT, "paper_2101_05600_amd", "csrc")


_DECL = re.compile(r"^(\s*)__shared__\s+((?:__align__\(\d+\)|__attribute__\(\(aligned\(\d+\)\)\))\s+)?([^;]*);", re.M)


def _rewrite_lds(text):
    """`__shared__ T a[N], b;` -> references into the running work-group's LDS arena, which the
    emulation fills with a poison pattern before every work-group (as on the GPU, LDS holds
    whatever was there: a kernel that reads an element it has not written must not get zeros)."""
    def strip_comments(body):
        return "\n".join(line.split("//")[0] for line in body.split("\n"))

    def one(m):
        indent, align, body = m.group(1), m.group(2), strip_comments(m.group(3))
        al = re.search(r"\d+", align).group(0) if align else "16"
        parts = [d.strip() for d in body.replace("\n", " ").split(",")]
        first = re.match(r"^(.*?)(\w+)\s*((?:\[[^\]]*\])*)$", parts[0])
        base = first.group(1).strip()
        decls = [(first.group(2), first.group(3))]
        for d in parts[1:]:
            mm = re.match(r"^(\w+)\s*((?:\[[^\]]*\])*)$", d)
            decls.append((mm.group(1), mm.group(2)))
        out = []
        for name, dims in decls:
            out.append(f"{indent}typedef {base} emu_t_{name}{dims}; "
                       f"emu_t_{name}& {name} = *emu::lds<emu_t_{name}>(__COUNTER__, {al});")
        return "\n".join(out)
    return _DECL.sub(one, text)


def _patch(text):
    text = re.sub(r"extern\s+__shared__\s+(?:__align__\(\d+\)\s+)?unsigned char\s+(\w+)\[\];",
                  r"unsigned char* const \1 = emu::dyn_smem();", text)
    text, n = re.subn(r'asm volatile\("s_waitcnt lgkmcnt\(0\)\\n\\ts_barrier" ::: "memory"\);',
                      "emu::wg_barrier();", text)
    # (g++ wants the alignment of a file-scope array before `static`)
    text = re.sub(r"static __device__ __align__\((\d+)\) ", r"alignas(\1) static ", text)
    text = _rewrite_lds(text)
    text = text.replace('#include "../../include/ctcbs.h"', f'#include "{ROOT}/include/ctcbs.h"')
    return text


def build(out_dir, sanitize=True, plant=None):
    """-> path of libctcbs_emu.so.  sanitize: True = AddressSanitizer + UBSan, "thread" = ThreadSanitizer
    (work-items are OS threads and LDS is ordinary memory, so a missing barrier shows as a data race),
    False = plain.  plant: optional (file name, old text, new text) applied to the copied source: a
    deliberate mistake, for the self-test that shows the sanitizer run notices one."""
    src_dir = os.path.join(out_dir, "src")
    shutil.rmtree(src_dir, ignore_errors=True)
    os.makedirs(src_dir)
    for name in os.listdir(CSRC):
        with open(os.path.join(CSRC, name)) as f:
            text = _patch(f.read())
        if "asm volatile" in text:
            raise RuntimeError(f"{name}: inline assembly the CPU build does not know")
        if plant and plant[0] == name:
            if plant[1] not in text:
                raise RuntimeError(f"{name}: the text to replace is not there")
            text = text.replace(plant[1], plant[2], 1)
        out_name = "ctcbs.cpp" if name == "ctcbs.hip" else name
        with open(os.path.join(src_dir, out_name), "w") as f:
            f.write(text)
    so = os.path.join(out_dir, "libctcbs_emu.so")
    cmd = ["g++", "-std=c++20", "-O1", "-g", "-fPIC", "-shared", "-pthread", "-fno-strict-aliasing",
           "-I", HERE, "-o", so, os.path.join(src_dir, "ctcbs.cpp")]
    if sanitize == "thread":
        cmd[1:1] = ["-fsanitize=thread", "-fno-omit-frame-pointer"]
    elif sanitize:
        cmd[1:1] = ["-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-fno-sanitize=alignment,float-cast-overflow"]
    subprocess.check_call(cmd)
    return so


if __name__ == "__main__":
    import sys
    print(build(sys.argv[1] if len(sys.argv) > 1 else os.path.join(ROOT, "_build", "cpu_emu"),
                sanitize=False if "--plain" in sys.argv else ("thread" if "--thread" in sys.argv else True)))
