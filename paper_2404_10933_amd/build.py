"""Builds libllmem.so (gfx950) in-tree with hipcc.

Two stages.  First every HIP source is compiled and linked into a bootstrap library whose list
of built-in specialized kernels is empty; its host-only entry point llmem_compiled_tables then
turns each table set the library ships with into the words a specialized kernel holds as
constants.  Second, estimate_batch.hip is compiled once per (table set, flavour) with those
words (LLMEM_SPECIALIZED), the list of what was built is written to csrc/aot_registry.inc, and
everything is linked into libllmem.so.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libllmem.so")
WORK = os.path.join(ROOT, "_build")
SOURCES = ("estimate.hip", "estimate_batch.hip", "specialize.hip", "decide.hip", "timeline.hip", "generate.hip")
# what the run-time build of the specialized kernel compiles: the kernel source first, then the
# headers it includes, each under its bare name
EMBEDDED = (("estimate_batch.hip", os.path.join(CSRC, "estimate_batch.hip")),
            ("llmem.h", os.path.join(HERE, "..", "include", "llmem.h")),
            ("estimate_args.h", os.path.join(CSRC, "estimate_args.h")),
            ("grid_draws.h", os.path.join(CSRC, "grid_draws.h")),
            ("wave.h", os.path.join(CSRC, "wave.h")))
HIPCC_FLAGS = ("--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops")
FLAVOURS = ("peaks", "detail", "sweep")          # LLMEM_SPEC_FLAVOUR 0, 1, 2
PROGRAM_WORDS = 704
JOBS = min(8, os.cpu_count() or 1)


def shipped_table_sets():
    """The table sets the library has built-in specialized kernels for: (name, [tables]).
    LLMEM_BUILD_TABLES=package.module:function adds the caller's own: the function returns
    further (name, [tables]) pairs (names of letters, digits and underscores), so that tables
    the library does not ship get kernels of the same kind without the run-time compiler."""
    from workloads import tables as T
    sets = []
    for family, make in T.FAMILIES.items():
        sets.append((family, [make()]))
        sets.append((family + "_full", [make(checkpoint=False)]))
    sets.append(("zoo", [T.gpt_table(), T.opt_table(), T.llama_table()]))
    extra = os.environ.get("LLMEM_BUILD_TABLES", "")
    if extra:
        import importlib
        module, _, function = extra.partition(":")
        taken = {name for name, _ in sets}
        for name, tables in getattr(importlib.import_module(module), function)():
            if not name.replace("_", "").isalnum() or name in taken:
                raise ValueError(f"LLMEM_BUILD_TABLES: bad or repeated table set name {name!r}")
            taken.add(name)
            sets.append((name, list(tables)))
    return sets


def _hipcc() -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return hipcc if os.path.exists(hipcc) else "hipcc"


def _run(cmd) -> None:
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + res.stdout + res.stderr)


def write_embedded_sources() -> str:
    """csrc/embedded_sources.inc: the kernel source and its headers as string literals."""
    out = ["// written by build.py from the files next to it; not edited by hand",
           f"static const int EMBEDDED_COUNT = {len(EMBEDDED)};",
           "static const char *const EMBEDDED_NAMES[] = {" + ", ".join(f'"{n}"' for n, _ in EMBEDDED) + "};",
           "static const char *const EMBEDDED_TEXTS[] = {"]
    for _, path in EMBEDDED:
        text = open(path).read()
        assert ')LLMEM_SRC"' not in text
        # string literals are limited in length by some compilers: one literal per 8 KB, concatenated
        chunks = [text[i:i + 8192] for i in range(0, len(text), 8192)]
        out.append("\n".join(f'R"LLMEM_SRC({c})LLMEM_SRC"' for c in chunks) + ",")
    out.append("};")
    path = os.path.join(CSRC, "embedded_sources.inc")
    with open(path, "w") as f:
        f.write("\n".join(out) + "\n")
    return path


def _compile(source: str, obj: str, defines=()) -> str:
    _run([_hipcc(), *HIPCC_FLAGS, *defines, "-c", os.path.join(CSRC, source), "-o", obj])
    return obj


def _link(objects, lib: str) -> None:
    _run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objects, "-lhiprtc"])


def compiled_words(lib_path: str, tables):
    """(words, first) of a table set from the host-only entry point of the library at lib_path."""
    from . import binding
    lib = ctypes.CDLL(lib_path)
    lib.llmem_compiled_tables.argtypes = [ctypes.c_void_p, ctypes.POINTER(ctypes.c_uint32), ctypes.c_int32,
                                          ctypes.POINTER(ctypes.c_int32)]
    lib.llmem_compiled_tables.restype = ctypes.c_int
    tab = binding.Tables(tables, device=None)
    words = (ctypes.c_uint32 * PROGRAM_WORDS)()
    first = (ctypes.c_int32 * binding.MAX_ARCH)()
    n = lib.llmem_compiled_tables(ctypes.byref(tab.struct), words, PROGRAM_WORDS, first)
    if n < 0:
        raise RuntimeError(f"llmem_compiled_tables: error {n}")
    return list(words[:n]), list(first)


def _word_list(words) -> str:
    rows = [", ".join(f"0x{w:08x}u" for w in words[i:i + 8]) for i in range(0, len(words), 8)]
    return ", \\\n".join(rows)


def write_constants(path: str, n_arch: int, words, first) -> None:
    """The constants of one specialized build as macros (what estimate_batch.hip includes)."""
    with open(path, "w") as f:
        f.write("#pragma once\n"
                f"#define LLMEM_SPEC_WAVES {5 if n_arch == 1 else 3}\n"      # waves per SIMD the build aims at
                f"#define LLMEM_SPEC_ARCHS {n_arch}\n"
                f"#define LLMEM_SPEC_FIRSTS {', '.join(str(v) for v in first)}\n"
                f"#define LLMEM_SPEC_WORDS \\\n{_word_list(words)}\n")


def write_registry(path: str, entries) -> None:
    """csrc/aot_registry.inc: the built-in specialized kernels and the words they were made from.
    entries: (set name, flavour, n_arch, first, words, entry symbol)."""
    out = ["// written by build.py; not edited by hand"]
    seen = {}
    for name, flavour, n_arch, first, words, symbol in entries:
        out.append(f'extern "C" const void *{symbol}();')
        if name not in seen:
            seen[name] = f"AOT_WORDS_{len(seen)}"
            out.append(f"static const uint32_t {seen[name]}[] = {{\n{_word_list(words).replace(chr(92), '')}}};")
    out.append("static const llmem::Prebuilt PREBUILT[] = {")
    for name, flavour, n_arch, first, words, symbol in entries:
        out.append(f'    {{"{name}", {flavour}, {n_arch}, {{{", ".join(str(v) for v in first)}}}, {len(words)}, '
                   f"{seen[name]}, {symbol}}},")
    if not entries:
        out.append('    {"", -1, 0, {0, 0, 0, 0, 0, 0, 0, 0}, 0, nullptr, nullptr},')
    out.append("};")
    out.append(f"static const int PREBUILT_COUNT = {len(entries)};")
    with open(path, "w") as f:
        f.write("\n".join(out) + "\n")


def build(verbose: bool = False) -> str:
    """Compile every HIP source into the shared library; always recompiles."""
    os.makedirs(WORK, exist_ok=True)
    write_embedded_sources()
    registry = os.path.join(CSRC, "aot_registry.inc")
    empty = os.path.join(WORK, "aot_registry_empty.inc")
    write_registry(empty, [])
    with ThreadPoolExecutor(JOBS) as pool:
        # ---- stage 1: the library without built-in specializations
        jobs = [pool.submit(_compile, s, os.path.join(WORK, s + ".o"),
                            (f'-DLLMEM_AOT_REGISTRY="{empty}"',) if s == "specialize.hip" else ())
                for s in SOURCES]
        objects = [j.result() for j in jobs]
        bootstrap = os.path.join(WORK, "libllmem_bootstrap.so")
        _link(objects, bootstrap)
        # ---- stage 2: one kernel per shipped table set and flavour
        entries, jobs = [], []
        for name, tables in shipped_table_sets():
            words, first = compiled_words(bootstrap, tables)
            header = os.path.join(WORK, f"aot_{name}.h")
            write_constants(header, len(tables), words, first)
            for flavour, tag in enumerate(FLAVOURS):
                kernel = f"llmem_aot_{name}_{tag}"
                entries.append((name, flavour, len(tables), first, words, kernel + "_entry"))
                jobs.append(pool.submit(_compile, "estimate_batch.hip", os.path.join(WORK, f"aot_{name}_{tag}.o"),
                                        ("-DLLMEM_SPECIALIZED", f"-DLLMEM_SPEC_FLAVOUR={flavour}",
                                         f'-DLLMEM_SPEC_HEADER="{header}"', f"-DLLMEM_SPEC_KERNEL={kernel}",
                                         f"-DLLMEM_SPEC_ENTRY={kernel}_entry")))
        write_registry(registry, entries)
        jobs.append(pool.submit(_compile, "specialize.hip", os.path.join(WORK, "specialize_final.o")))
        aot_objects = [j.result() for j in jobs]
    final = [o for o in objects if not o.endswith("specialize.hip.o")] + aot_objects
    _link(final, LIB)
    if verbose:
        print(f"{LIB}: {len(entries)} built-in specialized kernels")
    return LIB


def build_calibrate() -> str:
    """Compile the stand-alone calibration program (instruction issue rates, HBM read rate)."""
    exe = os.path.join(HERE, "calibrate")
    _run([_hipcc(), "--offload-arch=gfx950", "-O2", "-Xclang", "-target-feature", "-Xclang",
          "-packed-fp32-ops", "-o", exe, os.path.join(CSRC, "calibrate.hip")])
    return exe


if __name__ == "__main__":
    import sys
    sys.path.insert(0, ROOT)
    print(build(verbose=True))
    print(build_calibrate())
