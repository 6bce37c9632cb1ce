"""The boundary header is plain C: a C99 translation unit that includes it, fills the shape
struct and takes the address of every declared function compiles with -pedantic.  Linking
that unit against the built library resolves every symbol (no C++ name mangling leaked)."""
import os
import re
import subprocess
import tempfile

from paper_2509_19729_amd import binding as ab

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = {"amoeba.h": ab.EXPORTS, "amoeba_measure.h": ab.MEASURE_EXPORTS}


def declared_functions(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(amoeba_[a-z_0-9]+)\s*\(", text)))


def test_header_compiles_as_c99_and_links_against_the_library():
    names = []
    for header, exports in HEADERS.items():
        found = declared_functions(header)
        assert set(found) == set(exports), header
        names += found
    body = "\n".join(f"  sink((void*)&{n});" for n in names)
    src = f"""#include "amoeba.h"
#include "amoeba_measure.h"
static void sink(void* p) {{ (void)p; }}
int main(void) {{
  amoeba_model_shape s = {{0}};
  s.n_layers = 1; s.elem_bytes = 2; s.n_experts = 0; s.pad_page_bytes = 0; s.kv_blocks_bound = 0;
  (void)s;
{body}
  return AMOEBA_OK + AMOEBA_KV_HEAD_MAJOR + AMOEBA_W_DENSE + AMOEBA_T_Q + AMOEBA_PART_ALL +
         AMOEBA_TUNE_W_GRID;
}}
"""
    with tempfile.TemporaryDirectory() as tmp:
        c = os.path.join(tmp, "use_header.c")
        open(c, "w").write(src)
        # function-pointer-to-void* casts are not strictly ISO C, hence no -pedantic-errors
        subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-I",
                               os.path.join(ROOT, "include"), "-c", c, "-o",
                               os.path.join(tmp, "use_header.o")])
        if os.path.exists(ab.LIB_PATH):
            libdir = os.path.dirname(ab.LIB_PATH)
            subprocess.check_call(["gcc", os.path.join(tmp, "use_header.o"), "-L", libdir,
                                   "-lamoeba", "-Wl,--allow-shlib-undefined", "-o",
                                   os.path.join(tmp, "use_header")])
