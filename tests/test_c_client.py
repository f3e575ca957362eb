"""The boundary is plain C: include/lsp.h compiles as strict C99 and as C++, and a client written
in C that sees nothing but that header links against liblsp.so and gets the documented error codes
(host-side validation only: no GPU is touched)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INC = os.path.join(ROOT, "include")

CLIENT = r"""
#include <stdio.h>
#include <string.h>
#include "lsp.h"

int main(void) {
  lsp_attn_desc ad;
  lsp_commit_desc cd;
  int rc;
  if (strstr(lsp_version(), "gfx950") == NULL) return 10;
  memset(&ad, 0, sizeof ad);
  memset(&cd, 0, sizeof cd);
  /* null operands: refused on the host, nothing launched */
  rc = lsp_confidence(LSP_BF16, NULL, 1, 1, 8, 0, 0, NULL, NULL, NULL, NULL, NULL, 0, NULL);
  if (rc != LSP_ERR_INVALID_ARG || strlen(lsp_last_error()) == 0) return 11;
  rc = lsp_attn_step(&ad, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL);
  if (rc != LSP_ERR_INVALID_ARG) return 12;
  rc = lsp_commit(&cd, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, NULL, 0, NULL);
  if (rc != LSP_ERR_INVALID_ARG) return 13;
  rc = lsp_confidence_static(LSP_BF16, NULL, 1, 1, 8, 0, 0, NULL, NULL, NULL, NULL, NULL);
  if (rc != LSP_ERR_INVALID_ARG) return 14;
  if (lsp_confidence_static_scratch_bytes() != 65536) return 15;
  if (lsp_confidence_workspace_bytes(1, 4, 126464) == 0) return 16; /* four long rows are split over workgroups */
  printf("%s\n", lsp_version());
  return 0;
}
"""


def test_header_is_strict_c99_and_cxx(tmp_path):
    for lang, std in (("c", "-std=c99"), ("c++", "-std=c++11")):
        src = tmp_path / ("t.c" if lang == "c" else "t.cpp")
        src.write_text('#include "lsp.h"\nint main(void) { return sizeof(lsp_attn_desc) > 0 ? 0 : 1; }\n')
        r = subprocess.run(["gcc" if lang == "c" else "g++", std, "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only",
                            "-I", INC, str(src)], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr


def test_a_client_written_in_c_links_and_gets_the_documented_errors(tmp_path):
    import paper_2603_05454_amd as lsp
    if not os.path.exists(lsp.LIB_PATH):
        from paper_2603_05454_amd.build import build
        build()
    libdir = os.path.dirname(lsp.LIB_PATH)
    src = tmp_path / "client.c"
    exe = tmp_path / "client"
    src.write_text(CLIENT)
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", INC, str(src), "-o", str(exe),
                        "-L", libdir, "-l:liblsp.so", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib"],
                       capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert "gfx950" in r.stdout
