"""include/hbp.h is plain C: a C99 translation unit that includes it compiles without warnings under
-Wall -Wextra -pedantic, links against libhbp.so and calls the host-only entry points."""
import os
import subprocess
import tempfile

import paper_2503_07680_amd as H

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

PROGRAM = r"""
#include <stdio.h>
#include "hbp.h"

int main(void) {
  int32_t lengths[5] = {512, 256, 128, 64, 64};
  int32_t cu[6], n_samples = 0, n_consumed = 0, n_tiles = 0;
  hbp_tile tiles[16];
  int64_t cost[16], pack_cost = 0;
  hbp_status st = hbp_pack_plan(lengths, 5, 1024, 128, HBP_TILES_QUERY, cu, 6, &n_samples, &n_consumed,
                                tiles, cost, 16, &n_tiles, &pack_cost);
  int32_t rows = 0;
  if (st != HBP_OK || hbp_tile_rows(128, 128, HBP_BWD, &rows) != HBP_OK) return 1;
  printf("%s %d %d %d %lld %d %d %lu\n", hbp_status_string(st), (int)n_samples, (int)n_tiles, (int)cu[5],
         (long long)pack_cost, (int)tiles[0].row_begin, (int)rows, (unsigned long)HBP_STATIC_SCRATCH_BYTES);
  return hbp_pack_plan(lengths, 5, 0, 128, HBP_TILES_QUERY, cu, 6, &n_samples, &n_consumed, tiles, cost, 16,
                       &n_tiles, &pack_cost) == HBP_ERR_INVALID_ARG ? 0 : 2;
}
"""


def test_header_is_plain_c_and_the_library_links_from_c():
    H.load_library()
    lib_dir = os.path.dirname(H.library_path())
    with tempfile.TemporaryDirectory() as tmp:
        src, exe = os.path.join(tmp, "use_hbp.c"), os.path.join(tmp, "use_hbp")
        open(src, "w").write(PROGRAM)
        cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"), src,
               "-o", exe, "-L", lib_dir, "-l:libhbp.so", "-Wl,-rpath," + lib_dir]
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert r.returncode == 0, r.stdout
        r = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
        assert r.returncode == 0, r.stdout
        assert r.stdout.split() == ["ok", "5", "9", "1024", "352256", "384", "128", str((64 << 20) + 4096)], r.stdout
