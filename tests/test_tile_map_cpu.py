"""The work-item -> tile map of the product kernels, compiled for the host: every grid size must give
each tile exactly once (a tile visited twice or an index outside the grid would be a wrong result or
an out-of-bounds access on the GPU, so this is checked here, without one)."""
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "paper_2503_06564_amd", "csrc", "gemm_common.h")

MAIN = r"""
int main()
{
    for (int tiles_m = 1; tiles_m <= 300; ++tiles_m)
        for (int tiles_n = 1; tiles_n <= 80; ++tiles_n) {
            std::vector<char> seen(tiles_m * tiles_n, 0);
            for (int id = 0; id < tiles_m * tiles_n; ++id) {
                int tm = -1, tn = -1;
                trdq::gemm::tile_map(id, tiles_m, tiles_n, tm, tn);
                if (tm < 0 || tm >= tiles_m || tn < 0 || tn >= tiles_n || seen[tm * tiles_n + tn]) {
                    std::printf("grid %d x %d: item %d -> (%d, %d)\n", tiles_m, tiles_n, id, tm, tn);
                    return 1;
                }
                seen[tm * tiles_n + tn] = 1;
            }
        }
    std::printf("ok\n");
    return 0;
}
"""


def test_tile_map_is_a_bijection_for_every_grid(tmp_path):
    text = open(HEADER).read()
    start = text.index("// Workgroups are handed to the 8 accelerator dies")
    end = text.index("// ---- pieces shared by the direct-to-LDS kernels")
    src = tmp_path / "tile_map.cpp"
    src.write_text("#include <cstdio>\n#include <vector>\n#define __device__\n#define __forceinline__ inline\n"
                   "namespace trdq { namespace gemm {\n" + text[start:end] + "} }\n" + MAIN)
    exe = tmp_path / "tile_map"
    subprocess.run(["g++", "-O2", "-std=c++17", "-o", str(exe), str(src)], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and r.stdout.strip() == "ok", r.stdout[-500:]
