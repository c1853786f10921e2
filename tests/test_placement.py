"""Host-side check of the work-item placement (XCD-aware blockIdx -> (group, item) mapping).

The prefill kernels find their work item with `place_item` (csrc/common.h) and the launchers size the grid with
`placed_workgroups`.  A mapping that skips or repeats an item would only show on the GPU as a wrong or missing
output somewhere in a large launch, so the arithmetic is compiled for the host here (the function bodies are taken
from the header as they stand, with the device qualifiers defined away) and checked exhaustively on small launches:
every (group, item) is produced exactly once, nothing else is produced, and with a map of gc groups at a time a
workgroup on XCD x (= blockIdx % 8) only ever works on groups congruent to x mod gc.
"""
import re
import subprocess
from pathlib import Path

ROOT = Path(__file__).resolve().parents[1]
HEADER = ROOT / "paper_2406_09827_amd" / "csrc" / "common.h"

MAIN = r"""
#include <cstdio>
#include <vector>
using namespace hipattn;
int main()
{
    long cases = 0;
    const int maps[] = {0, 1, 2, 4, 8};
    for (int xcd_map : maps)
        for (int upw : {1, 4})
            for (uint32_t per_group = upw; per_group <= 200; per_group += upw)   // the launchers require per_group % upw == 0 with a map
                for (uint32_t groups : {8u, 16u, 24u, 40u}) {
                    if (xcd_map && per_group > 64 && per_group % 12) continue;   // thin out the large ones
                    const int64_t wgs = placed_workgroups(xcd_map, upw, per_group, groups);
                    std::vector<int> seen((size_t)groups * per_group, 0);
                    for (int64_t bid = 0; bid < wgs; ++bid)
                        for (int unit = 0; unit < upw; ++unit) {
                            uint32_t group = ~0u, o = ~0u;
                            if (!place_item(xcd_map, (uint32_t)bid, upw, unit, per_group, groups, group, o)) continue;
                            if (group >= groups || o >= per_group) {
                                std::printf("out of range: map %d upw %d per_group %u groups %u bid %lld unit %d -> (%u, %u)\n",
                                            xcd_map, upw, per_group, groups, (long long)bid, unit, group, o);
                                return 1;
                            }
                            if (xcd_map && group % (uint32_t)xcd_map != (uint32_t)(bid & 7) % (uint32_t)xcd_map) {
                                std::printf("wrong XCD: map %d bid %lld -> group %u\n", xcd_map, (long long)bid, group);
                                return 1;
                            }
                            ++seen[(size_t)group * per_group + o];
                        }
                    for (size_t i = 0; i < seen.size(); ++i)
                        if (seen[i] != 1) {
                            std::printf("item (%zu, %zu) produced %d times: map %d upw %d per_group %u groups %u\n",
                                        i / per_group, i % per_group, seen[i], xcd_map, upw, per_group, groups);
                            return 1;
                        }
                    ++cases;
                }
    // how many groups at a time: the largest power of two up to 8 whose rows stay within the budget
    const int64_t mb = 1 << 20;
    if (groups_at_a_time(8 * mb, 160 * mb) != 8 || groups_at_a_time(32 * mb, 160 * mb) != 4 || groups_at_a_time(64 * mb, 160 * mb) != 2 ||
        groups_at_a_time(256 * mb, 160 * mb) != 1 || groups_at_a_time(128 * mb, 768 * mb) != 4 || groups_at_a_time(512 * mb, 768 * mb) != 1 ||
        groups_at_a_time(96 * mb, 768 * mb) != 8) {
        std::printf("groups_at_a_time\n");
        return 1;
    }
    std::printf("ok %ld\n", cases);
    return 0;
}
"""


def placement_source() -> str:
    text = HEADER.read_text()
    m = re.search(r"(__device__ __forceinline__ bool place_item\(.*?)\ntemplate <int CTRL>", text, flags=re.S)
    assert m, "place_item / placed_workgroups / groups_at_a_time not found where expected in common.h"
    body = m.group(1)
    assert "placed_workgroups" in body and "groups_at_a_time" in body
    return ("#include <cstdint>\n#define __device__\n#define __forceinline__ inline\nnamespace hipattn {\n" + body +
            "\n}\n" + MAIN)


def test_every_work_item_is_placed_exactly_once(tmp_path):
    src = tmp_path / "place_check.cpp"
    src.write_text(placement_source())
    exe = tmp_path / "place_check"
    subprocess.run(["g++", "-O1", "-std=c++17", "-Wall", "-Werror", "-o", str(exe), str(src)], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.startswith("ok ") and int(r.stdout.split()[1]) > 500
