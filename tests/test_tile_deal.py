"""The chunked deal of M tiles to the XCDs (FcDeal in csrc/geom.h), checked on the CPU.

The persistent streaming kernels walk `t = first(part, slot); t < MT; t += stride`.  A small C++
driver includes the same header the kernels use and enumerates that walk for many tile counts,
slot counts and row lengths: every tile must be visited exactly once, chunks must go to the XCDs
in turn, and the tiles an XCD holds at any step must lie inside one window of `stride` tiles (the
compact write front the deal exists for).
"""
import os
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2601_11608_amd", "csrc")

DRIVER = r"""
#include <cstdio>
#include <vector>
#include "geom.h"
int main() {
    long cases = 0;
    const unsigned mts[] = {1, 2, 7, 8, 9, 31, 64, 250, 511, 512, 513, 784, 1000, 3136, 6272, 6273, 50001};
    const unsigned slots[] = {1, 2, 3, 5, 8, 16, 32, 51, 85, 256};
    const int wfs[] = {1, 7, 14, 28, 224, 500, 4000};
    for (unsigned MT : mts) for (unsigned sl : slots) for (int wf : wfs) for (int KH = 1; KH <= 3; KH += 2)
    for (unsigned parts = 1; parts <= 8; parts += 7) {
        const FcDeal d = fc_make_deal(MT, parts, sl, KH, wf);
        if (d.parts != parts || d.J < 1 || d.CH < 1 || d.J % d.CH != 0 || d.stride != d.J * parts || d.J > sl) return 2;
        if (parts == 1 && d.CH != 1) return 3;
        std::vector<int> seen(MT, 0);
        for (unsigned part = 0; part < parts; ++part)
            for (unsigned j0 = 0; j0 < d.J; ++j0) {
                const unsigned first = fc_deal_first_tile(d, part, j0);
                if (first >= d.stride) return 4;                       // step 0 lies inside the first window
                if ((first / d.CH) % parts != part) return 5;          // chunk c belongs to XCD c % parts
                for (unsigned long long t = first; t < MT; t += d.stride) {
                    if (seen[t]++) return 6;
                }
            }
        for (unsigned t = 0; t < MT; ++t)
            if (seen[t] != 1) return 7;
        ++cases;
    }
    // the headline layer: 6272 tiles, 16 tiles in flight per XCD, 14 folded pixels per row -> chunks of 2
    const FcDeal h = fc_make_deal(6272, 8, 16, 3, 14);
    if (h.CH != 2 || h.J != 16 || h.stride != 128) return 8;
    // long rows (the zero-padded reference: 224 pixels = 7 tiles per row) take longer chunks
    const FcDeal p = fc_make_deal(100352, 8, 256, 3, 224);
    if (p.CH != 32 || p.J != 256) return 9;
    // a slot count that is not a multiple of the chunk is rounded down
    const FcDeal q = fc_make_deal(3136, 8, 85, 3, 28);
    if (q.CH != 4 || q.J != 84) return 10;
    printf("%ld\n", cases);
    return 0;
}
"""


def test_every_tile_is_dealt_exactly_once():
    cxx = shutil.which("g++")
    if cxx is None:
        pytest.skip("no host compiler")
    with tempfile.TemporaryDirectory() as tmp:
        src = os.path.join(tmp, "deal.cpp")
        exe = os.path.join(tmp, "deal")
        with open(src, "w") as f:
            f.write(DRIVER)
        subprocess.check_call([cxx, "-std=c++17", "-O1", "-Wall", "-Werror", "-I", CSRC, src, "-o", exe])
        out = subprocess.run([exe], capture_output=True, text=True)
        assert out.returncode == 0, "tile deal check failed with status %d" % out.returncode
        assert int(out.stdout) > 1000
