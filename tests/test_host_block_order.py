"""CPU-only check of the host logic that orders the work-groups of small causal grids
(csrc/block_order.hpp): compiled with g++ into a tiny program that prints the table."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER_DIR = os.path.join(ROOT, "paper_2510_04212_amd", "csrc")

MAIN = r"""
#include "block_order.hpp"
#include <cstdio>
#include <cstdlib>
int main(int argc, char** argv) {
  BlockOrder ord;
  const bool ok = fill_block_order(ord, atoi(argv[1]), atoi(argv[2]), atoi(argv[3]));
  printf("%d %d\n", ok ? 1 : 0, (int)ord.n);
  for (int i = 0; i < ord.n; ++i) printf("%d\n", (int)ord.pos[i]);
  return 0;
}
"""


@pytest.fixture(scope="module")
def table(tmp_path_factory):
    d = tmp_path_factory.mktemp("block_order")
    src = d / "main.cpp"
    src.write_text(MAIN)
    exe = d / "main"
    subprocess.run(["g++", "-std=c++17", "-O1", "-I", HEADER_DIR, str(src), "-o", str(exe)], check=True)

    def run(per, nblk, resident):
        out = subprocess.run([str(exe), str(per), str(nblk), str(resident)], check=True,
                             capture_output=True, text=True).stdout.split()
        ok, n = int(out[0]), int(out[1])
        return ok, [int(v) for v in out[2:2 + n]]
    return run


def _weight(j, nblk):
    return 2 * (nblk - j % nblk) + 1


def _unit_loads(pos, nblk, placed):
    loads = [0] * 32
    for s in range(placed):
        loads[s % 32] += _weight(pos[s], nblk)
    return loads


@pytest.mark.parametrize("per,nblk,resident", [(96, 8, 3), (96, 8, 4), (96, 8, 2), (48, 8, 4), (64, 4, 2),
                                               (255, 5, 2), (32, 32, 1), (8, 8, 2)])
def test_table_is_a_permutation_and_balances_the_units(table, per, nblk, resident):
    ok, pos = table(per, nblk, resident)
    assert ok == 1 and sorted(pos) == list(range(per))          # every work item exactly once
    placed = min(per, 32 * resident)
    loads = _unit_loads(pos, nblk, placed)
    used = [l for l in loads if l > 0]
    # what is placed at launch is the heaviest part of the grid ...
    w = sorted((_weight(j, nblk) for j in range(per)), reverse=True)
    assert sorted((_weight(j, nblk) for j in pos[:placed]), reverse=True) == w[:placed]
    # ... spread so that no unit carries more than one heaviest block above the lightest unit
    if placed >= 32:
        assert max(used) - min(used) <= _weight(0, nblk)
    # the rest follows heaviest first
    rest = [_weight(j, nblk) for j in pos[placed:]]
    assert rest == sorted(rest, reverse=True)


def test_three_resident_groups_of_eight_blocks_balance_to_within_one_block(table):
    """The case of 12 heads x 8 blocks per XCD with three work-groups per unit: the fixed
    heavy-to-light order stacks equal weight classes (spread 51 vs 9); the table evens them out."""
    _, pos = table(96, 8, 3)
    loads = _unit_loads(pos, 8, 96)
    naive = _unit_loads(list(range(96)), 8, 96)
    assert max(naive) - min(naive) == 3 * (17 - 3)
    assert max(loads) - min(loads) <= 4
    assert sum(loads) == sum(naive)


@pytest.mark.parametrize("per,nblk,resident", [(256, 8, 2), (100, 8, 2), (0, 8, 2), (96, 8, 0)])
def test_table_declines_what_it_cannot_express(table, per, nblk, resident):
    ok, pos = table(per, nblk, resident)
    assert ok == 0 and pos == []
