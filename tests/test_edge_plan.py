"""The rules that lay out the deterministic edge pass (tile size, LDS budgets, which kernel and launch shape, sorted or
unsorted records, record phases) are plain C++ in csrc/edge_plan.h: compiled here with the host compiler and checked on the
five benchmark configurations and at the limits, without a GPU."""
import json
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

DRIVER = r"""
#include <stdio.h>
#include <stdlib.h>
#include "edge_plan.h"
using namespace nomad;
// argv: n E s pool_size pool_block pool_line pool_distinct tune_edge_block tune_wg tune_pool_kernel tune_sort tune_flush tune_phases
int main(int argc, char** argv) {
    if (argc != 14) return 2;
    EdgePlanRequest q;
    q.n = atoll(argv[1]); q.E = atoll(argv[2]); q.s = atoi(argv[3]);
    q.pool_size = atoi(argv[4]); q.pool_block = atoi(argv[5]); q.pool_line = atoi(argv[6]); q.pool_distinct = atoi(argv[7]) != 0;
    q.tune_edge_block = atoi(argv[8]); q.tune_wg_per_cu = atoi(argv[9]); q.tune_pool_kernel = atoi(argv[10]);
    q.tune_record_sort = atoi(argv[11]); q.tune_flush_rounds = atoi(argv[12]);
    const EdgePlan p = plan_edge_pass(q);
    const int phases = p.bin_block ? plan_record_phases(q.E, q.s, p.bin_block, atoi(argv[13])) : 0;
    size_t lds = 0;
    if (p.pool_rounds && p.distinct_kernel) lds = distinct_lds_bytes(p.n_bins, q.pool_size, q.pool_size / q.pool_line, p.pool_rounds);
    else if (p.pool_rounds) lds = pooled_lds_bytes(p.n_bins, q.pool_block, q.pool_size);
    else if (p.bin_block) lds = binned_lds_bytes(p.n_bins, q.s, p.bin_block, p.sorted);
    printf("{\"tile_bits\": %d, \"n_bins\": %u, \"bin_block\": %d, \"wg_per_cu\": %d, \"sorted\": %d, \"flush_rounds\": %d, "
           "\"pool_rounds\": %d, \"distinct\": %d, \"phases\": %d, \"lds\": %zu, \"max_lds\": %zu, \"chunk\": %d}\n",
           p.tile_bits, p.n_bins, p.bin_block, p.wg_per_cu, (int)p.sorted, p.flush_rounds, p.pool_rounds, (int)p.distinct_kernel,
           phases, lds, kMaxLdsBytes, kChunk);
    return 0;
}
"""


@pytest.fixture(scope="module")
def planner(tmp_path_factory):
    d = tmp_path_factory.mktemp("edge_plan")
    src, exe = d / "plan.cpp", d / "plan"
    src.write_text(DRIVER)
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-Werror", "-I", os.path.join(ROOT, "paper_2505_15511_amd", "csrc"),
                    str(src), "-o", str(exe)], check=True, capture_output=True, text=True)

    def plan(n, E, s, pool=(0, 0, 1, 0), edge_block=0, wg=0, pool_kernel=1, sort=0, flush=0, phases=0):
        out = subprocess.run([str(exe)] + [str(int(v)) for v in (n, E, s, *pool, edge_block, wg, pool_kernel, sort, flush, phases)],
                             check=True, capture_output=True, text=True).stdout
        return json.loads(out)
    return plan


CONFIGS = {1: (2_000, 46_734, 5), 2: (100_000, 2_606_656, 5), 3: (1_000_000, 29_778_474, 5), 4: (10_000_000, 299_112_914, 5),
           5: (60_000_000, 1_198_388_818, 2)}


def test_benchmark_configurations(planner):
    for cfg, (n, E, s) in CONFIGS.items():
        p = planner(n, E, s)
        assert p["bin_block"] == 1024 and p["wg_per_cu"] == 1 and p["pool_rounds"] == 0, cfg
        assert p["lds"] <= p["max_lds"], cfg
        assert (p["n_bins"] - 1) << p["tile_bits"] < n <= p["n_bins"] << p["tile_bits"], cfg
    # about a thousand tiles while a tile may grow, 8,192 points a tile beyond 8 M points
    assert planner(*CONFIGS[3])["n_bins"] == 977 and planner(*CONFIGS[3])["tile_bits"] == 10
    assert planner(*CONFIGS[4])["n_bins"] == 1221 and planner(*CONFIGS[4])["tile_bits"] == 13
    assert planner(*CONFIGS[5])["n_bins"] == 7325 and planner(*CONFIGS[5])["tile_bits"] == 13
    # configurations 1-4 sort a round's records (more records than tiles); configuration 5 does not, two rounds per flush
    for cfg in (1, 2, 3, 4):
        p = planner(*CONFIGS[cfg])
        assert p["sorted"] == 1 and p["flush_rounds"] == 1, cfg
    p5 = planner(*CONFIGS[5])
    assert p5["sorted"] == 0 and p5["flush_rounds"] == 2
    # record phases: one below 8 GB of records per step, 4 at configuration 4 (21.5 GB), 16 at configuration 5 (43 GB: the 4 GB rule)
    assert [planner(*CONFIGS[c])["phases"] for c in (1, 2, 3, 4, 5)] == [1, 1, 1, 4, 16]
    for cfg, (n, E, s) in CONFIGS.items():
        per_phase = E * (s + 1) * 12 / planner(n, E, s)["phases"]
        assert per_phase <= (4e9 if E * (s + 1) * 12 > 32e9 else 8e9)


def test_knobs_and_limits(planner):
    n, E, s = CONFIGS[4]
    assert planner(n, E, s, sort=2)["sorted"] == 0 and planner(n, E, s, sort=2, flush=1)["flush_rounds"] == 1
    assert planner(*CONFIGS[5], sort=1)["sorted"] == 1 and planner(*CONFIGS[5], sort=1)["lds"] <= planner(*CONFIGS[5])["max_lds"]
    assert planner(n, E, s, phases=7)["phases"] == 7
    assert planner(2_000, 500, 5, phases=64)["phases"] == 1            # never more phases than blocks of positions
    p512 = planner(*CONFIGS[3], edge_block=512)
    assert p512["bin_block"] == 512 and p512["wg_per_cu"] == 2 and 2 * (p512["lds"] + 256) <= 160 * 1024
    assert planner(*CONFIGS[4], edge_block=512)["bin_block"] == 512
    assert planner(*CONFIGS[5], edge_block=512)["bin_block"] == 1024    # two workgroups' tables do not fit there
    assert planner(n, E, s, wg=3)["wg_per_cu"] == 3
    # the sorted form gives every thread at most eight tiles and needs the round's records in LDS: beyond that, nothing fits
    big = planner(2 ** 31 - 300, 10 ** 9, 5, sort=1)
    assert big["bin_block"] == 0 and big["phases"] == 0
    # the unsorted form is bounded by the per-tile tables alone: 16 B per tile
    assert planner(80_000_000, 10 ** 9, 5, sort=2)["bin_block"] == 1024
    assert planner(90_000_000, 10 ** 9, 5, sort=2)["bin_block"] == 0


def test_pooled_kernels_are_chosen_when_their_tables_fit(planner):
    n, E, s = CONFIGS[4]
    p = planner(n, E, s, pool=(2048, 8192, 16, 1))
    assert p["pool_rounds"] == 8 and p["distinct"] == 1 and p["bin_block"] == 1024 and p["lds"] <= p["max_lds"]
    p = planner(n, E, s, pool=(4096, 8192, 1, 1))                     # 4,096 lines of one point
    assert p["pool_rounds"] == 8 and p["distinct"] == 1 and p["lds"] <= p["max_lds"]
    p = planner(n, E, s, pool=(1024, 4096, 1, 0))
    assert p["pool_rounds"] == 4 and p["distinct"] == 0
    assert planner(n, E, s, pool=(48, 100, 1, 0))["pool_rounds"] == 0          # a block that is no multiple of 1,024 positions
    assert planner(n, E, s, pool=(2048, 3072, 16, 1))["pool_rounds"] == 0      # three rounds: no such kernel
    assert planner(n, E, s, pool=(2048, 8192, 16, 1), pool_kernel=0)["pool_rounds"] == 0
    # the kernel with distinct picks addresses col / head and the rows with 32-bit byte offsets
    assert planner(*CONFIGS[5], pool=(2048, 8192, 16, 1))["distinct"] == 0
    assert planner(2 ** 29, 10 ** 8, 5, pool=(2048, 8192, 16, 1))["pool_rounds"] == 0
