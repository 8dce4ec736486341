"""The host-side planner compiled with AddressSanitizer and UBSan (host code only, no HIP)
and driven through a sweep of boxes, lengths and tensor lists."""
import os
import shutil
import subprocess
import sys

import pytest

from conftest import ROOT

DRIVER = r'''
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "plan.h"

static void one(const std::vector<int>& dims, uint64_t count, ddl_dtype_t dtype,
                const std::vector<uint64_t>& off, const std::vector<uint64_t>& cnt) {
    int P = 1;
    for (int d : dims) P *= d;
    if (ddl::validate_dims(dims.data(), (int)dims.size(), P) != DDL_OK) std::abort();
    ddl_plan plan;
    plan.dims = dims;
    plan.P = P;
    plan.count = count;
    plan.dtype = dtype;
    plan.elem_size = ddl::dtype_size(dtype);
    plan.seg_off = off;
    plan.seg_count = cnt;
    ddl::build_schedule(&plan);
    size_t steps = 0;
    for (int d : dims) steps += 2 * (d - 1);
    if (plan.steps.size() != steps) std::abort();
    if (plan.ops.size() != steps * off.size() * (size_t)P) std::abort();
    for (const ddl::Op& op : plan.ops)
        if (op.off + op.n > count || op.src < 0 || op.src >= P || op.dst < 0 || op.dst >= P) std::abort();
    // work lists: whole items are interior rows of their operation, every row of the shifted
    // tiling is covered exactly once
    const uint64_t G = 16 / (uint64_t)plan.elem_size;
    if (off.size() > 1) {
        std::vector<uint64_t> covered(plan.ops.size(), 0);
        for (const ddl::BlockDesc& d : plan.whole) {
            if (d.op >= plan.ops.size()) std::abort();
            const uint64_t nv = plan.ops[d.op].n / G;
            if (d.row < 1 || (uint64_t(d.row) + ddl::kListRows) * 64 > nv) std::abort();
            covered[d.op] += ddl::kListRows;
        }
        for (const ddl::BlockDesc& d : plan.ragged) {
            if (d.op >= plan.ops.size()) std::abort();
            const uint64_t rows = (plan.ops[d.op].n / G + 1 + 63 + 63) / 64;
            if (d.row >= rows) std::abort();
            covered[d.op] += rows - d.row < (uint64_t)ddl::kListTailRows ? rows - d.row : ddl::kListTailRows;
        }
        for (size_t i = 0; i < plan.ops.size(); ++i) {
            const uint64_t rows = plan.ops[i].n ? (plan.ops[i].n / G + 1 + 63 + 63) / 64 : 0;
            if (covered[i] != rows) std::abort();
        }
    } else if (!plan.whole.empty() || !plan.ragged.empty()) {
        std::abort();
    }
    // ring-walk rows: in bounds, d distinct members of one ring, same range as the phases
    ddl::build_walk(&plan);
    {
        size_t expect = 0;
        for (int d : dims) expect += d > 1;
        if (plan.walk_levels.size() != expect) std::abort();
        uint64_t bytes = 0;
        const size_t rows = off.size() * (size_t)P;
        for (const ddl::WalkLevel& lv : plan.walk_levels) {
            for (int half = 0; half < 2; ++half)
                for (size_t r = 0; r < rows; ++r) {
                    const uint64_t* row = plan.walk_plan.data() + (half ? lv.gather_plan : lv.reduce_plan) + r * (lv.d + 2);
                    if (row[0] + row[1] > count || row[1] > lv.max_n || row[2] != (uint64_t)(r % P)) std::abort();
                    for (int i = 0; i < lv.d; ++i) {
                        if (row[2 + i] >= (uint64_t)P) std::abort();
                        for (int j = 0; j < i; ++j)
                            if (row[2 + i] == row[2 + j]) std::abort();
                    }
                    const bool last = &lv == &plan.walk_levels.back();
                    bytes += row[1] * plan.elem_size * (last ? (half ? 0 : 2 * lv.d) : (half ? lv.d : 2 * lv.d - 1));
                }
            if (off.size() == 1 && (lv.reduce_count || lv.gather_count)) std::abort();
        }
        if (bytes != plan.walk_bytes || plan.walk_bytes > plan.bytes_total) std::abort();
        for (const ddl::BlockDesc& it : plan.walk_items)
            if (it.op >= rows) std::abort();
    }
    // the self-check accepts the plan and trips on planted mistakes
    if (ddl::verify_plan(plan) != DDL_OK) std::abort();
    if (!plan.ops.empty() && P > 1 && count >= 64 * (uint64_t)P) {
        size_t first = 0;
        while (plan.ops[first].n == 0) ++first;
        const ddl::Op keep = plan.ops[first];
        plan.ops[first].dst = keep.src;                          // a transfer to the wrong learner
        if (ddl::verify_plan(plan) == DDL_OK) std::abort();
        plan.ops[first] = keep;
        plan.ops[first].off += 1;                                // off the granule grid
        if (ddl::verify_plan(plan) == DDL_OK) std::abort();
        plan.ops[first] = keep;
        // a learner that receives the very range it sends in the first phase: a race
        const int nb = plan.ops[0].dst;
        const ddl::Op keep_nb = plan.ops[nb];
        plan.ops[nb].off = plan.ops[0].off;
        plan.ops[nb].n = plan.ops[0].n;
        if (plan.ops[0].n > 0 && ddl::verify_plan(plan) == DDL_OK) std::abort();
        plan.ops[nb] = keep_nb;
        plan.own_n[0] += G;                                      // chunks no longer tile the tensor
        if (ddl::verify_plan(plan) == DDL_OK) std::abort();
        plan.own_n[0] -= G;
        if (ddl::verify_plan(plan) != DDL_OK) std::abort();
    }
    int levels = 0;
    for (int d : dims) levels += d > 1;
    if (P <= 64 && levels >= 1) {
        std::vector<uint32_t> seq, ctl;
        int padded = 0;
        if (ddl::build_fused_order(plan, &seq, &ctl, &padded) != levels) std::abort();
        for (uint32_t r : seq)
            if (r >= (uint32_t)P) std::abort();
    }
}

int main() {
    const std::vector<std::vector<int>> boxes = {{1}, {2}, {5}, {4, 4}, {3, 1, 2}, {2, 2, 2, 2}, {4, 8, 8}, {7, 3}, {1, 1}};
    const uint64_t counts[] = {0, 1, 4, 5, 37, 1000, 65537, 25557032};
    const ddl_dtype_t types[] = {DDL_F32, DDL_F64, DDL_F16};
    for (const auto& dims : boxes)
        for (uint64_t c : counts)
            for (ddl_dtype_t t : types) {
                if (c > 100000 && dims.size() > 3) continue;
                one(dims, c, t, {0}, {c});
                if (c >= 64) one(dims, c, t, {0, 16, 48}, {9, 32, c - 48});
                if (c >= 600000) one(dims, c, t, {0, 300000}, {299999, c - 300000});
            }
    int dims3[3];
    double bw[3] = {2e10, 1e10, 9.5e9}, lat[3] = {1e-5, 1e-5, 1e-5}, time = 0;
    int caps[3] = {4, 16, 0};
    if (ddl::choose_dims(256, 3.5e8, 3, bw, lat, caps, dims3, &time) != DDL_OK) std::abort();
    std::puts("planner sweep ok");
    return 0;
}
'''


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_planner_under_asan_and_ubsan(tmp_path):
    csrc = os.path.join(ROOT, "paper_1708_02188_amd", "csrc")
    drv = tmp_path / "driver.cpp"
    drv.write_text(DRIVER)
    exe = tmp_path / "planner_asan"
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",
           "-I", csrc, str(drv), os.path.join(csrc, "plan.cpp"), "-o", str(exe), "-pthread"]
    subprocess.run(cmd, check=True)
    run = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    sys.stdout.write(run.stdout)
    sys.stderr.write(run.stderr[-2000:])
    assert run.returncode == 0 and "planner sweep ok" in run.stdout
