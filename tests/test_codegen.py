"""Code-generation properties the step kernel's speed rests on, checked on the compiler's output.

On gfx950 vector loads and stores share one in-order counter (`vmcnt`).  The headline kernel reached the
rate of a bare stream only once (a) all six row loads of a wave were issued before anything waited for
one of them and (b) nothing after the barrier waited on that counter: a single vector load there (the
row offsets of W used to be one) makes the second row's gather wait for the first row's stores.  Both
are easy to lose to an innocent source change, and no functional test would notice.
"""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def decentlam_asm(tmp_path_factory):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not installed")
    from paper_2104_11981_amd import build

    out = tmp_path_factory.mktemp("asm") / "step_decentlam.s"
    flags = [f for f in build.FLAGS if f != "-fPIC"]
    subprocess.run([HIPCC] + flags + ["-S", "--cuda-device-only", os.path.join(build.CSRC, "step_decentlam.hip"),
                                      "-o", str(out)], check=True, capture_output=True)
    return out.read_text()


def instantiation(text, template_args, kernel="k_step"):
    """Instructions of one instantiation, found by its demangled name (`template_args` as a demangler prints
    them, e.g. "4, 2, 16, 0, 0, false, false"); without a demangler on the machine the Itanium encoding of the
    arguments is searched for instead."""
    import shutil

    labels = re.findall(r"^(_Z[\w$.]+):", text, re.M)
    tool = shutil.which("c++filt") or shutil.which("llvm-cxxfilt")
    if tool:
        plain = subprocess.run([tool], input="\n".join(labels), capture_output=True, text=True, check=True).stdout.split("\n")
    else:
        enc = "".join({"false": "Lb0E", "true": "Lb1E"}.get(a.strip(), f"Li{a.strip()}E") for a in template_args.split(","))
        plain = [f"{kernel}<{template_args}>(" if f"{kernel}I{enc}E" in lab else lab for lab in labels]
    want = f"{kernel}<{template_args}>("
    hits = [lab for lab, name in zip(labels, plain) if want in name]
    assert len(hits) == 1, f"{want}: {len(hits)} instantiations in the assembly"
    start = text.index("\n" + hits[0] + ":") + 1
    body = text[text.index("\n", start) + 1:text.index(".Lfunc_end", start)]
    return [ln.strip() for ln in body.split("\n") if ln.strip() and not ln.strip().startswith(";")]


@pytest.fixture(scope="module")
def headline_kernel_asm(decentlam_asm):
    # k_step<VEC = 4, RPT = 2, WAVES = 16, DecentLaM, fp32 gradients, no per-tensor sums, gathers>: the 32-node shape
    return instantiation(decentlam_asm, "4, 2, 16, 0, 0, false, false")


@pytest.fixture(scope="module")
def dense_kernel_asm(decentlam_asm):
    # the same with the mixing on the matrix cores
    return instantiation(decentlam_asm, "4, 2, 16, 0, 0, false, true")


def test_row_loads_are_issued_before_the_first_wait_on_them(headline_kernel_asm):
    wide = [k for k, ins in enumerate(headline_kernel_asm) if ins.startswith("global_load_dwordx4")]
    assert len(wide) >= 6, f"expected at least the six row loads (x, g, m of two rows), found {len(wide)}"
    waits = [k for k, ins in enumerate(headline_kernel_asm) if ins.startswith("s_waitcnt") and "vmcnt" in ins]
    assert waits, "no wait on the loads at all?"
    assert all(k < waits[0] for k in wide[:-1]), "a row load is issued only after a wait on an earlier one"
    # the last may sit just inside the block that first uses it, but still before any wait
    assert wide[-1] < waits[0] or not any(wide[-2] < w < wide[-1] for w in waits)


def test_nothing_after_the_barrier_waits_on_vector_memory(headline_kernel_asm):
    barrier = [k for k, ins in enumerate(headline_kernel_asm) if ins.startswith("s_barrier")]
    assert len(barrier) >= 1
    after = headline_kernel_asm[barrier[0]:]
    assert not [ins for ins in after if ins.startswith("s_waitcnt") and "vmcnt" in ins]
    assert not [ins for ins in after if ins.startswith(("global_load", "buffer_load", "flat_load"))]
    assert len([ins for ins in after if ins.startswith("global_store_dwordx4")]) >= 4   # m and x of two rows


def test_headline_kernel_fits_two_workgroups_per_cu(headline_kernel_asm):
    # 1024 threads per workgroup: two of them share a CU only up to 64 vector registers per lane
    text = "\n".join(headline_kernel_asm)
    m = re.search(r"\.amdhsa_next_free_vgpr\s+(\d+)", text)
    assert m and int(m.group(1)) <= 64
    assert not re.search(r"scratch_(load|store)", text)


def test_dense_kernel_multiplies_on_the_matrix_cores(dense_kernel_asm):
    """32 x 32 times 32 x 16 per wave in fp64: sixteen 16x16x4 products (the groups of four rows
    beyond n are skipped by uniform branches, so the blocks may sit anywhere in the text) and two
    barriers; nothing after the first barrier waits for a vector load; registers allow two workgroups
    per CU."""
    ins = dense_kernel_asm
    barrier = [k for k, i in enumerate(ins) if i.startswith("s_barrier")]
    assert len(barrier) >= 2
    mfma = [k for k, i in enumerate(ins) if i.startswith("v_mfma_f64_16x16x4")]
    assert len(mfma) >= 16 and barrier[0] < mfma[0]
    after = ins[barrier[0]:]
    assert not [i for i in after if i.startswith("s_waitcnt") and "vmcnt" in i]
    assert not [i for i in after if i.startswith(("global_load", "buffer_load", "flat_load"))]
    assert len([i for i in after if i.startswith("global_store_dwordx4")]) >= 4
    text = "\n".join(ins)
    m = re.search(r"\.amdhsa_next_free_vgpr\s+(\d+)", text)
    assert m and int(m.group(1)) <= 64
    assert not re.search(r"scratch_(load|store)", text)


def test_three_block_dense_kernel(decentlam_asm):
    """33-48 nodes: 48 x 48 times 48 x 16 per wave, thirty-six products; one workgroup per CU, so up to 128
    registers are fine, scratch is not."""
    ins = instantiation(decentlam_asm, "4, 3, 16, 0, 0, false, true")
    assert len([i for i in ins if i.startswith("v_mfma_f64_16x16x4")]) >= 36
    assert len([i for i in ins if i.startswith("s_barrier")]) >= 2
    text = "\n".join(ins)
    m = re.search(r"\.amdhsa_next_free_vgpr\s+(\d+)", text)
    assert m and int(m.group(1)) <= 128
    assert not re.search(r"scratch_(load|store)", text)


def test_chained_tile_kernel_fits_two_workgroups_per_cu(tmp_path):
    """k_step_chain keeps twelve values waiting across its loop on top of what k_step holds: it is built for
    exactly 64 registers per lane (two workgroups of 1024 threads per CU), and a spill would put memory traffic
    of its own into a kernel that is bound by memory."""
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not installed")
    from paper_2104_11981_amd import build

    out = tmp_path / "step_chain.s"
    flags = [f for f in build.FLAGS if f != "-fPIC"]
    subprocess.run([HIPCC] + flags + ["-S", "--cuda-device-only", os.path.join(build.CSRC, "step_chain.hip"), "-o", str(out)],
                   check=True, capture_output=True)
    text = out.read_text()
    for algo in (0, 1, 4):   # DecentLaM, DmSGD, AWC-DmSGD
        body = "\n".join(instantiation(text, str(algo), kernel="k_step_chain"))
        m = re.search(r"\.amdhsa_next_free_vgpr\s+(\d+)", body)
        assert m and int(m.group(1)) <= 64
        assert not re.search(r"scratch_(load|store)", body)
        assert len(re.findall(r"global_load_dwordx4", body)) >= 9     # three before the loop, six inside


def test_two_pass_kernels_keep_every_input_in_registers(tmp_path):
    """k_step_tall holds all twelve values per row of up to eight rows per thread (96 registers) across two LDS passes;
    a workgroup of 1024 threads has 128 registers per lane, and the shapes with three and four rows per thread are
    built for 64, so that two workgroups share a CU.  A spill would wait for a load the moment it is issued."""
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not installed")
    from paper_2104_11981_amd import build

    out = tmp_path / "step_tall.s"
    flags = [f for f in build.FLAGS if f != "-fPIC"]
    subprocess.run([HIPCC] + flags + ["-S", "--cuda-device-only", os.path.join(build.CSRC, "step_tall.hip"), "-o", str(out)],
                   check=True, capture_output=True)
    text = out.read_text()
    kernels = len(re.findall(r"^\s*\.amdhsa_kernel\s+\S*k_step_tall", text, re.M))
    assert kernels >= 42   # five methods x nine shapes, less AWC-DmSGD with four rows per thread
    assert not re.search(r"scratch_(load|store)", text)
    counts = [int(v) for v in re.findall(r"\.vgpr_count:\s+(\d+)", text)]
    spills = [int(v) for v in re.findall(r"\.vgpr_spill_count:\s+(\d+)", text)]
    assert len(counts) == kernels and max(counts) <= 128 and not any(spills)
    assert sum(c <= 64 for c in counts) >= 22   # the three- and four-row shapes


def test_gradient_sweep_kernels_do_not_spill(tmp_path):
    """k_fused keeps a row tile of A, its fp64 accumulators and (up to d = 16384) its chunks of x_i in registers; the
    widest form (d <= 32768, 1024 threads) fills all 128 registers of a lane and keeps x_i in LDS instead.  None of
    the forms may spill: a spilled tile register would wait for its load the moment it is issued."""
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not installed")
    from paper_2104_11981_amd import build

    out = tmp_path / "lsq_kernels.s"
    flags = [f for f in build.FLAGS if f != "-fPIC"]
    subprocess.run([HIPCC] + flags + ["-S", "--cuda-device-only", os.path.join(build.CSRC, "lsq_kernels.hip"), "-o", str(out)],
                   check=True, capture_output=True)
    text = out.read_text()
    assert len(re.findall(r"^\s*\.amdhsa_kernel\s+\S*k_fused", text, re.M)) >= 35
    assert len(re.findall(r"^\s*\.amdhsa_kernel\s+\S*k_fused_narrow", text, re.M)) >= 8    # rows off the 16-byte boundaries
    assert len(re.findall(r"^\s*\.amdhsa_kernel\s+\S*k_fused_rows", text, re.M)) >= 21     # short rows: a wave per row
    assert not re.search(r"scratch_(load|store)", text)
    assert not any(int(v) for v in re.findall(r"\.vgpr_spill_count:\s+(\d+)", text))


def test_wide_row_sweep_exchanges_without_fences_or_barriers(tmp_path):
    """k_fused_split (rows of more than 32768 columns): what crosses waves is one 8-byte word per wave and row, written
    and read with device-scope atomic accesses (`sc1` on this chip) -- and nothing else: no cache write-back or
    invalidate (a device-wide fence writes back a whole L2, of which the chip has eight), no workgroup barrier (the
    waves of a workgroup share nothing), no spill (248-252 registers in the wide shape, under 170 in the narrow one)."""
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not installed")
    from paper_2104_11981_amd import build

    out = tmp_path / "lsq_kernels.s"
    flags = [f for f in build.FLAGS if f != "-fPIC"]
    subprocess.run([HIPCC] + flags + ["-S", "--cuda-device-only", os.path.join(build.CSRC, "lsq_kernels.hip"), "-o", str(out)],
                   check=True, capture_output=True)
    text = out.read_text()
    for args, most_vgprs in (("8, 2, 1, 1, 1", 256), ("8, 2, 1, 1, 2", 256), ("4, 3, 2, 1, 1", 170)):
        body = instantiation(text, args, kernel="k_fused_split")
        assert [i for i in body if i.startswith("global_store_dwordx2") and " sc1" in i], args     # a share published
        assert [i for i in body if i.startswith("global_load_dwordx2") and " sc1" in i], args      # the shares collected
        assert not [i for i in body if i.startswith(("buffer_wbl2", "buffer_inv", "s_barrier", "scratch_"))], args
        assert len([i for i in body if i.startswith("global_load_dwordx4")]) >= int(args[0]), args   # the tile: 16-byte loads
        used = {int(v) for i in body for v in re.findall(r"\bv(\d+)\b", i)} | \
               {int(hi) for i in body for hi in re.findall(r"\bv\[\d+:(\d+)\]", i)}
        assert max(used) < most_vgprs, (args, max(used))


SPLIT_CHECK = r"""
#include <cstdio>
#include <vector>
#include "step_impl.hpp"
// Host run of the device function that maps (tile, lane) to columns in a split-tile launch: over
// `units` whole 64 KiB units every column must be owned exactly once, a tile must consist of two runs
// of 128 columns that lie 8192 columns apart inside one unit, and tile u + 1 must continue tile u.
int main() {
    using namespace dl::step;
    const int units = 5;
    std::vector<int> owner(static_cast<size_t>(units) * kSplitUnit, 0);
    for (unsigned tile = 0; tile < static_cast<unsigned>(units * kSplitTilesPerUnit); ++tile) {
        const long long first = split_column(tile, 0);
        if (first != split_column(tile, 0) || first / kSplitUnit != tile / kSplitTilesPerUnit) return 1;
        for (int lane = 0; lane < 64; ++lane) {
            const long long c = split_column(tile, lane);
            const long long expect = first + (lane >> 5) * kSplitDistance + (lane & 31) * 4;
            if (c != expect) return 2;
            if (c != split_column(tile, 0) + split_column(0, lane)) return 3;   // the kernel adds the two parts
            for (int v = 0; v < 4; ++v) {
                if (c + v < 0 || c + v >= static_cast<long long>(owner.size())) return 4;
                owner[c + v] += 1;
            }
        }
        if (tile % kSplitTilesPerUnit && split_column(tile, 0) != split_column(tile - 1, 0) + kSplitSegment) return 5;
    }
    for (int n : owner) if (n != 1) return 6;
    if (kSplitSegment * 4 != 512 || kSplitDistance * 4 != 32768 || kSplitUnit * 4 != 65536) return 7;
    std::puts("ok");
    return 0;
}
"""


def test_split_tile_column_map_owns_every_column_once(tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not installed")
    from paper_2104_11981_amd import build

    src = tmp_path / "split_check.hip"
    src.write_text(SPLIT_CHECK)
    exe = tmp_path / "split_check"
    subprocess.run([HIPCC, "--cuda-host-only", "-O1", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", build.CSRC,
                    str(src), "-o", str(exe)], check=True, capture_output=True)
    run = subprocess.run([str(exe)], capture_output=True, text=True)
    assert run.returncode == 0 and run.stdout.strip() == "ok", f"check {run.returncode} failed"


DENSE_CHECK = r"""
#include <cstdio>
#include <set>
#include "step_impl.hpp"
// Host run of the layout of W in LDS for the matrix-core mixing: every element has a slot of its own
// inside the array; a wave writing one row (lane = column) and a half-wave reading an A operand of the
// 16x16x4 instruction (lane l: row l % 16, column l / 16 of the 16 x 4 block) touch 32 different
// 8-byte banks; the kernel's way of composing an operand address from a per-lane and a per-block part
// gives the same slot.  And the switch-over rule: 46 - n entries per row up to 32 nodes (nothing below 23
// nodes), 38 - n / 4 entries per row from 33 to 48 nodes.
int check_layout(int rows) {   // the padded problem has `rows` rows and columns: 32 or 48
    using namespace dl::step;
    std::set<int> seen;
    for (int i = 0; i < rows; ++i)
        for (int k = 0; k < rows; ++k) {
            const int at = dense_w_at(i, k, rows);
            if (at < 0 || at >= dense_w_doubles(rows) || !seen.insert(at).second) return 1;
        }
    for (int i = 0; i < rows; ++i) {   // row write: lanes 0-31, then the rest
        for (int first = 0; first < rows; first += 32) {
            std::set<int> banks;
            const int last = first + 32 < rows ? first + 32 : rows;
            for (int k = first; k < last; ++k) banks.insert(dense_w_at(i, k, rows) % 32);
            if (static_cast<int>(banks.size()) != last - first) return 2;
        }
        for (int k = 0; k < rows; ++k)
            if (dense_w_at(i, k, rows) != dense_w_at(i, 0, rows) + dense_w_at(0, k, rows)) return 3;
    }
    for (int rb = 0; rb < rows / 16; ++rb)
        for (int s = 0; s < rows / 4; ++s)
            for (int half = 0; half < 2; ++half) {   // operand read, 32 lanes at a time
                std::set<int> banks;
                for (int lane = 32 * half; lane < 32 * half + 32; ++lane) {
                    const int at = dense_w_at(16 * rb + (lane & 15), 4 * s + (lane >> 4), rows);
                    if (at != dense_w_at(lane & 15, lane >> 4, rows) + dense_w_at(16 * rb, 4 * s, rows)) return 4;
                    banks.insert(at % 32);
                }
                if (banks.size() != 32) return 5;
            }
    return 0;
}
int main() {
    using namespace dl::step;
    if (int rc = check_layout(kDenseRows)) return rc;
    if (int rc = check_layout(kDenseRowsMax)) return 10 + rc;
    for (int n = 1; n <= 60; ++n)
        for (int per_row = 1; per_row <= n; ++per_row) {
            const bool want = (n >= 23 && n <= 32 && per_row >= 46 - n) || (n >= 33 && n <= 48 && 4 * per_row >= 152 - n);
            if (mixes_on_matrix_cores(n, per_row * n) != want) return 6;
        }
    std::puts("ok");
    return 0;
}
"""


def test_dense_weight_layout_is_conflict_free_and_rule_is_as_documented(tmp_path):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not installed")
    from paper_2104_11981_amd import build

    src = tmp_path / "dense_check.hip"
    src.write_text(DENSE_CHECK)
    exe = tmp_path / "dense_check"
    subprocess.run([HIPCC, "--cuda-host-only", "-O1", "-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", build.CSRC,
                    str(src), "-o", str(exe)], check=True, capture_output=True)
    run = subprocess.run([str(exe)], capture_output=True, text=True)
    assert run.returncode == 0 and run.stdout.strip() == "ok", f"check {run.returncode} failed"

