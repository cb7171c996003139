"""Static checks of the gfx950 code objects that the kernel sources compile to (cross-compiled here, no
GPU needed).  They guard assumptions that the hand-written parts of the kernels rely on and that a
compiler or flag change could silently break:

* no kernel spills registers or uses scratch memory;
* the register and LDS budgets behind the planned occupancy (workgroups per CU) hold;
* in the tile kernels every scalar memory load sits in the prologue, before the first LDS fragment
  read: their LDS waits are hand-placed counts, and a scalar load in flight (same counter, out-of-order
  return) would make a count pass early;
* no kernel calls a device-library function except the few listed (fp64 exp2/log2 on rare paths, the
  device clock of the stamp kernel): these sources switch a target feature off, LLVM then refuses to
  inline the library's functions, and blockIdx/threadIdx spelled the HIP way become real calls of
  hundreds of instructions at the top of every kernel (csrc/ids.hpp has the register reads);
* a scalar register written by a vector instruction (v_readfirstlane / v_readlane) is not used as the
  base of a vector-memory instruction before five wait states have passed -- the compiler inserts the
  wait states for its own instructions, but cannot for a load written as inline assembly;
* no instruction names a vector register that an LDS read or a vector-memory load still in flight is
  going to write before the s_waitcnt that covers it: around loads written as inline assembly the
  compiler may still place a register copy (it did once: a copy of an index entry ahead of the wait
  gave wrong rows in one parity case), and nothing in the hardware holds such an instruction back.
"""
import os
import re
import subprocess

import pytest

from paper_2602_14209_amd import build as mbuild

LLVM = "/opt/rocm/llvm/bin"
CSRC = mbuild.CSRC


def _code_object(tmp, name):
    co, elf = os.path.join(tmp, name + ".co"), os.path.join(tmp, name + ".elf")
    flags = [f for f in mbuild.FLAGS if f not in ("-shared", "-Wall", "-Wno-unused-function")]
    subprocess.run(["hipcc", "--genco", *flags, "-I", os.path.join(os.path.dirname(os.path.dirname(CSRC)), "include"),
                    os.path.join(CSRC, name + ".hip"), "-o", co], check=True, capture_output=True)
    subprocess.run([os.path.join(LLVM, "clang-offload-bundler"), "--unbundle", "--type=o", "--input=" + co,
                    "--targets=hipv4-amdgcn-amd-amdhsa--gfx950", "--output=" + elf], check=True, capture_output=True)
    notes = subprocess.run([os.path.join(LLVM, "llvm-readelf"), "--notes", elf], check=True, capture_output=True, text=True).stdout
    dis = subprocess.run([os.path.join(LLVM, "llvm-objdump"), "-d", elf], check=True, capture_output=True, text=True).stdout
    meta = {}
    for blk in notes.split("- .agpr_count:")[1:]:
        g = lambda key: int(re.search(r"\.%s:\s+(\d+)" % key, blk).group(1))
        sym = re.search(r"\.name:\s+(\S+)", blk).group(1)
        meta[sym] = {"agpr": int(blk.split()[0]), "vgpr": g("vgpr_count"), "lds": g("group_segment_fixed_size"),
                     "scratch": g("private_segment_fixed_size"), "vspill": g("vgpr_spill_count")}
    kernels, cur = {}, None
    for ln in dis.splitlines():
        m = re.match(r"^[0-9a-f]+ <(\S+)>:", ln)
        if m:
            cur = kernels.setdefault(m.group(1), [])
            continue
        if cur is not None and ln.strip():
            cur.append(ln.split("//")[0].strip())
    return meta, kernels


def _demangle(sym):
    return subprocess.run(["c++filt", sym], capture_output=True, text=True).stdout.strip().split("(")[0].replace("void ", "")


def _sgpr_hazards(ins):
    """vector-memory instructions whose scalar base was written by a vector instruction fewer than five
    wait states earlier"""
    bad = []
    for i, s in enumerate(ins):
        if not re.match(r"(global|buffer|flat|scratch)_", s):
            continue
        m = re.search(r"\bs\[(\d+):(\d+)\]", s)
        if not m:
            continue
        regs = set(range(int(m.group(1)), int(m.group(2)) + 1))
        states = 0
        for j in range(i - 1, max(i - 8, -1), -1):
            p = ins[j]
            w = re.match(r"v_read(firstlane|lane)_b32 s(\d+)", p)
            if w and int(w.group(2)) in regs and states < 5:
                bad.append((p, s, states))
            nop = re.match(r"s_nop (\d+)", p)
            states += int(nop.group(1)) + 1 if nop else 1
            if states >= 5:
                break
    return bad


def _vregs(tok):
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.fullmatch(r"v(\d+)", tok)
    return {int(m.group(1))} if m else set()


def _early_uses(ins):
    """Instructions that name a vector register which an LDS read or a vector-memory load still in flight
    will write, ahead of the s_waitcnt that covers that load.  The hardware does not interlock these: the
    instruction would see the old contents.  (The kernels issue such loads from inline assembly and place
    the waits by hand; what the compiler does around them -- a register copy, a hoisted use -- is not
    visible in the source.)  Linear scan: branches fall through, the in-flight lists are dropped at
    unconditional branches; returns are in order per counter, so a younger load of the same counter
    may reuse a destination."""
    lgkm, vm, bad = [], [], []               # operations in flight, oldest first: their destination VGPRs (may be none)
    for s in ins:
        op = s.split()[0]
        ops = [x.strip() for x in s.split(None, 1)[1].split(",")] if " " in s else []
        regs = [_vregs(o.split()[0]) if o else set() for o in ops]
        is_lgkm = op.startswith("ds_") or op.startswith("s_load") or op.startswith("s_buffer_load")
        is_vm = bool(re.match(r"(global|buffer|flat|scratch)_", op))
        dest = set()
        if op.startswith("ds_") and re.match(r"ds_(read|load|bpermute|permute|swizzle)|ds_.*_rtn", op):
            dest = regs[0]
        if is_vm and "load" in op and "lds" not in op:
            dest = regs[0]
        for queue, mine in ((lgkm, is_lgkm), (vm, is_vm)):
            for i, r in enumerate(regs):
                if mine and i == 0 and dest:      # a younger load into the same register: lands later, in order
                    continue
                if any(d & r for d in queue):
                    bad.append(s)
        if op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", s)
            if m:
                del lgkm[:len(lgkm) - int(m.group(1))]
            m = re.search(r"vmcnt\((\d+)\)", s)
            if m:
                del vm[:len(vm) - int(m.group(1))]
        elif is_lgkm:
            lgkm.append(dest)
        elif is_vm:
            vm.append(dest)
            if op.startswith("flat_"):
                lgkm.append(set())
        elif op in ("s_endpgm", "s_branch", "s_setpc_b64"):
            lgkm.clear()
            vm.clear()
    return bad


@pytest.fixture(scope="module")
def objects(tmp_path_factory):
    tmp = str(tmp_path_factory.mktemp("co"))
    return {n: _code_object(tmp, n) for n in ("attn_bf16", "sparse_bf16", "sparse_batch_bf16", "topk", "reduce", "quest", "attn_f32", "diag")}


def test_no_spills_no_scratch_and_budgets(objects):
    budgets = {                                   # demangled prefix -> (max VGPR+AGPR, max LDS bytes)
        "mage::attn_bf16_kernel<128, 0": (256, 136 * 1024),     # attention: 2 wavefronts per SIMD, one workgroup per CU
        "mage::attn_bf16_kernel<64, 0": (256, 80 * 1024),
        "mage::attn_bf16_kernel<128, 1": (128, 80 * 1024),      # row statistics: 4 per SIMD, two workgroups per CU
        "mage::attn_bf16_kernel<64, 1": (128, 80 * 1024),
        "mage::attn_bf16_kernel<256, 1": (256, 160 * 1024),
        "mage::colsum_bf16_kernel<128, 4>": (168, 53 * 1024 + 256),   # three workgroups per CU
        "mage::colsum_bf16_kernel<64, 4>": (168, 53 * 1024 + 256),
        "mage::colsum_bf16_kernel<128, 8>": (128, 80 * 1024),   # two workgroups per CU
        "mage::colsum_bf16_kernel<64, 8>": (128, 80 * 1024),
        "mage::colsum_bf16_kernel<256": (512, 160 * 1024),
        "mage::sparse_bf16_kernel": (256, 160 * 1024),
        "mage::sparse_batch_kernel": (128, 80 * 1024),          # batched sparse step: 4 per SIMD, two workgroups per CU
        "mage::compact_kernel": (128, 0),
        "mage::topk_kernel": (128, 160 * 1024),                 # 16 wavefronts = 4 per SIMD
        # small kernels and the fp32 vector path: 256 threads per workgroup, at least two workgroups per CU
        "mage::combine_kernel": (128, 8 * 1024),
        "mage::lse_kernel": (128, 1024),
        "mage::page_summary_kernel": (128, 1024),
        "mage::quest_query_kernel": (128, 1024),
        "mage::expand_pages_kernel": (128, 1024),
        "mage::overlap_kernel": (128, 1024),
        "mage::attn_f32_kernel": (256, 80 * 1024),              # two workgroups per CU by LDS
        "mage::colsum_f32_kernel": (256, 64 * 1024),
        "mage::diag_": (128, 8 * 1024),                         # measurement aids
    }
    seen = set()
    for meta, _ in objects.values():
        for sym, m in meta.items():
            name = _demangle(sym)
            assert m["scratch"] == 0 and m["vspill"] == 0, (name, m)
            keys = [k for k in budgets if name.startswith(k)]
            assert keys, f"no budget recorded for {name}"
            regs, lds = budgets[max(keys, key=len)]
            assert m["vgpr"] + m["agpr"] <= regs and m["lds"] <= lds, (name, m, regs, lds)
            seen.add(max(keys, key=len))
    assert seen == set(budgets)


def test_scalar_loads_stay_in_the_prologue_of_the_tile_kernels(objects):
    kernels = dict(objects["attn_bf16"][1])
    kernels.update(objects["sparse_batch_bf16"][1])
    checked = 0
    for sym, ins in kernels.items():
        if "attn_bf16_kernel" not in sym and "colsum_bf16_kernel" not in sym and "sparse_batch_kernel" not in sym:
            continue
        if "sparse_batch_kernel" in sym:
            # its prologue reads index entries from LDS with plain waits; the hand-counted waits start with
            # the first fragment read of the tile loop and end with the last MFMA
            first_lds = next(i for i, s in enumerate(ins) if s.startswith("ds_read_b128"))
            last = max(i for i, s in enumerate(ins) if s.startswith("v_mfma"))
        else:
            first_lds = next(i for i, s in enumerate(ins) if s.startswith("ds_read"))
            last = len(ins)
        late = [(i, s) for i, s in enumerate(ins) if re.match(r"s_(buffer_)?load|s_mem", s) and first_lds < i < last]
        assert not late, (_demangle(sym), late[:3])
        checked += 1
    assert checked == 15          # 7 attention/statistics + 6 column-sum + 2 batched instantiations


def test_no_device_library_calls_except_the_listed_ones(objects):
    allowed = {"mage::topk_kernel": 2,            # __ocml_exp2_f64 in the fp64 re-score of near-ties (rarely taken)
               "mage::lse_kernel": 1, "mage::combine_kernel": 1,      # __ocml_log2_f64, once per row at the very end
               "mage::diag_stamp_kernel": 1}      # the device clock
    for meta, kernels in objects.values():
        for sym, ins in kernels.items():
            name = _demangle(sym)
            calls = sum(1 for x in ins if x.startswith("s_swappc") or x.startswith("s_setpc"))
            if sym not in meta:                    # a function that is not a kernel: only the library functions named above
                assert any(n in sym for n in ("__ocml_exp2_f64", "__ocml_log2_f64", "__ockl_steadyctr_u64")), sym
                continue
            limit = max((v for k, v in allowed.items() if name.startswith(k)), default=0)
            assert calls <= limit, (name, calls)


def test_vector_written_scalar_bases_are_five_wait_states_old(objects):
    for _, kernels in objects.values():
        for sym, ins in kernels.items():
            bad = _sgpr_hazards(ins)
            assert not bad, (_demangle(sym), bad[:3])


def test_hazard_scan_notices_a_planted_hazard():
    ins = ["v_readfirstlane_b32 s8, v1", "v_mul_u32_u24_e32 v56, s18, v66", "v_readfirstlane_b32 s9, v58",
           "global_load_dwordx4 v[132:135], v56, s[8:9]"]
    assert _sgpr_hazards(ins)
    ok = ins[:3] + ["s_nop 4"] + ins[3:]
    assert not _sgpr_hazards(ok)


def test_no_register_is_named_before_the_wait_that_covers_its_load(objects):
    for _, kernels in objects.values():
        for sym, ins in kernels.items():
            bad = _early_uses(ins)
            assert not bad, (_demangle(sym), bad[:3])


def test_early_use_scan_notices_a_planted_copy():
    ins = ["ds_read_b32 v27, v23", "ds_read_b32 v26, v23", "v_mov_b32_e32 v18, v27", "s_waitcnt lgkmcnt(1)",
           "v_mad_u64_u32 v[18:19], s[4:5], v18, s22, v[70:71]"]
    assert _early_uses(ins) == ["v_mov_b32_e32 v18, v27"]
    ok = [ins[0], ins[1], ins[3], "v_mov_b32_e32 v18, v27", "s_waitcnt lgkmcnt(0)", "v_mov_b32_e32 v19, v26"]
    assert not _early_uses(ok)
    late = ["global_load_dword v5, v[2:3], off", "global_load_dword v6, v[2:3], off", "s_waitcnt vmcnt(1)", "v_add_u32_e32 v7, v5, v6"]
    assert _early_uses(late) == ["v_add_u32_e32 v7, v5, v6"]

