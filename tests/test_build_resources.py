"""The compiler's per-kernel resource report, kept by the build next to the library: no kernel may spill
vector registers to memory (a spill changes no result and halves a bandwidth-bound kernel's speed, so no
parity test sees it), and scratch memory is used nowhere but in the one slow path listed here."""
import re

from paper_2504_18658_amd import build

# the unaligned 16-per-node form of the rows kernel keeps 20 bytes of spilled scalar registers there
SCRATCH_ALLOWED = re.compile(r"k_share_rows_fusedILi\dELi16ELb0E")


def _report():
    build.build(force=False)          # compiles only when the library is not the sources' own
    rep = build.resources()
    if rep is None:                   # a library of this build without its report: make both anew
        build.build(force=True)
        rep = build.resources()
    assert rep, "no resource report next to the library"
    return rep


def test_no_kernel_spills_vector_registers():
    rep = _report()
    assert len(rep) > 100             # every template instance is a kernel of its own
    spilled = {k: v for k, v in rep.items() if v.get("vgpr_spill", 0)}
    assert not spilled, spilled


def test_scratch_memory_only_where_listed():
    rep = _report()
    used = sorted(k for k, v in rep.items() if v.get("scratch_bytes", 0) and not SCRATCH_ALLOWED.search(k))
    assert not used, used


def test_thousand_thread_blocks_fit_the_register_file():
    """A 1024-thread block is four wavefronts per SIMD: 128 vector registers each at most."""
    rep = _report()
    lds = {k: v for k, v in rep.items() if "k_reduce2l_lds" in k or "k_flat_lds" in k}
    assert lds
    assert max(v["vgpr"] for v in lds.values()) <= 128


def test_remark_parser_reads_the_compilers_format():
    text = """
step_kernels.hip:67:1: remark: Function Name: _Z3fooPf [-Rpass-analysis=kernel-resource-usage]
   67 | __global__ void foo(float* p) {
      | ^
step_kernels.hip:67:1: remark:     TotalSGPRs: 22 [-Rpass-analysis=kernel-resource-usage]
step_kernels.hip:67:1: remark:     VGPRs: 11 [-Rpass-analysis=kernel-resource-usage]
step_kernels.hip:67:1: remark:     AGPRs: 0 [-Rpass-analysis=kernel-resource-usage]
step_kernels.hip:67:1: remark:     ScratchSize [bytes/lane]: 160 [-Rpass-analysis=kernel-resource-usage]
step_kernels.hip:67:1: remark:     Dynamic Stack: False [-Rpass-analysis=kernel-resource-usage]
step_kernels.hip:67:1: remark:     Occupancy [waves/SIMD]: 4 [-Rpass-analysis=kernel-resource-usage]
step_kernels.hip:67:1: remark:     SGPRs Spill: 3 [-Rpass-analysis=kernel-resource-usage]
step_kernels.hip:67:1: remark:     VGPRs Spill: 40 [-Rpass-analysis=kernel-resource-usage]
step_kernels.hip:90:1: remark: Function Name: _Z3barPf [-Rpass-analysis=kernel-resource-usage]
step_kernels.hip:90:1: remark:     VGPRs: 7 [-Rpass-analysis=kernel-resource-usage]
step_kernels.hip:90:1: remark:     ScratchSize [bytes/lane]: 0 [-Rpass-analysis=kernel-resource-usage]
step_kernels.hip:90:1: remark:     VGPRs Spill: 0 [-Rpass-analysis=kernel-resource-usage]
"""
    rep = build._parse_resource_remarks(text)
    assert rep["_Z3fooPf"] == {"vgpr": 11, "scratch_bytes": 160, "occupancy": 4, "sgpr_spill": 3, "vgpr_spill": 40}
    assert rep["_Z3barPf"] == {"vgpr": 7, "scratch_bytes": 0, "vgpr_spill": 0}
