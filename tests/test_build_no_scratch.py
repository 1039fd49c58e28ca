"""Build check: no kernel of the library may spill registers to scratch memory,
except the few on the list below (each with its reason and its limit).  Every
source is compiled for the device with the compiler's resource remarks; nothing
runs, no GPU involved.  A spill in the matrix-core kernels costs tens of per
cent (their loops have no idle issue slots), and it shows in no parity test."""
import re
import subprocess

from paper_2010_00704_amd.build import resource_usage

# (pattern on the demangled kernel name, most bytes of scratch per lane, why it is tolerated)
ALLOWED = [
    (r"conv_branches_kernel<\d+, \d+, [01], [23], true>", 20,
     "module-tail forms of the vector-ALU branch kernel: scalar registers of the epilogue's addressing "
     "spill once, outside the loop"),
    (r"conv_valu_kernel<1, 2, [234], true>", 20,
     "module forms of the one-pixel-per-lane vector-ALU kernel: the same, outside the loop"),
    (r"conv_mfma_fp4_kernel<4, (12|14|15), true, false>", 72,
     "pad-word branch mode on the matrix cores: 256 accumulators plus the pad-word counts; the spilled "
     "values are epilogue parameters, reloaded once after the loop"),
]


def _demangle(names):
    out = subprocess.run(["c++filt"], input="\n".join(names), stdout=subprocess.PIPE, text=True, check=True)
    return out.stdout.splitlines()


def test_no_kernel_spills_to_scratch():
    usage = resource_usage()
    assert len(usage) > 100, "the resource remarks were not parsed"
    names = list(usage)
    offenders = []
    used = set()
    for sym, name in zip(names, _demangle(names)):
        u = usage[sym]
        assert "scratch" in u, name
        if u["scratch"] == 0:
            continue
        for i, (pat, limit, _why) in enumerate(ALLOWED):
            if re.search(pat, name) and u["scratch"] <= limit:
                used.add(i)
                break
        else:
            offenders.append("%s: %d B/lane, %d VGPR spills, %d SGPR spills (%s)" % (
                name.replace("(anonymous namespace)::", "").split("(")[0], u["scratch"], u.get("vgpr_spills", -1), u.get("sgpr_spills", -1), u["source"]))
    assert not offenders, "kernels with scratch memory:\n" + "\n".join(offenders)
    stale = [ALLOWED[i][0] for i in range(len(ALLOWED)) if i not in used]
    assert not stale, "allow-list entries that no kernel needs any more: %s" % stale
