"""Guards on the compiled attention kernel that no parity test can give: properties of the
generated gfx950 code the kernel's hand-managed memory waits rely on.  Compiles the kernel file
to assembly with the flags of the real build (no GPU needed) and checks, for attn_mfma_kernel<128>
(the 256-row tiling is attn_skew_mfma_kernel, which has its own tests below):
  * it uses no scratch memory (a spilled register would be reloaded with a vector-memory load the
    explicit wait counts do not account for, and a spill of a register that an in-flight load is
    about to write would save stale data);
  * between the asm-issued loads of the next chunk's rows and the counted wait that completes them,
    nothing reads or overwrites their destination registers except the inter-chunk product of the
    anti-causal walk (which runs before that walk issues its own loads);
  * the only vmcnt waits after the prologue are the kernel's own (they sit inside asm blocks)."""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2502_07563_amd", "csrc")


@pytest.fixture(scope="module")
def isa(tmp_path_factory):
    from paper_2502_07563_amd import build as b
    out = tmp_path_factory.mktemp("isa") / "kernels_mfma.s"
    flags = [f for f in b.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), *flags, "-S", "--cuda-device-only",
           "-o", str(out), os.path.join(SRC, "kernels_mfma.hip")]
    subprocess.run(cmd, check=True, capture_output=True)
    return open(out).read().split("\n")


def _kernels(lines):
    for i, l in enumerate(lines):
        m = re.match(r"^(_ZN.*attn_mfma_kernelILi(\d+).*):", l)
        if m:
            end = next(j for j in range(i, len(lines)) if "s_endpgm" in lines[j])
            yield m.group(2), lines[i:end], m.group(1)


def _regs(text):
    out = set()
    for m in re.finditer(r"v\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        out |= {int(m.group(3))} if m.group(3) else set(range(int(m.group(1)), int(m.group(2)) + 1))
    return out


def test_attention_kernels_do_not_spill(isa):
    text = "\n".join(isa)
    found = 0
    for cname, body, sym in _kernels(isa):
        found += 1
        assert not any("scratch_" in l for l in body), f"attn_mfma_kernel<{cname}> touches scratch memory"
        m = re.search(r"\.amdhsa_kernel " + re.escape(sym) + r".*?\.amdhsa_private_segment_fixed_size (\d+)",
                      text, flags=re.S)
        assert m and int(m.group(1)) == 0, f"attn_mfma_kernel<{cname}> has a private segment"
    assert found == 1


def test_in_flight_row_registers_are_left_alone(isa):
    for cname, body, _ in _kernels(isa):
        in_asm, asm_loads, asm_waits = False, [], []
        for i, l in enumerate(body):
            if "#ASMSTART" in l:
                in_asm = True
            elif "#ASMEND" in l:
                in_asm = False
            elif in_asm and "global_load_dwordx4" in l:
                asm_loads.append((i, _regs(l.split(",")[0])))
            elif in_asm and "s_waitcnt vmcnt" in l:
                asm_waits.append(i)
        assert len(asm_loads) == 24, (cname, len(asm_loads))     # prologue, causal site, anti-causal site
        token = [i for i in asm_waits if "vmcnt(8)" in body[i] and i > asm_loads[-1][0]]
        assert len(token) == 1, (cname, token)
        dest = set().union(*(r for _, r in asm_loads[8:]))
        assert len(dest) == 32
        causal_last, anti_first, anti_last = asm_loads[15][0], asm_loads[16][0], asm_loads[23][0]
        for i in range(causal_last + 1, token[0]):
            l = body[i].strip()
            if not l or l.startswith(";") or not (_regs(l) & dest):
                continue
            if anti_first <= i <= anti_last and "global_load_dwordx4" in l:
                continue                         # the anti-causal walk's own loads
            assert i < anti_first and l.startswith("v_mfma"), (cname, i, l)


def test_no_compiler_placed_vmcnt_wait_in_the_walk(isa):
    for cname, body, _ in _kernels(isa):
        first_barrier = next(i for i, l in enumerate(body) if "s_barrier" in l)
        in_asm = False
        for i, l in enumerate(body):
            if "#ASMSTART" in l:
                in_asm = True
            elif "#ASMEND" in l:
                in_asm = False
            elif "vmcnt" in l and i > first_barrier:
                assert in_asm, (cname, i, l.strip())


# (symbol fragment, number of walk copies in the function): attn_skew_mfma_kernel without / with decay
# (two halves x two directions), and the backward's launch for long slots (four copies of the
# anti-causal pair's walk: dV / dK rows x early / late row blocks, plus the causal walk's two halves)
SKEW = (("attn_skew_mfma_kernelILb0E", 4), ("attn_skew_mfma_kernelILb1E", 4), ("attn_bwd_pair_mfma_kernel", 6))


def _skew_blocks(lines, inst):
    """Basic blocks of one instantiation of attn_skew_mfma_kernel as (loop header or None, [instruction lines])."""
    start = next(i for i, l in enumerate(lines) if re.match(r"^_ZN.*" + inst + r".*:", l))
    end = next(i for i in range(start, len(lines)) if lines[i].startswith(".Lfunc_end"))
    blocks, cur = [], [None, []]
    for l in lines[start:end]:
        m = re.match(r"^(\.LBB\d+_\d+:|; %bb\.\d+:)(.*)", l)
        if m:
            blocks.append(cur)
            h = re.search(r"in Loop: Header=(BB\d+_\d+)", m.group(2))
            own = re.match(r"^\.L(BB\d+_\d+):", l) if "This Loop Header" in m.group(2) else None
            cur = [h.group(1) if h else (own.group(1) if own else None), []]
        else:
            cur[1].append(l)
    blocks.append(cur)
    return lines[start:end], blocks


@pytest.mark.parametrize("inst,ncopies", SKEW)
def test_skew_kernel_uses_no_scratch_and_waits_only_where_it_says(isa, inst, ncopies):
    """attn_skew_mfma_kernel and attn_bwd_pair_mfma_kernel (several copies of a walk in one function):
    no scratch memory, and inside the walks' loops no vector-memory wait placed by the compiler (the
    prologues, outside the loops, wait for the slot state with ordinary loads)."""
    body, blocks = _skew_blocks(isa, inst)
    assert not any("scratch_" in l for l in body), f"{inst} touches scratch memory"
    loops = {h for h, ins in blocks if h and any("v_mfma" in l for l in ins)}
    assert len(loops) == ncopies, loops            # one loop per copy of a walk
    for h, ins in blocks:
        if h not in loops:
            continue
        in_asm = False
        for l in ins:
            if "#ASMSTART" in l:
                in_asm = True
            elif "#ASMEND" in l:
                in_asm = False
            elif "vmcnt" in l:
                assert in_asm, (h, l.strip())


@pytest.mark.parametrize("inst,ncopies", SKEW)
def test_skew_kernel_leaves_the_rows_in_flight_alone(isa, inst, ncopies):
    """The rows of A are requested with asm loads one or two blocks before they are needed, and taken
    over by an OR with the zero that the counted wait returns.  Between the request and that OR no
    instruction may touch the 32 destination registers (a copy made while a load is on its way
    carries stale data; a request whose registers are dead lets the compiler reuse them at once: that
    is how a first version of this kernel failed).  Checked in layout order inside each walk's loop:
    from the request to the OR (second half's waves: block 0 to block 2), or from the request to the
    loop's end and from its start to the OR (first half's waves: block 2 to the next block 0); and for
    the requests before the loops, up to their full wait."""
    body, blocks = _skew_blocks(isa, inst)
    by_loop = {}
    for h, ins in blocks:
        if h:
            by_loop.setdefault(h, []).extend(ins)
    checked = 0
    for h, ins in by_loop.items():
        if not any("v_mfma" in l for l in ins):
            continue                      # the walk over the documents of a packed batch
        code, in_asm = [], False          # (text, inside an asm block)
        for l in ins:
            t = l.strip()
            if "#ASMSTART" in l:
                in_asm = True
            elif "#ASMEND" in l:
                in_asm = False
            elif t and not t.startswith(";") and not t.startswith("."):
                code.append((t, in_asm))
        loads = [i for i, (t, a) in enumerate(code) if a and t.startswith("global_load_dwordx4")]
        assert len(loads) == 8, (h, len(loads))
        dest = set().union(*(_regs(code[i][0].split(",")[0]) for i in loads))
        assert len(dest) == 32, (h, len(dest))
        ors = [i for i, (t, a) in enumerate(code) if not a and t.startswith("v_or_b32") and _regs(t.split(",", 1)[1]) & dest]
        # the take-over ORs share the wait's zero as their other operand (a later reuse of a freed
        # register in some other OR is not one of them)
        zero = code[ors[0]][0].split(",")[1].strip()
        takes = [i for i in ors if code[i][0].split(",")[1].strip() == zero]
        assert len(takes) == 32, (h, len(takes))
        first_take, issue = takes[0], loads[-1]
        regions = [range(issue + 1, first_take)] if first_take > issue else [range(issue + 1, len(code)), range(0, first_take)]
        for r in regions:
            for i in r:
                assert not (_regs(code[i][0]) & dest), (h, code[i][0])
        checked += 1
    assert checked == ncopies
    # requests before the loops (the first half's walks): nothing touches their registers until the wait
    in_asm, pending = False, None
    for h, ins in blocks:
        if h:
            pending = None
            continue
        for l in ins:
            t = l.strip()
            if "#ASMSTART" in l:
                in_asm = True
            elif "#ASMEND" in l:
                in_asm = False
            elif in_asm and "global_load_dwordx4" in l:
                pending = (pending or set()) | _regs(l.split(",")[0])
            elif in_asm and "s_waitcnt vmcnt(0)" in l:
                pending = None
            elif not in_asm and pending and t and not t.startswith(";") and not t.startswith("."):
                assert not (_regs(t) & pending), t


def test_decay_attention_kernels_keep_their_loads_in_flight(isa):
    """The decayed pass counts its stage loads and the loads of the next chunk's rows by hand like
    the undecayed one: no scratch memory, and after the first barrier no vmcnt wait outside the
    kernel's own asm blocks."""
    text = "\n".join(isa)
    found = 0
    for i, l in enumerate(isa):
        m = re.match(r"^(_ZN.*attn_decay_mfma_kernelILi(\d+).*):", l)
        if not m:
            continue
        found += 1
        sym, cname = m.group(1), m.group(2)
        end = next(j for j in range(i, len(isa)) if "s_endpgm" in isa[j])
        body = isa[i:end]
        assert not any("scratch_" in x for x in body), f"attn_decay_mfma_kernel<{cname}> touches scratch memory"
        k = re.search(r"\.amdhsa_kernel " + re.escape(sym) + r".*?\.amdhsa_private_segment_fixed_size (\d+)",
                      text, flags=re.S)
        assert k and int(k.group(1)) == 0, f"attn_decay_mfma_kernel<{cname}> has a private segment"
        first_barrier = next(j for j, x in enumerate(body) if "s_barrier" in x)
        in_asm = False
        for j, x in enumerate(body):
            if "#ASMSTART" in x:
                in_asm = True
            elif "#ASMEND" in x:
                in_asm = False
            elif "vmcnt" in x and j > first_barrier:
                assert in_asm, (cname, j, x.strip())
    assert found == 1


@pytest.fixture(scope="module")
def isa_softmax(tmp_path_factory):
    from paper_2502_07563_amd import build as b
    out = tmp_path_factory.mktemp("isa_sm") / "kernels_softmax.s"
    flags = [f for f in b.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc"), *flags, "-S", "--cuda-device-only",
           "-o", str(out), os.path.join(SRC, "kernels_softmax.hip")]
    subprocess.run(cmd, check=True, capture_output=True)
    return open(out).read().split("\n")


def test_softmax_kernels_keep_their_stage_loads_in_flight(isa_softmax):
    """The softmax kernels count their direct-to-LDS stage loads by hand as well.  A register spill
    inside their loops would be reloaded with a vector-memory load, for which the compiler waits
    with vmcnt(0): that drains every stage load in flight (seen once: the dQ kernel lost 13 %).
    So: no scratch memory at all, and after the first barrier no vmcnt wait outside the kernels'
    own asm blocks."""
    text = "\n".join(isa_softmax)
    found = 0
    for i, l in enumerate(isa_softmax):
        m = re.match(r"^(_ZN.*(softmax_fwd_mfma_kernel|softmax_bwd_dq_mfma_kernel|softmax_bwd_dkv_mfma_kernel).*):", l)
        if not m:
            continue
        found += 1
        sym, name = m.group(1), m.group(2)
        end = next(j for j in range(i, len(isa_softmax)) if "s_endpgm" in isa_softmax[j])
        body = isa_softmax[i:end]
        assert not any("scratch_" in x for x in body), f"{name} touches scratch memory"
        k = re.search(r"\.amdhsa_kernel " + re.escape(sym) + r".*?\.amdhsa_private_segment_fixed_size (\d+)",
                      text, flags=re.S)
        assert k and int(k.group(1)) == 0, f"{name} has a private segment"
        first_barrier = next(j for j, x in enumerate(body) if "s_barrier" in x)
        in_asm = False
        for j, x in enumerate(body):
            if "#ASMSTART" in x:
                in_asm = True
            elif "#ASMEND" in x:
                in_asm = False
            elif "vmcnt" in x and j > first_barrier:
                assert in_asm, (name, j, x.strip())
    assert found == 3


def test_states_kernel_store_count_matches_its_wait_arithmetic(isa):
    """states_mfma_kernel lets the stores of a slot's state stay outstanding while it waits for
    stage loads that are older than they are, by adding their number (16 per state tile held by a
    wave, NSTORE in the source) to the counted wait.  Fewer store instructions than that in the
    compiled code (merged stores) would make those waits too lenient."""
    found = 0
    for i, l in enumerate(isa):
        if re.match(r"^_ZN.*states_mfma_kernelILb[01].*:", l):
            found += 1
            end = next(j for j in range(i, len(isa)) if isa[j].startswith(".Lfunc_end"))
            body = isa[i:end]
            stores = [x for x in body if re.search(r"\bglobal_store", x)]
            assert len(stores) == 32 and all("global_store_dword " in x for x in stores), len(stores)
            assert any("vmcnt(38)" in x for x in body) and any("vmcnt(6)" in x for x in body)
    assert found == 2
