"""Host-side tests of the instruction-level schedule search (no GPU): parsing of the compiled
kernel's assembly, legality of moves, wait-counter bookkeeping, and that mutated kernels still
assemble.  The kernel is cross-compiled for gfx950 here; nothing is launched."""
import os
import random
import re
import shutil
import tempfile

import pytest

from paper_2403_16863_amd import sip

pytestmark = pytest.mark.skipif(shutil.which("hipcc") is None, reason="needs hipcc to produce the kernel assembly")

KNOBS = (64, 8, 1, 1, 1, 1, 4, 1)   # the ping-pong default for d = 128


@pytest.fixture(scope="module")
def base():
    d = tempfile.mkdtemp(prefix="sip_test_")
    try:
        text = sip.compile_base(d, 128, 1, True, KNOBS)
        yield d, text, sip.Kernel(text)
    finally:
        shutil.rmtree(d, ignore_errors=True)


def test_regs_of():
    assert sip.regs_of("v[10:12], s3, vcc, v7 offset:16") == {"v10", "v11", "v12", "s3", "vcc", "v7"}
    assert sip.regs_of("exec_lo, m0, 0x40") == {"exec", "m0"}


def test_round_trip_and_inventory(base):
    _, text, k = base
    assert k.render() == text                       # parsing loses nothing
    mov = [k.nodes[i] for i in sip.movable_positions(k.nodes)]
    assert len(mov) >= 50
    assert any(n.kind == "unit" for n in mov) and any(n.mnem.startswith("ds_read_b128") for n in mov)
    assert any(n.mnem.startswith("ds_read_b64_tr_b16") for n in mov)
    assert all(n.in_loop for n in mov)
    for n in mov:
        if n.kind == "unit":        # M0 set-up, wait state, load (+ the 64-bit add of its base): moved as one
            ins = [l.strip().split()[0] for l in n.lines if not l.strip().startswith(";")]
            assert ins[-3:] == ["s_mov_b32", "s_nop", "global_load_lds_dwordx4"]
            assert ins[:-3] in ([], ["s_add_u32", "s_addc_u32"])
            assert n.defs == ({"m0"} if len(ins) == 3 else {"m0", "scc"} | (n.defs - {"m0", "scc"}))
            assert len(n.defs - {"m0", "scc"}) in (0, 2)


def _instr_lines(text):
    return [l.strip() for l in text.split("\n") if l.strip() and not l.strip().startswith((";", "."))
            and not re.match(r"^[.\w$]+:", l.strip())]


def test_random_walk_keeps_the_program(base):
    d, text, k = base
    rng = random.Random(3)
    x = sip.Schedule(tuple(k.nodes))
    for _ in range(400):
        y = sip.propose(x, rng)
        assert y is not None
        x = y
    out = k.render(list(x.nodes))
    a, b = _instr_lines(text), _instr_lines(out)
    strip_wait = lambda ls: sorted(l for l in ls if not l.startswith("s_waitcnt"))
    assert strip_wait(a) == strip_wait(b)           # same instructions, only waits may change their count
    assert len([l for l in a if l.startswith("s_waitcnt")]) == len([l for l in b if l.startswith("s_waitcnt")])
    # everything that is not a moved memory instruction keeps its relative order
    movable_text = {n.text for n in k.nodes if n.is_movable()}
    keep = lambda nodes: [n.uid for n in nodes if n.kind != "other" and n.text not in movable_text]
    assert keep(k.nodes) == keep(x.nodes)
    # operations counted by one counter keep their order among themselves
    lgkm = lambda nodes: [n.uid for n in nodes if n.is_lgkm_op()]
    vmem = lambda nodes: [n.uid for n in nodes if n.is_vmem()]
    assert lgkm(k.nodes) == lgkm(x.nodes) and vmem(k.nodes) == vmem(x.nodes)
    # nothing left its basic block
    def blocks(nodes):
        out, cur = {}, 0
        for n in nodes:
            if n.is_fence():
                cur += 1
            elif n.is_movable():
                out[n.uid] = cur
        return out
    assert blocks(k.nodes) == blocks(x.nodes)
    # and the result still assembles
    assert os.path.exists(sip.assemble(out, d, "walk"))


def _mini(lines):
    body = "\n".join(["k:"] + ["\t" + l for l in lines] + ["\ts_endpgm"])
    text = "\t.amdhsa_kernel k\n" + body + "\n"
    k = sip.Kernel(text, kernel_name="k")
    for n in k.nodes:
        n.in_loop = True
    return k


def _idx(k, needle):
    return next(i for i, n in enumerate(k.nodes) if needle in n.text)


def test_dependences_block_moves():
    k = _mini(["v_add_u32_e32 v1, v2, v3", "ds_read_b128 v[4:7], v1", "v_mfma_f32_32x32x16_bf16 v[16:31], v[4:7], v[8:11], v[16:31]",
               "v_mov_b32_e32 v40, v41"])
    i = _idx(k, "ds_read")
    assert sip.try_move(k.nodes, i, -1) is None     # address register is written just above
    assert sip.try_move(k.nodes, i, +1) is None     # the MFMA reads the destination
    k = _mini(["v_mov_b32_e32 v40, v41", "ds_read_b128 v[4:7], v1", "v_mov_b32_e32 v42, v43"])
    i = _idx(k, "ds_read")
    up, down = sip.try_move(k.nodes, i, -1), sip.try_move(k.nodes, i, +1)
    assert [n.mnem for n in up if n.kind == "ins"][:2] == ["ds_read_b128", "v_mov_b32_e32"]
    assert [n.mnem for n in down if n.kind == "ins"][1:3] == ["v_mov_b32_e32", "ds_read_b128"]


def test_fences_and_counter_order():
    for fence in ("s_barrier", "s_cbranch_scc1 .L1", "s_mov_b64 exec, s[0:1]", "ds_read_b128 v[20:23], v9", "ds_write_b64 v9, v[50:51]"):
        k = _mini(["ds_read_b128 v[4:7], v1", fence])
        assert sip.try_move(k.nodes, _idx(k, "v[4:7]"), +1) is None, fence
    # a vector instruction with a scalar result is never crossed, and nothing is taken out from just below one
    k = _mini(["v_readlane_b32 s4, v255, 3", "ds_read_b128 v[4:7], v1", "v_mov_b32_e32 v40, v41"])
    i = _idx(k, "ds_read")
    assert sip.try_move(k.nodes, i, -1) is None and sip.try_move(k.nodes, i, +1) is None


def test_wait_counter_bookkeeping():
    k = _mini(["s_waitcnt lgkmcnt(2)", "ds_read_b128 v[4:7], v1"])
    up = sip.try_move(k.nodes, _idx(k, "ds_read"), -1)
    assert "lgkmcnt(3)" in up[_idx(k, "s_waitcnt") + 1].text      # one more read in flight at the wait
    k = _mini(["ds_read_b128 v[4:7], v1", "s_waitcnt lgkmcnt(2)"])
    down = sip.try_move(k.nodes, _idx(k, "ds_read"), +1)
    assert "lgkmcnt(1)" in down[_idx(k, "ds_read")].text          # the wait did not cover the read
    k = _mini(["ds_read_b128 v[4:7], v1", "s_waitcnt lgkmcnt(0)"])
    assert sip.try_move(k.nodes, _idx(k, "ds_read"), +1) is None   # the wait covered the read
    k = _mini(["s_waitcnt lgkmcnt(15)", "ds_read_b128 v[4:7], v1"])
    assert sip.try_move(k.nodes, _idx(k, "ds_read"), -1) is None   # counter field is full
    # a wait on the tile loads is what makes LDS contents valid (direct global->LDS loads, no
    # barrier needed when the reader is the loader): an LDS read stays on its side of it
    for wait in ("s_waitcnt vmcnt(0)", "s_waitcnt vmcnt(24)", "s_waitcnt vmcnt(0) lgkmcnt(1)"):
        k = _mini([wait, "ds_read_b128 v[4:7], v1"])
        assert sip.try_move(k.nodes, _idx(k, "ds_read"), -1) is None, wait
        k = _mini(["ds_read_b128 v[4:7], v1", wait])
        assert sip.try_move(k.nodes, _idx(k, "ds_read"), +1) is None, wait


def test_scalar_loads_pin_their_wait():
    """A wait that may guard a scalar load (these return out of order) is neither crossed nor
    re-counted: the snippet is the case where an `lgkmcnt(0)` protects an `s_load` result."""
    k = _mini(["s_load_dwordx2 s[4:5], s[0:1], 0x10", "ds_read_b128 v[8:11], v2", "s_waitcnt lgkmcnt(0)", "ds_read_b128 v[4:7], v1",
               "v_mov_b32_e32 v40, v41"])
    assert sip.try_move(k.nodes, _idx(k, "v[4:7]"), -1) is None     # would turn the wait into lgkmcnt(1)
    assert sip.try_move(k.nodes, _idx(k, "v[8:11]"), +1) is None    # the wait covers it anyway
    k = _mini(["s_load_dword s4, s[0:1], 0x0", "s_waitcnt lgkmcnt(1)", "ds_read_b128 v[4:7], v1"])
    assert sip.try_move(k.nodes, _idx(k, "ds_read"), -1) is None
    # once the counter is known to be zero behind the scalar load, waits further down are ordinary again
    k = _mini(["s_load_dword s4, s[0:1], 0x0", "s_waitcnt lgkmcnt(0)", "v_mov_b32_e32 v40, v41", "s_waitcnt lgkmcnt(2)",
               "ds_read_b128 v[4:7], v1"])
    up = sip.try_move(k.nodes, _idx(k, "ds_read"), -1)
    assert up is not None and "lgkmcnt(3)" in "\n".join(n.text for n in up)
    # a basic-block boundary also ends the look-back
    k = _mini(["s_load_dword s4, s[0:1], 0x0", "s_cbranch_scc1 .L1", "s_waitcnt lgkmcnt(2)", "ds_read_b128 v[4:7], v1"])
    assert sip.try_move(k.nodes, _idx(k, "ds_read"), -1) is not None


def test_register_tile_loads_move_like_the_papers_loads():
    """Tile loads into registers (the staged load path) are part of the pruned space: they move
    past arithmetic, never past another vector-memory operation, a vmcnt wait, or an instruction
    that touches their registers."""
    k = _mini(["v_mov_b32_e32 v40, v41", "buffer_load_dwordx4 v[4:7], v9, s[4:7], s12 offen", "v_mov_b32_e32 v42, v43"])
    i = _idx(k, "buffer_load")
    assert k.nodes[i].is_movable() and k.nodes[i].is_vmem()
    assert sip.try_move(k.nodes, i, -1) is not None and sip.try_move(k.nodes, i, +1) is not None
    for blocker in ("s_waitcnt vmcnt(2)", "buffer_load_dwordx4 v[12:15], v9, s[4:7], s13 offen", "v_mov_b32_e32 v9, v50",
                    "v_add_f32_e32 v60, v5, v5", "global_store_dwordx4 v[0:1], v[20:23], off"):
        k = _mini(["buffer_load_dwordx4 v[4:7], v9, s[4:7], s12 offen", blocker])
        assert sip.try_move(k.nodes, _idx(k, "v[4:7]"), +1) is None, blocker
    k = _mini(["v_mov_b32_e32 v40, v41", "buffer_load_dwordx4 v9, s[4:7], s12 offen lds"])
    assert not k.nodes[_idx(k, "buffer_load")].is_movable()          # a load to LDS outside its hand-written group stays


def test_tile_load_unit():
    unit = [";;#ASMSTART", "s_mov_b32 m0, s26", "s_nop 0", "global_load_lds_dwordx4 v217, s[0:1]", ";;#ASMEND"]
    k = _mini(["v_mov_b32_e32 v40, v41"] + unit + ["v_mov_b32_e32 v42, v43"])
    i = next(i for i, n in enumerate(k.nodes) if n.kind == "unit")
    assert k.nodes[i].uses == {"s26", "v217", "s0", "s1"}
    assert sip.try_move(k.nodes, i, -1) is not None and sip.try_move(k.nodes, i, +1) is not None
    for blocker in ("s_add_u32 s0, s0, 0x2000", "s_mov_b32 m0, s5", "s_waitcnt vmcnt(0)", "global_load_dwordx4 v[60:63], v[2:3], off",
                    "v_mov_b32_e32 v217, v1"):
        k = _mini([blocker] + unit)
        i = next(i for i, n in enumerate(k.nodes) if n.kind == "unit")
        assert sip.try_move(k.nodes, i, -1) is None, blocker
    k = _mini(["s_waitcnt lgkmcnt(1)"] + unit)                     # a wait on another counter does not hold it
    i = next(i for i, n in enumerate(k.nodes) if n.kind == "unit")
    assert sip.try_move(k.nodes, i, -1) is not None
    # the 64-bit add of the base travels with the load; the group writes the condition code
    grouped = ["s_add_u32 s0, s8, 0x2000", "s_addc_u32 s1, s9, 0"] + unit
    k = _mini(["v_mov_b32_e32 v40, v41"] + grouped + ["v_mov_b32_e32 v42, v43"])
    i = next(i for i, n in enumerate(k.nodes) if n.kind == "unit")
    assert k.nodes[i].defs == {"m0", "s0", "s1", "scc"} and k.nodes[i].uses == {"s26", "v217", "s8", "s9"}
    assert sip.try_move(k.nodes, i, -1) is not None and sip.try_move(k.nodes, i, +1) is not None
    for blocker in ("s_cmp_lt_i32 s20, s21", "s_cselect_b64 s[30:31], -1, 0", "s_mov_b32 s8, s40", "v_mov_b32_e32 v50, s0"):
        k = _mini(grouped + [blocker])
        i = next(i for i, n in enumerate(k.nodes) if n.kind == "unit")
        assert sip.try_move(k.nodes, i, +1) is None, blocker


def test_anneal_states_on_a_toy_schedule():
    # states are integers, neighbours +-1, runtime |x - 7| + 1: the search must find 7 from 0
    from paper_2403_16863_amd.search import anneal_states
    res = anneal_states(0, lambda x, rng: x + rng.choice((-1, 1)), lambda x: abs(x - 7) + 1.0,
                        lambda x: x != 3 or True, seed=5, t_max=0.5, t_min=1e-3, cool=1.03)
    assert res.t_best <= res.t0 and res.best in res.times
    assert res.t_best == min(res.times.values())
    res2 = anneal_states(0, lambda x, rng: x + rng.choice((-1, 1)), lambda x: abs(x - 7) + 1.0,
                         lambda x: True, seed=5, t_max=0.5, t_min=1e-3, cool=1.03)
    assert [s.candidate for s in res.steps] == [s.candidate for s in res2.steps]   # deterministic per seed


GEMM_KNOBS = (4, 32, 4, 0)


def test_gemm_kernel_parses_and_mutates():
    """The second workload's kernel: its steady-state loop is straight-line code at loop depth 1
    holding the counted wait, six LDS reads, four tile loads and two MFMAs; moves keep the
    multiset of instructions, never carry a read across the wait on the loads, and still assemble."""
    d = tempfile.mkdtemp(prefix="sip_gemm_test_")
    try:
        text = sip.compile_gemm_base(d, 0, GEMM_KNOBS)
        k = sip.Kernel(text, loop_depth=1)
        assert k.render() == text
        mov = [k.nodes[i] for i in sip.movable_positions(k.nodes)]
        assert sum(n.kind == "unit" for n in mov) >= 4 and sum(n.mnem.startswith("ds_read") for n in mov) >= 6
        rng = random.Random(1)
        x = sip.Schedule(tuple(k.nodes))
        for _ in range(300):
            y = sip.propose(x, rng)
            assert y is not None
            x = y
        assert sorted(_instr_lines(k.render(list(x.nodes)))) != [] and len(x.moves) == 300
        strip = lambda ls: sorted(re.sub(r"lgkmcnt\(\d+\)", "lgkmcnt(n)", l) for l in ls)
        assert strip(_instr_lines(k.render(list(x.nodes)))) == strip(_instr_lines(text))
        # every LDS read of the loop is still behind the loop's wait on the loads
        body = [n for n in x.nodes if n.in_loop and n.kind in ("ins", "unit")]
        first_wait = next(i for i, n in enumerate(body) if n.mnem == "s_waitcnt" and "vmcnt" in n.text)
        steady = body[:next(i for i, n in enumerate(body) if n.mnem.startswith("s_cbranch"))]
        assert all(not n.mnem.startswith("ds_read") for n in steady[:first_wait])
        assert sum(n.mnem.startswith("ds_read") for n in steady) == 6
        sip.assemble(k.render(list(x.nodes)), d, "mut")
    finally:
        shutil.rmtree(d, ignore_errors=True)
