"""Host-side checks on the kernel source for the two hardware hazards that the compiler does not
guard inside asm strings (gfx950 does not interlock them):
  1. a store of more than 64 bits reads its data registers for two more wait states, so every
     hand-written 16-byte store string must end in `s_nop 1`;
  2. a DPP operand must not be read within two wait states of the VALU write that produced it, so
     values that come out of the asm helpers vmax / vmin / vmax3 / vmin3 may reach a cross-lane
     move only through settled().
Also: bench.py's roofline.traffic comes from the counter summaries under profiles/."""
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2503_08154_amd", "csrc", "s2a_kernels.hpp")


def _source():
    text = open(SRC).read()
    return re.sub(r"//[^\n]*", "", text)          # comments out


def test_wide_store_strings_wait_before_their_registers_are_reused():
    text = _source()
    strings = re.findall(r'asm\s+volatile\s*\(\s*"((?:[^"\\]|\\.)*)"', text)
    wide = [s for s in strings if re.search(r"global_store_dwordx[34]|buffer_store_dwordx[34]", s)]
    assert wide, "no hand-written wide stores found: has the source moved?"
    for s in wide:
        assert s.rstrip().endswith(r"\n\ts_nop 1"), f"wide store without the trailing wait: {s!r}"
    # and no wide store is spelled any other way in an asm statement
    for s in re.findall(r'asm\s*\(\s*"((?:[^"\\]|\\.)*)"', text):
        assert "store_dwordx" not in s, f"a wide store in a non-volatile asm: {s!r}"


def test_asm_min_max_results_reach_cross_lane_moves_only_through_settled():
    text = _source()
    helpers = r"(?:vmax3|vmin3|vmax|vmin)"
    # 1. no cross-lane primitive is applied directly to a helper call
    for m in re.finditer(r"(dpp_move<[^>]*>|__builtin_amdgcn_update_dpp)\s*\(([^;]*);", text):
        assert not re.search(helpers + r"\s*\(", m.group(2)), f"cross-lane move of an unsettled value: {m.group(0)[:120]}"
    # 2. variables assigned from a helper are handed to group_max / group_min (which settle) or to
    #    settled(), never to a primitive or to the generic reductions
    assigned = set(re.findall(r"\b(\w+)\s*=\s*" + helpers + r"\s*\(", text))
    assert assigned, "no uses of the asm min/max helpers found: has the source moved?"
    inside_helpers = {"r"}                      # the helpers' own result variable
    for name in assigned - inside_helpers:
        # (names are matched file-wide; __shfl_xor is a ds_bpermute, an LDS-pipe instruction whose operands
        # are interlocked like any other, so it is not in this list)
        for prim in (r"dpp_move<[^>]*>", r"group_sum<[^>]*>", r"group_reduce<[^>]*>"):
            bad = re.search(prim + r"\s*\(\s*" + name + r"\b", text)
            assert not bad, f"{name} comes from an asm min/max and reaches {bad.group(0)} without settled()"
    # 3. the reductions that do take such values settle them, at entry and after every step
    for fn in ("group_max", "group_min"):
        body = re.search(fn + r"\s*\(float v\)\s*\{(.*?)\n\}", text, re.S).group(1)
        assert body.count("settled(") >= 2, f"{fn} no longer settles its operands"


def test_bench_traffic_comes_from_the_committed_counter_summaries():
    sys.path.insert(0, ROOT)
    import bench
    from paper_2503_08154_amd import workloads as wl
    table = bench.load_traffic()
    for name in ("vit_l16", "vit_g14", "vit_g14_f32", "vit_b16"):
        w = wl.WORKLOADS[name]
        alg = bench.bytes_per_direction(w.sizes()[0], w.dtype)
        for which in ("fwd", "bwd"):
            key = (name, f"s2a::{which}_kernel<{bench.dname(w.dtype)}>")
            assert key in table, f"profiles/ has no traffic line for {key}"
            entry = table[key]
            assert entry["algorithmic"] == alg
            assert abs(entry["bytes"] / alg - 1.0) < 0.01, f"{key}: counters saw {entry['bytes']} B against {alg} algorithmic"
            # what bench.py prints is this number, not a constant of its own
            res = {f"{which}_gbs": 1.0, f"{which}_us_per_launch": 1.0, f"{which}_us_median": 1.0, f"{which}_us_min": 1.0,
                   "bytes_per_launch": alg}
            assert bench.kernel_block(res, w, which, table)["traffic"] == entry["bytes"]
    assert not hasattr(bench, "MEASURED_TRAFFIC")
