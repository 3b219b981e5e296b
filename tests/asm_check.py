"""Static checker of the assembly text the per-matrix code generator emits (host only).

The generated kernels are straight-line code: one prologue, then one block per (row group,
K part) reached through a jump table, every block ending in s_endpgm.  That makes them easy
to interpret symbolically, and a mistake in the generator's index arithmetic would otherwise
first show on the GPU as a memory fault or as a result computed from a register whose load
has not arrived.  For every block this walks the instructions in order and checks

  * every buffer load / store: scalar offset + what the lane's address register has been
    advanced by + the largest lane offset + the access width stays inside the descriptor's
    num_records (and never goes below zero);
  * every LDS access: address-register class (lane * 4 / 8 / 16 plus a 64 KiB window) +
    offset + width stays inside the kernel's group segment;
  * no instruction reads or overwrites a register whose buffer load or LDS read may still be
    in flight: the s_waitcnt before it must have retired that load (vmcnt counts loads and
    stores on this target, LDS reads return in order under lgkmcnt), and no load is issued
    into a register whose previous load was never consumed;
  * every VGPR index is below next_free_vgpr, every SGPR index below next_free_sgpr; a
    workgroup's registers and its group segment fit one compute unit;
  * the jump table has one entry per block and every block ends the program.

`check(text, info)` returns a list of problems (empty = clean) and a few statistics.
"""
from __future__ import annotations

import re

_V = re.compile(r"\bv(\d+)\b|\bv\[(\d+):(\d+)\]")
_S = re.compile(r"\bs(\d+)\b|\bs\[(\d+):(\d+)\]")
_WIDTH = {"dword": 4, "dwordx2": 8, "dwordx4": 16, "short_d16": 2, "short": 2, "sbyte": 1, "ubyte": 1, "byte": 1}
_DSW = {"b32": 4, "b64": 8, "b128": 16}


def _vregs(tok):
    out = []
    for m in _V.finditer(tok):
        if m.group(1) is not None:
            out.append(int(m.group(1)))
        else:
            out.extend(range(int(m.group(2)), int(m.group(3)) + 1))
    return out


def _sregs(tok):
    out = []
    for m in _S.finditer(tok):
        if m.group(1) is not None:
            out.append(int(m.group(1)))
        else:
            out.extend(range(int(m.group(2)), int(m.group(3)) + 1))
    return out


def _imm(tok):
    tok = tok.strip()
    return int(tok, 16) if tok.lower().startswith(("0x", "-0x")) else int(tok)


def _signed32(x):
    x &= 0xFFFFFFFF
    return x - (1 << 32) if x & 0x80000000 else x


def check(text: str, info: dict, esz: int, osz: int):
    """info: the plan's INFO dictionary.  esz / osz: bytes of an operand / result element."""
    problems = []
    lines = [l.split(";")[0].rstrip() for l in text.splitlines()]
    meta = {}
    for l in lines:
        m = re.match(r"\s*\.amdhsa_(group_segment_fixed_size|next_free_vgpr|next_free_sgpr)\s+(\d+)", l)
        if m:
            meta[m.group(1)] = int(m.group(2))
    lds_bytes, n_vgpr, n_sgpr = meta["group_segment_fixed_size"], meta["next_free_vgpr"], meta["next_free_sgpr"]
    m = re.search(r"\.max_flat_workgroup_size:\s*(\d+)", text)
    waves = int(m.group(1)) // 64 if m else 0
    if waves < 1 or waves > 16:
        problems.append(f"workgroup of {waves} waves")
    if (waves + 3) // 4 * ((n_vgpr + 7) // 8 * 8) > 512:
        problems.append(f"a workgroup of {waves} waves with {n_vgpr} registers each does not fit a compute unit")
    if lds_bytes > 160 * 1024:
        problems.append(f"group segment of {lds_bytes} bytes exceeds a compute unit's LDS")
    V = max(1, info["spec_vec"])
    nvc = info["N"] // V
    lanes = info["spec_lanes"]
    in_lane_max = (nvc - 1) * V * esz      # byte offset of the last column a lane can own, inside a row of B / X
    out_lane_max = (nvc - 1) * V * osz

    # ---- prologue: descriptor extents and the class of the LDS address register
    body = [l.strip() for l in lines]
    first_block = next(i for i, l in enumerate(body) if l.startswith(".Lg0:"))
    func_end = next(i for i, l in enumerate(body) if l.startswith(".Lfunc_end:"))
    records = {}
    lds_class = {}    # vgpr -> (bytes per lane, base)
    for l in body[:first_block]:
        m = re.match(r"s_mov_b32 s(10|14), (0x[0-9a-f]+|\d+)$", l)
        if m:
            records[int(m.group(1))] = _imm(m.group(2))
        m = re.match(r"v_lshlrev_b32_e32 v1, (\d+), v0$", l)
        if m:
            lds_class[1] = (1 << int(m.group(1)), 0)
    # the code prefetch of the prologue: lane i touches byte i * stride + 128 j of its block, j = 0, 1, ...,
    # under a mask `length - 128 j > i * stride`; the loads must come in that order, each right after its
    # mask, their offsets must equal what has been subtracted from the length so far, and the
    # lines of one lane must not run into the next lane's
    pf_sub, pf_stride, pf_masked, pf_loads = 0, None, False, 0
    for l in body[:first_block]:
        m = re.match(r"v_mul_u32_u24_e32 v4, (0x[0-9a-f]+|\d+), v4$", l)
        if m:
            pf_stride = _imm(m.group(1))
        if re.match(r"v_cmpx_gt_i32_e32 vcc, s55, v4$", l):
            pf_masked = True
        elif re.match(r"s_sub_u32 s55, s55, 128$", l):
            pf_sub += 128
        elif l.startswith("global_load_dword"):
            m = re.match(r"global_load_dword v2, v4, s\[18:19\] offset:(\d+)$", l)
            if not m:
                problems.append(f"prologue: unexpected form of the code prefetch: `{l}`")
            elif not pf_masked or int(m.group(1)) != pf_sub or int(m.group(1)) > 4095:
                problems.append(f"prologue: code prefetch at offset {m.group(1)} is not covered by its length mask")
            pf_masked = False
            pf_loads += 1
        elif "exec" in l and pf_loads and not l.startswith("s_mov_b64 exec, s[22:23]"):
            problems.append(f"prologue: exec changed inside the code prefetch: `{l}`")
    if pf_loads and (pf_stride is None or pf_stride < 128 * pf_loads):
        problems.append("prologue: the prefetch lines of neighbouring lanes overlap")
    table = [l for l in body[:first_block] if l.startswith(".long .Lg")]
    n_blocks = sum(1 for l in body if re.match(r"\.Lg\d+:$", l))
    if len(table) != n_blocks:
        problems.append(f"jump table has {len(table)} entries for {n_blocks} blocks")
    if 10 not in records or 14 not in records:
        problems.append("descriptor extents not found in the prologue")
        return problems, {}

    stats = {"blocks": n_blocks, "loads": 0, "stores": 0, "lds": 0, "max_in_end": 0, "max_out_end": 0, "max_lds_end": 0,
             "prefetch_loads": pf_loads}

    # ---- blocks
    i = first_block
    while i < func_end:
        l = body[i]
        if not re.match(r"\.Lg\d+:$", l):
            i += 1
            continue
        label = l[:-1]
        i += 1
        sconst = {}
        advanced = 0            # bytes the lane's operand address register has been advanced by
        vm_issued = 0           # buffer loads and stores issued
        vm_done = 0             # ... known complete
        lg_issued = 0
        lg_done = 0
        pend_vm = {}            # vgpr -> sequence number of the buffer load it waits for
        pend_lg = {}
        classes = dict(lds_class)
        ended = False

        def bad(msg):
            problems.append(f"{label} line {i + 1}: {msg}: `{body[i]}`")

        def touch(regs, what):
            for r in regs:
                if r == 2 and pf_loads:
                    bad("v2 is where the prologue's code prefetch lands, at any time: no block may use it")
                if r >= n_vgpr:
                    bad(f"v{r} is beyond next_free_vgpr {n_vgpr}")
                if r in pend_vm and pend_vm[r] >= vm_done:
                    bad(f"{what} v{r} while its buffer load may be in flight")
                if r in pend_lg and pend_lg[r] >= lg_done:
                    bad(f"{what} v{r} while its LDS read may be in flight")

        while i < func_end and not re.match(r"\.Lg\d+:$", body[i]):
            l = body[i]
            if not l or l.startswith("."):
                i += 1
                continue
            if ended:
                bad("instruction after s_endpgm")
            op, _, rest = l.partition(" ")
            args = [a.strip() for a in rest.split(",")] if rest else []
            for r in _sregs(rest):
                if r >= n_sgpr + 6:   # vcc, flat_scratch and xnack_mask sit above next_free_sgpr
                    bad(f"s{r} is beyond the kernel's scalar registers")
            if op == "s_endpgm":
                ended = True
            elif op in ("s_mov_b32", "s_movk_i32") and re.match(r"s\d+$", args[0]) and re.match(r"(-?0x[0-9a-fA-F]+|-?\d+)$", args[1]):
                sconst[int(args[0][1:])] = _imm(args[1])
            elif op == "s_waitcnt":
                m = re.search(r"vmcnt\((\d+)\)", rest)
                if m:
                    vm_done = max(vm_done, vm_issued - int(m.group(1)))
                m = re.search(r"lgkmcnt\((\d+)\)", rest)
                if m:
                    lg_done = max(lg_done, lg_issued - int(m.group(1)))
            elif op.startswith("buffer_load_"):
                width = _WIDTH[op[len("buffer_load_"):]]
                dst, addr = _vregs(args[0]), _vregs(args[1])
                m = re.match(r"s(\d+) offen", args[3])
                soff = sconst.get(int(m.group(1))) if m else None
                if soff is None:
                    bad("scalar offset of the load is not a known constant")
                elif addr != [0]:
                    bad("operand loads are expected to address through v0")
                else:
                    lo, hi = soff + advanced, soff + advanced + in_lane_max + width
                    stats["max_in_end"] = max(stats["max_in_end"], hi)
                    if lo < 0 or hi > records[10]:
                        bad(f"load reaches bytes [{lo}, {hi}) of a {records[10]}-byte operand")
                touch(addr, "addressing with")
                for r in dst:
                    if r >= n_vgpr:
                        bad(f"v{r} is beyond next_free_vgpr {n_vgpr}")
                    if (r in pend_vm and pend_vm[r] >= vm_done) or (r in pend_lg and pend_lg[r] >= lg_done):
                        bad(f"load into v{r} whose previous load was never waited for")
                    pend_vm[r] = vm_issued
                    classes.pop(r, None)
                vm_issued += 1
                stats["loads"] += 1
            elif op.startswith("buffer_store_"):
                width = _WIDTH[op[len("buffer_store_"):]]
                src, addr = _vregs(args[0]), _vregs(args[1])
                m = re.match(r"s(\d+) offen", args[3])
                soff = sconst.get(int(m.group(1))) if m else None
                if soff is None:
                    bad("scalar offset of the store is not a known constant")
                elif addr != [3]:
                    bad("result stores are expected to address through v3")
                else:
                    hi = soff + out_lane_max + width
                    stats["max_out_end"] = max(stats["max_out_end"], hi)
                    if soff < 0 or hi > records[14]:
                        bad(f"store reaches byte {hi} of a {records[14]}-byte result")
                touch(src + addr, "storing")
                vm_issued += 1
                stats["stores"] += 1
            elif op.startswith("ds_read_") or op.startswith("ds_write_"):
                width = _DSW[op.split("_")[2]]
                is_read = op.startswith("ds_read_")
                addr = _vregs(args[0] if not is_read else args[1])
                data = _vregs(args[1] if not is_read else args[0])
                m = re.search(r"offset:(\d+)", rest)
                off = int(m.group(1)) if m else 0
                if off > 65535:
                    bad("LDS offset does not fit 16 bits")
                if len(addr) != 1 or addr[0] not in classes:
                    bad("LDS address register of unknown origin")
                else:
                    per_lane, base = classes[addr[0]]
                    # K-split exchange: only the lanes that own a column are active; staging
                    # variant: the area is laid out for all 64 lanes of a wave
                    top_lane = 63 if info["spec_mode"] == 2 else lanes - 1
                    end = base + per_lane * top_lane + off + width
                    stats["max_lds_end"] = max(stats["max_lds_end"], end)
                    if end > lds_bytes:
                        bad(f"LDS access ends at byte {end} of a {lds_bytes}-byte group segment")
                touch(addr, "addressing with")
                if is_read:
                    for r in data:
                        if r >= n_vgpr:
                            bad(f"v{r} is beyond next_free_vgpr {n_vgpr}")
                        if (r in pend_vm and pend_vm[r] >= vm_done) or (r in pend_lg and pend_lg[r] >= lg_done):
                            bad(f"LDS read into v{r} whose previous load was never waited for")
                        pend_lg[r] = lg_issued
                        classes.pop(r, None)
                else:
                    touch(data, "writing to LDS from")
                lg_issued += 1
                stats["lds"] += 1
            elif op.startswith("v_"):
                regs = _vregs(rest)
                touch(regs, "using")
                dst = _vregs(args[0]) if args and not op.startswith("v_cmp") else []
                # address arithmetic the exchange sets up: lane * 4n and 64 KiB windows
                if op == "v_add_u32_e32" and len(args) == 3 and dst == [0] and _vregs(args[2]) == [0]:
                    advanced += _signed32(_imm(args[1]))
                elif op == "v_add_u32_e32" and len(args) == 3 and _vregs(args[2]) and _vregs(args[2])[0] in classes and re.match(r"0x|\d", args[1]):
                    per_lane, base = classes[_vregs(args[2])[0]]
                    classes[dst[0]] = (per_lane, base + _imm(args[1]))
                elif op == "v_lshlrev_b32_e32" and len(args) == 3 and _vregs(args[2]) and _vregs(args[2])[0] in classes and args[1].isdigit():
                    per_lane, base = classes[_vregs(args[2])[0]]
                    classes[dst[0]] = (per_lane << int(args[1]), base << int(args[1]))
                else:
                    for r in dst:
                        if r != 1:
                            classes.pop(r, None)
                for r in regs:   # consumed: the register is an ordinary value again
                    if r in pend_vm and pend_vm[r] < vm_done:
                        del pend_vm[r]
                    if r in pend_lg and pend_lg[r] < lg_done:
                        del pend_lg[r]
            i += 1
        if not ended:
            problems.append(f"{label}: block does not end the program")
    return problems, stats
