#!/usr/bin/env python3
"""Writes score_asm.h: the score phase (S^T = K Q^T for one 32-key block) as ONE inline-asm
statement per head dimension, so that the LDS prefetch distance and the lgkmcnt waits are exactly
the ones written here (the compiler waits for every outstanding LDS read before an asm operand).

Per k-step kk (16 features): wait until key fragment kk has arrived, issue the 32x32x16 bf16 MFMA
that accumulates into the score registers (VGPR form: the AGPR half of the register file is full
of output accumulators), refill the fragment register with fragment kk + DEPTH.

Run from this directory:  python3 gen_score_asm.py > score_asm.h
"""

DEPTH = 6


def body(ks: int, depth: int) -> str:
    # operands: %0 scores (16 VGPRs), %1..%depth fragment registers, %(depth+1) LDS byte address,
    #           %(depth+2+kk) query fragment kk
    t = lambda i: f"%{1 + i}"
    addr = f"%{depth + 1}"
    q = lambda kk: f"%{depth + 2 + kk}"
    lines = []
    for d in range(min(depth, ks)):
        lines.append(f"ds_read_b128 {t(d)}, {addr} offset:{d * 32}")
    for kk in range(ks):
        newer = min(depth - 1, ks - 1 - kk)
        lines.append(f"s_waitcnt lgkmcnt({newer})")
        src_c = "0" if kk == 0 else "%0"
        lines.append(f"v_mfma_f32_32x32x16_bf16 %0, {t(kk % depth)}, {q(kk)}, {src_c}")
        if kk + depth < ks:
            lines.append(f"ds_read_b128 {t(kk % depth)}, {addr} offset:{(kk + depth) * 32}")
    # the last result must have left the matrix pipeline before a vector instruction reads it
    lines += ["s_nop 7", "s_nop 7", "s_nop 7"]
    return "".join(f'    "{l}\\n"\n' for l in lines)


def body_copy(ks: int, depth: int, n_copy: int, waves: int, hint: str = "") -> str:
    """Score phase with the global -> LDS copy of a later key tile woven in: one
    global_load_lds_dwordx4 every few matrix instructions, so that issuing the copy costs the
    matrix cores nothing. Extra operands after the query fragments: n_copy per-lane byte offsets,
    the largest valid offset (SGPR), the tile's global base (SGPR pair), the LDS base of this
    wave's first chunk (SGPR), and a scratch VGPR (output). `hint`: cache-policy modifier of the
    copy instructions (" nt" for data that is read once)."""
    t = lambda i: f"%{1 + i}"
    tmp = f"%{depth + 1}"                      # scratch VGPR (early-clobber output)
    addr = f"%{depth + 2}"
    q = lambda kk: f"%{depth + 3 + kk}"
    base = depth + 3 + ks
    voff = lambda c: f"%{base + c}"
    kmax, src, m0b = f"%{base + n_copy}", f"%{base + n_copy + 1}", f"%{base + n_copy + 2}"
    every = ks // n_copy
    lines = []
    for d in range(min(depth, ks)):
        lines.append(f"ds_read_b128 {t(d)}, {addr} offset:{d * 32}")
    c = 0
    for kk in range(ks):
        newer = min(depth - 1, ks - 1 - kk)
        lines.append(f"s_waitcnt lgkmcnt({newer})")
        src_c = "0" if kk == 0 else "%0"
        lines.append(f"v_mfma_f32_32x32x16_bf16 %0, {t(kk % depth)}, {q(kk)}, {src_c}")
        if kk + depth < ks:
            lines.append(f"ds_read_b128 {t(kk % depth)}, {addr} offset:{(kk + depth) * 32}")
        if c < n_copy and kk % every == every // 2:
            lines.append(f"v_min_u32 {tmp}, {kmax}, {voff(c)}")
            # (the scalar add also writes SCC: the statement names it as clobbered, or a compare the
            # compiler made before the statement and selects on after it reads the add's carry)
            lines.append(f"s_add_u32 m0, {m0b}, {c * waves * 1024}")
            lines.append("s_nop 0")
            lines.append(f"global_load_lds_dwordx4 {tmp}, {src}{hint}")
            c += 1
    assert c == n_copy
    lines += ["s_nop 7", "s_nop 7", "s_nop 7"]
    return "".join(f'    "{l}\\n"\n' for l in lines)


def macro_copy(dqk: int, n_copy: int, waves: int, hint: str = "") -> str:
    ks = dqk // 16
    depth = min(DEPTH, ks)
    outs = ['"=&v"(s_)'] + [f'"=&v"(kf_[{d}])' for d in range(depth)] + ['"=&v"(tmp_)']
    ins = ['"v"(addr_)'] + [f'"v"(qf_[{kk}])' for kk in range(ks)] + [f'"v"(voff_[{c}])' for c in range(n_copy)]
    ins += ['"s"(kmax_)', '"s"(src_)', '"s"(m0base_)']
    suffix = "_" + hint.strip().upper() if hint else ""
    text = f"// d_qk = {dqk}, {waves} waves per workgroup: as above, plus {n_copy} copy instructions of a later key tile"
    text += f" (cache policy:{hint})\n" if hint else "\n"
    text += f"#define LOZA_SCORE_PHASE_{dqk}_COPY_W{waves}{suffix}(s_, kf_, tmp_, addr_, qf_, voff_, kmax_, src_, m0base_) \\\n    asm volatile( \\\n"
    text += "".join(l.rstrip("\n") + " \\\n" for l in body_copy(ks, depth, n_copy, waves, hint).splitlines(True))
    text += "        : " + ", ".join(outs) + " \\\n        : " + ", ".join(ins) + " \\\n        : \"memory\", \"m0\", \"scc\")\n"
    text += f"#define LOZA_SCORE_COPIES_{dqk}_W{waves} {n_copy}\n"
    return text


def macro_bwd(ks: int, n_a: int, n_b: int, n_agpr: int, with_x: bool = True, n_voff: int = 0) -> str:
    """Phase 1 of the backward kernels: ks k-steps against stationary fragments of which the first
    n_agpr are read from AGPRs (the accumulators leave part of that file free) and the rest from
    VGPRs, with ALL of this wave's copy instructions of the next streamed tile woven in: n_a into the
    first sub-tile, n_b into the second, and one more (any sub-tile, with operands of its own) that
    only the first nextra_ waves issue. Chunk c of a sub-tile lands 4 KB after chunk c - 1 (four waves
    take turns)."""
    depth = min(DEPTH, ks)
    n_copy = n_a + n_b + (1 if with_x else 0)
    n_voff = max(n_voff, n_a + n_b + 1)       # length of the offset array; the extra instruction uses its last entry
    t = lambda i: f"%{1 + i}"
    tmp = f"%{depth + 1}"
    addr = f"%{depth + 2}"
    x = lambda kk: f"%{depth + 3 + kk}"
    base = depth + 3 + ks
    voff = lambda c: f"%{base + c}"
    sg = base + n_voff                      # scalar operands: (max, src, m0) of a, of b, of the extra one; its flag
    max_a, src_a, m0_a, max_b, src_b, m0_b, max_x, src_x, m0_x, wave, n_x = (f"%{sg + i}" for i in range(11))
    at = {((2 * c + 1) * ks) // (2 * n_copy): c for c in range(n_copy)}
    assert len(at) == n_copy, "at most one copy per k-step"
    lines = ["s_waitcnt lgkmcnt(0)"]        # the waits below count this statement's own LDS reads
    for d in range(depth):
        lines.append(f"ds_read_b128 {t(d)}, {addr} offset:{d * 32}")
    for kk in range(ks):
        lines.append(f"s_waitcnt lgkmcnt({min(depth - 1, ks - 1 - kk)})")
        lines.append(f"v_mfma_f32_32x32x16_bf16 %0, {t(kk % depth)}, {x(kk)}, {'0' if kk == 0 else '%0'}")
        if kk + depth < ks:
            lines.append(f"ds_read_b128 {t(kk % depth)}, {addr} offset:{(kk + depth) * 32}")
        if kk in at:
            c = at[kk]
            # (the scalar add and compare write SCC: the statement names it as clobbered)
            if c < n_a:
                lines += [f"v_min_u32 {tmp}, {max_a}, {voff(c)}", f"s_add_u32 m0, {m0_a}, {c * 4096}", "s_nop 0",
                          f"global_load_lds_dwordx4 {tmp}, {src_a}"]
            elif c < n_a + n_b:
                lines += [f"v_min_u32 {tmp}, {max_b}, {voff(c)}", f"s_add_u32 m0, {m0_b}, {(c - n_a) * 4096}", "s_nop 0",
                          f"global_load_lds_dwordx4 {tmp}, {src_b}"]
            else:
                lines += [f"s_cmp_ge_u32 {wave}, {n_x}", "s_cbranch_scc1 .Lloza_nox%=", f"v_min_u32 {tmp}, {max_x}, {voff(n_voff - 1)}",
                          f"s_mov_b32 m0, {m0_x}", "s_nop 0", f"global_load_lds_dwordx4 {tmp}, {src_x}", ".Lloza_nox%=:"]
    lines += ["s_nop 7", "s_nop 7", "s_nop 7"]
    outs = ['"=&v"(s_)'] + [f'"=&v"(kf_[{d}])' for d in range(depth)] + ['"=&v"(tmp_)']
    ins = ['"v"(addr_)'] + [f'"{"a" if kk < n_agpr else "v"}"(xf_[{kk}])' for kk in range(ks)]
    ins += [f'"v"(voff_[{c}])' for c in range(n_voff)]
    ins += [f'"s"({n})' for n in ("tc_.max1", "tc_.b1", "tc_.dst1", "tc_.max2", "tc_.b2", "tc_.dst2", "tc_.maxx", "tc_.bx", "tc_.dstx", "wave_")] + ['"n"(nextra_)']
    text = f"// backward, phase 1: {ks} k-steps, fragments 0..{n_agpr - 1} in AGPRs, {n_a} + {n_b} + {1 if with_x else 0} woven copies\n"
    text += f"#define LOZA_BWD_PHASE1_K{ks}_A{n_a}_B{n_b}{'' if with_x else 'N'}_G{n_agpr}(s_, kf_, tmp_, addr_, xf_, voff_, tc_, wave_, nextra_) \\\n    asm volatile( \\\n"
    text += "".join(f'    "{l}\\n" \\\n' for l in lines)
    text += "        : " + ", ".join(outs) + " \\\n        : " + ", ".join(ins) + " \\\n        : \"memory\", \"m0\", \"scc\")\n"
    return text


def macro(dqk: int) -> str:
    ks = dqk // 16
    depth = min(DEPTH, ks)
    outs = ['"=&v"(s_)'] + [f'"=&v"(kf_[{d}])' for d in range(depth)]
    ins = ['"v"(addr_)'] + [f'"v"(qf_[{kk}])' for kk in range(ks)]
    text = f"// d_qk = {dqk}: {ks} k-steps, prefetch depth {depth}\n"
    text += f"#define LOZA_SCORE_PHASE_{dqk}(s_, kf_, addr_, qf_) \\\n    asm volatile( \\\n"
    text += "".join(l.rstrip("\n") + " \\\n" for l in body(ks, depth).splitlines(True))
    text += "        : " + ", ".join(outs) + " \\\n        : " + ", ".join(ins) + " \\\n        : \"memory\")\n"
    text += f"#define LOZA_SCORE_DEPTH_{dqk} {depth}\n"
    return text


if __name__ == "__main__":
    print("// Generated by gen_score_asm.py -- do not edit by hand.")
    print("#ifndef LOZA_SCORE_ASM_H\n#define LOZA_SCORE_ASM_H\n")
    for dqk in (576, 128):
        print(macro(dqk))
    print(macro_copy(576, 9, 4))
    print(macro_copy(576, 4, 2, " nt"))
    # key-stationary kernel: 9 + 2 + 1 woven copies (the other 6 of the second sub-tile go out during the
    # elementwise step; the offset array keeps its 18 entries); row-stationary kernel: 9 + 0 + 1
    for ks, n_a, n_b, n_agpr in ((36, 9, 2, 32), (32, 9, 2, 24)):
        print(macro_bwd(ks, n_a, n_b, n_agpr, n_voff=18))
    for ks, n_a, n_b, n_agpr in ((36, 9, 0, 32), (32, 9, 0, 24)):
        print(macro_bwd(ks, n_a, n_b, n_agpr))
    print("#endif")
