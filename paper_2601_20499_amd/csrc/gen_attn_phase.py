#!/usr/bin/env python3
"""Writes df_attn_phase.inc: the MFMA phase of the attention kernel as one asm block per variant.

One MFMA phase of a wave is S^T = K Q^T for a 64-key tile (2 key blocks x D/16 k-steps of
v_mfma_f32_32x32x16_bf16, A operand = K rows read from LDS with ds_read_b128, B operand = the
wave's Q fragment in registers) followed, unless the variant only scores, by O^T += V^T P^T
(D/32 output blocks x 4 k-steps, A operand = V^T read from a row-major V tile with
ds_read_b64_tr_b16, B operand = P^T in registers).

Why one asm block: the LDS reads that feed the matrix core return asynchronously.  Between
the read and the s_waitcnt that covers it the destination registers must not be touched, and
the order "wait, MFMA, next read" must not change.  Inside a single asm statement both hold
by construction: the staging registers are fixed (declared as clobbers, so the compiler keeps
everything else out of them) and nothing can be scheduled into the block.  The block also
carries its own wait states: the compiler's hazard recogniser does not look into asm, so
  * an accumulator is only reused by the MFMA after next (two independent accumulators
    alternate in the first product, D/32 in the second): no dependent MFMAs back to back;
  * the block ends with 16 idle cycles, more than the 12 a vector instruction must keep
    from an 8-pass MFMA whose result it reads or overwrites.
DEPTH operands are in flight; waits are taken once per pair of MFMAs.

Run this script after changing the tile layout (TileLayout in df_attn.hip) or the schedule;
the include is committed and tests/test_abi.py checks that it is what this script writes.
"""
import os

KT = 64                 # keys per tile
DEPTH = 4               # operands (4 registers each) in flight
PRIORITY = 0            # wave priority during the block (0 = leave it alone)
STAGE0 = 256 - 4 * DEPTH


def layout(D):
    rowb = 2 * D
    rpg = 1024 // rowb
    ng = KT // rpg
    kgs, vgs = 1024 + 16, 1024 + 64
    k_row = lambda r: (r % ng) * kgs + (r // ng) * rowb
    v_row = lambda r: (r % ng) * vgs + (r // ng) * rowb
    return dict(rowb=rowb, ng=ng, kgs=kgs, vgs=vgs, k_row=k_row, v_row=v_row)


def ops_of(D, do_pv):
    """List of (mfma text pieces, [read instructions]) in issue order."""
    L = layout(D)
    KS, DB = D // 16, D // 32
    ops = []
    for i in range(2 * KS):
        ks, kb = i // 2, i % 2
        ops.append(dict(kind="qk", ks=ks, kb=kb, reads=[("b128", L["k_row"](32 * kb) + 32 * ks)]))
    if do_pv:
        for r in range(4 * DB):
            db, ts, kb = r % DB, (r // DB) % 2, r // (2 * DB)
            row0 = 32 * kb + 16 * ts
            ops.append(dict(kind="pv", db=db, ts=ts, kb=kb,
                            reads=[("tr", L["v_row"](row0) + 64 * db), ("tr", L["v_row"](row0 + 4) + 64 * db)]))
    return ops


def block(D, do_pv):
    ops = ops_of(D, do_pv)
    n = len(ops)
    lines = []
    slot = lambda i: STAGE0 + 4 * (i % DEPTH)

    def issue(i):
        if i >= n:
            return
        b = slot(i)
        op = ops[i]
        if op["kind"] == "qk":
            lines.append(f"ds_read_b128 v[{b}:{b + 3}], %[ka] offset:{op['reads'][0][1]}")
        else:
            lines.append(f"ds_read_b64_tr_b16 v[{b}:{b + 1}], %[va] offset:{op['reads'][0][1]}")
            lines.append(f"ds_read_b64_tr_b16 v[{b + 2}:{b + 3}], %[va] offset:{op['reads'][1][1]}")

    def mfma(i):
        b = slot(i)
        op = ops[i]
        if op["kind"] == "qk":
            acc = f"%[s{op['kb']}]"
            c = "0" if op["ks"] == 0 else acc
            lines.append(f"v_mfma_f32_32x32x16_bf16 {acc}, v[{b}:{b + 3}], %[q{op['ks']}], {c}")
        else:
            acc = f"%[o{op['db']}]"
            lines.append(f"v_mfma_f32_32x32x16_bf16 {acc}, v[{b}:{b + 3}], %[p{op['kb']}{op['ts']}], {acc}")

    if PRIORITY:
        lines.append(f"s_setprio {PRIORITY}")
    for i in range(min(DEPTH, n)):
        issue(i)
    for i in range(0, n, 2):
        issued_upto = min(i + DEPTH - 1, n - 1)          # last operand whose reads are out
        pending = sum(len(ops[j]["reads"]) for j in range(i + 2, issued_upto + 1))
        lines.append(f"s_waitcnt lgkmcnt({pending})")
        mfma(i)
        mfma(i + 1)
        issue(i + DEPTH)
        issue(i + DEPTH + 1)
    if PRIORITY:
        lines.append("s_setprio 0")
    lines.append("s_nop 7")
    lines.append("s_nop 7")
    return lines


def function(D, do_pv):
    KS, DB = D // 16, D // 32
    L = layout(D)
    body = block(D, do_pv)
    asm = "\n".join(f'        "{ln}\\n\\t"' for ln in body)
    outs = ['[s0] "=&v"(s[0])', '[s1] "=&v"(s[1])']
    if do_pv:
        outs += [f'[o{db}] "+v"(o[{db}])' for db in range(DB)]
    ins = ['[ka] "v"(k_addr)']
    if do_pv:
        ins.append('[va] "v"(v_addr)')
    ins += [f'[q{ks}] "v"(qf[{ks}])' for ks in range(KS)]
    if do_pv:
        ins += [f'[p{kb}{ts}] "v"(pb[{kb}][{ts}])' for kb in range(2) for ts in range(2)]
    clob = ", ".join(f'"v{r}"' for r in range(STAGE0, 256))
    return f"""template <>
struct MfmaPhase<{D}, {'true' if do_pv else 'false'}> {{
  static_assert(TileLayout<{D}>::NG == {L['ng']} && TileLayout<{D}>::KGS == {L['kgs']} && TileLayout<{D}>::VGS == {L['vgs']} &&
                TileLayout<{D}>::ROWB == {L['rowb']} && kKT == {KT}, "regenerate df_attn_phase.inc");
  static __device__ __forceinline__ void run(unsigned k_addr, unsigned v_addr, const bf16x8 (&qf)[{KS}],
                                             const bf16x8 (&pb)[2][2], f32x16 (&s)[2], f32x16 (&o)[{DB}]) {{
    asm volatile(
{asm}
        : {', '.join(outs)}
        : {', '.join(ins)}
        : {clob});
  }}
}};
"""


def text():
    head = ("// Generated by gen_attn_phase.py - do not edit; see that script for the schedule and its reasons.\n"
            "// MfmaPhase<D, DO_PV>::run: S^T = K Q^T of the tile at k_addr, then (DO_PV) O^T += V^T P^T of the tile\n"
            "// at v_addr.  k_addr / v_addr are the lane's LDS byte addresses of the first A operand.\n"
            f"// Staging registers v{STAGE0}..v255, {DEPTH} operands in flight.\n"
            "template <int D, bool DO_PV>\nstruct MfmaPhase;\n\n")
    return head + "\n".join(function(D, pv) for D in (128, 64) for pv in (True, False))


OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "df_attn_phase.inc")

if __name__ == "__main__":
    with open(OUT, "w") as f:
        f.write(text())
    print("wrote", OUT)
