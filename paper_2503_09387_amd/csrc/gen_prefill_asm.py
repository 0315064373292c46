#!/usr/bin/env python3
"""Writes vs_prefill_asm.inc: the gfx950 instruction sequences of the bf16 prefill kernel.

The prefill kernel keeps its matrix state in fixed registers and issues every matrix
instruction from hand-scheduled blocks of inline assembly:

  a[0:127]    output accumulators O^T: accumulator i = 4*row_group + dim_block in a[16i:16i+15]
  a[128:191]  query fragments: fragment 8*row_group + step in a[128+4i : 128+4i+3]
              (the compiler never sees these two as values; every block lists them as
              clobbered, which keeps it from holding anything of its own there across a block)
  v[128:191]  raw scores S[parity][row_group], 16 registers each: sub-block n (32 keys) of a
              key group uses parity n & 1; hidden from the compiler like the accumulators (the
              blocks list them as clobbered; the rare exact redo of a sub-block fetches them
              through an empty asm statement with a pinned output)
  v[192:207]  four buffers for K / V^T fragments read from LDS
  v[208:215]  temporaries and constants
  v[216:247]  packed bf16 probabilities P[parity][row_group][step], 4 registers each, hidden
              state like S

Everything else (addresses, softmax reference, scale, row sums) reaches a block as an ordinary
named operand.

The pipeline works on sub-blocks of 32 keys.  Step n of a key group does, in one block,
  QK(n+1): S[1-p] = K_{n+1} Q^T      (8 pairs of matrix instructions, p = n & 1)
  PV(n-1): O^T += V_{n-1}^T P[1-p]   (8 pairs)
  SM(n):   P[p] = bf16(2^(S[p]*scale - reference)), row sums of the rounded values
so that the softmax arithmetic of one sub-block is spread evenly under the matrix instructions
of its two neighbours.  S[p] is left untouched by SM(n): if the reference turns out too stale
(a sum above 2^8), the caller redoes sub-block n exactly from the raw scores.

Scheduling rules the blocks obey (gfx950, one wavefront per SIMD):
  * matrix instructions come in pairs that share the fragment read from LDS (row groups 0, 1);
  * the fragment of pair i+DIST is requested right after pair i and awaited with lgkmcnt just
    before its pair (LDS returns in order; a block starts with lgkmcnt(0));
  * ordinary instructions never read a matrix result inside the block that computes it, except
    after an explicit run of s_nop (an 8-pass instruction needs 11 idle issue slots);
  * a memory instruction reads a scalar register no earlier than five issue slots after a scalar
    instruction wrote it (the staging loads take their base address from s[88:91], which the
    caller sets before the block and the block leaves alone);
  * a transcendental result is not read by the next instruction; a mask written by a compare
    is not read by the next two; a dot-product result is read by other kinds of instruction no
    earlier than three instructions later; M0 is not used by the instruction after the one that
    writes it.

Row sums are taken over the bf16-rounded probabilities (v_dot2c_f32_bf16 against (1, 1)), the
values that enter P V, so that the output is an exact convex combination of V rows.
"""
import os
import sys

MFMA = "v_mfma_f32_32x32x16_bf16"
ROW = 256                      # bytes per K/V row in LDS
S_BASE = 128                   # S[par][r] at 128 + 32*par + 16*r
FR_BASE, NBUF, DIST = 192, 4, 3
TMP = 208                      # 208..211 item temporaries, 212 = -inf, 213 = bf16 (1, 1)
NEGINF, ONES = 212, 213
P_BASE = 216                   # P[par][r][t] at 216 + 4*(4*par + 2*r + t)


def S(par, r):
    return S_BASE + 32 * par + 16 * r


def P(par, r, t):
    return P_BASE + 4 * (4 * par + 2 * r + t)


def O(r, db):
    i = 4 * r + db
    return f"a[{16 * i}:{16 * i + 15}]"


def Q(r, kk):
    i = 128 + 4 * (8 * r + kk)
    return f"a[{i}:{i + 3}]"


def vr(lo, n):
    return f"v[{lo}:{lo + n - 1}]"


class Block:
    def __init__(self):
        self.lines = []

    def emit(self, s):
        self.lines.append(s)

    def text(self):
        return " \\\n".join('    "' + l + '\\n\\t"' for l in self.lines)


def emit_stage_load(b, u, first, last):
    """Staging load of this wave: chunk u of a K tile (u < 8) or chunk u-8 of a V tile, 16 bytes per
    lane straight into LDS.  s[88:89] / s[90:91] hold the address of the wave's first row of the
    tile, the operands ko0..7 / vo0..7 the lane's byte offset inside chunk u (its row and 16-byte
    piece, plus u chunks of 4 rows), M0 the LDS destination: it is set for the first chunk of a
    tile and stepped by 1 KB right after each load, so that the write and the next use are never
    neighbours."""
    which, base = ("k", 88) if u < 8 else ("v", 90)
    if first or u == 8:
        b.emit(f"s_mov_b32 m0, %[lds{which}]")
        b.emit("s_nop 0")
    b.emit(f"global_load_lds_dwordx4 %[{which}o{u & 7}], s[{base}:{base + 1}]")
    if not last and u != 7:
        b.emit("s_add_u32 m0, m0, 0x400")


def step(p, qk, pv, sm, masked=False, loads=()):
    """One pipeline step of parity p: any of QK(n+1), PV(n-1), SM(n).  `loads` lists the staging
    chunks this wave requests on the way, one behind each of the first pairs of matrix
    instructions."""
    b = Block()
    b.emit("s_waitcnt lgkmcnt(0)")
    half = 1 - p  # both matrix products work on half 1-p of their staged tiles

    # ---- the matrix pairs of this step and their LDS fragment reads
    plan = []  # (kind, index)
    if qk:
        plan += [("k", kk) for kk in range(8)]
    if pv:
        plan += [("v", i) for i in range(8)]

    def frag_read(j):
        kind, i = plan[j]
        buf = FR_BASE + 4 * (j % NBUF)
        if kind == "k":
            b.emit(f"ds_read_b128 {vr(buf, 4)}, %[ka{i}] offset:{half * 32 * ROW}")
            return 1
        t, db = divmod(i, 4)
        off = (db >> 1) * 128 + (32 * half + 16 * t) * ROW
        b.emit(f"ds_read_b64_tr_b16 {vr(buf, 2)}, %[va{db & 1}] offset:{off}")
        b.emit(f"ds_read_b64_tr_b16 {vr(buf + 2, 2)}, %[va{db & 1}] offset:{off + 8 * ROW}")
        return 2

    def mfma(j, r):
        kind, i = plan[j]
        buf = vr(FR_BASE + 4 * (j % NBUF), 4)
        if True:
            if kind == "k":
                d = vr(S(1 - p, r), 16)
                b.emit(f"{MFMA} {d}, {buf}, {Q(r, i)}, {'0' if i == 0 else d}")
            else:
                t, db = divmod(i, 4)
                b.emit(f"{MFMA} {O(r, db)}, {buf}, {vr(P(1 - p, r, t), 4)}, {O(r, db)}")

    # ---- SM(n): 16 items of two scores; item k: row group (k>>2)&1, elements 8*(k>>3)+2*(k&3), +1
    # (step t = 0 of both row groups first).  Items are emitted two at a time.
    def item_pair(k0):
        its = []
        for k in (k0, k0 + 1):
            r = (k >> 2) & 1
            e = 8 * (k >> 3) + 2 * (k & 3)
            its.append((r, e, S(p, r) + e, TMP + 2 * (k - k0)))
        if masked:
            # key offset of element e inside the sub-block, without the lane's 4*hi: the key is
            # visible iff that offset <= d_r
            for (r, e, src, tmp) in its:
                c0 = 8 * (e >> 2) + (e & 3)
                b.emit(f"v_cmp_ge_i32_e64 %[mk0], %[d{r}], {c0}")
                b.emit(f"v_cmp_ge_i32_e64 %[mk1], %[d{r}], {c0 + 1}")
                b.emit("s_nop 0")
                b.emit(f"v_cndmask_b32_e64 v{tmp}, v{NEGINF}, v{src}, %[mk0]")
                b.emit(f"v_cndmask_b32_e64 v{tmp + 1}, v{NEGINF}, v{src + 1}, %[mk1]")
                b.emit(f"v_fma_f32 v{tmp}, v{tmp}, %[scale], -%[ms{r}]")
                b.emit(f"v_fma_f32 v{tmp + 1}, v{tmp + 1}, %[scale], -%[ms{r}]")
        else:
            for (r, e, src, tmp) in its:
                b.emit(f"v_fma_f32 v{tmp}, v{src}, %[scale], -%[ms{r}]")
                b.emit(f"v_fma_f32 v{tmp + 1}, v{src + 1}, %[scale], -%[ms{r}]")
        for (r, e, src, tmp) in its:
            b.emit(f"v_exp_f32_e32 v{tmp}, v{tmp}")
            b.emit(f"v_exp_f32_e32 v{tmp + 1}, v{tmp + 1}")
        b.emit("s_nop 0")
        for (r, e, src, tmp) in its:
            t, j = divmod(e, 8)
            b.emit(f"v_cvt_pk_bf16_f32 v{P(p, r, t) + j // 2}, v{tmp}, v{tmp + 1}")
        for (r, e, src, tmp) in its:
            t, j = divmod(e, 8)
            b.emit(f"v_dot2c_f32_bf16_e32 %[sum{r}], v{P(p, r, t) + j // 2}, v{ONES}")

    def stage_load(j):
        emit_stage_load(b, loads[j], j == 0, j == len(loads) - 1)

    # ---- schedule
    n_pairs = len(plan)
    if sm:
        b.emit("v_mov_b32_e32 %[sum0], 0")
        b.emit("v_mov_b32_e32 %[sum1], 0")
        b.emit(f"v_mov_b32_e32 v{ONES}, 0x3f803f80")
        if masked:
            b.emit(f"v_mov_b32_e32 v{NEGINF}, 0xff800000")
    cnt = {}
    issued = 0
    while issued < min(DIST, n_pairs):
        cnt[issued] = frag_read(issued)
        issued += 1
    # The softmax arithmetic: the first item pair goes before the first matrix instruction
    # (it covers the LDS latency), the rest is dealt out evenly, a few instructions behind every
    # single matrix instruction.  A matrix instruction only shadows what follows it until the
    # next one is due, so two of them back to back would leave the first one's shadow empty.
    stream = []
    if sm:
        item_pair(0)
        main, b.lines = b.lines, stream
        for k in range(1, 8):
            item_pair(2 * k)
        b.lines = main
    n_slots = 2 * n_pairs
    take = [(len(stream) * (q + 1)) // n_slots - (len(stream) * q) // n_slots for q in range(n_slots)] if n_slots else []
    pos = 0
    if not n_slots:
        b.lines += stream
    for j in range(n_pairs):
        outstanding = sum(cnt[m] for m in range(j + 1, issued))
        b.emit(f"s_waitcnt lgkmcnt({outstanding})")
        for r in (0, 1):
            mfma(j, r)
            if r == 0 and issued < n_pairs:
                cnt[issued] = frag_read(issued)
                issued += 1
            if r == 1 and j < len(loads):
                stage_load(j)
            q = 2 * j + r
            b.lines += stream[pos:pos + take[q]]
            pos += take[q]
    if sm:
        # flag = lanes whose sub-block needs a closer look: a sum above 2^8 (or not a number), or a
        # row that had accumulated nothing before (sums are dot-product results: not read by
        # another kind of instruction for three slots)
        b.emit("v_cmp_eq_f32_e64 %[flag], 0, %[l0]")
        b.emit("v_cmp_eq_f32_e64 vcc, 0, %[l1]")
        b.emit("s_or_b64 %[flag], %[flag], vcc")
        b.emit("s_nop 0")
        b.emit("v_cmp_nge_f32_e64 vcc, %[k256], %[sum0]")
        b.emit("s_or_b64 %[flag], %[flag], vcc")
        b.emit("v_cmp_nge_f32_e64 vcc, %[k256], %[sum1]")
        b.emit("s_or_b64 %[flag], %[flag], vcc")
    if qk and not pv:
        # no matrix instructions follow inside the block: let the scores settle, the caller or
        # the next block reads them with ordinary instructions
        b.emit("s_nop 7")
        b.emit("s_nop 7")
    return b


def init_o():
    """O = 0: eight matrix instructions with zero operands write the 128 accumulator registers."""
    b = Block()
    for k in range(4):
        b.emit(f"v_mov_b32_e32 v{TMP + k}, 0")
    b.emit("s_nop 1")
    for i in range(8):
        b.emit(f"{MFMA} a[{16 * i}:{16 * i + 15}], {vr(TMP, 4)}, {vr(TMP, 4)}, 0")
    return b


def load_q():
    """Query fragments straight from global memory into a[128:191]: per row group one address
    (row, 8*hi elements in), fragment kk lies 32*kk bytes further."""
    b = Block()
    for r in range(2):
        for kk in range(8):
            i = 128 + 4 * (8 * r + kk)
            b.emit(f"global_load_dwordx4 a[{i}:{i + 3}], %[qa{r}], off offset:{32 * kk}")
    return b


def rescale():
    """O[r] *= alpha_r."""
    b = Block()
    b.emit("s_nop 7")
    b.emit("s_nop 7")
    for i0 in range(0, 128, 8):
        r = i0 // 64
        for k in range(8):
            b.emit(f"v_accvgpr_read_b32 v{TMP + k}, a{i0 + k}")
        for k in range(8):
            b.emit(f"v_mul_f32_e32 v{TMP + k}, %[alpha{r}], v{TMP + k}")
        for k in range(8):
            b.emit(f"v_accvgpr_write_b32 a{i0 + k}, v{TMP + k}")
    b.emit("s_nop 3")
    return b


def read_o():
    b = Block()
    b.emit("s_nop 7")
    b.emit("s_nop 7")
    b.emit("s_nop 3")
    for i in range(128):
        b.emit(f"v_accvgpr_read_b32 v{i}, a{i}")
    return b


def reglist(prefix, lo, hi):
    return ", ".join(f'"{prefix}{i}"' for i in range(lo, hi))


def main(out_path):
    blocks = {
        # name: step(parity, qk, pv, sm, masked, loads)
        "VS_ASM_QK0": step(1, True, False, False),                 # QK into S[0] (a group's first sub-block)
        "VS_ASM_QK0_LOADS": step(1, True, False, False, loads=range(8)),      # ... requesting a K tile
        "VS_ASM_FIRST": step(0, True, False, True),                # step 0: QK(1), SM(0)
        "VS_ASM_FIRST_LOADS": step(0, True, False, True, loads=range(8, 16)),  # ... requesting a V tile
        "VS_ASM_FIRST_MASKED": step(0, True, False, True, masked=True),
        "VS_ASM_ODD": step(1, True, True, True),                   # step 2t+1 with a next tile
        "VS_ASM_ODD_MASKED": step(1, True, True, True, masked=True),
        "VS_ASM_ODD_LOADS": step(1, True, True, True, loads=range(16)),
        "VS_ASM_ODD_LAST": step(1, False, True, True),             # step 2t+1 of the last tile
        "VS_ASM_ODD_LAST_MASKED": step(1, False, True, True, masked=True),
        "VS_ASM_EVEN": step(0, True, True, True),                  # step 2t+2
        "VS_ASM_EVEN_MASKED": step(0, True, True, True, masked=True),
        "VS_ASM_TAIL": step(0, False, True, False),                # PV of the last sub-block
        "VS_ASM_INIT_O": init_o(),
        "VS_ASM_LOAD_Q": load_q(),
        "VS_ASM_RESCALE": rescale(),
        "VS_ASM_READ_O": read_o(),
    }
    parts = ["// Generated by gen_prefill_asm.py: do not edit.\n"]
    for name, blk in blocks.items():
        parts.append(f"#define {name} \\\n{blk.text()}\n")
    parts += [
        "#define VS_CLOB_ACC " + reglist("a", 0, 192) + "\n",
        "#define VS_CLOB_S " + reglist("v", S_BASE, S_BASE + 64) + "\n",
        "#define VS_CLOB_P " + reglist("v", P_BASE, P_BASE + 32) + "\n",
        "#define VS_CLOB_FRAG " + reglist("v", FR_BASE, FR_BASE + 4 * NBUF) + "\n",
        "#define VS_CLOB_TMP " + reglist("v", TMP, TMP + 8) + "\n",
    ]
    with open(out_path, "w") as f:
        f.write("\n".join(parts))


if __name__ == "__main__":
    here = os.path.dirname(os.path.abspath(__file__))
    main(sys.argv[1] if len(sys.argv) > 1 else os.path.join(here, "vs_prefill_asm.inc"))
