#!/usr/bin/env python3
"""Writes pass_asm_gen.h: the inner loops of the two scoring passes as hand-scheduled inline
assembly for gfx950, as an experiment beside the compiled kernels (d_k = 128, six row blocks of 32
prompt rows, eight waves that share a problem's key blocks).

A wave takes whole 32-key blocks: the keys come straight from memory into the A operands (two
register buffers, the next block requested among the first matrix instructions of the current one),
the prompt-row operand of every matrix instruction comes from LDS through a ring of eight reads that
runs ahead of the matrix instructions, and the vector work of a pair of row blocks (multiply-add,
exp2, sum) is spread over the matrix instructions that follow the pair's own, three instruction
slots behind them.  Pass 1 takes no reference (sums of exp2(s * sc)); pass 2 folds the 16 per-lane
key sums over the row lanes and stores the block's 32 scores.  pass_asm_harness.hip checks both loops
against a CPU reference and times them at the size of the C4 workload.

Environment switches for the stripped variants that show where the time goes: NOLOAD=1 (no key loads),
NOQREAD=1 (no LDS reads: the matrix instructions take stale operands), NOVALU=1 (no vector work),
NOMFMA=1 (no matrix instructions), NOBRANCH=1.  Results of stripped variants are wrong on purpose;
run the harness with the argument `time` then.  FAIR=1 adds a feedback between the two waves of a
SIMD (waves w and w + 4): each publishes the number of blocks it has done in LDS once per block, reads
the other's, and takes the higher issue priority (s_setprio) while it is not ahead; without it the
wave that was launched first wins the arbitration and finishes 15-20 us before the other.

  python pass_asm.py && hipcc --offload-arch=gfx950 -O3 -Xclang -target-feature -Xclang -packed-fp32-ops \
      -o pass_asm_harness pass_asm_harness.hip && ./pass_asm_harness
"""
import sys, os
NOLOAD = os.environ.get('NOLOAD') == '1'
NOVALU = os.environ.get('NOVALU') == '1'
NOMFMA = os.environ.get('NOMFMA') == '1'
NOBRANCH = os.environ.get('NOBRANCH') == '1'
NOQREAD = os.environ.get('NOQREAD') == '1'
FAIR = os.environ.get('FAIR') == '1'

D = 128
KS = D // 16          # k-steps of 16 per 32x32x16 MFMA
DELTA = 3             # vector work lags the matrix work by this many MFMA slots
QSTRIDE = D * 2 + 16  # LDS row stride of the staged prompt rows

QRING = 8            # prompt-row operands are read from LDS this many matrix instructions ahead
NWAVES = 8           # waves that share the key blocks of a problem

class Regs:
    def __init__(self, QB):
        self.QB = QB
        self.NP = QB // 2
        v = 0
        self.kbuf = []
        for b in range(2):
            self.kbuf.append(('v', v)); v += 32
        self.sets = []
        for p in range(max(self.NP, 2)):
            self.sets.append((v, v + 16)); v += 32
        self.QST = v; v += 4 * QRING
        self.U = v; v += 16
        self.T = v; v += 8
        self.NEGL = v; v += QB          # pass 2: -lse of the lane's row in each row block
        self.Z = self.U                 # pass 1: 2 partial sums per row block, in the place of the key sums
        self.W = v; v += 8
        self.X = v; v += 4
        self.Y = v; v += 2
        self.KEEP = v; v += 1
        self.SEND = v; v += 1
        self.ZZ = v; v += 1
        self.TOT = v; v += 1
        self.PW = v; v += 1
        self.PR = v; v += 1
        self.PS = v; v += 1
        self.vtop = v
        assert v <= 246, v
        assert 2 * QB <= 16 and QB <= 8

def r(kind_base, n=4):
    k, b = kind_base
    return f"{k}[{b}:{b + n - 1}]"

def vr(b, n=1):
    return f"v{b}" if n == 1 else f"v[{b}:{b + n - 1}]"

# scalar registers used as temporaries (clobbered)
S_SEQ, S_BLK, S_T0, S_T1, S_BASE, S_SB, S_MASK, S_B1, S_EXEC = 64, 65, 66, 67, 68, 70, 72, 74, 76
S_T2, S_T3 = 78, 79

def load_block(R, buf, seq_off):
    """scalar address of the block `seq + seq_off` of this wave (clamped to a real block) and its 8 loads
    straight into key buffer `buf` (lane (t, h) takes row t, 16-byte pieces 2 s + h)"""
    k, b = R.kbuf[buf]
    L = []
    if seq_off == 0:
        L.append(f"s_mov_b32 s{S_T0}, s{S_SEQ}")
    else:
        L.append(f"s_add_u32 s{S_T0}, s{S_SEQ}, {seq_off}")
    L.append(f"s_mul_i32 s{S_T0}, s{S_T0}, {NWAVES}")
    L.append(f"s_add_u32 s{S_BLK}, s{S_T0}, %[wave]")          # block id = wave + NWAVES * seq
    L.append(f"s_cmp_lt_u32 s{S_BLK}, %[nbtot]")
    L.append(f"s_cselect_b32 s{S_BLK}, s{S_BLK}, %[wave]")      # past the end: the wave's first block again
    L.append(f"s_cmp_lt_u32 s{S_BLK}, %[nbc]")                  # scc = 1: a block of cache rows
    L.append(f"s_cselect_b32 s{S_BASE}, %[kc_lo], %[kk_lo]")
    L.append(f"s_cselect_b32 s{S_BASE + 1}, %[kc_hi], %[kk_hi]")
    L.append(f"s_sub_u32 s{S_T1}, s{S_BLK}, %[nbc]")
    L.append(f"s_cselect_b32 s{S_T0}, s{S_BLK}, s{S_T1}")       # block index inside its region
    L.append(f"s_mov_b32 s{S_T1}, 0")
    L.append(f"s_lshl_b64 s[{S_T0}:{S_T1}], s[{S_T0}:{S_T1}], 13")   # * 32 rows * 256 bytes
    L.append(f"s_add_u32 s{S_BASE}, s{S_BASE}, s{S_T0}")
    L.append(f"s_addc_u32 s{S_BASE + 1}, s{S_BASE + 1}, s{S_T1}")
    for s_ in range(KS):
        L.append(f"global_load_dwordx4 v[{b + 4 * s_}:{b + 4 * s_ + 3}], %[rowoff], s[{S_BASE}:{S_BASE + 1}] offset:{32 * s_}")
    return L

def q_read(R, n, q, s_):
    """the prompt-row operand of the matrix instruction number n (row block q, k-step s) into its ring slot"""
    slot = R.QST + 4 * (n % QRING)
    return f"ds_read_b128 v[{slot}:{slot + 3}], %[qaddr] offset:{q * 32 * QSTRIDE + 32 * s_}"

def mfma_seq(R):
    """(row block, k-step, accumulator, first?) of the matrix instructions of one key block, in issue order"""
    out = []
    for p in range(R.NP):
        s0, s1 = R.sets[p]
        for s_ in range(KS):
            for ch, acc in ((0, s0), (1, s1)):
                out.append((2 * p + ch, s_, acc, s_ == 0))
    return out

def mfma_list(R, buf):
    """the matrix instructions of one key block, each behind the wait for its prompt-row operand and
    followed by the LDS read of the operand QRING instructions further on (the ring runs on across blocks)"""
    out = []
    k, b = R.kbuf[buf]
    seq = mfma_seq(R)
    n_all = len(seq)
    for n, (q, s_, acc, first) in enumerate(seq):
        c = "0" if first else vr(acc, 16)
        slot = R.QST + 4 * (n % QRING)
        m = f"v_mfma_f32_32x32x16_bf16 {vr(acc, 16)}, v[{b + 4 * s_}:{b + 4 * s_ + 3}], v[{slot}:{slot + 3}], {c}"
        qn, sn, _, _ = seq[(n + QRING) % n_all]
        if NOQREAD:
            out.append([m])
        else:
            out.append([f"s_waitcnt lgkmcnt({QRING - 1})", m, q_read(R, n + QRING, qn, sn)])
    return out

def logit_stream(R, mode, p):
    """vector work of pair p of one key block (software pipelined inside the pair: multiply-add of
    logit n + 2, exponential of logit n + 1, sum of logit n).  mode 2: per-key sums; mode 1: per-row sums."""
    ops = []
    logits = []
    for ch in range(2):
        q = 2 * p + ch
        acc = R.sets[p][ch]
        for v in range(16):
            logits.append((q, acc + v, v))
    n = len(logits)
    for step in range(n + 2):
        if step < n:
            q, a, v = logits[step]
            if mode == 2:
                ops.append(f"v_fma_f32 v{R.T + step % 8}, v{a}, %[sc], v{R.NEGL + q}")
            else:
                ops.append(f"v_mul_f32 v{R.T + step % 8}, %[sc], v{a}")
        if 1 <= step <= n:
            i = step - 1
            q, a, v = logits[i]
            if mode == 2 and q == 0:
                ops.append(f"v_exp_f32 v{R.U + v}, v{R.T + i % 8}")
            else:
                ops.append(f"v_exp_f32 v{R.T + i % 8}, v{R.T + i % 8}")
        if step >= 2:
            i = step - 2
            q, a, v = logits[i]
            if mode == 2:
                if q != 0:
                    ops.append(f"v_add_f32 v{R.U + v}, v{R.U + v}, v{R.T + i % 8}")
            else:
                z = R.Z + q * 2 + (v % 2)
                ops.append(f"v_add_f32 v{z}, v{z}, v{R.T + i % 8}")
    return ops

def fold_store(R):
    """sum of each of the 16 per-lane key sums over the 32 row lanes of a lane half, then the store of
    the block whose sequence number is seq - 1 (skipped when there is no such block)"""
    U, W, X, Y = R.U, R.W, R.X, R.Y
    L = ["s_nop 1"]
    for i in range(8):
        L.append(f"v_permlane16_swap_b32 v{U + i}, v{U + i + 8}")
    L.append("s_nop 1")
    for i in range(8):
        L.append(f"v_add_f32 v{W + i}, v{U + i}, v{U + i + 8}")
    L.append("s_nop 1")
    for i in range(4):
        L.append(f"v_add_f32_dpp v{X + i}, v{W + i}, v{W + i} row_ror:8 row_mask:0xf bank_mask:0x3")
    for i in range(4):
        L.append(f"v_add_f32_dpp v{X + i}, v{W + i + 4}, v{W + i + 4} row_ror:8 row_mask:0xf bank_mask:0xc")
    L.append("s_nop 1")
    for i in range(2):
        L.append(f"v_add_f32_dpp v{Y + i}, v{X + i}, v{X + i} row_half_mirror row_mask:0xf bank_mask:0x5")
    for i in range(2):
        L.append(f"v_add_f32_dpp v{Y + i}, v{X + i + 2}, v{X + i + 2} row_half_mirror row_mask:0xf bank_mask:0xa")
    L.append(f"v_cndmask_b32 v{R.SEND}, v{Y + 1}, v{Y}, s[{S_B1}:{S_B1 + 1}]")
    L.append(f"v_cndmask_b32 v{R.KEEP}, v{Y}, v{Y + 1}, s[{S_B1}:{S_B1 + 1}]")
    L.append("s_nop 1")
    L.append(f"v_add_f32_dpp v{R.ZZ}, v{R.SEND}, v{R.KEEP} quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf")
    L.append("s_nop 1")
    L.append(f"v_add_f32_dpp v{R.TOT}, v{R.ZZ}, v{R.ZZ} quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf")
    # the block before the current one: seq - 1 (seq is the section's own block)
    L.append(("store",))
    return L

def store_code(R, label):
    L = []
    L.append(f"s_sub_u32 s{S_T2}, s{S_SEQ}, 1")
    L.append(f"s_mul_i32 s{S_T2}, s{S_T2}, {NWAVES}")
    L.append(f"s_add_u32 s{S_T2}, s{S_T2}, %[wave]")
    L.append(f"s_cmp_ge_u32 s{S_T2}, %[nbtot]")
    L.append(f"s_cbranch_scc1 {label}f")
    L.append(f"s_cmp_lt_u32 s{S_T2}, %[nbc]")
    L.append(f"s_sub_u32 s{S_T3}, s{S_T2}, %[nbc]")
    L.append(f"s_lshl_b32 s{S_T3}, s{S_T3}, 5")
    L.append(f"s_add_u32 s{S_T3}, s{S_T3}, %[c]")
    L.append(f"s_lshl_b32 s{S_T2}, s{S_T2}, 5")
    L.append(f"s_cselect_b32 s{S_T2}, s{S_T2}, s{S_T3}")       # first key of the block among the candidates
    L.append(f"s_mov_b32 s{S_T3}, 0")
    L.append(f"s_lshl_b64 s[{S_T2}:{S_T3}], s[{S_T2}:{S_T3}], 2")
    L.append(f"s_add_u32 s{S_SB}, %[sp_lo], s{S_T2}")
    L.append(f"s_addc_u32 s{S_SB + 1}, %[sp_hi], s{S_T3}")
    L.append(f"s_mov_b32 exec_lo, 0x55555555")
    L.append(f"s_mov_b32 exec_hi, 0x55555555")
    L.append("s_nop 4")
    L.append(f"global_store_dword %[stoff], v{R.TOT}, s[{S_SB}:{S_SB + 1}]")
    L.append("s_mov_b64 exec, -1")
    L.append("s_nop 4")
    L.append(f"{label}:")
    return L

def spread(ops, lo, hi):
    """ops over stream slots [lo, hi), evenly, in order"""
    out = {}
    n = len(ops)
    w = hi - lo
    for j in range(w):
        out[lo + j] = ops[j * n // w:(j + 1) * n // w]
    return out

def stream_slots(R, mode):
    """vector work of one key block by stream slot: slot j runs in slot j + START of the block's own
    section (of the next section where that is past its end).  The vector work of pair p may start
    DELTA slots after the pair's last matrix instruction, i.e. at stream slot 16 p."""
    slots = {}
    for p in range(R.NP):
        part = logit_stream(R, mode, p)
        if p == R.NP - 1 and mode == 2:
            part = part + fold_store(R)
        slots.update(spread(part, 16 * p, 16 * p + 16))
    return slots

START = 16 + DELTA

def section(R, mode, buf, sec, tag):
    """one key block: its matrix instructions with the loads of the next block among the first of them,
    and the vector work whose slots fall into this section (the end of the previous block's, the
    beginning of its own)"""
    L = []
    L.append("s_waitcnt vmcnt(0)")          # this block's keys (requested during the section before)
    if FAIR:
        L.append(f"v_mov_b32 v{R.PW}, s{S_SEQ}")
        L.append(f"ds_write_b32 %[paddr], v{R.PW}")
        L.append(f"ds_read_b32 v{R.PR}, v{R.PS}")
    loads = [] if NOLOAD else load_block(R, (buf + 1) % 2, 1)
    scalar = [x for x in loads if not x.startswith("global_load")]
    vmem = [x for x in loads if x.startswith("global_load")]
    L += scalar
    # vcc = 0 in the section a wave starts with: there is no previous block whose vector work could run
    L.append(f"s_cmp_lg_u32 s{S_SEQ}, 0")
    L.append("s_cselect_b64 vcc, -1, 0")
    M = mfma_list(R, buf)
    nslots = len(M)
    S = stream_slots(R, mode)
    for k in range(nslots):
        if not NOMFMA:
            L += M[k]
        if k < len(vmem):
            L.append(vmem[k])
        prev = k < START
        ops = S[k - START + nslots] if prev else S[k - START]
        if NOVALU:
            ops = [o for o in ops if isinstance(o, tuple)]
        if prev and ops and not NOBRANCH:
            L.append(f"s_cbranch_vccz {tag}{sec}{k:02d}f")
        for op in ops:
            if isinstance(op, tuple):
                assert op[0] == "store" and prev
                L += store_code(R, f"{tag}{sec}9")
            else:
                L.append(op)
        if prev and ops and not NOBRANCH:
            L.append(f"{tag}{sec}{k:02d}:")
    if FAIR:
        # whoever of the SIMD's two waves is behind takes the higher priority for the next block
        L.append(f"v_readfirstlane_b32 s{S_T2}, v{R.PR}")
        L.append(f"s_cmp_le_u32 s{S_SEQ}, s{S_T2}")
        L.append(f"s_cbranch_scc0 {tag}{sec}97f")
        L.append("s_setprio 3")
        L.append(f"s_branch {tag}{sec}98f")
        L.append(f"{tag}{sec}97:")
        L.append("s_setprio 0")
        L.append(f"{tag}{sec}98:")
    L.append(f"s_add_u32 s{S_SEQ}, s{S_SEQ}, 1")
    return L

def epilogue(R, mode, tag):
    """what is left of the last block's stream after the loop (seq points one past it)"""
    nslots = 16 * R.NP
    S = stream_slots(R, mode)
    L = []
    for j in range(nslots - START, nslots):
        for op in S[j]:
            if isinstance(op, tuple):
                assert op[0] == "store"
                L += store_code(R, f"{tag}89")
            else:
                L.append(op)
    return L

def emit(QB, mode):
    R = Regs(QB)
    tag = f"{mode}{QB}"
    L = []
    L.append("s_waitcnt vmcnt(0) lgkmcnt(0)")
    if mode == 2:
        for q in range(QB):
            L.append(f"ds_read_b32 v{R.NEGL + q}, %[laddr] offset:{q * 128}")
    L.append(f"s_mov_b32 s{S_SEQ}, 0")
    if FAIR:
        L.append(f"v_xor_b32 v{R.PS}, 16, %[paddr]")
    L.append(f"s_mov_b32 s{S_B1}, 0xcccccccc")
    L.append(f"s_mov_b32 s{S_B1 + 1}, 0xcccccccc")
    # the first prompt-row operands into the ring
    seq = mfma_seq(R)
    for n in range(QRING):
        q, s_, _, _ = seq[n]
        L.append(q_read(R, n, q, s_))
    for (s0, s1) in R.sets:
        for v in range(32):
            L.append(f"v_mov_b32 v{s0 + v}, 0")
    for v in range(16):
        L.append(f"v_mov_b32 v{R.U + v}, 0")
    for v in range(8):
        L.append(f"v_mov_b32 v{R.T + v}, 0")
    # A wave with an odd number of blocks starts with the second section of the loop body (whose
    # keys are in the second buffer), one with an even number with the first: the body holds two
    # sections and ends when the last block is done.
    L.append("s_bitcmp1_b32 %[nw], 0")
    L.append(f"s_cbranch_scc1 {tag}7f")
    L += load_block(R, 0, 0)
    L.append(f"s_branch {tag}1f")
    L.append(f"{tag}7:")
    L += load_block(R, 1, 0)
    L.append(f"s_branch {tag}2f")
    L.append(f"{tag}1:")
    L += section(R, mode, 0, 0, tag)
    L.append(f"{tag}2:")
    L += section(R, mode, 1, 1, tag)
    L.append(f"s_cmp_lt_u32 s{S_SEQ}, %[nw]")
    L.append(f"s_cbranch_scc1 {tag}1b")
    L += epilogue(R, mode, tag)
    if mode == 1:
        for q in range(QB):
            z = R.Z + 2 * q
            L.append(f"v_add_f32 v{z}, v{z}, v{z + 1}")
        for q in range(QB):
            L.append(f"ds_write_b32 %[zaddr], v{R.Z + 2 * q} offset:{q * 256}")
    if FAIR:
        L.append("s_setprio 0")
    L.append("s_waitcnt vmcnt(0) lgkmcnt(0)")
    return R, L

def function(QB, mode):
    R, L = emit(QB, mode)
    name = f"pass{mode}_asm_qb{QB}"
    body = "\n".join(f'      "{x}\\n\\t"' for x in L)
    vclob = ",".join(f'"v{i}"' for i in range(R.vtop))
    sclob = ",".join(f'"s{i}"' for i in range(64, 80))
    if mode == 2:
        sig = ("const void* kcache, const void* kchunk, float* scores, int c, int nbc, int nbtot, int wave, int nw, "
               "float sc, unsigned qaddr, unsigned laddr, unsigned rowoff, unsigned stoff, unsigned paddr")
        extra_in = ', [sp_lo] "s"(sp_lo), [sp_hi] "s"(sp_hi), [c] "s"(c), [stoff] "v"(stoff)'
        pre = ("  const unsigned sp_lo = U((unsigned)(unsigned long long)scores), sp_hi = U((unsigned)((unsigned long long)scores >> 32));\n"
               "  c = (int)U(c);\n")
    else:
        sig = ("const void* kcache, const void* kchunk, int nbc, int nbtot, int wave, int nw, "
               "float sc, unsigned qaddr, unsigned laddr, unsigned rowoff, unsigned zaddr, unsigned paddr")
        extra_in = ', [zaddr] "v"(zaddr)'
        pre = ""
    return f'''
// {"per-key sums of exp2(s * sc - lse[row])" if mode == 2 else "per-row sums of exp2(s * sc)"} over the wave's full 32-key blocks
// (block ids wave, wave + {NWAVES}, ... below nbtot; ids below nbc are blocks of cache rows, the others of
// chunk rows); nw = number of such blocks, at least 1.  {R.vtop} VGPRs.
__device__ __forceinline__ void {name}({sig}) {{
  // (scalar operands: made uniform explicitly, or the compiler may hand the asm a vector register)
  const auto U = [](unsigned x) {{ return (unsigned)__builtin_amdgcn_readfirstlane((int)x); }};
  const unsigned kc_lo = U((unsigned)(unsigned long long)kcache), kc_hi = U((unsigned)((unsigned long long)kcache >> 32));
  const unsigned kk_lo = U((unsigned)(unsigned long long)kchunk), kk_hi = U((unsigned)((unsigned long long)kchunk >> 32));
  nbc = (int)U(nbc); nbtot = (int)U(nbtot); wave = (int)U(wave); nw = (int)U(nw);
  sc = __builtin_bit_cast(float, U(__builtin_bit_cast(unsigned, sc)));
{pre}  asm volatile(
{body}
      :
      : [kc_lo] "s"(kc_lo), [kc_hi] "s"(kc_hi), [kk_lo] "s"(kk_lo), [kk_hi] "s"(kk_hi), [nbc] "s"(nbc),
        [nbtot] "s"(nbtot), [wave] "s"(wave), [nw] "s"(nw), [sc] "s"(sc), [qaddr] "v"(qaddr),
        [laddr] "v"(laddr), [rowoff] "v"(rowoff), [paddr] "v"(paddr){extra_in}
      : {vclob},
        {sclob}, "scc", "vcc", "memory");
}}
'''

if __name__ == "__main__":
    out = sys.argv[1] if len(sys.argv) > 1 else os.path.join(os.path.dirname(os.path.abspath(__file__)), "pass_asm_gen.h")
    qbs = [6]
    text = "// written by pass_asm.py - do not edit\n#pragma once\n"
    for QB in qbs:
        for mode in (1, 2):
            text += function(QB, mode)
    open(out, "w").write(text)
    print("wrote", out)
