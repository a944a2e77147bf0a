#!/usr/bin/env python3
"""Writes mttkrp_rows_pipe.inc: the software-pipelined inner loops of the second
schedule (mttkrp_rowsum_kernel, contraction over mode 0) as inline assembly, one
per instantiation (data type, column blocks CB of the column space, output column
blocks JB).

Why assembly: as compiled from plain HIP, the ring of operand sets of that kernel
waits for all outstanding loads at the top of every pass (the compiler's waits
are conservative across the loop's back edge), so a wavefront never overlaps its
own loads with its own MFMAs.  The generated loop keeps D steps of loads in flight
while the MFMAs of an earlier step run, as gen_pipe.py does for the streaming
kernel; the structure (ring of D + 1 operand sets at the top of the register
budget, exit check per step, one drain tail per ring position, waits that name how
many younger loads may be outstanding) is the same.

One step = 16 rows of mode 0: for each of the CB column blocks the lane's four
tensor rows 4 kq .. 4 kq + 3 of its column (fp32: one 16-byte load; fp64: see
below), for each of the four rows t
the lane's JB entries of that row of A_0 (one load per chunk of the wide column
layout of mttkrp.hip, up to four), and 4 * CB * JB 16x16x4 MFMAs: MFMA (t, cb, jb) takes
row t of column block cb and of output column block jb.  The tensor pointers (one
per column block, per lane) advance by 16 rows, the byte offsets into A_0 (per
lane, relative to four wave-uniform row pointers) by 16 rows of A_0.

fp64 tensor loads.  A lane needs 32 bytes of its column's 128-byte line, and the
MFMA layout gives a column only four lanes, so no single load can read a whole line
into place; two loads that each read half of every line make the second depend on
the line staying cached, which fails when the 16 columns lie a large power of two
apart and evict each other from one cache set.  Instead the two lanes of an
even/odd column pair (same kq) work together: load 0 reads the even column's line
with the pair's eight lanes (lane e = 0, 1 of the pair takes 16-byte piece 2 kq + e),
load 1 the odd column's line likewise, so every load reads whole lines of eight
columns; then the two lanes exchange, within the wavefront (one DPP move per
register), the pieces that belong to the other's column.

Run by build.py before hipcc on every build; the output is a build product and is
not kept under version control.
"""
import os

D_MAX = 3
OTHERS = {2: 40, 1: 44}      # registers the rest of the kernel keeps live across a run (fp64, fp32)
X_FLAGS = ""                 # cache policy of the tensor loads (plain: cache-bypassing flags measured slower)
TILES = [(1, 1), (1, 2), (1, 3), (1, 4), (1, 5), (1, 6), (1, 7), (1, 8),
         (2, 1), (2, 2), (2, 3), (2, 4), (3, 1), (3, 2), (4, 1), (4, 2)]


class Inst:
    def __init__(self, w, cb, jb):
        self.w, self.cb, self.jb = w, cb, jb            # w: registers per value (2 = fp64, 1 = fp32)
        self.xregs = cb * 4 * w
        self.brow = jb * w + ((jb * w) & 1)             # registers per row of A_0 entries (register tuples start even)
        self.bregs = 4 * self.brow
        self.set = self.xregs + self.bregs
        self.acc = cb * jb * 4 * w
        g = 16 // (4 * w)                               # values per 16-byte load
        self.chunks = [min(g, jb - g * ch) for ch in range((jb + g - 1) // g)]   # blocks per chunk of output columns
        self.g = g
        self.xloads = w                                 # load instructions per column block
        self.swz = w == 2                               # fp64: whole-line loads by column pairs + exchange
        self.loads = cb * self.xloads + 4 * len(self.chunks)
        self.pick()

    def ring(self, d):
        return self.set * (d + 1) + (4 if self.w == 2 else 0)     # fp64: four temporaries of the exchange

    def pick(self):
        # the most wavefronts per SIMD for which at least two steps in flight fit, else one step at two wavefronts
        self.budget = 0
        for d_min in (2, 1):
            for budget, waves in ((128, 4), (168, 3), (256, 2)):
                for d in range(D_MAX, d_min - 1, -1):
                    if d * self.loads > 63:
                        continue
                    if self.acc + OTHERS[self.w] + self.ring(d) <= budget:
                        self.budget, self.waves, self.d = budget, waves, d
                        self.t0 = budget - self.ring(d)
                        self.t0 -= self.t0 & 1
                        return

    def tag(self):
        return "%s%d%d" % ("d" if self.w == 2 else "f", self.cb, self.jb)

    def ctype(self):
        return "double" if self.w == 2 else "float"

    # --- registers
    @staticmethod
    def reg(base, n):
        return "v%d" % base if n == 1 else "v[%d:%d]" % (base, base + n - 1)

    def base(self, s):
        return self.t0 + self.set * s

    def xval(self, s, c, t):
        return self.reg(self.base(s) + (c * 4 + t) * self.w, self.w)

    def bval(self, s, t, j):
        return self.reg(self.base(s) + self.xregs + t * self.brow + j * self.w, self.w)

    def last_reg(self):
        return self.t0 + self.ring(self.d) - 1

    @property
    def tmp(self):
        return self.t0 + self.set * (self.d + 1)

    # --- code
    def issue(self, s):
        o = []
        width = {1: "dword", 2: "dwordx2", 3: "dwordx3", 4: "dwordx4"}
        for c in range(self.cb):
            if self.swz:
                for h in range(2):      # h = 0: the pair's even column, h = 1: its odd column
                    o.append("global_load_dwordx4 %s, %%[x%d%s], off%s" % (
                        self.reg(self.base(s) + c * 8 + 4 * h, 4), c, "ab"[h], X_FLAGS))
            else:
                o.append("global_load_dwordx4 %s, %%[x%d], off%s" % (self.reg(self.base(s) + c * 4, 4), c, X_FLAGS))
        for t in range(4):
            for ch, n in enumerate(self.chunks):
                o.append("global_load_%s %s, %%[bo%d], %%[bb%d]" % (
                    width[n * self.w],
                    self.reg(self.base(s) + self.xregs + t * self.brow + ch * self.g * self.w, n * self.w), ch, t))
        for c in range(self.cb):
            for nm in (["x%da" % c, "x%db" % c] if self.swz else ["x%d" % c]):
                o.append("v_lshl_add_u64 %%[%s], %%[%s], 0, %%[xs]" % (nm, nm))
        for ch in range(len(self.chunks)):
            o.append("v_add_u32 %%[bo%d], %%[bs], %%[bo%d]" % (ch, ch))
        return o

    def consume(self, s, wait):
        mfma = "v_mfma_f64_16x16x4_f64" if self.w == 2 else "v_mfma_f32_16x16x4_f32"
        o = ["s_waitcnt vmcnt(%d)" % wait]
        if self.swz:
            # vcc = odd lanes (e = 1).  Per register r of the two loads H0 (even column), H1 (odd
            # column): send what belongs to the partner (e = 0 sends H1, e = 1 sends H0), swap it
            # between the two lanes, then H0 := piece 2 kq (rows 4 kq, 4 kq + 1) and H1 := piece
            # 2 kq + 1 (rows 4 kq + 2, 4 kq + 3) of the lane's own column.
            for c in range(self.cb):
                h0 = self.base(s) + c * 8
                h1 = h0 + 4
                for r in range(4):
                    o.append("v_cndmask_b32 v%d, v%d, v%d, vcc" % (self.tmp + r, h1 + r, h0 + r))
                o.append("s_nop 1")
                for r in range(4):
                    o.append("v_mov_b32_dpp v%d, v%d quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" % (
                        self.tmp + r, self.tmp + r))
                o.append("s_nop 1")
                for r in range(4):
                    o.append("v_cndmask_b32 v%d, v%d, v%d, vcc" % (h0 + r, h0 + r, self.tmp + r))
                    o.append("v_cndmask_b32 v%d, v%d, v%d, vcc" % (h1 + r, self.tmp + r, h1 + r))
            o.append("s_nop 1")
        for t in range(4):
            for c in range(self.cb):
                for j in range(self.jb):
                    a = "%%[a%d%d]" % (c, j)
                    o.append("%s %s, %s, %s, %s" % (mfma, a, self.xval(s, c, t), self.bval(s, t, j), a))
        return o

    def block(self):
        d, s_n, l = self.d, self.d + 1, self.loads
        o = ["s_nop 4"]
        if self.swz:
            o = ["s_mov_b32 vcc_lo, 0xaaaaaaaa", "s_mov_b32 vcc_hi, 0xaaaaaaaa", "s_nop 4"]
        for k in range(d):
            o += self.issue(k)
        o.append("1:")
        for u in range(s_n):
            o.append("s_cmp_eq_u32 %[n], 0")
            o.append("s_cbranch_scc1 %df" % (10 + u))
            o += self.issue((u + d) % s_n)
            o.append("s_sub_u32 %[n], %[n], 1")
            o += self.consume(u, d * l)
        o.append("s_branch 1b")
        for u in range(s_n):
            o.append("%d:" % (10 + u))
            for k in range(d):
                o += self.consume((u + k) % s_n, (d - 1 - k) * l)
            if u < s_n - 1:
                o.append("s_branch 9f")
        o.append("9:")
        o += ["s_nop 7", "s_nop 7", "s_nop 7"]
        return o

    def emit(self):
        t = self.tag().upper()
        c = self.ctype()
        out = "// %s: CB = %d, JB = %d; %d steps in flight, ring of %d sets in v[%d:%d], %d wavefronts per SIMD\n" % (
            c, self.cb, self.jb, self.d, self.d + 1, self.t0, self.last_reg(), self.waves)
        out += "#define MTTKRP_ROWS_PIPE_%s_ASM \\\n" % t
        out += " \\\n".join('    "%s\\n"' % line for line in self.block()) + "\n"
        clob = ", ".join('"v%d"' % v for v in range(self.t0, self.last_reg() + 1))
        accs = ", ".join('[a%d%d] "+v"(acc[%d][%d])' % (a, j, a, j) for a in range(self.cb) for j in range(self.jb))
        if self.swz:
            xops = ", ".join('[x%da] "+v"(xq[%d]), [x%db] "+v"(xq[%d])' % (a, 2 * a, a, 2 * a + 1) for a in range(self.cb))
        else:
            xops = ", ".join('[x%d] "+v"(xq[%d])' % (a, a) for a in range(self.cb))
        outs = xops + ", " + \
               ", ".join('[bo%d] "+v"(bo[%d])' % (ch, ch) for ch in range(len(self.chunks))) + ', [n] "+s"(n_more), ' + accs
        ins = '[xs] "s"(x_step_bytes), [bs] "s"(b_step_bytes), ' + \
              ", ".join('[bb%d] "s"(bb[%d])' % (r, r) for r in range(4))
        out += "template <> struct RowsPipe<%s, %d, %d> {\n" % (c, self.cb, self.jb)
        out += "    static constexpr bool value = true;\n"
        out += "    static constexpr int depth = %d;\n    static constexpr int waves = %d;\n" % (self.d, self.waves)
        out += "    static constexpr int xptrs = %d;         // tensor pointers per lane: one per column block, or two (column pair)\n" % (
            self.cb * (2 if self.swz else 1))
        out += "    static __device__ __forceinline__ void run(typename Mfma<%s>::acc_t (&acc)[%d][%d], const %s* (&xq)[%d],\n" % (
            c, self.cb, self.jb, c, self.cb * (2 if self.swz else 1))
        out += "                                               int64_t x_step_bytes, const %s* const (&bb)[4], uint32_t (&bo)[%d],\n" % (
            c, len(self.chunks))
        out += "                                               uint32_t b_step_bytes, int n_more)\n    {\n"
        out += "        asm volatile(MTTKRP_ROWS_PIPE_%s_ASM : %s : %s : %s, \"scc\", %s\"memory\");\n" % (
            t, outs, ins, clob, '\"vcc\", ' if self.swz else "")
        out += "    }\n};\n\n"
        return out


def main(path=None):
    """Writes the include file (next to this script unless a path is given) and returns its path."""
    insts = [Inst(w, cb, jb) for w in (2, 1) for cb, jb in TILES]
    insts = [i for i in insts if i.budget]
    out = "// Generated by gen_rows_pipe.py; do not edit.\n"
    out += "// Primary template: no pipelined run for an instantiation (the kernel then uses its plain loop).\n"
    out += "template <typename T, int CB, int JB> struct RowsPipe {\n"
    out += "    static constexpr bool value = false;\n    static constexpr int depth = 1 << 30;\n"
    out += "    static constexpr int waves = 0;\n    static constexpr int xptrs = CB;\n"
    out += "    static __device__ __forceinline__ void run(typename Mfma<T>::acc_t (&)[CB][JB], const T* (&)[CB], int64_t,\n"
    out += "                                               const T* const (&)[4], uint32_t (&)[(JB * (int)sizeof(T) + 15) / 16], uint32_t, int)\n    {\n    }\n};\n\n"
    for i in insts:
        out += i.emit()
    if path is None:
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "mttkrp_rows_pipe.inc")
    with open(path, "w") as f:
        f.write(out)
    for i in insts:
        print("%s: acc %3d, set %2d, depth %d, budget %d (%d waves), ring v[%d:%d], loads/step %d" % (
            i.tag(), i.acc, i.set, i.d, i.budget, i.waves, i.t0, i.last_reg(), i.loads))
    return path


if __name__ == "__main__":
    print(main())
