#!/usr/bin/env python3
"""Writes mttkrp_pipe.inc: the software-pipelined inner loops of the streaming
kernel as inline assembly, one per instantiation (data type, row blocks RB,
column blocks JB) and load flavour (non-temporal or not, fp64 only).

Why assembly: the compiler places its waits for outstanding loads conservatively
around control flow, which keeps a wavefront from overlapping its own loads with
its own MFMAs.  The generated loop keeps D steps of loads in flight while the
MFMAs of an earlier step run.

One step = four tensor columns: the X loads of the tile's RB row blocks, the
loads of the inner factor's entries for the JB column blocks (both in the lane
layout the kernel defines: `Lay` / `LayRows` in mttkrp.hip), JB multiplies by
the sweep weight and RB * JB 16x16x4 MFMAs.  A run covers any n >= D consecutive
unmasked steps of one sweep: the X pointer and the factor offsets advance by
constant strides.  Operand sets live in a ring of S = D + 1 register sets at
fixed registers at the top of the wavefront's register budget (declared as
clobbers); the loads of step t go to set t mod S; every wait names how many
younger loads may still be outstanding (loads return in issue order).

Structure of a run: D steps are issued up front; then every pass through a ring
position checks whether steps are left, issues one more and consumes the oldest;
when none are left, the D steps in flight are consumed with waits that shrink
to 0 (one copy of that tail per ring position, because the registers differ).

Per instantiation the script picks the register budget (128 / 168 / 256
registers = 4 / 3 / 2 wavefronts per SIMD) and the depth D: the most
wavefronts for which accumulators + ring + an allowance for everything else the
kernel keeps live still fit, with 3 <= D <= 5.

Run by build.py before hipcc on every build; the output is a build product and is
not kept under version control.
"""
import os

D_MAX = 5
D_MIN = 3
OTHERS = {2: 60, 1: 56}      # registers the rest of the kernel keeps live across a run (fp64, fp32)


def even(n):
    return n + (n & 1)


class Inst:
    def __init__(self, w, rb, jb):
        self.w, self.rb, self.jb = w, rb, jb            # w: registers per value (2 = fp64, 1 = fp32)
        self.xregs = even(rb * w)
        self.bregs = even(jb * w)
        self.set = self.xregs + self.bregs
        self.bc = even(jb * w)
        self.acc = rb * jb * 4 * w
        # loads of one step: (destination offset in the set, registers, which pointer, byte offset)
        self.xloads = []
        if w == 2:
            if rb in (2, 4):                             # one 8-byte load per row block
                self.xloads = [(2 * r, 2, "xq", 128 * r) for r in range(rb)]
            elif rb == 1:
                self.xloads = [(0, 2, "xq", 0)]
            else:                                        # rb == 3: rows 2m, 2m+1 then row 32 + m
                self.xloads = [(0, 4, "xq", 0), (4, 2, "xq1", 0)]
            g = 2
        else:
            self.xloads = [(0, rb, "xq", 0)]
            g = 4
        n0 = min(jb, g)
        n1 = jb - n0
        self.bloads = [(0, n0 * w, "bo0")]
        if n1:
            self.bloads.append((n0 * w, n1 * w, "bo1"))
        self.two_x = any(p == "xq1" for _, _, p, _ in self.xloads)
        self.two_b = n1 > 0
        self.loads = len(self.xloads) + len(self.bloads)
        self.pick()

    def ring(self, d):
        return self.set * (d + 1) + self.bc

    def pick(self):
        for budget, waves in ((128, 4), (168, 3), (256, 2)):
            for d in range(D_MAX, D_MIN - 1, -1):
                if d * self.loads > 63:
                    continue
                if self.acc + OTHERS[self.w] + self.ring(d) <= budget:
                    self.budget, self.waves, self.d = budget, waves, d
                    self.t0 = budget - self.ring(d)
                    self.t0 -= self.t0 & 1
                    return
        self.budget = 0      # nothing fits: no pipelined run for this instantiation

    def tag(self):
        return "%s%d%d" % ("d" if self.w == 2 else "f", self.rb, self.jb)

    def ctype(self):
        return "double" if self.w == 2 else "float"

    # --- registers
    def reg(self, base, n):
        return "v%d" % base if n == 1 else "v[%d:%d]" % (base, base + n - 1)

    def xbase(self, s):
        return self.t0 + self.set * s

    def xval(self, s, r):
        return self.reg(self.xbase(s) + r * self.w, self.w)

    def bval(self, s, j):
        return self.reg(self.xbase(s) + self.xregs + j * self.w, self.w)

    def bcval(self, j):
        return self.reg(self.t0 + self.set * (self.d + 1) + j * self.w, self.w)

    def last_reg(self):
        return self.t0 + self.ring(self.d) - 1

    # --- code
    def issue(self, s, nt):
        o = []
        width = {1: "dword", 2: "dwordx2", 3: "dwordx3", 4: "dwordx4"}
        for off, n, ptr, byte in self.xloads:
            o.append("global_load_%s %s, %%[%s], off%s%s" % (
                width[n], self.reg(self.xbase(s) + off, n), ptr, " offset:%d" % byte if byte else "", nt))
        for off, n, ptr in self.bloads:
            o.append("global_load_%s %s, %%[%s], %%[bb]" % (width[n], self.reg(self.xbase(s) + self.xregs + off, n), ptr))
        o.append("v_lshl_add_u64 %[xq], %[xq], 0, %[xs]")
        if self.two_x:
            o.append("v_lshl_add_u64 %[xq1], %[xq1], 0, %[xs]")
        o.append("v_add_u32 %[bo0], %[bs], %[bo0]")
        if self.two_b:
            o.append("v_add_u32 %[bo1], %[bs], %[bo1]")
        return o

    def consume(self, s, wait):
        mul = "v_mul_f64" if self.w == 2 else "v_mul_f32"
        mfma = "v_mfma_f64_16x16x4_f64" if self.w == 2 else "v_mfma_f32_16x16x4_f32"
        o = ["s_waitcnt vmcnt(%d)" % wait]
        for j in range(self.jb):
            o.append("%s %s, %s, %%[q%d]" % (mul, self.bcval(j), self.bval(s, j), j))
        o.append("s_nop 1")
        for r in range(self.rb):
            for j in range(self.jb):
                a = "%%[a%d%d]" % (r, j)
                o.append("%s %s, %s, %s, %s" % (mfma, a, self.xval(s, r), self.bcval(j), a))
        return o

    def block(self, nt):
        d, s_n, l = self.d, self.d + 1, self.loads
        o = ["s_nop 4"]
        for k in range(d):
            o += self.issue(k, nt)
        o.append("1:")
        for u in range(s_n):
            o.append("s_cmp_eq_u32 %[n], 0")
            o.append("s_cbranch_scc1 %df" % (10 + u))
            o += self.issue((u + d) % s_n, nt)
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
        out = "// %s: RB = %d, JB = %d; %d steps in flight, ring of %d sets in v[%d:%d], %d wavefronts per SIMD\n" % (
            c, self.rb, self.jb, self.d, self.d + 1, self.t0, self.last_reg(), self.waves)
        flavours = [("", "")] + ([("_NT", " nt")] if self.w == 2 else [])
        for suffix, nt in flavours:
            out += "#define MTTKRP_PIPE_%s_ASM%s \\\n" % (t, suffix)
            out += " \\\n".join('    "%s\\n"' % line for line in self.block(nt)) + "\n"
        clob = ", ".join('"v%d"' % v for v in range(self.t0, self.last_reg() + 1))
        accs = ", ".join('[a%d%d] "+v"(acc[%d][%d])' % (r, j, r, j) for r in range(self.rb) for j in range(self.jb))
        outs = '[xq] "+v"(xq), ' + ('[xq1] "+v"(xq1), ' if self.two_x else "") + '[bo0] "+v"(bo0), ' + \
               ('[bo1] "+v"(bo1), ' if self.two_b else "") + '[n] "+s"(n_more), ' + accs
        ins = '[xs] "s"(x_step_bytes), [bb] "s"(bbase), [bs] "s"(b_step_bytes), ' + \
              ", ".join('[q%d] "v"(q[%d])' % (j, j) for j in range(self.jb))
        out += "template <> struct Pipe<%s, %d, %d> {\n" % (c, self.rb, self.jb)
        out += "    static constexpr bool value = true;\n"
        out += "    static constexpr int depth = %d;\n    static constexpr int waves = %d;\n" % (self.d, self.waves)
        out += "    template <bool NT>\n"
        out += "    static __device__ __forceinline__ void run(typename Mfma<%s>::acc_t (&acc)[%d][%d], const %s*& xq,\n" % (c, self.rb, self.jb, c)
        out += "                                               const %s* xq1, int64_t x_step_bytes, const %s* bbase,\n" % (c, c)
        out += "                                               uint32_t bo0, uint32_t bo1, uint32_t b_step_bytes,\n"
        out += "                                               const %s (&q)[%d], int n_more)\n    {\n" % (c, self.jb)
        if not self.two_x:
            out += "        (void)xq1;\n"
        if not self.two_b:
            out += "        (void)bo1;\n"
        if self.w == 2:
            out += "        if (NT)\n"
            out += "            asm volatile(MTTKRP_PIPE_%s_ASM_NT : %s : %s : %s, \"scc\", \"memory\");\n" % (t, outs, ins, clob)
            out += "        else\n    "
        out += "        asm volatile(MTTKRP_PIPE_%s_ASM : %s : %s : %s, \"scc\", \"memory\");\n" % (t, outs, ins, clob)
        out += "    }\n};\n\n"
        return out


def main(path=None):
    """Writes the include file (next to this script unless a path is given) and returns its path."""
    insts = [Inst(w, rb, jb) for w in (2, 1) for rb in (1, 2, 3, 4) for jb in (1, 2, 3, 4)]
    insts = [i for i in insts if i.budget]
    out = "// Generated by gen_pipe.py; do not edit.\n"
    out += "// Primary template: no pipelined run for an instantiation (the kernel then uses batches only).\n"
    out += "template <typename T, int RB, int JB> struct Pipe {\n"
    out += "    static constexpr bool value = false;\n    static constexpr int depth = 1 << 30;\n"
    out += "    static constexpr int waves = 0;\n"
    out += "    template <bool NT>\n"
    out += "    static __device__ __forceinline__ void run(typename Mfma<T>::acc_t (&)[RB][JB], const T*&, const T*, int64_t,\n"
    out += "                                               const T*, uint32_t, uint32_t, uint32_t, const T (&)[JB], int)\n    {\n    }\n};\n\n"
    for i in insts:
        out += i.emit()
    if path is None:
        path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "mttkrp_pipe.inc")
    with open(path, "w") as f:
        f.write(out)
    for i in insts:
        print("%s: acc %3d, set %2d, depth %d, budget %d (%d waves), ring v[%d:%d], loads/step %d" % (
            i.tag(), i.acc, i.set, i.d, i.budget, i.waves, i.t0, i.last_reg(), i.loads))
    return path


if __name__ == "__main__":
    print(main())
