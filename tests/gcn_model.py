"""A small functional model of one gfx9 wavefront - TEST INFRASTRUCTURE.

It executes the assembly that ``csrc/gen_dispatch.py`` generates (the step interpreter
and its table of FMA blocks) on the CPU, so that the interpreter and the encoder's
streams can be checked against the oracle without a GPU.  Only the instructions the
generator emits are modelled, with their architectural semantics (no timing, no
hazards): scalar moves / adds / relative moves, scalar loads, computed jumps, LDS
reads, v_add_u32 and v_fmac_f32 on 64 lanes.  Memory results are delivered as LATE as
the architecture allows: a scalar load or an LDS read only lands when the wavefront
executes ``s_waitcnt lgkmcnt(0)``, and touching its destination before that is an
error - so a missing wait shows up as a failure instead of passing by luck.  fp32 FMAs are evaluated as the
correctly rounded sum in double precision of the exact product, which is the fused
result except for double rounding on rare ties.

Addresses: the program is laid out from ``CODE_BASE`` with the sizes of the real
encodings (4 bytes, 8 with a 32-bit literal, 8 for SMEM and DS), honouring
``.p2align``.  The generated code checks at assembly time that every block fits its
slot, so block starts - the only jump targets - coincide with the real layout.
"""

from __future__ import annotations

import re
from typing import Dict, List

import numpy as np

CODE_BASE = 0x7F00_0010_0000         # multiple of every alignment used
STREAM_BASE = 0x7E00_0000_0000
WAVE = 64


class ModelError(AssertionError):
    pass


def _is_inline_const(v: int) -> bool:
    return -16 <= v <= 64


class Program:
    """Decoded program: instruction list, address of each, label -> address."""

    def __init__(self, lines: List[str], code_base: int = CODE_BASE):
        self.ins = []          # (mnemonic, [operands], address)
        self.at: Dict[int, int] = {}
        self.labels: Dict[str, int] = {}
        self.base = code_base  # a multiple of every alignment used
        pc = code_base
        for raw in lines:
            line = raw.strip()
            if not line:
                continue
            if line.startswith(".p2align"):
                a = 1 << int(line.split()[1])
                pc = (pc + a - 1) // a * a
                continue
            if line.startswith((".if", ".error", ".endif")):
                continue
            if line.endswith(":"):
                self.labels[line[:-1]] = pc
                continue
            m = re.match(r"(\S+)\s*(.*)", line)
            op, rest = m.group(1), m.group(2)
            offset = 0
            mo = re.search(r"\s+offset:(\S+)$", rest)
            if mo:
                offset = int(mo.group(1), 0)
                rest = rest[:mo.start()]
            pair = re.search(r"\s+(offset0:\d+\s+offset1:\d+)$", rest)
            if pair:
                rest = rest[:pair.start()]
            args = [a.strip() for a in rest.split(",")] if rest else []
            if pair:
                args.append(pair.group(1))
            size = 4
            if op.startswith(("s_load", "ds_")):
                size = 8
            elif op.startswith(("s_add", "s_addc", "s_mov_b32", "s_sub", "s_and", "s_lshl", "s_lshr", "s_mul")):
                for a in args[1:]:
                    if re.match(r"^-?(0x[0-9a-fA-F]+|\d+)$", a):
                        if not _is_inline_const(int(a, 0)):
                            size = 8
                    elif a.startswith("."):
                        size = 8
            self.at[pc] = len(self.ins)
            self.ins.append((op, args, pc, offset, size))
            pc += size
        self.end = pc
        self.label_addresses = set(self.labels.values())

    def label_expr(self, expr: str) -> int:
        m = re.match(r"^(\.\S+?)-(\.\S+)$", expr)
        if not m:
            raise ModelError(f"cannot evaluate {expr}")
        return self.labels[m.group(1)] - self.labels[m.group(2)]


class Wave:
    def __init__(self, prog: Program, stream: np.ndarray, lds: np.ndarray):
        self.p = prog
        self.stream = np.ascontiguousarray(stream, dtype=np.uint32).ravel()
        self.lds = lds                     # uint32 view of the workgroup's LDS
        self.s = np.zeros(128, dtype=np.uint64)     # scalar registers (32-bit values)
        self.m0 = 0
        self.scc = 0
        self.v: Dict[str, np.ndarray] = {}          # vector operands by name, uint32[64]
        self.sop: Dict[str, int] = {}               # scalar operands by name
        self.executed = 0
        self.jumps = 0
        self.return_points = set()
        self.pending_v: Dict[str, np.ndarray] = {}  # LDS reads in flight
        self.pending_s: Dict[int, int] = {}         # scalar loads in flight

    # ---- operand access
    def _sreg(self, name: str) -> int:
        return int(name[1:])

    def rd32(self, a: str) -> int:
        if a == "m0":
            return self.m0
        if a.startswith("%["):
            v = self.sop[a[2:-1]]
            return v & 0xFFFFFFFF
        if re.match(r"^s\d+$", a):
            if self._sreg(a) in self.pending_s:
                raise ModelError(f"{a} read while a scalar load into it is in flight")
            return int(self.s[self._sreg(a)])
        if a.startswith("."):
            return self.p.label_expr(a) & 0xFFFFFFFF
        return int(a, 0) & 0xFFFFFFFF

    def wr32(self, a: str, v: int):
        v &= 0xFFFFFFFF
        if a == "m0":
            self.m0 = v
        else:
            if self._sreg(a) in self.pending_s:
                raise ModelError(f"{a} written while a scalar load into it is in flight")
            self.s[self._sreg(a)] = v

    def pair(self, a: str):
        m = re.match(r"^s\[(\d+):(\d+)\]$", a)
        lo, hi = int(m.group(1)), int(m.group(2))
        if lo % 2:
            raise ModelError(f"misaligned register pair {a}")
        return lo, hi

    def rd64(self, a: str) -> int:
        if a.startswith("%["):
            return self.sop[a[2:-1]]
        lo, hi = self.pair(a)
        assert hi == lo + 1
        if lo in self.pending_s or hi in self.pending_s:
            raise ModelError(f"{a} read while a scalar load into it is in flight")
        return int(self.s[lo]) | (int(self.s[hi]) << 32)

    def wr64(self, a: str, v: int):
        lo, hi = self.pair(a)
        assert hi == lo + 1
        if lo in self.pending_s or hi in self.pending_s:
            raise ModelError(f"{a} written while a scalar load into it is in flight")
        self.s[lo] = v & 0xFFFFFFFF
        self.s[hi] = (v >> 32) & 0xFFFFFFFF

    @staticmethod
    def vkey(a: str) -> str:
        """Vector operand -> key: the name of a %[...] operand, or a fixed register vN."""
        return a[2:-1] if a.startswith("%[") else a

    def vreg(self, a: str) -> np.ndarray:
        name = self.vkey(a)
        if name in self.pending_v:
            raise ModelError(f"vector operand {name} used while an LDS read into it is in flight")
        if name not in self.v:
            raise ModelError(f"vector operand {name} read before it was written")
        return self.v[name]

    def _computed_target(self, target: int) -> int:
        """A computed jump may only land on the start of a block (every block start and
        the exit carry a label) or on the instruction after a call."""
        if target not in self.p.label_addresses and target not in self.return_points:
            raise ModelError(f"computed jump to {target - self.p.base:#x}, which is not a block start")
        return target

    # ---- execution
    def run(self, max_instructions: int = 50_000_000) -> None:
        p = self.p
        pc = p.base
        s = self.s
        while True:
            if pc == p.end:                              # fell off the end of the statement
                if self.pending_v or self.pending_s:
                    raise ModelError("the statement ends with loads in flight")
                return
            if pc not in p.at:
                raise ModelError(f"jump into the middle of nowhere: {pc - p.base:#x}")
            op, a, addr, off, size = p.ins[p.at[pc]]
            nxt = pc + size
            self.executed += 1
            if self.executed > max_instructions:
                raise ModelError("program does not end")
            if op == "v_fmac_f32":
                d = self.vreg(a[0])
                wv = np.array([self.rd32(a[1])], dtype=np.uint32).view(np.float32)[0]
                x = self.vreg(a[2]).view(np.float32)
                r = (np.float64(wv) * x.astype(np.float64) + d.view(np.float32).astype(np.float64))
                self.v[self.vkey(a[0])] = r.astype(np.float32).view(np.uint32)
            elif op == "ds_read_b32":
                va = self.vreg(a[1]).astype(np.int64) + off
                if (va % 4).any() or (va < 0).any() or (va + 4 > self.lds.size * 4).any():
                    raise ModelError(f"LDS read out of the staged region at {addr - p.base:#x}")
                if self.vkey(a[0]) in self.pending_v:
                    raise ModelError("two LDS reads in flight into one register")
                self.pending_v[self.vkey(a[0])] = self.lds[va // 4].copy()
            elif op == "ds_read_b64":
                va = self.vreg(a[1]).astype(np.int64) + off
                if (va % 8).any() or (va < 0).any() or (va + 8 > self.lds.size * 4).any():
                    raise ModelError(f"misaligned or out-of-range 64-bit LDS read at {addr - p.base:#x}")
                lo, hi = re.match(r"^v\[(\d+):(\d+)\]$", a[0]).groups()
                if int(hi) != int(lo) + 1 or int(lo) % 2:
                    raise ModelError(f"bad 64-bit destination {a[0]}")
                for k in range(2):
                    if f"v{int(lo) + k}" in self.pending_v:
                        raise ModelError("two LDS reads in flight into one register")
                    self.pending_v[f"v{int(lo) + k}"] = self.lds[va // 4 + k].copy()
            elif op == "ds_read2_b32":
                m2 = re.match(r"^offset0:(\d+)\s+offset1:(\d+)$", a[2]) if len(a) > 2 else None
                if not m2:
                    raise ModelError(f"ds_read2_b32 operands not understood: {a}")
                lo, hi = re.match(r"^v\[(\d+):(\d+)\]$", a[0]).groups()
                if int(hi) != int(lo) + 1:
                    raise ModelError(f"bad destination {a[0]}")
                for k in range(2):
                    o = int(m2.group(1 + k))
                    if o > 255:
                        raise ModelError("ds_read2_b32 offset above 255 dwords")
                    va = self.vreg(a[1]).astype(np.int64) + 4 * o
                    if (va % 4).any() or (va < 0).any() or (va + 4 > self.lds.size * 4).any():
                        raise ModelError(f"LDS read out of the staged region at {addr - p.base:#x}")
                    if f"v{int(lo) + k}" in self.pending_v:
                        raise ModelError("two LDS reads in flight into one register")
                    self.pending_v[f"v{int(lo) + k}"] = self.lds[va // 4].copy()
            elif op == "v_add_u32":
                src0 = a[1]
                x0 = self.vreg(src0) if self.vkey(src0) in self.v else \
                    np.full(WAVE, self.rd32(src0), dtype=np.uint32)
                self.v[self.vkey(a[0])] = (x0.astype(np.uint64) + self.vreg(a[2])).astype(np.uint32)
            elif op in ("s_add_u32", "s_addc_u32"):
                r = self.rd32(a[1]) + self.rd32(a[2]) + (self.scc if op == "s_addc_u32" else 0)
                self.scc = 1 if r >> 32 else 0
                self.wr32(a[0], r)
            elif op == "s_mov_b32":
                self.wr32(a[0], self.rd32(a[1]))
            elif op == "s_mov_b64":
                self.wr64(a[0], self.rd64(a[1]))
            elif op == "s_movrels_b32":
                if self._sreg(a[1]) + self.m0 in self.pending_s:
                    raise ModelError("relative move from a register with a scalar load in flight")
                self.wr32(a[0], int(s[self._sreg(a[1]) + self.m0]))
            elif op == "s_movrels_b64":
                lo, hi = self.pair(a[1])
                src = lo + self.m0
                if src % 2:
                    raise ModelError("s_movrels_b64 from an odd register")
                if src in self.pending_s or src + 1 in self.pending_s:
                    raise ModelError("relative move from a register with a scalar load in flight")
                self.wr64(a[0], int(s[src]) | (int(s[src + 1]) << 32))
            elif op in ("s_load_dwordx16", "s_load_dwordx8"):
                n = 16 if op.endswith("16") else 8
                lo, hi = re.match(r"^s\[(\d+):(\d+)\]$", a[0]).groups()
                lo, hi = int(lo), int(hi)
                if hi - lo + 1 != n or lo % 4:
                    raise ModelError(f"bad SMEM destination {a[0]}")
                ea = self.rd64(a[1]) + int(a[2], 0) + off - STREAM_BASE
                if ea % 4 or ea < 0 or ea // 4 + n > self.stream.size:
                    raise ModelError("scalar load outside the step array")
                for k in range(n):
                    if lo + k in self.pending_s:
                        raise ModelError("two scalar loads in flight into one register")
                    self.pending_s[lo + k] = int(self.stream[ea // 4 + k])
            elif op == "s_getpc_b64":
                self.wr64(a[0], nxt)
            elif op == "s_swappc_b64":
                self.wr64(a[0], nxt)
                self.return_points.add(nxt)
                nxt = self._computed_target(self.rd64(a[1]))
                self.jumps += 1
            elif op == "s_setpc_b64":
                nxt = self._computed_target(self.rd64(a[0]))
                self.jumps += 1
            elif op == "s_branch":
                nxt = p.labels[a[0]]
                self.jumps += 1
            elif op == "s_waitcnt":
                if a != ["lgkmcnt(0)"]:
                    raise ModelError(f"wait not modelled: {a}")
                for name, val in self.pending_v.items():
                    self.v[name] = val
                for reg, val in self.pending_s.items():
                    s[reg] = val
                self.pending_v.clear()
                self.pending_s.clear()
            elif op == "s_nop":
                pass
            else:
                raise ModelError(f"instruction not modelled: {op}")
            pc = nxt
