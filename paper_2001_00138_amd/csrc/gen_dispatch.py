#!/usr/bin/env python3
"""Generates the step-stream interpreter of the tiled pattern-sparse kernels.

For one register geometry (G filter slots, PR x PC output patch per lane, stride S,
TGX lanes across a band) and one MODE this writes a C++ header with an explicit
specialisation

    template <> struct StreamLoop<G, PR, PC, S, TGX, MODE> {
        static constexpr unsigned kBlockBytes, kTableOff, kCtrlBytes, kRecords;
        static void run(acc, lane_lds, stream, entry);
    };

whose body is ONE inline-assembly statement, hand-scheduled for gfx950.
MODE bit 0: two sets of window registers; bit 1: threaded dispatch; bit 2: the window
lives in fixed vector registers and is read from LDS two floats at a time; bit 3: the
staged channel is laid out band by band (bank-conflict-free window reads) instead of
row by row.

The encoder turns the kept kernels of one filter group and one chunk of staged input
channels into a sequence of fixed-size *steps* (24 dwords each); all kernels of a step
read the same input channel (a channel with more kernels in the group than a step
holds continues in the next step).  The interpreter

  * keeps two sets of scalar registers and fetches step k+1 over the scalar data path
    while step k executes - one wait per step, for data requested a whole step ago;
  * runs, per kernel, one straight-line block out of a table with one block per
    (window set, filter slot, pattern): the 4*PR*PC FMAs of that pattern on the
    accumulators of that slot, ``v_fmac_f32 acc, s_weight, v_window`` with every
    register fixed at generation time.  This is the "one generated code body per
    pattern, no indirect access, no branches" of paper section 5.2 / 5.4, with a jump
    table in place of per-layer code generation.  The pattern index ranges over the 56
    four-entry patterns that keep the centre (section 4.1), in lexicographic order of
    their other three positions;
  * loads a lane's input window of one staged channel from LDS into registers once
    per channel and filter group, where every kernel of the group on that channel
    uses it (load-redundancy elimination, section 5.4).  With two sets of window
    registers the window of the NEXT channel is requested at the start of a step and
    lands while the current channel's kernels run.

Call dispatch (MODE bit 1 clear).  Step: dwords 0..15 the four weights of up to 4
kernels, 16..19 their code offsets, 20 the window block to run first, 21 the LDS byte
offset of its channel.  A central dispatcher calls every block (s_swappc_b64) and the
block returns (s_setpc_b64): two jumps per kernel.

Threaded dispatch (MODE bit 1 set).  Step: three records of six dwords (four weights,
code offset, zero), dword 22 the code offset that follows a full step, dword 23 the LDS
byte offset of the step's window.  Every FMA block ends by fetching the next record
(s_movrels, M0 = register index of the record) and jumping straight to its block; the
record after the last kernel of a step names one of six step-transition blocks (which
register set the next step is in x which window to load), or the end: one jump per
kernel plus two per step.

Only plain (non-packed) fp32 FMAs are emitted.  Nothing is written through the scalar
data path: it is used for loads only.  Every block carries an assembler-time check
that it fits its slot, so the offsets the encoder computes are the real ones.

Run by ``buildlib.py``; output goes to ``csrc/gen/`` and is not committed.
``program()`` returns the assembly as a list of lines; the host tests execute those
lines on a small model of the machine against the encoder's streams.
"""

import itertools
import os
import sys

STEP_DWORDS = 24
# fixed scalar registers of the interpreter (declared as clobbers)
SET_A, SET_B = 36, 60          # 24 registers each
W = 84                         # current kernel's weights s[84:87]
CTRL_SLOT = 512                # bytes per control block

# call dispatch
C_TGT, C_RET, C_BASE, C_SP, C_WOFF = 88, 90, 92, 94, 96
C_CLOBBER = (36, 96)
C_RECORDS = 4
PF_A, PF_B, PF_NONE, DONE_A, DONE_B, END = range(6)      # control blocks, in code order
C_NUM_CTRL = 6

# threaded dispatch
T_TGT, T_BASE, T_SP, T_SAVE = 88, 90, 92, 94
T_CLOBBER = (36, 94)
T_RECORDS = 3
T_REC_DWORDS = 6
T_TERM_FULL, T_WOFF = 22, 23   # step dwords: code offset after a full step; window LDS offset
T_END = 6                      # control blocks: 3*set + action (0 none, 1 / 2 load window 0 / 1); then end
T_NUM_CTRL = 7


def universe():
    others = [p for p in range(9) if p != 4]
    return [sorted(combo + (4,)) for combo in itertools.combinations(others, 3)]


def pow2_at_least(n):
    p = 1
    while p < n:
        p *= 2
    return p


def geometry(G, PR, PC, S, TGX, MODE):
    WR, WC = (PR - 1) * S + 3, (PC - 1) * S + 3
    band_cols = (TGX * PC - 1) * S + 3
    if MODE & 8:
        # band-major LDS layout: a band's window rows follow each other; bands start
        # (lanes-per-band step) mod 32 banks apart (the kernel's Geo computes the same)
        pitch = band_cols
        band = WR * band_cols
        band_stride = band + ((TGX * PC * S) % 32 - band % 32 + 32) % 32
    else:
        pitch = (64 // TGX) * band_cols                # floats per staged row: the bands side by side
        band_stride = band_cols
    nacc = PR * PC
    threaded = bool(MODE & 2)
    tail = 7 if threaded else 1                        # 4-byte scalar instructions after the FMAs
    block_bytes = pow2_at_least(4 * (4 * nacc + tail))
    num_ctrl = T_NUM_CTRL if threaded else C_NUM_CTRL
    return dict(WR=WR, WC=WC, pitch=pitch, band_stride=band_stride, band_cols=band_cols,
                band_major=bool(MODE & 8), nacc=nacc, nwin=WR * WC, block_bytes=block_bytes,
                table_off=num_ctrl * CTRL_SLOT, sets=2 if MODE & 1 else 1, threaded=threaded,
                wide=bool(MODE & 4),
                records=T_RECORDS if threaded else C_RECORDS, ctrl_bytes=CTRL_SLOT,
                clobber=T_CLOBBER if threaded else C_CLOBBER)


class _Asm:
    def __init__(self):
        self.lines = []
        self.nblocks = 0

    def __call__(self, line):
        self.lines.append(line)

    def begin_block(self, log2):
        """Aligned start of a block that must fit 2**log2 bytes."""
        self(f".p2align {log2}")
        self(f".Lblk{self.nblocks}_%=:")

    def end_block(self, log2):
        self(f".if . - .Lblk{self.nblocks}_%= > {1 << log2}")
        self('.error "code block larger than its slot"')
        self(".endif")
        self.nblocks += 1


WIDE_WINDOW_BASE = 128         # first fixed window register of MODE bit 2


def _win(g, ws, i):
    """Operand text of window register i of set ws."""
    if g["wide"]:
        return f"v{WIDE_WINDOW_BASE + ws * g['nwin'] + i}"
    return f"%[x{ws}_{i}]"


def _window_reads(asm, g, ws):
    if g["wide"] and g["WC"] % 2 == 0:
        # rows start 8-byte aligned in LDS (even patch width, even pitch): two floats per read
        for q in range(g["WR"]):
            for r in range(0, g["WC"], 2):
                v = WIDE_WINDOW_BASE + ws * g["nwin"] + q * g["WC"] + r
                asm(f"ds_read_b64 v[{v}:{v + 1}], %[addr] offset:{4 * (q * g['pitch'] + r)}")
        return
    if g["wide"]:
        # odd window width: any two window elements per read (ds_read2_b32 takes two dword
        # offsets below 256, which the band-major layout keeps them under)
        base = WIDE_WINDOW_BASE + ws * g["nwin"]
        offs = [q * g["pitch"] + r for q in range(g["WR"]) for r in range(g["WC"])]
        for i in range(0, g["nwin"] - 1, 2):
            asm(f"ds_read2_b32 v[{base + i}:{base + i + 1}], %[addr] offset0:{offs[i]} offset1:{offs[i + 1]}")
        if g["nwin"] % 2:
            asm(f"ds_read_b32 v{base + g['nwin'] - 1}, %[addr] offset:{4 * offs[-1]}")
        return
    for i in range(g["nwin"]):
        q, r = divmod(i, g["WC"])
        asm(f"ds_read_b32 %[x{ws}_{i}], %[addr] offset:{4 * (q * g['pitch'] + r)}")


def _fmas(G, PR, PC, S, g, ws, slot, taps):
    out = []
    for t, pos in enumerate(taps):
        kh, kw = divmod(pos, 3)
        for r in range(PR):
            for c in range(PC):
                x = (r * S + kh) * g["WC"] + c * S + kw
                out.append(f"v_fmac_f32 %[a{slot}_{r * PC + c}], s{W + t}, {_win(g, ws, x)}")
    return out


def _program_call(G, PR, PC, S, TGX, MODE, g):
    DW = MODE & 1
    TGT, RET, BASE, SP, WOFF = C_TGT, C_RET, C_BASE, C_SP, C_WOFF
    R = C_RECORDS
    ctrl_log2 = CTRL_SLOT.bit_length() - 1
    block_log2 = g["block_bytes"].bit_length() - 1
    asm = _Asm()
    # ---- set-up: table address, first step
    asm(f"s_getpc_b64 s[{BASE}:{BASE + 1}]")
    asm(".Lpc%=:")
    asm(f"s_add_u32 s{BASE}, s{BASE}, .Lbase%=-.Lpc%=")
    asm(f"s_addc_u32 s{BASE + 1}, s{BASE + 1}, 0")
    asm(f"s_mov_b64 s[{SP}:{SP + 1}], %[sp]")

    def fetch(dst):
        asm(f"s_load_dwordx16 s[{dst}:{dst + 15}], s[{SP}:{SP + 1}], 0x0")
        asm(f"s_load_dwordx8 s[{dst + 16}:{dst + 23}], s[{SP}:{SP + 1}], 0x40")
        asm(f"s_add_u32 s{SP}, s{SP}, {4 * STEP_DWORDS}")
        asm(f"s_addc_u32 s{SP + 1}, s{SP + 1}, 0")

    def call(target_sgpr):
        asm(f"s_add_u32 s{TGT}, s{BASE}, s{target_sgpr}")
        asm(f"s_addc_u32 s{TGT + 1}, s{BASE + 1}, 0")
        asm(f"s_swappc_b64 s[{RET}:{RET + 1}], s[{TGT}:{TGT + 1}]")

    fetch(SET_A)
    for name, cur, nxt in (("A", SET_A, SET_B), ("B", SET_B, SET_A)):
        asm(f".Lstep{name}%=:")
        asm("s_waitcnt lgkmcnt(0)")
        if DW:
            fetch(nxt)                       # next step's registers, in flight during this step
        asm(f"s_mov_b32 s{WOFF}, s{cur + 21}")
        call(cur + 20)                       # window block
        if not DW:
            fetch(nxt)                       # after the window has landed (its block waits)
        for i in range(R):
            asm(f"s_mov_b64 s[{W}:{W + 1}], s[{cur + 4 * i}:{cur + 4 * i + 1}]")
            asm(f"s_mov_b64 s[{W + 2}:{W + 3}], s[{cur + 4 * i + 2}:{cur + 4 * i + 3}]")
            call(cur + 16 + i)
    asm("s_branch .LstepA%=")

    # ---- control blocks, CTRL_SLOT bytes apart
    def ctrl_begin(k):
        asm.begin_block(ctrl_log2)
        if k == 0:
            asm(".Lbase%=:")

    for s in range(2):
        ctrl_begin(PF_A + s)
        asm(f"v_add_u32 %[addr], s{WOFF}, %[lane]")
        _window_reads(asm, g, s if DW else 0)
        if not DW:
            asm("s_waitcnt lgkmcnt(0)")
        asm(f"s_setpc_b64 s[{RET}:{RET + 1}]")
        asm.end_block(ctrl_log2)
    ctrl_begin(PF_NONE)
    asm(f"s_setpc_b64 s[{RET}:{RET + 1}]")
    asm.end_block(ctrl_log2)
    ctrl_begin(DONE_A)
    asm("s_branch .LstepB%=")
    asm.end_block(ctrl_log2)
    ctrl_begin(DONE_B)
    asm("s_branch .LstepA%=")
    asm.end_block(ctrl_log2)
    ctrl_begin(END)                          # the exit is beyond the reach of s_branch
    asm(f"s_add_u32 s{TGT}, s{BASE}, .Lexit%=-.Lbase%=")
    asm(f"s_addc_u32 s{TGT + 1}, s{BASE + 1}, 0")
    asm(f"s_setpc_b64 s[{TGT}:{TGT + 1}]")
    asm.end_block(ctrl_log2)
    asm(f".p2align {ctrl_log2}")

    # ---- the table: block ((set*G + slot)*56 + pattern) at table_off + index*block_bytes
    for ws in range(g["sets"]):
        for slot in range(G):
            for taps in universe():
                asm.begin_block(block_log2)
                for line in _fmas(G, PR, PC, S, g, ws, slot, taps):
                    asm(line)
                asm(f"s_setpc_b64 s[{RET}:{RET + 1}]")
                asm.end_block(block_log2)
    asm(".Lexit%=:")
    asm("s_waitcnt lgkmcnt(0)")
    return asm.lines


def _program_threaded(G, PR, PC, S, TGX, MODE, g):
    DW = MODE & 1
    TGT, BASE, SP, SAVE = T_TGT, T_BASE, T_SP, T_SAVE
    ctrl_log2 = CTRL_SLOT.bit_length() - 1
    block_log2 = g["block_bytes"].bit_length() - 1
    asm = _Asm()

    def fetch(dst):
        asm(f"s_load_dwordx16 s[{dst}:{dst + 15}], s[{SP}:{SP + 1}], 0x0")
        asm(f"s_load_dwordx8 s[{dst + 16}:{dst + 23}], s[{SP}:{SP + 1}], 0x40")
        asm(f"s_add_u32 s{SP}, s{SP}, {4 * STEP_DWORDS}")
        asm(f"s_addc_u32 s{SP + 1}, s{SP + 1}, 0")

    def jump(target_sgpr):
        asm(f"s_add_u32 s{TGT}, s{BASE}, {target_sgpr}")
        asm(f"s_addc_u32 s{TGT + 1}, s{BASE + 1}, 0")
        asm(f"s_setpc_b64 s[{TGT}:{TGT + 1}]")

    # ---- set-up: M0 is given back at the end; table address; first step; first transition
    asm(f"s_mov_b32 s{SAVE}, m0")
    asm(f"s_getpc_b64 s[{BASE}:{BASE + 1}]")
    asm(".Lpc%=:")
    asm(f"s_add_u32 s{BASE}, s{BASE}, .Lbase%=-.Lpc%=")
    asm(f"s_addc_u32 s{BASE + 1}, s{BASE + 1}, 0")
    asm(f"s_mov_b64 s[{SP}:{SP + 1}], %[sp]")
    fetch(SET_A)
    jump("%[entry]")

    # ---- step transitions: control block 3*set + action, then the end block
    first = True
    for cur, nxt in ((SET_A, SET_B), (SET_B, SET_A)):
        for action in range(3):
            asm.begin_block(ctrl_log2)
            if first:
                asm(".Lbase%=:")
                first = False
            asm("s_waitcnt lgkmcnt(0)")      # this step's registers (and, with two window sets, its window)
            if DW:
                fetch(nxt)
            if action:
                asm(f"v_add_u32 %[addr], s{cur + T_WOFF}, %[lane]")
                _window_reads(asm, g, (action - 1) if DW else 0)
            # first record of the step; M0 = register index (from SET_A) of the second; the jump
            # target.  With one window set this scalar work runs while the window reads are in
            # flight (the FMAs that read the weight registers were all issued before).
            asm(f"s_mov_b64 s[{W}:{W + 1}], s[{cur}:{cur + 1}]")
            asm(f"s_mov_b64 s[{W + 2}:{W + 3}], s[{cur + 2}:{cur + 3}]")
            asm(f"s_mov_b32 m0, {cur - SET_A + T_REC_DWORDS}")
            asm(f"s_add_u32 s{TGT}, s{BASE}, s{cur + 4}")
            asm(f"s_addc_u32 s{TGT + 1}, s{BASE + 1}, 0")
            if not DW:
                if action:
                    asm("s_waitcnt lgkmcnt(0)")
                fetch(nxt)
            asm(f"s_setpc_b64 s[{TGT}:{TGT + 1}]")
            asm.end_block(ctrl_log2)
    asm.begin_block(ctrl_log2)               # end of the chunk's stream
    asm("s_waitcnt lgkmcnt(0)")              # the step fetched ahead
    asm(f"s_mov_b32 m0, s{SAVE}")
    jump(".Lexit%=-.Lbase%=")
    asm.end_block(ctrl_log2)
    asm(f".p2align {ctrl_log2}")

    # ---- the table
    for ws in range(g["sets"]):
        for slot in range(G):
            for taps in universe():
                asm.begin_block(block_log2)
                # the next record's block address first: it is ready long before the jump
                asm(f"s_movrels_b32 s{TGT}, s{SET_A + 4}")
                asm(f"s_add_u32 s{TGT}, s{TGT}, s{BASE}")
                asm(f"s_addc_u32 s{TGT + 1}, s{BASE + 1}, 0")
                for line in _fmas(G, PR, PC, S, g, ws, slot, taps):
                    asm(line)
                # next record -> weight registers (the FMAs above have read the current ones)
                asm(f"s_movrels_b64 s[{W}:{W + 1}], s[{SET_A}:{SET_A + 1}]")
                asm(f"s_movrels_b64 s[{W + 2}:{W + 3}], s[{SET_A + 2}:{SET_A + 3}]")
                asm(f"s_add_u32 m0, m0, {T_REC_DWORDS}")
                asm(f"s_setpc_b64 s[{TGT}:{TGT + 1}]")
                asm.end_block(block_log2)
    asm(".Lexit%=:")
    return asm.lines


def program(G, PR, PC, S, TGX, MODE):
    """(assembly lines, geometry).  Operands: %[a<slot>_<i>] accumulators, %[x<set>_<i>]
    window registers, %[addr] a scratch VGPR, %[lane] the lane's LDS byte address of the
    staged chunk, %[sp] the 64-bit address of the first step, %[entry] (threaded) the
    code offset of the first step transition."""
    g = geometry(G, PR, PC, S, TGX, MODE)
    if g["wide"] and g["WC"] % 2 == 0 and ((PC * S) % 2 or g["pitch"] % 2):
        raise ValueError("64-bit window reads need an even lane step and an even row pitch")
    if g["wide"] and g["WC"] % 2 and (g["WR"] - 1) * g["pitch"] + g["WC"] > 255:
        raise ValueError("paired window reads need every window offset below 256 dwords (band-major layout)")
    if g["wide"] and g["sets"] * g["nwin"] % 2 and g["sets"] > 1:
        raise ValueError("two fixed window sets need an even window size")
    build = _program_threaded if g["threaded"] else _program_call
    return build(G, PR, PC, S, TGX, MODE, g), g


def generate(G, PR, PC, S, TGX, MODE):
    lines, g = program(G, PR, PC, S, TGX, MODE)
    nacc, nwin, sets = g["nacc"], g["nwin"], g["sets"]
    L = []
    emit = L.append
    emit("// Generated by gen_dispatch.py - do not edit.")
    emit(f"// G={G} PR={PR} PC={PC} S={S} TGX={TGX} MODE={MODE}: {sets * G * 56} FMA blocks of "
         f"{g['block_bytes']} bytes.")
    emit(f"template <> struct StreamLoop<{G}, {PR}, {PC}, {S}, {TGX}, {MODE}> {{")
    emit(f"    static constexpr unsigned kBlockBytes = {g['block_bytes']}u;")
    emit(f"    static constexpr unsigned kTableOff = {g['table_off']}u;")
    emit(f"    static constexpr unsigned kCtrlBytes = {CTRL_SLOT}u;")
    emit(f"    static constexpr unsigned kRecords = {g['records']}u;")
    emit(f"    static __device__ __forceinline__ void run(float (&acc)[{G}][{nacc}], unsigned lane_lds,")
    emit("                                               const uint32_t* stream, unsigned entry)")
    emit("    {")
    if not g["wide"]:
        emit(f"        float win[{sets}][{nwin}];")
    emit("        unsigned addr;")
    if not g["threaded"]:
        emit("        (void)entry;")
    emit("        asm volatile(")
    # one string literal per block keeps the source readable for the compiler's lexer
    chunk = []
    for line in lines:
        chunk.append(line.replace("\\", "\\\\").replace('"', '\\"'))
        if len(chunk) == 32:
            emit('            "' + "\\n".join(chunk) + '\\n"')
            chunk = []
    if chunk:
        emit('            "' + "\\n".join(chunk) + '\\n"')
    outs = ", ".join(f'[a{s}_{i}] "+v"(acc[{s}][{i}])' for s in range(G) for i in range(nacc))
    if not g["wide"]:
        outs += ", " + ", ".join(f'[x{ws}_{i}] "=&v"(win[{ws}][{i}])' for ws in range(sets) for i in range(nwin))
    outs += ', [addr] "=&v"(addr)'
    ins = '[lane] "v"(lane_lds), [sp] "s"(stream)'
    if g["threaded"]:
        ins += ', [entry] "s"(entry)'
    lo, hi = g["clobber"]
    clob = ", ".join(f'"s{i}"' for i in range(lo, hi + 1))
    if g["wide"]:
        clob += ", " + ", ".join(f'"v{WIDE_WINDOW_BASE + i}"' for i in range(sets * nwin))
    emit(f"            : {outs}")
    emit(f"            : {ins}")
    emit(f'            : {clob}, "scc", "memory");')
    emit("    }")
    emit("};")
    return "\n".join(L) + "\n"


def main(argv):
    out_dir = argv[1]
    os.makedirs(out_dir, exist_ok=True)
    text = ""
    for spec in sorted(set(argv[2:])):
        text += generate(*(int(v) for v in spec.split(",")))
    path = os.path.join(out_dir, "dispatch_all.inc")
    if not os.path.exists(path) or open(path).read() != text:
        with open(path, "w") as f:
            f.write(text)


if __name__ == "__main__":
    main(sys.argv)
