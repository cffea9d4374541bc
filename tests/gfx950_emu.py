"""A small functional emulator of the gfx950 instruction subset the generated decode kernels use.

Test infrastructure only.  It runs one workgroup (4 waves of 64 lanes) of a kernel from the
generated assembly text on the CPU with numpy, against a bounds-checked flat memory, so that
addressing, control flow, LDS layout, the software pipeline and the arithmetic of the assembly
kernels can be checked without a GPU.  It also models *when results become visible*:

  * LDS reads, SMEM loads and VMEM loads deliver their result only when an `s_waitcnt` forces
    them to (latest legal time).  Reading a register whose load is still pending is reported as
    an error, which checks the lgkmcnt / vmcnt bookkeeping of the generator.
  * direct-to-LDS loads write LDS either at issue or at the wait that retires them (`dma_late`);
    a kernel that synchronises correctly gives the same result both ways.
  * SMEM shares lgkmcnt with LDS and may return out of order: `smem_first` chooses which of the
    two an under-specified wait retires first.

Instruction semantics follow the public CDNA3/CDNA4 ISA documents; the MFMA operand layout and the
lane mapping of `ds_read_b64_tr_b16` are the ones measured on the hardware by this build's probes:
  v_mfma_f32_32x32x16_bf16: A lane l holds row l%32, k = 8*(l//32)+0..7; B lane l holds column
      l%32, same k; C/D register r of lane l is row 8*(r//4) + 4*(l//32) + r%4, column l%32.
  ds_read_b64_tr_b16: within each group of 16 lanes, lane i receives, for j = 0..3, element i%4 of
      the 4 x b16 that lane (i//4 + 4j) of the group addressed.
A static pass (`check_hazards`) looks for the software-visible hazards the kernels must respect.
"""
from __future__ import annotations

import re
import struct

import numpy as np

LANES = 64
U32 = np.uint32
MASK32 = 0xFFFFFFFF


class EmuError(Exception):
    pass


# --------------------------------------------------------------------------------------------
# flat, bounds-checked memory
# --------------------------------------------------------------------------------------------
class Memory:
    def __init__(self):
        self.bufs = []          # (base, bytearray-like np.uint8 array, name, writable)
        self.next = 0x1000_0000

    def add(self, name, data: np.ndarray, writable=False):
        raw = np.frombuffer(np.ascontiguousarray(data).tobytes(), dtype=np.uint8).copy()
        base = self.next
        self.next += ((len(raw) + 0xFFFFF) // 0x100000 + 1) * 0x100000
        self.bufs.append([base, raw, name, writable])
        return base

    def find(self, addr, n, write=False):
        for base, raw, name, writable in self.bufs:
            if base <= addr and addr + n <= base + len(raw):
                if write and not writable:
                    raise EmuError(f"write to read-only buffer {name} at +{addr - base}")
                return raw, addr - base
        raise EmuError(f"out-of-bounds {'write' if write else 'read'} of {n} bytes at 0x{addr:x}")

    def read(self, addr, n):
        raw, off = self.find(addr, n)
        return raw[off:off + n]

    def write(self, addr, data):
        raw, off = self.find(addr, len(data), write=True)
        raw[off:off + len(data)] = data

    def get(self, name):
        for base, raw, nm, _ in self.bufs:
            if nm == name:
                return raw
        raise KeyError(name)


# --------------------------------------------------------------------------------------------
# parsing
# --------------------------------------------------------------------------------------------
def parse_kernel(text: str, name: str):
    """Returns (instructions, labels) of one kernel: instructions are (mnemonic, [operands], modifiers)."""
    lines = text.splitlines()
    start = lines.index(f"{name}:")
    ins, labels = [], {}
    for ln in lines[start + 1:]:
        s = ln.split(";")[0].strip()
        if not s:
            continue
        if s.startswith(".Lfunc_end"):
            break
        if s.endswith(":"):
            labels[s[:-1]] = len(ins)
            continue
        if s.startswith("."):
            continue
        parts = s.split(None, 1)
        mnem = parts[0]
        ops, mods = [], {}
        if len(parts) > 1:
            rest = parts[1]
            for tok in [t.strip() for t in rest.split(",")]:
                sub = tok.split()
                ops.append(sub[0])
                for extra in sub[1:]:
                    if ":" in extra:
                        k, v = extra.split(":")
                        mods[k] = int(v, 0)
                    else:
                        mods[extra] = True
        for suffix in ("_e32", "_e64"):
            if mnem.endswith(suffix):
                mnem = mnem[: -len(suffix)]
        ins.append((mnem, ops, mods))
    return ins, labels


REG_RE = re.compile(r"^(-?)([vsa])(\d+)$|^(-?)([vsa])\[(\d+):(\d+)\]$")


def parse_reg(tok):
    """-> (kind, first, count, neg) or None."""
    m = REG_RE.match(tok)
    if not m:
        return None
    if m.group(2):
        return m.group(2), int(m.group(3)), 1, m.group(1) == "-"
    return m.group(5), int(m.group(6)), int(m.group(7)) - int(m.group(6)) + 1, m.group(4) == "-"


def literal_bits(tok):
    if re.match(r"^-?\d+\.\d*$", tok):
        return struct.unpack("<I", struct.pack("<f", float(tok)))[0]
    return int(tok, 0) & MASK32


def f32(a):
    return np.asarray(a, dtype=U32).view(np.float32)


def bits(a):
    return np.asarray(a, dtype=np.float32).view(U32)


def bf16_to_f32(h):
    return (np.asarray(h, dtype=np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16(x):
    u = np.asarray(x, dtype=np.float32).view(np.uint32)
    nan = np.isnan(np.asarray(x, dtype=np.float32))
    r = ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint32)
    return np.where(nan, np.uint32(0x7FC0), r)


TRANS = {"v_exp_f32", "v_log_f32", "v_rcp_f32", "v_rsq_f32", "v_sqrt_f32"}


# --------------------------------------------------------------------------------------------
# one wave
# --------------------------------------------------------------------------------------------
class Wave:
    def __init__(self, wg, wave_id):
        self.wg = wg
        self.id = wave_id
        self.s = np.zeros(128, dtype=U32)
        self.v = np.zeros((512, LANES), dtype=U32)      # 0..255 arch, 256..511 acc
        self.vcc = 0
        self.exec = (1 << 64) - 1
        self.scc = 0
        self.m0 = 0
        self.pc = 0
        self.done = False
        self.at_barrier = False
        self.lds_q = []      # pending LDS reads: (dst_first, count, data[count, 64])
        self.smem_q = []     # pending SMEM: (dst_first, data[count])
        self.vm_q = []       # pending VMEM loads, in order: ("v", first, data) or ("lds", addr_list, data_list)
        self.pend_v = {}     # vgpr index -> number of pending writes
        self.pend_s = {}
        self.icount = 0

    # ---- register access ----
    def lane_mask(self):
        return np.array([(self.exec >> i) & 1 for i in range(LANES)], dtype=bool)

    def chk_v(self, idx, n=1, what="read"):
        for i in range(idx, idx + n):
            if self.pend_v.get(i):
                raise EmuError(f"wave {self.id} pc {self.pc}: {what} of v{i} (a{i - 256} if >= 256) while a load into it is pending")

    def chk_s(self, idx, n=1):
        for i in range(idx, idx + n):
            if self.pend_s.get(i):
                raise EmuError(f"wave {self.id} pc {self.pc}: read of s{i} while an s_load into it is pending")

    def src(self, tok, as64=False):
        """32-bit source as a [64] uint32 array (or python int pair handling for 64-bit sgprs)."""
        r = parse_reg(tok)
        if r:
            kind, first, cnt, neg = r
            if kind == "v" or kind == "a":
                base = first + (256 if kind == "a" else 0)
                self.chk_v(base, cnt)
                val = self.v[base].copy() if cnt == 1 else self.v[base:base + cnt].copy()
            else:
                self.chk_s(first, cnt)
                if cnt == 1:
                    val = np.full(LANES, self.s[first], dtype=U32)
                else:
                    val = [int(self.s[first + i]) for i in range(cnt)]
            if neg:
                val = bits(-f32(val))
            return val
        if tok == "vcc":
            return self.vcc
        if tok == "exec":
            return self.exec
        if tok == "exec_lo":
            return np.full(LANES, self.exec & MASK32, dtype=U32)
        if tok == "m0":
            return np.full(LANES, self.m0, dtype=U32)
        return np.full(LANES, literal_bits(tok), dtype=U32)

    def ssrc(self, tok):
        """scalar source -> python int (32-bit) or 64-bit for pairs / vcc / exec."""
        r = parse_reg(tok)
        if r:
            kind, first, cnt, _ = r
            assert kind == "s", tok
            self.chk_s(first, cnt)
            if cnt == 1:
                return int(self.s[first])
            return int(self.s[first]) | (int(self.s[first + 1]) << 32)
        if tok == "vcc":
            return self.vcc
        if tok == "exec":
            return self.exec
        if tok == "m0":
            return self.m0
        return literal_bits(tok)

    def sdst(self, tok, val):
        r = parse_reg(tok)
        if r:
            kind, first, cnt, _ = r
            assert kind == "s"
            if cnt == 1:
                self.s[first] = val & MASK32
            else:
                self.s[first] = val & MASK32
                self.s[first + 1] = (val >> 32) & MASK32
        elif tok == "vcc":
            self.vcc = val & ((1 << 64) - 1)
        elif tok == "exec":
            self.exec = val & ((1 << 64) - 1)
        elif tok == "m0":
            self.m0 = val & MASK32
        else:
            raise EmuError("bad sdst " + tok)

    def vdst(self, tok, val, masked=True):
        kind, first, cnt, _ = parse_reg(tok)
        base = first + (256 if kind == "a" else 0)
        val = np.asarray(val, dtype=U32)
        m = self.lane_mask() if masked else np.ones(LANES, bool)
        if cnt == 1:
            self.v[base][m] = val[m]
        else:
            for i in range(cnt):
                self.v[base + i][m] = val[i][m]

    def mask_to_int(self, b):
        out = 0
        m = self.lane_mask()
        for i in range(LANES):
            if b[i] and m[i]:
                out |= 1 << i
        return out

    # ---- pending-result machinery ----
    def _mark(self, table, first, n, d):
        for i in range(first, first + n):
            table[i] = table.get(i, 0) + d

    def retire_lds(self):
        first, n, data = self.lds_q.pop(0)
        for i in range(n):
            self.v[first + i] = data[i]
        self._mark(self.pend_v, first, n, -1)

    def retire_smem(self):
        first, data = self.smem_q.pop(0)
        for i, x in enumerate(data):
            self.s[first + i] = x
        self._mark(self.pend_s, first, len(data), -1)

    def retire_vm(self):
        item = self.vm_q.pop(0)
        if item[0] == "v":
            _, first, data, mask = item
            for i in range(data.shape[0]):
                self.v[first + i][mask] = data[i][mask]
            self._mark(self.pend_v, first, data.shape[0], -1)
        elif item[0] == "lds":
            _, writes = item
            if writes is not None:
                for addr, chunk in writes:
                    self.wg.lds_write(addr, chunk)
        # stores retire with no effect (already applied)

    def waitcnt(self, vm, lgkm):
        if vm is not None:
            while len(self.vm_q) > vm:
                self.retire_vm()
        if lgkm is not None:
            while len(self.lds_q) + len(self.smem_q) > lgkm:
                if self.smem_q and (self.wg.smem_first or not self.lds_q):
                    self.retire_smem()
                else:
                    self.retire_lds()

    # ---- execution ----
    def step(self):
        ins = self.wg.ins
        if self.pc >= len(ins):
            raise EmuError("ran off the end")
        mnem, ops, mods = ins[self.pc]
        self.icount += 1
        nxt = self.pc + 1
        W = self
        try:
            nxt = self.execute(mnem, ops, mods, nxt)
        except EmuError:
            raise
        except Exception as e:  # noqa: BLE001
            raise EmuError(f"wave {self.id} pc {self.pc} `{mnem} {', '.join(ops)}`: {type(e).__name__}: {e}") from e
        self.pc = nxt

    def execute(self, mnem, ops, mods, nxt):
        S, V = self.ssrc, self.src
        lab = self.wg.labels

        # ---------------- program flow / sync
        if mnem == "s_endpgm":
            self.done = True
            return nxt
        if mnem == "s_barrier":
            self.at_barrier = True
            return nxt
        if mnem == "s_nop":
            return nxt
        if mnem == "s_waitcnt":
            vm = lg = None
            for o in ops + [k for k in mods]:
                m = re.match(r"(vmcnt|lgkmcnt)\((\d+)\)", o)
                if m:
                    if m.group(1) == "vmcnt":
                        vm = int(m.group(2))
                    else:
                        lg = int(m.group(2))
            self.waitcnt(vm, lg)
            return nxt
        if mnem == "s_branch":
            return lab[ops[0]]
        if mnem.startswith("s_cbranch_"):
            cond = {"scc0": self.scc == 0, "scc1": self.scc == 1, "execz": self.exec == 0,
                    "execnz": self.exec != 0, "vccz": self.vcc == 0, "vccnz": self.vcc != 0}[mnem[len("s_cbranch_"):]]
            return lab[ops[0]] if cond else nxt

        # ---------------- SMEM
        if mnem.startswith("s_load_dword"):
            n = {"s_load_dword": 1, "s_load_dwordx2": 2, "s_load_dwordx4": 4, "s_load_dwordx8": 8,
                 "s_load_dwordx16": 16}[mnem]
            kind, first, cnt, _ = parse_reg(ops[0])
            base = S(ops[1])
            off = S(ops[2])
            raw = self.wg.mem.read(base + off, 4 * n)
            data = np.frombuffer(raw.tobytes(), dtype=U32).copy()
            self.smem_q.append((first, data))
            self._mark(self.pend_s, first, n, +1)
            return nxt

        # ---------------- SALU
        if mnem in ("s_mov_b32", "s_mov_b64"):
            val = S(ops[1])
            if mnem == "s_mov_b64" and re.fullmatch(r"-\d+", ops[1]):
                val = int(ops[1]) & ((1 << 64) - 1)          # a negative inline constant is sign-extended to 64 bits
            self.sdst(ops[0], val)
            return nxt
        if mnem in ("s_and_b32", "s_or_b32", "s_andn2_b32", "s_and_b64", "s_or_b64"):
            a, b = S(ops[1]), S(ops[2])
            if mnem.startswith("s_and_b"):
                r = a & b
            elif mnem.startswith("s_or_b"):
                r = a | b
            else:
                r = a & ~b & MASK32
            self.sdst(ops[0], r)
            self.scc = int(r != 0)
            return nxt
        if mnem in ("s_lshr_b32", "s_lshl_b32"):
            a, b = S(ops[1]), S(ops[2]) & 31
            r = (a >> b) if mnem == "s_lshr_b32" else (a << b) & MASK32
            self.sdst(ops[0], r)
            self.scc = int(r != 0)
            return nxt
        if mnem == "s_lshl_b64":
            a, b = S(ops[1]), S(ops[2]) & 63
            r = (a << b) & ((1 << 64) - 1)
            self.sdst(ops[0], r)
            self.scc = int(r != 0)
            return nxt
        if mnem in ("s_add_u32", "s_addc_u32", "s_sub_u32", "s_add_i32", "s_sub_i32"):
            a, b = S(ops[1]), S(ops[2])
            if mnem == "s_add_u32":
                r = a + b
                self.scc = int(r > MASK32)
            elif mnem == "s_addc_u32":
                r = a + b + self.scc
                self.scc = int(r > MASK32)
            elif mnem == "s_sub_u32":
                r = a - b
                self.scc = int(b > a)
            elif mnem == "s_add_i32":
                r = a + b
                sa, sb = a >> 31, b >> 31
                self.scc = int(sa == sb and ((r >> 31) & 1) != sa)
            else:
                r = a - b
                sa, sb = a >> 31, b >> 31
                self.scc = int(sa != sb and ((r >> 31) & 1) != sa)
            self.sdst(ops[0], r & MASK32)
            return nxt
        if mnem == "s_mul_i32":
            self.sdst(ops[0], (S(ops[1]) * S(ops[2])) & MASK32)
            return nxt
        if mnem == "s_mul_hi_u32":
            self.sdst(ops[0], (S(ops[1]) * S(ops[2])) >> 32)
            return nxt
        if mnem in ("s_min_i32", "s_max_i32"):
            a, b = S(ops[1]), S(ops[2])
            sa = a - (1 << 32) if a >> 31 else a
            sb = b - (1 << 32) if b >> 31 else b
            first = sa < sb if mnem == "s_min_i32" else sa > sb
            self.sdst(ops[0], a if first else b)
            self.scc = int(first)
            return nxt
        if mnem == "s_min_u32":
            a, b = S(ops[1]), S(ops[2])
            self.sdst(ops[0], min(a, b))
            self.scc = int(a < b)
            return nxt
        if mnem == "s_cselect_b32":
            self.sdst(ops[0], S(ops[1]) if self.scc else S(ops[2]))
            return nxt
        if mnem.startswith("s_cmp_"):
            a, b = S(ops[0]), S(ops[1])
            op = mnem[len("s_cmp_"):]
            cmp, ty = op.rsplit("_", 1)
            if ty == "i32":
                a = a - (1 << 32) if a >> 31 else a
                b = b - (1 << 32) if b >> 31 else b
            self.scc = int({"eq": a == b, "lg": a != b, "ge": a >= b, "gt": a > b, "le": a <= b, "lt": a < b}[cmp])
            return nxt
        if mnem == "s_bitcmp1_b32":
            self.scc = (S(ops[0]) >> (S(ops[1]) & 31)) & 1
            return nxt
        if mnem == "s_and_saveexec_b64":
            old = self.exec
            self.sdst(ops[0], old)
            self.exec = old & S(ops[1])
            self.scc = int(self.exec != 0)
            return nxt

        # ---------------- LDS
        if mnem == "ds_read_b128":
            kind, first, cnt, _ = parse_reg(ops[0])
            addr = V(ops[1]).astype(np.int64) + mods.get("offset", 0)
            data = np.zeros((4, LANES), dtype=U32)
            for l in range(LANES):
                if addr[l] % 16:
                    raise EmuError(f"misaligned ds_read_b128 at {addr[l]}")
                data[:, l] = np.frombuffer(self.wg.lds_read(int(addr[l]), 16).tobytes(), dtype=U32)
            self.lds_q.append((first, 4, data))
            self._mark(self.pend_v, first, 4, +1)
            return nxt
        if mnem == "ds_read_b64_tr_b16":
            kind, first, cnt, _ = parse_reg(ops[0])
            addr = V(ops[1]).astype(np.int64) + mods.get("offset", 0)
            elems = np.zeros((LANES, 4), dtype=np.uint16)
            for l in range(LANES):
                if addr[l] % 8:
                    raise EmuError(f"misaligned ds_read_b64_tr_b16 at {addr[l]}")
                elems[l] = np.frombuffer(self.wg.lds_read(int(addr[l]), 8).tobytes(), dtype=np.uint16)
            out = np.zeros((LANES, 4), dtype=np.uint16)
            for l in range(LANES):
                g, i = l // 16, l % 16
                for j in range(4):
                    out[l, j] = elems[g * 16 + (i // 4) + 4 * j, i % 4]
            data = np.zeros((2, LANES), dtype=U32)
            data[0] = out[:, 0].astype(U32) | (out[:, 1].astype(U32) << 16)
            data[1] = out[:, 2].astype(U32) | (out[:, 3].astype(U32) << 16)
            self.lds_q.append((first, 2, data))
            self._mark(self.pend_v, first, 2, +1)
            return nxt

        # ---------------- VMEM
        if mnem == "global_load_lds_dwordx4":
            voff = V(ops[0]).astype(np.int64)
            base = S(ops[1])
            writes = []
            m = self.lane_mask()
            for l in range(LANES):
                if m[l]:
                    chunk = self.wg.mem.read(base + int(voff[l]) + mods.get("offset", 0), 16).copy()
                    writes.append((self.m0 + mods.get("offset", 0) + 16 * l, chunk))
            if self.wg.dma_late:
                self.vm_q.append(("lds", writes))
            else:
                for addr, chunk in writes:
                    self.wg.lds_write(addr, chunk)
                self.vm_q.append(("lds", None))
            return nxt
        if mnem == "global_load_dwordx4":
            kind, first, cnt, _ = parse_reg(ops[0])
            a = V(ops[1])
            addr = a[0].astype(np.int64) | (a[1].astype(np.int64) << 32)
            data = np.zeros((4, LANES), dtype=U32)
            m = self.lane_mask()
            for l in range(LANES):
                if m[l]:
                    data[:, l] = np.frombuffer(self.wg.mem.read(int(addr[l]) + mods.get("offset", 0), 16).tobytes(), dtype=U32)
            self.vm_q.append(("v", first, data, m))
            self._mark(self.pend_v, first, 4, +1)
            return nxt
        if mnem.startswith("global_store_dword"):
            n = {"global_store_dword": 1, "global_store_dwordx2": 2, "global_store_dwordx4": 4}[mnem]
            m = self.lane_mask()
            data = V(ops[1])
            if n == 1:
                data = data[None, :]
            if ops[2] == "off":
                a = V(ops[0])
                addr = a[0].astype(np.int64) | (a[1].astype(np.int64) << 32)
            else:
                addr = V(ops[0]).astype(np.int64) + S(ops[2])
            for l in range(LANES):
                if m[l]:
                    self.wg.mem.write(int(addr[l]) + mods.get("offset", 0),
                                      np.frombuffer(np.ascontiguousarray(data[:, l]).tobytes(), dtype=np.uint8))
            self.vm_q.append(("st",))
            return nxt

        # ---------------- MFMA
        if mnem == "v_mfma_f32_32x32x16_bf16":
            A, B = V(ops[1]), V(ops[2])
            rc = parse_reg(ops[3])
            C = V(ops[3]) if rc else np.zeros((16, LANES), dtype=U32)
            def halves(X):
                lo = bf16_to_f32(X & np.uint32(0xFFFF)).astype(np.float64)
                hi = bf16_to_f32(X >> np.uint32(16)).astype(np.float64)
                out = np.empty((8, LANES))
                out[0::2], out[1::2] = lo, hi
                return out
            av, bv = halves(A), halves(B)
            a_mat = np.concatenate([av[:, :32].T, av[:, 32:].T], axis=1)      # [32 rows, 16 k]
            b_mat = np.concatenate([bv[:, :32], bv[:, 32:]], axis=0)          # [16 k, 32 cols]
            prod = a_mat @ b_mat
            r_idx = np.arange(16)[:, None]
            l_idx = np.arange(LANES)[None, :]
            rows = 8 * (r_idx // 4) + 4 * (l_idx // 32) + (r_idx % 4)
            cf = f32(C).astype(np.float64)
            D = bits((cf + prod[rows, l_idx % 32]).astype(np.float32))
            self.vdst(ops[0], D, masked=False)
            return nxt

        # ---------------- VALU
        if mnem in ("v_accvgpr_write_b32", "v_accvgpr_read_b32", "v_mov_b32"):
            self.vdst(ops[0], V(ops[1]))
            return nxt
        if mnem == "v_ldexp_f32":
            x = f32(V(ops[1])).astype(np.float64)
            n = V(ops[2]).astype(np.int32).astype(np.int64)
            with np.errstate(over="ignore", under="ignore"):
                self.vdst(ops[0], bits(np.ldexp(x, np.clip(n, -300, 300)).astype(np.float32)))
            return nxt
        if mnem == "v_readfirstlane_b32":
            x = V(ops[1])
            lane = next((i for i in range(LANES) if (self.exec >> i) & 1), 0)
            self.sdst(ops[0], int(x[lane]))
            return nxt
        if mnem in ("v_and_b32", "v_or_b32", "v_add_u32", "v_sub_u32", "v_mul_u32_u24", "v_min_u32", "v_max_i32",
                    "v_lshrrev_b32", "v_lshlrev_b32"):
            a, b = V(ops[1]).astype(np.uint64), V(ops[2]).astype(np.uint64)
            if mnem == "v_and_b32":
                r = a & b
            elif mnem == "v_or_b32":
                r = a | b
            elif mnem == "v_add_u32":
                r = a + b
            elif mnem == "v_sub_u32":
                r = a - b
            elif mnem == "v_mul_u32_u24":
                r = (a & 0xFFFFFF) * (b & 0xFFFFFF)
            elif mnem == "v_min_u32":
                r = np.minimum(a, b)
            elif mnem == "v_max_i32":
                r = np.maximum(a.astype(U32).view(np.int32), b.astype(U32).view(np.int32)).view(U32).astype(np.uint64)
            elif mnem == "v_lshrrev_b32":
                r = b >> (a & 31)
            else:
                r = b << (a & 31)
            self.vdst(ops[0], (r & MASK32).astype(U32))
            return nxt
        if mnem == "v_lshl_add_u32":
            a, b, c = (V(o).astype(np.uint64) for o in ops[1:4])
            self.vdst(ops[0], (((a << (b & 31)) + c) & MASK32).astype(U32))
            return nxt
        if mnem == "v_add_i32":
            a = V(ops[1]).view(np.int32).astype(np.int64)
            b = V(ops[2]).view(np.int32).astype(np.int64)
            r = a + b
            if mods.get("clamp"):
                r = np.clip(r, -2 ** 31, 2 ** 31 - 1)
            self.vdst(ops[0], (r & MASK32).astype(U32))
            return nxt
        if mnem == "v_mad_u64_u32":
            a, b = V(ops[2]).astype(np.uint64), V(ops[3]).astype(np.uint64)
            c = S(ops[4]) if parse_reg(ops[4]) and parse_reg(ops[4])[0] == "s" else None
            if c is None:
                cc = V(ops[4])
                c = cc[0].astype(np.uint64) | (cc[1].astype(np.uint64) << np.uint64(32))
            r = a * b + np.uint64(c) if not isinstance(c, np.ndarray) else a * b + c
            self.vdst(ops[0], np.stack([(r & np.uint64(MASK32)).astype(U32), (r >> np.uint64(32)).astype(U32)]))
            self.sdst(ops[1], 0)
            return nxt
        if mnem == "v_add_co_u32":
            a, b = V(ops[2]).astype(np.uint64), V(ops[3]).astype(np.uint64)
            r = a + b
            self.vdst(ops[0], (r & MASK32).astype(U32))
            self.sdst(ops[1], self.mask_to_int(r > MASK32))
            return nxt
        if mnem == "v_addc_co_u32":
            a, b = V(ops[2]).astype(np.uint64), V(ops[3]).astype(np.uint64)
            cin = S(ops[4])
            carry = np.array([(cin >> i) & 1 for i in range(LANES)], dtype=np.uint64)
            r = a + b + carry
            self.vdst(ops[0], (r & MASK32).astype(U32))
            self.sdst(ops[1], self.mask_to_int(r > MASK32))
            return nxt
        if mnem in ("v_mbcnt_lo_u32_b32", "v_mbcnt_hi_u32_b32"):
            mask = V(ops[1]).astype(np.uint64)
            acc = V(ops[2]).astype(np.uint64)
            out = np.zeros(LANES, dtype=np.uint64)
            for l in range(LANES):
                if mnem.endswith("lo_u32_b32"):
                    below = ((1 << min(l, 32)) - 1)
                else:
                    below = ((1 << max(l - 32, 0)) - 1)
                out[l] = bin(int(mask[l]) & below).count("1") + acc[l]
            self.vdst(ops[0], out.astype(U32))
            return nxt
        if mnem == "v_cndmask_b32":
            a, b = V(ops[1]), V(ops[2])
            sel = S(ops[3])
            pick = np.array([(sel >> i) & 1 for i in range(LANES)], dtype=bool)
            self.vdst(ops[0], np.where(pick, b, a))
            return nxt
        if mnem.startswith("v_cmp_"):
            op = mnem[len("v_cmp_"):]
            cmp, ty = op.rsplit("_", 1)
            a, b = V(ops[1]), V(ops[2])
            if ty == "f32":
                a, b = f32(a), f32(b)
            elif ty == "i32":
                a, b = a.view(np.int32), b.view(np.int32)
            with np.errstate(invalid="ignore"):
                res = {"gt": a > b, "lt": a < b, "ge": a >= b, "le": a <= b, "eq": a == b, "ne": a != b,
                       "neq": ~(a == b), "lg": a != b}[cmp]
            self.sdst(ops[0], self.mask_to_int(res))
            return nxt
        if mnem == "v_permlane32_swap_b32":
            kind0, f0, _, _ = parse_reg(ops[0])
            kind1, f1, _, _ = parse_reg(ops[1])
            self.chk_v(f0)
            self.chk_v(f1)
            a, b = self.v[f0].copy(), self.v[f1].copy()
            a_new, b_new = a.copy(), b.copy()
            a_new[32:] = b[:32]
            b_new[:32] = a[32:]
            self.v[f0], self.v[f1] = a_new, b_new
            return nxt
        # float ops
        with np.errstate(all="ignore"):
            if mnem in ("v_add_f32", "v_sub_f32", "v_mul_f32", "v_max_f32", "v_min_f32"):
                a, b = f32(V(ops[1])), f32(V(ops[2]))
                r = {"v_add_f32": lambda: a + b, "v_sub_f32": lambda: a - b, "v_mul_f32": lambda: a * b,
                     "v_max_f32": lambda: np.fmax(a, b), "v_min_f32": lambda: np.fmin(a, b)}[mnem]()
                self.vdst(ops[0], bits(r.astype(np.float32)))
                return nxt
            if mnem == "v_max3_f32":
                a, b, c = (f32(V(o)) for o in ops[1:4])
                self.vdst(ops[0], bits(np.fmax(np.fmax(a, b), c)))
                return nxt
            if mnem == "v_fma_f32":
                a, b, c = (f32(V(o)).astype(np.float64) for o in ops[1:4])
                self.vdst(ops[0], bits((a * b + c).astype(np.float32)))
                return nxt
            if mnem == "v_rndne_f32":
                self.vdst(ops[0], bits(np.rint(f32(V(ops[1])))))
                return nxt
            if mnem == "v_exp_f32":
                self.vdst(ops[0], bits(np.exp2(f32(V(ops[1])).astype(np.float64)).astype(np.float32)))
                return nxt
            if mnem == "v_log_f32":
                self.vdst(ops[0], bits(np.log2(f32(V(ops[1])).astype(np.float64)).astype(np.float32)))
                return nxt
            if mnem == "v_rcp_f32":
                self.vdst(ops[0], bits((1.0 / f32(V(ops[1])).astype(np.float64)).astype(np.float32)))
                return nxt
            if mnem == "v_cvt_i32_f32":
                x = f32(V(ops[1])).astype(np.float64)
                x = np.where(np.isnan(x), 0, np.clip(np.trunc(x), -2 ** 31, 2 ** 31 - 1))
                self.vdst(ops[0], (x.astype(np.int64) & MASK32).astype(U32))
                return nxt
            if mnem in ("v_cvt_f32_i32", "v_cvt_f32_u32"):
                x = V(ops[1])
                x = x.view(np.int32) if mnem.endswith("i32") else x
                self.vdst(ops[0], bits(x.astype(np.float32)))
                return nxt
            if mnem == "v_cvt_pk_bf16_f32":
                lo, hi = f32_to_bf16(f32(V(ops[1]))), f32_to_bf16(f32(V(ops[2])))
                self.vdst(ops[0], (lo | (hi << np.uint32(16))).astype(U32))
                return nxt
            if mnem == "v_dot2c_f32_bf16":
                a, b, c = V(ops[1]), V(ops[2]), f32(V(ops[0])).astype(np.float64)
                r = (bf16_to_f32(a & np.uint32(0xFFFF)).astype(np.float64) * bf16_to_f32(b & np.uint32(0xFFFF))
                     + bf16_to_f32(a >> np.uint32(16)).astype(np.float64) * bf16_to_f32(b >> np.uint32(16)) + c)
                self.vdst(ops[0], bits(r.astype(np.float32)))
                return nxt
            if mnem == "v_dot2_f32_bf16":
                a, b, c = V(ops[1]), V(ops[2]), f32(V(ops[3])).astype(np.float64)
                r = (bf16_to_f32(a & np.uint32(0xFFFF)).astype(np.float64) * bf16_to_f32(b & np.uint32(0xFFFF))
                     + bf16_to_f32(a >> np.uint32(16)).astype(np.float64) * bf16_to_f32(b >> np.uint32(16)) + c)
                self.vdst(ops[0], bits(r.astype(np.float32)))
                return nxt
        raise EmuError(f"unsupported instruction {mnem}")


class Workgroup:
    def __init__(self, ins, labels, mem, kernarg_addr, wg_x, wg_y, lds_bytes, dma_late=False, smem_first=False,
                 max_steps=400000):
        self.ins, self.labels, self.mem = ins, labels, mem
        self.lds = np.zeros(lds_bytes, dtype=np.uint8)
        self.lds_init = np.zeros(lds_bytes, dtype=bool)
        self.dma_late, self.smem_first = dma_late, smem_first
        self.waves = []
        self.max_steps = max_steps
        for w in range(4):
            wave = Wave(self, w)
            wave.s[0] = kernarg_addr & MASK32
            wave.s[1] = kernarg_addr >> 32
            wave.s[2] = wg_x
            wave.s[3] = wg_y
            # uninitialised registers hold arbitrary values: poison them so a stale read shows
            wave.s[4:] = 0xBAD00000 + np.arange(4, 128, dtype=U32)
            wave.vcc = 0xBAD0BAD0BAD0BAD0
            wave.m0 = 0xBAD0BAD0
            wave.scc = 1
            wave.v[:] = 0xDEAD0000 + np.arange(512, dtype=U32)[:, None]
            wave.v[0] = np.arange(LANES, dtype=U32) + 64 * w
            self.waves.append(wave)

    def lds_read(self, addr, n):
        if addr < 0 or addr + n > len(self.lds):
            raise EmuError(f"LDS read out of range at {addr}")
        if not self.lds_init[addr:addr + n].all():
            raise EmuError(f"LDS read of uninitialised bytes at {addr}")
        return self.lds[addr:addr + n]

    def lds_write(self, addr, data):
        if addr < 0 or addr + len(data) > len(self.lds):
            raise EmuError(f"LDS write out of range at {addr}")
        self.lds[addr:addr + len(data)] = data
        self.lds_init[addr:addr + len(data)] = True

    def run(self):
        steps = 0
        while not all(w.done for w in self.waves):
            progressed = False
            for w in self.waves:
                while not w.done and not w.at_barrier:
                    w.step()
                    steps += 1
                    progressed = True
                    if steps > self.max_steps:
                        raise EmuError("step limit exceeded (hang?)")
            live = [w for w in self.waves if not w.done]
            if live and all(w.at_barrier for w in live):
                for w in live:
                    w.at_barrier = False
                progressed = True
            if not progressed:
                raise EmuError("deadlock at barrier")
        return steps


# --------------------------------------------------------------------------------------------
# static hazard check over the instruction stream (straight-line distance, conservative)
# --------------------------------------------------------------------------------------------
def _regs_of(tok):
    if tok in ("vcc", "vcc_lo", "vcc_hi"):
        return {("s", 106), ("s", 107)} if tok == "vcc" else {("s", 106 if tok == "vcc_lo" else 107)}
    r = parse_reg(tok)
    if not r:
        return set()
    kind, first, cnt, _ = r
    return {(kind, first + i) for i in range(cnt)}


def _is_valu(m):
    return m.startswith("v_") and not m.startswith("v_mfma")


def _dst_src(mnem, ops):
    """(written registers, read registers) — enough for the hazard rules below."""
    if not ops:
        return set(), set()
    if mnem.startswith("global_store") or mnem.startswith("s_cmp") or mnem.startswith("s_cbranch") or \
            mnem in ("s_waitcnt", "s_nop", "s_barrier", "s_branch", "s_bitcmp1_b32"):
        rd = set()
        for o in ops:
            rd |= _regs_of(o)
        return set(), rd
    if mnem == "global_load_lds_dwordx4":
        return set(), _regs_of(ops[0]) | _regs_of(ops[1])
    wr = _regs_of(ops[0])
    start = 1
    if mnem in ("v_mad_u64_u32", "v_add_co_u32", "v_addc_co_u32"):
        wr |= _regs_of(ops[1])
        start = 2
    if mnem == "v_permlane32_swap_b32":
        wr |= _regs_of(ops[1])
        start = 0
    if mnem == "v_dot2c_f32_bf16":
        start = 0
    rd = set()
    for o in ops[start:]:
        rd |= _regs_of(o)
    return wr, rd


def check_hazards(ins, labels):
    """Returns a list of strings describing violated rules.  From every producer the following 40
    issue slots are walked along the fall-through path and along every branch target (forward or
    backward), counting one wait state per instruction plus the count of `s_nop`."""
    problems = []
    WINDOW = 40

    def cost(k):
        m, o, _ = ins[k]
        return (int(o[0], 0) + 1) if m == "s_nop" else 1

    def visit(i, m, ops, wr, j, gap, seen):
        """Walk consumers starting at instruction j, `gap` wait states after producer i."""
        while j < len(ins) and gap < WINDOW and wr:
            if (j, frozenset(wr)) in seen:
                return
            seen.add((j, frozenset(wr)))
            m2, ops2, _ = ins[j]
            wr2, rd2 = _dst_src(m2, ops2)
            hit = wr & rd2
            if hit:
                if _is_valu(m) and m2 in ("v_readfirstlane_b32", "v_readlane_b32") and gap < 1:
                    problems.append(f"{i}:{m} -> {j}:{m2}: needs a wait state")
                if _is_valu(m) and m2 == "v_permlane32_swap_b32" and gap < 2:
                    problems.append(f"{i}:{m} -> {j}:{m2}: needs two wait states")
                if m == "v_dot2c_f32_bf16" and gap < 3 and not (m2 == m and hit <= _regs_of(ops2[0])
                                                                and not hit & (_regs_of(ops2[1]) | _regs_of(ops2[2]))):
                    problems.append(f"{i}:{m} -> {j}:{m2}: dot result read after {gap} wait states")
                if _is_valu(m) and _is_valu(m2) and gap < 2 and any(k == "s" for k, _ in hit):
                    problems.append(f"{i}:{m} -> {j}:{m2}: VALU-written SGPR / VCC read by a VALU instruction after {gap} wait states")
                if m in TRANS and _is_valu(m2) and gap < 1:
                    problems.append(f"{i}:{m} -> {j}:{m2}: trans result used by the next VALU op")
                if m.startswith("v_mfma") and not m2.startswith("v_mfma") and gap < 18:
                    problems.append(f"{i}:{m} -> {j}:{m2}: MFMA result read after {gap} wait states")
                if m.startswith("v_mfma") and m2.startswith("v_mfma"):
                    a2 = _regs_of(ops2[1]) | _regs_of(ops2[2])     # only accumulate-into-itself may follow closely
                    if wr & a2 and gap < 18:
                        problems.append(f"{i}:{m} -> {j}:{m2}: MFMA result used as A/B operand")
                if _is_valu(m) and m2.startswith("v_mfma") and gap < 2:
                    problems.append(f"{i}:{m} -> {j}:{m2}: VALU result feeds MFMA after {gap} wait states")
                if (m.startswith("v_cmp") or m == "v_readfirstlane_b32") and m2.startswith("global_") and gap < 5 \
                        and any(k == "s" for k, _ in hit):
                    problems.append(f"{i}:{m} -> {j}:{m2}: VALU-written SGPR used by VMEM")
            if ops and ops[0] == "m0" and m.startswith("s_") and m2 == "global_load_lds_dwordx4" and gap < 1:
                problems.append(f"{i}:{m} -> {j}:{m2}: M0 write directly before LDS DMA")
            if m.startswith("v_mfma") and not m2.startswith("v_mfma") and wr & wr2 and not hit and gap < 18:
                problems.append(f"{i}:{m} -> {j}:{m2}: MFMA result overwritten after {gap} wait states")
            if m == "v_dot2c_f32_bf16" and wr & wr2 and not hit and gap < 3:
                problems.append(f"{i}:{m} -> {j}:{m2}: dot result overwritten after {gap} wait states")
            wr = wr - wr2 if not hit else wr                       # a later overwrite ends the window
            if m2 == "s_endpgm":
                return
            if m2 == "s_branch":
                j = labels[ops2[0]]
                gap += 1
                continue
            if m2.startswith("s_cbranch"):
                visit(i, m, ops, set(wr), labels[ops2[0]], gap + 1, seen)
            gap += cost(j)
            j += 1

    for i, (m, ops, mods) in enumerate(ins):
        wr, _ = _dst_src(m, ops)
        if m in ("global_store_dwordx3", "global_store_dwordx4") and i + 1 < len(ins):
            m2, ops2, _ = ins[i + 1]                               # wide store data must survive one more slot
            if _is_valu(m2) and _dst_src(m2, ops2)[0] & _regs_of(ops[1]):
                problems.append(f"{i}:{m} -> {i + 1}:{m2}: store data overwritten in the next slot")
        if ops and ops[0] == "m0":
            wr = wr | {("m", 0)}
        if wr:
            visit(i, m, ops, set(wr), i + 1, 0, set())
    return sorted(set(problems))
