#!/usr/bin/env python3
"""Writes fa_attention_wide64_loop.inc: the check-free main loop of fa_fwd_wide64_kernel as one inline-assembly
block per storage type -- the software-pipelined form of the attention loop for waves of 64 query rows (two 32-row
blocks rb = 0, 1 that share every K and V fragment read from LDS).  One wave per SIMD, the whole register file.

Why assembly, and why generated: with one wave per SIMD nothing hides a wave's vector work but the wave itself, so
the instruction stream has to alternate -- one matrix instruction, then about as many vector / LDS / load
instructions as issue while it runs, then the next -- with three pieces of work in flight that do not depend on
each other.  The compiler's scheduler undoes such an interleaving and the rotating buffers confuse its register
allocator, hence fixed registers and a fixed order; the loop is regular, hence written by a script.  The build runs
this script (paper_2410_16663_amd/build.py); the .inc file is its output and is not kept under version control.

Register plan (per lane):
    a0   .. a127   O accumulators, O[rb][db] = a[64*rb + 16*db : +15]        (outputs of the block)
    a128 .. a191   Q fragments,    Q[rb][kb] = a[128 + 32*rb + 4*kb : +3]    (inputs)
    v0   .. v127   four unit buffers x two row blocks, X[b][rb] = v[32*b + 16*rb : +15]: unit u lives in X[u % 4],
                   first as logits, then (overwritten in place) as packed exponentials P[jj] = first 4 registers of
                   each half
    v128 .. v143   four K fragments in flight;   v144 .. v159   four V^T fragments in flight
    v160+rb m_ref, v162+rb l_run, v164+rb l_rnd                               (outputs)
    v166, v167     K fragment address, even (input) / odd k-step
    v168 .. v171   V^T fragment address per 32-row block of O^T (v168 input)
    v172, v173     per-lane byte offsets of the K and V loads from global memory (inputs)
    v174 .. v185   temporaries, six per row block;   v186 .. v193   per-lane offsets of the four loads per tensor
Scalar registers s60 .. s69 are scratch of the block.

A UNIT is 32 keys x the wave's 64 rows.  In step u the wave issues
    the 16 matrix instructions of unit u+1's logits   S(u+1) = K Q^T,
    the 16 matrix instructions of unit u-1's second product   O += V^T P(u-1),
    and BETWEEN them the ~150 vector instructions of unit u's softmax   S(u) -> P(u)   (both row blocks), the
    LDS reads of the fragments three matrix-instruction pairs ahead, and this wave's share of a tile's loads,
each matrix instruction followed by at most CAP cycles' worth of the others (by a simple cost table; the best CAP
was found by timing).  The test "row sum <= 256" (which proves that no exponential exceeded 256, see the kernel)
is computed at the end of the step's vector work and branched on after its last matrix instruction; the rare other
case runs a block out of line that recomputes the unit's logits, takes the row maxima, moves the references,
rescales the accumulators (through v_accvgpr_read / write) and redoes the exponentials.

LDS: four stages of (K tile, V tile); tile t lives in stage t % 4.  Barrier k (the k-th of the walk, the same count
as in the compiler-scheduled loop around this block) publishes tile k+1 and certifies that no wave reads tile k-1
any more; between barrier k and barrier k+1 every wave issues its share (four loads per tensor) of tile k+3.

Steps: the block computes S(0), runs step 0 (no second product yet), then the steady loop -- eight steps per pass,
so that buffers and stages come round to where they started -- and leaves after step 2J-1 (J = number of tiles, even)
through one of two exits, each followed by the second product of the last unit.

Hazards the hardware does not interlock, spaced by hand: 11 wait states between a matrix instruction and a vector
instruction touching its result (here: always a whole step apart, except in the blocks out of line, which wait);
results of v_exp_f32 are consumed several instructions later; 3 wait states between a dot-product instruction and
another kind of instruction reading its result, 2 between v_cvt_pk and the dot product reading it; 2 around
v_permlane32_swap.
"""
import os

KB, DB = 8, 4
KBLK = 1088
KTILEB = 16 * KBLK      # 17408
TILEB = 16384
NSTAGE = 4
CAP = 30                # cycles of other instructions issued behind a matrix instruction (measured best of 22..60)
NW = 4                  # waves per workgroup
NI = 16 // NW           # load instructions per wave, tensor and tile


def O(rb, db):
    r = 64 * rb + 16 * db
    return f"a[{r}:{r + 15}]"


def Q(rb, kb):
    r = 128 + 32 * rb + 4 * kb
    return f"a[{r}:{r + 3}]"


def X(b, rb):
    r = 32 * b + 16 * rb
    return f"v[{r}:{r + 15}]"


def x(b, rb, i):
    return f"v{32 * b + 16 * rb + i}"


def P(b, rb, jj):
    r = 32 * b + 16 * rb + 8 * jj
    return f"v[{r}:{r + 3}]"


def KF(b):
    return f"v[{128 + 4 * b}:{128 + 4 * b + 3}]"


def VF(b):
    return f"v[{144 + 4 * b}:{144 + 4 * b + 3}]"


def VFlo(b):
    return f"v[{144 + 4 * b}:{144 + 4 * b + 1}]"


def VFhi(b):
    return f"v[{144 + 4 * b + 2}:{144 + 4 * b + 3}]"


M_REF = lambda rb: f"v{160 + rb}"
L_RUN = lambda rb: f"v{162 + rb}"
L_RND = lambda rb: f"v{164 + rb}"
KADDR = lambda odd: f"v{166 + odd}"
VADDR = lambda db: f"v{168 + db}"
KVOFF, VVOFF = "v172", "v173"
T = lambda rb, i: f"v{174 + 6 * rb + i}"
DMAOFF = lambda tensor, n: f"v{186 + 4 * tensor + n}"     # per-lane byte offset of load n of a K / V tile


class Gen:
    def __init__(self, bf16):
        self.bf16 = bf16
        self.mfma = "v_mfma_f32_32x32x16_bf16" if bf16 else "v_mfma_f32_32x32x16_f16"
        self.cvt = "v_cvt_pk_bf16_f32" if bf16 else "v_cvt_pk_f16_f32"
        self.dot = "v_dot2c_f32_bf16_e32" if bf16 else "v_dot2c_f32_f16_e32"
        self.ones = "0x3f803f80" if bf16 else "0x3c003c00"
        self.out = []
        self.cold = []
        self.queue = []          # ids of LDS reads in flight, oldest first
        self.next_id = 0
        self.nlabel = 0

    def emit(self, line):
        self.out.append(line)

    # ---- LDS reads and the waits for them (reads return in order)
    def lds_read(self, text):
        self.emit(text)
        self.queue.append(self.next_id)
        self.next_id += 1
        return self.next_id - 1

    def wait_for(self, rid):
        if rid not in self.queue:
            return
        i = self.queue.index(rid)
        n_after = len(self.queue) - 1 - i
        assert n_after <= 15
        self.emit(f"s_waitcnt lgkmcnt({n_after})")
        self.queue = self.queue[i + 1:]

    def k_read(self, unit, kb):
        st, c = (unit >> 1) % NSTAGE, unit & 1
        off = st * KTILEB + c * 8 * KBLK + (kb >> 1) * 64
        return self.lds_read(f"ds_read_b128 {KF(kb % 4)}, {KADDR(kb & 1)} offset:{off}")

    def v_read(self, unit, g):
        st, c = (unit >> 1) % NSTAGE, unit & 1
        jj, db = g // DB, g % DB
        off = st * TILEB + 4096 * (2 * c + jj)
        self.lds_read(f"ds_read_b64_tr_b16 {VFlo(g % 4)}, {VADDR(db)} offset:{off}")
        return self.lds_read(f"ds_read_b64_tr_b16 {VFhi(g % 4)}, {VADDR(db)} offset:{off + 2048}")

    # ---- the vector work of one unit and row block, as a list of instructions (buffer b)
    def softmax_list(self, b, rb, interleave=True):
        """In place: logits X[b][rb] -> exponentials against the current reference, packed as P[b][rb][0..1]; leaves
        the unit's sums in temporaries: T0, T1 = partial sums of the exponentials (bf16; fp16: of the rounded ones),
        and for bf16 T2, T3 = partial sums of the rounded ones.  The exponentials of one group of four elements
        alternate with the additions / conversions of the previous group."""
        L = []
        ta, tb, tc, td = T(rb, 0), T(rb, 1), T(rb, 2), T(rb, 3)
        if self.bf16:
            L += [f"v_mov_b32 {tc}, 0", f"v_mov_b32 {td}, 0"]
        else:
            L += [f"v_mov_b32 {ta}, 0", f"v_mov_b32 {tb}, 0"]

        def consume_parts(g):          # elements 4g .. 4g+3: two pairs -> ([adds+cvt of pair 0], [.. pair 1], [dots])
            parts, dots = [], []
            for pr in (2 * g, 2 * g + 1):          # pair pr = elements 2pr, 2pr+1 -> register 8*jj + v2
                jj, v2 = pr // 4, pr % 4
                a, bb = x(b, rb, 2 * pr), x(b, rb, 2 * pr + 1)
                dst = x(b, rb, 8 * jj + v2)
                one = []
                if self.bf16:
                    acc = ta if pr % 2 == 0 else tb
                    if pr < 2:
                        one.append(f"v_add_f32 {acc}, {a}, {bb}")
                    else:
                        one.append(f"v_add_f32 {acc}, {acc}, {a}")
                        one.append(f"v_add_f32 {acc}, {acc}, {bb}")
                one.append(f"{self.cvt} {dst}, {a}, {bb}")
                parts.append(one)
                acc = (tc if pr % 2 == 0 else td) if self.bf16 else (ta if pr % 2 == 0 else tb)
                dots.append(f"{self.dot} {acc}, {self.ones}, {dst}")
            return parts[0], parts[1], dots

        for g in range(4):
            for i in range(4 * g, 4 * g + 4):
                L.append(f"v_fma_f32 {x(b, rb, i)}, {x(b, rb, i)}, %[c], -{M_REF(rb)}")
            ex = [f"v_exp_f32 {x(b, rb, i)}, {x(b, rb, i)}" for i in range(4 * g, 4 * g + 4)]
            if g == 0:
                L += ex
            else:
                p0, p1, dots = consume_parts(g - 1)
                # the dot products read what the conversions wrote at least two instructions earlier
                L += [ex[0]] + p0 + [ex[1]] + p1 + [ex[2], ex[3]] + dots
        p0, p1, dots = consume_parts(3)
        L += ["s_nop 1"] + p0 + p1 + ["s_nop 1"] + dots
        return L

    def softmax_both(self, b):
        """The two row blocks' lists, interleaved four instructions at a time (they share no register, so every
        distance inside a list only grows)."""
        A, B = self.softmax_list(b, 0), self.softmax_list(b, 1)
        L = []
        for i in range(0, max(len(A), len(B)), 4):
            L += A[i:i + 4]
            L += B[i:i + 4]
        return L

    def pending_sums(self):
        """Adds the previous unit's sums (left in the temporaries by its vector work and its check) to the running
        sums: the first vector instructions of the next step, or of the drain."""
        L = []
        for rb in (0, 1):
            ta, tb, tc, td = T(rb, 0), T(rb, 1), T(rb, 2), T(rb, 3)
            L.append(f"v_add_f32 {L_RUN(rb)}, {L_RUN(rb)}, {ta}")
            if self.bf16:
                L.append(f"v_add_f32 {tc}, {tc}, {td}")
        if self.bf16:
            for rb in (0, 1):
                L.append(f"v_add_f32 {L_RND(rb)}, {L_RND(rb)}, {T(rb, 2)}")
        return L

    def check_list(self):
        """Both row blocks' sums and the test sum <= 256 (which proves that no exponential exceeded 256), leaving the
        outcome in vcc: the last vector instructions of a step."""
        L = ["s_nop 3"]
        for rb in (0, 1):
            L.append(f"v_add_f32 {T(rb, 0)}, {T(rb, 0)}, {T(rb, 1)}")
        L.append(f"v_cmp_nge_f32 vcc, 0x43800000, {T(0, 0)}")        # not (256 >= sum): also true for inf and NaN
        L.append("s_mov_b64 s[68:69], vcc")
        L.append(f"v_cmp_nge_f32 vcc, 0x43800000, {T(1, 0)}")
        L.append("s_or_b64 vcc, vcc, s[68:69]")
        return L

    def finish_sums(self, unit, inflight_text):
        """After the step's last matrix instruction: if some sum exceeded 256, a block out of line computes both row
        blocks' logits again, moves the references up to the row maxima, rescales, and redoes the exponentials."""
        e = self.emit
        b = unit % 4
        k = self.nlabel
        self.nlabel += 1
        e(f"s_cbranch_vccnz .Lfw64_redo_{k}_%=")
        e(f".Lfw64_back_{k}_%=:")
        # ---- the block out of line
        main, self.out = self.out, []
        st, c = (unit >> 1) % NSTAGE, unit & 1
        e(f".Lfw64_redo_{k}_%=:")
        e("s_waitcnt lgkmcnt(0)")
        for rb in (0, 1):
            ta, tb = T(rb, 0), T(rb, 1)
            t4, t5 = T(rb, 4), T(rb, 5)
            for kb in range(KB):
                off = st * KTILEB + c * 8 * KBLK + (kb >> 1) * 64
                e(f"ds_read_b128 {KF(3)}, {KADDR(kb & 1)} offset:{off}")
                e("s_waitcnt lgkmcnt(0)")
                e(f"{self.mfma} {X(b, rb)}, {KF(3)}, {Q(rb, kb)}, {'0' if kb == 0 else X(b, rb)}")
            e("s_nop 15")
            e("s_nop 3")
            e(f"v_max3_f32 {t4}, {x(b, rb, 0)}, {x(b, rb, 1)}, {x(b, rb, 2)}")
            for i in range(3, 15, 2):
                e(f"v_max3_f32 {t4}, {t4}, {x(b, rb, i)}, {x(b, rb, i + 1)}")
            e(f"v_max_f32 {t4}, {t4}, {x(b, rb, 15)}")
            e(f"v_mov_b32 {t5}, {t4}")
            e("s_nop 1")
            e(f"v_permlane32_swap_b32_e32 {t4}, {t5}")      # the two half-waves hold different keys of one query
            e("s_nop 1")
            e(f"v_max_f32 {t4}, {t4}, {t5}")
            e(f"v_mul_f32 {t4}, %[c], {t4}")                # in log2 units
            e(f"v_cmp_gt_f32 vcc, {t4}, {M_REF(rb)}")
            e(f"v_sub_f32 {t5}, {M_REF(rb)}, {t4}")
            e(f"v_exp_f32 {t5}, {t5}")
            e(f"v_cndmask_b32 {M_REF(rb)}, {M_REF(rb)}, {t4}, vcc")
            e("s_nop 1")
            e(f"v_cndmask_b32 {t5}, 1.0, {t5}, vcc")
            e(f"v_mul_f32 {L_RUN(rb)}, {t5}, {L_RUN(rb)}")
            if self.bf16:
                e(f"v_mul_f32 {L_RND(rb)}, {t5}, {L_RND(rb)}")
            # the accumulators live in AGPRs: out, times alpha, back in -- four at a time through the K fragment
            # registers of slot 3 (free here); the second products issued earlier in this step have long retired
            # (the 20 wait states above), and the matrix instructions that follow read them as their C operand
            tmp = [f"v{128 + 12 + i}" for i in range(4)]
            for i0 in range(0, 64, 4):
                for i in range(4):
                    e(f"v_accvgpr_read_b32 {tmp[i]}, a{64 * rb + i0 + i}")
                e("s_nop 0")
                for i in range(4):
                    e(f"v_mul_f32 {tmp[i]}, {t5}, {tmp[i]}")
                e("s_nop 0")
                for i in range(4):
                    e(f"v_accvgpr_write_b32 a{64 * rb + i0 + i}, {tmp[i]}")
            for ln in self.softmax_list(b, rb):
                e(ln)
            e("s_nop 3")
            e(f"v_add_f32 {ta}, {ta}, {tb}")
        for ln in inflight_text:
            e(ln)
        e("s_nop 7")
        e(f"s_branch .Lfw64_back_{k}_%=")
        self.cold += self.out
        self.out = main

    def dma_groups(self, tile):
        """This wave's share of the loads of a tile as a list of short groups of instructions (one load each, then
        the advance of the two tile pointers s[60:61] / s[62:63]), to be spread over a step."""
        st = tile % NSTAGE
        G = []
        for tensor in (0, 1):
            ptr = "s[60:61]" if tensor == 0 else "s[62:63]"
            for n in range(NI):
                if tensor == 0:
                    g = [f"s_add_u32 m0, %[ldsk], {st * KTILEB + NW * n * KBLK}"]
                else:
                    g = [f"s_add_u32 m0, %[ldsv], {st * TILEB + NW * n * 1024}"]
                g.append("s_nop 0")
                g.append(f"global_load_lds_dwordx4 {DMAOFF(tensor, n)}, {ptr} offset:0")
                G.append(g)
        G.append([f"s_add_u32 s60, s60, {TILEB}", "s_addc_u32 s61, s61, 0",
                  f"s_add_u32 s62, s62, {TILEB}", "s_addc_u32 s63, s63, 0"])
        return G

    @staticmethod
    def cost(ln):
        op = ln.split()[0]
        if op == "v_exp_f32":
            return 8
        if op == "s_nop":
            return int(ln.split()[1]) + 1
        if op.startswith("s_"):
            return 2
        return 4

    # ---- one step: logits of unit u+1, softmax of unit u, second product of unit u-1.
    # kpre: read ids of K fragments 0..2 of unit u+1, already issued.  dma: groups of load instructions to spread
    # over the step (the loads requested behind the barrier that ended the previous step).
    def step(self, u, kpre, with_pv=True, dma=()):
        e = self.emit
        valu = (self.pending_sums() if u > 0 else []) + self.softmax_both(u % 4) + self.check_list()
        # the load groups go in between, evenly
        groups = [[ln] for ln in valu]
        if dma:
            every = max(1, len(groups) // (len(dma) + 1))
            for gi, g in enumerate(dma):
                groups.insert(min(len(groups), (gi + 1) * every + gi), list(g))
        xq, xp = (u + 1) % 4, (u - 1) % 4
        if with_pv:
            slots = [("qk", 0), ("qk", 1), ("qk", 2)]
            for i in range(3, 8):
                slots += [("qk", i), ("pv", i - 3)]
            slots += [("pv", 5), ("pv", 6), ("pv", 7)]
        else:
            slots = [("qk", i) for i in range(8)]
        nsub = 2 * len(slots)                    # two matrix instructions per slot
        total = sum(self.cost(ln) for g in groups for ln in g)
        kids = dict(enumerate(kpre))
        vids = {}
        next_k = None
        inflight_next = []        # text of the next step's K prefetch, for the block out of line
        sub = 0
        done_cost = 0
        gi = 0
        for si, (kind, i) in enumerate(slots):
            for rb in (0, 1):
                n_before = len(self.out)
                if kind == "qk":
                    if rb == 0:
                        self.wait_for(kids[i])
                        n_before = len(self.out)
                    e(f"{self.mfma} {X(xq, rb)}, {KF(i % 4)}, {Q(rb, i)}, {'0' if i == 0 else X(xq, rb)}")
                    if rb == 1:
                        if i + 3 < KB:
                            kids[i + 3] = self.k_read(u + 1, i + 3)
                        if with_pv and i < 3:
                            vids[i] = self.v_read(u - 1, i)
                else:
                    if rb == 0:
                        self.wait_for(vids[i])
                        n_before = len(self.out)
                    jj, db = i // DB, i % DB
                    e(f"{self.mfma} {O(rb, db)}, {VF(i % 4)}, {P(xp, rb, jj)}, {O(rb, db)}")
                    if rb == 1 and i + 3 < 2 * DB:
                        vids[i + 3] = self.v_read(u - 1, i + 3)
                sub += 1
                # vector (and load) instructions behind this matrix instruction: as many as issue while it runs
                # (CAP cycles, less what the LDS reads just issued take), never fewer than an even share
                n_lds = len(self.out) - n_before - 1
                room = CAP - 4 * n_lds
                used = 0
                goal = total * sub / nsub
                while gi < len(groups):
                    c = sum(self.cost(l) for l in groups[gi])
                    if sub < nsub and used + c > room and done_cost + c / 2 > goal:
                        break
                    for ln in groups[gi]:
                        e(ln)
                    done_cost += c
                    used += c
                    gi += 1
        assert gi == len(groups)
        odd = u & 1
        if odd:
            # the next step's logits read the same tile: its first fragments go out now
            n0 = len(self.out)
            next_k = [self.k_read(u + 2, f) for f in range(3)]
            inflight_next = self.out[n0:]
        self.finish_sums(u, inflight_next)
        next_dma = []
        if not odd:
            # mid-tile barrier number u/2: tile u/2+1 is published (this wave's share has landed: all loads but the
            # newest tile's), tile u/2-1 is free; this wave's share of tile u/2+3 goes out during the next step
            e(f"s_waitcnt vmcnt({2 * NI})")
            e("s_barrier")
            next_dma = self.dma_groups(u // 2 + 3)
            next_k = [self.k_read(u + 2, f) for f in range(3)]
        return next_k, next_dma

    def drain(self, u):
        """Second product of unit u after the last step, and that unit's sums."""
        e = self.emit
        self.emit("s_waitcnt lgkmcnt(0)")      # the K fragments read ahead for a step that does not come
        self.queue = []
        vids = {g: self.v_read(u, g) for g in range(3)}
        for g in range(2 * DB):
            self.wait_for(vids[g])
            jj, db = g // DB, g % DB
            for rb in (0, 1):
                e(f"{self.mfma} {O(rb, db)}, {VF(g % 4)}, {P(u % 4, rb, jj)}, {O(rb, db)}")
            if g + 3 < 2 * DB:
                vids[g + 3] = self.v_read(u, g + 3)
        assert not self.queue
        for ln in self.pending_sums():
            e(ln)
        e("s_branch .Lfw64_end_%=")

    def block(self):
        e = self.emit
        e(f"v_xor_b32 {KADDR(1)}, 32, {KADDR(0)}")
        e(f"v_xor_b32 {VADDR(1)}, 64, {VADDR(0)}")
        e(f"v_xor_b32 {VADDR(2)}, 128, {VADDR(0)}")
        e(f"v_xor_b32 {VADDR(3)}, 192, {VADDR(0)}")
        for tensor in (0, 1):
            for n in range(NI):
                e(f"v_add_u32 {DMAOFF(tensor, n)}, {n * NW * 1024}, {KVOFF if tensor == 0 else VVOFF}")
        e("s_mov_b64 s[60:61], %[kptr]")
        e("s_mov_b64 s[62:63], %[vptr]")
        e("s_mov_b32 s67, %[npairs]")
        for r in range(128):
            e(f"v_accvgpr_write_b32 a{r}, 0")
        for rb in (0, 1):
            e(f"v_mov_b32 {M_REF(rb)}, 0xf149f2ca")    # -1e30
            e(f"v_mov_b32 {L_RUN(rb)}, 0")
            e(f"v_mov_b32 {L_RND(rb)}, 0")
        # this wave's share of tile 2 (tiles 0 and 1 were issued, tile 0 published, before the block)
        for g in self.dma_groups(2):
            for ln in g:
                e(ln)
        # logits of unit 0
        ids = [self.k_read(0, f) for f in range(3)]
        for kb in range(KB):
            self.wait_for(ids[kb])
            for rb in (0, 1):
                e(f"{self.mfma} {X(0, rb)}, {KF(kb % 4)}, {Q(rb, kb)}, {'0' if kb == 0 else X(0, rb)}")
            if kb + 3 < KB:
                ids.append(self.k_read(0, kb + 3))
        kpre = [self.k_read(1, f) for f in range(3)]
        e("s_nop 15")                               # the first step's vector work reads these logits
        kpre, dma = self.step(0, kpre, with_pv=False)
        e(".Lfw64_loop_%=:")
        entry_queue = list(self.queue)
        for u in (1, 2, 3):
            kpre, dma = self.step(u, kpre, dma=dma)
        e("s_sub_u32 s67, s67, 1")
        e("s_cmp_eq_u32 s67, 0")
        e("s_cbranch_scc1 .Lfw64_drain_a_%=")
        state_a = (list(self.queue), self.next_id)
        for u in (4, 5, 6, 7):
            kpre, dma = self.step(u, kpre, dma=dma)
        e("s_sub_u32 s67, s67, 1")
        e("s_cmp_eq_u32 s67, 0")
        e("s_cbranch_scc1 .Lfw64_drain_b_%=")
        state_b = (list(self.queue), self.next_id)
        kpre, dma = self.step(8, kpre, dma=dma)
        assert len(self.queue) == len(entry_queue) == 3
        e("s_branch .Lfw64_loop_%=")
        e(".Lfw64_drain_a_%=:")
        self.queue = state_a[0]
        self.drain(3)
        e(".Lfw64_drain_b_%=:")
        self.queue = state_b[0]
        self.drain(7)
        self.out += self.cold
        e(".Lfw64_end_%=:")
        e("s_nop 15")      # the accumulators are read by compiler-generated code next
        e("s_nop 3")
        return "\n".join(self.out)


CLOBBER_V = list(range(0, 160)) + [167, 169, 170, 171] + list(range(174, 194))
CLOBBER_S = list(range(60, 70))


def generate(path):
    """Writes the generated fragment to `path` (only if its text changes, so that build time stamps stay put)."""
    parts = ["// GENERATED by gen_fa_wide64_loop.py -- do not edit; change the script and build again.",
             "// The software-pipelined check-free main loop of fa_fwd_wide64_kernel as inline assembly with hand-chosen",
             "// registers and instruction order (plan and reasons are in the script's header).  A fragment of fa_fwd.hip.", ""]
    for name, bf16 in (("FA_WIDE64_LOOP_ASM_F16", False), ("FA_WIDE64_LOOP_ASM_BF16", True)):
        parts.append(f"#define {name} \\")
        lines = Gen(bf16).block().split("\n")
        parts.append(" \\\n".join('    "' + ln + '\\n\\t"' for ln in lines))
        parts.append("")
    clob = ", ".join([f'"v{r}"' for r in CLOBBER_V] + [f'"s{r}"' for r in CLOBBER_S] + ['"vcc"', '"scc"', '"m0"', '"memory"'])
    parts.append(f"#define FA_WIDE64_LOOP_CLOBBERS {clob}")
    parts.append("")
    text = "\n".join(parts)
    try:
        if open(path).read() == text:
            return
    except OSError:
        pass
    with open(path, "w") as f:
        f.write(text)


if __name__ == "__main__":
    generate(os.path.join(os.path.dirname(os.path.abspath(__file__)), "fa_attention_wide64_loop.inc"))
