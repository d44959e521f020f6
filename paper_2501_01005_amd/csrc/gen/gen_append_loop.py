#!/usr/bin/env python3
"""Writes append_loop_{bf16,f16}[_cap|_contig|_var|_ps|_rows|_contig_ps|_contig_rows].inc: the hand-scheduled
steady-state loop of the append kernel and its variants (soft cap; contiguous KV; ALiBi and / or sliding window; page
sizes 4, 8, 32; page sizes 1, 2; the last two also for contiguous KV).

The loop covers all KV tiles of a work item whose first tile every row of the CTA sees in full:
first the tiles that need no masking, then, with a compare-and-select on the logits in front of
the softmax, the tiles that the causal diagonal or the end of the chunk cuts.  The C++ kernel
around it does the epilogue (and whole work items that do not qualify).  One wavefront owns 32
query rows; per 32-token step it issues

    block 1:  S^T(next step) = K . Q^T   (8 MFMA)   ||  softmax of the current step, V^T reads
    block 2:  O^T += V^T . P^T           (8 MFMA)   ||  row sum, K reads two steps ahead, staging

so that inside a wavefront every matrix instruction is followed by a share of the vector and
LDS work of a neighbouring step (a wavefront issues in order: a run of dependent matrix
instructions would otherwise keep its own vector work waiting, and the other way round).  The
KV tiles are triple-buffered in LDS so that the next tile's K can be read before the CTA
barrier that publishes the tile after it.

All working registers are fixed (see the map below) and listed as clobbers; the C++ side
passes only addresses and scalars in, and the loop ends with the epilogue: it writes o, lse
and the optional cast of o itself.

Work items overlap at their seams.  The block reads the plan entry of the CTA's next work item
while it runs (outputs of the asm statement), and if that item will run this loop too, it
requests, right before its epilogue, the first two K tiles of that item into LDS buffers 0 and 1
and the first two V tiles, as stored, into a staging area (both with loads that write LDS
directly: nothing is held in registers across the C++ code between two work items).  The next
block is then entered with `pre` set and starts from LDS instead of waiting for its page ids and
for the tiles one after the other.  The epilogue's transpose area lies clear of those regions.

Run this script after changing it; the .inc files it writes are committed with it.
"""
import os
import sys

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
from emit import Emitter  # noqa: E402

# ---- fixed vector registers (the compiler keeps v0..v15) ----
NINF = 16
NEGMS, MRUN, LSUM, ONES, MAXT, X0, X1 = 17, 18, 19, 20, 21, 22, 23
ACC, Q, KA, VT, S0, S1, H, T, ST = 24, 88, 120, 152, 184, 200, 216, 224, 240
KAD = ST                       # ST..ST+7: LDS addresses of this lane's eight K operand reads; ST+8..ST+15: staged V
FIRST_FIXED_VGPR = 16
# ---- fixed scalar registers ----
S_T, S_TMP = 64, 65
S_OFFS = (66, 67, 86, 87)
S_IDS, S_IDN = 68, 72          # page ids of the tile to fetch next / of the one after it
S_PG0, S_PG1, S_LO, S_HI, S_KA, S_VA, S_THR, S_REM = 76, 77, 78, 79, 80, 82, 84, 85
S_IDA, S_IDB = 88, 92          # two more page id groups, start-up only
S_EXEC = 96
S_IDK = 88                     # page ids of the tile whose K goes to LDS next (takes over S_IDA after start-up)
S_ONES = 98                    # var variant: fp16 ones in both halves (the vector register of the constant is needed otherwise)
S_NP, S_HQ = 99, 100           # var variant: n_pos and num_qo_heads, unpacked from %[gl]
S_PSL, S_W4 = 98, 99           # page-size variant: log2 of the page size (from %[gl]); 4 * (wavefront % 4) = first row of its row group
S_G0, S_G1 = 68, 88            # per-row variant: two groups of eight page ids (a wavefront's 2 x 4 rows of a tile); there S_W4 = 4 * wavefront
ROW_MASKS = ((0xffff, 0), (0xffff0000, 0), (0, 0xffff), (0, 0xffff0000))   # exec_lo, exec_hi of the 16 lanes that load row q
S_M0 = 97                      # saved m0 (the register doubles as half of S_EXEC, which is used only after m0 is restored)
S_NX = 92                      # this wavefront's page ids of tiles 0 and 1 of the CTA's next work item (takes over S_IDB after start-up)
S_STP = 96                     # which page of a 32-token half this thread's staging rows are in (wavefront / 4); the epilogue reuses the register
FIXED_SGPRS = list(range(64, 101))
CAPV, WLO = 20, 21             # var variant: capped upper bound / lower bound of the tokens a lane's row sees, minus 4 c
FLOOR = 0xf149f2ca             # -1e30: reference of a row that has not seen a key yet (var variant)
NO_DIAG = 0x3FFFFFFF           # w_diag0 of a non-causal work item
LOOP_MIN_TOKENS = 128          # shorter chunks never run this loop

KROW, VROW = 256, 320          # LDS row pitch in bytes: K rows are packed (16-byte chunks XOR-swizzled by row), V rows padded
KTILE, VTILE = 64 * KROW, 64 * VROW
V_BASE = 65536                 # V buffers start where the generic path has them
STAGE = 2 * KTILE              # the next item's V tiles 0 and 1 as stored: K buffer 2 and the 16 KB after the K buffers
NBUF = 3
LAZY_THR = 0x5C005C00          # fp16 2^8 in both halves: P above it raises the reference


def float_bits(x):
    import struct
    return struct.unpack('<I', struct.pack('<f', float(x)))[0]


def vr(base, n=1):
    return 'v%d' % base if n == 1 else 'v[%d:%d]' % (base, base + n - 1)


def emit_item(e, o):
    """one instruction, or a tuple of instructions that must follow each other directly (vector moves under a
    narrowed exec mask: nothing else may run while the mask is narrow)"""
    for x in (o if isinstance(o, tuple) else (o,)):
        e.emit(x)


def spread(e, mfmas, others):
    """each matrix instruction is followed by an even share of the other instructions"""
    n = len(mfmas)
    k = 0
    for i, m in enumerate(mfmas):
        e.emit(m)
        hi = (len(others) * (i + 1)) // n
        for o in others[k:hi]:
            emit_item(e, o)
        k = hi


def merge_even(*lists):
    total = sum(len(l) for l in lists)
    out = []
    idx = [0] * len(lists)
    for _ in range(total):
        best = max(range(len(lists)),
                   key=lambda i: (len(lists[i]) - idx[i]) / max(len(lists[i]), 1) if idx[i] < len(lists[i]) else -1)
        out.append(lists[best][idx[best]])
        idx[best] += 1
    return out


class Gen:
    def __init__(self, bf16, cap=False, contig=False, var=False, anyps=False, rowids=False):
        self.bf = bf16
        # Page sizes 1 and 2 (the plain loop): the four token rows a wavefront stages per load lie in different pages,
        # so a lane addresses its row with 64 bits: pool base + page id * page bytes + the lane's offset in the row
        # group.  The ids of a wavefront's rows are scalar as before; a lane picks its row's id by four moves under
        # exec masks of 16 lanes.  A wavefront needs 2 x 4 ids per tile; two groups of eight scalar registers alternate: K of tile
        # t + 2 is requested from group 0 at the head of tile t, which then receives the ids of tile t + 4; V of tile
        # t + 3 is requested from group 1 at the tile's end; after the barrier (which waits for the ids) the groups
        # swap.  The next work item's first tiles are not requested ahead (sixteen more scalar registers).
        self.rowids = rowids
        assert not (rowids and (cap or var or anyps))
        # in the tile loop: ids of the tile whose K is requested next / where the ids requested at a tile's head go /
        # ids of the tile whose V is requested at the tile's end
        self.gk, self.gn, self.gs = (S_G0, S_G0, S_G1) if rowids else (S_IDK, S_IDN, S_IDS)
        # Page sizes 4, 8 and 32 (the plain loop): a wavefront stages four consecutive token rows per load, all in one
        # page, so what changes is which page id it fetches for them: token (64 t + 16 r + first row of its group)
        # >> log2(page size) of the chunk, for each 16-token segment r of tile t.  The row's place inside its page
        # is part of the per-lane offsets the C++ side passes.  %[gl] carries log2 of the page size in bits 8..
        self.anyps = anyps
        assert not (anyps and (cap or var))
        # ALiBi bias and sliding window (Sec. 3.2.3) for causal work items: like the soft cap, the logits of a step are
        # transformed in place as soon as they are complete: s <- s * sm_scale * log2(e) + slope * (t - pos), then -inf
        # where t < pos - W.  Per lane: %[cap] carries lim - 4 c uncapped (lim = chunk-local index of the row's own
        # token), %[slope] the head's slope times log2(e) (0 = no bias); %[win] = W (a huge value = no window).  The
        # capped bound (v20) and the window's lower bound (v21) are derived in the prologue; their registers are taken
        # from the constant of ones (then a scalar) and from the temporary of the lazy check (then one of the
        # exponentials' temporaries).  A row may see nothing in a step, a tile or the whole chunk: its reference then
        # stays at a large negative floor (so that masked logits still give P = 0 and the first visible one raises the
        # reference), and the epilogue writes o = 0, lse = -inf for a row without any visible key.
        self.var = var
        self.inplace = cap or var     # the S registers hold final logits in log2 units; the softmax scale is 1
        self.capreg = 'v%d' % CAPV if var else '%[cap]'
        self.maxt = T + 15 if var else MAXT
        self.ones = 's%d' % S_ONES if var else 'v%d' % ONES
        # the bias / window variant has one more scalar operand (the window) than scalar registers are left: there
        # %[gl] carries log2 g (bits 0..4, only ever used as a shift amount), n_pos (bits 5..15) and num_qo_heads
        # (bits 16..31), unpacked in the prologue
        self.np = 's%d' % S_NP if var else '%[np]'
        self.hq = 's%d' % S_HQ if var else '%[hq]'
        # contiguous KV (App. B's dense baseline): page j of the chunk is page kv_page0 + j of the pool, so the ids are
        # computed, not loaded; %[idblo] then carries the chunk's kv_page0 (the page-id array does not exist)
        self.contig = contig
        # logits soft cap (Sec. 3.2.3): the logits are transformed in place as soon as they are complete.  The block
        # has no scalar register to spare for the two constants of the transform, so in this variant the operand
        # of the softmax scale (which is 1 after the transform) carries the first and the operand of the wavefront
        # index the second; the wavefront index then rides in bits 8.. of the operand that holds log2 of the group
        # size, which is only ever used as a shift amount (the hardware takes the low five bits).
        self.cap = cap
        self.e = Emitter()
        self.mid_state = {}  # per masked tile of the rotation: loads in flight between its two steps

    def wave_shift(self, dst, op, amount):
        """s<dst> <- wavefront index shifted left (lshl) or right (lshr) by amount"""
        if not self.cap:
            return ['s_%s_b32 s%d, %%[stp8], %d' % (op, dst, amount)]
        if op == 'lshr':
            return ['s_lshr_b32 s%d, %%[gl], %d' % (dst, 8 + amount)]
        return ['s_lshr_b32 s%d, %%[gl], 8' % dst, 's_lshl_b32 s%d, s%d, %d' % (dst, dst, amount)]

    # ---- building blocks ----
    def qk(self, Sn, s):
        op = 'v_mfma_f32_32x32x16_bf16' if self.bf else 'v_mfma_f32_32x32x16_f16'
        c = '0' if s == 0 else vr(Sn, 16)
        return '%s %s, %s, %s, %s' % (op, vr(Sn, 16), vr(KA + 4 * s, 4), vr(Q + 4 * s, 4), c)

    def pv(self, db, j):
        a = ACC + 16 * db
        return 'v_mfma_f32_32x32x16_f16 %s, %s, %s, %s' % (vr(a, 16), vr(VT + 8 * db + 4 * j, 4), vr(H + 4 * j, 4), vr(a, 16))

    def exps(self, Sc):
        ops = []
        for j in range(8):
            a, b = T + 2 * j, T + 2 * j + 1
            if self.inplace:
                ops += ['v_add_f32 v%d, v%d, v%d' % (a, Sc + 2 * j, NEGMS), 'v_add_f32 v%d, v%d, v%d' % (b, Sc + 2 * j + 1, NEGMS)]
            else:
                ops += ['v_fma_f32 v%d, v%d, %%[sc], v%d' % (a, Sc + 2 * j, NEGMS),
                        'v_fma_f32 v%d, v%d, %%[sc], v%d' % (b, Sc + 2 * j + 1, NEGMS)]
            ops += ['v_exp_f32 v%d, v%d' % (a, a), 'v_exp_f32 v%d, v%d' % (b, b)]
        for j in range(8):
            ops.append('v_cvt_pk_f16_f32 v%d, v%d, v%d' % (H + j, T + 2 * j, T + 2 * j + 1))
        return ops

    def soft_cap(self, Sx):
        """s <- c * tanh(s * sm_scale / c) in log2 units, in place on the 16 logits of a step:
        tanh(x) = 1 - 2 / (exp(2 x) + 1); %[sc] holds 2 * sm_scale * log2(e) / c, %[stp8] holds c * log2(e).  Afterwards the
        softmax scale of the loop is 1.  Stage by stage over the 16 registers, so that no instruction reads the
        result of the one before it."""
        if not self.cap:
            return []
        ops = ['v_mul_f32 v%d, %%[sc], v%d' % (T + r, Sx + r) for r in range(16)]
        ops += ['v_exp_f32 v%d, v%d' % (T + r, T + r) for r in range(16)]
        ops += ['v_add_f32 v%d, 1.0, v%d' % (T + r, T + r) for r in range(16)]
        ops += ['v_rcp_f32 v%d, v%d' % (T + r, T + r) for r in range(16)]
        ops += ['v_fma_f32 v%d, v%d, -2.0, 1.0' % (T + r, T + r) for r in range(16)]
        ops += ['v_mul_f32 v%d, %%[stp8], v%d' % (Sx + r, T + r) for r in range(16)]
        return ops

    def transform(self, Sx, base_add):
        """the in-place logits transform of a step whose first token is 64 * S_T + base_add (chunk-local)"""
        if self.cap:
            return self.soft_cap(Sx)
        if not self.var:
            return []
        ops = ['s_lshl_b32 s%d, s%d, 6' % (S_TMP, S_T)]
        if base_add:
            ops.append('s_add_u32 s%d, s%d, %d' % (S_TMP, S_TMP, base_add))
        # X1 <- slope * (step base - (lim - 4 c)): the bias of the lane's first token of the step
        ops += ['v_sub_u32 v%d, s%d, %%[cap]' % (X1, S_TMP), 'v_cvt_f32_i32 v%d, v%d' % (X1, X1),
                'v_mul_f32 v%d, %%[slope], v%d' % (X1, X1)]
        ops += ['v_fma_f32 v%d, v%d, %%[sc], v%d' % (Sx + r, Sx + r, X1) for r in range(16)]
        for r in range(1, 16):
            k = 8 * (r // 4) + r % 4
            ops.append('v_fmamk_f32 v%d, %%[slope], 0x%08x, v%d' % (Sx + r, float_bits(k), Sx + r))
        # window: token k of the lane's 16 is visible iff k >= (lim - 4 c - W) - step base
        ops.append('v_subrev_u32 v%d, s%d, v%d' % (X0, S_TMP, WLO))
        for r in range(16):
            ops.append('v_cmp_ge_i32 vcc, %d, v%d' % (8 * (r // 4) + r % 4, X0))
            ops.append('v_cndmask_b32 v%d, v%d, v%d, vcc' % (Sx + r, NINF, Sx + r))
        return ops

    def mask(self, Sc, u):
        """logits of tokens past this lane's last visible one become -inf: register r holds token
        32 s + 4 c + 8 (r / 4) + r % 4 of the step, and cap = last visible token - 4 c"""
        ops = ['s_lshl_b32 s%d, s%d, 6' % (S_TMP, S_T)]
        if u:
            ops.append('s_add_u32 s%d, s%d, 32' % (S_TMP, S_TMP))
        ops.append('v_subrev_u32 v%d, s%d, %s' % (X1, S_TMP, self.capreg))
        for r in range(16):
            ops.append('v_cmp_le_i32 vcc, %d, v%d' % (8 * (r // 4) + r % 4, X1))
            ops.append('v_cndmask_b32 v%d, v%d, v%d, vcc' % (Sc + r, NINF, Sc + r))
        return ops

    def lazy_check(self):
        # P >= 0, so fp16 order is unsigned order on the bit patterns; any half above 2^8 -> vcc != 0
        mt = self.maxt
        ops = ['v_pk_max_u16 v%d, v%d, v%d' % (mt, H, H + 1)]
        for j in range(2, 8):
            ops.append('v_pk_max_u16 v%d, v%d, v%d' % (mt, mt, H + j))
        ops.append('v_pk_min_u16 v%d, v%d, s%d' % (X0, mt, S_THR))
        ops.append('v_cmp_ne_u32 vcc, v%d, v%d' % (X0, mt))
        return ops

    def rowsum(self):
        return ['v_dot2_f32_f16 v%d, v%d, %s, v%d' % (LSUM, H + j, self.ones, LSUM) for j in range(8)]

    def k_reads(self, buf, u):
        return ['ds_read_b128 %s, v%d offset:%d' % (vr(KA + 4 * s, 4), KAD + s, buf * KTILE + u * 32 * KROW)
                for s in range(8)]

    def v_reads(self, buf, u):
        ops = []
        for db in range(4):
            for j in range(2):
                r = VT + 8 * db + 4 * j
                base = buf * VTILE + u * 32 * VROW + 64 * db
                ops.append('ds_read_b64_tr_b16 %s, %%[va] offset:%d' % (vr(r, 2), base + (16 * j) * VROW))
                ops.append('ds_read_b64_tr_b16 %s, %%[va] offset:%d' % (vr(r + 2, 2), base + (16 * j + 8) * VROW))
        return ops

    def v_convert(self, base=ST):
        if not self.bf:
            return []
        ops = []
        for x in range(base + 8, base + 16):  # bf16 pairs -> fp16 pairs, toward zero
            ops += ['v_lshlrev_b32 v%d, 16, v%d' % (X0, x), 'v_and_b32 v%d, 0xffff0000, v%d' % (X1, x),
                    'v_cvt_pkrtz_f16_f32 v%d, v%d, v%d' % (x, X0, X1)]
        return ops

    def stores(self, buf, base=ST):
        ops = []
        for r in range(2):
            ops.append('ds_write_b128 %%[wv], %s offset:%d' % (vr(base + 8 + 4 * r, 4), buf * VTILE + r * 32 * VROW))
        return ops

    def v_zero_tail(self, ahead, base=ST):
        """V rows of tile t + ahead at or past the end of the chunk must not reach P.V (their
        logits are masked, but 0 x garbage need not be 0): this thread's rows are 32 r + st_tok"""
        ops = ['s_add_u32 s%d, s%d, %d' % (S_TMP, S_T, ahead), 's_lshl_b32 s%d, s%d, 6' % (S_TMP, S_TMP),
               's_sub_i32 s%d, %%[kvl], s%d' % (S_REM, S_TMP),  # rows of that tile inside the chunk (may be <= 0 or > 64)
               's_lshl_b32 s%d, s%d, 4' % (S_REM, S_REM)]          # (st_tok = thread / 16 < rows  <=>  thread < 16 rows)
        for r in range(2):
            if r:
                ops.append('s_sub_i32 s%d, s%d, 512' % (S_REM, S_REM))
            ops.append('v_cmp_gt_i32 vcc, s%d, %%[tid]' % S_REM)
            for x in range(base + 8 + 4 * r, base + 12 + 4 * r):
                ops.append('v_cndmask_b32 v%d, 0, v%d, vcc' % (x, x))
        return ops

    def row_ids(self, ids, dst):
        """v<dst> <- the page id of this lane's row: s[ids + q] for the 16 lanes of row q (one unit: nothing else may
        run while the exec mask is narrow)"""
        ops = []
        for q, (lo, hi) in enumerate(ROW_MASKS):
            ops += ['s_mov_b32 exec_lo, 0x%x' % lo, 's_mov_b32 exec_hi, 0x%x' % hi, 'v_mov_b32 v%d, s%d' % (dst, ids + q)]
        return tuple(ops + ['s_mov_b64 exec, -1'])

    def row_address(self, dst, idreg, tmp, spair, lo, hi, off):
        """v[dst:dst+1] <- pool base + page id * page bytes + this lane's offset in the row group (vcc is clobbered:
        callers place this where no comparison result is pending)"""
        return ['s_mov_b32 s%d, %%[%s]' % (spair, lo), 's_mov_b32 s%d, %%[%s]' % (spair + 1, hi),
                'v_mov_b32 v%d, %%[sp]' % tmp,
                'v_mad_u64_u32 %s, s[%d:%d], v%d, v%d, s[%d:%d]' % (vr(dst, 2), S_LO, S_HI, idreg, tmp, spair, spair + 1),
                'v_add_co_u32 v%d, vcc, v%d, %%[%s]' % (dst, dst, off),
                'v_addc_co_u32 v%d, vcc, 0, v%d, vcc' % (dst + 1, dst + 1)]

    def page_select(self, ids):
        return ['s_cmp_eq_u32 s%d, 0' % S_STP,
                's_cselect_b32 s%d, s%d, s%d' % (S_PG0, ids, ids + 1),
                's_cselect_b32 s%d, s%d, s%d' % (S_PG1, ids + 2, ids + 3)]

    def fetch(self, ids=S_IDS, base=ST):
        """global loads of the V rows of the tile whose four page ids are in s[ids..+3]; this
        thread's two pages are 2 r + st_page, r = 0, 1"""
        if self.rowids:  # (address and id pass through the registers the load then fills)
            ops = []
            for r in range(2):
                dst = base + 8 + 4 * r
                ops += [self.row_ids(ids + 4 * r, dst + 2)] + self.row_address(dst, dst + 2, dst + 3, S_VA, 'vblo', 'vbhi', 'so')
                ops.append('global_load_dwordx4 %s, %s, off' % (vr(dst, 4), vr(dst, 2)))
            return ops
        ops = self.page_select(ids)
        for r, pg in enumerate((S_PG0, S_PG1)):
            ops += ['s_mul_hi_u32 s%d, s%d, %%[sp]' % (S_HI, pg), 's_mul_i32 s%d, s%d, %%[sp]' % (S_LO, pg),
                    's_add_u32 s%d, %%[vblo], s%d' % (S_VA, S_LO), 's_addc_u32 s%d, %%[vbhi], s%d' % (S_VA + 1, S_HI),
                    'global_load_dwordx4 %s, %%[so], s[%d:%d]' % (vr(base + 8 + 4 * r, 4), S_VA, S_VA + 1)]
        return ops

    def k_to_lds(self, ids, buf):
        """K rows of that tile straight into LDS buffer `buf` (no registers, no LDS store
        instruction): a wavefront's load lands as 1 KB = its four consecutive 256-byte rows at m0,
        lane l at m0 + 16 l, and each lane fetches the chunk that the swizzle puts there"""
        if self.rowids:
            ops = []
            for r in range(2):
                ops += [self.row_ids(ids + 4 * r, X0)] + self.row_address(X0, X0, X1, S_KA, 'kblo', 'kbhi', 'sok')
                ops += ['s_add_u32 m0, %%[kd], %d' % (buf * KTILE + r * 32 * KROW), 's_nop 0',
                        'global_load_lds_dwordx4 %s, off' % vr(X0, 2)]
            return ops
        ops = self.page_select(ids)
        for r, pg in enumerate((S_PG0, S_PG1)):
            ops += ['s_mul_hi_u32 s%d, s%d, %%[sp]' % (S_HI, pg), 's_mul_i32 s%d, s%d, %%[sp]' % (S_LO, pg),
                    's_add_u32 s%d, %%[kblo], s%d' % (S_KA, S_LO), 's_addc_u32 s%d, %%[kbhi], s%d' % (S_KA + 1, S_HI),
                    's_add_u32 m0, %%[kd], %d' % (buf * KTILE + r * 32 * KROW), 's_nop 0',
                    'global_load_lds_dwordx4 %%[sok], s[%d:%d]' % (S_KA, S_KA + 1)]
        return ops

    def ids_load(self, ahead, dst=S_IDN):
        """request the page ids of tile t + ahead; each of the four is clamped to the chunk's last
        page, so a partial last tile still gets its own pages and nothing past the chunk is read"""
        ops = []
        if self.rowids:
            # token 64 t + 32 r + 4 * wavefront + q of the chunk -> its page -> byte offset of the page id, clamped
            if ahead:
                ops.append('s_add_u32 s%d, s%d, %d' % (S_TMP, S_T, ahead))
                ops.append('s_lshl_b32 s%d, s%d, 6' % (S_TMP, S_TMP))
            else:
                ops.append('s_lshl_b32 s%d, s%d, 6' % (S_TMP, S_T))
            ops.append('s_add_u32 s%d, s%d, s%d' % (S_TMP, S_TMP, S_W4))
            for r in range(2):
                for q, off in enumerate(S_OFFS):
                    if 32 * r + q:
                        ops.append('s_add_u32 s%d, s%d, %d' % (off, S_TMP, 32 * r + q))
                        ops.append('s_lshr_b32 s%d, s%d, s%d' % (off, off, S_PSL))
                    else:
                        ops.append('s_lshr_b32 s%d, s%d, s%d' % (off, S_TMP, S_PSL))
                    ops += ['s_lshl_b32 s%d, s%d, 2' % (off, off), 's_min_u32 s%d, s%d, %%[npg1]' % (off, off)]
                    ops += self.id_at(dst + 4 * r + q, off)
            return ops
        if self.anyps:
            # token of this wavefront's first row in segment r of the tile -> its page -> byte offset of the page id
            if ahead:
                ops.append('s_add_u32 s%d, s%d, %d' % (S_TMP, S_T, ahead))
                ops.append('s_lshl_b32 s%d, s%d, 6' % (S_TMP, S_TMP))
            else:
                ops.append('s_lshl_b32 s%d, s%d, 6' % (S_TMP, S_T))
            ops.append('s_add_u32 s%d, s%d, s%d' % (S_TMP, S_TMP, S_W4))
            for r, off in enumerate(S_OFFS):
                if r:
                    ops.append('s_add_u32 s%d, s%d, %d' % (off, S_TMP, 16 * r))
                    ops.append('s_lshr_b32 s%d, s%d, s%d' % (off, off, S_PSL))
                else:
                    ops.append('s_lshr_b32 s%d, s%d, s%d' % (off, S_TMP, S_PSL))
                ops += ['s_lshl_b32 s%d, s%d, 2' % (off, off), 's_min_u32 s%d, s%d, %%[npg1]' % (off, off)]
                ops += self.id_at(dst + r, off)
            return ops
        if ahead:
            ops.append('s_add_u32 s%d, s%d, %d' % (S_TMP, S_T, ahead))
            ops.append('s_lshl_b32 s%d, s%d, 4' % (S_TMP, S_TMP))
        else:
            ops.append('s_lshl_b32 s%d, s%d, 4' % (S_TMP, S_T))
        for r, off in enumerate(S_OFFS):
            if r:
                ops.append('s_add_u32 s%d, s%d, %d' % (off, S_TMP, 4 * r))
                ops.append('s_min_u32 s%d, s%d, %%[npg1]' % (off, off))
            else:
                ops.append('s_min_u32 s%d, s%d, %%[npg1]' % (off, S_TMP))
            ops += self.id_at(dst + r, off)
        return ops

    def id_at(self, dst, off):
        """s<dst> <- the page id at byte offset s<off> of the chunk's ids: loaded, or, with contiguous KV, computed"""
        if self.contig:
            return ['s_lshr_b32 s%d, s%d, 2' % (dst, off), 's_add_u32 s%d, s%d, %%[idblo]' % (dst, dst)]
        return ['s_load_dword s%d, %%[idp], s%d' % (dst, off)]

    def header_next(self):
        """request the plan entry of the CTA's next work item (of this one again if it is the last): the seven
        fields are consecutive arrays, wstr bytes apart; the results are outputs of the asm statement"""
        ops = ['s_and_b32 s%d, %%[woff], -4' % S_TMP]  # (the two low bits of woff are flags)
        for k, out in enumerate(('nq', 'nn', 'npg', 'nks', 'nkl', 'ndg', 'nos')):
            if k:
                ops.append('s_add_u32 s%d, s%d, %%[wstr]' % (S_TMP, S_TMP))
            ops.append('s_load_dword %%[%s], %%[wq0], s%d' % (out, S_TMP))
        return ops

    def next_decision_and_ids(self, tag, lbl):
        """the next item's plan entry has arrived: will it run this loop (the item-dependent part of the C++ side's
        test: at least LOOP_MIN_TOKENS tokens, first tile seen in full by every row)?  If so, request the page ids
        of its tiles 0 and 1, each clamped to the chunk's last page"""
        no = 'nopre_%s_%s' % (tag, lbl)
        vis = 'vis_%s_%s' % (tag, lbl)
        if self.rowids:
            return ['s_mov_b32 %[preo], 0']
        ops = ['s_mov_b32 %[preo], 0',
               's_bitcmp0_b32 %[woff], 0', 's_cbranch_scc1 ' + no,
               's_cmp_lt_u32 %%[nkl], %d' % LOOP_MIN_TOKENS, 's_cbranch_scc1 ' + no,
               's_mov_b32 s%d, %%[nkl]' % S_REM,
               's_cmp_eq_u32 %%[ndg], 0x%x' % NO_DIAG, 's_cbranch_scc1 ' + vis,
               # tokens the tile's first position sees: diag0 - kv_start + 1, at least 0
               's_sub_i32 s%d, %%[ndg], %%[nks]' % S_LO, 's_add_i32 s%d, s%d, 1' % (S_LO, S_LO),
               's_max_i32 s%d, s%d, 0' % (S_LO, S_LO), 's_min_i32 s%d, s%d, s%d' % (S_REM, S_REM, S_LO),
               vis + ':',
               's_cmp_lt_u32 s%d, 64' % S_REM, 's_cbranch_scc1 ' + no,
               's_mov_b32 %[preo], 1']
        # byte offset of the chunk's last page id (S_REM); address of its first one (S_KA pair)
        if self.anyps:
            ops += ['s_lshl_b32 s%d, 1, s%d' % (S_REM, S_PSL), 's_sub_u32 s%d, s%d, 1' % (S_REM, S_REM),
                    's_add_u32 s%d, s%d, %%[nkl]' % (S_REM, S_REM), 's_lshr_b32 s%d, s%d, s%d' % (S_REM, S_REM, S_PSL)]
        else:
            ops += ['s_add_u32 s%d, %%[nkl], 15' % S_REM, 's_lshr_b32 s%d, s%d, 4' % (S_REM, S_REM)]
        ops += ['s_sub_u32 s%d, s%d, 1' % (S_REM, S_REM), 's_lshl_b32 s%d, s%d, 2' % (S_REM, S_REM),
               's_mov_b32 s%d, %%[npg]' % S_LO, 's_mov_b32 s%d, 0' % S_HI,
               's_lshl_b64 s[%d:%d], s[%d:%d], 2' % (S_LO, S_HI, S_LO, S_HI),
               's_add_u32 s%d, %%[idblo], s%d' % (S_KA, S_LO), 's_addc_u32 s%d, %%[idbhi], s%d' % (S_KA + 1, S_HI)]
        # of a tile's four pages this thread's rows are in pages S_STP and 2 + S_STP
        if self.anyps:  # (token of this wavefront's first row in half i of the first two tiles: 32 i + 4 * wavefront)
            ops += ['s_lshl_b32 s%d, s%d, 4' % (S_LO, S_STP), 's_add_u32 s%d, s%d, s%d' % (S_LO, S_LO, S_W4)]
        else:
            ops.append('s_lshl_b32 s%d, s%d, 2' % (S_LO, S_STP))
        for i in range(4):
            if self.anyps:
                ops += ['s_add_u32 s%d, s%d, %d' % (S_TMP, S_LO, 32 * i), 's_lshr_b32 s%d, s%d, s%d' % (S_TMP, S_TMP, S_PSL),
                        's_lshl_b32 s%d, s%d, 2' % (S_TMP, S_TMP), 's_min_u32 s%d, s%d, s%d' % (S_TMP, S_TMP, S_REM)]
            else:
                ops += ['s_add_u32 s%d, s%d, %d' % (S_TMP, S_LO, 8 * i), 's_min_u32 s%d, s%d, s%d' % (S_TMP, S_TMP, S_REM)]
            if self.contig:  # the next item's page ids follow from its kv_page0
                ops += ['s_lshr_b32 s%d, s%d, 2' % (S_NX + i, S_TMP), 's_add_u32 s%d, s%d, %%[npg]' % (S_NX + i, S_NX + i)]
            else:
                ops.append('s_load_dword s%d, s[%d:%d], s%d' % (S_NX + i, S_KA, S_KA + 1, S_TMP))
        ops.append(no + ':')
        return ops

    def k_next_to_lds(self, pages, buf):
        """as k_to_lds, for the two pages whose ids are in s[pages], s[pages + 1]"""
        ops = []
        for r, pg in enumerate((pages, pages + 1)):
            ops += ['s_mul_hi_u32 s%d, s%d, %%[sp]' % (S_HI, pg), 's_mul_i32 s%d, s%d, %%[sp]' % (S_LO, pg),
                    's_add_u32 s%d, %%[kblo], s%d' % (S_KA, S_LO), 's_addc_u32 s%d, %%[kbhi], s%d' % (S_KA + 1, S_HI),
                    's_add_u32 m0, %%[kd], %d' % (buf * KTILE + r * 32 * KROW), 's_nop 0',
                    'global_load_lds_dwordx4 %%[sok], s[%d:%d]' % (S_KA, S_KA + 1)]
        return ops

    def v_to_stage(self, pages, st):
        """V rows of that tile of the next work item, as stored, straight into the staging area: a wavefront's
        load lands as its four consecutive 256-byte rows, lane l at m0 + 16 l, each lane its own chunk"""
        ops = []
        for r, pg in enumerate((pages, pages + 1)):
            ops += ['s_mul_hi_u32 s%d, s%d, %%[sp]' % (S_HI, pg), 's_mul_i32 s%d, s%d, %%[sp]' % (S_LO, pg),
                    's_add_u32 s%d, %%[vblo], s%d' % (S_VA, S_LO), 's_addc_u32 s%d, %%[vbhi], s%d' % (S_VA + 1, S_HI),
                    's_add_u32 m0, %%[kd], %d' % (STAGE + st * KTILE + r * 32 * KROW), 's_nop 0',
                    'global_load_lds_dwordx4 %%[so], s[%d:%d]' % (S_VA, S_VA + 1)]
        return ops

    def prefetch_next(self, tag, lbl):
        """at the end of a work item (every wavefront is past its last tile read and has no load in flight): if the
        next item runs this loop, request its K tiles 0 and 1 into buffers 0 and 1 and its V tiles 0 and 1 into the
        staging area"""
        skip = 'nopf_%s_%s' % (tag, lbl)
        if self.rowids:
            return []
        ops = ['s_waitcnt lgkmcnt(0)', 's_cmp_eq_u32 %[preo], 0', 's_cbranch_scc1 ' + skip]
        for t in range(2):
            ops += self.k_next_to_lds(S_NX + 2 * t, t)
        for t in range(2):
            ops += self.v_to_stage(S_NX + 2 * t, t)
        ops.append(skip + ':')
        return ops

    def stage_reads(self, lbl):
        """this thread's pieces of the staged V tiles 0 and 1 (the ones it requested itself at the end of the
        previous work item) into the registers the start-up converts them from"""
        ops = self.wave_shift(S_TMP, 'lshl', 10) + ['s_sub_u32 s%d, %%[kd], s%d' % (S_TMP, S_TMP),  # LDS offset of the tile area
               'v_lshrrev_b32 v%d, 4, %%[tid]' % X0, 'v_lshlrev_b32 v%d, 8, v%d' % (X0, X0),   # 256 * st_tok
               'v_and_b32 v%d, 15, %%[tid]' % X1, 'v_lshl_add_u32 v%d, v%d, 4, v%d' % (X0, X1, X0),  # + 16 * st_chunk
               'v_add_u32 v%d, s%d, v%d' % (X0, S_TMP, X0)]
        for t, base in ((0, VT), (1, KA)):
            for r in range(2):
                ops.append('ds_read_b128 %s, v%d offset:%d' % (vr(base + 8 + 4 * r, 4), X0, STAGE + t * KTILE + r * 32 * KROW))
        return ops

    def ids_take(self):
        if self.rowids:   # the two groups swap
            ops = []
            for i in range(0, 8, 2):
                ops += ['s_mov_b64 s[%d:%d], s[%d:%d]' % (S_LO, S_HI, S_G0 + i, S_G0 + i + 1),
                        's_mov_b64 s[%d:%d], s[%d:%d]' % (S_G0 + i, S_G0 + i + 1, S_G1 + i, S_G1 + i + 1),
                        's_mov_b64 s[%d:%d], s[%d:%d]' % (S_G1 + i, S_G1 + i + 1, S_LO, S_HI)]
            return ops
        return ['s_mov_b64 s[%d:%d], s[%d:%d]' % (S_IDK, S_IDK + 1, S_IDS, S_IDS + 1),
                's_mov_b64 s[%d:%d], s[%d:%d]' % (S_IDK + 2, S_IDK + 3, S_IDS + 2, S_IDS + 3),
                's_mov_b64 s[%d:%d], s[%d:%d]' % (S_IDS, S_IDS + 1, S_IDN, S_IDN + 1),
                's_mov_b64 s[%d:%d], s[%d:%d]' % (S_IDS + 2, S_IDS + 3, S_IDN + 2, S_IDN + 3)]

    def row_max(self, Sc):
        """X0 <- max(MRUN, maximum of the 32 logits of this lane's row)"""
        ops = ['v_max3_f32 v%d, v%d, v%d, v%d' % (X0, Sc, Sc + 1, Sc + 2)]
        for i in range(3, 15, 2):
            ops.append('v_max3_f32 v%d, v%d, v%d, v%d' % (X0, X0, Sc + i, Sc + i + 1))
        ops.append('v_max_f32 v%d, v%d, v%d' % (X0, X0, Sc + 15))
        # the other half of the wavefront holds the row's other 16 tokens
        ops += ["v_mov_b32 v%d, v%d" % (X1, X0), "s_nop 1", "v_permlane32_swap_b32 v%d, v%d" % (X0, X1), "s_nop 1",
                'v_max3_f32 v%d, v%d, v%d, v%d' % (X0, X0, X1, MRUN)]
        return ops

    def set_reference(self):
        return ['v_mov_b32 v%d, v%d' % (MRUN, X0),
                'v_mov_b32 v%d, v%d' % (NEGMS, X0) if self.inplace else 'v_mul_f32 v%d, v%d, %%[sc]' % (NEGMS, X0),
                'v_xor_b32 v%d, 0x80000000, v%d' % (NEGMS, NEGMS)]

    def raise_reference(self, Sc):
        """out-of-line: raise the reference to the row maximum, rescale the state, redo P"""
        ops = self.row_max(Sc)
        ops += ['v_sub_f32 v%d, v%d, v%d' % (X1, MRUN, X0)] + ([] if self.inplace else ['v_mul_f32 v%d, v%d, %%[sc]' % (X1, X1)]) + [
                'v_exp_f32 v%d, v%d' % (X1, X1)]
        ops += self.set_reference()
        ops.append('v_mul_f32 v%d, v%d, v%d' % (LSUM, LSUM, X1))
        for i in range(64):
            ops.append('v_mul_f32 v%d, v%d, v%d' % (ACC + i, ACC + i, X1))
        ops += self.exps(Sc)
        ops.append('s_nop 4')  # vector writes of the accumulators settle before the next matrix instruction reads them
        return ops

    # ---- program ----
    def tile(self, k, lbl, masked):
        e = self.e
        cur, nxt, wr = k % NBUF, (k + 1) % NBUF, (k + 2) % NBUF
        kind = 'm' if masked else 'p'
        e.label('tile_%s%d_%s' % (kind, k, lbl))
        if masked:
            # none of this wavefront's rows sees a token of this tile or of any later one (its last row, lane 31,
            # sees the most): from here on it only helps with the staging, then writes its outputs
            e.raw('v_readlane_b32 s%d, %s, 31' % (S_TMP, self.capreg))
            e.raw('s_lshl_b32 s%d, s%d, 6' % (S_REM, S_T))
            e.raw('s_cmp_gt_i32 s%d, s%d' % (S_REM, S_TMP))
            e.raw('s_cbranch_scc1 tile_j%d_%s' % (k, lbl))
        # canonical state after the barrier: no LDS operation in flight, the four loads of the
        # staged tile (K0, V0, K1, V1) possibly still in flight
        e.lgkm = []
        e.vm = [set(('v', ST + 8 + 4 * r + i) for i in range(4)) for r in (0, 1)]
        for u in range(2):
            Sc, Sn = (S0, S1) if u == 0 else (S1, S0)
            if masked and u == 1:
                # the same test for the tile's second 32-token step: the wavefront leaves the tile half way and
                # does the rest of its staging share in half_j
                self.mid_state[k] = ([set(d) for d in e.lgkm], [set(d) for d in e.vm])
                e.raw('v_readlane_b32 s%d, %s, 31' % (S_TMP, self.capreg))
                e.raw('s_lshl_b32 s%d, s%d, 6' % (S_REM, S_T))
                e.raw('s_add_u32 s%d, s%d, 32' % (S_REM, S_REM))
                e.raw('s_cmp_gt_i32 s%d, s%d' % (S_REM, S_TMP))
                e.raw('s_cbranch_scc1 half_j%d_%s' % (k, lbl))
            # block 1
            # the tile after next: its K goes to the LDS buffer that the barrier before this tile freed
            head = self.k_to_lds(self.gk, wr) + self.ids_load(4, self.gn) if u == 0 else []
            soft = (self.mask(Sc, u) if masked else []) + self.exps(Sc) + self.lazy_check()
            spread(e, [self.qk(Sn, s) for s in range(8)], head + merge_even(self.v_reads(cur, u), soft))
            e.raw('s_cbranch_vccnz raise_%s%d%d_%s' % (kind, k, u, lbl))
            e.label('back_%s%d%d_%s' % (kind, k, u, lbl))
            # block 2
            kn = self.k_reads(nxt, u)
            # (with the soft cap: the next step's logits, complete since the matrix instructions of block 1, are
            # transformed behind the last products of this block; the temporaries of the exponentials are free here)
            if u == 0:
                rest = merge_even(kn, self.rowsum() + self.v_convert()) + self.transform(Sn, 32)
            else:
                rest = merge_even(kn, self.rowsum() + self.v_zero_tail(2)) + self.stores(wr) + self.fetch(self.gs) + self.transform(Sn, 64)
            spread(e, [self.pv(db, j) for j in range(2) for db in range(4)], rest)
        e.wait_lds_loads()
        e.emit('s_barrier')
        for o in self.ids_take():
            e.raw(o)
        e.raw('s_add_u32 s%d, s%d, 1' % (S_T, S_T))
        e.raw('s_cmp_ge_u32 s%d, %%[nt]' % S_T)
        e.raw('s_cbranch_scc1 exit_%s' % lbl)
        kn = (k + 1) % NBUF
        if masked:
            e.raw('s_branch tile_m%d_%s' % (kn, lbl)) if kn == 0 else None  # masked tiles follow each other in memory
        else:
            e.raw('s_cmp_lt_u32 s%d, %%[nf]' % S_T)
            e.raw('s_cbranch_scc0 tile_m%d_%s' % (kn, lbl))
            if kn == 0:
                e.raw('s_branch tile_p0_%s' % lbl)

    def idle_half(self, k, lbl):
        """second half of tile k for a wavefront that left it after the first 32-token step: what is left of its
        staging share, the barrier, then idle tiles up to the epilogue"""
        e = self.e
        wr = (k + 2) % NBUF
        e.label('half_j%d_%s' % (k, lbl))
        e.lgkm, e.vm = [set(d) for d in self.mid_state[k][0]], [set(d) for d in self.mid_state[k][1]]
        for o in self.v_zero_tail(2) + self.stores(wr) + self.fetch(self.gs):
            emit_item(e, o)
        e.wait_lds_loads()
        e.emit('s_barrier')
        for o in self.ids_take():
            e.raw(o)
        e.raw('s_add_u32 s%d, s%d, 1' % (S_T, S_T))
        e.raw('s_cmp_ge_u32 s%d, %%[nt]' % S_T)
        e.raw('s_cbranch_scc1 exit_%s' % lbl)
        e.raw('s_branch tile_j%d_%s' % ((k + 1) % NBUF, lbl))

    def idle_tile(self, k, lbl, tag='i', leave='done'):
        """a tile for a wavefront none of whose rows exists (the query tile is shorter than the CTA's
        256 rows; tag i, leaves without outputs), or whose rows are all past their last visible token
        (tag j, leaves through the epilogue): it only does its share of the staging, then waits at the
        barrier, which leaves the SIMD to the wavefront it shares it with"""
        e = self.e
        wr = (k + 2) % NBUF
        e.label('tile_%s%d_%s' % (tag, k, lbl))
        e.lgkm = []
        e.vm = [set(('v', ST + 8 + 4 * r + i) for i in range(4)) for r in (0, 1)]
        for o in (self.k_to_lds(self.gk, wr) + self.ids_load(4, self.gn) + self.v_convert() + self.v_zero_tail(2) + self.stores(wr) +
                  self.fetch(self.gs)):
            emit_item(e, o)
        e.wait_lds_loads()
        e.emit('s_barrier')
        for o in self.ids_take():
            e.raw(o)
        e.raw('s_add_u32 s%d, s%d, 1' % (S_T, S_T))
        e.raw('s_cmp_ge_u32 s%d, %%[nt]' % S_T)
        e.raw('s_cbranch_scc1 %s_%s' % (leave, lbl))
        if (k + 1) % NBUF == 0:
            e.raw('s_branch tile_%s0_%s' % (tag, lbl))

    def program(self):
        e = self.e
        lbl = '%='
        # constants and zero state
        e.raw('s_mov_b32 s%d, m0' % S_M0)
        e.raw('s_mov_b32 s%d, 0' % S_T)
        e.raw('s_mov_b32 s%d, 0x%x' % (S_THR, LAZY_THR))
        for o in self.wave_shift(S_STP, 'lshr', 2):
            e.raw(o)
        if self.anyps:
            e.raw('s_lshr_b32 s%d, %%[gl], 8' % S_PSL)
            e.raw('s_and_b32 s%d, %%[stp8], 3' % S_W4)
            e.raw('s_lshl_b32 s%d, s%d, 2' % (S_W4, S_W4))
        if self.rowids:
            e.raw('s_lshr_b32 s%d, %%[gl], 8' % S_PSL)
            e.raw('s_lshl_b32 s%d, %%[stp8], 2' % S_W4)
        for s in range(8):
            e.emit('global_load_dwordx4 %s, %%[qp], off offset:%d' % (vr(Q + 4 * s, 4), 32 * s))
        for o in self.header_next():
            e.raw(o)
        if self.var:
            e.raw('s_mov_b32 s%d, 0x3c003c00' % S_ONES)
            e.raw('s_bfe_u32 s%d, %%[gl], 0x%x' % (S_NP, (11 << 16) | 5))
            e.raw('s_lshr_b32 s%d, %%[gl], 16' % S_HQ)
            # 4 c of this lane -> upper bound capped at the chunk's last token, lower bound of the window
            for o in ['v_mbcnt_lo_u32_b32 v%d, -1, 0' % X0, 'v_mbcnt_hi_u32_b32 v%d, -1, v%d' % (X0, X0),
                      'v_lshrrev_b32 v%d, 5, v%d' % (X0, X0), 'v_lshlrev_b32 v%d, 2, v%d' % (X0, X0),
                      'v_sub_u32 v%d, %%[kvl], v%d' % (X1, X0), 'v_subrev_u32 v%d, 1, v%d' % (X1, X1),
                      'v_min_i32 v%d, %%[cap], v%d' % (CAPV, X1), 'v_subrev_u32 v%d, %%[win], %%[cap]' % WLO]:
                e.raw(o)
        else:
            e.raw('v_mov_b32 v%d, 0x3c003c00' % ONES)
        e.raw('v_mov_b32 v%d, 0' % LSUM)
        e.raw('v_mov_b32 v%d, 0xff800000' % MRUN)
        e.raw('v_mov_b32 v%d, 0xff800000' % NINF)
        for i in range(64):
            e.raw('v_mov_b32 v%d, 0' % (ACC + i))
        # the eight K operand reads of a lane: row n, chunk (2 s + c) ^ (n % 16) -> kb + (32 s ^ kxs)
        e.raw('v_bfe_u32 v%d, %%[tid], 1, 3' % X0)   # ((n >> 1) & 7) * 32, n = thread % 32
        e.raw('v_lshlrev_b32 v%d, 5, v%d' % (X0, X0))
        for s_ in range(8):
            e.raw('v_xor_b32 v%d, %d, v%d' % (KAD + s_, 32 * s_, X0))
            e.raw('v_add_u32 v%d, v%d, %%[kb]' % (KAD + s_, KAD + s_))
        q_loads = list(e.vm)
        if not self.rowids:  # (the per-row variant never has tiles requested ahead)
            e.raw('s_bitcmp0_b32 %[woff], 1')
            e.raw('s_cbranch_scc0 staged_%s' % lbl)
        # start-up from memory: the page ids of tiles 0..3 in one go, then K of tiles 0 and 1 straight into LDS and
        # V of tiles 0, 1, 2 in flight together (tiles 0 and 1 borrow operand registers as staging)
        if self.rowids:
            # two groups of ids: tiles 0 and 1 first (K into LDS, V into borrowed registers), then tiles 2 and 3,
            # which leaves group 0 = tile 2 (K at the head of the first tile) and group 1 = tile 3 (V at its end)
            for t, dst in ((0, S_G0), (1, S_G1)):
                for o in self.ids_load(t, dst):
                    e.raw(o)
            e.raw('s_waitcnt lgkmcnt(0)')
            for t, ids in ((0, S_G0), (1, S_G1)):
                for o in self.k_to_lds(ids, t):
                    emit_item(e, o)
            for ids, base in ((S_G0, VT), (S_G1, KA)):
                for o in self.fetch(ids, base):
                    emit_item(e, o)
            for t, dst in ((2, S_G0), (3, S_G1)):
                for o in self.ids_load(t, dst):
                    e.raw(o)
            e.raw('s_waitcnt lgkmcnt(0)')
            for o in self.fetch(S_G0, ST):
                emit_item(e, o)
        else:
            for t, dst in enumerate((S_IDA, S_IDB, S_IDN, S_IDS)):
                for o in self.ids_load(t, dst):
                    e.raw(o)
            e.raw('s_waitcnt lgkmcnt(0)')
            for t, ids in ((0, S_IDA), (1, S_IDB)):
                for o in self.k_to_lds(ids, t):
                    e.emit(o)
            for ids, base in ((S_IDA, VT), (S_IDB, KA), (S_IDN, ST)):
                for o in self.fetch(ids, base):
                    e.emit(o)
        for o in self.next_decision_and_ids('a', lbl):
            e.raw(o)
        for t, base in ((0, VT), (1, KA)):
            for o in self.v_convert(base) + self.v_zero_tail(t, base) + self.stores(t, base):
                e.emit(o)
        e.wait_lds_loads()
        if not self.rowids:
            e.raw('s_mov_b64 s[%d:%d], s[%d:%d]' % (S_IDK, S_IDK + 1, S_IDN, S_IDN + 1))
            e.raw('s_mov_b64 s[%d:%d], s[%d:%d]' % (S_IDK + 2, S_IDK + 3, S_IDN + 2, S_IDN + 3))
        e.emit('s_barrier')
        e.raw('s_branch started_%s' % lbl)
        # start-up from LDS: K of tiles 0 and 1 is in its buffers, V of tiles 0 and 1 in the staging area
        e.label('staged_%s' % lbl)
        e.lgkm = []
        e.vm = list(q_loads)
        for t, dst in (() if self.rowids else ((2, S_IDN), (3, S_IDS))):
            for o in self.ids_load(t, dst):
                e.raw(o)
        if not self.rowids:
            for o in self.stage_reads(lbl):
                e.emit(o)
            e.drain(lgkm=True, vm=False)
            for o in self.fetch(S_IDN, ST):
                e.emit(o)
            for o in self.next_decision_and_ids('b', lbl):
                e.raw(o)
            for t, base in ((0, VT), (1, KA)):
                for o in self.v_convert(base) + self.v_zero_tail(t, base) + self.stores(t, base):
                    e.emit(o)
            e.raw('s_mov_b64 s[%d:%d], s[%d:%d]' % (S_IDK, S_IDK + 1, S_IDN, S_IDN + 1))
            e.raw('s_mov_b64 s[%d:%d], s[%d:%d]' % (S_IDK + 2, S_IDK + 3, S_IDN + 2, S_IDN + 3))
            e.emit('s_barrier')
        e.label('started_%s' % lbl)
        # either way: nothing of LDS in flight; of the loads, at most Q and the V rows of tile 2, in this order
        e.lgkm = []
        e.vm = list(q_loads) + [set(('v', ST + 8 + 4 * r + i) for i in range(4)) for r in (0, 1)]
        # a wavefront whose first row is past the end of the query tile only helps with the staging
        for o in self.wave_shift(S_TMP, 'lshl', 5):            # first tile row of this wavefront
            e.raw(o)
        e.raw('s_lshr_b32 s%d, s%d, %%[gl]' % (S_TMP, S_TMP))  # its position
        e.raw('s_cmp_ge_u32 s%d, %s' % (S_TMP, self.np))
        e.raw('s_cbranch_scc1 tile_i0_%s' % lbl)
        # first step: S^T(0, 0), the K operands of step (0, 1), the first reference
        for o in self.k_reads(0, 0):
            e.emit(o)
        for s in range(8):
            e.emit(self.qk(S0, s))
        for o in self.k_reads(0, 1):
            e.emit(o)
        e.raw('s_nop 15')
        e.raw('s_nop 15')
        floor = ['v_max_f32 v%d, 0x%08x, v%d' % (X0, FLOOR, X0)] if self.var else []
        for o in self.transform(S0, 0) + self.row_max(S0) + floor + self.set_reference():
            e.emit(o)
        e.drain(lgkm=True, vm=False)
        e.raw('s_cmp_lt_u32 s%d, %%[nf]' % S_T)  # t = 0: a first tile that needs masking is possible when nf = 0
        e.raw('s_cbranch_scc0 tile_m0_%s' % lbl)
        # steady state, one copy per LDS buffer rotation: unmasked tiles, then masked ones
        for masked in (False, True):
            for k in range(NBUF):
                self.tile(k, lbl, masked)
        e.raw('s_branch exit_%s' % lbl)
        for k in range(NBUF):
            self.idle_tile(k, lbl)
        for k in range(NBUF):
            self.idle_tile(k, lbl, 'j', 'exit')
        for k in range(NBUF):
            self.idle_half(k, lbl)
        # out-of-line reference raises
        for kind in 'pm':
            for k in range(NBUF):
                for u in range(2):
                    e.label('raise_%s%d%d_%s' % (kind, k, u, lbl))
                    for o in self.raise_reference(S0 if u == 0 else S1):
                        e.raw(o)
                    e.raw('s_branch back_%s%d%d_%s' % (kind, k, u, lbl))
        # epilogue (every wavefront is past its last tile read: the exit follows a barrier):
        # o = O / l, lse = ln(sum exp) = (reference * scale_log2 + log2 l) * ln 2.  The accumulators
        # hold 16-byte pieces of 32 different rows per lane column, which would make every output
        # store touch 32 rows; they go through a wavefront-private LDS area (32 rows x 288 B, one
        # half of the head dimension at a time) so that a store instruction writes four rows of
        # 256 contiguous bytes.
        EPITCH = 288
        e.label('exit_%s' % lbl)
        e.raw('s_waitcnt vmcnt(0)')
        for o in self.prefetch_next('x', lbl):
            e.raw(o)
        e.raw('s_mov_b32 m0, s%d' % S_M0)
        e.raw('s_nop 15')
        e.raw('s_nop 15')
        for o in ['v_mov_b32 v%d, v%d' % (X0, LSUM), 'v_mov_b32 v%d, v%d' % (X1, LSUM), 's_nop 1',
                  'v_permlane32_swap_b32 v%d, v%d' % (X0, X1), 's_nop 1', 'v_add_f32 v%d, v%d, v%d' % (LSUM, X0, X1),
                  # (a transcendental result needs a wait state before an ordinary vector instruction reads it)
                  'v_log_f32 v%d, v%d' % (X1, LSUM), 'v_rcp_f32 v%d, v%d' % (X0, LSUM), 's_nop 1'] + (
                  # a row without a visible key: l = 0 -> o = 0 (lse = reference + log2(0) = -inf by itself)
                  ['v_cmp_neq_f32 vcc, 0, v%d' % LSUM, 'v_cndmask_b32 v%d, 0, v%d, vcc' % (X0, X0)] if self.var else []) + [
                  'v_add_f32 v%d, v%d, v%d' % (X1, MRUN, X1) if self.inplace else 'v_fma_f32 v%d, v%d, %%[sc], v%d' % (X1, MRUN, X1),
                  'v_mul_f32 v%d, 0x3f317218, v%d' % (X1, X1),
                  's_mov_b64 s[%d:%d], exec' % (S_EXEC, S_EXEC + 1),
                  # one lane per live row writes lse: lane < 32 and position of row 32 wave + lane % 32 < n_pos
                  'v_mbcnt_lo_u32_b32 v%d, -1, 0' % (T + 15), 'v_mbcnt_hi_u32_b32 v%d, -1, v%d' % (T + 15, T + 15),
                  'v_and_b32 v%d, 31, v%d' % (T + 14, T + 15)] + self.wave_shift(S_TMP, 'lshl', 5) + [
                  'v_add_u32 v%d, s%d, v%d' % (T + 14, S_TMP, T + 14), 'v_lshrrev_b32 v%d, %%[gl], v%d' % (T + 14, T + 14),
                  'v_cmp_gt_i32 vcc, %s, v%d' % (self.np, T + 14), 's_and_b64 exec, exec, vcc',
                  'v_cmp_gt_u32 vcc, 32, v%d' % (T + 15), 's_and_b64 exec, exec, vcc',
                  'v_lshrrev_b32 v%d, 9, %%[ooff]' % T, 'v_lshlrev_b32 v%d, 2, v%d' % (T, T),
                  'global_store_dword v%d, v%d, %%[lb] nt' % (T, X1), 's_mov_b64 exec, s[%d:%d]' % (S_EXEC, S_EXEC + 1)]:
            e.raw(o)
        for i in range(64):
            e.raw('v_mul_f32 v%d, v%d, v%d' % (ACC + i, ACC + i, X0))
        # store instruction k of a half covers tile rows 32 w + 4 k + lane / 16: their output byte offsets (KA + k),
        # halved for the rounded copy (S0 + k), and whether the row exists (scalar masks)
        OFF, COFF, ROW0 = KA, S0, T
        masks = [S_IDA, S_IDA + 2, S_IDB, S_IDB + 2, S_IDS, S_IDS + 2, S_IDN, S_IDN + 2]
        L16 = T + 5   # 16 * (thread % 16): the 16-byte piece of a row this lane stores
        for o in ['v_lshrrev_b32 v%d, 6, %%[tid]' % ROW0, 'v_lshlrev_b32 v%d, 5, v%d' % (ROW0, ROW0),
                  'v_bfe_u32 v%d, %%[tid], 4, 2' % (T + 1), 'v_or_b32 v%d, v%d, v%d' % (ROW0, ROW0, T + 1),
                  'v_and_b32 v%d, 15, %%[tid]' % L16, 'v_lshlrev_b32 v%d, 4, v%d' % (L16, L16)]:
            e.raw(o)
        for k in range(8):
            R, P, B = T + 2, T + 3, T + 4
            for o in ['v_add_u32 v%d, %d, v%d' % (R, 4 * k, ROW0), 'v_lshrrev_b32 v%d, %%[gl], v%d' % (P, R),
                      'v_lshlrev_b32 v%d, %%[gl], v%d' % (B, P), 'v_sub_u32 v%d, v%d, v%d' % (B, R, B),
                      'v_mad_u32_u24 v%d, v%d, %s, v%d' % (B, P, self.hq, B), 'v_add_u32 v%d, %%[rb], v%d' % (B, B),
                      'v_lshlrev_b32 v%d, 9, v%d' % (B, B), 'v_add_u32 v%d, v%d, v%d' % (OFF + k, B, L16),
                      'v_lshrrev_b32 v%d, 1, v%d' % (COFF + k, OFF + k),
                      'v_cmp_gt_i32 s[%d:%d], %s, v%d' % (masks[k], masks[k] + 1, self.np, P)]:
                e.raw(o)
        cvt = 'v_cvt_pk_bf16_f32' if self.bf else 'v_cvt_pk_f16_f32'
        for h in range(2):
            for db in (2 * h, 2 * h + 1):
                for q in range(4):
                    e.raw('ds_write_b128 %%[ew], %s offset:%d' % (vr(ACC + 16 * db + 4 * q, 4), 128 * (db - 2 * h) + 32 * q))
            e.raw('s_waitcnt lgkmcnt(0)')
            for k in range(8):
                e.raw('ds_read_b128 %s, %%[er] offset:%d' % (vr(VT + 4 * k, 4), 4 * k * EPITCH))
            if h == 0:
                # the tiles requested for the next work item have landed before the output stores go out: loads and
                # stores share one counter and return out of order, so later they could not be waited for apart
                e.raw('s_waitcnt vmcnt(0)')
            # %[oc]: 0 = the fp32 rows only, 1 = those and the copy rounded to the input type, 2 = the rounded copy only
            e.raw('s_cmp_eq_u32 %[oc], 0')
            e.raw('s_cbranch_scc0 cast%d_%s' % (h, lbl))
            for wide, with_cast in ((True, False), (True, True), (False, True)):
                if with_cast:
                    e.label('%s%d_%s' % ('cast' if wide else 'only', h, lbl))
                    if wide:
                        e.raw('s_cmp_eq_u32 %[oc], 2')
                        e.raw('s_cbranch_scc1 only%d_%s' % (h, lbl))
                for k in range(8):
                    e.raw('s_waitcnt lgkmcnt(%d)' % (7 - k))
                    e.raw('s_mov_b64 exec, s[%d:%d]' % (masks[k], masks[k] + 1))
                    if wide:
                        e.raw('global_store_dwordx4 v%d, %s, %%[ob] offset:%d nt' % (OFF + k, vr(VT + 4 * k, 4), 256 * h))
                    if with_cast:
                        t = S1 + 2 * k
                        e.raw('%s v%d, v%d, v%d' % (cvt, t, VT + 4 * k, VT + 4 * k + 1))
                        e.raw('%s v%d, v%d, v%d' % (cvt, t + 1, VT + 4 * k + 2, VT + 4 * k + 3))
                        e.raw('global_store_dwordx2 v%d, %s, %%[cb] offset:%d nt' % (COFF + k, vr(t, 2), 128 * h))
                e.raw('s_mov_b64 exec, s[%d:%d]' % (S_EXEC, S_EXEC + 1))
                if wide:
                    e.raw('s_branch half%d_%s' % (h, lbl))
            e.label('half%d_%s' % (h, lbl))
        e.raw('s_branch end_%s' % lbl)
        e.label('done_%s' % lbl)  # idle wavefronts: nothing to write
        e.raw('s_waitcnt vmcnt(0)')
        for o in self.prefetch_next('i', lbl):
            e.raw(o)
        e.raw('s_waitcnt vmcnt(0)')
        e.raw('s_mov_b32 m0, s%d' % S_M0)
        e.label('end_%s' % lbl)
        return e.out


def clobbers():
    c = ['"v%d"' % i for i in range(FIRST_FIXED_VGPR, 256)] + ['"s%d"' % i for i in FIXED_SGPRS]
    return c + ['"vcc"', '"scc"', '"memory"']


def write(path, lines, name):
    with open(path, 'w') as f:
        f.write('// Generated by gen/gen_append_loop.py (%s); do not edit by hand.\n' % name)
        for l in lines:
            f.write('"%s\\n\\t"\n' % l)


if __name__ == '__main__':
    here = os.path.dirname(os.path.abspath(__file__))
    out_dir = sys.argv[1] if len(sys.argv) > 1 else os.path.join(here, '..')
    for bf, cap, contig, name in ((True, False, False, 'bf16'), (False, False, False, 'f16'), (True, True, False, 'bf16_cap'),
                                  (False, True, False, 'f16_cap'), (True, False, True, 'bf16_contig'),
                                  (False, False, True, 'f16_contig'), (True, False, False, 'bf16_var'),
                                  (False, False, False, 'f16_var'), (True, False, False, 'bf16_ps'),
                                  (False, False, False, 'f16_ps'), (True, False, False, 'bf16_rows'),
                                  (False, False, False, 'f16_rows'), (True, False, True, 'bf16_contig_ps'),
                                  (False, False, True, 'f16_contig_ps'), (True, False, True, 'bf16_contig_rows'),
                                  (False, False, True, 'f16_contig_rows')):
        lines = Gen(bf, cap, contig, var=name.endswith('_var'), anyps=name.endswith('_ps'),
                    rowids=name.endswith('_rows')).program()
        write(os.path.join(out_dir, 'append_loop_%s.inc' % name), lines, name)
        n_mfma = sum(1 for l in lines if l.startswith('v_mfma'))
        print('%s: %d lines, %d matrix instructions, %d waits' % (name, len(lines), n_mfma, sum(1 for l in lines if l.startswith('s_waitcnt'))))
    with open(os.path.join(out_dir, 'append_loop_clobbers.inc'), 'w') as f:
        f.write('// Generated by gen/gen_append_loop.py; do not edit by hand.\n')
        f.write(', '.join(clobbers()) + '\n')
