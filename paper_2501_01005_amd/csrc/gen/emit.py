"""Helper for hand-scheduled gfx950 inline assembly.

Keeps the list of LDS operations and of vector-memory loads that are still in flight, both of
which complete in issue order, and puts the counted s_waitcnt in front of the first instruction
that touches a register such an operation writes.  Scalar loads are not tracked: they only make
the LDS counter read higher than assumed, so a counted wait is never too short; their results
are consumed after an explicit lgkmcnt(0).
"""
import re

_REG = re.compile(r'\b([va])(\d+)\b|\b([va])\[(\d+):(\d+)\]')


def regs_of(text):
    out = set()
    for m in _REG.finditer(text):
        if m.group(1):
            out.add((m.group(1), int(m.group(2))))
        else:
            for i in range(int(m.group(4)), int(m.group(5)) + 1):
                out.add((m.group(3), i))
    return out


class Emitter:
    LGKM_MAX = 15  # width of the lgkmcnt field

    def __init__(self):
        self.out = []
        self.lgkm = []  # destination register sets of LDS operations in flight, oldest first
        self.vm = []    # same for global loads

    def _wait_for(self, used):
        need_l = need_v = None
        for i, d in enumerate(self.lgkm):
            if d & used:
                need_l = len(self.lgkm) - 1 - i
        for i, d in enumerate(self.vm):
            if d & used:
                need_v = len(self.vm) - 1 - i
        parts = []
        if need_v is not None:
            parts.append('vmcnt(%d)' % need_v)
            self.vm = self.vm[len(self.vm) - need_v:] if need_v else []
        if need_l is not None:
            n = min(need_l, self.LGKM_MAX)
            parts.append('lgkmcnt(%d)' % n)
            self.lgkm = self.lgkm[len(self.lgkm) - n:] if n else []
        if parts:
            self.out.append('s_waitcnt ' + ' '.join(parts))

    def emit(self, text):
        op = text.split()[0]
        args = text[len(op):].split(',')
        used = regs_of(text)
        if op.startswith('ds_read'):
            self._wait_for(used)
            self.out.append(text)
            self.lgkm.append(regs_of(args[0]))
        elif op.startswith('ds_write'):
            self._wait_for(used)
            self.out.append(text)
            self.lgkm.append(set())
        elif op.startswith('global_load_lds'):  # lands in LDS, not in registers: waited for by wait_lds_loads()
            self._wait_for(used)
            self.out.append(text)
            self.vm.append({('lds', len(self.out))})
        elif op.startswith('global_load'):
            self._wait_for(used)
            self.out.append(text)
            self.vm.append(regs_of(args[0]))
        elif op == 's_barrier':
            self.drain(lgkm=True, vm=False)
            self.out.append(text)
        else:
            self._wait_for(used)
            self.out.append(text)

    def wait_lds_loads(self):
        """counted wait for every global load in flight whose destination is LDS"""
        pending = set()
        for d in self.vm:
            pending |= set(x for x in d if x[0] == 'lds')
        if pending:
            self._wait_for(pending)

    def drain(self, lgkm=True, vm=True):
        parts = []
        if vm and self.vm:
            parts.append('vmcnt(0)')
            self.vm = []
        if lgkm:
            parts.append('lgkmcnt(0)')  # also covers scalar loads, which are not tracked
            self.lgkm = []
        if parts:
            self.out.append('s_waitcnt ' + ' '.join(parts))

    def raw(self, text):
        self.out.append(text)

    def label(self, name):
        self.out.append(name + ':')
