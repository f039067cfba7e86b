"""Pool oracle: the per-head ragged KV pool kept as plain Python lists.

TEST INFRASTRUCTURE ONLY (see ``oracle/__init__.py``).

State per head: a list of frames in ascending frame-id order, each frame a
tuple (frame_id, score, K, V) with K, V numpy arrays [tokens_per_frame, D] of
raw 16-bit words.  ``append`` follows the cache life-cycle of Sec. 2.2 (new
keys/values are written into the candidate history after a generation step)
with the per-head retention rules of ``oracle.policy``; ``tables`` lays the
state out the way the flattened pool of Sec. 4.3 is stored: head after head,
each head's frames packed to the left of its region.
"""
import numpy as np

from . import policy as P


class CapacityError(Exception):
    pass


class PoolOracle:
    def __init__(self, policies, tokens_per_frame, head_dim):
        self.policies = list(policies)
        self.tpf = tokens_per_frame
        self.D = head_dim
        self.T = 0
        self.frames = [[] for _ in self.policies]       # per head: [(id, score, K, V)]

    # ------------------------------------------------------------------ append
    def append(self, k_new, v_new, scores=None):
        """k_new, v_new: uint16 [H, n_new, tpf, D]; scores: float32 [H, n_new] or None."""
        H = len(self.policies)
        n_new = k_new.shape[1]
        assert k_new.shape == (H, n_new, self.tpf, self.D) and v_new.shape == k_new.shape
        T_new = self.T + n_new
        staged = []
        for h, pol in enumerate(self.policies):
            cand = list(self.frames[h])
            for j in range(n_new):
                sc = np.float32(0.0) if scores is None else np.float32(scores[h, j])
                cand.append((self.T + j, sc, k_new[h, j].copy(), v_new[h, j].copy()))
            score_of = {f[0]: f[1] for f in cand}
            keep = set(P.retained_frames(pol, T_new, [f[0] for f in cand], score_of))
            kept = [f for f in cand if f[0] in keep]
            if len(kept) > pol.slots - self.merged_slots(pol):
                raise CapacityError("head %d needs %d slots, has %d" % (h, len(kept), pol.slots - self.merged_slots(pol)))
            staged.append(kept)
        self.frames = staged                            # nothing changes if any head overflowed
        self.T = T_new

    # ----------------------------------------------------------- cache merging
    @staticmethod
    def merged_slots(pol):
        """Slots at the end of a head's region reserved for merged frames (Veil heads with cache merging)."""
        return pol.cap if (pol.type == P.VEIL and pol.cap > 0) else 0

    def merged_frame(self, h, w0):
        """K, V (uint16 [tpf, D]) of the merged frame of the window starting at frame w0 (Sec. 4.2): row r is token
        ``tok`` of frame w0+i for the r-th (i, tok) pair of ``policy.merged_rows``."""
        pol = self.policies[h]
        by_id = {f[0]: f for f in self.frames[h]}
        K = np.zeros((self.tpf, self.D), np.uint16)
        V = np.zeros((self.tpf, self.D), np.uint16)
        for r, (i, tok) in enumerate(P.merged_rows(pol.period, self.tpf)):
            K[r] = by_id[w0 + i][2][tok]
            V[r] = by_id[w0 + i][3][tok]
        return K, V

    def merged_windows(self, h):
        """[(local slot, w0)] of the merged frames head h holds at the current history length: window j
        (0 = nearest) sits in the head's slot ``slots - 1 - j``."""
        pol = self.policies[h]
        if not self.merged_slots(pol):
            return []
        out = []
        for j in range(pol.cap):
            w0 = self.T - pol.recent - (j + 1) * pol.period
            if w0 >= pol.sink:
                out.append((pol.slots - 1 - j, w0))
        return out

    # ------------------------------------------------------------------ layout
    def slot_base(self):
        base = [0]
        for pol in self.policies:
            base.append(base[-1] + pol.slots)
        return base

    def tables(self):
        """n_frames [H], frame_ids [total_slots] (-1 = free), frame_score [total_slots] (0 = free)."""
        base = self.slot_base()
        n_frames = np.zeros(len(self.policies), np.int32)
        frame_ids = np.full(base[-1], -1, np.int32)
        frame_score = np.zeros(base[-1], np.float32)
        for h, fr in enumerate(self.frames):
            n_frames[h] = len(fr)
            for j, f in enumerate(fr):
                frame_ids[base[h] + j] = f[0]
                frame_score[base[h] + j] = f[1]
            for slot, w0 in self.merged_windows(h):
                frame_ids[base[h] + slot] = P.MERGED | w0
        return n_frames, frame_ids, frame_score

    def resident_kv(self):
        """Yield (global_slot, K, V) for every resident frame, merged frames included."""
        base = self.slot_base()
        for h, fr in enumerate(self.frames):
            for j, f in enumerate(fr):
                yield base[h] + j, f[2], f[3]
            for slot, w0 in self.merged_windows(h):
                K, V = self.merged_frame(h, w0)
                yield base[h] + slot, K, V

    # ------------------------------------------------------------------- index
    def build_index(self, max_sel):
        """sel_count [H], sel_frames / sel_slots [H, max_sel] (-1 padded; slots are
        global pool slots), cu_seqlens [H+1] in tokens of selected history."""
        base = self.slot_base()
        H = len(self.policies)
        sel_count = np.zeros(H, np.int32)
        sel_frames = np.full((H, max_sel), -1, np.int32)
        sel_slots = np.full((H, max_sel), -1, np.int32)
        for h, pol in enumerate(self.policies):
            score_of = {f[0]: f[1] for f in self.frames[h]}
            where = {f[0]: j for j, f in enumerate(self.frames[h])}
            where.update({P.MERGED | w0: slot for slot, w0 in self.merged_windows(h)})
            sel = P.selected_frames(pol, self.T, score_of)
            assert len(sel) <= max_sel
            sel_count[h] = len(sel)
            for j, f in enumerate(sel):
                sel_frames[h, j] = f
                sel_slots[h, j] = base[h] + where[f]    # KeyError = selection not resident
        cu = np.asarray(P.cu_seqlens(sel_count.tolist(), self.tpf), np.int32)
        return sel_count, sel_frames, sel_slots, cu

    def head_kv(self, h, frame_ids):
        """Concatenated K, V (uint16 [len*tpf, D]) of the given frames of head h."""
        by_id = {f[0]: f for f in self.frames[h]}
        ks, vs = [], []
        for f in frame_ids:
            if f & P.MERGED:
                K, V = self.merged_frame(h, f & ~P.MERGED)
            else:
                K, V = by_id[f][2], by_id[f][3]
            ks.append(K)
            vs.append(V)
        if not ks:
            z = np.zeros((0, self.D), np.uint16)
            return z, z
        return np.concatenate(ks, 0), np.concatenate(vs, 0)

