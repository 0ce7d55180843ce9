"""Oracle for the MoE-shaped all-to-all (low-latency dispatch and combine in traffic shape).

TEST INFRASTRUCTURE ONLY, like the rest of this package: imported by tests and by the
benchmark's cpu_baseline leg, never by the GPU package.

What is modelled (Sec. IV-E "Low-Latency Kernel Integration", Sec. V-C "Low-Latency Kernels"):
every PE holds a small batch of tokens, each routed to up to top-k experts; experts are spread
evenly over the PEs.  Dispatch sends, for every (token, expert) route, one message of 16 bytes of
source-index metadata followed by the token's bytes straight into a receive slot at the expert's
owner; once all messages of one (sender, expert) pair are on their way the sender delivers the
pair's token count with a zero-byte put carrying a SignalAdd, so the count can only be seen after
the data (the release/acquire idiom of Sec. IV-B).  The receiver reads the signals and packs what
arrived per local expert.  Combine sends every expert output back to the token's source PE and
raises one flag signal per (expert, destination) pair; the destination then reduces the copies of
each token.  Quantisation, compression and the weighted floating-point reduction are not part of
this model: payloads are opaque bytes and the reduction is a wrapping sum of 32-bit words, which
still forces the receiver to read every message after the acquire.

Choices the paper leaves open (kept identical on the GPU side, stated in the design notes):
- metadata words (int32): source token index, source PE, position in the token's top-k list,
  global expert id;
- the signal of pair (local expert le, sender s) has ID le * npes + s and receives count + 1, so
  that "arrived with zero tokens" differs from "not arrived";
- a (sender, expert) pair's messages occupy slots 0..count-1 in ascending token order, and the
  packed output of a local expert lists senders in ascending PE order.

All steps go through the World's one-sided calls (put, signal_add); in its SHUFFLED mode puts are
delivered late and out of order unless a signal or quiet forces them, so a missing ordering step
shows up as wrong data.
"""
from __future__ import annotations

import numpy as np

META_BYTES = 16


class MoeLayout:
    """Symmetric-heap offsets used by the model (all PEs alike)."""

    def __init__(self, npes, num_experts, max_tokens, topk, hidden_bytes, base=0):
        assert num_experts % npes == 0 and hidden_bytes % 4 == 0
        self.npes, self.num_experts, self.max_tokens, self.topk, self.hidden = npes, num_experts, max_tokens, topk, hidden_bytes
        self.epp = num_experts // npes
        self.msg = META_BYTES + hidden_bytes                      # dispatch message size
        up = lambda v: (v + 255) // 256 * 256
        self.send = base                                           # one message being assembled
        self.recv = up(self.send + self.msg)                       # [epp][npes][max_tokens] dispatch slots
        self.dsig = up(self.recv + self.epp * npes * max_tokens * self.msg)   # uint64 [epp * npes]
        self.comb = up(self.dsig + 8 * self.epp * npes)            # [max_tokens][topk] combine slots
        self.csig = up(self.comb + max_tokens * topk * hidden_bytes)          # uint64 [num_experts]
        self.end = up(self.csig + 8 * num_experts)

    def slot(self, le, s, i):
        return self.recv + ((le * self.npes + s) * self.max_tokens + i) * self.msg


def _sig(w, pe, off):
    return w.heap(pe)[off:off + 8].view(np.uint64)


def dispatch(w, lay: MoeLayout, x: np.ndarray, topk_idx: np.ndarray, ntok: np.ndarray):
    """One dispatch.  x uint8 [npes, max_tokens, hidden]; topk_idx int32 [npes, max_tokens, topk].

    Returns (recv_x uint8 [npes, epp, npes*max_tokens, hidden], recv_info int32 [npes, epp,
    npes*max_tokens, 4], recv_range int32 [npes, epp, npes, 2] = (begin, count), recv_count
    int32 [npes, epp]); unused rows stay zero.
    """
    P, E, T, K, Hb, epp = lay.npes, lay.num_experts, lay.max_tokens, lay.topk, lay.hidden, lay.epp
    # --- senders: per destination expert, its tokens in ascending order, then the count --------
    for s in range(P):
        heap = w.heap(s)
        for e in range(E):
            owner, le = divmod(e, epp)
            n = 0
            for t in range(int(ntok[s])):
                for j in range(K):
                    if int(topk_idx[s, t, j]) != e:
                        continue
                    heap[lay.send:lay.send + META_BYTES] = np.array([t, s, j, e], dtype=np.int32).view(np.uint8)
                    heap[lay.send + META_BYTES:lay.send + lay.msg] = x[s, t]
                    w.put(s, lay.slot(le, s, n), lay.send, lay.msg, owner)    # source is snapshot at the call
                    n += 1
            # zero-byte put + SignalAdd: lands after every earlier put of s to owner is visible there
            w.signal_add(s, lay.dsig + 8 * (le * P + s), n + 1, owner)
    # --- receivers: read the counts, pack per local expert --------------------------------------
    recv_x = np.zeros((P, epp, P * T, Hb), dtype=np.uint8)
    recv_info = np.zeros((P, epp, P * T, 4), dtype=np.int32)
    recv_range = np.zeros((P, epp, P, 2), dtype=np.int32)
    recv_count = np.zeros((P, epp), dtype=np.int32)
    for r in range(P):
        heap = w.heap(r)
        for le in range(epp):
            begin = 0
            for s in range(P):
                sig = _sig(w, r, lay.dsig + 8 * (le * P + s))
                if int(sig[0]) == 0:
                    raise RuntimeError(f"count of pair (expert {r * epp + le}, sender {s}) never arrived")
                n = int(sig[0]) - 1
                sig[0] = 0                                           # ready for the next dispatch
                recv_range[r, le, s] = (begin, n)
                for i in range(n):
                    o = lay.slot(le, s, i)
                    recv_info[r, le, begin + i] = heap[o:o + META_BYTES].view(np.int32)
                    recv_x[r, le, begin + i] = heap[o + META_BYTES:o + lay.msg]
                begin += n
            recv_count[r, le] = begin
    return recv_x, recv_info, recv_range, recv_count


def combine(w, lay: MoeLayout, expert_out: np.ndarray, recv_info: np.ndarray, recv_range: np.ndarray,
            topk_idx: np.ndarray, ntok: np.ndarray, epoch: int = 1):
    """One combine (the `epoch`-th on this layout: flag signals count calls and are never reset).

    expert_out uint8 [npes, epp, npes*max_tokens, hidden] in the packed order dispatch produced.
    Returns combined uint8 [npes, max_tokens, hidden]: per token the wrapping uint32 sum of the
    expert outputs of its valid routes (rows at or beyond ntok stay zero).
    """
    P, T, K, Hb, epp = lay.npes, lay.max_tokens, lay.topk, lay.hidden, lay.epp
    for r in range(P):
        heap = w.heap(r)
        for le in range(epp):
            for s in range(P):
                b, n = (int(v) for v in recv_range[r, le, s])
                for i in range(b, b + n):
                    t, src, j, e = (int(v) for v in recv_info[r, le, i])
                    assert src == s and e == r * epp + le
                    heap[lay.send:lay.send + Hb] = expert_out[r, le, i]
                    w.put(r, lay.comb + (t * K + j) * Hb, lay.send, Hb, s)
                w.signal_add(r, lay.csig + 8 * (r * epp + le), 1, s)       # flag: expert's outputs for s are in
    combined = np.zeros((P, T, Hb), dtype=np.uint8)
    for s in range(P):
        heap = w.heap(s)
        for t in range(int(ntok[s])):
            acc = np.zeros(Hb // 4, dtype=np.uint32)
            for j in range(K):
                e = int(topk_idx[s, t, j])
                if e < 0:
                    continue
                if int(_sig(w, s, lay.csig + 8 * e)[0]) < epoch:
                    raise RuntimeError(f"flag of expert {e} never reached PE {s}")
                o = lay.comb + (t * K + j) * Hb
                acc += heap[o:o + Hb].view(np.uint32)                      # wraps modulo 2^32
            combined[s, t] = acc.view(np.uint8)
    return combined
