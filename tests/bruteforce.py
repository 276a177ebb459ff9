"""Pure-Python brute force used only to pin the CPU oracle on tiny inputs.

No gather, no numpy arithmetic: every (sequence, key) is translated on the fly
through the block table (Algorithm 1: b = t div P, o = t mod P, slot = table[s][b]*P + o)
and every sum is a Python float loop over the textbook softmax definition.
"""
import math
import struct


def bf16_to_float(bits: int) -> float:
    return struct.unpack("<f", struct.pack("<I", (int(bits) & 0xFFFF) << 16))[0]


def value(x, is_bf16):
    return bf16_to_float(x) if is_bf16 else float(x)


def attention(k_cache, v_cache, q, block_table, seq_lens, cu_q_lens, scale, causal, is_bf16):
    """k_cache/v_cache: nested lists [NP][P][Hkv][d]; q: [total_q][Hq][d].
    Returns (out [total_q][Hq][d], lse [total_q][Hq], weights [total_q][Hq][len])."""
    P = len(k_cache[0])
    Hkv = len(k_cache[0][0])
    d = len(k_cache[0][0][0])
    Hq = len(q[0]) if q else 0
    G = Hq // Hkv if Hkv else 0
    out, lse, wts = [], [], []
    for s, L in enumerate(seq_lens):
        Tq = cu_q_lens[s + 1] - cu_q_lens[s]
        for i in range(Tq):
            row = cu_q_lens[s] + i
            out.append([])
            lse.append([])
            wts.append([])
            pos = L - Tq + i
            for h in range(Hq):
                kvh = h // G
                allowed = [j for j in range(L) if (not causal) or j <= pos]
                xs = []
                for j in allowed:
                    page = block_table[s][j // P]
                    o = j % P
                    acc = 0.0
                    for e in range(d):
                        acc += value(q[row][h][e], is_bf16) * value(k_cache[page][o][kvh][e], is_bf16)
                    xs.append(scale * acc)
                if not allowed:
                    out[-1].append([0.0] * d)
                    lse[-1].append(-math.inf)
                    wts[-1].append([])
                    continue
                m = max(xs)
                es = [math.exp(x - m) for x in xs]
                Z = math.fsum(es)
                o_vec = [0.0] * d
                for w, j in zip(es, allowed):
                    page = block_table[s][j // P]
                    o = j % P
                    for e in range(d):
                        o_vec[e] += (w / Z) * value(v_cache[page][o][kvh][e], is_bf16)
                out[-1].append(o_vec)
                lse[-1].append(m + math.log(Z))
                wts[-1].append([w / Z for w in es])
    return out, lse, wts
