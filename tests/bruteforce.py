"""Independent brute-force statement of the estimate, used to pin the C oracle.

Deliberately shares nothing with oracle/: no path lists (recursion over the successor
lists from the request's own stage), queue position by O(n^2) counting, Python's
unbounded integers.  Only usable on tiny inputs.
"""
from fractions import Fraction
import math

INT32_MAX = 2**31 - 1


def _succ(S, row_ptr, col):
    return [[int(col[e]) for e in range(int(row_ptr[s]), int(row_ptr[s + 1]))] for s in range(S)]


def cost(lat, B, W, a):
    """wait of a requests ahead + execution, via exact rationals (floor at the end of the wait)."""
    batches = math.ceil(Fraction(a, B))
    wait = math.floor(Fraction(batches * int(lat[B - 1]), W))
    return wait + int(lat[min(B, a + 1) - 1])


def brute(w, consistent=False, ranked=False):
    """est, drop, pos for every request of workload w (any K).  consistent: a request's position
    counts only the requests ahead of it that were kept, decided one after the other in queue order.
    ranked: in a later queue the request is put where that queue's order puts a newcomer with its
    deadline (behind the requests already there when keys tie, at the very back in arrival order),
    and the requests ahead of it are the ones in front of that place."""
    n = w.n
    est = [0] * n
    drop = [0] * n
    pos = [0] * n
    for u in range(w.K):
        d = 0 if w.dag_shared else u
        S = w.S
        rp = w.dag_row_ptr[d * (S + 1):(d + 1) * (S + 1)]
        base = sum(int(w.dag_row_ptr[dd * (S + 1) + S]) for dd in range(d))
        cl = w.dag_col[base:base + int(rp[S])]
        succ = _succ(S, rp, cl)
        B = w.batch[d * S:(d + 1) * S]
        W = w.workers[d * S:(d + 1) * S]
        L = w.lat_us[d * S * 64:(d + 1) * S * 64].reshape(S, 64)
        M = w.order_mode[d * S:(d + 1) * S]
        lo, hi = int(w.snap_ptr[u]), int(w.snap_ptr[u + 1])
        stage = [min(max(int(s), 0), S - 1) for s in w.stage[lo:hi]]
        qlen = [stage.count(s) for s in range(S)]

        def key(i):
            s = stage[i]
            if M[s] == 1:
                return -int(w.deadline[lo + i])
            if M[s] == 2:
                return int(w.arrival[lo + i])
            return int(w.deadline[lo + i])

        def place(t, i):             # requests in front of request i once it has joined the queue of stage t
            if not ranked:
                return qlen[t]
            newcomer = hi - lo           # an index after everybody's: loses every tie
            if M[t] == 2:
                rows = [(int(w.arrival[lo + j]), j) for j in range(hi - lo) if stage[j] == t] + [(math.inf, newcomer)]
            else:
                sign = -1 if M[t] == 1 else 1
                rows = [(sign * int(w.deadline[lo + j]), j) for j in range(hi - lo) if stage[j] == t]
                rows.append((sign * int(w.deadline[lo + i]), newcomer))
            return sorted(rows).index(rows[-1])

        def downstream(s, i=None):   # worst total cost of everything after stage s (for request i when ranked)
            best = 0
            for t in succ[s]:
                best = max(best, cost(L[t], int(B[t]), int(W[t]), place(t, i)) + downstream(t, i))
            return best

        if not consistent:
            for i in range(hi - lo):
                k = stage[i]
                ahead = sum(1 for j in range(hi - lo)
                            if stage[j] == k and (key(j), j) < (key(i), i))
                e = cost(L[k], int(B[k]), int(W[k]), ahead) + downstream(k, i)
                pos[lo + i] = ahead
                est[lo + i] = min(e, INT32_MAX)
                finish = min(int(w.now[u]) + e, INT32_MAX)
                drop[lo + i] = 1 if finish > int(w.deadline[lo + i]) else 0
        else:
            for k in range(S):
                queue = sorted((i for i in range(hi - lo) if stage[i] == k), key=lambda i: (key(i), i))
                kept = 0
                for i in queue:
                    e = cost(L[k], int(B[k]), int(W[k]), kept) + downstream(k)
                    pos[lo + i] = kept
                    est[lo + i] = min(e, INT32_MAX)
                    finish = min(int(w.now[u]) + e, INT32_MAX)
                    drop[lo + i] = 1 if finish > int(w.deadline[lo + i]) else 0
                    kept += 1 - drop[lo + i]
    return est, drop, pos
