"""Scheduler oracle: Bubble Monitor zero-count, Algorithm 1 and the Kernel Barrier rules.

Follows Sec. 3.3: the monitor records the number of training kernels issued per period into a sliding window
and reports the number of continuous zero counts Z_c; Algorithm 1 maps Z_c to (tokens, status) in three
phases; the barrier forwards queued inference kernels while tokens last (offline) or pulls one request at a
time while the status is idle (online).

Readings where Algorithm 1 is silent (all integers, floor division):
  * `tokens * gamma` can never leave 0 after the conservative phase, so the state is a per-GPU `pool`
    that restarts from a seed T0:  pool <- min(limit, floor(max(pool, T0) * gamma)),  limit = LL
    (incremental) or UL (stable);  the conservative phase sets pool <- 0.
  * the value handed to each of the m instances is grant = floor(pool / m); the pool, not the grant, is
    what the next period multiplies (otherwise the grant shrinks whenever gamma <= m).
  * gamma is the rational gamma_num / gamma_den.
  * a grant replaces the instance's balance each period; a queued kernel is forwarded iff balance >= cost,
    then balance -= cost; FIFO, the head of the queue blocks what is behind it.
The constants themselves (alpha, beta, gamma, LL, UL, T0) are not given by the paper: parity unpinned.
"""
from collections import deque

BUSY, IDLE = 0, 1


def zero_count(window):
    """Number of consecutive zero counts ending at the newest sample (last element)."""
    z = 0
    for c in reversed(list(window)):
        if c != 0:
            break
        z += 1
    return z


class BubbleMonitor:
    """Sliding window of per-period kernel counts (Sec. 3.3 "Bubble Monitor")."""

    def __init__(self, window):
        self.window = deque(maxlen=window)

    def push(self, count):
        self.window.append(int(count))
        return zero_count(self.window)


def alg1_step(zc, pool, alpha, beta, gamma_num, gamma_den, m, ll, ul, t0):
    """One evaluation of Algorithm 1.  Returns (pool', grant per instance, status)."""
    if zc <= alpha:                                   # conservative phase
        return 0, 0, BUSY
    grown = (max(pool, t0) * gamma_num) // gamma_den
    if zc <= beta:                                    # incremental phase
        pool = min(ll, grown)
        return pool, pool // m, BUSY
    pool = min(ul, grown)                             # stable phase
    return pool, pool // m, IDLE


def kb_release(costs, balance):
    """Offline barrier: how many kernels from the head of the FIFO `costs` are forwarded with `balance`
    tokens.  Returns (n_released, balance left)."""
    n = 0
    for c in costs:
        if balance < c:
            break
        balance -= c
        n += 1
    return n, balance


def online_pull_ok(status, queue_len, predicted_remaining, predicted_request):
    """Online barrier: pull exactly one request iff the status is idle, a request waits, and the predicted
    rest of the bubble holds it (Principle-II guarantees this can be true at least once per iteration)."""
    return status == IDLE and queue_len > 0 and predicted_remaining >= predicted_request


def run_trace(counts, costs, window, alpha, beta, gamma_num, gamma_den, m, ll, ul, t0):
    """Drive monitor -> Algorithm 1 -> offline barrier over a trace of per-period training-kernel counts.
    `costs` is the FIFO of queued inference kernel costs.  Returns one tuple per period:
    (Z_c, pool, grant, status, n_released)."""
    bm = BubbleMonitor(window)
    pool, head, out = 0, 0, []
    for c in counts:
        zc = bm.push(c)
        pool, grant, status = alg1_step(zc, pool, alpha, beta, gamma_num, gamma_den, m, ll, ul, t0)
        n, _ = kb_release(costs[head:], grant)
        head += n
        out.append((zc, pool, grant, status, n))
    return out


def principle_1(peak_bytes, capacity_bytes):
    """Collocation Principle-I (Sec. 3.2): the peaks of all collocated instances must sum below capacity."""
    return sum(peak_bytes) < capacity_bytes


def principle_2(min_exec_ns, max_bubble_ns):
    """Collocation Principle-II (Sec. 3.2): a batch-1 online request must be shorter than the longest bubble."""
    return min_exec_ns < max_bubble_ns


# ---- concurrent filling with feedback (Sec. 5.2, the outlook given for pipeline parallelism) ---------------
# The paper's stated plan for pipeline-parallel training: run inference beside training as much as possible
# until the Bubble Monitor sees that training iterations have become longer.  It gives no rule; the reading
# taken here is additive increase / multiplicative decrease on a share of wall time, in parts per million:
#   * `share` = fraction of a busy period during which an inference kernel may be running;
#   * after every training iteration: if it took longer than ref * (1 + eps) the share is halved, otherwise it
#     grows by `add` up to `cap`;
#   * bubbles keep being filled under Algorithm 1's tokens; beside that the barrier keeps a time account for the
#     busy phases: every period adds period * share, never above `burst`; a kernel that the tokens do not cover
#     is forwarded iff the account holds its predicted time, which is then taken off.
# Parity unpinned against the paper (it prints neither a rule nor constants).
PPM = 1_000_000


def feedback_share(share_ppm, step_ns, ref_ns, eps_ppm, add_ppm, cap_ppm=PPM):
    """Share of busy time granted to inference after an iteration that took step_ns (reference ref_ns)."""
    if step_ns * PPM > ref_ns * (PPM + eps_ppm):      # the iteration has lengthened: back off
        return share_ppm // 2
    return min(cap_ppm, share_ppm + add_ppm)


def concurrent_account(balance_ns, share_ppm, period_ns, burst_ns):
    """Time account of the barrier after one period."""
    return min(burst_ns, balance_ns + (period_ns * share_ppm) // PPM)
