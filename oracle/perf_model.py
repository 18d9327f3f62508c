"""CPU checker (test infrastructure only) for the paper's performance model and node assignment: the closed forms
of Sec. 4.2.1 (Eqs. 2-4), the program of Sec. 4.2.2 (Eq. 5) solved by plain enumeration, and the parameter-server
model of Sec. 7.1 (Eqs. 6-7).  Counts are numbers of 32-bit values, bandwidth is bit/s."""
import math

BITS = 32.0


def allreduce_rounds(n_c: int) -> int:
    """Recursive doubling (Sec. 4.1.2): log2 n_c rounds for a power of two, otherwise one round to fold the surplus
    workers in, floor(log2 n_c) doubling rounds, and one round to send the result back."""
    if n_c <= 1:
        return 0
    lg = int(math.floor(math.log2(n_c)))
    while 2 ** (lg + 1) <= n_c:      # guard the float log
        lg += 1
    while 2 ** lg > n_c:
        lg -= 1
    return lg if 2 ** lg == n_c else lg + 2


def stanza_time(T_c, T_f, A, K, P_c, bw, n_c, n_f):
    t_compute = T_c + (n_c / n_f) * T_f                              # Eq. 2
    t_conv_fc = 2 * n_c * A * K * BITS / (n_f * bw)                  # activations out, gradients back
    t_conv = P_c * BITS * allreduce_rounds(n_c) / bw                 # one P_c-sized message per round
    return t_compute + t_conv_fc + t_conv                            # Eq. 3


def stanza_throughput(T_c, T_f, A, K, P_c, bw, n_c, n_f):
    return n_c * K / stanza_time(T_c, T_f, A, K, P_c, bw, n_c, n_f)  # Eq. 4


def assign(T_c, T_f, A, K, P_c, bw, N):
    """Eq. 5 by exhaustive search; ties go to the smallest n_c."""
    best = max(range(1, N), key=lambda c: (stanza_throughput(T_c, T_f, A, K, P_c, bw, c, N - c), -c))
    return best, N - best, stanza_throughput(T_c, T_f, A, K, P_c, bw, best, N - best)


def ps_time(P, T_ps, n_w, n_s, bw):
    return 2 * n_w * P * BITS / (n_s * bw) + T_ps                    # Eq. 6


def ps_throughput(P, T_ps, K, n_w, n_s, bw):
    return n_w * K / ps_time(P, T_ps, n_w, n_s, bw)                  # Eq. 7
