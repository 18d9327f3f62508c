// Performance model and node assignment of the paper (Sec. 4.2: Eqs. 2-5; Sec. 7.1: Eqs. 6-7): host arithmetic
// that turns the measured single-worker times of the kernels in this library into an iteration time and a
// CONV/FC worker split.  No device code.
#include "../../include/stanza.h"

static const double kBitsPerValue = 32.0;

extern "C" int32_t stanza_model_allreduce_rounds(int32_t n_c)
{
    if (n_c <= 1) return 0;
    int32_t lg = 0;
    while ((int64_t(1) << (lg + 1)) <= n_c) ++lg;          // floor(log2 n_c)
    return ((int64_t(1) << lg) == n_c) ? lg : lg + 2;
}

static bool model_ok(const stanza_model_params *m)
{
    return m && m->T_c >= 0 && m->T_f >= 0 && m->A >= 0 && m->K > 0 && m->P_c >= 0 && m->bandwidth_bits > 0;
}

extern "C" double stanza_model_stanza_time(const stanza_model_params *m, int32_t n_c, int32_t n_f)
{
    if (!model_ok(m) || n_c < 1 || n_f < 1) return -1.0;
    const double compute = m->T_c + ((double)n_c / n_f) * m->T_f;
    const double conv_fc = 2.0 * n_c * m->A * m->K * kBitsPerValue / (n_f * m->bandwidth_bits);
    const double conv_conv = m->P_c * kBitsPerValue * stanza_model_allreduce_rounds(n_c) / m->bandwidth_bits;
    return compute + conv_fc + conv_conv;
}

extern "C" double stanza_model_stanza_throughput(const stanza_model_params *m, int32_t n_c, int32_t n_f)
{
    const double t = stanza_model_stanza_time(m, n_c, n_f);
    return t > 0 ? n_c * m->K / t : -1.0;
}

extern "C" int stanza_model_assign(const stanza_model_params *m, int32_t N, int32_t *n_c, int32_t *n_f, double *throughput)
{
    if (!m || !n_c || !n_f) return STANZA_ENULL;
    if (!model_ok(m) || N < 2) return STANZA_EINVAL;
    double best = -1.0;
    int32_t arg = 1;
    for (int32_t c = 1; c < N; ++c) {                      // ties: the smallest n_c wins
        const double th = stanza_model_stanza_throughput(m, c, N - c);
        if (th > best) { best = th; arg = c; }
    }
    *n_c = arg;
    *n_f = N - arg;
    if (throughput) *throughput = best;
    return STANZA_OK;
}

extern "C" double stanza_model_ps_time(double P, double T_ps, int32_t n_w, int32_t n_s, double bandwidth_bits)
{
    if (P < 0 || T_ps < 0 || n_w < 1 || n_s < 1 || !(bandwidth_bits > 0)) return -1.0;
    return 2.0 * n_w * P * kBitsPerValue / (n_s * bandwidth_bits) + T_ps;
}

extern "C" double stanza_model_ps_throughput(double P, double T_ps, double K, int32_t n_w, int32_t n_s, double bandwidth_bits)
{
    const double t = stanza_model_ps_time(P, T_ps, n_w, n_s, bandwidth_bits);
    return (t > 0 && K > 0) ? n_w * K / t : -1.0;
}
