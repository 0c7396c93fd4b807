// CPU oracle for the MoE layer forward.  TEST INFRASTRUCTURE ONLY: see the header
// for the definition it states (steps O1..O7), the readings of the paper it
// takes, and who may call it.  Plain loops, double accumulation, no blocking,
// no BLAS, no intrinsics.  OpenMP only spreads independent rows over cores.
#include "moe_oracle.h"

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

int g_threads = 0;  // 0 = OpenMP default

// ---- storage dtypes: exact widening ------------------------------------------------
inline float bits_to_float(uint32_t u) {
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}
inline uint32_t float_to_bits(float f) {
    uint32_t u;
    std::memcpy(&u, &f, 4);
    return u;
}

struct F32 {
    typedef float store_t;
    static double load(const void* p, int64_t i) { return (double)((const float*)p)[i]; }
};
struct BF16 {
    typedef uint16_t store_t;
    // bfloat16 is the upper half of an IEEE binary32
    static double load(const void* p, int64_t i) {
        return (double)bits_to_float((uint32_t)((const uint16_t*)p)[i] << 16);
    }
};
struct F16 {
    typedef uint16_t store_t;
    // IEEE binary16: 1 sign, 5 exponent (bias 15), 10 fraction bits
    static double load(const void* p, int64_t i) {
        const uint16_t h = ((const uint16_t*)p)[i];
        const int sign = h >> 15, ex = (h >> 10) & 31, fr = h & 1023;
        double v;
        if (ex == 0) v = std::ldexp((double)fr, -24);                   // subnormal / zero
        else if (ex == 31) v = fr ? NAN : INFINITY;
        else v = std::ldexp((double)(fr | 1024), ex - 25);
        return sign ? -v : v;
    }
};

// Round a double to a binary format with `p` significand bits (hidden bit counted),
// minimum normal exponent `emin`, largest finite exponent `emax`; ties to even.
// The result is returned as a double that the format represents exactly.
double round_to_format(double v, int p, int emin, int emax) {
    if (v == 0.0 || std::isnan(v) || std::isinf(v)) return v;
    int e = std::ilogb(v);
    if (e < emin) e = emin;                                  // subnormal range: fixed quantum
    const double q = std::ldexp(1.0, e - (p - 1));
    double r = std::nearbyint(v / q) * q;                    // default rounding mode: nearest even
    const double maxfin = std::ldexp(2.0 - std::ldexp(1.0, -(p - 1)), emax);
    if (std::fabs(r) > maxfin) r = std::copysign(INFINITY, v);
    return r;
}

uint16_t double_to_bf16_bits(double v) {
    const double r = round_to_format(v, 8, -126, 127);
    return (uint16_t)(float_to_bits((float)r) >> 16);         // exact: r fits in bf16
}

uint16_t double_to_f16_bits(double v) {
    const double r = round_to_format(v, 11, -14, 15);
    const uint16_t sign = std::signbit(r) ? 0x8000 : 0;
    const double a = std::fabs(r);
    if (std::isnan(r)) return 0x7e00;
    if (std::isinf(r)) return sign | 0x7c00;
    if (a == 0.0) return sign;
    const int e = std::ilogb(a);
    if (e < -14) return sign | (uint16_t)std::ldexp(a, 24);   // subnormal: a = fr * 2^-24
    const uint16_t fr = (uint16_t)(std::ldexp(a, 10 - e) - 1024.0);
    return sign | (uint16_t)((e + 15) << 10) | fr;
}

// ---- activation --------------------------------------------------------------------
double activation(double v, int act) {
    switch (act) {
        case 0: return v > 0.0 ? v : 0.0;
        case 1: {  // GELU, tanh form
            const double c = std::sqrt(2.0 / M_PI);
            return 0.5 * v * (1.0 + std::tanh(c * (v + 0.044715 * v * v * v)));
        }
        case 2: return 0.5 * v * (1.0 + std::erf(v / std::sqrt(2.0)));  // GELU, erf form
        default: return v;
    }
}

// derivative of the activation with respect to its argument
double activation_grad(double v, int act) {
    switch (act) {
        case 0: return v > 0.0 ? 1.0 : 0.0;
        case 1: {  // d/dv [ v/2 (1 + tanh u) ], u = c (v + 0.044715 v^3)
            const double c = std::sqrt(2.0 / M_PI);
            const double t = std::tanh(c * (v + 0.044715 * v * v * v));
            return 0.5 * (1.0 + t) + 0.5 * v * (1.0 - t * t) * c * (1.0 + 3.0 * 0.044715 * v * v);
        }
        case 2:    // d/dv [ v Phi(v) ] = Phi(v) + v pdf(v)
            return 0.5 * (1.0 + std::erf(v / std::sqrt(2.0))) + v * std::exp(-0.5 * v * v) / std::sqrt(2.0 * M_PI);
        default: return 1.0;
    }
}

// ---- B1..B5: gradients of the layer under a fixed routing (see the header) ----------
template <class S>
void backward_t(const void* x, const void* Wg, const float* gate_bias, const void* W1, const void* b1,
                const void* W2, const void* b2, const int32_t* topk_expert, const int32_t* slot,
                const double* dout, int T, int H, int I, int E, int k, int act, double* dx, double* dWg,
                double* dgate_bias, double* dW1, double* db1, double* dW2, double* db2) {
    const int64_t P = (int64_t)T * k;
    // B1: combine weights as functions of the logits, in double (softmax over the k selected logits)
    std::vector<double> w(P);
    for (int i = 0; i < T; ++i) {
        std::vector<double> l(k);
        double m = -INFINITY;
        for (int j = 0; j < k; ++j) {
            const int e = topk_expert[(int64_t)i * k + j];
            double acc = gate_bias ? (double)gate_bias[e] : 0.0;
            for (int h = 0; h < H; ++h) acc += S::load(x, (int64_t)i * H + h) * S::load(Wg, (int64_t)h * E + e);
            l[j] = acc;
            if (acc > m) m = acc;
        }
        double z = 0.0;
        for (int j = 0; j < k; ++j) z += std::exp(l[j] - m);
        for (int j = 0; j < k; ++j) w[(int64_t)i * k + j] = std::exp(l[j] - m) / z;
    }
    std::vector<double> dweight(P, 0.0);                     // dL/dw_ij; stays zero for dropped pairs
    std::vector<double> dx_pair((size_t)P * H, 0.0);         // the expert path's part of dL/dx_i, per pair
    // B2 + B3, one expert at a time (an expert's gradients depend on its own kept pairs only)
#pragma omp parallel for schedule(dynamic, 1)
    for (int e = 0; e < E; ++e) {
        std::vector<double> a(I), hh(I), da(I), y(H), gy(H);
        const int64_t w1 = (int64_t)e * H * I, w2 = (int64_t)e * I * H;
        for (int i = 0; i < T; ++i)
            for (int j = 0; j < k; ++j) {
                const int64_t p = (int64_t)i * k + j;
                if (topk_expert[p] != e || slot[p] < 0) continue;
                // forward of this pair: a = x W1 + b1, h = phi(a), y = h W2 + b2
                for (int q = 0; q < I; ++q) a[q] = b1 ? S::load(b1, (int64_t)e * I + q) : 0.0;
                for (int h = 0; h < H; ++h) {
                    const double xv = S::load(x, (int64_t)i * H + h);
                    for (int q = 0; q < I; ++q) a[q] += xv * S::load(W1, w1 + (int64_t)h * I + q);
                }
                for (int q = 0; q < I; ++q) hh[q] = activation(a[q], act);
                for (int h = 0; h < H; ++h) y[h] = b2 ? S::load(b2, (int64_t)e * H + h) : 0.0;
                for (int q = 0; q < I; ++q)
                    for (int h = 0; h < H; ++h) y[h] += hh[q] * S::load(W2, w2 + (int64_t)q * H + h);
                // out_i = sum_j w_ij y_ij:  dL/dw_ij = <dout_i, y_ij>,  dL/dy_ij = w_ij dout_i
                double dw = 0.0;
                for (int h = 0; h < H; ++h) dw += dout[(int64_t)i * H + h] * y[h];
                dweight[p] = dw;
                for (int h = 0; h < H; ++h) gy[h] = w[p] * dout[(int64_t)i * H + h];
                // through y = h W2 + b2
                if (db2) for (int h = 0; h < H; ++h) db2[(int64_t)e * H + h] += gy[h];
                for (int q = 0; q < I; ++q) {
                    double dh = 0.0;
                    for (int h = 0; h < H; ++h) {
                        if (dW2) dW2[w2 + (int64_t)q * H + h] += hh[q] * gy[h];
                        dh += gy[h] * S::load(W2, w2 + (int64_t)q * H + h);
                    }
                    da[q] = dh * activation_grad(a[q], act);
                }
                // through a = x W1 + b1
                if (db1) for (int q = 0; q < I; ++q) db1[(int64_t)e * I + q] += da[q];
                for (int h = 0; h < H; ++h) {
                    const double xv = S::load(x, (int64_t)i * H + h);
                    double g = 0.0;
                    for (int q = 0; q < I; ++q) {
                        if (dW1) dW1[w1 + (int64_t)h * I + q] += xv * da[q];
                        g += da[q] * S::load(W1, w1 + (int64_t)h * I + q);
                    }
                    dx_pair[(size_t)p * H + h] = g;
                }
            }
    }
    // B4 + B5, token by token: softmax Jacobian of the gate, then both paths into x
    for (int i = 0; i < T; ++i) {
        double mean = 0.0;                                   // sum_j w_ij dL/dw_ij
        for (int j = 0; j < k; ++j) mean += w[(int64_t)i * k + j] * dweight[(int64_t)i * k + j];
        if (dx)
            for (int h = 0; h < H; ++h) {
                double g = 0.0;
                for (int j = 0; j < k; ++j) g += dx_pair[((size_t)i * k + j) * H + h];
                dx[(int64_t)i * H + h] = g;
            }
        for (int j = 0; j < k; ++j) {
            const int e = topk_expert[(int64_t)i * k + j];
            const double dl = w[(int64_t)i * k + j] * (dweight[(int64_t)i * k + j] - mean);
            if (dgate_bias) dgate_bias[e] += dl;
            for (int h = 0; h < H; ++h) {
                if (dWg) dWg[(int64_t)h * E + e] += S::load(x, (int64_t)i * H + h) * dl;
                if (dx) dx[(int64_t)i * H + h] += dl * S::load(Wg, (int64_t)h * E + e);
            }
        }
    }
}

// ---- O6: one expert FFN applied to one token row (Eq. ffn, row-vector reading) -----
template <class S>
void ffn_row(const void* x, int64_t token, const void* W1, const void* b1, const void* W2,
             const void* b2, int64_t expert, int H, int I, int act, double* hbuf, double* y) {
    const int64_t w1_base = expert * (int64_t)H * I;   // W1[e] is [H, I]
    const int64_t w2_base = expert * (int64_t)I * H;   // W2[e] is [I, H]
    for (int i = 0; i < I; ++i) hbuf[i] = b1 ? S::load(b1, expert * I + i) : 0.0;
    for (int h = 0; h < H; ++h) {
        const double xv = S::load(x, token * H + h);
        for (int i = 0; i < I; ++i) hbuf[i] += xv * S::load(W1, w1_base + (int64_t)h * I + i);
    }
    for (int i = 0; i < I; ++i) hbuf[i] = activation(hbuf[i], act);
    for (int h = 0; h < H; ++h) y[h] = b2 ? S::load(b2, expert * H + h) : 0.0;
    for (int i = 0; i < I; ++i) {
        const double hv = hbuf[i];
        for (int h = 0; h < H; ++h) y[h] += hv * S::load(W2, w2_base + (int64_t)i * H + h);
    }
}

template <class S>
void ffn_rows_t(const void* x, const void* W1, const void* b1, const void* W2, const void* b2,
                const int32_t* pair_token, const int32_t* pair_expert, int n, int H, int I,
                int act, double* y) {
#pragma omp parallel
    {
        std::vector<double> hbuf(I);
#pragma omp for schedule(dynamic, 1)
        for (int p = 0; p < n; ++p)
            ffn_row<S>(x, pair_token[p], W1, b1, W2, b2, pair_expert[p], H, I, act, hbuf.data(),
                       y + (int64_t)p * H);
    }
}

template <class S>
void gate_logits_t(const void* x, const void* Wg, const float* bias, int T, int H, int E,
                   float* logits) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < T; ++i) {
        std::vector<double> acc(E);
        for (int e = 0; e < E; ++e) acc[e] = bias ? (double)bias[e] : 0.0;
        for (int h = 0; h < H; ++h) {
            const double xv = S::load(x, (int64_t)i * H + h);
            for (int e = 0; e < E; ++e) acc[e] += xv * S::load(Wg, (int64_t)h * E + e);
        }
        for (int e = 0; e < E; ++e) logits[(int64_t)i * E + e] = (float)acc[e];
    }
}

struct ThreadScope {
    int saved;
    ThreadScope() : saved(0) {
#ifdef _OPENMP
        saved = omp_get_max_threads();
        if (g_threads > 0) omp_set_num_threads(g_threads);
#endif
    }
    ~ThreadScope() {
#ifdef _OPENMP
        omp_set_num_threads(saved);
#endif
    }
};

}  // namespace

extern "C" {

int oracle_set_threads(int n) {
    g_threads = n > 0 ? n : 0;
    return oracle_get_threads();
}

int oracle_get_threads(void) {
#ifdef _OPENMP
    return g_threads > 0 ? g_threads : omp_get_max_threads();
#else
    return 1;
#endif
}

int32_t oracle_capacity(int32_t T, int32_t E, int32_t k, float cf, int32_t capacity_override) {
    if (T <= 0 || E <= 0 || k <= 0 || k > E) return -1;
    if (capacity_override > 0) return capacity_override;
    if (!(cf > 0.0f)) return -1;
    const double c = std::ceil((double)cf * (double)k * (double)T / (double)E);
    return c < 1.0 ? 1 : (int32_t)c;
}

int32_t oracle_capacity_layout(int32_t T, int32_t E, float cf) {
    if (T <= 0 || E <= 0 || !(cf > 0.0f)) return -1;
    const double c = std::ceil((double)cf * (double)T / (double)E);
    return c < 1.0 ? 1 : (int32_t)c;
}

int32_t oracle_align_up(int32_t C, int32_t bM) { return ((C + bM - 1) / bM) * bM; }

double oracle_symmetric_layout_bytes(int64_t S, int64_t E, int64_t H, int64_t bM,
                                     int64_t elem_bytes) {
    const int64_t C = (S + E - 1) / E;                       // uniform case of Sec. 3.2
    const int64_t C_pad = ((C + bM - 1) / bM) * bM;          // in-place padding, Sec. 3.2.1
    return 4.0 * (double)E * (double)C_pad * (double)H * (double)elem_bytes;
}

double oracle_activation(double v, int32_t act) { return activation(v, act); }

double oracle_load_elem(const void* p, int64_t idx, int32_t dtype) {
    return dtype == 0 ? F32::load(p, idx) : dtype == 1 ? BF16::load(p, idx) : F16::load(p, idx);
}

void oracle_store_elem(void* p, int64_t idx, int32_t dtype, double v) {
    if (dtype == 0) ((float*)p)[idx] = (float)v;             // double -> float is RNE
    else if (dtype == 1) ((uint16_t*)p)[idx] = double_to_bf16_bits(v);
    else ((uint16_t*)p)[idx] = double_to_f16_bits(v);
}

void oracle_gate_logits(const void* x, const void* Wg, const float* gate_bias, int32_t T,
                        int32_t H, int32_t E, int32_t dtype, float* logits) {
    ThreadScope ts;
    if (dtype == 0) gate_logits_t<F32>(x, Wg, gate_bias, T, H, E, logits);
    else if (dtype == 1) gate_logits_t<BF16>(x, Wg, gate_bias, T, H, E, logits);
    else gate_logits_t<F16>(x, Wg, gate_bias, T, H, E, logits);
}

void oracle_topk(const float* logits, int32_t T, int32_t E, int32_t k, int32_t* topk_expert,
                 float* topk_weight) {
    std::vector<char> taken(E);
    std::vector<double> ex(k);
    for (int i = 0; i < T; ++i) {
        const float* l = logits + (int64_t)i * E;
        std::fill(taken.begin(), taken.end(), 0);
        // O2: k rounds of "largest remaining logit, smaller index on equal values"
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int e = 0; e < E; ++e) {
                if (taken[e]) continue;
                if (best < 0 || l[e] > l[best]) best = e;     // strict >: earlier index keeps ties
            }
            taken[best] = 1;
            topk_expert[(int64_t)i * k + j] = best;
        }
        // O3: softmax over the k selected logits
        const double m = (double)l[topk_expert[(int64_t)i * k]];
        double sum = 0.0;
        for (int j = 0; j < k; ++j) {
            ex[j] = std::exp((double)l[topk_expert[(int64_t)i * k + j]] - m);
            sum += ex[j];
        }
        for (int j = 0; j < k; ++j) topk_weight[(int64_t)i * k + j] = (float)(ex[j] / sum);
    }
}

void oracle_slots(const int32_t* topk_expert, const float* topk_weight, int32_t T, int32_t E,
                  int32_t k, int32_t C, int32_t* slot, int32_t* expert_demand,
                  int32_t* slot_token, float* slot_weight) {
    std::vector<int32_t> cnt(E, 0);
    if (slot_token) for (int64_t q = 0; q < (int64_t)E * C; ++q) slot_token[q] = -1;
    if (slot_weight) for (int64_t q = 0; q < (int64_t)E * C; ++q) slot_weight[q] = 0.0f;
    for (int i = 0; i < T; ++i) {
        for (int j = 0; j < k; ++j) {
            const int64_t p = (int64_t)i * k + j;
            const int e = topk_expert[p];
            const int s = cnt[e]++;
            if (s < C) {
                if (slot) slot[p] = s;
                if (slot_token) slot_token[(int64_t)e * C + s] = i;
                if (slot_weight) slot_weight[(int64_t)e * C + s] = topk_weight[p];
            } else if (slot) {
                slot[p] = -1;
            }
        }
    }
    if (expert_demand) for (int e = 0; e < E; ++e) expert_demand[e] = cnt[e];
}

void oracle_slots_choice_major(const int32_t* topk_expert, const float* topk_weight, int32_t T,
                               int32_t E, int32_t k, int32_t C, int32_t* slot,
                               int32_t* expert_demand, int32_t* slot_token, float* slot_weight) {
    std::vector<int32_t> cnt(E, 0);
    if (slot_token) for (int64_t q = 0; q < (int64_t)E * C; ++q) slot_token[q] = -1;
    if (slot_weight) for (int64_t q = 0; q < (int64_t)E * C; ++q) slot_weight[q] = 0.0f;
    for (int j = 0; j < k; ++j) {                      // every token's j-th choice before any (j+1)-th choice
        for (int i = 0; i < T; ++i) {
            const int64_t p = (int64_t)i * k + j;
            const int e = topk_expert[p];
            const int s = cnt[e]++;
            if (s < C) {
                if (slot) slot[p] = s;
                if (slot_token) slot_token[(int64_t)e * C + s] = i;
                if (slot_weight) slot_weight[(int64_t)e * C + s] = topk_weight[p];
            } else if (slot) {
                slot[p] = -1;
            }
        }
    }
    if (expert_demand) for (int e = 0; e < E; ++e) expert_demand[e] = cnt[e];
}

void oracle_ffn_rows(const void* x, const void* W1, const void* b1, const void* W2,
                     const void* b2, const int32_t* pair_token, const int32_t* pair_expert,
                     int32_t n, int32_t H, int32_t I, int32_t act, int32_t dtype, double* y) {
    ThreadScope ts;
    if (dtype == 0) ffn_rows_t<F32>(x, W1, b1, W2, b2, pair_token, pair_expert, n, H, I, act, y);
    else if (dtype == 1) ffn_rows_t<BF16>(x, W1, b1, W2, b2, pair_token, pair_expert, n, H, I, act, y);
    else ffn_rows_t<F16>(x, W1, b1, W2, b2, pair_token, pair_expert, n, H, I, act, y);
}

void oracle_ffn_combine(const void* x, const void* W1, const void* b1, const void* W2,
                        const void* b2, const int32_t* topk_expert, const float* topk_weight,
                        const int32_t* slot, int32_t T, int32_t H, int32_t I, int32_t E,
                        int32_t k, int32_t act, int32_t dtype, const int32_t* tokens,
                        int32_t n_tokens, double* out_f64, void* out) {
    (void)E;
    if (!tokens) n_tokens = T;
    // kept pairs of the requested tokens, in (token, choice) order
    std::vector<int32_t> pt, pe;
    for (int q = 0; q < n_tokens; ++q) {
        const int i = tokens ? tokens[q] : q;
        for (int j = 0; j < k; ++j)
            if (slot[(int64_t)i * k + j] >= 0) {
                pt.push_back(i);
                pe.push_back(topk_expert[(int64_t)i * k + j]);
            }
    }
    std::vector<double> y((size_t)pt.size() * H);
    oracle_ffn_rows(x, W1, b1, W2, b2, pt.data(), pe.data(), (int32_t)pt.size(), H, I, act, dtype,
                    y.data());
    // O7: weighted sum in ascending choice order; zero row if every choice was dropped
    std::vector<double> row(H);
    size_t p = 0;
    for (int q = 0; q < n_tokens; ++q) {
        const int i = tokens ? tokens[q] : q;
        std::fill(row.begin(), row.end(), 0.0);
        for (int j = 0; j < k; ++j) {
            if (slot[(int64_t)i * k + j] < 0) continue;
            const double w = (double)topk_weight[(int64_t)i * k + j];
            for (int h = 0; h < H; ++h) row[h] += w * y[p * H + h];
            ++p;
        }
        for (int h = 0; h < H; ++h) {
            if (out_f64) out_f64[(int64_t)q * H + h] = row[h];
            if (out) oracle_store_elem(out, (int64_t)q * H + h, dtype, row[h]);
        }
    }
}

void oracle_backward(const void* x, const void* Wg, const float* gate_bias, const void* W1,
                     const void* b1, const void* W2, const void* b2, const int32_t* topk_expert,
                     const int32_t* slot, const double* dout, int32_t T, int32_t H, int32_t I, int32_t E,
                     int32_t k, int32_t act, int32_t dtype, double* dx, double* dWg, double* dgate_bias,
                     double* dW1, double* db1, double* dW2, double* db2) {
    ThreadScope ts;
    auto zero = [](double* p, int64_t n) { if (p) std::fill(p, p + n, 0.0); };
    zero(dx, (int64_t)T * H); zero(dWg, (int64_t)H * E); zero(dgate_bias, E);
    zero(dW1, (int64_t)E * H * I); zero(db1, (int64_t)E * I); zero(dW2, (int64_t)E * I * H); zero(db2, (int64_t)E * H);
    if (dtype == 0) backward_t<F32>(x, Wg, gate_bias, W1, b1, W2, b2, topk_expert, slot, dout, T, H, I, E, k, act, dx, dWg, dgate_bias, dW1, db1, dW2, db2);
    else if (dtype == 1) backward_t<BF16>(x, Wg, gate_bias, W1, b1, W2, b2, topk_expert, slot, dout, T, H, I, E, k, act, dx, dWg, dgate_bias, dW1, db1, dW2, db2);
    else backward_t<F16>(x, Wg, gate_bias, W1, b1, W2, b2, topk_expert, slot, dout, T, H, I, E, k, act, dx, dWg, dgate_bias, dW1, db1, dW2, db2);
}

double oracle_activation_grad(double v, int32_t act) { return activation_grad(v, act); }

int32_t oracle_forward(const void* x, const void* Wg, const float* gate_bias, const void* W1,
                       const void* b1, const void* W2, const void* b2, int32_t T, int32_t H,
                       int32_t I, int32_t E, int32_t k, float capacity_factor,
                       int32_t capacity_override, int32_t act, int32_t dtype, float* gate_logits,
                       int32_t* topk_expert, float* topk_weight, int32_t* slot,
                       int32_t* expert_demand, int32_t* slot_token, float* slot_weight,
                       double* out_f64, void* out) {
    const int32_t C = oracle_capacity(T, E, k, capacity_factor, capacity_override);
    if (C < 0 || H <= 0 || I <= 0) return -1;
    std::vector<float> logits_own, w_own;
    std::vector<int32_t> te_own, slot_own;
    if (!gate_logits) { logits_own.resize((size_t)T * E); gate_logits = logits_own.data(); }
    if (!topk_expert) { te_own.resize((size_t)T * k); topk_expert = te_own.data(); }
    if (!topk_weight) { w_own.resize((size_t)T * k); topk_weight = w_own.data(); }
    if (!slot) { slot_own.resize((size_t)T * k); slot = slot_own.data(); }
    oracle_gate_logits(x, Wg, gate_bias, T, H, E, dtype, gate_logits);
    oracle_topk(gate_logits, T, E, k, topk_expert, topk_weight);
    oracle_slots(topk_expert, topk_weight, T, E, k, C, slot, expert_demand, slot_token, slot_weight);
    if (out_f64 || out)
        oracle_ffn_combine(x, W1, b1, W2, b2, topk_expert, topk_weight, slot, T, H, I, E, k, act,
                           dtype, nullptr, T, out_f64, out);
    return C;
}

}  // extern "C"
