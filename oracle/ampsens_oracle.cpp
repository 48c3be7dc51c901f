// ampsens_oracle.cpp -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
//
// Plain, slow, single-threaded CPU statement of what the per-operator loss-MSE
// sensitivity pass computes.  Only tests, the smoke check and the benchmark's
// cpu_baseline leg may call it; the GPU library never links, loads or includes
// anything from this directory, and nothing here includes anything of the GPU
// library.  Floating point: the one multiply that decides an FP8 code is an fp32
// round-to-nearest-even multiply (compile with -ffp-contract=off, SSE2 fp32);
// every sum is fp64 in plain left-to-right order.
//
// What follows the paper and what follows the format standard:
//   * A  = sum_k z_k^2 zdot_k^2 restricted to one operand: the per-sample
//          sensitivity ||z (.) zdot||^2 of Sec. 2.2 (definition of s_l^r).
//   * E  = sum_k zdot_k^2 (z_k - ztilde_k)^2: the first-order Taylor term
//          (ztilde)^T zdot of Sec. 2.2 with the actual rounding error of an FP8
//          cast in place of the uniform-noise model, cross terms dropped under the
//          independence assumption stated with the definition of s_l^r.
//   * alpha_f = 2^(-2 m_f)/12 (Sec. 2.2, noise-variance equation); d = s alpha
//          (per-sample and averaged loss MSE); d_{j,p} additive over a group's
//          layers (last equation of Sec. 2.2).
//   * eq. (ip) of Sec. 2.1: maximise sum of gains subject to sum of loss MSE
//          <= budget with one choice per group -- by exhaustive enumeration, and by
//          a dominance-pruned enumeration for larger instances.
//   * The paper names its FP8 format only by its bit split, four exponent and three mantissa
//          bits (Sec. 3.1), and is
//          silent on the cast itself.  The cast here is the OCP 8-bit floating point
//          definition: E4M3 (bias 7, no infinities, S.1111.111 is NaN, max 448) and
//          E5M2 (bias 15, IEEE-like, max 57344), round to nearest, ties to even,
//          saturating; per-tensor absmax scale, element multiplied by the
//          reciprocal scale.
//
// Pins (tests/ with -m "not gpu"): decode tables against hand-derived codes and
// a library decode; the encoder against brute-force nearest-value search over all
// 65536 bf16 patterns; idempotence / symmetry / monotonicity / half-ulp bound;
// the exact closed form mean(e^2)/ulp^2 = (1 + 2/n^2)/12 on uniform mantissas;
// A against an fp64 library dot product; E against hand-worked tiny cases;
// selection against itertools brute force and the invariances of eq. (ip).
// Parity unpinned by the paper: it prints no worked number for the statistic.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#include <algorithm>
#include <limits>

namespace {

enum { FMT_E4M3 = 0, FMT_E5M2 = 1 };

struct Fmt {
    int ebits, mbits, bias;
    double fmax;
};

inline bool fmt_of(int fmt, Fmt* f) {
    if (fmt == FMT_E4M3) { *f = Fmt{4, 3, 7, 448.0}; return true; }
    if (fmt == FMT_E5M2) { *f = Fmt{5, 2, 15, 57344.0}; return true; }
    return false;
}

// bf16 storage -> the real it denotes (fp32 holds it exactly).
inline float bf16_val(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

// Value of an FP8 code straight from the format definition.
double fp8_value(const Fmt& f, unsigned code) {
    unsigned sign = (code >> 7) & 1u;
    unsigned efield = (code >> f.mbits) & ((1u << f.ebits) - 1u);
    unsigned mant = code & ((1u << f.mbits) - 1u);
    double mag;
    unsigned emax_field = (1u << f.ebits) - 1u;
    if (f.ebits == 4) {
        // E4M3: only exponent-all-ones with mantissa-all-ones is NaN; no infinity.
        if (efield == emax_field && mant == (1u << f.mbits) - 1u)
            return std::numeric_limits<double>::quiet_NaN();
    } else {
        // E5M2: IEEE-like top exponent.
        if (efield == emax_field) {
            if (mant == 0) return sign ? -INFINITY : INFINITY;
            return std::numeric_limits<double>::quiet_NaN();
        }
    }
    if (efield == 0)
        mag = std::ldexp((double)mant, 1 - f.bias - f.mbits);            // subnormal
    else
        mag = std::ldexp((double)((1u << f.mbits) + mant), (int)efield - f.bias - f.mbits);
    return sign ? -mag : mag;
}

// Round a finite fp32 value to the format: clamp to +-max, nearest, ties to the even
// integer multiple of the local quantum (= even mantissa LSB of the code).
unsigned fp8_encode(const Fmt& f, float yf) {
    unsigned sign = std::signbit(yf) ? 0x80u : 0u;
    unsigned nan_code = 0x7Fu;                         // both formats: all ones below sign
    if (std::isnan(yf)) return sign | nan_code;
    double a = std::fabs((double)yf);
    if (a > f.fmax) a = f.fmax;                        // saturate (also +-inf)
    if (a == 0.0) return sign;
    int ex;
    (void)std::frexp(a, &ex);                          // a = frac * 2^ex, frac in [0.5,1)
    int e = ex - 1;                                    // floor(log2 a)
    int emin = 1 - f.bias;
    int eeff = e < emin ? emin : e;
    double k = std::ldexp(a, f.mbits - eeff);          // exact: a / quantum
    double fl = std::floor(k);
    double frac = k - fl;
    uint64_t r = (uint64_t)fl;
    if (frac > 0.5 || (frac == 0.5 && (r & 1u))) r += 1;
    unsigned mag;
    if (e < emin) mag = (unsigned)r;                   // subnormal field; r = 2^m carries to min normal
    else mag = ((unsigned)(eeff + f.bias) << f.mbits) + (unsigned)(r - (1u << f.mbits));
    return sign | mag;
}

struct Layout {
    int64_t n;        // dense: elements per sample (causal == 0)
    int64_t batch, rows, cols;
    int causal;       // 1: per sample [batch, rows, cols], entry (b,i,j) is part of the
                      // operand iff j <= i + (cols - rows); other entries are not read
};

inline int64_t layout_stride(const Layout& L) {
    return L.causal ? L.batch * L.rows * L.cols : L.n;
}

inline int64_t causal_row_len(const Layout& L, int64_t i) {
    int64_t len = i + 1 + (L.cols - L.rows);
    if (len < 0) len = 0;
    if (len > L.cols) len = L.cols;
    return len;
}

// The two sums of one operand over one sample.
void sens_sample(const uint16_t* x, const uint16_t* dx, const Layout& L,
                 float scale, float inv, const Fmt& f, double* E_out, double* A_out) {
    double E = 0.0, A = 0.0;
    auto element = [&](int64_t idx) {
        float xf = bf16_val(x[idx]);
        float gf = bf16_val(dx[idx]);
        float y = xf * inv;                             // the one fp32 multiply
        unsigned code = fp8_encode(f, y);
        double q = fp8_value(f, code);
        double xt = q * (double)scale;                  // exact in fp64
        double e = (double)xf - xt;
        double t = (double)gf * e;
        E += t * t;
        double a = (double)gf * (double)xf;
        A += a * a;
    };
    if (!L.causal) {
        for (int64_t i = 0; i < L.n; ++i) element(i);
    } else {
        for (int64_t b = 0; b < L.batch; ++b)
            for (int64_t i = 0; i < L.rows; ++i) {
                int64_t len = causal_row_len(L, i);
                int64_t base = (b * L.rows + i) * L.cols;
                for (int64_t j = 0; j < len; ++j) element(base + j);
            }
    }
    *E_out = E;
    *A_out = A;
}

}  // namespace

extern "C" {

// ---- formats ---------------------------------------------------------------------------

int orc_fp8_decode_table(int fmt, double* table256) {
    Fmt f;
    if (!fmt_of(fmt, &f)) return 1;
    for (unsigned c = 0; c < 256; ++c) table256[c] = fp8_value(f, c);
    return 0;
}

double orc_fp8_max(int fmt) {
    Fmt f;
    if (!fmt_of(fmt, &f)) return std::numeric_limits<double>::quiet_NaN();
    return f.fmax;
}

int orc_fp8_mantissa_bits(int fmt) {
    Fmt f;
    if (!fmt_of(fmt, &f)) return -1;
    return f.mbits;
}

// Encode fp32 values (no scale applied).
int orc_fp8_encode_f32(int fmt, const float* y, int64_t n, uint8_t* codes) {
    Fmt f;
    if (!fmt_of(fmt, &f)) return 1;
    for (int64_t i = 0; i < n; ++i) codes[i] = (uint8_t)fp8_encode(f, y[i]);
    return 0;
}

void orc_bf16_to_f32(const uint16_t* x, int64_t n, float* out) {
    for (int64_t i = 0; i < n; ++i) out[i] = bf16_val(x[i]);
}

// alpha_f = 2^(-2 m_f) / 12, Sec. 2.2 noise-variance equation.
double orc_alpha(int mantissa_bits) {
    return std::ldexp(1.0, -2 * mantissa_bits) / 12.0;
}

// ---- absmax and scale ------------------------------------------------------------------

// amax over the entries that belong to the operand (all samples), then the two fp32
// divisions.  flags bit 0: a non-finite entry was seen.  amax == 0, or a reciprocal that
// overflows fp32, gives scale = inv = 1.
int orc_absmax_scale(const uint16_t* x, int64_t n, int causal, int64_t batch, int64_t rows,
                     int64_t cols, int fmt, float* amax_out, float* scale_out, float* inv_out,
                     uint32_t* flags_out) {
    Fmt f;
    if (!fmt_of(fmt, &f)) return 1;
    float amax = 0.0f;
    uint32_t flags = 0;
    auto visit = [&](int64_t idx) {
        float v = std::fabs(bf16_val(x[idx]));
        if (!(v <= std::numeric_limits<float>::max())) flags |= 1u;   // inf or NaN
        if (std::isnan(v)) { amax = v; return; }
        if (!std::isnan(amax) && v > amax) amax = v;
    };
    if (!causal) {
        for (int64_t i = 0; i < n; ++i) visit(i);
    } else {
        Layout L{0, batch, rows, cols, 1};
        int64_t per = batch * rows * cols;
        int64_t reps = per ? n / per : 0;
        for (int64_t s = 0; s < reps; ++s)
            for (int64_t b = 0; b < batch; ++b)
                for (int64_t i = 0; i < rows; ++i) {
                    int64_t len = causal_row_len(L, i);
                    int64_t base = s * per + (b * rows + i) * cols;
                    for (int64_t j = 0; j < len; ++j) visit(base + j);
                }
    }
    float fmaxf_ = (float)f.fmax;
    float scale, inv;
    if (amax == 0.0f) {
        scale = 1.0f; inv = 1.0f;
    } else {
        scale = amax / fmaxf_;
        inv = fmaxf_ / amax;
        if (std::isinf(inv)) { scale = 1.0f; inv = 1.0f; }
    }
    *amax_out = amax; *scale_out = scale; *inv_out = inv; *flags_out = flags;
    return 0;
}

// Power-of-two scales (a scale policy the paper leaves open, common for FP8 hardware with
// exponent-only scale factors): the smallest power of two s with amax / s <= FMAX, and inv = 1 / s,
// both exact.  amax == 0, or an inv that is not a finite fp32 number, gives scale = inv = 1.
// amax_bits: bf16 pattern of amax (sign ignored).
int orc_scale_pow2(uint16_t amax_bits, int fmt, float* scale_out, float* inv_out) {
    Fmt f;
    if (!fmt_of(fmt, &f)) return 1;
    double a = std::fabs((double)bf16_val(amax_bits));
    *scale_out = 1.0f;
    *inv_out = 1.0f;
    if (a == 0.0 || !(a <= std::numeric_limits<double>::max())) return 0;
    int k = (int)std::ceil(std::log2(a / f.fmax));
    // log2 in floating point may be off by one ulp at exact powers of two: settle k exactly
    while (std::ldexp(f.fmax, k) < a) ++k;
    while (std::ldexp(f.fmax, k - 1) >= a) --k;
    double s = std::ldexp(1.0, k), inv = std::ldexp(1.0, -k);
    if ((double)(float)inv != inv || std::isinf((float)inv) || (double)(float)s != s || (float)s == 0.0f) return 0;
    *scale_out = (float)s;
    *inv_out = (float)inv;
    return 0;
}

// ---- fake quantisation -----------------------------------------------------------------

int orc_fake_quant_fp8(const uint16_t* x, int64_t n, float scale, float inv, int fmt,
                       uint8_t* codes, float* dequant /* nullable */) {
    Fmt f;
    if (!fmt_of(fmt, &f)) return 1;
    for (int64_t i = 0; i < n; ++i) {
        float xf = bf16_val(x[i]);
        float y = xf * inv;
        unsigned c = fp8_encode(f, y);
        codes[i] = (uint8_t)c;
        if (dequant) {
            float q = (float)fp8_value(f, c);          // exact: <= 4 significant bits
            dequant[i] = q * scale;                     // one fp32 multiply
        }
    }
    return 0;
}

// ---- the statistic ---------------------------------------------------------------------

// One operand: samples are consecutive blocks of x_stride / dx_stride elements
// (x_stride == 0: the same x for every sample, as for a weight).
// out_E[r], out_A[r] for r in [0,R).
int orc_sens_operand(const uint16_t* x, const uint16_t* dx, int R, int64_t x_stride,
                     int64_t dx_stride, int64_t n, int causal, int64_t batch, int64_t rows,
                     int64_t cols, float scale, float inv, int fmt, double* out_E,
                     double* out_A) {
    Fmt f;
    if (!fmt_of(fmt, &f)) return 1;
    Layout L{n, batch, rows, cols, causal};
    for (int r = 0; r < R; ++r)
        sens_sample(x + (int64_t)r * x_stride, dx + (int64_t)r * dx_stride, L, scale, inv, f,
                    &out_E[r], &out_A[r]);
    return 0;
}

// Linear layer: X, Xdot [rows_total, C] with sample r owning rows
// [row_off[r], row_off[r+1]); W [K, C] shared; Wdot [R, K, C].
// out[r][4] = (E_X, A_X, E_W, A_W).
int orc_sens_linear(const uint16_t* x, const uint16_t* dx, const uint16_t* w,
                    const uint16_t* dw, int64_t C, int64_t K, int R, const int64_t* row_off,
                    float x_scale, float x_inv, float w_scale, float w_inv, int fmt,
                    double* out) {
    Fmt f;
    if (!fmt_of(fmt, &f)) return 1;
    for (int r = 0; r < R; ++r) {
        Layout Lx{(row_off[r + 1] - row_off[r]) * C, 0, 0, 0, 0};
        Layout Lw{K * C, 0, 0, 0, 0};
        sens_sample(x + row_off[r] * C, dx + row_off[r] * C, Lx, x_scale, x_inv, f,
                    &out[4 * r + 0], &out[4 * r + 1]);
        sens_sample(w, dw + (int64_t)r * K * C, Lw, w_scale, w_inv, f, &out[4 * r + 2],
                    &out[4 * r + 3]);
    }
    return 0;
}

// BGEMM: both operands carry one block per sample.  out[r][4] = (E_0, A_0, E_1, A_1).
int orc_sens_bgemm(const uint16_t* x0, const uint16_t* dx0, int64_t n0, int causal0,
                   int64_t batch0, int64_t rows0, int64_t cols0, const uint16_t* x1,
                   const uint16_t* dx1, int64_t n1, int causal1, int64_t batch1, int64_t rows1,
                   int64_t cols1, int R, float s0, float i0, float s1, float i1, int fmt,
                   double* out) {
    Fmt f;
    if (!fmt_of(fmt, &f)) return 1;
    Layout L0{n0, batch0, rows0, cols0, causal0};
    Layout L1{n1, batch1, rows1, cols1, causal1};
    int64_t st0 = layout_stride(L0), st1 = layout_stride(L1);
    for (int r = 0; r < R; ++r) {
        sens_sample(x0 + r * st0, dx0 + r * st0, L0, s0, i0, f, &out[4 * r + 0], &out[4 * r + 1]);
        sens_sample(x1 + r * st1, dx1 + r * st1, L1, s1, i1, f, &out[4 * r + 2], &out[4 * r + 3]);
    }
    return 0;
}

// ---- scale per row (finer granularity than the tensor) ----------------------------------
// The paper leaves the scale granularity open (it only mentions that scales exist, Sec. 3.1).
// Per-row scales: the operand is a [n_rows, row_len] array (token x channel activations: one
// scale per token; a weight [K, C]: one scale per output channel) and row i is cast with
// its own scale_i = amax_i / FMAX, inv_i = FMAX / amax_i, the same two fp32 divisions as for a
// whole tensor.  causal: n_rows = (number of matrices) * rows, row_len = cols, and row rho of
// matrix rho / rows owns its first causal_row_len(rho % rows) entries.

int orc_absmax_scale_rows(const uint16_t* x, int64_t n_rows, int64_t row_len, int causal,
                          int64_t rows, int fmt, float* amax_out, float* scale_out,
                          float* inv_out, uint32_t* flags_out) {
    uint32_t flags = 0;
    Layout L{0, 1, rows, row_len, 1};
    for (int64_t rho = 0; rho < n_rows; ++rho) {
        int64_t len = causal ? causal_row_len(L, rho % rows) : row_len;
        uint32_t fl = 0;
        int rc = orc_absmax_scale(x + rho * row_len, len, 0, 0, 0, 0, fmt, &amax_out[rho],
                                  &scale_out[rho], &inv_out[rho], &fl);
        if (rc) return rc;
        flags |= fl;
    }
    *flags_out = flags;
    return 0;
}

// E and A of one sample's block [n_rows, row_len] with one (scale, inv) per row.
int orc_sens_operand_rows(const uint16_t* x, const uint16_t* dx, int64_t n_rows,
                          int64_t row_len, int causal, int64_t rows, const float* scale,
                          const float* inv, int fmt, double* out_E, double* out_A) {
    Fmt f;
    if (!fmt_of(fmt, &f)) return 1;
    Layout L{0, 1, rows, row_len, 1};
    double E = 0.0, A = 0.0;
    for (int64_t rho = 0; rho < n_rows; ++rho) {
        int64_t len = causal ? causal_row_len(L, rho % rows) : row_len;
        for (int64_t j = 0; j < len; ++j) {
            int64_t idx = rho * row_len + j;
            float xf = bf16_val(x[idx]);
            float gf = bf16_val(dx[idx]);
            float y = xf * inv[rho];                        // the one fp32 multiply
            double q = fp8_value(f, fp8_encode(f, y));
            double e = (double)xf - q * (double)scale[rho];
            double t = (double)gf * e;
            E += t * t;
            double a = (double)gf * (double)xf;
            A += a * a;
        }
    }
    *out_E = E;
    *out_A = A;
    return 0;
}

// ---- scale per block of a row (1 x B tiles) -----------------------------------------------
// A finer granularity still, common for FP8 hardware with scale factors per tile: every row of the
// [n_rows, row_len] operand is cut into row_len / B blocks of B consecutive elements and block
// (i, b) is cast with its own scale, derived from the block's absmax by the same arithmetic as for
// a whole tensor.  Outputs are [n_rows][row_len / B] arrays.  B must divide row_len.

int orc_absmax_scale_blocks(const uint16_t* x, int64_t n_rows, int64_t row_len, int64_t B, int fmt,
                            float* amax_out, float* scale_out, float* inv_out, uint32_t* flags_out) {
    if (B <= 0 || row_len % B != 0) return 2;
    const int64_t per_row = row_len / B;
    uint32_t flags = 0;
    for (int64_t i = 0; i < n_rows; ++i)
        for (int64_t b = 0; b < per_row; ++b) {
            uint32_t fl = 0;
            const int64_t o = i * per_row + b;
            int rc = orc_absmax_scale(x + i * row_len + b * B, B, 0, 0, 0, 0, fmt, &amax_out[o], &scale_out[o],
                                      &inv_out[o], &fl);
            if (rc) return rc;
            flags |= fl;
        }
    *flags_out = flags;
    return 0;
}

// E and A of one sample's block [n_rows, row_len] with one (scale, inv) per 1 x B block.
int orc_sens_operand_blocks(const uint16_t* x, const uint16_t* dx, int64_t n_rows, int64_t row_len,
                            int64_t B, const float* scale, const float* inv, int fmt, double* out_E,
                            double* out_A) {
    Fmt f;
    if (!fmt_of(fmt, &f)) return 1;
    if (B <= 0 || row_len % B != 0) return 2;
    const int64_t per_row = row_len / B;
    double E = 0.0, A = 0.0;
    for (int64_t i = 0; i < n_rows; ++i)
        for (int64_t j = 0; j < row_len; ++j) {
            const int64_t idx = i * row_len + j;
            const int64_t blk = i * per_row + j / B;        // the block element (i, j) lies in
            float xf = bf16_val(x[idx]);
            float gf = bf16_val(dx[idx]);
            float y = xf * inv[blk];                        // the one fp32 multiply
            double q = fp8_value(f, fp8_encode(f, y));
            double e = (double)xf - q * (double)scale[blk];
            double t = (double)gf * e;
            E += t * t;
            double a = (double)gf * (double)xf;
            A += a * a;
        }
    *out_E = E;
    *out_A = A;
    return 0;
}

// ---- epilogue (Sec. 2.2) ---------------------------------------------------------------

// s_l = (1/R) sum_r (A_0^r + A_1^r);  returns s_l.
double orc_layer_sensitivity(const double* A0, const double* A1, int R) {
    double s = 0.0;
    for (int r = 0; r < R; ++r) s += A0[r] + A1[r];
    return R > 0 ? s / (double)R : 0.0;
}

// d_{j,p} = sum_l s_{l_{j,l}} alpha_{Q_{j,lp}} for every column p of Q_j, column p
// being the base-F digits of p (layer 0 = least significant digit).
// alpha[F] (alpha of the high-precision format is 0).  d has F^Lj entries.
int orc_group_mse(const double* s, int Lj, const double* alpha, int F, double* d) {
    int64_t ncol = 1;
    for (int l = 0; l < Lj; ++l) ncol *= F;
    for (int64_t p = 0; p < ncol; ++p) {
        int64_t q = p;
        double acc = 0.0;
        for (int l = 0; l < Lj; ++l) {
            int fidx = (int)(q % F);
            q /= F;
            acc += s[l] * alpha[fidx];
        }
        d[p] = acc;
    }
    return 0;
}

// ---- selection, eq. (ip) ---------------------------------------------------------------

// Definition by enumeration of every combination.  Ties: larger gain, then smaller
// total mse, then lexicographically smaller choice vector.  Returns 0, or 6 when no
// combination is feasible.
int orc_select_exhaustive(int J, const int32_t* n_choices, const double* gain,
                          const double* mse, double budget, int32_t* choice,
                          double* total_gain, double* total_mse) {
    std::vector<int64_t> off(J + 1, 0);
    for (int j = 0; j < J; ++j) off[j + 1] = off[j] + n_choices[j];
    std::vector<int32_t> cur(J, 0), best(J, 0);
    bool have = false;
    double bg = 0, bd = 0;
    while (true) {
        double g = 0, d = 0;
        for (int j = 0; j < J; ++j) { g += gain[off[j] + cur[j]]; d += mse[off[j] + cur[j]]; }
        if (d <= budget) {
            bool better = !have || g > bg || (g == bg && d < bd);
            // equal (g, d): lexicographic order is enumeration order with group 0 most
            // significant, arranged below, so the first one found stays.
            if (better) { have = true; bg = g; bd = d; best = cur; }
        }
        int j = J - 1;
        while (j >= 0) {
            if (++cur[j] < n_choices[j]) break;
            cur[j] = 0;
            --j;
        }
        if (j < 0) break;
    }
    if (!have) return 6;
    for (int j = 0; j < J; ++j) choice[j] = best[j];
    *total_gain = bg; *total_mse = bd;
    return 0;
}

// Same optimum for larger instances: enumerate group by group, keeping only partial
// combinations that are feasible and not dominated (another partial with mse <= and
// gain >=).  Exact.  Returns 7 when the kept list would exceed max_states.
int orc_select_pareto(int J, const int32_t* n_choices, const double* gain, const double* mse,
                      double budget, int64_t max_states, int32_t* choice, double* total_gain,
                      double* total_mse) {
    struct St { double d, g; int32_t parent; int32_t pick; };
    std::vector<std::vector<St>> layers(J + 1);
    layers[0].push_back(St{0.0, 0.0, -1, -1});
    int64_t off = 0;
    for (int j = 0; j < J; ++j) {
        std::vector<St> cand;
        for (int32_t s = 0; s < (int32_t)layers[j].size(); ++s)
            for (int32_t p = 0; p < n_choices[j]; ++p) {
                double d = layers[j][s].d + mse[off + p];
                if (d > budget) continue;
                cand.push_back(St{d, layers[j][s].g + gain[off + p], s, p});
            }
        std::sort(cand.begin(), cand.end(), [](const St& a, const St& b) {
            if (a.d != b.d) return a.d < b.d;
            return a.g > b.g;
        });
        double best_g = -INFINITY;
        for (const St& c : cand)
            if (c.g > best_g) { layers[j + 1].push_back(c); best_g = c.g; }
        if ((int64_t)layers[j + 1].size() > max_states) return 7;
        if (layers[j + 1].empty()) return 6;
        off += n_choices[j];
    }
    const std::vector<St>& last = layers[J];
    int32_t bi = 0;
    for (int32_t s = 1; s < (int32_t)last.size(); ++s)
        if (last[s].g > last[bi].g) bi = s;
    *total_gain = last[bi].g; *total_mse = last[bi].d;
    int32_t s = bi;
    for (int j = J; j >= 1; --j) {
        choice[j - 1] = layers[j][s].pick;
        s = layers[j][s].parent;
    }
    return 0;
}

}  // extern "C"
