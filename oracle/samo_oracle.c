/*
 * CPU oracle for the SAMO compressed-parameter pipeline (Singh & Bhatele,
 * "Exploiting Sparsity in Pruned Neural Networks to Optimize Large Model
 * Training", Section III).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path, and nothing in the product path may call it.  Every
 * function is a single scalar loop in the order the paper states the
 * operation; there is no blocking, fusion, vectorisation or threading.
 *
 * Storage follows Section III-A/III-B: per layer one ascending int32 index of
 * the unpruned positions of the flattened 1-D view, shared by every compressed
 * tensor; fp32 master parameters and optimizer state hold values only at those
 * positions; the fp16 parameters stay dense with explicit zeros.
 *
 * Floating point: state is *stored* in fp32 (Section III, mixed precision);
 * each Adam update is *evaluated* in fp64 from the fp32 inputs and rounded to
 * fp32 once per stored quantity, so the result is the exact update up to one
 * fp32 rounding, independent of operation order or FMA contraction.
 *
 * Parity pins (tests/test_oracle_*.py): the 2x2 worked example of Section
 * III-B; brute force over all masks of tiny layers; the fp16 converters against
 * numpy's casts over every fp32 / fp16 bit pattern; expand = compress^-1
 * (Section III-C); dense Adam on the masked tensor via torch.optim.Adam; the
 * closed form of the first Adam step; Eq. (1)-(5) values printed in Section
 * III-D; for the widened path (tests/test_oracle_next.py) numpy's half addition
 * and direct double->half cast, torch's clip_grad_norm_ and torch.optim.SGD;
 * for single precision (tests/test_oracle_fp32.py) torch.optim.Adam on the dense
 * masked fp32 problem, numpy's fp32 multiply and the expand/compress identity.
 * No function here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <string.h>

static uint32_t bits_of_f32(float x) { uint32_t u; memcpy(&u, &x, 4); return u; }
static float f32_of_bits(uint32_t u) { float x; memcpy(&x, &u, 4); return x; }

/* IEEE 754 binary32 -> binary16, round to nearest, ties to even.  Subnormal
 * halves are produced (never flushed); magnitudes that round past 65504 become
 * infinity; NaN stays a quiet NaN; the sign of a zero result is kept.
 * (Section III-C: "a copy of theta32 in 16-bit" — the paper fixes no rounding
 * mode; round-to-nearest-even is the IEEE default and the reading taken.) */
uint16_t samo_oracle_f32_to_f16(float x)
{
    uint32_t u = bits_of_f32(x);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t bexp = (u >> 23) & 0xffu;
    uint32_t man = u & 0x7fffffu;

    if (bexp == 0xffu)                         /* inf or NaN */
        return (uint16_t)(sign | (man ? 0x7e00u : 0x7c00u));

    int e = (int)bexp - 127;                   /* value = 1.man * 2^e (or subnormal fp32) */
    if (e > 15)
        return (uint16_t)(sign | 0x7c00u);     /* >= 65536: infinity */

    if (e >= -14) {                            /* lands in the normal half range */
        uint32_t h = ((uint32_t)(e + 15) << 10) | (man >> 13);
        uint32_t rem = man & 0x1fffu;          /* 13 discarded bits */
        if (rem > 0x1000u || (rem == 0x1000u && (h & 1u)))
            h += 1;                            /* a carry may reach the exponent, up to inf */
        return (uint16_t)(sign | h);
    }

    if (e < -25)                               /* below half of the smallest subnormal */
        return sign;                           /* (fp32 subnormals and zero land here too) */

    /* subnormal half: result counts units of 2^-24 */
    uint32_t full = man | 0x800000u;           /* 24-bit significand, value = full * 2^(e-23) */
    int shift = -1 - e;                        /* 14 (e = -15) ... 24 (e = -25) */
    uint32_t h = full >> shift;
    uint32_t rem = full & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rem > half || (rem == half && (h & 1u)))
        h += 1;                                /* 1023 -> 1024 is the smallest normal: correct */
    return (uint16_t)(sign | h);
}

/* IEEE 754 binary16 -> binary32; exact for every input. */
float samo_oracle_f16_to_f32(uint16_t h)
{
    uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    uint32_t bexp = (h >> 10) & 0x1fu;
    uint32_t man = h & 0x3ffu;

    if (bexp == 0x1fu)
        return f32_of_bits(sign | 0x7f800000u | (man << 13));
    if (bexp != 0)
        return f32_of_bits(sign | ((bexp + 112u) << 23) | (man << 13));
    if (man == 0)
        return f32_of_bits(sign);
    /* subnormal half = man * 2^-24: normalise */
    int e = -14;
    while (!(man & 0x400u)) { man <<= 1; e -= 1; }
    man &= 0x3ffu;
    return f32_of_bits(sign | ((uint32_t)(e + 127) << 23) | (man << 13));
}

/* IEEE 754 binary64 -> binary16, round to nearest even, directly (one rounding). */
uint16_t samo_oracle_f64_to_f16(double x)
{
    uint64_t u;
    memcpy(&u, &x, 8);
    uint16_t sign = (uint16_t)((u >> 48) & 0x8000u);
    int bexp = (int)((u >> 52) & 0x7ffu);
    uint64_t man = u & 0xfffffffffffffull;

    if (bexp == 0x7ff)
        return (uint16_t)(sign | (man ? 0x7e00u : 0x7c00u));
    int e = bexp - 1023;
    if (e > 15)
        return (uint16_t)(sign | 0x7c00u);
    if (e >= -14) {
        uint32_t h = ((uint32_t)(e + 15) << 10) | (uint32_t)(man >> 42);
        uint64_t rem = man & ((1ull << 42) - 1), half = 1ull << 41;
        if (rem > half || (rem == half && (h & 1u)))
            h += 1;
        return (uint16_t)(sign | h);
    }
    if (e < -25 || bexp == 0)
        return sign;
    uint64_t full = man | (1ull << 52);          /* value = full * 2^(e-52); unit 2^-24 */
    int shift = 28 - e;                          /* 43 (e = -15) ... 53 (e = -25) */
    uint32_t h = (uint32_t)(full >> shift);
    uint64_t rem = full & ((1ull << shift) - 1), half = 1ull << (shift - 1);
    if (rem > half || (rem == half && (h & 1u)))
        h += 1;
    return (uint16_t)(sign | h);
}

void samo_oracle_f32_to_f16_array(const float *x, uint16_t *h, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) h[i] = samo_oracle_f32_to_f16(x[i]);
}

void samo_oracle_f16_to_f32_array(const uint16_t *h, float *x, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) x[i] = samo_oracle_f16_to_f32(h[i]);
}

/* ind_i of Section III: positions of the unpruned parameters of one layer, as
 * offsets into its flattened 1-D view (Section III-B: a 2x2 tensor with
 * non-zeros at (0,0),(1,1) gives [0,3]), in ascending order.  The mask, not the
 * weight value, says what is unpruned.  Returns nnz; idx may be NULL to count. */
int64_t samo_oracle_build_index(const uint8_t *mask, int64_t n, int32_t *idx)
{
    int64_t k = 0;
    for (int64_t j = 0; j < n; ++j) {
        if (mask[j] != 0) {
            if (idx) idx[k] = (int32_t)j;
            k += 1;
        }
    }
    return k;
}

/* "Expansion" (Section III-C, optimizer step): the inverse of compression.
 * The 16-bit copy of theta32 is made value by value and placed at ind; every
 * other position of the dense fp16 buffer is +0 ("zeros explicitly filled in",
 * Section III-C, forward pass), whatever the buffer held before. */
void samo_oracle_decompress(const float *p, const int32_t *idx, int64_t nnz,
                            uint16_t *w, int64_t n)
{
    for (int64_t j = 0; j < n; ++j) w[j] = 0;
    for (int64_t i = 0; i < nnz; ++i) w[idx[i]] = samo_oracle_f32_to_f16(p[i]);
}

/* Compression of the dense fp16 gradient of one layer (Section III-C, backward
 * pass) merged with the up-cast to fp32 (optimizer step, first operation) and
 * the loss-scale division of mixed-precision training: one exact fp16->fp32
 * conversion and one fp32 multiply.  Gradient values at pruned positions are
 * never read. */
void samo_oracle_gather(const uint16_t *g, const int32_t *idx, int64_t nnz,
                        float inv_loss_scale, float *gc)
{
    for (int64_t i = 0; i < nnz; ++i) {
        volatile float t = samo_oracle_f16_to_f32(g[idx[i]]) * inv_loss_scale;
        gc[i] = t;                              /* volatile: a single fp32 rounding, no excess precision */
    }
}

/* Plain compression of an fp16 dense tensor (Section III-B): values at ind. */
void samo_oracle_compress_f16(const uint16_t *dense, const int32_t *idx, int64_t nnz,
                              uint16_t *out)
{
    for (int64_t i = 0; i < nnz; ++i) out[i] = dense[idx[i]];
}

/* Accumulation of one more micro-batch into the stored compressed fp16 gradient (Section III-A
 * keeps grad theta16 compressed; Section II-E: the runtime splits a batch into micro-batches).
 * The paper does not say how micro-batch gradients are combined; the reading taken is an fp16
 * sum, correctly rounded once: the exact sum of two halves fits a double. */
void samo_oracle_accumulate_f16(const uint16_t *g, const int32_t *idx, int64_t nnz, uint16_t *gc16)
{
    for (int64_t i = 0; i < nnz; ++i) {
        const double a = (double)samo_oracle_f16_to_f32(gc16[i]);
        const double b = (double)samo_oracle_f16_to_f32(g[idx[i]]);
        gc16[i] = samo_oracle_f64_to_f16(a + b);
    }
}

/* Optimizer step, first operation (Section III-C): up-cast of the compressed fp16 gradient to
 * fp32 "directly on the compressed tensors", with the loss-scale division: one exact
 * conversion, one fp32 multiply. */
void samo_oracle_upcast(const uint16_t *gc16, int64_t nnz, float inv_loss_scale, float *gc)
{
    for (int64_t i = 0; i < nnz; ++i) {
        volatile float t = samo_oracle_f16_to_f32(gc16[i]) * inv_loss_scale;
        gc[i] = t;
    }
}

/* Sum of squares of a compressed fp32 gradient, in double, in index order; and whether any value
 * is NaN or infinite.  Gradient clipping by global norm (the paper trains with the original
 * authors' hyper-parameters including gradient clipping, Section V) needs the first, mixed
 * precision's overflow check (Micikevicius et al., cited in Section III) the second. */
double samo_oracle_sum_squares(const float *gc, int64_t nnz)
{
    double s = 0.0;
    for (int64_t i = 0; i < nnz; ++i) s += (double)gc[i] * (double)gc[i];
    return s;
}

int32_t samo_oracle_has_nonfinite(const float *gc, int64_t nnz)
{
    for (int64_t i = 0; i < nnz; ++i)
        if (isnan(gc[i]) || isinf(gc[i])) return 1;
    return 0;
}

/* gc[i] *= coef: one fp32 multiply per element (clipping coefficient applied to the gradient). */
void samo_oracle_scale(float *gc, int64_t nnz, float coef)
{
    for (int64_t i = 0; i < nnz; ++i) {
        volatile float t = gc[i] * coef;
        gc[i] = t;
    }
}

/* SGD with momentum on the compressed tensors (one fp32 state per parameter; the paper's CNN
 * runs use SGD, Section V, and Section III-D notes SAMO extends to other optimizers):
 * buf = mu * buf + g (+ weight_decay * p in g); p = p - lr * buf.  buf starts at zero.
 * Evaluated in fp64 from the fp32 state, one rounding per stored value. */
void samo_oracle_sgd(float *p, float *buf, const float *gc, int64_t nnz,
                     float lr, float momentum, float weight_decay)
{
    for (int64_t i = 0; i < nnz; ++i) {
        const double theta = p[i];
        double g = gc[i];
        if (weight_decay != 0.0f) g += (double)weight_decay * theta;
        const double b = (double)momentum * (double)buf[i] + g;
        p[i] = (float)(theta - (double)lr * b);
        buf[i] = (float)b;
    }
}

/* Adam (Kingma & Ba, Algorithm 1; the optimizer assumed in Section III-D, with
 * two fp32 states per parameter) on the compressed tensors (Section III-C,
 * optimizer step, second operation).  t = step >= 1, m0 = v0 = 0, eps is added
 * after the square root of the bias-corrected second moment.  weight_decay is
 * either added to the gradient (L2) or applied decoupled (AdamW, used for the
 * paper's GPT runs, Section V). */
void samo_oracle_adam(float *p, float *m, float *v, const float *gc, int64_t nnz,
                      float lr, float beta1, float beta2, float eps,
                      float weight_decay, int32_t decoupled_wd, int32_t step)
{
    const double b1 = beta1, b2 = beta2;
    const double bc1 = 1.0 - pow(b1, (double)step);
    const double bc2 = 1.0 - pow(b2, (double)step);
    for (int64_t i = 0; i < nnz; ++i) {
        double g = gc[i];
        const double theta = p[i];
        if (weight_decay != 0.0f && !decoupled_wd)
            g += (double)weight_decay * theta;
        const double mn = b1 * (double)m[i] + (1.0 - b1) * g;
        const double vn = b2 * (double)v[i] + (1.0 - b2) * g * g;
        const double mhat = mn / bc1;
        const double vhat = vn / bc2;
        double update = mhat / (sqrt(vhat) + (double)eps);
        if (weight_decay != 0.0f && decoupled_wd)
            update += (double)weight_decay * theta;
        p[i] = (float)(theta - (double)lr * update);
        m[i] = (float)mn;
        v[i] = (float)vn;
    }
}

/* One full SAMO optimizer phase for a layer, in the paper's order (Section
 * III-C): compress + up-cast the gradient, run the optimizer on the compressed
 * state, make the 16-bit copy and expand it.  gc is caller-provided scratch of
 * nnz floats. */
void samo_oracle_step(const uint16_t *g, uint16_t *w, int64_t n,
                      const int32_t *idx, int64_t nnz,
                      float *p, float *m, float *v, float *gc,
                      float inv_loss_scale,
                      float lr, float beta1, float beta2, float eps,
                      float weight_decay, int32_t decoupled_wd, int32_t step)
{
    samo_oracle_gather(g, idx, nnz, inv_loss_scale, gc);
    samo_oracle_adam(p, m, v, gc, nnz, lr, beta1, beta2, eps, weight_decay, decoupled_wd, step);
    samo_oracle_decompress(p, idx, nnz, w, n);
}

/* ---- single-precision SAMO ------------------------------------------------------------------
 * Section III notes that the optimizations also apply to single-precision training.  The paper
 * gives no details; the reading taken: theta32 is the only copy of the parameters and stays dense
 * with explicit zeros (it is what forward and backward use, Section III-C), the dense fp32
 * gradient is compressed at ind, the optimizer state is compressed; there are no 16-bit copies
 * and no loss scale (a gradient factor is kept for clipping).  One optimizer phase in the paper's
 * order: compress the gradient, compress theta32, run the optimizer on the compressed tensors,
 * expand theta32. */

/* values at ind of a dense fp32 tensor, times `factor`: one fp32 multiply (exact for 1.0f) */
void samo_oracle_compress_f32(const float *dense, const int32_t *idx, int64_t nnz, float factor, float *out)
{
    for (int64_t i = 0; i < nnz; ++i) {
        volatile float t = dense[idx[i]] * factor;
        out[i] = t;
    }
}

/* inverse of compression for fp32: +0 everywhere, then the values at ind */
void samo_oracle_expand_f32(const float *c, const int32_t *idx, int64_t nnz, float *dense, int64_t n)
{
    for (int64_t j = 0; j < n; ++j) dense[j] = 0.0f;
    for (int64_t i = 0; i < nnz; ++i) dense[idx[i]] = c[i];
}

/* gc and pc are caller-provided scratch of nnz floats */
void samo_oracle_step_fp32(const float *g32, float *w32, int64_t n,
                           const int32_t *idx, int64_t nnz,
                           float *m, float *v, float *gc, float *pc,
                           float grad_factor,
                           float lr, float beta1, float beta2, float eps,
                           float weight_decay, int32_t decoupled_wd, int32_t step)
{
    samo_oracle_compress_f32(g32, idx, nnz, grad_factor, gc);
    samo_oracle_compress_f32(w32, idx, nnz, 1.0f, pc);
    samo_oracle_adam(pc, m, v, gc, nnz, lr, beta1, beta2, eps, weight_decay, decoupled_wd, step);
    samo_oracle_expand_f32(pc, idx, nnz, w32, n);
}

