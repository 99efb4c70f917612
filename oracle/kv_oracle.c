/*
 * CPU oracle for per-key gradient aggregation fused with the SGD update.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the reference the GPU library is
 * checked against; the product never calls it.  It shares no code with the HIP
 * sources.  It is a plain loop over ranks and elements of one key (the loop
 * over keys lives in the Python wrapper), one scalar at a time, with no
 * blocking, fusion or reordering beyond what the definitions below state.
 *
 * What is computed for every element i of a key (paper: Parallel SGD section,
 * eq. (1), and the KVStore API section):
 *
 *   s     = sum over ranks r = 0..W-1 of g_r[i]      push aggregates all
 *                                                    gradients of one key; the
 *                                                    paper's collective is an
 *                                                    elementwise MPI_SUM of
 *                                                    MPI_FLOAT, i.e. fp32
 *   ghat  = rescale * s                              the aggregate times a
 *                                                    scale factor
 *   t     = ghat + wd * w[i]                         L2 weight decay (extension)
 *   dw    = momentum * m[i] - lr * t                 eq. (1): dw = -eta * g,
 *                                                    extended by momentum
 *   w'[i] = w[i] + dw,  m'[i] = dw                   eq. (1): w_{t+1} = w_t + dw
 *
 * Precision: IEEE binary32 for every operation, one rounding per operation (this
 * file must be compiled with -ffp-contract=off and without fast-math), round to
 * nearest even, subnormals kept.  Half-precision gradients are widened exactly
 * to binary32 before the sum.
 *
 * Order of the sum (the paper leaves it to the MPI library):
 *   KVO_SEQUENTIAL  s = g_0; s = s + g_r for r = 1..W-1.  The first term is g_0
 *                   itself, not 0 + g_0, so that a sum of negative zeros stays -0.
 *   KVO_PAIRWISE    balanced tree in rank order:
 *                   sum(lo, 1) = g_lo,
 *                   sum(lo, n) = sum(lo, h) + sum(lo + h, n - h),
 *                   h = largest power of two strictly below n.
 *
 * Parity pins: tests/test_oracle_pins.py (closed forms, hand-computed cases,
 * exact-sum error bound, order-sensitive cases); tests/test_oracle_mutants.py
 * shows that copies of this file with one planted mistake each fail them.
 * The momentum / weight-decay form is not given by the paper: it is pinned only
 * by those closed forms and by the special case momentum = wd = 0, which is
 * eq. (1) with the averaged gradient.
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>

enum { KVO_SEQUENTIAL = 0, KVO_PAIRWISE = 1 };
enum { KVO_F32 = 0, KVO_F16 = 1 };

#define KVO_MAX_W 4096

/* IEEE binary16 bit pattern -> binary32 value, exact for every input. */
float kvo_half_to_float(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    uint32_t e = (h >> 10) & 0x1Fu;
    uint32_t f = h & 0x3FFu;
    uint32_t bits;
    if (e == 0x1Fu) {                       /* inf / nan: keep payload */
        bits = sign | 0x7F800000u | (f << 13);
    } else if (e != 0) {                    /* normal: rebias 15 -> 127 */
        bits = sign | ((e + 112u) << 23) | (f << 13);
    } else if (f == 0) {                    /* signed zero */
        bits = sign;
    } else {                                /* subnormal: value = f * 2^-24 */
        int shift = 0;
        while ((f & 0x400u) == 0) { f <<= 1; ++shift; }
        f &= 0x3FFu;
        bits = sign | ((uint32_t)(113 - shift) << 23) | (f << 13);
    }
    float out;
    memcpy(&out, &bits, sizeof out);
    return out;
}

/*
 * binary32 value -> IEEE binary16 bit pattern, round to nearest, ties to even; overflow goes to
 * infinity, results below the smallest normal half are subnormal halves.  Used for the fp16
 * replicas of the updated weights (the broadcast phase of the paper's collective, done in half
 * precision as an extension).
 */
uint16_t kvo_float_to_half(float x)
{
    uint32_t bits;
    memcpy(&bits, &x, sizeof bits);
    uint16_t sign = (uint16_t)((bits >> 16) & 0x8000u);
    uint32_t a = bits & 0x7FFFFFFFu;
    if (a > 0x7F800000u) {                         /* nan: keep it a nan */
        uint16_t m = (uint16_t)((a >> 13) & 0x3FFu);
        return (uint16_t)(sign | 0x7C00u | (m ? m : 0x200u));
    }
    if (a >= 0x477FF000u) return (uint16_t)(sign | 0x7C00u);   /* 65520 = max half + half an ulp: rounds up to infinity; so does infinity itself */
    if (a >= 0x38800000u) {                        /* result is a normal half (>= 2^-14) */
        uint32_t e = (a >> 23) - 112u;             /* rebias 127 -> 15 */
        uint32_t q = (e << 10) | ((a >> 13) & 0x3FFu);
        uint32_t rem = a & 0x1FFFu;
        if (rem > 0x1000u || (rem == 0x1000u && (q & 1u))) ++q;   /* a carry runs into the exponent */
        return (uint16_t)(sign | q);
    }
    if (a < 0x33000000u) return sign;              /* below 2^-25: rounds to zero */
    {                                              /* subnormal half: multiples of 2^-24 */
        uint32_t e = a >> 23;                      /* 102 .. 112 */
        uint32_t mant = (a & 0x7FFFFFu) | 0x800000u;
        uint32_t shift = 126u - e;                 /* 24 .. 14 */
        uint32_t q = mant >> shift;
        uint32_t rem = mant & ((1u << shift) - 1u);
        uint32_t half = 1u << (shift - 1u);
        if (rem > half || (rem == half && (q & 1u))) ++q;
        return (uint16_t)(sign | q);
    }
}

/* out[i] = kvo_float_to_half(in[i]) for i in [0, n). */
void kvo_round_to_half(const float* in, int64_t n, uint16_t* out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = kvo_float_to_half(in[i]);
}

static float fold_sequential(const float* v, int W)
{
    float s = v[0];
    for (int r = 1; r < W; ++r) s = s + v[r];
    return s;
}

static float fold_pairwise(const float* v, int lo, int n)
{
    if (n == 1) return v[lo];
    int h = 1;
    while (2 * h < n) h *= 2;               /* largest power of two < n */
    float a = fold_pairwise(v, lo, h);
    float b = fold_pairwise(v, lo + h, n - h);
    return a + b;
}

/* Sum over ranks of element i; grads[r] points at rank r's copy of the key. */
static float reduce_element(const void* const* grads, int dtype, int W, int order, int64_t i)
{
    float v[KVO_MAX_W];
    for (int r = 0; r < W; ++r) {
        if (dtype == KVO_F16) v[r] = kvo_half_to_float(((const uint16_t*)grads[r])[i]);
        else                  v[r] = ((const float*)grads[r])[i];
    }
    return order == KVO_PAIRWISE ? fold_pairwise(v, 0, W) : fold_sequential(v, W);
}

/*
 * Raw aggregation of one key over elements [lo, hi): sum_out[i] = s.
 * Returns 0, or -1 on a bad argument.
 */
int kvo_reduce_key(const void* const* grads, int dtype, int W, int order,
                   int64_t lo, int64_t hi, float* sum_out)
{
    if (!grads || !sum_out || W < 1 || W > KVO_MAX_W || lo < 0 || hi < lo) return -1;
    if (dtype != KVO_F32 && dtype != KVO_F16) return -1;
    if (order != KVO_SEQUENTIAL && order != KVO_PAIRWISE) return -1;
    for (int64_t i = lo; i < hi; ++i) sum_out[i] = reduce_element(grads, dtype, W, order, i);
    return 0;
}

/*
 * One full step of one key over elements [lo, hi): aggregate, scale, update
 * w and m in place.  sum_out may be NULL; if given it receives the raw sum.
 */
int kvo_step_key(const void* const* grads, int dtype, int W, int order,
                 float rescale, float lr, float momentum, float wd,
                 float* w, float* m, float* sum_out, int64_t lo, int64_t hi)
{
    if (!grads || !w || !m || W < 1 || W > KVO_MAX_W || lo < 0 || hi < lo) return -1;
    if (dtype != KVO_F32 && dtype != KVO_F16) return -1;
    if (order != KVO_SEQUENTIAL && order != KVO_PAIRWISE) return -1;
    for (int64_t i = lo; i < hi; ++i) {
        float s = reduce_element(grads, dtype, W, order, i);
        float ghat = rescale * s;
        float wdw = wd * w[i];
        float t = ghat + wdw;
        float mm = momentum * m[i];
        float lt = lr * t;
        float dw = mm - lt;
        float wn = w[i] + dw;
        if (sum_out) sum_out[i] = s;
        m[i] = dw;
        w[i] = wn;
    }
    return 0;
}
