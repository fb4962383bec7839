// Modular arithmetic on the FP64 vector ALU.
//
// Why floating point: on CDNA the 32-bit integer multiplies a 64-bit Shoup/Barrett
// product needs (about ten per modular multiply) issue at quarter rate, while
// v_fma_f64 issues at full rate.  For moduli p < 2^51 a modular product can be made
// EXACT with six FP64 instructions: the product is split error-free into
// h = RN(a*b) and l = fma(a,b,-h); the quotient estimate q = rint(a * (b/p)) is
// within one unit of the true quotient; fma(-q,p,h) + l then equals a*b - q*p
// exactly because that integer is below 2^53.  Every quantity below is an integer
// held in a double; "exact" means no rounding ever happens on the value path.
//
// Ranges (p < 2^51, so 4p <= 2^53):
//   mulmod_w(y, w)  : |y| <= 2^53, |w| <= p/2 prepared as (w, RN(w/p))
//                     result r = y*w - q*p with |r| <= (1/2 + |y|*2^-53) p  (< 1.5 p)
//   mulmod(a, b)    : |a|,|b| <= p, result |r| <= 1.25 p
//   reduce_balanced : |x| <= 2^53 -> |r| <= p/2 + 1
//   canon           : |x| <= 2^53 -> [0, p)
#pragma once

struct WMulD { double w, wp; };

__device__ __forceinline__ double u2d(unsigned long long x) {  // x < 2^52, exact
    return __longlong_as_double((long long)(x | 0x4330000000000000ull)) - 4503599627370496.0;
}
__device__ __forceinline__ unsigned long long d2u(double d) {  // integer 0 <= d < 2^52
    return (unsigned long long)__double_as_longlong(d + 4503599627370496.0) & 0x000FFFFFFFFFFFFFull;
}

__device__ __forceinline__ double mulmod_w(double y, double w, double wp, double p) {
    double h = y * w;
    double l = fma(y, w, -h);
    double q = rint(y * wp);
    double c = fma(-q, p, h);
    return c + l;
}

__device__ __forceinline__ double mulmod(double a, double b, double p, double pinv) {
    double h = a * b;
    double l = fma(a, b, -h);
    double q = rint(h * pinv);
    double c = fma(-q, p, h);
    return c + l;
}

__device__ __forceinline__ double reduce_balanced(double x, double p, double pinv) {
    return fma(-rint(x * pinv), p, x);
}

__device__ __forceinline__ double canon(double x, double p, double pinv) {
    double r = reduce_balanced(x, p, pinv);
    return r < 0.0 ? r + p : r;
}

// value known to lie in (-p, p)
__device__ __forceinline__ double canon_small(double r, double p) { return r < 0.0 ? r + p : r; }

__device__ __forceinline__ bool is_p51(const P51Mask &m, int t) { return (m.w[t >> 6] >> (t & 63)) & 1ull; }

// Intermediate between the two passes of a transform (never visible outside the library): the balanced-reduced
// value stored as the bits of the double itself.  Saves the canonical form and both integer conversions.
__device__ __forceinline__ unsigned long long mid_store(double x, double p, double pinv) {
    return (unsigned long long)__double_as_longlong(reduce_balanced(x, p, pinv));
}
__device__ __forceinline__ double mid_load(unsigned long long bits) { return __longlong_as_double((long long)bits); }
