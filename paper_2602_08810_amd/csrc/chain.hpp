// Helpers shared by the scans that cut the time axis into groups chained through global memory
// (the LTI scan, its adjoint, and the scan with caller-supplied coefficients): complex arithmetic on float2,
// uniform-row addressing, and the publish/poll protocol of the chain.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace lrnnx {

__device__ __forceinline__ float2 cmul(float2 a, float2 b) {
    return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
// a^e by repeated squaring, carried in double precision and rounded once.  The powers lambda^len multiply the states
// carried between wavefronts and workgroups; a relative error eps in lambda^len acts like an error eps/len in lambda
// itself, to which a state with memory 1/(1-|lambda|) steps is 1/(1-|lambda|) times as sensitive: squaring in fp32
// (eps of about len * 2^-24) cost an order of magnitude in the accuracy of x and of the gradient with respect to lambda.
__device__ __forceinline__ float2 cpow(float2 a, int64_t e) {
    double ar = a.x, ai = a.y, rr = 1.0, ri = 0.0;
    while (e > 0) {
        if (e & 1) { const double t = rr * ar - ri * ai; ri = rr * ai + ri * ar; rr = t; }
        const double t = ar * ar - ai * ai; ai = 2.0 * ar * ai; ar = t;
        e >>= 1;
    }
    return make_float2((float)rr, (float)ri);
}
__device__ __forceinline__ float2 cfma(float2 a, float2 b, float2 c) {   // a*b + c
    return make_float2(__builtin_fmaf(a.x, b.x, __builtin_fmaf(-a.y, b.y, c.x)),
                       __builtin_fmaf(a.x, b.y, __builtin_fmaf(a.y, b.x, c.y)));
}

constexpr int kSpinLimit = 1 << 22;          // polls before a waiting wavefront gives up
constexpr int kAnchor = 16;                  // every 16th group publishes its true end state

// element of a wave-uniform row at a lane's 32-bit byte offset (scalar base + vector offset addressing)
__device__ __forceinline__ const float2 &at(const float2 *row, unsigned byte_off) {
    return *reinterpret_cast<const float2 *>(reinterpret_cast<const char *>(row) + byte_off);
}
__device__ __forceinline__ float2 &at(float2 *row, unsigned byte_off) {
    return *reinterpret_cast<float2 *>(reinterpret_cast<char *>(row) + byte_off);
}

// A published slot is an 8-byte complex value written by one relaxed atomic store at agent scope; kNotReady
// (all ones, a NaN pattern that arithmetic does not produce from other inputs) marks an empty slot, and a
// value that happens to equal it is stored as the canonical NaN instead.
constexpr unsigned long long kNotReady = ~0ull;
__device__ __forceinline__ void publish(float2 *slot, float2 val) {
    unsigned long long bits = ((unsigned long long)__float_as_uint(val.y) << 32) | __float_as_uint(val.x);
    if (bits == kNotReady) bits = 0x7fc000007fc00000ull;
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(slot), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long peek(const float2 *slot) {
    return __hip_atomic_load(reinterpret_cast<const unsigned long long *>(slot), __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 from_bits(unsigned long long bits) {
    return make_float2(__uint_as_float((unsigned)bits), __uint_as_float((unsigned)(bits >> 32)));
}

}  // namespace lrnnx
