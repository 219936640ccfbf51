// Seeded synthetic inputs on the device: a counter-based generator (Philox-4x32-10, the published algorithm)
// followed by a Box-Muller transform whose logarithm, sine and cosine are short polynomials evaluated with
// additions, multiplications, one division and one square root in double precision -- operations IEEE 754 rounds
// the same way everywhere -- so that the NumPy twin in paper_2504_06323_amd/counter_rng.py produces the same
// bytes on any host.  Built into a library of its own (libmosaic_synth.so): it manufactures input bytes and holds
// nothing of the pruning method.
//
// Element i of stream s of a tensor with seed k: counter (i / 4, s), key k; the four 32-bit outputs of the block
// give two (u1, u2) pairs and each pair two normals, z[4 c + 0 .. 3] = (r1 cos t1, r1 sin t1, r2 cos t2, r2 sin t2).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

constexpr uint32_t kM0 = 0xD2511F53u, kM1 = 0xCD9E8D57u, kW0 = 0x9E3779B9u, kW1 = 0xBB67AE85u;

struct U4 {
    uint32_t x, y, z, w;
};

__device__ __forceinline__ U4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = static_cast<uint64_t>(kM0) * c0, p1 = static_cast<uint64_t>(kM1) * c2;
        const uint32_t n0 = static_cast<uint32_t>(p1 >> 32) ^ c1 ^ k0, n1 = static_cast<uint32_t>(p1);
        const uint32_t n2 = static_cast<uint32_t>(p0 >> 32) ^ c3 ^ k1, n3 = static_cast<uint32_t>(p0);
        c0 = n0;
        c1 = n1;
        c2 = n2;
        c3 = n3;
        k0 += kW0;
        k1 += kW1;
    }
    return {c0, c1, c2, c3};
}

// ln(u) for u = (x + 0.5) / 2^32, x a 32-bit integer: u = m 2^e with m in [sqrt(1/2), sqrt(2)),
// ln m = 2 z (1 + z^2/3 + z^4/5 + ...), z = (m - 1) / (m + 1), |z| < 0.172, eleven terms.
__device__ __forceinline__ double ln_unit(uint32_t x) {
    const double u = (static_cast<double>(x) + 0.5) * (1.0 / 4294967296.0);
    const uint64_t bits = static_cast<uint64_t>(__double_as_longlong(u));
    int e = static_cast<int>((bits >> 52) & 0x7ff) - 1022;                               // u = m 2^e, m in [0.5, 1)
    double m = __longlong_as_double(static_cast<long long>((bits & 0x000fffffffffffffull) | 0x3fe0000000000000ull));
    if (m < 0.70710678118654752440) {
        m = m * 2.0;
        e -= 1;
    }
    const double z = (m - 1.0) / (m + 1.0), z2 = z * z;
    double p = 1.0 / 21.0;
    p = p * z2 + 1.0 / 19.0;
    p = p * z2 + 1.0 / 17.0;
    p = p * z2 + 1.0 / 15.0;
    p = p * z2 + 1.0 / 13.0;
    p = p * z2 + 1.0 / 11.0;
    p = p * z2 + 1.0 / 9.0;
    p = p * z2 + 1.0 / 7.0;
    p = p * z2 + 1.0 / 5.0;
    p = p * z2 + 1.0 / 3.0;
    p = p * z2 + 1.0;
    return static_cast<double>(e) * 0.69314718055994530942 + 2.0 * z * p;
}

// cos and sin of 2 pi x / 2^32: the top two bits pick the quadrant, the rest is an angle in [0, pi/2)
// whose sine and cosine are Taylor polynomials (degrees 23 and 22).
__device__ __forceinline__ void cos_sin_turn(uint32_t x, double &c, double &s) {
    const double a = static_cast<double>(x & 0x3fffffffu) * (1.57079632679489661923 / 1073741824.0), a2 = a * a;
    double ps = -1.0 / 25852016738884976640000.0;  // -1/23!
    ps = ps * a2 + 1.0 / 51090942171709440000.0;   //  1/21!
    ps = ps * a2 - 1.0 / 121645100408832000.0;     // -1/19!
    ps = ps * a2 + 1.0 / 355687428096000.0;        //  1/17!
    ps = ps * a2 - 1.0 / 1307674368000.0;          // -1/15!
    ps = ps * a2 + 1.0 / 6227020800.0;             //  1/13!
    ps = ps * a2 - 1.0 / 39916800.0;               // -1/11!
    ps = ps * a2 + 1.0 / 362880.0;                 //  1/9!
    ps = ps * a2 - 1.0 / 5040.0;                   // -1/7!
    ps = ps * a2 + 1.0 / 120.0;                    //  1/5!
    ps = ps * a2 - 1.0 / 6.0;                      // -1/3!
    ps = ps * a2 + 1.0;
    const double sn = a * ps;
    double pc = 1.0 / 1124000727777607680000.0;    //  1/22!
    pc = pc * a2 - 1.0 / 2432902008176640000.0;    // -1/20!
    pc = pc * a2 + 1.0 / 6402373705728000.0;       //  1/18!
    pc = pc * a2 - 1.0 / 20922789888000.0;         // -1/16!
    pc = pc * a2 + 1.0 / 87178291200.0;            //  1/14!
    pc = pc * a2 - 1.0 / 479001600.0;              // -1/12!
    pc = pc * a2 + 1.0 / 3628800.0;                //  1/10!
    pc = pc * a2 - 1.0 / 40320.0;                  // -1/8!
    pc = pc * a2 + 1.0 / 720.0;                    //  1/6!
    pc = pc * a2 - 1.0 / 24.0;                     // -1/4!
    pc = pc * a2 + 1.0 / 2.0;                      //  1/2!
    const double cs = 1.0 - a2 * pc;
    const uint32_t q = x >> 30;
    c = q == 0 ? cs : q == 1 ? -sn : q == 2 ? -cs : sn;
    s = q == 0 ? sn : q == 1 ? cs : q == 2 ? -sn : -cs;
}

// the four standard normals of counter block `block` of stream `stream`
__device__ __forceinline__ void normal4(uint64_t block, uint32_t stream, uint64_t seed, double (&z)[4]) {
    const U4 r = philox4x32_10(static_cast<uint32_t>(block), static_cast<uint32_t>(block >> 32), stream, 0u,
                               static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32));
    double c, s;
    const double r1 = sqrt(-2.0 * ln_unit(r.x));
    cos_sin_turn(r.y, c, s);
    z[0] = r1 * c;
    z[1] = r1 * s;
    const double r2 = sqrt(-2.0 * ln_unit(r.z));
    cos_sin_turn(r.w, c, s);
    z[2] = r2 * c;
    z[3] = r2 * s;
}

__device__ __forceinline__ uint16_t to_bf16(float f) {  // round to nearest, ties to even (finite values only)
    const uint32_t b = __float_as_uint(f);
    return static_cast<uint16_t>((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
}

// out[r, c] = value(r * cols + c) * col_scale[c]; kind[c] != 0: the value is a Student-t draw with three degrees of
// freedom, z0 / sqrt((z1^2 + z2^2 + z3^2) / 3), its four normals taken from streams stream .. stream + 3 at the
// element's own index; otherwise a standard normal from `stream`.  A thread produces four consecutive elements.
template <bool BF16>
__global__ __launch_bounds__(256) void fill_normal(void *out, int64_t rows, int64_t cols, int64_t ld, uint64_t seed,
                                                   uint32_t stream, const float *__restrict__ col_scale,
                                                   const uint8_t *__restrict__ kind, double scale) {
    const int64_t n = rows * cols;
    const int64_t blocks4 = (n + 3) / 4;
    for (int64_t b = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; b < blocks4;
         b += static_cast<int64_t>(gridDim.x) * 256) {
        double z[4];
        normal4(static_cast<uint64_t>(b), stream, seed, z);
        bool any_t = false;
        if (kind) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t i = 4 * b + j;
                if (i < n && kind[i % cols]) any_t = true;
            }
        }
        double t[4] = {0.0, 0.0, 0.0, 0.0};
        if (any_t) {
            double z1[4], z2[4], z3[4];
            normal4(static_cast<uint64_t>(b), stream + 1, seed, z1);
            normal4(static_cast<uint64_t>(b), stream + 2, seed, z2);
            normal4(static_cast<uint64_t>(b), stream + 3, seed, z3);
#pragma unroll
            for (int j = 0; j < 4; ++j) t[j] = z[j] / sqrt((z1[j] * z1[j] + z2[j] * z2[j] + z3[j] * z3[j]) / 3.0);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t i = 4 * b + j;
            if (i >= n) break;
            const int64_t r = i / cols, c = i - r * cols;
            double v = (kind && kind[c]) ? t[j] : z[j];
            v = v * scale;
            if (col_scale) v = v * static_cast<double>(col_scale[c]);
            const float f = static_cast<float>(v);
            if (BF16)
                static_cast<uint16_t *>(out)[r * ld + c] = to_bf16(f);
            else
                static_cast<float *>(out)[r * ld + c] = f;
        }
    }
}

// out[i] = 32-bit output (i % 4) of counter block i / 4 of `stream` (uniform integers, e.g. for planted zeros)
__global__ __launch_bounds__(256) void fill_bits(uint32_t *out, int64_t n, uint64_t seed, uint32_t stream) {
    const int64_t blocks4 = (n + 3) / 4;
    for (int64_t b = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; b < blocks4;
         b += static_cast<int64_t>(gridDim.x) * 256) {
        const U4 r = philox4x32_10(static_cast<uint32_t>(b), static_cast<uint32_t>(static_cast<uint64_t>(b) >> 32), stream,
                                   0u, static_cast<uint32_t>(seed), static_cast<uint32_t>(seed >> 32));
        const uint32_t v[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (4 * b + j < n) out[4 * b + j] = v[j];
    }
}

}  // namespace

// dtype: 0 float32, 1 bfloat16.  All pointers are device pointers; col_scale and kind may be null.
// Returns 0, or -1 for bad arguments / a refused launch.
extern "C" int synth_fill_normal(void *out, int dtype, int64_t rows, int64_t cols, int64_t ld, uint64_t seed,
                                 uint32_t stream, const float *col_scale, const uint8_t *kind, double scale,
                                 void *hip_stream) {
    if (!out || rows < 0 || cols <= 0 || ld < cols || (dtype != 0 && dtype != 1)) return -1;
    if (rows == 0) return 0;
    const int64_t blocks4 = (rows * cols + 3) / 4;
    int64_t grid = (blocks4 + 255) / 256;
    if (grid > 65536) grid = 65536;
    if (dtype == 1)
        hipLaunchKernelGGL(fill_normal<true>, dim3(static_cast<unsigned>(grid)), dim3(256), 0,
                           static_cast<hipStream_t>(hip_stream), out, rows, cols, ld, seed, stream, col_scale, kind, scale);
    else
        hipLaunchKernelGGL(fill_normal<false>, dim3(static_cast<unsigned>(grid)), dim3(256), 0,
                           static_cast<hipStream_t>(hip_stream), out, rows, cols, ld, seed, stream, col_scale, kind, scale);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}

extern "C" int synth_fill_bits(uint32_t *out, int64_t n, uint64_t seed, uint32_t stream, void *hip_stream) {
    if (!out || n < 0) return -1;
    if (n == 0) return 0;
    int64_t grid = ((n + 3) / 4 + 255) / 256;
    if (grid > 65536) grid = 65536;
    hipLaunchKernelGGL(fill_bits, dim3(static_cast<unsigned>(grid)), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       out, n, seed, stream);
    return hipGetLastError() == hipSuccess ? 0 : -1;
}
