// Device-side building blocks shared by the kernels of the tree-verification step.
//
// Data layouts (all chosen so that a 64-lane wavefront touches memory in whole,
// contiguous 1 KiB lines and the 32x32 MFMA operands need no shuffles):
//
//  * "vector-major" activations  A[F/E][Tp][E]: E = elements per 16 bytes (8 for bf16,
//    4 for fp32), Tp = token count padded to a multiple of 32.  The E consecutive
//    features of one token are one 16-byte vector, and the vectors of consecutive
//    tokens are adjacent.  This is exactly the B-operand fragment order of the MFMA
//    (lane = token, 16 bytes along the contraction axis).
//  * tiled weights  W[strip][frag][lane][E]: a strip is 32 output rows, a frag is 2E
//    input columns; lane (r = lane%32, g = lane/32) holds W[row(strip, r)][frag*2E + g*E ..].
//    One frag of one strip is 1 KiB and is the A operand of one MFMA step.
//  * MFMA 32x32 accumulator: lane (t = lane%32, g = lane/32), register i holds the
//    output for token t and row m = 8*(i/4) + 4*g + i%4 of the strip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

struct BF16 {};
struct F32 {};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    __bf16 a = (__bf16)lo, b = (__bf16)hi;   // round to nearest even
    return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
}
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) {
    return __builtin_bit_cast(float, (uint32_t)b << 16);
}

// what is left of v after rounding it to bf16: v = hi + lo with hi = bf16(v) exactly representable,
// and lo itself rounded to bf16 carries v to about 16 mantissa bits
__device__ __forceinline__ float bf16_residual(float v) {
    __bf16 h = (__bf16)v;
    return v - bf16_bits_to_f32(__builtin_bit_cast(uint16_t, h));
}

template <typename EL> struct Tr;

template <> struct Tr<BF16> {
    static constexpr int E = 8;     // elements per 16-byte vector
    static constexpr int ESZ = 2;   // bytes per element
    typedef uint16_t elem_t;
    static __device__ __forceinline__ floatx16 mma(const uint4& a, const uint4& b, floatx16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                       __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ float load(const void* p, size_t i) {
        return bf16_bits_to_f32(((const uint16_t*)p)[i]);
    }
    static __device__ __forceinline__ void store(void* p, size_t i, float v) {
        __bf16 h = (__bf16)v;
        ((uint16_t*)p)[i] = __builtin_bit_cast(uint16_t, h);
    }
    // pack E probabilities / values p[0..E) into one operand vector
    static __device__ __forceinline__ uint4 pack(const float* p) {
        uint4 r;
        r.x = pack_bf16x2(p[0], p[1]); r.y = pack_bf16x2(p[2], p[3]);
        r.z = pack_bf16x2(p[4], p[5]); r.w = pack_bf16x2(p[6], p[7]);
        return r;
    }
};

template <> struct Tr<F32> {
    static constexpr int E = 4;
    static constexpr int ESZ = 4;
    typedef float elem_t;
    static __device__ __forceinline__ floatx16 mma(const uint4& a, const uint4& b, floatx16 c) {
        const float4 x = __builtin_bit_cast(float4, a), y = __builtin_bit_cast(float4, b);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(x.x, y.x, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(x.y, y.y, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(x.z, y.z, c, 0, 0, 0);
        c = __builtin_amdgcn_mfma_f32_32x32x2f32(x.w, y.w, c, 0, 0, 0);
        return c;
    }
    static __device__ __forceinline__ float load(const void* p, size_t i) { return ((const float*)p)[i]; }
    static __device__ __forceinline__ void store(void* p, size_t i, float v) { ((float*)p)[i] = v; }
    static __device__ __forceinline__ uint4 pack(const float* p) {
        return __builtin_bit_cast(uint4, make_float4(p[0], p[1], p[2], p[3]));
    }
};

// ---- hand-off of data between workgroups of one launch (partial tiles, attention partials).
// Two things are needed and they are provided separately.  (1) Visibility in hardware: the XCDs'
// L2 caches are not coherent with each other, so the payload is written with write-through
// (agent-scope) stores and read with agent-scope loads, and the producer waits for the stores'
// acknowledgement (vmcnt(0)) before it draws the ticket.  An agent-scope release fence would do
// that too, but by writing back the whole L2, once per workgroup: measured 3x the step time.
// (2) Ordering in the compiler: the payload accesses must not be moved across the ticket
// operation.  These workgroup-scope fences do that (a fence orders all memory operations around
// it, atomic or not); at this scope they cost no cache maintenance, only wait counts.
__device__ __forceinline__ void handoff_release() {
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): stores count in vmcnt on this target
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
}
__device__ __forceinline__ void handoff_acquire() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup"); }

// ---- stores of activations and cache rows (read by later launches: plain stores)
__device__ __forceinline__ void st_u64(void* p, uint64_t v) { *(uint64_t*)p = v; }
__device__ __forceinline__ void st_f32(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_f4(float4* p, float4 v) { *p = v; }
// one cache element (bf16 or fp32)
template <typename EL> __device__ __forceinline__ void st_elem(void* p, size_t i, float v) { Tr<EL>::store(p, i, v); }

// four consecutive cache elements starting at element index i (i % 4 == 0)
template <typename EL> __device__ __forceinline__ void st_cache4(void* p, size_t i, const float (&v)[4]) {
    if constexpr (Tr<EL>::E == 8) {
        st_u64((char*)p + i * 2, (uint64_t)pack_bf16x2(v[0], v[1]) | ((uint64_t)pack_bf16x2(v[2], v[3]) << 32));
    } else {
        st_f4((float4*)((float*)p + i), make_float4(v[0], v[1], v[2], v[3]));
    }
}

// Store four consecutive features f0..f0+3 (f0 % 4 == 0) of token t into a vector-major
// activation buffer.
template <typename EL>
__device__ __forceinline__ void store4_act(void* base, int Tp, int f0, int t, float a, float b, float c, float d) {
    if constexpr (Tr<EL>::E == 8) {
        char* p = (char*)base + ((size_t)(f0 >> 3) * Tp + t) * 16 + (f0 & 7) * 2;
        st_u64(p, (uint64_t)pack_bf16x2(a, b) | ((uint64_t)pack_bf16x2(c, d) << 32));
    } else {
        st_f4((float4*)base + ((size_t)(f0 >> 2) * Tp + t), make_float4(a, b, c, d));
    }
}

// Element index of (position pos, feature f) inside one (layer, kv-head) K slab:
// [pos/32][D/(2E)][32 positions][2E features]; a wavefront reads one (block, frag) tile
// of 1 KiB as the A operand of K*Q^T.
template <typename EL, int D>
__device__ __forceinline__ size_t kcache_index(int pos, int f) {
    constexpr int E = Tr<EL>::E;
    return (((size_t)(pos >> 5) * (D / (2 * E)) + f / (2 * E)) * 32 + (pos & 31)) * (2 * E) + f % (2 * E);
}

// Element index of (pos, feature f) inside one (layer, kv-head) V slab:
// [pos/32][D/32][32/(2E)][32 features][2 lane groups][E positions]; the E positions a lane
// holds are those whose probabilities the same lane owns in the 32x32 accumulator of
// the score tile: accumulator register i <-> position 8*(i/4) + 4*g + i%4 in the block.
template <typename EL, int D>
__device__ __forceinline__ size_t vcache_index(int pos, int f) {
    constexpr int E = Tr<EL>::E;
    constexpr int NQ = 32 / (2 * E);
    const int p = pos & 31;
    const int i = 4 * (p >> 3) + (p & 3);   // accumulator register that owns position p
    const int g = (p >> 2) & 1;             // lane group that owns it
    const int q = i / E, e = i % E;
    return ((((size_t)(pos >> 5) * (D / 32) + (f >> 5)) * NQ + q) * 32 + (f & 31)) * (2 * E) + g * E + e;
}
