// Device-side building blocks shared by the flat-scan and graph-search kernels
// (gfx950 / CDNA4 only: 64-wide wavefronts, MFMA, LDS).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits.h>
#include <math.h>
#include <utility>

namespace ann {

constexpr int WAVE = 64;

typedef uint32_t u4 __attribute__((ext_vector_type(4)));       // one raw 16-byte chunk
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef __bf16 b8 __attribute__((ext_vector_type(8)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));

// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop the compiler
// cannot decline to unroll, so register arrays indexed by it stay in registers
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f) {
    static_for_impl(static_cast<F &&>(f), std::make_integer_sequence<int, N>{});
}

struct F16 { static constexpr int bytes = 2; };
struct BF16 { static constexpr int bytes = 2; };
struct F32 { static constexpr int bytes = 4; };

// ---- order -------------------------------------------------------------------------------
// (s, id) precedes (s2, id2): larger score first, equal scores by lower id.
__device__ __forceinline__ bool precedes(float s, int id, float s2, int id2) {
    return s > s2 || (s == s2 && id < id2);
}

constexpr int EMPTY_ID = INT_MAX;   // id of an unused list slot (its score is -inf)

// Sorted list of the KP best (score, id) pairs, held in registers (every index
// is a compile-time constant after unrolling).
template <int KP>
struct TopList {
    float s[KP];
    int id[KP];

    __device__ __forceinline__ void init() {
#pragma unroll
        for (int i = 0; i < KP; ++i) { s[i] = -INFINITY; id[i] = EMPTY_ID; }
    }
    // true when (v, vid) would enter the list
    __device__ __forceinline__ bool admits(float v, int vid) const {
        return precedes(v, vid, s[KP - 1], id[KP - 1]);
    }
    // insert (v, vid); a pair that does not precede the last entry is dropped
    __device__ __forceinline__ void insert(float v, int vid) {
#pragma unroll
        for (int i = KP - 1; i > 0; --i) {
            const bool before_prev = precedes(v, vid, s[i - 1], id[i - 1]);
            const bool before_this = precedes(v, vid, s[i], id[i]);
            const float ns = before_prev ? s[i - 1] : (before_this ? v : s[i]);
            const int nid = before_prev ? id[i - 1] : (before_this ? vid : id[i]);
            s[i] = ns;
            id[i] = nid;
        }
        if (precedes(v, vid, s[0], id[0])) { s[0] = v; id[0] = vid; }
    }
    // merge with the list held by lane (lane ^ mask); the two lists must hold
    // different ids (empty slots aside), nothing is de-duplicated
    __device__ __forceinline__ void merge_xor(int mask) {
        float ps[KP];
        int pid[KP];
#pragma unroll
        for (int i = 0; i < KP; ++i) { ps[i] = __shfl_xor(s[i], mask); pid[i] = __shfl_xor(id[i], mask); }
#pragma unroll
        for (int i = 0; i < KP; ++i)
            if (admits(ps[i], pid[i])) insert(ps[i], pid[i]);
    }
};

// ---- selection across lanes ------------------------------------------------------------------
// (score, id) -> 64-bit key whose unsigned order is the list order: larger score first, equal
// scores by lower id.  -0 is folded into +0 so that equal scores compare equal; an empty slot
// (-inf, EMPTY_ID) maps to the smallest key any list entry can have.
__device__ __forceinline__ uint64_t order_key(float s, int id) {
    uint32_t b = __float_as_uint(s + 0.0f);
    b = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    return ((uint64_t)b << 32) | (uint32_t)~id;
}
__device__ __forceinline__ void order_key_decode(uint64_t key, float &s, int &id) {
    uint32_t b = (uint32_t)(key >> 32);
    b = (b & 0x80000000u) ? (b ^ 0x80000000u) : ~b;
    s = __uint_as_float(b);
    id = (int)~(uint32_t)key;
}

// out <- the KP best entries of the sorted lists `in` held by the lanes whose numbers differ
// only in the bits LO <= bit < HI (LO, HI powers of two; HI = 64: up to the whole wave);
// every lane of such a group receives the same result.  KP rounds of "largest head wins and
// is popped": a round costs one max-reduction instead of a full list merge.  An entry held
// by several lanes is taken once.
template <int KP, int LP, int LO, int HI>
__device__ __forceinline__ void group_top(const TopList<LP> &in, TopList<KP> &out) {
    uint64_t key[LP];
#pragma unroll
    for (int i = 0; i < LP; ++i) key[i] = order_key(in.s[i], in.id[i]);
    const uint64_t empty = order_key(-INFINITY, EMPTY_ID);
#pragma unroll
    for (int r = 0; r < KP; ++r) {
        uint64_t m = key[0];
#pragma unroll
        for (int mask = LO; mask < HI; mask <<= 1) {
            const uint32_t lo = __shfl_xor((uint32_t)m, mask), hi = __shfl_xor((uint32_t)(m >> 32), mask);
            const uint64_t o = ((uint64_t)hi << 32) | lo;
            m = o > m ? o : m;
        }
        if (key[0] == m) {
#pragma unroll
            for (int i = 0; i + 1 < LP; ++i) key[i] = key[i + 1];
            key[LP - 1] = empty;
        }
        order_key_decode(m, out.s[r], out.id[r]);
    }
}

// ---- 16-byte chunks -----------------------------------------------------------------------
__device__ __forceinline__ u4 load_chunk(const void *p) { return *reinterpret_cast<const u4 *>(p); }

__device__ __forceinline__ u4 zero_chunk() { u4 z = {0u, 0u, 0u, 0u}; return z; }

// acc + <x, q> over one 16-byte chunk of each operand, fp32 accumulation,
// products formed exactly (16-bit inputs) or by fp32 FMA.
template <class T>
__device__ __forceinline__ float dot_chunk(u4 x, u4 q, float acc);

// 16-bit inputs: v_dot2c_f32_{f16,bf16}, two exact products added to the fp32 accumulator per
// instruction (four instructions per chunk instead of eight conversions and eight FMAs).
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));

template <>
__device__ __forceinline__ float dot_chunk<F16>(u4 x, u4 q, float acc) {
    const h8 a = __builtin_bit_cast(h8, x), b = __builtin_bit_cast(h8, q);
#pragma unroll
    for (int i = 0; i < 4; ++i)
        acc = __builtin_amdgcn_fdot2(h2{a[2 * i], a[2 * i + 1]}, h2{b[2 * i], b[2 * i + 1]}, acc, false);
    return acc;
}

template <>
__device__ __forceinline__ float dot_chunk<BF16>(u4 x, u4 q, float acc) {
    const b8 a = __builtin_bit_cast(b8, x), b = __builtin_bit_cast(b8, q);
#pragma unroll
    for (int i = 0; i < 4; ++i)
        acc = __builtin_amdgcn_fdot2_f32_bf16(bf2{a[2 * i], a[2 * i + 1]}, bf2{b[2 * i], b[2 * i + 1]}, acc, false);
    return acc;
}

template <>
__device__ __forceinline__ float dot_chunk<F32>(u4 x, u4 q, float acc) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc = fmaf(__uint_as_float(x[i]), __uint_as_float(q[i]), acc);
    return acc;
}

// The same with four accumulators, one per 4 bytes of the chunk: four independent chains, for
// callers whose lanes add up many chunks one after the other (a dependent chain of dot
// instructions issues several times slower than independent ones).  The caller adds the four.
template <class T>
__device__ __forceinline__ void dot_chunk4(u4 x, u4 q, f4 &acc);

template <>
__device__ __forceinline__ void dot_chunk4<F16>(u4 x, u4 q, f4 &acc) {
    const h8 a = __builtin_bit_cast(h8, x), b = __builtin_bit_cast(h8, q);
#pragma unroll
    for (int i = 0; i < 4; ++i)
        acc[i] = __builtin_amdgcn_fdot2(h2{a[2 * i], a[2 * i + 1]}, h2{b[2 * i], b[2 * i + 1]}, acc[i], false);
}

template <>
__device__ __forceinline__ void dot_chunk4<BF16>(u4 x, u4 q, f4 &acc) {
    const b8 a = __builtin_bit_cast(b8, x), b = __builtin_bit_cast(b8, q);
#pragma unroll
    for (int i = 0; i < 4; ++i)
        acc[i] = __builtin_amdgcn_fdot2_f32_bf16(bf2{a[2 * i], a[2 * i + 1]}, bf2{b[2 * i], b[2 * i + 1]}, acc[i], false);
}

template <>
__device__ __forceinline__ void dot_chunk4<F32>(u4 x, u4 q, f4 &acc) {
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = fmaf(__uint_as_float(x[i]), __uint_as_float(q[i]), acc[i]);
}

// ---- MFMA ---------------------------------------------------------------------------------
// D[16x16] += A[16x32] * B[32x16].  Lane l supplies A[l % 16][8*(l/16) .. +8) and
// B[8*(l/16) .. +8)[l % 16]; it receives D[4*(l/16) + i][l % 16], i = 0..3.
template <class T>
__device__ __forceinline__ f4 mfma16(u4 a, u4 b, f4 c);

template <>
__device__ __forceinline__ f4 mfma16<F16>(u4 a, u4 b, f4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, b), c, 0, 0, 0);
}
template <>
__device__ __forceinline__ f4 mfma16<BF16>(u4 a, u4 b, f4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(b8, a), __builtin_bit_cast(b8, b), c, 0, 0, 0);
}

// D[32x32] += A[32x16] * B[16x32].  Lane l supplies A[l % 32][8*(l/32) .. +8) and
// B[8*(l/32) .. +8)[l % 32]; it receives D[8*(i/4) + 4*(l/32) + i%4][l % 32], i = 0..15.
template <class T>
__device__ __forceinline__ f16v mfma32(u4 a, u4 b, f16v c);

template <>
__device__ __forceinline__ f16v mfma32<F16>(u4 a, u4 b, f16v c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(h8, a), __builtin_bit_cast(h8, b), c, 0, 0, 0);
}
template <>
__device__ __forceinline__ f16v mfma32<BF16>(u4 a, u4 b, f16v c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(b8, a), __builtin_bit_cast(b8, b), c, 0, 0, 0);
}

// Continuation of an exact search: with a boundary pair per query, only rows that come strictly
// after (s[q], id[q]) in the order are candidates of query q.  Null pointers: no boundary.
struct After {
    const float *s = nullptr;
    const int *id = nullptr;
};
// The score of a row for the selection: unchanged when the row comes after the boundary (or the
// boundary score is NaN: nothing excluded), NaN otherwise, and a NaN score is never listed.
__device__ __forceinline__ float after_boundary(float s, int id, float bs, int bid) {
    const bool keep = bs > s || (bs == s && bid < id) || bs != bs;
    return keep ? s : __builtin_nanf("");
}

// One (score, id) pair as stored in the partial-result workspace.
struct Cand {
    float s;
    int id;
};

}  // namespace ann
