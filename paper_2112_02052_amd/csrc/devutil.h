// Device-side helpers: 16-byte feature chunks of fp32 / bf16 / fp16 rows unpacked to fp32,
// and fp32 -> storage-type conversion for outputs.
#pragma once
#include <type_traits>

#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "tcgnn.h"

namespace tcg {

template <int DT> struct Elem;  // VEC = elements in one 16-byte chunk
template <> struct Elem<TCG_F32>  { static constexpr int VEC = 4; static constexpr int BYTES = 4; };
template <> struct Elem<TCG_BF16> { static constexpr int VEC = 8; static constexpr int BYTES = 2; };
template <> struct Elem<TCG_F16>  { static constexpr int VEC = 8; static constexpr int BYTES = 2; };

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

__device__ __forceinline__ float f16_bits_to_f32(uint32_t b)
{
    return __half2float(__ushort_as_half((unsigned short)b));
}

// Unpacks one 16-byte chunk into VEC floats (element k of the chunk -> v[k]).
template <int DT>
__device__ __forceinline__ void unpack16(const uint4 &raw, float *v)
{
    if constexpr (DT == TCG_F32) {
        v[0] = __uint_as_float(raw.x);
        v[1] = __uint_as_float(raw.y);
        v[2] = __uint_as_float(raw.z);
        v[3] = __uint_as_float(raw.w);
    } else if constexpr (DT == TCG_BF16) {
        const uint32_t r[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[2 * k] = __uint_as_float(r[k] << 16);
            v[2 * k + 1] = __uint_as_float(r[k] & 0xFFFF0000u);
        }
    } else {
        const uint32_t r[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            v[2 * k] = f16_bits_to_f32(r[k] & 0xFFFFu);
            v[2 * k + 1] = f16_bits_to_f32(r[k] >> 16);
        }
    }
}

// The unit a lane reads from a feature row: PB bytes = VEC elements.  16-byte chunks are the normal case;
// rows whose width, leading dimension or base address rule them out are read in 4-byte units (one fp32
// or two 16-bit elements) or, failing that, element by element.
template <int DT, int PB>
struct Piece {
    static constexpr int BYTES = PB;
    static constexpr int VEC = PB / Elem<DT>::BYTES;
    static_assert(PB == 16 || PB == 4 || PB == Elem<DT>::BYTES, "unsupported piece size");
    // p must be valid and PB-aligned; v receives VEC floats
    static __device__ __forceinline__ void load(const char *p, float *v)
    {
        if constexpr (PB == 16) {
            unpack16<DT>(*reinterpret_cast<const uint4 *>(p), v);
        } else if constexpr (DT == TCG_F32) {
            v[0] = *reinterpret_cast<const float *>(p);
        } else if constexpr (PB == 4) {
            const uint32_t r = *reinterpret_cast<const uint32_t *>(p);
            if constexpr (DT == TCG_BF16) {
                v[0] = __uint_as_float(r << 16);
                v[1] = __uint_as_float(r & 0xFFFF0000u);
            } else {
                v[0] = f16_bits_to_f32(r & 0xFFFFu);
                v[1] = f16_bits_to_f32(r >> 16);
            }
        } else if constexpr (DT == TCG_BF16) {
            v[0] = bf16_bits_to_f32(*reinterpret_cast<const uint16_t *>(p));
        } else {
            v[0] = f16_bits_to_f32(*reinterpret_cast<const uint16_t *>(p));
        }
    }
};

// Largest piece smaller than 16 bytes that rows of `width` elements with leading dimensions ld_a, ld_b
// (elements) at base addresses a, b allow for element size es.
inline int small_piece_bytes(int es, int64_t width, int64_t ld_a, int64_t ld_b, const void *a, const void *b)
{
    if (es == 4) return 4;
    const bool pair = width % 2 == 0 && ld_a % 2 == 0 && ld_b % 2 == 0 &&
                      (reinterpret_cast<uintptr_t>(a) & 3) == 0 && (reinterpret_cast<uintptr_t>(b) & 3) == 0;
    return pair ? 4 : 2;
}

// Scalar element load as fp32.
__device__ __forceinline__ float load_elem(const void *base, int64_t idx, int dt)
{
    if (dt == TCG_F32) return static_cast<const float *>(base)[idx];
    uint32_t b = static_cast<const uint16_t *>(base)[idx];
    return dt == TCG_BF16 ? bf16_bits_to_f32(b) : f16_bits_to_f32(b);
}

// fp32 -> bf16 bits, round to nearest even; NaN stays NaN.
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40u);
    return (uint16_t)((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);
}

__device__ __forceinline__ void store_elem(void *base, int64_t idx, int dt, float v)
{
    if (dt == TCG_F32) static_cast<float *>(base)[idx] = v;
    else if (dt == TCG_BF16) static_cast<uint16_t *>(base)[idx] = f32_to_bf16_bits(v);
    else static_cast<uint16_t *>(base)[idx] = __half_as_ushort(__float2half_rn(v));
}

// Streaming stores for outputs that the kernel never reads back (the result matrix of an SpMM): marked
// non-temporal, they do not claim L2 lines that the gathered neighbour rows would otherwise keep.
__device__ __forceinline__ void stream_store(float *p, float a, float b, float c, float d)
{
    typedef float f32x4_t __attribute__((ext_vector_type(4)));
    const f32x4_t v = {a, b, c, d};
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4_t *>(p));
}
__device__ __forceinline__ void stream_store(uint16_t *p, uint32_t lo, uint32_t hi)
{
    typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
    const u32x2_t v = {lo, hi};
    __builtin_nontemporal_store(v, reinterpret_cast<u32x2_t *>(p));
}

// Four consecutive outputs of a row: one 16-byte (fp32) or 8-byte (16-bit) store when aligned, else scalars.
__device__ __forceinline__ void store4(void *Y, int y_dt, int64_t o, const float4 &v, bool y_vec)
{
    if (y_dt == TCG_F32) {
        float *y = static_cast<float *>(Y) + o;
        if (y_vec) stream_store(y, v.x, v.y, v.z, v.w);
        else { y[0] = v.x; y[1] = v.y; y[2] = v.z; y[3] = v.w; }
    } else {
        uint16_t *y = static_cast<uint16_t *>(Y) + o;
        uint2 pk;
        if (y_dt == TCG_BF16) {
            pk.x = (uint32_t)f32_to_bf16_bits(v.x) | ((uint32_t)f32_to_bf16_bits(v.y) << 16);
            pk.y = (uint32_t)f32_to_bf16_bits(v.z) | ((uint32_t)f32_to_bf16_bits(v.w) << 16);
        } else {
            pk.x = (uint32_t)__half_as_ushort(__float2half_rn(v.x)) | ((uint32_t)__half_as_ushort(__float2half_rn(v.y)) << 16);
            pk.y = (uint32_t)__half_as_ushort(__float2half_rn(v.z)) | ((uint32_t)__half_as_ushort(__float2half_rn(v.w)) << 16);
        }
        if (y_vec) stream_store(y, pk.x, pk.y);
        else { y[0] = (uint16_t)pk.x; y[1] = (uint16_t)(pk.x >> 16); y[2] = (uint16_t)pk.y; y[3] = (uint16_t)(pk.y >> 16); }
    }
}

// Eight consecutive 16-bit outputs of a row as one 16-byte streaming store; p is 16-byte aligned.
__device__ __forceinline__ void store8_16bit(uint16_t *p, int y_dt, const float (&v)[8])
{
    uint32_t w[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (y_dt == TCG_BF16)
            w[i] = (uint32_t)f32_to_bf16_bits(v[2 * i]) | ((uint32_t)f32_to_bf16_bits(v[2 * i + 1]) << 16);
        else
            w[i] = (uint32_t)__half_as_ushort(__float2half_rn(v[2 * i])) |
                   ((uint32_t)__half_as_ushort(__float2half_rn(v[2 * i + 1])) << 16);
    }
    typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
    const u32x4_t q = {w[0], w[1], w[2], w[3]};
    __builtin_nontemporal_store(q, reinterpret_cast<u32x4_t *>(p));
}

// The value that lane SRC of the caller's group of G lanes holds (SRC < G, both known at compile time), in every
// lane of the group.  A group of 16 is a row of the data-parallel primitives, so the broadcast is one vector
// instruction (row_newbcast) instead of a trip through the LDS crossbar (ds_bpermute), whose issue rate the
// gather kernels' sixteen shuffles per step were measured to strain; a group of 8 takes two broadcasts and a
// select.  As with __shfl, the lanes of a group must be active together.
template <int G, int SRC>
__device__ __forceinline__ int32_t group_lane(int32_t v)
{
    static_assert(SRC >= 0 && SRC < G, "source lane outside the group");
    if constexpr (G == 16) {
        return __builtin_amdgcn_update_dpp(0, v, 0x150 + SRC, 0xf, 0xf, false);
    } else if constexpr (G == 8) {
        const int32_t a = __builtin_amdgcn_update_dpp(0, v, 0x150 + SRC, 0xf, 0xf, false);
        const int32_t b = __builtin_amdgcn_update_dpp(0, v, 0x150 + SRC + 8, 0xf, 0xf, false);
        return (threadIdx.x & 8) ? b : a;
    } else {
        return __shfl(v, SRC, G);
    }
}

// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{}): a loop whose counter is a
// compile-time constant inside the body.
template <int N, int I = 0, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<N, I + 1>(f);
    }
}

// The lanes of a group loaded a block of values together, lane l holding elements l, l + G, ... of the block in
// m[0], m[1], ...; out[u] = element S * UNROLL + u, the u-th value of step S of the block.
template <int G, int UNROLL, int PER, int S, int U = 0>
__device__ __forceinline__ void block_ids(const int32_t (&m)[PER], int32_t (&out)[UNROLL])
{
    if constexpr (U < UNROLL) {
        constexpr int Q = S * UNROLL + U;
        out[U] = group_lane<G, Q % G>(m[Q / G]);
        block_ids<G, UNROLL, PER, S, U + 1>(m, out);
    }
}
template <int G, int UNROLL, int PER, int S, int U = 0>
__device__ __forceinline__ void block_ids(const float (&m)[PER], float (&out)[UNROLL])
{
    if constexpr (U < UNROLL) {
        constexpr int Q = S * UNROLL + U;
        out[U] = __int_as_float(group_lane<G, Q % G>(__float_as_int(m[Q / G])));
        block_ids<G, UNROLL, PER, S, U + 1>(m, out);
    }
}

// Sums UNROLL per-lane partials across the G lanes of a group.  On return, lane j (j < UNROLL,
// position inside the group) holds the total of partial j -- if G >= UNROLL; otherwise every
// lane holds all totals in p[].  Must be executed by all lanes of the group.
template <int G, int UNROLL>
__device__ __forceinline__ float group_reduce(float (&p)[UNROLL], int lane)
{
    if constexpr (G >= UNROLL) {
        // Butterfly: at step with distance `off`, a lane keeps the half of its live partials whose
        // index bit matches its own lane bit and receives the partner's copies of that half.
        int live = UNROLL;
#pragma unroll
        for (int off = 1; off < UNROLL; off <<= 1) {
            live >>= 1;
            const bool upper = (lane & off) != 0;
#pragma unroll
            for (int k = 0; k < live; ++k) {
                float keep = upper ? p[2 * k + 1] : p[2 * k];
                float send = upper ? p[2 * k] : p[2 * k + 1];
                p[k] = keep + __shfl_xor(send, off, G);
            }
        }
        float r = p[0];
#pragma unroll
        for (int off = UNROLL; off < G; off <<= 1) r += __shfl_xor(r, off, G);
        return r;
    } else {
#pragma unroll
        for (int k = 0; k < UNROLL; ++k)
#pragma unroll
            for (int off = 1; off < G; off <<= 1) p[k] += __shfl_xor(p[k], off, G);
        return 0.f;
    }
}

}  // namespace tcg
