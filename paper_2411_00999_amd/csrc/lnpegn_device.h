// Device-side helpers for the gfx950 LayerNorm-backward kernels: wave64 reductions on DPP,
// 16-byte row vectors of bf16 / fp32, and fixed-order block reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lnpegn {

constexpr int kWave = 64;

// What a deferred backward call leaves at the start of its workspace for the batched reduction
// (written by the row kernel, read by the reduction kernels).
struct DeferHeader {
    float *dgamma, *dbeta, *pe_gamma_sq, *pe_beta_sq, *big_sq;
    int n_slots, gs, G1, n_ex, ex_gs, accumulate;
};

// ---------------------------------------------------------------------------------------
// Wave64 all-lanes sum on the DPP cross-lane network (no LDS traffic).  The order of the
// additions is fixed, so the result is reproducible.  Every lane of the wave must be active.
// ---------------------------------------------------------------------------------------
template <int kCtrl, int kRowMask>
__device__ __forceinline__ float dpp_take(float v)
{
    // lanes that are masked off, or whose source lane does not exist, receive 0
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, kRowMask, 0xf, false));
}

__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_take<0xB1, 0xf>(v);   // quad_perm [1,0,3,2]
    v += dpp_take<0x4E, 0xf>(v);   // quad_perm [2,3,0,1]
    v += dpp_take<0x141, 0xf>(v);  // row_half_mirror: 8 lanes
    v += dpp_take<0x140, 0xf>(v);  // row_mirror: 16 lanes, every lane holds its row's sum
    v += dpp_take<0x142, 0xa>(v);  // row_bcast15 into rows 1 and 3
    v += dpp_take<0x143, 0xc>(v);  // row_bcast31 into rows 2 and 3: lane 63 holds the total
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

__device__ __forceinline__ void wave_sum2(float &a, float &b)
{
    // two independent chains interleaved for instruction-level parallelism
    a += dpp_take<0xB1, 0xf>(a);
    b += dpp_take<0xB1, 0xf>(b);
    a += dpp_take<0x4E, 0xf>(a);
    b += dpp_take<0x4E, 0xf>(b);
    a += dpp_take<0x141, 0xf>(a);
    b += dpp_take<0x141, 0xf>(b);
    a += dpp_take<0x140, 0xf>(a);
    b += dpp_take<0x140, 0xf>(b);
    a += dpp_take<0x142, 0xa>(a);
    b += dpp_take<0x142, 0xa>(b);
    a += dpp_take<0x143, 0xc>(a);
    b += dpp_take<0x143, 0xc>(b);
    a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a), 63));
    b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, b), 63));
}

__device__ __forceinline__ void wave_sum3(float &a, float &b, float &c)
{
    a += dpp_take<0xB1, 0xf>(a);
    b += dpp_take<0xB1, 0xf>(b);
    c += dpp_take<0xB1, 0xf>(c);
    a += dpp_take<0x4E, 0xf>(a);
    b += dpp_take<0x4E, 0xf>(b);
    c += dpp_take<0x4E, 0xf>(c);
    a += dpp_take<0x141, 0xf>(a);
    b += dpp_take<0x141, 0xf>(b);
    c += dpp_take<0x141, 0xf>(c);
    a += dpp_take<0x140, 0xf>(a);
    b += dpp_take<0x140, 0xf>(b);
    c += dpp_take<0x140, 0xf>(c);
    a += dpp_take<0x142, 0xa>(a);
    b += dpp_take<0x142, 0xa>(b);
    c += dpp_take<0x142, 0xa>(c);
    a += dpp_take<0x143, 0xc>(a);
    b += dpp_take<0x143, 0xc>(b);
    c += dpp_take<0x143, 0xc>(c);
    a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a), 63));
    b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, b), 63));
    c = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, c), 63));
}

__device__ __forceinline__ double wave_sum_f64(double v)
{
    // fp64 is only used in the small finalize kernels: plain shuffles are fine there
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// ---------------------------------------------------------------------------------------
// Row vectors: 16 bytes per lane per access.  dx is written once and never read back here, so
// it is stored with the non-temporal (streaming) hint; measured on MI355X the same hint on the
// loads of x and dy helps narrow rows (one or two waves per row) and hurts wide ones.
// ---------------------------------------------------------------------------------------
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));

struct bf16_t {
    uint16_t bits;
};

// ---------------------------------------------------------------------------------------
// Buffer addressing.  A row is described by a buffer resource (base address, size in bytes); a
// lane whose byte offset lies beyond the size reads zeros and its stores are dropped by the
// hardware, so rows that do not fill every lane need no branch around their memory accesses.
// kAux selects the cache policy of the access: 0 = default (cached, write-back), 1 = sc0,
// 2 = nt (streaming), 16 = sc1, and their sums.
// ---------------------------------------------------------------------------------------
typedef __amdgpu_buffer_rsrc_t rsrc_t;

__device__ __forceinline__ rsrc_t make_rsrc(const void *base, int bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, bytes, 0x00020000);
}

template <int kAux>
__device__ __forceinline__ u32x4_t buffer_load16(rsrc_t r, int byte_offset)
{
    return __builtin_amdgcn_raw_buffer_load_b128(r, byte_offset, 0, kAux);
}

template <int kAux>
__device__ __forceinline__ void buffer_store16(rsrc_t r, int byte_offset, u32x4_t v)
{
    __builtin_amdgcn_raw_buffer_store_b128(v, r, byte_offset, 0, kAux);
}

template <typename T>
struct Vec;

template <>
struct Vec<float> {
    static constexpr int kElems = 4;
    using Raw = float4;
    __device__ static __forceinline__ Raw zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ static __forceinline__ Raw load_stream(const Raw *p)
    {
        const f32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(p));
        return make_float4(t.x, t.y, t.z, t.w);
    }
    __device__ static __forceinline__ void store_stream(Raw *p, const Raw &v)
    {
        const f32x4_t t = {v.x, v.y, v.z, v.w};
        __builtin_nontemporal_store(t, reinterpret_cast<f32x4_t *>(p));
    }
    template <int kAux>
    __device__ static __forceinline__ Raw load_buf(rsrc_t r, int byte_offset)
    {
        const f32x4_t t = __builtin_bit_cast(f32x4_t, buffer_load16<kAux>(r, byte_offset));
        return make_float4(t.x, t.y, t.z, t.w);
    }
    template <int kAux>
    __device__ static __forceinline__ void store_buf(rsrc_t r, int byte_offset, const Raw &v)
    {
        const f32x4_t t = {v.x, v.y, v.z, v.w};
        buffer_store16<kAux>(r, byte_offset, __builtin_bit_cast(u32x4_t, t));
    }
    __device__ static __forceinline__ void unpack(const Raw &r, float (&f)[4])
    {
        f[0] = r.x; f[1] = r.y; f[2] = r.z; f[3] = r.w;
    }
    __device__ static __forceinline__ Raw pack(const float (&f)[4])
    {
        return make_float4(f[0], f[1], f[2], f[3]);
    }
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    // round-to-nearest-even conversion; gfx950 has a packed hardware instruction for it
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float floatx2_t __attribute__((ext_vector_type(2)));
    floatx2_t v = {lo, hi};
    bf16x2_t r = __builtin_convertvector(v, bf16x2_t);
    return __builtin_bit_cast(uint32_t, r);
}

template <>
struct Vec<bf16_t> {
    static constexpr int kElems = 8;
    using Raw = uint4;
    __device__ static __forceinline__ Raw zero() { return make_uint4(0u, 0u, 0u, 0u); }
    __device__ static __forceinline__ Raw load_stream(const Raw *p)
    {
        const u32x4_t t = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
        return make_uint4(t.x, t.y, t.z, t.w);
    }
    __device__ static __forceinline__ void store_stream(Raw *p, const Raw &v)
    {
        const u32x4_t t = {v.x, v.y, v.z, v.w};
        __builtin_nontemporal_store(t, reinterpret_cast<u32x4_t *>(p));
    }
    template <int kAux>
    __device__ static __forceinline__ Raw load_buf(rsrc_t r, int byte_offset)
    {
        const u32x4_t t = buffer_load16<kAux>(r, byte_offset);
        return make_uint4(t.x, t.y, t.z, t.w);
    }
    template <int kAux>
    __device__ static __forceinline__ void store_buf(rsrc_t r, int byte_offset, const Raw &v)
    {
        const u32x4_t t = {v.x, v.y, v.z, v.w};
        buffer_store16<kAux>(r, byte_offset, t);
    }
    __device__ static __forceinline__ void unpack(const Raw &r, float (&f)[8])
    {
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __builtin_bit_cast(float, w[i] << 16);
            f[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xffff0000u);
        }
    }
    __device__ static __forceinline__ Raw pack(const float (&f)[8])
    {
        return make_uint4(pack_bf16x2(f[0], f[1]), pack_bf16x2(f[2], f[3]), pack_bf16x2(f[4], f[5]),
                          pack_bf16x2(f[6], f[7]));
    }
};

// scalar element access for the generic (any D, any alignment) kernels
template <typename T>
__device__ __forceinline__ float load_elem(const void *p, int64_t i);
template <>
__device__ __forceinline__ float load_elem<float>(const void *p, int64_t i)
{
    return static_cast<const float *>(p)[i];
}
template <>
__device__ __forceinline__ float load_elem<bf16_t>(const void *p, int64_t i)
{
    return __builtin_bit_cast(float, static_cast<uint32_t>(static_cast<const uint16_t *>(p)[i]) << 16);
}
template <typename T>
__device__ __forceinline__ void store_elem(void *p, int64_t i, float v);
template <>
__device__ __forceinline__ void store_elem<float>(void *p, int64_t i, float v)
{
    static_cast<float *>(p)[i] = v;
}
template <>
__device__ __forceinline__ void store_elem<bf16_t>(void *p, int64_t i, float v)
{
    static_cast<uint16_t *>(p)[i] = static_cast<uint16_t>(pack_bf16x2(v, 0.f) & 0xffffu);
}

__device__ __forceinline__ float load_gamma(const void *gamma, int gamma_is_f32, int64_t i)
{
    return gamma_is_f32 ? load_elem<float>(gamma, i) : load_elem<bf16_t>(gamma, i);
}

// ---------------------------------------------------------------------------------------
// Block-wide sums in a fixed order (wave sum, then the waves' partials added in wave order).
// `slots` needs one element per wave.  Contains two barriers; all threads must call it.
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ float block_sum(float v, float *slots)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_sum(v);
    if (lane == 0) slots[wave] = v;
    __syncthreads();
    float t = 0.f;
    for (int w = 0; w < nw; ++w) t += slots[w];
    __syncthreads();
    return t;
}

__device__ __forceinline__ double block_sum_f64(double v, double *slots)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = (blockDim.x + 63) >> 6;
    v = wave_sum_f64(v);
    if (lane == 0) slots[wave] = v;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < nw; ++w) t += slots[w];
    __syncthreads();
    return t;
}


// Kernel launch that reports its own status: hipLaunchKernel returns the launch's error, so no
// call here reads (or clears) the thread's last-error state, which may belong to the caller.
template <typename T>
struct launch_identity {
    using type = T;
};
template <typename... KArgs>
inline hipError_t launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t stream,
                         typename launch_identity<KArgs>::type... args)
{
    void *ptrs[] = {const_cast<void *>(static_cast<const void *>(&args))...};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, block, ptrs, lds, stream);
}

}  // namespace lnpegn
