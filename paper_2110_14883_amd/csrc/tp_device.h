// Device-side helpers shared by the gfx950 kernels of libtplinear: vector types, buffer loads,
// bf16 packing, the erf-GeLU arithmetic, the LDS tile layout with its global -> register -> LDS
// staging classes and the tile-order map.  Included by the .hip sources only.
#pragma once
#include <atomic>
#include <tuple>
#include <type_traits>

#include "tp_internal.h"

namespace tpl {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

constexpr int BK = 64;              // K tile (elements): one LDS row = 128 bytes = 8 chunks of 16 B
constexpr int NTHREADS = 512;       // 8 waves
constexpr uint32_t OOB_OFFSET = 0x80000000u;   // >= every num_records we ever set
constexpr uint32_t MAX_RECORDS = 0x80000000u;
constexpr int N_XCD = 8;
enum { EPI_NONE = 0, EPI_BIAS = 1, EPI_BIAS_GELU = 2, EPI_MUL_DGELU = 3 };   // epilogue kinds compiled into the GEMM
constexpr int EPI_BYTES_PER_WAVE = 4096;      // epilogue staging patch: 32 rows x 128 bytes per wave

// Launch through the call that RETURNS the launch's own status: an error some other code left
// behind on this thread is neither reported as ours nor cleared.
template <class... P, class... A>
inline hipError_t launch_kernel(void (*kernel)(P...), dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, A... args) {
    std::tuple<P...> vals{static_cast<P>(args)...};
    void* ptrs[sizeof...(P)];
    size_t i = 0;
    std::apply([&](auto&... v) { ((ptrs[i++] = const_cast<void*>(static_cast<const void*>(&v))), ...); }, vals);
    return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, lds_bytes, stream);
}

// ---------------------------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, int64_t bytes) {
    uint32_t n = bytes > (int64_t)MAX_RECORDS ? MAX_RECORDS : (bytes < 0 ? 0u : (uint32_t)bytes);
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), (short)0, (int)n, 0x00020000);
}

__device__ __forceinline__ u32x4_t buf_load16(__amdgpu_buffer_rsrc_t r, uint32_t voff) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, 0, 0);     // default cache policy: the nt hint measured 23 % slower
}

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xFFFF0000u); }

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {   // a -> low half, RNE
    f32x2_t f = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

// Standard normal cdf and pdf in fp32.  erfc(x) for x >= 0 is taken from the five-term
// rational form of Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7 on erf), which is an erfc
// formula to begin with, so the negative tail of Phi keeps its relative accuracy.
__device__ __forceinline__ void normal_cdf_pdf(float a, float& cdf, float& pdf) {
    const float x = fabsf(a) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    float p = fmaf(t, 1.061405429f, -1.453152027f);
    p = fmaf(t, p, 1.421413741f);
    p = fmaf(t, p, -0.284496736f);
    p = fmaf(t, p, 0.254829592f);
    p *= t;
    const float e = __builtin_amdgcn_exp2f(a * a * -0.72134752044448170f);   // exp(-a^2/2)
    const float tail = 0.5f * p * e;                                           // Phi(-|a|)
    cdf = a < 0.0f ? tail : 1.0f - tail;
    pdf = e * 0.39894228040143268f;
}
__device__ __forceinline__ float gelu_f(float a) {
    float c, d;
    normal_cdf_pdf(a, c, d);
    return a * c;
}
__device__ __forceinline__ float dgelu_f(float a) {
    float c, d;
    normal_cdf_pdf(a, c, d);
    return fmaf(a, d, c);
}

struct Epilogue {
    void* out; int64_t ldo; int out_f32;
    void* pre; int64_t ldp;
    const void* bias; int gelu;
    const void* dg; int64_t lddg;
};

// v = 4 consecutive columns n..n+3 of row m of the accumulated product
__device__ __forceinline__ void epilogue4(const Epilogue& e, float (&v)[4], int m, int n) {
    if (e.bias) {
        const u32x2_t b = *reinterpret_cast<const u32x2_t*>(static_cast<const uint16_t*>(e.bias) + n);
        v[0] += bf16_lo(b[0]); v[1] += bf16_hi(b[0]); v[2] += bf16_lo(b[1]); v[3] += bf16_hi(b[1]);
    }
    if (e.pre) {
        u32x2_t s = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        *reinterpret_cast<u32x2_t*>(static_cast<uint16_t*>(e.pre) + (int64_t)m * e.ldp + n) = s;
    }
    if (e.gelu) {
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = gelu_f(v[i]);
    }
    if (e.dg) {
        const u32x2_t g = *reinterpret_cast<const u32x2_t*>(static_cast<const uint16_t*>(e.dg) + (int64_t)m * e.lddg + n);
        v[0] *= dgelu_f(bf16_lo(g[0])); v[1] *= dgelu_f(bf16_hi(g[0]));
        v[2] *= dgelu_f(bf16_lo(g[1])); v[3] *= dgelu_f(bf16_hi(g[1]));
    }
    if (e.out_f32) {
        f32x4_t s = {v[0], v[1], v[2], v[3]};
        *reinterpret_cast<f32x4_t*>(static_cast<float*>(e.out) + (int64_t)m * e.ldo + n) = s;
    } else {
        u32x2_t s = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
        *reinterpret_cast<u32x2_t*>(static_cast<uint16_t*>(e.out) + (int64_t)m * e.ldo + n) = s;
    }
}

// ---------------------------------------------------------------------------------------------
// LDS layout and global -> register -> LDS staging of one operand tile (R rows of 64 k in LDS)
// ---------------------------------------------------------------------------------------------
// byte offset of row r (128 B), 16-byte chunk c.  The swizzle keeps both the fragment reads (16 consecutive rows, one chunk) and the transposed
// 128-bit writes (rows 8 apart, one chunk) free of bank conflicts
__device__ __forceinline__ uint32_t lds_off(int r, int c) {
    return (uint32_t)(((r << 3) + (c ^ (((r >> 1) & 7) ^ ((r >> 4) & 3)))) << 4);
}

// contraction-contiguous operand staged by 256 threads: chunk c = tg%8 of rows tg/8 + 32 i
template <int R>
struct HalfKC {
    static constexpr int NCH = R / 32;
    u32x4_t reg[NCH];
    __device__ __forceinline__ void load(const uint16_t* ptr, int ld, int rows, int row0, int K, int k0, int tg) {
        const int c = tg & 7, r0 = tg >> 3;
        const uint16_t* base = ptr + (int64_t)row0 * ld + k0;
        const int64_t rem = ((int64_t)(rows - row0 - 1) * ld + (K - k0)) * 2;
        __amdgpu_buffer_rsrc_t rs = make_rsrc(base, rem);
        const bool kok = (k0 + c * 8) < K;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const uint32_t off = (uint32_t)(((r0 + 32 * i) * ld + c * 8) * 2);
            reg[i] = buf_load16(rs, kok ? off : OOB_OFFSET);
        }
    }
    __device__ __forceinline__ void store(char* lds, int tg) const {
        const int c = tg & 7, r0 = tg >> 3;
#pragma unroll
        for (int i = 0; i < NCH; ++i)
            *reinterpret_cast<u32x4_t*>(lds + lds_off(r0 + 32 * i, c)) = reg[i];
    }
};

// operand stored [k][x]: one 8 (k) x 8 (x) block per thread, transposed with byte permutes and
// written as 8 rows of 8 consecutive k (128-bit writes).  R = 256 uses all 256 threads, R = 128 half.
template <int R>
struct HalfXC {
    static constexpr int XB = R / 8;            // x blocks per tile
    u32x4_t reg[8];
    __device__ __forceinline__ void load(const uint16_t* ptr, int ld, int krows, int k0, int X, int x0, int tg) {
        const int x = (tg % XB) * 8, k = (tg / XB) * 8;
        const uint16_t* base = ptr + (int64_t)k0 * ld + x0;
        const int64_t rem = ((int64_t)(krows - k0 - 1) * ld + (X - x0)) * 2;
        __amdgpu_buffer_rsrc_t rs = make_rsrc(base, rem);
        const bool ok = (x0 + x) < X && k < BK;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t off = (uint32_t)(((k + i) * ld + x) * 2);
            reg[i] = buf_load16(rs, ok ? off : OOB_OFFSET);
        }
    }
    __device__ __forceinline__ void store(char* lds, int tg) const {
        const int x = (tg % XB) * 8, k = (tg / XB) * 8;
        if (k >= BK) return;
        const int c = k >> 3;
#pragma unroll
        for (int wd = 0; wd < 4; ++wd) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const uint32_t sel = e ? 0x07060302u : 0x05040100u;
                u32x4_t v = {__builtin_amdgcn_perm(reg[1][wd], reg[0][wd], sel), __builtin_amdgcn_perm(reg[3][wd], reg[2][wd], sel),
                             __builtin_amdgcn_perm(reg[5][wd], reg[4][wd], sel), __builtin_amdgcn_perm(reg[7][wd], reg[6][wd], sel)};
                *reinterpret_cast<u32x4_t*>(lds + lds_off(x + 2 * wd + e, c)) = v;
            }
        }
    }
};

// virtual tile id -> (tile_m, tile_n, split index).  Workgroup b runs on XCD b % 8 and takes ids b,
// b + grid, ... (grid is a multiple of 8 whenever there is more than one round), so ids congruent
// mod 8 stay on one XCD: give every XCD one contiguous range of the grouped tile order.
__device__ __forceinline__ void tile_of_id(const GemmArgs& p, const int lin, int& tm, int& tn, int& z) {
    const int G = p.tiles_m * p.tiles_n;
    const int total = G * p.split_k;
    const int base = total / N_XCD, rem = total % N_XCD;
    const int xcd = lin % N_XCD, local = lin / N_XCD;
    const int v = xcd * base + (xcd < rem ? xcd : rem) + local;
    z = v / G;
    const int pid = v - z * G;
    const int per_group = p.group_m * p.tiles_n;
    const int g = pid / per_group;
    const int first_m = g * p.group_m;
    const int gsz = (p.tiles_m - first_m) < p.group_m ? (p.tiles_m - first_m) : p.group_m;
    const int in_g = pid - g * per_group;
    tm = first_m + in_g % gsz;
    tn = in_g / gsz;
}

}  // namespace tpl
