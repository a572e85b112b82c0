// gfx950 (MI355X, CDNA4) kernels for one rank's share of a tensor-parallel linear layer
// (paper Section 2.2, tensor parallelism: the local block products of the 1D / 2D-SUMMA / 2.5D /
// 3D schemes, C = sum_k A_k B_k over the steps, then bias + erf-GeLU; and the two backward
// products).  bf16 operands, fp32 accumulation in MFMA 32x32x16 tiles.
//
// One kernel template serves the three memory forms (NN forward, NT dX, TN dW):
//   * a workgroup of 8 wave64 (2 along M x 4 along N) owns one BM x BN tile of C and keeps it in
//     accumulator registers across ALL steps and all K tiles -- no partial C leaves the chip
//     unless the host asked for a cross-workgroup split of K;
//   * K tiles of 64 are double-buffered in LDS; the next tile is fetched with 128-bit buffer loads
//     (out-of-range chunks read as zero, which is how ragged M / K tails are masked) while the
//     current one feeds the MFMAs;
//   * operands whose contraction index is not contiguous in memory are transposed in registers
//     (byte permutes) on the way into LDS, so the MFMA side always reads 8 consecutive k with one
//     ds_read_b128;  LDS rows are 128 B with the 16-byte chunk index XOR-swizzled by (row/2)%8;
//   * the MFMA is issued with the operands swapped (C^T = B^T A^T) so that each lane ends up with
//     4 consecutive columns of one row of C: bias / GeLU / GeLU' run in registers and the stores
//     are 8- or 16-byte wide;
//   * workgroup ids are spread so that each XCD (own L2) works on a compact patch of tiles.
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

// ---------------------------------------------------------------------------------------------
// small device helpers
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, int64_t bytes) {
    uint32_t n = bytes > (int64_t)MAX_RECORDS ? MAX_RECORDS : (bytes < 0 ? 0u : (uint32_t)bytes);
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), (short)0, (int)n, 0x00020000);
}

__device__ __forceinline__ u32x4_t buf_load16(__amdgpu_buffer_rsrc_t r, uint32_t voff) {
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, 0, 0);
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

// byte offset inside one operand tile in LDS: row r (128 B), 16-byte chunk c, swizzled
__device__ __forceinline__ uint32_t lds_off(int r, int c) {
    return (uint32_t)(((r << 3) + (c ^ ((r >> 1) & 7))) << 4);
}

// ---------------------------------------------------------------------------------------------
// global -> register -> LDS staging of one operand tile (R rows of 64 k each, in LDS)
// ---------------------------------------------------------------------------------------------
// Contraction-contiguous operand: memory [row][k].  Thread t fetches chunk c = t%8 of rows t/8 + 64 i.
template <int R>
struct StageKC {
    static constexpr int NCH = R / 64;
    u32x4_t reg[NCH];

    __device__ __forceinline__ void load(const uint16_t* ptr, int ld, int rows, int row0, int K, int k0, int t) {
        const int c = t & 7, r0 = t >> 3;
        const uint16_t* base = ptr + (int64_t)row0 * ld + k0;
        const int64_t rem = ((int64_t)(rows - row0 - 1) * ld + (K - k0)) * 2;
        __amdgpu_buffer_rsrc_t rs = make_rsrc(base, rem);
        const bool kok = (k0 + c * 8) < K;
#pragma unroll
        for (int i = 0; i < NCH; ++i) {
            const uint32_t off = (uint32_t)(((r0 + 64 * i) * ld + c * 8) * 2);
            reg[i] = buf_load16(rs, kok ? off : OOB_OFFSET);
        }
    }
    __device__ __forceinline__ void store(char* lds, int t) const {
        const int c = t & 7, r0 = t >> 3;
#pragma unroll
        for (int i = 0; i < NCH; ++i)
            *reinterpret_cast<u32x4_t*>(lds + lds_off(r0 + 64 * i, c)) = reg[i];
    }
};

// Operand stored [k][x] (x = the tile's row index in LDS): each thread fetches KR k-rows of 8 x,
// transposes them with byte permutes and writes 8 LDS rows of KR consecutive k.
template <int R>
struct StageXC {
    static constexpr int KR = R / 64;          // 4 (R = 256) or 2 (R = 128)
    static constexpr int XG = R / 64;          // x groups of 64 per tile
    u32x4_t reg[KR];

    __device__ __forceinline__ void load(const uint16_t* ptr, int ld, int krows, int k0, int X, int x0, int t) {
        const int l = t & 63, w = t >> 6;
        const int xg = w % XG, kg = w / XG;
        const int x = xg * 64 + (l & 7) * 8;
        const int k = kg * (8 * KR) + (l >> 3) * KR;
        const uint16_t* base = ptr + (int64_t)k0 * ld + x0;
        const int64_t rem = ((int64_t)(krows - k0 - 1) * ld + (X - x0)) * 2;
        __amdgpu_buffer_rsrc_t rs = make_rsrc(base, rem);
        const bool xok = (x0 + x) < X;
#pragma unroll
        for (int i = 0; i < KR; ++i) {
            const uint32_t off = (uint32_t)(((k + i) * ld + x) * 2);
            reg[i] = buf_load16(rs, xok ? off : OOB_OFFSET);
        }
    }
    __device__ __forceinline__ void store(char* lds, int t) const {
        const int l = t & 63, w = t >> 6;
        const int xg = w % XG, kg = w / XG;
        const int x = xg * 64 + (l & 7) * 8;
        const int k = kg * (8 * KR) + (l >> 3) * KR;       // first k of this thread, 0..63
        const int c = k >> 3;
        const uint32_t boff = (uint32_t)((k & 7) * 2);
#pragma unroll
        for (int wd = 0; wd < 4; ++wd) {
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const uint32_t sel = e ? 0x07060302u : 0x05040100u;
                const int r = x + 2 * wd + e;
                char* dst = lds + lds_off(r, c) + boff;
                if constexpr (KR == 4) {
                    u32x2_t v = {__builtin_amdgcn_perm(reg[1][wd], reg[0][wd], sel),
                                 __builtin_amdgcn_perm(reg[3][wd], reg[2][wd], sel)};
                    *reinterpret_cast<u32x2_t*>(dst) = v;
                } else {
                    *reinterpret_cast<uint32_t*>(dst) = __builtin_amdgcn_perm(reg[1][wd], reg[0][wd], sel);
                }
            }
        }
    }
};

// workgroup id -> (tile_m, tile_n, split index): consecutive hardware ids go to different XCDs, so
// give every XCD one contiguous range of the grouped tile order.
__device__ __forceinline__ void tile_of_block(const GemmArgs& p, int& tm, int& tn, int& z) {
    const int G = p.tiles_m * p.tiles_n;
    const int total = G * p.split_k;
    const int lin = blockIdx.x;
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

// ---------------------------------------------------------------------------------------------
// the GEMM kernel
// ---------------------------------------------------------------------------------------------
template <int BM, int BN, bool A_KC, bool B_KC, int PF, bool PRIO>
__global__ __launch_bounds__(NTHREADS) void tp_gemm_kernel(const GemmArgs p) {
    constexpr int TM = BM / 64;      // 32-row MFMA tiles per wave along M (2 waves along M)
    constexpr int TN = BN / 128;     // 32-col MFMA tiles per wave along N (4 waves along N)
    constexpr int A_BYTES = BM * BK * 2;
    constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int t = threadIdx.x;
    const int l = t & 63, w = t >> 6;
    const int wm = w & 1, wn = w >> 1;

    int tile_m, tile_n, z;
    tile_of_block(p, tile_m, tile_n, z);
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int KT = (p.K + BK - 1) / BK;
    const int T = p.n_steps * KT;
    const int Z = p.split_k;
    const int my_tiles = (T - z + Z - 1) / Z;       // tiles z, z+Z, ... (every step is visited)

    using StageA = typename std::conditional<A_KC, StageKC<BM>, StageXC<BM>>::type;
    using StageB = typename std::conditional<B_KC, StageKC<BN>, StageXC<BN>>::type;
    StageA sa[PF];
    StageB sb[PF];

    auto fetch = [&](int tile, StageA& qa, StageB& qb) {
        const int s = tile / KT;
        const int k0 = (tile - s * KT) * BK;
        const uint16_t* ap = static_cast<const uint16_t*>(p.a[s]);
        const uint16_t* bp = static_cast<const uint16_t*>(p.b[s]);
        if constexpr (A_KC) qa.load(ap, p.lda[s], p.M, m0, p.K, k0, t);
        else                qa.load(ap, p.lda[s], p.K, k0, p.M, m0, t);
        if constexpr (B_KC) qb.load(bp, p.ldb[s], p.N, n0, p.K, k0, t);
        else                qb.load(bp, p.ldb[s], p.K, k0, p.N, n0, t);
    };
    auto stash = [&](int buf, const StageA& qa, const StageB& qb) {
        qa.store(lds + buf * STAGE_BYTES, t);
        qb.store(lds + buf * STAGE_BYTES + A_BYTES, t);
    };

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // per-lane fragment addressing: row inside the wave's slab, k chunk = 2 ks + lane/32
    const int ra = wm * (BM / 2) + (l & 31);
    const int rb = wn * (BN / 4) + (l & 31);
    const int ch = l >> 5;

    auto compute = [&](int cur) {
        const char* la = lds + cur * STAGE_BYTES;
        const char* lb = la + A_BYTES;
        if constexpr (PRIO) __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t fa[TM], fb[TN];
#pragma unroll
            for (int i2 = 0; i2 < TM; ++i2)
                fa[i2] = *reinterpret_cast<const bf16x8_t*>(la + lds_off(ra + 32 * i2, 2 * ks + ch));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const bf16x8_t*>(lb + lds_off(rb + 32 * j, 2 * ks + ch));
#pragma unroll
            for (int i2 = 0; i2 < TM; ++i2)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i2][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i2], acc[i2][j], 0, 0, 0);
        }
        if constexpr (PRIO) __builtin_amdgcn_s_setprio(0);
    };

    if constexpr (PF == 1) {
        // the tile after the current one travels through registers while the current one is multiplied
        fetch(z, sa[0], sb[0]);
        stash(0, sa[0], sb[0]);
        __syncthreads();
        for (int i = 0; i < my_tiles; ++i) {
            const int cur = i & 1;
            const bool more = (i + 1) < my_tiles;
            if (more && (p.dbg == 0 || p.dbg == 3)) fetch(p.dbg == 3 ? z : z + (i + 1) * Z, sa[0], sb[0]);
            compute(cur);
            if (more && p.dbg < 2) stash(cur ^ 1, sa[0], sb[0]);
            __syncthreads();
        }
    } else {
        // two tiles in flight: tile i+1 waits in one register set (fetched an iteration ago) while
        // tile i+2 is being fetched into the other
        fetch(z, sa[0], sb[0]);
        stash(0, sa[0], sb[0]);
        if (my_tiles > 1) fetch(z + Z, sa[0], sb[0]);
        __syncthreads();
        for (int i = 0; i < my_tiles; i += 2) {
            // even iteration: LDS buffer 0 is current, set 0 holds tile i+1, set 1 receives tile i+2
            if (i + 2 < my_tiles) fetch(z + (i + 2) * Z, sa[1], sb[1]);
            compute(0);
            if (i + 1 < my_tiles) stash(1, sa[0], sb[0]);
            __syncthreads();
            if (i + 1 >= my_tiles) break;
            // odd iteration: buffer 1 is current, set 1 holds tile i+2, set 0 receives tile i+3
            if (i + 3 < my_tiles) fetch(z + (i + 3) * Z, sa[0], sb[0]);
            compute(1);
            if (i + 2 < my_tiles) stash(0, sa[1], sb[1]);
            __syncthreads();
        }
    }

    // ------------------------------------------------------------------ epilogue
    // acc[i][j][v]: row m = 32 i + lane%32, columns n = 32 j + 8 (v/4) + 4 (lane/32) + v%4
    if (Z > 1) {
        float* wsz = p.ws + (int64_t)z * p.M * p.N;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = m0 + wm * (BM / 2) + 32 * i + (l & 31);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = n0 + wn * (BN / 4) + 32 * j + 8 * g + 4 * ch;
                    if (m < p.M && n < p.N) {
                        f32x4_t s = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                        *reinterpret_cast<f32x4_t*>(wsz + (int64_t)m * p.N + n) = s;
                    }
                }
        }
        return;
    }
    Epilogue e{p.out, p.ldo, p.out_f32, p.pre, p.ldp, p.bias, p.gelu, p.dg, p.lddg};
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm * (BM / 2) + 32 * i + (l & 31);
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn * (BN / 4) + 32 * j + 8 * g + 4 * ch;
                if (m < p.M && n < p.N) {
                    float v[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                    epilogue4(e, v, m, n);
                }
            }
    }
}

// ---------------------------------------------------------------------------------------------
// Ping-pong variant.  Waves 0-3 ("P", one per SIMD) stage operand A, waves 4-7 ("Q") stage operand
// B, each with 256 threads.  Inside one K tile P multiplies first and refills LDS afterwards, Q
// refills first and multiplies afterwards, so on every SIMD one wave has MFMAs ready while the
// other one is busy with global loads and LDS writes.  One workgroup barrier per K tile.
// ---------------------------------------------------------------------------------------------
// swizzle that keeps both the fragment reads (16 consecutive rows, one chunk) and the transposed
// 128-bit writes (rows 8 apart, one chunk) free of bank conflicts
__device__ __forceinline__ uint32_t lds_off2(int r, int c) {
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
            *reinterpret_cast<u32x4_t*>(lds + lds_off2(r0 + 32 * i, c)) = reg[i];
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
                *reinterpret_cast<u32x4_t*>(lds + lds_off2(x + 2 * wd + e, c)) = v;
            }
        }
    }
};

template <int BM, int BN, bool A_KC, bool B_KC>
__global__ __launch_bounds__(NTHREADS) void tp_gemm_pp_kernel(const GemmArgs p) {
    constexpr int TM = BM / 64;
    constexpr int TN = BN / 128;
    constexpr int A_BYTES = BM * BK * 2;
    constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
    extern __shared__ __attribute__((aligned(16))) char lds[];

    const int t = threadIdx.x;
    const int l = t & 63, w = __builtin_amdgcn_readfirstlane(t >> 6);     // wave index, known uniform
    const int wm = w & 1, wn = ((w >> 1) & 1) | ((w >> 2) << 1);          // P waves: wn in {0,1}; Q waves: wn in {2,3}
    const bool is_p = w < 4;
    const int tg = t & 255;

    int tile_m, tile_n, z;
    tile_of_block(p, tile_m, tile_n, z);
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int KT = (p.K + BK - 1) / BK;
    const int T = p.n_steps * KT;
    const int Z = p.split_k;
    const int my_tiles = (T - z + Z - 1) / Z;

    using StageA = typename std::conditional<A_KC, HalfKC<BM>, HalfXC<BM>>::type;
    using StageB = typename std::conditional<B_KC, HalfKC<BN>, HalfXC<BN>>::type;

    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    const int ra = wm * (BM / 2) + (l & 31);
    const int rb = wn * (BN / 4) + (l & 31);
    const int ch = l >> 5;

    auto compute = [&](int cur) {
        const char* la = lds + cur * STAGE_BYTES;
        const char* lb = la + A_BYTES;
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8_t fa[TM], fb[TN];
#pragma unroll
            for (int i2 = 0; i2 < TM; ++i2)
                fa[i2] = *reinterpret_cast<const bf16x8_t*>(la + lds_off2(ra + 32 * i2, 2 * ks + ch));
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const bf16x8_t*>(lb + lds_off2(rb + 32 * j, 2 * ks + ch));
#pragma unroll
            for (int i2 = 0; i2 < TM; ++i2)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i2][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i2], acc[i2][j], 0, 0, 0);
        }
        __builtin_amdgcn_s_setprio(0);
    };

    if (is_p) {
        StageA sa;
        auto fetch = [&](int tile) {
            const int s = tile / KT;
            const int k0 = (tile - s * KT) * BK;
            const uint16_t* ap = static_cast<const uint16_t*>(p.a[s]);
            if constexpr (A_KC) sa.load(ap, p.lda[s], p.M, m0, p.K, k0, tg);
            else                sa.load(ap, p.lda[s], p.K, k0, p.M, m0, tg);
        };
        fetch(z);
        sa.store(lds, tg);
        if (my_tiles > 1) fetch(z + Z);
        __syncthreads();
        for (int i = 0; i < my_tiles; ++i) {
            const int cur = i & 1;
            compute(cur);
            if (i + 1 < my_tiles && p.dbg != 2) sa.store(lds + (cur ^ 1) * STAGE_BYTES, tg);
            if (i + 2 < my_tiles && (p.dbg == 0 || p.dbg == 3)) fetch(p.dbg == 3 ? z : z + (i + 2) * Z);
            __syncthreads();
        }
    } else {
        StageB sb;
        auto fetch = [&](int tile) {
            const int s = tile / KT;
            const int k0 = (tile - s * KT) * BK;
            const uint16_t* bp = static_cast<const uint16_t*>(p.b[s]);
            if constexpr (B_KC) sb.load(bp, p.ldb[s], p.N, n0, p.K, k0, tg);
            else                sb.load(bp, p.ldb[s], p.K, k0, p.N, n0, tg);
        };
        fetch(z);
        sb.store(lds + A_BYTES, tg);
        if (my_tiles > 1) fetch(z + Z);
        __syncthreads();
        for (int i = 0; i < my_tiles; ++i) {
            const int cur = i & 1;
            if (i + 1 < my_tiles && p.dbg != 2) sb.store(lds + (cur ^ 1) * STAGE_BYTES + A_BYTES, tg);
            if (i + 2 < my_tiles && (p.dbg == 0 || p.dbg == 3)) fetch(p.dbg == 3 ? z : z + (i + 2) * Z);
            compute(cur);
            __syncthreads();
        }
    }

    // ------------------------------------------------------------------ epilogue (as in tp_gemm_kernel)
    if (Z > 1) {
        float* wsz = p.ws + (int64_t)z * p.M * p.N;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = m0 + wm * (BM / 2) + 32 * i + (l & 31);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = n0 + wn * (BN / 4) + 32 * j + 8 * g + 4 * ch;
                    if (m < p.M && n < p.N) {
                        f32x4_t s = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                        *reinterpret_cast<f32x4_t*>(wsz + (int64_t)m * p.N + n) = s;
                    }
                }
        }
        return;
    }
    Epilogue e{p.out, p.ldo, p.out_f32, p.pre, p.ldp, p.bias, p.gelu, p.dg, p.lddg};
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int m = m0 + wm * (BM / 2) + 32 * i + (l & 31);
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn * (BN / 4) + 32 * j + 8 * g + 4 * ch;
                if (m < p.M && n < p.N) {
                    float v[4] = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                    epilogue4(e, v, m, n);
                }
            }
    }
}

// ---------------------------------------------------------------------------------------------
// split-K fix-up: sum the fp32 partials in a fixed order, then the same epilogue
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void tp_reduce_kernel(const ReduceArgs p) {
    const int n4 = p.N >> 2;
    const int64_t total = (int64_t)p.M * n4;
    const int64_t plane = (int64_t)p.M * p.N;
    Epilogue e{p.out, p.ldo, p.out_f32, p.pre, p.ldp, p.bias, p.gelu, p.dg, p.lddg};
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x) {
        const int m = (int)(idx / n4);
        const int n = (int)(idx - (int64_t)m * n4) * 4;
        const float* src = p.ws + (int64_t)m * p.N + n;
        f32x4_t s = *reinterpret_cast<const f32x4_t*>(src);
        for (int zz = 1; zz < p.split_k; ++zz) {
            const f32x4_t q = *reinterpret_cast<const f32x4_t*>(src + zz * plane);
            s[0] += q[0]; s[1] += q[1]; s[2] += q[2]; s[3] += q[3];
        }
        float v[4] = {s[0], s[1], s[2], s[3]};
        epilogue4(e, v, m, n);
    }
}

// ---------------------------------------------------------------------------------------------
// da = bf16(dy * GeLU'(pre)), 8 elements per thread per trip
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void tp_dgelu_kernel(const uint16_t* dy, int64_t ld_dy, const uint16_t* pre,
                                                       int64_t ld_pre, uint16_t* da, int64_t ld_da,
                                                       int64_t rows, int cols8) {
    const int64_t total = rows * cols8;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = idx / cols8;
        const int c = (int)(idx - r * cols8) * 8;
        const u32x4_t g = *reinterpret_cast<const u32x4_t*>(dy + r * ld_dy + c);
        const u32x4_t a = *reinterpret_cast<const u32x4_t*>(pre + r * ld_pre + c);
        u32x4_t o;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            o[i] = pack_bf16(bf16_lo(g[i]) * dgelu_f(bf16_lo(a[i])), bf16_hi(g[i]) * dgelu_f(bf16_hi(a[i])));
        *reinterpret_cast<u32x4_t*>(da + r * ld_da + c) = o;
    }
}

// column sums of a bf16 [rows][cols] block into fp32 [cols]; one workgroup per 64 columns,
// fixed summation order (deterministic)
__global__ __launch_bounds__(256) void tp_colsum_kernel(const uint16_t* da, int64_t ld, int64_t rows, int cols, float* out) {
    __shared__ float part[32][65];
    const int cl = threadIdx.x & 7, rl = threadIdx.x >> 3;        // 8 chunk lanes x 32 row lanes
    const int c = blockIdx.x * 64 + cl * 8;
    float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (c < cols) {
        for (int64_t r = rl; r < rows; r += 32) {
            const u32x4_t v = *reinterpret_cast<const u32x4_t*>(da + r * ld + c);
#pragma unroll
            for (int i = 0; i < 4; ++i) { s[2 * i] += bf16_lo(v[i]); s[2 * i + 1] += bf16_hi(v[i]); }
        }
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) part[rl][cl * 8 + i] = s[i];
    __syncthreads();
    if (threadIdx.x < 64) {
        float tot = 0.0f;
        for (int r = 0; r < 32; ++r) tot += part[r][threadIdx.x];
        const int cc = blockIdx.x * 64 + threadIdx.x;
        if (cc < cols) out[cc] = tot;
    }
}

// ---------------------------------------------------------------------------------------------
// host launchers
// ---------------------------------------------------------------------------------------------
void tile_shape(int tile_id, int* bm, int* bn) {
    switch (tile_id) {
        case TILE_128x256: *bm = 128; *bn = 256; break;
        case TILE_256x128: *bm = 256; *bn = 128; break;
        case TILE_128x128: *bm = 128; *bn = 128; break;
        default:           *bm = 256; *bn = 256; break;
    }
}

template <int BM, int BN, bool A_KC, bool B_KC, int PF, bool PRIO>
static hipError_t launch_one(const GemmArgs& a, hipStream_t stream) {
    constexpr int lds_bytes = 2 * (BM + BN) * BK * 2;
    static bool attr_set = false;           // same value every time: a repeated set is harmless
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&tp_gemm_kernel<BM, BN, A_KC, B_KC, PF, PRIO>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const unsigned grid = (unsigned)(a.tiles_m * a.tiles_n * a.split_k);
    hipLaunchKernelGGL((tp_gemm_kernel<BM, BN, A_KC, B_KC, PF, PRIO>), dim3(grid), dim3(NTHREADS), lds_bytes, stream, a);
    return hipGetLastError();
}

template <int BM, int BN, bool A_KC, bool B_KC>
static hipError_t launch_pp(const GemmArgs& a, hipStream_t stream) {
    constexpr int lds_bytes = 2 * (BM + BN) * BK * 2;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&tp_gemm_pp_kernel<BM, BN, A_KC, B_KC>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const unsigned grid = (unsigned)(a.tiles_m * a.tiles_n * a.split_k);
    hipLaunchKernelGGL((tp_gemm_pp_kernel<BM, BN, A_KC, B_KC>), dim3(grid), dim3(NTHREADS), lds_bytes, stream, a);
    return hipGetLastError();
}

template <bool A_KC, bool B_KC>
static hipError_t launch_form(int tile_id, const GemmArgs& a, hipStream_t s) {
    if (a.variant == 0) {
        switch (tile_id) {
            case TILE_256x256: return launch_pp<256, 256, A_KC, B_KC>(a, s);
            case TILE_128x256: return launch_pp<128, 256, A_KC, B_KC>(a, s);
            case TILE_256x128: return launch_pp<256, 128, A_KC, B_KC>(a, s);
            case TILE_128x128: return launch_pp<128, 128, A_KC, B_KC>(a, s);
            default: return hipErrorInvalidValue;
        }
    }
    switch (tile_id) {
        case TILE_256x256:
            switch (a.variant) {
                case 2: return launch_one<256, 256, A_KC, B_KC, 1, true>(a, s);
                default: return launch_one<256, 256, A_KC, B_KC, 1, false>(a, s);
            }
        case TILE_128x256: return launch_one<128, 256, A_KC, B_KC, 1, false>(a, s);
        case TILE_256x128: return launch_one<256, 128, A_KC, B_KC, 1, false>(a, s);
        case TILE_128x128: return launch_one<128, 128, A_KC, B_KC, 1, false>(a, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_gemm(int form, int tile_id, const GemmArgs& a, hipStream_t s) {
    switch (form) {
        case FORM_NN: return launch_form<true, false>(tile_id, a, s);
        case FORM_NT: return launch_form<true, true>(tile_id, a, s);
        case FORM_TN: return launch_form<false, false>(tile_id, a, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_reduce(const ReduceArgs& a, hipStream_t s) {
    const int64_t total = (int64_t)a.M * (a.N >> 2);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(tp_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_dgelu(const void* dy, int64_t ld_dy, const void* pre, int64_t ld_pre, void* da, int64_t ld_da,
                        int64_t rows, int64_t cols, hipStream_t s) {
    const int64_t total = rows * (cols >> 3);
    if (total == 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(tp_dgelu_kernel, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const uint16_t*>(dy), ld_dy,
                       static_cast<const uint16_t*>(pre), ld_pre, static_cast<uint16_t*>(da), ld_da, rows,
                       (int)(cols >> 3));
    return hipGetLastError();
}

hipError_t launch_colsum(const void* da, int64_t ld, int64_t rows, int64_t cols, float* out, hipStream_t s) {
    const unsigned blocks = (unsigned)((cols + 63) / 64);
    hipLaunchKernelGGL(tp_colsum_kernel, dim3(blocks), dim3(256), 0, s, static_cast<const uint16_t*>(da), ld, rows,
                       (int)cols, out);
    return hipGetLastError();
}

}  // namespace tpl
