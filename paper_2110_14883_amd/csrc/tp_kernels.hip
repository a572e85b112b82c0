// gfx950 (MI355X, CDNA4) kernels for one rank's share of a tensor-parallel linear layer
// (paper Section 2.2, tensor parallelism: the local block products of the 1D / 2D-SUMMA / 2.5D /
// 3D schemes, C = sum_k A_k B_k over the steps, then bias + erf-GeLU; and the two backward
// products).  bf16 operands, fp32 accumulation in MFMA 32x32x16 tiles.
//
// The eight-wave GEMM of this file serves the 128 x 256, 256 x 128 and 128 x 128 macro-tiles (and 256 x 256
// on request), the rest of the file the split-K fix-up and the elementwise kernels.  One kernel template
// serves the three memory forms (NN forward, NT dX, TN dW):
//   * persistent workgroups (one per CU) of 8 wave64 walk over the BM x BN tiles of C; a tile's
//     accumulators stay in registers across ALL steps and all K tiles -- no partial C leaves the
//     chip unless the host asked for a cross-workgroup split of K;
//   * ping-pong: waves 0-3 ("P", one per SIMD) stage operand A, waves 4-7 ("Q") stage operand B.
//     Inside one K tile P multiplies first and refills LDS afterwards, Q refills first and
//     multiplies afterwards, so every SIMD always has one wave with MFMAs ready while the other
//     one waits on global loads or writes LDS.  One workgroup barrier per K tile;
//   * K tiles of 64 are double-buffered in LDS (2 x 64 KB); the tile after next travels through
//     registers, fetched with 128-bit buffer loads whose out-of-range chunks read as zero (that
//     is how ragged M / K tails are masked);
//   * operands whose contraction index is not contiguous in memory are transposed in registers
//     (8 x 8 blocks, byte permutes) on the way into LDS, so the MFMA side always reads 8
//     consecutive k with one ds_read_b128; LDS rows are 128 B with the 16-byte chunk index
//     XOR-swizzled so that fragment reads and both kinds of writes are free of bank conflicts;
//   * the MFMA is issued with the operands swapped (C^T = B^T A^T) so that each lane ends up with
//     4 consecutive columns of one row of C: bias / GeLU / GeLU' run in registers, and each 32-row
//     slab then passes through a wave-private LDS patch so that the stores are whole 128-byte row
//     segments.  (This kernel's pipeline drains at every C tile: the next tile's first fetch is
//     issued after the epilogue.  The four-wave kernel of tp_gemm4.hip, which takes the 256 x 256
//     tiles, keeps its K tiles flowing across C tiles.)
//   * tile ids are spread so that each XCD (own L2) works on a compact patch of tiles.
#include "tp_device.h"

namespace tpl {

template <int V> using KS = std::integral_constant<int, V>;

struct TileCoord { int m0, n0, z, rot, g; };

// ---------------------------------------------------------------------------------------------
// one wave group's part of the GEMM (IS_P: waves 0-3, stage A;  else waves 4-7, stage B)
// ---------------------------------------------------------------------------------------------
template <int BM, int BN, bool A_KC, bool B_KC, int EPI, bool F32_OUT, bool IS_P>
__device__ __forceinline__ void gemm_role(const GemmArgs& p, char* lds, const int t, const int w) {
    constexpr int TM = BM / 64;      // 32-row MFMA tiles per wave along M (2 waves along M)
    constexpr int TN = BN / 128;     // 32-col MFMA tiles per wave along N (4 waves along N)
    constexpr int A_BYTES = BM * BK * 2;
    constexpr int STAGE_BYTES = (BM + BN) * BK * 2;
    constexpr int PART = IS_P ? 0 : A_BYTES;          // where this group's operand sits inside a stage
    using Stage = typename std::conditional<IS_P,
        typename std::conditional<A_KC, HalfKC<BM>, HalfXC<BM>>::type,
        typename std::conditional<B_KC, HalfKC<BN>, HalfXC<BN>>::type>::type;

    const int l = t & 63, tg = t & 255;
    const int wm = w & 1, wn = ((w >> 1) & 1) | ((w >> 2) << 1);   // P waves: wn in {0,1}; Q waves: wn in {2,3}
    const int ra = wm * (BM / 2) + (l & 31);       // fragment rows inside the wave's slab
    const int rb = wn * (BN / 4) + (l & 31);
    const int ch = l >> 5;                         // k chunk = 2 ks + lane/32
    char* const eps = lds + 2 * STAGE_BYTES + w * EPI_BYTES_PER_WAVE;   // wave-private epilogue patch

    const int KT = (p.K + BK - 1) / BK;
    const int T = p.n_steps * KT;
    const int Z = p.split_k;
    const int total = p.tiles_m * p.tiles_n * Z;

    Stage st;
    // Inside a step the K tiles are taken in a rotated order that differs from C tile to C tile, so
    // that the CUs of one XCD are not all asking the same memory channel for the same K offset.
    // Operand stream of this wave group.  The K tiles of a C tile are fetched strictly in order (units
    // z, z+Z, z+2Z, ... of the n_steps x KT sequence), so the step a fetch belongs to is tracked
    // incrementally: the operand block's pointer and leading dimension are re-read from the argument
    // block only when the step changes, and nothing is divided inside the K loop.
    int f_step = 0, f_kt = 0;                     // step (operand slot) and K tile inside it, before the rotation
    const uint16_t* f_ptr = nullptr;
    int f_ld = 0;
    auto open_step = [&](int s) __attribute__((always_inline)) {
        f_step = s;
        if constexpr (IS_P) { f_ptr = static_cast<const uint16_t*>(p.a[s]); f_ld = p.lda[s]; }
        else                { f_ptr = static_cast<const uint16_t*>(p.b[s]); f_ld = p.ldb[s]; }
    };
    auto seek = [&](const TileCoord& c, int unit) __attribute__((always_inline)) {
        const int s = unit / KT;
        f_kt = unit - s * KT;
        open_step(s + c.g);                       // a grouped launch has one step per group: operand slot = group
    };
    auto fetch_next = [&](const TileCoord& c) __attribute__((always_inline)) {
        int kt = f_kt + c.rot;
        if (kt >= KT) kt -= KT;
        const int k0 = kt * BK;
        // (the leading dimension is made opaque here: seen as loop-invariant, the per-lane row offsets
        // of all eight loads would be kept in registers across the K loop, which does not have them)
        asm volatile("" : "+s"(f_ld));
        if constexpr (IS_P) {
            if constexpr (A_KC) st.load(f_ptr, f_ld, p.M, c.m0, p.K, k0, tg);
            else                st.load(f_ptr, f_ld, p.K, k0, p.M, c.m0, tg);
        } else {
            if constexpr (B_KC) st.load(f_ptr, f_ld, p.N, c.n0, p.K, k0, tg);
            else                st.load(f_ptr, f_ld, p.K, k0, p.N, c.n0, tg);
        }
        f_kt += Z;
        while (f_kt >= KT && f_step + 1 < TP_MAX_STEPS) {      // (past the last step only after the tile's last fetch)
            f_kt -= KT;
            open_step(f_step + 1);
        }
    };
    auto locate = [&](int v) __attribute__((always_inline)) {
        int tm, tn, z;
        tile_of_id(p, v, tm, tn, z);
        const int rot = p.rotate ? ((tm * 3 + tn * 5) & 7) % KT : 0;
        int g = 0;
        if (p.n_groups > 1) {
            if (p.group_along_n) { g = tn / p.group_tiles; tn -= g * p.group_tiles; }
            else                 { g = tm / p.group_tiles; tm -= g * p.group_tiles; }
        }
        return TileCoord{tm * BM, tn * BN, z, rot, g};
    };

    f32x16_t acc[TM][TN];
    // One K tile = 4 MFMA k-steps.  The fragment reads of step ks+1 are issued while the MFMAs of
    // step ks run: the B fragments are double-buffered, an A fragment's registers are re-read as
    // soon as its two MFMAs have issued.  The sched_group_barrier calls pin that interleaving
    // (2 MFMA, 1 LDS read, ...), so a wave that multiplies alone still keeps the MFMA pipe busy.
    auto compute = [&](int cur) __attribute__((always_inline)) {
        const char* la = lds + cur * STAGE_BYTES;
        const char* lb = la + A_BYTES;
        bf16x8_t fa[TM], fb[2][TN];
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[0][j] = *reinterpret_cast<const bf16x8_t*>(lb + lds_off(rb + 32 * j, ch));
#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[i] = *reinterpret_cast<const bf16x8_t*>(la + lds_off(ra + 32 * i, ch));
        __builtin_amdgcn_sched_group_barrier(0x100, TM + TN, 0);
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            const bool more = ks + 1 < BK / 16;
            if (more) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    fb[(ks + 1) & 1][j] = *reinterpret_cast<const bf16x8_t*>(lb + lds_off(rb + 32 * j, 2 * (ks + 1) + ch));
                __builtin_amdgcn_sched_group_barrier(0x100, TN, 0);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks & 1][j], fa[i], acc[i][j], 0, 0, 0);
                __builtin_amdgcn_sched_group_barrier(0x008, TN, 0);
                if (more) {
                    fa[i] = *reinterpret_cast<const bf16x8_t*>(la + lds_off(ra + 32 * i, 2 * (ks + 1) + ch));
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
            }
        }
        __builtin_amdgcn_s_setprio(0);
    };

    int v = blockIdx.x;
    if (v >= total) return;
    TileCoord cur_tile = locate(v);
    seek(cur_tile, cur_tile.z);
    fetch_next(cur_tile);

    while (true) {
        const int z = cur_tile.z;
        const int my_tiles = (T - z + Z - 1) / Z;       // K tiles z, z+Z, ...: every step is visited
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

        // K tile 0 -> LDS stage 0, K tile 1 -> registers
        st.store(lds + PART, tg);
        if (my_tiles > 1) fetch_next(cur_tile);
        __syncthreads();

        for (int i = 0; i < my_tiles; ++i) {
            const int cur = i & 1;
            char* refill = lds + (cur ^ 1) * STAGE_BYTES + PART;    // last read one iteration ago, by everybody
            if constexpr (IS_P) {
                compute(cur);
                if (i + 1 < my_tiles) st.store(refill, tg);
                if (i + 2 < my_tiles) fetch_next(cur_tile);
            } else {
                if (i + 1 < my_tiles) st.store(refill, tg);
                if (i + 2 < my_tiles) fetch_next(cur_tile);
                compute(cur);
            }
            __syncthreads();
        }


        // ---------------------------------------------------------------- epilogue
        // acc[i][j][e]: row m = 32 i + lane%32, columns n = 32 j + 8 (e/4) + 4 (lane/32) + e%4.
        // Bias / GeLU / GeLU' are applied in registers; every 32-row slab then passes through a
        // wave-private 4 KB LDS patch so that the global stores are whole 128-byte row segments.
        {
            const int m_sub = cur_tile.m0 + wm * (BM / 2);          // first row of this wave's slab
            const int n_sub = cur_tile.n0 + wn * (BN / 4);          // first column
            // (lane-derived values of the epilogue are formed here, from an opaque copy of the lane id, so
            // that none of them is computed ahead of the K loop and carried across it in a register)
            int le = l;
            asm volatile("" : "+v"(le));
            const int r = le & 31;                                  // row of this lane inside a 32-row slab
            const int ch = le >> 5;                                 // which half of each 8-column group this lane holds
            const int l = le;
            const bool partial = Z > 1;          // split K: raw fp32 partials, the fix-up kernel runs the epilogue
            constexpr bool use_bias = EPI == EPI_BIAS || EPI == EPI_BIAS_GELU;
            constexpr bool use_gelu = EPI == EPI_BIAS_GELU;
            constexpr bool use_dg = EPI == EPI_MUL_DGELU;
            const bool use_pre = !use_dg && p.pre != nullptr;

            // value functors: 4 consecutive columns (j, g) of row r of slab i
            auto raw4 = [&](int i, int j, int g, float (&v)[4]) __attribute__((always_inline)) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * g + e];
            };
            auto preact4 = [&](int i, int j, int g, float (&v)[4]) __attribute__((always_inline)) {
                raw4(i, j, g, v);
                if constexpr (use_bias) {
                    const int n = n_sub + 32 * j + 8 * g + 4 * ch;
                    u32x2_t b = {0u, 0u};
                    if (n < p.N) b = *reinterpret_cast<const u32x2_t*>(static_cast<const uint16_t*>(p.bias) + n);
                    v[0] += bf16_lo(b[0]); v[1] += bf16_hi(b[0]); v[2] += bf16_lo(b[1]); v[3] += bf16_hi(b[1]);
                }
            };
            auto final4 = [&](int i, int j, int g, float (&v)[4]) __attribute__((always_inline)) {
                preact4(i, j, g, v);
                if constexpr (use_gelu) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] = gelu_f(v[e]);
                }
                if constexpr (use_dg) {
                    const int m = m_sub + 32 * i + r, n = n_sub + 32 * j + 8 * g + 4 * ch;
                    if (m < p.M && n < p.N) {
                        const u32x2_t a = *reinterpret_cast<const u32x2_t*>(static_cast<const uint16_t*>(p.dg) + (int64_t)m * p.lddg + n);
                        v[0] *= dgelu_f(bf16_lo(a[0])); v[1] *= dgelu_f(bf16_hi(a[0]));
                        v[2] *= dgelu_f(bf16_lo(a[1])); v[3] *= dgelu_f(bf16_hi(a[1]));
                    }
                }
            };
            // bf16 slab: rows of 32*TN bf16 (RB bytes); lane writes 8 bytes, reads back 16
            constexpr int RB = 32 * TN * 2, CPR = RB / 16, RPI = 64 / CPR;      // chunks per row, rows per instruction
            auto sw16 = [](int row) { return (row / (256 / RB)) & (CPR - 1); };
            auto slab_bf16 = [&](int i, auto value4, uint16_t* base, int64_t ld) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        float x[4];
                        value4(i, j, g, x);
                        const u32x2_t v = {pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3])};
                        *reinterpret_cast<u32x2_t*>(eps + r * RB + (((4 * j + g) ^ sw16(r)) << 4) + 8 * ch) = v;
                    }
#pragma unroll
                for (int it = 0; it < 32 / RPI; ++it) {
                    const int rr = it * RPI + l / CPR, c = l % CPR;
                    const u32x4_t v = *reinterpret_cast<const u32x4_t*>(eps + rr * RB + ((c ^ sw16(rr)) << 4));
                    const int m = m_sub + 32 * i + rr, n = n_sub + 8 * c;
                    if (m < p.M && n < p.N) *reinterpret_cast<u32x4_t*>(base + (int64_t)m * ld + n) = v;
                }
            };
            // fp32 slab, one 32-column block at a time: rows of 128 bytes; lane writes 16 bytes, reads back 16
            auto slab_f32 = [&](int i, auto value4, float* base, int64_t ld) __attribute__((always_inline)) {
#pragma unroll
                for (int j = 0; j < TN; ++j) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        float x[4];
                        value4(i, j, g, x);
                        const f32x4_t v = {x[0], x[1], x[2], x[3]};
                        *reinterpret_cast<f32x4_t*>(eps + r * 128 + (((2 * g + ch) ^ ((r >> 1) & 7)) << 4)) = v;
                    }
#pragma unroll
                    for (int it = 0; it < 4; ++it) {
                        const int rr = it * 8 + (l >> 3), c = l & 7;
                        const f32x4_t v = *reinterpret_cast<const f32x4_t*>(eps + rr * 128 + ((c ^ ((rr >> 1) & 7)) << 4));
                        const int m = m_sub + 32 * i + rr, n = n_sub + 32 * j + 4 * c;
                        if (m < p.M && n < p.N) *reinterpret_cast<f32x4_t*>(base + (int64_t)m * ld + n) = v;
                    }
                }
            };

            if (partial) {
                float* const wsz = p.ws + ((int64_t)z * p.n_groups + cur_tile.g) * p.M * p.N;
#pragma unroll
                for (int i = 0; i < TM; ++i) slab_f32(i, raw4, wsz, (int64_t)p.N);
            } else {
#pragma unroll
                for (int i = 0; i < TM; ++i) {
                    if constexpr (!use_dg) {
                        if (use_pre) slab_bf16(i, preact4, static_cast<uint16_t*>(p.pre), p.ldp);
                    }
                    if constexpr (F32_OUT) slab_f32(i, final4, static_cast<float*>(p.outs[cur_tile.g]), p.ldos[cur_tile.g]);
                    else                   slab_bf16(i, final4, static_cast<uint16_t*>(p.outs[cur_tile.g]), p.ldos[cur_tile.g]);
                }
            }
        }
        v += gridDim.x;
        if (v >= total) break;
        cur_tile = locate(v);
        seek(cur_tile, cur_tile.z);
        fetch_next(cur_tile);
    }
}

template <int BM, int BN, bool A_KC, bool B_KC, int EPI, bool F32_OUT>
__global__ __launch_bounds__(NTHREADS) void tp_gemm_kernel(const GemmArgs p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int t = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);     // wave index, known uniform
    if (w < 4) gemm_role<BM, BN, A_KC, B_KC, EPI, F32_OUT, true>(p, lds, t, w);
    else       gemm_role<BM, BN, A_KC, B_KC, EPI, F32_OUT, false>(p, lds, t, w);
}

// ---------------------------------------------------------------------------------------------
// split-K fix-up: sum the fp32 partials in a fixed order, then the same epilogue
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void tp_reduce_kernel(const ReduceArgs p) {
    const int n4 = p.N >> 2;
    const int64_t total = (int64_t)p.M * n4;
    const int64_t plane = p.plane;
    Epilogue e{p.out, p.ldo, p.out_f32, p.pre, p.ldp, p.bias, p.gelu, p.dg, p.lddg};
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x) {
        const int m = (int)(idx / n4);
        const int n = (int)(idx - (int64_t)m * n4) * 4;
        const float* src = p.ws + (int64_t)m * p.N + n;
        f32x4_t s = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(src));
        for (int zz = 1; zz < p.split_k; ++zz) {
            const f32x4_t q = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(src + zz * plane));
            s[0] += q[0]; s[1] += q[1]; s[2] += q[2]; s[3] += q[3];
        }
        float v[4] = {s[0], s[1], s[2], s[3]};
        epilogue4(e, v, m, n);
    }
}

// ---------------------------------------------------------------------------------------------
// da = bf16(dy * GeLU'(pre)).  8 elements per 128-bit access; every thread keeps two independent
// trips (four loads) in flight.  GeLU'(a) = 1 + h for a >= 0 and -h for a < 0 with
// h = |a| phi(a) - Phi(-|a|), which needs the sign only once, at the end.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float dgelu_times(float g, float a) {
    const float x = fabsf(a) * 0.70710678118654752f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, x, 1.0f));
    float q = fmaf(t, 0.5f * 1.061405429f, 0.5f * -1.453152027f);      // half the erfc polynomial: Phi(-|a|) = q e
    q = fmaf(t, q, 0.5f * 1.421413741f);
    q = fmaf(t, q, 0.5f * -0.284496736f);
    q = fmaf(t, q, 0.5f * 0.254829592f);
    q *= t;
    const float e = __builtin_amdgcn_exp2f(a * a * -0.72134752044448170f);   // exp(-a^2/2)
    const float h = e * fmaf(x, 0.56418958354775629f, -q);                    // |a| phi(a) = x e / sqrt(pi)
    return g * (a < 0.0f ? -h : 1.0f + h);
}
__device__ __forceinline__ u32x4_t dgelu8(const u32x4_t g, const u32x4_t a) {
    u32x4_t o;
#pragma unroll
    for (int i = 0; i < 4; ++i)
        o[i] = pack_bf16(dgelu_times(bf16_lo(g[i]), bf16_lo(a[i])), dgelu_times(bf16_hi(g[i]), bf16_hi(a[i])));
    return o;
}
// One 128-bit access per thread and a grid that covers the block (the loop only runs again beyond 2^30
// workgroups): neighbouring workgroups then touch neighbouring memory, which measured 15 % faster than a
// persistent grid-stride loop with several loads in flight; the streaming (nontemporal) hint on loads and
// stores is worth another 9 %: 6.4 TB/s against 5.9 for a plain bf16 add of the same shape.
__global__ __launch_bounds__(256) void tp_dgelu_kernel(const uint16_t* dy, int64_t ld_dy, const uint16_t* pre,
                                                       int64_t ld_pre, uint16_t* da, int64_t ld_da,
                                                       int64_t rows, int cols8) {
    const int64_t total = rows * cols8;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = idx / cols8;
        const int c = (int)(idx - r * cols8) * 8;
        const u32x4_t g = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(dy + r * ld_dy + c));
        const u32x4_t a = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(pre + r * ld_pre + c));
        __builtin_nontemporal_store(dgelu8(g, a), reinterpret_cast<u32x4_t*>(da + r * ld_da + c));
    }
}

// y = [GeLU](c + bias) over an fp32 block (what follows the summation of forward partials),
// optional bf16 copy of c + bias; 4 elements per thread, same launch shape and hints as tp_dgelu_kernel
__global__ __launch_bounds__(256) void tp_bias_act_kernel(const float* c, int64_t ldc, const uint16_t* bias, int gelu,
                                                          void* y, int64_t ldy, int y_f32, uint16_t* pre, int64_t ldp,
                                                          int64_t rows, int cols4) {
    const int64_t total = rows * cols4;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = idx / cols4;
        const int n = (int)(idx - r * cols4) * 4;
        const f32x4_t x = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(c + r * ldc + n));
        float v[4] = {x[0], x[1], x[2], x[3]};
        if (bias) {
            const u32x2_t b = *reinterpret_cast<const u32x2_t*>(bias + n);
            v[0] += bf16_lo(b[0]); v[1] += bf16_hi(b[0]); v[2] += bf16_lo(b[1]); v[3] += bf16_hi(b[1]);
        }
        if (pre) {
            const u32x2_t s = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
            __builtin_nontemporal_store(s, reinterpret_cast<u32x2_t*>(pre + r * ldp + n));
        }
        if (gelu) {
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = gelu_f(v[i]);
        }
        if (y_f32) {
            const f32x4_t o = {v[0], v[1], v[2], v[3]};
            __builtin_nontemporal_store(o, reinterpret_cast<f32x4_t*>(static_cast<float*>(y) + r * ldy + n));
        } else {
            const u32x2_t o = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])};
            __builtin_nontemporal_store(o, reinterpret_cast<u32x2_t*>(static_cast<uint16_t*>(y) + r * ldy + n));
        }
    }
}

// Column sums of a bf16 [rows][cols] block into fp32.  Workgroup (bx, by) sums rows
// [by * rows_per_split, ...) of columns 64 bx .. 64 bx + 63 into out[by][cols]; with one split that is the
// result, with several tp_colsum_finish_kernel adds the splits in ascending order.  Every order of
// summation is fixed by (rows, cols) alone: the result is reproducible.
__global__ __launch_bounds__(256) void tp_colsum_kernel(const uint16_t* da, int64_t ld, int64_t rows, int cols, float* out,
                                                        int64_t rows_per_split) {
    __shared__ float part[32][65];
    const int cl = threadIdx.x & 7, rl = threadIdx.x >> 3;        // 8 chunk lanes x 32 row lanes
    const int c = blockIdx.x * 64 + cl * 8;
    const int64_t r_begin = (int64_t)blockIdx.y * rows_per_split;
    const int64_t r_end = r_begin + rows_per_split < rows ? r_begin + rows_per_split : rows;
    float s[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    if (c < cols) {
        int64_t r = r_begin + rl;
        for (; r + 96 < r_end; r += 128) {                        // four independent loads in flight
            u32x4_t v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(da + (r + 32 * u) * ld + c));
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) { s[2 * i] += bf16_lo(v[u][i]); s[2 * i + 1] += bf16_hi(v[u][i]); }
        }
        for (; r < r_end; r += 32) {
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
        if (cc < cols) out[(int64_t)blockIdx.y * cols + cc] = tot;
    }
}
__global__ __launch_bounds__(256) void tp_colsum_finish_kernel(const float* part, int splits, int cols, float* out) {
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= cols) return;
    float tot = 0.0f;
    for (int r = 0; r < splits; ++r) tot += part[(int64_t)r * cols + c];
    out[c] = tot;
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

template <int BM, int BN, bool A_KC, bool B_KC, int EPI, bool F32_OUT>
static hipError_t launch_one(const GemmArgs& a, hipStream_t stream) {
    constexpr int lds_bytes = 2 * (BM + BN) * BK * 2 + 8 * EPI_BYTES_PER_WAVE;
    // the LDS limit is a per-device attribute of the kernel: set it once on every device that launches
    // it (same value every time, so a repeated or concurrent set is harmless)
    static std::atomic<uint64_t> attr_done{0};
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (!(attr_done.load(std::memory_order_relaxed) & bit)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&tp_gemm_kernel<BM, BN, A_KC, B_KC, EPI, F32_OUT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_done.fetch_or(bit, std::memory_order_relaxed);
    }
    // persistent: never more workgroups than the chip holds at once (one per CU with this much LDS)
    const int total = a.tiles_m * a.tiles_n * a.split_k;
    const unsigned grid = (unsigned)(total < a.max_workgroups ? total : a.max_workgroups);
    return launch_kernel(tp_gemm_kernel<BM, BN, A_KC, B_KC, EPI, F32_OUT>, dim3(grid), dim3(NTHREADS), lds_bytes, stream, a);
}

template <int BM, int BN>
static hipError_t launch_tile(int form, const GemmArgs& a, hipStream_t s) {
    // the epilogue is compiled in, per memory form: forward (NN) adds bias / GeLU, dX (NT) may
    // multiply by GeLU', dW (TN) stores plain fp32.  A launch that splits K writes raw partials.
    const int epi = a.split_k > 1 ? EPI_NONE : (a.dg ? EPI_MUL_DGELU : (a.gelu ? EPI_BIAS_GELU : (a.bias ? EPI_BIAS : EPI_NONE)));
    const bool f32 = a.split_k > 1 || a.out_f32;
    switch (form) {
        case FORM_NN:
            if (epi == EPI_BIAS_GELU) return f32 ? launch_one<BM, BN, true, false, EPI_BIAS_GELU, true>(a, s) : launch_one<BM, BN, true, false, EPI_BIAS_GELU, false>(a, s);
            if (epi == EPI_BIAS)      return f32 ? launch_one<BM, BN, true, false, EPI_BIAS, true>(a, s) : launch_one<BM, BN, true, false, EPI_BIAS, false>(a, s);
            if (epi == EPI_NONE)      return f32 ? launch_one<BM, BN, true, false, EPI_NONE, true>(a, s) : launch_one<BM, BN, true, false, EPI_NONE, false>(a, s);
            return hipErrorInvalidValue;
        case FORM_NT:
            if (epi == EPI_MUL_DGELU) return f32 ? launch_one<BM, BN, true, true, EPI_MUL_DGELU, true>(a, s) : launch_one<BM, BN, true, true, EPI_MUL_DGELU, false>(a, s);
            if (epi == EPI_NONE)      return f32 ? launch_one<BM, BN, true, true, EPI_NONE, true>(a, s) : launch_one<BM, BN, true, true, EPI_NONE, false>(a, s);
            return hipErrorInvalidValue;
        case FORM_TN:
            if (epi == EPI_NONE && f32) return launch_one<BM, BN, false, false, EPI_NONE, true>(a, s);
            return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_gemm(int form, int tile_id, const GemmArgs& args, hipStream_t s) {
    GemmArgs a = args;
    if (a.n_groups <= 1) {             // a plain launch is one group whose output is `out`
        a.n_groups = 1; a.group_along_n = 1; a.group_tiles = a.tiles_n;
        a.outs[0] = a.out; a.ldos[0] = a.ldo;
    } else if (a.n_steps != 1 || a.n_groups > TP_MAX_STEPS || a.group_tiles < 1 || a.bias || a.dg || a.pre ||
               (a.group_along_n ? a.tiles_n : a.tiles_m) != a.n_groups * a.group_tiles) {
        return hipErrorInvalidValue;
    }
    switch (tile_id) {
        case TILE_256x256: return launch_tile<256, 256>(form, a, s);
        case TILE_128x256: return launch_tile<128, 256>(form, a, s);
        case TILE_256x128: return launch_tile<256, 128>(form, a, s);
        case TILE_128x128: return launch_tile<128, 128>(form, a, s);
        case TILE_256x256_W4: return launch_gemm4(form, a, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_reduce(const ReduceArgs& a, hipStream_t s) {
    const int64_t total = (int64_t)a.M * (a.N >> 2);
    int64_t blocks = (total + 255) / 256;
    if (blocks > ((int64_t)1 << 30)) blocks = (int64_t)1 << 30;
    if (blocks < 1) blocks = 1;
    return launch_kernel(tp_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
}

hipError_t launch_dgelu(const void* dy, int64_t ld_dy, const void* pre, int64_t ld_pre, void* da, int64_t ld_da,
                        int64_t rows, int64_t cols, hipStream_t s) {
    const int64_t total = rows * (cols >> 3);
    if (total == 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > ((int64_t)1 << 30)) blocks = (int64_t)1 << 30;
    return launch_kernel(tp_dgelu_kernel, dim3((unsigned)blocks), dim3(256), 0, s, static_cast<const uint16_t*>(dy), ld_dy,
                         static_cast<const uint16_t*>(pre), ld_pre, static_cast<uint16_t*>(da), ld_da, rows,
                         (int)(cols >> 3));
}

hipError_t launch_bias_act(const float* c, int64_t ldc, const void* bias, int gelu, void* y, int64_t ldy, int y_f32,
                           void* pre, int64_t ldp, int64_t rows, int64_t cols, hipStream_t s) {
    const int64_t total = rows * (cols >> 2);
    if (total == 0) return hipSuccess;
    int64_t blocks = (total + 255) / 256;
    if (blocks > ((int64_t)1 << 30)) blocks = (int64_t)1 << 30;
    return launch_kernel(tp_bias_act_kernel, dim3((unsigned)blocks), dim3(256), 0, s, c, ldc, static_cast<const uint16_t*>(bias),
                         gelu, y, ldy, y_f32, static_cast<uint16_t*>(pre), ldp, rows, (int)(cols >> 2));
}

// Row splits of the column sum: enough workgroups to fill the chip four times over, at least 256 rows each.
int colsum_splits(int64_t rows, int64_t cols) {
    const int64_t col_blocks = (cols + 63) / 64;
    if (col_blocks >= 256) return 1;                    // one workgroup per 64 columns already fills the chip
    int64_t r = col_blocks > 0 ? (1024 + col_blocks - 1) / col_blocks : 1;
    const int64_t by_rows = (rows + 255) / 256;
    if (r > by_rows) r = by_rows;
    if (r > 64) r = 64;
    return r < 1 ? 1 : (int)r;
}
size_t colsum_ws_bytes(int64_t rows, int64_t cols) {
    const int r = colsum_splits(rows, cols);
    return r > 1 ? (size_t)r * (size_t)cols * 4 : 0;
}
// ws: colsum_ws_bytes(rows, cols) bytes, or null for the single-pass form (one workgroup per 64 columns)
hipError_t launch_colsum(const void* da, int64_t ld, int64_t rows, int64_t cols, float* out, float* ws, hipStream_t s) {
    const unsigned col_blocks = (unsigned)((cols + 63) / 64);
    const int splits = ws ? colsum_splits(rows, cols) : 1;
    if (splits == 1)
        return launch_kernel(tp_colsum_kernel, dim3(col_blocks), dim3(256), 0, s, static_cast<const uint16_t*>(da), ld, rows,
                             (int)cols, out, rows);
    const int64_t per = ((rows + splits - 1) / splits + 31) / 32 * 32;
    if (hipError_t e = launch_kernel(tp_colsum_kernel, dim3(col_blocks, (unsigned)splits), dim3(256), 0, s,
                                     static_cast<const uint16_t*>(da), ld, rows, (int)cols, ws, per); e != hipSuccess)
        return e;
    return launch_kernel(tp_colsum_finish_kernel, dim3((unsigned)((cols + 255) / 256)), dim3(256), 0, s,
                         static_cast<const float*>(ws), splits, (int)cols, out);
}

}  // namespace tpl
