// gfx950 (MI355X, CDNA4): the 256 x 256 macro-tile GEMM of libtplinear as ONE software pipeline per
// workgroup (paper Section 2.2, tensor parallelism: the local block products C = sum_k A_k B_k of
// the 1D / 2D / 2.5D / 3D schemes and the two backward products).
//
//   * four wave64 per workgroup, one per SIMD, each owning a 128 x 128 block of the C tile: 16 MFMA
//     32x32x16 accumulators = 256 registers in the accumulator half of the register file, and only
//     32 LDS fragment reads per 64 MFMAs (the eight-wave kernel reads 48);
//   * the K tiles of ALL the C tiles a persistent workgroup owns form one stream: K tile u is being
//     multiplied out of one LDS stage while tile u+1 travels from registers into the other stage and
//     tile u+2 is being fetched from memory, across C-tile boundaries too, so the epilogue of a C tile
//     runs with the first two K tiles of the next one already on their way;
//   * every LDS write, global load and fragment read has a fixed slot between two MFMAs of the
//     64-MFMA K tile (scheduling fences pin the order); the one workgroup barrier per K tile sits
//     after MFMA 48, and the last 16 MFMAs cover the first fragment reads of the next K tile, so no
//     LDS latency is exposed at the tile boundary;
//   * LDS layout, register transposes of the operands that are not contraction-contiguous, tile
//     order and epilogue (bias / GeLU / GeLU' in registers, then through a wave-private LDS patch so
//     that stores are whole 128-byte row segments) are those of the eight-wave kernel.
#include <utility>

#include "tp_device.h"

namespace tpl {

namespace {

template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// a value every lane agrees on, pinned to a scalar register (keeps the cursor arithmetic on the scalar unit)
__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ const uint16_t* uni_ptr(const void* q) {
    const uint64_t v = reinterpret_cast<uint64_t>(q);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return reinterpret_cast<const uint16_t*>(((uint64_t)hi << 32) | lo);
}

// LDS access by 32-bit byte address.  The kernel has no static LDS, so its dynamic LDS starts at
// address 0 and an address is the offset into it.
typedef __attribute__((address_space(3))) u32x4_t lds_u32x4_t;
typedef __attribute__((address_space(3))) bf16x8_t lds_bf16x8_t;
__device__ __forceinline__ void lds_store16(uint32_t addr, u32x4_t v) { *reinterpret_cast<lds_u32x4_t*>(addr) = v; }
__device__ __forceinline__ bf16x8_t lds_load_frag(uint32_t addr) { return *reinterpret_cast<const lds_bf16x8_t*>(addr); }

// One direct-to-LDS load: each lane's 16 bytes go from global memory straight into LDS, lane l at
// byte lds_base + 16 l (lds_base: wave-uniform, travels in M0), without touching the vector registers.
// Out-of-range lanes write zeros.  The compiler does not see this load: whoever reads the data waits
// for it with wait_vm() and a barrier.
__device__ __forceinline__ void dtl_load16(u32x4_t rsrc_words, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :: "s"(lds_base), "v"(voff), "s"(rsrc_words) : "memory");
}
template <int N> __device__ __forceinline__ void wait_vm() {      // at most N vector-memory operations outstanding
    static_assert(N >= 0 && N < 64);
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

constexpr int W4_THREADS = 256;
constexpr int W4_BM = 256, W4_BN = 256;
constexpr int W4_STAGE_STRIDE = W4_BM * BK * 2;              // 32 KB: one stage of one operand
constexpr int W4_B_BASE = 2 * W4_STAGE_STRIDE;               // LDS: A stage 0 | A stage 1 | B stage 0 | B stage 1 | epilogue
constexpr int W4_EPI_BASE = 4 * W4_STAGE_STRIDE;
constexpr int W4_EPI_BYTES_PER_WAVE = 8192;                  // 32 rows x 256 bytes
constexpr int W4_LDS_BYTES = W4_EPI_BASE + 4 * W4_EPI_BYTES_PER_WAVE;

// Slot tables: after which MFMA (0..63) of a K tile each staging operation is issued.  All four waves
// run the same schedule, so a slot with a global load asks the CU's one address path for 4 KB and a
// slot with an LDS write sends 4 KB over the LDS data bus: loads are kept three or four slots apart,
// writes two or three, and all writes come before the barrier that follows slot 47.  A
// contraction-contiguous operand frees one register quad per write and reloads it soon after; a
// transposed operand needs all its eight quads for every write (the permutes that form a write's four
// words go one slot earlier), so it is written out first and fast, and its reloads follow its last write.
//   pm(n): slot of the permutes of the n-th write (transposed operands), wr(n): slot of the n-th LDS
//   write of an operand, ld(n): slot of its n-th global load.
struct Slots { int pm[8]; int wr[8]; int ld[8]; };
template <bool KC, bool FIRST, bool OTHER_KC>
constexpr Slots make_slots() {
    Slots s{};
    for (int n = 0; n < 8; ++n) {
        if (KC && OTHER_KC) {                    // both contiguous: writes every third slot, loads every fourth
            const int m = FIRST ? n : n + 8;
            s.pm[n] = -1; s.wr[n] = 3 * m + 1; s.ld[n] = 4 * m + 2;
        } else if (!KC && FIRST) {               // transposed, first: slots 0 .. 15, reloads 16 .. 37
            s.pm[n] = 2 * n; s.wr[n] = 2 * n + 1; s.ld[n] = 16 + 3 * n;
        } else if (!KC) {                        // transposed, second: slots 16 .. 31, reloads 40 .. 61
            s.pm[n] = 16 + 2 * n; s.wr[n] = 17 + 2 * n; s.ld[n] = 40 + 3 * n;
        } else {                                 // contiguous, after a transposed one
            s.pm[n] = -1; s.wr[n] = 17 + 3 * n; s.ld[n] = 40 + 3 * n;
        }
    }
    return s;
}

}  // namespace

template <bool A_KC, bool B_KC, int EPI, bool F32_OUT>
__global__ __launch_bounds__(W4_THREADS) __attribute__((amdgpu_waves_per_eu(1, 1)))
void tp_gemm4_kernel(const GemmArgs p) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    constexpr int TM = 4, TN = 4;                  // 32 x 32 MFMA tiles per wave along M and N
    // the transposed operand (if there is exactly one) is staged first: its reloads need the longer lead
    constexpr bool A_FIRST = A_KC ? B_KC : true;
    // A contraction-contiguous operand goes from memory to LDS directly: both operands of the NT form,
    // operand A of the NN form (HYB: B then takes the register path with its transposes).
    constexpr bool DA = A_KC, DB = A_KC && B_KC;
    constexpr bool DTL = DA && DB, HYB = DA && !DB;
    static constexpr Slots SA = make_slots<A_KC, A_FIRST, B_KC>();
    static constexpr Slots SB = make_slots<B_KC, !A_FIRST, A_KC>();

    const int t = threadIdx.x;
    const int l = t & 63;
    const int w = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = w & 1, wn = w >> 1;
    char* const eps = lds + W4_EPI_BASE + w * W4_EPI_BYTES_PER_WAVE;

    const int KT = (p.K + BK - 1) / BK;
    const int T = p.n_steps * KT;
    const int Z = p.split_k;
    const int total = p.tiles_m * p.tiles_n * Z;
    const int grid = (int)gridDim.x;

    // ------------------------------------------------------------------ LDS addresses (bytes), per lane
    // LDS map: A stage 0 | A stage 1 | B stage 0 | B stage 1 (32 KB each) | epilogue patches.  The two
    // stages of an operand are 32 KB apart, which fits the 16-bit immediate offset of the LDS
    // instructions: the K tiles of a C tile alternate between two compiled bodies that differ only in
    // those immediates, and no address is recomputed inside the loop.
    // Fragment of 32 rows x 16 k for MFMA step ks, row block i: lane reads row lr + 32 i of the wave's
    // 128-row slab, chunk 2 ks + lane/32.  With the swizzle of lds_off() the chunk position is
    // L ^ 2 (ks ^ (i & 1)) with L a lane constant: four address registers per operand cover every
    // (ks, i); 32 i rows = an immediate offset of 4096 i bytes.
    const int lr = l & 31, ch = l >> 5;
    uint32_t ra_addr[4], rb_addr[4];
    {
        const int L = ch ^ ((lr >> 1) & 7) ^ (lr >> 4);
#pragma unroll
        for (int vi = 0; vi < 4; ++vi) {
            ra_addr[vi] = (uint32_t)((wm * 128 + lr) * 128 + ((L ^ (2 * vi)) << 4));
            rb_addr[vi] = (uint32_t)(W4_B_BASE + (wn * 128 + lr) * 128 + ((L ^ (2 * vi)) << 4));
        }
    }
    // Writes of a contraction-contiguous operand: thread holds chunk c = t % 8 of rows t / 8 + 32 i
    // (two address variants by the parity of i).  Writes of a transposed operand: thread holds the
    // 8 x 8 block (x = 8 (t % 32), k = 8 (t / 32)) and writes rows x + e (four variants by e / 2).
    constexpr int NWA = A_KC ? 2 : 4, NWB = B_KC ? 2 : 4;
    uint32_t wa_addr[NWA], wb_addr[NWB];
    {
        const int c8 = t & 7, r0 = t >> 3;
        const int Lw = c8 ^ ((r0 >> 1) & 7) ^ (r0 >> 4);
        const int tx = t & 31, kc = t >> 5;
        const int Lx = kc ^ ((tx & 1) << 2) ^ ((tx >> 1) & 3);
#pragma unroll
        for (int h = 0; h < NWA; ++h)
            wa_addr[h] = (A_KC ? (uint32_t)(r0 * 128 + ((Lw ^ (2 * h)) << 4)) : (uint32_t)(tx * 1024 + ((Lx ^ h) << 4)));
#pragma unroll
        for (int h = 0; h < NWB; ++h)
            wb_addr[h] = W4_B_BASE + (B_KC ? (uint32_t)(r0 * 128 + ((Lw ^ (2 * h)) << 4)) : (uint32_t)(tx * 1024 + ((Lx ^ h) << 4)));
    }
    // ------------------------------------------------------------------ cursors over the K-tile stream
    // left: K tiles of the cursor's C tile still to come (the current one included); odd: that C tile has
    // an odd number of K tiles, so one all-zero tile follows its last one (the loop body handles K tiles
    // in pairs); live: 0 = the cursor stands on such a zero tile, or past the end of the stream
    struct Cursor { int v, m0, n0, z, rot, g, step, kt, left, odd, live; };
    auto start = [&](Cursor& c, int v) __attribute__((always_inline)) {
        c.v = v;
        c.left = 0; c.odd = 0; c.live = 0;
        if (v >= total) return;
        int tm, tn, z;
        tile_of_id(p, v, tm, tn, z);
        c.rot = uni(p.rotate ? ((tm * 3 + tn * 5) & 7) % KT : 0);
        int g = 0;
        if (p.n_groups > 1) {
            if (p.group_along_n) { g = tn / p.group_tiles; tn -= g * p.group_tiles; }
            else                 { g = tm / p.group_tiles; tm -= g * p.group_tiles; }
        }
        c.m0 = uni(tm * W4_BM); c.n0 = uni(tn * W4_BN); c.z = uni(z); c.g = uni(g);
        const int s = z / KT;
        c.kt = uni(z - s * KT);
        c.step = uni(s + g);                      // a grouped launch has one step per group: operand slot = group
        c.left = uni((T - z + Z - 1) / Z);        // K tiles z, z + Z, ... of the n_steps x KT sequence
        c.odd = c.left & 1; c.live = 1;
    };
    Cursor f, c;                                  // fetch cursor (three K tiles ahead) and compute cursor

    // ------------------------------------------------------------------ staging registers and their operations
    // Per (C tile, step) an operand has one buffer descriptor that starts at the tile's first row (or
    // column) and ends with the operand block, so rows past a ragged edge read as zero; per K tile only
    // the lane offsets move.  (The host sends a product here only if those offsets fit 31 bits.)
    u32x4_t sa[2][8], sb[2][8];                    // two K tiles in flight through registers
    __amdgpu_buffer_rsrc_t rs_a, rs_b;
    // direct-to-LDS operands: descriptor words; lane offsets of loads 2 j and 2 j + 1 at k = 0 and for the
    // fetch cursor's K tile.  Load n of wave w brings rows 32 n + 8 w .. + 7 (1 KB of LDS); lane l holds
    // LDS position l % 8 of row 8 w + l / 8, i.e. the chunk the swizzle of lds_off() puts there, which
    // differs between even and odd n by chunk ^ 2.
    u32x4_t rw_a, rw_b;
    uint32_t dl_a[2], dl_b[2], dv_a[2], dv_b[2];
    // HYB: operand A is loaded one K tile behind the fetch cursor (its LDS stage is free only after the
    // barrier, operand B's registers a tile earlier): these hold the cursor's previous descriptor and offsets
    u32x4_t rw_l;
    uint32_t dv_l[2];
    int step_l;
    const int d_rl = w * 8 + (l >> 3);
    const int d_c0 = (l & 7) ^ ((d_rl >> 1) & 7) ^ (d_rl >> 4);
    const uint32_t s_wbase = (uint32_t)(w * 1024);
    uint32_t la_off, lb_off;                       // per-lane byte offset of load 0 at k = 0 (OOB_OFFSET: lane masked)
    uint32_t va_off[2], vb_off[2];                 // the same for the K tile whose loads are being issued, and the next
    int a_step, b_step, a_kmul, b_kmul;            // bytes between a lane's loads; bytes per unit of k
    auto open_operand = [&](auto is_a) __attribute__((always_inline)) {
        constexpr bool IS_A = decltype(is_a)::value;
        constexpr bool KC = IS_A ? A_KC : B_KC;
        const bool ok = f.live != 0;
        const int s = f.step < TP_MAX_STEPS ? f.step : TP_MAX_STEPS - 1;
        const uint16_t* ptr = uni_ptr(IS_A ? p.a[s] : p.b[s]);
        const int ld = uni(IS_A ? p.lda[s] : p.ldb[s]);
        const int X = IS_A ? p.M : p.N, x0 = IS_A ? f.m0 : f.n0;
        const int xs = (X - x0) < 256 ? (X - x0) : 256;       // rows (columns) of this tile that exist
        __amdgpu_buffer_rsrc_t rs;
        uint32_t lane;
        int step, kmul;
        if constexpr (IS_A ? DA : DB) {
            const int64_t nrec = ok ? ((int64_t)(xs - 1) * ld + p.K) * 2 : 0;
            const uint64_t base = reinterpret_cast<uint64_t>(ptr + (int64_t)x0 * ld);
            const u32x4_t rw = {(uint32_t)uni((int)(uint32_t)base), (uint32_t)uni((int)((uint32_t)(base >> 32) & 0xffffu)),
                                (uint32_t)uni((int)(uint32_t)nrec), 0x00020000u};
            if constexpr (IS_A) { rw_a = rw; a_step = uni(64 * ld); }
            else                { rw_b = rw; b_step = uni(64 * ld); }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint32_t off = (uint32_t)((d_rl * ld + (d_c0 ^ (2 * h)) * 8) * 2);
                if constexpr (IS_A) dl_a[h] = off; else dl_b[h] = off;
            }
            return;
        } else if constexpr (KC) {                 // [x][k]: chunk c = t % 8 of rows t / 8 + 32 i
            const int cc = t & 7, r0 = t >> 3;
            const int64_t nrec = ok ? ((int64_t)(xs - 1) * ld + p.K) * 2 : 0;
            rs = make_rsrc(uni_ptr(ptr + (int64_t)x0 * ld), nrec);
            lane = (uint32_t)((r0 * ld + cc * 8) * 2);
            step = 64 * ld; kmul = 2;
        } else {                                   // [k][x]: rows k + i of the 8 x 8 block at x = 8 (t % 32), k = 8 (t / 32)
            const int x = (t & 31) * 8, k = (t >> 5) * 8;
            const int64_t nrec = ok ? ((int64_t)(p.K - 1) * ld + xs) * 2 : 0;
            rs = make_rsrc(uni_ptr(ptr + x0), nrec);
            lane = x < xs ? (uint32_t)((k * ld + x) * 2) : OOB_OFFSET;
            step = 2 * ld; kmul = 2 * ld;
        }
        if constexpr (IS_A) { rs_a = rs; la_off = lane; a_step = uni(step); a_kmul = uni(kmul); }
        else                { rs_b = rs; lb_off = lane; b_step = uni(step); b_kmul = uni(kmul); }
    };
    // lane offsets of the fetch cursor's K tile, into copy Q
    auto prep_tile = [&](auto Q_) __attribute__((always_inline)) {
        constexpr int Q = decltype(Q_)::value;
        int kt = f.kt + f.rot;
        if (kt >= KT) kt -= KT;
        const int k0 = kt * BK;
        if constexpr (DA || DB) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const bool kok = (k0 + (d_c0 ^ (2 * h)) * 8) < p.K;
                if constexpr (DA) dv_a[h] = kok ? dl_a[h] + (uint32_t)(k0 * 2) : OOB_OFFSET;
                if constexpr (DB) dv_b[h] = kok ? dl_b[h] + (uint32_t)(k0 * 2) : OOB_OFFSET;
            }
        }
        if constexpr (!DA) {
            if constexpr (A_KC) va_off[Q] = (k0 + (t & 7) * 8) < p.K ? la_off + (uint32_t)(k0 * 2) : OOB_OFFSET;
            else                va_off[Q] = la_off + (uint32_t)(k0 * a_kmul);
        }
        if constexpr (!DB) {
            if constexpr (B_KC) vb_off[Q] = (k0 + (t & 7) * 8) < p.K ? lb_off + (uint32_t)(k0 * 2) : OOB_OFFSET;
            else                vb_off[Q] = lb_off + (uint32_t)(k0 * b_kmul);
        }
    };
    // Move the fetch cursor to the next K tile of the stream.  The common case (same C tile, same step)
    // is a few scalar instructions issued between two MFMAs; a change of step or of C tile needs other
    // blocks and other descriptors and is left to advance_slow() at the end of the K tile.
    bool f_reopen = false;
    auto advance_fast = [&]() __attribute__((always_inline)) {
        const int live = f.left != 0;             // past the end nothing moves: every further tile reads as zero
        f.left -= live;
        f.kt += live ? Z : 0;
        f_reopen = live && (f.left == 0 || f.kt >= KT);
    };
    auto advance_slow = [&]() __attribute__((always_inline)) {
        {
            if (f.left != 0) {                    // next step of this C tile
                do { f.kt -= KT; ++f.step; } while (f.kt >= KT);
            } else if (f.odd) {                   // the zero tile that makes the count even
                f.odd = 0; f.live = 0; f.left = 1;
            } else {
                start(f, f.v + grid);             // next C tile (or the end)
            }
            open_operand(std::true_type{});
            open_operand(std::false_type{});
        }
    };
    // n-th load of an operand into register set R
    auto load1 = [&](auto is_a, auto n_, auto R_) __attribute__((always_inline)) {
        constexpr bool IS_A = decltype(is_a)::value;
        constexpr int n = decltype(n_)::value, R = decltype(R_)::value;
        // (register set R is refilled while stage 1 - R is multiplied; the offsets of that K tile are copy
        // 1 - R, or the one copy there is when the cursor moves before the loads of a body instead of after)
        constexpr int Q = HYB ? 0 : 1 - R;
        if constexpr (IS_A) sa[R][n] = buf_load16(rs_a, va_off[Q] + (uint32_t)(n * a_step));
        else                sb[R][n] = buf_load16(rs_b, vb_off[Q] + (uint32_t)(n * b_step));
    };
    // n-th direct-to-LDS load of an operand into stage S
    auto dtl1 = [&](auto is_a, auto n_, auto S_) __attribute__((always_inline)) {
        constexpr bool IS_A = decltype(is_a)::value;
        constexpr int n = decltype(n_)::value;
        constexpr uint32_t dst = (IS_A ? 0u : (uint32_t)W4_B_BASE) + decltype(S_)::value * W4_STAGE_STRIDE + n * 4096;
        if constexpr (IS_A) dtl_load16(rw_a, dv_a[n & 1] + (uint32_t)(n * a_step), s_wbase + dst);
        else                dtl_load16(rw_b, dv_b[n & 1] + (uint32_t)(n * b_step), s_wbase + dst);
    };
    auto dtl1_lag = [&](auto n_, auto S_) __attribute__((always_inline)) {       // operand A, one K tile behind the cursor
        constexpr int n = decltype(n_)::value;
        constexpr uint32_t dst = decltype(S_)::value * W4_STAGE_STRIDE + n * 4096;
        dtl_load16(rw_l, dv_l[n & 1] + (uint32_t)(n * step_l), s_wbase + dst);
    };
    // n-th LDS write of an operand from register set R into stage S.  A transposed operand's write is
    // row x + n of its 8 x 8 block: word wd = n / 2 of the eight loaded rows, low or high halves, formed
    // by perm1 (one slot earlier) into tw_a / tw_b.
    u32x4_t tw_a, tw_b;
    auto perm1 = [&](auto is_a, auto n_, auto R_) __attribute__((always_inline)) {
        constexpr bool IS_A = decltype(is_a)::value;
        constexpr int n = decltype(n_)::value, R = decltype(R_)::value;
        constexpr int wd = n >> 1, e = n & 1;
        constexpr uint32_t sel = e ? 0x07060302u : 0x05040100u;
        const u32x4_t (&r)[8] = IS_A ? sa[R] : sb[R];
        const u32x4_t v = {__builtin_amdgcn_perm(r[1][wd], r[0][wd], sel), __builtin_amdgcn_perm(r[3][wd], r[2][wd], sel),
                           __builtin_amdgcn_perm(r[5][wd], r[4][wd], sel), __builtin_amdgcn_perm(r[7][wd], r[6][wd], sel)};
        if constexpr (IS_A) tw_a = v; else tw_b = v;
    };
    auto store1 = [&](auto is_a, auto n_, auto R_, auto S_) __attribute__((always_inline)) {
        constexpr bool IS_A = decltype(is_a)::value;
        constexpr bool KC = IS_A ? A_KC : B_KC;
        constexpr int n = decltype(n_)::value, R = decltype(R_)::value;
        constexpr int so = decltype(S_)::value * W4_STAGE_STRIDE;
        if constexpr (KC) {
            const uint32_t base = IS_A ? wa_addr[n & 1] : wb_addr[n & 1];
            lds_store16(base + (so + n * 4096), IS_A ? sa[R][n] : sb[R][n]);
        } else {
            const uint32_t base = IS_A ? wa_addr[(n >> 1) % NWA] : wb_addr[(n >> 1) % NWB];
            lds_store16(base + (so + n * 128), IS_A ? tw_a : tw_b);
        }
    };

    // ------------------------------------------------------------------ fragments and accumulators
    bf16x8_t fa[2][TM], fb[2][TN];
    f32x16_t acc[TM][TN];
    auto read_a = [&](auto ks_, auto i_, auto S_) __attribute__((always_inline)) {
        constexpr int ks = decltype(ks_)::value, i = decltype(i_)::value;
        fa[ks & 1][i] = lds_load_frag(ra_addr[(ks & 3) ^ (i & 1)] + (decltype(S_)::value * W4_STAGE_STRIDE + i * 4096));
    };
    auto read_b = [&](auto ks_, auto j_, auto S_) __attribute__((always_inline)) {
        constexpr int ks = decltype(ks_)::value, j = decltype(j_)::value;
        fb[ks & 1][j] = lds_load_frag(rb_addr[(ks & 3) ^ (j & 1)] + (decltype(S_)::value * W4_STAGE_STRIDE + j * 4096));
    };
    // first fragments (MFMA step 0) of the K tile in stage S
    auto read_first = [&](auto S_) __attribute__((always_inline)) {
        static_for<4>([&](auto i_) __attribute__((always_inline)) {
            read_a(std::integral_constant<int, 0>{}, i_, S_);
            read_b(std::integral_constant<int, 0>{}, i_, S_);
        });
    };
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
    };

    // ------------------------------------------------------------------ one K tile: 64 MFMA slots
    // k_tile<S, LAST>: multiplies the K tile in stage S, refills stage 1 - S from the staging registers
    // and reloads those with the fetch cursor's tile.  Slot s = 16 ks + 4 i + j issues MFMA (ks, i, j),
    // then whatever the tables put after it.  Fragment reads of MFMA step ks + 1 go after the even slots
    // of step ks, in the order the next step needs them (B0, A0, B1, B2, B3, A1, A2, A3); those of step
    // 0 of the NEXT K tile are read during step 3, from the other stage, after the barrier that follows
    // slot 47 -- unless this is the LAST K tile of its C tile: the epilogue comes next and wants the
    // registers, so those fragments are read after it.  The fetch cursor moves on during step 3.
    auto k_tile = [&](auto S_) __attribute__((always_inline)) {
        constexpr int S = decltype(S_)::value;
        using SR = std::integral_constant<int, S>;          // stage read
        using SW = std::integral_constant<int, 1 - S>;      // stage refilled, from register set 1 - S
        [[maybe_unused]] SR sr_unused{};
        static_for<64>([&](auto s_) __attribute__((always_inline)) {
            constexpr int s = decltype(s_)::value;
            constexpr int ks = s >> 4, i = (s >> 2) & 3, j = s & 3;
            if constexpr (s == 48) {
                // every LDS write of this K tile was issued before here; after the barrier the other
                // stage is complete, and nobody reads the current one any more (the step-3 fragments
                // were requested during step 2 and have arrived: the barrier waits for them)
                // this wave's direct-to-LDS loads of the next K tile have landed (HYB: all but this body's
                // eight register loads, which are younger)
                if constexpr (DTL) wait_vm<0>();
                if constexpr (HYB) wait_vm<8>();
                __syncthreads();
            }
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks & 1][j], fa[ks & 1][i], acc[i][j], 0, 0, 0);
            if constexpr ((s & 1) == 0) {
                constexpr int n = (s & 15) >> 1;
                using KN = std::integral_constant<int, ks + 1>;
                using ST = std::integral_constant<int, ks == 3 ? 1 - S : S>;
                if constexpr (n == 0)      read_b(KN{}, std::integral_constant<int, 0>{}, ST{});
                else if constexpr (n == 1) read_a(KN{}, std::integral_constant<int, 0>{}, ST{});
                else if constexpr (n <= 4) read_b(KN{}, std::integral_constant<int, n - 1>{}, ST{});
                else                       read_a(KN{}, std::integral_constant<int, n - 4>{}, ST{});
            }
            if constexpr (DTL) {
                // The K tile at the fetch cursor: operand B during MFMA step 0 (into the stage being
                // refilled), then the cursor moves on, and after the barrier operand A of the following
                // K tile goes into the stage this body has just finished reading.
                if constexpr ((s & 1) == 1 && s < 16) dtl1(std::false_type{}, std::integral_constant<int, s / 2>{}, SW{});
                if constexpr ((s & 1) == 1 && s > 48) dtl1(std::true_type{}, std::integral_constant<int, (s - 49) / 2>{}, SR{});
                if constexpr (s == 38) advance_fast();
                if constexpr (s == 40) { if (f_reopen) advance_slow(); }
                if constexpr (s == 42) prep_tile(SW{});
            }
            if constexpr (HYB) {
                // The cursor moves first (operand A's descriptor and offsets of the tile it leaves are kept:
                // that tile's A loads come last in this body), then operand B: out of its registers into the
                // stage being refilled, and the cursor's K tile into those registers.
                if constexpr (s == 2) {
                    rw_l = rw_a; step_l = a_step; dv_l[0] = dv_a[0]; dv_l[1] = dv_a[1];
                    advance_fast();
                }
                if constexpr (s == 4) { if (f_reopen) advance_slow(); }
                if constexpr (s == 6) prep_tile(std::integral_constant<int, 0>{});
                static_for<8>([&](auto n_) __attribute__((always_inline)) {
                    constexpr int n = decltype(n_)::value;
                    if constexpr (SB.pm[n] == s) perm1(std::false_type{}, n_, SW{});
                    if constexpr (SB.wr[n] == s) store1(std::false_type{}, n_, SW{}, SW{});
                    if constexpr (SB.ld[n] == s) load1(std::false_type{}, n_, SW{});
                });
                if constexpr ((s & 1) == 1 && s > 48) dtl1_lag(std::integral_constant<int, (s - 49) / 2>{}, SR{});
            }
            if constexpr (!DA) static_for<8>([&](auto n_) __attribute__((always_inline)) {
                constexpr int n = decltype(n_)::value;
                if constexpr (!A_KC && SA.pm[n] == s) perm1(std::true_type{}, n_, SW{});
                if constexpr (!B_KC && SB.pm[n] == s) perm1(std::false_type{}, n_, SW{});
                if constexpr (SA.wr[n] == s) store1(std::true_type{}, n_, SW{}, SW{});
                if constexpr (SB.wr[n] == s) store1(std::false_type{}, n_, SW{}, SW{});
                if constexpr (SA.ld[n] == s) load1(std::true_type{}, n_, SW{});
                if constexpr (SB.ld[n] == s) load1(std::false_type{}, n_, SW{});
            });
            // the fetch cursor moves on to the K tile the NEXT body loads, and that tile's lane offsets go
            // into the other copy; descriptors stay as they are until this tile's last load has been issued
            if constexpr (!DA && s == 3) advance_fast();
            if constexpr (!DA && s == 9) prep_tile(SW{});
            __builtin_amdgcn_sched_barrier(0);
        });
        if constexpr (!DA) {
            if (f_reopen) {
                advance_slow();
                prep_tile(SW{});
            }
        }
    };

    // ------------------------------------------------------------------ epilogue of the compute cursor's C tile
    // acc[i][j][e]: row m = 32 i + lane%32, columns n = 32 j + 8 (e/4) + 4 (lane/32) + e%4.
    // No branch depends on a lane: every global access goes through a buffer descriptor that starts at
    // the first row of this wave's 128 x 128 block and ends with the last row of the matrix, so rows
    // below a ragged edge are dropped by the range check, and a lane whose columns lie beyond N carries
    // an out-of-range offset.  One slab = 32 rows x 128 columns passes through the wave's LDS patch so
    // that stores are whole row segments.
    auto epilogue = [&]() __attribute__((always_inline)) {
        const int m_sub = c.m0 + wm * 128, n_sub = c.n0 + wn * 128;
        const int r = lr;
        const bool partial = Z > 1;          // split K: raw fp32 partials, the fix-up kernel runs the epilogue
        constexpr bool use_bias = EPI == EPI_BIAS || EPI == EPI_BIAS_GELU;
        constexpr bool use_gelu = EPI == EPI_BIAS_GELU;
        constexpr bool use_dg = EPI == EPI_MUL_DGELU;
        const bool use_pre = !use_dg && p.pre != nullptr;
        const int rows_left = p.M - m_sub;
        // rows m_sub .. M - 1 of a matrix with leading dimension ld (elements of es bytes), N columns
        auto block_rsrc = [&](const void* base, int64_t ld, int es) __attribute__((always_inline)) {
            const int64_t nrec = rows_left > 0 ? ((int64_t)(rows_left - 1) * ld + p.N) * es : 0;
            return make_rsrc(uni_ptr(static_cast<const char*>(base) + (int64_t)m_sub * ld * es), nrec);
        };
        u32x2_t bias_v[TN][4];
        if constexpr (use_bias) {
            const __amdgpu_buffer_rsrc_t rs_bias = make_rsrc(uni_ptr(p.bias), (int64_t)p.N * 2);
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const u32x2_t b = __builtin_amdgcn_raw_buffer_load_b64(rs_bias, (n_sub + 32 * j + 8 * g + 4 * ch) * 2, 0, 0);
                    bias_v[j][g] = b;
                }
        }
        __amdgpu_buffer_rsrc_t rs_dg;
        uint32_t dg_lane = 0;
        if constexpr (use_dg) {
            rs_dg = block_rsrc(p.dg, p.lddg, 2);
            dg_lane = (uint32_t)((r * (int)p.lddg + n_sub + 4 * ch) * 2);   // columns past N: the next row's values or zeros, never stored
        }
        // The accumulators stay where the MFMAs keep them (the accumulator half of the register file) and
        // are fetched four at a time, where they are used: left to itself the compiler copies all 256 out
        // at once, which cannot fit beside the staging registers.
        auto raw4 = [&](int i, int j, int g, float (&v)[4]) __attribute__((always_inline)) {
#pragma unroll
            for (int e = 0; e < 4; ++e) asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v[e]) : "a"(acc[i][j][4 * g + e]));
        };
        auto preact4 = [&](int i, int j, int g, float (&v)[4]) __attribute__((always_inline)) {
            raw4(i, j, g, v);
            if constexpr (use_bias) {
                const u32x2_t b = bias_v[j][g];
                v[0] += bf16_lo(b[0]); v[1] += bf16_hi(b[0]); v[2] += bf16_lo(b[1]); v[3] += bf16_hi(b[1]);
            }
        };
        u32x2_t dg_v[TN][4];
        auto load_dg = [&](int i) __attribute__((always_inline)) {
            if constexpr (use_dg) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int g = 0; g < 4; ++g)
                        dg_v[j][g] = __builtin_amdgcn_raw_buffer_load_b64(rs_dg, dg_lane + (uint32_t)(((32 * i) * (int)p.lddg + 32 * j + 8 * g) * 2), 0, 0);
            }
        };
        auto final4 = [&](int i, int j, int g, float (&v)[4]) __attribute__((always_inline)) {
            preact4(i, j, g, v);
            if constexpr (use_gelu) {
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = gelu_f(v[e]);
            }
            if constexpr (use_dg) {
                const u32x2_t a = dg_v[j][g];
                v[0] *= dgelu_f(bf16_lo(a[0])); v[1] *= dgelu_f(bf16_hi(a[0]));
                v[2] *= dgelu_f(bf16_lo(a[1])); v[3] *= dgelu_f(bf16_hi(a[1]));
            }
        };
        // bf16 slab of 32 rows x 128 columns: rows of 256 bytes in the patch; a lane writes 8 bytes and
        // reads back 16 (chunk index XOR row keeps both conflict-free), stores are 256-byte row segments:
        // lane l stores columns 8 (l % 16) .. + 7 of rows l / 16 + 4 it
        auto slab_bf16 = [&](int i, auto value4, __amdgpu_buffer_rsrc_t rs, int ld) __attribute__((always_inline)) {
            const uint32_t lane = (n_sub + 8 * (l & 15)) < p.N ? (uint32_t)(((l >> 4) * ld + n_sub + 8 * (l & 15)) * 2) : OOB_OFFSET;
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float x[4];
                    value4(i, j, g, x);
                    const u32x2_t v = {pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3])};
                    *reinterpret_cast<u32x2_t*>(eps + r * 256 + (((4 * j + g) ^ (r & 15)) << 4) + 8 * ch) = v;
                }
#pragma unroll
            for (int it = 0; it < 8; ++it) {
                const int rr = it * 4 + (l >> 4), cc = l & 15;
                const u32x4_t v = *reinterpret_cast<const u32x4_t*>(eps + rr * 256 + ((cc ^ (rr & 15)) << 4));
                __builtin_amdgcn_raw_buffer_store_b128(v, rs, (int)(lane + (uint32_t)((32 * i + 4 * it) * ld * 2)), 0, 0);
            }
        };
        // fp32 slab, one 32-column block at a time: rows of 128 bytes; lane l stores columns
        // 4 (l % 8) .. + 3 of rows l / 8 + 8 it
        auto slab_f32 = [&](int i, auto value4, __amdgpu_buffer_rsrc_t rs, int ld) __attribute__((always_inline)) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const int n = n_sub + 32 * j + 4 * (l & 7);
                const uint32_t lane = n < p.N ? (uint32_t)(((l >> 3) * ld + n) * 4) : OOB_OFFSET;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float x[4];
                    value4(i, j, g, x);
                    const f32x4_t v = {x[0], x[1], x[2], x[3]};
                    *reinterpret_cast<f32x4_t*>(eps + r * 128 + (((2 * g + ch) ^ ((r >> 1) & 7)) << 4)) = v;
                }
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int rr = it * 8 + (l >> 3), cc = l & 7;
                    const u32x4_t v = *reinterpret_cast<const u32x4_t*>(eps + rr * 128 + ((cc ^ ((rr >> 1) & 7)) << 4));
                    __builtin_amdgcn_raw_buffer_store_b128(v, rs, (int)(lane + (uint32_t)((32 * i + 8 * it) * ld * 4)), 0, 0);
                }
            }
        };
        // The loads of the K tile after next are in flight.  Loads and stores complete out of order
        // with respect to each other, so a wait for those loads issued after the first store would
        // have to wait for every store as well: take the loads in before the first store instead.
        // (Direct-to-LDS loads feed no register: nothing to take in; HYB issued eight of them last.)
        if constexpr (HYB) wait_vm<8>();
        else if constexpr (!DTL) wait_vm<0>();
        // (the last MFMA's result is read by hand-placed instructions: give it the 19 cycles it needs)
        asm volatile("s_nop 7\n\ts_nop 7\n\ts_nop 7" ::: "memory");
        if (partial) {
            const __amdgpu_buffer_rsrc_t rs_ws = block_rsrc(p.ws + ((int64_t)c.z * p.n_groups + c.g) * p.M * p.N, (int64_t)p.N, 4);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                slab_f32(i, raw4, rs_ws, p.N);
                __builtin_amdgcn_sched_barrier(0);
            }
        } else {
            const int ldo = (int)p.ldos[c.g];
            const __amdgpu_buffer_rsrc_t rs_out = block_rsrc(p.outs[c.g], ldo, F32_OUT ? 4 : 2);
            __amdgpu_buffer_rsrc_t rs_pre;
            if constexpr (!use_dg) rs_pre = block_rsrc(p.pre, p.ldp, 2);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                load_dg(i);
                if constexpr (!use_dg) {
                    if (use_pre) slab_bf16(i, preact4, rs_pre, (int)p.ldp);
                }
                if constexpr (F32_OUT) slab_f32(i, final4, rs_out, ldo);
                else                   slab_bf16(i, final4, rs_out, ldo);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // ------------------------------------------------------------------ the stream
    start(f, (int)blockIdx.x);
    if (f.left == 0) return;
    c = f;
    open_operand(std::true_type{});
    open_operand(std::false_type{});
    // K tile 0 -> register set 0 -> stage 0;  K tile 1 -> set 1;  K tile 2 -> set 0
    // (loads and writes in the order the loop body uses: the first operand's eight, then the other's)
    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, 1>;
    auto move_on = [&](auto Q_) __attribute__((always_inline)) {
        advance_fast();
        if (f_reopen) advance_slow();
        prep_tile(Q_);
    };
    auto load_all = [&](auto R_) __attribute__((always_inline)) {
        static_for<8>([&](auto n_) __attribute__((always_inline)) { load1(std::integral_constant<bool, A_FIRST>{}, n_, R_); });
        static_for<8>([&](auto n_) __attribute__((always_inline)) { load1(std::integral_constant<bool, !A_FIRST>{}, n_, R_); });
    };
    if constexpr (DTL) {
        // K tile 0 -> stage 0 (both operands), operand A of K tile 1 -> stage 1; operand B of K tile 1 is the
        // first thing the loop body loads
        prep_tile(S0{});
        static_for<8>([&](auto n_) __attribute__((always_inline)) { dtl1(std::true_type{}, n_, S0{}); });
        static_for<8>([&](auto n_) __attribute__((always_inline)) { dtl1(std::false_type{}, n_, S0{}); });
        move_on(S0{});
        static_for<8>([&](auto n_) __attribute__((always_inline)) { dtl1(std::true_type{}, n_, S1{}); });
        wait_vm<8>();
    } else if constexpr (HYB) {
        // K tile 0: A -> stage 0, B -> register set 0 -> stage 0;  K tile 1: A -> stage 1, B -> set 1;
        // K tile 2: B -> set 0 (its A is the first body's business).  The cursor stays on K tile 2.
        using Q0 = std::integral_constant<int, 0>;
        prep_tile(Q0{});
        static_for<8>([&](auto n_) __attribute__((always_inline)) { dtl1(std::true_type{}, n_, S0{}); });
        static_for<8>([&](auto n_) __attribute__((always_inline)) { load1(std::false_type{}, n_, S0{}); });
        move_on(Q0{});
        static_for<8>([&](auto n_) __attribute__((always_inline)) { dtl1(std::true_type{}, n_, S1{}); });
        static_for<8>([&](auto n_) __attribute__((always_inline)) { load1(std::false_type{}, n_, S1{}); });
        static_for<8>([&](auto n_) __attribute__((always_inline)) {
            perm1(std::false_type{}, n_, S0{});
            store1(std::false_type{}, n_, S0{}, S0{});
        });
        move_on(Q0{});
        static_for<8>([&](auto n_) __attribute__((always_inline)) { load1(std::false_type{}, n_, S0{}); });
        wait_vm<24>();                             // operand A of K tile 0 is the oldest of the 40 loads
    } else {
    prep_tile(S1{});
    load_all(S0{});                                // (set 0 takes its offsets from copy 1, set 1 from copy 0)
    move_on(S0{});
    load_all(S1{});
    static_for<8>([&](auto n_) __attribute__((always_inline)) {
        using FA = std::integral_constant<bool, A_FIRST>;
        if constexpr (!(A_FIRST ? A_KC : B_KC)) perm1(FA{}, n_, S0{});
        store1(FA{}, n_, S0{}, S0{});
    });
    static_for<8>([&](auto n_) __attribute__((always_inline)) {
        using FB = std::integral_constant<bool, !A_FIRST>;
        if constexpr (!(A_FIRST ? B_KC : A_KC)) perm1(FB{}, n_, S0{});
        store1(FB{}, n_, S0{}, S0{});
    });
    move_on(S1{});
    load_all(S0{});
    move_on(S0{});                                 // the first loop body (stage 0) refills set 1 from copy 0
    }
    __syncthreads();
    read_first(S0{});

    while (true) {
        zero_acc();
        for (int n = c.left + c.odd; n > 0; n -= 2) {
            k_tile(S0{});
            k_tile(S1{});
        }
        epilogue();
        start(c, c.v + grid);
        if (c.left == 0) break;
    }
}

// ---------------------------------------------------------------------------------------------
// host launcher
// ---------------------------------------------------------------------------------------------
template <bool A_KC, bool B_KC, int EPI, bool F32_OUT>
static hipError_t launch4_one(const GemmArgs& a, hipStream_t stream) {
    static std::atomic<uint64_t> attr_done{0};
    int dev = 0;
    if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
    const uint64_t bit = 1ull << (dev & 63);
    if (!(attr_done.load(std::memory_order_relaxed) & bit)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&tp_gemm4_kernel<A_KC, B_KC, EPI, F32_OUT>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, W4_LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done.fetch_or(bit, std::memory_order_relaxed);
    }
    const int total = a.tiles_m * a.tiles_n * a.split_k;
    const unsigned grid = (unsigned)(total < a.max_workgroups ? total : a.max_workgroups);
    return launch_kernel(tp_gemm4_kernel<A_KC, B_KC, EPI, F32_OUT>, dim3(grid), dim3(W4_THREADS), W4_LDS_BYTES, stream, a);
}

hipError_t launch_gemm4(int form, const GemmArgs& a, hipStream_t s) {
    const int epi = a.split_k > 1 ? EPI_NONE : (a.dg ? EPI_MUL_DGELU : (a.gelu ? EPI_BIAS_GELU : (a.bias ? EPI_BIAS : EPI_NONE)));
    const bool f32 = a.split_k > 1 || a.out_f32;
    switch (form) {
        case FORM_NN:
            if (epi == EPI_BIAS_GELU) return f32 ? launch4_one<true, false, EPI_BIAS_GELU, true>(a, s) : launch4_one<true, false, EPI_BIAS_GELU, false>(a, s);
            if (epi == EPI_BIAS)      return f32 ? launch4_one<true, false, EPI_BIAS, true>(a, s) : launch4_one<true, false, EPI_BIAS, false>(a, s);
            if (epi == EPI_NONE)      return f32 ? launch4_one<true, false, EPI_NONE, true>(a, s) : launch4_one<true, false, EPI_NONE, false>(a, s);
            return hipErrorInvalidValue;
        case FORM_NT:
            if (epi == EPI_MUL_DGELU) return f32 ? launch4_one<true, true, EPI_MUL_DGELU, true>(a, s) : launch4_one<true, true, EPI_MUL_DGELU, false>(a, s);
            if (epi == EPI_NONE)      return f32 ? launch4_one<true, true, EPI_NONE, true>(a, s) : launch4_one<true, true, EPI_NONE, false>(a, s);
            return hipErrorInvalidValue;
        case FORM_TN:
            if (epi == EPI_NONE && f32) return launch4_one<false, false, EPI_NONE, true>(a, s);
            return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

}  // namespace tpl
