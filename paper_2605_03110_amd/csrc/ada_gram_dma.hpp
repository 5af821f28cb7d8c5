// k_gram_dma: the lower-triangular Gram of the full selection (Definition "Gram threshold", Section 2.1) for bf16
// rows that can be fetched in whole 64-byte pieces.  Included by ada_kernels.hip after the tile helpers.
//
// What bounds this kernel is the rate at which a CU can pull operands out of the L2: about 25 bytes per clock per CU
// when all 256 CUs pull at once (45 when few do), against an MFMA rate that consumes 128 (a + b) bytes per a b / 32
// clocks for an a x b tile.  A 128 x 256 tile needs 47 B/clk and is L2-bound at half the MFMA rate; 256 x 256 needs 32.
// So a workgroup is four wavefronts in a 2 x 2 grid, one per SIMD, each holding a 128 x 128 accumulator (256
// registers), which is the largest square the register file allows.  Operands go global -> LDS directly
// (global_load_lds, 16 bytes per lane) in half chunks of 32 elements: 512 rows x 64 bytes = 32 KB per stage, a ring of
// four stages, three half chunks in flight while one is multiplied; waits are counted by hand and the barrier is the
// bare instruction, because a fenced barrier would drain the loads.
//
// Work units.  Off-diagonal 256 x 256 blocks of the triangle are "big" units.  A diagonal 256-block would waste a
// quarter of its MFMAs on s > t, and 256-blocks quantise badly (T = 8192: 528 blocks on 256 CUs), so each diagonal
// block is cut into three 128 x 128 "small" units (the same code with 64 x 64 per wave).  For mid-sized T, where
// 256-blocks cannot fill the chip, the whole triangle is cut into small units.  Units are handed out big first: the
// first one by workgroup id (a contiguous range per XCD, so neighbours share rows in that XCD's L2), the rest from an
// atomic counter, which packs the short units into the tail.  The counter and the sign-off tickets (counted per XCD
// first, as in the cascade step) live in the workspace and are zero between launches: the last workgroup to leave
// resets them.
#pragma once

struct DmaGeom {
    static constexpr int THREADS = 256, NS = 4;
    static constexpr int HC = 32;                              // elements per half chunk (64 bytes of bf16)
    static constexpr int STAGE = 512 * 64;                     // bytes per ring stage at the big tile
    static constexpr int META = 4 * 256 * 4;                   // s_tok, t_tok, s_scale, t_scale
    static constexpr int LDS = META + NS * STAGE;              // 132 KB: one workgroup per CU
};

#ifdef ADA_PHASE_CLOCKS
// (constant-rate 100 MHz counter; the stamps of the last unit a workgroup ran stay)
#define DMA_CLK(i) do { if (threadIdx.x == 0) { const unsigned long long t_ = __builtin_amdgcn_s_memrealtime(); \
    if (blockIdx.x == (ADA_PHASE_CLOCKS)) g_phase_clk[(i) + 48] = t_; if ((i) < 8) g_pass_clk[(blockIdx.x & 511) * 8 + (i)] = t_; } } while (0)
#define DMA_CLK_ANY(i) do { if (threadIdx.x == 0) g_phase_clk[(i) + 48] = __builtin_amdgcn_s_memrealtime(); } while (0)
#else
#define DMA_CLK(i) do { } while (0)
#define DMA_CLK_ANY(i) do { } while (0)
#endif

// One WM*2 x WM*2 tile: "against" rows s0.. on the MFMA M side, tested rows t0.. on the N side; the rows' inverse norms
// come from p.inv_norm.
template <int WM>
__device__ inline void gram_tile_dma(const GramParams& p, int s0, int t0, bool need_order, char* lds) {
    using G = DmaGeom;
    constexpr int BT = 2 * WM, ROWS = 2 * BT, NB = WM / 32, LPT = ROWS / 64, NS = G::NS, HC = G::HC;
    constexpr int STAGE = ROWS * 64;
    int* s_tok = reinterpret_cast<int*>(lds);
    int* t_tok = s_tok + BT;
    float* s_scale = reinterpret_cast<float*>(t_tok + BT);
    float* t_scale = s_scale + BT;
    char* ring = lds + G::META;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, half = lane >> 5;
    const int ws = wave >> 1, wt = wave & 1;
    DMA_CLK(4);
    const int T = p.T;
    const uint16_t* X = reinterpret_cast<const uint16_t*>(p.X);

    for (int i = tid; i < ROWS; i += G::THREADS) {
        const bool isS = i < BT;
        const int tok = isS ? s0 + i : t0 + (i - BT);
        const bool ok = tok < T;
        const float sc = ok ? p.inv_norm[ok ? tok : 0] : 0.f;
        if (isS) { s_tok[i] = ok ? tok : INT_MAX; s_scale[i] = sc; }
        else { t_tok[i - BT] = ok ? tok : -1; t_scale[i - BT] = sc; }
    }

    // Stage layout: rows of 64 bytes = 4 pieces; piece c of row r sits at slot c ^ ((r >> 2) & 3).  Sixteen lanes that
    // read the same piece of 16 consecutive rows then cover one whole 256-byte bank row (rows with equal r % 4 share
    // bank columns and get four different slots).  One load instruction fills 1 KB = 16 rows; lane l serves row
    // l / 4, slot l % 4 and therefore fetches piece (l % 4) ^ ((l / 16) % 4).  Rows past the end re-read row T - 1.
    const uint16_t* rowp[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int row = (j * 4 + wave) * 16 + (lane >> 2);
        const int tok = min(row < BT ? s0 + row : t0 + (row - BT), T - 1);
        rowp[j] = X + (size_t)tok * (size_t)p.ld + (((lane & 3) ^ ((lane >> 4) & 3)) << 3);
    }
    const int nh = p.d / HC;
    auto issue = [&](int stage_off, int h) {
        const int hc = min(h, nh - 1);                         // surplus issues repeat the last half chunk into a dead stage
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            char* dst = ring + stage_off + (j * 4 + wave) * 1024;               // wave-uniform
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(rowp[j] + hc * HC),
                                             (void __attribute__((address_space(3)))*)dst, 16, 0, 0);
        }
    };

    f32x16 acc[NB][NB];
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // lane part of a fragment address for k-step ks of a half chunk: row l32 of a 32-row block, piece 2 ks + half
    const int lo0 = l32 * 64 + (((0 + half) ^ ((l32 >> 2) & 3)) << 4);
    const int lo1 = l32 * 64 + (((2 + half) ^ ((l32 >> 2) & 3)) << 4);
    const char* abase = ring + (ws * WM) * 64;
    const char* bbase = ring + (BT + wt * WM) * 64;
    u32x4 fa[2][NB], fb[2][NB];
    auto read_frags = [&](int set, int stage_off, int ks) {
        const int lo = ks ? lo1 : lo0;
#pragma unroll
        for (int a = 0; a < NB; ++a) fa[set][a] = *reinterpret_cast<const u32x4*>(abase + stage_off + a * 2048 + lo);
#pragma unroll
        for (int b = 0; b < NB; ++b) fb[set][b] = *reinterpret_cast<const u32x4*>(bbase + stage_off + b * 2048 + lo);
    };
    auto mma = [&](int set) {
#pragma unroll
        for (int a = 0; a < NB; ++a)
#pragma unroll
            for (int b = 0; b < NB; ++b) Mfma<uint16_t>::run(acc[a][b], fa[set][a], fb[set][b]);
    };

    // Half step h multiplies half chunk h (two k-steps of 16).  With one wave per SIMD nothing else hides latency, so
    // the order is fixed by hand: the fragments of k-step 1 are read while k-step 0 multiplies; then the barrier that
    // opens half chunk h + 1, the fragment reads of its k-step 0 and the loads of half chunk h + 4 (into the stage
    // everybody has just left) are issued in the shadow of k-step 1's MFMAs, one load per MFMA.
    auto step = [&](int cur_off, int nxt_off, int h) {
        __builtin_amdgcn_sched_barrier(0);
        read_frags(1, cur_off, 1);
        mma(0);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(2 * LPT));   // h + 1 has landed; my reads of this stage have returned
        __builtin_amdgcn_s_barrier();
        read_frags(0, nxt_off, 0);
        issue(cur_off, h + 4);
        mma(1);
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * NB, 0);  // the LDS reads first
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // then one MFMA ...
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // ... per global load
        }
        if constexpr (NB * NB > LPT) __builtin_amdgcn_sched_group_barrier(0x008, NB * NB - LPT, 0);
    };
    issue(0 * STAGE, 0);
    issue(1 * STAGE, 1);
    issue(2 * STAGE, 2);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(2 * LPT));     // half chunk 0 has landed (this wave's part)
    __builtin_amdgcn_s_barrier();
    issue(3 * STAGE, 3);
    read_frags(0, 0, 0);
    DMA_CLK(0);
    int h = 0;
    for (; h + NS < nh; h += NS) {                             // every step here has a successor: no branches inside
#pragma unroll
        for (int s = 0; s < NS; ++s) step(s * STAGE, ((s + 1) % NS) * STAGE, h + s);
    }
    for (; h + 1 < nh; ++h) step((h % NS) * STAGE, ((h + 1) % NS) * STAGE, h);
    __builtin_amdgcn_sched_barrier(0);
    read_frags(1, (h % NS) * STAGE, 1);                        // last half chunk
    mma(0);
    mma(1);
    DMA_CLK(1);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));           // surplus loads land before the ring is reused
    __syncthreads();
    DMA_CLK(2);

    uint32_t* gamma_bits = reinterpret_cast<uint32_t*>(p.gamma);
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int nl = wt * WM + b * 32 + l32;
        const int ttok = t_tok[nl];
        float m = 0.f;
#pragma unroll
        for (int a = 0; a < NB; ++a)
            m = fmaxf(m, block_max(acc[a][b], s_scale, s_tok, ws * WM + a * 32, half, need_order, ttok));
        publish_max(m, t_scale[nl], ttok, half, gamma_bits);
        if (p.hits) {                                              // greedy covering: one bit per pair s < t as well
#pragma unroll
            for (int a = 0; a < NB; ++a)
                publish_hits(acc[a][b], s_scale, s_tok, ws * WM + a * 32, half, need_order, ttok, t_scale[nl], p.thr,
                             p.hits, T, s0 + ws * WM + a * 32);
        }
    }
    DMA_CLK(3);
}

// ---- the one-launch form (T <= 4096, d a multiple of 64): tiles with few MFMAs per load ----------------------------
// Eight waves, four loaders and four multipliers in a 2 x 2 grid of WA x WB blocks (split_loader / split_multiplier, the
// scheme of the cascade step's large tiles), four stages of whole 128-byte chunks.
// The rows' sums of squares (Section 2.1) come from the fragments in hand instead of a pass of their own: a 32-row
// block is held by two waves, each wave sums the blocks at its even local positions, and the local order of a wave's
// blocks is permuted (block a ^ parity) so that those positions cover every block and the K loop stays straight-line
// code (a side with one block per wave is summed by both of its waves, which write the same bits).
struct SplitGeom {
    static constexpr int THREADS = 512, NS = 4, EPC = SPLIT_EPC;
};

// One (2 WA) x (2 WB) tile: "against" rows s0.. on the MFMA M side, tested rows t0.. on the N side.
template <int WA, int WB>
__device__ inline void gram_tile_split(const GramParams& p, int s0, int t0, bool need_order, char* lds) {
    using G = DmaGeom;
    constexpr int BS = 2 * WA, BT = 2 * WB, ROWS = BS + BT, NA = WA / 32, NB = WB / 32;
    constexpr int LPT = ROWS / 32, STAGE = ROWS * 128;
    static_assert(ROWS % 32 == 0 && SplitGeom::NS * STAGE <= G::NS * G::STAGE && 2 * (BS + BT) * 4 <= G::META,
                  "ring and tables fit");
    int* s_tok = reinterpret_cast<int*>(lds);
    int* t_tok = s_tok + BS;
    float* s_scale = reinterpret_cast<float*>(t_tok + BT);
    float* t_scale = s_scale + BS;
    char* ring = lds + G::META;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave8 >= 4;
    const int wave = wave8 & 3;                                // place among the waves of its kind
    const int l32 = lane & 31, half = lane >> 5;
    const int ws = wave >> 1, wt = wave & 1;
    DMA_CLK(4);
    const int T = p.T;
    for (int i = tid; i < BS + BT; i += SplitGeom::THREADS) {
        const bool isS = i < BS;
        const int tok = isS ? s0 + i : t0 + (i - BS);
        const bool ok = tok < T;
        if (isS) { s_tok[i] = ok ? tok : INT_MAX; s_scale[i] = 0.f; }
        else { t_tok[i - BS] = ok ? tok : -1; t_scale[i - BS] = 0.f; }
    }
    f32x16 acc[NA][NB];
    // local block a of this wave is block a ^ pa of its NA "against" blocks, likewise b ^ pb for the tested blocks
    const int pa = NA > 1 ? wt : 0, pb = NB > 1 ? ws : 0;
    constexpr int DA = (NA + 1) / 2, DB = (NB + 1) / 2;       // blocks a wave sums on each side
    float ssa[DA], ssb[DB];
    if (loader) {
        // rows past the end re-read row T - 1 (and are never published)
        split_loader<SplitGeom::NS, LPT, STAGE>(reinterpret_cast<const uint16_t*>(p.X), p.ld, p.d, ring, wave, lane,
            [&](int, int row) { return min(row < BS ? s0 + row : t0 + (row - BS), T - 1); });
    } else {
#pragma unroll
        for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
#pragma unroll
        for (int i = 0; i < DA; ++i) ssa[i] = 0.f;
#pragma unroll
        for (int i = 0; i < DB; ++i) ssb[i] = 0.f;
        // fragment addresses: row l32 of a 32-row block, piece 2 ks + half of the chunk (k-step ks of four)
        const char* aptr[4][NA];
        const char* bptr[4][NB];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
            for (int a = 0; a < NA; ++a) aptr[ks][a] = ring + lds_off(ws * WA + (a ^ pa) * 32 + l32, 2 * ks + half);
#pragma unroll
            for (int b = 0; b < NB; ++b) bptr[ks][b] = ring + lds_off(BS + wt * WB + (b ^ pb) * 32 + l32, 2 * ks + half);
        }
        u32x4 fa[2][NA], fb[2][NB];
        DMA_CLK(0);
        split_multiplier<SplitGeom::NS, STAGE>(p.d / SplitGeom::EPC,
            [&](int set, int stage_off, int ks) {
#pragma unroll
                for (int a = 0; a < NA; ++a) fa[set][a] = *reinterpret_cast<const u32x4*>(aptr[ks][a] + stage_off);
#pragma unroll
                for (int b = 0; b < NB; ++b) fb[set][b] = *reinterpret_cast<const u32x4*>(bptr[ks][b] + stage_off);
            },
            [&](int set) {
#pragma unroll
                for (int a = 0; a < NA; ++a)
#pragma unroll
                    for (int b = 0; b < NB; ++b) Mfma<uint16_t>::run(acc[a][b], fa[set][a], fb[set][b]);
#pragma unroll
                for (int i = 0; i < NA; i += 2) ssa[i >> 1] += piece_sumsq_fast<uint16_t>(fa[set][i]);
#pragma unroll
                for (int i = 0; i < NB; i += 2) ssb[i >> 1] += piece_sumsq_fast<uint16_t>(fb[set][i]);
            });
    }
    DMA_CLK(1);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));           // surplus loads land before the ring is reused
    __syncthreads();
    DMA_CLK(2);
    if (!loader) {
        // the two lane halves hold different k pieces; rows that do not exist keep scale 0
#pragma unroll
        for (int i = 0; i < DA; ++i) {
            const float va = ssa[i] + __shfl_xor(ssa[i], 32, 64);
            const int ra = ws * WA + ((2 * i) ^ pa) * 32 + l32;
            if (half == 0) s_scale[ra] = (s_tok[ra] != INT_MAX && va > 0.f) ? 1.0f / sqrtf(va) : 0.f;   // a zero row normalises to zero
        }
#pragma unroll
        for (int i = 0; i < DB; ++i) {
            const float vb = ssb[i] + __shfl_xor(ssb[i], 32, 64);
            const int rb = wt * WB + ((2 * i) ^ pb) * 32 + l32;
            if (half == 0) t_scale[rb] = (t_tok[rb] >= 0 && vb > 0.f) ? 1.0f / sqrtf(vb) : 0.f;
        }
    }
    __syncthreads();
    if (loader) return;                                        // (no barrier follows inside the tile)
    uint32_t* gamma_bits = reinterpret_cast<uint32_t*>(p.gamma);
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int nl = wt * WB + (b ^ pb) * 32 + l32;
        const int ttok = t_tok[nl];
        float m = 0.f;
#pragma unroll
        for (int a = 0; a < NA; ++a)
            m = fmaxf(m, block_max(acc[a][b], s_scale, s_tok, ws * WA + (a ^ pa) * 32, half, need_order, ttok));
        publish_max(m, t_scale[nl], ttok, half, gamma_bits);
    }
    DMA_CLK(3);
}

// A 128-token block ON the diagonal: its rows are staged once, and of its sixteen 32 x 32 blocks only the ten with
// "against" block <= tested block are multiplied, three per wave and k-step instead of four: wave 0 holds (0,0), (0,1),
// (1,1), wave 1 holds (2,2), (2,3), (3,3), wave 2 holds (0,2), (0,3) and wave 3 holds (1,2), (1,3).  Written as one code
// path: four fragments P, Q, R, S per wave and the products P x Q, P x R, S x R (the third is idle work in waves 2
// and 3).
__device__ inline void gram_tile_diag(const GramParams& p, int t0, char* lds) {
    using G = DmaGeom;
    constexpr int ROWS = 128, LPT = ROWS / 32, STAGE = ROWS * 128;
    int* s_tok = reinterpret_cast<int*>(lds);                  // INT_MAX past the end (never "earlier")
    int* t_tok = s_tok + ROWS;                                 // -1 past the end (never published)
    float* scale = reinterpret_cast<float*>(t_tok + ROWS);
    char* ring = lds + G::META;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave8 >= 4;
    const int wave = wave8 & 3;
    const int l32 = lane & 31, half = lane >> 5;
    const bool tri = wave < 2;
    const int bP = tri ? 2 * wave : wave - 2, bQ = tri ? bP : 2, bR = tri ? bP + 1 : 3, bS = tri ? bP + 1 : bP;
    DMA_CLK(4);
    const int T = p.T;
    for (int i = tid; i < ROWS; i += SplitGeom::THREADS) {
        const bool ok = t0 + i < T;
        s_tok[i] = ok ? t0 + i : INT_MAX;
        t_tok[i] = ok ? t0 + i : -1;
        scale[i] = 0.f;
    }
    f32x16 acc[3];
    float ssP = 0.f, ssR = 0.f;                                // waves 0 and 1 cover the four blocks; 2 and 3 repeat two
    if (loader) {
        split_loader<SplitGeom::NS, LPT, STAGE>(reinterpret_cast<const uint16_t*>(p.X), p.ld, p.d, ring, wave, lane,
            [&](int, int row) { return min(t0 + row, T - 1); });
    } else {
#pragma unroll
        for (int a = 0; a < 3; ++a)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][i] = 0.f;
        const int blk[4] = {bP, bQ, bR, bS};
        const char* fptr[4][4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int f = 0; f < 4; ++f) fptr[ks][f] = ring + lds_off(blk[f] * 32 + l32, 2 * ks + half);
        u32x4 fr[2][4];
        DMA_CLK(0);
        split_multiplier<SplitGeom::NS, STAGE>(p.d / SplitGeom::EPC,
            [&](int set, int stage_off, int ks) {
#pragma unroll
                for (int f = 0; f < 4; ++f) fr[set][f] = *reinterpret_cast<const u32x4*>(fptr[ks][f] + stage_off);
            },
            [&](int set) {
                Mfma<uint16_t>::run(acc[0], fr[set][0], fr[set][1]);
                Mfma<uint16_t>::run(acc[1], fr[set][0], fr[set][2]);
                Mfma<uint16_t>::run(acc[2], fr[set][3], fr[set][2]);
                ssP += piece_sumsq_fast<uint16_t>(fr[set][0]);
                ssR += piece_sumsq_fast<uint16_t>(fr[set][2]);
            });
    }
    DMA_CLK(1);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));           // surplus loads land before the ring is reused
    __syncthreads();
    DMA_CLK(2);
    if (!loader) {
        const float vP = ssP + __shfl_xor(ssP, 32, 64), vR = ssR + __shfl_xor(ssR, 32, 64);
        // (waves that sum the same block write the same bits: same pieces, same order)
        if (half == 0) {
            const int rP = bP * 32 + l32, rR = bR * 32 + l32;
            scale[rP] = (t_tok[rP] >= 0 && vP > 0.f) ? 1.0f / sqrtf(vP) : 0.f;    // a zero row normalises to zero
            scale[rR] = (t_tok[rR] >= 0 && vR > 0.f) ? 1.0f / sqrtf(vR) : 0.f;
        }
    }
    __syncthreads();
    if (loader) return;
    uint32_t* gamma_bits = reinterpret_cast<uint32_t*>(p.gamma);
    const int sblk[3] = {bP, bP, bS}, tblk[3] = {bQ, bR, bR};
#pragma unroll
    for (int a = 0; a < 3; ++a) {
        if (a == 2 && !tri) break;                             // (wave-uniform)
        const int nl = tblk[a] * 32 + l32;
        const int ttok = t_tok[nl];
        const float m = block_max(acc[a], scale, s_tok, sblk[a] * 32, half, sblk[a] == tblk[a], ttok);
        publish_max(m, scale[nl], ttok, half, gamma_bits);
    }
    DMA_CLK(3);
}

// mode 0: 128 x 128 units over the whole triangle; 1: 256 x 256 off the diagonal ("big"), the diagonal 256-blocks in
// three 128 x 128 units; 2: 64 x 128 units off the diagonal of 128-blocks ("big": two per pair of blocks, 192 rows
// staged instead of 256, for sizes where 128 x 128 units leave CUs idle), the diagonal blocks as gram_tile_diag units.
struct DmaUnits {
    long long n_big, n_units;
    __host__ __device__ DmaUnits(int T, int mode) {
        const long long nb256 = (T + 255) / 256, nb128 = (T + 127) / 128;
        n_big = mode == 1 ? nb256 * (nb256 - 1) / 2 : mode == 2 ? nb128 * (nb128 - 1) : 0;
        n_units = mode == 1 ? n_big + 3 * nb256 : mode == 2 ? n_big + nb128 : nb128 * (nb128 + 1) / 2;
    }
};

// Mode 2: unit u -> tested 128-block tb >= 1 against the 64-block sb < 2 tb, or (sb < 0) the diagonal block tb.  The order
// goes patch by patch -- four 128-blocks of tested rows against eight 64-blocks, 32 units -- so that the contiguous
// range of units an XCD starts with needs about a thousand rows instead of most of the matrix (every XCD has an L2 of
// its own): first the patches on the diagonal (their 64 x 128 units and their diagonal units), then the others.
struct DmaUnit2 { int tb, sb; };
__device__ inline DmaUnit2 dma_unit2(int u, int nb) {
    const int P = (nb + 3) >> 2;
    int acc = 0;
    for (int g = 0; g < P; ++g) {
        const int t_lo = 4 * g, n_t = min(4, nb - t_lo), n_rect = n_t * (n_t - 1), cnt = n_rect + n_t;
        if (u < acc + cnt) {
            const int w = u - acc;
            if (w >= n_rect) return {t_lo + (w - n_rect), -1};
            const int tl = w < 2 ? 1 : w < 6 ? 2 : 3;          // rows 1, 2, 3 of the patch hold 2, 4, 6 units
            return {t_lo + tl, 8 * g + (w - tl * (tl - 1))};
        }
        acc += cnt;
    }
    for (int gt = 1; gt < P; ++gt) {
        const int t_lo = 4 * gt, n_t = min(4, nb - t_lo), row = n_t * 8;
        if (u < acc + gt * row) {
            const int w = u - acc, gs = w / row, v = w - gs * row;
            return {t_lo + (v >> 3), 8 * gs + (v & 7)};
        }
        acc += gt * row;
    }
    return {0, -1};                                            // (not reached for u < nb * nb)
}

// largest n with n (n + 1) / 2 <= v
__device__ inline int tri_row(long long v) {
    int n = (int)((sqrtf(8.f * (float)v + 1.f) - 1.f) * 0.5f);
    while ((long long)(n + 1) * (n + 2) / 2 <= v) ++n;
    while ((long long)n * (n + 1) / 2 > v) --n;
    return n;
}

// Definition "Gram threshold", last step, run by the workgroup that leaves the launch last (u.counts != NULL): the
// row maxima are complete then, so the threshold test and the compaction need no launch of their own.
// acc_reset: the maxima were accumulated in a workspace array that is zero between calls (no launch cleared it):
// hand them to the caller's array (gamma_out, may be NULL) and zero the accumulator again.
__device__ inline void full_selection_finish(UpdateParams u, float* gamma, int* sh /* 3 x 32 ints */, bool acc_reset,
                                             float* gamma_out) {
    const int tid = threadIdx.x, nthr = blockDim.x;
    const int T = u.T;
    constexpr int MG = 4;                                      // groups of four tokens per thread on the fast path
    const bool vec = T % 4 == 0 && T <= nthr * 4 * MG && ((uintptr_t)gamma & 15) == 0 &&
                     (!gamma_out || ((uintptr_t)gamma_out & 15) == 0) && (!u.mask || ((uintptr_t)u.mask & 3) == 0);
    if (vec) {
        // one trip to memory: a thread's (up to) sixteen consecutive maxima in four 16-byte reads, kept in registers
        // across the scan; mask, maxima and the cleared accumulator leave in whole words
        const int ng = T >> 2;
        float4 v[MG];
        int c_idx = 0;
#pragma unroll
        for (int j = 0; j < MG; ++j) {
            const int g = tid * MG + j;
            v[j] = g < ng ? reinterpret_cast<const float4*>(gamma)[g] : float4{INFINITY, INFINITY, INFINITY, INFINITY};
            c_idx += (v[j].x < u.thr) + (v[j].y < u.thr) + (v[j].z < u.thr) + (v[j].w < u.thr);   // strict "<" of the Definition
        }
        int n_idx;
        int o_idx = block_exclusive_scan(c_idx, &n_idx, sh);
#pragma unroll
        for (int j = 0; j < MG; ++j) {
            const int g = tid * MG + j;
            if (g >= ng) continue;
            const float e[4] = {v[j].x, v[j].y, v[j].z, v[j].w};
            uint32_t m4 = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const bool keep = e[k] < u.thr;
                m4 |= (keep ? 1u : 0u) << (8 * k);
                if (keep) { if (u.idx) u.idx[o_idx] = 4 * g + k; ++o_idx; }
            }
            if (u.mask) reinterpret_cast<uint32_t*>(u.mask)[g] = m4;
            if (acc_reset) {
                if (gamma_out) reinterpret_cast<float4*>(gamma_out)[g] = v[j];
                reinterpret_cast<float4*>(gamma)[g] = float4{0.f, 0.f, 0.f, 0.f};
            }
        }
        if (tid == 0) {
            u.counts[0] = n_idx; u.counts[1] = n_idx; u.counts[2] = 0; u.counts[3] = ADA_OK;
            if (u.gram_ops) *u.gram_ops = (unsigned long long)T * (unsigned long long)T;   // Table 6 / eq. (6)
        }
        return;
    }
    const int chunk = (T + nthr - 1) / nthr;
    const int lo = min(T, tid * chunk), hi = min(T, lo + chunk);
    int c_idx = 0;
    for (int t = lo; t < hi; ++t) c_idx += gamma[t] < u.thr;          // strict "<" of the Definition
    int n_idx;
    int o_idx = block_exclusive_scan(c_idx, &n_idx, sh);
    for (int t = lo; t < hi; ++t) {
        const float g = gamma[t];
        const bool keep = g < u.thr;
        if (u.mask) u.mask[t] = keep ? 1 : 0;
        if (keep) { if (u.idx) u.idx[o_idx] = t; ++o_idx; }
        if (acc_reset) {
            if (gamma_out) gamma_out[t] = g;
            gamma[t] = 0.f;
        }
    }
    if (tid == 0) {
        u.counts[0] = n_idx; u.counts[1] = n_idx; u.counts[2] = 0; u.counts[3] = ADA_OK;
        if (u.gram_ops) *u.gram_ops = (unsigned long long)T * (unsigned long long)T;   // Table 6 / eq. (6)
    }
}

template <bool NORMS>
__global__ __launch_bounds__(NORMS ? SplitGeom::THREADS : DmaGeom::THREADS) void k_gram_dma(GramParams p, int big_mode, int* meta, UpdateParams upd, float* gamma_out) {
    extern __shared__ __align__(16) char lds[];
    __shared__ long long s_next;
    __shared__ int s_last, s_scan[32];
    gram_group_offset(p);
    if (p.ws_gs) meta = reinterpret_cast<int*>(reinterpret_cast<char*>(meta) + (long long)blockIdx.y * p.ws_gs);
    int* queue = meta + META_QUEUE;                            // the workspace's unit counter and its sign-off tickets
    int* ticket = meta + META_TICKET;
    const DmaUnits U(p.T, big_mode);
    const int G = gridDim.x;
    DMA_CLK(5);
    long long u = (long long)(blockIdx.x & 7) * (G >> 3) + (blockIdx.x >> 3);     // first unit: contiguous range per XCD
    while (u < U.n_units) {
        long long nxt = 0;
        // next unit: the reply arrives behind the tile (no unit is left when each workgroup starts with one)
        if (threadIdx.x == 0) nxt = U.n_units > G ? (long long)G + atomicAdd(queue, 1) : U.n_units;
        if constexpr (NORMS) {                                 // (launched with mode 0 or 2)
            if (big_mode == 2) {
                const DmaUnit2 w = dma_unit2((int)u, (p.T + 127) >> 7);
                if (w.sb >= 0) gram_tile_split<32, 64>(p, w.sb * 64, w.tb * 128, false, lds);
                else gram_tile_diag(p, w.tb * 128, lds);
            } else {
                const int tb = tri_row(u);                     // 128-blocks: 0 <= sb <= tb
                const int sb = (int)(u - (long long)tb * (tb + 1) / 2);
                gram_tile_split<64, 64>(p, sb * 128, tb * 128, sb == tb, lds);
            }
        } else if (u < U.n_big) {
            const int tb = tri_row(u) + 1;                     // off-diagonal 256-blocks: 0 <= sb < tb
            const int sb = (int)(u - (long long)tb * (tb - 1) / 2);
            gram_tile_dma<128>(p, sb * 256, tb * 256, false, lds);
        } else if (big_mode) {
            const long long v = u - U.n_big;                   // diagonal 256-block i in three 128 x 128 units
            const int i = (int)(v / 3), k = (int)(v % 3);
            const int t0 = (2 * i + (k >= 1)) * 128, s0 = (2 * i + (k == 2)) * 128;
            if (t0 < p.T) gram_tile_dma<64>(p, s0, t0, k != 1, lds);
        } else {
            const int tb = tri_row(u);                         // 128-blocks: 0 <= sb <= tb
            const int sb = (int)(u - (long long)tb * (tb + 1) / 2);
            gram_tile_dma<64>(p, sb * 128, tb * 128, sb == tb, lds);
        }
        if (threadIdx.x == 0) s_next = nxt;
        __syncthreads();
        u = s_next;
        __syncthreads();
    }
    // This workgroup's row maxima left the CU as device-scope atomics; once they are acknowledged (vmcnt(0)) and the
    // workgroup has met, it signs off.  Every workgroup's last fetch precedes its sign-off, so whoever signs off last
    // may clear both counters, and sees every row maximum after one invalidate.
    DMA_CLK(6);
    drain_stores();
    __syncthreads();
    DMA_CLK(7);
    if (threadIdx.x == 0) {
        const bool last = take_ticket(ticket, G);              // (per XCD first: one counter would serve 256 in turn)
        if (last) { atomicExch(queue, 0); reset_tickets(ticket); }
        s_last = last ? 1 : 0;
    }
    __syncthreads();
    DMA_CLK(8);
    if (!upd.counts || !s_last) return;
    DMA_CLK_ANY(9);
    if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    __syncthreads();
    DMA_CLK_ANY(10);
    if (upd.go.ws) {                                         // several problems: blockIdx.y is the problem
        const long long g = blockIdx.y;
        if (upd.mask) upd.mask += g * (long long)upd.T;
        if (upd.idx) upd.idx += g * upd.go.list;
        upd.counts += g * upd.go.counts;
        if (upd.gram_ops) upd.gram_ops += g * upd.go.ops;
    }
    if (NORMS && gamma_out && upd.go.ws) gamma_out = nullptr; // (several problems: no gamma output)
    full_selection_finish(upd, p.gamma, s_scan, NORMS, gamma_out);   // (p.gamma is this problem's: gram_group_offset)
    DMA_CLK_ANY(11);
}
