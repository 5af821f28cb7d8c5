// Fused cascade step (Algorithm 1) in ONE launch.  Included by ada_kernels.hip inside its anonymous namespace.
//
// Work: every token t (tested, MFMA N side) against every inherited representative s (MFMA M side): the T x r
// entries eq. (6) counts.  A workgroup owns a 64 x 64 tile over all of K and, per tile,
//   * streams the 128 rows through LDS once, accumulating the raw dot products on MFMA and, from the same
//     registers, each row's sum of squares (Algorithm 1 step 1 costs no extra pass over X);
//   * turns the accumulators into cosines and records, per tested token, one 32-bit word of "hits"
//     (|cos| >= 1 - tau^2) per 32 representatives.  For an inherited token only earlier representatives count
//     (steps 3-4); for any other token all of them do (steps 7-8), or only earlier ones with the earlier-only flag.
// Validity of a representative (step 5) is "no hit in its own row"; a non-inherited token is new (step 9) iff it has
// no hit on a VALID representative.  Both are resolved from the hit words by the workgroup that finishes last
// (ticket counter, no waiting), which also compacts R_valid u R_new (step 10) and writes the counts.
// Deferring validity this way lets the r x r and the (T-r) x r products run as one batch of tiles.
//
// K is split over KG groups of 4 wavefronts (chunk c goes to group c % KG); inside a group each wavefront takes one
// 16-element k-step of the chunk for the whole tile.  Partial tiles are summed through LDS in a fixed order.

#ifdef ADA_PHASE_CLOCKS
__device__ unsigned long long g_phase_clk[64];
// (the constant-rate 100 MHz counter, comparable across workgroups and XCDs)
#define ADA_CLK(i) do { if (threadIdx.x == 0 && blockIdx.x == (ADA_PHASE_CLOCKS)) g_phase_clk[i] = __builtin_amdgcn_s_memrealtime(); } while (0)
#define ADA_CLK_LAST(i) do { if (threadIdx.x == 0) g_phase_clk[i] = __builtin_amdgcn_s_memrealtime(); } while (0)
#else
#define ADA_CLK(i) do { } while (0)
#define ADA_CLK_LAST(i) do { } while (0)
#endif

struct FusedParams {
    const void* X;
    long long ld;
    int T, d;
    const int32_t* prev_idx;
    const int32_t* r_dev;    // optional device count
    int r_host;              // count, or capacity of prev_idx when r_dev is given
    float thr;
    int earlier_only;
    uint32_t* hits;          // [W][T] word-major: word w of token t covers inherited representatives 32w .. 32w+31
    int W;                   // hit words per token (covers r_host)
    float* gamma;            // optional, zero on entry: max |cos| over the columns that count for the token
    int32_t* ticket;         // zero on entry, zero again on exit; ticket[TICKET_XCD0 + 32 x] (x < 8): first-level counters
    int32_t* idx;
    int32_t* adds;           // may be NULL
    int32_t* removes;        // may be NULL
    int32_t* counts;         // [4]
    unsigned long long* gram_ops;   // may be NULL
    // nearest-representative assignment (Section 2.3) instead of the cascade step: prev_idx is the set R itself
    int assign_mode;
    unsigned long long* best;       // [T], zero on entry and on exit: (bits of the max |cos|) << 32 | (INT_MAX - token id)
    int32_t* assign;                // [T]
    float* corr;                    // [T], may be NULL
    // the list was written earlier in this same launch by another workgroup (k_cascade_pass): read it past the
    // caches instead of invalidating them
    int coherent_list;
    // tile shape of the two-group direct-to-LDS form: n > 0 = choose per step for a chip of n CUs (cascade_tile_shape);
    // 0, -1, -2 = always shape 0, 1, 2
    int tile_pick;
    // workgroups of the launch (a multiple of 8), filled in by the launcher: the built-in grid size sits in another
    // cache line of the launch's argument block, and waiting for that line is a trip to memory at every kernel start
    int grid;
    // Several independent problems of one shape in one launch (heads of one matrix, or sequences stacked in one
    // allocation): groups > 1.  Workgroup b serves group b % groups as its worker b / groups of wpg (grid = groups x
    // wpg); the pointers above are group 0's, group g's lie g strides further on.
    int groups, wpg;
    long long x_gs;          // bytes between consecutive groups' X
    long long list_gs;       // int32 elements between groups in prev_idx, idx, adds, removes
    long long counts_gs;     // int32 elements between groups in counts and r_dev
    long long ops_gs;        // elements between groups in gram_ops
    long long ws_gs;         // bytes between groups' hit tables and tickets
    // Threshold adapted from layer to layer (Section 8.1): this step's tau / threshold are read from device memory
    // (thr_in overrides thr), and the workgroup that updates the set also writes the next step's (tau_out may be NULL)
    const double* tau_in;
    const float* thr_in;
    double* tau_out;
    float* thr_out;
    double kappa, eta_target, tau_min, tau_max;
    // assignment: optional [T], the POSITION in R of every token's representative (what the attention's hand-over
    // needs).  The arg-max keys then carry positions instead of token ids: R is ascending, so the order among equal
    // cosines is the same.
    int32_t* pos_out;
    // cascade step: [T], zero on entry and on exit (it shares the arg-max table's memory: the two modes never run on one
    // workspace at once).  first[t] = 0xFFFFFFFF - (smallest list position of a representative that hits token t), 0 if
    // none does: what the set update needs of a token's hit words in all but rare cases (see fused_update_rec).
    uint32_t* first;
    // cascade step with a gamma output: Algorithm 1's gamma^cross is the maximum over the VALID representatives, which are
    // known only after all products.  The tiles therefore also keep, per non-inherited token, the arg max over all
    // inherited representatives (p.best, keyed by list position); the workgroup that updates the set lists the tokens
    // whose nearest representative was removed (fix_list), clears their gamma and leaves the list's length, the set size
    // and a status in the workspace's scalars (fix_meta: META_NONREP, META_R, META_STATUS) for the launch that recomputes
    // those tokens' maxima against the valid representatives: the cross-Gram tiles of the step's other form, on that list.
    int32_t* fix_list;
    int32_t* fix_meta;
};

// Section 8.1's rule as read here: the turnover eta = (adds + removes) / r of the step just made (eq. (8)) moves tau
// by kappa (eta_target - eta): a stable set (low turnover) tightens the threshold (larger tau: fewer representatives),
// an evolving one loosens it; the result is clipped to [tau_min, tau_max].  Plain IEEE double operations, one
// rounding each (no fused multiply-add), so that a float64 CPU evaluation of the same expression gives the same bits.
__device__ inline void adapt_tau(const FusedParams& p, int r, int n_add, int n_rem, bool step_ok) {
#pragma clang fp contract(off)                               // a * b + c stays two roundings (device code contracts by default)
    if (!p.tau_out) return;
    const double tau = *p.tau_in;
    double next = tau;
    if (step_ok && r > 0) {
        const double eta = (double)(n_add + n_rem) / (double)r;
        const double gap = p.eta_target - eta;
        const double move = p.kappa * gap;
        next = tau + move;
        next = fmin(fmax(next, p.tau_min), p.tau_max);
    }
    const double sq = next * next;
    *p.tau_out = next;
    *p.thr_out = (float)(1.0 - sq);
}

// Tile shapes (representatives x tested tokens): 0 = 64 x 64, 1 = 64 x 128, 2 = 128 x 128.  A step's cost is taken as
// rounds x (operand bytes per tile + a fixed part worth about 56 rows of 4096 two-byte elements: set size, list and
// first-chunk trips before the K loop, norms and hit words after it), rounds = tiles over the workgroups that share
// them: operand bytes per Gram entry fall with the tile size, but a tile count below the worker count leaves CUs idle.
__host__ __device__ inline int tile_rows_r(int shape) { return shape >= 2 ? 128 : 64; }
__host__ __device__ inline int tile_rows_t(int shape) { return shape == 0 ? 64 : shape == 3 ? 256 : 128; }
// (T <= FUSED_MAX_T: every count fits 32 bits, and 32-bit divisions are what the start of a launch can afford)
__host__ __device__ inline int tile_count(int r, int T, int shape) {
    const int br = tile_rows_r(shape), bt = tile_rows_t(shape);
    return ((r + br - 1) / br) * ((T + bt - 1) / bt);
}
// pick > 0: choose; pick = 0, -1, -2, -3: always shape 0, 1, 2, 3.  workers: workgroups that share the step's tiles.
// nshapes: 4 when the ring tiles apply (bf16 rows in whole 64-byte pieces), else 3.  The operand bytes are weighted by
// how far from the CU's fill rate each engine was measured (quarters): the 64 x 64 tile and the ring tiles run at it,
// the register-free 64 x 128 tile at 5/4 and the 128 x 128 tile of the same engine (fp32 only now) at twice that time.
__host__ __device__ inline int cascade_tile_shape(int r, int T, int d, int pick, int workers, int nshapes = 4) {
    if (pick <= 0) return -pick < nshapes ? -pick : nshapes - 1;
    const unsigned wk = workers > 0 ? (unsigned)workers : 1u;
    const unsigned dd = (unsigned)(d < 65536 ? d : 65536);   // keeps the products below 2^32 (tiles <= 65536 / 8 per round matter)
    int best = 0;
    unsigned long long best_cost = 0;
    for (int shape = 0; shape < nshapes; ++shape) {
        const unsigned tiles = (unsigned)tile_count(r, T, shape);
        const unsigned rounds = (tiles + wk - 1u) / wk;
        const unsigned weight = shape == 1 ? 5u : (shape == 2 && nshapes == 3) ? 8u : 4u;
        const unsigned long long cost = (unsigned long long)rounds *
            ((unsigned long long)(unsigned)(tile_rows_r(shape) + tile_rows_t(shape)) * dd * weight + 4ull * 56u * 4096u);
        if (shape == 0 || cost < best_cost) { best = shape; best_cost = cost; }
    }
    return best;
}

// Last-arriver detection in two levels.  Atomics on one address are served one after the other at the memory side
// (about 25 ns each here), so a single counter taken by 256 workgroups that finish together costs the last of them 6 us.
// Workgroups first count per XCD (blockIdx % 8: eight counters on separate cache lines); the last of each XCD then
// takes the device-wide ticket.  Called by one thread; true in exactly one workgroup, after all others have called.
constexpr int TICKET_XCD0 = 64;                          // ints from the device-wide ticket to the first XCD counter
__device__ inline bool take_ticket(int32_t* ticket, int grid) {
    const int per = grid >> 3;                           // grids are multiples of 8
    if (atomicAdd(ticket + TICKET_XCD0 + 32 * (blockIdx.x & 7), 1) != per - 1) return false;
    return atomicAdd(ticket, 1) == 7;
}
__device__ inline void reset_tickets(int32_t* ticket) {   // by the last arriver: nobody else touches them any more
    __hip_atomic_store(ticket, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
    for (int x = 0; x < 8; ++x)
        __hip_atomic_store(ticket + TICKET_XCD0 + 32 * x, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ inline int list_at(const FusedParams& p, int j) {
    return p.coherent_list ? __hip_atomic_load(p.prev_idx + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : p.prev_idx[j];
}

// DMA = operands go global -> LDS directly (global_load_lds, 16 bytes per lane) through a ring of NS stages per
// K-group; otherwise they pass through registers (needed when a row chunk can be ragged or unaligned).
template <int KG, bool DMA> struct FusedGeom {
    static constexpr int THREADS = 256 * KG;
    static constexpr int D = 4;                           // register path: prefetch depth (steps of one group), even
    static constexpr int NS = 4;                          // DMA path: LDS stages per K-group
    static constexpr int LPT = 4;                         // 16-byte pieces per thread per chunk
    static constexpr int STAGE = 128 * 128;               // one chunk of 128 rows
    static constexpr int NPART = DMA ? 2 * KG : KG;       // partial sums of squares per row
    static constexpr int OFF_STOK = 0;                    // int[64]   token id of each "against" row (INT_MAX: none)
    static constexpr int OFF_REPF = 256;                  // int[64]   tested token is inherited
    static constexpr int OFF_SS = 512;                    // float[NPART][128] partial sums of squares
    static constexpr int OFF_SCALE = OFF_SS + NPART * 512;   // float[128] 1/norm (0 for rows that do not exist)
    static constexpr int OFF_SCAN = OFF_SCALE + 512;      // scan scratch of the update phase
    static constexpr int META = OFF_SCAN + 512;
    static constexpr int RING = DMA ? KG * NS * STAGE : KG * 2 * STAGE;
    static constexpr int RINGMAX = 3 * 384 * 128;         // the widest ring tile: three stages of 384 rows (144 KB)
    static constexpr int BODY = (KG == 2 && DMA) ? RINGMAX : (RING > 65536 ? RING : 65536);   // stages / reduction scratch (64 KB) / update state
    static constexpr int OFF_BIG = META + BODY;           // metadata of the wide tiles (two-group direct-to-LDS form)
    static constexpr int LDS = META + BODY + ((KG == 2 && DMA) ? 8192 : 0);
    static_assert(LDS <= 160 * 1024, "one workgroup's LDS");
};

constexpr int waitcnt_vm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }   // s_waitcnt vmcnt(n) only (gfx9 encoding)

template <typename In> __device__ inline float piece_sumsq_fast(u32x4 v);
template <> __device__ inline float piece_sumsq_fast<float>(u32x4 v) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) { const float f = __uint_as_float(v[i]); s = fmaf(f, f, s); }
    return s;
}
template <> __device__ inline float piece_sumsq_fast<uint16_t>(u32x4 v) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    // two exact bf16 products added in fp32 per instruction; the four words are named one by one on purpose
    const uint32_t w0 = v[0], w1 = v[1], w2 = v[2], w3 = v[3];
    const bf16x2 x0 = __builtin_bit_cast(bf16x2, w0), x1 = __builtin_bit_cast(bf16x2, w1);
    const bf16x2 x2 = __builtin_bit_cast(bf16x2, w2), x3 = __builtin_bit_cast(bf16x2, w3);
    float s = __builtin_amdgcn_fdot2_f32_bf16(x0, x0, 0.f, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(x1, x1, s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(x2, x2, s, false);
    s = __builtin_amdgcn_fdot2_f32_bf16(x3, x3, s, false);
    return s;
}

// Epilogue of one 32 x 32 block (rows: 32 representatives, columns: 32 tested tokens, one token per lane pair):
// scale the raw dot products to cosines, then either the hit word of Algorithm 1 or the arg-max key of Section 2.3.
// s_tok32 / scale32: token ids and 1/norm of the block's 32 representative rows; tsc: 1/norm of this lane's token t;
// word: index of the hit word these 32 representatives fill.
__device__ inline void finish_block(const FusedParams& p, const f32x16& tot, const int* s_tok32, const float* scale32,
                                    float tsc, int mode, int t, int word, int half) {
    const bool ordered = (mode & 1) != 0;             // only earlier representatives count for this token
    const bool inherited = (mode & 2) != 0;           // the token is itself an inherited representative
    // accumulator register 4q+e of a 32x32 MFMA block is row 8q + 4*half + e: four consecutive rows per q
    f32x4 sc4[4];
    i32x4 tk4[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        sc4[q] = *reinterpret_cast<const f32x4*>(scale32 + 8 * q + 4 * half);
        tk4[q] = *reinterpret_cast<const i32x4*>(s_tok32 + 8 * q + 4 * half);
    }
    if (p.assign_mode) {                              // uniform
        // Section 2.3: the largest |cos| over this tile's representatives and who holds it.  A non-negative float
        // orders like its bit pattern, so (bits << 32 | INT_MAX - token id) under an integer max is an exact,
        // order-independent arg max that prefers the smaller token id among equals; padding rows (token id
        // INT_MAX, scale 0) give key 0 and never win.
        unsigned long long key = 0ull;
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float c = (fabsf(tot[4 * q + e]) * sc4[q][e]) * tsc;
                const int who = p.pos_out ? word * 32 + 8 * q + 4 * half + e : tk4[q][e];   // (rows past r: c = 0)
                const unsigned long long k = ((unsigned long long)__float_as_uint(c) << 32) |
                                             (unsigned long long)(uint32_t)(INT_MAX - who);
                key = k > key ? k : key;
            }
        const unsigned long long other = ((unsigned long long)(uint32_t)__shfl_xor((int)(key >> 32), 32, 64) << 32) |
                                         (unsigned long long)(uint32_t)__shfl_xor((int)(uint32_t)key, 32, 64);
        key = other > key ? other : key;
        if (half == 0 && t < p.T) atomicMax(p.best + t, key);
        return;
    }
    uint32_t bits = 0u;
    float m = 0.f;
    int who = 0;                                      // row (within the block's 32) that holds this lane's maximum
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float c = (fabsf(tot[4 * q + e]) * sc4[q][e]) * tsc;
            if (ordered && !(tk4[q][e] < t)) c = 0.f;     // only earlier representatives count
            if (c >= p.thr) bits |= 1u << (8 * q + 4 * half + e);
            if (c > m) { m = c; who = 8 * q + 4 * half + e; }   // strict: the smaller position among equals
        }
    bits |= (uint32_t)__shfl_xor((int)bits, 32, 64);
    {
        const float mo = __shfl_xor(m, 32, 64);
        const int wo = __shfl_xor(who, 32, 64);
        if (mo > m || (mo == m && wo < who)) { m = mo; who = wo; }
    }
    if (half == 0 && t < p.T) {
        // word-major: 32 lanes store 32 consecutive words.  The store is a device-scope atomic (written through
        // the L2 to where every XCD sees it), so that handing the words over needs no L2 write-back: a write-back
        // per workgroup serialises on the L2 and was the longest single wait of the step.
        __hip_atomic_store(p.hits + (size_t)word * p.T + t, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        // the earliest representative that hits t, over all tiles: an integer max of the inverted position (exact and
        // order-independent); few tokens have hits in more than one or two blocks of 32
        if (bits != 0u && p.first) atomicMax(p.first + t, 0xFFFFFFFFu - (uint32_t)(word * 32 + __builtin_ctz(bits)));
        if (p.gamma && m > 0.f) {
            atomicMax(reinterpret_cast<uint32_t*>(p.gamma) + t, __float_as_uint(m));
            // step 8 needs to know WHO holds a non-inherited token's maximum: the assignment's packed key (value bits,
            // then the smaller list position), exact and order-independent
            if (!inherited && p.fix_list)
                atomicMax(p.best + t, ((unsigned long long)__float_as_uint(m) << 32) |
                                      (unsigned long long)(uint32_t)(INT_MAX - (word * 32 + who)));
        }
    }
}

template <typename In, bool ALIGNED, int KG, bool DMA>
__device__ inline void fused_tile(const FusedParams& p, int r, int s0, int t0, int sb, char* lds) {
    using G = FusedGeom<KG, DMA>;
    constexpr int B = 64;
    constexpr int EPP = 16 / (int)sizeof(In);
    constexpr int EPC = 8 * EPP;
    constexpr int LPT = G::LPT, D = G::D;

    int* s_tok = reinterpret_cast<int*>(lds + G::OFF_STOK);
    int* repf = reinterpret_cast<int*>(lds + G::OFF_REPF);
    float* ssq = reinterpret_cast<float*>(lds + G::OFF_SS);
    float* scale = reinterpret_cast<float*>(lds + G::OFF_SCALE);
    char* body = lds + G::META;

    const int tid = threadIdx.x, t256 = tid & 255;
    // wave-uniform values are pinned to scalar registers so that code selected by them branches, not predicates
    const int g = __builtin_amdgcn_readfirstlane(tid >> 8);
    const int wave = __builtin_amdgcn_readfirstlane(t256 >> 6);
    const int lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    char* buf0 = body + g * 2 * G::STAGE;
    char* buf1 = buf0 + G::STAGE;
    const In* X = reinterpret_cast<const In*>(p.X);

    ADA_CLK(1);
    // every list entry this thread needs is requested before anything waits: one trip to memory, not two
    const int pc = t256 & 7, rb = t256 >> 3;
    int ptok[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int li = s0 + rb + 32 * j;                 // only used for rows 0..63 (representatives)
        ptok[j] = list_at(p, li < r ? li : r - 1);
    }
    if (tid < B) {
        const int li = s0 + tid;
        const bool ok = li < r;
        int tok = list_at(p, ok ? li : r - 1);
        tok = min(max(tok, 0), p.T - 1);
        s_tok[tid] = ok ? tok : INT_MAX;
        repf[tid] = 0;
    }
    __syncthreads();
    // which tested tokens of this tile are inherited: a pass over the whole list, run behind the first operand loads
    // (the flags are not read before the epilogue)
    auto mark_inherited = [&]() {
        for (int j = tid; j < r; j += G::THREADS) {
            const unsigned q = (unsigned)(list_at(p, j) - t0);
            if (q < (unsigned)B) repf[q] = 1;
        }
    };

    const In* rowp[LPT];
    int woff[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int row = rb + 32 * j;                     // rows 0..63: representatives, 64..127: tested tokens
        const int tok = row < B ? min(max(ptok[j], 0), p.T - 1) : min(t0 + row - B, p.T - 1);
        rowp[j] = X + (size_t)tok * (size_t)p.ld;
        woff[j] = lds_off(row, pc);
    }
    const int nk = (p.d + EPC - 1) / EPC;
    const int nsteps = (nk + KG - 1) / KG;               // steps of this group; step k handles chunk k * KG + g
    // Wave w of a K-group owns the 32 x 32 block (wa, wb) = (w >> 1, w & 1) of the tile over all four k-steps of each of
    // the group's chunks, so a block has only one partial sum per K-group and the epilogue needs one small exchange.
    // Two accumulators (even / odd k-steps) keep two independent MFMA chains in flight.
    const int wa = wave >> 1, wb = wave & 1;
    u32x4 fa[2][4], fb[2][4];
    f32x16 acc[2];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
    auto read_frags = [&](const char* stage, int f) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int piece = 2 * ks + half;
            fa[f][ks] = *reinterpret_cast<const u32x4*>(stage + lds_off(wa * 32 + l32, piece));
            fb[f][ks] = *reinterpret_cast<const u32x4*>(stage + lds_off(B + wb * 32 + l32, piece));
        }
    };
    auto mma = [&](int f) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) Mfma<In>::run(acc[ks & 1], fa[f][ks], fb[f][ks]);
    };

    if constexpr (DMA) {
        // ---- operands go straight from global memory into LDS.  One wave instruction moves 64 x 16 bytes to 1 KB of
        // contiguous LDS = 8 rows of a stage; lane l serves row l / 8, slot l % 8 and therefore fetches piece
        // (l % 8) ^ lds_swz(row), which reproduces the XOR-swizzled layout the fragment reads expect.  The waits are
        // counted by hand (NS - 3 chunks stay in flight across the barrier) and the barrier is the bare instruction:
        // a fenced barrier would drain the loads.  Chunk indices past the end are clamped, so every step issues the
        // same number of loads and the counts stay valid; such a chunk is never multiplied.
        constexpr int NS = G::NS;
        char* ring = body + g * NS * G::STAGE;
        const int pcd = pc ^ lds_swz(rb);                 // 32 j leaves bits 0..3 of the row alone
        float ssa = 0.f, ssb = 0.f;
        auto issue = [&](int stage, int k) {
            const int chunk = min(k * KG + g, nk - 1);
#pragma unroll
            for (int j = 0; j < LPT; ++j) {
                char* dst = ring + stage * G::STAGE + (wave * 8 + 32 * j) * 128;      // wave-uniform
                __builtin_amdgcn_global_load_lds(
                    (const void __attribute__((address_space(1)))*)(rowp[j] + chunk * EPC + pcd * EPP),
                    (void __attribute__((address_space(3)))*)dst, 16, 0, 0);
            }
        };
        auto mma_and_norms = [&](int f, int k) {
            if (k * KG + g < nk) {                       // scalar: a clamped (repeated) chunk is skipped
                mma(f);
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    // Section 2.1: ||x||^2 from the fragments already in hand.  The two waves that share a block of rows
                    // split its four k-steps, so every wave sums four fragments per chunk (scalar selects).
                    ssa += piece_sumsq_fast<In>(wb == 0 ? fa[f][ks] : fa[f][ks + 2]);
                    ssb += piece_sumsq_fast<In>(wa == 0 ? fb[f][ks] : fb[f][ks + 2]);
                }
            }
        };
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) issue(s, s);
        if (!p.assign_mode) mark_inherited();            // its loads are younger than the ring's: the wait below covers stage 0
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
        ADA_CLK(2);
        __builtin_amdgcn_s_barrier();
        ADA_CLK(3);
        read_frags(ring, 0);
        // When the steps come in whole blocks of NS, the last block is written out on its own: it issues only the one
        // chunk that is still missing and lowers its waits accordingly, so no chunk is fetched twice (the clamped
        // surplus loads of the general form are 3 chunks in every nsteps of L2 -> CU traffic).
        const bool clean = nsteps % NS == 0;
        const int nmain = clean ? nsteps - NS : nsteps;
        for (int k0 = 0; k0 < nmain; k0 += NS) {
#pragma unroll
            for (int s = 0; s < NS; ++s) {               // NS is even: stage and fragment buffer indices are static
                const int k = k0 + s;
                __builtin_amdgcn_sched_barrier(0);
                __builtin_amdgcn_s_waitcnt(waitcnt_vm((NS - 3) * LPT));      // chunk k+1 has landed (this wave's part)
                __builtin_amdgcn_s_barrier();                               // ... and everybody's; stage (k-1) % NS is free
                issue((s + NS - 1) % NS, k + NS - 1);                       // first: the loads are what the loop waits for
                read_frags(ring + ((s + 1) % NS) * G::STAGE, (s + 1) & 1);
                mma_and_norms(s & 1, k);
            }
        }
        if (clean) {
            static_assert(NS == 4, "the last block is written for four stages");
            auto last = [&](auto S) {
                constexpr int s = decltype(S)::value;
                const int k = nsteps - NS + s;
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (s < NS - 1) {               // chunk k+1 exists: wait for it; chunks k+2 .. nsteps-1 may fly
                    __builtin_amdgcn_s_waitcnt(waitcnt_vm((s == 0 ? NS - 3 : NS - 2 - s) * LPT));
                    __builtin_amdgcn_s_barrier();
                    if constexpr (s == 0) issue(NS - 1, k + NS - 1);
                    read_frags(ring + ((s + 1) % NS) * G::STAGE, (s + 1) & 1);
                }
                mma_and_norms(s & 1, k);
            };
            last(std::integral_constant<int, 0>{});
            last(std::integral_constant<int, 1>{});
            last(std::integral_constant<int, 2>{});
            last(std::integral_constant<int, 3>{});
        }
        __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));        // (general form) surplus loads must land before the ring is reused
        ADA_CLK(4);
        ssa += __shfl_xor(ssa, 32, 64);                    // the two lane halves hold different k pieces
        ssb += __shfl_xor(ssb, 32, 64);
        __syncthreads();                                  // every wave is done with the ring
        ADA_CLK(16);
        if (half == 0) {                                  // two partial sums per row and K-group
            ssq[(g * 2 + wb) * 128 + wa * 32 + l32] = ssa;
            ssq[(g * 2 + wa) * 128 + B + wb * 32 + l32] = ssb;
        }
    } else {
    u32x4 pre[D][LPT];
    float ss[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) ss[j] = 0.f;

    auto fetch = [&](int set, int k) {
#pragma unroll
        for (int j = 0; j < LPT; ++j)
            pre[set][j] = fetch_piece<In, ALIGNED>(rowp[j], (k * KG + g) * EPC + pc * EPP, p.d);
    };
    auto store = [&](char* stage, int set, int k) {
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            const u32x4 v = finish_piece<ALIGNED>(pre[set][j], (k * KG + g) * EPC + pc * EPP, p.d);
            *reinterpret_cast<u32x4*>(stage + woff[j]) = v;
            ss[j] += piece_sumsq_fast<In>(v);            // Section 2.1: ||x||^2 from the registers already in hand
        }
    };
    // software pipeline: see gram_tile; steps past the end handle all-zero chunks
#pragma unroll
    for (int s = 0; s < D; ++s) {
        fetch(s, s);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (!p.assign_mode) mark_inherited();
    store(buf0, 0, 0);
    fetch(0, D);
    __builtin_amdgcn_sched_barrier(0);
    store(buf1, 1, 1);
    fetch(1, D + 1);
    __builtin_amdgcn_sched_barrier(0);
    ADA_CLK(2);
    __syncthreads();
    ADA_CLK(3);
    read_frags(buf0, 0);
    for (int k0 = 0; k0 < nsteps; k0 += D) {
#pragma unroll
        for (int s = 0; s < D; ++s) {
            const int k = k0 + s;
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            read_frags((s & 1) ? buf0 : buf1, (s + 1) & 1);
            store((s & 1) ? buf1 : buf0, (s + 2) % D, k + 2);
            fetch((s + 2) % D, k + 2 + D);
            mma(s & 1);
        }
    }

    ADA_CLK(4);
    // ---- norms: 8 consecutive lanes staged one row
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        float v = ss[j];
        v += __shfl_xor(v, 1, 64);
        v += __shfl_xor(v, 2, 64);
        v += __shfl_xor(v, 4, 64);
        ss[j] = v;
    }
    __syncthreads();                                      // every wave is done with the stages
    ADA_CLK(16);
    if (pc == 0) {
#pragma unroll
        for (int j = 0; j < LPT; ++j) ssq[g * 128 + rb + 32 * j] = ss[j];
    }
    }
    // the second K-group hands its partial blocks over through LDS as 16-byte vectors: slot (wave * 4 + q) * 64 + lane
    // holds accumulator registers 4q .. 4q+3 (consecutive lanes, consecutive 16 bytes: conflict-free)
    f32x16 tot;
#pragma unroll
    for (int i = 0; i < 16; ++i) tot[i] = acc[0][i] + acc[1][i];
    f32x4* red = reinterpret_cast<f32x4*>(body);
    if (KG == 2 && g == 1) {
#pragma unroll
        for (int q = 0; q < 4; ++q) red[(wave * 4 + q) * 64 + lane] = f32x4{tot[4 * q], tot[4 * q + 1], tot[4 * q + 2], tot[4 * q + 3]};
    }
    __syncthreads();
    ADA_CLK(17);
    if (tid < 2 * B) {
        float sum = 0.f;
#pragma unroll
        for (int part = 0; part < G::NPART; ++part) sum += ssq[part * 128 + tid];
        float sc = sum > 0.f ? 1.0f / sqrtf(sum) : 0.f;   // a zero row normalises to zero: all its cosines are 0
        if (tid < B ? (s_tok[tid] == INT_MAX) : (t0 + tid - B >= p.T)) sc = 0.f;
        scale[tid] = sc;
    }
    if (KG == 2 && g == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 o = red[(wave * 4 + q) * 64 + lane];
#pragma unroll
            for (int e = 0; e < 4; ++e) tot[4 * q + e] += o[e];
        }
    }
    __syncthreads();
    ADA_CLK(18);
    ADA_CLK(19);
    if (g == 0) {
        const int a = wa, b = wb;
        const int nl = b * 32 + l32;
        const int t = t0 + nl;
        finish_block(p, tot, s_tok + a * 32, scale + a * 32, scale[B + nl], (repf[nl] != 0 ? 3 : 0) | (p.earlier_only ? 1 : 0), t,
                     sb * 2 + a, half);
    }
    ADA_CLK(5);
}

// The same step on a wider tile: BR = 32 RB representatives (RB = 2 or 4) against 128 tested tokens, 8 waves on one
// chunk at a time, rows in whole aligned 128-byte chunks.  Per Gram entry the 128 x 128 tile pulls half and the
// 64 x 128 tile three quarters of the 64 x 64 tile's L2 -> CU bytes; they pay when the step has enough tiles to keep
// the CUs busy anyway.  The 32 x 32 blocks are dealt to the waves in row-major order, NBW = RB / 2 token blocks per
// wave: wave w owns representative block wa = w / WPB and token blocks NBW (w % WPB) ... (WPB = 8 / RB waves share
// a representative block).
template <typename In, int RB>
__device__ inline void fused_tile_wide(const FusedParams& p, int r, int s0, int t0, char* lds) {
    using G = FusedGeom<2, true>;
    static_assert(RB == 2 || RB == 4, "64 or 128 representatives per tile");
    constexpr int BR = 32 * RB, BT = 128, ROWS = BR + BT, EPP = 16 / (int)sizeof(In), EPC = 8 * EPP;
    constexpr int LPT = ROWS / 64, LR = BR / 64, NS = 4, STAGE = ROWS * 128, NBW = RB / 2, WPB = 8 / RB;
    static_assert(NS * STAGE <= G::BODY, "ring does not fit");
    int* s_tok = reinterpret_cast<int*>(lds + G::OFF_BIG);       // [BR] (room for 128)
    int* repf = s_tok + 128;                                     // [128]
    float* ssq = reinterpret_cast<float*>(repf + 128);           // [ROWS] sums of squares (room for 256)
    float* scale = ssq + 256;                                    // [ROWS]
    char* ring = lds + G::META;

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wa = wave / WPB, wp = wave % WPB, b0 = NBW * wp;
    const In* X = reinterpret_cast<const In*>(p.X);

    // lane l of wave w serves stage rows 8 w + l / 8 + 64 j (slot l % 8): j < LR are representatives, the rest tokens
    const int r8 = lane >> 3;
    int ptok[LR];
#pragma unroll
    for (int j = 0; j < LR; ++j) {
        const int li = s0 + wave * 8 + r8 + 64 * j;
        ptok[j] = list_at(p, li < r ? li : r - 1);
    }
    if (tid < BR) {
        const int li = s0 + tid;
        const bool ok = li < r;
        int tok = list_at(p, ok ? li : r - 1);
        tok = min(max(tok, 0), p.T - 1);
        s_tok[tid] = ok ? tok : INT_MAX;
    }
    if (tid < BT) repf[tid] = 0;
    __syncthreads();
    const int pcd = (lane & 7) ^ lds_swz(wave * 8 + r8);          // 64 j leaves bits 0..3 of the row alone
    const In* rowp[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int row = wave * 8 + r8 + 64 * j;
        int tok;
        if (j < LR) tok = min(max(ptok[j < LR ? j : 0], 0), p.T - 1);
        else tok = min(t0 + row - BR, p.T - 1);
        rowp[j] = X + (size_t)tok * (size_t)p.ld + pcd * EPP;
    }
    const int nk = p.d / EPC;
    auto issue = [&](int stage, int k) {
        const int chunk = min(k, nk - 1);                        // surplus issues repeat the last chunk into a dead stage
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            char* dst = ring + stage * STAGE + (wave * 8 + 64 * j) * 128;      // wave-uniform
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(rowp[j] + chunk * EPC),
                                             (void __attribute__((address_space(3)))*)dst, 16, 0, 0);
        }
    };
    u32x4 fa[2][4], fb[2][NBW][4];
    f32x16 acc[NBW];
#pragma unroll
    for (int c = 0; c < NBW; ++c)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[c][i] = 0.f;
    auto read_frags = [&](const char* stage, int f) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int piece = 2 * ks + half;
            fa[f][ks] = *reinterpret_cast<const u32x4*>(stage + lds_off(wa * 32 + l32, piece));
#pragma unroll
            for (int c = 0; c < NBW; ++c)
                fb[f][c][ks] = *reinterpret_cast<const u32x4*>(stage + lds_off(BR + (b0 + c) * 32 + l32, piece));
        }
    };
    float ssa = 0.f, ssb[NBW];
#pragma unroll
    for (int c = 0; c < NBW; ++c) ssb[c] = 0.f;
    // Section 2.1: ||x||^2 from the fragments already in hand.  Every block of rows is summed by ONE of the waves that
    // hold it, chosen so that no wave sums more than eight fragments per chunk.
    //   RB = 4: representative block wa by waves (0,1) (1,1) (2,0) (3,0); token blocks 2 wp, 2 wp + 1 by (0,0) and (3,1)
    //   RB = 2: representative block wa by waves (0,1) and (1,2); token block wp by waves (0,0) (1,1) (0,2) (1,3)
    const bool do_a = RB == 4 ? (wa < 2 ? wp == 1 : wp == 0) : (wp == wa + 1);
    const bool do_b = RB == 4 ? (wp == 0 ? wa == 0 : wa == 3) : (wa == (wp & 1));
    auto mma_and_norms = [&](int f, int k) {
        if (k < nk) {                                            // scalar: a clamped (repeated) chunk is skipped
#pragma unroll
            for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                for (int c = 0; c < NBW; ++c) Mfma<In>::run(acc[c], fa[f][ks], fb[f][c][ks]);
            // The choice is a plain scalar branch around code with fixed registers: selecting fragments by a computed
            // index sends them through scratch memory, whose loads count in vmcnt and drain the ring.
            if (do_a) {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) ssa += piece_sumsq_fast<In>(fa[f][ks]);
            }
            if (do_b) {
#pragma unroll
                for (int ks = 0; ks < 4; ++ks)
#pragma unroll
                    for (int c = 0; c < NBW; ++c) ssb[c] += piece_sumsq_fast<In>(fb[f][c][ks]);
            }
        }
    };
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue(s, s);
    if (!p.assign_mode) {                                        // which tested tokens are inherited (read in the epilogue)
        for (int j = tid; j < r; j += G::THREADS) {
            const unsigned q = (unsigned)(list_at(p, j) - t0);
            if (q < (unsigned)BT) repf[q] = 1;
        }
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    __builtin_amdgcn_s_barrier();
    read_frags(ring, 0);
    const bool clean = nk % NS == 0;                             // see fused_tile: the last block on its own
    const int nmain = clean ? nk - NS : nk;
    for (int k0 = 0; k0 < nmain; k0 += NS) {
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const int k = k0 + s;
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_waitcnt(waitcnt_vm((NS - 3) * LPT));   // chunk k+1 has landed (this wave's part)
            __builtin_amdgcn_s_barrier();                            // ... and everybody's; stage (k-1) % NS is free
            issue((s + NS - 1) % NS, k + NS - 1);
            read_frags(ring + ((s + 1) % NS) * STAGE, (s + 1) & 1);
            mma_and_norms(s & 1, k);
        }
    }
    if (clean) {
        static_assert(NS == 4, "the last block is written for four stages");
        auto last = [&](auto S) {
            constexpr int s = decltype(S)::value;
            const int k = nk - NS + s;
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (s < NS - 1) {
                __builtin_amdgcn_s_waitcnt(waitcnt_vm((s == 0 ? NS - 3 : NS - 2 - s) * LPT));
                __builtin_amdgcn_s_barrier();
                if constexpr (s == 0) issue(NS - 1, k + NS - 1);
                read_frags(ring + ((s + 1) % NS) * STAGE, (s + 1) & 1);
            }
            mma_and_norms(s & 1, k);
        };
        last(std::integral_constant<int, 0>{});
        last(std::integral_constant<int, 1>{});
        last(std::integral_constant<int, 2>{});
        last(std::integral_constant<int, 3>{});
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));                    // (general form) surplus loads must land before the ring is reused
    ssa += __shfl_xor(ssa, 32, 64);                               // the two lane halves hold different k pieces
#pragma unroll
    for (int c = 0; c < NBW; ++c) ssb[c] += __shfl_xor(ssb[c], 32, 64);
    __syncthreads();
    if (half == 0) {
        if (do_a) ssq[wa * 32 + l32] = ssa;
        if (do_b) {
#pragma unroll
            for (int c = 0; c < NBW; ++c) ssq[BR + (b0 + c) * 32 + l32] = ssb[c];
        }
    }
    __syncthreads();
    if (tid < ROWS) {
        const float sum = ssq[tid];
        float sc = sum > 0.f ? 1.0f / sqrtf(sum) : 0.f;           // a zero row normalises to zero: all its cosines are 0
        if (tid < BR ? (s_tok[tid] == INT_MAX) : (t0 + tid - BR >= p.T)) sc = 0.f;
        scale[tid] = sc;
    }
    __syncthreads();
#pragma unroll
    for (int c = 0; c < NBW; ++c) {
        const int nl = (b0 + c) * 32 + l32;
        finish_block(p, acc[c], s_tok + wa * 32, scale + wa * 32, scale[BR + nl], (repf[nl] != 0 ? 3 : 0) | (p.earlier_only ? 1 : 0),
                     t0 + nl, (s0 >> 5) + wa, half);
    }
}

// s_waitcnt vmcnt(n) lgkmcnt(0): the direct-to-LDS loads are counted, every LDS read of this wave has returned
constexpr int waitcnt_vm_lgkm0(int n) { return 0x0070 | (n & 15) | ((n >> 4) << 14); }

// The same step with the hand-ordered ring of the direct-to-LDS full-Gram kernel (k_gram_dma), for bf16 rows in whole
// aligned 128-byte chunks: 128 NT tested tokens (MFMA N side) against 64 NR inherited representatives (M side); eight
// waves as 4 (tokens) x 2 (representatives), each holding a 32 NT x 32 NR block of accumulators over ALL of K, two
// waves per SIMD.  Operands go global -> LDS in whole 128-byte chunks (one cache line per row and stage: what the
// memory side serves at its best rate is requests, not bytes, so a line is asked for once and whole), a ring of NS
// stages; the order of fragment reads, barrier, loads and MFMAs is pinned by hand, the waits are counted, and there
// is one barrier per chunk (four k-steps).  Operand requests per Gram entry fall as 1 / tokens + 1 / representatives,
// which is why the tile is as large as the step's tile count allows.  Sums of squares (Section 2.1) come from the
// fragments in hand, every 32-row block summed by exactly one of the waves that hold it.
template <int NT, int NR>
__device__ inline void fused_tile_ring(const FusedParams& p, int r, int s0, int t0, char* lds) {
    using G = FusedGeom<2, true>;
    constexpr int BR = 64 * NR, BT = 128 * NT, ROWS = BR + BT, EPC = 64, STAGE = ROWS * 128;
    constexpr int NS = 4 * STAGE <= G::BODY ? 4 : 3;
    static_assert(ROWS % 64 == 0, "every wave issues the same number of 8-row loads per stage");
    constexpr int LPT = ROWS / 64;
    static_assert(NS * STAGE <= G::RINGMAX, "ring does not fit");
    static_assert(BR <= 256 && BT <= 256, "metadata area");
    int* s_tok = reinterpret_cast<int*>(lds + G::OFF_BIG);        // [BR] token id of each representative row (INT_MAX: none)
    int* repf = s_tok + 256;                                      // [BT] tested token is inherited
    float* ssq = reinterpret_cast<float*>(repf + 256);            // [ROWS] sums of squares
    float* scale = ssq + 512;                                     // [ROWS] 1 / norm (0 for rows that do not exist)
    char* ring = lds + G::META;

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wt = wave & 3, wr = wave >> 2;
    const uint16_t* X = reinterpret_cast<const uint16_t*>(p.X);
    const int T = p.T;

    // One load instruction fills 1 KB = 8 rows of a stage: lane l serves row l / 8, slot l % 8, and fetches piece
    // (l % 8) ^ lds_swz(row), which reproduces the XOR-swizzled layout the fragment reads expect (see fused_tile).
    // Instruction j of wave w covers rows 8 (8 j + w) ...; rows below BR are representatives (through the list), the
    // rest tested tokens.
    const int r8 = lane >> 3;
    int ptok[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int row = (j * 8 + wave) * 8 + r8;
        const int li = s0 + min(row, BR - 1);
        ptok[j] = list_at(p, li < r ? li : r - 1);               // every list entry is requested before anything waits
    }
    for (int i = tid; i < BR; i += G::THREADS) {
        const int li = s0 + i;
        const bool ok = li < r;
        int tok = list_at(p, ok ? li : r - 1);
        tok = min(max(tok, 0), T - 1);
        s_tok[i] = ok ? tok : INT_MAX;
    }
    for (int i = tid; i < BT; i += G::THREADS) repf[i] = 0;
    const int pcd = (lane & 7) ^ lds_swz(wave * 8 + r8);          // 64 j leaves bits 0..3 of the row alone
    const uint16_t* rowp[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int row = (j * 8 + wave) * 8 + r8;
        const int tok = row < BR ? min(max(ptok[j], 0), T - 1) : min(t0 + row - BR, T - 1);
        rowp[j] = X + (size_t)tok * (size_t)p.ld + pcd * 8;
    }
    const int nk = p.d / EPC;
    auto issue = [&](int stage_off, int k) {
        const int chunk = min(k, nk - 1);                        // surplus issues repeat the last chunk into a dead stage
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            char* dst = ring + stage_off + (j * 8 + wave) * 1024;                // wave-uniform
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(rowp[j] + chunk * EPC),
                                             (void __attribute__((address_space(3)))*)dst, 16, 0, 0);
        }
    };
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue(s * STAGE, s);
    __syncthreads();                                              // (drains the loads above as well: the prologue waits anyway)
    if (!p.assign_mode) {                                         // which tested tokens are inherited (read in the epilogue)
        for (int j = tid; j < r; j += G::THREADS) {
            const unsigned q = (unsigned)(list_at(p, j) - t0);
            if (q < (unsigned)BT) repf[q] = 1;
        }
    }

    f32x16 acc[NR][NT];
#pragma unroll
    for (int a = 0; a < NR; ++a)
#pragma unroll
        for (int b = 0; b < NT; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    // Which 32-row blocks a wave holds, in which order.  A token block is held by the two waves wr = 0, 1 and a
    // representative block by the four waves wt = 0 .. 3; each block's sum of squares is needed once.  So that the K loop
    // stays straight-line code (a branch per block would cut it into pieces and undo the pinned order), every wave sums
    // the blocks at FIXED local positions -- its representative block 0 and its even token blocks -- and the local order
    // is permuted per wave so that those positions cover every block: local representative block a is block
    // a ^ (wt % NR) of the wave's NR, local token block b is block b ^ wr of its NT (NT >= 2).  Where more waves hold a
    // block than are needed (wt >= NR; wr = 1 with NT = 1) the surplus sums are simply not written.
    constexpr int PR = NR >= 4 ? 3 : NR - 1, PT = NT >= 2 ? 1 : 0;
    static_assert(NR <= 4, "a representative block is summed by one of four waves");
    int ablk[NR], bblk[NT];                                       // block index within the tile's representative / token rows
#pragma unroll
    for (int a = 0; a < NR; ++a) ablk[a] = wr * NR + (a ^ (wt & PR));
#pragma unroll
    for (int b = 0; b < NT; ++b) bblk[b] = wt * NT + (b ^ (wr & PT));
    // fragment addresses: row l32 of a 32-row block, piece 2 ks + half of the chunk (k-step ks of four)
    const char* aptr[4][NR];
    const char* bptr[4][NT];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int a = 0; a < NR; ++a) aptr[ks][a] = ring + lds_off(ablk[a] * 32 + l32, 2 * ks + half);
#pragma unroll
        for (int b = 0; b < NT; ++b) bptr[ks][b] = ring + lds_off(BR + bblk[b] * 32 + l32, 2 * ks + half);
    }
    u32x4 fa[2][NR], fb[2][NT];
    auto read_frags = [&](int set, int stage_off, int ks) {
#pragma unroll
        for (int a = 0; a < NR; ++a) fa[set][a] = *reinterpret_cast<const u32x4*>(aptr[ks][a] + stage_off);
#pragma unroll
        for (int b = 0; b < NT; ++b) fb[set][b] = *reinterpret_cast<const u32x4*>(bptr[ks][b] + stage_off);
    };
    float ssa = 0.f, ssb[(NT + 1) / 2];
#pragma unroll
    for (int b = 0; b < (NT + 1) / 2; ++b) ssb[b] = 0.f;
    auto mma = [&](int set) {
#pragma unroll
        for (int a = 0; a < NR; ++a)
#pragma unroll
            for (int b = 0; b < NT; ++b) Mfma<uint16_t>::run(acc[a][b], fa[set][a], fb[set][b]);
        ssa += piece_sumsq_fast<uint16_t>(fa[set][0]);            // Section 2.1: ||x||^2 from the fragments in hand
#pragma unroll
        for (int b = 0; b < NT; b += 2) ssb[b >> 1] += piece_sumsq_fast<uint16_t>(fb[set][b]);
    };
    // Chunk k (four k-steps) with the fragments of its k-step 0 already in set 0.  The fragments of k-step i + 1 are
    // read while k-step i multiplies; before the last k-step comes the barrier that opens chunk k + 1 (everybody's part
    // of it has landed, and everybody has read the last fragments of chunk k), then the fragment reads of its k-step 0
    // and the loads of chunk k + NS into the stage just left, issued in the shadow of the last k-step's MFMAs.
    auto step = [&](int cur_off, int nxt_off, int k) {
        __builtin_amdgcn_sched_barrier(0);
        read_frags(1, cur_off, 1);
        mma(0);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(0, cur_off, 2);
        mma(1);
        __builtin_amdgcn_sched_barrier(0);
        read_frags(1, cur_off, 3);
        mma(0);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NS - 2) * LPT));   // chunk k + 1 has landed (this wave's part)
        __builtin_amdgcn_s_barrier();
        read_frags(0, nxt_off, 0);
        issue(cur_off, k + NS);
        mma(1);
        __builtin_amdgcn_sched_group_barrier(0x100, NR + NT, 0);  // the LDS reads first
        constexpr int PAIRS = NR * NT < LPT ? NR * NT : LPT;
#pragma unroll
        for (int j = 0; j < PAIRS; ++j) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);    // then one MFMA ...
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);    // ... per global load
        }
        if constexpr (LPT > PAIRS) __builtin_amdgcn_sched_group_barrier(0x020, LPT - PAIRS, 0);
        if constexpr (NR * NT > PAIRS) __builtin_amdgcn_sched_group_barrier(0x008, NR * NT - PAIRS, 0);
    };
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));              // chunks 0 .. NS - 2 and the list have landed (this wave's part)
    __builtin_amdgcn_s_barrier();
    issue((NS - 1) * STAGE, NS - 1);
    read_frags(0, 0, 0);
    int k = 0;
    for (; k + NS < nk; k += NS) {                               // every step here has a successor: no branches inside
#pragma unroll
        for (int s = 0; s < NS; ++s) step(s * STAGE, ((s + 1) % NS) * STAGE, k + s);
    }
    for (; k + 1 < nk; ++k) step((k % NS) * STAGE, ((k + 1) % NS) * STAGE, k);
    {                                                            // last chunk
        const int off = (k % NS) * STAGE;
        __builtin_amdgcn_sched_barrier(0);
        read_frags(1, off, 1);
        mma(0);
        read_frags(0, off, 2);
        mma(1);
        read_frags(1, off, 3);
        mma(0);
        mma(1);
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));             // surplus loads land before the ring is reused
    ssa += __shfl_xor(ssa, 32, 64);                               // the two lane halves hold different k pieces
#pragma unroll
    for (int b = 0; b < (NT + 1) / 2; ++b) ssb[b] += __shfl_xor(ssb[b], 32, 64);
    if (half == 0) {
        if (wt < NR) ssq[ablk[0] * 32 + l32] = ssa;
        if (NT >= 2 || wr == 0) {
#pragma unroll
            for (int b = 0; b < NT; b += 2) ssq[BR + bblk[b] * 32 + l32] = ssb[b >> 1];
        }
    }
    __syncthreads();
    for (int i = tid; i < ROWS; i += G::THREADS) {
        const float sum = ssq[i];
        float sc = sum > 0.f ? 1.0f / sqrtf(sum) : 0.f;          // a zero row normalises to zero: all its cosines are 0
        if (i < BR ? (s_tok[i] == INT_MAX) : (t0 + i - BR >= T)) sc = 0.f;
        scale[i] = sc;
    }
    __syncthreads();
#pragma unroll
    for (int b = 0; b < NT; ++b) {
        const int nl = bblk[b] * 32 + l32;
        const int ordered = (repf[nl] != 0 ? 3 : 0) | (p.earlier_only ? 1 : 0);
        const float tsc = scale[BR + nl];
#pragma unroll
        for (int a = 0; a < NR; ++a)
            finish_block(p, acc[a][b], s_tok + ablk[a] * 32, scale + ablk[a] * 32, tsc, ordered, t0 + nl,
                         (s0 >> 5) + ablk[a], half);
    }
}

// ---- loader waves and multiplying waves (bf16 rows in whole aligned 128-byte chunks) -----------------------------
// A wave that issues a load waits for room in the memory pipeline; where few MFMAs stand against each load, those
// waits add to the MFMA time instead of hiding behind it.  The tiles below therefore run with eight waves: waves
// 4 .. 7 do nothing but issue the loads of the coming chunks (and count them in), waves 0 .. 3 multiply and never
// touch memory inside the K loop.  A ring of NS stages of whole 128-byte chunks (one cache line per row and stage, the
// swizzle of lds_off), ONE barrier per chunk of four k-steps, which both kinds of wave meet: a loader when its part of
// the next chunk has landed, a multiplier when its reads of the current one have returned.
constexpr int SPLIT_EPC = 64;                                 // elements per chunk

// The loader waves' K loop: LPT instructions of 1 KB (8 rows x 128 bytes) per wave and chunk; instruction j of loader
// wave w fills rows 8 (4 j + w) .. + 7 of the stage, lane l row l / 8 of them; tok_of(j, row): the row of X to fetch.
template <int NS, int LPT, int STAGE, typename TokOf>
__device__ inline void split_loader(const uint16_t* X, long long ld, int d, char* ring, int wave, int lane, TokOf tok_of) {
    static_assert(NS >= 3 && (NS - 1) * LPT < 64, "the loads in flight can be counted");
    const int r8 = lane >> 3;
    const int pcd = (lane & 7) ^ lds_swz(wave * 8 + r8);       // (32 j leaves bits 0..3 of the row alone)
    const uint16_t* rowp[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) rowp[j] = X + (size_t)tok_of(j, (j * 4 + wave) * 8 + r8) * (size_t)ld + pcd * 8;
    const int nk = d / SPLIT_EPC;
    auto issue = [&](int stage_off, int k) {
        const int chunk = min(k, nk - 1);                      // surplus issues repeat the last chunk into a dead stage
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
            char* dst = ring + stage_off + (j * 4 + wave) * 1024;               // wave-uniform
            __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(rowp[j] + chunk * SPLIT_EPC),
                                             (void __attribute__((address_space(3)))*)dst, 16, 0, 0);
        }
    };
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue(s * STAGE, s);
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NS - 2) * LPT));   // chunk 0 has landed (this wave's part)
    __builtin_amdgcn_s_barrier();
    issue((NS - 1) * STAGE, NS - 1);
    for (int k = 0; k + 1 < nk; ++k) {                         // the barrier of step k: k + 1 has landed, k is free
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0((NS - 2) * LPT));
        __builtin_amdgcn_s_barrier();
        issue((k % NS) * STAGE, k + NS);
    }
}

// The multiplying waves' K loop around read(set, stage_off, ks) and mma(set): the fragments of k-step ks + 1 are read
// while k-step ks multiplies; the barrier sits before the last k-step of a chunk.
template <int NS, int STAGE, typename Read, typename Mma>
__device__ inline void split_multiplier(int nk, Read read, Mma mma) {
    auto cstep = [&](int cur_off, int nxt_off) {
        __builtin_amdgcn_sched_barrier(0);
        read(1, cur_off, 1);
        mma(0);
        __builtin_amdgcn_sched_barrier(0);
        read(0, cur_off, 2);
        mma(1);
        __builtin_amdgcn_sched_barrier(0);
        read(1, cur_off, 3);
        mma(0);
        __builtin_amdgcn_sched_barrier(0);
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(63));     // my reads of this stage have returned
        __builtin_amdgcn_s_barrier();
        read(0, nxt_off, 0);
        mma(1);
        __builtin_amdgcn_sched_barrier(0);
    };
    __builtin_amdgcn_s_barrier();                              // chunk 0 has landed
    read(0, 0, 0);
    int k = 0;
    for (; k + NS < nk; k += NS) {
#pragma unroll
        for (int s = 0; s < NS; ++s) cstep(s * STAGE, ((s + 1) % NS) * STAGE);
    }
    for (; k + 1 < nk; ++k) cstep((k % NS) * STAGE, ((k + 1) % NS) * STAGE);
    const int last_off = (k % NS) * STAGE;                     // last chunk
    __builtin_amdgcn_sched_barrier(0);
    read(1, last_off, 1);
    mma(0);
    read(0, last_off, 2);
    mma(1);
    read(1, last_off, 3);
    mma(0);
    mma(1);
}

// One step's tile on that scheme: 128 NT tested tokens (MFMA N side) against 64 NR inherited representatives (M side);
// the multiplying waves are a 2 (representatives) x 2 (tokens) grid, each holding NR x 2 NT blocks of 32 x 32 over ALL of
// K.  Operand requests per Gram entry fall as 1 / tokens + 1 / representatives, which is why the tile is as large as the
// step's tile count allows.  Sums of squares (Section 2.1) come from the fragments in hand: a 32-row block is held by
// two waves, each wave sums the blocks at its even local positions, and the local order of a wave's blocks is permuted
// (block a ^ parity) so that those positions cover every block and the K loop stays straight-line code.
template <int NT, int NR>
__device__ inline void fused_tile_split(const FusedParams& p, int r, int s0, int t0, char* lds) {
    using G = FusedGeom<2, true>;
    constexpr int BR = 64 * NR, BT = 128 * NT, ROWS = BR + BT, STAGE = ROWS * 128;
    constexpr int NS = 4 * STAGE <= G::BODY ? 4 : 3;
    constexpr int LPT = ROWS / 32, NA = NR, NB = 2 * NT;
    static_assert(NS * STAGE <= G::RINGMAX, "ring does not fit");
    static_assert(BR <= 256 && BT <= 256 && G::THREADS == 512, "metadata area; four loader and four multiplying waves");
    int* s_tok = reinterpret_cast<int*>(lds + G::OFF_BIG);        // [BR] token id of each representative row (INT_MAX: none)
    int* repf = s_tok + 256;                                      // [BT] tested token is inherited
    float* ssq = reinterpret_cast<float*>(repf + 256);            // [ROWS] sums of squares
    float* scale = ssq + 512;                                     // [ROWS] 1 / norm (0 for rows that do not exist)
    char* ring = lds + G::META;

    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave8 >= 4;
    const int wave = wave8 & 3;                                   // place among the waves of its kind
    const int wr = wave >> 1, wt = wave & 1;
    const int T = p.T;

    // the loaders' representative rows go through the list: every entry is requested before anything waits
    int ptok[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int row = (j * 4 + wave) * 8 + (lane >> 3);
        const int li = s0 + min(row, BR - 1);
        ptok[j] = loader ? list_at(p, li < r ? li : r - 1) : 0;
    }
    for (int i = tid; i < BR; i += G::THREADS) {
        const int li = s0 + i;
        const bool ok = li < r;
        int tok = list_at(p, ok ? li : r - 1);
        tok = min(max(tok, 0), T - 1);
        s_tok[i] = ok ? tok : INT_MAX;
    }
    for (int i = tid; i < BT; i += G::THREADS) repf[i] = 0;
    __syncthreads();

    f32x16 acc[NA][NB];
    // local block a of this wave is block a ^ pa of its NA representative blocks, likewise b ^ pb for its token blocks
    const int pa = NA > 1 ? wt : 0, pb = wr;
    constexpr int DA = (NA + 1) / 2, DB = NB / 2;                // blocks a wave sums on each side
    float ssa[DA], ssb[DB];
    if (loader) {
        split_loader<NS, LPT, STAGE>(reinterpret_cast<const uint16_t*>(p.X), p.ld, p.d, ring, wave, lane,
            [&](int j, int row) { return row < BR ? min(max(ptok[j], 0), T - 1) : min(t0 + row - BR, T - 1); });
    } else {
        if (!p.assign_mode) {                                     // which tested tokens are inherited (read in the epilogue)
            for (int j = tid; j < r; j += G::THREADS / 2) {
                const unsigned q = (unsigned)(list_at(p, j) - t0);
                if (q < (unsigned)BT) repf[q] = 1;
            }
        }
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
        // Fragment addresses: row l32 of a 32-row block, piece 2 ks + half of the chunk (k-step ks of four).  Within a
        // stage the offset of (local block, k-step) is one base per side XOR a constant: a block is 4096 bytes, the
        // local order flips block bits (a ^ pa), and the swizzled slot (2 ks + half) ^ swz is (half ^ swz) ^ 2 ks; so
        // two registers hold what 4 (NA + NB) pointers would.
        static_assert((NA & (NA - 1)) == 0 && (NB & (NB - 1)) == 0 && BR % (32 * NB) == 0, "block bits do not carry");
        const uint32_t abase = (uint32_t)lds_off((wr * NA + pa) * 32 + l32, half);
        const uint32_t bbase = (uint32_t)lds_off(BR + (wt * NB + pb) * 32 + l32, half);
        u32x4 fa[2][NA], fb[2][NB];
        split_multiplier<NS, STAGE>(p.d / SPLIT_EPC,
            [&](int set, int stage_off, int ks) {
                uint32_t ab = abase, bb = bbase;               // (opaque: the XORs are redone here, not kept in 24 registers)
                asm volatile("" : "+v"(ab), "+v"(bb));
#pragma unroll
                for (int a = 0; a < NA; ++a)
                    fa[set][a] = *reinterpret_cast<const u32x4*>(ring + stage_off + (ab ^ (uint32_t)((a << 12) | (ks << 5))));
#pragma unroll
                for (int b = 0; b < NB; ++b)
                    fb[set][b] = *reinterpret_cast<const u32x4*>(ring + stage_off + (bb ^ (uint32_t)((b << 12) | (ks << 5))));
            },
            [&](int set) {
#pragma unroll
                for (int a = 0; a < NA; ++a)
#pragma unroll
                    for (int b = 0; b < NB; ++b) Mfma<uint16_t>::run(acc[a][b], fa[set][a], fb[set][b]);
#pragma unroll
                for (int i = 0; i < NA; i += 2) ssa[i >> 1] += piece_sumsq_fast<uint16_t>(fa[set][i]);   // Section 2.1
#pragma unroll
                for (int i = 0; i < NB; i += 2) ssb[i >> 1] += piece_sumsq_fast<uint16_t>(fb[set][i]);
            });
    }
    __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(0));             // surplus loads land before the ring is reused
    if (!loader) {
        // the two lane halves hold different k pieces (a block summed by two waves gets the same bits from both)
#pragma unroll
        for (int i = 0; i < DA; ++i) {
            const float v = ssa[i] + __shfl_xor(ssa[i], 32, 64);
            if (half == 0) ssq[(wr * NA + ((2 * i) ^ pa)) * 32 + l32] = v;
        }
#pragma unroll
        for (int i = 0; i < DB; ++i) {
            const float v = ssb[i] + __shfl_xor(ssb[i], 32, 64);
            if (half == 0) ssq[BR + (wt * NB + ((2 * i) ^ pb)) * 32 + l32] = v;
        }
    }
    __syncthreads();
    for (int i = tid; i < ROWS; i += G::THREADS) {
        const float sum = ssq[i];
        float sc = sum > 0.f ? 1.0f / sqrtf(sum) : 0.f;          // a zero row normalises to zero: all its cosines are 0
        if (i < BR ? (s_tok[i] == INT_MAX) : (t0 + i - BR >= T)) sc = 0.f;
        scale[i] = sc;
    }
    __syncthreads();
    if (loader) return;                                           // (no barrier follows inside the tile)
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int nl = (wt * NB + (b ^ pb)) * 32 + l32;
        const int ordered = (repf[nl] != 0 ? 3 : 0) | (p.earlier_only ? 1 : 0);
        const float tsc = scale[BR + nl];
#pragma unroll
        for (int a = 0; a < NA; ++a) {
            const int ablk = wr * NA + (a ^ pa);
            finish_block(p, acc[a][b], s_tok + ablk * 32, scale + ablk * 32, tsc, ordered, t0 + nl, (s0 >> 5) + ablk, half);
        }
    }
}

// exclusive prefix sum of one 64-bit value per thread over the workgroup (three 21-bit counters ride in one scan)
__device__ inline unsigned long long block_exclusive_scan64(unsigned long long v, unsigned long long* total,
                                                            unsigned long long* wave_tot /* >= 17 words of LDS */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    unsigned long long inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned lo = __shfl_up((unsigned)inc, o, 64), hi = __shfl_up((unsigned)(inc >> 32), o, 64);
        if (lane >= o) inc += ((unsigned long long)hi << 32) | lo;
    }
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long run = 0;
        for (int w = 0; w < nw; ++w) { const unsigned long long t = wave_tot[w]; wave_tot[w] = run; run += t; }
        wave_tot[16] = run;
    }
    __syncthreads();
    *total = wave_tot[16];
    return wave_tot[wave] + inc - v;
}

// Ranks for stream compaction of three classes at once: thread tid owns U consecutive items, f[c][u] says whether item
// u is in class c.  below[c] = members of class c among the items of all threads before this one, tot[c] = members in
// the workgroup.  Inside a wave the counts come from ballots (no cross-lane data movement); across waves from one
// exchange through LDS (scratch: THREADS / 64 x 4 ints).
template <int THREADS, int U>
__device__ inline void block_rank3(const bool (&f)[3][U], int (&below)[3], int (&tot)[3], int* scratch) {
    constexpr int NW = THREADS / 64;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int wtot[3];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
        below[c] = 0;
        wtot[c] = 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const unsigned long long m = __ballot(f[c][u]);
            below[c] += (int)__builtin_amdgcn_mbcnt_hi((unsigned)(m >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)m, 0u));
            wtot[c] += __popcll(m);
        }
    }
    if (lane == 0) *reinterpret_cast<int4*>(scratch + 4 * wave) = int4{wtot[0], wtot[1], wtot[2], 0};
    __syncthreads();
#pragma unroll
    for (int c = 0; c < 3; ++c) tot[c] = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const int4 v = *reinterpret_cast<const int4*>(scratch + 4 * w);
        const int vv[3] = {v.x, v.y, v.z};
#pragma unroll
        for (int c = 0; c < 3; ++c) {
            tot[c] += vv[c];
            below[c] += w < wave ? vv[c] : 0;
        }
    }
}

// Algorithm 1 steps 5, 9, 10 and the bookkeeping (run by one workgroup).  Two forms: from the first-hit records
// (fused_update_rec, whenever T is a multiple of 4) and from the hit words alone (fused_update's general path).
// In the general path per-token state lives in LDS (T <= FUSED_MAX_T bytes): bit 0 = inherited, bit 1 = kept.  The hit
// table is word-major (hits[w * T + t]), so a thread that owns token t reads its words with loads that are coalesced
// across the workgroup, independent of each other and branch-free (indices are clamped, results masked): a whole batch
// is in flight before the first use.

// Algorithm 1 step 8 for callers that ask for gamma: once validity is known (vmask: one bit per list position), list the
// non-inherited tokens whose nearest inherited representative was removed -- their maximum over the VALID
// representatives is not the one the tiles accumulated -- and clear their gamma for the recomputation.  The arg-max
// keys are cleared on the way (the table is zero between calls).  ok == false: a rejected step, only the clearing is
// done and the list is empty.
template <int THREADS>
__device__ inline void gamma_fix_collect(const FusedParams& p, int r, const uint32_t* vmask, bool ok) {
    if (!p.fix_list) return;                             // uniform
    __shared__ int s_fix;
    const int tid = threadIdx.x;
    if (tid == 0) s_fix = 0;
    __syncthreads();
    auto one = [&](int t, unsigned long long key) {
        if (t >= p.T || key == 0ull) return;
        p.best[t] = 0ull;
        if (!ok) return;
        const int pos = min(max(INT_MAX - (int)(uint32_t)key, 0), r - 1);
        if (!((vmask[pos >> 5] >> (pos & 31)) & 1u)) {
            p.fix_list[atomicAdd(&s_fix, 1)] = t;
            p.gamma[t] = 0.f;                            // empty max: the recomputation accumulates into it
        }
    };
    for (int base = tid; base < p.T; base += 4 * THREADS) {                 // four keys per thread in flight per trip
        const int t0 = base, t1 = base + THREADS, t2 = base + 2 * THREADS, t3 = base + 3 * THREADS;
        const unsigned long long k0 = p.best[min(t0, p.T - 1)], k1 = p.best[min(t1, p.T - 1)];
        const unsigned long long k2 = p.best[min(t2, p.T - 1)], k3 = p.best[min(t3, p.T - 1)];
        one(t0, k0);
        one(t1, k1);
        one(t2, k2);
        one(t3, k3);
    }
    __syncthreads();
    if (tid == 0) {
        p.fix_meta[META_R] = ok ? r : 0;
        p.fix_meta[META_NONREP] = s_fix;
        p.fix_meta[META_STATUS] = ADA_OK;
    }
}

// Algorithm 1 steps 5, 9, 10 from the first-hit records.  For every token the tiles left, next to its hit words, the
// smallest list position of a representative that hits it (p.first).  That decides almost everything:
//   * an inherited representative is valid (step 5) iff it has no hit at all (its words hold earlier ones only);
//   * any other token is new (step 9) if it has no hit, and covered if its earliest hit is a valid representative.
// Only a token whose earliest hit turns out invalid needs its hit words (is one of the later hits valid?): a chain
// t ~ s1 ~ s0 with t not ~ s0, which clustered activations produce rarely.  So the workgroup reads 4 T bytes instead of
// the whole hit table (T x ceil(r / 32) words: 114 KB at T = 2048, r = 435; 720 KB at T = 8192, r = 700), which was most
// of this phase.  Thread tid owns the 4 NV consecutive tokens from 4 NV tid on (T a multiple of 4, T <= 4 NV THREADS);
// the records are cleared as they are read, so the table is zero again for the next call.
template <int THREADS, int NV>
__device__ inline int fused_update_rec(const FusedParams& p, int r, int q0, int qp0, char* lds, int* scan_scratch) {
    constexpr int U = 4 * NV;
    const int tid = threadIdx.x;
    const int T = p.T, T4 = T >> 2;
    const int Wa = (r + 31) >> 5;
    uint16_t* pos = reinterpret_cast<uint16_t*>(lds);                        // [T] list position of an inherited token
    uint32_t* vmask = reinterpret_cast<uint32_t*>(lds + FUSED_MAX_T * 2);    // [Wa] valid bits by list position
    u32x4 key[NV];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int t4 = tid * NV + v;
        u32x4* src = reinterpret_cast<u32x4*>(p.first) + min(t4, T4 - 1);   // clamped: no lane is switched off at the load
        key[v] = *src;
        if (t4 < T4) {
            *reinterpret_cast<unsigned long long*>(pos + 4 * t4) = ~0ull;    // 0xFFFF: not inherited
        } else {
            key[v] = u32x4{0u, 0u, 0u, 0u};
        }
    }
#pragma unroll
    for (int v = 0; v < NV; ++v) {                                           // (after every load of this thread: a store
        const int t4 = tid * NV + v;                                         //  in between would make the loads wait)
        if (t4 < T4) reinterpret_cast<u32x4*>(p.first)[t4] = u32x4{0u, 0u, 0u, 0u};
    }
    for (int w = tid; w < Wa; w += THREADS) vmask[w] = 0u;
    __syncthreads();
    int ok = 1;
    for (int j = tid; j < r; j += THREADS) {            // the list: strictly ascending token ids in range
        const int q = j < THREADS ? q0 : list_at(p, j);
        const int qp = j < THREADS ? qp0 : list_at(p, j - 1);
        if (q < 0 || q >= T || (j > 0 && !(qp < q))) ok = 0;
        else pos[q] = (uint16_t)j;
    }
    ok = __syncthreads_and(ok);
    if (!ok) {
        gamma_fix_collect<THREADS>(p, r, vmask, false);
        if (tid == 0) {
            p.counts[0] = 0; p.counts[1] = 0; p.counts[2] = 0; p.counts[3] = ADA_ERR_INDEX;
            if (p.gram_ops) *p.gram_ops = 0ull;
            adapt_tau(p, r, 0, 0, false);
            reset_tickets(p.ticket);
        }
        return 0;
    }
    // step 5: an inherited representative with a hit from an earlier inherited one is removed (the tile epilogue kept
    // only earlier representatives in an inherited token's words, so any hit at all removes it)
    int jpos[U];
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int t4 = tid * NV + v;
        const unsigned long long pk = t4 < T4 ? *reinterpret_cast<const unsigned long long*>(pos + 4 * t4) : ~0ull;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int j = (int)((pk >> (16 * u)) & 0xFFFFu);
            jpos[4 * v + u] = j;
            if (j != 0xFFFF && key[v][u] == 0u) atomicOr(&vmask[j >> 5], 1u << (j & 31));
        }
    }
    __syncthreads();
    gamma_fix_collect<THREADS>(p, r, vmask, true);       // (gamma output only)
    // step 9: any other token with a hit on a VALID representative is covered
    bool f[3][U];                                        // in R^(l+1) | added | removed
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        const int t4 = tid * NV + v;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = 4 * v + u;
            const bool own = t4 < T4, inh = jpos[i] != 0xFFFF;
            const uint32_t k = key[v][u];
            bool covered = false;
            if (own && !inh && k != 0u) {
                const uint32_t fp = 0xFFFFFFFFu - k;     // earliest hit; a position below r by construction (clamped anyway)
                const uint32_t fw = min(fp >> 5, (uint32_t)(Wa - 1));
                covered = (vmask[fw] >> (fp & 31)) & 1u;
                if (!covered) {                          // rare: is one of the later hits valid?
                    const int t = 4 * t4 + u;
                    uint32_t any = 0u;
                    for (int w = (int)fw; w < Wa; ++w) any |= p.hits[(size_t)w * T + t] & vmask[w];
                    covered = any != 0u;
                }
            }
            const int st = !own ? 0 : inh ? (k == 0u ? 3 : 1) : (k == 0u ? 2 : (covered ? 0 : 2));
            f[0][i] = (st & 2) != 0;
            f[1][i] = st == 2;
            f[2][i] = st == 1;
        }
    }
    int below[3], tot[3];
    block_rank3<THREADS, U>(f, below, tot, scan_scratch);
    int o_idx = below[0], o_add = below[1], o_rem = below[2];
    const int n_idx = tot[0], n_add = tot[1], n_rem = tot[2];
#pragma unroll
    for (int i = 0; i < U; ++i) {                        // step 10
        const int t = U * tid + i;
        if (f[0][i]) p.idx[o_idx++] = t;
        if (f[1][i]) { if (p.adds) p.adds[o_add] = t; ++o_add; }
        if (f[2][i]) { if (p.removes) p.removes[o_rem] = t; ++o_rem; }
    }
    if (tid == 0) {
        p.counts[0] = n_idx; p.counts[1] = n_add; p.counts[2] = n_rem; p.counts[3] = ADA_OK;
        adapt_tau(p, r, n_add, n_rem, true);
        if (p.gram_ops) {
            const unsigned long long TT = (unsigned long long)T, rr = (unsigned long long)r;
            *p.gram_ops = rr * rr + (TT - rr) * (unsigned long long)(r - n_rem);   // entries Algorithm 1 needs
        }
        reset_tickets(p.ticket);
    }
    return n_idx;
}

// Returns |R^(l+1)| to every thread (0 if the step is rejected).
template <int THREADS>
__device__ inline int fused_update(const FusedParams& p, int r, bool r_ok, int q0, int qp0, char* lds, int* scan_scratch) {
    constexpr int WU = 11;                              // hit words fetched per batch by one thread (22, 33, ... words: whole batches)
    const int tid = threadIdx.x, lane = tid & 63;
    const int T = p.T;
    if (r_ok && p.first && (T & 3) == 0 && T <= 32 * THREADS) {             // uniform
        const int t4 = T >> 2;
        if (t4 <= THREADS) return fused_update_rec<THREADS, 1>(p, r, q0, qp0, lds, scan_scratch);
        if (t4 <= 2 * THREADS) return fused_update_rec<THREADS, 2>(p, r, q0, qp0, lds, scan_scratch);
        if (t4 <= 4 * THREADS) return fused_update_rec<THREADS, 4>(p, r, q0, qp0, lds, scan_scratch);
        return fused_update_rec<THREADS, 8>(p, r, q0, qp0, lds, scan_scratch);
    }
    uint8_t* flag = reinterpret_cast<uint8_t*>(lds);                         // [T]
    uint32_t* vmask = reinterpret_cast<uint32_t*>(lds + FUSED_MAX_T);        // one bit per inherited representative: valid
    const int Wa = r_ok ? (r + 31) >> 5 : 0;            // hit words in use per token
    for (int t = tid; t < T; t += THREADS) flag[t] = 2;                      // not inherited, kept unless covered
    // the token pass's first batch of hit words does not depend on the validity mask: fetch it now, use it later
    const bool vec = (T & 3) == 0;
    u32x4 pre[WU];
    if (vec && r_ok) {                                  // uniform; clamped address, used only by threads that own tokens
        const int t4c = min(tid, (T >> 2) - 1);
#pragma unroll
        for (int v = 0; v < WU; ++v) pre[v] = *reinterpret_cast<const u32x4*>(p.hits + (size_t)min(v, Wa - 1) * T + 4 * t4c);
    }
    __syncthreads();
    ADA_CLK_LAST(10);
    // step 5: an inherited representative with a hit from an earlier inherited one is removed.  The list is checked
    // on the way (strictly ascending token ids in range); token ids are clamped so that a bad list cannot fault.
    // Lanes of a wave hold 64 consecutive list positions, so a ballot is two words of the validity mask.
    int ok = 1;
    if (r_ok) {
        // two list entries per thread and round (j and j + THREADS), with the words of both requested before either is
        // used: the scattered loads are trips to memory, and this halves their number
        for (int j0 = 0; j0 < r; j0 += 2 * THREADS) {
            int tok[2];
            bool have[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int j = j0 + e * THREADS + tid;
                have[e] = j < r;
                const int q = !have[e] ? 0 : (j < THREADS ? q0 : list_at(p, j));
                const int qp = !have[e] || j == 0 ? -1 : (j < THREADS ? qp0 : list_at(p, j - 1));
                if (have[e] && (q < 0 || q >= T || !(qp < q))) ok = 0;
                tok[e] = min(max(q, 0), T - 1);
            }
            uint32_t any[2] = {0u, 0u};
            for (int w0 = 0; w0 < Wa; w0 += WU) {
                uint32_t x[2][WU];
#pragma unroll
                for (int e = 0; e < 2; ++e)
#pragma unroll
                    for (int v = 0; v < WU; ++v) x[e][v] = p.hits[(size_t)min(w0 + v, Wa - 1) * T + tok[e]];
#pragma unroll
                for (int e = 0; e < 2; ++e)
#pragma unroll
                    for (int v = 0; v < WU; ++v) any[e] |= (w0 + v < Wa) ? x[e][v] : 0u;
            }
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int j = j0 + e * THREADS + tid;
                if (have[e]) flag[tok[e]] = any[e] ? 1 : 3;
                const unsigned long long valid = __ballot(have[e] && any[e] == 0u);   // 64 consecutive list positions
                if (lane == 0 && j < r) {
                    vmask[j >> 5] = (uint32_t)valid;
                    if ((j >> 5) + 1 < Wa) vmask[(j >> 5) + 1] = (uint32_t)(valid >> 32);
                }
            }
        }
    }
    ok = __syncthreads_and(ok);
    const int status = !r_ok ? ADA_ERR_SHAPE : (!ok ? ADA_ERR_INDEX : ADA_OK);
    gamma_fix_collect<THREADS>(p, r, vmask, status == ADA_OK);               // (gamma output only)
    if (status != ADA_OK) {
        if (tid == 0) {
            p.counts[0] = 0; p.counts[1] = 0; p.counts[2] = 0; p.counts[3] = status;
            if (p.gram_ops) *p.gram_ops = 0ull;
            adapt_tau(p, r, 0, 0, false);
            reset_tickets(p.ticket);
        }
        return 0;
    }
    ADA_CLK_LAST(12);
    // step 9: any other token with a hit on a VALID representative is covered
    if (vec) {
        // Work items (four tokens, one batch of WU words), one after the other per thread; item k + 1 is requested
        // before item k is used, so that the phase runs at the CU's load rate and not at one trip to memory per batch.
        // Addresses are clamped and the values masked where they are used (nothing waits at a load).
        const int T4 = T >> 2, nb = (Wa + WU - 1) / WU, n_it = (T4 + THREADS - 1) / THREADS, items = nb * n_it;
        auto request = [&](u32x4 (&x)[WU], int k) {
            const int it = k / nb, w0 = (k - it * nb) * WU;
            const int t4 = min(tid + it * THREADS, T4 - 1);
#pragma unroll
            for (int v = 0; v < WU; ++v) x[v] = *reinterpret_cast<const u32x4*>(p.hits + (size_t)min(w0 + v, Wa - 1) * T + 4 * t4);
        };
        u32x4 any = {0u, 0u, 0u, 0u};
        auto use = [&](const u32x4 (&x)[WU], int k) {
            const int it = k / nb, b = k - it * nb, w0 = b * WU;
            if (b == 0) any = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
            for (int v = 0; v < WU; ++v) any |= x[v] & ((w0 + v < Wa) ? vmask[w0 + v] : 0u);
            const int t4 = tid + it * THREADS;
            if (b == nb - 1 && t4 < T4) {
                uint32_t f4 = *reinterpret_cast<const uint32_t*>(flag + 4 * t4);
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    if (((f4 >> (8 * u)) & 0xFFu) == 2u && any[u]) f4 &= ~(0xFFu << (8 * u));
                *reinterpret_cast<uint32_t*>(flag + 4 * t4) = f4;
            }
        };
        u32x4 xa[WU], xb[WU];
#pragma unroll
        for (int v = 0; v < WU; ++v) xa[v] = pre[v];          // item 0 was requested before the validity pass
        for (int k = 0; k < items; k += 2) {
            if (k + 1 < items) request(xb, k + 1);
            use(xa, k);
            if (k + 1 < items) {
                if (k + 2 < items) request(xa, k + 2);
                use(xb, k + 1);
            }
        }
    } else {
        for (int t = tid; t < T; t += THREADS) {
            uint32_t any = 0u;
            for (int w0 = 0; w0 < Wa; w0 += WU) {
                uint32_t x[WU];
#pragma unroll
                for (int v = 0; v < WU; ++v) x[v] = p.hits[(size_t)min(w0 + v, Wa - 1) * T + t];
#pragma unroll
                for (int v = 0; v < WU; ++v) any |= x[v] & ((w0 + v < Wa) ? vmask[w0 + v] : 0u);
            }
            if (flag[t] == 2 && any) flag[t] = 0;
        }
    }
    __syncthreads();
    ADA_CLK_LAST(13);
    const int chunk = (T + THREADS - 1) / THREADS;
    const int lo = min(T, tid * chunk), hi = min(T, lo + chunk);
    unsigned long long c = 0;                            // kept | added << 21 | removed << 42
    for (int t = lo; t < hi; ++t) {
        const unsigned f = flag[t];
        c += (unsigned long long)((f >> 1) & 1u) | ((unsigned long long)(f == 2u) << 21) |
             ((unsigned long long)(f == 1u) << 42);
    }
    unsigned long long tot;
    const unsigned long long o = block_exclusive_scan64(c, &tot, reinterpret_cast<unsigned long long*>(scan_scratch));
    int o_idx = (int)(o & 0x1FFFFF), o_add = (int)((o >> 21) & 0x1FFFFF), o_rem = (int)((o >> 42) & 0x1FFFFF);
    const int n_idx = (int)(tot & 0x1FFFFF), n_add = (int)((tot >> 21) & 0x1FFFFF), n_rem = (int)((tot >> 42) & 0x1FFFFF);
    ADA_CLK_LAST(14);
    for (int t = lo; t < hi; ++t) {                     // step 10
        const int f = flag[t];
        if (f & 2) p.idx[o_idx++] = t;
        if (f == 2) { if (p.adds) p.adds[o_add] = t; ++o_add; }
        if (f == 1) { if (p.removes) p.removes[o_rem] = t; ++o_rem; }
    }
    if (tid == 0) {
        p.counts[0] = n_idx; p.counts[1] = n_add; p.counts[2] = n_rem; p.counts[3] = ADA_OK;
        adapt_tau(p, r, n_add, n_rem, true);
        if (p.gram_ops) {
            const unsigned long long TT = (unsigned long long)T, rr = (unsigned long long)r;
            *p.gram_ops = rr * rr + (TT - rr) * (unsigned long long)(r - n_rem);   // entries Algorithm 1 needs
        }
        reset_tickets(p.ticket);                                    // leave the workspace ready for the next call
    }
    return n_idx;
}

// Section 2.3, last step (run by one workgroup): unpack the per-token arg max, make every member of R its own
// representative, check the list, and leave the key table zero for the next call.
// info[0] = tokens represented by another token (T - r), info[3] = status.
template <int THREADS>
__device__ inline void assign_finish(const FusedParams& p, int r, bool r_ok, int q0, int qp0) {
    const int tid = threadIdx.x;
    const int T = p.T;
    for (int t = tid; t < T; t += THREADS) {
        const unsigned long long key = p.best[t];
        p.best[t] = 0ull;
        const int who = INT_MAX - (int)(uint32_t)key;
        if (p.pos_out) {                                 // keys carry positions: the token id comes from the list
            const int pos = r_ok ? min(max(who, 0), r - 1) : 0;
            p.pos_out[t] = pos;
            p.assign[t] = r_ok ? list_at(p, pos) : 0;
        } else {
            p.assign[t] = who;
        }
        if (p.corr) p.corr[t] = __uint_as_float((uint32_t)(key >> 32));
    }
    int ok = 1;
    __syncthreads();                                     // fenced: the stores above have completed before a member of R
    if (r_ok) {                                          // is overwritten with itself by another thread
        for (int j = tid; j < r; j += THREADS) {
            const int q = j < THREADS ? q0 : list_at(p, j);
            const int qp = j < THREADS ? qp0 : list_at(p, j - 1);
            if (q < 0 || q >= T || (j > 0 && !(qp < q))) { ok = 0; continue; }
            p.assign[q] = q;
            if (p.pos_out) p.pos_out[q] = j;
            if (p.corr) p.corr[q] = 1.0f;
        }
    }
    ok = __syncthreads_and(ok);
    if (tid == 0) {
        const int status = !r_ok ? ADA_ERR_SHAPE : (!ok ? ADA_ERR_INDEX : ADA_OK);
        p.counts[0] = status == ADA_OK ? T - r : 0;
        p.counts[1] = 0; p.counts[2] = 0; p.counts[3] = status;
        reset_tickets(p.ticket);
    }
}

// The tiles of one step, dealt to the workgroups in contiguous ranges per XCD (blockIdx % 8), the representative block
// fastest, so that one XCD's L2 serves a contiguous range of tested rows.
template <typename In, bool ALIGNED, int KG, bool DMA>
__device__ inline void fused_step_tiles(const FusedParams& p, int r, char* lds, unsigned local, unsigned workers) {
    int shape = 0;
    constexpr int NSHAPES = sizeof(In) == 2 ? 4 : 3;                      // the ring tiles are bf16 only
    if constexpr (ALIGNED && KG == 2 && DMA)
        shape = cascade_tile_shape(r, p.T, p.d, p.tile_pick, p.groups > 1 ? (int)workers : p.tile_pick, NSHAPES);
    const int sr = shape >= 2 ? 7 : 6, st = shape == 0 ? 6 : shape == 3 ? 8 : 7;   // log2 of the tile's rows
    const unsigned nbS = (unsigned)(r + (1 << sr) - 1) >> sr;
    const unsigned ntiles = nbS * ((unsigned)(p.T + (1 << st) - 1) >> st);
    // Contiguous tile ranges per XCD (workgroup b of the launch runs on XCD b % 8), so that the tiles an L2 serves at
    // one time share their rows.  One problem: worker b is on XCD b % 8.  Groups: worker `local` of group g is
    // workgroup local * groups + g, so a group's workers live on nx = 8 / gcd(8, groups) XCDs, worker `local` on the
    // (local % nx)-th of them.
    const unsigned G = p.groups > 1 ? (unsigned)p.groups : 1u;
    const unsigned low = G & (0u - G);                                    // lowest set bit of the group count
    const unsigned nx0 = 8u / (low < 8u ? low : 8u);
    const unsigned nx = nx0 < workers ? nx0 : workers;                    // (fewer workers than XCDs: one range each)
    const unsigned xi = local % nx, li = local / nx;
    const unsigned per = (ntiles + nx - 1u) / nx;
    const unsigned base = xi * per;
    const unsigned slots = (workers - xi + nx - 1u) / nx;                 // workers of this problem on this XCD
    for (unsigned slot = li; slot < per; slot += slots) {
        const unsigned tile = base + slot;
        if (tile >= ntiles) break;
        const int tb = (int)(tile / nbS), sb = (int)(tile - (unsigned)tb * nbS);
        if constexpr (ALIGNED && KG == 2 && DMA) {
            if constexpr (sizeof(In) == 2) {
                // (measured both ways: loader waves gain 10% at 128 x 128; at 128 x 256 the eight multiplying waves of
                // the ring tile are 3% ahead for one sequence and level for stacked ones)
                if (shape == 3) fused_tile_ring<2, 2>(p, r, sb * 128, tb * 256, lds);
                else if (shape == 2) fused_tile_split<1, 2>(p, r, sb * 128, tb * 128, lds);
                else if (shape == 1) fused_tile_wide<In, 2>(p, r, sb * 64, tb * 128, lds);   // (loader waves: no gain here)
                else fused_tile<In, ALIGNED, KG, DMA>(p, r, sb * 64, tb * 64, sb, lds);
            } else {
                if (shape == 2) fused_tile_wide<In, 4>(p, r, sb * 128, tb * 128, lds);
                else if (shape == 1) fused_tile_wide<In, 2>(p, r, sb * 64, tb * 128, lds);
                else fused_tile<In, ALIGNED, KG, DMA>(p, r, sb * 64, tb * 64, sb, lds);
            }
        } else {
            fused_tile<In, ALIGNED, KG, DMA>(p, r, sb * 64, tb * 64, sb, lds);
        }
        __syncthreads();
    }
}

// Grid: a multiple of 8 workgroups (see k_gram for the XCD-aware tile ranges); tiles with the representative
// block fastest, so one XCD's L2 serves a contiguous range of tested rows.
template <typename In, bool ALIGNED, int KG, bool DMA>
__global__ __launch_bounds__(256 * KG) void k_cascade_fused(FusedParams p) {
    extern __shared__ __align__(16) char lds[];
    using G = FusedGeom<KG, DMA>;
    __shared__ int s_last;
    ADA_CLK(0);
    unsigned local = blockIdx.x, workers = (unsigned)p.grid;
    if (p.groups > 1) {                                      // uniform: this workgroup's problem
        const unsigned g = blockIdx.x % (unsigned)p.groups;
        local = blockIdx.x / (unsigned)p.groups;
        workers = (unsigned)p.wpg;
        p.X = reinterpret_cast<const char*>(p.X) + (long long)g * p.x_gs;
        p.prev_idx += (long long)g * p.list_gs;
        if (p.r_dev) p.r_dev += (long long)g * p.counts_gs;
        p.hits = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(p.hits) + (long long)g * p.ws_gs);
        p.ticket = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(p.ticket) + (long long)g * p.ws_gs);
        if (p.first) p.first = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(p.first) + (long long)g * p.ws_gs);
        p.idx += (long long)g * p.list_gs;
        if (p.adds) p.adds += (long long)g * p.list_gs;
        if (p.removes) p.removes += (long long)g * p.list_gs;
        p.counts += (long long)g * p.counts_gs;
        if (p.gram_ops) p.gram_ops += (long long)g * p.ops_gs;
    }
    if (p.thr_in) p.thr = *p.thr_in;                         // adaptive threshold: travels with the set size
    const int r = p.r_dev ? *p.r_dev : p.r_host;
    const bool r_ok = r >= 1 && r <= p.r_host && r <= p.T;
    if (r_ok) fused_step_tiles<In, ALIGNED, KG, DMA>(p, r, lds, local, workers);
    // The workgroup that takes the last ticket finishes the step.  Hit words and row maxima leave the CU as
    // device-scope atomics (written through the L2), so once every thread's stores are acknowledged (vmcnt(0)) and
    // the workgroup has met at the barrier, the ticket can be taken: nothing is left in the L2 to write back.
    ADA_CLK(6);
    // the update phase's first slice of the inherited list: input data, so it can be fetched behind the store drain
    // (entries below r_host are the caller's memory whatever r turns out to be)
    const int jq = min((int)threadIdx.x, max(p.r_host, 1) - 1);
    const int q0 = list_at(p, jq), qp0 = list_at(p, max(jq - 1, 0));
    drain_stores();                                          // this thread's stores have left the CU
    __syncthreads();
    // (a group's few workers count on one word: the two levels are for a whole chip of workgroups)
    if (threadIdx.x == 0)
        s_last = (p.groups > 1 ? atomicAdd(p.ticket, 1) == (int)workers - 1 : take_ticket(p.ticket, p.grid)) ? 1 : 0;
    __syncthreads();
    ADA_CLK(7);
    if (!s_last) return;
    ADA_CLK_LAST(8);
    // see the other workgroups' hit words, not stale lines: one invalidate for the workgroup (the caches it clears
    // are shared by the CU), then a barrier
    if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    __syncthreads();
    ADA_CLK_LAST(9);
    if (p.assign_mode) assign_finish<G::THREADS>(p, r, r_ok, q0, qp0);
    else fused_update<G::THREADS>(p, r, r_ok, q0, qp0, lds + G::META, reinterpret_cast<int*>(lds + G::OFF_SCAN));
    ADA_CLK_LAST(15);
}

// ------------------------------------------------------------------------------------------------
// k_cascade_pass: the layer loop of Section 4.1 in ONE launch.  Between two launches of k_cascade_fused the device
// idles for about 4 us and the new launch starts with a trip to memory for the set size; here the workgroups stay
// resident and walk through the layers.  A layer's last workgroup (ticket) updates the set as before, then publishes
// (layers done << 21 | set size) in one word; the others wait for that word before they start the next layer.
// The grid must be co-resident (one workgroup per CU: the launcher asks for no more workgroups than CUs, and the LDS
// footprint admits one per CU).  The wait is bounded: a workgroup that does not see the word within spin_limit polls
// gives up and leaves, the others then run into the same bound, and the layers that were not finished keep the
// status the launcher wrote into their counts beforehand.  Every wave therefore reaches the end of the kernel.
constexpr int PASS_MAX_LAYERS = 64;

struct PassParams {
    FusedParams f;                     // shape, threshold, hit table, ticket; the per-layer pointers are set in the kernel
    const void* X[PASS_MAX_LAYERS];    // X of the n cascade layers of this launch
    int n;                             // cascade layers in this launch (1 .. PASS_MAX_LAYERS)
    int32_t* idx_row0;                 // row of the set inherited by the first layer; layer i writes row i + 1
    int32_t* counts_row0;              // likewise ([4] per row); counts_row0[0] is the first inherited size
    unsigned long long* gram_ops_row0; // likewise
    int32_t* adds_row0;                // row i + 1 for layer i, or NULL
    int32_t* removes_row0;             // likewise
    int32_t* epoch;                    // zero on entry and on exit
    int spin_limit;
};

#ifdef ADA_PHASE_CLOCKS
__device__ unsigned long long g_pass_clk[512 * 8];
#define PASS_CLK(k) do { if (threadIdx.x == 0 && i == 5) g_pass_clk[blockIdx.x * 8 + (k)] = __builtin_amdgcn_s_memrealtime(); } while (0)
#else
#define PASS_CLK(k) do { } while (0)
#endif

template <typename In, bool ALIGNED, int KG, bool DMA>
__global__ __launch_bounds__(256 * KG) void k_cascade_pass(PassParams pp) {
    extern __shared__ __align__(16) char lds[];
    using G = FusedGeom<KG, DMA>;
    __shared__ int s_last, s_word;
    FusedParams p = pp.f;
    const int T = p.T;
    // No cache is invalidated between layers.  X is read-only.  A row of the set is written (and written back) before
    // anybody reads it and is never read before that, so plain loads are safe when rows do not share cache lines;
    // otherwise (coherent_list, set by the launcher) the list is read past the caches.
    for (int i = 0; i < pp.n; ++i) {
        PASS_CLK(0);
        // ---- the inherited set: from the previous launch for the first layer, from this launch's previous layer after
        if (threadIdx.x == 0) {
            int word;
            if (i == 0) {
                word = pp.counts_row0[0] & 0x1FFFFF;
            } else {
                word = -1;
                for (int n = 0; n < pp.spin_limit; ++n) {
                    const int v = __hip_atomic_load(pp.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if ((v >> 21) == i) { word = v & 0x1FFFFF; break; }
                    __builtin_amdgcn_s_sleep(2);
                }
            }
            s_word = word;
        }
        __syncthreads();
        const int r = s_word;
        if (r < 0) break;                                    // uniform: gave up waiting
        PASS_CLK(1);
        const size_t row = (size_t)(i + 1) * (size_t)T;
        p.X = pp.X[i];
        p.prev_idx = pp.idx_row0 + row - T;
        p.idx = pp.idx_row0 + row;
        p.adds = pp.adds_row0 ? pp.adds_row0 + row : nullptr;
        p.removes = pp.removes_row0 ? pp.removes_row0 + row : nullptr;
        p.counts = pp.counts_row0 + (size_t)(i + 1) * 4;
        p.gram_ops = pp.gram_ops_row0 + (i + 1);
        const bool r_ok = r >= 1 && r <= T;
        if (r_ok) fused_step_tiles<In, ALIGNED, KG, DMA>(p, r, lds, blockIdx.x, (unsigned)p.grid);
        PASS_CLK(2);
        const int jq = min((int)threadIdx.x, T - 1);         // the row has T entries whatever r is
        const int q0 = list_at(p, jq), qp0 = list_at(p, max(jq - 1, 0));
        drain_stores();                                      // this thread's stores have left the CU
        __syncthreads();
        if (threadIdx.x == 0) s_last = take_ticket(p.ticket, p.grid) ? 1 : 0;
        __syncthreads();
        PASS_CLK(3);
        if (s_last) {                                        // uniform
            if (threadIdx.x == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            __syncthreads();
            const int r_new = fused_update<G::THREADS>(p, r, r_ok, q0, qp0, lds + G::META,
                                                       reinterpret_cast<int*>(lds + G::OFF_SCAN));
            __syncthreads();
            if (threadIdx.x == 0) {
                // the ticket is back at zero and the set is written: hand both over with one release
                const int word = i + 1 < pp.n ? (((i + 1) << 21) | (r_new & 0x1FFFFF)) : 0;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                __hip_atomic_store(pp.epoch, word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            PASS_CLK(4);
        }
        __syncthreads();
    }
}
