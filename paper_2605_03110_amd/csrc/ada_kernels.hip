// libada device code and C ABI for gfx950 (MI355X).
//
// What is computed (paper: "Cascade Token Selection for Transformer Attention Acceleration"):
//   Section 2.1      Xhat = D^-1 X, G = Xhat Xhat^T (never stored: tiles live in MFMA accumulators)
//   Definition 2.2   gamma_t = max_{s<t} |G_st|, representative iff gamma_t < 1 - tau^2
//   Algorithm 1      cascade step: r x r Gram among inherited rows, (T-r) x r_valid cross-Gram, set update
//   eq. (6), Table 6 Gram-operation count
//
// Kernel plan (one stream, no host round trips inside a call):
//   k_norm_prep   1/||x_t|| for every row (one wavefront per row, 16-byte coalesced loads), clears gamma;
//                 in cascade mode one extra workgroup validates the inherited list and builds the
//                 complement list (the "gather" is an index list: rows are read in place)
//   k_gram        tiles of |<x_s,x_t>| * inv_s * inv_t on MFMA (bf16 32x32x16 / fp32 32x32x2, fp32 accumulate),
//                 epilogue = scale, order / validity mask, in-lane max over the "against" rows,
//                 one cross-half shuffle, atomicMax of the float bits into gamma[t]
//   k_update      threshold + compaction into idx / adds / removes / counts / gram_ops
//
// The MFMA operand roles are chosen so that the max over "against" tokens s runs over accumulator
// registers of one lane: s rows feed the A operand (M), the tested tokens t feed the B operand (N).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <limits.h>
#include <math.h>
#include <stdlib.h>
#include <functional>
#include <mutex>
#include <queue>
#include <string>
#include <type_traits>
#include <vector>

#include "../../include/ada.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

enum { MODE_FULL = 0, MODE_REP = 1, MODE_CROSS = 2 };
// meta: 8 words of scalars, then (from word META_TICKET + 64 on, one per 128-byte line) the per-XCD ticket counters
constexpr size_t META_BYTES = 2048;
enum { META_R = 0, META_NONREP = 1, META_STATUS = 2, META_SPARE = 3, META_TICKET = 4, META_QUEUE = 5 /* and 6 */, META_EPOCH = 7, META_WORDS = 8 };

// The one-launch cascade step keeps one hit word per token and per 32 inherited representatives; beyond this T
// the table would dominate the workspace and the two-launch path is used instead.
constexpr int FUSED_MAX_T = 16384;

struct Workspace {
    float* inv_norm;     // [T]
    float* gamma;        // [T]
    int32_t* nonrep_idx; // [T]
    uint8_t* is_rep;     // [T]
    int32_t* meta;       // [META_WORDS]; meta[META_TICKET], the META_QUEUE pair and meta[META_EPOCH] are zero between calls
    uint32_t* hits;      // [T][hit_words(T)] (only for T <= FUSED_MAX_T)
    unsigned long long* best;   // [T] arg-max keys (assignment; cascade step with a gamma output); zero between calls
    uint32_t* first;            // [T] first-hit records of the one-launch cascade step; zero between calls
};

__host__ __device__ constexpr size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
constexpr int hit_words(int r_cap) {                         // whole 64- or 128-row tiles, whichever needs more words
    return 2 * ((r_cap + 63) / 64) > 4 * ((r_cap + 127) / 128) ? 2 * ((r_cap + 63) / 64) : 4 * ((r_cap + 127) / 128);
}

constexpr size_t ws_bytes_for(int T) {
    return align_up((size_t)T * 4, 256) * 3 + align_up((size_t)T, 256) + META_BYTES +
           (T <= FUSED_MAX_T ? align_up((size_t)T * hit_words(T) * 4, 256) : 0) + align_up((size_t)T * 8, 256) +
           align_up((size_t)T * 4, 256);
}

inline Workspace carve(void* ws, int T) {
    char* p = (char*)ws;
    size_t t4 = align_up((size_t)T * 4, 256), t1 = align_up((size_t)T, 256);
    Workspace w;
    w.inv_norm = (float*)p; p += t4;
    w.gamma = (float*)p; p += t4;
    w.nonrep_idx = (int32_t*)p; p += t4;
    w.is_rep = (uint8_t*)p; p += t1;
    w.meta = (int32_t*)p; p += META_BYTES;
    w.hits = (uint32_t*)p; p += T <= FUSED_MAX_T ? align_up((size_t)T * hit_words(T) * 4, 256) : 0;
    w.best = (unsigned long long*)p; p += align_up((size_t)T * 8, 256);
    w.first = (uint32_t*)p;
    return w;
}

// ------------------------------------------------------------------------------------------------
// element access

template <typename In> __device__ inline float to_f32(In v);
template <> __device__ inline float to_f32<float>(float v) { return v; }
template <> __device__ inline float to_f32<uint16_t>(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// One 16-byte piece of a row starting at element e0; elements at or beyond d read as zero.
// The aligned form is split in two so that loads can run ahead of their use: fetch_piece issues a branch-free
// load from an address clamped into the row (a run of them stays in one basic block, which lets the compiler keep
// several chunks in flight with counted waits), finish_piece zeroes an out-of-range piece when it is consumed.
// The element-wise form does both in fetch_piece.
template <typename In, bool ALIGNED>
__device__ inline u32x4 fetch_piece(const In* row, int e0, int d) {
    constexpr int EPP = 16 / (int)sizeof(In);
    if (ALIGNED) {
        const int e = min(e0, d - EPP);                     // d is a positive multiple of EPP here
        return *reinterpret_cast<const u32x4*>(row + e);
    } else {
        union { u32x4 v; In e[EPP]; } u;
        u.v = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < EPP; ++i)
            if (e0 + i < d) u.e[i] = row[e0 + i];
        return u.v;
    }
}

template <bool ALIGNED>
__device__ inline u32x4 finish_piece(u32x4 v, int e0, int d) {
    if (ALIGNED && e0 >= d) v = u32x4{0u, 0u, 0u, 0u};
    return v;
}

template <typename In, bool ALIGNED>
__device__ inline u32x4 load_piece(const In* row, int e0, int d) {
    return finish_piece<ALIGNED>(fetch_piece<In, ALIGNED>(row, e0, d), e0, d);
}

template <typename In>
__device__ inline float piece_sumsq(u32x4 v) {
    constexpr int EPP = 16 / (int)sizeof(In);
    union { u32x4 v; In e[EPP]; } u;
    u.v = v;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < EPP; ++i) { float f = to_f32<In>(u.e[i]); s = fmaf(f, f, s); }
    return s;
}

// Hand-over of results to the workgroup that finishes a launch.  Results leave the CU as device-scope atomic stores
// (written through the L2, where every XCD sees them); on this chip such a store is acknowledged in the vector-memory
// counter, so once vmcnt is zero the data is visible device-wide and a relaxed ticket may follow.  The empty asm
// statements keep the compiler from moving memory operations across the wait in either direction; the reader
// invalidates its CU's caches once (acquire fence by one thread, then a barrier) before it loads.
__device__ inline void drain_stores() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_waitcnt(0x0F70);                  // vmcnt(0); the other counters are left alone
    asm volatile("" ::: "memory");
}

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// exclusive prefix sum of one int per thread over the workgroup (blockDim.x multiple of 64, <= 1024)
__device__ inline int block_exclusive_scan(int v, int* total, int* wave_tot /* >= 17 ints of LDS */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int n = __shfl_up(inc, o, 64);
        if (lane >= o) inc += n;
    }
    __syncthreads();
    if (lane == 63) wave_tot[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int w = 0; w < nw; ++w) { int t = wave_tot[w]; wave_tot[w] = run; run += t; }
        wave_tot[16] = run;
    }
    __syncthreads();
    *total = wave_tot[16];
    return wave_tot[wave] + inc - v;
}

// ------------------------------------------------------------------------------------------------
// k_norm_prep: row norms (+ optional cascade preparation in the last workgroup)

// Several problems of one shape in one launch of the full-selection kernels: blockIdx.y is the problem, whose
// pointers lie g strides after problem 0's (ws: the workspaces, back to back).  All zero: one problem.
struct GroupOff {
    long long x;        // bytes between consecutive problems' X
    long long ws;       // bytes between their workspaces
    long long list;     // int32 elements between their idx rows
    long long counts;   // int32 elements between their counts
    long long ops;      // elements between their gram_ops
};

struct PrepParams {
    const int32_t* prev_idx;
    const int32_t* r_dev;
    int r_host;
    int enabled;
};

template <typename In, bool ALIGNED>
__global__ __launch_bounds__(256) void k_norm_prep(const In* __restrict__ X, long long ld, int T, int d,
                                                   float* __restrict__ inv_norm, float* __restrict__ gamma,
                                                   Workspace w, PrepParams prep, int n_norm_blocks, GroupOff go) {
    constexpr int EPP = 16 / (int)sizeof(In);
    __shared__ int sh[32];
    if (go.ws) {                                             // (the cascade preparation below is not used with groups)
        X = reinterpret_cast<const In*>(reinterpret_cast<const char*>(X) + (long long)blockIdx.y * go.x);
        inv_norm = reinterpret_cast<float*>(reinterpret_cast<char*>(inv_norm) + (long long)blockIdx.y * go.ws);
        gamma = reinterpret_cast<float*>(reinterpret_cast<char*>(gamma) + (long long)blockIdx.y * go.ws);
    }
    if ((int)blockIdx.x < n_norm_blocks) {
        const int lane = threadIdx.x & 63;
        const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
        if (t >= T) return;
        const In* row = X + (size_t)t * (size_t)ld;
        float s0 = 0.f, s1 = 0.f;
        const int np = (d + EPP - 1) / EPP;
        int pi = lane;
        for (; pi + 64 < np; pi += 128) {
            u32x4 a = load_piece<In, ALIGNED>(row, pi * EPP, d);
            u32x4 b = load_piece<In, ALIGNED>(row, (pi + 64) * EPP, d);
            s0 += piece_sumsq<In>(a);
            s1 += piece_sumsq<In>(b);
        }
        if (pi < np) s0 += piece_sumsq<In>(load_piece<In, ALIGNED>(row, pi * EPP, d));
        float ss = wave_sum(s0 + s1);
        if (lane == 0) {
            inv_norm[t] = ss > 0.f ? 1.0f / sqrtf(ss) : 0.f;   // a zero row normalises to zero: all its cosines are 0
            gamma[t] = 0.f;                                      // empty max
        }
        return;
    }
    // ---- cascade preparation (one workgroup): Algorithm 1 steps 2 and 6 as index lists
    if (!prep.enabled) return;
    const int tid = threadIdx.x;
    int r = prep.r_dev ? *prep.r_dev : prep.r_host;
    int status = ADA_OK;
    if (r < 1 || r > prep.r_host || r > T) { status = ADA_ERR_SHAPE; r = 0; }
    for (int t = tid; t < T; t += 256) w.is_rep[t] = 0;
    __syncthreads();
    int ok = 1;
    for (int j = tid; j < r; j += 256) {
        int p = prep.prev_idx[j];
        bool in = p >= 0 && p < T;
        if (!in) ok = 0;
        if (j > 0 && !(prep.prev_idx[j - 1] < p)) ok = 0;
        if (in) w.is_rep[p] = 1;
    }
    ok = __syncthreads_and(ok);
    if (!ok) status = ADA_ERR_INDEX;
    if (status != ADA_OK) {
        if (tid == 0) { w.meta[META_R] = 0; w.meta[META_NONREP] = 0; w.meta[META_STATUS] = status; }
        return;
    }
    const int chunk = (T + 255) / 256;
    const int lo = min(T, tid * chunk), hi = min(T, lo + chunk);
    int c = 0;
    for (int t = lo; t < hi; ++t) c += w.is_rep[t] ? 0 : 1;
    int total;
    int off = block_exclusive_scan(c, &total, sh);
    for (int t = lo; t < hi; ++t)
        if (!w.is_rep[t]) w.nonrep_idx[off++] = t;
    if (tid == 0) { w.meta[META_R] = r; w.meta[META_NONREP] = total; w.meta[META_STATUS] = ADA_OK; }
}

// ------------------------------------------------------------------------------------------------
// k_gram: MFMA Gram tiles with the fused scale / mask / max epilogue

struct GramParams {
    const void* X;
    long long ld;
    int T, d;
    const int32_t* prev_idx;
    const int32_t* nonrep_idx;
    const int32_t* meta;
    const float* inv_norm;
    float* gamma;
    float thr;
    int mode;
    int order_mask;   // require s < t in token order (always in FULL / REP; CROSS only with the earlier-only flag)
    long long x_gs, ws_gs;   // MODE_FULL with blockIdx.y = problem: bytes between problems' X / workspaces (0: one problem)
    uint32_t* hits;          // MODE_FULL, optional: word-major bit table, bit (s mod 32) of hits[(s div 32) * T + t] =
                             // "|G_st| >= threshold and s < t" (the greedy covering of Section 2.5 is resolved from it)
};

__device__ inline void gram_group_offset(GramParams& p) {
    if (p.ws_gs) {
        p.X = reinterpret_cast<const char*>(p.X) + (long long)blockIdx.y * p.x_gs;
        p.inv_norm = reinterpret_cast<const float*>(reinterpret_cast<const char*>(p.inv_norm) + (long long)blockIdx.y * p.ws_gs);
        p.gamma = reinterpret_cast<float*>(reinterpret_cast<char*>(p.gamma) + (long long)blockIdx.y * p.ws_gs);
    }
}

template <typename In> struct Mfma;
template <> struct Mfma<uint16_t> {
    static __device__ inline void run(f32x16& acc, u32x4 a, u32x4 b) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                      acc, 0, 0, 0);
    }
};
template <> struct Mfma<float> {
    static __device__ inline void run(f32x16& acc, u32x4 a, u32x4 b) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a[q]), __uint_as_float(b[q]), acc, 0, 0, 0);
    }
};

// LDS staging buffer: rows of 128 bytes = 8 pieces; piece c of row r sits at slot c ^ lds_swz(r).  The LDS of this
// chip serves 64 banks (256 bytes) per clock, so a 16-byte read is conflict-free when 16 consecutive lanes (16
// consecutive rows, same piece) cover a whole 256-byte bank row: even rows need 8 distinct slots, and so do odd rows.
// (r & 7) alone repeats after 8 rows and halves the read rate; folding bit 3 into bit 0 satisfies both.
__device__ inline int lds_swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }
__device__ inline int lds_off(int row, int piece) { return row * 128 + ((piece ^ lds_swz(row)) << 4); }

// Tile geometry.  A workgroup of 4 wavefronts owns a B x B tile ("against" rows s x tested rows t) over all of K.
//   B = 128: the waves form a 2 x 2 grid of 64 x 64 sub-tiles (2 x 2 MFMA blocks each).
//   B = 64 : every wave computes the whole 64 x 64 tile for one quarter of each K chunk (k-split inside the
//            workgroup, same LDS traffic per MFMA as the 128 case); the four partial tiles are summed through LDS
//            in a fixed order before the epilogue, so results do not depend on scheduling.
// K advances in chunks of 128 bytes per row.  Global loads run D chunks ahead of the MFMAs in registers and pass
// through a double-buffered LDS stage.
template <int B> struct TileGeom {
    static constexpr bool KSPLIT = (B == 64);
    static constexpr int D = KSPLIT ? 4 : 2;                 // prefetch depth in chunks (even)
    static constexpr int ROWS = 2 * B;                       // "against" rows first, then tested rows
    static constexpr int LPT = ROWS / 32;                    // 16-byte pieces each thread moves per chunk
    static constexpr int STAGE = ROWS * 128;                 // bytes per LDS stage
    static constexpr int META = 4 * B * 4;                   // s_tok, t_tok, s_scale, t_scale
    static constexpr int RED = KSPLIT ? 4 * 4 * 16 * 64 * 4 : 0;   // cross-wave reduction scratch (aliases the stages)
    static constexpr int LDS = META + (2 * STAGE > RED ? 2 * STAGE : RED);
};

// max over the 16 accumulator rows this lane holds of |acc| * scale[s], optionally masked by token order
__device__ inline float block_max(const f32x16& v, const float* s_scale, const int* s_tok, int s_row0, int half,
                                  bool need_order, int ttok) {
    float m = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int sl = s_row0 + (i & 3) + 4 * half + 8 * (i >> 2);   // MFMA 32x32 accumulator row of register i
        float x = fabsf(v[i]) * s_scale[sl];
        if (need_order && !(s_tok[sl] < ttok)) x = 0.f;
        m = fmaxf(m, x);
    }
    return m;
}

__device__ inline void publish_max(float m, float tscale, int ttok, int half, uint32_t* gamma_bits) {
    m *= tscale;
    m = fmaxf(m, __shfl_xor(m, 32, 64));                       // the two lane halves hold different s rows
    // non-negative floats order like their bit patterns, so an integer atomicMax is an exact, order-independent max
    if (half == 0 && ttok >= 0 && m > 0.f) atomicMax(gamma_bits + ttok, __float_as_uint(m));
}

// The threshold test of one 32 x 32 block for tested token ttok, bit = "against" row within the block; the products are
// rounded exactly as for the row maximum ((|acc| * scale_s) * scale_t), so bits and maxima never disagree.
__device__ inline void publish_hits(const f32x16& v, const float* s_scale, const int* s_tok, int s_row0, int half,
                                    bool need_order, int ttok, float tscale, float thr, uint32_t* hits, int T, int s_glob0) {
    uint32_t bits = 0u;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int r32 = (i & 3) + 4 * half + 8 * (i >> 2);
        const int sl = s_row0 + r32;
        float x = (fabsf(v[i]) * s_scale[sl]) * tscale;
        if (need_order && !(s_tok[sl] < ttok)) x = 0.f;
        if (x >= thr) bits |= 1u << r32;
    }
    bits |= (uint32_t)__shfl_xor((int)bits, 32, 64);
    // (a block of "against" rows past the end has no word in the table: tiles are padded further than the table is)
    if (half == 0 && ttok >= 0 && s_glob0 < T) hits[(size_t)(s_glob0 >> 5) * (size_t)T + ttok] = bits;
}

template <typename In, int B, bool ALIGNED>
__device__ inline void gram_tile(const GramParams& p, const int32_t* listS, const int32_t* listT, int s0, int t0,
                                 int nS, int nT, bool need_order, char* lds) {
    using G = TileGeom<B>;
    constexpr int EPP = 16 / (int)sizeof(In);
    constexpr int EPC = 8 * EPP;
    constexpr int LPT = G::LPT, D = G::D;

    int* s_tok = reinterpret_cast<int*>(lds);
    int* t_tok = s_tok + B;
    float* s_scale = reinterpret_cast<float*>(t_tok + B);
    float* t_scale = s_scale + B;
    char* buf0 = lds + G::META;
    char* buf1 = buf0 + G::STAGE;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: code selected by it branches, not predicates
    const int l32 = lane & 31, half = lane >> 5;
    const In* X = reinterpret_cast<const In*>(p.X);

    // per-row metadata of the tile
    for (int i = tid; i < G::ROWS; i += 256) {
        const bool isS = i < B;
        const int li = isS ? s0 + i : t0 + (i - B);
        const int n = isS ? nS : nT;
        const int32_t* list = isS ? listS : listT;
        const bool ok = li < n;
        const int lc = ok ? li : n - 1;
        int tok = list ? list[lc] : lc;
        tok = min(max(tok, 0), p.T - 1);
        float sc = ok ? p.inv_norm[tok] : 0.f;
        if (isS) {
            if (p.mode == MODE_CROSS && !(p.gamma[tok] < p.thr)) sc = 0.f;   // Algorithm 1 step 7: valid representatives only
            s_tok[i] = ok ? tok : INT_MAX;
            s_scale[i] = sc;
        } else {
            t_tok[i - B] = ok ? tok : -1;
            t_scale[i - B] = sc;
        }
    }

    // the rows this thread stages: 8 consecutive lanes fetch one row's 128-byte chunk
    const int pc = tid & 7, rb = tid >> 3;
    const In* rowp[LPT];
    int woff[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
        const int row = rb + 32 * j;
        const bool isS = row < B;
        const int li = isS ? s0 + row : t0 + (row - B);
        const int n = isS ? nS : nT;
        const int32_t* list = isS ? listS : listT;
        const int lc = li < n ? li : n - 1;        // rows past the end re-read the last row; their results are masked
        int tok = list ? list[lc] : lc;
        tok = min(max(tok, 0), p.T - 1);
        rowp[j] = X + (size_t)tok * (size_t)p.ld;
        woff[j] = lds_off(row, pc);
    }

    constexpr int NB = G::KSPLIT ? 2 : (B / 2) / 32;   // MFMA blocks per wave per edge
    constexpr int WB = G::KSPLIT ? B : B / 2;          // wave tile edge
    constexpr int KS = G::KSPLIT ? 1 : 4;              // 16-element k-steps this wave runs per chunk
    const int ws = G::KSPLIT ? 0 : (wave >> 1), wt = G::KSPLIT ? 0 : (wave & 1);
    const int nk = (p.d + EPC - 1) / EPC;              // run as a multiple of D; the surplus chunks are all zero

    u32x4 pre[D][LPT];                                 // global prefetch: D chunks in flight per thread
    u32x4 fa[2][KS][NB], fb[2][KS][NB];                // MFMA operand fragments, double-buffered
    f32x16 acc[NB][NB];
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    auto fetch = [&](int set, int kc) {
#pragma unroll
        for (int j = 0; j < LPT; ++j) pre[set][j] = fetch_piece<In, ALIGNED>(rowp[j], kc * EPC + pc * EPP, p.d);
    };
    auto store = [&](char* stage, int set, int kc) {
#pragma unroll
        for (int j = 0; j < LPT; ++j)
            *reinterpret_cast<u32x4*>(stage + woff[j]) = finish_piece<ALIGNED>(pre[set][j], kc * EPC + pc * EPP, p.d);
    };
    auto read_frags = [&](const char* stage, int f) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int piece = (G::KSPLIT ? 2 * wave : 2 * ks) + half;
#pragma unroll
            for (int a = 0; a < NB; ++a)
                fa[f][ks][a] = *reinterpret_cast<const u32x4*>(stage + lds_off(ws * WB + a * 32 + l32, piece));
#pragma unroll
            for (int b = 0; b < NB; ++b)
                fb[f][ks][b] = *reinterpret_cast<const u32x4*>(stage + lds_off(B + wt * WB + b * 32 + l32, piece));
        }
    };
    auto mma = [&](int f) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int b = 0; b < NB; ++b) Mfma<In>::run(acc[a][b], fa[f][ks][a], fb[f][ks][b]);
    };

    // Software pipeline.  In iteration k the workgroup, after one barrier,
    //   reads the fragments of chunk k+1 from LDS stage (k+1)&1           (used by the MFMAs of iteration k+1)
    //   writes chunk k+2 from its prefetch registers into LDS stage k&1   (its global loads were issued D iterations ago)
    //   issues the global loads of chunk k+2+D into the registers just freed
    //   runs the MFMAs of chunk k on fragments read one iteration earlier,
    // so no instruction waits on a memory operation issued in the same iteration.  sched_barrier keeps the
    // program order of the loads, which is what lets the waits be counted (vmcnt) instead of draining.
#pragma unroll
    for (int s = 0; s < D; ++s) {
        fetch(s, s);
        __builtin_amdgcn_sched_barrier(0);
    }
    store(buf0, 0, 0);
    fetch(0, D);
    __builtin_amdgcn_sched_barrier(0);
    store(buf1, 1, 1);
    fetch(1, D + 1);
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
    read_frags(buf0, 0);
    for (int kc0 = 0; kc0 < nk; kc0 += D) {
#pragma unroll
        for (int s = 0; s < D; ++s) {                        // D is even: stages, fragment buffers and sets are static
            const int k = kc0 + s;
            __builtin_amdgcn_sched_barrier(0);
            __syncthreads();
            read_frags((s & 1) ? buf0 : buf1, (s + 1) & 1);
            store((s & 1) ? buf1 : buf0, (s + 2) % D, k + 2);
            fetch((s + 2) % D, k + 2 + D);
            mma(s & 1);
        }
    }

    // epilogue: a lane holds tested column n = l32 and 16 of the 32 "against" rows of each MFMA block
    uint32_t* gamma_bits = reinterpret_cast<uint32_t*>(p.gamma);
    if (G::KSPLIT) {
        // sum the four K-quarter partial tiles in wave order 0,1,2,3; wave w finishes block w = (a, b) = (w >> 1, w & 1)
        float* red = reinterpret_cast<float*>(buf0);          // [src wave][block][register][lane]
        __syncthreads();                                      // all waves are done reading the stages
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
            if (blk != wave) {
#pragma unroll
                for (int i = 0; i < 16; ++i) red[((wave * 4 + blk) * 16 + i) * 64 + lane] = acc[blk >> 1][blk & 1][i];
            }
        __syncthreads();
        f32x16 own;
        switch (wave) {
            case 0: own = acc[0][0]; break;
            case 1: own = acc[0][1]; break;
            case 2: own = acc[1][0]; break;
            default: own = acc[1][1]; break;
        }
        f32x16 tot;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            float v = 0.f;
#pragma unroll
            for (int src = 0; src < 4; ++src)
                v += (src == wave) ? own[i] : red[((src * 4 + wave) * 16 + i) * 64 + lane];
            tot[i] = v;
        }
        const int a = wave >> 1, b = wave & 1;
        const int nl = b * 32 + l32;
        const int ttok = t_tok[nl];
        const float m = block_max(tot, s_scale, s_tok, a * 32, half, need_order, ttok);
        publish_max(m, t_scale[nl], ttok, half, gamma_bits);
        if (p.hits)
            publish_hits(tot, s_scale, s_tok, a * 32, half, need_order, ttok, t_scale[nl], p.thr, p.hits, p.T, s0 + a * 32);
    } else {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int nl = wt * WB + b * 32 + l32;
            const int ttok = t_tok[nl];
            float m = 0.f;
#pragma unroll
            for (int a = 0; a < NB; ++a)
                m = fmaxf(m, block_max(acc[a][b], s_scale, s_tok, ws * WB + a * 32, half, need_order, ttok));
            publish_max(m, t_scale[nl], ttok, half, gamma_bits);
            if (p.hits) {
#pragma unroll
                for (int a = 0; a < NB; ++a)
                    publish_hits(acc[a][b], s_scale, s_tok, ws * WB + a * 32, half, need_order, ttok, t_scale[nl], p.thr,
                                 p.hits, p.T, s0 + ws * WB + a * 32);
            }
        }
    }
}

// Grid: a multiple of 8 workgroups.  Workgroup ids are dealt round-robin to the 8 XCDs, each with its own L2, so
// XCD x = blockIdx % 8 takes the contiguous tile range [x * per, (x + 1) * per): tiles that share operand rows run
// on one L2.  Tiles are numbered with the "against" block fastest.
template <typename In, int B, bool ALIGNED>
__global__ __launch_bounds__(256) void k_gram(GramParams p) {
    extern __shared__ __align__(16) char lds[];
    gram_group_offset(p);
    int nS, nT;
    const int32_t *listS = nullptr, *listT = nullptr;
    if (p.mode == MODE_FULL) {
        nS = nT = p.T;
    } else if (p.mode == MODE_REP) {
        nS = nT = p.meta[META_R];
        listS = listT = p.prev_idx;
    } else {
        nS = p.meta[META_R];
        nT = p.meta[META_NONREP];
        listS = p.prev_idx;
        listT = p.nonrep_idx;
    }
    if (nS < 1 || nT < 1) return;
    const long long nbS = (nS + B - 1) / B, nbT = (nT + B - 1) / B;
    const bool tri = p.mode != MODE_CROSS;
    const long long ntiles = tri ? nbT * (nbT + 1) / 2 : nbS * nbT;
    const long long per = (ntiles + 7) / 8;
    const int xcd = blockIdx.x & 7, slots = gridDim.x >> 3;
    for (long long slot = blockIdx.x >> 3; slot < per; slot += slots) {
        const long long tile = xcd * per + slot;
        if (tile >= ntiles) break;
        int tb, sb;
        if (tri) {
            tb = (int)((sqrtf(8.f * (float)tile + 1.f) - 1.f) * 0.5f);
            while ((long long)(tb + 1) * (tb + 2) / 2 <= tile) ++tb;
            while ((long long)tb * (tb + 1) / 2 > tile) --tb;
            sb = (int)(tile - (long long)tb * (tb + 1) / 2);
        } else {
            tb = (int)(tile / nbS);
            sb = (int)(tile % nbS);
        }
        const bool need_order = p.order_mask && (!tri || sb == tb);
        gram_tile<In, B, ALIGNED>(p, listS, listT, sb * B, tb * B, nS, nT, need_order, lds);
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------------
// k_update: threshold + compaction (one workgroup)

struct UpdateParams {
    const float* gamma;
    const uint8_t* is_rep;   // NULL: full selection (nothing inherited)
    const int32_t* meta;     // NULL in full selection
    int T;
    float thr;
    uint8_t* mask;           // may be NULL
    int32_t* idx;            // may be NULL
    int32_t* adds;           // may be NULL
    int32_t* removes;        // may be NULL
    int32_t* counts;         // [4]
    unsigned long long* gram_ops;   // may be NULL
    GroupOff go;             // full selection of several problems: blockIdx.x is the problem
};

__global__ __launch_bounds__(1024) void k_update(UpdateParams u) {
    __shared__ int sh[3][32];
    const int tid = threadIdx.x;
    if (u.go.ws) {
        const long long g = blockIdx.x;
        u.gamma = reinterpret_cast<const float*>(reinterpret_cast<const char*>(u.gamma) + g * u.go.ws);
        if (u.mask) u.mask += g * (long long)u.T;
        if (u.idx) u.idx += g * u.go.list;
        u.counts += g * u.go.counts;
        if (u.gram_ops) u.gram_ops += g * u.go.ops;
    }
    const bool full = u.is_rep == nullptr;
    int r_prev = 0;
    if (!full) {
        const int status = u.meta[META_STATUS];
        if (status != ADA_OK) {
            if (tid == 0) {
                u.counts[0] = 0; u.counts[1] = 0; u.counts[2] = 0; u.counts[3] = status;
                if (u.gram_ops) *u.gram_ops = 0ull;
            }
            return;
        }
        r_prev = u.meta[META_R];
    }
    const int T = u.T;
    const int chunk = (T + 1023) / 1024;
    const int lo = min(T, tid * chunk), hi = min(T, lo + chunk);
    int c_idx = 0, c_add = 0, c_rem = 0;
    for (int t = lo; t < hi; ++t) {
        const bool keep = u.gamma[t] < u.thr;           // strict "<" of the Definition
        const bool inh = !full && u.is_rep[t];
        c_idx += keep;
        c_add += keep && !inh;
        c_rem += !keep && inh;
    }
    int n_idx, n_add, n_rem;
    int o_idx = block_exclusive_scan(c_idx, &n_idx, sh[0]);
    int o_add = block_exclusive_scan(c_add, &n_add, sh[1]);
    int o_rem = block_exclusive_scan(c_rem, &n_rem, sh[2]);
    for (int t = lo; t < hi; ++t) {
        const bool keep = u.gamma[t] < u.thr;
        const bool inh = !full && u.is_rep[t];
        if (u.mask) u.mask[t] = keep ? 1 : 0;
        if (keep) { if (u.idx) u.idx[o_idx] = t; ++o_idx; }
        if (keep && !inh) { if (u.adds) u.adds[o_add] = t; ++o_add; }
        if (!keep && inh) { if (u.removes) u.removes[o_rem] = t; ++o_rem; }
    }
    if (tid == 0) {
        u.counts[0] = n_idx;
        u.counts[1] = n_add;
        u.counts[2] = n_rem;
        u.counts[3] = ADA_OK;
        if (u.gram_ops) {
            // Table 6 / eq. (6): one operation = one Gram entry
            const unsigned long long TT = (unsigned long long)T, r = (unsigned long long)r_prev;
            *u.gram_ops = full ? TT * TT : r * r + (TT - r) * (unsigned long long)(r_prev - n_rem);
        }
    }
}

__global__ __launch_bounds__(1024) void k_overlap(const uint8_t* a, const uint8_t* b, int T, int32_t* out) {
    __shared__ int sh[2][32];
    int ci = 0, cu = 0;
    for (int t = threadIdx.x; t < T; t += 1024) {
        const bool x = a[t] != 0, y = b[t] != 0;
        ci += x && y;
        cu += x || y;
    }
    int ti, tu;
    block_exclusive_scan(ci, &ti, sh[0]);
    block_exclusive_scan(cu, &tu, sh[1]);
    if (threadIdx.x == 0) { out[0] = ti; out[1] = tu; }
}

__global__ __launch_bounds__(256) void k_fill_u32(uint32_t* p, size_t n, uint32_t v) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = v;
}

// plain 16-byte copy of known size: the yardstick the HBM-traffic counters are scaled by
// two bf16 values with random sign and mantissa, magnitude in [0.5, 1): realistic switching activity, no overflow
__device__ inline uint32_t probe_bf16x2(uint32_t& s) {
    s = s * 1664525u + 1013904223u;
    const uint32_t a = s >> 16;
    s = s * 1664525u + 1013904223u;
    const uint32_t b = s >> 16;
    return ((a & 0x807Fu) | 0x3F00u) | (((b & 0x807Fu) | 0x3F00u) << 16);
}

__global__ __launch_bounds__(256) void k_mfma_probe(float* sink, int iters) {
    f32x16 acc[16];
#pragma unroll
    for (int a = 0; a < 16; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[a][i] = 0.f;
    uint32_t seed = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    u32x4 x[4], y[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int i = 0; i < 4; ++i) { x[q][i] = probe_bf16x2(seed); y[q][i] = probe_bf16x2(seed); }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) Mfma<uint16_t>::run(acc[a * 4 + b], x[a], y[b]);
    }
    float sum = 0.f;
#pragma unroll
    for (int a = 0; a < 16; ++a)
#pragma unroll
        for (int i = 0; i < 16; ++i) sum += acc[a][i];
    if (sum == 123.456f) sink[blockIdx.x] = sum;           // sums of +-[0.25, 1) products: never this value in practice
}

__global__ __launch_bounds__(256) void k_copy_probe(u32x4* __restrict__ dst, const u32x4* __restrict__ src, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

#include "ada_fused.hpp"
#include "ada_gram_dma.hpp"
#include "ada_attn.hpp"

// ------------------------------------------------------------------------------------------------
// host side

// Measurement aid: when enabled, every kernel launch is bracketed by two HIP events recorded on the stream the
// kernel is launched on; ada_profile_collect() turns them into per-kernel-class totals.
struct ProfRecord { int cls; hipEvent_t a, b; };
bool g_prof_on = false;
std::vector<ProfRecord> g_prof;
std::mutex g_prof_mu;

struct ProfScope {
    hipStream_t st;
    bool on;
    ProfRecord rec;
    ProfScope(int cls, hipStream_t s) : st(s), on(g_prof_on) {
        if (!on) return;
        rec.cls = cls;
        if (hipEventCreate(&rec.a) != hipSuccess || hipEventCreate(&rec.b) != hipSuccess) { on = false; return; }
        (void)hipEventRecord(rec.a, st);
    }
    ~ProfScope() {
        if (!on) return;
        (void)hipEventRecord(rec.b, st);
        std::lock_guard<std::mutex> lk(g_prof_mu);
        g_prof.push_back(rec);
    }
};

// ------------------------------------------------------------------------------------------------
// k_greedy_resolve: the greedy covering of Section 2.5 from the bit table of the full Gram.
//   token t is a representative iff no EARLIER REPRESENTATIVE s has |G_st| >= threshold.
// The decision of token t needs the decisions of all s < t, so one workgroup walks the tokens in blocks of 64:
//   inside a block, wave 0 decides the 64 tokens one after the other with scalar bit operations (the block's own
//   two words of every token hold its earlier hits inside the block);
//   then every thread pushes the block's new representatives to the later tokens it owns: token t' is covered as
//   soon as one of its two words for this block meets the block's representative bits.
// The words of block b + 1 are requested before block b is decided (they do not depend on it), so the trips to
// memory overlap the serial part.  covered[] lives in LDS (T <= FUSED_MAX_T bytes).
struct GreedyParams {
    const uint32_t* hits;    // [words][T]
    int T;
    uint8_t* mask;           // [T], may be NULL
    int32_t* idx;            // [T], may be NULL
    int32_t* counts;         // [4] = {r, r, 0, 0}
    unsigned long long* gram_ops;   // may be NULL
};

constexpr int GREEDY_THREADS = 1024;

// TPT: tokens a thread owns (T <= TPT * 1024); AHEAD: how many blocks ahead of the decisions the words are requested
// (registers: 2 * TPT * (AHEAD + 1) words per thread; the deeper ring of the small shapes hides a trip to memory
// behind several blocks' decisions, which take well under a microsecond each)
template <int TPT, int AHEAD>
__global__ __launch_bounds__(GREEDY_THREADS) void k_greedy_resolve(GreedyParams g) {
    __shared__ uint8_t covered[TPT * GREEDY_THREADS];
    __shared__ uint32_t repw[TPT * GREEDY_THREADS / 32];
    __shared__ uint32_t own_lo[64], own_hi[64];
    __shared__ int sh[32];
    const int tid = threadIdx.x, lane = tid & 63;
    const int T = g.T, nblk = (T + 63) >> 6;
    for (int t = tid; t < T; t += GREEDY_THREADS) covered[t] = 0;
    for (int w = tid; w < 2 * nblk; w += GREEDY_THREADS) repw[w] = 0u;
    __syncthreads();
    // This thread owns tokens tid, tid + 1024, ...; ring[k]: their two words for block (current + k).  Addresses are
    // clamped and the values masked where they are USED, so nothing waits at the load.
    uint32_t lo[AHEAD + 1][TPT], hi[AHEAD + 1][TPT];
    auto fetch = [&](int b, uint32_t (&a)[TPT], uint32_t (&c)[TPT]) {
        const int bc = b < nblk ? b : nblk - 1;
#pragma unroll
        for (int j = 0; j < TPT; ++j) {
            const int t = tid + j * GREEDY_THREADS;
            const int tc = t < T ? t : 0;
            a[j] = g.hits[(size_t)(2 * bc) * T + tc];
            c[j] = g.hits[(size_t)(2 * bc + 1) * T + tc];
        }
    };
#pragma unroll
    for (int k = 0; k < AHEAD; ++k) fetch(k, lo[k], hi[k]);
    for (int b = 0; b < nblk; ++b) {
        fetch(b + AHEAD, lo[AHEAD], hi[AHEAD]);              // in flight while this and the next blocks are decided
        // hand the block's own words to wave 0 through LDS (token 64 b + l is owned by thread (64 b + l) % 1024)
#pragma unroll
        for (int j = 0; j < TPT; ++j) {
            const int t = tid + j * GREEDY_THREADS;
            // (the block's second word may lie wholly past the end of the sequence: nobody wrote it)
            if ((t >> 6) == b && t < T) { own_lo[t & 63] = lo[0][j]; own_hi[t & 63] = 64 * b + 32 < T ? hi[0][j] : 0u; }
        }
        __syncthreads();
        if (tid < 64) {                                      // wave 0: the block's decisions, in token order
            const int t = 64 * b + lane;
            const bool exists = t < T;
            const uint32_t mlo = exists ? own_lo[lane] : 0u, mhi = exists ? own_hi[lane] : 0u;
            // tokens no earlier block's representative covers; only these can become representatives
            unsigned long long cand = __ballot(exists && covered[exists ? t : 0] == 0);
            unsigned long long rep = 0ull;
            while (cand) {                                   // scalar loop over the candidates
                const int i = __builtin_amdgcn_readfirstlane((int)__ffsll((long long)cand) - 1);
                cand &= cand - 1;
                const unsigned long long h = ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)mhi, i) << 32) |
                                             (unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)mlo, i);
                if (!(h & rep)) rep |= 1ull << i;            // no earlier representative of this block is within tau
            }
            if (lane == 0) { repw[2 * b] = (uint32_t)rep; repw[2 * b + 1] = (uint32_t)(rep >> 32); }
        }
        __syncthreads();
        const uint32_t rlo = repw[2 * b], rhi = 64 * b + 32 < T ? repw[2 * b + 1] : 0u;
#pragma unroll
        for (int j = 0; j < TPT; ++j) {                      // push: later tokens hit by one of the new representatives
            const int t = tid + j * GREEDY_THREADS;
            if (t < T && (t >> 6) > b && ((lo[0][j] & rlo) | (hi[0][j] & rhi))) covered[t] = 1;
        }
#pragma unroll
        for (int k = 0; k < AHEAD; ++k)
#pragma unroll
            for (int j = 0; j < TPT; ++j) { lo[k][j] = lo[k + 1][j]; hi[k][j] = hi[k + 1][j]; }
        __syncthreads();
    }
    // representatives -> mask, ascending index list, count
    const int chunk = (T + GREEDY_THREADS - 1) / GREEDY_THREADS;
    const int t_lo = min(T, tid * chunk), t_hi = min(T, t_lo + chunk);
    int c = 0;
    for (int t = t_lo; t < t_hi; ++t) c += (repw[t >> 5] >> (t & 31)) & 1u;
    int total;
    int off = block_exclusive_scan(c, &total, sh);
    for (int t = t_lo; t < t_hi; ++t) {
        const int is = (repw[t >> 5] >> (t & 31)) & 1u;
        if (g.mask) g.mask[t] = (uint8_t)is;
        if (is && g.idx) g.idx[off] = t;
        off += is;
    }
    if (tid == 0) {
        g.counts[0] = total; g.counts[1] = total; g.counts[2] = 0; g.counts[3] = ADA_OK;
        if (g.gram_ops) *g.gram_ops = (unsigned long long)T * (unsigned long long)T;
    }
}

template <int B> constexpr int gram_lds_bytes() { return TileGeom<B>::LDS; }

template <typename In, int B, bool ALIGNED>
hipError_t launch_gram(const GramParams& p, long long tiles_upper, hipStream_t st, int groups = 1) {
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    constexpr int lds = gram_lds_bytes<B>();
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gram<In, B, ALIGNED>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    if (attr_err != hipSuccess) return attr_err;
    if (tiles_upper < 1) return hipSuccess;
    const unsigned grid = (unsigned)((tiles_upper < 65528 ? tiles_upper : 65528) + 7) / 8 * 8;   // multiple of 8 (XCDs)
    ProfScope ps(p.mode == MODE_FULL ? ADA_K_GRAM_FULL : p.mode == MODE_REP ? ADA_K_GRAM_REP : ADA_K_GRAM_CROSS, st);
    hipLaunchKernelGGL((k_gram<In, B, ALIGNED>), dim3(grid, groups), dim3(256), lds, st, p);
    return hipGetLastError();
}

inline long long tiles_for(int mode, int nS, int nT, int B) {
    const long long nbS = (nS + B - 1) / B, nbT = (nT + B - 1) / B;
    return mode == MODE_CROSS ? nbS * nbT : nbT * (nbT + 1) / 2;
}

// Development switches (listed in include/ada.h) force code paths for tests and measurements.  They are honoured only
// when ADA_DEV_SWITCHES=1 is set as well, so that a stray variable in a user's environment changes nothing.
const char* dev_switch(const char* name) {
    const char* on = getenv("ADA_DEV_SWITCHES");
    if (!on || on[0] != '1' || on[1] != '\0') return nullptr;
    return getenv(name);
}

int tile_override() {
    const char* e = dev_switch("ADA_TILE");
    if (!e) return 0;
    const int v = atoi(e);
    return (v == 64 || v == 128) ? v : 0;
}

// Compute units of the current device, rounded down to whole XCDs (at least 8).
int device_cus() {
    static std::once_flag once;
    static int cus = 256;
    std::call_once(once, [] {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n >= 8)
            cus = n / 8 * 8;
    });
    return cus;
}

// Makespan of handing the units out big first to G workgroups, in units of one big tile; a small unit was measured at
// about 0.4 of a big one.
inline double dma_makespan(int T, int big_mode, int G) {
    const DmaUnits U(T, big_mode);
    if (U.n_units > 64LL * G) return ((double)U.n_big + 0.4 * (double)(U.n_units - U.n_big)) / G;
    std::vector<double> fin(G, 0.0);
    for (long long u = 0; u < U.n_units; ++u) {
        int best = 0;
        for (int g = 1; g < G; ++g) if (fin[g] < fin[best]) best = g;
        fin[best] += u < U.n_big ? 1.0 : 0.4;
    }
    double m = 0.0;
    for (double f : fin) m = f > m ? f : m;
    return m;
}

// Makespan, in staged rows, of the one-launch form's units (big first, then the shared-row diagonal blocks of 128
// rows) handed to G workgroups: what a CU can pull out of the L2 bounds these sizes, so rows are the cost.
inline long long dma_makespan_norms(int T, int mode, int G) {
    const DmaUnits U(T, mode);
    std::priority_queue<long long, std::vector<long long>, std::greater<long long>> fin;
    for (int g = 0; g < G; ++g) fin.push(0);
    long long m = 0;
    for (long long u = 0; u < U.n_units; ++u) {
        long long rows;
        if (mode == 2) rows = u < U.n_big ? 192 : 128;
        else rows = 256;
        const long long f = fin.top() + rows + 64;            // (+ a unit's fixed part, in the same currency)
        fin.pop();
        fin.push(f);
        m = f > m ? f : m;
    }
    return m;
}

// mode: 0 = 128 x 128 units everywhere, 1 = 256 x 256 off the diagonal, 2 = 64 x 128 off the diagonal (one-launch form
// only), -1 = whichever hands out better
// u.counts != NULL: the workgroup that leaves last also applies the threshold and compacts the set (no update launch)
template <bool NORMS>
hipError_t launch_gram_dma(const GramParams& p, int32_t* meta, int mode, hipStream_t st, int groups,
                           const UpdateParams& u, float* gamma_out = nullptr) {
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gram_dma<NORMS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, DmaGeom::LDS);
    });
    if (attr_err != hipSuccess) return attr_err;
    int G = device_cus();                                      // one workgroup per CU (LDS), whole XCDs
    if (groups > 1) {                                          // the problems share the chip; units beyond a problem's
        G = G / groups / 8 * 8;                                // workgroups are handed out through its queue
        if (G < 8) G = 8;
    }
    if (NORMS) {                                               // the one-launch form runs on 128-row units: whole or halved
        if (mode == 1) mode = 0;                               // (256-row units are not built for this form)
        if (mode < 0) {
            static std::mutex mu;
            static int last_T = 0, last_G = 0, last_mode = 0;
            std::lock_guard<std::mutex> lock(mu);
            if (last_T != p.T || last_G != G) {
                last_mode = dma_makespan_norms(p.T, 2, G) < dma_makespan_norms(p.T, 0, G) ? 2 : 0;
                last_T = p.T;
                last_G = G;
            }
            mode = last_mode;
        }
    } else if (mode == 2) {
        mode = 0;                                              // (64 x 128 units exist in the one-launch form only)
    } else if (mode < 0) {
        static std::mutex mu;
        static int last_T = 0, last_G = 0, last_mode = 0;     // the choice depends on both the size and the workgroups
        std::lock_guard<std::mutex> lock(mu);
        if (last_T != p.T || last_G != G) {
            last_mode = dma_makespan(p.T, 1, G) < dma_makespan(p.T, 0, G) ? 1 : 0;
            last_T = p.T;
            last_G = G;
        }
        mode = last_mode;
    }
    ProfScope ps(ADA_K_GRAM_FULL, st);
    hipLaunchKernelGGL(k_gram_dma<NORMS>, dim3(G, groups), dim3(NORMS ? SplitGeom::THREADS : DmaGeom::THREADS), DmaGeom::LDS, st, p, mode, meta, u,
                       gamma_out);
    return hipGetLastError();
}

// nS_upper / nT_upper: host-known upper bounds of the list lengths (the kernel reads the actual ones).
// 128-tiles need half the operand traffic per flop but only pay off when they still fill the chip; with sizes
// known only on the device (exact == false) the 64-tile, which suits every skinny cascade shape, is used.
template <typename In, bool ALIGNED>
hipError_t launch_gram_any(const GramParams& p, int nS_upper, int nT_upper, bool exact, hipStream_t st, int groups = 1) {
    int B = (exact && tiles_for(p.mode, nS_upper, nT_upper, 128) * groups >= 192) ? 128 : 64;
    if (int o = tile_override()) B = o;
    if (B == 128) return launch_gram<In, 128, ALIGNED>(p, tiles_for(p.mode, nS_upper, nT_upper, 128), st, groups);
    return launch_gram<In, 64, ALIGNED>(p, tiles_for(p.mode, nS_upper, nT_upper, 64), st, groups);
}

template <typename In, bool ALIGNED>
hipError_t launch_norm_prep(const void* X, long long ld, int T, int d, float* gamma, const Workspace& w,
                            const PrepParams& prep, hipStream_t st, const GroupOff& go = GroupOff{0, 0, 0, 0, 0},
                            int groups = 1) {
    const int nb = (T + 3) / 4;
    ProfScope ps(ADA_K_NORM_PREP, st);
    hipLaunchKernelGGL((k_norm_prep<In, ALIGNED>), dim3(nb + (prep.enabled ? 1 : 0), groups), dim3(256), 0, st,
                       reinterpret_cast<const In*>(X), ld, T, d, w.inv_norm, gamma, w, prep, nb, go);
    return hipGetLastError();
}

int launch_update(const UpdateParams& u, hipStream_t st, int groups = 1) {
    ProfScope ps(ADA_K_UPDATE, st);
    hipLaunchKernelGGL(k_update, dim3(groups), dim3(1024), 0, st, u);
    return hipGetLastError() == hipSuccess ? ADA_OK : ADA_ERR_DEVICE;
}

template <typename In_, bool A_> struct Variant { using In = In_; static constexpr bool aligned = A_; };

// 16-byte vector loads need an aligned base, ld and d that are multiples of the piece size; anything else
// takes the element-wise loader.
template <typename F>
hipError_t dispatch(int dtype, const void* X, long long ld, int d, F&& f) {
    const int epp = dtype == ADA_BF16 ? 8 : 4;
    const bool al = ((uintptr_t)X % 16 == 0) && (ld % epp == 0) && (d % epp == 0);
    if (dtype == ADA_BF16) return al ? f(Variant<uint16_t, true>{}) : f(Variant<uint16_t, false>{});
    return al ? f(Variant<float, true>{}) : f(Variant<float, false>{});
}

// bf16: the kernel that keeps scores and weights in registers (eight waves: four multiply, four fetch)
template <int DH>
hipError_t launch_attn_regs(const AttnParams& p, hipStream_t st) {
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    constexpr int lds = AttnGeom2<DH>::LDS;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_rep2<DH>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    if (attr_err != hipSuccess) return attr_err;
    ProfScope ps(ADA_K_ATTN, st);
    int gx = (p.r_host + 63) / 64;
    if (p.r_dev) {
        const int fit = (device_cus() + p.H - 1) / p.H;
        gx = gx < fit ? gx : fit;
    }
    hipLaunchKernelGGL((k_attn_rep2<DH>), dim3(gx, p.H), dim3(512), lds, st, p);
    return hipGetLastError();
}

template <typename In, int DH>
hipError_t launch_attn(const AttnParams& p, hipStream_t st) {
    if constexpr (sizeof(In) == 2) {
        static const bool first_kernel = [] {             // development switch: ADA_ATTN=lds keeps the first kernel
            const char* e = dev_switch("ADA_ATTN");
            return e && std::string(e) == "lds";
        }();
        // its hand-over stores 16 bytes per lane
        const bool out16 = (uintptr_t)p.out % 16 == 0 && p.ld_out % 4 == 0;
        if (!first_kernel && out16) return launch_attn_regs<DH>(p, st);
    }
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    constexpr int lds = AttnGeom<In, DH>::LDS;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_attn_rep<In, DH>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    if (attr_err != hipSuccess) return attr_err;
    ProfScope ps(ADA_K_ATTN, st);
    int gx = (p.r_host + 63) / 64;
    if (p.r_dev) {                                         // size known on the device only: about one workgroup per CU
        const int fit = (device_cus() + p.H - 1) / p.H;
        gx = gx < fit ? gx : fit;
    }
    hipLaunchKernelGGL((k_attn_rep<In, DH>), dim3(gx, p.H), dim3(256), lds, st, p);
    return hipGetLastError();
}

int check_common(const void* X, int T, int d, int64_t ld, int dtype, float tau, void* ws, size_t ws_bytes) {
    if (!X || !ws) return ADA_ERR_NULL;
    if (dtype != ADA_F32 && dtype != ADA_BF16) return ADA_ERR_DTYPE;
    if (T < 1 || d < 1 || ld < d || T > ADA_MAX_T) return ADA_ERR_SHAPE;
    if (!(tau > 0.f && tau < 1.f)) return ADA_ERR_TAU;
    if (ws_bytes < ws_bytes_for(T) || ((uintptr_t)ws % 256) != 0) return ADA_ERR_WORKSPACE;
    return ADA_OK;
}

// 1 - tau^2 evaluated in double and rounded once to the fp32 the comparisons run in
inline float threshold_of(float tau) { return (float)(1.0 - (double)tau * (double)tau); }

// Definition "Gram threshold": norms, lower-triangular Gram tiles, threshold + compaction.  Arguments checked by the caller.
int run_full(const void* X, int T, int d, long long ld, int dtype, float tau, uint8_t* mask, int32_t* idx,
             int32_t* counts, uint64_t* gram_ops, float* gamma, void* ws, hipStream_t st,
             int groups = 1, const GroupOff& go = GroupOff{0, 0, 0, 0, 0}, bool greedy = false) {
    // groups > 1: that many problems in each of the three launches (go: their strides; gamma must be NULL, so that
    // every problem's row maxima live in its own workspace)
    const Workspace w = carve(ws, T);
    float* g = gamma ? gamma : w.gamma;
    const float thr = threshold_of(tau);
    const PrepParams prep = {nullptr, nullptr, 0, 0};
    // greedy covering (Section 2.5): the tiles also leave the threshold bits of every pair s < t, and the set is
    // resolved from them in token order (one problem, T <= FUSED_MAX_T: checked by the caller)
    const GramParams p = {X, ld, T, d, nullptr, nullptr, nullptr, w.inv_norm, g, thr, MODE_FULL, 1, go.x, go.ws,
                          greedy ? w.hits : nullptr};
    const UpdateParams u = {g, nullptr, nullptr, T, thr, mask, idx, nullptr, nullptr, counts,
                            reinterpret_cast<unsigned long long*>(gram_ops), go};
    // Up to T = 4096 a launch is mostly latency, and the direct-to-LDS kernel finishes the selection itself (its last
    // workgroup applies the threshold and compacts): one launch and one gap less.  Beyond that the tiles keep the
    // chip busy for hundreds of microseconds and the update stays a launch of its own.
    const bool finish_in_kernel = !greedy && T <= 4096;
    const UpdateParams in_kernel = finish_in_kernel ? u : UpdateParams{};
    bool finished = false;
    const char* path_env = dev_switch("ADA_GRAM");               // development switch: tile, dma0, dma1, dma2
    const std::string path = path_env ? path_env : "";
    const long long ld_seen = (groups > 1 && go.x % 16 != 0) ? 1 : ld;   // every problem's rows must suit the loader
    hipError_t e = dispatch(dtype, X, ld_seen, d, [&](auto v) {
        using V = decltype(v);
        using In = typename V::In;
        if constexpr (V::aligned && sizeof(In) == 2) {
            // whole 64-byte pieces of bf16 rows: the direct-to-LDS kernel
            const bool can = d % DmaGeom::HC == 0 && go.x % 64 == 0;
            if (can && (path == "dma0" || path == "dma1" || path == "dma2" || (path.empty() && T >= 1536))) {
                const int mode = path.empty() ? -1 : path == "dma1" ? 1 : path == "dma2" ? 2 : 0;
                if (finish_in_kernel && d % SplitGeom::EPC == 0) {
                    // ONE launch: the norms come from the tiles' own fragments, and the row maxima are accumulated in a
                    // workspace array that is zero between calls (the workgroup that finishes hands them over and
                    // clears it again), so nothing has to be computed or cleared ahead of the tiles.
                    GramParams q = p;
                    q.inv_norm = nullptr;
                    q.gamma = reinterpret_cast<float*>(w.first);
                    finished = true;
                    return launch_gram_dma<true>(q, w.meta, mode, st, groups, in_kernel, gamma);
                }
                hipError_t e0 = launch_norm_prep<In, V::aligned>(X, ld, T, d, g, w, prep, st, go, groups);
                if (e0 != hipSuccess) return e0;
                return launch_gram_dma<false>(p, w.meta, mode, st, groups, in_kernel);
            }
        }
        hipError_t e1 = launch_norm_prep<In, V::aligned>(X, ld, T, d, g, w, prep, st, go, groups);
        if (e1 != hipSuccess) return e1;
        return launch_gram_any<In, V::aligned>(p, T, T, true, st, groups);
    });
    if (e != hipSuccess) return ADA_ERR_DEVICE;
    if (greedy) {
        const GreedyParams gp = {w.hits, T, mask, idx, counts, reinterpret_cast<unsigned long long*>(gram_ops)};
        ProfScope ps(ADA_K_UPDATE, st);
        if (T <= 2 * GREEDY_THREADS) hipLaunchKernelGGL((k_greedy_resolve<2, 4>), dim3(1), dim3(GREEDY_THREADS), 0, st, gp);
        else if (T <= 4 * GREEDY_THREADS) hipLaunchKernelGGL((k_greedy_resolve<4, 3>), dim3(1), dim3(GREEDY_THREADS), 0, st, gp);
        else if (T <= 8 * GREEDY_THREADS) hipLaunchKernelGGL((k_greedy_resolve<8, 3>), dim3(1), dim3(GREEDY_THREADS), 0, st, gp);
        else hipLaunchKernelGGL((k_greedy_resolve<FUSED_MAX_T / GREEDY_THREADS, 1>), dim3(1), dim3(GREEDY_THREADS), 0, st, gp);
        return hipGetLastError() == hipSuccess ? ADA_OK : ADA_ERR_DEVICE;
    }
    if (finished) return ADA_OK;
    return launch_update(u, st, groups);
}

hipError_t fill_u32(void* p, size_t n_words, uint32_t v, hipStream_t st) {
    if (n_words == 0) return hipSuccess;
    const unsigned grid = (unsigned)((n_words + 255) / 256 < 2048 ? (n_words + 255) / 256 : 2048);
    hipLaunchKernelGGL(k_fill_u32, dim3(grid), dim3(256), 0, st, (uint32_t*)p, n_words, v);
    return hipGetLastError();
}

template <typename In, bool ALIGNED, int KG, bool DMA>
hipError_t launch_fused(const FusedParams& p, hipStream_t st, int prof_class = ADA_K_CASCADE_FUSED) {
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    constexpr int lds = FusedGeom<KG, DMA>::LDS;
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_cascade_fused<In, ALIGNED, KG, DMA>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    if (attr_err != hipSuccess) return attr_err;
    FusedParams q = p;
    unsigned grid;
    if (p.groups > 1) {
        // the groups share the chip: about one workgroup per CU in all, and no more per group than it has tiles
        const long long tiles = tile_count(p.r_host, p.T, 0);
        long long wpg = device_cus() / p.groups;
        if (wpg < 1) wpg = 1;
        if (wpg > tiles) wpg = tiles;
        q.wpg = (int)wpg;
        grid = (unsigned)(p.groups * wpg);
    } else {
        // with the set size known here the tile shape is too (the kernel makes the same choice from the same numbers)
        int shape = 0;
        if (ALIGNED && KG == 2 && DMA && !p.r_dev)
            shape = cascade_tile_shape(p.r_host, p.T, p.d, p.tile_pick, p.tile_pick, sizeof(In) == 2 ? 4 : 3);
        long long tiles = tile_count(p.r_host, p.T, shape);
        // Workgroups loop over tiles, so any grid is correct.  With the set size known only on the device the bound
        // r_host = T would launch mostly idle workgroups, and dispatching those is not free: cap at one per CU (the LDS
        // footprint admits no more at a time anyway).
        const long long cap = p.r_dev ? device_cus() : 2048;
        if (tiles > cap) tiles = cap;
        grid = (unsigned)(tiles + 7) / 8 * 8;                        // multiple of 8 (XCDs)
    }
    q.grid = (int)grid;
    // first-hit records are kept only where the update can take them (four tokens per 16-byte load, 32 per thread)
    if (p.T % 4 != 0 || p.T > 32 * 256 * KG) q.first = nullptr;
    ProfScope ps(prof_class, st);
    hipLaunchKernelGGL((k_cascade_fused<In, ALIGNED, KG, DMA>), dim3(grid), dim3(256 * KG), lds, st, q);
    return hipGetLastError();
}

int kgroups_override() {
    const char* e = dev_switch("ADA_KGROUPS");
    if (!e) return 0;
    const int v = atoi(e);
    return (v == 1 || v == 2) ? v : 0;
}

// FusedParams::tile_pick: the CU count (automatic choice per step) unless the development switch fixes the shape.
int cascade_tile_pick() {
    const char* e = dev_switch("ADA_CASCADE_TILE");          // representatives x tokens: 64, 64x128, 128, 256x128 (tokens x reps)
    if (e) {
        const std::string v(e);
        if (v == "64") return 0;
        if (v == "64x128") return -1;
        if (v == "128") return -2;
        if (v == "256x128") return -3;
    }
    return device_cus();
}

// Picks the form of the one-launch kernel: two K-groups unless overridden; direct-to-LDS operand loads when rows come
// in whole, aligned 128-byte chunks.
int launch_fused_any(const FusedParams& p, int dtype, int prof_class, hipStream_t st) {
    int kg = 2;
    if (int o = kgroups_override()) kg = o;
    const char* no_dma = dev_switch("ADA_NO_DMA");
    // the form of the kernel must suit every group's rows: a group stride off the 16-byte grid takes the element-wise
    // loader for all of them (dispatch looks at base, ld and d)
    const long long ld_seen = (p.groups > 1 && p.x_gs % 16 != 0) ? 1 : p.ld;
    hipError_t e = dispatch(dtype, p.X, ld_seen, p.d, [&](auto v) {
        using V = decltype(v);
        using In = typename V::In;
        constexpr int epc = 128 / (int)sizeof(In);
        if constexpr (V::aligned) {
            if (p.d % epc == 0 && !(no_dma && no_dma[0] == '1'))
                return kg == 2 ? launch_fused<In, true, 2, true>(p, st, prof_class)
                               : launch_fused<In, true, 1, true>(p, st, prof_class);
        }
        return kg == 2 ? launch_fused<In, V::aligned, 2, false>(p, st, prof_class)
                       : launch_fused<In, V::aligned, 1, false>(p, st, prof_class);
    });
    return e == hipSuccess ? ADA_OK : ADA_ERR_DEVICE;
}

// Algorithm 1 in one launch (ada_fused.hpp).  gamma, if given, receives for an inherited token gamma^rep and for any
// other token gamma^cross.  The tiles accumulate a token's maximum over ALL inherited representatives; for the tokens
// whose nearest one turned out removed (listed by the workgroup that updates the set) the maximum over the VALID ones is
// recomputed by the cross-Gram tiles of the step's other form on that list: a norm launch and a tile launch more.
int run_cascade_fused(const void* X, int T, int d, long long ld, int dtype, float tau, const int32_t* prev_idx, int r,
                      const int32_t* r_dev, int32_t* idx, int32_t* adds, int32_t* removes, int32_t* counts,
                      uint64_t* gram_ops, float* gamma, void* ws, hipStream_t st, unsigned flags,
                      const ada_groups* grp = nullptr, const ada_tau_control* ctl = nullptr, const double* tau_in = nullptr,
                      const float* thr_in = nullptr, double* tau_out = nullptr, float* thr_out = nullptr) {
    const Workspace w = carve(ws, T);
    if (gamma && fill_u32(gamma, (size_t)T, 0u, st) != hipSuccess) return ADA_ERR_DEVICE;
    FusedParams p = {X, ld, T, d, prev_idx, r_dev, r, threshold_of(tau),
                     (flags & ADA_FLAG_CROSS_EARLIER_ONLY) ? 1 : 0, w.hits, hit_words(r), gamma,
                     w.meta + META_TICKET, idx, adds, removes, counts,
                     reinterpret_cast<unsigned long long*>(gram_ops), 0, nullptr, nullptr, nullptr, 0, cascade_tile_pick()};
    p.first = w.first;
    if (gamma && !(grp && grp->G > 1)) {                          // Algorithm 1's gamma^cross: see above
        p.best = w.best; p.fix_list = w.nonrep_idx; p.fix_meta = w.meta;
    }
    if (ctl) {                                                   // Section 8.1: threshold carried on the device
        p.tau_in = tau_in; p.thr_in = thr_in; p.tau_out = tau_out; p.thr_out = thr_out;
        p.kappa = ctl->kappa; p.eta_target = ctl->eta_target; p.tau_min = ctl->tau_min; p.tau_max = ctl->tau_max;
    }
    if (grp && grp->G > 1) {                                     // ws: G workspaces back to back
        p.groups = grp->G;
        p.x_gs = grp->x_gstride * (dtype == ADA_BF16 ? 2 : 4);
        p.list_gs = grp->list_gstride;
        p.counts_gs = grp->counts_gstride;
        p.ops_gs = grp->ops_gstride;
        p.ws_gs = (long long)ws_bytes_for(T);
    }
    const int rc = launch_fused_any(p, dtype, ADA_K_CASCADE_FUSED, st);
    if (rc != ADA_OK || !p.fix_list) return rc;
    // (a rejected step leaves an empty list; the validity of a representative is read off its own gamma^rep < threshold,
    //  as in the step's other form)
    GramParams cross = {X, ld, T, d, prev_idx, w.nonrep_idx, w.meta, w.inv_norm, gamma, threshold_of(tau), MODE_CROSS,
                        (flags & ADA_FLAG_CROSS_EARLIER_ONLY) ? 1 : 0};
    const PrepParams norms_only = {nullptr, nullptr, 0, 0};
    const hipError_t e = dispatch(dtype, X, ld, d, [&](auto v) {
        using V = decltype(v);
        hipError_t e1 = launch_norm_prep<typename V::In, V::aligned>(X, ld, T, d, w.gamma, w, norms_only, st);
        if (e1 != hipSuccess) return e1;
        return launch_gram_any<typename V::In, V::aligned>(cross, r, T - 1 > 0 ? T - 1 : 1, false, st);
    });
    return e == hipSuccess ? ADA_OK : ADA_ERR_DEVICE;
}

// Section 2.3 on the same tile engine: T x r products against the set R, per-token arg max.
// pos: optional [T], the position in R of every token's representative (for the attention that follows)
int run_assign(const void* X, int T, int d, long long ld, int dtype, const int32_t* idx, int r, const int32_t* r_dev,
               int32_t* assign, float* corr, int32_t* info, void* ws, hipStream_t st, int32_t* pos = nullptr) {
    const Workspace w = carve(ws, T);
    FusedParams p = {X, ld, T, d, idx, r_dev, r, 2.0f, 0, nullptr, 0, nullptr, w.meta + META_TICKET,
                     nullptr, nullptr, nullptr, info, nullptr, 1, w.best, assign, corr, 0, cascade_tile_pick()};
    p.pos_out = pos;
    return launch_fused_any(p, dtype, ADA_K_ASSIGN, st);
}

__global__ void k_fill_status(int32_t* counts, int rows, int status) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < rows * 4) counts[i] = (i & 3) == 3 ? status : 0;
}

template <typename In, bool ALIGNED, int KG, bool DMA>
hipError_t launch_pass(const PassParams& pp, hipStream_t st) {
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    constexpr int lds = FusedGeom<KG, DMA>::LDS;
    static_assert(lds > 80 * 1024, "the pass kernel relies on one workgroup per CU");
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_cascade_pass<In, ALIGNED, KG, DMA>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    if (attr_err != hipSuccess) return attr_err;
    PassParams q = pp;
    q.f.grid = device_cus();
    ProfScope ps(ADA_K_CASCADE_FUSED, st);
    hipLaunchKernelGGL((k_cascade_pass<In, ALIGNED, KG, DMA>), dim3(q.f.grid), dim3(256 * KG), lds, st, q);
    return hipGetLastError();
}

// Layers first .. first + n - 1 (all cascade layers, first >= 1) in one resident launch; see k_cascade_pass.
// Needs whole, aligned 128-byte row chunks in every layer (the direct-to-LDS form, whose LDS footprint keeps the grid
// to one workgroup per CU); the caller falls back to one launch per layer otherwise.
bool pass_eligible(const void* const* X_layers, int L, int T, int d, long long ld, int dtype, unsigned flags) {
    if (!(flags & ADA_FLAG_RESIDENT_PASS) || (flags & ADA_FLAG_TWO_PASS) || T > FUSED_MAX_T || L < 2) return false;
    if (dev_switch("ADA_NO_DMA") || kgroups_override() == 1) return false;
    const int epc = dtype == ADA_BF16 ? 64 : 32;
    if (d % epc != 0 || ld % (epc / 8) != 0) return false;
    for (int l = 0; l < L; ++l)
        if ((uintptr_t)X_layers[l] % 16 != 0) return false;
    return true;
}

int run_cascade_pass(const void* const* X_layers, int first, int n, int T, int d, long long ld, int dtype, float tau,
                     int32_t* idx_all, int32_t* counts_all, uint64_t* gram_ops_all, int32_t* adds_all,
                     int32_t* removes_all, void* ws, hipStream_t st, unsigned flags) {
    const Workspace w = carve(ws, T);
    PassParams pp;
    pp.f = {nullptr, ld, T, d, nullptr, nullptr, T, threshold_of(tau), (flags & ADA_FLAG_CROSS_EARLIER_ONLY) ? 1 : 0,
            w.hits, hit_words(T), nullptr, w.meta + META_TICKET, nullptr, nullptr, nullptr, nullptr, nullptr,
            0, nullptr, nullptr, nullptr, 0, cascade_tile_pick()};
    pp.f.first = T % 4 == 0 ? w.first : nullptr;              // (two K-groups: T <= 16384 fits)
    // rows of idx_all that share a 128-byte line with their neighbour could be cached half-written
    pp.f.coherent_list = ((uintptr_t)idx_all % 128 != 0 || T % 32 != 0) ? 1 : 0;
    for (int i = 0; i < n; ++i) pp.X[i] = X_layers[first + i];
    for (int i = n; i < PASS_MAX_LAYERS; ++i) pp.X[i] = nullptr;
    pp.n = n;
    const size_t row0 = (size_t)(first - 1);
    pp.idx_row0 = idx_all + row0 * (size_t)T;
    pp.counts_row0 = counts_all + row0 * 4;
    pp.gram_ops_row0 = reinterpret_cast<unsigned long long*>(gram_ops_all) + row0;
    pp.adds_row0 = adds_all ? adds_all + row0 * (size_t)T : nullptr;
    pp.removes_row0 = removes_all ? removes_all + row0 * (size_t)T : nullptr;
    pp.epoch = w.meta + META_EPOCH;
    pp.spin_limit = 1 << 20;                                 // about a second of polling
    if (const char* e = dev_switch("ADA_SPIN_LIMIT")) { const int v = atoi(e); if (v >= 1) pp.spin_limit = v; }
    // a layer that is never finished (a workgroup gave up waiting) keeps this status
    hipLaunchKernelGGL(k_fill_status, dim3((n * 4 + 255) / 256), dim3(256), 0, st, pp.counts_row0 + 4, n, (int)ADA_ERR_DEVICE);
    if (hipGetLastError() != hipSuccess) return ADA_ERR_DEVICE;
    const hipError_t e = dtype == ADA_BF16 ? launch_pass<uint16_t, true, 2, true>(pp, st)
                                           : launch_pass<float, true, 2, true>(pp, st);
    return e == hipSuccess ? ADA_OK : ADA_ERR_DEVICE;
}

// Algorithm 1 in separate launches (norms + lists, r x r Gram, cross-Gram against the valid representatives, update):
// gamma holds the exact gamma^cross of step 8.  Arguments checked by the caller; adds / removes / gram_ops / gamma may be NULL.
int run_cascade(const void* X, int T, int d, long long ld, int dtype, float tau, const int32_t* prev_idx, int r,
                const int32_t* r_dev, int32_t* idx, int32_t* adds, int32_t* removes, int32_t* counts,
                uint64_t* gram_ops, float* gamma, void* ws, hipStream_t st, unsigned flags) {
    if (!(flags & ADA_FLAG_TWO_PASS) && T <= FUSED_MAX_T)
        return run_cascade_fused(X, T, d, ld, dtype, tau, prev_idx, r, r_dev, idx, adds, removes, counts, gram_ops,
                                 gamma, ws, st, flags);
    const Workspace w = carve(ws, T);
    float* g = gamma ? gamma : w.gamma;
    const float thr = threshold_of(tau);
    const PrepParams prep = {prev_idx, r_dev, r, 1};
    const int nS_up = r;                         // inherited representatives (upper bound when r_dev is given)
    const int nT_up = r_dev ? T - 1 : T - r;     // all other tokens
    GramParams rep = {X, ld, T, d, prev_idx, w.nonrep_idx, w.meta, w.inv_norm, g, thr, MODE_REP, 1};
    GramParams cross = rep;
    cross.mode = MODE_CROSS;
    cross.order_mask = (flags & ADA_FLAG_CROSS_EARLIER_ONLY) ? 1 : 0;
    hipError_t e = dispatch(dtype, X, ld, d, [&](auto v) {
        using V = decltype(v);
        // step 1 (norms) + steps 2, 6 (index lists)
        hipError_t e1 = launch_norm_prep<typename V::In, V::aligned>(X, ld, T, d, g, w, prep, st);
        if (e1 != hipSuccess) return e1;
        // steps 3-5: r x r Gram among the inherited rows, strict lower triangle in token order
        e1 = launch_gram_any<typename V::In, V::aligned>(rep, nS_up, nS_up, r_dev == nullptr, st);
        if (e1 != hipSuccess || nT_up < 1) return e1;
        // steps 6-9: every other token against the valid representatives
        return launch_gram_any<typename V::In, V::aligned>(cross, nS_up, nT_up, r_dev == nullptr, st);
    });
    if (e != hipSuccess) return ADA_ERR_DEVICE;
    // step 10 and the bookkeeping of eq. (6) / eq. (8)
    const UpdateParams u = {g, w.is_rep, w.meta, T, thr, nullptr, idx, adds, removes, counts,
                            reinterpret_cast<unsigned long long*>(gram_ops)};
    return launch_update(u, st);
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// C ABI

extern "C" {

const char* ada_status_string(int status) {
    switch (status) {
        case ADA_OK: return "ADA_OK";
        case ADA_ERR_NULL: return "ADA_ERR_NULL: a required pointer is NULL";
        case ADA_ERR_SHAPE: return "ADA_ERR_SHAPE: bad T, d, ld, r or L";
        case ADA_ERR_TAU: return "ADA_ERR_TAU: tau must lie in (0,1)";
        case ADA_ERR_INDEX: return "ADA_ERR_INDEX: inherited indices must be strictly ascending token ids in [0,T)";
        case ADA_ERR_WORKSPACE: return "ADA_ERR_WORKSPACE: workspace too small or not 256-byte aligned";
        case ADA_ERR_DEVICE: return "ADA_ERR_DEVICE: a HIP call failed";
        case ADA_ERR_DTYPE: return "ADA_ERR_DTYPE: unknown element type";
        default: return "unknown ada_status";
    }
}

size_t ada_workspace_bytes(int T) { return (T < 1 || T > ADA_MAX_T) ? 0 : ws_bytes_for(T); }

int ada_workspace_init(void* ws, size_t ws_bytes, void* stream) {
    if (!ws) return ADA_ERR_NULL;
    if (((uintptr_t)ws % 256) != 0 || ws_bytes % 4 != 0) return ADA_ERR_WORKSPACE;
    return fill_u32(ws, ws_bytes / 4, 0u, (hipStream_t)stream) == hipSuccess ? ADA_OK : ADA_ERR_DEVICE;
}

int ada_select_full(const void* X, int T, int d, int64_t ld, int dtype, float tau, uint8_t* mask, int32_t* idx,
                    int32_t* count, float* gamma, void* ws, size_t ws_bytes, void* stream, unsigned flags) {
    if (!mask || !count) return ADA_ERR_NULL;
    if (int e = check_common(X, T, d, ld, dtype, tau, ws, ws_bytes)) return e;
    const bool greedy = (flags & ADA_FLAG_GREEDY_COVER) != 0;
    if (greedy && T > FUSED_MAX_T) return ADA_ERR_SHAPE;     // the pair bits live in the workspace's hit table
    return run_full(X, T, d, ld, dtype, tau, mask, idx, count, nullptr, gamma, ws, (hipStream_t)stream, 1,
                    GroupOff{0, 0, 0, 0, 0}, greedy);
}

int ada_select_full_grouped(const ada_groups* groups, const void* X, int T, int d, int64_t ld, int dtype, float tau,
                            uint8_t* mask, int32_t* idx, int32_t* counts, void* ws, size_t ws_bytes, void* stream,
                            unsigned flags) {
    (void)flags;
    if (!groups || !idx || !counts) return ADA_ERR_NULL;
    if (T < 1 || T > ADA_MAX_T) return ADA_ERR_SHAPE;
    const int G = groups->G;
    if (G < 1 || G > ADA_MAX_BATCH) return ADA_ERR_SHAPE;
    if (G > 1 && (groups->x_gstride < d || groups->list_gstride < T || groups->counts_gstride < 4)) return ADA_ERR_SHAPE;
    const size_t one = ws_bytes_for(T);
    if (ws && ws_bytes / (size_t)G < one) return ADA_ERR_WORKSPACE;
    if (int e = check_common(X, T, d, ld, dtype, tau, ws, one)) return e;
    const long long esz = dtype == ADA_BF16 ? 2 : 4;
    const GroupOff go = {G > 1 ? (long long)groups->x_gstride * esz : 0, G > 1 ? (long long)one : 0, groups->list_gstride,
                         groups->counts_gstride, 0};
    return run_full(X, T, d, ld, dtype, tau, mask, idx, counts, nullptr, nullptr, ws, (hipStream_t)stream, G, go);
}

// pos_given: the positions of the tokens' representatives are already in the workspace's position array (left there
// by the assignment of the same workspace): the position pass and its validation are skipped.
static int attention_run(const void* Q, const void* K, const void* V, int T, int H, int d_h, int64_t ld, int dtype,
                         const int32_t* idx, int r, const int32_t* r_dev, const int32_t* assign, float* out,
                         int64_t ld_out, int32_t* info, void* ws, size_t ws_bytes, void* stream, unsigned flags,
                         bool pos_given) {
    if (!Q || !K || !V || !idx || !assign || !out || !info || !ws) return ADA_ERR_NULL;
    if (dtype != ADA_F32 && dtype != ADA_BF16) return ADA_ERR_DTYPE;
    if (T < 1 || T > ADA_MAX_T || H < 1 || H > 65535 || r < 1 || r > T) return ADA_ERR_SHAPE;
    const bool dh_ok = dtype == ADA_BF16 ? (d_h == 64 || d_h == 128 || d_h == 256) : (d_h == 64 || d_h == 128);
    const int64_t D = (int64_t)H * d_h;
    const int esz = dtype == ADA_BF16 ? 2 : 4;
    if (!dh_ok || ld < D || ld_out < D || (ld * esz) % 16 != 0) return ADA_ERR_SHAPE;
    if ((uintptr_t)Q % 16 || (uintptr_t)K % 16 || (uintptr_t)V % 16) return ADA_ERR_SHAPE;
    if (ws_bytes < ws_bytes_for(T) || ((uintptr_t)ws % 256) != 0) return ADA_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const Workspace w = carve(ws, T);
    // positions and validation; its workgroups' status words go to the (otherwise unused) row-maximum array
    const int nerr = pos_given ? 0 : (T + 255) / 256;      // (r <= T)
    int32_t* err = reinterpret_cast<int32_t*>(w.gamma);
    if (!pos_given) {
        hipLaunchKernelGGL(k_attn_pos, dim3(nerr), dim3(256), 0, st, idx, r_dev, r, assign, T, w.nonrep_idx, err);
        if (hipGetLastError() != hipSuccess) return ADA_ERR_DEVICE;
    }
    const AttnParams p = {Q, K, V, ld, T, H, idx, r_dev, r, w.nonrep_idx, out, ld_out,
                          (float)(1.0 / sqrt((double)d_h)), (flags & ADA_FLAG_ATTN_CAUSAL) ? 1 : 0, info, err, nerr};
    hipError_t e;
    if (dtype == ADA_BF16)
        e = d_h == 64 ? launch_attn<uint16_t, 64>(p, st) : d_h == 128 ? launch_attn<uint16_t, 128>(p, st)
                                                                      : launch_attn<uint16_t, 256>(p, st);
    else
        e = d_h == 64 ? launch_attn<float, 64>(p, st) : launch_attn<float, 128>(p, st);
    return e == hipSuccess ? ADA_OK : ADA_ERR_DEVICE;
}

int ada_attention_compressed(const void* Q, const void* K, const void* V, int T, int H, int d_h, int64_t ld, int dtype,
                             const int32_t* idx, int r, const int32_t* r_dev, const int32_t* assign, float* out,
                             int64_t ld_out, int32_t* info, void* ws, size_t ws_bytes, void* stream, unsigned flags) {
    return attention_run(Q, K, V, T, H, d_h, ld, dtype, idx, r, r_dev, assign, out, ld_out, info, ws, ws_bytes, stream,
                         flags, false);
}

int ada_assign_nearest(const void* X, int T, int d, int64_t ld, int dtype, const int32_t* idx, int r,
                       const int32_t* r_dev, int32_t* assign, float* corr, int32_t* info, void* ws, size_t ws_bytes,
                       void* stream, unsigned flags) {
    (void)flags;
    if (!idx || !assign || !info) return ADA_ERR_NULL;
    if (int e = check_common(X, T, d, ld, dtype, 0.5f, ws, ws_bytes)) return e;
    if (r < 1 || r > T) return ADA_ERR_SHAPE;
    return run_assign(X, T, d, ld, dtype, idx, r, r_dev, assign, corr, info, ws, (hipStream_t)stream);
}

int ada_cascade_step(const void* X, int T, int d, int64_t ld, int dtype, float tau, const int32_t* prev_idx, int r,
                     const int32_t* r_dev, int32_t* idx, int32_t* adds, int32_t* removes, int32_t* counts,
                     uint64_t* gram_ops, float* gamma, void* ws, size_t ws_bytes, void* stream, unsigned flags) {
    if (!prev_idx || !idx || !adds || !removes || !counts) return ADA_ERR_NULL;
    if (int e = check_common(X, T, d, ld, dtype, tau, ws, ws_bytes)) return e;
    if (r < 1 || r > T) return ADA_ERR_SHAPE;
    return run_cascade(X, T, d, ld, dtype, tau, prev_idx, r, r_dev, idx, adds, removes, counts, gram_ops, gamma, ws,
                       (hipStream_t)stream, flags);
}

// ------------------------------------------------------------------------------------------------
// ada_cascade_step_static: the same step on a workspace that lives in this library's image, for callers that cannot
// allocate.  `scratch` is a host-side stand-in for the array; its device address is looked up once per device.
static __device__ __align__(256) unsigned char scratch[ws_bytes_for(ADA_STATIC_MAX_T)];

namespace {
constexpr int STATIC_MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[STATIC_MAX_DEVICES];          // per device: every GPU holds its own copy of the array

// The array's address on the current device (looked up on the first call there), or NULL.
void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= STATIC_MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

int ada_cascade_step_static(const void* X, int T, int d, int64_t ld, int dtype, float tau, const int32_t* prev_idx, int r,
                            const int32_t* r_dev, int32_t* idx, int32_t* adds, int32_t* removes, int32_t* counts,
                            uint64_t* gram_ops, float* gamma, void* stream, unsigned flags) {
    if (!prev_idx || !idx || !adds || !removes || !counts) return ADA_ERR_NULL;
    if (T > ADA_STATIC_MAX_T) return ADA_ERR_SHAPE;            // beyond what the array holds
    void* ws = static_scratch();
    if (!ws) return ADA_ERR_DEVICE;
    const size_t ws_bytes = ws_bytes_for(ADA_STATIC_MAX_T);
    if (int e = check_common(X, T, d, ld, dtype, tau, ws, ws_bytes)) return e;
    if (r < 1 || r > T) return ADA_ERR_SHAPE;
    // The counters a step relies on being zero (tickets, queue, hand-over word) are cleared by a fill kernel, so the
    // array is good whatever an earlier call left behind; everything else a step reads it writes first.
    const Workspace w = carve(ws, T);
    if (fill_u32(w.meta, META_BYTES / 4, 0u, (hipStream_t)stream) != hipSuccess) return ADA_ERR_DEVICE;
    if (fill_u32(w.best, (size_t)T * 2, 0u, (hipStream_t)stream) != hipSuccess ||                       // arg-max keys
        fill_u32(w.first, (size_t)T, 0u, (hipStream_t)stream) != hipSuccess) return ADA_ERR_DEVICE;         // first-hit records
    return run_cascade(X, T, d, ld, dtype, tau, prev_idx, r, r_dev, idx, adds, removes, counts, gram_ops, gamma, ws,
                       (hipStream_t)stream, flags);
}

namespace {
int check_groups(const ada_groups* g, int T, int d) {
    if (!g) return ADA_ERR_NULL;
    if (g->G < 1 || g->G > ADA_MAX_BATCH) return ADA_ERR_SHAPE;
    if (g->G > 1 && (g->x_gstride < d || g->list_gstride < T || g->counts_gstride < 4 || g->ops_gstride < 1)) return ADA_ERR_SHAPE;
    return ADA_OK;
}

// one cascade step for every group: one launch when the one-launch form applies, else group by group
int run_cascade_grouped(const ada_groups& g, const void* X, int T, int d, long long ld, int dtype, float tau,
                        const int32_t* prev_idx, int r, const int32_t* r_dev, int32_t* idx, int32_t* adds,
                        int32_t* removes, int32_t* counts, uint64_t* gram_ops, void* ws, hipStream_t st, unsigned flags) {
    if (g.G == 1)
        return run_cascade(X, T, d, ld, dtype, tau, prev_idx, r, r_dev, idx, adds, removes, counts, gram_ops, nullptr, ws,
                           st, flags);
    if (!(flags & ADA_FLAG_TWO_PASS) && T <= FUSED_MAX_T)
        return run_cascade_fused(X, T, d, ld, dtype, tau, prev_idx, r, r_dev, idx, adds, removes, counts, gram_ops, nullptr,
                                 ws, st, flags, &g);
    const size_t esz = dtype == ADA_BF16 ? 2 : 4, one = ws_bytes_for(T);
    for (int i = 0; i < g.G; ++i) {
        const long long lo = (long long)i * g.list_gstride, co = (long long)i * g.counts_gstride;
        const int e = run_cascade((const char*)X + (size_t)i * (size_t)g.x_gstride * esz, T, d, ld, dtype, tau, prev_idx + lo,
                                  r, r_dev ? r_dev + co : nullptr, idx + lo, adds ? adds + lo : nullptr,
                                  removes ? removes + lo : nullptr, counts + co,
                                  gram_ops ? gram_ops + (long long)i * g.ops_gstride : nullptr, nullptr,
                                  (char*)ws + (size_t)i * one, st, flags);
        if (e != ADA_OK) return e;
    }
    return ADA_OK;
}
}  // namespace

int ada_cascade_step_grouped(const ada_groups* groups, const void* X, int T, int d, int64_t ld, int dtype, float tau,
                             const int32_t* prev_idx, int r, const int32_t* r_dev, int32_t* idx, int32_t* adds,
                             int32_t* removes, int32_t* counts, uint64_t* gram_ops, void* ws, size_t ws_bytes, void* stream,
                             unsigned flags) {
    if (!prev_idx || !idx || !adds || !removes || !counts) return ADA_ERR_NULL;
    if (T < 1 || T > ADA_MAX_T) return ADA_ERR_SHAPE;
    if (int e = check_groups(groups, T, d)) return e;
    const size_t one = ws_bytes_for(T);
    if (ws && ws_bytes / (size_t)groups->G < one) return ADA_ERR_WORKSPACE;
    if (int e = check_common(X, T, d, ld, dtype, tau, ws, one)) return e;
    if (r < 1 || r > T) return ADA_ERR_SHAPE;
    return run_cascade_grouped(*groups, X, T, d, ld, dtype, tau, prev_idx, r, r_dev, idx, adds, removes, counts, gram_ops,
                               ws, (hipStream_t)stream, flags);
}

int ada_cascade_layers_grouped(const ada_groups* groups, const void* const* X_layers, int L, int T, int d, int64_t ld,
                               int dtype, float tau, int32_t* idx_all, int32_t* counts_all, uint64_t* gram_ops_all,
                               int32_t* adds_all, int32_t* removes_all, void* ws, size_t ws_bytes, void* stream,
                               unsigned flags) {
    if (!groups || !X_layers || !idx_all || !counts_all || !gram_ops_all) return ADA_ERR_NULL;
    if (L < 1 || T < 1 || T > ADA_MAX_T) return ADA_ERR_SHAPE;
    if (groups->G < 1 || groups->G > ADA_MAX_BATCH || (groups->G > 1 && groups->x_gstride < d)) return ADA_ERR_SHAPE;
    for (int l = 0; l < L; ++l)
        if (!X_layers[l]) return ADA_ERR_NULL;
    const size_t one = ws_bytes_for(T);
    if (ws && ws_bytes / (size_t)groups->G < one) return ADA_ERR_WORKSPACE;
    if (int e = check_common(X_layers[0], T, d, ld, dtype, tau, ws, one)) return e;
    hipStream_t st = (hipStream_t)stream;
    // the outputs are [G][L][...] blocks, so a group's rows are L rows apart
    const ada_groups g = {groups->G, groups->x_gstride, (int64_t)L * T, (int64_t)L * 4, (int64_t)L};
    const size_t esz = dtype == ADA_BF16 ? 2 : 4;
    // layer 0: every group's full selection in the same three launches
    {
        const GroupOff go = {g.G > 1 ? (long long)g.x_gstride * (long long)esz : 0, g.G > 1 ? (long long)one : 0,
                             g.list_gstride, g.counts_gstride, g.ops_gstride};
        const int e = run_full(X_layers[0], T, d, ld, dtype, tau, nullptr, idx_all, counts_all, gram_ops_all, nullptr, ws, st,
                               g.G, go);
        if (e != ADA_OK) return e;
    }
    // layers >= 1: one launch serves all groups
    for (int l = 1; l < L; ++l) {
        const size_t o = (size_t)l * (size_t)T;
        const int e = run_cascade_grouped(g, X_layers[l], T, d, ld, dtype, tau, idx_all + o - T, T,
                                          counts_all + (size_t)(l - 1) * 4, idx_all + o, adds_all ? adds_all + o : nullptr,
                                          removes_all ? removes_all + o : nullptr, counts_all + (size_t)l * 4,
                                          gram_ops_all + l, ws, st, flags & ~ADA_FLAG_RESIDENT_PASS);
        if (e != ADA_OK) return e;
    }
    return ADA_OK;
}

int ada_cascade_layers(const void* const* X_layers, int L, int T, int d, int64_t ld, int dtype, float tau,
                       int32_t* idx_all, int32_t* counts_all, uint64_t* gram_ops_all, int32_t* adds_all,
                       int32_t* removes_all, void* ws, size_t ws_bytes, void* stream, unsigned flags) {
    if (!X_layers || !idx_all || !counts_all || !gram_ops_all) return ADA_ERR_NULL;
    if (L < 1) return ADA_ERR_SHAPE;
    for (int l = 0; l < L; ++l)
        if (!X_layers[l]) return ADA_ERR_NULL;
    if (int e = check_common(X_layers[0], T, d, ld, dtype, tau, ws, ws_bytes)) return e;
    hipStream_t st = (hipStream_t)stream;
    // layer 0: the full T x T selection; layers >= 1 inherit the previous layer's set on the device (Section 4.1)
    int e = run_full(X_layers[0], T, d, ld, dtype, tau, nullptr, idx_all, counts_all, gram_ops_all, nullptr, ws, st);
    if (e == ADA_OK && pass_eligible(X_layers, L, T, d, ld, dtype, flags)) {
        for (int first = 1; first < L && e == ADA_OK; first += PASS_MAX_LAYERS) {
            const int n = L - first < PASS_MAX_LAYERS ? L - first : PASS_MAX_LAYERS;
            e = run_cascade_pass(X_layers, first, n, T, d, ld, dtype, tau, idx_all, counts_all, gram_ops_all, adds_all,
                                 removes_all, ws, st, flags);
        }
        return e;
    }
    for (int l = 1; l < L && e == ADA_OK; ++l) {
        const size_t o = (size_t)l * (size_t)T;
        e = run_cascade(X_layers[l], T, d, ld, dtype, tau, idx_all + o - T, T, counts_all + (size_t)(l - 1) * 4,
                        idx_all + o, adds_all ? adds_all + o : nullptr, removes_all ? removes_all + o : nullptr,
                        counts_all + (size_t)l * 4, gram_ops_all + l, nullptr, ws, st, flags);
    }
    return e;
}

int ada_cascade_layers_batched(const void* const* X_layers, int B, int L, int T, int d, int64_t ld, int dtype, float tau,
                               int32_t* idx_all, int32_t* counts_all, uint64_t* gram_ops_all, int32_t* adds_all,
                               int32_t* removes_all, void* ws, size_t ws_bytes, void* const* streams, void* stream,
                               unsigned flags) {
    if (!X_layers || !idx_all || !counts_all || !gram_ops_all) return ADA_ERR_NULL;
    if (B < 1 || B > ADA_MAX_BATCH || L < 1) return ADA_ERR_SHAPE;
    for (long long i = 0; i < (long long)B * L; ++i)
        if (!X_layers[i]) return ADA_ERR_NULL;
    if (T < 1 || T > ADA_MAX_T) return ADA_ERR_SHAPE;
    const size_t one = ada_workspace_bytes(T);
    if (!ws) return ADA_ERR_NULL;
    if (ws_bytes / (size_t)B < one) return ADA_ERR_WORKSPACE;
    for (int b = 0; b < B; ++b)
        if (int e = check_common(X_layers[(size_t)b * L], T, d, ld, dtype, tau, (char*)ws + (size_t)b * one, one)) return e;
    hipStream_t main = (hipStream_t)stream;
    // fork: every chain starts after what the caller has enqueued on `stream` so far
    hipEvent_t fork = nullptr;
    if (streams) {
        if (hipEventCreateWithFlags(&fork, hipEventDisableTiming) != hipSuccess) return ADA_ERR_DEVICE;
        bool ok = hipEventRecord(fork, main) == hipSuccess;
        for (int b = 0; b < B && ok; ++b)
            if ((hipStream_t)streams[b] != main) ok = hipStreamWaitEvent((hipStream_t)streams[b], fork, 0) == hipSuccess;
        (void)hipEventDestroy(fork);                      // released by the runtime once it has completed
        if (!ok) return ADA_ERR_DEVICE;
    }
    // layer-major issue order, so that the sequences' launches interleave from the first layer on; the resident pass
    // needs the whole device for one sequence and is not used here
    const unsigned fl = flags & ~ADA_FLAG_RESIDENT_PASS;
    int rc = ADA_OK;
    for (int l = 0; l < L && rc == ADA_OK; ++l) {
        for (int b = 0; b < B && rc == ADA_OK; ++b) {
            hipStream_t st = streams ? (hipStream_t)streams[b] : main;
            const size_t row = (size_t)b * L + l, o = row * (size_t)T;
            void* wsb = (char*)ws + (size_t)b * one;
            if (l == 0)
                rc = run_full(X_layers[row], T, d, ld, dtype, tau, nullptr, idx_all + o, counts_all + row * 4,
                              gram_ops_all + row, nullptr, wsb, st);
            else
                rc = run_cascade(X_layers[row], T, d, ld, dtype, tau, idx_all + o - T, T, counts_all + (row - 1) * 4,
                                 idx_all + o, adds_all ? adds_all + o : nullptr, removes_all ? removes_all + o : nullptr,
                                 counts_all + row * 4, gram_ops_all + row, nullptr, wsb, st, fl);
        }
    }
    // join: what the caller enqueues on `stream` next sees every chain's results (also after an error part-way)
    if (streams) {
        for (int b = 0; b < B; ++b) {
            hipStream_t st = (hipStream_t)streams[b];
            if (st == main) continue;
            hipEvent_t done = nullptr;
            if (hipEventCreateWithFlags(&done, hipEventDisableTiming) != hipSuccess) return ADA_ERR_DEVICE;
            const bool ok = hipEventRecord(done, st) == hipSuccess && hipStreamWaitEvent(main, done, 0) == hipSuccess;
            (void)hipEventDestroy(done);
            if (!ok) return ADA_ERR_DEVICE;
        }
    }
    return rc;
}

int ada_pipeline_layers(const void* const* X_layers, const void* const* Q_layers, const void* const* K_layers,
                        const void* const* V_layers, int L, int T, int H, int d_h, int64_t ld, int dtype, float tau,
                        int32_t* idx_all, int32_t* counts_all, uint64_t* gram_ops_all, int32_t* assign_all,
                        int32_t* info_all, float* const* out_layers, int64_t ld_out, void* ws, size_t ws_bytes,
                        void* stream_sel, void* stream_attn, void* stream, unsigned flags) {
    if (!X_layers || !Q_layers || !K_layers || !V_layers || !out_layers) return ADA_ERR_NULL;
    if (!idx_all || !counts_all || !gram_ops_all || !assign_all || !info_all || !ws) return ADA_ERR_NULL;
    if (L < 1 || H < 1 || H > 65535 || d_h < 1 || d_h > (1 << 20)) return ADA_ERR_SHAPE;
    const int64_t D64 = (int64_t)H * d_h;
    if (D64 > (1 << 24)) return ADA_ERR_SHAPE;
    const int d = (int)D64;
    for (int l = 0; l < L; ++l)
        if (!X_layers[l] || !Q_layers[l] || !K_layers[l] || !V_layers[l] || !out_layers[l]) return ADA_ERR_NULL;
    if (T < 1 || T > ADA_MAX_T) return ADA_ERR_SHAPE;
    const size_t one = ws_bytes_for(T);
    if (ws_bytes / 2 < one) return ADA_ERR_WORKSPACE;
    if (int e = check_common(X_layers[0], T, d, ld, dtype, tau, ws, one)) return e;
    void* ws_attn = (char*)ws + one;
    hipStream_t main = (hipStream_t)stream;
    hipStream_t ss = stream_sel ? (hipStream_t)stream_sel : main, sa = stream_attn ? (hipStream_t)stream_attn : main;
    // the attention-side calls check their own arguments; run those checks before anything is enqueued
    if (ld_out < D64 || ((int64_t)ld * (dtype == ADA_BF16 ? 2 : 4)) % 16 != 0) return ADA_ERR_SHAPE;
    const bool dh_ok = dtype == ADA_BF16 ? (d_h == 64 || d_h == 128 || d_h == 256) : (d_h == 64 || d_h == 128);
    if (!dh_ok) return ADA_ERR_SHAPE;
    for (int l = 0; l < L; ++l)
        if ((uintptr_t)Q_layers[l] % 16 || (uintptr_t)K_layers[l] % 16 || (uintptr_t)V_layers[l] % 16) return ADA_ERR_SHAPE;

    auto fork = [&](hipStream_t from, hipStream_t to) -> bool {   // `to` continues after what `from` holds now
        if (from == to) return true;
        hipEvent_t ev = nullptr;
        if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) return false;
        const bool ok = hipEventRecord(ev, from) == hipSuccess && hipStreamWaitEvent(to, ev, 0) == hipSuccess;
        (void)hipEventDestroy(ev);                               // released by the runtime once it has completed
        return ok;
    };
    if (!fork(main, ss) || !fork(main, sa)) return ADA_ERR_DEVICE;
    int rc = ADA_OK;
    for (int l = 0; l < L && rc == ADA_OK; ++l) {
        const size_t o = (size_t)l * (size_t)T;
        // selection of layer l (Section 4.1): needs only the previous layer's set
        if (l == 0)
            rc = run_full(X_layers[0], T, d, ld, dtype, tau, nullptr, idx_all, counts_all, gram_ops_all, nullptr, ws, ss);
        else
            rc = run_cascade(X_layers[l], T, d, ld, dtype, tau, idx_all + o - T, T, counts_all + (size_t)(l - 1) * 4,
                             idx_all + o, nullptr, nullptr, counts_all + (size_t)l * 4, gram_ops_all + l, nullptr, ws, ss,
                             flags & (ADA_FLAG_CROSS_EARLIER_ONLY | ADA_FLAG_TWO_PASS));
        if (rc != ADA_OK) break;
        // layer l's assignment and attention wait for that set only; the selection stream goes on to layer l + 1
        if (!fork(ss, sa)) { rc = ADA_ERR_DEVICE; break; }
        // the assignment also leaves every token's position in R where the attention looks for it: no position pass
        rc = run_assign(X_layers[l], T, d, ld, dtype, idx_all + o, T, counts_all + (size_t)l * 4, assign_all + o, nullptr,
                        info_all + (size_t)l * 8, ws_attn, sa, carve(ws_attn, T).nonrep_idx);
        if (rc != ADA_OK) break;
        rc = attention_run(Q_layers[l], K_layers[l], V_layers[l], T, H, d_h, ld, dtype, idx_all + o, T,
                           counts_all + (size_t)l * 4, assign_all + o, out_layers[l], ld_out,
                           info_all + (size_t)l * 8 + 4, ws_attn, one, sa, flags & ADA_FLAG_ATTN_CAUSAL, true);
    }
    // join: work enqueued on `stream` after the call sees everything (also after an error part-way)
    if (!fork(ss, main) || !fork(sa, main)) return ADA_ERR_DEVICE;
    return rc;
}

namespace {
__global__ void k_tau_init(double* tau_all, float* thr_all, double tau0, float thr0, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) { tau_all[i] = tau0; thr_all[i] = thr0; }
}
}  // namespace

int ada_cascade_layers_adaptive(const void* const* X_layers, int L, int T, int d, int64_t ld, int dtype, float tau0,
                                const ada_tau_control* ctl, int32_t* idx_all, int32_t* counts_all,
                                uint64_t* gram_ops_all, int32_t* adds_all, int32_t* removes_all, double* tau_all,
                                float* thr_all, void* ws, size_t ws_bytes, void* stream, unsigned flags) {
    if (!X_layers || !ctl || !idx_all || !counts_all || !gram_ops_all || !tau_all || !thr_all) return ADA_ERR_NULL;
    if (L < 1) return ADA_ERR_SHAPE;
    for (int l = 0; l < L; ++l)
        if (!X_layers[l]) return ADA_ERR_NULL;
    if (int e = check_common(X_layers[0], T, d, ld, dtype, tau0, ws, ws_bytes)) return e;
    if (!(ctl->tau_min > 0.0 && ctl->tau_min <= ctl->tau_max && ctl->tau_max < 1.0)) return ADA_ERR_TAU;
    if (!((double)tau0 >= ctl->tau_min && (double)tau0 <= ctl->tau_max)) return ADA_ERR_TAU;
    if (!(ctl->kappa == ctl->kappa) || !(ctl->eta_target == ctl->eta_target)) return ADA_ERR_TAU;     // NaN
    if (T > FUSED_MAX_T || (flags & ADA_FLAG_TWO_PASS)) return ADA_ERR_SHAPE;   // the one-launch step carries the threshold
    hipStream_t st = (hipStream_t)stream;
    // every layer's tau starts as tau0 (layers 0 and 1 use it as it is: no turnover is known before the first step)
    hipLaunchKernelGGL(k_tau_init, dim3((L + 255) / 256), dim3(256), 0, st, tau_all, thr_all, (double)tau0,
                       threshold_of(tau0), L);
    if (hipGetLastError() != hipSuccess) return ADA_ERR_DEVICE;
    int e = run_full(X_layers[0], T, d, ld, dtype, tau0, nullptr, idx_all, counts_all, gram_ops_all, nullptr, ws, st);
    for (int l = 1; l < L && e == ADA_OK; ++l) {
        const size_t o = (size_t)l * (size_t)T;
        const bool last = l + 1 == L;
        e = run_cascade_fused(X_layers[l], T, d, ld, dtype, tau0, idx_all + o - T, T, counts_all + (size_t)(l - 1) * 4,
                              idx_all + o, adds_all ? adds_all + o : nullptr, removes_all ? removes_all + o : nullptr,
                              counts_all + (size_t)l * 4, gram_ops_all + l, nullptr, ws, st,
                              flags & ADA_FLAG_CROSS_EARLIER_ONLY, nullptr, ctl, tau_all + l, thr_all + l,
                              last ? nullptr : tau_all + l + 1, last ? nullptr : thr_all + l + 1);
    }
    return e;
}

int ada_plan_tile_shape(int r, int T, int d, int workgroups) {
    if (r < 1 || T < 1 || r > T || d < 1 || workgroups < 1) return -1;
    return cascade_tile_shape(r, T, d, workgroups, workgroups);
}

int ada_plan_full_units(int T, int d, int workgroups) {
    if (T < 1536 || T > ADA_MAX_T || d < 1 || d % DmaGeom::HC != 0 || workgroups < 8) return -1;
    const int G = workgroups / 8 * 8;
    if (T <= 4096 && d % SplitGeom::EPC == 0) return dma_makespan_norms(T, 2, G) < dma_makespan_norms(T, 0, G) ? 2 : 0;
    return dma_makespan(T, 1, G) < dma_makespan(T, 0, G) ? 1 : 0;
}

int ada_set_overlap(const uint8_t* mask_a, const uint8_t* mask_b, int T, int32_t* out, void* stream) {
    if (!mask_a || !mask_b || !out) return ADA_ERR_NULL;
    if (T < 1 || T > ADA_MAX_T) return ADA_ERR_SHAPE;
    hipLaunchKernelGGL(k_overlap, dim3(1), dim3(1024), 0, (hipStream_t)stream, mask_a, mask_b, T, out);
    return hipGetLastError() == hipSuccess ? ADA_OK : ADA_ERR_DEVICE;
}

int ada_profile_copy_probe(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src) return ADA_ERR_NULL;
    if (bytes % 16 != 0 || ((uintptr_t)dst % 16) != 0 || ((uintptr_t)src % 16) != 0) return ADA_ERR_SHAPE;
    if (bytes == 0) return ADA_OK;
    hipLaunchKernelGGL(k_copy_probe, dim3(4096), dim3(256), 0, (hipStream_t)stream, (u32x4*)dst, (const u32x4*)src,
                       bytes / 16);
    return hipGetLastError() == hipSuccess ? ADA_OK : ADA_ERR_DEVICE;
}

int ada_profile_mfma_probe(int workgroups, int iters, float* sink, void* stream) {
    if (!sink) return ADA_ERR_NULL;
    if (workgroups < 1 || iters < 1 || workgroups > (1 << 20) || iters > (1 << 20)) return ADA_ERR_SHAPE;
    ProfScope ps(ADA_K_MFMA_PROBE, (hipStream_t)stream);
    hipLaunchKernelGGL(k_mfma_probe, dim3(workgroups), dim3(256), 0, (hipStream_t)stream, sink, iters);
    return hipGetLastError() == hipSuccess ? ADA_OK : ADA_ERR_DEVICE;
}

int ada_profile_enable(int on) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof_on = on != 0;
    return ADA_OK;
}

int ada_profile_collect(double* ms_sum, int* launches) {
    if (!ms_sum || !launches) return ADA_ERR_NULL;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (int k = 0; k < ADA_K_COUNT; ++k) { ms_sum[k] = 0.0; launches[k] = 0; }
    int rc = ADA_OK;
    for (ProfRecord& r : g_prof) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) rc = ADA_ERR_DEVICE;
        else { ms_sum[r.cls] += (double)ms; launches[r.cls] += 1; }
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    g_prof.clear();
    return rc;
}

#ifdef ADA_PHASE_CLOCKS
int ada_debug_pass_clocks(unsigned long long* out) {   // development builds only
    return hipMemcpyFromSymbol(out, HIP_SYMBOL(g_pass_clk), sizeof(unsigned long long) * 512 * 8) == hipSuccess ? 0 : 6;
}
int ada_debug_phase_clocks(unsigned long long* out) {   // development builds only
    return hipMemcpyFromSymbol(out, HIP_SYMBOL(g_phase_clk), sizeof(unsigned long long) * 64) == hipSuccess ? 0 : 6;
}
#endif

int ada_cascade_report(int L, int T, const int32_t* counts_all, const uint64_t* gram_ops_all, double* jaccard,
                       double* turnover, double* savings) {
    if (!counts_all || !gram_ops_all) return ADA_ERR_NULL;
    if (L < 1 || T < 1) return ADA_ERR_SHAPE;
    double ops = 0.0;
    for (int l = 0; l < L; ++l) {
        ops += (double)gram_ops_all[l];
        double j = 0.0, eta = 0.0;
        if (l > 0) {
            const int r_prev = counts_all[(l - 1) * 4], n_add = counts_all[l * 4 + 1], n_rem = counts_all[l * 4 + 2];
            if (r_prev > 0) {
                j = (double)(r_prev - n_rem) / (double)(r_prev + n_add);   // eq. (3) on R^(l-1), R^(l)
                eta = (double)(n_add + n_rem) / (double)r_prev;            // eq. (8)
            }
        }
        if (jaccard) jaccard[l] = j;
        if (turnover) turnover[l] = eta;
    }
    if (savings) *savings = 1.0 - ops / ((double)L * (double)T * (double)T);   // Table 6
    return ADA_OK;
}

}  // extern "C"
