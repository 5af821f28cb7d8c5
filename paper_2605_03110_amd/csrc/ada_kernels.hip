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
#include <mutex>

#include "../../include/ada.h"

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

enum { MODE_FULL = 0, MODE_REP = 1, MODE_CROSS = 2 };
enum { META_R = 0, META_NONREP = 1, META_STATUS = 2, META_WORDS = 8 };

struct Workspace {
    float* inv_norm;     // [T]
    float* gamma;        // [T]
    int32_t* nonrep_idx; // [T]
    uint8_t* is_rep;     // [T]
    int32_t* meta;       // [META_WORDS]
};

__host__ __device__ inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

inline size_t ws_bytes_for(int T) {
    size_t t4 = align_up((size_t)T * 4, 256), t1 = align_up((size_t)T, 256);
    return t4 * 3 + t1 + 256;
}

inline Workspace carve(void* ws, int T) {
    char* p = (char*)ws;
    size_t t4 = align_up((size_t)T * 4, 256), t1 = align_up((size_t)T, 256);
    Workspace w;
    w.inv_norm = (float*)p; p += t4;
    w.gamma = (float*)p; p += t4;
    w.nonrep_idx = (int32_t*)p; p += t4;
    w.is_rep = (uint8_t*)p; p += t1;
    w.meta = (int32_t*)p;
    return w;
}

// ------------------------------------------------------------------------------------------------
// element access

template <typename In> __device__ inline float to_f32(In v);
template <> __device__ inline float to_f32<float>(float v) { return v; }
template <> __device__ inline float to_f32<uint16_t>(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

// One 16-byte piece of a row starting at element e0; elements at or beyond d read as zero.
template <typename In, bool ALIGNED>
__device__ inline u32x4 load_piece(const In* row, int e0, int d) {
    constexpr int EPP = 16 / (int)sizeof(In);
    u32x4 out = {0u, 0u, 0u, 0u};
    if (ALIGNED) {
        if (e0 < d) out = *reinterpret_cast<const u32x4*>(row + e0);
    } else {
        union { u32x4 v; In e[EPP]; } u;
        u.v = out;
#pragma unroll
        for (int i = 0; i < EPP; ++i)
            if (e0 + i < d) u.e[i] = row[e0 + i];
        out = u.v;
    }
    return out;
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

struct PrepParams {
    const int32_t* prev_idx;
    const int32_t* r_dev;
    int r_host;
    int enabled;
};

template <typename In, bool ALIGNED>
__global__ __launch_bounds__(256) void k_norm_prep(const In* __restrict__ X, long long ld, int T, int d,
                                                   float* __restrict__ inv_norm, float* __restrict__ gamma,
                                                   Workspace w, PrepParams prep, int n_norm_blocks) {
    constexpr int EPP = 16 / (int)sizeof(In);
    __shared__ int sh[32];
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
};

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

// LDS staging buffer: rows of 128 bytes = 8 pieces; piece c of row r sits at slot c ^ (r & 7) so that the
// 16-byte fragment reads of 8 consecutive rows touch all 32 banks.
__device__ inline int lds_off(int row, int piece) { return row * 128 + ((piece ^ (row & 7)) << 4); }

template <typename In, int B, bool ALIGNED>
__device__ inline void gram_tile(const GramParams& p, const int32_t* listS, const int32_t* listT, int s0, int t0,
                                 int nS, int nT, bool need_order, char* lds) {
    constexpr int EPP = 16 / (int)sizeof(In);
    constexpr int EPC = 8 * EPP;
    constexpr int ROWS = 2 * B;          // "against" rows first, then tested rows
    constexpr int LPT = ROWS / 32;       // pieces each thread moves per chunk
    constexpr int STAGE = ROWS * 128;
    constexpr int WB = B / 2;            // wave tile edge (2 x 2 waves)
    constexpr int NB = WB / 32;          // 32x32 MFMA blocks per wave per edge

    char* buf0 = lds;
    char* buf1 = lds + STAGE;
    int* s_tok = reinterpret_cast<int*>(lds + 2 * STAGE);
    int* t_tok = s_tok + B;
    float* s_scale = reinterpret_cast<float*>(t_tok + B);
    float* t_scale = s_scale + B;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int ws = wave >> 1, wt = wave & 1;
    const In* X = reinterpret_cast<const In*>(p.X);

    // per-row metadata of the tile
    for (int i = tid; i < ROWS; i += 256) {
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

    // the rows this thread stages
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
        const int lc = li < n ? li : n - 1;
        int tok = list ? list[lc] : lc;
        tok = min(max(tok, 0), p.T - 1);
        rowp[j] = X + (size_t)tok * (size_t)p.ld;
        woff[j] = lds_off(row, pc);
    }

    const int nk = (p.d + EPC - 1) / EPC;
    u32x4 pre[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) pre[j] = load_piece<In, ALIGNED>(rowp[j], pc * EPP, p.d);
#pragma unroll
    for (int j = 0; j < LPT; ++j) *reinterpret_cast<u32x4*>(buf0 + woff[j]) = pre[j];
    __syncthreads();

    f32x16 acc[NB][NB];
#pragma unroll
    for (int a = 0; a < NB; ++a)
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;

    for (int kc = 0; kc < nk; ++kc) {
        const bool more = kc + 1 < nk;
        if (more) {
#pragma unroll
            for (int j = 0; j < LPT; ++j) pre[j] = load_piece<In, ALIGNED>(rowp[j], (kc + 1) * EPC + pc * EPP, p.d);
        }
        const char* cur = (kc & 1) ? buf1 : buf0;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int piece = 2 * ks + half;
            u32x4 fa[NB], fb[NB];
#pragma unroll
            for (int a = 0; a < NB; ++a) fa[a] = *reinterpret_cast<const u32x4*>(cur + lds_off(ws * WB + a * 32 + l32, piece));
#pragma unroll
            for (int b = 0; b < NB; ++b) fb[b] = *reinterpret_cast<const u32x4*>(cur + lds_off(B + wt * WB + b * 32 + l32, piece));
#pragma unroll
            for (int a = 0; a < NB; ++a)
#pragma unroll
                for (int b = 0; b < NB; ++b) Mfma<In>::run(acc[a][b], fa[a], fb[b]);
        }
        if (more) {
            char* nxt = (kc & 1) ? buf0 : buf1;
#pragma unroll
            for (int j = 0; j < LPT; ++j) *reinterpret_cast<u32x4*>(nxt + woff[j]) = pre[j];
        }
        __syncthreads();
    }

    // epilogue: lane holds column n = l32 (tested token) and rows m = (i & 3) + 4 * half + 8 * (i >> 2)
    uint32_t* gamma_bits = reinterpret_cast<uint32_t*>(p.gamma);
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int nl = wt * WB + b * 32 + l32;
        const int ttok = t_tok[nl];
        float m = 0.f;
#pragma unroll
        for (int a = 0; a < NB; ++a) {
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const int sl = ws * WB + a * 32 + (i & 3) + 4 * half + 8 * (i >> 2);
                float v = fabsf(acc[a][b][i]) * s_scale[sl];
                if (need_order && !(s_tok[sl] < ttok)) v = 0.f;
                m = fmaxf(m, v);
            }
        }
        m *= t_scale[nl];
        m = fmaxf(m, __shfl_xor(m, 32, 64));
        if (half == 0 && ttok >= 0 && m > 0.f) atomicMax(gamma_bits + ttok, __float_as_uint(m));
    }
}

template <typename In, int B, bool ALIGNED>
__global__ __launch_bounds__(256) void k_gram(GramParams p) {
    extern __shared__ __align__(16) char lds[];
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
    for (long long tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
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
};

__global__ __launch_bounds__(1024) void k_update(UpdateParams u) {
    __shared__ int sh[3][32];
    const int tid = threadIdx.x;
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

// ------------------------------------------------------------------------------------------------
// host side

template <int B> constexpr int gram_lds_bytes() { return 2 * (2 * B) * 128 + 4 * B * 4; }

template <typename In, int B, bool ALIGNED>
hipError_t launch_gram(const GramParams& p, long long tiles_upper, hipStream_t st) {
    static std::once_flag once;
    static hipError_t attr_err = hipSuccess;
    constexpr int lds = gram_lds_bytes<B>();
    std::call_once(once, [] {
        attr_err = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gram<In, B, ALIGNED>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    });
    if (attr_err != hipSuccess) return attr_err;
    if (tiles_upper < 1) return hipSuccess;
    const unsigned grid = (unsigned)(tiles_upper < 65535 ? tiles_upper : 65535);
    hipLaunchKernelGGL((k_gram<In, B, ALIGNED>), dim3(grid), dim3(256), lds, st, p);
    return hipGetLastError();
}

inline long long tiles_for(int mode, int nS, int nT, int B) {
    const long long nbS = (nS + B - 1) / B, nbT = (nT + B - 1) / B;
    return mode == MODE_CROSS ? nbS * nbT : nbT * (nbT + 1) / 2;
}

int tile_override() {
    const char* e = getenv("ADA_TILE");
    if (!e) return 0;
    const int v = atoi(e);
    return (v == 64 || v == 128) ? v : 0;
}

// nS_upper / nT_upper: host-known upper bounds of the list lengths (the kernel reads the actual ones)
template <typename In, bool ALIGNED>
hipError_t launch_gram_any(const GramParams& p, int nS_upper, int nT_upper, hipStream_t st) {
    int B = tiles_for(p.mode, nS_upper, nT_upper, 128) >= 192 ? 128 : 64;
    if (int o = tile_override()) B = o;
    if (B == 128) return launch_gram<In, 128, ALIGNED>(p, tiles_for(p.mode, nS_upper, nT_upper, 128), st);
    return launch_gram<In, 64, ALIGNED>(p, tiles_for(p.mode, nS_upper, nT_upper, 64), st);
}

template <typename In, bool ALIGNED>
hipError_t launch_norm_prep(const void* X, long long ld, int T, int d, float* gamma, const Workspace& w,
                            const PrepParams& prep, hipStream_t st) {
    const int nb = (T + 3) / 4;
    hipLaunchKernelGGL((k_norm_prep<In, ALIGNED>), dim3(nb + (prep.enabled ? 1 : 0)), dim3(256), 0, st,
                       reinterpret_cast<const In*>(X), ld, T, d, w.inv_norm, gamma, w, prep, nb);
    return hipGetLastError();
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
             int32_t* counts, uint64_t* gram_ops, float* gamma, void* ws, hipStream_t st) {
    const Workspace w = carve(ws, T);
    float* g = gamma ? gamma : w.gamma;
    const float thr = threshold_of(tau);
    const PrepParams prep = {nullptr, nullptr, 0, 0};
    const GramParams p = {X, ld, T, d, nullptr, nullptr, nullptr, w.inv_norm, g, thr, MODE_FULL, 1};
    hipError_t e = dispatch(dtype, X, ld, d, [&](auto v) {
        using V = decltype(v);
        hipError_t e1 = launch_norm_prep<typename V::In, V::aligned>(X, ld, T, d, g, w, prep, st);
        if (e1 != hipSuccess) return e1;
        return launch_gram_any<typename V::In, V::aligned>(p, T, T, st);
    });
    if (e != hipSuccess) return ADA_ERR_DEVICE;
    const UpdateParams u = {g, nullptr, nullptr, T, thr, mask, idx, nullptr, nullptr, counts,
                            reinterpret_cast<unsigned long long*>(gram_ops)};
    hipLaunchKernelGGL(k_update, dim3(1), dim3(1024), 0, st, u);
    return hipGetLastError() == hipSuccess ? ADA_OK : ADA_ERR_DEVICE;
}

// Algorithm 1.  Arguments checked by the caller; adds / removes / gram_ops / gamma may be NULL.
int run_cascade(const void* X, int T, int d, long long ld, int dtype, float tau, const int32_t* prev_idx, int r,
                const int32_t* r_dev, int32_t* idx, int32_t* adds, int32_t* removes, int32_t* counts,
                uint64_t* gram_ops, float* gamma, void* ws, hipStream_t st, unsigned flags) {
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
        e1 = launch_gram_any<typename V::In, V::aligned>(rep, nS_up, nS_up, st);
        if (e1 != hipSuccess || nT_up < 1) return e1;
        // steps 6-9: every other token against the valid representatives
        return launch_gram_any<typename V::In, V::aligned>(cross, nS_up, nT_up, st);
    });
    if (e != hipSuccess) return ADA_ERR_DEVICE;
    // step 10 and the bookkeeping of eq. (6) / eq. (8)
    const UpdateParams u = {g, w.is_rep, w.meta, T, thr, nullptr, idx, adds, removes, counts,
                            reinterpret_cast<unsigned long long*>(gram_ops)};
    hipLaunchKernelGGL(k_update, dim3(1), dim3(1024), 0, st, u);
    return hipGetLastError() == hipSuccess ? ADA_OK : ADA_ERR_DEVICE;
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

int ada_select_full(const void* X, int T, int d, int64_t ld, int dtype, float tau, uint8_t* mask, int32_t* idx,
                    int32_t* count, float* gamma, void* ws, size_t ws_bytes, void* stream, unsigned flags) {
    (void)flags;
    if (!mask || !count) return ADA_ERR_NULL;
    if (int e = check_common(X, T, d, ld, dtype, tau, ws, ws_bytes)) return e;
    return run_full(X, T, d, ld, dtype, tau, mask, idx, count, nullptr, gamma, ws, (hipStream_t)stream);
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
    for (int l = 1; l < L && e == ADA_OK; ++l) {
        const size_t o = (size_t)l * (size_t)T;
        e = run_cascade(X_layers[l], T, d, ld, dtype, tau, idx_all + o - T, T, counts_all + (size_t)(l - 1) * 4,
                        idx_all + o, adds_all ? adds_all + o : nullptr, removes_all ? removes_all + o : nullptr,
                        counts_all + (size_t)l * 4, gram_ops_all + l, nullptr, ws, st, flags);
    }
    return e;
}

int ada_set_overlap(const uint8_t* mask_a, const uint8_t* mask_b, int T, int32_t* out, void* stream) {
    if (!mask_a || !mask_b || !out) return ADA_ERR_NULL;
    if (T < 1 || T > ADA_MAX_T) return ADA_ERR_SHAPE;
    hipLaunchKernelGGL(k_overlap, dim3(1), dim3(1024), 0, (hipStream_t)stream, mask_a, mask_b, T, out);
    return hipGetLastError() == hipSuccess ? ADA_OK : ADA_ERR_DEVICE;
}

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
