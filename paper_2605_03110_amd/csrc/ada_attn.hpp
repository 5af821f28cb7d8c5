// Attention on the representative set -- eq. (1) of Section 2.3 -- and the hand-over of each representative's output row
// to the tokens it represents.  Included by ada_kernels.hip after the tile helpers (Mfma, lds_swz, u32x4, f32x16).
//
// Per head: O_R = softmax(Q_R K_R^T / sqrt(d_h)) V_R on the r representative rows only (r x r instead of T x T), then
// out[t] = O_R[position of assign[t] in R].  The work is small (a few GFLOP at r ~ 400), so the kernel is a plain
// blocked softmax attention: one workgroup per (64 query representatives, head), key / value rows in blocks of 64
// gathered through the index list, scores and weights kept in fp32, running row maximum and sum across key blocks.
//   * S = Q K^T: the Gram tile pattern (both operands K-contiguous rows in LDS, 32x32 MFMA blocks, one per wave).
//   * P V needs V with the key index contiguous, so V blocks are transposed while they are staged into LDS.
//   * For bf16 inputs the weights enter the second product as hi + lo bf16 pairs (p = hi + lo to 2^-17 relative), so
//     the product keeps fp32-level accuracy; fp32 inputs use fp32 MFMA throughout.
// LDS rows are XOR-swizzled in 16-byte pieces so that 16 consecutive rows read at one piece index cover 16 different
// bank groups of the 64-bank LDS (rows of 128 bytes: lds_swz; rows of 256 or 512 bytes: row % 16).
#pragma once

struct AttnParams {
    const void* Q;
    const void* K;
    const void* V;
    long long ld;
    int T, H;
    const int32_t* idx;        // R, ascending
    const int32_t* r_dev;      // optional device count
    int r_host;
    const int32_t* pos;        // [T] position of assign[t] in R (k_attn_pos)
    float* out;
    long long ld_out;
    float scale;               // 1 / sqrt(d_h)
    int causal;
    int32_t* info;             // [4]: written by workgroup (0, 0) of the attention kernel
    const int32_t* err;        // [nerr] one status word per workgroup of k_attn_pos
    int nerr;
};

// position of every token's representative in R, by binary search; validates R (strictly ascending, in range) and
// assign (a member of R).  Every workgroup leaves ONE status word (its own, written whatever it found: nothing has
// to be cleared beforehand); the attention kernel reads them all.
__global__ __launch_bounds__(256) void k_attn_pos(const int32_t* __restrict__ idx, const int32_t* r_dev, int r_host,
                                                  const int32_t* __restrict__ assign, int T, int32_t* __restrict__ pos,
                                                  int32_t* __restrict__ err) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int r = r_dev ? *r_dev : r_host;
    const bool r_ok = r >= 1 && r <= r_host && r <= T;         // the same for every thread of the launch
    int bad = 0;
    if (!r_ok) {
        if (i < T) pos[i] = 0;
    } else {
        if (i < r) {
            const int q = idx[i];
            if (q < 0 || q >= T || (i > 0 && !(idx[i - 1] < q))) bad = 1;
        }
        if (i < T) {
            const int a = assign[i];
            int lo = 0, hi = r - 1;
            while (lo < hi) {                              // first position with idx[pos] >= a
                const int mid = (lo + hi) >> 1;
                if (idx[mid] < a) lo = mid + 1; else hi = mid;
            }
            if (idx[lo] != a) bad = 1;
            pos[i] = lo;
        }
    }
    bad = __syncthreads_or(bad);
    if (threadIdx.x == 0) err[blockIdx.x] = !r_ok ? (int)ADA_ERR_SHAPE : bad ? (int)ADA_ERR_INDEX : (int)ADA_OK;
}

// The status of the call (the worst word k_attn_pos left), the same in every thread; workgroup (0, 0) reports it.
__device__ inline int attn_status(const AttnParams& p, int r) {
    const int lane = threadIdx.x & 63;
    int e = (r >= 1 && r <= p.r_host && r <= p.T) ? 0 : (int)ADA_ERR_SHAPE;   // (positions from elsewhere: nerr = 0)
    for (int i = lane; i < p.nerr; i += 64) e = max(e, p.err[i]);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) e = max(e, __shfl_xor(e, o, 64));
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        p.info[0] = e == (int)ADA_ERR_SHAPE ? 0 : r;
        p.info[1] = 0;
        p.info[2] = 0;
        p.info[3] = e;
    }
    return e;
}

// Workgroup -> (head, first query block).  Workgroups go to the eight XCDs in turn by their linear index, and every
// XCD has an L2 of its own: with the launch's natural order the query blocks of one head would sit on eight different
// XCDs and each of them would pull that head's K and V rows from memory.  When the head count is a multiple of 8 the
// index is re-read so that a head's workgroups share an XCD (head % 8).
struct AttnWho { int h, qblk; };
__device__ inline AttnWho attn_who(int H) {
    const int gx = gridDim.x, lin = blockIdx.y * gx + blockIdx.x;
    if (H % 8 != 0) return {(int)blockIdx.y, (int)blockIdx.x};
    const int xcd = lin & 7, slot = lin >> 3;
    return {(slot / gx) * 8 + xcd, slot % gx};
}

__device__ inline int attn_off(int row, int piece, int ppr) {
    const int swz = ppr >= 16 ? (row & 15) : lds_swz(row);
    return row * ppr * 16 + ((piece ^ swz) << 4);
}

template <typename In> __device__ inline In attn_elem(u32x4 v, int e);
template <> __device__ inline uint16_t attn_elem<uint16_t>(u32x4 v, int e) { return (uint16_t)(v[e >> 1] >> (16 * (e & 1))); }
template <> __device__ inline float attn_elem<float>(u32x4 v, int e) { return __uint_as_float(v[e]); }

__device__ inline uint32_t attn_bf16_rne(float f) {        // finite inputs; rounds the magnitude, keeps the sign
    const uint32_t u = __float_as_uint(f);
    return ((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16) & 0xFFFFu;
}

template <typename In, int DH> struct AttnGeom {
    static constexpr int E = (int)sizeof(In), EPP = 16 / E;
    static constexpr int ROWB = DH * E, PPR = ROWB / 16;              // a Q / K row of one head
    static constexpr int PPRV = 64 * E / 16;                          // a V^T or P row: 64 keys
    static constexpr int OFF_Q = 0, OFF_K = 64 * ROWB, OFF_VT = 2 * 64 * ROWB;
    static constexpr int OFF_S = 3 * 64 * ROWB;                       // float[64][65]
    static constexpr int OFF_P = OFF_S + 64 * 65 * 4;                 // weights: bf16 hi then lo (8 KB each), or fp32 (16 KB)
    static constexpr int OFF_ROW = OFF_P + 16384;                     // alpha[64], lsum[64], qtok[64], ktok[64]
    static constexpr int OFF_LIST = OFF_ROW + 4 * 64 * 4;             // int[256] + counter
    static constexpr int LDS = OFF_LIST + 257 * 4;
    static_assert(PPR == 8 || PPR == 16 || PPR == 32, "head rows of 128, 256 or 512 bytes");
    static_assert(DH % 64 == 0, "head dimension in multiples of 64");
};

#ifdef ADA_PHASE_CLOCKS
#define ATTN_CLK(k) do { if (threadIdx.x == 0 && (k) < 8) g_pass_clk[((blockIdx.y * gridDim.x + blockIdx.x) & 511) * 8 + ((k) & 7)] = __builtin_amdgcn_s_memrealtime(); } while (0)
#else
#define ATTN_CLK(k) do { } while (0)
#endif

template <typename In, int DH>
__global__ __launch_bounds__(256) void k_attn_rep(AttnParams p) {
    using G = AttnGeom<In, DH>;
    constexpr int EPP = G::EPP, PPR = G::PPR, PPRV = G::PPRV, NB = DH / 64;
    extern __shared__ __align__(16) char lds[];
    char* qbuf = lds + G::OFF_Q;
    char* kbuf = lds + G::OFF_K;
    char* vtbuf = lds + G::OFF_VT;
    float* sbuf = reinterpret_cast<float*>(lds + G::OFF_S);
    char* pbuf = lds + G::OFF_P;
    float* alpha = reinterpret_cast<float*>(lds + G::OFF_ROW);
    float* lsum = alpha + 64;
    int* qtok = reinterpret_cast<int*>(lsum + 64);
    int* ktok = qtok + 64;
    int* list = reinterpret_cast<int*>(lds + G::OFF_LIST);

    ATTN_CLK(0);
    const int r = p.r_dev ? *p.r_dev : p.r_host;
    if (attn_status(p, r) != ADA_OK) return;               // k_attn_pos rejected the set or the assignment
    const AttnWho who = attn_who(p.H);
    const int h = who.h;
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // query blocks are dealt round-robin over gridDim.x: with the set size known only on the device the launcher
    // sizes the grid for the chip, not for the largest possible set (idle workgroups of this LDS size are not free)
    for (int q0 = who.qblk * 64; q0 < r; q0 += gridDim.x * 64) {
    __syncthreads();                                       // a previous query block's hand-over is done with the LDS
    const In* Qh = reinterpret_cast<const In*>(p.Q) + (size_t)h * DH;
    const In* Kh = reinterpret_cast<const In*>(p.K) + (size_t)h * DH;
    const In* Vh = reinterpret_cast<const In*>(p.V) + (size_t)h * DH;

    constexpr int NP = PPR / 4;                            // 16-byte pieces per thread per 64-row block
    if (tid < 64) qtok[tid] = min(max(p.idx[min(q0 + tid, r - 1)], 0), p.T - 1);
    __syncthreads();
    {   // Q block: rows gathered through the list; all loads are issued before the first store
        u32x4 qreg[NP];
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const int i = tid + 256 * j, row = i / PPR, pc = i % PPR;
            qreg[j] = *reinterpret_cast<const u32x4*>(Qh + (size_t)qtok[row] * (size_t)p.ld + pc * EPP);
        }
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const int i = tid + 256 * j, row = i / PPR, pc = i % PPR;
            *reinterpret_cast<u32x4*>(qbuf + attn_off(row, pc, PPR)) = qreg[j];
        }
    }
    // K and V blocks travel through registers one block ahead of the products.  K pieces are fetched row-major
    // (coalesced); V pieces with the key row fastest across lanes, so that the transposed 2- or 4-byte stores of one
    // wave instruction fill one whole row of V^T instead of colliding on a few banks.
    // The token ids of a block are requested one block before its rows, so that neither trip to memory is waited for
    // in the middle of a block: ids(kb + 2) and fetch(kb + 1) are issued behind the products of block kb.
    u32x4 kreg[NP], vreg[NP];
    int ktid[NP], vtid;
    auto ids = [&](int kb) {
#pragma unroll
        for (int j = 0; j < NP; ++j) ktid[j] = p.idx[min(kb * 64 + (tid + 256 * j) / PPR, r - 1)];
        vtid = p.idx[min(kb * 64 + (tid & 63), r - 1)];
    };
    auto fetch = [&]() {                                   // rows of the block whose ids are in ktid / vtid
        const size_t vt = (size_t)min(max(vtid, 0), p.T - 1) * (size_t)p.ld;
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const int i = tid + 256 * j;
            const int kpc = i % PPR, vpc = i >> 6;
            kreg[j] = *reinterpret_cast<const u32x4*>(Kh + (size_t)min(max(ktid[j], 0), p.T - 1) * (size_t)p.ld + kpc * EPP);
            vreg[j] = *reinterpret_cast<const u32x4*>(Vh + vt + vpc * EPP);
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int j = 0; j < NP; ++j) {
            const int i = tid + 256 * j;
            const int krow = i / PPR, kpc = i % PPR, vrow = i & 63, vpc = i >> 6;
            *reinterpret_cast<u32x4*>(kbuf + attn_off(krow, kpc, PPR)) = kreg[j];
            // V^T: element (key row, column c) goes to row c, key position row
#pragma unroll
            for (int e = 0; e < EPP; ++e) {
                const int c = vpc * EPP + e;
                *reinterpret_cast<In*>(vtbuf + attn_off(c, vrow / EPP, PPRV) + (vrow % EPP) * G::E) = attn_elem<In>(vreg[j], e);
            }
        }
    };

    // running maximum and sum of the row this thread helps with (four threads per row hold the same values)
    const int srow = tid >> 2, spart = tid & 3;
    float m_run = -INFINITY, l_run = 0.f;
    f32x16 acc_o[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc_o[i][e] = 0.f;

    const int nkb_all = (r + 63) / 64;
    const int nkb = p.causal ? min(nkb_all, q0 / 64 + 1) : nkb_all;   // R is in sequence order: later key blocks are fully masked
    ids(0);
    fetch();
    ids(1);
    ATTN_CLK(1);
    for (int kb = 0; kb < nkb; ++kb) {
        if (kb == 1) ATTN_CLK(2);
        __syncthreads();                                   // the previous block's products are done with K, V^T, P
        if (tid < 64) ktok[tid] = min(max(p.idx[min(kb * 64 + tid, r - 1)], 0), p.T - 1);
        stash();
        __syncthreads();
        if (kb == 1) ATTN_CLK(3);
        if (kb + 1 < nkb) { fetch(); ids(kb + 2); }        // in flight behind this block's products
        {   // ---- S = Q K^T for this wave's 32 x 32 block, scaled and masked, to LDS
            const int wa = wave >> 1, wb = wave & 1;
            f32x16 acc;
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < PPR / 2; ++ks) {
                const u32x4 fa = *reinterpret_cast<const u32x4*>(qbuf + attn_off(wa * 32 + l32, 2 * ks + half, PPR));
                const u32x4 fb = *reinterpret_cast<const u32x4*>(kbuf + attn_off(wb * 32 + l32, 2 * ks + half, PPR));
                Mfma<In>::run(acc, fa, fb);
            }
            const int kc = wb * 32 + l32;                  // key column of this lane
            const bool k_in = kb * 64 + kc < r;
            const int kt = p.causal ? ktok[kc] : INT_MIN;  // without the mask no key is "later"
            i32x4 qt4[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) qt4[q] = *reinterpret_cast<const i32x4*>(qtok + wa * 32 + 8 * q + 4 * half);
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int qr = wa * 32 + (e & 3) + 4 * half + 8 * (e >> 2);
                const bool masked = !k_in | (kt > qt4[e >> 2][e & 3]);
                sbuf[qr * 65 + kc] = masked ? -INFINITY : acc[e] * p.scale;
            }
        }
        __syncthreads();
        {   // ---- softmax bookkeeping for row srow, columns 16 spart .. 16 spart + 15
            float s[16];
            float mx = -INFINITY;
#pragma unroll
            for (int j = 0; j < 16; ++j) { s[j] = sbuf[srow * 65 + spart * 16 + j]; mx = fmaxf(mx, s[j]); }
            mx = fmaxf(mx, __shfl_xor(mx, 1, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 2, 64));
            const float m_new = fmaxf(m_run, mx);
            const float a = m_new == -INFINITY ? 1.f : __expf(m_run - m_new);    // exp(-inf) = 0 on the first block
            float sum = 0.f;
#pragma unroll
            for (int j = 0; j < 16; ++j) { s[j] = m_new == -INFINITY ? 0.f : __expf(s[j] - m_new); sum += s[j]; }
            sum += __shfl_xor(sum, 1, 64);
            sum += __shfl_xor(sum, 2, 64);
            l_run = l_run * a + sum;
            m_run = m_new;
            if (spart == 0) alpha[srow] = a;
            if constexpr (sizeof(In) == 2) {               // hi + lo bf16 pairs, 8 weights per 16-byte piece
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    u32x4 hi, lo;
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        uint32_t hw = 0u, lw = 0u;
#pragma unroll
                        for (int z = 0; z < 2; ++z) {
                            const float pv = s[q * 8 + w * 2 + z];
                            const uint32_t hb = attn_bf16_rne(pv);
                            const uint32_t lo16 = attn_bf16_rne(pv - __uint_as_float(hb << 16));   // signed remainder
                            hw |= hb << (16 * z);
                            lw |= (lo16 & 0xFFFFu) << (16 * z);
                        }
                        hi[w] = hw; lo[w] = lw;
                    }
                    *reinterpret_cast<u32x4*>(pbuf + attn_off(srow, spart * 2 + q, PPRV)) = hi;
                    *reinterpret_cast<u32x4*>(pbuf + 8192 + attn_off(srow, spart * 2 + q, PPRV)) = lo;
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<u32x4*>(pbuf + attn_off(srow, spart * 4 + q, PPRV)) =
                        u32x4{__float_as_uint(s[4 * q]), __float_as_uint(s[4 * q + 1]), __float_as_uint(s[4 * q + 2]),
                              __float_as_uint(s[4 * q + 3])};
            }
        }
        __syncthreads();
        // ---- O = alpha O + P V for this wave's blocks (block b: query half b % 2, column block b / 2)
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int b = wave + 4 * i, qa = b & 1, cb = b >> 1;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 a4 = *reinterpret_cast<const f32x4*>(alpha + qa * 32 + 8 * q + 4 * half);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc_o[i][4 * q + e] *= a4[e];
            }
#pragma unroll
            for (int ks = 0; ks < PPRV / 2; ++ks) {
                const u32x4 fb = *reinterpret_cast<const u32x4*>(vtbuf + attn_off(cb * 32 + l32, 2 * ks + half, PPRV));
                const u32x4 fa = *reinterpret_cast<const u32x4*>(pbuf + attn_off(qa * 32 + l32, 2 * ks + half, PPRV));
                Mfma<In>::run(acc_o[i], fa, fb);
                if constexpr (sizeof(In) == 2) {
                    const u32x4 fl = *reinterpret_cast<const u32x4*>(pbuf + 8192 + attn_off(qa * 32 + l32, 2 * ks + half, PPRV));
                    Mfma<In>::run(acc_o[i], fl, fb);
                }
            }
        }
    }
    ATTN_CLK(6);
    if (spart == 0) lsum[srow] = l_run;
    __syncthreads();                                       // everybody is done with Q, K (O is laid over them)
    float* obuf = reinterpret_cast<float*>(lds + G::OFF_Q);   // [64][DH]
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int b = wave + 4 * i, qa = b & 1, cb = b >> 1;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 l4 = *reinterpret_cast<const f32x4*>(lsum + qa * 32 + 8 * q + 4 * half);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int qr = qa * 32 + e + 4 * half + 8 * q;
                const float inv = l4[e] > 0.f ? 1.0f / l4[e] : 0.f;
                obuf[qr * DH + cb * 32 + l32] = acc_o[i][4 * q + e] * inv;
            }
        }
    }
    __syncthreads();
    ATTN_CLK(7);
    // ---- hand-over: every token whose representative sits in this block takes that row (tokens in chunks of 256)
    float* outh = p.out + (size_t)h * DH;
    for (int tb = 0; tb < p.T; tb += 8 * 256) {            // positions of 2048 tokens at a time, one trip to memory
        int rel[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int t = tb + u * 256 + tid;
            rel[u] = t < p.T ? p.pos[t] - q0 : -1;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (tb + u * 256 >= p.T) break;                // uniform
            if (tid == 0) list[256] = 0;
            __syncthreads();
            if ((unsigned)rel[u] < 64u) list[atomicAdd(&list[256], 1)] = ((tb + u * 256 + tid) << 6) | rel[u];
            __syncthreads();
            const int n = list[256];
            for (int j = wave; j < n; j += 4) {            // one wave per token row
                const int e = list[j], tt = e >> 6, row = e & 63;
                float* dst = outh + (size_t)tt * (size_t)p.ld_out;
#pragma unroll
                for (int c = 0; c < DH; c += 64) dst[c + lane] = obuf[row * DH + c + lane];
            }
            __syncthreads();
        }
    }
    ATTN_CLK(4);
    }
}


// ------------------------------------------------------------------------------------------------
// k_attn_rep2 (bf16): the same computation with the scores kept in registers.
//   The first kernel sends every block of scores through LDS twice (scores out, weights back) and meets at five
//   barriers per key block; with r / 64 key blocks in sequence that chain, not the arithmetic, is its duration.
//   Here S^T = K Q^T is computed instead of S (keys on the MFMA M side): an accumulator register then belongs to a key
//   and a LANE to a query, so a query's maximum and sum over the 64 keys of a block are in-lane reductions plus one
//   exchange between the lane halves, and the weights are already laid out as the B operand of the second product,
//   O^T = V^T P^T, if the keys of V^T are stored in the matching order (within every 16 keys the two middle groups of
//   four swap places: an accumulator's registers cover keys 0-3, 8-11 in one lane half and 4-7, 12-15 in the other).
//   Wave w serves the 32 queries of block w % 2 against the 32 keys of half w / 2 of every key block, with a running
//   maximum, sum and O^T (all d_h columns) of its own; the two waves of a query block are merged once, after the last
//   key block (the usual rescaling to the common maximum).  Nothing is exchanged inside the loop, and a lane handles
//   16 scores per block.  Two barriers per key block remain (see below).
//   Weights are powers of 2 against a reference that only moves when a block's maximum passes it by more than 10
//   (the accumulated rows are rescaled on few blocks, and stay in the accumulation registers otherwise).
//   K rows go global -> LDS directly into one of two stages; token indices are read once per block (lane = row) and
//   handed out by lane reads.
//   V is read the way K is (whole 128-byte lines per instruction: a lane group of 8 takes one line of a row, a thread
//   takes the same columns of two neighbouring keys) and transposed on the way into LDS, two keys per 32-bit write.
//   A V^T row's eight 16-byte slots are permuted by (c ^ (c >> 3)) & 7: the transposing writes (same keys, rows 8 apart)
//   and the operand reads (same slot, 16 consecutive rows) are then both spread over all banks.
typedef __bf16 attn_bf16x2 __attribute__((ext_vector_type(2)));
typedef float attn_f32x2 __attribute__((ext_vector_type(2)));
__device__ inline int attn_vt_off(int c, int piece) { return c * 128 + ((piece ^ ((c ^ (c >> 3)) & 7)) << 4); }

template <int DH> struct AttnGeom2 {
    static constexpr int ROWB = DH * 2, PPR = ROWB / 16, PPRV = 8;
    static constexpr int KSTAGE = 64 * ROWB;                                           // K: two stages (even and odd key blocks)
    static constexpr int OFF_Q = 0, OFF_K = 64 * ROWB, OFF_VT = 3 * 64 * ROWB;        // V^T: DH rows of 128 bytes
    static constexpr int OS = DH + 4;      // row of the output block: 16-byte accesses, consecutive rows one slot apart
    static constexpr int OFF_TAKERS = (64 * OS * 4 + 15) / 16 * 16;                    // behind the output block
    static constexpr int MAIN = (4 * 64 * ROWB > OFF_TAKERS + 2048 * 4) ? 4 * 64 * ROWB : OFF_TAKERS + 2048 * 4;
    static constexpr int OFF_ROW = MAIN;                                               // qtok[64], ktok[64], m[2][64], l[2][64]
    static constexpr int OFF_LIST = OFF_ROW + 6 * 64 * 4;
    static constexpr int LDS = OFF_LIST + 257 * 4;
};

// EIGHT waves: waves 0 .. 3 multiply as described and never touch memory inside the key-block loop; waves 4 .. 7 fetch
// (K rows straight into LDS, V rows through their registers and transposed into LDS, the token indices of the coming
// blocks).  A wave that issues a load waits for room in the memory pipeline; when the four multiplying waves fetched
// for themselves (one wave per SIMD), that wait -- a microsecond per key block here -- and the staging of V added to the
// time of the products (41.7 against 32.2 us at 16 heads x 256, r = 434).  With half the register file per wave, the
// operand addresses inside the loop are one base per buffer XOR a constant.  Two barriers per key block kb, met by all
// eight waves:
//   A(kb): K(kb) has landed in its stage and V(kb) in the loaders' registers; the multipliers have left V^T(kb - 1).
//          Then the loaders write V^T(kb) and ask for V(kb + 1); the multipliers form the scores and weights of kb.
//   B(kb): V^T(kb) is written; the multipliers have left K(kb).  Then the loaders ask for K(kb + 2) into the stage just
//          left and for the indices of block kb + 3; the multipliers add weights x V^T(kb) to their rows.
template <int DH>
__global__ __launch_bounds__(512) void k_attn_rep2(AttnParams p) {
    using In = uint16_t;
    using G = AttnGeom2<DH>;
    constexpr int EPP = 8, PPR = G::PPR, NB = DH / 32, KS = DH / 16, NP = PPR / 4;
    extern __shared__ __align__(16) char lds[];
    char* qbuf = lds + G::OFF_Q;
    char* kbuf = lds + G::OFF_K;
    char* vtbuf = lds + G::OFF_VT;
    int* qtok = reinterpret_cast<int*>(lds + G::OFF_ROW);
    int* ktok = qtok + 64;
    float* mrow = reinterpret_cast<float*>(ktok + 64);     // [2][64] running maxima and sums of the two key halves
    float* lrow = mrow + 128;
    int* list = reinterpret_cast<int*>(lds + G::OFF_LIST);                 // the takers' counter
    int* takers = reinterpret_cast<int*>(lds + G::OFF_TAKERS);            // up to 2048 (token, row) pairs

    const int r = p.r_dev ? *p.r_dev : p.r_host;
    if (attn_status(p, r) != ADA_OK) return;               // k_attn_pos rejected the set or the assignment
    const AttnWho who = attn_who(p.H);
    const int h = who.h;
    const int tid = threadIdx.x, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave8 >= 4;
    const int wave = wave8 & 3;                            // place among the waves of its kind
    const int qb = wave & 1, kh = wave >> 1;
    ATTN_CLK(0);
    for (int q0 = who.qblk * 64; q0 < r; q0 += gridDim.x * 64) {
    __syncthreads();                                       // a previous query block's hand-over is done with the LDS
    const In* Qh = reinterpret_cast<const In*>(p.Q) + (size_t)h * DH;
    const In* Kh = reinterpret_cast<const In*>(p.K) + (size_t)h * DH;
    const In* Vh = reinterpret_cast<const In*>(p.V) + (size_t)h * DH;
    auto ids = [&](int kb) { return min(max(p.idx[min(kb * 64 + lane, r - 1)], 0), p.T - 1); };
    // every wave keeps the 64 query tokens in one register (lane = row) and hands them out with lane reads
    const int qtokv = min(max(p.idx[min(q0 + lane, r - 1)], 0), p.T - 1);
    int tok_cur = 0, tok_n1 = 0, tok_n2 = 0;               // loaders: the tokens of key blocks kb, kb + 1, kb + 2 (lane = row)
    if (loader) { tok_cur = ids(0); tok_n1 = ids(1); tok_n2 = ids(2); }
    const int nkb_all = (r + 63) / 64;
    const int nkb = p.causal ? min(nkb_all, q0 / 64 + 1) : nkb_all;

    float m_run = -INFINITY, l_run = 0.f;                  // of query qb * 32 + l32 over THIS wave's keys (both lane halves alike)
    f32x16 acc_o[NB];                                      // O^T blocks: rows = output columns 32 i + ..., lane = query
    const int my_q = qb * 32 + l32;
    if (loader) {
        // K: 1 KB (64 / PPR rows) per wave instruction, the 16-byte slots of a row permuted on the global side so that
        // the LDS image is the swizzled one the operand reads expect.  V: thread (wave, lane) takes keys
        // 16 wave + 2 (lane / 8) + {0, 1} and, for j / 2 = line, columns 64 line + 8 (lane % 8) .. + 7.
        u32x4 vreg[NP];
        const int vkey = 16 * wave + 2 * (lane >> 3), vp8 = lane & 7;
        auto fetch_k = [&](int stage, int tok) {
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                const int krow = (j * 4 + wave) * (64 / PPR) + lane / PPR, slot = lane % PPR;
                const int kpc = slot ^ (PPR >= 16 ? (krow & 15) : lds_swz(krow));
                const In* src = Kh + (size_t)__shfl(tok, krow, 64) * (size_t)p.ld + kpc * EPP;
                char* dst = kbuf + stage * G::KSTAGE + (j * 4 + wave) * 1024;           // wave-uniform
                __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)src,
                                                 (void __attribute__((address_space(3)))*)dst, 16, 0, 0);
            }
        };
        auto fetch_v = [&](int tok) {
            const size_t vt0 = (size_t)__shfl(tok, vkey, 64) * (size_t)p.ld;
            const size_t vt1 = (size_t)__shfl(tok, vkey + 1, 64) * (size_t)p.ld;
#pragma unroll
            for (int j = 0; j < NP; ++j)
                vreg[j] = *reinterpret_cast<const u32x4*>(Vh + ((j & 1) ? vt1 : vt0) + ((j >> 1) * 8 + vp8) * EPP);
        };
        auto stash = [&]() {
            // V^T with the keys of every group of 16 in the order the weights' registers have: 0-3, 8-11, 4-7, 12-15
            const int o = vkey & 15;
            const int pos = (vkey & ~15) | ((o & 3) | ((o & 4) << 1) | ((o & 8) >> 1));          // even: this key and the next
#pragma unroll
            for (int j = 0; j < NP; j += 2)
#pragma unroll
                for (int e = 0; e < EPP; ++e) {
                    const int c = ((j >> 1) * 8 + vp8) * EPP + e;
                    const uint32_t two = (uint32_t)attn_elem<In>(vreg[j], e) | ((uint32_t)attn_elem<In>(vreg[j + 1], e) << 16);
                    *reinterpret_cast<uint32_t*>(vtbuf + attn_vt_off(c, pos >> 3) + (pos & 7) * 2) = two;
                }
        };
        fetch_k(0, tok_cur);
        fetch_v(tok_cur);
        fetch_k(1, tok_n1);
        for (int kb = 0; kb < nkb; ++kb) {
            if (p.causal && wave == 0) ktok[lane] = tok_cur;              // the tokens of the block about to be multiplied
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(NP));  // K(kb) and V(kb) are here; K(kb + 1) may still be on its way
            __builtin_amdgcn_s_barrier();                      // A(kb)
            stash();
            fetch_v(tok_n1);                                   // V(kb + 1) (past the last block: a repeat nobody uses)
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(63)); // V^T(kb) is written
            __builtin_amdgcn_s_barrier();                      // B(kb)
            tok_cur = tok_n1;
            tok_n1 = tok_n2;
            tok_n2 = ids(kb + 3);
            fetch_k(kb & 1, tok_n1);                           // K(kb + 2) into the stage the multipliers have just left
        }
    } else {
        // Q goes through the multiplying waves' registers into LDS while the loaders fetch the first key blocks; barrier
        // A(0) is also the one behind which Q is staged
        {
            u32x4 qreg[NP];
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                const int i = tid + 256 * j, row = i / PPR, pc = i % PPR;
                qreg[j] = *reinterpret_cast<const u32x4*>(Qh + (size_t)__shfl(qtokv, row, 64) * (size_t)p.ld + pc * EPP);
            }
#pragma unroll
            for (int j = 0; j < NP; ++j) {
                const int i = tid + 256 * j, row = i / PPR, pc = i % PPR;
                *reinterpret_cast<u32x4*>(qbuf + attn_off(row, pc, PPR)) = qreg[j];
            }
        }
#pragma unroll
        for (int i = 0; i < NB; ++i)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc_o[i][e] = 0.f;
        const float sc2 = p.scale * 1.44269504088896340736f;
        // The query operands of the first k-steps stay in registers (this lane's query row), as many as the register
        // file has room for beside the rows; the rest is read from LDS in every block.
        constexpr int QREG = KS <= 8 ? KS : 2;
        u32x4 qf[QREG];
        // Operand addresses inside the loop: one base per buffer XOR a constant (the slot of k-step ks is
        // (half ^ swizzle) ^ 2 ks; a V^T row block i flips one more slot bit), recomputed where they are used: the
        // 48 addresses would not fit beside the rows in the half register file a wave has here.
        const uint32_t k_base = (uint32_t)attn_off(kh * 32 + l32, half, PPR);
        const uint32_t q_base = (uint32_t)attn_off(my_q, half, PPR);
        const uint32_t v_base = (uint32_t)attn_vt_off(l32, 4 * kh + half);
        __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(63));     // my share of Q is written
        __builtin_amdgcn_s_barrier();                          // A(0): Q is staged as well
        ATTN_CLK(1);
#pragma unroll
        for (int ks = 0; ks < QREG; ++ks)
            qf[ks] = *reinterpret_cast<const u32x4*>(qbuf + attn_off(my_q, 2 * ks + half, PPR));
        for (int kb = 0; kb < nkb; ++kb) {
            if (kb > 0) {
                __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(63)); // my reads of V^T(kb - 1) have returned
                __builtin_amdgcn_s_barrier();                      // A(kb)
                if (kb == 1) ATTN_CLK(2);
            }
            const char* kcur = kbuf + (kb & 1) * G::KSTAGE;
            // ---- S^T = K Q^T: this wave's 32 keys (half kh of the block) against its 32 queries
            f32x16 acc_s;
#pragma unroll
            for (int e = 0; e < 16; ++e) acc_s[e] = 0.f;
            uint32_t kb_ = k_base, qb_ = q_base, vb_ = v_base;
            asm volatile("" : "+v"(kb_), "+v"(qb_), "+v"(vb_));   // (opaque: keeps the XORs below out of registers)
            // (fragments are read two k-steps ahead of the MFMA that takes them: sixteen dependent MFMAs each waiting
            //  for an LDS round trip were the longest part of a block)
            u32x4 fkr[3], fqr[3];
            auto rd = [&](int ks) {
                fkr[ks % 3] = *reinterpret_cast<const u32x4*>(kcur + (kb_ ^ (uint32_t)(ks << 5)));
                if (ks >= QREG) fqr[ks % 3] = *reinterpret_cast<const u32x4*>(qbuf + (qb_ ^ (uint32_t)(ks << 5)));
            };
            rd(0);
            if (KS > 1) rd(1);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (ks + 2 < KS) rd(ks + 2);
                Mfma<In>::run(acc_s, fkr[ks % 3], ks < QREG ? qf[ks < QREG ? ks : 0] : fqr[ks % 3]);
            }
            // ---- weights of this lane's query (register e is key 32 kh + (e & 3) + 4 half + 8 (e >> 2)), in base 2:
            // t = s * scale * log2(e), weight = 2^(t - m).  m is a reference, not the exact running maximum: it moves only
            // when a block's maximum passes it by more than 10, so weights stay below 2^10 and the accumulated rows are
            // rescaled on few blocks (the quotient sum(w v) / sum(w) does not depend on the reference).
            if (p.causal || kb * 64 + 64 > r) {                // uniform: only then can a key be masked
                const int qt = __shfl(qtokv, my_q, 64);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    i32x4 kt4 = {INT_MIN, INT_MIN, INT_MIN, INT_MIN};                 // without the mask no key is "later"
                    if (p.causal) kt4 = *reinterpret_cast<const i32x4*>(ktok + kh * 32 + 8 * q + 4 * half);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int kk = kb * 64 + kh * 32 + 8 * q + 4 * half + e;
                        if ((kk >= r) | (kt4[e] > qt)) acc_s[4 * q + e] = -INFINITY;
                    }
                }
            }
            float mx = -INFINITY;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                acc_s[e] *= sc2;
                mx = fmaxf(mx, acc_s[e]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));            // the other half of the keys
            const bool grow = mx > m_run + 10.f;               // (false while both are -inf)
            if (__builtin_amdgcn_ballot_w64(grow) != 0ull) {
                const float m_new = grow ? mx : m_run;
                const float a = grow ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;   // 0 when the old reference is -inf
                l_run *= a;
                m_run = m_new;
                if (kb > 0) {                                  // (the rows are still zero on the first block)
#pragma unroll
                    for (int i = 0; i < NB; ++i)
#pragma unroll
                        for (int e = 0; e < 16; ++e) acc_o[i][e] *= a;
                }
            }
            const float m_use = m_run == -INFINITY ? 0.f : m_run;                     // all keys masked so far: weights 0
            float sum = 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float pv = __builtin_amdgcn_exp2f(acc_s[e] - m_use);
                acc_s[e] = pv;
                sum += pv;
            }
            sum += __shfl_xor(sum, 32, 64);
            l_run += sum;
            __builtin_amdgcn_s_waitcnt(waitcnt_vm_lgkm0(63)); // my reads of K(kb) (and of the key tokens) have returned
            __builtin_amdgcn_s_barrier();                      // B(kb)
            if (kb == 1) ATTN_CLK(3);
            // ---- O^T += V^T P^T: the weights of k-step j (16 keys) are registers 8 j .. 8 j + 7; each weight is split
            // into a bf16 head and a bf16 remainder (hardware round-to-nearest-even pairs), two products per step
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                u32x4 hi, lo;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const attn_f32x2 pv = {acc_s[8 * j + 2 * w], acc_s[8 * j + 2 * w + 1]};
                    const uint32_t hw = __builtin_bit_cast(uint32_t, __builtin_convertvector(pv, attn_bf16x2));
                    const attn_f32x2 rem = {pv[0] - __uint_as_float(hw << 16), pv[1] - __uint_as_float(hw & 0xFFFF0000u)};
                    hi[w] = hw;
                    lo[w] = __builtin_bit_cast(uint32_t, __builtin_convertvector(rem, attn_bf16x2));
                }
#pragma unroll
                for (int i = 0; i < NB; ++i) {
                    const u32x4 fv = *reinterpret_cast<const u32x4*>(vtbuf + (vb_ ^ (uint32_t)((i << 12) | (j << 5) | ((i & 1) << 6))));
                    Mfma<In>::run(acc_o[i], fv, hi);
                    Mfma<In>::run(acc_o[i], fv, lo);
                }
            }
        }
    }
    ATTN_CLK(6);
    int rel[4];                                            // hand-over: positions of 2048 tokens, relative to this block
    auto load_rel = [&](int tb) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = tb + u * 512 + tid;
            rel[u] = t < p.T ? p.pos[t] - q0 : -1;
        }
    };
    load_rel(0);                                           // in flight behind the merge
    // ---- the two waves of a query block hold sums over different keys: exchange (m, l), bring both to the common
    // maximum and the common denominator, and add the second wave's rows onto the first's in the output block
    if (!loader && half == 0) { mrow[kh * 64 + my_q] = m_run; lrow[kh * 64 + my_q] = l_run; }
    __syncthreads();                                       // also: everybody is done with Q, K, V^T (O is laid over them),
    float* obuf = reinterpret_cast<float*>(lds);           // [64][OS]                  and the loaders' last loads have landed
    float f = 0.f;
    if (!loader) {
        const float m_o = mrow[(kh ^ 1) * 64 + my_q], l_o = lrow[(kh ^ 1) * 64 + my_q];
        const float m_all = fmaxf(m_run, m_o);
        const float w_me = m_run == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_run - m_all);
        const float w_o = m_o == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m_o - m_all);
        const float l_all = l_run * w_me + l_o * w_o;
        f = l_all > 0.f ? w_me / l_all : 0.f;
    }
    // each wave hands the half of the columns it does not finish to its partner through the output block itself
    // (disjoint places), then adds its own share onto what it received: every place has one writer at a time
    auto give = [&](auto khc) {                            // (register blocks are addressed with constants only)
        constexpr int KH = decltype(khc)::value;
#pragma unroll
        for (int i = 0; i < NB / 2; ++i) {
            const int blk = (1 - KH) * (NB / 2) + i;       // given away
#pragma unroll
            for (int q = 0; q < 4; ++q)                    // registers 4 q .. 4 q + 3 are four consecutive columns
                *reinterpret_cast<float4*>(obuf + my_q * G::OS + 32 * blk + 8 * q + 4 * half) =
                    float4{acc_o[blk][4 * q] * f, acc_o[blk][4 * q + 1] * f, acc_o[blk][4 * q + 2] * f,
                           acc_o[blk][4 * q + 3] * f};
        }
    };
    auto finish = [&](auto khc) {
        constexpr int KH = decltype(khc)::value;
#pragma unroll
        for (int i = 0; i < NB / 2; ++i) {
            const int blk = KH * (NB / 2) + i;             // finished here
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float4* at = reinterpret_cast<float4*>(obuf + my_q * G::OS + 32 * blk + 8 * q + 4 * half);
                const float4 o = *at;
                *at = float4{o.x + acc_o[blk][4 * q] * f, o.y + acc_o[blk][4 * q + 1] * f,
                             o.z + acc_o[blk][4 * q + 2] * f, o.w + acc_o[blk][4 * q + 3] * f};
            }
        }
    };
    if (!loader) { if (kh == 0) give(std::integral_constant<int, 0>{}); else give(std::integral_constant<int, 1>{}); }
    __syncthreads();
    if (!loader) { if (kh == 0) finish(std::integral_constant<int, 0>{}); else finish(std::integral_constant<int, 1>{}); }
    __syncthreads();
    ATTN_CLK(4);
    // ---- hand-over: every token whose representative sits in this block takes that row.  The positions of 2048
    // tokens are read in one trip to memory and the takers collected in one list; a wave then copies a whole row
    // (d_h floats) per store instruction.
    float* outh = p.out + (size_t)h * DH;
    for (int tb = 0; tb < p.T; tb += 4 * 512) {
        if (tb > 0) load_rel(tb);                          // (the first 2048 were asked for before the merge)
        if (tid == 0) list[0] = 0;
        __syncthreads();
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if ((unsigned)rel[u] < 64u) takers[atomicAdd(&list[0], 1)] = ((tb + u * 512 + tid) << 6) | rel[u];
        __syncthreads();
        const int n = list[0];
        constexpr int LPR = DH / 4, RPI = 64 / LPR, NW = 8; // lanes per row (a float4 each), rows per instruction, waves
        const int sub = lane / LPR, c4 = (lane % LPR) * 4;
        // a wave's share of the list (entries wave8 * RPI + sub + NW RPI k) is read 64 entries at a time, one per lane,
        // and handed to the lane groups by lane reads; eight rows are in flight per lane group
        constexpr int KPB = 64 / RPI;                      // steps k per batch
        const int steps = (n - wave8 * RPI + NW * RPI - 1) / (NW * RPI);          // k with a first entry below n
        for (int k0 = 0; k0 < steps; k0 += KPB) {
            const int mine = takers[min(wave8 * RPI + (lane % RPI) + NW * RPI * (k0 + lane / RPI), n - 1)];
            const int kend = min(KPB, steps - k0);
            for (int kk = 0; kk < kend; kk += 8) {
                int ent[8];
                float4 v4[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) ent[u] = __shfl(mine, min(kk + u, KPB - 1) * RPI + sub, 64);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    v4[u] = *reinterpret_cast<const float4*>(obuf + (ent[u] & 63) * G::OS + c4);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (kk + u < kend && wave8 * RPI + sub + NW * RPI * (k0 + kk + u) < n)
                        *reinterpret_cast<float4*>(outh + (size_t)(ent[u] >> 6) * (size_t)p.ld_out + c4) = v4[u];
            }
        }
        __syncthreads();
    }
    }
    ATTN_CLK(7);
}
