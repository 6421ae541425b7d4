// Language-model head fused with the GRPO objective: the logits z = h W^T of the policy of
// section 3.4 are produced, reduced and differentiated here instead of being handed in.
// This file is the second half of grpo.hip's translation unit (it is included at its end
// and uses the row arithmetic, the workspace header and the small kernels defined there).
//
// Everything heavy is one bf16 MFMA kernel, lm_gemm_nt: C[M x N] = A[M x K] B[N x K]^T with
// both operands contiguous along K, fp32 accumulation.  It runs three times:
//   logits   z  = H W^T        (K = d_model)  epilogue: per-row softmax partials in fp32
//                                             from the accumulators, z_y, optional fp32 z
//   dL/dH       = G  (W^T)^T   (K = vocab)    epilogue: bf16 store
//   dL/dW       = G^T (H^T)^T  (K = tokens)   epilogue: fp32 store or accumulate
// G = dL/dz is formed once, in bf16, by an elementwise kernel that also writes G^T; W^T
// and H^T are transposed copies, so every operand of every product is K-contiguous and
// one kernel serves all three.
//
// Kernel shape (gfx950): 512 lanes = 8 wavefronts per workgroup (two per SIMD), one
// 256 x 256 tile of C per workgroup, K in steps of 64.  Each wavefront owns a 128 x 64 part
// as 4 x 2 blocks of v_mfma_f32_32x32x16_bf16 (128 accumulator registers per lane).  Eight
// wavefronts rather than four because one wavefront sustains only about one 16-byte-per-lane
// load every 170 cycles and one ds_read_b128 every 58 (measured, whatever is in flight):
// at four wavefronts the tile's operand loads take longer than its products.  Operand
// tiles go from global memory straight into LDS (global_load_lds_dwordx4, no register
// staging) through a ring of five 32 KB slots, all 160 KB of a CU.  Inside a tile row
// the eight 16-byte chunks are stored at chunk ^ ((row >> 1) & 7), applied on the
// global-address side, so that 16 consecutive rows of one logical chunk (a quarter of a
// ds_read_b128 fragment read) fall on 16 different groups of four banks.

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr int LM_BM = 256, LM_BN = 256, LM_BK = 64;
constexpr int LM_THREADS = 512;                      // 8 wavefronts, two per SIMD
constexpr int LM_WM = 2, LM_WN = 4;                  // wavefront grid over the tile
constexpr int LM_FA = 4, LM_FB = 2;                  // 32 x 32 blocks per wavefront: 128 x 64
constexpr int LM_CPR = LM_BK / 8;                    // 16-byte chunks per tile row: 8
constexpr int LM_TILE_BYTES = LM_BM * LM_BK * 2;     // one operand tile: 32 KB
constexpr int LM_SLOTS = 5;                          // operand tiles resident in LDS: all 160 KB
constexpr int LM_LPT = LM_BM * LM_CPR / LM_THREADS;  // 16-byte loads per lane and operand tile: 4
constexpr int LM_LDS_BYTES = LM_SLOTS * LM_TILE_BYTES;
constexpr int LM_GROUP_M = 8;                        // tile rows that share a sweep along N

enum { LM_EPI_LSE = 0, LM_EPI_BF16 = 1, LM_EPI_F32 = 2 };

struct GemmParams {
    const __bf16 *A;
    const __bf16 *B;
    long long lda, ldb;  // elements; rows 16-byte aligned
    int M, N, K;         // K % LM_BK == 0, K > 0
    int tiles_m, tiles_n;
    // LM_EPI_BF16 / LM_EPI_F32
    void *C;
    long long ldc;
    int accumulate;      // LM_EPI_F32: C += result
    // LM_EPI_LSE
    const long long *tokens;
    const unsigned char *mask;
    float k;             // log2(e) / T
    float *part_m, *part_s;  // [tiles_n][M]: max and sum of exp2(z k - max) over the tile's columns, y left out
    float *zy;               // [M]: the accumulator at the sampled token's column
    float *Z;                // optional fp32 copy of the logits, [M][ldz]
    long long ldz;
};

// Workgroup -> tile.  The hardware deals consecutive workgroups to the 8 XCDs in turn;
// each XCD has its own L2.  Workgroups of one XCD are given a contiguous run of the
// tile order below, and that order walks LM_GROUP_M tile rows down before it moves one
// tile column on, so the tiles in flight on an XCD at any moment share a few A and B
// panels and most operand traffic is served by that XCD's L2.
__device__ __forceinline__ bool lm_map_tile(const GemmParams &p, int &tm, int &tn)
{
    const int total = p.tiles_m * p.tiles_n;
    const int per_xcd = (total + 7) / 8;
    const int L = (int)(blockIdx.x & 7) * per_xcd + (int)(blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || L >= total) return false;
    const int group_tiles = LM_GROUP_M * p.tiles_n;
    const int grp = L / group_tiles;
    const int in_grp = L - grp * group_tiles;
    const int rows_here = min(LM_GROUP_M, p.tiles_m - grp * LM_GROUP_M);
    tm = grp * LM_GROUP_M + in_grp % rows_here;
    tn = in_grp / rows_here;
    return true;
}

template <int CTRL>
__device__ __forceinline__ float lm_dpp(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf,
                                                                   0xf, true));
}
// Reductions over the 32 lanes that hold one row of a 32 x 32 accumulator block: quad
// swaps, mirror inside 8, mirror inside 16 (all DPP), then the other 16 lanes.
__device__ __forceinline__ float lm_row32_max(float v)
{
    v = fmaxf(v, lm_dpp<0xB1>(v));
    v = fmaxf(v, lm_dpp<0x4E>(v));
    v = fmaxf(v, lm_dpp<0x141>(v));
    v = fmaxf(v, lm_dpp<0x140>(v));
    return fmaxf(v, __shfl_xor(v, 16, 64));
}
__device__ __forceinline__ float lm_row32_sum(float v)
{
    v += lm_dpp<0xB1>(v);
    v += lm_dpp<0x4E>(v);
    v += lm_dpp<0x141>(v);
    v += lm_dpp<0x140>(v);
    return v + __shfl_xor(v, 16, 64);
}

template <int EPI, bool STORE_Z>
__global__ void __launch_bounds__(LM_THREADS) lm_gemm_nt(GemmParams p)
{
    extern __shared__ __attribute__((aligned(1024))) char lm_smem[];
    int tm, tn;
    if (!lm_map_tile(p, tm, tn)) return;  // whole workgroup alike, before any barrier

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / LM_WN, wn = wave % LM_WN;  // this wavefront's 128 x 64 part of the tile
    const int row0 = tm * LM_BM, col0 = tn * LM_BN;

    // Byte offsets of this lane's four 16-byte loads per operand tile, relative to the
    // tile's first row at k = 0.  Load i of a wavefront fills LDS chunks [i*512 + wave*64,
    // +64) of the tile; chunk c sits in tile row c / 8 at physical position c % 8 and holds
    // logical chunk (c % 8) ^ ((row >> 1) & 7).  Rows past the end of the matrix re-read the
    // last row (their results are never stored).
    unsigned a_off[LM_LPT], b_off[LM_LPT];
#pragma unroll
    for (int i = 0; i < LM_LPT; ++i) {
        const int c = i * LM_THREADS + tid;
        const int r = c / LM_CPR, pc = c % LM_CPR;
        const int lc = pc ^ ((r >> 1) & (LM_CPR - 1));
        const int ra = min(row0 + r, p.M - 1) - row0;
        const int rb = min(col0 + r, p.N - 1) - col0;
        a_off[i] = (unsigned)(((long long)ra * p.lda + lc * 8) * 2);
        b_off[i] = (unsigned)(((long long)rb * p.ldb + lc * 8) * 2);
    }
    const char *a_tile = (const char *)p.A + (long long)row0 * p.lda * 2;
    const char *b_tile = (const char *)p.B + (long long)col0 * p.ldb * 2;
    const int KT = p.K / LM_BK;

    // LDS is a ring of five 32 KB slots that operand tiles pass through in the order
    // A(0), B(0), A(1), B(1), ...: entry q = 2 kt + (0 for A, 1 for B) lives in slot q % 5.
    // Two slots hold the tile being multiplied, the other three the next loads, which are
    // issued two at a time between the products.  Past the last tile the last one is loaded
    // again, into a slot nobody reads any more: every iteration then issues the same number
    // of loads and "landed" is a fixed vmcnt value.
    auto slot_of = [&](int q) { return lm_smem + (q % LM_SLOTS) * LM_TILE_BYTES; };
    auto issue_half = [&](int q, bool b_operand, int half) {
        const long long k0 = (long long)min(q >> 1, KT - 1) * (LM_BK * 2);
        char *sd = slot_of(q) + wave * 1024;
        const char *src = (b_operand ? b_tile : a_tile) + k0;
#pragma unroll
        for (int i = half * (LM_LPT / 2); i < (half + 1) * (LM_LPT / 2); ++i)
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void *)(src + (b_operand ? b_off[i] : a_off[i])),
                (__attribute__((address_space(3))) void *)(sd + i * (LM_THREADS * 16)), 16, 0, 0);
    };

    // Fragment addresses: lane (r = lane % 32, half = lane / 32) reads, for k-step ks, the
    // logical chunk 2 ks + half of tile row (block row) + r.
    const int fr = lane & 31, fh = lane >> 5;
    unsigned frag_off[LM_BK / 16];
#pragma unroll
    for (int ks = 0; ks < LM_BK / 16; ++ks)
        frag_off[ks] = (unsigned)((fr * LM_CPR + ((2 * ks + fh) ^ ((fr >> 1) & (LM_CPR - 1)))) * 16);
    const unsigned a_wave = (unsigned)(wm * (LM_FA * 32) * LM_BK * 2);
    const unsigned b_wave = (unsigned)(wn * (LM_FB * 32) * LM_BK * 2);

    f32x16 acc[LM_FA][LM_FB];
#pragma unroll
    for (int i = 0; i < LM_FA; ++i)
#pragma unroll
        for (int j = 0; j < LM_FB; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // Fragments are double buffered in registers (F[0], F[1]) and read one k-step ahead of
    // the products that use them.  One barrier per tile, before its last k-step: by then
    // every wavefront holds that k-step's fragments in registers, so the tile's two slots
    // are free, and everybody's loads of the next tile have landed.
    bf16x8 F[2][LM_FA + LM_FB];
    auto read_frags = [&](bf16x8 (&f)[LM_FA + LM_FB], int kt, int ks) {
        const char *sa = slot_of(2 * kt), *sb = slot_of(2 * kt + 1);
#pragma unroll
        for (int i = 0; i < LM_FA; ++i)
            f[i] = *(const bf16x8 *)(sa + a_wave + i * (32 * LM_BK * 2) + frag_off[ks]);
#pragma unroll
        for (int j = 0; j < LM_FB; ++j)
            f[LM_FA + j] = *(const bf16x8 *)(sb + b_wave + j * (32 * LM_BK * 2) + frag_off[ks]);
    };
    auto products = [&](const bf16x8 (&f)[LM_FA + LM_FB]) {
#pragma unroll
        for (int i = 0; i < LM_FA; ++i)
#pragma unroll
            for (int j = 0; j < LM_FB; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i], f[LM_FA + j], acc[i][j], 0, 0, 0);
    };
    // one k-step: 6 LDS reads, 8 products, 2 global -> LDS loads: a read with each of the
    // first six products, then the two loads after a product each
    auto interleave = [&]() {
#pragma unroll
        for (int i = 0; i < LM_FA + LM_FB; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
#pragma unroll
        for (int i = 0; i < LM_LPT / 2; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    static_assert(LM_BK / 16 == 4 && LM_SLOTS == 5 && LM_LPT == 4 && LM_FA * LM_FB >= LM_FA + LM_FB + LM_LPT / 2,
                  "the pipeline and its wait counts are written for 4 k-steps, 5 slots, 4 loads per operand tile");

    // Memory loads return in order, so "at most n outstanding" means that everything older
    // than the n youngest loads is in LDS.  The wait, the wait for the own LDS reads and the
    // workgroup barrier are one asm statement so that nothing is scheduled in between.
    issue_half(0, false, 0);
    issue_half(0, false, 1);
    issue_half(1, true, 0);
    issue_half(1, true, 1);
    issue_half(2, false, 0);
    issue_half(2, false, 1);
    issue_half(3, true, 0);
    asm volatile("s_waitcnt vmcnt(6) lgkmcnt(0)\n\ts_barrier" ::: "memory");  // A(0), B(0) are there
    read_frags(F[0], 0, 0);
    for (int kt = 0; kt < KT; ++kt) {
        read_frags(F[1], kt, 1);
        products(F[0]);
        issue_half(2 * kt + 3, true, 1);   // rest of B(kt + 1)
        interleave();
        read_frags(F[0], kt, 2);
        products(F[1]);
        issue_half(2 * kt + 4, false, 0);  // A(kt + 2)
        interleave();
        read_frags(F[1], kt, 3);
        products(F[0]);
        issue_half(2 * kt + 4, false, 1);
        interleave();
        // outstanding, oldest first: ..., B(kt + 1), A(kt + 2): 4 left = tile kt + 1 landed
        asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        read_frags(F[0], kt + 1, 0);
        products(F[1]);
        issue_half(2 * kt + 5, true, 0);   // B(kt + 2) into the slot A(kt) just left
        interleave();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

    // Accumulator layout of a 32 x 32 block: lane l holds column l % 32; register v holds
    // row 8 (v / 4) + 4 (l / 32) + v % 4.
    const int cl = lane & 31, g = lane >> 5;
    const int wrow = wm * (LM_FA * 32), wcol = wn * (LM_FB * 32);
    if (EPI == LM_EPI_BF16 || EPI == LM_EPI_F32) {
#pragma unroll
        for (int i = 0; i < LM_FA; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + wrow + i * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                if (row >= p.M) continue;
#pragma unroll
                for (int j = 0; j < LM_FB; ++j) {
                    const int col = col0 + wcol + j * 32 + cl;
                    if (col >= p.N) continue;
                    if (EPI == LM_EPI_BF16) {
                        ((__bf16 *)p.C)[(long long)row * p.ldc + col] = (__bf16)acc[i][j][v];
                    } else {
                        float *c = (float *)p.C + (long long)row * p.ldc + col;
                        *c = p.accumulate ? *c + acc[i][j][v] : acc[i][j][v];
                    }
                }
            }
        return;
    }

    // Softmax partials of this tile: for every row the maximum of z k over the tile's
    // columns and the sum of exp2(z k - max), the sampled token's column left out of both
    // (its accumulator goes to zy instead) so that 1 - p_y keeps its precision later.
    __syncthreads();  // the operand slots are free now: reuse their start as scratch
    float *red_m = (float *)lm_smem;  // [LM_WN][256]
    float *red_s = red_m + LM_WN * LM_BM;
    int *ycol_s = (int *)(red_s + LM_WN * LM_BM);
    if (tid < LM_BM) {
        // column of the sampled token inside this tile, -1 when it is elsewhere or the row
        // takes no part
        const int r = row0 + tid;
        int yc = -1;
        if (r < p.M && (!p.mask || p.mask[r])) {
            const long long y = p.tokens[r];
            if (y >= col0 && y < (long long)col0 + LM_BN && y < p.N) yc = (int)(y - col0);
        }
        ycol_s[tid] = yc;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < LM_FA; ++i)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int rl0 = wrow + i * 32 + q * 8 + g * 4;
            const i32x4 yv = *(const i32x4 *)(ycol_s + rl0);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int rl = rl0 + e;
                const int row = row0 + rl;
                float a[LM_FB];
#pragma unroll
                for (int j = 0; j < LM_FB; ++j) {
                    const int cloc = wcol + j * 32 + cl;
                    const float z = acc[i][j][q * 4 + e];
                    const bool in = col0 + cloc < p.N;
                    if (STORE_Z && in && row < p.M) p.Z[(long long)row * p.ldz + col0 + cloc] = z;
                    const bool is_y = cloc == yv[e];
                    if (is_y) p.zy[row] = z;
                    a[j] = (is_y || !in) ? -INFINITY : z * p.k;
                }
                float m = a[0];
#pragma unroll
                for (int j = 1; j < LM_FB; ++j) m = fmaxf(m, a[j]);
                m = lm_row32_max(m);
                const float ref = m == -INFINITY ? 0.f : m;  // a row of the tile with nothing to sum
                float s = 0.f;
#pragma unroll
                for (int j = 0; j < LM_FB; ++j) s += __builtin_amdgcn_exp2f(a[j] - ref);
                s = lm_row32_sum(s);
                if (cl == 0) {
                    red_m[wn * LM_BM + rl] = m;
                    red_s[wn * LM_BM + rl] = s;
                }
            }
        }
    __syncthreads();
    if (tid < LM_BM) {
        const int row = row0 + tid;
        if (row < p.M) {
            float m = -INFINITY;
#pragma unroll
            for (int w = 0; w < LM_WN; ++w) m = fmaxf(m, red_m[w * LM_BM + tid]);
            float s = 0.f;
#pragma unroll
            for (int w = 0; w < LM_WN; ++w) {
                const float mw = red_m[w * LM_BM + tid];
                if (mw != -INFINITY) s += red_s[w * LM_BM + tid] * __builtin_amdgcn_exp2f(mw - m);
            }
            p.part_m[(long long)tn * p.M + row] = m;
            p.part_s[(long long)tn * p.M + row] = s;
        }
    }
}

// Per-row arrays the fused path keeps between its kernels.
struct LmRows {
    float *zy;     // logit of the sampled token (fp32 accumulator)
    float *shift;  // max k + log2(sum): p_j = exp2(z_j k - shift)
    float *q;      // c / T, 0 for rows without gradient
    float *gy;     // gradient at the sampled token: q (1 - p_y), from the sum without y
    float *part_m, *part_s;
    int tiles_n;
};

// Merges the tile partials of each row, then the objective's once-per-row arithmetic.
__global__ void __launch_bounds__(256) lm_combine(RowParams p, LmRows w)
{
    const long long row = (long long)blockIdx.x * 256 + threadIdx.x;
    if (row >= p.n_tokens) return;
    bool live = p.mask ? (p.mask[row] != 0) : true;
    bool bad = false;
    if (live) {
        const long long y = p.tokens[row];
        if (y < 0 || y >= p.vocab) {
            live = false;
            bad = true;
        }
    }
    if (!live) {
        write_row_outputs(p, row, (bad && !p.bwd) ? NAN : 0.f, 0.f, 0);
        if (bad && p.bwd) atomicOr(&p.hdr->error, 1);
        if (p.bwd) {
            w.q[row] = 0.f;
            w.gy[row] = 0.f;
            w.shift[row] = 0.f;
        }
        return;
    }
    float m = -INFINITY;
    for (int t = 0; t < w.tiles_n; ++t) m = fmaxf(m, w.part_m[(long long)t * p.n_tokens + row]);
    const float zy = w.zy[row];
    const float mk = fmaxf(m, zy * p.k);  // the sampled token may be the row's maximum
    float s_excl = 0.f;
    for (int t = 0; t < w.tiles_n; ++t) {
        const float mt = w.part_m[(long long)t * p.n_tokens + row];
        if (mt != -INFINITY)
            s_excl += w.part_s[(long long)t * p.n_tokens + row] * __builtin_amdgcn_exp2f(mt - mk);
    }
    const RowScalars o = row_scalars(p, row, zy, mk, s_excl);
    write_row_outputs(p, row, o.logp, o.J, o.flags);
    if (p.bwd) {
        const float q = o.c * p.inv_T;
        w.q[row] = q;
        w.gy[row] = q * (o.s_excl / o.s);
        w.shift[row] = o.shift;
    }
}

// G = dL/dz in bf16, row-major [M][ldg] and transposed [V][ldgt], from the fp32 logits:
// g_j = -q p_j, g_y = q (1 - p_y).  64 x 64 tiles; padding columns of both (up to ldg,
// ldgt) are written as zeros so that the products can run over whole K steps.
__global__ void __launch_bounds__(256) lm_grad_logits(const float *Z, long long ldz, int M, int V,
                                                      const long long *tokens, LmRows w, float k,
                                                      __bf16 *G, long long ldg, __bf16 *Gt,
                                                      long long ldgt)
{
    __shared__ float tile[64][65];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;  // 64 columns x 4 rows per pass
#pragma unroll 4
    for (int i = 0; i < 16; ++i) {
        const int r = r0 + ty + 4 * i, c = c0 + tx;
        float gv = 0.f;
        if (r < M && c < V) {
            const float q = w.q[r];
            if (q != 0.f) {
                const long long y = tokens[r];
                gv = c == y ? w.gy[r]
                            : -q * __builtin_amdgcn_exp2f(fmaf(Z[(long long)r * ldz + c], k, -w.shift[r]));
            }
        }
        if (r < M && c < ldg) G[(long long)r * ldg + c] = (__bf16)gv;
        tile[ty + 4 * i][tx] = gv;
    }
    __syncthreads();
#pragma unroll 4
    for (int i = 0; i < 16; ++i) {
        const int c = c0 + ty + 4 * i, r = r0 + tx;
        if (c < V && r < ldgt) Gt[(long long)c * ldgt + r] = (__bf16)tile[tx][ty + 4 * i];
    }
}

// out[c][r] = in[r][c] for r < R, c < C; columns R .. ldo of out are zero-filled.
__global__ void __launch_bounds__(256) lm_transpose(const __bf16 *in, long long ldi, int R, int C,
                                                    __bf16 *out, long long ldo)
{
    __shared__ unsigned short tile[64][66];
    const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const unsigned short *src = (const unsigned short *)in;
    unsigned short *dst = (unsigned short *)out;
#pragma unroll 4
    for (int i = 0; i < 16; ++i) {
        const int r = r0 + ty + 4 * i, c = c0 + tx;
        tile[ty + 4 * i][tx] = (r < R && c < C) ? src[(long long)r * ldi + c] : (unsigned short)0;
    }
    __syncthreads();
#pragma unroll 4
    for (int i = 0; i < 16; ++i) {
        const int c = c0 + ty + 4 * i, r = r0 + tx;
        if (c < C && r < ldo) dst[(long long)c * ldo + r] = tile[tx][ty + 4 * i];
    }
}

// rows x cols zeros into a row-strided fp32 matrix (a fill kernel rather than a memset, so
// that the call can be captured into a graph)
__global__ void __launch_bounds__(256) lm_zero_f32(float *out, long long rows, long long cols, long long ld)
{
    const long long total = rows * cols;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256)
        out[(i / cols) * ld + i % cols] = 0.f;
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------

template <int EPI, bool STORE_Z>
hipError_t lm_launch_gemm(GemmParams p, hipStream_t st)
{
    static bool attr_done[64] = {false};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !attr_done[dev]) {
        e = hipFuncSetAttribute((const void *)lm_gemm_nt<EPI, STORE_Z>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, LM_LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done[dev] = true;
    }
    p.tiles_m = (p.M + LM_BM - 1) / LM_BM;
    p.tiles_n = (p.N + LM_BN - 1) / LM_BN;
    const long long total = (long long)p.tiles_m * p.tiles_n;
    const long long grid = (total + 7) / 8 * 8;
    hipLaunchKernelGGL((lm_gemm_nt<EPI, STORE_Z>), dim3((unsigned)grid), dim3(LM_THREADS), LM_LDS_BYTES, st, p);
    return hipGetLastError();
}

struct LmLayout {
    size_t rows_bytes;  // the objective's own workspace (header, J, flags, ...)
    size_t zy, shift, q, gy, part_m, part_s, Z, G, Gt, Wt, Ht, total;
    long long ldz, ldg, ldgt;  // vocab and token counts rounded up to whole K steps
    int tiles_n;
};

LmLayout lm_layout(int64_t n, int64_t V, int64_t d, bool bwd)
{
    LmLayout L = {};
    L.tiles_n = (int)((V + LM_BN - 1) / LM_BN);
    L.ldz = L.ldg = (long long)align_up((size_t)V, 64);  // whole K steps, 128-byte rows
    L.ldgt = (long long)align_up((size_t)n, 64);
    size_t off = align_up(grpo_workspace_bytes(n), 256);
    L.rows_bytes = off;
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += align_up(bytes, 256);
        return at;
    };
    L.zy = take((size_t)n * 4);
    L.part_m = take((size_t)L.tiles_n * n * 4);
    L.part_s = take((size_t)L.tiles_n * n * 4);
    if (bwd) {
        L.shift = take((size_t)n * 4);
        L.q = take((size_t)n * 4);
        L.gy = take((size_t)n * 4);
        L.Z = take((size_t)n * L.ldz * 4);
        L.G = take((size_t)n * L.ldg * 2);
        L.Gt = take((size_t)V * L.ldgt * 2);
        L.Wt = take((size_t)d * L.ldg * 2);
        L.Ht = take((size_t)d * L.ldgt * 2);
    }
    L.total = off;
    return L;
}

grpo_status lm_check_common(const void *hidden, int64_t hidden_stride, const void *weight,
                            int64_t weight_stride, int64_t n_tokens, int64_t vocab, int64_t d_model,
                            const int64_t *tokens, float temperature)
{
    if (n_tokens < 0 || n_tokens > 0x7fffff00ll || vocab <= 0 || vocab > kMaxVocab || d_model <= 0 ||
        d_model > (1 << 20) || d_model % LM_BK != 0 || hidden_stride < d_model || weight_stride < d_model)
        return GRPO_ERR_SHAPE;
    if (!(temperature > 0.f) || !std::isfinite(temperature)) return GRPO_ERR_PARAM;
    if (n_tokens == 0) return GRPO_OK;
    if (!hidden || !weight || !tokens) return GRPO_ERR_NULL;
    if (((uintptr_t)hidden & 15u) || ((uintptr_t)weight & 15u) || ((hidden_stride * 2) & 15) ||
        ((weight_stride * 2) & 15))
        return GRPO_ERR_ALIGN;
    // byte offsets inside one 256-row operand tile must fit 32 bits
    if (hidden_stride * 2 * LM_BM >= (1ll << 32) || weight_stride * 2 * LM_BN >= (1ll << 32))
        return GRPO_ERR_SHAPE;
    return GRPO_OK;
}

grpo_status lm_impl(bool bwd, const void *hidden, int64_t hidden_stride, const void *weight,
                    int64_t weight_stride, int64_t n_tokens, int64_t vocab, int64_t d_model,
                    const int64_t *tokens, const float *old_logprobs, const float *advantages,
                    const uint8_t *mask, float eps_low, float eps_high, float delta, float temperature,
                    double denom, float grad_scale, float *loss_out, float *logprobs_out,
                    int64_t *counts_out, void *grad_hidden, int64_t grad_hidden_stride,
                    float *grad_weight, int64_t grad_weight_stride, int accumulate_grad_weight,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    grpo_status rc = lm_check_common(hidden, hidden_stride, weight, weight_stride, n_tokens, vocab,
                                     d_model, tokens, temperature);
    if (rc != GRPO_OK) return rc;
    if (bwd) {
        if (!(eps_low >= 0.f && eps_low <= 1.f) || !(eps_high >= 0.f) || !std::isfinite(eps_high) ||
            !(delta > 1.f + eps_high) || std::isnan(denom) || std::isnan(grad_scale))
            return GRPO_ERR_PARAM;
        if (!loss_out) return GRPO_ERR_NULL;
        if (n_tokens > 0 && (!old_logprobs || !advantages || !grad_hidden)) return GRPO_ERR_NULL;
        if (!grad_weight) return GRPO_ERR_NULL;
        if (grad_hidden_stride < d_model || grad_weight_stride < d_model) return GRPO_ERR_SHAPE;
    } else {
        if (n_tokens == 0) return GRPO_OK;
        if (!logprobs_out) return GRPO_ERR_NULL;
    }
    const LmLayout L = lm_layout(n_tokens, vocab, d_model, bwd);
    if (!workspace || ((uintptr_t)workspace & 255u) != 0 || workspace_bytes < L.total)
        return GRPO_ERR_WORKSPACE;

    char *ws = (char *)workspace;
    hipStream_t st = (hipStream_t)stream;
    const size_t col = align_up((size_t)n_tokens * 4, 256);
    WsHeader *hdr = (WsHeader *)ws;
    float *J_ws = (float *)(ws + kHeaderBytes);
    float *H_ws = (float *)(ws + kHeaderBytes + 2 * col);
    unsigned char *flags_ws = (unsigned char *)(ws + kHeaderBytes + 3 * col);

    if (bwd)
        hipLaunchKernelGGL(grpo_prepare, dim3(1), dim3(1024), 0, st, mask, (const float *)nullptr,
                           (long long)n_tokens, denom, hdr);
    if (n_tokens > 0) {
        LmRows w = {};
        w.zy = (float *)(ws + L.zy);
        w.part_m = (float *)(ws + L.part_m);
        w.part_s = (float *)(ws + L.part_s);
        w.tiles_n = L.tiles_n;
        if (bwd) {
            w.shift = (float *)(ws + L.shift);
            w.q = (float *)(ws + L.q);
            w.gy = (float *)(ws + L.gy);
        }
        const float k = (float)((double)kLog2e / (double)temperature);

        GemmParams g = {};
        g.A = (const __bf16 *)hidden;
        g.lda = hidden_stride;
        g.B = (const __bf16 *)weight;
        g.ldb = weight_stride;
        g.M = (int)n_tokens;
        g.N = (int)vocab;
        g.K = (int)d_model;
        g.tokens = (const long long *)tokens;
        g.mask = mask;
        g.k = k;
        g.part_m = w.part_m;
        g.part_s = w.part_s;
        g.zy = w.zy;
        g.Z = bwd ? (float *)(ws + L.Z) : nullptr;
        g.ldz = L.ldz;
        hipError_t e = bwd ? lm_launch_gemm<LM_EPI_LSE, true>(g, st) : lm_launch_gemm<LM_EPI_LSE, false>(g, st);
        if (e != hipSuccess) return GRPO_ERR_HIP;

        RowParams p = {};
        p.tokens = (const long long *)tokens;
        p.old_lp = old_logprobs;
        p.adv = advantages;
        p.mask = mask;
        p.logprobs_out = logprobs_out;
        p.J_ws = J_ws;
        p.flags_ws = flags_ws;
        p.hdr = hdr;
        p.n_tokens = n_tokens;
        p.vocab = vocab;
        p.inv_T = 1.0f / temperature;
        p.k = k;
        p.lo = 1.0f - eps_low;
        p.hi = 1.0f + eps_high;
        p.delta = delta;
        p.grad_scale = grad_scale;
        p.bwd = bwd ? 1 : 0;
        hipLaunchKernelGGL(lm_combine, dim3((unsigned)((n_tokens + 255) / 256)), dim3(256), 0, st, p, w);

        if (bwd) {
            __bf16 *G = (__bf16 *)(ws + L.G), *Gt = (__bf16 *)(ws + L.Gt);
            __bf16 *Wt = (__bf16 *)(ws + L.Wt), *Ht = (__bf16 *)(ws + L.Ht);
            const int M = (int)n_tokens, V = (int)vocab, D = (int)d_model;
            hipLaunchKernelGGL(lm_grad_logits, dim3((unsigned)(L.ldg / 64), (unsigned)(L.ldgt / 64)), dim3(256),
                               0, st, (const float *)(ws + L.Z), L.ldz, M, V, (const long long *)tokens, w, k,
                               G, L.ldg, Gt, L.ldgt);
            // W^T [d][ldg] and H^T [d][ldgt]
            hipLaunchKernelGGL(lm_transpose, dim3((unsigned)((D + 63) / 64), (unsigned)(L.ldg / 64)), dim3(256), 0, st,
                               (const __bf16 *)weight, (long long)weight_stride, V, D, Wt, L.ldg);
            hipLaunchKernelGGL(lm_transpose, dim3((unsigned)((D + 63) / 64), (unsigned)(L.ldgt / 64)), dim3(256), 0, st,
                               (const __bf16 *)hidden, (long long)hidden_stride, M, D, Ht, L.ldgt);

            GemmParams gh = {};  // dL/dH [M][d] = G [M][V] . W [V][d]
            gh.A = G;
            gh.lda = L.ldg;
            gh.B = Wt;
            gh.ldb = L.ldg;
            gh.M = M;
            gh.N = D;
            gh.K = (int)L.ldg;
            gh.C = grad_hidden;
            gh.ldc = grad_hidden_stride;
            e = lm_launch_gemm<LM_EPI_BF16, false>(gh, st);
            if (e != hipSuccess) return GRPO_ERR_HIP;

            GemmParams gw = {};  // dL/dW [V][d] = G^T [V][M] . H [M][d]
            gw.A = Gt;
            gw.lda = L.ldgt;
            gw.B = Ht;
            gw.ldb = L.ldgt;
            gw.M = V;
            gw.N = D;
            gw.K = (int)L.ldgt;
            gw.C = grad_weight;
            gw.ldc = grad_weight_stride;
            gw.accumulate = accumulate_grad_weight ? 1 : 0;
            e = lm_launch_gemm<LM_EPI_F32, false>(gw, st);
            if (e != hipSuccess) return GRPO_ERR_HIP;
        }
    } else if (bwd && !accumulate_grad_weight && vocab > 0) {
        // no tokens: the weight gradient is zero
        hipLaunchKernelGGL(lm_zero_f32, dim3(4096), dim3(256), 0, st, grad_weight, (long long)vocab,
                           (long long)d_model, (long long)grad_weight_stride);
    }
    if (bwd)
        hipLaunchKernelGGL(grpo_finalize, dim3(1), dim3(1024), 0, st, J_ws, (const float *)nullptr, H_ws,
                           flags_ws, (long long)n_tokens, hdr, 0.f, 0.f, loss_out, (long long *)counts_out);
    return hipGetLastError() == hipSuccess ? GRPO_OK : GRPO_ERR_HIP;
}

}  // namespace

extern "C" {

size_t grpo_lmhead_workspace_bytes(int64_t n_tokens, int64_t vocab, int64_t d_model, int with_backward)
{
    if (n_tokens < 0 || vocab <= 0 || d_model <= 0) return 0;
    return lm_layout(n_tokens, vocab, d_model, with_backward != 0).total;
}

grpo_status grpo_lmhead_logprobs_fwd(const void *hidden, int64_t hidden_stride, const void *weight,
                                     int64_t weight_stride, int64_t n_tokens, int64_t vocab,
                                     int64_t d_model, const int64_t *tokens, const uint8_t *mask,
                                     float temperature, float *logprobs_out, void *workspace,
                                     size_t workspace_bytes, void *stream)
{
    return lm_impl(false, hidden, hidden_stride, weight, weight_stride, n_tokens, vocab, d_model, tokens,
                   nullptr, nullptr, mask, 0.f, 0.f, 0.f, temperature, 0.0, 0.f, nullptr, logprobs_out,
                   nullptr, nullptr, 0, nullptr, 0, 0, workspace, workspace_bytes, stream);
}

grpo_status grpo_lmhead_loss_fwd_bwd(const void *hidden, int64_t hidden_stride, const void *weight,
                                     int64_t weight_stride, int64_t n_tokens, int64_t vocab,
                                     int64_t d_model, const int64_t *tokens, const float *old_logprobs,
                                     const float *advantages, const uint8_t *mask, float eps_low,
                                     float eps_high, float delta, float temperature, double denom,
                                     float grad_scale, float *loss_out, float *logprobs_out,
                                     int64_t *counts_out, void *grad_hidden, int64_t grad_hidden_stride,
                                     float *grad_weight, int64_t grad_weight_stride,
                                     int accumulate_grad_weight, void *workspace, size_t workspace_bytes,
                                     void *stream)
{
    return lm_impl(true, hidden, hidden_stride, weight, weight_stride, n_tokens, vocab, d_model, tokens,
                   old_logprobs, advantages, mask, eps_low, eps_high, delta, temperature, denom, grad_scale,
                   loss_out, logprobs_out, counts_out, grad_hidden, grad_hidden_stride, grad_weight,
                   grad_weight_stride, accumulate_grad_weight, workspace, workspace_bytes, stream);
}

}  // extern "C"
