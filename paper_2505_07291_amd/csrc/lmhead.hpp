// Language-model head fused with the GRPO objective: the logits z = h W^T of the policy of
// section 3.4 are produced, reduced and differentiated here instead of being handed in.
// This file is the second half of grpo.hip's translation unit (it is included at its end
// and uses the row arithmetic, the workspace header and the small kernels defined there).
//
// Everything heavy is one bf16 MFMA kernel, lm_gemm_nt: C[M x N] = A[M x K] B[N x K]^T with
// fp32 accumulation.  An operand is either contiguous along K ([M][K], the plain case) or
// "K-major" ([K][M], read from LDS with the transposing reads of gfx950).  It runs three times:
//   logits   z  = H W^T        (K = d_model)  A = H, B = W, both plain
//                                             epilogue: per-row softmax partials in fp32
//                                             from the accumulators, z_y, optional fp32 z
//   dL/dH       = G W          (K = vocab)    A = G plain, B = W K-major; epilogue: bf16 store
//   dL/dW       = G^T H        (K = tokens)   A = G K-major, B = H^T plain; epilogue: fp32 store
//                                             or accumulate
// G = dL/dz is formed once, in bf16, by an elementwise kernel and serves both gradient
// products as it lies; W is never copied; H^T (the chunk's gradient rows, [d][rows]) is the
// one transposed copy, 1/30 of G's size.
//
// The backward works through the rows that take part in chunks of at most `cap` rows (a
// multiple of 256 chosen from the size of the caller's workspace): logits, G and H^T
// exist for one chunk at a time, dL/dH rows of different chunks are disjoint and dL/dW is
// accumulated in fp32 from chunk to chunk.  The workspace is therefore bounded by the
// chunk, not by the number of tokens.  The live rows are dealt evenly over the chunks
// that are needed (lm_chunk_range, computed on the device from the live count), so no
// chunk is a small remainder.
//
// Kernel shape (gfx950): 512 lanes = 8 wavefronts per workgroup (two per SIMD), one
// 256 x 256 tile of C per workgroup, K in steps of 64.  Each wavefront owns a 128 x 64 part
// as 4 x 2 blocks of v_mfma_f32_32x32x16_bf16 (128 accumulator registers per lane).  Eight
// wavefronts rather than four because one wavefront sustains only about one 16-byte-per-lane
// load every 170 cycles and one ds_read_b128 every 58 (measured, whatever is in flight):
// at four wavefronts the tile's operand loads take longer than its products.  Operand
// tiles go from global memory straight into LDS (buffer_load_dwordx4 ... lds, no register
// staging, no vector address arithmetic) through a ring of five 32 KB slots, all 160 KB of a
// CU.  Inside a tile row the eight 16-byte chunks are stored at chunk ^ ((row >> 1) & 7),
// applied on the global-address side, so that 16 consecutive rows of one logical chunk (a
// quarter of a ds_read_b128 fragment read) fall on 16 different groups of four banks.
// After the last K step the same LDS serves the epilogue: the accumulators are turned round
// through it so that the per-row softmax partials are plain loops, one row per lane.

#include <algorithm>

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
constexpr int LM_GM_BWD = 4;                         // the same for the two gradient products: their A panels (of G)
                                                     // come from HBM, and a lower group re-reads them less often
constexpr int LM_SPLIT_MAX = 32;                     // parts the contraction of one tile of dL/dH may be cut into

enum { LM_EPI_LSE = 0, LM_EPI_BF16 = 1, LM_EPI_F32 = 2 };

struct GemmParams {
    const __bf16 *A;
    const __bf16 *B;
    long long lda, ldb;  // elements; rows 16-byte aligned
    int M, N, K;         // host-side sizes: M and K are upper bounds when the device values below are given
    const int *M_dev;    // optional: number of rows of A actually present (<= M)
    int chunk, chunk_cap;  // chunk_cap > 0: *M_dev counts the rows of ALL chunks and this launch works on chunk
                           // number `chunk` of them (lm_chunk_range): A, tokens32 and zy start at the
                           // chunk's first row, the partials and Z are the chunk's own
    const int *K_dev;    // optional: length of the contraction actually present, rounded up to LM_BK
                         // in the kernel (the padding must hold zeros); 0 gives a zero result
    int tiles_n;
    int group_m;         // tile rows that share a sweep along N (0: LM_GROUP_M)
    // LM_EPI_BF16 / LM_EPI_F32
    void *C;
    long long ldc;
    const int *c_rows;   // LM_EPI_BF16, optional: row i of the result goes to row c_rows[i] of C
    // LM_EPI_BF16, optional split of the contraction (split_items > 0): the tiles that do not fill
    // a whole round of the CUs are cut into parts along K (lm_plan_split, from the live tile count);
    // part s of the t-th such tile goes as a 256 x 256 fp32 block to split_ws[t * parts + s] and
    // lm_split_reduce finishes.  split_items: how many such blocks split_ws holds.
    int split_items, n_cu;
    float *split_ws;
    int accumulate;      // LM_EPI_F32: C += result
    // LM_EPI_LSE
    const int *tokens32; // [M]: sampled token of each row of A
    float k;             // log2(e) / T
    float *part_m, *part_s;  // [tiles_n][part_stride]: max of z over the tile's columns and sum of exp2((z - max) k), y left out
    float *part_w;           // with the auxiliary terms: sum of exp2(a) a, a = (z - max) k, over the same columns
    long long part_stride;
    float *zy;               // [M]: the accumulator at the sampled token's column
    float *Z;                // optional fp32 copy of the logits, [M][ldz]
    long long ldz;
    // K-major operands (AKM / BKM: stored [K][M] resp. [K][N], contiguous along M resp. N, lda / ldb between
    // k rows): how many elements of a k row exist (a multiple of 8; chunks past them re-read the last one)
    int a_cols, b_cols;
    // K-major B: how many k rows exist when that is fewer than K (0: all of them).  The rows past them read
    // as zeros: the buffer descriptor of the last K step ends with the last row that exists, and a load
    // past a descriptor's end puts zeros into LDS (measured on gfx950).
    int b_rows;
};

// Which of n_live rows chunk number `chunk` covers when no chunk may hold more than cap rows
// (cap a multiple of 256): the fewest chunks that can hold them, each of the same size rounded
// up to whole 256-row tiles.  Chunks beyond those are empty (count 0).
__host__ __device__ inline void lm_chunk_range(int n_live, int cap, int chunk, int &base, int &count)
{
    const int needed = (n_live + cap - 1) / cap;
    if (chunk >= needed) {
        base = n_live;
        count = 0;
        return;
    }
    const int per = ((n_live + needed - 1) / needed + 255) / 256 * 256;  // <= cap
    base = chunk * per;  // < n_live: (needed - 1) cap < n_live and per <= cap
    count = n_live - base < per ? n_live - base : per;
}

// Workgroup -> tile.  The hardware deals consecutive workgroups to the 8 XCDs in turn;
// each XCD has its own L2.  Workgroups of one XCD are given a contiguous run of the
// tile order below, and that order walks LM_GROUP_M tile rows down before it moves one
// tile column on, so the tiles in flight on an XCD at any moment share a few A and B
// panels and most operand traffic is served by that XCD's L2.  The number of tile rows
// comes from the device-side row count, so that the live tiles are spread over all XCDs
// whatever part of the launched grid they are.
__device__ __forceinline__ void lm_tile_of(int L, int tiles_m, int tiles_n, int group_m, int &tm, int &tn)
{
    const int group_tiles = group_m * tiles_n;
    const int grp = L / group_tiles;
    const int in_grp = L - grp * group_tiles;
    const int rows_here = min(group_m, tiles_m - grp * group_m);
    tm = grp * group_m + in_grp % rows_here;
    tn = in_grp / rows_here;
}

// A product whose tiles do not fill whole rounds of the CUs (780 tiles on 256 CUs: three rounds
// and twelve tiles) would run its last round on a few CUs, each for a whole tile's time.  The
// first `full` tiles of the order above (whole rounds) are therefore computed as they are, and
// each of the `rest` that remain is cut into s2 parts along the contraction, so that the last
// round is s2 times shorter and spread over all CUs: s2 minimises the rounds of parts, counted in
// tile times, with a small charge per part for the fp32 partial results and their sum.  Every
// workgroup, and lm_split_reduce, computes the same plan from the same numbers.
struct LmSplit {
    int full, rest, s2;
};
__device__ __forceinline__ LmSplit lm_plan_split(int tiles, int k_tiles, int max_items, int n_cu)
{
    LmSplit sp;
    sp.rest = max_items > 0 ? tiles % n_cu : 0;
    sp.full = tiles - sp.rest;
    sp.s2 = 1;
    if (sp.rest == 0) return sp;
    const int lim = min(min(LM_SPLIT_MAX, k_tiles / 8), max_items / sp.rest);
    float best = 1.f;
    for (int S = 2; S <= lim; ++S) {
        const float cost = (float)((sp.rest * S + n_cu - 1) / n_cu) / (float)S + 0.002f * (float)S;
        if (cost < best) {
            best = cost;
            sp.s2 = S;
        }
    }
    return sp;
}

// Workgroup -> tile (and part).  Each XCD takes a contiguous run of the whole tiles, then a
// contiguous run of the parts, so that both kinds of work are spread evenly over the XCDs; the
// parts are ordered part by part (the same K range of neighbouring tiles shares operand panels).
// rest_index: which of the cut tiles this is, -1 for a whole tile.
__device__ __forceinline__ bool lm_map_tile(int tiles_m, int tiles_n, const LmSplit &sp, int group_m, int &tm, int &tn,
                                            int &part, int &rest_index)
{
    const int xcd = (int)(blockIdx.x & 7), idx = (int)(blockIdx.x >> 3);
    const int per_xcd = (sp.full + 7) / 8;
    int L;
    part = 0;
    rest_index = -1;
    if (idx < per_xcd) {
        L = xcd * per_xcd + idx;
        if (L >= sp.full) return false;
    } else {
        const int items = sp.rest * sp.s2, items_per_xcd = (items + 7) / 8;
        const int j = xcd * items_per_xcd + (idx - per_xcd);
        if (idx - per_xcd >= items_per_xcd || j >= items) return false;
        part = j / sp.rest;
        rest_index = j - part * sp.rest;
        L = sp.full + rest_index;
    }
    lm_tile_of(L, tiles_m, tiles_n, group_m, tm, tn);
    return true;
}

// A K-major operand tile in LDS is [64 k][256 m] bf16, 512 bytes per k row.  The 16-byte chunk at
// position pc of row k holds logical chunk pc ^ lm_km_swizzle(k) (applied on the global-address side):
// a transposing fragment read touches rows k .. k + 3 (and k + 8 .. k + 11 in the other half of the
// wavefront), 64 bytes of each, and with the swizzle those land on different banks.
__device__ __forceinline__ int lm_km_swizzle(int k) { return (4 * (k & 3)) ^ (2 * ((k >> 3) & 1)); }

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

template <int EPI, bool STORE_Z, bool AUX = false, bool AKM = false, bool BKM = false>
__global__ void __launch_bounds__(LM_THREADS) lm_gemm_nt(GemmParams p)
{
    extern __shared__ __attribute__((aligned(1024))) char lm_smem[];
    int M = p.M_dev ? min(*p.M_dev, p.M) : p.M;
    int chunk_base = 0;  // first row of this launch's chunk in A, tokens32 and zy
    if (p.chunk_cap > 0) {
        int count;
        lm_chunk_range(*p.M_dev, p.chunk_cap, p.chunk, chunk_base, count);
        M = min(count, p.M);
    }
    const int K = p.K_dev ? min((*p.K_dev + LM_BK - 1) / LM_BK * LM_BK, p.K) : p.K;
    if (EPI == LM_EPI_F32 && p.accumulate && K == 0) return;  // nothing to add (an empty chunk)
    int tm, tn, part = 0, parts = 1, rest_index = -1;
    {
        const int tiles_m = (M + LM_BM - 1) / LM_BM;
        const LmSplit sp = lm_plan_split(tiles_m * p.tiles_n, K / LM_BK, EPI == LM_EPI_BF16 ? p.split_items : 0,
                                         p.n_cu > 0 ? p.n_cu : 256);
        if (!lm_map_tile(tiles_m, p.tiles_n, sp, p.group_m, tm, tn, part, rest_index))
            return;  // whole workgroup alike, before any barrier
        if (rest_index >= 0) parts = sp.s2;
    }

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // in a scalar register: LDS targets are uniform
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
        const int ra = min(row0 + r, M - 1) - row0;
        const int rb = min(col0 + r, p.N - 1) - col0;
        // K-major operand: the tile is [64 k rows][256 m]; chunk c is k row c / 32 at position c % 32 and holds
        // logical chunk (c % 32) ^ lm_km_swizzle(k row); chunks past the end of the operand's k row re-read
        // its last chunk (they belong to rows or columns of C that are never stored)
        const int kk = c >> 5, lck = (c & 31) ^ lm_km_swizzle(kk);
        if constexpr (AKM) {
            const int ch = min((row0 >> 3) + lck, (p.a_cols >> 3) - 1) - (row0 >> 3);
            a_off[i] = (unsigned)((long long)kk * p.lda * 2 + ch * 16);
        } else {
            a_off[i] = (unsigned)(((long long)ra * p.lda + lc * 8) * 2);
        }
        if constexpr (BKM) {
            const int ch = min((col0 >> 3) + lck, (p.b_cols >> 3) - 1) - (col0 >> 3);
            b_off[i] = (unsigned)((long long)kk * p.ldb * 2 + ch * 16);
        } else {
            b_off[i] = (unsigned)(((long long)rb * p.ldb + lc * 8) * 2);
        }
    }
    // this workgroup's part of the contraction: K steps [kt0, kt0 + KT)
    const int kt0 = (int)((long long)(K / LM_BK) * part / parts);
    const int KT = (int)((long long)(K / LM_BK) * (part + 1) / parts) - kt0;
    const char *a_tile = AKM ? (const char *)p.A + ((long long)kt0 * LM_BK * p.lda + row0) * 2
                             : (const char *)p.A + ((long long)(chunk_base + row0) * p.lda + (long long)kt0 * LM_BK) * 2;
    const char *b_tile = BKM ? (const char *)p.B + ((long long)kt0 * LM_BK * p.ldb + col0) * 2
                             : (const char *)p.B + ((long long)col0 * p.ldb + (long long)kt0 * LM_BK) * 2;
    const long long a_kstep = (long long)LM_BK * p.lda * 2, b_kstep = (long long)LM_BK * p.ldb * 2;  // K-major only

    // LDS is a ring of five 32 KB slots that operand tiles pass through in the order
    // A(0), B(0), A(1), B(1), ...: entry q = 2 kt + (0 for A, 1 for B) lives in slot q % 5.
    // Two slots hold the tile being multiplied, the other three the next loads, which are
    // issued two at a time between the products.  Past the last tile the last one is loaded
    // again, into a slot nobody reads any more: every iteration then issues the same number
    // of loads and "landed" is a fixed vmcnt value.
    auto slot_of = [&](int q) { return lm_smem + (q % LM_SLOTS) * LM_TILE_BYTES; };
    // The loads are buffer loads with LDS as their target: the tile's first row at this
    // workgroup's first K step is the buffer's base, the lane's offset inside the tile a
    // vector register, the K position a scalar one, the LDS address goes through M0 - no
    // vector arithmetic per load.  The range check of the buffer is left wide open (rows are
    // clamped above and K steps below, so every address is inside the operand).
    const __amdgpu_buffer_rsrc_t a_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)a_tile, 0, -1, 0x00020000);
    const __amdgpu_buffer_rsrc_t b_rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)b_tile, 0, -1, 0x00020000);
    // A K-major operand moves by whole k rows from step to step, further than a 32-bit offset reaches:
    // its descriptor is made again for every step (scalar arithmetic).
    auto issue_half = [&](int q, bool b_operand, int half) {
        const int kt = min(q >> 1, KT - 1);
        char *sd = slot_of(q) + wave * 1024;
        if (b_operand ? BKM : AKM) {
            const char *base = b_operand ? b_tile + kt * b_kstep : a_tile + kt * a_kstep;
            unsigned bytes = 0xffffffffu;  // range check wide open, except for a ragged last step of B
            const int k0 = (kt0 + kt) * LM_BK;
            if (b_operand && p.b_rows > 0 && k0 + LM_BK > p.b_rows)
                bytes = (unsigned)((long long)(p.b_rows - k0 - 1) * p.ldb * 2 + (long long)(p.b_cols - col0) * 2);
            const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)bytes, 0x00020000);
#pragma unroll
            for (int i = half * (LM_LPT / 2); i < (half + 1) * (LM_LPT / 2); ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc,
                                                         (__attribute__((address_space(3))) void *)(sd + i * (LM_THREADS * 16)),
                                                         16, (int)(b_operand ? b_off[i] : a_off[i]), 0, 0, 0);
            return;
        }
        const int k0 = kt * (LM_BK * 2);
#pragma unroll
        for (int i = half * (LM_LPT / 2); i < (half + 1) * (LM_LPT / 2); ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(b_operand ? b_rsrc : a_rsrc,
                                                     (__attribute__((address_space(3))) void *)(sd + i * (LM_THREADS * 16)),
                                                     16, (int)(b_operand ? b_off[i] : a_off[i]), k0, 0, 0);
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
    // K-major tiles are read with the transposing 64-bit LDS read: lane i of a group of 16 lanes gives the
    // address of 4 consecutive m at k row i / 4 (piece i % 4 of 16 m) and receives the 4 k values of m = i.
    // Two such reads (k rows +0..3 and +4..7) make the 8 consecutive k of m = lane % 32 that a lane holds
    // for the 32 x 32 x 16 product: lanes 0-15 and 16-31 cover m 0-15 and 16-31, lanes 32-63 the k rows + 8.
    unsigned akm_off[LM_FA], bkm_off[LM_FB];
    {
        const int kh = lane >> 5, mg = (lane >> 4) & 1, i16 = lane & 15;
        const int kkl = 8 * kh + (i16 >> 2), sw = lm_km_swizzle(kkl);
#pragma unroll
        for (int i = 0; i < LM_FA; ++i) {
            const int ml = wm * (LM_FA * 32) + i * 32 + 16 * mg + 4 * (i16 & 3);
            akm_off[i] = (unsigned)(kkl * (LM_BM * 2) + (((ml >> 3) ^ sw) * 16) + (ml & 7) * 2);
        }
#pragma unroll
        for (int j = 0; j < LM_FB; ++j) {
            const int nl = wn * (LM_FB * 32) + j * 32 + 16 * mg + 4 * (i16 & 3);
            bkm_off[j] = (unsigned)(kkl * (LM_BN * 2) + (((nl >> 3) ^ sw) * 16) + (nl & 7) * 2);
        }
    }
    // Written as assembly: the compiler holds the builtin form of this read back behind every outstanding
    // load to LDS (s_waitcnt vmcnt(0) in front of each k-step's reads), which the pipeline below exists to
    // avoid.  The results arrive asynchronously; every use sits behind the explicit lgkmcnt(0) of lds_landed().
    auto tr_frag = [&](const char *s) {
        typedef short s16x4 __attribute__((ext_vector_type(4)));
        s16x4 lo, hi;
        const unsigned at = (unsigned)(uintptr_t)(__attribute__((address_space(3))) const char *)s;
        asm volatile("ds_read_b64_tr_b16 %0, %2\n\tds_read_b64_tr_b16 %1, %2 offset:2048"
                     : "=&v"(lo), "=&v"(hi)
                     : "v"(at)
                     : "memory");
        return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    static_assert(4 * (LM_BM * 2) == 2048, "the second read's offset is written into the assembly");

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
        for (int i = 0; i < LM_FA; ++i) {
            if constexpr (AKM)
                f[i] = tr_frag(sa + akm_off[i] + ks * (16 * LM_BM * 2));
            else
                f[i] = *(const bf16x8 *)(sa + a_wave + i * (32 * LM_BK * 2) + frag_off[ks]);
        }
#pragma unroll
        for (int j = 0; j < LM_FB; ++j) {
            if constexpr (BKM)
                f[LM_FA + j] = tr_frag(sb + bkm_off[j] + ks * (16 * LM_BN * 2));
            else
                f[LM_FA + j] = *(const bf16x8 *)(sb + b_wave + j * (32 * LM_BK * 2) + frag_off[ks]);
        }
    };
    auto products = [&](const bf16x8 (&f)[LM_FA + LM_FB]) {
#pragma unroll
        for (int i = 0; i < LM_FA; ++i)
#pragma unroll
            for (int j = 0; j < LM_FB; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[i], f[LM_FA + j], acc[i][j], 0, 0, 0);
    };
    // One k-step: wait for the fragments read during the previous k-step (they had all of its
    // products' time to arrive), issue the six reads of the next k-step's fragments, then the
    // eight products with the two global -> LDS loads behind the second and the fourth.  The
    // wait is written out so that it sits in front of the new reads: left to itself the
    // compiler puts one wait for everything between the reads and the first product.
    auto lds_landed = [&]() {
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0) and nothing else
        __builtin_amdgcn_sched_barrier(0);
    };
    auto interleave = [&]() {
        __builtin_amdgcn_sched_group_barrier(0x100, (AKM ? 2 : 1) * LM_FA + (BKM ? 2 : 1) * LM_FB, 0);
#pragma unroll
        for (int i = 0; i < LM_LPT / 2; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, LM_FA * LM_FB - LM_LPT, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    static_assert(LM_BM == 256 && LM_BN == 256, "K-major tiles: 32 chunks per k row");
    static_assert(LM_BK / 16 == 4 && LM_SLOTS == 5 && LM_LPT == 4 && LM_FA * LM_FB >= LM_LPT,
                  "the pipeline and its wait counts are written for 4 k-steps, 5 slots, 4 loads per operand tile");

    // Memory loads return in order, so "at most n outstanding" means that everything older
    // than the n youngest loads is in LDS.  The wait, the wait for the own LDS reads and the
    // workgroup barrier are one asm statement so that nothing is scheduled in between.
    if (KT > 0) {
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
        lds_landed();
        read_frags(F[1], kt, 1);
        products(F[0]);
        issue_half(2 * kt + 3, true, 1);   // rest of B(kt + 1)
        interleave();
        lds_landed();
        read_frags(F[0], kt, 2);
        products(F[1]);
        issue_half(2 * kt + 4, false, 0);  // A(kt + 2)
        interleave();
        lds_landed();
        read_frags(F[1], kt, 3);
        products(F[0]);
        issue_half(2 * kt + 4, false, 1);
        interleave();
        // outstanding, oldest first: ..., B(kt + 1), A(kt + 2): 4 left = tile kt + 1 landed
        asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        lds_landed();
        read_frags(F[0], kt + 1, 0);
        products(F[1]);
        issue_half(2 * kt + 5, true, 0);   // B(kt + 2) into the slot A(kt) just left
        interleave();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }  // KT > 0

    // Accumulator layout of a 32 x 32 block: lane l holds column l % 32; register v holds
    // row 8 (v / 4) + 4 (l / 32) + v % 4.
    const int cl = lane & 31, g = lane >> 5;
    const int wrow = wm * (LM_FA * 32), wcol = wn * (LM_FB * 32);
    if (EPI == LM_EPI_F32 && p.accumulate) {
        // C += result.  All loads of a block row first, then the sums and stores: element by element the
        // dependent load in front of every store made this epilogue take 2 ms longer than the plain store
        // (dL/dW of the second and later chunks).
#pragma unroll
        for (int i = 0; i < LM_FA; ++i) {
            float old[16][LM_FB];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + wrow + i * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
#pragma unroll
                for (int j = 0; j < LM_FB; ++j) {
                    const int col = col0 + wcol + j * 32 + cl;
                    old[v][j] = (row < M && col < p.N) ? ((const float *)p.C)[(long long)row * p.ldc + col] : 0.f;
                }
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + wrow + i * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
#pragma unroll
                for (int j = 0; j < LM_FB; ++j) {
                    const int col = col0 + wcol + j * 32 + cl;
                    if (row < M && col < p.N) ((float *)p.C)[(long long)row * p.ldc + col] = old[v][j] + acc[i][j][v];
                }
            }
        }
        return;
    }
    if (EPI == LM_EPI_BF16 || EPI == LM_EPI_F32) {
#pragma unroll
        for (int i = 0; i < LM_FA; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + wrow + i * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
                if (row >= M) continue;
                const long long orow = (EPI == LM_EPI_BF16 && p.c_rows) ? p.c_rows[row] : row;
#pragma unroll
                for (int j = 0; j < LM_FB; ++j) {
                    const int col = col0 + wcol + j * 32 + cl;
                    if (col >= p.N) continue;
                    if (EPI == LM_EPI_BF16 && parts > 1) {
                        p.split_ws[(((long long)rest_index * parts + part) << 16) + (row - row0) * LM_BN + (col - col0)] =
                            acc[i][j][v];
                    } else if (EPI == LM_EPI_BF16) {
                        ((__bf16 *)p.C)[orow * p.ldc + col] = (__bf16)acc[i][j][v];
                    } else {
                        ((float *)p.C)[orow * p.ldc + col] = acc[i][j][v];
                    }
                }
            }
        return;
    }

    // Softmax partials of this tile: for every row the maximum of z k over the tile's
    // columns and the sum of exp2(z k - max), the sampled token's column left out of both
    // (its accumulator goes to zy instead) so that 1 - p_y keeps its precision later.
    //
    // An accumulator block spreads a row over 32 lanes; reducing it there costs ten cross-lane
    // steps per row.  Instead every wavefront turns its part of the tile round through LDS
    // (free now), 64 rows at a time: written as accumulators, read back one whole row per
    // lane, so that maximum and sum are plain loops with every lane busy, and the fp32 copy of
    // the logits leaves in 16-byte pieces.  Rows are LM_EPI_PITCH floats apart: 16-byte aligned,
    // and neither the row-per-lane reads nor the 16-lanes-per-row reads collide on banks.
    constexpr int LM_EPI_PITCH = 68;
    constexpr int LM_EPI_WAVE_BYTES = 64 * LM_EPI_PITCH * 4;
    static_assert(8 * LM_EPI_WAVE_BYTES + (3 * LM_WN * LM_BM + LM_BM) * 4 <= LM_LDS_BYTES, "epilogue staging fits LDS");
    static_assert(LM_FA == 4 && LM_FB == 2 && LM_WM * LM_WN == 8, "the staging below is written for 128 x 64 parts");
    __syncthreads();  // the operand slots are free now
    float *stage = (float *)(lm_smem + wave * LM_EPI_WAVE_BYTES);
    float *red_m = (float *)(lm_smem + 8 * LM_EPI_WAVE_BYTES);  // [LM_WN][256]
    float *red_s = red_m + LM_WN * LM_BM;
    float *red_w = red_s + LM_WN * LM_BM;
    int *ycol_s = (int *)(red_w + LM_WN * LM_BM);
    if (tid < LM_BM) {
        // column of the sampled token inside this tile, -1 when it is elsewhere
        const int r = row0 + tid;
        int yc = -1;
        if (r < M) {
            const int y = p.tokens32[chunk_base + r];
            if (y >= col0 && y < col0 + LM_BN && y < p.N) yc = y - col0;
        }
        ycol_s[tid] = yc;
    }
    __syncthreads();
    const int ncols = min(64, p.N - col0 - wcol);  // columns of this wavefront's part inside the matrix
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        // accumulators of block rows 2h, 2h + 1 -> stage[64][pitch]
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int v = 0; v < 16; ++v)
#pragma unroll
                for (int j = 0; j < LM_FB; ++j)
                    stage[(ii * 32 + 8 * (v >> 2) + 4 * g + (v & 3)) * LM_EPI_PITCH + j * 32 + cl] = acc[2 * h + ii][j][v];
        // LDS serves a wavefront's accesses in order: what follows sees these writes
        const int rbase = wrow + h * 64;  // first of the 64 rows inside the tile
        if (STORE_Z && col0 + wcol < p.ldz) {
            // 16 lanes per row, four rows per instruction; the columns between N and the row
            // pitch of Z receive the products with the clamped operand rows: never read
            const int rr = lane >> 4, c4 = (lane & 15) * 4;
#pragma unroll
            for (int it = 0; it < 16; ++it) {
                const int rl = it * 4 + rr;
                const int row = row0 + rbase + rl;
                const f32x4 zq = *(const f32x4 *)(stage + rl * LM_EPI_PITCH + c4);
                if (row < M) *(f32x4 *)(p.Z + (long long)row * p.ldz + col0 + wcol + c4) = zq;
            }
        }
        // lane = row: take the sampled token's logit out, blank what lies outside the matrix
        float *myrow = stage + lane * LM_EPI_PITCH;
        const int yc = ycol_s[rbase + lane] - wcol;
        if (yc >= 0 && yc < 64) {
            p.zy[chunk_base + row0 + rbase + lane] = myrow[yc];
            myrow[yc] = -INFINITY;
        }
        if (ncols < 64)
            for (int c = max(ncols, 0); c < 64; ++c) myrow[c] = -INFINITY;
        f32x4 zv[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) zv[c] = *(const f32x4 *)(myrow + 4 * c);
        float mz = -INFINITY;
#pragma unroll
        for (int c = 0; c < 16; ++c) mz = fmaxf(fmaxf(fmaxf(mz, zv[c][0]), fmaxf(zv[c][1], zv[c][2])), zv[c][3]);
        float s0 = 0.f, s1 = 0.f;
        if constexpr (AUX) {
            // exponents (z - max) k, exactly 0 at the maximum: the entropy gradient of a near-one-hot
            // row depends on it (see row_scalars_aux); elements at -inf contribute 0, not 0 * inf
            const float refz = mz == -INFINITY ? 0.f : mz;
            float w0 = 0.f, w1 = 0.f;
#pragma unroll
            for (int c = 0; c < 16; ++c)
#pragma unroll
                for (int e = 0; e < 4; e += 2) {
                    const float a0 = (zv[c][e] - refz) * p.k, a1 = (zv[c][e + 1] - refz) * p.k;
                    const float e0 = __builtin_amdgcn_exp2f(a0), e1 = __builtin_amdgcn_exp2f(a1);
                    s0 += e0;
                    s1 += e1;
                    w0 = fmaf(e0, fmaxf(a0, kExpFloor), w0);
                    w1 = fmaf(e1, fmaxf(a1, kExpFloor), w1);
                }
            red_w[wn * LM_BM + rbase + lane] = w0 + w1;
        } else {
            const float ref = mz == -INFINITY ? 0.f : mz * p.k;  // 0 for a row with nothing to sum
#pragma unroll
            for (int c = 0; c < 16; ++c) {
                s0 += __builtin_amdgcn_exp2f(fmaf(zv[c][0], p.k, -ref)) + __builtin_amdgcn_exp2f(fmaf(zv[c][1], p.k, -ref));
                s1 += __builtin_amdgcn_exp2f(fmaf(zv[c][2], p.k, -ref)) + __builtin_amdgcn_exp2f(fmaf(zv[c][3], p.k, -ref));
            }
        }
        red_m[wn * LM_BM + rbase + lane] = mz;  // in units of z
        red_s[wn * LM_BM + rbase + lane] = s0 + s1;
    }
    __syncthreads();
    if (tid < LM_BM) {
        const int row = row0 + tid;
        if (row < M) {
            float m = -INFINITY;
#pragma unroll
            for (int w = 0; w < LM_WN; ++w) m = fmaxf(m, red_m[w * LM_BM + tid]);
            float s = 0.f, ws = 0.f;
#pragma unroll
            for (int w = 0; w < LM_WN; ++w) {
                const float mw = red_m[w * LM_BM + tid];
                if (mw != -INFINITY) {
                    const float d = (mw - m) * p.k;  // <= 0; exactly 0 for the part that holds the maximum
                    const float f = __builtin_amdgcn_exp2f(d);
                    const float sw = red_s[w * LM_BM + tid];
                    s = fmaf(sw, f, s);
                    if constexpr (AUX) ws = fmaf(f, fmaf(d, sw, red_w[w * LM_BM + tid]), ws);
                }
            }
            p.part_m[(long long)tn * p.part_stride + row] = m;
            p.part_s[(long long)tn * p.part_stride + row] = s;
            if constexpr (AUX) p.part_w[(long long)tn * p.part_stride + row] = ws;
        }
    }
}

// Per-row arrays the fused path keeps between its kernels.  Rows that take part (mask 1,
// token id inside the vocabulary) are compacted: "compact row i" is original row rows[i],
// i < *n_live.  Of those, the ones with a gradient (c != 0) are compacted once more for
// the backward: "gradient row j" is compact row rows2[j], original row orig2[j], j < *n_grad.
// The masked tail of every rollout and the clipped tokens then cost no matrix work at all.
struct LmRows {
    int *rows, *tokens32, *n_live;   // [n], [n] (by compact row), [1]
    int *rows2, *orig2, *n_grad;     // [n], [n], [1]
    float *zy;     // by compact row: logit of the sampled token (fp32 accumulator)
    float *shift;  // max k + log2(sum): p_j = exp2(z_j k - shift)
    float *q;      // c / T
    float *gy;     // gradient at the sampled token: q (1 - p_y), from the sum without y
    // with the auxiliary terms: g_j = p_j (q2 + bq a_j), a_j = (z_j - mx) k - log2s = log2 p_j
    float *mx, *log2s, *q2, *bq;
    float *part_m, *part_s, *part_w;  // [tiles_n][part_stride], by row inside the chunk
    long long part_stride;
    int tiles_n;
    int chunk, chunk_cap;  // the chunk of compact rows the per-chunk kernels work on (lm_chunk_range)
};

// Ordered compaction by one workgroup: keeps the indices i < n with keep(i), in order.
// `emit(pos, i)` stores entry number pos; returns the count (in every lane).
template <typename Keep, typename Emit>
__device__ __forceinline__ int lm_ordered_select(long long n, Keep keep, Emit emit)
{
    __shared__ int wave_tot[16];
    __shared__ int base;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    if (tid == 0) base = 0;
    __syncthreads();
    for (long long i0 = 0; i0 < n; i0 += 1024) {
        const long long i = i0 + tid;
        const int kp = (i < n && keep(i)) ? 1 : 0;
        int incl = kp;  // inclusive scan inside the wavefront
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const int up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        if (lane == 63) wave_tot[wv] = incl;
        __syncthreads();
        int before = base;
        for (int w2 = 0; w2 < wv; ++w2) before += wave_tot[w2];
        if (kp) emit(before + incl - 1, i);
        __syncthreads();
        if (tid == 0) {
            int tot = 0;
            for (int w2 = 0; w2 < 16; ++w2) tot += wave_tot[w2];
            base += tot;
        }
        __syncthreads();
    }
    return base;
}

// Rows that take part -> rows[], tokens32[], *n_live; rows that do not get their defined
// outputs here (log-prob 0, or NaN for a bad token id in the log-probs-only call).
__global__ void __launch_bounds__(1024) lm_select_rows(RowParams p, LmRows w)
{
    const int total = lm_ordered_select(
        p.n_tokens,
        [&](long long r) {
            bool live = p.mask ? (p.mask[r] != 0) : true;
            if (live && p.token_w && p.token_w[r] == 0.f) live = false;  // a zero weight masks the row
            bool bad = false;
            if (live) {
                const long long y = p.tokens[r];
                if (y < 0 || y >= p.vocab) {
                    live = false;
                    bad = true;
                }
            }
            if (!live) {
                write_row_outputs(p, r, (bad && !p.bwd) ? NAN : 0.f, 0.f, 0);
                write_row_aux(p, r, 0.f, 0.f);
                if (bad && p.bwd) atomicOr(&p.hdr->error, 1);
            }
            return live;
        },
        [&](int pos, long long r) {
            w.rows[pos] = (int)r;
            w.tokens32[pos] = (int)p.tokens[r];
        });
    if (threadIdx.x == 0) *w.n_live = total;
}

// Compact rows of the current chunk with a gradient -> rows2[] (compact row), orig2[] (original
// row), *n_grad.
__global__ void __launch_bounds__(1024) lm_select_grad_rows(LmRows w)
{
    int base, count;
    lm_chunk_range(*w.n_live, w.chunk_cap, w.chunk, base, count);
    const int total = lm_ordered_select(
        count, [&](long long j) { return w.q[base + j] != 0.f || (w.bq && w.bq[base + j] != 0.f); },
        [&](int pos, long long j) {
            w.rows2[pos] = base + (int)j;
            w.orig2[pos] = w.rows[base + j];
        });
    if (threadIdx.x == 0) *w.n_grad = total;
}

// out[i][:] = in[rowmap[i]][:] for i < *count: d bf16 values per row, 16 bytes per lane.
__global__ void __launch_bounds__(256) lm_gather_rows(const __bf16 *in, long long ldi, const int *rowmap,
                                                      const int *count, int d, __bf16 *out, long long ldo)
{
    const int n = *count;
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        const u32x4 *src = (const u32x4 *)(in + (long long)rowmap[i] * ldi);
        u32x4 *dst = (u32x4 *)(out + (long long)i * ldo);
        for (int c = threadIdx.x; c < d / 8; c += 256) dst[c] = src[c];
    }
}

// Merges the tile partials of each compact row, then the objective's once-per-row arithmetic.
// A workgroup takes 16 compact rows; 16 lanes share a row, each merging every 16th tile, and
// their results meet in LDS in lane order (fixed order: the bits repeat from run to run).
constexpr int LM_CMB_ROWS = 16, LM_CMB_LANES = 16;
template <bool AUX>
__global__ void __launch_bounds__(LM_CMB_ROWS * LM_CMB_LANES) lm_combine(RowParams p, LmRows w)
{
    __shared__ float sh_m[LM_CMB_LANES][LM_CMB_ROWS + 1], sh_s[LM_CMB_LANES][LM_CMB_ROWS + 1];
    __shared__ float sh_w[LM_CMB_LANES][LM_CMB_ROWS + 1];
    const int rl = threadIdx.x % LM_CMB_ROWS, tl = threadIdx.x / LM_CMB_ROWS;
    int base, count;
    lm_chunk_range(*w.n_live, w.chunk_cap, w.chunk, base, count);
    const long long il = (long long)blockIdx.x * LM_CMB_ROWS + rl;  // row inside the chunk: the partials' index
    const long long i = base + il;                                  // compact row: the per-row arrays' index
    const bool live = il < count;
    float mz = -INFINITY;  // maximum over the tiles, in units of z
    if (live)
        for (int t = tl; t < w.tiles_n; t += LM_CMB_LANES) mz = fmaxf(mz, w.part_m[(long long)t * w.part_stride + il]);
    sh_m[tl][rl] = mz;
    __syncthreads();
#pragma unroll
    for (int l = 0; l < LM_CMB_LANES; ++l) mz = fmaxf(mz, sh_m[l][rl]);
    const float zy = live ? w.zy[i] : 0.f;
    const float mx = fmaxf(mz, zy);  // the sampled token may be the row's maximum
    const float mk = mx * p.k;
    float s = 0.f, ws = 0.f;
    if (live)
        for (int t = tl; t < w.tiles_n; t += LM_CMB_LANES) {
            const float mt = w.part_m[(long long)t * w.part_stride + il];
            if (mt == -INFINITY) continue;
            const float st = w.part_s[(long long)t * w.part_stride + il];
            if constexpr (AUX) {
                const float d = (mt - mx) * p.k;
                const float f = __builtin_amdgcn_exp2f(d);
                s = fmaf(st, f, s);
                ws = fmaf(f, fmaf(d, st, w.part_w[(long long)t * w.part_stride + il]), ws);
            } else {
                s = fmaf(st, __builtin_amdgcn_exp2f(fmaf(mt, p.k, -mk)), s);
            }
        }
    sh_s[tl][rl] = s;
    if constexpr (AUX) sh_w[tl][rl] = ws;
    __syncthreads();
    if (tl != 0 || !live) return;
    float s_excl = 0.f, w_excl = 0.f;
#pragma unroll
    for (int l = 0; l < LM_CMB_LANES; ++l) {
        s_excl += sh_s[l][rl];
        if constexpr (AUX) w_excl += sh_w[l][rl];
    }
    const long long row = w.rows[i];
    if constexpr (AUX) {
        float kl, H;
        const RowScalars o = row_scalars_aux(p, row, zy, mx, s_excl, w_excl, kl, H);
        write_row_aux(p, row, kl, H);
        write_row_outputs(p, row, o.logp, o.J, o.flags);
        const float q = o.c * p.inv_T;
        w.q[i] = q;
        w.gy[i] = q * (o.s_excl / o.s) + o.gy_ent;
        w.mx[i] = o.mx;
        w.log2s[i] = o.log2s;
        w.q2[i] = o.q2;
        w.bq[i] = o.bq;
    } else {
        const RowScalars o = row_scalars(p, row, zy, mk, s_excl);
        write_row_outputs(p, row, o.logp, o.J, o.flags);
        if (p.bwd) {
            const float q = o.c * p.inv_T;
            w.q[i] = q;
            w.gy[i] = q * (o.s_excl / o.s);
            w.shift[i] = o.shift;
        }
    }
}

// G = dL/dz in bf16 for the chunk's gradient rows, row-major [n_grad][ldg], from the fp32 logits:
// g_j = -q p_j, g_y = q (1 - p_y).  A wavefront takes 512 consecutive entries of a row, eight per lane
// (two 16-byte reads, one 16-byte write); a workgroup 16 rows of them.  Padding is written as zeros: the
// columns V .. ldg (dL/dH runs over whole K steps of the vocabulary) and the rows n_grad .. the next
// multiple of 64 (dL/dW runs over whole K steps of rows).
constexpr int LM_GL_COLS = 512, LM_GL_ROWS = 16;
template <bool AUX>
__global__ void __launch_bounds__(256) lm_grad_logits(const float *Z, long long ldz, int V, LmRows w,
                                                      float k, __bf16 *G, long long ldg, int col_groups)
{
    const int n2 = *w.n_grad, n2_pad = (n2 + 63) / 64 * 64;
    const int r0 = (int)(blockIdx.x / (unsigned)col_groups) * LM_GL_ROWS;
    if (r0 >= n2_pad) return;  // LM_GL_ROWS divides 64: a workgroup's rows are all inside or all outside
    int zbase, zcount;  // Z holds the current chunk's rows only
    lm_chunk_range(*w.n_live, w.chunk_cap, w.chunk, zbase, zcount);
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int c = (int)(blockIdx.x % (unsigned)col_groups) * LM_GL_COLS + lane * 8;
    if (c >= ldg) return;  // ldg is a multiple of 64: whole groups of eight
#pragma unroll
    for (int i = 0; i < LM_GL_ROWS / 4; ++i) {
        const int r = r0 + wv + 4 * i;
        float gv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (r < n2 && c < V) {
            const int ci = w.rows2[r];
            float q = 0.f, sh = 0.f, mxr = 0.f, l2s = 0.f, q2 = 0.f, bq = 0.f;
            if constexpr (AUX) {
                mxr = w.mx[ci], l2s = w.log2s[ci], q2 = w.q2[ci], bq = w.bq[ci];
            } else {
                q = w.q[ci], sh = w.shift[ci];
            }
            const int y = w.tokens32[ci];
            const float *zrow = Z + (long long)(ci - zbase) * ldz + c;
            float z[8];
            if (c + 7 < V) {
                const f32x4 z0 = *(const f32x4 *)zrow, z1 = *(const f32x4 *)(zrow + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) z[e] = z0[e], z[4 + e] = z1[e];
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) z[e] = c + e < V ? zrow[e] : -INFINITY;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if constexpr (AUX) {
                    // g_j = p_j (q2 + bq log2 p_j): policy, KL and entropy parts in one (see grad_vec_aux)
                    const float a = fmaxf(fmaf(z[e] - mxr, k, -l2s), kExpFloor);
                    gv[e] = __builtin_amdgcn_exp2f(a) * fmaf(bq, a, q2);
                } else {
                    gv[e] = -q * __builtin_amdgcn_exp2f(fmaf(z[e], k, -sh));
                }
                if (c + e == y) gv[e] = w.gy[ci];
                if (c + e >= V) gv[e] = 0.f;
            }
        }
        u32x4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            out[e] = __builtin_bit_cast(unsigned, __builtin_convertvector((f32x2){gv[2 * e], gv[2 * e + 1]}, bf16x2));
        *(u32x4 *)(G + (long long)r * ldg + c) = out;
    }
}

// out[c][r] = in[rowmap ? rowmap[r] : r][c] for r < R (R = *R_dev when given), c < C; the
// columns R .. ldo of out are zero-filled.  64 x 64 tiles through LDS, four consecutive
// elements (8 bytes) per lane on both sides; C and ldo are multiples of 4 and both matrices
// 8-byte aligned (the operands of this path: d_model is a multiple of 64, rows 16-byte aligned).
__global__ void __launch_bounds__(256) lm_transpose(const __bf16 *in, long long ldi, int R, const int *R_dev,
                                                    const int *rowmap, int C, __bf16 *out, long long ldo)
{
    __shared__ unsigned short tile[64][66];
    if (R_dev) R = min(R, *R_dev);
    // x walks the rows of `in` (the vocabulary for W: the y extent of a grid ends at 65535)
    const int r0 = blockIdx.x * 64, c0 = blockIdx.y * 64;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;  // 16 lanes x 4 elements across, 16 down
    const unsigned short *src = (const unsigned short *)in;
    unsigned short *dst = (unsigned short *)out;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int rl = ty + 16 * i, r = r0 + rl, c = c0 + tx * 4;
        unsigned lo = 0, hi = 0;
        if (r < R && c < C) {
            const unsigned *q = (const unsigned *)(src + (long long)(rowmap ? rowmap[r] : r) * ldi + c);
            lo = q[0];
            hi = q[1];
        }
        tile[rl][tx * 4 + 0] = (unsigned short)lo;
        tile[rl][tx * 4 + 1] = (unsigned short)(lo >> 16);
        tile[rl][tx * 4 + 2] = (unsigned short)hi;
        tile[rl][tx * 4 + 3] = (unsigned short)(hi >> 16);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int cl2 = ty + 16 * i, c = c0 + cl2, r = r0 + tx * 4;  // a row of the output, four of its columns
        if (c < C && r < ldo) {
            unsigned *q = (unsigned *)(dst + (long long)c * ldo + r);
            q[0] = (unsigned)tile[tx * 4][cl2] | ((unsigned)tile[tx * 4 + 1][cl2] << 16);
            q[1] = (unsigned)tile[tx * 4 + 2][cl2] | ((unsigned)tile[tx * 4 + 3][cl2] << 16);
        }
    }
}

// Sum of the parts of the tiles lm_gemm_nt has cut: C[c_rows[r]][:] = bf16(sum over s of the
// tile's partial blocks) for the rows present, parts in order.  Does nothing when no tile was cut.
__global__ void __launch_bounds__(256) lm_split_reduce(const float *ws, const int *M_dev, int M, int N, int tiles_n,
                                                       int k_tiles, int max_items, int n_cu, int group_m,
                                                       const int *c_rows, __bf16 *C, long long ldc)
{
    const int rows = M_dev ? min(*M_dev, M) : M;
    const int tiles_m = (rows + LM_BM - 1) / LM_BM;
    const LmSplit sp = lm_plan_split(tiles_m * tiles_n, k_tiles, max_items, n_cu);
    if (sp.s2 == 1) return;
    constexpr int quads = LM_BN / 4;
    const long long total = (long long)sp.rest * LM_BM * quads;
    for (long long e = (long long)blockIdx.x * 256 + threadIdx.x; e < total; e += (long long)gridDim.x * 256) {
        const int t = (int)(e / (LM_BM * quads)), in_tile = (int)(e % (LM_BM * quads));
        const int r = in_tile / quads, c = in_tile % quads * 4;
        int tm, tn;
        lm_tile_of(sp.full + t, tiles_m, tiles_n, group_m, tm, tn);
        const int row = tm * LM_BM + r, col = tn * LM_BN + c;
        if (row >= rows || col >= N) continue;  // N is a multiple of LM_BK: a quad is inside or outside
        const float *src = ws + (((long long)t * sp.s2) << 16) + r * LM_BN + c;
        f32x4 a = *(const f32x4 *)src;
        for (int s = 1; s < sp.s2; ++s) a += *(const f32x4 *)(src + ((long long)s << 16));
        const bf16x2 lo = __builtin_convertvector((f32x2){a[0], a[1]}, bf16x2);
        const bf16x2 hi = __builtin_convertvector((f32x2){a[2], a[3]}, bf16x2);
        unsigned *dst = (unsigned *)(C + (long long)(c_rows ? c_rows[row] : row) * ldc + col);
        dst[0] = __builtin_bit_cast(unsigned, lo);
        dst[1] = __builtin_bit_cast(unsigned, hi);
    }
}

// rows x cols zeros into a row-strided matrix (fill kernels rather than memsets, so that
// the call can be captured into a graph)
template <typename T>
__global__ void __launch_bounds__(256) lm_zero(T *out, long long rows, long long cols, long long ld)
{
    const long long total = rows * cols;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256)
        out[(i / cols) * ld + i % cols] = (T)0;
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------

template <int EPI, bool STORE_Z, bool AUX = false, bool AKM = false, bool BKM = false>
hipError_t lm_launch_gemm(GemmParams p, hipStream_t st)
{
    static std::atomic<bool> attr_done[64];      // setting the attribute twice is harmless
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && !attr_done[dev].load()) {
        e = hipFuncSetAttribute((const void *)lm_gemm_nt<EPI, STORE_Z, AUX, AKM, BKM>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, LM_LDS_BYTES);
        if (e != hipSuccess) return e;
        attr_done[dev].store(true);
    }
    p.tiles_n = (p.N + LM_BN - 1) / LM_BN;
    if (p.group_m <= 0) p.group_m = LM_GROUP_M;
    // upper bound: every tile whole, plus the most parts a plan can have (fewer than n_cu tiles cut)
    const long long tiles = (long long)((p.M + LM_BM - 1) / LM_BM) * p.tiles_n;
    const long long items = EPI == LM_EPI_BF16 && p.split_items > 0
                                ? (long long)(p.n_cu > 0 ? p.n_cu : 256) * LM_SPLIT_MAX : 0;
    const long long grid = ((tiles + 7) / 8 + (items + 7) / 8) * 8;
    hipLaunchKernelGGL((lm_gemm_nt<EPI, STORE_Z, AUX, AKM, BKM>), dim3((unsigned)grid), dim3(LM_THREADS), LM_LDS_BYTES, st, p);
    return hipGetLastError();
}

struct LmLayout {
    size_t rows, tokens32, rows2, orig2, counts, zy, shift, q, gy, mx, log2s, q2, bq, part_m, part_s, part_w, Hc, Z, G, Ht,
        total;
    long long ldz, ldg, ldgt;  // vocab and chunk rows rounded up to whole K steps
    int tiles_n;
    int cap;  // rows per chunk: what the partials, Z, G and H^T are sized for
};

// Default limit of a chunk of the backward: 10240 rows keep the workspace at V = 152064 under
// 10 GB whatever the number of tokens (6 bytes per chunk row and vocabulary entry), and a chunk
// still fills the chip (40 tile rows: 23760 tiles of the logits product, 800 of dL/dH).  A caller
// that brings more gets larger chunks.
constexpr int64_t kLmChunkRows = 10240;
constexpr int64_t kLmChunkMax = 1 << 20;  // rows; keeps every per-chunk grid extent and 32-bit offset in range

int64_t lm_cap_limit(int64_t n) { return std::min<int64_t>(kLmChunkMax, std::max<int64_t>(256, (n + 255) / 256 * 256)); }

// cap: rows per chunk, a multiple of 256 in [256, lm_cap_limit(n)] (the forward alone is one chunk)
LmLayout lm_layout(int64_t n, int64_t V, int64_t d, bool bwd, int64_t cap)
{
    LmLayout L = {};
    L.cap = (int)cap;
    L.tiles_n = (int)((V + LM_BN - 1) / LM_BN);
    L.ldz = L.ldg = (long long)align_up((size_t)V, 64);  // whole K steps, 128-byte rows
    L.ldgt = (long long)align_up((size_t)cap, 64);
    size_t off = align_up(grpo_workspace_bytes(n), 256);
    auto take = [&](size_t bytes) {
        const size_t at = off;
        off += align_up(bytes, 256);
        return at;
    };
    L.counts = take(256);
    L.rows = take((size_t)n * 4);
    L.tokens32 = take((size_t)n * 4);
    L.zy = take((size_t)n * 4);
    L.part_m = take((size_t)L.tiles_n * cap * 4);
    L.part_s = take((size_t)L.tiles_n * cap * 4);
    L.Hc = take((size_t)n * d * 2);
    if (bwd) {
        L.rows2 = take((size_t)cap * 4);
        L.orig2 = take((size_t)cap * 4);
        L.shift = take((size_t)n * 4);
        L.q = take((size_t)n * 4);
        L.gy = take((size_t)n * 4);
        L.mx = take((size_t)n * 4);  // these four and part_w: only the call with the auxiliary terms
        L.log2s = take((size_t)n * 4);
        L.q2 = take((size_t)n * 4);
        L.bq = take((size_t)n * 4);
        L.part_w = take((size_t)L.tiles_n * cap * 4);
        L.Z = take((size_t)cap * L.ldz * 4);
        L.G = take((size_t)cap * L.ldg * 2);
        L.Ht = take((size_t)d * L.ldgt * 2);
    }
    L.total = off;
    return L;
}

// The largest chunk (multiple of 256 rows) whose workspace fits `bytes`; 0 if not even 256 rows do.
int64_t lm_cap_for_workspace(int64_t n, int64_t V, int64_t d, size_t bytes)
{
    int64_t lo = 0, hi = lm_cap_limit(n) / 256;  // in units of 256 rows; the size grows with the chunk
    while (lo < hi) {
        const int64_t mid = (lo + hi + 1) / 2;
        if (lm_layout(n, V, d, true, mid * 256).total <= bytes)
            lo = mid;
        else
            hi = mid - 1;
    }
    return lo * 256;
}

bool lm_sizes_ok(int64_t n_tokens, int64_t vocab, int64_t d_model)
{
    return n_tokens >= 0 && n_tokens <= 0x7fffff00ll && vocab > 0 && vocab <= kMaxVocab && d_model > 0 &&
           d_model <= (1 << 20) && d_model % LM_BK == 0;
}
// With the backward G is an operand whose rows are align64(vocab) elements long: the byte offset
// of row 255 of an operand tile must fit 32 bits.
bool lm_bwd_vocab_ok(int64_t vocab) { return (int64_t)align_up((size_t)vocab, 64) * 2 * LM_BM < (1ll << 32); }

grpo_status lm_check_common(const void *hidden, int64_t hidden_stride, const void *weight,
                            int64_t weight_stride, int64_t n_tokens, int64_t vocab, int64_t d_model,
                            const int64_t *tokens, float temperature, bool bwd)
{
    if (!lm_sizes_ok(n_tokens, vocab, d_model) || hidden_stride < d_model || weight_stride < d_model)
        return GRPO_ERR_SHAPE;
    if (bwd && !lm_bwd_vocab_ok(vocab)) return GRPO_ERR_SHAPE;
    if (!(temperature > 0.f) || !std::isfinite(temperature)) return GRPO_ERR_PARAM;
    if (n_tokens == 0) return GRPO_OK;
    if (!hidden || !weight || !tokens) return GRPO_ERR_NULL;
    if (((uintptr_t)hidden & 15u) || ((uintptr_t)weight & 15u) || ((hidden_stride * 2) & 15) ||
        ((weight_stride * 2) & 15))
        return GRPO_ERR_ALIGN;
    // byte offsets inside one 256-row operand tile must fit 32 bits
    if (weight_stride * 2 * LM_BN >= (1ll << 32)) return GRPO_ERR_SHAPE;
    return GRPO_OK;
}

grpo_status lm_impl(bool bwd, bool aux, const void *hidden, int64_t hidden_stride, const void *weight,
                    int64_t weight_stride, int64_t n_tokens, int64_t vocab, int64_t d_model,
                    const int64_t *tokens, const float *old_logprobs, const float *ref_logprobs,
                    const float *advantages, const uint8_t *mask, const float *token_weights, float eps_low,
                    float eps_high, float delta, float temperature, float kl_coef, float entropy_coef,
                    double denom, float grad_scale, float *loss_out, float *logprobs_out, float *entropy_out,
                    int64_t *counts_out, void *grad_hidden, int64_t grad_hidden_stride,
                    float *grad_weight, int64_t grad_weight_stride, int accumulate_grad_weight,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    grpo_status rc = lm_check_common(hidden, hidden_stride, weight, weight_stride, n_tokens, vocab,
                                     d_model, tokens, temperature, bwd);
    if (rc != GRPO_OK) return rc;
    if (bwd) {
        if (!(eps_low >= 0.f && eps_low <= 1.f) || !(eps_high >= 0.f) || !std::isfinite(eps_high) ||
            !(delta > 1.f + eps_high) || std::isnan(denom) || std::isnan(grad_scale) ||
            !std::isfinite(kl_coef) || !std::isfinite(entropy_coef))
            return GRPO_ERR_PARAM;
        if (!loss_out) return GRPO_ERR_NULL;
        if (n_tokens > 0 && (!old_logprobs || !advantages || !grad_hidden)) return GRPO_ERR_NULL;
        if (n_tokens > 0 && kl_coef != 0.f && !ref_logprobs) return GRPO_ERR_NULL;
        if (!grad_weight) return GRPO_ERR_NULL;
        if (grad_hidden_stride < d_model || grad_weight_stride < d_model) return GRPO_ERR_SHAPE;
    } else {
        if (n_tokens == 0) return GRPO_OK;
        if (!logprobs_out) return GRPO_ERR_NULL;
    }
    if (!workspace || ((uintptr_t)workspace & 255u) != 0) return GRPO_ERR_WORKSPACE;
    // the forward alone keeps nothing per logit and takes the largest chunk there is (one chunk up
    // to 2^20 tokens); the backward takes the largest chunk the caller's workspace holds
    const int64_t cap = bwd ? lm_cap_for_workspace(n_tokens, vocab, d_model, workspace_bytes) : lm_cap_limit(n_tokens);
    if (cap == 0) return GRPO_ERR_WORKSPACE;
    const LmLayout L = lm_layout(n_tokens, vocab, d_model, bwd, cap);
    if (workspace_bytes < L.total) return GRPO_ERR_WORKSPACE;

    char *ws = (char *)workspace;
    hipStream_t st = (hipStream_t)stream;
    const size_t col = align_up((size_t)n_tokens * 4, 256);
    WsHeader *hdr = (WsHeader *)ws;
    float *J_ws = (float *)(ws + kHeaderBytes);
    float *KL_ws = (float *)(ws + kHeaderBytes + col);
    float *H_ws = (float *)(ws + kHeaderBytes + 2 * col);
    unsigned char *flags_ws = (unsigned char *)(ws + kHeaderBytes + 3 * col);
    FinPartial *partials = (FinPartial *)(ws + kHeaderBytes + 3 * col + align_up((size_t)n_tokens, 256));

    if (bwd)
        hipLaunchKernelGGL(grpo_prepare, dim3(1), dim3(1024), 0, st, mask, aux ? token_weights : (const float *)nullptr,
                           (long long)n_tokens, denom, hdr);
    if (n_tokens > 0) {
        const int M = (int)n_tokens, V = (int)vocab, D = (int)d_model;
        const int Mc = (int)std::min<int64_t>(cap, n_tokens);  // most rows a chunk can have
        const int n_chunks = (int)((n_tokens + cap - 1) / cap);
        LmRows w = {};
        w.n_live = (int *)(ws + L.counts);
        w.n_grad = w.n_live + 1;
        w.rows = (int *)(ws + L.rows);
        w.tokens32 = (int *)(ws + L.tokens32);
        w.zy = (float *)(ws + L.zy);
        w.part_m = (float *)(ws + L.part_m);
        w.part_s = (float *)(ws + L.part_s);
        w.part_stride = cap;
        w.tiles_n = L.tiles_n;
        w.chunk_cap = (int)cap;
        if (aux) {
            w.part_w = (float *)(ws + L.part_w);
            w.mx = (float *)(ws + L.mx);
            w.log2s = (float *)(ws + L.log2s);
            w.q2 = (float *)(ws + L.q2);
            w.bq = (float *)(ws + L.bq);
        }
        if (bwd) {
            w.rows2 = (int *)(ws + L.rows2);
            w.orig2 = (int *)(ws + L.orig2);
            w.shift = (float *)(ws + L.shift);
            w.q = (float *)(ws + L.q);
            w.gy = (float *)(ws + L.gy);
        }
        const float k = (float)((double)kLog2e / (double)temperature);

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
        if (aux) {
            p.ref_lp = kl_coef != 0.f ? ref_logprobs : nullptr;
            p.token_w = token_weights;
            p.KL_ws = KL_ws;
            p.H_ws = H_ws;
            p.entropy_out = entropy_out;
            p.kl_coef = kl_coef;
            p.ent_coef = entropy_coef;
        }

        // rows that take part, and their hidden states side by side
        __bf16 *Hc = (__bf16 *)(ws + L.Hc);
        hipLaunchKernelGGL(lm_select_rows, dim3(1), dim3(1024), 0, st, p, w);
        hipLaunchKernelGGL(lm_gather_rows, dim3((unsigned)(M < 8192 ? M : 8192)), dim3(256), 0, st,
                           (const __bf16 *)hidden, (long long)hidden_stride, (const int *)w.rows,
                           (const int *)w.n_live, D, Hc, (long long)d_model);
        __bf16 *G = nullptr, *Ht = nullptr;
        const int n_cu = cu_count();
        if (bwd) {
            G = (__bf16 *)(ws + L.G), Ht = (__bf16 *)(ws + L.Ht);
            // rows without gradient keep the zeros written here
            hipLaunchKernelGGL(lm_zero<unsigned short>, dim3(2048), dim3(256), 0, st, (unsigned short *)grad_hidden,
                               (long long)n_tokens, (long long)d_model, (long long)grad_hidden_stride);
        }

        for (int c = 0; c < n_chunks; ++c) {
            w.chunk = c;
            GemmParams g = {};  // logits of the chunk's rows: softmax partials, z_y, fp32 copy for the backward
            g.A = Hc;
            g.lda = d_model;
            g.B = (const __bf16 *)weight;
            g.ldb = weight_stride;
            g.M = Mc;
            g.M_dev = w.n_live;
            g.chunk = c;
            g.chunk_cap = (int)cap;
            g.N = V;
            g.K = D;
            g.tokens32 = w.tokens32;
            g.k = k;
            g.part_m = w.part_m;
            g.part_s = w.part_s;
            g.part_w = w.part_w;
            g.part_stride = cap;
            g.zy = w.zy;
            g.Z = bwd ? (float *)(ws + L.Z) : nullptr;
            g.ldz = L.ldz;
            hipError_t e = aux   ? lm_launch_gemm<LM_EPI_LSE, true, true>(g, st)
                           : bwd ? lm_launch_gemm<LM_EPI_LSE, true>(g, st)
                                 : lm_launch_gemm<LM_EPI_LSE, false>(g, st);
            if (e != hipSuccess) return GRPO_ERR_HIP;

            const dim3 cmb_grid((unsigned)((Mc + LM_CMB_ROWS - 1) / LM_CMB_ROWS));
            if (aux)
                hipLaunchKernelGGL(lm_combine<true>, cmb_grid, dim3(LM_CMB_ROWS * LM_CMB_LANES), 0, st, p, w);
            else
                hipLaunchKernelGGL(lm_combine<false>, cmb_grid, dim3(LM_CMB_ROWS * LM_CMB_LANES), 0, st, p, w);
            if (!bwd) continue;

            hipLaunchKernelGGL(lm_select_grad_rows, dim3(1), dim3(1024), 0, st, w);
            const int gl_cols = (int)((L.ldg + LM_GL_COLS - 1) / LM_GL_COLS);
            // rows up to the next multiple of 64: the padding rows are written too (G has cap >= 256 rows)
            const dim3 gl_grid((unsigned)((long long)gl_cols * ((Mc + 63) / 64 * (64 / LM_GL_ROWS))));
            if (aux)
                hipLaunchKernelGGL(lm_grad_logits<true>, gl_grid, dim3(256), 0, st, (const float *)(ws + L.Z), L.ldz,
                                   V, w, k, G, L.ldg, gl_cols);
            else
                hipLaunchKernelGGL(lm_grad_logits<false>, gl_grid, dim3(256), 0, st, (const float *)(ws + L.Z), L.ldz,
                                   V, w, k, G, L.ldg, gl_cols);
            // H^T of the chunk's gradient rows [d][ldgt]
            hipLaunchKernelGGL(lm_transpose, dim3((unsigned)(L.ldgt / 64), (unsigned)((D + 63) / 64)), dim3(256), 0,
                               st, (const __bf16 *)hidden, (long long)hidden_stride, M, (const int *)w.n_grad,
                               (const int *)w.orig2, D, Ht, L.ldgt);

            GemmParams gh = {};  // dL/dH [gradient rows][d] = G . W, scattered to the original rows; W is read as it
                                 // lies, [vocab][d]: K-major, its rows past the vocabulary read as zeros
            gh.A = G;
            gh.lda = L.ldg;
            gh.B = (const __bf16 *)weight;
            gh.ldb = weight_stride;
            gh.b_cols = D;
            gh.b_rows = V;
            gh.M = Mc;
            gh.M_dev = w.n_grad;
            gh.N = D;
            gh.K = (int)L.ldg;
            gh.C = grad_hidden;
            gh.ldc = grad_hidden_stride;
            gh.c_rows = w.orig2;
            gh.group_m = LM_GM_BWD;
            // The fp32 logits are no longer needed: their space takes the partial results (blocks of
            // 256 x 256 fp32) of the tiles whose contraction over the vocabulary is cut into parts.
            const size_t z_blocks = (size_t)cap * (size_t)L.ldz * 4 / ((size_t)LM_BM * LM_BN * 4);
            gh.split_items = (int)(z_blocks < 0x7fffffffu ? z_blocks : 0x7fffffffu);
            gh.split_ws = (float *)(ws + L.Z);
            gh.n_cu = n_cu;
            e = lm_launch_gemm<LM_EPI_BF16, false, false, false, true>(gh, st);
            if (e != hipSuccess) return GRPO_ERR_HIP;
            if (gh.split_items > 0)
                hipLaunchKernelGGL(lm_split_reduce, dim3(2048), dim3(256), 0, st, (const float *)gh.split_ws,
                                   (const int *)w.n_grad, Mc, D, (D + LM_BN - 1) / LM_BN, (int)(L.ldg / LM_BK),
                                   gh.split_items, n_cu, LM_GM_BWD, (const int *)w.orig2, (__bf16 *)grad_hidden,
                                   (long long)grad_hidden_stride);

            GemmParams gw = {};  // dL/dW [V][d] (+)= G^T . H over the chunk's gradient rows; G is read as it lies,
                                 // [rows][ldg]: K-major
            gw.A = G;
            gw.lda = L.ldg;
            gw.a_cols = (int)L.ldg;
            gw.B = Ht;
            gw.ldb = L.ldgt;
            gw.M = V;
            gw.N = D;
            gw.K = (int)L.ldgt;
            gw.K_dev = w.n_grad;
            gw.C = grad_weight;
            gw.ldc = grad_weight_stride;
            gw.accumulate = (accumulate_grad_weight || c > 0) ? 1 : 0;  // the first chunk starts the sum
            gw.group_m = LM_GM_BWD;
            e = lm_launch_gemm<LM_EPI_F32, false, false, true, false>(gw, st);
            if (e != hipSuccess) return GRPO_ERR_HIP;
        }
    } else if (bwd && !accumulate_grad_weight && vocab > 0) {
        // no tokens: the weight gradient is zero
        hipLaunchKernelGGL(lm_zero<float>, dim3(4096), dim3(256), 0, st, grad_weight, (long long)vocab,
                           (long long)d_model, (long long)grad_weight_stride);
    }
    if (bwd)
        hipLaunchKernelGGL(grpo_finalize, dim3(fin_blocks(n_tokens)), dim3(1024), 0, st, J_ws,
                           aux ? KL_ws : (const float *)nullptr, H_ws, flags_ws, (long long)n_tokens, hdr, partials,
                           kl_coef, entropy_coef, loss_out, (long long *)counts_out, (int *)nullptr);
    return hipGetLastError() == hipSuccess ? GRPO_OK : GRPO_ERR_HIP;
}

}  // namespace

extern "C" {

size_t grpo_lmhead_workspace_bytes(int64_t n_tokens, int64_t vocab, int64_t d_model, int with_backward)
{
    if (!lm_sizes_ok(n_tokens, vocab, d_model) || (with_backward && !lm_bwd_vocab_ok(vocab))) return 0;
    const int64_t cap = with_backward ? std::min<int64_t>(lm_cap_limit(n_tokens), kLmChunkRows) : lm_cap_limit(n_tokens);
    return lm_layout(n_tokens, vocab, d_model, with_backward != 0, cap).total;
}

size_t grpo_lmhead_workspace_bytes_for_chunk(int64_t n_tokens, int64_t vocab, int64_t d_model, int64_t chunk_rows)
{
    if (!lm_sizes_ok(n_tokens, vocab, d_model) || !lm_bwd_vocab_ok(vocab) || chunk_rows <= 0) return 0;
    const int64_t cap = std::min<int64_t>(lm_cap_limit(n_tokens), (std::min<int64_t>(chunk_rows, kLmChunkMax) + 255) / 256 * 256);
    return lm_layout(n_tokens, vocab, d_model, true, cap).total;
}

grpo_status grpo_lmhead_logprobs_fwd(const void *hidden, int64_t hidden_stride, const void *weight,
                                     int64_t weight_stride, int64_t n_tokens, int64_t vocab,
                                     int64_t d_model, const int64_t *tokens, const uint8_t *mask,
                                     float temperature, float *logprobs_out, void *workspace,
                                     size_t workspace_bytes, void *stream)
{
    return lm_impl(false, false, hidden, hidden_stride, weight, weight_stride, n_tokens, vocab, d_model, tokens,
                   nullptr, nullptr, nullptr, mask, nullptr, 0.f, 0.f, 0.f, temperature, 0.f, 0.f, 0.0, 0.f, nullptr,
                   logprobs_out, nullptr, nullptr, nullptr, 0, nullptr, 0, 0, workspace, workspace_bytes, stream);
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
    return lm_impl(true, false, hidden, hidden_stride, weight, weight_stride, n_tokens, vocab, d_model, tokens,
                   old_logprobs, nullptr, advantages, mask, nullptr, eps_low, eps_high, delta, temperature, 0.f, 0.f,
                   denom, grad_scale, loss_out, logprobs_out, nullptr, counts_out, grad_hidden, grad_hidden_stride,
                   grad_weight, grad_weight_stride, accumulate_grad_weight, workspace, workspace_bytes, stream);
}

grpo_status grpo_lmhead_loss_aux_fwd_bwd(const void *hidden, int64_t hidden_stride, const void *weight,
                                         int64_t weight_stride, int64_t n_tokens, int64_t vocab,
                                         int64_t d_model, const int64_t *tokens, const float *old_logprobs,
                                         const float *ref_logprobs, const float *advantages,
                                         const uint8_t *mask, const float *token_weights, float eps_low,
                                         float eps_high, float delta, float temperature, float kl_coef,
                                         float entropy_coef, double denom, float grad_scale, float *loss_out,
                                         float *logprobs_out, float *entropy_out, int64_t *counts_out,
                                         void *grad_hidden, int64_t grad_hidden_stride, float *grad_weight,
                                         int64_t grad_weight_stride, int accumulate_grad_weight,
                                         void *workspace, size_t workspace_bytes, void *stream)
{
    return lm_impl(true, true, hidden, hidden_stride, weight, weight_stride, n_tokens, vocab, d_model, tokens,
                   old_logprobs, ref_logprobs, advantages, mask, token_weights, eps_low, eps_high, delta,
                   temperature, kl_coef, entropy_coef, denom, grad_scale, loss_out, logprobs_out, entropy_out,
                   counts_out, grad_hidden, grad_hidden_stride, grad_weight, grad_weight_stride,
                   accumulate_grad_weight, workspace, workspace_bytes, stream);
}

}  // extern "C"
