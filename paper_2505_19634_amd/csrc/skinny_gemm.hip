// skinny_gemm: Y[M][N] = X[M][K] W[N][K]^T for the B * (k + 1) new tokens of a verify forward (M up to
// 256) against one weight matrix (paper Section 3.1: the step is bound by loading the weights; Appendix:
// 64 GB of weights for the 32B model).  bf16 in, fp32 accumulate on the matrix cores, bf16 out.
// HBM-bound on streaming W once: 2 * M flop per weight byte is far below the MFMA balance.
//
//   skinny_gemm_kernel<MT>  up to 64 tokens; grid (blocks of 128 weight rows, K splits).  Each of the 4 wavefronts owns 32
//       weight rows and walks the K range in chunks of 128: the W tile (32 x 128, 8 KB) comes in with
//       coalesced non-temporal 16-byte loads two chunks ahead, is staged through a wavefront-private LDS
//       slab and read back as the MFMA A operand; the X chunk (up to 256 x 128) is fetched once per
//       workgroup from the L2 into a double-buffered LDS tile shared by the 4 wavefronts (one barrier per
//       chunk) and read as the B operand.  Y^T[n][m] accumulates in registers over the whole K range.
//   skinny_gemm_wide_kernel<MT, WAVES>  more than 64 tokens, or long K runs; grid (blocks of 256 weight rows,
//       K splits): 8 wavefronts with one row tile each (two wavefronts per SIMD) up to 224 tokens; 4 wavefronts
//       with two row tiles each (every X fragment read from LDS feeds two MFMAs) at 225..256.
//   skinny_gemm_wide8_kernel<MT>  129..256 tokens on long K runs: the eight-wavefront shape with X brought in by
//       global-to-LDS loads into two half-chunk stages instead of through registers.
//   skinny_gemm_reduce_kernel  only when K is split across workgroups (few weight rows): sums the fp32
//       partials in a fixed order and converts.
#include "lotts_common.h"

namespace lotts {

typedef __bf16 g_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 g_bf16x4 __attribute__((ext_vector_type(4)));
typedef float g_f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned g_u32x4 __attribute__((ext_vector_type(4)));

constexpr int kGemmThreads = 256;
constexpr int kGemmWaves = 4;
constexpr int kGemmRows = 32;                         // weight rows per wavefront = M of the MFMA
constexpr int kGemmBlockN = kGemmWaves * kGemmRows;   // weight rows per workgroup
constexpr int kGemmChunk = 128;                       // K elements per chunk
constexpr int kGemmRowBytes = kGemmChunk * 2 + 16;    // LDS row pitch: conflict-free 16-byte row reads
constexpr int kGemmMaxM = 256;
constexpr int kGemmMaxSplit = 32;

struct GemmParams {
    const __bf16 *X, *W;
    __bf16* Y;
    float* part;  // [ksplit][M][N] fp32 when ksplit > 1
    int M, N, K, ksplit;
    long long ldx, ldw, ldy;
};

struct GemmPlan {
    int mt, wide, rt, nblocks, ksplit;  // rt: row tiles per wavefront of the wide kernel (8 / wavefronts)
    int staged;                         // X through global-to-LDS stages (skinny_gemm_wide8_kernel)
};
// K split for `nblocks` blocks of weight rows.  Few blocks: split K so that the launch fills the chip.
// Measured on the 32B-shaped layers: a workgroup count just above the number of compute units is the
// worst choice (a few units run two workgroups and everybody waits for them), so the count stays at
// or below one per unit -- or, when two fit a unit and every workgroup still gets a long run of
// chunks, at or below two per unit.
static inline int plan_ksplit(int nblocks, int chunks, bool two_per_cu) {
    if (nblocks >= kNumCU) return 1;
    int ks = two_per_cu ? (2 * kNumCU) / nblocks : kNumCU / nblocks;
    if (two_per_cu && chunks / ks < 16) ks = kNumCU / nblocks;
    const int max_ks = chunks / 4 > 0 ? chunks / 4 : 1;  // at least 4 chunks per workgroup
    if (ks > max_ks) ks = max_ks;
    if (ks > kGemmMaxSplit) ks = kGemmMaxSplit;
    return ks < 1 ? 1 : ks;
}

static inline GemmPlan plan_gemm(int M, int N, int K, long long ldx) {
    GemmPlan pl;
    pl.mt = (M + 31) / 32;
    const int chunks = K / kGemmChunk;
    // The wide kernel covers 256 weight rows per workgroup, one workgroup per unit, so an X chunk staged
    // in LDS serves twice the rows of the narrow kernel.  Up to 64 tokens it wins when its workgroups still get long
    // runs of chunks (gate+up, down) and loses on short ones (QKV, O).  It runs on eight wavefronts with one row
    // tile each: two wavefronts per SIMD hide each other's barrier and load waits, measured 4..22 % faster on the
    // 32B-shaped layers than four wavefronts with two row tiles each (where an X fragment read from LDS feeds two
    // MFMAs) at every token count that fits -- 256 tokens do not (the accumulators leave room for one wavefront
    // per SIMD only) and take the four-wavefront shape, unless the staged kernel below serves them.
    pl.rt = pl.mt <= 7 ? 1 : 2;
    const int nb_wide = (N + 2 * kGemmBlockN - 1) / (2 * kGemmBlockN);
    const int ks_wide = plan_ksplit(nb_wide, chunks, false);
    pl.wide = (pl.mt > 2 || chunks / ks_wide >= 16) ? 1 : 0;
    pl.staged = 0;
    if (pl.wide) {
        pl.nblocks = nb_wide;
        pl.ksplit = ks_wide;
        // The staged kernel, where it measured faster on the 32B-shaped layers (gate+up: 40 chunks per workgroup,
        // from 129 tokens; down: 18, from 161; QKV and O: 5..10, at 225..256 only), and where a lane's byte offset
        // into X fits the 32 bits its loads take.
        const int run = chunks / pl.ksplit;
        const bool pays = pl.mt == 8 || (pl.mt >= 5 && run >= 32) || (pl.mt >= 6 && run >= 16);
        pl.staged = (pays && (long long)(M - 1) * ldx * 2 + 256 < (1LL << 32)) ? 1 : 0;
    } else {
        pl.nblocks = (N + kGemmBlockN - 1) / kGemmBlockN;
        pl.ksplit = plan_ksplit(pl.nblocks, chunks, true);
    }
    return pl;
}

template <int MT>
__global__ __launch_bounds__(kGemmThreads, 2) void skinny_gemm_kernel(const GemmParams p) {
    constexpr int XROWS = 32 * MT;
    __shared__ __attribute__((aligned(16))) unsigned char xbuf[2][XROWS * kGemmRowBytes];
    __shared__ __attribute__((aligned(16))) unsigned char wslab_all[kGemmWaves][kGemmRows * kGemmRowBytes];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid & (kWave - 1);
    const int ln = lane & 31, hh = lane >> 5;
    const int n0 = blockIdx.x * kGemmBlockN + wave * kGemmRows;
    const int chunks = p.K / kGemmChunk;
    const int c_lo = (int)((long long)blockIdx.y * chunks / p.ksplit);
    const int c_hi = (int)((long long)(blockIdx.y + 1) * chunks / p.ksplit);
    unsigned char* wslab = wslab_all[wave];

    // W tile: 8 load instructions, each covering 4 whole 256-byte row pieces
    const int w_row = lane >> 4, w_ch = lane & 15;
    // Two W chunks are in flight per wavefront (16 KB), in two register sets that take turns: a set is
    // refilled with chunk c + 2 as soon as chunk c has been copied from it into the LDS slab.
    g_u32x4 w_even[8], w_odd[8];
    auto fetch_w = [&](int c, g_u32x4 (&dst)[8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int n = n0 + i * 4 + w_row;
            n = n < p.N ? n : p.N - 1;  // rows past the end re-read the last row; never stored
            dst[i] = __builtin_nontemporal_load(
                reinterpret_cast<const g_u32x4*>(p.W + (long long)n * p.ldw + (long long)c * kGemmChunk + w_ch * 8));
        }
    };
    // X chunk: XROWS rows x 16 pieces of 16 bytes, 2 * MT pieces per thread
    g_u32x4 x_even[2 * MT], x_odd[2 * MT];
    auto fetch_x = [&](int c, g_u32x4 (&xst)[2 * MT]) {
#pragma unroll
        for (int i = 0; i < 2 * MT; ++i) {
            const int idx = tid + i * kGemmThreads;
            int m = idx >> 4;
            m = m < p.M ? m : p.M - 1;
            xst[i] = *reinterpret_cast<const g_u32x4*>(p.X + (long long)m * p.ldx + (long long)c * kGemmChunk + (idx & 15) * 8);
        }
    };
    g_f32x16 acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    // One chunk.  Loads complete in issue order and every chunk's X piece is issued before its W piece,
    // so the barrier (X staged by all four wavefronts) never waits for anybody's W data: each wavefront
    // waits for its own W chunk after the barrier and the four drift apart by up to one chunk.
    auto chunk = [&](int c, g_u32x4 (&w)[8], g_u32x4 (&xst)[2 * MT]) {
        unsigned char* xb = xbuf[(c - c_lo) & 1];
#pragma unroll
        for (int i = 0; i < 2 * MT; ++i) {
            const int idx = tid + i * kGemmThreads;
            *reinterpret_cast<g_u32x4*>(xb + (idx >> 4) * kGemmRowBytes + (idx & 15) * 16) = xst[i];
        }
        __syncthreads();  // the X chunk is complete; the other buffer is free for chunk c + 1
#pragma unroll
        for (int i = 0; i < 8; ++i)
            *reinterpret_cast<g_u32x4*>(wslab + (i * 4 + w_row) * kGemmRowBytes + w_ch * 16) = w[i];
        if (c + 2 < c_hi) {
            fetch_x(c + 2, xst);
            fetch_w(c + 2, w);
        }
        // Y^T[n][m] += sum_k W[n][k] X[m][k]   (A = W rows, B = X rows, 8 steps of 16 k); the fragments of
        // step s + 1 are requested before the MFMAs of step s (see the wide kernel)
        auto frags = [&](int s, g_bf16x8& a, g_bf16x8 (&b)[MT]) {
            a = *reinterpret_cast<const g_bf16x8*>(wslab + ln * kGemmRowBytes + (2 * s + hh) * 16);
#pragma unroll
            for (int t = 0; t < MT; ++t)
                b[t] = *reinterpret_cast<const g_bf16x8*>(xb + (t * 32 + ln) * kGemmRowBytes + (2 * s + hh) * 16);
        };
        g_bf16x8 fa[2], fb[2][MT];
        frags(0, fa[0], fb[0]);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            if (s + 1 < 8) frags(s + 1, fa[(s + 1) & 1], fb[(s + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < MT; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s & 1], fb[s & 1][t], acc[t], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (c_lo < c_hi) {
        fetch_x(c_lo, x_even);
        fetch_w(c_lo, w_even);
    }
    if (c_lo + 1 < c_hi) {
        fetch_x(c_lo + 1, x_odd);
        fetch_w(c_lo + 1, w_odd);
    }
    for (int c = c_lo; c < c_hi; c += 2) {
        chunk(c, w_even, x_even);
        if (c + 1 < c_hi) chunk(c + 1, w_odd, x_odd);
    }
    // register i of this lane: output row m = t * 32 + ln, column n = n0 + (i / 4) * 8 + hh * 4 + i % 4
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int m = t * 32 + ln;
        if (m >= p.M) continue;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int n = n0 + q4 * 8 + hh * 4;
            if (n >= p.N) continue;  // N is a multiple of 8: the 4 columns are in or out together
            if (p.ksplit == 1) {
                g_bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[t][q4 * 4 + e];
                *reinterpret_cast<g_bf16x4*>(p.Y + (long long)m * p.ldy + n) = o;
            } else {
                *reinterpret_cast<float4*>(p.part + ((long long)blockIdx.y * p.M + m) * p.N + n) =
                    make_float4(acc[t][q4 * 4 + 0], acc[t][q4 * 4 + 1], acc[t][q4 * 4 + 2], acc[t][q4 * 4 + 3]);
            }
        }
    }
}

// More than 64 tokens, and long K runs at any M.  A workgroup of WAVES wavefronts covers 256 weight rows:
// each wavefront owns RT = 8 / WAVES MFMA row tiles (32 * RT rows) and all M tokens; with RT = 2 an X
// fragment read from LDS feeds two MFMAs.  One W chunk (8 KB * RT per wavefront) is in flight while the
// previous one is multiplied, as in the attention kernel; one X tile in LDS, rewritten behind a barrier
// once every wavefront has finished with it.
template <int MT, int WAVES>
__global__ __launch_bounds__(WAVES * kWave, 1) void skinny_gemm_wide_kernel(const GemmParams p) {
    constexpr int RT = 8 / WAVES;
    constexpr int kThreads = WAVES * kWave;
    constexpr int WROWS = 32 * RT;
    constexpr int XROWS = 32 * MT;
    constexpr int XPT = (XROWS * 16 + kThreads - 1) / kThreads;  // 16-byte pieces of an X chunk per thread
    __shared__ __attribute__((aligned(16))) unsigned char xbuf[XROWS * kGemmRowBytes];
    __shared__ __attribute__((aligned(16))) unsigned char wslab_all[WAVES][WROWS * kGemmRowBytes];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid & (kWave - 1);
    const int ln = lane & 31, hh = lane >> 5;
    const int n0 = blockIdx.x * (WAVES * WROWS) + wave * WROWS;
    const int chunks = p.K / kGemmChunk;
    const int c_lo = (int)((long long)blockIdx.y * chunks / p.ksplit);
    const int c_hi = (int)((long long)(blockIdx.y + 1) * chunks / p.ksplit);
    unsigned char* wslab = wslab_all[wave];

    const int w_row = lane >> 4, w_ch = lane & 15;  // a load instruction covers 4 whole 256-byte row pieces
    g_u32x4 wst[8 * RT], xst[XPT];
    auto fetch_w = [&](int c) {
#pragma unroll
        for (int i = 0; i < 8 * RT; ++i) {
            int n = n0 + i * 4 + w_row;
            n = n < p.N ? n : p.N - 1;  // rows past the end re-read the last row; never stored
            wst[i] = __builtin_nontemporal_load(
                reinterpret_cast<const g_u32x4*>(p.W + (long long)n * p.ldw + (long long)c * kGemmChunk + w_ch * 8));
        }
    };
    auto fetch_x = [&](int c) {
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            const int idx = tid + i * kThreads;
            int m = idx >> 4;
            m = m < p.M ? m : p.M - 1;
            xst[i] = *reinterpret_cast<const g_u32x4*>(p.X + (long long)m * p.ldx + (long long)c * kGemmChunk + (idx & 15) * 8);
        }
    };
    g_f32x16 acc[RT][MT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[r][t][i] = 0.f;

    if (c_lo < c_hi) {
        fetch_x(c_lo);  // X before W: loads complete in issue order and X is wanted first
        fetch_w(c_lo);
    }
    for (int c = c_lo; c < c_hi; ++c) {
        __syncthreads();  // every wavefront has multiplied the previous chunk out of the X tile
#pragma unroll
        for (int i = 0; i < XPT; ++i) {
            const int idx = tid + i * kThreads;
            if (idx < XROWS * 16)  // the last piece of a thread may lie past the tile when 512 threads share it
                *reinterpret_cast<g_u32x4*>(xbuf + (idx >> 4) * kGemmRowBytes + (idx & 15) * 16) = xst[i];
        }
        __syncthreads();  // the X chunk is complete
#pragma unroll
        for (int i = 0; i < 8 * RT; ++i)
            *reinterpret_cast<g_u32x4*>(wslab + (i * 4 + w_row) * kGemmRowBytes + w_ch * 16) = wst[i];
        if (c + 1 < c_hi) {
            fetch_x(c + 1);
            fetch_w(c + 1);
        }
        // Y^T[n][m] += sum_k W[n][k] X[m][k]: RT W fragments per k step, every X fragment feeds RT MFMAs.
        // The fragments of step s + 1 are requested before the MFMAs of step s are issued (the scheduling
        // barriers keep the compiler from sinking each read down to its use, where it would be waited for
        // with nothing else in flight: at most two wavefronts per SIMD are too few to hide an LDS latency).
        auto frags = [&](int s, g_bf16x8 (&a)[RT], g_bf16x8 (&b)[MT]) {
#pragma unroll
            for (int r = 0; r < RT; ++r)
                a[r] = *reinterpret_cast<const g_bf16x8*>(wslab + (r * 32 + ln) * kGemmRowBytes + (2 * s + hh) * 16);
#pragma unroll
            for (int t = 0; t < MT; ++t)
                b[t] = *reinterpret_cast<const g_bf16x8*>(xbuf + (t * 32 + ln) * kGemmRowBytes + (2 * s + hh) * 16);
        };
        // Two fragment sets, or one where registers run out: at 256 tokens, and at 224 with two wavefronts
        // per SIMD (256 registers each).
        constexpr int NF = (MT <= 7 && !(WAVES == 8 && MT >= 7)) ? 2 : 1;
        g_bf16x8 fa[NF][RT], fb[NF][MT];
        if (NF == 2) frags(0, fa[0], fb[0]);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            if (NF == 2) {
                if (s + 1 < 8) frags(s + 1, fa[(s + 1) & (NF - 1)], fb[(s + 1) & (NF - 1)]);
            } else {
                frags(s, fa[0], fb[0]);  // all reads of the step first, then the MFMAs as their operands arrive
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < MT; ++t) {
#pragma unroll
                for (int r = 0; r < RT; ++r)
                    acc[r][t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s & (NF - 1)][r], fb[s & (NF - 1)][t], acc[r][t], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // register i of this lane: output row m = t * 32 + ln, column n = n0 + r * 32 + (i / 4) * 8 + hh * 4 + i % 4
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int t = 0; t < MT; ++t) {
            const int m = t * 32 + ln;
            if (m >= p.M) continue;
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int n = n0 + r * 32 + q4 * 8 + hh * 4;
                if (n >= p.N) continue;  // N is a multiple of 8: the 4 columns are in or out together
                if (p.ksplit == 1) {
                    g_bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[r][t][q4 * 4 + e];
                    *reinterpret_cast<g_bf16x4*>(p.Y + (long long)m * p.ldy + n) = o;
                } else {
                    *reinterpret_cast<float4*>(p.part + ((long long)blockIdx.y * p.M + m) * p.N + n) =
                        make_float4(acc[r][t][q4 * 4 + 0], acc[r][t][q4 * 4 + 1], acc[r][t][q4 * 4 + 2],
                                    acc[r][t][q4 * 4 + 3]);
                }
            }
        }
}

// Many tokens on long K runs (see plan_gemm): eight wavefronts (two per SIMD), each with one MFMA row tile of 32
// weight rows and all M tokens, as the eight-wavefront shape of the kernel above.  W as there: one chunk (8 KB per
// wavefront) in flight in registers while the previous one is multiplied out of the wavefront's LDS slab.  X does
// not pass through registers: global-to-LDS loads (16 bytes per lane, written at a wavefront-uniform LDS base +
// 16 * lane) fill one of two half-chunk stages (64 k each) while the other is multiplied, one barrier per stage.
// That frees the 32 registers (256 tokens then fit two wavefronts per SIMD) and the LDS store instructions the X
// staging takes, and halves the lead of the X prefetch (half a chunk instead of one): a gain where a chunk takes
// long (many tokens, long runs), a loss where it is short.  A stage keeps rows of 128 bytes back to back (a load instruction
// fills 8 whole rows), so the 16-byte pieces of a row are stored permuted -- piece p of row r at slot
// p ^ ((r >> 1) & 7) -- which spreads the 16 lanes of a fragment read over all 64 banks.
template <int MT>
__global__ __launch_bounds__(8 * kWave, 1) void skinny_gemm_wide8_kernel(const GemmParams p) {
    constexpr int XROWS = 32 * MT;
    constexpr int XINSTR = XROWS / 8;            // load instructions per stage, dealt to the 8 wavefronts
    constexpr int XI = (XINSTR + 7) / 8;         // at most this many per wavefront
    constexpr int kStageRow = 128;               // bytes per row of a stage
    __shared__ __attribute__((aligned(1024))) unsigned char xs0[XROWS * kStageRow];
    __shared__ __attribute__((aligned(1024))) unsigned char xs1[XROWS * kStageRow];
    __shared__ __attribute__((aligned(16))) unsigned char wslab_all[8][32 * kGemmRowBytes];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid & (kWave - 1);
    const int ln = lane & 31, hh = lane >> 5;
    const int n0 = blockIdx.x * 256 + wave * 32;
    const int chunks = p.K / kGemmChunk;
    const int c_lo = (int)((long long)blockIdx.y * chunks / p.ksplit);
    const int c_hi = (int)((long long)(blockIdx.y + 1) * chunks / p.ksplit);
    unsigned char* wslab = wslab_all[wave];

    const int w_row = lane >> 4, w_ch = lane & 15;  // a W load instruction covers 4 whole 256-byte row pieces
    g_u32x4 wst[8];
    auto fetch_w = [&](int c) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            int n = n0 + i * 4 + w_row;
            n = n < p.N ? n : p.N - 1;  // rows past the end re-read the last row; never stored
            wst[i] = __builtin_nontemporal_load(
                reinterpret_cast<const g_u32x4*>(p.W + (long long)n * p.ldw + (long long)c * kGemmChunk + w_ch * 8));
        }
    };
    // lane -> (row of the instruction's 8, slot); the piece fetched for a slot is slot ^ swizzle(row).  The byte
    // offset of the lane's piece inside a half chunk of X is the same for every chunk: a 32-bit register per
    // instruction (the host checks that it fits), on top of a scalar base that moves along K.
    const int x_row = lane >> 3, x_slot = lane & 7;
    unsigned x_off[XI];
#pragma unroll
    for (int i = 0; i < XI; ++i) {
        const int r = (wave + i * 8) * 8 + x_row;
        const int m = r < p.M ? r : p.M - 1;
        x_off[i] = (unsigned)((long long)m * p.ldx * 2) + (unsigned)((x_slot ^ ((r >> 1) & 7)) * 16);
    }
    auto fetch_x = [&](int c, int half, unsigned char* stage) {
        const __bf16* base = p.X + (long long)c * kGemmChunk + half * 64;  // uniform
#pragma unroll
        for (int i = 0; i < XI; ++i) {
            const int j = wave + i * 8;  // uniform over the wavefront
            if (j < XINSTR) {
                // Written as an instruction: through the builtin the compiler makes every later LDS access of the
                // kernel wait for ALL loads in flight (it cannot tell which LDS bytes the transfer writes), which
                // would stall the W chunk that is meant to stay in flight.  M0 carries the LDS base.  No "memory"
                // clobber (with one the compiler again waits for everything before the next LDS read): the
                // barrier statements of the chunk loop, which have it, fence every read of a stage against the
                // transfer that refills it, and volatile statements keep their order among themselves.
                const unsigned lds_base = __builtin_amdgcn_readfirstlane(
                    (unsigned)(uintptr_t)(__attribute__((address_space(3))) void*)(stage + j * 8 * kStageRow));
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"  // M0 is on the clobber list on purpose
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                             :
                             : "v"(x_off[i]), "s"(base), "s"(lds_base)
                             : "m0");
#pragma clang diagnostic pop
            }
        }
    };
    g_f32x16 acc[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;

    const int swz = (ln >> 1) & 7;  // (row >> 1) & 7 of this lane's rows t * 32 + ln
    // four k steps of one stage: the W fragment comes from k steps 4 * half .. of the slab, the X fragments from the stage
    auto multiply = [&](int half, const unsigned char* stage) {
        constexpr int NF = MT <= 6 ? 2 : 1;  // two fragment sets while 256 registers hold them
        g_bf16x8 fa[NF], fb[NF][MT];
        auto frags = [&](int s, g_bf16x8& a, g_bf16x8 (&b)[MT]) {
            a = *reinterpret_cast<const g_bf16x8*>(wslab + ln * kGemmRowBytes + (2 * (4 * half + s) + hh) * 16);
#pragma unroll
            for (int t = 0; t < MT; ++t)
                b[t] = *reinterpret_cast<const g_bf16x8*>(stage + (t * 32 + ln) * kStageRow + (((2 * s + hh) ^ swz) * 16));
        };
        if (NF == 2) frags(0, fa[0], fb[0]);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (NF == 2) {
                if (s + 1 < 4) frags(s + 1, fa[(s + 1) & (NF - 1)], fb[(s + 1) & (NF - 1)]);
            } else {
                frags(s, fa[0], fb[0]);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < MT; ++t)
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s & (NF - 1)], fb[s & (NF - 1)][t], acc[t], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    if (c_lo < c_hi) {
        fetch_x(c_lo, 0, xs0);
        fetch_w(c_lo);
    }
    // The waits before the barriers are written out: a wavefront's global-to-LDS loads count in vmcnt like its
    // other loads, in issue order, and a stage must have landed before the barrier that publishes it.
    for (int c = c_lo; c < c_hi; ++c) {
        const bool more = c + 1 < c_hi;  // uniform
        // first half of chunk c: its X stage and W chunk c have been requested and nothing else is in flight
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");  // everybody's part of xs0 has landed; xs1 is free
#pragma unroll
        for (int i = 0; i < 8; ++i)
            *reinterpret_cast<g_u32x4*>(wslab + (i * 4 + w_row) * kGemmRowBytes + w_ch * 16) = wst[i];
        fetch_x(c, 1, xs1);
        __builtin_amdgcn_sched_barrier(0);  // the wait below counts on this order: the stage's loads, then the 8 of W
        if (more) fetch_w(c + 1);
        __builtin_amdgcn_sched_barrier(0);
        multiply(0, xs0);
        // second half: the stage requested above has landed; the 8 W loads issued after it, if any, stay in flight
        if (more)
            asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)\n\ts_barrier" ::: "memory");  // xs1 has landed; xs0 is free
        else
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (more) fetch_x(c + 1, 0, xs0);
        multiply(1, xs1);
    }
    // register i of this lane: output row m = t * 32 + ln, column n = n0 + (i / 4) * 8 + hh * 4 + i % 4
#pragma unroll
    for (int t = 0; t < MT; ++t) {
        const int m = t * 32 + ln;
        if (m >= p.M) continue;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int n = n0 + q4 * 8 + hh * 4;
            if (n >= p.N) continue;  // N is a multiple of 8: the 4 columns are in or out together
            if (p.ksplit == 1) {
                g_bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[t][q4 * 4 + e];
                *reinterpret_cast<g_bf16x4*>(p.Y + (long long)m * p.ldy + n) = o;
            } else {
                *reinterpret_cast<float4*>(p.part + ((long long)blockIdx.y * p.M + m) * p.N + n) =
                    make_float4(acc[t][q4 * 4 + 0], acc[t][q4 * 4 + 1], acc[t][q4 * 4 + 2], acc[t][q4 * 4 + 3]);
            }
        }
    }
}

__global__ __launch_bounds__(256) void skinny_gemm_reduce_kernel(const GemmParams p) {
    const long long i4 = ((long long)blockIdx.x * 256 + threadIdx.x) * 4;  // 4 consecutive columns of one row
    if (i4 >= (long long)p.M * p.N) return;
    const int m = (int)(i4 / p.N), n = (int)(i4 - (long long)m * p.N);
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int ks = 0; ks < p.ksplit; ++ks) {  // fixed order: deterministic
        const float4 v = *reinterpret_cast<const float4*>(p.part + ((long long)ks * p.M + m) * p.N + n);
        s.x += v.x;
        s.y += v.y;
        s.z += v.z;
        s.w += v.w;
    }
    g_bf16x4 o;
    o[0] = (__bf16)s.x;
    o[1] = (__bf16)s.y;
    o[2] = (__bf16)s.z;
    o[3] = (__bf16)s.w;
    *reinterpret_cast<g_bf16x4*>(p.Y + (long long)m * p.ldy + n) = o;
}

static inline bool gemm_sizes_ok(int M, int N, int K) {
    return M >= 1 && M <= kGemmMaxM && N >= 8 && (N % 8) == 0 && K >= kGemmChunk && (K % kGemmChunk) == 0 &&
           (long long)M * N < (1LL << 40);
}

}  // namespace lotts

extern "C" size_t skinny_gemm_workspace_bytes(int32_t M, int32_t N, int32_t K) {
    if (!lotts::gemm_sizes_ok(M, N, K)) return 0;
    const lotts::GemmPlan pl = lotts::plan_gemm(M, N, K, K);  // the K split does not depend on the row pitch of X
    const size_t bytes = pl.ksplit > 1 ? (size_t)pl.ksplit * M * N * sizeof(float) : 0;
    return bytes < 256 ? 256 : bytes;
}

extern "C" int skinny_gemm(int32_t M, int32_t N, int32_t K, const void* X, int64_t ldx, const void* W, int64_t ldw,
                           void* Y, int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
    using namespace lotts;
    if (!gemm_sizes_ok(M, N, K)) return LOTTS_ERR_SHAPE;
    if (!X || !W || !Y || !workspace) return LOTTS_ERR_NULL;
    if (ldx < K || ldw < K || ldy < N || (ldx % 8) || (ldw % 8) || (ldy % 4)) return LOTTS_ERR_SHAPE;
    if ((((uintptr_t)X | (uintptr_t)W | (uintptr_t)workspace) & 15) || ((uintptr_t)Y & 7)) return LOTTS_ERR_SHAPE;
    if (workspace_bytes < skinny_gemm_workspace_bytes(M, N, K)) return LOTTS_ERR_WORKSPACE;
    GemmPlan pl = plan_gemm(M, N, K, ldx);
    GemmParams p;

    p.X = static_cast<const __bf16*>(X);
    p.W = static_cast<const __bf16*>(W);
    p.Y = static_cast<__bf16*>(Y);
    p.part = static_cast<float*>(workspace);
    p.M = M; p.N = N; p.K = K; p.ksplit = pl.ksplit;
    p.ldx = ldx; p.ldw = ldw; p.ldy = ldy;
    hipStream_t s = (hipStream_t)stream;
    const dim3 grid(pl.nblocks, pl.ksplit), block(kGemmThreads), wide8(8 * kWave);
    if (pl.staged) {
        switch (pl.mt) {
            case 5: LOTTS_LAUNCH((skinny_gemm_wide8_kernel<5>), grid, wide8, s, p); break;
            case 6: LOTTS_LAUNCH((skinny_gemm_wide8_kernel<6>), grid, wide8, s, p); break;
            case 7: LOTTS_LAUNCH((skinny_gemm_wide8_kernel<7>), grid, wide8, s, p); break;
            default: LOTTS_LAUNCH((skinny_gemm_wide8_kernel<8>), grid, wide8, s, p); break;
        }
    } else if (pl.wide) {
        switch (pl.mt) {
            case 1: LOTTS_LAUNCH((skinny_gemm_wide_kernel<1, 8>), grid, wide8, s, p); break;
            case 2: LOTTS_LAUNCH((skinny_gemm_wide_kernel<2, 8>), grid, wide8, s, p); break;
            case 3: LOTTS_LAUNCH((skinny_gemm_wide_kernel<3, 8>), grid, wide8, s, p); break;
            case 4: LOTTS_LAUNCH((skinny_gemm_wide_kernel<4, 8>), grid, wide8, s, p); break;
            case 5: LOTTS_LAUNCH((skinny_gemm_wide_kernel<5, 8>), grid, wide8, s, p); break;
            case 6: LOTTS_LAUNCH((skinny_gemm_wide_kernel<6, 8>), grid, wide8, s, p); break;
            case 7: LOTTS_LAUNCH((skinny_gemm_wide_kernel<7, 8>), grid, wide8, s, p); break;
            default: LOTTS_LAUNCH((skinny_gemm_wide_kernel<8, 4>), grid, block, s, p); break;
        }
    } else if (pl.mt == 1) {
        LOTTS_LAUNCH(skinny_gemm_kernel<1>, grid, block, s, p);
    } else {
        LOTTS_LAUNCH(skinny_gemm_kernel<2>, grid, block, s, p);
    }
    int rc = check_launch();
    if (rc != LOTTS_OK || pl.ksplit == 1) return rc;
    const long long quads = ((long long)M * N + 3) / 4;
    LOTTS_LAUNCH(skinny_gemm_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), s, p);
    return check_launch();
}
