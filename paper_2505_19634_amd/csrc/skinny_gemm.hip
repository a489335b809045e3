// skinny_gemm: Y[M][N] = X[M][K] W[N][K]^T for the B * (k + 1) new tokens of a verify forward (M up to
// 256) against one weight matrix (paper Section 3.1: the step is bound by loading the weights; Appendix:
// 64 GB of weights for the 32B model).  bf16 in, fp32 accumulate on the matrix cores, bf16 out.
// HBM-bound on streaming W once: 2 * M flop per weight byte is far below the MFMA balance.
//
//   skinny_gemm_stream_kernel<MT, RT, WAVES>  grid (blocks of 32 * WAVES weight rows, K splits).  Each wavefront
//       owns an MFMA row tile of 32 weight rows and walks the K range in steps of half a chunk (64 k); W and X both go
//       from global memory straight into LDS stages, with no registers in between; Y^T[n][m] accumulates in
//       registers over the whole K range.  WAVES = 8 (256 weight rows, one workgroup per unit): long K runs and
//       every launch with more than 128 tokens.  WAVES = 4 (128 weight rows, two workgroups per unit): up to 128
//       tokens on short K runs (QKV, O), where more, smaller workgroups keep every unit streaming.
//   skinny_gemm_reduce_kernel  only when K is split across workgroups (few weight rows): sums the fp32
//       partials in a fixed order and converts.
#include "lotts_common.h"

namespace lotts {

typedef __bf16 g_bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 g_bf16x4 __attribute__((ext_vector_type(4)));
typedef float g_f32x16 __attribute__((ext_vector_type(16)));

constexpr int kGemmRows = 32;               // weight rows per wavefront = M of the MFMA
constexpr int kGemmBlockN = 4 * kGemmRows;  // weight rows of a four-wavefront workgroup; eight cover twice that
constexpr int kGemmChunk = 128;             // K elements per chunk
constexpr int kGemmMaxM = 256;
constexpr int kGemmMaxSplit = 32;

struct GemmParams {
    const __bf16 *X, *W;
    __bf16* Y;
    float* part;  // [ksplit][M][N] fp32 when ksplit > 1
    int M, N, K, ksplit;
    int rows;  // weight rows a wavefront owns: 32, or fewer (a multiple of 4) when that fills the chip better
    long long ldx, ldw, ldy;
};

struct GemmPlan {
    int mt, stream, nblocks, ksplit, rows;  // rows: weight rows per wavefront; stream: eight wavefronts, 256 weight rows per workgroup; else four and 128
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

static inline GemmPlan plan_gemm(int M, int N, int K) {
    GemmPlan pl;
    pl.mt = (M + 31) / 32;
    const int chunks = K / kGemmChunk;
    // Eight wavefronts cover 256 weight rows per workgroup, one workgroup per unit, so an X chunk staged in LDS
    // serves twice the rows of the four-wavefront form.  Up to 128 tokens they win when the workgroups still get long
    // runs of chunks (gate+up, down on the 32B-shaped layers) and lose on short ones (QKV, O: the four-wavefront form
    // splits K less, so fewer fp32 partials are written and added up); above 128 tokens two workgroups per unit do
    // not fit (LDS stages, accumulators), and the eight-wavefront form always runs.
    pl.rows = kGemmRows;
    int nb_stream = (N + 8 * kGemmRows - 1) / (8 * kGemmRows);
    int ks_stream = plan_ksplit(nb_stream, chunks, false);
    if (pl.mt <= 2) {
        // Up to 64 tokens the launch is HBM-bound and what counts is how many units stream: with 28 weight rows per
        // wavefront instead of 32 the 55296 rows of the 32B shape's gate+up make 247 workgroups instead of 216, and
        // the LM head's last round of workgroups is fuller (measured 1..2 % and 2..7 % faster; with more tokens the
        // padded MFMA rows cost more than the idle units).  Taken when it fills the last round visibly better.
        const int nb28 = (N + 8 * 28 - 1) / (8 * 28), ks28 = plan_ksplit(nb28, chunks, false);
        auto fill = [](int wgs) { return (double)wgs / (double)(((wgs + kNumCU - 1) / kNumCU) * kNumCU); };
        if (fill(nb28 * ks28) > fill(nb_stream * ks_stream) + 0.03) {
            pl.rows = 28;
            nb_stream = nb28;
            ks_stream = ks28;
        }
    }
    pl.stream = (pl.mt > 4 || chunks / ks_stream >= 16) ? 1 : 0;
    if (pl.stream) {
        pl.nblocks = nb_stream;
        pl.ksplit = ks_stream;
    } else {
        pl.rows = kGemmRows;
        pl.nblocks = (N + kGemmBlockN - 1) / kGemmBlockN;
        pl.ksplit = plan_ksplit(pl.nblocks, chunks, true);
    }
    return pl;
}

// The kernel.  WAVES wavefronts (eight: two per SIMD, one workgroup per unit; four: two workgroups per unit),
// 32 * WAVES weight rows per workgroup: each wavefront owns one MFMA row tile of 32 weight rows and
// all M tokens -- or, for an even number of token tiles from 4 on (97..128, 161..192, 225..256 tokens), two
// neighbouring wavefronts own two row tiles together and half of the token tiles each: a k step then reads
// 2 + MT / 2 fragments for MT MFMAs instead of 1 + MT, and LDS reads are what bounds the loop at these token counts
// (measured 1..11 % faster on the 32B-shaped layers).
// Neither operand passes through registers: global-to-LDS loads (16 bytes per lane, landing at a wavefront-uniform
// LDS base + 16 * lane) fill stages of half a chunk (64 k) --
//   X: two stages per workgroup, one multiplied while the other is filled, one barrier per stage;
//   W: three stages per wavefront (32 rows x 64 k, 4 KB): one multiplied, two on their way, so that a W transfer has
//      a whole chunk of time to arrive from HBM; non-temporal; private to the wavefront, or to the pair (each
//      fills its half of the pair's stage; the step barrier that publishes X publishes these too).
// A stage keeps rows of 128 bytes back to back (a load instruction fills 8 whole rows), so the 16-byte pieces of a
// row are stored permuted -- piece p of row r at slot p ^ ((r >> 1) & 7) -- which spreads the 16 lanes of a
// fragment read over all 64 banks without padding.  With no staging registers there is room for two fragment sets
// beside the accumulators of 256 tokens: the LDS reads of k step s + 1 run under the MFMAs of step s.
//
// The loads are written out as instructions.  Through the compiler's builtin every later LDS access of the kernel
// would wait for ALL loads in flight (the compiler cannot tell which LDS bytes a transfer writes), which stalls the
// transfers that are meant to stay in flight; and without a "memory" clobber, with which the same wait comes
// back: the barrier statements of the step loop, which have it, fence every read of a stage against the transfer
// that refills it, and volatile statements keep their order among themselves.  M0 carries the LDS base.  Since the
// compiler does not know of the loads, the waits are written out too: before the barrier of a step, vmcnt(4) -- the
// step's X transfers have landed, and with them the older W stage; only the 4 W transfers issued after them (the
// next step's stage) may still be in flight -- or vmcnt(0) in the last step, after which nothing was issued.
template <int MT, int RT, int WAVES>
__global__ __launch_bounds__(WAVES * kWave, 8 / WAVES) void skinny_gemm_stream_kernel(const GemmParams p) {
    static_assert(RT == 1 || (RT == 2 && MT % 2 == 0), "a pair of wavefronts splits the token tiles evenly");
    constexpr int TT = MT / RT;  // token tiles per wavefront
    constexpr int XROWS = 32 * MT;
    constexpr int XINSTR = XROWS / 8;
    constexpr int XI = (XINSTR + WAVES - 1) / WAVES;
    constexpr int kStageRow = 128;
    constexpr int XSTAGE = XROWS * kStageRow, WSTAGE = 32 * kStageRow;
    __shared__ __attribute__((aligned(1024))) unsigned char lds[2 * XSTAGE + WAVES * 3 * WSTAGE];
    const int tid = threadIdx.x, wave = tid / kWave, lane = tid & (kWave - 1);
    const int ln = lane & 31, hh = lane >> 5;
    // RT = 1: wavefront w owns row tile w and all tokens.  RT = 2: wavefronts 2j and 2j + 1 own row tiles 2j and
    // 2j + 1 together, each half of the token tiles, and share the W stages of their 64 rows.
    const int grp = RT == 1 ? wave : wave >> 1, th = RT == 1 ? 0 : wave & 1;
    const int n0 = blockIdx.x * (p.rows * WAVES) + grp * (p.rows * RT);  // pairs always own 2 x 32 rows
    const int chunks = p.K / kGemmChunk;
    const int c_lo = (int)((long long)blockIdx.y * chunks / p.ksplit);
    const int c_hi = (int)((long long)(blockIdx.y + 1) * chunks / p.ksplit);
    const int G = 2 * (c_hi - c_lo);  // half-chunk steps
    unsigned char* xs = lds;
    unsigned char* wsl = lds + 2 * XSTAGE + grp * (3 * RT * WSTAGE);

    // Per-lane source addresses of the transfers, for K offset 0 of the workgroup's range: 64-bit, so that neither
    // operand is limited to 4 GB.  lane -> (row of the instruction's 8, slot); the piece fetched for a slot is
    // slot ^ swizzle(row).
    const int l_row = lane >> 3, l_slot = lane & 7;
    const __bf16* x_src[XI];
    const __bf16* w_src[4];
#pragma unroll
    for (int i = 0; i < XI; ++i) {
        const int r = (wave + i * WAVES) * 8 + l_row;
        const int m = r < p.M ? r : p.M - 1;
        x_src[i] = p.X + (long long)m * p.ldx + (long long)c_lo * kGemmChunk + (l_slot ^ ((r >> 1) & 7)) * 8;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int r = th * 32 + i * 8 + l_row;  // of a pair, each wavefront brings in 32 of the 64 rows
        int n = n0 + (RT == 1 && r >= p.rows ? p.rows - 1 : r);  // a short tile re-reads its last row
        n = n < p.N ? n : p.N - 1;  // rows past the end re-read the last row; never stored
        w_src[i] = p.W + (long long)n * p.ldw + (long long)c_lo * kGemmChunk + (l_slot ^ ((r >> 1) & 7)) * 8;
    }
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"  // M0 is on the clobber list on purpose
    auto fetch_x = [&](int g) {
        unsigned char* stage = xs + (g & 1) * XSTAGE;
#pragma unroll
        for (int i = 0; i < XI; ++i) {
            const int j = wave + i * WAVES;
            if (j < XINSTR) {
                const unsigned lds_base = __builtin_amdgcn_readfirstlane(
                    (unsigned)(uintptr_t)(__attribute__((address_space(3))) void*)(stage + j * 8 * kStageRow));
                asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                             :
                             : "v"(x_src[i] + (long long)g * 64), "s"(lds_base)
                             : "m0");
            }
        }
    };
    auto fetch_w = [&](int g) {
        unsigned char* stage = wsl + (g % 3) * (RT * WSTAGE) + th * WSTAGE;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const unsigned lds_base = __builtin_amdgcn_readfirstlane(
                (unsigned)(uintptr_t)(__attribute__((address_space(3))) void*)(stage + i * 8 * kStageRow));
            asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off nt"
                         :
                         : "v"(w_src[i] + (long long)g * 64), "s"(lds_base)
                         : "m0");
        }
    };
#pragma clang diagnostic pop
    g_f32x16 acc[RT][TT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int t = 0; t < TT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[r][t][i] = 0.f;

    const int swz = (ln >> 1) & 7;
    auto multiply = [&](const unsigned char* xst, const unsigned char* wst) {
        g_bf16x8 fa[2][RT], fb[2][TT];
        auto frags = [&](int s, g_bf16x8 (&a)[RT], g_bf16x8 (&b)[TT]) {
#pragma unroll
            for (int r = 0; r < RT; ++r)
                a[r] = *reinterpret_cast<const g_bf16x8*>(wst + (r * 32 + ln) * kStageRow + (((2 * s + hh) ^ swz) * 16));
#pragma unroll
            for (int t = 0; t < TT; ++t)
                b[t] = *reinterpret_cast<const g_bf16x8*>(xst + ((th * TT + t) * 32 + ln) * kStageRow +
                                                          (((2 * s + hh) ^ swz) * 16));
        };
        frags(0, fa[0], fb[0]);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            if (s + 1 < 4) frags(s + 1, fa[(s + 1) & 1], fb[(s + 1) & 1]);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int t = 0; t < TT; ++t)
                    acc[r][t] =
                        __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[s & 1][r], fb[s & 1][t], acc[r][t], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    if (G > 0) {
        fetch_x(0);
        fetch_w(0);
        fetch_w(1);  // G is even: step 1 exists
    }
    for (int g = 0; g < G; ++g) {
        // issued after step g's X: the 4 W transfers of step g + 1, unless there is none
        if (g + 1 < G)
            asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        else
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (g + 1 < G) fetch_x(g + 1);
        if (g + 2 < G) fetch_w(g + 2);
        multiply(xs + (g & 1) * XSTAGE, wsl + (g % 3) * (RT * WSTAGE));
    }
    // register i of accumulator (r, t) of this lane: output row m = (th * TT + t) * 32 + ln,
    // column n = n0 + r * 32 + (i / 4) * 8 + hh * 4 + i % 4
#pragma unroll
    for (int t = 0; t < TT; ++t) {
        const int m = (th * TT + t) * 32 + ln;
        if (m >= p.M) continue;
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int n = n0 + r * 32 + q4 * 8 + hh * 4;
                if (RT == 1 && q4 * 8 + hh * 4 >= p.rows) continue;  // beyond a short tile (rows is a multiple of 4)
                if (n >= p.N) continue;  // N is a multiple of 8: the 4 columns are in or out together
                if (p.ksplit == 1) {
                    g_bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[r][t][q4 * 4 + e];
                    *reinterpret_cast<g_bf16x4*>(p.Y + (long long)m * p.ldy + n) = o;
                } else {
                    *reinterpret_cast<float4*>(p.part + ((long long)blockIdx.y * p.M + m) * p.N + n) = make_float4(
                        acc[r][t][q4 * 4 + 0], acc[r][t][q4 * 4 + 1], acc[r][t][q4 * 4 + 2], acc[r][t][q4 * 4 + 3]);
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
    const lotts::GemmPlan pl = lotts::plan_gemm(M, N, K);
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
    const GemmPlan pl = plan_gemm(M, N, K);
    GemmParams p;

    p.X = static_cast<const __bf16*>(X);
    p.W = static_cast<const __bf16*>(W);
    p.Y = static_cast<__bf16*>(Y);
    p.part = static_cast<float*>(workspace);
    p.M = M; p.N = N; p.K = K; p.ksplit = pl.ksplit; p.rows = pl.rows;
    p.ldx = ldx; p.ldw = ldw; p.ldy = ldy;
    hipStream_t s = (hipStream_t)stream;
    const dim3 grid(pl.nblocks, pl.ksplit), block4(4 * kWave), block8(8 * kWave);
    if (pl.stream) {
        switch (pl.mt) {
            case 1: LOTTS_LAUNCH((skinny_gemm_stream_kernel<1, 1, 8>), grid, block8, s, p); break;
            case 2: LOTTS_LAUNCH((skinny_gemm_stream_kernel<2, 1, 8>), grid, block8, s, p); break;
            case 3: LOTTS_LAUNCH((skinny_gemm_stream_kernel<3, 1, 8>), grid, block8, s, p); break;
            case 4: LOTTS_LAUNCH((skinny_gemm_stream_kernel<4, 2, 8>), grid, block8, s, p); break;
            case 5: LOTTS_LAUNCH((skinny_gemm_stream_kernel<5, 1, 8>), grid, block8, s, p); break;
            case 6: LOTTS_LAUNCH((skinny_gemm_stream_kernel<6, 2, 8>), grid, block8, s, p); break;
            case 7: LOTTS_LAUNCH((skinny_gemm_stream_kernel<7, 1, 8>), grid, block8, s, p); break;
            default: LOTTS_LAUNCH((skinny_gemm_stream_kernel<8, 2, 8>), grid, block8, s, p); break;
        }
    } else if (pl.mt == 1) {
        LOTTS_LAUNCH((skinny_gemm_stream_kernel<1, 1, 4>), grid, block4, s, p);
    } else if (pl.mt == 2) {
        LOTTS_LAUNCH((skinny_gemm_stream_kernel<2, 1, 4>), grid, block4, s, p);
    } else if (pl.mt == 3) {
        LOTTS_LAUNCH((skinny_gemm_stream_kernel<3, 1, 4>), grid, block4, s, p);
    } else {
        LOTTS_LAUNCH((skinny_gemm_stream_kernel<4, 2, 4>), grid, block4, s, p);
    }
    int rc = check_launch();
    if (rc != LOTTS_OK || pl.ksplit == 1) return rc;
    const long long quads = ((long long)M * N + 3) / 4;
    LOTTS_LAUNCH(skinny_gemm_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), s, p);
    return check_launch();
}
