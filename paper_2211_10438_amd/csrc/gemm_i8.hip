// INT8 x INT8 -> INT32 MFMA GEMM / batched GEMM for gfx950 with a fused dequantizing epilogue.
//
// Computes the integer contraction of Eq. 2, acc[m, n] = sum_k A[m, k] * B[n, k] (both operands
// K-contiguous: activations [T, C_i], prepared weights [C_o, C_i]), and applies the outer-dimension
// scaling of Eq. 2 (per-token Delta_X times Delta_W, optional bias / ReLU / residual) to the int32
// accumulators while they are still in registers.
//
// Design (CDNA4):
//  * v_mfma_i32_32x32x32_i8, one wave owns a (MI*32) x (NI*32) block of accumulators; the prefill
//    tiles (256x256, 256x192, 256x384) run 8 waves = 2 per SIMD, so one wave's barrier / LDS waits are
//    covered by the other wave's MFMAs.
//  * Operand tiles travel HBM -> LDS with global_load_lds_dwordx4 (no VGPR staging), NSTAGE deep.
//    LDS holds a tile as 16-row blocks of 1 KB, row-major (64 B per row) with the four 16-byte
//    K-chunks of a row XOR-permuted: (a) one wave-wide load instruction fills a block from 16 rows
//    x 64 contiguous bytes of global memory, four neighbouring lanes per row (coalesced), and (b)
//    the ds_read_b128 operand reads of the MFMAs spread over all banks.
//  * One s_barrier per 64-wide K step; operand fragments are double buffered in registers so the
//    LDS reads of the next half step are in flight while the MFMAs of this half step issue.
//  * Tiles are enumerated XCD-aware: the workgroups an XCD runs concurrently cover a compact
//    block of output tiles, so its L2 serves the shared A rows / B rows.
//  * Optional split-K writes int32 partial tiles to a workspace, reduced (exactly, int32) by a
//    second small kernel that also runs the epilogue.
#include <mutex>
#include <type_traits>

#include "gemm_args.h"

namespace {

enum { EPI_DEQUANT = 0, EPI_I32 = 1 };

// BM x BN output tile per workgroup, WGM x WGN waves, BK = 64 bytes of K per pipeline stage.
// BT = false: B is [N, K] (K-contiguous rows, like A).  BT = true: B is [K, N] (the V operand of
// attention's P V product): its tiles are read through registers, transposed bytewise in registers
// and written to the same LDS layout, so the MFMA loop is identical.
//
// LAY selects the operand layouts in global memory:
//   LAY_ROWS  A [M, K] and B [N, K] row-major (K contiguous);
//   LAY_BT    A row-major, B [K, N] (transposed, see above);
//   LAY_TILED A and B in the tiled layout of sq_layout SQ_TILED: 16-row x 64-byte blocks of 1 KB,
//             stored block-row-major, each block an exact image of the LDS block (chunk permutation
//             included).  One wave-wide load then copies 1 KB of contiguous global memory -- eight whole
//             128-byte lines instead of sixteen 64-byte row segments -- which is what the L2 -> CU path
//             serves best.
enum { LAY_ROWS = 0, LAY_BT = 1, LAY_TILED = 2 };

//
// ONESHOT (host guarantees K <= 64 * (NSTAGE - 1)): the whole K range is fetched up front into NSTAGE - 1
// buffers, no refills, no barriers in the K loop.  Used for attention scores (K = head_dim), where the
// kernel is bound by writing its output and several small workgroups per CU (OCC) overlap each other's
// load, MFMA and store phases.
//
// MF selects the MFMA shape: 32 = v_mfma_i32_32x32x32_i8 (two per 64-byte K step and accumulator block), 16 =
// v_mfma_i32_16x16x64_i8 (one per K step; a 1 KB LDS block is exactly one operand).  On quantized operands the matrix
// pipes draw less power per multiply-accumulate in the 16x16x64 shape (a register-fed loop of it sustains 4.1-4.2 POP/s
// under the socket's power cap where the 32x32x32 shape sustains 3.6), and the compute-bound tiles run at that cap.
template <int BM, int BN, int WGM, int WGN, int NSTAGE, int EPI, bool BF16, int LAY, int OCC = 1, bool ONESHOT = false, int MF = 32>
__global__ __launch_bounds__(WGM* WGN * 64, OCC) void gemm_i8_kernel(const GemmArgs p)
{
    constexpr bool BT = LAY == LAY_BT, TILED = LAY == LAY_TILED;
    constexpr int NW = WGM * WGN, BK = 64;
    constexpr int WM = BM / WGM, WN = BN / WGN, MI = WM / MF, NI = WN / MF;
    constexpr int AV = MF * MF / 64;  // accumulator registers per block
    constexpr int QG = AV / 4;        // runs of four neighbouring output columns a lane holds per block
    static_assert(MF == 32 || (MF == 16 && !BT && !ONESHOT && MI == 4 && NI % 2 == 0 && NI >= 6), "MFMA shape");
    constexpr int A_BYTES = BM * BK, B_BYTES = BN * BK, STAGE = A_BYTES + B_BYTES;
    constexpr int RBA = BM / 16, RBB = BN / 16;  // 16-row blocks per operand tile
    constexpr int SA = (RBA + NW - 1) / NW, SB = (RBB + NW - 1) / NW;  // BT: SB raw 1 KB blocks of the [64, BN] B tile
    constexpr int KR = BT ? BN / 16 : 0;  // BT: each lane transposes a KR (k) x 4 (n) byte block per stage
    constexpr int LPS = SA + SB;          // vector-memory loads per wave per stage
    static_assert(!BT || (NW == 4 && BN == 128 && RBB % NW == 0), "transposed-B path assumes 256 lanes and 128 columns");
    static_assert(WM % MF == 0 && WN % MF == 0, "wave tile must be a multiple of the MFMA block");
    static_assert(NSTAGE >= (BT ? 4 : 3) && (NSTAGE - 2) * LPS <= 63, "pipeline depth exceeds the 6-bit vmcnt");
    static_assert(NSTAGE * STAGE <= 160 * 1024, "LDS budget");
    // The epilogue stages the 16-bit tile in LDS; a tile too large for that goes in EG groups of GR rows.
    constexpr int EG = BM * (BN * 2 + 16) <= 160 * 1024 ? 1 : 2;
    constexpr int GR = BM / EG;
    constexpr int EPI_BYTES = EPI == EPI_DEQUANT ? GR * (BN * 2 + 16) : 0;
    // BT: behind the ring, three buffers hold the B tile in MFMA operand layout (see transpose_stage).
    constexpr int BOP = NSTAGE * STAGE;
    constexpr int RING_BYTES = (ONESHOT ? NSTAGE - 1 : NSTAGE) * STAGE + (BT ? 3 * B_BYTES : 0);
    constexpr int SMEM_BYTES = RING_BYTES > EPI_BYTES ? RING_BYTES : EPI_BYTES;
    static_assert(!ONESHOT || !BT, "one-shot loading is not combined with the transposed-B path");
    static_assert(SMEM_BYTES <= 160 * 1024, "LDS budget");
    __shared__ __attribute__((aligned(1024))) char smem[SMEM_BYTES];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    // ---- which tile: hardware deals consecutive workgroup ids round-robin to the 8 XCDs; give
    // each XCD a contiguous range of the logical order, and make that order walk groups of 8
    // m-tiles column by column so that concurrently running tiles share operand rows in L2.
    // Batched launches (attention heads) are enumerated the same way over (batch, tile) jointly: an XCD
    // then works through whole heads, and the tiles of a head that share its Q / K / V rows run together.
    const int64_t total = (int64_t)gridDim.x * gridDim.y;
    int64_t pid;
    {
        const int64_t wg = (int64_t)blockIdx.y * gridDim.x + blockIdx.x, j = wg >> 3;
        const int xcd = (int)(wg & 7);
        const int64_t q = total >> 3;
        const int r = (int)(total & 7);
        pid = xcd * q + (xcd < r ? xcd : r) + j;
    }
    const int tiles = p.tiles_m * p.tiles_n;
    const int per_batch = (int)gridDim.x;  // tiles * splits
    const int batch = (int)(pid / per_batch);
    const int pin = (int)(pid - (int64_t)batch * per_batch);
    const int split = pin / tiles;
    int tm, tn;
    {
        const int t = pin - split * tiles;
        constexpr int GM = 8;
        const int per_group = GM * p.tiles_n;
        const int g = t / per_group, first_m = g * GM;
        const int gsz = (p.tiles_m - first_m) < GM ? (p.tiles_m - first_m) : GM;
        const int in = t - g * per_group;
        tm = first_m + in % gsz;
        tn = in / gsz;
    }
    const int m0 = tm * BM, n0 = tn * BN;
    const int nk_total = (p.K + BK - 1) / BK;
    const int kbeg = split * p.iters_per_split;
    const int nk = (nk_total - kbeg) < p.iters_per_split ? (nk_total - kbeg) : p.iters_per_split;
    const int tail_chunks = (p.K & (BK - 1)) >> 4;  // valid 16-byte chunks of the last K step (0 = all 4)

    // Tiled operands: a 16-row block row is 16*K contiguous bytes and a K step advances 1 KB.
    constexpr int KSTEP = TILED ? 1024 : BK;
    const int8_t* Ab = p.A + (int64_t)batch * p.strideA + (int64_t)m0 * p.lda + (int64_t)kbeg * KSTEP;
    const int8_t* Bb = BT ? p.B + (int64_t)batch * p.strideB + n0
                          : p.B + (int64_t)batch * p.strideB + (int64_t)n0 * p.ldb + (int64_t)kbeg * KSTEP;

    // ---- global -> LDS load slots of this wave.  Slot i moves 16-row block (i*NW + wave), 1 KB per
    // stage.  Lane l lands at LDS byte l*16 of the block, i.e. the block is row-major (64 B per row),
    // and fetches row (l >> 2): four neighbouring lanes read one contiguous 64-byte segment, which
    // the vector memory path coalesces.  Inside a row the four 16-byte chunks are permuted
    // (position = chunk ^ swz(row)) so that the MFMA operand reads below stay bank-conflict free.
    auto swz = [](int r) { return ((r >> 1) & 3) ^ ((r >> 3) & 1); };
    const int chunk = (lane & 3) ^ swz(lane >> 2);
    uint32_t offA[SA], offB[SB + 1];
    int ldsA[SA], ldsB[SB + 1];
#pragma unroll
    for (int i = 0; i < SA; ++i) {
        const int rb = (i * NW + wave) % RBA;  // wraps only when RBA is not a multiple of NW: a benign duplicate
        if constexpr (TILED) {
            const int last_rb = (p.M - 1 - m0) >> 4;  // ragged M: re-read the last valid block row
            offA[i] = (uint32_t)((rb < last_rb ? rb : last_rb) * 16 * (int)p.lda + lane * 16);
        } else {
            int row = rb * 16 + (lane >> 2);
            const int last = p.M - 1 - m0;
            row = row < last ? row : last;
            offA[i] = (uint32_t)(row * (int)p.lda + chunk * 16);
        }
        ldsA[i] = rb * 1024;
    }
    // BT: raw block (i*NW + wave) holds 1024/BN consecutive k rows of the stage, BN/16 lanes per row.
    int rawrow[SB + 1], rawcol = 0;
    if constexpr (BT) {
        rawcol = (lane % (BN / 16)) * 16;
        if (n0 + rawcol + 16 > p.N) rawcol = p.N - 16 - n0;  // ragged N tile: re-read valid columns (N % 16 == 0)
#pragma unroll
        for (int i = 0; i < SB; ++i) {
            rawrow[i] = (i * NW + wave) * (1024 / BN) + lane / (BN / 16);
            ldsB[i] = A_BYTES + (i * NW + wave) * 1024;
        }
    }
#pragma unroll
    for (int i = 0; i < (BT ? 0 : SB); ++i) {
        const int rb = (i * NW + wave) % RBB;
        if constexpr (TILED) {
            const int last_rb = (p.N - 1 - n0) >> 4;
            offB[i] = (uint32_t)((rb < last_rb ? rb : last_rb) * 16 * (int)p.ldb + lane * 16);
        } else {
            int row = rb * 16 + (lane >> 2);
            const int last = p.N - 1 - n0;
            row = row < last ? row : last;
            offB[i] = (uint32_t)(row * (int)p.ldb + chunk * 16);
        }
        ldsB[i] = A_BYTES + rb * 1024;
    }

    // K tail (K % 64 != 0 happens only in the globally last K step): lanes whose chunk lies beyond K
    // re-read chunk 0 (valid memory); their A fragments are zeroed in registers before the MFMAs.
    const bool has_tail = tail_chunks != 0 && (kbeg + nk == nk_total);
    auto issue_stage = [&](int kt, int buf) {
        const int8_t* a = Ab + (int64_t)kt * KSTEP;
        const int8_t* b = Bb + (int64_t)kt * KSTEP;
        char* base = smem + buf * STAGE;
        const uint32_t back = (has_tail && kt == nk - 1 && chunk >= tail_chunks) ? (uint32_t)chunk * 16u : 0u;
#pragma unroll
        for (int i = 0; i < SA; ++i)
            __builtin_amdgcn_global_load_lds(GPTR(a + (offA[i] - back)), LPTR(base + ldsA[i]), 16, 0, 0);
        if constexpr (BT) {
            // raw [64, BN] tile of B = [K, N]; rows past K (K tail) re-read row K-1, where the A fragments are zero
#pragma unroll
            for (int i = 0; i < SB; ++i) {
                int k = (kbeg + kt) * BK + rawrow[i];
                k = k < p.K ? k : p.K - 1;
                __builtin_amdgcn_global_load_lds(GPTR(Bb + (int64_t)k * p.ldb + rawcol), LPTR(base + ldsB[i]), 16, 0, 0);
            }
        } else {
#pragma unroll
            for (int i = 0; i < SB; ++i)
                __builtin_amdgcn_global_load_lds(GPTR(b + (offB[i] - back)), LPTR(base + ldsB[i]), 16, 0, 0);
        }
    };

    // ---- transposed-B path.  The raw [64 k, BN n] tile of a stage arrives in the ring like A does (LDS-DMA,
    // NSTAGE deep, so no global-memory latency sits in the K loop).  One K step before a stage is consumed
    // every lane reads a KR (k) x 4 (n) byte block of it from LDS, transposes it bytewise in registers
    // (v_perm_b32) and writes it, n-major, into one of three operand-layout buffers behind the ring; the
    // MFMA loop then reads B fragments from there exactly as it reads them from the ring otherwise.
    const int bt_cg = BT ? (int)(threadIdx.x % (BN / 4)) : 0;   // column group: columns 4*cg .. 4*cg+3
    const int bt_ks = BT ? (int)(threadIdx.x / (BN / 4)) : 0;   // k slab: rows ks*KR .. ks*KR+KR-1 of the stage
    auto transpose_stage = [&](int ring_buf, int op_buf) {
        if constexpr (BT) {
            const char* raw = smem + ring_buf * STAGE + A_BYTES + (bt_ks * KR) * BN + bt_cg * 4;
            uint32_t breg[KR + 1];
#pragma unroll
            for (int j = 0; j < KR; ++j) breg[j] = *(const uint32_t*)(raw + j * BN);
            // 4x4 byte transposes: out[e][m] = bytes e of rows 4m .. 4m+3
            uint32_t out[4][KR / 4 + 1];
#pragma unroll
            for (int m = 0; m < KR / 4; ++m) {
                const uint32_t r0 = breg[4 * m], r1 = breg[4 * m + 1], r2 = breg[4 * m + 2], r3 = breg[4 * m + 3];
                const uint32_t t0 = __builtin_amdgcn_perm(r1, r0, 0x05010400u), t1 = __builtin_amdgcn_perm(r1, r0, 0x07030602u);
                const uint32_t u0 = __builtin_amdgcn_perm(r3, r2, 0x05010400u), u1 = __builtin_amdgcn_perm(r3, r2, 0x07030602u);
                out[0][m] = __builtin_amdgcn_perm(u0, t0, 0x05040100u);
                out[1][m] = __builtin_amdgcn_perm(u0, t0, 0x07060302u);
                out[2][m] = __builtin_amdgcn_perm(u1, t1, 0x05040100u);
                out[3][m] = __builtin_amdgcn_perm(u1, t1, 0x07060302u);
            }
            char* base = smem + BOP + op_buf * B_BYTES;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int n = bt_cg * 4 + e, r = n & 15;
                const int pos = (bt_ks >> 1) ^ swz(r);  // KR = 8: a lane holds half a 16-byte chunk
                *(v2u*)(base + (n >> 4) * 1024 + r * 64 + pos * 16 + (bt_ks & 1) * 8) = v2u{out[e][0], out[e][1]};
            }
        }
    };

    // ---- MFMA operand fragments.  For the 32x32x32 MFMA lane l feeds row (l & 31) with the 16
    // bytes of K-chunk kk*2 + (l >> 5) of the 64-wide K step; chunk c of row r sits at position
    // c ^ swz(r), and kk only flips bit 1 of the position: byte address ^ 32.
    // For the 16x16x64 MFMA lane l feeds row (l & 15) with the 16 bytes of K-chunk (l >> 4): one 1 KB block, whole.
    const int frow = lane & 15;
    const int lane_off = MF == 32 ? ((lane & 31) >> 4) * 1024 + frow * 64 + (((lane >> 5) ^ swz(frow)) * 16)
                                  : frow * 64 + (((lane >> 4) ^ swz(frow)) * 16);
    const int fragA0 = wm * (WM / 16) * 1024 + lane_off;
    const int fragB0 = (BT ? 0 : A_BYTES) + wn * (WN / 16) * 1024 + lane_off;

    typedef int acc_t __attribute__((ext_vector_type(AV)));
    acc_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int v = 0; v < AV; ++v) acc[i][j][v] = 0;

    if constexpr (MF == 32) {
    v4i fa0[MI], fb0[NI], fa1[MI], fb1[NI];

    auto read_frags = [&](v4i(&fa)[MI], v4i(&fb)[NI], int buf, int kk, int op_buf) {
        const char* sa = smem + buf * STAGE + (fragA0 ^ (kk * 32));
        const char* sb = smem + (BT ? BOP + op_buf * B_BYTES : buf * STAGE) + (fragB0 ^ (kk * 32));
#pragma unroll
        for (int i = 0; i < MI; ++i) fa[i] = *(const v4i*)(sa + i * 2048);
#pragma unroll
        for (int j = 0; j < NI; ++j) fb[j] = *(const v4i*)(sb + j * 2048);
    };
    auto mfma_all = [&](const v4i(&fa)[MI], const v4i(&fb)[NI]) {
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[j], fa[i], acc[i][j], 0, 0, 0);
    };
    // (B rows feed the MFMA's first operand: each accumulator block is the transpose of its 32x32 output
    // block, so a lane ends up with runs of four neighbouring output columns of one row -- see the epilogue.)
    // Scheduling hint for one half step (MI+NI fragment reads of the next half, MI*NI MFMAs of this
    // one): interleave the LDS reads with the MFMAs so the four waves of the workgroup do not hit
    // the LDS pipe in one burst.
    auto interleave_hint = [&](auto NV) {
        // one MFMA, one DS read (and, in the half step that refills a buffer, one global->LDS load)
        // per group; the MFMAs left over close the half step, which gives the last read time to land
        // before the next half step waits for it.
        constexpr int READS = MI + NI, MFMAS = MI * NI, VMEM = decltype(NV)::value;
        constexpr int GROUPS = READS > VMEM ? READS : VMEM;
#pragma unroll
        for (int r = 0; r < GROUPS; ++r) {
            if (r < MFMAS) __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (r < VMEM) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            if (r < READS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        if (MFMAS > GROUPS) __builtin_amdgcn_sched_group_barrier(0x008, MFMAS - GROUPS, 0);
    };

    // ---- pipeline prologue: stages 0 .. NSTAGE-2 in flight, stage 0 landed, first fragments read.
    // Every K step issues exactly one stage of loads; past the end of the K range the last stage is
    // simply fetched again into a buffer nobody reads.  That keeps the number of loads in flight
    // constant (one immediate s_waitcnt value) and the loop body free of branches, so the loads and
    // LDS reads can be interleaved with the MFMAs by the scheduler hints below.
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) {
        if constexpr (ONESHOT) {
            if (s < nk) issue_stage(s, s);
        } else {
            issue_stage(s < nk ? s : nk - 1, s);
        }
    }
    if constexpr (ONESHOT) {
        wait_vmcnt_imm<0>();
    } else if constexpr (BT) {
        // stages 0 and 1 landed; their B tiles go to operand buffers 0 and 1
        wait_vmcnt_imm<(NSTAGE - 3) * LPS>();
        __builtin_amdgcn_s_barrier();
        transpose_stage(0, 0);
        transpose_stage(1, 1);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    } else {
        wait_vmcnt_imm<(NSTAGE - 2) * LPS>();
    }
    __builtin_amdgcn_s_barrier();
    read_frags(fa0, fb0, 0, 0, 0);

    int buf = 0, ob = 0;  // ring buffer and operand buffer of the current K step
    for (int it = 0; it < nk - 1; ++it) {
        // first half of K step `it`
        read_frags(fa1, fb1, buf, 1, ob);
        mfma_all(fa0, fb0);
        interleave_hint(std::integral_constant<int, 0>{});
        // second half; meanwhile make stage it+1 visible and refill the buffer freed by step it-1
        const int nbuf = buf + 1 == NSTAGE ? 0 : buf + 1;
        const int nob = ob == 2 ? 0 : ob + 1;
        if constexpr (!ONESHOT) {
            // BT needs stage it+2 landed (its B tile is transposed now, for the step after next)
            wait_vmcnt_imm<(NSTAGE - (BT ? 4 : 3)) * LPS>();
            __builtin_amdgcn_s_barrier();
            if constexpr (BT) transpose_stage(buf + 2 >= NSTAGE ? buf + 2 - NSTAGE : buf + 2, ob == 0 ? 2 : ob - 1);
            issue_stage(it + NSTAGE - 1 < nk ? it + NSTAGE - 1 : nk - 1, buf == 0 ? NSTAGE - 1 : buf - 1);
        }
        read_frags(fa0, fb0, nbuf, 0, nob);
        mfma_all(fa1, fb1);
        interleave_hint(std::integral_constant<int, (BT || ONESHOT) ? 0 : SA + SB>{});
        buf = nbuf;
        ob = nob;
    }
    // last K step
    read_frags(fa1, fb1, buf, 1, ob);
    if (has_tail) {
        // chunk index of this lane inside the 64-byte step: kk*2 + (lane >> 5)
        const int c0 = lane >> 5, c1 = 2 + (lane >> 5);
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            if (c0 >= tail_chunks) fa0[i] = v4i{0, 0, 0, 0};
            if (c1 >= tail_chunks) fa1[i] = v4i{0, 0, 0, 0};
        }
    }
    mfma_all(fa0, fb0);
    mfma_all(fa1, fb1);
    } else {
    // ---- 16x16x64 shape.  A wave owns 64 rows x WN columns.  Its four A fragments of a K step stay in registers for the
    // whole step (the next step's four are read meanwhile into a second set); the NI B fragments come in NP parts of
    // two, double buffered: while the 8 MFMAs of a part issue, the two fragments of the next part are read.
    // Per step 4 + NI reads of 1 KB and 4 NI MFMAs.  The barrier that publishes stage it + 1 sits in front of the third
    // part from the end; the reads that belong to the next step (its A fragments, its first part of B) come after it.
    constexpr int NQ = 2, NP = NI / NQ, PB = NP - 3;
    static_assert(PB >= 0, "parts of a K step");
    v4i fa[2][MI], fbq[2][NQ];
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) issue_stage(s < nk ? s : nk - 1, s);
    wait_vmcnt_imm<(NSTAGE - 2) * LPS>();
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int i = 0; i < MI; ++i) fa[0][i] = *(const v4i*)(smem + fragA0 + i * 1024);
#pragma unroll
    for (int k = 0; k < NQ; ++k) fbq[0][k] = *(const v4i*)(smem + fragB0 + k * 1024);

    // Every step is the same code: the last one also reads "next" fragments (from a buffer that holds an old stage:
    // valid LDS, values never used) and refills a buffer nobody reads.  The host sends only K ranges of an even number
    // of whole steps here (K % 128 == 0, no K split), so the loop runs in pairs and there is no second copy of the step
    // outside it (with one, the register allocation of the epilogue spilled hundreds of registers per lane).
    // P0: which of the two B fragment sets the step's first part finds filled (with an odd number of parts per step the
    // two steps of the unrolled pair start on different sets).
    auto step = [&](auto P0_, v4i(&cur)[MI], v4i(&nxt)[MI], int it, int buf) {
        constexpr int P0 = decltype(P0_)::value;
        const int nbuf = buf + 1 == NSTAGE ? 0 : buf + 1;
        const char* sb = smem + buf * STAGE + fragB0;
        const char* sn = smem + nbuf * STAGE;
        // the stage this step fetches (past the end of the K range the last one again), into the buffer of step it - 1
        const int kt = it + NSTAGE - 1 < nk ? it + NSTAGE - 1 : nk - 1;
        const int8_t* ga = Ab + (int64_t)kt * KSTEP;
        const int8_t* gb = Bb + (int64_t)kt * KSTEP;
        char* refill = smem + (buf == 0 ? NSTAGE - 1 : buf - 1) * STAGE;
        static_for<NP>([&](auto Q_) {
            constexpr int q = decltype(Q_)::value;
            if constexpr (q == PB) {
                wait_vmcnt_imm<(NSTAGE - 3) * LPS>();
                __builtin_amdgcn_s_barrier();
            }
            // next step's A fragments: two each in the last two parts.  (None in the first part behind the barrier: there
            // the eight waves run in step and their stage loads and reads meet in the LDS; with two of the four reads
            // there the whole step took an eighth longer.)
            constexpr int pa = q - PB;  // parts behind the barrier so far
            constexpr int an0 = pa <= 1 ? 0 : 2;
            constexpr int an_cnt = pa <= 0 ? 0 : 2;
            // The part in the instruction stream, fixed by scheduling fences: its first MFMA (in front of it the wait
            // for this part's fragments, which is exact there: nothing younger is in flight), then the reads of the
            // next part and, behind the barrier, the stage's global->LDS loads, then the other seven MFMAs, which
            // cover the latency of those reads.
            acc[0][q * NQ] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fbq[(q + P0) & 1][0], cur[0], acc[0][q * NQ], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (q >= PB) {
                // the stage's loads (the first SA are A blocks, the others B blocks), spread over the parts behind the
                // barrier: issued in one burst they cost an eighth more time per step
                constexpr int per = (LPS + NP - PB - 1) / (NP - PB), i0 = (q - PB) * per, i1 = i0 + per < LPS ? i0 + per : LPS;
                static_for<(i1 > i0 ? i1 - i0 : 0)>([&](auto D_) {
                    constexpr int i = i0 + decltype(D_)::value;
                    // (the offset is made opaque here so that its widening to 64 bits stays next to the load: hoisted out
                    // of the loop it costs a register pair per load and the scalar-base addressing form)
                    uint32_t o = i < SA ? offA[i < SA ? i : 0] : offB[i < SA ? 0 : i - SA];
                    asm volatile("" : "+v"(o));
                    if constexpr (i < SA) __builtin_amdgcn_global_load_lds(GPTR(ga + o), LPTR(refill + ldsA[i]), 16, 0, 0);
                    else __builtin_amdgcn_global_load_lds(GPTR(gb + o), LPTR(refill + ldsB[i - SA]), 16, 0, 0);
                });
            }
            if constexpr (q < NP - 1) {
#pragma unroll
                for (int k = 0; k < NQ; ++k) fbq[(q + 1 + P0) & 1][k] = *(const v4i*)(sb + ((q + 1) * NQ + k) * 1024);
            } else {
#pragma unroll
                for (int k = 0; k < NQ; ++k) fbq[(q + 1 + P0) & 1][k] = *(const v4i*)(sn + fragB0 + k * 1024);
            }
            static_for<an_cnt>([&](auto K_) {
                constexpr int k = an0 + decltype(K_)::value;
                nxt[k] = *(const v4i*)(sn + fragA0 + k * 1024);
            });
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < NQ; ++k)
#pragma unroll
                for (int i = 0; i < MI; ++i)
                    if (k + i > 0)
                        acc[i][q * NQ + k] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fbq[(q + P0) & 1][k], cur[i], acc[i][q * NQ + k], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    int buf = 0;
    for (int it = 0; it < nk; it += 2) {
        step(std::integral_constant<int, 0>{}, fa[0], fa[1], it, buf);
        buf = buf + 1 == NSTAGE ? 0 : buf + 1;
        step(std::integral_constant<int, NP & 1>{}, fa[1], fa[0], it + 1, buf);
        buf = buf + 1 == NSTAGE ? 0 : buf + 1;
    }
    }
    wait_vmcnt_imm<0>();  // the refills issued past the end of the K range have landed

    // ---- epilogue.  Accumulator block (i, j) is the transposed 32x32 output block: lane l, register v
    // holds output row (l & 31), column 8*(v/4) + 4*(l >> 5) + (v & 3) of the block, i.e. registers
    // 4g .. 4g+3 are four neighbouring columns of one row.  (16x16 blocks: row (l & 15), columns 4*(l >> 4) + v.)
    const int row_l = lane & (MF - 1), col_l = (lane >> (MF == 32 ? 5 : 4)) * 4;
    if constexpr (EPI == EPI_I32) {
        int32_t* out = p.acc_out + ((int64_t)split * p.M) * p.N;
        const bool vec4 = (p.N & 3) == 0;  // 16-byte stores stay aligned and inside the row
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            const int row = m0 + wm * WM + i * MF + row_l;
            if (row < p.M) {
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int g = 0; g < QG; ++g) {
                        const int col = n0 + wn * WN + j * MF + 8 * g + col_l;
                        int32_t* dst = out + (int64_t)row * p.N + col;
                        if (vec4 && col < p.N) {
                            *(v4i*)dst = v4i{acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (col + e < p.N) dst[e] = acc[i][j][4 * g + e];
                        }
                    }
            }
        }
    } else {
        // The 16-bit tile is staged in LDS (free once the K loop is over) so that global memory is
        // written in whole 512-byte row segments, 16 bytes per lane, instead of 2-byte scatters; the
        // residual tile is fetched the same way.  Row pitch +16 B keeps the two half-waves (4 rows
        // apart) on different banks.
        constexpr int PITCH = BN * 2 + 16;
        constexpr int CPR = BN / 8;  // 16-byte chunks per tile row
        static_assert(GR * PITCH <= SMEM_BYTES && GR % 32 == 0, "epilogue staging must fit in the LDS allocation");
        uint16_t* C = (uint16_t*)p.C + (int64_t)batch * p.strideC;
        const uint16_t* R = (const uint16_t*)p.residual;
        const bool vec_ok = (p.N & 7) == 0;  // 16-byte chunks never straddle the row end and stay aligned
        const float ws = (p.x_scale && !p.w_per_channel) ? p.w_scale[0] : 0.0f;
        const float xs0 = (p.x_scale && !p.per_token) ? p.x_scale[0] : 0.0f;
        // Accumulators to fp32 in place, before anything else of the epilogue: the conversion does not depend on the
        // row group or on the optional terms, so the compiler moves it in front of the loop and the switch below
        // anyway, and into new registers if left to itself (the 384-wide tile then spilled thirty per lane).
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                typedef float accf_t __attribute__((ext_vector_type(AV)));
                acc[i][j] = __builtin_bit_cast(acc_t, __builtin_convertvector(acc[i][j], accf_t));
            }
        float rq = 0.0f;
        if (p.q8_step) {
            const float delta = p.q8_step[0];
            rq = delta > 0.0f ? 1.0f / delta : 0.0f;
        }
#pragma unroll
        for (int eg = 0; eg < EG; ++eg) {
        const int g0 = eg * GR;  // first tile row of this group
        // A zero the compiler cannot see through, added to the row and column offsets below: without it every index,
        // bounds predicate and bias / scale address of all variants of phase1 counts as independent of the row group and
        // is computed in front of this loop, where some ninety such values stay live next to the accumulators.
        int opaque0;
        asm volatile("s_mov_b32 %0, 0" : "=s"(opaque0));
        __syncthreads();  // operand reads (first group) or the previous group's stores out of LDS are done
        if (R) {
            for (int q = threadIdx.x; q < GR * CPR; q += NW * 64) {
                const int r = q / CPR, c8 = (q - r * CPR) * 8;
                const int row = m0 + g0 + r, col = n0 + c8;
                v4u val = {0, 0, 0, 0};
                if (row < p.M && col < p.N) {
                    const uint16_t* src = R + (int64_t)row * p.N + col;
                    if (vec_ok) {
                        val = *(const v4u*)src;
                    } else {
                        uint32_t e[8];
#pragma unroll
                        for (int t = 0; t < 8; ++t) e[t] = (col + t < p.N) ? src[t] : 0u;
                        val = v4u{e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16)};
                    }
                }
                *(v4u*)(smem + r * PITCH + c8 * 2) = val;
            }
            __syncthreads();
        }
        // The optional terms are compile-time flags inside the loop (one uniform switch outside) so the
        // common cases cost convert + multiply + round per element and one 8-byte LDS write per four.
        auto phase1 = [&](auto HB, auto RL, auto HR) {
            constexpr bool has_bias = decltype(HB)::value, relu = decltype(RL)::value, has_res = decltype(HR)::value;
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                if (EG > 1 && (wm * WM + i * MF) / GR != eg) continue;  // rows of another group
                const int lrow = wm * WM + i * MF + row_l - g0 + opaque0;
                const int row = m0 + g0 + lrow;
                const float xrow = p.x_scale ? (p.per_token ? p.x_scale[row < p.M ? row : p.M - 1] : xs0) : 0.0f;
                float c;
                if (p.x_scale) c = xrow * ws;
                else c = p.alpha;
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int g = 0; g < QG; ++g) {
                        const int lcol = wn * WN + j * MF + 8 * g + col_l + opaque0;
                        float cq[4] = {c, c, c, c};
                        if (p.w_per_channel) {  // c = Delta_X[row] * Delta_W[col]
#pragma unroll
                            for (int e = 0; e < 4; ++e) cq[e] = xrow * ((n0 + lcol + e < p.N) ? p.w_scale[n0 + lcol + e] : 0.0f);
                        }
                        float bq[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                        if constexpr (has_bias) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) bq[e] = (n0 + lcol + e < p.N) ? p.bias[n0 + lcol + e] : 0.0f;
                        }
                        v2u* slot = (v2u*)(smem + lrow * PITCH + lcol * 2);
                        v2u rb = {0u, 0u};
                        if constexpr (has_res) rb = *slot;
                        auto fa = [&](int e) {
                            const int bits = acc[i][j][4 * g + e];  // a copy: a vector element is no object to cast from
                            return __builtin_bit_cast(float, bits);
                        };
                        const uint32_t o01 = dequant_pair_f<BF16>(fa(0), fa(1), cq[0], cq[1], bq[0], bq[1], has_bias, relu, rb[0], has_res);
                        const uint32_t o23 = dequant_pair_f<BF16>(fa(2), fa(3), cq[2], cq[3], bq[2], bq[3], has_bias, relu, rb[1], has_res);
                        *slot = v2u{o01, o23};
                    }
            }
        };
        using T_ = std::true_type;
        using F_ = std::false_type;
        switch ((p.bias ? 1 : 0) | (p.relu ? 2 : 0) | (R ? 4 : 0)) {
            case 0: phase1(F_{}, F_{}, F_{}); break;
            case 1: phase1(T_{}, F_{}, F_{}); break;
            case 2: phase1(F_{}, T_{}, F_{}); break;
            case 3: phase1(T_{}, T_{}, F_{}); break;
            case 4: phase1(F_{}, F_{}, T_{}); break;
            case 5: phase1(T_{}, F_{}, T_{}); break;
            case 6: phase1(F_{}, T_{}, T_{}); break;
            default: phase1(T_{}, T_{}, T_{}); break;
        }
        __syncthreads();
        // int8 codes in the tiled layout leave in another order: a wave instruction covers 8 rows x 64 columns, which are
        // 512 contiguous bytes of a 1 KB block (walking along a row it would write 64-byte pieces of eight blocks)
        const bool q8_blocks = p.q8_step && p.q8_tiled && (BN % 64 == 0);
        for (int q = threadIdx.x; q < GR * CPR; q += NW * 64) {
            int r = q / CPR, c8 = (q - r * CPR) * 8;
            if (q8_blocks) {
                const int blk = q >> 6, cb = blk % (BN / 64);
                r = (blk / (BN / 64)) * 8 + ((q >> 3) & 7);
                c8 = (cb * 8 + (q & 7)) * 8;
            }
            const int row = m0 + g0 + r, col = n0 + c8;
            if (row < p.M && col < p.N) {
                const v4u val = *(const v4u*)(smem + r * PITCH + c8 * 2);
                if (p.q8_step) {
                    // int8 output: quantize the eight 16-bit values of this chunk (they never straddle a
                    // 16-byte chunk of the tiled layout) and store 8 codes
                    // (clamp + add of 1.5 * 2^23: the code in the low byte, the same integer as requant_code's rint + clamp)
                    uint32_t cq[8];
#pragma unroll
                    for (int t = 0; t < 8; ++t) cq[t] = code_bits(load16_bits<BF16>(val[t >> 1] >> ((t & 1) * 16)) * rq);
                    int8_t* dq = code_dst(p.q8_out, row, col, p.N, p.q8_tiled != 0);
                    if (vec_ok) {
                        *(v2u*)dq = v2u{pack4_low_bytes(cq[0], cq[1], cq[2], cq[3]), pack4_low_bytes(cq[4], cq[5], cq[6], cq[7])};
                    } else {
#pragma unroll
                        for (int t = 0; t < 8; ++t)
                            if (col + t < p.N) dq[t] = (int8_t)(cq[t] & 0xffu);
                    }
                    continue;
                }
                uint16_t* dst = C + (int64_t)row * p.N + col;
                if (vec_ok) {
                    __builtin_nontemporal_store(val, (v4u*)dst);
                } else {
#pragma unroll
                    for (int t = 0; t < 8; ++t)
                        if (col + t < p.N) dst[t] = (uint16_t)(val[t >> 1] >> ((t & 1) * 16));
                }
            }
        }
        }  // row groups
    }
}

// Split-K reduction: sums the int32 partial tiles (exact) and applies the same epilogue.
template <bool BF16>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const GemmArgs p, int to_i32)
{
    const int64_t total = (int64_t)p.M * p.N;
    for (int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * blockDim.x) {
        int sum = 0;
        for (int s = 0; s < p.splits; ++s) sum += p.acc_out[(int64_t)s * total + idx];
        const int row = (int)(idx / p.N), col = (int)(idx - (int64_t)row * p.N);
        if (to_i32) {
            ((int32_t*)p.C)[idx] = sum;
        } else {
            float c;
            if (p.x_scale) c = (p.per_token ? p.x_scale[row] : p.x_scale[0]) * p.w_scale[p.w_per_channel ? col : 0];
            else c = p.alpha;
            const uint16_t* R = (const uint16_t*)p.residual;
            const uint32_t o = dequant_one<BF16>(sum, c, p.bias ? p.bias[col] : 0.0f, p.bias != nullptr, p.relu != 0,
                                                 R ? R[idx] : 0u, R != nullptr);
            if (p.q8_step) {
                const float delta = p.q8_step[0];
                code_dst(p.q8_out, row, col & ~7, p.N, p.q8_tiled != 0)[col & 7] =
                    (int8_t)requant_code<BF16>(o, delta > 0.0f ? 1.0f / delta : 0.0f);
            } else {
                ((uint16_t*)p.C)[idx] = (uint16_t)o;
            }
        }
    }
}

// ---------------------------------------------------------------- host side: tile / split choice

constexpr int kNumCU = 256;

struct Plan {
    int cfg;     // 0: 256x256 (prefill)  1: 128x256  2: 64x256  3: 32x256  5: 256x128 B^T  6: 256x192
                 // 7: 128x128, three workgroups per CU (short K: the output stream dominates)
                 // 8: 128x128, K <= 128 fetched in one go, four workgroups per CU
                 // 9: 256x384 (a round of tiles saved on wide outputs)
                 // 10, 11, 12: 256x256, 256x384 and 256x192 with the 16x16x64 MFMA
    int bm, bn;
    int splits, iters_per_split;
    int tiles_m, tiles_n;
};

Plan make_plan(int64_t M, int64_t N, int64_t K, int64_t batch, bool allow_split, bool b_transposed = false)
{
    Plan pl{};
    pl.bn = 256;
    if (b_transposed) {
        pl.bm = 256;
        pl.cfg = 5;
        pl.bn = 128;
        allow_split = false;
    }
    else if (M > 128 && K <= 128) {
        // The same, with the whole K range fetched in one go and four workgroups per CU.
        pl.cfg = 8;
        pl.bm = 128;
        pl.bn = 128;
        allow_split = false;
    }
    else if (M > 128 && K <= 256) {
        // Two to four K steps per tile (attention scores, K = head_dim): loading, MFMAs and the epilogue of
        // one tile cannot overlap each other, so several small workgroups share a CU and overlap between
        // themselves; the kernel is bound by writing the output.
        pl.cfg = 7;
        pl.bm = 128;
        pl.bn = 128;
        allow_split = false;
    }
    else if (M > 128) {
        // Compute-bound shapes: time = rounds of tiles over the 256 CUs x cost of one tile; pick the cheapest width.
        // Cost of a tile in microseconds, measured on quantized Gaussian operands (the clock that the power cap allows
        // is part of these figures): K steps x 0.59 + 10 (256x192: fewer MFMAs per operand fragment read), x 0.70 + 18
        // (256x256), x 1.12 + 8 (256x384: 192 accumulator registers per lane, the whole 160 KB of LDS, the epilogue in
        // two halves) with the 32x32x32 MFMA; the 256- and 384-wide tiles also exist with the 16x16x64 MFMA, which
        // draws less power per multiply-accumulate: x 0.66 + 18 and x 1.03 + 8; the 192-wide one too, x 0.52 + 14 (a
        // 5-stage ring: the barrier of a step sits at its start), taken from 192 K steps on.  That form needs an even
        // number of whole K steps and no K split (see the kernel); other shapes keep the 32x32x32 form.
        pl.cfg = 0;
        pl.bm = 256;
        const bool mf16 = (K & 127) == 0;
        const int64_t tm = (M + 255) / 256;
        const int64_t rounds256 = (tm * ((N + 255) / 256) * batch + kNumCU - 1) / kNumCU;
        const int64_t rounds192 = (tm * ((N + 191) / 192) * batch + kNumCU - 1) / kNumCU;
        const int64_t rounds384 = (tm * ((N + 383) / 384) * batch + kNumCU - 1) / kNumCU;
        const double nks = (double)((K + 63) / 64);
        const bool mf16_192 = mf16 && nks >= 192.0;  // (its longer ring costs more per tile: it pays on long K ranges only)
        const double t192 = rounds192 * (mf16_192 ? nks * 0.522 + 14.0 : nks * 0.588 + 10.0);
        const double t256 = rounds256 * (nks * (mf16 ? 0.66 : 0.70) + 18.0);
        const double t384 = rounds384 * (nks * (mf16 ? 1.03 : 1.12) + 8.0);
        double t_now = t256;
        if (t192 < t256) { pl.cfg = 6; pl.bn = 192; t_now = t192; }
        if (t384 < 0.98 * t_now) { pl.cfg = 9; pl.bn = 384; }
    }
    else if (M > 64) { pl.cfg = 1; pl.bm = 128; }
    else if (M > 32) { pl.cfg = 2; pl.bm = 64; }
    else { pl.cfg = 3; pl.bm = 32; }
    pl.tiles_m = (int)((M + pl.bm - 1) / pl.bm);
    pl.tiles_n = (int)((N + pl.bn - 1) / pl.bn);
    const int nk = (int)((K + 63) / 64);
    int splits = 1;
    if (allow_split && batch == 1) {
        const int64_t tiles = (int64_t)pl.tiles_m * pl.tiles_n;
        const int max_splits = nk / 8 > 0 ? nk / 8 : 1;  // at least 8 K steps per split
        if (pl.bm == 256) {
            // Compute-bound tiles: a K split pays (int32 partials through HBM, a second kernel), so it is chosen
            // by a small time model in microseconds: rounds x (K steps x 0.7 + 12 for fill and epilogue), plus,
            // when split, 5 for the reduction launch and the partials written and read back at about 4 TB/s
            // (the write overlaps the GEMM half way).
            double best = 1e30;
            for (int sp = 1; sp <= 8 && sp <= max_splits; ++sp) {
                const int64_t rounds = (tiles * sp + kNumCU - 1) / kNumCU;
                double t_us = (double)rounds * (((nk + sp - 1) / sp) * 0.7 * pl.bn / 256.0 + 12.0);
                if (sp > 1) t_us += 5.0 + 1.5 * sp * (double)M * (double)N * 4.0 / 4e6;
                if (t_us < best * 0.97) { best = t_us; splits = sp; }
            }
        } else if (tiles < 2 * kNumCU) {
            // Weight-streaming shapes: a few workgroups per CU keep every HBM channel busy.
            splits = (int)((2 * kNumCU + tiles - 1) / tiles);
            if (splits > max_splits) splits = max_splits;
            if (splits > 32) splits = 32;
        }
    }
    int per = (nk + splits - 1) / splits;
    splits = (nk + per - 1) / per;  // no empty split
    pl.splits = splits;
    pl.iters_per_split = per;
    if ((K & 127) == 0 && splits == 1) {  // the 16x16x64 form of the tile
        if (pl.cfg == 0) pl.cfg = 10;
        if (pl.cfg == 9) pl.cfg = 11;
        if (pl.cfg == 6 && K >= 192 * 64) pl.cfg = 12;
    }
    return pl;
}

template <int EPI, bool BF16>
void launch_cfg(const Plan& pl, const GemmArgs& a, int batch, hipStream_t st, bool tiled)
{
    dim3 grid((unsigned)(pl.tiles_m * pl.tiles_n * pl.splits), (unsigned)batch);
#define SQ_LAUNCH_MF(BM, BN, WGM, WGN, NST, MF)                                                                   \
    do {                                                                                                          \
        if (tiled) sq_launch((gemm_i8_kernel<BM, BN, WGM, WGN, NST, EPI, BF16, LAY_TILED, 1, false, MF>), grid, dim3(WGM * WGN * 64), 0, st, a); \
        else sq_launch((gemm_i8_kernel<BM, BN, WGM, WGN, NST, EPI, BF16, LAY_ROWS, 1, false, MF>), grid, dim3(WGM * WGN * 64), 0, st, a); \
    } while (0)
#define SQ_LAUNCH(BM, BN, WGM, WGN, NST) SQ_LAUNCH_MF(BM, BN, WGM, WGN, NST, 32)
    switch (pl.cfg) {
        case 0: SQ_LAUNCH(256, 256, 2, 4, 4); break;
        case 1: SQ_LAUNCH(128, 256, 1, 4, 6); break;
        case 2: SQ_LAUNCH(64, 256, 1, 4, 7); break;
        case 3: SQ_LAUNCH(32, 256, 1, 4, 8); break;
        case 6: SQ_LAUNCH(256, 192, 4, 2, 4); break;
        case 9: SQ_LAUNCH(256, 384, 2, 4, 4); break;
        case 10: SQ_LAUNCH_MF(256, 256, 4, 2, 4, 16); break;
        case 11: SQ_LAUNCH_MF(256, 384, 4, 2, 4, 16); break;
        case 12: SQ_LAUNCH_MF(256, 192, 4, 2, 5, 16); break;
        case 8:
            if (tiled) sq_launch((gemm_i8_kernel<128, 128, 2, 2, 3, EPI, BF16, LAY_TILED, 4, true>), grid, dim3(256), 0, st, a);
            else sq_launch((gemm_i8_kernel<128, 128, 2, 2, 3, EPI, BF16, LAY_ROWS, 4, true>), grid, dim3(256), 0, st, a);
            break;
        case 7:
            if (tiled) sq_launch((gemm_i8_kernel<128, 128, 2, 2, 3, EPI, BF16, LAY_TILED, 3>), grid, dim3(256), 0, st, a);
            else sq_launch((gemm_i8_kernel<128, 128, 2, 2, 3, EPI, BF16, LAY_ROWS, 3>), grid, dim3(256), 0, st, a);
            break;
        default:
            if constexpr (EPI == EPI_DEQUANT) {
                sq_launch((gemm_i8_kernel<256, 128, 4, 1, 5, EPI, BF16, LAY_BT>), grid, dim3(256), 0, st, a);
            }
            break;
    }
#undef SQ_LAUNCH
#undef SQ_LAUNCH_MF
}

// allow_split = false: the caller has no workspace to offer (sq_w8a8_bmm), so only plans that finish in one kernel
// are considered.
sq_status run_gemm(GemmArgs a, int64_t batch, bool to_i32, bool bf16, void* workspace, size_t ws_bytes, hipStream_t st,
                   bool b_transposed = false, bool tiled = false, bool allow_split = true)
{
    const int64_t total = (int64_t)a.M * a.N;
    auto reduce = [&](void* final_out) {  // a.acc_out = partials [a.splits][M][N]
        a.C = final_out;
        int blocks = (int)((total + 255) / 256);
        if (blocks > 4096) blocks = 4096;
        if (bf16) sq_launch(splitk_reduce_kernel<true>, dim3(blocks), dim3(256), 0, st, a, to_i32 ? 1 : 0);
        else sq_launch(splitk_reduce_kernel<false>, dim3(blocks), dim3(256), 0, st, a, to_i32 ? 1 : 0);
    };
    int ss = b_transposed ? 0 : sq_stream_gemm_splits(a.M, a.N, a.K, batch, tiled);
    if (ss > 1 && !allow_split) ss = 0;  // the streaming plan wants a K split: leave the shape to the tile kernels
    if (ss) {
        // few tokens, wide C_o: stream W once through one workgroup per CU
        if (ss > 1) {
            const size_t need = (size_t)ss * total * sizeof(int32_t);
            if (!workspace || ws_bytes < need) return SQ_ERR_WORKSPACE;
            void* final_out = to_i32 ? (void*)a.acc_out : a.C;
            a.acc_out = (int32_t*)workspace;
            a.splits = ss;
            sq_stream_gemm_launch(a, true, false, tiled, st);
            reduce(final_out);
        } else {
            sq_stream_gemm_launch(a, to_i32, bf16, tiled, st);
        }
        return sq_launch_status();
    }
    Plan pl = make_plan(a.M, a.N, a.K, batch, allow_split, b_transposed);
    a.tiles_m = pl.tiles_m;
    a.tiles_n = pl.tiles_n;
    a.splits = pl.splits;
    a.iters_per_split = pl.iters_per_split;
    if (pl.splits > 1) {
        const size_t need = (size_t)pl.splits * a.M * a.N * sizeof(int32_t);
        if (!workspace || ws_bytes < need) return SQ_ERR_WORKSPACE;
        void* final_out = to_i32 ? (void*)a.acc_out : a.C;
        a.acc_out = (int32_t*)workspace;
        launch_cfg<EPI_I32, false>(pl, a, 1, st, tiled);
        reduce(final_out);
    } else if (to_i32) {
        launch_cfg<EPI_I32, false>(pl, a, (int)batch, st, tiled);
    } else if (bf16) {
        launch_cfg<EPI_DEQUANT, true>(pl, a, (int)batch, st, tiled);
    } else {
        launch_cfg<EPI_DEQUANT, false>(pl, a, (int)batch, st, tiled);
    }
    return sq_launch_status();
}

bool dims_ok(int64_t t, int64_t c_i, int64_t c_o)
{
    const int64_t lim = (int64_t)1 << 31;
    return t > 0 && c_i > 0 && c_o > 0 && t < lim && c_i < lim && c_o < lim && t * c_o < ((int64_t)1 << 40) &&
           256 * c_i < lim;
}

}  // namespace

extern "C" {

size_t sq_gemm_workspace_bytes(int64_t t, int64_t c_i, int64_t c_o)
{
    if (!dims_ok(t, c_i, c_o)) return 0;
    // the layout is not known here: enough for the plan of either
    const int ss_rows = sq_stream_gemm_splits(t, c_o, c_i, 1, false), ss_tiled = sq_stream_gemm_splits(t, c_o, c_i, 1, true);
    if (const int ss = ss_rows > ss_tiled ? ss_rows : ss_tiled) return ss > 1 ? (size_t)ss * t * c_o * sizeof(int32_t) : 0;
    Plan pl = make_plan(t, c_o, c_i, 1, true);
    return pl.splits > 1 ? (size_t)pl.splits * t * c_o * sizeof(int32_t) : 0;
}

sq_status sq_w8a8_linear(const int8_t* xq, const float* x_scale, int x_scale_per_token, const int8_t* wq,
                         const float* w_scale, int w_scale_per_channel, const float* bias, const void* residual, int relu, void* y,
                         sq_dtype out, int64_t t, int64_t c_i, int64_t c_o, sq_layout layout, void* workspace,
                         size_t ws_bytes, void* stream)
{
    if (!xq || !x_scale || !wq || !w_scale || !y) return SQ_ERR_NULL;
    if (!dims_ok(t, c_i, c_o)) return SQ_ERR_SHAPE;
    if (out != SQ_F16 && out != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if (layout != SQ_ROW_MAJOR && layout != SQ_TILED) return SQ_ERR_UNSUPPORTED;
    if (layout == SQ_TILED && (c_i & 63)) return SQ_ERR_ALIGN;
    if ((c_i & 15) || !sq_aligned16(xq) || !sq_aligned16(wq) || !sq_aligned16(y) ||
        (residual && !sq_aligned16(residual)) || (workspace && !sq_aligned16(workspace)))
        return SQ_ERR_ALIGN;
    GemmArgs a{};
    a.A = xq; a.B = wq;
    a.M = (int)t; a.N = (int)c_o; a.K = (int)c_i;
    a.lda = c_i; a.ldb = c_i;
    a.C = y; a.x_scale = x_scale; a.per_token = x_scale_per_token ? 1 : 0; a.w_scale = w_scale;
    a.w_per_channel = w_scale_per_channel ? 1 : 0;
    a.bias = bias; a.residual = residual; a.relu = relu ? 1 : 0;
    return run_gemm(a, 1, false, out == SQ_BF16, workspace, ws_bytes, (hipStream_t)stream, false, layout == SQ_TILED);
}

sq_status sq_w8a8_linear_q8(const int8_t* xq, const float* x_scale, int x_scale_per_token, const int8_t* wq,
                            const float* w_scale, int w_scale_per_channel, const float* bias, const void* residual,
                            int relu, sq_dtype mid, const float* y_step, int8_t* yq, sq_layout yq_layout, int64_t t,
                            int64_t c_i, int64_t c_o, sq_layout layout, void* workspace, size_t ws_bytes, void* stream)
{
    if (!xq || !x_scale || !wq || !w_scale || !y_step || !yq) return SQ_ERR_NULL;
    if (!dims_ok(t, c_i, c_o)) return SQ_ERR_SHAPE;
    if (mid != SQ_F16 && mid != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if (layout != SQ_ROW_MAJOR && layout != SQ_TILED) return SQ_ERR_UNSUPPORTED;
    if (yq_layout != SQ_ROW_MAJOR && yq_layout != SQ_TILED) return SQ_ERR_UNSUPPORTED;
    if (layout == SQ_TILED && (c_i & 63)) return SQ_ERR_ALIGN;
    if (yq_layout == SQ_TILED && (c_o & 63)) return SQ_ERR_ALIGN;
    if ((c_i & 15) || (c_o & 7) || !sq_aligned16(xq) || !sq_aligned16(wq) || !sq_aligned16(yq) ||
        (residual && !sq_aligned16(residual)) || (workspace && !sq_aligned16(workspace)))
        return SQ_ERR_ALIGN;
    GemmArgs a{};
    a.A = xq; a.B = wq;
    a.M = (int)t; a.N = (int)c_o; a.K = (int)c_i;
    a.lda = c_i; a.ldb = c_i;
    a.C = yq;  // never written: the epilogues branch on q8_step
    a.x_scale = x_scale; a.per_token = x_scale_per_token ? 1 : 0; a.w_scale = w_scale;
    a.w_per_channel = w_scale_per_channel ? 1 : 0;
    a.bias = bias; a.residual = residual; a.relu = relu ? 1 : 0;
    a.q8_step = y_step; a.q8_out = yq; a.q8_tiled = yq_layout == SQ_TILED ? 1 : 0;
    return run_gemm(a, 1, false, mid == SQ_BF16, workspace, ws_bytes, (hipStream_t)stream, false, layout == SQ_TILED);
}

sq_status sq_i8_gemm_i32(const int8_t* xq, const int8_t* wq, int32_t* acc, int64_t t, int64_t c_i, int64_t c_o,
                         sq_layout layout, void* workspace, size_t ws_bytes, void* stream)
{
    if (!xq || !wq || !acc) return SQ_ERR_NULL;
    if (!dims_ok(t, c_i, c_o)) return SQ_ERR_SHAPE;
    if (layout != SQ_ROW_MAJOR && layout != SQ_TILED) return SQ_ERR_UNSUPPORTED;
    if (layout == SQ_TILED && (c_i & 63)) return SQ_ERR_ALIGN;
    if ((c_i & 15) || !sq_aligned16(xq) || !sq_aligned16(wq) || !sq_aligned16(acc) ||
        (workspace && !sq_aligned16(workspace)))
        return SQ_ERR_ALIGN;
    GemmArgs a{};
    a.A = xq; a.B = wq;
    a.M = (int)t; a.N = (int)c_o; a.K = (int)c_i;
    a.lda = c_i; a.ldb = c_i;
    a.acc_out = acc;
    a.C = acc;
    return run_gemm(a, 1, true, false, workspace, ws_bytes, (hipStream_t)stream, false, layout == SQ_TILED);
}

// ---- sq_w8a8_linear for callers that cannot allocate: the K-split scratch lives in a device array of the library.
// Each GPU the library runs on holds its own copy of the array (at its own address) until the process ends.
}  // extern "C"

namespace {
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
constexpr int kMaxDevices = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
namespace {
std::mutex scratch_mu;
void* scratch_addr[kMaxDevices];  // device address of `scratch` on each device, resolved on first use

// The array's name is a host-side handle only; kernels get the device address hipGetSymbolAddress reports for
// the current device.
sq_status static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SQ_ERR_HIP;
    std::lock_guard<std::mutex> lock(scratch_mu);
    if (!scratch_addr[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SQ_ERR_HIP;
        scratch_addr[dev] = ptr;
    }
    *out = scratch_addr[dev];
    return SQ_OK;
}
}  // namespace

extern "C" {

size_t sq_static_scratch_bytes(void) { return kStaticScratchBytes; }

sq_status sq_w8a8_linear_noalloc(const int8_t* xq, const float* x_scale, int x_scale_per_token, const int8_t* wq,
                                 const float* w_scale, int w_scale_per_channel, const float* bias, const void* residual,
                                 int relu, void* y, sq_dtype out, int64_t t, int64_t c_i, int64_t c_o, sq_layout layout,
                                 void* stream)
{
    if (!xq || !x_scale || !wq || !w_scale || !y) return SQ_ERR_NULL;
    if (!dims_ok(t, c_i, c_o)) return SQ_ERR_SHAPE;
    const size_t need = sq_gemm_workspace_bytes(t, c_i, c_o);
    if (need > kStaticScratchBytes) return SQ_ERR_WORKSPACE;  // shape beyond the built-in scratch: use sq_w8a8_linear
    void* ws = nullptr;
    if (need) {
        const sq_status st = static_scratch(&ws);
        if (st != SQ_OK) return st;
    }
    // Every K split writes its whole [t, c_o] slice of the partial sums before the reduction reads it, so nothing
    // in the scratch has to start at zero and the previous call's contents do not matter.
    return sq_w8a8_linear(xq, x_scale, x_scale_per_token, wq, w_scale, w_scale_per_channel, bias, residual, relu, y, out,
                          t, c_i, c_o, layout, ws, need ? kStaticScratchBytes : 0, stream);
}

// Attention BMM dispatcher behind sq_w8a8_bmm (arguments already validated).
sq_status sq_internal_bmm(const int8_t* a_, const int8_t* b_, int trans_b, float alpha, void* c, sq_dtype out,
                          int64_t batch, int64_t m, int64_t n, int64_t k, int64_t stride_a, int64_t stride_b,
                          int64_t stride_c, void* stream)
{
    GemmArgs a{};
    a.A = a_; a.B = b_;
    a.M = (int)m; a.N = (int)n; a.K = (int)k;
    a.lda = k;
    a.ldb = trans_b ? k : n;  // trans_b: rows of B are K-contiguous; otherwise B is [k, n]
    a.strideA = stride_a; a.strideB = stride_b; a.strideC = stride_c;
    a.C = c; a.alpha = alpha;
    if (trans_b && sq_strip_bmm_eligible(m, n, k, batch)) {
        sq_strip_bmm_launch(a, (int)batch, out == SQ_BF16, (hipStream_t)stream);
        return sq_launch_status();
    }
    return run_gemm(a, batch, false, out == SQ_BF16, nullptr, 0, (hipStream_t)stream, !trans_b, false, false);
}

}  // extern "C"
