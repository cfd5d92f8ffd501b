// Weight-streaming INT8 GEMM for few-token (decode) shapes, gfx950.
//
// With T <= 128 tokens the contraction of Eq. 2 reads every weight byte once and does little
// arithmetic with it: the layer is bound by how fast W streams out of HBM.  This kernel is built
// around that stream instead of around an output tile:
//  * The C_o axis is cut into 16-column units and the units are dealt evenly to one workgroup per
//    compute unit (a "slab" of 1..16 units each, every slab over the whole K range).  One round of
//    workgroups, each streaming the same number of bytes: no tail round, no split-K partials, no
//    second kernel; the dequantizing epilogue of Eq. 2 runs on the accumulators in registers.
//  * v_mfma_i32_16x16x64_i8: a 16-row x 64-byte block of 1 KB is exactly one MFMA operand, for the
//    activation rows as for a unit of W, so slab widths need only be multiples of 16.
//  * HBM -> LDS with global_load_lds (1 KB per wave instruction), up to 16 stages deep and sized
//    so that tens of KB per CU are in flight; thin slabs put several 64-byte K steps into one stage
//    to keep the work per barrier constant.
//  * The (small) activation block is re-read by every workgroup from L2.
#include <type_traits>

#include "gemm_args.h"

namespace {

constexpr int kSmemBytes = 152 * 1024;
constexpr int kMaxStageBlocks = 24;  // 1 KB blocks per stage
constexpr int kMaxLoads = kMaxStageBlocks / 4;  // per wave per stage

struct StreamArgs {
    int groups;      // workgroups
    int units;       // 16-column units of N
    int na;          // 16-row blocks of A
    int ksub;        // 64-byte K steps per stage
    int loads;       // global -> LDS loads per wave per stage
    int iters;       // K / 64 / ksub
    int tiled, to_i32, bf16;
};

// Pipeline depth as a function of the loads one wave issues per stage (a stage holds at most 4 * loads
// KB, so depth * stage stays below the LDS allocation), and the matching wait: stage `it` has landed
// when at most (depth - 2) younger stages, `loads` instructions each, are still in flight.
__host__ __device__ constexpr int stage_depth(int loads)
{
    return loads <= 2 ? 16 : loads == 3 ? 12 : loads == 4 ? 9 : loads == 5 ? 7 : 6;
}
SQ_DEVICE void wait_stage_landed(int loads)
{
    switch (loads) {
        case 1: wait_vmcnt_imm<(stage_depth(1) - 2) * 1>(); break;
        case 2: wait_vmcnt_imm<(stage_depth(2) - 2) * 2>(); break;
        case 3: wait_vmcnt_imm<(stage_depth(3) - 2) * 3>(); break;
        case 4: wait_vmcnt_imm<(stage_depth(4) - 2) * 4>(); break;
        case 5: wait_vmcnt_imm<(stage_depth(5) - 2) * 5>(); break;
        default: wait_vmcnt_imm<(stage_depth(6) - 2) * 6>(); break;
    }
}

// MB: 16-row blocks of A per wave; WM: waves along the token axis (the other 4/WM waves deal the
// slab's units among themselves); NUW: most units one wave accumulates.
template <int MB, int WM, int NUW>
__global__ __launch_bounds__(256, 1) void gemm_i8_stream_kernel(const GemmArgs p, const StreamArgs q)
{
    constexpr int WN = 4 / WM;
    __shared__ __attribute__((aligned(1024))) char smem[kSmemBytes];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int g = blockIdx.x;
    const int u0 = (int)((int64_t)g * q.units / q.groups), u1 = (int)((int64_t)(g + 1) * q.units / q.groups);
    const int nu = u1 - u0;           // units of this workgroup
    const int nblk = q.na + nu;       // block rows per stage
    const int ksub = q.ksub;
    const int sblocks = nblk * ksub;  // 1 KB blocks per stage
    const int stage_bytes = sblocks * 1024;
    const int L = q.loads;  // loads per wave per stage, the same for every wave (see below)
    const int nstage = stage_depth(L);

    // ---- global -> LDS slots of this wave: stage block sb = i*4 + wave = (block row b, K sub-step ks).
    // Tiled operands: lane l copies bytes 16 l .. 16 l + 15 of the 1 KB block.  Row-major operands:
    // four neighbouring lanes copy the 64 bytes of one row, chunks permuted (position = chunk ^ swz(row)).
    auto swz = [](int r) { return ((r >> 1) & 3) ^ ((r >> 3) & 1); };
    const int64_t kstep = q.tiled ? 1024 : 64;
    // A wave whose last slot falls past the stage re-reads stage block 0 into a spare KB at the end of the
    // allocation: every wave then has the same number of loads in flight, which the wait above relies on.
    const int8_t* src[kMaxLoads];
    int dst[kMaxLoads];
#pragma unroll
    for (int i = 0; i < kMaxLoads; ++i) {
        int sb = i * 4 + wave;
        dst[i] = sb < sblocks ? sb * 1024 : -1;
        sb = sb < sblocks ? sb : 0;
        const int b = sb / ksub, ks = sb - b * ksub;
        const bool is_a = b < q.na;
        const int8_t* base = is_a ? p.A : p.B;
        const int64_t ld = is_a ? p.lda : p.ldb;
        const int rows = is_a ? p.M : p.N;
        int br = is_a ? b : u0 + (b - q.na);  // 16-row block row of the operand
        if (q.tiled) {
            if (is_a) {  // ragged M: blocks past the last one re-read it (their rows are never stored)
                const int last = (p.M - 1) >> 4;
                br = br < last ? br : last;
            }
            src[i] = base + (int64_t)br * 16 * ld + ks * kstep + lane * 16;
        } else {
            int row = br * 16 + (lane >> 2);
            row = row < rows ? row : rows - 1;
            const int chunk = (lane & 3) ^ swz(lane >> 2);
            src[i] = base + (int64_t)row * ld + ks * kstep + chunk * 16;
        }
    }
    auto issue_stage = [&](int it, int slot) {
        const int64_t koff = (int64_t)it * ksub * kstep;
        char* base = smem + slot * stage_bytes;
#pragma unroll
        for (int i = 0; i < kMaxLoads; ++i)
            if (i < L)
                __builtin_amdgcn_global_load_lds(GPTR(src[i] + koff), LPTR(dst[i] >= 0 ? base + dst[i] : smem + kSmemBytes - 1024),
                                                 16, 0, 0);
    };

    // ---- MFMA operands: lane l feeds row (l & 15) with K-chunk (l >> 4) of the 64-byte step.
    const int frow = lane & 15;
    const int frag_off = frow * 64 + (((lane >> 4) ^ swz(frow)) << 4);

    v4i acc[MB][NUW];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NUW; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    const int iters = q.iters;
    for (int s = 0; s < nstage - 1; ++s) issue_stage(s < iters ? s : iters - 1, s);

    // The K loop is instantiated once per number of units this wave accumulates (CNT), so its body has
    // no branches: all operand reads of a K step are issued together, then the MFMAs.
    const int cnt = nu > wn ? (nu - wn + WN - 1) / WN : 0;
    auto k_loop = [&](auto CNT_) {
        constexpr int CNT = decltype(CNT_)::value;
        int slot = 0;
        for (int it = 0; it < iters; ++it) {
            wait_stage_landed(L);            // this wave's share of stage `it` has landed
            __builtin_amdgcn_s_barrier();    // everyone's share has; everyone is done with stage it-1
            {
                const int nxt = it + nstage - 1;
                issue_stage(nxt < iters ? nxt : iters - 1, slot == 0 ? nstage - 1 : slot - 1);
            }
            const char* sa = smem + slot * stage_bytes + frag_off + wm * MB * ksub * 1024;
            const char* sb = smem + slot * stage_bytes + frag_off + (q.na + wn) * ksub * 1024;
            for (int ks = 0; ks < ksub; ++ks) {
                v4i fa[MB], fb[CNT > 0 ? CNT : 1];
#pragma unroll
                for (int i = 0; i < MB; ++i) fa[i] = *(const v4i*)(sa + (i * ksub + ks) * 1024);
#pragma unroll
                for (int j = 0; j < CNT; ++j) fb[j] = *(const v4i*)(sb + (j * WN * ksub + ks) * 1024);
#pragma unroll
                for (int j = 0; j < CNT; ++j)
#pragma unroll
                    for (int i = 0; i < MB; ++i)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
            }
            slot = slot + 1 == nstage ? 0 : slot + 1;
        }
    };
#define SQ_CASE(N) case N: if constexpr (N <= NUW) k_loop(std::integral_constant<int, N>{}); break;
    switch (cnt) {
        SQ_CASE(0) SQ_CASE(1) SQ_CASE(2) SQ_CASE(3) SQ_CASE(4) SQ_CASE(5) SQ_CASE(6) SQ_CASE(7) SQ_CASE(8)
        SQ_CASE(9) SQ_CASE(10) SQ_CASE(11) SQ_CASE(12) SQ_CASE(13) SQ_CASE(14) SQ_CASE(15) SQ_CASE(16)
        default: break;
    }
#undef SQ_CASE
    wait_vmcnt_imm<0>();  // the refills issued past the end of the K range have landed

    // ---- epilogue.  16x16 accumulator layout: lane l, register v holds row 4*(l >> 4) + v, column l & 15.
    const int col_l = lane & 15, row_l = (lane >> 4) * 4;
    const float ws = (!q.to_i32 && p.x_scale) ? p.w_scale[0] : 0.0f;
    const uint16_t* R = (const uint16_t*)p.residual;
#pragma unroll
    for (int j = 0; j < NUW; ++j) {
        const int u = j * WN + wn;
        if (u >= nu) continue;
        const int col = (u0 + u) * 16 + col_l;
        if (col >= p.N) continue;
        const float bias = (!q.to_i32 && p.bias) ? p.bias[col] : 0.0f;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = (wm * MB + i) * 16 + row_l + v;
                if (row >= p.M) continue;
                const int64_t idx = (int64_t)row * p.N + col;
                if (q.to_i32) {
                    p.acc_out[idx] = acc[i][j][v];
                } else {
                    float c;
                    if (p.x_scale) c = (p.per_token ? p.x_scale[row] : p.x_scale[0]) * ws;
                    else c = p.alpha;
                    const uint32_t rb = R ? (uint32_t)R[idx] : 0u;
                    const uint32_t o = q.bf16 ? dequant_one<true>(acc[i][j][v], c, bias, p.bias != nullptr, p.relu != 0, rb, R != nullptr)
                                              : dequant_one<false>(acc[i][j][v], c, bias, p.bias != nullptr, p.relu != 0, rb, R != nullptr);
                    ((uint16_t*)p.C)[idx] = (uint16_t)o;
                }
            }
    }
}

int num_cus()
{
    static int n = 0;
    if (n == 0) {
        int dev = 0, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            n = v;
        else
            n = 256;
    }
    return n;
}

// Slab plan: one workgroup per CU (times an integer when slabs would exceed 16 units).
bool make_stream_plan(int64_t M, int64_t N, int64_t K, int64_t batch, StreamArgs* out)
{
    if (batch != 1 || M < 1 || M > 128 || (K & 63) || K < 64) return false;
    const int64_t units = (N + 15) / 16;
    const int cus = num_cus();
    if (units < cus) return false;
    const int64_t rounds = (units + (int64_t)cus * 16 - 1) / ((int64_t)cus * 16);
    const int64_t groups = cus * rounds;
    const int64_t upw = (units + groups - 1) / groups;
    if ((double)units / (double)(groups * upw) < 0.85) return false;  // uneven slabs: the tile kernels do better
    StreamArgs q{};
    q.groups = (int)groups;
    q.units = (int)units;
    q.na = M <= 16 ? 1 : M <= 32 ? 2 : M <= 64 ? 4 : 8;
    const int nblk = q.na + (int)upw;
    const int nk = (int)(K >> 6);
    q.ksub = 1;
    for (int c = 4; c > 1; c >>= 1)
        if (nblk * c <= kMaxStageBlocks && nk % c == 0) { q.ksub = c; break; }
    const int sblocks = nblk * q.ksub;
    q.loads = (sblocks + 3) / 4;
    static_assert(stage_depth(1) * 4 * 1 + 1 <= kSmemBytes / 1024 && stage_depth(2) * 4 * 2 + 1 <= kSmemBytes / 1024 &&
                  stage_depth(3) * 4 * 3 + 1 <= kSmemBytes / 1024 && stage_depth(4) * 4 * 4 + 1 <= kSmemBytes / 1024 &&
                  stage_depth(5) * 4 * 5 + 1 <= kSmemBytes / 1024 && stage_depth(6) * 4 * 6 + 1 <= kSmemBytes / 1024,
                  "stages plus the spare KB fit the LDS allocation");
    q.iters = nk / q.ksub;
    if (out) *out = q;
    return true;
}

}  // namespace

bool sq_stream_gemm_eligible(int64_t M, int64_t N, int64_t K, int64_t batch)
{
    return make_stream_plan(M, N, K, batch, nullptr);
}

void sq_stream_gemm_launch(const GemmArgs& a, bool to_i32, bool bf16, bool tiled, hipStream_t st)
{
    StreamArgs q{};
    if (!make_stream_plan(a.M, a.N, a.K, 1, &q)) return;
    q.tiled = tiled ? 1 : 0;
    q.to_i32 = to_i32 ? 1 : 0;
    q.bf16 = bf16 ? 1 : 0;
    const dim3 grid((unsigned)q.groups), block(256);
    switch (q.na) {
        case 1: hipLaunchKernelGGL((gemm_i8_stream_kernel<1, 1, 4>), grid, block, 0, st, a, q); break;
        case 2: hipLaunchKernelGGL((gemm_i8_stream_kernel<1, 2, 8>), grid, block, 0, st, a, q); break;
        case 4: hipLaunchKernelGGL((gemm_i8_stream_kernel<1, 4, 16>), grid, block, 0, st, a, q); break;
        default: hipLaunchKernelGGL((gemm_i8_stream_kernel<2, 4, 16>), grid, block, 0, st, a, q); break;
    }
}
