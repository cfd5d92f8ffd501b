// Weight-streaming INT8 GEMM for few-token (decode) shapes, gfx950.
//
// With T <= 128 tokens the contraction of Eq. 2 reads every weight byte once and does little
// arithmetic with it: the layer is bound by how fast W streams out of HBM.  This kernel is built
// around that stream instead of around an output tile:
//  * The C_o axis is cut into 16-column units and the units are dealt evenly to the workgroups, one
//    workgroup per compute unit (a "slab" of 1..16 units each).  One round of workgroups, each streaming
//    the same number of bytes: no tail round.  For up to 32 tokens every slab runs over the whole K range
//    and the dequantizing epilogue of Eq. 2 is applied to the accumulators in registers: no workspace, no
//    second kernel.
//  * Every workgroup also pulls the activation rows of its K range through its CU's vector cache, and a
//    CU sustains only a few tens of GB/s while most of its loads miss to HBM.  With 64..128 tokens the
//    activation bytes per weight byte (tokens / slab width) decide the speed, so narrow slabs are traded
//    for wide ones over a fraction of K (a host-side cost model picks slab width and K split); the int32
//    partial sums then go to the workspace and the split-K reduction kernel applies the epilogue.
//  * v_mfma_i32_16x16x64_i8: a 16-row x 64-byte block of 1 KB is exactly one MFMA operand, for the
//    activation rows as for a unit of W, so slab widths need only be multiples of 16.
//  * HBM -> LDS with global_load_lds (1 KB per wave instruction, non-temporal for W) through a 4-stage ring; thin slabs put
//    several 64-byte K steps into one stage to keep the work per barrier constant.  (Measured: deeper
//    rings do not stream faster; the outstanding-miss capacity of the CU is the limit, not the ring.)
#include <type_traits>

#include "gemm_args.h"

namespace {

constexpr int kDepth = 4;            // pipeline stages
// 1 KB blocks per stage: 24 for the 4-wave shapes (up to 32 tokens), 32 for the 8-wave shapes
constexpr int max_stage_blocks(int waves) { return waves == 4 ? 24 : 32; }

struct StreamArgs {
    int gn;          // slabs (workgroups along C_o)
    int gk;          // K splits (workgroups along K); > 1: int32 partials go to acc_out[gk][M][N]
    int units;       // 16-column units of N
    int na;          // 16-row blocks of A
    int ksub;        // 64-byte K steps per stage
    int iters;       // stages per workgroup: K / 64 / gk / ksub
    int nt_w;        // weight loads carry the non-temporal hint
    int regs;        // the register-direct kernel (tiled operands) runs this plan
    int tiled, to_i32, bf16;
};

// Stage `it` of this wave has landed when at most (kDepth - 2) younger stages, `loads` instructions
// each, are still in flight.
SQ_DEVICE void wait_stage_landed(int loads)
{
    switch (loads) {
        case 0: break;
        case 1: wait_vmcnt_imm<(kDepth - 2) * 1>(); break;
        case 2: wait_vmcnt_imm<(kDepth - 2) * 2>(); break;
        case 3: wait_vmcnt_imm<(kDepth - 2) * 3>(); break;
        case 4: wait_vmcnt_imm<(kDepth - 2) * 4>(); break;
        case 5: wait_vmcnt_imm<(kDepth - 2) * 5>(); break;
        case 6: wait_vmcnt_imm<(kDepth - 2) * 6>(); break;
        case 7: wait_vmcnt_imm<(kDepth - 2) * 7>(); break;
        default: wait_vmcnt_imm<(kDepth - 2) * 8>(); break;
    }
}
static_assert(kDepth >= 3 && (kDepth - 2) * (max_stage_blocks(4) / 4) <= 63, "depth and vmcnt limits");

// MB: 16-row blocks of A per wave; WM: waves along the token axis (the other NWAVE/WM waves deal the
// slab's units among themselves); NUW: most units one wave accumulates.  The 8-wave shapes put two
// waves on each SIMD, so one wave's LDS reads overlap the other's MFMAs.
template <int MB, int WM, int NUW, int NWAVE, bool NT>
__global__ __launch_bounds__(NWAVE * 64, 1) void gemm_i8_stream_kernel(const GemmArgs p, const StreamArgs q)
{
    constexpr int WN = NWAVE / WM;
    constexpr int kLoads = max_stage_blocks(NWAVE) / NWAVE;
    __shared__ __attribute__((aligned(1024))) char smem[kDepth * max_stage_blocks(NWAVE) * 1024];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int wm = wave / WN, wn = wave % WN;
    const int gs = blockIdx.x % q.gn, gki = blockIdx.x / q.gn;
    const int u0 = (int)((int64_t)gs * q.units / q.gn), u1 = (int)((int64_t)(gs + 1) * q.units / q.gn);
    const int nu = u1 - u0;           // units of this workgroup
    const int nblk = q.na + nu;       // block rows per stage
    const int ksub = q.ksub;
    const int sblocks = nblk * ksub;  // 1 KB blocks per stage
    const int stage_bytes = sblocks * 1024;
    const int L = sblocks > wave ? (sblocks - wave + NWAVE - 1) / NWAVE : 0;  // loads of this wave per stage

    // ---- global -> LDS slots of this wave: stage block sb = i*NWAVE + wave = (block row b, K sub-step ks).
    // Tiled operands: lane l copies bytes 16 l .. 16 l + 15 of the 1 KB block.  Row-major operands:
    // four neighbouring lanes copy the 64 bytes of one row, chunks permuted (position = chunk ^ swz(row)).
    auto swz = [](int r) { return ((r >> 1) & 3) ^ ((r >> 3) & 1); };
    const int64_t kstep = q.tiled ? 1024 : 64;
    const int64_t kbeg = (int64_t)gki * q.iters * ksub * kstep;  // first byte of this workgroup's K range
    const int8_t* src[kLoads];
    bool isw[kLoads];
#pragma unroll
    for (int i = 0; i < kLoads; ++i) {
        int sb = i * NWAVE + wave;
        sb = sb < sblocks ? sb : 0;  // unused slot (i >= L)
        const int b = sb / ksub, ks = sb - b * ksub;
        const bool is_a = b < q.na;
        isw[i] = !is_a;
        const int8_t* base = is_a ? p.A : p.B;
        const int64_t ld = is_a ? p.lda : p.ldb;
        const int rows = is_a ? p.M : p.N;
        int br = is_a ? b : u0 + (b - q.na);  // 16-row block row of the operand
        if (q.tiled) {
            if (is_a) {  // ragged M: blocks past the last one re-read it (their rows are never stored)
                const int last = (p.M - 1) >> 4;
                br = br < last ? br : last;
            }
            src[i] = base + (int64_t)br * 16 * ld + kbeg + ks * kstep + lane * 16;
        } else {
            int row = br * 16 + (lane >> 2);
            row = row < rows ? row : rows - 1;
            const int chunk = (lane & 3) ^ swz(lane >> 2);
            src[i] = base + (int64_t)row * ld + kbeg + ks * kstep + chunk * 16;
        }
    }
    auto issue_stage = [&](int it, int slot) {
        const int64_t koff = (int64_t)it * ksub * kstep;
        char* base = smem + slot * stage_bytes + wave * 1024;
#pragma unroll
        for (int i = 0; i < kLoads; ++i)
            if (i < L) {
                // NT: weight blocks carry the non-temporal hint (aux bit 1), activation blocks do not
                if (NT && isw[i]) __builtin_amdgcn_global_load_lds(GPTR(src[i] + koff), LPTR(base + i * NWAVE * 1024), 16, 0, 2);
                else __builtin_amdgcn_global_load_lds(GPTR(src[i] + koff), LPTR(base + i * NWAVE * 1024), 16, 0, 0);
            }
    };

    // ---- MFMA operands: lane l feeds row (l & 15) with K-chunk (l >> 4) of the 64-byte step.
    const int frow = lane & 15;
    const int frag_off = frow * 64 + (((lane >> 4) ^ swz(frow)) << 4);

    v4i acc[MB][NUW];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NUW; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    // Every K step issues exactly one stage of loads (past the end of the range the last stage again,
    // into a slot nobody reads), so the number of loads in flight at each wait is a constant.
    const int iters = q.iters;
#pragma unroll
    for (int s = 0; s < kDepth - 1; ++s) issue_stage(s < iters ? s : iters - 1, s);

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
                const int nxt = it + kDepth - 1;
                issue_stage(nxt < iters ? nxt : iters - 1, slot == 0 ? kDepth - 1 : slot - 1);
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
            slot = slot + 1 == kDepth ? 0 : slot + 1;
        }
    };
#define SQ_CASE(N) case N: if constexpr (N <= NUW) k_loop(std::integral_constant<int, N>{}); break;
    switch (cnt) {
        SQ_CASE(0) SQ_CASE(1) SQ_CASE(2) SQ_CASE(3) SQ_CASE(4) SQ_CASE(5) SQ_CASE(6) SQ_CASE(7) SQ_CASE(8)
        SQ_CASE(9) SQ_CASE(10) SQ_CASE(11) SQ_CASE(12) SQ_CASE(13) SQ_CASE(14) SQ_CASE(15) SQ_CASE(16)
        default: break;  // NUW <= 16 in every instantiation
    }
#undef SQ_CASE
    wait_vmcnt_imm<0>();  // the refills issued past the end of the K range have landed

    // ---- epilogue.  16x16 accumulator layout: lane l, register v holds row 4*(l >> 4) + v, column l & 15.
    const int col_l = lane & 15, row_l = (lane >> 4) * 4;
    const bool raw = q.to_i32 || q.gk > 1;
    int32_t* out32 = p.acc_out + (int64_t)gki * p.M * p.N;
    const float ws = (!raw && p.x_scale && !p.w_per_channel) ? p.w_scale[0] : 0.0f;
    const uint16_t* R = (const uint16_t*)p.residual;
    float rq = 0.0f;
    if (!raw && p.q8_step) {
        const float delta = p.q8_step[0];
        rq = delta > 0.0f ? 1.0f / delta : 0.0f;
    }
#pragma unroll
    for (int j = 0; j < NUW; ++j) {
        const int u = j * WN + wn;
        if (u >= nu) continue;
        const int col = (u0 + u) * 16 + col_l;
        if (col >= p.N) continue;
        const float bias = (!raw && p.bias) ? p.bias[col] : 0.0f;
        const float wsc = (!raw && p.x_scale && p.w_per_channel) ? p.w_scale[col] : ws;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int row = (wm * MB + i) * 16 + row_l + v;
                if (row >= p.M) continue;
                const int64_t idx = (int64_t)row * p.N + col;
                if (raw) {
                    out32[idx] = acc[i][j][v];
                } else {
                    float c;
                    if (p.x_scale) c = (p.per_token ? p.x_scale[row] : p.x_scale[0]) * wsc;
                    else c = p.alpha;
                    const uint32_t rb = R ? (uint32_t)R[idx] : 0u;
                    const uint32_t o = q.bf16 ? dequant_one<true>(acc[i][j][v], c, bias, p.bias != nullptr, p.relu != 0, rb, R != nullptr)
                                              : dequant_one<false>(acc[i][j][v], c, bias, p.bias != nullptr, p.relu != 0, rb, R != nullptr);
                    if (p.q8_step) {
                        const int code = q.bf16 ? requant_code<true>(o, rq) : requant_code<false>(o, rq);
                        code_dst(p.q8_out, row, col & ~7, p.N, p.q8_tiled != 0)[col & 7] = (int8_t)code;
                    } else {
                        ((uint16_t*)p.C)[idx] = (uint16_t)o;
                    }
                }
            }
    }
}

// ---- Variant for tiled operands: weights straight into registers, activations through two loader waves.
// Two measurements with pure read loops (256 workgroups, 4 streaming waves each) shape it:
//  * a wave's loads return in issue order, so an activation block that would be an L2 hit waits behind the HBM
//    misses the same wave issued before it.  A QKV-sized weight stream (453 MB) takes 65 us alone; with every wave
//    also reading its share of a 1.5 MB block common to all workgroups (128 tokens) 108 us; with the common block read
//    by two extra waves of each workgroup instead 75 us;
//  * more requests in flight than the latency needs cost bandwidth: 9 interleaved 1 KB streams per wave deliver
//    6.9 TB/s with 9 loads in flight per wave, 5.8 with 18, 5.3 with 27, 4.8 with 45.
//  * in a loop of this kind (fragment reads and MFMAs in one instruction stream) v_mfma_i32_16x16x64_i8 came out every 48
//    cycles from one wave per SIMD and every 32 from two (from registers alone a wave issues one every 17): with 128
//    tokens a single compute wave per SIMD is bound by its MFMAs.
// In the tiled layout a 1 KB block is one MFMA operand as it lies in memory, so the compute waves fetch their weight
// blocks with one 16-byte load per lane straight into registers (no LDS, no barrier, no other wave to wait for), D of
// their K steps deep, about a dozen loads in flight.  Six compute waves = 3 unit groups x 2 K parities: wave (ug, kp)
// owns the units ug, ug + 3, ... of the slab on the K steps 2 t + kp, so two compute waves share a SIMD, every weight
// block is fetched by exactly one wave and every activation fragment is read from LDS by three.  Waves 6 and 7 do
// nothing but copy the activation blocks into a 4-stage LDS ring (global_load_lds, a stage = 4 K steps of all token
// blocks), three stages ahead; one barrier per stage.  Used from 33 tokens on; below, where the activation bytes hardly
// matter, the kernel above is faster (all eight waves' loads feed one ring).
// Tried on top of this, no gain: the 32x32x32 MFMA on operands loaded half a block per instruction (twice the cache
// lines per load: a third slower) or formed from whole blocks of two units with v_permlane16_swap (same time: the
// MFMAs are not what the waves wait for); four compute waves, one per SIMD (3-8 % slower); K slices instead of units
// per wave with both operands straight into registers (the activation blocks then wait behind the weight blocks again).
constexpr int kRegsStageSteps = 4, kRegsStages = 4, kRegsMaxUnits = 12;
constexpr int regs_depth(int cntw) { return cntw <= 1 ? 8 : 4; }  // own K steps of weight blocks in flight per wave

template <int MB, int CNT, bool NT>
__global__ __launch_bounds__(512, 1) void gemm_i8_stream_regs_kernel(const GemmArgs p, const StreamArgs q)
{
    constexpr int CNTW = (CNT + 2) / 3;       // units per compute wave
    constexpr int D = regs_depth(CNTW);
    constexpr int S = kRegsStageSteps, NS = kRegsStages;
    constexpr int STAGE = S * MB * 1024;      // bytes
    constexpr int LW = S * MB / 2;            // loads per loader wave and stage
    constexpr int PITCH = CNT * 16 + 4;       // ints per row of the output staging buffer
    constexpr int RING = NS * STAGE, RED = MB * 16 * PITCH * 4;
    __shared__ __attribute__((aligned(1024))) char smem[RING > RED ? RING : RED];
    static_assert(S == 4 && D % 2 == 0, "a stage is two own steps of a compute wave; whole stages in the unrolled body");
    static_assert(S * MB % 2 == 0 && 3 * LW <= 63, "loads of a loader wave: whole, and countable by vmcnt");

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int gs = blockIdx.x % q.gn, gki = blockIdx.x / q.gn;
    const int u0 = (int)((int64_t)gs * q.units / q.gn), u1 = (int)((int64_t)(gs + 1) * q.units / q.gn);
    const int nu = u1 - u0;     // 1 <= nu <= CNT; units past the slab re-read its last one and their sums are dropped
    const int n = q.iters;      // 64-byte K steps of this workgroup: at least 2 D (the host sees to it)
    const int nst = (n + S - 1) / S;  // stages
    const int64_t k0 = (int64_t)gki * n * 1024;
    // lane l feeds row (l & 15), K chunk (l >> 4) of a block; the chunks of a row are stored permuted
    const int frow = lane & 15;
    const uint32_t frag_off = (uint32_t)(frow * 64 + ((((lane >> 4) ^ ((frow >> 1) & 3) ^ ((frow >> 3) & 1))) << 4));
    const int ug = wave % 3, kp = wave / 3;  // compute waves 0..5

    v4i acc[MB][CNTW];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < CNTW; ++j) acc[i][j] = v4i{0, 0, 0, 0};

    if (wave >= 6) {
        // ---- loader waves: block b of a stage = (K step b / MB of the stage, token block b % MB); wave 6 takes the
        // even blocks, wave 7 the odd ones.  Ragged M: blocks past the last one re-read it (their rows are never stored).
        const int lw = wave - 6;
        const int last_a = (p.M - 1) >> 4;
        const int8_t* src[LW];
        int step_of[LW];
#pragma unroll
        for (int i = 0; i < LW; ++i) {
            const int b = 2 * i + lw;
            const int blk = b % MB;
            step_of[i] = b / MB;
            src[i] = p.A + (int64_t)(blk < last_a ? blk : last_a) * 16 * p.lda + k0 + lane * 16;
        }
        auto issue_stage = [&](int t, int slot) {
            char* base = smem + slot * STAGE + lw * 1024;
#pragma unroll
            for (int i = 0; i < LW; ++i) {
                int s = t * S + step_of[i];
                s = s < n ? s : n - 1;  // past the end of the K range: the last step again, nobody reads it
                __builtin_amdgcn_global_load_lds(GPTR(src[i] + (int64_t)s * 1024), LPTR(base + i * 2048), 16, 0, 0);
            }
        };
        // Every iteration issues exactly one stage of loads (past the end the last stage again, into a slot nobody
        // reads), so the wait is one immediate: stage t has landed when at most two younger stages are in flight.
#pragma unroll
        for (int t = 0; t < NS - 1; ++t) issue_stage(t < nst ? t : nst - 1, t);
        int slot = 0;
        for (int t = 0; t < nst; ++t) {
            wait_vmcnt_imm<2 * LW>();
            __builtin_amdgcn_s_barrier();  // stage t is there for everyone; everyone is done with stage t - 1
            const int nxt = t + NS - 1;
            issue_stage(nxt < nst ? nxt : nst - 1, slot == 0 ? NS - 1 : slot - 1);
            slot = slot + 1 == NS ? 0 : slot + 1;
        }
        wait_vmcnt_imm<0>();
    } else {
        // ---- compute waves: own step t is K step 2 t + kp, in stage t / 2
        const int8_t* pw[CNTW];
#pragma unroll
        for (int j = 0; j < CNTW; ++j) {
            const int u = ug + j * 3;
            pw[j] = p.B + (int64_t)(u0 + (u < nu ? u : nu - 1)) * 16 * p.ldb + k0;
        }
        v4i fb[D][CNTW];
        auto load_w = [&](int d, int j, int s) {
            const uint32_t off = frag_off + (uint32_t)s * 1024u;
            if (NT) fb[d][j] = __builtin_nontemporal_load((const v4i*)(pw[j] + off));
            else fb[d][j] = *(const v4i*)(pw[j] + off);
        };
        // Every step issues its refills, past the end of the range the last step again (L2 hits whose data nobody
        // uses): the number of loads issued after any given one is then the same on every path, and the waits the
        // compiler places leave exactly the younger loads in flight.  (With a refill under a condition it has to
        // assume the refill did not happen, and waits for everything.)
#pragma unroll
        for (int d = 0; d < D; ++d)
#pragma unroll
            for (int j = 0; j < CNTW; ++j) load_w(d, j, 2 * d + kp);
        int slot = 0;
        for (int t0 = 0; t0 < 2 * nst; t0 += D) {
#pragma unroll
            for (int d = 0; d < D; ++d) {
                if (d % 2 == 0) {
                    if (t0 + d >= 2 * nst) break;  // the later stages of the last round may not exist
                    __builtin_amdgcn_s_barrier();
                }
                const int g = 2 * (t0 + d) + kp;
                const bool live = g < n;
                const int gw = g + 2 * D;
                const int sw = gw < n ? gw : n - 1;
                const char* sa = smem + slot * STAGE + (2 * (d % 2) + kp) * MB * 1024 + frag_off;
                v4i fa[MB];
#pragma unroll
                for (int i = 0; i < MB; ++i) fa[i] = *(const v4i*)(sa + i * 1024);
#pragma unroll
                for (int j = 0; j < CNTW; ++j) {
                    if (live) {
#pragma unroll
                        for (int i = 0; i < MB; ++i)
                            acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[i], fb[d][j], acc[i][j], 0, 0, 0);
                    }
                    load_w(d, j, sw);
                }
                if (d % 2 == 1) slot = slot + 1 == NS ? 0 : slot + 1;
            }
        }
    }

    // ---- the accumulators meet in LDS (the ring is free now): the waves of K parity 0 store, those of parity 1 add
    // (the same lane of the same unit group owns an element in both), and the epilogue writes whole rows of the slab.
    // 16x16 accumulator layout: lane l, register v holds row 4*(l >> 4) + v, column l & 15.
    int* red = (int*)smem;
    __syncthreads();  // everyone is done with the ring
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
        if (wave < 6 && kp == pass) {
            const int col_l = lane & 15, row_l = (lane >> 4) * 4;
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < CNTW; ++j) {
                    const int u = ug + j * 3;
                    if (u >= nu) continue;  // a re-read unit
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        int* dst = &red[(i * 16 + row_l + v) * PITCH + u * 16 + col_l];
                        *dst = pass ? *dst + acc[i][j][v] : acc[i][j][v];
                    }
                }
        }
        __syncthreads();
    }

    // ---- epilogue: two neighbouring columns per thread
    const bool raw = q.to_i32 || q.gk > 1;
    int32_t* out32 = p.acc_out + (int64_t)gki * p.M * p.N;
    const float ws = (!raw && p.x_scale && !p.w_per_channel) ? p.w_scale[0] : 0.0f;
    const uint16_t* R = (const uint16_t*)p.residual;
    float rq = 0.0f;
    if (!raw && p.q8_step) {
        const float delta = p.q8_step[0];
        rq = delta > 0.0f ? 1.0f / delta : 0.0f;
    }
    const int pairs = nu * 8;  // column pairs per row
    const int rows = p.M < MB * 16 ? p.M : MB * 16;
    for (int idx = threadIdx.x; idx < rows * pairs; idx += 512) {
        const int row = idx / pairs, cp = idx - row * pairs;
        const int col = u0 * 16 + cp * 2;
        if (col >= p.N) continue;
        const bool two = col + 1 < p.N;
        const int a0 = red[row * PITCH + cp * 2], a1 = red[row * PITCH + cp * 2 + 1];
        const int64_t o = (int64_t)row * p.N + col;
        if (raw) {
            out32[o] = a0;
            if (two) out32[o + 1] = a1;
            continue;
        }
        const float xs = p.x_scale ? (p.per_token ? p.x_scale[row] : p.x_scale[0]) : 0.0f;
        uint32_t ob[2];
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            if (e == 1 && !two) break;
            const float c = p.x_scale ? xs * (p.w_per_channel ? p.w_scale[col + e] : ws) : p.alpha;
            const float bias = p.bias ? p.bias[col + e] : 0.0f;
            const uint32_t rb = R ? (uint32_t)R[o + e] : 0u;
            const int a = e ? a1 : a0;
            ob[e] = q.bf16 ? dequant_one<true>(a, c, bias, p.bias != nullptr, p.relu != 0, rb, R != nullptr)
                           : dequant_one<false>(a, c, bias, p.bias != nullptr, p.relu != 0, rb, R != nullptr);
            if (p.q8_step) {
                const int code = q.bf16 ? requant_code<true>(ob[e], rq) : requant_code<false>(ob[e], rq);
                code_dst(p.q8_out, row, (col + e) & ~7, p.N, p.q8_tiled != 0)[(col + e) & 7] = (int8_t)code;
            }
        }
        if (p.q8_step) continue;
        uint16_t* dst = (uint16_t*)p.C + o;
        if (two && !(p.N & 1)) {
            *(uint32_t*)dst = (ob[0] & 0xffffu) | (ob[1] << 16);
        } else {
            dst[0] = (uint16_t)ob[0];
            if (two) dst[1] = (uint16_t)ob[1];
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

// Slab width and K split by a small cost model (seconds):
//   CU side:  every workgroup moves (A blocks + slab units) KB per K step through its CU's vector cache,
//             at about 26 GB/s while most loads miss to HBM; workgroups beyond one per CU run in rounds;
//   HBM side: W once plus the int32 partials when K is split, at about 5.5 TB/s;
//   a K split adds the reduction kernel (launch + reading the partials).
bool make_stream_plan(int64_t M, int64_t N, int64_t K, int64_t batch, bool tiled, StreamArgs* out)
{
    if (batch != 1 || M < 1 || M > 128 || (K & 63) || K < 64) return false;
    const int64_t units = (N + 15) / 16;
    const int cus = num_cus();
    if (units < cus) return false;  // narrow C_o: the tile kernels with split-K cover it
    const int na = M <= 16 ? 1 : M <= 32 ? 2 : M <= 64 ? 4 : 8;
    const int nk = (int)(K >> 6);
    // Tiled operands with more than 32 tokens go to the kernel with loader waves: a CU moves a little more per second
    // there (fitted to the OPT-175B layers at 64 and 128 tokens), and a wave accumulates up to 4 of at most 12 units.
    const bool regs = tiled && na >= 4;
    const double cu_rate = regs ? 32e9 : 26e9, hbm_rate = regs ? 6.0e12 : 5.5e12, red_rate = 4e12, red_launch = 5e-6;
    const int s_max = regs ? kRegsMaxUnits : (na == 8 ? 24 : 16);  // widest slab the kernel shapes accumulate
    double best = 1e30, best_cu = 1e30;
    int best_gn = 0, best_gk = 0;
    for (int gk = 1; gk <= 8; ++gk) {
        if (nk % gk) continue;
        if (gk > 1 && (nk / gk < 8 || M <= 32)) continue;
        for (int s = 1; s <= s_max; ++s) {
            const int64_t gn = (units + s - 1) / s;
            const int64_t smax = (units + gn - 1) / gn;  // widest slab after dealing the units evenly
            if (s > 1 && (units + s - 2) / (s - 1) == gn) continue;  // same plan as s - 1
            const int64_t rounds = (gn * gk + cus - 1) / cus;
            const double t_cu = (double)rounds * (double)(na + smax) * 1024.0 * (nk / gk) / cu_rate;
            const double part = gk > 1 ? (double)gk * M * N * 4.0 : 0.0;
            const double t_hbm = ((double)N * K + part) / hbm_rate;
            double t = t_cu > t_hbm ? t_cu : t_hbm;
            if (gk > 1) t += red_launch + (part + 2.0 * M * N) / red_rate;
            // a clear win, or about the same modelled time with more headroom on the CU side
            if (t < best * 0.97 || (t < best * 1.03 && t_cu < best_cu)) {
                best = t < best ? t : best;
                best_cu = t_cu;
                best_gn = (int)gn;
                best_gk = gk;
            }
        }
    }
    if (!best_gn) return false;
    StreamArgs q{};
    q.gn = best_gn;
    q.gk = best_gk;
    q.units = (int)units;
    q.na = na;
    const int nblk = na + (int)((units + best_gn - 1) / best_gn);
    const int nks = nk / best_gk;
    q.ksub = 1;
    q.regs = regs ? 1 : 0;
    if (regs) {
        // a compute wave starts with its first 8 K steps of weight blocks (every other one of 16); shorter ranges go
        // to the LDS-ring kernel
        if (nks < 16) return make_stream_plan(M, N, K, batch, false, out);
    }
    if (!regs)
        for (int c = 4; c > 1; c >>= 1)
            if (nblk * c <= max_stage_blocks(na >= 4 ? 8 : 4) && nks % c == 0) { q.ksub = c; break; }
    q.iters = nks / q.ksub;
    // W is read exactly once: the non-temporal hint keeps it from displacing the activation block in the caches.
    // Measured: +7..12 % at up to 16 tokens; with more tokens it pays only for wide slabs (at least 10 units and
    // three times as many units as activation blocks) and costs a few percent otherwise.
    const int smax = nblk - na;
    q.nt_w = (regs || na == 1 || (smax >= 3 * na && smax >= 10)) ? 1 : 0;
    if (out) *out = q;
    return true;
}

}  // namespace

int sq_stream_gemm_splits(int64_t M, int64_t N, int64_t K, int64_t batch, bool tiled)
{
    StreamArgs q{};
    return make_stream_plan(M, N, K, batch, tiled, &q) ? q.gk : 0;
}

void sq_stream_gemm_launch(const GemmArgs& a, bool to_i32, bool bf16, bool tiled, hipStream_t st)
{
    StreamArgs q{};
    if (!make_stream_plan(a.M, a.N, a.K, 1, tiled, &q)) return;
    q.tiled = tiled ? 1 : 0;
    q.to_i32 = to_i32 ? 1 : 0;
    q.bf16 = bf16 ? 1 : 0;
    const dim3 grid((unsigned)(q.gn * q.gk)), block(256), block8(512);
    if (q.regs) {
        const int cnt = (q.units + q.gn - 1) / q.gn;  // widest slab
#define SQ_R(MB, C) case C: sq_launch((gemm_i8_stream_regs_kernel<MB, C, true>), grid, block8, 0, st, a, q); break;
#define SQ_R12(MB) SQ_R(MB, 1) SQ_R(MB, 2) SQ_R(MB, 3) SQ_R(MB, 4) SQ_R(MB, 5) SQ_R(MB, 6) SQ_R(MB, 7) SQ_R(MB, 8) \
                   SQ_R(MB, 9) SQ_R(MB, 10) SQ_R(MB, 11) SQ_R(MB, 12)
        static_assert(kRegsMaxUnits == 12, "launch table");
        switch (q.na) {
            case 4: switch (cnt) { SQ_R12(4) default: break; } break;
            default: switch (cnt) { SQ_R12(8) default: break; } break;
        }
#undef SQ_R12
#undef SQ_R
        return;
    }
    switch (q.na * 2 + q.nt_w) {
        case 2: sq_launch((gemm_i8_stream_kernel<1, 1, 4, 4, false>), grid, block, 0, st, a, q); break;
        case 3: sq_launch((gemm_i8_stream_kernel<1, 1, 4, 4, true>), grid, block, 0, st, a, q); break;
        case 4: sq_launch((gemm_i8_stream_kernel<1, 2, 8, 4, false>), grid, block, 0, st, a, q); break;
        case 5: sq_launch((gemm_i8_stream_kernel<1, 2, 8, 4, true>), grid, block, 0, st, a, q); break;
        case 8: sq_launch((gemm_i8_stream_kernel<1, 4, 8, 8, false>), grid, block8, 0, st, a, q); break;
        case 9: sq_launch((gemm_i8_stream_kernel<1, 4, 8, 8, true>), grid, block8, 0, st, a, q); break;
        default: sq_launch((gemm_i8_stream_kernel<2, 4, 12, 8, false>), grid, block8, 0, st, a, q); break;
    }
}
