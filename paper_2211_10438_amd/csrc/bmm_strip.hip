// Attention scores S = Q K^T in INT8 for a short contraction (K = head_dim <= 128): a kernel bound by
// writing its 16-bit output.  One workgroup owns 128 rows of one (batch, head) and walks along the row
// of 128-column tiles ("strip"), so that
//   * its Q rows are fetched once and live in registers as MFMA operands for the whole strip,
//   * the K tiles stream through a small LDS ring (global_load_lds, NS deep) filled by a fifth wave that does
//     nothing else: loads and stores of one wave retire in issue order (one vmcnt), so a wave that waited for
//     its tile loads would also wait for the stores it issued before them,
//   * every wave owns 32 complete rows x 128 columns of a tile: it stages its own 16-bit results in a
//     private LDS patch and writes 128-byte row segments, no workgroup barrier in the epilogue, and
//   * the stores of a tile stay in flight while the next tiles are computed; no compute wave ever waits for one.
// The arithmetic is the BMM of the attention block: int32 accumulators, then (float)acc * alpha rounded
// once to fp16 / bf16 (outer-dimension scaling after the integer product, Eq. 2).
#include "gemm_args.h"

namespace {

constexpr int SB_BM = 128, SB_BN = 128;
constexpr int SB_TILE = SB_BN * 128;       // one K tile in LDS: 128 rows (n) x 128 bytes (k), 16 KB
constexpr int SB_PITCH = 128 + 16;         // staging row: 64 columns of 16 bit + pad
constexpr int SB_STG = 32 * SB_PITCH;      // per-wave staging patch
constexpr int SB_LPT = SB_TILE / 1024;     // global->LDS loads of the loader wave per tile

struct StripArgs {
    int tiles_m, tiles_n, nsplit, tiles_per_wg;
};

// WPE: waves per SIMD the register allocation must allow (five waves per workgroup).
template <bool BF16, int NS, int WPE>
__global__ __launch_bounds__(320, WPE) void bmm_strip_kernel(const GemmArgs p, const StripArgs q)
{
    __shared__ __attribute__((aligned(1024))) char smem[NS * SB_TILE + 4 * SB_STG];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

    // Consecutive workgroup ids go round-robin to the 8 XCDs; give each XCD a contiguous range of the
    // logical order so that the strips of one head (they share its K rows) run on one L2.
    const int64_t total = gridDim.x;
    int64_t pid;
    {
        const int64_t wg = blockIdx.x, j = wg >> 3;
        const int xcd = (int)(wg & 7);
        const int64_t per = total >> 3;
        const int r = (int)(total & 7);
        pid = xcd * per + (xcd < r ? xcd : r) + j;
    }
    const int per_batch = q.tiles_m * q.nsplit;
    const int batch = (int)(pid / per_batch);
    const int pin = (int)(pid - (int64_t)batch * per_batch);
    const int sp = pin / q.tiles_m, tm = pin - sp * q.tiles_m;
    const int t0 = sp * q.tiles_per_wg;
    const int nt = (q.tiles_n - t0) < q.tiles_per_wg ? (q.tiles_n - t0) : q.tiles_per_wg;
    const int m0 = tm * SB_BM;
    const int kchunks = p.K >> 4;
    const int nks = (p.K + 31) >> 5;
    // The strips of a head start at different tiles of their row and wrap around.  Strips that run side by side
    // would otherwise all write the same 256-byte column range of their rows at the same time, i.e. addresses that
    // agree in the bits that select the memory channel; measured at 768 heads x 2048 x 2048 that costs a third of
    // the store bandwidth, while shapes that happen to fall out of step by themselves gain nothing from lockstep.
    const int rot = tm % nt;
    auto tile_at = [&](int j) { const int t = j + rot; return t0 + (t < nt ? t : t - nt); };

    if (wave == 4) {
        // ---- loader wave.  LDS image of a K tile: row n at n*128, its eight 16-byte chunks XOR-permuted with
        // (n & 7) so that the operand reads (32 rows, one chunk) spread over all banks.  One wave-wide load fills
        // 1 KB = 8 rows; lane l lands at byte l*16 of the block and therefore fetches chunk (l & 7) ^ (l >> 3) of
        // row (l >> 3): eight neighbouring lanes read one whole 128-byte row.  Chunks past K re-read chunk 0
        // (their Q side is zero).  Past the end of the strip the last tile is fetched again into a buffer nobody
        // reads, which keeps the number of loads in flight (the s_waitcnt immediate) constant.
        const int8_t* Bb = p.B + (int64_t)batch * p.strideB;
        const int lrow = lane >> 3;
        int c = (lane & 7) ^ lrow;
        c = c < kchunks ? c : 0;
        const uint32_t off0 = (uint32_t)(lrow * (int)p.ldb + c * 16);
        const uint32_t blk = (uint32_t)(8 * (int)p.ldb);
        auto issue_tile = [&](int t, int buf) {
            const int8_t* b = Bb + (int64_t)t * SB_BN * p.ldb + off0;
#pragma unroll
            for (int i = 0; i < SB_LPT; ++i)
                __builtin_amdgcn_global_load_lds(GPTR(b + i * blk), LPTR(smem + buf * SB_TILE + i * 1024), 16, 0, 0);
        };
#pragma unroll
        for (int s = 0; s < NS - 1; ++s) issue_tile(tile_at(s < nt ? s : nt - 1), s);
        int buf = 0;
        for (int j = 0; j < nt; ++j) {
            wait_vmcnt_imm<(NS - 2) * SB_LPT>();  // tile j has landed
            __builtin_amdgcn_s_barrier();         // ... is visible to the compute waves, and they are done with tile j-1
            const int nxt = j + NS - 1;
            issue_tile(tile_at(nxt < nt ? nxt : nt - 1), buf == 0 ? NS - 1 : buf - 1);
            buf = buf + 1 == NS ? 0 : buf + 1;
        }
        wait_vmcnt_imm<0>();  // nothing may still be landing when the workgroup's LDS is released
        return;
    }

    // ---- compute waves: 32 rows each.  Q operand fragments (second MFMA operand): lane l feeds output row
    // (l & 31) of this wave with the 16 bytes of K chunk 2*ks + (l >> 5).  Rows past M repeat row M-1 (their
    // results are written onto row M-1 with identical values); chunks past K are zero.
    v4i fq[4];
    {
        int row = m0 + wave * 32 + (lane & 31);
        row = row < p.M ? row : p.M - 1;
        const int8_t* qp = p.A + (int64_t)batch * p.strideA + (int64_t)row * p.lda;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int c = 2 * ks + (lane >> 5);
            fq[ks] = v4i{0, 0, 0, 0};
            if (c < kchunks) fq[ks] = *(const v4i*)(qp + c * 16);
        }
    }
    // K operand fragment of n block jn, K step ks: row 32*jn + (l & 31), chunk 2*ks + (l >> 5)
    int foff[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) foff[ks] = (lane & 31) * 128 + (((2 * ks + (lane >> 5)) ^ (lane & 7)) * 16);

    uint16_t* C = (uint16_t*)p.C + (int64_t)batch * p.strideC;
    char* stg = smem + NS * SB_TILE + wave * SB_STG;
    // staging: results of lane l go to row (l & 31); reading back, lane l takes chunk (l & 7) of row 8*i + (l >> 3)
    const int st_w = (lane & 31) * SB_PITCH + (lane >> 5) * 8;
    const int st_r = (lane >> 3) * SB_PITCH + (lane & 7) * 16;
    int64_t dst_off[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int row = m0 + wave * 32 + i * 8 + (lane >> 3);
        row = row < p.M ? row : p.M - 1;
        dst_off[i] = (int64_t)row * p.N + (lane & 7) * 8;
    }
    const float alpha = p.alpha;

    int buf = 0;
    for (int j = 0; j < nt; ++j) {
        __builtin_amdgcn_s_barrier();  // tile j is in LDS
        v16i acc[4];
        const char* tb = smem + buf * SB_TILE;
#pragma unroll
        for (int jn = 0; jn < 4; ++jn) {
            const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
            acc[jn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(*(const v4i*)(tb + jn * 4096 + foff[0]), fq[0], zero, 0, 0, 0);
        }
#pragma unroll
        for (int ks = 1; ks < 4; ++ks) {
            if (ks < nks) {
#pragma unroll
                for (int jn = 0; jn < 4; ++jn)
                    acc[jn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(*(const v4i*)(tb + jn * 4096 + foff[ks]), fq[ks], acc[jn], 0, 0, 0);
            }
        }
        // ---- epilogue: accumulator block jn is the transposed 32x32 output block, lane l register v holds output
        // row (l & 31), column 8*(v/4) + 4*(l >> 5) + (v & 3); two halves of 64 columns go through the staging patch.
        // The stores are never waited for: they drain while the following tiles are computed.
        uint16_t* ct = C + (int64_t)tile_at(j) * SB_BN;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
#pragma unroll
            for (int jj = 0; jj < 2; ++jj)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const uint32_t o01 = dequant_pair<BF16>(acc[2 * h + jj][4 * g], acc[2 * h + jj][4 * g + 1], alpha, alpha, 0.0f, 0.0f, false,
                                                            false, 0u, false);
                    const uint32_t o23 = dequant_pair<BF16>(acc[2 * h + jj][4 * g + 2], acc[2 * h + jj][4 * g + 3], alpha, alpha, 0.0f, 0.0f,
                                                            false, false, 0u, false);
                    *(v2u*)(stg + st_w + (jj * 32 + 8 * g) * 2) = v2u{o01, o23};
                }
            __builtin_amdgcn_wave_barrier();  // LDS serves one wave's accesses in order; keep the compiler from reordering
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const v4u val = *(const v4u*)(stg + st_r + i * 8 * SB_PITCH);
                __builtin_nontemporal_store(val, (v4u*)(ct + dst_off[i] + h * 64));
            }
            __builtin_amdgcn_wave_barrier();
        }
        buf = buf + 1 == NS ? 0 : buf + 1;
    }
}

}  // namespace

bool sq_strip_bmm_eligible(int64_t M, int64_t N, int64_t K, int64_t batch)
{
    // whole 128-column tiles, the contraction in one LDS row, enough rows that Q reuse pays; the grid is one-dimensional
    const int64_t wgs = batch * ((M + SB_BM - 1) / SB_BM) * (N / SB_BN);  // upper bound: every strip split into single tiles
    return M > 128 && K <= 128 && (K & 15) == 0 && (N & 127) == 0 && batch >= 1 && wgs < ((int64_t)1 << 31);
}

void sq_strip_bmm_launch(const GemmArgs& a, int batch, bool bf16, hipStream_t st)
{
    StripArgs q{};
    q.tiles_m = (a.M + SB_BM - 1) / SB_BM;
    q.tiles_n = a.N / SB_BN;
    // Short strips when there are few (batch, row block) pairs: about eight workgroups per CU keep the chip full.
    int nsplit = 1;
    while ((int64_t)batch * q.tiles_m * nsplit < 8 * 256 && nsplit * 2 <= q.tiles_n) nsplit *= 2;
    q.tiles_per_wg = (q.tiles_n + nsplit - 1) / nsplit;
    q.nsplit = (q.tiles_n + q.tiles_per_wg - 1) / q.tiles_per_wg;
    dim3 grid((unsigned)((int64_t)batch * q.tiles_m * q.nsplit));
    // Long strips: a three-deep ring and two workgroups per CU.  Short strips (the prologue weighs more): a
    // two-deep ring, three workgroups per CU.
    if (q.tiles_per_wg <= 6) {
        if (bf16) sq_launch((bmm_strip_kernel<true, 2, 4>), grid, dim3(320), 0, st, a, q);
        else sq_launch((bmm_strip_kernel<false, 2, 4>), grid, dim3(320), 0, st, a, q);
    } else {
        if (bf16) sq_launch((bmm_strip_kernel<true, 3, 3>), grid, dim3(320), 0, st, a, q);
        else sq_launch((bmm_strip_kernel<false, 3, 3>), grid, dim3(320), 0, st, a, q);
    }
}
