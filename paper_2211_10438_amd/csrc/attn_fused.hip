// Fused INT8 attention for gfx950: O = (P_q V_q) * alpha2 with P_q = round(127 * softmax16(S)), S = round16((Q_q K_q^T) * alpha1),
// in one kernel that never writes the score or probability tensors.
//
// The attention block of Sec. 4 runs both batched matmuls in INT8 and keeps the softmax in the 16-bit
// floating type; the unfused chain (sq_w8a8_bmm, sq_softmax_quant_p, sq_w8a8_bmm) moves the [s_q, s_k]
// tensors S (16-bit) and P_q (int8) through HBM twice each, 19 of the 20 GB it touches at 768 heads x 2048^2.
// This kernel keeps the same quantization points -- scores rounded to 16 bits before the softmax,
// probabilities rounded to 16 bits and then to codes with the fixed step 1/127 -- and recomputes Q K^T
// instead of storing it:
//   pass 1  over the key tiles: S tile by MFMA, running row maximum and sum of exponentials (online softmax);
//   pass 2  over the key tiles again: S tile by MFMA, p = e^(s - m) / l, p16, code = round(127 p16); the 16
//           codes a lane produces from one 32x32 accumulator block ARE its operand fragment of the P V
//           MFMA (second operand: row l & 31, contraction bytes 16 (l >> 5) ..), so P_q never leaves registers.
// One workgroup owns 128 query rows of one (batch, head): four waves of 32 rows, the Q operand fragments in
// registers for the whole kernel.  K and V tiles of 128 keys travel L2 -> LDS with global_load_lds, double
// buffered, one s_barrier per tile.  Because the Q K^T MFMA takes the K rows as first operand, an accumulator
// block is the transpose of its output block: a lane holds, for its row, the columns 8g + 4h + e of a 32-key
// block (h = l >> 5).  That fixes the order of the contraction bytes of the P V MFMA; the V operand is fetched
// in the same order with the LDS transpose read (ds_read_b64_tr_b8), whose eight source rows are named by the
// lanes and can therefore be any eight keys.
// The kernel is bound by the vector ALU (about 21 issue slots per score over both passes against 0.75 MFMA
// cycles); two workgroups per compute unit let one wave's MFMAs run under the other's exponentials.
#include <type_traits>

#include "gemm_args.h"

namespace {

struct AttnArgs {
    const int8_t* Q;  // [b][s_q, d]
    const int8_t* K;  // [b][s_k, d]
    const int8_t* V;  // [b][s_k, d]
    void* O;          // [b][s_q, d] 16-bit
    int8_t* P;        // optional [b][s_q, s_k]: the probability codes, for inspection; or NULL
    int s_q, s_k, tiles_m;  // tiles_m: workgroups per batch entry (row blocks of 128 queries; pairs of them in the causal form)
    int64_t stride_q, stride_k, stride_v, stride_o;  // batch strides in elements
    float alpha1, alpha2;
};

constexpr float kLog2e = 1.44269504088896340736f;
constexpr int kIntMin = -2147483647 - 1;

// MODE, one instantiation each, so that the common case carries no mask tests (with the first two forms in one kernel
// the register allocation spilled):
//   kAll     every query sees every key, and the key count is a multiple of 128;
//   kTail    the same with any key count that is a multiple of 16: the last tile is masked at 16-key granularity;
//   kCausal  query i sees the keys j <= i + (s_k - s_q) (the decoder's mask; the last query sees every key).  A workgroup
//            stops after the last tile any of its rows sees; a wave runs the unmasked tile body on the tiles all its 32
//            rows see in full, an element-wise masked one on the one or two tiles the diagonal crosses, and nothing on
//            the tiles past its rows.  The element mask also hides keys past s_k, so no separate tail form is needed.
constexpr int kAll = 0, kTail = 1, kCausal = 2;

template <bool BF16, int HD, int MODE>
__global__ __launch_bounds__(256, 2) void attn_i8_kernel(const AttnArgs p)
{
    constexpr bool TAIL = MODE == kTail;
    constexpr int TK = 128;               // keys per tile
    constexpr int SLOT = 16384;           // LDS bytes reserved per tile
    constexpr int TILE = TK * HD;         // bytes of a K or V tile
    constexpr int LPT = TILE / 1024 / 4;  // global->LDS loads per wave and tile
    constexpr int CH = HD / 16;           // 16-byte chunks per row
    constexpr int RPB = 1024 / HD;        // rows per 1 KB block
    constexpr int NKS = HD / 32;          // MFMA steps of Q K^T
    constexpr int NB = HD / 32;           // 32-column blocks of O
    static_assert(HD == 128 || HD == 64, "head dimension");
    __shared__ __attribute__((aligned(1024))) char smem[4 * SLOT];  // stage s: K tile at slot 2s, V tile at slot 2s + 1

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r32 = lane & 31, h = lane >> 5;

    // Consecutive workgroup ids go round-robin to the 8 XCDs; give each XCD a contiguous range of the logical
    // order so that the row blocks of one head (they share its K and V) run on one L2.
    const int64_t total = gridDim.x;
    int64_t pid;
    {
        const int64_t wg = blockIdx.x, j = wg >> 3;
        const int xcd = (int)(wg & 7);
        const int64_t per = total >> 3;
        const int r = (int)(total & 7);
        pid = xcd * per + (xcd < r ? xcd : r) + j;
    }
    // Causal form: a workgroup owns TWO row blocks of its head, number `pair` from the top and from the bottom of the
    // query range, one after the other: block t sees t + 1 of the key tiles (with s_k = s_q), so every pair sees the
    // same number of tiles and the workgroups finish together (with one block each, the blocks that start last
    // decided the time: 157 us against 99 us of work per slot at 288 heads x 1024^2).  tiles_m counts pairs then.
    const int blocks_m = (p.s_q + 127) / 128;
    const int batch = (int)(pid / p.tiles_m);
    const int pair = (int)(pid - (int64_t)batch * p.tiles_m);
    const int nrep = (MODE == kCausal && blocks_m - 1 - pair != pair) ? 2 : 1;
    for (int rep = 0; rep < nrep; ++rep) {
        if (rep) __syncthreads();  // the staging patches of the first block's epilogue lie in the tile buffers
        const int mt = MODE == kCausal ? (rep == 0 ? blocks_m - 1 - pair : pair) : pair;
        const int m0 = mt * 128;
        const int nt_all = (p.s_k + TK - 1) / TK;
        const int last16 = (p.s_k - (nt_all - 1) * TK) >> 4;  // valid 16-key groups of the last tile (8 = full; s_k % 16 == 0)
        // Causal: keys visible to row r: 0 .. r + coff.  Tiles of this workgroup: up to the last key its last valid row sees;
        // tiles j < jfull are seen in full by every row of this wave, tiles j >= jend by none of them.
        const int coff = p.s_k - p.s_q;
        int nt = nt_all, jfull = nt_all, jend = nt_all;
        if constexpr (MODE == kCausal) {
            const int last_row = m0 + 127 < p.s_q ? m0 + 127 : p.s_q - 1;
            nt = (last_row + coff + 1 + TK - 1) / TK;
            const int w0 = m0 + wave * 32;
            jfull = (w0 + coff + 1) / TK;
            jend = (w0 + 31 + coff + 1 + TK - 1) / TK;
            jfull = jfull < nt ? jfull : nt;
            jend = jend < nt ? jend : nt;
        }
        // key index of accumulator register 4 g + e of key block ks in tile j: 128 j + 32 ks + 8 g + 4 h + e; it is visible
        // to this lane's row when 32 ks + 8 g + e <= rowlim - 128 j
        const int rowlim = m0 + wave * 32 + r32 + coff - 4 * h;

        // ---- LDS images.  K tile: row n at n * HD, its 16-byte chunks XOR-permuted (position = chunk ^ swzK(n)) so
        // that the operand reads (32 rows, one chunk) spread over the banks.  V tile: row k at k * HD, position =
        // chunk ^ swzV(k), chosen so that the eight rows of one transpose read sit at eight different positions.
        auto swzK = [](int r) { return HD == 128 ? (r & 7) : (((r >> 1) & 3) ^ ((r >> 3) & 1)); };
        auto swzV = [](int k) { return HD == 128 ? ((k & 3) | (((k >> 3) & 1) << 2)) : (k & 3); };
        // Key rows past s_k (last, partial tile) re-read row s_k - 1: their scores are masked below and their V rows meet
        // codes that are zero.
        int lrow[LPT];
        uint32_t cK[LPT], cV[LPT];
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const int row = (i * 4 + wave) * RPB + lane / CH, pos = lane % CH;
            lrow[i] = row;
            cK[i] = (uint32_t)((pos ^ swzK(row)) * 16);
            cV[i] = (uint32_t)((pos ^ swzV(row)) * 16);
        }
        const int8_t* Kb = p.K + (int64_t)batch * p.stride_k;
        const int8_t* Vb = p.V + (int64_t)batch * p.stride_v;
        auto issue = [&](int j, int stage, bool with_v) {
            char* dk = smem + (2 * stage) * SLOT;
            int64_t roff[LPT];
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                int r = j * TK + lrow[i];
                r = r < p.s_k ? r : p.s_k - 1;
                roff[i] = (int64_t)r * HD;
            }
#pragma unroll
            for (int i = 0; i < LPT; ++i)
                __builtin_amdgcn_global_load_lds(GPTR(Kb + roff[i] + cK[i]), LPTR(dk + (i * 4 + wave) * 1024), 16, 0, 0);
            if (with_v) {
#pragma unroll
                for (int i = 0; i < LPT; ++i)
                    __builtin_amdgcn_global_load_lds(GPTR(Vb + roff[i] + cV[i]), LPTR(dk + SLOT + (i * 4 + wave) * 1024), 16, 0, 0);
            }
        };

        // ---- Q operand fragments (second MFMA operand): lane l feeds query row (l & 31) of this wave with the 16
        // bytes of chunk 2 ks + (l >> 5).  Rows past s_q repeat the last row; they are never stored.
        v4i fq[NKS];
        {
            int row = m0 + wave * 32 + r32;
            row = row < p.s_q ? row : p.s_q - 1;
            const int8_t* qp = p.Q + (int64_t)batch * p.stride_q + (int64_t)row * HD;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) fq[ks] = *(const v4i*)(qp + (2 * ks + h) * 16);
        }
        // K operand fragment (first operand) of key block jn, step ks: key row 32 jn + (l & 31), chunk 2 ks + (l >> 5)
        int koff[NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) koff[ks] = r32 * HD + (((2 * ks + h) ^ swzK(r32)) * 16);
        // V operand fragment (first operand of the P V MFMA) of key block ks, column block jn: column n = 32 jn + (l & 31),
        // contraction bytes in the order the codes have in the P fragment: byte 4g + e <-> key 32 ks + 8g + 4h + e.
        // Within 16 lanes, source lanes 2j and 2j + 1 of a transpose read name the two 8-byte halves of the 16 columns
        // of one key row, and lane i receives column i of the eight rows: rows j = 0..3 are keys 4h + j, rows 4..7 keys
        // 8 + 4h + (j - 4); the second read takes the keys 16 further on.
        int voff;
        {
            const int s = lane & 15, j = s >> 1, cb = (lane >> 4) & 1;
            const int key = 4 * h + (j & 3) + 8 * (j >> 2);
            voff = key * HD + ((cb ^ swzV(key)) * 16) + (s & 1) * 8;  // chunk 2 jn + cb: jn enters below (XOR on bits 1.., swzV < 8)
        }
        auto v_frag = [&](const char* vt, int ks, int jn) {
            // position of chunk (2 jn + cb) = (2 jn + cb) ^ swz = ((2 jn) ^ (cb ^ swz)) as 2 jn has bit 0 clear
            const int a = (voff ^ ((2 * jn) << 4)) + ks * 32 * HD;
            const v2i lo = __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) v2i*)(vt + a));
            const v2i hi = __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) v2i*)(vt + a + 16 * HD));
            return v4i{lo.x, lo.y, hi.x, hi.y};
        };

        // S tile = Q K^T for the 128 keys of a stage: acc[jn] is the transposed 32x32 block of key block jn
        auto scores = [&](const char* kt, v16i(&acc)[4]) {
#pragma unroll
            for (int jn = 0; jn < 4; ++jn) {
                const v16i zero = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
                acc[jn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(*(const v4i*)(kt + jn * 32 * HD + koff[0]), fq[0], zero, 0, 0, 0);
            }
#pragma unroll
            for (int ks = 1; ks < NKS; ++ks)
#pragma unroll
                for (int jn = 0; jn < 4; ++jn)
                    acc[jn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(*(const v4i*)(kt + jn * 32 * HD + koff[ks]), fq[ks], acc[jn], 0, 0, 0);
        };
        // score of one accumulator as the 16-bit tensor element it stands for, widened again: round16(fl32(acc * alpha1))
        const float alpha1 = p.alpha1;
        auto s16f = [&](int a) { return load16_bits<BF16>(store16_bits<BF16>((float)a * alpha1)); };
        // two scores at once: one narrowing instruction for the pair
        auto s16f2 = [&](int a0, int a1, float& s0, float& s1) {
            const uint32_t h = store16x2_bits<BF16>((float)a0 * alpha1, (float)a1 * alpha1);
            s0 = load16_bits<BF16>(h);
            s1 = load16_bits<BF16>(h >> 16);
        };
        // (Both passes must round the scores the same way: where one key dominates a row, l is 1 up to rounding, and a
        // score that came out one 16-bit ulp lower in pass 1 than in pass 2 would give that key a probability above 1.
        // A single-rounding v_fma_mixlo_f16 in pass 1 was tried for its one issue slot and did exactly that.)

        // ---- pass 1: row maximum m and l = sum e^(s - m), online.  The maximum is taken on the integer accumulators
        // (s is monotone in acc: alpha1 > 0).  A row's scores are split between lanes r and r + 32.
        float m_run = -__builtin_inff(), l_run = 0.0f;
        // MASK: a 16-key group q = 2 jn + (v >> 3) of the tile is valid when q < tail16 (8 for every tile but the last) (uniform over the wave: the accumulator registers 8 (q & 1) .. 8 (q & 1) + 7 of block jn)
        // EM: element-wise mask (the diagonal tiles of the causal form), lim = rowlim - 128 j
        auto pass1_tile = [&](const char* kt, int tail16, auto EM_, int lim) {
            constexpr bool MASK = TAIL;
            constexpr bool EM = decltype(EM_)::value;
            v16i acc[4];
            scores(kt, acc);
            int imax = EM ? kIntMin : acc[0][0];  // (key 0 of a tile is always valid without the element mask)
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                if (MASK && q >= tail16) continue;
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    const int r = 8 * (q & 1) + v;  // register 4 g + e
                    int a = acc[q >> 1][r];
                    if (EM) a = 32 * (q >> 1) + 8 * (r >> 2) + (r & 3) <= lim ? a : kIntMin;
                    imax = a > imax ? a : imax;
                }
            }
            const int other = __shfl_xor(imax, 32, 64);
            imax = other > imax ? other : imax;
            const float m_new = __builtin_fmaxf(m_run, s16f(imax));
            l_run *= __builtin_amdgcn_exp2f((m_run - m_new) * kLog2e);
            m_run = m_new;
            const float nm = -m_new * kLog2e;
            float part = 0.0f;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                if (MASK && q >= tail16) continue;
#pragma unroll
                for (int v = 0; v < 8; v += 2) {
                    float s0, s1;
                    const int r = 8 * (q & 1) + v;
                    s16f2(acc[q >> 1][r], acc[q >> 1][r + 1], s0, s1);
                    const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s0, kLog2e, nm));
                    const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s1, kLog2e, nm));
                    const int idx = 32 * (q >> 1) + 8 * (r >> 2) + (r & 3);
                    // (a hidden key's exponential may be anything, even infinite: it is dropped, not multiplied away)
                    part += (!EM || idx <= lim) ? e0 : 0.0f;
                    part += (!EM || idx + 1 <= lim) ? e1 : 0.0f;
                }
            }
            l_run += part;
        };
        using Plain = std::false_type;
        using Masked = std::true_type;
        issue(0, 0, false);
        for (int j = 0; j < nt; ++j) {
            wait_vmcnt_imm<0>();           // this wave's part of tile j has landed
            __builtin_amdgcn_s_barrier();  // ... everybody's has, and everybody is done with tile j - 1
            if (j + 1 < nt) issue(j + 1, (j + 1) & 1, false);
            const char* kt1 = smem + (2 * (j & 1)) * SLOT;
            if constexpr (MODE == kCausal) {
                if (j < jfull) pass1_tile(kt1, 8, Plain{}, 0);
                else if (j < jend) pass1_tile(kt1, 8, Masked{}, rowlim - j * TK);
            } else {
                pass1_tile(kt1, j == nt - 1 ? last16 : 8, Plain{}, 0);
            }
        }
        // p = e^(s - m) / l = 2^(s log2(e) - (m log2(e) + log2(l))): the division is folded into the exponent
        const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
        const float nm = -m_run * kLog2e - __builtin_amdgcn_logf(l_tot);

        // ---- pass 2: codes and P V.
        v16i acc_o[NB];
#pragma unroll
        for (int jn = 0; jn < NB; ++jn)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc_o[jn][v] = 0;
        int8_t* Prow = nullptr;
        if (p.P) {
            const int row = m0 + wave * 32 + r32;
            if (row < p.s_q) Prow = p.P + ((int64_t)batch * p.s_q + row) * (int64_t)p.s_k + 4 * h;
        }
        auto pass2_tile = [&](const char* kt, int j, int tail16, auto EM_, int lim) {
            constexpr bool MASK = TAIL;
            constexpr bool EM = decltype(EM_)::value;
            const char* vt = kt + SLOT;
            v16i acc[4];
            scores(kt, acc);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (MASK && 2 * ks >= tail16) break;  // no valid key in this block or the following ones
                // the 16 codes of this lane for key block ks: word g holds columns 8g + 4h + 0..3
                v4i fp;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    if (MASK && 2 * ks + (g >> 1) >= tail16) {  // masked keys: probability 0
                        fp[g] = 0;
                        continue;
                    }
                    uint32_t ph[2];  // the probabilities of columns e = 0,1 and 2,3 as 16-bit pairs (the softmax output is a 16-bit tensor)
#pragma unroll
                    for (int e = 0; e < 4; e += 2) {
                        float s0, s1;
                        s16f2(acc[ks][4 * g + e], acc[ks][4 * g + e + 1], s0, s1);
                        float pr0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s0, kLog2e, nm));
                        float pr1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s1, kLog2e, nm));
                        if (EM) {  // hidden keys: probability 0
                            pr0 = 32 * ks + 8 * g + e <= lim ? pr0 : 0.0f;
                            pr1 = 32 * ks + 8 * g + e + 1 <= lim ? pr1 : 0.0f;
                        }
                        ph[e >> 1] = store16x2_bits<BF16>(pr0, pr1);
                    }
                    if constexpr (BF16) {
                        // round(127 p16): the product is exact in fp32, the add of 1.5 * 2^23 rounds it to nearest-even and
                        // leaves the code in the low mantissa byte
                        uint32_t q[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            q[e] = __builtin_bit_cast(uint32_t, __builtin_fmaf(load16_bits<true>(ph[e >> 1] >> ((e & 1) * 16)), 127.0f, 12582912.0f));
                        fp[g] = (int)pack4_low_bytes(q[0], q[1], q[2], q[3]);
                    } else {
                        // the same in packed fp16, two codes per instruction: fma(p16, 127, 1024) is one rounding of the exact
                        // 127 p16 + 1024 to a grid of spacing 1 (fp16 in [1024, 2048)), i.e. 1024 + round-half-even(127 p16), the
                        // code in the low byte of each half; one byte permute gathers the four codes
                        const sq_f16x2 k127 = {(_Float16)127.0f, (_Float16)127.0f}, k1024 = {(_Float16)1024.0f, (_Float16)1024.0f};
                        const uint32_t c01 = __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(__builtin_bit_cast(sq_f16x2, ph[0]), k127, k1024));
                        const uint32_t c23 = __builtin_bit_cast(uint32_t, __builtin_elementwise_fma(__builtin_bit_cast(sq_f16x2, ph[1]), k127, k1024));
                        fp[g] = (int)__builtin_amdgcn_perm(c23, c01, 0x06040200u);
                    }
                }
                if (Prow) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const bool inside = MODE == kCausal ? j * TK + ks * 32 + 8 * g + 4 * h < p.s_k : (!MASK || 2 * ks + (g >> 1) < tail16);
                        if (inside) *(int*)(Prow + j * TK + ks * 32 + 8 * g) = fp[g];
                    }
                }
#pragma unroll
                for (int jn = 0; jn < NB; ++jn)
                    acc_o[jn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(v_frag(vt, ks, jn), fp, acc_o[jn], 0, 0, 0);
            }
        };
        __syncthreads();  // every wave is done with the last tile of pass 1 before its buffer is refilled
        issue(0, 0, true);
        for (int j = 0; j < nt; ++j) {
            wait_vmcnt_imm<0>();
            __builtin_amdgcn_s_barrier();
            if (j + 1 < nt) issue(j + 1, (j + 1) & 1, true);
            const char* kt2 = smem + (2 * (j & 1)) * SLOT;
            if constexpr (MODE == kCausal) {
                if (j < jfull) pass2_tile(kt2, j, 8, Plain{}, 0);
                else if (j < jend) pass2_tile(kt2, j, 8, Masked{}, rowlim - j * TK);
            } else {
                pass2_tile(kt2, j, j == nt - 1 ? last16 : 8, Plain{}, 0);
            }
        }
        if constexpr (MODE == kCausal) {
            // the codes of the tiles this wave skipped are 0
            if (Prow)
                for (int c = jend * TK; c + 4 * h < p.s_k; c += 8) *(int*)(Prow + c) = 0;  // (Prow already points at column 4 h)
        }

        // ---- epilogue: o = round16(fl32(acc * alpha2)).  Accumulator block jn is the transposed output block: lane l,
        // register v holds row (l & 31), column 32 jn + 8 (v / 4) + 4 (l >> 5) + (v & 3).  Each wave stages its 32 rows in
        // its own part of the (now free) tile buffers and writes whole rows in 16-byte pieces.
        constexpr int PITCH = HD * 2 + 16;
        __syncthreads();
        char* stg = smem + wave * SLOT;
        const float alpha2 = p.alpha2;
#pragma unroll
        for (int jn = 0; jn < NB; ++jn)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const uint32_t o01 = dequant_pair<BF16>(acc_o[jn][4 * g], acc_o[jn][4 * g + 1], alpha2, alpha2, 0.0f, 0.0f, false, false, 0u, false);
                const uint32_t o23 = dequant_pair<BF16>(acc_o[jn][4 * g + 2], acc_o[jn][4 * g + 3], alpha2, alpha2, 0.0f, 0.0f, false, false, 0u, false);
                *(v2u*)(stg + r32 * PITCH + (32 * jn + 8 * g + 4 * h) * 2) = v2u{o01, o23};
            }
        __builtin_amdgcn_wave_barrier();
        uint16_t* Ob = (uint16_t*)p.O + (int64_t)batch * p.stride_o;
        constexpr int CPR = HD / 8;  // 16-byte pieces per row
#pragma unroll
        for (int it = 0; it < 32 * CPR / 64; ++it) {
            const int idx = it * 64 + lane, r = idx / CPR, c = idx - r * CPR;
            const int row = m0 + wave * 32 + r;
            const v4u val = *(const v4u*)(stg + r * PITCH + c * 16);
            if (row < p.s_q) __builtin_nontemporal_store(val, (v4u*)(Ob + (int64_t)row * HD + c * 8));
        }
    }  // row blocks of this workgroup
}

}  // namespace

static sq_status attention(const int8_t* q, const int8_t* k, const int8_t* v, float alpha1, float alpha2, void* o,
                           sq_dtype out, int64_t b, int64_t s_q, int64_t s_k, int64_t d, int64_t stride_q,
                           int64_t stride_k, int64_t stride_v, int64_t stride_o, int8_t* p_codes, void* stream, bool causal)
{
    if (!q || !k || !v || !o) return SQ_ERR_NULL;
    const int64_t lim = (int64_t)1 << 31;
    if (b <= 0 || s_q <= 0 || s_k <= 0 || d <= 0 || s_q >= lim || s_k >= lim) return SQ_ERR_SHAPE;
    if (causal && s_k < s_q) return SQ_ERR_SHAPE;  // the first queries would see no key at all
    const int64_t tiles_m = (s_q + 127) / 128;
    if (b * tiles_m >= lim) return SQ_ERR_SHAPE;
    if (stride_q < s_q * d || stride_k < s_k * d || stride_v < s_k * d || stride_o < s_q * d) return SQ_ERR_SHAPE;
    if (out != SQ_F16 && out != SQ_BF16) return SQ_ERR_UNSUPPORTED;
    if (d != 64 && d != 128) return SQ_ERR_UNSUPPORTED;
    if (s_k & 15) return SQ_ERR_ALIGN;
    if (!(alpha1 > 0.0f) || !(alpha1 < __builtin_inff()) || !(alpha2 == alpha2)) return SQ_ERR_UNSUPPORTED;
    if ((stride_q & 15) || (stride_k & 15) || (stride_v & 15) || (stride_o & 7) || !sq_aligned16(q) || !sq_aligned16(k) ||
        !sq_aligned16(v) || !sq_aligned16(o) || (p_codes && (reinterpret_cast<uintptr_t>(p_codes) & 3u)))
        return SQ_ERR_ALIGN;
    AttnArgs a{};
    a.Q = q; a.K = k; a.V = v; a.O = o; a.P = p_codes;
    a.s_q = (int)s_q; a.s_k = (int)s_k;
    a.tiles_m = (int)(causal ? (tiles_m + 1) / 2 : tiles_m);  // causal: workgroups own pairs of row blocks
    a.stride_q = stride_q; a.stride_k = stride_k; a.stride_v = stride_v; a.stride_o = stride_o;
    a.alpha1 = alpha1; a.alpha2 = alpha2;
    const dim3 grid((unsigned)(b * a.tiles_m)), block(256);
    hipStream_t st = (hipStream_t)stream;
    const bool tail = (s_k & 127) != 0;
#define SQ_ATTN(BF, HD)                                                                        \
    do {                                                                                       \
        if (causal) sq_launch((attn_i8_kernel<BF, HD, kCausal>), grid, block, 0, st, a);       \
        else if (tail) sq_launch((attn_i8_kernel<BF, HD, kTail>), grid, block, 0, st, a);      \
        else sq_launch((attn_i8_kernel<BF, HD, kAll>), grid, block, 0, st, a);                 \
    } while (0)
    if (d == 128) {
        if (out == SQ_BF16) SQ_ATTN(true, 128); else SQ_ATTN(false, 128);
    } else {
        if (out == SQ_BF16) SQ_ATTN(true, 64); else SQ_ATTN(false, 64);
    }
#undef SQ_ATTN
    return sq_launch_status();
}

extern "C" sq_status sq_w8a8_attention(const int8_t* q, const int8_t* k, const int8_t* v, float alpha1, float alpha2, void* o,
                                       sq_dtype out, int64_t b, int64_t s_q, int64_t s_k, int64_t d, int64_t stride_q,
                                       int64_t stride_k, int64_t stride_v, int64_t stride_o, int8_t* p_codes, void* stream)
{
    return attention(q, k, v, alpha1, alpha2, o, out, b, s_q, s_k, d, stride_q, stride_k, stride_v, stride_o, p_codes, stream, false);
}

extern "C" sq_status sq_w8a8_attention_causal(const int8_t* q, const int8_t* k, const int8_t* v, float alpha1, float alpha2, void* o,
                                              sq_dtype out, int64_t b, int64_t s_q, int64_t s_k, int64_t d, int64_t stride_q,
                                              int64_t stride_k, int64_t stride_v, int64_t stride_o, int8_t* p_codes, void* stream)
{
    return attention(q, k, v, alpha1, alpha2, o, out, b, s_q, s_k, d, stride_q, stride_k, stride_v, stride_o, p_codes, stream, true);
}
