// Streaming GEMM kernel for bf16 on gfx950: C[M][N] = A[M][K] * B[N][K]^T with both
// operands K-contiguous (the GMM template with A as MK and B as NK, and equally a 1x1
// stride-1 convolution over NHWC activations with OHWI weights), fp32 accumulation.
//
// BT: B is stored [K][N] instead (row-major B, the GMM's default layout).  Its stage is then
// [BK rows of k][BN columns], still loaded straight into LDS in 16-byte chunks of eight
// columns, and the MFMA operand (eight consecutive k of one column per lane) comes out of it
// through the LDS transpose read of gfx950 (ds_read_b64_tr_b16): the 16 lanes of a group each
// give the address of four consecutive columns, lanes 4j .. 4j+3 on row j, and lane i
// receives column i of the four rows.  Two such reads (rows 0..3 and 4..7 of the lane's k
// half) make one 16-byte fragment, so the B layout costs no register transposes and no extra
// LDS traffic, only two 8-byte reads where the NK layout takes one 16-byte read.
//
// Both operand tiles of a K step go from global memory straight into a ring of LDS
// stages (no registers in between); everything else is the machinery of the direct
// convolution (dconv.h): asynchronous fragment reads that run ahead of the MFMAs,
// K groups inside the workgroup, the fused split-K tail, the shared epilogue.
#pragma once

#include "dconv.h"

namespace alt {

// KW groups of WGM x WGN waves; group kg handles channels [kg, kg + 1) * Cs / KW of the
// workgroup's slice in steps of BK (64 or 32), through a ring of NS stages of its own.
// While a step computes, NS - 2 later stages are in flight: deep rings of small stages
// (BK = 32) cover the load latency with the same LDS as shallow rings of large ones.
template <int BM, int BN, int WGM, int WGN, int KW, int NS, int BK, bool BT = false>
__global__ __launch_bounds__(64 * WGM * WGN * KW, ALT_DCONV_MIN_WAVES((BM / WGM) * (BN / WGN) / 64, WGM * WGN * KW))
void dstream_kernel(const DconvParams p)
{
    constexpr int NWG = WGM * WGN;                         // waves per K group
    constexpr int WTM = BM / WGM, WTN = BN / WGN;
    constexpr int TM = WTM / 32, TN = WTN / 32;
    constexpr int NKC = BK / 16;
    constexpr int CPR = BK / 8;                            // 16-byte chunks per tile row of a stage
    constexpr int RP = 256 / (BK * 2);                     // tile rows per 256 bytes of LDS
    constexpr int A_STAGE = BM * BK * 2, B_STAGE = BN * BK * 2;     // bytes: [rows][CPR chunks of 16 B]
    constexpr int STAGE = A_STAGE + B_STAGE;
    constexpr int RING = NS * STAGE;
    constexpr int NLA = A_STAGE / 1024 / NWG, NLB = B_STAGE / 1024 / NWG;   // wave-loads per wave per stage
    constexpr int LPS = NLA + NLB;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && TM >= 1 && TN >= 1, "wave tile");
    static_assert(A_STAGE % (1024 * NWG) == 0 && B_STAGE % (1024 * NWG) == 0 && NLA >= 1 && NLB >= 1,
                  "a stage is a whole number of wave-loads per wave");
    static_assert(BK == 64 || BK == 32, "K step");
    static_assert(NS >= 3 && (NS - 1) * LPS < 60, "pipeline depth against the vmcnt range");
    static_assert((NS * NKC) % 4 == 0, "a round over the stages is a whole number of fragment-buffer cycles");
    constexpr int RB = BT ? 2 : 1;                         // LDS reads per B fragment
    static_assert(TM + RB * TN <= 15, "fragment reads in flight against the lgkmcnt range");
    // BT: 16-byte chunks per stage row, and the XOR (in chunks, a function of k % 4) that spreads the four rows
    // a transpose read touches over the banks: rows of 64 columns are 128 bytes, so rows two apart collide
    // unless one of them swaps its halves; rows of 128 columns and more all start at bank 0 and rotate by
    // 64 bytes per row; rows of 32 columns are 64 bytes and four of them cover the banks as they are
    constexpr int CPRB = BN / 8;
    auto swz_b = [](int k) { return BN >= 128 ? (k & 3) * 4 : BN == 64 ? ((k >> 1) & 1) * 4 : 0; };

    extern __shared__ uint4 smem_u4[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem_u4;

    const int t = threadIdx.x, lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int kg = wave / NWG, wq = wave % NWG;
    const int wm = wq / WGN, wn = wq % WGN;

    // workgroup -> (m tile, n tile, channel slice), as in the direct convolution
    int mt, nt, split;
    {
        const int ntot = p.tiles_m * p.tiles_n * p.splitk;
        const int logical = igemm_logical_tile(ntot);
        const int rest = (int)div32((uint32_t)logical, p.d_tm);
        mt = logical - rest * p.tiles_m;
        split = (int)div32((uint32_t)rest, p.d_tn);
        nt = rest - split * p.tiles_n;
    }
    const int m0 = mt * BM, n0 = nt * BN;
    const int bz = blockIdx.y;                             // batch entry

    const i32x4_t x_rsrc = make_rsrc((const char *)p.x + (int64_t)bz * p.x_bstride, p.x_bytes);
    const i32x4_t w_rsrc = make_rsrc((const char *)p.w + (int64_t)bz * p.w_bstride, p.w_bytes);

    // ---- loads: slot s = (i*NWG + wq)*64 + lane of an operand's stage holds chunk (s % CPR) ^ swz(row) of
    // row s / CPR (rows that share LDS banks, RP apart, get different chunk orders)
    const int nk = p.ncc;                                  // K steps of a group
    const uint32_t k_off0 = (uint32_t)(split * p.Cs + kg * (nk * BK)) * 2u;
    uint32_t a_voff[NLA], b_voff[NLB];
#pragma unroll
    for (int i = 0; i < NLA; ++i) {
        const int s = (i * NWG + wq) * 64 + lane;
        const int row = s / CPR, c = (s % CPR) ^ ((row / RP) & (CPR - 1));
        const int m = m0 + row;
        // (blocked activations: a K step is BK / block whole blocks, so the chunk's place inside the step and the
        // step's distance are both fixed)
        a_voff[i] = m < p.M ? dconv_in_elem(p, m, split * p.Cs + kg * (nk * BK) + c * 8) * 2u : kOutOfRange;
    }
#pragma unroll
    for (int i = 0; i < NLB; ++i) {
        const int s = (i * NWG + wq) * 64 + lane;
        if constexpr (BT) {
            // slot s of the stage: row k = s / CPRB, chunk position s % CPRB, which holds chunk position ^ swz(k)
            const int k = s / CPRB, c = (s % CPRB) ^ swz_b(k);
            const int n = n0 + c * 8;
            b_voff[i] = n < p.Nc ? (uint32_t)((split * p.Cs + kg * (nk * BK) + k) * p.Nc + n) * 2u : kOutOfRange;
        } else {
            const int row = s / CPR, c = (s % CPR) ^ ((row / RP) & (CPR - 1));
            const int n = n0 + row;
            b_voff[i] = n < p.Nc ? (uint32_t)(n * p.C) * 2u + k_off0 + (uint32_t)c * 16u : kOutOfRange;
        }
    }
    // byte distance between consecutive K steps of B: BK columns of a row, or BK rows; of A: BK channels of a
    // pixel, or BK / block channel blocks (planes of H*W pixels)
    const uint32_t b_step = BT ? (uint32_t)(BK * p.Nc) * 2u : (uint32_t)(BK * 2);
    const uint32_t a_step = p.x_blk ? (uint32_t)(BK * p.H * p.W) * 2u : (uint32_t)(BK * 2);
    const uint32_t ring0 = lds0 + kg * RING;
    const uint32_t ldsW = ring0 + wq * 1024;
    // load cursor: K step `lstep` goes to stage `lstage`; past the last step the last one is
    // loaded again (into stages nobody reads any more), which keeps the load count per step fixed
    int lstep = 0, lstage = 0;
    auto issue_stage = [&]() {
        const uint32_t soff = (uint32_t)min(lstep, nk - 1) * a_step, soff_b = (uint32_t)min(lstep, nk - 1) * b_step;
        const uint32_t dst = ldsW + lstage * STAGE;
#pragma unroll
        for (int i = 0; i < NLA; ++i) dma_load16_s(x_rsrc, a_voff[i], soff, dst + i * (NWG * 1024));
#pragma unroll
        for (int i = 0; i < NLB; ++i) dma_load16_s(w_rsrc, b_voff[i], soff_b, dst + A_STAGE + i * (NWG * 1024));
        ++lstep;
        lstage = lstage + 1 == NS ? 0 : lstage + 1;
    };
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue_stage();

    // ---- operand addresses of this lane in stage 0: row (lane % 32) of each 32-row MFMA tile, k half (lane / 32)
    uint32_t a_rd[TM][NKC], b_rd[TN][NKC];
    {
        const uint32_t khalf = (lane >> 5) * 16;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int r = wm * WTM + i * 32 + (lane & 31);
            const uint32_t swz = ((r / RP) & (CPR - 1)) * 16;
#pragma unroll
            for (int kc = 0; kc < NKC; ++kc) a_rd[i][kc] = ring0 + r * (BK * 2) + ((kc * 32 + khalf) ^ swz);
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            if constexpr (BT) {
                // lane l: group l / 16 = (k half, 16-column block), inside it row (l % 16) / 4 and four columns
                const int grp = lane >> 4, j4 = (lane & 15) >> 2, c4 = lane & 3;
                const int col = wn * WTN + j * 32 + (grp & 1) * 16 + c4 * 4;
                const uint32_t base = ring0 + A_STAGE + ((grp >> 1) * 8 + j4) * (BN * 2) + (((col >> 3) ^ swz_b(j4)) * 16) + (col & 7) * 2;
#pragma unroll
                for (int kc = 0; kc < NKC; ++kc) b_rd[j][kc] = base + kc * 16 * (BN * 2);
            } else {
                const int r = wn * WTN + j * 32 + (lane & 31);
                const uint32_t swz = ((r / RP) & (CPR - 1)) * 16;
#pragma unroll
                for (int kc = 0; kc < NKC; ++kc) b_rd[j][kc] = ring0 + A_STAGE + r * (BK * 2) + ((kc * 32 + khalf) ^ swz);
            }
        }
    }

    floatx16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // Operand reads run D k-chunks ahead of the MFMAs that use them; k chunk g (counted
    // from the start of a round over the stages) uses register buffer g % NBUF.
    // (wave tiles of eight or more MFMAs per k chunk run a hand-pinned schedule, one chunk ahead: see do_step)
    constexpr bool kPinned = KW == 1 && TM * TN >= 8 && TM >= 2 && LPS <= NKC * TM;
    constexpr int D0 = kPinned ? 1 : (TM + RB * TN) * 3 <= 15 ? 3 : (TM + RB * TN) * 2 <= 15 ? 2 : 1;
    constexpr int D = D0 < NKC ? D0 : NKC;                 // the look-ahead stays within the next step
    constexpr int NBUF = 4;
    static_assert(D < NBUF && NBUF % NKC == 0, "fragment buffers");
    u32x4_t af[NBUF][TM], bf[NBUF][TN];
    u32x2_t bh[NBUF][BT ? TN : 1][2];                      // BT: the two 8-byte halves of a B fragment as they are read
    auto read_b = [&](auto BUF, auto J, auto OFF, uint32_t addr) {
        constexpr int buf = decltype(BUF)::value, j = decltype(J)::value, off = decltype(OFF)::value;
        if constexpr (BT) {
            lds_read8_tr_async_at<off>(bh[buf][j][0], addr);
            lds_read8_tr_async_at<off + 4 * (BN * 2)>(bh[buf][j][1], addr);
        } else {
            lds_read16_async_at<off>(bf[buf][j], addr);
        }
    };
    // waits until at most N chunks' worth of reads are outstanding, ties the fragments of buffer `buf` to that
    // point and (BT) joins the halves of its B fragments
    auto frag_wait = [&](auto NCH, auto BUF) {
        constexpr int n = decltype(NCH)::value, buf = decltype(BUF)::value;
        if constexpr (BT) {
            lds_wait_tr<n * (TM + RB * TN)>(af[buf], bh[buf]);
#pragma unroll
            for (int j = 0; j < TN; ++j) bf[buf][j] = (u32x4_t){bh[buf][j][0].x, bh[buf][j][0].y, bh[buf][j][1].x, bh[buf][j][1].y};
        } else {
            lds_wait<n * (TM + TN)>(af[buf], bf[buf]);
        }
    };
    // reads of k chunk G of a round (G / NKC = stage, wrapping into the next round's first stage)
    auto reads = [&](auto GI) {
        constexpr int g = decltype(GI)::value;
        constexpr int st = (g / NKC) % NS, kc = g % NKC, buf = g % NBUF, off = st * STAGE;
#pragma unroll
        for (int i = 0; i < TM; ++i) lds_read16_async_at<off>(af[buf][i], a_rd[i][kc]);
        static_for<TN>([&](auto JC) {
            read_b(std::integral_constant<int, buf>{}, JC, std::integral_constant<int, off>{}, b_rd[decltype(JC)::value][kc]);
        });
    };

    wait_vmcnt<(NS - 2) * LPS>();                          // stage 0 (this wave's share)
    lds_barrier();
    // (D = 1 for the wave tiles with a pinned schedule.  BT: the compiler copies fragment registers at
    // control-flow joins, and a copy of a register whose read is still in flight copies stale data: the NK
    // kernels' register assignment happens to need no such copies, the BT kernels' does.  So with BT no read is
    // in flight across a branch: every whole round, and every step of the last, partial round, issues its own
    // first D chunks, looks ahead only inside itself and ends with every read consumed.)
    if constexpr (!BT) static_for<D>(reads);

    // One K step in stage st.  At its barrier every wave has its share of the next stage
    // landed, so both are complete for everybody afterwards and the look-ahead may run into
    // the next stage; the barrier also says the previous stage is consumed, and its refill
    // is issued right after it.  Past the last step the look-ahead reads whatever the
    // repeated loads left in the next stage (never used).
    //
    // Large wave tiles (kPinned: at least eight MFMAs per k chunk, one wave per SIMD) fix the
    // instruction order by hand: with nobody else on the SIMD to fill a gap, whatever stands
    // between two MFMAs and does not fit the first one's shadow is lost.  After each row of
    // TN MFMAs come a few of the next chunk's operand reads (all of them within the first
    // TM - 1 rows, so that the last row's MFMAs cover their latency) and one of the step's
    // direct-to-LDS loads; scheduling barriers keep the compiler from regrouping them.
    auto issue_one = [&](int i) {                          // load i of the stage the cursor is on
        const uint32_t soff = (uint32_t)min(lstep, nk - 1) * a_step, soff_b = (uint32_t)min(lstep, nk - 1) * b_step;
        const uint32_t dst = ldsW + lstage * STAGE;
        if (i < NLA) dma_load16_s(x_rsrc, a_voff[i], soff, dst + i * (NWG * 1024));
        else dma_load16_s(w_rsrc, b_voff[i - NLA], soff_b, dst + A_STAGE + (i - NLA) * (NWG * 1024));
    };
    // GEND: the look-ahead reads k chunks below GEND only (0: no limit, the NK kernels); FIRST: this step
    // issues its own first D chunks
    auto do_step_lim = [&](auto ST, auto GEND_, auto FIRST_) {
        constexpr int st = decltype(ST)::value, GEND = decltype(GEND_)::value;
        constexpr bool FIRST = decltype(FIRST_)::value;
        wait_vmcnt<(NS - 3) * LPS>();
        if constexpr (NWG > 1) asm volatile("s_barrier" ::: "memory");
        if constexpr (!kPinned) {
            issue_stage();
            if constexpr (FIRST)
                static_for<D>([&](auto GI) { reads(std::integral_constant<int, st * NKC + decltype(GI)::value>{}); });
            static_for<NKC>([&](auto KC) {
                constexpr int g = st * NKC + decltype(KC)::value, buf = g % NBUF;
                constexpr bool look = GEND == 0 || g + D < GEND;
                constexpr int ahead = look ? D : GEND - 1 - g;                  // chunks read after this one and still in flight
                if constexpr (look) reads(std::integral_constant<int, g + D>{});
                frag_wait(std::integral_constant<int, ahead>{}, std::integral_constant<int, buf>{});
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, bf[buf][j]),
                                                                            __builtin_bit_cast(bf16x8_t, af[buf][i]),
                                                                            acc[i][j], 0, 0, 0);
            });
        } else {
            static_for<NKC>([&](auto KC) {
                constexpr int kc = decltype(KC)::value, g = st * NKC + kc, buf = g % NBUF;
                // the chunk this one's rows read ahead for: D = 1 here (TM + TN reads fill the counter's range)
                constexpr int gn = g + 1, stn = (gn / NKC) % NS, kcn = gn % NKC, bufn = gn % NBUF, offn = stn * STAGE;
                constexpr int RPS = (TM + TN + TM - 2) / (TM - 1);             // reads per row slot, rows 0 .. TM - 2
                constexpr bool look = GEND == 0 || gn < GEND;
                if constexpr (FIRST && kc == 0) reads(std::integral_constant<int, g>{});
                frag_wait(std::integral_constant<int, 0>{}, std::integral_constant<int, buf>{});
                static_for<TM>([&](auto IR) {
                    constexpr int i = decltype(IR)::value;
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, bf[buf][j]),
                                                                            __builtin_bit_cast(bf16x8_t, af[buf][i]),
                                                                            acc[i][j], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                    static_for<RPS>([&](auto RR) {
                        constexpr int r = i * RPS + decltype(RR)::value;
                        if constexpr (!look) {
                        } else if constexpr (r < TM) lds_read16_async_at<offn>(af[bufn][r], a_rd[r][kcn]);
                        else if constexpr (r < TM + TN)
                            read_b(std::integral_constant<int, bufn>{}, std::integral_constant<int, r - TM>{},
                                   std::integral_constant<int, offn>{}, b_rd[r - TM][kcn]);
                    });
                    if constexpr (kc * TM + i < LPS) issue_one(kc * TM + i);
                    __builtin_amdgcn_sched_barrier(0);
                });
            });
            ++lstep;
            lstage = lstage + 1 == NS ? 0 : lstage + 1;
        }
    };
    int ks0 = 0;
    if constexpr (BT) {
        for (; ks0 + NS <= nk; ks0 += NS)                  // whole rounds: look-ahead inside the round
            static_for<NS>([&](auto ST) {
                do_step_lim(ST, std::integral_constant<int, NS * NKC>{}, std::integral_constant<bool, decltype(ST)::value == 0>{});
            });
        static_for<NS - 1>([&](auto ST) {                  // the last, partial round: look-ahead inside a step
            if (ks0 + decltype(ST)::value < nk)
                do_step_lim(ST, std::integral_constant<int, (decltype(ST)::value + 1) * NKC>{}, std::true_type{});
        });
    } else {
        auto do_step = [&](auto ST) { do_step_lim(ST, std::integral_constant<int, 0>{}, std::false_type{}); };
        for (; ks0 + NS <= nk; ks0 += NS)                  // whole rounds over the stages, no exit inside
            static_for<NS>(do_step);
        static_for<NS - 1>([&](auto ST) {                  // the last, partial round
            if (ks0 + decltype(ST)::value < nk) do_step(ST);
        });
    }

    wait_vmcnt<0>();                                       // the repeated loads past the last step
    // the look-ahead reads past the last step still land in their registers: tie them to a wait
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int kc = 0; kc < NBUF; ++kc) {
#pragma unroll
        for (int i = 0; i < TM; ++i) asm volatile("" : "+v"(af[kc][i]));
#pragma unroll
        for (int j = 0; j < TN; ++j) asm volatile("" : "+v"(bf[kc][j]));
        if constexpr (BT) {
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                asm volatile("" : "+v"(bh[kc][j][0]));
                asm volatile("" : "+v"(bh[kc][j][1]));
            }
        }
    }

    if constexpr (kBandedEpilogue<BM, BN, WGN, KW>) {
        static_assert(KW == 1, "banded epilogue: one K group");
        dconv_epilogue_banded<BM, BN, WGM, WGN>(p, acc, smem_u4, lane, wave, wm, wn, m0, n0,
                                                (char *)p.y + (int64_t)bz * p.y_bstride);
    } else {
        dconv_epilogue<BM, BN, WGM, WGN, KW>(p, acc, smem_u4, t, lane, wave, kg, wq, wm, wn, m0, n0, mt, nt, split,
                                             (char *)p.y + (int64_t)bz * p.y_bstride);
    }
}

// LDS bytes of one workgroup: the K groups' operand rings, or the output staging.
// (kernels whose whole-tile staging exceeds LDS stage 32 rows per wave at a time: see kBandedEpilogue)
inline bool dstream_banded(int BM, int BN, int waves_n, int kw)
{
    return (size_t)kw * BM * (BN + 8 * waves_n) * 4 + 16 > 160 * 1024;
}

inline size_t dstream_lds_bytes(int BM, int BN, int bk, int NS, int waves_m, int waves_n, int kw)
{
    const size_t main_loop = (size_t)kw * NS * (BM + BN) * bk * 2;
    const size_t staging = dstream_banded(BM, BN, waves_n, kw)
        ? (size_t)waves_m * waves_n * 32 * (BN / waves_n + 4) * 4
        : (size_t)kw * BM * (BN + 8 * waves_n) * 4 + 16;
    return main_loop > staging ? main_loop : staging;
}

template <int BM, int BN, int WGM, int WGN, int KW, int NS, int BK, bool BT = false>
hipError_t dstream_launch(const DconvParams &p, size_t lds, hipStream_t st)
{
    if (p.bk != BK) return hipErrorInvalidValue;
    auto kern = dstream_kernel<BM, BN, WGM, WGN, KW, NS, BK, BT>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int tiles = p.tiles_m * p.tiles_n;
    const unsigned grid = (unsigned)(tiles * p.splitk);
    hipLaunchKernelGGL(kern, dim3(grid, (unsigned)p.batch), dim3(64 * WGM * WGN * KW), lds, st, p);
    return hipGetLastError();
}

}  // namespace alt
