// Direct-to-LDS ABFT-protected MFMA GEMM kernel for gfx950 (MI355X): the main path for
// 16-byte aligned operands.
//
// Workgroup tile (32 TM WAVES_M) x (32 TN WAVES_N) x (128 bytes of k); each wavefront owns a
// (32 TM) x (32 TN) register tile of MFMA 32x32 blocks.  The flagship instance is 256 x 256
// with eight wavefronts of 128 x 64, two per SIMD (128 accumulators per lane); smaller
// instances with wide-in-N wavefront tiles serve mid-size layers.  In the global scheme the
// kernel also forms the checksum dot product of its tile, from the A tiles it loads and the
// weight checksums of its column block, which travel with the operand tiles: on the matrix
// unit (fp16, int8), with vector FMAs on the A chunks in LDS (bf16, the 256 x 256 tile), or,
// when the layer before handed over the column sums of A, with one multiplication per lane
// and k tile.
//
// Data flow: global_load_lds_dwordx4 moves 16-byte chunks from HBM straight into LDS
// (no staging registers), NSTAGE LDS stages, rows of 128 bytes stored with an XOR
// swizzle of the chunk position (key (row >> 1) & 7) so that ds_read_b128 fragment reads are free of bank
// conflicts; out-of-range rows (and convolution padding taps) read from a small block
// of zeros, so ragged edges need no special case.  Requirements checked by the
// dispatcher: 16-byte aligned operands with k contiguous, leading dimensions multiples
// of 16 bytes, K a multiple of the k tile.
#pragma once
#include <type_traits>

#include "gemm_common.h"

namespace abft {

// zeros that stand in for rows beyond the matrix edge and for convolution padding
__device__ __attribute__((aligned(256))) static const char g_zero_chunk[256] = {0};

// Workgroup index -> output tile.  Workgroups are dealt round-robin to the 8 XCDs, each
// with its own L2; the remap hands every XCD a contiguous run of tiles and walks those in
// bands of 8 tile rows, so that the tiles resident on an XCD at one time share A row
// blocks and B column blocks in its L2.
__device__ __forceinline__ void tile_of_block(int bid, int tiles_m, int tiles_n, int& tm, int& tn) {
    const int total = tiles_m * tiles_n;
    int lin = bid;
    if ((total & 7) == 0) lin = (bid & 7) * (total >> 3) + (bid >> 3);
    constexpr int GM = 8;
    const int per_group = GM * tiles_n;
    const int group = lin / per_group;
    const int first_m = group * GM;
    const int gsz = min(tiles_m - first_m, GM);
    const int in_group = lin - group * per_group;
    tn = in_group / gsz;
    tm = first_m + (in_group - tn * gsz);
}

// vmcnt(n) with expcnt / lgkmcnt left open (gfx9 encoding: vmcnt in bits 3:0 and 15:14)
constexpr int waitcnt_vm(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0F70; }

template <class CFG, int NSTAGE>
struct FastLayout {
    static constexpr int ROWB = 128;                            // bytes per LDS row
    static constexpr int WAVES = CFG::WAVES_M * CFG::WAVES_N;
    static constexpr int A_STAGE = CFG::BM * ROWB;
    static constexpr int AB_STAGE = (CFG::BM + CFG::BN) * ROWB;
    // global scheme: behind the operand tiles of a stage, the k tile's record of weight checksums of
    // the workgroup's column block (1 KB, copied by wavefront 0 like one more group of eight rows of B)
    static constexpr int BETA_REC = 1024;
    static constexpr int STAGE = AB_STAGE + BETA_REC;
    // global scheme: 512 bytes behind everything else for the cross-wavefront sums of the epilogue
    // (never aliased with a stage, so that the epilogue waits for no other wavefront)
    static constexpr int EPI_BYTES = 512;
    static constexpr int LDS_BYTES = NSTAGE * STAGE + EPI_BYTES;
    // Activation checksums handed over by the layer before travel in runs of 256 floats, four k
    // tiles at a time, through a ring of two 1 KB slots per wavefront (its 32-row block's sums) behind the stages
    // and, with them, 256 floats of the column block's weight checksums through one such ring for the
    // workgroup (a quarter of the copies that a record per k tile would take)
    static constexpr int RING_A = NSTAGE * STAGE, RING_B = RING_A + WAVES * 2048;
    static constexpr int LDS_BYTES_FED = RING_B + 2048 + EPI_BYTES;
    static constexpr int NQA = CFG::BM / (8 * WAVES);           // 1 KB copies per wave per k tile
    static constexpr int NQB = CFG::BN / (8 * WAVES);
    static_assert(CFG::BM % (8 * WAVES) == 0 && CFG::BN % (8 * WAVES) == 0, "tile rows vs waves");
    static_assert((CFG::MI == 32 || CFG::MI == 16) && CFG::BKB == 128, "32x32 or 16x16 MFMA shapes, 128-byte k tile");
    static_assert((NSTAGE - 2) * (NQA + NQB) <= 63, "vmcnt range");
};

template <class CFG, int NSTAGE, int MODE, bool INJ, bool CONV>
__global__ __launch_bounds__(CFG::THREADS) void gemm_fast_kernel(const GemmArgs p) {
    typedef FastLayout<CFG, NSTAGE> LAY;
    constexpr int DT = CFG::DT;
    constexpr int MI = CFG::MI;
    typedef Mma<DT, MI> MMA;
    typedef typename MMA::Acc Acc;
    constexpr int TM = CFG::TM, TN = CFG::TN, BM = CFG::BM, BN = CFG::BN, BKB = 128;
    constexpr int ESIZE = CFG::ESIZE, BK = CFG::BK;
    constexpr int ROWB = LAY::ROWB, A_STAGE = LAY::A_STAGE, STAGE = LAY::STAGE;
    constexpr int WAVES = LAY::WAVES, NQA = LAY::NQA, NQB = LAY::NQB;
    constexpr int NQ = NQA > NQB ? NQA : NQB;
    constexpr bool GDOT = MODE == MODE_GLOBAL;  // in-kernel checksum dot product
    // ... formed on the matrix unit (fp16, int8: the weight checksums, cut into two pieces that the
    // operand type holds, are two more columns of B) or with vector FMAs (bf16, which wants three
    // pieces; the 256 x 256 tile, which has no registers left for one more accumulator block)
    constexpr bool MDOT = GDOT && DT != DT_BF16 && CFG::MI == 32 && TM * TN <= 4;
    // (16x16 shapes, int8: the same with the block rows of A split over a row of wavefronts and only the
    // first two columns of the extra block of B in use)
    // int8 only: on all-positive fp16 / bf16 operands and short k loops its fp32 sums of whole block
    // rows times the (large) weight checksums came to 0.6-1.0 of the comparison's tolerance, against
    // 0.1-0.2 for the vector form, which leaves fp32 after eight products
    constexpr bool MDOT16 = GDOT && CFG::MI == 16 && DT == DT_I8;
    constexpr bool VDOT = GDOT && !MDOT && !MDOT16;
    static_assert(!MDOT || TM == CFG::WAVES_N, "one block row of the extra product per wavefront of a row of wavefronts");
    static_assert(!MDOT16 || TM % CFG::WAVES_N == 0, "the block rows of the extra product split evenly over a row of wavefronts");
    // ... or reduced to one multiplication per lane and k tile because the layer before left the
    // column sums of this layer's A (per block of 32 rows: one block per wavefront here)
    constexpr bool FED = MODE == MODE_GLOBAL_FED;
    // (one 32-row block per wavefront, or per row of wavefronts whose first one then takes it)
    constexpr bool FED_PER_ROW = CFG::WAVES_M * CFG::WAVES_N * 32 != BM;
    static_assert(!FED || (DT != DT_I8 && (!FED_PER_ROW || CFG::WM == 32)), "a 32-row block per wavefront or per row of wavefronts");
    constexpr int EMODE = (MODE == MODE_GLOBAL_PRE || FED) ? MODE_GLOBAL : MODE;  // the epilogue's scheme
    constexpr bool IS_INT = DT == DT_I8;

    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave / CFG::WAVES_N, wave_n = wave % CFG::WAVES_N;

    int tile_m, tile_n;
    tile_of_block((int)blockIdx.x, p.tiles_m, p.tiles_n, tile_m, tile_n);
    const int bm0 = tile_m * BM, bn0 = tile_n * BN;
    const int M = p.M, N = p.N;
    const int nkt = p.K / BK;
    // scratch of the global scheme's epilogue: behind the stages this launch asked for (a k loop
    // shorter than the pipeline gets no more) or behind the rings of the handed-over sums
    char* const epi = smem + (FED ? LAY::RING_B + 2048 : (nkt < NSTAGE ? (nkt < 1 ? 1 : nkt) : NSTAGE) * STAGE);
    if constexpr (EMODE == MODE_GLOBAL) {
        if (tid == 0) *reinterpret_cast<unsigned*>(epi + 256) = 0u;  // the ticket counter; the barrier after the prologue publishes it
    }

    // ---- global -> LDS copy: this lane always fills LDS slot `lane` of a 1 KB block
    // (8 rows x 8 chunks): row lane/8, position lane%8, which holds chunk (lane%8) ^ key(row)
    const int crow = lane >> 3;
    // swizzle key of a row: (row >> 1) & 7.  The LDS serves 16 lanes of a ds_read_b128 at a time
    // over 64 banks (256 bytes = two rows), so the 8 even and the 8 odd rows of any 16 rows
    // must each spread over the 8 chunk positions.  Every 1 KB block starts at a row that is a
    // multiple of 8, and the parity of that multiple is the parity of the wave index.
    const int ckc = (lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7);
    const char* zero = g_zero_chunk + ckc * 16;

    const char* aptr[NQA];
    const char* bptr[NQB];
    unsigned a_valid = 0, b_valid = 0;
    // convolution: image offset and top-left input pixel of each of this lane's rows
    long long a_img[CONV ? NQA : 1];
    int a_ih0[CONV ? NQA : 1], a_iw0[CONV ? NQA : 1];
    int tap_c = 0, tap_kh = 0, tap_kw = 0;
    (void)NQ;
#pragma unroll
    for (int q = 0; q < NQB; ++q) {
        const int n = bn0 + (q * WAVES + wave) * 8 + crow;
        if (n < N) b_valid |= 1u << q;
        bptr[q] = n < N ? p.B + (long long)n * p.ldb * ESIZE + ckc * 16 : zero;
    }
#pragma unroll
    for (int q = 0; q < NQA; ++q) {
        const int m = bm0 + (q * WAVES + wave) * 8 + crow;
        if (m < M) a_valid |= 1u << q;
        if constexpr (!CONV) {
            aptr[q] = m < M ? p.A + (long long)m * p.lda * ESIZE + ckc * 16 : zero;
        } else {
            const int mm = m < M ? m : 0;
            const int img = mm / (p.OH * p.OW);
            const int rem = mm - img * (p.OH * p.OW);
            const int oh = rem / p.OW, ow = rem - oh * p.OW;
            a_img[q] = (long long)img * p.imgpitch;
            a_ih0[q] = oh * p.stride - p.pad;
            a_iw0[q] = ow * p.stride - p.pad;
            aptr[q] = zero;
        }
    }
    // weight checksums of this tile's column block: one record of 1 KB per k tile (layout:
    // weight_checksum_kernel: fp16 halves hi / lo at bytes 0 / 128 and floats at 256; bf16 the floats;
    // int8 low / high digits at 0 / 128), copied by one wavefront, 16 bytes per lane
    constexpr bool BREC = GDOT;
    const char* beta_rec = zero;
    int rec_turn = 0;  // the wavefront that copies the next record
    if constexpr (BREC) beta_rec = p.beta_r + (long long)tile_n * nkt * 1024 + lane * 16;
    // Handed-over activation checksums.  Group g = k tiles 4 g .. 4 g + 3 = floats 256 g .. 256 g + 255 of
    // this wavefront's row of sums (lane l copies floats 4 l .. 4 l + 3 of the group) and, by wavefront 0
    // for everyone, of the column block's weight checksums; group g sits in
    // slot g % 2 and is copied while group g - 1 is in use.  These copies are older than the operand
    // copies any later wait counts on, so every such wait covers them too.
    const char* fed_alpha = nullptr;
    const char* fed_beta = nullptr;
    // (a row of wavefronts per block: one of them takes it, chosen so that the takers sit on different
    // SIMDs -- wavefront w runs on SIMD w % 4 --, wavefront 0, which copies the weight checksums, among them)
    const bool fed_on = !FED_PER_ROW || wave_n == ((wave_m >> 1) % CFG::WAVES_N);
    if constexpr (FED) {
        const int blk = tile_m * (BM / 32) + (FED_PER_ROW ? wave_m : wave);
        if (blk * 32 < M && fed_on) fed_alpha = reinterpret_cast<const char*>(p.alpha_in + (long long)blk * p.K);
        fed_beta = p.beta_k + (long long)tile_n * p.K * 4;
    }
    auto issue_group = [&](int g) {
        if constexpr (FED) {
            if (!fed_on) return;
            const int f0 = 256 * g + 4 * lane;                 // first of this lane's four floats
            const bool in_k = f0 + 4 <= p.K;                   // (K is a multiple of 64: whole lanes)
            const char* src = (fed_alpha && in_k) ? fed_alpha + (long long)f0 * 4 : zero;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(smem + LAY::RING_A + (wave * 2 + (g & 1)) * 1024),
                                             16, 0, 0);
            if (wave == 0) {
                const char* srcb = in_k ? fed_beta + (long long)f0 * 4 : zero;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)srcb,
                                                 (__attribute__((address_space(3))) void*)(smem + LAY::RING_B + (g & 1) * 1024),
                                                 16, 0, 0);
            }
        }
    };
    if constexpr (CONV) {
        const int k = ckc * (16 / ESIZE);
        const int tap = k / p.Cin;
        tap_c = k - tap * p.Cin;
        tap_kh = tap / p.KW;
        tap_kw = tap - tap_kh * p.KW;
    }

    auto issue_loads = [&](int stage) {
        char* abase = smem + stage * STAGE + wave * 1024;
        char* bbase = abase + A_STAGE;
#pragma unroll
        for (int q = 0; q < NQA; ++q) {
            const char* src = aptr[q];
            if constexpr (CONV) {
                // a chunk never straddles a filter tap (Cin is a multiple of the chunk length)
                const int ih = a_ih0[q] + tap_kh, iw = a_iw0[q] + tap_kw;
                const bool ok = ((a_valid >> q) & 1u) && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
                src = ok ? p.A + (a_img[q] + (long long)ih * p.rowpitch + (long long)iw * p.pix + tap_c) * ESIZE : zero;
            }
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(abase + q * WAVES * 1024), 16, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < NQB; ++q)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)bptr[q],
                                             (__attribute__((address_space(3))) void*)(bbase + q * WAVES * 1024), 16, 0, 0);
        if constexpr (BREC) {
            // (the wavefronts take turns, so that none carries the extra copy every tile)
            if (rec_turn == wave)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)beta_rec,
                                                 (__attribute__((address_space(3))) void*)(smem + stage * STAGE + LAY::AB_STAGE), 16, 0, 0);
            rec_turn = rec_turn + 1 == WAVES ? 0 : rec_turn + 1;
        }
    };
    auto advance = [&]() {
        if constexpr (BREC) beta_rec += 1024;
        if constexpr (!CONV) {
#pragma unroll
            for (int q = 0; q < NQA; ++q) aptr[q] += ((a_valid >> q) & 1u) ? BKB : 0;
        }
#pragma unroll
        for (int q = 0; q < NQB; ++q) bptr[q] += ((b_valid >> q) & 1u) ? BKB : 0;
        if constexpr (CONV) {
            tap_c += BK;
            while (tap_c >= p.Cin) {
                tap_c -= p.Cin;
                if (++tap_kw == p.KW) {
                    tap_kw = 0;
                    ++tap_kh;
                }
            }
        }
    };

    Acc acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < MMA::NACC; ++r) acc[i][j][r] = 0;
    constexpr int NCHK = CheckRegs<CFG, MODE>::N;
    Acc chk[NCHK];
#pragma unroll
    for (int i = 0; i < NCHK; ++i)
#pragma unroll
        for (int r = 0; r < MMA::NACC; ++r) chk[i][r] = 0;

    // ---- fragment reads: lane l reads row l%32 of a 32-row block, k chunk 2*kk + l/32,
    // stored at position chunk ^ ((row >> 1) & 7), which is (l >> 1) & 7 for every block
    // (16x16 shapes: row l%16 of a 16-row block, k chunk 4*step + l/16 of the two 64-byte k steps;
    // the key of a row is still (l >> 1) & 7: blocks start at multiples of 16 rows)
    const int frow = lane & (MI - 1), fgrp = lane / MI, fx = (lane >> 1) & 7;
    const int a_off = (wave_m * CFG::WM + frow) * ROWB;
    const int b_off = A_STAGE + (wave_n * CFG::WN + frow) * ROWB;
    int pos[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) pos[kk] = MI == 32 ? ((2 * kk + fgrp) ^ fx) * 16 : ((4 * (kk & 1) + fgrp) ^ fx) * 16;

    // fragments of one k step: double buffered so that the reads of step kk+1 run under
    // the MFMAs of step kk
    // Global scheme, in-kernel checksum dot product (Sec. 2.4 steps 1-3 fused into the loop):
    // sum over the tile's rows m and all k of A[m][k] * beta_j[k].  Every lane re-reads from LDS
    // the NQA chunks of the A tile that it copied itself (row-major slots, free of bank
    // conflicts; together the lanes cover the tile exactly once) and multiplies them with the
    // 8 (16 for int8) weight checksums of its k chunk, with vector FMAs / dot4 that run beside
    // the MFMAs.  Per k tile the fp32 / int32 partial sums move into a wide accumulator.
    const int beta_off = LAY::AB_STAGE + (IS_INT ? ckc * 16 : 256 + ckc * 32);  // this lane's k chunk in the record
    ChecksumDot<DT> dot;
    float fed_a = 0.f, fed_b = 0.f;
    auto fed_tile = [&](const char* st, int kt) {
        if constexpr (FED) {
            if (!fed_on) return;
            // lane l: (column sum of the wavefront's 32 rows at k = l of the tile) x (weight checksum
            // there); the product is taken one tile later, when the two reads have long landed
            dot.total += (double)fed_a * (double)fed_b;
            const int off = ((kt >> 2) & 1) * 1024 + ((kt & 3) * 64 + lane) * 4;
            fed_a = *reinterpret_cast<const float*>(smem + LAY::RING_A + wave * 2048 + off);
            fed_b = *reinterpret_cast<const float*>(smem + LAY::RING_B + off);
            // the slot of the group before is free (everyone read its last tile before the barrier
            // of that tile): the next group goes there
            if ((kt & 3) == 0 && kt >= 4 && 4 * ((kt >> 2) + 1) < nkt) issue_group((kt >> 2) + 1);
        }
    };
    auto dot_tile = [&](const char* st) {
        if constexpr (VDOT) {
            const i32x4 b0 = *reinterpret_cast<const i32x4*>(st + beta_off);
            const i32x4 b1 = *reinterpret_cast<const i32x4*>(st + beta_off + (IS_INT ? 128 : 16));
#pragma unroll
            for (int q = 0; q < NQA; ++q)
                dot.chunk(*reinterpret_cast<const i32x4*>(st + (q * WAVES + wave) * 1024 + lane * 16), b0, b1, q);
            dot.flush();
        }
    };
    // Matrix-unit form of that dot product: one more 32-column block of B whose columns hold the
    // pieces of the weight checksums, multiplied with ONE of the TM blocks of A per wavefront
    // (wavefront column c of a row of wavefronts takes block row c): one more MFMA per k step and
    // wavefront.  To read the slot once per k tile instead of once per k step, lane (column g,
    // half h) keeps the 16 bytes of piece g % 2, k chunk 2 (g / 2) + h of the tile, and at k step kk
    // only the columns with g / 2 == kk pass them on (the others pass zeros): column 2 kk + s of the
    // result block then holds A . piece s restricted to the k of step kk, and the columns of equal
    // parity add up to A . piece s.  Four selects per k step, no other vector arithmetic.
    const int gcol = lane & 31;
    const int g_step = gcol >> 1;  // the k step whose chunk this lane holds (>= 4: none)
    const int gb_off = LAY::AB_STAGE + (gcol & 1) * 128 + (g_step & 3) * 32 + fgrp * 16;
    i32x4 g_tile = {0, 0, 0, 0};
    auto read_checksum_frag = [&](const char* st) {
        if constexpr (MDOT) g_tile = *reinterpret_cast<const i32x4*>(st + gb_off);
    };
    auto checksum_frag = [&](int kk) {
        const i32x4 z = {0, 0, 0, 0};
        return g_step == kk ? g_tile : z;
    };
    Acc gchk;
#pragma unroll
    for (int r = 0; r < MMA::NACC; ++r) gchk[r] = 0;
    i32x4 fa[2][TM], fb[2][TN];
    auto read_frags = [&](const char* st, int kk, int buf) {
        const int ps = pos[kk];

#pragma unroll
        for (int i = 0; i < TM; ++i)
            fa[buf][i] = *reinterpret_cast<const i32x4*>(st + a_off + i * MI * ROWB + ps);
#pragma unroll
        for (int j = 0; j < TN; ++j)
            fb[buf][j] = *reinterpret_cast<const i32x4*>(st + b_off + j * MI * ROWB + ps);
    };
    auto mma_step = [&](int buf, const i32x4& fg) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = MMA::run(fa[buf][i], fb[buf][j], acc[i][j]);
        if constexpr (MDOT) {
            // (the wavefront's block row: a selection by a wavefront-uniform index)
            i32x4 a_sel = fa[buf][0];
#pragma unroll
            for (int i = 1; i < TM; ++i) a_sel = wave_n == i ? fa[buf][i] : a_sel;
            gchk = MMA::run(a_sel, fg, gchk);
        }
        if constexpr (mode_is_wave_level(MODE)) check_step<CFG, MODE>(fa[buf], fb[buf], chk);
    };

    // Pipeline: tile t lives in LDS stage t % NSTAGE and is copied in while earlier tiles are
    // being multiplied.  The workgroup barrier sits before the last k step of each tile,
    // whose fragments are already in registers, so the barrier wait, the issue of the next
    // copies and the first fragment reads of the next tile all run under those MFMAs.
    // copies per wave per tile (the one more of the wavefront whose turn it is to copy the record makes
    // its waits at most one copy stricter than needed)
    constexpr int NL = NQA + NQB;
    if constexpr (FED) {
        issue_group(0);
        if (nkt > 4) issue_group(1);
    }
#pragma unroll
    for (int t = 0; t < NSTAGE; ++t) {
        if (t < nkt) {
            if (t > 0) advance();
            issue_loads(t);
        }
    }
    if (nkt >= NSTAGE) __builtin_amdgcn_s_waitcnt(waitcnt_vm((NSTAGE - 1) * NL));  // tile 0 has landed
    else __builtin_amdgcn_s_waitcnt(waitcnt_vm(0));
    __syncthreads();
    int stage = 0;
    // one k tile; CUR is the fragment buffer that holds the step multiplied after the barrier
    // (a compile-time constant, so that the fragment arrays stay in registers)
    auto tile_step = [&](int kt, auto cur_c) {
        constexpr int CUR = decltype(cur_c)::value;
        const char* st = smem + stage * STAGE;
        dot_tile(st);
        fed_tile(st, kt);
        {
#pragma unroll
            for (int kk = 0; kk < 3; ++kk) {
                read_frags(st, kk + 1, (kk + 1) & 1);
                mma_step(kk & 1, checksum_frag(kk));
                {
                    // fragment reads of the next step go out early, one per MFMA, so that the last
                    // of them has the rest of the step's MFMAs to land; the vector work of the
                    // protected schemes (global: reads and FMAs of the checksum dot product;
                    // thread-level: the sums of the B fragments) is spread between the MFMAs
                    constexpr int NF = TM + TN;
                    constexpr int NM = TM * TN + (MDOT ? 1 : 0) +
                                       (MODE == MODE_REPL ? TM * TN : (mode_is_wave_level(MODE) ? CheckRegs<CFG, EMODE>::N : 0));
                    // vector instructions per MFMA slot: the exact tile checksum's pieces cost about
                    // 14 (fp16, int8) or 22 (bf16) instructions per 16 bytes of each lane's B
                    // fragments; sums in the operand type one (fp16) or six (bf16) per register
                    constexpr int VSTEP = MODE == MODE_THREAD && ChecksumForm<CFG>::SPLIT ? (DT == DT_BF16 ? 22 : 14) * 4
                                          : (MODE == MODE_THREAD_H ? (TN - 1) * 4 * (DT == DT_BF16 ? 6 : 1)
                                             : (MODE == MODE_TWOSIDED ? (TN + TM - 2) * 4 * (DT == DT_BF16 ? 6 : 1)
                                                : (MDOT ? 4 * TM : 0)));  // (matrix-unit dot: the selects of its operands)
                    constexpr int VT = (VSTEP + NM - 1) / NM;
#pragma unroll
                    for (int g = 0; g < NM; ++g) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // 1 MFMA
                        if (g < NF) {  // LDS reads
                            if (VDOT && kk == 0) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                            else __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                        }
                        if constexpr (VDOT) __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);  // 2 VALU
                        if constexpr (VT > 0) __builtin_amdgcn_sched_group_barrier(0x002, VT, 0);
                    }
                }
            }
        }
        const int next = stage + 1 == NSTAGE ? 0 : stage + 1;
        const i32x4 fg_last = checksum_frag(3);  // (before the next tile's chunk replaces this one's)
        if (kt + 1 < nkt) {
            // this wave's copies of tile kt+1 have landed (the barrier makes it everyone's) and
            // every wave is done reading this stage, which the copies of tile kt+NSTAGE overwrite
            if (kt + NSTAGE < nkt) __builtin_amdgcn_s_waitcnt(waitcnt_vm((NSTAGE - 2) * NL) & ~0x0F00);
            else __builtin_amdgcn_s_waitcnt(0x0070);  // tail: vmcnt(0) lgkmcnt(0)
            __syncthreads();
            if (kt + NSTAGE < nkt) {
                advance();
                issue_loads(stage);
            }
            read_frags(smem + next * STAGE, 0, 0);
            read_checksum_frag(smem + next * STAGE);
        }
        mma_step(CUR, fg_last);
        stage = next;
        if constexpr (INJ) {
            // the running accumulator that holds the products just before k_after: the last k step
            if (kt == p.f_kt) inject_fault<CFG>(acc, p, TileCoords<CFG>(tile_m, tile_n));
        }
    };
    // 16x16x32 shapes (two k steps of 64 bytes per tile; at the power limit the chip sustains about an
    // eighth more of them per second than of the 32x32x16 ones): hand-placed.  A block row i of A is
    // multiplied with the TN blocks of B, then its fragment is read again in place for the step
    // after (only the B fragments are double buffered: 8 + 2 x 4 fragment registers instead of
    // 2 x 12).  The barrier sits between the two steps, as in the 32x32 form.
    auto tile_step16 = [&](int kt) {
        const char* st = smem + stage * STAGE;
        fed_tile(st, kt);
        i32x4 b0 = {0, 0, 0, 0}, b1 = {0, 0, 0, 0};
        if constexpr (VDOT) {
            b0 = *reinterpret_cast<const i32x4*>(st + beta_off);
            b1 = *reinterpret_cast<const i32x4*>(st + beta_off + (IS_INT ? 128 : 16));
        }
        // matrix-unit dot product: column 0 / 1 of the extra block of B is the first / second piece of
        // the weight checksums (lane: column l % 16, the 16 bytes of k group l / 16 of the step); the
        // fragments of both k steps are read here, before the barrier gives the stage away
        i32x4 fg[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
        if constexpr (MDOT16) {
            const i32x4 z = {0, 0, 0, 0};
            constexpr int NPC = 2;  // the low and the high digits: at bytes 0 and 128 of the record
            const int pc = lane & 15;
            const char* rec = st + LAY::AB_STAGE + (pc & 1) * 128 + fgrp * 16;
            const i32x4 r0 = *reinterpret_cast<const i32x4*>(rec), r1 = *reinterpret_cast<const i32x4*>(rec + 64);
            fg[0] = pc < NPC ? r0 : z;
            fg[1] = pc < NPC ? r1 : z;
        }
        auto half = [&](const char* src, int ps, int cur, bool dots) {
#pragma unroll
            for (int i = 0; i < TM; ++i) {
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = MMA::run(fa[0][i], fb[cur][j], acc[i][j]);
                if constexpr (MDOT16) {
                    // (wavefront column c of a row of wavefronts takes its share of the block rows: 2 c and 2 c + 1 of eight over four)
                    if (i / (TM / CFG::WAVES_N) == wave_n) gchk = MMA::run(fa[0][i], fg[cur], gchk);
                }
                __builtin_amdgcn_sched_barrier(0);  // (the read below must not move above the MFMAs: it reuses their register)
                fa[0][i] = *reinterpret_cast<const i32x4*>(src + a_off + i * MI * ROWB + ps);
                // (the TN fragments of B spread over the first block rows: one each, or TN / TM each)
                constexpr int BPG = TN > TM ? TN / TM : 1;
#pragma unroll
                for (int j = i * BPG; j < (i + 1) * BPG && j < TN; ++j)
                    fb[cur ^ 1][j] = *reinterpret_cast<const i32x4*>(src + b_off + j * MI * ROWB + ps);
                if constexpr (VDOT) {
                    // vector form of the in-loop dot product: this lane's NQA chunks of A (the ones it
                    // copied) spread over the block rows of the first step, the flush behind the last
                    constexpr int CPG = NQA > TM ? NQA / TM : 1, DSTR = NQA > TM ? 1 : TM / NQA;
                    static_assert(NQA > TM ? NQA % TM == 0 : TM % NQA == 0, "chunks of A over block rows");
                    if (dots && i % DSTR == 0) {
#pragma unroll
                        for (int q = (i / DSTR) * CPG; q < (i / DSTR + 1) * CPG && q < NQA; ++q)
                            dot.chunk(*reinterpret_cast<const i32x4*>(st + (q * WAVES + wave) * 1024 + lane * 16), b0, b1, q);
                    }
                    if (dots && i == TM - 1) dot.flush();
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        };
        static_assert(MI == 32 || TM >= TN || TN % TM == 0, "the reads of B behind the block rows");
        half(st, pos[1], 0, true);
        const int next = stage + 1 == NSTAGE ? 0 : stage + 1;
        const char* src = st;  // (last tile: the reads of the second step fetch nothing that is used)
        if (kt + 1 < nkt) {
            if (kt + NSTAGE < nkt) __builtin_amdgcn_s_waitcnt(waitcnt_vm((NSTAGE - 2) * NL) & ~0x0F00);
            else __builtin_amdgcn_s_waitcnt(0x0070);  // tail: vmcnt(0) lgkmcnt(0)
            __syncthreads();
            if (kt + NSTAGE < nkt) {
                advance();
                issue_loads(stage);
            }
            src = smem + next * STAGE;
        }
        half(src, pos[0], 1, false);
        stage = next;
        if constexpr (INJ) {
            if (kt == p.f_kt) inject_fault<CFG>(acc, p, TileCoords<CFG>(tile_m, tile_n));
        }
    };
    if constexpr (MI == 16) {
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[0][i] = *reinterpret_cast<const i32x4*>(smem + a_off + i * MI * ROWB + pos[0]);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[0][j] = *reinterpret_cast<const i32x4*>(smem + b_off + j * MI * ROWB + pos[0]);
        // (not unrolled: the unrolled body of the handed-over form spills its copy pointers, and a
        // reload of those waits, with everything else in flight, at the head of every tile)
#pragma nounroll
        for (int kt = 0; kt < nkt; ++kt) tile_step16(kt);
    } else {
    read_frags(smem, 0, 0);
    read_checksum_frag(smem);
    // the last of the four k steps sits in buffer 1
    for (int kt = 0; kt < nkt; ++kt) tile_step(kt, std::integral_constant<int, 1>());
    }
    if constexpr (INJ) {
        // a fault in the finished accumulator
        if (p.f_kt < 0) inject_fault<CFG>(acc, p, TileCoords<CFG>(tile_m, tile_n));
    }
    if constexpr (FED) dot.total += (double)fed_a * (double)fed_b;  // the last tile's
    if constexpr (MDOT16) {
        // this lane's share of the dot product: column 0 / 1 of the extra block holds A . (low / high digits)
        int g_lo = 0, g_hi = 0;
#pragma unroll
        for (int r = 0; r < MMA::NACC; ++r) {
            g_lo += gchk[r] & 0xffff;
            g_hi += gchk[r] >> 16;
        }
        dot.total = (((long long)g_hi << 16) + (long long)g_lo) * ((lane & 15) == 1 ? 256 : 1);
    }
    if constexpr (MDOT) {
        // this lane's share of the dot product: even columns hold A . (first piece), odd columns
        // A . (second piece), which carries a factor 2^11 (fp16) or stands for the digit of weight 256 (int8)
        if constexpr (IS_INT) {
            int g_lo = 0, g_hi = 0;
#pragma unroll
            for (int r = 0; r < MMA::NACC; ++r) {
                g_lo += gchk[r] & 0xffff;
                g_hi += gchk[r] >> 16;
            }
            dot.total = (((long long)g_hi << 16) + (long long)g_lo) * ((gcol & 1) ? 256 : 1);
        } else {
            double g = 0.0;
#pragma unroll
            for (int r = 0; r < MMA::NACC; r += 4) g += (double)((gchk[r] + gchk[r + 1]) + (gchk[r + 2] + gchk[r + 3]));
            dot.total = g * ((gcol & 1) ? 1.0 / 2048.0 : 1.0);
        }
    }
    epilogue<CFG, EMODE>(acc, chk, p, tile_m, tile_n, smem, true, -1, (GDOT || FED) ? &dot.total : nullptr, epi);
}

}  // namespace abft
