// Streaming ABFT-protected MFMA GEMM kernel for gfx950 (MI355X): layers of a few output
// tiles, whose time is the latency of one workgroup's k loop rather than bandwidth or MFMA
// rate (small-batch MLP layers, batch-1 convolutions).
//
// Workgroup tile (32 TM) x (32 TN), four wavefronts that ALL own the whole tile and split
// the k loop between them: wavefront w multiplies the k tiles t with t % 4 == w (a k tile is
// 128 bytes of k).  Each wavefront streams its own k tiles from HBM straight into its own
// ring of LDS stages (global_load_lds_dwordx4) and reads them back as MFMA fragments, so the
// k loop has no workgroup barrier at all: a wavefront only ever waits for its own copies.
// The four partial tiles are added through LDS in wavefront order, every wavefront adding and
// storing a quarter of the tile; every protected scheme makes its comparison on the added-up
// tile (one per tile), so the final addition is inside the check as well.
//
// Same alignment requirements and LDS row swizzle as the direct-to-LDS kernel, but K may be any
// whole number of 16-byte chunks: the wavefront that owns a short last k tile copies zeros in
// place of the chunks (and weight checksums) beyond K.
#pragma once
#include "gemm_fast.h"

namespace abft {

template <class CFG, int NST>
struct StreamLayout {
    static constexpr int KW = 4;                                 // wavefronts per workgroup
    static constexpr int AB_STAGE = (CFG::BM + CFG::BN) * 128;
    static constexpr int WSTAGE = AB_STAGE + 768;                // one wavefront's stage: A, B, weight checksums (six planes of 128 bytes)
    static constexpr int LDS_BYTES = KW * NST * WSTAGE;
    static constexpr int NQA = CFG::BM / 8, NQB = CFG::BN / 8;   // 1 KB copies per k tile
    static_assert(CFG::WAVES_M == 1 && CFG::WAVES_N == 1 && CFG::MI == 32 && CFG::BKB == 128, "one register tile");
    static_assert((NST - 1) * (NQA + NQB + 1) <= 63, "vmcnt range");
    static_assert(LDS_BYTES >= KW * CFG::TM * CFG::TN * 16 * 64 * 4, "LDS for the final sum");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS of one compute unit");
};

// One output tile, by all 256 threads of the workgroup (uniform call: it holds workgroup barriers).
// FRESH_A: the A operand was written earlier in the same launch by other compute units of this
// die (a chain of layers in one kernel): its copies go past the compute unit's own cache.
template <class CFG, int NST, int MODE, bool INJ, bool CONV, bool RAGGED, bool FRESH_A>
__device__ __forceinline__ void stream_tile(const GemmArgs& p, int tile_m, int tile_n, char* smem) {
    typedef StreamLayout<CFG, NST> LAY;
    constexpr int DT = CFG::DT;
    typedef Mma<DT, 32> MMA;
    typedef typename MMA::Acc Acc;
    typedef typename MMA::AccT AccT;
    constexpr int TM = CFG::TM, TN = CFG::TN, BM = CFG::BM, BN = CFG::BN, BKB = 128;
    constexpr int ESIZE = CFG::ESIZE, BK = CFG::BK;
    constexpr bool WGT = MODE == MODE_GLOBAL_W;  // three independent checksum pairs per tile (Sec. 2.4, last paragraph)
    constexpr bool GDOT = MODE == MODE_GLOBAL || WGT;  // global scheme: in-kernel checksum dot product
    // ... on the matrix unit (fp16, int8): the weight checksums, split in two exact pieces, are two
    // columns of an extra B operand, multiplied with every A fragment; the unit idles in these
    // latency-bound products, and the vector FMAs of the other form would cost more.  bf16 (three
    // pieces) keeps the vector form.
    constexpr bool MDOT = GDOT && DT != DT_BF16;
    constexpr bool IS_INT = DT == DT_I8;
    static_assert(!WGT || MDOT, "the weighted checksums ride in spare columns of the matrix-unit form");
    // copies of weight-checksum planes per k tile: the plain pair, and for the weighted scheme the
    // column-weighted checksums behind it (fp16: two planes of halves; int8: four planes of digits)
    constexpr int NBETA = !GDOT ? 0 : (WGT ? (IS_INT ? 3 : 2) : 1);
    constexpr int KW = LAY::KW, WSTAGE = LAY::WSTAGE, NQA = LAY::NQA, NQB = LAY::NQB, NL = NQA + NQB + NBETA;
    constexpr int ROWB = 128, A_STAGE = BM * ROWB;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int bm0 = tile_m * BM, bn0 = tile_n * BN;
    const int M = p.M, N = p.N;
    // K is a whole number of 16-byte chunks; the last k tile may hold fewer than eight of them
    const int nkt = (p.K + BK - 1) / BK;
    const int n_own = nkt > wave ? (nkt - wave + KW - 1) / KW : 0;  // k tiles wave, wave + 4, ...
    const int rem_chunks = RAGGED ? ((p.K * ESIZE) & 127) >> 4 : 0;  // chunks of a short last tile, 0: it is whole
    // the wavefront that owns the short tile (as the last of its own) copies zeros in place of the
    // chunks, and weight checksums, beyond K
    const bool owns_short = RAGGED && rem_chunks != 0 && wave == (nkt - 1) % KW;
    int issued = 0;  // own tiles whose copies have gone out
    char* const wbase = smem + wave * (NST * WSTAGE);

    // ---- global -> LDS copy: lane fills slot `lane` of a 1 KB block (8 rows x 8 chunks): row
    // lane/8, position lane%8, which holds chunk (lane%8) ^ key(row), key(row) = (row >> 1) & 7.
    // Block q starts at row 8q, so the key is (lane >> 4) + 4 (q & 1): two chunk columns per lane.
    const int crow = lane >> 3;
    const int ckc[2] = {(lane & 7) ^ (lane >> 4), (lane & 7) ^ ((lane >> 4) + 4)};
    const char* aptr[NQA];
    const char* bptr[NQB];
    unsigned a_valid = 0, b_valid = 0;
    long long a_img[CONV ? NQA : 1];
    int a_ih0[CONV ? NQA : 1], a_iw0[CONV ? NQA : 1];
    int tap_c[2] = {0, 0}, tap_kh[2] = {0, 0}, tap_kw[2] = {0, 0};  // per chunk column (q parity)
    // (row pointers: one 64-bit product each for A and B, then uniform steps of 8 rows)
    const char* const b_row0 = p.B + ((long long)(bn0 + crow) * p.ldb + (long long)wave * BK) * ESIZE;
    const long long b_step = 8 * p.ldb * ESIZE;
#pragma unroll
    for (int q = 0; q < NQB; ++q) {
        const int n = bn0 + q * 8 + crow;
        if (n < N) b_valid |= 1u << q;
        bptr[q] = n < N ? b_row0 + q * b_step + ckc[q & 1] * 16 : g_zero_chunk + ckc[q & 1] * 16;
    }
    const char* const a_row0 = p.A + ((long long)(bm0 + crow) * p.lda + (long long)wave * BK) * ESIZE;
    const long long a_step = 8 * p.lda * ESIZE;
#pragma unroll
    for (int q = 0; q < NQA; ++q) {
        const int m = bm0 + q * 8 + crow;
        const char* zero = g_zero_chunk + ckc[q & 1] * 16;
        if (m < M) a_valid |= 1u << q;
        if constexpr (!CONV) {
            aptr[q] = m < M ? a_row0 + q * a_step + ckc[q & 1] * 16 : zero;
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
    // weight checksums of this tile's column block: lane l copies bytes 4l .. 4l+3 of the k tile's
    // 256 (fp16 / bf16: float l of 64; int8: low digits in lanes 0-31, high digits in lanes 32-63)
    const char* beta_ptr = g_zero_chunk;
    const char* betaw_ptr = g_zero_chunk;   // weighted scheme: the column-weighted checksums' planes
    if constexpr (GDOT) {
        const long long blk = (long long)tile_n * p.K;
        // (int8 digits and fp16 halves: two planes per block, 128 bytes of each per k tile, the first
        // copied by lanes 0-31, the second by lanes 32-63; bf16: 64 floats per k tile)
        if constexpr (IS_INT) beta_ptr = p.beta_k + blk * 2 + (lane >> 5) * (long long)p.K + (long long)wave * BK + (lane & 31) * 4;
        else if constexpr (MDOT) beta_ptr = p.beta_p + blk * 8 + (lane >> 5) * 2 * (long long)p.K + (long long)wave * BK * 2 + (lane & 31) * 4;
        else beta_ptr = p.beta_k + (blk + (long long)wave * BK + lane) * 4;
        if constexpr (WGT) {
            // fp16: planes 2, 3 of the block (halves); int8: four planes of digits in the same region
            if constexpr (IS_INT) betaw_ptr = p.beta_p + blk * 8 + (lane >> 5) * (long long)p.K + (long long)wave * BK + (lane & 31) * 4;
            else betaw_ptr = p.beta_p + blk * 8 + (2 + (lane >> 5)) * 2 * (long long)p.K + (long long)wave * BK * 2 + (lane & 31) * 4;
        }
    }
    constexpr int BETA_ADV = KW * (MDOT ? 128 : BK * 4);
    // first k offset (within a k tile) of the four bytes this lane copies: one float, two halves of a
    // plane, or four digits of a plane
    const int beta_k0 = IS_INT ? (lane & 31) * 4 : (MDOT ? (lane & 31) * 2 : lane);
    if constexpr (CONV) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int k = wave * BK + ckc[h] * (16 / ESIZE);
            const int tap = k / p.Cin;
            tap_c[h] = k - tap * p.Cin;
            tap_kh[h] = tap / p.KW;
            tap_kw[h] = tap - tap_kh[h] * p.KW;
        }
    }

    // SHORT: the tile is the short last one (a wavefront-uniform case of its own, so that whole
    // tiles pay nothing for it)
    auto issue_tile = [&](int stage, auto short_c) {
        constexpr bool SHORT = decltype(short_c)::value;
        char* abase = wbase + stage * WSTAGE;
        char* bbase = abase + A_STAGE;
        // (chunk columns of this lane that lie beyond K in the short tile)
        const bool cut[2] = {SHORT && ckc[0] >= rem_chunks, SHORT && ckc[1] >= rem_chunks};
#pragma unroll
        for (int q = 0; q < NQA; ++q) {
            const char* src = aptr[q];
            if constexpr (CONV) {
                // a chunk never straddles a filter tap (Cin is a multiple of the chunk length)
                const int ih = a_ih0[q] + tap_kh[q & 1], iw = a_iw0[q] + tap_kw[q & 1];
                const bool ok = ((a_valid >> q) & 1u) && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W;
                src = ok ? p.A + (a_img[q] + (long long)ih * p.rowpitch + (long long)iw * p.pix + tap_c[q & 1]) * ESIZE
                         : g_zero_chunk + ckc[q & 1] * 16;
            }
            if (cut[q & 1]) src = g_zero_chunk + ckc[q & 1] * 16;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(abase + q * 1024), 16, 0,
                                             FRESH_A ? 16 : 0);  // (cpol bit 4: device scope, served by the die's L2)
        }
#pragma unroll
        for (int q = 0; q < NQB; ++q) {
            const char* src = cut[q & 1] ? g_zero_chunk + ckc[q & 1] * 16 : bptr[q];
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                             (__attribute__((address_space(3))) void*)(bbase + q * 1024), 16, 0, 0);
        }
        if constexpr (GDOT) {
            // this lane's four bytes of weight checksums cover k offsets beta_k0 .. of the tile
            const bool past = SHORT && beta_k0 >= rem_chunks * (16 / ESIZE);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(past ? g_zero_chunk : beta_ptr),
                                             (__attribute__((address_space(3))) void*)(abase + LAY::AB_STAGE), 4, 0, 0);
            if constexpr (WGT) {
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(past ? g_zero_chunk : betaw_ptr),
                                                 (__attribute__((address_space(3))) void*)(abase + LAY::AB_STAGE + 256), 4, 0, 0);
                if constexpr (IS_INT)   // digits 2 and 3 of the column-weighted checksums
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void*)(past ? g_zero_chunk : betaw_ptr + 2 * (long long)p.K),
                        (__attribute__((address_space(3))) void*)(abase + LAY::AB_STAGE + 512), 4, 0, 0);
            }
        }
    };
    auto issue_loads = [&](int stage) {
        if constexpr (RAGGED) {
            const bool short_tile = owns_short && issued == n_own - 1;
            ++issued;
            if (short_tile) {
                issue_tile(stage, std::true_type());
                return;
            }
        }
        issue_tile(stage, std::false_type());
    };
    // to this wavefront's next k tile: KW tiles further along k
    auto advance = [&]() {
        if constexpr (GDOT) beta_ptr += BETA_ADV;
        if constexpr (WGT) betaw_ptr += BETA_ADV;
        if constexpr (!CONV) {
#pragma unroll
            for (int q = 0; q < NQA; ++q) aptr[q] += ((a_valid >> q) & 1u) ? KW * BKB : 0;
        }
#pragma unroll
        for (int q = 0; q < NQB; ++q) bptr[q] += ((b_valid >> q) & 1u) ? KW * BKB : 0;
        if constexpr (CONV) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                tap_c[h] += KW * BK;
                while (tap_c[h] >= p.Cin) {
                    tap_c[h] -= p.Cin;
                    if (++tap_kw[h] == p.KW) {
                        tap_kw[h] = 0;
                        ++tap_kh[h];
                    }
                }
            }
        }
    };

    // ---- this wavefront's pipeline: own tile i lives in stage i % NST.  The first copies go out
    // before anything else is set up, so that the rest of the prologue runs under their latency.
#pragma unroll
    for (int s = 0; s < NST; ++s) {
        if (s < n_own) {
            if (s > 0) advance();
            issue_loads(s);
        }
    }

    Acc acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    constexpr int NCHK = CheckRegs<CFG, MODE>::N;
    Acc chk[NCHK];
#pragma unroll
    for (int i = 0; i < NCHK; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) chk[i][r] = 0;

    // ---- fragment reads: lane l reads row l%32 of a 32-row block, k chunk 2*kk + l/32, stored
    // at position chunk ^ ((row >> 1) & 7)
    const int frow = lane & 31, fgrp = lane >> 5, fx = (lane >> 1) & 7;
    const int a_off = frow * ROWB;
    const int b_off = A_STAGE + frow * ROWB;
    int pos[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) pos[kk] = ((2 * kk + fgrp) ^ fx) * 16;

    // global scheme: every lane multiplies the A chunks it copied itself with the weight
    // checksums of their k chunk (two chunk columns per lane: even and odd 1 KB blocks)
    ChecksumDot<DT> dot;
    auto dot_tile = [&](const char* st) {
        if constexpr (GDOT && !MDOT) {
            i32x4 b0[2], b1[2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const char* bs = st + LAY::AB_STAGE + ckc[h] * (IS_INT ? 16 : 32);
                b0[h] = *reinterpret_cast<const i32x4*>(bs);
                b1[h] = *reinterpret_cast<const i32x4*>(bs + (IS_INT ? 128 : 16));
            }
#pragma unroll
            for (int q = 0; q < NQA; ++q)
                dot.chunk(*reinterpret_cast<const i32x4*>(st + q * 1024 + lane * 16), b0[q & 1], b1[q & 1], q);
            dot.flush();
        }
    };
    // matrix-unit form: lanes of column 0 / 1 of the extra B operand read the first / second plane of
    // the weight checksums (their k chunk, like any fragment), all other columns are zero
    // (weighted scheme: the planes of the column-weighted checksums follow in columns 2 ..)
    constexpr int GCOLS = WGT ? (IS_INT ? 6 : 4) : 2;
    const int gcol = lane & 31;
    const int gb_off = LAY::AB_STAGE + (gcol < GCOLS ? gcol : 0) * 128 + fgrp * 16;
    i32x4 fg[2];
    Acc gchk[MDOT ? TM : 1];
    if constexpr (MDOT) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) gchk[i][r] = 0;
    }
    i32x4 fa[2][TM], fb[2][TN];
    auto read_frags = [&](const char* st, int kk, int buf) {
        if constexpr (MDOT) {
            const i32x4 g = *reinterpret_cast<const i32x4*>(st + gb_off + kk * 32);
            const i32x4 z = {0, 0, 0, 0};
            fg[buf] = gcol < GCOLS ? g : z;
        }
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[buf][i] = *reinterpret_cast<const i32x4*>(st + a_off + i * 32 * ROWB + pos[kk]);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[buf][j] = *reinterpret_cast<const i32x4*>(st + b_off + j * 32 * ROWB + pos[kk]);
    };
    auto mma_step = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) acc[i][j] = MMA::run(fa[buf][i], fb[buf][j], acc[i][j]);
        if constexpr (MDOT) {
#pragma unroll
            for (int i = 0; i < TM; ++i) gchk[i] = MMA::run(fa[buf][i], fg[buf], gchk[i]);
        }
        if constexpr (mode_is_wave_level(MODE)) check_step<CFG, MODE>(fa[buf], fb[buf], chk);
    };

    constexpr int VM_STEADY = waitcnt_vm((NST - 1) * NL);  // the oldest tile in flight has landed
    constexpr int VM_ALL = waitcnt_vm(0);
    if (n_own > 0) {
        if (n_own >= NST) __builtin_amdgcn_s_waitcnt(VM_STEADY);
        else __builtin_amdgcn_s_waitcnt(VM_ALL);
        read_frags(wbase, 0, 0);
    }
    int stage = 0;
    for (int i = 0; i < n_own; ++i) {
        const char* st = wbase + stage * WSTAGE;
        dot_tile(st);
#pragma unroll
        for (int kk = 0; kk < 3; ++kk) {
            read_frags(st, kk + 1, (kk + 1) & 1);
            mma_step(kk & 1);
        }
        const int next = stage + 1 == NST ? 0 : stage + 1;
        if (i + 1 < n_own) {
            // every fragment of this stage is in registers: the stage can take tile i + NST
            __builtin_amdgcn_s_waitcnt(0xC07F);  // lgkmcnt(0)
            if (i + NST < n_own) {
                advance();
                issue_loads(stage);
                __builtin_amdgcn_s_waitcnt(VM_STEADY);
            } else {
                __builtin_amdgcn_s_waitcnt(VM_ALL);
            }
            read_frags(wbase + next * WSTAGE, 0, 0);
        }
        mma_step(1);
        stage = next;
        if constexpr (INJ) {
            // the running accumulator that holds the products just before k_after
            if (wave + KW * i == p.f_kt) inject_fault<CFG>(acc, p, TileCoords<CFG>(tile_m, tile_n, 0));
        }
    }
    if constexpr (INJ) {
        // a fault in a finished accumulator: that of the wavefront holding the last k tile
        if (p.f_kt == -1 && wave == (nkt - 1) % KW) inject_fault<CFG>(acc, p, TileCoords<CFG>(tile_m, tile_n, 0));
    }

    // ---- the partial tiles are added in wavefront order; wavefront w adds and stores accumulator
    // registers 4w .. 4w+3 of every MFMA block (rows 8w + 4 (lane / 32) + 0..3 of the block).
    // Every protected scheme compares the ADDED-UP tile: its output summation (Sec. 2.5) runs over
    // the finished values as they are stored, so a fault in a partial accumulator and a fault in
    // this final addition both show.  The other side of the comparison is the tile's checksum
    // dot product (global scheme) or the sum of the four wavefronts' redundant accumulators
    // (thread-level schemes: checksum products of the partial products add up to the checksum
    // product of the whole, Sec. 5.2.2).
    static_assert(MODE != MODE_GLOBAL_PRE, "streaming configurations form the checksum dot product themselves");
    constexpr bool CHECKED = MODE != MODE_NONE;
    __syncthreads();  // the sum reuses every wavefront's stages
    AccT* red = reinterpret_cast<AccT*>(smem);
    constexpr int NV = TM * TN * 16;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) red[(wave * NV + (i * TN + j) * 16 + r) * 64 + lane] = acc[i][j][r];
    __syncthreads();
    const TileCoords<CFG> tc(tile_m, tile_n, 0);
    // tiles that lie wholly inside C take 8-byte stores of four columns per lane
    const bool whole = tc.bm0 + BM <= M && tc.bn0 + BN <= N && (p.ldc & 3) == 0 &&
                       (reinterpret_cast<uintptr_t>(p.C) & 7u) == 0;
    typedef typename ChecksumDot<DT>::Wide Wide;
    Wide s_sum = 0;
    int s_lo = 0, s_hi = 0;
    float f2 = 0.f, l1 = 0.f;
    // weighted scheme: output summations with the rows / the columns of the tile weighted (int8:
    // weights i + 1 and j + 1; floating point: (i + 1) / BM and (j + 1) / BN), and their norms
    Wide s_rows = 0, s_cols = 0;
    float f2_rows = 0.f, l1_rows = 0.f, f2_cols = 0.f, l1_cols = 0.f;
    // test hook: a fault in a finished value after the addition (k_after = -2): block, register
    // and lane that hold element (f_row, f_col)
    int f_blk = -1, f_rr = 0;
    if constexpr (INJ) {
        const int rr = p.f_row - tc.bm0, cc = p.f_col - tc.bn0;
        if (p.f_kt == -2 && rr >= 0 && rr < BM && cc >= 0 && cc < BN) {
            const int in_blk = rr & 31, r = (in_blk >> 3) * 4 + (in_blk & 3);
            if (wave == (r >> 2) && tc.lrow == (cc & 31) && tc.lgrp == ((in_blk >> 2) & 1)) {
                f_blk = (rr >> 5) * TN + (cc >> 5);
                f_rr = r & 3;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = tc.col(j);
            AccT v[4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) {
                const int r = 4 * wave + rr;
                v[rr] = 0;
#pragma unroll
                for (int w = 0; w < KW; ++w) v[rr] += red[(w * NV + (i * TN + j) * 16 + r) * 64 + lane];
            }
            if constexpr (INJ) {
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const unsigned mask = (f_blk == i * TN + j && f_rr == rr) ? (1u << p.f_bit) : 0u;
                    v[rr] = bitcast<AccT>(bitcast<unsigned>(v[rr]) ^ mask);
                }
            }
            // stored values: after the activation function; the checks below see the product
            AccT o[4];
#pragma unroll
            for (int rr = 0; rr < 4; ++rr) o[rr] = (p.act && !(v[rr] > 0)) ? (AccT)0 : v[rr];
            if constexpr (CFG::CSIZE == 2) {
                if (whole) {
                    // rows 8w + 4 (lane / 32) + 0..3 of this block, four columns per lane
                    char* dst = p.C + ((long long)(tc.bm0 + i * 32 + 8 * wave + 4 * tc.lgrp + (lane & 3)) * p.ldc +
                                       tc.bn0 + j * 32 + (tc.lrow & ~3)) * 2;
                    store_quad_rows<DT>(o[0], o[1], o[2], o[3], dst, lane);
                }
            }
            if (CFG::CSIZE != 2 || !whole) {
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int row = tc.bm0 + i * 32 + 8 * wave + 4 * tc.lgrp + rr;
                    if (row < M && col < N) {
                        char* dst = p.C + ((long long)row * p.ldc + col) * CFG::CSIZE;
                        if constexpr (DT == DT_F16) *reinterpret_cast<_Float16*>(dst) = (_Float16)o[rr];
                        else if constexpr (DT == DT_BF16) *reinterpret_cast<__bf16*>(dst) = (__bf16)o[rr];
                        else *reinterpret_cast<int*>(dst) = o[rr];
                    }
                }
            }
            if constexpr (CHECKED) {
                if constexpr (IS_INT) {
#pragma unroll
                    for (int rr = 0; rr < 4; ++rr) {
                        s_lo += v[rr] & 0xffff;
                        s_hi += v[rr] >> 16;
                    }
                } else {
                    s_sum += (double)((v[0] + v[1]) + (v[2] + v[3]));
                    f2 += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
                    if constexpr (GDOT)
                        l1 += (__builtin_fabsf(v[0]) + __builtin_fabsf(v[1])) + (__builtin_fabsf(v[2]) + __builtin_fabsf(v[3]));
                }
            }
            if constexpr (WGT) {
                const int col_l = j * 32 + tc.lrow;
#pragma unroll
                for (int rr = 0; rr < 4; ++rr) {
                    const int row_l = i * 32 + 8 * wave + 4 * tc.lgrp + rr;
                    if constexpr (IS_INT) {
                        s_rows += (long long)v[rr] * (row_l + 1);
                        s_cols += (long long)v[rr] * (col_l + 1);
                    } else {
                        const float xr = v[rr] * ((float)(row_l + 1) * (1.0f / BM));
                        const float xc = v[rr] * ((float)(col_l + 1) * (1.0f / BN));
                        s_rows += (double)v[rr] * ((double)(row_l + 1) * (1.0 / BM));
                        s_cols += (double)v[rr] * ((double)(col_l + 1) * (1.0 / BN));
                        f2_rows += xr * xr;
                        l1_rows += __builtin_fabsf(xr);
                        f2_cols += xc * xc;
                        l1_cols += __builtin_fabsf(xc);
                    }
                }
            }
        }
    if constexpr (WGT) {
        // ---- three comparisons for this tile (Sec. 2.4, last paragraph): the plain one, one with
        // the rows weighted, one with the columns weighted.  Checksum side, from the extra result
        // blocks: columns 0, 1 hold A . (plain weight checksums, two pieces) row by row, so weighting
        // their rows gives (w^T A)(B 1); columns 2 .. hold A . (column-weighted weight checksums).
        if constexpr (IS_INT) s_sum = ((long long)s_hi << 16) + (long long)s_lo;
        Wide d_plain = 0, d_rows = 0, d_cols = 0;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row_l = i * 32 + 8 * (r >> 2) + 4 * tc.lgrp + (r & 3);
                if constexpr (IS_INT) {
                    const long long g = gchk[i][r];
                    if (gcol < 2) {
                        const long long x = gcol == 1 ? 256 * g : g;
                        d_plain += x;
                        d_rows += x * (row_l + 1);
                    } else if (gcol < 6) {
                        d_cols += g << (8 * (gcol - 2));
                    }
                } else {
                    const double g = (double)gchk[i][r] * ((gcol & 1) ? 1.0 / 2048.0 : 1.0);
                    if (gcol < 2) {
                        d_plain += g;
                        d_rows += g * ((double)(row_l + 1) * (1.0 / BM));
                    } else if (gcol < 4) {
                        d_cols += g;
                    }
                }
            }
        Wide sums[6] = {s_sum, s_rows, s_cols, d_plain, d_rows, d_cols};
        float norms[6] = {f2, l1, f2_rows, l1_rows, f2_cols, l1_cols};
#pragma unroll
        for (int q = 0; q < 6; ++q) {
            sums[q] = wave_sum(sums[q]);
            norms[q] = IS_INT ? 0.f : wave_sum(norms[q]);
        }
        __syncthreads();  // everyone is done reading the partial tiles
        double* redd = reinterpret_cast<double*>(smem);
        Wide* redw = reinterpret_cast<Wide*>(smem) + 6 * KW;
        if (lane == 0) {
#pragma unroll
            for (int q = 0; q < 6; ++q) {
                redd[6 * wave + q] = (double)norms[q];
                redw[6 * wave + q] = sums[q];
            }
        }
        __syncthreads();
        if (tid == 0) {
            double tn_[6];
            Wide ts_[6];
            for (int q = 0; q < 6; ++q) {
                tn_[q] = 0.0;
                ts_[q] = 0;
                for (int w = 0; w < KW; ++w) {
                    tn_[q] += redd[6 * w + q];
                    ts_[q] += redw[6 * w + q];
                }
            }
            const unsigned t = (unsigned)(tile_m * p.tiles_n + tile_n);
            bool bad = false;
            double ratio[3], tau0 = 0.0;
            for (int c = 0; c < 3; ++c) {
                const double res = __builtin_fabs((double)(ts_[c] - ts_[3 + c]));
                if constexpr (IS_INT) {
                    const bool differs = ts_[c] != ts_[3 + c];
                    bad |= differs;
                    ratio[c] = differs ? __builtin_huge_val() : 0.0;
                } else {
                    const double tau = p.tol_coeff * __builtin_sqrt(tn_[2 * c]) + p.tol_l1 * tn_[2 * c + 1];
                    const bool finite = __builtin_isfinite((double)ts_[c]) && __builtin_isfinite((double)ts_[3 + c]) &&
                                        __builtin_isfinite(tn_[2 * c]);
                    bad |= !finite || !(res <= tau);
                    ratio[c] = !finite ? __builtin_huge_val() : (tau > 0.0 ? res / tau : (res > 0.0 ? __builtin_huge_val() : 0.0));
                    if (c == 0) tau0 = tau;
                }
            }
            if (bad) atomicOr(p.flag, 1u);
            if (p.report) {
                // where a single wrong element of this tile would sit: its weights are the ratios of
                // the weighted residuals to the plain one
                Located loc = {-1, -1, 0.0, ratio[1], ratio[2]};
                const double r0 = (double)(ts_[0] - ts_[3]);
                if (ratio[0] > 1.0 && r0 != 0.0) {
                    const double wr = (double)(ts_[1] - ts_[4]) / r0, wc = (double)(ts_[2] - ts_[5]) / r0;
                    const long long li = __builtin_llrint(IS_INT ? wr : wr * BM) - 1, lj = __builtin_llrint(IS_INT ? wc : wc * BN) - 1;
                    if (li >= 0 && li < BM && lj >= 0 && lj < BN) {
                        loc.row = tile_m * BM + (int)li;
                        loc.col = tile_n * BN + (int)lj;
                        loc.delta = r0;
                    }
                }
                const double worst = ratio[0] > ratio[1] ? (ratio[0] > ratio[2] ? ratio[0] : ratio[2])
                                                         : (ratio[1] > ratio[2] ? ratio[1] : ratio[2]);
                report_update(p.report, worst, (double)ts_[0], (double)ts_[3], tau0, __builtin_sqrt(tn_[0]), tn_[1], t, &loc);
            }
        }
        return;
    }
    if constexpr (CHECKED) {
        // comparison (Sec. 2.4 step 4 / Sec. 5.2.2) for this tile
        if constexpr (IS_INT) s_sum = ((long long)s_hi << 16) + (long long)s_lo;
        // this lane's share of the other side
        Wide lane_dot = dot.total;
        if constexpr (mode_is_wave_level(MODE)) lane_dot = lane_check_sum<CFG, MODE>(chk, lane);
        if constexpr (MDOT) {
            // column 0 of the extra result blocks holds A . (first plane), column 1 A . (second plane)
            if constexpr (IS_INT) {
                int g_lo = 0, g_hi = 0;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        g_lo += gchk[i][r] & 0xffff;
                        g_hi += gchk[i][r] >> 16;
                    }
                lane_dot = (((long long)g_hi << 16) + (long long)g_lo) * (gcol == 1 ? 256 : 1);
            } else {
                double g = 0.0;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < 16; r += 4)
                        g += (double)((gchk[i][r] + gchk[i][r + 1]) + (gchk[i][r + 2] + gchk[i][r + 3]));
                lane_dot = g * (gcol == 1 ? 1.0 / 2048.0 : 1.0);
            }
        }
        // cross-lane sums: the norms of the tolerance in fp32; the two sides of the comparison in
        // wide arithmetic, as one sum of their per-lane difference unless the report wants them apart
        Wide wdot = 0;
        if (p.report) {
            s_sum = wave_sum(s_sum);
            wdot = wave_sum(lane_dot);
        } else {
            s_sum = wave_sum((Wide)(s_sum - lane_dot));
        }
        const double F2 = IS_INT ? 0.0 : (double)wave_sum(f2);
        const double L1 = (IS_INT || !GDOT) ? 0.0 : (double)wave_sum(l1);
        __syncthreads();  // everyone is done reading the partial tiles
        double* redd = reinterpret_cast<double*>(smem);
        Wide* redw = reinterpret_cast<Wide*>(smem) + 2 * KW;
        if (lane == 0) {
            redd[2 * wave] = F2;
            redd[2 * wave + 1] = L1;
            redw[2 * wave] = s_sum;
            redw[2 * wave + 1] = wdot;
        }
        __syncthreads();
        if (tid == 0) {
            double tf = 0.0, tl = 0.0;
            Wide ts = 0, sab = 0;
            for (int w = 0; w < KW; ++w) {
                tf += redd[2 * w];
                tl += redd[2 * w + 1];
                ts += redw[2 * w];
                sab += redw[2 * w + 1];
            }
            const unsigned t = (unsigned)(tile_m * p.tiles_n + tile_n);
            if constexpr (IS_INT) {
                // (replication: a block that took several products may have wrapped where the
                // product's own blocks did not; the two sides still agree modulo 2^32, and a
                // flipped bit never changes a sum by a multiple of 2^32)
                const bool bad = MODE == MODE_REPL ? (unsigned int)(ts - sab) != 0u : ts != sab;
                if (bad) atomicOr(p.flag, 1u);
                if (p.report)
                    report_update(p.report, bad ? __builtin_huge_val() : 0.0, (double)ts, (double)sab, 0.0, 0.0, 0.0, t);
            } else {
                const double frob = __builtin_sqrt(tf);
                const double tau = p.tol_coeff * frob + (GDOT ? p.tol_l1 * tl : 0.0);
                const double res = __builtin_fabs((double)ts - (double)sab);
                // a sum of squares beyond the fp32 range cannot come from a fault-free tile
                const bool finite = __builtin_isfinite((double)ts) && __builtin_isfinite((double)sab) && __builtin_isfinite(tf);
                const bool bad = !finite || !(res <= tau);
                if (bad) atomicOr(p.flag, 1u);
                if (p.report) {
                    const double ratio = !finite ? __builtin_huge_val()
                                                 : (tau > 0.0 ? res / tau : (res > 0.0 ? __builtin_huge_val() : 0.0));
                    report_update(p.report, ratio, (double)ts, (double)sab, tau, frob, tl, t);
                }
            }
        }
    }
}

// RAGGED: K is a whole number of 16-byte chunks but not of k tiles (an instance of its own, so that
// products of whole k tiles pay nothing for the short last tile)
template <class CFG, int NST, int MODE, bool INJ, bool CONV, bool RAGGED = false>
__global__ __launch_bounds__(256) void gemm_stream_kernel(const GemmArgs p) {
    extern __shared__ __attribute__((aligned(16))) char smem[];
    int tile_m, tile_n;
    tile_of_block((int)blockIdx.x, p.tiles_m, p.tiles_n, tile_m, tile_n);
    stream_tile<CFG, NST, MODE, INJ, CONV, RAGGED, false>(p, tile_m, tile_n, smem);
}

}  // namespace abft
