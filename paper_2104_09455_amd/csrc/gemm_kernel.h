// Generic ABFT-protected MFMA GEMM kernel for gfx950 (MI355X): any shape, alignment,
// weight layout, and convolutions read as an implicit im2col matrix.
//
// Data flow per workgroup: 16-byte (or element-wise) global loads -> registers -> LDS
// (double buffered, padded rows) -> ds_read_b128 MFMA fragments -> accumulators ->
// checksum epilogue -> C.
#pragma once
#include "gemm_common.h"

namespace abft {

// ---------------------------------------------------------------------------
// The kernel
// ---------------------------------------------------------------------------
template <class CFG, int MODE, bool INJ, bool CONV, bool GENERIC>
__global__ __launch_bounds__(CFG::THREADS) void gemm_kernel(const GemmArgs p) {
    typedef Mma<CFG::DT, CFG::MI> MMA;
    typedef typename MMA::Acc Acc;
    typedef typename MMA::AccT AccT;
    constexpr int MI = CFG::MI, TM = CFG::TM, TN = CFG::TN;
    constexpr int ESIZE = CFG::ESIZE, EPC = CFG::EPC;
    constexpr int BM = CFG::BM, BN = CFG::BN, BK = CFG::BK, BKB = CFG::BKB;
    constexpr int STRIDE = CFG::LDS_STRIDE, CPR = CFG::CPR, RPP = CFG::ROWS_PER_PASS;
    constexpr int NA = CFG::NA, NB = CFG::NB;
    constexpr int KSTEPS = BKB / MMA::KBYTES;
    constexpr int NGRP = 64 / MI;  // k-groups per fragment (2 or 4)
    constexpr bool IS_INT = CFG::DT == DT_I8;

    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wave_m = wave / CFG::WAVES_N, wave_n = wave % CFG::WAVES_N;
    const int lrow = lane % MI, lgrp = lane / MI;

    // workgroup -> tile: consecutive workgroups walk down M within a band of tile columns
    const int bid = blockIdx.x;
    const int tile_n = bid / p.tiles_m;
    const int tile_m = bid - tile_n * p.tiles_m;
    const int bm0 = tile_m * BM, bn0 = tile_n * BN;

    const int M = p.M, N = p.N, K = p.K;
    const int nkt = (K + BK - 1) / BK;

    // this thread's chunk column (same for all its chunks) and first row
    const int kc = tid % CPR;
    const int r0 = tid / CPR;

    // ---- implicit-GEMM row state: image offset and top-left input pixel per chunk row
    constexpr int NCONV = CONV ? NA : 1;
    long long a_row_off[NCONV];
    int a_ih0[NCONV], a_iw0[NCONV];
    int tap_c = 0, tap_kh = 0, tap_kw = 0;  // decomposition of this thread's k for the current tile
    if constexpr (CONV) {
#pragma unroll
        for (int t = 0; t < NA; ++t) {
            int m = bm0 + r0 + t * RPP;
            int mm = m < M ? m : 0;
            int img = mm / (p.OH * p.OW);
            int rem = mm - img * (p.OH * p.OW);
            int oh = rem / p.OW, ow = rem - oh * p.OW;
            a_row_off[t] = (long long)img * p.imgpitch;
            a_ih0[t] = oh * p.stride - p.pad;
            a_iw0[t] = ow * p.stride - p.pad;
        }
        int k = kc * EPC;
        int tap = k / p.Cin;
        tap_c = k - tap * p.Cin;
        tap_kh = tap / p.KW;
        tap_kw = tap - tap_kh * p.KW;
    } else {
        a_row_off[0] = 0;
        a_ih0[0] = 0;
        a_iw0[0] = 0;
    }

    auto load_a = [&](int kt, i32x4(&regs)[NA]) {
        const int k0 = kt * BK + kc * EPC;  // first k of this thread's chunk
        if constexpr (!CONV) {
            if (!GENERIC || p.a_vec) {
#pragma unroll
                for (int t = 0; t < NA; ++t) {
                    int m = bm0 + r0 + t * RPP;
                    i32x4 v = {0, 0, 0, 0};
                    if (m < M && k0 < K) v = ld16(p.A + ((long long)m * p.lda + k0) * ESIZE);
                    regs[t] = v;
                }
            } else {
#pragma unroll
                for (int t = 0; t < NA; ++t) {
                    int m = bm0 + r0 + t * RPP;
                    int nv = (m < M) ? (K - k0) : 0;
                    regs[t] = gather16<ESIZE>(p.A + ((long long)(m < M ? m : 0) * p.lda + k0) * ESIZE, ESIZE, nv);
                }
            }
        } else {
        if (!GENERIC || p.a_vec) {
            // a chunk never straddles a filter tap (Cin is a multiple of the chunk length)
#pragma unroll
            for (int t = 0; t < NA; ++t) {
                int m = bm0 + r0 + t * RPP;
                int ih = a_ih0[t] + tap_kh, iw = a_iw0[t] + tap_kw;
                i32x4 v = {0, 0, 0, 0};
                if (m < M && k0 < K && ih >= 0 && ih < p.H && iw >= 0 && iw < p.W)
                    v = ld16(p.A + (a_row_off[t] + (long long)ih * p.rowpitch + (long long)iw * p.pix + tap_c) * ESIZE);
                regs[t] = v;
            }
        } else {
            // element gather (channel counts that are no multiple of the chunk): the filter taps of
            // this thread's EPC values of k are the same for all its rows, so they are taken apart once
            int e_kh[EPC], e_kw[EPC];
            long long e_off[EPC];
            {
                int c = tap_c, kh = tap_kh, kw = tap_kw;
#pragma unroll
                for (int e = 0; e < EPC; ++e) {
                    e_kh[e] = k0 + e < K ? kh : (1 << 28);  // beyond K: never in range
                    e_kw[e] = kw;
                    e_off[e] = kh * p.rowpitch + (long long)kw * p.pix + c;
                    if (++c == p.Cin) {
                        c = 0;
                        if (++kw == p.KW) {
                            kw = 0;
                            ++kh;
                        }
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < NA; ++t) {
                const int m = bm0 + r0 + t * RPP;
                i32x4 v = {0, 0, 0, 0};
                if (m < M) {
                    const char* base = p.A + (a_row_off[t] + a_ih0[t] * p.rowpitch + (long long)a_iw0[t] * p.pix) * ESIZE;
#pragma unroll
                    for (int e = 0; e < EPC; ++e) {
                        const unsigned ih = (unsigned)(a_ih0[t] + e_kh[e]), iw = (unsigned)(a_iw0[t] + e_kw[e]);
                        unsigned x = 0;
                        if (ih < (unsigned)p.H && iw < (unsigned)p.W) {
                            const char* src = base + e_off[e] * ESIZE;
                            x = ESIZE == 2 ? (unsigned)*reinterpret_cast<const unsigned short*>(src)
                                           : (unsigned)*reinterpret_cast<const unsigned char*>(src);
                        }
                        if constexpr (ESIZE == 2) v[e >> 1] |= (int)(x << (16 * (e & 1)));
                        else v[e >> 2] |= (int)(x << (8 * (e & 3)));
                    }
                }
                regs[t] = v;
            }
        }
        }
    };
    // advance this thread's filter-tap decomposition by one k-tile
    auto advance_taps = [&]() {
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
    auto load_b = [&](int kt, i32x4(&regs)[NB]) {
        const int k0 = kt * BK + kc * EPC;
        if (!GENERIC || p.b_vec) {
#pragma unroll
            for (int t = 0; t < NB; ++t) {
                int n = bn0 + r0 + t * RPP;
                i32x4 v = {0, 0, 0, 0};
                if (n < N && k0 < K) v = ld16(p.B + ((long long)n * p.ldb + k0) * ESIZE);
                regs[t] = v;
            }
        } else {
#pragma unroll
            for (int t = 0; t < NB; ++t) {
                int n = bn0 + r0 + t * RPP;
                int nv = (n < N) ? (K - k0) : 0;
                regs[t] = gather16<ESIZE>(p.B + ((long long)(n < N ? n : 0) * p.b_sn + (long long)k0 * p.b_sk) * ESIZE,
                                          p.b_sk * ESIZE, nv);
            }
        }
    };
    auto store_tiles = [&](int buf, const i32x4(&ra)[NA], const i32x4(&rb)[NB]) {
        char* as = smem + buf * CFG::STAGE_BYTES;
        char* bs = as + BM * STRIDE;
#pragma unroll
        for (int t = 0; t < NA; ++t)
            *reinterpret_cast<i32x4*>(as + (r0 + t * RPP) * STRIDE + kc * 16) = ra[t];
#pragma unroll
        for (int t = 0; t < NB; ++t)
            *reinterpret_cast<i32x4*>(bs + (r0 + t * RPP) * STRIDE + kc * 16) = rb[t];
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

    i32x4 ra[NA], rb[NB];
    load_a(0, ra);
    load_b(0, rb);
    store_tiles(0, ra, rb);
    __syncthreads();

    for (int kt = 0; kt < nkt; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nkt;
        if (more) {
            advance_taps();
            load_a(kt + 1, ra);
            load_b(kt + 1, rb);
        }
        const char* as = smem + cur * CFG::STAGE_BYTES + (wave_m * CFG::WM + lrow) * STRIDE + lgrp * 16;
        const char* bs = smem + cur * CFG::STAGE_BYTES + BM * STRIDE + (wave_n * CFG::WN + lrow) * STRIDE + lgrp * 16;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            i32x4 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                a[i] = *reinterpret_cast<const i32x4*>(as + i * MI * STRIDE + kk * MMA::KBYTES);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                b[j] = *reinterpret_cast<const i32x4*>(bs + j * MI * STRIDE + kk * MMA::KBYTES);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) acc[i][j] = MMA::run(a[i], b[j], acc[i][j]);
            if constexpr (mode_is_wave_level(MODE)) check_step<CFG, MODE>(a, b, chk);
        }
        if (more) store_tiles(cur ^ 1, ra, rb);
        __syncthreads();
        if constexpr (INJ) {
            if (kt == p.f_kt) inject_fault<CFG>(acc, p, TileCoords<CFG>(tile_m, tile_n));
        }
    }
    if constexpr (INJ) {
        if (p.f_kt < 0) inject_fault<CFG>(acc, p, TileCoords<CFG>(tile_m, tile_n));
    }
    (void)NGRP;

    epilogue<CFG, MODE>(acc, chk, p, tile_m, tile_n, smem);
}

}  // namespace abft
