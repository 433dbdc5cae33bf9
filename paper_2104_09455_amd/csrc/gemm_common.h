// Shared device code of the ABFT-protected MFMA GEMM kernels for gfx950 (MI355X).
//
// The kernel templates cover the unprotected product, global ABFT (fused output
// summation, paper Sec. 2.5) and thread-level one-sided ABFT (paper Sec. 5.2.2)
// carried out per wavefront register tile.  A is M x K (row-major or an NHWC
// tensor read as an implicit im2col matrix), B is K x N, C is M x N (Sec. 2.1).
//
// Data flow per workgroup: 16-byte global loads -> registers -> LDS (double
// buffered, padded rows) -> ds_read_b128 MFMA fragments -> accumulators.
#pragma once  // shared device code: types, MFMA wrappers, reductions, tile checksum, epilogue
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace abft {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

enum { DT_F16 = 0, DT_BF16 = 1, DT_I8 = 2 };
// MODE_GLOBAL_PRE (kernel-internal): the global scheme with the checksum dot products left by
// the activation-checksum kernel instead of formed inside the product's loop
enum { MODE_NONE = 0, MODE_GLOBAL = 1, MODE_THREAD = 2, MODE_GLOBAL_PRE = 3, MODE_REPL = 4, MODE_THREAD_H = 5,
       MODE_TWOSIDED = 6, MODE_GLOBAL_W = 7, MODE_GLOBAL_FED = 8 };
// MODE_GLOBAL_FED (kernel-internal): the global scheme with the activation checksums handed over
// by the layer before (Sec. 2.4 step 4: the previous layer's epilogue forms them from the values
// it stores), as column sums per block of 32 rows; direct-to-LDS kernel, fp16 / bf16.
// MODE_GLOBAL_W: the global scheme with three independent checksum pairs per workgroup tile
// (Sec. 2.4, last paragraph): plain, rows weighted, columns weighted; streaming kernel only.
// MODE_REPL: thread-level replication with single accumulation (Sec. 5.1): every MFMA of the
// product is issued a second time into one accumulator block per A fragment; the sum of those
// blocks must equal the sum of the wavefront tile.  Checked exactly like MODE_THREAD.
// MODE_THREAD_H: one-sided thread-level ABFT with the tile checksum added up in the operand
// type, as the paper does it (Sec. 5.2.2: packed half-precision adds): one extra MFMA per A
// fragment and k step.  MODE_TWOSIDED: two-sided thread-level ABFT (Sec. 5.2.1): the checksums of
// both the A fragments and the B fragments, added up in the operand type, one extra MFMA per k
// step.  Both carry the rounding of those adds in their tolerance.
constexpr bool mode_is_wave_level(int mode) {
    return mode == MODE_THREAD || mode == MODE_REPL || mode == MODE_THREAD_H || mode == MODE_TWOSIDED;
}

struct Report {  // mirrors abft_report_t
    double lhs, rhs, tau, worst_ratio;
    unsigned long long tiles;
    double frob, l1;
    unsigned int lock, region;
    // weighted global scheme: where a single wrong element of the reported region would sit
    int fault_row, fault_col;
    double fault_delta, ratio_rows, ratio_cols;
};
// localisation fields of one comparison (weighted global scheme)
struct Located {
    int row, col;
    double delta, ratio_rows, ratio_cols;
};

// Record one comparison in the optional diagnostics block: counts it and, under a small
// spin lock (one lane per wavefront ever takes it, and only when diagnostics were asked
// for), keeps the fields of the comparison with the largest ratio -- ties go to the lowest
// region index, so the outcome does not depend on scheduling.  The spin is bounded; a
// wavefront that cannot get the lock skips its update.
__device__ __forceinline__ void report_update(Report* rep, double ratio, double lhs, double rhs, double tau,
                                              double frob, double l1, unsigned region, const Located* loc = nullptr) {
    atomicAdd(&rep->tiles, 1ull);
    volatile Report* v = rep;
    {
        // A comparison that cannot displace the stored one leaves without the lock.  The stored
        // entry only ever moves to a larger ratio, or at the same ratio to a lower region, so
        // losing against what was read (region first, then ratio) means losing against what is
        // there now; ties are settled without the lock only at ratio 0, where every earlier
        // entry had ratio 0 as well.
        const unsigned reg = v->region;
        const double cur = v->worst_ratio;
        if (reg != 0u && (ratio < cur || (ratio == 0.0 && cur == 0.0 && region + 1u >= reg))) return;
    }
    bool got = false;
    for (int spin = 0; spin < (1 << 22) && !got; ++spin) got = atomicCAS(&rep->lock, 0u, 1u) == 0u;
    if (!got) return;
    __threadfence();
    const bool first = v->region == 0u;
    const double cur = v->worst_ratio;
    if (first || ratio > cur || (ratio == cur && region + 1u < v->region)) {
        v->worst_ratio = ratio;
        v->lhs = lhs;
        v->rhs = rhs;
        v->tau = tau;
        v->frob = frob;
        v->l1 = l1;
        v->region = region + 1u;
        if (loc) {
            v->fault_row = loc->row;
            v->fault_col = loc->col;
            v->fault_delta = loc->delta;
            v->ratio_rows = loc->ratio_rows;
            v->ratio_cols = loc->ratio_cols;
        }
    }
    __threadfence();
    atomicExch(&rep->lock, 0u);
}

struct GemmArgs {
    const char* A;
    const char* B;
    char* C;
    int M, N, K;
    long long lda, ldb, ldc;  // elements
    // element strides of B for the generic loader: B[k][n] at B + n*b_sn + k*b_sk
    long long b_sn, b_sk;
    int a_vec, b_vec;  // operands qualify for 16-byte loads along k
    // implicit-GEMM geometry (conv != 0): A is an NHWC tensor
    int conv, H, W, Cin, KH, KW, stride, pad, OH, OW;
    // input element (img, ih, iw, c) sits at img * imgpitch + ih * rowpitch + iw * pix + c (a plain
    // NHWC tensor: pix = Cin, rowpitch = W Cin, imgpitch = H W Cin)
    long long imgpitch, rowpitch;
    int pix;
    // ABFT outputs
    const char* beta_k;       // GLOBAL, direct-to-LDS kernel: weight checksums per column block for the in-kernel
                              // checksum dot product: float[K] per block (fp16 / bf16), or K low digits then
                              // K high digits (balanced base 256, one byte each) per block (int8)
    const char* beta_p;       // GLOBAL, streaming kernel, fp16: the same checksums as two planes of halves per
                              // block, K values hi = fl16(beta) then K values lo = fl16((beta - hi) 2^11)
    const char* beta_r;       // GLOBAL, direct-to-LDS kernel: the same checksums as one 1 KB record per block and k
                              // tile, copied with the operand tiles (layout: weight_checksum_kernel)
    const void* partial_dots; // GLOBAL otherwise: per tile n_parts partial checksum dot products (double / int64)
    int n_parts;
    double tol_l1;           // GLOBAL: coefficient of the tile's sum of magnitudes in tau
    unsigned int* flag;      // OR-ed with 1 on mismatch
    Report* report;          // optional diagnostics (THREAD only here)
    double tol_coeff;        // THREAD: tau = tol_coeff * ||C_tile||_F
    // fault injection (test hook): flip bit f_bit of accumulator (f_row, f_col)
    // after k-tile f_kt has been accumulated (f_kt < 0: after the last one)
    int f_row, f_col, f_bit, f_kt;
    int tiles_m, tiles_n;    // grid shape in tiles
    // activation function applied to the finished values as they are stored (Sec. 2.4 step 4:
    // after the checks, which see the accumulators as the product left them): 0 none, 1 max(x, 0)
    int act;
    // Activation checksums for the NEXT layer (Sec. 2.4 step 4), or null: alpha_out[b * ld_alpha_out + n] =
    // sum over the rows m of 32-row block b of the value stored at C[m][n] (after the activation
    // function, rounded to the output type), as a float.  fp16 / bf16, 32 x 32 MFMA shapes.
    float* alpha_out;
    long long ld_alpha_out;
    // MODE_GLOBAL_FED: the same from the layer before, for this layer's A: alpha_in[b * K + k]
    const float* alpha_in;
};

template <typename To, typename Ti>
__device__ __forceinline__ To bitcast(const Ti& v) {
    static_assert(sizeof(To) == sizeof(Ti), "size");
    return __builtin_bit_cast(To, v);
}

// ---------------------------------------------------------------------------
// MFMA wrappers.  Operands travel as 16 bytes per lane.
// 32x32 shapes: lane l feeds row/column l%32, k-group l/32 (2 groups of 16 bytes);
//               result register r of lane l is row 8*(r/4) + 4*(l/32) + r%4, column l%32.
// 16x16 shapes: lane l feeds row/column l%16, k-group l/16 (4 groups);
//               result register r of lane l is row 4*(l/16) + r, column l%16.
// ---------------------------------------------------------------------------
template <int DT, int MI>
struct Mma;

template <>
struct Mma<DT_F16, 32> {
    typedef f32x16 Acc;
    typedef float AccT;
    static constexpr int NACC = 16, KBYTES = 32;
    static __device__ __forceinline__ Acc run(i32x4 a, i32x4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(bitcast<f16x8>(a), bitcast<f16x8>(b), c, 0, 0, 0);
    }
};
template <>
struct Mma<DT_BF16, 32> {
    typedef f32x16 Acc;
    typedef float AccT;
    static constexpr int NACC = 16, KBYTES = 32;
    static __device__ __forceinline__ Acc run(i32x4 a, i32x4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(bitcast<bf16x8>(a), bitcast<bf16x8>(b), c, 0, 0, 0);
    }
};
template <>
struct Mma<DT_I8, 32> {
    typedef i32x16 Acc;
    typedef int AccT;
    static constexpr int NACC = 16, KBYTES = 32;
    static __device__ __forceinline__ Acc run(i32x4 a, i32x4 b, Acc c) {
        return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0);
    }
};
template <>
struct Mma<DT_F16, 16> {
    typedef f32x4 Acc;
    typedef float AccT;
    static constexpr int NACC = 4, KBYTES = 64;
    static __device__ __forceinline__ Acc run(i32x4 a, i32x4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(bitcast<f16x8>(a), bitcast<f16x8>(b), c, 0, 0, 0);
    }
};
template <>
struct Mma<DT_BF16, 16> {
    typedef f32x4 Acc;
    typedef float AccT;
    static constexpr int NACC = 4, KBYTES = 64;
    static __device__ __forceinline__ Acc run(i32x4 a, i32x4 b, Acc c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(bitcast<bf16x8>(a), bitcast<bf16x8>(b), c, 0, 0, 0);
    }
};
template <>
struct Mma<DT_I8, 16> {
    typedef i32x4 Acc;
    typedef int AccT;
    static constexpr int NACC = 4, KBYTES = 64;
    static __device__ __forceinline__ Acc run(i32x4 a, i32x4 b, Acc c) {
        return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
    }
};

// ---------------------------------------------------------------------------
// Wavefront reductions in registers (DPP within rows of 16 lanes, v_readlane
// across the four rows).  Fixed order, so results are run-to-run identical.
// ---------------------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ int dpp_i32(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
template <int CTRL, typename T>
__device__ __forceinline__ T dpp_move(T v) {
    if constexpr (sizeof(T) == 4) {
        return bitcast<T>(dpp_i32<CTRL>(bitcast<int>(v)));
    } else {
        static_assert(sizeof(T) == 8, "4 or 8 bytes");
        unsigned long long u = bitcast<unsigned long long>(v);
        int lo = dpp_i32<CTRL>((int)(u & 0xffffffffu));
        int hi = dpp_i32<CTRL>((int)(u >> 32));
        u = ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo;
        return bitcast<T>(u);
    }
}
template <typename T>
__device__ __forceinline__ T readlane(T v, int lane) {
    if constexpr (sizeof(T) == 4) {
        return bitcast<T>(__builtin_amdgcn_readlane(bitcast<int>(v), lane));
    } else {
        unsigned long long u = bitcast<unsigned long long>(v);
        int lo = __builtin_amdgcn_readlane((int)(u & 0xffffffffu), lane);
        int hi = __builtin_amdgcn_readlane((int)(u >> 32), lane);
        u = ((unsigned long long)(unsigned)hi << 32) | (unsigned)lo;
        return bitcast<T>(u);
    }
}
// sum over the 64 lanes, returned in every lane
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
    v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]: lane ^ 1
    v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]: lane ^ 2
    v += dpp_move<0x141>(v);  // row_half_mirror: the other quad of the half row
    v += dpp_move<0x140>(v);  // row_mirror: the other half row
    T a = readlane(v, 0), b = readlane(v, 16), c = readlane(v, 32), d = readlane(v, 48);
    return (a + b) + (c + d);
}

// ---------------------------------------------------------------------------
// Tile configuration
// ---------------------------------------------------------------------------
template <int DT_, int MI_, int TM_, int TN_, int WAVES_M_, int WAVES_N_, int BKB_>
struct Cfg {
    static constexpr int DT = DT_, MI = MI_, TM = TM_, TN = TN_;
    static constexpr int WAVES_M = WAVES_M_, WAVES_N = WAVES_N_, BKB = BKB_;
    static constexpr int ESIZE = (DT_ == DT_I8) ? 1 : 2;  // bytes per input element
    static constexpr int CSIZE = (DT_ == DT_I8) ? 4 : 2;  // bytes per output element
    static constexpr int EPC = 16 / ESIZE;                // elements per 16-byte chunk
    static constexpr int WM = MI_ * TM_, WN = MI_ * TN_;  // wavefront register tile
    static constexpr int BM = WM * WAVES_M_, BN = WN * WAVES_N_;
    static constexpr int BK = BKB_ / ESIZE;
    static constexpr int THREADS = 64 * WAVES_M_ * WAVES_N_;
    static constexpr int LDS_STRIDE = BKB_ + 16;  // padded row, bytes
    static constexpr int CPR = BKB_ / 16;         // 16-byte chunks per tile row
    static constexpr int ROWS_PER_PASS = THREADS / CPR;
    static constexpr int NA = BM / ROWS_PER_PASS;  // chunks of A per thread per k-tile
    static constexpr int NB = BN / ROWS_PER_PASS;
    static constexpr int STAGE_BYTES = (BM + BN) * LDS_STRIDE;
    static constexpr int LDS_BYTES = 2 * STAGE_BYTES;
    static_assert(THREADS % CPR == 0, "threads must cover whole tile rows");
    static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "tile rows vs threads");
    static_assert(BKB_ % Mma<DT_, MI_>::KBYTES == 0, "k tile vs MFMA depth");
};

__device__ __forceinline__ i32x4 ld16(const char* p) { return *reinterpret_cast<const i32x4*>(p); }

// 16 bytes gathered element by element: element e of the chunk is at base + e*stride
// (bytes) and is taken only while e < n_valid.  Every load reads an element of the run (the
// index is clamped to the last valid one, the value dropped afterwards), so that the loads
// carry no condition and go out together instead of one round trip after the other.
template <int ESIZE>
__device__ __forceinline__ i32x4 gather16(const char* base, long long stride_bytes, int n_valid) {
    i32x4 out = {0, 0, 0, 0};
    if (n_valid <= 0) return out;
    const int last = n_valid - 1;
    if constexpr (ESIZE == 2) {
        unsigned v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            v[e] = *reinterpret_cast<const unsigned short*>(base + (e < last ? e : last) * stride_bytes);
#pragma unroll
        for (int e = 0; e < 8; ++e) out[e >> 1] |= (int)((e <= last ? v[e] : 0u) << (16 * (e & 1)));
    } else {
        unsigned v[16];
#pragma unroll
        for (int e = 0; e < 16; ++e)
            v[e] = *reinterpret_cast<const unsigned char*>(base + (e < last ? e : last) * stride_bytes);
#pragma unroll
        for (int e = 0; e < 16; ++e) out[e >> 2] |= (int)((e <= last ? v[e] : 0u) << (8 * (e & 3)));
    }
    return out;
}

// ---------------------------------------------------------------------------
// Tile-local weight checksum for the thread-level scheme (Sec. 5.2.1-5.2.2): per k step the
// checksum of the wavefront tile's B fragments,
//   chi[k] = sum over the wave tile's columns of B[k][.],
// goes to the matrix unit as extra B operand(s), multiplied with every A fragment.  A lane holds
// one column of each of the TN fragments (MFMA block columns), so the vector unit adds the TN
// fragments element by element and the matrix unit finishes the sum over the 32 columns of
// the block: summing the checksum accumulators over their columns at the end gives
// sum_k A[i][k] chi[k].
//  * Plain form (TN = 1): nothing to add, the operand is the fragment itself (one block
//    column per wavefront tile: the scheme coincides with replication, Table 1's M_t / 2 extra
//    MMAs being all of them).
//  * Split form (TN >= 2): the element-wise sums are handed on in exactly representable
//    pieces, one operand and one set of accumulators per piece (below).
// ---------------------------------------------------------------------------
// ---------------------------------------------------------------------------
// Split form of the tile checksum for fp16: no cross-lane step at all.  The column sums s (fp32, one per lane and k) are handed to
// the matrix unit as two operands, hi = fl16(s) and lo = fl16((s - hi) * 2^11), each
// multiplied with the A fragments into its own accumulators; the checksum product is
// sum(hi accumulators) + 2^-11 sum(lo accumulators).  Twice the checksum MFMAs of the
// folded form, but half the vector work -- the right trade where the matrix unit idles.
// v_fma_mix_f32 converts and accumulates a half in one instruction.
// ---------------------------------------------------------------------------
template <int TN>
struct TileChecksumSplitF16 {
    static __device__ __forceinline__ float acc_lo(int packed, float s) {
        float r;
        asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(packed), "v"(s));
        return r;
    }
    static __device__ __forceinline__ float acc_hi(int packed, float s) {
        float r;
        asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(packed), "v"(s));
        return r;
    }
    // s - (half `sel` of packed), exact
    static __device__ __forceinline__ float sub_lo(int packed, float s) {
        float r;
        asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(packed), "v"(s));
        return r;
    }
    static __device__ __forceinline__ float sub_hi(int packed, float s) {
        float r;
        asm("v_fma_mix_f32 %0, %1, -1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(packed), "v"(s));
        return r;
    }
    // weight of the low operand's products in the checksum sum
    static constexpr double LO_SCALE = TN == 2 ? 1.0 : 1.0 / 2048.0;
    static __device__ __forceinline__ void make(const i32x4 (&b)[TN], i32x4& hi, i32x4& lo) {
        if constexpr (TN == 2) {
            // two fragments: an error-free sum in packed fp16 (six instructions per register):
            // hi = fl16(x + y) and lo = (x + y) - hi exactly, subnormal results included (the
            // matrix unit takes fp16 subnormals as they are)
            typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const f16x2 x = bitcast<f16x2>(b[0][d]), y = bitcast<f16x2>(b[1][d]);
                const f16x2 s = x + y;
                const f16x2 yy = s - x;
                const f16x2 e = (x - (s - yy)) + (y - yy);
                hi[d] = bitcast<int>(s);
                lo[d] = bitcast<int>(e);
            }
            return;
        }
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            float s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                s0 = acc_lo(b[j][d], s0);
                s1 = acc_hi(b[j][d], s1);
            }
            // round to nearest (v_cvt_pk_f16_f32): hi is within 2^-11 of s, lo within 2^-11 of the
            // remainder, so hi + 2^-11 lo matches s to 22 bits
            typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
            f16x2 hp;
            hp[0] = (_Float16)s0;
            hp[1] = (_Float16)s1;
            const int h = bitcast<int>(hp);
            const float d0 = sub_lo(h, s0) * 2048.f, d1 = sub_hi(h, s1) * 2048.f;
            f16x2 lp;
            lp[0] = (_Float16)d0;
            lp[1] = (_Float16)d1;
            hi[d] = h;
            lo[d] = bitcast<int>(lp);
        }
    }
};

// Split form for bf16: the column sums (fp32, exact: a few bf16 values) go out as three bf16
// operands hi + mid + lo = s exactly (3 x 8 significant bits), each multiplied with the A
// fragments into its own accumulators.  No cross-lane step.
template <int TN>
struct TileChecksumSplitBF16 {
    static __device__ __forceinline__ float lo_f(int packed) { return bitcast<float>(packed << 16); }
    static __device__ __forceinline__ float hi_f(int packed) { return bitcast<float>((int)(packed & 0xffff0000)); }
    static __device__ __forceinline__ int pack(float a, float b) {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        bf16x2 h;
        h[0] = (__bf16)a;  // round to nearest even
        h[1] = (__bf16)b;
        return bitcast<int>(h);
    }
    static __device__ __forceinline__ void make(const i32x4 (&b)[TN], i32x4& x0, i32x4& x1, i32x4& x2) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            float s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                s0 += lo_f(b[j][d]);
                s1 += hi_f(b[j][d]);
            }
            const int h = pack(s0, s1);
            const float r0 = s0 - lo_f(h), r1 = s1 - hi_f(h);  // exact remainders
            const int m = pack(r0, r1);
            const float q0 = r0 - lo_f(m), q1 = r1 - hi_f(m);
            x0[d] = h;
            x1[d] = m;
            x2[d] = pack(q0, q1);
        }
    }
};

// Split form for int8: the column sums (at most 10 bits) are formed in packed 16-bit lanes
// (even and odd bytes of each register apart) and go out as two operands of balanced
// base-256 digits, s = lo + 256 hi exactly.  No cross-lane step.
template <int TN>
struct TileChecksumSplitI8 {
    typedef short s16x2 __attribute__((ext_vector_type(2)));
    static __device__ __forceinline__ void make(const i32x4 (&b)[TN], i32x4& lo, i32x4& hi) {
#pragma unroll
        for (int d = 0; d < 4; ++d) {
            s16x2 se = {0, 0}, so = {0, 0};
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const s16x2 x = bitcast<s16x2>(b[j][d]);
                se += (s16x2)(x << 8) >> 8;  // bytes 0 and 2, sign extended
                so += x >> 8;                // bytes 1 and 3
            }
            const s16x2 le = (s16x2)(se << 8) >> 8, lod = (s16x2)(so << 8) >> 8;  // low digits
            const s16x2 he = (se - le) >> 8, hod = (so - lod) >> 8;              // high digits
            lo[d] = (bitcast<int>(le) & 0x00ff00ff) | ((bitcast<int>(lod) & 0x00ff00ff) << 8);
            hi[d] = (bitcast<int>(he) & 0x00ff00ff) | ((bitcast<int>(hod) & 0x00ff00ff) << 8);
        }
    }
};

// The split form for any operand type: NP operands x[0..NP) whose accumulators, weighted with
// scale(piece) (int8: 1 and 256, applied in integers by the epilogue), add up to the checksum
// product.
template <int DT, int TN>
struct TileChecksumSplit {
    static constexpr int NP = DT == DT_BF16 ? 3 : 2;
    static __device__ __forceinline__ void make(const i32x4 (&b)[TN], i32x4 (&x)[NP]) {
        if constexpr (DT == DT_F16) TileChecksumSplitF16<TN>::make(b, x[0], x[1]);
        else if constexpr (DT == DT_BF16) TileChecksumSplitBF16<TN>::make(b, x[0], x[1], x[2]);
        else TileChecksumSplitI8<TN>::make(b, x[0], x[1]);
    }
    static constexpr double scale(int piece) {
        return (DT == DT_F16 && piece == 1) ? TileChecksumSplitF16<TN>::LO_SCALE : 1.0;
    }
};

// acc + (half SEL of `packed`, an fp16 or bf16 value) * b, in fp32
template <int DT, int SEL>
__device__ __forceinline__ float mul_add_half(int packed, float b, float acc) {
    if constexpr (DT == DT_F16) {
        float r;
        if constexpr (SEL == 0)
            asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(packed), "v"(b), "v"(acc));
        else
            asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(packed), "v"(b), "v"(acc));
        return r;
    } else {
        const float a = bitcast<float>(SEL == 0 ? (packed << 16) : (int)(packed & 0xffff0000));
        return __builtin_fmaf(a, b, acc);
    }
}

// Running checksum dot product of the global scheme inside a product kernel (Sec. 2.4 steps 1-3):
// sum of A[m][k] * beta[k] over 16-byte chunks of A read back from LDS, each with the weight
// checksums of its 8 (fp16 / bf16) or 16 (int8) values of k: b0, b1 = 8 floats, or 16 low digits
// and 16 high digits (balanced base 256).  Products are summed in fp32 / int32 within a k tile
// (at most a few dozen terms per lane) and in double / int64 above that.
template <int DT>
struct ChecksumDot {
    typedef typename std::conditional<DT == DT_I8, long long, double>::type Wide;
    float f[4] = {0.f, 0.f, 0.f, 0.f};
    int lo = 0, hi = 0;
    Wide total = 0;
    __device__ __forceinline__ void chunk(const i32x4& c, const i32x4& b0, const i32x4& b1, int slot) {
        if constexpr (DT == DT_I8) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                lo = __builtin_amdgcn_sdot4(c[d], b0[d], lo, false);
                hi = __builtin_amdgcn_sdot4(c[d], b1[d], hi, false);
            }
        } else {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const float w0 = bitcast<float>(d < 2 ? b0[2 * d] : b1[2 * d - 4]);
                const float w1 = bitcast<float>(d < 2 ? b0[2 * d + 1] : b1[2 * d - 3]);
                f[slot & 3] = mul_add_half<DT, 0>(c[d], w0, f[slot & 3]);
                f[slot & 3] = mul_add_half<DT, 1>(c[d], w1, f[slot & 3]);
            }
        }
    }
    // end of a k tile
    __device__ __forceinline__ void flush() {
        if constexpr (DT == DT_I8) {
            total += (long long)lo + 256ll * (long long)hi;
            lo = hi = 0;
        } else {
            total += (double)((f[0] + f[1]) + (f[2] + f[3]));
            f[0] = f[1] = f[2] = f[3] = 0.f;
        }
    }
};

// Which form of the tile checksum a configuration uses, and how many checksum
// accumulators per A fragment that takes.
template <class CFG>
struct ChecksumForm {
    static constexpr bool SPLIT = CFG::TN >= 2;
    static constexpr int NP = SPLIT ? (CFG::DT == DT_BF16 ? 3 : 2) : 1;  // checksum operands per k step
    static constexpr int NCHK = NP * CFG::TM;
};
// The thread-level scheme's extra MFMAs of one k step (a: A fragments, b: B fragments).
template <class CFG>
__device__ __forceinline__ void thread_checksum_step(const i32x4 (&a)[CFG::TM], const i32x4 (&b)[CFG::TN],
                                                     typename Mma<CFG::DT, CFG::MI>::Acc (&chk)[ChecksumForm<CFG>::NCHK]) {
    typedef Mma<CFG::DT, CFG::MI> MMA;
    constexpr int TM = CFG::TM;
    if constexpr (ChecksumForm<CFG>::SPLIT) {
        typedef TileChecksumSplit<CFG::DT, CFG::TN> SPL;
        i32x4 x[SPL::NP];
        SPL::make(b, x);
#pragma unroll
        for (int pc = 0; pc < SPL::NP; ++pc)
#pragma unroll
            for (int i = 0; i < TM; ++i) chk[pc * TM + i] = MMA::run(a[i], x[pc], chk[pc * TM + i]);
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i) chk[i] = MMA::run(a[i], b[0], chk[i]);
    }
}
// Redundant accumulator blocks a wavefront carries under each scheme.
template <class CFG, int MODE>
struct CheckRegs {
    static constexpr int N = MODE == MODE_THREAD ? ChecksumForm<CFG>::NCHK
                             : ((MODE == MODE_REPL || MODE == MODE_THREAD_H) ? CFG::TM : 1);
};

// Element-wise sum of two fragments in the operand type (fp16: one packed add per register;
// bf16: widened, added and rounded to nearest even).  int8 sums do not fit the operand type:
// integer layers run the exact scheme instead.
template <int DT>
__device__ __forceinline__ i32x4 add_in_operand_type(const i32x4& x, const i32x4& y) {
    static_assert(DT != DT_I8, "floating-point operands only");
    i32x4 out;
#pragma unroll
    for (int d = 0; d < 4; ++d) {
        if constexpr (DT == DT_F16) {
            typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
            out[d] = bitcast<int>((f16x2)(bitcast<f16x2>(x[d]) + bitcast<f16x2>(y[d])));
        } else {
            typedef TileChecksumSplitBF16<2> BF;
            out[d] = BF::pack(BF::lo_f(x[d]) + BF::lo_f(y[d]), BF::hi_f(x[d]) + BF::hi_f(y[d]));
        }
    }
    return out;
}

// The redundant MFMAs of one k step under a wavefront-level scheme (a: A fragments, b: B
// fragments of the step; Table 1 of the paper counts exactly these).
template <class CFG, int MODE>
__device__ __forceinline__ void check_step(const i32x4 (&a)[CFG::TM], const i32x4 (&b)[CFG::TN],
                                           typename Mma<CFG::DT, CFG::MI>::Acc (&chk)[(CheckRegs<CFG, MODE>::N)]) {
    typedef Mma<CFG::DT, CFG::MI> MMA;
    constexpr int TM = CFG::TM, TN = CFG::TN;
    if constexpr (MODE == MODE_THREAD) {
        thread_checksum_step<CFG>(a, b, chk);
    } else if constexpr (MODE == MODE_REPL) {
        // every product once more, all of an A fragment's into one block (Sec. 5.1)
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) chk[i] = MMA::run(a[i], b[j], chk[i]);
    } else if constexpr (MODE == MODE_THREAD_H || MODE == MODE_TWOSIDED) {
        i32x4 x = b[0];
#pragma unroll
        for (int j = 1; j < TN; ++j) x = add_in_operand_type<CFG::DT>(x, b[j]);
        if constexpr (MODE == MODE_THREAD_H) {
#pragma unroll
            for (int i = 0; i < TM; ++i) chk[i] = MMA::run(a[i], x, chk[i]);
        } else {
            i32x4 y = a[0];
#pragma unroll
            for (int i = 1; i < TM; ++i) y = add_in_operand_type<CFG::DT>(y, a[i]);
            chk[0] = MMA::run(y, x, chk[0]);
        }
    }
}

// ---------------------------------------------------------------------------
// Per-thread view of the tiling: which wavefront tile this lane works on and which
// element of C each accumulator register holds.
// ---------------------------------------------------------------------------
template <class CFG>
struct TileCoords {
    int lane, wave, wave_m, wave_n, lrow, lgrp, bm0, bn0;
    // wave_mn: position of the wavefront in the WAVES_M x WAVES_N grid when the workgroup has
    // more wavefronts than that (several share a register tile along k); -1: tid / 64
    __device__ __forceinline__ TileCoords(int tile_m, int tile_n, int wave_mn = -1) {
        const int tid = threadIdx.x;
        lane = tid & 63;
        wave = wave_mn >= 0 ? wave_mn : tid >> 6;
        wave_m = wave / CFG::WAVES_N;
        wave_n = wave % CFG::WAVES_N;
        lrow = lane % CFG::MI;
        lgrp = lane / CFG::MI;
        bm0 = tile_m * CFG::BM;
        bn0 = tile_n * CFG::BN;
    }
    // global row / column of accumulator register r of MFMA tile (i, j) in this lane
    __device__ __forceinline__ int row(int i, int r) const {
        int in_tile = (CFG::MI == 32) ? (8 * (r >> 2) + 4 * lgrp + (r & 3)) : (4 * lgrp + r);
        return bm0 + wave_m * CFG::WM + i * CFG::MI + in_tile;
    }
    __device__ __forceinline__ int col(int j) const { return bn0 + wave_n * CFG::WN + j * CFG::MI + lrow; }
};

// Fault injection (test hook): flips bit f_bit of the accumulator that holds element
// (f_row, f_col).  The register is identified by a wave-uniform flat index plus the
// owning lane, so the unrolled loop is a chain of selects.
template <class CFG>
__device__ __forceinline__ void inject_fault(typename Mma<CFG::DT, CFG::MI>::Acc (&acc)[CFG::TM][CFG::TN],
                                             const GemmArgs& p, const TileCoords<CFG>& tc) {
    typedef Mma<CFG::DT, CFG::MI> MMA;
    typedef typename MMA::AccT AccT;
    constexpr int MI = CFG::MI, TM = CFG::TM, TN = CFG::TN;
    const int rr = p.f_row - (tc.bm0 + tc.wave_m * CFG::WM);
    const int cc = p.f_col - (tc.bn0 + tc.wave_n * CFG::WN);
    if (rr >= 0 && rr < CFG::WM && cc >= 0 && cc < CFG::WN) {
        const int i = rr / MI, in_tile = rr % MI;
        const int j = cc / MI, own_col = cc % MI;
        int r, own_grp;
        if (MI == 32) {
            r = (in_tile >> 3) * 4 + (in_tile & 3);
            own_grp = (in_tile >> 2) & 1;
        } else {
            r = in_tile & 3;
            own_grp = in_tile >> 2;
        }
        const int flat = (i * TN + j) * MMA::NACC + r;
        const bool mine = (tc.lrow == own_col) && (tc.lgrp == own_grp);
        const unsigned mask = mine ? (1u << p.f_bit) : 0u;
#pragma unroll
        for (int ii = 0; ii < TM; ++ii)
#pragma unroll
            for (int jj = 0; jj < TN; ++jj)
#pragma unroll
                for (int q = 0; q < MMA::NACC; ++q) {
                    unsigned w = bitcast<unsigned>(acc[ii][jj][q]);
                    w ^= ((ii * TN + jj) * MMA::NACC + q == flat) ? mask : 0u;
                    acc[ii][jj][q] = bitcast<AccT>(w);
                }
    }
}

// Store of four consecutive rows x four adjacent columns of 16-bit outputs held by a quad of
// lanes (MFMA 32x32 layout: a lane holds one column of rows r..r+3 in four registers).  The
// values are rounded, packed in pairs and transposed inside the quad with two DPP exchanges,
// so that lane q of the quad writes row r + q, all four columns, as one 8-byte store: a quarter
// of the store instructions of element-wise writing.  `dst` is this lane's 8-byte destination.
template <int DT>
__device__ __forceinline__ int pack_out16(float a, float b) {
    if constexpr (DT == DT_F16) {
        typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
        f16x2 h;
        h[0] = (_Float16)a;
        h[1] = (_Float16)b;
        return bitcast<int>(h);
    } else {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        bf16x2 h;
        h[0] = (__bf16)a;
        h[1] = (__bf16)b;
        return bitcast<int>(h);
    }
}
template <int DT>
__device__ __forceinline__ void store_quad_rows(float v0, float v1, float v2, float v3, char* dst, int lane) {
    const int p01 = pack_out16<DT>(v0, v1), p23 = pack_out16<DT>(v2, v3);
    const bool odd = lane & 1, upper = lane & 2;
    // exchange with lane ^ 1: even lanes collect rows 0 / 2 of columns (c, c+1), odd lanes rows 1 / 3
    const int r01 = __builtin_amdgcn_update_dpp(0, p01, 0xB1, 0xF, 0xF, false);
    const int r23 = __builtin_amdgcn_update_dpp(0, p23, 0xB1, 0xF, 0xF, false);
    const unsigned sel = odd ? 0x03020706u : 0x05040100u;
    const int q01 = (int)__builtin_amdgcn_perm((unsigned)r01, (unsigned)p01, sel);
    const int q23 = (int)__builtin_amdgcn_perm((unsigned)r23, (unsigned)p23, sel);
    // exchange with lane ^ 2: lanes 0, 1 complete rows 0, 1; lanes 2, 3 rows 2, 3
    const int t = upper ? q01 : q23;
    const int x = __builtin_amdgcn_update_dpp(0, t, 0x4E, 0xF, 0xF, false);
    i32x2 out;
    out[0] = upper ? x : q01;
    out[1] = upper ? q23 : x;
    *reinterpret_cast<i32x2*>(dst) = out;
}

// This lane's share of the sum of a wavefront's redundant accumulator blocks under a
// wavefront-level scheme, weighted as the form of the tile checksum says, so that the sum over
// the lanes is the checksum product (Sec. 5.2.2) resp. the replicated output sum (Sec. 5.1).
// int8: exact 64-bit sums from 16-bit pieces (low halves unsigned, high halves signed, of up to
// 256 accumulators each: far inside int32).  Floating point: groups of four accumulators are
// summed in fp32, everything above that in fp64.
template <class CFG, int MODE>
__device__ __forceinline__ typename std::conditional<CFG::DT == DT_I8, long long, double>::type lane_check_sum(
    const typename Mma<CFG::DT, CFG::MI>::Acc (&chk)[(CheckRegs<CFG, MODE>::N)], int lane) {
    typedef Mma<CFG::DT, CFG::MI> MMA;
    constexpr int MI = CFG::MI, TM = CFG::TM, TN = CFG::TN;
    constexpr bool SPLIT_FORM = MODE == MODE_THREAD && ChecksumForm<CFG>::SPLIT;
    constexpr int NBLK = CheckRegs<CFG, MODE>::N;
    if constexpr (CFG::DT == DT_I8) {
        long long rsum = 0;
        if constexpr (SPLIT_FORM) {
            // accumulators of the low-digit operand, then 256 x those of the high-digit one
#pragma unroll
            for (int pc = 0; pc < 2; ++pc) {
                int r_lo = 0, r_hi = 0;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < MMA::NACC; ++r) {
                        r_lo += chk[pc * TM + i][r] & 0xffff;
                        r_hi += chk[pc * TM + i][r] >> 16;
                    }
                const long long part = ((long long)r_hi << 16) + (long long)r_lo;
                rsum += pc == 0 ? part : 256 * part;
            }
        } else {
            int r_lo = 0, r_hi = 0;
#pragma unroll
            for (int i = 0; i < NBLK; ++i)
#pragma unroll
                for (int r = 0; r < MMA::NACC; ++r) {
                    r_lo += chk[i][r] & 0xffff;
                    r_hi += chk[i][r] >> 16;
                }
            rsum = ((long long)r_hi << 16) + (long long)r_lo;
        }
        return rsum;
    } else {
        double rsum = 0.0;
        if constexpr (SPLIT_FORM) {
            typedef TileChecksumSplit<CFG::DT, TN> SPL;
#pragma unroll
            for (int pc = 0; pc < SPL::NP; ++pc) {
                double part = 0.0;
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int r = 0; r < MMA::NACC; r += 4)
                        part += (double)((chk[pc * TM + i][r] + chk[pc * TM + i][r + 1]) +
                                         (chk[pc * TM + i][r + 2] + chk[pc * TM + i][r + 3]));
                rsum += part * SPL::scale(pc);
            }
        } else {
#pragma unroll
            for (int i = 0; i < NBLK; ++i)
#pragma unroll
                for (int r = 0; r < MMA::NACC; r += 4)
                    rsum += (double)((chk[i][r] + chk[i][r + 1]) + (chk[i][r + 2] + chk[i][r + 3]));
        }
        return rsum;
    }
}

// Which wavefront adds up what every wavefront of the workgroup left in LDS.  Without a scratch
// area of its own (the sums sit in LDS that held operands): wavefront 0, after a barrier.  With
// one (epi: the sums at its start, a counter that starts at zero 256 bytes in): whichever
// wavefront arrives last, so that no wavefront waits.  A wavefront's LDS operations execute in
// the order it issued them, so the counter value that marks the last arrival is returned only
// after every earlier arrival's sums are in place.
template <class CFG>
__device__ __forceinline__ bool cross_wave_last(char* epi, int lane, int wave) {
    if (!epi) {
        __syncthreads();
        return wave == 0;
    }
    unsigned seen = 0;
    if (lane == 0)
        seen = __hip_atomic_fetch_add(reinterpret_cast<unsigned*>(epi + 256), 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_WORKGROUP);
    return __builtin_amdgcn_readfirstlane(seen) == (unsigned)(CFG::WAVES_M * CFG::WAVES_N - 1);
}

// Checksum epilogue (taken from the accumulators, before down-conversion) and store of C.
//  GLOBAL: fused output summation (Sec. 2.5) of the workgroup tile, compared right here with
//          the tile's checksum dot product (Sec. 2.4 steps 3-4).  lane_dot (a double, or a
//          long long for int8) is this lane's share of that dot product when the kernel formed
//          it itself from the A fragments and the weight checksums; null: the partial dot
//          products were left by the activation-checksum kernel, which ran before on the stream.
//  THREAD: the wavefront tile's output summation against the sum of its checksum
//          accumulators (Sec. 5.2.2), compared here; p.flag is touched only on mismatch.
template <class CFG, int MODE>
__device__ __forceinline__ void epilogue(typename Mma<CFG::DT, CFG::MI>::Acc (&acc)[CFG::TM][CFG::TN],
                                         typename Mma<CFG::DT, CFG::MI>::Acc (&chk)[(CheckRegs<CFG, MODE>::N)],
                                         const GemmArgs& p, int tile_m, int tile_n, char* smem, bool store = true,
                                         int wave_mn = -1, const void* lane_dot = nullptr, char* epi = nullptr) {
    typedef Mma<CFG::DT, CFG::MI> MMA;
    constexpr int MI = CFG::MI, TM = CFG::TM, TN = CFG::TN;
    constexpr bool IS_INT = CFG::DT == DT_I8;
    const TileCoords<CFG> tc(tile_m, tile_n, wave_mn);
    const int tid = threadIdx.x, lane = tc.lane, wave = tc.wave;
    const int M = p.M, N = p.N;
    // index of this wavefront's register tile in the partition of C into such tiles (row-major,
    // edge tiles clipped); a register tile that lies wholly outside C (the launched grid is whole
    // workgroup tiles) holds zeros and is left out of the diagnostics
    const int wave_row = tile_m * CFG::WAVES_M + tc.wave_m, wave_col = tile_n * CFG::WAVES_N + tc.wave_n;
    const bool wave_inside = wave_row * CFG::WM < M && wave_col * CFG::WN < N;
    const unsigned wave_tile_index = (unsigned)(wave_row * ((N + CFG::WN - 1) / CFG::WN) + wave_col);
    (void)wave_tile_index;
    (void)wave_inside;
    auto acc_row = [&](int i, int r) { return tc.row(i, r); };
    auto acc_col = [&](int j) { return tc.col(j); };
    // ---- checksum epilogue: taken from the accumulators, before down-conversion
    if constexpr (MODE != MODE_NONE) {
        if constexpr (IS_INT) {
            // exact 64-bit sum from 32-bit pieces: low halves (unsigned 16 bits) and high halves
            // (signed) of up to 256 accumulators each stay far inside int32
            int s_lo = 0, s_hi = 0;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < MMA::NACC; ++r) {
                        s_lo += acc[i][j][r] & 0xffff;
                        s_hi += acc[i][j][r] >> 16;
                    }
            long long s = ((long long)s_hi << 16) + (long long)s_lo;
            s = wave_sum(s);
            if constexpr (MODE == MODE_GLOBAL) {
                long long* red = reinterpret_cast<long long*>(epi ? epi : smem);
                long long wdot = 0;
                if (lane_dot) wdot = wave_sum(*reinterpret_cast<const long long*>(lane_dot));
                if (!epi) __syncthreads();
                if (lane == 0) {
                    red[2 * wave] = s;
                    red[2 * wave + 1] = wdot;
                }
                if (cross_wave_last<CFG>(epi, lane, wave)) {
                    // comparison (Sec. 2.4 step 4) for this tile: its output summation against the
                    // sum of the partial checksum dot products the activation-checksum kernel left
                    long long tot = 0, sab = 0;
                    for (int w = 0; w < CFG::WAVES_M * CFG::WAVES_N; ++w) {
                        tot += red[2 * w];
                        sab += red[2 * w + 1];
                    }
                    const long long t = (long long)tile_m * p.tiles_n + tile_n;
                    if (!lane_dot) {
                        const long long* pd = reinterpret_cast<const long long*>(p.partial_dots) + t * p.n_parts;
                        for (int c = lane; c < p.n_parts; c += 64) sab += pd[c];
                        sab = wave_sum(sab);
                    }
                    if (lane == 0) {
                        const bool bad = tot != sab;
                        if (bad) atomicOr(p.flag, 1u);
                        if (p.report)
                            report_update(p.report, bad ? __builtin_huge_val() : 0.0, (double)tot, (double)sab, 0.0, 0.0,
                                          0.0, (unsigned)t);
                    }
                }
            } else {
                const long long rsum = wave_sum(lane_check_sum<CFG, MODE>(chk, lane));
                if (lane == 0) {
                    // (replication: a block that took several products may have wrapped where the
                    // product's own blocks did not; the two sides still agree modulo 2^32, and a
                    // flipped bit never changes a sum by a multiple of 2^32)
                    bool bad = MODE == MODE_REPL ? (unsigned int)(s - rsum) != 0u : s != rsum;
                    if (bad) atomicOr(p.flag, 1u);
                    if (p.report && wave_inside)
                        report_update(p.report, bad ? __builtin_huge_val() : 0.0, (double)s, (double)rsum, 0.0, 0.0, 0.0,
                                      wave_tile_index);
                }
            }
        } else {
            // groups of four accumulators are summed in fp32 (three roundings), everything
            // above that in fp64, so the summation adds nothing visible to the comparison
            double s = 0.0;
            float f2 = 0.f, l1 = 0.f;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int r = 0; r < MMA::NACC; r += 4) {
                        float v0 = acc[i][j][r], v1 = acc[i][j][r + 1], v2 = acc[i][j][r + 2], v3 = acc[i][j][r + 3];
                        s += (double)((v0 + v1) + (v2 + v3));
                        f2 += v0 * v0 + v1 * v1 + v2 * v2 + v3 * v3;
                        if constexpr (MODE == MODE_GLOBAL)
                            l1 += (__builtin_fabsf(v0) + __builtin_fabsf(v1)) + (__builtin_fabsf(v2) + __builtin_fabsf(v3));
                    }
            // cross-lane sums: the norms of the tolerance in fp32; the two sides of the comparison in
            // fp64, as one sum of their per-lane difference unless the report wants them apart
            const double F2 = (double)wave_sum(f2);
            if constexpr (MODE == MODE_GLOBAL) {
                const double L1 = (double)wave_sum(l1);
                double wdot = 0.0;
                if (lane_dot && !p.report) {
                    s = wave_sum(s - *reinterpret_cast<const double*>(lane_dot));
                } else {
                    s = wave_sum(s);
                    if (lane_dot) wdot = wave_sum(*reinterpret_cast<const double*>(lane_dot));
                }
                double* red = reinterpret_cast<double*>(epi ? epi : smem);
                if (!epi) __syncthreads();
                if (lane == 0) {
                    red[4 * wave] = s;
                    red[4 * wave + 1] = F2;
                    red[4 * wave + 2] = L1;
                    red[4 * wave + 3] = wdot;
                }
                if (cross_wave_last<CFG>(epi, lane, wave)) {
                    // comparison (Sec. 2.4 step 4) for this tile: its output summation against the
                    // sum of the partial checksum dot products the activation-checksum kernel left
                    double ts = 0.0, tf = 0.0, tl = 0.0, sab = 0.0;
                    for (int w = 0; w < CFG::WAVES_M * CFG::WAVES_N; ++w) {
                        ts += red[4 * w];
                        tf += red[4 * w + 1];
                        tl += red[4 * w + 2];
                        sab += red[4 * w + 3];
                    }
                    const long long t = (long long)tile_m * p.tiles_n + tile_n;
                    if (!lane_dot) {
                        const double* pd = reinterpret_cast<const double*>(p.partial_dots) + t * p.n_parts;
                        for (int c = lane; c < p.n_parts; c += 64) sab += pd[c];
                        sab = wave_sum(sab);
                    }
                    if (lane == 0) {
                        const double frob = __builtin_sqrt(tf);
                        const double tau = p.tol_coeff * frob + p.tol_l1 * tl;
                        const double res = __builtin_fabs(ts - sab);
                        // a sum of squares beyond the fp32 range cannot come from a fault-free tile
                        const bool finite = __builtin_isfinite(ts) && __builtin_isfinite(sab) && __builtin_isfinite(tf);
                        const bool bad = !finite || !(res <= tau);
                        if (bad) atomicOr(p.flag, 1u);
                        if (p.report) {
                            const double ratio = !finite ? __builtin_huge_val()
                                                         : (tau > 0.0 ? res / tau : (res > 0.0 ? __builtin_huge_val() : 0.0));
                            report_update(p.report, ratio, ts, sab, tau, frob, tl, (unsigned)t);
                        }
                    }
                }
            } else {
                double rsum = lane_check_sum<CFG, MODE>(chk, lane);
                if (p.report) {
                    s = wave_sum(s);
                    rsum = wave_sum(rsum);
                } else {
                    s = wave_sum(s - rsum);
                    rsum = 0.0;
                }
                if (lane == 0) {
                    double tau = p.tol_coeff * __builtin_sqrt(F2);
                    double res = __builtin_fabs(s - rsum);
                    // a sum of squares beyond the fp32 range cannot come from a fault-free tile
                    bool finite = __builtin_isfinite(s) && __builtin_isfinite(rsum) && __builtin_isfinite(F2);
                    bool bad = !finite || !(res <= tau);
                    if (bad) atomicOr(p.flag, 1u);
                    if (p.report && wave_inside) {
                        double ratio = !finite ? __builtin_huge_val() : (tau > 0.0 ? res / tau : (res > 0.0 ? __builtin_huge_val() : 0.0));
                        report_update(p.report, ratio, s, rsum, tau, __builtin_sqrt(F2), 0.0, wave_tile_index);
                    }
                }
            }
        }
    }

    if (!store) return;
    if (p.act) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < MMA::NACC; ++r) acc[i][j][r] = acc[i][j][r] > 0 ? acc[i][j][r] : 0;
    }
    // ---- activation checksums for the next layer: per 32-row block and column, the sum of the
    // values as they are stored (a lane holds 16 rows of one column of each MFMA block, the
    // lane 32 further on the other 16); rows past M hold zeros
    if constexpr (CFG::CSIZE == 2 && MI == 32) {
        if (p.alpha_out) {
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    // (the pairs the store packs: rounded once, widened again inside the addition)
                    float cs = 0.f;
#pragma unroll
                    for (int r = 0; r < MMA::NACC; r += 2) {
                        const int pk = pack_out16<CFG::DT>(acc[i][j][r], acc[i][j][r + 1]);
                        cs = mul_add_half<CFG::DT, 0>(pk, 1.0f, cs);
                        cs = mul_add_half<CFG::DT, 1>(pk, 1.0f, cs);
                    }
                    cs += __shfl_xor(cs, 32);
                    const int col = acc_col(j);
                    const int blk = (tc.bm0 + tc.wave_m * CFG::WM) / 32 + i;
                    if (lane < 32 && col < N && blk * 32 < M) p.alpha_out[(long long)blk * p.ld_alpha_out + col] = cs;
                }
        }
    }
    if constexpr (CFG::CSIZE == 2 && MI == 16 && TM % 2 == 0) {
        // (16x16 shapes, direct-to-LDS kernel: a lane holds 4 rows of one column of each block; two
        // block rows make a 32-row block, the lanes 16, 32 and 48 further on hold its other rows)
        if (p.alpha_out) {
#pragma unroll
            for (int i = 0; i < TM; i += 2)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    float cs = 0.f;
#pragma unroll
                    for (int ii = i; ii < i + 2; ++ii)
#pragma unroll
                        for (int r = 0; r < MMA::NACC; r += 2) {
                            const int pk = pack_out16<CFG::DT>(acc[ii][j][r], acc[ii][j][r + 1]);
                            cs = mul_add_half<CFG::DT, 0>(pk, 1.0f, cs);
                            cs = mul_add_half<CFG::DT, 1>(pk, 1.0f, cs);
                        }
                    cs += __shfl_xor(cs, 16);
                    cs += __shfl_xor(cs, 32);
                    const int col = acc_col(j);
                    const int blk = (tc.bm0 + tc.wave_m * CFG::WM) / 32 + i / 2;
                    if (lane < 16 && col < N && blk * 32 < M) p.alpha_out[(long long)blk * p.ld_alpha_out + col] = cs;
                }
        }
        // wavefront tiles that lie wholly inside C: 8-byte stores of four columns per lane
        const int wrow0 = tc.bm0 + tc.wave_m * CFG::WM, wcol0 = tc.bn0 + tc.wave_n * CFG::WN;
        const bool whole = wrow0 + CFG::WM <= M && wcol0 + CFG::WN <= N && (p.ldc & 3) == 0 &&
                           (reinterpret_cast<uintptr_t>(p.C) & 7u) == 0;
        if (whole) {
            const long long ldcb = p.ldc * 2;
            char* base = p.C + ((long long)(wrow0 + 4 * tc.lgrp + (lane & 3)) * p.ldc + wcol0 + (tc.lrow & ~3)) * 2;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    store_quad_rows<CFG::DT>(acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3],
                                             base + (i * 16) * ldcb + j * 32, lane);
            return;
        }
    }
    // ---- store C (rounded to the output type)
    if constexpr (CFG::CSIZE == 2 && MI == 32) {
        // wavefront tiles that lie wholly inside C: 8-byte stores of four columns per lane
        const int wrow0 = tc.bm0 + tc.wave_m * CFG::WM, wcol0 = tc.bn0 + tc.wave_n * CFG::WN;
        const bool whole = wrow0 + CFG::WM <= M && wcol0 + CFG::WN <= N && (p.ldc & 3) == 0 &&
                           (reinterpret_cast<uintptr_t>(p.C) & 7u) == 0;
        if (whole) {
            const long long ldcb = p.ldc * 2;
            char* base = p.C + ((long long)(wrow0 + 4 * tc.lgrp + (lane & 3)) * p.ldc + wcol0 + (tc.lrow & ~3)) * 2;
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int g = 0; g < 4; ++g)
#pragma unroll
                    for (int j = 0; j < TN; ++j)
                        store_quad_rows<CFG::DT>(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2],
                                                 acc[i][j][4 * g + 3], base + (i * 32 + 8 * g) * ldcb + j * 64, lane);
            return;
        }
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int col = acc_col(j);
#pragma unroll
            for (int r = 0; r < MMA::NACC; ++r) {
                const int row = acc_row(i, r);
                if (row < M && col < N) {
                    char* dst = p.C + ((long long)row * p.ldc + col) * CFG::CSIZE;
                    if constexpr (CFG::DT == DT_F16) *reinterpret_cast<_Float16*>(dst) = (_Float16)acc[i][j][r];
                    else if constexpr (CFG::DT == DT_BF16) *reinterpret_cast<__bf16*>(dst) = (__bf16)acc[i][j][r];
                    else *reinterpret_cast<int*>(dst) = acc[i][j][r];
                }
            }
        }
}

}  // namespace abft
